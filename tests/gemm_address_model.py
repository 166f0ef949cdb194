"""A CPU model of every global address the bf16 grouped-GEMM kernels of the expert FFN form for one shape.

The model restates, in numpy over the 64 lanes of a wave, the integer arithmetic of paper_2501_10714_amd/csrc/gemm_mfma.hip
that leads to a global address: the tile map (count_tiles / tile_at / dealt_tile), the lane offsets and scalar bases of the
direct-to-LDS loads of both K pipelines and of the weight-gradient kernel (with their clamps, the stepping along K, the
jump to the second operand pair, the re-fetches past the end), and the loads and stores of the epilogues.  Every 16-byte
access is checked against the extent of the tensor it is meant for, with tensors of exactly the sizes include/moe_mi355x.h
asks of the caller; the weight-gradient loads are also checked to stay inside the rows of their own expert.  It is a
bounds check of the addressing on the host, not a test of the kernels' results (the GPU parity tests are that)."""
import numpy as np
BM = BN = 256; BK = 32; BK2 = 64; kLoads = 4; kPartBytes = 4096; kRegionBytes = 8192; kDmaBias = 4096
kBand = 8; kChunk = 32
KC, TR = 0, 1
lane = np.arange(64)

class Mem:
    """Tensors at made-up addresses, far apart."""
    def __init__(self): self.t = {}; self.next = 1 << 32
    def alloc(self, name, nbytes):
        b = self.next; self.next += ((nbytes + (1 << 24)) >> 24 << 24) + (1 << 24); self.t[name] = (b, nbytes); return b
    def check(self, name, addr, what):
        b, n = self.t[name]
        addr = np.asarray(addr, dtype=np.int64)
        bad = (addr < b) | (addr + 16 > b + n) | (addr % 16 != 0)
        if bad.any():
            i = np.argmax(bad)
            raise AssertionError(f"{what}: access at {name}+{int(addr.flat[i]) - b} outside [0,{n}) or misaligned")
mem = Mem()

def tr_swz(k): return (k & 3) << 1
def kc64_swz(row): return (row >> 1) & 7

def count_tiles(p, n_nt, mt_fix, ragged):
    if ragged: return (2 * p['E'] if p['n_pairs'] == 2 else p['E']) * mt_fix * n_nt
    return sum(((p['row_end'][e] - p['offsets'][e] + BM - 1) // BM) * n_nt for e in range(p['E']))

def tile_at(p, n_nt, mt_fix, L, ragged):
    g = 0; mt_g = mt_fix
    if ragged:
        g = L // (mt_fix * n_nt); L -= g * mt_fix * n_nt
    else:
        while True:
            mt_g = (p['row_end'][g] - p['offsets'][g] + BM - 1) // BM
            cnt = mt_g * n_nt
            if L < cnt: break
            L -= cnt; g += 1
    nbands = max(1, (mt_g + kBand // 2) // kBand)
    bh = mt_g // nbands; tall = mt_g % nbands
    tall_tiles = tall * (bh + 1) * n_nt
    if L < tall_tiles:
        bsz = bh + 1; band = L // (bsz * n_nt); rem = L - band * bsz * n_nt
    else:
        bsz = bh; l2 = L - tall_tiles; band = tall + l2 // (bsz * n_nt); rem = l2 - (band - tall) * bsz * n_nt
    t = dict(nt=rem // bsz, mt=band * bh + min(band, tall) + rem % bsz, e=g % p['E'], set=g // p['E'])
    t = {k_: int(v_) for k_, v_ in t.items()}
    t['r0'] = int(p['offsets'][t['e']]); t['rows'] = int(p['row_end'][t['e']]) - t['r0']
    return t

def tiles(p, n_nt, mt_fix, ragged, grid):
    total = count_tiles(p, n_nt, mt_fix, ragged)
    seen = set()
    for b in range(grid):
        slot = b >> 3
        L = (((slot // kChunk) << 3) + (b & 7)) * kChunk + slot % kChunk
        if L >= total: continue
        assert L not in seen; seen.add(L)
        yield tile_at(p, n_nt, mt_fix, L, ragged)
    assert len(seen) == total, (len(seen), total)

def epilogue(p, t, epi, ragged):
    glu = epi == 'GLU_FWD'
    kOutCols = BN // 2 if glu else BN
    m_limit = p['Mfix'] if ragged else t['rows']
    lpr = 8 if glu else 16; rpp = 64 // lpr; passes = 32 // rpp
    pr = lane // lpr; c8 = (lane % lpr) * 8
    nx = 2 if epi == 'GLU_BWD' else 1 if epi in ('ACT_BWD', 'ACCUM') else 0
    for wave in range(4):
        wm, wn = wave >> 1, wave & 1
        col = t['nt'] * kOutCols + wn * 64 + c8 if glu else t['nt'] * BN + wn * 128 + c8
        col_ok = col < p['N']
        def out_off(mrow, c):
            return (t['e'] * p['gC'] + mrow * p['ldc'] if ragged else (t['r0'] + mrow) * p['ldc']) + c
        for fm in range(4):
            for ps in range(passes):
                if nx:
                    cc = np.minimum(col, p['N'] - 8)
                    mrow = np.minimum(t['mt'] * BM + wm * 128 + fm * 32 + ps * rpp + pr, m_limit - 1)
                    off = out_off(mrow, cc)
                    for x in range(nx):
                        name = p['C'][0] if epi == 'ACCUM' else p['X'][x]
                        mem.check(name, mem.t[name][0] + off * 2, f"epilogue prefetch {epi}")
                mrow = t['mt'] * BM + wm * 128 + fm * 32 + ps * rpp + pr
                ok = (mrow < m_limit) & col_ok
                if not ok.any(): continue
                off = out_off(mrow, col)[ok]
                outs = {'PLAIN': lambda: [p['C'][t['set'] if ragged else 0]], 'ACT_FWD': lambda: [p['C'][0], p['C'][2]], 'GLU_FWD': lambda: p['C'][:3],
                        'ACCUM': lambda: [p['C'][0]], 'ACT_BWD': lambda: [p['C'][0]], 'GLU_BWD': lambda: p['C'][:2]}[epi]()
                for name in outs:
                    mem.check(name, mem.t[name][0] + off * 2, f"epilogue store {epi}")

def kernel64(p, LB, epi):
    glu = epi == 'GLU_FWD'
    kOutCols = BN // 2 if glu else BN
    n_nt = -(-p['N'] // kOutCols)
    rows_bound = min(p['max_rows'] * p['E'], p['total_rows_bound'])
    max_tiles = ((rows_bound + BM - 1) // BM + p['E']) * n_nt
    grid = -(-max_tiles // 256) * 256
    sum_pairs = p['n_pairs'] if not glu else 1
    nb1 = p['Kfix'] // BK2; nb = nb1 * sum_pairs
    lda = p['sAi']; ldb = p['sBk'] if LB == TR else p['sBn']
    ntile = 0
    for t in tiles(p, n_nt, 0, False, grid):
        ntile += 1
        A0 = mem.t[p['A'][0]][0]; B0 = mem.t[p['B'][0]][0]
        B1 = mem.t[p['B'][1]][0] if glu else B0
        for wave in range(4):
            sa = A0 + (t['r0'] + t['mt'] * BM) * lda * 2 - kDmaBias
            sb = B0 + (t['e'] * p['gB'] + (t['nt'] * BN * ldb if LB == KC else t['nt'] * kOutCols)) * 2 - kDmaBias
            sb3 = B1 + (t['e'] * p['gB'] + t['nt'] * kOutCols) * 2 - kDmaBias
            va = []; vb = []; offs = []
            for j in range(8):
                OFF = -4096 + 1024 * j
                bias = kDmaBias - OFF
                row = wave * 64 + j * 8 + (lane >> 3); slot = lane & 7
                c = slot ^ kc64_swz(row)
                rrow = np.minimum(t['mt'] * BM + row, t['rows'] - 1) - t['mt'] * BM
                assert (rrow >= 0).all()
                va.append((rrow * (lda * 2) + c * 16 + bias).astype(np.int64) & 0xFFFFFFFF)
                if LB == KC:
                    rn = np.minimum(t['nt'] * BN + row, p['N'] - 1) - t['nt'] * BN
                    assert (rn >= 0).all()
                    vb.append((rn * (ldb * 2) + c * 16 + bias).astype(np.int64) & 0xFFFFFFFF); offs.append(OFF)
                elif glu:
                    krow = wave * 16 + (j & 3) * 4 + (lane >> 4); pos = lane & 15
                    seg = (pos >> 1) ^ tr_swz(krow)
                    rcol = np.minimum(t['nt'] * kOutCols + (seg * 2 + (pos & 1)) * 8, p['N'] - 8) - t['nt'] * kOutCols
                    assert (rcol >= 0).all()
                    OFFB = -2048 + 1024 * (j & 3)
                    vb.append((krow * (ldb * 2) + rcol * 2 + (kDmaBias - OFFB)).astype(np.int64) & 0xFFFFFFFF); offs.append(OFFB)
                else:
                    krow = wave * 16 + j * 2 + (lane >> 5); pos = lane & 31
                    seg = (pos >> 1) ^ tr_swz(krow)
                    rcol = np.minimum(t['nt'] * BN + (seg * 2 + (pos & 1)) * 8, p['N'] - 8) - t['nt'] * BN
                    assert (rcol >= 0).all()
                    vb.append((krow * (ldb * 2) + rcol * 2 + bias).astype(np.int64) & 0xFFFFFFFF); offs.append(OFF)
            a_step = BK2 * 2; b_step = (BK2 if LB == KC else BK2 * ldb) * 2
            a_jump = mem.t[p['A'][1]][0] - A0 - nb1 * a_step if sum_pairs == 2 else 0
            b_jump = mem.t[p['B'][1]][0] - B0 - nb1 * b_step if sum_pairs == 2 else 0
            # the issue sequence: prologue A B A, then half-steps: H=0 issues B, H=1 issues A
            nh = 2 * nb
            seq = ['A', 'B', 'A'] + ['B' if (h % 2 == 0) else 'A' for h in range(nh)]
            ia = ib = 0
            for what in seq:
                if what == 'A':
                    pair = 1 if (sum_pairs == 2 and ia >= nb1) else 0
                    for q in range(8):
                        mem.check(p['A'][pair], sa + va[q] + (-4096 + 1024 * q), f"A batch {ia}")
                    last = ia + 1 >= nb
                    if not last:
                        sa += a_step + (a_jump if (ia + 1 == nb1 and sum_pairs == 2) else 0); ia += 1
                else:
                    pair = 1 if (sum_pairs == 2 and ib >= nb1) else 0
                    for q in range(8):
                        if glu:
                            mem.check(p['B'][0 if q < 4 else 1], (sb if q < 4 else sb3) + vb[q] + offs[q], f"B batch {ib} (glu)")
                        else:
                            mem.check(p['B'][pair], sb + vb[q] + offs[q], f"B batch {ib}")
                    last = ib + 1 >= nb
                    if not last:
                        d = b_step + (b_jump if (ib + 1 == nb1 and sum_pairs == 2) else 0); sb += d; sb3 += d; ib += 1
            assert ia == nb - 1 and ib == nb - 1
        epilogue(p, t, epi, False)
    return ntile

def kernel32(p, LB, epi):
    """gg_mfma_kernel<KC, LB, EPI, false>: ragged M, K a multiple of 32 but not of 64"""
    glu = epi == 'GLU_FWD'
    kOutCols = BN // 2 if glu else BN
    n_nt = -(-p['N'] // kOutCols)
    rows_bound = min(p['max_rows'] * p['E'], p['total_rows_bound'])
    max_tiles = ((rows_bound + BM - 1) // BM + p['E']) * n_nt
    grid = -(-max_tiles // 256) * 256
    sum_pairs = p['n_pairs'] if not glu else 1
    nk1 = -(-p['Kfix'] // BK); nk = nk1 * sum_pairs
    lda = p['sAi']; ldb = p['sBk'] if LB == TR else p['sBn']
    ntile = 0
    for t in tiles(p, n_nt, 0, False, grid):
        ntile += 1
        A0 = mem.t[p['A'][0]][0]; B0 = mem.t[p['B'][0]][0]
        B1 = mem.t[p['B'][1]][0] if glu else B0
        for wave in range(4):
            sa = A0 + (t['r0'] + t['mt'] * BM) * lda * 2 - kDmaBias
            sb = B0 + (t['e'] * p['gB'] + (t['nt'] * BN * ldb if LB == KC else t['nt'] * BN)) * 2 - kDmaBias
            va = []; vb = []; gb = []; gbname = []
            for j in range(kLoads):
                blk = wave * kLoads + j
                bias_a = kDmaBias - (-kPartBytes + 1024 * j); bias_b = kDmaBias - 1024 * j
                row = blk * 16 + (lane >> 2); slot = lane & 3
                c = slot ^ ((row >> 2) & 3)
                rrow = np.minimum(t['mt'] * BM + row, t['rows'] - 1) - t['mt'] * BM
                assert (rrow >= 0).all()
                va.append((rrow * (lda * 2) + c * 16 + bias_a).astype(np.int64) & 0xFFFFFFFF)
                if LB == KC:
                    rn = np.minimum(t['nt'] * BN + row, p['N'] - 1) - t['nt'] * BN
                    assert (rn >= 0).all()
                    vb.append((rn * (ldb * 2) + c * 16 + bias_b).astype(np.int64) & 0xFFFFFFFF)
                else:
                    krow = blk * 2 + (lane >> 5); pos = lane & 31
                    seg = (pos >> 1) ^ tr_swz(krow)
                    cc = seg * 2 + (pos & 1)
                    if glu:
                        col = np.minimum(t['nt'] * kOutCols + (cc >> 4) * 64 + (cc & 7) * 8, p['N'] - 8)
                        which = (cc >> 3) & 1
                        gb.append(np.where(which == 1, B1, B0) + (t['e'] * p['gB'] + krow * ldb + col) * 2); gbname.append(which)
                        vb.append(None)
                    else:
                        rcol = np.minimum(t['nt'] * BN + cc * 8, p['N'] - 8) - t['nt'] * BN
                        assert (rcol >= 0).all()
                        vb.append(((rcol * 2 + bias_b) + krow * (ldb * 2)).astype(np.int64) & 0xFFFFFFFF)
            a_step = BK * 2; b_step = (BK if LB == KC else BK * ldb) * 2
            a_jump = mem.t[p['A'][1]][0] - A0 - nk1 * a_step if sum_pairs == 2 else 0
            b_jump = mem.t[p['B'][1]][0] - B0 - nk1 * b_step if sum_pairs == 2 else 0
            it_load = 0; gstep = 0
            for _ in range(3 + nk):
                pair = 1 if (sum_pairs == 2 and it_load >= nk1) else 0
                for j in range(kLoads):
                    mem.check(p['A'][pair], sa + va[j] + (-kPartBytes + 1024 * j), f"A stage {it_load}")
                    if glu:
                        a = gb[j] + gstep
                        for wsel in (0, 1):
                            if (gbname[j] == wsel).any(): mem.check(p['B'][wsel], a[gbname[j] == wsel], f"B stage {it_load} (glu)")
                    else:
                        mem.check(p['B'][pair], sb + vb[j] + 1024 * j, f"B stage {it_load}")
                last = it_load + 1 >= nk
                if not last:
                    jump = it_load + 1 == nk1 and sum_pairs == 2
                    sa += a_step + (a_jump if jump else 0)
                    d = b_step + (b_jump if jump else 0)
                    sb += d; gstep += d; it_load += 1
            assert it_load == nk - 1
        epilogue(p, t, epi, False)
    return ntile

def kernel32_ragged(p):
    """gg_mfma_kernel<TR, TR, PLAIN, true>"""
    n_nt = -(-p['N'] // BN); mt_fix = -(-p['Mfix'] // BM)
    max_tiles = (2 if p['n_pairs'] == 2 else 1) * p['E'] * mt_fix * n_nt
    grid = -(-max_tiles // 256) * 256
    lda = p['sAk']; ldb = p['sBk']
    ntile = 0
    for t in tiles(p, n_nt, mt_fix, True, grid):
        ntile += 1
        Kg = t['rows']; nk = -(-Kg // BK)
        A0 = mem.t[p['A'][0]][0]; Bn = p['B'][t['set']]; B0 = mem.t[Bn][0]
        if nk == 0:
            epilogue(p, t, 'PLAIN', True); continue
        for wave in range(4):
            sa = A0 + (t['r0'] * lda + t['mt'] * BM) * 2 - kDmaBias
            sb = B0 + (t['r0'] * ldb + t['nt'] * BN) * 2 - kDmaBias
            va = []; vb = []; ka = []; kb = []
            for j in range(kLoads):
                blk = wave * kLoads + j
                bias_a = kDmaBias - (-kPartBytes + 1024 * j); bias_b = kDmaBias - 1024 * j
                krow = blk * 2 + (lane >> 5); pos = lane & 31
                seg = (pos >> 1) ^ tr_swz(krow)
                ri = np.minimum(t['mt'] * BM + (seg * 2 + (pos & 1)) * 8, p['Mfix'] - 8) - t['mt'] * BM
                assert (ri >= 0).all()
                va.append(ri * 2 + bias_a); ka.append(krow * (lda * 2))
                rcol = np.minimum(t['nt'] * BN + (seg * 2 + (pos & 1)) * 8, p['N'] - 8) - t['nt'] * BN
                assert (rcol >= 0).all()
                vb.append(rcol * 2 + bias_b); kb.append(krow * (ldb * 2))
            a_step = BK * lda * 2; b_step = BK * ldb * 2
            n_issue = 3 + nk   # prologue 3 stages + one per iteration
            it_load = 0
            for _ in range(n_issue):
                last_row = min(Kg - 1 - it_load * BK, BK)
                assert last_row >= 0
                for j in range(kLoads):
                    a = sa + ((va[j] + np.minimum(ka[j], last_row * lda * 2)) & 0xFFFFFFFF) + (-kPartBytes + 1024 * j)
                    mem.check(p['A'][0], a, f"ragged A stage {it_load}")
                    # rows read must belong to this expert
                    arow = (a - A0) // (lda * 2)
                    assert ((arow >= t['r0']) & (arow < t['r0'] + Kg)).all(), "A row of another expert"
                    b = sb + ((vb[j] + np.minimum(kb[j], last_row * ldb * 2)) & 0xFFFFFFFF) + 1024 * j
                    mem.check(Bn, b, f"ragged B stage {it_load}")
                    brow = (b - B0) // (ldb * 2)
                    assert ((brow >= t['r0']) & (brow < t['r0'] + Kg)).all(), "B row of another expert"
                last = it_load + 1 >= nk
                if not last:
                    sa += a_step; sb += b_step; it_load += 1
        epilogue(p, t, 'PLAIN', True)
    return ntile

def run_case(N, M, E, H, k, cap, offsets, glu=True, shrink=None):
    """All six launches of the expert FFN forward and backward, with the choice of K pipeline the launcher makes."""
    assert M % 32 == 0 and H % 32 == 0, "other shapes take the plain kernel"
    A_rows = N * k
    global mem
    mem = Mem()
    for n, sz in (('xe', A_rows * M), ('q', A_rows * M), ('dq', A_rows * M), ('dxe', A_rows * M), ('a1', A_rows * H), ('a3', A_rows * H),
                  ('hh', A_rows * H), ('w1', E * M * H), ('w3', E * M * H), ('w2', E * H * M), ('dw1', E * M * H), ('dw3', E * M * H),
                  ('dw2', E * H * M), ('da1', A_rows * H), ('da3', A_rows * H)):
        mem.alloc(n, sz * 2 - (shrink or {}).get(n, 0))
    off = [int(v) for v in offsets]
    assert off[-1] <= A_rows
    base = dict(offsets=off[:-1], row_end=off[1:], E=E, n_pairs=1, max_rows=min(N, cap if cap > 0 else N, N * k), total_rows_bound=N * k,
                gB=0, gC=0, Mfix=0, X=[None, None])
    nonragged = lambda p, LB, epi: kernel64(p, LB, epi) if p['Kfix'] % BK2 == 0 else kernel32(p, LB, epi)
    r = {}
    p = dict(base, A=['xe'], sAi=M, sAk=1, B=['w1', 'w3'], sBk=H, sBn=1, gB=M * H, C=['a1', 'a3', 'hh'], ldc=H, N=H, Kfix=M)
    r['fwd1'] = nonragged(p, TR, 'GLU_FWD' if glu else 'ACT_FWD')
    p = dict(base, A=['hh'], sAi=H, sAk=1, B=['w2'], sBk=M, sBn=1, gB=H * M, C=['q'], ldc=M, N=M, Kfix=H)
    r['fwd2'] = nonragged(p, TR, 'PLAIN')
    p = dict(base, A=['dq'], sAi=M, sAk=1, B=['w2'], sBk=1, sBn=M, gB=H * M, C=['da1', 'da3'], X=['a1', 'a3'], ldc=H, N=H, Kfix=M)
    r['dhh'] = nonragged(p, KC, 'GLU_BWD' if glu else 'ACT_BWD')
    p = dict(base, A=['hh'], sAi=1, sAk=H, B=['dq'], sBk=M, sBn=1, C=['dw2'], ldc=M, gC=H * M, Mfix=H, N=M)
    r['dw2'] = kernel32_ragged(p)
    p = dict(base, A=['da1', 'da3'], sAi=H, sAk=1, B=['w1', 'w3'], sBk=1, sBn=H, gB=M * H, n_pairs=2 if glu else 1, C=['dxe'], ldc=M, N=M, Kfix=H)
    r['dxe'] = nonragged(p, KC, 'PLAIN')
    p = dict(base, A=['xe'], sAi=1, sAk=M, B=['da1', 'da3'], sBk=H, sBn=1, n_pairs=2 if glu else 1, C=['dw1', 'dw3'], ldc=H, gC=M * H, Mfix=M, N=H)
    r['dw1'] = kernel32_ragged(p)
    return r
