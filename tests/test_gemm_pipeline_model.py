"""The load / wait / barrier schedule of the two K pipelines of the bf16 grouped GEMM (csrc/gemm_mfma.hip), as a model.

The kernels move operands global -> LDS with loads that write LDS when they land, some time after they are issued; the
only things that order a landing against another wave's LDS read are `s_waitcnt vmcnt(n)` (all but the n youngest loads
of THIS wave have landed; loads of a wave land in issue order) followed by `s_barrier`.  The model below writes out, per
wave, the sequence of events of each kernel as its control flow produces it (prologue, unrolled turns of the ring, the
tail, loads past the end that re-fetch into a free buffer) and checks, for every number of K steps:

  read-after-write   every fragment read of a buffer happens after a barrier at which every wave has waited for the
                     loads of the batch it reads;
  write-after-read   no load that could overwrite a batch is issued before a barrier that follows the last read of it
                     (a load may land at once);
  the epilogue's reuse of the LDS starts after every load has landed in every wave.

It also shows what the abandoned variant did in which a wave left out a group of MFMAs together with the load that is
interleaved with them: the wave's count of issued loads falls short, `vmcnt(n)` returns early and the read-after-write
condition fails (wrong data; whether that variant also formed a wrong address is not something this model holds)."""
import pytest

LOADS_PER_BATCH = 8  # wave-level loads a wave issues per stage (32-k kernel: A and B) or per batch (64-k kernel)


class Wave:
    """One wave's program: events in issue order.  All waves run the same program on their own share of every buffer."""

    def __init__(self):
        self.ev = []

    def issue(self, buf, batch):
        self.ev.append(("issue", buf, batch))

    def read(self, buf, batch):
        self.ev.append(("read", buf, batch))

    def write(self, buf, batch):
        self.ev.append(("write", buf, batch))

    def barrier(self, vmcnt):
        self.ev.append(("barrier", vmcnt))


def check(prog, n_real):
    """prog: a Wave.  Batches >= n_real are re-fetches that nobody reads."""
    issued = []          # (buf, batch) per wave-level load, in order
    landed = 0           # loads guaranteed landed in every wave at the last barrier
    interval = 0
    issue_interval = {}  # (buf, batch) -> interval of its first load
    last_read = {}       # buf -> (batch, interval) of the latest read
    for e in prog.ev:
        if e[0] == "barrier":
            landed = max(landed, len(issued) - e[1])
            interval += 1
        elif e[0] == "issue":
            _, buf, batch = e
            issued.append((buf, batch))
            issue_interval.setdefault((buf, batch), interval)
            if buf in last_read:  # write-after-read: the batch in this buffer was last read strictly before a barrier
                rb, ri = last_read[buf]
                assert batch == rb or ri < interval, f"load of batch {batch} into buffer {buf} may land under the reads of batch {rb}"
        else:
            _, buf, batch = e
            assert batch < n_real, f"a re-fetched batch {batch} is used"
            idx = [i for i, l in enumerate(issued) if l == (buf, batch)]
            assert len(idx) == LOADS_PER_BATCH, f"batch {batch} was not loaded into buffer {buf} in full"
            assert idx[-1] < landed, f"batch {batch} in buffer {buf} is used before a barrier has proved it landed"
            newer = [l for l in issued[idx[-1] + 1:] if l[0] == buf]
            assert not newer, f"buffer {buf} may already hold batch {newer[0][1]} when batch {batch} is used"
            if e[0] == "read":
                last_read[buf] = (batch, interval)
    assert landed == len(issued), "the LDS goes to the epilogue with loads in flight"


def program32(nk, ragged_tail=False, skip=None, vmcnt=16, target=lambda S: (S + 3) % 4):
    """gg_mfma_kernel: four LDS stages of 32 k, three in flight, one barrier (vmcnt 16) per K stage."""
    w = Wave()
    if nk > 0:
        for s in range(3):
            for _ in range(LOADS_PER_BATCH):
                w.issue(s, s)

        def iteration(S, it):
            w.barrier(vmcnt)
            if ragged_tail and it == nk - 1:
                w.write(S, it)   # rows past the expert's last are zeroed in LDS
                w.barrier(0)     # __syncthreads()
            for half in range(2):
                for j in range(4):
                    w.read(S, it)                                  # fragment reads of this stage
                    if skip != (it, half, j):
                        w.issue(target(S), it + 3)                 # one load of K stage it + 3 per group
        iteration(0, 0)
        it = 1
        while it + 4 <= nk:
            for S in (1, 2, 3, 0):
                iteration(S, it); it += 1
        base = it
        if base < nk: iteration(1, base)
        if base + 1 < nk: iteration(2, base + 1)
        if base + 2 < nk: iteration(3, base + 2)
    w.barrier(0)  # s_waitcnt vmcnt(0); __syncthreads(): the epilogue takes the LDS
    return w


def program64(nb, skip=None, vmcnt=8):
    """gg_mfma64_kernel: 64-k batches in a ring of five buffers, A and B batches alternate, one barrier (vmcnt 8) per 64 k."""
    w = Wave()
    if nb > 0:
        for j in range(3):                     # A0 B0 A1
            for _ in range(LOADS_PER_BATCH):
                w.issue(j % 5, j)

        def half_step(ph, m):
            U, H = ph // 2, ph % 2
            abuf, bbuf = (2 * U) % 5, (2 * U + 1) % 5
            lbuf = (2 * U + 3) % 5 if H == 0 else (2 * U + 4) % 5
            nominal = 2 * m + 3 if H == 0 else 2 * m + 4
            assert abuf == (2 * m) % 5 and bbuf == (2 * m + 1) % 5 and lbuf == nominal % 5
            if H == 0:
                w.barrier(vmcnt)
            for part in range(2):
                for j in range(4):
                    w.read(bbuf if j < 2 else abuf, 2 * m + 1 if j < 2 else 2 * m)
                    if skip != (m, H, part, j):
                        w.issue(lbuf, nominal)
        nh = 2 * nb
        half_step(0, 0)
        h = 1
        while h + 10 <= nh:
            for ph in (1, 2, 3, 4, 5, 6, 7, 8, 9, 0):
                half_step(ph, h // 2); h += 1
        rest = nh - h
        for r in range(rest):
            half_step(1 + r, (h + r) // 2)
    w.barrier(0)
    return w


@pytest.mark.parametrize("nk", range(0, 23))
def test_the_32k_pipeline_never_reads_a_stage_that_may_not_have_landed(nk):
    check(program32(nk), nk)
    check(program32(nk, ragged_tail=True), nk)


@pytest.mark.parametrize("nb", range(0, 34))
def test_the_64k_ring_never_reads_a_batch_that_may_not_have_landed(nb):
    check(program64(nb), 2 * nb)


def test_a_wave_that_leaves_out_a_group_breaks_the_wait_arithmetic():
    with pytest.raises(AssertionError, match="not loaded|before a barrier"):
        check(program32(12, skip=(3, 1, 2)), 12)
    with pytest.raises(AssertionError, match="not loaded|before a barrier"):
        check(program64(12, skip=(4, 0, 1, 3)), 24)


def test_the_check_notices_a_weaker_wait_and_a_buffer_reused_too_early():
    with pytest.raises(AssertionError, match="before a barrier"):
        check(program32(9, vmcnt=17), 9)      # one load of the stage about to be read may still be in flight
    with pytest.raises(AssertionError, match="before a barrier"):
        check(program64(9, vmcnt=9), 18)
    with pytest.raises(AssertionError, match="may land under the reads|may already hold"):
        check(program32(9, target=lambda S: S), 9)            # loading into the stage that is being read
    check(program32(9, vmcnt=15), 9)          # a stronger wait is still correct
