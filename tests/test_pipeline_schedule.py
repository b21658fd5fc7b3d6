"""CPU models of the software pipelines in csrc/kernel_mfma_lds.hip.h and
csrc/kernel_mfma_packed.hip.h.

The kernel keeps three rings per wavefront -- G register slots of weight lines
in flight from memory, S slots of B fragments, two fragment buffers fed from
the wave's LDS tile -- and unrolls U k-steps per loop iteration, leaving out in
the last iteration the prefetches that would run past the last k-step.  This
model replays that schedule (same slot arithmetic, same compile-time
predicates) and checks that every load index is in range, that every k-step is
loaded exactly once, and that each multiply consumes the fragments of its own
step.  An out-of-range prefetch is a GPU memory fault, so the schedule is
checked here, on the CPU, for every ring configuration the kernel instantiates.
"""
import pytest


def replay(G, S, U, nks, NBH=1):
    """NBH: B fetches (sub-steps) per k-step; sub-step ss = ks*NBH + hb lives in B slot ss % S."""
    assert nks >= U and nks % U == 0 and (U * NBH) % S == 0
    greg = [None] * G
    bring = [None] * S
    afr = [None, None]
    a_ks = 0
    b_col = 0              # k-step the B column cursor points at
    loaded_a, loaded_b = [], []

    def load_a(slot):
        assert 0 <= a_ks < nks, ("weight prefetch out of range", a_ks, nks)
        greg[slot] = a_ks
        loaded_a.append(a_ks)

    def load_b(slot, hb):
        assert 0 <= b_col < nks, ("B prefetch out of range", b_col, nks)
        bring[slot] = (b_col, hb)
        loaded_b.append((b_col, hb))

    # prologue
    for p in range(G):
        load_a(p)
        a_ks += 1
    for ss in range(S - 1):
        load_b(ss % S, ss % NBH)
        if ss % NBH == NBH - 1:
            b_col += 1
    lds = greg[0]
    afr[0] = lds
    ks = 0
    niter = nks // U
    for it in range(niter):
        last = it == niter - 1
        for p in range(U):
            stage_next = (not last) or (p + 1 < U)
            fetch_a = (not last) or (p + G < U)
            assert afr[p & 1] == ks, ("fragments of the wrong step", afr[p & 1], ks)
            for hb in range(NBH):
                ss = p * NBH + hb
                assert bring[ss % S] == (ks, hb), ("B fragments of the wrong sub-step", bring[ss % S], ks, hb)
                tgt = ss + S - 1
                fetch_b = (not last) or (tgt < U * NBH)
                if hb == 0:
                    if stage_next:
                        assert greg[(p + 1) % G] == ks + 1, ("lines of the wrong step go to LDS", greg, ks)
                        lds = greg[(p + 1) % G]
                    if fetch_a:
                        load_a(p % G)
                if fetch_b:
                    load_b(tgt % S, tgt % NBH)
                    if tgt % NBH == NBH - 1:
                        b_col += 1
                if hb == NBH - 1 and stage_next:
                    afr[(p + 1) & 1] = lds
            if fetch_a:
                a_ks += 1
            ks += 1
    assert ks == nks
    assert sorted(loaded_a) == list(range(nks)), "each k-step's weight lines are loaded exactly once"
    assert sorted(loaded_b) == [(k, h) for k in range(nks) for h in range(NBH)], "each B sub-step is loaded exactly once"


# (G, S, NBH) per number of time tiles as in MfmaLdsCfg:
# NT <= 2 -> (4, 4, 1); NT = 4 -> (2, 2, 1); NT = 8 -> (4, 2, 1); NT = 16 -> (2, 2, 2)
@pytest.mark.parametrize("G,S,NBH", [(4, 4, 1), (2, 2, 1), (4, 2, 1), (2, 2, 2)])
@pytest.mark.parametrize("nks", [2, 4, 8, 12, 16, 32, 64, 128])
def test_schedule_is_in_range_and_complete(G, S, NBH, nks):
    U = max(G, S)
    if nks < U or nks % U:
        pytest.skip("the kernel takes its unpipelined path for this k-step count")
    replay(G, S, U, nks, NBH)


def replay_packed(SA, SB, U, nks, NBH=1):
    """The packed-weight kernel: SA register slots of weight fragments (step ks in
    slot ks % SA, refilled SA-1 steps ahead while step ks is multiplied), SB slots
    of B fragments (sub-step ss in slot ss % SB, requested SB-1 sub-steps ahead)."""
    assert nks >= U and nks % U == 0 and U % SA == 0 and (U * NBH) % SB == 0
    aring = [None] * SA
    bring = [None] * SB
    a_ks = 0
    b_col = 0
    loaded_a, loaded_b = [], []

    def load_a(slot):
        assert 0 <= a_ks < nks, ("weight prefetch out of range", a_ks, nks)
        aring[slot] = a_ks
        loaded_a.append(a_ks)

    def load_b(slot, hb):
        assert 0 <= b_col < nks, ("B prefetch out of range", b_col, nks)
        bring[slot] = (b_col, hb)
        loaded_b.append((b_col, hb))

    for p in range(SA - 1):
        load_a(p)
        a_ks += 1
    for ss in range(SB - 1):
        load_b(ss % SB, ss % NBH)
        if ss % NBH == NBH - 1:
            b_col += 1
    ks = 0
    niter = nks // U
    for it in range(niter):
        last = it == niter - 1
        for p in range(U):
            fetch_a = (not last) or (p + SA - 1 < U)
            assert aring[p % SA] == ks, ("weight fragments of the wrong step", aring, ks)
            for hb in range(NBH):
                ss = p * NBH + hb
                assert bring[ss % SB] == (ks, hb), ("B fragments of the wrong sub-step", bring[ss % SB], ks, hb)
                tgt = ss + SB - 1
                fetch_b = (not last) or (tgt < U * NBH)
                if fetch_b:
                    # the slot being refilled must not be the one this sub-step multiplies from
                    assert tgt % SB != ss % SB or SB == 1
                    load_b(tgt % SB, tgt % NBH)
                    if tgt % NBH == NBH - 1:
                        b_col += 1
                if hb == 0 and fetch_a:
                    assert (p + SA - 1) % SA != p % SA
                    load_a((p + SA - 1) % SA)
            if fetch_a:
                a_ks += 1
            ks += 1
    assert ks == nks
    assert sorted(loaded_a) == list(range(nks))
    assert sorted(loaded_b) == [(k, h) for k in range(nks) for h in range(NBH)]


# (SA, SB, NBH) per number of time tiles as in MfmaPkCfg: NT <= 4 -> (4, 4, 1); NT = 8 -> (4, 2, 1); NT = 16 -> (4, 2, 2);
# 8-bit weights: NT = 1 -> (4, 4, 1); NT = 2, 4 -> (4, 2, 1); NT = 8 -> (4, 2, 2); NT = 16 -> (4, 2, 8)
@pytest.mark.parametrize("SA,SB,NBH", [(4, 4, 1), (4, 2, 1), (4, 2, 2), (4, 2, 4), (4, 2, 8)])
@pytest.mark.parametrize("nks", [4, 8, 16, 32, 64])
def test_packed_schedule_is_in_range_and_complete(SA, SB, NBH, nks):
    replay_packed(SA, SB, max(SA, SB), nks, NBH)


def test_model_catches_a_prefetch_that_reaches_too_far():
    """The schedule that refills a slot G+1 steps ahead (one more than the ring
    allows) must be rejected: it reads one k-step past the end."""
    G = S = U = 4
    nks = 8
    a_ks = G + 1          # prologue of that schedule: steps 0..G-1 plus one more
    ks = 0
    with pytest.raises(AssertionError):
        for it in range(nks // U):
            last = it == nks // U - 1
            for p in range(U):
                fetch_a = (not last) or (p + 1 + G < U)
                if fetch_a:
                    assert a_ks < nks, "out of range"
                    a_ks += 1
                ks += 1
