"""CPU model of the wavefront schedule's buffer use (csrc/ssrnn.hip, forward()).

A launch holds the stages (block b, layer l) with the same b + l.  Stage (b, l)
reads layer l's input buffer of parity b % 2 and the state c[l]; for the QRNN it
also reads the end of block b-1 in layer l+1's other buffer (the window rows it
copies in front of its output); it writes layer l+1's input buffer of parity
b % 2 (or h for the top layer) and c[l].  Layer 0's buffers are filled from x:
block 0 by a launch of its own, block s+1 by an extra row of workgroups in the
first launch of step s.  The model replays that
with a tag per buffer (the block whose rows it holds) and checks what the
kernels rely on: inside a launch nothing written by one stage is touched by
another, and every read finds the block it expects.  A schedule with a single
buffer per layer must fail the same checks.
"""
import pytest

MAX_BATCH = 8


def run_schedule(n_layers, nblocks, qrnn, stage_in, buffers_per_layer=2):
    act = {}                                  # (layer, parity) -> block held
    c = {l: -1 for l in range(n_layers)}      # layer -> last block folded into the state (-1: initial state)
    h = set()
    par = (lambda b: b % 2) if buffers_per_layer == 2 else (lambda b: 0)
    launches = 0
    if stage_in:
        act[(0, par(0))] = 0                  # staging launch of block 0, ahead of everything in stream order
    for step in range(nblocks + n_layers - 1):
        l_lo = step - (nblocks - 1) if step >= nblocks else 0
        l_hi = min(step, n_layers - 1)
        for l0 in range(l_lo, l_hi + 1, MAX_BATCH):
            stages = [(step - l, l) for l in range(l0, min(l0 + MAX_BATCH, l_hi + 1))]
            launches += 1
            reads, writes = [], []
            for b, l in stages:
                r, w = set(), set()
                if l > 0 or stage_in:
                    r.add(("act", l, par(b)))
                    assert act.get((l, par(b))) == b, ("input buffer holds the wrong block", b, l, act.get((l, par(b))))
                assert c[l] == b - 1, ("state of the wrong block", b, l, c[l])
                r.add(("c", l)); w.add(("c", l))
                if l == n_layers - 1:
                    w.add(("h", b))
                else:
                    w.add(("act", l + 1, par(b)))
                    if qrnn and b > 0:
                        r.add(("act", l + 1, par(b - 1)))
                        assert act.get((l + 1, par(b - 1))) == b - 1, ("window rows come from the wrong block", b, l)
                reads.append(r); writes.append(w)
            staged = stage_in and l0 == l_lo and step + 1 < nblocks
            if staged:                                   # the launch's staging row: block step + 1 into layer 0's buffer
                stages = stages + [("stage-in", step + 1)]
                reads.append(set()); writes.append({("act", 0, par(step + 1))})
            for i in range(len(stages)):
                for j in range(len(stages)):
                    if i != j:
                        assert not (writes[i] & (reads[j] | writes[j])), ("two stages of a launch share a buffer", stages[i], stages[j])
            if staged:
                act[(0, par(step + 1))] = step + 1
                stages = stages[:-1]
            for (b, l), w in zip(stages, writes):       # apply the launch's writes
                c[l] = b
                if l == n_layers - 1:
                    h.add(b)
                else:
                    act[(l + 1, par(b))] = b
    assert h == set(range(nblocks)) and all(c[l] == nblocks - 1 for l in range(n_layers))
    return launches


@pytest.mark.parametrize("n_layers", [1, 2, 3, 4, 8, 9, 19])
@pytest.mark.parametrize("nblocks", [1, 2, 3, 7, 40])
@pytest.mark.parametrize("qrnn", [False, True])
@pytest.mark.parametrize("stage_in", [False, True])
def test_wavefront_buffers_never_collide(n_layers, nblocks, qrnn, stage_in):
    launches = run_schedule(n_layers, nblocks, qrnn, stage_in or qrnn)
    if n_layers <= MAX_BATCH:
        assert launches == nblocks + n_layers - 1


def test_one_buffer_per_layer_would_collide():
    """The model must be able to fail: with a single hand-off buffer per layer, stage (b+1, l-1) overwrites
    what stage (b, l) reads in the same launch."""
    with pytest.raises(AssertionError):
        run_schedule(3, 4, False, True, buffers_per_layer=1)
