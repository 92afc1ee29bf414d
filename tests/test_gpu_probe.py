"""The measurement aids behind `bench.py --ceiling` (needs an MI355X): they must touch exactly what they claim to."""
import numpy as np
import pytest
import torch

import paper_1909_10802_amd as ga

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n_read,n_write", [(1, 1), (5, 4), (2, 0), (0, 2), (4, 1)])
def test_stream_probe_reads_and_writes_the_named_arrays(n_read, n_write):
    n = 4 * 70_001                                               # several blocks and a ragged last one
    guard = 64
    reads = [torch.full((n + guard,), float(i + 1), device="cuda:0") for i in range(n_read)]
    writes = [torch.full((n + guard,), -7.0, device="cuda:0") for _ in range(n_write)]
    ga.ga_probe_streams(reads, writes, n)
    torch.cuda.synchronize()
    total = float(sum(range(1, n_read + 1)))
    for i, w in enumerate(writes):
        h = w.cpu().numpy()
        assert np.all(h[:n] == total + i) and np.all(h[n:] == -7.0)
    for i, r in enumerate(reads):
        assert bool((r == float(i + 1)).all())


@pytest.mark.parametrize("n_resident", [0, 1, 2])
def test_stream_probe_in_place_with_a_resident_prefix(n_resident):
    # outputs that are the inputs of the same index (the fused update's pattern); the hint changes no value
    n = 4 * 70_001
    guard = 64
    arrays = [torch.full((n + guard,), float(i + 1), device="cuda:0") for i in range(5)]
    ga.ga_probe_streams(arrays, arrays[:4], n, n_resident=n_resident)
    torch.cuda.synchronize()
    for i, a in enumerate(arrays):
        h = a.cpu().numpy()
        want = 15.0 + i if i < 4 else 5.0
        assert np.all(h[:n] == want) and np.all(h[n:] == float(i + 1))


def test_stream_probe_with_tiled_state_arrays():
    # the first three arrays interleaved by tiles of 8192 floats in one buffer, as a master lays out theta, v, m
    n, tile = 4 * 6_001, 8192                                   # three tiles, the last one ragged
    tiles = (n + tile - 1) // tile
    state = torch.full((3 * tiles * tile,), -1.0, device="cuda:0")
    idx = torch.arange(n, device="cuda:0")
    where = (idx // tile) * (3 * tile) + idx % tile
    for a in range(3):
        state[where + a * tile] = float(a + 1)
    rows = [torch.full((n + 64,), float(i + 1), device="cuda:0") for i in (3, 4)]
    arrays = [state, state[tile:], state[2 * tile:]] + rows
    ga.ga_probe_streams(arrays, arrays[:4], n, tiled=True)
    torch.cuda.synchronize()
    h = state.cpu().numpy()
    w = where.cpu().numpy()
    for a in range(3):
        assert np.all(h[w + a * tile] == 15.0 + a)
    untouched = np.ones(h.size, bool)
    for a in range(3):
        untouched[w + a * tile] = False
    assert np.all(h[untouched] == -1.0)
    assert np.all(rows[0].cpu().numpy()[:n] == 18.0) and np.all(rows[0].cpu().numpy()[n:] == 4.0)
    assert bool((rows[1] == 5.0).all())


def test_probe_argument_errors():
    x = torch.zeros(64, device="cuda:0")
    out = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    with pytest.raises(ga.GaError):
        ga.ga_probe_streams([x] * 3, [x], 64)                    # three read streams are not offered
    with pytest.raises(ga.GaError):
        ga.ga_probe_streams([], [], 64)
    with pytest.raises(ga.GaError):
        ga.ga_probe_streams([x], [x], 62)                        # not a multiple of four
    with pytest.raises(ga.GaError):
        ga.ga_probe_streams([x], [x], 64, n_resident=3)          # at most two arrays without the hint
    with pytest.raises(ga.GaError):
        ga.ga_probe_valu(99, 8, 8, out)
    for op in ga.PROBE_OPS:
        ga.ga_probe_valu(op, 4, 16, out)
    torch.cuda.synchronize()
    assert int(out.item()) == 0
