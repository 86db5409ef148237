"""The measurement helpers of the library do what their declarations say (GPU)."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gs():
    import paper_2007_03179_amd as gs
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    gs.lib()
    return gs


@pytest.mark.parametrize("row_bytes,lanes,load,policy", [(128, 8, 16, 0), (128, 8, 16, 1), (128, 8, 16, 2), (128, 16, 8, 0),
                                                         (128, 32, 4, 0), (32, 2, 16, 0), (128, 4, 16, 0), (256, 16, 16, 0),
                                                         (1024, 64, 16, 0)])
@pytest.mark.parametrize("flight", [2, 16])
def test_shaped_gather_reads_the_requested_part_of_every_requested_row(gs, row_bytes, lanes, load, policy, flight):
    rows, n = 3000, 77_777
    words = row_bytes // 4
    table = torch.arange(rows, dtype=torch.float32, device="cuda").repeat_interleave(words).view(rows, words).contiguous()
    idx = torch.from_numpy(np.random.default_rng(6).integers(0, rows, n).astype(np.int32)).cuda()
    print(f"  case gather shape row={row_bytes} lanes={lanes} load={load} policy={policy} flight={flight}", flush=True)
    out = gs.gespmm_calibration_gather_shape(table, row_bytes, idx, lanes, load, flight, policy)
    torch.cuda.synchronize()
    # every gathered word of row k holds k; a request reads lanes * load / 4 words; positions past the end of
    # idx re-read its last element (each group of lanes handles `flight` consecutive requests)
    tail = (-n) % flight
    want = (float(idx.double().sum()) + tail * float(idx[-1])) * lanes * load / 4
    assert abs(float(out.double().sum()) - want) <= 1e-6 * want


def test_shaped_gather_rejects_shapes_it_does_not_have(gs):
    table = torch.zeros(1024, device="cuda")
    idx = torch.zeros(10, dtype=torch.int32, device="cuda")
    for bad in (dict(lanes_per_row=3), dict(load_bytes=12), dict(in_flight=5), dict(cache_policy=3),
                dict(lanes_per_row=16, load_bytes=16), dict(lanes_per_row=16, load_bytes=8, cache_policy=1)):
        with pytest.raises(gs.GespmmError):
            gs.gespmm_calibration_gather_shape(table, 128, idx, **bad)
