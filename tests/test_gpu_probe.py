"""The bare gather behind bench.py's `roofline.bare_gather` (stgn_probe_gather, through the C ABI): every
group of 16 lanes sums its rows; lane s of a group owns floats 4 s .. 4 s + 3 of every 64-float piece of a row.
Checked against the same sums in numpy (fp64), so that the timed launch is known to read what it claims."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("width,groups,per", [(64, 37, 5), (256, 1000, 3), (256, 1, 1), (64, 4099, 20)])
def test_bare_gather_sums_the_rows_it_is_given(width, groups, per):
    import torch
    from paper_2603_21090_amd import binding
    binding.load_library()
    rng = np.random.default_rng(width + groups)
    rows = 5000
    table = rng.standard_normal((rows, width)).astype(np.float32)
    idx = rng.integers(0, rows, groups * per).astype(np.int32)
    t = torch.from_numpy(table).cuda()
    i = torch.from_numpy(idx).cuda()
    out = torch.full((groups * 16,), float("nan"), dtype=torch.float32, device="cuda")
    binding.probe_gather(t, i, per, out, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    got = out.cpu().numpy().reshape(groups, 16)
    picked = table[idx.reshape(groups, per)].astype(np.float64)                 # [groups, per, width]
    want = picked.reshape(groups, per, width // 64, 16, 4).sum(axis=(1, 2, 4))  # lane s: floats 4 s .. 4 s + 3 of every piece
    scale = np.abs(picked).reshape(groups, per, width // 64, 16, 4).sum(axis=(1, 2, 4))
    assert np.all(np.abs(got - want) <= 1e-5 * scale + 1e-6)


def test_bare_gather_rejects_what_it_cannot_run():
    import torch
    from paper_2603_21090_amd import binding
    L = binding.load_library()
    t = torch.zeros((10, 48), dtype=torch.float32, device="cuda")
    i = torch.zeros(4, dtype=torch.int32, device="cuda")
    o = torch.zeros(64, dtype=torch.float32, device="cuda")
    assert L.stgn_probe_gather(t.data_ptr(), 10, 192, i.data_ptr(), 4, 1, o.data_ptr(), None) == -1     # row size
    assert L.stgn_probe_gather(None, 10, 256, i.data_ptr(), 4, 1, o.data_ptr(), None) == -1
    assert L.stgn_probe_gather(t.data_ptr(), 10, 256, i.data_ptr(), 0, 1, o.data_ptr(), None) == -1
