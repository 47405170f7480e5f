"""GPU tests of the two measurement aids of the C boundary: the read-only row-maximum reduction
(checked against its plain definition, numpy's max over the same values) and the per-launch
durations of the profiled kernel."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,V,stride", [(3, 1, 8), (5, 1000, 1000), (7, 4099, 4104), (33, 40000, 40000),
                                        (4, 128256, 128256)])
def test_stream_probe_row_max(dtype, B, V, stride):
    import torch
    from paper_2512_00719_amd import binding
    print(f"stream probe {dtype} B={B} V={V} stride={stride}", flush=True)
    rng = np.random.default_rng(B * 1000 + V)
    x = (rng.standard_normal((B, stride)) * 6.0).astype(np.float32)
    x[0, : min(V, 17)] = -np.inf                      # -inf values take part like any other
    x[:, V:] = 1e30                                   # padding columns must not be read
    if dtype == "bf16":
        bits = (x.view(np.uint32) >> 16).astype(np.uint16)
        x = (bits.astype(np.uint32) << 16).view(np.float32)
        dev = torch.from_numpy(bits.view(np.int16)).cuda()
        code = binding.SIMPLE_BF16
    else:
        dev = torch.from_numpy(x).cuda()
        code = binding.SIMPLE_F32
    want = x[:, :V].max(axis=1)
    out = torch.full((B,), 123.0, dtype=torch.float32, device="cuda")
    rc = binding.simple_stream_probe(dev.data_ptr(), B, V, code, stride, out.data_ptr(),
                                     torch.cuda.current_stream().cuda_stream)
    assert rc == 0
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), want)


def test_stream_probe_argument_errors():
    import torch
    from paper_2512_00719_amd import binding
    x = torch.zeros(4, 64, device="cuda")
    out = torch.zeros(4, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    assert binding.simple_stream_probe(x.data_ptr(), 0, 64, 0, 64, out.data_ptr(), st) == 0
    assert binding.simple_stream_probe(0, 4, 64, 0, 64, out.data_ptr(), st) == binding.SIMPLE_EINVAL
    assert binding.simple_stream_probe(x.data_ptr(), 4, 64, 0, 63, out.data_ptr(), st) == binding.SIMPLE_EINVAL
    assert binding.simple_stream_probe(x.data_ptr(), 4, 64, 7, 64, out.data_ptr(), st) == binding.SIMPLE_EINVAL
    assert binding.simple_stream_probe(x.data_ptr() + 4, 3, 60, 0, 64, out.data_ptr(), st) == binding.SIMPLE_EINVAL
    assert binding.simple_stream_probe(x.data_ptr(), 4, 61, 0, 61, out.data_ptr(), st) == binding.SIMPLE_EINVAL
    torch.cuda.synchronize()


def test_profile_read_launches():
    import torch
    import parity_util as P
    from paper_2512_00719_amd import binding, synth
    w = synth.make_config(1)
    s = binding.Sampler(w.V, int(np.diff(w.hist_ptr).max()) if w.hist_ids.size else 0)
    dev = P.to_device(w)
    assert binding.simple_profile_enable(s.ctx, True) == 0
    for step in range(5):
        P.run_gpu_no_diag(w, step, sampler=s, dev=dev)
    torch.cuda.synchronize()
    n, total = binding.simple_profile_read(s.ctx)
    ms = binding.simple_profile_read_launches(s.ctx)
    assert n == 5 and ms.shape == (5,)
    assert np.all(ms > 0) and abs(float(ms.sum()) - total) < 1e-3 * total + 1e-6
    assert binding.simple_profile_read_launches(s.ctx, cap=2).shape == (2,)
    binding.simple_profile_enable(s.ctx, False)
    s.close()
