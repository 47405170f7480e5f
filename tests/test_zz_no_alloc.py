"""The entry point that allocates nothing (simple_sample_static: its queues, workspace slots and
hot-set bitmap live in a static device array) against simple_sample on the same inputs, through the
C boundary: two calls in a row, the second with a smaller input, on workloads whose rows use every
part of that array (rows queued for the sliced kernels and for the general kernel, a hot set, more
rows than one launch of the static entry point takes)."""
import numpy as np
import pytest

import parity_util as P
from paper_2512_00719_amd import binding, synth

pytestmark = pytest.mark.gpu


def _workload(B, V, nnz, H, seed_shift):
    w = synth.make_config(3, B=B, V=V, nnz=nnz)
    rng = np.random.default_rng(77 + seed_shift)
    # a third of the rows sample with top-p alone at a high temperature (nucleus wider than the
    # on-chip list: workspace slots), some with penalties that raise logits (general kernel)
    wide = rng.random(B) < 0.35
    w.params["top_k"][wide] = 0
    w.params["min_p"][wide] = 0.0
    w.params["temperature"][wide] = 1.2
    w.params["top_p"][wide] = 0.97
    raising = rng.random(B) < 0.1
    w.params["rep_penalty"][raising] = 0.8
    return w.with_hot(H)


def _static_call(w, dev, step, with_diag, check_mem=True):
    import torch
    out = torch.full((w.B,), -7, dtype=torch.int32, device="cuda:0")
    diag = torch.zeros(w.B * 32, dtype=torch.uint8, device="cuda:0") if with_diag else None
    lg = dev["logits"]
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    rc = binding.simple_sample_static(
        lg.data_ptr(), w.B, w.V, binding.SIMPLE_F32 if w.dtype == "f32" else binding.SIMPLE_BF16, lg.stride(0),
        dev["params"].data_ptr(), dev["hist_ptr"].data_ptr(), dev["hist_ids"].data_ptr(),
        dev["hot_ids"].data_ptr(), dev["hot_ids"].numel(), w.seed, step, 0, out.data_ptr(),
        0 if diag is None else diag.data_ptr(), torch.cuda.current_stream().cuda_stream)
    assert rc == binding.SIMPLE_OK, binding.simple_strerror(rc)
    torch.cuda.synchronize()
    if check_mem:
        assert torch.cuda.mem_get_info()[0] == free_before  # the call took no device memory
    return out.cpu().numpy(), None if diag is None else diag.cpu().numpy().view(binding.ROW_DIAG_DTYPE)


def test_static_entry_point_matches_the_context_entry_point():
    import torch
    first = _workload(150, 40_000, 1500, 3000, 0)   # 150 rows: three launches of the static entry point
    second = _workload(37, 20_000, 600, 500, 1)     # smaller in every size
    for i, w in enumerate((first, second)):
        dev = P.to_device(w)
        s = binding.Sampler(w.V, int(np.diff(w.hist_ptr).max()), max_B=w.B)
        ids_ctx, dg_ctx = P.run_gpu(w, 3 + i, sampler=s, dev=dev)
        s.close()
        torch.cuda.synchronize()
        if i == 0:  # the first call on a device looks the static array up (the runtime places it then)
            _static_call(w, dev, 3 + i, True, check_mem=False)
        ids, dg = _static_call(w, dev, 3 + i, True)
        ids_nd, _ = _static_call(w, dev, 3 + i, False)
        assert np.array_equal(ids, ids_ctx) and np.array_equal(ids_nd, ids_ctx)
        assert ids.min() >= 0 and ids.max() < w.V
        for f in ("alpha", "s_k", "p_chosen", "n_survivors", "flags"):
            a, b = dg[f], dg_ctx[f]
            assert np.array_equal(a, b) or np.array_equal(np.isnan(a), np.isnan(b)) and np.array_equal(a[~np.isnan(a)], b[~np.isnan(b)]), f
        wide = int(((dg["flags"] & binding.DIAG_WIDE) > 0).sum())
        general = int(((dg["flags"] & binding.DIAG_GENERAL) > 0).sum())
        print(f"call {i}: B={w.B} V={w.V}: {wide} rows through the workspace slots, {general} through the general kernel", flush=True)
        assert wide > 0 and general > 0
        # and against the oracle, to the bar of the other parity tests
        P.compare(ids, dg, P.run_oracle(w, 3 + i), range(w.B))
