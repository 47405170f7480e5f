"""The same call gives the same ids every time: on a sampler that was just created, on one that
has served other shapes, with and without a diagnostics buffer.  The ids are a function of the
inputs, the seed, the step and the row index alone (paper section 5.1, deterministic random
numbers), so any difference between two calls is a race or a read of stale on-chip memory in a
kernel; the workloads here send many rows through the multi-pass route of the general kernel (large
top-k with penalties on rows that are not 16-byte aligned), through the sliced whole-vocabulary
kernels and through the pattern-count kernel, the routes with the most hand-offs between waves."""
import numpy as np
import pytest

import parity_util as P
import test_gpu_random_mixes as M
from paper_2512_00719_amd import binding, synth

pytestmark = pytest.mark.gpu


def _ids(w, dev, with_diag, sampler=None):
    import torch
    own = sampler is None
    if own:
        nnz_max = int(np.diff(w.hist_ptr).max()) if w.hist_ids.size else 0
        sampler = binding.Sampler(w.V, nnz_max)
    diag = torch.zeros(w.B * 32, dtype=torch.uint8, device="cuda:0") if with_diag else None
    out = sampler.sample(dev["logits"], dev["params"], dev["hist_ptr"], dev["hist_ids"], dev["hot_ids"],
                         seed=w.seed, step=0, diag=diag, V=w.V)
    torch.cuda.synchronize()
    ids = out.cpu().numpy().copy()
    if own:
        sampler.close()
    return ids


@pytest.mark.parametrize("seed", [0, 1, 2, 5])
def test_fresh_samplers_repeat_the_ids(seed):
    """Twelve rounds; in each, another workload's call comes first (other kernels, other shapes: what
    they leave in the compute units' on-chip memory is not what this call left there last time), then
    this workload on a sampler of its own, with and without the diagnostics buffer."""
    w = M._random_workload(seed, large_batch=True)
    other = M._random_workload(seed + 7)
    print(f"seed {seed}: B={w.B} V={w.V} {w.dtype} nnz={w.hist_ids.size}", flush=True)
    want = P.run_oracle(w, 0)
    ref = None
    for rnd in range(12):
        _ids(other, P.to_device(other), rnd % 2 == 0)
        dev = P.to_device(w)  # uploaded again: a first call on memory no kernel has touched
        for with_diag in (True, False):
            ids = _ids(w, dev, with_diag)
            if ref is None:
                ref = ids
                hard = [r for r, o in enumerate(want) if int(ids[r]) != o.id and not (o.ambiguous and int(ids[r]) in o.alt_ids)]
                assert not hard, hard[:10]
            d = np.flatnonzero(ids != ref)
            assert d.size == 0, (rnd, with_diag, d[:10], ids[d[:10]], ref[d[:10]])


def test_one_sampler_repeats_the_ids_across_routes():
    """A reduced C3 batch (float32, histories, the mix of controls of that configuration: single-pass
    kernel, sliced kernels, general kernel) and a bfloat16 batch without penalties (pattern-count kernel), 40 calls each on
    one sampler, alternating with the other shape's calls."""
    import torch
    a = synth.make_config(3, B=192, V=40_064, nnz=300)
    z = synth.zipf_profile_logits(96, 50_048, 1.1, 1.0, np.random.default_rng(11), "bf16", np.random.default_rng(12).permutation(50_048))
    b = synth.Workload("bf16-plain", 96, 50_048, "bf16", z, synth.make_params(96, temperature=0.9, top_p=0.95), np.zeros(97, np.int64),
                       np.zeros(0, np.int32))
    devs = {w.name: P.to_device(w) for w in (a, b)}
    nnz_max = int(np.diff(a.hist_ptr).max())
    s = binding.Sampler(max(a.V, b.V), nnz_max)
    ref = {}
    for i in range(40):
        for w in (a, b):
            ids = _ids(w, devs[w.name], i % 3 == 0, sampler=s)
            if w.name not in ref:
                ref[w.name] = ids
            d = np.flatnonzero(ids != ref[w.name])
            assert d.size == 0, (w.name, i, d[:10])
    s.close()
    torch.cuda.synchronize()
