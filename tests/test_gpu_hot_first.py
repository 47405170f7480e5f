"""SHVS on a hot-first vocabulary with caller-supplied tail statistics (simple_sample_hot_first)
against the CPU oracle's SHVS with hot_ids = 0 .. H-1: ids, p~, alpha, the acceptance decision.
Rows served from the hot columns (accepted), rows that stream their tail (rejected), rows the
general kernel takes (truncated, greedy, invalid), data errors in the hot part, in the tail and in
the statistics, H = V, float32 and bfloat16."""
import numpy as np
import pytest

import parity_util as P
from oracle import simple_oracle as O
from paper_2512_00719_amd import binding, synth

pytestmark = pytest.mark.gpu


def _dev(x):
    import torch
    return torch.from_numpy(np.ascontiguousarray(x)).to("cuda:0")


def tail_stats(z32, params, H):
    """What the producer of the logits would supply: maximum and tempered exponential sum of the tail."""
    B, V = z32.shape
    ts = np.zeros(B, binding.TAIL_STATS_DTYPE)
    for b in range(B):
        t = z32[b, H:].astype(np.float64)
        tau = float(params["temperature"][b])
        if t.size == 0:
            ts["tail_max"][b] = -np.inf
            continue
        m = np.max(t) if not np.isnan(t).any() else np.nan
        ts["tail_max"][b] = m
        if tau > 0 and np.isfinite(m):
            y = (z32[b, H:] / np.float32(tau)).astype(np.float32).astype(np.float64)   # the tempered values the sampler defines
            ts["tail_sum"][b] = np.sum(np.exp(y - np.float64(np.float32(np.float32(m) / np.float32(tau)))))
    return ts


def _workload(dtype, B, V, seed):
    rng = np.random.default_rng(seed)
    perm = np.arange(V, dtype=np.int64)           # hot-first: column = profile rank
    logits = synth.zipf_profile_logits(B, V, 1.2, 1.0, rng, dtype, perm)
    temp = rng.choice(np.array([0.7, 1.0, 1.3], np.float32), B)
    par = synth.make_params(B, temperature=temp)
    par["top_k"][1] = 40                           # rows the general kernel takes
    par["top_p"][2] = 0.9
    par["min_p"][3] = 0.05
    par["temperature"][4] = 0.0
    par["temperature"][5] = -1.0
    par["rep_penalty"][6] = 1.2                    # (no history is passed: the penalty touches nothing, the row still goes the general way)
    return synth.Workload(f"hot-first-{dtype}", B, V, dtype, logits, par, np.zeros(B + 1, np.int64), np.zeros(0, np.int32), perm=perm)


@pytest.mark.parametrize("dtype,H", [("f32", 2048), ("f32", 8192), ("bf16", 2048), ("bf16", 16384)])
def test_hot_first_matches_the_oracles_shvs(dtype, H):
    import torch
    B, V = 96, 40_960 + 24
    w = _workload(dtype, B, V, 50 + H)
    z32 = w.logits_f32().copy()
    if dtype == "f32":
        w.logits[8, 17] = np.nan; z32[8, 17] = np.nan           # a NaN among the hot columns
        w.logits[9, H + 5] = np.nan; z32[9, H + 5] = np.nan     # a NaN in the tail (the statistics carry it)
    ts = tail_stats(z32, w.params, H)
    wh = synth.Workload(w.name, B, V, dtype, w.logits, w.params, w.hist_ptr, w.hist_ids, hot_ids=np.arange(H, dtype=np.int32), seed=w.seed)
    dev = P.to_device(wh)
    s = binding.Sampler(V, 0, max_B=B)
    ts_dev = _dev(ts.view(np.uint8).reshape(B, 16))
    stream = torch.cuda.current_stream().cuda_stream
    acc = 0
    for step in range(3):
        out = torch.full((B,), -9, dtype=torch.int32, device="cuda:0")
        diag = torch.zeros(B * 32, dtype=torch.uint8, device="cuda:0")
        lg = dev["logits"]
        rc = binding.simple_sample_hot_first(s.ctx, lg.data_ptr(), B, V, binding.SIMPLE_F32 if dtype == "f32" else binding.SIMPLE_BF16,
                                             lg.stride(0), dev["params"].data_ptr(), H, ts_dev.data_ptr(), w.seed, step, 0,
                                             out.data_ptr(), diag.data_ptr(), stream)
        assert rc == 0, binding.simple_strerror(rc)
        torch.cuda.synchronize()
        ids = out.cpu().numpy()
        dg = diag.cpu().numpy().view(binding.ROW_DIAG_DTYPE)
        want = P.run_oracle(wh, step)
        summary = P.compare(ids, dg, want, range(B))
        general = (dg["flags"] & binding.DIAG_GENERAL) > 0
        pattern = (dg["flags"] & binding.DIAG_PATTERN) > 0
        # only the rows that are not plain temperature sampling; of those, a bfloat16 call completes the truncated ones
        # without penalties in force (top-p, min-p, a penalty that meets no history) from counts per bit pattern
        assert (general | pattern)[1:7].all() and not (general | pattern)[10:].any()
        assert pattern[[2, 3, 6]].all() == (dtype == "bf16") and not pattern[[1, 4, 5]].any() and general[[1, 4, 5]].all()
        acc += int(((dg["flags"] & binding.DIAG_ACCEPTED) > 0)[10:].sum())
        if dtype == "f32":
            assert ids[8] == -1 and ids[9] == -1 and want[8].id == -1 and want[9].id == -1
    n = 3 * (B - 10)
    print(f"{dtype} H={H}: {summary}; accepted {acc} of {n} plain rows", flush=True)
    assert 0 < acc < n     # both the hot draw and the tail draw were exercised
    s.close()


def test_hot_first_whole_vocabulary_hot_and_argument_errors():
    import torch
    B, V = 12, 8192
    w = _workload("f32", B, V, 77)
    ts = tail_stats(w.logits, w.params, V)
    wh = synth.Workload(w.name, B, V, "f32", w.logits, w.params, w.hist_ptr, w.hist_ids, hot_ids=np.arange(V, dtype=np.int32), seed=w.seed)
    dev = P.to_device(wh)
    s = binding.Sampler(V, 0, max_B=B)
    ts_dev = _dev(ts.view(np.uint8).reshape(B, 16))
    out = torch.full((B,), -9, dtype=torch.int32, device="cuda:0")
    diag = torch.zeros(B * 32, dtype=torch.uint8, device="cuda:0")
    lg = dev["logits"]

    def call(H, logits=lg, tsd=ts_dev):
        return binding.simple_sample_hot_first(s.ctx, logits.data_ptr(), B, V, binding.SIMPLE_F32, logits.stride(0), dev["params"].data_ptr(),
                                               H, tsd.data_ptr(), w.seed, 2, 0, out.data_ptr(), diag.data_ptr(),
                                               torch.cuda.current_stream().cuda_stream)
    assert call(V) == 0
    torch.cuda.synchronize()
    ids = out.cpu().numpy()
    dg = diag.cpu().numpy().view(binding.ROW_DIAG_DTYPE)
    P.compare(ids, dg, P.run_oracle(wh, 2), range(B))
    plain = np.ones(B, bool); plain[1:7] = False
    assert ((dg["flags"] & binding.DIAG_ACCEPTED) > 0)[plain].all()    # no tail: every draw is accepted
    # the ids equal those of the call without a hot set (all of V hot: same uniform, same walk)
    base = synth.Workload(w.name, B, V, "f32", w.logits, w.params, w.hist_ptr, w.hist_ids, seed=w.seed)
    assert np.array_equal(ids, P.run_gpu(base, 2)[0])
    assert call(1000) == binding.SIMPLE_EINVAL          # not a whole number of tiles
    assert call(V + 1024) == binding.SIMPLE_EINVAL      # beyond the vocabulary
    flat = torch.zeros(B * V + 1, dtype=torch.float32, device="cuda:0")
    assert call(1024, logits=flat[1:].view(B, V)) == binding.SIMPLE_EINVAL   # rows not 16-byte aligned
    # statistics that cannot be: the row is a data error
    bad = ts.copy()
    bad["tail_sum"][10] = -1.0
    bad["tail_max"][11] = np.inf
    assert call(2048, tsd=_dev(bad.view(np.uint8).reshape(B, 16))) == 0
    torch.cuda.synchronize()
    ids = out.cpu().numpy()
    assert ids[10] == -1 and ids[11] == -1 and (ids[[0, 7, 8, 9]] >= 0).all()
    s.close()


def test_hot_first_at_the_size_of_the_shvs_configuration():
    """B = 512, V = 201,088 bf16 (the shape of the SHVS sweep), H = 16384, in the launch configuration the
    benchmark's hot-first sweep times: every row for range, flags and determinism, a seeded sample of
    rows (accepted and rejected ones) against the oracle."""
    import torch
    B, V, H = 512, 201_088, 16_384
    w = _workload("bf16", B, V, 91)
    w.params["top_k"][:] = 0; w.params["top_p"][:] = 1.0; w.params["min_p"][:] = 0.0
    w.params["temperature"][:] = 1.0; w.params["rep_penalty"][:] = 1.0
    ts = tail_stats(w.logits_f32(), w.params, H)
    wh = synth.Workload(w.name, B, V, "bf16", w.logits, w.params, w.hist_ptr, w.hist_ids, hot_ids=np.arange(H, dtype=np.int32), seed=w.seed)
    dev = P.to_device(wh)
    s = binding.Sampler(V, 0, max_B=B)
    ts_dev = _dev(ts.view(np.uint8).reshape(B, 16))
    lg = dev["logits"]
    res = []
    for rep in range(2):
        out = torch.full((B,), -9, dtype=torch.int32, device="cuda:0")
        diag = torch.zeros(B * 32, dtype=torch.uint8, device="cuda:0")
        rc = binding.simple_sample_hot_first(s.ctx, lg.data_ptr(), B, V, binding.SIMPLE_BF16, lg.stride(0), dev["params"].data_ptr(), H,
                                             ts_dev.data_ptr(), w.seed, 4, 0, out.data_ptr(), diag.data_ptr() if rep == 0 else 0,
                                             torch.cuda.current_stream().cuda_stream)
        assert rc == 0
        torch.cuda.synchronize()
        res.append((out.cpu().numpy(), diag.cpu().numpy().view(binding.ROW_DIAG_DTYPE)))
    ids, dg = res[0]
    assert np.array_equal(ids, res[1][0])                     # the same call without a diagnostics buffer
    assert ids.min() >= 0 and ids.max() < V and not (dg["flags"] & (binding.DIAG_ERROR | binding.DIAG_GENERAL)).any()
    acc = (dg["flags"] & binding.DIAG_ACCEPTED) > 0
    assert np.all(ids[acc] < H) and np.all(ids[~acc] >= H) and 0 < (~acc).sum() < B // 4
    rng = np.random.default_rng(3)
    rows = sorted(set(rng.choice(B, 40, replace=False).tolist()) | set(np.flatnonzero(~acc)[:12].tolist()))
    summary = P.compare(ids, dg, P.run_oracle(wh, 4, rows=rows), rows)
    print(f"full size: {summary}; accepted {int(acc.sum())} of {B}", flush=True)
    s.close()
