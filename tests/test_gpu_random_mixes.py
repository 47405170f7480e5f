"""GPU parity on seeded random workloads: shapes, dtypes, logit profiles, per-row controls (edge
values included), history lengths and hot sets are all drawn at random, and every row of every call
is compared with the CPU oracle to the bar of test_gpu_parity.py.  The cases are fixed by their
seeds; they exist to reach combinations of routes that no hand-written case names."""
import numpy as np
import pytest

import parity_util as P
from paper_2512_00719_amd import synth

pytestmark = pytest.mark.gpu


def _random_workload(seed, large_batch=False, with_errors=False):
    rng = np.random.default_rng(1000 + seed + (5000 if large_batch else 0))
    dtype = "f32" if rng.random() < 0.5 else "bf16"
    if large_batch:  # more rows than two per compute unit: the 256-thread form of the single-pass kernel
        V = int(rng.choice([8191, 20_000, 33_336]))
        B = int(rng.integers(300, 700))  # 257..512 rows: 512 threads per row; more: 256
    else:
        V = int(rng.choice([97, 1000, 4096, 8191, 20_000, 33_333, 50_008, 70_016]))
        B = int(rng.integers(1, 40))
    kind = rng.integers(0, 4)
    if kind == 0:    # flat
        z = rng.standard_normal((B, V)) * rng.uniform(0.2, 2.0)
    elif kind == 1:  # peaked: a few dominant columns
        z = rng.standard_normal((B, V)) * 1.0
        for b in range(B):
            z[b, rng.choice(V, int(rng.integers(1, 6)), replace=False)] += rng.uniform(4, 15)
    elif kind == 2:  # Zipf profile + noise
        perm = rng.permutation(V)
        z = np.empty((B, V))
        z[:, perm] = -rng.uniform(0.8, 1.4) * np.log(np.arange(1, V + 1))[None, :]
        z += rng.standard_normal((B, V)) * rng.uniform(0.3, 1.5)
    else:            # plateaus: few distinct values
        z = rng.integers(-6, 3, (B, V)).astype(np.float64) * 0.75
    z = z.astype(np.float32)
    if rng.random() < 0.3:
        z[rng.integers(0, B), rng.choice(V, min(V, 50), replace=False)] = -np.inf  # masked tokens
    lens = np.where(rng.random(B) < 0.25, 0, rng.integers(0, 800 if large_batch else 3000, B))
    if rng.random() < 0.5:
        lens[:] = 0
    head = np.argsort(-z, axis=1)[:, : max(1, min(V, 2000))]
    hist_ptr = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    parts = [rng.choice(head[b], int(lens[b])) if rng.random() < 0.7 else rng.integers(0, V, int(lens[b])) for b in range(B)]
    hist_ids = (np.concatenate(parts) if lens.sum() else np.zeros(0)).astype(np.int32)

    def pick(options, p=None):
        return rng.choice(np.array(options, dtype=np.float64), B, p=p)
    params = synth.make_params(
        B,
        temperature=pick([0.0, 0.3, 0.7, 1.0, 1.0, 1.5, 4.0]),
        top_k=pick([0, 0, 1, 5, 40, 200, 1024, 1025, 3000, V - 1, V, V + 5]).astype(np.int32),
        top_p=pick([1.0, 1.0, 0.99, 0.9, 0.5, 0.1, 0.0]),
        min_p=pick([0.0, 0.0, 0.0, 1e-5, 1e-2, 0.3]),
        rep_penalty=pick([1.0, 1.0, 1.05, 1.3, 0.8]),
        freq_penalty=pick([0.0, 0.0, 0.2, 1.0, -0.3]),
        pres_penalty=pick([0.0, 0.0, 0.1, 0.8, -0.2]),
        n_prompt=pick([0, 0, 10, 500, 100_000]).astype(np.int32))
    if with_errors:  # data and parameter errors: the row's id is -1, its neighbours are untouched
        for b in rng.choice(B, max(1, B // 4), replace=False):
            what = rng.integers(0, 5)
            if what == 0:
                z[b, rng.integers(0, V)] = np.nan
            elif what == 1:
                z[b, rng.integers(0, V)] = np.inf
            elif what == 2:
                z[b] = -np.inf
            elif what == 3:
                params["temperature"][b] = -0.5
            else:
                params["rep_penalty"][b] = rng.choice([0.0, -1.0])
    hot = None
    if rng.random() < 0.4:
        hot = np.sort(rng.choice(V, int(rng.integers(1, max(2, V // 3))), replace=False)).astype(np.int32)
    logits = synth.f32_to_bf16_bits(z) if dtype == "bf16" else z
    return synth.Workload(f"random-{seed}", B, V, dtype, logits, params, hist_ptr, hist_ids, hot_ids=hot)


@pytest.mark.parametrize("seed", range(200))
def test_random_mix(seed):
    w = _random_workload(seed)
    print(f"seed {seed}: B={w.B} V={w.V} {w.dtype} nnz={w.hist_ids.size} hot={None if w.hot_ids is None else w.hot_ids.size}", flush=True)
    for step in (0, 1):
        ids, dg = P.run_gpu(w, step)
        P.compare(ids, dg, P.run_oracle(w, step), range(w.B))


@pytest.mark.parametrize("seed", range(24))
def test_random_mix_large_batch(seed):
    w = _random_workload(seed, large_batch=True)
    print(f"seed {seed}: B={w.B} V={w.V} {w.dtype} nnz={w.hist_ids.size} hot={None if w.hot_ids is None else w.hot_ids.size}", flush=True)
    ids, dg = P.run_gpu(w, 0)
    P.compare(ids, dg, P.run_oracle(w, 0), range(w.B))


@pytest.mark.parametrize("seed", range(40))
def test_random_mix_with_error_rows(seed):
    """NaN / +inf logits, all -inf rows, negative temperatures and non-positive repetition penalties in
    a quarter of the rows: those rows return -1 with the error flag, the others their oracle ids."""
    w = _random_workload(3000 + seed, with_errors=True)
    print(f"seed {seed}: B={w.B} V={w.V} {w.dtype} nnz={w.hist_ids.size} hot={None if w.hot_ids is None else w.hot_ids.size}", flush=True)
    ids, dg = P.run_gpu(w, 0)
    want = P.run_oracle(w, 0)
    P.compare(ids, dg, want, range(w.B))
    err = np.array([o.id < 0 for o in want])
    assert err.any() and np.array_equal((dg["flags"] & 1) > 0, err)
