"""GPU parity at the full sizes of the five benchmark configurations, in the launch configuration
the benchmark times.  One oracle row costs about ten milliseconds, so the first call is compared
with the oracle on every row of C2, C3 and C4 and on a seeded sample of C5's 4096 rows, the second
call on a smaller sample; all rows of every call are checked for properties that hold at any size:
ids inside [0, V), no error flags, greedy rows flagged greedy, determinism."""
import numpy as np
import pytest

import parity_util as P
from paper_2512_00719_amd import synth

pytestmark = pytest.mark.gpu


def _sample_rows(w, n, seed):
    rng = np.random.default_rng(seed)
    rows = set(rng.choice(w.B, size=min(n, w.B), replace=False).tolist())
    # make sure every parameter class of the heterogeneous configs is represented
    for k in np.unique(w.params["top_k"]):
        for greedy in (False, True):
            m = np.flatnonzero((w.params["top_k"] == k) & ((w.params["temperature"] == 0) == greedy))
            rows.update(m[:2].tolist())
    return sorted(rows)


@pytest.mark.parametrize("idx,n_first,n_rows", [(2, 256, 40), (3, 1024, 72), (4, 512, 24), (5, 256, 40)])
def test_full_size_config(idx, n_first, n_rows):
    from paper_2512_00719_amd import binding
    print(f"config {idx}: generating", flush=True)
    w = synth.make_config(idx)
    rows_by_step = {0: _sample_rows(w, n_first, 200 + idx), 1: _sample_rows(w, n_rows, 100 + idx)}
    nnz_max = int(np.diff(w.hist_ptr).max()) if w.hist_ids.size else 0
    s = binding.Sampler(w.V, nnz_max)
    dev = P.to_device(w)
    for step in (0, 1):
        rows = rows_by_step[step]
        print(f"config {idx}: step {step} on {w.B} x {w.V} {w.dtype}, {len(rows)} rows against the oracle", flush=True)
        ids, dg = P.run_gpu(w, step, sampler=s, dev=dev)
        assert ids.min() >= 0 and ids.max() < w.V
        assert not (dg["flags"] & binding.DIAG_ERROR).any()
        greedy = w.params["temperature"] == 0
        assert np.array_equal((dg["flags"] & binding.DIAG_GREEDY) > 0, greedy)
        assert np.all(dg["p_chosen"] > 0) and np.all(dg["p_chosen"] <= 1.0 + 1e-6)
        if w.hot_ids is not None:
            assert ((dg["flags"] & binding.DIAG_SHVS) > 0)[~greedy].all()
            a = dg["alpha"][~greedy]
            assert np.all((a >= 0) & (a <= 1))
        ids2, _ = P.run_gpu(w, step, sampler=s, dev=dev)
        assert np.array_equal(ids, ids2)  # same call twice: same ids
        summary = P.compare(ids, dg, P.run_oracle(w, step, rows=rows), rows)
        print(f"config {idx}: step {step} parity {summary}; wide rows {int(((dg['flags'] & 4) > 0).sum())}, "
              f"careful rows {int(((dg['flags'] & 32) > 0).sum())}", flush=True)
    s.close()
