"""GPU parity: the HIP library (through the C boundary) against the CPU oracle, element by element.

Bar: token ids bit-exact, except rows where a decision lies within 1e-6 (relative) of a boundary
-- those may return one of the oracle's alternative ids and are limited to 1e-4 of the rows (at
least one row on small batches); p~ of the chosen token within 1e-5 relative.
"""
import numpy as np
import pytest

import parity_util as P
from oracle import simple_oracle as O
from paper_2512_00719_amd import synth

pytestmark = pytest.mark.gpu


def _binding():
    from paper_2512_00719_amd import binding
    return binding


def _check(w, steps=(0, 1), rows=None, **kw):
    rows = list(range(w.B)) if rows is None else list(rows)
    out = []
    for step in steps:
        ids, dg = P.run_gpu(w, step)
        out.append((ids, dg, P.compare(ids, dg, P.run_oracle(w, step, rows=rows), rows, **kw)))
    return out


# ---------------------------------------------------------------- reduced versions of the configs
@pytest.mark.parametrize("idx,B,V,nnz,H", [
    (1, None, None, None, None),          # Tiny, as specified
    (2, 24, 30_000 + 8, 300, None),       # bf16, k=20, p=0.8
    (3, 96, 33_000, 700, None),           # fp32 heterogeneous rows, greedy rows
    (4, 24, 40_000 + 16, None, 3000),     # bf16 SHVS, nucleus over all of V
    (5, 48, 50_000 + 24, 1500, 5000),     # bf16, all penalties, SHVS
])
def test_reduced_configs_all_rows(idx, B, V, nnz, H):
    w = synth.make_config(idx, B=B, V=V, nnz=nnz, H=H)
    res = _check(w, steps=(0, 1, 2))
    if idx in (4, 5):
        assert all((dg["flags"] & 8).any() for _, dg, _ in res)  # SHVS was used


def test_several_tiles_and_ragged_tail_fp32_unaligned_stride():
    """V not a multiple of the vector width, row stride larger than V and odd: scalar-load route."""
    import torch
    binding = _binding()
    w = synth.make_config(3, B=12, V=9001, nnz=300)
    stride = 9001 + 3
    padded = np.full((w.B, stride), 1e30, np.float32)  # padding must never be read as a logit
    padded[:, :w.V] = w.logits
    dev = P.to_device(w)
    dev["logits"] = torch.from_numpy(padded).cuda()
    ids, dg = P.run_gpu(w, 5, dev=dev)
    P.compare(ids, dg, P.run_oracle(w, 5), range(w.B))
    # and a base pointer that is not 16-byte aligned
    flat = torch.zeros(w.B * stride + 1, dtype=torch.float32, device="cuda")
    flat[1:] = torch.from_numpy(padded).cuda().reshape(-1)
    dev["logits"] = flat[1:].view(w.B, stride)
    ids2, dg2 = P.run_gpu(w, 5, dev=dev)
    assert np.array_equal(ids, ids2)


@pytest.mark.parametrize("V", [1, 2, 3, 7, 64, 1023, 1024, 1025, 4096, 4097, 8192 + 5])
def test_small_and_odd_vocabularies(V):
    rng = np.random.default_rng(V)
    B = 6
    logits = (rng.standard_normal((B, V)) * 2).astype(np.float32)
    params = synth.make_params(B, temperature=[0.7, 1.0, 0.0, 1.3, 0.9, 1.0], top_k=[0, 3, 0, 50, 2000, 0],
                               top_p=[0.9, 1.0, 1.0, 0.95, 0.5, 1.0], min_p=[0, 0, 0, 0.02, 0, 0.1],
                               rep_penalty=1.2, freq_penalty=0.1, pres_penalty=0.05)
    nnz = min(V, 5)
    hist_ptr = np.arange(B + 1, dtype=np.int64) * nnz
    hist_ids = rng.integers(0, V, B * nnz).astype(np.int32)
    w = synth.Workload(f"odd{V}", B, V, "f32", logits, params, hist_ptr, hist_ids)
    _check(w, steps=(0, 3))


def test_bf16_ties_everywhere():
    """Coarse bf16 values produce large tie groups at every cut; ids must follow (y desc, id asc)."""
    rng = np.random.default_rng(5)
    B, V = 16, 20_000
    x = np.round(rng.standard_normal((B, V)) * 2).astype(np.float32) / 2  # ~20 distinct values
    params = synth.make_params(B, temperature=0.8, top_k=[0, 1, 5, 40, 300, 1000, 1024, 1500] * 2,
                               top_p=[1.0, 0.3, 0.9, 0.7] * 4, min_p=[0, 0, 0.2, 0] * 4)
    w = synth.Workload("ties", B, V, "bf16", synth.f32_to_bf16_bits(x), params,
                       np.zeros(B + 1, np.int64), np.zeros(0, np.int32))
    _check(w, steps=(0, 1))


def test_degenerate_rows():
    B, V = 10, 6000
    rng = np.random.default_rng(6)
    z = (rng.standard_normal((B, V)) * 2).astype(np.float32)
    z[0, :] = 1.25                       # all equal
    z[1, :] = np.arange(V) * 1e-3        # ascending: every element beats all before it
    z[2, :] = -np.arange(V) * 1e-3       # descending
    z[3, 100:] = -np.inf                 # mostly -inf
    z[4, 17] = np.nan                    # NaN -> id -1
    z[5, 4000] = np.inf                  # +inf -> id -1
    z[6, :] = -np.inf                    # nothing to draw -> id -1
    z[7, :] = 0.0; z[7, 5] = -0.0        # signed zeros tie
    z[8, :] = 3e38                       # overflow of z / tau -> error
    params = synth.make_params(B, temperature=[1.0, 0.7, 0.7, 1.0, 1.0, 1.0, 1.0, 1.0, 0.5, 0.0],
                               top_k=[7, 100, 100, 0, 10, 10, 10, 3, 10, 0], top_p=[1.0, 0.9, 0.9, 1.0, 1, 1, 1, 1, 1, 1])
    w = synth.Workload("degenerate", B, V, "f32", z, params, np.zeros(B + 1, np.int64), np.zeros(0, np.int32))
    for step in (0, 1, 2):
        ids, dg = P.run_gpu(w, step)
        orc = P.run_oracle(w, step)
        P.compare(ids, dg, orc, range(B))
        assert list(ids[[4, 5, 6, 8]]) == [-1, -1, -1, -1] and all(dg["flags"][[4, 5, 6, 8]] & 1)
        assert ids[0] < 7 and ids[7] < 3


def test_wide_routes_top_k_above_list_and_no_truncation():
    rng = np.random.default_rng(7)
    B, V = 12, 30_000
    z = (rng.standard_normal((B, V)) * 1.5).astype(np.float32)
    params = synth.make_params(B, temperature=[1.0, 0.8, 1.2] * 4,
                               top_k=[0, 2000, 29_999, 5000, 0, 0, 1025, 0, 3000, 0, 0, 20_000],
                               top_p=[1.0, 1.0, 1.0, 0.9, 0.999, 0.5, 0.99, 1.0, 0.2, 0.97, 1.0, 0.6],
                               min_p=[0, 0, 0, 0, 0, 0, 0, 1e-4, 0, 1e-3, 1e-6, 0])
    w = synth.Workload("wide", B, V, "f32", z, params, np.zeros(B + 1, np.int64), np.zeros(0, np.int32))
    res = _check(w, steps=(0, 1, 2))
    assert (res[0][1]["flags"] & 4).sum() >= 8  # most of these rows need the multi-pass route


def test_penalty_variants_prompt_split_and_ragged_history():
    rng = np.random.default_rng(8)
    B, V = 16, 12_000
    z = (rng.standard_normal((B, V)) * 2).astype(np.float32)
    lens = rng.integers(0, 900, B)
    lens[0] = 0
    lens[1] = 1
    hist_ptr = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    top = np.argsort(-z, axis=1)[:, :40]  # history hits the head of the distribution, with repeats
    hist_ids = np.concatenate([rng.choice(top[b], lens[b]) for b in range(B)]).astype(np.int32)
    params = synth.make_params(
        B, temperature=[0.9, 0.0] * 8, top_k=[0, 30, 200, 0] * 4, top_p=[0.9, 1.0, 0.8, 0.95] * 4,
        rep_penalty=[1.3, 1.0, 0.8, 1.1] * 4,          # below one raises logits: per-element route
        freq_penalty=[0.5, 0.0, -0.3, 0.2] * 4, pres_penalty=[0.1, 0.4, 0.0, -0.2] * 4,
        n_prompt=[0, 5, 1000, 3] * 4)
    w = synth.Workload("pen", B, V, "f32", z, params, hist_ptr, hist_ids)
    _check(w, steps=(0, 1, 2))


def test_history_errors_are_flagged_not_fatal():
    binding = _binding()
    w = synth.make_config(1)
    w.hist_ids = w.hist_ids.copy()
    w.hist_ids[3] = w.V + 5      # row 0: ignored and flagged
    w.hist_ids[64 + 7] = -2      # row 1
    ids, dg = P.run_gpu(w, 0)
    assert (dg["flags"][:2] & binding.DIAG_BAD_HISTORY_ID).all() and not (dg["flags"][2:] & binding.DIAG_BAD_HISTORY_ID).any()
    good = synth.make_config(1)
    keep = np.ones(good.hist_ids.size, bool)
    keep[[3, 64 + 7]] = False
    good.hist_ids = good.hist_ids[keep]
    good.hist_ptr = np.array([0, 63, 126, 190, 254], np.int64)
    P.compare(ids, dg, P.run_oracle(good, 0), range(4))
    # history longer than the context allows: that row errors, the others are unaffected
    import torch
    s = binding.Sampler(w.V, 32)
    dev = P.to_device(synth.make_config(1))
    dev["hist_ptr"] = torch.tensor([0, 20, 84, 100, 132], dtype=torch.int64, device="cuda")
    good.hist_ptr = np.array([0, 20, 84, 100, 132], np.int64)
    good.hist_ids = synth.make_config(1).hist_ids
    ids, dg = P.run_gpu(good, 0, sampler=s, dev=dev)
    assert ids[1] == -1 and dg["flags"][1] & binding.DIAG_HISTORY_TOO_LONG
    orc = P.run_oracle(good, 0, rows=[0, 2, 3])
    P.compare(ids, dg, orc, [0, 2, 3])
    s.close()


def test_bad_parameters_give_minus_one():
    w = synth.make_config(1)
    w.params = w.params.copy()
    w.params["temperature"][1] = -0.5
    w.params["rep_penalty"][2] = 0.0
    ids, dg = P.run_gpu(w, 0)
    orc = P.run_oracle(w, 0)
    assert [o.id for o in orc][1:3] == [-1, -1] and list(ids[1:3]) == [-1, -1]
    P.compare(ids, dg, orc, range(4))


# ---------------------------------------------------------------- determinism --------------------
def test_ids_do_not_depend_on_how_the_batch_is_split():
    """Section 5.1: partitioning the rows over samplers must not change any id."""
    import torch
    binding = _binding()
    w = synth.make_config(3, B=40, V=20_000, nnz=400)
    whole, _ = P.run_gpu(w, 9)
    dev = P.to_device(w)
    s = binding.Sampler(w.V, 400)
    parts = np.full(w.B, -7, np.int32)
    for lo, hi in ((0, 1), (1, 17), (17, 40)):
        hp = dev["hist_ptr"][lo:hi + 1].clone()
        out = s.sample(dev["logits"][lo:hi], dev["params"][lo:hi], hp, dev["hist_ids"], seed=w.seed, step=9,
                       row_offset=lo, V=w.V)
        torch.cuda.synchronize()
        parts[lo:hi] = out.cpu().numpy()
    again, _ = P.run_gpu(w, 9, sampler=s, dev=dev)
    s.close()
    assert np.array_equal(whole, parts) and np.array_equal(whole, again)


def test_uniform_logits_expose_the_random_bits():
    """All-equal logits without truncation: id = floor(u_draw * V), so the device's Philox words
    and the uniform conversion are compared bit for bit through the ids."""
    B, V = 512, 4096
    w = synth.Workload("philox", B, V, "f32", np.zeros((B, V), np.float32), synth.make_params(B),
                       np.zeros(B + 1, np.int64), np.zeros(0, np.int32))
    for step in (0, 1, (1 << 40) + 3):
        ids, _ = P.run_gpu(w, step)
        u = O.row_uniforms(w.seed, np.arange(B), step)[0]
        assert np.array_equal(ids, np.floor(u * V).astype(np.int32))


# ---------------------------------------------------------------- SHVS ---------------------------
def test_shvs_whole_vocabulary_hot_set_equals_full_path():
    w = synth.make_config(4, B=16, V=30_000, H=30_000)
    w.hot_ids = np.arange(w.V, dtype=np.int32)
    ids_hot, dg = P.run_gpu(w, 4)
    w.hot_ids = None
    ids_full, _ = P.run_gpu(w, 4)
    assert np.array_equal(ids_hot, ids_full) and (dg["flags"] & 16).all() and np.allclose(dg["alpha"], 1.0)


def test_shvs_distribution_chi_square_and_acceptance_rate():
    """One row replicated over the batch (each copy has its own row index, hence its own uniforms):
    the drawn ids fit the oracle's p~ and the acceptance rate fits alpha."""
    from scipy import stats
    rng = np.random.default_rng(12)
    B, V = 4096, 3000
    row = (rng.standard_normal(V) * 2.2).astype(np.float32)
    hot = np.argsort(-row)[:40].astype(np.int32)
    hot = hot[rng.permutation(40)]
    for par in (synth.make_params(B, temperature=1.1, top_p=0.98), synth.make_params(B, top_k=300, temperature=1.4)):
        w = synth.Workload("chi", B, V, "f32", np.tile(row, (B, 1)), par, np.zeros(B + 1, np.int64),
                           np.zeros(0, np.int32), hot_ids=hot)
        counts = np.zeros(V)
        acc = 0
        steps = 25
        for step in range(steps):
            ids, dg = P.run_gpu(w, step)
            counts += np.bincount(ids, minlength=V)
            acc += int(((dg["flags"] & 16) > 0).sum())
        d = O.row_distribution(row, par[0])
        p = d.probs()
        alpha = O.shvs_masses(d, O.hot_mask_from_ids(hot, V))[2]
        N = B * steps
        assert abs(acc / N - alpha) < 4 * np.sqrt(alpha * (1 - alpha) / N)
        assert np.all(counts[p == 0] == 0)
        order = np.argsort(-p)
        e, c = p[order] * N, counts[order]
        cut = int(np.searchsorted(-e, -5.0))
        if e[cut:].sum() > 0:  # pool the low-probability tail into one cell
            e, c = np.append(e[:cut], e[cut:].sum()), np.append(c[:cut], c[cut:].sum())
        else:
            e, c = e[:cut], c[:cut]
        assert stats.chisquare(c, e * c.sum() / e.sum()).pvalue > 1e-4
        np.testing.assert_allclose(dg["alpha"], alpha, rtol=1e-6)


def test_shvs_installed_hot_set_and_bad_hot_ids():
    import torch
    binding = _binding()
    w = synth.make_config(4, B=8, V=20_000, H=1500)
    per_call, _ = P.run_gpu(w, 2)
    s = binding.Sampler(w.V, 0)
    dev = P.to_device(w)
    s.set_hot_set(dev["hot_ids"], w.V)
    out = s.sample(dev["logits"], dev["params"], H=-1, seed=w.seed, step=2, V=w.V)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), per_call)
    # duplicate and out-of-range hot ids are ignored and flagged
    bad = torch.cat([dev["hot_ids"], dev["hot_ids"][:3], torch.tensor([w.V, -1], dtype=torch.int32, device="cuda")])
    diag = torch.zeros(w.B * 32, dtype=torch.uint8, device="cuda")
    out = s.sample(dev["logits"], dev["params"], hot_ids=bad, seed=w.seed, step=2, V=w.V, diag=diag)
    torch.cuda.synchronize()
    dg = diag.cpu().numpy().view(binding.ROW_DIAG_DTYPE)
    assert np.array_equal(out.cpu().numpy(), per_call) and (dg["flags"] & binding.DIAG_BAD_HOT_SET).all()
    s.close()


# ---------------------------------------------------------------- boundary on the device ---------
def test_boundary_argument_errors_and_empty_batch():
    import torch
    binding = _binding()
    s = binding.Sampler(1024, 0)
    w = synth.make_config(1)
    dev = P.to_device(w)
    out = torch.full((4,), -5, dtype=torch.int32, device="cuda")
    args = dict(seed=1, step=0)

    def rc(**kw):
        a = dict(ctx=s.ctx, logits_ptr=dev["logits"].data_ptr(), B=4, V=1024, dtype=0, row_stride=1024,
                 params_ptr=dev["params"].data_ptr(), hist_ptr_ptr=0, hist_ids_ptr=0, hot_ids_ptr=0, H=0,
                 seed=1, step=0, row_offset=0, out_ids_ptr=out.data_ptr(), diag_ptr=0)
        a.update(kw)
        return binding.simple_sample(**a)

    assert rc() == binding.SIMPLE_OK
    assert rc(B=0) == binding.SIMPLE_OK
    assert rc(B=-1) == rc(V=0) == rc(dtype=7) == rc(row_stride=1000) == binding.SIMPLE_EINVAL
    assert rc(logits_ptr=0) == rc(params_ptr=0) == rc(out_ids_ptr=0) == binding.SIMPLE_EINVAL
    assert rc(H=5) == rc(H=-2) == rc(H=-1) == binding.SIMPLE_EINVAL
    assert rc(hot_ids_ptr=dev["params"].data_ptr(), H=2000) == binding.SIMPLE_EINVAL
    assert rc(hist_ptr_ptr=dev["hist_ptr"].data_ptr()) == binding.SIMPLE_EINVAL
    assert rc(V=2048, row_stride=2048) == binding.SIMPLE_ECAPACITY
    assert rc(hist_ptr_ptr=dev["hist_ptr"].data_ptr(), hist_ids_ptr=dev["hist_ids"].data_ptr()) == binding.SIMPLE_ECAPACITY
    torch.cuda.synchronize()
    out.fill_(-5)
    assert rc(V=0) == binding.SIMPLE_EINVAL
    torch.cuda.synchronize()
    assert (out.cpu().numpy() == -5).all()  # nothing is written on a host-side error
    assert binding.simple_lds_bytes(s.ctx) > 32 * 1024
    s.close()
    with pytest.raises(binding.SimpleError) as e:
        binding.Sampler(4_000_000, 60_000)  # one row's state would not fit the LDS of a compute unit
    assert e.value.code == binding.SIMPLE_ECAPACITY


def test_single_best_token_among_thousands_of_ties_in_the_general_kernel():
    """top_p <= 0 keeps one token, the lowest id at the maximum.  With top-k above the candidate list's
    reach the row takes the general kernel's multi-pass route, which must stop at the first of the
    columns that tie at the maximum (it used to admit them all and then find no id)."""
    rng = np.random.default_rng(41)
    B, V = 4, 50_008
    z = (rng.integers(-6, 3, (B, V)) * 0.75).astype(np.float32)   # nine distinct values, thousands of ties
    params = synth.make_params(B, temperature=[1.0, 4.0, 0.5, 1.0], top_k=[1025, 3000, V - 1, 1025],
                               top_p=[0.0, 0.0, -1.0, 0.0], min_p=[0.0, 0.01, 0.0, 0.0])
    for dtype in ("f32", "bf16"):
        logits = synth.f32_to_bf16_bits(z) if dtype == "bf16" else z
        w = synth.Workload("one-of-many", B, V, dtype, logits, params, np.zeros(B + 1, np.int64), np.zeros(0, np.int32))
        for ids, dg, _ in _check(w, steps=(0, 1)):
            assert np.array_equal(ids, np.argmax(z, axis=1)) and (dg["n_survivors"] == 1).all()


@pytest.mark.parametrize("V,dtype", [(1 << 18, "f32"), ((1 << 18) + 1000, "bf16"), (300_001, "f32"), ((1 << 18) + 8, "bf16")])
def test_vocabularies_of_two_to_the_eighteen_columns_and_more(V, dtype):
    """From 2^18 columns on the general kernel serves the whole batch (the single-pass kernel's fixed
    point is sized for fewer); whole-vocabulary nuclei, large top-k and min-p rows take its multi-pass
    route: aligned rows in 16-byte loads (a row length that is and is not a multiple of the stream's
    group of 1024 columns), the odd float32 length element by element."""
    rng = np.random.default_rng(V % 1000 + 11)
    B = 12
    z = synth.zipf_profile_logits(B, V, 1.1, 1.5, rng, "f32", rng.permutation(V))
    z[3, rng.choice(V, 5000, replace=False)] = z[3].max()          # a plateau at the maximum
    z[5] = np.round(z[5] * 2) / 2                                   # few distinct values: ties at every cut
    lens = np.array([0, 700, 3000, 50, 0, 1500, 200, 0, 4000, 10, 900, 0])
    head = np.argsort(-z, axis=1)[:, :3000]
    hist_ptr = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    hist_ids = np.concatenate([rng.choice(head[b], int(lens[b])) for b in range(B)]).astype(np.int32)
    params = synth.make_params(
        B, temperature=[1.0, 0.8, 1.2, 1.0, 0.0, 0.7, 1.0, 1.5, 0.9, 1.0, 0.6, 1.0],
        top_k=[0, 3000, 0, 0, 0, 20_000, V - 1, 0, 1500, 0, 50, 0],
        top_p=[0.9, 0.95, 0.999, 0.5, 1.0, 0.9, 0.8, 1.0, 1.0, 0.97, 0.9, 0.3],
        min_p=[0, 0, 1e-5, 0, 0, 0, 0, 1e-4, 0, 1e-3, 0, 0],
        rep_penalty=1.1, freq_penalty=0.2, pres_penalty=0.1)
    hot = np.sort(rng.choice(V, 40_000, replace=False)).astype(np.int32) if dtype == "bf16" else None
    logits = synth.f32_to_bf16_bits(z) if dtype == "bf16" else z
    w = synth.Workload(f"large-V-{V}", B, V, dtype, logits, params, hist_ptr, hist_ids, hot_ids=hot)
    res = _check(w, steps=(0, 1))
    flags = res[0][1]["flags"]
    assert not (flags & 128).any()       # no row came through the single-pass kernel's queue
    assert (flags & 4).sum() >= 6        # the whole-vocabulary and large-k rows: multi-pass route


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_multi_pass_route_cuts_inside_and_above_a_plateau(dtype):
    """Top-k cuts that fall inside a plateau of 12,000 equal logits (the first r ties by id survive),
    with a nucleus inside that prefix: the nucleus descent meets every tie of the plateau, also the
    ones the top-k cut left out, so the keys it sets aside for its last level overflow and that
    level reads the row instead; with the cut above the plateau the keys fit.  Rows 6 and 7 carry
    histories that move some of the ties."""
    rng = np.random.default_rng(5)
    B, V = 8, 40_000
    z = (rng.standard_normal((B, V)) * 0.5 - 6.0).astype(np.float32)
    for b in range(B):
        perm = rng.permutation(V)
        z[b, perm[:1500]] = rng.uniform(1.0, 6.0, 1500).astype(np.float32)   # the head
        z[b, perm[1500:13_500]] = 0.5                                          # the plateau
    lens = np.array([0, 0, 0, 0, 0, 0, 2500, 600])
    hist_ptr = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    order = np.argsort(-z, axis=1, kind="stable")
    hist_ids = np.concatenate([rng.choice(order[b, :9000], int(lens[b])) for b in range(B)]).astype(np.int32)
    params = synth.make_params(
        B, temperature=[1.0, 1.0, 0.7, 1.3, 1.0, 1.0, 1.0, 0.9],
        top_k=[3000, 3000, 9000, 13_499, 1400, 0, 3000, 5000],
        top_p=[0.99, 0.5, 0.999, 0.97, 0.9, 0.98, 0.95, 0.999],
        min_p=[0, 0, 0, 0, 0, 1e-3, 0, 0],
        rep_penalty=1.2, freq_penalty=0.1, pres_penalty=0.05)
    hot = np.sort(rng.choice(V, 6000, replace=False)).astype(np.int32) if dtype == "bf16" else None
    logits = synth.f32_to_bf16_bits(z) if dtype == "bf16" else z
    w = synth.Workload(f"plateau-cuts-{dtype}", B, V, dtype, logits, params, hist_ptr, hist_ids, hot_ids=hot)
    res = _check(w, steps=(0, 1, 2))
    assert (res[0][1]["flags"] & 4).sum() >= 5  # the multi-pass route of the general kernel


def test_aggregate_stats_equal_the_sum_over_the_row_records():
    """simple_set_stats: the device-side aggregate of two calls equals what the per-row diagnostics
    records of the same calls add up to (rows, greedy, SHVS accepted / rejected, second-pass and
    general-kernel rows, the fixed-point sum of alpha, the error bits), and nothing is added once it
    is removed."""
    import torch
    from paper_2512_00719_amd import binding
    w = synth.make_config(3, B=96, V=33_000, nnz=700).with_hot(2500)
    w.params["temperature"][5] = -1.0                 # a parameter error (general kernel)
    w.params["top_k"][7:11] = 0                       # nuclei over the whole vocabulary
    w.params["min_p"][7:11] = 0.0
    w.params["temperature"][7:11] = 1.3
    w.logits[12, 100] = np.nan                        # a data error
    dev = P.to_device(w)
    s = binding.Sampler(w.V, 700, max_B=w.B)
    stats = torch.zeros(64, dtype=torch.uint8, device="cuda:0")
    assert binding.simple_set_stats(s.ctx, stats.data_ptr() + 4) == binding.SIMPLE_EINVAL
    assert binding.simple_set_stats(s.ctx, stats.data_ptr()) == binding.SIMPLE_OK
    want = np.zeros(1, binding.STATS_DTYPE)[0]
    for step in (0, 1):
        diag = torch.zeros(w.B * 32, dtype=torch.uint8, device="cuda:0")
        s.sample(dev["logits"], dev["params"], dev["hist_ptr"], dev["hist_ids"], dev["hot_ids"], seed=w.seed, step=step, diag=diag, V=w.V)
        torch.cuda.synchronize()
        dg = diag.cpu().numpy().view(binding.ROW_DIAG_DTYPE)
        f = dg["flags"]
        ok_shvs = ((f & binding.DIAG_SHVS) > 0) & ((f & binding.DIAG_ERROR) == 0)
        want["rows"] += w.B
        want["greedy_rows"] += int(((f & binding.DIAG_GREEDY) > 0).sum())
        want["shvs_accepted"] += int((ok_shvs & ((f & binding.DIAG_ACCEPTED) > 0)).sum())
        want["shvs_rejected"] += int((ok_shvs & ((f & binding.DIAG_ACCEPTED) == 0)).sum())
        want["second_pass_rows"] += int(((f & binding.DIAG_WIDE) > 0).sum())
        want["general_rows"] += int(((f & binding.DIAG_GENERAL) > 0).sum())
        want["sum_alpha_q32"] += int(sum(int(np.rint(a * 2.0 ** 32)) for a in dg["alpha"][ok_shvs]))
        err_bits = binding.DIAG_ERROR | binding.DIAG_BAD_PARAM | binding.DIAG_BAD_LOGIT | binding.DIAG_BAD_HISTORY_ID | \
            binding.DIAG_HISTORY_TOO_LONG | binding.DIAG_BAD_HOT_SET
        want["error_flags"] |= int(np.bitwise_or.reduce(f) & err_bits)
    got = stats.cpu().numpy().view(binding.STATS_DTYPE)[0]
    for name in binding.STATS_DTYPE.names:
        assert got[name] == want[name], (name, got, want)
    assert got["shvs_accepted"] > 0 and got["shvs_rejected"] > 0 and got["second_pass_rows"] > 0 and got["general_rows"] > 0
    assert got["error_flags"] & binding.DIAG_BAD_PARAM and got["error_flags"] & binding.DIAG_BAD_LOGIT
    assert binding.simple_set_stats(s.ctx, 0) == binding.SIMPLE_OK
    s.sample(dev["logits"], dev["params"], dev["hist_ptr"], dev["hist_ids"], dev["hot_ids"], seed=w.seed, step=2, V=w.V)
    torch.cuda.synchronize()
    assert stats.cpu().numpy().view(binding.STATS_DTYPE)[0] == got
    s.close()


def test_decision_outputs_log_probability_and_eos_flag():
    """simple_set_decision_outputs: ln p~ of the returned id against the oracle (1e-5: the tolerance on
    p~ itself), 0 for greedy rows, -inf and no flag for an error row; the EOS flag marks exactly the
    rows whose id is one of the installed ids; rows of every route (list, whole-vocabulary kernels,
    general kernel)."""
    import torch
    from paper_2512_00719_amd import binding
    w = synth.make_config(3, B=64, V=33_000, nnz=300)
    w.params["top_k"][3:7] = 0
    w.params["min_p"][3:7] = 0.0
    w.params["temperature"][3:7] = 1.3
    w.params["rep_penalty"][9] = 0.7
    w.logits[11, 5] = np.nan
    ids, dg = P.run_gpu(w, 1)
    want = P.run_oracle(w, 1)
    eos = sorted({int(ids[0]), int(ids[20]), int(ids[33])})
    dev = P.to_device(w)
    s = binding.Sampler(w.V, 300, max_B=w.B)
    lp = torch.full((w.B,), 7.0, dtype=torch.float32, device="cuda:0")
    fl = torch.full((w.B,), 9, dtype=torch.uint8, device="cuda:0")
    assert binding.simple_set_decision_outputs(s.ctx, lp.data_ptr(), fl.data_ptr(), eos) == binding.SIMPLE_OK
    assert binding.simple_set_decision_outputs(s.ctx, 0, 0, list(range(9))) == binding.SIMPLE_EINVAL
    out = s.sample(dev["logits"], dev["params"], dev["hist_ptr"], dev["hist_ids"], seed=w.seed, step=1, V=w.V)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), ids)
    lp, fl = lp.cpu().numpy(), fl.cpu().numpy()
    routes = set()
    for b, o in enumerate(want):
        if o.id < 0:
            assert ids[b] == -1 and lp[b] == -np.inf and fl[b] == 0
            continue
        greedy = w.params["temperature"][b] == 0
        if int(ids[b]) == o.id:
            assert any(abs(lp[b] - np.log(p)) <= 1e-5 for p in ((1.0,) if greedy else (o.p_chosen, *o.alt_p))), (b, lp[b], o.p_chosen)
        assert lp[b] <= 0 and fl[b] == (1 if int(ids[b]) in eos else 0)
        routes.add(int(dg["flags"][b]) & (binding.DIAG_WIDE | binding.DIAG_GENERAL))
    assert fl.sum() >= 3 and len(routes) == 3 and (w.params["temperature"] == 0).any()
    assert binding.simple_set_decision_outputs(s.ctx, 0, 0, []) == binding.SIMPLE_OK
    s.close()


def test_tvd_instrument_shvs_against_the_baseline_sampler():
    """The paper's exactness experiment (section 7: cumulative mean TVD between the SHVS sampler's and
    the baseline sampler's token distributions, below 1 %), on one row replicated over the batch:
    the TVD between the two samplers stays at what sampling noise alone gives, for two hot-set
    sizes, and so does the TVD of either against the oracle's exact p~."""
    from paper_2512_00719_amd import tvd
    rng = np.random.default_rng(21)
    B, V, steps = 4096, 6000, 30
    perm = rng.permutation(V)
    row = np.empty(V, np.float32)
    row[perm] = (-1.2 * np.log(np.arange(1, V + 1)) + rng.standard_normal(V)).astype(np.float32)
    par = synth.make_params(B, temperature=1.0, top_p=0.95)
    d = O.row_distribution(row, par[0])
    p = d.probs()
    noise = tvd.expected_tvd_of_sampling(p, B * steps)
    for H in (64, 1024):
        hot = perm[:H].astype(np.int32)
        base = synth.Workload("tvd", B, V, "f32", np.tile(row, (B, 1)), par, np.zeros(B + 1, np.int64), np.zeros(0, np.int32))
        shvs = synth.Workload("tvd", B, V, "f32", base.logits, par, base.hist_ptr, base.hist_ids, hot_ids=hot, seed=base.seed + 1)
        acc = tvd.CumulativeTvd(V)
        for step in range(steps):
            acc.add(P.run_gpu(shvs, step)[0], P.run_gpu(base, step)[0])
        two_sample = np.sqrt(2.0) * noise   # both sides are empirical
        print(f"H={H}: final TVD {acc.history[-1]:.4f}, cumulative mean {acc.mean:.4f}, sampling noise alone {two_sample:.4f}", flush=True)
        assert acc.history[-1] < 1.25 * two_sample and acc.history[-1] < 0.05
        assert tvd.tvd(acc.a, p) < 1.25 * noise and tvd.tvd(acc.b, p) < 1.25 * noise
