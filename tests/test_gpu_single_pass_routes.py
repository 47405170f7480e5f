"""GPU parity on the routes of the single-pass kernel and of the kernels behind it.

Each case is built so that a known route must be taken (checked through the diagnostic flags) and
the ids are compared with the CPU oracle row by row, to the bar of test_gpu_parity.py.  Routes:
the sorted small-list epilogue, the long-list epilogue (top-k near the list's limit), the
whole-vocabulary nucleus (sliced bins / classify / finish kernels; with history, SHVS, bf16, a
ragged row end, more rows than workspace slots), and the rows the single-pass kernel must leave to
the general kernel."""
import numpy as np
import pytest

import parity_util as P
from paper_2512_00719_amd import synth

pytestmark = pytest.mark.gpu

WIDE, SHVS, GENERAL = 4, 8, 128  # diagnostic flag bits of the C boundary
WIDE_SLOTS = 4096  # rows of one launch (the whole-vocabulary-nucleus kernels have a workspace slot for each)


def _head_history(z, lens, rng, head=300):
    """History ids drawn (with repeats) from the head of each row's distribution."""
    B = z.shape[0]
    top = np.argsort(-z, axis=1)[:, :head]
    hist_ptr = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    ids = [rng.choice(top[b], int(lens[b])) for b in range(B)]
    return hist_ptr, (np.concatenate(ids) if ids else np.zeros(0)).astype(np.int32)


def _run(w, steps=(0, 1), sampler=None, dev=None):
    out = []
    for step in steps:
        ids, dg = P.run_gpu(w, step, sampler=sampler, dev=dev)
        P.compare(ids, dg, P.run_oracle(w, step), range(w.B))
        out.append((ids, dg))
    return out


def _flat_logits(rng, B, V, sigma=1.2):
    """Rows without a dominant head: a nucleus of 0.9 and more spans thousands of columns."""
    return (rng.standard_normal((B, V)) * sigma).astype(np.float32)


def test_whole_vocabulary_nucleus_with_history_f32_ragged_row_end():
    import torch
    rng = np.random.default_rng(21)
    B, V, stride = 10, 33_001, 33_004  # V is no multiple of the vector width: the last group is partial
    z = _flat_logits(rng, B, V)
    lens = rng.integers(200, 1500, B)
    hist_ptr, hist_ids = _head_history(z, lens, rng, head=2000)
    params = synth.make_params(B, temperature=[1.0, 0.9, 1.1, 1.3, 0.8] * 2, top_p=[0.9, 0.95, 0.8, 0.99, 0.97] * 2,
                               rep_penalty=[1.2, 1.05] * 5, freq_penalty=[0.3, 0.0] * 5, pres_penalty=[0.0, 0.2] * 5,
                               n_prompt=[0, 100, 5000, 7, 300] * 2)
    w = synth.Workload("wide-hist", B, V, "f32", z, params, hist_ptr, hist_ids)
    padded = np.full((B, stride), 1e30, np.float32)  # padding must never be read as a logit
    padded[:, :V] = z
    dev = P.to_device(w)
    dev["logits"] = torch.from_numpy(padded).cuda()
    for ids, dg in _run(w, steps=(0, 1, 2), dev=dev):
        f = dg["flags"]
        assert ((f & WIDE) > 0).sum() >= 8
        assert not ((f & WIDE) > 0)[(f & GENERAL) > 0].any()  # these rows were finished by the sliced kernels


def test_whole_vocabulary_nucleus_bf16_shvs_history():
    rng = np.random.default_rng(22)
    B, V = 8, 40_000 + 8
    z32 = _flat_logits(rng, B, V, sigma=1.5)
    bits = synth.f32_to_bf16_bits(z32)  # many exact ties after rounding
    zf = synth.bf16_bits_to_f32(bits)
    lens = rng.integers(0, 1200, B)
    hist_ptr, hist_ids = _head_history(zf, lens, rng, head=1000)
    params = synth.make_params(B, temperature=[1.0, 0.7, 1.2, 1.0] * 2, top_p=[0.9, 0.97, 0.85, 0.999] * 2,
                               rep_penalty=1.15, freq_penalty=0.1, pres_penalty=0.1, n_prompt=50)
    hot = np.argsort(-zf.mean(axis=0))[:3000].astype(np.int32)
    w = synth.Workload("wide-bf16-shvs", B, V, "bf16", bits, params, hist_ptr, hist_ids, hot_ids=np.sort(hot))
    for ids, dg in _run(w, steps=(0, 1, 2, 3)):
        f = dg["flags"]
        assert ((f & WIDE) > 0).sum() >= 6 and ((f & SHVS) > 0).all()
        assert not ((f & WIDE) > 0)[(f & GENERAL) > 0].any()


def test_more_whole_vocabulary_rows_than_one_launch_takes():
    """A launch takes as many rows as there are workspace slots, so a larger batch of rows that all need
    the sliced kernels goes out in two launches and none of them falls to the general kernel."""
    from paper_2512_00719_amd import binding
    rng = np.random.default_rng(23)
    B, V = WIDE_SLOTS + 52, 8192 + 64
    z = _flat_logits(rng, B, V)
    params = synth.make_params(B, temperature=1.0, top_p=0.9)
    w = synth.Workload("wide-many", B, V, "f32", z, params, np.zeros(B + 1, np.int64), np.zeros(0, np.int32))
    s = binding.Sampler(V, 0)
    dev = P.to_device(w)
    rows = sorted(set(rng.choice(B, 48, replace=False).tolist()) | {0, 1, WIDE_SLOTS - 1, WIDE_SLOTS, B - 1})
    ids, dg = P.run_gpu(w, 3, sampler=s, dev=dev)
    P.compare(ids, dg, P.run_oracle(w, 3, rows=rows), rows)
    f = dg["flags"]
    assert ((f & WIDE) > 0).all() and not ((f & GENERAL) > 0).any()
    assert ids.min() >= 0 and ids.max() < V
    ids2, _ = P.run_gpu(w, 3, sampler=s, dev=dev)
    assert np.array_equal(ids, ids2)
    s.close()


def test_long_list_epilogue_top_k_near_the_limit():
    rng = np.random.default_rng(24)
    B, V = 12, 60_000
    z = _flat_logits(rng, B, V, sigma=2.0)
    lens = rng.integers(0, 800, B)
    hist_ptr, hist_ids = _head_history(z, lens, rng, head=1500)
    params = synth.make_params(B, temperature=[0.8, 1.0, 1.2] * 4, top_k=[1000, 1024, 700, 600, 900, 513] * 2,
                               top_p=[1.0, 0.95, 0.9, 1.0, 0.99, 0.8] * 2, min_p=[0, 0, 0, 1e-4, 0, 0] * 2,
                               rep_penalty=1.1, freq_penalty=0.2, pres_penalty=0.1)
    w = synth.Workload("long-list", B, V, "f32", z, params, hist_ptr, hist_ids)
    for ids, dg in _run(w, steps=(0, 1, 2)):
        assert ((dg["flags"] & GENERAL) > 0).sum() <= 2  # the sampled threshold may miss now and then
        assert dg["n_survivors"].max() > 512


def test_rows_the_single_pass_kernel_must_leave_to_the_general_kernel():
    rng = np.random.default_rng(25)
    B, V = 8, 20_000
    z = _flat_logits(rng, B, V, sigma=2.0)
    # row 0: more ids than the 512 threads this small batch gets per row hold in registers (16 each)
    lens = np.array([9000, 5000, 300, 300, 300, 0, 300, 300])
    hist_ptr, hist_ids = _head_history(z, lens, rng, head=3000)
    params = synth.make_params(
        B, temperature=[1.0, 1.0, 1.0, 1.0, 0.9, 1.0, 1.0, 0.0],
        top_k=[0, 50, 0, 40, 1500, 0, 0, 0],
        top_p=[0.9, 0.9, 1.0, 0.9, 1.0, 1.0, 0.9, 1.0],
        rep_penalty=[1.1, 1.1, 1.1, 0.9, 1.1, 1.0, 1.1, 1.2],       # row 3 raises logits
        freq_penalty=[0.1, 0.1, 0.0, 0.0, 0.0, 0.0, -0.2, 0.0])     # row 6 too
    w = synth.Workload("leave", B, V, "f32", z, params, hist_ptr, hist_ids)
    for ids, dg in _run(w, steps=(0, 1)):
        general = (dg["flags"] & GENERAL) > 0
        wide = (dg["flags"] & WIDE) > 0
        # 3: top-k with penalties that raise logits
        assert general[3]
        # 0: a long history is corrected by claims, not left; 2, 5: no truncation at all, 4: top-k alone
        # above the list's limit and 6: no top-k with penalties that raise logits: straight to the
        # whole-vocabulary kernels
        assert not general[[0, 1, 2, 5, 7]].any() and wide[[2, 5]].all()
        assert (wide[[4, 6]] | general[[4, 6]]).all()


def test_nucleus_rows_with_more_history_ids_than_registers_hold():
    """top-p without top-k keeps the mass below the threshold exact by correcting every distinct
    history column once; with more ids than 16 per thread the columns are claimed by rank."""
    rng = np.random.default_rng(35)
    B, V = 600, 20_480  # more rows than two per compute unit: 256 threads per row, 4096 ids in registers
    z = _flat_logits(rng, B, V, sigma=3.5)
    lens = rng.integers(0, 3000, B)
    lens[:24] = rng.integers(4097, 12_000, 24)
    hist_ptr, hist_ids = _head_history(z, lens, rng, head=6000)
    params = synth.make_params(B, temperature=[0.9, 1.0, 1.1] * 200, top_p=[0.9, 0.8, 0.95, 0.7] * 150,
                               rep_penalty=1.2, freq_penalty=0.15, pres_penalty=0.1, n_prompt=[0, 2000, 50] * 200)
    w = synth.Workload("long-hist", B, V, "f32", z, params, hist_ptr, hist_ids)
    rows = sorted(set(range(24)) | set(rng.choice(B, 24, replace=False).tolist()))
    for step in (0, 1):
        ids, dg = P.run_gpu(w, step)
        P.compare(ids, dg, P.run_oracle(w, step, rows=rows), rows)
        f = dg["flags"]
        # most of them are settled by the list (a history that covers the whole head of the row can
        # still push the cut above the threshold, which the general kernel resolves)
        assert ((f & GENERAL) > 0)[:24].sum() <= 4
        assert (((f & WIDE) == 0) & ((f & GENERAL) == 0))[:24].sum() >= 12


def test_one_context_alternating_routes_call_after_call():
    """The queues of a context alternate between launches: results must not depend on what the call before queued."""
    from paper_2512_00719_amd import binding
    rng = np.random.default_rng(26)
    B, V = 16, 24_000
    z = _flat_logits(rng, B, V)
    empty = (np.zeros(B + 1, np.int64), np.zeros(0, np.int32))
    wide = synth.Workload("a", B, V, "f32", z, synth.make_params(B, temperature=1.0, top_p=0.9), *empty)
    topk = synth.Workload("b", B, V, "f32", z, synth.make_params(B, temperature=0.8, top_k=20, top_p=0.9), *empty)
    plain = synth.Workload("c", B, V, "f32", z, synth.make_params(B, temperature=1.0, top_k=2000, top_p=0.95), *empty)  # general kernel
    s = binding.Sampler(V, 0)
    want = {}
    for step, w in enumerate([wide, topk, plain, wide, wide, plain, topk, topk, wide, plain, plain, wide]):
        ids, dg = P.run_gpu(w, step % 3, sampler=s)
        key = (w.name, step % 3)
        if key not in want:
            P.compare(ids, dg, P.run_oracle(w, step % 3), range(B))
            want[key] = ids.copy()
        assert np.array_equal(ids, want[key]), (step, w.name)
        f = dg["flags"]
        if w is wide:
            assert ((f & WIDE) > 0).all() and not ((f & GENERAL) > 0).any()
        if w is plain:
            assert ((f & GENERAL) > 0).all()
        if w is topk:
            assert not ((f & (WIDE | GENERAL)) > 0).any()
    s.close()


def test_no_truncation_rows_every_column_survives():
    """temperature only: the rows skip the candidate list and go straight to the sliced kernels,
    with any penalties (also ones that raise logits), history longer than the register budget, SHVS."""
    rng = np.random.default_rng(27)
    B, V = 12, 36_000 + 4
    z = _flat_logits(rng, B, V, sigma=1.8)
    z[3, 17] = -np.inf  # a masked token: probability zero, never drawn
    lens = rng.integers(0, 1400, B)
    lens[5] = 5000
    hist_ptr, hist_ids = _head_history(z, lens, rng, head=2500)
    params = synth.make_params(B, temperature=[1.0, 0.6, 1.4] * 4,
                               rep_penalty=[1.0, 1.2, 0.85, 1.1] * 3, freq_penalty=[0.0, 0.3, -0.2] * 4,
                               pres_penalty=[0.0, 0.1, 0.0, -0.1] * 3, n_prompt=[0, 40, 10_000] * 4)
    hot = np.sort(np.argsort(-z.mean(axis=0))[:2000]).astype(np.int32)
    for hot_ids in (None, hot):
        w = synth.Workload("all", B, V, "f32", z, params, hist_ptr, hist_ids, hot_ids=hot_ids)
        for ids, dg in _run(w, steps=(0, 1, 2)):
            f = dg["flags"]
            assert ((f & WIDE) > 0).all() and not ((f & GENERAL) > 0).any()
            assert (dg["n_survivors"] == V).all() and ids[3] != 17


def test_no_truncation_bf16_ties():
    rng = np.random.default_rng(28)
    B, V = 6, 48_000 + 16
    bits = synth.f32_to_bf16_bits(_flat_logits(rng, B, V, sigma=1.0))
    w = synth.Workload("all-bf16", B, V, "bf16", bits, synth.make_params(B, temperature=[1.0, 0.8, 1.3] * 2),
                       np.zeros(B + 1, np.int64), np.zeros(0, np.int32))
    for ids, dg in _run(w, steps=(0, 1, 2, 3)):
        assert ((dg["flags"] & WIDE) > 0).all() and not ((dg["flags"] & GENERAL) > 0).any()


def test_min_p_cut_below_the_reach_of_the_list():
    """min-p alone with thousands of survivors: the cut is a value, found from the row maximum."""
    rng = np.random.default_rng(29)
    B, V = 10, 40_000
    z = _flat_logits(rng, B, V, sigma=1.5)
    lens = rng.integers(0, 900, B)
    hist_ptr, hist_ids = _head_history(z, lens, rng, head=800)  # the history holds the largest logits: the maximum moves
    params = synth.make_params(B, temperature=[1.0, 1.3, 0.8, 1.1, 1.0] * 2, min_p=[1e-3, 1e-4, 3e-3, 1e-5, 0.05] * 2,
                               rep_penalty=1.2, freq_penalty=0.4, pres_penalty=0.2)
    w = synth.Workload("minp", B, V, "f32", z, params, hist_ptr, hist_ids)
    for ids, dg in _run(w, steps=(0, 1, 2)):
        f = dg["flags"]
        assert ((f & WIDE) > 0).sum() >= 6 and not ((f & GENERAL) > 0).any()
        assert dg["n_survivors"].max() > 3072


def test_nucleus_rows_whose_candidates_overflow_the_list():
    """bf16 ties at the threshold put more columns at or above g than the list holds; rows with a nucleus
    over all of V still finish in the sliced kernels."""
    rng = np.random.default_rng(30)
    B, V = 8, 64_000
    z = np.round(_flat_logits(rng, B, V, sigma=1.0) * 4) / 4  # 0.25-spaced values: tie groups of thousands
    bits = synth.f32_to_bf16_bits(z.astype(np.float32))
    params = synth.make_params(B, temperature=[1.0, 0.9] * 4, top_p=[0.9, 0.95, 0.5, 0.99] * 2)
    w = synth.Workload("overflow", B, V, "bf16", bits, params, np.zeros(B + 1, np.int64), np.zeros(0, np.int32))
    for ids, dg in _run(w, steps=(0, 1)):
        f = dg["flags"]
        assert ((f & WIDE) > 0).all()
        # tie groups wider than the boundary table may still need the general kernel
        assert ((f & GENERAL) > 0).sum() <= B


def test_rows_the_sliced_kernels_hand_on():
    """Cases the sliced kernels detect and leave to the general kernel: a cut inside a plateau of
    equal values wider than the boundary table (spread out, and packed into one slice), a mass the
    fixed point cannot carry on a row without truncation, and data errors on such rows."""
    rng = np.random.default_rng(31)
    B, V = 8, 50_000
    z = (rng.standard_normal((B, V)) * 0.5 - 12.0).astype(np.float32)
    head = rng.choice(V, 300, replace=False)
    z[:, head] = (rng.standard_normal((B, 300)) * 0.3 + 1.0).astype(np.float32)   # about half of the mass
    spread = rng.choice(np.setdiff1d(np.arange(V), head), 9000, replace=False)
    z[0, spread] = -2.5    # 9000 equal columns carrying the other half: the 0.8 cut falls among them
    z[1, spread] = -2.5
    packed = np.setdiff1d(np.arange(3000, 9000), head)
    z[2, packed] = -2.0    # the same, packed into two slices
    z[3] = (rng.standard_normal(V) * 1.0).astype(np.float32)
    z[3, 777] = 120.0      # no truncation and one dominant logit: exp overflows the fixed point
    z[4] = z[3]
    z[4, 778] = np.nan     # data errors on rows without truncation
    z[5] = z[3]
    z[5, 779] = np.inf
    z[6] = -np.inf         # nothing to draw from
    params = synth.make_params(B, temperature=[1.0, 0.9, 1.0, 1.0, 1.0, 1.0, 1.0, 0.8],
                               top_p=[0.8, 0.8, 0.8, 1.0, 1.0, 1.0, 1.0, 0.9])
    w = synth.Workload("hand-on", B, V, "f32", z, params, np.zeros(B + 1, np.int64), np.zeros(0, np.int32))
    for step in (0, 1, 2):
        ids, dg = P.run_gpu(w, step)
        P.compare(ids, dg, P.run_oracle(w, step), range(B))
        f = dg["flags"]
        assert ((f & GENERAL) > 0)[[0, 1, 2, 3, 4, 5, 6]].all(), f
        assert ids[3] == 777 and list(ids[[4, 5, 6]]) == [-1, -1, -1] and (f[[4, 5, 6]] & 1).all()
        assert not (f[7] & GENERAL)


def test_top_p_and_min_p_together_beyond_the_list():
    """Both cuts on a flat row: the shorter prefix wins, whichever it is (min-p above the nucleus'
    boundary bin, inside it, or below it), with history, bf16 ties and SHVS."""
    rng = np.random.default_rng(32)
    B, V = 12, 44_000
    z = _flat_logits(rng, B, V, sigma=1.3)
    lens = rng.integers(0, 1000, B)
    hist_ptr, hist_ids = _head_history(z, lens, rng, head=900)
    params = synth.make_params(B, temperature=[1.0, 1.2, 0.9] * 4,
                               top_p=[0.9, 0.9, 0.9, 0.97, 0.97, 0.97, 0.6, 0.6, 0.6, 0.999, 0.999, 0.999],
                               min_p=[1e-2, 1e-3, 1e-4, 3e-3, 3e-4, 1e-5, 2e-2, 2e-3, 1e-6, 1e-3, 1e-4, 1e-5],
                               rep_penalty=1.15, freq_penalty=0.2, pres_penalty=0.1)
    w = synth.Workload("p+minp", B, V, "f32", z, params, hist_ptr, hist_ids)
    n_seen = set()
    for ids, dg in _run(w, steps=(0, 1, 2)):
        f = dg["flags"]
        assert ((f & WIDE) > 0).sum() >= 8 and not ((f & GENERAL) > 0).any()
        n_seen.update(int(x) for x in dg["n_survivors"])
    assert len(n_seen) >= 8  # the cuts differ from row to row
    bits = synth.f32_to_bf16_bits(z)
    hot = np.sort(np.argsort(-z.mean(axis=0))[:1500]).astype(np.int32)
    wb = synth.Workload("p+minp-bf16", B, V, "bf16", bits, params, hist_ptr, hist_ids, hot_ids=hot)
    for ids, dg in _run(wb, steps=(0, 1)):
        assert not ((dg["flags"] & GENERAL) > 0).any()


def test_plateau_at_the_cut_staged_over_several_slices_of_one_workgroup():
    """A cut inside a plateau of 3000 equal values below the list's threshold, with enough rows that a
    workgroup of the classifying pass meets several slices of one row in a row: its stage of boundary
    columns is written out in the middle of a row, and the tie is resolved by token id."""
    from paper_2512_00719_amd import binding
    rng = np.random.default_rng(33)
    B, V = 640, 5 * 4096
    z = (rng.standard_normal((B, V)) * 0.5 - 12.0).astype(np.float32)
    cols = rng.permutation(V)
    head, plateau = cols[:2000], cols[2000:5000]
    z[:, head] = (rng.standard_normal((B, 2000)) * 0.3 + 1.0).astype(np.float32)  # about three quarters of the mass
    z[:, plateau] = -0.5                                                        # the rest: the 0.8 cut falls here
    params = synth.make_params(B, temperature=1.0, top_p=0.8)
    w = synth.Workload("plateau-staged", B, V, "f32", z, params, np.zeros(B + 1, np.int64), np.zeros(0, np.int32))
    s = binding.Sampler(V, 0)
    dev = P.to_device(w)
    rows = sorted(set(rng.choice(B, 40, replace=False).tolist()) | {0, B - 1})
    for step in (0, 1):
        ids, dg = P.run_gpu(w, step, sampler=s, dev=dev)
        P.compare(ids, dg, P.run_oracle(w, step, rows=rows), rows)
        f = dg["flags"]
        assert ((f & WIDE) > 0).all() and not ((f & GENERAL) > 0).any()
        assert (dg["n_survivors"] > 2000).all() and (dg["n_survivors"] < 5000).all()
    s.close()


def test_history_denser_than_the_per_slice_stage():
    """More than 512 distinct history columns inside one slice of 4096: the ones beyond the stage that
    spreads them over all threads stay with their mask word's thread."""
    rng = np.random.default_rng(34)
    B, V = 6, 3 * 4096 + 40
    z = _flat_logits(rng, B, V)
    lens = np.array([3000, 2500, 0, 4000, 600, 3500])
    pool = rng.choice(4096, 2200, replace=False) + 4096  # all inside the second slice
    hist_ptr = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    hist_ids = np.concatenate([rng.choice(pool, int(n)) for n in lens]).astype(np.int32)
    params = synth.make_params(B, temperature=[1.0, 0.8, 1.2] * 2, top_p=[0.9, 1.0, 0.95, 0.97, 1.0, 0.9],
                               rep_penalty=1.15, freq_penalty=0.25, pres_penalty=0.1, n_prompt=[0, 500, 0, 100, 0, 3500])
    w = synth.Workload("dense-hist", B, V, "f32", z, params, hist_ptr, hist_ids)
    for ids, dg in _run(w, steps=(0, 1, 2)):
        f = dg["flags"]
        assert ((f & WIDE) > 0).all() and not ((f & GENERAL) > 0).any()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_top_k_alone_beyond_the_list(dtype):
    """top-k above 1024 without top-p or min-p: the sliced kernels find the k-th column by count (bins
    that count their columns, then a radix descent by count inside the cut's bin; bf16 ties in
    hundreds), with any penalties and history."""
    rng = np.random.default_rng(36)
    B, V = 12, 50_000 + 8
    z = _flat_logits(rng, B, V, sigma=2.0)
    lens = rng.integers(0, 2500, B)
    hist_ptr, hist_ids = _head_history(z, lens, rng, head=4000)
    ks = [1025, 1500, 2000, 3000, 5000, 8000, 1025, 2048, 4097, 12_000, 30_000, V - 1]
    params = synth.make_params(B, temperature=[1.0, 0.7, 1.3] * 4, top_k=ks,
                               rep_penalty=[1.0, 1.2, 0.9, 1.1] * 3, freq_penalty=[0.0, 0.2, -0.1] * 4,
                               pres_penalty=[0.0, 0.1] * 6, n_prompt=[0, 300, 10_000] * 4)
    logits = synth.f32_to_bf16_bits(z) if dtype == "bf16" else z
    w = synth.Workload("big-k", B, V, dtype, logits, params, hist_ptr, hist_ids)
    for ids, dg in _run(w, steps=(0, 1, 2)):
        f = dg["flags"]
        wide, general = (f & WIDE) > 0, (f & GENERAL) > 0
        assert (wide | general).all()
        assert wide[:9].all() and not general[:9].any()  # k up to 5000: always within the bins' reach
        assert np.array_equal(dg["n_survivors"][wide], np.array(ks)[wide])


def test_whole_vocabulary_routes_at_extreme_temperatures_and_thresholds_near_zero():
    """The classifying pass turns the cut into thresholds on the logit by a search over floats that
    starts from a closed-form guess; small and large temperatures and a threshold near zero (where the
    guess loses its digits) must give the same ids as the oracle."""
    rng = np.random.default_rng(37)
    V = 40_000 + 24
    taus = [0.05, 0.2, 1.0, 5.0, 30.0, 0.05, 0.2, 1.0, 5.0, 30.0]
    B = len(taus)
    z = np.empty((B, V), np.float32)
    for b, tau in enumerate(taus):
        sigma = 1.3 * min(tau, 3.0)            # tempered spread about 1.3 (less for the largest tau): wide nuclei
        shift = -2.9 * sigma if b >= 5 else 4.0 * sigma  # second half: the list's threshold lands near zero
        z[b] = (rng.standard_normal(V) * sigma + shift).astype(np.float32)
    lens = rng.integers(100, 900, B)
    hist_ptr, hist_ids = _head_history(z, lens, rng, head=1500)
    params = synth.make_params(B, temperature=taus, top_p=[0.9, 0.95, 0.8, 0.9, 0.99] * 2,
                               min_p=[0, 0, 1e-4, 0, 0, 1e-5, 0, 0, 0, 1e-6],
                               rep_penalty=1.1, freq_penalty=0.1)
    w = synth.Workload("taus", B, V, "f32", z, params, hist_ptr, hist_ids)
    for ids, dg in _run(w, steps=(0, 1, 2)):
        f = dg["flags"]
        assert ((f & WIDE) > 0).sum() >= 7 and not ((f & GENERAL) > 0).any()
    # min-p alone (the cut is a tempered value) at the same temperatures
    params2 = synth.make_params(B, temperature=taus, min_p=[1e-3, 1e-4, 1e-5, 1e-3, 1e-4] * 2, rep_penalty=1.1)
    w2 = synth.Workload("taus-minp", B, V, "f32", z, params2, hist_ptr, hist_ids)
    for ids, dg in _run(w2, steps=(0, 1)):
        assert not ((dg["flags"] & GENERAL) > 0).any()


def test_top_k_alone_beyond_the_list_with_a_hot_set():
    rng = np.random.default_rng(38)
    B, V = 8, 30_000
    z = _flat_logits(rng, B, V, sigma=1.5)
    hot = np.sort(rng.choice(V, 3000, replace=False)).astype(np.int32)
    params = synth.make_params(B, temperature=[1.0, 0.8] * 4, top_k=[1500, 2500, 4000, 1025, 6000, 2000, 1200, 9000])
    w = synth.Workload("big-k-hot", B, V, "f32", z, params, np.zeros(B + 1, np.int64), np.zeros(0, np.int32), hot_ids=hot)
    for ids, dg in _run(w, steps=(0, 1, 2, 3)):
        f = dg["flags"]
        assert ((f & WIDE) > 0).all() and ((f & SHVS) > 0).all() and not ((f & GENERAL) > 0).any()
        assert np.array_equal(dg["n_survivors"], params["top_k"])
