"""GPU parity on the pattern-count route: bfloat16 rows without top-k and without penalties in
force are completed from counts per bit pattern (one LDS atomic per column), the cut and the class
masses from the counts, the drawn id from a second read.  Every case is compared with the CPU
oracle row by row, to the bar of test_gpu_parity.py, and the diagnostic flag of the route says which
rows took it.  Cases: nuclei of every width, min-p, no truncation, temperatures, with and without a
hot set, a ragged row end behind a padded stride, rows made of a handful of distinct values (the
cut falls inside a pattern with thousands of tied columns), masked (-inf) columns, rows the route must hand back (+inf, NaN, a value
outside its bins, a row maximum near zero), rows that must not take it
(top-k, penalties in force, float32)."""
import numpy as np
import pytest

import parity_util as P
from paper_2512_00719_amd import binding, synth

pytestmark = pytest.mark.gpu

PATTERN, WIDE, SHVS, GENERAL = binding.DIAG_PATTERN, binding.DIAG_WIDE, binding.DIAG_SHVS, binding.DIAG_GENERAL


def _bf16(z32):
    bits = synth.f32_to_bf16_bits(np.asarray(z32, np.float32))
    return bits, synth.bf16_bits_to_f32(bits)


def _run(w, steps=(0, 1), dev=None):
    out = []
    for step in steps:
        ids, dg = P.run_gpu(w, step, dev=dev)
        s = P.compare(ids, dg, P.run_oracle(w, step), range(w.B))
        out.append((ids, dg, s))
    return out


def _zipf_rows(rng, B, V, s=1.0, sigma=1.0):
    base = -s * np.log(np.arange(1, V + 1, dtype=np.float64))
    z = np.empty((B, V), np.float32)
    for b in range(B):
        z[b, rng.permutation(V)] = base + sigma * rng.standard_normal(V)
    return z + 12.0


@pytest.mark.parametrize("hot", [False, True])
def test_nuclei_min_p_and_no_truncation(hot):
    rng = np.random.default_rng(31 + hot)
    B, V = 24, 50_000 + 16
    bits, zf = _bf16(_zipf_rows(rng, B, V, s=1.1, sigma=1.2))
    top_p = np.array([0.3, 0.9, 0.95, 0.999, 1.0, 1.0, 0.5, 0.99] * 3, np.float32)
    min_p = np.array([0.0, 0.0, 0.0, 0.0, 0.0, 1e-4, 1e-3, 0.02] * 3, np.float32)
    temp = np.array([1.0] * 8 + [0.6] * 8 + [1.7] * 8, np.float32)
    params = synth.make_params(B, temperature=temp, top_p=top_p, min_p=min_p)
    hot_ids = np.sort(np.argsort(-zf.mean(axis=0))[:4000]).astype(np.int32) if hot else None
    w = synth.Workload("pattern", B, V, "bf16", bits, params, np.zeros(B + 1, np.int64), np.zeros(0, np.int32), hot_ids=hot_ids)
    for ids, dg, s in _run(w, steps=(0, 1, 2)):
        f = dg["flags"]
        assert ((f & PATTERN) > 0).all() and ((f & WIDE) > 0).all() and not (f & GENERAL).any(), [hex(int(x)) for x in f]
        assert (((f & SHVS) > 0) == hot).all()
        print("pattern route:", s, "accepted", int(((f & binding.DIAG_ACCEPTED) > 0).sum()), flush=True)


def test_few_distinct_values_cut_inside_a_pattern():
    """Logits on a grid of a few dozen values: every pattern holds thousands of tied columns, so the
    nucleus ends inside one and takes its first j columns in ascending id."""
    rng = np.random.default_rng(33)
    B, V = 16, 30_000 + 8
    z = np.round(rng.standard_normal((B, V)) * 2.0) * 0.5 + 3.0
    z[:, ::1000] += 0.25  # a few columns of their own value
    bits, zf = _bf16(z)
    params = synth.make_params(B, temperature=[1.0, 0.8, 1.3, 1.0] * 4, top_p=[0.5, 0.9, 0.97, 0.2] * 4,
                               min_p=[0.0, 0.0, 0.05, 0.0] * 4)
    hot_ids = np.sort(rng.choice(V, 6000, replace=False)).astype(np.int32)
    w = synth.Workload("pattern-ties", B, V, "bf16", bits, params, np.zeros(B + 1, np.int64), np.zeros(0, np.int32), hot_ids=hot_ids)
    for ids, dg, s in _run(w, steps=(0, 1, 2, 3)):
        assert ((dg["flags"] & PATTERN) > 0).all()
    w.hot_ids = None
    for ids, dg, s in _run(w, steps=(4, 5)):
        assert ((dg["flags"] & PATTERN) > 0).all()


def test_ragged_row_end_behind_a_padded_stride():
    import torch
    rng = np.random.default_rng(34)
    B, V, stride = 12, 33_003, 33_008  # V is no multiple of the vector width: the last columns are read one by one
    z = rng.standard_normal((B, V)) * 1.5
    z[:, V - 2] = 9.0  # a likely draw in the ragged end
    z[3, V - 1] = 11.0
    bits, zf = _bf16(z)
    params = synth.make_params(B, temperature=[1.0, 0.7, 1.2] * 4, top_p=[0.9, 1.0, 0.99, 0.6] * 3)
    hot_ids = np.sort(np.concatenate([rng.choice(V - 8, 3000, replace=False), [V - 2]])).astype(np.int32)
    w = synth.Workload("pattern-ragged", B, V, "bf16", bits, params, np.zeros(B + 1, np.int64), np.zeros(0, np.int32), hot_ids=hot_ids)
    padded = np.full((B, stride), 0x7F80, np.uint16)  # +inf in the padding: it must never be read as a logit
    padded[:, :V] = bits
    dev = P.to_device(w)
    dev["logits"] = torch.from_numpy(padded.view(np.int16)).cuda().view(torch.bfloat16)
    got_end = 0
    for ids, dg, s in _run(w, steps=tuple(range(6)), dev=dev):
        assert ((dg["flags"] & PATTERN) > 0).all()
        got_end += int((ids >= V - 3).sum())
    assert got_end > 0  # the draw did land behind the last whole group


def test_rows_handed_back_and_rows_that_never_take_the_route():
    rng = np.random.default_rng(35)
    B, V = 16, 20_000
    z = _zipf_rows(rng, B, V, s=1.0, sigma=1.0)
    z[0, 5:400] = -np.inf           # masked columns: taken, they have no mass
    z[0, 1000:1100] = -300.0        # ... as have values this far down
    z[1, 77] = 300.0                # a value outside the bins
    z[2] = rng.standard_normal(V) * 1e-6   # row maximum near zero
    z[3] = 0.0                      # all columns equal
    z[4, 9] = np.inf                # an error row
    z[5, 11] = np.nan
    z[6] = np.where(rng.random(V) < 0.002, 0.0, z[6])  # some exact zeros among ordinary values
    bits, zf = _bf16(z)
    params = synth.make_params(B, temperature=1.0, top_p=0.9)
    params["top_k"][8] = 50                 # top-k: the single-pass kernel's list
    params["rep_penalty"][9] = 1.2          # penalties in force (history below)
    params["temperature"][10] = 0.0         # greedy
    params["top_p"][11] = 0.0               # keeps one token
    params["top_p"][12] = 1.0               # no truncation at all
    params["min_p"][13] = 0.1
    lens = np.zeros(B, np.int64); lens[9] = 40; lens[14] = 25   # row 14: a history, but no penalty in force
    hist_ptr = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    hist_ids = rng.integers(0, V, int(hist_ptr[-1])).astype(np.int32)
    w = synth.Workload("pattern-edges", B, V, "bf16", bits, params, hist_ptr, hist_ids)
    for ids, dg, s in _run(w, steps=(0, 1)):
        f = dg["flags"]
        took = (f & PATTERN) > 0
        assert not took[[1, 2, 3, 4, 5, 8, 9, 10, 11]].any(), took
        assert took[[0, 6, 7, 12, 13, 14, 15]].all(), took
        assert ids[4] == -1 and ids[5] == -1 and (ids[[0, 1, 2, 3]] >= 0).all()
    # float32 calls never take it
    w32 = synth.Workload("pattern-f32", B, V, "f32", zf.copy(), params, hist_ptr, hist_ids)
    w32.logits[4, 9] = 1.0; w32.logits[5, 11] = 1.0
    ids, dg = P.run_gpu(w32, 0)
    assert not (dg["flags"] & PATTERN).any()


def test_decision_outputs_and_aggregate_on_the_route():
    """Log-probabilities, EOS flags and the aggregate of a call come out of this route as of the others."""
    import torch
    rng = np.random.default_rng(36)
    B, V = 64, 16_384
    bits, zf = _bf16(_zipf_rows(rng, B, V))
    params = synth.make_params(B, temperature=1.0, top_p=0.9)
    w = synth.Workload("pattern-out", B, V, "bf16", bits, params, np.zeros(B + 1, np.int64), np.zeros(0, np.int32))
    dev = P.to_device(w)
    ctx = binding.Sampler(V, 0, max_B=B)
    lp = torch.full((B,), 7.0, dtype=torch.float32, device="cuda:0")
    eos = torch.full((B,), 9, dtype=torch.uint8, device="cuda:0")
    stats = torch.zeros(binding.STATS_DTYPE.itemsize, dtype=torch.uint8, device="cuda:0")
    want = P.run_oracle(w, 0)
    eos_id = int(want[0].id)
    assert binding.simple_set_decision_outputs(ctx.ctx, lp.data_ptr(), eos.data_ptr(), [eos_id]) == 0
    assert binding.simple_set_stats(ctx.ctx, stats.data_ptr()) == 0
    diag = torch.zeros(B * 32, dtype=torch.uint8, device="cuda:0")
    out = ctx.sample(dev["logits"], dev["params"], None, None, None, seed=w.seed, step=0, diag=diag, V=V)
    torch.cuda.synchronize()
    ids = out.cpu().numpy()
    dg = diag.cpu().numpy().view(binding.ROW_DIAG_DTYPE)
    P.compare(ids, dg, want, range(B))
    assert ((dg["flags"] & PATTERN) > 0).all()
    assert np.allclose(lp.cpu().numpy(), np.log(dg["p_chosen"]), rtol=0, atol=1e-6)
    assert np.array_equal(eos.cpu().numpy() == 1, ids == eos_id)
    st = stats.cpu().numpy().view(binding.STATS_DTYPE)[0]
    assert int(st["rows"]) == B and int(st["second_pass_rows"]) == B and int(st["general_rows"]) == 0
    ctx.close()


def test_masked_columns_have_no_mass_but_count_where_nothing_is_truncated():
    """Rows in which a third of the columns is -inf (an allow-list, a padded vocabulary): the route
    takes them; without truncation |K_b| still counts every column, as the oracle does."""
    rng = np.random.default_rng(37)
    B, V = 8, 24_000 + 8
    z = _zipf_rows(rng, B, V, s=1.0, sigma=1.5)
    z[:, rng.random(V) < 0.33] = -np.inf
    z[:, V - 40:] = -np.inf                    # a padded end
    bits, zf = _bf16(z)
    bits[7, 123] = 0xFFC0                      # a NaN with the sign bit set: an error row
    params = synth.make_params(B, temperature=[1.0, 0.7, 1.4, 1.0] * 2, top_p=[0.9, 1.0, 1.0, 0.99] * 2,
                               min_p=[0.0, 0.0, 0.05, 1e-30] * 2)
    hot_ids = np.sort(rng.choice(V, 3000, replace=False)).astype(np.int32)
    w = synth.Workload("pattern-masked", B, V, "bf16", bits, params, np.zeros(B + 1, np.int64), np.zeros(0, np.int32), hot_ids=hot_ids)
    for ids, dg, s in _run(w, steps=(0, 1, 2)):
        took = (dg["flags"] & PATTERN) > 0
        assert took[:7].all() and not took[7], took
        assert ids[7] == -1 and (dg["flags"][7] & binding.DIAG_BAD_LOGIT)
        assert dg["n_survivors"][1] == V and dg["n_survivors"][5] == V


def test_more_rows_than_one_launch_and_a_row_offset():
    """4200 rows go out in two launches; the Philox counter of a row is its index plus row_offset."""
    rng = np.random.default_rng(38)
    B, V = 4200, 16_384 + 8
    bits, zf = _bf16(rng.standard_normal((B, V)).astype(np.float32) * 2.0 + 3.0)
    params = synth.make_params(B, temperature=1.0, top_p=0.9)
    params["top_p"][::3] = 1.0
    params["min_p"][1::5] = 0.01
    w = synth.Workload("pattern-many", B, V, "bf16", bits, params, np.zeros(B + 1, np.int64), np.zeros(0, np.int32))
    ids, dg = P.run_gpu(w, 2, row_offset=(1 << 32) - 100)
    rows = list(range(0, B, 7)) + list(range(4090, 4110))
    P.compare(ids, dg, P.run_oracle(w, 2, rows=rows, row_offset=(1 << 32) - 100), rows)
    assert ((dg["flags"] & PATTERN) > 0).all() and ids.min() >= 0


def test_state_and_static_entry_points_take_the_route():
    """A row whose sequence has tokens but no penalty in force is a row of the route, also through
    simple_sample_state; simple_sample_static returns the ids of simple_sample."""
    import torch
    rng = np.random.default_rng(39)
    B, V, L = 12, 20_000, 64
    bits, zf = _bf16(_zipf_rows(rng, B, V))
    params = synth.make_params(B, temperature=[1.0, 0.8, 1.3] * 4, top_p=[0.9, 0.95, 1.0, 0.7] * 3)
    w = synth.Workload("pattern-state", B, V, "bf16", bits, params, np.zeros(B + 1, np.int64), np.zeros(0, np.int32))
    dev = P.to_device(w)
    want = P.run_oracle(w, 5)
    ctx = binding.Sampler(V, L, max_B=B)
    st = binding.simple_state_create(0, B, V, L)
    stream = torch.cuda.current_stream().cuda_stream
    lens = rng.integers(1, 40, B)
    ptr = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    toks = rng.integers(0, V, int(ptr[-1])).astype(np.int32)
    p_d, t_d = torch.from_numpy(ptr).cuda(), torch.from_numpy(toks).cuda()
    assert binding.simple_state_restart(st, 0, B, p_d.data_ptr(), t_d.data_ptr(), 0, stream) == 0
    out = torch.full((B,), -9, dtype=torch.int32, device="cuda:0")
    diag = torch.zeros(B * 32, dtype=torch.uint8, device="cuda:0")
    lg = dev["logits"]
    rc = binding.simple_sample_state(ctx.ctx, st, 0, lg.data_ptr(), B, V, binding.SIMPLE_BF16, lg.stride(0), dev["params"].data_ptr(),
                                     0, 0, w.seed, 5, 0, out.data_ptr(), diag.data_ptr(), stream)
    assert rc == 0, binding.simple_strerror(rc)
    torch.cuda.synchronize()
    ids, dg = out.cpu().numpy(), diag.cpu().numpy().view(binding.ROW_DIAG_DTYPE)
    P.compare(ids, dg, want, range(B))
    assert ((dg["flags"] & PATTERN) > 0).all()
    out2 = torch.full((B,), -9, dtype=torch.int32, device="cuda:0")
    diag2 = torch.zeros(B * 32, dtype=torch.uint8, device="cuda:0")
    rc = binding.simple_sample_static(lg.data_ptr(), B, V, binding.SIMPLE_BF16, lg.stride(0), dev["params"].data_ptr(), 0, 0, 0, 0,
                                      w.seed, 5, 0, out2.data_ptr(), diag2.data_ptr(), stream)
    assert rc == 0, binding.simple_strerror(rc)
    torch.cuda.synchronize()
    assert np.array_equal(out2.cpu().numpy(), ids)
    assert ((diag2.cpu().numpy().view(binding.ROW_DIAG_DTYPE)["flags"] & PATTERN) > 0).all()
    binding.simple_state_destroy(st)
    ctx.close()


def test_seeded_random_rows():
    """Sixty seeded random cases: batch, vocabulary size (ragged ends behind padded strides), value
    distribution (normal, Zipf profile, coarse grids with thousands of ties, sparse spikes, tiny and
    large ranges), masked columns, out-of-range values, temperatures, top-p, min-p, a stray top-k
    row, hot sets of any size; every row against the oracle."""
    import torch
    tot = {"rows": 0, "ambiguous": 0, "soft": 0, "pattern": 0}
    for case in range(60):
        rng = np.random.default_rng(7000 + case)
        B = int(rng.integers(1, 16))
        V = int(rng.integers(2100, 12000)) * 8 + (int(rng.integers(1, 8)) if rng.random() < 0.3 else 0)
        stride = (V + 7) // 8 * 8 + 8 * int(rng.integers(0, 3))
        kind = int(rng.integers(0, 5))
        if kind == 0:
            z = rng.standard_normal((B, V)) * rng.uniform(0.5, 4.0)
        elif kind == 1:
            z = _zipf_rows(rng, B, V, s=rng.uniform(0.7, 1.5), sigma=rng.uniform(0.3, 2.0)) - 12.0 + rng.uniform(0, 25)
        elif kind == 2:
            z = np.round(rng.standard_normal((B, V)) * rng.uniform(1, 3)) * rng.choice([0.25, 0.5, 1.0]) + rng.uniform(-3, 8)
        elif kind == 3:
            z = rng.standard_normal((B, V)) * 2 + np.where(rng.random((B, V)) < 0.001, rng.uniform(5, 20), 0)
        else:
            z = rng.uniform(-1, 1, (B, V)) * rng.choice([1e-3, 0.1, 10, 100])
        if rng.random() < 0.3:
            z[:, rng.random(V) < rng.uniform(0.01, 0.9)] = -np.inf
        if rng.random() < 0.1:
            z[rng.integers(0, B), rng.integers(0, V)] = rng.choice([300.0, -300.0, 255.0])
        bits, _ = _bf16(z)
        params = synth.make_params(B, temperature=rng.uniform(0.3, 2.0, B).astype(np.float32),
                                   top_p=np.where(rng.random(B) < 0.25, 1.0, rng.uniform(0.05, 1.0, B)).astype(np.float32),
                                   min_p=np.where(rng.random(B) < 0.6, 0.0, 10 ** rng.uniform(-6, -0.5, B)).astype(np.float32))
        if rng.random() < 0.2:
            params["top_k"][rng.integers(0, B)] = int(rng.integers(1, 200))
        hot = np.sort(rng.choice(V, int(rng.integers(1, V // 2)), replace=False)).astype(np.int32) if rng.random() < 0.6 else None
        w = synth.Workload(f"random{case}", B, V, "bf16", bits, params, np.zeros(B + 1, np.int64), np.zeros(0, np.int32),
                           hot_ids=hot, seed=int(rng.integers(1, 1 << 40)))
        padded = np.full((B, stride), 0x7FC0, np.uint16)  # NaN in the padding: it must never be read as a logit
        padded[:, :V] = bits
        dev = P.to_device(w)
        dev["logits"] = torch.from_numpy(padded.view(np.int16)).cuda().view(torch.bfloat16)
        step = int(rng.integers(0, 1 << 20))
        ids, dg = P.run_gpu(w, step, dev=dev)
        s = P.compare(ids, dg, P.run_oracle(w, step), range(B), max_mismatch_frac=0.2)
        tot["rows"] += s["rows"]; tot["ambiguous"] += s["ambiguous"]; tot["soft"] += s["soft_mismatch"]
        tot["pattern"] += int(((dg["flags"] & PATTERN) > 0).sum())
    print("random rows:", tot, flush=True)
    assert tot["pattern"] > 0.8 * tot["rows"] and tot["soft"] <= 2


@pytest.mark.parametrize("ties", [False, True])
def test_top_k_beyond_what_the_candidate_list_certifies(ties):
    """top-k above 1024 (alone, with top-p scaled by the mass of the top-k prefix, with min-p): exactly
    k columns survive, the last of them the first few of their pattern in ascending id."""
    rng = np.random.default_rng(41 + ties)
    B, V = 12, 40_000
    if ties:
        z = np.round(rng.standard_normal((B, V)) * 2.5) * 0.5 + 2.25  # (no exact zeros: thousands of them would send the row back)
    else:
        z = _zipf_rows(rng, B, V, s=0.9, sigma=1.5)
    bits, zf = _bf16(z)
    params = synth.make_params(B, temperature=[1.0, 0.8, 1.5] * 4, top_k=[1025, 3000, 20000, 39999] * 3,
                               top_p=[1.0, 0.9, 0.99, 1.0, 0.5, 1.0] * 2, min_p=[0.0, 0.0, 1e-3, 0.0] * 3)
    hot_ids = np.sort(rng.choice(V, 5000, replace=False)).astype(np.int32)
    w = synth.Workload("pattern-topk", B, V, "bf16", bits, params, np.zeros(B + 1, np.int64), np.zeros(0, np.int32), hot_ids=hot_ids)
    for ids, dg, s in _run(w, steps=(0, 1, 2)):
        assert ((dg["flags"] & PATTERN) > 0).all() and not (dg["flags"] & GENERAL).any()
    assert (dg["n_survivors"][[0, 3]] == [1025, 39999]).all()  # top-k alone keeps exactly k
