"""The incremental penalty state (paper section 5.2) on the GPU: over consecutive decode steps, where
every step's sampled id is appended to its sequence, the ids of `simple_sample_state` equal those of
the stateless call that is handed the same token lists as CSR history, and both equal the CPU oracle
(its own incremental state and its rebuild from the token list).  Covers prompts of different
lengths (none included), restarts of single slots in mid-run, a slot permutation, a sequence that
outgrows its slot, rows of every route (candidate list, nucleus over the whole vocabulary, general
kernel) and a hot set."""
import numpy as np
import pytest

import parity_util as P
from oracle import simple_oracle as O
from paper_2512_00719_amd import binding, synth

pytestmark = pytest.mark.gpu


def _dev(x):
    import torch
    return torch.from_numpy(np.ascontiguousarray(x)).to("cuda:0")


def _csr(prompts, gen):
    rows = [np.concatenate([p, np.array(g, dtype=np.int32)]).astype(np.int32) for p, g in zip(prompts, gen)]
    ptr = np.concatenate([[0], np.cumsum([r.size for r in rows])]).astype(np.int64)
    ids = np.concatenate(rows).astype(np.int32) if ptr[-1] else np.zeros(1, np.int32)
    return ptr, ids


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_stateful_steps_match_the_stateless_call_and_the_oracle(dtype):
    import torch
    B, V, L_max, steps = 40, 33_000, 160, 72
    rng = np.random.default_rng(5 if dtype == "f32" else 6)
    base = synth.make_config(3 if dtype == "f32" else 5, B=B, V=V, nnz=0, H=2000)
    par = base.params.copy()
    par["top_k"][3:6] = 0          # nuclei over the whole vocabulary, with and without a min-p bound
    par["min_p"][3:5] = 0.0
    par["temperature"][3:6] = 1.2
    par["rep_penalty"][8] = 0.8    # penalties that raise logits with top-k: general kernel
    par["top_k"][8] = 20
    par["temperature"][8] = 0.9
    par["n_prompt"][:] = 0         # ignored by the stateful call; the stateless call gets the true lengths below
    hot_ids = None if dtype == "f32" else base.hot_ids
    logits_np = [base.logits, np.roll(base.logits, 7, axis=1).copy(), np.roll(base.logits, 4001, axis=1).copy()]
    if dtype == "f32":
        logits = [_dev(x) for x in logits_np]
        logits_f32 = logits_np
    else:
        logits = [_dev(x.view(np.int16)).view(torch.bfloat16) for x in logits_np]
        logits_f32 = [synth.bf16_bits_to_f32(x) for x in logits_np]
    rank_p = np.arange(1, V + 1, dtype=np.float64) ** -1.1
    rank_p /= rank_p.sum()

    def prompt(n):
        return base.perm[rng.choice(V, size=n, p=rank_p)].astype(np.int32)

    prompts = [prompt(int(n)) for n in rng.integers(0, 90, B)]
    prompts[0] = np.zeros(0, np.int32)           # no prompt at all
    prompts[1] = prompt(L_max - 30)              # outgrows its slot after 30 steps
    gen = [[] for _ in range(B)]
    slots = rng.permutation(B + 5)[:B].astype(np.int32)   # rows use a permuted subset of B + 5 slots
    slots_dev = _dev(slots)

    ctx = binding.Sampler(V, L_max, max_B=B)
    st = binding.simple_state_create(0, B + 5, V, L_max)
    stream = torch.cuda.current_stream().cuda_stream
    ost = O.IncrementalHistory(B, V, L_max + 8)

    def restart(rows):
        ptr = np.concatenate([[0], np.cumsum([prompts[b].size for b in rows])]).astype(np.int64)
        ids = np.concatenate([prompts[b] for b in rows]).astype(np.int32) if ptr[-1] else np.zeros(1, np.int32)
        s_d, p_d, i_d = _dev(slots[rows]), _dev(ptr), _dev(ids)
        assert binding.simple_state_restart(st, s_d.data_ptr(), len(rows), p_d.data_ptr(), i_d.data_ptr(), 0, stream) == 0
        torch.cuda.synchronize()
        for b in rows:
            gen[b] = []
            ost.restart(b, prompts[b])

    restart(list(range(B)))
    hot_dev = None if hot_ids is None else _dev(hot_ids)
    summary = {"rows": 0, "ambiguous": 0, "soft": 0, "too_long": 0, "wide": 0, "general": 0}
    for step in range(steps):
        if step in (20, 41):   # two sequences end; their slots are given to new ones
            rows = [int(x) for x in rng.choice(np.arange(2, B), 2, replace=False)]
            for b in rows:
                prompts[b] = prompt(int(rng.integers(0, 60)))
            restart(rows)
        lg = logits[step % 3]
        params = par.copy()
        params_dev = _dev(params.view(np.uint8).reshape(B, 32))
        out_s = torch.full((B,), -9, dtype=torch.int32, device="cuda:0")
        diag_s = torch.zeros(B * 32, dtype=torch.uint8, device="cuda:0")
        rc = binding.simple_sample_state(ctx.ctx, st, slots_dev.data_ptr(), lg.data_ptr(), B, V,
                                         binding.SIMPLE_F32 if dtype == "f32" else binding.SIMPLE_BF16, lg.stride(0),
                                         params_dev.data_ptr(), 0 if hot_dev is None else hot_dev.data_ptr(),
                                         0 if hot_dev is None else hot_dev.numel(), base.seed, step, 0,
                                         out_s.data_ptr(), diag_s.data_ptr(), stream)
        assert rc == 0, binding.simple_strerror(rc)
        # the stateless call on the same token lists (prompt first, its length in n_prompt)
        ptr, ids = _csr(prompts, gen)
        params_c = par.copy()
        params_c["n_prompt"] = [p.size for p in prompts]
        diag_c = torch.zeros(B * 32, dtype=torch.uint8, device="cuda:0")
        out_c = ctx.sample(lg, _dev(params_c.view(np.uint8).reshape(B, 32)), _dev(ptr), _dev(ids), hot_dev,
                           seed=base.seed, step=step, diag=diag_c, V=V)
        torch.cuda.synchronize()
        ids_s, ids_c = out_s.cpu().numpy(), out_c.cpu().numpy()
        dg_s = diag_s.cpu().numpy().view(binding.ROW_DIAG_DTYPE)
        dg_c = diag_c.cpu().numpy().view(binding.ROW_DIAG_DTYPE)
        assert np.array_equal(ids_s, ids_c), (step, np.flatnonzero(ids_s != ids_c)[:8], ids_s[ids_s != ids_c][:8], ids_c[ids_s != ids_c][:8])
        for f in ("p_chosen", "n_survivors"):
            assert np.array_equal(dg_s[f], dg_c[f]), (step, f)
        assert np.array_equal(dg_s["flags"] & 0x1F9F, dg_c["flags"] & 0x1F9F), step   # all but the careful / replay notes
        too_long = np.array([p.size + len(g) > L_max for p, g in zip(prompts, gen)])
        assert np.array_equal(ids_s < 0, too_long), (step, np.flatnonzero(ids_s < 0), np.flatnonzero(too_long))
        assert np.array_equal((dg_s["flags"] & binding.DIAG_HISTORY_TOO_LONG) > 0, too_long)
        summary["too_long"] += int(too_long.sum())
        summary["wide"] += int(((dg_s["flags"] & binding.DIAG_WIDE) > 0).sum())
        summary["general"] += int(((dg_s["flags"] & binding.DIAG_GENERAL) > 0).sum())
        if step % 6 == 0 or step == steps - 1:   # the oracle, both ways
            rows = [b for b in range(B) if not too_long[b]]
            z = logits_f32[step % 3]
            want = O.sample(z, params_c, ptr, ids, hot_ids, base.seed, step, rows=rows)
            want_inc = O.sample_with_state(z, params, ost, hot_ids, base.seed, step)
            for b, o in zip(rows, want):
                assert (o.id, o.n) == (want_inc[b].id, want_inc[b].n) and abs(o.p_chosen - want_inc[b].p_chosen) < 1e-15
            s = P.compare(ids_s, dg_s, want, rows)
            summary["rows"] += s["rows"]; summary["ambiguous"] += s["ambiguous"]; summary["soft"] += s["soft_mismatch"]
        new = ids_s.copy()
        new_dev = _dev(new.astype(np.int32))
        assert binding.simple_state_append(st, slots_dev.data_ptr(), new_dev.data_ptr(), B, stream) == 0
        torch.cuda.synchronize()
        for b in range(B):
            if new[b] >= 0:
                gen[b].append(int(new[b]))
        ost.append(np.where(too_long, -1, new))
    print(f"{dtype}: {steps} steps, {summary}", flush=True)
    assert summary["too_long"] > 0 and summary["wide"] > 0 and summary["general"] > 0
    binding.simple_state_destroy(st)
    ctx.close()


def test_state_argument_errors_on_the_device_side():
    """A slot outside the state, a state of another vocabulary size, a context whose history capacity
    is below the state's, and a token id outside the vocabulary."""
    import torch
    V, L = 4096, 32
    w = synth.make_config(1, B=4, V=V, nnz=0)
    lg, params = _dev(w.logits), _dev(w.params.view(np.uint8).reshape(4, 32))
    out = torch.empty(4, dtype=torch.int32, device="cuda:0")
    diag = torch.zeros(4 * 32, dtype=torch.uint8, device="cuda:0")
    ctx = binding.Sampler(V, L, max_B=4)
    small = binding.Sampler(V, L // 2, max_B=4)
    st = binding.simple_state_create(0, 4, V, L)
    other = binding.simple_state_create(0, 4, V + 64, L)
    stream = torch.cuda.current_stream().cuda_stream

    def call(c, s, slots=None):
        return binding.simple_sample_state(c.ctx, s, 0 if slots is None else slots.data_ptr(), lg.data_ptr(), 4, V, binding.SIMPLE_F32,
                                           lg.stride(0), params.data_ptr(), 0, 0, w.seed, 0, 0, out.data_ptr(), diag.data_ptr(), stream)
    assert call(ctx, other) == binding.SIMPLE_EINVAL
    assert call(small, st) == binding.SIMPLE_ECAPACITY
    slots = _dev(np.array([0, 9, 2, -1], np.int32))
    assert call(ctx, st, slots) == 0
    torch.cuda.synchronize()
    ids = out.cpu().numpy()
    dg = diag.cpu().numpy().view(binding.ROW_DIAG_DTYPE)
    assert ids[1] == -1 and ids[3] == -1 and ids[0] >= 0 and ids[2] >= 0
    assert dg["flags"][1] & binding.DIAG_HISTORY_TOO_LONG and dg["flags"][3] & binding.DIAG_HISTORY_TOO_LONG
    # an id outside the vocabulary is kept, ignored and reported; append / restart skip slots outside the state
    new = _dev(np.array([5, 7, V + 3, 8], np.int32))
    assert binding.simple_state_append(st, slots.data_ptr(), new.data_ptr(), 4, stream) == 0
    assert call(ctx, st) == 0
    torch.cuda.synchronize()
    dg = diag.cpu().numpy().view(binding.ROW_DIAG_DTYPE)
    assert dg["flags"][2] & binding.DIAG_BAD_HISTORY_ID and not dg["flags"][0] & binding.DIAG_BAD_HISTORY_ID
    assert (out.cpu().numpy() >= 0).all()
    for s in (st, other):
        binding.simple_state_destroy(s)
    ctx.close(); small.close()
