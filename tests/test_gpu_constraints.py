"""Logit bias and allow-lists on the GPU: the constraint pass against the oracle's apply_constraints,
bit for bit, and the sampling call on its output against the oracle's sample on the same
constrained rows (ids, p~, survivor counts).  Rows with a bias list, an allow-list, both or neither;
repeated and out-of-range ids; float32 and bfloat16 logits; in place for float32."""
import numpy as np
import pytest

import parity_util as P
from oracle import simple_oracle as O
from paper_2512_00719_amd import binding, synth

pytestmark = pytest.mark.gpu


def _dev(x):
    import torch
    return torch.from_numpy(np.ascontiguousarray(x)).to("cuda:0")


def _csr(lists, dtype):
    ptr = np.concatenate([[0], np.cumsum([len(x) for x in lists])]).astype(np.int64)
    flat = np.concatenate([np.asarray(x, dtype=dtype) for x in lists]) if ptr[-1] else np.zeros(1, dtype)
    return ptr, flat.astype(dtype)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_constraint_pass_and_sampling_on_its_output(dtype):
    import torch
    rng = np.random.default_rng(41 if dtype == "f32" else 42)
    w = synth.make_config(3 if dtype == "f32" else 5, B=28, V=20_008, nnz=400, H=1500)
    B, V = w.B, w.V
    top = np.argsort(-w.logits_f32(), axis=1)[:, :300]
    bias_ids, bias_vals, allow = [], [], []
    for b in range(B):
        kind = b % 4   # 0 nothing, 1 bias, 2 allow-list, 3 both
        nb = int(rng.integers(1, 60)) if kind in (1, 3) else 0
        ids = np.concatenate([rng.choice(top[b], nb // 2 + 1), rng.integers(0, V, nb // 2)])[:nb] if nb else np.zeros(0, np.int64)
        vals = (rng.standard_normal(nb) * 4).astype(np.float32)
        if nb > 4:
            ids[1] = ids[0]           # the same column twice: the additions are ordered
            ids[3] = V + 7            # outside the vocabulary: ignored
            vals[2] = -np.inf         # bans a token
            vals[4] = 30.0            # all but forces one
        bias_ids.append(ids.astype(np.int32)); bias_vals.append(vals)
        na = int(rng.choice([1, 5, 200, 3000])) if kind in (2, 3) else 0
        al = np.concatenate([rng.choice(top[b], min(na, 100), replace=False), rng.integers(0, V, max(na - 100, 0))]) if na else np.zeros(0, np.int64)
        if na > 3:
            al[2] = -3                # outside the vocabulary: ignored
        allow.append(al.astype(np.int32))
    bp, bi = _csr(bias_ids, np.int32)
    _, bv = _csr(bias_vals, np.float32)
    ap, ai = _csr(allow, np.int32)
    z32 = w.logits_f32()
    want = np.stack([O.apply_constraints(z32[b],
                                         [i for i in bias_ids[b] if 0 <= i < V], [v for i, v in zip(bias_ids[b], bias_vals[b]) if 0 <= i < V],
                                         [i for i in allow[b] if 0 <= i < V] if len(allow[b]) else None) for b in range(B)])
    dev = P.to_device(w)
    lg = dev["logits"]
    stride = V + 24
    out = torch.full((B, stride), 7.0, dtype=torch.float32, device="cuda:0")
    stream = torch.cuda.current_stream().cuda_stream
    args = (_dev(bp), _dev(bi), _dev(bv), _dev(ap), _dev(ai))
    rc = binding.simple_apply_logit_constraints(lg.data_ptr(), B, V, binding.SIMPLE_F32 if dtype == "f32" else binding.SIMPLE_BF16, lg.stride(0),
                                                *[t.data_ptr() for t in args], out.data_ptr(), stride, stream)
    assert rc == 0, binding.simple_strerror(rc)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert np.array_equal(got[:, :V].view(np.uint32), want.view(np.uint32))   # bit for bit, -inf included
    assert np.all(got[:, V:] == 7.0)                                          # nothing written past a row's V columns
    if dtype == "f32":  # in place
        lg2 = lg.clone()
        rc = binding.simple_apply_logit_constraints(lg2.data_ptr(), B, V, binding.SIMPLE_F32, lg2.stride(0),
                                                    *[t.data_ptr() for t in args], lg2.data_ptr(), lg2.stride(0), stream)
        torch.cuda.synchronize()
        assert rc == 0 and np.array_equal(lg2.cpu().numpy().view(np.uint32), want.view(np.uint32))
    # bias lists alone / allow-lists alone (the other pair NULL)
    only_bias = torch.empty((B, V), dtype=torch.float32, device="cuda:0")
    rc = binding.simple_apply_logit_constraints(lg.data_ptr(), B, V, binding.SIMPLE_F32 if dtype == "f32" else binding.SIMPLE_BF16, lg.stride(0),
                                                args[0].data_ptr(), args[1].data_ptr(), args[2].data_ptr(), 0, 0, only_bias.data_ptr(), V, stream)
    torch.cuda.synchronize()
    ref = np.stack([O.apply_constraints(z32[b], [i for i in bias_ids[b] if 0 <= i < V],
                                        [v for i, v in zip(bias_ids[b], bias_vals[b]) if 0 <= i < V]) for b in range(B)])
    assert rc == 0 and np.array_equal(only_bias.cpu().numpy().view(np.uint32), ref.view(np.uint32))
    # the sampling call on the constrained rows: ids, p~ and survivor counts against the oracle
    cw = synth.Workload("constrained", B, V, "f32", want, w.params, w.hist_ptr, w.hist_ids, hot_ids=w.hot_ids, seed=w.seed)
    s = binding.Sampler(V, 400, max_B=B)
    cdev = {"logits": out[:, :V], "params": dev["params"], "hist_ptr": dev["hist_ptr"], "hist_ids": dev["hist_ids"], "hot_ids": dev["hot_ids"]}
    for step in (0, 1):
        ids, dg = P.run_gpu(cw, step, sampler=s, dev=cdev)
        summary = P.compare(ids, dg, P.run_oracle(cw, step), range(B))
        for b in range(B):
            if len(allow[b]):
                assert ids[b] in set(int(i) for i in allow[b])        # only allowed tokens are ever drawn
    print(f"{dtype}: {summary}", flush=True)
    s.close()
