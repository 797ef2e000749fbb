"""GPU parity of the packed variable-length entry points: every sequence of the pack against the oracle run on
that sequence alone (the recurrence of Eq. 5 restarts at each boundary)."""
import numpy as np
import pytest

import oracle
import sla_inputs as si
from gpu_util import GDN, GLA, RETNET, TOL, rel_err, to_device
from oracle import sla_backward as ob

pytestmark = pytest.mark.gpu

LENGTHS = [37, 1, 0, 300, 16, 129, 64]  # ragged, block-aligned, single-token and empty sequences


def pack(variant, dtype, lengths, H, dk, dv, seed):
    T = int(sum(lengths))
    d = si.custom(variant, dtype, B=1, T=T, H=H, dk=dk, dv=dv, seed=seed)
    cu = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)
    return d, cu


def seq(d, variant, cu, i):
    a, b = int(cu[i]), int(cu[i + 1])
    f = lambda x: None if x is None else x[:, a:b]
    out = {k: f(d[k]) for k in ("q", "k", "v", "q_logits", "k_logits", "beta")}
    out["log_decay"] = d["log_decay"] if variant == RETNET else d["log_decay"][:, a:b]
    return out, a, b


@pytest.mark.parametrize("variant", [RETNET, GLA, GDN])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_forward_varlen(variant, dtype):
    import torch
    import paper_2602_01744_amd as sla

    H, dk, dv = 3, 128, 128
    d, cu = pack(variant, dtype, LENGTHS, H, dk, dv, seed=1400 + variant)
    B = len(LENGTHS)
    s0 = si.initial_state(B, H, dk, dv, seed=14)
    g, _ = to_device(d, dtype, variant)
    sq = lambda t: None if t is None else (t if t.dim() == 1 else t[0].contiguous())
    out, fin = sla.forward_varlen(variant, sq(g["q"]), sq(g["k"]), sq(g["v"]), sq(g["q_logits"]), sq(g["k_logits"]),
                                  sq(g["log_decay"]), sq(g["beta"]), torch.from_numpy(cu).cuda(),
                                  torch.from_numpy(s0).cuda())
    torch.cuda.synchronize()
    out = out.float().cpu().numpy().astype(np.float64)
    fin = fin.cpu().numpy().astype(np.float64)
    for i in range(B):
        ds, a, b = seq(d, variant, cu, i)
        if b == a:
            assert np.array_equal(fin[i], s0[i].astype(np.float64))  # an empty sequence passes its state through
            continue
        ro, rf = oracle.forward(variant, ds["q"], ds["k"], ds["v"], ds["q_logits"], ds["k_logits"], ds["log_decay"],
                                ds["beta"], s0[i:i + 1])
        eo, ef = rel_err(out[a:b], ro[0]), rel_err(fin[i], rf[0])
        print(f"[varlen] {si.VARIANT_NAMES[variant]} {dtype} seq {i} len {b - a}: out {eo:.2e} state {ef:.2e}", flush=True)
        assert eo <= TOL[dtype] and ef <= TOL[dtype]


@pytest.mark.parametrize("variant", [RETNET, GLA])
@pytest.mark.parametrize("dtype,dk", [("bf16", 128), ("f32", 128), ("bf16", 32)])
def test_backward_varlen(variant, dtype, dk):
    import torch
    import paper_2602_01744_amd as sla

    H, dv = 3, 64
    d, cu = pack(variant, dtype, LENGTHS, H, dk, dv, seed=1410 + variant)
    B, T = len(LENGTHS), int(cu[-1])
    s0 = si.initial_state(B, H, dk, dv, seed=15)
    cot = si.cotangents(1, T, H, dk, dv, seed=1411)
    dsf = si.initial_state(B, H, dk, dv, seed=16)
    g, tdt = to_device(d, dtype, variant)
    sq = lambda t: None if t is None else (t if t.dim() == 1 else t[0].contiguous())
    res = sla.backward_varlen(variant, sq(g["q"]), sq(g["k"]), sq(g["v"]), sq(g["q_logits"]), sq(g["k_logits"]),
                              sq(g["log_decay"]), torch.from_numpy(cot["d_out"][0]).to(tdt).cuda(),
                              torch.from_numpy(cu).cuda(), torch.from_numpy(s0).cuda(), torch.from_numpy(dsf).cuda(),
                              want_d_initial_state=True)
    torch.cuda.synchronize()
    got = {n: None if t is None else t.float().cpu().numpy().astype(np.float64) for n, t in res.items()}
    names = {"dq": "dq", "dk": "dk", "dv": "dv", "dq_head_logits": "dq_logits", "dk_head_logits": "dk_logits"}
    if variant == GLA:
        names["dlog_decay"] = "dlog_decay"
    for i in range(B):
        ds, a, b = seq(d, variant, cu, i)
        if b == a:
            assert np.array_equal(got["d_initial_state"][i], dsf[i].astype(np.float64))
            continue
        ref = ob.backward(variant, ds["q"], ds["k"], ds["v"], ds["q_logits"], ds["k_logits"], ds["log_decay"],
                          cot["d_out"][:, a:b], s0[i:i + 1], dsf[i:i + 1])
        errs = {n: rel_err(got[n][a:b], ref[rn][0]) for n, rn in names.items()}
        errs["d_initial_state"] = rel_err(got["d_initial_state"][i], ref["dinitial_state"][0])
        print(f"[varlen backward] {dtype} {si.VARIANT_NAMES[variant]} seq {i} len {b - a}: " +
              " ".join(f"{n}={e:.2e}" for n, e in errs.items()), flush=True)
        for n, e in errs.items():
            assert e <= TOL[dtype], (i, n, e)


def test_backward_varlen_gdn():
    import torch
    import paper_2602_01744_amd as sla

    H, dk, dv = 3, 64, 128
    d, cu = pack(GDN, "bf16", LENGTHS, H, dk, dv, seed=1420)
    B, T = len(LENGTHS), int(cu[-1])
    s0 = si.initial_state(B, H, dk, dv, seed=17)
    cot = si.cotangents(1, T, H, dk, dv, seed=1421)
    dsf = si.initial_state(B, H, dk, dv, seed=18)
    g, _ = to_device(d, "bf16", GDN)
    sq = lambda t: None if t is None else t[0].contiguous()
    res = sla.backward_gdn_varlen(sq(g["q"]), sq(g["k"]), sq(g["v"]), sq(g["q_logits"]), sq(g["k_logits"]),
                                  sq(g["log_decay"]), sq(g["beta"]),
                                  torch.from_numpy(cot["d_out"][0]).to(torch.bfloat16).cuda(),
                                  torch.from_numpy(cu).cuda(), torch.from_numpy(s0).cuda(), torch.from_numpy(dsf).cuda(),
                                  want_d_initial_state=True)
    torch.cuda.synchronize()
    got = {n: None if t is None else t.float().cpu().numpy().astype(np.float64) for n, t in res.items()}
    names = {"dq": "dq", "dk": "dk", "dv": "dv", "dq_head_logits": "dq_logits", "dk_head_logits": "dk_logits",
             "dlog_decay": "dlog_decay", "dbeta": "dbeta"}
    for i in range(B):
        ds, a, b = seq(d, GDN, cu, i)
        if b == a:
            assert np.array_equal(got["d_initial_state"][i], dsf[i].astype(np.float64))
            continue
        ref = ob.backward(GDN, ds["q"], ds["k"], ds["v"], ds["q_logits"], ds["k_logits"], ds["log_decay"],
                          cot["d_out"][:, a:b], s0[i:i + 1], dsf[i:i + 1], beta=ds["beta"])
        errs = {n: rel_err(got[n][a:b], ref[rn][0]) for n, rn in names.items()}
        errs["d_initial_state"] = rel_err(got["d_initial_state"][i], ref["dinitial_state"][0])
        print(f"[varlen backward] gdn seq {i} len {b - a}: " + " ".join(f"{n}={e:.2e}" for n, e in errs.items()),
              flush=True)
        for n, e in errs.items():
            assert e <= TOL["bf16"], (i, n, e)


def test_varlen_equals_batch_for_equal_lengths():
    """A pack of equal-length sequences is the rectangular batch: the two entry points agree bit for bit."""
    import torch
    import paper_2602_01744_amd as sla

    B, T, H, dk, dv = 4, 96, 4, 64, 128
    d = si.custom(GLA, "bf16", B=B, T=T, H=H, dk=dk, dv=dv, seed=1420)
    g, _ = to_device(d, "bf16", GLA)
    out, fin = sla.forward(GLA, g["q"], g["k"], g["v"], g["q_logits"], g["k_logits"], g["log_decay"])
    cu = torch.arange(0, (B + 1) * T, T, dtype=torch.int32).cuda()
    fl = lambda t: t.reshape((B * T,) + tuple(t.shape[2:])).contiguous()
    out2, fin2 = sla.forward_varlen(GLA, fl(g["q"]), fl(g["k"]), fl(g["v"]), fl(g["q_logits"]), fl(g["k_logits"]),
                                    fl(g["log_decay"]), None, cu)
    torch.cuda.synchronize()
    assert torch.equal(fl(out), out2) and torch.equal(fin, fin2)


@pytest.mark.parametrize("variant", [GLA, GDN])
def test_tokens_outside_every_sequence_are_left_untouched(variant):
    """cu_seqlens[0] > 0 and cu_seqlens[B] < T: the tokens before the first and after the last sequence belong to no
    sequence.  Forward and backward must neither read them into a result nor write their rows: every output tensor
    is pre-filled with a canary, which must survive there, while the sequences still agree with the oracle."""
    import torch
    import paper_2602_01744_amd as sla

    H, dk, dv, lead, tail = 3, 64, 64, 11, 5
    lengths = [40, 0, 70]
    T = lead + sum(lengths) + tail
    d = si.custom(variant, "bf16", B=1, T=T, H=H, dk=dk, dv=dv, seed=1430 + variant)
    cu = (lead + np.concatenate([[0], np.cumsum(lengths)])).astype(np.int32)
    B = len(lengths)
    cot = si.cotangents(1, T, H, dk, dv, seed=1431)
    g, _ = to_device(d, "bf16", variant)
    sq = lambda t: None if t is None else (t if t.dim() == 1 else t[0].contiguous())
    q, k, v, ql, kl, ld, beta = (sq(g[n]) for n in ("q", "k", "v", "q_logits", "k_logits", "log_decay", "beta"))
    dout = torch.from_numpy(cot["d_out"][0]).to(torch.bfloat16).cuda()
    cud = torch.from_numpy(cu).cuda()
    CAN = 7.0
    can = lambda like: torch.full_like(like, CAN)
    out, fin = can(v), torch.empty((B, H, dk, dv), dtype=torch.float32, device="cuda")
    ptr = lambda t: None if t is None else t.data_ptr()
    st = torch.cuda.current_stream().cuda_stream
    params = sla.SlaParams(variant, sla.BF16, B, T, H, dk, dv, 0, 0, 1)
    rc = sla.sla_forward_varlen(params, ptr(q), ptr(k), ptr(v), ptr(ql), ptr(kl), ptr(ld), ptr(beta), ptr(cud), None,
                                ptr(out), ptr(fin), st)
    assert rc == 0
    gr = {n: can(t) for n, t in (("dq", q), ("dk", k), ("dv", v), ("dql", ql), ("dkl", kl))}
    if variant == GLA:
        gr["dld"] = can(ld)
        need = sla.sla_backward_varlen_workspace_bytes(params)
        ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
        rc = sla.sla_backward_varlen(params, ptr(q), ptr(k), ptr(v), ptr(ql), ptr(kl), ptr(ld), ptr(cud), None, ptr(dout),
                                     None, ptr(gr["dq"]), ptr(gr["dk"]), ptr(gr["dv"]), ptr(gr["dql"]), ptr(gr["dkl"]),
                                     ptr(gr["dld"]), None, ptr(ws), need, st)
    else:
        gr["dld"], gr["dbeta"] = can(ld), can(beta)
        need = sla.sla_backward_gdn_varlen_workspace_bytes(params)
        ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
        rc = sla.sla_backward_gdn_varlen(params, ptr(q), ptr(k), ptr(v), ptr(ql), ptr(kl), ptr(ld), ptr(beta), ptr(cud),
                                         None, ptr(dout), None, ptr(gr["dq"]), ptr(gr["dk"]), ptr(gr["dv"]),
                                         ptr(gr["dql"]), ptr(gr["dkl"]), ptr(gr["dld"]), ptr(gr["dbeta"]), None, ptr(ws),
                                         need, st)
    assert rc == 0
    torch.cuda.synchronize()
    lo, hi = int(cu[0]), int(cu[-1])
    for name, t in [("out", out)] + list(gr.items()):
        x = t.float().cpu().numpy()
        assert np.all(x[:lo] == CAN) and np.all(x[hi:] == CAN), f"{name}: rows outside the sequences were written"
        assert np.all(np.isfinite(x[lo:hi])), name
    # the sequences themselves: first and last against the oracle
    names = {"dq": "dq", "dk": "dk", "dv": "dv", "dql": "dq_logits", "dkl": "dk_logits", "dld": "dlog_decay"}
    if variant == GDN:
        names["dbeta"] = "dbeta"
    for i in (0, 2):
        ds, a, b = seq(d, variant, cu, i)
        ro, _ = oracle.forward(variant, ds["q"], ds["k"], ds["v"], ds["q_logits"], ds["k_logits"], ds["log_decay"],
                               ds["beta"], None)
        assert rel_err(out.float().cpu().numpy().astype(np.float64)[a:b], ro[0]) <= TOL["bf16"]
        ref = ob.backward(variant, ds["q"], ds["k"], ds["v"], ds["q_logits"], ds["k_logits"], ds["log_decay"],
                          cot["d_out"][:, a:b], beta=ds["beta"])
        for n, rn in names.items():
            e = rel_err(gr[n].float().cpu().numpy().astype(np.float64)[a:b], ref[rn][0])
            assert e <= TOL["bf16"], (i, n, e)
