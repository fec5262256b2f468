"""Helpers of the GPU-vs-oracle parity tests (not collected by pytest)."""
from __future__ import annotations

import math

import torch

import oracle
import paper_2511_06010_amd as moska
from moska_inputs import Inputs, Problem

# absolute tolerances of the benchmark definition and internal relative-RMS bars (outputs on the
# synthetic data are small, |O| ~ 0.02..0.3, so the absolute bars alone would pass a wrong kernel)
ABS_TOL = {"f32": None, "bf16": 2e-2, "fp8": 4e-2}
RMS_TOL = {"f32": 5e-6, "bf16": 5e-3, "fp8": 3e-2}
TIE_WINDOW = 1e-6


def tol_key(p: Problem) -> str:
    return "fp8" if p.kv_dtype == "fp8" else p.q_dtype


def assert_vectors_close(got: torch.Tensor, want: torch.Tensor, key: str, what: str):
    """got/want [..., D]; per-vector bound of the benchmark definition plus the relative-RMS bar."""
    got, want = got.to(torch.float64).cpu(), want.to(torch.float64)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    assert torch.isfinite(got).all(), f"{what}: non-finite values"
    err = (got - want).abs().amax(dim=-1)
    if key == "f32":
        bound = 1e-5 * want.abs().amax(dim=-1).clamp_min(1e-30)
    else:
        bound = torch.full_like(err, ABS_TOL[key])
    bad = err > bound
    assert not bad.any(), f"{what}: {int(bad.sum())} vectors out of tolerance, worst {float((err / bound).max()):.3g}x"
    rms = float((got - want).norm() / want.norm().clamp_min(1e-300))
    assert rms <= RMS_TOL[key], f"{what}: relative RMS error {rms:.3g} > {RMS_TOL[key]}"


def assert_lse_close(got: torch.Tensor, want: torch.Tensor, key: str, what: str):
    got, want = got.to(torch.float64).cpu(), want.to(torch.float64)
    inf = torch.isinf(want)
    assert torch.equal(torch.isinf(got), inf) and (got[inf] == want[inf]).all(), f"{what}: -inf pattern differs"
    d = (got[~inf] - want[~inf]).abs()
    bound = 1e-5 * want[~inf].abs().clamp_min(1.0) if key == "f32" else torch.full_like(d, ABS_TOL[key])
    assert (d <= bound).all(), f"{what}: worst LSE error {float(d.max()):.3g}"


def check_route(p: Problem, gpu_ids: torch.Tensor, o_ids: torch.Tensor, all_scores: torch.Tensor) -> int:
    """ids must be bit-exact; a difference is excused only among chunks whose oracle score lies
    within TIE_WINDOW of the oracle's k-th score.  Returns the number of excused (b,h) pairs."""
    g, o = gpu_ids.cpu(), o_ids
    if torch.equal(g, o):
        return 0
    excused = 0
    diff = (g != o).any(dim=-1).nonzero()
    for b, h in diff.tolist():
        s = all_scores[b, h]
        kth = s[o[b, h, -1].long()]
        gs, os_ = set(g[b, h].tolist()), set(o[b, h].tolist())
        assert len(gs) == p.k, f"route: duplicate ids at {(b, h)}"
        for c in gs ^ os_:
            assert abs(float(s[c] - kth)) <= TIE_WINDOW, f"route: ids differ outside the tie window at {(b, h)}"
        # the common part must be in the same order wherever scores are separated
        for j in range(p.k):
            if g[b, h, j] != o[b, h, j]:
                sj = float(s[o[b, h, j].long()])
                assert abs(float(s[g[b, h, j].long()]) - sj) <= TIE_WINDOW, f"route: order differs at {(b, h, j)}"
        excused += 1
    return excused


def gpu_pipeline(inp: Inputs, ids_override: torch.Tensor | None = None, fused: bool = False):
    """Run the five calls through the C interface.  Returns the Buffers (device tensors)."""
    p = inp.prob
    buf = moska.Buffers(p)
    buf.part_O.fill_(float("nan"))          # every slot must be written by the kernels
    buf.part_LSE.fill_(float("nan"))
    if fused:
        moska.decode_step(p, inp.Q, inp.E, inp.Ks, inp.Vs, inp.scale_k, inp.scale_v, inp.Ku, inp.Vu, inp.unique_len,
                          buf.ids, buf.bucket_off, buf.bucket_items, buf.part_O, buf.part_LSE, buf.O, buf.LSE, buf.ws)
    else:
        moska.route(p, inp.Q, inp.E, buf.ids, buf.scores, buf.ws)
        buf.routed_ids = buf.ids.clone()
        if ids_override is not None:
            buf.ids.copy_(ids_override)
        moska.bucket(p, buf.ids, buf.bucket_off, buf.bucket_items, buf.ws)
        moska.shared_attn(p, inp.Q, inp.Ks, inp.Vs, inp.scale_k, inp.scale_v, buf.ids, buf.bucket_off,
                          buf.bucket_items, buf.part_O, buf.part_LSE, buf.ws)
        moska.unique_attn(p, inp.Q, inp.Ku, inp.Vu, inp.unique_len, buf.part_O, buf.part_LSE, buf.ws)
        moska.merge(p, buf.part_O, buf.part_LSE, buf.O, buf.LSE)
    torch.cuda.synchronize()
    return buf


def check_against_oracle(inp_cpu: Inputs, label: str = ""):
    """Whole-problem parity: every call's output against the oracle on the same stored bits."""
    p = inp_cpu.prob
    key = tol_key(p)
    o_ids, _, o_all = oracle.route(p, inp_cpu.Q, inp_cpu.E, want_all_scores=True)
    inp = inp_cpu.to("cuda")
    buf = gpu_pipeline(inp)
    excused = check_route(p, buf.routed_ids, o_ids, o_all)
    if excused:                                   # attention is then checked on the oracle's routing
        buf = gpu_pipeline(inp, ids_override=o_ids.cuda())
    # selected scores (f32 output of an fp64 accumulation)
    if not excused:
        want = torch.gather(o_all, 2, o_ids.long())
        got = buf.scores.cpu().to(torch.float64)
        assert ((got - want).abs() <= 1e-6 * want.abs().clamp_min(1.0)).all(), f"{label} route scores"
    st = oracle.decode_step(inp_cpu, ids=o_ids)
    assert torch.equal(buf.bucket_off.cpu(), st.bucket_off), f"{label} bucket_off"
    assert torch.equal(buf.bucket_items.cpu(), st.bucket_items), f"{label} bucket_items"
    assert_vectors_close(buf.part_O, st.part_O, key, f"{label} part_O")
    assert_lse_close(buf.part_LSE, st.part_LSE, key, f"{label} part_LSE")
    assert_vectors_close(buf.O, st.O_direct, key, f"{label} O")
    assert_lse_close(buf.LSE, st.LSE_direct, key, f"{label} LSE")
    # the single-call entry point must give the same bits as the five calls
    if not excused:
        fb = gpu_pipeline(inp, fused=True)
        assert torch.equal(fb.ids, buf.ids) and torch.equal(fb.bucket_items, buf.bucket_items)
        assert torch.equal(fb.bucket_off, buf.bucket_off), f"{label} decode_step bucket_off"
        assert torch.equal(fb.O.view(torch.uint8), buf.O.view(torch.uint8)), f"{label} decode_step != five calls"
        # shared attention that makes its own bucket lists from ids
        own = moska.Buffers(p)
        moska.shared_attn(p, inp.Q, inp.Ks, inp.Vs, inp.scale_k, inp.scale_v, buf.ids, None, None, own.part_O,
                          own.part_LSE, own.ws)
        torch.cuda.synchronize()
        assert torch.equal(own.part_O[:, :, :p.k].view(torch.uint8), buf.part_O[:, :, :p.k].view(torch.uint8)), \
            f"{label} shared_attn from ids != from bucket lists"
        assert torch.equal(own.part_LSE[:, :, :p.k].view(torch.uint8), buf.part_LSE[:, :, :p.k].view(torch.uint8))
    return buf, st


def sub_inputs(inp: Inputs, ids: torch.Tensor, b: int, heads=None) -> tuple[Inputs, torch.Tensor]:
    """The single-query-token problem of token b on KV heads `heads` (default: all of them): for
    each head its k routed chunks gathered into a compact store (compact chunk j of head h is chunk
    ids[b,h,j]), the query heads of those groups and the unique context the token may see, as CPU
    tensors for the oracle.  With several query tokens per request, b counts query tokens (request
    b // T, token b % T) and the context is cut at the token."""
    p = inp.prob
    G = p.G
    hs = list(range(p.Hkv)) if heads is None else list(heads)
    dev = inp.Ks.device
    hv = torch.tensor(hs, device=dev)
    req, t = divmod(b, p.T)
    sel = ids[b, hs].long().to(dev).t().contiguous()              # [k, nh]: chunk of (slot j, head)
    qrows = torch.cat([torch.arange(h * G, (h + 1) * G) for h in hs]).to(dev)
    sp = p.with_(B=1, T=1, Hq=G * len(hs), Hkv=len(hs), C=p.k, name=p.name + f"-sub{b}")
    cpu = lambda x: x.contiguous().cpu()
    sub = Inputs(
        sp,
        Q=cpu(inp.Q[b:b + 1, qrows]),
        E=cpu(inp.E[hv[None, :], sel].permute(1, 0, 2)),          # [nh, k, D]
        Ks=cpu(inp.Ks[sel, hv[None, :]]),                         # [k, nh, L, D]
        Vs=cpu(inp.Vs[sel, hv[None, :]]),
        scale_k=None if inp.scale_k is None else cpu(inp.scale_k[sel, hv[None, :]]),
        scale_v=None if inp.scale_v is None else cpu(inp.scale_v[sel, hv[None, :]]),
        Ku=cpu(inp.Ku[req:req + 1, hv]),
        Vu=cpu(inp.Vu[req:req + 1, hv]),
        unique_len=cpu((inp.unique_len[req:req + 1] - (p.T - 1 - t)).clamp_min(0)),
        cstar=cpu(inp.cstar[req:req + 1]),
    )
    sub_ids = torch.arange(p.k, dtype=torch.int32).reshape(1, 1, p.k).repeat(1, len(hs), 1).contiguous()
    return sub, sub_ids


def stratified_tokens(p: Problem, off: torch.Tensor, items: torch.Tensor, n: int, seed: int) -> list[int]:
    """n query tokens chosen by bucket popularity: the first and last item of the hottest and of the
    coldest non-empty bucket, one item of the buckets at the size quartiles, then seeded random tokens."""
    sizes = off[1:] - off[:-1]
    nz = torch.nonzero(sizes > 0).flatten()
    order = nz[torch.argsort(sizes[nz], stable=True)]
    picks = [order[-1], order[0]] + [order[int(q * (len(order) - 1))] for q in (0.25, 0.5, 0.75)]
    toks = []
    for bk in picks:
        for item in (items[off[bk]], items[off[bk + 1] - 1]):
            toks.append(int(item) // p.k)
    g = torch.Generator().manual_seed(seed)
    out = list(dict.fromkeys(toks))
    while len(out) < min(n, p.Bq):
        t = int(torch.randint(0, p.Bq, (1,), generator=g))
        if t not in out:
            out.append(t)
    return out
