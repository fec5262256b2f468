"""Pins of the CPU oracle against things it did not compute itself.

The paper prints no worked numeric example (its evaluation is an analytical model), so the
oracle is pinned by mathematics: library routines (scipy softmax / logsumexp, numpy lexsort
and stable argsort, torch dtype conversions), closed forms, symmetries, brute force on small
inputs, and one hand-worked fixture under tests/golden/.
"""
import math
import os

import numpy as np
import pytest
import torch
from scipy.special import logsumexp, softmax

import oracle
from moska_inputs import Problem, generate, config

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def small(**kw):
    base = dict(B=5, Hq=6, Hkv=2, D=16, C=6, L=24, k=3, U=20, q_dtype="f32", kv_dtype="f32")
    base.update(kw)
    return Problem(**base)


def f64(t):
    """Library widening (torch), independent of the oracle's own decoder."""
    return t.to(torch.float64).numpy()


def dense_reference(inp, ids):
    """Attention of every (b,hq) over concat(routed chunks, unique[:len]) with scipy."""
    p = inp.prob
    Q, Ks, Vs, Ku, Vu = map(f64, (inp.Q, inp.Ks, inp.Vs, inp.Ku, inp.Vu))
    if inp.scale_k is not None:
        Ks = Ks * f64(inp.scale_k)[:, :, None, None]
        Vs = Vs * f64(inp.scale_v)[:, :, None, None]
    O = np.zeros((p.B, p.Hq, p.D))
    LSE = np.zeros((p.B, p.Hq))
    for b in range(p.B):
        n = int(inp.unique_len[b])
        for hq in range(p.Hq):
            h = hq // p.G
            sel = [int(c) for c in ids[b, h]]
            K = np.concatenate([Ks[c, h] for c in sel] + [Ku[b, h, :n]], axis=0)
            V = np.concatenate([Vs[c, h] for c in sel] + [Vu[b, h, :n]], axis=0)
            z = p.scale * (K @ Q[b, hq])
            O[b, hq] = softmax(z) @ V
            LSE[b, hq] = logsumexp(z)
    return O, LSE


# ------------------------------------------------------------------ widening of stored dtypes

def test_widen_fp8_all_bytes_matches_torch():
    b = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn)
    got, want = oracle.widen(b).numpy(), b.to(torch.float64).numpy()
    assert np.array_equal(np.isnan(got), np.isnan(want))
    assert np.array_equal(got[~np.isnan(got)], want[~np.isnan(want)])
    assert np.nanmax(got) == 448.0 and got[1] == 2.0 ** -9      # format constants (OCP e4m3fn)


def test_widen_bf16_and_f32_match_torch():
    g = torch.Generator().manual_seed(1)
    bits = torch.randint(0, 1 << 16, (4096,), generator=g, dtype=torch.int32).to(torch.uint16)
    bits = bits[(bits & 0x7F80) != 0x7F80]                      # drop inf/nan patterns
    x = bits.view(torch.bfloat16)
    assert np.array_equal(oracle.widen(x).numpy(), x.to(torch.float64).numpy())
    y = torch.randn(1000, generator=g)
    assert np.array_equal(oracle.widen(y).numpy(), y.to(torch.float64).numpy())


# ------------------------------------------------------------------ S1/S2 routing

@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_route_matches_bruteforce_lexsort(dt):
    p = small(q_dtype=dt, kv_dtype=dt, B=7, C=9, k=4)
    inp = generate(p, seed=3)
    ids, sel, allv = oracle.route(p, inp.Q, inp.E, want_all_scores=True)
    Q, E = f64(inp.Q), f64(inp.E)
    qs = Q.reshape(p.B, p.Hkv, p.G, p.D).sum(axis=2)
    s = np.einsum("bhd,hcd->bhc", qs, E)
    np.testing.assert_allclose(allv.numpy(), s, rtol=0, atol=1e-12)
    for b in range(p.B):
        for h in range(p.Hkv):
            order = np.lexsort((np.arange(p.C), -allv[b, h].numpy()))   # score desc, then id asc
            assert list(ids[b, h].numpy()) == list(order[:p.k])
            np.testing.assert_array_equal(sel[b, h].numpy(), allv[b, h].numpy()[order[:p.k]])


def test_route_tie_break_prefers_lower_chunk_id():
    p = small(C=6, k=3)
    inp = generate(p, seed=5)
    E = inp.E.clone()
    E[:, 4] = E[:, 1]                  # chunks 1 and 4 tie exactly
    E[:, 5] = E[:, 1]
    ids, _, allv = oracle.route(p, inp.Q, E, want_all_scores=True)
    for b in range(p.B):
        for h in range(p.Hkv):
            got = list(ids[b, h].numpy())
            for c in (4, 5):
                if c in got:
                    assert 1 in got and got.index(1) < got.index(c)
            if 5 in got:
                assert got.index(4) < got.index(5)


def test_route_zero_query_returns_first_k_ids():
    p = small(C=7, k=4)
    inp = generate(p, seed=6)
    ids, sel = oracle.route(p, torch.zeros_like(inp.Q), inp.E)
    assert (ids == torch.arange(4, dtype=torch.int32)).all() and (sel == 0).all()


def test_route_group_scores_add_over_the_heads_of_a_group():
    # one head of the group carries the query, the others are zero: the selection must equal
    # a single-head routing of that query (sum over the group, not max / first head)
    p = small(Hq=4, Hkv=1, C=8, k=3)
    inp = generate(p, seed=8)
    Q = torch.zeros_like(inp.Q)
    Q[:, 2] = inp.Q[:, 2]
    ids, _ = oracle.route(p, Q, inp.E)
    s = f64(Q[:, 2]) @ f64(inp.E[0]).T
    for b in range(p.B):
        assert list(ids[b, 0].numpy()) == list(np.lexsort((np.arange(p.C), -s[b]))[:p.k])


def test_generator_aims_queries_at_cstar():
    # data-model property: the top-1 routed chunk is the chunk the query was drawn around
    p = config(0)
    inp = generate(p, seed=20251106)
    ids, _ = oracle.route(p, inp.Q, inp.E)
    assert (ids[:, :, 0] == inp.cstar[:, None].to(torch.int32)).all()
    p1 = Problem(B=32, Hq=8, Hkv=2, D=128, C=16, L=64, k=2, U=8)
    inp = generate(p1, seed=9)
    ids, _ = oracle.route(p1, inp.Q, inp.E)
    assert (ids[:, :, 0] == inp.cstar[:, None].to(torch.int32)).float().mean() > 0.97


# ------------------------------------------------------------------ bucketing

def test_bucket_matches_stable_argsort():
    p = small(B=9, C=5, k=3, Hkv=2, Hq=4)
    inp = generate(p, seed=11)
    ids, _ = oracle.route(p, inp.Q, inp.E)
    off, items = oracle.bucket(p, ids)
    off, items = off.numpy(), items.numpy()
    assert off[0] == 0 and off[-1] == p.B * p.Hkv * p.k
    for h in range(p.Hkv):
        key = ids[:, h, :].numpy().reshape(-1)              # item index b*k+j -> chunk
        order = np.argsort(key, kind="stable")
        lo, hi = off[h * p.C], off[(h + 1) * p.C]
        assert list(items[lo:hi]) == list(order)
        counts = np.bincount(key, minlength=p.C)
        assert list(np.diff(off[h * p.C:(h + 1) * p.C + 1])) == list(counts)


# ------------------------------------------------------------------ S3/S4/S5 attention

@pytest.mark.parametrize("dt,kv", [("f32", "f32"), ("bf16", "bf16"), ("bf16", "fp8")])
def test_topk_equals_all_chunks_is_dense_attention(dt, kv):
    # k = C: routing prunes nothing, so the result is dense softmax attention over
    # concat(all shared chunks, unique context) -- computed here with scipy.
    p = small(q_dtype=dt, kv_dtype=kv, C=4, k=4, scale=0.7)
    inp = generate(p, seed=12, unique_len="ragged")
    st = oracle.decode_step(inp)
    assert sorted(st.ids[0, 0].tolist()) == [0, 1, 2, 3]
    O, LSE = dense_reference(inp, st.ids)
    np.testing.assert_allclose(st.O_direct.numpy(), O, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(st.LSE_direct.numpy(), LSE, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(st.O.numpy(), O, rtol=1e-12, atol=1e-13)       # merged partials
    np.testing.assert_allclose(st.LSE.numpy(), LSE, rtol=1e-12, atol=1e-13)


def test_routed_subset_matches_scipy_on_the_same_subset():
    p = small(C=7, k=2, Hq=8, Hkv=4, B=4, scale=1.3)
    inp = generate(p, seed=13, unique_len="ragged")
    st = oracle.decode_step(inp)
    O, LSE = dense_reference(inp, st.ids)
    np.testing.assert_allclose(st.O.numpy(), O, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(st.O_direct.numpy(), O, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(st.LSE.numpy(), LSE, rtol=1e-12, atol=1e-13)


def test_partials_are_per_chunk_scipy_attention():
    p = small(C=5, k=3, B=3)
    inp = generate(p, seed=14)
    ids, _ = oracle.route(p, inp.Q, inp.E)
    pO, pL = oracle.partials(inp, ids)
    Q, Ks, Vs, Ku, Vu = map(f64, (inp.Q, inp.Ks, inp.Vs, inp.Ku, inp.Vu))
    for b in range(p.B):
        for hq in range(p.Hq):
            h = hq // p.G
            for j in range(p.k + 1):
                K, V = (Ks[ids[b, h, j], h], Vs[ids[b, h, j], h]) if j < p.k else (Ku[b, h], Vu[b, h])
                z = K @ Q[b, hq]
                np.testing.assert_allclose(pO[b, hq, j].numpy(), softmax(z) @ V, rtol=1e-12, atol=1e-14)
                np.testing.assert_allclose(pL[b, hq, j].item(), logsumexp(z), rtol=1e-13)


def test_merge_of_any_partition_equals_attention_over_union():
    rng = np.random.default_rng(15)
    D, n = 8, 57
    q, K, V = rng.normal(size=D), rng.normal(size=(n, D)) * 2, rng.normal(size=(n, D))
    want_O, want_lse = softmax(K @ q) @ V, logsumexp(K @ q)
    for trial in range(20):
        parts = rng.integers(1, 6)
        cuts = np.sort(rng.integers(0, n + 1, size=parts - 1))       # uneven, possibly empty parts
        perm = rng.permutation(n)
        pieces = np.split(perm, cuts)
        pO, pL = [], []
        for idx in pieces:
            o, l = oracle.attend(torch.tensor(q), torch.tensor(K[idx]).reshape(-1, D),
                                 torch.tensor(V[idx]).reshape(-1, D))
            pO.append(o)
            pL.append(l)
        O, LSE = oracle.merge(torch.stack(pO)[None], torch.tensor(pL, dtype=torch.float64)[None])
        np.testing.assert_allclose(O[0].numpy(), want_O, rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(LSE[0].item(), want_lse, rtol=1e-13)


def test_merge_all_empty_is_zero_and_minus_inf():
    O, LSE = oracle.merge(torch.zeros(1, 3, 4), torch.full((1, 3), -math.inf))
    assert (O == 0).all() and LSE[0].item() == -math.inf


def test_closed_forms():
    rng = np.random.default_rng(16)
    D, n = 8, 33
    q, K, V = rng.normal(size=D), rng.normal(size=(n, D)), rng.normal(size=(n, D))
    t = torch.tensor
    # constant values: the output is that vector whatever the weights are
    v0 = rng.normal(size=D)
    O, _ = oracle.attend(t(q), t(K), t(np.tile(v0, (n, 1))))
    np.testing.assert_allclose(O.numpy(), v0, rtol=1e-13)
    # zero query: uniform weights, LSE = ln n
    O, lse = oracle.attend(t(np.zeros(D)), t(K), t(V))
    np.testing.assert_allclose(O.numpy(), V.mean(axis=0), rtol=1e-12, atol=1e-15)
    assert abs(lse - math.log(n)) < 1e-13
    # identical keys: LSE = scale*q.k + ln n
    k0 = rng.normal(size=D)
    O, lse = oracle.attend(t(q), t(np.tile(k0, (n, 1))), t(V), scale=0.3)
    assert abs(lse - (0.3 * q @ k0 + math.log(n))) < 1e-12
    np.testing.assert_allclose(O.numpy(), V.mean(axis=0), rtol=1e-12, atol=1e-15)
    # a single key: O = v, LSE = the logit
    O, lse = oracle.attend(t(q), t(K[:1]), t(V[:1]), scale=2.0)
    np.testing.assert_allclose(O.numpy(), V[0], rtol=1e-15)
    assert abs(lse - 2.0 * q @ K[0]) < 1e-13
    # empty set
    O, lse = oracle.attend(t(q), t(K[:0]), t(V[:0]))
    assert (O == 0).all() and lse == -math.inf
    # a huge logit must not overflow (max subtraction)
    O, lse = oracle.attend(t(q * 0 + 1), t(np.full((2, D), 200.0)), t(V[:2]))
    assert abs(lse - (1600.0 + math.log(2))) < 1e-9


def test_hand_worked_two_key_fixture():
    # tests/golden/softmax_two_keys.txt: numbers worked by hand from the softmax definition
    vals = {}
    for line in open(os.path.join(GOLDEN, "softmax_two_keys.txt")):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split("=")
            vals[k.strip()] = [float(x) for x in v.split()]
    q = torch.tensor(vals["q"], dtype=torch.float64)
    K = torch.tensor(vals["K"], dtype=torch.float64).reshape(2, 2)
    V = torch.tensor(vals["V"], dtype=torch.float64).reshape(2, 2)
    O, lse = oracle.attend(q, K, V, scale=vals["scale"][0])
    np.testing.assert_allclose(O.numpy(), vals["O"], rtol=0, atol=1e-14)
    assert abs(lse - vals["LSE"][0]) < 1e-14


def test_symmetries():
    p = small(C=6, k=3)
    inp = generate(p, seed=17)
    st = oracle.decode_step(inp)
    g = torch.Generator().manual_seed(0)
    # permuting the tokens inside every chunk changes nothing
    perm = torch.randperm(p.L, generator=g)
    inp2 = generate(p, seed=17)
    inp2.Ks, inp2.Vs = inp.Ks[:, :, perm].contiguous(), inp.Vs[:, :, perm].contiguous()
    st2 = oracle.decode_step(inp2)
    assert torch.equal(st.ids, st2.ids)
    np.testing.assert_allclose(st2.O.numpy(), st.O.numpy(), rtol=1e-12, atol=1e-14)
    # relabelling the chunks (store and embeddings together) relabels ids, same output
    cp = torch.randperm(p.C, generator=g)
    inp3 = generate(p, seed=17)
    inp3.Ks, inp3.Vs, inp3.E = inp.Ks[cp].contiguous(), inp.Vs[cp].contiguous(), inp.E[:, cp].contiguous()
    st3 = oracle.decode_step(inp3)
    assert torch.equal(torch.sort(cp[st3.ids.long()], dim=-1).values, torch.sort(st.ids.long(), dim=-1).values)
    np.testing.assert_allclose(st3.O.numpy(), st.O.numpy(), rtol=1e-12, atol=1e-14)
    # permuting the requests permutes the outputs
    bp = torch.randperm(p.B, generator=g)
    inp4 = generate(p, seed=17)
    inp4.Q, inp4.Ku, inp4.Vu = inp.Q[bp].contiguous(), inp.Ku[bp].contiguous(), inp.Vu[bp].contiguous()
    st4 = oracle.decode_step(inp4)
    np.testing.assert_allclose(st4.O.numpy(), st.O[bp].numpy(), rtol=1e-12, atol=1e-14)


def test_config0_shapes_and_self_consistency():
    inp = generate(config(0))
    st = oracle.decode_step(inp)
    p = inp.prob
    assert st.ids.shape == (p.B, p.Hkv, p.k) and st.part_O.shape == (p.B, p.Hq, p.k + 1, p.D)
    np.testing.assert_allclose(st.O.numpy(), st.O_direct.numpy(), rtol=1e-12, atol=1e-14)
    O, LSE = dense_reference(inp, st.ids)
    np.testing.assert_allclose(st.O.numpy(), O, rtol=1e-12, atol=1e-14)


def read_config0_golden():
    ids, O, LSE = {}, {}, {}
    for line in open(os.path.join(GOLDEN, "config0_oracle.txt")):
        f = line.split("#")[0].split()
        if not f:
            continue
        tgt = {"ids": ids, "O": O, "LSE": LSE}[f[0]]
        tgt[int(f[1])] = [float(x) for x in f[2:]]
    return ids, O, LSE


def test_config0_matches_stored_oracle_values():
    # regression pin: the oracle (and the generator) still produce the stored configuration-0 values
    ids, O, LSE = read_config0_golden()
    st = oracle.decode_step(generate(config(0), seed=20251106))
    for b in range(8):
        assert [int(c) for c in st.ids[b, 0]] == [int(c) for c in ids[b]]
        np.testing.assert_allclose(st.O_direct[b, 0, :8].numpy(), O[b], rtol=1e-12, atol=1e-15)
        np.testing.assert_allclose(st.LSE_direct[b].numpy(), LSE[b], rtol=1e-13)


# ------------------------------------------------------------------ offline cache construction

def test_quantize_fp8_matches_torch_conversion():
    # library rounding (torch float8_e4m3fn, round to nearest even) on a dense sweep of values,
    # ties, subnormals and the saturation edge; the block's amax is 448 so its scale is exactly 1
    x = torch.cat([torch.linspace(-448, 448, 100001), torch.randn(50000) * 0.01,
                   torch.tensor([2.0 ** -10, 2.0 ** -9, 1.5 * 2.0 ** -10, 2.0 ** -10 * 1.0001, 0.0, -0.0, 447.9,
                                 448.0, 0.0175, 0.0185, 13.0, 15.0, 17.0, 0.0009765625 * 3])])
    n = (x.numel() + 15) // 16 * 16
    xx = torch.zeros(n)
    xx[:x.numel()] = x
    xx = xx.to(torch.bfloat16)
    p = Problem(B=1, Hq=1, Hkv=1, D=16, C=1, L=n // 16, k=1, U=0, q_dtype="bf16", kv_dtype="fp8")
    X8, sc = oracle.quantize_fp8(p, xx.reshape(1, 1, p.L, 16))
    assert sc.item() == 1.0
    want = xx.float().clamp(-448, 448).to(torch.float8_e4m3fn)
    assert torch.equal(X8.view(torch.uint8).flatten(), want.view(torch.uint8))


def test_quantize_fp8_scales_and_roundtrip():
    p = small(q_dtype="bf16", kv_dtype="fp8", D=16, C=3, L=40)
    g = torch.Generator().manual_seed(21)
    X = (torch.randn(p.C, p.Hkv, p.L, p.D, generator=g) * torch.tensor([0.01, 1.0, 300.0]).view(3, 1, 1, 1)).to(torch.bfloat16)
    X8, sc = oracle.quantize_fp8(p, X)
    amax = X.float().abs().amax(dim=(2, 3))
    assert torch.equal(sc, amax / 448.0)
    want = (X.float() / sc[:, :, None, None]).clamp(-448, 448).to(torch.float8_e4m3fn)
    assert torch.equal(X8.view(torch.uint8), want.view(torch.uint8))
    back = X8.float() * sc[:, :, None, None]
    assert ((back - X.float()).abs() <= amax[:, :, None, None] * 2.0 ** -4 + 1e-12).all()   # half an ulp at the top binade


def test_quantize_fp8_all_zero_block_gets_the_floor_scale():
    # a block of zeros (positive and negative) has amax 0: its scale is the floor 1e-30 in f32, every
    # byte encodes a zero (the sign bit may survive, the magnitude bits may not), and the block
    # decodes to exact zeros; its neighbour is quantised as usual
    p = small(q_dtype="bf16", kv_dtype="fp8", D=16, C=2, L=24, Hkv=1, Hq=1)
    g = torch.Generator().manual_seed(22)
    X = torch.randn(p.C, p.Hkv, p.L, p.D, generator=g).to(torch.bfloat16)
    X[0] = 0.0
    X[0, 0, 3, 5] = -0.0
    X8, sc = oracle.quantize_fp8(p, X)
    assert sc[0, 0].item() == torch.tensor(1e-30, dtype=torch.float32).item()
    assert ((X8[0].view(torch.uint8) & 0x7F) == 0).all()
    assert (oracle.widen(X8[0]) * float(sc[0, 0]) == 0).all()
    amax = X[1].float().abs().max()
    assert sc[1, 0].item() == (amax / 448.0).item()
    want = (X[1].float() / sc[1, 0]).clamp(-448, 448).to(torch.float8_e4m3fn)
    assert torch.equal(X8[1].view(torch.uint8), want.view(torch.uint8))


@pytest.mark.parametrize("dt,kv", [("f32", "f32"), ("bf16", "bf16"), ("bf16", "fp8")])
def test_chunk_embeddings_are_the_mean_key(dt, kv):
    p = small(q_dtype=dt, kv_dtype=kv, C=4, L=37, D=32)
    inp = generate(p, seed=22)
    E = oracle.chunk_embeddings(p, inp.Ks, inp.scale_k)
    K = f64(inp.Ks)
    if inp.scale_k is not None:
        K = K * f64(inp.scale_k)[:, :, None, None]
    want = torch.tensor(K.mean(axis=2)).permute(1, 0, 2).to(torch.float32).to(inp.E.dtype)
    assert torch.equal(E.view(torch.uint8), want.contiguous().view(torch.uint8))
    # and it is what the generator ships as E
    assert torch.equal(E.view(torch.uint8), inp.E.view(torch.uint8))


# ------------------------------------------------------------------ several query tokens per request

def dense_reference_multi_token(inp, ids):
    """scipy attention of every query token (b,t) and head: routed chunks in full, unique context
    cut at the token's own position (the T new tokens are the last T unique tokens)."""
    p = inp.prob
    Q, Ks, Vs, Ku, Vu = map(f64, (inp.Q, inp.Ks, inp.Vs, inp.Ku, inp.Vu))
    O = np.zeros((p.Bq, p.Hq, p.D))
    LSE = np.full((p.Bq, p.Hq), -np.inf)
    for b in range(p.B):
        for t in range(p.T):
            r = b * p.T + t
            n = max(int(inp.unique_len[b]) - (p.T - 1 - t), 0)
            for hq in range(p.Hq):
                h = hq // p.G
                sel = [int(c) for c in ids[r, h]]
                K = np.concatenate([Ks[c, h] for c in sel] + [Ku[b, h, :n]], axis=0)
                V = np.concatenate([Vs[c, h] for c in sel] + [Vu[b, h, :n]], axis=0)
                z = p.scale * (K @ Q[r, hq])
                O[r, hq] = softmax(z) @ V
                LSE[r, hq] = logsumexp(z)
    return O, LSE


def test_multi_token_direct_matches_scipy_with_causal_unique_context():
    p = small(T=3, B=4, U=9)
    inp = generate(p, seed=41, unique_len="ragged")     # includes unique_len 0 (< T-1) and U
    inp.unique_len[2] = 1                                # shorter than the T-1 tokens before the last one
    st = oracle.decode_step(inp)
    assert st.ids.shape == (p.B * p.T, p.Hkv, p.k)
    O, LSE = dense_reference_multi_token(inp, st.ids)
    np.testing.assert_allclose(st.O_direct.numpy(), O, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(st.LSE_direct.numpy(), LSE, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(st.O.numpy(), O, rtol=1e-10, atol=1e-12)       # merged partials


def test_multi_token_rows_equal_single_token_problems():
    # token t of request b == a one-token request with that query and the unique context cut there
    p = small(T=4, B=3, U=12, k=2)
    inp = generate(p, seed=42)
    inp.unique_len[:] = torch.tensor([12, 7, 2], dtype=torch.int32)
    st = oracle.decode_step(inp)
    p1 = p.with_(T=1, B=1)
    for b in range(p.B):
        for t in range(p.T):
            r = b * p.T + t
            one = generate(p1, seed=42)
            one.Q, one.E, one.Ks, one.Vs = inp.Q[r:r + 1].contiguous(), inp.E, inp.Ks, inp.Vs
            one.Ku, one.Vu = inp.Ku[b:b + 1].contiguous(), inp.Vu[b:b + 1].contiguous()
            one.unique_len = torch.tensor([max(int(inp.unique_len[b]) - (p.T - 1 - t), 0)], dtype=torch.int32)
            s1 = oracle.decode_step(one)
            assert torch.equal(s1.ids[0], st.ids[r])
            np.testing.assert_allclose(st.part_O[r].numpy(), s1.part_O[0].numpy(), rtol=0, atol=0)
            np.testing.assert_allclose(st.part_LSE[r].numpy(), s1.part_LSE[0].numpy(), rtol=0, atol=0)
            np.testing.assert_allclose(st.O_direct[r].numpy(), s1.O_direct[0].numpy(), rtol=0, atol=0)


def test_multi_token_bucket_items_are_token_major():
    p = small(T=2, B=3)
    inp = generate(p, seed=43)
    ids, _ = oracle.route(p, inp.Q, inp.E)
    off, items = oracle.bucket(p, ids)
    assert off[-1] == p.B * p.T * p.Hkv * p.k
    flat = ids.numpy()
    for h in range(p.Hkv):
        chunk_of_item = flat[:, h, :].reshape(-1)                       # item = (b*T + t)*k + j
        order = np.argsort(chunk_of_item, kind="stable")
        want = order.astype(np.int32)
        got = items[off[h * p.C]:off[(h + 1) * p.C]].numpy()
        assert np.array_equal(got, want)
