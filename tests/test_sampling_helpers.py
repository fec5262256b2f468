"""Pins of the helpers that the full-size GPU parity tests lean on (CPU only).

At the benchmark sizes the oracle cannot compute every row, so those tests hand it one query token
at a time as a problem of its own (parity.sub_inputs) and choose the tokens by bucket popularity
(parity.stratified_tokens).  A mistake in either helper would make the full-size checks compare the
GPU with the wrong thing, or with nothing: here the sub-problem's result is held against the rows of
the whole problem's result, both from the oracle, on problems small enough to compute in full.
"""
import numpy as np
import pytest
import torch

import oracle
from moska_inputs import Problem, generate
from parity import stratified_tokens, sub_inputs


def problem(**kw):
    base = dict(B=6, Hq=8, Hkv=2, D=16, C=7, L=9, k=3, U=11, q_dtype="bf16", kv_dtype="bf16")
    base.update(kw)
    return Problem(**base)


@pytest.mark.parametrize("kw", [dict(), dict(kv_dtype="fp8"), dict(T=3, U=12), dict(q_dtype="f32", kv_dtype="f32", Hq=6)],
                         ids=["bf16", "fp8", "three-tokens", "f32"])
@pytest.mark.parametrize("heads", [None, [1], [1, 0]], ids=["all-heads", "one-head", "two-heads-reordered"])
def test_sub_problem_reproduces_the_rows_of_the_whole_problem(kw, heads):
    p = problem(**kw)
    inp = generate(p, seed=77, unique_len="ragged")
    whole = oracle.decode_step(inp)
    G = p.G
    hs = list(range(p.Hkv)) if heads is None else heads
    rows = np.concatenate([np.arange(h * G, (h + 1) * G) for h in hs])
    for b in range(p.Bq):
        sub, sub_ids = sub_inputs(inp, whole.ids, b, heads)
        assert sub.prob.B == 1 and sub.prob.C == p.k and sub.prob.Hkv == len(hs)
        part = oracle.decode_step(sub, ids=sub_ids)
        # slot j of the sub-problem is compact chunk j = the token's j-th routed chunk; slot k the unique context
        np.testing.assert_array_equal(part.part_LSE[0].numpy(), whole.part_LSE[b, rows].numpy())
        np.testing.assert_array_equal(part.part_O[0].numpy(), whole.part_O[b, rows].numpy())
        np.testing.assert_array_equal(part.O_direct[0].numpy(), whole.O_direct[b, rows].numpy())
        np.testing.assert_array_equal(part.LSE_direct[0].numpy(), whole.LSE_direct[b, rows].numpy())
        # and the compact store's routing puts the chunks back in the order they were routed in
        # (their scores are the whole problem's scores of those chunks, already sorted)
        r_ids, _ = oracle.route(sub.prob, sub.Q, sub.E)
        full_ids, _, all_scores = oracle.route(p, inp.Q, inp.E, want_all_scores=True)
        for n, h in enumerate(hs):
            sc = all_scores[b, h, whole.ids[b, h].long()]
            if (sc[:-1] - sc[1:]).min() > 0:                 # strictly decreasing: the order is unique
                assert r_ids[0, n].tolist() == list(range(p.k))


def test_stratified_tokens_reach_the_extreme_buckets_and_are_distinct():
    p = problem(B=40, C=12, k=2, popularity="zipf", zipf_s=1.3)
    inp = generate(p, seed=5)
    st = oracle.decode_step(inp, want_direct=False)
    off, items = st.bucket_off, st.bucket_items
    toks = stratified_tokens(p, off, items, 16, seed=3)
    assert len(toks) == 16 and len(set(toks)) == 16 and all(0 <= t < p.Bq for t in toks)
    sizes = (off[1:] - off[:-1]).numpy()
    hot, cold = int(np.argmax(sizes)), int(np.where(sizes > 0, sizes, sizes.max() + 1).argmin())
    members = lambda bk: {int(i) // p.k for i in items[off[bk]:off[bk + 1]]}
    assert members(hot) & set(toks) and members(cold) & set(toks)
    # asking for more tokens than there are returns every token once
    assert sorted(stratified_tokens(p, off, items, 1000, seed=3)) == list(range(p.Bq))
