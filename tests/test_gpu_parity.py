"""GPU-vs-oracle parity through the C interface (needs an MI355X; run with -m gpu)."""
import math

import pytest
import torch

import oracle
import paper_2511_06010_amd as moska
from moska_inputs import Problem, config, generate
from parity import (assert_lse_close, assert_vectors_close, check_against_oracle, check_route, gpu_pipeline, stratified_tokens,
                    sub_inputs, tol_key)

pytestmark = pytest.mark.gpu


def P(**kw):
    base = dict(B=8, Hq=8, Hkv=2, D=128, C=8, L=256, k=2, U=128, q_dtype="bf16", kv_dtype="bf16")
    base.update(kw)
    return Problem(**base)


SMALL = {
    # the fp32 configuration (vector-ALU path), and variants of it
    "cfg0": config(0),
    "f32-ragged-odd": P(q_dtype="f32", kv_dtype="f32", B=7, Hq=6, Hkv=3, D=64, C=5, L=100, k=2, U=77),
    "f32-d128-k1": P(q_dtype="f32", kv_dtype="f32", B=5, Hq=4, Hkv=4, D=128, C=3, L=65, k=1, U=9),
    "f32-k-eq-C": P(q_dtype="f32", kv_dtype="f32", B=6, Hq=4, Hkv=2, D=32, C=4, L=130, k=4, U=64),
    # bf16 on the MFMA path: several tiles, ragged tails, row counts off the tile size
    "bf16-base": P(),
    "bf16-ragged": P(B=37, Hq=16, Hkv=4, C=12, L=200, k=3, U=150),
    "bf16-long-chunk": P(B=9, Hq=8, Hkv=2, C=3, L=1100, k=2, U=1000),
    "bf16-hot-bucket": P(B=96, Hq=8, Hkv=2, C=2, L=160, k=1, U=40),      # ~190 rows per bucket
    "bf16-g1": P(B=20, Hq=4, Hkv=4, C=6, L=96, k=2, U=33),
    "bf16-g8": P(B=11, Hq=16, Hkv=2, C=6, L=96, k=3, U=70),
    "bf16-g16-k-eq-C": P(B=3, Hq=16, Hkv=1, C=4, L=64, k=4, U=31),
    "bf16-u0": P(B=6, U=0),
    "bf16-tiny-L": P(B=6, L=5, U=3),
    "bf16-scale": P(B=10, scale=0.37),
    # few (request, KV head) pairs and a long unique context: the context is split over workgroups
    "bf16-split-unique": P(B=2, Hq=8, Hkv=2, C=4, L=64, k=2, U=3000),
    "bf16-split-unique-ragged": P(B=3, Hq=16, Hkv=2, C=4, L=64, k=1, U=2500),
    # few buckets of long chunks: every chunk is split over workgroups (all tile classes)
    "bf16-split-shared": P(B=12, Hq=8, Hkv=2, C=4, L=2500, k=2, U=40),
    "bf16-split-shared-hot": P(B=200, Hq=16, Hkv=2, C=2, L=1536, k=1, U=16),
    "fp8-split-shared": P(kv_dtype="fp8", B=40, Hq=16, Hkv=2, C=3, L=1100, k=2, U=30),
    # several query tokens per request: token t sees the unique context up to its own position
    "bf16-t3-ragged": P(T=3, B=7, Hq=8, Hkv=2, C=6, L=100, k=2, U=90),
    "bf16-t8-g4": P(T=8, B=5, Hq=16, Hkv=4, C=6, L=96, k=2, U=200),                # 32 rows per (request, KV head)
    "bf16-t5-g8-ragged": P(T=5, B=3, Hq=16, Hkv=2, C=5, L=64, k=2, U=150),         # 40 rows: the 64-row kernel
    "bf16-t40": P(T=40, B=2, Hq=4, Hkv=2, C=5, L=64, k=2, U=130),                  # two row tiles, two masked key tiles
    "bf16-t2-split-unique-ragged": P(T=2, B=2, Hq=8, Hkv=2, C=4, L=64, k=2, U=3000),
    "fp8-t4": P(kv_dtype="fp8", T=4, B=6, Hq=16, Hkv=2, C=4, L=128, k=2, U=70),
    "f32-t3-ragged": P(q_dtype="f32", kv_dtype="f32", T=3, B=4, Hq=6, Hkv=3, D=64, C=5, L=60, k=2, U=50),
    # degenerate sizes: one request, one head, one chunk of one token, one unique token
    "bf16-single": P(B=1, Hq=1, Hkv=1, C=1, L=1, k=1, U=1),
    "f32-single": P(q_dtype="f32", kv_dtype="f32", B=1, Hq=1, Hkv=1, D=16, C=1, L=1, k=1, U=1),
    "fp8-single-request": P(kv_dtype="fp8", B=1, Hq=8, Hkv=2, C=3, L=33, k=2, U=7),
    # more (KV head, chunk) buckets than the tile-list kernel stages in LDS (16 384 > 15 360), most of them empty
    "bf16-many-buckets": P(B=40, Hq=16, Hkv=8, C=2048, L=32, k=3, U=40),
    # head sizes 256 (widest matrix-core routing kernel) and 48 (vector-ALU routing kernel)
    "bf16-d256": P(D=256, B=19, Hq=8, Hkv=2, C=21, L=70, k=3, U=20),
    "f32-d256": P(q_dtype="f32", kv_dtype="f32", D=256, B=5, Hq=4, Hkv=2, C=18, L=40, k=2, U=10),
    "bf16-d48": P(D=48, B=7, Hq=4, Hkv=2, C=10, L=50, k=2, U=12),
    # bf16 with a head size the MFMA kernels do not cover (vector-ALU path)
    "bf16-d64": P(D=64, B=10, L=150, U=90),
    # thousands of chunks and a large k (the paper's 75 % sparsity): routing by sorting, hundreds of partial slots
    "bf16-route-sort-1500": P(B=6, Hq=8, Hkv=2, C=1500, L=6, k=300, U=10),
    "fp8-route-sort-4096": P(kv_dtype="fp8", B=3, Hq=8, Hkv=2, C=4096, L=3, k=1024, U=5),
    # thousands of buckets: the small tiles go two to a workgroup, in one launch with the 256-row tiles
    # (light bf16 tiles; an fp8 store whose rows sit mostly in large buckets, skewed popularity)
    "bf16-paired-light": P(B=256, Hq=8, Hkv=2, C=1024, L=70, k=8, U=8, popularity="zipf", zipf_s=1.1),
    "fp8-paired-remainders": P(kv_dtype="fp8", B=512, Hq=8, Hkv=2, C=512, L=40, k=32, U=4, popularity="zipf", zipf_s=1.1),
    # thousands of buckets of an fp8 store with under 128 rows each on average: the tiles of up to 64 rows run
    # three workgroups to a compute unit in a launch of their own, the 128- and 256-row tiles in two more
    "fp8-light-many-buckets": P(kv_dtype="fp8", B=400, Hq=8, Hkv=2, C=512, L=70, k=8, U=5, popularity="zipf", zipf_s=1.1),
    # fp8 shared store
    "fp8-base": P(kv_dtype="fp8", B=24, Hq=16, Hkv=2, C=6, L=300, k=2, U=100),
    "fp8-hot": P(kv_dtype="fp8", B=80, Hq=16, Hkv=2, C=2, L=128, k=1, U=16),
    "fp8-d64": P(kv_dtype="fp8", D=64, B=9, L=70, U=20),
}


@pytest.mark.parametrize("name", list(SMALL))
def test_small_problem_matches_oracle(name):
    p = SMALL[name]
    ragged = "ragged" if ("ragged" in name or "odd" in name) else "full"
    print(f"case {name}: {p}", flush=True)
    check_against_oracle(generate(p, seed=101, unique_len=ragged), name)


def _random_problem(rng):
    """A small problem with sizes drawn around the tile, stage and group boundaries of the kernels."""
    dt = rng.choice(["bf16", "bf16", "fp8", "f32"])
    G, Hkv = rng.choice([1, 2, 3, 4, 6, 8, 16]), rng.choice([1, 2, 3, 4, 8])
    D = 128 if dt != "f32" else rng.choice([16, 32, 64, 128])
    if dt == "bf16" and rng.random() < 0.15:
        D = rng.choice([48, 64, 256])
    C = rng.choice([1, 2, 3, 5, 8, 17, 40])
    k = rng.randint(1, min(C, 5))
    L = rng.choice([1, 7, 31, 32, 33, 64, 100, 129, 300, 1100, 2500])
    U = rng.choice([0, 1, 5, 33, 64, 150, 700])
    T = rng.choice([1, 1, 1, 2, 3, 5])
    B = rng.choice([1, 2, 3, 9, 30, 70, 150, 400])
    if dt == "f32":
        B, L, U = min(B, 9), min(L, 300), min(U, 150)
    while B * T * G * Hkv * (k * L + U) * D > 1.5e9 and B > 1:       # keeps the oracle to well under a second
        B = max(1, B // 2)
    return Problem(B=B, Hq=G * Hkv, Hkv=Hkv, D=D, C=C, L=L, k=k, U=max(U, T if U else 0), T=T,
                   q_dtype="f32" if dt == "f32" else "bf16", kv_dtype=dt,
                   popularity=rng.choice(["uniform", "zipf"]), zipf_s=1.5, scale=rng.choice([1.0, 1.0, 0.5]))


def test_random_small_problems():
    # 80 seeded random shapes (dtypes, group sizes, head sizes, ragged contexts, several tokens per
    # request, skewed popularity): every one against the oracle
    import random
    rng = random.Random(20251106)
    for i in range(80):
        p = _random_problem(rng)
        ragged = rng.choice(["full", "ragged"])
        print(f"random case {i}: {p} {ragged}", flush=True)
        check_against_oracle(generate(p, seed=3000 + i, unique_len=ragged), f"random{i}")


def test_random_problems_with_paired_small_tiles():
    # seeded random shapes with thousands of buckets, where the small tiles of shared attention go two to a
    # workgroup in the launch of the 256-row tiles: light bf16 tiles, and fp8 stores whose rows sit mostly in
    # large buckets; short chunks keep the oracle fast
    import random
    rng = random.Random(77)
    for i in range(8):
        fp8 = i % 2 == 1
        Hkv, G = rng.choice([(2, 4), (4, 2), (8, 1), (2, 8)])
        C = rng.choice([512, 700, 1024]) if not fp8 else rng.choice([128, 256, 512])
        while Hkv * C < 1024:
            C *= 2
        L = rng.choice([33, 64, 70, 130])
        if fp8:                                   # expected rows per bucket B*k*G/C >= 128
            k = rng.choice([8, 16, 32])
            B = -(-128 * C // (k * G)) + rng.randint(0, 40)
        else:                                     # <= 48
            k = rng.choice([4, 8])
            B = max(1024 // (Hkv * k) + 1, min(2000, rng.choice([12, 25, 40]) * C // (k * G)))
        p = P(kv_dtype="fp8" if fp8 else "bf16", B=B, Hq=Hkv * G, Hkv=Hkv, C=C, L=L, k=k, U=rng.choice([0, 5, 40]),
              popularity=rng.choice(["uniform", "zipf"]), zipf_s=1.2)
        assert min(p.B * p.Hkv * p.k, p.Hkv * p.C) >= 1024
        print(f"paired case {i}: {p}", flush=True)
        check_against_oracle(generate(p, seed=4000 + i, unique_len="ragged"), f"paired{i}")


def test_config0_matches_stored_oracle_values():
    # expected values stored by tests/golden/make_config0_golden.py (oracle only)
    from test_oracle_pins import read_config0_golden
    ids, O, LSE = read_config0_golden()
    buf = gpu_pipeline(generate(config(0), seed=20251106).to("cuda"))
    for b in range(8):
        assert buf.ids[b, 0].tolist() == [int(c) for c in ids[b]]
        want = torch.tensor(O[b], dtype=torch.float64)
        got = buf.O[b, 0, :8].double().cpu()
        assert (got - want).abs().max() <= 1e-5 * want.abs().max()
        torch.testing.assert_close(buf.LSE[b].double().cpu(), torch.tensor(LSE[b], dtype=torch.float64), rtol=1e-5, atol=1e-5)


def test_zipf_popularity_and_empty_buckets():
    # strongly skewed targets: one very hot bucket, many buckets that receive nothing
    p = P(B=64, Hq=8, Hkv=2, C=40, L=96, k=2, U=50, popularity="zipf", zipf_s=2.0)
    inp = generate(p, seed=5)
    buf, st = check_against_oracle(inp, "zipf")
    sizes = (st.bucket_off[1:] - st.bucket_off[:-1])
    assert (sizes == 0).any() and sizes.max() >= 12


def test_batching_invariance():
    # Sec. III-A: batching the queries of a bucket into one matrix must not change any row --
    # a request processed alone gives the same partial as in the batch.  The two runs use
    # different tile kernels (their running softmax maxima differ, and with them the bf16
    # rounding of the probabilities), so they agree to bf16 level, not bit for bit.
    p = P(B=32, C=2, k=1, L=192, U=16)
    cpu_inp = generate(p, seed=7)
    inp = cpu_inp.to("cuda")
    full = gpu_pipeline(inp)
    st = oracle.decode_step(cpu_inp, ids=full.ids.cpu())      # both runs are also held against the oracle
    assert_vectors_close(full.part_O, st.part_O, "bf16", "batched part_O")
    assert_lse_close(full.part_LSE, st.part_LSE, "bf16", "batched part_LSE")
    for b in (0, 5, 31):
        one = generate(p.with_(B=1), seed=7).to("cuda")
        one.Q, one.Ku, one.Vu = inp.Q[b:b + 1].contiguous(), inp.Ku[b:b + 1].contiguous(), inp.Vu[b:b + 1].contiguous()
        one.E, one.Ks, one.Vs, one.unique_len = inp.E, inp.Ks, inp.Vs, inp.unique_len[b:b + 1].contiguous()
        solo = gpu_pipeline(one)
        assert torch.equal(solo.ids[0], full.ids[b])
        assert_vectors_close(solo.part_O[0], st.part_O[b], "bf16", f"request {b} alone, part_O")
        assert_lse_close(solo.part_LSE[0], st.part_LSE[b], "bf16", f"request {b} alone, part_LSE")
        torch.testing.assert_close(solo.part_O[0], full.part_O[b], rtol=0, atol=3e-3)
        torch.testing.assert_close(solo.part_LSE[0], full.part_LSE[b], rtol=0, atol=1e-4)


def test_run_twice_is_bit_identical():
    p = P(B=40, Hq=16, Hkv=4, C=10, L=300, k=3, U=200)
    inp = generate(p, seed=9, unique_len="ragged").to("cuda")
    a, b = gpu_pipeline(inp), gpu_pipeline(inp)
    for name in ("ids", "bucket_off", "bucket_items", "part_O", "part_LSE", "O", "LSE"):
        x, y = getattr(a, name), getattr(b, name)
        assert torch.equal(x.view(torch.uint8), y.view(torch.uint8)), name


def test_route_ties_and_zero_query():
    p = P(B=6, C=9, k=4)
    inp = generate(p, seed=11)
    inp.E[:, 7] = inp.E[:, 2]                       # exact ties: lower chunk id first
    inp.E[:, 8] = inp.E[:, 2]
    inp.Q[0] = 0                                    # all scores equal: ids 0..k-1
    o_ids, _, o_all = oracle.route(p, inp.Q, inp.E, want_all_scores=True)
    d = inp.to("cuda")
    ids = torch.empty_like(o_ids, device="cuda")
    moska.route(p, d.Q, d.E, ids, None, moska.Buffers(p).ws)
    torch.cuda.synchronize()
    assert torch.equal(ids.cpu(), o_ids)
    assert ids[0].cpu().tolist() == [[0, 1, 2, 3]] * p.Hkv


def test_bucket_handles_many_items_per_wave_slice():
    p = P(B=700, Hq=4, Hkv=2, C=37, k=5, L=16, U=0, D=64)
    g = torch.Generator().manual_seed(3)
    ids = torch.stack([torch.stack([torch.randperm(p.C, generator=g)[:p.k] for _ in range(p.Hkv)])
                       for _ in range(p.B)]).to(torch.int32)
    off, items = oracle.bucket(p, ids)
    buf = moska.Buffers(p)
    moska.bucket(p, ids.cuda(), buf.bucket_off, buf.bucket_items, buf.ws)
    torch.cuda.synchronize()
    assert torch.equal(buf.bucket_off.cpu(), off) and torch.equal(buf.bucket_items.cpu(), items)


def test_bucket_over_several_workgroups_per_head():
    # 42 000 items per KV head: the head is bucketed by several workgroups (count, scan, scatter)
    p = P(B=700, Hq=6, Hkv=3, C=300, k=60, L=16, U=0, D=64)
    g = torch.Generator().manual_seed(4)
    ids = torch.stack([torch.stack([torch.randperm(p.C, generator=g)[:p.k] for _ in range(p.Hkv)])
                       for _ in range(p.B)]).to(torch.int32)
    ids[:, 1, :] = ids[:, 1, :] % 7                  # a head whose items crowd into seven buckets (repeated ids)
    off, items = oracle.bucket(p, ids)
    buf = moska.Buffers(p)
    moska.bucket(p, ids.cuda(), buf.bucket_off, buf.bucket_items, buf.ws)
    torch.cuda.synchronize()
    assert torch.equal(buf.bucket_off.cpu(), off) and torch.equal(buf.bucket_items.cpu(), items)


def test_repeated_chunk_ids_fill_every_slot():
    # ids chosen by the caller may name a chunk twice for one (request, KV head): both slots are work
    # items of the same bucket (a bucket then holds more rows than there are requests x group heads)
    # and both must come out as that chunk's partial
    p = P(B=5, Hq=8, Hkv=2, C=3, L=70, k=3, U=20)
    inp = generate(p, seed=13)
    ids = torch.tensor([[0, 0, 0], [1, 1, 2]], dtype=torch.int32).repeat(p.B, 1, 1).contiguous()   # [B,Hkv,k]
    want_O, want_L = oracle.partials(inp, ids)
    d = inp.to("cuda")
    buf = moska.Buffers(p)
    buf.part_O.fill_(float("nan"))
    buf.part_LSE.fill_(float("nan"))
    moska.bucket(p, ids.cuda(), buf.bucket_off, buf.bucket_items, buf.ws)
    off, items = oracle.bucket(p, ids)
    moska.shared_attn(p, d.Q, d.Ks, d.Vs, None, None, ids.cuda(), buf.bucket_off, buf.bucket_items, buf.part_O,
                      buf.part_LSE, buf.ws)
    torch.cuda.synchronize()
    assert torch.equal(buf.bucket_off.cpu(), off) and torch.equal(buf.bucket_items.cpu(), items)
    assert_vectors_close(buf.part_O[:, :, :p.k], want_O[:, :, :p.k], "bf16", "repeated ids part_O")
    assert_lse_close(buf.part_LSE[:, :, :p.k], want_L[:, :, :p.k], "bf16", "repeated ids part_LSE")


def test_merge_many_slots():
    # hundreds of partial slots: the workgroup-per-row merge, with empty slots and an all-empty row
    p = P(B=3, Hq=4, Hkv=2, C=400, k=300, D=128)
    g = torch.Generator().manual_seed(6)
    pO = torch.randn(p.B, p.Hq, p.k + 1, p.D, generator=g)
    pL = torch.randn(p.B, p.Hq, p.k + 1, generator=g) * 3
    pL[0, :, 5::7] = -math.inf
    pL[1, 2] = -math.inf
    pO[1, 2] = float("nan")
    want_O, want_L = oracle.merge(torch.nan_to_num(pO), pL)
    O = torch.empty(p.B, p.Hq, p.D, dtype=torch.bfloat16, device="cuda")
    LSE = torch.empty(p.B, p.Hq, device="cuda")
    moska.merge(p, pO.cuda(), pL.cuda(), O, LSE)
    torch.cuda.synchronize()
    assert (O[1, 2] == 0).all() and torch.isinf(LSE[1, 2])
    torch.testing.assert_close(O.cpu().double(), want_O, rtol=0, atol=2e-2)
    assert ((O.cpu().double() - want_O).norm() / want_O.norm()) < 5e-3
    torch.testing.assert_close(LSE.cpu().double(), want_L, rtol=0, atol=1e-5)


def test_merge_empty_slots():
    p = P(B=3, Hq=4, Hkv=2, k=2, D=64)
    pO = torch.randn(p.B, p.Hq, 3, p.D)
    pL = torch.randn(p.B, p.Hq, 3)
    pL[0, :, 1] = -math.inf                          # one empty slot
    pL[1] = -math.inf                                # a row with nothing at all
    pO[1] = float("nan")                             # empty slots' O must never be read
    want_O, want_L = oracle.merge(pO[[0, 2]], pL[[0, 2]])
    O = torch.empty(p.B, p.Hq, p.D, dtype=torch.bfloat16, device="cuda")
    LSE = torch.empty(p.B, p.Hq, device="cuda")
    moska.merge(p, pO.cuda(), pL.cuda(), O, LSE)
    torch.cuda.synchronize()
    assert (O[1] == 0).all() and torch.isinf(LSE[1]).all()
    torch.testing.assert_close(O[[0, 2]].cpu().double(), want_O, rtol=0, atol=2e-2)
    torch.testing.assert_close(LSE[[0, 2]].cpu().double(), want_L, rtol=0, atol=1e-5)


@pytest.mark.parametrize("dt,kv,D", [("f32", "f32", 64), ("bf16", "bf16", 128), ("bf16", "fp8", 128), ("bf16", "bf16", 48)])
def test_chunk_embeddings_match_oracle(dt, kv, D):
    p = P(q_dtype=dt, kv_dtype=kv, D=D, C=5, L=333, Hkv=3, Hq=6)
    inp = generate(p, seed=31)
    want = oracle.chunk_embeddings(p, inp.Ks, inp.scale_k)
    d = inp.to("cuda")
    E = torch.empty_like(d.E)
    moska.chunk_embeddings(p, d.Ks, d.scale_k, E)
    torch.cuda.synchronize()
    assert torch.equal(E.cpu().view(torch.uint8), want.view(torch.uint8))


def test_quantize_shared_matches_oracle_bit_for_bit():
    p = P(kv_dtype="fp8", C=6, L=100, Hkv=2)
    g = torch.Generator().manual_seed(32)
    mag = torch.tensor([1e-3, 0.05, 1.0, 7.0, 300.0, 0.0]).view(6, 1, 1, 1)
    X = (torch.randn(p.C, p.Hkv, p.L, p.D, generator=g) * mag).to(torch.bfloat16)
    want8, want_s = oracle.quantize_fp8(p, X)
    X8 = torch.empty(X.shape, dtype=torch.float8_e4m3fn, device="cuda")
    sc = torch.empty(p.C, p.Hkv, device="cuda")
    moska.quantize_shared(p, X.cuda(), X8, sc)
    torch.cuda.synchronize()
    assert torch.equal(sc.cpu(), want_s)
    assert torch.equal(X8.cpu().view(torch.uint8), want8.view(torch.uint8))


def test_decode_step_replays_from_a_hip_graph():
    # the five stages captured once and replayed: no call allocates, synchronises or records a
    # memset, so a replay must give the bits of an eager run -- also after the inputs changed
    p = P(B=24, Hq=16, Hkv=4, C=12, L=300, k=3, U=260)
    inp = generate(p, seed=31).to("cuda")
    other = generate(p, seed=32).to("cuda")
    buf = moska.Buffers(p)

    def step():
        moska.decode_step(p, inp.Q, inp.E, inp.Ks, inp.Vs, inp.scale_k, inp.scale_v, inp.Ku, inp.Vu, inp.unique_len,
                          buf.ids, buf.bucket_off, buf.bucket_items, buf.part_O, buf.part_LSE, buf.O, buf.LSE, buf.ws)

    def eager_bits():
        step()
        torch.cuda.synchronize()
        return buf.O.view(torch.uint8).clone(), buf.ids.clone()

    want = {0: eager_bits()}
    # the eager result the replays are compared with is itself held against the oracle
    st = oracle.decode_step(generate(p, seed=31), ids=want[0][1].cpu())
    assert_vectors_close(buf.O, st.O_direct, "bf16", "eager decode_step O")
    saved_q = inp.Q.clone()
    inp.Q.copy_(other.Q)
    want[1] = eager_bits()
    inp.Q.copy_(saved_q)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                        # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for which in (0, 1, 0, 1):
        inp.Q.copy_(other.Q if which else saved_q)      # eager work between the replays
        buf.O.zero_()
        buf.part_O.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(buf.O.view(torch.uint8), want[which][0]), f"replay with inputs {which}"
        assert torch.equal(buf.ids, want[which][1])


def test_invalid_arguments_are_rejected_before_launch():
    p = P()
    buf = moska.Buffers(p)
    inp = generate(p, seed=1).to("cuda")
    with pytest.raises(moska.MoskaError, match="invalid"):
        moska.route(p.with_(k=9), inp.Q, inp.E, torch.empty(p.B, p.Hkv, 9, dtype=torch.int32, device="cuda"), None,
                    buf.ws)
    with pytest.raises(moska.MoskaError, match="workspace"):
        moska.route(p, inp.Q, inp.E, buf.ids, None, buf.ws[:16])
    with pytest.raises(moska.MoskaError, match="unsupported"):
        moska.workspace_bytes(p.with_(D=72))
    with pytest.raises(moska.MoskaError, match="invalid"):
        moska.workspace_bytes(p.with_(T=-1))
    assert moska.workspace_bytes(p.with_(T=0)) == moska.workspace_bytes(p)       # q_len 0 reads as 1
    with pytest.raises(moska.MoskaError, match="workspace"):
        moska.bucket(p, buf.ids, buf.bucket_off, buf.bucket_items, buf.ws[:16])
    with pytest.raises(moska.MoskaError, match="invalid"):       # fp8 store without scales
        q = p.with_(kv_dtype="fp8")
        k8 = torch.zeros(p.C, p.Hkv, p.L, p.D, dtype=torch.uint8, device="cuda").view(torch.float8_e4m3fn)
        moska.shared_attn(q, inp.Q, k8, k8, None, None, buf.ids, buf.bucket_off, buf.bucket_items, buf.part_O,
                          buf.part_LSE, buf.ws)
    torch.cuda.synchronize()


# ---------------------------------------------------------------- full benchmark sizes

def _full_size_check(p, seed: int, n_tokens: int = 64, heads_per_token=None, ragged: bool = False, label: str = ""):
    """Routing and bucketing verified for every item; attention on a popularity-stratified sample of
    query tokens -- every KV head (or the first heads_per_token, where one token's chunks are
    gigabytes), all G heads of the group, all k+1 partials and the merged row -- that the oracle
    computes one token at a time from the same bits."""
    label = label or p.name
    print(f"full-size {label}: {p}", flush=True)
    inp = generate(p, seed=seed, device="cuda", unique_len="ragged" if ragged else "full")
    o_ids, _, o_all = oracle.route(p, inp.Q.cpu(), inp.E.cpu(), want_all_scores=True)
    buf = gpu_pipeline(inp)
    excused = check_route(p, buf.routed_ids, o_ids, o_all)
    print(f"  route ok ({excused} tie-excused pairs)", flush=True)
    del o_all
    if excused:
        buf = gpu_pipeline(inp, ids_override=o_ids.cuda())
    off, items = oracle.bucket(p, o_ids)
    assert torch.equal(buf.bucket_off.cpu(), off) and torch.equal(buf.bucket_items.cpu(), items)
    toks = stratified_tokens(p, off, items, n_tokens, seed)
    if p.T > 1:                   # the first and the last token of the requests with an empty and a full context
        toks = list(dict.fromkeys([0, p.T - 1, p.T, 2 * p.T - 1] + toks))
    key = tol_key(p)
    G = p.G
    heads = None if heads_per_token is None else list(range(heads_per_token))
    rows = slice(None) if heads is None else slice(0, heads_per_token * G)
    got = {n: [] for n in ("part_O", "part_LSE", "O", "LSE")}
    want = {n: [] for n in got}
    for i, b in enumerate(toks):
        sub, sub_ids = sub_inputs(inp, o_ids, b, heads)
        st = oracle.decode_step(sub, ids=sub_ids)
        for n, w in (("part_O", st.part_O), ("part_LSE", st.part_LSE), ("O", st.O_direct), ("LSE", st.LSE_direct)):
            got[n].append(getattr(buf, n)[b, rows].cpu())
            want[n].append(w[0])
        if i % 16 == 15:
            print(f"  oracle done for {i + 1} of {len(toks)} tokens", flush=True)
    for n in got:
        check = assert_vectors_close if n in ("part_O", "O") else assert_lse_close
        check(torch.stack(got[n]), torch.stack(want[n]), key, f"{label} {n}")
    # properties that hold at any size: every slot written, outputs finite, LSE of the merge
    # above every partial LSE
    assert torch.isfinite(buf.part_O).all() and torch.isfinite(buf.part_LSE[..., :p.k]).all()
    assert not torch.isnan(buf.part_LSE).any()           # the unique slot is -inf where a token sees no unique key
    assert (buf.LSE[..., None] >= buf.part_LSE - 1e-3).all()
    sizes = off[1:] - off[:-1]
    print(f"  attention ok on {len(toks)} sampled query tokens x {p.Hkv if heads is None else heads_per_token} KV heads"
          f" (bucket rows: max {int(sizes.max()) * G}, mean {float(sizes.float().mean()) * G:.0f})", flush=True)
    del inp, buf
    torch.cuda.empty_cache()


def test_config1_full():
    inp = generate(config(1), seed=20251107, device="cuda")
    check_against_oracle(inp.to("cpu"), "cfg1")


@pytest.mark.parametrize("cfg_idx", [2, 3, 4])
def test_full_size_sampled(cfg_idx):
    _full_size_check(config(cfg_idx), 20251106 + cfg_idx)


def test_full_size_sampled_four_tokens_per_request():
    p = config(2)
    _full_size_check(p.with_(T=4, B=p.B // 4, name=p.name + "-qlen4"), 20251108, ragged=True)


# ---------------------------------------------------------------- the paper's operating point
# Sec. IV: FP8 shared store, 75 % routing sparsity (k = C/4), Hq/Hkv = 32/8, batch up to 256.

def test_paper_operating_point_small():
    p = P(kv_dtype="fp8", B=16, Hq=32, Hkv=8, C=64, L=256, k=16, U=300, name="paper-point-small")
    check_against_oracle(generate(p, seed=41, unique_len="ragged"), p.name)


def test_route_by_sorting_ties_and_padding():
    # C between two powers of two (the sort pads), exact ties across the k-th place, an all-zero query
    p = P(B=5, Hq=8, Hkv=2, C=1100, L=2, k=400, U=1)
    inp = generate(p, seed=17)
    inp.E[:, 700:1100] = inp.E[:, 300:700]          # every score of chunks 300..699 appears twice
    inp.Q[0] = 0
    o_ids, _ = oracle.route(p, inp.Q, inp.E)
    d = inp.to("cuda")
    ids = torch.empty_like(o_ids, device="cuda")
    moska.route(p, d.Q, d.E, ids, None, moska.Buffers(p).ws)
    torch.cuda.synchronize()
    assert torch.equal(ids.cpu(), o_ids)
    assert ids[0, 0].cpu().tolist() == list(range(p.k))


@pytest.mark.parametrize("B", [16, 256])
def test_paper_operating_point_full_chunk_length(B):
    p = P(kv_dtype="fp8", B=B, Hq=32, Hkv=8, C=64, L=4096, k=16, U=8192, name=f"paper-point-b{B}")
    _full_size_check(p, 20251106, n_tokens=min(B, 64))


def test_paper_operating_point_16M_shared_tokens():
    # the paper's own shared context: 4096 chunks x 4096 tokens (16M tokens, 34 GB in fp8), top-k = 1024,
    # 64K unique tokens per request; one KV head of each sampled token (its 1024 chunks are 1 GB)
    p = P(kv_dtype="fp8", B=32, Hq=32, Hkv=8, C=4096, L=4096, k=1024, U=65536, name="paper-point-16M-b32")
    _full_size_check(p, 20251106, n_tokens=6, heads_per_token=1)
