"""The roofline arithmetic of bench.py against figures worked by hand (CPU only): the algorithmic bytes and
flops per call at benchmark configuration 2, and where a bucket passes from the HBM to the MFMA roofline."""
import torch

import bench
from moska_inputs import config


def uniform_buckets(n_buckets, items_each):
    return torch.arange(n_buckets + 1, dtype=torch.int64) * items_each


def test_algorithmic_work_at_config_2():
    p = config(2)                                   # B=256, Hq/Hkv=32/8, D=128, C=256 x L=4096, k=8, U=4096, bf16
    assert (p.B, p.Hq, p.Hkv, p.D, p.C, p.L, p.k, p.U) == (256, 32, 8, 128, 256, 4096, 8, 4096)
    w = bench.algorithmic_work(p, uniform_buckets(2048, 8))          # 16384 items over 2048 buckets
    # every bucket's K and V once (2 MiB), every routed row's query in (256 B) and partial out (516 B)
    assert w["shared_attn"]["bytes"] == 2048 * 2 * 4096 * 128 * 2 + 65536 * (256 + 516) == 4_345_561_088
    assert w["shared_attn"]["flops"] == 4 * 128 * 65536 * 4096 == 137_438_953_472
    # every request's K and V once per KV head, the step's queries in and slot-k partials out
    assert w["unique_attn"]["bytes"] == 2 * 256 * 8 * 4096 * 128 * 2 + 8192 * (256 + 516) == 4_301_291_520
    assert w["unique_attn"]["flops"] == 4 * 128 * 8192 * 4096
    assert w["merge"]["bytes"] == 8192 * (9 * 129 * 4 + 256 + 4)
    # an empty bucket streams nothing
    half = torch.cat([uniform_buckets(1024, 16), torch.full((1024,), 16384, dtype=torch.int64)])
    assert bench.algorithmic_work(p, half)["shared_attn"]["bytes"] == 1024 * 2 * 4096 * 128 * 2 + 65536 * 772


def test_attainable_time_and_the_ridge():
    p = config(2)
    # 32 rows per bucket: bound by the bucket's bytes at 8 TB/s
    t = bench.shared_attainable_s(p, uniform_buckets(2048, 8))
    assert abs(t - 2048 * (2 * 4096 * 128 * 2 + 32 * 772) / 8e12) < 1e-12
    one = lambda rows, q: bench.shared_attainable_s(q, uniform_buckets(1, rows // q.G))
    mem = lambda rows, esz: (2 * 4096 * 128 * esz + rows * 772) / 8e12
    mfma = lambda rows: 4 * 128 * rows * 4096 / 2.5e15
    # bf16 store: K and V alone give 2.5 PFLOP/s over 8 TB/s = 312.5 rows; with the rows' own 772 bytes the
    # ridge lies at 353 rows
    assert abs(one(352, p) - mem(352, 2)) < 1e-15 and mem(352, 2) > mfma(352)
    assert abs(one(356, p) - mfma(356)) < 1e-15 and mfma(356) > mem(356, 2)
    # fp8 store: half the K/V bytes, ridge at 177 rows
    p8 = p.with_(kv_dtype="fp8")
    assert abs(one(176, p8) - mem(176, 1)) < 1e-15 and mem(176, 1) > mfma(176)
    assert abs(one(180, p8) - mfma(180)) < 1e-15 and mfma(180) > mem(180, 1)


def test_peaks_are_the_published_ones():
    assert bench.HBM_PEAK_GBS == 8000.0 and bench.MFMA_BF16_PEAK_TFLOPS == 2500.0
