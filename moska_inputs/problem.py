"""Problem descriptor and the five workload configurations.

Notation (paper, Sec. III-A/B): B concurrent requests with one query token each,
Hq query heads grouped G = Hq/Hkv to a KV head, head dimension D; the shared KV
space is C chunks ("experts") of L tokens, of which the router keeps the top k per
(request, KV head); every request also owns U tokens of unique KV.

Extension (not in the paper): T = q_len query tokens per request (speculative decoding,
chunked prefill).  Query token (b,t) is row b*T + t of Q, ids, partials and outputs; it is routed on
its own, attends to every token of its routed chunks, and to the request's unique context up to
and including its own position: the T new tokens are the last T of the unique_len[b] unique
tokens, so token t sees the first unique_len[b] - (T-1-t) of them.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
import torch

# dtype codes shared by the oracle's C interface and the HIP library's C interface
DTYPE_CODES = {"f32": 0, "bf16": 1, "fp8": 2}


def torch_dtype(name: str) -> torch.dtype:
    return {"f32": torch.float32, "bf16": torch.bfloat16, "fp8": torch.float8_e4m3fn}[name]


@dataclass(frozen=True)
class Problem:
    B: int
    Hq: int
    Hkv: int
    D: int
    C: int
    L: int
    k: int
    U: int                      # padded unique length U_max
    q_dtype: str = "bf16"       # dtype of Q, E, unique K/V and the final output
    kv_dtype: str = "bf16"      # dtype of the shared K/V store
    scale: float = 1.0          # logit scale (queries of the workloads are pre-scaled)
    popularity: str = "uniform"  # "uniform" or "zipf"
    zipf_s: float = 0.0
    name: str = ""
    T: int = 1                  # query tokens per request (q_len)

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def P(self) -> int:         # partial slots: k shared + 1 unique
        return self.k + 1

    @property
    def Bq(self) -> int:        # query tokens in the step
        return self.B * self.T

    def with_(self, **kw) -> "Problem":
        return replace(self, **kw)


# The five configurations of the benchmark definition (index = config number).
CONFIGS = (
    Problem(B=8, Hq=4, Hkv=1, D=64, C=4, L=256, k=2, U=128,
            q_dtype="f32", kv_dtype="f32", name="cfg0-tiny-f32"),
    Problem(B=64, Hq=32, Hkv=8, D=128, C=32, L=2048, k=4, U=2048,
            name="cfg1-llama8b-64k"),
    Problem(B=256, Hq=32, Hkv=8, D=128, C=256, L=4096, k=8, U=4096,
            name="cfg2-b256-1M"),
    Problem(B=1024, Hq=32, Hkv=8, D=128, C=1024, L=4096, k=16, U=8192,
            popularity="zipf", zipf_s=1.1, name="cfg3-b1024-4M-zipf"),
    Problem(B=2048, Hq=64, Hkv=8, D=128, C=512, L=4096, k=8, U=4096,
            kv_dtype="fp8", popularity="zipf", zipf_s=1.2, name="cfg4-70b-fp8-zipf"),
)


def config(i: int) -> Problem:
    return CONFIGS[i]
