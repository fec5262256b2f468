"""ctypes front end of the fp64 CPU oracle (oracle/moska_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the benchmark's
cpu_baseline leg, never by the product package.  Takes torch CPU tensors holding the
stored bits (f32 / bf16 / float8_e4m3fn) and returns fp64 results.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "moska_oracle.c")
_LIB = os.path.join(_HERE, "libmoska_oracle.so")
_DT = {"f32": 0, "bf16": 1, "fp8": 2}
_TORCH_DT = {torch.float32: 0, torch.bfloat16: 1, torch.float8_e4m3fn: 2}


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (host only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-std=c99", "-shared", "-fPIC", "-Wall",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


class _Problem(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("B", "Hq", "Hkv", "D", "C", "L", "k", "U", "q_dtype", "kv_dtype")] \
        + [("scale", ctypes.c_double), ("T", ctypes.c_int32)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        for name in ("mo_widen", "mo_route", "mo_bucket", "mo_attend", "mo_partials", "mo_direct", "mo_merge",
                     "mo_threads", "mo_chunk_embeddings", "mo_quantize_fp8"):
            getattr(_lib, name).restype = ctypes.c_int
    return _lib


def _cprob(p) -> _Problem:
    return _Problem(p.B, p.Hq, p.Hkv, p.D, p.C, p.L, p.k, p.U, _DT[p.q_dtype], _DT[p.kv_dtype], float(p.scale),
                    int(getattr(p, "T", 1)))


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return ctypes.c_void_p(0)
    assert t.device.type == "cpu" and t.is_contiguous(), "oracle takes contiguous CPU tensors"
    return ctypes.c_void_p(t.data_ptr())


def _check(t: torch.Tensor, shape, dtype_name=None, dtype=None):
    assert tuple(t.shape) == tuple(shape), (tuple(t.shape), tuple(shape))
    if dtype_name is not None:
        assert _TORCH_DT[t.dtype] == _DT[dtype_name], (t.dtype, dtype_name)
    if dtype is not None:
        assert t.dtype == dtype, (t.dtype, dtype)


def threads() -> int:
    return lib().mo_threads()


def widen(t: torch.Tensor) -> torch.Tensor:
    """Stored bits -> fp64, element by element."""
    t = t.contiguous()
    out = torch.empty(t.shape, dtype=torch.float64)
    rc = lib().mo_widen(_TORCH_DT[t.dtype], _ptr(t), ctypes.c_int64(t.numel()), _ptr(out))
    assert rc == 0
    return out


def route(p, Q, E, want_all_scores: bool = False):
    """S1+S2.  Returns ids [B,Hkv,k] int32, selected scores [B,Hkv,k] f64, (all scores [B,Hkv,C])."""
    _check(Q, (p.Bq, p.Hq, p.D), p.q_dtype)
    _check(E, (p.Hkv, p.C, p.D), p.q_dtype)
    ids = torch.empty((p.Bq, p.Hkv, p.k), dtype=torch.int32)
    sel = torch.empty((p.Bq, p.Hkv, p.k), dtype=torch.float64)
    allv = torch.empty((p.Bq, p.Hkv, p.C), dtype=torch.float64) if want_all_scores else None
    cp = _cprob(p)
    rc = lib().mo_route(ctypes.byref(cp), _ptr(Q), _ptr(E), _ptr(ids), _ptr(sel), _ptr(allv))
    assert rc == 0, rc
    return (ids, sel, allv) if want_all_scores else (ids, sel)


def bucket(p, ids):
    """Group items by (KV head, chunk).  Returns off [Hkv*C+1], items [B*Hkv*k] (int32)."""
    _check(ids, (p.Bq, p.Hkv, p.k), dtype=torch.int32)
    off = torch.empty((p.Hkv * p.C + 1,), dtype=torch.int32)
    items = torch.empty((p.Bq * p.Hkv * p.k,), dtype=torch.int32)
    cp = _cprob(p)
    rc = lib().mo_bucket(ctypes.byref(cp), _ptr(ids), _ptr(off), _ptr(items))
    assert rc == 0, rc
    return off, items


def attend(q, K, V, scale: float = 1.0):
    """Softmax attention of one fp64 row q[D] over fp64 K,V [n,D].  Returns (O[D], lse)."""
    q, K, V = (x.to(torch.float64).contiguous() for x in (q, K, V))
    D, n = q.numel(), K.shape[0]
    O = torch.empty((D,), dtype=torch.float64)
    lse = ctypes.c_double(0.0)
    rc = lib().mo_attend(D, ctypes.c_int64(n), _ptr(q), _ptr(K), _ptr(V), ctypes.c_double(scale), _ptr(O),
                         ctypes.byref(lse))
    assert rc == 0
    return O, lse.value


def _check_inputs(inp):
    p = inp.prob
    _check(inp.Q, (p.Bq, p.Hq, p.D), p.q_dtype)
    _check(inp.Ks, (p.C, p.Hkv, p.L, p.D), p.kv_dtype)
    _check(inp.Vs, (p.C, p.Hkv, p.L, p.D), p.kv_dtype)
    _check(inp.Ku, (p.B, p.Hkv, p.U, p.D), p.q_dtype)
    _check(inp.Vu, (p.B, p.Hkv, p.U, p.D), p.q_dtype)
    _check(inp.unique_len, (p.B,), dtype=torch.int32)
    if p.kv_dtype == "fp8":
        _check(inp.scale_k, (p.C, p.Hkv), dtype=torch.float32)
        _check(inp.scale_v, (p.C, p.Hkv), dtype=torch.float32)


def partials(inp, ids):
    """S4.  Returns part_O [B,Hq,k+1,D], part_LSE [B,Hq,k+1] (fp64)."""
    p = inp.prob
    _check_inputs(inp)
    _check(ids, (p.Bq, p.Hkv, p.k), dtype=torch.int32)
    pO = torch.empty((p.Bq, p.Hq, p.k + 1, p.D), dtype=torch.float64)
    pL = torch.empty((p.Bq, p.Hq, p.k + 1), dtype=torch.float64)
    cp = _cprob(p)
    rc = lib().mo_partials(ctypes.byref(cp), _ptr(inp.Q), _ptr(inp.Ks), _ptr(inp.Vs), _ptr(inp.scale_k),
                           _ptr(inp.scale_v), _ptr(inp.Ku), _ptr(inp.Vu), _ptr(inp.unique_len), _ptr(ids),
                           _ptr(pO), _ptr(pL))
    assert rc == 0
    return pO, pL


def direct(inp, ids):
    """S3.  Returns O [B,Hq,D], LSE [B,Hq] (fp64): attention over the routed union."""
    p = inp.prob
    _check_inputs(inp)
    _check(ids, (p.Bq, p.Hkv, p.k), dtype=torch.int32)
    O = torch.empty((p.Bq, p.Hq, p.D), dtype=torch.float64)
    LSE = torch.empty((p.Bq, p.Hq), dtype=torch.float64)
    cp = _cprob(p)
    rc = lib().mo_direct(ctypes.byref(cp), _ptr(inp.Q), _ptr(inp.Ks), _ptr(inp.Vs), _ptr(inp.scale_k),
                         _ptr(inp.scale_v), _ptr(inp.Ku), _ptr(inp.Vu), _ptr(inp.unique_len), _ptr(ids),
                         _ptr(O), _ptr(LSE))
    assert rc == 0
    return O, LSE


def merge(part_O, part_LSE):
    """S5.  part_O [...,P,D], part_LSE [...,P] fp64 -> O [...,D], LSE [...]."""
    part_O = part_O.to(torch.float64).contiguous()
    part_LSE = part_LSE.to(torch.float64).contiguous()
    P, D = part_O.shape[-2], part_O.shape[-1]
    lead = part_O.shape[:-2]
    rows = int(torch.tensor(lead).prod().item()) if len(lead) else 1
    O = torch.empty(tuple(lead) + (D,), dtype=torch.float64)
    LSE = torch.empty(tuple(lead), dtype=torch.float64)
    rc = lib().mo_merge(ctypes.c_int64(rows), P, D, _ptr(part_O), _ptr(part_LSE), _ptr(O), _ptr(LSE))
    assert rc == 0
    return O, LSE


@dataclass
class DecodeStep:
    ids: torch.Tensor
    scores: torch.Tensor
    bucket_off: torch.Tensor
    bucket_items: torch.Tensor
    part_O: torch.Tensor
    part_LSE: torch.Tensor
    O: torch.Tensor          # merged (S5)
    LSE: torch.Tensor
    O_direct: torch.Tensor   # over the union (S3)
    LSE_direct: torch.Tensor


def decode_step(inp, ids: Optional[torch.Tensor] = None, want_direct: bool = True) -> DecodeStep:
    """The whole path on CPU tensors: route -> bucket -> partials -> merge (+ direct)."""
    p = inp.prob
    r_ids, scores = route(p, inp.Q, inp.E)
    if ids is None:
        ids = r_ids
    off, items = bucket(p, ids)
    pO, pL = partials(inp, ids)
    O, LSE = merge(pO, pL)
    Od, Ld = direct(inp, ids) if want_direct else (None, None)
    return DecodeStep(ids, scores, off, items, pO, pL, O, LSE, Od, Ld)


def chunk_embeddings(p, Ks, scale_k=None):
    """Mean key of every (chunk, KV head) block, rounded to the q dtype.  Returns E [Hkv,C,D]."""
    _check(Ks, (p.C, p.Hkv, p.L, p.D), p.kv_dtype)
    E = torch.empty((p.Hkv, p.C, p.D), dtype={"f32": torch.float32, "bf16": torch.bfloat16}[p.q_dtype])
    cp = _cprob(p)
    rc = lib().mo_chunk_embeddings(ctypes.byref(cp), _ptr(Ks), _ptr(scale_k), _ptr(E))
    assert rc == 0
    return E


def quantize_fp8(p, X):
    """X [C,Hkv,L,D] (q dtype) -> (fp8 tensor, scale [C,Hkv] f32) with X ~= scale * fp8."""
    _check(X, (p.C, p.Hkv, p.L, p.D), p.q_dtype)
    X8 = torch.empty((p.C, p.Hkv, p.L, p.D), dtype=torch.uint8)
    scale = torch.empty((p.C, p.Hkv), dtype=torch.float32)
    cp = _cprob(p)
    rc = lib().mo_quantize_fp8(ctypes.byref(cp), _ptr(X), _ptr(X8), _ptr(scale))
    assert rc == 0
    return X8.view(torch.float8_e4m3fn), scale
