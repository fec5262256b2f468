"""Thin ctypes binding of libmoska.so: argument marshalling only.

Every function has the name and argument order of its C entry point in include/moska.h and
takes torch tensors that already live on the GPU; the work is enqueued on torch's current
stream.  There is no fallback: if the HIP library is missing or a call fails, it raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libmoska.so")

F32, BF16, FP8_E4M3 = 0, 1, 2
_DT = {"f32": F32, "bf16": BF16, "fp8": FP8_E4M3}
_TORCH = {F32: torch.float32, BF16: torch.bfloat16, FP8_E4M3: torch.float8_e4m3fn}

EXPORTS = ("moska_workspace_bytes", "moska_route", "moska_bucket", "moska_shared_attn", "moska_unique_attn",
           "moska_merge", "moska_decode_step", "moska_decode_step_static", "moska_chunk_embeddings", "moska_quantize_shared", "moska_status_string")


class MoskaError(RuntimeError):
    pass


class ProblemT(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("B", "Hq", "Hkv", "D", "C", "L", "k", "U_max", "q_dtype", "shared_kv_dtype")] + \
               [("scale", ctypes.c_float), ("q_len", ctypes.c_int32)]

    @property
    def Bq(self) -> int:
        """Query tokens in the step: the leading size of Q, ids, partials and outputs."""
        return self.B * max(self.q_len, 1)


_lib = None


def load_library() -> ctypes.CDLL:
    """Load the built HIP library; fail loudly if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise MoskaError(f"{LIB_PATH} is missing: run `python -m paper_2511_06010_amd.build` first")
        lib = ctypes.CDLL(LIB_PATH)
        for name in EXPORTS:
            getattr(lib, name).restype = ctypes.c_int
        lib.moska_status_string.restype = ctypes.c_char_p
        _lib = lib
    return _lib


def problem_t(p) -> ProblemT:
    """moska_inputs.Problem (or anything with the same fields) -> moska_problem_t."""
    if isinstance(p, ProblemT):
        return p
    return ProblemT(p.B, p.Hq, p.Hkv, p.D, p.C, p.L, p.k, p.U, _DT[p.q_dtype], _DT[p.kv_dtype], float(p.scale),
                    int(getattr(p, "T", 1)))


def _check(rc: int, what: str):
    if rc != 0:
        msg = load_library().moska_status_string(rc).decode()
        raise MoskaError(f"{what} failed: {msg} ({rc})")


def _dev(t: Optional[torch.Tensor], dtype=None, shape=None, name="tensor"):
    if t is None:
        return ctypes.c_void_p(0)
    if not t.is_cuda or not t.is_contiguous():
        raise MoskaError(f"{name} must be a contiguous GPU tensor")
    if dtype is not None and t.dtype != dtype:
        raise MoskaError(f"{name} has dtype {t.dtype}, expected {dtype}")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise MoskaError(f"{name} has shape {tuple(t.shape)}, expected {tuple(shape)}")
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def workspace_bytes(p) -> int:
    cp, out = problem_t(p), ctypes.c_size_t(0)
    _check(load_library().moska_workspace_bytes(ctypes.byref(cp), ctypes.byref(out)), "moska_workspace_bytes")
    return out.value


def route(p, Q, E, ids, scores, ws):
    cp = problem_t(p)
    qd = _TORCH[cp.q_dtype]
    rc = load_library().moska_route(
        ctypes.byref(cp), _dev(Q, qd, (cp.Bq, cp.Hq, cp.D), "Q"), _dev(E, qd, (cp.Hkv, cp.C, cp.D), "E"),
        _dev(ids, torch.int32, (cp.Bq, cp.Hkv, cp.k), "ids"),
        _dev(scores, torch.float32, (cp.Bq, cp.Hkv, cp.k), "scores"),
        _dev(ws, torch.uint8, name="ws"), ctypes.c_size_t(0 if ws is None else ws.numel()), _stream())
    _check(rc, "moska_route")


def bucket(p, ids, bucket_off, bucket_items, ws):
    cp = problem_t(p)
    rc = load_library().moska_bucket(
        ctypes.byref(cp), _dev(ids, torch.int32, (cp.Bq, cp.Hkv, cp.k), "ids"),
        _dev(bucket_off, torch.int32, (cp.Hkv * cp.C + 1,), "bucket_off"),
        _dev(bucket_items, torch.int32, (cp.Bq * cp.Hkv * cp.k,), "bucket_items"),
        _dev(ws, torch.uint8, name="ws"), ctypes.c_size_t(0 if ws is None else ws.numel()), _stream())
    _check(rc, "moska_bucket")


def shared_attn(p, Q, Ks, Vs, scale_k, scale_v, ids, bucket_off, bucket_items, part_O, part_LSE, ws):
    cp = problem_t(p)
    qd, kd = _TORCH[cp.q_dtype], _TORCH[cp.shared_kv_dtype]
    kv_shape = (cp.C, cp.Hkv, cp.L, cp.D)
    rc = load_library().moska_shared_attn(
        ctypes.byref(cp), _dev(Q, qd, (cp.Bq, cp.Hq, cp.D), "Q"), _dev(Ks, kd, kv_shape, "Ks"),
        _dev(Vs, kd, kv_shape, "Vs"), _dev(scale_k, torch.float32, (cp.C, cp.Hkv), "scale_k"),
        _dev(scale_v, torch.float32, (cp.C, cp.Hkv), "scale_v"),
        _dev(ids, torch.int32, (cp.Bq, cp.Hkv, cp.k), "ids"),
        _dev(bucket_off, torch.int32, (cp.Hkv * cp.C + 1,), "bucket_off"),
        _dev(bucket_items, torch.int32, (cp.Bq * cp.Hkv * cp.k,), "bucket_items"),
        _dev(part_O, torch.float32, (cp.Bq, cp.Hq, cp.k + 1, cp.D), "part_O"),
        _dev(part_LSE, torch.float32, (cp.Bq, cp.Hq, cp.k + 1), "part_LSE"),
        _dev(ws, torch.uint8, name="ws"), ctypes.c_size_t(0 if ws is None else ws.numel()), _stream())
    _check(rc, "moska_shared_attn")


def unique_attn(p, Q, Ku, Vu, unique_len, part_O, part_LSE, ws):
    cp = problem_t(p)
    qd = _TORCH[cp.q_dtype]
    kv_shape = (cp.B, cp.Hkv, cp.U_max, cp.D)
    rc = load_library().moska_unique_attn(
        ctypes.byref(cp), _dev(Q, qd, (cp.Bq, cp.Hq, cp.D), "Q"), _dev(Ku, qd, kv_shape, "Ku"),
        _dev(Vu, qd, kv_shape, "Vu"), _dev(unique_len, torch.int32, (cp.B,), "unique_len"),
        _dev(part_O, torch.float32, (cp.Bq, cp.Hq, cp.k + 1, cp.D), "part_O"),
        _dev(part_LSE, torch.float32, (cp.Bq, cp.Hq, cp.k + 1), "part_LSE"),
        _dev(ws, torch.uint8, name="ws"), ctypes.c_size_t(0 if ws is None else ws.numel()), _stream())
    _check(rc, "moska_unique_attn")


def merge(p, part_O, part_LSE, O, LSE=None):
    cp = problem_t(p)
    rc = load_library().moska_merge(
        ctypes.byref(cp), _dev(part_O, torch.float32, (cp.Bq, cp.Hq, cp.k + 1, cp.D), "part_O"),
        _dev(part_LSE, torch.float32, (cp.Bq, cp.Hq, cp.k + 1), "part_LSE"),
        _dev(O, _TORCH[cp.q_dtype], (cp.Bq, cp.Hq, cp.D), "O"), _dev(LSE, torch.float32, (cp.Bq, cp.Hq), "LSE"),
        _stream())
    _check(rc, "moska_merge")


def decode_step(p, Q, E, Ks, Vs, scale_k, scale_v, Ku, Vu, unique_len, ids, bucket_off, bucket_items,
                part_O, part_LSE, O, LSE, ws):
    cp = problem_t(p)
    qd, kd = _TORCH[cp.q_dtype], _TORCH[cp.shared_kv_dtype]
    rc = load_library().moska_decode_step(
        ctypes.byref(cp), _dev(Q, qd, (cp.Bq, cp.Hq, cp.D), "Q"), _dev(E, qd, (cp.Hkv, cp.C, cp.D), "E"),
        _dev(Ks, kd, (cp.C, cp.Hkv, cp.L, cp.D), "Ks"), _dev(Vs, kd, (cp.C, cp.Hkv, cp.L, cp.D), "Vs"),
        _dev(scale_k, torch.float32, (cp.C, cp.Hkv), "scale_k"), _dev(scale_v, torch.float32, (cp.C, cp.Hkv), "scale_v"),
        _dev(Ku, qd, (cp.B, cp.Hkv, cp.U_max, cp.D), "Ku"), _dev(Vu, qd, (cp.B, cp.Hkv, cp.U_max, cp.D), "Vu"),
        _dev(unique_len, torch.int32, (cp.B,), "unique_len"),
        _dev(ids, torch.int32, (cp.Bq, cp.Hkv, cp.k), "ids"),
        _dev(bucket_off, torch.int32, (cp.Hkv * cp.C + 1,), "bucket_off"),
        _dev(bucket_items, torch.int32, (cp.Bq * cp.Hkv * cp.k,), "bucket_items"),
        _dev(part_O, torch.float32, (cp.Bq, cp.Hq, cp.k + 1, cp.D), "part_O"),
        _dev(part_LSE, torch.float32, (cp.Bq, cp.Hq, cp.k + 1), "part_LSE"),
        _dev(O, qd, (cp.Bq, cp.Hq, cp.D), "O"), _dev(LSE, torch.float32, (cp.Bq, cp.Hq), "LSE"),
        _dev(ws, torch.uint8, name="ws"), ctypes.c_size_t(0 if ws is None else ws.numel()), _stream())
    _check(rc, "moska_decode_step")


STATIC_SCRATCH_BYTES = 16 << 20        # MOSKA_STATIC_SCRATCH_BYTES


def decode_step_static(p, Q, E, Ks, Vs, scale_k, scale_v, Ku, Vu, unique_len, ids, bucket_off, bucket_items,
                       part_O, part_LSE, O, LSE):
    cp = problem_t(p)
    qd, kd = _TORCH[cp.q_dtype], _TORCH[cp.shared_kv_dtype]
    rc = load_library().moska_decode_step_static(
        ctypes.byref(cp), _dev(Q, qd, (cp.Bq, cp.Hq, cp.D), "Q"), _dev(E, qd, (cp.Hkv, cp.C, cp.D), "E"),
        _dev(Ks, kd, (cp.C, cp.Hkv, cp.L, cp.D), "Ks"), _dev(Vs, kd, (cp.C, cp.Hkv, cp.L, cp.D), "Vs"),
        _dev(scale_k, torch.float32, (cp.C, cp.Hkv), "scale_k"), _dev(scale_v, torch.float32, (cp.C, cp.Hkv), "scale_v"),
        _dev(Ku, qd, (cp.B, cp.Hkv, cp.U_max, cp.D), "Ku"), _dev(Vu, qd, (cp.B, cp.Hkv, cp.U_max, cp.D), "Vu"),
        _dev(unique_len, torch.int32, (cp.B,), "unique_len"),
        _dev(ids, torch.int32, (cp.Bq, cp.Hkv, cp.k), "ids"),
        _dev(bucket_off, torch.int32, (cp.Hkv * cp.C + 1,), "bucket_off"),
        _dev(bucket_items, torch.int32, (cp.Bq * cp.Hkv * cp.k,), "bucket_items"),
        _dev(part_O, torch.float32, (cp.Bq, cp.Hq, cp.k + 1, cp.D), "part_O"),
        _dev(part_LSE, torch.float32, (cp.Bq, cp.Hq, cp.k + 1), "part_LSE"),
        _dev(O, qd, (cp.Bq, cp.Hq, cp.D), "O"), _dev(LSE, torch.float32, (cp.Bq, cp.Hq), "LSE"), _stream())
    _check(rc, "moska_decode_step_static")


def chunk_embeddings(p, Ks, scale_k, E):
    cp = problem_t(p)
    rc = load_library().moska_chunk_embeddings(
        ctypes.byref(cp), _dev(Ks, _TORCH[cp.shared_kv_dtype], (cp.C, cp.Hkv, cp.L, cp.D), "Ks"),
        _dev(scale_k, torch.float32, (cp.C, cp.Hkv), "scale_k"),
        _dev(E, _TORCH[cp.q_dtype], (cp.Hkv, cp.C, cp.D), "E"), _stream())
    _check(rc, "moska_chunk_embeddings")


def quantize_shared(p, X, X8, scale):
    cp = problem_t(p)
    rc = load_library().moska_quantize_shared(
        ctypes.byref(cp), _dev(X, torch.bfloat16, (cp.C, cp.Hkv, cp.L, cp.D), "X"),
        _dev(X8, torch.float8_e4m3fn, (cp.C, cp.Hkv, cp.L, cp.D), "X8"),
        _dev(scale, torch.float32, (cp.C, cp.Hkv), "scale"), _stream())
    _check(rc, "moska_quantize_shared")


class Buffers:
    """Caller-owned device buffers for one problem (allocation is the caller's job, done here once)."""

    def __init__(self, p, device="cuda"):
        cp = problem_t(p)
        dev = torch.device(device)
        self.ids = torch.empty((cp.Bq, cp.Hkv, cp.k), dtype=torch.int32, device=dev)
        self.scores = torch.empty((cp.Bq, cp.Hkv, cp.k), dtype=torch.float32, device=dev)
        self.bucket_off = torch.empty((cp.Hkv * cp.C + 1,), dtype=torch.int32, device=dev)
        self.bucket_items = torch.empty((cp.Bq * cp.Hkv * cp.k,), dtype=torch.int32, device=dev)
        self.part_O = torch.empty((cp.Bq, cp.Hq, cp.k + 1, cp.D), dtype=torch.float32, device=dev)
        self.part_LSE = torch.empty((cp.Bq, cp.Hq, cp.k + 1), dtype=torch.float32, device=dev)
        self.O = torch.empty((cp.Bq, cp.Hq, cp.D), dtype=_TORCH[cp.q_dtype], device=dev)
        self.LSE = torch.empty((cp.Bq, cp.Hq), dtype=torch.float32, device=dev)
        self.ws = torch.empty((workspace_bytes(p),), dtype=torch.uint8, device=dev)
