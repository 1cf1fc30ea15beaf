"""ctypes binding of libesp.so: same names as the C ABI (include/esp.h), argument marshalling only.

PyTorch provides device memory and the current stream; every step of the path runs in the
library's HIP kernels.  Importing this module fails loudly if the library is missing: there is
no CPU or PyTorch fallback.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libesp.so")

ESP_OK, ESP_ERR_INVALID_ARG, ESP_ERR_UNSUPPORTED, ESP_ERR_WORKSPACE, ESP_ERR_HIP = 0, -1, -2, -3, -4
ESP_MAX_PARTIALS = 16

EXPORTS = (
    "esp_partial_attn_prefill", "esp_prefill_workspace_bytes", "esp_partial_attn_decode",
    "esp_decode_workspace_bytes", "esp_merge_partials", "esp_kv_append", "esp_last_error", "esp_version",
    "esp_plan_prefill_batches", "esp_fit_prefill_model",
    "esp_kv_gather", "esp_partial_attn_prefill_pool", "esp_prefill_pool_workspace_bytes",
    "esp_probe_mfma_bf16", "esp_probe_stream_read",
    "esp_partial_attn_prefill_f32", "esp_merge_partials_f32",
    "esp_debug_set_validate", "esp_debug_set_prefill_sync_ticks",
    "esp_partial_attn_decode_static", "esp_partial_attn_prefill_retain", "esp_plan_prefill_batches_monotone",
    "esp_partial_attn_decode_merge", "esp_partial_attn_prefill_pool_direct",
)
ESP_DECODE_STATIC_SCRATCH_BYTES = 32 << 20


class EspError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"libesp status {status}: {message}")
        self.status = status


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -c 'import __graft_entry__ as g; g.build()'` "
            "(hipcc --offload-arch=gfx950).  There is no fallback path.")
    L = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, f32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float, ctypes.c_size_t
    L.esp_partial_attn_prefill.argtypes = [vp] * 7 + [i32] * 8 + [f32, i32, vp, vp, vp, sz, vp]
    L.esp_partial_attn_prefill.restype = i32
    L.esp_partial_attn_prefill_f32.argtypes = L.esp_partial_attn_prefill.argtypes
    L.esp_partial_attn_prefill_f32.restype = i32
    L.esp_merge_partials_f32.argtypes = [vp, vp, i32, i32, i32, i32, vp, vp, vp]
    L.esp_merge_partials_f32.restype = i32
    L.esp_debug_set_validate.argtypes = [i32]
    L.esp_debug_set_validate.restype = i32
    L.esp_debug_set_prefill_sync_ticks.argtypes = [i32]
    L.esp_debug_set_prefill_sync_ticks.restype = i32
    L.esp_partial_attn_prefill_retain.argtypes = [vp] * 7 + [i32] * 8 + [f32, i32, vp, vp, vp, i64, i32, vp, vp, vp, sz, vp]
    L.esp_partial_attn_prefill_retain.restype = i32
    L.esp_prefill_workspace_bytes.argtypes = [i32] * 6
    L.esp_prefill_workspace_bytes.restype = sz
    L.esp_partial_attn_decode.argtypes = [vp, vp, vp, i64, vp, vp, i32, i32, i32, i32, i32, i32, f32, vp, vp, vp, sz, vp]
    L.esp_partial_attn_decode.restype = i32
    L.esp_partial_attn_decode_merge.argtypes = [vp, vp, vp, i64, vp, vp, i32, i32, i32, i32, i32, i32, f32, vp, vp, i32,
                                                vp, vp, vp, sz, vp]
    L.esp_partial_attn_decode_merge.restype = i32
    L.esp_partial_attn_decode_static.argtypes = [vp, vp, vp, i64, vp, vp, i32, i32, i32, i32, i32, i32, f32, vp, vp, vp]
    L.esp_partial_attn_decode_static.restype = i32
    L.esp_decode_workspace_bytes.argtypes = [i32] * 6
    L.esp_decode_workspace_bytes.restype = sz
    L.esp_merge_partials.argtypes = [vp, vp, i32, i32, i32, i32, vp, vp, vp]
    L.esp_merge_partials.restype = i32
    L.esp_kv_append.argtypes = [vp, vp, vp, i32, vp, vp, i64, i32, i32, vp]
    L.esp_kv_append.restype = i32
    L.esp_kv_gather.argtypes = [vp, vp, vp, i32, i64, i32, i32, vp, vp, vp]
    L.esp_kv_gather.restype = i32
    L.esp_partial_attn_prefill_pool.argtypes = [vp, vp, vp, i64] + [vp] * 5 + [i32] * 8 + [f32, i32, vp, vp, vp, sz, vp]
    L.esp_partial_attn_prefill_pool.restype = i32
    L.esp_partial_attn_prefill_pool_direct.argtypes = [vp, vp, vp, i64] + [vp] * 5 + [i32] * 8 + [f32, i32, i32, vp, vp, vp, sz, vp]
    L.esp_partial_attn_prefill_pool_direct.restype = i32
    L.esp_prefill_pool_workspace_bytes.argtypes = [i32] * 6
    L.esp_prefill_pool_workspace_bytes.restype = sz
    L.esp_probe_mfma_bf16.argtypes = [vp, i64, i32, vp, vp, vp]
    L.esp_probe_mfma_bf16.restype = i32
    L.esp_probe_stream_read.argtypes = [vp, i64, vp, vp]
    L.esp_probe_stream_read.restype = i32
    L.esp_plan_prefill_batches.argtypes = [vp, i32, vp, i32, vp, vp, vp, vp, vp, vp, vp]
    L.esp_plan_prefill_batches.restype = i32
    L.esp_plan_prefill_batches_monotone.argtypes = L.esp_plan_prefill_batches.argtypes
    L.esp_plan_prefill_batches_monotone.restype = i32
    L.esp_fit_prefill_model.argtypes = [vp, vp, vp, vp, i32, vp]
    L.esp_fit_prefill_model.restype = i32
    L.esp_last_error.argtypes = []
    L.esp_last_error.restype = ctypes.c_char_p
    L.esp_version.argtypes = []
    L.esp_version.restype = ctypes.c_char_p
    return L


lib = _load()


def last_error() -> str:
    return lib.esp_last_error().decode()


def version() -> str:
    return lib.esp_version().decode()


def _check(status: int) -> None:
    if status != ESP_OK:
        raise EspError(status, last_error())


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _dev(t: torch.Tensor, dtype, name: str) -> torch.Tensor:
    if not t.is_cuda:
        raise ValueError(f"{name}: must live in device memory")
    if t.dtype != dtype:
        raise ValueError(f"{name}: expected {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name}: must be contiguous")
    return t


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _workspace(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def esp_debug_set_validate(on: bool) -> bool:
    """Host-side check of device index arrays before every launch (a debugging aid); returns the previous setting."""
    return bool(lib.esp_debug_set_validate(1 if on else 0))


def esp_debug_set_prefill_sync_ticks(ticks: int) -> int:
    """Longest start-of-round wait of the prefill kernel in 10 ns ticks (negative: the default); returns the previous value."""
    return int(lib.esp_debug_set_prefill_sync_ticks(int(ticks)))


def esp_prefill_workspace_bytes(Tq, Tkv, batch, Hq, Hkv, D) -> int:
    return int(lib.esp_prefill_workspace_bytes(Tq, Tkv, batch, Hq, Hkv, D))


def esp_decode_workspace_bytes(B, total_tokens, max_len, Hq, Hkv, D) -> int:
    return int(lib.esp_decode_workspace_bytes(B, total_tokens, max_len, Hq, Hkv, D))


def esp_partial_attn_prefill(q, k, v, q_pos, kv_pos, cu_q=None, cu_kv=None, max_q=None, max_kv=None,
                             softmax_scale=None, causal=True, O=None, LSE=None, workspace=None, out_dtype=torch.bfloat16):
    """q [Tq,Hq,D], k/v [Tkv,Hkv,D] bf16; q_pos/kv_pos int32; cu_q/cu_kv int32 [batch+1] or None.
    Returns (O [Tq,Hq,D], LSE fp32 [Tq,Hq]) of attention against this one KV shard.  O is bf16
    (esp_partial_attn_prefill) or, if `O` is a float32 tensor or out_dtype is torch.float32, fp32
    (esp_partial_attn_prefill_f32)."""
    _dev(q, torch.bfloat16, "q"); _dev(k, torch.bfloat16, "k"); _dev(v, torch.bfloat16, "v")
    _dev(q_pos, torch.int32, "q_pos"); _dev(kv_pos, torch.int32, "kv_pos")
    Tq, Hq, D = q.shape
    Tkv, Hkv, Dk = k.shape
    if v.shape != k.shape or Dk != D or q_pos.shape != (Tq,) or kv_pos.shape != (Tkv,):
        raise ValueError("prefill: shape mismatch")
    batch = 1
    if cu_q is not None:
        _dev(cu_q, torch.int32, "cu_q"); _dev(cu_kv, torch.int32, "cu_kv")
        batch = cu_q.numel() - 1
        if cu_kv.numel() != batch + 1:
            raise ValueError("prefill: cu_q and cu_kv differ in length")
        if max_q is None or max_kv is None:
            raise ValueError("prefill: max_q and max_kv are required with cu_q/cu_kv")
    else:
        max_q, max_kv = Tq, Tkv
    if softmax_scale is None:
        softmax_scale = D ** -0.5
    if O is None:
        O = torch.empty(q.shape, dtype=out_dtype, device=q.device)
    if LSE is None:
        LSE = torch.empty((Tq, Hq), dtype=torch.float32, device=q.device)
    if O.dtype not in (torch.bfloat16, torch.float32):
        raise ValueError("prefill: O must be bf16 or fp32")
    _dev(O, O.dtype, "O"); _dev(LSE, torch.float32, "LSE")
    if O.shape != q.shape or LSE.shape != (Tq, Hq):
        raise ValueError("prefill: output shape mismatch")
    if workspace is None:
        workspace = _workspace(esp_prefill_workspace_bytes(Tq, Tkv, batch, Hq, Hkv, D), q.device)
    call = lib.esp_partial_attn_prefill_f32 if O.dtype == torch.float32 else lib.esp_partial_attn_prefill
    _check(call(_ptr(q), _ptr(k), _ptr(v), _ptr(q_pos), _ptr(kv_pos), _ptr(cu_q), _ptr(cu_kv),
                                        batch, Tq, Tkv, int(max_q), int(max_kv), Hq, Hkv, D, float(softmax_scale),
                                        int(bool(causal)), _ptr(O), _ptr(LSE), _ptr(workspace), workspace.numel(),
                                        _stream()))
    return O, LSE


def esp_partial_attn_prefill_retain(q, k, v, q_pos, kv_pos, retain_slot, k_pool, v_pool, cu_q=None, cu_kv=None, max_q=None,
                                    max_kv=None, softmax_scale=None, causal=True, O=None, LSE=None, workspace=None,
                                    out_dtype=torch.bfloat16):
    """esp_partial_attn_prefill that also keeps the shard rows t with retain_slot[t] >= 0 in the pool (in place),
    from the tiles that pass through on-chip memory.  Returns (O, LSE); O bf16 or fp32 as in esp_partial_attn_prefill."""
    _dev(q, torch.bfloat16, "q"); _dev(k, torch.bfloat16, "k"); _dev(v, torch.bfloat16, "v")
    _dev(q_pos, torch.int32, "q_pos"); _dev(kv_pos, torch.int32, "kv_pos"); _dev(retain_slot, torch.int32, "retain_slot")
    _dev(k_pool, torch.bfloat16, "k_pool"); _dev(v_pool, torch.bfloat16, "v_pool")
    Tq, Hq, D = q.shape
    Tkv, Hkv, Dk = k.shape
    if (v.shape != k.shape or Dk != D or q_pos.shape != (Tq,) or kv_pos.shape != (Tkv,) or retain_slot.shape != (Tkv,)
            or k_pool.shape != v_pool.shape or k_pool.shape[1:] != k.shape[1:]):
        raise ValueError("prefill (retain): shape mismatch")
    batch = 1
    if cu_q is not None:
        _dev(cu_q, torch.int32, "cu_q"); _dev(cu_kv, torch.int32, "cu_kv")
        batch = cu_q.numel() - 1
        if cu_kv.numel() != batch + 1:
            raise ValueError("prefill (retain): cu_q and cu_kv differ in length")
        if max_q is None or max_kv is None:
            raise ValueError("prefill (retain): max_q and max_kv are required with cu_q/cu_kv")
    else:
        max_q, max_kv = Tq, Tkv
    if softmax_scale is None:
        softmax_scale = D ** -0.5
    if O is None:
        O = torch.empty(q.shape, dtype=out_dtype, device=q.device)
    if LSE is None:
        LSE = torch.empty((Tq, Hq), dtype=torch.float32, device=q.device)
    if O.dtype not in (torch.bfloat16, torch.float32):
        raise ValueError("prefill (retain): O must be bf16 or fp32")
    _dev(O, O.dtype, "O"); _dev(LSE, torch.float32, "LSE")
    if O.shape != q.shape or LSE.shape != (Tq, Hq):
        raise ValueError("prefill (retain): output shape mismatch")
    if workspace is None:
        workspace = _workspace(esp_prefill_workspace_bytes(Tq, Tkv, batch, Hq, Hkv, D), q.device)
    _check(lib.esp_partial_attn_prefill_retain(_ptr(q), _ptr(k), _ptr(v), _ptr(q_pos), _ptr(kv_pos), _ptr(cu_q), _ptr(cu_kv), batch,
                                               Tq, Tkv, int(max_q), int(max_kv), Hq, Hkv, D, float(softmax_scale),
                                               int(bool(causal)), _ptr(retain_slot), _ptr(k_pool), _ptr(v_pool), k_pool.shape[0],
                                               1 if O.dtype == torch.float32 else 0, _ptr(O), _ptr(LSE), _ptr(workspace),
                                               workspace.numel(), _stream()))
    return O, LSE


def esp_partial_attn_decode(q, k_pool, v_pool, slot_idx, seq_offsets, max_len, softmax_scale=None,
                            O=None, LSE=None, workspace=None):
    """q [B,Hq,D] bf16, pools [S,Hkv,D] bf16, slot_idx int32 [total], seq_offsets int32 [B+1].
    Returns (O bf16 [B,Hq,D], LSE fp32 [B,Hq]) of attention against the resident pool rows."""
    _dev(q, torch.bfloat16, "q"); _dev(k_pool, torch.bfloat16, "k_pool"); _dev(v_pool, torch.bfloat16, "v_pool")
    _dev(slot_idx, torch.int32, "slot_idx"); _dev(seq_offsets, torch.int32, "seq_offsets")
    B, Hq, D = q.shape
    S, Hkv, Dk = k_pool.shape
    if v_pool.shape != k_pool.shape or Dk != D or seq_offsets.numel() != B + 1:
        raise ValueError("decode: shape mismatch")
    total = slot_idx.numel()
    if softmax_scale is None:
        softmax_scale = D ** -0.5
    if O is None:
        O = torch.empty_like(q)
    if LSE is None:
        LSE = torch.empty((B, Hq), dtype=torch.float32, device=q.device)
    _dev(O, torch.bfloat16, "O"); _dev(LSE, torch.float32, "LSE")
    if workspace is None:
        workspace = _workspace(esp_decode_workspace_bytes(B, total, int(max_len), Hq, Hkv, D), q.device)
    _check(lib.esp_partial_attn_decode(_ptr(q), _ptr(k_pool), _ptr(v_pool), S, _ptr(slot_idx), _ptr(seq_offsets), B,
                                       total, int(max_len), Hq, Hkv, D, float(softmax_scale), _ptr(O), _ptr(LSE),
                                       _ptr(workspace), workspace.numel(), _stream()))
    return O, LSE


def esp_partial_attn_decode_static(q, k_pool, v_pool, slot_idx, seq_offsets, max_len, softmax_scale=None, O=None, LSE=None):
    """esp_partial_attn_decode on the library's built-in scratch block: the call itself allocates nothing (O and LSE
    must be given for that to hold on this side too)."""
    _dev(q, torch.bfloat16, "q"); _dev(k_pool, torch.bfloat16, "k_pool"); _dev(v_pool, torch.bfloat16, "v_pool")
    _dev(slot_idx, torch.int32, "slot_idx"); _dev(seq_offsets, torch.int32, "seq_offsets")
    B, Hq, D = q.shape
    S, Hkv, Dk = k_pool.shape
    if v_pool.shape != k_pool.shape or Dk != D or seq_offsets.numel() != B + 1:
        raise ValueError("decode: shape mismatch")
    if softmax_scale is None:
        softmax_scale = D ** -0.5
    if O is None:
        O = torch.empty_like(q)
    if LSE is None:
        LSE = torch.empty((B, Hq), dtype=torch.float32, device=q.device)
    _dev(O, torch.bfloat16, "O"); _dev(LSE, torch.float32, "LSE")
    _check(lib.esp_partial_attn_decode_static(_ptr(q), _ptr(k_pool), _ptr(v_pool), S, _ptr(slot_idx), _ptr(seq_offsets), B,
                                              slot_idx.numel(), int(max_len), Hq, Hkv, D, float(softmax_scale), _ptr(O), _ptr(LSE),
                                              _stream()))
    return O, LSE


def esp_partial_attn_decode_merge(q, k_pool, v_pool, slot_idx, seq_offsets, max_len, peer_O: Sequence[torch.Tensor],
                                  peer_LSE: Sequence[torch.Tensor], softmax_scale=None, O=None, LSE=None, workspace=None):
    """esp_partial_attn_decode combined, in the same pass, with the partial results peers returned for the same
    queries (peer_O[p] bf16 [B,Hq,D], peer_LSE[p] fp32 [B,Hq]).  Returns the final (O bf16, LSE fp32)."""
    _dev(q, torch.bfloat16, "q"); _dev(k_pool, torch.bfloat16, "k_pool"); _dev(v_pool, torch.bfloat16, "v_pool")
    _dev(slot_idx, torch.int32, "slot_idx"); _dev(seq_offsets, torch.int32, "seq_offsets")
    B, Hq, D = q.shape
    S, Hkv, Dk = k_pool.shape
    if v_pool.shape != k_pool.shape or Dk != D or seq_offsets.numel() != B + 1:
        raise ValueError("decode: shape mismatch")
    P = len(peer_O)
    if P != len(peer_LSE):
        raise ValueError("decode (merge): peer_O and peer_LSE differ in length")
    for i in range(P):
        _dev(peer_O[i], torch.bfloat16, f"peer_O[{i}]"); _dev(peer_LSE[i], torch.float32, f"peer_LSE[{i}]")
        if peer_O[i].shape != q.shape or peer_LSE[i].shape != (B, Hq):
            raise ValueError("decode (merge): peer partial shapes differ from the queries'")
    total = slot_idx.numel()
    if softmax_scale is None:
        softmax_scale = D ** -0.5
    if O is None:
        O = torch.empty_like(q)
    if LSE is None:
        LSE = torch.empty((B, Hq), dtype=torch.float32, device=q.device)
    _dev(O, torch.bfloat16, "O"); _dev(LSE, torch.float32, "LSE")
    if workspace is None:
        workspace = _workspace(esp_decode_workspace_bytes(B, total, int(max_len), Hq, Hkv, D), q.device)
    op = (ctypes.c_void_p * max(P, 1))(*[t.data_ptr() for t in peer_O])
    lp = (ctypes.c_void_p * max(P, 1))(*[t.data_ptr() for t in peer_LSE])
    _check(lib.esp_partial_attn_decode_merge(_ptr(q), _ptr(k_pool), _ptr(v_pool), S, _ptr(slot_idx), _ptr(seq_offsets), B,
                                             total, int(max_len), Hq, Hkv, D, float(softmax_scale), op, lp, P,
                                             _ptr(O), _ptr(LSE), _ptr(workspace), workspace.numel(), _stream()))
    return O, LSE


def esp_merge_partials(O_parts: Sequence[torch.Tensor], LSE_parts: Sequence[torch.Tensor], O=None, LSE=None,
                       want_lse: bool = True):
    """Combine P partial results (O_p bf16 or, all of them, fp32 [T,Hq,D]; LSE_p fp32 [T,Hq]) into
    (O bf16, LSE fp32 or None): esp_merge_partials or esp_merge_partials_f32 by the partials' type."""
    P = len(O_parts)
    if P != len(LSE_parts):
        raise ValueError("merge: O_parts and LSE_parts differ in length")
    if P == 0:
        raise ValueError("merge: need at least one partial")
    pdt = O_parts[0].dtype
    if pdt not in (torch.bfloat16, torch.float32):
        raise ValueError("merge: partials must be bf16 or fp32")
    for i in range(P):
        _dev(O_parts[i], pdt, f"O_parts[{i}]"); _dev(LSE_parts[i], torch.float32, f"LSE_parts[{i}]")
        if O_parts[i].shape != O_parts[0].shape or LSE_parts[i].shape != O_parts[0].shape[:-1]:
            raise ValueError("merge: partial shapes differ")
    *lead, Hq, D = O_parts[0].shape
    T = 1
    for s in lead:
        T *= s
    if O is None:
        O = torch.empty(O_parts[0].shape, dtype=torch.bfloat16, device=O_parts[0].device)
    _dev(O, torch.bfloat16, "O")
    if LSE is None and want_lse:
        LSE = torch.empty(O_parts[0].shape[:-1], dtype=torch.float32, device=O.device)
    op = (ctypes.c_void_p * P)(*[t.data_ptr() for t in O_parts])
    lp = (ctypes.c_void_p * P)(*[t.data_ptr() for t in LSE_parts])
    call = lib.esp_merge_partials_f32 if pdt == torch.float32 else lib.esp_merge_partials
    _check(call(op, lp, P, T, Hq, D, _ptr(O), _ptr(LSE), _stream()))
    return O, LSE


def esp_kv_append(k, v, slot_idx, k_pool, v_pool) -> None:
    """k_pool[slot_idx[t]] = k[t], v_pool[slot_idx[t]] = v[t] for slot_idx[t] >= 0 (in place)."""
    _dev(k, torch.bfloat16, "k"); _dev(v, torch.bfloat16, "v"); _dev(slot_idx, torch.int32, "slot_idx")
    _dev(k_pool, torch.bfloat16, "k_pool"); _dev(v_pool, torch.bfloat16, "v_pool")
    T, Hkv, D = k.shape
    if v.shape != k.shape or slot_idx.shape != (T,) or k_pool.shape != v_pool.shape or k_pool.shape[1:] != k.shape[1:]:
        raise ValueError("append: shape mismatch")
    _check(lib.esp_kv_append(_ptr(k), _ptr(v), _ptr(slot_idx), T, _ptr(k_pool), _ptr(v_pool), k_pool.shape[0], Hkv, D,
                             _stream()))


def esp_kv_gather(k_pool, v_pool, slot_idx, k=None, v=None):
    """k[t] = k_pool[slot_idx[t]], v[t] = v_pool[slot_idx[t]]; a slot outside the pool gives a zero row.  Returns (k, v)."""
    _dev(k_pool, torch.bfloat16, "k_pool"); _dev(v_pool, torch.bfloat16, "v_pool"); _dev(slot_idx, torch.int32, "slot_idx")
    S, Hkv, D = k_pool.shape
    T = slot_idx.numel()
    if v_pool.shape != k_pool.shape or slot_idx.dim() != 1:
        raise ValueError("gather: shape mismatch")
    if k is None:
        k = torch.empty((T, Hkv, D), dtype=torch.bfloat16, device=k_pool.device)
    if v is None:
        v = torch.empty((T, Hkv, D), dtype=torch.bfloat16, device=k_pool.device)
    _dev(k, torch.bfloat16, "k"); _dev(v, torch.bfloat16, "v")
    if k.shape != (T, Hkv, D) or v.shape != (T, Hkv, D):
        raise ValueError("gather: output shape mismatch")
    _check(lib.esp_kv_gather(_ptr(k_pool), _ptr(v_pool), _ptr(slot_idx), T, S, Hkv, D, _ptr(k), _ptr(v), _stream()))
    return k, v


def esp_prefill_pool_workspace_bytes(Tq, Tkv, batch, Hq, Hkv, D) -> int:
    return int(lib.esp_prefill_pool_workspace_bytes(Tq, Tkv, batch, Hq, Hkv, D))


def esp_partial_attn_prefill_pool_direct(q, k_pool, v_pool, slot_idx, q_pos, kv_pos, cu_q=None, cu_kv=None, max_q=None,
                                         max_kv=None, softmax_scale=None, causal=True, O=None, LSE=None, workspace=None,
                                         out_dtype=None):
    """esp_partial_attn_prefill over the shard whose row i is pool row slot_idx[i], the tile transfers reading the pool
    rows themselves (no staging copy).  O bf16, or fp32 with out_dtype=torch.float32 / an fp32 O.  Returns (O, LSE)."""
    return esp_partial_attn_prefill_pool(q, k_pool, v_pool, slot_idx, q_pos, kv_pos, cu_q, cu_kv, max_q, max_kv, softmax_scale,
                                         causal, O, LSE, workspace, _direct=True, _out_dtype=out_dtype)


def esp_partial_attn_prefill_pool(q, k_pool, v_pool, slot_idx, q_pos, kv_pos, cu_q=None, cu_kv=None, max_q=None, max_kv=None,
                                  softmax_scale=None, causal=True, O=None, LSE=None, workspace=None, _direct=False,
                                  _out_dtype=None):
    """esp_partial_attn_prefill over the shard whose row i is pool row slot_idx[i].  Returns (O, LSE)."""
    _dev(q, torch.bfloat16, "q"); _dev(k_pool, torch.bfloat16, "k_pool"); _dev(v_pool, torch.bfloat16, "v_pool")
    _dev(slot_idx, torch.int32, "slot_idx"); _dev(q_pos, torch.int32, "q_pos"); _dev(kv_pos, torch.int32, "kv_pos")
    Tq, Hq, D = q.shape
    S, Hkv, Dk = k_pool.shape
    Tkv = slot_idx.numel()
    if Dk != D or v_pool.shape != k_pool.shape or q_pos.shape != (Tq,) or kv_pos.shape != (Tkv,) or slot_idx.dim() != 1:
        raise ValueError("prefill (pool): shape mismatch")
    batch = 1
    if cu_q is not None:
        _dev(cu_q, torch.int32, "cu_q"); _dev(cu_kv, torch.int32, "cu_kv")
        batch = cu_q.numel() - 1
        if cu_kv.numel() != batch + 1:
            raise ValueError("prefill (pool): cu_q and cu_kv differ in length")
        if max_q is None or max_kv is None:
            raise ValueError("prefill (pool): max_q and max_kv are required with cu_q/cu_kv")
    else:
        max_q, max_kv = Tq, Tkv
    if softmax_scale is None:
        softmax_scale = D ** -0.5
    odt = torch.bfloat16
    if _direct:
        odt = O.dtype if O is not None else (_out_dtype or torch.bfloat16)
        if odt not in (torch.bfloat16, torch.float32):
            raise ValueError("prefill (pool): O must be bf16 or fp32")
    if O is None:
        O = torch.empty(q.shape, dtype=odt, device=q.device)
    if LSE is None:
        LSE = torch.empty((Tq, Hq), dtype=torch.float32, device=q.device)
    _dev(O, odt, "O"); _dev(LSE, torch.float32, "LSE")
    if O.shape != q.shape or LSE.shape != (Tq, Hq):
        raise ValueError("prefill (pool): output shape mismatch")
    if _direct:
        if workspace is None:
            workspace = _workspace(esp_prefill_workspace_bytes(Tq, Tkv, batch, Hq, Hkv, D), q.device)
        _check(lib.esp_partial_attn_prefill_pool_direct(_ptr(q), _ptr(k_pool), _ptr(v_pool), S, _ptr(slot_idx), _ptr(q_pos),
                                                        _ptr(kv_pos), _ptr(cu_q), _ptr(cu_kv), batch, Tq, Tkv, int(max_q), int(max_kv),
                                                        Hq, Hkv, D, float(softmax_scale), 1 if causal else 0,
                                                        1 if odt == torch.float32 else 0, _ptr(O), _ptr(LSE), _ptr(workspace),
                                                        workspace.numel(), _stream()))
        return O, LSE
    if workspace is None:
        workspace = _workspace(esp_prefill_pool_workspace_bytes(Tq, Tkv, batch, Hq, Hkv, D), q.device)
    _check(lib.esp_partial_attn_prefill_pool(_ptr(q), _ptr(k_pool), _ptr(v_pool), S, _ptr(slot_idx), _ptr(q_pos), _ptr(kv_pos),
                                             _ptr(cu_q), _ptr(cu_kv), batch, Tq, Tkv, int(max_q), int(max_kv), Hq, Hkv, D,
                                             float(softmax_scale), 1 if causal else 0, _ptr(O), _ptr(LSE), _ptr(workspace),
                                             workspace.numel(), _stream()))
    return O, LSE


def esp_probe_mfma_bf16(operands, iters, sink) -> int:
    """Launches the bare MFMA loop on register operands taken from `operands` (bf16); returns the FLOPs of the launch."""
    _dev(operands, torch.bfloat16, "operands"); _dev(sink, torch.float32, "sink")
    flops = ctypes.c_int64(0)
    _check(lib.esp_probe_mfma_bf16(_ptr(operands), operands.numel() * 2, int(iters), _ptr(sink), ctypes.byref(flops), _stream()))
    return int(flops.value)


def esp_probe_stream_read(src, sink) -> int:
    """Launches one streaming read of `src` (any dtype, contiguous); returns the bytes read."""
    if not src.is_cuda or not src.is_contiguous():
        raise ValueError("probe: src must be a contiguous device tensor")
    _dev(sink, torch.float32, "sink")
    nbytes = src.numel() * src.element_size()
    _check(lib.esp_probe_stream_read(_ptr(src), nbytes, _ptr(sink), _stream()))
    return nbytes


def esp_plan_prefill_batches(req_len, free_slots, coefs, with_tables=False, monotone=False):
    """Batching plan of the prefill phase (host code); monotone: the search bounded by the split points of Eq. 6
    (esp_plan_prefill_batches_monotone: a valid plan, usually but not always the cheapest).  req_len: tokens per request, longest first; free_slots:
    unused KV slots per instance; coefs: [n_inst][3] = (alpha, beta, gamma) at degree of parallelism 1..n_inst.
    Returns (cost, req_cuts, inst_cuts) -- cost inf and empty cuts if nothing fits -- plus the two split tables
    if with_tables."""
    import numpy as np
    rl = np.ascontiguousarray(req_len, dtype=np.int64); fs = np.ascontiguousarray(free_slots, dtype=np.int64)
    cf = np.ascontiguousarray(coefs, dtype=np.float64)
    n, m = rl.size, fs.size
    if cf.shape != (m, 3):
        raise ValueError("plan: coefs must be [n_inst][3]")
    nb_max = max(1, min(n, m))
    rc = np.zeros(nb_max, np.int32); ic = np.zeros(nb_max, np.int32)
    nb = ctypes.c_int32(0); cost = ctypes.c_double(0.0)
    sr = np.zeros((n + 1, m + 1), np.int32) if with_tables else None
    si = np.zeros((n + 1, m + 1), np.int32) if with_tables else None
    p = lambda arr: ctypes.c_void_p(arr.ctypes.data) if arr is not None else ctypes.c_void_p(0)
    call = lib.esp_plan_prefill_batches_monotone if monotone else lib.esp_plan_prefill_batches
    _check(call(p(rl), n, p(fs), m, p(cf), p(rc), p(ic), ctypes.addressof(nb), ctypes.addressof(cost), p(sr), p(si)))
    out = (cost.value, rc[:nb.value].tolist(), ic[:nb.value].tolist())
    return out + (sr, si) if with_tables else out


def esp_fit_prefill_model(sum_len, sum_len_sq, seconds, weights=None):
    """Least-squares (alpha, beta, gamma) of seconds ~ alpha + beta * sum_len + gamma * sum_len_sq (host code);
    weights: optional per-sample factors on the equations (1 / seconds: relative residual)."""
    import numpy as np
    a = np.ascontiguousarray(sum_len, dtype=np.float64); b = np.ascontiguousarray(sum_len_sq, dtype=np.float64)
    t = np.ascontiguousarray(seconds, dtype=np.float64)
    if not (a.size == b.size == t.size):
        raise ValueError("fit: arrays differ in length")
    w = None if weights is None else np.ascontiguousarray(weights, dtype=np.float64)
    if w is not None and w.size != t.size:
        raise ValueError("fit: weights differ in length")
    out = np.zeros(3, np.float64)
    _check(lib.esp_fit_prefill_model(ctypes.c_void_p(a.ctypes.data), ctypes.c_void_p(b.ctypes.data),
                                     ctypes.c_void_p(t.ctypes.data), ctypes.c_void_p(w.ctypes.data if w is not None else 0),
                                     a.size, ctypes.c_void_p(out.ctypes.data)))
    return out
