"""ctypes binding of libkvzap.so: the same four calls as include/kvzap.h.

Argument marshalling only: tensors are checked for device, dtype and
contiguity, outputs and workspaces are allocated with torch when the caller
does not pass them, raw pointers and the current HIP stream are handed to the C
ABI.  Every step of the prune path runs in the library's kernels; there is no
fallback, and a missing library is an error.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libkvzap.so")

CALL_SCORE, CALL_MASK, CALL_COMPACT, CALL_DECODE_EVICT, CALL_ATTEND_DECODE = 0, 1, 2, 3, 4
CALL_ASSIGN_PAGES, CALL_TOPK_THRESHOLD, CALL_TEACHER_SCORES, CALL_COMPRESS = 5, 6, 7, 8
CALL_MASK_COMPACT = 9

_c_void_p, _c_int, _c_float, _c_size_t, _c_int64 = (
    ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t, ctypes.c_int64)

# name -> (restype, argtypes); mirrors include/kvzap.h
SIGNATURES = {
    "kvzap_status_string": (ctypes.c_char_p, [_c_int]),
    "kvzap_version": (ctypes.c_char_p, []),
    "kvzap_workspace_bytes": (_c_size_t, [_c_int] * 6),
    "kvzap_score": (_c_int, [_c_void_p] * 6 + [_c_int] * 5 + [_c_void_p, _c_size_t, _c_void_p]),
    "kvzap_mask": (_c_int, [_c_void_p, _c_float, _c_int, _c_void_p, _c_int, _c_int, _c_int,
                            _c_void_p, _c_void_p, _c_void_p, _c_void_p, _c_size_t, _c_void_p]),
    "kvzap_mask_static": (_c_int, [_c_void_p, _c_float, _c_int, _c_void_p, _c_int, _c_int, _c_int,
                                   _c_void_p, _c_void_p, _c_void_p, _c_void_p]),
    "kvzap_prepare_scorer": (_c_int, [_c_void_p, _c_int, _c_int, _c_void_p, _c_size_t, _c_void_p]),
    "kvzap_score_prepared": (_c_int, [_c_void_p] * 6 + [_c_int] * 5 + [_c_void_p]),
    "kvzap_prepare_scorer_rmsnorm": (_c_int, [_c_void_p, _c_void_p, _c_int, _c_int, _c_void_p, _c_size_t,
                                              _c_void_p]),
    "kvzap_score_rmsnorm": (_c_int, [_c_void_p] * 3 + [_c_float] + [_c_void_p] * 6 + [_c_int] * 5 +
                            [_c_void_p]),
    "kvzap_compress": (_c_int, [_c_void_p] * 7 + [_c_float, _c_int] + [_c_void_p] * 7 + [_c_int64] +
                       [_c_int] * 6 + [_c_void_p, _c_size_t, _c_void_p]),
    "kvzap_mask_compact": (_c_int, [_c_void_p, _c_float, _c_int] + [_c_void_p] * 8 + [_c_int64] +
                           [_c_int] * 4 + [_c_void_p, _c_size_t, _c_void_p]),
    "kvzap_teacher_scores": (_c_int, [_c_void_p] * 4 + [_c_float, _c_void_p] + [_c_int] * 6 +
                             [_c_void_p, _c_size_t, _c_void_p]),
    "kvzap_topk_threshold": (_c_int, [_c_void_p, _c_int, _c_void_p, _c_int64, _c_int, _c_int, _c_int,
                                      _c_int, _c_void_p, _c_void_p, _c_size_t, _c_void_p]),
    "kvzap_mask_per_head": (_c_int, [_c_void_p, _c_void_p, _c_int, _c_void_p, _c_int, _c_int, _c_int,
                                     _c_void_p, _c_void_p, _c_void_p, _c_void_p, _c_size_t,
                                     _c_void_p]),
    "kvzap_compact": (_c_int, [_c_void_p] * 7 + [_c_int64] + [_c_int] * 4 + [_c_void_p]),
    "kvzap_decode_evict": (_c_int, [_c_void_p] * 5 + [_c_int, _c_int] + [_c_void_p] * 12 +
                           [_c_float] + [_c_int] * 4 + [_c_void_p, _c_void_p, _c_size_t,
                                                        _c_void_p]),
    "kvzap_attend_decode": (_c_int, [_c_void_p] * 3 + [_c_int64] + [_c_void_p] * 5 +
                            [_c_int, _c_int, _c_float, _c_void_p] + [_c_int] * 4 +
                            [_c_void_p, _c_size_t, _c_void_p]),
    "kvzap_assign_pages": (_c_int, [_c_void_p, _c_int, _c_int, _c_int, _c_int, _c_void_p, _c_int,
                                    _c_void_p, _c_int, _c_void_p, _c_void_p, _c_size_t, _c_void_p]),
    "kvzap_extend_pages": (_c_int, [_c_void_p, _c_void_p, _c_int, _c_int, _c_int, _c_int, _c_void_p,
                                    _c_int, _c_void_p, _c_int, _c_void_p, _c_void_p, _c_size_t,
                                    _c_void_p]),
    "kvzap_decode_evict_paged": (_c_int, [_c_void_p] * 5 + [_c_int, _c_int] + [_c_void_p] * 5 +
                                 [_c_int, _c_void_p, _c_int, _c_int] + [_c_void_p] * 5 +
                                 [_c_float] + [_c_int] * 4 + [_c_void_p, _c_void_p, _c_size_t,
                                                              _c_void_p]),
    "kvzap_compact_paged": (_c_int, [_c_void_p] * 6 + [_c_int, _c_int, _c_void_p, _c_void_p] +
                            [_c_int] * 5 + [_c_void_p]),
    "kvzap_attend_decode_paged": (_c_int, [_c_void_p] * 3 + [_c_int, _c_void_p, _c_int, _c_int] +
                                  [_c_void_p] * 4 + [_c_int, _c_int, _c_float, _c_void_p] +
                                  [_c_int] * 4 + [_c_void_p, _c_size_t, _c_void_p]),
}


class KvzapError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().kvzap_status_string(status).decode()
        super().__init__(f"{where} failed: {msg} (status {status})")


_lib = None


def lib() -> ctypes.CDLL:
    """Load libkvzap.so (built by `python -m paper_2601_07891_amd.build`)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with __graft_entry__.build() "
                "or `python paper_2601_07891_amd/build.py`; there is no fallback path")
        handle = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(handle, name)
            fn.restype = res
            fn.argtypes = args
        _lib = handle
    return _lib


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    if isinstance(stream, torch.cuda.Stream):
        return stream.cuda_stream or None
    return int(stream) or None


def _check(t: Optional[torch.Tensor], dtype, name: str, optional: bool = False):
    if t is None:
        if optional:
            return
        raise ValueError(f"{name} is required")
    if not t.is_cuda:
        raise ValueError(f"{name} must be a device tensor")
    if t.dtype != dtype:
        raise ValueError(f"{name} must be {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")


def _workspace(nbytes: int, device, workspace: Optional[torch.Tensor], stream=None):
    if nbytes == 0:
        return workspace, (0 if workspace is None else workspace.numel() * workspace.element_size())
    if workspace is None:
        workspace = torch.empty(nbytes, dtype=torch.uint8, device=device)
        # A temporary allocated here goes back to torch's caching allocator when the wrapper
        # returns, while the kernels enqueued on `stream` may still be using it: tell the
        # allocator, so that the block is not handed out again before that stream gets there
        # (a no-op cost when `stream` is the current stream)
        if stream is not None:
            if not isinstance(stream, torch.cuda.Stream):
                stream = torch.cuda.ExternalStream(int(stream), device=device) if int(stream) \
                    else torch.cuda.default_stream(device)
            workspace.record_stream(stream)
    return workspace, workspace.numel() * workspace.element_size()


def kvzap_workspace_bytes(which_call: int, B: int, T: int, Dh: int, M: int, H: int) -> int:
    return int(lib().kvzap_workspace_bytes(which_call, B, T, Dh, M, H))


def kvzap_score(hidden: torch.Tensor, W1: torch.Tensor, b1: Optional[torch.Tensor],
                W2: Optional[torch.Tensor], b2: Optional[torch.Tensor],
                scores: Optional[torch.Tensor] = None,
                workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """hidden bf16 [B,T,Dh]; MLP: W1 [M,Dh], b1 [M], W2 [H,M], b2 [H];
    linear: W1 [H,Dh], b1 [H], W2 = b2 = None.  Returns scores fp32 [B,H,T]."""
    bf = torch.bfloat16
    _check(hidden, bf, "hidden"); _check(W1, bf, "W1")
    _check(b1, bf, "b1", True); _check(W2, bf, "W2", True); _check(b2, bf, "b2", True)
    B, T, Dh = hidden.shape
    if W2 is not None:
        M, H = W1.shape[0], W2.shape[0]
        if W1.shape != (M, Dh) or W2.shape != (H, M):
            raise ValueError("W1 must be [M,Dh] and W2 [H,M]")
        if (b1 is not None and b1.shape != (M,)) or (b2 is not None and b2.shape != (H,)):
            raise ValueError("b1 must be [M] and b2 [H]")
    else:
        M, H = 0, W1.shape[0]
        if W1.shape != (H, Dh) or (b1 is not None and b1.shape != (H,)):
            raise ValueError("W1 must be [H,Dh] and b1 [H]")
    if scores is None:
        scores = torch.empty((B, H, T), dtype=torch.float32, device=hidden.device)
    _check(scores, torch.float32, "scores")
    if scores.shape != (B, H, T):
        raise ValueError("scores must be [B,H,T]")
    ws, ws_bytes = _workspace(kvzap_workspace_bytes(CALL_SCORE, B, T, Dh, M, H), hidden.device,
                              workspace, stream)
    rc = lib().kvzap_score(_ptr(hidden), _ptr(W1), _ptr(b1), _ptr(W2), _ptr(b2), _ptr(scores),
                           B, T, Dh, M, H, _ptr(ws), ws_bytes, _stream(stream))
    if rc != 0:
        raise KvzapError(rc, "kvzap_score")
    return scores


def kvzap_mask(scores: torch.Tensor, tau: float, window: int,
               seq_lens: Optional[torch.Tensor] = None,
               keep_idx: Optional[torch.Tensor] = None,
               lengths: Optional[torch.Tensor] = None,
               offsets: Optional[torch.Tensor] = None,
               workspace: Optional[torch.Tensor] = None, stream=None
               ) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    """scores fp32 [B,H,T] -> (keep_idx int32 [B*H*T] packed, lengths int32 [B,H],
    offsets int64 [B*H+1])."""
    _check(scores, torch.float32, "scores")
    _check(seq_lens, torch.int32, "seq_lens", True)
    B, H, T = scores.shape
    dev = scores.device
    if keep_idx is None:
        keep_idx = torch.empty(B * H * T, dtype=torch.int32, device=dev)
    if lengths is None:
        lengths = torch.empty((B, H), dtype=torch.int32, device=dev)
    if offsets is None:
        offsets = torch.empty(B * H + 1, dtype=torch.int64, device=dev)
    _check(keep_idx, torch.int32, "keep_idx"); _check(lengths, torch.int32, "lengths")
    _check(offsets, torch.int64, "offsets")
    if keep_idx.numel() < B * H * T or lengths.numel() != B * H or offsets.numel() != B * H + 1:
        raise ValueError("output buffers have the wrong size")
    ws, ws_bytes = _workspace(kvzap_workspace_bytes(CALL_MASK, B, T, 0, 0, H), dev, workspace, stream)
    rc = lib().kvzap_mask(_ptr(scores), float(tau), int(window), _ptr(seq_lens), B, H, T,
                          _ptr(keep_idx), _ptr(lengths), _ptr(offsets), _ptr(ws), ws_bytes,
                          _stream(stream))
    if rc != 0:
        raise KvzapError(rc, "kvzap_mask")
    return keep_idx, lengths, offsets


def kvzap_mask_static(scores: torch.Tensor, tau: float, window: int,
                      seq_lens: Optional[torch.Tensor], keep_idx: torch.Tensor,
                      lengths: torch.Tensor, offsets: torch.Tensor, stream=None) -> None:
    """kvzap_mask on the library's built-in scratch: the caller passes every output buffer and
    this wrapper allocates nothing either."""
    _check(scores, torch.float32, "scores")
    _check(seq_lens, torch.int32, "seq_lens", True)
    _check(keep_idx, torch.int32, "keep_idx"); _check(lengths, torch.int32, "lengths")
    _check(offsets, torch.int64, "offsets")
    B, H, T = scores.shape
    if keep_idx.numel() < B * H * T or lengths.numel() != B * H or offsets.numel() != B * H + 1:
        raise ValueError("output buffers have the wrong size")
    rc = lib().kvzap_mask_static(_ptr(scores), float(tau), int(window), _ptr(seq_lens), B, H, T,
                                 _ptr(keep_idx), _ptr(lengths), _ptr(offsets), _stream(stream))
    if rc != 0:
        raise KvzapError(rc, "kvzap_mask_static")


def kvzap_compact(K: torch.Tensor, V: torch.Tensor, keep_idx: torch.Tensor,
                  lengths: torch.Tensor, offsets: torch.Tensor,
                  K_out: Optional[torch.Tensor] = None, V_out: Optional[torch.Tensor] = None,
                  cap_rows: Optional[int] = None, stream=None
                  ) -> Tuple[torch.Tensor, torch.Tensor]:
    """K, V bf16 [B,H,T,D] -> packed (K_out, V_out) bf16 [cap_rows, D]."""
    bf = torch.bfloat16
    _check(K, bf, "K"); _check(V, bf, "V")
    _check(keep_idx, torch.int32, "keep_idx"); _check(lengths, torch.int32, "lengths")
    _check(offsets, torch.int64, "offsets")
    B, H, T, D = K.shape
    if V.shape != K.shape:
        raise ValueError("K and V must have the same shape")
    if cap_rows is None:
        cap_rows = B * H * T if K_out is None else K_out.shape[0]
    if K_out is None:
        K_out = torch.empty((cap_rows, D), dtype=bf, device=K.device)
    if V_out is None:
        V_out = torch.empty((cap_rows, D), dtype=bf, device=K.device)
    _check(K_out, bf, "K_out"); _check(V_out, bf, "V_out")
    if K_out.shape[0] < cap_rows or V_out.shape[0] < cap_rows or K_out.shape[1] != D:
        raise ValueError("K_out / V_out smaller than cap_rows")
    rc = lib().kvzap_compact(_ptr(K), _ptr(V), _ptr(keep_idx), _ptr(lengths), _ptr(offsets),
                             _ptr(K_out), _ptr(V_out), int(cap_rows), B, H, T, D,
                             _stream(stream))
    if rc != 0:
        raise KvzapError(rc, "kvzap_compact")
    return K_out, V_out


class DecodeState:
    """Device buffers of the decode cache layout described in include/kvzap.h
    (allocation and bookkeeping only; all updates happen in the library)."""

    def __init__(self, B: int, H: int, D: int, window: int, slab_capacity, device):
        cap = torch.as_tensor(slab_capacity, dtype=torch.int32).reshape(B * H)
        off = torch.zeros(B * H, dtype=torch.int64)
        off[1:] = torch.cumsum(cap.to(torch.int64), 0)[:-1]
        total = int(cap.to(torch.int64).sum())
        bf = torch.bfloat16
        self.B, self.H, self.D, self.window = B, H, D, window
        self.slab_capacity = cap.to(device)
        self.slab_offsets = off.to(device)
        self.K_prefix = torch.zeros((max(total, 1), D), dtype=bf, device=device)
        self.V_prefix = torch.zeros((max(total, 1), D), dtype=bf, device=device)
        self.prefix_pos = torch.full((max(total, 1),), -1, dtype=torch.int32, device=device)
        w = max(window, 1)
        self.K_ring = torch.zeros((B, H, w, D), dtype=bf, device=device)
        self.V_ring = torch.zeros((B, H, w, D), dtype=bf, device=device)
        self.score_ring = torch.zeros((B, H, w), dtype=torch.float32, device=device)
        self.lengths = torch.zeros((B, H), dtype=torch.int32, device=device)
        self.seq_pos = torch.zeros(B, dtype=torch.int32, device=device)
        self.error_flag = torch.zeros(4, dtype=torch.int32, device=device)


def kvzap_decode_evict(hidden_new: torch.Tensor, W1: torch.Tensor, b1, W2, b2,
                       k_new: torch.Tensor, v_new: torch.Tensor, state: DecodeState,
                       tau: float, workspace: Optional[torch.Tensor] = None,
                       stream=None) -> None:
    """One decode step of one layer: hidden_new bf16 [B,Dh], k_new/v_new bf16 [B,H,D];
    `state` is updated in place."""
    bf = torch.bfloat16
    _check(hidden_new, bf, "hidden_new"); _check(W1, bf, "W1"); _check(b1, bf, "b1", True)
    _check(W2, bf, "W2", True); _check(b2, bf, "b2", True)
    _check(k_new, bf, "k_new"); _check(v_new, bf, "v_new")
    B, Dh = hidden_new.shape
    M = W1.shape[0] if W2 is not None else 0
    st = state
    if (B, st.H, st.D) != tuple(k_new.shape) or k_new.shape != v_new.shape or B != st.B:
        raise ValueError("k_new / v_new must be [B,H,D] matching the state")
    ws, ws_bytes = _workspace(
        kvzap_workspace_bytes(CALL_DECODE_EVICT, B, 1, Dh, M, st.H), hidden_new.device, workspace, stream)
    ring = st.window > 0
    rc = lib().kvzap_decode_evict(
        _ptr(hidden_new), _ptr(W1), _ptr(b1), _ptr(W2), _ptr(b2), Dh, M,
        _ptr(k_new), _ptr(v_new), _ptr(st.K_prefix), _ptr(st.V_prefix), _ptr(st.prefix_pos),
        _ptr(st.slab_offsets), _ptr(st.slab_capacity),
        _ptr(st.K_ring) if ring else None, _ptr(st.V_ring) if ring else None,
        _ptr(st.score_ring) if ring else None, _ptr(st.lengths), _ptr(st.seq_pos),
        float(tau), int(st.window), B, st.H, st.D, _ptr(st.error_flag),
        _ptr(ws), ws_bytes, _stream(stream))
    if rc != 0:
        raise KvzapError(rc, "kvzap_decode_evict")


def kvzap_attend_decode(q: torch.Tensor, K_rows: torch.Tensor, V_rows: torch.Tensor,
                        row_offsets: torch.Tensor, lengths: torch.Tensor,
                        K_ring: Optional[torch.Tensor], V_ring: Optional[torch.Tensor],
                        seq_pos: Optional[torch.Tensor], window: int, max_rows: int,
                        scale: float, out: Optional[torch.Tensor] = None,
                        workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """q bf16 [B,HQ,D]; K_rows/V_rows bf16 [total_rows,D]; row_offsets int64 [B*H];
    lengths int32 [B,H]; ring tensors bf16 [B,H,window,D] and seq_pos int32 [B] (None when
    window == 0).  Returns out bf16 [B,HQ,D]."""
    bf = torch.bfloat16
    _check(q, bf, "q"); _check(K_rows, bf, "K_rows"); _check(V_rows, bf, "V_rows")
    _check(row_offsets, torch.int64, "row_offsets"); _check(lengths, torch.int32, "lengths")
    B, HQ, D = q.shape
    if lengths.dim() != 2 or lengths.shape[0] != B:
        raise ValueError("lengths must be [B,H]")
    H = lengths.shape[1]
    if row_offsets.numel() != B * H:
        raise ValueError("row_offsets must have B*H entries")
    if K_rows.dim() != 2 or K_rows.shape[1] != D or K_rows.shape != V_rows.shape:
        raise ValueError("K_rows and V_rows must both be [total_rows, D]")
    if window > 0:
        _check(K_ring, bf, "K_ring"); _check(V_ring, bf, "V_ring")
        _check(seq_pos, torch.int32, "seq_pos")
        if tuple(K_ring.shape) != (B, H, window, D) or K_ring.shape != V_ring.shape:
            raise ValueError("K_ring and V_ring must be [B,H,window,D]")
        if seq_pos.numel() != B:
            raise ValueError("seq_pos must have B entries")
    if out is None:
        out = torch.empty((B, HQ, D), dtype=bf, device=q.device)
    else:
        _check(out, bf, "out")
        if out.shape != q.shape:
            raise ValueError("out must be [B,HQ,D]")
    ws, ws_bytes = _workspace(
        kvzap_workspace_bytes(CALL_ATTEND_DECODE, B, int(max_rows), HQ, int(window), H),
        q.device, workspace, stream)
    ring = window > 0
    total_rows = K_rows.shape[0]
    rc = lib().kvzap_attend_decode(
        _ptr(q), _ptr(K_rows) if total_rows else None, _ptr(V_rows) if total_rows else None,
        total_rows, _ptr(row_offsets), _ptr(lengths),
        _ptr(K_ring) if ring else None, _ptr(V_ring) if ring else None,
        _ptr(seq_pos) if ring else None, int(window), int(max_rows), float(scale), _ptr(out),
        B, H, HQ, D, _ptr(ws), ws_bytes, _stream(stream))
    if rc != 0:
        raise KvzapError(rc, "kvzap_attend_decode")
    return out


def kvzap_assign_pages(lengths: torch.Tensor, page_rows: int, free_pages: torch.Tensor,
                       max_pages: int, reserve_rows: int = 0,
                       block_table: Optional[torch.Tensor] = None,
                       result: Optional[torch.Tensor] = None,
                       workspace: Optional[torch.Tensor] = None, stream=None):
    """lengths int32 [B,H]; free_pages int32 [n_free].  Returns (block_table int32
    [B*H, max_pages], result int32 [2] = (pages taken, status)), both on the device."""
    _check(lengths, torch.int32, "lengths"); _check(free_pages, torch.int32, "free_pages")
    B, H = lengths.shape
    if block_table is None:
        block_table = torch.empty((B * H, max_pages), dtype=torch.int32, device=lengths.device)
    else:
        _check(block_table, torch.int32, "block_table")
        if tuple(block_table.shape) != (B * H, max_pages):
            raise ValueError("block_table must be [B*H, max_pages]")
    if result is None:
        result = torch.empty(4, dtype=torch.int32, device=lengths.device)
    else:
        _check(result, torch.int32, "result")
    ws, ws_bytes = _workspace(kvzap_workspace_bytes(CALL_ASSIGN_PAGES, B, 1, 0, 0, H),
                              lengths.device, workspace, stream)
    n_free = free_pages.numel()
    rc = lib().kvzap_assign_pages(_ptr(lengths), B, H, int(page_rows), int(reserve_rows),
                                  _ptr(free_pages) if n_free else None, n_free,
                                  _ptr(block_table), int(max_pages), _ptr(result),
                                  _ptr(ws), ws_bytes, _stream(stream))
    if rc != 0:
        raise KvzapError(rc, "kvzap_assign_pages")
    return block_table, result


def kvzap_compact_paged(K: torch.Tensor, V: torch.Tensor, keep_idx: torch.Tensor,
                        lengths: torch.Tensor, offsets: torch.Tensor,
                        block_table: torch.Tensor, page_rows: int, K_pool: torch.Tensor,
                        V_pool: torch.Tensor, stream=None) -> None:
    """K, V bf16 [B,H,T,D]; pools bf16 [num_pages, page_rows, D], written in place."""
    bf = torch.bfloat16
    _check(K, bf, "K"); _check(V, bf, "V"); _check(K_pool, bf, "K_pool"); _check(V_pool, bf, "V_pool")
    _check(keep_idx, torch.int32, "keep_idx"); _check(lengths, torch.int32, "lengths")
    _check(offsets, torch.int64, "offsets"); _check(block_table, torch.int32, "block_table")
    B, H, T, D = K.shape
    if V.shape != K.shape or K_pool.shape != V_pool.shape:
        raise ValueError("K/V and the two pools must have matching shapes")
    if K_pool.dim() != 3 or K_pool.shape[1] != page_rows or K_pool.shape[2] != D:
        raise ValueError("pools must be [num_pages, page_rows, D]")
    if block_table.dim() != 2 or block_table.shape[0] != B * H:
        raise ValueError("block_table must be [B*H, max_pages]")
    num_pages = K_pool.shape[0]
    rc = lib().kvzap_compact_paged(_ptr(K), _ptr(V), _ptr(keep_idx), _ptr(lengths), _ptr(offsets),
                                   _ptr(block_table), block_table.shape[1], int(page_rows),
                                   _ptr(K_pool) if num_pages else None,
                                   _ptr(V_pool) if num_pages else None, num_pages,
                                   B, H, T, D, _stream(stream))
    if rc != 0:
        raise KvzapError(rc, "kvzap_compact_paged")


def kvzap_attend_decode_paged(q: torch.Tensor, K_pool: torch.Tensor, V_pool: torch.Tensor,
                              block_table: torch.Tensor, page_rows: int, lengths: torch.Tensor,
                              K_ring: Optional[torch.Tensor], V_ring: Optional[torch.Tensor],
                              seq_pos: Optional[torch.Tensor], window: int, max_rows: int,
                              scale: float, out: Optional[torch.Tensor] = None,
                              workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """kvzap_attend_decode over pools bf16 [num_pages, page_rows, D] and a block table int32
    [B*H, max_pages]."""
    bf = torch.bfloat16
    _check(q, bf, "q"); _check(K_pool, bf, "K_pool"); _check(V_pool, bf, "V_pool")
    _check(block_table, torch.int32, "block_table"); _check(lengths, torch.int32, "lengths")
    B, HQ, D = q.shape
    if lengths.dim() != 2 or lengths.shape[0] != B:
        raise ValueError("lengths must be [B,H]")
    H = lengths.shape[1]
    if K_pool.dim() != 3 or K_pool.shape[1:] != (page_rows, D) or K_pool.shape != V_pool.shape:
        raise ValueError("pools must both be [num_pages, page_rows, D]")
    if block_table.dim() != 2 or block_table.shape[0] != B * H:
        raise ValueError("block_table must be [B*H, max_pages]")
    if window > 0:
        _check(K_ring, bf, "K_ring"); _check(V_ring, bf, "V_ring")
        _check(seq_pos, torch.int32, "seq_pos")
        if tuple(K_ring.shape) != (B, H, window, D) or K_ring.shape != V_ring.shape:
            raise ValueError("K_ring and V_ring must be [B,H,window,D]")
    if out is None:
        out = torch.empty((B, HQ, D), dtype=bf, device=q.device)
    else:
        _check(out, bf, "out")
    ws, ws_bytes = _workspace(
        kvzap_workspace_bytes(CALL_ATTEND_DECODE, B, int(max_rows), HQ, int(window), H),
        q.device, workspace, stream)
    ring = window > 0
    num_pages = K_pool.shape[0]
    rc = lib().kvzap_attend_decode_paged(
        _ptr(q), _ptr(K_pool) if num_pages else None, _ptr(V_pool) if num_pages else None,
        num_pages, _ptr(block_table), block_table.shape[1], int(page_rows), _ptr(lengths),
        _ptr(K_ring) if ring else None, _ptr(V_ring) if ring else None,
        _ptr(seq_pos) if ring else None, int(window), int(max_rows), float(scale), _ptr(out),
        B, H, HQ, D, _ptr(ws), ws_bytes, _stream(stream))
    if rc != 0:
        raise KvzapError(rc, "kvzap_attend_decode_paged")
    return out


def kvzap_extend_pages(lengths: torch.Tensor, page_counts: torch.Tensor, page_rows: int,
                       free_pages: torch.Tensor, block_table: torch.Tensor,
                       reserve_rows: int = 0, result: Optional[torch.Tensor] = None,
                       workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Appends pages behind the page_counts[b,h] a head owns (both updated in place).
    Returns result int32 [2] = (pages taken, status) on the device."""
    _check(lengths, torch.int32, "lengths"); _check(page_counts, torch.int32, "page_counts")
    _check(free_pages, torch.int32, "free_pages"); _check(block_table, torch.int32, "block_table")
    B, H = lengths.shape
    if page_counts.numel() != B * H or block_table.dim() != 2 or block_table.shape[0] != B * H:
        raise ValueError("page_counts must have B*H entries and block_table B*H rows")
    if result is None:
        result = torch.empty(4, dtype=torch.int32, device=lengths.device)
    ws, ws_bytes = _workspace(kvzap_workspace_bytes(CALL_ASSIGN_PAGES, B, 1, 0, 0, H),
                              lengths.device, workspace, stream)
    n_free = free_pages.numel()
    rc = lib().kvzap_extend_pages(_ptr(lengths), _ptr(page_counts), B, H, int(page_rows),
                                  int(reserve_rows), _ptr(free_pages) if n_free else None, n_free,
                                  _ptr(block_table), block_table.shape[1], _ptr(result),
                                  _ptr(ws), ws_bytes, _stream(stream))
    if rc != 0:
        raise KvzapError(rc, "kvzap_extend_pages")
    return result


class PagedDecodeState:
    """Device buffers of the paged decode cache described in include/kvzap.h (allocation
    only; all updates happen in the library)."""

    def __init__(self, B: int, H: int, D: int, window: int, page_rows: int, num_pages: int,
                 max_pages: int, device):
        bf = torch.bfloat16
        self.B, self.H, self.D, self.window = B, H, D, window
        self.page_rows, self.num_pages, self.max_pages = page_rows, num_pages, max_pages
        n = max(num_pages, 1)
        self.K_pool = torch.zeros((n, page_rows, D), dtype=bf, device=device)
        self.V_pool = torch.zeros((n, page_rows, D), dtype=bf, device=device)
        self.pos_pool = torch.full((n, page_rows), -1, dtype=torch.int32, device=device)
        self.block_table = torch.full((B * H, max_pages), -1, dtype=torch.int32, device=device)
        self.page_counts = torch.zeros((B, H), dtype=torch.int32, device=device)
        w = max(window, 1)
        self.K_ring = torch.zeros((B, H, w, D), dtype=bf, device=device)
        self.V_ring = torch.zeros((B, H, w, D), dtype=bf, device=device)
        self.score_ring = torch.zeros((B, H, w), dtype=torch.float32, device=device)
        self.lengths = torch.zeros((B, H), dtype=torch.int32, device=device)
        self.seq_pos = torch.zeros(B, dtype=torch.int32, device=device)
        self.error_flag = torch.zeros(4, dtype=torch.int32, device=device)


def kvzap_decode_evict_paged(hidden_new: torch.Tensor, W1: torch.Tensor, b1, W2, b2,
                             k_new: torch.Tensor, v_new: torch.Tensor, state: PagedDecodeState,
                             tau: float, workspace: Optional[torch.Tensor] = None,
                             stream=None) -> None:
    """One decode step of one layer on the paged cache; `state` is updated in place."""
    bf = torch.bfloat16
    _check(hidden_new, bf, "hidden_new"); _check(W1, bf, "W1"); _check(b1, bf, "b1", True)
    _check(W2, bf, "W2", True); _check(b2, bf, "b2", True)
    _check(k_new, bf, "k_new"); _check(v_new, bf, "v_new")
    B, Dh = hidden_new.shape
    M = W1.shape[0] if W2 is not None else 0
    st = state
    if (B, st.H, st.D) != tuple(k_new.shape) or k_new.shape != v_new.shape or B != st.B:
        raise ValueError("k_new / v_new must be [B,H,D] matching the state")
    ws, ws_bytes = _workspace(
        kvzap_workspace_bytes(CALL_DECODE_EVICT, B, 1, Dh, M, st.H), hidden_new.device, workspace, stream)
    ring = st.window > 0
    rc = lib().kvzap_decode_evict_paged(
        _ptr(hidden_new), _ptr(W1), _ptr(b1), _ptr(W2), _ptr(b2), Dh, M,
        _ptr(k_new), _ptr(v_new), _ptr(st.K_pool), _ptr(st.V_pool), _ptr(st.pos_pool),
        st.num_pages, _ptr(st.block_table), st.max_pages, st.page_rows,
        _ptr(st.K_ring) if ring else None, _ptr(st.V_ring) if ring else None,
        _ptr(st.score_ring) if ring else None, _ptr(st.lengths), _ptr(st.seq_pos),
        float(tau), int(st.window), B, st.H, st.D, _ptr(st.error_flag),
        _ptr(ws), ws_bytes, _stream(stream))
    if rc != 0:
        raise KvzapError(rc, "kvzap_decode_evict_paged")


def kvzap_topk_threshold(scores: torch.Tensor, window: int, k: int, per_layer: bool,
                         seq_lens: Optional[torch.Tensor] = None,
                         tau_out: Optional[torch.Tensor] = None,
                         workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """scores fp32 [B,H,T] -> tau fp32 [B,H]: the k-th largest non-window score per head, or
    per sequence over its pooled heads."""
    _check(scores, torch.float32, "scores"); _check(seq_lens, torch.int32, "seq_lens", True)
    B, H, T = scores.shape
    if tau_out is None:
        tau_out = torch.empty((B, H), dtype=torch.float32, device=scores.device)
    else:
        _check(tau_out, torch.float32, "tau_out")
    ws, ws_bytes = _workspace(
        kvzap_workspace_bytes(CALL_TOPK_THRESHOLD, B, T, 0, 1 if per_layer else 0, H),
        scores.device, workspace, stream)
    rc = lib().kvzap_topk_threshold(_ptr(scores), int(window), _ptr(seq_lens), int(k),
                                    1 if per_layer else 0, B, H, T, _ptr(tau_out), _ptr(ws),
                                    ws_bytes, _stream(stream))
    if rc != 0:
        raise KvzapError(rc, "kvzap_topk_threshold")
    return tau_out


def kvzap_mask_per_head(scores: torch.Tensor, tau: torch.Tensor, window: int,
                        seq_lens: Optional[torch.Tensor] = None,
                        keep_idx: Optional[torch.Tensor] = None,
                        lengths: Optional[torch.Tensor] = None,
                        offsets: Optional[torch.Tensor] = None,
                        workspace: Optional[torch.Tensor] = None, stream=None):
    """kvzap_mask with tau fp32 [B,H] on the device.  Returns (keep_idx, lengths, offsets)."""
    _check(scores, torch.float32, "scores"); _check(tau, torch.float32, "tau")
    _check(seq_lens, torch.int32, "seq_lens", True)
    B, H, T = scores.shape
    if tau.numel() != B * H:
        raise ValueError("tau must have B*H entries")
    dev = scores.device
    if keep_idx is None:
        keep_idx = torch.empty(B * H * T, dtype=torch.int32, device=dev)
    if lengths is None:
        lengths = torch.empty((B, H), dtype=torch.int32, device=dev)
    if offsets is None:
        offsets = torch.empty(B * H + 1, dtype=torch.int64, device=dev)
    ws, ws_bytes = _workspace(kvzap_workspace_bytes(CALL_MASK, B, T, 0, 0, H), dev, workspace, stream)
    rc = lib().kvzap_mask_per_head(_ptr(scores), _ptr(tau), int(window), _ptr(seq_lens), B, H, T,
                                   _ptr(keep_idx), _ptr(lengths), _ptr(offsets), _ptr(ws),
                                   ws_bytes, _stream(stream))
    if rc != 0:
        raise KvzapError(rc, "kvzap_mask_per_head")
    return keep_idx, lengths, offsets


def kvzap_teacher_scores(q: torch.Tensor, k: torch.Tensor, T: int, scale: float,
                         vnorm: Optional[torch.Tensor] = None,
                         hnorm: Optional[torch.Tensor] = None,
                         log_s: Optional[torch.Tensor] = None,
                         workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """q bf16 [HQ,Tq,D] (queries of the repeated prompt), k bf16 [H,Tk,D] (all keys of the
    extended prompt), vnorm fp32 [H,T], hnorm fp32 [Tq] -> log scores fp32 [H,T]."""
    bf = torch.bfloat16
    _check(q, bf, "q"); _check(k, bf, "k")
    _check(vnorm, torch.float32, "vnorm", True); _check(hnorm, torch.float32, "hnorm", True)
    HQ, Tq, D = q.shape
    H, Tk, Dk = k.shape
    if Dk != D:
        raise ValueError("q and k must have the same head dimension")
    if vnorm is not None and tuple(vnorm.shape) != (H, T):
        raise ValueError("vnorm must be [H,T]")
    if hnorm is not None and hnorm.numel() != Tq:
        raise ValueError("hnorm must have Tq entries")
    if log_s is None:
        log_s = torch.empty((H, T), dtype=torch.float32, device=q.device)
    else:
        _check(log_s, torch.float32, "log_s")
    ws, ws_bytes = _workspace(kvzap_workspace_bytes(CALL_TEACHER_SCORES, 1, int(T), HQ, Tq, H),
                              q.device, workspace, stream)
    rc = lib().kvzap_teacher_scores(_ptr(q), _ptr(k), _ptr(vnorm), _ptr(hnorm), float(scale),
                                    _ptr(log_s), H, HQ, Tq, Tk, int(T), D, _ptr(ws), ws_bytes,
                                    _stream(stream))
    if rc != 0:
        raise KvzapError(rc, "kvzap_teacher_scores")
    return log_s


def kvzap_mask_compact(scores: torch.Tensor, tau: float, window: int, K: torch.Tensor,
                       V: torch.Tensor, seq_lens: Optional[torch.Tensor] = None,
                       keep_idx: Optional[torch.Tensor] = None,
                       lengths: Optional[torch.Tensor] = None,
                       offsets: Optional[torch.Tensor] = None,
                       K_out: Optional[torch.Tensor] = None, V_out: Optional[torch.Tensor] = None,
                       cap_rows: Optional[int] = None,
                       workspace: Optional[torch.Tensor] = None, stream=None):
    """kvzap_mask + kvzap_compact in one library call.  Returns (keep_idx, lengths, offsets,
    K_out, V_out) as the two separate calls would."""
    bf = torch.bfloat16
    _check(scores, torch.float32, "scores"); _check(K, bf, "K"); _check(V, bf, "V")
    _check(seq_lens, torch.int32, "seq_lens", True)
    B, H, T = scores.shape
    if tuple(K.shape[:3]) != (B, H, T) or K.shape != V.shape:
        raise ValueError("K and V must be [B,H,T,D]")
    D = K.shape[3]
    dev = scores.device
    if keep_idx is None:
        keep_idx = torch.empty(B * H * T, dtype=torch.int32, device=dev)
    if lengths is None:
        lengths = torch.empty((B, H), dtype=torch.int32, device=dev)
    if offsets is None:
        offsets = torch.empty(B * H + 1, dtype=torch.int64, device=dev)
    if cap_rows is None:
        cap_rows = B * H * T if K_out is None else K_out.shape[0]
    if K_out is None:
        K_out = torch.empty((cap_rows, D), dtype=bf, device=dev)
    if V_out is None:
        V_out = torch.empty((cap_rows, D), dtype=bf, device=dev)
    _check(keep_idx, torch.int32, "keep_idx"); _check(lengths, torch.int32, "lengths")
    _check(offsets, torch.int64, "offsets"); _check(K_out, bf, "K_out"); _check(V_out, bf, "V_out")
    if keep_idx.numel() < B * H * T or lengths.numel() != B * H or offsets.numel() != B * H + 1:
        raise ValueError("output buffers have the wrong size")
    if K_out.shape[0] < cap_rows or V_out.shape[0] < cap_rows or K_out.shape[1] != D or V_out.shape[1] != D:
        raise ValueError("K_out and V_out must be [>= cap_rows, D]")
    ws, ws_bytes = _workspace(max(kvzap_workspace_bytes(CALL_MASK_COMPACT, B, T, 0, 0, H), 256), dev,
                              workspace, stream)
    rc = lib().kvzap_mask_compact(_ptr(scores), float(tau), int(window), _ptr(seq_lens), _ptr(K),
                                  _ptr(V), _ptr(keep_idx), _ptr(lengths), _ptr(offsets), _ptr(K_out),
                                  _ptr(V_out), int(cap_rows), B, H, T, D, _ptr(ws), ws_bytes,
                                  _stream(stream))
    if rc != 0:
        raise KvzapError(rc, "kvzap_mask_compact")
    return keep_idx, lengths, offsets, K_out, V_out


def kvzap_compress(hidden: torch.Tensor, W1: torch.Tensor, b1, W2, b2, K: torch.Tensor,
                   V: torch.Tensor, tau: float, window: int,
                   seq_lens: Optional[torch.Tensor] = None,
                   workspace: Optional[torch.Tensor] = None, stream=None):
    """Algorithm 1 for one layer in one library call.  Returns (scores, keep_idx, lengths,
    offsets, K_out, V_out) as the three separate calls would."""
    bf = torch.bfloat16
    _check(hidden, bf, "hidden"); _check(W1, bf, "W1"); _check(b1, bf, "b1", True)
    _check(W2, bf, "W2", True); _check(b2, bf, "b2", True); _check(K, bf, "K"); _check(V, bf, "V")
    _check(seq_lens, torch.int32, "seq_lens", True)
    B, T, Dh = hidden.shape
    M = W1.shape[0] if W2 is not None else 0
    H = W2.shape[0] if W2 is not None else W1.shape[0]
    if tuple(K.shape[:3]) != (B, H, T) or K.shape != V.shape:
        raise ValueError("K and V must be [B,H,T,D]")
    D = K.shape[3]
    dev = hidden.device
    scores = torch.empty((B, H, T), dtype=torch.float32, device=dev)
    keep_idx = torch.empty(B * H * T, dtype=torch.int32, device=dev)
    lengths = torch.empty((B, H), dtype=torch.int32, device=dev)
    offsets = torch.empty(B * H + 1, dtype=torch.int64, device=dev)
    K_out = torch.empty((B * H * T, D), dtype=bf, device=dev)
    V_out = torch.empty((B * H * T, D), dtype=bf, device=dev)
    ws, ws_bytes = _workspace(max(kvzap_workspace_bytes(CALL_COMPRESS, B, T, Dh, M, H), 256), dev,
                              workspace, stream)
    rc = lib().kvzap_compress(_ptr(hidden), _ptr(W1), _ptr(b1), _ptr(W2), _ptr(b2), _ptr(K), _ptr(V),
                              float(tau), int(window), _ptr(seq_lens), _ptr(scores), _ptr(keep_idx),
                              _ptr(lengths), _ptr(offsets), _ptr(K_out), _ptr(V_out), B * H * T,
                              B, T, Dh, M, H, D, _ptr(ws), ws_bytes, _stream(stream))
    if rc != 0:
        raise KvzapError(rc, "kvzap_compress")
    return scores, keep_idx, lengths, offsets, K_out, V_out


def kvzap_prepare_scorer(W1: torch.Tensor, stream=None) -> torch.Tensor:
    """W1 bf16 [M,Dh] of an MLP surrogate -> the copy kvzap_score_prepared takes (opaque bytes)."""
    _check(W1, torch.bfloat16, "W1")
    M, Dh = W1.shape
    nbytes = max(kvzap_workspace_bytes(CALL_SCORE, 1, 1, Dh, M, 1), 256)
    out = torch.empty(nbytes, dtype=torch.uint8, device=W1.device)
    rc = lib().kvzap_prepare_scorer(_ptr(W1), Dh, M, _ptr(out), nbytes, _stream(stream))
    if rc != 0:
        raise KvzapError(rc, "kvzap_prepare_scorer")
    return out


def kvzap_prepare_scorer_rmsnorm(W1: torch.Tensor, gain: torch.Tensor, stream=None) -> torch.Tensor:
    """W1 bf16 [M,Dh] and the norm's gain bf16 [Dh] -> the copy kvzap_score_rmsnorm takes."""
    _check(W1, torch.bfloat16, "W1"); _check(gain, torch.bfloat16, "gain")
    M, Dh = W1.shape
    if gain.shape != (Dh,):
        raise ValueError("gain must be [Dh]")
    nbytes = max(kvzap_workspace_bytes(CALL_SCORE, 1, 1 << 20, Dh, M, 1), 256)
    out = torch.empty(nbytes, dtype=torch.uint8, device=W1.device)
    rc = lib().kvzap_prepare_scorer_rmsnorm(_ptr(W1), _ptr(gain), Dh, M, _ptr(out), nbytes,
                                            _stream(stream))
    if rc != 0:
        raise KvzapError(rc, "kvzap_prepare_scorer_rmsnorm")
    return out


def kvzap_score_rmsnorm(x: torch.Tensor, W1_prepared: torch.Tensor, gain: torch.Tensor, eps: float,
                        b1: Optional[torch.Tensor], W2: torch.Tensor, b2: Optional[torch.Tensor],
                        want_normed: bool = False, scores: Optional[torch.Tensor] = None,
                        rstd: Optional[torch.Tensor] = None, normed: Optional[torch.Tensor] = None,
                        stream=None):
    """The MLP surrogate on the un-normalised residual stream x bf16 [B,T,Dh].  Returns
    (scores fp32 [B,H,T], rstd fp32 [B,T], normed bf16 [B,T,Dh] or None)."""
    bf = torch.bfloat16
    _check(x, bf, "x"); _check(gain, bf, "gain"); _check(b1, bf, "b1", True); _check(W2, bf, "W2")
    _check(b2, bf, "b2", True)
    B, T, Dh = x.shape
    H, M = W2.shape
    if W1_prepared.dtype != torch.uint8 or W1_prepared.numel() < M * Dh * 2:
        raise ValueError("W1_prepared must come from kvzap_prepare_scorer_rmsnorm")
    if gain.shape != (Dh,):
        raise ValueError("gain must be [Dh]")
    if scores is None:
        scores = torch.empty((B, H, T), dtype=torch.float32, device=x.device)
    if rstd is None:
        rstd = torch.empty((B, T), dtype=torch.float32, device=x.device)
    if normed is None and want_normed:
        normed = torch.empty_like(x)
    _check(scores, torch.float32, "scores"); _check(rstd, torch.float32, "rstd")
    _check(normed, bf, "normed", True)
    if scores.shape != (B, H, T) or rstd.shape != (B, T) or (normed is not None and normed.shape != x.shape):
        raise ValueError("scores must be [B,H,T], rstd [B,T], normed like x")
    rc = lib().kvzap_score_rmsnorm(_ptr(x), _ptr(W1_prepared), _ptr(gain), float(eps), _ptr(b1),
                                   _ptr(W2), _ptr(b2), _ptr(scores), _ptr(rstd), _ptr(normed),
                                   B, T, Dh, M, H, _stream(stream))
    if rc != 0:
        raise KvzapError(rc, "kvzap_score_rmsnorm")
    return scores, rstd, normed


def kvzap_score_prepared(hidden: torch.Tensor, W1_prepared: torch.Tensor, b1, W2: torch.Tensor, b2,
                         scores: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """kvzap_score with W1 replaced by kvzap_prepare_scorer's output; no workspace."""
    bf = torch.bfloat16
    _check(hidden, bf, "hidden"); _check(W1_prepared, torch.uint8, "W1_prepared")
    _check(b1, bf, "b1", True); _check(W2, bf, "W2"); _check(b2, bf, "b2", True)
    B, T, Dh = hidden.shape
    H, M = W2.shape
    if W1_prepared.numel() < M * Dh * 2:
        raise ValueError("W1_prepared is smaller than M*Dh bf16 values")
    if scores is None:
        scores = torch.empty((B, H, T), dtype=torch.float32, device=hidden.device)
    _check(scores, torch.float32, "scores")
    if scores.shape != (B, H, T):
        raise ValueError("scores must be [B,H,T]")
    rc = lib().kvzap_score_prepared(_ptr(hidden), _ptr(W1_prepared), _ptr(b1), _ptr(W2), _ptr(b2),
                                    _ptr(scores), B, T, Dh, M, H, _stream(stream))
    if rc != 0:
        raise KvzapError(rc, "kvzap_score_prepared")
    return scores
