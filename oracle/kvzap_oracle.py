"""Float64 CPU oracle of the KVzap prune step (test infrastructure, not product).

What is computed follows the paper directly:

* surrogate forward   -- Sec. 3.3 and Sec. 4.1: a per-layer linear map D_h -> H,
  or an MLP D_h -> D_h/8 -> GELU -> H, applied independently at every position;
  weight shapes as in App. B (W1 in R^{D_h x D_h/8}, W2 in R^{D_h/8 x H}).
* threshold + window  -- Sec. 3.3 and Algorithm 1: the last `window` positions
  are forced to +inf, a KV pair is kept iff its score is >= tau.
* ragged gather       -- Algorithm 1: kept rows of K and V in row-major
  (head, position) order, hence a different length per head (Sec. 5).
* decode              -- caption of Algorithm 1: the same rule applied one
  token at a time with a buffer of the scores still inside the window.

Everything is the plain definition written out with numpy in float64, with no
blocking, fusion or reordering.  K/V rows are carried as raw uint16 bf16 bit
patterns so that the gather is a byte copy.  Readings taken where the paper is
silent are listed beside each function.

Parity pins (tests/test_oracle_*.py): tau=-inf identity, tau=+inf window only,
nested kept sets in tau, brute-force mask enumeration at tiny T, hand loops vs
the library GEMM / erf / nonzero, exact-integer inputs, GELU identities and the
second moment E[GELU(z)^2], the closed forms and printed percentages of App. B,
decode == prefill on the grown prefix, conservation of lengths/offsets; the
row normalisation against a hand loop, its unit-mean-square, scale-invariance
and identity cases (tests/test_oracle_rmsnorm.py).
Absolute score values for real prompts are "parity unpinned": the paper prints
none and its trained weights are not available here.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np
from scipy import special as _sp_special


# --------------------------------------------------------------------------
# bf16 bit patterns <-> float64 (exact: bf16 is the top half of an fp32)
# --------------------------------------------------------------------------
def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact up-cast of bf16 bit patterns (uint16) to float64."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    as_f32 = (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)
    return as_f32.astype(np.float64)


# --------------------------------------------------------------------------
# surrogate forward (Sec. 3.3, Sec. 4.1, App. B Eq. 5-6)
# --------------------------------------------------------------------------
def gelu(z: np.ndarray) -> np.ndarray:
    """Exact GELU, z * Phi(z), in float64 (Sec. 4.1 says only "GELU": the
    erf form is taken, not the tanh approximation)."""
    z = np.asarray(z, dtype=np.float64)
    return 0.5 * z * (1.0 + _sp_special.erf(z / math.sqrt(2.0)))


def score_linear(hidden: np.ndarray, W: np.ndarray,
                 b: Optional[np.ndarray] = None) -> np.ndarray:
    """KVzap-Linear (Sec. 4.1; App. B Eq. 6).

    hidden [T, D_h], W [D_h, H], b [H] or None -- float64 values.
    Returns scores [H, T]: the module's output is (T, H) (Sec. 4.1) while
    Algorithm 1 indexes positions on the last axis, so it is transposed here.
    """
    hidden = np.asarray(hidden, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    S = hidden @ W
    if b is not None:
        S = S + np.asarray(b, dtype=np.float64)[None, :]
    return np.ascontiguousarray(S.T)


def score_mlp(hidden: np.ndarray, W1: np.ndarray, b1: Optional[np.ndarray],
              W2: np.ndarray, b2: Optional[np.ndarray]) -> np.ndarray:
    """KVzap-MLP (Sec. 4.1; App. B Eq. 5): one hidden layer of width D_h/8
    shared by all heads, GELU, then H outputs.  No intermediate rounding.

    hidden [T, D_h], W1 [D_h, M], b1 [M]|None, W2 [M, H], b2 [H]|None.
    Returns scores [H, T].
    """
    hidden = np.asarray(hidden, dtype=np.float64)
    Z = hidden @ np.asarray(W1, dtype=np.float64)
    if b1 is not None:
        Z = Z + np.asarray(b1, dtype=np.float64)[None, :]
    G = gelu(Z)
    S = G @ np.asarray(W2, dtype=np.float64)
    if b2 is not None:
        S = S + np.asarray(b2, dtype=np.float64)[None, :]
    return np.ascontiguousarray(S.T)


# --------------------------------------------------------------------------
# surrogate on the un-normalised residual stream (Sec. 3: the surrogate reads the
# layer's *input hidden states*; Sec. 5: what an engine has to fuse)
# --------------------------------------------------------------------------
def rmsnorm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    """Root-mean-square layer normalisation of every row (the input norm of a
    decoder layer in the models of App. B):

        y[t, k] = x[t, k] / sqrt(mean_k x[t, k]^2 + eps) * gain[k]

    x float64 [T, D_h], gain float64 [D_h].  Reading: the paper does not say
    whether its "input hidden states" are taken before or after this norm; the
    fused entry point serves a caller that holds the residual stream and wants
    the surrogate applied to the normalised states, as the layer's own
    projections are.
    """
    x = np.asarray(x, dtype=np.float64)
    gain = np.asarray(gain, dtype=np.float64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + float(eps)) * gain


def rstd(x: np.ndarray, eps: float) -> np.ndarray:
    """1 / sqrt(mean_k x[t, k]^2 + eps) per row: what a consumer needs to apply
    the norm itself (float64 [T])."""
    x = np.asarray(x, dtype=np.float64)
    return 1.0 / np.sqrt(np.mean(x * x, axis=-1) + float(eps))


def score_mlp_rmsnorm(x: np.ndarray, gain: np.ndarray, eps: float, W1: np.ndarray,
                      b1: Optional[np.ndarray], W2: np.ndarray,
                      b2: Optional[np.ndarray]) -> np.ndarray:
    """KVzap-MLP applied to rmsnorm(x): scores [H, T].  No rounding of the
    normalised states in between (a bf16 model would round them; the GPU path
    does not materialise them for the surrogate at all)."""
    return score_mlp(rmsnorm(x, gain, eps), W1, b1, W2, b2)


# --------------------------------------------------------------------------
# threshold + sliding window (Sec. 3.3, Algorithm 1)
# --------------------------------------------------------------------------
def keep_mask(scores: np.ndarray, tau: float, window: int,
              seq_len: Optional[int] = None) -> np.ndarray:
    """keep[h, t] = (t >= T_b - window) or (scores[h, t] >= tau).

    Readings: equality keeps (Algorithm 1 uses >=); a NaN score compares false
    and is dropped unless protected; window = 0 protects nothing (the w = 0
    ablation of Sec. 4.8 means "no local window"); window >= T keeps all;
    with seq_len = T_b < T (right-padded batch) positions >= T_b do not exist
    and the window is counted from T_b.
    """
    scores = np.asarray(scores)
    H, T = scores.shape
    Tb = T if seq_len is None else int(seq_len)
    if not (0 <= Tb <= T):
        raise ValueError("seq_len out of range")
    if window < 0:
        raise ValueError("window must be >= 0")
    t = np.arange(T)
    tau = np.asarray(tau, dtype=np.float64)
    if tau.ndim == 1:                       # one threshold per head (fixed-budget variants)
        tau = tau[:, None]
    with np.errstate(invalid="ignore"):
        keep = scores >= tau
    keep = keep | (t >= Tb - window)[None, :]
    keep = keep & (t < Tb)[None, :]
    return keep


def kept_indices(keep: np.ndarray) -> Tuple[List[np.ndarray], np.ndarray]:
    """Ascending kept positions per head and their counts (Algorithm 1:
    torch.where enumerates true entries in row-major order)."""
    H = keep.shape[0]
    idx = [np.nonzero(keep[h])[0].astype(np.int32) for h in range(H)]
    lengths = np.array([len(i) for i in idx], dtype=np.int32)
    return idx, lengths


def exclusive_offsets(lengths: np.ndarray) -> np.ndarray:
    """offsets[i] = sum(lengths[:i]) over (sequence, head) row-major, with the
    grand total appended: where each head's rows start in the packed cache."""
    flat = np.asarray(lengths, dtype=np.int64).reshape(-1)
    out = np.zeros(flat.size + 1, dtype=np.int64)
    np.cumsum(flat, out=out[1:])
    return out


def gather_rows(X_bits: np.ndarray, idx: Sequence[np.ndarray]) -> np.ndarray:
    """Packed kept rows, heads in order, positions ascending (Algorithm 1:
    keys[indices]).  X_bits is [H, T, D] uint16; the copy is bit-exact."""
    X_bits = np.asarray(X_bits)
    parts = [X_bits[h][idx[h]] for h in range(X_bits.shape[0])]
    if not parts:
        return np.zeros((0, X_bits.shape[-1]), dtype=X_bits.dtype)
    return np.concatenate(parts, axis=0)


@dataclass
class PruneResult:
    idx: List[List[np.ndarray]]          # [B][H] ascending int32 positions
    lengths: np.ndarray                  # [B, H] int32
    offsets: np.ndarray                  # [B*H + 1] int64
    K_out: Optional[np.ndarray] = None   # [n_total, D] uint16
    V_out: Optional[np.ndarray] = None

    def flat_idx(self) -> np.ndarray:
        parts = [i for per_b in self.idx for i in per_b]
        return np.concatenate(parts) if parts else np.zeros(0, np.int32)


def prune(scores: np.ndarray, tau: float, window: int,
          K_bits: Optional[np.ndarray] = None,
          V_bits: Optional[np.ndarray] = None,
          seq_lens: Optional[Sequence[int]] = None) -> PruneResult:
    """Algorithm 1 after the scorer, for a batch: scores [B, H, T],
    K_bits / V_bits [B, H, T, D] uint16 (optional)."""
    scores = np.asarray(scores)
    B, H, T = scores.shape
    all_idx, all_len = [], []
    for b in range(B):
        Tb = None if seq_lens is None else int(seq_lens[b])
        tau_b = tau if np.ndim(tau) == 0 else np.asarray(tau)[b]    # scalar, or [B, H]
        idx, n = kept_indices(keep_mask(scores[b], tau_b, window, Tb))
        all_idx.append(idx)
        all_len.append(n)
    lengths = (np.stack(all_len) if B else np.zeros((0, H), np.int32)).astype(np.int32)
    res = PruneResult(all_idx, lengths, exclusive_offsets(lengths))
    if K_bits is not None:
        D = K_bits.shape[-1]
        ks = [gather_rows(K_bits[b], all_idx[b]) for b in range(B)]
        vs = [gather_rows(V_bits[b], all_idx[b]) for b in range(B)]
        res.K_out = np.concatenate(ks, axis=0) if ks else np.zeros((0, D), np.uint16)
        res.V_out = np.concatenate(vs, axis=0) if vs else np.zeros((0, D), np.uint16)
    return res


def compress(hidden_bits: np.ndarray, K_bits: np.ndarray, V_bits: np.ndarray,
             weights: dict, tau: float, window: int = 128,
             seq_lens: Optional[Sequence[int]] = None
             ) -> Tuple[np.ndarray, PruneResult]:
    """The whole of Algorithm 1 for one layer.

    hidden_bits [B, T, D_h] uint16 bf16 patterns; weights holds float64 arrays
    in the paper's orientation: {"W": [D_h,H], "b"} for the linear surrogate or
    {"W1": [D_h,M], "b1", "W2": [M,H], "b2"} for the MLP (biases may be None).
    Returns (scores [B,H,T] float64, PruneResult).
    """
    B = hidden_bits.shape[0]
    per_b = []
    for b in range(B):
        h64 = bf16_bits_to_f64(hidden_bits[b])
        if "W1" in weights:
            per_b.append(score_mlp(h64, weights["W1"], weights.get("b1"),
                                   weights["W2"], weights.get("b2")))
        else:
            per_b.append(score_linear(h64, weights["W"], weights.get("b")))
    scores = np.stack(per_b)
    return scores, prune(scores, tau, window, K_bits, V_bits, seq_lens)


def tau_at_keep_fraction(scores: np.ndarray, window: int, keep_fraction: float,
                         seq_lens: Optional[Sequence[int]] = None) -> float:
    """Threshold at which `keep_fraction` of the non-window tokens (pooled over
    sequences and heads) score >= tau: the midpoint between the two adjacent
    order statistics, rounded to fp32 so that a float32 consumer compares
    against the identical value.  (Workload recipe, not part of the method.)"""
    scores = np.asarray(scores, dtype=np.float64)
    B, H, T = scores.shape
    pool = []
    for b in range(B):
        Tb = T if seq_lens is None else int(seq_lens[b])
        pool.append(scores[b, :, :max(Tb - window, 0)].reshape(-1))
    pool = np.sort(np.concatenate(pool))
    n = pool.size
    if n < 2:
        raise ValueError("not enough non-window tokens for a quantile")
    k = int(round(keep_fraction * n))          # tokens kept = the k largest
    k = min(max(k, 1), n - 1)
    lo, hi = pool[n - k - 1], pool[n - k]
    return float(np.float32(0.5 * (lo + hi)))


# --------------------------------------------------------------------------
# decode (caption of Algorithm 1; Sec. 2 "delayed eviction with a sliding
# window"; Sec. 3.3: the surrogate depends only on hidden states, so it can be
# applied while decoding)
# --------------------------------------------------------------------------
@dataclass
class DecodeHeadState:
    positions: List[int] = field(default_factory=list)   # ascending
    K_rows: List[np.ndarray] = field(default_factory=list)
    V_rows: List[np.ndarray] = field(default_factory=list)


class DecodeOracle:
    """Canonical decode state: per (sequence, head) the ascending list of kept
    positions with their rows; per sequence the next position p; per
    (sequence, head) the scores of the positions still inside the window.

    One step for sequence b at position p (reading of the caption):
      1. s = surrogate(h_new)                       (H scores)
      2. the new pair is appended at position p and its score remembered;
      3. q = p - w is the position that has left the window now that p is in
         it; if q >= 0 and not (score[q] >= tau) the pair at q is removed from
         the head (for w = 0 this is the token just appended: q = p).
    Appending first and evicting second is the order step() takes; evicting
    first gives the same state for w > 0 (q != p), and is undefined for w = 0.
    After the step the kept set equals Algorithm 1 applied to the p+1 scores.
    """

    def __init__(self, B: int, H: int, window: int, tau: float):
        self.B, self.H, self.w, self.tau = B, H, int(window), float(tau)
        self.heads = [[DecodeHeadState() for _ in range(H)] for _ in range(B)]
        self.next_pos = [0] * B
        self.win_scores = [[dict() for _ in range(H)] for _ in range(B)]

    def load_prefill(self, b: int, scores_b: np.ndarray,
                     K_bits_b: np.ndarray, V_bits_b: np.ndarray) -> None:
        """Initialise sequence b from a prefill of T tokens pruned by
        Algorithm 1 with the same tau and window."""
        H, T = scores_b.shape
        keep = keep_mask(scores_b, self.tau, self.w)
        for h in range(H):
            st = self.heads[b][h]
            pos = np.nonzero(keep[h])[0]
            st.positions = [int(t) for t in pos]
            st.K_rows = [K_bits_b[h, t].copy() for t in pos]
            st.V_rows = [V_bits_b[h, t].copy() for t in pos]
            self.win_scores[b][h] = {int(t): float(scores_b[h, t])
                                     for t in range(max(T - self.w, 0), T)}
        self.next_pos[b] = T

    def step(self, scores_new: np.ndarray, k_new: np.ndarray,
             v_new: np.ndarray) -> None:
        """scores_new [B, H] float64, k_new / v_new [B, H, D] uint16."""
        for b in range(self.B):
            p = self.next_pos[b]
            q = p - self.w
            for h in range(self.H):
                st = self.heads[b][h]
                ws = self.win_scores[b][h]
                # the new token enters first, so that for w = 0 it is itself
                # the token that "leaves" (q == p)
                st.positions.append(p)
                st.K_rows.append(np.array(k_new[b, h], copy=True))
                st.V_rows.append(np.array(v_new[b, h], copy=True))
                ws[p] = float(scores_new[b, h])
                if q >= 0:
                    s_q = ws.pop(q)
                    if not (s_q >= self.tau):
                        j = st.positions.index(q)
                        del st.positions[j], st.K_rows[j], st.V_rows[j]
            self.next_pos[b] = p + 1

    def canonical(self, b: int, h: int):
        st = self.heads[b][h]
        D = st.K_rows[0].shape[0] if st.K_rows else 0
        K = np.stack(st.K_rows) if st.K_rows else np.zeros((0, D), np.uint16)
        V = np.stack(st.V_rows) if st.V_rows else np.zeros((0, D), np.uint16)
        return np.array(st.positions, dtype=np.int64), K, V


# --------------------------------------------------------------------------
# analytic overhead model (App. B Eq. 4-6 and the overhead table)
# --------------------------------------------------------------------------
def flops_layer_linear_projections(H_Q: int, H: int, D: int, D_h: int,
                                   D_int: int) -> int:
    """Eq. 4: attention projections plus SwiGLU FFN, per token."""
    return 4 * D_h * (H_Q * D + H * D) + 6 * D_h * D_int


def flops_kvzap_mlp(D_h: int, H: int) -> int:
    """Eq. 5: 2*D_h*(D_h/8) + 2*(D_h/8)*H per token."""
    M = D_h // 8
    return 2 * D_h * M + 2 * M * H


def flops_kvzap_linear(D_h: int, H: int) -> int:
    """Eq. 6: 2*D_h*H per token."""
    return 2 * D_h * H


def param_count(kind: str, L: int, D_h: int, H: int, biases: bool = False) -> int:
    """Parameters of a list of L per-layer surrogates (Sec. 4.1 shapes)."""
    M = D_h // 8
    if kind == "mlp":
        per = D_h * M + M * H + ((M + H) if biases else 0)
    elif kind == "linear":
        per = D_h * H + (H if biases else 0)
    else:
        raise ValueError(kind)
    return L * per


# --------------------------------------------------------------------------
# consumer of the ragged cache: one decoding step of attention over per-head
# caches of different lengths (Sec. 5 names such a kernel as the engineering
# that turns the compression into savings; the weights are the a_ji of Eq. 2)
# --------------------------------------------------------------------------
def attend_decode(q: np.ndarray, caches, scale: float) -> np.ndarray:
    """Softmax attention of one new query per (sequence, query head) over the
    kept KV pairs of its KV head (grouped-query attention: query head g uses KV
    head g // (H_Q // H), as in the models of App. B).

    q       float64 [B, H_Q, D]
    caches  caches[b][h] = (K [n_bh, D], V [n_bh, D]) float64, n_bh >= 1, in any
            row order (the result does not depend on it)
    Returns float64 [B, H_Q, D]:  out = sum_i softmax_i(scale * q . K_i) V_i.
    """
    q = np.asarray(q, dtype=np.float64)
    B, HQ, D = q.shape
    H = len(caches[0])
    G = HQ // H
    assert G * H == HQ
    out = np.zeros((B, HQ, D))
    for b in range(B):
        for g in range(HQ):
            K, V = caches[b][g // G]
            s = (np.asarray(K, dtype=np.float64) @ q[b, g]) * scale
            s = s - s.max()
            p = np.exp(s)
            p = p / p.sum()
            out[b, g] = p @ np.asarray(V, dtype=np.float64)
    return out


# --------------------------------------------------------------------------
# paged layout of the ragged cache (Sec. 1, criterion 3: compatibility with
# paged attention; Sec. 5: heads of different lengths need pages per head)
# --------------------------------------------------------------------------
def pages_needed(n_rows: int, page_rows: int, reserve_rows: int = 0) -> int:
    """Pages of `page_rows` rows that hold n_rows + reserve_rows rows (0 for 0)."""
    total = int(n_rows) + int(reserve_rows)
    return 0 if total <= 0 else (total + page_rows - 1) // page_rows


def assign_pages(lengths: np.ndarray, page_rows: int, free_pages: Sequence[int],
                 max_pages: int, reserve_rows: int = 0):
    """Give every head, in (sequence, head) order, the next pages of the free
    list.  Reading (the paper fixes no allocator): first-fit in list order, so
    the result is unique.  Returns (block_table [B*H, max_pages] int32 with -1
    in unused entries, pages_used, ok); when the free list is too short or a
    head needs more than max_pages, nothing is assigned and ok is False."""
    n = np.asarray(lengths, dtype=np.int64).reshape(-1)
    need = [pages_needed(int(x), page_rows, reserve_rows) for x in n]
    table = np.full((n.size, max_pages), -1, dtype=np.int32)
    if sum(need) > len(free_pages) or (need and max(need) > max_pages):
        return table, 0, False
    pos = 0
    for bh, c in enumerate(need):
        for i in range(c):
            table[bh, i] = int(free_pages[pos])
            pos += 1
    return table, pos, True


def scatter_to_pages(rows_per_head: Sequence[np.ndarray], table: np.ndarray,
                     page_rows: int, num_pages: int, D: int) -> np.ndarray:
    """Write row j of head bh to row j % page_rows of page table[bh, j // page_rows].
    rows_per_head[bh] is uint16 [n_bh, D].  Returns the pool uint16
    [num_pages, page_rows, D], zero where nothing was written."""
    pool = np.zeros((num_pages, page_rows, D), dtype=np.uint16)
    for bh, rows in enumerate(rows_per_head):
        for j in range(rows.shape[0]):
            pool[table[bh, j // page_rows], j % page_rows] = rows[j]
    return pool


def gather_from_pages(pool: np.ndarray, table_row: np.ndarray, n_rows: int,
                      page_rows: int) -> np.ndarray:
    """The first n_rows rows of one head, read back through its block table."""
    out = np.zeros((n_rows, pool.shape[2]), dtype=pool.dtype)
    for j in range(n_rows):
        out[j] = pool[table_row[j // page_rows], j % page_rows]
    return out


def extend_pages(lengths: np.ndarray, page_counts: np.ndarray, table: np.ndarray,
                 page_rows: int, free_pages: Sequence[int], reserve_rows: int = 0):
    """Bring every head up to pages_needed(length, reserve) pages by appending the next
    entries of the free list behind the page_counts[bh] entries it already owns, heads in
    (sequence, head) order.  Returns (new table, new page_counts, pages_used, ok); when the
    list is too short or a head would exceed the table width, nothing changes and ok is
    False.  assign_pages is the case page_counts == 0 on an all -1 table."""
    n = np.asarray(lengths, dtype=np.int64).reshape(-1)
    have = np.asarray(page_counts, dtype=np.int64).reshape(-1)
    table = np.array(table, dtype=np.int32, copy=True)
    max_pages = table.shape[1]
    add = [max(0, pages_needed(int(n[i]), page_rows, reserve_rows) - int(have[i]))
           for i in range(n.size)]
    if sum(add) > len(free_pages) or any(int(have[i]) + add[i] > max_pages for i in range(n.size)):
        return table, np.array(have, dtype=np.int32), 0, False
    pos = 0
    new_counts = np.array(have, dtype=np.int32)
    for bh, c in enumerate(add):
        for i in range(c):
            table[bh, int(have[bh]) + i] = int(free_pages[pos])
            pos += 1
        new_counts[bh] += c
    return table, new_counts, pos, True


# --------------------------------------------------------------------------
# fixed-budget selection on the same scores (Sec. 3.3: KVzip keeps a fixed
# fraction; ablation of Sec. 4: fixed-ratio top-k per head, or per layer as in
# AdaKV, against thresholding)
# --------------------------------------------------------------------------
def topk_threshold(scores: np.ndarray, window: int, k: int, per_layer: bool,
                   seq_lens: Optional[Sequence[int]] = None) -> np.ndarray:
    """Thresholds that turn Algorithm 1's comparison into a fixed-budget rule.

    Population of sequence b, head h: its non-window positions t < T_b - window
    whose score is not NaN.  per_layer = False: tau[b,h] is the k-th largest
    score of that population (each head keeps its own top k).  per_layer = True:
    the populations of all H heads of sequence b are pooled and tau[b,:] is the
    k-th largest of the pool (the heads share one budget of k).  k <= 0 gives
    +inf (only the window is kept), k >= population size gives -inf.

    Reading: the kept set is {score >= tau}, so entries tied with the k-th
    largest are all kept (the unique set; equal to a top-k whenever scores are
    distinct), and the window stays protected as in Algorithm 1.
    Returns float64 [B, H].
    """
    scores = np.asarray(scores, dtype=np.float64)
    B, H, T = scores.shape
    tau = np.empty((B, H))
    for b in range(B):
        Tb = T if seq_lens is None else int(seq_lens[b])
        n_pop = max(Tb - window, 0)
        pops = []
        for h in range(H):
            pop = scores[b, h, :n_pop]
            pops.append(pop[~np.isnan(pop)])
        groups = [np.concatenate(pops)] * H if per_layer else pops
        for h in range(H):
            pop = groups[h]
            if k <= 0:
                tau[b, h] = np.inf
            elif k >= pop.size:
                tau[b, h] = -np.inf
            else:
                tau[b, h] = np.sort(pop)[::-1][k - 1]
    return tau


# --------------------------------------------------------------------------
# the scores the surrogate is trained on (Sec. 3.1 Eq. 1: KVzip; Sec. 3.2
# Eq. 3: KVzip+), on an extended prompt "prompt, instruction, repeated prompt"
# --------------------------------------------------------------------------
def teacher_log_scores(q: np.ndarray, k: np.ndarray, scale: float, T: int,
                       vnorm: Optional[np.ndarray] = None,
                       hnorm: Optional[np.ndarray] = None) -> np.ndarray:
    """log s_i^+ for the T positions of the original prompt, per KV head.

    q      float64 [H_Q, Tq, D]: queries of the Tq positions of the repeated
           prompt, which sit at positions P0 .. P0+Tq-1 with P0 = Tk - Tq
    k      float64 [H, Tk, D]: keys of all positions of the extended prompt
    a_ji   causal softmax over the keys i' <= P0 + j of scale * q_j . k_i'
    vnorm  [H, T] = ||W_O v_i|| (None = 1: Eq. 1), hnorm [Tq] = ||h_j|| (None = 1)
    s_i = max over j and over the query heads g of the KV head's group of
          a_ji * vnorm[h, i] / hnorm[j]                               (Eq. 3)
    Returned in log space (what the surrogate regresses, Sec. 3.3), float64
    [H, T]; requires T <= P0 so that every scored key is visible to every query.
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    HQ, Tq, D = q.shape
    H, Tk, _ = k.shape
    G = HQ // H
    P0 = Tk - Tq
    if G * H != HQ or P0 < 0 or not (0 <= T <= P0):
        raise ValueError("shapes do not describe an extended prompt")
    out = np.full((H, T), -np.inf)
    lv = np.zeros((H, T)) if vnorm is None else np.log(np.asarray(vnorm, dtype=np.float64))
    lh = np.zeros(Tq) if hnorm is None else np.log(np.asarray(hnorm, dtype=np.float64))
    visible = np.arange(Tk)[None, :] <= (P0 + np.arange(Tq))[:, None]
    for g in range(HQ):
        h = g // G
        s = (q[g] @ k[h].T) * scale                       # [Tq, Tk]
        s = np.where(visible, s, -np.inf)
        m = s.max(axis=1, keepdims=True)
        lse = m + np.log(np.exp(s - m).sum(axis=1, keepdims=True))
        log_a = s - lse                                   # log a_ji
        cand = (log_a[:, :T] - lh[:, None]).max(axis=0)   # max over j
        out[h] = np.maximum(out[h], cand)                 # max over the group
    return out + lv
