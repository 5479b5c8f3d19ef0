// One decoding step of one layer (caption of Algorithm 1; Sec. 2 "delayed
// eviction with a sliding window"): score the new token of each sequence with
// the surrogate, test the token that leaves the window against tau, append it
// to the head's kept prefix or drop it, and put the new pair in its ring slot.
//
// Two launches:
//   1. decode_partial : the first MLP projection for B new tokens is a skinny
//      GEMM bound by reading W1 once; (unit-block x K-slice) blocks run
//      v_mfma_f32_32x32x16_bf16 on operands loaded straight from global memory
//      and write fp32 partial sums (fixed order -> deterministic).
//   2. decode_finish  : one block per sequence sums the K-slices, applies bias,
//      GELU and the M -> H projection in fp32, then performs the O(1)-row cache
//      update of its H heads.  For the linear surrogate step 1 is skipped and the
//      block computes the H dot products itself.
// State layout: an append-only ascending prefix per (b,h) plus a `window`-row
// ring indexed by position mod window: a token that leaves the window is copied
// ring -> prefix tail if kept and is simply overwritten by the new token if not,
// because the new token's slot (p mod w) is the leaving token's slot.
#include "kvzap_internal.h"

namespace kvzap {
namespace {

constexpr int kPThreads = 256;
constexpr int kMaxKSplit = 16;

// how many K-slices the first projection is cut into
inline int decode_ksplit(int B, int Dh, int M) {
  const int nub = M / 32, ntb = (B + 63) / 64;
  int target = 256 / (nub * ntb);
  if (target < 1) target = 1;
  if (target > kMaxKSplit) target = kMaxKSplit;
  const int units = Dh / 64;               // a slice is a multiple of 64 inputs
  int ks = 1;
  for (int d = 1; d <= units && d <= target; ++d)
    if (units % d == 0) ks = d;
  return ks;
}

__global__ __launch_bounds__(kPThreads) void decode_partial_kernel(
    const unsigned short* __restrict__ hidden, const unsigned short* __restrict__ W1,
    float* __restrict__ partial, int B, int Dh, int M, int kslice) {
  __shared__ float red[4][2][16][64];
  const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
  const int l32 = lane & 31, kg = lane >> 5;
  const int ub = blockIdx.x, ks = blockIdx.y, tok0 = blockIdx.z * 64;
  const int kw = kslice / 4;                           // inputs per wavefront (multiple of 16)
  const int k_begin = ks * kslice + wid * kw + kg * 8;
  const unsigned short* a_ptr = W1 + (size_t)(ub * 32 + l32) * Dh + k_begin;
  const unsigned short* b_ptr[2];
#pragma unroll
  for (int tb = 0; tb < 2; ++tb) {
    int tok = tok0 + tb * 32 + l32;
    if (tok > B - 1) tok = B - 1;                      // clamp, discarded later
    b_ptr[tb] = hidden + (size_t)tok * Dh + k_begin;
  }
  floatx16 acc[2];
#pragma unroll
  for (int tb = 0; tb < 2; ++tb)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[tb][e] = 0.0f;
  // latency-bound: keep the operand loads of four k-steps (12 x 16 B per lane) in flight
  int k = 0;
  for (; k + 64 <= kw; k += 64) {
    bf16x8 a[4], b0[4], b1[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      a[s] = *reinterpret_cast<const bf16x8*>(a_ptr + k + 16 * s);
      b0[s] = *reinterpret_cast<const bf16x8*>(b_ptr[0] + k + 16 * s);
      b1[s] = *reinterpret_cast<const bf16x8*>(b_ptr[1] + k + 16 * s);
    }
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[s], b0[s], acc[0], 0, 0, 0);
      acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[s], b1[s], acc[1], 0, 0, 0);
    }
  }
  for (; k < kw; k += 16) {
    const bf16x8 a = *reinterpret_cast<const bf16x8*>(a_ptr + k);
    const bf16x8 b0 = *reinterpret_cast<const bf16x8*>(b_ptr[0] + k);
    const bf16x8 b1 = *reinterpret_cast<const bf16x8*>(b_ptr[1] + k);
    acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b0, acc[0], 0, 0, 0);
    acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b1, acc[1], 0, 0, 0);
  }
#pragma unroll
  for (int tb = 0; tb < 2; ++tb)
#pragma unroll
    for (int r = 0; r < 16; ++r) red[wid][tb][r][lane] = acc[tb][r];
  __syncthreads();
  for (int e = tid; e < 2 * 16 * 64; e += kPThreads) {
    const int ln = e & 63, r = (e >> 6) & 15, tb = e >> 10;
    const float s = ((red[0][tb][r][ln] + red[1][tb][r][ln]) + red[2][tb][r][ln]) + red[3][tb][r][ln];
    const int unit = ub * 32 + 8 * (r / 4) + 4 * (ln >> 5) + (r % 4);
    const int tok = tok0 + tb * 32 + (ln & 31);
    if (tok < B) partial[((size_t)ks * B + tok) * M + unit] = s;
  }
}

constexpr int kFThreads = 256;

__global__ __launch_bounds__(kFThreads) void decode_finish_kernel(DecodeArgs a, int ksplit) {
  extern __shared__ __align__(16) unsigned char smem[];
  float* g = reinterpret_cast<float*>(smem);          // [M] (MLP) -- or unused
  __shared__ float s_new[16];
  __shared__ int s_keep[16];
  const int b = blockIdx.x, tid = threadIdx.x;
  const int H = a.H, D = a.D, w = a.window, M = a.M, Dh = a.Dh;
  const unsigned short* b1 = static_cast<const unsigned short*>(a.b1);
  const unsigned short* b2 = static_cast<const unsigned short*>(a.b2);

  // ---- 0. everything the cache update needs that does not depend on the new score is
  // fetched first, so that its (HBM) latency overlaps the scorer arithmetic below: the
  // position, and per (head, 16-byte piece) the new rows, the ring rows of the slot that is
  // about to be vacated (read speculatively: they are only used if the token is kept), the
  // head's length, slab offset and capacity, and the leaving token's score.
  const int p = a.seq_pos[b];
  const int q = p - w;
  const int slot = (w > 0) ? (p % w) : 0;
  const int lpr = D / 8;
  const int npieces = H * lpr;                         // <= 16 * 64 = 1024 -> at most 4 per thread
  constexpr int kMaxPer = 4;
  u32x4 k_in[kMaxPer], v_in[kMaxPer], k_old[kMaxPer], v_old[kMaxPer];
  int len_r[kMaxPer], cap_r[kMaxPer];
  long long slab_r[kMaxPer];
  const u32x4* kn = static_cast<const u32x4*>(a.k_new) + (size_t)b * H * lpr;
  const u32x4* vn = static_cast<const u32x4*>(a.v_new) + (size_t)b * H * lpr;
  u32x4* Kp = static_cast<u32x4*>(a.K_prefix);
  u32x4* Vp = static_cast<u32x4*>(a.V_prefix);
  u32x4* Kr = static_cast<u32x4*>(a.K_ring);
  u32x4* Vr = static_cast<u32x4*>(a.V_ring);
#pragma unroll
  for (int c = 0; c < kMaxPer; ++c) {
    const int i = tid + c * kFThreads;
    if (i < npieces) {
      const int h = i / lpr, piece = i % lpr, bh = b * H + h;
      k_in[c] = kn[i];
      v_in[c] = vn[i];
      len_r[c] = a.lengths[bh];
      if (a.block_table) {
        // paged prefix: the next row is row len % page_rows of the page in table slot
        // len / page_rows.  Expressed as a slab whose row `len` is that row, with room for
        // exactly one more row if the slot holds a page of the pool.
        const int len = len_r[c] < 0 ? 0 : len_r[c];
        const int pslot = len >> a.log_page;
        const int page = pslot < a.max_pages ? a.block_table[(size_t)bh * a.max_pages + pslot] : -1;
        const bool ok = page >= 0 && page < a.num_pages;
        cap_r[c] = ok ? len_r[c] + 1 : len_r[c];
        slab_r[c] = (((long long)(ok ? page : 0)) << a.log_page) + (len & ((1 << a.log_page) - 1)) - len_r[c];
      } else {
        cap_r[c] = a.slab_capacity[bh];
        slab_r[c] = a.slab_offsets[bh];
      }
      if (w > 0 && q >= 0) {
        const size_t ring_at = ((size_t)bh * w + slot) * lpr + piece;
        k_old[c] = Kr[ring_at];
        v_old[c] = Vr[ring_at];
      }
    }
  }
  float s_q_r = 0.0f;
  if (tid < H && w > 0 && q >= 0) s_q_r = a.score_ring[(size_t)(b * H + tid) * w + slot];
  // second-projection weights of this thread's hidden units (M <= 640 -> at most 3 per head)
  constexpr int kMaxUnits = 3;
  unsigned short w2r[16][kMaxUnits];
  if (M > 0) {
    const unsigned short* W2 = static_cast<const unsigned short*>(a.W2);
#pragma unroll
    for (int h = 0; h < 16; ++h)
#pragma unroll
      for (int u = 0; u < kMaxUnits; ++u) {
        const int m = tid + u * kFThreads;
        w2r[h][u] = (h < H && m < M) ? W2[(size_t)h * M + m] : (unsigned short)0;
      }
  }

  // ---- 1. scores of the new token ----
  if (M > 0) {
    const float* partial = static_cast<const float*>(a.workspace);
    for (int m = tid; m < M; m += kFThreads) {
      // the partial sums were written by other XCDs, so each read is a trip to memory: issue
      // all K-slices' loads together (ksplit <= kMaxKSplit), then add them in a fixed order
      float part[kMaxKSplit];
#pragma unroll
      for (int ks = 0; ks < kMaxKSplit; ++ks)
        part[ks] = (ks < ksplit) ? partial[((size_t)ks * a.B + b) * M + m] : 0.0f;
      float z = 0.f;
#pragma unroll
      for (int ks = 0; ks < kMaxKSplit; ++ks) z += part[ks];
      if (b1) z += bf16_bits_to_float(b1[m]);
      g[m] = 0.5f * z * (1.0f + erff(z * 0.70710678118654752f));
    }
    __syncthreads();
  }
  // all H dot products at once: every load below is independent of the others, and a single
  // block reduction follows (a loop over heads with a barrier each would serialise H memory
  // round trips)
  float dot[16];
#pragma unroll
  for (int h = 0; h < 16; ++h) dot[h] = 0.f;
  if (M > 0) {
#pragma unroll
    for (int u = 0; u < kMaxUnits; ++u) {
      const int m = tid + u * kFThreads;
      const float gm = (m < M) ? g[m] : 0.f;
#pragma unroll
      for (int h = 0; h < 16; ++h) dot[h] += gm * bf16_bits_to_float(w2r[h][u]);
    }
  } else {
    const unsigned short* hid = static_cast<const unsigned short*>(a.hidden_new) + (size_t)b * Dh;
    const unsigned short* W = static_cast<const unsigned short*>(a.W1);
    for (int k = tid; k < Dh; k += kFThreads) {
      const float x = bf16_bits_to_float(hid[k]);
#pragma unroll
      for (int h = 0; h < 16; ++h)
        if (h < H) dot[h] += x * bf16_bits_to_float(W[(size_t)h * Dh + k]);
    }
  }
  __shared__ float red[16][kFThreads / 64];
#pragma unroll
  for (int h = 0; h < 16; ++h) {
    if (h < H) {
      float v = dot[h];
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
      if ((tid & 63) == 0) red[h][tid >> 6] = v;
    }
  }
  __syncthreads();
  if (tid < H) {
    float s = 0.f;
#pragma unroll
    for (int wv = 0; wv < kFThreads / 64; ++wv) s += red[tid][wv];
    const unsigned short* bias = (M > 0) ? b2 : b1;
    s_new[tid] = s + (bias ? bf16_bits_to_float(bias[tid]) : 0.f);
  }
  __syncthreads();

  // ---- 2. is the token that leaves the window kept ----
  if (tid < H) {
    const float s_q = (w > 0) ? s_q_r : s_new[tid];      // w == 0: the new token itself
    s_keep[tid] = (q >= 0) && (s_q >= a.tau);
  }
  __syncthreads();

  // ---- 3. move rows: ring -> prefix tail (kept), new -> ring slot ----
#pragma unroll
  for (int c = 0; c < kMaxPer; ++c) {
    const int i = tid + c * kFThreads;
    if (i < npieces) {
      const int h = i / lpr, piece = i % lpr, bh = b * H + h;
      if (s_keep[h] && len_r[c] < cap_r[c]) {
        const size_t dst = ((size_t)slab_r[c] + len_r[c]) * lpr + piece;
        Kp[dst] = (w > 0) ? k_old[c] : k_in[c];
        Vp[dst] = (w > 0) ? v_old[c] : v_in[c];
      }
      if (w > 0) {
        const size_t ring_at = ((size_t)bh * w + slot) * lpr + piece;
        Kr[ring_at] = k_in[c];
        Vr[ring_at] = v_in[c];
      }
      // ---- 4. bookkeeping, by the thread that owns piece 0 of the head ----
      if (piece == 0) {
        if (s_keep[h]) {
          if (len_r[c] < cap_r[c]) {
            a.prefix_pos[(size_t)slab_r[c] + len_r[c]] = q;
            a.lengths[bh] = len_r[c] + 1;
          } else if (a.error_flag) {
            *a.error_flag = 1;
          }
        }
        if (w > 0) a.score_ring[(size_t)bh * w + slot] = s_new[h];
      }
    }
  }
  if (tid == 0) a.seq_pos[b] = p + 1;
}

}  // namespace

size_t decode_workspace_bytes(int B, int Dh, int M, int H) {
  (void)H;
  if (M == 0) return 0;
  return align_up((size_t)decode_ksplit(B, Dh, M) * B * M * sizeof(float), 256);
}

int launch_decode_evict(const DecodeArgs& a, hipStream_t stream) {
  int ks = 0;
  if (a.M > 0) {
    ks = decode_ksplit(a.B, a.Dh, a.M);
    const dim3 grid(a.M / 32, ks, (a.B + 63) / 64);
    decode_partial_kernel<<<grid, kPThreads, 0, stream>>>(
        static_cast<const unsigned short*>(a.hidden_new),
        static_cast<const unsigned short*>(a.W1), static_cast<float*>(a.workspace), a.B,
        a.Dh, a.M, a.Dh / ks);
  }
  const size_t lds = (size_t)(a.M > 0 ? a.M : 1) * sizeof(float);
  decode_finish_kernel<<<a.B, kFThreads, lds, stream>>>(a, ks);
  return hipGetLastError() == hipSuccess ? KVZAP_OK : KVZAP_ERR_RUNTIME;
}

}  // namespace kvzap
