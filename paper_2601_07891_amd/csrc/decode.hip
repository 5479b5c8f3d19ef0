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
//      GELU and the M -> H projection in fp32, and performs the O(1)-row cache
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

constexpr int kFThreads = 1024;
constexpr int kFWaves = kFThreads / 64;       // 16 >= H: wavefront h reduces head h, its lane 0 owns it
constexpr int kKGroups = 4;                   // thread t sums K-slices 4*(t/256) .. +4 of unit pair t%256
constexpr int kPairs = kFThreads / kKGroups;  // unit pairs per round
constexpr int kUnitRounds = 2;                // M <= 1024
static_assert(kKGroups * 4 == kMaxKSplit, "four K-slices per group");

// low / high bf16 of a 32-bit word as fp32
__device__ __forceinline__ float bf16_lo(unsigned int u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(unsigned int u) { return __uint_as_float(u & 0xffff0000u); }

// sum over the 8 bf16 pairs of two 16-byte operands
__device__ __forceinline__ float dot8_bf16(const u32x4& x, const u32x4& y) {
  float s = 0.f;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    s += bf16_lo(x[e]) * bf16_lo(y[e]);
    s += bf16_hi(x[e]) * bf16_hi(y[e]);
  }
  return s;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

__device__ __forceinline__ float gelu_erf(float z) {
  return 0.5f * z * (1.0f + erff(z * 0.70710678118654752f));
}

// The step is a chain of dependent memory round trips, so the kernel is written around
// their number and around how fast a wavefront issues instructions, not around arithmetic:
//  * every load whose address does not depend on loaded data is issued at entry without a
//    branch around it (out-of-range lanes read a clamped address and discard the value; a
//    branch with a load inside makes the wavefront wait for that load on the spot), the
//    loads that need the position follow as soon as it arrives;
//  * a lone wavefront per SIMD issues an instruction only every ~10 cycles, so the block
//    has 16 wavefronts and every thread few loads: a quarter of the K-slices of one pair of
//    hidden units, one 16-byte piece of the new rows, one head's second-projection weights;
//  * with a window, whether the leaving token is kept depends only on the score already in
//    the ring, so the row moves follow the first barrier and do not wait for the new score.
// kMlp: MLP surrogate (a.M > 0) or linear.
template <bool kMlp>
__global__ __launch_bounds__(kFThreads) void decode_finish_kernel(DecodeArgs a, int ksplit) {
  extern __shared__ __align__(16) unsigned char smem[];
  float* g = reinterpret_cast<float*>(smem);          // [M] hidden activations (MLP)
  float* zpart = g + a.M;                             // [kKGroups][M] sums of four K-slices each
  __shared__ int s_keep[16];
  __shared__ float s_red[16][kFWaves];                 // linear scorer: per-wavefront sums
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int H = a.H, D = a.D, w = a.window, M = a.M, Dh = a.Dh;
  const int p = a.seq_pos[b];
  // lane 0 of wavefront h owns head h: it reads the leaving token's score, decides keep /
  // drop and later writes the new score to the same ring slot
  const bool owner = lane == 0 && wv < H;
  const int hw = wv < H ? wv : H - 1;                  // this wavefront's head (clamped)

  // ---- 0a. loads that need nothing but the block index ----
  const int lpr = D / 8;
  const int npieces = H * lpr;                         // <= 16 * 64 = kFThreads
  const int pi = tid < npieces ? tid : npieces - 1;    // this thread's 16-byte piece of the new rows
  const int head_r = pi / lpr, piece_r = pi - head_r * lpr, bh_r = b * H + head_r;
  u32x4* Kp = static_cast<u32x4*>(a.K_prefix);
  u32x4* Vp = static_cast<u32x4*>(a.V_prefix);
  u32x4* Kr = static_cast<u32x4*>(a.K_ring);
  u32x4* Vr = static_cast<u32x4*>(a.V_ring);
  const u32x4 k_in = static_cast<const u32x4*>(a.k_new)[(size_t)b * npieces + pi];
  const u32x4 v_in = static_cast<const u32x4*>(a.v_new)[(size_t)b * npieces + pi];
  const int len_r = a.lengths[bh_r];
  int cap_r = 0;
  long long slab_r = 0;
  if (!a.block_table) {
    cap_r = a.slab_capacity[bh_r];
    slab_r = a.slab_offsets[bh_r];
  }
  // an absent bias is read from a stand-in address and discarded
  const unsigned short* bias2p = static_cast<const unsigned short*>(kMlp ? a.b2 : a.b1);
  const unsigned short* bias2_at = bias2p ? bias2p + hw : static_cast<const unsigned short*>(a.k_new);
  const unsigned short bias2_raw = *bias2_at;
  const unsigned short bias2 = bias2p ? bias2_raw : (unsigned short)0;

  const int kq = tid / kPairs, pr = tid - kq * kPairs;
  float2 part[kUnitRounds][4];
  unsigned int bias1 = 0;
  u32x4 w2[kUnitRounds];
  float dot[16];
  if constexpr (kMlp) {
    const float* partial = static_cast<const float*>(a.workspace);
    const unsigned short* b1 = static_cast<const unsigned short*>(a.b1);
    const unsigned short* W2 = static_cast<const unsigned short*>(a.W2);
#pragma unroll
    for (int r = 0; r < kUnitRounds; ++r) {
      if (r == 0 || M > r * 2 * kPairs) {
        int m0 = 2 * pr + r * 2 * kPairs;
        if (m0 > M - 2) m0 = M - 2;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int ks = 4 * kq + j;
          const int kc = ks < ksplit ? ks : ksplit - 1;
          part[r][j] = *reinterpret_cast<const float2*>(partial + ((size_t)kc * a.B + b) * M + m0);
        }
      }
      if (r == 0 || M > r * 512) {
        int u0 = (r * 64 + lane) * 8;
        if (u0 > M - 8) u0 = M - 8;
        w2[r] = *reinterpret_cast<const u32x4*>(W2 + (size_t)hw * M + u0);
      }
    }
    // the first bias of the pair this thread finishes after the first barrier (pair = tid)
    int mb = 2 * tid;
    if (mb > M - 2) mb = M - 2;
    const unsigned int raw = *reinterpret_cast<const unsigned int*>(b1 ? b1 + mb : static_cast<const unsigned short*>(a.k_new));
    bias1 = b1 ? raw : 0u;
  } else {
    const u32x4* hid = reinterpret_cast<const u32x4*>(static_cast<const unsigned short*>(a.hidden_new) + (size_t)b * Dh);
    const u32x4* W = static_cast<const u32x4*>(a.W1);
    const int nchunk = Dh / 8;
#pragma unroll
    for (int h = 0; h < 16; ++h) dot[h] = 0.f;
    for (int c0 = 0; c0 < nchunk; c0 += kFThreads) {
      int ch = c0 + tid;
      const bool ok = ch < nchunk;
      if (!ok) ch = nchunk - 1;
      const u32x4 x = hid[ch];
      u32x4 wt[16];
#pragma unroll
      for (int h = 0; h < 16; ++h)
        if (h < H) wt[h] = W[(size_t)h * nchunk + ch];
#pragma unroll
      for (int h = 0; h < 16; ++h)
        if (h < H) dot[h] += ok ? dot8_bf16(x, wt[h]) : 0.f;
    }
  }

  // ---- 0b. loads that need the position: the ring rows of the slot about to be vacated
  // (read before it is known whether they are needed), the leaving token's score, and for
  // the paged layout the page of the prefix's next row
  const int q = p - w;
  const int slot = (w > 0) ? (p % w) : 0;
  float s_q = 0.f;
  u32x4 k_old = k_in, v_old = v_in;                      // no window: the new token itself may be kept
  if (w > 0) {
    const size_t ring_at = ((size_t)bh_r * w + slot) * lpr + piece_r;
    k_old = Kr[ring_at];
    v_old = Vr[ring_at];
    s_q = a.score_ring[(size_t)(b * H + hw) * w + slot];
  }
  if (a.block_table) {
    // paged prefix: the next row is row len % page_rows of the page in table slot
    // len / page_rows.  Expressed as a slab whose row `len` is that row, with room for
    // exactly one more row if the slot holds a page of the pool.
    const int len = len_r < 0 ? 0 : len_r;
    const int pslot = len >> a.log_page;
    const int pc = pslot < a.max_pages ? pslot : a.max_pages - 1;
    const int entry = a.block_table[(size_t)bh_r * a.max_pages + pc];
    const int page = pslot < a.max_pages ? entry : -1;
    const bool ok = page >= 0 && page < a.num_pages;
    cap_r = ok ? len_r + 1 : len_r;
    slab_r = (((long long)(ok ? page : 0)) << a.log_page) + (len & ((1 << a.log_page) - 1)) - len_r;
  }

  // ---- 1. partial sums (MLP) or per-wavefront sums (linear) into LDS; keep flags ----
  if constexpr (kMlp) {
#pragma unroll
    for (int r = 0; r < kUnitRounds; ++r) {
      if (r == 0 || M > r * 2 * kPairs) {
        const int m0 = 2 * pr + r * 2 * kPairs;
        float2 z = {0.f, 0.f};                             // this group's K-slices in order
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const bool on = 4 * kq + j < ksplit;
          z.x += on ? part[r][j].x : 0.f;
          z.y += on ? part[r][j].y : 0.f;
        }
        if (m0 < M) *reinterpret_cast<float2*>(zpart + (size_t)kq * M + m0) = z;
      }
    }
  } else {
#pragma unroll
    for (int h = 0; h < 16; ++h) {
      if (h < H) {
        const float v = wave_sum(dot[h]);
        if (lane == 0) s_red[h][wv] = v;
      }
    }
  }
  if (w > 0 && owner) s_keep[wv] = (q >= 0) && (s_q >= a.tau);
  __syncthreads();

  // ring -> prefix tail (kept), new -> ring slot, and the head's bookkeeping by the thread
  // that owns piece 0
  auto move_rows = [&]() {
    if (tid < npieces) {
      const bool keep = s_keep[head_r] != 0;
      if (keep && len_r < cap_r) {
        const size_t dst = ((size_t)slab_r + len_r) * lpr + piece_r;
        Kp[dst] = k_old;
        Vp[dst] = v_old;
      }
      if (w > 0) {
        const size_t ring_at = ((size_t)bh_r * w + slot) * lpr + piece_r;
        Kr[ring_at] = k_in;
        Vr[ring_at] = v_in;
      }
      if (piece_r == 0 && keep) {
        if (len_r < cap_r) {
          a.prefix_pos[(size_t)slab_r + len_r] = q;
          a.lengths[bh_r] = len_r + 1;
        } else if (a.error_flag) {
          *a.error_flag = 1;
        }
      }
    }
  };
  if (w > 0) move_rows();

  // ---- 2. scores of the new token: head wv by this wavefront, result in its lane 0 ----
  float s_new = 0.f;
  if constexpr (kMlp) {
    // the groups' sums in a fixed order, bias, GELU: pair `tid`
    if (2 * tid < M) {
      float2 z = *reinterpret_cast<const float2*>(zpart + 2 * tid);
#pragma unroll
      for (int x = 1; x < kKGroups; ++x) {
        const float2 t = *reinterpret_cast<const float2*>(zpart + (size_t)x * M + 2 * tid);
        z.x += t.x;
        z.y += t.y;
      }
      float2 gv;
      gv.x = gelu_erf(z.x + bf16_lo(bias1));
      gv.y = gelu_erf(z.y + bf16_hi(bias1));
      *reinterpret_cast<float2*>(g + 2 * tid) = gv;
    }
    __syncthreads();
    if (wv < H) {
      float acc = 0.f;
#pragma unroll
      for (int r = 0; r < kUnitRounds; ++r) {
        if (r == 0 || M > r * 512) {
          const int u0 = (r * 64 + lane) * 8;
          if (u0 < M) {
            const floatx4 g0 = *reinterpret_cast<const floatx4*>(g + u0);
            const floatx4 g1 = *reinterpret_cast<const floatx4*>(g + u0 + 4);
            const u32x4 wq = w2[r];
            acc += g0[0] * bf16_lo(wq[0]) + g0[1] * bf16_hi(wq[0]) + g0[2] * bf16_lo(wq[1]) +
                   g0[3] * bf16_hi(wq[1]) + g1[0] * bf16_lo(wq[2]) + g1[1] * bf16_hi(wq[2]) +
                   g1[2] * bf16_lo(wq[3]) + g1[3] * bf16_hi(wq[3]);
          }
        }
      }
      s_new = wave_sum(acc);
    }
  } else if (owner) {
#pragma unroll
    for (int x = 0; x < kFWaves; ++x) s_new += s_red[wv][x];
  }
  s_new += bf16_bits_to_float(bias2);
  if (w > 0) {
    if (owner) a.score_ring[(size_t)(b * H + wv) * w + slot] = s_new;
  } else {
    // no window: the new token itself is tested
    if (owner) s_keep[wv] = (q >= 0) && (s_new >= a.tau);
    __syncthreads();
    move_rows();
  }
  if (tid == 0) a.seq_pos[b] = p + 1;
}

}  // namespace

// The skinny first projection on its own (the prefill scorer uses it for short prompts):
// partial[ks][rows][M] fp32, ks = skinny_ksplit(rows, Dh, M, target_blocks).
int skinny_ksplit(long long rows, int Dh, int M, int target_blocks) {
  const long long nub = M / 32, ntb = (rows + 63) / 64;
  long long target = target_blocks / (nub * ntb);
  if (target < 1) target = 1;
  if (target > kMaxKSplit) target = kMaxKSplit;
  const int units = Dh / 64;               // a slice is a multiple of 64 inputs
  int ks = 1;
  for (int d = 1; d <= units && d <= target; ++d)
    if (units % d == 0) ks = d;
  return ks;
}

int launch_skinny_gemm(const void* hidden, const void* W1, float* partial, long long rows, int Dh,
                       int M, int ks, hipStream_t stream) {
  const dim3 grid(M / 32, ks, (unsigned)((rows + 63) / 64));
  decode_partial_kernel<<<grid, kPThreads, 0, stream>>>(
      static_cast<const unsigned short*>(hidden), static_cast<const unsigned short*>(W1), partial,
      (int)rows, Dh, M, Dh / ks);
  return hipGetLastError() == hipSuccess ? KVZAP_OK : KVZAP_ERR_RUNTIME;
}

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
  const size_t lds = (size_t)(a.M > 0 ? (1 + kKGroups) * a.M : 4) * sizeof(float);
  if (a.M > 0) decode_finish_kernel<true><<<a.B, kFThreads, lds, stream>>>(a, ks);
  else         decode_finish_kernel<false><<<a.B, kFThreads, lds, stream>>>(a, ks);
  return hipGetLastError() == hipSuccess ? KVZAP_OK : KVZAP_ERR_RUNTIME;
}

}  // namespace kvzap
