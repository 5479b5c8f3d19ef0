// KVzap-MLP forward (Sec. 3.3, Sec. 4.1; App. B Eq. 5):
//   scores = GELU(hidden . W1^T + b1) . W2^T + b2
//
// 99.8 % of the flops are the first projection, a [tokens x D_h] x [D_h x M]
// contraction: it runs on v_mfma_f32_32x32x16_bf16.  It is computed transposed,
// with the M hidden units on the MFMA row side and tokens on the column side, so
// that the fp32 accumulator layout (lane = token, registers = units) is exactly
// the B-operand layout of a second MFMA: bias, GELU and the M -> H projection
// are then fused into the epilogue without moving data between lanes, and the
// [tokens x M] activation never exists in memory.
//
// Block = 512 threads (8 wavefronts) = all M units x 128 tokens, so `hidden` is
// read from HBM exactly once and W1 (<= 6.6 MB, L2 resident) once per block.
// Wavefront (wu, wt): units [wu*M/4, (wu+1)*M/4) x tokens [wt*64, wt*64+64):
// UB x 2 accumulator blocks of 32x32.  K is walked in tiles of 64 (one 128-byte
// line per row); tile k+1 is fetched into registers while tile k is consumed
// from LDS.  LDS rows are 128 B with the 16-byte piece index XOR-swizzled by the
// row, which keeps both the ds_write_b128 and the operand ds_read_b128 free of
// bank conflicts.
#include "kvzap_internal.h"

namespace kvzap {
namespace {

constexpr int kThreads = 512;
constexpr int kTok = 128;     // tokens per block
constexpr int kBK = 64;       // K per LDS tile

__device__ __forceinline__ float gelu_exact(float z) {
  return 0.5f * z * (1.0f + erff(z * 0.70710678118654752f));
}

__device__ __forceinline__ int lds_off(int row, int piece) {   // bytes
  return row * 128 + ((piece ^ (row & 7)) << 4);
}

template <int UB>
__global__ __launch_bounds__(kThreads) void score_mlp_kernel(
    const unsigned short* __restrict__ hidden, const unsigned short* __restrict__ W1,
    const unsigned short* __restrict__ b1, const unsigned short* __restrict__ W2,
    const unsigned short* __restrict__ b2, float* __restrict__ scores,
    long long rows, int T, int Dh, int H) {
  constexpr int U = 128 * UB;                // = M
  constexpr int R = U + kTok;                // LDS tile rows: W1 rows then token rows
  constexpr int CH = R * 8 / kThreads;       // 16-byte pieces per thread per tile
  constexpr int CHW = U * 8 / kThreads;      // of which W1 pieces
  static_assert(R * 8 % kThreads == 0 && U * 8 % kThreads == 0, "tile split");
  extern __shared__ __align__(16) unsigned char smem[];

  const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
  const int wu = wid & 3, wt = wid >> 2;
  const int l32 = lane & 31, kg = lane >> 5;
  const long long row0 = (long long)blockIdx.x * kTok;

  // ---- global -> register staging: piece c of this thread is tile row (tid>>3)+64c ----
  const int ld_row = tid >> 3, ld_piece = tid & 7;
  const unsigned short* src[CH];
  int dst[CH];
#pragma unroll
  for (int c = 0; c < CH; ++c) {
    const int r = ld_row + 64 * c;
    if (c < CHW) {
      src[c] = W1 + (size_t)r * Dh + ld_piece * 8;
    } else {
      long long hr = row0 + (r - U);
      if (hr > rows - 1) hr = rows - 1;      // clamp: stays in bounds, result discarded
      src[c] = hidden + (size_t)hr * Dh + ld_piece * 8;
    }
    dst[c] = lds_off(r, ld_piece);
  }

  floatx16 acc[UB][2];
#pragma unroll
  for (int ub = 0; ub < UB; ++ub)
#pragma unroll
    for (int tb = 0; tb < 2; ++tb)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[ub][tb][e] = 0.0f;

  u32x4 stage[CH];
#pragma unroll
  for (int c = 0; c < CH; ++c) stage[c] = *reinterpret_cast<const u32x4*>(src[c]);
#pragma unroll
  for (int c = 0; c < CH; ++c) *reinterpret_cast<u32x4*>(smem + dst[c]) = stage[c];
  __syncthreads();

  const int a_row0 = wu * (32 * UB) + l32;          // + 32*ub
  const int b_row0 = U + wt * 64 + l32;             // + 32*tb
  const int nk = Dh / kBK;
  for (int kt = 0; kt < nk; ++kt) {
    const bool more = kt + 1 < nk;
    if (more) {
      const int koff = (kt + 1) * kBK;
#pragma unroll
      for (int c = 0; c < CH; ++c) stage[c] = *reinterpret_cast<const u32x4*>(src[c] + koff);
    }
#pragma unroll
    for (int kk = 0; kk < kBK / 16; ++kk) {
      const int piece = kk * 2 + kg;
      bf16x8 a[UB], b[2];
#pragma unroll
      for (int ub = 0; ub < UB; ++ub)
        a[ub] = *reinterpret_cast<const bf16x8*>(smem + lds_off(a_row0 + 32 * ub, piece));
#pragma unroll
      for (int tb = 0; tb < 2; ++tb)
        b[tb] = *reinterpret_cast<const bf16x8*>(smem + lds_off(b_row0 + 32 * tb, piece));
#pragma unroll
      for (int ub = 0; ub < UB; ++ub)
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
          acc[ub][tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ub], b[tb], acc[ub][tb], 0, 0, 0);
    }
    __syncthreads();                       // every wavefront is done with this tile
    if (more) {
#pragma unroll
      for (int c = 0; c < CH; ++c) *reinterpret_cast<u32x4*>(smem + dst[c]) = stage[c];
    }
    __syncthreads();
  }

  // ---- epilogue: bias + GELU, then the M -> H projection as a second MFMA ----
  // acc[ub][tb][r] is unit  ubase + 32*ub + 8*(r/4) + 4*kg + r%4  of token  l32 (+32*tb).
  // Registers 8s..8s+7 form the B operand of MFMA step s; the matching A operand
  // holds W2[head = l32][the same eight units] (zero for padded heads).
  const int ubase = wu * (32 * UB);
  floatx16 acc2[2];
#pragma unroll
  for (int tb = 0; tb < 2; ++tb)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc2[tb][e] = 0.0f;

#pragma unroll
  for (int ub = 0; ub < UB; ++ub) {
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      const int u0 = ubase + 32 * ub + 16 * s + 4 * kg;   // units u0..u0+3 and u0+8..u0+11
      u32x4 w2 = {0u, 0u, 0u, 0u};
      if (l32 < H) {
        const uint2 p0 = *reinterpret_cast<const uint2*>(W2 + (size_t)l32 * U + u0);
        const uint2 p1 = *reinterpret_cast<const uint2*>(W2 + (size_t)l32 * U + u0 + 8);
        w2.x = p0.x; w2.y = p0.y; w2.z = p1.x; w2.w = p1.y;
      }
      float bias[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int u = u0 + 8 * (e / 4) + (e % 4);
        bias[e] = b1 ? bf16_bits_to_float(b1[u]) : 0.0f;
      }
#pragma unroll
      for (int tb = 0; tb < 2; ++tb) {
        unsigned hi[4], lo[4];
#pragma unroll
        for (int e2 = 0; e2 < 4; ++e2) {
          unsigned short h16[2], l16[2];
#pragma unroll
          for (int q = 0; q < 2; ++q) {
            const int e = 2 * e2 + q;
            const float g = gelu_exact(acc[ub][tb][8 * s + e] + bias[e]);
            h16[q] = float_to_bf16_bits(g);
            l16[q] = float_to_bf16_bits(g - bf16_bits_to_float(h16[q]));
          }
          hi[e2] = (unsigned)h16[0] | ((unsigned)h16[1] << 16);
          lo[e2] = (unsigned)l16[0] | ((unsigned)l16[1] << 16);
        }
        const u32x4 ghi = {hi[0], hi[1], hi[2], hi[3]};
        const u32x4 glo = {lo[0], lo[1], lo[2], lo[3]};
        acc2[tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
            __builtin_bit_cast(bf16x8, w2), __builtin_bit_cast(bf16x8, ghi), acc2[tb], 0, 0, 0);
        acc2[tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
            __builtin_bit_cast(bf16x8, w2), __builtin_bit_cast(bf16x8, glo), acc2[tb], 0, 0, 0);
      }
    }
  }

  // ---- reduce the four unit-quarters through LDS, add b2, store [B,H,T] ----
  // acc2[tb][r] is head 8*(r/4) + 4*kg + r%4 of token wt*64 + 32*tb + l32
  float* red = reinterpret_cast<float*>(smem);     // [4][H][128]
#pragma unroll
  for (int tb = 0; tb < 2; ++tb)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int head = 8 * (r / 4) + 4 * kg + (r % 4);
      if (head < H) red[(wu * H + head) * kTok + wt * 64 + 32 * tb + l32] = acc2[tb][r];
    }
  __syncthreads();
  for (int i = tid; i < H * kTok; i += kThreads) {
    const int head = i / kTok, tok = i % kTok;
    const long long r = row0 + tok;
    if (r < rows) {
      float s = red[(0 * H + head) * kTok + tok];
      s += red[(1 * H + head) * kTok + tok];
      s += red[(2 * H + head) * kTok + tok];
      s += red[(3 * H + head) * kTok + tok];
      if (b2) s += bf16_bits_to_float(b2[head]);
      const long long bidx = r / T, t = r - bidx * T;
      scores[((size_t)bidx * H + head) * T + t] = s;
    }
  }
}

template <int UB>
int launch_one(const void* hidden, const void* W1, const void* b1, const void* W2,
               const void* b2, float* scores, long long rows, int T, int Dh, int H,
               hipStream_t stream) {
  constexpr size_t lds = (size_t)(128 * UB + kTok) * 128;
  static bool attr_set = false;
  if (!attr_set) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(score_mlp_kernel<UB>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
      return KVZAP_ERR_RUNTIME;
    attr_set = true;
  }
  const long long blocks = (rows + kTok - 1) / kTok;
  score_mlp_kernel<UB><<<dim3((unsigned)blocks), kThreads, lds, stream>>>(
      static_cast<const unsigned short*>(hidden), static_cast<const unsigned short*>(W1),
      static_cast<const unsigned short*>(b1), static_cast<const unsigned short*>(W2),
      static_cast<const unsigned short*>(b2), scores, rows, T, Dh, H);
  return hipGetLastError() == hipSuccess ? KVZAP_OK : KVZAP_ERR_RUNTIME;
}

}  // namespace

int launch_score_mlp(const void* hidden, const void* W1, const void* b1, const void* W2,
                     const void* b2, float* scores, int B, int T, int Dh, int M, int H,
                     hipStream_t stream) {
  const long long rows = (long long)B * T;
  switch (M / 128) {
    case 1: return launch_one<1>(hidden, W1, b1, W2, b2, scores, rows, T, Dh, H, stream);
    case 2: return launch_one<2>(hidden, W1, b1, W2, b2, scores, rows, T, Dh, H, stream);
    case 3: return launch_one<3>(hidden, W1, b1, W2, b2, scores, rows, T, Dh, H, stream);
    case 4: return launch_one<4>(hidden, W1, b1, W2, b2, scores, rows, T, Dh, H, stream);
    case 5: return launch_one<5>(hidden, W1, b1, W2, b2, scores, rows, T, Dh, H, stream);
    default: return KVZAP_ERR_UNSUPPORTED;
  }
}

}  // namespace kvzap
