// KVzap-Linear forward (Sec. 3.3, Sec. 4.1; App. B Eq. 6): scores = hidden . W^T + b.
//
// With H = 8 outputs the arithmetic intensity is H flop per byte of hidden
// state: the kernel is bound by streaming `hidden` from HBM exactly once.  Plain
// vector ALUs would need 64 FMAs plus bf16 unpacking per 16-byte load, which at
// 8 TB/s is more than the chip's fp32 vector rate; the matrix cores do the same
// work at a few per cent utilisation, so the contraction runs on
// v_mfma_f32_16x16x32_bf16 with tokens on the N side and heads (padded to 16) on
// the M side:
//   A (16 x 32)  = W rows (heads) from LDS, staged once per block
//   B (32 x 16)  = 16 tokens x 32 inputs, loaded straight from global memory in
//                  the instruction's operand layout (lane = token + 16*k-group,
//                  16 bytes per lane), no LDS round trip for the streamed data.
//                  Ordinary (cached) loads on purpose: a 128-byte line is
//                  consumed by two consecutive load instructions of the same
//                  wavefront, and with the non-temporal hint the second one
//                  fetched the line again (5.1 instead of 6.0 TB/s measured;
//                  a pure read stream reaches 6.0-6.4 TB/s on this part)
//   C (16 x 16)  = fp32 accumulators, heads 0..15 x 16 tokens
// Each wavefront owns groups of 16 consecutive tokens and walks the whole D_h.
#include "kvzap_internal.h"

namespace kvzap {
namespace {

// kThreads: wavefronts of a block share one copy of W in LDS; kUnroll: independent 16-byte
// loads in flight per lane
template <int kThreads, int kUnroll>
__global__ __launch_bounds__(kThreads) void score_linear_kernel(
    const unsigned short* __restrict__ hidden, const unsigned short* __restrict__ W,
    const unsigned short* __restrict__ bias, float* __restrict__ scores,
    long long rows, int T, int Dh, int H, int groups_per_block) {
  constexpr int kWaves = kThreads / 64;
  extern __shared__ __align__(16) unsigned char smem[];
  // W as [H][Dh/8 + 4] 16-byte pieces: the 64-byte pad per row spreads the 16
  // (head, k-group) pieces one ds_read_b128 touches over distinct banks
  u32x4* sW = reinterpret_cast<u32x4*>(smem);
  const int pieces_per_row = Dh / 8;
  const int lds_stride = pieces_per_row + 4;
  // W is contiguous ([H][Dh]): piece i of the whole matrix goes to row i / pieces_per_row.
  // Eight loads in flight per thread: one at a time, this staging was a chain of memory
  // round trips that took most of a short call (16 us of 20).
  const int total_pieces = H * pieces_per_row;
  for (int base = 0; base < total_pieces; base += kThreads * 8) {
    u32x4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int i = base + u * kThreads + (int)threadIdx.x;
      v[u] = reinterpret_cast<const u32x4*>(W)[i < total_pieces ? i : total_pieces - 1];
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int i = base + u * kThreads + (int)threadIdx.x;
      if (i < total_pieces) {
        const int h = i / pieces_per_row, p = i - h * pieces_per_row;
        sW[h * lds_stride + p] = v[u];
      }
    }
  }
  __syncthreads();

  const int lane = threadIdx.x & 63, wid = threadIdx.x >> 6;
  const int col = lane & 15;          // token within the group (B operand) / head (A operand)
  const int kg = lane >> 4;           // which 8 of the 32 inputs of one MFMA
  const long long ngroups = (rows + 15) / 16;
  const long long g_begin = (long long)blockIdx.x * groups_per_block;
  long long g_end = g_begin + groups_per_block;
  if (g_end > ngroups) g_end = ngroups;
  // lanes of the padded heads (col >= H) read a real row and zero it afterwards
  const bool head_ok = col < H;
  const u32x4* sWrow = sW + (size_t)(col % H) * lds_stride + kg;   // + 4*i per MFMA step
  const int steps = Dh / 32;
  const int steps_main = steps / kUnroll * kUnroll;
  const u32x4 zero4 = {0u, 0u, 0u, 0u};

  for (long long g = g_begin + wid; g < g_end; g += kWaves) {
    long long r = g * 16 + col;
    const bool valid = r < rows;
    if (!valid) r = rows - 1;          // clamp: loads stay in bounds, result discarded
    const u32x4* hrow = reinterpret_cast<const u32x4*>(hidden + (size_t)r * Dh) + kg;
    floatx4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int i0 = 0; i0 < steps_main; i0 += kUnroll) {
      u32x4 b[kUnroll];
#pragma unroll
      for (int u = 0; u < kUnroll; ++u)
        b[u] = hrow[(size_t)(i0 + u) * 4];
      // the W fragments of the whole batch are read from LDS while the global loads are in
      // flight: read one by one in front of their MFMAs, each exposed its LDS latency when a
      // wavefront is alone on its SIMD (13 of the 18 us of a short call)
      u32x4 a[kUnroll];
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        const u32x4 w = sWrow[(size_t)(i0 + u) * 4];
        a[u] = head_ok ? w : zero4;
      }
      __builtin_amdgcn_sched_barrier(0);               // keep the reads ahead of the MFMAs
#pragma unroll
      for (int u = 0; u < kUnroll; ++u)
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
            __builtin_bit_cast(bf16x8, a[u]), __builtin_bit_cast(bf16x8, b[u]), acc, 0, 0, 0);
    }
    for (int i = steps_main; i < steps; ++i) {
      const u32x4 b = hrow[(size_t)i * 4];
      const u32x4 a = head_ok ? sWrow[(size_t)i * 4] : zero4;
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
          __builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
    }
    // C layout: lane holds token `col`, heads 4*kg + e
    if (valid) {
      const long long bidx = r / T;
      const long long t = r - bidx * T;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int h = 4 * kg + e;
        if (h < H) {
          const float bv = bias ? bf16_bits_to_float(bias[h]) : 0.0f;
          scores[((size_t)bidx * H + h) * T + t] = acc[e] + bv;
        }
      }
    }
  }
}

// Short inputs (up to 512 groups of 16 tokens; 1024 tokens: 10 us against 18 us): with one group per wavefront the walk over
// D_h above is what a call costs (13 us at D_h = 4096: 128 operand loads through one CU's
// texture path per wavefront, however many are in flight).  Here the four wavefronts of a
// block share ONE group and take a quarter of D_h each, W comes straight from global memory
// (L2) like the tokens, so there is no staging and a single batch of loads; the four partial
// accumulators are added in a fixed order through LDS.
__global__ __launch_bounds__(256) void score_linear_short_kernel(
    const unsigned short* __restrict__ hidden, const unsigned short* __restrict__ W,
    const unsigned short* __restrict__ bias, float* __restrict__ scores,
    long long rows, int T, int Dh, int H) {
  __shared__ floatx4 red[4][64];
  const int lane = threadIdx.x & 63, wid = threadIdx.x >> 6;
  const int col = lane & 15, kg = lane >> 4;
  long long r = (long long)blockIdx.x * 16 + col;
  const bool valid = r < rows;
  if (!valid) r = rows - 1;
  const bool head_ok = col < H;
  const int per = Dh / 128;                              // MFMA steps per wavefront (D_h % 128 == 0)
  const u32x4* hrow = reinterpret_cast<const u32x4*>(hidden + (size_t)r * Dh) + kg + (size_t)wid * per * 4;
  const u32x4* wrow = reinterpret_cast<const u32x4*>(W + (size_t)(col % H) * Dh) + kg + (size_t)wid * per * 4;
  const u32x4 zero4 = {0u, 0u, 0u, 0u};
  floatx4 acc = {0.f, 0.f, 0.f, 0.f};
  constexpr int kBatch = 16;
  for (int i0 = 0; i0 < per; i0 += kBatch) {
    u32x4 a[kBatch], b[kBatch];
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int i = i0 + u < per ? i0 + u : per - 1;     // clamped; the surplus is not accumulated
      b[u] = hrow[(size_t)i * 4];
      a[u] = wrow[(size_t)i * 4];
    }
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      if (i0 + u < per)                                  // uniform
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
            __builtin_bit_cast(bf16x8, head_ok ? a[u] : zero4), __builtin_bit_cast(bf16x8, b[u]),
            acc, 0, 0, 0);
    }
  }
  red[wid][lane] = acc;
  __syncthreads();
  if (wid == 0 && valid) {
    const floatx4 s = ((red[0][lane] + red[1][lane]) + red[2][lane]) + red[3][lane];
    const long long bidx = r / T;
    const long long t = r - bidx * T;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int h = 4 * kg + e;
      if (h < H) {
        const float bv = bias ? bf16_bits_to_float(bias[h]) : 0.0f;
        scores[((size_t)bidx * H + h) * T + t] = s[e] + bv;
      }
    }
  }
}

template <int kThreads, int kUnroll>
int launch_linear(const void* hidden, const void* W, const void* b, float* scores, long long rows,
                  int T, int Dh, int H, long long want_blocks, hipStream_t stream) {
  constexpr int kWaves = kThreads / 64;
  const long long ngroups = (rows + 15) / 16;
  long long gpb = (ngroups + want_blocks - 1) / want_blocks;
  if (gpb < kWaves) gpb = kWaves;                     // at least one group per wavefront
  const long long blocks = (ngroups + gpb - 1) / gpb;
  const size_t lds = (size_t)H * ((size_t)Dh * 2 + 64);   // validated <= 160 KB by the caller
  // once per process, which drives one GPU (thread-safe: a function-local static)
  static const hipError_t attr_rc =
      hipFuncSetAttribute(reinterpret_cast<const void*>(score_linear_kernel<kThreads, kUnroll>),
      hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
  if (attr_rc != hipSuccess) return KVZAP_ERR_RUNTIME;
  score_linear_kernel<kThreads, kUnroll><<<dim3((unsigned)blocks), kThreads, lds, stream>>>(
      static_cast<const unsigned short*>(hidden), static_cast<const unsigned short*>(W),
      static_cast<const unsigned short*>(b), scores, rows, T, Dh, H, (int)gpb);
  return hipGetLastError() == hipSuccess ? KVZAP_OK : KVZAP_ERR_RUNTIME;
}

}  // namespace

int launch_score_linear(const void* hidden, const void* W, const void* b, float* scores,
                        int B, int T, int Dh, int H, hipStream_t stream) {
  const long long rows = (long long)B * T;
  const long long ngroups = (rows + 15) / 16;
  // from 64k tokens: 16-wavefront blocks (W is staged into LDS once per block, and 16 x 8
  // loads in flight per block are what the HBM stream needs: 128k tokens 194 us against
  // 205 us with small blocks); shorter inputs: 4-wavefront blocks so that more CUs take part
  // (32k tokens: 60 us against 69 us)
  if (ngroups >= 4096) return launch_linear<1024, 8>(hidden, W, b, scores, rows, T, Dh, H, 1024, stream);
  if (ngroups > 512 || Dh % 128 != 0)       // 16k tokens: 26 us with the kernel above, 32 us here
    return launch_linear<256, 8>(hidden, W, b, scores, rows, T, Dh, H, 1024, stream);
  score_linear_short_kernel<<<dim3((unsigned)ngroups), 256, 0, stream>>>(
      static_cast<const unsigned short*>(hidden), static_cast<const unsigned short*>(W),
      static_cast<const unsigned short*>(b), scores, rows, T, Dh, H);
  return hipGetLastError() == hipSuccess ? KVZAP_OK : KVZAP_ERR_RUNTIME;
}

}  // namespace kvzap
