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
// Which kernel runs (launch_score_mlp): D_h >= 256 takes score_mlp_frag_kernel (below, the
// one the throughput figures are about) -- cut over K as well while its token blocks do not
// fill the chip, and replaced by the decode path's skinny GEMM for a few hundred tokens
// (both finish in score_finish_kernel); D_h < 256 takes score_mlp_kernel, described here:
//
// Block = 512 threads (8 wavefronts) = all M units x 128 tokens, so `hidden` is
// read from HBM exactly once and W1 (<= 6.6 MB, L2 resident) once per block.
// Wavefront (wu, wt): units [wu*M/4, (wu+1)*M/4) x tokens [wt*64, wt*64+64):
// UB x 2 accumulator blocks of 32x32.  K is walked in tiles of 64 (one 128-byte
// line per row); tile k+1 is fetched into registers while tile k is consumed
// from LDS.  LDS rows are 128 B with the 16-byte piece index XOR-swizzled by the
// row, which keeps both the ds_write_b128 and the operand ds_read_b128 free of
// bank conflicts.
#include <type_traits>
#include <utility>

#include "frag_schedule.h"
#include "kvzap_internal.h"

namespace kvzap {
namespace {

constexpr int kThreads = 512;
constexpr int kTok = 128;     // tokens per block
constexpr int kBK = 64;       // K per LDS tile

// GELU(z) = z * Phi(z) with Phi from the rational erfc approximation of Abramowitz & Stegun
// 7.1.26 (|error| <= 1.5e-7 on erf, i.e. at fp32 rounding level): one rcp, one exp2 and
// ten FMA-class operations per element instead of the ~40 of a library erff, which matters
// because the epilogue's vector ALU work is not overlapped with matrix-core work.
__device__ __forceinline__ float gelu_exact(float z) {
  const float x = fabsf(z);
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f * 0.70710678118654752f, x, 1.0f));
  // 0.5 * (a1 t + ... + a5 t^5): the 0.5 of Phi is folded into the coefficients
  float p = fmaf(t, 0.5f * 1.061405429f, 0.5f * -1.453152027f);
  p = fmaf(t, p, 0.5f * 1.421413741f);
  p = fmaf(t, p, 0.5f * -0.284496736f);
  p = fmaf(t, p, 0.5f * 0.254829592f);
  // exp(-z^2 / 2) = 2^(-z^2 * log2(e) / 2)
  const float e = __builtin_amdgcn_exp2f(z * z * (-0.5f * 1.4426950408889634f));
  const float half_erfc = (t * p) * e;                 // 0.5 * erfc(|z| / sqrt 2) = Phi(-|z|)
  // Phi(z) = 0.5 + copysign(0.5 - Phi(-|z|), z)
  const float phi = 0.5f + copysignf(0.5f - half_erfc, z);
  return z * phi;
}

// The fused epilogue's GELU: z * sigmoid(z * (c0 + c1 z^2 + c2 z^4)), the coefficients fitted
// to z * Phi(z) (the erf form) in the minimax sense: |error| <= 2.6e-5 absolute for every z
// (z^2 is clamped at 64, beyond which the sigmoid is 0 or 1 to 1e-12).  Its result is rounded
// to fp16 for the second projection (relative 4.9e-4), so the 1.5e-7 of gelu_exact would buy
// nothing there; this form is seven plain operations, one exp2 and one rcp, half the vector
// work of gelu_exact, and that work is not overlapped with matrix-core work.  The constants
// carry the factor -log2(e): sigmoid(x) = 1 / (1 + 2^(-x log2 e)).  z -> -inf gives -0, NaN
// stays NaN.
__device__ __forceinline__ float gelu_fused(float z) {
  const float z2 = fminf(z * z, 64.0f);
  float q = fmaf(z2, 0.001014264184050262f, -0.10677573084831238f);
  q = fmaf(z2, q, -2.301121234893799f);
  const float e = __builtin_amdgcn_exp2f(z * q);
  return z * __builtin_amdgcn_rcpf(1.0f + e);
}

// LDS tile of 128-byte rows (eight 16-byte pieces): byte offset of logical piece `piece` of
// `row`.  The piece index is XOR-ed with bits 1..3 of the row: a ds_read_b128 serves 16 lanes
// (16 consecutive rows, one piece each) at a time, and with two rows per 256 bytes of banks
// the 16 accesses then fall on 16 different 16-byte bank groups (with row & 7 rows r and r+8
// met in the same group).
__device__ __forceinline__ int lds_swizzle(int row) { return (row >> 1) & 7; }
__device__ __forceinline__ int lds_off(int row, int piece) {   // bytes
  return row * 128 + ((piece ^ lds_swizzle(row)) << 4);
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
        // GELU output as a bf16 pair: ghi = round(g), glo = round(g - ghi) (hardware RNE
        // conversions, two values per instruction)
        bf16x8 ghi, glo;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float g = gelu_exact(acc[ub][tb][8 * s + e] + bias[e]);
          ghi[e] = (__bf16)g;
          glo[e] = (__bf16)(g - (float)ghi[e]);
        }
        acc2[tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, w2), ghi,
                                                           acc2[tb], 0, 0, 0);
        acc2[tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, w2), glo,
                                                           acc2[tb], 0, 0, 0);
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


// ---------------------------------------------------------------------------
// Main variant (D_h >= 256).  A 128k-token launch moves 4.3 GB of W1 operands from L2 to
// the CUs and 1 GB of hidden states from HBM; the structure keeps both off the matrix
// cores' critical path, and W1 never passes through LDS:
//   * a tiny pre-pass copies W1 into the workspace in MFMA A-fragment order
//     ([k-tile][32-unit block][k-step][lane] x 16 B), so that every A fragment
//     is ONE fully coalesced 1 KB load straight into registers;
//   * each of the 4 wavefronts owns M/4 units x all 128 tokens (UB x 4
//     accumulator blocks in the accumulation registers) and keeps up to two K tiles
//     of its own A fragments in registers: a fragment is re-loaded with the data of
//     tile t+2 one MFMA group after its last use;
//   * only `hidden` goes through LDS: a ring of kPD+1 stages of 128 rows x
//     128 B filled by load-to-LDS kPD tiles ahead (it is the HBM-latency
//     stream), rows swizzled by XOR-ing the 16-byte piece index with bits 1..3 of the row
//     on the global-address side;
//   * one barrier per 64-wide K tile; loads and LDS reads sit between the MFMAs in
//     source order, pinned with scheduling barriers;
//   * every operand load is issued as inline asm and waited for with a count that is a
//     constant expression of that fixed order (the compiler's own counts do not see the
//     load-to-LDS operations in the same in-order queue and always wait for too much).
//     To the compiler such a load has written its register when it is issued: the build
//     checks the generated assembly for any use of a register before its wait
//     (isa_lint.py), and no branch may sit between such a load and its wait.
// ---------------------------------------------------------------------------
constexpr int kChipCUs = 256;                // compute units of the part (8 XCDs x 32)
constexpr int kPD = 3;                       // hidden tiles in flight
constexpr int kNS = kPD + 1;                 // LDS stages

// W1 [M][Dh] -> A-fragment order: [Dh/64][M/32][4][64 lanes] x 16 B, where lane
// (i = lane & 31, kg = lane >> 5) of k-step kk holds W1[rb*32 + i][kt*64 + kk*16 + kg*8 .. +8]
// gain (optional, bf16 [Dh]): the copy holds W1[m][k] * gain[k] rounded to bf16 -- the first
// projection of a surrogate that is applied to gain-scaled (normalised) states
__global__ __launch_bounds__(256) void arrange_w1_kernel(const u32x4* __restrict__ W1,
                                                         u32x4* __restrict__ W1f, int M, int Dh,
                                                         const u32x4* __restrict__ gain) {
  const int n = M * (Dh / 8);
  const int rbs = M / 32;
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) {
    const int lane = i & 63, kk = (i >> 6) & 3, rb = (i >> 8) % rbs, kt = i / (256 * rbs);
    const int row = rb * 32 + (lane & 31), piece = kt * 8 + kk * 2 + (lane >> 5);
    u32x4 w = W1[(size_t)row * (Dh / 8) + piece];
    if (gain) {
      const u32x4 g = gain[piece];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float lo = __uint_as_float(w[e] << 16) * __uint_as_float(g[e] << 16);
        const float hi = __uint_as_float(w[e] & 0xffff0000u) * __uint_as_float(g[e] & 0xffff0000u);
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        const bf16x2 p = {(__bf16)lo, (__bf16)hi};
        w[e] = __builtin_bit_cast(unsigned int, p);
      }
    }
    W1f[i] = w;
  }
}

// What the kernel does besides scoring when its input is the un-normalised residual stream
// (kNorm): every token's 1 / sqrt(mean x^2 + eps) is accumulated next to the first projection
// (the B fragments are in registers anyway), applied to the accumulators before b1 and GELU
// -- the gain is already in the prepared W1 -- written to `rstd`, and, if `normed` is given,
// the block finally re-reads its own rows and writes x * rstd * gain as bf16.
struct NormArgs {
  const unsigned short* gain;    // bf16 [Dh]
  float eps;
  float* rstd;                   // fp32 [rows]
  unsigned short* normed;        // bf16 [rows, Dh] or nullptr
};

// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>), in order: loops whose index
// has to be a constant expression (an instruction's immediate offset, a wait count)
template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// One A fragment: 16 bytes per lane from  sbase + voff + OFF  (sbase uniform, in scalar
// registers).  Issued as inline asm so that the compiler does not size the wait for it:
// its own count knows nothing of the load-to-LDS operations that share the in-order
// vector-memory queue and therefore always waits for more than the fragment (the hidden
// tiles issued behind it as well, i.e. for HBM).  The matching wait is wait_fragment().
template <int OFF>
__device__ __forceinline__ void load_fragment(bf16x8& dst, unsigned voff, const unsigned char* sbase) {
  asm volatile("global_load_dwordx4 %0, %1, %2 offset:%3" : "=v"(dst) : "v"(voff), "s"(sbase), "n"(OFF));
}
// Wait until at most N vector-memory operations issued after the fragment's load are still
// outstanding.  A scheduling barrier keeps every use of the fragment behind the wait (a register
// tie would do that too, but costs a hazard s_nop after each wait); the build's check of the
// generated assembly is what holds it to that.
template <int N>
__device__ __forceinline__ void wait_fragment(bf16x8& frag) {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  (void)frag;
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N));
  __builtin_amdgcn_sched_barrier(0);
}

// Small loads of the block's constants (W2, b1, b2), issued ahead of everything else and used
// after the prologue's wait: issued by hand for the same reason -- the compiler, which does not
// see the hand-issued operations behind them, would wait for ALL of those before the first
// use.  Every lane loads, from an address clamped into the array, and what should not have been
// loaded is zeroed after the wait: between a load and arrived() its destination must not pass
// through a branch, where the compiler would copy the not yet written register.
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void load_async(u32x4& dst, const void* p) {
  asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(dst) : "v"(p));
}
__device__ __forceinline__ void load_async(u32x2& dst, const void* p) {
  asm volatile("global_load_dwordx2 %0, %1, off" : "=v"(dst) : "v"(p));
}
__device__ __forceinline__ void load_async_u16(unsigned& dst, const void* p) {   // zero-extended
  asm volatile("global_load_ushort %0, %1, off" : "=v"(dst) : "v"(p));
}
template <class T>
__device__ __forceinline__ void arrived(T& v) {      // orders every use of v behind the wait before it
  asm volatile("" : "+v"(v));
}

// The same for a B fragment from LDS (16 bytes per lane at byte address addr + OFF): the
// compiler places a wait for everything outstanding at the head of a loop whose entry and
// back edge arrive with different reads in flight, which exposes the latency of the read
// issued just before.  LDS operations of a wavefront complete in issue order.
template <int OFF>
__device__ __forceinline__ void read_fragment(bf16x8& dst, unsigned addr) {
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFF));
}
template <int N>
__device__ __forceinline__ void wait_lds_fragment(bf16x8& frag) {
  static_assert(N >= 0 && N < 16, "lgkmcnt is a 4-bit counter");
  (void)frag;
  asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N));
  __builtin_amdgcn_sched_barrier(0);
}

// UB 32-unit blocks per wavefront, TB 32-token blocks per block; kSplit: the block covers one
// K-slice (blockIdx.y) and writes its part of the first projection to `partial`
template <int UB, int TB, bool kSplit, bool kNorm = false>
__global__ __launch_bounds__(256) void score_mlp_frag_kernel(
    const unsigned short* hidden, const unsigned char* W1f,   // not __restrict__: their loads must stay ordered w.r.t. the waits
    const unsigned short* __restrict__ b1, const unsigned short* __restrict__ W2,
    const unsigned short* __restrict__ b2, float* __restrict__ scores,
    long long rows, int T, int Dh, int H, int nk, float* __restrict__ partial, NormArgs norm) {
  static_assert(!(kSplit && kNorm), "the normalising form is the single-kernel path");
  constexpr int U = 128 * UB;
  constexpr int TOK = 32 * TB;               // tokens per block
  constexpr int STAGE = TOK * 128;           // bytes per LDS stage (TOK rows of one K tile)
  constexpr int NDJ = TB;                    // load-to-LDS instructions per wavefront per tile
  extern __shared__ __align__(16) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wid = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, kg = lane >> 5;
  const long long row0 = (long long)blockIdx.x * TOK;
  const int rows_here = (rows - row0 < TOK) ? (int)(rows - row0) : TOK;

  // The epilogue's A operand (W2, a few KB) is staged in LDS behind the ring, converted to
  // fp16 and zero-filled up to 16 heads: read from global memory in the epilogue, every one of
  // its small loads would expose a full memory round trip with nothing to overlap it.  b1 is
  // what the accumulators start from.  Both are loaded here, ahead of the prologue's traffic,
  // and used as soon as they have arrived, while that traffic is still on its way
  // (vector-memory operations complete in issue order).
  constexpr int kW2Pieces = U / 128;                    // 16-byte pieces of the 16 x U matrix per thread
  unsigned char* const sW2 = smem + kNS * STAGE;        // [16][U] fp16
  u32x4 w2_stage[kW2Pieces];
#pragma unroll
  for (int i = 0; i < kW2Pieces; ++i) {
    const int piece = i * 256 + tid, last = H * (U / 8) - 1;
    load_async(w2_stage[i], reinterpret_cast<const u32x4*>(W2) + (piece < last ? piece : last));
  }
  // accumulator register 4q+e of block (ub, .) is unit wid*32*UB + 32*ub + 8*q + 4*kg + e
  u32x2 b1_stage[UB][4];
  if constexpr (!kSplit) {
#pragma unroll
    for (int ub = 0; ub < UB; ++ub)
#pragma unroll
      for (int q = 0; q < 4; ++q)   // without b1: the same offsets into W2 (H*U >= U elements), zeroed later
        load_async(b1_stage[ub][q], (b1 ? b1 : W2) + wid * (32 * UB) + 32 * ub + 8 * q + 4 * kg);
  }

  // b2 is loaded here and waits in LDS for the very end: a global load in the tail would
  // expose a memory round trip with nothing left to overlap it
  float* const sB2 = reinterpret_cast<float*>(sW2 + 16 * U * 2 + 2 * TOK * sizeof(float) + U * sizeof(float));   // [16]
  unsigned b2_stage;
  load_async_u16(b2_stage, b2 ? b2 + (tid < H ? tid : 0) : W2);

  // hidden load-to-LDS: instruction j (0..3) of wavefront w fills LDS chunk j*4+w of a
  // stage = rows (j*4+w)*8 + lane/8, physical piece lane%8 <- logical piece (lane%8) ^ lds_swizzle(row)
  // blockIdx.y: the K-slice of nk tiles this block covers (one slice unless `partial` is set)
  const int kt0 = kSplit ? blockIdx.y * nk : 0;
  const unsigned char* hb = reinterpret_cast<const unsigned char*>(hidden + (size_t)row0 * Dh) + (size_t)kt0 * (kBK * 2);
  unsigned h_off[NDJ];
#pragma unroll
  for (int j = 0; j < NDJ; ++j) {
    int r = (j * 4 + wid) * 8 + (lane >> 3);
    const int p = (lane & 7) ^ lds_swizzle(r);
    if (r > rows_here - 1) r = rows_here - 1;            // clamp: in bounds, result discarded
    h_off[j] = (unsigned)r * (unsigned)Dh * 2u + (unsigned)p * 16u;
  }
  const unsigned lds0 = lds_address(smem);
  auto dma = [&](int j, int tile) {
    // streamed (non-temporal): every hidden byte is read once, while the W1 fragments that all
    // blocks share have to stay in the same L2; measured 2 % on the launch
    load_to_lds_b128_stream(hb + (size_t)tile * (kBK * 2), h_off[j],
                            lds0 + (unsigned)((tile % kNS) * STAGE + (j * 4 + wid) * 1024));
  };
  // A fragments of this wavefront: unit blocks rb = wid*UB + ub; fragment (ub, kk) of K tile t
  // is the KB at  abase + t*kATile + (ub*4 + kk)*1024, 16 bytes per lane.  They are loaded
  // kLead tiles ahead into kLead register sets.
  constexpr int kLead = (UB <= 4 && !kNorm) ? 2 : 1;
  constexpr size_t kATile = (size_t)(U / 32) * 4 * 1024;
  const unsigned char* abase = W1f + ((size_t)kt0 * (U / 32) * 4 + (size_t)wid * UB * 4) * 1024;
  unsigned a_voff[UB];
#pragma unroll
  for (int ub = 0; ub < UB; ++ub) a_voff[ub] = (unsigned)lane * 16u + (unsigned)ub * 4096u;

  floatx16 acc[UB][TB];

  // kNorm: sum of x^2 of token 32*wid + l32 over this lane's half of every K step (a wavefront
  // beyond the last token block re-reads that block and drops the result)
  float ssq = 0.0f;
  bf16x8 xb[4];
  const int xblock = wid < TB ? wid : TB - 1;
  // nk >= kPD + 1 tiles (checked by the launcher)
  // a[s][kk][ub]: register set s holds step kk of K tile t for (t + nk) % kLead == s, and is
  // re-filled fragment by fragment with tile t + kLead
  bf16x8 a[kLead][4][UB];
  bf16x8 b[2][TB];
  // ---- prologue: the A fragments of tiles 0..kLead-1, then hidden tiles 0..kPD-1 ----
  auto load_tile_fragments = [&](auto set_, int tile) {
    constexpr int set = decltype(set_)::value;
    const unsigned char* sb = abase + (size_t)tile * kATile;
    static_for<4 * UB>([&](auto g_) {
      constexpr int kk = decltype(g_)::value / UB, ub = decltype(g_)::value % UB;
      load_fragment<kk * 1024>(a[set][kk][ub], a_voff[ub], sb);
    });
  };
  // Issue order: fragments of tile 0, hidden tiles 0 and 1, (fragments of tile 1,) hidden tile
  // 2.  Everything up to hidden tile 1 must have arrived before tile 0 starts: its fragments,
  // hidden tile 0, and hidden tile 1, which tile 0's hand-over cannot count for because no
  // whole tile of fragment loads follows it yet.  Tile 1's fragments stay in flight; each is
  // followed by hidden tile 2's NDJ operations, at least as many as tile_body() assumes behind
  // a fragment's load.
  static_assert(kPD == 3, "the wait counts are written for three hidden tiles in flight");
  auto issue_hidden = [&](int d) {
#pragma unroll
    for (int j = 0; j < NDJ; ++j) dma(j, d);
  };
  if constexpr (kLead == 1) {
    load_tile_fragments(std::integral_constant<int, 0>{}, 0);
    issue_hidden(0); issue_hidden(1); issue_hidden(2);
  } else {
    if (nk & 1) {
      load_tile_fragments(std::integral_constant<int, 1>{}, 0);
      issue_hidden(0); issue_hidden(1);
      load_tile_fragments(std::integral_constant<int, 0>{}, 1);
    } else {
      load_tile_fragments(std::integral_constant<int, 0>{}, 0);
      issue_hidden(0); issue_hidden(1);
      load_tile_fragments(std::integral_constant<int, 1>{}, 1);
    }
    issue_hidden(2);
  }
  // The block's constants were issued ahead of all that and arrive one L2 round trip later:
  // they are converted and the accumulators are set while the fragments and the hidden tiles
  // are still on their way.
  __builtin_amdgcn_sched_barrier(0);
  wait_vmcnt<kLead * 4 * UB + kPD * NDJ>();
#pragma unroll
  for (int i = 0; i < kW2Pieces; ++i) {
    arrived(w2_stage[i]);
    if (i * 256 + tid >= H * (U / 8)) w2_stage[i] = u32x4{0u, 0u, 0u, 0u};
  }
  if constexpr (!kSplit) {
#pragma unroll
    for (int ub = 0; ub < UB; ++ub)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        arrived(b1_stage[ub][q]);
        if (!b1) b1_stage[ub][q] = u32x2{0u, 0u};
      }
  }
  arrived(b2_stage);
  if (!b2 || tid >= H) b2_stage = 0u;
#pragma unroll
  for (int i = 0; i < kW2Pieces; ++i) {
    f16x8 w;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      w[2 * e] = (_Float16)__uint_as_float(w2_stage[i][e] << 16);
      w[2 * e + 1] = (_Float16)__uint_as_float(w2_stage[i][e] & 0xffff0000u);
    }
    reinterpret_cast<f16x8*>(sW2)[i * 256 + tid] = w;
  }
  if (tid < 16) sB2[tid] = bf16_bits_to_float((unsigned short)b2_stage);
  if constexpr (kNorm) {
    // b1 comes after the row scale: it waits in LDS for the epilogue instead of riding in
    // the accumulators (one lane of every 32 holds each unit's value)
    float* const sB1 = reinterpret_cast<float*>(sW2 + 16 * U * 2 + TOK * sizeof(float));   // [U]
    if (l32 == 0) {
#pragma unroll
      for (int ub = 0; ub < UB; ++ub)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const floatx4 v = {__uint_as_float(b1_stage[ub][q].x << 16), __uint_as_float(b1_stage[ub][q].x & 0xffff0000u),
                             __uint_as_float(b1_stage[ub][q].y << 16), __uint_as_float(b1_stage[ub][q].y & 0xffff0000u)};
          *reinterpret_cast<floatx4*>(sB1 + wid * (32 * UB) + 32 * ub + 8 * q + 4 * kg) = v;
        }
    }
  }
  // the first projection accumulates on top of b1 (a K-slice of a split launch: on zero)
#pragma unroll
  for (int ub = 0; ub < UB; ++ub)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      float v[4] = {0.f, 0.f, 0.f, 0.f};
      if constexpr (!kSplit && !kNorm) {
        v[0] = __uint_as_float(b1_stage[ub][q].x << 16); v[1] = __uint_as_float(b1_stage[ub][q].x & 0xffff0000u);
        v[2] = __uint_as_float(b1_stage[ub][q].y << 16); v[3] = __uint_as_float(b1_stage[ub][q].y & 0xffff0000u);
      }
#pragma unroll
      for (int tb = 0; tb < TB; ++tb)
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[ub][tb][4 * q + e] = v[e];
    }
  // now everything up to hidden tile 1 (all but tile 1's fragments and hidden tile 2)
  __builtin_amdgcn_sched_barrier(0);
  wait_vmcnt<frag::prologue_wait(UB, NDJ, kLead)>();
#pragma unroll
  for (int s2 = 0; s2 < kLead; ++s2)
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
#pragma unroll
      for (int ub = 0; ub < UB; ++ub) arrived(a[s2][kk][ub]);
  block_barrier_no_drain();
  // B fragment (step kk, token block tb) of a tile: lane (l32, kg) reads piece kk*2+kg of row
  // 32*tb + l32; the swizzle depends on l32 and kk only, token blocks are 4 KB apart
  unsigned b_off[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) b_off[kk] = lds0 + (unsigned)lds_off(l32, kk * 2 + kg);
  auto read_b = [&](auto kk_, auto tb_, int tile) {          // into b[kk & 1][tb]
    constexpr int kk = decltype(kk_)::value, tb = decltype(tb_)::value;
    read_fragment<tb * 4096>(b[kk & 1][tb], b_off[kk] + (unsigned)((tile % kNS) * STAGE));
  };
  // the reads of step kk+1 are issued during step kk, token block tb's in group tb*UB/TB
  constexpr auto reads_in_group = [](int ub) {
    int n = 0;
    for (int tb = 0; tb < TB; ++tb) n += (tb * UB / TB == ub) ? 1 : 0;
    return n;
  };
  static_for<TB>([&](auto tb_) { read_b(std::integral_constant<int, 0>{}, tb_, 0); });

  // One K tile.  R = min(nk - t, kPD + 1) is a compile-time tag: it says which later tiles
  // exist (t+1: hand-over; t+kLead: fragments to re-load; t+kPD: hidden tile to fetch) and
  // which earlier tiles issued what, i.e. everything the wait counts depend on; the body is a
  // single basic block whose instruction order is the source order.
  //
  // The hand-over to tile t+1 sits in the MIDDLE of tile t (before k-step 2), not at its
  // end: after that barrier the B reads of (t+1, step 0) are spread over k-step 3 like any
  // other step's, so no LDS latency is exposed between tiles, and the load-to-LDS of tile
  // t+kPD (which overwrites the stage of tile t-1, read for the last time before every
  // wavefront's arrival at this barrier) is issued during k-steps 2 and 3.
  //
  // Vector-memory operations of a wavefront complete in issue order.  Per tile, in order:
  //   group G = kk*UB + ub (0 .. 4*UB-1):  [wait for fragment G]  MFMA  MFMA
  //                                        [load-to-LDS j of tile t+kPD, if G == dma_group(j)]
  //                                        MFMA  [load fragment G-1]  (MFMA)
  //   end of tile:                         [load fragment 4*UB-1]
  // so the number of operations issued after fragment G's load (kLead tiles back) and before
  // its wait is known at compile time, and that many may stay outstanding.
  // The counts live in frag_schedule.h (a host test simulates the queue against them).
  constexpr int NG = frag::groups(UB);
  static_assert(frag::kHiddenAhead == kPD, "one constant, two names");
  static_assert(frag::lead_is_safe(UB, NDJ, kLead), "tile 1's hand-over is not covered with this shape");
  auto tile_body = [&](int t, auto r_tag, auto set_tag) {
    constexpr int R = decltype(r_tag)::value, set = decltype(set_tag)::value;
    constexpr bool next = R > 1, more = frag::reloads_fragments(R, 0, kLead),
                   more_pd = frag::fetches_hidden(R, 0);
    const unsigned char* a_next = abase + (size_t)(t + kLead) * kATile;
    static_for<NG>([&](auto g_) {
      constexpr int G = decltype(g_)::value, kk = G / UB, ub = G % UB;
      if constexpr (next && kk == 2 && ub == 0) {      // hidden tile t+1 must have landed
        wait_vmcnt<frag::handover_wait(UB, NDJ, kLead, R)>();
        block_barrier_no_drain();
      }
      // The group's TB MFMAs with its other instructions spread between them, a few behind
      // each MFMA (bunched at the group's head they take longer to issue than the MFMA before
      // them runs, and the matrix pipe waits):
      //   [wait: fragment G]  MFMA 0  [B reads for the next step]  MFMA 1  [load-to-LDS]
      //   MFMA 2  [re-load fragment G-1 with tile t+kLead's data]  (MFMA 3)
      constexpr bool reads = kk < 3 || next;
      // one wait per pair of groups (every instruction between the MFMAs costs issue time)
      if constexpr (G % 2 == 0) wait_fragment<frag::fragment_pair_wait(UB, NDJ, kLead, R, G)>(a[set][kk][ub]);
      // token blocks in alternating direction: the MFMA that opens a group then keeps the B
      // operand of the one before it (both operands switch at once otherwise); measured 1-2 %
      static_for<TB>([&](auto i_) {
        constexpr int i = decltype(i_)::value, tb = (ub & 1) ? TB - 1 - i : i;
        if constexpr (ub == 0 && i < 2) {
          // this step's B fragments were read during the step before, token block 0's first:
          // MFMA 0 waits for that one (TB-1 younger reads), MFMA 1 for all the others, behind
          // which only this group's reads for the next step (issued after MFMA 0) may remain
          wait_lds_fragment<i == 0 ? TB - 1 : (reads ? reads_in_group(0) : 0)>(b[kk & 1][tb]);
        }
        acc[ub][tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[set][kk][ub], b[kk & 1][tb],
                                                              acc[ub][tb], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (i == 0 && reads) {
          static_for<TB>([&](auto tb_) {
            if constexpr (decltype(tb_)::value * UB / TB == ub) {
              if constexpr (kk < 3) read_b(std::integral_constant<int, kk + 1>{}, tb_, t);
              else read_b(std::integral_constant<int, 0>{}, tb_, t + 1);
            }
          });
          __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (i == 1) {
          if constexpr (more_pd) {
#pragma unroll
            for (int j = 0; j < NDJ; ++j)
              if (frag::dma_group(UB, NDJ, j) == G) dma(j, t + kPD);
          }
          if constexpr (kNorm) {
            // Sum of squares of the tokens' states: wavefront w owns token block w and reads
            // that block's four fragments of the current tile from LDS once more, into
            // registers of its own (the copy among its B fragments sits in a register only a
            // compile-time index reaches), during K steps 0-1; the 16 two-element dot
            // products follow in K steps 2-3.  No branch; all in the MFMA shadow.
            constexpr int kHalf = 2 * UB;                  // groups in half a tile
#pragma unroll
            for (int f = 0; f < 4; ++f) {
              // (the same read as B fragment (step f, token block xblock); hand-issued like those,
              // or the compiler's wait for it would also wait for the B reads just issued.  No
              // wait of its own: it is used two K steps later, behind that step's waits, which
              // leave only reads younger than this one outstanding)
              if (f * kHalf / 4 == G)
                read_fragment<0>(xb[f], b_off[f] + (unsigned)((t % kNS) * STAGE + xblock * 4096));
              if (f * kHalf / 4 == G - kHalf) {
                arrived(xb[f]);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
                  const bf16x2 p = {xb[f][2 * e], xb[f][2 * e + 1]};
                  ssq = __builtin_amdgcn_fdot2_f32_bf16(p, p, ssq, false);
                }
              }
            }
          }
          __builtin_amdgcn_sched_barrier(0);
        }
        // the fragment of the PREVIOUS group: a load issued right behind the MFMAs that still
        // read its destination registers costs extra issue cycles
        if constexpr (i == 2 && more && G > 0) {
          constexpr int pk = (G - 1) / UB, pu = (G - 1) % UB;
          load_fragment<pk * 1024>(a[set][pk][pu], a_voff[pu], a_next);
          __builtin_amdgcn_sched_barrier(0);
        }
      });
    });
    if constexpr (more) {
      load_fragment<3 * 1024>(a[set][3][UB - 1], a_voff[UB - 1], a_next);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // nk >= kPD + 1 (checked by the launcher): all tiles but the last kPD are of the full kind
  {
    using std::integral_constant;
    constexpr integral_constant<int, 0> s0{};
    constexpr integral_constant<int, kLead - 1> s1{};     // the set of the last tile
    int t = 0;
    if constexpr (kLead == 1) {
      for (; t + kPD < nk; ++t) tile_body(t, integral_constant<int, kPD + 1>{}, s0);
    } else {
      // set of tile t = (t + nk) & 1: the last tile always uses set 1, whatever nk
      if (!(nk & 1)) { tile_body(0, integral_constant<int, kPD + 1>{}, s0); t = 1; }
      for (; t + kPD < nk; t += 2) {
        tile_body(t, integral_constant<int, kPD + 1>{}, s1);
        tile_body(t + 1, integral_constant<int, kPD + 1>{}, s0);
      }
    }
    tile_body(nk - 3, integral_constant<int, 3>{}, s1);
    tile_body(nk - 2, integral_constant<int, 2>{}, s0);
    tile_body(nk - 1, integral_constant<int, 1>{}, s1);
  }
  if constexpr (kSplit) {
    // split-K launch: the slice's part of the first projection goes to partial[slice][row][unit]
    // as it is; bias, GELU and the second projection follow in score_finish_kernel
    float* out = partial + ((size_t)blockIdx.y * rows + row0) * U + wid * (32 * UB) + 4 * kg;
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
      const int r = 32 * tb + l32;
      if (r < rows_here) {
#pragma unroll
        for (int ub = 0; ub < UB; ++ub)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            floatx4 v4;
#pragma unroll
            for (int e = 0; e < 4; ++e) v4[e] = acc[ub][tb][4 * q + e];
            *reinterpret_cast<floatx4*>(out + (size_t)r * U + 32 * ub + 8 * q) = v4;
          }
      }
    }
    return;
  }
  if constexpr (kNorm) {
    // each token's sum of squares (both lane halves) goes through LDS to the lanes that hold
    // its accumulators; the barrier below publishes it
    float* sSsq = reinterpret_cast<float*>(sW2 + 16 * U * 2 + TOK * sizeof(float) + U * sizeof(float));  // [TOK]
    const float both = ssq + __shfl_xor(ssq, 32, 64);
    if (kg == 0 && wid < TB) sSsq[32 * wid + l32] = both;
  }
  __syncthreads();      // LDS is reused for the reduction below

  if constexpr (!kSplit) {
    // Warm the L2 for the block that starts on this CU when this one ends: workgroups go to
    // the 8 XCDs round-robin and to a CU as it frees up, so with one block per CU that block is
    // blockIdx.x + (number of CUs), on the same XCD and therefore behind the same L2.  One lane
    // per 128-byte line of its first kPD hidden tiles.  The loaded dwords are never used, only
    // where they leave the lines matters: they go to the ring's last stage, which nothing reads
    // any more (the reduction below uses the first two), as load-to-LDS because an ordinary load
    // would need a register that stays reserved until it returns.
    const long long nrow0 = row0 + (long long)kChipCUs * TOK;
#pragma unroll
    for (int i0 = 0; i0 < kPD * TOK; i0 += 256) {
      const int i = i0 + tid, d = i / TOK, r = i - d * TOK;
      if (i < kPD * TOK && nrow0 + r < rows)
        load_to_lds_b32(hidden + (size_t)(nrow0 + r) * Dh + (size_t)(kt0 + d) * kBK,
                        lds0 + (unsigned)((kNS - 1) * STAGE + wid * 256));
    }
  }

  // ---- epilogue: GELU, then the M -> H projection as a second MFMA (fp16 operands) ----
  // acc[ub][tb][r] is z of unit  ubase + 32*ub + 8*(r/4) + 4*kg + r%4  of token 32*tb + l32.
  // Registers 8s..8s+7 form the B operand of MFMA step s; the matching A operand holds
  // W2[head = l32][the same eight units] (zero for heads >= H).
  const int ubase = wid * (32 * UB);
  // kNorm: the row scale of token 32*tb + l32 (the lane pair l32, l32 + 32 holds the two
  // halves of every K step); z = rstd * acc + b1
  float rs[TB];
  if constexpr (kNorm) {
    const float* sSsq = reinterpret_cast<const float*>(sW2 + 16 * U * 2 + TOK * sizeof(float) + U * sizeof(float));
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
      rs[tb] = 1.0f / sqrtf(sSsq[32 * tb + l32] / (float)Dh + norm.eps);
    }
    if (wid == 0 && kg == 0) {
#pragma unroll
      for (int tb = 0; tb < TB; ++tb)
        if (32 * tb + l32 < rows_here) norm.rstd[row0 + 32 * tb + l32] = rs[tb];
    }
  }
  floatx16 acc2[TB];
#pragma unroll
  for (int tb = 0; tb < TB; ++tb)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc2[tb][e] = 0.0f;
#pragma unroll
  for (int ub = 0; ub < UB; ++ub) {
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      const int u0 = ubase + 32 * ub + 16 * s + 4 * kg;
      u32x4 w2 = {0u, 0u, 0u, 0u};
      if (l32 < 16) {
        const uint2 p0 = *reinterpret_cast<const uint2*>(sW2 + ((size_t)l32 * U + u0) * 2);
        const uint2 p1 = *reinterpret_cast<const uint2*>(sW2 + ((size_t)l32 * U + u0 + 8) * 2);
        w2.x = p0.x; w2.y = p0.y; w2.z = p1.x; w2.w = p1.y;
      }
      float bias[8];
      if constexpr (kNorm) {
        const float* sB1 = reinterpret_cast<const float*>(sW2 + 16 * U * 2 + TOK * sizeof(float));
        const floatx4 lo = *reinterpret_cast<const floatx4*>(sB1 + u0);
        const floatx4 hi = *reinterpret_cast<const floatx4*>(sB1 + u0 + 8);
#pragma unroll
        for (int e = 0; e < 8; ++e) bias[e] = e < 4 ? lo[e] : hi[e - 4];
      }
#pragma unroll
      for (int tb = 0; tb < TB; ++tb) {
        f16x8 g;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          float z = acc[ub][tb][8 * s + e];
          if constexpr (kNorm) z = fmaf(z, rs[tb], bias[e]);
          g[e] = (_Float16)gelu_fused(z);
        }
        acc2[tb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, w2), g,
                                                          acc2[tb], 0, 0, 0);
      }
    }
  }
  float* red = reinterpret_cast<float*>(smem);     // [4][H][TOK]
  // acc2[tb][r] is head 8*(r/4) + 4*kg + r%4 of token 32*tb + l32
#pragma unroll
  for (int tb = 0; tb < TB; ++tb)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      if (8 * q + 8 <= H) {                        // uniform: all eight heads of this group exist
#pragma unroll
        for (int e = 0; e < 4; ++e)
          red[(wid * H + 8 * q + 4 * kg + e) * TOK + 32 * tb + l32] = acc2[tb][4 * q + e];
      } else if (8 * q < H) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int head = 8 * q + 4 * kg + e;
          if (head < H) red[(wid * H + head) * TOK + 32 * tb + l32] = acc2[tb][4 * q + e];
        }
      }
    }
  __syncthreads();
  // sequence and position of the block's first token: one 64-bit division per block, the
  // elements then only step over sequence ends
  const long long b_first = row0 / T;
  const int t_first = (int)(row0 - b_first * T);
  for (int i = tid; i < H * TOK; i += 256) {
    const int head = i / TOK, tok = i % TOK;
    if (tok < rows_here) {
      float s = red[(0 * H + head) * TOK + tok];
      s += red[(1 * H + head) * TOK + tok];
      s += red[(2 * H + head) * TOK + tok];
      s += red[(3 * H + head) * TOK + tok];
      s += sB2[head];
      long long bidx = b_first;
      long long t = (long long)t_first + tok;
      while (t >= T) { t -= T; ++bidx; }
      scores[((size_t)bidx * H + head) * T + t] = s;
    }
  }
  if constexpr (kNorm) {
    if (norm.normed) {
      // the normalised states for the layer's own projections: the row scale is known only
      // now, so the block goes over its rows a second time (x * rstd * gain, rounded to bf16)
      float* sR = reinterpret_cast<float*>(sW2 + 16 * U * 2);     // [TOK]
      if (wid == 0 && kg == 0) {
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) sR[32 * tb + l32] = rs[tb];
      }
      __syncthreads();
      const int ppr = Dh / 8;                                      // 16-byte pieces per row
      const u32x4* xin = reinterpret_cast<const u32x4*>(hidden + (size_t)row0 * Dh);
      u32x4* yout = reinterpret_cast<u32x4*>(norm.normed + (size_t)row0 * Dh);
      const u32x4* gain8 = reinterpret_cast<const u32x4*>(norm.gain);
      const int total = rows_here * ppr;
      // only this block's 256 threads are on the CU: eight 16-byte pieces in flight per thread
      constexpr int kFly = 8;
      for (int p0 = tid; p0 < total; p0 += 256 * kFly) {
        u32x4 x[kFly];
#pragma unroll
        for (int u = 0; u < kFly; ++u) {
          const int p = p0 + 256 * u;
          if (p < total) x[u] = __builtin_nontemporal_load(xin + p);
        }
#pragma unroll
        for (int u = 0; u < kFly; ++u) {
          const int p = p0 + 256 * u;
          if (p < total) {
            const int r = p / ppr, c = p - r * ppr;
            const u32x4 g = gain8[c];
            const float sc = sR[r];
            u32x4 y;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const float lo = __uint_as_float(x[u][e] << 16) * sc * __uint_as_float(g[e] << 16);
              const float hi = __uint_as_float(x[u][e] & 0xffff0000u) * sc * __uint_as_float(g[e] & 0xffff0000u);
              typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
              const bf16x2 pr = {(__bf16)lo, (__bf16)hi};
              y[e] = __builtin_bit_cast(unsigned int, pr);
            }
            __builtin_nontemporal_store(y, yout + p);
          }
        }
      }
    }
  }
}

// ---- short prompts ----
// One block of the kernels above walks all of K for its tokens, which takes 50-85 us however
// few blocks there are.  Two remedies, both with the first projection's partial sums in the
// workspace and this kernel to finish (K-slices in a fixed order, bias, GELU, second
// projection in fp32; one wavefront per token, 8 hidden units per lane and round):
//  * while the token blocks do not fill the chip, the main kernel is cut over K as well
//    (frag_ksplit): 37-50 us from 640 to 4096 tokens, 68 us at 8192, against 85-88 us;
//  * up to kTwoStageRows tokens the decode path's skinny GEMM over (unit block x K-slice x
//    64 tokens) blocks is faster still (128 tokens 20 us, 256: 26 us); it reads its operands
//    from global memory in 32-byte pieces and re-reads W1 per 64 tokens, so it loses beyond
//    a few hundred tokens (512: 38 us, 1024: 49 us, 4096: 120 us).
constexpr long long kTwoStageRows = 384;
constexpr int kTwoStageBlocks = 2048;

__global__ __launch_bounds__(256) void score_finish_kernel(
    const float* __restrict__ partial, const unsigned short* __restrict__ b1,
    const unsigned short* __restrict__ W2, const unsigned short* __restrict__ b2,
    float* __restrict__ scores, long long rows, int T, int M, int H, int ks) {
  const int lane = threadIdx.x & 63;
  const long long row = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;                                  // uniform per wavefront; no barrier below
  float acc[16];
#pragma unroll
  for (int h = 0; h < 16; ++h) acc[h] = 0.f;
  for (int u0 = lane * 8; u0 < M; u0 += 512) {
    floatx4 z0 = {0.f, 0.f, 0.f, 0.f}, z1 = {0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < ks; ++s) {
      const float* p = partial + ((size_t)s * rows + row) * M + u0;
      z0 += *reinterpret_cast<const floatx4*>(p);
      z1 += *reinterpret_cast<const floatx4*>(p + 4);
    }
    u32x4 bb = {0u, 0u, 0u, 0u};
    if (b1) bb = *reinterpret_cast<const u32x4*>(b1 + u0);
    float g[8];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      g[2 * e] = gelu_exact((e < 2 ? z0[2 * e] : z1[2 * e - 4]) + __uint_as_float(bb[e] << 16));
      g[2 * e + 1] = gelu_exact((e < 2 ? z0[2 * e + 1] : z1[2 * e - 3]) + __uint_as_float(bb[e] & 0xffff0000u));
    }
#pragma unroll
    for (int h = 0; h < 16; ++h) {
      if (h < H) {
        const u32x4 w = *reinterpret_cast<const u32x4*>(W2 + (size_t)h * M + u0);
#pragma unroll
        for (int e = 0; e < 4; ++e)
          acc[h] += g[2 * e] * __uint_as_float(w[e] << 16) + g[2 * e + 1] * __uint_as_float(w[e] & 0xffff0000u);
      }
    }
  }
  const long long bidx = row / T;
  const int t = (int)(row - bidx * T);
#pragma unroll
  for (int h = 0; h < 16; ++h) {
    if (h < H) {
      float v = acc[h];
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
      if (lane == 0) scores[((size_t)bidx * H + h) * T + t] = v + (b2 ? bf16_bits_to_float(b2[h]) : 0.f);
    }
  }
}

// K-slices for a launch of `blocks` token blocks over nk_total K tiles: enough blocks for the
// chip's 256 CUs, slices of at least kPD + 1 tiles that divide K evenly, at most 8.
inline int frag_ksplit(long long blocks, int nk_total) {
  int ks = 1;
  for (int d = 2; d <= 8; ++d)
    if (nk_total % d == 0 && nk_total / d >= kPD + 1 && blocks * d <= 256 && blocks <= 112) ks = d;
  return ks;
}

template <int UB, int TB>
int launch_frag(const void* hidden, const void* W1, const void* b1, const void* W2,
                const void* b2, float* scores, long long rows, int T, int Dh, int H,
                void* workspace, hipStream_t stream, const NormArgs* norm) {
  constexpr int TOK = 32 * TB;
  constexpr size_t ring = (size_t)kNS * TOK * 128;
  static_assert(ring >= (size_t)4 * 16 * TOK * sizeof(float), "reduction buffer fits");
  // + W2 as [16][M] fp16, then (normalising form) the row scales, b1 and the sums of squares as fp32
  constexpr size_t lds = ring + (size_t)16 * (128 * UB) * 2 + TOK * sizeof(float) +
                         (128 * UB) * sizeof(float) + TOK * sizeof(float) + 16 * sizeof(float);   // + b2
  // once per process, which drives one GPU (thread-safe: a function-local static)
  static const hipError_t attr_rc =
      hipFuncSetAttribute(reinterpret_cast<const void*>(score_mlp_frag_kernel<UB, TB, false>),
      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  static const hipError_t attr_rc_split =
      hipFuncSetAttribute(reinterpret_cast<const void*>(score_mlp_frag_kernel<UB, TB, true>),
      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  static const hipError_t attr_rc_norm =
      hipFuncSetAttribute(reinterpret_cast<const void*>(score_mlp_frag_kernel<UB, TB, false, true>),
      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (attr_rc != hipSuccess || attr_rc_split != hipSuccess || attr_rc_norm != hipSuccess)
    return KVZAP_ERR_RUNTIME;
  const int M = 128 * UB;
  if (norm) {     // residual stream in, W1 already prepared with the gain folded in
    score_mlp_frag_kernel<UB, TB, false, true><<<dim3((unsigned)((rows + TOK - 1) / TOK)), 256, lds, stream>>>(
        static_cast<const unsigned short*>(hidden), static_cast<const unsigned char*>(W1),
        static_cast<const unsigned short*>(b1), static_cast<const unsigned short*>(W2),
        static_cast<const unsigned short*>(b2), scores, rows, T, Dh, H, Dh / kBK, nullptr, *norm);
    return hipGetLastError() == hipSuccess ? KVZAP_OK : KVZAP_ERR_RUNTIME;
  }
  // workspace == nullptr: W1 already is the fragment-ordered copy (launch_prepare_w1)
  if (workspace)
    arrange_w1_kernel<<<512, 256, 0, stream>>>(static_cast<const u32x4*>(W1),
                                               static_cast<u32x4*>(workspace), M, Dh, nullptr);
  const void* w1f = workspace ? workspace : W1;
  const long long blocks = (rows + TOK - 1) / TOK;
  // Few blocks (mid-length prompts): a block needs 50-85 us for all of K whatever the grid,
  // so K is cut over blockIdx.y and the epilogue moves to score_finish_kernel; the partial
  // sums live behind the fragment copy in the workspace (only with a workspace).
  const int ks = workspace ? frag_ksplit(blocks, Dh / kBK) : 1;
  float* partial = ks > 1 ? reinterpret_cast<float*>(static_cast<char*>(workspace) +
                                                     align_up((size_t)M * Dh * 2, 256))
                          : nullptr;
  if (ks > 1)
    score_mlp_frag_kernel<UB, TB, true><<<dim3((unsigned)blocks, ks), 256, lds, stream>>>(
        static_cast<const unsigned short*>(hidden), static_cast<const unsigned char*>(w1f),
        static_cast<const unsigned short*>(b1), static_cast<const unsigned short*>(W2),
        static_cast<const unsigned short*>(b2), scores, rows, T, Dh, H, Dh / kBK / ks, partial, NormArgs{});
  else
    score_mlp_frag_kernel<UB, TB, false><<<dim3((unsigned)blocks), 256, lds, stream>>>(
        static_cast<const unsigned short*>(hidden), static_cast<const unsigned char*>(w1f),
        static_cast<const unsigned short*>(b1), static_cast<const unsigned short*>(W2),
        static_cast<const unsigned short*>(b2), scores, rows, T, Dh, H, Dh / kBK, nullptr, NormArgs{});
  if (hipGetLastError() != hipSuccess) return KVZAP_ERR_RUNTIME;
  if (ks > 1)
    score_finish_kernel<<<dim3((unsigned)((rows + 3) / 4)), 256, 0, stream>>>(
        partial, static_cast<const unsigned short*>(b1), static_cast<const unsigned short*>(W2),
        static_cast<const unsigned short*>(b2), scores, rows, T, M, H, ks);
  return hipGetLastError() == hipSuccess ? KVZAP_OK : KVZAP_ERR_RUNTIME;
}

template <int UB>
int launch_one(const void* hidden, const void* W1, const void* b1, const void* W2,
               const void* b2, float* scores, long long rows, int T, int Dh, int H,
               hipStream_t stream) {
  constexpr size_t lds = (size_t)(128 * UB + kTok) * 128;
  // once per process, which drives one GPU (thread-safe: a function-local static)
  static const hipError_t attr_rc =
      hipFuncSetAttribute(reinterpret_cast<const void*>(score_mlp_kernel<UB>),
      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (attr_rc != hipSuccess) return KVZAP_ERR_RUNTIME;
  const long long blocks = (rows + kTok - 1) / kTok;
  score_mlp_kernel<UB><<<dim3((unsigned)blocks), kThreads, lds, stream>>>(
      static_cast<const unsigned short*>(hidden), static_cast<const unsigned short*>(W1),
      static_cast<const unsigned short*>(b1), static_cast<const unsigned short*>(W2),
      static_cast<const unsigned short*>(b2), scores, rows, T, Dh, H);
  return hipGetLastError() == hipSuccess ? KVZAP_OK : KVZAP_ERR_RUNTIME;
}

__global__ __launch_bounds__(256) void copy_w1_kernel(const u32x4* __restrict__ W1,
                                                      u32x4* __restrict__ out, int n) {
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x)
    out[i] = W1[i];
}

}  // namespace

// The form of W1 that launch_score_mlp takes with workspace == nullptr: fragment order for
// the main kernel, a plain copy for the small-D_h kernel.
int launch_prepare_w1(const void* W1, const void* gain, int Dh, int M, void* out, hipStream_t stream) {
  const bool frag = (Dh / kBK) >= kPD + 1;
  if (gain && !frag) return KVZAP_ERR_UNSUPPORTED;
  if (frag)
    arrange_w1_kernel<<<512, 256, 0, stream>>>(static_cast<const u32x4*>(W1),
                                               static_cast<u32x4*>(out), M, Dh,
                                               static_cast<const u32x4*>(gain));
  else
    copy_w1_kernel<<<64, 256, 0, stream>>>(static_cast<const u32x4*>(W1),
                                           static_cast<u32x4*>(out), M * (Dh / 8));
  return hipGetLastError() == hipSuccess ? KVZAP_OK : KVZAP_ERR_RUNTIME;
}

size_t score_mlp_workspace_bytes(long long rows, int Dh, int M) {
  size_t need = align_up((size_t)M * Dh * 2, 256);                 // W1 in fragment order
  if (rows > 0 && rows <= kTwoStageRows) {
    const size_t part = align_up((size_t)skinny_ksplit(rows, Dh, M, kTwoStageBlocks) * rows * M * sizeof(float), 256);
    need = need > part ? need : part;
  } else if (rows > 0 && (Dh / kBK) >= kPD + 1) {
    // mid-length prompts: the main kernel split over K, partial sums behind the fragment copy
    const int tok = 32 * (M / 128 <= 4 ? 4 : 3);
    const int ks = frag_ksplit((rows + tok - 1) / tok, Dh / kBK);
    if (ks > 1) need += align_up((size_t)ks * rows * M * sizeof(float), 256);
  }
  return need;
}

bool score_rmsnorm_supports(int Dh) { return (Dh / kBK) >= kPD + 1; }

int launch_score_mlp_rmsnorm(const void* x, const void* W1_prepared, const void* gain, float eps,
                             const void* b1, const void* W2, const void* b2, float* scores,
                             float* rstd, void* normed, int B, int T, int Dh, int M, int H,
                             hipStream_t stream) {
  const long long rows = (long long)B * T;
  const NormArgs norm{static_cast<const unsigned short*>(gain), eps, rstd,
                      static_cast<unsigned short*>(normed)};
  switch (M / 128) {
    case 1: return launch_frag<1, 4>(x, W1_prepared, b1, W2, b2, scores, rows, T, Dh, H, nullptr, stream, &norm);
    case 2: return launch_frag<2, 4>(x, W1_prepared, b1, W2, b2, scores, rows, T, Dh, H, nullptr, stream, &norm);
    case 3: return launch_frag<3, 4>(x, W1_prepared, b1, W2, b2, scores, rows, T, Dh, H, nullptr, stream, &norm);
    case 4: return launch_frag<4, 4>(x, W1_prepared, b1, W2, b2, scores, rows, T, Dh, H, nullptr, stream, &norm);
    case 5: return launch_frag<5, 3>(x, W1_prepared, b1, W2, b2, scores, rows, T, Dh, H, nullptr, stream, &norm);
    default: return KVZAP_ERR_UNSUPPORTED;
  }
}

int launch_score_mlp(const void* hidden, const void* W1, const void* b1, const void* W2,
                     const void* b2, float* scores, int B, int T, int Dh, int M, int H,
                     void* workspace, hipStream_t stream) {
  const long long rows = (long long)B * T;
  if (workspace && rows <= kTwoStageRows) {        // short prompt and the original W1 at hand
    const int ks = skinny_ksplit(rows, Dh, M, kTwoStageBlocks);
    const int rc = launch_skinny_gemm(hidden, W1, static_cast<float*>(workspace), rows, Dh, M, ks, stream);
    if (rc != KVZAP_OK) return rc;
    score_finish_kernel<<<dim3((unsigned)((rows + 3) / 4)), 256, 0, stream>>>(
        static_cast<const float*>(workspace), static_cast<const unsigned short*>(b1),
        static_cast<const unsigned short*>(W2), static_cast<const unsigned short*>(b2), scores,
        rows, T, M, H, ks);
    return hipGetLastError() == hipSuccess ? KVZAP_OK : KVZAP_ERR_RUNTIME;
  }
  const bool frag = (Dh / kBK) >= kPD + 1;     // the main variant needs at least kPD+1 K tiles
#define KVZAP_MLP_CASE(UBV)                                                                     \
  case UBV:                                                                                     \
    return frag ? launch_frag<UBV, (UBV <= 4 ? 4 : 3)>(hidden, W1, b1, W2, b2, scores, rows, T, \
                                                       Dh, H, workspace, stream, nullptr)       \
                : launch_one<UBV>(hidden, W1, b1, W2, b2, scores, rows, T, Dh, H, stream);
  switch (M / 128) {
    KVZAP_MLP_CASE(1)
    KVZAP_MLP_CASE(2)
    KVZAP_MLP_CASE(3)
    KVZAP_MLP_CASE(4)
    KVZAP_MLP_CASE(5)   // M = 640: 96-token blocks so that the 5 x 3 accumulator blocks fit (240 registers)
    default: return KVZAP_ERR_UNSUPPORTED;
  }
#undef KVZAP_MLP_CASE
}

}  // namespace kvzap
