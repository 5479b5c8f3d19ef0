// The scores the surrogate is trained on (Sec. 3.1 Eq. 1: KVzip; Sec. 3.2 Eq. 3: KVzip+):
// on an extended prompt "prompt, instruction, repeated prompt", the score of prompt position
// i in KV head h is the largest attention weight a_ji any repeated-prompt query j of the
// head's group puts on it, weighted by ||W_O v_i|| / ||h_j||.  Computed in log space:
//
//   log2 s_i = max_{g,j} [ c * q_gj . k_i  -  (m_gj + log2 l_gj + log2 ||h_j||) ] + log2 ||W_O v_i||
//
// with (m, l) the row maximum and the sum of exp2 of row j's causal softmax (c = scale*log2 e).
// The maximum over j commutes with exp2, so the column pass needs no exponential at all:
//
//   pass 1 (teacher_rowstat_kernel)  per query row: m, l over all visible keys -> one bias
//   pass 2 (teacher_colmax_kernel)   per prompt key: max over queries of (logit + bias)
//   pass 3 (teacher_finish_kernel)   max over the query splits, + log ||W_O v||, natural log
//
// Both passes are Q K^T on v_mfma_f32_32x32x16_bf16 with the *reduced* index on the MFMA
// row side (C rows live in a lane's 16 registers) and the kept index on the column side
// (one lane = one query in pass 1, one key in pass 2), so the reductions are per-lane.
// The operand that stays (128 rows of Q, resp. K) sits in registers; the other one streams
// straight from global memory in operand layout (16 bytes of one row per lane and k-step),
// one tile ahead.
#include "kvzap_internal.h"

namespace kvzap {
namespace {

constexpr int kD = 128;
constexpr int kRowVec = kD * 2 / 16;       // 16-byte pieces per row
constexpr int kSteps = kD / 16;            // MFMA k-steps per tile
constexpr int kStay = 4;                   // 32-row tiles of the operand kept in registers
constexpr float kNegBig = -1.0e30f;        // "minus infinity" that survives subtraction
constexpr float kLazyMargin = 16.0f;

struct Tile {
  u32x4 f[kSteps];
};

// rows [row0, row0+32) of a row-major [rows][128] bf16 matrix as an MFMA operand: lane
// (r = lane%32, kg = lane/32) holds elements 16s + 8kg .. +8 of row row0 + r for k-step s.
// Rows past `last` are read from row `last` (the caller masks them).
__device__ __forceinline__ void load_tile(Tile& t, const u32x4* base, int row0, int last, int lane) {
  int row = row0 + (lane & 31);
  row = row < last ? row : last;
  const u32x4* p = base + (size_t)row * kRowVec + (lane >> 5);
#pragma unroll
  for (int s = 0; s < kSteps; ++s) t.f[s] = p[2 * s];
}

__device__ __forceinline__ floatx16 tile_product(const Tile& a, const Tile& b) {
  floatx16 c;
#pragma unroll
  for (int e = 0; e < 16; ++e) c[e] = 0.f;
#pragma unroll
  for (int s = 0; s < kSteps; ++s)
    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a.f[s]),
                                                __builtin_bit_cast(bf16x8, b.f[s]), c, 0, 0, 0);
  return c;
}

// row of C register e in lane half kg: 8*(e/4) + 4*kg + e%4
__device__ __forceinline__ int c_row(int e, int kg) { return 8 * (e >> 2) + 4 * kg + (e & 3); }

// ---- pass 1: grid (ceil(Tq / (4*128)), HQ), 256 threads; a wavefront owns 128 queries ----
__global__ __launch_bounds__(256) void teacher_rowstat_kernel(
    const u32x4* __restrict__ q, const u32x4* __restrict__ k, const float* __restrict__ hnorm,
    int G, int Tq, int Tk, int tq_pad, float cscale, float* __restrict__ rowbias) {
  const int g = blockIdx.y, h = g / G;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane & 31, kg = lane >> 5;
  const int q0 = (blockIdx.x * 4 + wave) * (kStay * 32);
  if (q0 >= tq_pad) return;
  const int P0 = Tk - Tq;
  const u32x4* qh = q + (size_t)g * Tq * kRowVec;
  const u32x4* kh = k + (size_t)h * Tk * kRowVec;

  Tile qt[kStay];                                        // B operands: the wavefront's queries
#pragma unroll
  for (int t = 0; t < kStay; ++t) load_tile(qt[t], qh, q0 + 32 * t, Tq - 1, lane);
  float m[kStay], l[kStay];
#pragma unroll
  for (int t = 0; t < kStay; ++t) { m[t] = kNegBig; l[t] = 0.f; }

  // keys visible to the wavefront's last query
  int last_q = q0 + kStay * 32 - 1;
  last_q = last_q < Tq - 1 ? last_q : Tq - 1;
  const int ntiles = (P0 + last_q) / 32 + 1;

  auto consume = [&](const Tile& kt, int tile) {
    const int key0 = tile * 32;
#pragma unroll
    for (int t = 0; t < kStay; ++t) {
      const int qcol = q0 + 32 * t + r;                  // this lane's query
      if (key0 > P0 + q0 + 32 * t + 31) continue;        // nothing of this tile is visible (uniform)
      const floatx16 s = tile_product(kt, qt[t]);
      float x[16];
#pragma unroll
      for (int e = 0; e < 16; ++e) x[e] = s[e] * cscale;
      if (key0 + 31 > P0 + q0 + 32 * t) {                // the diagonal crosses this tile (uniform)
#pragma unroll
        for (int e = 0; e < 16; ++e)
          if (key0 + c_row(e, kg) > P0 + qcol) x[e] = -INFINITY;
      }
      float mx = x[0];
#pragma unroll
      for (int e = 1; e < 16; ++e) mx = fmaxf(mx, x[e]);
      if (__any(mx > m[t] + kLazyMargin)) {              // per-lane statistics: no cross-lane step
        const float mn = fmaxf(m[t], mx);
        l[t] *= __builtin_amdgcn_exp2f(m[t] - mn);
        m[t] = mn;
      }
      float sum = 0.f;
#pragma unroll
      for (int e = 0; e < 16; ++e) sum += __builtin_amdgcn_exp2f(x[e] - m[t]);
      l[t] += sum;
    }
  };

  Tile ka, kb;
  load_tile(ka, kh, 0, Tk - 1, lane);
  int tile = 0;
  while (tile + 2 < ntiles) {
    load_tile(kb, kh, (tile + 1) * 32, Tk - 1, lane);
    consume(ka, tile);
    load_tile(ka, kh, (tile + 2) * 32, Tk - 1, lane);
    consume(kb, tile + 1);
    tile += 2;
  }
  if (tile + 1 < ntiles) {
    load_tile(kb, kh, (tile + 1) * 32, Tk - 1, lane);
    consume(ka, tile);
    consume(kb, tile + 1);
  } else {
    consume(ka, tile);
  }

  // the two lane halves hold disjoint key rows of the same query: merge, then one bias per row
#pragma unroll
  for (int t = 0; t < kStay; ++t) {
    const float mo = __shfl_xor(m[t], 32, 64), lo = __shfl_xor(l[t], 32, 64);
    const float M = fmaxf(m[t], mo);
    const float L = l[t] * __builtin_amdgcn_exp2f(m[t] - M) + lo * __builtin_amdgcn_exp2f(mo - M);
    const int j = q0 + 32 * t + r;
    if (kg == 0 && j < tq_pad) {
      float bias = -INFINITY;                            // padded rows never win a maximum
      if (j < Tq) bias = -(M + __log2f(L) + (hnorm ? __log2f(hnorm[j]) : 0.f));
      rowbias[(size_t)g * tq_pad + j] = bias;
    }
  }
}

// ---- pass 2: grid (ceil(T / 128), H, JS), 64 threads; a wavefront owns 128 prompt keys ----
__global__ __launch_bounds__(64) void teacher_colmax_kernel(
    const u32x4* __restrict__ q, const u32x4* __restrict__ k, const float* __restrict__ rowbias,
    int G, int Tq, int Tk, int T, int tq_pad, float cscale, float* __restrict__ part) {
  const int h = blockIdx.y, js = blockIdx.z, JS = gridDim.z, H = gridDim.y;
  const int lane = threadIdx.x, r = lane & 31, kg = lane >> 5;
  const int k0 = blockIdx.x * (kStay * 32);
  const u32x4* kh = k + (size_t)h * Tk * kRowVec;

  Tile kt[kStay];                                        // B operands: the wavefront's keys
#pragma unroll
  for (int t = 0; t < kStay; ++t) load_tile(kt[t], kh, k0 + 32 * t, T - 1, lane);
  float cm[kStay];
#pragma unroll
  for (int t = 0; t < kStay; ++t) cm[t] = -INFINITY;

  // the G * (tq_pad / 32) query tiles of the group, split evenly over the JS blocks
  const int ntq = tq_pad / 32, total = G * ntq;
  const int first = (int)((long long)total * js / JS), end = (int)((long long)total * (js + 1) / JS);
  // (a split with no item leaves -inf partials)

  auto fetch = [&](Tile& qt, floatx4 (&bias)[4], int item) {
    const int g = h * G + item / ntq, j0 = (item % ntq) * 32;
    load_tile(qt, q + (size_t)g * Tq * kRowVec, j0, Tq - 1, lane);
    const float* rb = rowbias + (size_t)g * tq_pad + j0 + 4 * kg;
#pragma unroll
    for (int a = 0; a < 4; ++a) bias[a] = *reinterpret_cast<const floatx4*>(rb + 8 * a);
  };
  auto consume = [&](const Tile& qt, const floatx4 (&bias)[4]) {
#pragma unroll
    for (int t = 0; t < kStay; ++t) {
      const floatx16 s = tile_product(qt, kt[t]);
      float best = cm[t];
#pragma unroll
      for (int e = 0; e < 16; ++e) best = fmaxf(best, fmaf(s[e], cscale, bias[e >> 2][e & 3]));
      cm[t] = best;
    }
  };

  if (first < end) {
    Tile qa, qb;
    floatx4 ba[4], bb[4];
    fetch(qa, ba, first);
    int item = first;
    while (item + 2 < end) {
      fetch(qb, bb, item + 1);
      consume(qa, ba);
      fetch(qa, ba, item + 2);
      consume(qb, bb);
      item += 2;
    }
    if (item + 1 < end) {
      fetch(qb, bb, item + 1);
      consume(qa, ba);
      consume(qb, bb);
    } else {
      consume(qa, ba);
    }
  }
#pragma unroll
  for (int t = 0; t < kStay; ++t) {
    const float other = __shfl_xor(cm[t], 32, 64);
    const int key = k0 + 32 * t + r;
    if (kg == 0 && key < T) part[((size_t)js * H + h) * T + key] = fmaxf(cm[t], other);
  }
}

// ---- pass 3: max over the splits, weight of the value, natural log ----
__global__ __launch_bounds__(256) void teacher_finish_kernel(const float* __restrict__ part,
                                                            const float* __restrict__ vnorm,
                                                            int n, int JS, float* __restrict__ out) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  float best = -INFINITY;
  for (int s = 0; s < JS; ++s) best = fmaxf(best, part[(size_t)s * n + i]);
  out[i] = best * 0.69314718055994531f + (vnorm ? __logf(vnorm[i]) : 0.f);
}

}  // namespace

int teacher_splits(int H, int G, int Tq, int T) {
  const int tq_pad = (Tq + 31) / 32 * 32;
  const long long col_blocks = (long long)((T + kStay * 32 - 1) / (kStay * 32)) * H;
  long long js = col_blocks > 0 ? (2048 + col_blocks - 1) / col_blocks : 1;
  const long long items = (long long)G * (tq_pad / 32);
  if (js > items) js = items;
  if (js > 256) js = 256;
  return js < 1 ? 1 : (int)js;
}

size_t teacher_workspace_bytes(int H, int HQ, int Tq, int T) {
  const int tq_pad = (Tq + 31) / 32 * 32;
  const int js = teacher_splits(H, HQ / H, Tq, T);
  return align_up((size_t)HQ * tq_pad * sizeof(float), 256) +
         align_up((size_t)js * H * (T > 0 ? T : 1) * sizeof(float), 256);
}

int launch_teacher_scores(const void* q, const void* k, const float* vnorm, const float* hnorm,
                          float scale, float* log_s, int H, int HQ, int Tq, int Tk, int T,
                          void* workspace, hipStream_t stream) {
  if (T == 0) return KVZAP_OK;
  const int G = HQ / H;
  const int tq_pad = (Tq + 31) / 32 * 32;
  const int JS = teacher_splits(H, G, Tq, T);
  float* rowbias = static_cast<float*>(workspace);
  float* part = reinterpret_cast<float*>(static_cast<char*>(workspace) +
                                         align_up((size_t)HQ * tq_pad * sizeof(float), 256));
  const float cscale = scale * 1.4426950408889634f;
  const auto* qv = static_cast<const u32x4*>(q);
  const auto* kv = static_cast<const u32x4*>(k);
  const dim3 g1((tq_pad + 4 * kStay * 32 - 1) / (4 * kStay * 32), HQ);
  teacher_rowstat_kernel<<<g1, 256, 0, stream>>>(qv, kv, hnorm, G, Tq, Tk, tq_pad, cscale, rowbias);
  if (hipGetLastError() != hipSuccess) return KVZAP_ERR_RUNTIME;
  const dim3 g2((T + kStay * 32 - 1) / (kStay * 32), H, JS);
  teacher_colmax_kernel<<<g2, 64, 0, stream>>>(qv, kv, rowbias, G, Tq, Tk, T, tq_pad, cscale, part);
  if (hipGetLastError() != hipSuccess) return KVZAP_ERR_RUNTIME;
  const int n = H * T;
  teacher_finish_kernel<<<(n + 255) / 256, 256, 0, stream>>>(part, vnorm, n, JS, log_s);
  return hipGetLastError() == hipSuccess ? KVZAP_OK : KVZAP_ERR_RUNTIME;
}

}  // namespace kvzap
