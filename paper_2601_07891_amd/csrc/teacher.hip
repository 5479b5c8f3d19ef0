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
constexpr int kStay = 4;                   // 32-row tiles of the operand kept in registers (column pass)
constexpr int kStayRow = 2;                // row pass: it is bound by the exponentials, not by operand reuse,
                                           // and two tiles leave room for two wavefronts per SIMD
constexpr float kNegBig = -1.0e30f;        // "minus infinity" that survives subtraction
constexpr float kLazyLimit = 1048576.0f;    // 2^20: a tile's 16 terms may sum to this before the reference moves

// The streamed operand goes through an LDS ring filled by load-to-LDS kAhead tiles ahead, so
// that the four wavefronts of a block share one copy, the global reads are whole 256-byte
// rows, and the prefetch depth costs no registers.
constexpr int kAhead = 3;
constexpr int kStages = kAhead + 1;
constexpr int kTileBytes = 32 * kD * 2;                  // 8 KB: 32 rows
constexpr int kBiasBytes = 4 * 256;                      // pass 2: one 256-byte slot per wavefront
constexpr int kStageBytes = kTileBytes + kBiasBytes;

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

// One wavefront's share of a 32-row tile on its way to LDS: two load-to-LDS instructions,
// each 4 whole rows (lane i: row i/16 of the four, physical piece i%16).  The 16-byte pieces
// of a row are XOR-swizzled with the row number so that the operand reads below spread over
// the banks.  Rows past `last` re-read row `last`.
__device__ __forceinline__ void stream_tile_to_lds(const u32x4* base, int row0, int last,
                                                   unsigned stage_lds, int wave, int lane) {
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int chunk = 2 * wave + j;                      // 4 rows each
    const int row_in_tile = 4 * chunk + (lane >> 4);
    int row = row0 + row_in_tile;
    row = row < last ? row : last;
    const int piece = (lane & 15) ^ (row_in_tile & 15);
    load_to_lds_b128(base + (size_t)row * kRowVec + piece, stage_lds + chunk * 1024);
  }
}

// The tile as an MFMA operand, from LDS (same register layout as load_tile).
__device__ __forceinline__ void read_tile_from_lds(Tile& t, const unsigned char* stage, int lane) {
  const int r = lane & 31, kg = lane >> 5;
#pragma unroll
  for (int s = 0; s < kSteps; ++s)
    t.f[s] = *reinterpret_cast<const u32x4*>(stage + r * 256 + (((2 * s + kg) ^ (r & 15)) << 4));
}

// The kStay products of one streamed tile with the tiles that stay, as kStay independent
// MFMA chains issued round-robin (a single chain on one accumulator would wait for each
// result before the next step).  The streamed tile is the A (row) operand.
template <bool kZeroInit, int KS>
__device__ __forceinline__ void tile_products(const Tile& stream, const Tile (&stay)[KS],
                                              const floatx16& init, floatx16 (&c)[KS]) {
#pragma unroll
  for (int t = 0; t < KS; ++t) {
    if (kZeroInit) {                                     // a literal zero is an MFMA immediate: no moves
#pragma unroll
      for (int e = 0; e < 16; ++e) c[t][e] = 0.f;
    } else {
      c[t] = init;
    }
  }
#pragma unroll
  for (int s = 0; s < kSteps; ++s)
#pragma unroll
    for (int t = 0; t < KS; ++t)
      c[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, stream.f[s]),
                                                     __builtin_bit_cast(bf16x8, stay[t].f[s]),
                                                     c[t], 0, 0, 0);
}

// row of C register e in lane half kg: 8*(e/4) + 4*kg + e%4
__device__ __forceinline__ int c_row(int e, int kg) { return 8 * (e >> 2) + 4 * kg + (e & 3); }

// ---- pass 1: grid (ceil(Tq / 256), HQ), 256 threads; a wavefront owns 64 queries, the
// block streams the keys its last query sees ----
__global__ __launch_bounds__(256, 2) void teacher_rowstat_kernel(
    const u32x4* q, const u32x4* k, const float* __restrict__ hnorm, int G, int Tq, int Tk,
    int tq_pad, float cscale, float* __restrict__ rowbias) {
  extern __shared__ __align__(16) unsigned char smem[];
  // Blocks are handed out in the order of the linear block index, and a block of late
  // queries sees up to twice the keys of an early one: the index is mapped so that the
  // longest blocks of all heads start first and the shortest fill the tail.
  const int lin = blockIdx.y * gridDim.x + blockIdx.x;
  const int bx = gridDim.x - 1 - lin / gridDim.y;
  const int g = lin % gridDim.y, h = g / G;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int r = lane & 31, kg = lane >> 5;
  const int q0 = (bx * 4 + wave) * (kStayRow * 32);
  const int P0 = Tk - Tq;
  const u32x4* qh = q + (size_t)g * Tq * kRowVec;
  const u32x4* kh = k + (size_t)h * Tk * kRowVec;
  const unsigned lds0 = lds_address(smem);

  // every wavefront walks all the key tiles of the block (barriers), also one whose queries
  // are all padding
  int block_last_q = bx * 4 * (kStayRow * 32) + 4 * kStayRow * 32 - 1;
  block_last_q = block_last_q < Tq - 1 ? block_last_q : Tq - 1;
  const int ntiles = (P0 + block_last_q) / 32 + 1;

  auto stream = [&](int tile) {                          // clamped: a tile past the end re-reads the last
    const int tl = tile < ntiles ? tile : ntiles - 1;
    stream_tile_to_lds(kh, tl * 32, Tk - 1, lds0 + (unsigned)((tile % kStages) * kStageBytes), wave, lane);
  };
#pragma unroll
  for (int d = 0; d < kStages; ++d) stream(d);            // all stages: tiles 0 .. kAhead

  Tile qt[kStayRow];                                        // B operands: the wavefront's queries
#pragma unroll
  for (int t = 0; t < kStayRow; ++t) load_tile(qt[t], qh, q0 + 32 * t, Tq - 1, lane);
  float m[kStayRow], l[kStayRow];
#pragma unroll
  for (int t = 0; t < kStayRow; ++t) { m[t] = kNegBig; l[t] = 0.f; }
  floatx16 zero;
#pragma unroll
  for (int e = 0; e < 16; ++e) zero[e] = 0.f;

  // softmax statistics of one key tile from its logits s (C[key][query])
  auto reduce = [&](floatx16 (&s)[kStayRow], int tile) {
    const int key0 = tile * 32;
#pragma unroll
    for (int t = 0; t < kStayRow; ++t) {
      const int qcol = q0 + 32 * t + r;                  // this lane's query
      if (key0 > P0 + q0 + 32 * t + 31) continue;        // nothing of this tile is visible (uniform)
      float x[16];
#pragma unroll
      for (int e = 0; e < 16; ++e) x[e] = s[t][e];
      if (key0 + 31 > P0 + q0 + 32 * t) {                // the diagonal crosses this tile (uniform)
#pragma unroll
        for (int e = 0; e < 16; ++e)
          if (key0 + c_row(e, kg) > P0 + qcol) x[e] = -INFINITY;
      }
      // The reference m is lazy: the tile is summed against the current one, and only if
      // some lane's sum leaves the safe range (an element more than kLazyLimit above the
      // reference, an overflow to infinity, the first tile) is the tile's maximum taken and
      // the tile summed again.  That keeps the 16 maximum operations out of the common path
      // (three vector operations per logit instead of four).
      float neg_m = -m[t];
      float sum = 0.f;
#pragma unroll
      for (int e = 0; e < 16; ++e) sum += __builtin_amdgcn_exp2f(fmaf(x[e], cscale, neg_m));
      if (__any(!(sum <= kLazyLimit))) {                 // per-lane statistics: no cross-lane step
        float mx = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
        mx = fmaxf(mx, fmaxf(fmaxf(fmaxf(x[8], x[9]), fmaxf(x[10], x[11])),
                             fmaxf(fmaxf(x[12], x[13]), fmaxf(x[14], x[15]))));
        mx *= cscale;                                    // cscale > 0: max commutes with the scaling
        const float mn = fmaxf(m[t], mx);
        l[t] *= __builtin_amdgcn_exp2f(m[t] - mn);
        m[t] = mn;
        neg_m = -mn;
        sum = 0.f;
#pragma unroll
        for (int e = 0; e < 16; ++e) sum += __builtin_amdgcn_exp2f(fmaf(x[e], cscale, neg_m));
      }
      l[t] += sum;
    }
  };

  // Software pipeline: while the vector ALUs turn tile i's logits into statistics, the matrix
  // cores work on tile i+1 and tiles i+2, i+3 are on their way to LDS (tile i+4 follows as
  // soon as every wavefront is done with tile i's stage).  Each wavefront issues two
  // load-to-LDS per tile and nothing else on the vector-memory path inside the loop, so
  // "tile i+1 has landed" is "at most 2*(kAhead-1) operations outstanding".
  Tile ta;
  floatx16 sa[kStayRow], sb[kStayRow];
  wait_vmcnt<2 * kAhead>();                              // tile 0 landed (kAhead younger tiles in flight)
  block_barrier_no_drain();
  read_tile_from_lds(ta, smem, lane);
  tile_products<true, kStayRow>(ta, qt, zero, sa);                 // tile 0, C[key][query]
  auto step = [&](floatx16 (&s_cur)[kStayRow], floatx16 (&s_next)[kStayRow], int tile) {
    wait_vmcnt<2 * (kAhead - 1)>();                      // own part of tile+1 landed
    block_barrier_no_drain();                            // everyone's part; everyone done with `tile`
    stream(tile + kStages);                              // into the stage of `tile`
    read_tile_from_lds(ta, smem + ((tile + 1) % kStages) * kStageBytes, lane);
    tile_products<true, kStayRow>(ta, qt, zero, s_next);
    reduce(s_cur, tile);
  };
  for (int tile = 0; tile < ntiles; tile += 2) {
    step(sa, sb, tile);
    step(sb, sa, tile + 1);
  }
  wait_vmcnt<0>();                                       // nothing may land in LDS after the block is gone

  // the two lane halves hold disjoint key rows of the same query: merge, then one bias per row
#pragma unroll
  for (int t = 0; t < kStayRow; ++t) {
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

// ---- pass 2: grid (ceil(T / 512), H, JS), 256 threads; a wavefront owns 128 prompt keys,
// the block streams its share of the group's query tiles ----
__global__ __launch_bounds__(256) void teacher_colmax_kernel(
    const u32x4* q, const u32x4* k, const float* rowbias, int G, int Tq, int Tk, int T,
    int tq_pad, float cscale, float* __restrict__ part) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int h = blockIdx.y, js = blockIdx.z, JS = gridDim.z, H = gridDim.y;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int r = lane & 31, kg = lane >> 5;
  const int k0 = (blockIdx.x * 4 + wave) * (kStay * 32);
  const u32x4* kh = k + (size_t)h * Tk * kRowVec;
  const unsigned lds0 = lds_address(smem);

  // the G * (tq_pad / 32) query tiles of the group, split evenly over the JS blocks
  const int ntq = tq_pad / 32, total = G * ntq;
  const int first = (int)((long long)total * js / JS), end = (int)((long long)total * (js + 1) / JS);
  const int n = end - first;                             // >= 1: JS <= total
  // A query tile and the biases of its 32 rows (each wavefront fetches its own copy of the
  // 128 bytes, which keeps the count of vector-memory operations per wavefront uniform).
  auto stream = [&](int i) {                             // clamped: re-reading an item cannot change a maximum
    const int item = first + (i < n ? i : n - 1);
    const int g = h * G + item / ntq, j0 = (item % ntq) * 32;
    const unsigned stage = lds0 + (unsigned)((i % kStages) * kStageBytes);
    stream_tile_to_lds(q + (size_t)g * Tq * kRowVec, j0, Tq - 1, stage, wave, lane);
    load_to_lds_b32(rowbias + (size_t)g * tq_pad + j0 + (lane & 31), stage + kTileBytes + wave * 256);
  };
#pragma unroll
  for (int d = 0; d < kStages; ++d) stream(d);            // all stages: tiles 0 .. kAhead

  Tile kt[kStay];                                        // B operands: the wavefront's keys
#pragma unroll
  for (int t = 0; t < kStay; ++t) load_tile(kt[t], kh, k0 + 32 * t, T - 1, lane);
  float cm[kStay];
#pragma unroll
  for (int t = 0; t < kStay; ++t) cm[t] = -INFINITY;

  // The bias of a row, divided by the logit scale (which is applied after the maximum), is
  // the initial value of the row's accumulators: C[query][key] then holds logit + bias / c and
  // the column pass is a bare maximum.
  const float inv_c = 1.0f / cscale;
  auto read = [&](Tile& qt, floatx16& init, int i) {
    const unsigned char* stage = smem + (i % kStages) * kStageBytes;
    read_tile_from_lds(qt, stage, lane);
    const float* rb = reinterpret_cast<const float*>(stage + kTileBytes + wave * 256) + 4 * kg;
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      const floatx4 b4 = *reinterpret_cast<const floatx4*>(rb + 8 * a);
#pragma unroll
      for (int e = 0; e < 4; ++e) init[4 * a + e] = b4[e] * inv_c;
    }
  };
  auto reduce = [&](const floatx16 (&s)[kStay]) {
#pragma unroll
    for (int t = 0; t < kStay; ++t) {
      float best = cm[t];
#pragma unroll
      for (int e = 0; e < 16; ++e) best = fmaxf(best, s[t][e]);
      cm[t] = best;
    }
  };

  // software pipeline as in the row pass; three load-to-LDS per wavefront and item
  Tile qa;
  floatx16 ia, sa[kStay], sb[kStay];
  wait_vmcnt<3 * kAhead>();
  block_barrier_no_drain();
  read(qa, ia, 0);
  tile_products<false, kStay>(qa, kt, ia, sa);                  // item 0, C[query][key]
  auto step = [&](floatx16 (&s_cur)[kStay], floatx16 (&s_next)[kStay], int i) {
    wait_vmcnt<3 * (kAhead - 1)>();
    block_barrier_no_drain();
    stream(i + kStages);
    read(qa, ia, i + 1);
    tile_products<false, kStay>(qa, kt, ia, s_next);
    reduce(s_cur);
  };
  for (int i = 0; i < n; i += 2) {
    step(sa, sb, i);
    step(sb, sa, i + 1);                                 // i + 1 == n: a re-read item, harmless
  }
  wait_vmcnt<0>();

#pragma unroll
  for (int t = 0; t < kStay; ++t) {
    const float other = __shfl_xor(cm[t], 32, 64);
    const int key = k0 + 32 * t + r;
    if (kg == 0 && key < T) part[((size_t)js * H + h) * T + key] = fmaxf(cm[t], other) * cscale;
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
  const long long col_blocks = (long long)((T + 4 * kStay * 32 - 1) / (4 * kStay * 32)) * H;
  long long js = col_blocks > 0 ? (512 + col_blocks - 1) / col_blocks : 1;   // ~2 blocks per CU
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
  const dim3 g1((tq_pad + 4 * kStayRow * 32 - 1) / (4 * kStayRow * 32), HQ);
  constexpr size_t lds = (size_t)kStages * kStageBytes;
  teacher_rowstat_kernel<<<g1, 256, lds, stream>>>(qv, kv, hnorm, G, Tq, Tk, tq_pad, cscale, rowbias);
  if (hipGetLastError() != hipSuccess) return KVZAP_ERR_RUNTIME;
  const dim3 g2((T + 4 * kStay * 32 - 1) / (4 * kStay * 32), H, JS);
  teacher_colmax_kernel<<<g2, 256, lds, stream>>>(qv, kv, rowbias, G, Tq, Tk, T, tq_pad, cscale, part);
  if (hipGetLastError() != hipSuccess) return KVZAP_ERR_RUNTIME;
  const int n = H * T;
  teacher_finish_kernel<<<(n + 255) / 256, 256, 0, stream>>>(part, vnorm, n, JS, log_s);
  return hipGetLastError() == hipSuccess ? KVZAP_OK : KVZAP_ERR_RUNTIME;
}

}  // namespace kvzap
