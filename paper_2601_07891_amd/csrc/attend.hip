// Decode-step attention over the ragged per-head cache (Sec. 5; weights of Sec. 3.2
// Eq. 2): for every KV head, its G = HQ/H query heads attend to the head's packed
// rows and to the rows still inside the window ring.
//
// The kernel is bound by reading K and V once (512 bytes per row against 4*G*128
// flops), so the design is about streaming rows with as few vector-ALU instructions
// per byte as possible; both contractions run on v_mfma_f32_16x16x32_bf16 straight
// from the registers the global loads fill, with no LDS and no barrier:
//
//   one wave = one split of one KV head, 32-row chunks, the next chunk's loads in
//   flight while the current one is consumed.
//
//   S^T = K q^T      A = K   lane (i = l%16, kg = l/16) loads 16 bytes of row rho(i) at
//                            byte 64*kk + 16*kg for kk = 0..3 (the k-slices an MFMA
//                            step wants); two 16-row sets per chunk
//                    B = q   lane (g = l%16, kg) holds q[g][32kk + 8kg ..+8], zero for
//                            g >= G
//                    C       lane (g, s = l/16), register r: row i = 4s + r of the set
//   with rho(t, i) = 16t + 4(i%4) + i/4, so lane (g, s) ends up with the scores of the
//   chunk rows 4j + s, j = 4t + r = 0..7: exactly the eight k-slots of B in
//
//   O^T = V^T P^T    A = V^T lane (c = l%16, s = l/16) loads piece c (8 values,
//                            d = 8c..8c+7) of the rows 4j + s, j = 0..7, fully
//                            coalesced (a load instruction covers 4 whole rows); one
//                            v_perm per register pairs rows (2j', 2j'+1) of one d,
//                            which is the k-pair layout of the A operand for the
//                            d-tile {8c + e : c = 0..15}
//                    B = P^T the exponentiated scores of lane (g, s), packed to bf16
//                    C       lane (g, s), tile e, register r: d = 32s + 8r + e
//   plus one more MFMA with A = ones whose result is the softmax denominator (the sum of
//   the bf16-rounded weights, already reduced over all 32 rows).
//
// The softmax reference m is lazy: scores are exponentiated relative to a per-head
// reference that is only raised (with a rescale of the accumulators) when some score
// exceeds it by more than 2^16; fp32 and bf16 carry that range without loss, so the
// common chunk needs no cross-lane traffic at all.
//
// A second small kernel combines the splits of each head and writes bf16.
#include "kvzap_internal.h"

namespace kvzap {
namespace {

constexpr int kD = 128;                 // head dimension (elements)
constexpr int kChunkRows = 32;
constexpr float kLazyMargin = 16.0f;    // log2 units

// Rows of one head: packed prefix [0, n_p) at row offset `off`, ring [0, n_r).
struct HeadExtent {
  int64_t off;
  int n_p, n_r;
};

// Contiguous layout: head bh owns rows row_offsets[bh] .. of a store of cap_rows rows.
// Paged layout (row_offsets == nullptr): its rows are addressed through its block table and
// cap_rows is what the table can address (max_pages * page_rows, 0 for an empty pool).
__device__ __forceinline__ HeadExtent head_extent(const int64_t* row_offsets,
                                                  const int32_t* lengths,
                                                  const int32_t* seq_pos, int window,
                                                  int64_t cap_rows, int bh, int b) {
  HeadExtent e;
  e.off = row_offsets ? row_offsets[bh] : 0;
  int64_t n = lengths[bh];
  if (e.off < 0 || e.off > cap_rows) { e.off = 0; n = 0; }
  if (n < 0) n = 0;
  if (n > cap_rows - e.off) n = cap_rows - e.off;
  e.n_p = (int)n;
  int r = 0;
  if (window > 0) {
    r = seq_pos[b];
    r = r < 0 ? 0 : (r > window ? window : r);
  }
  e.n_r = r;
  return e;
}

__device__ __forceinline__ int chunks_of(int rows) { return (rows + kChunkRows - 1) / kChunkRows; }

struct Chunk {
  u32x4 k[2][4];   // [set][k-step]
  u32x4 v[8];      // [row group j]
};

// Where the rows of one head live.
struct Source {
  const u32x4* K;            // packed rows of this head (contiguous) or the page pool (paged)
  const u32x4* V;
  const u32x4* Kr;           // ring rows of this head
  const u32x4* Vr;
  const int32_t* pages;      // paged: this head's block-table row
  int log_page, max_pages, num_pages;
  int n_p, n_r;
};

constexpr int kRowVec = kD * 2 / 16;   // 16-byte pieces per row

// Offset (in 16-byte pieces) of packed row r of the head from Source::K / Source::V.  Paged:
// row r is row r % page_rows of page pages[r / page_rows]; a table entry outside the pool is
// clamped into it, so nothing outside the pool is ever read.
template <bool kPaged>
__device__ __forceinline__ size_t prefix_offset(const Source& s, int r) {
  if (!kPaged) return (size_t)r * kRowVec;
  int slot = r >> s.log_page;
  slot = slot < s.max_pages - 1 ? slot : s.max_pages - 1;
  int page = s.pages[slot];
  page = page < 0 ? 0 : (page < s.num_pages ? page : s.num_pages - 1);
  return (((size_t)page << s.log_page) + (size_t)(r & ((1 << s.log_page) - 1))) * kRowVec;
}

// Loads chunk `vc` of the head's chunk list (prefix chunks, then ring chunks).  Rows past
// the end of the segment are read from its last row (their weights are forced to zero).
// A page holds a multiple of 16 rows, so each 16-row half of a chunk is contiguous.
template <bool kPaged>
__device__ __forceinline__ void load_chunk(Chunk& c, int vc, int cp, const Source& s, int li,
                                           int lg, int& row0, int& n_seg) {
  const bool ring = vc >= cp;
  const u32x4* Kb = ring ? s.Kr : s.K;
  const u32x4* Vb = ring ? s.Vr : s.V;
  n_seg = ring ? s.n_r : s.n_p;
  row0 = (ring ? vc - cp : vc) * kChunkRows;
  const int klocal = 4 * (li & 3) + (li >> 2);          // row of this lane inside a 16-row set
  if (row0 + kChunkRows <= n_seg) {
    size_t half[2];
    if (kPaged && !ring) {
      half[0] = prefix_offset<kPaged>(s, row0);
      half[1] = prefix_offset<kPaged>(s, row0 + 16);
    } else {
      half[0] = (size_t)row0 * kRowVec;
      half[1] = half[0] + 16 * kRowVec;
    }
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const u32x4* kp = Kb + half[t] + klocal * kRowVec + lg;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) c.k[t][kk] = kp[kk * 4];
    }
#pragma unroll
    for (int j = 0; j < 8; ++j)
      c.v[j] = Vb[half[j >> 2] + (size_t)(4 * (j & 3) + lg) * kRowVec + li];
  } else {
    const int last = n_seg - 1;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      int r = row0 + 16 * t + klocal;
      r = r < last ? r : last;
      const size_t o = (kPaged && !ring) ? prefix_offset<kPaged>(s, r) : (size_t)r * kRowVec;
      const u32x4* kp = Kb + o + lg;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) c.k[t][kk] = kp[kk * 4];
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      int r = row0 + 4 * j + lg;
      r = r < last ? r : last;
      const size_t o = (kPaged && !ring) ? prefix_offset<kPaged>(s, r) : (size_t)r * kRowVec;
      c.v[j] = Vb[o + li];
    }
  }
}

struct Accum {
  floatx4 o[8];    // [d-tile e][r]: d = 32s + 8r + e
  floatx4 l;       // every register: sum of the weights of head g
  float m;         // reference exponent of head g (scaled log2 units)
};

__device__ __forceinline__ float shfl_xor_f(float x, int mask) {
  return __shfl_xor(x, mask, 64);
}

__device__ __forceinline__ void consume_chunk(const Chunk& c, const u32x4 (&qb)[4], Accum& a,
                                              int row0, int n_seg, int lg, float cscale) {
  floatx4 s[2];
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    s[t] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
      s[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, c.k[t][kk]),
                                                     __builtin_bit_cast(bf16x8, qb[kk]), s[t],
                                                     0, 0, 0);
  }
  float x[8];
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int r = 0; r < 4; ++r) x[4 * t + r] = s[t][r] * cscale;
  if (row0 + kChunkRows > n_seg) {
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (row0 + 4 * j + lg >= n_seg) x[j] = -INFINITY;
  }
  float mx = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])),
                   fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
  if (__any(mx > a.m + kLazyMargin)) {
    // raise the reference to the exact running maximum of each head and rescale
    float mn = fmaxf(mx, shfl_xor_f(mx, 16));
    mn = fmaxf(mn, shfl_xor_f(mn, 32));
    mn = fmaxf(mn, a.m);
    const float alpha = __builtin_amdgcn_exp2f(a.m - mn);   // 0 when a.m = -inf
#pragma unroll
    for (int e = 0; e < 8; ++e) a.o[e] *= alpha;
    a.l *= alpha;
    a.m = mn;
  }
  bf16x8 p;
#pragma unroll
  for (int j = 0; j < 8; ++j) p[j] = (__bf16)__builtin_amdgcn_exp2f(x[j] - a.m);

  constexpr unsigned kSelLo = 0x05040100u, kSelHi = 0x07060302u;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    u32x4 vt;
#pragma unroll
    for (int jp = 0; jp < 4; ++jp)
      vt[jp] = __builtin_amdgcn_perm(c.v[2 * jp + 1][e >> 1], c.v[2 * jp][e >> 1],
                                     (e & 1) ? kSelHi : kSelLo);
    a.o[e] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vt), p, a.o[e],
                                                     0, 0, 0);
  }
  const u32x4 ones = {0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};
  a.l = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ones), p, a.l, 0, 0, 0);
}

// grid (NS, B*H), 64 threads.  part: [B*H][NS][G][128] fp32, ml: [B*H][NS][G][2] fp32.
// Contiguous layout: K_rows/V_rows are the row store, row_offsets the heads' first rows.
// Paged layout: K_rows/V_rows are the page pool, row_offsets is null, block_table given.
template <bool kPaged>
__global__ __launch_bounds__(64, 2) void attend_partial_kernel(
    const u32x4* q, const u32x4* K_rows, const u32x4* V_rows, int64_t cap_rows,
    const int64_t* row_offsets, const int32_t* block_table, int max_pages, int log_page,
    int num_pages, const int32_t* lengths, const u32x4* K_ring, const u32x4* V_ring,
    const int32_t* seq_pos, int window, float cscale, int H, int G, int spc, float* part,
    float* ml) {
  const int bh = blockIdx.y, split = blockIdx.x, NS = gridDim.x;
  const int b = bh / H;
  const HeadExtent e = head_extent(row_offsets, lengths, seq_pos, window, cap_rows, bh, b);
  const int cp = chunks_of(e.n_p), ct = cp + chunks_of(e.n_r);
  const int c0 = split * spc;
  // the last split runs to the end of the list, so a head longer than the host's bound
  // is still covered
  const int c1 = (split == NS - 1) ? ct : (c0 + spc < ct ? c0 + spc : ct);
  if (c0 >= c1) return;

  const int lane = threadIdx.x, li = lane & 15, lg = lane >> 4;
  Source src;
  src.K = K_rows + (size_t)e.off * kRowVec;
  src.V = V_rows + (size_t)e.off * kRowVec;
  src.Kr = K_ring + (size_t)bh * (window > 0 ? window : 0) * kRowVec;
  src.Vr = V_ring + (size_t)bh * (window > 0 ? window : 0) * kRowVec;
  src.pages = kPaged ? block_table + (size_t)bh * max_pages : nullptr;
  src.log_page = log_page; src.max_pages = max_pages; src.num_pages = num_pages;
  src.n_p = e.n_p; src.n_r = e.n_r;

  // q as the B operand: lane (g = li, kg = lg), k-step kk: q[g][32kk + 8kg ..+8]
  u32x4 qb[4];
  {
    const u32x4 zero = {0u, 0u, 0u, 0u};
    const u32x4* qp = q + ((size_t)bh * G + (li < G ? li : 0)) * kRowVec + lg;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) qb[kk] = li < G ? qp[kk * 4] : zero;
  }

  Accum acc;
#pragma unroll
  for (int t = 0; t < 8; ++t) acc.o[t] = floatx4{0.f, 0.f, 0.f, 0.f};
  acc.l = floatx4{0.f, 0.f, 0.f, 0.f};
  acc.m = -INFINITY;

  // Two chunk buffers; the steady-state loop has no branch around a load, so the
  // compiler's wait counts let the loads of one buffer fly while the other is consumed.
  Chunk ca, cb;
  int row0a, nsega, row0b, nsegb;
  load_chunk<kPaged>(ca, c0, cp, src, li, lg, row0a, nsega);
  int vc = c0;
  while (vc + 2 < c1) {
    load_chunk<kPaged>(cb, vc + 1, cp, src, li, lg, row0b, nsegb);
    consume_chunk(ca, qb, acc, row0a, nsega, lg, cscale);
    load_chunk<kPaged>(ca, vc + 2, cp, src, li, lg, row0a, nsega);
    consume_chunk(cb, qb, acc, row0b, nsegb, lg, cscale);
    vc += 2;
  }
  if (vc + 1 < c1) {
    load_chunk<kPaged>(cb, vc + 1, cp, src, li, lg, row0b, nsegb);
    consume_chunk(ca, qb, acc, row0a, nsega, lg, cscale);
    consume_chunk(cb, qb, acc, row0b, nsegb, lg, cscale);
  } else {
    consume_chunk(ca, qb, acc, row0a, nsega, lg, cscale);
  }

  if (li < G) {
    const size_t slot = ((size_t)bh * NS + split) * G + li;
    float* dst = part + slot * kD + 32 * lg;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      floatx4 lo = {acc.o[0][r], acc.o[1][r], acc.o[2][r], acc.o[3][r]};
      floatx4 hi = {acc.o[4][r], acc.o[5][r], acc.o[6][r], acc.o[7][r]};
      *reinterpret_cast<floatx4*>(dst + 8 * r) = lo;
      *reinterpret_cast<floatx4*>(dst + 8 * r + 4) = hi;
    }
    if (lg == 0) {
      ml[slot * 2] = acc.m;
      ml[slot * 2 + 1] = acc.l[0];
    }
  }
}

// grid B*H*G, 256 threads: thread (c = tid%32, sg = tid/32) folds the splits sg, sg+8, ...
// of output elements 4c..4c+3 with a running reference, then the 8 groups meet in LDS.
constexpr int kCombineGroups = 8;

__global__ __launch_bounds__(256) void attend_combine_kernel(
    const float* part, const float* ml, int64_t total_rows, const int64_t* row_offsets,
    const int32_t* lengths, const int32_t* seq_pos, int window, int H, int G, int NS, int spc,
    unsigned short* out) {
  __shared__ floatx4 s_num[kCombineGroups][32];
  __shared__ float s_m[kCombineGroups], s_den[kCombineGroups];
  const int bh = blockIdx.x / G, g = blockIdx.x % G;
  const int c = threadIdx.x & 31, sg = threadIdx.x >> 5;
  const HeadExtent e = head_extent(row_offsets, lengths, seq_pos, window, total_rows, bh, bh / H);
  const int ct = chunks_of(e.n_p) + chunks_of(e.n_r);
  int ns = (ct + spc - 1) / spc;
  ns = ns < NS ? ns : NS;
  float m = -INFINITY, den = 0.f;
  floatx4 num = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
  for (int s = sg; s < ns; s += kCombineGroups) {
    const size_t slot = ((size_t)bh * NS + s) * G + g;
    const float ms = ml[slot * 2], ls = ml[slot * 2 + 1];
    const floatx4 a = *reinterpret_cast<const floatx4*>(part + slot * kD + 4 * c);
    const float mn = fmaxf(m, ms);
    const float w_old = __builtin_amdgcn_exp2f(m - mn), w_new = __builtin_amdgcn_exp2f(ms - mn);
    num = num * w_old + a * w_new;
    den = den * w_old + ls * w_new;
    m = mn;
  }
  s_num[sg][c] = num;
  if (c == 0) { s_m[sg] = m; s_den[sg] = den; }
  __syncthreads();
  if (sg == 0) {
    float mm = s_m[0];
#pragma unroll
    for (int k = 1; k < kCombineGroups; ++k) mm = fmaxf(mm, s_m[k]);
    floatx4 n = {0.f, 0.f, 0.f, 0.f};
    float dsum = 0.f;
#pragma unroll
    for (int k = 0; k < kCombineGroups; ++k) {
      // a group that saw no split has m = -inf and zero sums; exp2(-inf - mm) = 0 unless
      // mm is -inf too (no split at all), which the ns > 0 test below covers
      const float w = (s_m[k] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(s_m[k] - mm);
      n += s_num[k][c] * w;
      dsum += s_den[k] * w;
    }
    unsigned short* o = out + (size_t)blockIdx.x * kD + 4 * c;
    typedef unsigned short u16x4 __attribute__((ext_vector_type(4)));
    u16x4 r;
#pragma unroll
    for (int k = 0; k < 4; ++k) r[k] = float_to_bf16_bits(ns > 0 ? n[k] / dsum : 0.f);
    *reinterpret_cast<u16x4*>(o) = r;
  }
}

}  // namespace

// Chunks per split (one split = one wave).  Long splits amortise a wave's start-up (its
// first loads are not overlapped with anything), the partial result it writes and the work
// of the combine kernel, which folds every split of a head in one block; short ones fill
// the chip when there are few heads.  Aim at ~2048 waves if every head were at the bound,
// within 4..64 chunks (128..2048 rows).  Measured on 512 heads of 4k..32k rows: 16 chunks
// 5.62, 32: 5.76, 64: 5.87, 128: 5.54 TB/s; on 8 heads of 131072 rows a target of 8192
// waves (1025 splits per head) gives 4.4 TB/s, 2048 waves 5.2, 1024 waves 5.0.
int attend_split_chunks(int BH, int max_rows, int window) {
  const long long ct = (max_rows + kChunkRows - 1) / kChunkRows +
                       ((window > 0 ? window : 0) + kChunkRows - 1) / kChunkRows;
  long long want = ct * BH / 2048;
  int spc = 4;
  while (spc < 64 && spc < want) spc *= 2;
  return spc;
}

int attend_splits(int BH, int max_rows, int window) {
  const int ct = (max_rows + kChunkRows - 1) / kChunkRows +
                 ((window > 0 ? window : 0) + kChunkRows - 1) / kChunkRows;
  const int spc = attend_split_chunks(BH, max_rows, window);
  const int ns = (ct + spc - 1) / spc;
  return ns > 0 ? ns : 1;
}

size_t attend_workspace_bytes(int B, int H, int HQ, int max_rows, int window) {
  const size_t slots = (size_t)B * H * attend_splits(B * H, max_rows, window) * (HQ / H);
  return align_up(slots * kD * sizeof(float), 256) + align_up(slots * 2 * sizeof(float), 256);
}

int launch_attend_decode(const void* q, const void* K_rows, const void* V_rows,
                         int64_t total_rows, const int64_t* row_offsets,
                         const int32_t* block_table, int max_pages, int page_rows, int num_pages,
                         const int32_t* lengths, const void* K_ring, const void* V_ring,
                         const int32_t* seq_pos, int window, int max_rows, float scale,
                         void* out, int B, int H, int HQ, void* workspace,
                         hipStream_t stream) {
  const int G = HQ / H, BH = B * H;
  const int NS = attend_splits(BH, max_rows, window);
  const int spc = attend_split_chunks(BH, max_rows, window);
  const size_t slots = (size_t)BH * NS * G;
  float* part = static_cast<float*>(workspace);
  float* ml = reinterpret_cast<float*>(static_cast<char*>(workspace) +
                                       align_up(slots * kD * sizeof(float), 256));
  const float cscale = scale * 1.4426950408889634f;
  const bool paged = block_table != nullptr;
  int log_page = 0;
  while ((1 << log_page) < page_rows) ++log_page;
  // rows a head can address: the whole store, or what its block-table row covers
  const int64_t cap_rows = paged ? (num_pages > 0 ? (int64_t)max_pages * page_rows : 0) : total_rows;
  const auto* qv = static_cast<const u32x4*>(q);
  const auto* kv = static_cast<const u32x4*>(K_rows);
  const auto* vv = static_cast<const u32x4*>(V_rows);
  const auto* kr = static_cast<const u32x4*>(K_ring);
  const auto* vr = static_cast<const u32x4*>(V_ring);
  if (paged)
    hipLaunchKernelGGL(attend_partial_kernel<true>, dim3(NS, BH), dim3(64), 0, stream, qv, kv, vv,
                       cap_rows, nullptr, block_table, max_pages, log_page, num_pages, lengths, kr,
                       vr, seq_pos, window, cscale, H, G, spc, part, ml);
  else
    hipLaunchKernelGGL(attend_partial_kernel<false>, dim3(NS, BH), dim3(64), 0, stream, qv, kv, vv,
                       cap_rows, row_offsets, nullptr, 0, 0, 0, lengths, kr, vr, seq_pos, window,
                       cscale, H, G, spc, part, ml);
  if (hipGetLastError() != hipSuccess) return KVZAP_ERR_RUNTIME;
  hipLaunchKernelGGL(attend_combine_kernel, dim3(BH * G), dim3(256), 0, stream, part, ml,
                     cap_rows, paged ? nullptr : row_offsets, lengths, seq_pos, window, H, G, NS,
                     spc, static_cast<unsigned short*>(out));
  if (hipGetLastError() != hipSuccess) return KVZAP_ERR_RUNTIME;
  return KVZAP_OK;
}

}  // namespace kvzap
