// Ragged per-head gather of the kept K/V rows (Algorithm 1, last line; Sec. 5).
//
// Pure data movement, bound by HBM: every kept row is read once and written
// once, dropped rows are never touched.  A row of D bf16 values is moved as
// D/8 pieces of 16 bytes; consecutive lanes take consecutive pieces, so one
// wavefront reads and writes whole rows with 16-byte accesses (a 128-dim row
// is 256 B = 16 lanes, four rows per wavefront instruction).  Latency is covered
// by parallelism, not by per-thread unrolling: a thread moves one piece of one
// row per pass and the grid holds ~32k small blocks, which measured faster
// (5.6-5.9 TB/s) than 2-8 rows in flight per thread with fewer blocks
// (4.6-5.4 TB/s); non-temporal accesses are worth another 15 %.
// The grid is (tiles, B*H, {K,V}): blocks of one head stride over that head's kept
// rows, so no search for the owning head is needed and short heads simply run
// out of tiles early.
#include "kvzap_internal.h"

namespace kvzap {
namespace {

constexpr int kThreads = 256;

template <int LPR>  // lanes (16-byte pieces) per row
__global__ __launch_bounds__(kThreads) void compact_kernel(
    const u32x4* __restrict__ K, const u32x4* __restrict__ V,
    const int32_t* __restrict__ keep_idx, const int32_t* __restrict__ lengths,
    const int64_t* __restrict__ offsets, u32x4* __restrict__ K_out,
    u32x4* __restrict__ V_out, int64_t cap_rows, int T) {
  constexpr int kRowsPerPass = kThreads / LPR;            // rows one block covers at once
  const int bh = blockIdx.y;
  const int n = lengths[bh];
  const int64_t out0 = offsets[bh];
  const int piece = threadIdx.x % LPR;
  const int sub = threadIdx.x / LPR;
  // blockIdx.z selects the tensor: K and V rows are moved by different blocks (+3 %)
  const u32x4* src = (blockIdx.z ? V : K) + (size_t)bh * T * LPR;
  u32x4* dst = blockIdx.z ? V_out : K_out;
  for (int j0 = blockIdx.x * kRowsPerPass; j0 < n; j0 += gridDim.x * kRowsPerPass) {
    const int j = j0 + sub;
    if (j < n && out0 + j < cap_rows) {
      const int t = keep_idx[out0 + j];
      if (t >= 0 && t < T) {                                // never read outside the head
        const u32x4 row = __builtin_nontemporal_load(src + (size_t)t * LPR + piece);
        __builtin_nontemporal_store(row, dst + (size_t)(out0 + j) * LPR + piece);
      }
    }
  }
}

// any D that is a multiple of 8: one thread per 16-byte piece, pieces strided over the block
__global__ __launch_bounds__(kThreads) void compact_generic_kernel(
    const u32x4* __restrict__ K, const u32x4* __restrict__ V,
    const int32_t* __restrict__ keep_idx, const int32_t* __restrict__ lengths,
    const int64_t* __restrict__ offsets, u32x4* __restrict__ K_out,
    u32x4* __restrict__ V_out, int64_t cap_rows, int T, int lpr) {
  const int bh = blockIdx.y;
  const int n = lengths[bh];
  const int64_t out0 = offsets[bh];
  const u32x4* Kh = K + (size_t)bh * T * lpr;
  const u32x4* Vh = V + (size_t)bh * T * lpr;
  const int64_t pieces = (int64_t)n * lpr;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < pieces;
       i += (int64_t)gridDim.x * kThreads) {
    const int j = (int)(i / lpr), piece = (int)(i % lpr);
    if (out0 + j >= cap_rows) continue;
    const int t = keep_idx[out0 + j];
    if (t < 0 || t >= T) continue;
    K_out[(size_t)(out0 + j) * lpr + piece] = Kh[(size_t)t * lpr + piece];
    V_out[(size_t)(out0 + j) * lpr + piece] = Vh[(size_t)t * lpr + piece];
  }
}

}  // namespace

int launch_compact(const void* K, const void* V, const int32_t* keep_idx,
                   const int32_t* lengths, const int64_t* offsets, void* K_out,
                   void* V_out, int64_t cap_rows, int BH, int T, int D,
                   hipStream_t stream) {
  const int lpr = D / 8;
  // ~16k blocks (64 per CU), split evenly over heads
  int tiles_per_head;
  {
    const int rows_per_tile = kThreads / (lpr <= kThreads ? lpr : kThreads);
    const int max_tiles = (T + rows_per_tile - 1) / rows_per_tile;
    int want = (256 * 64 + BH - 1) / BH;
    tiles_per_head = want < max_tiles ? want : max_tiles;
    if (tiles_per_head < 1) tiles_per_head = 1;
  }
  const dim3 grid(tiles_per_head, BH, 2);
  const dim3 grid_generic(tiles_per_head, BH);
  const u32x4* k = static_cast<const u32x4*>(K);
  const u32x4* v = static_cast<const u32x4*>(V);
  u32x4* ko = static_cast<u32x4*>(K_out);
  u32x4* vo = static_cast<u32x4*>(V_out);
#define KVZAP_COMPACT_CASE(L)                                                              \
  case L:                                                                                  \
    compact_kernel<L><<<grid, kThreads, 0, stream>>>(k, v, keep_idx, lengths, offsets, ko, \
                                                     vo, cap_rows, T);                     \
    break;
  switch (lpr) {
    KVZAP_COMPACT_CASE(8)    // D = 64
    KVZAP_COMPACT_CASE(16)   // D = 128
    KVZAP_COMPACT_CASE(32)   // D = 256
    default:
      compact_generic_kernel<<<grid_generic, kThreads, 0, stream>>>(k, v, keep_idx, lengths, offsets,
                                                            ko, vo, cap_rows, T, lpr);
  }
#undef KVZAP_COMPACT_CASE
  return hipGetLastError() == hipSuccess ? KVZAP_OK : KVZAP_ERR_RUNTIME;
}

}  // namespace kvzap
