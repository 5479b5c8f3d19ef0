// Paged layout of the ragged cache (Sec. 1, criterion 3: compatibility with paged attention;
// Sec. 5: heads of different lengths need their own pages).  The kept rows of head (b,h)
// live in pages of `page_rows` rows of one pool; row j of the head is row j % page_rows of
// page block_table[b*H+h][j / page_rows].
//
//   assign_*  : every head, in (b,h) order, takes the next entries of the caller's free
//               list until it owns ceil((n + reserve) / page_rows) pages (first fit, so the
//               result is unique); "assign" starts from nothing, "extend" appends behind the
//               pages a head already owns
//   compact_* : the gather of Algorithm 1's last line, written through the block table
#include "kvzap_internal.h"

namespace kvzap {
namespace {

constexpr int kScanThreads = 1024;

__device__ __forceinline__ int pages_for(int n, int reserve, int log_page) {
  const long long total = (long long)(n < 0 ? 0 : n) + reserve;
  return total <= 0 ? 0 : (int)((total + (1ll << log_page) - 1) >> log_page);
}

// One block: pages to add per head -> exclusive scan -> start[0..BH], have[0..BH-1] (pages
// owned before the call; 0 without page_counts), result[0] = pages taken, result[1] = 0 ok /
// 1 free list too short / 2 a head would need more than max_pages.
__global__ __launch_bounds__(kScanThreads) void assign_scan_kernel(
    const int32_t* __restrict__ lengths, const int32_t* __restrict__ page_counts, int BH,
    int log_page, int reserve, int n_free, int max_pages, int32_t* __restrict__ start,
    int32_t* __restrict__ have, int32_t* __restrict__ result) {
  __shared__ long long s_sum[kScanThreads];
  __shared__ int s_over;
  const int tid = threadIdx.x;
  const int per = (BH + kScanThreads - 1) / kScanThreads;
  const int lo = tid * per, hi = lo + per < BH ? lo + per : BH;
  if (tid == 0) s_over = 0;
  __syncthreads();
  auto owned = [&](int i) {
    int h = page_counts ? page_counts[i] : 0;
    return h < 0 ? 0 : h;
  };
  auto to_add = [&](int i) {
    const int c = pages_for(lengths[i], reserve, log_page) - owned(i);
    return c > 0 ? c : 0;
  };
  long long mine = 0;
  bool over = false;
  for (int i = lo; i < hi; ++i) {
    const int c = to_add(i);
    over |= (long long)owned(i) + c > max_pages;
    mine += c;
  }
  if (over) s_over = 1;
  s_sum[tid] = mine;
  __syncthreads();
  // inclusive scan (Hillis-Steele) over the 1024 partial sums
  for (int d = 1; d < kScanThreads; d <<= 1) {
    const long long add = tid >= d ? s_sum[tid - d] : 0;
    __syncthreads();
    s_sum[tid] += add;
    __syncthreads();
  }
  const long long total = s_sum[kScanThreads - 1];
  const int status = s_over ? 2 : (total > n_free ? 1 : 0);
  long long run = s_sum[tid] - mine;                     // exclusive prefix of this thread
  for (int i = lo; i < hi; ++i) {
    start[i] = status ? 0 : (int32_t)run;
    have[i] = owned(i);
    run += to_add(i);
  }
  if (tid == 0) {
    start[BH] = status ? 0 : (int32_t)total;
    result[0] = status ? 0 : (int32_t)total;
    result[1] = status;
  }
}

// grid (tiles, B*H): the blocks of head bh write its new table entries.  kWholeRow (assign):
// the row is overwritten, -1 beyond its pages; otherwise (extend) only the appended entries
// are written and page_counts is updated.
template <bool kWholeRow>
__global__ __launch_bounds__(256) void assign_fill_kernel(
    const int32_t* __restrict__ start, const int32_t* __restrict__ have,
    const int32_t* __restrict__ free_pages, int32_t* __restrict__ block_table,
    int32_t* __restrict__ page_counts, int max_pages) {
  const int bh = blockIdx.y;
  const int s = start[bh], c = start[bh + 1] - s, h = have[bh];
  const int end = kWholeRow ? max_pages : (h + c < max_pages ? h + c : max_pages);
  for (int i = (kWholeRow ? 0 : h) + blockIdx.x * blockDim.x + threadIdx.x; i < end;
       i += gridDim.x * blockDim.x) {
    const int k = i - h;
    block_table[(size_t)bh * max_pages + i] = (k >= 0 && k < c) ? free_pages[s + k] : -1;
  }
  if (!kWholeRow && page_counts && blockIdx.x == 0 && threadIdx.x == 0 && c > 0)
    page_counts[bh] = h + c;
}

constexpr int kThreads = 256;

// Same work split as the contiguous gather: grid (tiles, B*H, {K,V}), a thread moves one
// 16-byte piece of one kept row per pass; only the destination differs.  Rows whose page
// slot lies beyond the table or whose table entry is not a page of the pool are skipped.
template <int LPR>
__global__ __launch_bounds__(kThreads) void compact_paged_kernel(
    const u32x4* __restrict__ K, const u32x4* __restrict__ V,
    const int32_t* __restrict__ keep_idx, const int32_t* __restrict__ lengths,
    const int64_t* __restrict__ offsets, const int32_t* __restrict__ block_table,
    int max_pages, int log_page, int num_pages, u32x4* __restrict__ K_pool,
    u32x4* __restrict__ V_pool, int T) {
  constexpr int kRowsPerPass = kThreads / LPR;
  const int bh = blockIdx.y;
  const int n = lengths[bh];
  const int64_t in0 = offsets[bh];
  const int piece = threadIdx.x % LPR;
  const int sub = threadIdx.x / LPR;
  const u32x4* src = (blockIdx.z ? V : K) + (size_t)bh * T * LPR;
  u32x4* dst = blockIdx.z ? V_pool : K_pool;
  const int32_t* pages = block_table + (size_t)bh * max_pages;
  for (int j0 = blockIdx.x * kRowsPerPass; j0 < n; j0 += gridDim.x * kRowsPerPass) {
    const int j = j0 + sub;
    if (j < n && (j >> log_page) < max_pages) {
      const int t = keep_idx[in0 + j];
      const int page = pages[j >> log_page];
      if (t >= 0 && t < T && page >= 0 && page < num_pages) {
        const u32x4 row = __builtin_nontemporal_load(src + (size_t)t * LPR + piece);
        const size_t out_row = ((size_t)page << log_page) + (size_t)(j & ((1 << log_page) - 1));
        __builtin_nontemporal_store(row, dst + out_row * LPR + piece);
      }
    }
  }
}

}  // namespace

size_t assign_pages_workspace_bytes(int BH) {
  return align_up((size_t)(2 * BH + 1) * sizeof(int32_t), 256);
}

// page_counts == nullptr: kvzap_assign_pages (nothing owned, whole rows written);
// otherwise kvzap_extend_pages.
int launch_assign_pages(const int32_t* lengths, int32_t* page_counts, int BH, int page_rows,
                        int reserve_rows, const int32_t* free_pages, int n_free,
                        int32_t* block_table, int max_pages, int32_t* result, void* workspace,
                        hipStream_t stream) {
  int log_page = 0;
  while ((1 << log_page) < page_rows) ++log_page;
  int32_t* start = static_cast<int32_t*>(workspace);
  int32_t* have = start + BH + 1;
  assign_scan_kernel<<<1, kScanThreads, 0, stream>>>(lengths, page_counts, BH, log_page,
                                                     reserve_rows, n_free, max_pages, start, have,
                                                     result);
  if (hipGetLastError() != hipSuccess) return KVZAP_ERR_RUNTIME;
  int tiles = (max_pages + 255) / 256;
  tiles = tiles < 64 ? tiles : 64;
  if (page_counts)
    assign_fill_kernel<false><<<dim3(tiles, BH), 256, 0, stream>>>(start, have, free_pages,
                                                                   block_table, page_counts, max_pages);
  else
    assign_fill_kernel<true><<<dim3(tiles, BH), 256, 0, stream>>>(start, have, free_pages,
                                                                  block_table, nullptr, max_pages);
  return hipGetLastError() == hipSuccess ? KVZAP_OK : KVZAP_ERR_RUNTIME;
}

int launch_compact_paged(const void* K, const void* V, const int32_t* keep_idx,
                         const int32_t* lengths, const int64_t* offsets,
                         const int32_t* block_table, int max_pages, int page_rows, void* K_pool,
                         void* V_pool, int num_pages, int BH, int T, int D, hipStream_t stream) {
  const int lpr = D / 8;
  int log_page = 0;
  while ((1 << log_page) < page_rows) ++log_page;
  const int rows_per_tile = kThreads / lpr;
  const int max_tiles = (T + rows_per_tile - 1) / rows_per_tile;
  int tiles = (256 * 64 + BH - 1) / BH;                  // ~16k blocks per tensor, as the contiguous gather
  tiles = tiles < max_tiles ? tiles : max_tiles;
  if (tiles < 1) tiles = 1;
  const dim3 grid(tiles, BH, 2);
  const u32x4* k = static_cast<const u32x4*>(K);
  const u32x4* v = static_cast<const u32x4*>(V);
  u32x4* kp = static_cast<u32x4*>(K_pool);
  u32x4* vp = static_cast<u32x4*>(V_pool);
  switch (lpr) {
    case 8:
      compact_paged_kernel<8><<<grid, kThreads, 0, stream>>>(k, v, keep_idx, lengths, offsets,
                                                             block_table, max_pages, log_page,
                                                             num_pages, kp, vp, T);
      break;
    case 16:
      compact_paged_kernel<16><<<grid, kThreads, 0, stream>>>(k, v, keep_idx, lengths, offsets,
                                                              block_table, max_pages, log_page,
                                                              num_pages, kp, vp, T);
      break;
    case 32:
      compact_paged_kernel<32><<<grid, kThreads, 0, stream>>>(k, v, keep_idx, lengths, offsets,
                                                              block_table, max_pages, log_page,
                                                              num_pages, kp, vp, T);
      break;
    default:
      return KVZAP_ERR_UNSUPPORTED;
  }
  return hipGetLastError() == hipSuccess ? KVZAP_OK : KVZAP_ERR_RUNTIME;
}

}  // namespace kvzap
