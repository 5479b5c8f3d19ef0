// Threshold + sliding-window mask and per-head index lists (Sec. 3.3, Algorithm 1).
//
// Small launches over scores [B*H, T] (4 bytes per flag, so the whole stage moves
// ~1 % of the bytes of the K/V compaction that follows; it is bound by the ~4 us
// floor of a kernel launch, so the number of launches is what matters):
//   1. count : one block per 1024-token chunk of one (b,h) row counts its kept flags
//   2. emit  : every chunk recomputes its flags (scores are L2-resident by now),
//              ranks them with a wave shuffle scan + LDS and writes the ascending
//              kept positions at its prefix.  With up to kFusedMaxChunks chunks each
//              block derives its own prefix by summing the counts of all chunks
//              before it (a few KB from L2), and the first chunk of every head
//              also writes lengths and offsets; beyond that a single-block scan
//              kernel runs between the two.
// No block waits for another, so there is nothing that can spin.
#include <mutex>

#include "kvzap_internal.h"

namespace kvzap {
namespace {

// Scratch of the allocation-free entry point (kvzap_mask_static): the chunk counts and chunk
// prefixes that kvzap_mask keeps in its caller's workspace, for up to kStaticMaskChunks
// 1024-token chunks.  One copy per GPU, at its own address on each, held until the process
// ends; every call on a GPU shares it, so calls that overlap on one GPU race.  Nothing in it
// has to start at zero: the count kernel writes every entry the later kernels read.
constexpr size_t kStaticCountBytes = (size_t)kStaticMaskChunks * sizeof(int32_t);
constexpr size_t kStaticScratchBytes = kStaticCountBytes + (size_t)kStaticMaskChunks * sizeof(int64_t);
static_assert(kStaticCountBytes % 256 == 0, "the prefix part stays 256-byte aligned");
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// In host code `scratch` is only a stand-in for the symbol, not a device address: the address
// on the current GPU is looked up once per device and kept here.
constexpr int kMaxDevices = 64;
std::mutex scratch_mutex;
void* scratch_ptr[kMaxDevices] = {};

int static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return KVZAP_ERR_RUNTIME;
  std::lock_guard<std::mutex> lock(scratch_mutex);
  if (!scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
      (void)hipGetLastError();
      return KVZAP_ERR_RUNTIME;
    }
    scratch_ptr[dev] = p;
  }
  *out = scratch_ptr[dev];
  return KVZAP_OK;
}

constexpr int kThreads = 256;            // 4 wavefronts
constexpr int kPerThread = kMaskChunk / kThreads;  // 4 consecutive tokens
static_assert(kPerThread == 4, "one float4 per thread");

// A sequence's own length, clamped into [0, T]: positions at or beyond T do not exist whatever
// the caller's array says (it lives on the device, so the host cannot reject it)
__device__ __forceinline__ int seq_len_of(const int32_t* __restrict__ seq_lens, int b, int T) {
  if (!seq_lens) return T;
  const int n = seq_lens[b];
  return n < 0 ? 0 : (n > T ? T : n);
}

// keep flags of tokens t0..t0+3 of one (b,h) row
__device__ __forceinline__ unsigned keep_bits4(const float* __restrict__ row, int t0, int T,
                                               int Tb, int window, float tau, bool vec_ok) {
  float s[4];
  if (vec_ok && t0 + 3 < T) {
    const floatx4 v = *reinterpret_cast<const floatx4*>(row + t0);
    s[0] = v.x; s[1] = v.y; s[2] = v.z; s[3] = v.w;
  } else {
#pragma unroll
    for (int e = 0; e < 4; ++e) s[e] = (t0 + e < T) ? row[t0 + e] : 0.0f;
  }
  const int first_protected = Tb - window;   // may be negative: everything protected
  unsigned bits = 0;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int t = t0 + e;
    const bool keep = (t < Tb) && ((t >= first_protected) || (s[e] >= tau));
    bits |= (keep ? 1u : 0u) << e;
  }
  return bits;
}

__global__ __launch_bounds__(kThreads) void mask_count_kernel(
    const float* __restrict__ scores, float tau_all, const float* __restrict__ tau_head, int window,
    const int32_t* __restrict__ seq_lens, int H, int T, int nchunks,
    int32_t* __restrict__ chunk_counts) {
  const int chunk = blockIdx.x, bh = blockIdx.y;
  const float tau = tau_head ? tau_head[bh] : tau_all;     // one threshold, or one per head
  const int Tb = seq_len_of(seq_lens, bh / H, T);
  const float* row = scores + (size_t)bh * T;
  const bool vec_ok = (T % 4) == 0;
  const int t0 = chunk * kMaskChunk + threadIdx.x * kPerThread;
  const int c = __popc(keep_bits4(row, t0, T, Tb, window, tau, vec_ok));
  // block sum: wave reduce then LDS
  int v = c;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
  __shared__ int wave_sum[kThreads / 64];
  if ((threadIdx.x & 63) == 0) wave_sum[threadIdx.x >> 6] = v;
  __syncthreads();
  if (threadIdx.x == 0) {
    int tot = 0;
#pragma unroll
    for (int w = 0; w < kThreads / 64; ++w) tot += wave_sum[w];
    chunk_counts[(size_t)bh * nchunks + chunk] = tot;
  }
}

constexpr int kScanThreads = 1024;

__global__ __launch_bounds__(kScanThreads) void mask_scan_kernel(
    const int32_t* __restrict__ chunk_counts, int64_t* chunk_prefix,
    int BH, int nchunks, int32_t* __restrict__ lengths, int64_t* __restrict__ offsets) {
  __shared__ long long wave_tot[kScanThreads / 64];
  __shared__ long long carry_s;
  const int n = BH * nchunks;
  const int lane = threadIdx.x & 63, wid = threadIdx.x >> 6;
  if (threadIdx.x == 0) carry_s = 0;
  __syncthreads();
  for (int base = 0; base < n; base += kScanThreads) {
    const int i = base + threadIdx.x;
    const long long v = (i < n) ? (long long)chunk_counts[i] : 0;
    long long incl = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const long long up = __shfl_up(incl, off, 64);
      if (lane >= off) incl += up;
    }
    if (lane == 63) wave_tot[wid] = incl;
    __syncthreads();
    long long before = carry_s;
    for (int w = 0; w < wid; ++w) before += wave_tot[w];
    if (i < n) chunk_prefix[i] = before + incl - v;
    __syncthreads();
    if (threadIdx.x == kScanThreads - 1) carry_s = before + incl;
    __syncthreads();
  }
  // head starts: the prefix of a head's first chunk; written by this block above
  __threadfence_block();
  __syncthreads();
  for (int bh = threadIdx.x; bh <= BH; bh += kScanThreads) {
    const long long start = (bh < BH) ? chunk_prefix[(size_t)bh * nchunks] : carry_s;
    offsets[bh] = start;
    if (bh < BH) {
      const long long end = (bh + 1 < BH) ? chunk_prefix[(size_t)(bh + 1) * nchunks] : carry_s;
      lengths[bh] = (int32_t)(end - start);
    }
  }
}

constexpr int kFusedMaxChunks = 8192;

// block-wide sum of a 64-bit value (all threads get the result)
__device__ __forceinline__ long long block_sum_i64(long long v, long long* lds_scratch) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) lds_scratch[threadIdx.x >> 6] = v;
  __syncthreads();
  long long s = 0;
#pragma unroll
  for (int w = 0; w < kThreads / 64; ++w) s += lds_scratch[w];
  return s;
}

template <bool kFused>
__global__ __launch_bounds__(kThreads) void mask_emit_kernel(
    const float* __restrict__ scores, float tau_all, const float* __restrict__ tau_head, int window,
    const int32_t* __restrict__ seq_lens, int H, int T, int nchunks,
    const int64_t* __restrict__ chunk_prefix, const int32_t* __restrict__ chunk_counts,
    int32_t* __restrict__ keep_idx, int32_t* __restrict__ lengths,
    int64_t* __restrict__ offsets) {
  const int chunk = blockIdx.x, bh = blockIdx.y;
  long long my_prefix;
  if (kFused) {
    __shared__ long long scratch[kThreads / 64];
    const int BH = gridDim.y;
    const int mine = bh * nchunks + chunk;               // chunks are ordered (b,h)-major
    long long before = 0;
    for (int i = threadIdx.x; i < mine; i += kThreads) before += chunk_counts[i];
    my_prefix = block_sum_i64(before, scratch);
    if (chunk == 0) {                                    // this head's length and start
      long long own = 0;
      for (int i = threadIdx.x; i < nchunks; i += kThreads) own += chunk_counts[mine + i];
      const long long head_total = block_sum_i64(own, scratch);
      if (threadIdx.x == 0) {
        offsets[bh] = my_prefix;
        lengths[bh] = (int32_t)head_total;
        if (bh == BH - 1) offsets[BH] = my_prefix + head_total;
      }
    }
  } else {
    my_prefix = chunk_prefix[(size_t)bh * nchunks + chunk];
  }
  const float tau = tau_head ? tau_head[bh] : tau_all;
  const int Tb = seq_len_of(seq_lens, bh / H, T);
  const float* row = scores + (size_t)bh * T;
  const bool vec_ok = (T % 4) == 0;
  const int t0 = chunk * kMaskChunk + threadIdx.x * kPerThread;
  const unsigned bits = keep_bits4(row, t0, T, Tb, window, tau, vec_ok);
  const int c = __popc(bits);
  // exclusive scan of c over the block: within the wave by shuffles, across waves via LDS
  const int lane = threadIdx.x & 63, wid = threadIdx.x >> 6;
  int incl = c;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int up = __shfl_up(incl, off, 64);
    if (lane >= off) incl += up;
  }
  __shared__ int wave_tot[kThreads / 64];
  if (lane == 63) wave_tot[wid] = incl;
  __syncthreads();
  int before = 0;
#pragma unroll
  for (int w = 0; w < kThreads / 64; ++w) before += (w < wid) ? wave_tot[w] : 0;
  int64_t pos = my_prefix + before + incl - c;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    if (bits & (1u << e)) keep_idx[pos++] = t0 + e;
  }
}

}  // namespace

int launch_mask(const float* scores, float tau, const float* tau_head, int window,
                const int32_t* seq_lens,
                int B, int H, int T, int32_t* keep_idx, int32_t* lengths,
                int64_t* offsets, void* workspace, hipStream_t stream) {
  const int BH = B * H;
  const int nchunks = mask_chunks(T);
  int32_t* chunk_counts = static_cast<int32_t*>(workspace);
  int64_t* chunk_prefix = reinterpret_cast<int64_t*>(
      static_cast<char*>(workspace) + align_up((size_t)BH * nchunks * sizeof(int32_t), 256));
  const dim3 grid(nchunks, BH);
  mask_count_kernel<<<grid, kThreads, 0, stream>>>(scores, tau, tau_head, window, seq_lens, H, T,
                                                   nchunks, chunk_counts);
  if ((long long)BH * nchunks <= kFusedMaxChunks) {
    mask_emit_kernel<true><<<grid, kThreads, 0, stream>>>(scores, tau, tau_head, window, seq_lens, H, T,
                                                          nchunks, chunk_prefix, chunk_counts,
                                                          keep_idx, lengths, offsets);
  } else {
    mask_scan_kernel<<<1, kScanThreads, 0, stream>>>(chunk_counts, chunk_prefix, BH, nchunks,
                                                     lengths, offsets);
    mask_emit_kernel<false><<<grid, kThreads, 0, stream>>>(scores, tau, tau_head, window, seq_lens, H, T,
                                                           nchunks, chunk_prefix, chunk_counts,
                                                           keep_idx, lengths, offsets);
  }
  return hipGetLastError() == hipSuccess ? KVZAP_OK : KVZAP_ERR_RUNTIME;
}

int launch_mask_static(const float* scores, float tau, int window, const int32_t* seq_lens, int B,
                       int H, int T, int32_t* keep_idx, int32_t* lengths, int64_t* offsets,
                       hipStream_t stream) {
  if ((long long)B * H * mask_chunks(T) > (long long)kStaticMaskChunks) return KVZAP_ERR_STATIC_LIMIT;
  void* ws = nullptr;
  const int rc = static_scratch(&ws);
  if (rc != KVZAP_OK) return rc;
  // launch_mask splits its workspace at align_up(chunks * 4, 256) <= kStaticCountBytes
  return launch_mask(scores, tau, nullptr, window, seq_lens, B, H, T, keep_idx, lengths, offsets,
                     ws, stream);
}

}  // namespace kvzap
