// Fixed-budget thresholds on the surrogate scores (Sec. 3.3: a fixed fraction is what KVzip
// keeps; Sec. 4 ablation: fixed-ratio top-k per head, or per layer as in AdaKV).  For each
// group -- one head, or the H heads of one sequence pooled -- the k-th largest score among
// its non-window, non-NaN entries is found by a most-significant-digit radix select on the
// order-preserving 32-bit image of the floats: four passes of 256-bin histograms.  The
// result is a threshold per head for the mask kernels, which keep {score >= tau}: entries
// tied with the k-th largest are all kept.
//
// No pass needs the host or a select kernel in between: a block of pass p recomputes the
// digits chosen by passes 0..p-1 from their (complete) histograms, which takes p scans of
// 256 bins.
#include "kvzap_internal.h"

namespace kvzap {
namespace {

constexpr int kThreads = 256;
constexpr int kPerThread = 16;                            // scores per thread per block
constexpr int kChunk = kThreads * kPerThread;             // 4096 scores per block

// descending key: a larger score has a smaller key
__device__ __forceinline__ unsigned desc_key(float s) {
  const unsigned b = __float_as_uint(s);
  const unsigned asc = (b & 0x80000000u) ? ~b : (b | 0x80000000u);
  return ~asc;
}
__device__ __forceinline__ float key_to_float(unsigned dk) {
  const unsigned asc = ~dk;
  const unsigned b = (asc & 0x80000000u) ? (asc & 0x7FFFFFFFu) : ~asc;
  return __uint_as_float(b);
}

// Digits chosen by passes 0..p-1 for group g: prefix (the key's top 8p bits) and the rank
// still to find below it.  hist: [4][groups][256].  All 256 threads call this; returns via
// shared memory.  rank <= 0 on entry means k <= 0.
struct Chain {
  unsigned prefix;
  long long rank;      // 1-based rank inside the bucket `prefix`
  long long total;     // population of the group
};

__device__ Chain follow_chain(const unsigned* __restrict__ hist, int groups, int g, int passes,
                              long long k) {
  __shared__ long long s_cum[kThreads];
  __shared__ unsigned s_digit;
  __shared__ long long s_rank;
  __shared__ long long s_total;
  const int tid = threadIdx.x;
  Chain c;
  c.prefix = 0;
  c.rank = k;
  c.total = 0;
  for (int p = 0; p < passes; ++p) {
    const unsigned h = hist[((size_t)p * groups + g) * 256 + tid];
    s_cum[tid] = h;
    __syncthreads();
    for (int d = 1; d < kThreads; d <<= 1) {
      const long long add = tid >= d ? s_cum[tid - d] : 0;
      __syncthreads();
      s_cum[tid] += add;
      __syncthreads();
    }
    const long long cum = s_cum[tid];
    if (tid == 0) { s_digit = 255u; s_rank = 0; }
    if (tid == kThreads - 1 && p == 0) s_total = cum;
    __syncthreads();
    if (cum >= c.rank && cum - (long long)h < c.rank) {   // exactly one bin when 1 <= rank <= total
      s_digit = (unsigned)tid;
      s_rank = c.rank - (cum - (long long)h);
    }
    __syncthreads();
    if (p == 0) c.total = s_total;
    c.prefix = (c.prefix << 8) | s_digit;
    c.rank = s_rank;
    __syncthreads();
  }
  return c;
}

__global__ __launch_bounds__(kThreads) void topk_zero_kernel(unsigned* hist, size_t n) {
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += (size_t)gridDim.x * kThreads)
    hist[i] = 0u;
}

// grid (chunks, B*H).  Pass p adds, for the entries of this block whose key starts with the
// group's prefix, the next 8 bits to hist[p][group].
__global__ __launch_bounds__(kThreads) void topk_hist_kernel(
    const float* __restrict__ scores, int window, const int32_t* __restrict__ seq_lens, int H,
    int T, int per_layer, int groups, long long k, int pass, unsigned* __restrict__ hist) {
  __shared__ unsigned s_hist[256];
  const int bh = blockIdx.y, b = bh / H;
  const int g = per_layer ? b : bh;
  const int Tb = seq_lens ? seq_lens[b] : T;
  const int n_pop = Tb - window;                          // entries [0, n_pop) form the population
  const int t0 = blockIdx.x * kChunk;
  if (t0 >= n_pop) return;
  s_hist[threadIdx.x] = 0u;
  unsigned prefix = 0;
  if (pass > 0) {
    const Chain c = follow_chain(hist, groups, g, pass, k);
    if (k <= 0 || k > c.total) return;                    // threshold is +inf / -inf: nothing to refine
    prefix = c.prefix;
  }
  __syncthreads();
  const float* row = scores + (size_t)bh * T;
  const int shift = 24 - 8 * pass;
#pragma unroll 4
  for (int i = 0; i < kPerThread; ++i) {
    const int t = t0 + i * kThreads + threadIdx.x;
    if (t < n_pop) {
      const float s = row[t];
      if (s == s) {                                       // NaN is not part of the population
        const unsigned dk = desc_key(s);
        if (pass == 0 || (dk >> (shift + 8)) == prefix) atomicAdd(&s_hist[(dk >> shift) & 255u], 1u);
      }
    }
  }
  __syncthreads();
  const unsigned v = s_hist[threadIdx.x];
  if (v) atomicAdd(&hist[((size_t)pass * groups + g) * 256 + threadIdx.x], v);
}

// grid groups: the full key after four passes, as a float, for every head of the group
__global__ __launch_bounds__(kThreads) void topk_final_kernel(
    const unsigned* __restrict__ hist, int groups, int H, int per_layer, long long k,
    float* __restrict__ tau_out) {
  const int g = blockIdx.x;
  const Chain c = follow_chain(hist, groups, g, 4, k);
  float tau;
  if (k <= 0) tau = INFINITY;
  else if (k >= c.total) tau = -INFINITY;                 // also k == total: keep the whole population
  else tau = key_to_float(c.prefix);
  if (per_layer) {
    for (int h = threadIdx.x; h < H; h += kThreads) tau_out[(size_t)g * H + h] = tau;
  } else if (threadIdx.x == 0) {
    tau_out[g] = tau;
  }
}

}  // namespace

size_t topk_workspace_bytes(int B, int H, bool per_layer) {
  const size_t groups = per_layer ? (size_t)B : (size_t)B * H;
  return align_up(4 * groups * 256 * sizeof(unsigned), 256);
}

int launch_topk_threshold(const float* scores, int window, const int32_t* seq_lens, long long k,
                          bool per_layer, int B, int H, int T, float* tau_out, void* workspace,
                          hipStream_t stream) {
  const int groups = per_layer ? B : B * H;
  unsigned* hist = static_cast<unsigned*>(workspace);
  const size_t n = (size_t)4 * groups * 256;
  int zb = (int)((n + kThreads - 1) / kThreads);
  zb = zb < 1024 ? zb : 1024;
  topk_zero_kernel<<<zb, kThreads, 0, stream>>>(hist, n);
  const dim3 grid((T + kChunk - 1) / kChunk, B * H);
  for (int pass = 0; pass < 4; ++pass)
    topk_hist_kernel<<<grid, kThreads, 0, stream>>>(scores, window, seq_lens, H, T,
                                                    per_layer ? 1 : 0, groups, k, pass, hist);
  topk_final_kernel<<<groups, kThreads, 0, stream>>>(hist, groups, H, per_layer ? 1 : 0, k, tau_out);
  return hipGetLastError() == hipSuccess ? KVZAP_OK : KVZAP_ERR_RUNTIME;
}

}  // namespace kvzap
