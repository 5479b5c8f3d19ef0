// Fixed-budget thresholds on the surrogate scores (Sec. 3.3: a fixed fraction is what KVzip
// keeps; Sec. 4 ablation: fixed-ratio top-k per head, or per layer as in AdaKV).  For each
// group -- one head, or the H heads of one sequence pooled -- the k-th largest score among
// its non-window, non-NaN entries is found by a most-significant-digit radix select on the
// order-preserving 32-bit image of the floats, in three passes over the scores with digits
// of 8, 12 and 12 bits.  The result is a threshold per head for the mask kernels, which keep
// {score >= tau}: entries tied with the k-th largest are all kept.
//
// The stage is a handful of launches over a few megabytes, so the number of launches and
// the barriers inside them are what it costs:
//   * pass 0 writes one 256-bin histogram PER BLOCK with plain stores (every block writes
//     its slot, also an empty one), so nothing has to be zeroed before it; its first block
//     of each group zeroes the group's two 4096-bin histograms of the later passes;
//   * a block of pass p recomputes the digits chosen by the passes before it from their
//     (complete) histograms -- a sum over the group's pass-0 slots, then one block scan per
//     level with two barriers -- so no select kernel and no host step sits between passes;
//   * the last kernel follows the whole chain and writes the thresholds.
// No block waits for another.
#include "kvzap_internal.h"

namespace kvzap {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kTile = 4096;                               // scores per block and step
constexpr int kBins0 = 256;                               // key bits 31..24
constexpr int kBinsN = 4096;                              // key bits 23..12, then 11..0
constexpr int kMaxSlots = 128;                            // pass-0 histograms per group

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

// Workspace (32-bit words): slots [groups][nslot][256], then hist1 and hist2 [groups][4096].
struct Layout {
  int gx;          // blocks per (b,h) row
  int nslot;       // pass-0 histograms per group
};
inline Layout topk_layout(int H, int T, bool per_layer) {
  const int tiles = (T + kTile - 1) / kTile;
  const int cap = per_layer ? (kMaxSlots / H > 0 ? kMaxSlots / H : 1) : kMaxSlots;
  Layout l;
  l.gx = tiles < cap ? tiles : cap;
  l.nslot = l.gx * (per_layer ? H : 1);
  return l;
}

// The bin holding the rank-th entry (1-based, in bin order) of a histogram whose bins
// [tid*NPT, tid*NPT + NPT) are in v.  Every thread of the block calls it and gets the same
// answer: bin, the rank inside that bin, and the histogram's total.  If rank is outside
// [1, total] the bin is meaningless and the caller looks at total.
struct Pick {
  unsigned bin;
  long long rank;
  long long total;
};
template <int NPT>
__device__ Pick pick_bin(const unsigned (&v)[NPT], long long rank) {
  __shared__ long long s_wave[kWaves];
  __shared__ unsigned s_bin;
  __shared__ long long s_rank;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  long long mine = 0;
#pragma unroll
  for (int i = 0; i < NPT; ++i) mine += v[i];
  long long inc = mine;                                    // inclusive scan inside the wavefront
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const long long up = __shfl_up(inc, off, 64);
    if (lane >= off) inc += up;
  }
  __syncthreads();                                         // the previous call's results are consumed
  if (lane == 63) s_wave[wv] = inc;
  if (tid == 0) { s_bin = 0u; s_rank = 0; }
  __syncthreads();
  long long before = 0, total = 0;
#pragma unroll
  for (int x = 0; x < kWaves; ++x) {
    const long long t = s_wave[x];
    if (x < wv) before += t;
    total += t;
  }
  const long long ex = before + inc - mine;                // entries in bins before this thread's
  if (ex < rank && rank <= ex + mine) {                    // exactly one thread when 1 <= rank <= total
    long long r = rank - ex;
    unsigned b = 0;
#pragma unroll
    for (int i = 0; i < NPT; ++i) {
      if (r > (long long)v[i] && i < NPT - 1 && b == (unsigned)i) { r -= v[i]; b = i + 1; }
    }
    s_bin = (unsigned)tid * NPT + b;
    s_rank = r;
  }
  __syncthreads();
  Pick p;
  p.bin = s_bin;
  p.rank = s_rank;
  p.total = total;
  return p;
}

// Digits chosen by the first `levels` passes for group g: the key's leading bits and the
// rank still to find below them.  ok == false: k is outside [1, population].
struct Chain {
  unsigned prefix;
  long long rank;
  long long total;
  bool ok;
};
__device__ Chain follow_chain(const unsigned* __restrict__ ws, int groups, int nslot, int g,
                              int levels, long long k) {
  __shared__ u32x4 s_part[kWaves][kBins0 / 4];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const u32x4* slots = reinterpret_cast<const u32x4*>(ws + (size_t)g * nslot * kBins0);
  const unsigned* hist1 = ws + (size_t)groups * nslot * kBins0 + (size_t)g * kBinsN;
  const unsigned* hist2 = hist1 + (size_t)groups * kBinsN;
  constexpr int NPT = kBinsN / kThreads;
  // every load of the chain is issued before the first barrier: the later levels' bins (their
  // addresses do not depend on the earlier picks), then the pass-0 slots, four bins per lane,
  // the slots dealt round-robin to the wavefronts and read eight at a time
  u32x4 h1[NPT / 4], h2[NPT / 4];
  if (levels >= 2) {
#pragma unroll
    for (int i = 0; i < NPT / 4; ++i) h1[i] = reinterpret_cast<const u32x4*>(hist1 + tid * NPT)[i];
  }
  if (levels >= 3) {
#pragma unroll
    for (int i = 0; i < NPT / 4; ++i) h2[i] = reinterpret_cast<const u32x4*>(hist2 + tid * NPT)[i];
  }
  u32x4 acc = {0u, 0u, 0u, 0u};
  for (int s0 = wv; s0 < nslot; s0 += kWaves * 8) {
    u32x4 q[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int ss = s0 + kWaves * u;
      q[u] = slots[(size_t)(ss < nslot ? ss : nslot - 1) * (kBins0 / 4) + lane];
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const unsigned on = (s0 + kWaves * u < nslot) ? 0xffffffffu : 0u;
      acc.x += q[u].x & on; acc.y += q[u].y & on; acc.z += q[u].z & on; acc.w += q[u].w & on;
    }
  }
  __syncthreads();                                         // an earlier call's s_part is consumed
  s_part[wv][lane] = acc;
  __syncthreads();
  unsigned v0[1];
  {
    const unsigned* flat = reinterpret_cast<const unsigned*>(&s_part[0][0]);
    unsigned t = 0;
#pragma unroll
    for (int x = 0; x < kWaves; ++x) t += flat[x * kBins0 + tid];
    v0[0] = t;
  }
  Chain c;
  const Pick p0 = pick_bin<1>(v0, k);
  c.total = p0.total;
  c.ok = k >= 1 && k <= p0.total;
  c.prefix = p0.bin;
  c.rank = p0.rank;
  if (!c.ok || levels < 2) return c;                       // uniform over the block
  unsigned v[NPT];
#pragma unroll
  for (int i = 0; i < NPT / 4; ++i) {
    v[4 * i] = h1[i].x; v[4 * i + 1] = h1[i].y; v[4 * i + 2] = h1[i].z; v[4 * i + 3] = h1[i].w;
  }
  const Pick p1 = pick_bin<NPT>(v, c.rank);
  c.prefix = (c.prefix << 12) | p1.bin;
  c.rank = p1.rank;
  if (levels < 3) return c;
#pragma unroll
  for (int i = 0; i < NPT / 4; ++i) {
    v[4 * i] = h2[i].x; v[4 * i + 1] = h2[i].y; v[4 * i + 2] = h2[i].z; v[4 * i + 3] = h2[i].w;
  }
  const Pick p2 = pick_bin<NPT>(v, c.rank);
  c.prefix = (c.prefix << 12) | p2.bin;
  c.rank = p2.rank;
  return c;
}

// The 16 scores of this thread in tile `tile` of the row, as keys, with a validity mask
// (inside the population and not NaN).  kVec: rows are 16-byte aligned (T % 4 == 0) and the
// thread reads four float4; otherwise 16 strided scalars.  Out-of-range elements re-read an
// in-range address and are masked.
template <bool kVec>
__device__ __forceinline__ unsigned load_keys(const float* __restrict__ row, int tile, int T,
                                              int n_pop, unsigned (&key)[16]) {
  const int tid = threadIdx.x;
  unsigned valid = 0;
  if (kVec) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int t = tile * kTile + i * (kThreads * 4) + tid * 4;
      const int tc = t <= T - 4 ? t : T - 4;
      const floatx4 q = *reinterpret_cast<const floatx4*>(row + tc);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float s = q[e];
        key[4 * i + e] = desc_key(s);
        if (t + e < n_pop && s == s) valid |= 1u << (4 * i + e);
      }
    }
  } else {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int t = tile * kTile + i * kThreads + tid;
      const float s = row[t < T ? t : T - 1];
      key[i] = desc_key(s);
      if (t < n_pop && s == s) valid |= 1u << i;
    }
  }
  return valid;
}

// grid (gx, B*H).  Pass 0: the histogram of the keys' top 8 bits over this block's tiles,
// stored to the block's own slot.
template <bool kVec>
__global__ __launch_bounds__(kThreads) void topk_first_kernel(
    const float* __restrict__ scores, int window, const int32_t* __restrict__ seq_lens, int H,
    int T, int per_layer, int groups, int nslot, unsigned* __restrict__ ws) {
  __shared__ unsigned s_hist[kWaves][kBins0];              // a copy per wavefront: fewer collisions
  const int tid = threadIdx.x, wv = tid >> 6;
  const int bh = blockIdx.y, b = bh / H, gx = gridDim.x;
  const int g = per_layer ? b : bh;
  const int slot = per_layer ? (bh - b * H) * gx + blockIdx.x : blockIdx.x;
  const int Tb = seq_lens ? (seq_lens[b] < T ? seq_lens[b] : T) : T;
  const int n_pop = Tb - window;                          // entries [0, n_pop) form the population
#pragma unroll
  for (int x = 0; x < kWaves; ++x) s_hist[x][tid] = 0u;
  if (slot == 0) {                                        // the group's later histograms start at zero
    u32x4* z = reinterpret_cast<u32x4*>(ws + (size_t)groups * nslot * kBins0 + (size_t)g * kBinsN);
    const u32x4 zero = {0u, 0u, 0u, 0u};
    for (int i = tid; i < kBinsN / 4; i += kThreads) {
      z[i] = zero;
      z[(size_t)groups * kBinsN / 4 + i] = zero;
    }
  }
  __syncthreads();
  const float* row = scores + (size_t)bh * T;
  const int tiles = (T + kTile - 1) / kTile;
  for (int tile = blockIdx.x; tile < tiles && tile * kTile < n_pop; tile += gx) {
    unsigned key[16];
    const unsigned valid = load_keys<kVec>(row, tile, T, n_pop, key);
#pragma unroll
    for (int i = 0; i < 16; ++i)
      if (valid >> i & 1u) atomicAdd(&s_hist[wv][key[i] >> 24], 1u);
  }
  __syncthreads();
  unsigned v = 0;
#pragma unroll
  for (int x = 0; x < kWaves; ++x) v += s_hist[x][tid];
  ws[((size_t)g * nslot + slot) * kBins0 + tid] = v;
}

// Passes 1 and 2: among the entries whose key starts with the group's prefix, the histogram
// of the next 12 bits, added to the group's histogram of that pass.
template <bool kVec>
__global__ __launch_bounds__(kThreads) void topk_refine_kernel(
    const float* __restrict__ scores, int window, const int32_t* __restrict__ seq_lens, int H,
    int T, int per_layer, int groups, int nslot, long long k, int pass, unsigned* __restrict__ ws) {
  __shared__ unsigned s_hist[kBinsN];
  const int tid = threadIdx.x;
  const int bh = blockIdx.y, b = bh / H, gx = gridDim.x;
  const int g = per_layer ? b : bh;
  const int Tb = seq_lens ? (seq_lens[b] < T ? seq_lens[b] : T) : T;
  const int n_pop = Tb - window;
  if ((int)blockIdx.x * kTile >= n_pop) return;           // uniform: no entry of the population here
  // the first tile's scores are on their way while the chain is followed
  const float* row = scores + (size_t)bh * T;
  unsigned key[16];
  unsigned valid = load_keys<kVec>(row, blockIdx.x, T, n_pop, key);
  for (int i = tid; i < kBinsN; i += kThreads) s_hist[i] = 0u;
  const Chain c = follow_chain(ws, groups, nslot, g, pass, k);   // its barriers also cover s_hist
  if (!c.ok) return;                                      // threshold is +inf / -inf: nothing to refine
  const int tiles = (T + kTile - 1) / kTile;
  const int shift = pass == 1 ? 12 : 0;                   // this pass's digit; the prefix is above it
  for (int tile = blockIdx.x; tile < tiles && tile * kTile < n_pop; tile += gx) {
    if (tile != (int)blockIdx.x) valid = load_keys<kVec>(row, tile, T, n_pop, key);
#pragma unroll
    for (int i = 0; i < 16; ++i)
      if ((valid >> i & 1u) && (key[i] >> (shift + 12)) == c.prefix)
        atomicAdd(&s_hist[(key[i] >> shift) & (kBinsN - 1)], 1u);
  }
  __syncthreads();
  unsigned* hist = ws + (size_t)groups * nslot * kBins0 + (size_t)(pass - 1) * groups * kBinsN +
                   (size_t)g * kBinsN;
  for (int i = tid; i < kBinsN; i += kThreads) {
    const unsigned v = s_hist[i];
    if (v) atomicAdd(&hist[i], v);
  }
}

// grid groups: the full key after the three passes, as a float, for every head of the group
__global__ __launch_bounds__(kThreads) void topk_final_kernel(
    const unsigned* __restrict__ ws, int groups, int nslot, int H, int per_layer, long long k,
    float* __restrict__ tau_out) {
  const int g = blockIdx.x;
  const Chain c = follow_chain(ws, groups, nslot, g, 3, k);
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

size_t topk_workspace_bytes(int B, int H, int T, bool per_layer) {
  if (B <= 0 || H <= 0 || T <= 0) return 0;
  const size_t groups = per_layer ? (size_t)B : (size_t)B * H;
  const Layout l = topk_layout(H, T, per_layer);
  return align_up((groups * l.nslot * kBins0 + 2 * groups * kBinsN) * sizeof(unsigned), 256);
}

int launch_topk_threshold(const float* scores, int window, const int32_t* seq_lens, long long k,
                          bool per_layer, int B, int H, int T, float* tau_out, void* workspace,
                          hipStream_t stream) {
  const int groups = per_layer ? B : B * H;
  const Layout l = topk_layout(H, T, per_layer);
  unsigned* ws = static_cast<unsigned*>(workspace);
  const dim3 grid(l.gx, B * H);
  const int pl = per_layer ? 1 : 0;
  if (T % 4 == 0) {
    topk_first_kernel<true><<<grid, kThreads, 0, stream>>>(scores, window, seq_lens, H, T, pl, groups, l.nslot, ws);
    for (int pass = 1; pass <= 2; ++pass)
      topk_refine_kernel<true><<<grid, kThreads, 0, stream>>>(scores, window, seq_lens, H, T, pl, groups, l.nslot, k, pass, ws);
  } else {
    topk_first_kernel<false><<<grid, kThreads, 0, stream>>>(scores, window, seq_lens, H, T, pl, groups, l.nslot, ws);
    for (int pass = 1; pass <= 2; ++pass)
      topk_refine_kernel<false><<<grid, kThreads, 0, stream>>>(scores, window, seq_lens, H, T, pl, groups, l.nslot, k, pass, ws);
  }
  topk_final_kernel<<<groups, kThreads, 0, stream>>>(ws, groups, l.nslot, H, pl, k, tau_out);
  return hipGetLastError() == hipSuccess ? KVZAP_OK : KVZAP_ERR_RUNTIME;
}

}  // namespace kvzap
