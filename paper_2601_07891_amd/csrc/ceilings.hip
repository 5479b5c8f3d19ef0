// kvzap_ceilings: measures, on the GPU it runs on, the practical ceilings the prune-step
// kernels are compared with, next to the published peaks (HBM 8 TB/s, bf16 MFMA 2.5 PFLOP/s):
//   1. sustained v_mfma_f32_32x32x16_bf16 rate from registers for constant, random-mantissa
//      and normally distributed operands, with few and with many operand registers (the more
//      the data toggles the datapath, the lower the clock the part sustains);
//   2. HBM read-stream bandwidth (16-byte loads, 1.25 GiB);
//   3. HBM copy bandwidth (read + write, 2 x 0.5 GiB).
// Stand-alone host program: `kvzap_ceilings` prints one line per measurement.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <vector>

#define CK(x)                                                                              \
  do {                                                                                     \
    hipError_t e_ = (x);                                                                   \
    if (e_ != hipSuccess) {                                                                \
      std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);           \
      std::exit(1);                                                                        \
    }                                                                                      \
  } while (0)

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

// MODE 0: one constant bit pattern; 1: random sign and mantissa, exponent of 1.0; 2: roughly
// normal values (sum of four uniform bytes), i.e. varying exponents too, as real activations
// and weights have.  NA x NB operand registers are cycled through: with 4 x 4 every MFMA of an
// iteration repeats the operands of the previous iteration, with 16 x 8 (what one K tile of the
// scorer holds) the datapath sees new values every time.
__device__ __forceinline__ unsigned next_rand(unsigned& x) { x ^= x << 13; x ^= x >> 17; x ^= x << 5; return x; }

__device__ __forceinline__ unsigned normal_bf16(unsigned& x) {
  const unsigned r = next_rand(x);
  const float f = ((r & 255) + ((r >> 8) & 255) + ((r >> 16) & 255) + ((r >> 24) & 255) - 510.f) * (1.f / 147.8f);
  return __float_as_uint(f) >> 16;
}

template <int MODE, int N>
__device__ __forceinline__ void fill_operands(bf16x8* v, unsigned seed) {
  for (int i = 0; i < N; ++i) {
    unsigned x = (threadIdx.x * 2654435761u) ^ (seed + i * 977u) ^ (blockIdx.x * 40503u) ^ 0x9e3779b9u;
    u32x4 w;
    for (int e = 0; e < 4; ++e) {
      if (MODE == 0) {
        w[e] = 0x12345678u & 0x807f807fu | 0x3f003f00u;
      } else if (MODE == 1) {
        const unsigned r = next_rand(x);
        w[e] = (r & 0x807f807fu) | 0x3f003f00u | ((r >> 3) & 0x00800080u);
      } else {
        const unsigned lo = normal_bf16(x), hi = normal_bf16(x);
        w[e] = lo | (hi << 16);
      }
    }
    v[i] = __builtin_bit_cast(bf16x8, w);
  }
}

template <int MODE, int NA, int NB>
__global__ __launch_bounds__(256) void mfma_rate_kernel(float* out, int iters, unsigned seed) {
  floatx16 acc[16];
  for (int i = 0; i < 16; ++i)
    for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
  bf16x8 a[NA], b[NB];
  fill_operands<MODE, NA>(a, seed);
  fill_operands<MODE, NB>(b, seed + 12345u);
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int r = 0; r < NA / 4; ++r)
#pragma unroll
      for (int i = 0; i < 16; ++i)
        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(i & 3) + 4 * r], b[(i >> 2) + 4 * (r % (NB / 4))],
                                                         acc[i], 0, 0, 0);
  }
  float s = 0;
  for (int i = 0; i < 16; ++i)
    for (int e = 0; e < 16; ++e) s += acc[i][e];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

__global__ __launch_bounds__(256) void read_stream_kernel(const u32x4* __restrict__ a,
                                                          unsigned* out, size_t n) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t st = (size_t)gridDim.x * 256;
  unsigned acc = 0;
  for (; i + 7 * st < n; i += 8 * st) {
    u32x4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(a + i + u * st);
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u].x ^ v[u].w;
  }
  for (; i < n; i += st) acc ^= a[i].x;
  if (acc == 0x12345u) out[0] = acc;
}

__global__ __launch_bounds__(256) void copy_kernel(const u32x4* __restrict__ a,
                                                   u32x4* __restrict__ b, size_t n) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t st = (size_t)gridDim.x * 256;
  for (; i + 3 * st < n; i += 4 * st) {
    const u32x4 v0 = __builtin_nontemporal_load(a + i), v1 = __builtin_nontemporal_load(a + i + st),
                v2 = __builtin_nontemporal_load(a + i + 2 * st),
                v3 = __builtin_nontemporal_load(a + i + 3 * st);
    __builtin_nontemporal_store(v0, b + i);
    __builtin_nontemporal_store(v1, b + i + st);
    __builtin_nontemporal_store(v2, b + i + 2 * st);
    __builtin_nontemporal_store(v3, b + i + 3 * st);
  }
  for (; i < n; i += st) b[i] = a[i];
}

template <class F>
static float median_ms(F f, int reps) {
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0));
  CK(hipEventCreate(&e1));
  for (int i = 0; i < 3; ++i) f(i);
  CK(hipDeviceSynchronize());
  std::vector<float> v;
  for (int r = 0; r < reps; ++r) {
    CK(hipEventRecord(e0));
    f(r);
    CK(hipEventRecord(e1));
    CK(hipEventSynchronize(e1));
    float ms;
    CK(hipEventElapsedTime(&ms, e0, e1));
    v.push_back(ms);
  }
  std::sort(v.begin(), v.end());
  return v[v.size() / 2];
}

int main() {
  float* out;
  CK(hipMalloc(&out, 1024 * 256 * sizeof(float)));
  // ~0.3 s per launch: long enough for the clock to settle at what the power draw allows
  const int iters = 256;
  const double flops = 1024.0 * 4 * iters * 16 * 32768.0;
  for (int w = 0; w < 6; ++w) mfma_rate_kernel<2, 4, 4><<<1024, 256>>>(out, iters, 7u + w);   // clocks settle
  CK(hipDeviceSynchronize());
  float t = median_ms([&](int r) { mfma_rate_kernel<0, 4, 4><<<1024, 256>>>(out, iters, 999u + r); }, 5);
  std::printf("mfma_bf16_32x32x16 constant operands, 4x4 registers:          %.0f TFLOP/s\n", flops / t / 1e9);
  t = median_ms([&](int r) { mfma_rate_kernel<1, 4, 4><<<1024, 256>>>(out, iters, 999u + r); }, 5);
  std::printf("mfma_bf16_32x32x16 random mantissas, 4x4 registers:           %.0f TFLOP/s\n", flops / t / 1e9);
  t = median_ms([&](int r) { mfma_rate_kernel<2, 4, 4><<<1024, 256>>>(out, iters, 999u + r); }, 5);
  std::printf("mfma_bf16_32x32x16 normal values, 4x4 registers:              %.0f TFLOP/s\n", flops / t / 1e9);
  t = median_ms([&](int r) { mfma_rate_kernel<2, 16, 8><<<1024, 256>>>(out, iters / 4, 999u + r); }, 5);
  std::printf("mfma_bf16_32x32x16 normal values, 16x8 registers (a K tile):   %.0f TFLOP/s\n", flops / t / 1e9);

  const size_t bytes = (size_t)1280 << 20, n = bytes / 16;
  u32x4 *a, *b;
  unsigned* flag;
  CK(hipMalloc(&a, bytes));
  CK(hipMalloc(&b, bytes));
  CK(hipMalloc(&flag, 64));
  CK(hipMemset(a, 1, bytes));
  CK(hipMemset(b, 2, bytes));
  t = median_ms([&](int r) { read_stream_kernel<<<8192, 256>>>((r & 1) ? a : b, flag, n); }, 10);
  std::printf("hbm read stream (1.25 GiB):            %.2f TB/s\n", bytes / t / 1e9);
  const size_t half = n / 2;   // copy 0.625 GiB -> 0.625 GiB inside distinct buffers
  t = median_ms([&](int r) { copy_kernel<<<8192, 256>>>(a + (r & 1) * half, b + (r & 1) * half, half); }, 10);
  std::printf("hbm copy (0.625 GiB read + write):     %.2f TB/s\n", 2.0 * half * 16 / t / 1e9);
  return hipDeviceSynchronize() == hipSuccess ? 0 : 1;
}
