// Internal declarations shared by the host API and the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "kvzap.h"

namespace kvzap {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

// tokens handled by one block of the mask kernels
constexpr int kMaskChunk = 1024;

inline int mask_chunks(int T) { return (T + kMaskChunk - 1) / kMaskChunk; }

// chunks (of all heads together) the built-in scratch of kvzap_mask_static has room for
constexpr int kStaticMaskChunks = KVZAP_MASK_STATIC_MAX_CHUNKS;

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// bf16 bit pattern -> fp32 (exact)
__device__ __forceinline__ float bf16_bits_to_float(unsigned short b) {
  return __uint_as_float(((unsigned int)b) << 16);
}

// fp32 -> bf16 bit pattern, round to nearest even (finite inputs)
__device__ __forceinline__ unsigned short float_to_bf16_bits(float f) {
  unsigned int u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (unsigned short)(u >> 16);
}

// ---- asynchronous global -> LDS loads with hand-counted completion ----
// Wait until at most N vector-memory operations of this wavefront are outstanding
// (they complete in issue order).  Written as asm with a memory clobber so that the
// compiler keeps every load that precedes it in the source before it.
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Workgroup barrier that does NOT wait for outstanding vector-memory traffic (a
// __syncthreads() would drain the prefetched tiles).  The caller has already
// waited for the loads it needs; every LDS read issued before this point has been
// consumed by an MFMA, so it has completed.  The "memory" clobber keeps the
// compiler from moving LDS accesses across it.
__device__ __forceinline__ void block_barrier_no_drain() {
  asm volatile("s_barrier" ::: "memory");
}

// One load-to-LDS instruction: every lane fetches 16 bytes from its own global address and
// the wavefront's 64 pieces land at LDS bytes [lds_base, lds_base + 1024) in lane order.
// Issued as inline asm on purpose: the compiler tracks the builtin form as an LDS write
// that may alias every later LDS read and then waits for ALL outstanding vector-memory
// operations before those reads, which would undo the multi-tile prefetch.  Completion is
// tracked by hand with wait_vmcnt(); the compiler's own vmcnt waits (for ordinary loads)
// do not know about these operations and therefore only ever wait longer, never shorter.
// M0 (the LDS base of the instruction) is written here and used nowhere else in the kernel.
__device__ __forceinline__ void load_to_lds_b128(const void* gptr, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
               ::"s"(lds_base), "v"(gptr)
               : "memory");
}

// The same with the non-temporal hint: for data that is read once (streamed), so that it
// does not push re-used lines out of the L2.
__device__ __forceinline__ void load_to_lds_b128_stream(const void* gptr, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off nt"
               ::"s"(lds_base), "v"(gptr)
               : "memory");
}

// ... and with the address as a uniform 64-bit base (scalar registers) plus a 32-bit offset per
// lane: no 64-bit vector add per instruction when only the base moves from tile to tile.
__device__ __forceinline__ void load_to_lds_b128_stream(const void* base, unsigned lane_offset,
                                                        unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 nt"
               ::"s"(lds_base), "v"(lane_offset), "s"(base)
               : "memory");
}

__device__ __forceinline__ unsigned lds_address(const void* p) {
  return (unsigned)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}

// The 4-byte form: lane i's dword lands at LDS byte lds_base + 4*i.
__device__ __forceinline__ void load_to_lds_b32(const void* gptr, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off"
               ::"s"(lds_base), "v"(gptr)
               : "memory");
}

// launchers (each returns a kvzap_status); arguments are already validated
int launch_mask(const float* scores, float tau, const float* tau_head, int window,
                const int32_t* seq_lens, int B, int H, int T, int32_t* keep_idx,
                int32_t* lengths, int64_t* offsets, void* workspace, hipStream_t stream);

// kvzap_mask on the library's own scratch (no workspace, nothing allocated)
int launch_mask_static(const float* scores, float tau, int window, const int32_t* seq_lens, int B,
                       int H, int T, int32_t* keep_idx, int32_t* lengths, int64_t* offsets,
                       hipStream_t stream);

int launch_topk_threshold(const float* scores, int window, const int32_t* seq_lens, long long k,
                          bool per_layer, int B, int H, int T, float* tau_out, void* workspace,
                          hipStream_t stream);
size_t topk_workspace_bytes(int B, int H, int T, bool per_layer);

int launch_teacher_scores(const void* q, const void* k, const float* vnorm, const float* hnorm,
                          float scale, float* log_s, int H, int HQ, int Tq, int Tk, int T,
                          void* workspace, hipStream_t stream);
size_t teacher_workspace_bytes(int H, int HQ, int Tq, int T);

int launch_compact(const void* K, const void* V, const int32_t* keep_idx,
                   const int32_t* lengths, const int64_t* offsets, void* K_out,
                   void* V_out, int64_t cap_rows, int BH, int T, int D,
                   hipStream_t stream);

int launch_score_linear(const void* hidden, const void* W, const void* b, float* scores,
                        int B, int T, int Dh, int H, hipStream_t stream);

int skinny_ksplit(long long rows, int Dh, int M, int target_blocks);
int launch_skinny_gemm(const void* hidden, const void* W1, float* partial, long long rows, int Dh,
                       int M, int ks, hipStream_t stream);
// bytes kvzap_score's workspace needs for an MLP surrogate on `rows` tokens
size_t score_mlp_workspace_bytes(long long rows, int Dh, int M);
// gain (optional): the prepared copy holds W1 * diag(gain), for launch_score_mlp_rmsnorm
int launch_prepare_w1(const void* W1, const void* gain, int Dh, int M, void* out, hipStream_t stream);
// the MLP surrogate on the un-normalised residual stream (single-kernel path only)
bool score_rmsnorm_supports(int Dh);
int launch_score_mlp_rmsnorm(const void* x, const void* W1_prepared, const void* gain, float eps,
                             const void* b1, const void* W2, const void* b2, float* scores,
                             float* rstd, void* normed, int B, int T, int Dh, int M, int H,
                             hipStream_t stream);
// workspace == nullptr: W1 is the copy made by launch_prepare_w1
int launch_score_mlp(const void* hidden, const void* W1, const void* b1, const void* W2,
                     const void* b2, float* scores, int B, int T, int Dh, int M, int H,
                     void* workspace, hipStream_t stream);

struct DecodeArgs {
  const void* hidden_new; const void* W1; const void* b1; const void* W2; const void* b2;
  int Dh, M;
  const void* k_new; const void* v_new;
  void* K_prefix; void* V_prefix; int32_t* prefix_pos;
  const int64_t* slab_offsets; const int32_t* slab_capacity;
  void* K_ring; void* V_ring; float* score_ring;
  int32_t* lengths; int32_t* seq_pos;
  float tau; int window, B, H, D;
  int32_t* error_flag;
  void* workspace;
  // paged prefix (block_table != nullptr): K_prefix / V_prefix / prefix_pos are the pools,
  // slab_offsets / slab_capacity are unused
  const int32_t* block_table;
  int max_pages, log_page, num_pages;
};
int launch_decode_evict(const DecodeArgs& a, hipStream_t stream);
size_t decode_workspace_bytes(int B, int Dh, int M, int H);

int launch_attend_decode(const void* q, const void* K_rows, const void* V_rows,
                         int64_t total_rows, const int64_t* row_offsets,
                         const int32_t* block_table, int max_pages, int page_rows, int num_pages,
                         const int32_t* lengths, const void* K_ring, const void* V_ring,
                         const int32_t* seq_pos, int window, int max_rows, float scale,
                         void* out, int B, int H, int HQ, void* workspace,
                         hipStream_t stream);
int launch_assign_pages(const int32_t* lengths, int32_t* page_counts, int BH, int page_rows,
                        int reserve_rows, const int32_t* free_pages, int n_free,
                        int32_t* block_table, int max_pages, int32_t* result, void* workspace,
                        hipStream_t stream);
size_t assign_pages_workspace_bytes(int BH);
int launch_compact_paged(const void* K, const void* V, const int32_t* keep_idx,
                         const int32_t* lengths, const int64_t* offsets,
                         const int32_t* block_table, int max_pages, int page_rows, void* K_pool,
                         void* V_pool, int num_pages, int BH, int T, int D, hipStream_t stream);
size_t attend_workspace_bytes(int B, int H, int HQ, int max_rows, int window);

}  // namespace kvzap
