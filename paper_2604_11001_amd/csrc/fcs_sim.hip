// Sample-path kernel: one wavefront (= one workgroup) simulates one path of the slot
// model (Section 2.1) under Algorithm 2 or its greedy limit, for slots 1..T.
//
// Data layout per path
//   active set   slots in activation order; requests that left stay behind as dead slots until an
//                order-preserving compaction removes them (once kCompactSlack have accumulated).
//                Slots [0, lcap) live in LDS, slots [lcap, lcap+hcap) in a per-path spill region
//                of the workspace.  Per slot:
//                  END    while decoding: the slot in which the request generates its last
//                         token if no token budget ever binds; -1 while prefilling or unused.
//                         An entry in [0, current slot) belongs to a request that completed in
//                         that slot and has not been accounted yet: latency statistics are
//                         taken when the dead slot is removed, for 64 slots at a time.
//                         The decode growth of a slot (Section 2.1: one more token per active
//                         request) therefore costs nothing per request: U grows by the number
//                         of decoding requests, and the entries are only looked at in slots
//                         for which the calendar (a bit per slot of the current 64-slot
//                         window, a superset of the slots with a completion) says so.  A slot
//                         whose budget binds moves the entries of the stalled requests by one.
//                  FOOT   l + o, what the request releases when it completes (LDS only, next
//                         to END: the two are read together)
//                  PLEFT  prompt tokens still to prefill; meaningful while END is -1 (0 = unused).  Once the
//                         request decodes the word means nothing to anybody but the slot loop, whose
//                         general prefill pass leaves -t there when the prompt ended in slot t (the
//                         stall pass of that slot reads it)
//                  REC    {l, o, arrival slot, id}
//   waiting queue  requests that were never activated are not stored: arrivals are a pure
//                function of (seed, replica, slot, index), so the FIFO of fresh requests is
//                re-generated 64 arrivals at a time when they are admitted.  Evicted requests
//                re-enter at the front of Q, newest eviction deepest: a stack (first
//                entries in LDS, the rest in the spill region).
//   scalars      U, |P|, cursors and counts are wave-uniform and stay in scalar registers;
//                statistics accumulate in lanes of a few vector registers.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "fcs_internal.h"

namespace fcs {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t& r0, uint32_t& r1,
                                              uint32_t& r2, uint32_t& r3) {
  constexpr uint32_t kMulA = 0xD2511F53u, kMulB = 0xCD9E8D57u;
  constexpr uint32_t kWeylA = 0x9E3779B9u, kWeylB = 0xBB67AE85u;
#pragma unroll
  for (int i = 0; i < 10; ++i) {
    const uint32_t a_hi = __umulhi(kMulA, c0), a_lo = kMulA * c0;
    const uint32_t b_hi = __umulhi(kMulB, c2), b_lo = kMulB * c2;
    const uint32_t x0 = b_hi ^ c1 ^ k0;
    const uint32_t x2 = a_hi ^ c3 ^ k1;
    c0 = x0;
    c1 = b_lo;
    c2 = x2;
    c3 = a_lo;
    k0 += kWeylA;
    k1 += kWeylB;
  }
  r0 = c0; r1 = c1; r2 = c2; r3 = c3;
}

__device__ __forceinline__ int rfl(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ int rdl(int v, int l) { return __builtin_amdgcn_readlane(v, l); }
// lane `l` (a constant) of v takes the wave-uniform value s
// (kPin: the compiler may hold s in a vector register; take its first lane)
template <int l, bool kPin>
__device__ __forceinline__ int wrl_c(int s, int v) {
  if (kPin) s = rfl(s);
  asm("v_writelane_b32 %0, %1, %2" : "+v"(v) : "s"(s), "n"(l));
  return v;
}
#define wrl(s, l, v) wrl_c<l, FCS_ALL_POLICIES != 0>((s), (v))

// Lanes of the wavefront exchange data through LDS and the spill region (lane 0 writes a slot
// that lane k reads later).  To the compiler each lane is a separate thread, so every such
// hand-over needs a wavefront-scope release/acquire; the hardware executes the memory
// operations of one wavefront in order, so this emits no instruction.
__device__ __forceinline__ void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Wavefront scans and reductions of non-negative values with DPP (row shifts inside the rows of 16
// lanes, then the last lane of a row broadcast to the rows after it); zero is the fill value and the
// identity of all three operations.
#define FCS_DPP(v, ctrl, row_mask) __builtin_amdgcn_update_dpp(0, (v), (ctrl), (row_mask), 0xf, false)
enum { DPP_ROW_SHR1 = 0x111, DPP_ROW_SHR2 = 0x112, DPP_ROW_SHR4 = 0x114, DPP_ROW_SHR8 = 0x118,
       DPP_ROW_BCAST15 = 0x142, DPP_ROW_BCAST31 = 0x143 };

__device__ __forceinline__ int wave_incl_sum(int v) {
  v += FCS_DPP(v, DPP_ROW_SHR1, 0xf);
  v += FCS_DPP(v, DPP_ROW_SHR2, 0xf);
  v += FCS_DPP(v, DPP_ROW_SHR4, 0xf);
  v += FCS_DPP(v, DPP_ROW_SHR8, 0xf);
  v += FCS_DPP(v, DPP_ROW_BCAST15, 0xa);
  v += FCS_DPP(v, DPP_ROW_BCAST31, 0xc);
  return v;
}

__device__ __forceinline__ int wave_incl_max(int v) {
  v = max(v, FCS_DPP(v, DPP_ROW_SHR1, 0xf));
  v = max(v, FCS_DPP(v, DPP_ROW_SHR2, 0xf));
  v = max(v, FCS_DPP(v, DPP_ROW_SHR4, 0xf));
  v = max(v, FCS_DPP(v, DPP_ROW_SHR8, 0xf));
  v = max(v, FCS_DPP(v, DPP_ROW_BCAST15, 0xa));
  v = max(v, FCS_DPP(v, DPP_ROW_BCAST31, 0xc));
  return v;
}

// OR over the wavefront, valid in lane 63 (returned from there)
__device__ __forceinline__ uint32_t wave_or(uint32_t u) {
  int v = static_cast<int>(u);
  v |= FCS_DPP(v, DPP_ROW_SHR1, 0xf);
  v |= FCS_DPP(v, DPP_ROW_SHR2, 0xf);
  v |= FCS_DPP(v, DPP_ROW_SHR4, 0xf);
  v |= FCS_DPP(v, DPP_ROW_SHR8, 0xf);
  v |= FCS_DPP(v, DPP_ROW_BCAST15, 0xa);
  v |= FCS_DPP(v, DPP_ROW_BCAST31, 0xc);
  return static_cast<uint32_t>(__builtin_amdgcn_readlane(v, kWave - 1));
}

__device__ __forceinline__ int lanes_below(uint64_t mask) {
  return __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(mask >> 32),
                                   __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(mask), 0u));
}

#define LIKELY(c) __builtin_expect(!!(c), 1)
#define UNLIKELY(c) __builtin_expect(!!(c), 0)

// 16-byte LDS / global accesses of four consecutive words (addresses are multiples of four words)
__device__ __forceinline__ v4i ld4(const int32_t* p) {
  return *reinterpret_cast<const v4i*>(__builtin_assume_aligned(p, 16));
}
__device__ __forceinline__ void st4(int32_t* p, v4i v) {
  *reinterpret_cast<v4i*>(__builtin_assume_aligned(p, 16)) = v;
}

// lanes of the per-slot statistics vector
enum { SL_SUM_U = 0, SL_SUM_P, SL_SUM_Q, SL_DEC_TOK, SL_ACT, SL_DONE, SL_EVICT, SL_OVF, SL_PF_TOK,
       SL_STALLED, SL_COUNT };

// The kernel of the FLOW and GREEDY cells is held to 128 vector registers, so that four wavefronts fit a
// SIMD (the fixed registers of the assembly loop are v84-v127): with 256 LDS slots per path a compute unit
// then holds 16 paths, which is what hides the latencies of a path's instruction chain best.
#define FCS_ALL_POLICIES 0
#define FCS_MC_KNOWN 0
#define FCS_SKIP_IDLE 0
#define FCS_KERNEL fcs_sim_kernel
#define FCS_KERNEL_ATTR __attribute__((amdgpu_waves_per_eu(4, 4)))
#include "fcs_sim_kernel.inc"
#undef FCS_KERNEL
#undef FCS_SKIP_IDLE

// the same with event skipping in the slot loop (FCS_FLAG_SKIP_IDLE)
#define FCS_SKIP_IDLE 1
#define FCS_KERNEL fcs_sim_skip_kernel
#include "fcs_sim_kernel.inc"
#undef FCS_ALL_POLICIES
#undef FCS_KERNEL
#undef FCS_KERNEL_ATTR
#undef FCS_SKIP_IDLE

#define FCS_ALL_POLICIES 1
#define FCS_SKIP_IDLE 0
#define FCS_KERNEL fcs_sim_all_kernel
#define FCS_KERNEL_ATTR
#include "fcs_sim_kernel.inc"
#undef FCS_KERNEL
#undef FCS_MC_KNOWN

// the same with the MC benchmark for known request types
#define FCS_MC_KNOWN 1
#define FCS_KERNEL fcs_sim_mck_kernel
#include "fcs_sim_kernel.inc"
#undef FCS_ALL_POLICIES
#undef FCS_KERNEL
#undef FCS_KERNEL_ATTR
#undef FCS_SKIP_IDLE
#undef FCS_MC_KNOWN


// Orders the cells of a launch by the time their slowest path took in the launch before (longest first;
// equal times in index order, so whatever the words hold the result is a permutation), and clears the words
// in which this launch records its own times.  A launch lasts as long as its last path, and what sets it is
// a few slow paths rather than the mean of a cell: workgroups are handed out in index order, so the cells
// that hold them should start first.
__global__ __launch_bounds__(1024) void fcs_order_kernel(uint32_t* sched, int n_cells, uint32_t seq) {
  // the times as 32-bit keys in LDS (saturated: an order is all that is wanted), so that the n^2 comparisons
  // read LDS words that all threads ask for at once instead of device memory
  __shared__ uint32_t key[kMaxOrderedCells];
  unsigned long long* const cost_prev = reinterpret_cast<unsigned long long*>(sched) + ((seq & 1u) ^ 1u) * n_cells;
  unsigned long long* const cost_cur = reinterpret_cast<unsigned long long*>(sched) + (seq & 1u) * n_cells;
  int32_t* const order = reinterpret_cast<int32_t*>(sched + 4u * n_cells);
  for (int i = static_cast<int>(threadIdx.x); i < n_cells; i += static_cast<int>(blockDim.x)) {
    const unsigned long long c = cost_prev[i];
    key[i] = c > 0xffffffffull ? 0xffffffffu : static_cast<uint32_t>(c);
  }
  __syncthreads();
  for (int i = static_cast<int>(threadIdx.x); i < n_cells; i += static_cast<int>(blockDim.x)) {
    const uint32_t mine = key[i];
    int rank = 0;
    for (int j = 0; j < n_cells; ++j) {
      const uint32_t other = key[j];
      rank += (other > mine || (other == mine && j < i)) ? 1 : 0;
    }
    order[rank] = i;
    cost_cur[i] = 0ull;
  }
}

}  // namespace

int launch_sim(KParams kp, uint32_t sched_off, void* stream) {
  const size_t lds = static_cast<size_t>(lds_words(kp.lcap, kp.stack_lds, kp.class_words + 2 * kp.wheel_slots)) * sizeof(int32_t);
  void (*kernel)(const KParams) = kp.all_policies ? (kp.wheel_slots > 0 ? fcs_sim_mck_kernel : fcs_sim_all_kernel)
                                  : (kp.flags & FCS_FLAG_SKIP_IDLE) ? fcs_sim_skip_kernel : fcs_sim_kernel;
  if (lds > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
    if (e != hipSuccess) return FCS_EDEVICE;
  }
  kp.order = nullptr;
  kp.cost = nullptr;
  if (kp.n_cells > 1 && kp.n_cells <= kMaxOrderedCells) {
    uint32_t* sched = const_cast<uint32_t*>(kp.blob) + sched_off;
    hipLaunchKernelGGL(fcs_order_kernel, dim3(1), dim3(1024), 0, static_cast<hipStream_t>(stream), sched, kp.n_cells,
                       kp.launch_seq);
    if (hipGetLastError() != hipSuccess) return FCS_EDEVICE;
    kp.order = reinterpret_cast<const int32_t*>(sched + 4u * kp.n_cells);
    kp.cost = reinterpret_cast<unsigned long long*>(sched) + (kp.launch_seq & 1u) * kp.n_cells;
  }
  hipLaunchKernelGGL(kernel, dim3(static_cast<unsigned>(kp.n_paths)), dim3(kWave), lds,
                     static_cast<hipStream_t>(stream), kp);
  return hipGetLastError() == hipSuccess ? FCS_OK : FCS_EDEVICE;
}

}  // namespace fcs
