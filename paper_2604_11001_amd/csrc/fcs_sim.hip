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
//                  PLEFT  prompt tokens still to prefill; meaningful while END is -1 (0 = unused)
//                  REC    {l, o, arrival slot, id}
//   waiting queue  requests that were never activated are not stored: arrivals are a pure
//                function of (seed, replica, slot, index), so the FIFO of fresh requests is
//                re-generated 64 arrivals at a time when they are admitted.  Evicted requests
//                re-enter at the front of Q, newest eviction deepest: a stack (first
//                kStackLds entries in LDS, the rest in the spill region).
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
template <int l>
__device__ __forceinline__ int wrl_c(int s, int v) {
  asm("v_writelane_b32 %0, %1, %2" : "+v"(v) : "s"(s), "n"(l));
  return v;
}
#define wrl(s, l, v) wrl_c<l>((s), (v))

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

__global__ __launch_bounds__(kWave) void fcs_sim_kernel(const KParams kp) {
  extern __shared__ __attribute__((aligned(16))) int32_t smem[];
  const int lane = static_cast<int>(threadIdx.x);
  const int path = static_cast<int>(blockIdx.x);
  if (path >= kp.n_paths) return;

  const int cell_i = path / kp.n_replicas;
  const uint32_t rep = kp.replica_base + static_cast<uint32_t>(path - cell_i * kp.n_replicas);
  const DLaw* __restrict__ laws = reinterpret_cast<const DLaw*>(kp.blob + kp.laws_off);
  const DCell cellp = reinterpret_cast<const DCell*>(kp.blob + kp.cells_off)[cell_i];
  const bool greedy = cellp.policy == FCS_POLICY_GREEDY;
  const int M = kp.M, T = kp.n_steps;
  const int LC = kp.lcap, HC = kp.hcap, HS = kp.hscap;
  const int CAP = LC + HC;            // slots of the active set
  const int SCAP = kStackLds + HS;    // entries of the evicted stack
  // LDS word offsets
  const int O_PL = 2 * LC, O_REC = 3 * LC, O_STK = kLdsWordsPerSlot * LC, O_SCR = O_STK + S_NFIELDS * kStackLds;
  // spill region of this path
  int32_t* const hREM = kp.spill + static_cast<size_t>(path) * kp.spill_stride;
#define hPL (hREM + HC)
#define hREC (hREM + 2 * static_cast<size_t>(HC))
#define hSTK (hREM + static_cast<size_t>(kSpillWordsPerSlot) * HC)

  // ---- record accessors (uniform position: every lane reads the same record) ---------
  auto rec_load = [&](int pos) __attribute__((always_inline)) -> v4i {
    if (pos < LC) return ld4(&smem[O_REC + 4 * pos]);
    return ld4(&hREC[4 * static_cast<size_t>(pos - LC)]);
  };
  // writes a whole slot; executed by one lane
  auto slot_store = [&](int pos, int end, int pleft, v4i rec) __attribute__((always_inline)) {
    if (LIKELY(pos < LC)) {
      smem[2 * pos] = end;
      smem[2 * pos + 1] = rec.x + rec.y;
      smem[O_PL + pos] = pleft;
      st4(&smem[O_REC + 4 * pos], rec);
    } else {
      const size_t q = static_cast<size_t>(pos - LC);
      hREM[q] = end;
      hPL[q] = pleft;
      st4(&hREC[4 * q], rec);
    }
  };
  // a request enters slot pos (in LDS its END entry is -1 already); executed by one lane
  auto slot_admit = [&](int pos, int pleft, v4i rec) __attribute__((always_inline)) {
    if (LIKELY(pos < LC)) {
      smem[O_PL + pos] = pleft;
      st4(&smem[O_REC + 4 * pos], rec);
    } else {
      const size_t q = static_cast<size_t>(pos - LC);
      hREM[q] = -1;  // the spill region starts out uninitialised
      hPL[q] = pleft;
      st4(&hREC[4 * q], rec);
    }
  };
  auto end_pl_load = [&](int pos, int& end, int& pl) __attribute__((always_inline)) {
    if (LIKELY(pos < LC)) { end = smem[2 * pos]; pl = smem[O_PL + pos]; }
    else { end = hREM[pos - LC]; pl = hPL[pos - LC]; }
  };
  auto end_pl_store = [&](int pos, int end, int pl) __attribute__((always_inline)) {
    if (LIKELY(pos < LC)) { smem[2 * pos] = end; smem[O_PL + pos] = pl; }
    else { hREM[pos - LC] = end; hPL[pos - LC] = pl; }
  };

  // ---- output rows of this path ------------------------------------------------------
  uint32_t* hist = kp.out.hist ? kp.out.hist + static_cast<size_t>(path) * kp.hist_bins : nullptr;
  int32_t* arr_rec = kp.out.arrival_step
                         ? kp.out.arrival_step + static_cast<size_t>(path) * kp.max_requests : nullptr;
  int32_t* comp_rec = kp.out.completion_step
                          ? kp.out.completion_step + static_cast<size_t>(path) * kp.max_requests : nullptr;
  if (hist) for (int i = lane; i < kp.hist_bins; i += kWave) hist[i] = 0u;
  if (arr_rec) for (int i = lane; i < kp.max_requests; i += kWave) arr_rec[i] = 0;
  if (comp_rec) for (int i = lane; i < kp.max_requests; i += kWave) comp_rec[i] = 0;
  for (int i = lane; i < LC; i += kWave) {
    smem[2 * i] = -1;
    smem[2 * i + 1] = 0;
    smem[O_PL + i] = 0;
  }
  wave_sync();
  // completions are accounted in the lanes that hold the dead slots: keep what that needs in
  // vector registers so that it costs no scalar registers in the main loop
  uint64_t hist_v = reinterpret_cast<uint64_t>(hist), comp_v = reinterpret_cast<uint64_t>(comp_rec);
  int hist_last_v = kp.hist_bins - 1, hist_shift_v = kp.hist_shift, max_req_v = kp.max_requests;
  asm volatile("" : "+v"(hist_v), "+v"(comp_v), "+v"(hist_last_v), "+v"(hist_shift_v), "+v"(max_req_v));

  // ---- state (wave-uniform) ------------------------------------------------------------
  int U = 0;           // sum over P of (l + j)
  int n_live = 0;      // |P|
  int n_dec = 0;       // requests of P that are decoding
  int n_pf = 0;        // requests of P that are still prefilling
  int n_slots = 0;     // slots in use, dead ones included
  int pf_first = 0;    // no prefilling request sits below this slot
  int sdepth = 0;      // evicted requests waiting at the front of Q
  uint32_t arrived = 0, fresh_next = 0;  // arrivals so far; id of the next never-activated request
  int head_l = -1;     // GREEDY: prompt length of the head of Q, -1 = not fetched
  int err = 0, err_step = 0;
  // fresh-request block: lane i holds arrival fb_base + i
  int fb_l = 0, fb_o = 0, fb_t = 0;
  uint32_t fb_base = 0;
  int fb_count = 0;
  uint32_t rd_t = 1;   // reader cursor: slot ...
  int rd_k = 0;        // ... and arrivals of that slot already handed out
  int win = 0;         // lane i: n_t | B_t << 16 for the i-th slot of the current window
  int win_t0 = 0;      // first slot of that window (0: none drawn yet)
  // calendars: bit i = some request may complete in the i-th slot of the current window; cal0 for
  // the requests in slots 0..255, cal1 for the others
  uint64_t cal0 = 0, cal1 = 0;
  // statistics: lane k of (acc_hi:acc_lo) is counter SL_k; lanes 0..2 of mx are max U, |P|, |Q|
  uint32_t acc_lo = 0, acc_hi = 0;
  int mx = 0;
  // per-lane partial sums over the requests whose completion this lane handled
  uint32_t lat_lo = 0, lat_hi = 0, use_lo = 0, use_hi = 0;
  int lat_max = 0;
  int trace_left = kp.trace_every > 0 ? kp.trace_every : 0x7fffffff, trace_idx = 0;  // T < 2^30

  // records the first error of the path (a macro: the error state must stay in registers)
#define FCS_FAIL(code, tt) do { if (!err) { err = (code); err_step = (tt); } } while (0)

  // n_t and B_t of slot t0 + lane (Section 2.1: n_t from a known law with mean lambda;
  // Theorem 2: B_t i.i.d. bounded integers with mean b)
  // the thresholds of the arrival law stay in lanes (at most kMaxCountThr of them)
  const DLaw arr_law = laws[cellp.arrival];
  const int arr_n = rfl(arr_law.n);
  const int arr_thr_v = lane < arr_n ? static_cast<int>(kp.blob[arr_law.off + static_cast<uint32_t>(lane)]) : -1;
  auto draw_slot = [&](uint32_t t0, int& n_out, int& b_out) __attribute__((always_inline)) {
    uint32_t w0, w1, w2, w3;
    philox4x32_10(0u, t0 + static_cast<uint32_t>(lane), rep, 0u, kp.seed_lo, kp.seed_hi, w0, w1, w2, w3);
    int n = 0;
    for (int i = 0; i < arr_n; ++i) n += (w0 >= static_cast<uint32_t>(rdl(arr_thr_v, i))) ? 1 : 0;
    n_out = n;
    // GREEDY is the limit of an unbounded B_t (remark after Theorem 2); 0x7fff exceeds any active set
    b_out = greedy ? 0x7fff : cellp.b_floor + ((w1 < cellp.b_frac_thr) ? 1 : 0);
  };

  // Generates the next block of never-activated requests, in arrival order, starting at
  // arrival index fresh_next (requires fresh_next == fb_base + fb_count).
  auto refill_block = [&]() __attribute__((always_inline)) {
    fb_base = fresh_next;
    fb_count = 0;
    while (fb_count == 0 && rd_t <= static_cast<uint32_t>(T)) {
      int n, b;
      if (rd_t == static_cast<uint32_t>(win_t0)) n = win & 0xffff;  // the window just drawn
      else draw_slot(rd_t, n, b);
      if (rd_t + static_cast<uint32_t>(lane) > static_cast<uint32_t>(T)) n = 0;
      if (lane == 0) n -= rd_k;
      const int incl = wave_incl_sum(n);
      const int total = rdl(incl, kWave - 1);
      const int excl = incl - n;
      if (total == 0) { rd_t += kWave; rd_k = 0; continue; }
      // expand: output lane i takes the slot s with excl[s] <= i < incl[s]
      smem[O_SCR + lane] = 0;
      wave_sync();
      if (n > 0 && excl < kWave) smem[O_SCR + excl] = lane + 1;
      wave_sync();
      const int mark = smem[O_SCR + lane];
      wave_sync();
      const int cnt = min(total, kWave);
      const bool valid = lane < cnt;
      const int owner = wave_incl_max(mark);
      const int src = valid ? owner - 1 : 0;
      const int ex_s = __shfl(excl, src, kWave);
      const int k = lane - ex_s + (src == 0 ? rd_k : 0);
      const uint32_t ta = rd_t + static_cast<uint32_t>(src);
      uint32_t w0, w1, w2, w3;
      philox4x32_10(static_cast<uint32_t>(k), ta, rep, 1u, kp.seed_lo, kp.seed_hi, w0, w1, w2, w3);
      const uint32_t* __restrict__ class_thr = kp.blob + kp.class_off;
      int cls = 0;
      for (int i = 0; i + 1 < kp.n_classes; ++i) cls += (w0 >= class_thr[i]) ? 1 : 0;
      const DLaw pl = laws[kp.n_arrival_laws + cls];
      const DLaw dl = laws[kp.n_arrival_laws + kp.n_classes + cls];
      // value = lo + #{thr <= u}: both laws bisected together inside the guide buckets of their words
      int lo1 = 0, hi1 = 0, lo2 = 0, hi2 = 0;
      if (valid) {
        if (pl.n > 0) {
          const uint32_t* g = kp.blob + pl.goff + (w1 >> (32 - kGuideBits));
          lo1 = static_cast<int>(g[0]); hi1 = static_cast<int>(g[1]);
        }
        if (dl.n > 0) {
          const uint32_t* g = kp.blob + dl.goff + (w2 >> (32 - kGuideBits));
          lo2 = static_cast<int>(g[0]); hi2 = static_cast<int>(g[1]);
        }
      }
      const uint32_t* th1 = kp.blob + pl.off;
      const uint32_t* th2 = kp.blob + dl.off;
      for (int it = 0; it < 34 && __any(lo1 < hi1 || lo2 < hi2); ++it) {
        const bool a1 = lo1 < hi1, a2 = lo2 < hi2;
        const int m1 = (lo1 + hi1) >> 1, m2 = (lo2 + hi2) >> 1;
        const uint32_t v1 = a1 ? th1[m1] : 0u;
        const uint32_t v2 = a2 ? th2[m2] : 0u;
        if (a1) { if (v1 <= w1) lo1 = m1 + 1; else hi1 = m1; }
        if (a2) { if (v2 <= w2) lo2 = m2 + 1; else hi2 = m2; }
      }
      fb_l = pl.lo + lo1;
      fb_o = dl.lo + lo2;
      fb_t = static_cast<int>(ta);
      fb_count = cnt;
      if (total <= kWave) {
        rd_t += kWave;
        rd_k = 0;
      } else {
        rd_k = rdl(k, kWave - 1) + 1;
        rd_t += static_cast<uint32_t>(rdl(src, kWave - 1));
      }
    }
  };

  // Statistics of completed requests (Section 4: average and tail latency), taken in the lanes
  // flagged `mine` from the record of the request and the slot `e` in which it completed.
  auto account = [&](bool mine, v4i rec, int e) __attribute__((always_inline)) {
    if (mine) {
      const int lat = e - rec.z + 1;              // arrival to completion, both slots counted
      const uint32_t s = lat_lo + static_cast<uint32_t>(lat);
      lat_hi += (s < lat_lo) ? 1u : 0u;
      lat_lo = s;
      const uint32_t u = use_lo + static_cast<uint32_t>(rec.y);
      use_hi += (u < use_lo) ? 1u : 0u;
      use_lo = u;
      lat_max = max(lat_max, lat);
      if (hist_v) atomicAdd(reinterpret_cast<uint32_t*>(hist_v) + min(lat >> hist_shift_v, hist_last_v), 1u);
      if (comp_v && rec.w < max_req_v) reinterpret_cast<int32_t*>(comp_v)[rec.w] = e;
    }
  };

  // Order-preserving removal of dead slots; tlive is the first slot in which a decoding request
  // that is still there generates a token (the current slot, or the next one once the
  // completions of the current slot are done).  Requests that completed are accounted here.
  auto compact = [&](int tlive) __attribute__((always_inline)) {
    int out = 0, new_pf = -1;
    for (int base = 0; base < n_slots; base += kWave) {
      const int pos = base + lane;
      const bool in = pos < n_slots;
      int end = -1, pl = 0;
      v4i rec = {0, 0, 0, 0};
      if (in) {
        if (LIKELY(base < LC)) {
          end = smem[2 * pos]; pl = smem[O_PL + pos];
          rec = ld4(&smem[O_REC + 4 * pos]);
        } else {
          end = hREM[pos - LC]; pl = hPL[pos - LC];
          rec = ld4(&hREC[4 * static_cast<size_t>(pos - LC)]);
        }
      }
      const bool pf = in && end < 0 && pl > 0;
      const bool live = pf || (in && end >= tlive);
      account(in && end >= 0 && end < tlive, rec, end);
      const uint64_t m = __ballot(live);
      const uint64_t pm = __ballot(pf);
      const int dst = out + lanes_below(m);
      if (pm != 0 && new_pf < 0) new_pf = out + __popcll(m & ((1ull << __builtin_ctzll(pm)) - 1ull));
      wave_sync();
      if (live) slot_store(dst, end, pf ? pl : 0, rec);
      wave_sync();
      out += __popcll(m);
    }
    for (int base = out; base < n_slots; base += kWave) {
      const int pos = base + lane;
      if (pos < n_slots) end_pl_store(pos, -1, 0);
    }
    wave_sync();
    n_slots = out;
    pf_first = new_pf < 0 ? n_slots : new_pf;
    cal0 |= cal1;  // requests moved towards slot 0
  };

  // Evicts the most recently activated request (Section 3.3: last in, first out); it loses
  // its progress and goes back to the front of Q.
  auto evict_newest = [&](int t) __attribute__((always_inline)) {
    int pos = n_slots - 1;
    int end = 0, pleft = 0;
    for (; pos >= 0; --pos) {
      end_pl_load(pos, end, pleft);
      end = rfl(end);
      pleft = rfl(pleft);
      if (end >= t || (end < 0 && pleft > 0)) break;
      if (end >= 0) {  // a request that completed: its slot goes away here, so account it here
        account(lane == 0, rec_load(pos), end);
        if (lane == 0) end_pl_store(pos, -1, 0);
      }
    }
    if (pos < 0) { FCS_FAIL(FCS_ESTATE, t); return; }
    const v4i rec = rec_load(pos);
    const int l = rfl(rec.x), o = rfl(rec.y);
    // a decoding request had end - t + 1 of its o tokens still to come (written without branches:
    // two branches that each decrement a counter get merged into a store through a selected
    // pointer, which forces both counters out of registers)
    const int pf = end < 0 ? 1 : 0;
    U -= l + (pf ? 0 : o - (end - t + 1));
    n_pf -= pf;
    n_dec -= 1 - pf;
    n_live -= 1;
    if (sdepth == SCAP) { FCS_FAIL(FCS_EOVERFLOW, t); return; }
    if (lane == 0) {
      if (sdepth < kStackLds) st4(&smem[O_STK + 4 * sdepth], rec);
      else st4(&hSTK[4 * static_cast<size_t>(sdepth - kStackLds)], rec);
      end_pl_store(pos, -1, 0);
    }
    wave_sync();
    sdepth += 1;
    n_slots = pos;
    if (pf_first > n_slots) pf_first = n_slots;
    head_l = l;
  };

  // =============================== slots 1..T ========================================
  // Two renditions of one slot.  `general_slot` handles every case (spill tier, evictions, budget
  // stalls, table refills, compaction) and can pick a slot up at any of its phases.  The loop
  // below it is the same slot restricted to what almost every slot needs (everything in LDS, no
  // eviction, no stall); when a slot needs more it hands over to `general_slot` at the phase it
  // has reached.  Variables of the slot in flight are shared between the two.
  int t = 1;
  int phase = 0;  // 0 slot start, 1 admission, 3 overflow check, 4 decode pass, 6 compaction only
  int resume = 0; // 1: the hand-scheduled loop takes the slot in flight up again at its admission step
  int x = 0;      // this slot's contribution to the statistics, one counter per lane
  int room = 0, admitted = 0, budget = 0, new_dec = 0;
  int rel_sum = 0, n_done = 0;  // completions of this slot: released footprint and count

  // called where the lanes of mask m0 (flag `mine`) hold a request, in slot `pos`, that generates
  // its last token in this slot: counts it and adds its footprint l + o to what the slot releases
  auto complete = [&](bool mine, uint64_t m0, int pos) __attribute__((always_inline)) {
    int relv = 0;
    if (mine) {
      if (LIKELY(pos < LC)) {
        relv = smem[2 * pos + 1];
      } else {
        const v4i rec = ld4(&hREC[4 * static_cast<size_t>(pos - LC)]);
        relv = rec.x + rec.y;
      }
    }
    n_done += static_cast<int>(__popcll(m0));
    rel_sum += rdl(relv, __builtin_ctzll(m0));
    uint64_t m = m0 & (m0 - 1);
    while (UNLIKELY(m != 0)) {
      rel_sum += rdl(relv, __builtin_ctzll(m));
      m &= m - 1;
    }
  };
  // step 5 (Section 2.1: U_t after processing, before completed requests leave) and step 6
  auto measure_and_release = [&](int tokens, int qlen) __attribute__((always_inline)) {
    U += tokens;
    n_dec += new_dec;
    x = wrl(U, SL_SUM_U, x);
    x = wrl(n_live, SL_SUM_P, x);
    x = wrl(qlen, SL_SUM_Q, x);
    x = wrl(tokens, SL_DEC_TOK, x);
    if (n_done) x = wrl(n_done, SL_DONE, x);
    const uint32_t s = acc_lo + static_cast<uint32_t>(x);
    acc_hi += (s < acc_lo) ? 1u : 0u;
    acc_lo = s;
    mx = max(mx, x);
    if (UNLIKELY(--trace_left == 0)) {
      trace_left = kp.trace_every;
      if (lane == 0) {
        if (kp.out.trace_q) kp.out.trace_q[static_cast<size_t>(path) * kp.n_trace + trace_idx] = qlen;
        if (kp.out.trace_u) kp.out.trace_u[static_cast<size_t>(path) * kp.n_trace + trace_idx] = U;
      }
      trace_idx += 1;
    }
    // the footprint of completed requests is released at the end of the slot
    U -= rel_sum;
    n_live -= n_done;
    n_dec -= n_done;
  };

  // Rebuilds the calendars of the window that starts at slot t0 from the END entries.
  auto calendars_of_window = [&](int t0) __attribute__((always_inline)) {
    uint32_t lo0 = 0, hi0 = 0, lo1 = 0, hi1 = 0;
    for (int base = 0; base < n_slots; base += kWave) {
      const int pos = base + lane;
      int v = -1;
      if (pos < n_slots) v = LIKELY(base < LC) ? smem[2 * pos] : hREM[pos - LC];
      const uint32_t d = static_cast<uint32_t>(v - t0);
      const uint32_t lo = d < 32u ? 1u << d : 0u;
      const uint32_t hi = (d >= 32u && d < 64u) ? 1u << (d - 32u) : 0u;
      if (base < kLdsBlock) { lo0 |= lo; hi0 |= hi; } else { lo1 |= lo; hi1 |= hi; }
    }
    cal0 = (static_cast<uint64_t>(wave_or(hi0)) << 32) | wave_or(lo0);
    cal1 = (static_cast<uint64_t>(wave_or(hi1)) << 32) | wave_or(lo1);
  };

  // A launch lasts as long as its slowest path and wavefronts share a SIMD, so a path that is
  // behind the others gets issue priority over its neighbours.  Every eighth window a path
  // publishes its pace (time per slot so far) into a sum over all paths of the launch and takes the
  // priority that the mean it read the time before gives it (that read has had eight windows to
  // arrive).  kp.pace holds {sum, count} twice: launches alternate between the two and clear the
  // other one, so the words need no clearing from the host.
  const unsigned long long t_begin = wall_clock64();
  unsigned long long* const pace_w = kp.pace ? kp.pace + 2 * (kp.launch_seq & 1u) : nullptr;
  if (kp.pace != nullptr && path == 0 && lane == 0) {
    kp.pace[2 * ((kp.launch_seq & 1u) ^ 1u)] = 0ull;
    kp.pace[2 * ((kp.launch_seq & 1u) ^ 1u) + 1] = 0ull;
  }
  unsigned long long pace_sum = 0, pace_cnt = 0;  // what this path last read
  uint32_t pace_mine = 0;                          // what it last published
  auto pacing = [&](int t0) __attribute__((always_inline)) {
    if (pace_w == nullptr || ((t0 - 1) & 511) != 0 || t0 <= 1) return;
    const unsigned long long dt = wall_clock64() - t_begin;
    const uint32_t pace = static_cast<uint32_t>(min(dt * 64ull / static_cast<unsigned long long>(t0 - 1), 0xffffffull));
    const unsigned long long sum = (static_cast<unsigned long long>(static_cast<uint32_t>(rfl(static_cast<int>(pace_sum >> 32)))) << 32) |
                                   static_cast<uint32_t>(rfl(static_cast<int>(pace_sum)));
    const uint32_t cnt = static_cast<uint32_t>(rfl(static_cast<int>(pace_cnt)));
    if (lane == 0) {
      // nothing comes back from the updates
      __hip_atomic_fetch_add(pace_w, static_cast<unsigned long long>(pace) - static_cast<unsigned long long>(pace_mine),
                             __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (pace_mine == 0) __hip_atomic_fetch_add(pace_w + 1, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      pace_sum = __hip_atomic_load(pace_w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      pace_cnt = __hip_atomic_load(pace_w + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    pace_mine = pace;
    if (cnt != 0) {
      const unsigned long long p = static_cast<unsigned long long>(pace) * cnt * 64ull;  // pace / mean in 64ths
      if (p >= sum * 77ull) __builtin_amdgcn_s_setprio(3);        // 20 % slower than the mean
      else if (p >= sum * 69ull) __builtin_amdgcn_s_setprio(2);   // 8 %
      else if (p >= sum * 63ull) __builtin_amdgcn_s_setprio(1);   // about the mean
      else __builtin_amdgcn_s_setprio(0);
    }
  };

  // First slot t0 of a 64-slot window: draws n_t and B_t of the window and rebuilds the calendar.
  auto window_start = [&](int t0) __attribute__((always_inline)) {
    pacing(t0);
    int n, b;
    draw_slot(static_cast<uint32_t>(t0), n, b);
    win = n | (b << 16);
    calendars_of_window(t0);
    win_t0 = t0;
    if (UNLIKELY(arrived >= 0x7ffe0000u)) FCS_FAIL(FCS_EOVERFLOW, t0);
    if (arr_rec) {  // arrival slots of the requests of this window, by arrival id
      const int tt = t0 + lane;
      const int ne = tt <= T ? n : 0;
      const int excl = wave_incl_sum(ne) - ne;
      for (int k = 0; k < ne; ++k) {
        const uint32_t id = arrived + static_cast<uint32_t>(excl + k);
        if (id < static_cast<uint32_t>(kp.max_requests)) arr_rec[id] = tt;
      }
    }
  };

  auto general_slot = [&]() __attribute__((always_inline)) {
    // ---- 1. arrivals ---------------------------------------------------------------
    if (phase <= 0) {
      x = 0;
      const int wi = (t - 1) & (kWave - 1);
      if (wi == 0 && win_t0 != t) window_start(t);
      const int nb = rdl(win, wi);
      arrived += static_cast<uint32_t>(nb & 0xffff);
      const int ql = sdepth + static_cast<int>(arrived - fresh_next);
      room = greedy ? ql : min(nb >> 16, ql);
      admitted = 0;
    }

    // ---- 2. admission: FLOW moves min(B_t, |Q|) head requests, GREEDY while the head fits ----
    if (phase <= 1) {
      while (room > 0 && LIKELY(!err)) {
        const bool from_stack = sdepth > 0;
        int idx = 0;
        if (!from_stack) {
          if (UNLIKELY(static_cast<int>(fresh_next - fb_base) >= fb_count)) refill_block();
          idx = static_cast<int>(fresh_next - fb_base);
          if (UNLIKELY(idx >= fb_count)) { FCS_FAIL(FCS_ESTATE, t); break; }
        }
        if (greedy) {
          if (head_l < 0) {
            if (from_stack) {
              const int d = sdepth - 1;
              head_l = rfl(d < kStackLds ? smem[O_STK + 4 * d] : hSTK[4 * static_cast<size_t>(d - kStackLds)]);
            } else {
              head_l = rdl(fb_l, idx);
            }
          }
          if (U + n_live + head_l + 1 > M) break;
        }
        if (UNLIKELY(n_slots == CAP)) {
          if (n_live < n_slots) compact(t);
          if (n_slots == CAP) { FCS_FAIL(FCS_EOVERFLOW, t); break; }
        }
        const int pos = n_slots;
        int l;
        if (from_stack) {
          const int d = sdepth - 1;
          v4i rec;
          if (d < kStackLds) rec = ld4(&smem[O_STK + 4 * d]);
          else rec = ld4(&hSTK[4 * static_cast<size_t>(d - kStackLds)]);
          l = rfl(rec.x);
          if (lane == 0) slot_admit(pos, l, rec);
          sdepth = d;
        } else {
          l = rdl(fb_l, idx);
          if (lane == idx) {
            const v4i rec = {fb_l, fb_o, fb_t, static_cast<int>(fresh_next)};
            slot_admit(pos, fb_l, rec);
          }
          fresh_next += 1u;
        }
        wave_sync();
        n_slots = pos + 1;
        if (n_pf == 0 || pf_first > pos) pf_first = pos;
        U += l;
        n_live += 1;
        n_pf += 1;
        admitted += 1;
        room -= 1;
        head_l = -1;
      }
      if (admitted) x = wrl(admitted, SL_ACT, x);
    }

    if (phase <= 3) {
      // ---- 3. overflow: evict newest while the provisioned usage exceeds M ------------------
      if (UNLIKELY(U + n_live > M)) {
        int ev = 0;
        do { evict_newest(t); ev += 1; } while (U + n_live > M && !err);
        x = wrl(ev, SL_EVICT, x);
        x = wrl(1, SL_OVF, x);
      }
      if (UNLIKELY(err)) return;

      // ---- 4a. chunked prefill under the token budget, activation order ---------------------
      budget = kp.tau;
      new_dec = 0;
      if (n_pf > 0) {
        int todo = n_pf;
        int base = pf_first & ~(kWave - 1);
        int first_left = -1;
        while (todo > 0 && budget > 0 && base < n_slots) {
          const int pos = base + lane;
          int pl = 0, lv = 0, ov = 0, e = 0;
          if (LIKELY(base < LC)) {
            pl = smem[O_PL + pos]; e = smem[2 * pos];
            lv = smem[O_REC + 4 * pos]; ov = smem[O_REC + 4 * pos + 1];
          } else if (pos < n_slots) {
            pl = hPL[pos - LC]; e = hREM[pos - LC];
            lv = hREC[4 * static_cast<size_t>(pos - LC)]; ov = hREC[4 * static_cast<size_t>(pos - LC) + 1];
          }
          uint64_t m = __ballot(e < 0 && pl > 0);
          while (m != 0 && budget > 0) {
            const int i = __builtin_ctzll(m);
            m &= m - 1;
            const int p = base + i;
            int left = rdl(pl, i);
            const int d = min(min(kp.chunk, left), budget);
            left -= d;
            budget -= d;
            todo -= 1;
            if (left == 0) {
              // the chunk that ends the prompt yields token 1 in this slot, so token o comes in
              // slot t + o - 1 (this very slot when o = 1)
              const int o = rdl(ov, i);
              const int foot = rdl(lv, i) + o;
              if (lane == 0) {
                if (LIKELY(p < LC)) { smem[2 * p] = t + o - 1; smem[2 * p + 1] = foot; smem[O_PL + p] = 0; }
                else { hREM[p - LC] = t + o - 1; hPL[p - LC] = 0; }
              }
              const int k = ((t - 1) & (kWave - 1)) + o - 1;
              if (k < kWave) {
                if (p < kLdsBlock) cal0 |= 1ull << k; else cal1 |= 1ull << k;
              }
              new_dec += 1;
            } else {
              if (lane == 0) {
                if (LIKELY(p < LC)) smem[O_PL + p] = left; else hPL[p - LC] = left;
              }
              if (first_left < 0) first_left = p;
            }
          }
          wave_sync();
          if (m != 0) {  // budget ran out inside this chunk
            if (first_left < 0) first_left = base + __builtin_ctzll(m);
            break;
          }
          base += kWave;
        }
        if (first_left >= 0) pf_first = first_left;
        else pf_first = (todo > 0) ? min(base, n_slots) : n_slots;
        n_pf -= new_dec;
        x = wrl(kp.tau - budget, SL_PF_TOK, x);
      }
    }

    if (phase <= 4) {
      const int qlen = sdepth + static_cast<int>(arrived - fresh_next);
      // ---- 4b. decode growth: one token per decoding request while budget lasts --------------
      rel_sum = 0;
      n_done = 0;
      int advanced;  // requests already decoding that got a token
      if (LIKELY(budget >= n_dec)) {
        // every decoding request gets its token; only the ones whose last token this is need a look
        advanced = n_dec;
        if (((cal0 | cal1) >> ((t - 1) & (kWave - 1))) & 1ull) {
          const int lim = min(n_slots, LC);
          for (int b0 = 0; b0 < lim; b0 += kLdsBlock) {  // four {END, FOOT} pairs per lane
            const int p0 = b0 + (lane << 2);
            const v4i a = ld4(&smem[2 * p0]), b = ld4(&smem[2 * p0 + 4]);
            const int cnt = (a.x == t ? 1 : 0) + (a.z == t ? 1 : 0) + (b.x == t ? 1 : 0) + (b.z == t ? 1 : 0);
            const int relv = (a.x == t ? a.y : 0) + (a.z == t ? a.w : 0) + (b.x == t ? b.y : 0) + (b.z == t ? b.w : 0);
            uint64_t m = __ballot(cnt != 0);
            while (m != 0) {
              const int i = __builtin_ctzll(m);
              m &= m - 1;
              n_done += rdl(cnt, i);
              rel_sum += rdl(relv, i);
            }
          }
          for (int base = LC; base < n_slots; base += kWave) {
            const int pos = base + lane;
            const bool d = pos < n_slots && hREM[pos - LC] == t;
            const uint64_t dm = __ballot(d);
            if (dm != 0) complete(d, dm, pos);
          }
        }
      } else {
        // budget binds: the first `budget` already-decoding requests in activation order advance
        // and the others finish one slot later; requests that finished their prompt in this slot
        // (all o tokens still to come) take token 1 for free
        int left = budget;
        advanced = 0;
        // LDS tier: four {END, FOOT} pairs per lane and pass, lanes in activation order
        const int lim = min(n_slots, LC);
        for (int b0 = 0; b0 < lim; b0 += kLdsBlock) {
          const int p0 = b0 + (lane << 2);
          v4i a = ld4(&smem[2 * p0]), b = ld4(&smem[2 * p0 + 4]);
          int o0 = 0, o1 = 0, o2 = 0, o3 = 0;
          if (new_dec > 0) {  // output lengths tell the requests that finished their prompt in this slot
            o0 = smem[O_REC + 4 * p0 + 1]; o1 = smem[O_REC + 4 * p0 + 5];
            o2 = smem[O_REC + 4 * p0 + 9]; o3 = smem[O_REC + 4 * p0 + 13];
          }
          const bool f0 = new_dec > 0 && a.x - t + 1 == o0, f1 = new_dec > 0 && a.z - t + 1 == o1;
          const bool f2 = new_dec > 0 && b.x - t + 1 == o2, f3 = new_dec > 0 && b.z - t + 1 == o3;
          const int d0 = a.x >= t && !f0, d1 = a.z >= t && !f1, d2 = b.x >= t && !f2, d3 = b.z >= t && !f3;
          const int cnt = d0 + d1 + d2 + d3;
          const int incl = wave_incl_sum(cnt);
          const int total = rdl(incl, kWave - 1);
          const int r0 = incl - cnt, r1 = r0 + d0, r2 = r1 + d1, r3 = r2 + d2;  // ranks among the old ones
          const bool g0 = d0 && r0 < left, g1 = d1 && r1 < left, g2 = d2 && r2 < left, g3 = d3 && r3 < left;
          const bool c0 = (g0 || (f0 && a.x >= t)) && a.x == t, c1 = (g1 || (f1 && a.z >= t)) && a.z == t;
          const bool c2 = (g2 || (f2 && b.x >= t)) && b.x == t, c3 = (g3 || (f3 && b.z >= t)) && b.z == t;
          const int ndone = c0 + c1 + c2 + c3;
          const int relv = (c0 ? a.y : 0) + (c1 ? a.w : 0) + (c2 ? b.y : 0) + (c3 ? b.w : 0);
          uint64_t m = __ballot(ndone != 0);
          while (m != 0) {
            const int i = __builtin_ctzll(m);
            m &= m - 1;
            n_done += rdl(ndone, i);
            rel_sum += rdl(relv, i);
          }
          const int took = min(total, left);
          if (took < total) {  // the requests past the budget finish one slot later
            a.x += (d0 && !g0) ? 1 : 0; a.z += (d1 && !g1) ? 1 : 0;
            b.x += (d2 && !g2) ? 1 : 0; b.z += (d3 && !g3) ? 1 : 0;
            st4(&smem[2 * p0], a);
            st4(&smem[2 * p0 + 4], b);
          }
          left -= took;
          advanced += took;
          wave_sync();
        }
        for (int base = LC; base < n_slots; base += kWave) {  // spill tier, 64 slots per pass
          const int pos = base + lane;
          const bool in = pos < n_slots;
          int v = -1, ov = 0;
          if (in) { v = hREM[pos - LC]; ov = hREC[4 * static_cast<size_t>(pos - LC) + 1]; }
          const bool dec = v >= t;
          const bool fresh = dec && new_dec > 0 && v - t + 1 == ov;
          const bool old = dec && !fresh;
          const uint64_t om = __ballot(old);
          const bool go = fresh || (old && lanes_below(om) < left);
          const int took = min(static_cast<int>(__popcll(om)), left);
          left -= took;
          advanced += took;
          const bool d = go && v == t;
          const uint64_t dm = __ballot(d);
          if (dm != 0) complete(d, dm, pos);
          if (old && !go) hREM[pos - LC] = v + 1;
          wave_sync();
        }
        // a stalled request moved to the next slot: keep the calendars supersets
        cal0 |= cal0 << 1;
        cal1 |= cal1 << 1;
        x = wrl(n_dec - advanced, SL_STALLED, x);
      }
      measure_and_release(advanced + new_dec, qlen);
    }
    if (n_slots - n_live >= kCompactSlack) compact(t + 1);
  };

  // The common slot (everything in LDS, no eviction, no stall) as hand-scheduled assembly; runs
  // slots until one needs the general code and returns with `phase` set.
  const int lds_base = static_cast<int>(
      reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) int32_t*)smem));
  auto fast_slots = [&]() __attribute__((always_inline)) {
#include "fcs_fast_slots.inc"
  };

  // its 32-bit sums over up to 64 slots need U and |Q| below 2^25
  const bool fast_ok = LC >= 2 * kLdsBlock && M < (1 << 25);
  while (t <= T && !err) {
    if (LIKELY(fast_ok) && LIKELY(n_slots <= LC) && LIKELY(arrived - fresh_next < (1u << 25))) {
      if (!resume && ((t - 1) & (kWave - 1)) == 0 && win_t0 != t) {
        window_start(t);
        if (UNLIKELY(err)) break;
      }
      fast_slots();
      resume = 0;
      if (t > T) break;
      // a new window: draw it and go on in the loop
      if (phase == 0 && ((t - 1) & (kWave - 1)) == 0 && win_t0 != t) continue;
      // the block of fresh requests ran out in the middle of an admission: refill it and go on
      if (phase == 1 && sdepth == 0 && n_slots < LC && static_cast<int>(fresh_next - fb_base) >= fb_count) {
        refill_block();
        if (LIKELY(static_cast<int>(fresh_next - fb_base) < fb_count)) { resume = 1; continue; }
      }
    }
    general_slot();
    ++t;
    phase = 0;
  }

  // ---- epilogue: digest of the final state, counters --------------------------------------------
  uint64_t h = 14695981039346656037ull;
  auto mix = [&](uint64_t w) __attribute__((always_inline)) { h = (h ^ w) * 1099511628211ull; };
  if (!err) {
    compact(t);  // t = T + 1 here
    mix(static_cast<uint64_t>(n_slots));
    for (int pos = 0; pos < n_slots; ++pos) {
      int rem, pleft;
      end_pl_load(pos, rem, pleft);
      rem = rfl(rem);
      pleft = rem < 0 ? rfl(pleft) : 0;
      const v4i rec = rec_load(pos);
      const int l = rfl(rec.x), o = rfl(rec.y), id = rfl(rec.w);
      mix(static_cast<uint64_t>(id));
      mix(static_cast<uint64_t>(rem > T ? o - (rem - T) : 0));  // rem - T tokens still to come
      mix(static_cast<uint64_t>(l - pleft));
    }
    mix(static_cast<uint64_t>(sdepth));
    for (int d = sdepth - 1; d >= 0; --d) {
      const int id = rfl(d < kStackLds ? smem[O_STK + 4 * d + 3] : hSTK[4 * static_cast<size_t>(d - kStackLds) + 3]);
      mix(static_cast<uint64_t>(id));
    }
    mix(static_cast<uint64_t>(arrived - fresh_next));
  }
  // reduce the per-lane completion sums over the wavefront
  uint64_t lat_sum = (static_cast<uint64_t>(lat_hi) << 32) | lat_lo;
  uint64_t use_sum = (static_cast<uint64_t>(use_hi) << 32) | use_lo;
#pragma unroll
  for (int d = kWave / 2; d > 0; d >>= 1) {
    lat_sum += __shfl_xor(lat_sum, d, kWave);
    use_sum += __shfl_xor(use_sum, d, kWave);
    lat_max = max(lat_max, __shfl_xor(lat_max, d, kWave));
  }
  uint64_t* C = kp.out.counters + static_cast<size_t>(path) * FCS_N_COUNTERS;
  const uint64_t acc = (static_cast<uint64_t>(acc_hi) << 32) | acc_lo;
  int slot = -1;
  switch (lane) {
    case SL_SUM_U: slot = FCS_C_SUM_U; break;
    case SL_SUM_P: slot = FCS_C_SUM_P; break;
    case SL_SUM_Q: slot = FCS_C_SUM_Q; break;
    case SL_DEC_TOK: slot = FCS_C_DECODE_TOKENS; break;
    case SL_ACT: slot = FCS_C_ACTIVATIONS; break;
    case SL_DONE: slot = FCS_C_COMPLETED; break;
    case SL_EVICT: slot = FCS_C_EVICTIONS; break;
    case SL_OVF: slot = FCS_C_OVERFLOW_STEPS; break;
    case SL_PF_TOK: slot = FCS_C_PREFILL_TOKENS; break;
    case SL_STALLED: slot = FCS_C_STALLED; break;
    default: break;
  }
  if (slot >= 0) C[slot] = acc;
  if (lane == SL_SUM_U) C[FCS_C_MAX_U] = static_cast<uint64_t>(mx);
  if (lane == SL_SUM_P) C[FCS_C_MAX_P] = static_cast<uint64_t>(mx);
  if (lane == SL_SUM_Q) C[FCS_C_MAX_Q] = static_cast<uint64_t>(mx);
  if (lane == 0) {
    C[FCS_C_ARRIVED] = arrived;
    C[FCS_C_USEFUL_TOKENS] = use_sum;
    C[FCS_C_SUM_LATENCY] = lat_sum;
    C[FCS_C_MAX_LATENCY] = static_cast<uint64_t>(lat_max);
    C[FCS_C_FINAL_U] = static_cast<uint64_t>(U);
    C[FCS_C_FINAL_P] = static_cast<uint64_t>(n_live);
    C[FCS_C_FINAL_Q] = static_cast<uint64_t>(sdepth) + static_cast<uint64_t>(arrived - fresh_next);
    C[FCS_C_DIGEST] = h;
    C[FCS_C_ERROR] = static_cast<uint64_t>(-err);
    C[FCS_C_ERROR_STEP] = static_cast<uint64_t>(err_step);
    C[FCS_C_RESERVED] = 0;
  }
}

}  // namespace

int launch_sim(const KParams& kp, void* stream) {
  const size_t lds = static_cast<size_t>(lds_words(kp.lcap)) * sizeof(int32_t);
  if (lds > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(fcs_sim_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
    if (e != hipSuccess) return FCS_EDEVICE;
  }
  hipLaunchKernelGGL(fcs_sim_kernel, dim3(static_cast<unsigned>(kp.n_paths)), dim3(kWave), lds,
                     static_cast<hipStream_t>(stream), kp);
  return hipGetLastError() == hipSuccess ? FCS_OK : FCS_EDEVICE;
}

}  // namespace fcs
