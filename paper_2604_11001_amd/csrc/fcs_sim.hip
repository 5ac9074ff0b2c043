// Sample-path kernel: one wavefront (= one workgroup) simulates one path of the slot
// model (Section 2.1) under Algorithm 2 or its greedy limit, for slots 1..T.
//
// Data layout per path
//   active set   slots in activation order; completed requests leave dead slots behind
//                ("tombstones") that an order-preserving compaction removes once kCompactSlack
//                of them have accumulated.  Slots [0, lcap) live in LDS, slots
//                [lcap, lcap+hcap) in a per-path spill region of the workspace.  Per slot:
//                  REM    o - j while decoding, negative otherwise.  The decode growth of a
//                         slot (Section 2.1: one more token per active request) is one
//                         decrement per slot of this array, four slots per lane per pass;
//                         a request completes when its entry reaches zero.
//                  PLEFT  prompt tokens still to prefill (0 once decoding, 0 for tombstones)
//                  REC    {l, o, arrival slot, id}, read when the request completes or is evicted
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

__device__ __forceinline__ int wave_incl_sum(int v, int lane) {
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    const int o = __shfl_up(v, d, kWave);
    if (lane >= d) v += o;
  }
  return v;
}

__device__ __forceinline__ int wave_incl_max(int v, int lane) {
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    const int o = __shfl_up(v, d, kWave);
    if (lane >= d) v = max(v, o);
  }
  return v;
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

// decode growth of four slots: entries of decoding requests (positive) lose one, others stay
__device__ __forceinline__ void dec4(v4i& v) {
  // max(v - 1, min(v, 0)) = median(v - 1, v, 0) is v - 1 for v > 0 and v otherwise
  v.x = max(v.x - 1, min(v.x, 0));
  v.y = max(v.y - 1, min(v.y, 0));
  v.z = max(v.z - 1, min(v.z, 0));
  v.w = max(v.w - 1, min(v.w, 0));
}

__device__ __forceinline__ uint32_t umin4(v4i v) {
  return min(min(static_cast<uint32_t>(v.x), static_cast<uint32_t>(v.y)),
             min(static_cast<uint32_t>(v.z), static_cast<uint32_t>(v.w)));
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
  const int O_PL = LC, O_REC = 2 * LC, O_STK = F_NFIELDS * LC, O_SCR = O_STK + S_NFIELDS * kStackLds;
  // spill region of this path
  int32_t* const hREM = kp.spill + static_cast<size_t>(path) * kp.spill_stride;
#define hPL (hREM + HC)
#define hREC (hREM + 2 * static_cast<size_t>(HC))
#define hSTK (hREM + static_cast<size_t>(F_NFIELDS) * HC)

  // ---- record accessors (uniform position: every lane reads the same record) ---------
  auto rec_load = [&](int pos) __attribute__((always_inline)) -> v4i {
    if (pos < LC) return ld4(&smem[O_REC + 4 * pos]);
    return ld4(&hREC[4 * static_cast<size_t>(pos - LC)]);
  };
  auto slot_store = [&](int pos, int rem, int pleft, v4i rec) __attribute__((always_inline)) {  // executed by one lane
    if (LIKELY(pos < LC)) {
      smem[pos] = rem;
      smem[O_PL + pos] = pleft;
      st4(&smem[O_REC + 4 * pos], rec);
    } else {
      const size_t q = static_cast<size_t>(pos - LC);
      hREM[q] = rem;
      hPL[q] = pleft;
      st4(&hREC[4 * q], rec);
    }
  };
  auto rem_pl_load = [&](int pos, int& rem, int& pl) __attribute__((always_inline)) {
    if (LIKELY(pos < LC)) { rem = smem[pos]; pl = smem[O_PL + pos]; }
    else { rem = hREM[pos - LC]; pl = hPL[pos - LC]; }
  };
  auto rem_pl_store = [&](int pos, int rem, int pl) __attribute__((always_inline)) {
    if (LIKELY(pos < LC)) { smem[pos] = rem; smem[O_PL + pos] = pl; }
    else { hREM[pos - LC] = rem; hPL[pos - LC] = pl; }
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
    smem[i] = -1;
    smem[O_PL + i] = 0;
  }
  wave_sync();
  // the completion handler runs in the lanes that own the finished slots: keep what it needs in
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
  // statistics: lane k of (acc_hi:acc_lo) is counter SL_k; lanes 0..2 of mx are max U, |P|, |Q|
  uint32_t acc_lo = 0, acc_hi = 0;
  int mx = 0;
  // per-lane partial sums over the requests whose completion this lane handled
  uint32_t lat_lo = 0, lat_hi = 0, use_lo = 0, use_hi = 0;
  int lat_max = 0;
  int trace_left = kp.trace_every > 0 ? kp.trace_every : 0x7fffffff, trace_idx = 0;  // T < 2^30

  auto fail = [&](int code, int t) __attribute__((always_inline)) {
    if (!err) { err = code; err_step = t; }
  };

  // n_t and B_t of slot t0 + lane (Section 2.1: n_t from a known law with mean lambda;
  // Theorem 2: B_t i.i.d. bounded integers with mean b)
  auto draw_slot = [&](uint32_t t0, int& n_out, int& b_out) __attribute__((always_inline)) {
    const DLaw arr = laws[cellp.arrival];
    const uint32_t* __restrict__ arr_thr = kp.blob + arr.off;
    uint32_t w0, w1, w2, w3;
    philox4x32_10(0u, t0 + static_cast<uint32_t>(lane), rep, 0u, kp.seed_lo, kp.seed_hi, w0, w1, w2, w3);
    int n = 0;
    for (int i = 0; i < arr.n; ++i) n += (w0 >= arr_thr[i]) ? 1 : 0;
    n_out = n;
    b_out = cellp.b_floor + ((w1 < cellp.b_frac_thr) ? 1 : 0);
  };

  // Generates the next block of never-activated requests, in arrival order, starting at
  // arrival index fresh_next (requires fresh_next == fb_base + fb_count).
  auto refill_block = [&]() __attribute__((always_inline)) {
    fb_base = fresh_next;
    fb_count = 0;
    while (fb_count == 0 && rd_t <= static_cast<uint32_t>(T)) {
      int n, b;
      draw_slot(rd_t, n, b);
      if (rd_t + static_cast<uint32_t>(lane) > static_cast<uint32_t>(T)) n = 0;
      if (lane == 0) n -= rd_k;
      const int incl = wave_incl_sum(n, lane);
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
      const int owner = wave_incl_max(mark, lane);
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

  // Order-preserving removal of dead slots.
  auto compact = [&]() __attribute__((always_inline)) {
    int out = 0, new_pf = -1;
    if (n_slots <= LC) {
      for (int base = 0; base < n_slots; base += kWave) {
        const int pos = base + lane;
        const int rem = smem[pos], pl = smem[O_PL + pos];
        const v4i rec = ld4(&smem[O_REC + 4 * pos]);
        const bool live = pos < n_slots && (rem > 0 || pl > 0);
        const uint64_t m = __ballot(live);
        const uint64_t pm = __ballot(live && pl > 0);
        const int dst = out + lanes_below(m);
        if (pm != 0 && new_pf < 0) new_pf = out + __popcll(m & ((1ull << __builtin_ctzll(pm)) - 1ull));
        wave_sync();
        if (live) {
          smem[dst] = rem;
          smem[O_PL + dst] = pl;
          st4(&smem[O_REC + 4 * dst], rec);
        }
        wave_sync();
        out += __popcll(m);
      }
      for (int base = out; base < n_slots; base += kWave) {
        const int pos = base + lane;
        if (pos < n_slots) { smem[pos] = -1; smem[O_PL + pos] = 0; }
      }
    } else {
      for (int base = 0; base < n_slots; base += kWave) {
        const int pos = base + lane;
        const bool in = pos < n_slots;
        int rem = -1, pl = 0;
        v4i rec = {0, 0, 0, 0};
        if (in) {
          if (base < LC) {
            rem = smem[pos]; pl = smem[O_PL + pos];
            rec = ld4(&smem[O_REC + 4 * pos]);
          } else {
            rem = hREM[pos - LC]; pl = hPL[pos - LC];
            rec = ld4(&hREC[4 * static_cast<size_t>(pos - LC)]);
          }
        }
        const bool live = in && (rem > 0 || pl > 0);
        const uint64_t m = __ballot(live);
        const uint64_t pm = __ballot(live && pl > 0);
        const int dst = out + lanes_below(m);
        if (pm != 0 && new_pf < 0) new_pf = out + __popcll(m & ((1ull << __builtin_ctzll(pm)) - 1ull));
        wave_sync();
        if (live) slot_store(dst, rem, pl, rec);
        wave_sync();
        out += __popcll(m);
      }
      for (int base = out; base < n_slots; base += kWave) {
        const int pos = base + lane;
        if (pos < n_slots) rem_pl_store(pos, -1, 0);
      }
    }
    wave_sync();
    n_slots = out;
    pf_first = new_pf < 0 ? n_slots : new_pf;
  };

  // Evicts the most recently activated request (Section 3.3: last in, first out); it loses
  // its progress and goes back to the front of Q.
  auto evict_newest = [&](int t) __attribute__((always_inline)) {
    int pos = n_slots - 1;
    int rem = 0, pleft = 0;
    for (; pos >= 0; --pos) {
      rem_pl_load(pos, rem, pleft);
      rem = rfl(rem);
      pleft = rfl(pleft);
      if (rem > 0 || pleft > 0) break;
    }
    if (pos < 0) { fail(FCS_ESTATE, t); return; }
    const v4i rec = rec_load(pos);
    const int l = rfl(rec.x), o = rfl(rec.y);
    if (pleft > 0) { U -= l; n_pf -= 1; }
    else { U -= l + (o - rem); n_dec -= 1; }
    n_live -= 1;
    if (sdepth == SCAP) { fail(FCS_EOVERFLOW, t); return; }
    if (lane == 0) {
      if (sdepth < kStackLds) st4(&smem[O_STK + 4 * sdepth], rec);
      else st4(&hSTK[4 * static_cast<size_t>(sdepth - kStackLds)], rec);
      rem_pl_store(pos, -1, 0);
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
  int x = 0;      // this slot's contribution to the statistics, one counter per lane
  int room = 0, admitted = 0, budget = 0, new_dec = 0;
  int rel_sum = 0, n_done = 0;  // completions of this slot: released footprint and count

  // called where the lanes of mask m0 (flag `mine`) own a request, in slot `pos`, that generated
  // its last token in this slot
  auto complete = [&](bool mine, uint64_t m0, int pos) __attribute__((always_inline)) {
    int relv = 0;
    if (mine) {
      v4i rec;
      if (LIKELY(pos < LC)) rec = ld4(&smem[O_REC + 4 * pos]);
      else rec = ld4(&hREC[4 * static_cast<size_t>(pos - LC)]);
      relv = rec.x + rec.y;                       // l + o, released at the end of the slot
      const int lat = t - rec.z + 1;              // arrival to completion, both slots counted
      const uint32_t s = lat_lo + static_cast<uint32_t>(lat);
      lat_hi += (s < lat_lo) ? 1u : 0u;
      lat_lo = s;
      const uint32_t u = use_lo + static_cast<uint32_t>(rec.y);
      use_hi += (u < use_lo) ? 1u : 0u;
      use_lo = u;
      lat_max = max(lat_max, lat);
      if (hist_v) atomicAdd(reinterpret_cast<uint32_t*>(hist_v) + min(lat >> hist_shift_v, hist_last_v), 1u);
      if (comp_v && rec.w < max_req_v) reinterpret_cast<int32_t*>(comp_v)[rec.w] = t;
    }
    n_done += static_cast<int>(__popcll(m0));
    rel_sum += rdl(relv, __builtin_ctzll(m0));
    uint64_t m = m0 & (m0 - 1);
    while (UNLIKELY(m != 0)) {
      rel_sum += rdl(relv, __builtin_ctzll(m));
      m &= m - 1;
    }
  };
  // completes every request of a four-slots-per-lane block whose entry reached zero and turns
  // the entry into a tombstone
  auto complete_block = [&](v4i& v, int p0) __attribute__((always_inline)) {
    bool any = umin4(v) == 0u;
    uint64_t m = __ballot(any);
    while (m != 0) {  // one pass unless a lane holds two completions
      const int c = v.x == 0 ? 0 : (v.y == 0 ? 1 : (v.z == 0 ? 2 : 3));
      complete(any, m, p0 + c);
      if (any) {
        v.x = c == 0 ? -1 : v.x;
        v.y = c == 1 ? -1 : v.y;
        v.z = c == 2 ? -1 : v.z;
        v.w = c == 3 ? -1 : v.w;
      }
      any = umin4(v) == 0u;
      m = __ballot(any);
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

  auto general_slot = [&]() __attribute__((always_inline)) {
    // ---- 1. arrivals ---------------------------------------------------------------
    if (phase <= 0) {
      x = 0;
      const int wi = (t - 1) & (kWave - 1);
      if (wi == 0) {
        int n, b;
        draw_slot(static_cast<uint32_t>(t), n, b);
        win = n | (b << 16);
        if (UNLIKELY(arrived >= 0x7ffe0000u)) fail(FCS_EOVERFLOW, t);
        if (arr_rec) {  // arrival slots of the requests of this window, by arrival id
          const int tt = t + lane;
          const int ne = tt <= T ? n : 0;
          const int excl = wave_incl_sum(ne, lane) - ne;
          for (int k = 0; k < ne; ++k) {
            const uint32_t id = arrived + static_cast<uint32_t>(excl + k);
            if (id < static_cast<uint32_t>(kp.max_requests)) arr_rec[id] = tt;
          }
        }
      }
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
          if (UNLIKELY(idx >= fb_count)) { fail(FCS_ESTATE, t); break; }
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
          if (n_live < n_slots) compact();
          if (n_slots == CAP) { fail(FCS_EOVERFLOW, t); break; }
        }
        const int pos = n_slots;
        int l;
        if (from_stack) {
          const int d = sdepth - 1;
          v4i rec;
          if (d < kStackLds) rec = ld4(&smem[O_STK + 4 * d]);
          else rec = ld4(&hSTK[4 * static_cast<size_t>(d - kStackLds)]);
          l = rfl(rec.x);
          if (lane == 0) slot_store(pos, -rec.y, l, rec);
          sdepth = d;
        } else {
          l = rdl(fb_l, idx);
          if (lane == idx) {
            const v4i rec = {fb_l, fb_o, fb_t, static_cast<int>(fresh_next)};
            slot_store(pos, -fb_o, fb_l, rec);
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
          int pl, ov;
          if (LIKELY(base < LC)) { pl = smem[O_PL + pos]; ov = smem[O_REC + 4 * pos + 1]; }
          else if (pos < n_slots) { pl = hPL[pos - LC]; ov = hREC[4 * static_cast<size_t>(pos - LC) + 1]; }
          else { pl = 0; ov = 0; }
          uint64_t m = __ballot(pl > 0);
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
              // the chunk that ends the prompt yields token 1: the entry becomes o here and the
              // decode pass of this slot makes it o - 1
              const int o = rdl(ov, i);
              if (lane == 0) rem_pl_store(p, o, 0);
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
        advanced = n_dec;
        const int lim = min(n_slots, LC);
        for (int b0 = 0; b0 < lim; b0 += kLdsBlock) {
          const int p0 = b0 + (lane << 2);
          v4i v = ld4(&smem[p0]);
          dec4(v);
          if (__ballot(umin4(v) == 0u) != 0) complete_block(v, p0);
          st4(&smem[p0], v);
          wave_sync();
        }
        for (int base = LC; base < n_slots; base += kWave) {
          const int pos = base + lane;
          const bool in = pos < n_slots;
          int v = in ? hREM[pos - LC] : -1;
          v -= (v > 0) ? 1 : 0;
          const bool d = in && v == 0;
          const uint64_t dm = __ballot(d);
          if (dm != 0) complete(d, dm, pos);
          if (in) hREM[pos - LC] = d ? -1 : v;
          wave_sync();
        }
      } else {
        // budget binds: the first `budget` already-decoding requests in activation order advance;
        // requests that finished their prompt in this slot (entry == o) take token 1 for free
        int left = budget;
        advanced = 0;
        for (int base = 0; base < n_slots; base += kWave) {
          const int pos = base + lane;
          const bool in = pos < n_slots;
          int v = -1, ov = 0;
          if (in) {
            if (base < LC) { v = smem[pos]; ov = smem[O_REC + 4 * pos + 1]; }
            else { v = hREM[pos - LC]; ov = hREC[4 * static_cast<size_t>(pos - LC) + 1]; }
          }
          const bool dec = v > 0;
          const bool fresh = dec && new_dec > 0 && v == ov;
          const bool old = dec && !fresh;
          const uint64_t om = __ballot(old);
          const bool go = fresh || (old && lanes_below(om) < left);
          const int took = min(static_cast<int>(__popcll(om)), left);
          left -= took;
          advanced += took;
          if (go) v -= 1;
          const bool d = go && v == 0;
          const uint64_t dm = __ballot(d);
          if (dm != 0) complete(d, dm, pos);
          if (go) {
            if (base < LC) smem[pos] = d ? -1 : v; else hREM[pos - LC] = d ? -1 : v;
          }
          wave_sync();
        }
        x = wrl(n_dec - advanced, SL_STALLED, x);
      }
      measure_and_release(advanced + new_dec, qlen);
    }
    if (n_slots - n_live >= kCompactSlack) compact();
  };

  // The common slot (everything in LDS, no eviction, no stall) as hand-scheduled assembly; runs
  // slots until one needs the general code and returns with `phase` set.
  const int lds_base = static_cast<int>(
      reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) int32_t*)smem));
  auto fast_slots = [&]() __attribute__((always_inline)) {
#include "fcs_fast_slots.inc"
  };

  const bool fast_ok = LC >= 2 * kLdsBlock;
  while (t <= T && !err) {
    general_slot();
    ++t;
    phase = 0;
    if (UNLIKELY(!fast_ok) || UNLIKELY(n_slots > LC) || UNLIKELY(err)) continue;
    fast_slots();
  }

  // ---- epilogue: digest of the final state, counters --------------------------------------------
  uint64_t h = 14695981039346656037ull;
  auto mix = [&](uint64_t w) __attribute__((always_inline)) { h = (h ^ w) * 1099511628211ull; };
  if (!err) {
    compact();
    mix(static_cast<uint64_t>(n_slots));
    for (int pos = 0; pos < n_slots; ++pos) {
      int rem, pleft;
      rem_pl_load(pos, rem, pleft);
      rem = rfl(rem);
      pleft = rfl(pleft);
      const v4i rec = rec_load(pos);
      const int l = rfl(rec.x), o = rfl(rec.y), id = rfl(rec.w);
      mix(static_cast<uint64_t>(id));
      mix(static_cast<uint64_t>(rem > 0 ? o - rem : 0));
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
