// Sample-path kernel: one wavefront (= one workgroup) simulates one path of the slot
// model (Section 2.1) under Algorithm 2 or its greedy limit, for slots 1..T.
//
// Data layout per path
//   active set   structure of arrays in activation order with dead slots left in place
//                ("tombstones"), compacted when kCompactSlack of them have accumulated.
//                Slots [0, lcap) live in LDS, slots [lcap, lcap+hcap) in a per-path spill
//                region of the workspace.  F_REM holds o - j for a decoding request and a
//                negative value otherwise, so the decode growth of a slot (Section 2.1: one
//                more token per active request) is one decrement per live slot and a
//                request completes when it reaches zero.
//   waiting queue  never materialised for requests that were not activated yet: arrivals
//                are a pure function of (seed, replica, slot, index), so the FIFO of fresh
//                requests is re-generated, 64 arrivals at a time, when they are admitted.
//                Evicted requests (which re-enter at the front, newest eviction deepest)
//                form a stack: first kStackLds entries in LDS, the rest in the spill region.
//   scalars      usage U, |P|, counts and all statistics stay in scalar registers.
#include <hip/hip_runtime.h>

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

__device__ __forceinline__ int lane_id() { return static_cast<int>(threadIdx.x); }

__device__ __forceinline__ int rfl(int v) { return __builtin_amdgcn_readfirstlane(v); }

__device__ __forceinline__ int wave_incl_sum(int v) {
  const int lane = lane_id();
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    const int o = __shfl_up(v, d, kWave);
    if (lane >= d) v += o;
  }
  return v;
}

__device__ __forceinline__ int wave_incl_max(int v) {
  const int lane = lane_id();
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    const int o = __shfl_up(v, d, kWave);
    if (lane >= d) v = max(v, o);
  }
  return v;
}

// Lanes of the wavefront exchange data through LDS and the spill region (lane 0 writes a slot
// that lane k reads later).  To the compiler each lane is a separate thread, so every such
// hand-over needs a wavefront-scope release/acquire; the hardware executes the memory
// operations of one wavefront in order, so this emits no instruction.
__device__ __forceinline__ void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ __forceinline__ int lanes_below(uint64_t mask) {
  return __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(mask >> 32),
                                   __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(mask), 0u));
}

__global__ __launch_bounds__(kWave) void fcs_sim_kernel(const KParams kp) {
  extern __shared__ int32_t smem[];
  const int lane = lane_id();
  const int path = static_cast<int>(blockIdx.x);
  if (path >= kp.n_paths) return;

  const int cell_i = path / kp.n_replicas;
  const uint32_t rep = kp.replica_base + static_cast<uint32_t>(path - cell_i * kp.n_replicas);
  const DLaw* __restrict__ laws = reinterpret_cast<const DLaw*>(kp.blob + kp.laws_off);
  const DCell cellp = reinterpret_cast<const DCell*>(kp.blob + kp.cells_off)[cell_i];
  const DLaw arr = laws[cellp.arrival];
  const uint32_t* __restrict__ arr_thr = kp.blob + arr.off;
  const uint32_t* __restrict__ class_thr = kp.blob + kp.class_off;
  const bool greedy = cellp.policy == FCS_POLICY_GREEDY;
  const int M = kp.M, T = kp.n_steps;
  const int LC = kp.lcap, HC = kp.hcap, HS = kp.hscap;
  const int CAP = LC + HC;            // slots of the active set
  const int SCAP = kStackLds + HS;    // entries of the evicted stack
  int32_t* __restrict__ hA = kp.spill + static_cast<size_t>(path) * kp.spill_stride;
  int32_t* __restrict__ hS = hA + static_cast<size_t>(F_NFIELDS) * HC;
  const int S_OFF = F_NFIELDS * LC;
  const int SCR = S_OFF + S_NFIELDS * kStackLds;

  // ---- tiered accessors ------------------------------------------------------
  auto a_get = [&](int f, int pos) -> int32_t {
    return pos < LC ? smem[f * LC + pos] : hA[static_cast<size_t>(f) * HC + (pos - LC)];
  };
  auto a_set = [&](int f, int pos, int32_t v) {
    if (pos < LC) smem[f * LC + pos] = v;
    else hA[static_cast<size_t>(f) * HC + (pos - LC)] = v;
  };
  auto s_get = [&](int f, int d) -> int32_t {
    return d < kStackLds ? smem[S_OFF + f * kStackLds + d]
                         : hS[static_cast<size_t>(f) * HS + (d - kStackLds)];
  };
  auto s_set = [&](int f, int d, int32_t v) {
    if (d < kStackLds) smem[S_OFF + f * kStackLds + d] = v;
    else hS[static_cast<size_t>(f) * HS + (d - kStackLds)] = v;
  };

  // ---- output rows of this path ------------------------------------------------
  uint32_t* hist = kp.out.hist ? kp.out.hist + static_cast<size_t>(path) * kp.hist_bins : nullptr;
  int32_t* arr_rec = kp.out.arrival_step
                         ? kp.out.arrival_step + static_cast<size_t>(path) * kp.max_requests : nullptr;
  int32_t* comp_rec = kp.out.completion_step
                          ? kp.out.completion_step + static_cast<size_t>(path) * kp.max_requests : nullptr;
  int32_t* trq = kp.out.trace_q ? kp.out.trace_q + static_cast<size_t>(path) * kp.n_trace : nullptr;
  int32_t* tru = kp.out.trace_u ? kp.out.trace_u + static_cast<size_t>(path) * kp.n_trace : nullptr;
  if (hist) for (int i = lane; i < kp.hist_bins; i += kWave) hist[i] = 0u;
  if (arr_rec) for (int i = lane; i < kp.max_requests; i += kWave) arr_rec[i] = 0;
  if (comp_rec) for (int i = lane; i < kp.max_requests; i += kWave) comp_rec[i] = 0;
  wave_sync();
  for (int i = lane; i < LC; i += kWave) {
    smem[F_REM * LC + i] = -1;
    smem[F_PLEFT * LC + i] = 0;
  }
  wave_sync();

  // ---- state (wave-uniform) ----------------------------------------------------
  int U = 0;           // sum over P of (l + j)
  int n_live = 0;      // |P|
  int n_dec = 0;       // requests of P that are decoding
  int n_pf = 0;        // requests of P that are still prefilling
  int n_slots = 0;     // slots in use, dead ones included
  int pf_first = 0;    // no prefilling request sits below this slot
  int sdepth = 0;      // evicted requests waiting at the front of Q
  uint32_t arrived = 0, fresh_next = 0;  // arrivals so far; id of the next never-activated request
  int err = 0, err_step = 0;

  // fresh-request block: lane i holds arrival fb_base + i
  int fb_l = 0, fb_o = 0, fb_t = 0;
  uint32_t fb_base = 0;
  int fb_count = 0;
  uint32_t rd_t = 1;   // reader cursor: slot ...
  int rd_k = 0;        // ... and arrivals of that slot already handed out
  int win = 0;         // lane i: n_t | B_t << 16 for slot win_t0 + i

  uint64_t c_act = 0, c_done = 0, c_evict = 0, c_ovf = 0, c_sum_u = 0, c_sum_p = 0, c_sum_q = 0;
  uint64_t c_dec_tok = 0, c_pf_tok = 0, c_useful = 0, c_stalled = 0, c_sum_lat = 0;
  int c_max_lat = 0, c_max_u = 0, c_max_p = 0, c_max_q = 0;
  int trace_left = kp.trace_every, trace_idx = 0;

  auto fail = [&](int code, int t) {
    if (!err) { err = code; err_step = t; }
  };

  // n_t and B_t of slot t0 + lane (Section 2.1: n_t from a known law with mean lambda;
  // Theorem 2: B_t i.i.d. bounded integers with mean b)
  auto draw_slot = [&](uint32_t t0, int& n_out, int& b_out) {
    uint32_t w0, w1, w2, w3;
    philox4x32_10(0u, t0 + static_cast<uint32_t>(lane), rep, 0u, kp.seed_lo, kp.seed_hi, w0, w1, w2, w3);
    int n = 0;
    for (int i = 0; i < arr.n; ++i) n += (w0 >= arr_thr[i]) ? 1 : 0;
    n_out = n;
    b_out = cellp.b_floor + ((w1 < cellp.b_frac_thr) ? 1 : 0);
  };

  // value = lo + #{thr <= u} by bisection inside the guide bucket of u
  auto invert = [&](const DLaw& L, uint32_t u, bool on) -> int {
    int lo = 0, hi = 0;
    if (on && L.n > 0) {
      const uint32_t* g = kp.blob + L.goff;
      const uint32_t b = u >> 24;
      lo = static_cast<int>(g[b]);
      hi = static_cast<int>(g[b + 1]);
    }
    const uint32_t* th = kp.blob + L.off;
    for (int it = 0; it < 34 && __any(lo < hi); ++it) {
      if (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (th[mid] <= u) lo = mid + 1; else hi = mid;
      }
    }
    return L.lo + lo;
  };

  // Generates the next block of never-activated requests, in arrival order, starting at
  // arrival index fresh_next (requires fresh_next == fb_base + fb_count).
  auto refill_block = [&]() {
    fb_base = fresh_next;
    fb_count = 0;
    while (fb_count == 0 && rd_t <= static_cast<uint32_t>(T)) {
      int n, b;
      draw_slot(rd_t, n, b);
      if (rd_t + static_cast<uint32_t>(lane) > static_cast<uint32_t>(T)) n = 0;
      if (lane == 0) n -= rd_k;
      const int incl = wave_incl_sum(n);
      const int total = __builtin_amdgcn_readlane(incl, kWave - 1);
      const int excl = incl - n;
      if (total == 0) { rd_t += kWave; rd_k = 0; continue; }
      // expand: output lane i takes the slot s with excl[s] <= i < incl[s]
      smem[SCR + lane] = 0;
      wave_sync();
      if (n > 0 && excl < kWave) smem[SCR + excl] = lane + 1;
      wave_sync();
      const int mark = smem[SCR + lane];
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
      int cls = 0;
      for (int i = 0; i + 1 < kp.n_classes; ++i) cls += (w0 >= class_thr[i]) ? 1 : 0;
      const DLaw pl = laws[kp.n_arrival_laws + cls];
      const DLaw dl = laws[kp.n_arrival_laws + kp.n_classes + cls];
      fb_l = invert(pl, w1, valid);
      fb_o = invert(dl, w2, valid);
      fb_t = static_cast<int>(ta);
      fb_count = cnt;
      if (total <= kWave) {
        rd_t += kWave;
        rd_k = 0;
      } else {
        const int s63 = __builtin_amdgcn_readlane(src, kWave - 1);
        rd_k = __builtin_amdgcn_readlane(k, kWave - 1) + 1;
        rd_t += static_cast<uint32_t>(s63);
      }
      if (arr_rec && valid) {
        const uint32_t id = fb_base + static_cast<uint32_t>(lane);
        if (id < static_cast<uint32_t>(kp.max_requests)) arr_rec[id] = fb_t;
      }
    }
  };

  // Order-preserving removal of dead slots.
  auto compact = [&]() {
    int out = 0, new_pf = -1;
    for (int base = 0; base < n_slots; base += kWave) {
      const int pos = base + lane;
      const bool in = pos < n_slots;
      int f[F_NFIELDS];
#pragma unroll
      for (int q = 0; q < F_NFIELDS; ++q) f[q] = in ? a_get(q, pos) : 0;
      const bool live = in && (f[F_REM] > 0 || f[F_PLEFT] > 0);
      const uint64_t m = __ballot(live);
      const int dst = out + lanes_below(m);
      const uint64_t pm = __ballot(live && f[F_PLEFT] > 0);
      if (pm != 0 && new_pf < 0) {
        const int first = __builtin_ctzll(pm);
        new_pf = out + __popcll(m & ((1ull << first) - 1ull));
      }
      if (live) {
#pragma unroll
        for (int q = 0; q < F_NFIELDS; ++q) a_set(q, dst, f[q]);
      }
      wave_sync();
      out += __popcll(m);
    }
    for (int base = out; base < n_slots; base += kWave) {
      const int pos = base + lane;
      if (pos < n_slots) { a_set(F_REM, pos, -1); a_set(F_PLEFT, pos, 0); }
    }
    wave_sync();
    n_slots = out;
    pf_first = new_pf < 0 ? n_slots : new_pf;
  };

  // Moves the head of Q into P (Algorithm 2: pick by FIFO, activate).
  auto admit_head = [&](int t) {
    int id, l, o, ta;
    if (sdepth > 0) {
      const int d = sdepth - 1;
      id = rfl(s_get(S_ID, d)); l = rfl(s_get(S_L, d)); o = rfl(s_get(S_O, d)); ta = rfl(s_get(S_TARR, d));
      sdepth = d;
    } else {
      if (static_cast<int>(fresh_next - fb_base) >= fb_count) refill_block();
      const int idx = static_cast<int>(fresh_next - fb_base);
      if (idx >= fb_count) { fail(FCS_ESTATE, t); return; }
      id = static_cast<int>(fresh_next);
      l = __builtin_amdgcn_readlane(fb_l, idx);
      o = __builtin_amdgcn_readlane(fb_o, idx);
      ta = __builtin_amdgcn_readlane(fb_t, idx);
      fresh_next += 1u;
    }
    if (n_slots == CAP) {
      if (n_live < n_slots) compact();
      if (n_slots == CAP) { fail(FCS_EOVERFLOW, t); return; }
    }
    const int pos = n_slots;
    if (lane == 0) {
      a_set(F_REM, pos, -1); a_set(F_PLEFT, pos, l); a_set(F_L, pos, l);
      a_set(F_O, pos, o); a_set(F_TARR, pos, ta); a_set(F_ID, pos, id);
    }
    wave_sync();
    n_slots = pos + 1;
    if (n_pf == 0 || pf_first > pos) pf_first = pos;
    U += l;
    n_live += 1;
    n_pf += 1;
    c_act += 1;
  };

  auto head_prompt = [&](int t) -> int {
    if (sdepth > 0) return rfl(s_get(S_L, sdepth - 1));
    if (static_cast<int>(fresh_next - fb_base) >= fb_count) refill_block();
    const int idx = static_cast<int>(fresh_next - fb_base);
    if (idx >= fb_count) { fail(FCS_ESTATE, t); return M; }
    return __builtin_amdgcn_readlane(fb_l, idx);
  };

  // Evicts the most recently activated request (Section 3.3: last in, first out).
  auto evict_newest = [&](int t) {
    int pos = n_slots - 1;
    int rem = 0, pleft = 0;
    for (; pos >= 0; --pos) {
      rem = rfl(a_get(F_REM, pos));
      pleft = rfl(a_get(F_PLEFT, pos));
      if (rem > 0 || pleft > 0) break;
    }
    if (pos < 0) { fail(FCS_ESTATE, t); return; }
    const int l = rfl(a_get(F_L, pos)), o = rfl(a_get(F_O, pos));
    const int ta = rfl(a_get(F_TARR, pos)), id = rfl(a_get(F_ID, pos));
    if (pleft > 0) { U -= l; n_pf -= 1; }
    else { U -= l + (o - rem); n_dec -= 1; }
    n_live -= 1;
    c_evict += 1;
    if (sdepth == SCAP) { fail(FCS_EOVERFLOW, t); return; }
    if (lane == 0) {
      s_set(S_ID, sdepth, id); s_set(S_L, sdepth, l); s_set(S_O, sdepth, o); s_set(S_TARR, sdepth, ta);
      a_set(F_REM, pos, -1);
      a_set(F_PLEFT, pos, 0);
    }
    wave_sync();
    sdepth += 1;
    n_slots = pos;
    if (pf_first > n_slots) pf_first = n_slots;
  };

  // per-slot accumulators of completions (released after U_t is measured: Section 2.1)
  int rel_sum = 0, n_done = 0;
  auto complete_at = [&](int pos, int t) {
    const int l = rfl(a_get(F_L, pos)), o = rfl(a_get(F_O, pos));
    const int ta = rfl(a_get(F_TARR, pos)), id = rfl(a_get(F_ID, pos));
    const int lat = t - ta + 1;
    rel_sum += l + o;
    n_done += 1;
    c_sum_lat += static_cast<uint64_t>(lat);
    c_max_lat = max(c_max_lat, lat);
    c_useful += static_cast<uint64_t>(o);
    if (lane == 0) {
      a_set(F_REM, pos, -1);
      if (hist) atomicAdd(&hist[min(lat >> kp.hist_shift, kp.hist_bins - 1)], 1u);
      if (comp_rec && id < kp.max_requests) comp_rec[id] = t;
    }
    wave_sync();
  };

  // =============================== slots 1..T ====================================
  for (int t = 1; t <= T && !err; ++t) {
    // ---- 1. arrivals -------------------------------------------------------------
    const int wi = (t - 1) & (kWave - 1);
    if (wi == 0) {
      int n, b;
      draw_slot(static_cast<uint32_t>(t), n, b);
      win = n | (b << 16);
    }
    const int nb = __builtin_amdgcn_readlane(win, wi);
    const int n_t = nb & 0xffff, B_t = nb >> 16;
    arrived += static_cast<uint32_t>(n_t);
    if (arrived >= 0x7fffff00u) fail(FCS_EOVERFLOW, t);

    // ---- 2. admission ------------------------------------------------------------
    int qlen = sdepth + static_cast<int>(arrived - fresh_next);
    if (!greedy) {
      int k = min(B_t, qlen);
      for (; k > 0 && !err; --k) admit_head(t);
    } else {
      while (qlen > 0 && !err) {
        const int lh = head_prompt(t);
        if (U + n_live + lh + 1 > M) break;
        admit_head(t);
        qlen -= 1;
      }
    }

    // ---- 3. overflow ---------------------------------------------------------------
    if (U + n_live > M) {
      c_ovf += 1;
      do { evict_newest(t); } while (U + n_live > M && !err);
    }
    if (err) break;
    qlen = sdepth + static_cast<int>(arrived - fresh_next);

    // ---- 4a. chunked prefill under the token budget, activation order ---------------
    int budget = kp.tau;
    int new_dec = 0;
    if (n_pf > 0) {
      int todo = n_pf;
      int base = pf_first;
      int first_left = -1;
      while (todo > 0 && budget > 0 && base < n_slots) {
        const int pos = base + lane;
        const int pl = pos < n_slots ? a_get(F_PLEFT, pos) : 0;
        uint64_t m = __ballot(pl > 0);
        int last_i = kWave - 1;
        while (m != 0 && budget > 0) {
          const int i = __builtin_ctzll(m);
          m &= m - 1;
          const int p = base + i;
          int left = __builtin_amdgcn_readlane(pl, i);
          const int d = min(min(kp.chunk, left), budget);
          left -= d;
          budget -= d;
          c_pf_tok += static_cast<uint64_t>(d);
          todo -= 1;
          if (left == 0) {
            // the chunk that ends the prompt yields token 1: enter decode with j = 0 here,
            // the decode pass of this slot makes it j = 1
            const int o = rfl(a_get(F_O, p));
            if (lane == 0) { a_set(F_PLEFT, p, 0); a_set(F_REM, p, o); }
            wave_sync();
            new_dec += 1;
          } else {
            if (lane == 0) a_set(F_PLEFT, p, left);
            wave_sync();
            if (first_left < 0) first_left = p;
          }
          last_i = i;
        }
        if (m != 0) {  // budget ran out inside this chunk
          if (first_left < 0) first_left = base + __builtin_ctzll(m);
          break;
        }
        (void)last_i;
        base += kWave;
      }
      if (first_left >= 0) pf_first = first_left;
      else pf_first = (todo > 0) ? min(base, n_slots) : n_slots;
      n_pf -= new_dec;
    }

    // ---- 4b. decode growth: one token per decoding request while budget lasts --------
    rel_sum = 0;
    n_done = 0;
    int advanced;  // old decoders that got a token
    if (budget >= n_dec) {
      advanced = n_dec;
      const int lim = min(n_slots, LC);
      for (int b0 = 0; b0 < lim; b0 += kLdsBlock) {
        const int p0 = b0 + (lane << 2);
        v4i v = *reinterpret_cast<v4i*>(&smem[F_REM * LC + p0]);
        v -= 1;
        *reinterpret_cast<v4i*>(&smem[F_REM * LC + p0]) = v;
        wave_sync();
        const uint32_t mn = min(min(static_cast<uint32_t>(v.x), static_cast<uint32_t>(v.y)),
                                min(static_cast<uint32_t>(v.z), static_cast<uint32_t>(v.w)));
        if (__ballot(mn == 0u) != 0) {
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            uint64_t m = __ballot(v[c] == 0);
            while (m != 0) {
              const int i = __builtin_ctzll(m);
              m &= m - 1;
              complete_at(b0 + (i << 2) + c, t);
            }
          }
        }
      }
      for (int base = LC; base < n_slots; base += kWave) {
        const int pos = base + lane;
        const bool in = pos < n_slots;
        int v = in ? hA[static_cast<size_t>(F_REM) * HC + (pos - LC)] : -1;
        v -= 1;
        if (in) hA[static_cast<size_t>(F_REM) * HC + (pos - LC)] = v;
        wave_sync();
        uint64_t m = __ballot(in && v == 0);
        while (m != 0) {
          const int i = __builtin_ctzll(m);
          m &= m - 1;
          complete_at(base + i, t);
        }
      }
    } else {
      // budget binds: the first `budget` old decoders in activation order advance; requests
      // that finished their prompt in this slot (rem == o) take their first token for free
      int left = budget;
      advanced = 0;
      for (int base = 0; base < n_slots; base += kWave) {
        const int pos = base + lane;
        const bool in = pos < n_slots;
        int v = in ? a_get(F_REM, pos) : -1;
        const bool dec = v > 0;
        const bool fresh = dec && new_dec > 0 && v == a_get(F_O, pos);
        const bool old = dec && !fresh;
        const uint64_t om = __ballot(old);
        const bool go = fresh || (old && lanes_below(om) < left);
        const int took = min(__popcll(om), left);
        left -= took;
        advanced += took;
        if (go) { v -= 1; a_set(F_REM, pos, v); }
        wave_sync();
        uint64_t m = __ballot(go && v == 0);
        while (m != 0) {
          const int i = __builtin_ctzll(m);
          m &= m - 1;
          complete_at(base + i, t);
        }
      }
      c_stalled += static_cast<uint64_t>(n_dec - advanced);
    }
    c_dec_tok += static_cast<uint64_t>(advanced + new_dec);
    U += advanced + new_dec;
    n_dec += new_dec;

    // ---- 5. measure -------------------------------------------------------------------
    c_sum_u += static_cast<uint64_t>(U);
    c_sum_p += static_cast<uint64_t>(n_live);
    c_sum_q += static_cast<uint64_t>(qlen);
    c_max_u = max(c_max_u, U);
    c_max_p = max(c_max_p, n_live);
    c_max_q = max(c_max_q, qlen);
    if (kp.trace_every > 0 && --trace_left == 0) {
      trace_left = kp.trace_every;
      if (lane == 0) {
        if (trq) trq[trace_idx] = qlen;
        if (tru) tru[trace_idx] = U;
      }
      trace_idx += 1;
    }

    // ---- 6. complete: release the footprint at the end of the slot -----------------------
    U -= rel_sum;
    n_live -= n_done;
    n_dec -= n_done;
    c_done += static_cast<uint64_t>(n_done);
    if (n_slots - n_live >= kCompactSlack) compact();
  }

  // ---- epilogue: arrival records of requests never activated, digest, counters ----------
  if (!err && arr_rec) {
    uint32_t keep = fresh_next;
    int guard = 0;
    while (fb_base + static_cast<uint32_t>(fb_count) < arrived && guard++ < (1 << 24)) {
      fresh_next = fb_base + static_cast<uint32_t>(fb_count);
      if (fresh_next >= static_cast<uint32_t>(kp.max_requests)) break;
      refill_block();
      if (fb_count == 0) break;
    }
    fresh_next = keep;
  }
  uint64_t h = 14695981039346656037ull;
  auto mix = [&](uint64_t x) { h = (h ^ x) * 1099511628211ull; };
  if (!err) {
    compact();
    mix(static_cast<uint64_t>(n_slots));
    for (int pos = 0; pos < n_slots; ++pos) {
      const int rem = rfl(a_get(F_REM, pos)), pleft = rfl(a_get(F_PLEFT, pos));
      const int l = rfl(a_get(F_L, pos)), o = rfl(a_get(F_O, pos)), id = rfl(a_get(F_ID, pos));
      mix(static_cast<uint64_t>(id));
      mix(static_cast<uint64_t>(rem > 0 ? o - rem : 0));
      mix(static_cast<uint64_t>(l - pleft));
    }
    mix(static_cast<uint64_t>(sdepth));
    for (int d = sdepth - 1; d >= 0; --d) mix(static_cast<uint64_t>(rfl(s_get(S_ID, d))));
    mix(static_cast<uint64_t>(arrived - fresh_next));
  }
  if (lane == 0) {
    uint64_t* C = kp.out.counters + static_cast<size_t>(path) * FCS_N_COUNTERS;
    C[FCS_C_ARRIVED] = arrived;
    C[FCS_C_ACTIVATIONS] = c_act;
    C[FCS_C_COMPLETED] = c_done;
    C[FCS_C_EVICTIONS] = c_evict;
    C[FCS_C_OVERFLOW_STEPS] = c_ovf;
    C[FCS_C_SUM_U] = c_sum_u;
    C[FCS_C_SUM_P] = c_sum_p;
    C[FCS_C_SUM_Q] = c_sum_q;
    C[FCS_C_DECODE_TOKENS] = c_dec_tok;
    C[FCS_C_PREFILL_TOKENS] = c_pf_tok;
    C[FCS_C_USEFUL_TOKENS] = c_useful;
    C[FCS_C_STALLED] = c_stalled;
    C[FCS_C_SUM_LATENCY] = c_sum_lat;
    C[FCS_C_MAX_LATENCY] = static_cast<uint64_t>(c_max_lat);
    C[FCS_C_MAX_U] = static_cast<uint64_t>(c_max_u);
    C[FCS_C_MAX_P] = static_cast<uint64_t>(c_max_p);
    C[FCS_C_MAX_Q] = static_cast<uint64_t>(c_max_q);
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
