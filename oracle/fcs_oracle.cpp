// Plain CPU oracle for the slot-level model of one LLM-serving worker and the
// flow-control admission rules (Section 2.1; Algorithm 2, Section 3.3; Algorithm 1,
// Section 3.2).
//
// THIS FILE IS TEST INFRASTRUCTURE.  It is the slow, obviously-correct statement
// of what a sample path is; only the tests, the smoke check and the benchmark's
// CPU-baseline leg may call it.  It shares no code with the GPU engine: it has
// its own Philox4x32-10, its own table inversion, its own queue mechanics, its
// own counter layout.  Every quantity is recomputed from its definition (for
// instance the KV usage is summed over the active set whenever it is needed).
//
// Model (per replica, slots t = 1..T; Q = waiting FIFO, P = active set in
// activation order):
//   1. arrivals       Section 2.1: n_t requests join the tail of Q.
//   2. admission      FLOW  : Algorithm 2, move min(B_t, |Q|) head requests to P, no fit test.
//                             B_t: floor(b) + Bernoulli(b - floor(b)), or drawn from any bounded
//                             integer law (both i.i.d. as Theorem 2 asks), or the deterministic
//                             floor(t b) - floor((t - 1) b) of a credit accumulator.
//                     GREEDY: the b -> infinity limit described after Theorem 2, with the
//                             "initial memory l+1" fit test of Section 4.1: move the head
//                             while usage-after-this-slot + l + 1 <= M.
//                     ALPHA : alpha-protection greedy baseline of Section 4.1: as GREEDY but
//                             against (1 - alpha) M; on overflow (step 3) ALL active requests
//                             go back to the waiting queue.
//                     MC    : memory-check benchmark of Section 4.1: first come first served, the
//                             head moves only if the memory stays within M in every future slot
//                             when all requests are taken to produce the longest possible output
//                             (unknown request types), or each its own output (known types).
//                     CLASSES: Algorithm 1 (known lengths): every class k has its own arrival
//                             stream n_{t,k}, its own FIFO and an integer budget b_k; in
//                             class order, min(b_k, |Q_k|) head requests of class k move
//                             to P.  There is no overflow branch in Algorithm 1 (Theorem 1
//                             keeps the usage below M when sum_k b_k w_k < M): step 3 only
//                             counts the slots in which the provisioned usage exceeds M.
//   3. overflow       Algorithm 2 "if Overflow": the usage this slot is about to reach is
//                     sum(l+j) + |P| (each active request may gain one token); while it
//                     exceeds M evict the most recently activated request (LIFO rule of
//                     Section 3.3); evicted requests lose all progress and go back to the
//                     FRONT of Q (they keep their place by arrival order).
//   4. process        token budget tau, chunk c (extension; with c >= l_max and tau = inf
//                     it is the paper's "process all requests in P", where the activation
//                     slot already yields token 1, cf. the expression for U_t in the proof
//                     of Theorem 2): first the prefilling requests in activation order,
//                     each advancing min(c, l-p, budget left), the slot that finishes the
//                     prompt also yields the first token at no extra budget; then the
//                     requests that were already decoding, in activation order, one token
//                     each while budget lasts, the rest stall.
//   5. measure        U_t = sum(l+j) over P (Section 2.1), |P_t|, |Q_t|.
//   6. complete       j == o: completion slot c_i = t, footprint released at the end of
//                     the same slot (Section 2.1); latency c_i - t_i + 1.
//
// Random draws: Philox4x32-10 (Salmon et al., SC'11), key = (seed lo, seed hi),
// counter = (k, t, replica, purpose); purpose 0, k = 0: word0 -> n_t, word1 -> B_t;
// purpose 1, k = index of the arrival within its slot: word0 -> class, word1 -> l,
// word2 -> o; purpose 2 (CLASSES), k = class: word0 -> n_{t,k}, and the requests of class k
// all have l = lo of its prompt law and o = lo of its decode law (both must be point laws);
// their ids are (index within the class) * n_classes + k.  Each word is inverted against a
// uint32 threshold table: value = lo + #{i : u >= thr[i]}.
//
// parity unpinned: the budget order of step 4, the provisioned-usage reading of
// "Overflow" in step 3 and the front-of-queue re-entry are this oracle's readings of
// passages the paper leaves open; they are pinned only by hand-computed trajectories.
// The same holds for ALPHA's use of that provisioned usage in its fit test and for keeping the
// prefill-first order of step 4 under it (Section 4.1 says it "prioritizes existing token jobs",
// which the one-token-per-active-request slot model already does when no token budget binds).
// Slots of variable duration (time_c0, time_cp, time_cd) are a linear stand-in for the batch times of
// Section 4.2, which the paper takes from a simulator: the form is this oracle's choice.
// The MC rule as a whole is a reading of one sentence of Section 4.1 (the rule comes from a cited
// paper): usage checked in every future slot, all outputs taken as one common longest length, or,
// with known request types, each as what it is.
#include <algorithm>
#include <atomic>
#include <cstdint>
#include <cstring>
#include <deque>
#include <thread>
#include <vector>

extern "C" {

struct fo_law {
  int32_t lo;
  int32_t n_thr;
  const uint32_t* thr;
};

struct fo_config {
  int32_t policy;  // 0 FLOW, 1 GREEDY, 2 CLASSES, 3 ALPHA, 4 MC
  int32_t n_classes;
  int64_t capacity;
  int64_t token_budget;
  int64_t prefill_chunk;
  int32_t b_floor;
  uint32_t b_frac_thr;
  fo_law arrivals;
  const uint32_t* class_thr;  // n_classes - 1
  const fo_law* prompt;       // n_classes
  const fo_law* decode;       // n_classes
  int32_t trace_every;
  int32_t hist_bins;
  int32_t hist_shift;
  int32_t reserved;
  int64_t max_requests;
  // forced inputs for hand-computed trajectories (n_forced < 0: draw from Philox)
  int64_t n_forced;
  const int32_t* forced_t;
  const int32_t* forced_l;
  const int32_t* forced_o;
  int64_t n_forced_B;  // 0: draw B_t; else B_t = forced_B[min(t, n) - 1]
  const int32_t* forced_B;
  // CLASSES only
  const fo_law* class_arrivals;  // n_classes laws of n_{t,k}
  const int32_t* class_budget;   // n_classes budgets b_k
  const int32_t* forced_cls;     // class of each forced arrival (with n_forced >= 0)
  // ALPHA only
  int64_t protect_limit;  // floor((1 - alpha) M): what admission may fill
  // FLOW: how B_t is formed (Theorem 2 asks for i.i.d. bounded nonnegative integers with mean b)
  int32_t budget_mode;    // 0: b_floor + Bernoulli; 1: drawn from budget_law; 2: credit accumulator
  int32_t reserved2;
  fo_law budget_law;      // mode 1: B_t = lo + #{thr <= word 1}
  int64_t budget_b16;     // mode 2: b in units of 2^-16; B_t = floor(t b) - floor((t - 1) b)
  // MC only
  int64_t assumed_o;      // output length every request is taken to reach in the prediction; 0: its own (known types)
  // Slots of variable duration (all three 0: every slot lasts one unit).  Time runs in units of the
  // arrival law: n_u requests arrive in unit u; slot t starts at time tau_t (tau_1 = 1), sees the
  // arrivals of the units up to tau_t, and lasts d_t = c0 + cp (prompt tokens it processed) + cd
  // (output tokens it generated) units.
  int64_t time_c0, time_cp, time_cd;
};

enum {
  FO_COMPLETED = 0,
  FO_ARRIVED,
  FO_EVICTIONS,
  FO_ACTIVATIONS,
  FO_SUM_P,
  FO_SUM_Q,
  FO_SUM_U,
  FO_OVERFLOW_STEPS,
  FO_SUM_LATENCY,
  FO_MAX_LATENCY,
  FO_USEFUL_TOKENS,
  FO_DECODE_TOKENS,
  FO_PREFILL_TOKENS,
  FO_STALLED,  // request-slots in which a decoding request got no token
  FO_MAX_P,
  FO_MAX_Q,
  FO_MAX_U,
  FO_FINAL_P,
  FO_FINAL_Q,
  FO_FINAL_U,
  FO_DIGEST,
  FO_ELAPSED,  // time units the T slots took (T when every slot lasts one unit)
  FO_N_COUNTERS
};

struct fo_outputs {
  uint64_t* counters;        // [n_ids][FO_N_COUNTERS]
  int32_t* trace_q;          // [n_ids][n_steps / trace_every] or null
  int32_t* trace_u;          // same
  uint32_t* hist;            // [n_ids][hist_bins] or null
  int32_t* arrival_step;     // [n_ids][max_requests] or null (0 = no such request)
  int32_t* completion_step;  // same (0 = not completed)
  int32_t* first_activation; // same, oracle-only
  int32_t* last_activation;  // same, oracle-only
  int32_t* req_l;            // same, oracle-only
  int32_t* req_o;            // same, oracle-only
  int32_t* step_u;           // [n_ids][n_steps] or null, oracle-only
  int32_t* step_p;
  int32_t* step_q;
  int32_t* step_n;           // arrivals drawn in each slot
  int32_t* step_b;           // activation budget B_t of each slot (FLOW)
};

}  // extern "C"

namespace {

// ---- Philox4x32-10, written from the published definition ------------------
inline void mulhilo(uint32_t a, uint32_t b, uint32_t& hi, uint32_t& lo) {
  uint64_t p = static_cast<uint64_t>(a) * static_cast<uint64_t>(b);
  hi = static_cast<uint32_t>(p >> 32);
  lo = static_cast<uint32_t>(p);
}

void philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    if (round > 0) {
      k0 += 0x9E3779B9u;
      k1 += 0xBB67AE85u;
    }
    uint32_t hi0, lo0, hi1, lo1;
    mulhilo(0xD2511F53u, c0, hi0, lo0);
    mulhilo(0xCD9E8D57u, c2, hi1, lo1);
    uint32_t n0 = hi1 ^ c1 ^ k0;
    uint32_t n1 = lo1;
    uint32_t n2 = hi0 ^ c3 ^ k1;
    uint32_t n3 = lo0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// value = lo + number of thresholds that are <= u
int64_t invert(const fo_law& law, uint32_t u) {
  int64_t n = 0;
  for (int32_t i = 0; i < law.n_thr; ++i)
    if (u >= law.thr[i]) ++n;
  return law.lo + n;
}

// The same by bisection (thresholds are sorted); used on the long tables.
int64_t invert_sorted(const fo_law& law, uint32_t u) {
  const uint32_t* e = std::upper_bound(law.thr, law.thr + law.n_thr, u);
  return law.lo + (e - law.thr);
}

struct Request {
  int64_t id, l, o, t_arr;
  int64_t cls = 0;
  int64_t p = 0;  // prompt tokens prefilled
  int64_t j = 0;  // output tokens generated
  bool was_active = false;
  bool decoding_at_slot_start = false;
};

uint64_t fnv_step(uint64_t h, uint64_t word) { return (h ^ word) * 1099511628211ull; }

int64_t usage(const std::vector<Request>& P) {  // Section 2.1: sum of (l_i + j_i)
  int64_t u = 0;
  for (const Request& r : P) u += r.l + r.j;
  return u;
}

void simulate(const fo_config& cfg, int64_t replica, int64_t T, uint64_t seed, int64_t slot,
              const fo_outputs& out) {
  const uint32_t key[2] = {static_cast<uint32_t>(seed), static_cast<uint32_t>(seed >> 32)};
  const int64_t M = cfg.capacity;
  std::deque<Request> Q;
  const bool by_class = cfg.policy == 2;
  std::vector<std::deque<Request>> Qk(by_class ? cfg.n_classes : 0);  // CLASSES: one FIFO per class
  std::vector<int64_t> next_in_class(by_class ? cfg.n_classes : 0, 0);
  std::vector<Request> P;
  uint64_t* C = out.counters + slot * FO_N_COUNTERS;
  std::memset(C, 0, sizeof(uint64_t) * FO_N_COUNTERS);
  const int64_t n_trace = cfg.trace_every > 0 ? T / cfg.trace_every : 0;
  int64_t next_id = 0;
  int64_t forced_pos = 0;
  const bool timed = cfg.time_c0 != 0 || cfg.time_cp != 0 || cfg.time_cd != 0;
  int64_t tau = 1;     // time at which the slot starts (= t while every slot lasts one unit)
  int64_t u_seen = 0;  // arrivals of the units 1 .. u_seen have joined Q
  auto rec = [&](int32_t* arr, int64_t id, int64_t v) {
    if (arr && id < cfg.max_requests) arr[slot * cfg.max_requests + id] = static_cast<int32_t>(v);
  };

  for (int64_t t = 1; t <= T; ++t) {
    // ---- 1. arrivals -------------------------------------------------------
    uint32_t blk[4];
    {
      const uint32_t ctr[4] = {0u, static_cast<uint32_t>(t), static_cast<uint32_t>(replica), 0u};
      philox4x32_10(ctr, key, blk);
    }
    int64_t n_t = 0;
    if (by_class) {
      auto arrive = [&](int64_t k) {
        Request r;
        r.cls = k;
        r.id = next_in_class[k]++ * cfg.n_classes + k;
        r.l = cfg.prompt[k].lo;
        r.o = cfg.decode[k].lo;
        r.t_arr = t;
        Qk[k].push_back(r);
        rec(out.arrival_step, r.id, t);
        rec(out.req_l, r.id, r.l);
        rec(out.req_o, r.id, r.o);
        ++n_t;
      };
      if (cfg.n_forced >= 0) {
        while (forced_pos < cfg.n_forced && cfg.forced_t[forced_pos] == t) arrive(cfg.forced_cls[forced_pos++]);
      } else {
        for (int64_t k = 0; k < cfg.n_classes; ++k) {
          const uint32_t ctr[4] = {static_cast<uint32_t>(k), static_cast<uint32_t>(t),
                                   static_cast<uint32_t>(replica), 2u};
          uint32_t w[4];
          philox4x32_10(ctr, key, w);
          const int64_t n_tk = invert(cfg.class_arrivals[k], w[0]);
          for (int64_t i = 0; i < n_tk; ++i) arrive(k);
        }
      }
    } else {
      // the arrivals of one time unit u join the tail of Q; a slot takes those of all units up to its start
      auto arrivals_of = [&](int64_t u) {
        int64_t n_u = 0;
        if (cfg.n_forced >= 0) {
          while (forced_pos < cfg.n_forced && cfg.forced_t[forced_pos] == u) {
            Request r;
            r.id = next_id++;
            r.l = cfg.forced_l[forced_pos];
            r.o = cfg.forced_o[forced_pos];
            r.t_arr = u;
            Q.push_back(r);
            ++forced_pos;
            ++n_u;
          }
        } else {
          uint32_t bu[4];
          const uint32_t cu[4] = {0u, static_cast<uint32_t>(u), static_cast<uint32_t>(replica), 0u};
          philox4x32_10(cu, key, bu);
          n_u = invert(cfg.arrivals, bu[0]);
          for (int64_t k = 0; k < n_u; ++k) {
            const uint32_t ctr[4] = {static_cast<uint32_t>(k), static_cast<uint32_t>(u),
                                     static_cast<uint32_t>(replica), 1u};
            uint32_t w[4];
            philox4x32_10(ctr, key, w);
            fo_law cls_law{0, cfg.n_classes - 1, cfg.class_thr};
            int64_t cls = invert(cls_law, w[0]);
            Request r;
            r.id = next_id++;
            r.l = invert_sorted(cfg.prompt[cls], w[1]);
            r.o = invert_sorted(cfg.decode[cls], w[2]);
            r.t_arr = u;
            Q.push_back(r);
          }
        }
        for (int64_t k = 0; k < n_u; ++k) {
          const Request& r = Q[Q.size() - n_u + k];
          rec(out.arrival_step, r.id, u);
          rec(out.req_l, r.id, r.l);
          rec(out.req_o, r.id, r.o);
        }
        return n_u;
      };
      while (u_seen < tau) n_t += arrivals_of(++u_seen);
    }
    C[FO_ARRIVED] += n_t;

    // ---- 2. admission ------------------------------------------------------
    int64_t B_t = 0;
    auto activate_head = [&]() {
      Request r = Q.front();
      Q.pop_front();
      r.p = 0;
      r.j = 0;
      if (!r.was_active) rec(out.first_activation, r.id, tau);
      rec(out.last_activation, r.id, tau);
      r.was_active = true;
      P.push_back(r);
      C[FO_ACTIVATIONS] += 1;
    };
    if (by_class) {
      for (int64_t k = 0; k < cfg.n_classes; ++k) {
        int64_t activated = 0;
        while (activated < cfg.class_budget[k] && !Qk[k].empty()) {
          Q.push_front(Qk[k].front());  // through the common helper: it takes the head of Q
          Qk[k].pop_front();
          activate_head();
          ++activated;
        }
      }
    } else if (cfg.policy == 0) {
      if (cfg.n_forced_B > 0)
        B_t = cfg.forced_B[std::min<int64_t>(t, cfg.n_forced_B) - 1];
      else
        if (cfg.budget_mode == 1)  // any bounded law on the integers (Theorem 2)
          B_t = invert(cfg.budget_law, blk[1]);
        else if (cfg.budget_mode == 2)  // deterministic: the credit t b, spent in whole requests
          B_t = ((static_cast<int64_t>(t) * cfg.budget_b16) >> 16) - ((static_cast<int64_t>(t - 1) * cfg.budget_b16) >> 16);
        else
          B_t = cfg.b_floor + (blk[1] < cfg.b_frac_thr ? 1 : 0);
      int64_t activated = 0;
      while (activated < B_t && !Q.empty()) {
        activate_head();
        ++activated;
      }
    } else if (cfg.policy == 4) {
      // MC benchmark (Section 4.1): first come first served; the head moves only if, with it, the
      // memory stays within M in every future slot of the prediction in which each request
      // produces o_hat tokens, one per slot from the slot s of its first token (the slot in which it
      // was, or is now, activated: no chunking and no token budget under this policy), holds
      // l + (tokens so far) and leaves after its last one.  The usage only drops when somebody
      // leaves, so the slots to look at are the last slots of the requests.
      // With known request types (assumed_o = 0) each request is predicted to produce its own o tokens;
      // with unknown types all of them the one length assumed_o.
      auto predicted = [&](const Request& r) { return cfg.assumed_o > 0 ? cfg.assumed_o : r.o; };
      auto fits_in_future = [&](const Request& c) {
        struct Pred { int64_t l, s, o_hat; };
        std::vector<Pred> S;
        for (const Request& r : P) S.push_back({r.l, t - r.j, predicted(r)});  // j tokens by slot t - 1: the first came in t - j
        S.push_back({c.l, t, predicted(c)});
        for (const Pred& k : S) {
          const int64_t u = k.s + k.o_hat - 1;  // k's last slot
          int64_t use = 0;
          for (const Pred& i : S)
            if (i.s + i.o_hat - 1 >= u) use += i.l + std::min(i.o_hat, u - i.s + 1);
          if (use > M) return false;
        }
        return true;
      };
      while (!Q.empty() && fits_in_future(Q.front())) activate_head();
    } else {
      // GREEDY fills the memory, ALPHA (Section 4.1, alpha-protection greedy) only its share
      // (1 - alpha) M: the head moves while the usage with its initial memory l + 1 stays within it
      const int64_t limit = cfg.policy == 3 ? cfg.protect_limit : M;
      while (!Q.empty()) {
        int64_t provisioned = usage(P) + static_cast<int64_t>(P.size());
        if (provisioned + Q.front().l + 1 > limit) break;
        activate_head();
      }
    }

    // ---- 3. overflow: evict newest until the provisioned usage fits ---------
    bool overflowed = false;
    if (by_class && usage(P) + static_cast<int64_t>(P.size()) > M) overflowed = true;  // counted, nobody leaves
    // (ALPHA: on overflow every active request goes back, newest first, so Q stays in arrival order)
    const bool evict_all = cfg.policy == 3 && usage(P) + static_cast<int64_t>(P.size()) > M;
    while (!by_class && (evict_all ? !P.empty() : usage(P) + static_cast<int64_t>(P.size()) > M)) {
      Request r = P.back();
      P.pop_back();
      r.p = 0;
      r.j = 0;
      Q.push_front(r);
      C[FO_EVICTIONS] += 1;
      overflowed = true;
    }
    if (overflowed) C[FO_OVERFLOW_STEPS] += 1;

    // ---- 4. process: prefill chunks first, then one token per decoding request
    int64_t budget = cfg.token_budget;
    const uint64_t pf_before = C[FO_PREFILL_TOKENS], dec_before = C[FO_DECODE_TOKENS];
    for (Request& r : P) r.decoding_at_slot_start = (r.p == r.l);
    for (Request& r : P) {
      if (r.p == r.l) continue;
      int64_t d = std::min(std::min(cfg.prefill_chunk, r.l - r.p), budget);
      r.p += d;
      budget -= d;
      C[FO_PREFILL_TOKENS] += d;
      if (r.p == r.l) {  // the chunk that ends the prompt also yields token 1
        r.j = 1;
        C[FO_DECODE_TOKENS] += 1;
      }
    }
    for (Request& r : P) {
      if (!r.decoding_at_slot_start) continue;
      if (budget > 0) {
        r.j += 1;
        budget -= 1;
        C[FO_DECODE_TOKENS] += 1;
      } else {
        C[FO_STALLED] += 1;
      }
    }

    // ---- 5. measure ----------------------------------------------------------
    const int64_t U_t = usage(P);
    const int64_t P_t = static_cast<int64_t>(P.size());
    int64_t Q_t = static_cast<int64_t>(Q.size());
    for (const auto& q : Qk) Q_t += static_cast<int64_t>(q.size());
    C[FO_SUM_U] += U_t;
    C[FO_SUM_P] += P_t;
    C[FO_SUM_Q] += Q_t;
    C[FO_MAX_U] = std::max<uint64_t>(C[FO_MAX_U], U_t);
    C[FO_MAX_P] = std::max<uint64_t>(C[FO_MAX_P], P_t);
    C[FO_MAX_Q] = std::max<uint64_t>(C[FO_MAX_Q], Q_t);
    if (cfg.trace_every > 0 && t % cfg.trace_every == 0) {
      int64_t idx = t / cfg.trace_every - 1;
      if (out.trace_q) out.trace_q[slot * n_trace + idx] = static_cast<int32_t>(Q_t);
      if (out.trace_u) out.trace_u[slot * n_trace + idx] = static_cast<int32_t>(U_t);
    }
    if (out.step_u) out.step_u[slot * T + (t - 1)] = static_cast<int32_t>(U_t);
    if (out.step_p) out.step_p[slot * T + (t - 1)] = static_cast<int32_t>(P_t);
    if (out.step_q) out.step_q[slot * T + (t - 1)] = static_cast<int32_t>(Q_t);
    if (out.step_n) out.step_n[slot * T + (t - 1)] = static_cast<int32_t>(n_t);
    if (out.step_b) out.step_b[slot * T + (t - 1)] = static_cast<int32_t>(B_t);

    // ---- 6. complete ---------------------------------------------------------
    // the slot lasted d_t units; what completes in it does so in its last unit, tau + d_t - 1
    const int64_t d_t = !timed ? 1
                               : cfg.time_c0 + cfg.time_cp * static_cast<int64_t>(C[FO_PREFILL_TOKENS] - pf_before) +
                                     cfg.time_cd * static_cast<int64_t>(C[FO_DECODE_TOKENS] - dec_before);
    std::vector<Request> keep;
    keep.reserve(P.size());
    for (const Request& r : P) {
      if (r.j == r.o) {
        int64_t latency = tau + d_t - r.t_arr;  // both ends counted: t - t_arr + 1 in unit slots
        C[FO_COMPLETED] += 1;
        C[FO_SUM_LATENCY] += latency;
        C[FO_MAX_LATENCY] = std::max<uint64_t>(C[FO_MAX_LATENCY], latency);
        C[FO_USEFUL_TOKENS] += r.o;
        rec(out.completion_step, r.id, tau + d_t - 1);
        if (out.hist && cfg.hist_bins > 0) {
          int64_t b = std::min<int64_t>(latency >> cfg.hist_shift, cfg.hist_bins - 1);
          out.hist[slot * cfg.hist_bins + b] += 1;
        }
      } else {
        keep.push_back(r);
      }
    }
    P.swap(keep);
    tau += d_t;
  }
  C[FO_ELAPSED] = static_cast<uint64_t>(tau - 1);

  C[FO_FINAL_P] = P.size();
  C[FO_FINAL_Q] = Q.size();
  for (const auto& q : Qk) C[FO_FINAL_Q] += q.size();
  C[FO_FINAL_U] = usage(P);
  // digest of the final state: FNV-1a over 64-bit words
  uint64_t h = 14695981039346656037ull;
  h = fnv_step(h, P.size());
  for (const Request& r : P) {
    h = fnv_step(h, r.id);
    h = fnv_step(h, r.j);
    h = fnv_step(h, r.p);
  }
  if (by_class) {  // the waiting requests of a class are interchangeable: their number says it all
    for (const auto& q : Qk) h = fnv_step(h, q.size());
  } else {
    uint64_t returned = 0;
    for (const Request& r : Q) returned += r.was_active ? 1 : 0;
    h = fnv_step(h, returned);
    for (const Request& r : Q)
      if (r.was_active) h = fnv_step(h, r.id);
    h = fnv_step(h, Q.size() - returned);
  }
  C[FO_DIGEST] = h;
}

}  // namespace

extern "C" {

int fo_n_counters() { return FO_N_COUNTERS; }

const char* fo_counter_name(int i) {
  static const char* names[FO_N_COUNTERS] = {
      "completed", "arrived", "evictions", "activations", "sum_p", "sum_q", "sum_u",
      "overflow_steps", "sum_latency", "max_latency", "useful_tokens", "decode_tokens",
      "prefill_tokens", "stalled", "max_p", "max_q", "max_u", "final_p", "final_q",
      "final_u", "digest", "elapsed"};
  return (i >= 0 && i < FO_N_COUNTERS) ? names[i] : nullptr;
}

void fo_philox(const uint32_t* ctr, const uint32_t* key, uint32_t* out) {
  philox4x32_10(ctr, key, out);
}

// Inverts n words against one law with both search routines; returns -1 if they differ.
int fo_invert(const fo_law* law, const uint32_t* u, int64_t n, int64_t* out) {
  for (int64_t i = 0; i < n; ++i) {
    out[i] = invert(*law, u[i]);
    if (out[i] != invert_sorted(*law, u[i])) return -1;
  }
  return 0;
}

// Simulates the listed replicas (the Philox replica index is replica_ids[i]);
// output row i belongs to replica_ids[i].  Returns 0, or -1 on bad arguments.
int fo_run(const fo_config* cfg, int64_t n_ids, const int64_t* replica_ids, int64_t n_steps,
           uint64_t seed, int32_t n_threads, const fo_outputs* out) {
  if (!cfg || !out || !out->counters || n_ids < 0 || n_steps < 0) return -1;
  if (cfg->policy < 0 || cfg->policy > 4) return -1;
  if (cfg->policy == 4) {  // the prediction is that of the slot model without chunking or token budget
    if (cfg->assumed_o < 0 || cfg->token_budget < (1ll << 30)) return -1;
    for (int32_t k = 0; k < cfg->n_classes; ++k) {
      if (cfg->prompt[k].lo + cfg->prompt[k].n_thr > cfg->prefill_chunk) return -1;
      // unknown types: the one assumed length covers every output; known types (0): the longest output itself
      const int64_t longest = cfg->assumed_o > 0 ? cfg->assumed_o : cfg->decode[k].lo + cfg->decode[k].n_thr;
      if (cfg->decode[k].lo + cfg->decode[k].n_thr > longest) return -1;
      if (cfg->prompt[k].lo + cfg->prompt[k].n_thr + longest > cfg->capacity) return -1;
    }
  }
  if (cfg->policy == 3 && (cfg->protect_limit < 0 || cfg->protect_limit > cfg->capacity)) return -1;
  if (cfg->budget_mode < 0 || cfg->budget_mode > 2 || (cfg->budget_mode != 0 && cfg->policy != 0)) return -1;
  if (cfg->time_c0 < 0 || cfg->time_cp < 0 || cfg->time_cd < 0) return -1;
  if ((cfg->time_c0 != 0 || cfg->time_cp != 0 || cfg->time_cd != 0) && (cfg->time_c0 < 1 || cfg->policy == 2)) return -1;
  if (cfg->budget_mode == 2 && (cfg->budget_b16 < 0 || cfg->budget_b16 > (30000ll << 16))) return -1;
  if (cfg->policy == 2) {
    if (!cfg->class_budget || (cfg->n_forced < 0 && !cfg->class_arrivals)) return -1;
    if (cfg->n_forced >= 0 && !cfg->forced_cls) return -1;
    for (int32_t k = 0; k < cfg->n_classes; ++k)
      if (cfg->prompt[k].n_thr != 0 || cfg->decode[k].n_thr != 0 || cfg->class_budget[k] < 0) return -1;
  }
  if (cfg->capacity < 1 || cfg->token_budget < 1 || cfg->prefill_chunk < 1) return -1;
  if (n_threads < 1) n_threads = 1;
  if (out->hist && cfg->hist_bins > 0)
    std::memset(out->hist, 0, sizeof(uint32_t) * n_ids * cfg->hist_bins);
  std::atomic<int64_t> next{0};
  auto worker = [&]() {
    for (;;) {
      int64_t i = next.fetch_add(1);
      if (i >= n_ids) break;
      simulate(*cfg, replica_ids[i], n_steps, seed, i, *out);
    }
  };
  std::vector<std::thread> pool;
  for (int32_t k = 1; k < n_threads; ++k) pool.emplace_back(worker);
  worker();
  for (auto& th : pool) th.join();
  return 0;
}

}  // extern "C"
