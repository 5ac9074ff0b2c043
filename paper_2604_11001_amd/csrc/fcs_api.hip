// Host side of libfcs: parameter validation, table blob, workspace layout, launches,
// read-back and derived statistics.  See include/fcs.h for the contract.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <atomic>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "fcs_internal.h"

using namespace fcs;

struct fcs_engine {
  // parameters (owned copies)
  int32_t M = 0, tau = 0, chunk = 0, n_classes = 0, n_arrival_laws = 0, n_cells = 0;
  int32_t trace_every = 0, hist_bins = 0, hist_shift = 0, max_requests = 0;
  int32_t max_active = 0, lds_slots_param = 0;
  int32_t l_min = 1;
  std::vector<DCell> cells;
  std::vector<uint32_t> blob;  // DLaw[], DCell[], class thresholds, thresholds, guides
  uint32_t laws_off = 0, cells_off = 0, class_off = 0, sched_off = 0;
  // binding
  bool bound = false;
  void* workspace = nullptr;
  size_t workspace_bytes = 0;
  int64_t bound_replicas = 0;
  fcs_outputs out{};
  int32_t lcap = 0, hcap = 0, hscap = 0, stack_lds = 0;
  int64_t spill_stride = 0;
  uint32_t launch_seq = 0;
  bool has_classes = false;
  bool has_alpha = false;  // ALPHA cells: an overflow sends the whole active set to the evicted stack
  bool has_budget_modes = false;  // FLOW cells whose B_t is not the Bernoulli split
  bool has_mc = false;
  int32_t wheel_slots = 0;  // MC cells with known request types: slots of the departure wheel (else 0)
  int32_t time_c0 = 0, time_cp = 0, time_cd = 0;
  int32_t flags = 0;
  int64_t classes_active = 0;  // CLASSES: most requests active at once when no prefill ever waits
  double expected_active = 0.0;  // FLOW and GREEDY cells: estimate of the mean |P| of the busiest cell (below)
  size_t blob_bytes_padded = 0;
  // last run
  bool ran = false;
  int64_t run_replicas = 0, run_steps = 0;
  void* run_stream = nullptr;
  int32_t run_lcap = 0, run_hcap = 0, run_stack_lds = 0;
  fcs_outputs run_out{};  // the output arrays that run wrote (those of fcs_bind, or of fcs_run_static)
  uint64_t uid = 0;       // distinguishes handles that follow each other at one address
};

namespace {

constexpr int32_t kLimit = 1 << 30;
constexpr double kLdsFill = 0.85;  // share of a path's LDS slots that its expected active set may take

size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

bool law_ok(const fcs_law& L, int32_t min_lo, int32_t max_thr) {
  if (L.lo < min_lo || L.n_thr < 0 || L.n_thr > max_thr) return false;
  if (L.n_thr > 0 && L.thr == nullptr) return false;
  if (static_cast<int64_t>(L.lo) + L.n_thr > kLimit) return false;
  for (int32_t i = 1; i < L.n_thr; ++i)
    if (L.thr[i] < L.thr[i - 1]) return false;
  return true;
}

bool params_ok(const fcs_params* p) {
  if (!p) return false;
  if (p->capacity < 1 || p->capacity > kLimit) return false;
  if (p->token_budget < 1 || p->token_budget > kLimit) return false;
  if (p->prefill_chunk < 1 || p->prefill_chunk > kLimit) return false;
  if (p->n_classes < 1 || p->n_classes > kMaxClasses || !p->prompt || !p->decode) return false;
  if (p->n_classes > 1 && !p->class_thr) return false;
  for (int32_t c = 0; c + 2 < p->n_classes; ++c)
    if (p->class_thr[c + 1] < p->class_thr[c]) return false;
  int64_t l_max = 0, o_max = 0;
  for (int32_t c = 0; c < p->n_classes; ++c) {
    if (!law_ok(p->prompt[c], 1, 1 << 24) || !law_ok(p->decode[c], 1, 1 << 24)) return false;
    l_max = std::max<int64_t>(l_max, static_cast<int64_t>(p->prompt[c].lo) + p->prompt[c].n_thr);
    o_max = std::max<int64_t>(o_max, static_cast<int64_t>(p->decode[c].lo) + p->decode[c].n_thr);
  }
  if (l_max + o_max > p->capacity) return false;
  if (p->n_arrival_laws < 1 || !p->arrival) return false;
  for (int32_t a = 0; a < p->n_arrival_laws; ++a)
    if (!law_ok(p->arrival[a], 0, kMaxCountThr)) return false;  // counts start at 0 where they are n_t (below)
  if (p->n_cells < 1 || !p->cells) return false;
  for (int32_t i = 0; i < p->n_cells; ++i) {
    const fcs_cell& c = p->cells[i];
    if (c.policy < FCS_POLICY_FLOW || c.policy > FCS_POLICY_MC) return false;
    if (c.policy == FCS_POLICY_MC) {  // the prediction is that of the slot model without chunking or token budget
      if (p->token_budget < kLimit || p->prefill_chunk < l_max) return false;
      // assumed_o = 0: known request types, every request predicted at its own length (one wheel entry per
      // future slot up to the longest output); else one common length that covers every output
      if (c.assumed_o == 0 ? o_max > kMaxWheelSlots : c.assumed_o < o_max) return false;
      const int64_t longest = c.assumed_o == 0 ? o_max : c.assumed_o;
      if (static_cast<int64_t>(l_max) + longest > p->capacity) return false;
      // the kernel sums l + j + o_hat over the active set in 32 bits
      const int64_t most_active = p->max_active > 0 ? p->max_active : 8192;
      if ((l_max + 2 * longest) * most_active >= (1ll << 31)) return false;
    }
    if (c.policy == FCS_POLICY_ALPHA && !(c.alpha >= 0.0 && c.alpha <= 1.0)) return false;
    if (c.budget_mode < FCS_BUDGET_SPLIT || c.budget_mode > FCS_BUDGET_CREDIT) return false;
    if (c.budget_mode != FCS_BUDGET_SPLIT && c.policy != FCS_POLICY_FLOW) return false;
    if (c.budget_mode == FCS_BUDGET_LAW) {
      if (c.budget_law < 0 || c.budget_law >= p->n_arrival_laws) return false;
      const fcs_law& bl = p->arrival[c.budget_law];
      if (bl.lo < 0 || static_cast<int64_t>(bl.lo) + bl.n_thr > 30000) return false;
    }
    if (c.budget_mode == FCS_BUDGET_CREDIT && (c.budget_b16 == 0 || c.budget_b16 > (30000u << 16))) return false;
    if (c.arrival < 0 || c.arrival >= p->n_arrival_laws || p->arrival[c.arrival].lo != 0) return false;
    if (c.b_floor < 0 || c.b_floor > 30000) return false;
    if (c.policy == FCS_POLICY_CLASSES) {  // Algorithm 1: known lengths, integer budgets
      if (!c.class_arrival || !c.class_budget) return false;
      int64_t total = 0;
      for (int32_t k = 0; k < p->n_classes; ++k) {
        if (p->prompt[k].n_thr != 0 || p->decode[k].n_thr != 0) return false;
        if (c.class_arrival[k] < 0 || c.class_arrival[k] >= p->n_arrival_laws) return false;
        if (p->arrival[c.class_arrival[k]].lo != 0) return false;
        if (c.class_budget[k] < 0 || c.class_budget[k] > kWave) return false;
        total += c.class_budget[k];
      }
      if (total > kWave) return false;
    }
  }
  if (p->time_c0 < 0 || p->time_cp < 0 || p->time_cd < 0) return false;
  if (p->time_c0 != 0 || p->time_cp != 0 || p->time_cd != 0) {  // slots of variable duration
    if (p->time_c0 < 1 || p->time_cp > (1 << 15) || p->time_cd > (1 << 15) || p->time_c0 > (1 << 20)) return false;
    for (int32_t i = 0; i < p->n_cells; ++i)
      if (p->cells[i].policy == FCS_POLICY_CLASSES) return false;
  }
  if (p->flags & ~(FCS_FLAG_SKIP_IDLE | FCS_FLAG_GENERAL_CODE)) return false;
  if (p->flags & FCS_FLAG_SKIP_IDLE) {  // only the kernel of the FLOW and GREEDY cells has it
    if (p->time_c0 != 0) return false;
    for (int32_t i = 0; i < p->n_cells; ++i)
      if (p->cells[i].policy > FCS_POLICY_GREEDY || p->cells[i].budget_mode != FCS_BUDGET_SPLIT) return false;
  }
  if (p->trace_every < 0 || p->hist_bins < 0 || p->hist_bins > (1 << 24)) return false;
  if (p->hist_shift < 0 || p->hist_shift > 30 || p->max_requests < 0) return false;
  if (p->max_active < 0 || p->max_active > (1 << 24)) return false;
  if (p->lds_slots != 0 &&
      (p->lds_slots < kLdsBlock || p->lds_slots > 4096 || p->lds_slots % kWave != 0 ||
       (p->lds_slots > 2 * kLdsBlock && p->lds_slots % kLdsBlock != 0)))
    return false;
  return true;
}

void append_law(std::vector<uint32_t>& blob, std::vector<DLaw>& laws, const fcs_law& L, bool guide) {
  DLaw d;
  d.lo = L.lo;
  d.n = L.n_thr;
  d.off = static_cast<uint32_t>(blob.size());
  blob.insert(blob.end(), L.thr, L.thr + L.n_thr);
  d.goff = 0;
  if (guide) {
    d.goff = static_cast<uint32_t>(blob.size());
    const uint32_t buckets = 1u << kGuideBits;
    for (uint32_t b = 0; b <= buckets; ++b) {
      // guide[b] = number of thresholds strictly below b << (32 - kGuideBits), all of them at the end
      uint32_t cnt;
      if (b == buckets) cnt = static_cast<uint32_t>(L.n_thr);
      else cnt = static_cast<uint32_t>(std::lower_bound(L.thr, L.thr + L.n_thr, b << (32 - kGuideBits)) - L.thr);
      blob.push_back(cnt);
    }
  }
  laws.push_back(d);
}

// E[X^k] of a threshold-table law, k = 1, 2
void law_moments(const fcs_law& L, double& m1, double& m2) {
  const double two32 = 4294967296.0;
  double prev = 0.0;
  m1 = m2 = 0.0;
  for (int32_t i = 0; i <= L.n_thr; ++i) {
    const double cur = (i < L.n_thr) ? static_cast<double>(L.thr[i]) : two32;
    const double pr = (cur - prev) / two32;
    const double v = static_cast<double>(L.lo) + i;
    m1 += pr * v;
    m2 += pr * v * v;
    prev = cur;
  }
}

// ---- device memory of fcs_run_static ----------------------------------------------------------------
// One array per GPU, there from the moment the library is loaded on that GPU until the process ends.
// Host code never uses the array's name as an address: the per-device address comes from
// hipGetSymbolAddress, once per device, and that pointer is what kernels, copies and fills receive.
constexpr size_t kStaticBytes = static_cast<size_t>(FCS_STATIC_WORKSPACE_BYTES);
constexpr size_t kStaticPaceOffset = kStaticBytes - 256;  // pacing words: the last 256 bytes
static __device__ __align__(256) unsigned char scratch[kStaticBytes];

constexpr int kMaxDevices = 64;
struct StaticSite {
  void* ptr = nullptr;       // device address of `scratch` on this GPU
  uint64_t blob_owner = 0;   // uid of the handle whose tables lie at the start of the array (0: none)
  uint32_t launch_seq = 0;   // launches that used the array's pacing words
};
StaticSite g_static[kMaxDevices];
std::mutex g_static_mu;
std::atomic<uint64_t> g_next_uid{1};

__global__ void fill_words_kernel(uint32_t* p, uint32_t v, int n) {
  const int i = static_cast<int>(blockIdx.x * blockDim.x + threadIdx.x);
  if (i < n) p[i] = v;
}

// E[ceil(X / c)] of a threshold-table law
double law_mean_chunks(const fcs_law& L, int64_t c) {
  const double two32 = 4294967296.0;
  double prev = 0.0, m = 0.0;
  for (int32_t i = 0; i <= L.n_thr; ++i) {
    const double cur = (i < L.n_thr) ? static_cast<double>(L.thr[i]) : two32;
    const int64_t v = static_cast<int64_t>(L.lo) + i;
    m += (cur - prev) / two32 * static_cast<double>((v + c - 1) / c);
    prev = cur;
  }
  return m;
}

// Estimate of the time-average |P| of a FLOW or GREEDY cell, used only to size the LDS part of the active
// set.  A request that is never held up is active for S = ceil(l / c) + o - 1 slots (Section 2.1 with
// chunked prefill: the chunk that ends the prompt yields token 1), so by Little's law |P| is about
// (activation rate) x E[S], the rate being at most the arrival rate and, under Algorithm 2, the mean
// budget b.  The memory caps it: over its stay a request holds l per prefill slot and l + j in the
// slot of token j, E[w] + E[l (ceil(l / c) - 1)] in all, so no more than M E[S] / that fit on average.
// Where the requests activated per slot want more than four fifths of the token budget (l prompt tokens
// and o output tokens each), prompts wait for budget inside the active set and evicted requests prefill
// again: the set then grows until the memory stops it, and the memory figure alone is the estimate.
double expected_active_of(const fcs_params* p, const fcs_cell& c) {
  const double two32 = 4294967296.0;
  const int64_t chunk = std::max<int64_t>(1, std::min<int64_t>(p->prefill_chunk, p->token_budget));
  double es = 0.0, hold = 0.0, prev = 0.0, tokens = 0.0;
  for (int32_t k = 0; k < p->n_classes; ++k) {
    const double cur = (k + 1 < p->n_classes) ? static_cast<double>(p->class_thr[k]) : two32;
    const double pk = (cur - prev) / two32;
    prev = cur;
    double el, el2, eo, eo2;
    law_moments(p->prompt[k], el, el2);
    law_moments(p->decode[k], eo, eo2);
    const double ech = law_mean_chunks(p->prompt[k], chunk);
    es += pk * (ech + eo - 1.0);
    tokens += pk * (el + eo);
    // l and o independent; E[l (ceil(l / c) - 1)] taken as E[l] E[ceil(l / c) - 1], good enough for a size
    hold += pk * (el * eo + 0.5 * (eo + eo2) + el * (ech - 1.0));
  }
  double lam, lam2;
  law_moments(p->arrival[c.arrival], lam, lam2);
  double rate = lam;
  if (c.policy == FCS_POLICY_FLOW && c.budget_mode == FCS_BUDGET_SPLIT)
    rate = std::min(rate, static_cast<double>(c.b_floor) + static_cast<double>(c.b_frac_thr) / two32);
  const double by_rate = rate * es;
  const double by_memory = hold > 0.0 ? static_cast<double>(p->capacity) * es / hold : by_rate;
  if (rate * tokens > 0.8 * static_cast<double>(p->token_budget)) return by_memory;
  return std::min(by_rate, by_memory);
}

// LDS words of a path beyond its active set, stack and scratch: the per-class tables of CLASSES cells and
// the departure wheel of MC cells with known request types (two words per slot)
int extra_lds_words(const fcs_engine* h) {
  return (h->has_classes ? class_lds_words(h->n_classes) : 0) + 2 * h->wheel_slots;
}

int sync_last(fcs_engine* h) {
  return hipStreamSynchronize(static_cast<hipStream_t>(h->run_stream)) == hipSuccess ? FCS_OK : FCS_EDEVICE;
}

}  // namespace

extern "C" {

int fcs_create(const fcs_params* p, fcs_handle* out) {
  if (!out) return FCS_EINVAL;
  *out = nullptr;
  if (!params_ok(p)) return FCS_EINVAL;
  fcs_engine* h = new (std::nothrow) fcs_engine();
  if (!h) return FCS_ENOMEM;
  h->uid = g_next_uid.fetch_add(1);
  try {  // the tables are std::vectors: running out of host memory must not leave through the C boundary
  h->M = p->capacity; h->tau = p->token_budget; h->chunk = p->prefill_chunk;
  h->n_classes = p->n_classes; h->n_arrival_laws = p->n_arrival_laws; h->n_cells = p->n_cells;
  h->trace_every = p->trace_every; h->hist_bins = p->hist_bins; h->hist_shift = p->hist_shift;
  h->max_requests = p->max_requests; h->max_active = p->max_active; h->lds_slots_param = p->lds_slots;
  h->time_c0 = p->time_c0; h->time_cp = p->time_cp; h->time_cd = p->time_cd;
  h->flags = p->flags;
  h->l_min = p->prompt[0].lo;
  for (int32_t c = 1; c < p->n_classes; ++c) h->l_min = std::min(h->l_min, p->prompt[c].lo);

  // blob: [DLaw x n_laws][DCell x n_cells][class thresholds][thresholds and guides]
  const int n_laws = p->n_arrival_laws + 2 * p->n_classes;
  std::vector<uint32_t> body;
  std::vector<DLaw> laws;
  const uint32_t head_words = static_cast<uint32_t>(4 * n_laws + 4 * p->n_cells + std::max(p->n_classes - 1, 0));
  for (int32_t a = 0; a < p->n_arrival_laws; ++a) append_law(body, laws, p->arrival[a], false);
  for (int32_t c = 0; c < p->n_classes; ++c) append_law(body, laws, p->prompt[c], true);
  for (int32_t c = 0; c < p->n_classes; ++c) append_law(body, laws, p->decode[c], true);
  std::vector<uint32_t> class_table_off(p->n_cells, 0u);
  for (int32_t i = 0; i < p->n_cells; ++i) {
    if (p->cells[i].policy != FCS_POLICY_CLASSES) continue;
    h->has_classes = true;
    // Algorithm 1 admits b_k requests of class k per slot and never evicts, so M does not bound the
    // active set; a request that is never held up stays ceil(l_k / chunk) + o_k slots
    int64_t active = 0;
    const int64_t chunk = std::max<int64_t>(1, std::min<int64_t>(p->prefill_chunk, p->token_budget));
    for (int32_t k = 0; k < p->n_classes; ++k)
      active += static_cast<int64_t>(p->cells[i].class_budget[k]) *
                ((p->prompt[k].lo + chunk - 1) / chunk + p->decode[k].lo + 1);
    h->classes_active = std::max(h->classes_active, active);
    class_table_off[i] = head_words + static_cast<uint32_t>(body.size());
    for (int32_t k = 0; k < p->n_classes; ++k) {
      body.push_back(static_cast<uint32_t>(p->cells[i].class_arrival[k]));
      body.push_back(static_cast<uint32_t>(p->cells[i].class_budget[k]));
    }
  }
  for (DLaw& d : laws) { d.off += head_words; if (d.goff) d.goff += head_words; }
  h->laws_off = 0;
  h->cells_off = static_cast<uint32_t>(4 * n_laws);
  h->class_off = h->cells_off + static_cast<uint32_t>(4 * p->n_cells);
  h->blob.resize(head_words);
  std::memcpy(h->blob.data(), laws.data(), sizeof(DLaw) * laws.size());
  for (int32_t i = 0; i < p->n_cells; ++i) {
    DCell d{p->cells[i].policy, p->cells[i].arrival, p->cells[i].b_floor, p->cells[i].b_frac_thr};
    if (d.policy == FCS_POLICY_CLASSES) d.b_frac_thr = class_table_off[i];
    if (d.policy == FCS_POLICY_MC) {
      d.b_frac_thr = static_cast<uint32_t>(p->cells[i].assumed_o);
      h->has_mc = true;
      if (p->cells[i].assumed_o == 0) {
        int64_t o_max = 0;
        for (int32_t c = 0; c < p->n_classes; ++c)
          o_max = std::max<int64_t>(o_max, static_cast<int64_t>(p->decode[c].lo) + p->decode[c].n_thr);
        h->wheel_slots = static_cast<int32_t>(round_up(static_cast<size_t>(o_max), kWave));
      }
    }
    if (d.policy == FCS_POLICY_ALPHA) {
      int32_t limit = 0;
      if (fcs_protect_limit(p->cells[i].alpha, p->capacity, &limit) != FCS_OK) { delete h; return FCS_EINVAL; }
      d.b_frac_thr = static_cast<uint32_t>(limit);
      h->has_alpha = true;
    }
    if (p->cells[i].budget_mode != FCS_BUDGET_SPLIT) {  // the mode rides in the bits above the policy
      d.policy |= p->cells[i].budget_mode << 8;
      if (p->cells[i].budget_mode == FCS_BUDGET_LAW) d.b_floor = p->cells[i].budget_law;
      else d.b_frac_thr = p->cells[i].budget_b16;
      h->has_budget_modes = true;
    }
    h->cells.push_back(d);
    std::memcpy(h->blob.data() + h->cells_off + 4 * i, &d, sizeof(d));
  }
  for (int32_t c = 0; c + 1 < p->n_classes; ++c) h->blob[h->class_off + c] = p->class_thr[c];
  // only the kernel of the FLOW and GREEDY cells takes LDS slots that are not a multiple of 256
  if (p->lds_slots % kLdsBlock != 0 &&
      (h->has_classes || h->has_alpha || h->has_budget_modes || h->has_mc || h->time_c0 != 0)) {
    delete h;
    return FCS_EINVAL;
  }
  for (int32_t i = 0; i < p->n_cells; ++i)
    if (p->cells[i].policy == FCS_POLICY_FLOW || p->cells[i].policy == FCS_POLICY_GREEDY)
      h->expected_active = std::max(h->expected_active, expected_active_of(p, p->cells[i]));
  h->blob.insert(h->blob.end(), body.begin(), body.end());
  // the schedule area (internal layout above): before the first launch the cells are ordered by a guess of
  // the time of a path, policy by policy and by arrival rate; from then on by what the last launch measured
  if (h->blob.size() % 2) h->blob.push_back(0u);
  h->sched_off = static_cast<uint32_t>(h->blob.size());
  h->blob.resize(h->blob.size() + sched_words(p->n_cells), 0u);
  for (int32_t i = 0; i < p->n_cells; ++i) {
    static const double weight[] = {1.0, 1.2, 1.0, 3.0, 2.0};  // FLOW, GREEDY, CLASSES, ALPHA, MC
    double lam, lam2;
    law_moments(p->arrival[p->cells[i].arrival], lam, lam2);
    const uint64_t guess = static_cast<uint64_t>(1000.0 * weight[p->cells[i].policy] * (1.0 + lam));
    std::memcpy(h->blob.data() + h->sched_off + 2 * i, &guess, sizeof(guess));
  }
  h->blob_bytes_padded = round_up(h->blob.size() * sizeof(uint32_t), 256);
  } catch (const std::bad_alloc&) {
    delete h;
    return FCS_ENOMEM;
  }
  *out = h;
  return FCS_OK;
}

static int geometry_for(fcs_engine* h, int64_t n_replicas, int32_t* lcap, int32_t* hcap, int32_t* hscap,
                        int32_t* stack_lds) {
  if (n_replicas < 1) return FCS_EINVAL;
  const int64_t n_paths = n_replicas * h->n_cells;
  if (n_paths > (1ll << 30)) return FCS_EINVAL;
  int64_t max_active = h->max_active;
  if (max_active == 0) max_active = std::min<int64_t>(std::max<int64_t>(h->M / (h->l_min + 1) + 1, h->classes_active), 8192);
  max_active = static_cast<int64_t>(round_up(static_cast<size_t>(max_active), kWave));
  int32_t lc = h->lds_slots_param;
  const bool plain = !(h->has_classes || h->has_alpha || h->has_budget_modes || h->has_mc || h->time_c0 != 0);
  if (lc == 0 && plain && n_paths > 2048) {
    // The kernel of the FLOW and GREEDY cells runs four wavefronts per SIMD, and a path is a chain of
    // dependent instructions: with more paths than the chip holds at two per SIMD, throughput is set by how
    // many are resident.  320 slots (with a stack of 64 entries, eight 1,280-byte granules of LDS) let 16
    // paths share a compute unit, 384 twelve, 448 eleven, 512 ten.  The fewest slots are taken that leave
    // the expected active set some 15 % of them for its fluctuations and for the dead slots between
    // compactions (measured on a heavy-tailed workload at several memory sizes: 320 slots beat 384 up to a
    // mean active set of about 275, 384 beat 512 beyond 290).  A path whose active set outgrows its slots
    // goes on in the spill region.
    const int64_t want = static_cast<int64_t>(round_up(static_cast<size_t>(std::ceil(h->expected_active / kLdsFill)), kWave));
    if (want <= 2 * kLdsBlock) lc = static_cast<int32_t>(std::max<int64_t>(want, kLdsBlock + kWave));
  }
  if (lc == 0) {
    // spread the paths over the 256 compute units and give each wavefront an equal share of
    // the 160 KB of LDS, between 4 and 8 wavefronts per unit (8 leaves 512 slots: both register blocks of
    // the hand-scheduled slot loop)
    int64_t per_cu = (n_paths + 255) / 256;
    per_cu = std::min<int64_t>(std::max<int64_t>(per_cu, 4), 8);
    const int64_t words = (160 * 1024 / per_cu) / 4 - S_NFIELDS * kStackLdsMin - kScratchWords -
                          extra_lds_words(h);
    lc = static_cast<int32_t>(words / kLdsWordsPerSlot / kLdsBlock * kLdsBlock);
    lc = std::min(std::max(lc, kLdsBlock), 2048);
  }
  // only the kernels of the FLOW and GREEDY cells take LDS slots that are not a multiple of 256
  if (!plain && lc % kLdsBlock != 0) return FCS_EINVAL;
  lc = static_cast<int32_t>(std::min<int64_t>(lc, static_cast<int64_t>(round_up(max_active, kLdsBlock))));
  *lcap = lc;
  *hcap = static_cast<int32_t>(std::max<int64_t>(max_active - lc, 0));
  // A compute unit hands its 160 KB of LDS out in 128 granules of 1,280 bytes (measured: 15,360 bytes per
  // workgroup run ten to a unit, 15,616 nine), and the FLOW/GREEDY kernels fit 16 wavefronts, the others 12.
  // The LDS part of the evicted stack takes what is left of the last granule without costing a resident
  // path: 48 entries with 512 slots (15 KB, ten paths per unit), 128 with 256 slots (16 paths).
  const int64_t fixed_bytes = 4 * (static_cast<int64_t>(kLdsWordsPerSlot) * lc + kScratchWords + extra_lds_words(h));
  const int64_t wave_cap = plain ? 16 : 12;
  auto resident = [&](int64_t stack) {
    const int64_t granules = (fixed_bytes + 4 * S_NFIELDS * stack + 1279) / 1280;
    return std::min<int64_t>(128 / std::max<int64_t>(granules, 1), wave_cap);
  };
  int32_t stack = kStackLdsMin;
  while (stack + 16 <= kStackLdsMax && resident(stack + 16) == resident(kStackLdsMin)) stack += 16;
  *stack_lds = stack;
  // the evicted stack holds what was evicted and not yet activated again; under ALPHA that can be a
  // whole active set on top of the rest of an earlier one
  *hscap = static_cast<int32_t>(std::max<int64_t>((h->has_alpha ? 2 : 1) * max_active - stack, 0));
  return FCS_OK;
}

int fcs_workspace_bytes(fcs_handle h, int64_t n_replicas, size_t* bytes) {
  if (!h || !bytes) return FCS_EINVAL;
  int32_t lc, hc, hs, sl;
  int rc = geometry_for(h, n_replicas, &lc, &hc, &hs, &sl);
  if (rc != FCS_OK) return rc;
  const size_t stride = static_cast<size_t>(kSpillWordsPerSlot) * hc + static_cast<size_t>(S_NFIELDS) * hs;
  *bytes = h->blob_bytes_padded + round_up(stride * sizeof(int32_t) * n_replicas * h->n_cells, 256) + 256;
  return FCS_OK;
}

int fcs_bind(fcs_handle h, void* ws, size_t bytes, int64_t n_replicas, const fcs_outputs* o, void* stream) {
  if (!h || !ws || !o || !o->counters) return FCS_EINVAL;
  if (reinterpret_cast<uintptr_t>(ws) % 256 != 0) return FCS_EINVAL;
  size_t need = 0;
  int rc = fcs_workspace_bytes(h, n_replicas, &need);
  if (rc != FCS_OK) return rc;
  if (bytes < need) return FCS_ENOMEM;
  rc = geometry_for(h, n_replicas, &h->lcap, &h->hcap, &h->hscap, &h->stack_lds);
  if (rc != FCS_OK) return rc;
  h->spill_stride = static_cast<int64_t>(kSpillWordsPerSlot) * h->hcap + static_cast<int64_t>(S_NFIELDS) * h->hscap;
  hipError_t e = hipMemcpyAsync(ws, h->blob.data(), h->blob.size() * sizeof(uint32_t),
                                hipMemcpyHostToDevice, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return FCS_EDEVICE;
  // the last 256 bytes hold the pacing words of the kernel; they start at zero
  if (hipMemsetAsync(static_cast<char*>(ws) + need - 256, 0, 256, static_cast<hipStream_t>(stream)) != hipSuccess)
    return FCS_EDEVICE;
  // the blob is pageable host memory owned by the handle: wait so it may change afterwards
  if (hipStreamSynchronize(static_cast<hipStream_t>(stream)) != hipSuccess) return FCS_EDEVICE;
  h->workspace = ws;
  h->workspace_bytes = bytes;
  h->bound_replicas = n_replicas;
  h->out = *o;
  h->bound = true;
  h->ran = false;
  return FCS_OK;
}

// Where a launch finds its device memory: the workspace (table blob, then the spill regions), the pacing
// words, the output arrays, and the geometry the spill regions were laid out for.
struct LaunchSite {
  void* workspace;
  unsigned long long* pace;
  uint32_t launch_seq;
  fcs_outputs out;
  int32_t lcap, hcap, hscap, stack_lds;
  int64_t spill_stride;
};

static int run_on(fcs_engine* h, const LaunchSite& site, int64_t replica_base, int64_t n_replicas, int64_t n_steps,
                  uint64_t seed, void* stream) {
  if (n_steps < 1 || n_steps >= kLimit) return FCS_EINVAL;
  if (replica_base < 0 || replica_base + n_replicas > 0xffffffffll) return FCS_EINVAL;
  KParams kp{};
  kp.blob = static_cast<const uint32_t*>(site.workspace);
  kp.laws_off = h->laws_off; kp.cells_off = h->cells_off; kp.class_off = h->class_off;
  kp.n_arrival_laws = h->n_arrival_laws; kp.n_classes = h->n_classes; kp.n_cells = h->n_cells;
  kp.M = h->M; kp.tau = h->tau; kp.chunk = h->chunk;
  kp.n_replicas = static_cast<int32_t>(n_replicas);
  kp.replica_base = static_cast<uint32_t>(replica_base);
  kp.n_steps = static_cast<int32_t>(n_steps);
  kp.seed_lo = static_cast<uint32_t>(seed);
  kp.seed_hi = static_cast<uint32_t>(seed >> 32);
  kp.lcap = site.lcap; kp.hcap = site.hcap; kp.hscap = site.hscap; kp.stack_lds = site.stack_lds;
  kp.class_words = h->has_classes ? class_lds_words(h->n_classes) : 0;
  kp.wheel_slots = h->wheel_slots;
  kp.all_policies = (h->has_classes || h->has_alpha || h->has_budget_modes || h->has_mc || h->time_c0 != 0) ? 1 : 0;
  kp.time_c0 = h->time_c0; kp.time_cp = h->time_cp; kp.time_cd = h->time_cd;
  kp.flags = h->flags;
  if (h->time_c0 != 0) {  // the clock of a path stays below 2^30
    const int64_t most_active = static_cast<int64_t>(site.lcap) + site.hcap;
    const int64_t d_max = h->time_c0 + static_cast<int64_t>(h->time_cp) * std::min<int64_t>(h->tau, h->M) +
                          static_cast<int64_t>(h->time_cd) * std::min<int64_t>(h->tau, most_active);
    if (n_steps * d_max >= kLimit) return FCS_EINVAL;
  }
  kp.spill = reinterpret_cast<int32_t*>(static_cast<char*>(site.workspace) + h->blob_bytes_padded);
  kp.spill_stride = site.spill_stride;
  kp.trace_every = h->trace_every;
  kp.n_trace = h->trace_every > 0 ? static_cast<int32_t>(n_steps / h->trace_every) : 0;
  kp.hist_bins = h->hist_bins; kp.hist_shift = h->hist_shift; kp.max_requests = h->max_requests;
  kp.n_paths = static_cast<int32_t>(n_replicas * h->n_cells);
  if (h->trace_every > 0 && (site.out.trace_q || site.out.trace_u) &&
      static_cast<int64_t>(kp.n_paths) * kp.n_trace > site.out.trace_entries)
    return FCS_EINVAL;  // the caller's trace arrays are too short for this run
  kp.pace = site.pace;
  kp.launch_seq = site.launch_seq;
  kp.out = site.out;
  if (h->hist_bins == 0) kp.out.hist = nullptr;
  if (h->max_requests == 0) { kp.out.arrival_step = nullptr; kp.out.completion_step = nullptr; }
  if (h->trace_every == 0) { kp.out.trace_q = nullptr; kp.out.trace_u = nullptr; }
  int rc = launch_sim(kp, h->sched_off, stream);
  if (rc != FCS_OK) return rc;
  h->ran = true;
  h->run_replicas = n_replicas;
  h->run_steps = n_steps;
  h->run_stream = stream;
  h->run_out = site.out;
  h->run_lcap = site.lcap;
  h->run_hcap = site.hcap;
  h->run_stack_lds = site.stack_lds;
  return FCS_OK;
}

int fcs_run_from(fcs_handle h, int64_t replica_base, int64_t n_replicas, int64_t n_steps, uint64_t seed,
                 void* stream) {
  if (!h) return FCS_EINVAL;
  if (!h->bound) return FCS_ESTATE;
  if (n_replicas < 1 || n_replicas > h->bound_replicas) return FCS_EINVAL;
  size_t need = 0;
  if (fcs_workspace_bytes(h, h->bound_replicas, &need) != FCS_OK) return FCS_ESTATE;
  LaunchSite site{};
  site.workspace = h->workspace;
  site.pace = reinterpret_cast<unsigned long long*>(static_cast<char*>(h->workspace) + need - 256);
  site.launch_seq = ++h->launch_seq;
  site.out = h->out;
  site.lcap = h->lcap; site.hcap = h->hcap; site.hscap = h->hscap; site.stack_lds = h->stack_lds;
  site.spill_stride = h->spill_stride;
  return run_on(h, site, replica_base, n_replicas, n_steps, seed, stream);
}

int fcs_run_static(fcs_handle h, const fcs_outputs* o, int64_t n_replicas, int64_t n_steps, uint64_t seed,
                   void* stream) {
  if (!h || !o || !o->counters) return FCS_EINVAL;
  LaunchSite site{};
  int rc = geometry_for(h, n_replicas, &site.lcap, &site.hcap, &site.hscap, &site.stack_lds);
  if (rc != FCS_OK) return rc;
  site.spill_stride = static_cast<int64_t>(kSpillWordsPerSlot) * site.hcap + static_cast<int64_t>(S_NFIELDS) * site.hscap;
  // the same layout as a caller's workspace, the pacing words apart at the end of the array
  const size_t spill_bytes = round_up(static_cast<size_t>(site.spill_stride) * sizeof(int32_t) *
                                          static_cast<size_t>(n_replicas) * static_cast<size_t>(h->n_cells), 256);
  if (h->blob_bytes_padded + spill_bytes > kStaticPaceOffset) return FCS_ENOMEM;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return FCS_EDEVICE;
  std::lock_guard<std::mutex> lock(g_static_mu);
  StaticSite& st = g_static[dev];
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (st.ptr == nullptr) {  // set-up, once per device, with that device current
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return FCS_EDEVICE;
    // the pacing words start at zero (a fill kernel, so that the call may be captured into a graph)
    hipLaunchKernelGGL(fill_words_kernel, dim3(1), dim3(64), 0, s,
                       reinterpret_cast<uint32_t*>(static_cast<char*>(p) + kStaticPaceOffset), 0u, 64);
    if (hipGetLastError() != hipSuccess) return FCS_EDEVICE;
    st.ptr = p;
  }
  if (st.blob_owner != h->uid) {  // another engine's tables (or none) lie there: upload this one's
    st.blob_owner = 0;
    if (hipMemcpyAsync(st.ptr, h->blob.data(), h->blob.size() * sizeof(uint32_t), hipMemcpyHostToDevice, s) !=
        hipSuccess)
      return FCS_EDEVICE;
    // the blob is pageable host memory owned by the handle: wait so it may go away afterwards
    if (hipStreamSynchronize(s) != hipSuccess) return FCS_EDEVICE;
    st.blob_owner = h->uid;
  }
  site.workspace = st.ptr;
  site.pace = reinterpret_cast<unsigned long long*>(static_cast<char*>(st.ptr) + kStaticPaceOffset);
  site.launch_seq = ++st.launch_seq;
  site.out = *o;
  return run_on(h, site, 0, n_replicas, n_steps, seed, stream);
}

int fcs_run(fcs_handle h, int64_t n_replicas, int64_t n_steps, uint64_t seed, void* stream) {
  return fcs_run_from(h, 0, n_replicas, n_steps, seed, stream);
}

int fcs_stats(fcs_handle h, int32_t cell, uint64_t* host_counters, fcs_summary* s) {
  if (!h) return FCS_EINVAL;
  if (!h->ran) return FCS_ESTATE;
  if (cell < -1 || cell >= h->n_cells) return FCS_EINVAL;
  int rc = sync_last(h);
  if (rc != FCS_OK) return rc;
  const int64_t n_paths = h->run_replicas * h->n_cells;
  std::vector<uint64_t> local;
  uint64_t* C = host_counters;
  if (!C) {
    try {
      local.resize(static_cast<size_t>(n_paths) * FCS_N_COUNTERS);
    } catch (const std::bad_alloc&) {
      return FCS_ENOMEM;
    }
    C = local.data();
  }
  if (hipMemcpy(C, h->run_out.counters, sizeof(uint64_t) * n_paths * FCS_N_COUNTERS, hipMemcpyDeviceToHost) !=
      hipSuccess)
    return FCS_EDEVICE;
  int64_t first_err = -1;
  int32_t err_code = 0;
  for (int64_t p = 0; p < n_paths; ++p) {
    if (C[p * FCS_N_COUNTERS + FCS_C_ERROR] != 0 && first_err < 0) {
      first_err = p;
      err_code = -static_cast<int32_t>(C[p * FCS_N_COUNTERS + FCS_C_ERROR]);
    }
  }
  if (s) {
    std::memset(s, 0, sizeof(*s));
    const int64_t lo = cell < 0 ? 0 : cell * h->run_replicas;
    const int64_t hi = cell < 0 ? n_paths : lo + h->run_replicas;
    uint64_t sum_u = 0, sum_q = 0, sum_lat = 0, useful = 0;
    for (int64_t p = lo; p < hi; ++p) {
      const uint64_t* c = C + p * FCS_N_COUNTERS;
      s->request_steps += c[FCS_C_SUM_P];
      s->arrived += c[FCS_C_ARRIVED];
      s->completed += c[FCS_C_COMPLETED];
      s->evictions += c[FCS_C_EVICTIONS];
      s->overflow_steps += c[FCS_C_OVERFLOW_STEPS];
      sum_u += c[FCS_C_SUM_U];
      sum_q += c[FCS_C_SUM_Q];
      sum_lat += c[FCS_C_SUM_LATENCY];
      useful += c[FCS_C_USEFUL_TOKENS];
    }
    s->n_paths = hi - lo;
    s->n_steps = h->run_steps;
    const double slots = static_cast<double>(s->n_paths) * static_cast<double>(h->run_steps);
    s->mean_latency = s->completed ? static_cast<double>(sum_lat) / static_cast<double>(s->completed) : 0.0;
    s->kv_utilisation = static_cast<double>(sum_u) / (slots * static_cast<double>(h->M));
    s->token_throughput = static_cast<double>(useful) / slots;
    s->prompt_throughput = static_cast<double>(s->completed) / slots;
    s->mean_queue = static_cast<double>(sum_q) / slots;
    s->mean_active = static_cast<double>(s->request_steps) / slots;
    s->first_error_path = first_err;
    s->error_code = err_code;
  }
  // the first failing path's own code: FCS_EOVERFLOW (it outgrew a capacity) or FCS_ESTATE (its state
  // became inconsistent, which no input should be able to cause)
  return first_err >= 0 ? (err_code == FCS_ESTATE ? FCS_ESTATE : FCS_EOVERFLOW) : FCS_OK;
}

int fcs_percentile(fcs_handle h, int64_t num, int64_t den, int32_t* value, uint8_t* saturated) {
  if (!h || !value || den < 1 || num < 0 || num > den) return FCS_EINVAL;
  if (!h->ran || h->hist_bins == 0 || !h->run_out.hist) return FCS_ESTATE;
  int rc = sync_last(h);
  if (rc != FCS_OK) return rc;
  const int64_t n_paths = h->run_replicas * h->n_cells;
  const int64_t bins = h->hist_bins;
  const int64_t batch = std::max<int64_t>(1, (64ll << 20) / (bins * 4));
  std::vector<uint32_t> buf;
  try {
    buf.resize(static_cast<size_t>(std::min(batch, n_paths) * bins));
  } catch (const std::bad_alloc&) {
    return FCS_ENOMEM;
  }
  for (int64_t p0 = 0; p0 < n_paths; p0 += batch) {
    const int64_t np = std::min(batch, n_paths - p0);
    if (hipMemcpy(buf.data(), h->run_out.hist + p0 * bins, sizeof(uint32_t) * np * bins, hipMemcpyDeviceToHost) !=
        hipSuccess)
      return FCS_EDEVICE;
    for (int64_t p = 0; p < np; ++p) {
      const uint32_t* hp = buf.data() + p * bins;
      uint64_t n = 0;
      for (int64_t b = 0; b < bins; ++b) n += hp[b];
      int64_t bucket = 0;
      if (n > 0) {
        // nearest rank: the k-th smallest with k = ceil(num * n / den), at least 1
        __uint128_t prod = static_cast<__uint128_t>(num) * n + static_cast<__uint128_t>(den - 1);
        uint64_t k = static_cast<uint64_t>(prod / static_cast<__uint128_t>(den));
        if (k < 1) k = 1;
        uint64_t cum = 0;
        for (bucket = 0; bucket < bins; ++bucket) {
          cum += hp[bucket];
          if (cum >= k) break;
        }
      }
      value[p0 + p] = static_cast<int32_t>(bucket << h->hist_shift);
      if (saturated) saturated[p0 + p] = (n > 0 && bucket == bins - 1) ? 1 : 0;
    }
  }
  return FCS_OK;
}

int fcs_stability_bound(const fcs_params* p, double* lambda_star) {
  if (!p || !lambda_star) return FCS_EINVAL;
  if (p->capacity < 1 || p->n_classes < 1 || p->n_classes > kMaxClasses || !p->prompt || !p->decode)
    return FCS_EINVAL;
  if (p->n_classes > 1 && !p->class_thr) return FCS_EINVAL;
  const double two32 = 4294967296.0;
  double ew = 0.0, prev = 0.0;
  for (int32_t c = 0; c < p->n_classes; ++c) {
    if (!law_ok(p->prompt[c], 0, 1 << 24) || !law_ok(p->decode[c], 0, 1 << 24)) return FCS_EINVAL;
    const double cur = (c + 1 < p->n_classes) ? static_cast<double>(p->class_thr[c]) : two32;
    const double pc = (cur - prev) / two32;
    prev = cur;
    double el, el2, eo, eo2;
    law_moments(p->prompt[c], el, el2);
    law_moments(p->decode[c], eo, eo2);
    ew += pc * (el * eo + 0.5 * (eo + eo2));  // E[l o + (o + o^2)/2], l and o independent
  }
  if (!(ew > 0.0)) return FCS_EINVAL;
  *lambda_star = static_cast<double>(p->capacity) / ew;
  return FCS_OK;
}

int fcs_protect_limit(double alpha, int32_t capacity, int32_t* limit) {
  if (!limit || !(alpha >= 0.0 && alpha <= 1.0) || capacity < 1 || capacity > kLimit) return FCS_EINVAL;
  const double room = (1.0 - alpha) * static_cast<double>(capacity);
  *limit = static_cast<int32_t>(std::floor(room));
  return FCS_OK;
}

int fcs_geometry(fcs_handle h, int32_t* lds_slots, int32_t* lds_bytes, int32_t* spill_slots) {
  if (!h) return FCS_EINVAL;
  if (!h->bound && !h->ran) return FCS_ESTATE;
  const int32_t lc = h->ran ? h->run_lcap : h->lcap, hc = h->ran ? h->run_hcap : h->hcap;
  if (lds_slots) *lds_slots = lc;
  if (lds_bytes) *lds_bytes = lds_words(lc, h->ran ? h->run_stack_lds : h->stack_lds, extra_lds_words(h)) * 4;
  if (spill_slots) *spill_slots = hc;
  return FCS_OK;
}

void fcs_destroy(fcs_handle h) { delete h; }

const char* fcs_strerror(int code) {
  switch (code) {
    case FCS_OK: return "ok";
    case FCS_EINVAL: return "invalid argument";
    case FCS_ENOMEM: return "workspace too small or out of host memory";
    case FCS_ESTATE: return "call out of order, or the state of a path became inconsistent";
    case FCS_EOVERFLOW: return "a path outgrew its active-set capacity";
    case FCS_EDEVICE: return "HIP error or no device";
    default: return "unknown error";
  }
}

int fcs_n_counters(void) { return FCS_N_COUNTERS; }

const char* fcs_counter_name(int i) {
  static const char* const names[FCS_N_COUNTERS] = {
      "arrived", "activations", "completed", "evictions", "overflow_steps", "sum_u", "sum_p", "sum_q",
      "decode_tokens", "prefill_tokens", "useful_tokens", "stalled", "sum_latency", "max_latency",
      "max_u", "max_p", "max_q", "final_u", "final_p", "final_q", "digest", "error", "error_step",
      "elapsed", "clock_start", "clock_end"};
  return (i >= 0 && i < FCS_N_COUNTERS) ? names[i] : nullptr;
}

}  // extern "C"
