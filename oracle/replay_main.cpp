// Stand-alone driver of the CPU oracle (test infrastructure, like the rest of this folder): reads one case as a
// stream of integers on stdin, runs fo_run single-threaded and prints the counters, the completion slots
// and the latency histogram.  It exists so that the oracle can be run under the host compiler's address and
// undefined-behaviour sanitizers (which cannot be loaded into an unsanitized Python process); the test
// compares what it prints with the same case run through the shared library.
#include "fcs_oracle.cpp"

#include <cstdio>
#include <iostream>

namespace {

int64_t next_int() {
  long long v = 0;
  if (!(std::cin >> v)) {
    std::fprintf(stderr, "replay: input ends early\n");
    std::exit(2);
  }
  return v;
}

struct LawStore {
  std::vector<std::vector<uint32_t>> thr;
  fo_law read() {
    fo_law L;
    L.lo = static_cast<int32_t>(next_int());
    L.n_thr = static_cast<int32_t>(next_int());
    thr.emplace_back(static_cast<size_t>(L.n_thr));
    for (auto& v : thr.back()) v = static_cast<uint32_t>(next_int());
    L.thr = thr.back().data();
    return L;
  }
};

std::vector<int32_t> read_i32(int64_t n) {
  std::vector<int32_t> v(static_cast<size_t>(n > 0 ? n : 0));
  for (auto& x : v) x = static_cast<int32_t>(next_int());
  return v;
}

}  // namespace

int main() {
  LawStore store;
  store.thr.reserve(256);  // fo_law keeps pointers into the vectors: they must not move
  fo_config c{};
  c.policy = static_cast<int32_t>(next_int());
  c.n_classes = static_cast<int32_t>(next_int());
  c.capacity = next_int();
  c.token_budget = next_int();
  c.prefill_chunk = next_int();
  c.b_floor = static_cast<int32_t>(next_int());
  c.b_frac_thr = static_cast<uint32_t>(next_int());
  c.arrivals = store.read();
  std::vector<uint32_t> class_thr(static_cast<size_t>(c.n_classes > 1 ? c.n_classes - 1 : 0));
  for (auto& v : class_thr) v = static_cast<uint32_t>(next_int());
  c.class_thr = class_thr.data();
  std::vector<fo_law> prompt, decode, class_arr;
  for (int k = 0; k < c.n_classes; ++k) prompt.push_back(store.read());
  for (int k = 0; k < c.n_classes; ++k) decode.push_back(store.read());
  c.prompt = prompt.data();
  c.decode = decode.data();
  c.trace_every = static_cast<int32_t>(next_int());
  c.hist_bins = static_cast<int32_t>(next_int());
  c.hist_shift = static_cast<int32_t>(next_int());
  c.max_requests = next_int();
  c.n_forced = next_int();
  std::vector<int32_t> ft = read_i32(c.n_forced), fl = read_i32(c.n_forced), fo = read_i32(c.n_forced),
                       fc = read_i32(c.n_forced);
  c.forced_t = ft.data(); c.forced_l = fl.data(); c.forced_o = fo.data(); c.forced_cls = fc.data();
  c.n_forced_B = next_int();
  std::vector<int32_t> fb = read_i32(c.n_forced_B);
  c.forced_B = fb.data();
  std::vector<int32_t> class_budget;
  if (next_int() != 0) {
    for (int k = 0; k < c.n_classes; ++k) class_arr.push_back(store.read());
    class_budget = read_i32(c.n_classes);
    c.class_arrivals = class_arr.data();
    c.class_budget = class_budget.data();
  }
  c.protect_limit = next_int();
  c.budget_mode = static_cast<int32_t>(next_int());
  c.budget_law = store.read();
  c.budget_b16 = next_int();
  c.assumed_o = next_int();
  c.time_c0 = next_int(); c.time_cp = next_int(); c.time_cd = next_int();
  const int64_t n_ids = next_int();
  std::vector<int64_t> ids(static_cast<size_t>(n_ids));
  for (auto& v : ids) v = next_int();
  const int64_t T = next_int();
  const uint64_t seed = static_cast<uint64_t>(next_int());

  std::vector<uint64_t> counters(static_cast<size_t>(n_ids) * FO_N_COUNTERS);
  const size_t nreq = static_cast<size_t>(n_ids) * static_cast<size_t>(c.max_requests);
  std::vector<int32_t> arr(nreq), comp(nreq), fa(nreq), la(nreq), rl(nreq), ro(nreq);
  std::vector<uint32_t> hist(static_cast<size_t>(n_ids) * static_cast<size_t>(c.hist_bins));
  const size_t ntr = c.trace_every > 0 ? static_cast<size_t>(n_ids) * static_cast<size_t>(T / c.trace_every) : 0;
  std::vector<int32_t> tq(ntr), tu(ntr);
  fo_outputs out{};
  out.counters = counters.data();
  if (c.max_requests > 0) {
    out.arrival_step = arr.data(); out.completion_step = comp.data(); out.first_activation = fa.data();
    out.last_activation = la.data(); out.req_l = rl.data(); out.req_o = ro.data();
  }
  if (c.hist_bins > 0) out.hist = hist.data();
  if (ntr > 0) { out.trace_q = tq.data(); out.trace_u = tu.data(); }
  const int rc = fo_run(&c, n_ids, ids.data(), T, seed, 1, &out);
  if (rc != 0) {
    std::fprintf(stderr, "replay: fo_run refused the case (%d)\n", rc);
    return 3;
  }
  for (int64_t i = 0; i < n_ids; ++i) {
    std::printf("counters");
    for (int k = 0; k < FO_N_COUNTERS; ++k)
      std::printf(" %llu", static_cast<unsigned long long>(counters[static_cast<size_t>(i) * FO_N_COUNTERS + k]));
    std::printf("\ncompletion");
    for (int64_t k = 0; k < c.max_requests; ++k) std::printf(" %d", comp[static_cast<size_t>(i * c.max_requests + k)]);
    std::printf("\nhist");
    for (int64_t k = 0; k < c.hist_bins; ++k) std::printf(" %u", hist[static_cast<size_t>(i * c.hist_bins + k)]);
    std::printf("\n");
  }
  return 0;
}
