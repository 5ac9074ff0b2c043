// Internal layout shared by the host API and the device kernel of libfcs.
#ifndef FCS_INTERNAL_H_
#define FCS_INTERNAL_H_

#include <stdint.h>

#include "fcs.h"

namespace fcs {

// A law as the kernel sees it: thresholds and a guide of 2^kGuideBits + 1 entries live in the
// table blob.  guide[b] = #{ i : thr[i] < (b << (32 - kGuideBits)) }, so the inversion of a word u
// lies in [guide[u >> (32 - kGuideBits)], guide[(u >> (32 - kGuideBits)) + 1]].
struct DLaw {
  int32_t lo;
  int32_t n;
  uint32_t off;   // word offset of thr[] in the blob
  uint32_t goff;  // word offset of guide[] in the blob (length laws only)
};

struct DCell {
  int32_t policy;       // bits 7:0 FCS_POLICY_*, bits 15:8 FCS_BUDGET_* (FLOW)
  int32_t arrival;
  int32_t b_floor;      // FCS_BUDGET_LAW: index of the law of B_t
  uint32_t b_frac_thr;  // CLASSES: word offset in the blob of {arrival law, budget} x n_classes;
                        // ALPHA: (1 - alpha) M; FCS_BUDGET_CREDIT: b in units of 2^-16
};

// Words of one active-set slot: in LDS {END, footprint} pairs, PLEFT and the 4-word record; in the
// spill region END, PLEFT and the record.
constexpr int kLdsWordsPerSlot = 7;
constexpr int kSpillWordsPerSlot = 6;
// Words of one entry of the stack of evicted requests (its record).
constexpr int S_NFIELDS = 4;

constexpr int kWave = 64;
constexpr int kGuideBits = 16;
constexpr int kLdsBlock = 256;       // slots per b128 pass over the LDS tier
// Evicted-stack entries kept in LDS: a launch parameter (KParams::stack_lds), chosen with the number of LDS
// slots so that a path's LDS comes to a whole number of kilobytes, the unit in which a compute unit hands
// its LDS out.
constexpr int kStackLdsMin = 48, kStackLdsMax = 128;
constexpr int kScratchWords = 64;
constexpr int kCompactSlack = 64;    // compact when this many dead slots have accumulated
constexpr int kLdsCompactMin = 16;   // ... or this many when the next slot would be the first outside LDS
constexpr int kMaxCountThr = 63;
constexpr int kMaxClasses = 16;
constexpr int kMaxWheelSlots = 1024;  // longest output under the MC benchmark with known request types

struct KParams {
  const uint32_t* blob;
  uint32_t laws_off, cells_off, class_off;
  int32_t n_arrival_laws, n_classes, n_cells;
  int32_t M, tau, chunk;
  int32_t n_replicas;
  uint32_t replica_base;
  int32_t n_steps;
  uint32_t seed_lo, seed_hi;
  int32_t lcap, hcap, hscap;  // LDS slots, spill slots, spill stack entries (per path)
  int32_t stack_lds;          // entries of the evicted stack kept in LDS (kStackLdsMin .. kStackLdsMax)
  int32_t class_words;        // LDS words of the per-class tables (0 without CLASSES cells)
  int32_t wheel_slots;        // MC cells with known request types: future slots that the wheel of predicted
                              // departures spans (a multiple of 64, at least the longest output; else 0)
  int32_t all_policies;       // some cell is neither FLOW nor GREEDY: run the kernel built with all policies
  int32_t time_c0, time_cp, time_cd;  // slots of variable duration (all-policies kernel), else 0
  int32_t flags;              // FCS_FLAG_*
  int32_t* spill;             // per path: kSpillWordsPerSlot*hcap + S_NFIELDS*hscap words
  int64_t spill_stride;       // words per path
  int32_t trace_every, n_trace, hist_bins, hist_shift, max_requests;
  int32_t n_paths;
  // launch order of the cells (by the time their slowest path took in the launch before): the cell of the
  // k-th group of n_replicas workgroups, and where this launch records the longest path time per cell; or null
  const int32_t* order;
  unsigned long long* cost;
  // pacing words ({sum of paces, paths} twice, used by alternate launches) or null
  unsigned long long* pace;
  uint32_t launch_seq;
  fcs_outputs out;
};

// CLASSES cells keep three tables of 64 words per class in LDS (arrival counts of the current window,
// cumulative counts of the block the reader of each class queue stands in, arrival-law thresholds)
inline int class_lds_words(int n_classes) { return 3 * kWave * n_classes; }
inline int lds_words(int lcap, int stack_lds, int class_words) {
  return kLdsWordsPerSlot * lcap + S_NFIELDS * stack_lds + kScratchWords + class_words;
}

// Cells of an engine that take part in the ordering of a launch (more than that: cells run in index order).
constexpr int kMaxOrderedCells = 8192;
// Words of the schedule area that follows the tables in the blob: the longest path time per cell of the last two launches
// (two arrays of 64-bit words, used by alternate launches) and the launch order of the cells.
inline uint32_t sched_words(int n_cells) { return 5u * static_cast<uint32_t>(n_cells); }

// Defined in fcs_sim.hip; launches one single-wavefront workgroup per path (and before it, for engines of
// several cells, the kernel that orders the cells; sched_off = word offset of the schedule area in the blob).
int launch_sim(KParams kp, uint32_t sched_off, void* stream);

}  // namespace fcs
#endif
