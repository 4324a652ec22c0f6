// Shared between the host-only and the kernel translation units of the library.
#ifndef SPAN_INTERNAL_H_
#define SPAN_INTERNAL_H_

#include <stddef.h>
#include <stdint.h>

#include "span_attn.h"

namespace spanattn {

constexpr int kWavesPerBlock = 4;          // 256 threads per workgroup
constexpr int kMaxSlice = 1 << 22;         // a slice may be a whole sequence (positions are tabulated window by window)
#ifndef SPAN_MIN_SLICE
#define SPAN_MIN_SLICE 128
#endif
constexpr int kMinSlice = SPAN_MIN_SLICE;  // do not cut work finer than this many positions
constexpr int kSliceGranule = 16;
constexpr int kUnsplitFromPairs = 512;     // level batches with at least this many (batch, head) pairs are not sliced
#ifndef SPAN_LARGE_SLICE
#define SPAN_LARGE_SLICE 1024
#endif
constexpr int kLargeSlice = SPAN_LARGE_SLICE;  // slices above this size are cut down to it, in several rounds of workgroups
constexpr int kMaxLen = 1 << 22;           // keeps every in-slab byte offset inside 32 bits
#ifndef SPAN_TARGET_WORKGROUPS
#define SPAN_TARGET_WORKGROUPS 2048
#endif
constexpr int64_t kTargetWorkgroups = SPAN_TARGET_WORKGROUPS;  // 256 CUs x 8 resident workgroups

constexpr int kInterleaveFrom = 384;        // slices at least this large deal their rows to the waves round-robin
constexpr int kMaxPlanSlices = 768;        // entries of the slice table passed as kernel argument
constexpr int kMaxPlanBatch = 1024;        // 10 bits of a table entry
constexpr int kMaxPlanSplits = 2047;       // 11 bits of a table entry
constexpr int kMaxQueryTokens = 64;        // few-query variant: query tokens per sequence and call

// Run mode: when the caller also hands in host copies of the span lists, the planner resolves every slice to its
// runs of consecutive cache positions and the runs travel in the kernel arguments (no span metadata is read from
// device memory before the first K row is requested).  Sized so that the arguments stay under 4 KB.
constexpr int kMaxRunSlices = 96;          // slices of all sequences (= grid.y)
constexpr int kMaxRuns = 288;              // runs of all slices
constexpr int kMaxRunSliceRows = 1024;     // rows of one slice: every wave's rows fit one position window

struct RunSlice {      // 16 bytes: one scalar load
  uint32_t entry;      // pack_slice(batch, slice, slices of the sequence), as in table mode
  uint32_t runs_of;    // first run | number of runs << 16
  int32_t rows;        // attended positions of the slice
  int32_t reserved;
};
struct RunTables {
  RunSlice slices[kMaxRunSlices];
  int32_t run[kMaxRuns][2];  // a run covers cache positions [run[.][0], run[.][0] + run[.][1])
};

// Slice table entry (exact mode): batch index | slice index within the sequence | slices of the sequence.
inline uint32_t pack_slice(uint32_t b, uint32_t split, uint32_t nsl) { return b | (split << 10) | (nsl << 21); }

struct Partition {
  bool exact;            // slices come from the table; otherwise the grid is (heads, num_splits, batch)
  bool even;             // a sequence's slices share its own token count evenly (needs the caller's counts)
  int32_t num_splits;    // uniform: KV slices per (batch, head); exact: most slices of any sequence
  int32_t slice_tokens;  // attended positions per slice (exact: upper bound)
  int32_t max_tokens;    // bound on attended positions per sequence
  int32_t total_slices;  // exact: table entries (grid.y); uniform: batch * num_splits
  int32_t queries_per_pass;  // query tokens one launch serves (1, 2, 4 or 16)
  int32_t granule;       // exact: sequence b is cut into ceil(n_b / granule) slices
  bool runs;             // the slices' position runs were resolved on the host (RunTables filled)
};

// Fills `table` (kMaxPlanSlices entries) when the partition is exact; table may be null to only size it.
// With `runs` given (span form only) and host copies of the span lists in the descriptor, tries run mode first.
Partition plan_partition(const span_attn_desc_t* d, uint32_t* table, RunTables* runs = nullptr);
inline Partition plan_partition(const span_attn_desc_t* d) { return plan_partition(d, nullptr, nullptr); }

int check_desc(const span_attn_desc_t* d);
int32_t query_tokens(const span_attn_desc_t* d);  // q_len of the descriptor, at least 1
size_t workspace_counter_bytes(const span_attn_desc_t* d);
size_t workspace_ml_bytes(const span_attn_desc_t* d, const Partition& p);
size_t workspace_bytes(const span_attn_desc_t* d, const Partition& p);

}  // namespace spanattn
#endif
