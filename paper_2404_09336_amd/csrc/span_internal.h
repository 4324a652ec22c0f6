// Shared between the host-only and the kernel translation units of the library.
#ifndef SPAN_INTERNAL_H_
#define SPAN_INTERNAL_H_

#include <stddef.h>
#include <stdint.h>

#include "span_attn.h"

namespace spanattn {

constexpr int kWavesPerBlock = 4;          // 256 threads per workgroup
constexpr int kMaxSlice = 1 << 22;         // a slice may be a whole sequence (positions are tabulated window by window)
constexpr int kMinSlice = 128;             // do not cut work finer than this many positions
constexpr int kSliceGranule = 16;
constexpr int kUnsplitFromPairs = 512;     // level batches with at least this many (batch, head) pairs are not sliced
constexpr int kLargeSlice = 1024;          // slices above this size are cut down to it, in several rounds of workgroups
constexpr int kMaxLen = 1 << 22;           // keeps every in-slab byte offset inside 32 bits
constexpr int64_t kTargetWorkgroups = 2048;  // 256 CUs x 8 resident workgroups

constexpr int kInterleaveFrom = 384;        // slices at least this large deal their rows to the waves round-robin
constexpr int kMaxPlanSlices = 768;        // entries of the slice table passed as kernel argument
constexpr int kMaxPlanBatch = 1024;        // 10 bits of a table entry
constexpr int kMaxPlanSplits = 2047;       // 11 bits of a table entry
constexpr int kMaxQueryTokens = 64;        // few-query variant: query tokens per sequence and call

// Slice table entry (exact mode): batch index | slice index within the sequence | slices of the sequence.
inline uint32_t pack_slice(uint32_t b, uint32_t split, uint32_t nsl) { return b | (split << 10) | (nsl << 21); }

struct Partition {
  bool exact;            // slices come from the table; otherwise the grid is (heads, num_splits, batch)
  bool even;             // a sequence's slices share its own token count evenly (needs the caller's counts)
  int32_t num_splits;    // uniform: KV slices per (batch, head); exact: most slices of any sequence
  int32_t slice_tokens;  // attended positions per slice (exact: upper bound)
  int32_t max_tokens;    // bound on attended positions per sequence
  int32_t total_slices;  // exact: table entries (grid.y); uniform: batch * num_splits
  int32_t queries_per_pass;  // query tokens one launch serves (1, 2 or 4)
};

// Fills `table` (kMaxPlanSlices entries) when the partition is exact; table may be null to only size it.
Partition plan_partition(const span_attn_desc_t* d, uint32_t* table);
inline Partition plan_partition(const span_attn_desc_t* d) { return plan_partition(d, nullptr); }

int check_desc(const span_attn_desc_t* d);
int32_t query_tokens(const span_attn_desc_t* d);  // q_len of the descriptor, at least 1
size_t workspace_counter_bytes(const span_attn_desc_t* d);
size_t workspace_ml_bytes(const span_attn_desc_t* d, const Partition& p);
size_t workspace_bytes(const span_attn_desc_t* d, const Partition& p);

}  // namespace spanattn
#endif
