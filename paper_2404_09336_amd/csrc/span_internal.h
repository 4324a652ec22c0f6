// Shared between the host-only and the kernel translation units of the library.
#ifndef SPAN_INTERNAL_H_
#define SPAN_INTERNAL_H_

#include <stddef.h>
#include <stdint.h>

#include "span_attn.h"

namespace spanattn {

constexpr int kWavesPerBlock = 4;          // 256 threads per workgroup
constexpr int kMaxSlice = 1024;            // attended positions one workgroup can own (LDS position table)
constexpr int kMinSlice = 64;              // do not cut work finer than this many positions
constexpr int kSliceGranule = 16;
constexpr int kMaxLen = 1 << 22;           // keeps every in-slab byte offset inside 32 bits
constexpr int64_t kTargetWorkgroups = 2048;  // 256 CUs x 8 resident workgroups

struct Partition {
  int32_t num_splits;    // KV slices per (batch, head)
  int32_t slice_tokens;  // attended positions per slice
  int32_t max_tokens;    // bound on attended positions per sequence used for the grid
};

int check_desc(const span_attn_desc_t* d);
Partition plan_partition(const span_attn_desc_t* d);
size_t workspace_counter_bytes(const span_attn_desc_t* d);
size_t workspace_ml_bytes(const span_attn_desc_t* d, const Partition& p);
size_t workspace_bytes(const span_attn_desc_t* d, const Partition& p);

}  // namespace spanattn
#endif
