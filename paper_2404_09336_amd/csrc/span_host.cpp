// Host-only parts of the span-attention library: span-list validation, work partitioning
// arithmetic and error strings.  No GPU call in this file.
#include <limits.h>

#include <algorithm>
#include <map>
#include <vector>

#include "span_attn.h"
#include "span_internal.h"

extern "C" int span_validate(int32_t batch, int32_t num_intervals, const int32_t* span_offsets,
                             const int32_t* span_starts, const int32_t* span_ends, const int32_t* ctx_lens,
                             int32_t* first_bad_seq, int32_t* first_bad_interval, int64_t* span_tokens_per_seq) {
  if (!span_offsets || !ctx_lens || !first_bad_seq || !first_bad_interval) return SPAN_ERR_NULL;
  if (num_intervals > 0 && (!span_starts || !span_ends)) return SPAN_ERR_NULL;
  if (batch < 0 || num_intervals < 0) return SPAN_ERR_SHAPE;
  *first_bad_seq = -1;
  *first_bad_interval = -1;
  for (int32_t b = 0; b < batch; ++b) {
    const int32_t first = span_offsets[b], last = span_offsets[b + 1];
    auto fail = [&](int code, int32_t interval) {
      *first_bad_seq = b;
      *first_bad_interval = interval;
      return code;
    };
    if (b == 0 && first != 0) return fail(SPAN_BAD_OFFSETS, -1);
    if (last < first || last > num_intervals) return fail(SPAN_BAD_OFFSETS, -1);
    if (last == first) return fail(SPAN_BAD_EMPTY_SPAN, -1);
    int64_t tokens = 0;
    int32_t prev_start = 0, prev_end = 0;
    for (int32_t i = first; i < last; ++i) {
      const int32_t s = span_starts[i], e = span_ends[i], k = i - first;
      if (s < 0 || e > ctx_lens[b]) return fail(SPAN_BAD_RANGE, k);
      if (s >= e) return fail(SPAN_BAD_EMPTY_INTERVAL, k);
      if (k > 0) {
        if (s < prev_start) return fail(SPAN_BAD_UNSORTED, k);
        if (s < prev_end) return fail(SPAN_BAD_OVERLAP, k);
      }
      tokens += (int64_t)e - (int64_t)s;
      prev_start = s;
      prev_end = e;
    }
    if (span_tokens_per_seq) span_tokens_per_seq[b] = tokens;
  }
  return SPAN_OK;
}

namespace spanattn {

int check_desc(const span_attn_desc_t* d) {
  if (!d) return SPAN_ERR_NULL;
  if (d->batch <= 0 || d->heads <= 0 || d->max_len <= 0 || d->max_len > kMaxLen) return SPAN_ERR_SHAPE;
  if (d->head_dim != 64 && d->head_dim != 128) return SPAN_ERR_SHAPE;
  if (d->num_intervals < 0 || d->max_tokens < 0 || d->num_splits < 0) return SPAN_ERR_SHAPE;
  if ((int64_t)d->batch * d->heads > INT_MAX / 2) return SPAN_ERR_SHAPE;
  if (d->batch > 65535) return SPAN_ERR_SHAPE;  // grid z limit
  if (d->dtype != SPAN_F32 && d->dtype != SPAN_F16 && d->dtype != SPAN_BF16) return SPAN_ERR_DTYPE;
  if (d->q_len < 0 || d->q_len > kMaxQueryTokens) return SPAN_ERR_SHAPE;
  return SPAN_OK;
}

int32_t query_tokens(const span_attn_desc_t* d) { return d->q_len > 1 ? d->q_len : 1; }

// Query tokens one launch serves: 1, 2 or 4 on the vector units (their register budget stops there), 16 on the
// matrix cores (16-bit types with head_dim 128).  The matrix pass takes over from three tokens: measured on
// batch 64 x ~155 attended positions, 32 heads, fp16: 3 tokens 31.9 us against 37.7 us for the four-token vector
// pass, 2 tokens 31.5 against 29.7; batch 8 x 300..2000 positions: 27.5 against 29.4 and 27.4 against 25.0.
#ifndef SPAN_MATRIX_PASS_FROM
#define SPAN_MATRIX_PASS_FROM 3
#endif
static int32_t queries_per_pass(const span_attn_desc_t* d) {
  const int32_t n = query_tokens(d);
  if (n >= SPAN_MATRIX_PASS_FROM && d->dtype != SPAN_F32 && d->head_dim == 128) return 16;
  return n >= 3 ? 4 : n;
}

// Workgroups of one resident round: the kernel for one query token runs 8 workgroups per CU, the one for
// two tokens 6, the ones for four and for sixteen tokens 4 (their register budgets).
static int64_t target_workgroups(const span_attn_desc_t* d) {
  const int32_t nq = queries_per_pass(d);
  return nq == 1 ? kTargetWorkgroups : kTargetWorkgroups * (nq == 2 ? 6 : 4) / 8;
}

static int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Slices (per head, over all sequences) a call aims at.  The upper end is one resident round of workgroups.  But
// few, large slices beat many small ones as long as the memory system stays busy and a ragged batch can still be
// levelled: a quarter of the wavefront slots saturates HBM, every slice costs its own start-up, and every extra
// slice of a pair a partial state and a ticket.  So: a quarter round, or two slices per sequence on average if
// that is more, never beyond one round.  Measured (batch x attended positions, 32 heads x 128, fp16; this rule
// against always filling the round): 1 x 8000 25.7 vs 30.5 us, 4 x 2000 26.5 vs 28.4, 8 x 200..1600 21.8 vs 23.1,
// 16 x 110..1100 30.0 vs 30.7, 8 x 6000 125.6 vs 130.8; 32 x 4096..16384 is one full round either way.
static int64_t slice_room(const span_attn_desc_t* d) {
  const int64_t round = target_workgroups(d);
  const int64_t most = round / d->heads, least = ceil_div(round / 4, d->heads);
  const int64_t room = std::max<int64_t>(least, 2 * (int64_t)d->batch);
  return std::max<int64_t>(1, std::min(room, most));
}

// Exact mode (the caller knows how many positions each sequence attends).
//
// All workgroups of a launch that fit on the chip at once start together and spend the same first
// microseconds walking the span metadata before any K row is requested; a second round of equal
// workgroups would repeat that dead time, and every extra slice costs a partial state and a ticket.
// So the aim is ONE resident round: the smallest slice size T for which all slices of all sequences,
// times heads, fit into kTargetWorkgroups.  Sequence b gets ceil(n_b / T) slices, which the kernel makes
// equal-sized.  When batch * heads alone exceeds a round, every sequence is one slice.
static int64_t slices_for(int64_t n, int64_t T) { return n <= 0 ? 1 : ceil_div(n, T); }

static bool plan_exact(const span_attn_desc_t* d, const int64_t* tokens_per_seq, int64_t max_tok, Partition* p,
                       uint32_t* table) {
  if (!tokens_per_seq || d->num_splits != 0 || d->batch > kMaxPlanBatch) return false;
  auto tokens = [&](int32_t b) {
    const int64_t n = tokens_per_seq[b];
    return n < 0 ? (int64_t)0 : (n > max_tok ? max_tok : n);
  };
  auto count = [&](int64_t T) {
    int64_t c = 0;
    for (int32_t b = 0; b < d->batch; ++b) c += slices_for(tokens(b), T);
    return c;
  };
  int64_t sum = 0, longest = 0;
  for (int32_t b = 0; b < d->batch; ++b) {
    sum += tokens(b);
    if (tokens(b) > longest) longest = tokens(b);
  }
  int64_t room = slice_room(d);  // slices (per head) the call aims at, at most one resident round
  if (room > kMaxPlanSlices) room = kMaxPlanSlices;
  int64_t T = ceil_div(sum, room);
  if (T < kMinSlice) T = kMinSlice;
  int64_t total = count(T);
  // A quarter of the chip's wavefront slots (512 workgroups) already keeps the memory system busy, and a
  // pair that is one workgroup needs no partial states and no tickets.  So a batch of at least 512 (batch,
  // head) pairs whose longest sequence is within 35 % of the mean runs unsplit (measured 5-10 % faster than
  // filling the round with slices: batch 16 x 555 tokens +-25 % 30.6 -> 27.9 us, batch 48 x 300 44.6 -> 42.3 us);
  // more ragged batches need the slices to level the work (batch 16, 112..1100 tokens: 30.3 split, 30.9 unsplit).
  const bool level = (int64_t)d->batch * d->heads >= kUnsplitFromPairs && longest * 100 * d->batch <= 135 * sum;
  if (room < d->batch || level) {  // whole sequences (batch * heads alone exceeds a round, or a level batch)
    T = max_tok > 0 ? max_tok : 1;
    total = count(T);
  } else {
    while (total > room) {  // grow T in proportion to the overshoot (at least one granule) and try again
      const int64_t next = ceil_div(ceil_div(T * total, room), kSliceGranule) * kSliceGranule;
      T = next > T ? next : T + kSliceGranule;
      total = count(T);
    }
    // fits: give back what the proportional step overshot
    for (int i = 0; i < 8 && T - kSliceGranule >= kMinSlice && count(T - kSliceGranule) <= room; ++i)
      T -= kSliceGranule;
    total = count(T);
  }
  // One round cannot always be level: when batch * heads (nearly) fills it, long and short sequences are
  // each one slice.  If the largest slice is then well above the average and large in itself, several
  // rounds of kLargeSlice-sized slices do better: their start-up hides behind the neighbours' streaming and
  // the hardware deals them to whichever CU is free.  (Level plans are left alone: cutting them further
  // only adds partial states; measured 2-4 % slower.)  The slice table bounds the number of slices.
  {
    int64_t largest_now = 1;
    for (int32_t b = 0; b < d->batch; ++b) {
      const int64_t n = tokens(b), per = ceil_div(n, slices_for(n, T));
      if (per > largest_now) largest_now = per;
    }
    if (largest_now > kLargeSlice && 2 * largest_now * total > 3 * sum) {
      int64_t T2 = kLargeSlice;
      while (T2 < T && count(T2) > kMaxPlanSlices) T2 += kLargeSlice / 4;
      if (T2 < T) {
        T = T2;
        total = count(T);
      }
    }
  }
  int64_t most = 1, least = kMaxPlanSplits + 1, largest = 1;
  for (int32_t b = 0; b < d->batch; ++b) {
    const int64_t n = tokens(b), nsl = slices_for(n, T);
    if (nsl > most) most = nsl;
    if (nsl < least) least = nsl;
    if (ceil_div(n, nsl) > largest) largest = ceil_div(n, nsl);
  }
  if (most != least) {  // sequences differ in their number of slices: the table is needed, and must fit
    if (total > kMaxPlanSlices || most > kMaxPlanSplits) return false;
    if (table) {
      int32_t y = 0;
      for (int32_t b = 0; b < d->batch; ++b) {
        const int64_t nsl = slices_for(tokens(b), T);
        for (int64_t s = 0; s < nsl; ++s) table[y++] = pack_slice((uint32_t)b, (uint32_t)s, (uint32_t)nsl);
      }
    }
  } else if (most > 65535) {
    return false;  // grid.y limit of the plain grid
  }
  p->exact = most != least;  // same count for every sequence: a (heads, slices, batch) grid says it all
  p->even = true;
  p->num_splits = (int32_t)most;
  p->slice_tokens = (int32_t)largest;
  p->max_tokens = (int32_t)max_tok;
  p->total_slices = (int32_t)total;
  p->queries_per_pass = queries_per_pass(d);
  p->granule = (int32_t)T;
  p->runs = false;
  return true;
}

static bool has_host_lists(const span_attn_desc_t* d) {
  return d->host_span_offsets && (d->num_intervals == 0 || (d->host_span_starts && d->host_span_ends));
}

// Attended positions of every sequence from the host copies of the span lists, with the clamps the kernel applies
// to the device lists (interval indices to [0, num_intervals], lengths to [0, max_len]).
static void tokens_from_host_lists(const span_attn_desc_t* d, std::vector<int64_t>* tokens) {
  tokens->assign((size_t)d->batch, 0);
  for (int32_t b = 0; b < d->batch; ++b) {
    const int32_t lo = std::min(std::max(d->host_span_offsets[b], 0), d->num_intervals);
    const int32_t hi = std::min(std::max(d->host_span_offsets[b + 1], lo), d->num_intervals);
    int64_t n = 0;
    for (int32_t i = lo; i < hi; ++i)
      n += std::min<int64_t>(std::max<int64_t>((int64_t)d->host_span_ends[i] - d->host_span_starts[i], 0), d->max_len);
    (*tokens)[(size_t)b] = n;
  }
}

// Run mode: resolves each slice of an exact plan to its runs of consecutive cache positions.  Sequence b has
// n_b attended positions, numbered 0 .. n_b-1 along its interval list, and ceil(n_b / granule) slices that share
// them evenly (as the kernel cuts them when it walks the device lists itself).  False if the plan does not fit the
// tables or a slice is larger than one position window per wave allows.
static bool plan_runs(const span_attn_desc_t* d, const int64_t* tokens_per_seq, const Partition& p, RunTables* r) {
  if (!p.even || d->batch > kMaxPlanBatch || p.total_slices > kMaxRunSlices) return false;
  int32_t y = 0, nruns = 0;
  for (int32_t b = 0; b < d->batch; ++b) {
    int64_t n = tokens_per_seq[b] < 0 ? 0 : tokens_per_seq[b];
    if (n > p.max_tokens) n = p.max_tokens;
    const int64_t nsl = slices_for(n, p.granule), T = ceil_div(n, nsl);
    if (T > kMaxRunSliceRows || nsl > kMaxPlanSplits) return false;
    const int32_t lo = std::min(std::max(d->host_span_offsets[b], 0), d->num_intervals);
    const int32_t hi = std::min(std::max(d->host_span_offsets[b + 1], lo), d->num_intervals);
    int32_t i = lo;        // interval the walk stands in
    int64_t before = 0;    // attended positions of the intervals before it
    for (int64_t s = 0; s < nsl; ++s) {
      if (y >= kMaxRunSlices) return false;
      const int64_t v0 = s * T, v1 = std::min(n, (s + 1) * T);  // the slice owns positions number v0 .. v1-1
      const int32_t first_run = nruns;
      for (int64_t v = v0; v < v1;) {
        int64_t len = 0;
        while (i < hi) {  // skip to the interval that holds position number v
          len = std::min<int64_t>(std::max<int64_t>((int64_t)d->host_span_ends[i] - d->host_span_starts[i], 0), d->max_len);
          if (v < before + len) break;
          before += len;
          ++i;
        }
        if (i >= hi) return false;  // (cannot happen: n was summed over the same list)
        const int64_t take = std::min(v1, before + len) - v;
        if (nruns >= kMaxRuns) return false;
        r->run[nruns][0] = (int32_t)std::min<int64_t>(std::max<int64_t>((int64_t)d->host_span_starts[i] + (v - before), INT32_MIN), INT32_MAX);
        r->run[nruns][1] = (int32_t)take;
        ++nruns;
        v += take;
      }
      r->slices[y].entry = pack_slice((uint32_t)b, (uint32_t)s, (uint32_t)nsl);
      r->slices[y].runs_of = (uint32_t)first_run | ((uint32_t)(nruns - first_run) << 16);
      r->slices[y].rows = (int32_t)(v1 > v0 ? v1 - v0 : 0);
      r->slices[y].reserved = 0;
      ++y;
    }
  }
  return y == p.total_slices;
}

// Uniform mode: every sequence gets the same number of slices, sized so that a call puts about
// kTargetWorkgroups workgroups on the chip (256 CUs x 8 resident workgroups), never fewer than kMinSlice
// positions per slice, never more than the kMaxSlice the kernel's position table holds.
Partition plan_partition(const span_attn_desc_t* d, uint32_t* table, RunTables* runs) {
  const int64_t max_tok = (d->max_tokens > 0 && d->max_tokens < d->max_len) ? d->max_tokens : d->max_len;
  Partition p;
  // Host copies of the span lists, when given, are the authority on the token counts (tokens_per_seq is then not
  // consulted), in every function that plans from this descriptor, so that they all agree.
  const int64_t* tokens = d->tokens_per_seq;
  std::vector<int64_t> from_lists;
  const bool lists = has_host_lists(d) && d->batch <= kMaxPlanBatch;
  if (lists) {
    tokens_from_host_lists(d, &from_lists);
    tokens = from_lists.data();
  }
  if (plan_exact(d, tokens, max_tok, &p, table)) {
    // Run mode pays where the launch carries a slice table anyway (sequences with different numbers of slices):
    // kernel arguments of that size cost a few tenths of a microsecond per launch, which a batch that needs no
    // table would pay on top (measured: batch 64 x 155 positions, one slice each, 27.7 -> 27.9 us with runs;
    // batch 8 and batch 16 sliced raggedly, 24.1 -> 23.7 us and 31.1 -> 30.8 us).
    if (lists && runs && p.exact) p.runs = plan_runs(d, tokens, p, runs);
    return p;
  }
  const int64_t pairs = (int64_t)d->batch * d->heads;
  int64_t splits = d->num_splits > 0 ? d->num_splits : slice_room(d) / d->batch;  // stay within one round
  const int64_t most = ceil_div(max_tok, kMinSlice);
  if (d->num_splits == 0 && splits > most) splits = most;
  if (splits > max_tok) splits = max_tok;
  if (splits < 1) splits = 1;
  int64_t slice = ceil_div(ceil_div(max_tok, splits), kSliceGranule) * kSliceGranule;
  if (slice > kMaxSlice) slice = kMaxSlice;
  while (ceil_div(max_tok, slice) > 65535) slice += kSliceGranule;  // grid.y limit
  splits = ceil_div(max_tok, slice);
  p.exact = false;
  p.even = false;
  p.num_splits = (int32_t)splits;
  p.slice_tokens = (int32_t)slice;
  p.max_tokens = (int32_t)max_tok;
  p.total_slices = (int32_t)(splits * d->batch);
  p.queries_per_pass = queries_per_pass(d);
  p.granule = (int32_t)slice;
  p.runs = false;
  return p;
}

size_t workspace_counter_bytes(const span_attn_desc_t* d) {
  const size_t n = (size_t)d->batch * d->heads * sizeof(int32_t);
  return (n + 255) & ~(size_t)255;
}

size_t workspace_ml_bytes(const span_attn_desc_t* d, const Partition& p) {
  const size_t n = (size_t)p.total_slices * d->heads * p.queries_per_pass * 2 * sizeof(float);
  return (n + 255) & ~(size_t)255;
}

size_t workspace_bytes(const span_attn_desc_t* d, const Partition& p) {
  if (p.num_splits <= 1) return 0;
  return workspace_counter_bytes(d) + workspace_ml_bytes(d, p) +
         (size_t)p.total_slices * d->heads * p.queries_per_pass * d->head_dim * sizeof(float);
}

}  // namespace spanattn

extern "C" int span_plan_query(const span_attn_desc_t* desc, span_plan_info_t* info) {
  if (!info) return SPAN_ERR_NULL;
  const int rc = spanattn::check_desc(desc);
  if (rc != SPAN_OK) return rc;
  spanattn::RunTables runs;
  const spanattn::Partition p = spanattn::plan_partition(desc, nullptr, &runs);
  info->runs_in_arguments = p.runs ? 1 : 0;
  info->queries_per_pass = p.queries_per_pass;
  info->exact = p.even ? 1 : 0;
  info->slice_tokens = p.slice_tokens;
  info->max_splits = p.num_splits;
  info->slice_limit = spanattn::kMaxSlice;
  info->workgroups = (int64_t)p.total_slices * desc->heads;
  info->workspace_bytes = (int64_t)spanattn::workspace_bytes(desc, p);
  return SPAN_OK;
}

extern "C" size_t span_workspace_bytes(const span_attn_desc_t* desc) {
  if (spanattn::check_desc(desc) != SPAN_OK) return 0;
  return spanattn::workspace_bytes(desc, spanattn::plan_partition(desc));
}

// ---- blocked encoding (block index + in-block bit mask) <-> interval lists ---------------------------
extern "C" int span_blocks_to_intervals(int32_t batch, int32_t block_size, const int32_t* block_offsets,
                                        const int32_t* block_idx, const uint32_t* block_masks, int32_t capacity,
                                        int32_t* span_offsets, int32_t* span_starts, int32_t* span_ends,
                                        int32_t* needed) {
  if (!block_offsets || !span_offsets || !needed) return SPAN_ERR_NULL;
  if (batch < 0 || capacity < 0 || block_size <= 0 || block_size % 32 != 0) return SPAN_ERR_SHAPE;
  if (capacity > 0 && (!span_starts || !span_ends)) return SPAN_ERR_NULL;
  const int32_t words = block_size / 32;
  int64_t count = 0;  // intervals produced so far (may run past capacity; writes stop at capacity)
  span_offsets[0] = 0;
  *needed = 0;
  for (int32_t b = 0; b < batch; ++b) {
    const int32_t first = block_offsets[b], last = block_offsets[b + 1];
    if ((b == 0 && first != 0) || last < first) return SPAN_BAD_OFFSETS;
    if (last > first && (!block_idx || !block_masks)) return SPAN_ERR_NULL;
    int64_t run_start = -1, run_end = -1;  // open run of attended positions, [run_start, run_end)
    auto close_run = [&]() {
      if (run_start < 0) return;
      if (count < capacity) {
        span_starts[count] = (int32_t)run_start;
        span_ends[count] = (int32_t)run_end;
      }
      ++count;
      run_start = -1;
    };
    for (int32_t j = first; j < last; ++j) {
      if (block_idx[j] < 0) return SPAN_BAD_RANGE;
      if (j > first && block_idx[j] <= block_idx[j - 1]) return SPAN_BAD_UNSORTED;
      const int64_t base = (int64_t)block_idx[j] * block_size;
      if (base + block_size > INT32_MAX) return SPAN_BAD_RANGE;
      for (int32_t w = 0; w < words; ++w) {
        const uint32_t m = block_masks[(size_t)j * words + w];
        for (int32_t t = 0; t < 32; ++t) {
          if (!((m >> t) & 1u)) continue;
          const int64_t pos = base + w * 32 + t;
          if (run_start >= 0 && pos == run_end) {
            ++run_end;
          } else {
            close_run();
            run_start = pos;
            run_end = pos + 1;
          }
        }
      }
    }
    close_run();
    if (count > INT32_MAX) return SPAN_ERR_SHAPE;
    span_offsets[b + 1] = (int32_t)count;
  }
  *needed = (int32_t)count;
  return count > capacity ? SPAN_ERR_CAPACITY : SPAN_OK;
}

extern "C" int span_intervals_to_blocks(int32_t batch, int32_t block_size, const int32_t* span_offsets,
                                        const int32_t* span_starts, const int32_t* span_ends, int32_t capacity,
                                        int32_t* block_offsets, int32_t* block_idx, uint32_t* block_masks,
                                        int32_t* needed) {
  if (!span_offsets || !block_offsets || !needed) return SPAN_ERR_NULL;
  if (batch < 0 || capacity < 0 || block_size <= 0 || block_size % 32 != 0) return SPAN_ERR_SHAPE;
  if (capacity > 0 && (!block_idx || !block_masks)) return SPAN_ERR_NULL;
  const int32_t words = block_size / 32;
  int64_t count = 0;
  block_offsets[0] = 0;
  *needed = 0;
  for (int32_t b = 0; b < batch; ++b) {
    const int32_t first = span_offsets[b], last = span_offsets[b + 1];
    if ((b == 0 && first != 0) || last < first) return SPAN_BAD_OFFSETS;
    if (last > first && (!span_starts || !span_ends)) return SPAN_ERR_NULL;
    std::map<int32_t, std::vector<uint32_t>> touched;  // block index -> mask words, ascending
    for (int32_t i = first; i < last; ++i) {
      const int32_t s = span_starts[i], e = span_ends[i];
      if (s < 0) return SPAN_BAD_RANGE;
      if (s >= e) return SPAN_BAD_EMPTY_INTERVAL;
      for (int64_t blk = s / block_size; blk * block_size < e; ++blk) {
        std::vector<uint32_t>& m = touched[(int32_t)blk];
        if (m.empty()) m.assign(words, 0u);
        const int64_t lo = std::max<int64_t>(s, blk * block_size) - blk * block_size;
        const int64_t hi = std::min<int64_t>(e, (blk + 1) * block_size) - blk * block_size;
        for (int64_t t = lo; t < hi; ++t) m[t / 32] |= 1u << (t % 32);
      }
    }
    for (const auto& kv : touched) {
      if (count < capacity) {
        block_idx[count] = kv.first;
        std::copy(kv.second.begin(), kv.second.end(), block_masks + (size_t)count * words);
      }
      ++count;
    }
    if (count > INT32_MAX) return SPAN_ERR_SHAPE;
    block_offsets[b + 1] = (int32_t)count;
  }
  *needed = (int32_t)count;
  return count > capacity ? SPAN_ERR_CAPACITY : SPAN_OK;
}

// ---- span builder: anchors + references -> sorted disjoint intervals ---------------------------------
extern "C" int span_build(int32_t num_anchors, const int32_t* anchor_starts, const int32_t* anchor_ends,
                          int32_t num_refs, const int32_t* ref_first, const int32_t* ref_last, int32_t prefix_end,
                          int32_t prev_line_start, int32_t cur_line_start, int32_t ctx_len, int32_t capacity,
                          int32_t* out_starts, int32_t* out_ends, int32_t* needed) {
  if (!needed) return SPAN_ERR_NULL;
  if (num_anchors < 0 || num_refs < 0 || capacity < 0 || ctx_len < 0) return SPAN_ERR_SHAPE;
  if (num_anchors > 0 && (!anchor_starts || !anchor_ends)) return SPAN_ERR_NULL;
  if (num_refs > 0 && (!ref_first || !ref_last)) return SPAN_ERR_NULL;
  if (capacity > 0 && (!out_starts || !out_ends)) return SPAN_ERR_NULL;
  *needed = 0;
  auto inside = [&](int32_t p) { return p >= 0 && p <= ctx_len; };
  if (!inside(prefix_end) || !inside(prev_line_start) || !inside(cur_line_start) || prev_line_start > cur_line_start)
    return SPAN_BAD_RANGE;
  std::vector<std::pair<int32_t, int32_t>> ranges;
  ranges.reserve((size_t)num_refs + 3);
  auto add = [&](int32_t s, int32_t e) {
    if (s < e) ranges.emplace_back(s, e);
  };
  add(0, prefix_end);
  add(cur_line_start, ctx_len);
  for (int32_t r = 0; r < num_refs; ++r) {
    if (ref_first[r] == -1) {  // the previous line
      add(prev_line_start, cur_line_start);
      continue;
    }
    if (ref_first[r] < 0 || ref_last[r] >= num_anchors || ref_first[r] > ref_last[r]) return SPAN_BAD_RANGE;
    for (int32_t k = ref_first[r]; k <= ref_last[r]; ++k) {
      if (anchor_starts[k] < 0 || anchor_ends[k] > ctx_len || anchor_starts[k] > anchor_ends[k]) return SPAN_BAD_RANGE;
      add(anchor_starts[k], anchor_ends[k]);
    }
  }
  std::sort(ranges.begin(), ranges.end());
  int64_t count = 0;
  int32_t cur_s = 0, cur_e = -1;  // open interval; cur_e < 0: none
  auto flush = [&]() {
    if (cur_e < 0) return;
    if (count < capacity) {
      out_starts[count] = cur_s;
      out_ends[count] = cur_e;
    }
    ++count;
  };
  for (const auto& r : ranges) {
    if (cur_e >= 0 && r.first <= cur_e) {  // overlapping or touching: extend
      if (r.second > cur_e) cur_e = r.second;
    } else {
      flush();
      cur_s = r.first;
      cur_e = r.second;
    }
  }
  flush();
  *needed = (int32_t)count;
  return count > capacity ? SPAN_ERR_CAPACITY : SPAN_OK;
}

extern "C" const char* span_strerror(int code) {
  switch (code) {
    case SPAN_OK: return "ok";
    case SPAN_ERR_NULL: return "a required pointer is NULL";
    case SPAN_ERR_SHAPE: return "unsupported shape (dims must be positive, head_dim 64 or 128, max_len <= 2^22)";
    case SPAN_ERR_DTYPE: return "unsupported dtype";
    case SPAN_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case SPAN_ERR_HIP: return "a HIP call failed (see span_last_hip_error)";
    case SPAN_ERR_CAPACITY: return "output array too small (needed size reported)";
    case SPAN_ERR_SCRATCH_LIMIT: return "the call needs more scratch than the library's static buffer holds";
    case SPAN_BAD_OFFSETS: return "span_offsets must start at 0, not decrease, and stay within num_intervals";
    case SPAN_BAD_RANGE: return "interval outside [0, ctx_len]";
    case SPAN_BAD_EMPTY_INTERVAL: return "interval with start >= end";
    case SPAN_BAD_OVERLAP: return "interval overlaps the previous one";
    case SPAN_BAD_UNSORTED: return "interval starts before the previous one";
    case SPAN_BAD_EMPTY_SPAN: return "sequence with no interval";
    default: return "unknown code";
  }
}
