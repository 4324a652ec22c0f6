/*
 * span_attn.h — C ABI of the span-restricted decode-attention library for MI355X (gfx950).
 *
 * The operation (paper Sec. 2.2, eqs. (4)-(6), for the single query row of the decoding
 * phase; Sec. 3.2 "Token generation" and Sec. 3.3 restrict it to the self-selected span):
 *
 *   S_b        = union of the half-open position intervals of sequence b
 *   s_j        = scale * q[b,h,:] . K[b,h,j,:]                       j in S_b
 *   out[b,h,:] = sum_j softmax_j(s)_j * V[b,h,j,:]
 *
 * Only K / V rows inside the intervals are read.  The span is kept per sequence and shared by
 * all heads (Sec. 3.3: separate metadata for each request of a batch; one kernel instance per
 * head and batch item).
 *
 * Conventions
 *   - "device" pointers are HIP device memory owned by the CALLER.  The library never
 *     allocates, frees or keeps them.  "host" pointers are ordinary CPU memory.
 *   - Work is enqueued on desc->stream; calls return without synchronising.
 *   - Return value: 0 = OK; negative = argument / runtime error found on the host before
 *     anything was launched (SPAN_ERR_*); positive = span-list validation class
 *     (SPAN_BAD_*, only from span_validate).  Nothing throws or aborts across this ABI.
 *   - Layouts, all contiguous: q and out [batch, heads, head_dim] ([batch, q_len, heads, head_dim]
 *     for span_decode_attn_multi); k_cache and v_cache
 *     [batch, heads, max_len, head_dim] (a KV cache pre-allocated to its maximum length, Sec. 4 "Hardware and software"),
 *     so an interval of n positions is one run of n*head_dim elements per (batch, head).
 *   - out is always fp32, whatever the input type.
 */
#ifndef SPAN_ATTN_H_
#define SPAN_ATTN_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { SPAN_F32 = 0, SPAN_F16 = 1, SPAN_BF16 = 2 } span_dtype_t;

enum {
  SPAN_OK = 0,
  SPAN_ERR_NULL = -1,      /* a required pointer is NULL                                       */
  SPAN_ERR_SHAPE = -2,     /* non-positive dimension, head_dim not 64 / 128, max_len > 2^22,
                              q_len outside what the entry point takes                         */
  SPAN_ERR_DTYPE = -3,     /* dtype is not a span_dtype_t                                      */
  SPAN_ERR_WORKSPACE = -4, /* workspace missing, misaligned (256 B) or smaller than required   */
  SPAN_ERR_HIP = -5,       /* a HIP call failed; see span_last_hip_error()                     */
  SPAN_ERR_CAPACITY = -6,  /* an output array is too small; the needed size is reported        */
  SPAN_ERR_SCRATCH_LIMIT = -7, /* span_decode_attn_static: the call needs more scratch than
                              SPAN_STATIC_SCRATCH_BYTES; use span_decode_attn with a workspace */
  SPAN_BAD_OFFSETS = 1,
  SPAN_BAD_RANGE = 2,
  SPAN_BAD_EMPTY_INTERVAL = 3,
  SPAN_BAD_OVERLAP = 4,
  SPAN_BAD_UNSORTED = 5,
  SPAN_BAD_EMPTY_SPAN = 6
};

typedef struct span_attn_desc {
  int32_t batch, heads;
  int32_t head_dim;        /* 64 or 128                                                          */
  int32_t max_len;         /* rows allocated per (batch, head) in the caches, <= 2^22            */
  int32_t dtype;           /* span_dtype_t of q, k_cache, v_cache                                */
  int32_t num_intervals;   /* entries held by span_starts / span_ends (span entry point only);
                              interval indices are clamped to it on the device                  */
  int32_t max_tokens;      /* upper bound on the attended positions of any one sequence (span
                              tokens, or ctx_lens for the dense call); sizes the grid.
                              0 = unknown, use max_len.  Positions beyond it are NOT attended.   */
  int32_t num_splits;      /* 0 = let the library choose; > 0 = requested number of KV slices
                              per (batch, head) (the library may raise it, see
                              span_plan_query)                                                   */
  const int64_t* tokens_per_seq; /* HOST int64 [batch] or NULL: attended positions of every sequence, as
                              span_validate returns them (for the dense call: ctx_lens widened).
                              Lets the library cut the batch into equal-sized slices with no idle
                              workgroup (ragged batches).  Read during the call only.  If it
                              understates a sequence, that sequence's excess positions may be
                              dropped; memory safety does not depend on it.  Ignored when
                              num_splits > 0 or batch > 1024.                                    */
  void* workspace;         /* device, 256-byte aligned, >= span_workspace_bytes(); may be NULL
                              when that is 0.  Its leading ticket counters must be zero before the
                              first call that uses it (span_workspace_init, or zero the buffer);
                              every call leaves them zero again.  Two calls that may overlap in
                              time must not share a workspace.                                  */
  size_t workspace_bytes;
  void* stream;            /* hipStream_t; NULL = the default stream                             */
  int32_t q_len;           /* query tokens per sequence: 0 or 1 for every entry point but
                              span_decode_attn_multi, which takes 1..64                          */
  const int32_t* host_span_offsets; /* HOST copies of span_offsets / span_starts / span_ends (the arrays     */
  const int32_t* host_span_starts;  /* span_validate was given), or all NULL.  The span is chosen once per   */
  const int32_t* host_span_ends;    /* group of tokens (Sec. 3.2 "Overhead"), so the host has the lists at
                              hand.  With them the library counts the attended positions itself
                              (tokens_per_seq is not consulted) and, when the sequences are cut into
                              different numbers of slices and the batch is small enough (<= 96 slices
                              and <= 288 position runs in all, <= 1024 positions per slice), resolves
                              every slice to its runs of cache positions on the host and passes the
                              runs in the kernel arguments in place of the slice table: the kernel
                              then reads no span metadata from device memory (about 2 % faster on
                              raggedly sliced batches).  The result is the same, bit for bit.  They must
                              describe the same spans as the device arrays (not checked; memory safety
                              does not depend on it) and are read during the call only.  Leave them
                              NULL when the device lists change without the host knowing (span_advance
                              inside a replayed graph) and for the dense calls.                        */
} span_attn_desc_t;

/*
 * Decode attention over each sequence's span (Sec. 3.2-3.3; Algorithm 1 gives the same
 * quantity block by block).
 *   q, k_cache, v_cache : device, desc->dtype, layouts above
 *   span_offsets        : device int32 [batch+1]; intervals of sequence b are
 *                         offsets[b] .. offsets[b+1]-1
 *   span_starts/ends    : device int32 [desc->num_intervals]; interval i covers positions
 *                         [starts[i], ends[i])
 *   ctx_lens            : device int32 [batch] or NULL.  Not needed to compute the result (the
 *                         intervals say which rows are read); accepted for symmetry with the
 *                         validator and ignored.
 *   scale               : multiplies every score (1/sqrt(head_dim) in the paper, eq. (4))
 *   out                 : device fp32 [batch, heads, head_dim]
 * The list is expected to have passed span_validate, but the kernel is correct for any order of
 * pairwise-disjoint intervals.  On a list that would not validate the result is unspecified, yet
 * no row outside [0, max_len) of the sequence's own cache slab is read, and interval indices
 * outside [0, num_intervals) are never read.  A sequence with no attended position gets an
 * all-zero output row (never NaN).
 */
int span_decode_attn(const span_attn_desc_t* desc, const void* q, const void* k_cache, const void* v_cache,
                     const int32_t* span_offsets, const int32_t* span_starts, const int32_t* span_ends,
                     const int32_t* ctx_lens, float scale, float* out);

/*
 * span_decode_attn for callers that cannot allocate device memory or hand in a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same plan, same
 * kernels and the same result as span_decode_attn; desc->workspace and desc->workspace_bytes are ignored.
 * The slices' partial softmax states and tickets go to an array the library itself owns in device memory:
 * SPAN_STATIC_SCRATCH_BYTES per GPU the library runs on, held until the process ends.  The call allocates
 * and frees nothing.  If the plan needs more than that (span_workspace_bytes(desc) tells), nothing is
 * launched and SPAN_ERR_SCRATCH_LIMIT is returned.
 * The device that owns desc->stream must be the current device.  The first call on a device looks up
 * where that device's array lives (do it once before a graph capture starts).  Every call clears the
 * tickets it will use (a small fill kernel on desc->stream ahead of the attention kernel), so the array
 * may hold anything from earlier calls of any shape.  All calls on one GPU share the one array: two
 * calls that may overlap in time on the same GPU (different streams, or graphs replayed concurrently)
 * race and give unspecified results - serialise them, or use span_decode_attn with separate workspaces.
 */
#define SPAN_STATIC_SCRATCH_BYTES (4u << 20)
int span_decode_attn_static(const span_attn_desc_t* desc, const void* q, const void* k_cache, const void* v_cache,
                            const int32_t* span_offsets, const int32_t* span_starts, const int32_t* span_ends,
                            const int32_t* ctx_lens, float scale, float* out);

/*
 * Few-query variant: desc->q_len consecutive new tokens of every sequence attend in one call, all
 * through the sequence's one span (a span is chosen once per group of tokens, Sec. 3.2, so the tokens
 * of a group share it).  Among themselves the tokens keep the causal mask of Sec. 2.2: query token j
 * of sequence b attends the span positions p <= q_pos[b] + j and no later one; eqs. (4)-(6) apply to
 * each query row.  Every K / V row of the span is fetched once per pass over the span and serves all
 * query tokens of the pass: up to 16 for fp16 / bf16 rows of head_dim 128 (from three tokens on the pass
 * runs on the matrix cores), up to 4 otherwise; q_len tokens take ceil(q_len / tokens per pass) passes
 * (span_plan_query reports the tokens per pass).  The weights of the matrix-core pass enter the p.V product
 * as two 16-bit terms (about 16 mantissa bits for bf16, 22 for fp16); sums and outputs are fp32.
 *   q      : device, desc->dtype, [batch, q_len, heads, head_dim]
 *   q_pos  : device int32 [batch], cache position of query token 0 (its K / V row, like those of the
 *            other new tokens, is already in the cache and inside the span if it is to be attended);
 *            NULL = no causal limit, every token attends the whole span
 *   out    : device fp32 [batch, q_len, heads, head_dim]
 * Everything else as for span_decode_attn; workspace size and plan depend on desc->q_len.  A query
 * token that sees no span position gets an all-zero row.
 */
int span_decode_attn_multi(const span_attn_desc_t* desc, const void* q, const void* k_cache, const void* v_cache,
                           const int32_t* span_offsets, const int32_t* span_starts, const int32_t* span_ends,
                           const int32_t* q_pos, float scale, float* out);

/*
 * Dense control: the same computation over S_b = [0, ctx_lens[b]) with no span metadata (decode
 * attention as in Sec. 2.2 "Token generation"; plays the role of the dense baseline of Sec. 4).
 *   ctx_lens : device int32 [batch]; values are clamped to [0, min(max_len, max_tokens)].
 */
int dense_decode_attn(const span_attn_desc_t* desc, const void* q, const void* k_cache, const void* v_cache,
                      const int32_t* ctx_lens, float scale, float* out);

/*
 * The two calls above fused with the step that precedes them in a decode loop: appending the new
 * token's K and V rows to the pre-allocated cache (Sec. 2.2 "KV-cache").  In one launch,
 *   k_cache[b, h, append_pos[b], :] = k_new[b, h, :]   (same for V)      for every b, h
 *   out = attention over the UPDATED cache (span / dense as above)
 *   k_new, v_new : device, desc->dtype, [batch, heads, head_dim]
 *   append_pos   : device int32 [batch]; a value outside [0, max_len) appends nothing for that sequence
 * The span (or ctx_lens) is expected to cover append_pos[b] - the new token attends to itself - but need
 * not; the row is appended even for a sequence that attends nothing.  Within the launch the row is taken from k_new / v_new, never re-read from the cache, so the
 * result does not depend on when the store lands; the cache holds the row when the call's work completes.
 */
int span_decode_attn_append(const span_attn_desc_t* desc, const void* q, const void* k_new, const void* v_new,
                            void* k_cache, void* v_cache, const int32_t* append_pos, const int32_t* span_offsets,
                            const int32_t* span_starts, const int32_t* span_ends, float scale, float* out);
int dense_decode_attn_append(const span_attn_desc_t* desc, const void* q, const void* k_new, const void* v_new,
                             void* k_cache, void* v_cache, const int32_t* append_pos, const int32_t* ctx_lens,
                             float scale, float* out);

/*
 * Few-query form of span_decode_attn_append: the desc->q_len new tokens of every sequence (a burst of
 * reference tokens, or speculated tokens, Sec. 3.2) are appended and attend in one call.  Token j of
 * sequence b goes to cache row append_pos[b] + j (rows outside [0, max_len) are not written) and attends
 * the span positions p <= append_pos[b] + j, as in span_decode_attn_multi with q_pos = append_pos.
 *   q, k_new, v_new : device, desc->dtype, [batch, q_len, heads, head_dim]
 *   out             : device fp32 [batch, q_len, heads, head_dim]
 * Within a launch the rows of that launch's tokens are taken from k_new / v_new, never re-read from the
 * cache; more tokens than one pass serves (16 or 4, see span_decode_attn_multi) take several launches on
 * the stream, each appending its own tokens' rows, which the later ones then read from the cache.
 */
int span_decode_attn_multi_append(const span_attn_desc_t* desc, const void* q, const void* k_new, const void* v_new,
                                  void* k_cache, void* v_cache, const int32_t* append_pos,
                                  const int32_t* span_offsets, const int32_t* span_starts, const int32_t* span_ends,
                                  float scale, float* out);

/*
 * The step between two decode steps of one group of tokens.  Anchors and references are generated
 * once per group (Sec. 3.2 "Overhead"), so the span is chosen per group: from one step of the group to
 * the next it only gains the tokens just decoded.  With n = max(desc->q_len, 1) tokens per step (1 for
 * the one-token calls, q_len for span_decode_attn_multi_append) and p = append_pos[b] the position the
 * first of them was appended at, for every sequence b, on desc->stream:
 *    if an interval ends at p + n (the appended tokens close it) and none of the positions
 *    p + n .. p + 2n - 1 is in the span yet, that interval now ends at p + 2n (the next step's tokens
 *    will attend themselves; their rows arrive with the next *_append call);
 *    append_pos[b] = p + n;  ctx_lens[b] += n when ctx_lens is not NULL.
 * Sequences with p < 0 or p + 2n > max_len (no room for another step) are left untouched.  All pointers
 * are device memory and are the arrays the next *_append call reads, so a decode loop over the group
 * needs no host work between steps and the pair of calls can be recorded into one HIP graph.  desc
 * supplies batch, max_len, num_intervals, q_len and stream.
 */
int span_advance(const span_attn_desc_t* desc, const int32_t* span_offsets, const int32_t* span_starts,
                 int32_t* span_ends, int32_t* append_pos, int32_t* ctx_lens);

/*
 * Span-list validation on the HOST (all pointers are host memory; pure CPU).
 * Sequences are scanned in index order; for a sequence its offsets are checked first, then its
 * intervals in list order, each against the rules in this order; the first failure is returned,
 * with *first_bad_seq and *first_bad_interval (index within the sequence's list, -1 when the
 * failure is not tied to one interval) set; both are -1 on success.
 *   SPAN_BAD_OFFSETS         offsets[0] != 0, offsets[b+1] < offsets[b] or offsets[b+1] > num_intervals
 *   SPAN_BAD_RANGE           start < 0 or end > ctx_lens[b]
 *   SPAN_BAD_EMPTY_INTERVAL  start >= end
 *   SPAN_BAD_OVERLAP         start_i >= start_{i-1} and start_i < end_{i-1}
 *   SPAN_BAD_UNSORTED        start_i < start_{i-1}
 *   SPAN_BAD_EMPTY_SPAN      the sequence has no interval (softmax over nothing)
 * Touching intervals (start_i == end_{i-1}) are legal.  span_tokens_per_seq (host int64 [batch],
 * may be NULL) receives sum(end - start) of every sequence that was scanned without failure.
 */
int span_validate(int32_t batch, int32_t num_intervals, const int32_t* span_offsets, const int32_t* span_starts,
                  const int32_t* span_ends, const int32_t* ctx_lens, int32_t* first_bad_seq,
                  int32_t* first_bad_interval, int64_t* span_tokens_per_seq);

/*
 * How the library would partition the call described by desc.  A (batch, head) pair whose span is
 * cut into one slice has its output row written directly; with more slices the partial softmax
 * states go through the workspace and the workgroup that finishes last for the pair merges them by
 * log-sum-exp (still one launch).  Pure host arithmetic.
 */
typedef struct span_plan_info {
  int32_t exact;           /* 1: slices sized from tokens_per_seq (no idle workgroup); 0: every
                              sequence gets max_splits slices of slice_tokens positions            */
  int32_t slice_tokens;    /* attended positions per slice (upper bound in exact mode)            */
  int32_t max_splits;      /* most slices any (batch, head) pair is cut into                      */
  int32_t slice_limit;     /* most positions one slice can own (a constant of the build)                */
  int64_t workgroups;      /* workgroups the call launches                                        */
  int64_t workspace_bytes; /* same value as span_workspace_bytes()                                */
  int32_t runs_in_arguments; /* 1: host_span_* were given and the plan fits: the slices' position runs
                              travel in the kernel arguments (span form)                          */
  int32_t queries_per_pass;  /* query tokens one launch serves (1, 2, 4 or 16): a call with q_len tokens
                              launches ceil(q_len / queries_per_pass) passes over the span        */
} span_plan_info_t;
int span_plan_query(const span_attn_desc_t* desc, span_plan_info_t* info);

/* Bytes of device workspace the call described by desc needs (0 when one slice is used). */
size_t span_workspace_bytes(const span_attn_desc_t* desc);

/*
 * Enqueues, on desc->stream, the zeroing of the ticket counters at the head of desc->workspace.
 * Needed once after the workspace is allocated (or after anything else wrote to it), not per call.
 * The zeroing is a small kernel launch, so the call may also be recorded into a HIP graph.
 */
int span_workspace_init(const span_attn_desc_t* desc);

/*
 * Blocked span encoding (Sec. 3.3 "Attention span encoding", Fig. 3): the context is cut into blocks
 * of block_size positions; a sequence lists only the blocks that contain span positions, each with its
 * block index and a mask of block_size bits (bit t of the mask, stored in 32-bit word t/32 at bit
 * t%32, stands for position block_idx*block_size + t).  These two HOST functions convert between that
 * encoding and the interval lists the kernels take.  All pointers are host memory.
 *
 * span_blocks_to_intervals: blocks of sequence b are block_offsets[b] .. block_offsets[b+1]-1 and must
 * have strictly increasing block_idx (else SPAN_BAD_UNSORTED; a negative index is SPAN_BAD_RANGE;
 * block_offsets that do not start at 0 or decrease are SPAN_BAD_OFFSETS; block_size must be a positive
 * multiple of 32, else SPAN_ERR_SHAPE).  Output: the maximal runs of set bits, in ascending order, runs
 * that continue across consecutive blocks joined - i.e. the unique sorted list of disjoint,
 * non-touching intervals of the same position set.  *needed receives the number of intervals; if it
 * exceeds capacity nothing past capacity is written and SPAN_ERR_CAPACITY is returned (span_offsets is
 * still complete, so a second call with enough room succeeds).
 *
 * span_intervals_to_blocks: the inverse, for any list of intervals with 0 <= start < end (order and
 * overlap do not matter: the result encodes the union).  Blocks come out in ascending order, untouched
 * blocks omitted.  *needed receives the number of blocks (same capacity rule; block_masks must hold
 * capacity * block_size/32 words).
 */
int span_blocks_to_intervals(int32_t batch, int32_t block_size, const int32_t* block_offsets,
                             const int32_t* block_idx, const uint32_t* block_masks, int32_t capacity,
                             int32_t* span_offsets, int32_t* span_starts, int32_t* span_ends, int32_t* needed);
int span_intervals_to_blocks(int32_t batch, int32_t block_size, const int32_t* span_offsets,
                             const int32_t* span_starts, const int32_t* span_ends, int32_t capacity,
                             int32_t* block_offsets, int32_t* block_idx, uint32_t* block_masks, int32_t* needed);

/*
 * Span builder (HOST, one sequence): anchors + references -> interval list (Sec. 3.2 "Anchors",
 * "Determining attention span", "Token generation"; Fig. 5 and Fig. 7 show the two reference styles).
 *   anchor_starts/ends [num_anchors] : position range [start, end) that anchor k stands for (the group of
 *                                      tokens it follows; whether the anchor's own tokens are inside the
 *                                      range is the caller's choice)
 *   ref_first/ref_last [num_refs]    : the references the model just emitted, each an inclusive range of
 *                                      anchor ids first..last (a single id has first == last; a line range
 *                                      "(a-b)" of the summarisation task is first = a, last = b).
 *                                      first == -1 is the special reference to the previous line,
 *                                      [prev_line_start, cur_line_start).
 *   prefix_end                       : the always-attended instruction is [0, prefix_end) (0 = none)
 *   cur_line_start, ctx_len          : the line being generated, [cur_line_start, ctx_len), is always
 *                                      attended (its own earlier tokens and the new token)
 * Output: the union of all those ranges as sorted, disjoint, non-touching intervals (so it passes
 * span_validate against ctx_len whenever it is not empty).  *needed receives their number; beyond
 * `capacity` nothing is written and SPAN_ERR_CAPACITY is returned.
 * Errors: an anchor id outside [0, num_anchors) or first > last -> SPAN_BAD_RANGE; a referenced anchor
 * whose range is not 0 <= start <= end <= ctx_len -> SPAN_BAD_RANGE; prefix_end, prev_line_start or
 * cur_line_start outside [0, ctx_len], or prev_line_start > cur_line_start -> SPAN_BAD_RANGE.
 */
int span_build(int32_t num_anchors, const int32_t* anchor_starts, const int32_t* anchor_ends, int32_t num_refs,
               const int32_t* ref_first, const int32_t* ref_last, int32_t prefix_end, int32_t prev_line_start,
               int32_t cur_line_start, int32_t ctx_len, int32_t capacity, int32_t* out_starts, int32_t* out_ends,
               int32_t* needed);

/* Static string for any code above. */
const char* span_strerror(int code);

/* The hipError_t (as int) of the last failed HIP call on this thread; 0 if none. */
int span_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* SPAN_ATTN_H_ */
