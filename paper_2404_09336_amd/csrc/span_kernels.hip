// Span-restricted single-query (decode) attention for gfx950: the kernel and the C entry points that launch it.
//
// What is computed: for every (batch b, head h), softmax over the scores of the positions in the
// sequence's span only, times the matching V rows (paper Sec. 2.2 eqs. (4)-(6) for one query row,
// restricted to the span as in Sec. 3.3).  The paper's own kernel visits fixed-size blocks that
// touch the span and masks inside them (Algorithm 1); here the span is a list of half-open position
// intervals, so exactly the rows inside the intervals are read and no mask exists.
//
// Mapping to the machine (single-query decode is a GEMV: one multiply-add per loaded element, so
// the kernel is bound by HBM and uses no matrix cores):
//   * grid = (heads, KV slices, batch).  A sequence's span is flattened into a virtual token index
//     0..n_b-1 (prefix sums of the interval lengths) and cut into slices; the host sizes the slices so
//     that one launch fills the chip about once (2048 workgroups), however large that makes a slice.
//     When the caller passes the per-sequence token counts, every sequence is cut into equal slices of
//     about the same size as everyone else's; if the sequences then differ in their number of slices the
//     grid becomes (heads, all slices of all sequences) and a table in the kernel arguments names each
//     slice's sequence, so ragged batches leave no idle workgroup.
//   * a workgroup is 4 wavefronts; each wavefront takes its share of the slice's rows (a contiguous
//     quarter, or every fourth 1 KiB unit of a large slice) and is independent of the others until the
//     final merge - it even builds its own part of the virtual-token -> position table (256 rows at a
//     time), so no barrier sits in front of the first K load.
//   * one 64-lane buffer load fetches 1 KiB = whole rows: D*sizeof(elt)/16 lanes per row, each lane a
//     128-bit piece, non-temporal.  The q.k dot product is finished with DPP adds inside those lanes;
//     every row group of a wavefront carries its own online-softmax state (m, l, acc), merged by
//     log-sum-exp at the end: first across row groups (shuffles), then across wavefronts (LDS), then
//     - only if the (batch, head) pair has more than one slice - across slices: every workgroup
//     publishes its state and takes a ticket; the one that arrives last for its pair merges them all,
//     so the whole call is a single launch.
//   * the append entry points also write the new token's K / V row into the cache; within that launch
//     the row is taken from the arguments, never read back from the cache.
//   * the few-query entry point serves 2 or 4 query tokens of a sequence with one pass over the span's rows
//     (template argument NQ): per-token softmax states in registers, each token under its own causal limit.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include <mutex>
#include <type_traits>

#include "span_attn.h"
#include "span_internal.h"

namespace spanattn {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

constexpr int kThreads = kWavesPerBlock * 64;
constexpr int kWin = 256;  // rows of a wave whose positions are tabulated at a time (one LDS window)

struct LaunchArgs {
  const void* q;
  const void* k;
  const void* v;
  float* out;
  const int32_t* offsets;
  const int32_t* starts;
  const int32_t* ends;
  const int32_t* ctx_lens;
  const void* k_new;           // append variant: the new token's K / V rows [batch, heads, D], else null
  const void* v_new;
  const int32_t* append_pos;   // append variant: [batch] cache row that receives them
  const int32_t* q_pos;        // few-query variant: [batch] cache position of query token 0 (causal limit), or null
  int32_t* counters;  // [batch*heads] arrival tickets of the slices; zero between calls
  // one slot per workgroup, slot = (first slice row of the sequence + slice) * heads + head:
  float* part_ml;   // [slots, NQ, 2]  (m in log2 units, l)
  float* part_acc;  // [slots, NQ, D]  un-normalised
  int32_t heads, max_len, num_intervals, slice_tokens, num_splits, max_tokens;
  int32_t q_len;                    // query tokens per sequence in q and out ([batch, q_len, heads, D])
  int32_t q_first;                  // few-query variant: first query token this launch handles
  float scale_log2e;
  int32_t total_slices;             // table mode: entries of `table` in use
  int32_t even;                     // 1: a sequence's slices share its own token count evenly; 0: slice_tokens each
  int32_t interleave;               // 1: rows dealt to the waves round-robin (large slices); 0: contiguous quarters
#ifdef SPAN_PHASE_TRACE
  unsigned long long* trace;        // diagnostic build only: [trace_workgroups, kTraceStamps] times of the phases, or null
  size_t trace_workgroups;
#endif
};
// Table mode: blockIdx.y indexes `table` (sequences have different numbers of slices).  The table makes
// the kernel arguments 3 KB larger, which costs about 0.35 us per launch, so calls that do not need it
// (every sequence has the same number of slices) use the plain arguments and a (heads, slices, batch) grid.
struct LaunchArgsTable : LaunchArgs {
  static constexpr bool kHasTable = true;
  static constexpr bool kHasRuns = false;
  uint32_t table[kMaxPlanSlices];   // pack_slice(batch, slice, slices of the sequence)
};
struct LaunchArgsPlain : LaunchArgs {
  static constexpr bool kHasTable = false;
  static constexpr bool kHasRuns = false;
};
// Run mode: blockIdx.y indexes the slices of all sequences, each resolved on the host to its runs of consecutive
// cache positions; the kernel reads no span metadata from device memory.
struct LaunchArgsRuns : LaunchArgs {
  static constexpr bool kHasTable = true;
  static constexpr bool kHasRuns = true;
  RunTables r;
};

// Diagnostic build (-DSPAN_PHASE_TRACE): every workgroup reads the constant-rate (100 MHz) clock at the phase
// boundaries named below into registers and thread 0 writes them out when the workgroup ends, so that taking a stamp
// puts no memory operation into the path it measures.  Each stamp names a value that must have been computed before
// the clock is read (the compiler may not move the read ahead of it).  The regular build compiles the stamps away.
// stamps: 0 kernel entry, 10 the sequence's interval range read (device lists), 1 span metadata read and slice known,
// 2 first position table built, 3 first K / V rows consumed, 4 all rows consumed, 5 waves merged in LDS, 6 output row
// stored and acknowledged (one slice per pair), 7 partial state published and acknowledged, 8 ticket returned,
// 9 slices merged, output row stored and acknowledged (last arrival only)
constexpr int kTraceStamps = 16;
#ifdef SPAN_PHASE_TRACE
#define SPAN_TRACE_DECL unsigned long long trace_t[11] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0}
#define SPAN_STAMP_AFTER(i, constraint, value)        \
  do {                                                \
    asm volatile("" ::constraint(value) : "memory");  \
    trace_t[i] = wall_clock64();                      \
    asm volatile("" ::: "memory");                    \
  } while (0)
#define SPAN_STAMP_ACKED(i)                                  \
  do {                                                       \
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory"); \
    trace_t[i] = wall_clock64();                             \
    asm volatile("" ::: "memory");                           \
  } while (0)
#define SPAN_TRACE_FLUSH()                                                                                     \
  do {                                                                                                         \
    const size_t wg_ = (size_t)(blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x;                 \
    if (threadIdx.x == 0 && a.trace && wg_ < a.trace_workgroups) {                                             \
      for (int i_ = 0; i_ < 11; ++i_) a.trace[wg_ * kTraceStamps + i_] = trace_t[i_];                          \
    }                                                                                                          \
  } while (0)
#else
#define SPAN_TRACE_DECL \
  do {                  \
  } while (0)
#define SPAN_STAMP_AFTER(i, constraint, value) \
  do {                                         \
  } while (0)
#define SPAN_STAMP_ACKED(i) \
  do {                      \
  } while (0)
#define SPAN_TRACE_FLUSH() \
  do {                     \
  } while (0)
#endif

// ---- storage types ---------------------------------------------------------------------------------
// unpack: 16 bytes of a row -> fp32 (for the V accumulation).
// The q.k partial product of a lane's 16 bytes never unpacks the 16-bit types: q stays in its stored
// form and v_dot2 multiplies two pairs per instruction into an fp32 sum (products of 16-bit floats are
// exact in fp32); the score scale is applied to the finished dot product (kPostScale).  fp32 rows use
// plain FMAs against a q that was scaled once up front.
struct F32 {
  static constexpr int kBytes = 4, kPerVec = 4;
  static constexpr bool kPostScale = false;
  static constexpr bool kHasMfma = false;  // (the sixteen-query pass exists for the 16-bit types)
  struct Q {
    float f[4];
  };
  static __device__ __forceinline__ void unpack(const u32x4& r, float* f) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t w = r[i];  // (bit_cast straight from a vector element reads element 0 every time)
      f[i] = __builtin_bit_cast(float, w);
    }
  }
  static __device__ __forceinline__ Q make_q(const u32x4& r, float scale) {
    Q q;
    unpack(r, q.f);
#pragma unroll
    for (int i = 0; i < 4; ++i) q.f[i] *= scale;
    return q;
  }
  static __device__ __forceinline__ float dot(const u32x4& k, const Q& q) {
    float kf[4];
    unpack(k, kf);
    float d = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) d = fmaf(kf[i], q.f[i], d);
    return d;
  }
};
struct F16 {
  static constexpr int kBytes = 2, kPerVec = 8;
  static constexpr bool kPostScale = true;
  static constexpr bool kHasMfma = true;
  static constexpr uint32_t kExponent = 0x7c00u;  // all ones: infinity or NaN
  typedef u32x4 Q;
  // C (16x16, fp32) += A (16x16) * B (16x16): four 16-bit elements of A and of B per lane, two dwords each
  static __device__ __forceinline__ f32x4 mfma(u32x2 a, u32x2 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(f16x4, a), __builtin_bit_cast(f16x4, b), c, 0, 0, 0);
  }
  // p (fp32, >= 0) as hi + lo in the storage type: hi is p rounded, lo the rounded remainder (together ~22 bits)
  static __device__ __forceinline__ void split(const float* p, u32x2& hi, u32x2& lo) {
    f16x4 h, r;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      h[i] = (_Float16)p[i];
      r[i] = (_Float16)(p[i] - (float)h[i]);
    }
    hi = __builtin_bit_cast(u32x2, h);
    lo = __builtin_bit_cast(u32x2, r);
  }
  static __device__ __forceinline__ void unpack(const u32x4& r, float* f) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t w = r[i];
      const f16x2 h = __builtin_bit_cast(f16x2, w);
      f[2 * i] = (float)h.x;
      f[2 * i + 1] = (float)h.y;
    }
  }
  static __device__ __forceinline__ Q make_q(const u32x4& r, float) { return r; }
  static __device__ __forceinline__ float dot(const u32x4& k, const Q& q) {
    float d = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t kw = k[i], qw = q[i];
      d = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, kw), __builtin_bit_cast(f16x2, qw), d, false);
    }
    return d;
  }
};
struct BF16 {
  static constexpr int kBytes = 2, kPerVec = 8;
  static constexpr bool kPostScale = true;
  static constexpr bool kHasMfma = true;
  static constexpr uint32_t kExponent = 0x7f80u;
  typedef u32x4 Q;
  static __device__ __forceinline__ f32x4 mfma(u32x2 a, u32x2 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(i16x4, a), __builtin_bit_cast(i16x4, b), c, 0, 0, 0);
  }
  static __device__ __forceinline__ uint32_t to_bf16(float x) {  // round to nearest even (x finite, >= 0 here)
    const uint32_t u = __builtin_bit_cast(uint32_t, x);
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
  }
  static __device__ __forceinline__ void split(const float* p, u32x2& hi, u32x2& lo) {
    uint32_t h[4], r[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      h[i] = to_bf16(p[i]);
      r[i] = to_bf16(p[i] - __builtin_bit_cast(float, h[i] << 16));
    }
    hi = u32x2{h[0] | (h[1] << 16), h[2] | (h[3] << 16)};
    lo = u32x2{r[0] | (r[1] << 16), r[2] | (r[3] << 16)};
  }
  static __device__ __forceinline__ void unpack(const u32x4& r, float* f) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t w = r[i];
      f[2 * i] = __builtin_bit_cast(float, w << 16);
      f[2 * i + 1] = __builtin_bit_cast(float, w & 0xffff0000u);
    }
  }
  static __device__ __forceinline__ Q make_q(const u32x4& r, float) { return r; }
  static __device__ __forceinline__ float dot(const u32x4& k, const Q& q) {
    float d = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t kw = k[i], qw = q[i];
      d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, kw), __builtin_bit_cast(bf16x2, qw), d, false);
    }
    return d;
  }
};

// ---- cross-lane helpers (wave64) ---------------------------------------------------------------
template <int kCtrl>
__device__ __forceinline__ float dpp_f(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), kCtrl, 0xf, 0xf, true));
}
template <int kCtrl>
__device__ __forceinline__ int dpp_i(int x) {
  return __builtin_amdgcn_update_dpp(0, x, kCtrl, 0xf, 0xf, true);
}

// Sum over each aligned group of kLanes lanes (8, 16 or 32); every lane of the group gets the sum.
template <int kLanes>
__device__ __forceinline__ float group_allreduce_sum(float x) {
  x += dpp_f<0xB1>(x);                          // quad_perm [1,0,3,2]
  x += dpp_f<0x4E>(x);                          // quad_perm [2,3,0,1]
  if (kLanes >= 8) x += dpp_f<0x141>(x);        // row_half_mirror
  if (kLanes >= 16) x += dpp_f<0x140>(x);       // row_mirror
  if (kLanes >= 32) x += __shfl_xor(x, 16, 64);
  return x;
}

// Inclusive prefix sum over the 64 lanes.
__device__ __forceinline__ int wave_inclusive_scan(int x, int lane) {
  x += dpp_i<0x111>(x);  // row_shr:1   (lanes without a source inside their row of 16 add 0)
  x += dpp_i<0x112>(x);  // row_shr:2
  x += dpp_i<0x114>(x);  // row_shr:4
  x += dpp_i<0x118>(x);  // row_shr:8
  const int t0 = __builtin_amdgcn_readlane(x, 15);
  const int t1 = __builtin_amdgcn_readlane(x, 31);
  const int t2 = __builtin_amdgcn_readlane(x, 47);
  const int row = lane >> 4;
  x += (row >= 1 ? t0 : 0) + (row >= 2 ? t1 : 0) + (row >= 3 ? t2 : 0);
  return x;
}

__device__ __forceinline__ int clampi(int x, int lo, int hi) { return x < lo ? lo : (x > hi ? hi : x); }

// K / V rows are fetched with raw buffer loads: the descriptor covers exactly one (batch, head) slab,
// so the hardware itself returns zeros for any offset outside it, and the cache policy is explicit.
// Non-temporal (streaming) loads: every row is used once; measured 17 % faster than default-policy loads.
// A wave sends its first batch of row loads, and consumes it, at raised instruction priority and drops back to the
// default for the rest of its rows.  Among waves of equal priority a SIMD issues the oldest first, so without this the
// waves of the workgroups that arrived last on a CU get their first rows only when the earlier ones are nearly done
// (per-workgroup stamps: first rows after 4 us for the first quarter of a launch, after 15-18 us for the last) and
// the launch ends on a thin tail of late starters.  Measured on batch 64 x ~155 positions: 27.67 -> 27.11 us; raising
// the priority for the start-up chain as well, or by progress through the rows, gains less or loses.  One-token
// kernels for 16-bit rows of 128 only, and only launches whose slices hold up to four batches of rows per wave (kBoost
// instances, chosen by the launcher): the passes that serve several tokens lose by it (3 tokens: 31.9 -> 33.6 us), fp32
// rows at the same shape (5 batches) lose 1 %, 16-bit rows of 64 lose 6 %, 9 batches (batch 8 x 300..2000) lose 0.5 %,
// 16 and more gain nothing;
// even the untaken branch in the loop costs the longer streams 0.5 %, hence instances of their own.
#ifndef SPAN_FIRST_BATCH_PRIORITY
#define SPAN_FIRST_BATCH_PRIORITY 3  // (a measurement build sets 0 to time the default arbitration)
#endif
constexpr int kBoostUpToBatches = 4;  // per wave
__device__ __forceinline__ void first_batch_priority(bool first_batch) {
#if SPAN_FIRST_BATCH_PRIORITY > 0
  if (first_batch) __builtin_amdgcn_s_setprio(SPAN_FIRST_BATCH_PRIORITY);
  else __builtin_amdgcn_s_setprio(0);
#else
  (void)first_batch;
#endif
}
#ifndef SPAN_ROW_LOAD_POLICY
#define SPAN_ROW_LOAD_POLICY 2  // (a measurement build overrides it to time the other policies)
#endif
constexpr int kRowLoadPolicy = SPAN_ROW_LOAD_POLICY;  // bit 0 = sc0, bit 1 = nt, bit 4 = sc1
__device__ __forceinline__ __amdgpu_buffer_rsrc_t slab_resource(const void* slab, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(slab), 0, bytes, 0x00020000);
}
__device__ __forceinline__ u32x4 load_row_piece(__amdgpu_buffer_rsrc_t slab, uint32_t byte_off) {
  return __builtin_amdgcn_raw_buffer_load_b128(slab, byte_off, 0, kRowLoadPolicy);
}

// Device-coherent store / load of one float that another workgroup reads / wrote in the same kernel.
__device__ __forceinline__ void publish(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float observe(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Merge two un-normalised softmax states held in log2 units.
__device__ __forceinline__ void merge_state(float& m, float& l, float* acc, int n, float m2, float l2,
                                            const float* acc2) {
  const float mn = fmaxf(m, m2);
  const float ms = (mn == -INFINITY) ? 0.f : mn;
  const float a = __builtin_amdgcn_exp2f(m - ms), b = __builtin_amdgcn_exp2f(m2 - ms);
  // one rounding order, written out: the compiler may contract x*a + y*b either way round, and every instance of
  // the kernel has to give the same bits
  l = fmaf(l, a, l2 * b);
  for (int i = 0; i < n; ++i) acc[i] = fmaf(acc[i], a, acc2[i] * b);
  m = mn;
}

// ---- the streaming kernel ------------------------------------------------------------------------
// NQ query tokens per sequence are served by one pass over the span's rows (NQ = 1: the decode step proper).
// The register budget is 64 per lane for one query (8 waves per SIMD), 80 for two (6) and 128 for four (4).
//
// NQ = 16 (16-bit types, D = 128) is a dense contraction and runs on the matrix cores: a wave takes its rows in
// tiles of 16, scores S^T = K Q^T and outputs O^T = V^T P^T are 16x16x16 MFMAs, the running sums stay in the
// accumulator layout.  Four waves per SIMD (128 registers) with one tile in flight per wave measured best: three
// waves with one or two tiles in flight are 10-14 % slower on batch 64 x ~155 positions.
#ifndef SPAN_MQ_WAVES
#define SPAN_MQ_WAVES 4  // (a measurement build overrides these two to time the other shapes)
#endif
#ifndef SPAN_MQ_TILES
#define SPAN_MQ_TILES 1
#endif
constexpr int waves_per_simd(int nq) { return nq == 1 ? 8 : (nq == 2 ? 6 : (nq == 4 ? 4 : SPAN_MQ_WAVES)); }

template <class Elt, int D, bool kDense, int U, int NQ, class Args, bool kBoost = false>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(waves_per_simd(NQ), waves_per_simd(NQ)))) void decode_kernel(
    const Args a) {
  constexpr int EPL = Elt::kPerVec;        // elements per lane (one 128-bit piece)
  constexpr int LPR = D / EPL;             // lanes per row
  constexpr int RPL = 64 / LPR;            // rows per wave-wide load
  constexpr uint32_t ROWB = D * Elt::kBytes;
  static_assert(LPR == 8 || LPR == 16 || LPR == 32, "row must span 8, 16 or 32 lanes");

  // heads vary fastest: consecutive workgroups go to different XCDs, and the 'is this slice empty'
  // answer is the same for all heads of a (batch, slice), so full and empty slices spread evenly
  SPAN_TRACE_DECL;
  SPAN_STAMP_AFTER(0, "s", 0);
  const int h = blockIdx.x;
  int b, split, nsl, y0;  // sequence, slice within it, slices of the sequence, first slice row of the sequence
  if constexpr (Args::kHasTable) {
    uint32_t e;
    if constexpr (Args::kHasRuns) e = a.r.slices[blockIdx.y].entry;
    else e = a.table[blockIdx.y];
    b = e & 1023u;
    split = (e >> 10) & 2047u;
    nsl = e >> 21;
    y0 = blockIdx.y - split;
  } else {
    b = blockIdx.z;
    split = blockIdx.y;
    nsl = a.num_splits;
    y0 = b * nsl;
  }
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // in a scalar register: what derives from it stays scalar
  const int grp = lane / LPR, lir = lane % LPR;
  const size_t bh = (size_t)b * a.heads + h;

  // Append variant.  Every lane fetches its piece of the new token's K / V row right away (the latency
  // hides behind the metadata chain).  The row is written into the cache by the first slice's workgroup
  // of each (batch, head) and, in this launch, never read back from the cache: the wave that meets
  // position new_pos in its rows takes it from the copy parked in LDS instead, so the kernel has no race.
  // With several query tokens (NQ > 1) every token brings a row, for positions append_pos[b] + token; they are
  // handled with the rows that only some tokens of the pass see (below) and new_pos stays unused.
  const bool append_many = NQ > 1 && a.append_pos != nullptr;
  const int new_pos = (NQ == 1 && a.append_pos) ? a.append_pos[b] : -2;  // -2 matches no position
  u32x4 kn_raw = {0u, 0u, 0u, 0u}, vn_raw = {0u, 0u, 0u, 0u};
  if (NQ == 1 && a.append_pos) {
    kn_raw = *reinterpret_cast<const u32x4*>((const char*)a.k_new + bh * ROWB + (uint32_t)lir * 16u);
    vn_raw = *reinterpret_cast<const u32x4*>((const char*)a.v_new + bh * ROWB + (uint32_t)lir * 16u);
  }

  // Tables of the streaming phase and the waves' states of the merge phase.  The sixteen-query pass overlays the
  // two (a barrier separates the phases there), which keeps it at four workgroups per CU.
  constexpr int kAccPad = NQ == 16 ? 4 : 0;  // (its rows are padded by 16 bytes: the accumulator layout's stores spread over the banks)
  constexpr int kQRow = 272;  // sixteen-query pass: q in rows of 256 + 16 bytes (operand reads spread over the banks)
  struct StreamTables {
    int pos[kWavesPerBlock][kWin];
    int pref[kWavesPerBlock][64];
    int start[kWavesPerBlock][64];
    unsigned char q[NQ == 16 ? 16 * kQRow : 16] __attribute__((aligned(16)));
  };
  typedef float WaveStates[kWavesPerBlock][NQ][D + kAccPad];
  struct Apart {
    StreamTables st;
    WaveStates acc;
  };
  union Overlaid {
    StreamTables st;
    WaveStates acc;
  };
  __shared__ __attribute__((aligned(16))) std::conditional_t<NQ == 16, Overlaid, Apart> s_u;
  auto& s_pos = s_u.st.pos;
  auto& s_pref = s_u.st.pref;
  auto& s_start = s_u.st.start;
  auto& s_acc = s_u.acc;
  __shared__ u32x4 s_new[NQ == 1 ? kWavesPerBlock : 1][2][LPR];  // append variant: the new K / V row, parked until its owner needs it
  __shared__ float s_ml[kWavesPerBlock][NQ][2];
  constexpr int kSliceGroups = NQ == 16 ? 1 : kThreads / D;  // thread groups of the slice merge, see step 5
  __shared__ float s_gm[kSliceGroups][NQ], s_gl[kSliceGroups][NQ];
  auto& s_q = s_u.st.q;
  __shared__ float s_wgt[NQ == 16 ? kWavesPerBlock : 1][16], s_M[16], s_L[16];
  __shared__ int s_ticket;
#ifdef SPAN_STAGE_LDS
  __shared__ u32x4 s_stage[kWavesPerBlock][2][U][64];  // measurement build: U K tiles and U V tiles of 1 KiB per wave
#endif

  // Query token j of this launch is row (b, q_first + j, h) of q and out; a launch whose last tokens do
  // not exist (q_len not a multiple of NQ) computes them from the last real one and never writes them.
  const int nq_here = NQ == 1 ? 1 : min(NQ, a.q_len - a.q_first);  // (the one-token kernel serves one token, whatever q_len says)
  auto qrow = [&](int j) { return ((size_t)b * a.q_len + (size_t)(a.q_first + min(j, nq_here - 1))) * a.heads + h; };
  // q pieces of this lane.  Scores carry the factor scale*log2(e), so that exp() becomes exp2(): fp32 q is
  // multiplied by it here, 16-bit q stays as stored and the finished dot product is multiplied instead.
  constexpr int kVq = NQ == 16 ? 1 : NQ;  // (the sixteen-query pass keeps q in the matrix operand layout instead)
  typename Elt::Q qv[kVq];
  if constexpr (NQ < 16) {
#pragma unroll
    for (int j = 0; j < NQ; ++j) {
      const u32x4 qr = *reinterpret_cast<const u32x4*>((const char*)a.q + qrow(j) * ROWB + (uint32_t)lir * 16u);
      qv[j] = Elt::make_q(qr, a.scale_log2e);
    }
  }
  const float post = Elt::kPostScale ? a.scale_log2e : 1.f;
  // Sixteen-query pass.  Lane (qi, c4) = (lane % 16, lane / 16).  One 16x16x16 MFMA contracts over 16 values k,
  // lane (i, c) supplying k = 4c .. 4c+3 of row i of A and of column i of B, and leaves C[4c + t][i] in lane (i, c).
  //  * scores: A = K tile (16 rows), B = Q^T, contraction over the head dimension, 8 MFMAs.  Any fixed assignment
  //    of the 128 dimensions to (MFMA, c, t) serves as long as K and q use the same: lane (i, c) holds bytes
  //    16 (4 mm + c) .. + 16 of its row, mm = 0..3, and each 16-byte piece feeds two MFMAs.  Lane (qi, c4) ends up
  //    with the scores of query qi against rows 4 c4 + t of the tile -
  //  * outputs: - which is the B operand (P^T) of O^T = V^T P^T, contraction over the tile's rows.  For A = V^T lane
  //    (i, c) needs V[4c + t][d_i]: it loads the 16-byte piece i of rows 4c + t (whole rows per quarter wave) and
  //    MFMA e = 0..7 takes element e of the four pieces, so d_i = 8 i + e and lane (qi, c4) accumulates
  //    O[qi][32 c4 + 8 t + e].  The rescaling factor of query qi is then a per-lane scalar.
  // q is the same for the four waves and stays in LDS (16 registers fewer per lane): thread tid fetches piece
  // tid % 16 of query row tid / 16 here and parks it once the span metadata is on its way.
  const int qi = lane & 15, c4 = lane >> 4;
  u32x4 q_piece = {0u, 0u, 0u, 0u};
  if constexpr (NQ == 16)
    q_piece = *reinterpret_cast<const u32x4*>((const char*)a.q + qrow(tid >> 4) * ROWB + 16u * (uint32_t)(tid & 15));
  // Causal limit (few-query variant): query token j sees no position after its own, q_pos[b] + q_first + j.
  int lim[NQ];
#pragma unroll
  for (int j = 0; j < NQ; ++j)  // (clamped: any q_pos at or beyond the cache length means "no limit", without overflow)
    lim[j] = a.q_pos ? min(a.q_pos[b], kMaxLen) + a.q_first + j : 0x7fffffff;

  // ---- step 1: how many attended positions does the sequence have, which are mine ----------------
  // with fixed-size slices the count may stop at the slice's end; even slices need the sequence's total
  const int scan_stop = a.even ? 0x7fffffff : (split + 1) * a.slice_tokens;
  int n_total;
  int n_int = 0, off0 = 0;
  int st0 = 0, len0 = 0, incl0 = 0;  // first chunk of 64 intervals, kept in registers
  if constexpr (Args::kHasRuns) {
    n_total = 0;  // the slice's rows come from the arguments, see below
  } else if (kDense) {
    n_total = clampi(a.ctx_lens[b], 0, a.max_len);
  } else {
    off0 = clampi(a.offsets[b], 0, a.num_intervals);
    const int off1 = clampi(a.offsets[b + 1], off0, a.num_intervals);
    off0 = __builtin_amdgcn_readfirstlane(off0);
    n_int = __builtin_amdgcn_readfirstlane(off1 - off0);
    SPAN_STAMP_AFTER(10, "s", n_int);
    if (lane < n_int) {
      st0 = a.starts[off0 + lane];
      len0 = clampi(a.ends[off0 + lane] - st0, 0, a.max_len);
    }
    incl0 = wave_inclusive_scan(len0, lane);
    n_total = __builtin_amdgcn_readlane(incl0, 63);
    for (int c0 = 64; c0 < n_int && n_total < scan_stop; c0 += 64) {
      int len = 0;
      if (c0 + lane < n_int) len = clampi(a.ends[off0 + c0 + lane] - a.starts[off0 + c0 + lane], 0, a.max_len);
      n_total += __builtin_amdgcn_readlane(wave_inclusive_scan(len, lane), 63);
    }
  }
  n_total = n_total < a.max_tokens ? n_total : a.max_tokens;
  int slice_begin, cnt;
  if constexpr (Args::kHasRuns) {  // rows are numbered within the slice
    slice_begin = 0;
    cnt = clampi(a.r.slices[blockIdx.y].rows, 0, kMaxRunSliceRows);
  } else {
    const int T = a.even ? (n_total + nsl - 1) / nsl : a.slice_tokens;
    slice_begin = split * T;
    cnt = __builtin_amdgcn_readfirstlane(clampi(n_total - slice_begin, 0, T));
  }
  SPAN_STAMP_AFTER(1, "s", cnt);

  // State of this slice once its waves are merged, un-normalised, m in log2 units: a thread that `owns` holds
  // output column t of query tokens jb .. jb + JT - 1.  Up to four tokens: all of them, in the first D threads;
  // sixteen: eight per thread, the two halves of the workgroup taking eight tokens each.
  constexpr int JT = NQ == 16 ? 8 : NQ;
  const int t = tid % D;
  const int jb = NQ == 16 ? (tid / D) * JT : 0;
  const bool owns = NQ == 16 ? true : tid < D;
  static_assert(NQ < 16 || kThreads == 2 * D, "sixteen tokens: two halves of D threads");
  float M[JT], L[JT], o[JT];
#pragma unroll
  for (int j = 0; j < JT; ++j) {
    M[j] = -INFINITY;
    L[j] = 0.f;
    o[j] = 0.f;
  }
  // Append variant: the first slice's workgroup writes the new row into the cache, whatever the span holds.
  if (NQ == 1 && a.append_pos && split == 0 && wave == 0 && lane < LPR && new_pos >= 0 && new_pos < a.max_len) {
    const size_t row = (bh * (size_t)a.max_len + (size_t)new_pos) * ROWB + (uint32_t)lir * 16u;
    *reinterpret_cast<u32x4*>((char*)a.k + row) = kn_raw;
    *reinterpret_cast<u32x4*>((char*)a.v + row) = vn_raw;
  }
  if constexpr (NQ > 1) {  // the rows of this pass's tokens, one token per wave
    if (append_many && split == 0 && lane < LPR) {
      for (int i = wave; i < nq_here; i += kWavesPerBlock) {
        const int pos_i = min(a.append_pos[b], kMaxLen) + a.q_first + i;
        if (pos_i >= 0 && pos_i < a.max_len) {
          const size_t src = qrow(i) * ROWB + (uint32_t)lir * 16u;
          const size_t row = (bh * (size_t)a.max_len + (size_t)pos_i) * ROWB + (uint32_t)lir * 16u;
          *reinterpret_cast<u32x4*>((char*)a.k + row) = *reinterpret_cast<const u32x4*>((const char*)a.k_new + src);
          *reinterpret_cast<u32x4*>((char*)a.v + row) = *reinterpret_cast<const u32x4*>((const char*)a.v_new + src);
        }
      }
    }
  }
  if (cnt > 0) {  // same decision in all 4 waves
  // How the slice's rows are dealt to the 4 waves.  My rows are numbered r = 0..nrows-1; row r is
  // virtual token vrow(r) of the sequence.
  //  * small slices: contiguous quarters (RPL-aligned), four short sequential streams;
  //  * large slices (a.interleave): units of RPL rows (one load instruction, 1 KiB) dealt round-robin,
  //    wave w owns units w, w+4, ...  The workgroup then reads one window that moves through the slice.
  //    Quarters of a large slice are a multiple of the memory-channel interleave apart, so the four
  //    streams (and those of the neighbouring heads, a power-of-two slab stride away) pile onto the same
  //    channels: measured 6.1 -> 6.8 TB/s on batch 64 x 1024 cached tokens when dealing round-robin,
  //    while slices of 100-170 rows are 2-4 % faster with quarters.
  int nrows, q_first = 0;
  if (a.interleave) {
    const int units_all = (cnt + RPL - 1) / RPL;
    const int units = units_all > wave ? (units_all - wave + kWavesPerBlock - 1) / kWavesPerBlock : 0;
    const bool own_last = units > 0 && (wave + (units - 1) * kWavesPerBlock) == units_all - 1;
    nrows = units * RPL - (own_last ? units_all * RPL - cnt : 0);
  } else {
    const int rpw = (((cnt + kWavesPerBlock - 1) / kWavesPerBlock) + RPL - 1) / RPL * RPL;
    q_first = min(wave * rpw, cnt);
    nrows = min(q_first + rpw, cnt) - q_first;
  }
  auto vrow = [&](int r) {
    return slice_begin + (a.interleave ? ((r / RPL) * kWavesPerBlock + wave) * RPL + (r % RPL) : q_first + r);
  };

  // ---- steps 2 and 3, one window of kWin rows at a time -----------------------------------------
  const uint32_t slab_bytes = (uint32_t)a.max_len * ROWB;
  const __amdgpu_buffer_rsrc_t kslab = slab_resource((const char*)a.k + bh * (size_t)slab_bytes, slab_bytes);
  const __amdgpu_buffer_rsrc_t vslab = slab_resource((const char*)a.v + bh * (size_t)slab_bytes, slab_bytes);
  const uint32_t lane_off = (uint32_t)lir * 16u;

  float m[kVq], l[kVq];
  float acc[kVq][EPL];
#pragma unroll
  for (int j = 0; j < kVq; ++j) {
    m[j] = -INFINITY;
    l[j] = 0.f;
#pragma unroll
    for (int i = 0; i < EPL; ++i) acc[j][i] = 0.f;
  }
  // Sixteen-query pass: state of query qi in lane (qi, c4).  ref is the reference exponent of the weights (the
  // running maximum minus 8, the same in the four lanes of a query), lsum this lane's share of their sum,
  // O[e][t] the un-normalised output column 32 c4 + 8 t + e.
  float ref = -INFINITY, lsum = 0.f;
  f32x4 O[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) O[e] = f32x4{0.f, 0.f, 0.f, 0.f};
  // Takes one tile of 16 rows into the state.  kr: this lane's four 16-byte pieces of K row qi of the tile; vr:
  // piece qi of V rows 4 c4 + t; vis[t]: query qi sees row 4 c4 + t (hidden pairs get weight zero, whatever K holds).
  // per_query (wave-uniform) with row_pos[t], the cache position of row 4 c4 + t: see the second product below.
  auto absorb = [&](const u32x4* kr, const u32x4* vr, const bool* vis, bool per_query, const int* row_pos) {
    if constexpr (NQ == 16) {
      f32x4 sc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int mm = 0; mm < 4; ++mm) {
        const u32x4 qm = *reinterpret_cast<const u32x4*>(&s_q[qi * kQRow + 16 * (4 * mm + c4)]);
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
          const uint32_t k0 = kr[mm][2 * hh], k1 = kr[mm][2 * hh + 1], q0 = qm[2 * hh], q1 = qm[2 * hh + 1];
          sc = Elt::mfma(u32x2{k0, k1}, u32x2{q0, q1}, sc);
        }
      }
      float w[4];
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const float d = sc[t];
        w[t] = vis[t] ? d * post : -INFINITY;
      }
      float mx = fmaxf(fmaxf(w[0], w[1]), fmaxf(w[2], w[3]));
      mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      // The weights go into the second product in the storage type, as a rounded value plus the rounded remainder.
      // With the reference 8 below the maximum they reach 2^8, which keeps the tail of a peaked distribution
      // (weights below 2^-14 of the largest) out of fp16's subnormal range.
      const float ref_new = fmaxf(ref, mx - 8.f);
      const float ref_safe = (ref_new == -INFINITY) ? 0.f : ref_new;
      const float alpha = __builtin_amdgcn_exp2f(ref - ref_safe);
#pragma unroll
      for (int t = 0; t < 4; ++t) w[t] = __builtin_amdgcn_exp2f(w[t] - ref_safe);
      lsum = fmaf(lsum, alpha, (w[0] + w[1]) + (w[2] + w[3]));
      ref = ref_new;
      if (__builtin_amdgcn_ballot_w64(alpha != 1.f) != 0) {  // (the maximum settles after the first tiles)
#pragma unroll
        for (int e = 0; e < 8; ++e) O[e] *= alpha;
      }
      u32x2 hi, lo;
      Elt::split(w, hi, lo);
      // element e of the four V pieces, as the 16-bit quadruple (rows 4 c4 .. 4 c4 + 3) the MFMA wants
      auto v_operand = [&](int e) {
        const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;
        const uint32_t v0 = vr[0][e >> 1], v1 = vr[1][e >> 1], v2 = vr[2][e >> 1], v3 = vr[3][e >> 1];
        return u32x2{__builtin_amdgcn_perm(v1, v0, sel), __builtin_amdgcn_perm(v3, v2, sel)};
      };
      if (!per_query) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const u32x2 va = v_operand(e);
          O[e] = Elt::mfma(va, hi, O[e]);
          O[e] = Elt::mfma(va, lo, O[e]);
        }
      } else {
        // Some V row of the tile is not finite and some query of the pass does not see it: weight zero would not
        // keep it out of that query's sums (0 * Inf), so the product is taken once per query, with the rows that
        // query does not see cleared from the V operand, and only that query's column of the result is kept.
#pragma unroll 1
        for (int qq = 0; qq < 16; ++qq) {
          const int last = lim[0] + qq;  // (this branch is only taken under a causal limit: no overflow)
          const uint32_t keep0 = (row_pos[0] <= last ? 0xffffu : 0u) | (row_pos[1] <= last ? 0xffff0000u : 0u);
          const uint32_t keep1 = (row_pos[2] <= last ? 0xffffu : 0u) | (row_pos[3] <= last ? 0xffff0000u : 0u);
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            u32x2 va = v_operand(e);
            va = u32x2{va[0] & keep0, va[1] & keep1};
            f32x4 part = Elt::mfma(va, hi, f32x4{0.f, 0.f, 0.f, 0.f});
            part = Elt::mfma(va, lo, part);
            if (qi == qq) O[e] += part;
          }
        }
      }
    }
  };

  if (NQ == 1 && a.append_pos && lane < LPR) {  // park the new row in LDS (frees the registers)
    s_new[wave][0][lane] = kn_raw;
    s_new[wave][1][lane] = vn_raw;
  }
  if constexpr (NQ == 16) {
    *reinterpret_cast<u32x4*>(&s_q[(tid >> 4) * kQRow + 16 * (tid & 15)]) = q_piece;
    __syncthreads();
  }

  // ---- step 2: virtual token -> KV position for a window's rows (span path only) -----------------
  // kFirst: the first 64 intervals are still in registers from step 1; later windows (slices of more
  // than kWin rows per wave) re-read them, so that nothing from step 1 stays live across the streaming loop.
  auto tabulate = [&](auto first_tag, int w0, int wn) {
    constexpr bool kFirst = decltype(first_tag)::value;
    const int vbeg = vrow(w0), vend = vrow(w0 + wn - 1) + 1;
    int carry = 0;
    for (int c0 = 0; c0 < n_int; c0 += 64) {
      int st = 0, len = 0, incl = 0;
      if (kFirst && c0 == 0) {
        st = st0;
        len = len0;
        incl = incl0;
      } else {
        if (c0 + lane < n_int) {
          st = a.starts[off0 + c0 + lane];
          len = clampi(a.ends[off0 + c0 + lane] - st, 0, a.max_len);
        }
        incl = wave_inclusive_scan(len, lane);
      }
      const int chunk_total = __builtin_amdgcn_readlane(incl, 63);
      if (carry + chunk_total > vbeg) {
        // the chunk's exclusive prefixes and starts go to this wave's private LDS rows; the wave
        // reads them back itself (LDS executes a wave's requests in order), so no block barrier
        s_pref[wave][lane] = carry + incl - len;
        s_start[wave][lane] = st;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const int n_here = min(64, n_int - c0);
        for (int r = lane; r < wn; r += 64) {
          const int v = vrow(w0 + r);
          if (v >= carry && v < carry + chunk_total) {
            int idx = 0;  // last interval of the chunk whose exclusive prefix is <= v
#pragma unroll
            for (int step = 32; step > 0; step >>= 1) {
              const int j = idx + step;
              if (j < n_here && s_pref[wave][j] <= v) idx = j;
            }
            const int p = s_start[wave][idx] + (v - s_pref[wave][idx]);
            s_pos[wave][r] = clampi(p, 0, a.max_len - 1);
          }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      }
      carry += chunk_total;
      if (carry >= vend) break;
    }
  };
  if constexpr (Args::kHasRuns) {
    // Run mode: the slice is a short list of runs [start, start + len) in the kernel arguments.  Row number v of
    // the slice lies in the last run whose rows-before count is <= v; a wave has at most kWin rows (the host
    // checked the slice size), four per lane, and walks the runs with scalar loads - no LDS search, and no
    // vector memory access ahead of the first K row.
    const uint32_t ro = a.r.slices[blockIdx.y].runs_of;
    const int run0 = min((int)(ro & 0xffffu), kMaxRuns), nrun = min((int)(ro >> 16), kMaxRuns - run0);
    int v[kWin / 64], p[kWin / 64];
#pragma unroll
    for (int k = 0; k < kWin / 64; ++k) {
      v[k] = vrow(lane + 64 * k);
      p[k] = 0;
    }
    int before = 0;
    constexpr int kRunBatch = 8;  // runs fetched together: their scalar loads are all in flight before the first is used
    for (int j0 = 0; j0 < nrun; j0 += kRunBatch) {
      int st[kRunBatch], ln[kRunBatch];
#pragma unroll
      for (int i = 0; i < kRunBatch; ++i) {
        const int idx = min(run0 + j0 + i, kMaxRuns - 1);
        st[i] = a.r.run[idx][0];
        ln[i] = a.r.run[idx][1];
      }
#pragma unroll
      for (int i = 0; i < kRunBatch; ++i) {
        const bool live = j0 + i < nrun;
#pragma unroll
        for (int k = 0; k < kWin / 64; ++k) p[k] = (live && v[k] >= before) ? st[i] + (v[k] - before) : p[k];
        before += live ? ln[i] : 0;
      }
    }
#pragma unroll
    for (int k = 0; k < kWin / 64; ++k)
      if (lane + 64 * k < nrows) s_pos[wave][lane + 64 * k] = clampi(p[k], 0, a.max_len - 1);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  } else {
    if (!kDense && nrows > 0) tabulate(std::true_type{}, 0, min(kWin, nrows));
  }
  SPAN_STAMP_AFTER(2, "v", lane_off);

  for (int w0 = 0; w0 < nrows; w0 += kWin) {
  const int wn = min(kWin, nrows - w0);  // rows w0 .. w0+wn-1 of mine
  if constexpr (!Args::kHasRuns) {
    if (!kDense && w0 > 0) tabulate(std::false_type{}, w0, wn);
  }

  if (NQ == 1 && a.append_pos) {  // is the appended row one of the window's rows?  Then row group 0 takes it in now.
    bool mine = false;
    for (int r = lane; r < wn; r += 64) mine = mine || (kDense ? vrow(w0 + r) : s_pos[wave][r]) == new_pos;
    if (__builtin_amdgcn_ballot_w64(mine) != 0) {  // wave-uniform
      float vf[EPL];
      Elt::unpack(s_new[wave][1][lir], vf);
      const float d = group_allreduce_sum<LPR>(Elt::dot(s_new[wave][0][lir], qv[0])) * post;
      if (grp == 0) {
        const float l_one = 1.f;
        merge_state(m[0], l[0], acc[0], EPL, d, l_one, vf);
      }
    }
  }

  if constexpr (NQ == 16) {
    // ---- step 3 of the sixteen-query pass ----------------------------------------------------------
    // Every span row that some real token of the pass sees goes through the tiles, masked per (query, row): rows up
    // to `last_all` are seen by all tokens, the few after it (the pass's own positions) by the later tokens only.
    // In the append form those rows are not in the cache yet for this launch: row i of the pass, at position
    // lim[0] + i, is fetched from k_new / v_new instead (a lane takes each of its rows from one source or the other).
    const bool limited = a.q_pos != nullptr;
    const int lim0 = limited ? lim[0] : 0x7fffffff;
    const int last_all = limited ? lim0 - (append_many ? 1 : 0) : 0x7fffffff;
    const int last_any = limited ? lim0 + nq_here - 1 : 0x7fffffff;
    constexpr uint32_t kNoRow = 0xffffff00u;  // an offset past every slab (and still so with a piece offset added)
    const size_t new_first = (((size_t)b * a.q_len + (size_t)a.q_first) * a.heads + h) * ROWB;
    const uint32_t new_stride = (uint32_t)a.heads * ROWB;
    const uint32_t new_bytes = (uint32_t)(nq_here - 1) * new_stride + ROWB;
    const __amdgpu_buffer_rsrc_t knew = append_many ? slab_resource((const char*)a.k_new + new_first, new_bytes) : kslab;
    const __amdgpu_buffer_rsrc_t vnew = append_many ? slab_resource((const char*)a.v_new + new_first, new_bytes) : vslab;
    for (int base = 0; base < wn; base += 16 * U) {
      u32x4 kr[U][4], vr[U][4];
      uint32_t okmask[U];  // bit i: row i of the tile takes part
      bool mixed[U];       // the tile holds rows that only some tokens of the pass see (wave-uniform)
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int live = wn - (base + 16 * u);          // rows of this tile that exist (may be <= 0)
        const int tb = min(base + 16 * u, kWin - 16);   // (a tile past the window reads table entries it does not use)
        const int pk = s_pos[wave][tb + qi];
        const bool okk = qi < live && pk <= last_any;
        okmask[u] = (uint32_t)__builtin_amdgcn_ballot_w64(okk);
        mixed[u] = __builtin_amdgcn_ballot_w64(okk && pk > last_all) != 0;
        if (!(mixed[u] && append_many)) {  // all rows come from the cache: no choice per lane
          const uint32_t koff = okk ? (uint32_t)pk * ROWB + 16u * (uint32_t)c4 : kNoRow;
#pragma unroll
          for (int mm = 0; mm < 4; ++mm) kr[u][mm] = load_row_piece(kslab, koff + 64u * mm);
          const i32x4 pv4 = *reinterpret_cast<const i32x4*>(&s_pos[wave][tb + 4 * c4]);  // positions of rows 4 c4 .. + 3
#pragma unroll
          for (int t = 0; t < 4; ++t) {
            const int pv = pv4[t];
            const bool okv = (okmask[u] >> (4 * c4 + t)) & 1u;
            vr[u][t] = load_row_piece(vslab, okv ? (uint32_t)pv * ROWB + 16u * (uint32_t)qi : kNoRow);
          }
        } else {
          if (okk && pk >= lim0) {
            const uint32_t koff = (uint32_t)(pk - lim0) * new_stride + 16u * (uint32_t)c4;
#pragma unroll
            for (int mm = 0; mm < 4; ++mm) kr[u][mm] = __builtin_amdgcn_raw_buffer_load_b128(knew, koff + 64u * mm, 0, 0);
          } else {
            const uint32_t koff = okk ? (uint32_t)pk * ROWB + 16u * (uint32_t)c4 : kNoRow;
#pragma unroll
            for (int mm = 0; mm < 4; ++mm) kr[u][mm] = load_row_piece(kslab, koff + 64u * mm);
          }
          const i32x4 pv4 = *reinterpret_cast<const i32x4*>(&s_pos[wave][tb + 4 * c4]);
#pragma unroll
          for (int t = 0; t < 4; ++t) {
            const int pv = pv4[t];
            const bool okv = (okmask[u] >> (4 * c4 + t)) & 1u;
            if (okv && pv >= lim0)
              vr[u][t] = __builtin_amdgcn_raw_buffer_load_b128(vnew, (uint32_t)(pv - lim0) * new_stride + 16u * (uint32_t)qi, 0, 0);
            else
              vr[u][t] = load_row_piece(vslab, okv ? (uint32_t)pv * ROWB + 16u * (uint32_t)qi : kNoRow);
          }
        }
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (base + 16 * u < wn) {
          const int tb = min(base + 16 * u, kWin - 16);
          bool vis[4];
          int row_pos[4];
          const i32x4 pv4 = *reinterpret_cast<const i32x4*>(&s_pos[wave][tb + 4 * c4]);
#pragma unroll
          for (int t = 0; t < 4; ++t) {
            const bool okv = (okmask[u] >> (4 * c4 + t)) & 1u;
            const int pv = pv4[t];
            row_pos[t] = okv ? pv : 0x7fffffff;
            vis[t] = okv && row_pos[t] - lim0 <= qi;  // (no limit: lim0 is the largest int and the difference negative)
          }
          bool wild = false;  // a V value that is not finite, in a tile with rows hidden from some tokens
          if (mixed[u]) {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
#pragma unroll
              for (int i = 0; i < 4; ++i) {
                const uint32_t w = vr[u][t][i];
                wild = wild || (w & Elt::kExponent) == Elt::kExponent || (w & (Elt::kExponent << 16)) == (Elt::kExponent << 16);
              }
            }
            wild = __builtin_amdgcn_ballot_w64(wild) != 0;
          }
          absorb(kr[u], vr[u], vis, wild, row_pos);
        }
      }
#ifdef SPAN_PHASE_TRACE
      if (w0 == 0 && base == 0) SPAN_STAMP_AFTER(3, "v", lsum);
#endif
      // Compiler barrier: without it the scheduler moves work of the next iteration (and of the merge phase) up into
      // this one, the 128 registers of four waves per SIMD no longer suffice, and the spill reloads land in this loop.
      asm volatile("" ::"v"(lsum) : "memory");
    }
  } else {
  // Passes of two or four tokens: the span rows between the first and the last token's causal limit (at most NQ - 1
  // positions of a sequence) are seen by the later tokens only.  The streaming loop below serves the rows every
  // token of the pass sees; these few are taken in here, one at a time, each into the states of exactly the
  // tokens that see it - a hidden row never meets a token's sums, not even with weight zero (0 * Inf).
  // In the append form the pass's own tokens sit at exactly these positions and at the first token's own: their
  // rows are not in the cache yet for this launch and come from k_new / v_new instead.
  if constexpr (NQ > 1) {
    if (a.q_pos) {
      const int first_here = lim[0] + (append_many ? 0 : 1);  // first position the streaming loop leaves out
      for (int r0 = 0; r0 < wn; r0 += 64) {
        const int p = r0 + lane < wn ? s_pos[wave][r0 + lane] : -1;
        uint64_t todo = __builtin_amdgcn_ballot_w64(p >= first_here && p <= lim[NQ - 1]);
        while (todo != 0) {  // wave-uniform
          const int pb = __builtin_amdgcn_readlane(p, __builtin_ctzll(todo));
          todo &= todo - 1;
          u32x4 kb, vb;  // every row group fetches the same row
          if (append_many) {
            const int i = pb - lim[0];     // the token that brought this row
            if (i >= nq_here) continue;    // (a padded pass: no such token, and no token that could see it)
            const size_t src = qrow(i) * ROWB + lane_off;
            kb = *reinterpret_cast<const u32x4*>((const char*)a.k_new + src);
            vb = *reinterpret_cast<const u32x4*>((const char*)a.v_new + src);
          } else {
            const uint32_t off = (uint32_t)pb * ROWB + lane_off;
            kb = load_row_piece(kslab, off);
            vb = load_row_piece(vslab, off);
          }
          float vf[EPL];
          Elt::unpack(vb, vf);
#pragma unroll
          for (int j = 0; j < NQ; ++j) {
            const float d = group_allreduce_sum<LPR>(Elt::dot(kb, qv[j])) * post;
            if (pb <= lim[j] && grp == 0) {
              const float l_one = 1.f;
              merge_state(m[j], l[j], acc[j], EPL, d, l_one, vf);
            }
          }
        }
      }
    }
  }

  // ---- step 3: stream the window's K and V rows, online softmax per row group -------------------
  for (int base = 0; base < wn; base += RPL * U) {
    if constexpr (kBoost) {  // (wave-uniform: set at the first batch, reset at the second)
      if (w0 + base <= RPL * U) first_batch_priority(w0 + base == 0);
    }
    u32x4 kr[U], vr[U];
    bool ok[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int r = base + u * RPL + grp;
      const int p = kDense ? vrow(w0 + min(r, wn - 1)) : s_pos[wave][min(r, wn - 1)];
      // Rows that take no part are not fetched at all: a row group past the window's end, the appended row
      // (not in the cache yet for this launch; its owner added it above), and span rows after the causal
      // limit of the first query token of the pass (masked positions have no influence, whatever the cache
      // holds there: Sec. 2.2, mask paragraph; the few rows that only later tokens of the pass see were
      // taken in above).  They request an offset past the slab instead, for which the buffer hardware
      // returns zeros, and get no weight.
      ok[u] = r < wn && p != new_pos && p <= lim[0] && !(append_many && p == lim[0]);
      const uint32_t off = ok[u] ? (uint32_t)p * ROWB + lane_off : 0xfffffff0u;
#ifdef SPAN_STAGE_LDS
      // measurement build: the same rows staged through LDS (direct-to-LDS loads, lane i's 16 bytes land in slot i)
#if defined(__HIP_DEVICE_COMPILE__)  // (the host pass has no LDS address space to type-check the builtin against)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(kslab, &s_stage[wave][0][u][0], 16, off, 0, 0, kRowLoadPolicy);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(vslab, &s_stage[wave][1][u][0], 16, off, 0, 0, kRowLoadPolicy);
#endif
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the tiles are in LDS
#pragma unroll
    for (int u = 0; u < U; ++u) {
      kr[u] = s_stage[wave][0][u][lane];
      vr[u] = s_stage[wave][1][u][lane];
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // read out before the next iteration's loads overwrite them
    {
#else
      kr[u] = load_row_piece(kslab, off);
      vr[u] = load_row_piece(vslab, off);
#endif
    }
    float w[NQ][U];  // scores first, then softmax weights
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int j = 0; j < NQ; ++j) {
        const float d = group_allreduce_sum<LPR>(Elt::dot(kr[u], qv[j])) * post;
        w[j][u] = ok[u] ? d : -INFINITY;
      }
    }
#pragma unroll
    for (int j = 0; j < NQ; ++j) {
      float mx = -INFINITY;
#pragma unroll
      for (int u = 0; u < U; ++u) mx = fmaxf(mx, w[j][u]);
      const float m_new = fmaxf(m[j], mx);
      const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
      const float alpha = __builtin_amdgcn_exp2f(m[j] - m_safe);
      l[j] *= alpha;
#pragma unroll
      for (int i = 0; i < EPL; ++i) acc[j][i] *= alpha;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        w[j][u] = __builtin_amdgcn_exp2f(w[j][u] - m_safe);
        l[j] += w[j][u];
      }
      m[j] = m_new;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float vf[EPL];
      Elt::unpack(vr[u], vf);
#pragma unroll
      for (int j = 0; j < NQ; ++j) {
#pragma unroll
        for (int i = 0; i < EPL; ++i) acc[j][i] = fmaf(w[j][u], vf[i], acc[j][i]);
      }
    }
#ifdef SPAN_PHASE_TRACE
    if (w0 == 0 && base == 0) SPAN_STAMP_AFTER(3, "v", acc[0][0]);
#endif
  }
  }  // fewer than sixteen queries
  }  // windows
  SPAN_STAMP_AFTER(4, "v", acc[0][0] + lsum);

  // ---- step 4: merge row groups (shuffles), then waves (LDS) ------------------------------------
  if constexpr (NQ == 16) {
    // the four lanes of a query hold the weights of disjoint rows and disjoint output columns
    lsum += __shfl_xor(lsum, 16, 64);
    lsum += __shfl_xor(lsum, 32, 64);
    __syncthreads();  // every wave is done with the streaming tables: the states may overwrite them
#pragma unroll
    for (int tt = 0; tt < 4; ++tt) {
      float* dst = &s_acc[wave][qi][32 * c4 + 8 * tt];
      *reinterpret_cast<f32x4*>(dst) = f32x4{O[0][tt], O[1][tt], O[2][tt], O[3][tt]};
      *reinterpret_cast<f32x4*>(dst + 4) = f32x4{O[4][tt], O[5][tt], O[6][tt], O[7][tt]};
    }
    if (c4 == 0) {
      s_ml[wave][qi][0] = ref;
      s_ml[wave][qi][1] = lsum;
    }
    __syncthreads();
    // the weight of wave w's state in query j's merged state is the same for all columns: 64 threads work them out
    if (tid < 64) {
      const int w = tid >> 4, j = tid & 15;
      const float mw = s_ml[w][j][0], lw = s_ml[w][j][1];
      float mx = lw > 0.f ? mw : -INFINITY;
      mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float wgt = lw > 0.f ? __builtin_amdgcn_exp2f(mw - mx) : 0.f;
      float lj = wgt * lw;
      lj += __shfl_xor(lj, 16, 64);
      lj += __shfl_xor(lj, 32, 64);
      s_wgt[w][j] = wgt;
      if (w == 0) {
        s_M[j] = mx;
        s_L[j] = lj;
      }
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < JT; ++j) {
      M[j] = s_M[jb + j];
      L[j] = s_L[jb + j];
#pragma unroll
      for (int w = 0; w < kWavesPerBlock; ++w) o[j] = fmaf(s_wgt[w][jb + j], s_acc[w][jb + j][t], o[j]);
    }
  } else {
#pragma unroll
  for (int j = 0; j < NQ; ++j) {
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1) {
      const float m2 = __shfl_xor(m[j], off, 64), l2 = __shfl_xor(l[j], off, 64);
      float acc2[EPL];
#pragma unroll
      for (int i = 0; i < EPL; ++i) acc2[i] = __shfl_xor(acc[j][i], off, 64);
      merge_state(m[j], l[j], acc[j], EPL, m2, l2, acc2);
    }
    if (lane < LPR) {
#pragma unroll
      for (int i = 0; i < EPL; ++i) s_acc[wave][j][lir * EPL + i] = acc[j][i];
      if (lane == 0) {
        s_ml[wave][j][0] = m[j];
        s_ml[wave][j][1] = l[j];
      }
    }
  }
  __syncthreads();
  if (tid < D) {
#pragma unroll
    for (int j = 0; j < NQ; ++j) {
#pragma unroll
      for (int w = 0; w < kWavesPerBlock; ++w)
        if (s_ml[w][j][1] > 0.f) M[j] = fmaxf(M[j], s_ml[w][j][0]);
#pragma unroll
      for (int w = 0; w < kWavesPerBlock; ++w) {
        const float wgt = s_ml[w][j][1] > 0.f ? __builtin_amdgcn_exp2f(s_ml[w][j][0] - M[j]) : 0.f;
        L[j] = fmaf(wgt, s_ml[w][j][1], L[j]);
        o[j] = fmaf(wgt, s_acc[w][j][tid], o[j]);
      }
    }
  }
  }  // up to four tokens
  }  // cnt > 0
  SPAN_STAMP_AFTER(5, "v", o[0]);

  // Output column t of an un-normalised state.  (The sixteen-token pass multiplies by the reciprocal of the
  // sum, one division per token instead of one per element.)
  auto store_rows = [&](const float* ll, const float* oo) {
#pragma unroll
    for (int j = 0; j < JT; ++j) {
      if (jb + j < nq_here) {
        float r;
        if constexpr (NQ == 16) r = ll[j] > 0.f ? oo[j] * (1.f / ll[j]) : 0.f;
        else r = ll[j] > 0.f ? oo[j] / ll[j] : 0.f;
        a.out[qrow(jb + j) * D + t] = r;
      }
    }
  };

  if (nsl == 1) {  // one slice for this (batch, head): this workgroup owns the output row
    if (owns) store_rows(L, o);
    SPAN_STAMP_ACKED(6);
    SPAN_TRACE_FLUSH();
    return;
  }

  // ---- step 5: several slices.  Publish this slice's state; the workgroup that arrives last for
  // (b, h) merges all of them by log-sum-exp and writes the output row (no second kernel launch).
  //
  // Cross-workgroup hand-over without cache-wide fences: the states are written and read with
  // device-scope relaxed atomics (write-through / cache-bypassing accesses, each coherent on its own),
  // the writer waits for its stores to be acknowledged before the ticket is taken, and the reader
  // only starts after its own ticket came back.  A device-scope fence would write back and
  // invalidate the whole L2 of the XCD for every workgroup, which costs far more than the merge.
  // state of slice s of (b, h) lives in slot (y0 + s) * heads + h
  const size_t H = (size_t)a.heads;
  const size_t my_slot = (size_t)(y0 + split) * H + h;
  if (owns) {
#pragma unroll
    for (int j = 0; j < JT; ++j) {
      if (jb + j >= nq_here) continue;  // (a padded pass: tokens that do not exist leave no state)
      if (cnt > 0) publish(&a.part_acc[(my_slot * NQ + jb + j) * D + t], o[j]);
      if (t == 0) {
        publish(&a.part_ml[(my_slot * NQ + jb + j) * 2], M[j]);
        publish(&a.part_ml[(my_slot * NQ + jb + j) * 2 + 1], L[j]);
      }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // my published stores are acknowledged
  }
  __syncthreads();
  SPAN_STAMP_AFTER(7, "s", 0);
  if (tid == 0) s_ticket = __hip_atomic_fetch_add(&a.counters[bh], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __syncthreads();
  SPAN_STAMP_AFTER(8, "v", s_ticket);
  if (s_ticket != nsl - 1) {
    SPAN_TRACE_FLUSH();
    return;
  }

  // Column t of tokens jb .. is merged by G threads, each over every G-th slice (sixteen tokens: G = 1, the two
  // halves of the workgroup already split the tokens).
  constexpr int G = kSliceGroups;
  const int g = NQ == 16 ? 0 : tid / D;
  const size_t slot0 = (size_t)y0 * H + h;  // slice s of this (b, h) is slot0 + s * H
  float mm[JT], ll[JT], oo[JT];
#pragma unroll
  for (int j = 0; j < JT; ++j) {
    mm[j] = -INFINITY;
    ll[j] = 0.f;
    oo[j] = 0.f;
  }
  // The states are fetched a batch at a time, all loads of a batch in flight together (one trip to memory for up
  // to kBatch * G slices), and merged in slice order.
  constexpr int kBatch = NQ == 1 ? 8 : (NQ == 2 ? 4 : (NQ == 4 ? 2 : 1));
  for (int s0 = g; s0 < nsl; s0 += G * kBatch) {
    float ms[kBatch][JT], ls[kBatch][JT], as[kBatch][JT];
#pragma unroll
    for (int k = 0; k < kBatch; ++k) {
      const size_t slot = slot0 + (size_t)min(s0 + k * G, nsl - 1) * H;  // (past the end: a slot that exists, unused)
#pragma unroll
      for (int j = 0; j < JT; ++j) {
        if (jb + j < nq_here) {
          ms[k][j] = observe(&a.part_ml[(slot * NQ + jb + j) * 2]);
          ls[k][j] = observe(&a.part_ml[(slot * NQ + jb + j) * 2 + 1]);
          as[k][j] = observe(&a.part_acc[(slot * NQ + jb + j) * D + t]);
        } else {
          ms[k][j] = -INFINITY;
          ls[k][j] = as[k][j] = 0.f;
        }
      }
    }
#pragma unroll
    for (int k = 0; k < kBatch; ++k) {
      if (s0 + k * G < nsl) {
#pragma unroll
        for (int j = 0; j < JT; ++j) {
          const bool full = ls[k][j] > 0.f;  // slot of an empty slice is never written: select, do not scale
          const float av = full ? as[k][j] : 0.f;
          merge_state(mm[j], ll[j], &oo[j], 1, full ? ms[k][j] : -INFINITY, full ? ls[k][j] : 0.f, &av);
        }
      }
    }
  }
  if constexpr (G > 1) {
    if (g > 0) {
#pragma unroll
      for (int j = 0; j < JT; ++j) {
        s_acc[g][j][t] = oo[j];
        if (t == 0) {
          s_gm[g][j] = mm[j];
          s_gl[g][j] = ll[j];
        }
      }
    }
    __syncthreads();
  }
  if (g == 0) {
    if constexpr (G > 1) {
#pragma unroll
      for (int j = 0; j < JT; ++j) {
#pragma unroll
        for (int k = 1; k < G; ++k) {
          const float o2 = s_acc[k][j][t];
          merge_state(mm[j], ll[j], &oo[j], 1, s_gm[k][j], s_gl[k][j], &o2);
        }
      }
    }
    store_rows(ll, oo);
    // leave the ticket counter ready for the next call (same device-coherent access path as the tickets)
    if (tid == 0) __hip_atomic_store(&a.counters[bh], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  SPAN_STAMP_ACKED(9);
  SPAN_TRACE_FLUSH();
}

// Zeroes n 32-bit words (a plain kernel, so that the call can also be recorded into a HIP graph).
__global__ __launch_bounds__(256) void zero_words_kernel(uint32_t* p, size_t n) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0u;
}

// One thread per sequence: the span gains the positions after the ones just appended (see span_advance).
__global__ __launch_bounds__(256) void advance_kernel(int batch, int max_len, int num_intervals, int count,
                                                      const int32_t* offsets, const int32_t* starts, int32_t* ends,
                                                      int32_t* append_pos, int32_t* ctx_lens) {
  const int b = blockIdx.x * 256 + threadIdx.x;
  if (b >= batch) return;
  const int p = append_pos[b];
  if (p < 0 || (long long)p + 2 * (long long)count > (long long)max_len) return;
  const int next = p + count;  // first position of the next step's tokens; they take next .. next + count - 1
  const int lo = clampi(offsets[b], 0, num_intervals), hi = clampi(offsets[b + 1], lo, num_intervals);
  int grow = -1;        // interval that ends right after the appended tokens
  bool taken = false;   // some of the next positions are already inside an interval
  for (int i = lo; i < hi; ++i) {
    const int st = starts[i], en = ends[i];
    if (st < en && en == next) grow = i;
    if (st < en && st < next + count && next < en) taken = true;
  }
  if (grow >= 0 && !taken) ends[grow] = next + count;
  append_pos[b] = next;
  if (ctx_lens) ctx_lens[b] += count;
}

thread_local int g_last_hip_error = 0;
#ifdef SPAN_PHASE_TRACE
unsigned long long* g_trace = nullptr;  // set by span_debug_set_trace
size_t g_trace_workgroups = 0;
#endif

// ---- scratch owned by the library, for span_decode_attn_static ---------------------------------------
// One array per GPU the library runs on, resident until the process ends.  `scratch` is only a host-side
// handle here: host code never passes it to a kernel or a copy, it asks the runtime once per device where
// that device's copy lives and uses that address from then on.
static __device__ __align__(256) unsigned char scratch[SPAN_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each device, null until first asked

// Address of the current device's scratch array; resolves it on the first call for that device.
int static_scratch(void** ptr) {
  int dev = -1;
  hipError_t err = hipGetDevice(&dev);
  if (err == hipSuccess && (dev < 0 || dev >= kMaxDevices)) err = hipErrorInvalidDevice;
  if (err == hipSuccess) {
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
      void* p = nullptr;
      err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
      if (err == hipSuccess && (!p || ((uintptr_t)p & 255u))) err = hipErrorInvalidSymbol;
      if (err == hipSuccess) g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
  }
  if (err != hipSuccess) {
    g_last_hip_error = (int)err;
    return SPAN_ERR_HIP;
  }
  return SPAN_OK;
}

// How the grid names its slices.
enum class GridMode { kPlain, kTable, kRuns };

template <class Elt, int D, bool kDense, int NQ>
int launch_typed(const LaunchArgsTable& a, const RunTables* runs, GridMode mode, int batch, hipStream_t stream) {
  // K loads (and as many V loads) a wave has in flight before it consumes the first: 4 KiB + 4 KiB, but
  // never more than 16 rows (with 128-byte rows that is 2 instructions of 8 rows); half of that when
  // several query tokens share the registers
  constexpr int kRowsPerLoad = 64 / (D / Elt::kPerVec);
#ifdef SPAN_IN_FLIGHT
  constexpr int kInFlight = SPAN_IN_FLIGHT;
#else
  constexpr int kInFlight = NQ == 16 ? SPAN_MQ_TILES /* tiles of 16 rows */ : (kRowsPerLoad >= 8 ? 2 : 4) / (NQ > 1 ? 2 : 1);
#endif
  // short slices of 16-bit rows, one token: the instances that send a wave's first batch at raised priority
  constexpr bool kCanBoost = NQ == 1 && Elt::kBytes == 2 && D == 128 && SPAN_FIRST_BATCH_PRIORITY > 0;
  const bool boost = kCanBoost && a.slice_tokens <= kBoostUpToBatches * kWavesPerBlock * kRowsPerLoad * kInFlight;
  if (mode == GridMode::kRuns) {
    if constexpr (!kDense) {
      const dim3 grid((unsigned)a.heads, (unsigned)a.total_slices, 1u);
      LaunchArgsRuns ra;
      static_cast<LaunchArgs&>(ra) = static_cast<const LaunchArgs&>(a);
      ra.r = *runs;
      if (boost) hipLaunchKernelGGL((decode_kernel<Elt, D, false, kInFlight, NQ, LaunchArgsRuns, kCanBoost>), grid, dim3(kThreads), 0, stream, ra);
      else hipLaunchKernelGGL((decode_kernel<Elt, D, false, kInFlight, NQ, LaunchArgsRuns>), grid, dim3(kThreads), 0, stream, ra);
    } else {
      return SPAN_ERR_SHAPE;  // (not reachable: the dense form never plans runs)
    }
  } else if (mode == GridMode::kTable) {
    const dim3 grid((unsigned)a.heads, (unsigned)a.total_slices, 1u);
    if (boost) hipLaunchKernelGGL((decode_kernel<Elt, D, kDense, kInFlight, NQ, LaunchArgsTable, kCanBoost>), grid, dim3(kThreads), 0, stream, a);
    else hipLaunchKernelGGL((decode_kernel<Elt, D, kDense, kInFlight, NQ, LaunchArgsTable>), grid, dim3(kThreads), 0, stream, a);
  } else {
    const dim3 grid((unsigned)a.heads, (unsigned)a.num_splits, (unsigned)batch);
    LaunchArgsPlain plain;
    static_cast<LaunchArgs&>(plain) = static_cast<const LaunchArgs&>(a);
    if (boost) hipLaunchKernelGGL((decode_kernel<Elt, D, kDense, kInFlight, NQ, LaunchArgsPlain, kCanBoost>), grid, dim3(kThreads), 0, stream, plain);
    else hipLaunchKernelGGL((decode_kernel<Elt, D, kDense, kInFlight, NQ, LaunchArgsPlain>), grid, dim3(kThreads), 0, stream, plain);
  }
  const hipError_t err = hipGetLastError();
  if (err != hipSuccess) {
    g_last_hip_error = (int)err;
    return SPAN_ERR_HIP;
  }
  return SPAN_OK;
}

template <class Elt, int D, bool kDense>
int launch_queries(const LaunchArgsTable& a, const RunTables* runs, int nq, GridMode mode, int batch,
                   hipStream_t stream) {
  if constexpr (!kDense) {  // the few-query variant exists for the span form only
    if (nq == 2) return launch_typed<Elt, D, false, 2>(a, runs, mode, batch, stream);
    if (nq == 4) return launch_typed<Elt, D, false, 4>(a, runs, mode, batch, stream);
    if constexpr (Elt::kHasMfma && D == 128) {
      if (nq == 16) return launch_typed<Elt, D, false, 16>(a, runs, mode, batch, stream);
    }
    if (nq != 1) return SPAN_ERR_SHAPE;  // (not reachable: the planner asks only for passes that exist)
  }
  return launch_typed<Elt, D, kDense, 1>(a, runs, mode, batch, stream);
}

template <bool kDense>
int launch(const span_attn_desc_t* d, const void* q, const void* k, const void* v, const int32_t* offsets,
           const int32_t* starts, const int32_t* ends, const int32_t* ctx_lens, float scale, float* out,
           const void* k_new = nullptr, const void* v_new = nullptr, const int32_t* append_pos = nullptr,
           const int32_t* q_pos = nullptr, bool few_query = false) {
  const int rc = check_desc(d);
  if (rc != SPAN_OK) return rc;
  if (query_tokens(d) > 1 && !few_query) return SPAN_ERR_SHAPE;  // only span_decode_attn_multi takes several
  if (!q || !k || !v || !out) return SPAN_ERR_NULL;
  if (kDense ? !ctx_lens : (!offsets || (d->num_intervals > 0 && (!starts || !ends)))) return SPAN_ERR_NULL;
  LaunchArgsTable a;
  RunTables runs;
  span_attn_desc_t own;
  if (kDense && (d->host_span_offsets || d->host_span_starts || d->host_span_ends)) {
    own = *d;  // span lists mean nothing to the dense form
    own.host_span_offsets = own.host_span_starts = own.host_span_ends = nullptr;
    d = &own;
  }
  const Partition p = plan_partition(d, a.table, kDense ? nullptr : &runs);
  const GridMode mode = p.runs ? GridMode::kRuns : (p.exact ? GridMode::kTable : GridMode::kPlain);
  const size_t need = workspace_bytes(d, p);
  if (need > 0 && (!d->workspace || ((uintptr_t)d->workspace & 255u) || d->workspace_bytes < need))
    return SPAN_ERR_WORKSPACE;

  a.q = q;
  a.k = k;
  a.v = v;
  a.out = out;
  a.offsets = offsets;
  a.starts = starts;
  a.ends = ends;
  a.ctx_lens = ctx_lens;
  a.k_new = k_new;
  a.v_new = v_new;
  a.append_pos = append_pos;
  a.q_pos = q_pos;
  a.q_len = query_tokens(d);
  a.counters = need ? (int32_t*)d->workspace : nullptr;
  a.part_ml = need ? (float*)((char*)d->workspace + workspace_counter_bytes(d)) : nullptr;
  a.part_acc = need ? (float*)((char*)d->workspace + workspace_counter_bytes(d) + workspace_ml_bytes(d, p)) : nullptr;
  a.heads = d->heads;
  a.max_len = d->max_len;
  a.num_intervals = d->num_intervals;
  a.slice_tokens = p.slice_tokens;
  a.num_splits = p.num_splits;
  a.max_tokens = p.max_tokens;
  a.even = p.even ? 1 : 0;
  a.interleave = p.slice_tokens >= kInterleaveFrom ? 1 : 0;
  a.total_slices = p.total_slices;
  a.scale_log2e = scale * 1.4426950408889634f;
#ifdef SPAN_PHASE_TRACE
  a.trace = g_trace;
  a.trace_workgroups = g_trace_workgroups;
#endif
  hipStream_t stream = (hipStream_t)d->stream;

  // One pass over the span serves up to p.queries_per_pass query tokens; more tokens take more passes,
  // one after the other on the stream (they share the workspace).
  const bool d128 = d->head_dim == 128;
  for (int32_t first = 0; first < a.q_len; first += p.queries_per_pass) {
    a.q_first = first;
    const int nq = p.queries_per_pass;
    int lrc;
    switch (d->dtype) {
      case SPAN_F32:
        lrc = d128 ? launch_queries<F32, 128, kDense>(a, &runs, nq, mode, d->batch, stream)
                   : launch_queries<F32, 64, kDense>(a, &runs, nq, mode, d->batch, stream);
        break;
      case SPAN_F16:
        lrc = d128 ? launch_queries<F16, 128, kDense>(a, &runs, nq, mode, d->batch, stream)
                   : launch_queries<F16, 64, kDense>(a, &runs, nq, mode, d->batch, stream);
        break;
      default:
        lrc = d128 ? launch_queries<BF16, 128, kDense>(a, &runs, nq, mode, d->batch, stream)
                   : launch_queries<BF16, 64, kDense>(a, &runs, nq, mode, d->batch, stream);
        break;
    }
    if (lrc != SPAN_OK) return lrc;
  }
  return SPAN_OK;
}

}  // namespace
}  // namespace spanattn

extern "C" int span_decode_attn(const span_attn_desc_t* desc, const void* q, const void* k_cache,
                                const void* v_cache, const int32_t* span_offsets, const int32_t* span_starts,
                                const int32_t* span_ends, const int32_t* ctx_lens, float scale, float* out) {
  (void)ctx_lens;
  return spanattn::launch<false>(desc, q, k_cache, v_cache, span_offsets, span_starts, span_ends, nullptr, scale, out);
}

extern "C" int span_decode_attn_static(const span_attn_desc_t* desc, const void* q, const void* k_cache,
                                       const void* v_cache, const int32_t* span_offsets, const int32_t* span_starts,
                                       const int32_t* span_ends, const int32_t* ctx_lens, float scale, float* out) {
  (void)ctx_lens;
  const int rc = spanattn::check_desc(desc);
  if (rc != SPAN_OK) return rc;
  span_attn_desc_t d = *desc;
  d.workspace = nullptr;
  d.workspace_bytes = 0;
  const spanattn::Partition p = spanattn::plan_partition(&d);
  const size_t need = spanattn::workspace_bytes(&d, p);
  if (need > SPAN_STATIC_SCRATCH_BYTES) return SPAN_ERR_SCRATCH_LIMIT;
  if (need > 0) {
    void* ptr = nullptr;
    const int src = spanattn::static_scratch(&ptr);
    if (src != SPAN_OK) return src;
    d.workspace = ptr;
    d.workspace_bytes = SPAN_STATIC_SCRATCH_BYTES;
    // the array keeps what the last call (of any shape) left: the tickets of this call's pairs start at zero
    const size_t words = spanattn::workspace_counter_bytes(&d) / sizeof(uint32_t);
    hipLaunchKernelGGL(spanattn::zero_words_kernel, dim3((unsigned)((words + 255) / 256)), dim3(256), 0,
                       (hipStream_t)d.stream, (uint32_t*)ptr, words);
    const hipError_t err = hipGetLastError();
    if (err != hipSuccess) {
      spanattn::g_last_hip_error = (int)err;
      return SPAN_ERR_HIP;
    }
  }
  return spanattn::launch<false>(&d, q, k_cache, v_cache, span_offsets, span_starts, span_ends, nullptr, scale, out);
}

extern "C" int span_decode_attn_multi(const span_attn_desc_t* desc, const void* q, const void* k_cache,
                                      const void* v_cache, const int32_t* span_offsets, const int32_t* span_starts,
                                      const int32_t* span_ends, const int32_t* q_pos, float scale, float* out) {
  return spanattn::launch<false>(desc, q, k_cache, v_cache, span_offsets, span_starts, span_ends, nullptr, scale, out,
                                 nullptr, nullptr, nullptr, q_pos, true);
}

extern "C" int dense_decode_attn(const span_attn_desc_t* desc, const void* q, const void* k_cache,
                                 const void* v_cache, const int32_t* ctx_lens, float scale, float* out) {
  return spanattn::launch<true>(desc, q, k_cache, v_cache, nullptr, nullptr, nullptr, ctx_lens, scale, out);
}

extern "C" int span_decode_attn_append(const span_attn_desc_t* desc, const void* q, const void* k_new, const void* v_new,
                                       void* k_cache, void* v_cache, const int32_t* append_pos,
                                       const int32_t* span_offsets, const int32_t* span_starts,
                                       const int32_t* span_ends, float scale, float* out) {
  if (!k_new || !v_new || !append_pos) return SPAN_ERR_NULL;
  return spanattn::launch<false>(desc, q, k_cache, v_cache, span_offsets, span_starts, span_ends, nullptr, scale, out,
                                 k_new, v_new, append_pos);
}

extern "C" int span_decode_attn_multi_append(const span_attn_desc_t* desc, const void* q, const void* k_new,
                                             const void* v_new, void* k_cache, void* v_cache,
                                             const int32_t* append_pos, const int32_t* span_offsets,
                                             const int32_t* span_starts, const int32_t* span_ends, float scale,
                                             float* out) {
  if (!k_new || !v_new || !append_pos) return SPAN_ERR_NULL;
  return spanattn::launch<false>(desc, q, k_cache, v_cache, span_offsets, span_starts, span_ends, nullptr, scale, out,
                                 k_new, v_new, append_pos, append_pos, true);
}

extern "C" int dense_decode_attn_append(const span_attn_desc_t* desc, const void* q, const void* k_new, const void* v_new,
                                        void* k_cache, void* v_cache, const int32_t* append_pos,
                                        const int32_t* ctx_lens, float scale, float* out) {
  if (!k_new || !v_new || !append_pos) return SPAN_ERR_NULL;
  return spanattn::launch<true>(desc, q, k_cache, v_cache, nullptr, nullptr, nullptr, ctx_lens, scale, out, k_new,
                                v_new, append_pos);
}

extern "C" int span_advance(const span_attn_desc_t* desc, const int32_t* span_offsets, const int32_t* span_starts,
                            int32_t* span_ends, int32_t* append_pos, int32_t* ctx_lens) {
  const int rc = spanattn::check_desc(desc);
  if (rc != SPAN_OK) return rc;
  if (!span_offsets || !append_pos || (desc->num_intervals > 0 && (!span_starts || !span_ends))) return SPAN_ERR_NULL;
  hipLaunchKernelGGL(spanattn::advance_kernel, dim3((unsigned)((desc->batch + 255) / 256)), dim3(256), 0,
                     (hipStream_t)desc->stream, desc->batch, desc->max_len, desc->num_intervals,
                     spanattn::query_tokens(desc), span_offsets, span_starts, span_ends, append_pos, ctx_lens);
  const hipError_t err = hipGetLastError();
  if (err != hipSuccess) {
    spanattn::g_last_hip_error = (int)err;
    return SPAN_ERR_HIP;
  }
  return SPAN_OK;
}

extern "C" int span_workspace_init(const span_attn_desc_t* desc) {
  const int rc = spanattn::check_desc(desc);
  if (rc != SPAN_OK) return rc;
  const spanattn::Partition p = spanattn::plan_partition(desc);
  const size_t need = spanattn::workspace_bytes(desc, p);
  if (need == 0) return SPAN_OK;
  if (!desc->workspace || ((uintptr_t)desc->workspace & 255u) || desc->workspace_bytes < need) return SPAN_ERR_WORKSPACE;
  const size_t words = spanattn::workspace_counter_bytes(desc) / sizeof(uint32_t);
  hipLaunchKernelGGL(spanattn::zero_words_kernel, dim3((unsigned)((words + 255) / 256)), dim3(256), 0,
                     (hipStream_t)desc->stream, (uint32_t*)desc->workspace, words);
  const hipError_t err = hipGetLastError();
  if (err != hipSuccess) {
    spanattn::g_last_hip_error = (int)err;
    return SPAN_ERR_HIP;
  }
  return SPAN_OK;
}

extern "C" int span_last_hip_error(void) { return spanattn::g_last_hip_error; }

#ifdef SPAN_PHASE_TRACE
// Diagnostic build only: device buffer of workgroups * 16 64-bit words that every later launch stamps (null = off);
// workgroups of a launch beyond `workgroups` leave no stamp.
extern "C" void span_debug_set_trace(void* device_words, size_t workgroups) {
  spanattn::g_trace = (unsigned long long*)device_words;
  spanattn::g_trace_workgroups = device_words ? workgroups : 0;
}
#endif
