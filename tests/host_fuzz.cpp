// Randomised driver for the host-only parts of the library (validator, span builder, blocked-encoding
// converters, partition planner).  Built with -fsanitize=address,undefined by tests/test_host_sanitizers.py:
// every array is heap-allocated at exactly the documented size, so any out-of-bounds access, signed overflow
// or use of an uninitialised slot the sanitizers can see aborts the run.  Results are also cross-checked
// against brute force where that is cheap.
#include <algorithm>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <set>
#include <vector>

#include "span_attn.h"
#include "span_internal.h"

#define REQUIRE(c)                                                      \
  do {                                                                  \
    if (!(c)) {                                                         \
      std::fprintf(stderr, "host_fuzz: %s failed at line %d\n", #c, __LINE__); \
      std::exit(1);                                                     \
    }                                                                   \
  } while (0)

static std::mt19937 rng(12345);
static int rnd(int lo, int hi) { return std::uniform_int_distribution<int>(lo, hi)(rng); }

static void fuzz_validate() {
  for (int it = 0; it < 20000; ++it) {
    const int B = rnd(1, 4), total = rnd(0, 10);
    std::vector<int32_t> off(B + 1), st(total), en(total), ctx(B);
    std::vector<int64_t> tok(B, -1);
    int acc = 0;
    for (int b = 0; b <= B; ++b) {
      off[b] = acc;
      acc += rnd(0, 3);
      if (rnd(0, 40) == 0) acc = rnd(-2, total + 2);
    }
    if (rnd(0, 3)) off[B] = total < off[B] ? off[B] : off[B];
    for (int i = 0; i < total; ++i) {
      st[i] = rnd(-1, 12);
      en[i] = st[i] + rnd(-1, 5);
    }
    for (int b = 0; b < B; ++b) ctx[b] = rnd(0, 14);
    int32_t bs = 99, bi = 99;
    const int rc = span_validate(B, total, off.data(), st.data(), en.data(), ctx.data(), &bs, &bi, tok.data());
    REQUIRE(rc >= 0 && rc <= 6);
    if (rc == 0) {
      REQUIRE(bs == -1 && bi == -1);
      for (int b = 0; b < B; ++b) {  // brute force: positions marked exactly once, ascending
        std::set<int> seen;
        int last = -1;
        for (int i = off[b]; i < off[b + 1]; ++i)
          for (int p = st[i]; p < en[i]; ++p) {
            REQUIRE(p >= 0 && p < ctx[b] && p > last && seen.insert(p).second);
            last = p;
          }
        REQUIRE(!seen.empty() && (int64_t)seen.size() == tok[b]);
      }
    } else {
      REQUIRE(bs >= 0 && bs < B);
    }
  }
}

static void fuzz_build() {
  for (int it = 0; it < 20000; ++it) {
    const int ctx = rnd(0, 60), na = rnd(0, 6), nr = rnd(0, 5), cap = rnd(0, 8);
    std::vector<int32_t> as(na), ae(na), rf(nr), rl(nr), os(cap), oe(cap);
    for (int k = 0; k < na; ++k) {
      as[k] = rnd(-1, ctx + 1);
      ae[k] = as[k] + rnd(-1, 20);
    }
    for (int r = 0; r < nr; ++r) {
      rf[r] = rnd(-2, na);
      rl[r] = rf[r] + rnd(-1, 2);
    }
    const int cur = rnd(-1, ctx + 1), prev = rnd(-1, ctx + 1), prefix = rnd(-1, ctx + 1);
    int32_t needed = -5;
    const int rc = span_build(na, as.data(), ae.data(), nr, rf.data(), rl.data(), prefix, prev, cur, ctx, cap,
                              os.data(), oe.data(), &needed);
    REQUIRE(rc == SPAN_OK || rc == SPAN_ERR_CAPACITY || rc == SPAN_BAD_RANGE);
    if (rc == SPAN_OK) {
      REQUIRE(needed >= 0 && needed <= cap);
      std::set<int> want, got;
      for (int p = 0; p < prefix; ++p) want.insert(p);
      for (int p = cur; p < ctx; ++p) want.insert(p);
      for (int r = 0; r < nr; ++r) {
        if (rf[r] == -1) {
          for (int p = prev; p < cur; ++p) want.insert(p);
        } else {
          for (int k = rf[r]; k <= rl[r]; ++k)
            for (int p = as[k]; p < ae[k]; ++p) want.insert(p);
        }
      }
      for (int i = 0; i < needed; ++i) {
        REQUIRE(os[i] < oe[i] && (i == 0 || os[i] > oe[i - 1]));
        for (int p = os[i]; p < oe[i]; ++p) got.insert(p);
      }
      REQUIRE(got == want);
    }
  }
}

static void fuzz_blocks() {
  for (int it = 0; it < 4000; ++it) {
    const int bs = 32 * rnd(1, 3), B = rnd(0, 3), words = bs / 32;
    std::vector<int32_t> boff(B + 1, 0), bidx;
    std::vector<uint32_t> masks;
    std::vector<std::set<int>> want(B);
    for (int b = 0; b < B; ++b) {
      int blk = rnd(0, 2);
      const int nb = rnd(0, 4);
      for (int j = 0; j < nb; ++j) {
        bidx.push_back(blk);
        for (int w = 0; w < words; ++w) {
          const uint32_t m = rnd(0, 3) == 0 ? 0xffffffffu : (uint32_t)rng() & (uint32_t)rng();
          masks.push_back(m);
          for (int t = 0; t < 32; ++t)
            if ((m >> t) & 1u) want[b].insert(blk * bs + w * 32 + t);
        }
        blk += rnd(1, 3);
      }
      boff[b + 1] = (int32_t)bidx.size();
    }
    const int cap = rnd(0, 40);
    std::vector<int32_t> off(B + 1, -7), st(cap), en(cap);
    int32_t needed = -1;
    int rc = span_blocks_to_intervals(B, bs, boff.data(), bidx.data(), masks.data(), cap, off.data(), st.data(),
                                      en.data(), &needed);
    REQUIRE(rc == SPAN_OK || rc == SPAN_ERR_CAPACITY);
    if (rc == SPAN_ERR_CAPACITY) {
      st.assign(needed, 0);
      en.assign(needed, 0);
      rc = span_blocks_to_intervals(B, bs, boff.data(), bidx.data(), masks.data(), needed, off.data(), st.data(),
                                    en.data(), &needed);
      REQUIRE(rc == SPAN_OK);
    }
    for (int b = 0; b < B; ++b) {
      std::set<int> got;
      for (int i = off[b]; i < off[b + 1]; ++i) {
        REQUIRE(st[i] < en[i] && (i == off[b] || st[i] > en[i - 1]));
        for (int p = st[i]; p < en[i]; ++p) got.insert(p);
      }
      REQUIRE(got == want[b]);
    }
    // and back
    const int bcap = rnd(0, 12);
    std::vector<int32_t> boff2(B + 1, -7), bidx2(bcap);
    std::vector<uint32_t> masks2((size_t)bcap * words);
    int32_t needed2 = -1;
    rc = span_intervals_to_blocks(B, bs, off.data(), st.data(), en.data(), bcap, boff2.data(), bidx2.data(),
                                  masks2.data(), &needed2);
    REQUIRE(rc == SPAN_OK || rc == SPAN_ERR_CAPACITY);
    if (rc == SPAN_OK) {
      size_t nonempty = 0;  // blocks whose mask is all zero are not listed on the way back
      for (size_t j = 0; j < bidx.size(); ++j) {
        bool any = false;
        for (int w = 0; w < words; ++w) any = any || masks[j * words + w] != 0;
        nonempty += any;
      }
      REQUIRE((size_t)needed2 == nonempty);
    }
  }
}

static void fuzz_plan() {
  std::vector<uint32_t> table(spanattn::kMaxPlanSlices);  // exactly the documented size
  for (int it = 0; it < 20000; ++it) {
    span_attn_desc_t d = {};
    d.batch = rnd(1, rnd(0, 5) ? 80 : 1200);
    d.heads = rnd(0, 3) ? 32 : rnd(1, 4000);
    d.head_dim = rnd(0, 1) ? 128 : 64;
    d.max_len = rnd(0, 3) ? rnd(1, 20000) : (1 << 22);
    d.dtype = rnd(0, 2);
    d.num_intervals = rnd(0, 100);
    d.max_tokens = rnd(0, 2) ? 0 : rnd(1, d.max_len);
    d.num_splits = rnd(0, 3) ? 0 : rnd(1, 70000);
    d.q_len = rnd(0, 2) ? 0 : rnd(1, 64);
    std::vector<int64_t> tok(d.batch);
    for (auto& t : tok) t = rnd(0, 9) == 0 ? rnd(-5, 0) : rnd(0, d.max_len + 10);
    d.tokens_per_seq = rnd(0, 1) ? tok.data() : nullptr;
    span_plan_info_t info;
    REQUIRE(span_plan_query(&d, &info) == SPAN_OK);
    const spanattn::Partition p = spanattn::plan_partition(&d, table.data());
    REQUIRE(p.num_splits >= 1 && p.slice_tokens >= 1 && p.total_slices >= 1);
    const bool matrix_pass = d.dtype != SPAN_F32 && d.head_dim == 128;  // 16-bit rows of 128: sixteen tokens a pass
    REQUIRE(p.queries_per_pass == (d.q_len >= 3 ? (matrix_pass ? 16 : 4) : (d.q_len == 2 ? 2 : 1)));
    REQUIRE(info.queries_per_pass == p.queries_per_pass);
    REQUIRE(info.workspace_bytes == (int64_t)span_workspace_bytes(&d));
    if (p.exact) {
      REQUIRE(p.total_slices <= spanattn::kMaxPlanSlices);
      int prev_b = -1, prev_s = -1;
      for (int y = 0; y < p.total_slices; ++y) {  // entries walk sequences and their slices in order
        const uint32_t e = table[y];
        const int b = e & 1023, s = (e >> 10) & 2047, n = e >> 21;
        REQUIRE(b < d.batch && s < n && n <= p.num_splits);
        REQUIRE((b == prev_b && s == prev_s + 1) || (b == prev_b + 1 && s == 0));
        prev_b = b;
        prev_s = s;
      }
      REQUIRE(prev_b == d.batch - 1);
    } else {
      REQUIRE(p.num_splits <= 65535 && p.total_slices == p.num_splits * d.batch);
    }
  }
}

// Run mode: with host copies of the span lists the planner resolves every slice to runs of cache positions.
// Brute force: write out the attended positions of each sequence in list order (with the clamps the kernel
// applies), cut them into the sequence's slices, and compare with what the runs enumerate.  Lists are mostly
// valid, sometimes garbage (negative lengths, offsets out of order or out of range).
static void fuzz_runs() {
  std::vector<uint32_t> table(spanattn::kMaxPlanSlices);
  int used = 0;
  for (int it = 0; it < 6000; ++it) {
    span_attn_desc_t d = {};
    d.batch = rnd(1, rnd(0, 3) ? 12 : 70);
    d.heads = rnd(0, 2) ? 32 : rnd(1, 64);
    d.head_dim = 128;
    d.max_len = rnd(0, 3) ? rnd(64, 5000) : rnd(1, 40);
    d.dtype = 1;
    d.q_len = rnd(0, 3) ? 0 : rnd(1, 8);
    const bool garbage = rnd(0, 9) == 0;
    std::vector<int32_t> off(d.batch + 1, 0), st, en;
    for (int b = 0; b < d.batch; ++b) {
      const int k = rnd(0, rnd(0, 4) ? 6 : 40);
      int pos = 0;
      for (int i = 0; i < k; ++i) {
        const int gap = rnd(0, 30), len = rnd(1, rnd(0, 2) ? 40 : 700);
        int s0 = pos + gap, e0 = s0 + len;
        if (e0 > d.max_len && !garbage) break;
        if (garbage && rnd(0, 5) == 0) e0 = s0 - rnd(0, 5);
        st.push_back(s0);
        en.push_back(e0);
        pos = e0 > pos ? e0 : pos;
      }
      off[b + 1] = (int32_t)st.size();
      if (garbage && rnd(0, 6) == 0) off[b + 1] = rnd(-3, (int)st.size() + 3);
    }
    d.num_intervals = (int32_t)st.size();
    if (garbage && d.num_intervals > 0 && rnd(0, 3) == 0) d.num_intervals -= 1;  // lists longer than declared
    d.max_tokens = rnd(0, 3) ? 0 : rnd(1, d.max_len);
    d.host_span_offsets = off.data();
    d.host_span_starts = st.data();  // exactly as long as the list: any read past num_intervals is caught
    d.host_span_ends = en.data();
    std::vector<int64_t> wrong(d.batch, 1);
    d.tokens_per_seq = rnd(0, 1) ? wrong.data() : nullptr;  // not consulted when the lists are there
    std::vector<spanattn::RunTables> rt(1);                   // heap copy: reads past the tables are caught too
    const spanattn::Partition p = spanattn::plan_partition(&d, table.data(), rt.data());
    span_plan_info_t info;
    REQUIRE(span_plan_query(&d, &info) == SPAN_OK);
    REQUIRE((info.runs_in_arguments != 0) == p.runs);
    REQUIRE(info.workspace_bytes == (int64_t)span_workspace_bytes(&d));
    if (!p.runs) continue;
    ++used;
    const spanattn::RunTables& r = rt[0];
    REQUIRE(p.even && p.total_slices <= spanattn::kMaxRunSlices);
    const int64_t max_tok = (d.max_tokens > 0 && d.max_tokens < d.max_len) ? d.max_tokens : d.max_len;
    int y = 0;
    for (int b = 0; b < d.batch; ++b) {
      std::vector<int64_t> want;  // attended positions in list order, before the position clamp
      const int lo = std::min(std::max(off[b], 0), d.num_intervals), hi = std::min(std::max(off[b + 1], lo), d.num_intervals);
      for (int i = lo; i < hi; ++i) {
        const int64_t len = std::min<int64_t>(std::max<int64_t>((int64_t)en[i] - st[i], 0), d.max_len);
        for (int64_t t = 0; t < len; ++t) want.push_back((int64_t)st[i] + t);
      }
      if ((int64_t)want.size() > max_tok) want.resize((size_t)max_tok);
      const int64_t n = (int64_t)want.size();
      const uint32_t e0 = r.slices[y].entry;
      const int nsl = (int)(e0 >> 21);
      REQUIRE(nsl >= 1);
      const int64_t T = (n + nsl - 1) / nsl;
      for (int s = 0; s < nsl; ++s, ++y) {
        REQUIRE(y < p.total_slices);
        const uint32_t e = r.slices[y].entry;
        REQUIRE((int)(e & 1023) == b && (int)((e >> 10) & 2047) == s && (int)(e >> 21) == nsl);
        const int run0 = (int)(r.slices[y].runs_of & 0xffff), nrun = (int)(r.slices[y].runs_of >> 16);
        REQUIRE(run0 + nrun <= spanattn::kMaxRuns);
        std::vector<int64_t> got;
        for (int j = run0; j < run0 + nrun; ++j) {
          REQUIRE(r.run[j][1] > 0);
          for (int t = 0; t < r.run[j][1]; ++t) got.push_back((int64_t)r.run[j][0] + t);
        }
        const int64_t v0 = std::min<int64_t>(n, (int64_t)s * T), v1 = std::min<int64_t>(n, (int64_t)(s + 1) * T);
        REQUIRE((int64_t)got.size() == v1 - v0 && r.slices[y].rows == (int32_t)(v1 - v0));
        REQUIRE(r.slices[y].rows <= spanattn::kMaxRunSliceRows);
        for (int64_t v = v0; v < v1; ++v) REQUIRE(got[(size_t)(v - v0)] == want[(size_t)v]);
      }
    }
    REQUIRE(y == p.total_slices);
  }
  REQUIRE(used > 500);  // the mode was actually exercised
}

int main() {
  fuzz_runs();
  fuzz_validate();
  fuzz_build();
  fuzz_blocks();
  fuzz_plan();
  std::puts("host_fuzz: ok");
  return 0;
}
