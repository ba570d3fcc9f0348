// The HIP library's per-rank code (bcast_device.hpp) compiled for the CPU, so
// that its logic and its index arithmetic can be checked against the oracle
// without a GPU, under gdb or a sanitizer if need be.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <ucontext.h>

#include <functional>

#include "../../paper_2407_18004_amd/csrc/bcast_device.hpp"

using namespace bcast;

// A wavefront on the CPU: every lane is a coroutine with a stack of its own.  A lane runs until
// it reaches a cross-lane operation and waits there; once every lane that has not finished is
// waiting, the operation is carried out over the waiting lanes (the active lanes of the GPU)
// and they go on.  Lanes that meet must have reached the same operation at the same place in
// the source and as their n-th operation, which holds for code whose cross-lane operations sit
// in control flow that is the same for all lanes; anything else is counted in `mismatches`.
namespace shim_wave {

constexpr int kLanes = 64;
constexpr size_t kStackBytes = 256 * 1024;

struct Lane {
  ucontext_t ctx;
  bool done, waiting;
  int op, value, arg, site, result;
  uint64_t n_ops;
};

static Lane lanes[kLanes];
static char *stacks = nullptr;
static ucontext_t scheduler;
static int current = -1;                     // lane that is running, -1 outside run()
static const std::function<void(int)> *body = nullptr;
static uint64_t mismatches = 0, operations = 0;

int cross_lane(Op op, int value, int arg, int site) {
  if (current < 0) return value;             // a wavefront of one lane
  Lane &l = lanes[current];
  l.op = op; l.value = value; l.arg = arg; l.site = site;
  l.waiting = true;
  ++l.n_ops;
  swapcontext(&l.ctx, &scheduler);
  return l.result;
}

static void lane_main() {
  (*body)(current);
  lanes[current].done = true;
  swapcontext(&lanes[current].ctx, &scheduler);
}

void run(int n_lanes, const std::function<void(int)> &f) {
  if (!stacks) stacks = (char *)malloc(kLanes * kStackBytes);
  body = &f;
  for (int l = 0; l < n_lanes; ++l) {
    Lane &ln = lanes[l];
    getcontext(&ln.ctx);
    ln.ctx.uc_stack.ss_sp = stacks + (size_t)l * kStackBytes;
    ln.ctx.uc_stack.ss_size = kStackBytes;
    ln.ctx.uc_link = &scheduler;
    makecontext(&ln.ctx, lane_main, 0);
    ln.done = false; ln.waiting = false; ln.n_ops = 0;
  }
  for (;;) {
    for (int l = 0; l < n_lanes; ++l) {
      if (lanes[l].done || lanes[l].waiting) continue;
      current = l;
      swapcontext(&scheduler, &lanes[l].ctx);
    }
    current = -1;
    int first = -1;
    for (int l = 0; l < n_lanes; ++l)
      if (!lanes[l].done) { first = l; break; }
    if (first < 0) break;
    // every lane still alive is waiting: carry out the operation over them
    const Lane &f0 = lanes[first];
    int any = 0;
    for (int l = 0; l < n_lanes; ++l) {
      if (lanes[l].done) continue;
      if (lanes[l].op != f0.op || lanes[l].site != f0.site || lanes[l].n_ops != f0.n_ops ||
          (f0.op == kShflXor && lanes[l].arg != f0.arg))
      { if (!mismatches && getenv("SHIM_WAVE_DEBUG")) fprintf(stderr, "mismatch: lane %d op %d site %d n %llu vs lane %d op %d site %d n %llu\n", l, lanes[l].op, lanes[l].site, (unsigned long long)lanes[l].n_ops, first, f0.op, f0.site, (unsigned long long)f0.n_ops); ++mismatches; }
      any |= lanes[l].value;
    }
    ++operations;
    for (int l = 0; l < n_lanes; ++l) {
      Lane &ln = lanes[l];
      if (ln.done) continue;
      if (ln.op == kAny) ln.result = any;
      else if (ln.op == kFirstLane) ln.result = f0.value;
      else {                                   // the partner's value; an idle partner gives one's own
        const int partner = l ^ ln.arg;
        ln.result = partner < n_lanes && !lanes[partner].done ? lanes[partner].value : ln.value;
      }
    }
    for (int l = 0; l < n_lanes; ++l) lanes[l].waiting = false;
  }
  body = nullptr;
}

}  // namespace shim_wave

static uint32_t q_of(uint32_t p) {
  uint32_t q = 0;
  while ((1ull << q) < (uint64_t)p) ++q;
  return q;
}

static uint64_t g_replays = 0, g_top_replays = 0, g_mid_replays = 0, g_from_table = 0, g_generic = 0;

extern "C" {

// tiles of the last shim_schedules_tiles call that replayed a lockstep record
uint64_t shim_last_replays(void) { return g_replays; }
// ... and that took over the state after the top levels
uint64_t shim_last_top_replays(void) { return g_top_replays; }
// tiles that took only the second part of the lockstep stretch from the record
uint64_t shim_last_mid_replays(void) { return g_mid_replays; }

// rows: m rows of 2q int32 (recv then send) for the physical ranks given.
// flags_out/hash_out (may be NULL): per-rank flags and row hash.
// flat != 0: with the search run through its one branch-free body, as the kernel for lists of
// arbitrary ranks runs it.
int shim_schedules_ranks(uint32_t p, uint32_t root, const uint32_t *ranks, uint64_t m, int flat,
                         int32_t *rows, uint32_t *flags_out, uint64_t *hash_out) {
  const uint32_t q = q_of(p);
  const Instance in = make_instance(p, q, root);
  for (uint64_t i = 0; i < m; ++i) {
    alignas(4) int8_t buf[72];              // rows are read by aligned words, a little past 2q bytes
    memset(buf, 0x55, sizeof buf);
    int b = 0;
    const uint32_t v = virtual_rank(in, ranks[i]);
    uint32_t fl;
    if (flat) {
      LockstepCache none;
      lockstep_cache_init(none, nullptr);
      DeepTable no_table;
      no_table.entries = nullptr; no_table.viol_by_e = nullptr; no_table.first_deep = 0; no_table.n_rho = 0;
      MemoOut unused;
      const uint32_t viol = compute_rank_phase1<false, true>(in, v, buf, buf + q, b, fl, none, false,
                                                             no_table, unused);
      fl |= resolve_by_search<true>(in, v, viol, buf + q);
    } else {
      fl = compute_rank(in, v, buf, buf + q, b);
    }
    for (uint32_t k = 0; k < 2 * q; ++k) rows[i * 2 * q + k] = buf[k];
    uint64_t h = 0;
    uint32_t fl2 = 0;
    digest_rank(in, ranks[i], v, b, buf, h, fl2);
    if (flags_out) flags_out[i] = fl | fl2;
    if (hash_out) hash_out[i] = h;
  }
  return (int)q;
}

// The same for n consecutive physical ranks from r_begin, the way the wavefronts of the kernels
// work through them: the tiles of 64 ranks are dealt out as runs of run_tiles tiles (0: one run),
// one wavefront to a run with a fresh record; inside a run the tiles are taken from the highest
// down with the receive rows of the tile above at hand (descending != 0: the kernels for p with
// violations of Algorithm 6) or from the lowest up without them (the kernels for p = 2^q and
// 2^q - 1).  Phase one of a tile runs as a wavefront of 64 lanes (shim_wave::run) with one
// record shared by the lanes, as in LDS; then violations are filled in from rows of the same
// tile or the tile above, then the rest by search.
// use_table != 0: with the table of deep entries (built here, one entry per rho, by the
// function the GPU's builder kernel calls), when p has enough levels above the deep ones.
int shim_schedules_tiles(uint32_t p, uint32_t root, uint32_t r_begin, uint64_t n,
                         uint32_t run_tiles, int descending, int use_table,
                         int32_t *rows, uint32_t *flags_out, uint64_t *hash_out,
                         uint64_t *n_from_tile) {
  const uint32_t q = q_of(p);
  const Instance in = make_instance(p, q, root);
  uint64_t borrowed = 0;
  static uint4 entries[kDeepMaxEntries];
  static uint16_t viol_by_e[kDeepEs * kDeepMaxEntries];
  DeepTable table;
  table.entries = nullptr; table.viol_by_e = nullptr; table.first_deep = 0; table.n_rho = 0;
  g_from_table = 0; g_generic = 0;
  if (use_table && q > 0 && first_deep_level(p - 1u) >= kDeepMinUpperLevels + 1u) {
    table.first_deep = first_deep_level(p - 1u);
    table.n_rho = deep_table_rhos(p - 1u, table.first_deep);
    if (table.n_rho > kDeepMaxEntries) return -1;
    for (uint32_t rho = 0; rho < table.n_rho; ++rho) {
      entries[rho] = deep_entry_build(p - 1u, q, table.first_deep, rho);
      for (uint32_t less = 1; less < kDeepEs; ++less)
        viol_by_e[less * kDeepMaxEntries + rho] = deep_viol_build(p - 1u, q, table.first_deep, rho, less);
    }
    table.entries = entries;
    table.viol_by_e = viol_by_e;
  }
  // one slice that is reused (rows of the previous tile stay where they are until they are
  // overwritten) and a copy of the receive rows of the tile above
  alignas(4) static int8_t tile[64 * 68];      // rows digest_row_pitch(q) apart, as k_digest keeps them
  const uint32_t pitch = digest_row_pitch(q);
  static int8_t above[64 * 31];
  static LockstepCacheSplit caches[64];            // one per lane (its number) ...
  static uint32_t record_mem[kRecordWords];   // ... the rest is the wavefront's
  g_replays = 0;
  g_top_replays = 0;
  g_mid_replays = 0;
  shim_wave::mismatches = 0;
  shim_wave::operations = 0;
  const uint64_t n_tiles = (n + 63) / 64;
  const uint64_t per_run = run_tiles ? run_tiles : (n_tiles ? n_tiles : 1);
  for (uint64_t run0 = 0; run0 < n_tiles; run0 += per_run) {
    const uint64_t run1 = run0 + per_run < n_tiles ? run0 + per_run : n_tiles;
    memset(tile, 0x55, sizeof tile);
    for (int l = 0; l < 64; ++l) lockstep_cache_init(caches[l], record_mem, (uint32_t)l, run1 - run0 >= 8);
    const bool long_run = run1 - run0 >= 3;   // as in the kernels
    uint32_t n_valid_next = 0;
    const int8_t *next_recv = nullptr;
    for (uint64_t step = 0; step < run1 - run0; ++step) {
      const uint64_t ti = descending ? run1 - 1 - step : run0 + step;
      const uint64_t row0 = ti * 64;
      const uint32_t n_valid = n - row0 < 64 ? (uint32_t)(n - row0) : 64u;
      uint32_t viol[64], fl[64], vr[64];
      int b[64];
      MemoOut memo[64];
      shim_wave::run((int)n_valid, [&](int lane) {
        vr[lane] = virtual_rank(in, (uint32_t)(r_begin + row0 + lane));
        if (table.entries)
          viol[lane] = compute_rank_phase1<true>(in, vr[lane], tile + lane * pitch,
                                                 tile + lane * pitch + q, b[lane], fl[lane],
                                                 caches[lane], long_run && n_valid == 64, table, memo[lane]);
        else
          viol[lane] = compute_rank_phase1(in, vr[lane], tile + lane * pitch,
                                           tile + lane * pitch + q, b[lane], fl[lane],
                                           caches[lane], long_run && n_valid == 64);
      });
      for (uint32_t lane = 0; lane < n_valid; ++lane) {
        int8_t *recv_row = tile + lane * pitch;
        uint32_t open = resolve_from_tiles(in, viol[lane], recv_row + q, tile, next_recv,
                                           pitch, q, lane, n_valid, n_valid_next);
        borrowed += (uint64_t)__popc(viol[lane] ^ open);
        if (table.entries) {
          const uint32_t left = resolve_from_table(in, table, vr[lane], memo[lane], open, recv_row + q);
          g_from_table += (uint64_t)__popc(open ^ left);
          g_generic += memo[lane].rho >= 2u;
          open = left;
        }
        fl[lane] |= resolve_by_search(in, vr[lane], open, recv_row + q);
      }
      for (uint32_t lane = 0; lane < n_valid; ++lane) {
        const uint64_t i = row0 + lane;
        const int8_t *recv_row = tile + lane * pitch;
        for (uint32_t k = 0; k < 2 * q; ++k) rows[i * 2 * q + k] = recv_row[k];
        uint64_t h = 0;
        uint32_t fl2 = 0;
        digest_rank(in, (uint32_t)(r_begin + i), vr[lane], b[lane], recv_row, h, fl2);
        if (flags_out) flags_out[i] = fl[lane] | fl2;
        if (hash_out) hash_out[i] = h;
        if (descending)
          for (uint32_t k = 0; k < q; ++k) above[lane * q + k] = recv_row[k];
      }
      if (descending) { next_recv = above; n_valid_next = n_valid; }
    }
    // the lanes of a tile bump the counters one after the other here, not together as on the
    // GPU: 64 per tile that replayed
    g_replays += record_mem[kRecReplays] / 64u;
    g_top_replays += record_mem[kTopReplays] / 64u;
    g_mid_replays += record_mem[kMidReplays] / 64u;
  }
  if (n_from_tile) *n_from_tile = borrowed;
  return (int)q;
}

// violations of the last shim_schedules_tiles call answered from the table of deep entries, and
// ranks that had a rho of 2 or more
uint64_t shim_last_from_table(void) { return g_from_table; }
uint64_t shim_last_generic(void) { return g_generic; }

// the table of deep entries of p (n entries of four words), as the builder kernel writes it
int shim_deep_table(uint32_t p, uint32_t *out, uint32_t cap) {
  const uint32_t q = q_of(p);
  if (q == 0) return 0;
  const uint32_t fd = first_deep_level(p - 1u);
  const uint32_t n = deep_table_rhos(p - 1u, fd);
  if (n > cap) return -1;
  for (uint32_t rho = 0; rho < n; ++rho) {
    const uint4 e = deep_entry_build(p - 1u, q, fd, rho);
    out[4 * rho] = e.x; out[4 * rho + 1] = e.y; out[4 * rho + 2] = e.z; out[4 * rho + 3] = e.w;
  }
  return (int)n;
}

// cross-lane operations carried out by the last shim_schedules_tiles call, and how many of them
// found lanes that had come from different places (must be 0)
uint64_t shim_wave_operations(void) { return shim_wave::operations; }
uint64_t shim_wave_mismatches(void) { return shim_wave::mismatches; }

// the two XOR contributions of one row to the edge check
void shim_edge_row(uint32_t p, uint32_t root, uint32_t r, const int32_t *row, uint64_t *xr,
                   uint64_t *xs) {
  const uint32_t q = q_of(p);
  const Instance in = make_instance(p, q, root);
  alignas(4) int8_t buf[72] = {0};
  for (uint32_t k = 0; k < 2 * q; ++k) buf[k] = (int8_t)row[k];
  edge_rank(in, r, buf, *xr, *xs);
}

// flags and hash of a row given by the caller (for planted mistakes)
void shim_digest_row(uint32_t p, uint32_t root, uint32_t r, const int32_t *row,
                     uint64_t *hash, uint32_t *flags) {
  const uint32_t q = q_of(p);
  const Instance in = make_instance(p, q, root);
  alignas(4) int8_t buf[72] = {0};
  for (uint32_t k = 0; k < 2 * q; ++k) buf[k] = (int8_t)row[k];
  const uint32_t v = virtual_rank(in, r);
  const int b = (int)q - (int)baseblock_level(in.pm1, q, v);
  digest_rank(in, r, v, b, buf, *hash, *flags);
}

// recvblock[0..q-1] of virtual rank v by the plain form of the search (recv_search) and by the
// form the kernels run (top_down_level + recv_ascent); returns how many entries each produced
// (plain in the low half, reorganised in the high half) and whether either raised an anomaly
uint32_t shim_recv_two_ways(uint32_t p, uint32_t v, int32_t *plain, int32_t *fast, uint32_t *anomalies) {
  const uint32_t q = q_of(p);
  const Instance in = make_instance(p, q, 0);
  TopDown s = top_down_start(p, v);
  uint32_t unused = 0;
  for (uint32_t j = 1; j <= q; ++j)
    top_down_level<false, false>(in.pm1, q, j, s, unused, [](uint32_t, int) {});
  bool an_plain = false, an_fast = false;
  const uint32_t n_plain = q ? recv_search(p, in.pm1, q, v, s.jb, q - 1u, an_plain,
                                           [&](uint32_t k, int x) { plain[k] = x; }) : 0u;
  LockstepCache none;
  lockstep_cache_init(none, nullptr);
  const uint32_t n_fast = q ? recv_ascent(p, in.pm1, q, s.jb, q - 1u, s.W, s.pathr, s.anom, an_fast,
                                          [&](uint32_t k, int x) { fast[k] = x; }, none, false) : 0u;
  *anomalies = (uint32_t)an_plain | ((uint32_t)an_fast << 1);
  return n_plain | (n_fast << 16);
}

// index helpers of the pass over the levels, for direct checks against Algorithm 2's skips
uint32_t shim_first_level_taken(uint32_t p, uint32_t v) { return first_level_taken(p - 1u, v); }
uint32_t shim_top_level_count(uint32_t p) { return top_level_count(p - 1u, q_of(p)); }
uint32_t shim_top_skip(void) { return kTopSkip; }

}  // extern "C"
