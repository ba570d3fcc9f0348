// gfx950 kernels and the C ABI of include/bcast.h.
//
// Launch shape shared by the schedule kernels: workgroups of 256 lanes = four
// wavefronts; a wavefront owns a tile of 64 consecutive ranks and never needs
// a workgroup barrier.  Each lane computes one rank (Algorithms 3, 5, 6) with
// its state in VGPRs and drops the 2q results as bytes into the wavefront's
// slice of LDS, laid out exactly like the output rows, so that the tile leaves
// the CU as 16-byte stores to consecutive addresses.  A wavefront works
// through one contiguous run of tiles and carries what neighbouring tiles have
// in common from one to the next (LockstepCache); the grid is sized so that
// runs are a few tiles long and there are several times more workgroups than
// fit on the chip at once.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>
#include <mutex>
#include <type_traits>

#include "../../include/bcast.h"
#include "bcast_device.hpp"

using namespace bcast;

namespace {

constexpr int kWave = 64;
constexpr int kWavesPerBlock = 4;
constexpr int kBlock = kWave * kWavesPerBlock;
constexpr int kMaxFields = 62;                       // 2q for q = 31
constexpr int kTileBytes = kWave * kMaxFields;       // 3968, a multiple of 16
constexpr int kInvalidEntry = INT32_MIN;           // row of a rank that is not in its instance

enum Layout : int { kInterleaved = 0, kSeparate = 1, kRowwise = 2 };

// Orders the byte stores of the compute phase before the word loads of the
// copy-out phase (and back) inside one wavefront.  LDS operations of a
// wavefront complete in order, so no workgroup barrier is needed.
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Copies n_bytes schedule bytes from LDS (4-byte aligned) to n_bytes int32 at
// dst, all 64 lanes of the wavefront cooperating, widest stores possible.
// With kMarkInvalid the byte kInvalidByte (never a schedule entry) widens to
// kInvalidEntry instead of to itself.
constexpr int kInvalidByte = -128;

template <bool kMarkInvalid>
__device__ __forceinline__ int widen(int byte_val) {
  if (kMarkInvalid) return byte_val == kInvalidByte ? kInvalidEntry : byte_val;
  return byte_val;
}

// kStream: the 16-byte stores are marked non-temporal.
template <bool kMarkInvalid, bool kStream = false>
__device__ __forceinline__ void tile_out(const uint32_t *lds_words, int32_t *dst,
                                         uint32_t n_bytes, uint32_t lane) {
  const uint32_t groups = n_bytes >> 2;
  const int8_t *bytes = reinterpret_cast<const int8_t *>(lds_words);
  if ((reinterpret_cast<uintptr_t>(dst) & 15u) == 0) {
    int4 *dst4 = reinterpret_cast<int4 *>(dst);
    for (uint32_t g = lane; g < groups; g += kWave) {
      const uint32_t w = lds_words[g];
      int4 o;
      o.x = widen<kMarkInvalid>((int)(int8_t)(w & 0xFF));
      o.y = widen<kMarkInvalid>((int)(int8_t)((w >> 8) & 0xFF));
      o.z = widen<kMarkInvalid>((int)(int8_t)((w >> 16) & 0xFF));
      o.w = widen<kMarkInvalid>((int)(int8_t)(w >> 24));
      if (kStream) {
        __builtin_nontemporal_store(o.x, &dst[4u * g]);
        __builtin_nontemporal_store(o.y, &dst[4u * g + 1u]);
        __builtin_nontemporal_store(o.z, &dst[4u * g + 2u]);
        __builtin_nontemporal_store(o.w, &dst[4u * g + 3u]);
      } else {
        dst4[g] = o;
      }
    }
  } else {
    for (uint32_t i = lane; i < (groups << 2); i += kWave)
      dst[i] = widen<kMarkInvalid>((int)bytes[i]);
  }
  for (uint32_t i = (groups << 2) + lane; i < n_bytes; i += kWave)
    dst[i] = widen<kMarkInvalid>((int)bytes[i]);
}

// ---------------------------------------------------------------- schedules

// How the tiles of a launch are dealt out: every wavefront works through one contiguous run of
// tiles.  The workgroups form kRunClasses classes by their number (class_blocks consecutive
// workgroups each); a class owns a contiguous range of tiles and deals it out evenly, so classes
// can be given runs of different lengths.
// k_digest records the lockstep stretch in two parts in runs of this many tiles and more (4 % faster
// with runs of 43 tiles).  k_schedules does not, and is compiled without that code: its long launches
// are bound by their stores, its short ones by latency, and the code alone cost the table of
// p = 1,000,003 3 us.
constexpr uint64_t kSplitRunTiles = 8;
constexpr uint32_t kRunClasses = 8;
struct RunSplit {
  uint32_t class_blocks;            // workgroups per class
  uint32_t first[kRunClasses];      // first tile of the class
  uint32_t base[kRunClasses];       // tiles per wavefront of the class ...
  uint32_t extra[kRunClasses];      // ... its first `extra` wavefronts take one more
};

struct SchedParams {
  uint32_t p, q, root;
  uint64_t r_begin, n_ranks;
  RunSplit runs;
  int32_t *recv, *send;
  int64_t ld;
  int layout;
  DeepTable table;                  // kernels with kMemo only
  // Entries of the send part that k_schedules<true, .> leaves open for k_fill_open (row of the
  // launch << 5 | round), or null: then the kernel fills them in itself, by search.
  // Two forms.  One list for the launch (open_segments = 0): open_count is one word, the entries
  // claimed so far (may run past open_cap), zero at launch.  A segment of open_cap entries per
  // wavefront (open_segments = wavefronts of the launch): segment w is open_list[w * open_cap ..],
  // and every wavefront stores how many it has used to open_count[w] before it ends, so nothing
  // has to be cleared ahead of the launch.
  unsigned long long *open_list;
  uint32_t *open_count;
  uint32_t open_cap;
  uint32_t open_segments;
};

// The run of wavefront `wave` (the same in all lanes) of this workgroup: first tile and number
// of tiles.  Everything stays below the number of tiles (< 2^32).
__device__ __forceinline__ void run_of_wave(const RunSplit &rs, uint32_t wave, uint32_t &t_lo,
                                            uint32_t &n_tiles) {
  uint32_t cls = blockIdx.x / rs.class_blocks;
  cls = cls < kRunClasses ? cls : kRunClasses - 1u;
  uint32_t first = rs.first[0], base = rs.base[0], extra = rs.extra[0];
#pragma unroll
  for (uint32_t c = 1; c < kRunClasses; ++c)
    if (cls == c) { first = rs.first[c]; base = rs.base[c]; extra = rs.extra[c]; }
  const uint32_t w = (blockIdx.x - cls * rs.class_blocks) * kWavesPerBlock + wave;
  t_lo = first + w * base + (w < extra ? w : extra);
  n_tiles = base + (w < extra ? 1u : 0u);
}

__device__ __forceinline__ void tile_run(const RunSplit &rs, uint64_t &t_lo, uint64_t &t_hi) {
  // the wavefront's number is the same in all its lanes: say so, or the loop over the run and
  // everything derived from it would be kept per lane
  uint32_t lo, n;
  run_of_wave(rs, (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x / kWave)), lo, n);
  t_lo = lo;
  t_hi = (uint64_t)lo + n;
}

// LDS of the tiled kernels is sized at launch: per wavefront one slice of 64
// rows of 2q bytes (rounded up to 16 bytes).
__host__ __device__ inline uint32_t slice_words(uint32_t q) { return ((kWave * 2u * q + 15u) / 16u) * 4u; }
// ... plus, for wavefronts that work through runs of tiles, kRecordWords words
// for what they carry from tile to tile (LockstepCache::mem), after all slices.
__host__ __device__ inline uint32_t lone_block_words(uint32_t q) {
  return kWavesPerBlock * (slice_words(q) + kRecordWords);
}

struct TileState {
  uint32_t v, n_valid, flags;
  int b;
};

// Computes the rows of tile `tile` (one per lane) into the wavefront's slice,
// violations of Algorithm 6 resolved from rows of the same tile or else by
// search on the spot: for p = 2^q and 2^q - 1, which have next to none.
// slices: the workgroup's four slices, slice_w words each.
template <bool kMemo, typename Cache>
__device__ __forceinline__ TileState tile_rows(const Instance &in, uint64_t r_begin,
                                               uint64_t n_ranks, uint64_t tile, uint64_t n_tiles,
                                               uint32_t *slices, uint32_t slice_w, uint32_t pitch,
                                               uint32_t send_off, uint32_t lane, uint32_t wave,
                                               Cache &cache, bool use_cache,
                                               const DeepTable &table) {
  TileState st;
  st.v = 0; st.flags = 0; st.b = 0;
  int8_t *tile_recv = reinterpret_cast<int8_t *>(slices + wave * slice_w);
  int8_t *recv_row = tile_recv + lane * pitch;
  int8_t *send_row = recv_row + send_off;
  const uint64_t row0 = tile * kWave;
  st.n_valid = tile < n_tiles ? (n_ranks - row0 < kWave ? (uint32_t)(n_ranks - row0) : kWave) : 0u;
  uint32_t viol = 0;
  MemoOut memo;
  memo.rho = 0; memo.room = 0;
  if (lane < st.n_valid) {
    st.v = virtual_rank(in, (uint32_t)(r_begin + row0 + lane));
    viol = compute_rank_phase1<kMemo>(in, st.v, recv_row, send_row, st.b, st.flags,
                                      cache, use_cache && st.n_valid == (uint32_t)kWave, table, memo);
  }
  wave_lds_sync();
  if (lane < st.n_valid) {
    uint32_t open = resolve_from_tiles(in, viol, send_row, tile_recv, nullptr, pitch, pitch,
                                       lane, st.n_valid, 0u);
    if (kMemo) open = resolve_from_table(in, table, st.v, memo, open, send_row);
    st.flags |= resolve_by_search(in, st.v, open, send_row);
  }
  wave_lds_sync();
  return st;
}

// Deferred violations of k_schedules<true>.  A wavefront works through its run
// of tiles from the highest down and keeps the receive rows of the tile it has
// just finished (64 rows of q bytes), so a violation of Algorithm 6 whose
// to-processor is at most one tile up is answered from LDS.  The others are not
// searched for on the spot, where they would occupy a few lanes of an otherwise
// idle wavefront per tile: the row leaves with the entry still open, its place
// (row within the run << 5 | k) goes into a queue in LDS, and whenever 64 are waiting, and once more at the
// end of the run, one search per lane fills them in and stores the entries
// straight into the table.  At the end of the run the four wavefronts of the
// workgroup, whose runs are neighbours, meet at a barrier: what the highest tile
// of a run left open is read from the next wavefront's lowest tile, and the
// remaining entries of all four are searched for together.
constexpr uint32_t kDeferCap = 128u;                 // queue entries per wavefront (tables)
constexpr uint32_t kRowQueueCap = 2u * kWave;         // ... of k_digest: 63 left over + 64 of a tile
constexpr uint32_t kQueueWords = kDeferCap > kRowQueueCap ? kDeferCap : kRowQueueCap;

// Of the receive rows of the tile above only rounds 0 .. kAboveRounds - 1 are kept: a violation in
// round k asks for the rank skip[k] further on, and only skip[0..7] <= 2^7 reach no further
// than the next tile from some lane of this one (skip[8] > 128).
constexpr uint32_t kAboveRounds = 8;
constexpr uint32_t kAboveWords = kWave * kAboveRounds / 4u;
// words of LDS per wavefront: slice, receive rows of the tile above, queue
__host__ __device__ inline uint32_t deferred_wave_words(uint32_t q) {
  return slice_words(q) + kAboveWords + kQueueWords + kRecordWords;
}
// The same for k_digest, whose rows never leave LDS and are laid out for word reads: 64 rows
// digest_row_pitch(q) bytes apart.
__host__ __device__ inline uint32_t digest_slice_words(uint32_t q) { return 16u * digest_row_pitch(q); }
__host__ __device__ inline uint32_t digest_lone_block_words(uint32_t q) {
  return kWavesPerBlock * (digest_slice_words(q) + kRecordWords);
}
__host__ __device__ inline uint32_t digest_deferred_wave_words(uint32_t q) {
  return digest_slice_words(q) + kAboveWords + kQueueWords + kRecordWords;
}

// Hands n entries (one per lane with `mine`, as row of the launch << 5 | round) to the list that
// k_fill_open works off after this kernel, if there is a list and it has room for all of them.
// Returns whether it did (the same in all lanes).
__device__ __forceinline__ bool publish_open(const SchedParams &prm, uint32_t wave_id, uint32_t &seg_used,
                                             uint32_t n, bool mine, unsigned long long entry, uint32_t lane) {
  if (prm.open_list == nullptr || n == 0u) return n == 0u && prm.open_list != nullptr;
  if (prm.open_segments != 0u) {                     // the wavefront's own segment
    if (wave_id >= prm.open_segments || n > prm.open_cap - seg_used) return false;
    const uint64_t who = __ballot(mine);
    if (mine)
      prm.open_list[(uint64_t)wave_id * prm.open_cap + seg_used + (uint32_t)__popcll(who & ((1ull << lane) - 1ull))] = entry;
    seg_used += n;
    return true;
  }
  uint32_t base = 0;
  if (lane == 0) base = atomicAdd(prm.open_count, n);
  base = lane0_of(base);
  if (base >= prm.open_cap) return false;            // full
  if (n > prm.open_cap - base) {                     // the claim does not fit: its slots stay unused
    if (base + lane < prm.open_cap) prm.open_list[base + lane] = ~0ull;     // fewer than 64 of them
    return false;
  }
  const uint64_t who = __ballot(mine);
  if (mine) prm.open_list[base + (uint32_t)__popcll(who & ((1ull << lane) - 1ull))] = entry;
  return true;
}

__device__ __forceinline__ void deferred_flush(const Instance &in, const SchedParams &prm,
                                               const uint32_t *queue, uint64_t run_row0,
                                               uint32_t lo, uint32_t hi, uint32_t lane,
                                               uint32_t wave_id, uint32_t &seg_used) {
  // The rows were stored by this wavefront; they must have landed before single
  // entries of them are overwritten.
  if (publish_open(prm, wave_id, seg_used, hi - lo, lo + lane < hi,
                   lo + lane < hi ? ((run_row0 + (queue[lo + lane] >> 5)) << 5) | (queue[lo + lane] & 31u) : 0ull,
                   lane))
    return;
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  if (lo + lane < hi) {
    const uint32_t item = queue[lo + lane];
    const uint64_t row = run_row0 + (item >> 5);     // row in the launch
    const uint32_t k = item & 31u;
    const uint32_t v = virtual_rank(in, (uint32_t)(prm.r_begin + row));
    uint32_t fl = 0;
    prm.send[row * (uint64_t)prm.ld + k] = search_entry(in, to_processor(in, v, k), k, fl);
  }
}

template <bool kShare, bool kMemo>
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(8, 8))) void k_schedules(SchedParams prm) {
  extern __shared__ __align__(16) uint32_t lds_dyn[];
  const uint32_t lane = threadIdx.x & (kWave - 1);
  const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x / kWave));
  const Instance in = make_instance(prm.p, prm.q, prm.root);
  const uint32_t q = prm.q;
  const uint32_t slice_w = slice_words(q);
  // row pitch, and offset of the send part inside the slice
  const uint32_t pitch = prm.layout == kSeparate ? q : 2u * q;
  const uint32_t send_off = prm.layout == kSeparate ? kWave * q : q;
  uint32_t *words = lds_dyn + wave * (kShare ? deferred_wave_words(q) : slice_w);
  int8_t *tile_recv = reinterpret_cast<int8_t *>(words);
  int8_t *recv_row = tile_recv + lane * pitch;
  int8_t *send_row = recv_row + send_off;
  const uint64_t n_tiles = (prm.n_ranks + kWave - 1) / kWave;

  auto copy_out = [&](uint64_t row0, uint32_t n_valid) {
    if (prm.layout == kInterleaved) {
      tile_out<false, kShare>(words, prm.recv + row0 * 2u * q, n_valid * 2u * q, lane);
    } else if (prm.layout == kSeparate) {
      tile_out<false, kShare>(words, prm.recv + row0 * q, n_valid * q, lane);
      tile_out<false, kShare>(words + (kWave * q) / 4, prm.send + row0 * q, n_valid * q, lane);
    } else if (lane < n_valid) {
      int32_t *rr = prm.recv + (row0 + lane) * (uint64_t)prm.ld;
      int32_t *sr = prm.send + (row0 + lane) * (uint64_t)prm.ld;
      for (uint32_t k = 0; k < q; ++k) { rr[k] = recv_row[k]; sr[k] = send_row[k]; }
    }
  };

  uint64_t t_lo, t_hi;
  tile_run(prm.runs, t_lo, t_hi);
  LockstepCache record;
  const bool long_run = t_hi - t_lo >= 3u;     // recording costs more than it saves on two tiles
  const bool split_stretch = false;            // tables are bound by their stores or by latency: see kSplitRunTiles
  if (!kShare) {
    lockstep_cache_init(record, lds_dyn + kWavesPerBlock * slice_w + wave * kRecordWords, lane, split_stretch);
    for (uint64_t tile = t_lo; tile < t_hi; ++tile) {
      const TileState st = tile_rows<kMemo>(in, prm.r_begin, prm.n_ranks, tile, n_tiles, lds_dyn, slice_w,
                                            pitch, send_off, lane, wave, record, long_run, prm.table);
      copy_out(tile * kWave, st.n_valid);
      wave_lds_sync();                         // the slice is rewritten next
    }
    return;
  }

  int8_t *above = reinterpret_cast<int8_t *>(words + slice_w);          // [64][kAboveRounds]
  uint32_t *queue = words + slice_w + kAboveWords;
  lockstep_cache_init(record, words + slice_w + kAboveWords + kQueueWords, lane, split_stretch);
  const uint64_t run_row0 = t_lo * kWave;
  const uint32_t wave_id = blockIdx.x * kWavesPerBlock + wave;
  uint32_t seg_used = 0;                       // entries in this wavefront's segment of the open list
  uint32_t n_queued = 0;                       // the same in all lanes
  uint32_t n_valid_above = 0;                  // 0: no tile above in LDS yet
  for (uint64_t tile = t_hi; tile-- > t_lo;) {
    const uint64_t row0 = tile * kWave;
    const uint32_t n_valid = prm.n_ranks - row0 < kWave ? (uint32_t)(prm.n_ranks - row0) : kWave;
    uint32_t v = 0, viol = 0, flags = 0;
    int b = 0;
    MemoOut memo;
    memo.rho = 0; memo.room = 0;
    if (lane < n_valid) {
      v = virtual_rank(in, (uint32_t)(prm.r_begin + row0 + lane));
      viol = compute_rank_phase1<kMemo>(in, v, recv_row, send_row, b, flags,
                                        record, long_run && n_valid == (uint32_t)kWave, prm.table, memo);
    }
    wave_lds_sync();
    uint32_t open = 0;
    if (lane < n_valid) {
      open = resolve_from_tiles(in, viol, send_row, tile_recv, n_valid_above ? above : nullptr,
                                pitch, kAboveRounds, lane, n_valid, n_valid_above);
      if (kMemo) open = resolve_from_table(in, prm.table, v, memo, open, send_row);
    }
    // Open violations go into the queue as (row within the run) << 5 | k.  A tile can have more
    // of them than the queue has room for: then the rows leave first, a batch of 64 entries is
    // filled in (their rows are in the table by then), and the rest is queued after that.
    const uint32_t rel = (uint32_t)(row0 + lane - run_row0);   // < 2^27: see run_grid
    bool rows_out = false;
    for (;;) {
      while (n_queued < kDeferCap && __any(open != 0)) {
        const bool has = open != 0;
        const uint64_t who = __ballot(has);
        const uint32_t slot = n_queued + (uint32_t)__popcll(who & ((1ull << lane) - 1ull));
        if (has && slot < kDeferCap) {
          const uint32_t k = (uint32_t)(__ffs((int)open) - 1);
          open &= open - 1u;
          queue[slot] = (rel << 5) | k;
        }
        const uint32_t n_new = n_queued + (uint32_t)__popcll(who);
        n_queued = n_new < kDeferCap ? n_new : kDeferCap;
      }
      wave_lds_sync();
      if (!rows_out) {
        copy_out(row0, n_valid);
        if (lane < n_valid)
          for (uint32_t k = 0; k < q && k < kAboveRounds; ++k) above[lane * kAboveRounds + k] = recv_row[k];
        n_valid_above = n_valid;
        rows_out = true;
      }
      const bool more = __any(open != 0);
      while (n_queued >= (uint32_t)kWave || (more && n_queued != 0u)) {
        const uint32_t n_batch = n_queued < (uint32_t)kWave ? n_queued : (uint32_t)kWave;
        deferred_flush(in, prm, queue, run_row0, n_queued - n_batch, n_queued, lane, wave_id, seg_used);
        n_queued -= n_batch;
        if (more) break;                       // room again: queue the rest first
      }
      if (!more) break;
      wave_lds_sync();
    }
    wave_lds_sync();                           // slice and queue are rewritten next
  }
  // End of the run: fewer than 64 entries are waiting.  The four wavefronts of the workgroup own
  // neighbouring runs, and each still holds the receive rows of its lowest tile, which is the
  // tile above the next wavefront's run: after a barrier those rows answer what the first tile
  // of a run had to leave open, and the rest is pooled so that one search pass serves the
  // workgroup.  (Every wavefront gets here, also one with an empty run.)
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wavefront's rows are in the table
  __syncthreads();
  const uint32_t wave_words = deferred_wave_words(q);
  const bool have = lane < n_queued;
  const uint32_t item = have ? queue[lane] : 0u;
  bool waiting = have;
  if (have) {
    const uint32_t k = item & 31u;
    const uint64_t row = run_row0 + (item >> 5);
    const uint64_t target = row + skip_at_level(in.pm1, q - k);          // row of the to-processor
    for (uint32_t u = wave + 1u; u < (uint32_t)kWavesPerBlock; ++u) {
      uint32_t u_lo, u_tiles;
      run_of_wave(prm.runs, u, u_lo, u_tiles);
      const uint64_t first = (uint64_t)u_lo * kWave;
      if (k < kAboveRounds && u_tiles != 0u && target >= first && target < first + kWave && target < prm.n_ranks) {
        const int8_t *above_u =
            reinterpret_cast<const int8_t *>(lds_dyn + u * wave_words + slice_w);
        prm.send[row * (uint64_t)prm.ld + k] = above_u[(uint32_t)(target - first) * kAboveRounds + k];
        waiting = false;
      }
    }
  }
  const uint64_t who = __ballot(waiting);
  const uint32_t n_left = (uint32_t)__popcll(who);
  wave_lds_sync();                                   // every lane has read its entry
  if (waiting) queue[__popcll(who & ((1ull << lane) - 1ull))] = item;
  if (lane == 0) queue[kQueueWords - 1u] = n_left;   // free: fewer than 64 entries are queued
  __syncthreads();
  // entries of the four queues, in the order of the wavefronts: 64 to a wavefront
  static_assert(kWavesPerBlock == 4, "four queues are pooled");
  const uint32_t count_at = slice_w + kAboveWords + kQueueWords - 1u;
  const uint32_t end0 = lds_dyn[count_at];
  const uint32_t end1 = end0 + lds_dyn[wave_words + count_at];
  const uint32_t end2 = end1 + lds_dyn[2u * wave_words + count_at];
  const uint32_t end3 = end2 + lds_dyn[3u * wave_words + count_at];
  const uint32_t mine = wave * kWave + lane;         // all four queues together hold < 256
  const bool have_one = mine < end3;
  uint64_t row = 0;
  uint32_t k = 0;
  if (have_one) {
    const uint32_t u = (mine >= end0 ? 1u : 0u) + (mine >= end1 ? 1u : 0u) + (mine >= end2 ? 1u : 0u);
    const uint32_t start = u == 0u ? 0u : u == 1u ? end0 : u == 2u ? end1 : end2;
    const uint32_t entry = lds_dyn[u * wave_words + slice_w + kAboveWords + (mine - start)];
    uint32_t u_lo, u_tiles;
    run_of_wave(prm.runs, u, u_lo, u_tiles);
    row = (uint64_t)u_lo * kWave + (entry >> 5);
    k = entry & 31u;
  }
  const uint32_t first = wave * kWave;               // this wavefront's share of the pool
  const uint32_t n_mine = end3 > first ? (end3 - first < (uint32_t)kWave ? end3 - first : (uint32_t)kWave) : 0u;
  const bool handed_on = n_mine == 0u || publish_open(prm, wave_id, seg_used, n_mine, have_one, (row << 5) | k, lane);
  if (prm.open_segments != 0u && wave_id < prm.open_segments && lane == 0) prm.open_count[wave_id] = seg_used;
  if (handed_on) return;
  if (have_one) {
    const uint32_t v = virtual_rank(in, (uint32_t)(prm.r_begin + row));
    uint32_t fl = 0;
    prm.send[row * (uint64_t)prm.ld + k] = search_entry(in, to_processor(in, v, k), k, fl);
  }
}

// The entries k_schedules<true, .> left open, from the table itself: sendblock[k] of rank r is
// recvblock[k] of its to-processor (Condition 2), whose row the same launch has written if it
// is in the range of the call; if not, by a search as before.
__global__ __launch_bounds__(kBlock) void k_fill_open(SchedParams prm) {
  const Instance in = make_instance(prm.p, prm.q, prm.root);
  // One list: every claim that fit was written in full; the one claim that reached past the end of
  // the list marked its slots unused; later claims start beyond the end.  Segments: the first
  // open_count[w] entries of segment w.
  const uint32_t claimed = prm.open_segments != 0u ? 0u : *prm.open_count;
  const uint64_t n = prm.open_segments != 0u ? (uint64_t)prm.open_segments * prm.open_cap
                                             : (claimed < prm.open_cap ? claimed : prm.open_cap);
  for (uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (uint64_t)gridDim.x * kBlock) {
    if (prm.open_segments != 0u && (uint32_t)(i % prm.open_cap) >= prm.open_count[i / prm.open_cap]) continue;
    const unsigned long long item = prm.open_list[i];
    if (item == ~0ull) continue;                     // a slot no claim that fit covers
    const uint64_t row = item >> 5;
    const uint32_t k = (uint32_t)(item & 31u);
    const uint32_t v = virtual_rank(in, (uint32_t)(prm.r_begin + row));
    const uint32_t t = to_processor(in, v, k);       // virtual rank of the to-processor
    const uint64_t t_phys = (uint64_t)t + prm.root >= prm.p ? (uint64_t)t + prm.root - prm.p : (uint64_t)t + prm.root;
    int val;
    if (t_phys >= prm.r_begin && t_phys - prm.r_begin < prm.n_ranks) {
      val = prm.recv[(t_phys - prm.r_begin) * (uint64_t)prm.ld + k];
    } else {
      uint32_t fl = 0;
      val = search_entry(in, t, k, fl);
    }
    prm.send[row * (uint64_t)prm.ld + k] = val;
  }
}


// ------------------------------------------------------------------- digest

struct DigestParams {
  uint32_t p, q, root;
  uint64_t r_begin, n_ranks;
  RunSplit runs;
  uint64_t *digest;
  uint32_t *flags;
  // Row (of the launch) >> slot_shift is the place of a rank's hash and flags in digest[] and
  // flags[] (edge check: digest[2 slot], digest[2 slot + 1]); 63: one place for all ranks.
  uint32_t slot_shift;
  DeepTable table;                  // kernels with kMemo only
  // Ranks that k_digest<true, ...> leaves to k_digest_listed (row of the launch), or null: then the
  // kernel computes them again itself, 64 at a time.  rank_count: entries claimed so far (may run
  // past rank_cap).
  uint32_t *rank_list;
  uint32_t *rank_count;
  uint32_t rank_cap;
};
constexpr uint32_t kNoRank = 0xFFFFFFFFu;            // a slot of the list that no claim that fit covers

// (`count`, or null: the count of the list of ranks, cleared for the kernels that follow)
__global__ void k_digest_init(uint64_t *digest, uint32_t *flags, uint32_t *count, uint64_t n_slots) {
  const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n_slots) { digest[i] = 0; flags[i] = 0; }
  if (i == 0 && count) *count = 0;
}

__global__ void k_edges_init(uint64_t *xors, uint32_t *count) {
  if (threadIdx.x == 0 && blockIdx.x == 0) { xors[0] = 0; xors[1] = 0; if (count) *count = 0; }
}

// kEdges = false: digest and flags.  kEdges = true: the two XOR sums of the
// edge check go to prm.digest[0] and prm.digest[1]; flags are not touched.
//
// kShare (p with violations): runs of tiles from the top down with the rows of
// the tile above in LDS, as in k_schedules<true>.  A row can only be hashed
// when it is complete, so here whole rows are deferred: a rank that still has
// an open violation after the look into the two tiles is put into the queue
// (row within the run), and whenever 64 are waiting, and at the end of the run,
// each lane computes one such rank again from scratch, violations by search,
// and hashes it.  That is 2 to 3 ranks in 64; it costs the slice its rows, so
// the record of the top levels starts again after a batch.
template <bool kShare, bool kEdges, bool kMemo>
// (The kernels with deferred violations hold seven workgroups per CU at large q, where their LDS
// sets the limit, and are compiled for seven wavefronts per SIMD and more: with the registers of
// eight, or of six, they are 2-3 % slower.)
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(kShare ? 7 : 8, 8))) void k_digest(DigestParams prm) {
  extern __shared__ __align__(16) uint32_t lds_dyn[];
  const uint32_t lane = threadIdx.x & (kWave - 1);
  const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x / kWave));
  const Instance in = make_instance(prm.p, prm.q, prm.root);
  const uint32_t q = prm.q;
  const uint32_t pitch = digest_row_pitch(q);
  const uint32_t slice_w = digest_slice_words(q);
  uint32_t *words = lds_dyn + wave * (kShare ? digest_deferred_wave_words(q) : slice_w);
  int8_t *tile_recv = reinterpret_cast<int8_t *>(words);
  int8_t *recv_row = tile_recv + lane * pitch;
  int8_t *send_row = recv_row + q;
  const uint64_t n_tiles = (prm.n_ranks + kWave - 1) / kWave;

  // What the lanes have gathered for the ranks of output slot cur_slot (the same in all lanes)
  // goes out whenever the wavefront moves on to ranks of another slot, and at the end.
  uint64_t acc = 0, acc2 = 0;
  uint32_t acc_flags = 0;
  uint32_t cur_slot = 0;
  auto flush = [&]() {
    acc = wave_xor64(acc);
    if (kEdges) acc2 = wave_xor64(acc2);
    acc_flags = wave_or32(acc_flags);
    if (lane == 0) {
      if (kEdges) {
        atomicXor(reinterpret_cast<unsigned long long *>(prm.digest + 2u * (uint64_t)cur_slot), (unsigned long long)acc);
        atomicXor(reinterpret_cast<unsigned long long *>(prm.digest + 2u * (uint64_t)cur_slot + 1u), (unsigned long long)acc2);
      } else {
        atomicXor(reinterpret_cast<unsigned long long *>(prm.digest + cur_slot), (unsigned long long)acc);
        if (acc_flags) atomicOr(prm.flags + cur_slot, acc_flags);
      }
    }
    acc = 0; acc2 = 0; acc_flags = 0;
  };
  auto enter_slot = [&](uint32_t slot) {                     // slot: the same in all lanes
    if (slot != cur_slot) { flush(); cur_slot = slot; }
  };
  auto take_row = [&](uint32_t r, uint32_t v, int b) {       // the lane's row is complete
    if (kEdges) {
      edge_rank(in, r, recv_row, acc, acc2);
    } else {
      uint64_t h;
      uint32_t fl2;
      digest_rank(in, r, v, b, recv_row, h, fl2);
      acc ^= h;
      acc_flags |= fl2;
    }
  };
  uint64_t t_lo, t_hi;
  tile_run(prm.runs, t_lo, t_hi);
  LockstepCacheSplit record;
  const bool long_run = t_hi - t_lo >= 3u;
  const bool split_stretch = t_hi - t_lo >= kSplitRunTiles;
  if (!kShare) {
    lockstep_cache_init(record, lds_dyn + kWavesPerBlock * slice_w + wave * kRecordWords, lane, split_stretch);
    for (uint64_t tile = t_lo; tile < t_hi; ++tile) {
      const TileState st = tile_rows<kMemo>(in, prm.r_begin, prm.n_ranks, tile, n_tiles, lds_dyn, slice_w,
                                            pitch, q, lane, wave, record, long_run, prm.table);
      enter_slot((uint32_t)((tile * kWave) >> prm.slot_shift));
      acc_flags |= st.flags;
      if (lane < st.n_valid) take_row((uint32_t)(prm.r_begin + tile * kWave + lane), st.v, st.b);
      wave_lds_sync();                         // the slice is rewritten next
    }
  } else {
    int8_t *above = reinterpret_cast<int8_t *>(words + slice_w);          // [64][kAboveRounds]
    uint32_t *queue = words + slice_w + kAboveWords;
    lockstep_cache_init(record, words + slice_w + kAboveWords + kQueueWords, lane, split_stretch);
    const uint64_t run_row0 = t_lo * kWave;
    uint32_t n_queued = 0;                     // the same in all lanes; at most 63 between tiles
    uint32_t n_valid_above = 0;
    uint64_t tile = t_hi;
    // One pass of the loop is either the next tile of the run or a batch of deferred ranks
    // (64 of them, or what is left once the tiles are done), one rank per lane in both cases.
    for (;;) {
      const bool batch = n_queued >= (uint32_t)kWave || (tile == t_lo && n_queued != 0u);
      if (batch && prm.rank_list != nullptr) {
        // With a list at hand the ranks that are waiting go there (one atomic for up to 64 of them)
        // and a second kernel computes them, which it does several times faster than a pass of
        // this loop: there every wavefront works on such ranks and nothing else.
        const uint32_t n_out = n_queued < (uint32_t)kWave ? n_queued : (uint32_t)kWave;
        uint32_t base = 0;
        if (lane == 0) base = atomicAdd(prm.rank_count, n_out);
        base = lane0_of(base);
        if (base < prm.rank_cap && n_out <= prm.rank_cap - base) {
          if (lane < n_out) prm.rank_list[base + lane] = (uint32_t)(run_row0 + queue[n_queued - n_out + lane]);
          n_queued -= n_out;
          wave_lds_sync();                     // the queue is written again below
          continue;
        }
        // the list is full: what this claim still covers is marked unused, the ranks stay here
        if (base < prm.rank_cap && base + lane < prm.rank_cap) prm.rank_list[base + lane] = kNoRank;
      }
      if (!batch && tile == t_lo) break;
      uint64_t row = 0;                        // the lane's rank, as a row of the launch
      uint64_t row0_of_pass = 0;               // first row of the tile, if the pass is a tile
      uint32_t n_here;                         // lanes with a rank in this pass
      if (batch) {
        n_here = n_queued < (uint32_t)kWave ? n_queued : (uint32_t)kWave;
        if (lane < n_here) row = run_row0 + queue[n_queued - n_here + lane];
      } else {
        --tile;
        const uint64_t row0 = tile * kWave;
        n_here = prm.n_ranks - row0 < kWave ? (uint32_t)(prm.n_ranks - row0) : kWave;
        row = row0 + lane;
        row0_of_pass = row0;
      }
      const uint32_t r = (uint32_t)(prm.r_begin + row);
      uint32_t v = 0, viol = 0, flags = 0;
      int b = 0;
      MemoOut memo;
      memo.rho = 0; memo.room = 0;
      if (lane < n_here) {
        v = virtual_rank(in, r);
        viol = compute_rank_phase1<kMemo>(in, v, recv_row, send_row, b, flags, record,
                                          !batch && long_run && n_here == (uint32_t)kWave, prm.table, memo);
      }
      wave_lds_sync();
      uint32_t open = 0;
      if (lane < n_here) {
        if (batch) {                           // no neighbours here: from the table, else by search
          const uint32_t left = kMemo ? resolve_from_table(in, prm.table, v, memo, viol, send_row) : viol;
          flags |= resolve_by_search(in, v, left, send_row);
        } else {
          open = resolve_from_tiles(in, viol, send_row, tile_recv, n_valid_above ? above : nullptr,
                                    pitch, kAboveRounds, lane, n_here, n_valid_above);
          if (kMemo) open = resolve_from_table(in, prm.table, v, memo, open, send_row);
        }
      }
      if (!batch) {                            // a tile lies in one slot
        enter_slot((uint32_t)(row0_of_pass >> prm.slot_shift));
        acc_flags |= flags;
        if (lane < n_here && open == 0) take_row(r, v, b);
      } else {                                 // ranks from anywhere in the run: slot by slot
        const uint32_t my_slot = (uint32_t)(row >> prm.slot_shift);
        bool todo = lane < n_here;
        for (uint64_t who = __ballot(todo); who != 0; who = __ballot(todo)) {
          const uint32_t slot = (uint32_t)__builtin_amdgcn_readlane((int)my_slot, __ffsll((long long)who) - 1);
          enter_slot(slot);
          if (todo && my_slot == slot) {
            acc_flags |= flags;
            take_row(r, v, b);
            todo = false;
          }
        }
      }
      if (batch) {
        n_queued -= n_here;
        lockstep_cache_rows_lost(record);      // the rows of the last tile are gone
      } else {
        const uint64_t who = __ballot(open != 0);
        const uint32_t slot = n_queued + (uint32_t)__popcll(who & ((1ull << lane) - 1ull));
        if (open != 0) {
          if (slot < kRowQueueCap) queue[slot] = (uint32_t)(row - run_row0);
          else acc_flags |= BCAST_F_SEARCH;    // cannot happen: at most 63 + 64 entries
        }
        const uint32_t n_new = n_queued + (uint32_t)__popcll(who);
        n_queued = n_new < kRowQueueCap ? n_new : kRowQueueCap;
        if (lane < n_here)
          for (uint32_t k = 0; k < q && k < kAboveRounds; ++k) above[lane * kAboveRounds + k] = recv_row[k];
        n_valid_above = n_here;
      }
      wave_lds_sync();                         // slice and queue are rewritten next
    }
  }
  flush();
}

// The ranks that k_digest<true, ...> put on the list: each lane computes one of them on its own
// (no neighbours, no records: the branch-free search throughout, as for lists of arbitrary
// ranks), violations by search, and adds its hash, or its edges, to the launch's result.  (Taking
// the deep levels and the violations from the table of deep entries here as well, the latter
// through the to-processor's own rho, was measured and is not faster: the lanes of this kernel
// are a third busy whichever way, and it takes a tenth of the call.)
__global__ __launch_bounds__(kBlock) void k_digest_listed(DigestParams prm) {
  extern __shared__ __align__(16) uint32_t lds_dyn[];
  const uint32_t lane = threadIdx.x & (kWave - 1);
  const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x / kWave));
  const Instance in = make_instance(prm.p, prm.q, prm.root);
  const uint32_t q = prm.q;
  const uint32_t pitch = digest_row_pitch(q);
  int8_t *recv_row = reinterpret_cast<int8_t *>(lds_dyn + wave * digest_slice_words(q)) + lane * pitch;
  int8_t *send_row = recv_row + q;
  // every claim that fit was written in full; the one claim that reached past the end of the
  // list marked its slots unused; later claims start beyond the end
  const uint32_t claimed = *prm.rank_count;
  const uint32_t n = claimed < prm.rank_cap ? claimed : prm.rank_cap;
  uint64_t acc = 0;
  uint32_t acc_flags = 0;
  uint32_t cur_slot = 0;                       // as in k_digest
  auto flush = [&]() {
    acc = wave_xor64(acc);
    acc_flags = wave_or32(acc_flags);
    if (lane == 0 && (acc != 0 || acc_flags != 0)) {
      atomicXor(reinterpret_cast<unsigned long long *>(prm.digest + cur_slot), (unsigned long long)acc);
      if (acc_flags) atomicOr(prm.flags + cur_slot, acc_flags);
    }
    acc = 0; acc_flags = 0;
  };
  const uint32_t n_waves = gridDim.x * kWavesPerBlock;
  for (uint32_t i0 = (blockIdx.x * kWavesPerBlock + wave) * kWave; i0 < n; i0 += n_waves * kWave) {
    const uint32_t row = i0 + lane < n ? prm.rank_list[i0 + lane] : kNoRank;
    uint64_t h = 0;
    uint32_t fl_row = 0;
    if (row != kNoRank) {
      const uint32_t r = (uint32_t)(prm.r_begin + row);
      const uint32_t v = virtual_rank(in, r);
      LockstepCache none;
      lockstep_cache_init(none, nullptr);
      DeepTable no_table;
      no_table.entries = nullptr; no_table.viol_by_e = nullptr; no_table.first_deep = 0; no_table.n_rho = 0;
      MemoOut unused;
      int b = 0;
      uint32_t flags = 0;
      const uint32_t viol = compute_rank_phase1<false, true>(in, v, recv_row, send_row, b, flags, none, false,
                                                             no_table, unused);
      flags |= resolve_by_search<true>(in, v, viol, send_row);
      uint32_t fl2;
      digest_rank(in, r, v, b, recv_row, h, fl2);
      fl_row = flags | fl2;
    }
    // the listed ranks come from anywhere in the range: slot by slot
    const uint32_t my_slot = row != kNoRank ? (uint32_t)((uint64_t)row >> prm.slot_shift) : 0u;
    bool todo = row != kNoRank;
    for (uint64_t who = __ballot(todo); who != 0; who = __ballot(todo)) {
      const uint32_t slot = (uint32_t)__builtin_amdgcn_readlane((int)my_slot, __ffsll((long long)who) - 1);
      if (slot != cur_slot) { flush(); cur_slot = slot; }
      if (todo && my_slot == slot) {
        acc ^= h;
        acc_flags |= fl_row;
        todo = false;
      }
    }
  }
  flush();
}

// ------------------------------------------------- table of deep entries

// One lane per rho for the entries (the first blocks_per_row workgroups), then one lane per
// (S - e, rho) for the second table (see DeepTable in the device header).
// `counter` (or null): a word to clear for the kernel that follows (the count of open entries), which
// saves that kernel a launch of its own.
__global__ __launch_bounds__(kBlock) void k_deep_table(uint4 *entries, uint16_t *viol_by_e, uint32_t p,
                                                       uint32_t q, uint32_t first_deep, uint32_t n_rho,
                                                       uint32_t blocks_per_row, uint32_t *counter) {
  if (counter != nullptr && blockIdx.x == 0 && threadIdx.x == 0) *counter = 0;
  const uint32_t row = blockIdx.x / blocks_per_row;            // 0: entries; 1 .. kDeepEs - 1: S - e
  const uint32_t rho = (blockIdx.x - row * blocks_per_row) * kBlock + threadIdx.x;
  if (rho >= n_rho) return;
  if (row == 0u) entries[rho] = deep_entry_build(p - 1u, q, first_deep, rho);
  else viol_by_e[row * kDeepMaxEntries + rho] = deep_viol_build(p - 1u, q, first_deep, rho, row);
}

// ----------------------------------------------------------------- doubling

struct DoubleParams {
  uint32_t p, q;                 // the given instance; the result has 2p ranks and q + 1 rounds
  const int32_t *in;             // [p][2q]
  int32_t *out;                  // [2p][2(q+1)]
};

// Observations 1 and 5: the schedules for 2p processors from those for p
// (root 0).  Rank r < p and rank r + p both start from row r: negative entries
// drop by one (q grows by one), and a new last round is added.
//   receive, r < p: the new entry is -1.  r = p: it is the new block q.
//            r > p: the row's one non-negative block b moves to the new round
//            and leaves -1 behind.
//   send,    r < p: the new entry is the rank's baseblock (q for the root).
//            r >= p: every non-negative entry becomes -1, so does the new one.
// A wavefront reads 64 rows once (as bytes into LDS), each lane rewrites its
// row twice, and both tiles leave as 16-byte stores: 8q bytes read and 16(q+1)
// bytes written per given rank, nothing else.
__global__ __launch_bounds__(kBlock) void k_double(DoubleParams prm) {
  extern __shared__ __align__(16) uint32_t lds_dyn[];
  const uint32_t lane = threadIdx.x & (kWave - 1);
  const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x / kWave));
  const uint32_t q = prm.q, q2 = q + 1u;
  const uint32_t in_w = slice_words(q), out_w = slice_words(q2);
  uint32_t *w_in = lds_dyn + wave * (in_w + 2u * out_w);
  uint32_t *w_lo = w_in + in_w, *w_hi = w_lo + out_w;
  const uint64_t n_tiles = ((uint64_t)prm.p + kWave - 1) / kWave;
  for (uint64_t tile = (uint64_t)blockIdx.x * kWavesPerBlock + wave; tile < n_tiles;
       tile += (uint64_t)gridDim.x * kWavesPerBlock) {
    const uint64_t row0 = tile * kWave;
    const uint32_t n_valid = prm.p - row0 < kWave ? (uint32_t)(prm.p - row0) : kWave;
    // the tile is contiguous in memory: n_valid * 2q int32, four to a lane
    const uint32_t n_in = n_valid * 2u * q;
    const int32_t *src = prm.in + row0 * 2u * q;
    int8_t *b_in = reinterpret_cast<int8_t *>(w_in);
    if ((reinterpret_cast<uintptr_t>(src) & 15u) == 0) {
      const int4 *src4 = reinterpret_cast<const int4 *>(src);
      for (uint32_t g = lane; g < (n_in >> 2); g += kWave) {
        const int4 x = src4[g];
        w_in[g] = ((uint32_t)x.x & 0xFFu) | (((uint32_t)x.y & 0xFFu) << 8) |
                  (((uint32_t)x.z & 0xFFu) << 16) | ((uint32_t)x.w << 24);
      }
      for (uint32_t i = (n_in & ~3u) + lane; i < n_in; i += kWave) b_in[i] = (int8_t)src[i];
    } else {
      for (uint32_t i = lane; i < n_in; i += kWave) b_in[i] = (int8_t)src[i];
    }
    wave_lds_sync();
    if (lane < n_valid) {
      const int8_t *row = b_in + lane * 2u * q;
      int8_t *lo = reinterpret_cast<int8_t *>(w_lo) + lane * 2u * q2;   // rank r
      int8_t *hi = reinterpret_cast<int8_t *>(w_hi) + lane * 2u * q2;   // rank r + p
      const bool is_root = row0 + lane == 0;
      int b = (int)q;                                   // baseblock: the non-negative receive entry
      for (uint32_t k = 0; k < q; ++k) {
        const int rv = row[k];
        b = rv >= 0 ? rv : b;
        lo[k] = (int8_t)(rv < 0 ? rv - 1 : rv);
        hi[k] = (int8_t)(rv < 0 ? rv - 1 : -1);
      }
      lo[q] = (int8_t)-1;
      hi[q] = (int8_t)b;                                // the root's copy receives the new block q
      for (uint32_t k = 0; k < q; ++k) {
        const int sv = row[q + k];
        lo[q2 + k] = (int8_t)(sv < 0 ? sv - 1 : sv);
        hi[q2 + k] = (int8_t)(sv < 0 ? sv - 1 : -1);
      }
      lo[q2 + q] = (int8_t)(is_root ? (int)q : b);
      hi[q2 + q] = (int8_t)-1;
    }
    wave_lds_sync();
    tile_out<false>(w_lo, prm.out + row0 * 2u * q2, n_valid * 2u * q2, lane);
    tile_out<false>(w_hi, prm.out + ((uint64_t)prm.p + row0) * 2u * q2, n_valid * 2u * q2, lane);
    wave_lds_sync();
  }
}

// ------------------------------------------------- baseblocks in linear time

// One step of the listing in the proof of Lemma 4: the baseblocks of the first skip[k] ranks are
// known; those of the ranks skip[k] .. skip[k+1]-1 are a copy of the first skip[k+1] - skip[k]
// of them (rank skip[k] takes the root's old entry k), and the root's entry becomes k + 1.
// `done` = skip[k], `upto` = skip[k+1] <= 2 done: source and destination never overlap.
__global__ __launch_bounds__(kBlock) void k_listing_step(uint8_t *list, uint32_t done, uint32_t upto) {
  const uint64_t n = (uint64_t)upto - done;                  // bytes to copy from list[0..n) to list[done..upto)
  const uint64_t stride = (uint64_t)gridDim.x * kBlock;
  const uint64_t tid = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
  // Destination in 16-byte groups from its first 16-byte boundary on; the source of a group
  // starts at any byte: five aligned words, shifted into place.  Ends by single bytes.
  const uintptr_t dst0 = reinterpret_cast<uintptr_t>(list) + done;
  uint64_t head = (16u - (dst0 & 15u)) & 15u;
  head = head < n ? head : n;
  const uint64_t n16 = (reinterpret_cast<uintptr_t>(list) & 3u) == 0u ? (n - head) / 16u : 0u;
  const uint32_t *words = reinterpret_cast<const uint32_t *>(list);
  uint4 *dst = reinterpret_cast<uint4 *>(list + done + head);
  for (uint64_t g = tid; g < n16; g += stride) {
    const uint64_t src = head + 16u * g;                     // byte offset of the group's source
    const uint64_t w = src >> 2;
    const uint32_t sh = (uint32_t)(src & 3u);
    // src + 16 <= n <= done: the bytes that are used all lie in list[0 .. n); the fifth word may
    // reach up to byte done + 2 < upto (allocated; what it holds beyond byte n is shifted out)
    const uint32_t a = words[w], b = words[w + 1], c = words[w + 2], d = words[w + 3];
    uint4 o;
    if (sh == 0u) {
      o.x = a; o.y = b; o.z = c; o.w = d;
    } else {
      const uint32_t e = words[w + 4];
      o.x = __builtin_amdgcn_alignbyte(b, a, sh);
      o.y = __builtin_amdgcn_alignbyte(c, b, sh);
      o.z = __builtin_amdgcn_alignbyte(d, c, sh);
      o.w = __builtin_amdgcn_alignbyte(e, d, sh);
    }
    dst[g] = o;
  }
  for (uint64_t b = tid; b < head; b += stride) list[done + b] = list[b];
  for (uint64_t b = head + n16 * 16u + tid; b < n; b += stride) list[done + b] = list[b];
}

__global__ void k_listing_root(uint8_t *list, uint32_t entry) {
  if (blockIdx.x == 0 && threadIdx.x == 0) list[0] = (uint8_t)entry;
}

// ------------------------------------------------------------------ batched

struct BatchParams {
  uint32_t n_inst, m, tiles_per_inst;
  const uint32_t *p, *root, *ranks;
  const uint64_t *row_off;
  int32_t *out;
  uint64_t out_elems;
  uint32_t *n_rejected;
};

__global__ void k_u32_zero(uint32_t *x) {
  if (threadIdx.x == 0 && blockIdx.x == 0) *x = 0;
}

// The ranks of a tile are arbitrary ranks of one instance, so a violation of Algorithm 6 has no
// neighbour's row to look at: every one takes a search of its own (search_entry: the levels from
// the top down, then the ascent until round k is out).  Searching where they arise would mean up
// to four searches in a row with the few lanes that have a first, second, ... violation; instead
// a tile's violations are collected (owner lane and round, 2 bytes each) and searched 64 at a
// time, one per lane.  Such a pass runs as long as its longest search: two moves for a violation
// in round 1, the most common one, and twenty and more for one in round 10.  So only the
// violations in rounds below kShortRounds, five in six, are searched with their tile, and
// answered in the tile's rows in LDS before these leave.  The others leave open: a wavefront
// takes kBatchTiles tiles of one instance in a row and queues them (row within the batch << 5 |
// round); whenever 64 are waiting, and at the end of the batch, they are searched and each
// answer goes to its place in the caller's table.  (All violations through that queue: fewer
// instructions and slower, because every answer and every owner's rank read again is a memory
// transaction of its own, and there are 0.8 violations per rank.)
constexpr uint32_t kBatchTiles = 16;
constexpr uint32_t kShortRounds = 4;
constexpr uint32_t kLongQueue = 2 * kWave;      // 63 waiting + one more from every lane

struct BatchLds {
  uint32_t *rows;                   // kTileBytes of the wavefront's own
  uint16_t *open_entry;             // kShortRounds * kWave: lane << 5 | k, one per rank and round below kShortRounds
  uint32_t *open_v;                 // kWave: the owner's virtual rank
  uint16_t *waiting;                // kLongQueue
};

// Tiles tile0 .. tile1 - 1 (at most kBatchTiles) of instance `inst`, whose rows begin at off0.
__device__ __forceinline__ void batch_tiles(const BatchParams &prm, const Instance &in, uint32_t inst,
                                            uint64_t off0, uint32_t tile0, uint32_t tile1,
                                            const BatchLds &mem, uint32_t lane) {
  const uint32_t p = in.p, q = in.q;
  const uint64_t below = (1ull << lane) - 1ull;
  const uint32_t *batch_ranks = prm.ranks + (uint64_t)inst * prm.m + (uint64_t)tile0 * kWave;
  int32_t *batch_out = prm.out + off0 + (uint64_t)tile0 * kWave * 2u * q;
  int8_t *recv_row = reinterpret_cast<int8_t *>(mem.rows) + lane * 2u * q;
  int8_t *send_row = recv_row + q;
  // Entries first .. first + count - 1 of the queue, one per lane: the owner's rank is read
  // again, the answer goes to the owner's row in the caller's table.  That row was stored by
  // other lanes of this wavefront; the wait lets those stores arrive before the entry is written.
  auto search_waiting = [&](uint32_t first, uint32_t count) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    if (lane < count) {
      const uint32_t item = mem.waiting[first + lane];
      const uint32_t row = item >> 5, k = item & 31u;
      const uint32_t v = virtual_rank(in, batch_ranks[row]);
      uint32_t fl = 0;
      batch_out[(uint64_t)row * 2u * q + q + k] = search_entry<true>(in, to_processor(in, v, k), k, fl);
    }
    wave_lds_sync();
  };
  uint32_t n_waiting = 0;                          // the same in all lanes
  for (uint32_t tile = tile0; tile < tile1; ++tile) {
    const uint32_t j0 = tile * kWave;
    const uint32_t n_valid = prm.m - j0 < (uint32_t)kWave ? prm.m - j0 : (uint32_t)kWave;
    uint32_t early = 0, late = 0;        // violations searched with the tile, and left to the queue
    if (lane < n_valid) {
      const uint32_t r = batch_ranks[j0 - tile0 * kWave + lane];
      if (r < p) {
        int b;
        uint32_t flags;
        LockstepCache none;
        lockstep_cache_init(none, nullptr);
        const uint32_t v = virtual_rank(in, r);
        mem.open_v[lane] = v;
        DeepTable no_table;
        no_table.entries = nullptr; no_table.viol_by_e = nullptr; no_table.first_deep = 0; no_table.n_rho = 0;
        MemoOut unused;
        const uint32_t viol = compute_rank_phase1<false, true>(in, v, recv_row, send_row, b, flags, none,
                                                               false, no_table, unused);
        early = viol & ((1u << kShortRounds) - 1u);
        late = viol & ~((1u << kShortRounds) - 1u);
      } else {                           // rank outside the instance: marked row
        for (uint32_t k = 0; k < 2u * q; ++k) recv_row[k] = (int8_t)kInvalidByte;
        if (prm.n_rejected) atomicAdd(prm.n_rejected, 1u);
      }
    }
    uint32_t n_open = 0;                 // the same in all lanes
    while (__any(early != 0)) {          // one more from every lane that has one
      const bool has = early != 0;
      const uint64_t who = __ballot(has);
      if (has) {
        mem.open_entry[n_open + (uint32_t)__popcll(who & below)] =
            (uint16_t)((lane << 5) | (uint32_t)(__ffs((int)early) - 1));
        early &= early - 1u;
      }
      n_open += (uint32_t)__popcll(who);
    }
    wave_lds_sync();
    for (uint32_t e = lane; e < n_open; e += kWave) {
      const uint32_t item = mem.open_entry[e];
      const uint32_t owner = item >> 5, k = item & 31u;
      uint32_t fl = 0;
      const int val = search_entry<true>(in, to_processor(in, mem.open_v[owner], k), k, fl);
      reinterpret_cast<int8_t *>(mem.rows)[owner * 2u * q + q + k] = (int8_t)val;
    }
    wave_lds_sync();
    tile_out<true>(mem.rows, prm.out + off0 + (uint64_t)j0 * 2u * q, n_valid * 2u * q, lane);
    while (__any(late != 0)) {
      const bool has = late != 0;
      const uint64_t who = __ballot(has);
      if (has) {
        mem.waiting[n_waiting + (uint32_t)__popcll(who & below)] =
            (uint16_t)((((tile - tile0) * kWave + lane) << 5) | (uint32_t)(__ffs((int)late) - 1));
        late &= late - 1u;
      }
      n_waiting += (uint32_t)__popcll(who);
      wave_lds_sync();
      if (n_waiting >= (uint32_t)kWave) { n_waiting -= kWave; search_waiting(n_waiting, kWave); }
    }
    wave_lds_sync();                     // the rows are rewritten next
  }
  if (n_waiting != 0) search_waiting(0, n_waiting);
}

// What the kernel can check of instance `inst` (the host sees none of it): false = it writes nothing.
__device__ __forceinline__ bool batch_instance(const BatchParams &prm, uint32_t inst, Instance &in,
                                               uint64_t &off0) {
  const uint32_t p = prm.p[inst];
  const uint32_t root = prm.root[inst];
  const uint32_t q = p > 1u ? 32u - (uint32_t)__clz((int)(p - 1u)) : 0u;
  off0 = prm.row_off[inst];
  const uint64_t off1 = prm.row_off[inst + 1];
  in = make_instance(p, q, root);
  return p >= 1u && p <= BCAST_MAX_P && root < p && off1 >= off0 &&
         off1 - off0 == (uint64_t)prm.m * 2u * q && off1 <= prm.out_elems;
}

__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(8, 8))) void k_batched(BatchParams prm) {
  __shared__ __align__(16) uint32_t lds[kWavesPerBlock][kTileBytes / 4];
  __shared__ uint16_t open_entry[kWavesPerBlock][kShortRounds * kWave];
  __shared__ uint32_t open_v[kWavesPerBlock][kWave];
  __shared__ uint16_t waiting[kWavesPerBlock][kLongQueue];
  const uint32_t lane = threadIdx.x & (kWave - 1);
  const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x / kWave));
  const BatchLds mem = {lds[wave], open_entry[wave], open_v[wave], waiting[wave]};
  const uint32_t batches_per_inst = (prm.tiles_per_inst + kBatchTiles - 1u) / kBatchTiles;
  const uint64_t n_work = (uint64_t)prm.n_inst * batches_per_inst;
  for (uint64_t work = (uint64_t)blockIdx.x * kWavesPerBlock + wave; work < n_work;
       work += (uint64_t)gridDim.x * kWavesPerBlock) {
    const uint32_t inst = (uint32_t)(work / batches_per_inst);
    const uint32_t batch = (uint32_t)(work % batches_per_inst);
    Instance in;
    uint64_t off0;
    if (!batch_instance(prm, inst, in, off0)) {
      if (batch == 0 && lane == 0 && prm.n_rejected) atomicAdd(prm.n_rejected, 1u);
      continue;
    }
    const uint32_t tile0 = batch * kBatchTiles;
    const uint32_t tile1 = prm.tiles_per_inst - tile0 < kBatchTiles ? prm.tiles_per_inst : tile0 + kBatchTiles;
    batch_tiles(prm, in, inst, off0, tile0, tile1, mem, lane);
  }
}

// ---------------------------------------------------------------- simulator

constexpr int kSimBlock = 128;

struct SimParams {
  uint32_t p, q, n, n_words, x;
  uint32_t rounds;
  const uint32_t *roots;         // device copy inside the workspace
  const int32_t *sched;          // [n_roots][p][2q] physical, or NULL
  const int32_t *table;          // [2q][p]: entry by virtual rank (when sched == NULL)
  uint32_t *possession;          // [n_roots][n_words][p]
  bcast_verdict *verdict;
};

// [p][c] -> [c][p], 64 rows to a wavefront: the replay reads the table it computes itself by
// columns, so that the 64 processors of a wavefront read 64 consecutive words.
__global__ __launch_bounds__(kWave) void k_rows_to_columns(const int32_t *in, int32_t *out,
                                                           uint32_t p, uint32_t c) {
  extern __shared__ __align__(16) uint32_t lds_dyn[];
  const uint32_t lane = threadIdx.x;
  const uint64_t row0 = (uint64_t)blockIdx.x * kWave;
  const uint32_t rows = p - row0 < kWave ? (uint32_t)(p - row0) : kWave;
  const uint32_t pitch = c | 1u;                              // odd: no bank conflicts by column
  const int32_t *src = in + row0 * c;
  for (uint32_t i = lane; i < rows * c; i += kWave) lds_dyn[(i / c) * pitch + i % c] = (uint32_t)src[i];
  wave_lds_sync();
  if (lane < rows)
    for (uint32_t k = 0; k < c; ++k) out[(uint64_t)k * p + row0 + lane] = (int32_t)lds_dyn[lane * pitch + k];
}

// The roots reach the device as kernel arguments, kRootBatch at a time: no copy from the
// caller's host array is left pending when the call returns, and nothing waits.
constexpr uint32_t kRootBatch = 256;
struct RootBatch {
  uint32_t first, count;
  uint32_t root[kRootBatch];
};

__global__ __launch_bounds__(kRootBatch) void k_store_roots(uint32_t *dst, RootBatch b) {
  if (threadIdx.x < b.count) dst[b.first + threadIdx.x] = b.root[threadIdx.x];
}

__global__ void k_verdict_init(bcast_verdict *vd, uint32_t n_roots, uint32_t rounds) {
  const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n_roots) {
    bcast_verdict z;
    z.flags = 0; z.rounds = rounds;
    z.n_bad_recv_dup = 0; z.n_bad_send_unheld = 0; z.n_edge_mismatch = 0;
    z.n_incomplete_ranks = 0; z.first_bad = UINT64_MAX;
    vd[i] = z;
  }
}

// One lane per processor, one grid row per root.  A processor's possession
// bits are written by its own lane only, and everything it needs from other
// processors is schedule data, so the lane walks through all rounds by itself:
// the sender-side check ("held before the round") reads the lane's own word
// before this round's receive is marked.
//
// kReverse: the reduction to the root, i.e. the same rounds from the last one
// down with all communication reversed.  The bits then mean "partial result
// already sent on"; a lane first marks the block it sends (its receive entry),
// then checks that what arrives (its send entry) is for a block it still has.
//
// Block numbers fit 32 bits with room to spare (n <= BCAST_MAX_N = 2^28).  Entries, which may be
// any int32, are clamped to [-C, C], C = n + 2q + 2, while staging: the adjustment
// q * floor(i / q) - x stays within [-q, n + q], so an entry of C or more is a block >= n - 1 in
// every round (it counts as n - 1) and one of -C or less is never a block.
//
// kPacked (C < 2^15, i.e. n below about 32,700): a round's two clamped entries share one LDS word
// as 16-bit halves: one LDS read per round instead of two, and half the LDS per workgroup, which
// is what limits the wavefronts per SIMD here.
template <bool kReverse, bool kPacked>
__global__ __launch_bounds__(kSimBlock) void k_simulate(SimParams prm) {
  using Blk = int32_t;
  // two [q][kSimBlock] arrays (one when packed), sized at launch: the lane's recvblock and
  // sendblock.  What the from-processor sends (its sendblock[k]) is compared with the lane's
  // recvblock[k] once, while staging; only rounds whose entries differ look it up again
  // (`differs`, bit k).
  extern __shared__ __align__(16) uint32_t lds_dyn[];
  typedef int32_t (*Staged)[kSimBlock];
  Staged st_recv = reinterpret_cast<Staged>(lds_dyn);
  Staged st_send = st_recv + (kPacked ? 0u : prm.q);
  const uint32_t lane_b = threadIdx.x;
  const uint32_t lane = threadIdx.x & (kWave - 1);
  const uint32_t root_idx = blockIdx.y;
  const uint32_t p = prm.p, q = prm.q, n = prm.n;
  const uint32_t pm1 = p - 1u;
  const uint32_t root = prm.roots[root_idx];
  const uint32_t v = blockIdx.x * kSimBlock + lane_b;
  const bool active = v < p;
  const uint32_t r_phys = active ? (v + root >= p ? v + root - p : v + root) : 0u;

  // per lane: counts fit 32 bits (at most one of each kind per round, rounds < 2^29), and the
  // first bad round is kept as a round number; the 64-bit forms are made at the end
  uint32_t c_dup = 0, c_unheld = 0, c_edge = 0, bad_round = 0xFFFFFFFFu;
  uint64_t n_incomplete = 0, first_bad = UINT64_MAX;

  const int32_t clamp_at = (int32_t)(n + 2u * q + 2u);
  auto staged = [&](int32_t x) -> int32_t {
    return x > clamp_at ? clamp_at : (x < -clamp_at ? -clamp_at : x);
  };
  if (prm.sched) {
    // A caller's table has rows by physical rank.  The workgroup's 128 consecutive virtual ranks
    // are consecutive physical ranks (starting at the root's offset, wrapping at p), so their
    // rows form one block of memory (two at the wrap): it is read in memory order, 128
    // consecutive words at a time, and each word goes to its place [column][processor] in LDS.
    const uint32_t c = 2u * q;
    const uint32_t v0 = blockIdx.x * kSimBlock;
    const uint32_t rows = p - v0 < (uint32_t)kSimBlock ? p - v0 : (uint32_t)kSimBlock;
    const uint32_t row_step = (uint32_t)kSimBlock / c, col_step = (uint32_t)kSimBlock % c;
    uint32_t row = lane_b / c, col = lane_b % c;
    while (row < rows) {
      const uint32_t u = v0 + row;
      const uint32_t u_phys = u + root >= p ? u + root - p : u + root;
      const int32_t val = staged(prm.sched[((uint64_t)root_idx * p + u_phys) * c + col]);
      if (kPacked) {
        const uint32_t k = col < q ? col : col - q;
        reinterpret_cast<uint16_t *>(lds_dyn)[(k * kSimBlock + row) * 2u + (col < q ? 0u : 1u)] =
            (uint16_t)val;
      } else {
        st_recv[col][row] = val;                   // st_send = st_recv + q
      }
      row += row_step;
      col += col_step;
      if (col >= c) { col -= c; ++row; }
    }
    __syncthreads();
  }

  if (active) {
    // entry c (recvblock[c] for c < q, sendblock[c - q] above) of virtual rank u: the table
    // computed in the call has columns by virtual rank
    auto entry = [&](uint32_t u, uint32_t c) -> int32_t {
      if (prm.sched) {
        const uint32_t u_phys = u + root >= p ? u + root - p : u + root;
        return prm.sched[((uint64_t)root_idx * p + u_phys) * 2u * q + c];
      }
      return prm.table[(uint64_t)c * p + u];
    };
    auto from_entry = [&](uint32_t k) -> int32_t {         // sendblock[k] of the from-processor
      const uint32_t sk = skip_at_level(pm1, q - k);
      return entry(v >= sk ? v - sk : v + (p - sk), q + k);
    };
    // `differs` compares clamped entries: two entries that clamp to the same value are equal, or
    // are both the block n - 1 in every round, or are both never a block
    uint32_t differs = 0;
    for (uint32_t k = 0; k < q; ++k) {
      int32_t mine, out;                           // clamped
      if (prm.sched) {
        if (kPacked) {
          const int32_t both = st_recv[k][lane_b];
          mine = (int32_t)(int16_t)(both & 0xFFFF);
          out = both >> 16;
        } else {
          mine = st_recv[k][lane_b];
          out = st_send[k][lane_b];
        }
      } else {
        mine = staged(entry(v, k));
        out = staged(entry(v, q + k));
      }
      // nothing is sent to the root: in the rounds whose to-processor is the root the send
      // entry is staged as "never a block"
      const bool to_root = v + skip_at_level(pm1, q - k) == p;
      out = to_root ? -clamp_at : out;
      if (kPacked) {
        st_recv[k][lane_b] = (int32_t)(((uint32_t)mine & 0xFFFFu) | ((uint32_t)out << 16));
      } else {
        st_recv[k][lane_b] = mine;
        st_send[k][lane_b] = out;
      }
      differs |= (uint32_t)(staged(from_entry(k)) != mine) << k;
    }
    uint32_t *col = prm.possession + (uint64_t)root_idx * prm.n_words * p + v;
    for (uint32_t w = 0; w < prm.n_words; ++w) col[(uint64_t)w * p] = 0u;

    if (v != 0) {
      const Blk nm1 = (Blk)n - 1;
      // round i = x + round uses entry k = i mod q advanced by q * floor(i / q) - x
      const uint32_t i0 = kReverse ? prm.x + prm.rounds - 1u : prm.x;
      uint32_t k = i0 % q;
      Blk shift = -(Blk)prm.x + (Blk)q * (Blk)(i0 / q);
      // The word of the possession column that was written last stays in a
      // register: blocks arrive in nearly increasing order, so a word serves
      // some 32 rounds before the next one is fetched.
      uint32_t cw = 0xFFFFFFFFu, cv = 0u;
      auto note = [&](uint32_t &count, bool bad, uint32_t round) {
        count += (uint32_t)bad;
        const uint32_t first = round < bad_round ? round : bad_round;
        bad_round = bad ? first : bad_round;
      };
      // One round.  with_edges: some entry of the from-processors differs from the lane's own,
      // which never happens on a valid table; then the rounds do not look at `differs` at all.
      auto one_round = [&](uint32_t step, auto with_edges) {
        const uint32_t round = kReverse ? prm.rounds - 1u - step : step;
        Blk rb, sb;
        if (kPacked) {
          const int32_t both = st_recv[k][lane_b];
          rb = (Blk)(int16_t)(both & 0xFFFF) + shift;
          sb = (Blk)(both >> 16) + shift;
        } else {
          rb = (Blk)st_recv[k][lane_b] + shift;
          sb = (Blk)st_send[k][lane_b] + shift;
        }
        const bool has_r = rb >= 0;
        rb = rb > nm1 ? nm1 : rb;
        if (decltype(with_edges)::value && ((differs >> k) & 1u)) {   // the entries differ: do the blocks?
          int64_t fb = (int64_t)from_entry(k) + (int64_t)shift;   // the entry as given, not clamped
          const bool has_f = fb >= 0;
          fb = fb > (int64_t)nm1 ? (int64_t)nm1 : fb;
          note(c_edge, has_r != has_f || (has_r && (int64_t)rb != fb), round);
        }
        const bool has_s = sb >= 0;
        sb = sb > nm1 ? nm1 : sb;
        if (!kReverse && has_s) {                   // state before this round
          const uint32_t w = (uint32_t)sb >> 5;
          const uint32_t word = w == cw ? cv : col[(uint64_t)w * p];
          note(c_unheld, ((word >> ((uint32_t)sb & 31u)) & 1u) == 0u, round);
        }
        if (has_r) {
          const uint32_t w = (uint32_t)rb >> 5;
          if (w != cw) {
            if (cw != 0xFFFFFFFFu) col[(uint64_t)cw * p] = cv;
            cw = w;
            cv = col[(uint64_t)w * p];
          }
          const uint32_t bit = 1u << ((uint32_t)rb & 31u);
          note(c_dup, (cv & bit) != 0u, round);
          cv |= bit;
        }
        if (kReverse && has_s) {                    // state after this round's send
          const uint32_t w = (uint32_t)sb >> 5;
          const uint32_t word = w == cw ? cv : col[(uint64_t)w * p];
          note(c_unheld, ((word >> ((uint32_t)sb & 31u)) & 1u) != 0u, round);
        }
        if (kReverse) {
          if (k == 0) { k = q - 1u; shift -= (Blk)q; } else { --k; }
        } else {
          if (++k == q) { k = 0; shift += (Blk)q; }
        }
      };
      if (__any(differs != 0u)) {
        for (uint32_t step = 0; step < prm.rounds; ++step) one_round(step, std::true_type{});
      } else {
        for (uint32_t step = 0; step < prm.rounds; ++step) one_round(step, std::false_type{});
      }
      if (cw != 0xFFFFFFFFu) col[(uint64_t)cw * p] = cv;
      if (bad_round != 0xFFFFFFFFu) first_bad = ((uint64_t)bad_round << 32) | r_phys;
      uint32_t have = 0;
      for (uint32_t w = 0; w < prm.n_words; ++w) {
        uint32_t word = col[(uint64_t)w * p];
        if (w == prm.n_words - 1u && (n & 31u)) word &= (1u << (n & 31u)) - 1u;
        have += (uint32_t)__popc(word);
      }
      if (have != n) {
        n_incomplete = 1;
        const uint64_t key = ((uint64_t)prm.rounds << 32) | r_phys;
        first_bad = key < first_bad ? key : first_bad;
      }
    }
  }
  uint64_t n_dup = c_dup, n_unheld = c_unheld, n_edge = c_edge;

  // wavefront reductions, then one atomic per counter that is not zero
  const uint64_t bad_lanes = __ballot(n_incomplete != 0);
  n_dup = wave_add64(n_dup);
  n_unheld = wave_add64(n_unheld);
  n_edge = wave_add64(n_edge);
  first_bad = wave_min64(first_bad);
  if (lane == 0) {
    bcast_verdict *vd = prm.verdict + root_idx;
    uint32_t fl = 0;
    if (n_dup) { fl |= BCAST_V_RECV_DUP; atomicAdd((unsigned long long *)&vd->n_bad_recv_dup, (unsigned long long)n_dup); }
    if (n_unheld) { fl |= BCAST_V_SEND_UNHELD; atomicAdd((unsigned long long *)&vd->n_bad_send_unheld, (unsigned long long)n_unheld); }
    if (n_edge) { fl |= BCAST_V_EDGE; atomicAdd((unsigned long long *)&vd->n_edge_mismatch, (unsigned long long)n_edge); }
    if (bad_lanes) { fl |= BCAST_V_INCOMPLETE; atomicAdd((unsigned long long *)&vd->n_incomplete_ranks, (unsigned long long)__popcll(bad_lanes)); }
    if (fl) {
      atomicOr(&vd->flags, fl);
      atomicMin((unsigned long long *)&vd->first_bad, (unsigned long long)first_bad);
    }
  }
}

// --------------------------------------------------------------- host side

int host_q(uint32_t p) {
  if (p == 0 || p > BCAST_MAX_P) return BCAST_EINVAL;
  int q = 0;
  while ((1ull << q) < (uint64_t)p) ++q;
  return q;
}

int persistent_grid(uint64_t n_blocks_wanted) {
  int dev = 0, n_cus = 0;
  if (hipGetDevice(&dev) != hipSuccess) return -1;
  if (hipDeviceGetAttribute(&n_cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cus <= 0)
    return -1;
  // Many more workgroups than fit at once: ranks take different numbers of
  // steps, and the dispatcher evens that out by handing out the next workgroup
  // whenever one ends.  64 per CU measured best on MI355X (8: 19 % slower;
  // one tile per wavefront: one atomic per wavefront on one address, 2x slower).
  const uint64_t cap = (uint64_t)n_cus * 64u;
  const uint64_t g = n_blocks_wanted < cap ? n_blocks_wanted : cap;
  return (int)(g == 0 ? 1 : g);
}

// Grid of the kernels whose wavefronts work through runs of 64-rank tiles and carry records from
// tile to tile: the first tile of a run has nothing to take over and costs about three times a
// later one, so runs should be long, while several resident sets of workgroups are still needed
// for the dispatcher to even out the load.  24 workgroups per CU (three resident sets) measured
// best on MI355X: against 64, 2^26 ranks of p = 2^31 - 1 hash 3 % faster, of p = 2^30 + 1 10 %
// faster, tables of 16 to 64 million ranks 2-4 % faster; 16 to 32 are level, 8 and 96 slower.
constexpr uint64_t kRunGridPerCu = 24;
int run_grid_cap() {
  const int cap = persistent_grid(UINT64_MAX);                  // 64 workgroups per CU
  return cap < 0 ? cap : (int)((uint64_t)cap / 64u * kRunGridPerCu);
}
int lone_grid(uint64_t n_blocks_wanted) {
  const int cap = run_grid_cap();
  if (cap < 0) return cap;
  const uint64_t g = n_blocks_wanted < (uint64_t)cap ? n_blocks_wanted : (uint64_t)cap;
  return (int)(g == 0 ? 1 : g);
}

bool launch_ok() { return hipGetLastError() == hipSuccess; }

// Runs of tiles for a grid of `grid` workgroups (see RunSplit).
//
// Workgroups start in the order of their numbers, and a SIMD serves its oldest wavefront first:
// of the wavefronts of one resident set with equal runs, those of the first workgroups end after
// 34 us and those of the last after 75-90 (p = 1,000,003), and with several sets the last
// workgroups to start set the end of the launch.  So the runs get shorter from class to class;
// the two sets of weights are the best of a dozen tried on MI355X (tables of 10^6 to 10^9 ranks:
// 2-13 % faster than equal runs).  Launches that fill less than seven eighths of the chip keep
// equal runs: there the classes do not line up with the order on a SIMD, and skewed runs are
// 3-30 % slower.
RunSplit split_runs(uint64_t n_tiles, int grid) {
  static const uint32_t kOneSet[kRunClasses] = {6, 5, 5, 4, 4, 3, 2, 1};
  static const uint32_t kManySets[kRunClasses] = {8, 8, 8, 8, 6, 4, 2, 1};
  const int64_t one_set = persistent_grid(UINT64_MAX) / 64 * 8;     // workgroups resident at once
  const uint32_t *weight = nullptr;
  if (one_set > 0 && (int64_t)grid * 8 >= one_set * 7) weight = grid <= 2 * one_set ? kOneSet : kManySets;
  RunSplit rs;
  const uint64_t g = (uint64_t)grid;
  rs.class_blocks = (uint32_t)((g + kRunClasses - 1) / kRunClasses);
  uint64_t share[kRunClasses], total = 0;
  for (uint32_t c = 0; c < kRunClasses; ++c) {
    const uint64_t lo = (uint64_t)c * rs.class_blocks;
    const uint64_t blocks = lo >= g ? 0 : (g - lo < rs.class_blocks ? g - lo : rs.class_blocks);
    share[c] = blocks * (weight ? weight[c] : 1u);
    total += share[c];
  }
  uint64_t done = 0, acc = 0;
  for (uint32_t c = 0; c < kRunClasses; ++c) {
    const uint64_t lo = (uint64_t)c * rs.class_blocks;
    const uint64_t blocks = lo >= g ? 0 : (g - lo < rs.class_blocks ? g - lo : rs.class_blocks);
    acc += share[c];
    // cumulative rounding: the classes' tiles add up to n_tiles exactly
    const uint64_t upto = total ? (uint64_t)((unsigned __int128)n_tiles * acc / total) : 0;
    const uint64_t tiles = upto - done;
    const uint64_t waves = blocks * kWavesPerBlock;
    rs.first[c] = (uint32_t)done;
    rs.base[c] = waves ? (uint32_t)(tiles / waves) : 0u;
    rs.extra[c] = waves ? (uint32_t)(tiles % waves) : 0u;
    done = upto;
  }
  return rs;
}

// Grid of k_schedules<true>, whose wavefronts each take one contiguous run of
// tiles.  Long runs make the deferred violations and the records cheap; more workgroups
// than fit at once even out the load, because a SIMD serves its oldest
// wavefront first and the young ones of a resident set fall behind by a factor
// of two.  Measured on MI355X: everything at once when it fits; else two tiles per wavefront
// until that makes three resident sets, and three sets from there on (tables of 3 to 6 million
// ranks 2-3 % faster than with two sets, the others level).  (With at most 2^25
// tiles on 24,576 wavefronts and run lengths that differ by a factor of 1.5 from the mean, a run
// stays below 2,100 tiles, so a row within a run fits 27 bits with room to spare: the queue
// entries of the kernels rely on that.)
int run_grid(uint64_t n_tiles, uint32_t resident_per_cu) {
  const int cap = run_grid_cap();                                 // three resident sets
  if (cap < 0) return -1;
  const uint64_t one_set = (uint64_t)cap / kRunGridPerCu * resident_per_cu;   // workgroups that fit at once
  const uint64_t per_wg = kWavesPerBlock;
  const uint64_t g_one = (n_tiles + per_wg - 1) / per_wg;        // one tile per wavefront
  if (g_one <= one_set) return (int)(g_one == 0 ? 1 : g_one);
  const uint64_t g_two = (n_tiles + per_wg * 2u - 1) / (per_wg * 2u);
  return (int)(g_two < (uint64_t)cap ? g_two : (uint64_t)cap);
}

// Algorithm 6 has (next to) no violations when every skip below p is a power of
// two (p = 2^q and p = 2^q - 1): then the few there are are searched for on the
// spot (tile_rows).  Otherwise the kernels keep the rows of the tile above and
// defer what those do not answer (k_schedules<true>, k_digest<true, .>).  The
// choice only affects speed.
bool keep_next_tile(uint32_t p) { return (p & (p - 1u)) != 0u && (p & (p + 1u)) != 0u; }

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

}  // namespace

// ------------------------------------------------------------------- C ABI

extern "C" {

int bcast_q(uint32_t p) { return host_q(p); }

int bcast_skips(uint32_t p, uint32_t *skips, int *q_out) {
  const int q = host_q(p);
  if (q < 0 || !skips) return BCAST_EINVAL;
  // Algorithm 2 halves with rounding up q - k times: skip[k] = ceil(p / 2^(q-k))
  for (int k = 0; k < q; ++k) skips[k] = ((p - 1u) >> (q - k)) + 1u;
  skips[q] = p;
  if (q_out) *q_out = q;
  return BCAST_OK;
}

}  // extern "C"

namespace {

// The table of deep entries of p in the caller's workspace (built on the stream, before the
// kernel that reads it), or none: no workspace, or p has too few levels above the deep ones.
// Returns false when a launch failed.
// Workspace of the *_ws calls: [table of deep entries][count of open entries][open entries].
constexpr size_t kEntriesBytes = (size_t)kDeepMaxEntries * sizeof(uint4) + 256u;
constexpr size_t kTableBytes = kEntriesBytes + (size_t)kDeepEs * kDeepMaxEntries * sizeof(uint16_t) + 256u;
uint32_t open_list_capacity(uint32_t p) {
  const uint64_t want = (uint64_t)p / 8u + 4096u;    // p = 1,000,003 leaves 39,000 open, p = 2^20 + 1 fewer than p / 16
  return (uint32_t)(want < (1ull << 22) ? want : (1ull << 22));
}
// The same room as segments of kOpenSegCap entries, one per wavefront, for the launches that no
// kernel precedes which could clear the list's counter (fewer than kTableMinRanks ranks: at most
// 8,192 wavefronts of one to three tiles, which leave two or three entries open per tile): a
// launch of its own to clear one word costs 4 us, a twentieth of the table of p = 1,000,003.
constexpr uint32_t kOpenSegCap = 64;
constexpr uint32_t kOpenSegWavesMax = 8192;
uint32_t open_segments_room(uint32_t p) {
  const uint64_t waves = ((uint64_t)p + kWave - 1) / kWave + kWavesPerBlock;
  return (uint32_t)(waves < kOpenSegWavesMax ? waves : kOpenSegWavesMax);
}
size_t open_bytes(uint32_t p) {                      // either form, after the tables
  const size_t list = 256u + (size_t)open_list_capacity(p) * 8u;
  const size_t segments = ((size_t)open_segments_room(p) * 4u + 255u) / 256u * 256u +
                          (size_t)open_segments_room(p) * kOpenSegCap * 8u;
  return (list > segments ? list : segments) + 256u;
}

// Building the tables takes one small kernel ahead of the main one, some 12 us from launch to end;
// it pays from a million ranks on (measured on MI355X, tables with a workspace: p = 1,000,003
// 89 us with it against 87 without, p = 1,100,003 94 against 99, p = 2,000,003 128 against 140,
// tables of 2^23 ranks 1.4 times faster), so shorter ranges are computed without them.
constexpr uint64_t kTableMinRanks = 1ull << 20;

// `counter`: cleared by the same kernel if the table is built (see k_deep_table); *cleared says whether.
bool prepare_table(uint32_t p, int q, uint64_t n_ranks, void *workspace, hipStream_t st, DeepTable &table,
                   uint32_t *counter = nullptr, bool *cleared = nullptr) {
  if (cleared) *cleared = false;
  table.entries = nullptr; table.viol_by_e = nullptr; table.first_deep = 0; table.n_rho = 0;
  if (!workspace || q <= 0 || n_ranks < kTableMinRanks) return true;
  uint32_t first_deep = 0;                         // as first_deep_level() on the device
  if (p - 1u >= kLockstepSkip) {
    uint32_t x = (p - 1u) / kLockstepSkip;
    while (x) { ++first_deep; x >>= 1; }
  }
  if (first_deep < kDeepMinUpperLevels + 1u) return true;
  const uint32_t n_rho = ((p - 1u) >> (first_deep - 1u)) + 1u;      // smallest skip above the deep levels
  if (n_rho > kDeepMaxEntries) return true;
  const uintptr_t base = align_up(reinterpret_cast<uintptr_t>(workspace), 256);
  uint4 *entries = reinterpret_cast<uint4 *>(base);
  uint16_t *viol_by_e = reinterpret_cast<uint16_t *>(base + kEntriesBytes);
  const uint32_t blocks_per_row = (n_rho + kBlock - 1) / kBlock;
  hipLaunchKernelGGL(k_deep_table, dim3(blocks_per_row * kDeepEs), dim3(kBlock), 0, st, entries, viol_by_e, p,
                     (uint32_t)q, first_deep, n_rho, blocks_per_row, counter);
  if (!launch_ok()) return false;
  if (cleared) *cleared = counter != nullptr;
  table.entries = entries; table.viol_by_e = viol_by_e; table.first_deep = first_deep; table.n_rho = n_rho;
  return true;
}

int schedules_impl(uint32_t p, uint32_t root, uint64_t r_begin, uint64_t r_end, int32_t *recv,
                   int32_t *send, int64_t ld, void *workspace, void *stream) {
  const int q = host_q(p);
  if (q < 0 || root >= p || r_begin > r_end || r_end > p) return BCAST_EINVAL;
  const uint64_t n = r_end - r_begin;
  if (n == 0 || q == 0) return BCAST_OK;
  if (!recv || !send || ld < q) return BCAST_EINVAL;
  SchedParams prm;
  prm.p = p; prm.q = (uint32_t)q; prm.root = root;
  prm.r_begin = r_begin; prm.n_ranks = n;
  prm.recv = recv; prm.send = send; prm.ld = ld;
  const int32_t *recv_end = recv + (n - 1) * (uint64_t)ld + q;
  const int32_t *send_end = send + (n - 1) * (uint64_t)ld + q;
  if (send == recv + q && ld == 2 * (int64_t)q) {
    prm.layout = kInterleaved;
  } else if (send >= recv_end || recv >= send_end) {
    prm.layout = ld == q ? kSeparate : kRowwise;
  } else {
    // interleaved rows with padding: legal when every send row sits in the gap
    // of the recv rows, i.e. the offset modulo ld leaves room for q entries
    const int64_t d = send > recv ? send - recv : recv - send;
    const int64_t m = d % ld;
    if (m < q || ld - m < q) return BCAST_EINVAL;
    prm.layout = kRowwise;
  }
  const uint64_t blocks = (n + kBlock - 1) / kBlock;
  const bool share = keep_next_tile(p);
  const int grid = share ? run_grid((n + kWave - 1) / kWave, 8u) : lone_grid(blocks);
  if (grid < 0) return BCAST_EHIP;
  prm.runs = split_runs((n + kWave - 1) / kWave, grid);
  prm.open_list = nullptr; prm.open_count = nullptr; prm.open_cap = 0; prm.open_segments = 0;
  if (share && workspace) {                          // entries left open go to a list, see k_fill_open
    const uintptr_t base = align_up(reinterpret_cast<uintptr_t>(workspace), 256) + kTableBytes;
    prm.open_count = reinterpret_cast<uint32_t *>(base);
    prm.open_list = reinterpret_cast<unsigned long long *>(base + 256u);
    prm.open_cap = open_list_capacity(p);
  }
  bool count_cleared = false;
  if (!prepare_table(p, q, n, workspace, (hipStream_t)stream, prm.table, prm.open_count, &count_cleared))
    return BCAST_EHIP;
  if (prm.open_list != nullptr && !count_cleared &&
      (uint64_t)grid * kWavesPerBlock <= (uint64_t)open_segments_room(p)) {
    // nothing ahead of the main kernel that could clear the counter: a segment per wavefront instead
    const uintptr_t base = reinterpret_cast<uintptr_t>(prm.open_count);
    const size_t counts = ((size_t)open_segments_room(p) * 4u + 255u) / 256u * 256u;
    prm.open_list = reinterpret_cast<unsigned long long *>(base + counts);
    prm.open_cap = kOpenSegCap;
    prm.open_segments = (uint32_t)grid * kWavesPerBlock;
    count_cleared = true;                            // there is no counter
  }
  const bool memo = prm.table.entries != nullptr;
  const size_t lds = share ? (size_t)kWavesPerBlock * deferred_wave_words(prm.q) * 4u
                           : (size_t)lone_block_words(prm.q) * 4u;
  if (prm.open_count != nullptr && !count_cleared) {
    hipLaunchKernelGGL(k_u32_zero, dim3(1), dim3(64), 0, (hipStream_t)stream, prm.open_count);
    if (!launch_ok()) return BCAST_EHIP;
  }
  if (share) {
    if (memo) hipLaunchKernelGGL((k_schedules<true, true>), dim3(grid), dim3(kBlock), lds, (hipStream_t)stream, prm);
    else hipLaunchKernelGGL((k_schedules<true, false>), dim3(grid), dim3(kBlock), lds, (hipStream_t)stream, prm);
    if (prm.open_list) {
      if (!launch_ok()) return BCAST_EHIP;
      const uint64_t most = prm.open_segments != 0u ? (uint64_t)prm.open_segments * prm.open_cap
                            : n * 4u < prm.open_cap ? n * 4u : prm.open_cap;    // (sizes the grid only: its threads stride over the list)
      const uint64_t blocks_fill = (most + kBlock - 1) / kBlock;
      hipLaunchKernelGGL(k_fill_open, dim3((unsigned)(blocks_fill < 2048u ? (blocks_fill ? blocks_fill : 1u) : 2048u)),
                         dim3(kBlock), 0, (hipStream_t)stream, prm);
    }
  } else {
    if (memo) hipLaunchKernelGGL((k_schedules<false, true>), dim3(grid), dim3(kBlock), lds, (hipStream_t)stream, prm);
    else hipLaunchKernelGGL((k_schedules<false, false>), dim3(grid), dim3(kBlock), lds, (hipStream_t)stream, prm);
  }
  return launch_ok() ? BCAST_OK : BCAST_EHIP;
}

// digest and flags (edges = false) or the two sums of the edge check (edges = true, into out64)
// slot_shift: 63 for one result, else log2 of the ranks per result (digest and flags only).
int digest_impl(bool edges, uint32_t p, uint32_t root, uint64_t r_begin, uint64_t r_end,
                uint64_t *out64, uint32_t *flags, void *workspace, void *stream,
                uint32_t slot_shift = 63u) {
  const int q = host_q(p);
  if (q < 0 || root >= p || r_begin > r_end || r_end > p) return BCAST_EINVAL;
  const uint64_t n = r_end - r_begin;
  const uint64_t n_slots = slot_shift >= 63u ? 1u : (n + (1ull << slot_shift) - 1u) >> slot_shift;
  if (n_slots != 0 && (!out64 || (!edges && !flags))) return BCAST_EINVAL;
  if (n_slots == 0) return BCAST_OK;             // an empty range in chunks: nothing to write
  const bool share = keep_next_tile(p);
  const bool work = n != 0 && !(edges && q == 0);
  int grid = 1;
  if (work) {
    grid = share ? run_grid((n + kWave - 1) / kWave, 8u) : lone_grid((n + kBlock - 1) / kBlock);
    if (grid < 0) return BCAST_EHIP;
  } else if (persistent_grid(1) < 0) {
    return BCAST_EHIP;
  }
  hipStream_t st = (hipStream_t)stream;
  // with a workspace, the ranks that the kernel for p with violations cannot finish go to a list
  // there (the room of the list of open entries, as 32-bit rows) and k_digest_listed computes them
  uint32_t *rank_count = nullptr, *rank_list = nullptr;
  if (work && share && workspace && !edges) {      // (the edge check is no faster with the list: 5.09 ms against 5.01)
    const uintptr_t base = align_up(reinterpret_cast<uintptr_t>(workspace), 256) + kTableBytes;
    rank_count = reinterpret_cast<uint32_t *>(base);
    rank_list = reinterpret_cast<uint32_t *>(base + 256u);
  }
  if (edges) hipLaunchKernelGGL(k_edges_init, dim3(1), dim3(64), 0, st, out64, rank_count);
  else hipLaunchKernelGGL(k_digest_init, dim3((unsigned)((n_slots + 63u) / 64u)), dim3(64), 0, st, out64, flags,
                          rank_count, n_slots);
  if (!launch_ok()) return BCAST_EHIP;
  if (!work) return BCAST_OK;
  DigestParams prm;
  prm.p = p; prm.q = (uint32_t)q; prm.root = root;
  prm.r_begin = r_begin; prm.n_ranks = n;
  prm.digest = out64; prm.flags = edges ? nullptr : flags;
  prm.slot_shift = slot_shift;
  prm.rank_list = rank_list; prm.rank_count = rank_count;
  prm.rank_cap = rank_list ? open_list_capacity(p) * 2u : 0u;
  prm.runs = split_runs((n + kWave - 1) / kWave, grid);
  if (!prepare_table(p, q, n, workspace, st, prm.table)) return BCAST_EHIP;
  const bool memo = prm.table.entries != nullptr;
  const size_t lds = share ? (size_t)kWavesPerBlock * digest_deferred_wave_words(prm.q) * 4u
                           : (size_t)digest_lone_block_words(prm.q) * 4u;
  const dim3 g(grid), b(kBlock);
#define BCAST_LAUNCH_DIGEST(S, E, M) hipLaunchKernelGGL((k_digest<S, E, M>), g, b, lds, st, prm)
  if (share) {
    if (edges) { if (memo) BCAST_LAUNCH_DIGEST(true, true, true); else BCAST_LAUNCH_DIGEST(true, true, false); }
    else { if (memo) BCAST_LAUNCH_DIGEST(true, false, true); else BCAST_LAUNCH_DIGEST(true, false, false); }
  } else {
    if (edges) { if (memo) BCAST_LAUNCH_DIGEST(false, true, true); else BCAST_LAUNCH_DIGEST(false, true, false); }
    else { if (memo) BCAST_LAUNCH_DIGEST(false, false, true); else BCAST_LAUNCH_DIGEST(false, false, false); }
  }
#undef BCAST_LAUNCH_DIGEST
  if (rank_list) {
    if (!launch_ok()) return BCAST_EHIP;
    const size_t lds_listed = (size_t)kWavesPerBlock * digest_slice_words(prm.q) * 4u;
    const uint64_t most = n < prm.rank_cap ? n : prm.rank_cap;
    const uint64_t blocks_listed = (most + kBlock - 1) / kBlock;
    const dim3 gl((unsigned)(blocks_listed < 4096u ? blocks_listed : 4096u));
    hipLaunchKernelGGL(k_digest_listed, gl, b, lds_listed, st, prm);
  }
  return launch_ok() ? BCAST_OK : BCAST_EHIP;
}

// workspace argument of a *_ws call: NULL is an error there, and so is one that is too small
int check_workspace(uint32_t p, const void *workspace, size_t workspace_bytes) {
  const size_t need = host_q(p) < 0 ? 0 : kTableBytes + open_bytes(p);
  if (need == 0 || !workspace) return BCAST_EINVAL;
  return workspace_bytes < need ? BCAST_ENOMEM : BCAST_OK;
}

}  // namespace

extern "C" {

// Bytes of the workspace of the *_ws calls: the table of deep entries and the list of entries
// left open.
size_t bcast_schedules_workspace(uint32_t p) {
  if (host_q(p) < 0) return 0;
  return kTableBytes + open_bytes(p);
}

int bcast_schedules(uint32_t p, uint32_t root, uint64_t r_begin, uint64_t r_end,
                    int32_t *recv, int32_t *send, int64_t ld, void *stream) {
  return schedules_impl(p, root, r_begin, r_end, recv, send, ld, nullptr, stream);
}

int bcast_schedules_ws(uint32_t p, uint32_t root, uint64_t r_begin, uint64_t r_end,
                       int32_t *recv, int32_t *send, int64_t ld, void *workspace,
                       size_t workspace_bytes, void *stream) {
  const int rc = check_workspace(p, workspace, workspace_bytes);
  if (rc != BCAST_OK) return rc;
  return schedules_impl(p, root, r_begin, r_end, recv, send, ld, workspace, stream);
}

int bcast_schedules_digest(uint32_t p, uint32_t root, uint64_t r_begin, uint64_t r_end,
                           uint64_t *digest, uint32_t *flags, void *stream) {
  return digest_impl(false, p, root, r_begin, r_end, digest, flags, nullptr, stream);
}

int bcast_schedules_digest_ws(uint32_t p, uint32_t root, uint64_t r_begin, uint64_t r_end,
                              uint64_t *digest, uint32_t *flags, void *workspace,
                              size_t workspace_bytes, void *stream) {
  const int rc = check_workspace(p, workspace, workspace_bytes);
  if (rc != BCAST_OK) return rc;
  return digest_impl(false, p, root, r_begin, r_end, digest, flags, workspace, stream);
}

int bcast_schedules_digest_chunks(uint32_t p, uint32_t root, uint64_t r_begin, uint64_t r_end,
                                  uint64_t chunk_ranks, uint64_t *digests, uint32_t *flags,
                                  void *workspace, size_t workspace_bytes, void *stream) {
  if (chunk_ranks < (uint64_t)kWave || (chunk_ranks & (chunk_ranks - 1u)) != 0 || chunk_ranks > (1ull << 62))
    return BCAST_EINVAL;
  uint32_t shift = 0;
  while ((1ull << shift) < chunk_ranks) ++shift;
  if (r_begin <= r_end && ((r_end - r_begin + chunk_ranks - 1u) >> shift) > 0xFFFFFFFFull) return BCAST_EINVAL;
  if (workspace || workspace_bytes != 0) {
    const int rc = check_workspace(p, workspace, workspace_bytes);
    if (rc != BCAST_OK) return rc;
  }
  return digest_impl(false, p, root, r_begin, r_end, digests, flags, workspace, stream, shift);
}

int bcast_schedules_edgecheck(uint32_t p, uint32_t root, uint64_t r_begin, uint64_t r_end,
                              uint64_t *xors, void *stream) {
  return digest_impl(true, p, root, r_begin, r_end, xors, nullptr, nullptr, stream);
}

int bcast_schedules_edgecheck_ws(uint32_t p, uint32_t root, uint64_t r_begin, uint64_t r_end,
                                 uint64_t *xors, void *workspace, size_t workspace_bytes,
                                 void *stream) {
  const int rc = check_workspace(p, workspace, workspace_bytes);
  if (rc != BCAST_OK) return rc;
  return digest_impl(true, p, root, r_begin, r_end, xors, nullptr, workspace, stream);
}

int bcast_schedules_double(uint32_t p, const int32_t *in, int32_t *out, void *stream) {
  const int q = host_q(p);
  if (q < 0 || p > BCAST_MAX_P / 2u || !out || (q > 0 && !in)) return BCAST_EINVAL;
  const uint64_t in_elems = (uint64_t)p * 2u * (uint32_t)q, out_elems = (uint64_t)p * 4u * ((uint32_t)q + 1u);
  if (in && out + out_elems > in && in + in_elems > out) return BCAST_EINVAL;   // overlap
  DoubleParams prm;
  prm.p = p; prm.q = (uint32_t)q; prm.in = in; prm.out = out;
  const uint64_t tiles = ((uint64_t)p + kWave - 1) / kWave;
  const int grid = persistent_grid((tiles + kWavesPerBlock - 1) / kWavesPerBlock);
  if (grid < 0) return BCAST_EHIP;
  const size_t lds = (size_t)kWavesPerBlock * (slice_words(prm.q) + 2u * slice_words(prm.q + 1u)) * 4u;
  hipLaunchKernelGGL(k_double, dim3(grid), dim3(kBlock), lds, (hipStream_t)stream, prm);
  return launch_ok() ? BCAST_OK : BCAST_EHIP;
}

int bcast_baseblocks(uint32_t p, uint8_t *list, void *stream) {
  const int q = host_q(p);
  if (q < 0 || !list) return BCAST_EINVAL;
  const int cap = persistent_grid(UINT64_MAX);
  if (cap < 0) return BCAST_EHIP;
  hipStream_t st = (hipStream_t)stream;
  // list of one rank: the root with entry 0; then one step per skip
  hipLaunchKernelGGL(k_listing_root, dim3(1), dim3(64), 0, st, list, 0u);
  if (!launch_ok()) return BCAST_EHIP;
  uint32_t skips[32];
  bcast_skips(p, skips, nullptr);
  for (int k = 0; k < q; ++k) {
    const uint64_t n = (uint64_t)skips[k + 1] - skips[k];
    if (n > 0) {
      const uint64_t want = (n / 16u + kBlock - 1) / kBlock + 1u;
      const int grid = (int)(want < (uint64_t)cap ? want : (uint64_t)cap);
      hipLaunchKernelGGL(k_listing_step, dim3(grid), dim3(kBlock), 0, st, list, skips[k], skips[k + 1]);
      if (!launch_ok()) return BCAST_EHIP;
    }
    // the root's entry changes after the copy has read it (same stream: in order)
    hipLaunchKernelGGL(k_listing_root, dim3(1), dim3(64), 0, st, list, (uint32_t)k + 1u);
    if (!launch_ok()) return BCAST_EHIP;
  }
  return BCAST_OK;
}

size_t bcast_schedules_doubling_workspace(uint32_t p) {
  const int q = host_q(p);
  if (q < 0) return 0;
  uint32_t j = 0;
  while (j < 31u && ((p >> j) & 1u) == 0u) ++j;          // p = m 2^j, m odd
  if (j == 0) return 256;                                 // odd p: nothing to double
  size_t bytes = 256;
  for (uint32_t i = 1; i <= 2u && i <= j; ++i) {          // the tables of p/2 and p/4
    const uint32_t pi = p >> i;
    const int qi = host_q(pi);
    bytes += align_up((size_t)pi * 2u * (size_t)qi * 4u, 256);
  }
  return bytes;
}

int bcast_schedules_doubling(uint32_t p, int32_t *out, void *workspace, size_t workspace_bytes,
                             void *stream) {
  const int q = host_q(p);
  if (q < 0) return BCAST_EINVAL;
  if (q == 0) return BCAST_OK;
  if (!out) return BCAST_EINVAL;
  uint32_t j = 0;
  while (j < 31u && ((p >> j) & 1u) == 0u) ++j;
  // a doubling is a launch of its own: below some 2^16 ranks the search is faster than that
  // (a table of 3 x 2^20 ranks: 0.38 ms with all 20 doublings), so it starts from there
  while (j > 0u && (p >> j) < 65536u) --j;
  if (j == 0) return bcast_schedules(p, 0, 0, p, out, out + q, 2 * (int64_t)q, stream);
  const size_t need = bcast_schedules_doubling_workspace(p);
  if (!workspace) return BCAST_EINVAL;
  if (workspace_bytes < need) return BCAST_ENOMEM;
  if (persistent_grid(1) < 0) return BCAST_EHIP;
  // two buffers: A holds the tables of p/2, p/8, ..., B those of p/4, p/16, ...
  uintptr_t base = align_up(reinterpret_cast<uintptr_t>(workspace), 256);
  int32_t *buf_a = reinterpret_cast<int32_t *>(base);
  base += align_up((size_t)(p >> 1) * 2u * (size_t)host_q(p >> 1) * 4u, 256);
  int32_t *buf_b = reinterpret_cast<int32_t *>(base);
  // the caller's table must not overlap the workspace that is in use
  {
    const uintptr_t o0 = reinterpret_cast<uintptr_t>(out), o1 = o0 + (size_t)p * 2u * (size_t)q * 4u;
    const uintptr_t w0 = reinterpret_cast<uintptr_t>(workspace), w1 = w0 + need;
    if (o0 < w1 && w0 < o1) return BCAST_EINVAL;
  }
  auto buffer_of = [&](uint32_t halvings) { return (halvings & 1u) ? buf_a : buf_b; };   // table of p >> halvings
  const uint32_t m = p >> j;
  const int qm = host_q(m);
  int32_t *cur = buffer_of(j);
  if (qm > 0) {
    const int rc = bcast_schedules(m, 0, 0, m, cur, cur + qm, 2 * (int64_t)qm, stream);
    if (rc != BCAST_OK) return rc;
  }
  for (uint32_t h = j; h >= 1u; --h) {                   // table of p >> (h - 1) from that of p >> h
    int32_t *next = h == 1u ? out : buffer_of(h - 1u);
    const int rc = bcast_schedules_double(p >> h, (p >> h) > 1u ? cur : nullptr, next, stream);
    if (rc != BCAST_OK) return rc;
    cur = next;
  }
  return BCAST_OK;
}

int bcast_schedules_batched(uint32_t n_inst, const uint32_t *p, const uint32_t *root,
                            const uint32_t *ranks, uint32_t m, const uint64_t *row_off,
                            int32_t *out, uint64_t out_elems, uint32_t *n_rejected,
                            void *stream) {
  if (n_rejected) {
    hipLaunchKernelGGL(k_u32_zero, dim3(1), dim3(64), 0, (hipStream_t)stream, n_rejected);
    if (!launch_ok()) return BCAST_EHIP;
  }
  if (n_inst == 0) return BCAST_OK;
  if (!p || !root || !ranks || !row_off || m == 0) return BCAST_EINVAL;
  if (!out && out_elems != 0) return BCAST_EINVAL;
  BatchParams prm;
  prm.n_inst = n_inst; prm.m = m; prm.tiles_per_inst = (m + kWave - 1) / kWave;
  prm.p = p; prm.root = root; prm.ranks = ranks; prm.row_off = row_off;
  prm.out = out; prm.out_elems = out_elems; prm.n_rejected = n_rejected;
  const uint64_t work = (uint64_t)n_inst * ((prm.tiles_per_inst + kBatchTiles - 1u) / kBatchTiles);
  // a batch is long enough for four times the usual number of workgroups: less of a tail
  int grid = persistent_grid(UINT64_MAX);
  if (grid < 0) return BCAST_EHIP;
  {
    const uint64_t want = (work + kWavesPerBlock - 1) / kWavesPerBlock, cap = (uint64_t)grid * 4u;
    grid = (int)(want < cap ? want : cap);
  }
  hipLaunchKernelGGL(k_batched, dim3(grid), dim3(kBlock), 0, (hipStream_t)stream, prm);
  return launch_ok() ? BCAST_OK : BCAST_EHIP;
}

// workspace: [roots: n_roots u32][table by rows: p*2q int32][the same by columns]
//            [possession: n_roots*n_words*p u32]
// 0 when the arguments are outside the domain or the size does not fit size_t.
size_t bcast_simulate_workspace(uint32_t p, uint32_t n, uint32_t n_roots) {
  const int q = host_q(p);
  if (q < 0 || n == 0 || n > BCAST_MAX_N || n_roots == 0 || n_roots > 65535u) return 0;
  const unsigned __int128 n_words = ((uint64_t)n + 31u) / 32u;
  const unsigned __int128 limit = (unsigned __int128)SIZE_MAX - 4096u;
  unsigned __int128 bytes = align_up((size_t)n_roots * 4, 256);
  bytes += 2u * (unsigned __int128)align_up((size_t)p * 2 * (size_t)q * 4, 256);   // < 2^40
  const unsigned __int128 possession = (unsigned __int128)n_roots * n_words * p * 4u;   // < 2^16 2^23 2^31 4
  if (possession > limit) return 0;
  bytes += (possession + 255u) / 256u * 256u;
  bytes += 256u;
  return bytes > limit ? 0 : (size_t)bytes;
}

static int simulate_impl(bool reverse, uint32_t p, uint32_t n, const uint32_t *roots,
                         uint32_t n_roots, const int32_t *sched, void *workspace,
                         size_t workspace_bytes, bcast_verdict *verdict, void *stream) {
  const int q = host_q(p);
  if (q < 0 || n == 0 || n > BCAST_MAX_N || n_roots == 0 || n_roots > 65535u || !roots || !verdict)
    return BCAST_EINVAL;
  for (uint32_t i = 0; i < n_roots; ++i)
    if (roots[i] >= p) return BCAST_EINVAL;
  const size_t need = bcast_simulate_workspace(p, n, n_roots);
  if (!workspace || need == 0) return BCAST_EINVAL;
  if (workspace_bytes < need) return BCAST_ENOMEM;
  // the last thing that can fail before a launch: asking the device for its size
  if (persistent_grid(1) < 0) return BCAST_EHIP;
  hipStream_t st = (hipStream_t)stream;
  const uint32_t rounds = q == 0 ? 0u : n - 1u + (uint32_t)q;
  hipLaunchKernelGGL(k_verdict_init, dim3((n_roots + 63) / 64), dim3(64), 0, st, verdict,
                     n_roots, rounds);
  if (!launch_ok()) return BCAST_EHIP;
  if (q == 0) return BCAST_OK;          // p = 1: the root holds everything, no rounds

  uintptr_t base = align_up(reinterpret_cast<uintptr_t>(workspace), 256);
  uint32_t *d_roots = reinterpret_cast<uint32_t *>(base);
  base += align_up((size_t)n_roots * 4, 256);
  int32_t *table = reinterpret_cast<int32_t *>(base);
  base += align_up((size_t)p * 2 * (size_t)q * 4, 256);
  int32_t *columns = reinterpret_cast<int32_t *>(base);
  base += align_up((size_t)p * 2 * (size_t)q * 4, 256);
  uint32_t *possession = reinterpret_cast<uint32_t *>(base);

  for (uint32_t first = 0; first < n_roots; first += kRootBatch) {
    RootBatch b;
    b.first = first;
    b.count = n_roots - first < kRootBatch ? n_roots - first : kRootBatch;
    memcpy(b.root, roots + first, (size_t)b.count * 4);
    if (b.count < kRootBatch) memset(b.root + b.count, 0, (size_t)(kRootBatch - b.count) * 4);
    hipLaunchKernelGGL(k_store_roots, dim3(1), dim3(kRootBatch), 0, st, d_roots, b);
    if (!launch_ok()) return BCAST_EHIP;
  }

  if (!sched) {
    const int rc = bcast_schedules(p, 0, 0, p, table, table + q, 2 * (int64_t)q, stream);
    if (rc != BCAST_OK) return rc;
    const uint32_t c = 2u * (uint32_t)q;
    hipLaunchKernelGGL(k_rows_to_columns, dim3((p + kWave - 1) / kWave), dim3(kWave),
                       (size_t)kWave * (c | 1u) * 4u, st, table, columns, p, c);
    if (!launch_ok()) return BCAST_EHIP;
  }
  SimParams prm;
  prm.p = p; prm.q = (uint32_t)q; prm.n = n; prm.n_words = (n + 31u) / 32u;
  prm.x = ((uint32_t)q - (n - 1u) % (uint32_t)q) % (uint32_t)q;
  prm.rounds = rounds;
  prm.roots = d_roots; prm.sched = sched; prm.table = columns;
  prm.possession = possession; prm.verdict = verdict;
  dim3 grid((p + kSimBlock - 1) / kSimBlock, n_roots);
  // clamped entries lie in [-C, C], C = n + 2q + 2: as 16-bit halves of one word when that fits
  const bool packed = (uint64_t)n + 2u * prm.q + 2u <= 32767u;
  const size_t lds = (size_t)(packed ? 1u : 2u) * prm.q * kSimBlock * sizeof(int32_t);
  if (reverse) {
    if (packed) hipLaunchKernelGGL((k_simulate<true, true>), grid, dim3(kSimBlock), lds, st, prm);
    else hipLaunchKernelGGL((k_simulate<true, false>), grid, dim3(kSimBlock), lds, st, prm);
  } else {
    if (packed) hipLaunchKernelGGL((k_simulate<false, true>), grid, dim3(kSimBlock), lds, st, prm);
    else hipLaunchKernelGGL((k_simulate<false, false>), grid, dim3(kSimBlock), lds, st, prm);
  }
  return launch_ok() ? BCAST_OK : BCAST_EHIP;
}

int bcast_simulate(uint32_t p, uint32_t n, const uint32_t *roots, uint32_t n_roots,
                   const int32_t *sched, void *workspace, size_t workspace_bytes,
                   bcast_verdict *verdict, void *stream) {
  return simulate_impl(false, p, n, roots, n_roots, sched, workspace, workspace_bytes, verdict,
                       stream);
}

int bcast_simulate_reduce(uint32_t p, uint32_t n, const uint32_t *roots, uint32_t n_roots,
                          const int32_t *sched, void *workspace, size_t workspace_bytes,
                          bcast_verdict *verdict, void *stream) {
  return simulate_impl(true, p, n, roots, n_roots, sched, workspace, workspace_bytes, verdict,
                       stream);
}

// ------------------------------------------------- the call that allocates nothing

namespace {

// The workspace of bcast_simulate for callers that cannot bring one: one array per GPU, there
// from the moment the library's code is loaded on that GPU until the process ends.
static __device__ __align__(256) unsigned char scratch[BCAST_NOALLOC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices];          // the array's address on each device, once asked for
std::mutex g_scratch_mutex;

// The address of `scratch` on the current device (the array's name is no device address in host
// code).  Asked for once per device, with that device current; nullptr if the runtime refuses.
void *scratch_on_current_device() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void *ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) {
      (void)hipGetLastError();
      return nullptr;
    }
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}

}  // namespace

int bcast_simulate_noalloc(uint32_t p, uint32_t n, const uint32_t *roots, uint32_t n_roots,
                           const int32_t *sched, bcast_verdict *verdict, void *stream) {
  const size_t need = bcast_simulate_workspace(p, n, n_roots);
  if (need == 0) return BCAST_EINVAL;
  if (need > (size_t)BCAST_NOALLOC_SCRATCH_BYTES) return BCAST_ENOMEM;
  void *ptr = scratch_on_current_device();
  if (ptr == nullptr) return BCAST_EHIP;
  // Nothing in the array has to start at zero: the replay clears the possession words it uses,
  // and the roots and the table are written before they are read.
  return simulate_impl(false, p, n, roots, n_roots, sched, ptr, (size_t)BCAST_NOALLOC_SCRATCH_BYTES,
                       verdict, stream);
}

const char *bcast_strerror(int code) {
  switch (code) {
    case BCAST_OK: return "ok";
    case BCAST_EINVAL: return "argument outside the documented domain";
    case BCAST_ENOMEM: return "workspace too small (bcast_simulate_noalloc: the replay needs more than BCAST_NOALLOC_SCRATCH_BYTES)";
    case BCAST_EHIP: return "HIP runtime error";
    default: return "unknown bcast error code";
  }
}

}  // extern "C"
