// Per-rank schedule computation for gfx950, one lane per rank.
//
// Everything here is 32-bit unsigned arithmetic on values below 2^32
// (p <= 2^31 - 1, so p + r and 2p fit).  Skip indices e = 0..q are handled as
// "levels" j = q - e, because skip[q - j] = ceil(p / 2^j) = ((p - 1) >> j) + 1
// (Algorithm 2 is repeated halving with rounding up), which costs a shift and
// an add and needs no table.  A set of skip indices is a 32-bit mask over
// levels; "next smaller remaining index" of the linked list of Algorithm 4 is
// "lowest set bit above the current level".
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/bcast.h"

namespace bcast {

constexpr uint32_t kEndLevel = 0xFFFFFFFFu;
constexpr uint32_t kLockstepSkip = 1024u;   // see recv_ascent: where the ascent re-synchronises

// skip[q - j]
__device__ __forceinline__ uint32_t skip_at_level(uint32_t pm1, uint32_t j) {
  return (pm1 >> j) + 1u;
}

// Lowest set bit of `live` strictly above level j, kEndLevel if none.
__device__ __forceinline__ uint32_t next_level(uint32_t live, uint32_t j) {
  const uint32_t above = live & ((0xFFFFFFFEu) << j);
  return (uint32_t)(__ffs((int)above) - 1);
}

// Algorithm 3 in level form: the level of the baseblock of virtual rank v,
// i.e. q - b.  The greedy walk takes skip[k] whenever it still fits; the last
// skip taken closes the sum and is the smallest index of the canonical skip
// sequence.  v = 0 takes nothing and yields level 0 (b = q).  (On its own, for
// callers that want the baseblock only; the kernels get it from top_down_level.)
__device__ __forceinline__ uint32_t baseblock_level(uint32_t pm1, uint32_t q, uint32_t v) {
  uint32_t rem = v, jb = 0;
  for (uint32_t j = 1; j <= q; ++j) {
    const uint32_t sk = skip_at_level(pm1, j);   // same for all lanes: a scalar
    const uint32_t t = rem - sk;                 // wraps above rem when sk > rem
    const uint32_t nr = t < rem ? t : rem;
    jb = nr != rem ? j : jb;
    rem = nr;
  }
  return jb;
}

// Algorithms 4 and 5: the receive search for virtual rank v, as an explicit
// state machine instead of recursion.  This is the search in its plain form,
// one list element per iteration from the first call on; the kernels run the
// reorganised form below (top_down_level + recv_ascent), which the CPU checks
// hold against this one.
//
// State, in the notation of Algorithm 4 with R = p + v:
//   D    = R - r'            distance still to cover (the frame's r')
//   Sd   = R - s             distance of the last accepted r'_k (0 while s = 2p:
//                            the test r' + skip[e] < s is then implied by the first)
//   j    = level of the list cursor e, kEndLevel when the list is exhausted
//   live = remaining skip indices, path = indices of the pending calls
// The two tests of the while body become  skip[e] + skip[k] <= D  and
// D - skip[e] > Sd, the test for a recursive call  skip[e] + skip[k+1] <= D, and
// the test after the call  D < skip[k+1]; none of them can overflow.
//
// A recursive call only ever scans levels above the one it was made for, so
// the pending calls form an increasing chain of levels: r' is recovered on
// return by adding the skip of the highest level in `path`.  The call made
// for index e would look at e itself first; that look always fails (checked
// exhaustively on the CPU for p <= 4096 and on samples of large p), so the
// cursor moves on at once and the case is only detected: it raises `anomaly`.
//
// `emit(k, value)` receives recvblock[k] for k = 0, 1, ... in order and the
// search stops once k exceeds k_last.  Returns the number of entries produced.
template <typename Emit>
__device__ __forceinline__ uint32_t recv_search(uint32_t p, uint32_t pm1, uint32_t q,
                                                uint32_t v, uint32_t jb, uint32_t k_last,
                                                bool &anomaly, Emit emit) {
  uint32_t D = p + v;
  uint32_t Sd = 0;
  uint32_t j = 0;
  uint32_t k = 0;
  uint32_t live = (q >= 31 ? 0xFFFFFFFFu : ((2u << q) - 1u)) & ~(1u << jb);
  uint32_t path = 0;
  uint32_t sk = 1u;                                   // skip[0]
  uint32_t sk1 = q > 0 ? skip_at_level(pm1, q - 1) : 1u;  // skip[1]
  const int b = (int)q - (int)jb;
  const uint32_t cap = 8u * q + 16u;
  for (uint32_t it = 0; k <= k_last && k < q; ++it) {
    if (it >= cap) { anomaly = true; break; }
    uint32_t jj, skj;
    bool post;
    if (j > q) {                     // list exhausted: return to the pending call
      if (path == 0) break;
      jj = 31u - (uint32_t)__clz((int)path);
      skj = skip_at_level(pm1, jj);
      D += skj;
      path &= ~(1u << jj);
      post = true;
    } else {
      jj = j;
      skj = skip_at_level(pm1, jj);
      const bool pass = (skj + sk <= D) && (D - skj > Sd);
      if (!pass) {
        j = next_level(live, jj);
        post = false;
      } else if (skj + sk1 <= D) {   // recursive call on r' + skip[e]
        D -= skj;
        path |= 1u << jj;
        if ((skj + sk <= D) && (D - skj > Sd)) anomaly = true;
        j = next_level(live, jj);
        post = false;
      } else {
        post = true;
      }
    }
    if (post) {
      if (D < sk1) {                 // r' > R - skip[k+1]: this frame returns
        j = kEndLevel;
      } else {                       // accept e for round k
        Sd = D - skj;
        emit(k, jj == 0 ? b : -(int)jj);
        ++k;
        sk = sk1;
        sk1 = k < q ? skip_at_level(pm1, q - k - 1) : 0xFFFFFFFFu;
        live &= ~(1u << jj);
        j = next_level(live, jj);
      }
    }
  }
  return k;
}

// Published SplitMix64 output function.
__device__ __forceinline__ uint64_t sm64(uint64_t z) {
  z += 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

struct Instance {
  uint32_t p, pm1, q, root;
};

__device__ __forceinline__ Instance make_instance(uint32_t p, uint32_t q, uint32_t root) {
  Instance in;
  in.p = p; in.pm1 = p - 1u; in.q = q; in.root = root;
  return in;
}

// (r - root + p) mod p without leaving 32 bits (Section 2: renumbering).
__device__ __forceinline__ uint32_t virtual_rank(const Instance &in, uint32_t r) {
  return r >= in.root ? r - in.root : r + (in.p - in.root);
}

struct TrackOff { static constexpr bool value = false; };
struct TrackOn { static constexpr bool value = true; };

// How far the difference x - y of a test "x >= y" is from flipping: the test keeps its outcome as
// long as the difference moves by no more than x - y (x >= y) or y - x - 1 (x < y).
// The records keep |x - y|, which is one instruction: exact for x >= y and one too many for
// x < y; every use of a margin made of these asks for one more than the shift (the "+ 1" in
// stretch_shift and in the test on the top levels), which covers it.
__device__ __forceinline__ uint32_t abs_difference(uint32_t x, uint32_t y) {
#ifdef BCAST_DEVICE_CODE_ON_HOST
  return x > y ? x - y : y - x;
#else
  uint32_t d;
  asm("v_sad_u32 %0, %1, %2, 0" : "=v"(d) : "v"(x), "v"(y));
  return d;
#endif
}

// How far the difference of any test of the lockstep stretch can move when D moves by dD and M by
// dM (as unsigned differences): its two sides are D + c, M + c or constants, so it moves by dD,
// dM, their difference, or not at all.  (M turns into a D + c or a constant along the way, which
// only makes it move less.)  Plus the one that the margins ask for.
__device__ __forceinline__ uint32_t stretch_shift(uint32_t dD, uint32_t dM) {
  auto mag = [](uint32_t d) { const int s = (int)d; return (uint32_t)(s < 0 ? -s : s); };
  const uint32_t a = mag(dD), b = mag(dM), c = mag(dD - dM);
  const uint32_t ab = a > b ? a : b;
  return (ab > c ? ab : c) + 1u;
}

// One pass over the levels j = 1 .. q, i.e. over skip[q-1] down to skip[0],
// serves three purposes at once, because all three walk down the same skips:
//   Algorithm 3: rem is what is left of v; a skip is taken when it still fits;
//     the last one taken (it brings rem to 0) is the baseblock's.
//   Algorithm 6 (kSend): its r' is the same rem, so "lower part" = skip not
//     taken; e, c and the violation tests as printed, round k = q - j.  While c
//     still stands for the baseblock, which is not known before the pass ends,
//     the entries written are placeholders (see first_level_taken).
//   Descent of the receive search (see recv_ascent): W = D - 2; a level is
//     pushed when its skip <= W, accepted for round 0 when skip = W + 1, and the
//     baseblock's level is not in the list.  A level is the baseblock's exactly
//     when it is taken and brings rem to 0, which is known on the spot.
struct TopDown {
  uint32_t rem, jb;
  bool closed;                      // the level before this one was the baseblock's
  int W;
  uint32_t pathr, anom;
  uint32_t e;
  int c;
  uint32_t viol;                    // round k at bit k - 1 after the last round
};

constexpr int kPendingB = 0;        // placeholder for "c = baseblock" inside the pass

__device__ __forceinline__ TopDown top_down_start(uint32_t p, uint32_t v) {
  const bool is_root = v == 0;
  TopDown s;
  s.rem = v; s.jb = 0; s.closed = is_root;
  // W = D - 2 as a signed number; after the accept W = -1, which neither fits
  // nor hits any more.  pathr holds the pending calls with level j at bit
  // 31 - j, so that the deepest one is the lowest set bit.  For v >= 2 the first
  // call (index q, skip p) is always recursive: the walk starts below it (and for
  // v = 1, W = -1 says that the same index was accepted: see recv_ascent).
  s.W = (int)((is_root ? p : v) - 2u);
  s.pathr = is_root ? 0u : 0x80000000u;
  s.anom = 0;
  s.e = p; s.c = kPendingB; s.viol = 0;
  return s;
}

// One level of the pass (see TopDown).
// kTrack: every test whose outcome depends on v also lowers `margin` to its
// flip distance (tests between constants of the instance are left out; a test
// that is not consulted may be included, which only makes the margin smaller).
// kDescent = false leaves the descent out (W, pathr, closed and anom are not touched): for the
// deep levels of a rank whose descent comes from the table of deep entries (see DeepEntry).
template <bool kSend, bool kTrack, bool kDescent = true, typename EmitSend>
__device__ __forceinline__ void top_down_level(uint32_t pm1, uint32_t q, uint32_t j, TopDown &s,
                                               uint32_t &margin, EmitSend emit_send) {
  auto see = [&](uint32_t x, uint32_t y) {
    if (kTrack) { const uint32_t fd = abs_difference(x, y); margin = fd < margin ? fd : margin; }
  };
  const uint32_t sk = skip_at_level(pm1, j);            // the same in all lanes: a scalar
  see(s.rem, sk);
  const bool lower = s.rem < sk;
  const uint32_t rem_new = lower ? s.rem : s.rem - sk;
  see(0u, rem_new);                                     // rem_new == 0
  if (kSend && j < q) {                                 // round k = q - j >= 1 of Algorithm 6
    const uint32_t k = q - j;
    const uint32_t skm = skip_at_level(pm1, j + 1u);    // skip[k - 1]
    const bool k_is_1 = k == 1u;
    const uint32_t s1 = s.rem + sk;
    const uint32_t em = s.e - sk;                       // meaningful in the upper part only
    see(s1, s.e);
    see(s.e, s1);
    see(s.rem, sk + 1u);
    // at k = 1: the baseblock is not 0 iff skip[0] will not be taken
    const bool ok_lower = (s1 < s.e) || (s.e < skm) || (k_is_1 && rem_new == 0u);
    const bool ok_upper = k_is_1 || (s.rem > sk) || (em < skm) || (s1 <= s.e);
    const bool bad = lower ? !ok_lower : !ok_upper;
    s.viol = (s.viol << 1) | (uint32_t)bad;
    s.c = lower ? s.c : (int)k - (int)q;
    s.e = lower ? (s.e < sk ? s.e : sk) : em;
    emit_send(k, s.c);
  }
  const bool closes = !lower && rem_new == 0u;          // this level is the baseblock's
  s.jb = lower ? s.jb : j;
  s.rem = rem_new;
  if (!kDescent) return;
  const int ski = (int)sk;
  const int t = s.W - ski;
  // the tests on t below (t >= -1, t >= 0, skip <= t + 1) between non-negative numbers: W >= -1
  const uint32_t w1 = (uint32_t)(s.W + 1);
  see(w1, sk);
  see(w1, sk + 1u);
  see(w1, 2u * sk);
  const bool take = !closes && t >= -1;                 // push (t >= 0) or accept (t = -1)
  // The call made for this index would look at the index again (skip + 1 <=
  // D - skip) and that look must fail.  It does whenever the level above was
  // looked at (skip[e+1] <= 2 skip[e]); only right below the baseblock's
  // level, which is not in the list, the test is made explicitly.
  s.anom |= (uint32_t)(s.closed && take && t >= 0 && ski <= t + 1);
  s.W = take ? t : s.W;
  s.pathr |= take ? (0x80000000u >> j) : 0u;            // the accepted level too, for now
  s.closed = closes;
}

// Rounds of Algorithm 6 at the top whose entry is the baseblock itself: those
// before the first skip that fits into v (c has not been set by an upper part
// yet).  Returns the first level taken, 1 <= jt <= q, for v >= 1.
__device__ __forceinline__ uint32_t first_level_taken(uint32_t pm1, uint32_t v) {
  // smallest j >= 1 with (pm1 >> j) + 1 <= v, i.e. (pm1 >> j) <= x = v - 1 < pm1
  const uint32_t x = v - 1u;
  const uint32_t len_p = 32u - (uint32_t)__clz((int)pm1);
  const uint32_t len_x = x == 0u ? 0u : 32u - (uint32_t)__clz((int)x);
  const uint32_t j1 = len_p - len_x;                   // (pm1 >> j1) has the length of x
  const uint32_t jt = (pm1 >> j1) <= x ? j1 : j1 + 1u;
  return jt == 0u ? 1u : jt;
}

// Number of levels at the top whose skip is at least min_skip (levels 1 .. n).
constexpr uint32_t kTopSkip = 4096u;
constexpr uint32_t kUpperSkip = 65536u;
constexpr uint32_t kCutSkip = 65536u;         // where the lockstep stretch is cut in two, see ascent_run
__device__ __forceinline__ uint32_t top_level_count(uint32_t pm1, uint32_t q, uint32_t min_skip = kTopSkip) {
  if (pm1 < min_skip) return 0u;
  // skip_at_level(j) >= min_skip  <=>  (pm1 >> j) >= min_skip - 1
  uint32_t n = 32u - (uint32_t)__clz((int)(pm1 / (min_skip - 1u)));   // first j with pm1 >> j < min_skip - 1
  n = n == 0u ? 0u : n - 1u;
  return n < q ? n : q;
}

// Cross-lane helpers for values that must be the same in all lanes.
__device__ __forceinline__ uint32_t lane0_of(uint32_t x) {
  return (uint32_t)__builtin_amdgcn_readfirstlane((int)x);
}
__device__ __forceinline__ uint32_t wave_min32(uint32_t x) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) {
    const uint32_t y = (uint32_t)__shfl_xor((int)x, m, 64);
    x = y < x ? y : x;
  }
  return x;
}

// What a wavefront remembers from one tile of its run to replay on the next
// ones: the lockstep stretch of the receive search (see recv_ascent) and the
// state after the top levels of the pass (see compute_rank_phase1).  Everything
// is kept in kRecordWords words of the wavefront's own LDS (`mem`), so that it costs no
// registers between tiles.  The lanes of a tile that records hold consecutive ranks, so what is
// a lane's own (v; D and M of the search) is the first lane's value plus the lane's number, or
// the same in all lanes, and the first lane's value stands for all of them; a tile for which
// that does not hold leaves no record.
enum RecordWord : uint32_t {
  kRecLevels = 0,                   // 32 bytes: level accepted for round k, k = k_entry .. q-1
  kRecValid = 8, kRecK, kRecLive, kRecPathr, kRecJ,   // state on entry to the stretch
  kRecMargin,                       // how far D and M may move before a test flips
  kRecIters,                        // iterations the stretch took
  kRecReplays,                      // tiles that took the record (statistics)
  kTopValid, kTopLevels,            // the top levels: valid, how many
  kTopT, kTopTw,                    // v - rem and v - W after them
  kTopJb, kTopPathr, kTopE, kTopViol, kTopBits, kTopC,   // bits: closed, anom
  kTopMargin, kTopReplays,
  kRecRowsHeld,                     // the wavefront's rows still hold the record's accepts, see ascent_run
  kRecRoundOfB,                     // the round in which the stretch accepts level 0 (block b), or none
  // the uppermost of the top levels (skips of kUpperSkip and more) once more, as a record of their own
  kUpValid, kUpLevels, kUpV0,       // valid, how many, the first lane's v when they were recorded
  kUpT, kUpTw, kUpJb, kUpPathr, kUpE, kUpViol, kUpBits, kUpC, kUpMargin,
  // the second part of the lockstep stretch (from round kMidK on) as a record of its own
  kMidValid, kMidK, kMidLive, kMidPathr, kMidJ, kMidMargin, kMidIters, kMidRoundOfB,
  kMidReplays,                      // tiles that took the second part alone (statistics)
  // D and M of the recording tile's lanes on entry to the stretch and to its second part: the
  // first lane's values; lane l had D + l and M + l (kRamp set) or M (kRamp clear)
  kRecD0, kRecM0, kRecRamp, kMidD0, kMidM0, kMidRamp,
  kTopV0,                           // the first lane's v when the top levels were recorded
  kRecordWords = 64
};
constexpr uint32_t kNoRound = 0xFFFFFFFFu;
constexpr uint32_t kWaveLanes = 64u;

// kCanSplit: the code that records the lockstep stretch in two parts is compiled in (it costs
// registers and code also where it does not run); `split` then switches it on.
template <bool kCanSplit>
struct LockstepCacheT {
  static constexpr bool can_split = kCanSplit;
  uint32_t *mem;
  uint32_t lane;                    // this lane's number in the wavefront
  bool split;                       // record the lockstep stretch in two parts (pays in long runs of tiles)
};
using LockstepCache = LockstepCacheT<false>;
using LockstepCacheSplit = LockstepCacheT<true>;

// D and M of the lanes of a wavefront as first lane's value + lane's number (D always, M if
// `ramp`) or the same in all lanes (M otherwise).  Returns whether they are of that form.
__device__ __forceinline__ bool lanes_in_a_row(uint32_t D, uint32_t M, uint32_t lane, uint32_t &D0,
                                               uint32_t &M0, uint32_t &ramp) {
  D0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)D);
  M0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)M);
  const bool flat = !__any(M != M0);
  const bool ramp_m = !__any(M - lane != M0);
  const bool ramp_d = !__any(D - lane != D0);
  ramp = flat ? 0u : 1u;
  return ramp_d && (flat || ramp_m);
}

// mem: kRecordWords words of the wavefront's own, or null for a rank on its own (no records).
template <typename Cache>
__device__ __forceinline__ void lockstep_cache_init(Cache &c, uint32_t *mem, uint32_t lane = 0u,
                                                    bool split = false) {
  c.mem = mem;
  c.lane = lane;
  c.split = split;
  if (mem != nullptr) {
    mem[kRecValid] = 0; mem[kRecReplays] = 0; mem[kTopValid] = 0; mem[kTopReplays] = 0;
    mem[kRecRowsHeld] = 0; mem[kUpValid] = 0; mem[kMidValid] = 0; mem[kMidReplays] = 0;
  }
}

// The wavefront's rows have been written by something other than its tiles (or are about to be):
// nothing that relies on entries staying in them from tile to tile may be taken over.
template <typename Cache>
__device__ __forceinline__ void lockstep_cache_rows_lost(Cache &c) {
  c.mem[kTopValid] = 0; c.mem[kUpValid] = 0; c.mem[kRecRowsHeld] = 0;
}

// The receive search again, in the form the kernels use: same state and same
// tests as recv_search, reorganised around how the search actually runs.
//
// 1. Descent.  With k = 0 the search first walks down the list once: a skip
//    that still leaves room for skip[1] = 2 is pushed (recursive call), the one
//    that lands exactly on R - 1 is accepted for round 0, everything else is
//    passed over.  With W = D - 2 this is "push if skip <= W, accept if
//    skip = W + 1".  All lanes look at the same level in the same iteration,
//    so the skip is a scalar and the body is a handful of instructions.
// 2. Ascent.  What follows is an irregular mix of returns, accepts and short
//    new descents; every lane makes whichever move its state asks for.
//
// The first call is for index q (skip p): for v >= 2 it is always a recursive
// call, so the walk starts below it with D = v and level 0 on the path; for
// the root level 0 is not in the list and the walk starts with D = p.  For
// v = 1 the first call accepts index q for round 0; the same start covers it:
// W = v - 2 = -1 reads as "accepted", no deeper level can be taken, and the
// accepted level is the deepest bit of the path, level 0, so D = p + 1.
//
// 3. Replay.  Once the lanes are in lockstep, the rest of the search is a
//    function of (k, live, path, cursor), which all lanes share, and of each
//    lane's D and M, which enter only through tests of the form x >= y where x
//    and y are D + c, M + c or constants.  The next tiles of a wavefront's run
//    usually arrive with the same shared state and with D and M moved by the
//    same small amount in every lane.  So a wavefront that runs the stretch
//    also records, per test, how far it was from flipping; a later tile whose
//    D and M differ from the recorded ones by less than the smallest such
//    distance makes the same moves, and takes the recorded accepts (level per
//    round) instead of running the loop.  The same bound, applied to the
//    differences between the lanes of the recording tile, shows that its lanes
//    did make the same moves.  The tests of the first rounds of the stretch, among
//    skips of a few thousand, flip every few tiles; those of the rounds with skips of
//    kUpperSkip and more hold for hundreds of tiles.  The stretch is therefore
//    recorded in two parts, cut where round q - (levels with such skips) begins: a
//    tile that cannot take the whole stretch over makes the moves of the first part
//    and, if it arrives at the cut in the recorded state with D and M within the
//    second part's margin, takes the second part from the record.  The whole stretch
//    can then be taken over again from this tile's D and M on entry, with what is
//    left of the second part's margin (its own less the shift at the cut; shifts
//    add up, and the shift at the cut of a later tile is no more than its shift on
//    entry, since D and M at the cut are D + c, M + c or constants too).  The second
//    part's bookkeeping costs a recording tile some instructions; wavefronts with
//    runs of a few tiles only record the stretch in one part (`split` of the cache).
//    `use_cache` = false: no replay; when it is true,
//    all lanes of the wavefront must be in the call, and every lane must pass the
//    same row to `emit` from tile to tile: the accepts of the stretch are minus the
//    level in every lane (only block b, for level 0, is the lane's own), so a tile
//    that takes the record over while the rows still hold them from the tile
//    before writes nothing but that one entry.
//
// The descent is made by the caller (top_down_level, together with Algorithms 3
// and 6, which walk over the same levels): W, pathr and anom_in are its result.
struct AscentState {
  uint32_t D, M, sk1, k, j, live, pathr;
};

// State of the search after the descent (W, pathr as top_down_level leaves them), including the
// accept at the bottom of the descent if there was one.
template <typename Emit>
__device__ __forceinline__ AscentState ascent_start(uint32_t pm1, uint32_t q, uint32_t jb, int W,
                                                    uint32_t pathr, Emit emit) {
  AscentState a;
  const bool hit = W == -1;
  // The accept, if any, was the last level taken: the deepest bit of pathr.
  const uint32_t jd = hit ? 31u - (uint32_t)(__ffs((int)pathr) - 1) : 0u;
  a.pathr = hit ? pathr & (pathr - 1u) : pathr;
  a.live = (q >= 31 ? 0xFFFFFFFFu : ((2u << q) - 1u)) & ~(1u << jb);
  a.D = hit ? (uint32_t)skip_at_level(pm1, jd) + 1u : (uint32_t)(W + 2);
  a.k = 0; a.j = kEndLevel;
  a.M = 1u;                                               // max(skip[k], Sd + 1)
  a.sk1 = 2u;                                             // skip[k + 1]
  if (hit) {                                              // round 0 accepted at level jd
    emit(0u, -(int)jd);
    a.live &= ~(1u << jd);
    a.k = 1;
    a.M = 2u;                                             // skip[1] = 2, Sd = 1
    a.sk1 = q >= 2 ? skip_at_level(pm1, q - 2) : 0xFFFFFFFFu;
    a.j = next_level(a.live, jd);
  }
  return a;
}

// Levels whose skip is below kLockstepSkip, as a mask; first_deep_level is the lowest of them.
__device__ __forceinline__ uint32_t first_deep_level(uint32_t pm1) {
  return pm1 >= kLockstepSkip ? 32u - (uint32_t)__clz((int)(pm1 / kLockstepSkip)) : 0u;
}
__device__ __forceinline__ uint32_t deep_level_mask(uint32_t pm1) {
  const uint32_t first_deep = first_deep_level(pm1);
  return first_deep < 32u ? 0xFFFFFFFFu << first_deep : 0u;
}

// The ascent from state `a` on.  kPrefix: only the first stretch (while levels with small skips
// remain), with `a` holding the state it ends in; a search that stops there because it runs out of
// pending calls is complete as far as it goes and raises nothing.
// kFlat: every move runs through one body without branches.  That costs more instructions per
// move than the one branch a wavefront in lockstep takes, and fewer than all the branches a
// wavefront of unrelated ranks takes one after the other: for lists of arbitrary ranks, for
// the searches that answer violations and for the builder of the table of deep entries.
template <bool kPrefix, bool kFlat = false, typename Emit, typename Cache>
__device__ __forceinline__ uint32_t ascent_run(uint32_t pm1, uint32_t q, uint32_t jb, uint32_t k_last,
                                               AscentState &a, uint32_t anom_in, bool &anomaly,
                                               Emit emit, Cache &cache, bool use_cache) {
  const int b = (int)q - (int)jb;
  uint32_t anom = anom_in;
  uint32_t D = a.D, M = a.M, sk1 = a.sk1, k = a.k, j = a.j, live = a.live, pathr = a.pathr;
  // Ascent.
  const uint32_t k_stop = k_last + 1u < q ? k_last + 1u : q;
  const uint32_t cap = 8u * q + 16u;
  // The ascent runs as two loops over the same body.  Lanes of a wavefront hold
  // consecutive ranks: their searches differ in the deep levels (small skips)
  // and agree, move for move, once those are all accepted.  The first loop
  // lets every lane finish its deep levels and wait; the second then runs with
  // all lanes making the same move, so each iteration takes one branch only.
  const uint32_t deep = deep_level_mask(pm1);   // levels whose skip is below kLockstepSkip
  bool go = k < k_stop && !((int)j < 0 && pathr == 0);
  uint32_t it = 0;
  uint32_t margin = 0xFFFFFFFFu;
  uint32_t b_word = kRecRoundOfB;     // where a recorded move notes the round of level 0
  // One move of the state machine.  With kTrack, every test that decides the
  // move also lowers `margin` to its flip distance.
  auto move = [&](auto track_tag) {
    constexpr bool kTrack = decltype(track_tag)::value;
    auto see = [&](uint32_t x, uint32_t y) {
      if (kTrack) { const uint32_t fd = abs_difference(x, y); margin = fd < margin ? fd : margin; }
    };
    uint32_t jj, a, t;
    bool post;
    if ((int)j < 0) {                       // list exhausted: back to the pending call
      jj = 31u - (uint32_t)(__ffs((int)pathr) - 1);
      a = skip_at_level(pm1, jj);
      t = D;                                // D - skip[e] seen from the caller's frame
      D += a;
      pathr ^= 0x80000000u >> jj;
      post = true;
    } else {
      jj = j;
      a = skip_at_level(pm1, jj);
      t = D - a;
      see(D, a);
      const bool fits = a <= D;
      if (kTrack && fits) see(t, M);
      const bool pass = fits && t >= M;
      if (kTrack && pass) see(t, sk1);
      const bool rec = pass && t >= sk1;
      post = pass && !rec;
      if (rec) {                            // recursive call on r' + skip[e]
        see(t, a);
        if (kTrack && a <= t) see(t - a, M);
        anom |= (uint32_t)(a <= t && t - a >= M);
        D = t;
        pathr |= 0x80000000u >> jj;
      }
    }
    bool ret = false;
    if (post) {
      see(D, sk1);
      if (D >= sk1) {                       // accept e for round k
        emit(k, jj == 0 ? b : -(int)jj);
        if (kTrack) {
          reinterpret_cast<uint8_t *>(cache.mem)[k] = (uint8_t)jj;
          if (jj == 0u) cache.mem[b_word] = k;
        }
        live ^= 1u << jj;
        see(sk1, t + 2u);
        M = sk1 > t + 1u ? sk1 : t + 1u;
        ++k;
        sk1 = skip_at_level(pm1, (q - k - 1u) & 31u);     // skip[k+1]; unused once k = q
      } else {
        ret = true;                         // r' > R - skip[k+1]: this frame returns
      }
    }
    j = ret ? kEndLevel : next_level(live, jj);
    go = k < k_stop && !((int)j < 0 && pathr == 0);
  };
  auto move_flat = [&]() {
    const bool pop = (int)j < 0;                          // list exhausted: back to the pending call
    const uint32_t jj = pop ? 31u - (uint32_t)(__ffs((int)pathr) - 1) : j;
    const uint32_t a = skip_at_level(pm1, jj);
    const uint32_t t = pop ? D : D - a;
    const bool pass = !pop && a <= D && t >= M;
    const bool rec = pass && t >= sk1;                    // recursive call on r' + skip[e]
    anom |= (uint32_t)(rec && a <= t && t - a >= M);
    const bool post = pop || (pass && !rec);
    const uint32_t bit = 0x80000000u >> jj;
    D = pop ? D + a : (rec ? t : D);
    pathr ^= (pop || rec) ? bit : 0u;                     // a return clears the bit, a call sets it
    const bool accept = post && D >= sk1;
    if (accept) emit(k, jj == 0 ? b : -(int)jj);
    live ^= accept ? 1u << jj : 0u;
    M = accept ? (sk1 > t + 1u ? sk1 : t + 1u) : M;
    k += (uint32_t)accept;
    sk1 = accept ? skip_at_level(pm1, (q - k - 1u) & 31u) : sk1;
    j = (post && !accept) ? kEndLevel : next_level(live, jj);
    go = k < k_stop && !((int)j < 0 && pathr == 0);
  };
  if (kFlat) {
    for (; it < cap && go && (!kPrefix || (live & deep) != 0u); ++it) move_flat();
    if (kPrefix) { a.D = D; a.M = M; a.sk1 = sk1; a.k = k; a.j = j; a.live = live; a.pathr = pathr; }
    anomaly = anomaly || anom != 0 || (!kPrefix && k < k_stop) || it >= cap;
    return k;
  }
  for (; it < cap && go && (live & deep) != 0u; ++it) move(TrackOff{});
  if (kPrefix) {
    a.D = D; a.M = M; a.sk1 = sk1; a.k = k; a.j = j; a.live = live; a.pathr = pathr;
    anomaly = anomaly || anom != 0 || it >= cap;
    return k;
  }
  // Lockstep stretch: replayed, recorded, or simply run.  (Whatever is the same in all lanes is
  // read from the first lane, so that it is held in scalar registers.)
  bool replayed = false, record = false;
  auto emit_recorded = [&](uint32_t from) {
    for (uint32_t kk = from; kk < q; ++kk) {
      const uint32_t jj = reinterpret_cast<const uint8_t *>(cache.mem)[kk];
      emit(kk, jj == 0 ? b : -(int)jj);
    }
  };
  // D - (D0 + lane), M - (M0 + lane or 0): how far this tile's lanes are from a recorded tile's
  auto shift_from = [&](uint32_t word_d0, uint32_t &dD, uint32_t &dM) {
    dD = D - (cache.mem[word_d0] + cache.lane);
    dM = M - (cache.mem[word_d0 + 1u] + (cache.mem[word_d0 + 2u] != 0u ? cache.lane : 0u));
  };
  static_assert(kRecM0 == kRecD0 + 1 && kRecRamp == kRecD0 + 2 && kMidM0 == kMidD0 + 1 && kMidRamp == kMidD0 + 2,
                "D0, M0 and the ramp flag of a record follow one another");
  uint32_t it_in = 0;
  if (use_cache && k_stop == q) {
    const uint32_t k0 = lane0_of(k), l0 = lane0_of(live), p0 = lane0_of(pathr), j0 = lane0_of(j);
    const bool shared = go && k == k0 && live == l0 && pathr == p0 && j == j0;
    if (!__any(!shared)) {
      if (cache.mem[kRecValid] && k0 == cache.mem[kRecK] && l0 == cache.mem[kRecLive] && p0 == cache.mem[kRecPathr] &&
          j0 == cache.mem[kRecJ]) {
        uint32_t dD, dM;
        shift_from(kRecD0, dD, dM);
        const uint32_t far = stretch_shift(dD, dM);
        const uint32_t dD0 = lane0_of(dD), dM0 = lane0_of(dM);   // read by all lanes, whatever the tests say
        const bool ok = dD == dD0 && dM == dM0 && far <= cache.mem[kRecMargin] &&
                        it + cache.mem[kRecIters] <= cap;
        if (!__any(!ok)) {
          if (cache.mem[kRecRowsHeld] != 0u) {
            const uint32_t kb = cache.mem[kRecRoundOfB], kb2 = cache.mem[kMidRoundOfB];
            if (kb != kNoRound) emit(kb, b);
            if (kb2 != kNoRound) emit(kb2, b);
          } else {
            emit_recorded(k0);
            cache.mem[kRecRowsHeld] = 1u;
          }
          k = q;
          it += cache.mem[kRecIters];
          go = false;
          replayed = true;
          cache.mem[kRecReplays] = cache.mem[kRecReplays] + 1u;
        }
      }
      if (!replayed) {
        // A record of the whole stretch starts here; it becomes valid at the end, if all goes well.
        record = true;
        uint32_t D0, M0, ramp;
        const bool in_a_row = lanes_in_a_row(D, M, cache.lane, D0, M0, ramp);
        cache.mem[kRecValid] = 0u;
        cache.mem[kRecK] = k0; cache.mem[kRecLive] = l0; cache.mem[kRecPathr] = p0; cache.mem[kRecJ] = j0;
        cache.mem[kRecD0] = D0; cache.mem[kRecM0] = M0; cache.mem[kRecRamp] = ramp;
        // lanes that are not in a row leave no record: a margin of 0 is never enough (see below)
        cache.mem[kRecMargin] = in_a_row ? 0xFFFFFFFFu : 0u;
        it_in = lane0_of(it);
      }
    }
  }
  // rows written by anything but this record's own accepts no longer hold them
  if (!replayed && cache.mem != nullptr) cache.mem[kRecRowsHeld] = 0u;
  if (use_cache && k_stop == q && !replayed) {
    // The moves of the first part, with their flip distances if the whole stretch can be recorded
    // (`record`: the lanes share the state on entry); lanes that have parted earlier usually
    // meet again at the cut.  The cut is the same in all lanes; a stretch that begins at or beyond
    // it, or an instance without such skips, has one part only.
    const uint32_t k_cut = q - top_level_count(pm1, q, kCutSkip);
    const bool two_parts = Cache::can_split && cache.split && k_cut < q && !__any(go && k >= k_cut);
    b_word = kRecRoundOfB;
    if (record) {
      cache.mem[kRecRoundOfB] = kNoRound;
      if (!two_parts) { cache.mem[kMidRoundOfB] = kNoRound; cache.mem[kMidValid] = 0u; }   // its accepts are overwritten
      for (; it < cap && go && (!two_parts || k < k_cut); ++it) move(TrackOn{});
    } else {
      for (; it < cap && go && (!two_parts || k < k_cut); ++it) move(TrackOff{});
    }
    // the smallest flip distance of the first part over all lanes (only a recording tile has one)
    const uint32_t m_first = record ? lane0_of(wave_min32(margin)) : 0u;
    uint32_t second_left = 0xFFFFFFFFu;        // how far the entry state may still move for the second part
    bool second_fine = true;                   // the second part is known to hold for all lanes of this tile
    if (two_parts) {
      margin = 0xFFFFFFFFu;
      const uint32_t kc = lane0_of(k), lc = lane0_of(live), pc = lane0_of(pathr), jc = lane0_of(j);
      const bool at_cut = go && k == kc && live == lc && pathr == pc && j == jc;
      bool taken = false;
      if (!__any(!at_cut)) {
        if (cache.mem[kMidValid] && kc == cache.mem[kMidK] && lc == cache.mem[kMidLive] && pc == cache.mem[kMidPathr] &&
            jc == cache.mem[kMidJ]) {
          uint32_t dD, dM;
          shift_from(kMidD0, dD, dM);
          const uint32_t far = stretch_shift(dD, dM);
          const uint32_t dD0 = lane0_of(dD), dM0 = lane0_of(dM);
          const bool ok = dD == dD0 && dM == dM0 && far <= cache.mem[kMidMargin] &&
                          it + cache.mem[kMidIters] <= cap;
          if (!__any(!ok)) {
            emit_recorded(kc);
            k = q;
            it += cache.mem[kMidIters];
            go = false;
            taken = true;
            second_left = cache.mem[kMidMargin] - lane0_of(far);
            cache.mem[kMidReplays] = cache.mem[kMidReplays] + 1u;
          }
        }
        if (!taken) {                            // the second part by its moves, recorded
          uint32_t D0, M0, ramp;
          const bool in_a_row = lanes_in_a_row(D, M, cache.lane, D0, M0, ramp);
          const uint32_t it_cut = lane0_of(it);
          cache.mem[kMidValid] = 0u;
          cache.mem[kMidK] = kc; cache.mem[kMidLive] = lc; cache.mem[kMidPathr] = pc; cache.mem[kMidJ] = jc;
          cache.mem[kMidD0] = D0; cache.mem[kMidM0] = M0; cache.mem[kMidRamp] = ramp;
          // a record of the whole stretch made by an earlier tile ends in the accepts overwritten now
          if (!record) cache.mem[kRecValid] = 0u;
          b_word = kMidRoundOfB;
          cache.mem[kMidRoundOfB] = kNoRound;
          for (; it < cap && go; ++it) move(TrackOn{});
          const uint32_t m_all = lane0_of(wave_min32(margin));
          const bool fine = k == q && anom == 0;
          // lanes in a row are at most 63 apart in D and M: stretch_shift(63, 0 or 63) = 64
          second_fine = in_a_row && !__any(!fine) && (uint32_t)kWaveLanes <= m_all;
          cache.mem[kMidValid] = (uint32_t)second_fine;
          cache.mem[kMidMargin] = m_all;
          cache.mem[kMidIters] = lane0_of(it) - it_cut;
          second_left = m_all;
        }
      } else {                                   // the lanes are not together at the cut: to the end as they are
        for (; it < cap && go; ++it) move(TrackOff{});
        second_fine = false;
      }
    }
    if (record) {
      // usable as a whole if it ran to the end without incident and no lane can have left the others
      const uint32_t m_both = m_first < second_left ? m_first : second_left;
      const uint32_t m_all = cache.mem[kRecMargin] < m_both ? cache.mem[kRecMargin] : m_both;   // 0: not in a row
      const bool fine = k == q && anom == 0;
      cache.mem[kRecValid] = (uint32_t)(second_fine && !__any(!fine) && (uint32_t)kWaveLanes <= m_all);
      cache.mem[kRecMargin] = m_all;
      cache.mem[kRecIters] = lane0_of(it) - it_in;
      cache.mem[kRecRowsHeld] = cache.mem[kRecValid];    // all 64 rows hold the accepts of both parts now
    }
  } else {
    for (; it < cap && go; ++it) move(TrackOff{});
  }
  anomaly = anomaly || anom != 0 || (k < k_stop);
  return k;
}

template <bool kFlat = false, typename Emit, typename Cache>
__device__ __forceinline__ uint32_t recv_ascent(uint32_t p, uint32_t pm1, uint32_t q,
                                                uint32_t jb, uint32_t k_last, int W,
                                                uint32_t pathr, uint32_t anom_in,
                                                bool &anomaly, Emit emit,
                                                Cache &cache, bool use_cache) {
  (void)p;
  AscentState a = ascent_start(pm1, q, jb, W, pathr, emit);
  return ascent_run<false, kFlat>(pm1, q, jb, k_last, a, anom_in, anomaly, emit, cache, use_cache);
}

// Table of deep entries.
//
// The levels whose skip is below kLockstepSkip ("deep" levels, first_deep_level .. q) see of a rank
// v only rho, what Algorithm 3 has left of v after the levels above them (rho < S, S the smallest
// skip above the deep levels): for rho >= 2 the baseblock's level is a deep one and a function of
// rho, the descent of the receive search arrives there with W = rho - 2, and the search then moves
// among the deep levels exactly as it does for every other rank with the same rho, until it has
// to go back to a call that is pending at a level above them (or has accepted all deep levels).
// That stretch, the same for some p / S ranks, is computed once per rho and kept in a table in
// device memory: the level of the baseblock, the levels accepted for rounds 0 .. K-1, and the
// state in which the search goes on (remaining deep levels, D, M; the cursor is past the end of
// the list and no deep call is pending).  16 bytes per rho:
//   x: bits 0-10 remaining deep levels (bit i: level first_deep + i), 11-14 baseblock's level
//      - first_deep, 15-18 K, 19-29 the deep levels Algorithm 3 takes (same numbering), bit 31 valid
//   y: D | M << 16
//   z, w: accepted levels - first_deep, four bits each, round k at nibble k (z: rounds 0-7);
//      w bits 16-26: the violations of Algorithm 6 in the deep rounds (as top_down_level collects
//      them: the round of level j at bit q - 1 - j) for a rank that arrives with e = S
// Algorithm 6 sees more of a rank than rho in these rounds: its e.  After the levels above, e is
// S less the number of odd skips met on the way: S itself for half of all ranks (for all of them
// when every skip is a power of two); those take the violations from the entry and the blocks to
// send from the levels taken (c is minus the last level taken, or what it was above), the others
// walk through the rounds.
// rho < 2 (the baseblock's level lies above, or the descent has ended there) has no entry: such
// ranks take the levels one by one.
//
// Ranks that arrive with a smaller e (a quarter with S - 1, an eighth with S - 2, ...; never less
// than S minus the number of levels above) find the violations of their deep rounds in a second
// table, one 16-bit word per (S - e, rho): bit 15 valid, bits 0-10 as in w above.
struct DeepTable {
  const uint4 *entries;             // kDeepMaxEntries of them, or null
  const uint16_t *viol_by_e;        // [kDeepEs][kDeepMaxEntries], row S - e (row 0 is not used), or null
  uint32_t first_deep;              // first deep level (>= 5 when the table is in use)
  uint32_t n_rho;                   // S: entries exist for rho < S
};

constexpr uint32_t kDeepMaxEntries = 2u * kLockstepSkip + 2u;   // S <= 2 kLockstepSkip + 1
constexpr uint32_t kDeepMinUpperLevels = 4u;
constexpr uint32_t kDeepEs = 32u;                               // S - e < kDeepEs has a row

__device__ __forceinline__ uint32_t deep_table_rhos(uint32_t pm1, uint32_t first_deep) {
  return first_deep >= 1u ? skip_at_level(pm1, first_deep - 1u) : 0u;
}

// The entry of rho, computed the way every rank with that rho would: the deep levels of the pass
// from the state in which the levels above leave them, then the search while it stays among
// the deep levels.
__device__ __forceinline__ uint4 deep_entry_build(uint32_t pm1, uint32_t q, uint32_t first_deep,
                                                  uint32_t rho) {
  uint4 e;
  e.x = 0; e.y = 0; e.z = 0; e.w = 0;
  if (rho < 2u) return e;
  TopDown s;
  s.rem = rho; s.jb = 0; s.closed = false;
  s.W = (int)rho - 2;
  s.pathr = 0; s.anom = 0; s.c = 0; s.viol = 0;
  s.e = deep_table_rhos(pm1, first_deep);              // S: Algorithm 6's e of half of all ranks
  uint32_t unused = 0, taken = 0;
  for (uint32_t j = first_deep; j <= q; ++j) {
    const uint32_t before = s.rem;
    top_down_level<true, false>(pm1, q, j, s, unused, [](uint32_t, int) {});
    taken |= (uint32_t)(s.rem != before) << (j - first_deep);
  }
  uint32_t lv_lo = 0, lv_hi = 0, n_out = 0;
  bool all_deep = true;
  auto note = [&](uint32_t k, int val) {
    const uint32_t level = (uint32_t)(-val);
    all_deep = all_deep && val < 0 && level >= first_deep && level - first_deep < 16u && k == n_out;
    const uint32_t nib = (level - first_deep) & 15u;
    if (k < 8u) lv_lo |= nib << (4u * k);
    else if (k < 16u) lv_hi |= nib << (4u * (k - 8u));
    ++n_out;
  };
  AscentState a = ascent_start(pm1, q, s.jb, s.W, s.pathr, note);
  bool anomaly = false;
  LockstepCache none;
  lockstep_cache_init(none, nullptr);
  // (the lanes of the builder hold unrelated rho: one branch-free body serves them best)
  ascent_run<true, true>(pm1, q, s.jb, q - 1u, a, s.anom, anomaly, note, none, false);
  const uint32_t live_deep = a.live >> first_deep;
  const bool ok = !anomaly && all_deep && s.rem == 0u && s.jb >= first_deep && s.jb - first_deep < 16u &&
                  a.pathr == 0u && (int)a.j < 0 && a.k == n_out && a.k <= 11u && a.k < q &&
                  live_deep < 2048u && a.D < 65536u && a.M < 65536u && taken < 2048u && s.viol < 2048u &&
                  (a.live & ((1u << first_deep) - 1u)) == ((1u << first_deep) - 1u);
  if (!ok) return e;
  e.x = live_deep | ((s.jb - first_deep) << 11) | (a.k << 15) | (taken << 19) | 0x80000000u;
  e.y = a.D | (a.M << 16);
  e.z = lv_lo; e.w = lv_hi | (s.viol << 16);
  return e;
}

// The violations of Algorithm 6 in the deep rounds of a rank that arrives at the deep levels with
// remainder rho and e = S - less, as a word of the second table: the same walk as the rank's own.
__device__ __forceinline__ uint16_t deep_viol_build(uint32_t pm1, uint32_t q, uint32_t first_deep,
                                                    uint32_t rho, uint32_t less) {
  const uint32_t S = deep_table_rhos(pm1, first_deep);
  if (rho < 2u || less >= S) return 0;
  TopDown s;
  s.rem = rho; s.jb = 0; s.closed = false;
  s.W = 0; s.pathr = 0; s.anom = 0; s.c = 0; s.viol = 0;
  s.e = S - less;
  uint32_t unused = 0;
  for (uint32_t j = first_deep; j <= q; ++j)
    top_down_level<true, false, false>(pm1, q, j, s, unused, [](uint32_t, int) {});
  return s.viol < 2048u ? (uint16_t)(s.viol | 0x8000u) : (uint16_t)0;
}

// Phase one of a rank: baseblock, receive schedule, send walk.  Writes
// recvblock[k] to recv_row[k] and sendblock[k] to send_row[k] (bytes), returns
// the mask of violation rounds still to be filled in, the baseblock and flags.
// `cache` is the wavefront's lockstep record; use_cache may be true only when
// all 64 lanes make this call together (a full tile).
//
// kMemo: the deep levels come from the table of deep entries (see DeepTable) wherever the rank
// has an entry, and the levels above them are all recorded and taken over together.  `room` then
// says how far above v the ranks still make the same decisions at the levels above the deep ones
// (their rho is rho(v) plus the distance), which is what answering a violation from the table
// needs; `rho` is v's own.
struct MemoOut {
  uint32_t rho, room;
};

template <bool kMemo, bool kFlat = false, typename Cache>
__device__ __forceinline__ uint32_t compute_rank_phase1(const Instance &in, uint32_t v,
                                                        int8_t *recv_row, int8_t *send_row,
                                                        int &b_out, uint32_t &flags,
                                                        Cache &cache, bool use_cache,
                                                        const DeepTable &table, MemoOut &memo) {
  const uint32_t q = in.q;
  flags = 0;
  b_out = 0;
  memo.rho = 0; memo.room = 0;
  if (q == 0) return 0;
  auto put_send = [&](uint32_t k, int val) { send_row[k] = (int8_t)val; };
  auto put_recv = [&](uint32_t k, int val) { recv_row[k] = (int8_t)val; };
  TopDown s = top_down_start(in.p, v);
  // the root and rank 1 start differently: their tile runs without the record
  const bool use = use_cache && !__any(v <= 1u);
  uint32_t j = 1, unused = 0;
  // Top levels.  64 consecutive ranks, and the ranks of the next tiles, make the same
  // decisions at the large skips; after them rem = v - T and W = v - Tw with the same T and
  // Tw, and everything else is a constant.  A tile that runs these levels records that state
  // (if it is indeed the same in all lanes) and how far v may move before any test flips; a
  // later tile whose ranks are closer than that takes the state over.  Its rows still hold
  // the top rounds of Algorithm 6 from the recording tile, which are what it would write.
  const uint32_t n_upper = kMemo ? table.first_deep - 1u : 0u;     // levels above the deep ones
  const uint32_t n_top = kMemo ? (use ? n_upper : 0u) : (use ? top_level_count(in.pm1, q) : 0u);
  uint32_t margin_own = 0xFFFFFFFFu;         // kMemo: flip distance of this lane's own tests
  bool took_over = false;
  if (n_top >= 4u) {
    // the lanes of a tile that uses the records hold consecutive v: the first lane's stands for all
    const uint32_t v0 = lane0_of(v);
    const bool in_a_row = v - cache.lane == v0;
    const uint32_t away = abs_difference(v0, cache.mem[kTopV0]);
    const bool near = cache.mem[kTopValid] != 0u && cache.mem[kTopLevels] == n_top && in_a_row &&
                      away + 1u <= cache.mem[kTopMargin];
    if (!__any(!near)) {
      s.rem = v - cache.mem[kTopT];
      s.W = (int)(v - cache.mem[kTopTw]);
      s.jb = cache.mem[kTopJb]; s.pathr = cache.mem[kTopPathr]; s.e = cache.mem[kTopE]; s.c = (int)cache.mem[kTopC];
      s.viol = cache.mem[kTopViol];
      s.closed = (cache.mem[kTopBits] & 1u) != 0u;
      s.anom = cache.mem[kTopBits] >> 1;
      cache.mem[kTopReplays] = cache.mem[kTopReplays] + 1u;
      took_over = true;
      if (kMemo) margin_own = cache.mem[kTopMargin] - away;     // >= 1: what is left of the margin
    } else {
      uint32_t margin = 0xFFFFFFFFu;
      // The decisions that flip from one tile to the next are nearly always those at the smaller
      // of these skips: the levels with skips of kUpperSkip and more are recorded once more on
      // their own, and a tile that cannot take all the top levels over usually still takes those
      // (their rounds of Algorithm 6 are in the rows from the tile that recorded them).  The lanes
      // of such a tile hold consecutive v, so the first lane's v stands for all of them.
      const uint32_t n_up = top_level_count(in.pm1, q, kUpperSkip);
      if (n_up >= 4u && n_up < n_top) {
        const uint32_t away_up = abs_difference(v0, cache.mem[kUpV0]);
        const bool near_up = cache.mem[kUpValid] != 0u && cache.mem[kUpLevels] == n_up && in_a_row &&
                             away_up + 1u <= cache.mem[kUpMargin];
        if (!__any(!near_up)) {
          s.rem = v - cache.mem[kUpT];
          s.W = (int)(v - cache.mem[kUpTw]);
          s.jb = cache.mem[kUpJb]; s.pathr = cache.mem[kUpPathr]; s.e = cache.mem[kUpE]; s.c = (int)cache.mem[kUpC];
          s.viol = cache.mem[kUpViol];
          s.closed = (cache.mem[kUpBits] & 1u) != 0u;
          s.anom = cache.mem[kUpBits] >> 1;
          margin = cache.mem[kUpMargin] - away_up;                // >= 1: what is left of their margin
        } else {
          for (; j <= n_up; ++j) top_down_level<true, true>(in.pm1, q, j, s, margin, put_send);
          const uint32_t T = v - s.rem, Tw = v - (uint32_t)s.W;
          const uint32_t bits = (uint32_t)s.closed | (s.anom << 1);
          const uint32_t T0 = lane0_of(T), Tw0 = lane0_of(Tw), jb0 = lane0_of(s.jb), pathr0 = lane0_of(s.pathr),
                         e0 = lane0_of(s.e), c0 = lane0_of((uint32_t)s.c), viol0 = lane0_of(s.viol),
                         bits0 = lane0_of(bits);
          const bool same = in_a_row && T == T0 && Tw == Tw0 && s.jb == jb0 && s.pathr == pathr0 && s.e == e0 &&
                            (uint32_t)s.c == c0 && s.viol == viol0 && bits == bits0;
          cache.mem[kUpValid] = (uint32_t)!__any(!same);
          cache.mem[kUpLevels] = n_up;
          cache.mem[kUpV0] = v0;
          cache.mem[kUpT] = T0; cache.mem[kUpTw] = Tw0; cache.mem[kUpJb] = jb0;
          cache.mem[kUpPathr] = pathr0; cache.mem[kUpE] = e0;
          cache.mem[kUpC] = c0; cache.mem[kUpViol] = viol0;
          cache.mem[kUpBits] = bits0;
          cache.mem[kUpMargin] = wave_min32(margin);
        }
        j = n_up + 1u;
      }
      for (; j <= n_top; ++j) top_down_level<true, true>(in.pm1, q, j, s, margin, put_send);
      const uint32_t T = v - s.rem, Tw = v - (uint32_t)s.W;
      const uint32_t bits = (uint32_t)s.closed | (s.anom << 1);
      // lane 0's values, read by all lanes before any of them is compared
      const uint32_t T0 = lane0_of(T), Tw0 = lane0_of(Tw), jb0 = lane0_of(s.jb), pathr0 = lane0_of(s.pathr),
                     e0 = lane0_of(s.e), c0 = lane0_of((uint32_t)s.c), viol0 = lane0_of(s.viol),
                     bits0 = lane0_of(bits);
      const bool same = in_a_row && T == T0 && Tw == Tw0 && s.jb == jb0 && s.pathr == pathr0 && s.e == e0 &&
                        (uint32_t)s.c == c0 && s.viol == viol0 && bits == bits0;
      cache.mem[kTopValid] = (uint32_t)!__any(!same);
      cache.mem[kTopLevels] = n_top;
      cache.mem[kTopV0] = v0;
      cache.mem[kTopT] = T0; cache.mem[kTopTw] = Tw0; cache.mem[kTopJb] = jb0;
      cache.mem[kTopPathr] = pathr0; cache.mem[kTopE] = e0;
      cache.mem[kTopC] = c0; cache.mem[kTopViol] = viol0;
      cache.mem[kTopBits] = bits0;
      cache.mem[kTopMargin] = wave_min32(margin);
      margin_own = margin;
    }
    j = n_top + 1u;
  }
  bool anomaly = false;
  uint32_t produced;
  if (!kMemo) {
    for (; j <= q; ++j) top_down_level<true, false>(in.pm1, q, j, s, unused, put_send);
  } else {
    // levels above the deep ones that no record covers (short runs, partial tiles, the first
    // ranks): one by one, keeping track of how far the decisions hold
    if (!took_over && j <= n_upper) {
      uint32_t margin = 0xFFFFFFFFu;
      for (; j <= n_upper; ++j) top_down_level<true, true>(in.pm1, q, j, s, margin, put_send);
      margin_own = margin;
    }
    j = n_upper + 1u;
    const uint32_t rho = s.rem;
    memo.rho = rho;
    memo.room = margin_own - 1u;                       // margin_own >= 1 (0 only if a test sat on its edge)
    memo.room = margin_own == 0u ? 0u : memo.room;
    bool generic = rho >= 2u && rho < table.n_rho && (uint32_t)s.W == rho - 2u && !s.closed;
    uint4 e;
    e.x = 0; e.y = 0; e.z = 0; e.w = 0;
    if (generic) e = table.entries[rho];
    generic = generic && (e.x >> 31) != 0u;
    AscentState a;
    if (generic) {
      // the descent and Algorithm 3's baseblock come from the entry, and so do the deep rounds
      // of Algorithm 6: what they send follows from the levels taken, their violations are in the
      // entry for a rank that arrives with e = S and in the second table for a smaller e
      // (Algorithm 6 walks through them if there is no such word)
      const uint32_t fd = table.first_deep;
      const uint32_t less = table.n_rho - s.e;                             // e <= S
      uint32_t deep_viol = 0x8000u | ((e.w >> 16) & 0x7FFu);
      if (less != 0u)
        deep_viol = less < kDeepEs && table.viol_by_e != nullptr ? table.viol_by_e[less * kDeepMaxEntries + rho] : 0u;
      if ((deep_viol & 0x8000u) != 0u) {
        const uint32_t taken = (e.x >> 19) & 0x7FFu;
        for (; j < q; ++j) {
          const uint32_t upto = taken & ((2u << (j - fd)) - 1u);         // levels taken so far
          const int last = (int)(fd + 31u) - (int)__clz((int)upto);      // the last of them
          s.c = upto != 0u ? -last : s.c;
          send_row[q - j] = (int8_t)s.c;
        }
        s.viol = (s.viol << (q - fd)) | (deep_viol & 0x7FFu);
      } else {
        for (; j <= q; ++j) top_down_level<true, false, false>(in.pm1, q, j, s, unused, put_send);
      }
      s.jb = fd + ((e.x >> 11) & 15u);
      const uint32_t n_acc = (e.x >> 15) & 15u;
      for (uint32_t k = 0; k < n_acc; ++k) {
        const uint32_t nib = k < 8u ? (e.z >> (4u * k)) & 15u : (e.w >> (4u * (k - 8u))) & 15u;
        recv_row[k] = (int8_t)(-(int)(fd + nib));
      }
      a.D = e.y & 0xFFFFu; a.M = e.y >> 16;
      a.k = n_acc;
      a.sk1 = skip_at_level(in.pm1, (q - n_acc - 1u) & 31u);    // skip[K + 1]; K < q
      a.j = kEndLevel;
      a.live = ((1u << fd) - 1u) | ((e.x & 0x7FFu) << fd);
      a.pathr = s.pathr;
    } else {
      for (; j <= q; ++j) top_down_level<true, false>(in.pm1, q, j, s, unused, put_send);
      a = ascent_start(in.pm1, q, s.jb, s.W, s.pathr, put_recv);
    }
    produced = ascent_run<false>(in.pm1, q, s.jb, q - 1u, a, s.anom, anomaly, put_recv, cache, use);
  }
  const uint32_t jb = s.jb;
  const int b = (int)q - (int)jb;
  b_out = b;
  uint32_t viol = s.viol << 1;                  // round k at bit k
  if (v == 0) {                                 // the root sends block k in round k
    for (uint32_t k = 0; k < q; ++k) send_row[k] = (int8_t)k;
    viol = 0;
  } else {
    // the rounds above the first skip taken send the baseblock; so does round 0 (Condition 4)
    const uint32_t jt = first_level_taken(in.pm1, v);
    for (uint32_t j = 1; j < jt; ++j) send_row[q - j] = (int8_t)b;
    send_row[0] = (int8_t)(b - (int)q);
  }
  if (!kMemo)
    produced = recv_ascent<kFlat>(in.p, in.pm1, q, jb, q - 1u, s.W, s.pathr, s.anom, anomaly, put_recv,
                                  cache, use);
  if (produced != q || anomaly) flags |= BCAST_F_SEARCH;
  if (__popc(viol) > 4) flags |= BCAST_F_VIOLATIONS;
  return viol;
}

// Without the table of deep entries.
template <typename Cache>
__device__ __forceinline__ uint32_t compute_rank_phase1(const Instance &in, uint32_t v,
                                                        int8_t *recv_row, int8_t *send_row,
                                                        int &b_out, uint32_t &flags,
                                                        Cache &cache, bool use_cache) {
  DeepTable none;
  none.entries = nullptr; none.viol_by_e = nullptr; none.first_deep = 0; none.n_rho = 0;
  MemoOut unused;
  return compute_rank_phase1<false>(in, v, recv_row, send_row, b_out, flags, cache, use_cache, none, unused);
}

// A violation of Algorithm 6 in round k answered from the table of deep entries: the
// to-processor t = v + skip[k] makes the same decisions as v at the levels above the deep ones
// (skip[k] <= room), so its rho is rho(v) + skip[k], and recvblock[k] of t is in its entry if the
// entry reaches round k.  Returns the violations that are still open.
__device__ __forceinline__ uint32_t resolve_from_table(const Instance &in, const DeepTable &table,
                                                       uint32_t v, const MemoOut &memo,
                                                       uint32_t viol, int8_t *send_row) {
  uint32_t open = 0;
  while (viol != 0) {
    const uint32_t k = (uint32_t)(__ffs((int)viol) - 1);
    viol &= viol - 1u;
    const uint32_t sk = skip_at_level(in.pm1, in.q - k);
    const uint32_t rho_t = memo.rho + sk;
    bool done = false;
    if (sk <= memo.room && rho_t < table.n_rho && rho_t >= 2u && v + sk < in.p && k < 12u) {
      const uint4 e = table.entries[rho_t];
      const uint32_t n_acc = (e.x >> 15) & 15u;
      if ((e.x >> 31) != 0u && k < n_acc) {
        const uint32_t nib = k < 8u ? (e.z >> (4u * k)) & 15u : (e.w >> (4u * (k - 8u))) & 15u;
        send_row[k] = (int8_t)(-(int)(table.first_deep + nib));
        done = true;
      }
    }
    if (!done) open |= 1u << k;
  }
  return open;
}

// Phase two, for tiles of consecutive ranks: a violation in round k needs
// recvblock[k] of rank r + skip[k].  If that rank sits skip[k] lanes further in
// the same tile, or in the following tile of 64 ranks whose rows are still in
// LDS, its row is read instead of recomputed.  tile_recv and next_recv point at
// the receive row of lane 0 of the two tiles (next_recv may be null); rows are
// row_pitch and next_pitch bytes apart, and of the following tile's rows only rounds
// 0 .. next_pitch - 1 are there (eight are enough: skip[8] > 128 reaches further).  Returns the violations that are still
// open.  Call after phase one of the tile is complete and visible.
__device__ __forceinline__ uint32_t resolve_from_tiles(const Instance &in, uint32_t viol,
                                                       int8_t *send_row, const int8_t *tile_recv,
                                                       const int8_t *next_recv, uint32_t row_pitch,
                                                       uint32_t next_pitch, uint32_t lane,
                                                       uint32_t n_valid, uint32_t n_valid_next) {
  uint32_t open = 0;
  while (viol != 0) {
    const uint32_t k = (uint32_t)(__ffs((int)viol) - 1);
    viol &= viol - 1u;
    const uint32_t tl = lane + skip_at_level(in.pm1, in.q - k);   // < 2^32: lane < 64, skip < 2^31
    if (tl < n_valid) send_row[k] = tile_recv[tl * row_pitch + k];
    else if (next_recv != nullptr && n_valid == 64u && tl - 64u < n_valid_next && k < next_pitch)
      send_row[k] = next_recv[(tl - 64u) * next_pitch + k];
    else open |= 1u << k;
  }
  return open;
}

// recvblock[k] of virtual rank t alone, by a receive search that stops once
// entry k is out: what a violation of Algorithm 6 in round k asks for.
template <bool kFlat = false>
__device__ __forceinline__ int search_entry(const Instance &in, uint32_t t, uint32_t k,
                                            uint32_t &flags) {
  const uint32_t q = in.q;
  TopDown s = top_down_start(in.p, t);
  uint32_t unused = 0;
  for (uint32_t j = 1; j <= q; ++j)
    top_down_level<false, false>(in.pm1, q, j, s, unused, [](uint32_t, int) {});
  const uint32_t jbt = s.jb;
  int val = 0;
  bool anomaly_t = false;
  auto take = [&](uint32_t kk, int x) { if (kk == k) val = x; };
  uint32_t got;
  LockstepCache none;
  lockstep_cache_init(none, nullptr);
  got = recv_ascent<kFlat>(in.p, in.pm1, q, jbt, k, s.W, s.pathr, s.anom, anomaly_t, take, none, false);
  if (got <= k || anomaly_t) flags |= BCAST_F_SEARCH;
  return val;
}

// The to-processor of virtual rank v in round k.
__device__ __forceinline__ uint32_t to_processor(const Instance &in, uint32_t v, uint32_t k) {
  const uint32_t t = v + skip_at_level(in.pm1, in.q - k);
  return t >= in.p ? t - in.p : t;
}

// Phase three: the remaining violations of Algorithm 6, each by its own search.
template <bool kFlat = false>
__device__ __forceinline__ uint32_t resolve_by_search(const Instance &in, uint32_t v,
                                                      uint32_t viol, int8_t *send_row) {
  uint32_t flags = 0;
  while (viol != 0) {
    const uint32_t k = (uint32_t)(__ffs((int)viol) - 1);
    viol &= viol - 1u;
    send_row[k] = (int8_t)search_entry<kFlat>(in, to_processor(in, v, k), k, flags);
  }
  return flags;
}

// All phases for a rank on its own (no neighbours to borrow from).
__device__ __forceinline__ uint32_t compute_rank(const Instance &in, uint32_t v,
                                                 int8_t *recv_row, int8_t *send_row,
                                                 int &b_out) {
  uint32_t flags;
  LockstepCache none;
  lockstep_cache_init(none, nullptr);
  const uint32_t viol = compute_rank_phase1(in, v, recv_row, send_row, b_out, flags, none, false);
  return flags | resolve_by_search(in, v, viol, send_row);
}

// Four (two) bytes of a row.  The kernels keep rows at 4-byte aligned addresses in LDS and read
// them with aligned 4-byte loads wherever they can: loads from odd addresses, and wide loads from
// addresses that are only 2-byte aligned, take several passes there (measured: reading rows of
// 62 bytes packed back to back that way cost more than the byte loads it replaced).
__device__ __forceinline__ uint32_t row_word(const int8_t *at) {
  uint32_t w;
  __builtin_memcpy(&w, at, 4);
  return w;
}
__device__ __forceinline__ uint32_t row_half(const int8_t *at) {
  uint16_t w;
  __builtin_memcpy(&w, at, 2);
  return w;
}
// Bytes shift .. shift + 3 (shift = 0..3) of the eight bytes lo, hi.
__device__ __forceinline__ uint32_t bytes_from(uint32_t hi, uint32_t lo, uint32_t shift) {
#ifdef BCAST_DEVICE_CODE_ON_HOST
  return (uint32_t)((((uint64_t)hi << 32) | lo) >> (8u * (shift & 3u)));
#else
  return __builtin_amdgcn_alignbyte(hi, lo, shift);
#endif
}

// Invariant flags of one rank from its 2q bytes, as they are defined, for any bytes at all:
// row[0..q-1] = recvblock, row[q..2q-1] = sendblock.
//   range:        an entry outside [-q, q-1];
//   Condition 3:  the q receive entries are not, each once, {-q..-1} without b - q plus b
//                 (the root: {-q..-1}); values v in range are bit v + q of a 64-bit set, and q
//                 entries make the wanted set of q values only if they are distinct and in range;
//   first send:   sendblock[0] is not b - q (the root: some sendblock[k] is not k);
//   Condition 4:  some sendblock[k], k >= 1, of a rank other than the root is neither b - q nor
//                 among recvblock[0..k-1].
// The kernels get here for the root's wavefront only (see row_flags_clear), so the plain
// quadratic form of Condition 4 is good enough.
__device__ __forceinline__ uint32_t row_flags_entrywise(const Instance &in, uint32_t v, int b,
                                                        const int8_t *row) {
  const int q = (int)in.q;
  const bool is_root = v == 0;
  const int8_t *send = row + q;
  bool out_of_range = false, recv_in_range = true;
  uint64_t got = 0;
  for (int k = 0; k < q; ++k) {
    const int rv = row[k], sv = send[k];
    const bool r_ok = rv >= -q && rv <= q - 1, s_ok = sv >= -q && sv <= q - 1;
    out_of_range = out_of_range || !r_ok || !s_ok;
    recv_in_range = recv_in_range && r_ok;
    if (r_ok) got |= 1ull << (uint32_t)(rv + q);
  }
  const uint64_t negatives = (1ull << q) - 1ull;     // q <= 31
  const uint64_t want = is_root ? negatives : ((negatives & ~(1ull << b)) | (1ull << (q + b)));
  bool bad_s0 = false, bad_c4 = false;
  if (is_root) {
    for (int k = 0; k < q; ++k) bad_s0 = bad_s0 || (int)send[k] != k;
  } else {
    bad_s0 = q > 0 && (int)send[0] != b - q;
    for (int k = 1; k < q; ++k) {
      bool had = (int)send[k] == b - q;
      for (int j = 0; j < k; ++j) had = had || row[j] == send[k];
      bad_c4 = bad_c4 || !had;
    }
  }
  return (recv_in_range && got == want ? 0u : BCAST_F_COND3) | (bad_s0 ? BCAST_F_SEND0 : 0u) |
         (bad_c4 ? BCAST_F_COND4 : 0u) | (out_of_range ? BCAST_F_RANGE : 0u);
}

// Whether all four flags of a rank other than the root are clear, with fewer operations than
// the entry-by-entry form: true exactly when that form returns 0.
//
// If every byte of the row is a six-bit value with its sign extended (bits 7..5 alike: one test
// over the words of the row), a value is known by its low six bits, and those serve as the bit
// number in the 64-bit set as they are: the shifts take their amount modulo 64.  The set starts
// as {b - q}; a send entry of round k >= 1 must be in it when its round begins, a receive entry
// joins it; in the end it must be {-q..-1} + {b}, q + 1 values.  The q receive entries can only
// get it there by being distinct, in that set and none of them b - q (Condition 3, and in
// range); a send entry found in the set is in range as well; sendblock[0] must be b - q.
__device__ __forceinline__ bool row_flags_clear(uint32_t q, int b, const int8_t *row) {
  const int8_t *send = row + q;
  // the send part starts q bytes into the row: its words are cut from aligned ones
  const int8_t *send_words = row + (q & ~3u);
  const uint32_t cut = q & 3u;
  uint64_t have = 1ull << ((uint32_t)(b - (int)q) & 63u);
  uint32_t spread = 0;                               // bits 7 and 6 of a byte: b7 ^ b6, b6 ^ b5
  // Round 0 needs no case of its own: sendblock[0] has to be b - q, which is in the set.
  uint32_t in_have = 1u;
  uint32_t k = 0;
  uint32_t lo = q >= 4u ? row_word(send_words) : 0u;
  for (; k + 4u <= q; k += 4u) {
    const uint32_t hi = row_word(send_words + k + 4u);           // still inside the row's pitch
    const uint32_t rw = row_word(row + k), sw = bytes_from(hi, lo, cut);
    lo = hi;
    spread |= (rw ^ (rw << 1)) | (sw ^ (sw << 1));
    in_have &= (uint32_t)(have >> (sw & 63u));
    have |= 1ull << (rw & 63u);
    in_have &= (uint32_t)(have >> ((sw >> 8) & 63u));
    have |= 1ull << ((rw >> 8) & 63u);
    in_have &= (uint32_t)(have >> ((sw >> 16) & 63u));
    have |= 1ull << ((rw >> 16) & 63u);
    in_have &= (uint32_t)(have >> ((sw >> 24) & 63u));
    have |= 1ull << ((rw >> 24) & 63u);
  }
  for (; k < q; ++k) {
    const uint32_t rb = (uint32_t)(uint8_t)row[k], sb = (uint32_t)(uint8_t)send[k];
    spread |= (rb ^ (rb << 1)) | (sb ^ (sb << 1));
    in_have &= (uint32_t)(have >> (sb & 63u));
    have |= 1ull << (rb & 63u);
  }
  const uint64_t negatives = ~0ull << (64u - q);     // the bits of -q..-1 (q >= 1)
  return (spread & 0xC0C0C0C0u) == 0u && (in_have & 1u) != 0u && have == (negatives | (1ull << b)) &&
         (int)send[0] == b - (int)q;
}

// 24 bits: the low six bits of the four bytes of w, bit 5 flipped ((x + 32) mod 64 for a byte x),
// the first byte lowest.
__device__ __forceinline__ uint32_t four_fields(uint32_t w) {
  const uint32_t x = (w & 0x3F3F3F3Fu) ^ 0x20202020u;
  const uint32_t y = (x & 0x003F003Fu) | ((x >> 2) & 0x0FC00FC0u);
  return (y & 0xFFFu) | ((y >> 4) & 0xFFF000u);
}

// Bytes from one row to the next where digest_rank reads them: a multiple of four that holds the
// 2q bytes of a row and the one aligned word that row_flags_clear reads past them when q is a
// multiple of four, and an odd number of words, so that the 64 lanes of a wavefront reading the
// same word of their rows hit different LDS banks.
__host__ __device__ inline uint32_t digest_row_pitch(uint32_t q) { return 4u * (((2u * q + 3u) / 4u) | 1u); }

// Invariant flags and row hash of one rank from its 2q bytes at a 4-byte aligned address, with
// the bytes up to digest_row_pitch(q) readable.  The hash takes the entries as
// six-bit fields (value + 32), ten to a 64-bit word in the order of the row, the last word
// filled up with zero bits; here 20 fields, two words, come from five 4-byte reads.
__device__ __forceinline__ void digest_rank(const Instance &in, uint32_t r, uint32_t v, int b,
                                            const int8_t *row, uint64_t &hash, uint32_t &flags) {
  const uint32_t q = in.q;
  const uint32_t two_q = 2u * q;
  const bool clear = q > 0 && v != 0 && row_flags_clear(q, b, row);
  flags = 0;
  if (__any(!clear)) {                               // the root's wavefront, and q = 0
    if (!clear) flags = row_flags_entrywise(in, v, b, row);
  }

  uint64_t h = sm64(((uint64_t)in.p << 32) ^ (uint64_t)r);
  uint32_t f0 = 0;
  for (; f0 + 20u <= two_q; f0 += 20u) {
    const uint64_t c0 = four_fields(row_word(row + f0)), c1 = four_fields(row_word(row + f0 + 4u));
    const uint64_t c2 = four_fields(row_word(row + f0 + 8u)), c3 = four_fields(row_word(row + f0 + 12u));
    const uint64_t c4 = four_fields(row_word(row + f0 + 16u));
    h = sm64(h ^ (c0 | (c1 << 24) | ((c2 & 0xFFFull) << 48)));
    h = sm64(h ^ ((c2 >> 12) | (c3 << 12) | (c4 << 36)));
  }
  if (f0 < two_q) {                                  // an even number of fields, 2 to 18, is left
    const uint32_t rem = two_q - f0;
    uint64_t c[5];
#pragma unroll
    for (uint32_t j = 0; j < 5; ++j) {
      uint32_t w = 0;
      if (4u * j + 4u <= rem) w = row_word(row + f0 + 4u * j);
      else if (4u * j + 2u <= rem) w = row_half(row + f0 + 4u * j);
      c[j] = four_fields(w);
    }
    // fields past the end of the row are zero bits in the word
    const uint64_t m0 = rem >= 10u ? ~0ull >> 4 : (1ull << (6u * rem)) - 1ull;
    h = sm64(h ^ ((c[0] | (c[1] << 24) | ((c[2] & 0xFFFull) << 48)) & m0));
    if (rem > 10u) {
      const uint64_t m1 = (1ull << (6u * (rem - 10u))) - 1ull;
      h = sm64(h ^ (((c[2] >> 12) | (c[3] << 12) | (c[4] << 36)) & m1));
    }
  }
  hash = h;
}

// Edge check of one rank (Conditions 1 and 2 as two XOR sums): what physical
// rank r expects to receive in round k, and what it sends to (r + skip[k]) mod p.
// g(rank, k, val) = sm64(rank << 11 | k << 6 | (val + 32)); row as in digest_rank.
__device__ __forceinline__ void edge_rank(const Instance &in, uint32_t r, const int8_t *row,
                                          uint64_t &xor_recv, uint64_t &xor_send) {
  const uint32_t q = in.q;
  for (uint32_t k = 0; k < q; ++k) {
    const uint32_t sk = skip_at_level(in.pm1, q - k);
    uint32_t t = r + sk;                               // < 2^32
    t = t >= in.p ? t - in.p : t;
    const uint64_t fr = (uint64_t)(((uint32_t)(int)row[k] + 32u) & 63u);
    const uint64_t fs = (uint64_t)(((uint32_t)(int)row[q + k] + 32u) & 63u);
    xor_recv ^= sm64(((uint64_t)r << 11) | ((uint64_t)k << 6) | fr);
    xor_send ^= sm64(((uint64_t)t << 11) | ((uint64_t)k << 6) | fs);
  }
}

__device__ __forceinline__ uint64_t wave_xor64(uint64_t x) {
  uint32_t lo = (uint32_t)x, hi = (uint32_t)(x >> 32);
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) {
    lo ^= (uint32_t)__shfl_xor((int)lo, m, 64);
    hi ^= (uint32_t)__shfl_xor((int)hi, m, 64);
  }
  return ((uint64_t)hi << 32) | lo;
}

__device__ __forceinline__ uint32_t wave_or32(uint32_t x) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) x |= (uint32_t)__shfl_xor((int)x, m, 64);
  return x;
}

__device__ __forceinline__ uint64_t wave_add64(uint64_t x) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) {
    uint32_t lo = (uint32_t)__shfl_xor((int)(uint32_t)x, m, 64);
    uint32_t hi = (uint32_t)__shfl_xor((int)(uint32_t)(x >> 32), m, 64);
    x += ((uint64_t)hi << 32) | lo;
  }
  return x;
}

__device__ __forceinline__ uint64_t wave_min64(uint64_t x) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) {
    uint32_t lo = (uint32_t)__shfl_xor((int)(uint32_t)x, m, 64);
    uint32_t hi = (uint32_t)__shfl_xor((int)(uint32_t)(x >> 32), m, 64);
    const uint64_t y = ((uint64_t)hi << 32) | lo;
    x = y < x ? y : x;
  }
  return x;
}

}  // namespace bcast
