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
// sequence.  v = 0 takes nothing and yields level 0 (b = q).
__device__ __forceinline__ uint32_t baseblock_level(uint32_t pm1, uint32_t q, uint32_t v) {
  uint32_t rem = v, jb = 0;
  for (uint32_t j = 1; j <= q; ++j) {
    const uint32_t sk = skip_at_level(pm1, j);
    const bool take = sk <= rem;
    rem = take ? rem - sk : rem;
    jb = take ? j : jb;
  }
  return jb;
}

// Algorithms 4 and 5: the receive search for virtual rank v, as an explicit
// state machine instead of recursion.
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

// Algorithm 6 without its violations: writes sendblock[k] through emit for
// k = q-1 .. 0 and returns the mask of rounds k whose entry must instead be
// taken from the receive schedule of the to-processor.
template <typename Emit>
__device__ __forceinline__ uint32_t send_walk(uint32_t p, uint32_t pm1, uint32_t q,
                                              uint32_t v, int b, Emit emit) {
  if (q == 0) return 0;
  uint32_t viol = 0;
  uint32_t rp = v, e = p;
  int c = b;
  const bool is_root = v == 0;
  for (uint32_t k = q - 1; k >= 1; --k) {
    const uint32_t skk = skip_at_level(pm1, q - k);
    const uint32_t skm = skip_at_level(pm1, q - k + 1);
    const bool lower = rp < skk;
    const bool ok_lower = (rp + skk < e) || (e < skm) || (k == 1 && b > 0);
    const bool ok_upper = (k == 1) || (rp > skk) || (e - skk < skm) || (rp + skk <= e);
    c = lower ? c : (int)k - (int)q;
    const bool ok = lower ? ok_lower : ok_upper;
    viol |= (ok || is_root) ? 0u : (1u << k);
    const uint32_t e_lo = e > skk ? skk : e;
    e = lower ? e_lo : e - skk;
    rp = lower ? rp : rp - skk;
    emit(k, is_root ? (int)k : c);
  }
  emit(0u, is_root ? 0 : b - (int)q);
  return viol;
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

// Computes the 2q entries of virtual rank v into LDS: recvblock[k] at
// recv_row[k], sendblock[k] at send_row[k] (bytes).  Returns the search flags
// (BCAST_F_SEARCH, BCAST_F_VIOLATIONS) and the baseblock through b_out.
__device__ __forceinline__ uint32_t compute_rank(const Instance &in, uint32_t v,
                                                 int8_t *recv_row, int8_t *send_row,
                                                 int &b_out) {
  const uint32_t q = in.q;
  uint32_t flags = 0;
  const uint32_t jb = baseblock_level(in.pm1, q, v);
  const int b = (int)q - (int)jb;
  b_out = b;
  if (q == 0) return 0;
  bool anomaly = false;
  const uint32_t produced =
      recv_search(in.p, in.pm1, q, v, jb, q - 1u, anomaly,
                  [&](uint32_t k, int val) { recv_row[k] = (int8_t)val; });
  if (produced != q || anomaly) flags |= BCAST_F_SEARCH;

  uint32_t viol = send_walk(in.p, in.pm1, q, v, b,
                            [&](uint32_t k, int val) { send_row[k] = (int8_t)val; });
  if (__popc(viol) > 4) flags |= BCAST_F_VIOLATIONS;
  // Violations of Algorithm 6: entry k is recvblock[k] of the to-processor.
  while (viol != 0) {
    const uint32_t k = (uint32_t)(__ffs((int)viol) - 1);
    viol &= viol - 1u;
    uint32_t t = v + skip_at_level(in.pm1, q - k);
    t = t >= in.p ? t - in.p : t;
    const uint32_t jbt = baseblock_level(in.pm1, q, t);
    int val = 0;
    bool anomaly_t = false;
    const uint32_t got = recv_search(in.p, in.pm1, q, t, jbt, k, anomaly_t,
                                     [&](uint32_t kk, int x) { if (kk == k) val = x; });
    if (got <= k || anomaly_t) flags |= BCAST_F_SEARCH;
    send_row[k] = (int8_t)val;
  }
  return flags;
}

// Invariant flags (Conditions 3 and 4, first send, range) and the row hash of
// one rank from its 2q bytes in LDS.
__device__ __forceinline__ void digest_rank(const Instance &in, uint32_t r, uint32_t v, int b,
                                            const int8_t *recv_row, const int8_t *send_row,
                                            uint64_t &hash, uint32_t &flags) {
  const int q = (int)in.q;
  const uint32_t two_q = 2u * in.q;
  const bool is_root = v == 0;
  uint32_t seen = 0, dup = 0, npos = 0, have_neg = 0, have_pos = 0;
  bool range_bad = false, pos_ok = true, send0_ok = true, cond4_ok = true;
  if (!is_root) have_neg = 1u << b;                 // b - q may always be sent
  uint64_t h = sm64(((uint64_t)in.p << 32) ^ (uint64_t)r);
  uint64_t w = 0;
  uint32_t sh = 0;
  for (int k = 0; k < q; ++k) {
    const int rv = recv_row[k];
    w |= (uint64_t)((uint32_t)(rv + 32) & 63u) << sh;
    sh += 6;
    if (sh == 60) { h = sm64(h ^ w); w = 0; sh = 0; }
    const bool in_range = (uint32_t)(rv + q) < two_q;
    range_bad |= !in_range;
    if (in_range) {
      const uint32_t bit = 1u << (rv < 0 ? rv + q : rv);
      dup |= seen & bit;
      seen |= bit;
      npos += rv >= 0 ? 1u : 0u;
      pos_ok = pos_ok && (rv < 0 || rv == b);
    }
  }
  for (int k = 0; k < q; ++k) {
    const int sv = send_row[k];
    const int rv = recv_row[k];
    w |= (uint64_t)((uint32_t)(sv + 32) & 63u) << sh;
    sh += 6;
    if (sh == 60) { h = sm64(h ^ w); w = 0; sh = 0; }
    const bool s_in = (uint32_t)(sv + q) < two_q;
    range_bad |= !s_in;
    if (is_root) {
      send0_ok = send0_ok && sv == k;
    } else {
      if (k == 0) {
        send0_ok = sv == b - q;
      } else {
        bool ok = false;
        if (s_in) ok = sv < 0 ? ((have_neg >> (sv + q)) & 1u) != 0 : ((have_pos >> sv) & 1u) != 0;
        cond4_ok = cond4_ok && ok;
      }
      if ((uint32_t)(rv + q) < two_q) {
        if (rv < 0) have_neg |= 1u << (rv + q); else have_pos |= 1u << rv;
      }
    }
  }
  if (sh != 0) h = sm64(h ^ w);
  const uint32_t full = q >= 32 ? 0xFFFFFFFFu : ((1u << q) - 1u);
  // q in-range entries that set q different bits, one of them (none for the
  // root) non-negative and equal to b: the multiset of Condition 3.
  const bool cond3_ok = dup == 0 && seen == full && npos == (is_root ? 0u : 1u) && pos_ok;
  hash = h;
  flags = (cond3_ok ? 0u : BCAST_F_COND3) | (send0_ok ? 0u : BCAST_F_SEND0) |
          (cond4_ok ? 0u : BCAST_F_COND4) | (range_bad ? BCAST_F_RANGE : 0u);
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
