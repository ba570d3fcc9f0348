// The HIP library's per-rank code (bcast_device.hpp) compiled for the CPU, so
// that its logic and its index arithmetic can be checked against the oracle
// without a GPU, under gdb or a sanitizer if need be.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include "../../paper_2407_18004_amd/csrc/bcast_device.hpp"

using namespace bcast;

static uint32_t q_of(uint32_t p) {
  uint32_t q = 0;
  while ((1ull << q) < (uint64_t)p) ++q;
  return q;
}

extern "C" {

// rows: m rows of 2q int32 (recv then send) for the physical ranks given.
// flags_out/hash_out (may be NULL): per-rank flags and row hash.
int shim_schedules_ranks(uint32_t p, uint32_t root, const uint32_t *ranks, uint64_t m,
                         int32_t *rows, uint32_t *flags_out, uint64_t *hash_out) {
  const uint32_t q = q_of(p);
  const Instance in = make_instance(p, q, root);
  for (uint64_t i = 0; i < m; ++i) {
    int8_t buf[64];
    memset(buf, 0x55, sizeof buf);
    int b = 0;
    const uint32_t v = virtual_rank(in, ranks[i]);
    uint32_t fl = compute_rank(in, v, buf, buf + q, b);
    for (uint32_t k = 0; k < 2 * q; ++k) rows[i * 2 * q + k] = buf[k];
    uint64_t h = 0;
    uint32_t fl2 = 0;
    digest_rank(in, ranks[i], v, b, buf, buf + q, h, fl2);
    if (flags_out) flags_out[i] = fl | fl2;
    if (hash_out) hash_out[i] = h;
  }
  return (int)q;
}

// flags and hash of a row given by the caller (for planted mistakes)
void shim_digest_row(uint32_t p, uint32_t root, uint32_t r, const int32_t *row,
                     uint64_t *hash, uint32_t *flags) {
  const uint32_t q = q_of(p);
  const Instance in = make_instance(p, q, root);
  int8_t buf[64];
  for (uint32_t k = 0; k < 2 * q; ++k) buf[k] = (int8_t)row[k];
  const uint32_t v = virtual_rank(in, r);
  const int b = (int)q - (int)baseblock_level(in.pm1, q, v);
  digest_rank(in, r, v, b, buf, buf + q, *hash, *flags);
}

}  // extern "C"
