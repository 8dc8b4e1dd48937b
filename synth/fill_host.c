/* Host fill of the seeded synthetic tensors (gcc; no method arithmetic here).
 * dst[i] = table[ synth_u16(key, first_elem + i) ], i in [0, n).
 */
#include "counter_rng.h"
#include <stddef.h>

int synth_fill_host(void* dst, int elem_bytes, const void* table, uint64_t key,
                    uint64_t first_elem, uint64_t n) {
  if (!dst || !table) return 1;
  if (elem_bytes == 2) {
    uint16_t* d = (uint16_t*)dst;
    const uint16_t* t = (const uint16_t*)table;
    for (uint64_t i = 0; i < n; ++i) d[i] = t[synth_u16(key, first_elem + i)];
  } else if (elem_bytes == 4) {
    uint32_t* d = (uint32_t*)dst;
    const uint32_t* t = (const uint32_t*)table;
    for (uint64_t i = 0; i < n; ++i) d[i] = t[synth_u16(key, first_elem + i)];
  } else {
    return 2;
  }
  return 0;
}

uint64_t synth_stream_key_c(uint64_t seed, uint64_t tensor_id) {
  return synth_stream_key(seed, tensor_id);
}

uint64_t synth_bits64_c(uint64_t key, uint64_t ctr) { return synth_bits64(key, ctr); }
