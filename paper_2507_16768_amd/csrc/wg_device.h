// Device-side views passed to the kernels by value, and the launcher prototypes.
#pragma once
#include <hip/hip_runtime.h>

#include "wg_internal.h"

namespace wg {

constexpr uint32_t kNoKey = 0xFFFFFFFFu;

struct DeviceTable {
    const StateDesc *states;
    const uint8_t *classes;      // 256-byte class tables
    const uint8_t *lit;          // literal byte per state
    uint32_t n_states;
    uint32_t lmax;
};

struct DeviceVocab {
    const uint8_t *bytes;        // CSR token bytes
    const uint32_t *offsets;     // V + 1
    uint32_t V, W;
    int32_t eos_id;
    uint32_t lmax;
};

struct MissEntry { uint32_t key, sid, aux, pad; };

struct Counters {
    uint32_t epoch;              // cache generation; built[key] == epoch <=> row valid
    uint32_t n_miss;             // entries in the miss list of the call in flight
    unsigned long long lookups, hits, builds, errors;
};

struct DeviceCache {
    Counters *ctr;
    uint32_t *built;             // per key: epoch in which its row was built
    uint32_t *arena;             // n_keys rows of row_stride words
    uint32_t *key_of;            // per request of the call in flight
    MissEntry *miss;             // per call, at most B entries
    uint32_t row_stride;         // words, multiple of 4
    uint32_t n_keys;
};

hipError_t launch_fill(const DeviceTable &T, const DeviceVocab &Vc, const DeviceCache &Cc,
                       const wg_state_t *states, uint32_t B, uint32_t *bitmask, uint32_t n_cu,
                       hipStream_t s);
hipError_t launch_clear(const DeviceCache &Cc, hipStream_t s);
hipError_t launch_apply(void *logits, int dtype, uint32_t B, uint32_t V, int64_t row_stride,
                        const uint32_t *bitmask, hipStream_t s);
hipError_t launch_advance(const DeviceTable &T, const DeviceVocab &Vc, const DeviceCache &Cc,
                          wg_state_t *states, const int32_t *tokens, uint32_t B, hipStream_t s);
hipError_t launch_select(const uint32_t *bitmask, uint32_t B, uint32_t V, const uint64_t *draws,
                         int32_t *tokens, hipStream_t s);

}  // namespace wg
