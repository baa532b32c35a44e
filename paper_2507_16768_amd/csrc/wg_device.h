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
    uint32_t n_classes;
};

// A token that leaves a checkpoint state before its last byte: the part of a mask that
// depends on what follows the state.  `off` bytes are consumed up to and including the
// exit byte, `rem` bytes remain, the first of which is `first`.
struct ExitEntry {
    uint32_t tok;
    uint8_t off, cls, first, rem;
};
static_assert(sizeof(ExitEntry) == 8, "entry layout");

struct DeviceVocab {
    const uint8_t *bytes;        // CSR token bytes (padded by 8)
    const uint32_t *offsets;     // V + 1
    const uint8_t *len8;         // token length in bytes (0 for EOS and byte-less tokens)
    const uint64_t *chunks;      // chunks[k * V + t] = bytes 8k .. 8k+7 of token t, zero padded
    const ExitEntry *lit_entries;   // tokens grouped by first byte (a literal state's candidates)
    const uint32_t *lit_start;   // 257 bucket boundaries into lit_entries
    const uint32_t *len_rows;    // row r (0 .. lmax+1): tokens with 1 <= length <= r
    uint32_t V, W;
    int32_t eos_id;
    uint32_t lmax;
    uint32_t n_chunks;           // ceil(lmax / 8)
    uint32_t row_stride;         // words per mask row in device arenas (multiple of 4)
};

// A successor state as key_build needs it for the first hop of a walk.
struct HopState {
    uint32_t kind, lit, next_a, next_b, max, cls;
};

// One state key to build, resolved by the lookup so that key_build starts from a single load.
struct MissEntry {
    uint32_t key, sid, aux, kind;
    uint32_t r;                  // allow-bytes that may still be consumed, capped at lmax
    uint32_t cls;                // WAIT / COND: class table id
    uint32_t ent_lo, ent_cnt;    // LIT: its first-byte bucket in the vocabulary's entry list
    uint32_t eos_next, next_a, next_b, pad;
    HopState hop[2];             // successors reached through exit A / exit B
};
static_assert(sizeof(MissEntry) == 96, "miss entry layout");

struct Counters {
    uint32_t n_miss;             // state keys to build in the call in flight
    uint32_t n_class_miss;       // class tables to scan in the call in flight
    unsigned long long lookups, hits, builds, class_scans, entries_walked, errors;
};

struct DeviceCache {
    Counters *ctr;
    // per state key
    uint32_t *built;             // epoch in which the key's row was built
    uint32_t *arena;             // n_keys rows of row_stride words
    // per class table (the context-free part of every mask of a state using that table)
    uint32_t *class_built;       // epoch in which the class index was built
    uint32_t *class_rows;        // 2 rows per class: [stay] all bytes stay, [end] exits on its last byte
    ExitEntry *class_entries;    // V entries reserved per class
    uint32_t *class_count;       // entries in use per class
    // per call
    uint32_t *key_of;            // [B]
    MissEntry *miss;             // [B]
    uint32_t *class_miss;        // [B]
    uint32_t row_stride;         // words, multiple of 4
    uint32_t n_keys;
    uint32_t epoch;              // cache generation of this call; tag == epoch <=> entry valid
};

// ev, when not null, holds eight events: a begin / end pair for each of the four kernels of a fill.
hipError_t launch_fill(const DeviceTable &T, const DeviceVocab &Vc, const DeviceCache &Cc,
                       const wg_state_t *states, uint32_t B, uint32_t *bitmask, uint32_t n_cu,
                       hipStream_t s, hipEvent_t *ev);
hipError_t launch_apply(void *logits, int dtype, uint32_t B, uint32_t V, int64_t row_stride,
                        const uint32_t *bitmask, hipStream_t s);
hipError_t launch_masked_argmax(const void *logits, int dtype, uint32_t B, uint32_t V, int64_t row_stride,
                                const uint32_t *bitmask, int32_t *tokens, hipStream_t s);
hipError_t launch_advance(const DeviceTable &T, const DeviceVocab &Vc, const DeviceCache &Cc,
                          wg_state_t *states, const int32_t *tokens, uint32_t B, hipStream_t s,
                          hipEvent_t *ev);
hipError_t launch_select(const uint32_t *bitmask, uint32_t B, uint32_t V, const uint64_t *draws,
                         int32_t *tokens, hipStream_t s);
hipError_t configure_kernels(uint32_t row_bytes);

}  // namespace wg
