// Device-side views passed to the kernels by value, and the launcher prototypes.
#pragma once
#include <hip/hip_runtime.h>

#include "wg_internal.h"

namespace wg {

constexpr uint32_t kNoKey = 0xFFFFFFFFu;

struct DeviceTable {
    const StateDesc *states;
    const uint8_t *classes;      // 256-byte class tables
    const ClassInfo *class_info; // one per class table
    const uint8_t *lit;          // literal byte per state
    uint32_t n_states;
    uint32_t lmax;
    uint32_t n_classes;
};

struct DeviceVocab {
    const uint8_t *bytes;        // CSR token bytes (padded by 8)
    const uint32_t *offsets;     // V + 1
    const uint8_t *len8;         // token length in bytes (0 for EOS and byte-less tokens)
    const uint64_t *chunks;      // chunks[k * V + t] = bytes 8k .. 8k+7 of token t, zero padded
    const uint64_t *sig;         // bit (x & 63) for every byte x of the token; all ones for a byte-less token
    const uint8_t *first8;       // the token's first byte (0 for a byte-less token)
    const ExitEntry *lit_entries;   // tokens grouped by (first byte, range): a literal state's candidates
    const uint32_t *lit_start;   // 256 * kParts + 1 bucket boundaries into lit_entries
    const uint32_t *len_rows;    // row r (0 .. lmax+1): tokens with 1 <= length <= r
    // The vocabulary in byte order (tokens that have bytes, compared as byte strings), as
    // entries {tok, off = 0, first = second byte, rem = length}, with the ranges of its one- and
    // two-byte prefixes: range y0 * 257 of dir0 holds the token that is the single byte y0,
    // range y0 * 257 + 1 + y1 the tokens of two or more bytes that start with y0 y1.
    const ExitEntry *sorted;
    const uint32_t *dir0;        // 256 * 257 + 1 boundaries into sorted
    // Every place inside a token where one byte follows another: entries {tok, off = index of the
    // second byte, first = that byte, rem = bytes from it to the end}, grouped by the byte pair;
    // range e * 256 + y of dirN holds the places where y follows e.
    const ExitEntry *bigram;
    const uint32_t *dirN;        // 65536 + 1 boundaries into bigram
    // The vocabulary by byte value, as token rows: row x (0 .. 255) holds the tokens that contain
    // the byte x, row 256 + x the tokens whose first byte is x.
    const uint32_t *byte_rows;   // 512 rows of row_stride words
    uint32_t V, W;
    int32_t eos_id;
    uint32_t lmax;
    uint32_t n_chunks;           // ceil(lmax / 8)
    uint32_t row_stride;         // words per mask row in device arenas (multiple of 4)
    uint32_t part_tok[kParts + 1];  // first token of each range; part_tok[kParts] == V
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
    uint32_t lit;                // LIT: the byte (its first-byte buckets hold the candidates)
    uint8_t mode;                // KB_*: where the candidate tokens of the key come from
    uint8_t n_a, n_b, pad0;      // KB_BIGRAM: how many exit bytes of each side are listed
    uint32_t eos_next, next_a, next_b;
    uint32_t slot;               // arena row of the result, or kNoSlot: only into the bitmask row of `req`
    uint32_t req;                // the request that claimed the key
    uint32_t exits[3];           // KB_BIGRAM: byte k of these 12 is exit byte k of side A (k < 6) or k - 6 of side B
    HopState hop[2];             // successors reached through exit A / exit B
};
// Where key_build finds the tokens that can leave the key's state before their last byte:
//   KB_LIST   the exit list of the state's class table, or the first-byte buckets of a literal
//             state: every entry is looked at (and, for a key whose successor is a checkpoint,
//             walked; such a key is cut into one work item per token range);
//   KB_SORTED a literal state followed by another literal byte, or by nothing that takes a byte:
//             the tokens that start with those two bytes, and the one-byte token, from the
//             vocabulary in byte order;
//   KB_BIGRAM a checkpoint whose exits lead to literal bytes (or to the end): the places in the
//             vocabulary where an exit byte is followed by the literal byte.
enum : uint8_t { KB_LIST = 0, KB_SORTED = 1, KB_BIGRAM = 2 };
static_assert(sizeof(MissEntry) == 112, "miss entry layout");

struct Counters {
    uint32_t n_deep;             // keys of the call in flight whose candidates all need a deep walk
    uint32_t n_plain;            // ... and the other keys (the two share the miss list, from its two ends)
    uint32_t n_claims;           // state keys claimed in the call in flight
    uint32_t n_class_miss;       // class tables to scan in the call in flight
    unsigned long long slot_ctr; // generation << 32 | arena rows in use in that generation (<= cap_rows)
    unsigned long long launch;   // number of the fill call in flight (its gather counts it up)
    unsigned long long lookups, hits, builds, uncached_builds, class_scans, entries_walked, errors;
};

// A key's 64-bit tag, by its top bit:
//   0: generation (30 bits) << 32 | arena row.  The row is valid if the generation is the
//      handle's current cache generation (1 .. 2^30-1); 0 means never built.
//   1: claimed - 1 << 63 | launch (46 bits) << 16 | request index (16 bits): request `index` of
//      the fill call `launch` builds the row.  key_build replaces the claim by the row's tag
//      once the row is in the arena; if the arena was full the claim stays: the row was built
//      straight into the bitmask row of the claiming request and is not kept, so the key is
//      missing again in the next call.
constexpr unsigned long long kTagClaim = 1ull << 63;
constexpr unsigned long long kTagLaunchMask = (1ull << 46) - 1ull;
constexpr uint32_t kNoSlot = 0xFFFFFFFFu;
// What lookup leaves per request for gather: the arena row of a mask cached before the call, or
// kRefByKey | key for a mask built in this call (its tag then says where it went), or kNoKey
// (no such state: a row of zeros).  Rows and keys stay below 2^30 and 2^31 - 1.
constexpr uint32_t kRefByKey = 0x80000000u;
constexpr uint32_t kRefSelf = 0xFFFFFFFEu;   // this request claimed the key: key_build writes its bitmask row itself
constexpr uint32_t kMaxRows = 1u << 30, kMaxKeys = 0x7FFFFFFEu;
constexpr uint32_t kMaxBatch = 65535u;     // request indexes fit the 16 bits of a tag (and grid.y)

struct DeviceCache {
    Counters *ctr;
    // per state key
    unsigned long long *tags;
    uint32_t *arena;             // cap_rows rows of row_stride words, handed out on demand
    uint32_t cap_rows;
    // per class table (the context-free part of every mask of a state using that table)
    uint32_t *class_built;       // generation in which the class index was built
    uint32_t *class_rows;        // 3 rows per class: [stay] all bytes stay, [end] exits on its last byte, [both]
    ExitEntry *const *class_entries;   // per class 2 V slots: [0, V) the list of the class table, range p of
                                 // the second V owns [V + part_tok[p], V + part_tok[p+1]); each filled
                                 // from both ends
    uint32_t *class_count;       // per class 2 + 2 * kParts counters (front, back of the class list, then of
                                 // each range), 128 bytes apart
    // per call
    uint32_t *row_ref;           // [B] arena row of the request's mask, kRefByKey | key, kRefSelf, or kNoKey
    MissEntry *miss;             // [miss_cap]: deep keys from the front, plain keys from the back
    uint32_t miss_cap;           // the largest batch so far
    uint32_t *class_miss;        // [B]
    uint32_t row_stride;         // words, multiple of 4
    uint32_t n_keys;
    uint32_t epoch;              // cache generation of this call
    uint32_t scan_batch;         // class tables a class_scan work item takes together; 0: chosen per call
};

// ev, when not null, holds eight events: a begin / end pair for each of the four kernels of a fill.
// With tokens != nullptr the states are first advanced by them (in place, in the lookup kernel);
// with logits != nullptr the mask is also applied to them (in the gather kernel when their
// layout allows 16-byte stores).
hipError_t launch_fill(const DeviceTable &T, const DeviceVocab &Vc, const DeviceCache &Cc,
                       wg_state_t *states, const int32_t *tokens, uint32_t B, uint32_t *bitmask,
                       void *logits, int dtype, int64_t logits_stride,
                       uint32_t n_cu, hipStream_t s, hipEvent_t *ev);
hipError_t launch_apply(void *logits, int dtype, uint32_t B, uint32_t V, int64_t row_stride,
                        const uint32_t *bitmask, hipStream_t s, hipEvent_t *ev);
hipError_t launch_masked_argmax(const void *logits, int dtype, uint32_t B, uint32_t V, int64_t row_stride,
                                const uint32_t *bitmask, int32_t *tokens, hipStream_t s);
// masked top-k: a workgroup ranks kTopkSlice tokens of a row; `lists` is the caller's workspace
// of B * ceil(V / kTopkSlice) * k 64-bit keys
constexpr uint32_t kTopkMax = 64;
constexpr uint32_t kTopkSlice = 8192;
constexpr uint32_t kTopkMergeKeys = 4096;    // most keys (slices * k) the merge of a row holds in LDS
hipError_t launch_masked_topk(const void *logits, int dtype, uint32_t B, uint32_t V, int64_t row_stride,
                              const uint32_t *bitmask, uint32_t k, int32_t *ids, void *values,
                              unsigned long long *lists, hipStream_t s);
// wg_masked_topk_static keeps its lists in a file-scope device array of this many 64-bit keys
// (4 MiB per GPU); static_topk_scratch gives the array's address on the current device.
constexpr uint64_t kTopkStaticKeys = 1ull << 19;
hipError_t static_topk_scratch(unsigned long long **out);
hipError_t launch_advance(const DeviceTable &T, const DeviceVocab &Vc, const DeviceCache &Cc,
                          wg_state_t *states, const int32_t *tokens, uint32_t B, hipStream_t s,
                          hipEvent_t *ev);
hipError_t launch_forced_bytes(const DeviceTable &T, const wg_state_t *states, uint32_t B, uint32_t cap,
                               uint8_t *bytes, uint32_t *lens, wg_state_t *end_states, hipStream_t s);
hipError_t launch_select(const uint32_t *bitmask, uint32_t B, uint32_t V, const uint64_t *draws,
                         int32_t *tokens, hipStream_t s);
hipError_t configure_kernels(uint32_t row_bytes);

}  // namespace wg
