// Internal layouts shared by the host lowering code and the HIP kernels.
#pragma once
#include <cstdint>
#include <string>
#include <vector>

#include "../../include/wg.h"

namespace wg {

constexpr uint32_t kSymEos = 256;

// Byte classes of a WAIT / COND state (one 256-entry table per distinct set triple).
enum : uint8_t { CLS_REJECT = 0, CLS_STAY = 1, CLS_EXIT_A = 2, CLS_EXIT_B = 3 };

// One leaf state as the kernels read it: 32 bytes, so a wave fetches a descriptor
// with one scalar 8-dword load.
struct StateDesc {
    uint32_t kind_byte;   // bits 0..7 WG_KIND_*, bits 8..15 the literal byte of a LIT state
    uint32_t next_a;      // LIT / WAIT successor, COND true target
    uint32_t next_b;      // COND false target
    uint32_t eos_next;    // state after EOS, WG_SID_ERROR if rejected
    uint32_t cls;         // WAIT / COND: index of the 256-byte class table; LIT: state after its Write
    uint32_t max;         // WAIT bound, WG_UNBOUNDED if none
    uint32_t key_base;    // first mask-cache key of this state
    uint32_t run;         // LIT: literal bytes from this state to the end of its Write
};
static_assert(sizeof(StateDesc) == 32, "descriptor layout");

// Result of lowering a set of template instances (host memory).
struct Table {
    std::vector<StateDesc> states;        // index = sid; [0] is FINAL
    std::vector<uint8_t> classes;         // n_class_tables * 256
    std::vector<uint8_t> lit;             // lit[sid] = byte of a LIT state (else 0)
    std::vector<uint32_t> tmpl;           // template instance of each state
    std::vector<uint32_t> start;          // start state of each instance
    std::vector<uint32_t> key_count;      // masks per state (1, or lmax+1 for a bounded Wait)
    uint32_t n_keys = 0;
    uint32_t lmax = 0;
    uint32_t flags = 0;
};

// The token ids are cut into kParts contiguous ranges (on 2048-token boundaries, so on 256-byte
// boundaries of a mask row; a class_scan workgroup takes kPartGroup tokens, all in one range).  Every list of candidate tokens is kept per range, so that the
// row of a state key whose candidates all need a deep walk can be built by several workgroups,
// each owning the words of its ranges, without any merging.
constexpr uint32_t kParts = 8;
constexpr uint32_t kPartGroup = 2048;

// What the kernels want to know about a class table without reading its 256 bytes: the bytes
// that leave through exit A / exit B (as long as there are at most kMaxExitBytes of them on a
// side), which first look the class scan takes, and the folded set of byte values that do not stay.
constexpr uint32_t kMaxExitBytes = 6;
struct ClassInfo {
    uint8_t n_a, n_b;            // bytes of class EXIT_A / EXIT_B, or 0xFF: more than kMaxExitBytes
    uint8_t scan, pad;           // SCAN_*: how class_scan takes its first look at a token
    uint8_t a[kMaxExitBytes], b[kMaxExitBytes];
    unsigned long long nonstay;  // SCAN_SIG: bit (x & 63) for every byte value x that does not stay (never 0)
    unsigned long long pad2;
};
static_assert(sizeof(ClassInfo) == 32, "class info layout");
// The first look class_scan takes at a token, chosen by what the table does with most bytes:
//   SCAN_SIG   nearly every byte value stays (a free-text Wait): a token none of whose bytes folds
//              onto a byte value that does not stay is all-stay, by one AND with its signature;
//   SCAN_HEAD  most byte values are rejected (an allow list): the first byte decides most tokens;
//   SCAN_CHUNK anything between: the first 8 bytes through the table.
enum : uint8_t { SCAN_CHUNK = 0, SCAN_SIG = 1, SCAN_HEAD = 2 };
constexpr uint8_t kManyExits = 0xFF;

// A token that leaves a checkpoint state before its last byte: the part of a mask that
// depends on what follows the state.  `off` bytes are consumed up to and including the
// exit byte, `rem` bytes remain, the first of which is `first`.
struct ExitEntry {
    uint32_t tok;
    uint8_t off, cls, first, rem;
};
static_assert(sizeof(ExitEntry) == 8, "entry layout");

// The static indexes of a vocabulary (they depend on the token bytes only), as host arrays in
// the layouts the kernels read.  Built once per vocabulary; wg_vocab_create copies them to the
// device as they are.
struct VocabIndex {
    uint32_t V = 0, W = 0, row_stride = 0, lmax = 0, n_chunks = 0;
    uint32_t part_tok[kParts + 1] = {};    // first token of each range; part_tok[kParts] == V
    std::vector<uint8_t> bytes;            // the token bytes, 8 zero bytes behind them
    std::vector<uint32_t> offsets;         // V + 1
    std::vector<uint8_t> len8, first8;     // per token
    std::vector<uint64_t> chunks;          // max(n_chunks, 1) * V
    std::vector<uint64_t> sig;             // per token
    std::vector<ExitEntry> lit_entries;    // never empty (one unused entry when no token has bytes)
    std::vector<uint32_t> lit_start;       // 256 * kParts + 1
    std::vector<uint32_t> len_rows;        // (lmax + 2) * row_stride
    std::vector<ExitEntry> sorted;         // never empty
    std::vector<uint32_t> dir0;            // 256 * 257 + 1
    std::vector<ExitEntry> bigram;         // never empty
    std::vector<uint32_t> dirN;            // 65536 + 1
    std::vector<uint32_t> byte_rows;       // 512 rows of row_stride words: 256 by any byte, 256 by the first byte
};

// Checks the vocabulary arguments of wg_vocab_create and builds the indexes.  Returns WG_OK, or
// an error code with the message in *err; `out` is then unspecified.
int build_vocab_index(const uint8_t *host_bytes, const uint64_t *host_offsets, uint32_t V, int32_t eos_id,
                      VocabIndex *out, std::string *err);

// The summary of one 256-byte class table that the kernels read in its place.
ClassInfo class_info_of(const uint8_t *table);

// The host operator compiler with its memory: parsed template texts (the static structures)
// and the class tables seen so far, so that instances can be added to a live table.
struct LoweringState;
class Lowering {
  public:
    Lowering(uint32_t flags, uint32_t lmax);
    ~Lowering();
    Lowering(const Lowering &) = delete;
    Lowering &operator=(const Lowering &) = delete;
    // Appends n template instances.  Throws std::runtime_error with a message naming the
    // template and the offset; the table is then as it was before the call.
    void add(const char *const *templates, const wg_args_t *args, uint32_t n);
    Table table;

  private:
    LoweringState *st_;
};

// Translates a regular expression into template text in the operator syntax; throws
// std::runtime_error when the expression has no translation.
std::string regex_to_template(const char *regex);

void set_last_error(const std::string &msg);

}  // namespace wg
