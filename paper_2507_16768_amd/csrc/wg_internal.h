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
