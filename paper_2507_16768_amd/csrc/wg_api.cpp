// C ABI: handles, device uploads, argument checks, kernel launches.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <memory>
#include <new>
#include <stdexcept>
#include <string>
#include <vector>

#include "wg_device.h"

namespace wg {
static thread_local std::string g_last_error;
void set_last_error(const std::string &msg) { g_last_error = msg; }
}  // namespace wg

using namespace wg;

struct wg_table_s {
    Lowering low;
    wg_table_s(uint32_t flags, uint32_t lmax) : low(flags, lmax) {}
};

struct wg_vocab_s {
    DeviceVocab dv{};
    uint8_t *d_bytes = nullptr, *d_len8 = nullptr;
    uint32_t *d_offsets = nullptr, *d_lit_start = nullptr, *d_len_rows = nullptr;
    uint64_t *d_chunks = nullptr, *d_sig = nullptr;
    uint8_t *d_first8 = nullptr;
    ExitEntry *d_lit_entries = nullptr, *d_sorted = nullptr, *d_bigram = nullptr;
    uint32_t *d_dir0 = nullptr, *d_dirN = nullptr, *d_byte_rows = nullptr;
    int device = 0;
    void release() {
        (void)hipFree(d_bytes); (void)hipFree(d_len8); (void)hipFree(d_offsets);
        (void)hipFree(d_lit_start); (void)hipFree(d_len_rows); (void)hipFree(d_chunks);
        (void)hipFree(d_lit_entries); (void)hipFree(d_sorted); (void)hipFree(d_bigram);
        (void)hipFree(d_dir0); (void)hipFree(d_dirN); (void)hipFree(d_byte_rows); (void)hipFree(d_sig); (void)hipFree(d_first8);
    }
};

struct wg_handle_s {
    wg_vocab_s *vocab = nullptr;
    Lowering low;
    DeviceTable dt{};
    DeviceCache dc{};
    // device copies of the table, with room to append (capacities in elements)
    StateDesc *d_states = nullptr;
    uint8_t *d_classes = nullptr, *d_lit = nullptr;
    ClassInfo *d_class_info = nullptr;
    uint32_t cap_states = 0, cap_classes = 0, cap_keys = 0;
    uint32_t up_states = 0, up_classes = 0;           // how much of the host table is on the device
    // class index storage: one buffer of V exit entries per class table in use, and the
    // device table of their addresses
    std::vector<ClassInfo> class_info;                // host copy, kept for the asynchronous uploads
    std::vector<ExitEntry *> class_bufs;
    std::vector<ExitEntry *> class_slabs;             // what was allocated: class_bufs point into these
    uint32_t slab_left = 0;                           // class buffers not handed out yet in the last slab
    ExitEntry **d_class_entries = nullptr;
    uint32_t max_batch = 0;
    uint32_t n_cu = 256;
    // kernel timing: events recorded since the last wg_profile_read
    bool profiling = false;
    std::vector<hipEvent_t> fill_events;       // 8 per wg_fill_masks call: begin / end of each kernel
    std::vector<hipEvent_t> advance_events;    // 2 per wg_advance call
    std::vector<hipEvent_t> apply_events;      // 2 per wg_profile_apply_mask call
    std::vector<hipEvent_t> spare_events;
    wg_handle_s(uint32_t flags, uint32_t lmax) : low(flags, lmax) {}
};

namespace {

int fail(int code, const std::string &msg) { set_last_error(msg); return code; }

constexpr uint32_t kDefaultBatch = 1024;   // requests per call a handle has room for after wg_compile

#define WG_HIP(call)                                                                          \
    do {                                                                                      \
        hipError_t e_ = (call);                                                               \
        if (e_ != hipSuccess)                                                                 \
            return fail(e_ == hipErrorOutOfMemory ? WG_ERR_NOMEM : WG_ERR_HIP,                \
                        std::string(#call) + ": " + hipGetErrorString(e_));                   \
    } while (0)

template <class T> hipError_t upload(T **dst, const T *src, size_t n) {
    hipError_t e = hipMalloc(reinterpret_cast<void **>(dst), (n ? n : 1) * sizeof(T));
    if (e != hipSuccess) return e;
    return n ? hipMemcpy(*dst, src, n * sizeof(T), hipMemcpyHostToDevice) : hipSuccess;
}

hipEvent_t take_event(wg_handle_s *h) {
    if (!h->spare_events.empty()) {
        hipEvent_t e = h->spare_events.back();
        h->spare_events.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    (void)hipEventCreate(&e);
    return e;
}

// Room for the per-call lists of a batch of B requests.  Never called from the step path: the
// device is synchronised and the lists are allocated anew.
int reserve_batch(wg_handle_s *h, uint32_t B) {
    if (B <= h->max_batch) return WG_OK;
    WG_HIP(hipDeviceSynchronize());
    if (h->dc.row_ref) (void)hipFree(h->dc.row_ref);
    if (h->dc.miss) (void)hipFree(h->dc.miss);
    if (h->dc.class_miss) (void)hipFree(h->dc.class_miss);
    h->dc.row_ref = nullptr; h->dc.miss = nullptr; h->dc.class_miss = nullptr; h->max_batch = 0;
    h->dc.miss_cap = 0;
    WG_HIP(hipMalloc(reinterpret_cast<void **>(&h->dc.row_ref), B * sizeof(uint32_t)));
    WG_HIP(hipMalloc(reinterpret_cast<void **>(&h->dc.miss), B * sizeof(MissEntry)));
    WG_HIP(hipMalloc(reinterpret_cast<void **>(&h->dc.class_miss), B * sizeof(uint32_t)));
    h->dc.miss_cap = B;
    h->max_batch = B;
    return WG_OK;
}

// Gives *p room for new_n elements, keeping the first keep_n and zero-filling the rest.
template <class T> int regrow(T **p, size_t keep_n, size_t new_n, size_t pad_bytes = 0) {
    T *q = nullptr;
    WG_HIP(hipMalloc(reinterpret_cast<void **>(&q), new_n * sizeof(T) + pad_bytes));
    hipError_t e = hipMemset(q, 0, new_n * sizeof(T) + pad_bytes);
    if (e == hipSuccess && keep_n && *p) e = hipMemcpy(q, *p, keep_n * sizeof(T), hipMemcpyDeviceToDevice);
    if (e != hipSuccess) {
        (void)hipFree(q);
        return fail(WG_ERR_HIP, std::string("growing a device table: ") + hipGetErrorString(e));
    }
    (void)hipFree(*p);
    *p = q;
    return WG_OK;
}

uint32_t grown(uint32_t need, uint32_t floor_n) {
    uint64_t n = need < floor_n ? floor_n : need;
    n += n / 2;                                        // headroom for instances added later
    return n > 0xFFFFFFF0ull ? 0xFFFFFFF0u : (uint32_t)n;
}

// Brings the device copy of the table up to date with the host table after instances were
// appended.  Within the reserved capacities this only copies the new slices (ordered on `s`
// with the caller's other work); beyond them the device is synchronised once and the tables move.
int sync_table(wg_handle_s *h, hipStream_t s) {
    const Table &t = h->low.table;
    const uint32_t n_states = (uint32_t)t.states.size(), n_classes = (uint32_t)(t.classes.size() / 256);
    const uint32_t row_stride = h->dc.row_stride, V = h->vocab->dv.V;
    if (n_states > h->cap_states || n_classes > h->cap_classes || t.n_keys > h->cap_keys)
        WG_HIP(hipDeviceSynchronize());
    if (n_states > h->cap_states) {
        const uint32_t nc = grown(n_states, 4096);
        int rc = regrow(&h->d_states, h->up_states, nc);
        // the literal bytes are read 8 at a time: keep 16 zero bytes behind the last state
        if (rc == WG_OK) rc = regrow(&h->d_lit, h->up_states, nc, 16);
        if (rc != WG_OK) return rc;
        h->cap_states = nc;
    }
    if (t.n_keys > kMaxKeys) return fail(WG_ERR_NOMEM, "more than 2^31 - 2 cache keys");
    if (t.n_keys > h->cap_keys) {
        const uint32_t nc = grown(t.n_keys, 4096);
        int rc = regrow(&h->dc.tags, h->cap_keys, nc);
        if (rc != WG_OK) return rc;
        h->cap_keys = nc;
    }
    if (n_classes > h->cap_classes) {
        const uint32_t nc = grown(n_classes, 64);
        int rc = regrow(&h->d_classes, (size_t)h->up_classes * 256, (size_t)nc * 256);
        if (rc == WG_OK) rc = regrow(&h->d_class_info, h->up_classes, nc);
        if (rc == WG_OK) rc = regrow(&h->dc.class_built, h->cap_classes, nc);
        // one pair of counters per class table, 128 bytes apart so that appends to different
        // tables do not meet in one cache line
        if (rc == WG_OK) rc = regrow(&h->dc.class_count, (size_t)h->cap_classes * 32, (size_t)nc * 32);
        if (rc == WG_OK) rc = regrow(&h->dc.class_rows, (size_t)h->cap_classes * 3 * row_stride, (size_t)nc * 3 * row_stride);
        if (rc == WG_OK) rc = regrow(&h->d_class_entries, h->cap_classes, nc);
        if (rc != WG_OK) return rc;
        h->cap_classes = nc;
    }
    const bool new_states = n_states > h->up_states, new_classes = n_classes > h->up_classes;
    if (new_states) {
        const uint32_t a = h->up_states, n = n_states - a;
        WG_HIP(hipMemcpyAsync(h->d_states + a, t.states.data() + a, n * sizeof(StateDesc), hipMemcpyHostToDevice, s));
        WG_HIP(hipMemcpyAsync(h->d_lit + a, t.lit.data() + a, n, hipMemcpyHostToDevice, s));
    }
    if (new_classes) {
        const uint32_t a = h->up_classes, n = n_classes - a;
        WG_HIP(hipMemcpyAsync(h->d_classes + (size_t)a * 256, t.classes.data() + (size_t)a * 256, (size_t)n * 256,
                              hipMemcpyHostToDevice, s));
        h->class_info.resize(n_classes);
        for (uint32_t c = a; c < n_classes; c++) h->class_info[c] = class_info_of(t.classes.data() + (size_t)c * 256);
        WG_HIP(hipMemcpyAsync(h->d_class_info + a, h->class_info.data() + a, n * sizeof(ClassInfo), hipMemcpyHostToDevice, s));
        // Per class table: V slots for the list of the whole table, V for the lists of its token
        // ranges.  The buffers are cut from slabs of several, so that an instance which brings
        // one new table does not pay for a device allocation of its own.
        const size_t per_class = 2u * (size_t)V;
        while (h->class_bufs.size() < n_classes) {           // (a call that failed half way left some)
            if (h->slab_left == 0) {
                const size_t missing = n_classes - h->class_bufs.size();
                const uint32_t count = (uint32_t)(missing > 8 ? missing : 8);
                ExitEntry *slab = nullptr;
                WG_HIP(hipMalloc(reinterpret_cast<void **>(&slab), count * per_class * sizeof(ExitEntry)));
                h->class_slabs.push_back(slab);
                h->slab_left = count;
                h->class_bufs.push_back(slab);
            } else {
                h->class_bufs.push_back(h->class_bufs.back() + per_class);
            }
            h->slab_left--;
        }
        WG_HIP(hipMemcpyAsync(h->d_class_entries + a, h->class_bufs.data() + a, n * sizeof(ExitEntry *),
                              hipMemcpyHostToDevice, s));
    }
    if (new_states || new_classes) {
        // the copies read pageable host memory that a later append may move
        WG_HIP(hipStreamSynchronize(s));
        h->up_states = n_states;
        h->up_classes = n_classes;
    }
    h->dt = DeviceTable{h->d_states, h->d_classes, h->d_class_info, h->d_lit, n_states, t.lmax, n_classes};
    h->dc.class_entries = h->d_class_entries;
    h->dc.n_keys = t.n_keys;
    return WG_OK;
}

int set_cache_rows(wg_handle_s *h, uint32_t rows) {
    const size_t row_bytes = (size_t)h->dc.row_stride * 4u;
    uint32_t *arena = nullptr;
    WG_HIP(hipMalloc(reinterpret_cast<void **>(&arena), (size_t)rows * row_bytes + 16));
    (void)hipFree(h->dc.arena);
    h->dc.arena = arena;
    h->dc.cap_rows = rows;
    return WG_OK;
}

// A new cache generation: every row and class index made so far is stale from the next call on.
int next_generation(wg_handle_s *h, hipStream_t s) {
    if (++h->dc.epoch >= (1u << 30)) {                 // out of generation numbers: reset the tags for real
        WG_HIP(hipMemsetAsync(h->dc.tags, 0, (size_t)h->cap_keys * sizeof(unsigned long long), s));
        WG_HIP(hipMemsetAsync(h->dc.class_built, 0, (size_t)h->cap_classes * sizeof(uint32_t), s));
        WG_HIP(hipMemsetAsync(&h->dc.ctr->slot_ctr, 0, sizeof(unsigned long long), s));
        h->dc.epoch = 1;
    }
    return WG_OK;
}

}  // namespace

extern "C" {

const char *wg_last_error(void) { return g_last_error.c_str(); }

// ---- vocabulary ------------------------------------------------------------------------------

int wg_vocab_create(const uint8_t *host_bytes, const uint64_t *host_offsets, uint32_t V,
                    int32_t eos_id, wg_vocab_t *out) {
    if (!out) return fail(WG_ERR_INVALID, "wg_vocab_create: out is null");
    *out = nullptr;
    if (!host_offsets || V == 0) return fail(WG_ERR_INVALID, "wg_vocab_create: empty vocabulary");
    if (eos_id >= (int64_t)V) return fail(WG_ERR_INVALID, "wg_vocab_create: eos_id outside the vocabulary");
    VocabIndex ix;
    {
        std::string err;
        const int rc = build_vocab_index(host_bytes, host_offsets, V, eos_id, &ix, &err);
        if (rc != WG_OK) return fail(rc, err);
    }
    std::unique_ptr<wg_vocab_s> v(new (std::nothrow) wg_vocab_s);
    if (!v) return fail(WG_ERR_NOMEM, "wg_vocab_create: out of host memory");
    WG_HIP(hipGetDevice(&v->device));
    {
        // set-up time on this device: the address of the library's own top-k workspace is asked
        // for here, so that wg_masked_topk_static finds it known (it asks itself otherwise)
        unsigned long long *unused = nullptr;
        (void)static_topk_scratch(&unused);
    }
    hipError_t e = upload(&v->d_bytes, ix.bytes.data(), ix.bytes.size());
    if (e == hipSuccess) e = upload(&v->d_offsets, ix.offsets.data(), ix.offsets.size());
    if (e == hipSuccess) e = upload(&v->d_len8, ix.len8.data(), ix.len8.size());
    if (e == hipSuccess) e = upload(&v->d_chunks, ix.chunks.data(), ix.chunks.size());
    if (e == hipSuccess) e = upload(&v->d_sig, ix.sig.data(), ix.sig.size());
    if (e == hipSuccess) e = upload(&v->d_first8, ix.first8.data(), ix.first8.size());
    if (e == hipSuccess) e = upload(&v->d_lit_entries, ix.lit_entries.data(), ix.lit_entries.size());
    if (e == hipSuccess) e = upload(&v->d_lit_start, ix.lit_start.data(), ix.lit_start.size());
    if (e == hipSuccess) e = upload(&v->d_len_rows, ix.len_rows.data(), ix.len_rows.size());
    if (e == hipSuccess) e = upload(&v->d_sorted, ix.sorted.data(), ix.sorted.size());
    if (e == hipSuccess) e = upload(&v->d_dir0, ix.dir0.data(), ix.dir0.size());
    if (e == hipSuccess) e = upload(&v->d_bigram, ix.bigram.data(), ix.bigram.size());
    if (e == hipSuccess) e = upload(&v->d_dirN, ix.dirN.data(), ix.dirN.size());
    if (e == hipSuccess) e = upload(&v->d_byte_rows, ix.byte_rows.data(), ix.byte_rows.size());
    if (e != hipSuccess) {
        v->release();
        return fail(e == hipErrorOutOfMemory ? WG_ERR_NOMEM : WG_ERR_HIP,
                    std::string("wg_vocab_create: ") + hipGetErrorString(e));
    }
    v->dv = DeviceVocab{v->d_bytes, v->d_offsets, v->d_len8, v->d_chunks, v->d_sig, v->d_first8, v->d_lit_entries,
                        v->d_lit_start, v->d_len_rows, v->d_sorted, v->d_dir0, v->d_bigram, v->d_dirN, v->d_byte_rows,
                        V, ix.W, eos_id, ix.lmax, ix.n_chunks, ix.row_stride, {}};
    for (uint32_t p = 0; p <= kParts; p++) v->dv.part_tok[p] = ix.part_tok[p];
    *out = v.release();
    return WG_OK;
}

void wg_vocab_destroy(wg_vocab_t v) {
    if (!v) return;
    v->release();
    delete v;
}

// ---- lowering (host only) ----------------------------------------------------------------------

int wg_lower(const char *const *templates, const wg_args_t *args, uint32_t n_templates,
             uint32_t flags, uint32_t lmax, wg_table_t *out) {
    if (!out) return fail(WG_ERR_INVALID, "wg_lower: out is null");
    *out = nullptr;
    if (!templates || n_templates == 0) return fail(WG_ERR_INVALID, "wg_lower: no templates");
    if (flags & ~(uint32_t)(WG_EOS_RESTART | WG_SHARE_STATES)) return fail(WG_ERR_INVALID, "wg_lower: unknown flag bits");
    try {
        std::unique_ptr<wg_table_s> t(new wg_table_s(flags, lmax));
        t->low.add(templates, args, n_templates);
        *out = t.release();
        return WG_OK;
    } catch (const std::bad_alloc &) {
        return fail(WG_ERR_NOMEM, "wg_lower: out of host memory");
    } catch (const std::exception &e) {
        return fail(WG_ERR_PARSE, e.what());
    }
}

int wg_table_add_instances(wg_table_t t, const char *const *templates, const wg_args_t *args,
                           uint32_t n_templates) {
    if (!t) return fail(WG_ERR_INVALID, "wg_table_add_instances: null table");
    if (!templates || n_templates == 0) return fail(WG_ERR_INVALID, "wg_table_add_instances: no templates");
    try {
        t->low.add(templates, args, n_templates);
        return WG_OK;
    } catch (const std::bad_alloc &) {
        return fail(WG_ERR_NOMEM, "wg_table_add_instances: out of host memory");
    } catch (const std::exception &e) {
        return fail(WG_ERR_PARSE, e.what());
    }
}

int wg_regex_to_template(const char *regex, char *out, uint64_t capacity, uint64_t *needed) {
    if (!regex) return fail(WG_ERR_INVALID, "wg_regex_to_template: regex is null");
    try {
        const std::string text = regex_to_template(regex);
        if (needed) *needed = text.size() + 1;
        if (!out || capacity < text.size() + 1)
            return fail(WG_ERR_INVALID, "wg_regex_to_template: the template needs " +
                                            std::to_string(text.size() + 1) + " bytes");
        std::memcpy(out, text.c_str(), text.size() + 1);
        return WG_OK;
    } catch (const std::bad_alloc &) {
        return fail(WG_ERR_NOMEM, "wg_regex_to_template: out of host memory");
    } catch (const std::exception &e) {
        return fail(WG_ERR_PARSE, e.what());
    }
}

uint32_t wg_table_num_instances(wg_table_t t) { return t ? (uint32_t)t->low.table.start.size() : 0; }

uint32_t wg_table_num_states(wg_table_t t) { return t ? (uint32_t)t->low.table.states.size() : 0; }

uint32_t wg_table_start_state(wg_table_t t, uint32_t i) {
    return (t && i < t->low.table.start.size()) ? t->low.table.start[i] : WG_SID_ERROR;
}

int wg_table_state(wg_table_t t, uint32_t sid, wg_state_info_t *out) {
    if (!t || !out || sid >= t->low.table.states.size()) return fail(WG_ERR_INVALID, "wg_table_state: bad argument");
    const Table &tb = t->low.table;
    const StateDesc &d = tb.states[sid];
    out->kind = d.kind_byte & 0xFFu; out->byte = (d.kind_byte >> 8) & 0xFFu;
    out->next_a = d.next_a; out->next_b = d.next_b; out->eos_next = d.eos_next; out->max = d.max;
    out->tmpl = tb.tmpl[sid]; out->n_keys = tb.key_count[sid]; out->key = d.key_base;
    return WG_OK;
}

int wg_table_symbol_class(wg_table_t t, uint32_t sid, uint32_t symbol) {
    if (!t || sid >= t->low.table.states.size() || symbol > kSymEos) return fail(WG_ERR_INVALID, "wg_table_symbol_class: bad argument");
    const StateDesc &d = t->low.table.states[sid];
    uint32_t kind = d.kind_byte & 0xFFu;
    if (symbol == kSymEos) return d.eos_next == WG_SID_ERROR ? CLS_REJECT : CLS_EXIT_A;
    if (kind == WG_KIND_LIT) return symbol == ((d.kind_byte >> 8) & 0xFFu) ? CLS_EXIT_A : CLS_REJECT;
    if (kind == WG_KIND_WAIT || kind == WG_KIND_COND) return t->low.table.classes[(size_t)d.cls * 256 + symbol];
    return CLS_REJECT;
}

void wg_table_destroy(wg_table_t t) { delete t; }

// ---- compile ------------------------------------------------------------------------------------

void wg_destroy(wg_handle_t h) {
    if (!h) return;
    (void)hipDeviceSynchronize();
    (void)hipFree(h->d_states); (void)hipFree(h->d_classes); (void)hipFree(h->d_lit); (void)hipFree(h->d_class_info);
    (void)hipFree(h->dc.ctr); (void)hipFree(h->dc.tags); (void)hipFree(h->dc.arena);
    (void)hipFree(h->dc.row_ref); (void)hipFree(h->dc.miss); (void)hipFree(h->dc.class_miss);
    (void)hipFree(h->dc.class_built); (void)hipFree(h->dc.class_rows);
    (void)hipFree(h->d_class_entries); (void)hipFree(h->dc.class_count);
    for (ExitEntry *b : h->class_slabs) (void)hipFree(b);
    for (auto *v : {&h->fill_events, &h->advance_events, &h->apply_events, &h->spare_events})
        for (hipEvent_t e : *v) if (e) (void)hipEventDestroy(e);
    delete h;
}

int wg_compile(const char *const *templates, const wg_args_t *args, uint32_t n_templates,
               wg_vocab_t vocab, uint32_t flags, wg_handle_t *out, wg_state_t *start_states_out) {
    if (!out) return fail(WG_ERR_INVALID, "wg_compile: out is null");
    *out = nullptr;
    if (!vocab) return fail(WG_ERR_INVALID, "wg_compile: vocab is null");
    if (!templates || n_templates == 0) return fail(WG_ERR_INVALID, "wg_compile: no templates");
    if (flags & ~(uint32_t)(WG_EOS_RESTART | WG_SHARE_STATES)) return fail(WG_ERR_INVALID, "wg_compile: unknown flag bits");
    std::unique_ptr<wg_handle_s, void (*)(wg_handle_t)> h(
        new (std::nothrow) wg_handle_s(flags, vocab->dv.lmax), wg_destroy);
    if (!h) return fail(WG_ERR_NOMEM, "wg_compile: out of host memory");
    try {
        h->low.add(templates, args, n_templates);
    } catch (const std::bad_alloc &) {
        return fail(WG_ERR_NOMEM, "wg_compile: out of host memory");
    } catch (const std::exception &e) {
        return fail(WG_ERR_PARSE, e.what());
    }
    h->vocab = vocab;
    const Table &t = h->low.table;
    WG_HIP(hipSetDevice(vocab->device));
    hipDeviceProp_t prop;
    WG_HIP(hipGetDeviceProperties(&prop, vocab->device));
    h->n_cu = prop.multiProcessorCount > 0 ? (uint32_t)prop.multiProcessorCount : 256u;

    const uint32_t row_stride = vocab->dv.row_stride;
    const uint64_t row_bytes = (uint64_t)row_stride * 4ull;
    {
        const hipError_t e = configure_kernels(row_stride * 4u);
        if (e == hipErrorInvalidValue)
            return fail(WG_ERR_INVALID, "wg_compile: a mask row does not fit the LDS of a compute unit next to the "
                                        "builder's queue (vocabulary too large)");
        WG_HIP(e);
    }
    h->dc.row_stride = row_stride;
    h->dc.epoch = 1;                                   // tags start at 0 = never built

    // The row cache: room for every key of the instances given here (at least 4096 rows), but
    // no more than a quarter of the free device memory; keys beyond it are served uncached.
    size_t free_b = 0, total_b = 0;
    WG_HIP(hipMemGetInfo(&free_b, &total_b));
    const uint64_t n_classes = t.classes.size() / 256;
    const uint64_t class_bytes = n_classes * (3ull * row_bytes + 2ull * vocab->dv.V * sizeof(ExitEntry));
    if (class_bytes > (uint64_t)free_b / 4)
        return fail(WG_ERR_NOMEM, "wg_compile: the class indexes (" + std::to_string(class_bytes >> 20) +
                                      " MiB for " + std::to_string(n_classes) +
                                      " allow / wait set tables) exceed a quarter of the free device memory");
    uint64_t rows = t.n_keys < 4096u ? 4096u : t.n_keys;
    const uint64_t fit = (uint64_t)free_b / 4 / row_bytes;
    if (rows > fit) rows = fit ? fit : 1;
    if (rows > kMaxRows) rows = kMaxRows;

    WG_HIP(hipMalloc(reinterpret_cast<void **>(&h->dc.ctr), sizeof(Counters)));
    WG_HIP(hipMemset(h->dc.ctr, 0, sizeof(Counters)));
    int rc = set_cache_rows(h.get(), (uint32_t)rows);
    if (rc == WG_OK) rc = sync_table(h.get(), nullptr);
    if (rc == WG_OK) rc = reserve_batch(h.get(), kDefaultBatch);
    if (rc != WG_OK) return rc;
    WG_HIP(hipDeviceSynchronize());
    if (start_states_out)
        for (uint32_t i = 0; i < n_templates; i++) start_states_out[i] = wg_state_t{t.start[i], 0u};
    *out = h.release();
    return WG_OK;
}

int wg_add_instances(wg_handle_t h, const char *const *templates, const wg_args_t *args,
                     uint32_t n_templates, wg_state_t *start_states_out, void *stream) {
    if (!h) return fail(WG_ERR_INVALID, "wg_add_instances: null handle");
    if (!templates || n_templates == 0) return fail(WG_ERR_INVALID, "wg_add_instances: no templates");
    const size_t first = h->low.table.start.size();
    try {
        h->low.add(templates, args, n_templates);
    } catch (const std::bad_alloc &) {
        return fail(WG_ERR_NOMEM, "wg_add_instances: out of host memory");
    } catch (const std::exception &e) {
        return fail(WG_ERR_PARSE, e.what());
    }
    WG_HIP(hipSetDevice(h->vocab->device));
    int rc = sync_table(h, static_cast<hipStream_t>(stream));
    if (rc != WG_OK) return rc;
    if (start_states_out)
        for (uint32_t i = 0; i < n_templates; i++)
            start_states_out[i] = wg_state_t{h->low.table.start[first + i], 0u};
    return WG_OK;
}

int wg_cache_resize(wg_handle_t h, uint32_t rows) {
    if (!h) return fail(WG_ERR_INVALID, "wg_cache_resize: null handle");
    if (rows == 0 || rows > kMaxRows) return fail(WG_ERR_INVALID, "wg_cache_resize: rows must be 1 .. 2^30");
    WG_HIP(hipSetDevice(h->vocab->device));
    WG_HIP(hipDeviceSynchronize());
    int rc = set_cache_rows(h, rows);
    if (rc != WG_OK) return rc;
    return next_generation(h, nullptr);
}

int wg_reserve_batch(wg_handle_t h, uint32_t max_batch) {
    if (!h) return fail(WG_ERR_INVALID, "wg_reserve_batch: null handle");
    if (max_batch == 0 || max_batch > kMaxBatch) return fail(WG_ERR_INVALID, "wg_reserve_batch: max_batch must be 1 .. 65535");
    WG_HIP(hipSetDevice(h->vocab->device));
    return reserve_batch(h, max_batch);
}

uint32_t wg_max_batch(wg_handle_t h) { return h ? h->max_batch : 0; }

int wg_set_scan_batch(wg_handle_t h, uint32_t tables) {
    if (!h) return fail(WG_ERR_INVALID, "wg_set_scan_batch: null handle");
    if (tables > 8u) return fail(WG_ERR_INVALID, "wg_set_scan_batch: tables must be 0 .. 8");
    h->dc.scan_batch = tables;
    return WG_OK;
}

uint32_t wg_num_instances(wg_handle_t h) { return h ? (uint32_t)h->low.table.start.size() : 0; }
uint32_t wg_num_states(wg_handle_t h) { return h ? h->dt.n_states : 0; }
uint32_t wg_mask_words(wg_handle_t h) { return h ? h->vocab->dv.W : 0; }

// ---- per-step calls -----------------------------------------------------------------------------

namespace {
int fill(wg_handle_t h, wg_state_t *d_states, const int32_t *d_tokens, uint32_t B, uint32_t *d_bitmask,
         void *stream, const char *who, void *d_logits = nullptr, int dtype = WG_F32, int64_t logits_stride = 0) {
    if (B == 0) return fail(WG_ERR_INVALID, std::string(who) + ": B is 0");
    if (B > kMaxBatch) return fail(WG_ERR_INVALID, std::string(who) + ": B above 65535");
    if (B > h->max_batch)
        return fail(WG_ERR_INVALID, std::string(who) + ": B = " + std::to_string(B) + " is above the " +
                                        std::to_string(h->max_batch) + " requests the handle has room for (wg_reserve_batch)");
    hipEvent_t ev[8];
    if (h->profiling) for (auto &e : ev) { e = take_event(h); h->fill_events.push_back(e); }
    WG_HIP(launch_fill(h->dt, h->vocab->dv, h->dc, d_states, d_tokens, B, d_bitmask, d_logits, dtype,
                       logits_stride, h->n_cu, static_cast<hipStream_t>(stream), h->profiling ? ev : nullptr));
    return WG_OK;
}
}  // namespace

int wg_fill_masks(wg_handle_t h, const wg_state_t *d_states, uint32_t B, uint32_t *d_bitmask,
                  void *stream) {
    if (!h || !d_states || !d_bitmask) return fail(WG_ERR_INVALID, "wg_fill_masks: null argument");
    // the states are only read when no tokens are given
    return fill(h, const_cast<wg_state_t *>(d_states), nullptr, B, d_bitmask, stream, "wg_fill_masks");
}

int wg_advance_fill_masks(wg_handle_t h, wg_state_t *d_states, const int32_t *d_tokens, uint32_t B,
                          uint32_t *d_bitmask, void *stream) {
    if (!h || !d_states || !d_tokens || !d_bitmask)
        return fail(WG_ERR_INVALID, "wg_advance_fill_masks: null argument");
    return fill(h, d_states, d_tokens, B, d_bitmask, stream, "wg_advance_fill_masks");
}

int wg_decode_step(wg_handle_t h, wg_state_t *d_states, const int32_t *d_tokens, uint32_t B,
                   uint32_t *d_bitmask, void *d_logits, wg_dtype_t dtype, int64_t row_stride_elems,
                   void *stream) {
    if (!h || !d_states || !d_bitmask || !d_logits) return fail(WG_ERR_INVALID, "wg_decode_step: null argument");
    if (dtype != WG_F32 && dtype != WG_BF16) return fail(WG_ERR_INVALID, "wg_decode_step: unknown dtype");
    if (row_stride_elems < (int64_t)h->vocab->dv.V) return fail(WG_ERR_INVALID, "wg_decode_step: row stride smaller than V");
    return fill(h, d_states, d_tokens, B, d_bitmask, stream, "wg_decode_step", d_logits, dtype, row_stride_elems);
}

int wg_apply_mask(void *d_logits, wg_dtype_t dtype, uint32_t B, uint32_t V, int64_t row_stride_elems,
                  const uint32_t *d_bitmask, void *stream) {
    if (!d_logits || !d_bitmask) return fail(WG_ERR_INVALID, "wg_apply_mask: null argument");
    if (B == 0 || V == 0) return fail(WG_ERR_INVALID, "wg_apply_mask: empty batch or vocabulary");
    if (dtype != WG_F32 && dtype != WG_BF16) return fail(WG_ERR_INVALID, "wg_apply_mask: unknown dtype");
    if (row_stride_elems < (int64_t)V) return fail(WG_ERR_INVALID, "wg_apply_mask: row stride smaller than V");
    if (B > kMaxBatch) return fail(WG_ERR_INVALID, "wg_apply_mask: B above 65535");
    WG_HIP(launch_apply(d_logits, dtype, B, V, row_stride_elems, d_bitmask, static_cast<hipStream_t>(stream), nullptr));
    return WG_OK;
}

int wg_profile_apply_mask(wg_handle_t h, void *d_logits, wg_dtype_t dtype, uint32_t B, uint32_t V,
                          int64_t row_stride_elems, const uint32_t *d_bitmask, void *stream) {
    if (!h) return fail(WG_ERR_INVALID, "wg_profile_apply_mask: null handle");
    if (!h->profiling) return wg_apply_mask(d_logits, dtype, B, V, row_stride_elems, d_bitmask, stream);
    if (!d_logits || !d_bitmask) return fail(WG_ERR_INVALID, "wg_profile_apply_mask: null argument");
    if (B == 0 || V == 0 || B > kMaxBatch) return fail(WG_ERR_INVALID, "wg_profile_apply_mask: bad batch or vocabulary size");
    if (dtype != WG_F32 && dtype != WG_BF16) return fail(WG_ERR_INVALID, "wg_profile_apply_mask: unknown dtype");
    if (row_stride_elems < (int64_t)V) return fail(WG_ERR_INVALID, "wg_profile_apply_mask: row stride smaller than V");
    hipEvent_t ev[2];
    for (auto &e : ev) { e = take_event(h); h->apply_events.push_back(e); }
    WG_HIP(launch_apply(d_logits, dtype, B, V, row_stride_elems, d_bitmask, static_cast<hipStream_t>(stream), ev));
    return WG_OK;
}

int wg_masked_argmax(const void *d_logits, wg_dtype_t dtype, uint32_t B, uint32_t V,
                     int64_t row_stride_elems, const uint32_t *d_bitmask, int32_t *d_tokens, void *stream) {
    if (!d_logits || !d_bitmask || !d_tokens) return fail(WG_ERR_INVALID, "wg_masked_argmax: null argument");
    if (B == 0 || V == 0) return fail(WG_ERR_INVALID, "wg_masked_argmax: empty batch or vocabulary");
    if (dtype != WG_F32 && dtype != WG_BF16) return fail(WG_ERR_INVALID, "wg_masked_argmax: unknown dtype");
    if (row_stride_elems < (int64_t)V) return fail(WG_ERR_INVALID, "wg_masked_argmax: row stride smaller than V");
    if (B > kMaxBatch) return fail(WG_ERR_INVALID, "wg_masked_argmax: B above 65535");
    WG_HIP(launch_masked_argmax(d_logits, dtype, B, V, row_stride_elems, d_bitmask, d_tokens,
                                static_cast<hipStream_t>(stream)));
    return WG_OK;
}

uint64_t wg_masked_topk_workspace(uint32_t B, uint32_t V, uint32_t k) {
    const uint64_t n_slices = ((uint64_t)V + kTopkSlice - 1u) / kTopkSlice;
    return (uint64_t)B * n_slices * k * sizeof(unsigned long long);
}

int wg_masked_topk(const void *d_logits, wg_dtype_t dtype, uint32_t B, uint32_t V, int64_t row_stride_elems,
                   const uint32_t *d_bitmask, uint32_t k, int32_t *d_ids, void *d_values,
                   void *d_workspace, uint64_t workspace_bytes, void *stream) {
    if (!d_logits || !d_bitmask || !d_ids || !d_values || !d_workspace)
        return fail(WG_ERR_INVALID, "wg_masked_topk: null argument");
    if (B == 0 || V == 0) return fail(WG_ERR_INVALID, "wg_masked_topk: empty batch or vocabulary");
    if (dtype != WG_F32 && dtype != WG_BF16) return fail(WG_ERR_INVALID, "wg_masked_topk: unknown dtype");
    if (row_stride_elems < (int64_t)V) return fail(WG_ERR_INVALID, "wg_masked_topk: row stride smaller than V");
    if (B > kMaxBatch) return fail(WG_ERR_INVALID, "wg_masked_topk: B above 65535");
    if (k == 0 || k > kTopkMax) return fail(WG_ERR_INVALID, "wg_masked_topk: k must be 1 .. 64");
    const uint64_t n_slices = ((uint64_t)V + kTopkSlice - 1u) / kTopkSlice;
    // the lists of a row's slices are merged in LDS, next to the merge's own 18 KB, within the
    // 64 KB a kernel gets without asking
    if (n_slices * k > kTopkMergeKeys)
        return fail(WG_ERR_INVALID, "wg_masked_topk: ceil(V / 8192) * k above 4096 (the lists of a row do not fit the merge)");
    if (workspace_bytes < wg_masked_topk_workspace(B, V, k))
        return fail(WG_ERR_INVALID, "wg_masked_topk: the workspace needs " +
                                        std::to_string(wg_masked_topk_workspace(B, V, k)) + " bytes");
    if (reinterpret_cast<uintptr_t>(d_workspace) % 8 != 0)
        return fail(WG_ERR_INVALID, "wg_masked_topk: the workspace must be 8-byte aligned");
    WG_HIP(launch_masked_topk(d_logits, dtype, B, V, row_stride_elems, d_bitmask, k, d_ids, d_values,
                              static_cast<unsigned long long *>(d_workspace), static_cast<hipStream_t>(stream)));
    return WG_OK;
}

uint64_t wg_masked_topk_static_capacity(void) { return kTopkStaticKeys * sizeof(unsigned long long); }

int wg_masked_topk_static(const void *d_logits, wg_dtype_t dtype, uint32_t B, uint32_t V, int64_t row_stride_elems,
                          const uint32_t *d_bitmask, uint32_t k, int32_t *d_ids, void *d_values, void *stream) {
    if (!d_logits || !d_bitmask || !d_ids || !d_values)
        return fail(WG_ERR_INVALID, "wg_masked_topk_static: null argument");
    if (B == 0 || V == 0) return fail(WG_ERR_INVALID, "wg_masked_topk_static: empty batch or vocabulary");
    if (dtype != WG_F32 && dtype != WG_BF16) return fail(WG_ERR_INVALID, "wg_masked_topk_static: unknown dtype");
    if (row_stride_elems < (int64_t)V) return fail(WG_ERR_INVALID, "wg_masked_topk_static: row stride smaller than V");
    if (B > kMaxBatch) return fail(WG_ERR_INVALID, "wg_masked_topk_static: B above 65535");
    if (k == 0 || k > kTopkMax) return fail(WG_ERR_INVALID, "wg_masked_topk_static: k must be 1 .. 64");
    const uint64_t n_slices = ((uint64_t)V + kTopkSlice - 1u) / kTopkSlice;
    if (n_slices * k > kTopkMergeKeys)
        return fail(WG_ERR_INVALID, "wg_masked_topk_static: ceil(V / 8192) * k above 4096 (the lists of a row do not fit the merge)");
    const uint64_t need = wg_masked_topk_workspace(B, V, k);
    if (need > wg_masked_topk_static_capacity())
        return fail(WG_ERR_INVALID, "wg_masked_topk_static: B * ceil(V / 8192) * k * 8 = " + std::to_string(need) +
                                        " bytes of lists, above the " + std::to_string(wg_masked_topk_static_capacity()) +
                                        " the library holds per GPU (use wg_masked_topk with a workspace)");
    unsigned long long *lists = nullptr;
    WG_HIP(static_topk_scratch(&lists));
    WG_HIP(launch_masked_topk(d_logits, dtype, B, V, row_stride_elems, d_bitmask, k, d_ids, d_values, lists,
                              static_cast<hipStream_t>(stream)));
    return WG_OK;
}

int wg_advance(wg_handle_t h, wg_state_t *d_states, const int32_t *d_tokens, uint32_t B, void *stream) {
    if (!h || !d_states || !d_tokens) return fail(WG_ERR_INVALID, "wg_advance: null argument");
    if (B == 0) return fail(WG_ERR_INVALID, "wg_advance: B is 0");
    hipEvent_t ev[2];
    if (h->profiling) for (auto &e : ev) { e = take_event(h); h->advance_events.push_back(e); }
    WG_HIP(launch_advance(h->dt, h->vocab->dv, h->dc, d_states, d_tokens, B,
                          static_cast<hipStream_t>(stream), h->profiling ? ev : nullptr));
    return WG_OK;
}

int wg_forced_bytes(wg_handle_t h, const wg_state_t *d_states, uint32_t B, uint32_t cap, uint8_t *d_bytes,
                    uint32_t *d_lens, wg_state_t *d_end_states, void *stream) {
    if (!h || !d_states || !d_bytes || !d_lens) return fail(WG_ERR_INVALID, "wg_forced_bytes: null argument");
    if (B == 0 || cap == 0) return fail(WG_ERR_INVALID, "wg_forced_bytes: B or cap is 0");
    WG_HIP(launch_forced_bytes(h->dt, d_states, B, cap, d_bytes, d_lens, d_end_states, static_cast<hipStream_t>(stream)));
    return WG_OK;
}

int wg_cache_clear(wg_handle_t h, void *stream) {
    if (!h) return fail(WG_ERR_INVALID, "wg_cache_clear: null handle");
    // The generation number travels with every later launch as a kernel argument, so the
    // clear is ordered with the caller's other calls on this handle without touching the GPU.
    return next_generation(h, static_cast<hipStream_t>(stream));
}

int wg_cache_stats(wg_handle_t h, wg_cache_stats_t *host_out) {
    if (!h || !host_out) return fail(WG_ERR_INVALID, "wg_cache_stats: null argument");
    Counters c;
    WG_HIP(hipDeviceSynchronize());
    WG_HIP(hipMemcpy(&c, h->dc.ctr, sizeof c, hipMemcpyDeviceToHost));
    host_out->lookups = c.lookups; host_out->hits = c.hits; host_out->builds = c.builds;
    host_out->uncached_builds = c.uncached_builds;
    host_out->class_scans = c.class_scans; host_out->entries_walked = c.entries_walked;
    host_out->keys = h->dc.n_keys;
    host_out->cache_rows = h->dc.cap_rows;
    const uint64_t taken = (uint32_t)(c.slot_ctr >> 32) == h->dc.epoch ? (uint32_t)c.slot_ctr : 0u;
    host_out->rows_in_use = taken < h->dc.cap_rows ? taken : h->dc.cap_rows;
    const uint64_t row_bytes = (uint64_t)h->dc.row_stride * 4ull;
    host_out->arena_bytes = (uint64_t)h->dc.cap_rows * row_bytes +
                            (uint64_t)(h->class_bufs.size() + h->slab_left) * (2ull * h->vocab->dv.V * sizeof(ExitEntry)) +
                            (uint64_t)h->cap_classes * 3ull * row_bytes;
    return WG_OK;
}

int wg_error_count(wg_handle_t h, uint64_t *host_out) {
    if (!h || !host_out) return fail(WG_ERR_INVALID, "wg_error_count: null argument");
    Counters c;
    WG_HIP(hipDeviceSynchronize());
    WG_HIP(hipMemcpy(&c, h->dc.ctr, sizeof c, hipMemcpyDeviceToHost));
    *host_out = c.errors;
    return WG_OK;
}

int wg_profile_enable(wg_handle_t h, int on) {
    if (!h) return fail(WG_ERR_INVALID, "wg_profile_enable: null handle");
    h->profiling = on != 0;
    return WG_OK;
}

int wg_profile_read(wg_handle_t h, wg_profile_t *host_out) {
    if (!h || !host_out) return fail(WG_ERR_INVALID, "wg_profile_read: null argument");
    WG_HIP(hipDeviceSynchronize());
    wg_profile_t p{};
    auto span = [](hipEvent_t a, hipEvent_t b) {
        float ms = 0.f;
        return (a && b && hipEventElapsedTime(&ms, a, b) == hipSuccess) ? (double)ms : 0.0;
    };
    for (size_t i = 0; i + 7 < h->fill_events.size(); i += 8) {
        hipEvent_t *e = &h->fill_events[i];
        p.lookup_ms += span(e[0], e[1]); p.scan_ms += span(e[2], e[3]);
        p.build_ms += span(e[4], e[5]); p.gather_ms += span(e[6], e[7]);
        p.fill_calls++;
    }
    for (size_t i = 0; i + 1 < h->advance_events.size(); i += 2) {
        p.advance_ms += span(h->advance_events[i], h->advance_events[i + 1]);
        p.advance_calls++;
    }
    for (size_t i = 0; i + 1 < h->apply_events.size(); i += 2) {
        p.apply_ms += span(h->apply_events[i], h->apply_events[i + 1]);
        p.apply_calls++;
    }
    for (auto *v : {&h->fill_events, &h->advance_events, &h->apply_events}) {
        h->spare_events.insert(h->spare_events.end(), v->begin(), v->end());
        v->clear();
    }
    *host_out = p;
    return WG_OK;
}

int wg_select_tokens(const uint32_t *d_bitmask, uint32_t B, uint32_t V, const uint64_t *d_draws,
                     int32_t *d_tokens, void *stream) {
    if (!d_bitmask || !d_draws || !d_tokens) return fail(WG_ERR_INVALID, "wg_select_tokens: null argument");
    if (B == 0 || V == 0) return fail(WG_ERR_INVALID, "wg_select_tokens: empty batch or vocabulary");
    WG_HIP(launch_select(d_bitmask, B, V, d_draws, d_tokens, static_cast<hipStream_t>(stream)));
    return WG_OK;
}

}  // extern "C"
