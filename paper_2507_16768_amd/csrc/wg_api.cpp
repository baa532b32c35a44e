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

struct wg_table_s { Table t; };

struct wg_vocab_s {
    DeviceVocab dv{};
    uint8_t *d_bytes = nullptr, *d_len8 = nullptr;
    uint32_t *d_offsets = nullptr, *d_lit_start = nullptr, *d_len_rows = nullptr;
    uint64_t *d_chunks = nullptr;
    ExitEntry *d_lit_entries = nullptr;
    int device = 0;
    void release() {
        (void)hipFree(d_bytes); (void)hipFree(d_len8); (void)hipFree(d_offsets);
        (void)hipFree(d_lit_start); (void)hipFree(d_len_rows); (void)hipFree(d_chunks);
        (void)hipFree(d_lit_entries);
    }
};

struct wg_handle_s {
    wg_vocab_s *vocab = nullptr;
    Table table;
    DeviceTable dt{};
    DeviceCache dc{};
    StateDesc *d_states = nullptr;
    uint8_t *d_classes = nullptr, *d_lit = nullptr;
    uint32_t max_batch = 0;
    uint32_t n_cu = 256;
    uint64_t arena_bytes = 0;
    // kernel timing: events recorded since the last wg_profile_read
    bool profiling = false;
    std::vector<hipEvent_t> fill_events;       // 8 per wg_fill_masks call: begin / end of each kernel
    std::vector<hipEvent_t> advance_events;    // 2 per wg_advance call
    std::vector<hipEvent_t> spare_events;
};

namespace {

int fail(int code, const std::string &msg) { set_last_error(msg); return code; }

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

int ensure_batch(wg_handle_s *h, uint32_t B) {
    if (B <= h->max_batch) return WG_OK;
    // grows only when a larger batch than ever before arrives (synchronises once)
    uint32_t nb = h->max_batch ? h->max_batch : 1024;
    while (nb < B) nb *= 2;
    WG_HIP(hipDeviceSynchronize());
    if (h->dc.key_of) (void)hipFree(h->dc.key_of);
    if (h->dc.miss) (void)hipFree(h->dc.miss);
    if (h->dc.class_miss) (void)hipFree(h->dc.class_miss);
    h->dc.key_of = nullptr; h->dc.miss = nullptr; h->dc.class_miss = nullptr; h->max_batch = 0;
    WG_HIP(hipMalloc(reinterpret_cast<void **>(&h->dc.key_of), nb * sizeof(uint32_t)));
    WG_HIP(hipMalloc(reinterpret_cast<void **>(&h->dc.miss), nb * sizeof(MissEntry)));
    WG_HIP(hipMalloc(reinterpret_cast<void **>(&h->dc.class_miss), nb * sizeof(uint32_t)));
    h->max_batch = nb;
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
    uint64_t total = host_offsets[V];
    if (total && !host_bytes) return fail(WG_ERR_INVALID, "wg_vocab_create: host_bytes is null");
    if (total >= 0xFFFFFFFFull) return fail(WG_ERR_INVALID, "wg_vocab_create: more than 4 GiB of token bytes");
    std::vector<uint32_t> off(V + 1);
    uint32_t lmax = 0;
    for (uint32_t t = 0; t <= V; t++) {
        if (t && host_offsets[t] < host_offsets[t - 1])
            return fail(WG_ERR_INVALID, "wg_vocab_create: offsets are not non-decreasing");
        off[t] = (uint32_t)host_offsets[t];
        if (t && off[t] - off[t - 1] > lmax) lmax = off[t] - off[t - 1];
    }
    if (host_offsets[0] != 0) return fail(WG_ERR_INVALID, "wg_vocab_create: offsets must start at 0");
    if (lmax > 248) return fail(WG_ERR_INVALID, "wg_vocab_create: tokens longer than 248 bytes are not supported");
    std::unique_ptr<wg_vocab_s> v(new (std::nothrow) wg_vocab_s);
    if (!v) return fail(WG_ERR_NOMEM, "wg_vocab_create: out of host memory");
    WG_HIP(hipGetDevice(&v->device));
    const uint32_t W = (V + 31u) / 32u, rs = (W + 3u) & ~3u;
    const uint32_t n_chunks = (lmax + 7u) / 8u;
    // Static indexes of the vocabulary (they depend on the token bytes only):
    //  - 8 bytes of padding so kernels may over-read a token's tail
    //  - len8 / chunks: fixed-stride view, 8 bytes per load, for the class scan
    //  - first-byte buckets: the only tokens a literal state can admit
    //  - per-length rows: tokens with 1 <= length <= r, for Waits with a byte budget
    std::vector<uint8_t> bytes(total + 8, 0), len8(V, 0);
    if (total) std::memcpy(bytes.data(), host_bytes, total);
    std::vector<uint64_t> chunks((size_t)(n_chunks ? n_chunks : 1) * V, 0);
    std::vector<uint32_t> lit_start(257, 0), len_rows((size_t)(lmax + 2) * rs, 0);
    for (uint32_t t = 0; t < V; t++) {
        uint32_t L = ((int64_t)t == eos_id) ? 0u : off[t + 1] - off[t];
        len8[t] = (uint8_t)L;
        for (uint32_t i = 0; i < L; i++)
            chunks[(size_t)(i / 8u) * V + t] |= (uint64_t)bytes[off[t] + i] << (8u * (i % 8u));
        if (L) {
            lit_start[bytes[off[t]] + 1u]++;
            for (uint32_t r = L; r <= lmax + 1u; r++) len_rows[(size_t)r * rs + (t >> 5)] |= 1u << (t & 31u);
        }
    }
    for (int y = 0; y < 256; y++) lit_start[y + 1] += lit_start[y];
    // Within a bucket the entries are ordered by remaining length, so that the lanes of a
    // wavefront walk remainders of similar length.
    std::vector<ExitEntry> lit_entries(lit_start[256] ? lit_start[256] : 1);
    {
        std::vector<uint32_t> order;
        order.reserve(V);
        for (uint32_t t = 0; t < V; t++) if (len8[t]) order.push_back(t);
        std::stable_sort(order.begin(), order.end(), [&](uint32_t a, uint32_t b) {
            const uint32_t fa = bytes[off[a]], fb = bytes[off[b]];
            return fa != fb ? fa < fb : len8[a] < len8[b];
        });
        for (size_t i = 0; i < order.size(); i++) {
            const uint32_t t = order[i], L = len8[t];
            ExitEntry e;
            e.tok = t; e.off = 1; e.cls = CLS_EXIT_A;
            e.first = L > 1 ? bytes[off[t] + 1] : 0; e.rem = (uint8_t)(L - 1);
            lit_entries[i] = e;
        }
    }
    hipError_t e = upload(&v->d_bytes, bytes.data(), bytes.size());
    if (e == hipSuccess) e = upload(&v->d_offsets, off.data(), off.size());
    if (e == hipSuccess) e = upload(&v->d_len8, len8.data(), len8.size());
    if (e == hipSuccess) e = upload(&v->d_chunks, chunks.data(), chunks.size());
    if (e == hipSuccess) e = upload(&v->d_lit_entries, lit_entries.data(), lit_entries.size());
    if (e == hipSuccess) e = upload(&v->d_lit_start, lit_start.data(), lit_start.size());
    if (e == hipSuccess) e = upload(&v->d_len_rows, len_rows.data(), len_rows.size());
    if (e != hipSuccess) {
        v->release();
        return fail(e == hipErrorOutOfMemory ? WG_ERR_NOMEM : WG_ERR_HIP,
                    std::string("wg_vocab_create: ") + hipGetErrorString(e));
    }
    v->dv = DeviceVocab{v->d_bytes, v->d_offsets, v->d_len8, v->d_chunks, v->d_lit_entries,
                        v->d_lit_start, v->d_len_rows, V, W, eos_id, lmax, n_chunks, rs};
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
    if (flags & ~(uint32_t)WG_EOS_RESTART) return fail(WG_ERR_INVALID, "wg_lower: unknown flag bits");
    try {
        std::unique_ptr<wg_table_s> t(new wg_table_s);
        lower(templates, args, n_templates, flags, lmax, t->t);
        *out = t.release();
        return WG_OK;
    } catch (const std::bad_alloc &) {
        return fail(WG_ERR_NOMEM, "wg_lower: out of host memory");
    } catch (const std::exception &e) {
        return fail(WG_ERR_PARSE, e.what());
    }
}

uint32_t wg_table_num_states(wg_table_t t) { return t ? (uint32_t)t->t.states.size() : 0; }

uint32_t wg_table_start_state(wg_table_t t, uint32_t i) {
    return (t && i < t->t.start.size()) ? t->t.start[i] : WG_SID_ERROR;
}

int wg_table_state(wg_table_t t, uint32_t sid, wg_state_info_t *out) {
    if (!t || !out || sid >= t->t.states.size()) return fail(WG_ERR_INVALID, "wg_table_state: bad argument");
    const StateDesc &d = t->t.states[sid];
    out->kind = d.kind_byte & 0xFFu; out->byte = (d.kind_byte >> 8) & 0xFFu;
    out->next_a = d.next_a; out->next_b = d.next_b; out->eos_next = d.eos_next; out->max = d.max;
    out->tmpl = t->t.tmpl[sid]; out->n_keys = t->t.key_count[sid];
    return WG_OK;
}

int wg_table_symbol_class(wg_table_t t, uint32_t sid, uint32_t symbol) {
    if (!t || sid >= t->t.states.size() || symbol > kSymEos) return fail(WG_ERR_INVALID, "wg_table_symbol_class: bad argument");
    const StateDesc &d = t->t.states[sid];
    uint32_t kind = d.kind_byte & 0xFFu;
    if (symbol == kSymEos) return d.eos_next == WG_SID_ERROR ? CLS_REJECT : CLS_EXIT_A;
    if (kind == WG_KIND_LIT) return symbol == ((d.kind_byte >> 8) & 0xFFu) ? CLS_EXIT_A : CLS_REJECT;
    if (kind == WG_KIND_WAIT || kind == WG_KIND_COND) return t->t.classes[(size_t)d.cls * 256 + symbol];
    return CLS_REJECT;
}

void wg_table_destroy(wg_table_t t) { delete t; }

// ---- compile ------------------------------------------------------------------------------------

void wg_destroy(wg_handle_t h) {
    if (!h) return;
    (void)hipFree(h->d_states); (void)hipFree(h->d_classes); (void)hipFree(h->d_lit);
    (void)hipFree(h->dc.ctr); (void)hipFree(h->dc.built); (void)hipFree(h->dc.arena);
    (void)hipFree(h->dc.key_of); (void)hipFree(h->dc.miss); (void)hipFree(h->dc.class_miss);
    (void)hipFree(h->dc.class_built); (void)hipFree(h->dc.class_rows);
    (void)hipFree(h->dc.class_entries); (void)hipFree(h->dc.class_count);
    for (auto *v : {&h->fill_events, &h->advance_events, &h->spare_events})
        for (hipEvent_t e : *v) if (e) (void)hipEventDestroy(e);
    delete h;
}

int wg_compile(const char *const *templates, const wg_args_t *args, uint32_t n_templates,
               wg_vocab_t vocab, uint32_t flags, wg_handle_t *out, wg_state_t *start_states_out) {
    if (!out) return fail(WG_ERR_INVALID, "wg_compile: out is null");
    *out = nullptr;
    if (!vocab) return fail(WG_ERR_INVALID, "wg_compile: vocab is null");
    if (!templates || n_templates == 0) return fail(WG_ERR_INVALID, "wg_compile: no templates");
    if (flags & ~(uint32_t)WG_EOS_RESTART) return fail(WG_ERR_INVALID, "wg_compile: unknown flag bits");
    std::unique_ptr<wg_handle_s, void (*)(wg_handle_t)> h(new (std::nothrow) wg_handle_s, wg_destroy);
    if (!h) return fail(WG_ERR_NOMEM, "wg_compile: out of host memory");
    try {
        lower(templates, args, n_templates, flags, vocab->dv.lmax, h->table);
    } catch (const std::bad_alloc &) {
        return fail(WG_ERR_NOMEM, "wg_compile: out of host memory");
    } catch (const std::exception &e) {
        return fail(WG_ERR_PARSE, e.what());
    }
    h->vocab = vocab;
    const Table &t = h->table;
    WG_HIP(hipSetDevice(vocab->device));
    hipDeviceProp_t prop;
    WG_HIP(hipGetDeviceProperties(&prop, vocab->device));
    h->n_cu = prop.multiProcessorCount > 0 ? (uint32_t)prop.multiProcessorCount : 256u;

    const uint32_t row_stride = vocab->dv.row_stride;
    const uint32_t n_classes = (uint32_t)(t.classes.size() / 256);
    if ((uint64_t)row_stride * 4ull > 160ull * 1024ull)
        return fail(WG_ERR_INVALID, "wg_compile: a mask row does not fit the 160 KB of LDS (vocabulary too large)");
    WG_HIP(configure_kernels(row_stride * 4u));
    // the class index: 2 rows and up to V exit entries per class table
    const uint64_t class_bytes = (uint64_t)n_classes * (2ull * row_stride * 4ull + (uint64_t)vocab->dv.V * sizeof(ExitEntry));
    uint64_t arena_bytes = (uint64_t)t.n_keys * row_stride * 4ull + class_bytes;
    size_t free_b = 0, total_b = 0;
    WG_HIP(hipMemGetInfo(&free_b, &total_b));
    if (arena_bytes > (uint64_t)free_b / 2)
        return fail(WG_ERR_NOMEM, "wg_compile: the mask cache (" + std::to_string(arena_bytes >> 20) +
                                      " MiB for " + std::to_string(t.n_keys) +
                                      " keys) exceeds half of the free device memory");
    WG_HIP(upload(&h->d_states, t.states.data(), t.states.size()));
    WG_HIP(upload(&h->d_classes, t.classes.data(), t.classes.size()));
    WG_HIP(upload(&h->d_lit, t.lit.data(), t.lit.size()));
    h->dt = DeviceTable{h->d_states, h->d_classes, h->d_lit, (uint32_t)t.states.size(), t.lmax, n_classes};

    WG_HIP(hipMalloc(reinterpret_cast<void **>(&h->dc.ctr), sizeof(Counters)));
    Counters init{};
    WG_HIP(hipMemcpy(h->dc.ctr, &init, sizeof init, hipMemcpyHostToDevice));
    h->dc.epoch = 1;                                   // tags start at 0 = never built
    WG_HIP(hipMalloc(reinterpret_cast<void **>(&h->dc.built), (size_t)t.n_keys * sizeof(uint32_t)));
    WG_HIP(hipMemset(h->dc.built, 0, (size_t)t.n_keys * sizeof(uint32_t)));
    WG_HIP(hipMalloc(reinterpret_cast<void **>(&h->dc.arena), (size_t)t.n_keys * row_stride * 4ull + 16));
    WG_HIP(hipMalloc(reinterpret_cast<void **>(&h->dc.class_built), n_classes * sizeof(uint32_t)));
    WG_HIP(hipMemset(h->dc.class_built, 0, n_classes * sizeof(uint32_t)));
    // one counter per class table, 128 bytes apart so that appends to different tables do not
    // meet in one cache line
    WG_HIP(hipMalloc(reinterpret_cast<void **>(&h->dc.class_count), n_classes * 32 * sizeof(uint32_t)));
    WG_HIP(hipMemset(h->dc.class_count, 0, n_classes * 32 * sizeof(uint32_t)));
    WG_HIP(hipMalloc(reinterpret_cast<void **>(&h->dc.class_rows), (size_t)n_classes * 2ull * row_stride * 4ull));
    WG_HIP(hipMalloc(reinterpret_cast<void **>(&h->dc.class_entries), (size_t)n_classes * vocab->dv.V * sizeof(ExitEntry)));
    h->arena_bytes = arena_bytes;
    h->dc.row_stride = row_stride;
    h->dc.n_keys = t.n_keys;
    int rc = ensure_batch(h.get(), 1024);
    if (rc != WG_OK) return rc;
    WG_HIP(hipDeviceSynchronize());
    if (start_states_out)
        for (uint32_t i = 0; i < n_templates; i++) start_states_out[i] = wg_state_t{t.start[i], 0u};
    *out = h.release();
    return WG_OK;
}

uint32_t wg_num_states(wg_handle_t h) { return h ? h->dt.n_states : 0; }
uint32_t wg_mask_words(wg_handle_t h) { return h ? h->vocab->dv.W : 0; }

// ---- per-step calls -----------------------------------------------------------------------------

int wg_fill_masks(wg_handle_t h, const wg_state_t *d_states, uint32_t B, uint32_t *d_bitmask,
                  void *stream) {
    if (!h || !d_states || !d_bitmask) return fail(WG_ERR_INVALID, "wg_fill_masks: null argument");
    if (B == 0) return fail(WG_ERR_INVALID, "wg_fill_masks: B is 0");
    int rc = ensure_batch(h, B);
    if (rc != WG_OK) return rc;
    if (B > 65535u) return fail(WG_ERR_INVALID, "wg_fill_masks: B above 65535");
    hipEvent_t ev[8];
    if (h->profiling) for (auto &e : ev) { e = take_event(h); h->fill_events.push_back(e); }
    WG_HIP(launch_fill(h->dt, h->vocab->dv, h->dc, d_states, B, d_bitmask, h->n_cu,
                       static_cast<hipStream_t>(stream), h->profiling ? ev : nullptr));
    return WG_OK;
}

int wg_apply_mask(void *d_logits, wg_dtype_t dtype, uint32_t B, uint32_t V, int64_t row_stride_elems,
                  const uint32_t *d_bitmask, void *stream) {
    if (!d_logits || !d_bitmask) return fail(WG_ERR_INVALID, "wg_apply_mask: null argument");
    if (B == 0 || V == 0) return fail(WG_ERR_INVALID, "wg_apply_mask: empty batch or vocabulary");
    if (dtype != WG_F32 && dtype != WG_BF16) return fail(WG_ERR_INVALID, "wg_apply_mask: unknown dtype");
    if (row_stride_elems < (int64_t)V) return fail(WG_ERR_INVALID, "wg_apply_mask: row stride smaller than V");
    if (B > 65535u) return fail(WG_ERR_INVALID, "wg_apply_mask: B above 65535");
    WG_HIP(launch_apply(d_logits, dtype, B, V, row_stride_elems, d_bitmask, static_cast<hipStream_t>(stream)));
    return WG_OK;
}

int wg_masked_argmax(const void *d_logits, wg_dtype_t dtype, uint32_t B, uint32_t V,
                     int64_t row_stride_elems, const uint32_t *d_bitmask, int32_t *d_tokens, void *stream) {
    if (!d_logits || !d_bitmask || !d_tokens) return fail(WG_ERR_INVALID, "wg_masked_argmax: null argument");
    if (B == 0 || V == 0) return fail(WG_ERR_INVALID, "wg_masked_argmax: empty batch or vocabulary");
    if (dtype != WG_F32 && dtype != WG_BF16) return fail(WG_ERR_INVALID, "wg_masked_argmax: unknown dtype");
    if (row_stride_elems < (int64_t)V) return fail(WG_ERR_INVALID, "wg_masked_argmax: row stride smaller than V");
    if (B > 65535u) return fail(WG_ERR_INVALID, "wg_masked_argmax: B above 65535");
    WG_HIP(launch_masked_argmax(d_logits, dtype, B, V, row_stride_elems, d_bitmask, d_tokens,
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

int wg_cache_clear(wg_handle_t h, void *stream) {
    if (!h) return fail(WG_ERR_INVALID, "wg_cache_clear: null handle");
    // The generation number travels with every later launch as a kernel argument, so the
    // clear is ordered with the caller's other calls on this handle without touching the GPU.
    if (++h->dc.epoch == 0) {                          // wrapped: reset the tags for real
        hipStream_t s = static_cast<hipStream_t>(stream);
        WG_HIP(hipMemsetAsync(h->dc.built, 0, (size_t)h->dc.n_keys * sizeof(uint32_t), s));
        WG_HIP(hipMemsetAsync(h->dc.class_built, 0, (size_t)h->dt.n_classes * sizeof(uint32_t), s));
        h->dc.epoch = 1;
    }
    return WG_OK;
}

int wg_cache_stats(wg_handle_t h, wg_cache_stats_t *host_out) {
    if (!h || !host_out) return fail(WG_ERR_INVALID, "wg_cache_stats: null argument");
    Counters c;
    WG_HIP(hipDeviceSynchronize());
    WG_HIP(hipMemcpy(&c, h->dc.ctr, sizeof c, hipMemcpyDeviceToHost));
    host_out->lookups = c.lookups; host_out->hits = c.hits; host_out->builds = c.builds;
    host_out->class_scans = c.class_scans; host_out->entries_walked = c.entries_walked;
    host_out->keys = h->dc.n_keys; host_out->arena_bytes = h->arena_bytes;
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
    for (auto *v : {&h->fill_events, &h->advance_events}) {
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
