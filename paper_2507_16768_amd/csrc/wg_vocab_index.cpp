// The static indexes of a vocabulary and the summaries of class tables: host code without any
// device call, so that it can also be built and checked on its own.
#include <algorithm>
#include <cstring>
#include <new>

#include "wg_internal.h"

namespace wg {

ClassInfo class_info_of(const uint8_t *table) {
    ClassInfo ci{};
    uint32_t n_a = 0, n_b = 0, live = 0;
    unsigned long long nonstay = 0;
    for (uint32_t x = 0; x < 256; x++) {
        const uint8_t c = table[x];
        live += c != CLS_REJECT;
        if (c != CLS_STAY) nonstay |= 1ull << (x & 63u);
        if (c == CLS_EXIT_A) { if (n_a < kMaxExitBytes) ci.a[n_a] = (uint8_t)x; n_a++; }
        if (c == CLS_EXIT_B) { if (n_b < kMaxExitBytes) ci.b[n_b] = (uint8_t)x; n_b++; }
    }
    ci.n_a = n_a > kMaxExitBytes ? kManyExits : (uint8_t)n_a;
    ci.n_b = n_b > kMaxExitBytes ? kManyExits : (uint8_t)n_b;
    // (a byte-less token's signature is all ones: any mask but 0 sends it to the second pass)
    ci.nonstay = nonstay ? nonstay : 1ull << 63;
    ci.scan = live <= 64 ? SCAN_HEAD : __builtin_popcountll(ci.nonstay) <= 8 ? SCAN_SIG : SCAN_CHUNK;
    return ci;
}

namespace {

int build(const uint8_t *host_bytes, const uint64_t *host_offsets, uint32_t V, int32_t eos_id,
          VocabIndex *out, std::string *err) {
    if (!host_offsets || V == 0) { *err = "wg_vocab_create: empty vocabulary"; return WG_ERR_INVALID; }
    if (eos_id >= (int64_t)V) { *err = "wg_vocab_create: eos_id outside the vocabulary"; return WG_ERR_INVALID; }
    uint64_t total = host_offsets[V];
    if (total && !host_bytes) { *err = "wg_vocab_create: host_bytes is null"; return WG_ERR_INVALID; }
    if (total >= 0xFFFFFFFFull) { *err = "wg_vocab_create: more than 4 GiB of token bytes"; return WG_ERR_INVALID; }
    std::vector<uint32_t> off(V + 1);
    uint32_t lmax = 0;
    for (uint32_t t = 0; t <= V; t++) {
        if (t && host_offsets[t] < host_offsets[t - 1])
            { *err = "wg_vocab_create: offsets are not non-decreasing"; return WG_ERR_INVALID; }
        off[t] = (uint32_t)host_offsets[t];
        if (t && off[t] - off[t - 1] > lmax) lmax = off[t] - off[t - 1];
    }
    if (host_offsets[0] != 0) { *err = "wg_vocab_create: offsets must start at 0"; return WG_ERR_INVALID; }
    if (lmax > 248) { *err = "wg_vocab_create: tokens longer than 248 bytes are not supported"; return WG_ERR_INVALID; }
    const uint32_t W = (V + 31u) / 32u, rs = (W + 3u) & ~3u;
    const uint32_t n_chunks = (lmax + 7u) / 8u;
    // Static indexes of the vocabulary (they depend on the token bytes only):
    //  - 8 bytes of padding so kernels may over-read a token's tail
    //  - len8 / chunks: fixed-stride view, 8 bytes per load, for the class scan
    //  - first-byte buckets (per token range): the only tokens a literal state can admit
    //  - per-length rows: tokens with 1 <= length <= r, for Waits with a byte budget
    std::vector<uint8_t> bytes(total + 8, 0), len8(V, 0);
    if (total) std::memcpy(bytes.data(), host_bytes, total);
    std::vector<uint64_t> chunks((size_t)(n_chunks ? n_chunks : 1) * V, 0);
    std::vector<uint32_t> lit_start(256 * kParts + 1, 0), len_rows((size_t)(lmax + 2) * rs, 0);
    // the token ranges that can split the work of one mask row
    uint32_t part_tok[kParts + 1];
    const uint32_t n_groups = (V + kPartGroup - 1u) / kPartGroup;
    for (uint32_t p = 0; p <= kParts; p++) {
        const uint64_t t0 = ((uint64_t)p * n_groups / kParts) * kPartGroup;
        part_tok[p] = (p == kParts || t0 > V) ? V : (uint32_t)t0;
    }
    auto part_of = [&](uint32_t t) {
        uint32_t p = 0;
        while (p + 1 < kParts && t >= part_tok[p + 1]) p++;
        return p;
    };
    //  - sig / first8: one AND, or one table look-up, decides most tokens in the class scan
    std::vector<uint64_t> sig(V, ~0ull);
    std::vector<uint8_t> first8(V, 0);
    for (uint32_t t = 0; t < V; t++) {
        uint32_t L = ((int64_t)t == eos_id) ? 0u : off[t + 1] - off[t];
        len8[t] = (uint8_t)L;
        if (L) {
            uint64_t m = 0;
            for (uint32_t i = 0; i < L; i++) m |= 1ull << (bytes[off[t] + i] & 63u);
            sig[t] = m;
            first8[t] = bytes[off[t]];
        }
        for (uint32_t i = 0; i < L; i++)
            chunks[(size_t)(i / 8u) * V + t] |= (uint64_t)bytes[off[t] + i] << (8u * (i % 8u));
        if (L) {
            lit_start[bytes[off[t]] * kParts + part_of(t) + 1u]++;
            for (uint32_t r = L; r <= lmax + 1u; r++) len_rows[(size_t)r * rs + (t >> 5)] |= 1u << (t & 31u);
        }
    }
    for (uint32_t y = 0; y < 256 * kParts; y++) lit_start[y + 1] += lit_start[y];
    // Within a bucket the entries are ordered by remaining length, so that the lanes of a
    // wavefront walk remainders of similar length.
    std::vector<ExitEntry> lit_entries(lit_start[256 * kParts] ? lit_start[256 * kParts] : 1);
    {
        std::vector<uint32_t> order;
        order.reserve(V);
        for (uint32_t t = 0; t < V; t++) if (len8[t]) order.push_back(t);
        std::stable_sort(order.begin(), order.end(), [&](uint32_t a, uint32_t b) {
            const uint32_t fa = bytes[off[a]] * kParts + part_of(a), fb = bytes[off[b]] * kParts + part_of(b);
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
    // The vocabulary in byte order (the prefix-indexed view of it): a literal state admits the
    // tokens that are prefixes of the bytes still to be written and the tokens that go on
    // after them, and both lie in the range of tokens sharing the literal's first two bytes.
    std::vector<ExitEntry> sorted;
    std::vector<uint32_t> dir0(256 * 257 + 1, 0);
    {
        std::vector<uint32_t> order;
        order.reserve(V);
        for (uint32_t t = 0; t < V; t++) if (len8[t]) order.push_back(t);
        std::sort(order.begin(), order.end(), [&](uint32_t a, uint32_t b) {
            const uint32_t la = len8[a], lb = len8[b];
            const int c = std::memcmp(bytes.data() + off[a], bytes.data() + off[b], la < lb ? la : lb);
            return c != 0 ? c < 0 : la != lb ? la < lb : a < b;
        });
        sorted.resize(order.size() ? order.size() : 1);
        auto range_of = [&](uint32_t t) {
            return (uint32_t)bytes[off[t]] * 257u + (len8[t] > 1 ? 1u + bytes[off[t] + 1] : 0u);
        };
        for (size_t i = 0; i < order.size(); i++) {
            const uint32_t t = order[i];
            ExitEntry e;
            e.tok = t; e.off = 0; e.cls = 0; e.first = len8[t] > 1 ? bytes[off[t] + 1] : 0; e.rem = len8[t];
            sorted[i] = e;
            dir0[range_of(t) + 1u]++;
        }
        for (uint32_t y = 0; y < 256 * 257; y++) dir0[y + 1] += dir0[y];
    }
    // Every byte pair inside a token, grouped by the pair: a checkpoint whose exit byte e leads to
    // a literal byte y can only be left early by tokens in which y follows e.
    std::vector<uint32_t> dirN(65536 + 1, 0);
    for (uint32_t t = 0; t < V; t++)
        for (uint32_t i = 1; i < len8[t]; i++) dirN[((uint32_t)bytes[off[t] + i - 1] << 8 | bytes[off[t] + i]) + 1u]++;
    for (uint32_t y = 0; y < 65536; y++) dirN[y + 1] += dirN[y];
    std::vector<ExitEntry> bigram(dirN[65536] ? dirN[65536] : 1);
    {
        std::vector<uint32_t> at(dirN.begin(), dirN.end() - 1);
        for (uint32_t t = 0; t < V; t++)
            for (uint32_t i = 1; i < len8[t]; i++) {
                ExitEntry e;
                e.tok = t; e.off = (uint8_t)i; e.cls = 0; e.first = bytes[off[t] + i]; e.rem = (uint8_t)(len8[t] - i);
                bigram[at[(uint32_t)bytes[off[t] + i - 1] << 8 | bytes[off[t] + i]]++] = e;
            }
    }
    // The vocabulary by byte value, as rows of tokens (which tokens contain the byte x, which start
    // with it): a class table's first look at 32 tokens is then the OR of a few words.
    std::vector<uint32_t> byte_rows((size_t)512 * rs, 0);
    for (uint32_t t = 0; t < V; t++) {
        for (uint32_t i = 0; i < len8[t]; i++) byte_rows[(size_t)bytes[off[t] + i] * rs + (t >> 5)] |= 1u << (t & 31u);
        if (len8[t]) byte_rows[(size_t)(256u + first8[t]) * rs + (t >> 5)] |= 1u << (t & 31u);
    }
    VocabIndex &ix = *out;
    ix.V = V; ix.W = W; ix.row_stride = rs; ix.lmax = lmax; ix.n_chunks = n_chunks;
    for (uint32_t p = 0; p <= kParts; p++) ix.part_tok[p] = part_tok[p];
    ix.bytes.swap(bytes); ix.offsets.swap(off); ix.len8.swap(len8); ix.first8.swap(first8);
    ix.chunks.swap(chunks); ix.sig.swap(sig); ix.lit_entries.swap(lit_entries); ix.lit_start.swap(lit_start);
    ix.len_rows.swap(len_rows); ix.sorted.swap(sorted); ix.dir0.swap(dir0); ix.bigram.swap(bigram);
    ix.dirN.swap(dirN); ix.byte_rows.swap(byte_rows);
    return WG_OK;
}

}  // namespace

int build_vocab_index(const uint8_t *host_bytes, const uint64_t *host_offsets, uint32_t V, int32_t eos_id,
                      VocabIndex *out, std::string *err) {
    try {
        return build(host_bytes, host_offsets, V, eos_id, out, err);
    } catch (const std::bad_alloc &) {
        *err = "wg_vocab_create: out of host memory";
        return WG_ERR_NOMEM;
    }
}

}  // namespace wg
