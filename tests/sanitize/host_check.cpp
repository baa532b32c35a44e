// Sanitizer driver for the host code (test infrastructure): runs the library's operator
// compiler and regular-expression translator, and the C oracle, over a case file, all built with
// -fsanitize=address,undefined, and checks that the two compilers agree on the state count.
// The library's vocabulary indexes and class-table summaries are built under the same sanitizers.
// Case file, one record per line, fields separated by a space, byte strings in hex ("-" = empty):
//   V <bytes> <off0,off1,...> <eos_id>     vocabulary for the oracle's masks
//   C <flags> <lmax>                       start a case
//   T <text>                               a template of the case
//   A <name> <bytes>                       an argument of the last template
//   G                                      compile what was collected (one add / one compile)
//   R <regex>                              translate, then compile the result in both
//   I                                      build the static indexes of the last vocabulary and check each
//                                          against its definition, recounted here token by token
// After every compile the summary of each new class table is checked against the table itself.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <algorithm>
#include <set>
#include <fstream>
#include <iostream>
#include <memory>
#include <sstream>
#include <string>
#include <vector>

#include "../../paper_2507_16768_amd/csrc/wg_internal.h"

extern "C" {
typedef struct wgo_handle wgo_handle;
typedef struct { uint32_t n; const char *const *names; const uint8_t *const *data; const uint64_t *lens; } wgo_args;
typedef struct { const uint8_t *bytes; const uint64_t *offsets; uint32_t V; int32_t eos_id; } wgo_vocab;
wgo_handle *wgo_compile(const char *const *texts, const wgo_args *args, uint32_t n, uint32_t flags,
                        char *err, uint64_t errlen);
void wgo_destroy(wgo_handle *h);
uint32_t wgo_num_states(const wgo_handle *h);
uint32_t wgo_start_state(const wgo_handle *h, uint32_t t);
void wgo_fill_masks(const wgo_handle *h, const wgo_vocab *v, const uint32_t *states, uint32_t B, uint32_t *out);
void wgo_advance(const wgo_handle *h, const wgo_vocab *v, uint32_t *states, const int32_t *tokens, uint32_t B);
}

namespace wg { void set_last_error(const std::string &) {} }

static std::string unhex(const std::string &h) {
    if (h == "-") return std::string();
    std::string out;
    for (size_t i = 0; i + 1 < h.size(); i += 2) out.push_back((char)std::stoi(h.substr(i, 2), nullptr, 16));
    return out;
}

struct Pending {
    std::vector<std::string> texts;
    std::vector<std::vector<std::pair<std::string, std::string>>> args;
};

static int failures = 0;


#define EXPECT(cond, ...) do { if (!(cond)) { std::printf("INDEX "); std::printf(__VA_ARGS__); std::printf("\n"); failures++; return; } } while (0)

// The indexes of a vocabulary, each recounted from the token bytes by its definition.
static void check_index(const uint8_t *vb, const uint64_t *off, uint32_t V, int32_t eos) {
    using namespace wg;
    VocabIndex ix;
    std::string err;
    const int rc = build_vocab_index(vb, off, V, eos, &ix, &err);
    EXPECT(rc == WG_OK, "build failed: %s", err.c_str());
    auto len = [&](uint32_t t) { return (int64_t)t == eos ? 0u : (uint32_t)(off[t + 1] - off[t]); };
    auto byte_at = [&](uint32_t t, uint32_t i) { return vb[off[t] + i]; };
    uint32_t lmax = 0, with_bytes = 0;
    uint64_t pairs = 0;
    for (uint32_t t = 0; t < V; t++) {
        lmax = std::max<uint32_t>(lmax, (uint32_t)(off[t + 1] - off[t]));
        with_bytes += len(t) > 0;
        pairs += len(t) > 1 ? len(t) - 1 : 0;
    }
    EXPECT(ix.V == V && ix.W == (V + 31) / 32 && ix.row_stride % 4 == 0 && ix.row_stride >= ix.W && ix.row_stride < ix.W + 4,
           "row geometry");
    EXPECT(ix.lmax == lmax && ix.n_chunks == (lmax + 7) / 8, "lmax %u %u", ix.lmax, lmax);
    // token ranges: whole 2048-token groups, in order, covering [0, V)
    EXPECT(ix.part_tok[0] == 0 && ix.part_tok[kParts] == V, "range ends");
    for (uint32_t p = 0; p < kParts; p++)
        EXPECT(ix.part_tok[p] <= ix.part_tok[p + 1] && (ix.part_tok[p] % kPartGroup == 0 || ix.part_tok[p] == V), "range %u", p);
    auto part_of = [&](uint32_t t) { uint32_t p = 0; while (!(ix.part_tok[p] <= t && t < ix.part_tok[p + 1])) p++; return p; };
    // per-token views
    EXPECT(ix.bytes.size() == off[V] + 8 && ix.offsets.size() == V + 1 && ix.len8.size() == V && ix.first8.size() == V &&
           ix.sig.size() == V && ix.chunks.size() == (size_t)std::max(1u, ix.n_chunks) * V, "array sizes");
    for (size_t i = 0; i < ix.bytes.size(); i++) EXPECT(ix.bytes[i] == (i < off[V] ? vb[i] : 0), "bytes %zu", i);
    for (uint32_t t = 0; t < V; t++) {
        const uint32_t L = len(t);
        EXPECT(ix.offsets[t] == off[t] && ix.len8[t] == L && ix.first8[t] == (L ? byte_at(t, 0) : 0), "token %u", t);
        uint64_t m = 0;
        for (uint32_t i = 0; i < L; i++) m |= 1ull << (byte_at(t, i) % 64);
        EXPECT(ix.sig[t] == (L ? m : ~0ull), "sig %u", t);
        for (uint32_t k = 0; k < ix.n_chunks; k++)
            for (uint32_t j = 0; j < 8; j++) {
                const uint8_t want = 8 * k + j < L ? byte_at(t, 8 * k + j) : 0;
                EXPECT((uint8_t)(ix.chunks[(size_t)k * V + t] >> (8 * j)) == want, "chunk %u %u %u", t, k, j);
            }
    }
    EXPECT(ix.offsets[V] == off[V], "last offset");
    // rows of tokens no longer than r
    EXPECT(ix.len_rows.size() == (size_t)(lmax + 2) * ix.row_stride, "len_rows size");
    for (uint32_t r = 0; r <= lmax + 1; r++)
        for (uint32_t w = 0; w < ix.row_stride; w++) {
            uint32_t want = 0;
            for (uint32_t b = 0; b < 32 && 32 * w + b < V; b++) { const uint32_t L = len(32 * w + b); if (L >= 1 && L <= r) want |= 1u << b; }
            EXPECT(ix.len_rows[(size_t)r * ix.row_stride + w] == want, "len_rows %u %u", r, w);
        }
    // first-byte buckets per range
    EXPECT(ix.lit_start.size() == 256 * kParts + 1 && ix.lit_start[0] == 0 && ix.lit_start.back() == with_bytes &&
           ix.lit_entries.size() == std::max(1u, with_bytes), "lit sizes");
    {
        std::vector<uint8_t> seen(V, 0);
        for (uint32_t y = 0; y < 256 * kParts; y++) {
            EXPECT(ix.lit_start[y] <= ix.lit_start[y + 1], "lit_start %u", y);
            for (uint32_t i = ix.lit_start[y]; i < ix.lit_start[y + 1]; i++) {
                const ExitEntry e = ix.lit_entries[i];
                EXPECT(e.tok < V && !seen[e.tok] && len(e.tok) >= 1, "lit entry %u", i);
                seen[e.tok] = 1;
                const uint32_t L = len(e.tok);
                EXPECT(byte_at(e.tok, 0) == y / kParts && part_of(e.tok) == y % kParts, "lit bucket of %u", e.tok);
                EXPECT(e.off == 1 && e.cls == CLS_EXIT_A && e.rem == L - 1 && e.first == (L > 1 ? byte_at(e.tok, 1) : 0), "lit fields %u", i);
                EXPECT(i == ix.lit_start[y] || ix.lit_entries[i - 1].rem <= e.rem, "lit order %u", i);
            }
        }
    }
    // the vocabulary in byte order and its prefix ranges
    EXPECT(ix.dir0.size() == 256 * 257 + 1 && ix.dir0[0] == 0 && ix.dir0.back() == with_bytes &&
           ix.sorted.size() == std::max(1u, with_bytes), "sorted sizes");
    {
        std::vector<uint8_t> seen(V, 0);
        for (uint32_t y = 0; y < 256 * 257; y++) {
            EXPECT(ix.dir0[y] <= ix.dir0[y + 1], "dir0 %u", y);
            for (uint32_t i = ix.dir0[y]; i < ix.dir0[y + 1]; i++) {
                const ExitEntry e = ix.sorted[i];
                EXPECT(e.tok < V && !seen[e.tok] && len(e.tok) >= 1, "sorted entry %u", i);
                seen[e.tok] = 1;
                const uint32_t L = len(e.tok);
                EXPECT(byte_at(e.tok, 0) == y / 257 && (y % 257 == 0 ? L == 1 : L >= 2 && byte_at(e.tok, 1) == y % 257 - 1), "range of %u", e.tok);
                EXPECT(e.off == 0 && e.cls == 0 && e.rem == L && e.first == (L > 1 ? byte_at(e.tok, 1) : 0), "sorted fields %u", i);
                if (i) {
                    const uint32_t p = ix.sorted[i - 1].tok, Lp = len(p);
                    const int c = std::memcmp(vb + off[p], vb + off[e.tok], std::min(Lp, L));
                    EXPECT(c < 0 || (c == 0 && (Lp < L || (Lp == L && p < e.tok))), "byte order at %u", i);
                }
            }
        }
    }
    // byte pairs inside tokens
    EXPECT(ix.dirN.size() == 65537 && ix.dirN[0] == 0 && ix.dirN.back() == pairs && ix.bigram.size() == std::max<uint64_t>(1, pairs),
           "pair sizes");
    {
        std::set<std::pair<uint32_t, uint32_t>> seen;
        for (uint32_t y = 0; y < 65536; y++) {
            EXPECT(ix.dirN[y] <= ix.dirN[y + 1], "dirN %u", y);
            for (uint32_t i = ix.dirN[y]; i < ix.dirN[y + 1]; i++) {
                const ExitEntry e = ix.bigram[i];
                EXPECT(e.tok < V && e.off >= 1 && e.off < len(e.tok), "pair entry %u", i);
                EXPECT(seen.insert({e.tok, e.off}).second, "pair twice %u", i);
                EXPECT(byte_at(e.tok, e.off - 1u) == y >> 8 && byte_at(e.tok, e.off) == (y & 255), "pair range %u", i);
                EXPECT(e.cls == 0 && e.first == (y & 255) && e.rem == len(e.tok) - e.off, "pair fields %u", i);
            }
        }
    }
    // the vocabulary by byte value as token rows: tokens that contain the byte, tokens that start with it
    EXPECT(ix.byte_rows.size() == (size_t)512 * ix.row_stride, "byte rows size");
    {
        std::vector<uint32_t> want((size_t)512 * ix.row_stride, 0);
        for (uint32_t t = 0; t < V; t++)
            for (uint32_t i = 0; i < len(t); i++) {
                want[(size_t)byte_at(t, i) * ix.row_stride + t / 32] |= 1u << (t % 32);
                if (i == 0) want[(size_t)(256 + byte_at(t, 0)) * ix.row_stride + t / 32] |= 1u << (t % 32);
            }
        for (size_t i = 0; i < want.size(); i++) EXPECT(ix.byte_rows[i] == want[i], "byte row %zu word %zu", i / ix.row_stride, i % ix.row_stride);
    }
    std::printf("index ok %u %u %llu\n", V, with_bytes, (unsigned long long)pairs);
}

// The summaries of the class tables from `first` on, each against its 256 bytes.
static void check_class_info(const wg::Table &t, size_t first) {
    using namespace wg;
    for (size_t c = first; c < t.classes.size() / 256; c++) {
        const uint8_t *tab = t.classes.data() + c * 256;
        const ClassInfo ci = class_info_of(tab);
        uint32_t cnt[4] = {0, 0, 0, 0};
        unsigned long long fold = 0;
        for (uint32_t x = 0; x < 256; x++) {
            EXPECT(tab[x] < 4, "class byte");
            cnt[tab[x]]++;
            if (tab[x] != CLS_STAY) fold |= 1ull << (x % 64);
        }
        EXPECT(ci.nonstay != 0 && (fold ? ci.nonstay == fold : true), "nonstay of %zu", c);
        EXPECT(ci.scan == SCAN_CHUNK || ci.scan == SCAN_SIG || ci.scan == SCAN_HEAD, "scan of %zu", c);
        const uint8_t n[2] = {ci.n_a, ci.n_b};
        const uint8_t *lists[2] = {ci.a, ci.b};
        for (int side = 0; side < 2; side++) {
            const uint32_t have = cnt[side ? CLS_EXIT_B : CLS_EXIT_A];
            EXPECT(n[side] == (have > kMaxExitBytes ? kManyExits : have), "exit count of %zu", c);
            if (n[side] == kManyExits) continue;
            for (uint32_t i = 0; i < n[side]; i++) {
                EXPECT(tab[lists[side][i]] == (side ? CLS_EXIT_B : CLS_EXIT_A), "exit byte of %zu", c);
                EXPECT(i == 0 || lists[side][i - 1] < lists[side][i], "exit order of %zu", c);
            }
        }
    }
}

static void compile_both(wg::Lowering &low, const Pending &p, uint32_t flags, const wgo_vocab *voc) {
    const uint32_t n = (uint32_t)p.texts.size();
    std::vector<const char *> texts(n);
    std::vector<std::vector<const char *>> names(n);
    std::vector<std::vector<const uint8_t *>> data(n);
    std::vector<std::vector<uint64_t>> lens(n);
    std::vector<wg_args_t> a(n);
    std::vector<wgo_args> oa(n);
    for (uint32_t i = 0; i < n; i++) {
        texts[i] = p.texts[i].c_str();
        for (auto &kv : p.args[i]) {
            names[i].push_back(kv.first.c_str());
            data[i].push_back(reinterpret_cast<const uint8_t *>(kv.second.data()));
            lens[i].push_back(kv.second.size());
        }
        a[i] = wg_args_t{(uint32_t)names[i].size(), names[i].data(), data[i].data(), lens[i].data()};
        oa[i] = wgo_args{(uint32_t)names[i].size(), names[i].data(), data[i].data(), lens[i].data()};
    }
    const size_t before = low.table.states.size(), classes_before = low.table.classes.size() / 256;
    bool lib_ok = true;
    try { low.add(texts.data(), a.data(), n); } catch (const std::exception &) { lib_ok = false; }
    check_class_info(low.table, lib_ok ? classes_before : 0);
    char err[256];
    wgo_handle *h = wgo_compile(texts.data(), oa.data(), n, flags & 1u, err, sizeof err);   // (bit 1 is the library's alone: shared keys)
    if (lib_ok != (h != nullptr)) { std::printf("MISMATCH accept %d %d: %s\n", (int)lib_ok, h != nullptr, texts[0]); failures++; }
    if (lib_ok && h) {
        // the library table may hold earlier cases too: compare what this add appended
        const size_t added = low.table.states.size() - before;
        if (added != wgo_num_states(h) - 1u) { std::printf("MISMATCH states %zu %u\n", added, wgo_num_states(h) - 1u); failures++; }
        if (voc) {
            const uint32_t ns = wgo_num_states(h), W = (voc->V + 31u) / 32u;
            std::vector<uint32_t> st(2 * (size_t)ns), rows((size_t)ns * W);
            for (uint32_t s = 0; s < ns; s++) { st[2 * s] = s; st[2 * s + 1] = s % 3u; }
            wgo_fill_masks(h, voc, st.data(), ns, rows.data());
            std::vector<int32_t> tok(ns);
            for (uint32_t s = 0; s < ns; s++) tok[s] = (int32_t)((s * 7u) % (voc->V + 2u)) - 1;   // also -1 and V
            wgo_advance(h, voc, st.data(), tok.data(), ns);
        }
    } else if (!lib_ok && low.table.states.size() != before) { std::printf("MISMATCH rollback\n"); failures++; }
    std::printf("%s %zu\n", lib_ok ? "ok" : "err", low.table.states.size());
    wgo_destroy(h);
}

int main(int argc, char **argv) {
    if (argc != 2) return 2;
    std::ifstream in(argv[1]);
    std::string line, vb;
    std::vector<uint64_t> voff;
    wgo_vocab voc{}; bool have_voc = false;
    std::unique_ptr<wg::Lowering> low;
    uint32_t flags = 0;
    Pending pend;
    while (std::getline(in, line)) {
        std::istringstream ss(line);
        std::string tag; ss >> tag;
        if (tag == "V") {
            std::string hb, offs; int eos; ss >> hb >> offs >> eos;
            vb = unhex(hb); voff.clear();
            std::istringstream os(offs); std::string x;
            while (std::getline(os, x, ',')) voff.push_back(std::stoull(x));
            voc = wgo_vocab{reinterpret_cast<const uint8_t *>(vb.data()), voff.data(), (uint32_t)voff.size() - 1u, eos};
            have_voc = true;
        } else if (tag == "I") {
            if (have_voc) check_index(voc.bytes, voc.offsets, voc.V, voc.eos_id);
        } else if (tag == "C") {
            uint32_t lmax; ss >> flags >> lmax;
            low.reset(new wg::Lowering(flags, lmax));
            pend = Pending{};
        } else if (tag == "T") {
            std::string h; ss >> h;
            pend.texts.push_back(unhex(h)); pend.args.emplace_back();
        } else if (tag == "A") {
            std::string name, h; ss >> name >> h;
            pend.args.back().emplace_back(name, unhex(h));
        } else if (tag == "G") {
            compile_both(*low, pend, flags, have_voc ? &voc : nullptr);
            pend = Pending{};
        } else if (tag == "R") {
            std::string h; ss >> h;
            const std::string rx = unhex(h);
            try {
                Pending p; p.texts.push_back(wg::regex_to_template(rx.c_str())); p.args.emplace_back();
                wg::Lowering l2(0, 8);
                compile_both(l2, p, 0, have_voc ? &voc : nullptr);
            } catch (const std::exception &) { std::printf("rxerr\n"); }
        }
    }
    std::printf("failures %d\n", failures);
    return failures ? 1 : 0;
}
