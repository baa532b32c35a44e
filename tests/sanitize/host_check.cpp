// Sanitizer driver for the host code (test infrastructure): runs the library's operator
// compiler and regular-expression translator, and the C oracle, over a case file, all built with
// -fsanitize=address,undefined, and checks that the two compilers agree on the state count.
// Case file, one record per line, fields separated by a space, byte strings in hex ("-" = empty):
//   V <bytes> <off0,off1,...> <eos_id>     vocabulary for the oracle's masks
//   C <flags> <lmax>                       start a case
//   T <text>                               a template of the case
//   A <name> <bytes>                       an argument of the last template
//   G                                      compile what was collected (one add / one compile)
//   R <regex>                              translate, then compile the result in both
#include <cstdint>
#include <cstdio>
#include <cstdlib>
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
    const size_t before = low.table.states.size();
    bool lib_ok = true;
    try { low.add(texts.data(), a.data(), n); } catch (const std::exception &) { lib_ok = false; }
    char err[256];
    wgo_handle *h = wgo_compile(texts.data(), oa.data(), n, flags, err, sizeof err);
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
