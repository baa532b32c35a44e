/*
 * Plain-C client of the C ABI.  TEST INFRASTRUCTURE: it links the HIP library and the C oracle
 * into one program and compares them call by call, with no Python and no torch in between --
 * memory from hipMalloc, a stream of its own, the calls exactly as include/wg.h declares them.
 *
 *   two template instances (tags around a free-text Wait with runtime arguments; a DoWhile of
 *   IfElse objects), 64 requests, a vocabulary of every string of up to three bytes over a
 *   14-byte alphabet.  Phase 1: wg_fill_masks, wg_apply_mask, wg_masked_argmax, wg_masked_topk,
 *   wg_advance on every step.  Phase 2: wg_decode_step on every step, cache cleared now and then.
 *
 * Exit status 0 and a last line "c_client ok" when everything matched; 77 when no GPU is there.
 */
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "wg.h"

/* the oracle's interface (oracle/wg_oracle.c) */
typedef struct wgo_handle wgo_handle;
typedef struct { uint32_t n; const char *const *names; const uint8_t *const *data; const uint64_t *lens; } wgo_args;
typedef struct { const uint8_t *bytes; const uint64_t *offsets; uint32_t V; int32_t eos_id; } wgo_vocab;
wgo_handle *wgo_compile(const char *const *texts, const wgo_args *args, uint32_t n, uint32_t flags,
                        char *err, uint64_t errlen);
void wgo_destroy(wgo_handle *h);
uint32_t wgo_start_state(const wgo_handle *h, uint32_t t);
void wgo_fill_masks(const wgo_handle *h, const wgo_vocab *v, const uint32_t *states, uint32_t B, uint32_t *out);
void wgo_apply_mask(void *logits, int dtype, uint32_t B, uint32_t V, int64_t row_stride, const uint32_t *bitmask);
void wgo_masked_argmax(const void *logits, int dtype, uint32_t B, uint32_t V, int64_t row_stride,
                       const uint32_t *bitmask, int32_t *tokens_out);
void wgo_masked_topk(const void *logits, int dtype, uint32_t B, uint32_t V, int64_t row_stride,
                     const uint32_t *bitmask, uint32_t k, int32_t *ids_out, void *values_out);
void wgo_advance(const wgo_handle *h, const wgo_vocab *v, uint32_t *states, const int32_t *tokens, uint32_t B);
int64_t wgo_select_bit(const uint32_t *row, uint32_t W, uint64_t k);

#define HIP(call) do { hipError_t e_ = (call); if (e_ != hipSuccess) { \
    fprintf(stderr, "%s: %s\n", #call, hipGetErrorString(e_)); return 1; } } while (0)
#define WG(call) do { int rc_ = (call); if (rc_ != WG_OK) { \
    fprintf(stderr, "%s: %d %s\n", #call, rc_, wg_last_error()); return 1; } } while (0)
#define CHECK(cond, ...) do { if (!(cond)) { fprintf(stderr, __VA_ARGS__); fprintf(stderr, "\n"); return 1; } } while (0)

static const char kTags[] =
    "Sequence(\n  Write($open),\n  Wait(denies={}, wait={\\x3C}, max=12),\n  Write($close))";
static const char kObjects[] =
    "Sequence(\n  Write(\"[\"),\n  DoWhile(\n    body=\n      Sequence(\n        Write($key),\n        IfElse(\n"
    "          condition=\n            Wait(allow={\\x20}, true_waits={\\x5B}, false_waits={\\x22}),\n"
    "          if_body=\n            Wait(allow=$idx, wait={\\x5D}),\n"
    "          else_body=\n            Wait(denies={}, wait={\\x22}, max=9)),\n        Write(\"}\")),\n"
    "    condition=\n      Wait(allow={\\x20}, true_waits={\\x2C}, false_waits={\\x5D})))";

static uint64_t lcg(uint64_t *s) { *s = *s * 6364136223846793005ull + 1442695040888963407ull; return *s >> 17; }

int main(void)
{
    int n_dev = 0;
    if (hipGetDeviceCount(&n_dev) != hipSuccess || n_dev == 0) { printf("c_client: no GPU\n"); return 77; }
    HIP(hipSetDevice(0));

    /* vocabulary: token 0 is EOS, then every string of 1..3 bytes over the alphabet */
    static const uint8_t alpha[] = "ab<>/[]{}\", 01";
    const uint32_t A = 14, V = 1 + A + A * A + A * A * A;
    uint8_t *bytes = (uint8_t *)malloc(3u * V);
    uint64_t *offsets = (uint64_t *)malloc((V + 1) * sizeof *offsets);
    uint32_t t = 0; uint64_t at = 0;
    offsets[t++] = 0;                                           /* EOS: no bytes */
    for (uint32_t len = 1; len <= 3; len++) {
        uint32_t count = len == 1 ? A : len == 2 ? A * A : A * A * A;
        for (uint32_t i = 0; i < count; i++) {
            offsets[t++] = at;
            uint32_t x = i;
            for (uint32_t j = 0; j < len; j++) { bytes[at++] = alpha[x % A]; x /= A; }
        }
    }
    offsets[t] = at;
    CHECK(t == V, "vocabulary size");
    const uint32_t W = (V + 31u) / 32u;

    /* two instances with runtime arguments */
    const char *texts[2] = {kTags, kObjects};
    const char *names0[2] = {"open", "close"}, *names1[2] = {"key", "idx"};
    const uint8_t *data0[2] = {(const uint8_t *)"<a b>", (const uint8_t *)"/a>"};
    const uint8_t *data1[2] = {(const uint8_t *)"{\"ab\"", (const uint8_t *)"01,"};
    const uint64_t lens0[2] = {5, 3}, lens1[2] = {5, 3};
    wg_args_t args[2] = {{2, names0, data0, lens0}, {2, names1, data1, lens1}};
    wgo_args oargs[2] = {{2, names0, data0, lens0}, {2, names1, data1, lens1}};

    char err[512];
    wgo_vocab ov = {bytes, offsets, V, 0};
    wgo_handle *o = wgo_compile(texts, oargs, 2, 1u, err, sizeof err);
    CHECK(o != NULL, "oracle: %s", err);

    wg_vocab_t vocab = NULL; wg_handle_t h = NULL; wg_state_t start[2];
    WG(wg_vocab_create(bytes, offsets, V, 0, &vocab));
    WG(wg_compile(texts, args, 2, vocab, WG_EOS_RESTART, &h, start));
    CHECK(wg_mask_words(h) == W, "mask words");
    for (uint32_t i = 0; i < 2; i++)
        CHECK(start[i].sid == wgo_start_state(o, i) && start[i].aux == 0, "start state of instance %u", i);

    enum { B = 64, K = 5, STEPS = 40 };
    hipStream_t stream;
    HIP(hipStreamCreate(&stream));
    uint32_t *states = (uint32_t *)malloc(B * 2 * sizeof *states);            /* the oracle's */
    for (uint32_t b = 0; b < B; b++) { states[2 * b] = start[b & 1].sid; states[2 * b + 1] = 0; }
    uint32_t *want_mask = (uint32_t *)malloc((size_t)B * W * 4), *got_mask = (uint32_t *)malloc((size_t)B * W * 4);
    float *logits = (float *)malloc((size_t)B * V * 4), *want_logits = (float *)malloc((size_t)B * V * 4);
    int32_t tokens[B], want_tok[B], got_tok[B], want_ids[B * K], got_ids[B * K];
    float want_vals[B * K], got_vals[B * K];
    uint32_t got_states[B * 2];

    wg_state_t *d_states; uint32_t *d_mask; float *d_logits; int32_t *d_tokens, *d_pick, *d_ids; float *d_vals; void *d_work;
    const uint64_t work_bytes = wg_masked_topk_workspace(B, V, K);
    HIP(hipMalloc((void **)&d_states, B * sizeof *d_states));
    HIP(hipMalloc((void **)&d_mask, (size_t)B * W * 4));
    HIP(hipMalloc((void **)&d_logits, (size_t)B * V * 4));
    HIP(hipMalloc((void **)&d_tokens, B * 4));
    HIP(hipMalloc((void **)&d_pick, B * 4));
    HIP(hipMalloc((void **)&d_ids, B * K * 4));
    HIP(hipMalloc((void **)&d_vals, B * K * 4));
    HIP(hipMalloc(&d_work, work_bytes));
    HIP(hipMemcpy(d_states, states, B * 8, hipMemcpyHostToDevice));

    uint64_t seed = 20250716u;
    for (int phase = 0; phase < 2; phase++) {
        for (int step = 0; step < STEPS; step++) {
            for (size_t i = 0; i < (size_t)B * V; i++)
                logits[i] = (float)((int64_t)(lcg(&seed) % 4001u) - 2000) / 64.0f;   /* many ties */
            wgo_fill_masks(o, &ov, states, B, want_mask);
            HIP(hipMemcpyAsync(d_logits, logits, (size_t)B * V * 4, hipMemcpyHostToDevice, stream));
            if (phase == 0) {
                WG(wg_fill_masks(h, d_states, B, d_mask, stream));
                WG(wg_masked_argmax(d_logits, WG_F32, B, V, V, d_mask, d_pick, stream));
                WG(wg_masked_topk(d_logits, WG_F32, B, V, V, d_mask, K, d_ids, d_vals, d_work, work_bytes, stream));
                WG(wg_apply_mask(d_logits, WG_F32, B, V, V, d_mask, stream));
            } else {
                if (step % 7 == 3) WG(wg_cache_clear(h, stream));
                WG(wg_decode_step(h, d_states, step == 0 ? NULL : d_tokens, B, d_mask, d_logits, WG_F32, V, stream));
                HIP(hipMemcpyAsync(got_states, d_states, B * 8, hipMemcpyDeviceToHost, stream));
            }
            HIP(hipMemcpyAsync(got_mask, d_mask, (size_t)B * W * 4, hipMemcpyDeviceToHost, stream));
            HIP(hipMemcpyAsync(want_logits, d_logits, (size_t)B * V * 4, hipMemcpyDeviceToHost, stream));
            HIP(hipStreamSynchronize(stream));
            CHECK(memcmp(got_mask, want_mask, (size_t)B * W * 4) == 0, "phase %d step %d: masks differ", phase, step);
            if (phase == 1)
                CHECK(memcmp(got_states, states, B * 8) == 0, "phase 1 step %d: states differ", step);
            if (phase == 0) {
                wgo_masked_argmax(logits, 0, B, V, V, want_mask, want_tok);
                wgo_masked_topk(logits, 0, B, V, V, want_mask, K, want_ids, want_vals);
                HIP(hipMemcpy(got_tok, d_pick, B * 4, hipMemcpyDeviceToHost));
                HIP(hipMemcpy(got_ids, d_ids, B * K * 4, hipMemcpyDeviceToHost));
                HIP(hipMemcpy(got_vals, d_vals, B * K * 4, hipMemcpyDeviceToHost));
                CHECK(memcmp(got_tok, want_tok, B * 4) == 0, "step %d: greedy tokens differ", step);
                CHECK(memcmp(got_ids, want_ids, B * K * 4) == 0, "step %d: top-k ids differ", step);
                CHECK(memcmp(got_vals, want_vals, B * K * 4) == 0, "step %d: top-k values differ", step);
            }
            wgo_apply_mask(logits, 0, B, V, V, want_mask);
            CHECK(memcmp(want_logits, logits, (size_t)B * V * 4) == 0, "phase %d step %d: masked logits differ", phase, step);
            /* the next token of every request: some allowed token of its mask */
            for (uint32_t b = 0; b < B; b++) {
                uint64_t pop = 0;
                for (uint32_t w = 0; w < W; w++) pop += (uint64_t)__builtin_popcount(want_mask[(size_t)b * W + w]);
                CHECK(pop > 0, "request %u has no allowed token", b);
                tokens[b] = (int32_t)wgo_select_bit(want_mask + (size_t)b * W, W, lcg(&seed) % pop);
            }
            HIP(hipMemcpyAsync(d_tokens, tokens, B * 4, hipMemcpyHostToDevice, stream));
            wgo_advance(o, &ov, states, tokens, B);
            if (phase == 0) {
                WG(wg_advance(h, d_states, d_tokens, B, stream));
                HIP(hipMemcpyAsync(got_states, d_states, B * 8, hipMemcpyDeviceToHost, stream));
                HIP(hipStreamSynchronize(stream));
                CHECK(memcmp(got_states, states, B * 8) == 0, "step %d: states differ after advance", step);
            }
        }
        if (phase == 0) {
            /* phase 2 starts over from the start states; the tokens of its step k are fed in step k+1 */
            for (uint32_t b = 0; b < B; b++) { states[2 * b] = start[b & 1].sid; states[2 * b + 1] = 0; }
            HIP(hipMemcpy(d_states, states, B * 8, hipMemcpyHostToDevice));
        }
    }
    uint64_t errors = 1; wg_cache_stats_t st;
    WG(wg_error_count(h, &errors));
    WG(wg_cache_stats(h, &st));
    CHECK(errors == 0, "device error counter %llu", (unsigned long long)errors);
    CHECK(st.lookups == 2ull * STEPS * B && st.hits > 0 && st.builds > 0, "cache statistics");
    printf("lookups %llu hits %llu builds %llu class scans %llu\n", (unsigned long long)st.lookups,
           (unsigned long long)st.hits, (unsigned long long)st.builds, (unsigned long long)st.class_scans);
    wg_destroy(h); wg_vocab_destroy(vocab); wgo_destroy(o);
    hipFree(d_states); hipFree(d_mask); hipFree(d_logits); hipFree(d_tokens); hipFree(d_pick);
    hipFree(d_ids); hipFree(d_vals); hipFree(d_work);
    hipStreamDestroy(stream);
    printf("c_client ok\n");
    return 0;
}
