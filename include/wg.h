/*
 * wg.h -- C ABI of the MI355X structured-decoding hot path.
 *
 * The library implements the per-output-token work of operator-based structured
 * decoding (Sequence / Write / Wait / IfElse / DoWhile operators tracked by a
 * finite-state machine, masks built from each operator's allow / wait sets and
 * cached globally): for every request of a decode batch it produces the
 * vocabulary mask of the request's current state, sets the logits of disallowed
 * tokens to -inf, and advances the state on the sampled token.  All per-step
 * work runs in HIP kernels on gfx950; there is no CPU fallback.
 *
 * Conventions
 *   - Symbols are bytes 0..255 plus end-of-sequence.  A vocabulary token is a
 *     byte string; the token `eos_id` is the one-symbol string [EOS].  A token
 *     is allowed in a state iff feeding its bytes one at a time never meets an
 *     undefined transition.
 *   - A request's state is (sid, aux): sid is the leaf state (0 = FINAL,
 *     0xFFFFFFFF = ERROR), aux the number of allow-bytes consumed so far inside
 *     a bounded Wait (0 elsewhere).
 *   - Leaf states are numbered per template in pre-order (Sequence children in
 *     order; a Wait, then its body; IfElse: condition, if_body, else_body;
 *     DoWhile: body, then condition), one id per Write byte, then one END id.
 *     Template 0 starts at id 1, template k where k-1 ended.
 *   - Masks are [B][W] uint32, W = ceil(V/32); token t is bit (t & 31) of word
 *     t >> 5; bits at and above V are zero.
 *   - "device" pointers are HIP device memory owned by the caller, "host"
 *     pointers are ordinary memory.  `stream` is a hipStream_t passed as
 *     void* (NULL = the default stream).
 *   - Every function returns WG_OK (0) or a negative wg_status_t and never
 *     throws or exits; wg_last_error() describes the last failure on the
 *     calling thread.
 *   - The per-step calls only enqueue work on their stream: they do not
 *     synchronise, allocate or copy between host and device.  A handle has
 *     room for batches of up to 1,024 requests per call; wg_reserve_batch
 *     makes room for more (and synchronises), and a per-step call with a
 *     larger batch than reserved fails with WG_ERR_INVALID and launches
 *     nothing.  wg_add_instances and wg_cache_resize say what they wait for.
 *     Calls on one handle must be
 *     ordered on one stream (or otherwise serialised by the caller); the mask
 *     cache of a handle is shared state.
 *   - A vocabulary lives on the device that was current in wg_vocab_create, and
 *     so does every handle compiled against it.  wg_compile, wg_add_instances
 *     and wg_cache_resize make that device current; the per-step calls expect
 *     the caller to have it current (their pointers and stream belong to it).
 */
#ifndef WG_H
#define WG_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct wg_vocab_s  *wg_vocab_t;    /* device copy of the token-byte vocabulary */
typedef struct wg_handle_s *wg_handle_t;   /* compiled templates + device mask cache */
typedef struct wg_table_s  *wg_table_t;    /* host-only lowered state table (inspection) */

typedef struct { uint32_t sid; uint32_t aux; } wg_state_t;

#define WG_SID_FINAL 0u
#define WG_SID_ERROR 0xFFFFFFFFu
#define WG_UNBOUNDED 0xFFFFFFFFu

typedef enum { WG_F32 = 0, WG_BF16 = 1 } wg_dtype_t;

/* What an accepted end-of-sequence does: stop in FINAL (which then only accepts
 * further EOS), or re-arm the request at its template's start state (continuous
 * batching: the slot is reused by the next request of the same shape). */
enum { WG_EOS_STOP = 0u, WG_EOS_RESTART = 1u };
/* May be or-ed to either: states with equal futures share their cache keys, also across
 * instances of different shapes and inside one instance.  Two states are taken as equal when
 * they agree in what they do with every byte (kind, literal byte, allow / wait sets, bound,
 * whether EOS is accepted) and, one level less deep, so do their successors, down to as many
 * levels as the longest token has bytes: no token can tell such states apart, so their masks are
 * the same (the global cache of the section "Mask Generation and Global Caching": a mask depends
 * on what the operators ahead accept, not on which request or template they belong to).  Costs
 * host time when instances are compiled or added (every new state is compared level by level);
 * without it only instances that are equal as a whole share keys. */
enum { WG_SHARE_STATES = 2u };

typedef enum {
    WG_OK = 0,
    WG_ERR_INVALID = -1,    /* null pointer, zero size, bad enum, size mismatch */
    WG_ERR_PARSE = -2,      /* malformed template or argument binding */
    WG_ERR_NOMEM = -3,      /* host or device allocation failed / cache would not fit */
    WG_ERR_HIP = -4         /* a HIP runtime call failed */
} wg_status_t;

/* Runtime snippet arguments of one template instance: names[i] binds $names[i]
 * to the bytes data[i][0 .. lens[i]).  In Write($x) the bytes are the literal;
 * in a set position (allow=$x, wait={a, $x}) they are the set of those bytes. */
typedef struct {
    uint32_t n;
    const char *const *names;
    const uint8_t *const *data;
    const uint64_t *lens;
} wg_args_t;

typedef struct {
    uint64_t lookups;       /* request-steps served by wg_fill_masks */
    uint64_t hits;          /* ... whose mask was already cached */
    uint64_t builds;        /* mask rows built (one per distinct missing key) */
    uint64_t uncached_builds;/* ... of which could not be kept because every cache row was taken */
    uint64_t class_scans;   /* vocabulary scans (one per distinct missing allow/wait class table) */
    uint64_t entries_walked;/* candidate tokens examined by the row builds (index ranges and class lists) */
    uint64_t keys;          /* distinct masks the compiled instances can ask for (instances of one shape share theirs) */
    uint64_t cache_rows;    /* rows the cache can hold (wg_cache_resize) */
    uint64_t rows_in_use;   /* rows holding a mask since the last clear */
    uint64_t arena_bytes;   /* device bytes reserved for cached rows and class indexes */
} wg_cache_stats_t;

/* State kinds reported by wg_table_state. */
enum { WG_KIND_FINAL = 0, WG_KIND_LIT = 1, WG_KIND_WAIT = 2, WG_KIND_COND = 3, WG_KIND_END = 4 };

typedef struct {
    uint32_t kind;          /* WG_KIND_* */
    uint32_t byte;          /* LIT: the expected byte */
    uint32_t next_a;        /* LIT / WAIT: successor; COND: target of true_waits */
    uint32_t next_b;        /* COND: target of false_waits */
    uint32_t eos_next;      /* state after EOS, or WG_SID_ERROR if EOS is rejected */
    uint32_t max;           /* WAIT: bound on consumed allow-bytes, or WG_UNBOUNDED */
    uint32_t tmpl;          /* template instance the state belongs to */
    uint32_t n_keys;        /* distinct masks this state can have (budget variants) */
    uint32_t key;           /* the first of its cache keys (states that share keys report the same) */
} wg_state_info_t;

/* ---- vocabulary (the token map the structure factory of the section "Collaborative Parsing"
 * is built over: every structure and every request of an engine shares one vocabulary) ------
 * CSR token bytes: token t is host_bytes[host_offsets[t] .. host_offsets[t+1]).  Both
 * arrays are host memory and are copied; eos_id < 0 means "no EOS token".  A token
 * with no bytes other than eos_id is never allowed.  The vocabulary is uploaded to
 * HBM once and may be shared by several handles; destroy it after them. */
int wg_vocab_create(const uint8_t *host_bytes, const uint64_t *host_offsets, uint32_t V,
                    int32_t eos_id, wg_vocab_t *out);
void wg_vocab_destroy(wg_vocab_t v);

/* ---- compilation (the paper's split into a static structure precompiled once and
 * dynamic arguments instantiated per request; section "Collaborative Parsing") ---------
 * templates[i] is UTF-8 text in the operator syntax of the paper's listing in the
 * section "Operator Building and State Tracking":
 *     Sequence(op, ...)            Write("bytes") | Write($arg)
 *     Wait(allow={..} | denies={..}, wait={..} [, max=N] [, body=op])
 *     Wait(allow={..}, true_waits={..}, false_waits={..})        (condition)
 *     IfElse(condition=Wait(..), if_body=op|None, else_body=op|None)
 *     DoWhile(body=op|None, condition=Wait(..))
 * Set elements: a byte, \d \w \s, \xHH, \n \t \r, \c (the byte c), [a-z0-9] classes,
 * <eos>, $arg.  Identical template texts are parsed once and instantiated per args[i]
 * (args may be NULL when no template has holes).  start_states_out[i] (host, may be
 * NULL) receives the start state of instance i.  The resulting handle serves a
 * heterogeneous batch: state ids are global to the handle.  Every instance has state ids of
 * its own; instances whose states are equal one for one (the same structure instantiated with
 * the same arguments) share their cache keys, so their masks are built and held once (the global
 * cache of the section "Mask Generation and Global Caching"); with WG_SHARE_STATES in flags so do
 * any two states that no token can tell apart.
 * wg_lower does the host part only (no GPU needed) and returns an inspectable table;
 * lmax is the longest token length the masks will be built for. */
int wg_lower(const char *const *templates, const wg_args_t *args, uint32_t n_templates,
             uint32_t flags, uint32_t lmax, wg_table_t *out);
/* wg_regex_to_template: a constraint given as a regular expression, turned into template text
 * for wg_compile / wg_lower (the translation of the section "Operator Building and State
 * Tracking": literals -> Write, classes -> Wait, * + ? | -> DoWhile / IfElse around condition
 * Waits).  Bytes, not code points; the whole output must match; syntax: literals, escapes
 * (\d \w \s \D \W \S \n \t \r \f \v \0 \xHH, \c for a punctuation byte c), '.', [..] and
 * [^..] with ranges, ( ) and (?: ), |, * + ? {m} {m,} {m,n}, ^ and $ at the ends.  The operators
 * decide on one byte, consume it, and have two ways out of a checkpoint, so an expression is
 * refused (WG_ERR_PARSE, with the rule it breaks) unless: every optional or repeated group and
 * each side of an alternation starts with a single byte or class; what follows such a group is
 * a single byte or class or the end; the byte sets a decision tells apart, and a repeated
 * class and its terminators, are disjoint; an alternation has two sides (any number when all
 * are single bytes).  The text is written to out[0 .. capacity) with its terminating 0;
 * *needed (may be NULL) receives the size required, also when capacity is too small
 * (WG_ERR_INVALID).  The expression ends at the end of generation: its last checkpoint
 * accepts <eos>. */
int wg_regex_to_template(const char *regex, char *out, uint64_t capacity, uint64_t *needed);

/* appends instances to a table, numbering their states after the existing ones (the host
 * half of wg_add_instances); on WG_ERR_PARSE the table is unchanged */
int wg_table_add_instances(wg_table_t t, const char *const *templates, const wg_args_t *args,
                           uint32_t n_templates);
uint32_t wg_table_num_instances(wg_table_t t);
uint32_t wg_table_num_states(wg_table_t t);
uint32_t wg_table_start_state(wg_table_t t, uint32_t instance);
int wg_table_state(wg_table_t t, uint32_t sid, wg_state_info_t *out);
/* class of a byte in state sid: 0 reject, 1 stay, 2 exit to next_a, 3 exit to next_b;
 * for symbol 256 (EOS): 2 if accepted (the state after it is eos_next), else 0 */
int wg_table_symbol_class(wg_table_t t, uint32_t sid, uint32_t symbol);
void wg_table_destroy(wg_table_t t);

int wg_compile(const char *const *templates, const wg_args_t *args, uint32_t n_templates,
               wg_vocab_t vocab, uint32_t flags, wg_handle_t *out, wg_state_t *start_states_out);
void wg_destroy(wg_handle_t h);

/* wg_add_instances: instantiate further requests on a live handle (a new request arriving in a
 * running batch brings its own dynamic arguments; the static structure of a template text seen
 * before is reused).  State ids, cached rows and class indexes of the existing instances stay
 * valid; start_states_out[i] (host, may be NULL) receives the start state of new instance i.
 * The new table slices are copied on `stream`, which is synchronised before the call returns;
 * when the tables outgrow the room reserved for them (half again of what was needed at the
 * last growth) the whole device is synchronised once and the tables move.  On WG_ERR_PARSE
 * nothing was added; on WG_ERR_NOMEM / WG_ERR_HIP the instances are in the host table but their
 * states are out of range for the device (all-zero masks) until a later call succeeds.  Not to be called while another thread enqueues work on the handle. */
int wg_add_instances(wg_handle_t h, const char *const *templates, const wg_args_t *args,
                     uint32_t n_templates, wg_state_t *start_states_out, void *stream);
uint32_t wg_num_instances(wg_handle_t h);

/* wg_cache_resize: the cache holds `rows` mask rows from now on (one row is 4*ceil(V/128)*4
 * bytes).  wg_compile sizes it for every key of its instances (at least 4096 rows, at most a
 * quarter of the free device memory).  Rows are handed out in order of first use; once all are
 * taken, further keys are still served correctly but rebuilt on every call that needs them
 * (wg_cache_stats.uncached_builds counts them) until wg_cache_clear or a resize.  Synchronises
 * the device and clears the cache. */
int wg_cache_resize(wg_handle_t h, uint32_t rows);

/* wg_reserve_batch: room for calls with up to max_batch requests (1 .. 65535) in the handle's
 * per-call lists (which request refers to which cache row, the keys and class tables a call has
 * to build).  wg_compile reserves 1,024.  Only ever grows; when it grows, the device is
 * synchronised and the lists are allocated anew, so a HIP graph recorded before has to be
 * recorded again.  Call it at set-up, never between the steps of a decode loop: the per-step
 * calls themselves never allocate and refuse a batch above the reservation. */
int wg_reserve_batch(wg_handle_t h, uint32_t max_batch);
uint32_t wg_max_batch(wg_handle_t h);       /* the current reservation */

/* wg_set_scan_batch: how many of the class tables a call has to index (the context-free part of
 * the masks, "Mask Generation and Global Caching": a mask depends on the allow / wait sets only)
 * one workgroup takes through its share of the vocabulary together: 1 .. 8, or 0 (what wg_compile
 * sets) to let each call choose -- one table while the call brings few, more as it brings many,
 * and always one for a handle with few class tables.  A tuning knob: every setting gives the same
 * masks.  Takes effect with the next call; a HIP graph recorded before keeps the old setting. */
int wg_set_scan_batch(wg_handle_t h, uint32_t tables);

uint32_t wg_num_states(wg_handle_t h);
uint32_t wg_mask_words(wg_handle_t h);      /* W = ceil(V/32) */

/* ---- per-step calls (device pointers, enqueue only) -------------------------------------
 * wg_fill_masks: d_bitmask[b][0..W) <- mask of d_states[b] (mask creation with the global
 * cache of the section "Mask Generation and Global Caching"): cached rows are gathered,
 * missing ones are built once per distinct key and cached.  An ERROR or out-of-range
 * state gets an all-zero row. */
int wg_fill_masks(wg_handle_t h, const wg_state_t *d_states, uint32_t B, uint32_t *d_bitmask,
                  void *stream);

/* wg_apply_mask: the mask is applied to the logits before sampling (Introduction: the binary
 * tensor over the vocabulary, ones for allowed tokens, zeros for disallowed ones, applied to the
 * logits prior to sampling).  In place, logits[b][t] <- -inf (0xFF800000 / 0xFF80) where the mask
 * bit is 0; other elements keep their bit pattern.  Row b starts row_stride_elems * b elements
 * after d_logits (row_stride_elems >= V); the mask row stride is ceil(V/32) words. */
int wg_apply_mask(void *d_logits, wg_dtype_t dtype, uint32_t B, uint32_t V,
                  int64_t row_stride_elems, const uint32_t *d_bitmask, void *stream);

/* wg_masked_argmax: greedy decoding fused with the mask, the step that follows mask application
 * when sampling is greedy: d_tokens[b] <- the allowed token of row b with the largest logit.  The
 * logits are only read (nothing is set to -inf), so this call replaces wg_apply_mask + argmax.
 * A NaN ranks below every number (also below -inf), equal values (-0.0 equals +0.0) keep the
 * lowest token id, a row that allows nothing gives -1.  Layout of logits and mask as in
 * wg_apply_mask.  The workgroups of a row merge through a per-GPU scratch array inside the
 * library, so two wg_masked_argmax calls must not overlap on one GPU (order them on one stream). */
int wg_masked_argmax(const void *d_logits, wg_dtype_t dtype, uint32_t B, uint32_t V,
                     int64_t row_stride_elems, const uint32_t *d_bitmask, int32_t *d_tokens,
                     void *stream);

/* wg_masked_topk: the candidates of top-k sampling taken under the mask, logits read once and
 * never written (the paper applies the mask to the logits before sampling, Introduction; this
 * is the step after, fused with it like wg_masked_argmax).
 * d_ids[b][r], r = 0 .. k-1: the allowed tokens of row b with the k largest logits, best
 * first; equal logits (-0.0 equals +0.0) by lower token id, NaNs after every number (also after
 * -inf).  d_values[b][r]: that token's logit, the raw element in the logits' dtype.  A row that
 * allows fewer than k tokens ends with ids of -1 and values of -inf.  1 <= k <= 64;
 * B <= 65535; ceil(V / 8192) * k <= 4096.  d_ids is int32 [B][k], d_values [B][k] of `dtype`.
 * d_workspace: device memory of at least wg_masked_topk_workspace(B, V, k) bytes, 8-byte
 * aligned, owned by the caller, overwritten by the call (it holds the best k of every 8,192
 * tokens of a row between the call's two kernels); calls that share a workspace must not
 * overlap.  Mask bits at and above V must be zero, as wg_fill_masks leaves them.  Enqueues
 * two kernels on `stream`; nothing is allocated.  Arguments outside the limits above, a null
 * pointer or a workspace that is too small or misaligned give WG_ERR_INVALID and launch nothing. */
uint64_t wg_masked_topk_workspace(uint32_t B, uint32_t V, uint32_t k);
int wg_masked_topk(const void *d_logits, wg_dtype_t dtype, uint32_t B, uint32_t V,
                   int64_t row_stride_elems, const uint32_t *d_bitmask, uint32_t k,
                   int32_t *d_ids, void *d_values, void *d_workspace, uint64_t workspace_bytes,
                   void *stream);

/* wg_masked_topk_static: wg_masked_topk for callers that cannot allocate device memory, not
 * even a workspace: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, limits and results as wg_masked_topk, except that the lists between
 * its two kernels live in a device array inside the library (4 MiB per GPU, held until the
 * process ends; wg_masked_topk_static_capacity() returns its size in bytes), so a call needs
 * B * ceil(V / 8192) * k * 8 <= 4,194,304 (B = 256, V = 151,936, k = 64 takes 2.5 MB); anything
 * larger gives WG_ERR_INVALID and launches nothing.  The call allocates and frees nothing and
 * enqueues two kernels on `stream`; the array's address on the current device is asked of the
 * HIP runtime once (by wg_vocab_create on that device, else by the first call).  Every call on a
 * GPU uses that GPU's one array: calls that overlap on one GPU (two streams, two threads) race;
 * order them on one stream.  Nothing has to be cleared between calls: the first kernel writes
 * every key the second reads. */
uint64_t wg_masked_topk_static_capacity(void);
int wg_masked_topk_static(const void *d_logits, wg_dtype_t dtype, uint32_t B, uint32_t V,
                          int64_t row_stride_elems, const uint32_t *d_bitmask, uint32_t k,
                          int32_t *d_ids, void *d_values, void *stream);

/* wg_advance: d_states[b] <- state after d_tokens[b] (section "Operator Building and State
 * Tracking": the state machine follows the output symbol by symbol, constant work per symbol).  A token the state rejects, or a token id outside [0, V), gives
 * {WG_SID_ERROR, 0} and increments the handle's device error counter. */
int wg_advance(wg_handle_t h, wg_state_t *d_states, const int32_t *d_tokens, uint32_t B,
               void *stream);

/* wg_forced_bytes (jump-forward): what request b can only produce next.  A Write is a chain of
 * checkpoints that each admit one symbol (section "Mask Generation and Global Caching": Write
 * as a sequence of specialised Waits), so from a state inside a Write the continuation is fixed
 * up to the next Wait, condition or end of the template, and an engine may append those bytes
 * without sampling them.  d_bytes[b][0 .. d_lens[b]) receives the rest of the request's Write and
 * of the Writes that follow it directly, cut at cap bytes (d_bytes is [B][cap] uint8, d_lens [B]
 * uint32); d_lens[b] is 0 for a state that is not a Write byte (also ERROR and out-of-range
 * states).  d_end_states[b] (may be NULL) receives the state after those bytes: feeding them
 * through wg_advance as tokens leads to the same state; a request with nothing forced keeps its
 * state, aux included.  The states themselves are only read.  One kernel, enqueued on `stream`. */
int wg_forced_bytes(wg_handle_t h, const wg_state_t *d_states, uint32_t B, uint32_t cap,
                    uint8_t *d_bytes, uint32_t *d_lens, wg_state_t *d_end_states, void *stream);

/* wg_advance_fill_masks: wg_advance followed by wg_fill_masks on the new states, for the decode
 * loop, where the two always meet (the token sampled under step k's mask is consumed, then step
 * k+1's mask is produced): same results, one kernel launch and one pass over the state
 * descriptors fewer.  In wg_profile_read the combined first kernel is counted as the lookup. */
int wg_advance_fill_masks(wg_handle_t h, wg_state_t *d_states, const int32_t *d_tokens, uint32_t B,
                          uint32_t *d_bitmask, void *stream);

/* wg_decode_step: the whole per-step path in one call, for the decode loop: the states are
 * advanced by the tokens sampled in the step before (d_tokens == NULL skips this: first step),
 * the masks of the new states are produced into d_bitmask as by wg_fill_masks and applied to
 * d_logits ([B][V] with V of the handle's vocabulary, layout as in wg_apply_mask) as by
 * wg_apply_mask.  Same results as wg_advance + wg_fill_masks + wg_apply_mask in four kernel
 * launches instead of six: the advance rides in the lookup kernel and the masking in the gather
 * kernel (rows whose address or stride rules out 16-byte stores are masked by the separate
 * apply kernels instead).  In wg_profile_read the combined kernels count as lookup and gather. */
int wg_decode_step(wg_handle_t h, wg_state_t *d_states, const int32_t *d_tokens, uint32_t B,
                   uint32_t *d_bitmask, void *d_logits, wg_dtype_t dtype, int64_t row_stride_elems,
                   void *stream);

/* Forget every cached mask row and every class-table index built from the operators' allow /
 * wait sets.  O(1) and launches nothing: the handle's cache generation is bumped on the host
 * and travels with every later call as a kernel argument (so a clear recorded into a HIP
 * graph has no effect on replays, and a graph holding calls of this handle has to be recorded
 * again after a clear, a resize or wg_add_instances).  The static indexes of the vocabulary itself (made by
 * wg_vocab_create) are not part of the cache. */
int wg_cache_clear(wg_handle_t h, void *stream);

/* ---- introspection (these synchronise the device) ---------------------------------------- */
int wg_cache_stats(wg_handle_t h, wg_cache_stats_t *host_out);
int wg_error_count(wg_handle_t h, uint64_t *host_out);
const char *wg_last_error(void);

/* ---- kernel timing (tracing aid; off by default) ------------------------------------------
 * While enabled, wg_fill_masks and wg_advance launch each of their kernels with a pair of HIP
 * events that take the kernel's own begin and end timestamps (this allocates events on the
 * host as needed).  wg_profile_read
 * synchronises, adds up the elapsed times since the last read and resets the record. */
typedef struct {
    uint64_t fill_calls, advance_calls;
    double lookup_ms, scan_ms, build_ms, gather_ms, advance_ms;   /* summed kernel durations */
    uint64_t apply_calls;
    double apply_ms;
} wg_profile_t;
int wg_profile_enable(wg_handle_t h, int on);
int wg_profile_read(wg_handle_t h, wg_profile_t *host_out);
/* wg_apply_mask with its kernel's begin and end taken into the handle's record while timing is
 * enabled (apply_calls, apply_ms); exactly wg_apply_mask while it is not. */
int wg_profile_apply_mask(wg_handle_t h, void *d_logits, wg_dtype_t dtype, uint32_t B, uint32_t V,
                          int64_t row_stride_elems, const uint32_t *d_bitmask, void *stream);

/* ---- sampler stand-in for harnesses (not part of the decoding path) ----------------------
 * d_tokens[b] <- index of the (d_draws[b] mod popcount)-th set bit of mask row b, or -1 for
 * an all-zero row. */
int wg_select_tokens(const uint32_t *d_bitmask, uint32_t B, uint32_t V, const uint64_t *d_draws,
                     int32_t *d_tokens, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* WG_H */
