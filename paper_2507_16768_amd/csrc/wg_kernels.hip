// HIP kernels of the structured-decoding hot path for gfx950 (wave64).
//
//   lookup       : request state -> cache key, claims missing keys and class tables
//                  (advance_lookup: after advancing the state by the sampled token)
//   class_scan   : every vocabulary token against one checkpoint's byte-class table: a first look
//                  that settles most tokens with one instruction or table look-up each (64-lane
//                  ballots pack the row words), the rest byte by byte through the table in LDS
//                  (class_scan_batch, for handles with many tables: several tables per pass
//                  over the tokens, the first look from the vocabulary's rows by byte value)
//   key_build    : a workgroup assembles the row of a missing key (or its words for one token
//                  range) in LDS from the class index and the tokens that leave the state early,
//                  which it finds in the vocabulary's indexes (byte order, byte pairs) or in the
//                  class index's lists
//   gather       : cached row -> bitmask[b]   (gather_apply: and -inf into the logits)
//   apply        : logits <- -inf where the mask bit is 0
//   masked_argmax: greedy choice under the mask, logits only read
//   advance      : per-request walk of the sampled token
//   forced_bytes : per request, the rest of the Write run its state lies in
//   select       : harness sampler stand-in (k-th set bit of a row)
//
// No MFMA anywhere: the path is byte matching and memory traffic.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <mutex>

#include "wg_device.h"
#include "wg_order.h"

namespace wg {

constexpr uint32_t kScanGroup = 2048;     // tokens per class_scan workgroup
static_assert(kScanGroup == kPartGroup, "a class_scan workgroup's tokens lie in one token range");
static_assert(2u + 2u * kParts <= 32u, "the counters of a class fit its 128 bytes");
constexpr uint32_t kCountStride = 32;     // class_count entries are 128 bytes apart
constexpr uint32_t kXcds = 8;             // accelerator complex dies, each with a private L2
constexpr uint32_t kShortRem = 4;         // exit entries with at most this many bytes left are "short"

// ---------------------------------------------------------------------------------------------
// Generic per-lane walker: feeds `len` bytes at `p` to the FSM from (sid, aux).
// Returns false on the first rejected byte.  Every state entered mid-token starts with
// aux = 0; only a bounded Wait counts.
__device__ __forceinline__ bool walk_bytes(const DeviceTable &T, uint32_t &sid, uint32_t &aux,
                                           const uint8_t *__restrict__ p, uint32_t len)
{
    uint32_t cur = WG_SID_ERROR;          // sid whose descriptor is loaded
    uint32_t kind = 0, lit = 0, na = 0, nb = 0, mx = 0;
    const uint8_t *cls = nullptr;
    for (uint32_t i = 0; i < len; i++) {
        if (sid != cur) {
            if (sid >= T.n_states) return false;            // ERROR or corrupt state
            const StateDesc &d = T.states[sid];
            kind = d.kind_byte & 0xFFu; lit = (d.kind_byte >> 8) & 0xFFu;
            na = d.next_a; nb = d.next_b; mx = d.max;
            cls = T.classes + (size_t)d.cls * 256u;
            cur = sid;
        }
        uint32_t x = p[i];
        if (kind == WG_KIND_LIT) {
            if (x != lit) return false;
            sid = na; aux = 0;
        } else if (kind == WG_KIND_WAIT || kind == WG_KIND_COND) {
            uint32_t c = cls[x];
            if (c == CLS_STAY) {
                if (mx != WG_UNBOUNDED) { if (aux >= mx) return false; aux++; }
            } else if (c == CLS_EXIT_A) { sid = na; aux = 0; }
            else if (c == CLS_EXIT_B) { sid = nb; aux = 0; }
            else return false;
        } else return false;                                // FINAL / END accept no byte
    }
    return true;
}

// Verdict and next state of one token (EOS is the one-symbol string [EOS]).
__device__ __forceinline__ bool walk_token(const DeviceTable &T, const DeviceVocab &Vc,
                                           uint32_t &sid, uint32_t &aux, int64_t t)
{
    if (t < 0 || t >= (int64_t)Vc.V || sid >= T.n_states) return false;
    if ((int64_t)Vc.eos_id == t) {
        uint32_t e = T.states[sid].eos_next;
        if (e == WG_SID_ERROR) return false;
        sid = e; aux = 0;
        return true;
    }
    uint32_t lo = Vc.offsets[t], hi = Vc.offsets[t + 1];
    if (hi <= lo) return false;                             // byte-less non-EOS token
    return walk_bytes(T, sid, aux, Vc.bytes + lo, hi - lo);
}

// Eight bytes of a token (held as three 8-byte chunks) starting at byte i.
__device__ __forceinline__ uint64_t token_window(uint64_t c0, uint64_t c1, uint64_t c2, uint32_t i)
{
    const uint32_t q = i >> 3, sh = (i & 7u) * 8u;
    const uint64_t w0 = q == 0 ? c0 : q == 1 ? c1 : c2;
    const uint64_t w1 = q == 0 ? c1 : q == 1 ? c2 : 0ull;
    return sh ? (w0 >> sh) | (w1 << (64u - sh)) : w0;
}

// Walks bytes [i, L) of a token held in registers (L <= 24) from (sid, aux), consuming up to
// eight bytes per state visit: a run of literal states is one masked 8-byte compare against
// the state table's literal bytes, a stay-run inside a checkpoint is eight independent class
// look-ups.  Returns false on the first rejected byte.
__device__ __forceinline__ bool walk_chunks(const DeviceTable &T, uint32_t &sid, uint32_t &aux,
                                            uint64_t c0, uint64_t c1, uint64_t c2, uint32_t i, uint32_t L)
{
    const uint64_t *lit64 = reinterpret_cast<const uint64_t *>(T.lit);
    while (i < L) {
        if (sid >= T.n_states) return false;
        const StateDesc d = T.states[sid];
        const uint32_t kind = d.kind_byte & 0xFFu;
        const uint32_t n = L - i < 8u ? L - i : 8u;
        const uint64_t tb = token_window(c0, c1, c2, i);
        if (kind == WG_KIND_LIT) {
            const uint32_t sh = (sid & 7u) * 8u;
            const uint64_t l0 = lit64[sid >> 3], l1 = lit64[(sid >> 3) + 1u];
            const uint64_t lv = sh ? (l0 >> sh) | (l1 << (64u - sh)) : l0;
            const uint32_t m = n < d.run ? n : d.run;            // literal bytes compared now
            const uint64_t mask = m == 8u ? ~0ull : (1ull << (8u * m)) - 1ull;
            if ((tb ^ lv) & mask) return false;
            sid = m == d.run ? d.cls : sid + m;                  // d.cls: state after the Write
            aux = 0; i += m;
        } else if (kind == WG_KIND_WAIT || kind == WG_KIND_COND) {
            const uint8_t *cls = T.classes + (size_t)d.cls * 256u;
            uint32_t code = 0;
#pragma unroll
            for (int k = 0; k < 8; k++) code |= (uint32_t)cls[(tb >> (8 * k)) & 0xFFu] << (2 * k);
            const uint32_t x = code ^ 0x5555u;
            const uint32_t mm = (x | (x >> 1)) & 0x5555u & ((1u << (2u * n)) - 1u);
            const uint32_t stays = mm ? (uint32_t)__builtin_ctz(mm) >> 1 : n;
            if (d.max != WG_UNBOUNDED && stays) {                // each stay needs budget left
                if (aux + stays > d.max) return false;
                aux += stays;
            }
            i += stays;
            if (mm) {
                const uint32_t c = (code >> (2u * stays)) & 3u;
                if (c == CLS_REJECT) return false;
                sid = c == CLS_EXIT_A ? d.next_a : d.next_b;
                aux = 0; i += 1u;
            }
        } else return false;                                     // FINAL / END accept no byte
    }
    return true;
}

// ---------------------------------------------------------------------------------------------
// lookup: state -> cache key.  A missing key is claimed by exactly one request (CAS on the
// key's tag), gets a row of the arena (or, when the arena is full, is built straight into
// the claimer's bitmask row and not kept) and is queued for key_build: the i-th claim of a call
// takes the i-th free row, so the order of the claims is their row allocation and the count
// of rows in use is brought up to date once per call, by the last kernel of the fill; if the key's state is a
// checkpoint whose class table has no index yet in this generation, the table is claimed and
// queued for class_scan.

// What a lookup reads from the handle's counters before anything depends on it.
struct LookupEnv {
    unsigned long long launch;   // number of this fill call
    uint32_t rows0;              // arena rows in use before this call
};

__device__ __forceinline__ LookupEnv lookup_env(const DeviceCache &Cc)
{
    const unsigned long long sc = Cc.ctr->slot_ctr;
    return LookupEnv{Cc.ctr->launch & kTagLaunchMask, (uint32_t)(sc >> 32) == Cc.epoch ? (uint32_t)sc : 0u};
}

// The lookup of request b in state (sid, aux); every lane of the wavefront calls it, `live`
// says whether the lane has a request.
__device__ __forceinline__ void lookup_one(const DeviceTable &T, const DeviceCache &Cc,
                                           const LookupEnv &env, uint32_t b, bool live, uint32_t sid, uint32_t aux)
{
    const uint32_t lane = threadIdx.x & 63u;
    bool hit = false, claimed = false;
    uint32_t key = kNoKey, kind = 0, variant = 0;
    const uint32_t epoch = Cc.epoch;
    const unsigned long long launch = env.launch;
    const uint32_t rows0 = env.rows0;
    uint32_t ref = kNoKey;
    StateDesc d{}, dn[2] = {};
    ClassInfo ci{};
    uint32_t class_gen = 0;
    if (live) {
        if (sid < T.n_states) {
            d = T.states[sid];
            kind = d.kind_byte & 0xFFu;
            if (kind == WG_KIND_WAIT && d.max != WG_UNBOUNDED) {
                const uint32_t left = d.max > aux ? d.max - aux : 0u;
                variant = T.lmax - (left < T.lmax ? left : T.lmax);
            }
            key = d.key_base + variant;
            const unsigned long long t = __hip_atomic_load(&Cc.tags[key], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            // Requested right behind the key's tag, although only a missing key needs them: the
            // two successors' descriptors and the generation of the class index.  Plain loads
            // from clamped indexes, so that nothing waits for them before the tag has decided.
            dn[0] = T.states[d.next_a < T.n_states ? d.next_a : 0u];
            dn[1] = T.states[d.next_b < T.n_states ? d.next_b : 0u];
            const uint32_t own_class = (kind == WG_KIND_WAIT || kind == WG_KIND_COND) ? d.cls : 0u;
            class_gen = __hip_atomic_load(&Cc.class_built[own_class], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            ci = T.class_info[own_class];
            // anything but a row of this generation or a claim made in this very call is stale
            hit = (uint32_t)(t >> 32) == epoch;
            const bool this_call = t >= kTagClaim && ((t >> 16) & kTagLaunchMask) == launch;
            if (!hit && !this_call)
                claimed = atomicCAS(&Cc.tags[key], t, kTagClaim | (launch << 16) | b) == t;
            ref = hit ? (uint32_t)t : claimed ? kRefSelf : kRefByKey | key;
        }
        Cc.row_ref[b] = ref;
    }
    // The claimers of a wavefront take their arena rows and their places in the miss list
    // together.  A key whose candidate tokens all need a deep walk (its state hands over to
    // another checkpoint) goes to the front of the list: key_build cuts it into one work item per
    // token range and starts those first; every other key is one work item, from the back.
    const unsigned long long cm = __ballot(claimed);
    if (cm) {
        HopState hop[2];
        bool deep = false;
        if (claimed) {
#pragma unroll
            for (int w = 0; w < 2; w++) {
                const uint32_t t = w ? d.next_b : d.next_a;
                const StateDesc &td = dn[w];
                hop[w] = HopState{0xFFu, 0u, WG_SID_ERROR, WG_SID_ERROR, WG_UNBOUNDED, 0u};
                if (t < T.n_states)
                    hop[w] = HopState{td.kind_byte & 0xFFu, (td.kind_byte >> 8) & 0xFFu,
                                      td.next_a, td.next_b, td.max, td.cls};
            }
            const bool ckpt0 = hop[0].kind == WG_KIND_WAIT || hop[0].kind == WG_KIND_COND;
            const bool ckpt1 = hop[1].kind == WG_KIND_WAIT || hop[1].kind == WG_KIND_COND;
            deep = ((kind == WG_KIND_LIT || kind == WG_KIND_WAIT) && ckpt0) || (kind == WG_KIND_COND && (ckpt0 || ckpt1));
        }
        const unsigned long long dm = __ballot(claimed && deep), pm = cm & ~dm;
        // The claim of the class table goes out first, so that its compare-and-swap is in flight
        // together with the three counters of the key claims (three counters, three lanes).
        const bool ckpt = kind == WG_KIND_WAIT || kind == WG_KIND_COND;
        const bool want_class = claimed && ckpt && class_gen != epoch;
        uint32_t class_was = epoch;
        if (want_class) class_was = atomicCAS(&Cc.class_built[d.cls], class_gen, epoch);
        uint32_t got = 0;
        if (lane == 0) got = atomicAdd(&Cc.ctr->n_claims, (uint32_t)__popcll(cm));
        else if (lane == 1 && dm) got = atomicAdd(&Cc.ctr->n_deep, (uint32_t)__popcll(dm));
        else if (lane == 2 && pm) got = atomicAdd(&Cc.ctr->n_plain, (uint32_t)__popcll(pm));
        const uint32_t first_key = __shfl(got, 0), first_deep = __shfl(got, 1), first_plain = __shfl(got, 2);
        const bool class_claimed = want_class && class_was == class_gen;
        const unsigned long long ccm = __ballot(class_claimed);
        uint32_t first_class = 0;
        if (ccm) {
            if (lane == 0) first_class = atomicAdd(&Cc.ctr->n_class_miss, (uint32_t)__popcll(ccm));
            first_class = __shfl(first_class, 0);
        }
        if (claimed) {
            const unsigned long long below = (1ull << lane) - 1ull;
            const uint32_t idx = first_key + (uint32_t)__popcll(cm & below);
            const uint32_t slot = Cc.cap_rows - rows0 > idx ? rows0 + idx : kNoSlot;
            // this request builds the key: resolve what key_build needs into the miss entry
            MissEntry me{};
            me.key = key; me.sid = sid; me.aux = aux; me.kind = kind;
            me.r = T.lmax - variant; me.cls = d.cls; me.eos_next = d.eos_next;
            me.next_a = d.next_a; me.next_b = d.next_b;
            me.slot = slot; me.req = b;
            me.hop[0] = hop[0]; me.hop[1] = hop[1];
            me.lit = (d.kind_byte >> 8) & 0xFFu;
            // Where the candidates come from.  A key that is not deep has, behind each exit, a
            // literal byte or a state that takes no byte at all: its candidates are found in
            // the static indexes of the vocabulary by the bytes involved (tokens of at most 24
            // bytes: the walkers of those paths hold a token in registers).
            me.mode = KB_LIST;
            if (!deep && T.lmax <= 24u) {
                const bool lit0 = hop[0].kind == WG_KIND_LIT, lit1 = hop[1].kind == WG_KIND_LIT;
                if (kind == WG_KIND_LIT) me.mode = KB_SORTED;
                else if (ckpt && (!lit0 || ci.n_a != kManyExits) && (!lit1 || ci.n_b != kManyExits)) {
                    me.mode = KB_BIGRAM;
                    me.n_a = lit0 ? ci.n_a : 0; me.n_b = lit1 ? ci.n_b : 0;
                    me.exits[0] = ci.a[0] | ci.a[1] << 8 | ci.a[2] << 16 | (uint32_t)ci.a[3] << 24;
                    me.exits[1] = ci.a[4] | ci.a[5] << 8 | ci.b[0] << 16 | (uint32_t)ci.b[1] << 24;
                    me.exits[2] = ci.b[2] | ci.b[3] << 8 | ci.b[4] << 16 | (uint32_t)ci.b[5] << 24;
                }
            }
            Cc.miss[deep ? first_deep + (uint32_t)__popcll(dm & below)
                         : Cc.miss_cap - 1u - (first_plain + (uint32_t)__popcll(pm & below))] = me;
            if (class_claimed) {
                // the class list and the list of each token range: short entries fill from the
                // front, long ones from the back
                const uint32_t c = d.cls;
#pragma unroll
                for (uint32_t i = 0; i < 2u + 2u * kParts; i++) Cc.class_count[c * kCountStride + i] = 0;
                Cc.class_miss[first_class + (uint32_t)__popcll(ccm & below)] = c;
            }
        }
    }
    const unsigned long long hv = __ballot(hit), lv = __ballot(live);
    if (lane == 0) {
        atomicAdd(&Cc.ctr->lookups, (unsigned long long)__popcll(lv));
        atomicAdd(&Cc.ctr->hits, (unsigned long long)__popcll(hv));
    }
}

__global__ void __launch_bounds__(64)
lookup_kernel(DeviceTable T, DeviceCache Cc, const wg_state_t *__restrict__ states, uint32_t B)
{
    const uint32_t b = blockIdx.x * blockDim.x + threadIdx.x;
    const bool live = b < B;
    const LookupEnv env = lookup_env(Cc);
    uint32_t sid = 0, aux = 0;
    if (live) { sid = states[b].sid; aux = states[b].aux; }
    lookup_one(T, Cc, env, b, live, sid, aux);
}

// ---------------------------------------------------------------------------------------------
// class_scan: runs every vocabulary token through one checkpoint's class table (the part of
// a mask that depends only on the operator's allow / wait sets, hence shared by every state
// and request using the same sets).  Per token: the first byte that does not stay and its
// class.  Results: row [stay] = tokens whose bytes all stay, row [end] = tokens that exit on
// their last byte, and one ExitEntry per token that exits earlier.
//
// A workgroup handles one (class table, 2048-token group): the 256-byte table sits in LDS and
// every lane owns 8 tokens (one in each of its wavefront's 8 slices of 64).  A first look
// settles most tokens with one instruction or one table look-up each (which one depends on the
// table: all bytes stay by the token's byte signature, rejected by the first byte, or the first
// 8 bytes through the table); the rest are queued in LDS and finished byte by byte on full
// wavefronts.  Rows and exit entries are assembled in LDS and leave in whole runs; the places of
// the entries in the global lists are taken with four atomics per workgroup.

// Classifies up to 8 bytes of one chunk.  Returns true once the token is decided.
__device__ __forceinline__ bool scan_chunk(const uint8_t *lut, uint64_t cb, uint32_t L, uint32_t k,
                                           uint32_t &res, uint32_t &j)
{
    const uint32_t lo = (uint32_t)cb, hi = (uint32_t)(cb >> 32);
    uint32_t code = 0;
#pragma unroll
    for (int i = 0; i < 4; i++) {
        code |= (uint32_t)lut[(lo >> (8 * i)) & 0xFFu] << (2 * i);
        code |= (uint32_t)lut[(hi >> (8 * i)) & 0xFFu] << (2 * i + 8);
    }
    const uint32_t nvalid = L - 8u * k < 8u ? L - 8u * k : 8u;
    const uint32_t x = code ^ 0x5555u;               // a 2-bit field is 0 iff its byte stays
    const uint32_t mm = (x | (x >> 1)) & 0x5555u & ((1u << (2u * nvalid)) - 1u);
    if (mm) {
        const uint32_t jj = (uint32_t)__builtin_ctz(mm) >> 1;
        j = 8u * k + jj;
        res = (code >> (2u * jj)) & 3u;              // 0 reject, 2 / 3 exit
        return true;
    }
    if (L <= 8u * k + 8u) { res = 1u; return true; } // every byte stays
    return false;
}

// Appends the early exits of a wavefront's tokens to the workgroup's staging list in LDS: those
// with a short remainder from the front, the others from the back (a token leaves at most one
// entry, so the two ends cannot meet); one LDS atomic per wavefront and end.
__device__ __forceinline__ void stage_entry(uint2 *ent, uint32_t *n_ent, bool early, uint32_t tok, uint32_t nx,
                                            uint32_t res, uint32_t first, uint32_t rem)
{
    const uint32_t lane = threadIdx.x & 63u;
    const bool is_long = rem > kShortRem;
    const unsigned long long bx = __ballot(early && !is_long), by = __ballot(early && is_long);
    if (!(bx | by)) return;
    uint32_t b0 = 0, b1 = 0;
    if (lane == 0) {
        if (bx) b0 = atomicAdd(&n_ent[0], (uint32_t)__popcll(bx));
        if (by) b1 = atomicAdd(&n_ent[1], (uint32_t)__popcll(by));
    }
    b0 = __shfl(b0, 0); b1 = __shfl(b1, 0);
    if (early) {
        const uint32_t rank = (uint32_t)__popcll((is_long ? by : bx) & ((1ull << lane) - 1ull));
        ent[is_long ? kScanGroup - 1u - (b1 + rank) : b0 + rank] = uint2{tok, nx | res << 8 | first << 16 | rem << 24};
    }
}

constexpr uint32_t kScanThreads = 256;
constexpr uint32_t kScanWgs = 5;          // workgroups of class_scan a compute unit holds (its registers)
constexpr uint32_t kScanPer = kScanGroup / kScanThreads;     // tokens per lane of class_scan
static_assert(kScanPer * kScanThreads == kScanGroup, "a lane owns a whole number of tokens");

__global__ void __launch_bounds__(kScanThreads) __attribute__((amdgpu_waves_per_eu(5, 8)))
class_scan_kernel(DeviceTable T, DeviceVocab Vc, DeviceCache Cc)
{
    __shared__ __attribute__((aligned(16))) uint8_t lut[256];
    __shared__ uint32_t row_s[kScanGroup / 32u], row_e[kScanGroup / 32u];   // the group's words of the two rows
    __shared__ uint2 ent[kScanGroup];                // early exits of the group, from both ends
    __shared__ uint16_t que[kScanGroup];             // tokens (by their place in the group) the first look did not decide
    __shared__ uint32_t n_ent[2], n_que;
    __shared__ uint32_t list_base[2][2];             // where this workgroup's entries start in the two lists
    const uint32_t n = Cc.ctr->n_class_miss;
    const uint32_t groups = (Vc.V + kScanGroup - 1u) / kScanGroup;
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6, tid = threadIdx.x;
    const uint32_t V = Vc.V;
    // Workgroups are handed to the 8 XCDs round-robin and each XCD has its own L2.  XCD x takes
    // the token groups g with g % 8 == x for every class table, so a group's bytes are fetched
    // into one L2 once and then shared by all tables, instead of once per XCD.
    const uint32_t nx = gridDim.x < kXcds ? gridDim.x : kXcds;           // a tiny grid uses fewer
    const uint32_t xcd = blockIdx.x % nx, local = blockIdx.x / nx;
    const uint32_t local_wgs = (gridDim.x - xcd + nx - 1u) / nx;         // workgroups on this XCD
    const uint32_t my_groups = groups > xcd ? (groups - xcd + nx - 1u) / nx : 0u;
    // Work item = (class table ci of the call's list, token group) with the table index in the
    // upper part, so that which list entry a workgroup reads first depends on its place in the
    // grid only: it is requested together with the length of the list, not after it.
    const uint64_t total = (uint64_t)n * my_groups;
    const uint32_t ci_first = my_groups ? local / my_groups : 0u;
    const uint32_t c_first = Cc.class_miss[ci_first < Cc.miss_cap ? ci_first : 0u];   // the list has miss_cap places
    for (uint64_t item = local; item < total; item += local_wgs) {
        const uint32_t ci = (uint32_t)(item / my_groups);
        const uint32_t g = (uint32_t)(item % my_groups) * nx + xcd;
        // What the first look needs of a token does not depend on the table: the signatures and
        // first bytes of the lane's tokens are requested before the table is known.  A lane owns
        // kScanPer tokens, one in each of its wavefront's slices of 64, so that a ballot over a
        // slice is two words of a row.
        unsigned long long sg[kScanPer];
        uint32_t fb[kScanPer];
#pragma unroll
        for (uint32_t s = 0; s < kScanPer; s++) {
            const uint32_t tk = g * kScanGroup + (wave * kScanPer + s) * 64u + lane;
            sg[s] = tk < V ? Vc.sig[tk] : 0ull;
            fb[s] = tk < V ? Vc.first8[tk] : 0u;
        }
        const uint32_t c = item == local ? c_first : Cc.class_miss[ci];
        uint32_t part = 0;
#pragma unroll
        for (uint32_t q = 1; q < kParts; q++) part += g * kScanGroup >= Vc.part_tok[q];
        __syncthreads();                             // the item before is done with the LDS
        if (tid < 64u)
            reinterpret_cast<uint32_t *>(lut)[tid] = reinterpret_cast<const uint32_t *>(T.classes + (size_t)c * 256u)[tid];
        if (tid < kScanGroup / 32u) row_e[tid] = 0;
        if (tid == 0) { n_ent[0] = 0; n_ent[1] = 0; n_que = 0; }
        const uint32_t scan = T.class_info[c].scan;
        const unsigned long long nonstay = T.class_info[c].nonstay;
        __syncthreads();
        // First look, every token.  It settles the tokens whose bytes all stay (a table where
        // nearly every byte value stays: none of the token's bytes folds onto one that does not),
        // the tokens rejected by their first byte (a table that rejects most byte values), or what
        // the first 8 bytes settle without leaving an exit entry; every other token is queued,
        // so that the byte-by-byte work runs on full wavefronts.
        unsigned long long qm[kScanPer];             // per slice: the lanes whose token is queued
        uint32_t n_mine = 0;                         // queued tokens of this wavefront
#pragma unroll
        for (uint32_t s = 0; s < kScanPer; s++) {
            const uint32_t tk = g * kScanGroup + (wave * kScanPer + s) * 64u + lane;
            const bool valid = tk < V;
            bool stays = false, ends = false, queued = false;
            if (scan == SCAN_SIG) {
                queued = valid && (sg[s] & nonstay) != 0ull;
                stays = valid && !queued;
            } else if (scan == SCAN_HEAD) {
                queued = valid && lut[fb[s]] != CLS_REJECT;
            } else if (valid) {
                const uint32_t L = Vc.len8[tk];
                uint32_t res = 0, j = 0;
                const bool decided = L == 0u || scan_chunk(lut, Vc.chunks[tk], L, 0, res, j);
                stays = decided && res == 1u;
                ends = decided && res >= 2u && j + 1u == L;
                queued = !decided || (res >= 2u && j + 1u < L);
            }
            const unsigned long long bs = __ballot(stays), be = __ballot(ends);
            if (lane == 0) {
                row_s[(wave * kScanPer + s) * 2u] = (uint32_t)bs; row_s[(wave * kScanPer + s) * 2u + 1u] = (uint32_t)(bs >> 32);
                if (be) { row_e[(wave * kScanPer + s) * 2u] = (uint32_t)be; row_e[(wave * kScanPer + s) * 2u + 1u] = (uint32_t)(be >> 32); }
            }
            qm[s] = __ballot(queued);
            n_mine += (uint32_t)__popcll(qm[s]);
        }
        {
            // the wavefront's queued tokens take their places together: one LDS atomic, then a
            // token's place is the wavefront's first place, plus the queued tokens of the slices
            // before, plus the queued lanes below in its own slice
            uint32_t qb = 0;
            if (lane == 0 && n_mine) qb = atomicAdd(&n_que, n_mine);
            qb = __shfl(qb, 0);
#pragma unroll
            for (uint32_t s = 0; s < kScanPer; s++) {
                if ((qm[s] >> lane) & 1ull)
                    que[qb + (uint32_t)__popcll(qm[s] & ((1ull << lane) - 1ull))] = (uint16_t)((wave * kScanPer + s) * 64u + lane);
                qb += (uint32_t)__popcll(qm[s]);
            }
        }
        __syncthreads();
        // Second look: the queued tokens byte by byte, one per thread and round.
        const uint32_t nq = n_que;
        for (uint32_t i0 = 0; i0 < nq; i0 += kScanThreads) {
            const bool act = i0 + tid < nq;
            const uint32_t idx = que[act ? i0 + tid : 0u];
            const uint32_t tok = g * kScanGroup + idx;           // below V
            const uint32_t Lq = act ? Vc.len8[tok] : 0u;
            // (all three chunks are requested at once, whatever the length: no load waits for another)
            const uint64_t d0 = Vc.chunks[tok];
            const uint64_t d1 = Vc.chunks[(Vc.n_chunks > 1u ? (size_t)V : 0u) + tok];
            const uint64_t d2 = Vc.chunks[(Vc.n_chunks > 2u ? 2ull * V : 0ull) + tok];
            uint32_t res = 0, j = 0;
            if (Lq) {
                bool decided = scan_chunk(lut, d0, Lq, 0, res, j);
                if (!decided) decided = scan_chunk(lut, d1, Lq, 1, res, j);
                if (!decided) decided = scan_chunk(lut, d2, Lq, 2, res, j);
                for (uint32_t k = 3; k < Vc.n_chunks && !decided; k++)
                    decided = scan_chunk(lut, Vc.chunks[(size_t)k * V + tok], Lq, k, res, j);
            }
            const bool exits = res >= 2u;
            if (res == 1u) atomicOr(&row_s[idx >> 5], 1u << (idx & 31u));
            if (exits && j + 1u == Lq) atomicOr(&row_e[idx >> 5], 1u << (idx & 31u));
            const uint32_t nxt = j + 1u;
            const bool early = exits && nxt < Lq;
            uint32_t first = 0;
            if (early) {
                if (nxt < 24u) {
                    const uint64_t cw = nxt < 8u ? d0 : nxt < 16u ? d1 : d2;
                    first = (uint32_t)(cw >> (8u * (nxt & 7u))) & 0xFFu;
                } else first = Vc.bytes[Vc.offsets[tok] + nxt];
            }
            stage_entry(ent, n_ent, early, tok, nxt, res, first, Lq - nxt);
        }
        __syncthreads();
        // Out: the workgroup's entries go to two lists, the one of the whole class table (first V
        // slots of the class's buffer), read by keys that are built by one workgroup, and the one
        // of its token range (second V slots, range p owning [V + part_tok[p], V + part_tok[p+1])),
        // read by the work items of keys that are cut by range; short remainders fill a list from
        // the front, long ones from the back, so that a wavefront of key_build walks remainders of
        // similar length.  The four places are taken with four atomics that are in flight together.
        const uint32_t n_short = n_ent[0], n_long = n_ent[1];
        if (tid < 4u) {
            const uint32_t side = tid & 1u, which = tid >> 1;              // which: 0 class, 1 range
            const uint32_t cnt = side ? n_long : n_short;
            const uint32_t ctr = which ? 2u + 2u * part + side : side;
            list_base[which][side] = cnt ? atomicAdd(&Cc.class_count[c * kCountStride + ctr], cnt) : 0u;
        }
        __syncthreads();
        uint2 *out = reinterpret_cast<uint2 *>(Cc.class_entries[c]);
        const uint32_t out_lo = V + Vc.part_tok[part], out_hi = V + Vc.part_tok[part + 1u];
        for (uint32_t i = tid; i < n_short; i += kScanThreads) {
            const uint2 e = ent[i];
            out[list_base[0][0] + i] = e;
            out[out_lo + list_base[1][0] + i] = e;
        }
        for (uint32_t i = tid; i < n_long; i += kScanThreads) {
            const uint2 e = ent[kScanGroup - 1u - i];
            out[V - 1u - (list_base[0][1] + i)] = e;
            out[out_hi - 1u - (list_base[1][1] + i)] = e;
        }
        // the three rows of the class index: all bytes stay, exit on the last byte, and their union
        if (tid < kScanGroup / 32u) {
            const uint32_t w = g * (kScanGroup / 32u) + tid;
            if (w < Vc.W) {
                uint32_t *rows = Cc.class_rows + (size_t)(3u * c) * Cc.row_stride;
                const uint32_t a = row_s[tid], b = row_e[tid];
                rows[w] = a; rows[Cc.row_stride + w] = b; rows[2u * Cc.row_stride + w] = a | b;
            }
        }
    }
    if (blockIdx.x == 0 && threadIdx.x == 0 && n) atomicAdd(&Cc.ctr->class_scans, (unsigned long long)n);
}

// ---------------------------------------------------------------------------------------------
// class_scan for a call that brings many class tables: a workgroup takes a 2048-token group
// through up to kScanBatch tables together.  What a table-by-table pass pays once per table --
// the chain first look -> queue -> byte-by-byte look -> list places -> stores, each link a trip
// to memory -- is paid once per batch, and the byte-by-byte look runs on the queued tokens of
// all the batch's tables, so on full wavefronts.
//
// The first look takes 32 tokens at a time, from the vocabulary's rows by byte value: the tokens
// that contain a byte which does not stay are the OR of the rows of those bytes, and every other
// token with bytes is all-stay; of the former, the tokens whose first byte is not rejected (an OR
// of first-byte rows, of the rejected bytes and complemented when those are fewer) are queued,
// the others are rejected by their first byte.  A side with more than kScanRowsMax rows lets
// every token through instead, which costs work, not correctness: the queue may hold any token,
// the byte-by-byte look decides.  That look has two stages: the first 8 bytes of every queued
// token, then the longer tokens those 8 bytes did not decide, queued again so that they too fill
// their wavefronts.
// Results are the ones class_scan_kernel leaves (rows, lists, counters); the order of entries
// inside a list differs, which no reader depends on.
constexpr uint32_t kScanBatch = 8;        // class tables of one work item
constexpr uint32_t kScanQueue = 4096;     // places of the queue for the byte-by-byte look
constexpr uint32_t kScanLong = 1024;      // places of the queue for its second stage
constexpr uint32_t kScanStage = 768;      // exit entries held in LDS before they leave
constexpr uint32_t kScanRowsMax = 64;     // most rows ORed for one side of a table's first look
constexpr uint32_t kScanRowsUnroll = 8;   // rows a wavefront requests together
constexpr uint32_t kScanFixed = 3;        // what a work item costs before its first table, in tables
constexpr uint32_t kScanBatchWgs = 5;     // workgroups of this kernel a compute unit holds (its LDS and registers)
constexpr uint32_t kScanBatchFrom = 4096; // (class tables of a handle) x (token groups) above which it takes this kernel
static_assert(kScanBatch <= 8u && kScanGroup <= 2048u, "a queue place holds table and token in 14 bits");
static_assert(kScanStage <= 4096u && kScanThreads <= kScanStage, "the rank of a staged entry has 12 bits; a round's entries fit");
static_assert(kScanThreads <= kScanLong && kScanGroup <= kScanQueue, "a round fits the second queue, a table's tokens the first");

__global__ void __launch_bounds__(kScanThreads) __attribute__((amdgpu_waves_per_eu(5, 8)))
class_scan_batch_kernel(DeviceTable T, DeviceVocab Vc, DeviceCache Cc)
{
    __shared__ __attribute__((aligned(16))) uint8_t lut[kScanBatch][256];
    __shared__ uint32_t row_s[kScanBatch][kScanGroup / 32u], row_e[kScanBatch][kScanGroup / 32u];
    __shared__ uint2 ent[kScanStage];                // early exits of the batch's tables, in the order found
    __shared__ uint16_t meta[kScanStage];            // of a staged entry: table | long << 3 | rank in (table, side) << 4
    __shared__ uint16_t que[kScanQueue];             // table << 11 | the token's place in the group
    __shared__ uint16_t que_long[kScanLong];         // the same, tokens the first 8 bytes did not decide
    __shared__ uint32_t acc[kScanBatch][2][kScanGroup / 32u];   // the ORs of the first look: [0] has a byte that does not stay, [1] by first byte
    __shared__ uint16_t row_list[kScanBatch * 2u * kScanRowsMax];   // the rows to OR: table << 9 | row of byte_rows
    __shared__ uint8_t first_inv[kScanBatch];        // the first-byte OR is of the rejected bytes
    __shared__ uint32_t cls_s[kScanBatch];
    __shared__ uint32_t n_ent[kScanBatch][2], list_base[kScanBatch][2][2];
    __shared__ uint32_t n_rows, n_que, n_long, n_stage;
    const uint32_t n = Cc.ctr->n_class_miss;
    if (n == 0) return;
    const uint32_t groups = (Vc.V + kScanGroup - 1u) / kScanGroup;
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6, tid = threadIdx.x;
    const uint32_t V = Vc.V;
    // how many of the lanes before this one are set in a ballot
    auto before = [](unsigned long long bal) {
        return (uint32_t)__builtin_amdgcn_mbcnt_hi((uint32_t)(bal >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0u));
    };
    // (the same hand-out of token groups to XCDs as in class_scan_kernel)
    const uint32_t nx = gridDim.x < kXcds ? gridDim.x : kXcds;
    const uint32_t xcd = blockIdx.x % nx, local = blockIdx.x / nx;
    const uint32_t local_wgs = (gridDim.x - xcd + nx - 1u) / nx;
    const uint32_t my_groups = groups > xcd ? (groups - xcd + nx - 1u) / nx : 0u;
    // Tables per work item.  The launch is one workgroup per place the chip has for this kernel,
    // and a workgroup takes every local_wgs-th item of its XCD; an item costs a fixed part (the
    // trips to memory of its chain) and a part per table.  The number of tables is the one under
    // which the busiest XCD is done soonest by that count.
    uint32_t per = Cc.scan_batch;
    if (!per) {
        const uint32_t most_groups = (groups + nx - 1u) / nx, fewest_wgs = gridDim.x / nx ? gridDim.x / nx : 1u;
        uint32_t best = 0xFFFFFFFFu;
        for (uint32_t p = 1; p <= kScanBatch; p++) {
            const uint64_t wide = (uint64_t)((n + p - 1u) / p) * most_groups;
            const uint32_t items = wide > 0x7FFFFFFFull ? 0x7FFFFFFFu : (uint32_t)wide;
            const uint32_t cost = ((items + fewest_wgs - 1u) / fewest_wgs) * (kScanFixed + p);
            if (cost < best) { best = cost; per = p; }
        }
    }
    per = per < 1u ? 1u : per > kScanBatch ? kScanBatch : per;
    const uint32_t batches = (n + per - 1u) / per;
    const uint64_t total = (uint64_t)batches * my_groups;
    for (uint64_t item = local; item < total; item += local_wgs) {
        const uint32_t t0 = (uint32_t)(item / my_groups) * per;
        const uint32_t nt = n - t0 < per ? n - t0 : per;
        const uint32_t g = (uint32_t)(item % my_groups) * nx + xcd;
        // the tokens of this thread's word of the group that have bytes (none beyond V)
        const uint32_t word_hb = g * (kScanGroup / 32u) + (tid >> 2);
        const uint32_t has_bytes = word_hb < Vc.row_stride ? Vc.len_rows[(size_t)(Vc.lmax + 1u) * Vc.row_stride + word_hb] : 0u;
        uint32_t part = 0;
#pragma unroll
        for (uint32_t q = 1; q < kParts; q++) part += g * kScanGroup >= Vc.part_tok[q];
        const uint32_t out_lo = V + Vc.part_tok[part], out_hi = V + Vc.part_tok[part + 1u];
        if (tid == 0) { n_rows = 0; n_que = 0; n_long = 0; n_stage = 0; }   // (the item before is past their last use)
        __syncthreads();                             // the item before is done with the LDS
        // The tables come in, a wavefront one table at a time, a lane 4 of its byte values; what
        // the lanes see of the table says which rows its first look ORs.
        for (uint32_t i = tid; i < nt * 64u; i += kScanThreads) {
            const uint32_t t = i >> 6;               // (the same for the whole wavefront)
            const uint32_t c = Cc.class_miss[t0 + t];
            const uint32_t cw = reinterpret_cast<const uint32_t *>(T.classes + (size_t)c * 256u)[lane];
            reinterpret_cast<uint32_t *>(lut[t])[lane] = cw;
            unsigned long long moves[4], lives[4];   // per byte value 4 * lane + k: does not stay / is not rejected
            uint32_t n_moves = 0, n_lives = 0;
#pragma unroll
            for (uint32_t k = 0; k < 4u; k++) {
                const uint32_t cl = (cw >> (8u * k)) & 0xFFu;
                moves[k] = __ballot(cl != CLS_STAY);
                lives[k] = __ballot(cl != CLS_REJECT);
                n_moves += (uint32_t)__popcll(moves[k]);
                n_lives += (uint32_t)__popcll(lives[k]);
            }
            const bool all_a = n_moves > kScanRowsMax;
            const bool inv = n_lives > kScanRowsMax, all_b = inv && 256u - n_lives > kScanRowsMax;
            const uint32_t cnt_a = all_a ? 0u : n_moves, cnt_b = all_b ? 0u : inv ? 256u - n_lives : n_lives;
            row_e[t][lane] = 0;
            acc[t][0][lane] = all_a ? 0xFFFFFFFFu : 0u;
            acc[t][1][lane] = all_b ? 0xFFFFFFFFu : 0u;
            uint32_t at = 0;
            if (lane == 0) {
                cls_s[t] = c; n_ent[t][0] = 0; n_ent[t][1] = 0; first_inv[t] = inv && !all_b;
                if (cnt_a + cnt_b) at = atomicAdd(&n_rows, cnt_a + cnt_b);
            }
            at = __shfl(at, 0);
#pragma unroll
            for (uint32_t k = 0; k < 4u; k++) {
                if (!all_a) {
                    if ((moves[k] >> lane) & 1ull)
                        row_list[at + before(moves[k])] = (uint16_t)(t << 9 | (4u * lane + k));
                    at += (uint32_t)__popcll(moves[k]);
                }
            }
#pragma unroll
            for (uint32_t k = 0; k < 4u; k++) {
                if (!all_b) {
                    const unsigned long long pick = inv ? ~lives[k] : lives[k];
                    if ((pick >> lane) & 1ull)
                        row_list[at + before(pick)] = (uint16_t)(t << 9 | 256u | (4u * lane + k));
                    at += (uint32_t)__popcll(pick);
                }
            }
        }
        __syncthreads();

        uint32_t stage_bound = 0, que_bound = 0, long_bound = 0;   // no fewer than n_stage / n_que / n_long, known without a look
        // The staged entries leave: per table and side, a run in the list of the whole table and a
        // run in the list of the token range, their places taken with one atomic each.
        // (Called by the whole workgroup, after a barrier that follows the last staged entry.)
        auto flush = [&]() {
            const uint32_t ns = n_stage;
            if (tid < nt * 4u) {
                const uint32_t t = tid >> 2, side = tid & 1u, which = (tid >> 1) & 1u;
                const uint32_t cnt = n_ent[t][side];
                const uint32_t ctr = which ? 2u + 2u * part + side : side;
                list_base[t][which][side] = cnt ? atomicAdd(&Cc.class_count[cls_s[t] * kCountStride + ctr], cnt) : 0u;
            }
            __syncthreads();
            for (uint32_t i = tid; i < ns; i += kScanThreads) {
                const uint2 e = ent[i];
                const uint32_t m = meta[i], t = m & 7u, r = m >> 4;
                uint2 *out = reinterpret_cast<uint2 *>(Cc.class_entries[cls_s[t]]);
                if (!(m & 8u)) {
                    out[list_base[t][0][0] + r] = e;
                    out[out_lo + list_base[t][1][0] + r] = e;
                } else {
                    out[V - 1u - (list_base[t][0][1] + r)] = e;
                    out[out_hi - 1u - (list_base[t][1][1] + r)] = e;
                }
            }
            __syncthreads();
            if (tid < nt * 2u) n_ent[tid >> 1][tid & 1u] = 0;
            if (tid == 0) n_stage = 0;
            stage_bound = 0;
            __syncthreads();
        };
        // Room in the staging list for the entries of one more round (every thread takes the same way).
        auto stage_room = [&]() {
            if (stage_bound + kScanThreads > kScanStage) {
                // count exactly, between two barriers so that every thread reads the same number
                __syncthreads();
                const uint32_t staged = n_stage;
                __syncthreads();
                if (staged + kScanThreads > kScanStage) flush();
                else stage_bound = staged;
            }
            stage_bound += kScanThreads;
        };
        // What the byte-by-byte look found for a token goes to the rows and the staging list: the
        // first byte that does not stay is byte j with class res (1: none, all bytes stay).
        auto settle = [&](uint32_t t, uint32_t idx, uint32_t tok, uint32_t Lq, uint32_t res, uint32_t j, uint32_t first) {
            const bool exits = res >= 2u;
            if (res == 1u) atomicOr(&row_s[t][idx >> 5], 1u << (idx & 31u));
            if (exits && j + 1u == Lq) atomicOr(&row_e[t][idx >> 5], 1u << (idx & 31u));
            const uint32_t nxt = j + 1u;
            const bool early = exits && nxt < Lq;
            const unsigned long long be = __ballot(early);
            if (!be) return;
            uint32_t base = 0;
            if (lane == 0) base = atomicAdd(&n_stage, (uint32_t)__popcll(be));
            base = __shfl(base, 0);
            if (early) {
                const uint32_t rem = Lq - nxt, side = rem > kShortRem;
                const uint32_t r = atomicAdd(&n_ent[t][side], 1u);
                const uint32_t at = base + before(be);
                ent[at] = uint2{tok, nxt | res << 8 | first << 16 | rem << 24};
                meta[at] = (uint16_t)(t | side << 3 | r << 4);
            }
        };
        // Second stage: the tokens longer than 8 bytes whose first 8 all stay, from byte 8 on.
        // (Called by the whole workgroup, after a barrier that follows the last write to its queue.)
        auto drain_long = [&]() {
            const uint32_t nl = n_long;
            __syncthreads();                         // every thread has read the length
            for (uint32_t i0 = 0; i0 < nl; i0 += kScanThreads) {
                stage_room();
                if (i0 + wave * 64u >= nl) continue;                    // nothing for this wavefront in the last round
                const bool act = i0 + tid < nl;
                const uint32_t q = que_long[act ? i0 + tid : 0u];
                const uint32_t t = q >> 11, idx = q & (kScanGroup - 1u);
                const uint32_t tok = g * kScanGroup + idx;               // below V
                const uint32_t Lq = act ? Vc.len8[tok] : 0u;             // above 8
                const uint64_t d1 = Vc.chunks[(Vc.n_chunks > 1u ? (size_t)V : 0u) + tok];
                const uint64_t d2 = Vc.chunks[(Vc.n_chunks > 2u ? 2ull * V : 0ull) + tok];
                uint32_t res = 0, j = 0;
                if (Lq) {
                    bool decided = scan_chunk(lut[t], d1, Lq, 1, res, j);
                    if (!decided) decided = scan_chunk(lut[t], d2, Lq, 2, res, j);
                    for (uint32_t k = 3; k < Vc.n_chunks && !decided; k++)
                        decided = scan_chunk(lut[t], Vc.chunks[(size_t)k * V + tok], Lq, k, res, j);
                }
                uint32_t first = 0;
                if (res >= 2u && j + 1u < Lq) {
                    const uint32_t nxt = j + 1u;
                    if (nxt < 24u) first = (uint32_t)((nxt < 16u ? d1 : d2) >> (8u * (nxt & 7u))) & 0xFFu;
                    else first = Vc.bytes[Vc.offsets[tok] + nxt];
                }
                settle(t, idx, tok, Lq, res, j, first);
            }
            __syncthreads();                         // the rounds are over
            if (tid == 0) n_long = 0;
            long_bound = 0;
            __syncthreads();
        };
        // First stage: the first 8 bytes of every queued token, one token per thread and round.
        // (Called by the whole workgroup, after a barrier that follows the last write to the queue.)
        auto drain = [&]() {
            const uint32_t nq = n_que;
            __syncthreads();                         // every thread has read the length
            // what a round needs of its tokens is requested a round ahead, so that the trip to
            // memory of one round runs under the work of the round before
            uint32_t q_next = 0, L_next = 0;
            uint64_t d_next = 0;
            auto request = [&](uint32_t i0) {
                const bool act = i0 + tid < nq;
                q_next = que[act ? i0 + tid : 0u];
                const uint32_t tok = g * kScanGroup + (q_next & (kScanGroup - 1u));   // below V
                L_next = act ? Vc.len8[tok] : 0u;
                d_next = Vc.chunks[tok];
            };
            if (nq) request(0u);
            for (uint32_t i0 = 0; i0 < nq; i0 += kScanThreads) {
                if (long_bound + kScanThreads > kScanLong) {
                    // the second queue may be short of room for a round: count exactly, empty it if need be
                    __syncthreads();
                    const uint32_t waiting = n_long;
                    __syncthreads();
                    if (waiting + kScanThreads > kScanLong) drain_long();
                    else long_bound = waiting;
                }
                long_bound += kScanThreads;
                stage_room();                        // (after the second stage may have run: it stages entries too)
                const uint32_t q = q_next, Lq = L_next;
                const uint64_t d0 = d_next;
                if (i0 + kScanThreads < nq) request(i0 + kScanThreads);
                if (i0 + wave * 64u >= nq) continue;                    // nothing for this wavefront in the last round
                const uint32_t t = q >> 11, idx = q & (kScanGroup - 1u);
                const uint32_t tok = g * kScanGroup + idx;
                uint32_t res = 0, j = 0;
                const bool decided = Lq == 0u || scan_chunk(lut[t], d0, Lq, 0, res, j);
                // undecided: to the second queue
                const unsigned long long bu = __ballot(!decided);
                if (bu) {
                    uint32_t base = 0;
                    if (lane == 0) base = atomicAdd(&n_long, (uint32_t)__popcll(bu));
                    base = __shfl(base, 0);
                    if (!decided) que_long[base + before(bu)] = (uint16_t)q;
                }
                uint32_t first = 0;
                if (decided && res >= 2u && j + 1u < Lq) {
                    const uint32_t nxt = j + 1u;     // at most 8
                    first = nxt < 8u ? (uint32_t)(d0 >> (8u * nxt)) & 0xFFu : (uint32_t)Vc.chunks[(size_t)V + tok] & 0xFFu;
                }
                settle(t, idx, tok, decided ? Lq : 0u, decided ? res : 0u, j, first);
            }
            __syncthreads();                         // the rounds are over: the second queue is written
            if (tid == 0) n_que = 0;
            que_bound = 0;
            __syncthreads();
        };

        // First look, the ORs: a lane takes one word (32 tokens) of the group, a wavefront every
        // fourth stretch of kScanRowsUnroll rows of the list, requested together; the ORs meet in LDS.
        {
            const uint32_t gw = g * (kScanGroup / 32u) + lane;
            const bool in_row = gw < Vc.row_stride;
            const uint32_t nr = n_rows;
            for (uint32_t base = wave * kScanRowsUnroll; base < nr; base += 4u * kScanRowsUnroll) {
                uint32_t code[kScanRowsUnroll], x[kScanRowsUnroll];
#pragma unroll
                for (uint32_t u = 0; u < kScanRowsUnroll; u++) {
                    code[u] = row_list[base + u < nr ? base + u : base];
                    x[u] = in_row ? Vc.byte_rows[(size_t)(code[u] & 511u) * Vc.row_stride + gw] : 0u;
                }
#pragma unroll
                for (uint32_t u = 0; u < kScanRowsUnroll; u++)
                    if (base + u < nr && x[u]) atomicOr(&acc[code[u] >> 9][(code[u] >> 8) & 1u][lane], x[u]);
            }
        }
        __syncthreads();
        // First look, the tokens: a thread takes a byte of a word (8 tokens): all-stay tokens go to
        // the row, queued ones take their places in the queue.
        for (uint32_t t = 0; t < nt; t++) {
            if (que_bound + kScanGroup > kScanQueue) {
                // the queue may be short of room for a whole group: count exactly, empty it if need be
                __syncthreads();
                const uint32_t waiting = n_que;
                __syncthreads();
                if (waiting + kScanGroup > kScanQueue) drain();
                else que_bound = waiting;
            }
            que_bound += kScanGroup;
            const uint32_t wd = tid >> 2, bi = tid & 3u;
            const uint32_t a = acc[t][0][wd];
            const uint32_t b = first_inv[t] ? ~acc[t][1][wd] : acc[t][1][wd];
            if (bi == 0) row_s[t][wd] = ~a & has_bytes;
            const uint32_t mine = ((a & b & has_bytes) >> (8u * bi)) & 0xFFu;
            // places in the queue: one LDS atomic per wavefront; a token's place follows from the
            // ballots of the 8 token positions of a thread
            unsigned long long bal[8];
            uint32_t n_mine = 0;
#pragma unroll
            for (uint32_t j = 0; j < 8u; j++) {
                bal[j] = __ballot((mine >> j) & 1u);
                n_mine += (uint32_t)__popcll(bal[j]);
            }
            uint32_t at = 0;
            if (lane == 0 && n_mine) at = atomicAdd(&n_que, n_mine);
            at = __shfl(at, 0);
#pragma unroll
            for (uint32_t j = 0; j < 8u; j++) {
                if ((mine >> j) & 1u)
                    que[at + before(bal[j])] = (uint16_t)(t << 11 | (wd * 32u + bi * 8u + j));
                at += (uint32_t)__popcll(bal[j]);
            }
        }
        __syncthreads();
        drain();
        drain_long();
        if (n_stage) flush();                        // (read behind the barrier that ends drain_long, the same for every thread)
        for (uint32_t i = tid; i < nt * (kScanGroup / 32u); i += kScanThreads) {
            const uint32_t t = i / (kScanGroup / 32u), wd = i % (kScanGroup / 32u);
            const uint32_t w = g * (kScanGroup / 32u) + wd;
            if (w < Vc.W) {
                uint32_t *rows = Cc.class_rows + (size_t)(3u * cls_s[t]) * Cc.row_stride;
                const uint32_t a = row_s[t][wd], b = row_e[t][wd];
                rows[w] = a; rows[Cc.row_stride + w] = b; rows[2u * Cc.row_stride + w] = a | b;
            }
        }
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) atomicAdd(&Cc.ctr->class_scans, (unsigned long long)n);
}

// ---------------------------------------------------------------------------------------------
// key_build: a workgroup assembles the mask row of a missing state key in LDS -- or, for a key
// whose candidates all need a deep walk, its words for one of the kParts token ranges, so that
// such a key is shared among kParts workgroups instead of holding up the whole launch:
//   (a) the context-free part from the class index (budget-limited through the per-length
//       rows of the vocabulary), zeros for a literal / END / FINAL state;
//   (b) the tokens that leave the state early (exit list of the class table, or the
//       first-byte buckets of a literal state): first all of them are filtered, then the rest
//       of each survivor is walked from the successor state, and an accepted token sets its bit
//       with an LDS atomic.  The two possible successors are workgroup-uniform, so their
//       descriptors and class tables are staged in LDS and the first hop of every walk runs out
//       of LDS and registers; only a token that leaves the successor as well continues through
//       the table in HBM;
//   (c) the EOS bit, then the words go to the cache arena.
__device__ __forceinline__ uint32_t token_byte(uint64_t c0, uint64_t c1, uint64_t c2, uint32_t i)
{
    const uint64_t cw = i < 8u ? c0 : i < 16u ? c1 : c2;
    return (uint32_t)(cw >> (8u * (i & 7u))) & 0xFFu;
}

// Walks bytes [i, L) of a token held in registers (L <= 24) from the staged successor; hands
// over to walk_chunks when the token moves on to a third state.
__device__ __forceinline__ bool walk_first_hop(const DeviceTable &T, const HopState &h,
                                               const uint8_t *lut, uint64_t c0, uint64_t c1, uint64_t c2, uint32_t i, uint32_t L)
{
    uint32_t sid, aux = 0;
    if (h.kind == WG_KIND_LIT) {
        if (token_byte(c0, c1, c2, i) != h.lit) return false;
        sid = h.next_a; i++;
    } else if (h.kind == WG_KIND_WAIT || h.kind == WG_KIND_COND) {
        for (;;) {
            if (i >= L) return true;
            const uint32_t c = lut[token_byte(c0, c1, c2, i)];
            i++;
            if (c == CLS_STAY) {
                if (h.max != WG_UNBOUNDED) { if (aux >= h.max) return false; aux++; }
                continue;
            }
            if (c == CLS_EXIT_A) { sid = h.next_a; break; }
            if (c == CLS_EXIT_B) { sid = h.next_b; break; }
            return false;
        }
        aux = 0;
    } else return false;
    return walk_chunks(T, sid, aux, c0, c1, c2, i, L);
}

// True iff the first n bytes of a token held in registers (n <= 24) all stay in the checkpoint
// whose class table is `lut`.
__device__ __forceinline__ bool stays_prefix(const uint8_t *lut, uint64_t c0, uint64_t c1, uint64_t c2, uint32_t n)
{
    for (uint32_t i = 0; i < n; i++)
        if (lut[token_byte(c0, c1, c2, i)] != CLS_STAY) return false;
    return true;
}

constexpr uint32_t kKbThreads = 512;       // two workgroups per compute unit
constexpr uint32_t kKbSegs = 2u * kMaxExitBytes;   // index ranges a key of the direct paths reads (2 for KB_SORTED)
constexpr uint32_t kKbPer = 8;             // candidates a thread filters per pass
static_assert(kKbPer % 2u == 0u, "deep items take their candidates two at a time");
constexpr uint32_t kKbQueue = kKbThreads * kKbPer;   // candidates waiting for their walk: a whole pass fits (48 KB of LDS)
typedef __attribute__((address_space(1))) uint2 global_u2;   // a load known to go to device memory

// Walks what is left of a candidate token from the state its exit leads to.
__device__ __forceinline__ bool walk_candidate(const DeviceTable &T, const DeviceVocab &Vc, const MissEntry &me,
                                               const uint8_t (*hop_lut)[256], const ExitEntry &x, bool regs_ok,
                                               uint64_t c0)
{
    const int w = x.cls == CLS_EXIT_B;
    if (regs_ok) {
        const uint32_t L = (uint32_t)x.off + x.rem;
        const uint64_t c1 = L > 8u ? Vc.chunks[(size_t)Vc.V + x.tok] : 0ull;
        const uint64_t c2 = L > 16u ? Vc.chunks[2ull * Vc.V + x.tok] : 0ull;
        return walk_first_hop(T, me.hop[w], hop_lut[w], c0, c1, c2, x.off, L);
    }
    uint32_t sid = w ? me.next_b : me.next_a, aux = 0;
    return walk_bytes(T, sid, aux, Vc.bytes + Vc.offsets[x.tok] + x.off, x.rem);
}

__global__ void __launch_bounds__(kKbThreads) __attribute__((amdgpu_waves_per_eu(4, 4)))
key_build_kernel(DeviceTable T, DeviceVocab Vc, DeviceCache Cc, uint32_t *__restrict__ bitmask)
{
    extern __shared__ __attribute__((aligned(16))) uint32_t row[];
    __shared__ __attribute__((aligned(16))) uint8_t hop_lut[2][256];
    __shared__ __attribute__((aligned(16))) uint8_t own_lut[256];
    __shared__ uint2 queue[kKbQueue];
    __shared__ uint32_t queued[2];                   // candidates queued in the passes of even / odd number
    __shared__ uint32_t seg_at[kKbSegs], seg_len[kKbSegs];   // direct paths: the index ranges of the key
    // One sequence of work items for the whole grid: first the range items of the deep keys (front
    // of the miss list, kParts items per key), which take longest, then the plain keys (back of the
    // list), handed out round-robin.  Which miss entry a workgroup's first item reads is only
    // known once the counts have arrived; it is requested beforehand as if the item were a deep
    // one, and requested again if it turns out to be a plain one.
    const uint32_t n_deep = Cc.ctr->n_deep, n_plain = Cc.ctr->n_plain, n_claims = Cc.ctr->n_claims;
    const uint32_t rs = Cc.row_stride, tid = threadIdx.x, lane = tid & 63u;
    const bool regs_ok = Vc.lmax <= 24u;             // a whole token fits three 8-byte chunks
    const uint32_t n_deep_items = n_deep * kParts, n_items = n_deep_items + n_plain;
    auto entry_of = [&](uint32_t list, uint32_t item) {
        const uint32_t at = list == 0u ? item / kParts : Cc.miss_cap - 1u - item;
        return at < Cc.miss_cap ? at : 0u;
    };
    MissEntry me = Cc.miss[entry_of(0u, blockIdx.x)];
    {
    for (uint32_t unit = blockIdx.x; unit < n_items; unit += gridDim.x) {
        const uint32_t list = unit < n_deep_items ? 0u : 1u;
        const uint32_t item = list == 0u ? unit : unit - n_deep_items;
        if (unit != blockIdx.x || list == 1u) me = Cc.miss[entry_of(list, item)];
        const uint32_t kind = me.kind, r = me.r;
        const uint32_t p0 = list == 0u ? item % kParts : 0u, span = list == 0u ? 1u : kParts;
        // this item's words of the row, in 16-byte units
        const uint32_t q_lo = Vc.part_tok[p0] >> 7;
        const uint32_t q_hi = p0 + span == kParts ? rs / 4u : Vc.part_tok[p0 + span] >> 7;
        // Its candidate tokens, ents[i < n_front ? at_front + i : at_back + i - n_front]: the
        // first-byte buckets of a literal state (contiguous over these ranges), or the two-ended
        // list of a checkpoint's class table: the whole one, or the one of range p0.
        const ExitEntry *ents = nullptr;
        uint32_t cnt = 0, n_front = 0, at_front = 0, at_back = 0;
        const uint4 *stay = nullptr, *end = nullptr;
        const uint32_t mode = me.mode;
        const bool ckpt = kind == WG_KIND_WAIT || kind == WG_KIND_COND;
        if (kind == WG_KIND_LIT && mode == KB_LIST) {
            ents = Vc.lit_entries;
            at_front = Vc.lit_start[me.lit * kParts + p0];
            cnt = n_front = Vc.lit_start[me.lit * kParts + p0 + span] - at_front;
        } else if (ckpt) {
            if (mode == KB_LIST) {
                ents = Cc.class_entries[me.cls];
                const uint32_t *cc = Cc.class_count + me.cls * kCountStride + (span == kParts ? 0u : 2u + 2u * p0);
                n_front = cc[0];
                const uint32_t n_back = cc[1];
                cnt = n_front + n_back;
                at_front = span == kParts ? 0u : Vc.V + Vc.part_tok[p0];
                at_back = (span == kParts ? Vc.V : Vc.V + Vc.part_tok[p0 + 1u]) - n_back;
            }
            stay = reinterpret_cast<const uint4 *>(Cc.class_rows + (size_t)(3u * me.cls) * rs);
            end = stay + rs / 4u;
        }
        // the two possible successors: class tables staged in LDS for the first hop
#pragma unroll
        for (int w = 0; w < 2; w++)
            if ((me.hop[w].kind == WG_KIND_WAIT || me.hop[w].kind == WG_KIND_COND) && tid < 64u)
                reinterpret_cast<uint32_t *>(hop_lut[w])[tid] =
                    reinterpret_cast<const uint32_t *>(T.classes + (size_t)me.hop[w].cls * 256u)[tid];
        if (mode == KB_BIGRAM && tid >= 64u && tid < 128u)
            reinterpret_cast<uint32_t *>(own_lut)[tid - 64u] =
                reinterpret_cast<const uint32_t *>(T.classes + (size_t)me.cls * 256u)[tid - 64u];
        // Direct paths: the few index ranges that hold the key's candidates.  A literal state:
        // the token that is its byte alone, and the tokens that go on with the literal byte
        // after it (none when no byte can follow).  A checkpoint: for each exit byte e of a side
        // whose exit leads to a literal byte y, the places in the vocabulary where y follows e.
        uint32_t n_seg = 0;
        if (mode == KB_SORTED) n_seg = me.hop[0].kind == WG_KIND_LIT ? 2u : 1u;
        else if (mode == KB_BIGRAM) n_seg = (uint32_t)me.n_a + me.n_b;
        if (tid < n_seg) {
            const uint32_t *dir;
            uint32_t at;
            if (mode == KB_SORTED) { dir = Vc.dir0; at = me.lit * 257u + (tid ? 1u + me.hop[0].lit : 0u); }
            else {
                const uint32_t w = tid >= me.n_a, k = w ? kMaxExitBytes + tid - me.n_a : tid;
                const uint32_t word = k < 4u ? me.exits[0] : k < 8u ? me.exits[1] : me.exits[2];
                const uint32_t e = (word >> (8u * (k & 3u))) & 0xFFu;
                dir = Vc.dirN; at = (e << 8) | (w ? me.hop[1].lit : me.hop[0].lit);
            }
            const uint32_t lo = dir[at], hi = dir[at + 1u];
            seg_at[tid] = lo; seg_len[tid] = hi - lo;
        }
        if (tid == 0) { queued[0] = 0; queued[1] = 0; }
        // The first pass of candidates is requested before the row is set up, so that the loads
        // are under way while (a) runs: kKbPer per thread, plain 8-byte loads from clamped
        // indexes (a load inside a lane-dependent branch would be waited for on the spot).
        const global_u2 *ents2 = (const global_u2 *)(ents ? ents : Vc.lit_entries);
        // (an empty list still issues one load: from the first bucket entry, which always exists)
        if (cnt == 0u) { ents2 = (const global_u2 *)Vc.lit_entries; at_back = 0u; }
        uint2 x[kKbPer];
        auto request = [&](uint32_t i0) {
#pragma unroll
            for (uint32_t j = 0; j < kKbPer; j++) {
                uint32_t i = i0 + j * kKbThreads + tid;
                i = i < cnt ? i : (cnt ? cnt - 1u : 0u);
                const global_u2 *src = ents2 + (i < n_front ? at_front + i : at_back + (i - n_front));
                x[j] = uint2{src->x, src->y};
            }
        };
        request(0);
        // (a)
        uint4 *row4 = reinterpret_cast<uint4 *>(row);
        if (!stay) {
            for (uint32_t q = q_lo + tid; q < q_hi; q += kKbThreads) row4[q] = uint4{0u, 0u, 0u, 0u};
        } else if (r >= Vc.lmax) {
            const uint4 *both = end + rs / 4u;
            for (uint32_t q = q_lo + tid; q < q_hi; q += kKbThreads) row4[q] = both[q];
        } else {
            // r allow-bytes may still be consumed: all-stay tokens need length <= r, tokens
            // that exit on their last byte have length - 1 stay bytes
            const uint4 *l0 = reinterpret_cast<const uint4 *>(Vc.len_rows + (size_t)r * rs);
            const uint4 *l1 = l0 + rs / 4u;
            for (uint32_t q = q_lo + tid; q < q_hi; q += kKbThreads) {
                const uint4 a = stay[q], b = end[q], x = l0[q], y = l1[q];
                row4[q] = uint4{(a.x & x.x) | (b.x & y.x), (a.y & x.y) | (b.y & y.y),
                                (a.z & x.z) | (b.z & y.z), (a.w & x.w) | (b.w & y.w)};
            }
        }
        __syncthreads();
        // (b) The candidates, kKbThreads * kKbPer per pass.  (b1) filter: every candidate is
        // looked at once.  One that ends with its exit byte is accepted at once, one whose next
        // byte cannot start the literal that follows is dropped, the others wait in LDS for (b2)
        // their walk -- so that the walks, each a chain of dependent loads, run densely packed
        // instead of a few lanes of every wavefront holding the others up.
        uint32_t examined = 0;
        if (mode != KB_LIST) {
            // Every candidate of a direct path is walked: a token in byte order from the key's own
            // literal state, a byte pair from the first byte of its token -- the bytes before the
            // pair have to stay in the checkpoint (within its byte budget), the first of the pair
            // leaves it, and what follows is walked from the successor.
            const global_u2 *src = (const global_u2 *)(mode == KB_SORTED ? Vc.sorted : Vc.bigram);
            uint32_t total = 0;
            for (uint32_t sgi = 0; sgi < n_seg; sgi++) total += seg_len[sgi];
            for (uint32_t i = tid; i < total; i += kKbThreads) {
                uint32_t sgi = 0, at = i;
                while (at >= seg_len[sgi]) { at -= seg_len[sgi]; sgi++; }
                const global_u2 *pe = src + seg_at[sgi] + at;
                const uint32_t tok = pe->x, y = pe->y;
                const uint32_t off = y & 0xFFu, L = off + (y >> 24);
                const uint64_t c0 = Vc.chunks[tok];
                const uint64_t c1 = L > 8u ? Vc.chunks[(size_t)Vc.V + tok] : 0ull;
                const uint64_t c2 = L > 16u ? Vc.chunks[2ull * Vc.V + tok] : 0ull;
                bool ok;
                if (mode == KB_SORTED) {
                    uint32_t sid = me.sid, aux = 0;
                    ok = walk_chunks(T, sid, aux, c0, c1, c2, 0u, L);
                } else {
                    ok = off - 1u <= r && stays_prefix(own_lut, c0, c1, c2, off - 1u);
                    if (ok) {
                        const uint32_t cls = own_lut[token_byte(c0, c1, c2, off - 1u)];
                        ok = cls >= CLS_EXIT_A &&
                             (cls == CLS_EXIT_B ? walk_first_hop(T, me.hop[1], hop_lut[1], c0, c1, c2, off, L)
                                                : walk_first_hop(T, me.hop[0], hop_lut[0], c0, c1, c2, off, L));
                    }
                }
                if (ok) atomicOr(&row[tok >> 5], 1u << (tok & 31u));
            }
            examined = total;
            __syncthreads();
        }
        if (mode == KB_LIST && list == 0u) {
            // A range item of a deep key: every entry of its list that is within the byte budget
            // has to be walked (the successor is a checkpoint, so no first byte rules an entry
            // out), which leaves nothing to filter: each thread walks the entries it requested.
            for (uint32_t i0 = 0; i0 < cnt; i0 += kKbThreads * kKbPer) {
                if (i0) request(i0);
                // two candidates at a time, their first chunks requested together (most tokens
                // are no longer than that), so that the two walks do not queue up behind one
                // another's first load
#pragma unroll
                for (uint32_t j = 0; j < kKbPer; j += 2u) {
                    if (i0 + j * kKbThreads >= cnt) break;    // no candidate left for any thread
                    uint64_t first_chunk[2];
#pragma unroll
                    for (uint32_t u = 0; u < 2u; u++) first_chunk[u] = Vc.chunks[x[j + u].x < Vc.V ? x[j + u].x : 0u];
#pragma unroll
                    for (uint32_t u = 0; u < 2u; u++) {
                        ExitEntry e;
                        e.tok = x[j + u].x; e.off = (uint8_t)x[j + u].y; e.cls = (uint8_t)(x[j + u].y >> 8);
                        e.first = (uint8_t)(x[j + u].y >> 16); e.rem = (uint8_t)(x[j + u].y >> 24);
                        if (i0 + (j + u) * kKbThreads + tid < cnt && (uint32_t)e.off - 1u <= r &&
                            (e.rem == 0 || walk_candidate(T, Vc, me, hop_lut, e, regs_ok, first_chunk[u])))
                            atomicOr(&row[e.tok >> 5], 1u << (e.tok & 31u));
                    }
                }
            }
            examined = cnt;
            cnt = 0;                                     // nothing left for the filter below
            __syncthreads();
        }
        constexpr uint32_t kAnyByte = 0x100u;        // no literal follows this exit
        const uint32_t next_lit[2] = {me.hop[0].kind == WG_KIND_LIT ? me.hop[0].lit : kAnyByte,
                                      me.hop[1].kind == WG_KIND_LIT ? me.hop[1].lit : kAnyByte};
        uint32_t pass = 0;
        for (uint32_t i0 = 0; i0 < cnt; i0 += kKbThreads * kKbPer, pass ^= 1u) {
            if (i0) request(i0);
            uint32_t slot[kKbPer], in_wave = 0;               // place among the wavefront's candidates to walk
            uint32_t need = 0;                                   // bit j: x[j] has to be walked
#pragma unroll
            for (uint32_t j = 0; j < kKbPer; j++) {
                if (i0 + j * kKbThreads >= cnt) break;        // no candidate left for any thread
                const uint32_t off = x[j].y & 0xFFu, cls = (x[j].y >> 8) & 0xFFu, first = (x[j].y >> 16) & 0xFFu, rem = x[j].y >> 24;
                const bool live = i0 + j * kKbThreads + tid < cnt && off - 1u <= r;
                const uint32_t lit = cls == CLS_EXIT_B ? next_lit[1] : next_lit[0];
                const bool walk = live && rem != 0 && (lit == kAnyByte || first == lit);
                if (live && rem == 0) atomicOr(&row[x[j].x >> 5], 1u << (x[j].x & 31u));
                const unsigned long long wm = __ballot(walk);
                slot[j] = in_wave + (uint32_t)__popcll(wm & ((1ull << lane) - 1ull));
                in_wave += (uint32_t)__popcll(wm);
                need |= (uint32_t)walk << j;
            }
            if (in_wave) {                                       // one LDS atomic per wavefront and pass
                uint32_t base = 0;
                if (lane == 0) base = atomicAdd(&queued[pass], in_wave);
                base = __shfl(base, 0);
#pragma unroll
                for (uint32_t j = 0; j < kKbPer; j++)
                    if ((need >> j) & 1u) queue[base + slot[j]] = x[j];
            }
            __syncthreads();
            // (b2) walk the queued candidates, one per thread and round
            // The other counter is cleared for the next pass here, between the two barriers of
            // this pass: its last readers passed the barrier that ended the pass before, and its
            // next writers wait behind the barrier that ends this one.
            const uint32_t n_queued = queued[pass];
            if (tid == 0) queued[pass ^ 1u] = 0;
            for (uint32_t i = tid; i < n_queued; i += kKbThreads) {
                const uint2 q = queue[i];
                ExitEntry e;
                e.tok = q.x; e.off = (uint8_t)q.y; e.cls = (uint8_t)(q.y >> 8); e.first = (uint8_t)(q.y >> 16); e.rem = (uint8_t)(q.y >> 24);
                if (walk_candidate(T, Vc, me, hop_lut, e, regs_ok, Vc.chunks[e.tok])) atomicOr(&row[e.tok >> 5], 1u << (e.tok & 31u));
            }
            __syncthreads();
        }
        if (tid == 0) atomicAdd(&Cc.ctr->entries_walked, (unsigned long long)cnt + examined);
        if (tid == 0 && Vc.eos_id >= 0 && me.eos_next != WG_SID_ERROR) {
            const uint32_t ew = (uint32_t)Vc.eos_id >> 5;
            if (ew >= 4u * q_lo && ew < 4u * q_hi) row[ew] |= 1u << ((uint32_t)Vc.eos_id & 31u);
        }
        __syncthreads();
        // (c) to its arena row (unless the arena had no row left) and to the bitmask row of the
        // request that claimed the key, which the gather then leaves alone
        if (me.slot != kNoSlot) {
            uint4 *dst = reinterpret_cast<uint4 *>(Cc.arena + (size_t)me.slot * rs);
            for (uint32_t q = q_lo + tid; q < q_hi; q += kKbThreads) dst[q] = row4[q];
            if (tid == 0 && p0 == 0) Cc.tags[me.key] = ((unsigned long long)Cc.epoch << 32) | me.slot;
        }
        {
            uint32_t *dst = bitmask + (size_t)me.req * Vc.W;
            if (Vc.W % 4u == 0u && reinterpret_cast<uintptr_t>(bitmask) % 16u == 0u) {
                uint4 *dst4 = reinterpret_cast<uint4 *>(dst);
                for (uint32_t q = q_lo + tid; q < q_hi; q += kKbThreads) dst4[q] = row4[q];
            } else {
                const uint32_t w_hi = 4u * q_hi < Vc.W ? 4u * q_hi : Vc.W;
                for (uint32_t w = 4u * q_lo + tid; w < w_hi; w += kKbThreads) dst[w] = row[w];
            }
        }
        __syncthreads();
    }
    }
    if (blockIdx.x == 0 && threadIdx.x == 0 && n_claims) atomicAdd(&Cc.ctr->builds, (unsigned long long)n_claims);
}

// The miss lists have been consumed by the kernels that ran before the last kernel of a fill:
// one thread of it counts their rows as used and empties them for the next call.
__device__ __forceinline__ void close_fill(const DeviceCache &Cc)
{
    const unsigned long long sc = Cc.ctr->slot_ctr;
    const uint32_t used = (uint32_t)(sc >> 32) == Cc.epoch ? (uint32_t)sc : 0u;
    const uint32_t room = Cc.cap_rows - used, n = Cc.ctr->n_claims;
    if (n > room) Cc.ctr->uncached_builds += n - room;
    Cc.ctr->slot_ctr = ((unsigned long long)Cc.epoch << 32) | (used + (n < room ? n : room));
    Cc.ctr->n_deep = 0; Cc.ctr->n_plain = 0; Cc.ctr->n_claims = 0; Cc.ctr->n_class_miss = 0;
    Cc.ctr->launch++;
}

// Where the mask of request b is: a row of the arena, its own bitmask row already (`in_place`:
// b claimed the key and key_build wrote the row there), the bitmask row of the request that
// built it uncached, or nowhere (nullptr: a row of zeros).
__device__ __forceinline__ const uint32_t *mask_source(const DeviceCache &Cc, uint32_t b, uint32_t B, uint32_t W,
                                                       const uint32_t *bitmask, bool &in_place)
{
    in_place = false;
    const uint32_t ref = Cc.row_ref[b];
    if (ref < kRefByKey) return ref < Cc.cap_rows ? Cc.arena + (size_t)ref * Cc.row_stride : nullptr;   // cached before this call
    if (ref == kRefSelf) { in_place = true; return bitmask + (size_t)b * W; }    // written by key_build
    if (ref == kNoKey) return nullptr;
    const unsigned long long t = Cc.tags[ref & ~kRefByKey];
    if ((uint32_t)(t >> 32) == Cc.epoch) return Cc.arena + (size_t)(uint32_t)t * Cc.row_stride;
    const uint32_t req = (uint32_t)(t & 0xFFFFu);
    return req < B ? bitmask + (size_t)req * W : nullptr;                        // built uncached for another request of this call
}

template <bool kVec>
__global__ void __launch_bounds__(256)
gather_kernel(DeviceCache Cc, uint32_t W, uint32_t *__restrict__ bitmask)
{
    const uint32_t b = blockIdx.y;
    if (blockIdx.x == 0 && b == 0 && threadIdx.x == 0) close_fill(Cc);
    bool in_place;
    const uint32_t *src = mask_source(Cc, b, gridDim.y, W, bitmask, in_place);
    if (in_place) return;
    uint32_t *dst = bitmask + (size_t)b * W;
    if (kVec) {
        const uint4 *s4 = reinterpret_cast<const uint4 *>(src);
        uint4 *d4 = reinterpret_cast<uint4 *>(dst);
        for (uint32_t q = blockIdx.x * blockDim.x + threadIdx.x; q < W / 4u; q += gridDim.x * blockDim.x)
            d4[q] = src ? s4[q] : uint4{0u, 0u, 0u, 0u};
    } else {
        for (uint32_t w = blockIdx.x * blockDim.x + threadIdx.x; w < W; w += gridDim.x * blockDim.x)
            dst[w] = src ? src[w] : 0u;
    }
}

// ---------------------------------------------------------------------------------------------
// apply: a thread takes mask bytes (8 consecutive tokens each) 256 apart, all loaded before any
// is used.  Nothing is read from the logits:
// a fully allowed group is skipped, a group with no allowed token is overwritten with one
// 16-byte store per 8 bf16 (two for fp32), and a mixed group stores -inf element by element,
// one store per disallowed token (found by count-trailing-zeros, so a group inside a
// free-text Wait, which has one or two such tokens, issues one or two stores).
constexpr uint32_t kApplyGroups = 2;       // mask bytes per thread, 256 apart
template <typename Vec, int kVecs, typename Elem>
__global__ void __launch_bounds__(256)
apply_vec_kernel(Elem *__restrict__ logits, int64_t row_stride, uint32_t V, uint32_t W,
                 const uint32_t *__restrict__ bitmask, Elem ninf)
{
    const uint32_t b = blockIdx.y;
    const uint32_t g0 = blockIdx.x * (256u * kApplyGroups) + threadIdx.x;   // group of 8 tokens
    const uint8_t *row = reinterpret_cast<const uint8_t *>(bitmask + (size_t)b * W);
    uint32_t m[kApplyGroups];
#pragma unroll
    for (uint32_t i = 0; i < kApplyGroups; i++) {
        const uint32_t g = g0 + i * 256u;
        m[i] = g * 8u < V ? row[g] : 0xFFu;
    }
#pragma unroll
    for (uint32_t i = 0; i < kApplyGroups; i++) {
        if (m[i] == 0xFFu) continue;
        Elem *p = logits + (int64_t)b * row_stride + (int64_t)(g0 + i * 256u) * 8;
        uint32_t z = ~m[i] & 0xFFu;                                 // disallowed positions
        if (z == 0xFFu) {
            union { Vec v[kVecs]; Elem e[8]; } u;
#pragma unroll
            for (int k = 0; k < 8; k++) u.e[k] = ninf;
            Vec *pv = reinterpret_cast<Vec *>(p);
#pragma unroll
            for (int k = 0; k < kVecs; k++) pv[k] = u.v[k];
        } else {
            while (z) { p[__builtin_ctz(z)] = ninf; z &= z - 1u; }
        }
    }
}

// gather and apply in one pass, the last kernel of a whole decode step: a thread takes four
// mask bytes (8 tokens each) 256 apart, loaded together so that finding where the request's
// mask lives is paid once; each byte goes to the caller's bitmask row and its disallowed tokens
// are stored as -inf.
constexpr uint32_t kGaGroups = 4;          // mask bytes per thread of gather_apply, 256 apart
template <typename Vec, int kVecs, typename Elem>
__global__ void __launch_bounds__(256)
gather_apply_kernel(DeviceCache Cc, Elem *__restrict__ logits, int64_t row_stride, uint32_t V, uint32_t W,
                    uint32_t *__restrict__ bitmask, Elem ninf)
{
    const uint32_t b = blockIdx.y;
    bool in_place;
    const uint32_t *src = mask_source(Cc, b, gridDim.y, W, bitmask, in_place);
    const uint32_t g0 = blockIdx.x * (256u * kGaGroups) + threadIdx.x;      // group of 8 tokens
    uint32_t m[kGaGroups];
#pragma unroll
    for (uint32_t i = 0; i < kGaGroups; i++) {
        const uint32_t g = g0 + i * 256u;
        m[i] = (src && g < 4u * W) ? reinterpret_cast<const uint8_t *>(src)[g] : 0u;
    }
    if (!in_place) {
        uint8_t *dst = reinterpret_cast<uint8_t *>(bitmask + (size_t)b * W);
#pragma unroll
        for (uint32_t i = 0; i < kGaGroups; i++) {
            const uint32_t g = g0 + i * 256u;
            if (g < 4u * W) dst[g] = (uint8_t)m[i];
        }
    }
#pragma unroll
    for (uint32_t i = 0; i < kGaGroups; i++) {
        const uint32_t g = g0 + i * 256u;
        if (g * 8u >= V || m[i] == 0xFFu) continue;
        Elem *p = logits + (int64_t)b * row_stride + (int64_t)g * 8;
        uint32_t z = ~m[i] & 0xFFu;                                 // disallowed positions
        if (z == 0xFFu) {
            union { Vec v[kVecs]; Elem e[8]; } u;
#pragma unroll
            for (int k = 0; k < 8; k++) u.e[k] = ninf;
            Vec *pv = reinterpret_cast<Vec *>(p);
#pragma unroll
            for (int k = 0; k < kVecs; k++) pv[k] = u.v[k];
        } else {
            while (z) { p[__builtin_ctz(z)] = ninf; z &= z - 1u; }
        }
    }
    if (blockIdx.x == 0 && b == 0 && threadIdx.x == 0) close_fill(Cc);
}

// masked argmax: a row is split over several workgroups; a thread takes 32-token groups (one mask word and up
// to four 16-byte loads for bf16, eight for fp32), skips pieces with no allowed token without
// touching their logits, and keeps its best candidate as a 64-bit key: the logit mapped to an unsigned
// integer that orders like the number (NaN lowest, -0 folded into +0) in the high half, the
// complement of the token id in the low half, so that a plain maximum prefers the larger logit
// and then the lower id.  Key 0 means "no allowed token".  Workgroups merge their maxima with
// one 64-bit atomic max per row; the workgroup of a row that finishes last writes the token id.

// Per-row merge area of masked argmax, shared by the workgroups of a row: the running maximum
// of the keys and the number of workgroups that have reported.  File-scope device memory: all
// zero between calls (the last workgroup of a row clears what it reads), one copy per GPU, so
// two masked-argmax calls that overlap on one GPU would mix their rows.
constexpr uint32_t kArgmaxRows = 65536;
constexpr int kArgmaxPieces = 8;           // 16-byte pieces of logits per thread of masked_argmax
__device__ unsigned long long g_argmax_key[kArgmaxRows];

// The maximum over the allowed tokens of one 16-byte piece, folded into four accumulators.
// A disallowed token's bits are forced to all ones, which is a NaN in both formats, and the
// hardware maximum ignores NaNs, so NaN logits drop out the same way.
__device__ __forceinline__ void piece_max(const uint4 &v, uint32_t m, uint16_t, float acc[4])
{
    const uint32_t d[4] = {v.x, v.y, v.z, v.w};
    const uint32_t nm = ~m;
#pragma unroll
    for (int k = 0; k < 4; k++) {                     // dword k holds tokens 2k (low half) and 2k+1
        const uint32_t lo = (uint32_t)__builtin_amdgcn_sbfe(nm, 2 * k, 1), hi = (uint32_t)__builtin_amdgcn_sbfe(nm, 2 * k + 1, 1);
        const uint32_t x = d[k] | (lo & 0xFFFFu) | (hi << 16);
        acc[(2 * k) & 3] = __builtin_fmaxf(acc[(2 * k) & 3], __uint_as_float(x << 16));
        acc[(2 * k + 1) & 3] = __builtin_fmaxf(acc[(2 * k + 1) & 3], __uint_as_float(x & 0xFFFF0000u));
    }
}
__device__ __forceinline__ void piece_max(const uint4 &v, uint32_t m, uint32_t, float acc[4])
{
    const uint32_t d[4] = {v.x, v.y, v.z, v.w};
    const uint32_t nm = ~m;
#pragma unroll
    for (int k = 0; k < 4; k++)
        acc[k] = __builtin_fmaxf(acc[k], __uint_as_float(d[k] | (uint32_t)__builtin_amdgcn_sbfe(nm, k, 1)));
}

template <typename Elem, bool kAligned>
__global__ void __launch_bounds__(256)
masked_argmax_kernel(const Elem *__restrict__ logits, int64_t row_stride, uint32_t V, uint32_t W,
                     const uint32_t *__restrict__ bitmask)
{
    constexpr uint32_t kPer = 16 / sizeof(Elem);                  // tokens per 16-byte piece: 8 bf16, 4 fp32
    constexpr uint32_t kSubMask = (1u << kPer) - 1u;
    constexpr int kPieces = kArgmaxPieces;                        // pieces per thread, all in flight together
    __shared__ float part_v[4];
    __shared__ uint32_t part_t[4];
    const uint32_t b = blockIdx.y, tid = threadIdx.x;
    const uint32_t *mrow = bitmask + (size_t)b * W;
    const Elem *row = logits + (int64_t)b * row_stride;
    const uint32_t n_pieces = (V + kPer - 1u) / kPer;
    const uint32_t base = blockIdx.x * (kPieces * 256u);
    // Piece j of thread t is piece base + j*256 + t of the row: the 64 lanes of a wavefront read
    // 1 KB of consecutive logits with each load.  First every piece's mask bits, then the logits
    // of the pieces that hold an allowed token, then the arithmetic.
    uint32_t m[kPieces];
    union { uint4 v; Elem e[kPer]; } u[kPieces];
#pragma unroll
    for (int j = 0; j < kPieces; j++) {
        const uint32_t p = base + j * 256u + tid;
        m[j] = p < n_pieces ? (mrow[p * kPer >> 5] >> (p * kPer & 31u)) & kSubMask : 0u;
    }
#pragma unroll
    for (int j = 0; j < kPieces; j++) {
        const uint32_t p = base + j * 256u + tid;
        if (kAligned) u[j].v = m[j] ? *reinterpret_cast<const uint4 *>(row + (size_t)p * kPer) : uint4{0u, 0u, 0u, 0u};
        else {
#pragma unroll
            for (uint32_t i = 0; i < kPer; i++)
                u[j].e[i] = ((m[j] >> i) & 1u) ? row[(size_t)p * kPer + i] : (Elem)0;   // set bits are below V
        }
    }
    // Pass 1, branch-free: the maximum over the thread's allowed tokens as a float.
    const float nanv = __builtin_nanf("");
    float acc[4] = {nanv, nanv, nanv, nanv};
#pragma unroll
    for (int j = 0; j < kPieces; j++) piece_max(u[j].v, m[j], Elem(0), acc);
    const float tmax = __builtin_fmaxf(__builtin_fmaxf(acc[0], acc[1]), __builtin_fmaxf(acc[2], acc[3]));
    float wmax = tmax;                               // workgroup maximum
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) wmax = __builtin_fmaxf(wmax, __shfl_xor(wmax, o));
    if ((tid & 63u) == 0) part_v[tid >> 6] = wmax;
    __syncthreads();
    wmax = __builtin_fmaxf(__builtin_fmaxf(part_v[0], part_v[1]), __builtin_fmaxf(part_v[2], part_v[3]));
    // Pass 2, only in threads that hold the maximum: the lowest token whose logit equals it
    // (float equality, so -0.0 and +0.0 tie).  Without any number in this part of the row the
    // candidate is the lowest allowed token (its logit is a NaN).
    const bool number = wmax == wmax;
    uint32_t cand = 0xFFFFFFFFu;
    if (!number || tmax == wmax) {
#pragma unroll
        for (int j = kPieces - 1; j >= 0; j--) {
            uint32_t eq = 0;
#pragma unroll
            for (uint32_t i = 0; i < kPer; i++) eq |= (uint32_t)(elem_float(u[j].e[i]) == wmax) << i;
            eq = number ? eq & m[j] : m[j];
            if (eq) cand = (base + j * 256u + tid) * kPer + (uint32_t)__builtin_ctz(eq);
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) { const uint32_t other = __shfl_xor(cand, o); cand = other < cand ? other : cand; }
    if ((tid & 63u) == 0) part_t[tid >> 6] = cand;
    __syncthreads();
    if (tid == 0) {
        for (uint32_t w = 1; w < 4u; w++) cand = part_t[w] < cand ? part_t[w] : cand;
        if (cand != 0xFFFFFFFFu) {
            const uint32_t rank = number ? order_key(__float_as_uint(wmax)) : 0u;
            atomicMax(&g_argmax_key[b], ((unsigned long long)rank << 32) | (0xFFFFFFFFu - cand));
        }
    }
}

// Turns the merged keys into token ids and leaves the merge area zeroed for the next call.
__global__ void __launch_bounds__(256)
masked_argmax_finish_kernel(int32_t *__restrict__ tokens, uint32_t B)
{
    const uint32_t b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    const unsigned long long best = g_argmax_key[b];
    tokens[b] = best ? (int32_t)(0xFFFFFFFFu - (uint32_t)best) : -1;
    g_argmax_key[b] = 0ull;
}

template <typename Elem>
__global__ void __launch_bounds__(256)
apply_scalar_kernel(Elem *__restrict__ logits, int64_t row_stride, uint32_t V, uint32_t W,
                    const uint32_t *__restrict__ bitmask, Elem ninf)
{
    uint32_t b = blockIdx.y;
    uint32_t t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= V) return;
    uint32_t word = bitmask[(size_t)b * W + (t >> 5)];
    if (!((word >> (t & 31u)) & 1u)) logits[(int64_t)b * row_stride + t] = ninf;
}

// ---------------------------------------------------------------------------------------------
// advance: one thread per request.  The token's bytes are fetched as 8-byte chunks (three
// independent loads) and walked with walk_chunks; tokens longer than 24 bytes take the
// generic byte-at-a-time walker.
__device__ __forceinline__ void advance_one(const DeviceTable &T, const DeviceVocab &Vc, const DeviceCache &Cc,
                                            uint32_t &sid, uint32_t &aux, int64_t t)
{
    bool ok;
    if (Vc.lmax > 24u || t < 0 || t >= (int64_t)Vc.V || (int64_t)Vc.eos_id == t) {
        ok = walk_token(T, Vc, sid, aux, t);
    } else {
        const uint32_t L = Vc.len8[t];
        const uint64_t c0 = Vc.chunks[t];
        const uint64_t c1 = Vc.n_chunks > 1u ? Vc.chunks[(size_t)Vc.V + t] : 0ull;
        const uint64_t c2 = Vc.n_chunks > 2u ? Vc.chunks[2ull * Vc.V + t] : 0ull;
        ok = L != 0u && sid < T.n_states && walk_chunks(T, sid, aux, c0, c1, c2, 0u, L);
    }
    if (!ok) {
        sid = WG_SID_ERROR; aux = 0;
        atomicAdd(&Cc.ctr->errors, 1ull);
    }
}

__global__ void __launch_bounds__(64)
advance_kernel(DeviceTable T, DeviceVocab Vc, DeviceCache Cc, wg_state_t *__restrict__ states,
               const int32_t *__restrict__ tokens, uint32_t B)
{
    uint32_t b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    uint32_t sid = states[b].sid, aux = states[b].aux;
    advance_one(T, Vc, Cc, sid, aux, (int64_t)tokens[b]);
    states[b].sid = sid; states[b].aux = aux;
}

// advance followed by the lookup of the next step's fill, one thread per request: the new
// state goes straight from the walker into the cache lookup.
__global__ void __launch_bounds__(64)
advance_lookup_kernel(DeviceTable T, DeviceVocab Vc, DeviceCache Cc, wg_state_t *__restrict__ states,
                      const int32_t *__restrict__ tokens, uint32_t B)
{
    const uint32_t b = blockIdx.x * blockDim.x + threadIdx.x;
    const bool live = b < B;
    const LookupEnv env = lookup_env(Cc);
    uint32_t sid = 0, aux = 0;
    if (live) {
        sid = states[b].sid; aux = states[b].aux;
        advance_one(T, Vc, Cc, sid, aux, (int64_t)tokens[b]);
        states[b].sid = sid; states[b].aux = aux;
    }
    lookup_one(T, Cc, env, b, live, sid, aux);
}

// The bytes a request is forced to produce next: from a state inside a Write, the rest of that
// Write and of the Writes that follow it directly, up to the next state that is not a literal
// byte.  One thread per request; a run of literal states is copied from the state table's
// literal bytes.
__global__ void __launch_bounds__(64)
forced_bytes_kernel(DeviceTable T, const wg_state_t *__restrict__ states, uint32_t B, uint32_t cap,
                    uint8_t *__restrict__ bytes, uint32_t *__restrict__ lens, wg_state_t *__restrict__ end_states)
{
    const uint32_t b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    uint32_t sid = states[b].sid, n = 0;
    const uint32_t aux = states[b].aux;
    uint8_t *out = bytes + (size_t)b * cap;
    while (n < cap && sid < T.n_states) {
        const StateDesc d = T.states[sid];
        if ((d.kind_byte & 0xFFu) != WG_KIND_LIT) break;
        const uint32_t m = d.run < cap - n ? d.run : cap - n;
        for (uint32_t i = 0; i < m; i++) out[n + i] = T.lit[sid + i];
        n += m;
        sid = m == d.run ? d.cls : sid + m;                  // d.cls: state after the Write
    }
    lens[b] = n;
    if (end_states) end_states[b] = wg_state_t{sid, n ? 0u : aux};
}

// One block per row: d_tokens[b] = index of the (draw mod popcount)-th set bit.
__global__ void __launch_bounds__(256)
select_kernel(const uint32_t *__restrict__ bitmask, uint32_t W, const uint64_t *__restrict__ draws,
              int32_t *__restrict__ tokens)
{
    __shared__ uint32_t cnt[256];
    __shared__ uint32_t total;
    uint32_t b = blockIdx.x, tid = threadIdx.x;
    const uint32_t *row = bitmask + (size_t)b * W;
    uint32_t per = (W + 255u) / 256u, lo = tid * per, hi = lo + per < W ? lo + per : W;
    uint32_t c = 0;
    for (uint32_t w = lo; w < hi; w++) c += __popc(row[w]);
    cnt[tid] = c;
    __syncthreads();
    if (tid == 0) {
        uint32_t s = 0;
        for (int i = 0; i < 256; i++) { uint32_t x = cnt[i]; cnt[i] = s; s += x; }   // exclusive scan
        total = s;
        if (s == 0) tokens[b] = -1;
    }
    __syncthreads();
    if (total == 0) return;
    uint32_t k = (uint32_t)(draws[b] % (uint64_t)total);
    if (k >= cnt[tid] && k < cnt[tid] + c) {
        k -= cnt[tid];
        for (uint32_t w = lo; w < hi; w++) {
            uint32_t x = row[w], pc = __popc(x);
            if (k >= pc) { k -= pc; continue; }
            for (int bit = 0; bit < 32; bit++)
                if ((x >> bit) & 1u) { if (k == 0) { tokens[b] = (int32_t)(w * 32u + bit); return; } k--; }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// launchers (host)

static inline uint32_t cdiv(uint64_t a, uint64_t b) { return (uint32_t)((a + b - 1) / b); }

// key_build keeps a whole mask row (dynamic LDS) next to its candidate queue and tables (static
// LDS); together they may pass the 64 KB a kernel gets without asking.  The limit is a property
// of the kernel on a device, shared by every handle of the process, so it is only ever raised: a
// handle with short rows compiled later leaves the room a handle with long rows needs.  Returns
// hipErrorInvalidValue when a row does not fit the 160 KB of a compute unit at all.
hipError_t configure_kernels(uint32_t row_bytes)
{
    static std::mutex mu;
    static uint32_t granted[64];                     // per device: dynamic LDS key_build may ask for
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    hipFuncAttributes attr;
    e = hipFuncGetAttributes(&attr, reinterpret_cast<const void *>(key_build_kernel));
    if (e != hipSuccess) return e;
    if (attr.sharedSizeBytes + (size_t)row_bytes > 160u * 1024u) return hipErrorInvalidValue;
    std::lock_guard<std::mutex> lock(mu);
    const uint32_t slot = (uint32_t)dev < 64u ? (uint32_t)dev : 63u;
    if ((uint32_t)dev < 64u && row_bytes <= granted[slot]) return hipSuccess;
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(key_build_kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)row_bytes);
    if (e == hipSuccess && (uint32_t)dev < 64u) granted[slot] = row_bytes;
    return e;
}

// Launches on stream s; with a pair of events the kernel's own begin / end timestamps are
// recorded into them (hipExtLaunchKernelGGL), which times the kernel without the queue gaps
// that events recorded between launches would include.
template <typename K, typename... A>
static inline void launch(K kernel, dim3 grid, dim3 block, uint32_t lds, hipStream_t s, hipEvent_t *ev,
                          A... args)
{
    if (ev) hipExtLaunchKernelGGL(kernel, grid, block, lds, s, ev[0], ev[1], 0, args...);
    else hipLaunchKernelGGL(kernel, grid, block, lds, s, args...);
}

static bool apply_vec_ok(const void *logits, int dtype, uint32_t V, int64_t row_stride)
{
    const size_t esz = dtype == WG_F32 ? 4 : 2;
    return reinterpret_cast<uintptr_t>(logits) % 16 == 0 && (row_stride * (int64_t)esz) % 16 == 0 && V % 8u == 0;
}

hipError_t launch_fill(const DeviceTable &T, const DeviceVocab &Vc, const DeviceCache &Cc,
                       wg_state_t *states, const int32_t *tokens, uint32_t B, uint32_t *bitmask,
                       void *logits, int dtype, int64_t logits_stride,
                       uint32_t n_cu, hipStream_t s, hipEvent_t *ev)
{
    if (tokens) launch(advance_lookup_kernel, dim3(cdiv(B, 64)), dim3(64), 0, s, ev, T, Vc, Cc, states, tokens, B);
    else launch(lookup_kernel, dim3(cdiv(B, 64)), dim3(64), 0, s, ev, T, Cc, static_cast<const wg_state_t *>(states), B);
    // the number of misses is only known on the device: both build kernels stride a fixed
    // grid over whatever the lookup queued and fall through when nothing is queued
    // (a call scans at most one class table per request, and no more than the handle has; the
    // kernels hold 5 workgroups per compute unit, and a launch of more costs a warm step time)
    uint32_t groups = cdiv(Vc.V, kScanGroup);
    uint64_t scan_items = (uint64_t)(B < T.n_classes ? B : T.n_classes) * groups;
    uint32_t cap = n_cu * kScanWgs;
    // a handle with few class tables scans them one per work item; with many, a call may bring so
    // many that they are taken several at a time
    if (Cc.scan_batch ? Cc.scan_batch > 1u : (uint64_t)T.n_classes * groups > kScanBatchFrom)
        launch(class_scan_batch_kernel, dim3(scan_items < n_cu * kScanBatchWgs ? (uint32_t)scan_items : n_cu * kScanBatchWgs),
               dim3(kScanThreads), 0, s, ev ? ev + 2 : nullptr, T, Vc, Cc);
    else
        launch(class_scan_kernel, dim3(scan_items < cap ? (uint32_t)scan_items : cap), dim3(kScanThreads), 0, s,
               ev ? ev + 2 : nullptr, T, Vc, Cc);
    // up to kParts work items per key; two 512-thread workgroups fit a compute unit
    const uint32_t kb = n_cu * 2u;
    const uint64_t kb_items = (uint64_t)B * kParts;
    launch(key_build_kernel, dim3(kb_items < kb ? (uint32_t)kb_items : kb), dim3(kKbThreads), Cc.row_stride * 4u, s,
           ev ? ev + 4 : nullptr, T, Vc, Cc, bitmask);
    hipEvent_t *ge = ev ? ev + 6 : nullptr;
    if (logits && apply_vec_ok(logits, dtype, Vc.V, logits_stride)) {
        const dim3 g(cdiv(4u * Vc.W, 256 * kGaGroups), B);
        if (dtype == WG_F32)
            launch(gather_apply_kernel<uint4, 2, uint32_t>, g, dim3(256), 0, s, ge, Cc, (uint32_t *)logits,
                   logits_stride, Vc.V, Vc.W, bitmask, 0xFF800000u);
        else
            launch(gather_apply_kernel<uint4, 1, uint16_t>, g, dim3(256), 0, s, ge, Cc, (uint16_t *)logits,
                   logits_stride, Vc.V, Vc.W, bitmask, (uint16_t)0xFF80u);
        return hipGetLastError();
    }
    const bool vec = Vc.W % 4u == 0 && reinterpret_cast<uintptr_t>(bitmask) % 16 == 0;
    if (vec) launch(gather_kernel<true>, dim3(cdiv(Vc.W / 4u, 256), B), dim3(256), 0, s, ge, Cc, Vc.W, bitmask);
    else launch(gather_kernel<false>, dim3(cdiv(Vc.W, 256 * 4), B), dim3(256), 0, s, ge, Cc, Vc.W, bitmask);
    // logits that do not allow 16-byte stores take the separate apply kernels
    if (logits) return launch_apply(logits, dtype, B, Vc.V, logits_stride, bitmask, s, nullptr);
    return hipGetLastError();
}

hipError_t launch_apply(void *logits, int dtype, uint32_t B, uint32_t V, int64_t row_stride,
                        const uint32_t *bitmask, hipStream_t s, hipEvent_t *ev)
{
    uint32_t W = (V + 31u) / 32u;
    const bool vec_ok = apply_vec_ok(logits, dtype, V, row_stride);
    if (vec_ok) {
        dim3 g(cdiv(V / 8u, 256 * kApplyGroups), B);
        if (dtype == WG_F32)
            launch(apply_vec_kernel<uint4, 2, uint32_t>, g, dim3(256), 0, s, ev, (uint32_t *)logits, row_stride, V, W, bitmask, 0xFF800000u);
        else
            launch(apply_vec_kernel<uint4, 1, uint16_t>, g, dim3(256), 0, s, ev, (uint16_t *)logits, row_stride, V, W, bitmask, (uint16_t)0xFF80u);
    } else {
        dim3 g(cdiv(V, 256), B);
        if (dtype == WG_F32)
            launch(apply_scalar_kernel<uint32_t>, g, dim3(256), 0, s, ev, (uint32_t *)logits, row_stride, V, W, bitmask, 0xFF800000u);
        else
            launch(apply_scalar_kernel<uint16_t>, g, dim3(256), 0, s, ev, (uint16_t *)logits, row_stride, V, W, bitmask, (uint16_t)0xFF80u);
    }
    return hipGetLastError();
}

hipError_t launch_masked_argmax(const void *logits, int dtype, uint32_t B, uint32_t V, int64_t row_stride,
                                const uint32_t *bitmask, int32_t *tokens, hipStream_t s)
{
    uint32_t W = (V + 31u) / 32u;
    size_t esz = dtype == WG_F32 ? 4 : 2;
    bool vec_ok = (reinterpret_cast<uintptr_t>(logits) % 16 == 0) && ((row_stride * (int64_t)esz) % 16 == 0) &&
                  (V % 8u == 0);
    const uint32_t pieces = cdiv(V, dtype == WG_F32 ? 4 : 8);
    dim3 g(cdiv(pieces, kArgmaxPieces * 256), B);
    if (dtype == WG_F32) {
        if (vec_ok) masked_argmax_kernel<uint32_t, true><<<g, 256, 0, s>>>((const uint32_t *)logits, row_stride, V, W, bitmask);
        else masked_argmax_kernel<uint32_t, false><<<g, 256, 0, s>>>((const uint32_t *)logits, row_stride, V, W, bitmask);
    } else {
        if (vec_ok) masked_argmax_kernel<uint16_t, true><<<g, 256, 0, s>>>((const uint16_t *)logits, row_stride, V, W, bitmask);
        else masked_argmax_kernel<uint16_t, false><<<g, 256, 0, s>>>((const uint16_t *)logits, row_stride, V, W, bitmask);
    }
    masked_argmax_finish_kernel<<<cdiv(B, 256), 256, 0, s>>>(tokens, B);
    return hipGetLastError();
}

hipError_t launch_advance(const DeviceTable &T, const DeviceVocab &Vc, const DeviceCache &Cc,
                          wg_state_t *states, const int32_t *tokens, uint32_t B, hipStream_t s,
                          hipEvent_t *ev)
{
    launch(advance_kernel, dim3(cdiv(B, 64)), dim3(64), 0, s, ev, T, Vc, Cc, states, tokens, B);
    return hipGetLastError();
}

hipError_t launch_forced_bytes(const DeviceTable &T, const wg_state_t *states, uint32_t B, uint32_t cap,
                               uint8_t *bytes, uint32_t *lens, wg_state_t *end_states, hipStream_t s)
{
    forced_bytes_kernel<<<cdiv(B, 64), 64, 0, s>>>(T, states, B, cap, bytes, lens, end_states);
    return hipGetLastError();
}

hipError_t launch_select(const uint32_t *bitmask, uint32_t B, uint32_t V, const uint64_t *draws,
                         int32_t *tokens, hipStream_t s)
{
    select_kernel<<<B, 256, 0, s>>>(bitmask, (V + 31u) / 32u, draws, tokens);
    return hipGetLastError();
}

}  // namespace wg
