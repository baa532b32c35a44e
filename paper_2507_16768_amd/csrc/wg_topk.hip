// masked top-k for gfx950 (wave64): the k best allowed tokens of every row, logits read once and
// never written -- the candidate set a top-k sampler draws from, taken straight from the raw
// logits and the mask instead of from logits with -inf written into them.
//
// Every allowed token has a 64-bit rank key: the logit mapped to an unsigned integer that
// orders like the number (NaN lowest, -0 folded into +0) plus one in the high half, the
// complement of the token id in the low half.  Keys of different tokens differ, a larger key
// is a better token (larger logit, then lower id), and 0 means "not allowed / nothing".
//
//   topk_slice : a workgroup takes 8,192 tokens of one row, 32 per thread, held in registers.
//                The k-th largest of the 256 thread maxima is a lower bound for the slice's
//                k-th best token, so only tokens at or above it can matter: in practice little
//                more than k.  They go to LDS, are ranked by counting, and the best k leave
//                for the workspace, best first.  The bound is first taken on the logits as
//                floats (cheap, but any number of tokens may tie at it); if the candidates do
//                not fit their list it is taken again on the rank keys themselves, where at
//                most 32 k can reach it (k threads reach the bound, 32 tokens each).
//   topk_merge : a workgroup per row does the same with the keys the row's slices left (a
//                thread's share of them instead of a thread's tokens) and writes the ids and
//                the raw values of the best k.
// The k-th largest of 256 values, one per thread: each wavefront sorts its 64 values with
// lane exchanges (a bitonic network, no LDS traffic), the four sorted lists go to LDS, and a
// value's place among all 256 is its lane plus a binary search in each of the other three lists.
#include <hip/hip_runtime.h>

#include <mutex>

#include "wg_device.h"
#include "wg_order.h"

namespace wg {

// The workspace of wg_masked_topk_static: what wg_masked_topk takes from its caller, held by the
// library instead, for callers that cannot allocate.  One copy per GPU the library runs on, for
// the life of the process.  topk_slice writes every key of a call's lists before topk_merge reads
// them, so nothing has to be cleared between calls.  In host code the array's name is a stand-in
// only; its address on the current device comes from static_topk_scratch().
static __device__ __align__(256) unsigned long long scratch[kTopkStaticKeys];

constexpr uint32_t kTkThreads = 256;
constexpr uint32_t kTkPer = kTopkSlice / kTkThreads;     // tokens per thread
constexpr uint32_t kTkCand = kTopkMax * kTkPer;          // bound on the candidates of a slice
static_assert(kTkPer == 32, "a thread's tokens are four 16-byte pieces of bf16 or eight of fp32");
static_assert(kTkThreads == 256, "four wavefronts: kth_largest merges four sorted lists");
static_assert(kTopkMergeKeys <= kTkPer * kTkThreads, "a thread of the merge holds at most kTkPer keys (candidate bound)");

struct TopkShared {
    unsigned long long sorted[4][64];     // the wavefronts' values, each list largest first
    unsigned long long cand[kTkCand];     // keys at or above the bound
    uint32_t cand_id[kTkCand];            // (topk_slice: their token ids, before the keys are made)
    unsigned long long bound;
    uint32_t n_cand;
    uint32_t n_held;
};

static_assert(sizeof(TopkShared) + kTopkMergeKeys * sizeof(unsigned long long) <= 64u * 1024u,
              "the merge fits the LDS a kernel gets without asking");

// The k-th largest of the workgroup's 256 values `own` (nonzero values all differ), 0 when fewer
// than k of them are nonzero.  Also resets the candidate list.  Every thread calls it.  T is
// uint32_t or unsigned long long.
template <typename T>
__device__ __forceinline__ T kth_largest(TopkShared &sh, T own, uint32_t k)
{
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    T(*sorted)[64] = reinterpret_cast<T(*)[64]>(sh.sorted);
    T v = own;
#pragma unroll
    for (uint32_t size = 2; size <= 64u; size <<= 1) {
#pragma unroll
        for (uint32_t stride = size >> 1; stride > 0u; stride >>= 1) {
            const T other = __shfl_xor(v, (int)stride);
            const bool descending = (lane & size) == 0u;          // direction of this lane's block (64: all)
            const bool first = (lane & stride) == 0u;             // the lower lane of the pair
            const T hi = v > other ? v : other, lo = v > other ? other : v;
            v = (first == descending) ? hi : lo;
        }
    }
    __syncthreads();                                               // nobody still reads what an earlier call left
    sorted[wave][lane] = v;
    if (tid == 0) { sh.bound = 0ull; sh.n_cand = 0u; sh.n_held = 0u; }
    __syncthreads();
    uint32_t rank = lane;                                          // larger values in its own list
#pragma unroll
    for (uint32_t o = 1; o < 4u; o++) {
        const T *a = sorted[(wave + o) & 3u];                      // how many of this list are larger
        uint32_t pos = 0;
#pragma unroll
        for (uint32_t step = 32; step > 0u; step >>= 1) pos += a[pos + step - 1u] > v ? step : 0u;
        rank += pos + (a[pos] > v ? 1u : 0u);
    }
    if (v && rank == k - 1u) sh.bound = v;
    __syncthreads();
    return (T)sh.bound;
}

// Ranks the n candidates in LDS by counting; calls emit(rank, key) for those among the best k.
template <typename F>
__device__ __forceinline__ void rank_candidates(const TopkShared &sh, uint32_t n, uint32_t k, F emit)
{
    for (uint32_t i = threadIdx.x; i < n; i += kTkThreads) {
        const unsigned long long x = sh.cand[i];
        uint32_t r = 0;
        for (uint32_t q = 0; q < n; q++) r += sh.cand[q] > x;
        if (r < k) emit(r, x);
    }
}

// Appends a thread's c candidates: places by a prefix sum over the wavefront, one LDS atomic
// per wavefront.  Returns the thread's first place.
__device__ __forceinline__ uint32_t candidate_places(TopkShared &sh, uint32_t c)
{
    const uint32_t lane = threadIdx.x & 63u;
    uint32_t inc = c;
#pragma unroll
    for (uint32_t o = 1; o < 64u; o <<= 1) {
        const uint32_t below = __shfl_up(inc, o);
        if (lane >= o) inc += below;
    }
    uint32_t wave_base = 0;
    if (lane == 63u && inc) wave_base = atomicAdd(&sh.n_cand, inc);
    wave_base = __shfl(wave_base, 63);
    return wave_base + inc - c;
}

// The tokens of a 16-byte piece as floats, a disallowed one as a NaN (all bits set), which the
// hardware maximum and every comparison ignore.
__device__ __forceinline__ void piece_values(const uint4 &v, uint32_t m, uint16_t, float *x)
{
    const uint32_t d[4] = {v.x, v.y, v.z, v.w};
    const uint32_t nm = ~m;
#pragma unroll
    for (int q = 0; q < 4; q++) {                     // dword q holds tokens 2q (low half) and 2q+1
        const uint32_t lo = (uint32_t)__builtin_amdgcn_sbfe(nm, 2 * q, 1), hi = (uint32_t)__builtin_amdgcn_sbfe(nm, 2 * q + 1, 1);
        const uint32_t w = d[q] | (lo & 0xFFFFu) | (hi << 16);
        x[2 * q] = __uint_as_float(w << 16);
        x[2 * q + 1] = __uint_as_float(w & 0xFFFF0000u);
    }
}
__device__ __forceinline__ void piece_values(const uint4 &v, uint32_t m, uint32_t, float *x)
{
    const uint32_t d[4] = {v.x, v.y, v.z, v.w};
    const uint32_t nm = ~m;
#pragma unroll
    for (int q = 0; q < 4; q++) x[q] = __uint_as_float(d[q] | (uint32_t)__builtin_amdgcn_sbfe(nm, q, 1));
}

// The number whose order key is kk, for an order key of a number with its low 8 bits cleared: a
// number at or below the original (-inf where clearing the bits left the numbers).
__device__ __forceinline__ float key_floor_value(uint32_t kk)
{
    uint32_t u = (kk & 0x80000000u) ? (kk & 0x7FFFFFFFu) : ~kk;
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) u = 0xFF800000u;
    return __uint_as_float(u);
}

template <typename Elem, bool kAligned>
__global__ void __launch_bounds__(kTkThreads)
topk_slice_kernel(const Elem *__restrict__ logits, int64_t row_stride, uint32_t V, uint32_t W,
                  const uint32_t *__restrict__ bitmask, uint32_t k, unsigned long long *__restrict__ lists)
{
    constexpr uint32_t kPer = 16 / sizeof(Elem);                  // tokens per 16-byte piece: 8 bf16, 4 fp32
    constexpr uint32_t kPieces = kTkPer / kPer;                   // pieces per thread, all in flight together
    constexpr uint32_t kSubMask = (1u << kPer) - 1u;
    __shared__ TopkShared sh;
    const uint32_t b = blockIdx.y, tid = threadIdx.x;
    const uint32_t *mrow = bitmask + (size_t)b * W;
    const Elem *row = logits + (int64_t)b * row_stride;
    const uint32_t n_pieces = (V + kPer - 1u) / kPer;
    const uint32_t base = blockIdx.x * (kTopkSlice / kPer);       // first piece of the slice
    // Piece j of thread t is piece base + j*256 + t of the row: the 64 lanes of a wavefront read
    // 1 KB of consecutive logits with each load.  First every piece's mask bits, then the logits
    // of the pieces that hold an allowed token.
    uint32_t m[kPieces];
    union { uint4 v; Elem e[kPer]; } u[kPieces];
#pragma unroll
    for (uint32_t j = 0; j < kPieces; j++) {
        const uint32_t p = base + j * kTkThreads + tid;
        m[j] = p < n_pieces ? (mrow[p * kPer >> 5] >> (p * kPer & 31u)) & kSubMask : 0u;
    }
    uint32_t any = 0;
#pragma unroll
    for (uint32_t j = 0; j < kPieces; j++) any |= m[j];
    if (!__syncthreads_or((int)any)) {                 // nothing allowed in this slice
        for (uint32_t r = tid; r < k; r += kTkThreads) lists[((size_t)b * gridDim.x + blockIdx.x) * k + r] = 0ull;
        return;
    }
#pragma unroll
    for (uint32_t j = 0; j < kPieces; j++) {
        const uint32_t p = base + j * kTkThreads + tid;
        if (kAligned) u[j].v = m[j] ? *reinterpret_cast<const uint4 *>(row + (size_t)p * kPer) : uint4{0u, 0u, 0u, 0u};
        else {
#pragma unroll
            for (uint32_t i = 0; i < kPer; i++)
                u[j].e[i] = ((m[j] >> i) & 1u) ? row[(size_t)p * kPer + i] : (Elem)0;   // set bits are below V
        }
    }
    // The exact rank key of the thread's token e (0 = not allowed); a thread's tokens are in
    // ascending id order.
    auto rank_key = [&](uint32_t e) -> unsigned long long {
        if (!((m[e / kPer] >> (e % kPer)) & 1u)) return 0ull;
        const uint32_t hi = order_key(__float_as_uint(elem_float(u[e / kPer].e[e % kPer]))) + 1u;
        const uint32_t id = (base + (e / kPer) * kTkThreads + tid) * kPer + e % kPer;
        return ((unsigned long long)hi << 32) | (0xFFFFFFFFu - id);
    };
    // Fast path, in floats.  The k-th largest of the 256 thread maxima is a lower bound for the
    // slice's k-th best logit, so only tokens at or above it can matter -- in practice little
    // more than k.  The thread maxima are ranked as order keys whose low 8 bits give way to the
    // thread's number (that makes them differ; the bound only gets lower).
    float x[kTkPer];
#pragma unroll
    for (uint32_t j = 0; j < kPieces; j++) piece_values(u[j].v, m[j], Elem(0), x + j * kPer);
    float tm = __builtin_nanf("");
#pragma unroll
    for (uint32_t e = 0; e < kTkPer; e++) tm = __builtin_fmaxf(tm, x[e]);
    const uint32_t own32 = tm == tm ? (order_key(__float_as_uint(tm)) & 0xFFFFFF00u) | (255u - tid) : 0u;
    const uint32_t bound32 = kth_largest<uint32_t>(sh, own32, k);
    uint32_t mine = 0;                                // bit e: token e of this thread is a candidate
    if (bound32) {
        const float bound_value = key_floor_value(bound32 & 0xFFFFFF00u);
#pragma unroll
        for (uint32_t e = kTkPer; e-- > 0u;) mine = mine + mine + (x[e] >= bound_value ? 1u : 0u);
    } else {
        // fewer than k threads hold a number (a literal state's row, say): every allowed token
        // is a candidate, a NaN too
#pragma unroll
        for (uint32_t j = 0; j < kPieces; j++) mine |= m[j] << (j * kPer);
    }
    // A candidate takes its place in the list with an LDS atomic of its own (there are few) and
    // leaves its token id there; which of its registers held the logit is not known at compile
    // time, so the rank keys are made from the ids afterwards, with the logit read again (it
    // is in the L2), one candidate per thread.
    while (mine) {
        const uint32_t e = (uint32_t)__builtin_ctz(mine);
        mine &= mine - 1u;
        const uint32_t at = atomicAdd(&sh.n_cand, 1u);
        if (at < kTkCand) sh.cand_id[at] = (base + (e / kPer) * kTkThreads + tid) * kPer + e % kPer;
    }
    __syncthreads();
    const bool exact = sh.n_cand > kTkCand;           // thousands of tokens tie at the bound, or are NaN
    if (!exact) {
        for (uint32_t i = tid; i < sh.n_cand; i += kTkThreads) {
            const uint32_t id = sh.cand_id[i];
            sh.cand[i] = ((unsigned long long)(order_key(__float_as_uint(elem_float(row[id]))) + 1u) << 32) | (0xFFFFFFFFu - id);
        }
        __syncthreads();
    } else {
        // Exact path: the thread maxima as rank keys.  k threads reach the k-th largest of them
        // and a thread holds 32 tokens, so at most 32 k tokens are at or above it: they always
        // fit the candidate list.  (Fewer than k threads with an allowed token: no bound, every
        // allowed token is a candidate, fewer than 32 k.)
        unsigned long long own = 0ull;
#pragma unroll
        for (uint32_t e = 0; e < kTkPer; e++) { const unsigned long long r = rank_key(e); own = r > own ? r : own; }
        const unsigned long long bound = kth_largest<unsigned long long>(sh, own, k);
        uint32_t mine = 0;
        if (own >= bound) {
#pragma unroll
            for (uint32_t e = 0; e < kTkPer; e++) { const unsigned long long r = rank_key(e); mine |= (uint32_t)(r != 0ull && r >= bound) << e; }
        }
        uint32_t pos = candidate_places(sh, (uint32_t)__popc(mine));
        if (mine) {
#pragma unroll
            for (uint32_t e = 0; e < kTkPer; e++)
                if ((mine >> e) & 1u) { if (pos < kTkCand) sh.cand[pos] = rank_key(e); pos++; }
        }
        __syncthreads();
    }
    // the candidates are ranked by counting; the best k leave, best first, zeros behind them
    const uint32_t n = sh.n_cand < kTkCand ? sh.n_cand : kTkCand;
    unsigned long long *out = lists + ((size_t)b * gridDim.x + blockIdx.x) * k;
    rank_candidates(sh, n, k, [&](uint32_t r, unsigned long long key) { out[r] = key; });
    for (uint32_t r = n + tid; r < k; r += kTkThreads) out[r] = 0ull;
}

template <typename Elem>
__global__ void __launch_bounds__(kTkThreads)
topk_merge_kernel(const Elem *__restrict__ logits, int64_t row_stride, uint32_t n_slices, uint32_t k,
                  const unsigned long long *__restrict__ lists, int32_t *__restrict__ ids,
                  Elem *__restrict__ values, Elem ninf)
{
    extern __shared__ unsigned long long all[];                   // the keys the row's slices left
    __shared__ TopkShared sh;
    const uint32_t b = blockIdx.x, tid = threadIdx.x, n = n_slices * k;   // n <= kTopkMergeKeys: at most 16 per thread
    unsigned long long own = 0ull;
    uint32_t held = 0;
    for (uint32_t i = tid; i < n; i += kTkThreads) {
        const unsigned long long x = lists[(size_t)b * n + i];
        all[i] = x;
        own = x > own ? x : own;
        held += x != 0ull;
    }
    const unsigned long long bound = kth_largest<unsigned long long>(sh, own, k);
    uint32_t c = 0;
    if (own >= bound)
        for (uint32_t i = tid; i < n; i += kTkThreads) c += all[i] != 0ull && all[i] >= bound;   // its own entries
    uint32_t pos = candidate_places(sh, c);
    if (c)
        for (uint32_t i = tid; i < n; i += kTkThreads)
            if (all[i] != 0ull && all[i] >= bound) { if (pos < kTkCand) sh.cand[pos] = all[i]; pos++; }
    if (held) atomicAdd(&sh.n_held, held);
    __syncthreads();
    const uint32_t n_cand = sh.n_cand < kTkCand ? sh.n_cand : kTkCand;
    rank_candidates(sh, n_cand, k, [&](uint32_t r, unsigned long long x) {
        const uint32_t id = 0xFFFFFFFFu - (uint32_t)x;
        ids[(size_t)b * k + r] = (int32_t)id;
        values[(size_t)b * k + r] = logits[(int64_t)b * row_stride + id];
    });
    // fewer than k allowed tokens in the row: the rest says so
    for (uint32_t r = (sh.n_held < k ? sh.n_held : k) + tid; r < k; r += kTkThreads) {
        ids[(size_t)b * k + r] = -1;
        values[(size_t)b * k + r] = ninf;
    }
}

// The address of `scratch` on the current device, asked of the runtime once per device.
hipError_t static_topk_scratch(unsigned long long **out)
{
    constexpr int kDevices = 64;
    static std::mutex mu;
    static unsigned long long *ptr[kDevices];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        ptr[dev] = static_cast<unsigned long long *>(p);
    }
    *out = ptr[dev];
    return hipSuccess;
}

hipError_t launch_masked_topk(const void *logits, int dtype, uint32_t B, uint32_t V, int64_t row_stride,
                              const uint32_t *bitmask, uint32_t k, int32_t *ids, void *values,
                              unsigned long long *lists, hipStream_t s)
{
    const uint32_t W = (V + 31u) / 32u;
    const size_t esz = dtype == WG_F32 ? 4 : 2;
    const bool vec_ok = reinterpret_cast<uintptr_t>(logits) % 16 == 0 && (row_stride * (int64_t)esz) % 16 == 0 && V % 8u == 0;
    const uint32_t n_slices = (V + kTopkSlice - 1u) / kTopkSlice;
    const dim3 g(n_slices, B);
    const uint32_t lds = n_slices * k * (uint32_t)sizeof(unsigned long long);
    if (dtype == WG_F32) {
        const uint32_t *x = static_cast<const uint32_t *>(logits);
        if (vec_ok) topk_slice_kernel<uint32_t, true><<<g, kTkThreads, 0, s>>>(x, row_stride, V, W, bitmask, k, lists);
        else topk_slice_kernel<uint32_t, false><<<g, kTkThreads, 0, s>>>(x, row_stride, V, W, bitmask, k, lists);
        topk_merge_kernel<uint32_t><<<B, kTkThreads, lds, s>>>(x, row_stride, n_slices, k, lists, ids,
                                                        static_cast<uint32_t *>(values), 0xFF800000u);
    } else {
        const uint16_t *x = static_cast<const uint16_t *>(logits);
        if (vec_ok) topk_slice_kernel<uint16_t, true><<<g, kTkThreads, 0, s>>>(x, row_stride, V, W, bitmask, k, lists);
        else topk_slice_kernel<uint16_t, false><<<g, kTkThreads, 0, s>>>(x, row_stride, V, W, bitmask, k, lists);
        topk_merge_kernel<uint16_t><<<B, kTkThreads, lds, s>>>(x, row_stride, n_slices, k, lists, ids,
                                                        static_cast<uint16_t *>(values), (uint16_t)0xFF80u);
    }
    return hipGetLastError();
}

}  // namespace wg
