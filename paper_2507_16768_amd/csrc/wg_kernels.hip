// HIP kernels of the structured-decoding hot path for gfx950 (wave64).
//
//   lookup   : request state -> cache key, claims missing keys            (B threads)
//   build    : one wavefront per (missing key, 64-token slice): every lane walks one
//              token's bytes through the operator FSM, a 64-lane ballot packs the
//              verdicts into two mask words
//   gather   : cached row -> bitmask[b]
//   apply    : logits <- -inf where the mask bit is 0
//   advance  : per-request walk of the sampled token
//   select   : harness sampler stand-in (k-th set bit of a row)
//
// No MFMA anywhere: the path is byte matching and memory traffic.
#include <hip/hip_runtime.h>

#include "wg_device.h"

namespace wg {

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

// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
lookup_kernel(DeviceTable T, DeviceCache Cc, const wg_state_t *__restrict__ states, uint32_t B)
{
    uint32_t b = blockIdx.x * blockDim.x + threadIdx.x;
    bool live = b < B, hit = false;
    if (live) {
        uint32_t sid = states[b].sid, aux = states[b].aux;
        uint32_t key = kNoKey;
        if (sid < T.n_states) {
            const StateDesc &d = T.states[sid];
            uint32_t variant = 0;
            if ((d.kind_byte & 0xFFu) == WG_KIND_WAIT && d.max != WG_UNBOUNDED) {
                uint32_t left = d.max > aux ? d.max - aux : 0u;
                variant = T.lmax - (left < T.lmax ? left : T.lmax);
            }
            key = d.key_base + variant;
            uint32_t epoch = Cc.ctr->epoch;
            uint32_t old = __hip_atomic_load(&Cc.built[key], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            hit = true;
            if (old != epoch && atomicCAS(&Cc.built[key], old, epoch) == old) {
                hit = false;                                // this thread owns the build
                uint32_t pos = atomicAdd(&Cc.ctr->n_miss, 1u);
                Cc.miss[pos] = MissEntry{key, sid, aux, 0u};
            } else if (old != epoch) hit = false;           // another request claimed it just now
        }
        Cc.key_of[b] = key;
    }
    unsigned long long hv = __ballot(hit), lv = __ballot(live);
    if ((threadIdx.x & 63u) == 0) {
        atomicAdd(&Cc.ctr->lookups, (unsigned long long)__popcll(lv));
        atomicAdd(&Cc.ctr->hits, (unsigned long long)__popcll(hv));
    }
}

// One wavefront per (missing key, 64 consecutive tokens); work items are strided over the
// grid so the launch size does not depend on the (device-side) number of misses.
__global__ void __launch_bounds__(256)
build_kernel(DeviceTable T, DeviceVocab Vc, DeviceCache Cc)
{
    const uint32_t n_miss = Cc.ctr->n_miss;
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t slices = (Vc.V + 63u) / 64u;             // 64-token slices per row
    const uint32_t waves_per_block = blockDim.x / 64u;
    const uint64_t total = (uint64_t)n_miss * slices;
    uint64_t w = (uint64_t)blockIdx.x * waves_per_block + (threadIdx.x >> 6);
    const uint64_t stride = (uint64_t)gridDim.x * waves_per_block;
    for (; w < total; w += stride) {
        uint32_t m = (uint32_t)(w % n_miss), slice = (uint32_t)(w / n_miss);
        MissEntry e = Cc.miss[m];
        uint32_t t = slice * 64u + lane;
        uint32_t sid = e.sid, aux = e.aux;
        bool ok = walk_token(T, Vc, sid, aux, (int64_t)t);
        unsigned long long bits = __ballot(ok);
        if (lane == 0) {
            uint32_t *row = Cc.arena + (size_t)e.key * Cc.row_stride;
            uint32_t w0 = slice * 2u;
            row[w0] = (uint32_t)bits;
            if (w0 + 1u < Vc.W) row[w0 + 1u] = (uint32_t)(bits >> 32);
        }
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) atomicAdd(&Cc.ctr->builds, (unsigned long long)n_miss);
}

__global__ void __launch_bounds__(256)
gather_kernel(DeviceCache Cc, uint32_t W, uint32_t *__restrict__ bitmask)
{
    uint32_t b = blockIdx.y;
    uint32_t key = Cc.key_of[b];
    const uint32_t *src = Cc.arena + (size_t)key * Cc.row_stride;
    uint32_t *dst = bitmask + (size_t)b * W;
    for (uint32_t w = blockIdx.x * blockDim.x + threadIdx.x; w < W; w += gridDim.x * blockDim.x)
        dst[w] = key == kNoKey ? 0u : src[w];
    // the miss list has been consumed by the build that ran before this kernel
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) Cc.ctr->n_miss = 0;
}

__global__ void clear_kernel(DeviceCache Cc) { Cc.ctr->epoch += 1u; }

// ---------------------------------------------------------------------------------------------
// apply: thread = 8 consecutive tokens = one mask byte.
template <typename Vec, int kVecs, typename Elem>
__global__ void __launch_bounds__(256)
apply_vec_kernel(Elem *__restrict__ logits, int64_t row_stride, uint32_t V, uint32_t W,
                 const uint32_t *__restrict__ bitmask, Elem ninf)
{
    uint32_t b = blockIdx.y;
    uint32_t g = blockIdx.x * blockDim.x + threadIdx.x;      // group of 8 tokens
    if (g * 8u >= V) return;
    uint32_t m = reinterpret_cast<const uint8_t *>(bitmask + (size_t)b * W)[g];
    if (m == 0xFFu) return;
    Elem *p = logits + (int64_t)b * row_stride + (int64_t)g * 8;
    union { Vec v[kVecs]; Elem e[8]; } u;
    Vec *pv = reinterpret_cast<Vec *>(p);
#pragma unroll
    for (int i = 0; i < kVecs; i++) u.v[i] = pv[i];
#pragma unroll
    for (int i = 0; i < 8; i++) if (!((m >> i) & 1u)) u.e[i] = ninf;
#pragma unroll
    for (int i = 0; i < kVecs; i++) pv[i] = u.v[i];
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
__global__ void __launch_bounds__(256)
advance_kernel(DeviceTable T, DeviceVocab Vc, DeviceCache Cc, wg_state_t *__restrict__ states,
               const int32_t *__restrict__ tokens, uint32_t B)
{
    uint32_t b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    uint32_t sid = states[b].sid, aux = states[b].aux;
    if (walk_token(T, Vc, sid, aux, (int64_t)tokens[b])) {
        states[b].sid = sid; states[b].aux = aux;
    } else {
        states[b].sid = WG_SID_ERROR; states[b].aux = 0;
        atomicAdd(&Cc.ctr->errors, 1ull);
    }
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

hipError_t launch_fill(const DeviceTable &T, const DeviceVocab &Vc, const DeviceCache &Cc,
                       const wg_state_t *states, uint32_t B, uint32_t *bitmask, uint32_t n_cu,
                       hipStream_t s)
{
    lookup_kernel<<<cdiv(B, 256), 256, 0, s>>>(T, Cc, states, B);
    uint32_t slices = (Vc.V + 63u) / 64u;
    uint64_t max_waves = (uint64_t)B * slices;
    uint32_t blocks = cdiv(max_waves, 4);
    uint32_t cap = n_cu * 8u;
    build_kernel<<<blocks < cap ? blocks : cap, 256, 0, s>>>(T, Vc, Cc);
    dim3 g(cdiv(Vc.W, 256 * 4), B);
    gather_kernel<<<g, 256, 0, s>>>(Cc, Vc.W, bitmask);
    return hipGetLastError();
}

hipError_t launch_clear(const DeviceCache &Cc, hipStream_t s)
{
    clear_kernel<<<1, 1, 0, s>>>(Cc);
    return hipGetLastError();
}

hipError_t launch_apply(void *logits, int dtype, uint32_t B, uint32_t V, int64_t row_stride,
                        const uint32_t *bitmask, hipStream_t s)
{
    uint32_t W = (V + 31u) / 32u;
    size_t esz = dtype == WG_F32 ? 4 : 2;
    bool vec_ok = (reinterpret_cast<uintptr_t>(logits) % 16 == 0) && ((row_stride * (int64_t)esz) % 16 == 0) &&
                  (V % 8u == 0);
    if (vec_ok) {
        dim3 g(cdiv(V / 8u, 256), B);
        if (dtype == WG_F32)
            apply_vec_kernel<uint4, 2, uint32_t><<<g, 256, 0, s>>>((uint32_t *)logits, row_stride, V, W, bitmask, 0xFF800000u);
        else
            apply_vec_kernel<uint4, 1, uint16_t><<<g, 256, 0, s>>>((uint16_t *)logits, row_stride, V, W, bitmask, (uint16_t)0xFF80u);
    } else {
        dim3 g(cdiv(V, 256), B);
        if (dtype == WG_F32)
            apply_scalar_kernel<uint32_t><<<g, 256, 0, s>>>((uint32_t *)logits, row_stride, V, W, bitmask, 0xFF800000u);
        else
            apply_scalar_kernel<uint16_t><<<g, 256, 0, s>>>((uint16_t *)logits, row_stride, V, W, bitmask, (uint16_t)0xFF80u);
    }
    return hipGetLastError();
}

hipError_t launch_advance(const DeviceTable &T, const DeviceVocab &Vc, const DeviceCache &Cc,
                          wg_state_t *states, const int32_t *tokens, uint32_t B, hipStream_t s)
{
    advance_kernel<<<cdiv(B, 256), 256, 0, s>>>(T, Vc, Cc, states, tokens, B);
    return hipGetLastError();
}

hipError_t launch_select(const uint32_t *bitmask, uint32_t B, uint32_t V, const uint64_t *draws,
                         int32_t *tokens, hipStream_t s)
{
    select_kernel<<<B, 256, 0, s>>>(bitmask, (V + 31u) / 32u, draws, tokens);
    return hipGetLastError();
}

}  // namespace wg
