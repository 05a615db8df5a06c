// Device-side building blocks shared by the forward, replay and backward kernels (gfx950,
// 64-lane wavefronts): the counter-based sampler and the 16/8/4/2-byte feature-row chunks.
// HIP path only; the CPU oracle has its own, separate implementation.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fsa_layout.h"

namespace fsa {

constexpr int kWave = 64;

// ---------------------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11).  Only output word 0 is consumed: one generator call
// per Floyd step, so a draw is a pure function of (seed, node, hop, step).
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t philox4x32_10_word0(uint32_t c0, uint32_t c1, uint32_t c2,
                                                        uint32_t c3, uint32_t k0, uint32_t k1) {
    constexpr uint32_t kMulA = 0xD2511F53u, kMulB = 0xCD9E8D57u;
    constexpr uint32_t kWeylA = 0x9E3779B9u, kWeylB = 0xBB67AE85u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        if (r) { k0 += kWeylA; k1 += kWeylB; }
        const uint64_t pa = (uint64_t)kMulA * c0, pb = (uint64_t)kMulB * c2;   // one 32x32->64 multiply each
        const uint32_t hiA = (uint32_t)(pa >> 32), loA = (uint32_t)pa;
        const uint32_t hiB = (uint32_t)(pb >> 32), loB = (uint32_t)pb;
        const uint32_t n0 = hiB ^ c1 ^ k0;
        const uint32_t n2 = hiA ^ c3 ^ k1;
        c0 = n0; c1 = loB; c2 = n2; c3 = loA;
    }
    return c0;
}

__device__ __forceinline__ uint64_t lanemask_lt(int lane) { return (1ull << lane) - 1ull; }

// ---------------------------------------------------------------------------------------
// Floyd's k-of-deg selection, one lane per step, for several rows at once.
//
// The wave is cut into segments of k consecutive lanes starting at seg_base; lane
// seg_base+li runs step li of its segment's row.  All 64 lanes must call this together
// (it ballots and goes through the wave's LDS draw strip); lanes without a row pass
// active=false.
//
// Sequential Floyd inserts t_i unless it is already chosen, else J_i = deg-k+i.  Whatever
// happens at step m, t_m is in the set afterwards, and J_m is in it exactly when step m
// collided; J_i exceeds everything chosen before step i.  So the set before step i is
// {t_m : m<i} U {J_m : m<i, step m collided}, and
//     collided_i = (exists m<i: t_m == t_i)  or  (t_i == J_m for an m<i with collided_m).
// The first term is a segment-wide compare; the second is resolved by ballot rounds that
// propagate collisions along the (acyclic, backward-pointing) J dependencies.
//
// Returns this lane's position inside the row (0-based), or -1 for an unused slot.
// deg <= k keeps the whole row in CSR order (Sec. 3.2: t = min(k, |N(v)|)).
// ---------------------------------------------------------------------------------------
// The generator word of Floyd step li of a node's row: a pure function of (seed, node, hop,
// step), so it can be drawn before the row's extent is known.
__device__ __forceinline__ uint32_t floyd_word(uint64_t seed, uint32_t node, uint32_t hop, int li) {
    return philox4x32_10_word0(node, hop, (uint32_t)li, 0u, (uint32_t)seed, (uint32_t)(seed >> 32));
}

// The draw of step li for a row of length deg (only meaningful when deg > k): uniform in [0, J_li].
__device__ __forceinline__ uint32_t floyd_bound(uint32_t word, int k, int li, int64_t deg) {
    return __umulhi(word, (uint32_t)(deg - k) + (uint32_t)li + 1u);
}

// Turn the draws of a segment into positions (see above).  `t` is this lane's draw; `draws`
// is the wave's LDS strip of kDrawStripInts ints (free to reuse when this returns).
__device__ __forceinline__ int64_t floyd_resolve(uint32_t t, int k, int li, int seg_base, int64_t deg,
                                                 bool active, int lane, int* draws) {
    const bool floyd = active && deg > (int64_t)k;
    const uint32_t base = floyd ? (uint32_t)(deg - k) : 0u;          // J_i = base + li
    bool collided = false;
    if (__any(floyd)) {                                              // wave-uniform
        // duplicate of an earlier draw of the same segment: every lane publishes its draw and
        // reads its segment back four entries at a time (entries at or beyond li never match
        // the m < li test, so the overshoot past the segment is harmless)
        draws[lane] = (int)t;
        __builtin_amdgcn_wave_barrier();
        const int* seg = draws + seg_base;
        bool dup_earlier = false;
        for (int m0 = 0; m0 < k; m0 += 4) {
            const uint32_t t0 = (uint32_t)seg[m0], t1 = (uint32_t)seg[m0 + 1];
            const uint32_t t2 = (uint32_t)seg[m0 + 2], t3 = (uint32_t)seg[m0 + 3];
            dup_earlier = dup_earlier || (m0 < li && t0 == t) || (m0 + 1 < li && t1 == t) ||
                          (m0 + 2 < li && t2 == t) || (m0 + 3 < li && t3 == t);
        }
        __builtin_amdgcn_wave_barrier();
        const bool hits_J = floyd && t >= base && (t - base) < (uint32_t)li;
        const int dep_lane = seg_base + (int)(t - base);
        // Least fixed point of  c_i = dup_i | (hits_J_i & c_dep(i)):  dependencies only point to
        // earlier steps, so iterating from the dup flags converges to the sequential answer,
        // usually in one or two rounds because chains of replaced values are rare.
        uint64_t done = __ballot(floyd && dup_earlier);
        for (;;) {
            const uint64_t more = __ballot(hits_J && ((done >> (dep_lane & 63)) & 1ull));
            if ((more & ~done) == 0ull) break;
            done |= more;
        }
        collided = (done >> lane) & 1ull;
    }
    if (floyd) return collided ? (int64_t)(base + (uint32_t)li) : (int64_t)t;
    return (active && (int64_t)li < deg) ? (int64_t)li : -1;
}

// Inclusive prefix sum over the 64 lanes: four row-shift steps inside each row of 16 lanes,
// then the totals of the lower rows are added to the rows above them.
__device__ __forceinline__ int wave_inclusive_scan(int v, int lane) {
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, true);   // row_shr:1, lanes shifted in read 0
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, true);   // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, true);   // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, true);   // row_shr:8
    const int r0 = __builtin_amdgcn_readlane(v, 15);
    const int r1 = __builtin_amdgcn_readlane(v, 31);
    const int r2 = __builtin_amdgcn_readlane(v, 47);
    const int row = lane >> 4;
    return v + (row >= 1 ? r0 : 0) + (row >= 2 ? r1 : 0) + (row >= 3 ? r2 : 0);
}

template <typename IT>
__device__ __forceinline__ int64_t load_indptr(const void* indptr, int64_t i) {
    return (int64_t) static_cast<const IT*>(indptr)[i];
}

// ---------------------------------------------------------------------------------------
// A chunk is what one lane loads from a feature row in one instruction: VB bytes = VE
// elements, widened to fp32 accumulators.
// ---------------------------------------------------------------------------------------
struct f32_t { float v; };
struct bf16_t { uint16_t v; };
struct f16_t { uint16_t v; };

template <int VB> struct RawOf;
template <> struct RawOf<16> { using type = uint4; };
template <> struct RawOf<8>  { using type = uint2; };
template <> struct RawOf<4>  { using type = uint32_t; };
template <> struct RawOf<2>  { using type = uint16_t; };

__device__ __forceinline__ float bits_f32(uint32_t u) { return __uint_as_float(u); }

// 1/n for a small positive count n: the hardware reciprocal is within 1 ulp, far inside the
// 1e-5 relative budget of the means, and turns VE divisions per mean into VE multiplies.
__device__ __forceinline__ float inv_count(int n) { return __builtin_amdgcn_rcpf((float)n); }

template <typename XT, int VB> struct Chunk;

template <int VB> struct Chunk<f32_t, VB> {
    static constexpr int VE = VB / 4;
    using Raw = typename RawOf<VB>::type;
    static __device__ __forceinline__ void add(float (&acc)[VE], const Raw& r) {
        if constexpr (VB == 16) { acc[0] += bits_f32(r.x); acc[1] += bits_f32(r.y); acc[2] += bits_f32(r.z); acc[3] += bits_f32(r.w); }
        else if constexpr (VB == 8) { acc[0] += bits_f32(r.x); acc[1] += bits_f32(r.y); }
        else { acc[0] += bits_f32(r); }
    }
    // acc += w * row chunk (weighted mean)
    static __device__ __forceinline__ void fma(float (&acc)[VE], const Raw& r, float w) {
        if constexpr (VB == 16) { acc[0] = fmaf(w, bits_f32(r.x), acc[0]); acc[1] = fmaf(w, bits_f32(r.y), acc[1]); acc[2] = fmaf(w, bits_f32(r.z), acc[2]); acc[3] = fmaf(w, bits_f32(r.w), acc[3]); }
        else if constexpr (VB == 8) { acc[0] = fmaf(w, bits_f32(r.x), acc[0]); acc[1] = fmaf(w, bits_f32(r.y), acc[1]); }
        else { acc[0] = fmaf(w, bits_f32(r), acc[0]); }
    }
    static __device__ __forceinline__ Raw pack(const float (&v)[VE]) {
        Raw r;
        if constexpr (VB == 16) { r.x = __float_as_uint(v[0]); r.y = __float_as_uint(v[1]); r.z = __float_as_uint(v[2]); r.w = __float_as_uint(v[3]); }
        else if constexpr (VB == 8) { r.x = __float_as_uint(v[0]); r.y = __float_as_uint(v[1]); }
        else { r = __float_as_uint(v[0]); }
        return r;
    }
};

template <int VB> struct Chunk<bf16_t, VB> {
    static constexpr int VE = VB / 2;
    using Raw = typename RawOf<VB>::type;
    static __device__ __forceinline__ void add2(float& lo, float& hi, uint32_t w) {
        lo += bits_f32(w << 16);
        hi += bits_f32(w & 0xffff0000u);
    }
    static __device__ __forceinline__ void add(float (&acc)[VE], const Raw& r) {
        if constexpr (VB == 16) { add2(acc[0], acc[1], r.x); add2(acc[2], acc[3], r.y); add2(acc[4], acc[5], r.z); add2(acc[6], acc[7], r.w); }
        else if constexpr (VB == 8) { add2(acc[0], acc[1], r.x); add2(acc[2], acc[3], r.y); }
        else if constexpr (VB == 4) { add2(acc[0], acc[1], r); }
        else { acc[0] += bits_f32(((uint32_t)r) << 16); }
    }
    static __device__ __forceinline__ void fma2(float& lo, float& hi, uint32_t v, float w) {
        lo = fmaf(w, bits_f32(v << 16), lo);
        hi = fmaf(w, bits_f32(v & 0xffff0000u), hi);
    }
    // acc += w * row chunk (weighted mean)
    static __device__ __forceinline__ void fma(float (&acc)[VE], const Raw& r, float w) {
        if constexpr (VB == 16) { fma2(acc[0], acc[1], r.x, w); fma2(acc[2], acc[3], r.y, w); fma2(acc[4], acc[5], r.z, w); fma2(acc[6], acc[7], r.w, w); }
        else if constexpr (VB == 8) { fma2(acc[0], acc[1], r.x, w); fma2(acc[2], acc[3], r.y, w); }
        else if constexpr (VB == 4) { fma2(acc[0], acc[1], r, w); }
        else { acc[0] = fmaf(w, bits_f32(((uint32_t)r) << 16), acc[0]); }
    }
    static __device__ __forceinline__ uint32_t pack2(float lo, float hi) {
        // fptrunc to bfloat16 is round-to-nearest-even; gfx950 does a pair per instruction
        typedef float f32x2 __attribute__((ext_vector_type(2)));
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        const f32x2 v = {lo, hi};
        const bf16x2 b = __builtin_convertvector(v, bf16x2);
        uint32_t u;
        __builtin_memcpy(&u, &b, sizeof u);
        return u;
    }
    static __device__ __forceinline__ Raw pack(const float (&v)[VE]) {
        Raw r;
        if constexpr (VB == 16) { r.x = pack2(v[0], v[1]); r.y = pack2(v[2], v[3]); r.z = pack2(v[4], v[5]); r.w = pack2(v[6], v[7]); }
        else if constexpr (VB == 8) { r.x = pack2(v[0], v[1]); r.y = pack2(v[2], v[3]); }
        else if constexpr (VB == 4) { r = pack2(v[0], v[1]); }
        else { r = (uint16_t)(pack2(v[0], 0.0f) & 0xffffu); }
        return r;
    }
};

// IEEE half: widened and narrowed a pair at a time by the hardware converts (narrowing is
// round-to-nearest-even).
template <int VB> struct Chunk<f16_t, VB> {
    static constexpr int VE = VB / 2;
    using Raw = typename RawOf<VB>::type;
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
    static __device__ __forceinline__ f32x2 widen(uint32_t w) {
        f16x2 h;
        __builtin_memcpy(&h, &w, sizeof h);
        return __builtin_convertvector(h, f32x2);
    }
    static __device__ __forceinline__ float widen1(uint16_t w) {
        _Float16 h;
        __builtin_memcpy(&h, &w, sizeof h);
        return (float)h;
    }
    static __device__ __forceinline__ void add2(float& lo, float& hi, uint32_t w) {
        const f32x2 f = widen(w);
        lo += f[0];
        hi += f[1];
    }
    static __device__ __forceinline__ void add(float (&acc)[VE], const Raw& r) {
        if constexpr (VB == 16) { add2(acc[0], acc[1], r.x); add2(acc[2], acc[3], r.y); add2(acc[4], acc[5], r.z); add2(acc[6], acc[7], r.w); }
        else if constexpr (VB == 8) { add2(acc[0], acc[1], r.x); add2(acc[2], acc[3], r.y); }
        else if constexpr (VB == 4) { add2(acc[0], acc[1], r); }
        else { acc[0] += widen1(r); }
    }
    static __device__ __forceinline__ void fma2(float& lo, float& hi, uint32_t v, float w) {
        const f32x2 f = widen(v);
        lo = fmaf(w, f[0], lo);
        hi = fmaf(w, f[1], hi);
    }
    // acc += w * row chunk (weighted mean)
    static __device__ __forceinline__ void fma(float (&acc)[VE], const Raw& r, float w) {
        if constexpr (VB == 16) { fma2(acc[0], acc[1], r.x, w); fma2(acc[2], acc[3], r.y, w); fma2(acc[4], acc[5], r.z, w); fma2(acc[6], acc[7], r.w, w); }
        else if constexpr (VB == 8) { fma2(acc[0], acc[1], r.x, w); fma2(acc[2], acc[3], r.y, w); }
        else if constexpr (VB == 4) { fma2(acc[0], acc[1], r, w); }
        else { acc[0] = fmaf(w, widen1(r), acc[0]); }
    }
    static __device__ __forceinline__ uint32_t pack2(float lo, float hi) {
        const f32x2 v = {lo, hi};
        const f16x2 h = __builtin_convertvector(v, f16x2);
        uint32_t u;
        __builtin_memcpy(&u, &h, sizeof u);
        return u;
    }
    static __device__ __forceinline__ Raw pack(const float (&v)[VE]) {
        Raw r;
        if constexpr (VB == 16) { r.x = pack2(v[0], v[1]); r.y = pack2(v[2], v[3]); r.z = pack2(v[4], v[5]); r.w = pack2(v[6], v[7]); }
        else if constexpr (VB == 8) { r.x = pack2(v[0], v[1]); r.y = pack2(v[2], v[3]); }
        else if constexpr (VB == 4) { r = pack2(v[0], v[1]); }
        else { r = (uint16_t)(pack2(v[0], 0.0f) & 0xffffu); }
        return r;
    }
};

// Sum the chunk at byte offset `chunk_off` of rows ids[first], ids[first+stride], ... (index
// below count) into acc, in that order; WEIGHTED multiplies each row by wts[i] and adds the
// weights into wsum.  Up to UNROLL row loads are issued before the first add so that their
// latencies overlap.  `ids` and `wts` live in LDS.
template <typename XT, int VB, int UNROLL, bool WEIGHTED>
__device__ __forceinline__ void sum_row_chunks(const char* __restrict__ x, int64_t row_bytes,
                                               int64_t chunk_off, const int* ids, const float* wts, int first,
                                               int count, int stride,
                                               float (&acc)[Chunk<XT, VB>::VE], float& wsum) {
    using C = Chunk<XT, VB>;
    using Raw = typename C::Raw;
    for (int i0 = first; i0 < count; i0 += stride * UNROLL) {
        Raw r[UNROLL];
        float wr[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int i = i0 + u * stride;
            if (i < count) {
                if constexpr (WEIGHTED) wr[u] = wts[i];
                r[u] = *reinterpret_cast<const Raw*>(x + (int64_t)ids[i] * row_bytes + chunk_off);
            }
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int i = i0 + u * stride;
            if (i < count) {
                if constexpr (WEIGHTED) { C::fma(acc, r[u], wr[u]); wsum += wr[u]; }
                else C::add(acc, r[u]);
            }
        }
    }
}

// Sum of the weights of the lanes of a segment that carry this lane's ID, and whether this
// lane is the first of them.
__device__ __forceinline__ void merge_equal_ids_w(int id, float w, int k, int li, int seg_base, float& wsum,
                                                  bool& first) {
    wsum = 0.0f;
    first = true;
    for (int m0 = 0; m0 < k; m0 += 4) {
        int other[4];
        float ow[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) { other[j] = __shfl(id, seg_base + m0 + j); ow[j] = __shfl(w, seg_base + m0 + j); }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (m0 + j < k && other[j] == id) { wsum += ow[j]; if (m0 + j < li) first = false; }
        }
    }
}

}  // namespace fsa
