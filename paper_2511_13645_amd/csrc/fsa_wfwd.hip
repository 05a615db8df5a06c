// Weighted-mean forward kernels (Sec. 3.2 of arXiv 2511.13645, "Extension Feasibility": the
// same early fusion with weighted numerators and denominators streamed per sampled
// neighborhood), sampling and replay variants, for gfx950.
//
// Sampling is exactly that of the unweighted kernels (same draws, same IDs); every sampled
// edge slot also brings its weight edge_w[row start + position].  The mapping is the
// unweighted one -- wave per seed (1-hop); workgroup per root whose waves own interleaved
// hop-1 slots, flat row-balanced leaf list in LDS, sub-groups streaming rows (2-hop) -- with
// a multiply-add per row and a running weight per slot instead of a count.  A slot whose
// weights sum to zero counts as empty.  Kept in a file of its own so that the unweighted
// kernels stay exactly as tuned.
#include "fsa_device.hip.h"
#include "fsa_internal.h"

#ifndef FSA_UNROLL
#define FSA_UNROLL 8
#endif

namespace fsa {

struct WFwdParams {
    const void* indptr; const int32_t* indices; const float* edge_w; const char* x;
    const int32_t* seeds; const int32_t* ids1; const int32_t* ids2; const float* w1; const float* w2;
    char* out; char* out_h1; int32_t* out_ids1; int32_t* out_ids2; float* out_w1; float* out_w2;
    int64_t B; int64_t row_bytes; uint64_t seed;
    int k1, k2, chunks, sub, sub_shift, indptr_is64;
};

__device__ __forceinline__ void w_row_extent(const WFwdParams& p, int64_t i, int64_t& start, int64_t& deg) {
    int64_t lo, hi;
    if (p.indptr_is64) {
        const int64_t* q = static_cast<const int64_t*>(p.indptr) + i;
        lo = q[0]; hi = q[1];
    } else {
        const int32_t* q = static_cast<const int32_t*>(p.indptr) + i;
        lo = q[0]; hi = q[1];
    }
    start = lo;
    deg = hi - lo;
}

// Hop 0: lane i < k1 gets the i-th sampled (or saved) hop-1 ID and the weight of that edge.
template <bool REPLAY>
__device__ __forceinline__ int w_hop0(const WFwdParams& p, int64_t b, int lane, float& w) {
    w = 0.0f;
    if constexpr (REPLAY) {
        if (lane >= p.k1) return -1;
        w = p.w1[b * p.k1 + lane];
        return p.ids1[b * p.k1 + lane];
    } else {
        const int64_t r = p.seeds[b];
        int64_t s, deg;
        w_row_extent(p, r, s, deg);
        const int64_t pos = floyd_position(p.seed, (uint32_t)r, 0u, p.k1, lane, 0, deg, lane < p.k1, lane);
        if (pos < 0) return -1;
        w = p.edge_w[s + pos];
        return p.indices[s + pos];
    }
}

// ---------------------------------------------------------------------------------------
// 1-hop: wave per seed
// ---------------------------------------------------------------------------------------
template <typename XT, int VB, bool REPLAY>
__global__ __launch_bounds__(256) void wfwd1_kernel(const WFwdParams p) {
    using C = Chunk<XT, VB>;
    using Raw = typename C::Raw;
    constexpr int VE = C::VE;
    constexpr int U = FSA_UNROLL;
    extern __shared__ int smem[];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int64_t b = (int64_t)blockIdx.x * (blockDim.x >> 6) + wave;
    if (b >= p.B) return;                       // wave-uniform; no block barrier below
    int* ids = smem + wave * 2 * kWave;
    float* wts = reinterpret_cast<float*>(ids + kWave);

    float w;
    const int id = w_hop0<REPLAY>(p, b, lane, w);
    if (!REPLAY && lane < p.k1) {
        if (p.out_ids1) p.out_ids1[b * p.k1 + lane] = id;
        if (p.out_w1) p.out_w1[b * p.k1 + lane] = id >= 0 ? w : 0.0f;
    }
    const uint64_t valid = __ballot(id >= 0);
    const int cnt = __popcll(valid);
    if (id >= 0) {
        const int slot = __popcll(valid & lanemask_lt(lane));
        ids[slot] = id;
        wts[slot] = w;
    }
    __builtin_amdgcn_wave_barrier();

    const int sub = p.sub;
    const int sg = lane >> p.sub_shift;
    const int sl = lane & (sub - 1);
    const int nsg = kWave >> p.sub_shift;
    for (int c0 = 0; c0 < p.chunks; c0 += sub) {
        const int chunk = c0 + sl;
        const bool live = chunk < p.chunks;
        const int64_t load_off = live ? (int64_t)chunk * VB : 0;
        float acc[VE];
#pragma unroll
        for (int e = 0; e < VE; ++e) acc[e] = 0.0f;
        float wsum = 0.0f;
        // rows sg, sg+nsg, ...; past the end the last row is re-read and not accumulated
        const int n_mine = cnt > sg ? (cnt - sg + nsg - 1) / nsg : 0;
        for (int i0 = 0; i0 < n_mine; i0 += U) {
            Raw r[U];
            float wr[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int i = sg + (i0 + u < n_mine ? i0 + u : n_mine - 1) * nsg;
                wr[u] = wts[i];
                r[u] = *reinterpret_cast<const Raw*>(p.x + (int64_t)ids[i] * p.row_bytes + load_off);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (i0 + u < n_mine) { C::fma(acc, r[u], wr[u]); wsum += wr[u]; }
            }
        }
        for (int off = sub; off < kWave; off <<= 1) {
#pragma unroll
            for (int e = 0; e < VE; ++e) acc[e] += __shfl_xor(acc[e], off);
            wsum += __shfl_xor(wsum, off);
        }
        if (sg == 0 && live) {
            const float inv = wsum > 0.0f ? __builtin_amdgcn_rcpf(wsum) : 0.0f;
#pragma unroll
            for (int e = 0; e < VE; ++e) acc[e] = wsum > 0.0f ? acc[e] * inv : 0.0f;
            *reinterpret_cast<Raw*>(p.out + b * p.row_bytes + (int64_t)chunk * VB) = C::pack(acc);
        }
    }
}

// ---------------------------------------------------------------------------------------
// 2-hop: workgroup per root, waves own interleaved hop-1 slots
// ---------------------------------------------------------------------------------------
constexpr int kWPassGroup = 4;

// MT > 0: rows of 2 .. MT tiles of 64 lanes, all tiles of a row loaded back to back (the same
// wide-row gather as the unweighted kernel); MT = 0: one list walk per tile.
constexpr int kWMultiTiles = 8;

template <typename XT, int VB, bool REPLAY, int MT>
__global__ __launch_bounds__(512) void wfwd2_kernel(const WFwdParams p) {
    using C = Chunk<XT, VB>;
    using Raw = typename C::Raw;
    constexpr int VE = C::VE;
    constexpr int U = FSA_UNROLL;
    extern __shared__ int smem[];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int nw = blockDim.x >> 6;
    const int64_t b = blockIdx.x;
    const int k1 = p.k1, k2 = p.k2;

    // LDS per wave (n = nq_max*k2): flat row offsets int2 [n], slot-end records [n], flat
    // weights [n], leaf IDs by slot [n], leaf weights by slot [n], per-slot count [nq_max],
    // empty-slot list [nq_max], hop-0 weight of each slot [nq_max] (+1 pad if odd); then per
    // wave one outer-weight partial and [sub*VE] floats for the cross-wave reduction.
    const int nq_max = (k1 + nw - 1) / nw;
    const int n = nq_max * k2;
    const int per_wave = (6 * n + 3 * nq_max + 1) & ~1;
    int* base = smem + wave * per_wave;
    int2* flat = reinterpret_cast<int2*>(base);
    int* flat_meta = base + 2 * n;
    float* flat_w = reinterpret_cast<float*>(base + 3 * n);
    int* leaf = base + 4 * n;
    float* leaf_w = reinterpret_cast<float*>(base + 5 * n);
    int* cnt2 = base + 6 * n;
    int* empty_q = cnt2 + nq_max;
    float* slot_a = reinterpret_cast<float*>(empty_q + nq_max);
    float* red_w = reinterpret_cast<float*>(smem + nw * per_wave);
    float* red = red_w + nw;

    float a_mine;
    const int u_mine = w_hop0<REPLAY>(p, b, lane, a_mine);
    if (!REPLAY && wave == 0 && lane < k1) {
        if (p.out_ids1) p.out_ids1[b * k1 + lane] = u_mine;
        if (p.out_w1) p.out_w1[b * k1 + lane] = u_mine >= 0 ? a_mine : 0.0f;
    }

    const int nq = wave < k1 ? (k1 - wave + nw - 1) / nw : 0;
    const int own_src = lane < nq ? wave + lane * nw : 0;
    const int u_own = __shfl(u_mine, own_src);
    const float a_own = __shfl(a_mine, own_src);
    if (lane < nq) slot_a[lane] = a_own;
    const int spw = kWave / k2;
    const int g = lane / k2;
    const int li = lane - g * k2;
    const uint64_t seg_mask = k2 == 64 ? ~0ull : ((1ull << k2) - 1ull);
    int64_t s_own = 0;
    uint32_t deg_own = 0;
    if constexpr (!REPLAY) {
        if (lane < nq && u_own >= 0) {
            int64_t d;
            w_row_extent(p, u_own, s_own, d);
            deg_own = (uint32_t)d;
        }
    }
    // leaf IDs and weights of the owned slots, squeezed to the front of each slot
    for (int q0 = 0; q0 < nq; q0 += kWPassGroup * spw) {            // wave-uniform trip count
        int idv[kWPassGroup];
        float wv[kWPassGroup];
#pragma unroll
        for (int t = 0; t < kWPassGroup; ++t) {
            idv[t] = -1;
            wv[t] = 0.0f;
            if (q0 + t * spw < nq) {                                 // wave-uniform
                const int q = q0 + t * spw + g;
                const bool valid = g < spw && q < nq;
                const int src = valid ? q : 0;
                const int u = __shfl(u_own, src);
                const bool active = valid && u >= 0;
                if constexpr (REPLAY) {
                    if (active) {
                        idv[t] = p.ids2[(b * k1 + wave + q * nw) * k2 + li];
                        wv[t] = p.w2[(b * k1 + wave + q * nw) * k2 + li];
                    }
                } else {
                    const uint32_t s_lo = __shfl((uint32_t)s_own, src);
                    const uint32_t s_hi = __shfl((uint32_t)((uint64_t)s_own >> 32), src);
                    const int64_t s = (int64_t)(((uint64_t)s_hi << 32) | s_lo);
                    const int64_t deg = (int64_t)__shfl(deg_own, src);
                    const int64_t pos = floyd_position(p.seed, (uint32_t)u, 1u, k2, li, valid ? g * k2 : 0,
                                                       deg, active, lane);
                    if (pos >= 0) {
                        idv[t] = p.indices[s + pos];
                        wv[t] = p.edge_w[s + pos];
                    }
                }
            }
        }
#pragma unroll
        for (int t = 0; t < kWPassGroup; ++t) {
            if (q0 + t * spw < nq) {
                const int q = q0 + t * spw + g;
                const bool valid = g < spw && q < nq;
                if (!REPLAY && valid) {
                    const int64_t at = (b * k1 + wave + q * nw) * k2 + li;
                    if (p.out_ids2) p.out_ids2[at] = idv[t];
                    if (p.out_w2) p.out_w2[at] = idv[t] >= 0 ? wv[t] : 0.0f;
                }
                const uint64_t have = __ballot(valid && idv[t] >= 0) & (seg_mask << (valid ? g * k2 : 0));
                if (valid && idv[t] >= 0) {
                    const int slot = q * k2 + __popcll(have & lanemask_lt(lane));
                    leaf[slot] = idv[t];
                    leaf_w[slot] = wv[t];
                }
                if (valid && li == 0) cnt2[q] = __popcll(have);
            }
        }
    }
    __builtin_amdgcn_wave_barrier();
    const int c_own = lane < nq ? cnt2[lane] : 0;

    // place of each slot's rows in the flat list; row-balanced blocks of slots per sub-group
    int incl = c_own;
    for (int d = 1; d < nq; d <<= 1) {
        const int up = __shfl_up(incl, d);
        if (lane >= d) incl += up;
    }
    const int off_own = incl - c_own;
    const int total = __shfl(incl, nq > 0 ? nq - 1 : 0);
    const uint64_t empty_mask = __ballot(lane < nq && c_own == 0);
    const int n_empty = __popcll(empty_mask);
    if (lane < nq && c_own == 0) empty_q[__popcll(empty_mask & lanemask_lt(lane))] = lane;

    const int sub = p.sub;
    const int sg = lane >> p.sub_shift;
    const int sl = lane & (sub - 1);
    const int nsg = kWave >> p.sub_shift;
    int qa = 0, qb = 0;
    for (int s = 0; s <= nsg; ++s) {                                 // wave-uniform
        const int first_q = __popcll(__ballot(lane < nq && off_own * nsg < s * total));
        if (s == sg) qa = first_q;
        if (s == sg + 1) qb = first_q;
    }
    if (sg == nsg - 1) qb = nq;
    const int start_a = __shfl(off_own, qa < nq ? qa : 0);
    const int start_b = __shfl(off_own, qb < nq ? qb : 0);
    const int my_start = qa < nq ? start_a : total;
    const int my_len = (qb < nq ? start_b : total) - my_start;

    for (int q0 = 0; q0 < nq; q0 += spw) {
        const int q = q0 + g;
        const bool valid = g < spw && q < nq;
        const int off = __shfl(off_own, valid ? q : 0);
        const int c = __shfl(c_own, valid ? q : 0);
        if (valid && li < c) {
            const int at = off + li;
            const uint32_t last = li == c - 1 ? 1u : 0u;
            const uint64_t row_off = (uint64_t)(uint32_t)leaf[q * k2 + li] * (uint64_t)p.row_bytes;
            flat[at] = make_int2((int)(uint32_t)row_off, (int)((uint32_t)(row_off >> 32) | (last << 31)));
            flat_w[at] = leaf_w[q * k2 + li];
            if (last) flat_meta[at] = (wave + q * nw) | (q << 8);
        }
    }
    __builtin_amdgcn_wave_barrier();

    if constexpr (MT > 0) {
        // sub == 64: the wave walks its whole list, one row (all its tiles) at a time
        const int tiles = (p.chunks + kWave - 1) >> 6;
        float acc[MT][VE], root[MT][VE];
#pragma unroll
        for (int t = 0; t < MT; ++t) {
#pragma unroll
            for (int e = 0; e < VE; ++e) { acc[t][e] = 0.0f; root[t][e] = 0.0f; }
        }
        float wacc = 0.0f, rootw = 0.0f;
        if (p.out_h1) {                                              // empty slots get zero rows
            for (int i = 0; i < n_empty; ++i) {
                char* dst = p.out_h1 + (b * k1 + wave + empty_q[i] * nw) * p.row_bytes;
                for (int chunk = lane; chunk < p.chunks; chunk += kWave)
                    *reinterpret_cast<Raw*>(dst + (int64_t)chunk * VB) = C::pack(acc[0]);
            }
        }
        for (int i = 0; i < total; ++i) {
            const int2 ent = flat[i];
            const float wr = flat_w[i];
            const uint64_t row_off = ((uint64_t)((uint32_t)ent.y & 0x7fffffffu) << 32) | (uint32_t)ent.x;
            Raw r[MT];
#pragma unroll
            for (int t = 0; t < MT; ++t) {
                if (t < tiles) {                                     // wave-uniform
                    const int chunk = t * kWave + lane;              // lanes past the row width re-read chunk 0
                    r[t] = *reinterpret_cast<const Raw*>(p.x + row_off + (chunk < p.chunks ? (int64_t)chunk * VB : 0));
                }
            }
#pragma unroll
            for (int t = 0; t < MT; ++t)
                if (t < tiles) C::fma(acc[t], r[t], wr);
            wacc += wr;
            if (ent.y < 0) {                                         // last row of its slot
                const int meta = flat_meta[i];
                const float a = slot_a[meta >> 8];
                const bool part = wacc > 0.0f;
                const float inv = part ? __builtin_amdgcn_rcpf(wacc) : 0.0f;
                char* dst = p.out_h1 ? p.out_h1 + (b * k1 + (meta & 0xff)) * p.row_bytes : nullptr;
#pragma unroll
                for (int t = 0; t < MT; ++t) {
                    if (t < tiles) {
                        const int chunk = t * kWave + lane;
#pragma unroll
                        for (int e = 0; e < VE; ++e) {
                            acc[t][e] = part ? acc[t][e] * inv : 0.0f;
                            root[t][e] = fmaf(part ? a : 0.0f, acc[t][e], root[t][e]);
                        }
                        if (dst && chunk < p.chunks)
                            *reinterpret_cast<Raw*>(dst + (int64_t)chunk * VB) = C::pack(acc[t]);
#pragma unroll
                        for (int e = 0; e < VE; ++e) acc[t][e] = 0.0f;
                    }
                }
                rootw += part ? a : 0.0f;
                wacc = 0.0f;
            }
        }
        if (nw > 1 && lane == 0) red_w[wave] = rootw;
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            if (t < tiles) {                                         // workgroup-uniform
                const int chunk = t * kWave + lane;
                const bool live = chunk < p.chunks;
                if (nw == 1) {
                    const float inv1 = rootw > 0.0f ? __builtin_amdgcn_rcpf(rootw) : 0.0f;
#pragma unroll
                    for (int e = 0; e < VE; ++e) root[t][e] = rootw > 0.0f ? root[t][e] * inv1 : 0.0f;
                    if (live) *reinterpret_cast<Raw*>(p.out + b * p.row_bytes + (int64_t)chunk * VB) = C::pack(root[t]);
                } else {
#pragma unroll
                    for (int e = 0; e < VE; ++e) red[(wave * kWave + lane) * VE + e] = root[t][e];
                    __syncthreads();
                    if (wave == 0) {
                        float tot[VE];
#pragma unroll
                        for (int e = 0; e < VE; ++e) tot[e] = 0.0f;
                        float totw = 0.0f;
                        for (int w = 0; w < nw; ++w) {
#pragma unroll
                            for (int e = 0; e < VE; ++e) tot[e] += red[(w * kWave + lane) * VE + e];
                            totw += red_w[w];
                        }
                        const float inv1 = totw > 0.0f ? __builtin_amdgcn_rcpf(totw) : 0.0f;
#pragma unroll
                        for (int e = 0; e < VE; ++e) tot[e] = totw > 0.0f ? tot[e] * inv1 : 0.0f;
                        if (live) *reinterpret_cast<Raw*>(p.out + b * p.row_bytes + (int64_t)chunk * VB) = C::pack(tot);
                    }
                    __syncthreads();                                 // red is reused by the next tile
                }
            }
        }
        return;
    }

    for (int c0 = 0; c0 < p.chunks; c0 += sub) {
        const int chunk = c0 + sl;
        const bool live = chunk < p.chunks;
        const int64_t chunk_off = (int64_t)chunk * VB;
        const int64_t load_off = live ? chunk_off : 0;
        float acc[VE], root[VE];
#pragma unroll
        for (int e = 0; e < VE; ++e) { acc[e] = 0.0f; root[e] = 0.0f; }
        float wacc = 0.0f, rootw = 0.0f;
        if (p.out_h1 && live) {                                      // empty slots get zero rows
            for (int i = sg; i < n_empty; i += nsg)
                *reinterpret_cast<Raw*>(p.out_h1 + (b * k1 + wave + empty_q[i] * nw) * p.row_bytes + chunk_off) = C::pack(acc);
        }
        for (int i0 = 0; i0 < my_len; i0 += U) {
            int2 ent[U];
            float wr[U];
            Raw r[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int i = i0 + u < my_len ? i0 + u : my_len - 1;
                ent[u] = flat[my_start + i];
                wr[u] = flat_w[my_start + i];
                const uint64_t row_off = ((uint64_t)((uint32_t)ent[u].y & 0x7fffffffu) << 32) | (uint32_t)ent[u].x;
                r[u] = *reinterpret_cast<const Raw*>(p.x + row_off + load_off);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (i0 + u < my_len) {
                    C::fma(acc, r[u], wr[u]);
                    wacc += wr[u];
                    if (ent[u].y < 0) {                              // last row of its slot
                        const int meta = flat_meta[my_start + i0 + u];
                        const float a = slot_a[meta >> 8];
                        const bool part = wacc > 0.0f;
                        const float inv = part ? __builtin_amdgcn_rcpf(wacc) : 0.0f;
#pragma unroll
                        for (int e = 0; e < VE; ++e) {
                            acc[e] = part ? acc[e] * inv : 0.0f;
                            root[e] = fmaf(part ? a : 0.0f, acc[e], root[e]);
                        }
                        rootw += part ? a : 0.0f;
                        if (live && p.out_h1)
                            *reinterpret_cast<Raw*>(p.out_h1 + (b * k1 + (meta & 0xff)) * p.row_bytes + chunk_off) = C::pack(acc);
#pragma unroll
                        for (int e = 0; e < VE; ++e) acc[e] = 0.0f;
                        wacc = 0.0f;
                    }
                }
            }
        }
        // every lane of a sub-group carries the same rootw: reduce across sub-groups only
        for (int off = sub; off < kWave; off <<= 1) {
#pragma unroll
            for (int e = 0; e < VE; ++e) root[e] += __shfl_xor(root[e], off);
            rootw += __shfl_xor(rootw, off);
        }
        if (nw == 1) {
            if (sg == 0 && live) {
                const float inv1 = rootw > 0.0f ? __builtin_amdgcn_rcpf(rootw) : 0.0f;
#pragma unroll
                for (int e = 0; e < VE; ++e) root[e] = rootw > 0.0f ? root[e] * inv1 : 0.0f;
                *reinterpret_cast<Raw*>(p.out + b * p.row_bytes + chunk_off) = C::pack(root);
            }
            continue;
        }
        if (sg == 0) {
#pragma unroll
            for (int e = 0; e < VE; ++e) red[(wave * sub + sl) * VE + e] = root[e];
            if (sl == 0) red_w[wave] = rootw;
        }
        __syncthreads();
        if (wave == 0 && sg == 0 && live) {
            float tot[VE];
#pragma unroll
            for (int e = 0; e < VE; ++e) tot[e] = 0.0f;
            float totw = 0.0f;
            for (int w = 0; w < nw; ++w) {
#pragma unroll
                for (int e = 0; e < VE; ++e) tot[e] += red[(w * sub + sl) * VE + e];
                totw += red_w[w];
            }
            const float inv1 = totw > 0.0f ? __builtin_amdgcn_rcpf(totw) : 0.0f;
#pragma unroll
            for (int e = 0; e < VE; ++e) tot[e] = totw > 0.0f ? tot[e] * inv1 : 0.0f;
            *reinterpret_cast<Raw*>(p.out + b * p.row_bytes + chunk_off) = C::pack(tot);
        }
        if (c0 + sub < p.chunks) __syncthreads();       // red is reused by the next tile
    }
}

// ---------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------
template <typename XT, int VB>
static hipError_t launch_typed_w(const FwdArgs& a, const WFwdParams& p, hipStream_t stream) {
    constexpr int VE = Chunk<XT, VB>::VE;
    const bool replay = a.indptr == nullptr;
    if (a.hops == 1) {
        const int wpb = 4;
        const unsigned grid = (unsigned)((a.B + wpb - 1) / wpb);
        const size_t lds = sizeof(int) * 2 * kWave * wpb;
        if (replay) hipLaunchKernelGGL((wfwd1_kernel<XT, VB, true>), dim3(grid), dim3(wpb * kWave), lds, stream, p);
        else        hipLaunchKernelGGL((wfwd1_kernel<XT, VB, false>), dim3(grid), dim3(wpb * kWave), lds, stream, p);
    } else {
        int nw = 1;
        while (nw < 8 && nw * 2 <= a.k1 && a.B * nw < 4096) nw *= 2;
        const int nq_max = (a.k1 + nw - 1) / nw;
        const size_t per_wave = ((size_t)6 * nq_max * a.k2 + 3 * nq_max + 1) & ~(size_t)1;
        const size_t lds = sizeof(int) * (nw * per_wave + nw) + sizeof(float) * (size_t)nw * a.geom.sub * VE;
        const dim3 grid((unsigned)a.B), block(nw * kWave);
        const int tiles = a.geom.tiles;
#define FSA_LAUNCH_WFWD2(MT_)                                                                                  \
        do {                                                                                                   \
            if (replay) hipLaunchKernelGGL((wfwd2_kernel<XT, VB, true, MT_>), grid, block, lds, stream, p);    \
            else        hipLaunchKernelGGL((wfwd2_kernel<XT, VB, false, MT_>), grid, block, lds, stream, p);   \
        } while (0)
        if (tiles <= 1 || tiles > kWMultiTiles) FSA_LAUNCH_WFWD2(0);
        else if (tiles <= 4) FSA_LAUNCH_WFWD2(4);
        else FSA_LAUNCH_WFWD2(8);
#undef FSA_LAUNCH_WFWD2
    }
    return hipGetLastError();
}

hipError_t launch_forward_weighted(const FwdArgs& a, const WeightArgs& w, hipStream_t stream) {
    WFwdParams p;
    p.indptr = a.indptr; p.indices = a.indices; p.edge_w = w.edge_w; p.x = static_cast<const char*>(a.x);
    p.seeds = a.seeds; p.ids1 = a.ids1; p.ids2 = a.ids2; p.w1 = w.w1; p.w2 = w.w2;
    p.out = static_cast<char*>(a.out); p.out_h1 = static_cast<char*>(a.out_h1);
    p.out_ids1 = a.out_ids1; p.out_ids2 = a.out_ids2; p.out_w1 = w.out_w1; p.out_w2 = w.out_w2;
    p.B = a.B; p.row_bytes = a.D * (a.x_kind == 0 ? 4 : 2); p.seed = a.seed;
    p.k1 = a.k1; p.k2 = a.k2; p.chunks = a.geom.chunks; p.sub = a.geom.sub;
    p.sub_shift = __builtin_ctz((unsigned)a.geom.sub); p.indptr_is64 = a.indptr_is64;
    const int vb = a.geom.vec_bytes;
    if (a.x_kind == 1) {
        switch (vb) {
            case 16: return launch_typed_w<bf16_t, 16>(a, p, stream);
            case 8:  return launch_typed_w<bf16_t, 8>(a, p, stream);
            case 4:  return launch_typed_w<bf16_t, 4>(a, p, stream);
            default: return launch_typed_w<bf16_t, 2>(a, p, stream);
        }
    }
    if (a.x_kind == 2) {
        switch (vb) {
            case 16: return launch_typed_w<f16_t, 16>(a, p, stream);
            case 8:  return launch_typed_w<f16_t, 8>(a, p, stream);
            case 4:  return launch_typed_w<f16_t, 4>(a, p, stream);
            default: return launch_typed_w<f16_t, 2>(a, p, stream);
        }
    }
    switch (vb) {
        case 16: return launch_typed_w<f32_t, 16>(a, p, stream);
        case 8:  return launch_typed_w<f32_t, 8>(a, p, stream);
        default: return launch_typed_w<f32_t, 4>(a, p, stream);
    }
}

}  // namespace fsa
