// Forward kernels: fused sample + mean (Sec. 3.2 of arXiv 2511.13645) and the replay
// forward from saved IDs (Sec. 3.3, Prop. 1), for gfx950.
//
// Mapping (the paper's Sec. 4 uses warp-per-seed / block-per-root on 32-wide warps; this is
// the 64-wide-wavefront re-derivation):
//   1-hop: one wavefront per seed.  Lane i runs Floyd step i; the sampled IDs are staged in
//          a wave-private LDS strip; the wave is cut into 64/sub sub-groups of `sub` lanes,
//          each sub-group covers one feature row with 16/8/4-byte loads and the sub-groups
//          take different neighbor rows, so several rows are in flight per instruction.
//   2-hop: one workgroup per root, by default a single wave (more waves, each owning a
//          subset of the hop-1 slots, only for small batches).  The wave draws the hop-1
//          IDs (k1 lanes), reads their row extents (one lane per slot), samples their rows
//          in segments of k2 lanes (64/k2 rows per pass) and writes every sampled leaf ID
//          straight into a flat, row-balanced list in LDS; sub-groups then stream the
//          listed rows eight loads deep, closing a slot (mean -> out_h1, add to the root
//          sum) whenever a flagged entry goes by.  The root mean is reduced by shuffles
//          (and through LDS across waves) and written once.  No [B,k,D] gathered tensor
//          and no block structure ever exists.
// The replay kernels are the same code with the sampler swapped for loads of the saved IDs,
// which is what makes replay bitwise equal to the sampling forward.
#include "fsa_device.hip.h"
#include "fsa_internal.h"

#include <cstdlib>

#ifndef FSA_UNROLL
#define FSA_UNROLL 8
#endif
#ifndef FSA_PASS_GROUP
#define FSA_PASS_GROUP 4
#endif
#ifndef FSA_MULTI_LOADS
#define FSA_MULTI_LOADS 8
#endif
#ifndef FSA_FWD2_MIN_WAVES_PER_EU
#define FSA_FWD2_MIN_WAVES_PER_EU 1
#endif

namespace fsa {

struct FwdParams {
    const void* indptr; const int32_t* indices; const char* x;
    const int32_t* seeds; const int32_t* ids1; const int32_t* ids2;
    char* out; char* out_h1; int32_t* out_ids1; int32_t* out_ids2;
    int64_t B; int64_t row_bytes; uint64_t seed;
    int k1, k2, chunks, sub, sub_shift, indptr_is64;
    uint32_t hop_base;                      // hop counter of the seeds' own rows (0 unless chained)
    int32_t* out_live;                      // 2-hop, nullable: [B] hop-1 slots that took part
    const int32_t* slot_cnt;                // slot-mean kernel only: [B,k1] counts, > 0 = takes part
#ifdef FSA_TRACE
    long long* trace;                       // debug builds: [B][8] wall-clock stamps (10 ns units)
#endif
};

#ifdef FSA_TRACE
#define FSA_STAMP(slot) do { if (p.trace && threadIdx.x == 0) p.trace[blockIdx.x * 8 + (slot)] = wall_clock64(); } while (0)
#else
#define FSA_STAMP(slot) do { } while (0)
#endif

// Row start and length of node i: both indptr entries are requested before either is used.
__device__ __forceinline__ void row_extent(const FwdParams& p, int64_t i, int64_t& start, int64_t& deg) {
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

// Hop-0 step shared by both kernels: lane i < k1 ends up with the i-th sampled (or saved)
// hop-1 ID of root slot b, -1 in unused slots.  Replay keeps the saved layout (holes stay).
template <bool REPLAY>
__device__ __forceinline__ int hop0_id(const FwdParams& p, int64_t b, int lane) {
    if constexpr (REPLAY) {
        // chained calls pass the level above as `seeds`: a negative entry switches the root off
        if (p.seeds && p.seeds[b] < 0) return -1;
        return lane < p.k1 ? p.ids1[b * p.k1 + lane] : -1;
    } else {
        // a negative seed (an unused slot of the level above, when calls are chained) is an
        // empty row: nothing is read for it
        const int64_t r = p.seeds[b];
        int64_t s, deg;
        row_extent(p, r >= 0 ? r : 0, s, deg);
        if (r < 0) deg = 0;
        const int64_t pos = floyd_position(p.seed, (uint32_t)r, p.hop_base, p.k1, lane, 0, deg,
                                           lane < p.k1, lane);
        return pos >= 0 ? p.indices[s + pos] : -1;
    }
}

// One wave: mean of the rows of p.x named by the lanes' non-negative `id`s, in lane order,
// written to `dst`.  `ids` is the wave's LDS strip of 64 ints.
template <typename XT, int VB, int MT>
__device__ __forceinline__ void wave_mean_of_rows(const FwdParams& p, int id, int* ids, int lane, char* dst) {
    using C = Chunk<XT, VB>;
    constexpr int VE = C::VE;
    // stage the valid IDs, in slot order, in this wave's LDS strip
    const uint64_t valid = __ballot(id >= 0);
    const int cnt = __popcll(valid);
    if (id >= 0) ids[__popcll(valid & lanemask_lt(lane))] = id;
    __builtin_amdgcn_wave_barrier();

    if constexpr (MT > 0) {
        // rows of 2 .. MT tiles of 64 lanes: all tiles of a row are loaded back to back, so a
        // cache line shared by neighbouring tiles is fetched once
        using Raw = typename C::Raw;
        constexpr int R = FSA_MULTI_LOADS / MT;                    // rows in flight
        const int tiles = (p.chunks + kWave - 1) >> 6;
        const float inv = inv_count(cnt > 0 ? cnt : 1);
        float acc[MT][VE];
#pragma unroll
        for (int t = 0; t < MT; ++t) {
#pragma unroll
            for (int e = 0; e < VE; ++e) acc[t][e] = 0.0f;
        }
        for (int i0 = 0; i0 < cnt; i0 += R) {
            Raw r[R][MT];
#pragma unroll
            for (int u = 0; u < R; ++u) {
                const int64_t row_off = (int64_t)ids[i0 + u < cnt ? i0 + u : cnt - 1] * p.row_bytes;
#pragma unroll
                for (int t = 0; t < MT; ++t) {
                    if (t < tiles) {                               // wave-uniform
                        const int chunk = t * kWave + lane;        // lanes past the row width re-read chunk 0
                        r[u][t] = *reinterpret_cast<const Raw*>(p.x + row_off + (chunk < p.chunks ? (int64_t)chunk * VB : 0));
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < R; ++u) {
                if (i0 + u < cnt) {
#pragma unroll
                    for (int t = 0; t < MT; ++t)
                        if (t < tiles) C::add(acc[t], r[u][t]);
                }
            }
        }
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            const int chunk = t * kWave + lane;
            if (t < tiles && chunk < p.chunks) {
#pragma unroll
                for (int e = 0; e < VE; ++e) acc[t][e] *= inv;
                *reinterpret_cast<Raw*>(dst + (int64_t)chunk * VB) = C::pack(acc[t]);
            }
        }
        return;
    }

    const int sub = p.sub;
    const int sg = lane >> p.sub_shift;         // sub-group index within the wave
    const int sl = lane & (sub - 1);
    const int nsg = kWave >> p.sub_shift;
    const float inv_cnt = inv_count(cnt > 0 ? cnt : 1);
    for (int c0 = 0; c0 < p.chunks; c0 += sub) {
        const int chunk = c0 + sl;
        const bool live = chunk < p.chunks;
        float acc[VE];
#pragma unroll
        for (int e = 0; e < VE; ++e) acc[e] = 0.0f;
        if (live)
            sum_row_chunks<XT, VB, FSA_UNROLL>(p.x, p.row_bytes, (int64_t)chunk * VB, ids, sg, cnt,
                                               nsg, acc);
        for (int off = sub; off < kWave; off <<= 1) {
#pragma unroll
            for (int e = 0; e < VE; ++e) acc[e] += __shfl_xor(acc[e], off);
        }
        if (sg == 0 && live) {
#pragma unroll
            for (int e = 0; e < VE; ++e) acc[e] *= inv_cnt;
            *reinterpret_cast<typename C::Raw*>(dst + (int64_t)chunk * VB) = C::pack(acc);
        }
    }
}

// ---------------------------------------------------------------------------------------
// 1-hop: wave per seed
// ---------------------------------------------------------------------------------------
template <typename XT, int VB, bool REPLAY, int MT>
__global__ __launch_bounds__(256) void fwd1_kernel(const FwdParams p) {
    extern __shared__ int smem[];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int64_t b = (int64_t)blockIdx.x * (blockDim.x >> 6) + wave;
    if (b >= p.B) return;                       // wave-uniform; no block barrier below
    int* ids = smem + wave * kWave;

    int id = hop0_id<REPLAY>(p, b, lane);
    if (!REPLAY && p.out_ids1 && lane < p.k1) p.out_ids1[b * p.k1 + lane] = id;
    wave_mean_of_rows<XT, VB, MT>(p, id, ids, lane, p.out + b * p.row_bytes);
}

// Mean over the hop-1 slots that took part of the per-slot rows of a [B,k1,D] table (the last
// step of a chained, deeper-hop call): lane j names row b*k1+j when slot_cnt[b,j] > 0.
template <typename XT, int VB, int MT>
__global__ __launch_bounds__(256) void slot_mean_kernel(const FwdParams p) {
    extern __shared__ int smem[];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int64_t b = (int64_t)blockIdx.x * (blockDim.x >> 6) + wave;
    if (b >= p.B) return;                       // wave-uniform; no block barrier below
    const int id = (lane < p.k1 && p.slot_cnt[b * p.k1 + lane] > 0) ? (int)(b * p.k1 + lane) : -1;
    wave_mean_of_rows<XT, VB, MT>(p, id, smem + wave * kWave, lane, p.out + b * p.row_bytes);
}

// ---------------------------------------------------------------------------------------
// 2-hop: workgroup per root, waves own interleaved hop-1 slots
//
// A root costs a chain of dependent memory steps (seed -> indptr -> indices -> indptr ->
// indices -> feature rows); at the paper's batch sizes the launch is about as long as that
// chain, so the kernel is laid out to take each step ONCE per wave, for all of its slots:
//   step 1-3  hop 0 (every wave redraws it; lanes j < k1 end with U[j]);
//   step 4    lane q reads the indptr pair of owned slot q (all slots in one go); a scan of
//             the slot counts fixes where each slot's rows go in the flat list;
//   step 5    Floyd positions for (slot, step) pairs, 64/k2 slots per pass, with the
//             `indices` loads of up to kPassGroup passes in flight together; each ID is
//             stored as a 64-bit row byte offset, slot ends flagged in bit 63;
//   step 6    sub-groups walk contiguous, row-balanced blocks of the list, kUnroll row
//             loads in flight across slot boundaries instead of one slot at a time.
// ---------------------------------------------------------------------------------------
constexpr int kPassGroup = FSA_PASS_GROUP;

// MT > 0 selects the gather for rows wider than one tile of 64 lanes (2 .. MT tiles, MT at
// most kMultiTiles): all tiles of a row are loaded back to back, so the cache line that two
// neighbouring tiles share is fetched once -- walking the whole list once per tile fetched it
// twice, 20 % more HBM-side traffic than the rows themselves on 2408-byte rows.  MT = 0 is
// the single-tile gather (and the fallback for rows wider than kMultiTiles tiles).
constexpr int kMultiTiles = 8;

template <typename XT, int VB, bool REPLAY, int MT>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(FSA_FWD2_MIN_WAVES_PER_EU)))
void fwd2_kernel(const FwdParams p) {
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

    // LDS per wave: flat list of row byte offsets (int2, slot end flagged in bit 63)
    // [nq_max*k2], slot-end records [nq_max*k2], leaf IDs by slot [nq_max*k2] and per-slot
    // counts [nq_max] (both replay only), empty-slot list [nq_max]; then [nw] live-slot
    // counts and [nw][sub*VE] floats for the cross-wave reduction.
    const int nq_max = (k1 + nw - 1) / nw;
    const int per_wave = 4 * nq_max * k2 + 2 * nq_max;            // even: int2 stays 8-byte aligned
    int2* flat = reinterpret_cast<int2*>(smem + wave * per_wave);
    int* flat_meta = smem + wave * per_wave + 2 * nq_max * k2;
    int* leaf = flat_meta + nq_max * k2;
    int* cnt2 = leaf + nq_max * k2;
    int* empty_q = cnt2 + nq_max;
    int* live_slots = smem + nw * per_wave;
    float* red = reinterpret_cast<float*>(live_slots + nw);

    // hop 0, redundantly in every wave: lane j holds U[j]
    FSA_STAMP(0);
    const int u_mine = hop0_id<REPLAY>(p, b, lane);
    if (!REPLAY && wave == 0 && p.out_ids1 && lane < k1) p.out_ids1[b * k1 + lane] = u_mine;
    if (u_mine == 0x7ffffff0) FSA_STAMP(7);   // consume u_mine before the stamp
    FSA_STAMP(1);

    // owned slots: j = wave + q*nw, q < nq; lane q keeps slot q's node, row start, degree, count
    const int nq = wave < k1 ? (k1 - wave + nw - 1) / nw : 0;
    const int u_own = __shfl(u_mine, lane < nq ? wave + lane * nw : 0);
    const int spw = kWave / k2;                                   // slots handled per pass
    const int g = lane / k2;
    const int li = lane - g * k2;
    const uint64_t seg_mask = k2 == 64 ? ~0ull : ((1ull << k2) - 1ull);
    int64_t s_own = 0;
    uint32_t deg_own = 0;
    int c_own = 0;
    if constexpr (!REPLAY) {
        if (lane < nq && u_own >= 0) {
            int64_t d;
            row_extent(p, u_own, s_own, d);
            deg_own = (uint32_t)d;
            c_own = (int)(d < (int64_t)k2 ? d : (int64_t)k2);
        }
    } else {
        // saved leaf IDs of the owned slots: loads of a pass group overlap; holes are squeezed out
        for (int q0 = 0; q0 < nq; q0 += kPassGroup * spw) {       // wave-uniform trip count
            int idv[kPassGroup];
#pragma unroll
            for (int t = 0; t < kPassGroup; ++t) {
                idv[t] = -1;
                if (q0 + t * spw < nq) {
                    const int q = q0 + t * spw + g;
                    const bool valid = g < spw && q < nq;
                    const int u = __shfl(u_own, valid ? q : 0);
                    if (valid && u >= 0) idv[t] = p.ids2[(b * k1 + wave + q * nw) * k2 + li];
                }
            }
#pragma unroll
            for (int t = 0; t < kPassGroup; ++t) {
                if (q0 + t * spw < nq) {
                    const int q = q0 + t * spw + g;
                    const bool valid = g < spw && q < nq;
                    const uint64_t have = __ballot(valid && idv[t] >= 0) & (seg_mask << (valid ? g * k2 : 0));
                    if (valid && idv[t] >= 0) leaf[q * k2 + __popcll(have & lanemask_lt(lane))] = idv[t];
                    if (valid && li == 0) cnt2[q] = __popcll(have);
                }
            }
        }
        __builtin_amdgcn_wave_barrier();
        if (lane < nq) c_own = cnt2[lane];
    }
    if (deg_own == 0x7ffffff0u) FSA_STAMP(7);
    FSA_STAMP(2);

    // Where each slot's rows go in the flat list: exclusive prefix sum of the counts over
    // lanes q.  Sub-group sg later walks the rows of a contiguous block of slots [qa, qb).
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
    if (lane == 0) live_slots[wave] = nq - n_empty;

    const int sub = p.sub;
    const int sg = lane >> p.sub_shift;
    const int sl = lane & (sub - 1);
    const int nsg = kWave >> p.sub_shift;
    // Row-balanced split: sub-group s takes the slots whose first row lies in
    // [s*total/nsg, (s+1)*total/nsg); slots stay whole, so each sub-group is within one slot
    // of an even share.  first_q(s) = number of slots starting before row s*total/nsg.
    int qa = 0, qb = 0;
    for (int s = 0; s <= nsg; ++s) {                               // wave-uniform
        const int first_q = __popcll(__ballot(lane < nq && off_own * nsg < s * total));
        if (s == sg) qa = first_q;
        if (s == sg + 1) qb = first_q;
    }
    if (sg == nsg - 1) qb = nq;
    const int start_a = __shfl(off_own, qa < nq ? qa : 0);
    const int start_b = __shfl(off_own, qb < nq ? qb : 0);
    const int my_start = qa < nq ? start_a : total;
    const int my_len = (qb < nq ? start_b : total) - my_start;

    if constexpr (!REPLAY) {
        // hop 1: (slot, step) pairs in passes of spw slots.  The `indices` loads of a pass group
        // are all issued before the first one is used; each sampled ID goes straight to its
        // place in the flat list as a row byte offset.
        for (int q0 = 0; q0 < nq; q0 += kPassGroup * spw) {       // wave-uniform trip count
            int idv[kPassGroup], dstv[kPassGroup];
#pragma unroll
            for (int t = 0; t < kPassGroup; ++t) {
                idv[t] = -1;
                dstv[t] = -1;
                if (q0 + t * spw < nq) {                           // wave-uniform
                    const int q = q0 + t * spw + g;
                    const bool valid = g < spw && q < nq;
                    const int src = valid ? q : 0;
                    const int u = __shfl(u_own, src);
                    const bool active = valid && u >= 0;
                    const uint32_t s_lo = __shfl((uint32_t)s_own, src);
                    const uint32_t s_hi = __shfl((uint32_t)((uint64_t)s_own >> 32), src);
                    const int64_t s = (int64_t)(((uint64_t)s_hi << 32) | s_lo);
                    const int64_t deg = (int64_t)__shfl(deg_own, src);
                    const int off = __shfl(off_own, src);
                    const int64_t pos = floyd_position(p.seed, (uint32_t)u, p.hop_base + 1u, k2, li, valid ? g * k2 : 0,
                                                       deg, active, lane);
                    if (pos >= 0) {
                        idv[t] = p.indices[s + pos];
                        const int c = (int)(deg < (int64_t)k2 ? deg : (int64_t)k2);
                        dstv[t] = (off + li) | (li == c - 1 ? 0x40000000 : 0);
                    }
                }
            }
#pragma unroll
            for (int t = 0; t < kPassGroup; ++t) {
                if (q0 + t * spw < nq) {
                    const int q = q0 + t * spw + g;
                    const int j = wave + q * nw;
                    if (g < spw && q < nq && p.out_ids2) p.out_ids2[(b * k1 + j) * k2 + li] = idv[t];
                    if (dstv[t] >= 0) {
                        const int at = dstv[t] & 0x3fffffff;
                        const uint32_t last = (uint32_t)dstv[t] >> 30;
                        const uint64_t row_off = (uint64_t)(uint32_t)idv[t] * (uint64_t)p.row_bytes;
                        flat[at] = make_int2((int)(uint32_t)row_off, (int)((uint32_t)(row_off >> 32) | (last << 31)));
                        if (last) flat_meta[at] = j | ((li + 1) << 8);
                    }
                }
            }
        }
    } else {
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
                if (last) flat_meta[at] = (wave + q * nw) | (c << 8);
            }
        }
    }
    __builtin_amdgcn_wave_barrier();
    FSA_STAMP(3);

    // gather
    FSA_STAMP(4);
    if constexpr (MT > 0) {
        // rows wider than one tile: sub == 64, one sub-group, the wave walks its whole list
        constexpr int R = FSA_MULTI_LOADS / MT;                    // rows in flight: 2 x 4 tiles or 1 x 8
        const int tiles = (p.chunks + kWave - 1) >> 6;             // 2 .. MT, checked on the host
        float acc[MT][VE], root[MT][VE];
#pragma unroll
        for (int t = 0; t < MT; ++t) {
#pragma unroll
            for (int e = 0; e < VE; ++e) { acc[t][e] = 0.0f; root[t][e] = 0.0f; }
        }
        if (p.out_h1) {                                            // empty slots get zero rows
            for (int i = 0; i < n_empty; ++i) {
                char* dst = p.out_h1 + (b * k1 + wave + empty_q[i] * nw) * p.row_bytes;
                for (int chunk = lane; chunk < p.chunks; chunk += kWave)
                    *reinterpret_cast<Raw*>(dst + (int64_t)chunk * VB) = C::pack(acc[0]);
            }
        }
        for (int i0 = 0; i0 < total; i0 += R) {
            int2 ent[R];
            Raw r[R][MT];
#pragma unroll
            for (int u = 0; u < R; ++u) {
                const int i = i0 + u < total ? i0 + u : total - 1;
                ent[u] = flat[i];
                const uint64_t row_off = ((uint64_t)((uint32_t)ent[u].y & 0x7fffffffu) << 32) | (uint32_t)ent[u].x;
#pragma unroll
                for (int t = 0; t < MT; ++t) {
                    if (t < tiles) {                               // wave-uniform
                        const int chunk = t * kWave + lane;        // lanes past the row width re-read chunk 0
                        r[u][t] = *reinterpret_cast<const Raw*>(p.x + row_off + (chunk < p.chunks ? (int64_t)chunk * VB : 0));
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < R; ++u) {
                if (i0 + u < total) {
#pragma unroll
                    for (int t = 0; t < MT; ++t)
                        if (t < tiles) C::add(acc[t], r[u][t]);
                    if (ent[u].y < 0) {                            // last row of its slot
                        const int meta = flat_meta[i0 + u];
                        const float inv = inv_count(meta >> 8);
                        char* dst = p.out_h1 ? p.out_h1 + (b * k1 + (meta & 0xff)) * p.row_bytes : nullptr;
#pragma unroll
                        for (int t = 0; t < MT; ++t) {
                            if (t < tiles) {
                                const int chunk = t * kWave + lane;
#pragma unroll
                                for (int e = 0; e < VE; ++e) { acc[t][e] *= inv; root[t][e] += acc[t][e]; }
                                if (dst && chunk < p.chunks)
                                    *reinterpret_cast<Raw*>(dst + (int64_t)chunk * VB) = C::pack(acc[t]);
#pragma unroll
                                for (int e = 0; e < VE; ++e) acc[t][e] = 0.0f;
                            }
                        }
                    }
                }
            }
        }
        FSA_STAMP(5);
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            if (t < tiles) {                                       // workgroup-uniform
                const int chunk = t * kWave + lane;
                const bool live = chunk < p.chunks;
                if (nw == 1) {
                    const int c1 = live_slots[0];
                    if (t == 0 && lane == 0 && p.out_live) p.out_live[b] = c1;
                    const float inv1 = inv_count(c1 > 0 ? c1 : 1);
#pragma unroll
                    for (int e = 0; e < VE; ++e) root[t][e] *= inv1;
                    if (live) *reinterpret_cast<Raw*>(p.out + b * p.row_bytes + (int64_t)chunk * VB) = C::pack(root[t]);
                } else {
#pragma unroll
                    for (int e = 0; e < VE; ++e) red[(wave * kWave + lane) * VE + e] = root[t][e];
                    __syncthreads();
                    if (wave == 0) {
                        int c1 = 0;
                        for (int w = 0; w < nw; ++w) c1 += live_slots[w];
                        if (t == 0 && lane == 0 && p.out_live) p.out_live[b] = c1;
                        float tot[VE];
#pragma unroll
                        for (int e = 0; e < VE; ++e) tot[e] = 0.0f;
                        for (int w = 0; w < nw; ++w) {
#pragma unroll
                            for (int e = 0; e < VE; ++e) tot[e] += red[(w * kWave + lane) * VE + e];
                        }
                        const float inv1 = inv_count(c1 > 0 ? c1 : 1);
#pragma unroll
                        for (int e = 0; e < VE; ++e) tot[e] *= inv1;
                        if (live) *reinterpret_cast<Raw*>(p.out + b * p.row_bytes + (int64_t)chunk * VB) = C::pack(tot);
                    }
                    __syncthreads();                               // red is reused by the next tile
                }
            }
        }
    } else {
        for (int c0 = 0; c0 < p.chunks; c0 += sub) {
            const int chunk = c0 + sl;
            const bool live = chunk < p.chunks;
            const int64_t chunk_off = (int64_t)chunk * VB;
            float acc[VE], root[VE];
    #pragma unroll
            for (int e = 0; e < VE; ++e) { acc[e] = 0.0f; root[e] = 0.0f; }
            if (p.out_h1 && live) {                                    // empty slots get zero rows
                for (int i = sg; i < n_empty; i += nsg)
                    *reinterpret_cast<Raw*>(p.out_h1 + (b * k1 + wave + empty_q[i] * nw) * p.row_bytes + chunk_off) = C::pack(acc);
            }
            // Row loads carry no branch of their own: past the end of the list they re-read its
            // last row (a cache hit) and lanes beyond the row width re-read chunk 0; the results
            // are simply not accumulated.  This keeps kUnroll loads in flight per lane.
            const int64_t load_off = live ? chunk_off : 0;
            for (int i0 = 0; i0 < my_len; i0 += U) {
                int2 ent[U];
                Raw r[U];
    #pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int i = i0 + u < my_len ? i0 + u : my_len - 1;
                    ent[u] = flat[my_start + i];
                    const uint64_t row_off = ((uint64_t)((uint32_t)ent[u].y & 0x7fffffffu) << 32) | (uint32_t)ent[u].x;
                    r[u] = *reinterpret_cast<const Raw*>(p.x + row_off + load_off);
                }
    #pragma unroll
                for (int u = 0; u < U; ++u) {
                    if (i0 + u < my_len) {
                        C::add(acc, r[u]);
                        if (ent[u].y < 0) {                            // last row of its slot
                            const int meta = flat_meta[my_start + i0 + u];
                            const float inv = inv_count(meta >> 8);
    #pragma unroll
                            for (int e = 0; e < VE; ++e) { acc[e] *= inv; root[e] += acc[e]; }
                            if (live && p.out_h1)
                                *reinterpret_cast<Raw*>(p.out_h1 + (b * k1 + (meta & 0xff)) * p.row_bytes + chunk_off) = C::pack(acc);
    #pragma unroll
                            for (int e = 0; e < VE; ++e) acc[e] = 0.0f;
                        }
                    }
                }
            }
            for (int off = sub; off < kWave; off <<= 1) {
    #pragma unroll
                for (int e = 0; e < VE; ++e) root[e] += __shfl_xor(root[e], off);
            }
            FSA_STAMP(5);
            if (nw == 1) {
                if (c0 == 0 && lane == 0 && p.out_live) p.out_live[b] = live_slots[0];
                if (sg == 0 && live) {
                    const int c1 = live_slots[0];
                    const float inv1 = inv_count(c1 > 0 ? c1 : 1);
    #pragma unroll
                    for (int e = 0; e < VE; ++e) root[e] *= inv1;
                    *reinterpret_cast<Raw*>(p.out + b * p.row_bytes + chunk_off) = C::pack(root);
                }
                continue;
            }
            if (sg == 0) {
    #pragma unroll
                for (int e = 0; e < VE; ++e) red[(wave * sub + sl) * VE + e] = root[e];
            }
            __syncthreads();
            if (wave == 0 && sg == 0 && live) {
                int c1 = 0;
                for (int w = 0; w < nw; ++w) c1 += live_slots[w];
                if (c0 == 0 && sl == 0 && p.out_live) p.out_live[b] = c1;
                float tot[VE];
    #pragma unroll
                for (int e = 0; e < VE; ++e) tot[e] = 0.0f;
                for (int w = 0; w < nw; ++w) {
    #pragma unroll
                    for (int e = 0; e < VE; ++e) tot[e] += red[(w * sub + sl) * VE + e];
                }
                const float inv1 = inv_count(c1 > 0 ? c1 : 1);
    #pragma unroll
                for (int e = 0; e < VE; ++e) tot[e] *= inv1;
                *reinterpret_cast<Raw*>(p.out + b * p.row_bytes + chunk_off) = C::pack(tot);
            }
            if (c0 + sub < p.chunks) __syncthreads();       // red is reused by the next tile
        }
    }
}

// ---------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------
static int env_int(const char* name, int fallback) {
    const char* v = std::getenv(name);
    return v ? std::atoi(v) : fallback;
}

// Waves per root for the 2-hop kernel.  One wave per root keeps the most roots resident and
// needs no block barrier; small batches are spread over more waves (which then own fewer
// hop-1 slots each) until the chip holds about 16 waves per CU.  Measured on the product,
// social and citation shapes at B = 1024 .. 65536.
int fwd2_waves(int64_t B, int k1, const RowGeom&) {
    static const int forced = env_int("FSA_FWD2_WAVES", 0);
    if (forced >= 1 && forced <= 8) return forced;
    int nw = 1;
    while (nw < 8 && nw * 2 <= k1 && B * nw < 4096) nw *= 2;
    return nw;
}

template <typename XT, int VB>
static hipError_t launch_typed(const FwdArgs& a, const FwdParams& p, hipStream_t stream) {
    constexpr int VE = Chunk<XT, VB>::VE;
    const bool replay = a.indptr == nullptr;
    // rows of 2 .. kMultiTiles tiles of 64 lanes take the row-major multi-tile gather
    const int tiles = a.geom.tiles;
    const int mt = (tiles <= 1 || tiles > kMultiTiles) ? 0 : (tiles <= 4 ? 4 : 8);
    if (a.slot_cnt) {                           // mean over the per-slot rows of a [B,k1,D] table
        const int wpb = 4;
        const dim3 grid((unsigned)((a.B + wpb - 1) / wpb)), block(wpb * kWave);
        const size_t lds = sizeof(int) * kWave * wpb;
        if (mt == 0)      hipLaunchKernelGGL((slot_mean_kernel<XT, VB, 0>), grid, block, lds, stream, p);
        else if (mt == 4) hipLaunchKernelGGL((slot_mean_kernel<XT, VB, 4>), grid, block, lds, stream, p);
        else              hipLaunchKernelGGL((slot_mean_kernel<XT, VB, 8>), grid, block, lds, stream, p);
        return hipGetLastError();
    }
    if (a.hops == 1) {
        static const int wpb = [] { int v = env_int("FSA_FWD1_WAVES", 4); return v >= 1 && v <= 4 ? v : 4; }();
        const dim3 grid((unsigned)((a.B + wpb - 1) / wpb)), block(wpb * kWave);
        const size_t lds = sizeof(int) * kWave * wpb;
#define FSA_LAUNCH_FWD1(MT_)                                                                                   \
        do {                                                                                                   \
            if (replay) hipLaunchKernelGGL((fwd1_kernel<XT, VB, true, MT_>), grid, block, lds, stream, p);     \
            else        hipLaunchKernelGGL((fwd1_kernel<XT, VB, false, MT_>), grid, block, lds, stream, p);    \
        } while (0)
        if (mt == 0) FSA_LAUNCH_FWD1(0);
        else if (mt == 4) FSA_LAUNCH_FWD1(4);
        else FSA_LAUNCH_FWD1(8);
#undef FSA_LAUNCH_FWD1
    } else {
        const int nw = fwd2_waves(a.B, a.k1, a.geom);
        const int nq_max = (a.k1 + nw - 1) / nw;
        const size_t lds = sizeof(int) * ((size_t)nw * (4 * nq_max * a.k2 + 2 * nq_max) + nw)
                         + sizeof(float) * (size_t)nw * a.geom.sub * VE;
        const dim3 grid((unsigned)a.B), block(nw * kWave);
#define FSA_LAUNCH_FWD2(MT_)                                                                                   \
        do {                                                                                                   \
            if (replay) hipLaunchKernelGGL((fwd2_kernel<XT, VB, true, MT_>), grid, block, lds, stream, p);     \
            else        hipLaunchKernelGGL((fwd2_kernel<XT, VB, false, MT_>), grid, block, lds, stream, p);    \
        } while (0)
        if (mt == 0) FSA_LAUNCH_FWD2(0);
        else if (mt == 4) FSA_LAUNCH_FWD2(4);
        else FSA_LAUNCH_FWD2(8);
#undef FSA_LAUNCH_FWD2
    }
    return hipGetLastError();
}

hipError_t launch_forward(const FwdArgs& a, hipStream_t stream) {
    FwdParams p;
    p.indptr = a.indptr; p.indices = a.indices; p.x = static_cast<const char*>(a.x);
    p.seeds = a.seeds; p.ids1 = a.ids1; p.ids2 = a.ids2;
    p.out = static_cast<char*>(a.out); p.out_h1 = static_cast<char*>(a.out_h1);
    p.out_ids1 = a.out_ids1; p.out_ids2 = a.out_ids2;
    p.B = a.B; p.row_bytes = a.D * (a.x_kind == 0 ? 4 : 2); p.seed = a.seed;
    p.k1 = a.k1; p.k2 = a.k2; p.chunks = a.geom.chunks; p.sub = a.geom.sub;
    p.sub_shift = __builtin_ctz((unsigned)a.geom.sub); p.indptr_is64 = a.indptr_is64;
    p.hop_base = a.hop_base; p.out_live = a.out_live; p.slot_cnt = a.slot_cnt;
#ifdef FSA_TRACE
    { const char* t = std::getenv("FSA_TRACE_PTR"); p.trace = t ? reinterpret_cast<long long*>(std::strtoull(t, nullptr, 16)) : nullptr; }
#endif
    const int vb = a.geom.vec_bytes;
    if (a.x_kind == 1) {
        switch (vb) {
            case 16: return launch_typed<bf16_t, 16>(a, p, stream);
            case 8:  return launch_typed<bf16_t, 8>(a, p, stream);
            case 4:  return launch_typed<bf16_t, 4>(a, p, stream);
            default: return launch_typed<bf16_t, 2>(a, p, stream);
        }
    }
    if (a.x_kind == 2) {
        switch (vb) {
            case 16: return launch_typed<f16_t, 16>(a, p, stream);
            case 8:  return launch_typed<f16_t, 8>(a, p, stream);
            case 4:  return launch_typed<f16_t, 4>(a, p, stream);
            default: return launch_typed<f16_t, 2>(a, p, stream);
        }
    }
    switch (vb) {
        case 16: return launch_typed<f32_t, 16>(a, p, stream);
        case 8:  return launch_typed<f32_t, 8>(a, p, stream);
        default: return launch_typed<f32_t, 4>(a, p, stream);
    }
}

}  // namespace fsa
