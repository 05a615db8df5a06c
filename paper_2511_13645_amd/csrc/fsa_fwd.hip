// Forward kernels: fused sample + mean (Sec. 3.2 of arXiv 2511.13645), its weighted-mean
// extension (Sec. 3.2, "Extension Feasibility") and the replay forward from saved IDs
// (Sec. 3.3, Prop. 1), for gfx950.
//
// Mapping (the paper's Sec. 4 uses warp-per-seed / block-per-root on 32-wide warps; this is
// the 64-wide-wavefront re-derivation):
//   1-hop: one wavefront per seed.  Lane i runs Floyd step i; the sampled IDs are staged in
//          a wave-private LDS strip; the wave is cut into 64/sub sub-groups of `sub` lanes,
//          each sub-group covers one feature row with 16/8/4-byte loads and the sub-groups
//          take different neighbor rows, so several rows are in flight per instruction.
//   2-hop: one wave per root (for small batches several waves, each owning a subset of the
//          hop-1 slots).  The wave draws the hop-1 IDs (k1 lanes), reads their row extents
//          (one lane per slot), samples their rows in segments of k2 lanes (64/k2 rows per
//          pass) and writes every sampled leaf ID straight into a flat, row-balanced list in
//          LDS; sub-groups then stream the listed rows with a fixed number of loads in
//          flight, closing a slot (mean -> out_h1, add to the root sum) whenever a flagged
//          entry goes by.  The root mean is reduced by shuffles (and through LDS across
//          waves) and written once.  No [B,k,D] gathered tensor and no block structure ever
//          exists.
// The replay kernels are the same code with the sampler swapped for loads of the saved IDs,
// which is what makes replay bitwise equal to the sampling forward.  The weighted mean is
// the same code again (template flag): every sampled edge slot also brings its weight, rows
// are multiply-added and a slot's divisor is its weight sum; sampling itself stays uniform.
#include "fsa_device.hip.h"
#include "fsa_internal.h"

#ifndef FSA_UNROLL
#define FSA_UNROLL 4
#endif
#ifndef FSA_PASS_GROUP
#define FSA_PASS_GROUP 4
#endif
#ifndef FSA_MULTI_LOADS
#define FSA_MULTI_LOADS 8
#endif
#ifndef FSA_ROOTS_PER_WG
#define FSA_ROOTS_PER_WG 1
#endif

namespace fsa {

struct FwdParams {
    const void* indptr; const int32_t* indices; const float* edge_w; const char* x;
    const int32_t* seeds; const int32_t* ids1; const int32_t* ids2; const float* w1; const float* w2;
    char* out; char* out_h1; int32_t* out_ids1; int32_t* out_ids2; float* out_w1; float* out_w2;
    int64_t B; int64_t row_bytes; uint64_t seed;
    int k1, k2, chunks, sub, sub_shift, indptr_is64;
    uint32_t hop_base;                      // hop counter of the seeds' own rows (0 unless chained)
    int32_t* out_live;                      // 2-hop, nullable: [B] hop-1 slots that took part
    const int32_t* slot_cnt;                // slot-mean kernel only: [B,k1] counts, > 0 = takes part
    int waves_per_root;                     // 2-hop: waves that share one root (1: every wave has a root of its own)
    uint32_t hop1;                          // 2-hop kernel: hop counter of the rows its (slot, step) lanes sample
    int64_t packed_seeds;                   // > 0: the 2-hop kernel runs a 1-hop call over this many seeds, k1 of
                                            // them per wave as its "slots" (see launch_typed); 0 otherwise
#ifdef FSA_TRACE
    long long* trace;                       // debug builds: [B][4] start, gather start, end (10 ns units), leaf rows
#endif
};

#ifdef FSA_TRACE
#define FSA_STAMP(var) const long long var = wall_clock64()
#else
#define FSA_STAMP(var) do { } while (0)
#endif

// A value every lane of the wave holds, moved to scalar registers.
__device__ __forceinline__ int64_t wave_uniform(int64_t v) {
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)(uint64_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)((uint64_t)v >> 32));
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

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
// hop-1 ID of root slot b, -1 in unused slots, and (weighted mean) the weight of that edge.
// Replay keeps the saved layout (holes stay).
template <bool REPLAY, bool WEIGHTED>
__device__ __forceinline__ int hop0_id(const FwdParams& p, int64_t b, int lane, int* draws, float& w) {
    w = 0.0f;
    if constexpr (REPLAY) {
        // chained calls pass the level above as `seeds`: a negative entry switches the root off
        if (p.seeds && p.seeds[b] < 0) return -1;
        if (lane >= p.k1) return -1;
        if constexpr (WEIGHTED) w = p.w1[b * p.k1 + lane];
        return p.ids1[b * p.k1 + lane];
    } else {
        // a negative seed (an unused slot of the level above, when calls are chained) is an
        // empty row: nothing is read for it
        // b is the same in every lane of the wave: saying so lets the seed and its indptr pair come
        // through the scalar data path, ahead of the vector memory queue
        const int64_t bu = wave_uniform(b);
        const int64_t r = wave_uniform((int64_t)p.seeds[bu]);
        const bool active = lane < p.k1;
        int64_t s, deg;
        row_extent(p, r >= 0 ? r : 0, s, deg);
        if (r < 0) deg = 0;
        uint32_t word = 0u;
        if (__any(active && deg > (int64_t)p.k1)) word = floyd_word(p.seed, (uint32_t)r, p.hop_base, lane);   // wave-uniform
        const int64_t pos = floyd_resolve(floyd_bound(word, p.k1, lane, deg), p.k1, lane, 0, deg, active, lane, draws);
        if (pos < 0) return -1;
        if constexpr (WEIGHTED) w = p.edge_w[s + pos];
        return p.indices[s + pos];
    }
}

// The mean's divisor: 1/count, or 1/(weight sum) with a zero sum meaning "nothing to average".
__device__ __forceinline__ float inv_weight(float wsum) { return wsum > 0.0f ? __builtin_amdgcn_rcpf(wsum) : 0.0f; }

// One wave: mean of the rows of p.x named by the lanes' non-negative `id`s, in lane order,
// written to `dst`; WEIGHTED: the mean weighted by the lanes' `w`, zero when the weights sum
// to zero.  `ids` (64 ints) and `wts` (64 floats) are the wave's LDS strips.
template <typename XT, int VB, int MT, bool WEIGHTED>
__device__ __forceinline__ void wave_mean_of_rows(const FwdParams& p, int id, float w, int* ids, float* wts, int lane,
                                                  char* dst) {
    using C = Chunk<XT, VB>;
    constexpr int VE = C::VE;
    // stage the valid IDs, in slot order, in this wave's LDS strip
    const uint64_t valid = __ballot(id >= 0);
    const int cnt = __popcll(valid);
    if (id >= 0) {
        const int slot = __popcll(valid & lanemask_lt(lane));
        ids[slot] = id;
        if constexpr (WEIGHTED) wts[slot] = w;
    }
    __builtin_amdgcn_wave_barrier();

    if constexpr (MT > 0) {
        // rows of 2 .. MT tiles of 64 lanes: all tiles of a row are loaded back to back, so a
        // cache line shared by neighbouring tiles is fetched once
        using Raw = typename C::Raw;
        constexpr int R = FSA_MULTI_LOADS / MT;                    // rows in flight
        const int tiles = (p.chunks + kWave - 1) >> 6;
        float acc[MT][VE];
#pragma unroll
        for (int t = 0; t < MT; ++t) {
#pragma unroll
            for (int e = 0; e < VE; ++e) acc[t][e] = 0.0f;
        }
        float wsum = 0.0f;
        for (int i0 = 0; i0 < cnt; i0 += R) {
            Raw r[R][MT];
            float wr[R];
#pragma unroll
            for (int u = 0; u < R; ++u) {
                const int i = i0 + u < cnt ? i0 + u : cnt - 1;
                const int64_t row_off = (int64_t)ids[i] * p.row_bytes;
                if constexpr (WEIGHTED) wr[u] = wts[i];
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
                    for (int t = 0; t < MT; ++t) {
                        if (t < tiles) {
                            if constexpr (WEIGHTED) C::fma(acc[t], r[u][t], wr[u]);
                            else C::add(acc[t], r[u][t]);
                        }
                    }
                    if constexpr (WEIGHTED) wsum += wr[u];
                }
            }
        }
        const float inv = WEIGHTED ? inv_weight(wsum) : inv_count(cnt > 0 ? cnt : 1);
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
    for (int c0 = 0; c0 < p.chunks; c0 += sub) {
        const int chunk = c0 + sl;
        const bool live = chunk < p.chunks;
        float acc[VE];
#pragma unroll
        for (int e = 0; e < VE; ++e) acc[e] = 0.0f;
        float wsum = 0.0f;
        if (live)
            sum_row_chunks<XT, VB, FSA_UNROLL, WEIGHTED>(p.x, p.row_bytes, (int64_t)chunk * VB, ids, wts, sg, cnt, nsg,
                                                         acc, wsum);
        for (int off = sub; off < kWave; off <<= 1) {
#pragma unroll
            for (int e = 0; e < VE; ++e) acc[e] += __shfl_xor(acc[e], off);
            if constexpr (WEIGHTED) wsum += __shfl_xor(wsum, off);
        }
        if (sg == 0 && live) {
            const float inv = WEIGHTED ? inv_weight(wsum) : inv_count(cnt > 0 ? cnt : 1);
#pragma unroll
            for (int e = 0; e < VE; ++e) acc[e] *= inv;
            *reinterpret_cast<typename C::Raw*>(dst + (int64_t)chunk * VB) = C::pack(acc);
        }
    }
}

// ---------------------------------------------------------------------------------------
// 1-hop: wave per seed
// ---------------------------------------------------------------------------------------
template <typename XT, int VB, bool REPLAY, int MT, bool WEIGHTED>
__global__ __launch_bounds__(256) void fwd1_kernel(const FwdParams p) {
    extern __shared__ __align__(16) int smem[];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int64_t b = (int64_t)blockIdx.x * (blockDim.x >> 6) + wave;
    if (b >= p.B) return;                       // wave-uniform; no block barrier below
    int* ids = smem + wave * kFwd1StripInts;    // the duplicate test's draws use these ints first
    float* wts = reinterpret_cast<float*>(ids + 72);

    float w;
    const int id = hop0_id<REPLAY, WEIGHTED>(p, b, lane, ids, w);
    if (!REPLAY && lane < p.k1) {
        if (p.out_ids1) p.out_ids1[b * p.k1 + lane] = id;
        if constexpr (WEIGHTED) { if (p.out_w1) p.out_w1[b * p.k1 + lane] = id >= 0 ? w : 0.0f; }
    }
    wave_mean_of_rows<XT, VB, MT, WEIGHTED>(p, id, w, ids, wts, lane, p.out + b * p.row_bytes);
}

// Mean over the hop-1 slots that took part of the per-slot rows of a [B,k1,D] table (the last
// step of a chained, deeper-hop call): lane j names row b*k1+j when slot_cnt[b,j] > 0.
template <typename XT, int VB, int MT>
__global__ __launch_bounds__(256) void slot_mean_kernel(const FwdParams p) {
    extern __shared__ __align__(16) int smem[];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int64_t b = (int64_t)blockIdx.x * (blockDim.x >> 6) + wave;
    if (b >= p.B) return;                       // wave-uniform; no block barrier below
    const int id = (lane < p.k1 && p.slot_cnt[b * p.k1 + lane] > 0) ? (int)(b * p.k1 + lane) : -1;
    wave_mean_of_rows<XT, VB, MT, false>(p, id, 0.0f, smem + wave * kWave, nullptr, lane, p.out + b * p.row_bytes);
}

// ---------------------------------------------------------------------------------------
// 2-hop: a wave (or the waves of a workgroup) per root, waves own interleaved hop-1 slots
//
// A root costs a chain of dependent memory steps (seed -> indptr -> indices -> indptr ->
// indices -> feature rows), each about a microsecond, so the kernel takes each step ONCE per
// wave, for all of its slots:
//   step 1-3  hop 0 (every wave redraws it; lanes j < k1 end with U[j]);
//   step 4    lane q reads the indptr pair of owned slot q (all slots in one go); a scan of
//             the slot counts fixes where each slot's rows go in the flat list and each
//             slot's record (row start, degree, place) goes to LDS, where the lanes, from
//             here on one per (slot, Floyd step) pair, read it back;
//   step 5    Floyd positions for (slot, step) pairs, 64/k2 slots per pass, with the
//             `indices` loads of up to kPassGroup passes in flight together; each ID is
//             stored as a 64-bit row byte offset, slot ends flagged in bit 63;
//   step 6    sub-groups walk contiguous, row-balanced blocks of the list with kUnroll row
//             loads in flight at any time, across slot boundaries.
// ---------------------------------------------------------------------------------------
constexpr int kPassGroup = FSA_PASS_GROUP;
constexpr int kRootsPerWorkgroup = FSA_ROOTS_PER_WG;             // with one wave per root
#ifndef FSA_FWD1_PACKED_PASSES
#define FSA_FWD1_PACKED_PASSES 4
#endif
constexpr int kFwd1PackedPasses = FSA_FWD1_PACKED_PASSES;        // sampling passes of a packed 1-hop wave

// MT > 0 selects the gather for rows wider than one tile of 64 lanes (2 .. MT tiles, MT at
// most kMultiTiles): all tiles of a row are loaded back to back, so the cache line that two
// neighbouring tiles share is fetched once -- walking the whole list once per tile fetched it
// twice, 20 % more HBM-side traffic than the rows themselves on 2408-byte rows.  MT = 0 is
// the single-tile gather (and the fallback for rows wider than kMultiTiles tiles).
constexpr int kMultiTiles = 8;

__device__ __forceinline__ uint64_t row_offset_of(const int2& ent) {
    return ((uint64_t)((uint32_t)ent.y & 0x7fffffffu) << 32) | (uint32_t)ent.x;
}

template <typename XT, int VB, bool REPLAY, int MT, bool WEIGHTED>
__global__ __launch_bounds__(512) void fwd2_kernel(const FwdParams p) {
    using C = Chunk<XT, VB>;
    using Raw = typename C::Raw;
    constexpr int VE = C::VE;
    constexpr int U = FSA_UNROLL;
    extern __shared__ __align__(16) int smem[];
    const int lane = threadIdx.x & 63;
    const int strip = threadIdx.x >> 6;                           // wave of the workgroup: picks the LDS strip
    const int n_strips = blockDim.x >> 6;
    // Either the waves of a workgroup share one root (nw > 1) or every wave has a root of its
    // own (nw == 1; several roots per workgroup only shorten the dispatch of a large grid).
    const int nw = p.waves_per_root;
    const int wave = nw == 1 ? 0 : strip;
    const int64_t b = nw == 1 ? (int64_t)blockIdx.x * n_strips + strip : (int64_t)blockIdx.x;
    if (b >= p.B) return;                                          // nw == 1 only; no block barrier on that path
    const int k1 = p.k1, k2 = p.k2;
    // A packed 1-hop call: this wave's "hop-1 slots" are the seeds b*k1 .. b*k1+k1-1 themselves and
    // its per-slot outputs are the call's outputs; the last wave may have fewer seeds than k1, and
    // nothing may be read or written for the missing ones.
    const int64_t seeds_left = p.packed_seeds > 0 ? p.packed_seeds - b * k1 : (int64_t)k1;
    const int k1_live = seeds_left < (int64_t)k1 ? (int)seeds_left : k1;
    FSA_STAMP(t_start);

    const int nq_max = (k1 + nw - 1) / nw;
    const Fwd2Layout L = fwd2_layout(nq_max, k2, WEIGHTED);
    int* base = smem + strip * L.per_wave;
    int2* flat = reinterpret_cast<int2*>(base + L.flat);
    int* flat_meta = base + L.meta;
    float* flat_w = reinterpret_cast<float*>(base + L.flat_w);
    int* leaf = base + L.leaf;
    float* leaf_w = reinterpret_cast<float*>(base + L.leaf_w);
    int* cnt2 = base + L.cnt2;
    int* empty_q = base + L.empty_q;
    int4* rec = reinterpret_cast<int4*>(base + L.rec);
    float* slot_a = reinterpret_cast<float*>(base + L.slot_a);
    int* draws = base + L.draws;
    int* live_slots = smem + n_strips * L.per_wave;               // per strip: slots that took part (weighted: their weight)
    float* red = reinterpret_cast<float*>(live_slots + round_up4(n_strips));

    // hop 0, redundantly in every wave: lane j holds U[j]
    float a_mine = 0.0f;
    int u_mine;
    if (p.packed_seeds > 0) {                                      // kernel-uniform
        u_mine = -1;
        if (lane < k1_live) {
            if constexpr (REPLAY) u_mine = 0;                      // any node: a replayed slot only needs to exist
            else u_mine = p.seeds[b * k1 + lane];                  // (a negative seed is an empty row)
        }
    } else {
        u_mine = hop0_id<REPLAY, WEIGHTED>(p, b, lane, draws, a_mine);
    }
    if (!REPLAY && wave == 0 && lane < k1) {
        if (p.out_ids1) p.out_ids1[b * k1 + lane] = u_mine;
        if constexpr (WEIGHTED) { if (p.out_w1) p.out_w1[b * k1 + lane] = u_mine >= 0 ? a_mine : 0.0f; }
    }

    // owned slots: j = wave + q*nw, q < nq; lane q keeps slot q's node, row start, degree, count
    const int nq = owned_slots(k1_live, nw, wave);
    int u_own = u_mine;
    float a_own = a_mine;
    if (nw != 1) {
        const int src = lane < nq ? wave + lane * nw : 0;
        u_own = __shfl(u_mine, src);
        if constexpr (WEIGHTED) a_own = __shfl(a_mine, src);
    }
    if (lane >= nq) u_own = -1;
    if constexpr (WEIGHTED) { if (lane < nq) slot_a[lane] = a_own; }
    const int spw = kWave / k2;                                   // slots handled per pass
    const int g = lane / k2;
    const int li = lane - g * k2;
    const int seg_base = g < spw ? g * k2 : 0;
    const uint64_t seg_mask = k2 == 64 ? ~0ull : ((1ull << k2) - 1ull);
    int64_t s_own = 0;
    uint32_t deg_own = 0;
    int c_own = 0;
    if constexpr (!REPLAY) {
        if (lane < nq) cnt2[lane] = u_own;                        // read back below in the (slot, step) layout
        int64_t d = 0;
        if (u_own >= 0) row_extent(p, u_own, s_own, d);
        deg_own = (uint32_t)d;
        c_own = (int)(d < (int64_t)k2 ? d : (int64_t)k2);
    } else {
        // saved leaf IDs of the owned slots: loads of a pass group overlap; holes are squeezed out
        for (int q0 = 0; q0 < nq; q0 += kPassGroup * spw) {       // wave-uniform trip count
            int idv[kPassGroup];
            float wv[kPassGroup];
#pragma unroll
            for (int t = 0; t < kPassGroup; ++t) {
                idv[t] = -1;
                wv[t] = 0.0f;
                if (q0 + t * spw < nq) {
                    const int q = q0 + t * spw + g;
                    const bool valid = g < spw && q < nq;
                    const int u = __shfl(u_own, valid ? q : 0);
                    if (valid && u >= 0) {
                        const int64_t at = (b * k1 + wave + q * nw) * k2 + li;
                        idv[t] = p.ids2[at];
                        if constexpr (WEIGHTED) wv[t] = p.w2[at];
                    }
                }
            }
#pragma unroll
            for (int t = 0; t < kPassGroup; ++t) {
                if (q0 + t * spw < nq) {
                    const int q = q0 + t * spw + g;
                    const bool valid = g < spw && q < nq;
                    const uint64_t have = __ballot(valid && idv[t] >= 0) & (seg_mask << seg_base);
                    if (valid && idv[t] >= 0) {
                        const int slot = q * k2 + __popcll(have & lanemask_lt(lane));
                        leaf[slot] = idv[t];
                        if constexpr (WEIGHTED) leaf_w[slot] = wv[t];
                    }
                    if (valid && li == 0) cnt2[q] = __popcll(have);
                }
            }
        }
        __builtin_amdgcn_wave_barrier();
        if (lane < nq) c_own = cnt2[lane];
    }

    // Where each slot's rows go in the flat list: exclusive prefix sum of the counts over
    // lanes q (lanes without a slot count 0).  Sub-group sg later walks the rows of a
    // contiguous block of slots [qa, qb).
    const int incl = wave_inclusive_scan(c_own, lane);
    const int off_own = incl - c_own;
    const int total = __builtin_amdgcn_readlane(incl, 63);
    const uint64_t empty_mask = __ballot(lane < nq && c_own == 0);
    const int n_empty = __popcll(empty_mask);
    if (lane < nq && c_own == 0) empty_q[__popcll(empty_mask & lanemask_lt(lane))] = lane;
    if constexpr (!WEIGHTED) { if (lane == 0) live_slots[strip] = nq - n_empty; }
    if (lane < nq)
        rec[lane] = make_int4((int)(uint32_t)s_own, (int)(uint32_t)((uint64_t)s_own >> 32),
                              REPLAY ? c_own : (int)deg_own, off_own);

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
    __builtin_amdgcn_wave_barrier();

    if constexpr (!REPLAY) {
        // hop 1: (slot, step) pairs in passes of spw slots.  The `indices` loads of a pass group
        // are all issued before the first one is used; each sampled ID goes straight to its
        // place in the flat list as a row byte offset.
        for (int q0 = 0; q0 < nq; q0 += kPassGroup * spw) {       // wave-uniform trip count
            int idv[kPassGroup], dstv[kPassGroup];
            float wv[kPassGroup];
#pragma unroll
            for (int t = 0; t < kPassGroup; ++t) {
                idv[t] = -1;
                dstv[t] = -1;
                wv[t] = 0.0f;
                if (q0 + t * spw < nq) {                           // wave-uniform
                    const int q = q0 + t * spw + g;
                    const bool valid = g < spw && q < nq;
                    const int u = valid ? cnt2[q] : -1;
                    const bool active = valid && u >= 0;
                    int4 rc = make_int4(0, 0, 0, 0);
                    if (active) rc = rec[q];
                    const int64_t s = (int64_t)(((uint64_t)(uint32_t)rc.y << 32) | (uint32_t)rc.x);
                    const int64_t deg = (int64_t)(uint32_t)rc.z;
                    uint32_t wd = 0u;
                    if (__any(active && deg > (int64_t)k2)) wd = floyd_word(p.seed, (uint32_t)u, p.hop1, li);   // wave-uniform
                    const int64_t pos = floyd_resolve(floyd_bound(wd, k2, li, deg), k2, li, seg_base, deg, active, lane,
                                                      draws);
                    if (pos >= 0) {
                        idv[t] = p.indices[s + pos];
                        if constexpr (WEIGHTED) wv[t] = p.edge_w[s + pos];
                        const int c = (int)(deg < (int64_t)k2 ? deg : (int64_t)k2);
                        dstv[t] = (rc.w + li) | (li == c - 1 ? 0x40000000 : 0);
                    }
                }
            }
#pragma unroll
            for (int t = 0; t < kPassGroup; ++t) {
                if (q0 + t * spw < nq) {
                    const int q = q0 + t * spw + g;
                    const int j = wave + q * nw;
                    if (g < spw && q < nq) {
                        const int64_t at = (b * k1 + j) * k2 + li;
                        if (p.out_ids2) p.out_ids2[at] = idv[t];
                        if constexpr (WEIGHTED) { if (p.out_w2) p.out_w2[at] = idv[t] >= 0 ? wv[t] : 0.0f; }
                    }
                    if (dstv[t] >= 0) {
                        const int at = dstv[t] & 0x3fffffff;
                        const uint32_t last = (uint32_t)dstv[t] >> 30;
                        const uint64_t row_off = (uint64_t)(uint32_t)idv[t] * (uint64_t)p.row_bytes;
                        flat[at] = make_int2((int)(uint32_t)row_off, (int)((uint32_t)(row_off >> 32) | (last << 31)));
                        if constexpr (WEIGHTED) flat_w[at] = wv[t];
                        if (last) flat_meta[at] = j | (q << 8) | ((li + 1) << 16);
                    }
                }
            }
        }
    } else {
        for (int q0 = 0; q0 < nq; q0 += spw) {
            const int q = q0 + g;
            const bool valid = g < spw && q < nq;
            int4 rc = make_int4(0, 0, 0, 0);
            if (valid) rc = rec[q];
            const int c = rc.z;
            if (valid && li < c) {
                const int at = rc.w + li;
                const uint32_t last = li == c - 1 ? 1u : 0u;
                const uint64_t row_off = (uint64_t)(uint32_t)leaf[q * k2 + li] * (uint64_t)p.row_bytes;
                flat[at] = make_int2((int)(uint32_t)row_off, (int)((uint32_t)(row_off >> 32) | (last << 31)));
                if constexpr (WEIGHTED) flat_w[at] = leaf_w[q * k2 + li];
                if (last) flat_meta[at] = (wave + q * nw) | (q << 8) | (c << 16);
            }
        }
    }
    __builtin_amdgcn_wave_barrier();

    // gather
    FSA_STAMP(t_gather);
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
        float wacc = 0.0f, rootw = 0.0f;
        if (p.out_h1) {                                            // empty slots get zero rows
            for (int i = 0; i < n_empty; ++i) {
                char* dst = p.out_h1 + (b * k1 + wave + empty_q[i] * nw) * p.row_bytes;
                for (int chunk = lane; chunk < p.chunks; chunk += kWave)
                    *reinterpret_cast<Raw*>(dst + (int64_t)chunk * VB) = C::pack(acc[0]);
            }
        }
        for (int i0 = 0; i0 < total; i0 += R) {
            int2 ent[R];
            float wr[R];
            Raw r[R][MT];
#pragma unroll
            for (int u = 0; u < R; ++u) {
                const int i = i0 + u < total ? i0 + u : total - 1;
                ent[u] = flat[i];
                if constexpr (WEIGHTED) wr[u] = flat_w[i];
                const uint64_t row_off = row_offset_of(ent[u]);
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
                    for (int t = 0; t < MT; ++t) {
                        if (t < tiles) {
                            if constexpr (WEIGHTED) C::fma(acc[t], r[u][t], wr[u]);
                            else C::add(acc[t], r[u][t]);
                        }
                    }
                    if constexpr (WEIGHTED) wacc += wr[u];
                    if (ent[u].y < 0) {                            // last row of its slot
                        const int meta = flat_meta[i0 + u];
                        float inv, a = 1.0f;
                        if constexpr (WEIGHTED) {
                            inv = inv_weight(wacc);
                            a = wacc > 0.0f ? slot_a[(meta >> 8) & 0xff] : 0.0f;
                            rootw += a;
                            wacc = 0.0f;
                        } else {
                            inv = inv_count(meta >> 16);
                        }
                        char* dst = p.out_h1 ? p.out_h1 + (b * k1 + (meta & 0xff)) * p.row_bytes : nullptr;
#pragma unroll
                        for (int t = 0; t < MT; ++t) {
                            if (t < tiles) {
                                const int chunk = t * kWave + lane;
#pragma unroll
                                for (int e = 0; e < VE; ++e) {
                                    acc[t][e] *= inv;
                                    if constexpr (WEIGHTED) root[t][e] = fmaf(a, acc[t][e], root[t][e]);
                                    else root[t][e] += acc[t][e];
                                }
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
        if constexpr (WEIGHTED) { if (lane == 0) reinterpret_cast<float*>(live_slots)[strip] = rootw; }
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            if (t < tiles) {                                       // workgroup-uniform
                const int chunk = t * kWave + lane;
                const bool live = chunk < p.chunks;
                if (nw == 1) {
                    float inv1;
                    if constexpr (WEIGHTED) {
                        inv1 = inv_weight(rootw);
                    } else {
                        const int c1 = live_slots[strip];
                        if (t == 0 && lane == 0 && p.out_live) p.out_live[b] = c1;
                        inv1 = inv_count(c1 > 0 ? c1 : 1);
                    }
#pragma unroll
                    for (int e = 0; e < VE; ++e) root[t][e] *= inv1;
                    if (live && p.out) *reinterpret_cast<Raw*>(p.out + b * p.row_bytes + (int64_t)chunk * VB) = C::pack(root[t]);
                } else {
#pragma unroll
                    for (int e = 0; e < VE; ++e) red[(wave * kWave + lane) * VE + e] = root[t][e];
                    __syncthreads();
                    if (wave == 0) {
                        float inv1;
                        if constexpr (WEIGHTED) {
                            float totw = 0.0f;
                            for (int w = 0; w < nw; ++w) totw += reinterpret_cast<float*>(live_slots)[w];
                            inv1 = inv_weight(totw);
                        } else {
                            int c1 = 0;
                            for (int w = 0; w < nw; ++w) c1 += live_slots[w];
                            if (t == 0 && lane == 0 && p.out_live) p.out_live[b] = c1;
                            inv1 = inv_count(c1 > 0 ? c1 : 1);
                        }
                        float tot[VE];
#pragma unroll
                        for (int e = 0; e < VE; ++e) tot[e] = 0.0f;
                        for (int w = 0; w < nw; ++w) {
#pragma unroll
                            for (int e = 0; e < VE; ++e) tot[e] += red[(w * kWave + lane) * VE + e];
                        }
#pragma unroll
                        for (int e = 0; e < VE; ++e) tot[e] *= inv1;
                        if (live) *reinterpret_cast<Raw*>(p.out + b * p.row_bytes + (int64_t)chunk * VB) = C::pack(tot);
                    }
                    __syncthreads();                               // red is reused by the next tile
                }
            }
        }
    } else {
        // longest list of a sub-group: the trip count every lane of the wave shares
        int lmax = my_len;
        for (int off = sub; off < kWave; off <<= 1) {
            const int other = __shfl_xor(lmax, off);
            lmax = other > lmax ? other : lmax;
        }
        lmax = __builtin_amdgcn_readfirstlane(lmax);
        for (int c0 = 0; c0 < p.chunks; c0 += sub) {
            const int chunk = c0 + sl;
            const bool live = chunk < p.chunks;
            const int64_t chunk_off = (int64_t)chunk * VB;
            float acc[VE], root[VE];
#pragma unroll
            for (int e = 0; e < VE; ++e) { acc[e] = 0.0f; root[e] = 0.0f; }
            float wacc = 0.0f, rootw = 0.0f;
            if (p.out_h1 && live) {                                    // empty slots get zero rows
                for (int i = sg; i < n_empty; i += nsg)
                    *reinterpret_cast<Raw*>(p.out_h1 + (b * k1 + wave + empty_q[i] * nw) * p.row_bytes + chunk_off) = C::pack(acc);
            }
            // Rolling gather: U row loads per lane are in flight; as soon as the oldest one has
            // been added its register takes the load U entries further down the list.  The
            // loads carry no branch of their own (the hardware counter that orders them cannot
            // be tracked across one): past the end of its list a sub-group re-reads its last
            // row (a cache hit; a sub-group without rows re-reads the wave's first one) and
            // lanes beyond the row width re-read chunk 0; such results are never added.
            const int64_t load_off = live ? chunk_off : 0;
            if (lmax > 0) {                                            // wave-uniform
                const int list_at = my_len > 0 ? my_start : 0;
                const int last_i = my_len > 0 ? my_len - 1 : 0;
                Raw r[U];
                float wr[U];
                uint32_t ends = 0u;                                    // bit u: the entry in flight in r[u] ends its slot
                // add the row in r[u] (list entry i); close its slot if it is the last one
                auto consume = [&](int u, int i) {
                    if (i < my_len) {
                        if constexpr (WEIGHTED) { C::fma(acc, r[u], wr[u]); wacc += wr[u]; }
                        else C::add(acc, r[u]);
                        if ((ends >> u) & 1u) {
                            const int meta = flat_meta[my_start + i];
                            float inv, a = 1.0f;
                            if constexpr (WEIGHTED) {
                                inv = inv_weight(wacc);
                                a = wacc > 0.0f ? slot_a[(meta >> 8) & 0xff] : 0.0f;
                                rootw += a;
                                wacc = 0.0f;
                            } else {
                                inv = inv_count(meta >> 16);
                            }
#pragma unroll
                            for (int e = 0; e < VE; ++e) {
                                acc[e] *= inv;
                                if constexpr (WEIGHTED) root[e] = fmaf(a, acc[e], root[e]);
                                else root[e] += acc[e];
                            }
                            if (live && p.out_h1)
                                *reinterpret_cast<Raw*>(p.out_h1 + (b * k1 + (meta & 0xff)) * p.row_bytes + chunk_off) = C::pack(acc);
#pragma unroll
                            for (int e = 0; e < VE; ++e) acc[e] = 0.0f;
                        }
                    }
                };
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int ci = list_at + (u < last_i ? u : last_i);
                    const int2 ent = flat[ci];
                    if constexpr (WEIGHTED) wr[u] = flat_w[ci];
                    ends |= (uint32_t)(ent.y < 0 && u < my_len) << u;
                    r[u] = *reinterpret_cast<const Raw*>(p.x + row_offset_of(ent) + load_off);
                }
                int i0 = 0;
                for (; i0 + U < lmax; i0 += U) {                       // wave-uniform
                    int2 ent_n[U];
                    float wr_n[U];
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const int i = i0 + U + u;
                        const int ci = list_at + (i < last_i ? i : last_i);
                        ent_n[u] = flat[ci];
                        if constexpr (WEIGHTED) wr_n[u] = flat_w[ci];
                    }
                    uint32_t ends_n = 0u;
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        consume(u, i0 + u);
                        if constexpr (WEIGHTED) wr[u] = wr_n[u];
                        ends_n |= (uint32_t)(ent_n[u].y < 0 && i0 + U + u < my_len) << u;
                        r[u] = *reinterpret_cast<const Raw*>(p.x + row_offset_of(ent_n[u]) + load_off);
                    }
                    ends = ends_n;
                }
#pragma unroll
                for (int u = 0; u < U; ++u) consume(u, i0 + u);
            }
            for (int off = sub; off < kWave; off <<= 1) {
#pragma unroll
                for (int e = 0; e < VE; ++e) root[e] += __shfl_xor(root[e], off);
                if constexpr (WEIGHTED) rootw += __shfl_xor(rootw, off);
            }
            if (nw == 1) {
                float inv1;
                if constexpr (WEIGHTED) {
                    inv1 = inv_weight(rootw);
                } else {
                    const int c1 = live_slots[strip];
                    if (c0 == 0 && lane == 0 && p.out_live) p.out_live[b] = c1;
                    inv1 = inv_count(c1 > 0 ? c1 : 1);
                }
                if (sg == 0 && live && p.out) {                        // (a packed 1-hop call has no root mean)
#pragma unroll
                    for (int e = 0; e < VE; ++e) root[e] *= inv1;
                    *reinterpret_cast<Raw*>(p.out + b * p.row_bytes + chunk_off) = C::pack(root);
                }
                continue;
            }
            if (sg == 0) {
#pragma unroll
                for (int e = 0; e < VE; ++e) red[(wave * sub + sl) * VE + e] = root[e];
                if constexpr (WEIGHTED) { if (sl == 0) reinterpret_cast<float*>(live_slots)[wave] = rootw; }
            }
            __syncthreads();
            if (wave == 0 && sg == 0 && live) {
                float inv1;
                if constexpr (WEIGHTED) {
                    float totw = 0.0f;
                    for (int w = 0; w < nw; ++w) totw += reinterpret_cast<float*>(live_slots)[w];
                    inv1 = inv_weight(totw);
                } else {
                    int c1 = 0;
                    for (int w = 0; w < nw; ++w) c1 += live_slots[w];
                    if (c0 == 0 && sl == 0 && p.out_live) p.out_live[b] = c1;
                    inv1 = inv_count(c1 > 0 ? c1 : 1);
                }
                float tot[VE];
#pragma unroll
                for (int e = 0; e < VE; ++e) tot[e] = 0.0f;
                for (int w = 0; w < nw; ++w) {
#pragma unroll
                    for (int e = 0; e < VE; ++e) tot[e] += red[(w * sub + sl) * VE + e];
                }
#pragma unroll
                for (int e = 0; e < VE; ++e) tot[e] *= inv1;
                *reinterpret_cast<Raw*>(p.out + b * p.row_bytes + chunk_off) = C::pack(tot);
            }
            if (c0 + sub < p.chunks) __syncthreads();       // red is reused by the next tile
        }
    }
#ifdef FSA_TRACE
    if (p.trace && lane == 0 && wave == 0) {
        long long* t = p.trace + b * 4;
        t[0] = t_start; t[1] = t_gather; t[2] = wall_clock64(); t[3] = total;
    }
#endif
}

// ---------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------
// Waves per root for the 2-hop kernel.  One wave per root keeps the most roots resident and
// needs no block barrier; small batches are spread over more waves (which then own fewer
// hop-1 slots each) until the chip holds about 16 waves per CU.  Measured on the product,
// social and citation shapes at B = 1024 .. 65536.
int fwd2_waves(int64_t B, int k1, const RowGeom&) {
    const int forced = tune_int("FSA_FWD2_WAVES", 0);
    if (forced >= 1 && forced <= 8) return forced;
    int nw = 1;
    while (nw < 8 && nw * 2 <= k1 && B * nw < 4096) nw *= 2;
    return nw;
}

// Seeds per wave of a 1-hop call, or 0 for a wave per seed.  A wave per seed gives every seed the
// most lanes and loads in flight, which is best while the batch is within a few times the chip's
// wave slots (256 CUs x 4 SIMDs x 8 waves = 8192); beyond that, packing several seeds into one
// wave (64/k of them per sampling pass, at most kFwd1PackedPasses passes) multiplies the seeds in
// flight, and the launch is fastest with about one wave per slot.  Measured on the KG shape
// (2 rows per seed on average): B=65536 29.4 -> 23.7 us, B=262144 110 -> 68 us; at B=16384 a wave
// per seed is still ahead (11.1 against 12.3 us).
int fwd1_seeds_per_wave(int64_t B, int k) {
    const int forced = tune_int("FSA_FWD1_SEEDS_PER_WAVE", -1);
    if (forced >= 0) return forced > 64 ? 64 : forced;
    const int spw = kWave / k;
    if (B < 32768 || spw < 2) return 0;
    int64_t K = B / 8192;
    const int most = spw * kFwd1PackedPasses > 64 ? 64 : spw * kFwd1PackedPasses;
    if (K > most) K = most;
    return (int)K;                                                 // >= 4
}

// Dynamic LDS one workgroup may ask for on the current device.
static size_t lds_limit() {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess) return 0;
    return (size_t)v;
}

template <typename XT, int VB, bool WEIGHTED>
static hipError_t launch_typed(const FwdArgs& a, const FwdParams& p_in, hipStream_t stream) {
    constexpr int VE = Chunk<XT, VB>::VE;
    FwdParams p = p_in;
    const bool replay = a.indptr == nullptr;
    // rows of 2 .. kMultiTiles tiles of 64 lanes take the row-major multi-tile gather
    const int tiles = a.geom.tiles;
    const int mt = (tiles <= 1 || tiles > kMultiTiles) ? 0 : (tiles <= 4 ? 4 : 8);
    if constexpr (!WEIGHTED) {
        if (a.slot_cnt) {                       // mean over the per-slot rows of a [B,k1,D] table
            const int wpb = 4;
            const dim3 grid((unsigned)((a.B + wpb - 1) / wpb)), block(wpb * kWave);
            const size_t lds = sizeof(int) * kWave * wpb;
            if (mt == 0)      hipLaunchKernelGGL((slot_mean_kernel<XT, VB, 0>), grid, block, lds, stream, p);
            else if (mt == 4) hipLaunchKernelGGL((slot_mean_kernel<XT, VB, 4>), grid, block, lds, stream, p);
            else              hipLaunchKernelGGL((slot_mean_kernel<XT, VB, 8>), grid, block, lds, stream, p);
            return hipGetLastError();
        }
    }
    if (a.hops == 1 && fwd1_seeds_per_wave(a.B, a.k1) > 0 && !a.slot_cnt) {
        // Large 1-hop batches: several seeds per wave through the 2-hop kernel.  A seed of a sparse
        // graph names a handful of rows, so a wave of its own spends its life on the chain of
        // dependent loads (seed -> indptr -> indices -> rows) for a kilobyte or two; once the batch
        // exceeds the chip's wave slots that chain, not bandwidth, sets the rate.  Here a wave
        // takes K seeds as the "hop-1 slots" of the 2-hop kernel (hop 0 is skipped: its IDs are
        // the seeds), samples 64/k1 of them per pass with the seeds' own hop counter, and the
        // per-slot outputs of that kernel (mean, IDs, weights) are this call's outputs.
        const int K = fwd1_seeds_per_wave(a.B, a.k1);
        const size_t lds = (size_t)fwd2_lds_bytes(K, a.k1, 1, 1, WEIGHTED, a.geom.sub, VE);
        if (lds > lds_limit()) return hipErrorInvalidValue;
        p.packed_seeds = a.B;
        p.B = (a.B + K - 1) / K;
        p.k1 = K; p.k2 = a.k1;
        p.hop1 = a.hop_base;
        p.out_h1 = p.out; p.out = nullptr;
        p.out_ids2 = p.out_ids1; p.out_ids1 = nullptr;
        p.out_w2 = p.out_w1; p.out_w1 = nullptr;
        p.ids2 = p.ids1; p.ids1 = nullptr;
        p.w2 = p.w1; p.w1 = nullptr;
        p.out_live = nullptr;
        p.waves_per_root = 1;
        const dim3 grid((unsigned)p.B), block(kWave);
#define FSA_LAUNCH_FWD1P(MT_)                                                                                            \
        do {                                                                                                             \
            if (replay) hipLaunchKernelGGL((fwd2_kernel<XT, VB, true, MT_, WEIGHTED>), grid, block, lds, stream, p);     \
            else        hipLaunchKernelGGL((fwd2_kernel<XT, VB, false, MT_, WEIGHTED>), grid, block, lds, stream, p);    \
        } while (0)
        if (mt == 0) FSA_LAUNCH_FWD1P(0);
        else if (mt == 4) FSA_LAUNCH_FWD1P(4);
        else FSA_LAUNCH_FWD1P(8);
#undef FSA_LAUNCH_FWD1P
    } else if (a.hops == 1) {
        const int wpb_t = tune_int("FSA_FWD1_WAVES", 4);
        const int wpb = wpb_t >= 1 && wpb_t <= 4 ? wpb_t : 4;
        const dim3 grid((unsigned)((a.B + wpb - 1) / wpb)), block(wpb * kWave);
        const size_t lds = sizeof(int) * kFwd1StripInts * wpb;
#define FSA_LAUNCH_FWD1(MT_)                                                                                             \
        do {                                                                                                             \
            if (replay) hipLaunchKernelGGL((fwd1_kernel<XT, VB, true, MT_, WEIGHTED>), grid, block, lds, stream, p);     \
            else        hipLaunchKernelGGL((fwd1_kernel<XT, VB, false, MT_, WEIGHTED>), grid, block, lds, stream, p);    \
        } while (0)
        if (mt == 0) FSA_LAUNCH_FWD1(0);
        else if (mt == 4) FSA_LAUNCH_FWD1(4);
        else FSA_LAUNCH_FWD1(8);
#undef FSA_LAUNCH_FWD1
    } else {
        // waves per root: as few as the batch allows, but enough for the strips to fit in LDS
        int nw = fwd2_waves(a.B, a.k1, a.geom);
        const size_t limit = lds_limit();
        while (nw < 8 && nw * 2 <= a.k1 &&
               (size_t)fwd2_lds_bytes(a.k1, a.k2, nw, 1, WEIGHTED, a.geom.sub, VE) > limit)
            nw *= 2;
        // one wave per root: several roots share a workgroup when their LDS strips fit
        int rpw = 1;
        if (nw == 1) {
            rpw = tune_int("FSA_FWD2_ROOTS_PER_WG", kRootsPerWorkgroup);
            if (rpw < 1) rpw = 1;
            if (rpw > 8) rpw = 8;                                  // the kernel's launch bound is 8 waves
            while (rpw > 1 && (size_t)fwd2_lds_bytes(a.k1, a.k2, 1, rpw, WEIGHTED, a.geom.sub, VE) > 48 * 1024) rpw >>= 1;
        }
        const size_t lds = (size_t)fwd2_lds_bytes(a.k1, a.k2, nw, rpw, WEIGHTED, a.geom.sub, VE);
        if (lds > limit) return hipErrorInvalidValue;              // fanouts too large for this device's LDS
        const dim3 grid((unsigned)((a.B + rpw - 1) / rpw)), block(nw * rpw * kWave);
        p.waves_per_root = nw;
#define FSA_LAUNCH_FWD2(MT_)                                                                                             \
        do {                                                                                                             \
            if (replay) hipLaunchKernelGGL((fwd2_kernel<XT, VB, true, MT_, WEIGHTED>), grid, block, lds, stream, p);     \
            else        hipLaunchKernelGGL((fwd2_kernel<XT, VB, false, MT_, WEIGHTED>), grid, block, lds, stream, p);    \
        } while (0)
        if (mt == 0) FSA_LAUNCH_FWD2(0);
        else if (mt == 4) FSA_LAUNCH_FWD2(4);
        else FSA_LAUNCH_FWD2(8);
#undef FSA_LAUNCH_FWD2
    }
    return hipGetLastError();
}

template <bool WEIGHTED>
static hipError_t launch_forward_any(const FwdArgs& a, const WeightArgs* w, hipStream_t stream) {
    FwdParams p{};
    p.indptr = a.indptr; p.indices = a.indices; p.x = static_cast<const char*>(a.x);
    p.seeds = a.seeds; p.ids1 = a.ids1; p.ids2 = a.ids2;
    p.out = static_cast<char*>(a.out); p.out_h1 = static_cast<char*>(a.out_h1);
    p.out_ids1 = a.out_ids1; p.out_ids2 = a.out_ids2;
    if (w) { p.edge_w = w->edge_w; p.w1 = w->w1; p.w2 = w->w2; p.out_w1 = w->out_w1; p.out_w2 = w->out_w2; }
    p.B = a.B; p.row_bytes = a.D * (a.x_kind == 0 ? 4 : 2); p.seed = a.seed;
    p.k1 = a.k1; p.k2 = a.k2; p.chunks = a.geom.chunks; p.sub = a.geom.sub;
    p.sub_shift = __builtin_ctz((unsigned)a.geom.sub); p.indptr_is64 = a.indptr_is64;
    p.hop_base = a.hop_base; p.out_live = a.out_live; p.slot_cnt = a.slot_cnt;
    p.waves_per_root = 1;
    p.hop1 = a.hop_base + 1u;
    p.packed_seeds = 0;
#ifdef FSA_TRACE
    p.trace = g_trace;
#endif
    const int vb = a.geom.vec_bytes;
#ifdef FSA_FAST_BUILD
    // experiment builds: only the 16-byte-chunk kernels of the fp32 and bfloat16 tables
    if (vb != 16 || a.x_kind == 2) return hipErrorInvalidValue;
    if (a.x_kind == 1) return launch_typed<bf16_t, 16, WEIGHTED>(a, p, stream);
    return launch_typed<f32_t, 16, WEIGHTED>(a, p, stream);
#else
    if (a.x_kind == 1) {
        switch (vb) {
            case 16: return launch_typed<bf16_t, 16, WEIGHTED>(a, p, stream);
            case 8:  return launch_typed<bf16_t, 8, WEIGHTED>(a, p, stream);
            case 4:  return launch_typed<bf16_t, 4, WEIGHTED>(a, p, stream);
            default: return launch_typed<bf16_t, 2, WEIGHTED>(a, p, stream);
        }
    }
    if (a.x_kind == 2) {
        switch (vb) {
            case 16: return launch_typed<f16_t, 16, WEIGHTED>(a, p, stream);
            case 8:  return launch_typed<f16_t, 8, WEIGHTED>(a, p, stream);
            case 4:  return launch_typed<f16_t, 4, WEIGHTED>(a, p, stream);
            default: return launch_typed<f16_t, 2, WEIGHTED>(a, p, stream);
        }
    }
    switch (vb) {
        case 16: return launch_typed<f32_t, 16, WEIGHTED>(a, p, stream);
        case 8:  return launch_typed<f32_t, 8, WEIGHTED>(a, p, stream);
        default: return launch_typed<f32_t, 4, WEIGHTED>(a, p, stream);
    }
#endif
}

hipError_t launch_forward(const FwdArgs& a, hipStream_t stream) { return launch_forward_any<false>(a, nullptr, stream); }

hipError_t launch_forward_weighted(const FwdArgs& a, const WeightArgs& w, hipStream_t stream) {
    return launch_forward_any<true>(a, &w, stream);
}

}  // namespace fsa
