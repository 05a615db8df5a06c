// Forward kernels: fused sample + mean (Sec. 3.2 of arXiv 2511.13645) and the replay
// forward from saved IDs (Sec. 3.3, Prop. 1), for gfx950.
//
// Mapping (the paper's Sec. 4 uses warp-per-seed / block-per-root on 32-wide warps; this is
// the 64-wide-wavefront re-derivation):
//   1-hop: one wavefront per seed.  Lane i runs Floyd step i; the sampled IDs are staged in
//          a wave-private LDS strip; the wave is cut into 64/sub sub-groups of `sub` lanes,
//          each sub-group covers one feature row with 16/8/4-byte loads and the sub-groups
//          take different neighbor rows, so several rows are in flight per instruction.
//   2-hop: one workgroup per root.  Every wave redraws the root's hop-1 IDs (k1 lanes, no
//          block barrier needed) and owns the hop-1 slots j = wave, wave+W, ...; it samples
//          their rows in segments of k2 lanes (64/k2 rows at once), stages the leaf IDs in
//          its own LDS strip and then gathers them, one sub-group per slot, keeping each
//          slot's sum in registers.  Slot means go straight to out_h1; the root mean is
//          reduced across sub-groups by shuffles and across waves through LDS, and written
//          once.  No [B,k,D] gathered tensor and no block structure ever exists.
// The replay kernels are the same code with the sampler swapped for loads of the saved IDs,
// which is what makes replay bitwise equal to the sampling forward.
#include "fsa_device.hip.h"
#include "fsa_internal.h"

#include <cstdlib>

#ifndef FSA_UNROLL
#define FSA_UNROLL 10
#endif

namespace fsa {

struct FwdParams {
    const void* indptr; const int32_t* indices; const char* x;
    const int32_t* seeds; const int32_t* ids1; const int32_t* ids2;
    char* out; char* out_h1; int32_t* out_ids1; int32_t* out_ids2;
    int64_t B; int64_t row_bytes; uint64_t seed;
    int k1, k2, chunks, sub, sub_shift, indptr_is64;
};

__device__ __forceinline__ int64_t indptr_at(const FwdParams& p, int64_t i) {
    return p.indptr_is64 ? load_indptr<int64_t>(p.indptr, i) : load_indptr<int32_t>(p.indptr, i);
}

// Hop-0 step shared by both kernels: lane i < k1 ends up with the i-th sampled (or saved)
// hop-1 ID of root slot b, -1 in unused slots.  Replay keeps the saved layout (holes stay).
template <bool REPLAY>
__device__ __forceinline__ int hop0_id(const FwdParams& p, int64_t b, int lane) {
    if constexpr (REPLAY) {
        return lane < p.k1 ? p.ids1[b * p.k1 + lane] : -1;
    } else {
        const int64_t r = p.seeds[b];
        const int64_t s = indptr_at(p, r);
        const int64_t deg = indptr_at(p, r + 1) - s;
        const int64_t pos = floyd_position(p.seed, (uint32_t)r, 0u, p.k1, lane, 0, deg,
                                           lane < p.k1, lane);
        return pos >= 0 ? p.indices[s + pos] : -1;
    }
}

// ---------------------------------------------------------------------------------------
// 1-hop: wave per seed
// ---------------------------------------------------------------------------------------
template <typename XT, int VB, bool REPLAY>
__global__ __launch_bounds__(256) void fwd1_kernel(const FwdParams p) {
    using C = Chunk<XT, VB>;
    constexpr int VE = C::VE;
    extern __shared__ int smem[];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int64_t b = (int64_t)blockIdx.x * (blockDim.x >> 6) + wave;
    if (b >= p.B) return;                       // wave-uniform; no block barrier below
    int* ids = smem + wave * kWave;

    int id = hop0_id<REPLAY>(p, b, lane);
    if (!REPLAY && p.out_ids1 && lane < p.k1) p.out_ids1[b * p.k1 + lane] = id;
    // stage the valid IDs, in slot order, in this wave's LDS strip
    const uint64_t valid = __ballot(id >= 0);
    const int cnt = __popcll(valid);
    if (id >= 0) ids[__popcll(valid & lanemask_lt(lane))] = id;
    __builtin_amdgcn_wave_barrier();

    const int sub = p.sub;
    const int sg = lane >> p.sub_shift;         // sub-group index within the wave
    const int sl = lane & (sub - 1);
    const int nsg = kWave >> p.sub_shift;
    const float inv_guard = cnt > 0 ? (float)cnt : 1.0f;
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
            for (int e = 0; e < VE; ++e) acc[e] = acc[e] / inv_guard;
            *reinterpret_cast<typename C::Raw*>(p.out + b * p.row_bytes + (int64_t)chunk * VB) = C::pack(acc);
        }
    }
}

// ---------------------------------------------------------------------------------------
// 2-hop: workgroup per root, waves own interleaved hop-1 slots
// ---------------------------------------------------------------------------------------
template <typename XT, int VB, bool REPLAY>
__global__ __launch_bounds__(512) void fwd2_kernel(const FwdParams p) {
    using C = Chunk<XT, VB>;
    constexpr int VE = C::VE;
    extern __shared__ int smem[];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int nw = blockDim.x >> 6;
    const int64_t b = blockIdx.x;
    const int k1 = p.k1, k2 = p.k2;

    // LDS: per wave [nq_max*k2] leaf IDs + [nq_max] counts; then [nw] live-slot counts;
    // then [nw][sub*VE] floats for the cross-wave reduction.
    const int nq_max = (k1 + nw - 1) / nw;
    int* leaf = smem + wave * (nq_max * k2 + nq_max);
    int* cnt2 = leaf + nq_max * k2;
    int* live_slots = smem + nw * (nq_max * k2 + nq_max);
    float* red = reinterpret_cast<float*>(live_slots + nw);

    // hop 0, redundantly in every wave: lane j holds U[j]
    const int u_mine = hop0_id<REPLAY>(p, b, lane);
    if (!REPLAY && wave == 0 && p.out_ids1 && lane < k1) p.out_ids1[b * k1 + lane] = u_mine;

    // hop 1 for the slots this wave owns: j = wave + q*nw, q < nq
    const int nq = wave < k1 ? (k1 - wave + nw - 1) / nw : 0;
    const int spw = kWave / k2;                          // rows sampled at once
    const int g = lane / k2;
    const int li = lane - g * k2;
    for (int q0 = 0; q0 < nq; q0 += spw) {               // wave-uniform trip count
        const int q = q0 + g;
        const bool valid = g < spw && q < nq;
        const int j = wave + q * nw;
        const int u = __shfl(u_mine, valid ? j : 0);
        const bool active = valid && u >= 0;
        const int seg_base = valid ? g * k2 : 0;
        int id = -1;
        int c2 = 0;
        if constexpr (REPLAY) {
            if (active) id = p.ids2[(b * k1 + j) * k2 + li];
            const uint64_t seg = (k2 == 64 ? ~0ull : ((1ull << k2) - 1ull)) << seg_base;
            const uint64_t have = __ballot(id >= 0) & seg;
            c2 = __popcll(have);
            if (id >= 0) leaf[q * k2 + __popcll(have & lanemask_lt(lane))] = id;
        } else {
            int64_t s = 0, deg = 0;
            if (active) {
                s = indptr_at(p, u);
                deg = indptr_at(p, (int64_t)u + 1) - s;
            }
            const int64_t pos = floyd_position(p.seed, (uint32_t)u, 1u, k2, li, seg_base, deg,
                                               active, lane);
            if (pos >= 0) id = p.indices[s + pos];
            c2 = active ? (int)(deg < (int64_t)k2 ? deg : (int64_t)k2) : 0;
            if (valid) {
                leaf[q * k2 + li] = id;                  // valid IDs are a prefix of the slot
                if (p.out_ids2) p.out_ids2[(b * k1 + j) * k2 + li] = id;
            }
        }
        if (valid && li == 0) cnt2[q] = c2;
    }
    __builtin_amdgcn_wave_barrier();
    {
        const int mine = lane < nq ? cnt2[lane] : 0;
        const int n_live = __popcll(__ballot(mine > 0));
        if (lane == 0) live_slots[wave] = n_live;
    }

    // gather: one sub-group per owned slot
    const int sub = p.sub;
    const int sg = lane >> p.sub_shift;
    const int sl = lane & (sub - 1);
    const int nsg = kWave >> p.sub_shift;
    for (int c0 = 0; c0 < p.chunks; c0 += sub) {
        const int chunk = c0 + sl;
        const bool live = chunk < p.chunks;
        const int64_t chunk_off = (int64_t)chunk * VB;
        float root[VE];
#pragma unroll
        for (int e = 0; e < VE; ++e) root[e] = 0.0f;
        for (int q = sg; q < nq; q += nsg) {
            const int c = cnt2[q];
            float acc[VE];
#pragma unroll
            for (int e = 0; e < VE; ++e) acc[e] = 0.0f;
            if (live && c > 0) {
                sum_row_chunks<XT, VB, FSA_UNROLL>(p.x, p.row_bytes, chunk_off, leaf + q * k2, 0, c, 1, acc);
                const float fc = (float)c;
#pragma unroll
                for (int e = 0; e < VE; ++e) { acc[e] = acc[e] / fc; root[e] += acc[e]; }
            }
            if (live && p.out_h1) {
                const int64_t j = wave + q * nw;
                *reinterpret_cast<typename C::Raw*>(p.out_h1 + (b * k1 + j) * p.row_bytes + chunk_off) = C::pack(acc);
            }
        }
        for (int off = sub; off < kWave; off <<= 1) {
#pragma unroll
            for (int e = 0; e < VE; ++e) root[e] += __shfl_xor(root[e], off);
        }
        if (sg == 0) {
#pragma unroll
            for (int e = 0; e < VE; ++e) red[(wave * sub + sl) * VE + e] = root[e];
        }
        __syncthreads();
        if (wave == 0 && sg == 0 && live) {
            int c1 = 0;
            for (int w = 0; w < nw; ++w) c1 += live_slots[w];
            float tot[VE];
#pragma unroll
            for (int e = 0; e < VE; ++e) tot[e] = 0.0f;
            for (int w = 0; w < nw; ++w) {
#pragma unroll
                for (int e = 0; e < VE; ++e) tot[e] += red[(w * sub + sl) * VE + e];
            }
            const float fc1 = c1 > 0 ? (float)c1 : 1.0f;
#pragma unroll
            for (int e = 0; e < VE; ++e) tot[e] = tot[e] / fc1;
            *reinterpret_cast<typename C::Raw*>(p.out + b * p.row_bytes + chunk_off) = C::pack(tot);
        }
        if (c0 + sub < p.chunks) __syncthreads();       // red is reused by the next tile
    }
}

// ---------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------
static int env_int(const char* name, int fallback) {
    const char* v = std::getenv(name);
    return v ? std::atoi(v) : fallback;
}

// Waves per root for the 2-hop kernel: enough sub-groups that every hop-1 slot is gathered
// in one pass when that fits in 8 waves.
int fwd2_waves(int k1, const RowGeom& g) {
    static const int forced = env_int("FSA_FWD2_WAVES", 0);
    if (forced >= 1 && forced <= 8) return forced;
    const int per_wave = kWave / g.sub;
    int nw = (k1 + per_wave - 1) / per_wave;
    if (nw < 1) nw = 1;
    if (nw > 8) nw = 8;
    return nw;
}

template <typename XT, int VB>
static hipError_t launch_typed(const FwdArgs& a, const FwdParams& p, hipStream_t stream) {
    constexpr int VE = Chunk<XT, VB>::VE;
    const bool replay = a.indptr == nullptr;
    if (a.hops == 1) {
        static const int wpb = [] { int v = env_int("FSA_FWD1_WAVES", 4); return v >= 1 && v <= 4 ? v : 4; }();
        const unsigned grid = (unsigned)((a.B + wpb - 1) / wpb);
        const size_t lds = sizeof(int) * kWave * wpb;
        if (replay) hipLaunchKernelGGL((fwd1_kernel<XT, VB, true>), dim3(grid), dim3(wpb * kWave), lds, stream, p);
        else        hipLaunchKernelGGL((fwd1_kernel<XT, VB, false>), dim3(grid), dim3(wpb * kWave), lds, stream, p);
    } else {
        const int nw = fwd2_waves(a.k1, a.geom);
        const int nq_max = (a.k1 + nw - 1) / nw;
        const size_t lds = sizeof(int) * ((size_t)nw * (nq_max * a.k2 + nq_max) + nw)
                         + sizeof(float) * (size_t)nw * a.geom.sub * VE;
        if (replay) hipLaunchKernelGGL((fwd2_kernel<XT, VB, true>), dim3((unsigned)a.B), dim3(nw * kWave), lds, stream, p);
        else        hipLaunchKernelGGL((fwd2_kernel<XT, VB, false>), dim3((unsigned)a.B), dim3(nw * kWave), lds, stream, p);
    }
    return hipGetLastError();
}

hipError_t launch_forward(const FwdArgs& a, hipStream_t stream) {
    FwdParams p;
    p.indptr = a.indptr; p.indices = a.indices; p.x = static_cast<const char*>(a.x);
    p.seeds = a.seeds; p.ids1 = a.ids1; p.ids2 = a.ids2;
    p.out = static_cast<char*>(a.out); p.out_h1 = static_cast<char*>(a.out_h1);
    p.out_ids1 = a.out_ids1; p.out_ids2 = a.out_ids2;
    p.B = a.B; p.row_bytes = a.D * (a.x_is_bf16 ? 2 : 4); p.seed = a.seed;
    p.k1 = a.k1; p.k2 = a.k2; p.chunks = a.geom.chunks; p.sub = a.geom.sub;
    p.sub_shift = __builtin_ctz((unsigned)a.geom.sub); p.indptr_is64 = a.indptr_is64;
    const int vb = a.geom.vec_bytes;
    if (a.x_is_bf16) {
        switch (vb) {
            case 16: return launch_typed<bf16_t, 16>(a, p, stream);
            case 8:  return launch_typed<bf16_t, 8>(a, p, stream);
            case 4:  return launch_typed<bf16_t, 4>(a, p, stream);
            default: return launch_typed<bf16_t, 2>(a, p, stream);
        }
    }
    switch (vb) {
        case 16: return launch_typed<f32_t, 16>(a, p, stream);
        case 8:  return launch_typed<f32_t, 8>(a, p, stream);
        default: return launch_typed<f32_t, 4>(a, p, stream);
    }
}

}  // namespace fsa
