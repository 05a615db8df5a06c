// Backward kernels: the adjoint of the replay forward with respect to the feature table
// (Sec. 3.3 "Reproducibility" of arXiv 2511.13645: backward replays the saved IDs so that
// gradients reach the same sampled neighborhoods).  The paper does not describe a kernel.
//
// Mapping: the same ownership as the forward (wave per seed; workgroup per root with waves
// owning interleaved hop-1 slots).  For each owned slot the wave first aggregates inside
// itself: equal IDs within the slot (parallel edges) are merged into one entry with a
// multiplicity, so each distinct row receives one atomic per element.  Lanes then map to
// consecutive floats of the row, so one wave instruction adds 256 contiguous bytes with
// hardware fp32 atomics resolved at L2.
#include "fsa_device.hip.h"
#include "fsa_internal.h"

#include <cstdlib>

namespace fsa {

struct BwdParams {
    const float* grad_out; const float* grad_h1; const int32_t* ids1; const int32_t* ids2;
    float* grad_x; int64_t B; int64_t D; int k1, k2;
};

__device__ __forceinline__ void atomic_add_f32(float* addr, float v) {
    unsafeAtomicAdd(addr, v);        // global_atomic_add_f32, no return value
}

// Merge equal IDs inside a segment of `k` lanes starting at seg_base.  Returns how many
// times this lane's ID occurs in the segment and whether this lane is its first occurrence.
__device__ __forceinline__ void merge_equal_ids(int id, int k, int li, int seg_base, int& mult,
                                                bool& first) {
    mult = 0;
    first = true;
    for (int m = 0; m < k; ++m) {
        const int other = __shfl(id, seg_base + m);
        if (other == id) { ++mult; if (m < li) first = false; }
    }
}

__global__ __launch_bounds__(256) void bwd1_kernel(const BwdParams p) {
    extern __shared__ int smem[];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int64_t b = (int64_t)blockIdx.x * (blockDim.x >> 6) + wave;
    if (b >= p.B) return;                               // wave-uniform, no block barrier below
    int* rows = smem + wave * 2 * kWave;
    float* weight = reinterpret_cast<float*>(rows + kWave);

    const int id = lane < p.k1 ? p.ids1[b * p.k1 + lane] : -1;
    const int cnt = __popcll(__ballot(id >= 0));
    int mult; bool first;
    merge_equal_ids(id, p.k1, lane, 0, mult, first);
    const bool keep = id >= 0 && first;
    const uint64_t kept = __ballot(keep);
    const int n = __popcll(kept);
    if (keep) {
        const int slot = __popcll(kept & lanemask_lt(lane));
        rows[slot] = id;
        weight[slot] = (float)mult / (float)cnt;
    }
    __builtin_amdgcn_wave_barrier();
    for (int64_t d0 = 0; d0 < p.D; d0 += kWave) {
        const int64_t d = d0 + lane;
        if (d < p.D) {
            const float g = p.grad_out[b * p.D + d];
            for (int e = 0; e < n; ++e)
                atomic_add_f32(p.grad_x + (int64_t)rows[e] * p.D + d, g * weight[e]);
        }
    }
}

__global__ __launch_bounds__(512) void bwd2_kernel(const BwdParams p) {
    extern __shared__ int smem[];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int nw = blockDim.x >> 6;
    const int64_t b = blockIdx.x;
    const int k1 = p.k1, k2 = p.k2;
    const int nq_max = (k1 + nw - 1) / nw;
    // per wave: leaf rows, multiplicities, per-slot total count and distinct count
    const int per_wave = 2 * nq_max * k2 + 2 * nq_max;
    int* leaf = smem + wave * per_wave;
    int* mul = leaf + nq_max * k2;
    int* cnt2 = mul + nq_max * k2;
    int* uniq = cnt2 + nq_max;
    int* live_slots = smem + nw * per_wave;

    const int u_mine = lane < k1 ? p.ids1[b * k1 + lane] : -1;
    const int nq = wave < k1 ? (k1 - wave + nw - 1) / nw : 0;
    const int spw = kWave / k2;
    const int g = lane / k2;
    const int li = lane - g * k2;
    for (int q0 = 0; q0 < nq; q0 += spw) {              // wave-uniform trip count
        const int q = q0 + g;
        const bool valid = g < spw && q < nq;
        const int j = wave + q * nw;
        const int u = __shfl(u_mine, valid ? j : 0);
        const bool active = valid && u >= 0;
        const int seg_base = valid ? g * k2 : 0;
        const int id = active ? p.ids2[(b * k1 + j) * k2 + li] : -1;
        const uint64_t seg = (k2 == 64 ? ~0ull : ((1ull << k2) - 1ull)) << seg_base;
        const int c2 = __popcll(__ballot(id >= 0) & seg);
        int mult; bool first;
        merge_equal_ids(id, k2, li, seg_base, mult, first);
        const bool keep = id >= 0 && first;
        const uint64_t kept = __ballot(keep) & seg;
        if (keep) {
            const int slot = __popcll(kept & lanemask_lt(lane));
            leaf[q * k2 + slot] = id;
            mul[q * k2 + slot] = mult;
        }
        if (valid && li == 0) { cnt2[q] = c2; uniq[q] = __popcll(kept); }
    }
    __builtin_amdgcn_wave_barrier();
    {
        const int mine = lane < nq ? cnt2[lane] : 0;
        const int n_live = __popcll(__ballot(mine > 0));
        if (lane == 0) live_slots[wave] = n_live;
    }
    __syncthreads();
    int c1 = 0;
    for (int w = 0; w < nw; ++w) c1 += live_slots[w];
    if (c1 == 0) return;
    const float fc1 = (float)c1;

    for (int q = 0; q < nq; ++q) {
        const int c = cnt2[q];
        if (c == 0) continue;
        const int n = uniq[q];
        const int64_t j = wave + q * nw;
        const float fc = (float)c;
        for (int64_t d0 = 0; d0 < p.D; d0 += kWave) {
            const int64_t d = d0 + lane;
            if (d < p.D) {
                float gsum = p.grad_out[b * p.D + d] / fc1;
                if (p.grad_h1) gsum += p.grad_h1[(b * k1 + j) * p.D + d];
                gsum = gsum / fc;
                for (int e = 0; e < n; ++e)
                    atomic_add_f32(p.grad_x + (int64_t)leaf[q * k2 + e] * p.D + d,
                                   gsum * (float)mul[q * k2 + e]);
            }
        }
    }
}

static int env_int(const char* name, int fallback) {
    const char* v = std::getenv(name);
    return v ? std::atoi(v) : fallback;
}

hipError_t launch_backward(const BwdArgs& a, hipStream_t stream) {
    BwdParams p;
    p.grad_out = a.grad_out; p.grad_h1 = a.grad_h1; p.ids1 = a.ids1; p.ids2 = a.ids2;
    p.grad_x = a.grad_x; p.B = a.B; p.D = a.D; p.k1 = a.k1; p.k2 = a.k2;
    if (!a.ids2) {
        const int wpb = 4;
        const unsigned grid = (unsigned)((a.B + wpb - 1) / wpb);
        hipLaunchKernelGGL(bwd1_kernel, dim3(grid), dim3(wpb * kWave), sizeof(int) * 2 * kWave * wpb,
                           stream, p);
    } else {
        static const int forced = env_int("FSA_BWD2_WAVES", 0);
        int nw = (forced >= 1 && forced <= 8) ? forced : (a.k1 < 8 ? a.k1 : 8);
        const int nq_max = (a.k1 + nw - 1) / nw;
        const size_t lds = sizeof(int) * ((size_t)nw * (2 * nq_max * a.k2 + 2 * nq_max) + nw);
        hipLaunchKernelGGL(bwd2_kernel, dim3((unsigned)a.B), dim3(nw * kWave), lds, stream, p);
    }
    return hipGetLastError();
}

}  // namespace fsa
