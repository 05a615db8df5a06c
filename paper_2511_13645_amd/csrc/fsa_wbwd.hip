// Weighted-mean backward, 2-hop: the adjoint, with respect to the feature table, of the
// weighted replay forward (weights are data).  Same ownership and the same atomic row-adds as
// the unweighted backward; the share of a sampled row is its weight over the slot's weight
// sum instead of 1/count, and equal IDs inside a slot are merged by adding their weights.
// The 1-hop case runs in the unweighted 1-hop kernel (fsa_bwd.hip) with weight shares.
#include "fsa_device.hip.h"
#include "fsa_internal.h"

namespace fsa {

struct WBwdParams {
    const float* grad_out; const float* grad_h1; const int32_t* ids1; const int32_t* ids2;
    const float* w1; const float* w2; float* grad_x; int64_t B; int64_t D; int k1, k2;
};

__device__ __forceinline__ void w_atomic_add(float* addr, float v) { unsafeAtomicAdd(addr, v); }

__global__ __launch_bounds__(512) void wbwd2_kernel(const WBwdParams p) {
    extern __shared__ int smem[];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int nw = blockDim.x >> 6;
    const int64_t b = blockIdx.x;
    const int k1 = p.k1, k2 = p.k2;
    const int nq_max = (k1 + nw - 1) / nw;
    // per wave: distinct leaf rows and their shares [nq_max*k2] each, per-slot distinct count,
    // hop-0 weight and "takes part" flag [nq_max] each; then one outer-weight partial per wave
    const int per_wave = 2 * nq_max * k2 + 3 * nq_max;
    int* leaf = smem + wave * per_wave;
    float* share = reinterpret_cast<float*>(leaf + nq_max * k2);
    int* uniq = leaf + 2 * nq_max * k2;
    float* slot_a = reinterpret_cast<float*>(uniq + nq_max);
    int* part = uniq + 2 * nq_max;
    float* outer = reinterpret_cast<float*>(smem + nw * per_wave);

    const int u_mine = lane < k1 ? p.ids1[b * k1 + lane] : -1;
    const float a_mine = u_mine >= 0 ? p.w1[b * k1 + lane] : 0.0f;
    const int nq = wave < k1 ? (k1 - wave + nw - 1) / nw : 0;
    const int own_src = lane < nq ? wave + lane * nw : 0;
    const int u_own = __shfl(u_mine, own_src);
    const float a_own = __shfl(a_mine, own_src);
    const int spw = kWave / k2;
    const int g = lane / k2;
    const int li = lane - g * k2;
    const uint64_t seg_mask = k2 == 64 ? ~0ull : ((1ull << k2) - 1ull);
    float my_outer = 0.0f;                              // lane 0 of each segment adds its slot's weight
    for (int q0 = 0; q0 < nq; q0 += spw) {              // wave-uniform trip count
        const int q = q0 + g;
        const bool valid = g < spw && q < nq;
        const int j = wave + q * nw;
        const int u = __shfl(u_own, valid ? q : 0);
        const float a = __shfl(a_own, valid ? q : 0);
        const bool active = valid && u >= 0;
        const int seg_base = valid ? g * k2 : 0;
        const int id = active ? p.ids2[(b * k1 + j) * k2 + li] : -1;
        const float w = id >= 0 ? p.w2[(b * k1 + j) * k2 + li] : 0.0f;
        // weight sum of the segment: butterfly over the wave restricted to the segment by masking
        float tot = 0.0f;
        for (int m = 0; m < k2; ++m) tot += __shfl(w, seg_base + m);
        float wsum; bool first;
        merge_equal_ids_w(id, w, k2, li, seg_base, wsum, first);
        const bool takes_part = active && tot > 0.0f;
        const bool keep = id >= 0 && first && takes_part;
        const uint64_t kept = __ballot(keep) & (seg_mask << seg_base);
        if (keep) {
            const int slot = __popcll(kept & lanemask_lt(lane));
            leaf[q * k2 + slot] = id;
            share[q * k2 + slot] = wsum / tot;
        }
        if (valid && li == 0) {
            uniq[q] = __popcll(kept);
            slot_a[q] = a;
            part[q] = takes_part ? 1 : 0;
            if (takes_part) my_outer += a;
        }
    }
    for (int off = 1; off < kWave; off <<= 1) my_outer += __shfl_xor(my_outer, off);
    if (lane == 0) outer[wave] = my_outer;
    __syncthreads();
    float outer_total = 0.0f;
    for (int w = 0; w < nw; ++w) outer_total += outer[w];

    for (int q = 0; q < nq; ++q) {
        if (!part[q]) continue;
        const int n = uniq[q];
        const int64_t j = wave + q * nw;
        const float outer_share = outer_total > 0.0f ? slot_a[q] / outer_total : 0.0f;
        for (int64_t d0 = 0; d0 < p.D; d0 += kWave) {
            const int64_t d = d0 + lane;
            if (d < p.D) {
                float gsum = p.grad_out[b * p.D + d] * outer_share;
                if (p.grad_h1) gsum += p.grad_h1[(b * k1 + j) * p.D + d];
                for (int e = 0; e < n; ++e)
                    w_atomic_add(p.grad_x + (int64_t)leaf[q * k2 + e] * p.D + d, gsum * share[q * k2 + e]);
            }
        }
    }
}

hipError_t launch_backward_weighted(const BwdArgs& a, const WeightArgs& w, hipStream_t stream) {
    WBwdParams p;
    // the weighted backward is fp32 on both sides
    p.grad_out = static_cast<const float*>(a.grad_out); p.grad_h1 = static_cast<const float*>(a.grad_h1);
    p.ids1 = a.ids1; p.ids2 = a.ids2;
    p.w1 = w.w1; p.w2 = w.w2; p.grad_x = static_cast<float*>(a.grad_x); p.B = a.B; p.D = a.D; p.k1 = a.k1; p.k2 = a.k2;
    if (!a.ids2) {
        // 1-hop: the unweighted kernel with weight shares instead of 1/count (it merges the rows
        // the seeds of a workgroup share in LDS, which the hub rows of a skewed graph need)
        return launch_backward1_weighted(a, w.w1, stream);
    } else {
        const int nw = a.k1 < 8 ? a.k1 : 8;
        const int nq_max = (a.k1 + nw - 1) / nw;
        const size_t lds = sizeof(int) * ((size_t)nw * (2 * nq_max * a.k2 + 3 * nq_max) + nw);
        hipLaunchKernelGGL(wbwd2_kernel, dim3((unsigned)a.B), dim3(nw * kWave), lds, stream, p);
    }
    return hipGetLastError();
}

}  // namespace fsa
