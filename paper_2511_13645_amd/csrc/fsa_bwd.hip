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

#include <type_traits>

namespace fsa {

struct BwdParams {
    const void* grad_out; const void* grad_h1; const int32_t* ids1; const int32_t* ids2;
    void* grad_x; int64_t B; int64_t D; int k1, k2;
    const float* w1;                     // 1-hop weighted mean: [B,k1] weights of the sampled edges, else unused
    const int32_t* root_valid;           // 2-hop, nullable: [B], a negative entry switches root b off
};

// ---------------------------------------------------------------------------------------
// Element types of the incoming gradients (GT) and of grad_x (XG).  With an fp32 grad_x a
// lane owns one element of the row (EPL = 1), whatever the type of the incoming gradients, so
// that one wave instruction of global_atomic_add_f32 covers 256 contiguous bytes (pairs per
// lane would leave every instruction striding over twice as many cache lines: measured 1.7x
// slower).  With a 16-bit grad_x a lane owns two consecutive elements (EPL = 2; D is even)
// and adds the pair in ONE packed atomic (global_atomic_pk_add_bf16 / _f16), which halves the
// number of atomic operations per row -- the L2 atomic unit, not bandwidth, bounds this
// kernel.  Products and sums before the atomic are fp32; the value is rounded to the 16-bit
// type once (nearest-even) and every packed atomic rounds the running sum again.
// ---------------------------------------------------------------------------------------
struct g_f32 { using T = float; };
struct g_bf16 { using T = uint16_t; };
struct g_f16 { using T = uint16_t; };

template <typename GT, typename XG> struct Epl { static constexpr int value = 2; };
template <typename GT> struct Epl<GT, g_f32> { static constexpr int value = 1; };

typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));

// EPL consecutive gradient elements starting at element index `idx` (even when EPL == 2).
template <typename GT, int EPL>
__device__ __forceinline__ void load_grad(const void* base, int64_t idx, float (&g)[EPL]) {
    if constexpr (std::is_same<GT, g_f32>::value) {
        const float* p = static_cast<const float*>(base) + idx;
#pragma unroll
        for (int e = 0; e < EPL; ++e) g[e] = p[e];
    } else if constexpr (EPL == 1) {
        const uint16_t w = static_cast<const uint16_t*>(base)[idx];
        if constexpr (std::is_same<GT, g_bf16>::value) {
            g[0] = __uint_as_float((uint32_t)w << 16);
        } else {
            _Float16 h;
            __builtin_memcpy(&h, &w, sizeof h);
            g[0] = (float)h;
        }
    } else {
        const uint32_t w = *reinterpret_cast<const uint32_t*>(static_cast<const uint16_t*>(base) + idx);
        if constexpr (std::is_same<GT, g_bf16>::value) {
            g[0] = __uint_as_float(w << 16);
            g[1] = __uint_as_float(w & 0xffff0000u);
        } else {
            f16x2_t h;
            __builtin_memcpy(&h, &w, sizeof h);
            const f32x2_t f = __builtin_convertvector(h, f32x2_t);
            g[0] = f[0];
            g[1] = f[1];
        }
    }
}

// grad_x[idx .. idx+EPL) += v, by hardware atomics without a return value.
template <typename XG, int EPL>
__device__ __forceinline__ void atomic_add_row(void* base, int64_t idx, const float (&v)[EPL]) {
    if constexpr (std::is_same<XG, g_f32>::value) {
        float* p = static_cast<float*>(base) + idx;
#pragma unroll
        for (int e = 0; e < EPL; ++e) unsafeAtomicAdd(p + e, v[e]);          // global_atomic_add_f32
    } else {
        static_assert(EPL == 2, "16-bit grad_x takes packed pairs");
        const f32x2_t f = {v[0], v[1]};
        uint16_t* p = static_cast<uint16_t*>(base) + idx;
        if constexpr (std::is_same<XG, g_bf16>::value) {
            const bf16x2_t b = __builtin_convertvector(f, bf16x2_t);
            __builtin_amdgcn_global_atomic_fadd_v2bf16(reinterpret_cast<bf16x2_t*>(p), b);
        } else {
            const f16x2_t h = __builtin_convertvector(f, f16x2_t);
            __builtin_amdgcn_global_atomic_fadd_v2f16(reinterpret_cast<f16x2_t*>(p), h);
        }
    }
}

// Merge equal IDs inside a segment of `k` lanes starting at seg_base.  Returns how many
// times this lane's ID occurs in the segment and whether this lane is its first occurrence.
__device__ __forceinline__ void merge_equal_ids(int id, int k, int li, int seg_base, int& mult,
                                                bool& first) {
    mult = 0;
    first = true;
    for (int m0 = 0; m0 < k; m0 += 8) {                 // eight shuffles in flight at a time
        int other[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) other[j] = __shfl(id, seg_base + m0 + j);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if (m0 + j < k && other[j] == id) { ++mult; if (m0 + j < li) first = false; }
        }
    }
}

// ---------------------------------------------------------------------------------------
// 1-hop backward.  A workgroup of nw (16) waves takes nw*spw consecutive seeds (wave w the
// seeds w, w+nw, ...).  Rows that many seeds of the workgroup share -- the hub rows of a skewed
// graph, which would otherwise serialise thousands of atomics on one L2 channel -- are first
// summed in LDS and reach grad_x with ONE atomic row-add per workgroup:
//   pass 1  every sampled ID bumps an LDS counter at hash(id);
//   pass 2  the count threshold is doubled from kHotMin until no more buckets reach it than
//           there are LDS rows; IDs in such buckets claim them (first claimant wins; a
//           colliding ID simply stays on the direct path) and claimed buckets get an LDS row;
//   pass 3  per seed: equal IDs of the seed are merged (multiplicity), then each distinct row
//           receives grad_out[b,:] * mult/cnt -- into its LDS row if it owns a bucket, else
//           straight into grad_x with hardware fp32 atomics, 256 contiguous bytes per wave
//           instruction;
//   flush   LDS rows are added to grad_x.
// When no counter reaches kHotMin (uniform graphs) passes 2 and flush are skipped.
// ---------------------------------------------------------------------------------------
constexpr int kHotBuckets = 2048;
constexpr int kHotMin = 3;
constexpr int kHotRowsMax = 64;

__device__ __forceinline__ int hot_hash(int id) {
    return (int)(((uint32_t)id * 2654435761u) >> 21);              // 11 bits -> kHotBuckets
}

template <typename GT, typename XG, bool WEIGHTED>
__global__ __launch_bounds__(1024) void bwd1_kernel(const BwdParams p, int spw, int hot_rows) {
    constexpr int EPL = Epl<GT, XG>::value;
    extern __shared__ int smem[];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int nw = blockDim.x >> 6;
    // LDS: counters, tags, row-of-bucket [kHotBuckets] each; [2] flags; node of each LDS row
    // [kHotRowsMax]; per wave [64] rows + [64] weights + [64] hot-row index; then hot_rows * D
    // floats.
    int* count = smem;
    int* tag = count + kHotBuckets;
    int* row_of = tag + kHotBuckets;
    int* flags = row_of + kHotBuckets;                               // [0] any hot, [1] rows handed out
    int* row_node = flags + 2;
    int* rows = row_node + kHotRowsMax + wave * 3 * kWave;
    float* weight = reinterpret_cast<float*>(rows + kWave);
    int* hot_of = rows + 2 * kWave;
    float* hot = reinterpret_cast<float*>(row_node + kHotRowsMax + nw * 3 * kWave);
    const int64_t b0 = (int64_t)blockIdx.x * nw * spw;

    for (int i = threadIdx.x; i < kHotBuckets; i += blockDim.x) { count[i] = 0; tag[i] = -1; row_of[i] = -1; }
    if (threadIdx.x < 2) flags[threadIdx.x] = 0;
    __syncthreads();

    // pass 1: count IDs per bucket (lanes cover consecutive entries of the workgroup's seeds)
    const bool use_hot = hot_rows > 0;
    if (use_hot) {
        const int64_t first = b0 * p.k1;
        const int64_t n_ent = ((b0 + (int64_t)nw * spw < p.B ? b0 + (int64_t)nw * spw : p.B) - b0) * p.k1;
        bool saw_hot = false;
        for (int64_t e = threadIdx.x; e < n_ent; e += blockDim.x) {
            const int id = p.ids1[first + e];
            if (id >= 0) saw_hot = (atomicAdd(&count[hot_hash(id)], 1) + 1 >= kHotMin) || saw_hot;
        }
        if (saw_hot) flags[0] = 1;
        __syncthreads();
        if (flags[0]) {                                              // workgroup-uniform
            // pass 2: the busiest buckets, as many as there are LDS rows
            int thresh = kHotMin;
            for (;;) {                                               // workgroup-uniform trip count
                int mine = 0;
                for (int i = threadIdx.x; i < kHotBuckets; i += blockDim.x) mine += count[i] >= thresh;
                if (mine) atomicAdd(&flags[1], mine);
                __syncthreads();
                const int n_over = flags[1];
                __syncthreads();
                if (threadIdx.x == 0) flags[1] = 0;
                __syncthreads();
                if (n_over <= hot_rows) break;
                thresh *= 2;
            }
            for (int64_t e = threadIdx.x; e < n_ent; e += blockDim.x) {
                const int id = p.ids1[first + e];
                if (id >= 0 && count[hot_hash(id)] >= thresh) atomicCAS(&tag[hot_hash(id)], -1, id);
            }
            __syncthreads();
            for (int i = threadIdx.x; i < kHotBuckets; i += blockDim.x) {
                if (tag[i] >= 0) {                                   // at most hot_rows buckets qualify
                    const int r = atomicAdd(&flags[1], 1);
                    row_of[i] = r;
                    row_node[r] = tag[i];
                }
            }
            __syncthreads();
            const int n_rows = flags[1];
            for (int64_t i = threadIdx.x; i < (int64_t)n_rows * p.D; i += blockDim.x) hot[i] = 0.0f;
            __syncthreads();
        }
    }
    const bool any_hot = use_hot && flags[0] != 0;

    // pass 3: one seed at a time per wave
    for (int s = 0; s < spw; ++s) {
        const int64_t b = b0 + wave + (int64_t)s * nw;
        if (b >= p.B) break;                                         // wave-uniform
        const int id = lane < p.k1 ? p.ids1[b * p.k1 + lane] : -1;
        // share of the seed's gradient that this lane's row receives: multiplicity / count, or,
        // for the weighted mean, the summed weight of its occurrences / the seed's weight sum
        // (a seed whose weights sum to zero contributes nothing)
        float share;
        bool first;
        bool live_seed = true;
        if constexpr (WEIGHTED) {
            const float w = id >= 0 ? p.w1[b * p.k1 + lane] : 0.0f;
            float total = w;
            for (int off = 1; off < kWave; off <<= 1) total += __shfl_xor(total, off);
            float wsum;
            merge_equal_ids_w(id, w, p.k1, lane, 0, wsum, first);
            live_seed = total > 0.0f;
            share = live_seed ? wsum / total : 0.0f;
        } else {
            const int cnt = __popcll(__ballot(id >= 0));
            int mult;
            merge_equal_ids(id, p.k1, lane, 0, mult, first);
            share = (float)mult / (float)cnt;
        }
        const bool keep = id >= 0 && first && live_seed;
        const uint64_t kept = __ballot(keep);
        const int n = __popcll(kept);
        if (keep) {
            const int slot = __popcll(kept & lanemask_lt(lane));
            rows[slot] = id;
            weight[slot] = share;
            int hr = -1;
            if (any_hot) { const int h = hot_hash(id); if (tag[h] == id) hr = row_of[h]; }
            hot_of[slot] = hr;
        }
        __builtin_amdgcn_wave_barrier();
        for (int64_t d0 = 0; d0 < p.D; d0 += kWave * EPL) {
            const int64_t d = d0 + lane * EPL;
            if (d < p.D) {
                float g[EPL];
                load_grad<GT, EPL>(p.grad_out, b * p.D + d, g);
                for (int e = 0; e < n; ++e) {
                    const int hr = hot_of[e];
                    const float wt = weight[e];
                    float v[EPL];
#pragma unroll
                    for (int c = 0; c < EPL; ++c) v[c] = g[c] * wt;
                    if (hr >= 0) {
#pragma unroll
                        for (int c = 0; c < EPL; ++c) atomicAdd(&hot[(int64_t)hr * p.D + d + c], v[c]);
                    } else {
                        atomic_add_row<XG, EPL>(p.grad_x, (int64_t)rows[e] * p.D + d, v);
                    }
                }
            }
        }
        __builtin_amdgcn_wave_barrier();
    }

    if (any_hot) {                                                   // workgroup-uniform
        __syncthreads();
        const int n_rows = flags[1];
        for (int r = wave; r < n_rows; r += nw) {
            for (int64_t d = (int64_t)lane * EPL; d < p.D; d += kWave * EPL) {
                float v[EPL];
#pragma unroll
                for (int c = 0; c < EPL; ++c) v[c] = hot[(int64_t)r * p.D + d + c];
                atomic_add_row<XG, EPL>(p.grad_x, (int64_t)row_node[r] * p.D + d, v);
            }
        }
    }
}

template <typename GT, typename XG>
__global__ __launch_bounds__(512) void bwd2_kernel(const BwdParams p) {
    constexpr int EPL = Epl<GT, XG>::value;
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

    if (p.root_valid && p.root_valid[b] < 0) return;    // workgroup-uniform, before any barrier
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
        for (int64_t d0 = 0; d0 < p.D; d0 += kWave * EPL) {
            const int64_t d = d0 + lane * EPL;
            if (d < p.D) {
                float gsum[EPL];
                load_grad<GT, EPL>(p.grad_out, b * p.D + d, gsum);
#pragma unroll
                for (int c = 0; c < EPL; ++c) gsum[c] = gsum[c] / fc1;
                if (p.grad_h1) {
                    float gh[EPL];
                    load_grad<GT, EPL>(p.grad_h1, (b * k1 + j) * p.D + d, gh);
#pragma unroll
                    for (int c = 0; c < EPL; ++c) gsum[c] += gh[c];
                }
#pragma unroll
                for (int c = 0; c < EPL; ++c) gsum[c] = gsum[c] / fc;
                for (int e = 0; e < n; ++e) {
                    const float m = (float)mul[q * k2 + e];
                    float v[EPL];
#pragma unroll
                    for (int c = 0; c < EPL; ++c) v[c] = gsum[c] * m;
                    atomic_add_row<XG, EPL>(p.grad_x, (int64_t)leaf[q * k2 + e] * p.D + d, v);
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
// Three-hop backward, first step: the gradient that reaches each hop-1 slot's nested mean.
//   work[b,j,:] = (slot j took part ? grad_out[b,:] / c_b : 0) + grad_h1[b,j,:]
// where slot j took part iff ids1[b,j] >= 0 and some i has ids2[b,j,i] >= 0 and a non-negative
// ids3[b,j,i,:], and c_b counts such slots.
// One wave per root; the two-hop backward then runs over the B*k1 slots as its roots.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void deep_grad_kernel(const float* __restrict__ grad_out,
                                                        const float* __restrict__ grad_h1,
                                                        const int32_t* __restrict__ ids1,
                                                        const int32_t* __restrict__ ids2,
                                                        const int32_t* __restrict__ ids3, float* __restrict__ work,
                                                        int64_t B, int k1, int k2, int k3, int64_t D) {
    const int lane = threadIdx.x & 63;
    const int64_t b = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (b >= B) return;                                              // wave-uniform
    uint64_t part = 0;                                               // bit j: slot j took part
    const int per_slot = k2 * k3;
    for (int j = 0; j < k1; ++j) {
        if (ids1[b * k1 + j] < 0) continue;                          // wave-uniform
        const int32_t* q2 = ids2 + (b * k1 + j) * (int64_t)k2;
        const int32_t* q3 = ids3 + (b * k1 + j) * (int64_t)per_slot;
        bool any = false;
        for (int e = lane; e < per_slot; e += kWave) any = any || (q3[e] >= 0 && q2[e / k3] >= 0);
        if (__ballot(any)) part |= 1ull << j;
    }
    const int c = __popcll(part);
    const float inv = c > 0 ? 1.0f / (float)c : 0.0f;
    for (int64_t d = lane; d < D; d += kWave) {
        const float g = grad_out[b * D + d] * inv;
        for (int j = 0; j < k1; ++j) {
            float v = ((part >> j) & 1ull) ? g : 0.0f;
            if (grad_h1) v += grad_h1[(b * k1 + j) * D + d];
            work[(b * k1 + j) * D + d] = v;
        }
    }
}

hipError_t launch_deep_grad(const float* grad_out, const float* grad_h1, const int32_t* ids1, const int32_t* ids2,
                            const int32_t* ids3, float* work, int64_t B, int k1, int k2, int k3, int64_t D,
                            hipStream_t stream) {
    const int wpb = 4;
    const unsigned grid = (unsigned)((B + wpb - 1) / wpb);
    hipLaunchKernelGGL(deep_grad_kernel, dim3(grid), dim3(wpb * kWave), 0, stream, grad_out, grad_h1, ids1, ids2, ids3,
                       work, B, k1, k2, k3, D);
    return hipGetLastError();
}

template <typename GT, typename XG, bool WEIGHTED>
static hipError_t launch_bwd1(const BwdArgs& a, const BwdParams& p, hipStream_t stream) {
    // Workgroups of 16 waves: the rows the seeds of a workgroup share are merged in LDS, so the
    // more seeds a workgroup sees the fewer atomic row-adds reach a hub row, and 16 waves work
    // through them side by side.  Seeds per wave grow with the batch so that the launch keeps
    // a few hundred workgroups (measured on the KG shape, B = 1024 .. 262144: 14.7 us at
    // B=4096 against 20.4 us with 4-wave workgroups, 84 against 136 us at B=65536).
    const int forced_spw = tune_int("FSA_BWD1_SEEDS_PER_WAVE", 0);
    const int forced_nw = tune_int("FSA_BWD1_WAVES", 0);
    const int nw = (forced_nw >= 1 && forced_nw <= 16) ? forced_nw : 16;
    int spw = 1;
    while (spw < 16 && a.B / ((int64_t)nw * spw * 2) >= 256) spw *= 2;
    if (forced_spw >= 1 && forced_spw <= 64) spw = forced_spw;
    // LDS: the fixed part (hash tables, per-wave strips) plus as many fp32 rows as fit in 64 KB
    const size_t lds_fixed = sizeof(int) * (3 * kHotBuckets + 2 + kHotRowsMax + nw * 3 * kWave);
    int hot_rows = (int)((65536 - lds_fixed) / (sizeof(float) * (size_t)a.D));
    if (hot_rows > kHotRowsMax) hot_rows = kHotRowsMax;
    if (tune_int("FSA_BWD1_NO_HOT", 0)) hot_rows = 0;
    const unsigned grid = (unsigned)((a.B + nw * spw - 1) / (nw * spw));
    const size_t lds = lds_fixed + sizeof(float) * (size_t)hot_rows * a.D;
    hipLaunchKernelGGL((bwd1_kernel<GT, XG, WEIGHTED>), dim3(grid), dim3(nw * kWave), lds, stream, p, spw, hot_rows);
    return hipGetLastError();
}

template <typename GT, typename XG>
static hipError_t launch_backward_typed(const BwdArgs& a, const BwdParams& p, hipStream_t stream) {
    if (!a.ids2) {
        return launch_bwd1<GT, XG, false>(a, p, stream);
    } else {
        const int forced = tune_int("FSA_BWD2_WAVES", 0);
        int nw = (forced >= 1 && forced <= 8) ? forced : (a.k1 < 8 ? a.k1 : 8);
        const int nq_max = (a.k1 + nw - 1) / nw;
        const size_t lds = sizeof(int) * ((size_t)nw * (2 * nq_max * a.k2 + 2 * nq_max) + nw);
        hipLaunchKernelGGL((bwd2_kernel<GT, XG>), dim3((unsigned)a.B), dim3(nw * kWave), lds, stream, p);
    }
    return hipGetLastError();
}

hipError_t launch_backward(const BwdArgs& a, hipStream_t stream) {
    BwdParams p;
    p.grad_out = a.grad_out; p.grad_h1 = a.grad_h1; p.ids1 = a.ids1; p.ids2 = a.ids2;
    p.grad_x = a.grad_x; p.B = a.B; p.D = a.D; p.k1 = a.k1; p.k2 = a.k2; p.root_valid = a.root_valid; p.w1 = nullptr;
    // kinds: 0 fp32, 1 bfloat16, 2 fp16.  A 16-bit grad_x takes gradients of its own type or fp32.
    switch (a.grad_kind * 3 + a.grad_x_kind) {
        case 0 * 3 + 0: return launch_backward_typed<g_f32, g_f32>(a, p, stream);
        case 1 * 3 + 0: return launch_backward_typed<g_bf16, g_f32>(a, p, stream);
        case 2 * 3 + 0: return launch_backward_typed<g_f16, g_f32>(a, p, stream);
        case 0 * 3 + 1: return launch_backward_typed<g_f32, g_bf16>(a, p, stream);
        case 1 * 3 + 1: return launch_backward_typed<g_bf16, g_bf16>(a, p, stream);
        case 0 * 3 + 2: return launch_backward_typed<g_f32, g_f16>(a, p, stream);
        case 2 * 3 + 2: return launch_backward_typed<g_f16, g_f16>(a, p, stream);
        default: return hipErrorInvalidValue;
    }
}

// 1-hop weighted-mean backward (fp32): the 1-hop kernel with weight shares.
hipError_t launch_backward1_weighted(const BwdArgs& a, const float* w1, hipStream_t stream) {
    BwdParams p;
    p.grad_out = a.grad_out; p.grad_h1 = nullptr; p.ids1 = a.ids1; p.ids2 = nullptr;
    p.grad_x = a.grad_x; p.B = a.B; p.D = a.D; p.k1 = a.k1; p.k2 = 0; p.root_valid = nullptr; p.w1 = w1;
    return launch_bwd1<g_f32, g_f32, true>(a, p, stream);
}

}  // namespace fsa
