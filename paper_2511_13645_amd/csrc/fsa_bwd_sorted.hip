// 2-hop backward without atomics on the feature rows, for wide rows (or large batches of rows
// of 256 bytes and more) and a caller workspace (fsa_mean_bwd_ws).  The paper describes no backward kernel (Sec. 3.3 "Reproducibility" only
// asks that the saved IDs are replayed); this is the second design of this library.
//
// Why: a hardware fp32 atomic is one 4-byte operation per L2 channel and clock, so the atomic
// backward tops out at about 1.2 TB/s of payload wherever the rows live, and every sampled leaf
// costs a whole row of them.  Owning each destination row exclusively turns the update into a
// plain read-modify-write (about twice that rate) and lets the contributions of a row that was
// sampled several times in the batch be summed in registers first.
//
// Three launches on the caller's stream, all state in the caller's workspace:
//   clear   zero the bucket cursors and the overflow counter (a fill kernel: a memset node must
//           not end up in a captured graph);
//   bin     one workgroup per root: count the rows of every hop-1 slot and the slots that take
//           part, store the slot's two coefficients (1/(c1*c2) for grad_out, 1/c2 for grad_h1),
//           and append every leaf entry (row, slot) to the bucket its row hashes to; a bucket
//           that is full sends the entry to the overflow list;
//   reduce  one workgroup per bucket: sort its entries by (row, slot) in LDS, then wave by wave
//           take a distinct row, sum the gradients of its entries in sorted order and add the sum
//           to grad_x with ordinary loads and stores -- no other workgroup touches that row.
//           A bucket that overflowed adds its sums with atomics instead, because the waves of
//           the whole grid then share out the overflow entries (rows sampled thousands of times
//           in one batch: hubs) and add them to the same rows with the atomic row-add of the
//           other backward.
// Without overflow the result is bit-reproducible (fixed summation order).
#include "fsa_device.hip.h"
#include "fsa_internal.h"

namespace fsa {

constexpr int kBucketCap = 256;           // entries a bucket holds (2 KB of keys in LDS)
constexpr int kBucketFill = 32;           // expected entries per bucket when every slot is full: small buckets
                                          // mean many workgroups (balance: 16 / 32 / 64 / 128 per bucket measured
                                          // 232 / 230 / 237 / 251 us on the social shape) and short sorts
constexpr int kBucketFillNarrow = 64;     // rows under kSortedWideRowBytes: several rows per wave want more rows
                                          // per workgroup (D=128, 614 k leaves: 102 us against 108 with 32)
constexpr int64_t kSortedWideRowBytes = 1024;
constexpr int kSortedThreads = 256;       // threads of a reduce workgroup
constexpr int kCursorStride = 32;         // ints between two bucket cursors: one 128-byte line each, so that the
                                          // binning's atomics spread over all L2 channels
constexpr int kSortedMaxTiles = 8;        // row tiles of 64 lanes held in registers
static_assert(kBucketCap <= kSortedThreads, "the counting sort gives every entry a thread");

struct SortedWs {                          // carved out of the caller's workspace
    int* cursor;                           // [P * kCursorStride] entries appended to each bucket (may exceed the capacity)
    int* overflow_count;                   // [1]
    float2* coef;                          // [B*k1] per hop-1 slot: weight of grad_out[b], weight of grad_h1[b,j]
    unsigned long long* pairs;             // [P][kBucketCap] row << 32 | slot
    unsigned long long* overflow;          // [B*k1*k2]
    int log_p;                             // P = 1 << log_p buckets
};

struct SortedParams {
    const float* grad_out; const float* grad_h1; const int32_t* ids1; const int32_t* ids2;
    float* grad_x; int64_t B; int64_t D; int k1, k2;
    SortedWs ws;
    int chunks;                            // row chunks of VB bytes
};

static int sorted_log_p(int64_t B, int k1, int k2, int64_t D) {
    const int64_t entries = B * k1 * k2;
    const int fill = D * 4 < kSortedWideRowBytes ? kBucketFillNarrow : kBucketFill;
    int lp = 6;
    while (lp < 18 && ((int64_t)fill << lp) < entries) ++lp;
    return lp;
}

static void sorted_layout(int64_t B, int k1, int k2, int64_t D, size_t off[5], size_t& total, int& log_p) {
    log_p = sorted_log_p(B, k1, k2, D);
    const size_t P = (size_t)1 << log_p;
    auto up = [](size_t v) { return (v + 255) & ~(size_t)255; };
    size_t o = 0;
    off[0] = o; o += up(P * kCursorStride * sizeof(int));                  // cursor
    off[1] = o; o += up(sizeof(int));                                      // overflow_count
    off[2] = o; o += up((size_t)B * k1 * sizeof(float2));                  // coef
    off[3] = o; o += up(P * kBucketCap * sizeof(unsigned long long));      // pairs
    off[4] = o; o += up((size_t)B * k1 * k2 * sizeof(unsigned long long)); // overflow
    total = o;
}

__device__ __forceinline__ int bucket_of(int row, int log_p) {
    return (int)(((uint32_t)row * 2654435761u) >> (32 - log_p));
}

__global__ __launch_bounds__(256) void sorted_clear_kernel(int* cursor, int n_buckets, int* overflow_count) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_buckets) cursor[(size_t)i * kCursorStride] = 0;
    if (i == 0) *overflow_count = 0;
}

// One workgroup per root: slot counts, coefficients, entries into buckets.
__global__ __launch_bounds__(256) void sorted_bin_kernel(const SortedParams p) {
    __shared__ int u[64];
    __shared__ int cnt[64];
    __shared__ int c1_shared;
    const int64_t b = blockIdx.x;
    const int k1 = p.k1, k2 = p.k2;
    const int tid = threadIdx.x;
    if (tid < 64) {
        u[tid] = tid < k1 ? p.ids1[b * k1 + tid] : -1;
        cnt[tid] = 0;
    }
    __syncthreads();
    const int n_ent = k1 * k2;
    for (int e = tid; e < n_ent; e += blockDim.x) {
        const int j = e / k2;
        if (u[j] >= 0 && p.ids2[b * n_ent + e] >= 0) atomicAdd(&cnt[j], 1);
    }
    __syncthreads();
    if (tid < 64) {                                                   // wave 0
        const uint64_t live = __ballot(tid < k1 && cnt[tid] > 0);
        if (tid == 0) c1_shared = __popcll(live);
    }
    __syncthreads();
    const int c1 = c1_shared;
    if (tid < k1) {
        const int c2 = cnt[tid];
        float2 cf = make_float2(0.0f, 0.0f);
        if (c2 > 0) cf = make_float2(1.0f / ((float)c1 * (float)c2), 1.0f / (float)c2);
        p.ws.coef[b * k1 + tid] = cf;
    }
    for (int e = tid; e < n_ent; e += blockDim.x) {
        const int j = e / k2;
        const int id = u[j] >= 0 ? p.ids2[b * n_ent + e] : -1;
        if (id < 0) continue;
        const unsigned long long key = ((unsigned long long)(uint32_t)id << 32) | (uint32_t)(b * k1 + j);
        const int bucket = bucket_of(id, p.ws.log_p);
        const int pos = atomicAdd(&p.ws.cursor[(size_t)bucket * kCursorStride], 1);
        if (pos < kBucketCap) {
            p.ws.pairs[(size_t)bucket * kBucketCap + pos] = key;
        } else {
            const int o = atomicAdd(p.ws.overflow_count, 1);          // < B*k1*k2: every entry lands at most once
            p.ws.overflow[o] = key;
        }
    }
}

template <int VB> struct FloatChunk;
template <> struct FloatChunk<16> { using T = float4; static constexpr int VE = 4; };
template <> struct FloatChunk<8>  { using T = float2; static constexpr int VE = 2; };
template <> struct FloatChunk<4>  { using T = float;  static constexpr int VE = 1; };

template <int VE, typename T> __device__ __forceinline__ void fma_chunk(float (&acc)[VE], const T& v, float w) {
    if constexpr (VE == 4) { acc[0] = fmaf(w, v.x, acc[0]); acc[1] = fmaf(w, v.y, acc[1]); acc[2] = fmaf(w, v.z, acc[2]); acc[3] = fmaf(w, v.w, acc[3]); }
    else if constexpr (VE == 2) { acc[0] = fmaf(w, v.x, acc[0]); acc[1] = fmaf(w, v.y, acc[1]); }
    else { acc[0] = fmaf(w, v, acc[0]); }
}
template <int VE, typename T> __device__ __forceinline__ T add_chunk(const T& v, const float (&acc)[VE]) {
    T r = v;
    if constexpr (VE == 4) { r.x += acc[0]; r.y += acc[1]; r.z += acc[2]; r.w += acc[3]; }
    else if constexpr (VE == 2) { r.x += acc[0]; r.y += acc[1]; }
    else { r += acc[0]; }
    return r;
}

// Loads bucket `bucket`'s entries into `keys`, sorts them ascending -- (row, slot) order fixes the
// order of every later sum -- and lists the first entry of every distinct row in `heads`.
// Returns the number of entries (at most kBucketCap); *overflowed: more were appended than the
// bucket holds, the rest are in the overflow list.  Called by all threads of the workgroup.
__device__ __forceinline__ int sort_bucket(const SortedParams& p, int bucket, unsigned long long* keys, int* heads,
                                           int* n_heads, bool* overflowed) {
    const int tid = threadIdx.x;
    int n = p.ws.cursor[(size_t)bucket * kCursorStride];
    *overflowed = n > kBucketCap;
    if (n > kBucketCap) n = kBucketCap;
    if (tid == 0) *n_heads = 0;
    if (n == 0) return 0;                                             // workgroup-uniform
    const unsigned long long* src = p.ws.pairs + (size_t)bucket * kBucketCap;
    if (tid < n) keys[tid] = src[tid];
    __syncthreads();
    {
        // every entry counts the entries that go before it: one pass of LDS broadcast reads and a
        // single barrier (a bucket holds at most one entry per thread)
        unsigned long long mine = ~0ull;
        int rank = 0;
        if (tid < n) {
            mine = keys[tid];
            for (int j = 0; j < n; ++j) {
                const unsigned long long other = keys[j];
                rank += (other < mine) || (other == mine && j < tid);
            }
        }
        __syncthreads();
        if (tid < n) keys[rank] = mine;
        __syncthreads();
    }
    for (int i = tid; i < n; i += blockDim.x) {
        if (i == 0 || (uint32_t)(keys[i] >> 32) != (uint32_t)(keys[i - 1] >> 32)) heads[atomicAdd(n_heads, 1)] = i;
    }
    __syncthreads();
    return n;
}

// Overflow entries (a bucket holds kBucketCap; rows sampled thousands of times in one batch,
// hubs, fill theirs): shared out over all waves of the grid and added with hardware atomics,
// one element per lane, as the other backward does.  All entries of a row hash to one bucket,
// so only rows of buckets that overflowed receive such adds -- and those buckets' own sums
// went in by atomics too, never by plain stores.
__device__ __forceinline__ void add_overflow_entries(const SortedParams& p, int bucket, int wave, int lane) {
    const int n_over = *p.ws.overflow_count;
    if (n_over <= 0) return;                                          // grid-uniform
    const int total_waves = gridDim.x * (blockDim.x >> 6);
    for (int o = bucket * (int)(blockDim.x >> 6) + wave; o < n_over; o += total_waves) {
        const unsigned long long key = p.ws.overflow[o];
        const uint32_t row = (uint32_t)(key >> 32), s = (uint32_t)key;
        const float2 cf = p.ws.coef[s];
        const float* go = p.grad_out + (int64_t)(s / (uint32_t)p.k1) * p.D;
        const float* gh = p.grad_h1 ? p.grad_h1 + (int64_t)s * p.D : nullptr;
        float* dst = p.grad_x + (int64_t)row * p.D;
        for (int64_t d = lane; d < p.D; d += kWave) {
            float v = cf.x * go[d];
            if (gh) v = fmaf(cf.y, gh[d], v);
            unsafeAtomicAdd(dst + d, v);
        }
    }
}

// One workgroup (4 waves) per bucket.  MT: row tiles of 64 lanes x VB bytes kept in registers.
template <int VB, int MT>
__global__ __launch_bounds__(kSortedThreads) void sorted_reduce_kernel(const SortedParams p) {
    using T = typename FloatChunk<VB>::T;
    constexpr int VE = FloatChunk<VB>::VE;
    __shared__ unsigned long long keys[kBucketCap];
    __shared__ int heads[kBucketCap];
    __shared__ int n_heads;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int bucket = blockIdx.x;
    const int k1 = p.k1;
    const int tiles = (p.chunks + kWave - 1) >> 6;
    const int parts = (tiles + MT - 1) / MT;                          // a row is summed in `parts` pieces of MT tiles,
                                                                      // each by whichever wave comes to it
    __shared__ int next_item;
    if (tid == 0) next_item = 0;                                      // sort_bucket's barriers come before its first use
    bool overflowed;                                                  // some of this bucket's entries are in the overflow list
    const int n = sort_bucket(p, bucket, keys, heads, &n_heads, &overflowed);
    if (n > 0) {                                                      // workgroup-uniform
        const int nh = n_heads;
        // a wave takes the next piece of work when it is free (rows differ in how many entries
        // reach them: fixed shares would leave three waves waiting for the one with a hub row)
        for (;;) {
            int item = 0;
            if (lane == 0) item = atomicAdd(&next_item, 1);
            item = __builtin_amdgcn_readfirstlane(item);
            if (item >= nh * parts) break;                            // wave-uniform
            const int h = item / parts;
            const int tile0 = (item - h * parts) * MT;
            const int i0 = heads[h];
            const uint32_t row = (uint32_t)(keys[i0] >> 32);
            float* dst_f = p.grad_x + (int64_t)row * p.D;
            T* dst = reinterpret_cast<T*>(dst_f);
            float acc[MT][VE];
#pragma unroll
            for (int t = 0; t < MT; ++t) {
#pragma unroll
                for (int e = 0; e < VE; ++e) acc[t][e] = 0.0f;
            }
            for (int i = i0; i < n && (uint32_t)(keys[i] >> 32) == row; ++i) {    // wave-uniform
                const uint32_t s = (uint32_t)keys[i];
                const float2 cf = p.ws.coef[s];                   // travels with the row loads below
                const T* go = reinterpret_cast<const T*>(p.grad_out + (int64_t)(s / (uint32_t)k1) * p.D);
                const T* gh = p.grad_h1 ? reinterpret_cast<const T*>(p.grad_h1 + (int64_t)s * p.D) : nullptr;
                T a[MT], c[MT];
#pragma unroll
                for (int t = 0; t < MT; ++t) {
                    const int chunk = (tile0 + t) * kWave + lane;
                    if (chunk < p.chunks) {
                        a[t] = go[chunk];
                        if (gh) c[t] = gh[chunk];
                    }
                }
#pragma unroll
                for (int t = 0; t < MT; ++t) {
                    const int chunk = (tile0 + t) * kWave + lane;
                    if (chunk < p.chunks) {
                        fma_chunk<VE>(acc[t], a[t], cf.x);
                        if (gh) fma_chunk<VE>(acc[t], c[t], cf.y);
                    }
                }
            }
            if (overflowed) {                                         // workgroup-uniform
                // other workgroups add this bucket's overflow entries to the same rows with
                // atomics at the same time: the sums of a full bucket go in by atomics as well
#pragma unroll
                for (int t = 0; t < MT; ++t) {
                    const int chunk = (tile0 + t) * kWave + lane;
                    if (chunk < p.chunks) {
#pragma unroll
                        for (int e = 0; e < VE; ++e) unsafeAtomicAdd(dst_f + (int64_t)chunk * VE + e, acc[t][e]);
                    }
                }
            } else {
                // the row is read right before it is written back: the write finds its DRAM page
                // still open (requesting it before the first entry's gradients measured 15 % slower,
                // together with the last entry's 8 %)
                T old[MT];
#pragma unroll
                for (int t = 0; t < MT; ++t) {
                    const int chunk = (tile0 + t) * kWave + lane;
                    if (chunk < p.chunks) old[t] = dst[chunk];
                }
#pragma unroll
                for (int t = 0; t < MT; ++t) {
                    const int chunk = (tile0 + t) * kWave + lane;
                    if (chunk < p.chunks) dst[chunk] = add_chunk<VE>(old[t], acc[t]);
                }
            }
        }
    }
    add_overflow_entries(p, bucket, wave, lane);
}

// The same for rows of at most 64 chunks (under 1 KB): groups of `1 << sub_shift` lanes take a
// distinct row each, so a workgroup works on 4 .. 64 rows at a time, and a row's old value is
// requested before its gradients are summed: with rows this short the kernel is bound by the
// number of dependent memory round trips per wave, not by bytes.
template <int VB>
__global__ __launch_bounds__(kSortedThreads) void sorted_reduce_narrow_kernel(const SortedParams p, int sub_shift) {
    using T = typename FloatChunk<VB>::T;
    constexpr int VE = FloatChunk<VB>::VE;
    __shared__ unsigned long long keys[kBucketCap];
    __shared__ int heads[kBucketCap];
    __shared__ int n_heads;
    const int tid = threadIdx.x;
    const int bucket = blockIdx.x;
    bool overflowed;
    const int n = sort_bucket(p, bucket, keys, heads, &n_heads, &overflowed);
    if (n > 0) {                                                      // workgroup-uniform
        const int nh = n_heads;
        const int grp = tid >> sub_shift, sl = tid & ((1 << sub_shift) - 1);
        const int n_grp = kSortedThreads >> sub_shift;
        const bool live = sl < p.chunks;
        for (int h = grp; h < nh; h += n_grp) {                       // uniform within a group of lanes
            const int i0 = heads[h];
            const uint32_t row = (uint32_t)(keys[i0] >> 32);
            float* dst_f = p.grad_x + (int64_t)row * p.D;
            T* dst = reinterpret_cast<T*>(dst_f);
            T old{};
            if (live && !overflowed) old = dst[sl];                   // (after the sums: 2 % slower here)
            float acc[VE];
#pragma unroll
            for (int e = 0; e < VE; ++e) acc[e] = 0.0f;
            for (int i = i0; i < n && (uint32_t)(keys[i] >> 32) == row; ++i) {
                const uint32_t s = (uint32_t)keys[i];
                const float2 cf = p.ws.coef[s];
                if (live) {
                    const T a = reinterpret_cast<const T*>(p.grad_out + (int64_t)(s / (uint32_t)p.k1) * p.D)[sl];
                    if (p.grad_h1) {
                        const T c = reinterpret_cast<const T*>(p.grad_h1 + (int64_t)s * p.D)[sl];
                        fma_chunk<VE>(acc, a, cf.x);
                        fma_chunk<VE>(acc, c, cf.y);
                    } else {
                        fma_chunk<VE>(acc, a, cf.x);
                    }
                }
            }
            if (live) {
                if (overflowed) {                                     // see sorted_reduce_kernel
#pragma unroll
                    for (int e = 0; e < VE; ++e) unsafeAtomicAdd(dst_f + (int64_t)sl * VE + e, acc[e]);
                } else {
                    dst[sl] = add_chunk<VE>(old, acc);
                }
            }
        }
    }
    add_overflow_entries(p, bucket, tid >> 6, tid & 63);
}

// ---------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------
// The path pays when rows are wide (the per-row cost of the atomic unit grows with the row, the
// three launches and the binning do not) and the batch moves enough bytes to hide them.  Rows
// under 1 KB gain less -- every leaf re-reads its slot's gradient rows, which the atomic backward
// reads once per slot -- and only in large batches: D=128, 614 k leaves, 121 -> 102 us; D=100,
// 614 k leaves, 237 -> 210 us; but 154 k leaves, 64 -> 75 us.
constexpr int64_t kSortedMinRowBytes = kSortedWideRowBytes;
constexpr int64_t kSortedMinPayload = 32ll << 20;
constexpr int64_t kSortedNarrowMinRowBytes = 256;
constexpr int64_t kSortedNarrowMinEntries = 384 * 1024;

static int sorted_vec_bytes(const BwdArgs& a) {
    auto al = [](const void* q, uintptr_t m) { return q == nullptr || (reinterpret_cast<uintptr_t>(q) % m) == 0; };
    for (int vb = 16; vb > 4; vb >>= 1)
        if ((a.D * 4) % vb == 0 && al(a.grad_out, vb) && al(a.grad_h1, vb) && al(a.grad_x, vb)) return vb;
    return 4;
}

bool sorted_backward_shape_ok(int64_t B, int k1, int k2, int64_t D) {
    if (k2 <= 0 || D * 4 < kSortedNarrowMinRowBytes) return false;
    if (D * 4 < kSortedMinRowBytes) {
        if (B * k1 * k2 < kSortedNarrowMinEntries) return false;
    } else if (B * k1 * k2 * D * 4 < kSortedMinPayload) {
        return false;
    }
    if (B * k1 * k2 > (int64_t)INT32_MAX) return false;
    return D <= (int64_t)kSortedMaxTiles * kWave * 4;                 // fits the register tiles with 16-byte chunks
                                                                      // (the launch checks the real chunk width)
}

size_t sorted_workspace_bytes(int64_t B, int k1, int k2, int64_t D) {
    if (!sorted_backward_shape_ok(B, k1, k2, D)) return 0;
    size_t off[5], total;
    int lp;
    sorted_layout(B, k1, k2, D, off, total, lp);
    return total;
}

// Runs the sorted backward when the call is eligible and the workspace large enough and 256-byte
// aligned; otherwise launches nothing and sets *used = false (the caller falls back to atomics).
hipError_t launch_backward_sorted(const BwdArgs& a, void* workspace, size_t workspace_bytes, hipStream_t stream,
                                  bool* used) {
    *used = false;
    if (!a.ids2 || a.grad_kind != 0 || a.grad_x_kind != 0 || a.root_valid || !workspace) return hipSuccess;
    if (!sorted_backward_shape_ok(a.B, a.k1, a.k2, a.D)) return hipSuccess;
    if (reinterpret_cast<uintptr_t>(workspace) % 256 != 0) return hipSuccess;
    size_t off[5], total;
    int lp;
    sorted_layout(a.B, a.k1, a.k2, a.D, off, total, lp);
    if (workspace_bytes < total) return hipSuccess;
    const int vb = sorted_vec_bytes(a);
    const int chunks = (int)(a.D * 4 / vb);
    const int tiles = (chunks + kWave - 1) / kWave;
    if (tiles > kSortedMaxTiles) return hipSuccess;

    char* w = static_cast<char*>(workspace);
    SortedParams p;
    p.grad_out = static_cast<const float*>(a.grad_out); p.grad_h1 = static_cast<const float*>(a.grad_h1);
    p.ids1 = a.ids1; p.ids2 = a.ids2; p.grad_x = static_cast<float*>(a.grad_x);
    p.B = a.B; p.D = a.D; p.k1 = a.k1; p.k2 = a.k2; p.chunks = chunks;
    p.ws.cursor = reinterpret_cast<int*>(w + off[0]);
    p.ws.overflow_count = reinterpret_cast<int*>(w + off[1]);
    p.ws.coef = reinterpret_cast<float2*>(w + off[2]);
    p.ws.pairs = reinterpret_cast<unsigned long long*>(w + off[3]);
    p.ws.overflow = reinterpret_cast<unsigned long long*>(w + off[4]);
    p.ws.log_p = lp;
    const int P = 1 << lp;
    hipLaunchKernelGGL(sorted_clear_kernel, dim3((P + 255) / 256), dim3(256), 0, stream, p.ws.cursor, P, p.ws.overflow_count);
    hipLaunchKernelGGL(sorted_bin_kernel, dim3((unsigned)a.B), dim3(256), 0, stream, p);
    if (a.D * 4 < kSortedMinRowBytes && chunks <= kWave) {
        int sub_shift = 2;
        while ((1 << sub_shift) < chunks) ++sub_shift;                // 4 .. 64 lanes per row
        if (vb == 16)     hipLaunchKernelGGL((sorted_reduce_narrow_kernel<16>), dim3(P), dim3(kSortedThreads), 0, stream, p, sub_shift);
        else if (vb == 8) hipLaunchKernelGGL((sorted_reduce_narrow_kernel<8>), dim3(P), dim3(kSortedThreads), 0, stream, p, sub_shift);
        else              hipLaunchKernelGGL((sorted_reduce_narrow_kernel<4>), dim3(P), dim3(kSortedThreads), 0, stream, p, sub_shift);
        *used = true;
        return hipGetLastError();
    }
    // tiles of a row summed by one wave at a time: few, so that the kernel's registers allow 8 waves
    // per SIMD -- it is bound by dependent round trips per wave, which only more waves hide
    const int mt_t = tune_int("FSA_SORTED_MT", kSortedMaxTiles);
    const int mt = tiles < mt_t ? tiles : mt_t;
#define FSA_LAUNCH_SORTED(VB_)                                                                              \
    do {                                                                                                    \
        if (mt <= 1)      hipLaunchKernelGGL((sorted_reduce_kernel<VB_, 1>), dim3(P), dim3(kSortedThreads), 0, stream, p); \
        else if (mt <= 2) hipLaunchKernelGGL((sorted_reduce_kernel<VB_, 2>), dim3(P), dim3(kSortedThreads), 0, stream, p); \
        else if (mt <= 4) hipLaunchKernelGGL((sorted_reduce_kernel<VB_, 4>), dim3(P), dim3(kSortedThreads), 0, stream, p); \
        else if (mt <= 6) hipLaunchKernelGGL((sorted_reduce_kernel<VB_, 6>), dim3(P), dim3(kSortedThreads), 0, stream, p); \
        else              hipLaunchKernelGGL((sorted_reduce_kernel<VB_, 8>), dim3(P), dim3(kSortedThreads), 0, stream, p); \
    } while (0)
    if (vb == 16) FSA_LAUNCH_SORTED(16);
    else if (vb == 8) FSA_LAUNCH_SORTED(8);
    else FSA_LAUNCH_SORTED(4);
#undef FSA_LAUNCH_SORTED
    *used = true;
    return hipGetLastError();
}

}  // namespace fsa
