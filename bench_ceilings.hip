// Measurement aid, not part of the product API: what this GPU sustains on the plain access
// patterns the kernels are made of, so that their achieved rates can be read against a
// measured ceiling next to the nominal 8 TB/s.  Built as a library of its own
// (libbench_ceilings.so) and called only by the benchmark (bench.py --ceilings).
//   0  streaming read of the whole table, 16-byte loads
//   1  device copy of 4 GB (bytes read + bytes written)
//   2  gather of 256-byte rows at random places of the table, 16 lanes x 16 B per row,
//      8 row loads in flight per lane (the shape of the forward's row gather on a bf16 D=128 table)
//   3  the same with 512-byte rows (fp32 D=128)
//   4  fp32 atomic adds of 512-byte rows at random places, one lane per float (the backward)
//   5  packed bf16 atomic adds of 256-byte rows at random places, one lane per element pair
//   6  plain stores of 512-byte rows at random places
// The library allocates its own device memory (table_gb GiB + 4 GiB + the index arrays) and
// frees it before returning.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <vector>

namespace {

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

__global__ void read_kernel(const uint4* __restrict__ p, size_t n, uint32_t* sink) {
    size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
    const size_t st = (size_t)gridDim.x * blockDim.x;
    uint32_t a = 0;
    for (; i + 3 * st < n; i += 4 * st) {
        const uint4 v0 = p[i], v1 = p[i + st], v2 = p[i + 2 * st], v3 = p[i + 3 * st];
        a ^= v0.x ^ v0.y ^ v0.z ^ v0.w ^ v1.x ^ v1.y ^ v1.z ^ v1.w ^ v2.x ^ v2.y ^ v2.z ^ v2.w ^ v3.x ^ v3.y ^ v3.z ^ v3.w;
    }
    for (; i < n; i += st) { const uint4 v = p[i]; a ^= v.x ^ v.y ^ v.z ^ v.w; }
    if (a == 0x12345678u) sink[0] = a;                   // keeps the loads alive
}

__global__ void copy_kernel(const uint4* __restrict__ p, uint4* __restrict__ q, size_t n) {
    size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
    const size_t st = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += st) q[i] = p[i];
}

// rows of row16 * 16 bytes; row16 lanes per row; groups of lanes take 8 consecutive list entries
__global__ void gather_kernel(const uint4* __restrict__ x, const int* __restrict__ ids, size_t n_ids, int row16,
                              uint32_t* sink) {
    constexpr int U = 8;
    const size_t t = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
    const size_t n_thr = (size_t)gridDim.x * blockDim.x;
    const size_t grp = t / row16, n_grp = n_thr / row16;
    const int l = (int)(t % row16);
    uint32_t a = 0;
    for (size_t r = grp * U; r + U <= n_ids; r += n_grp * U) {
        uint4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = x[(size_t)ids[r + u] * row16 + l];
#pragma unroll
        for (int u = 0; u < U; ++u) a ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    if (a == 0x12345678u) sink[0] = a;
}

// one wave per list entry: lane l takes floats l, l+64, ... of a row of D floats
__global__ void atomic_rows_kernel(float* g, const int* __restrict__ ids, size_t n_ids, int D, float v) {
    const size_t wave = (blockIdx.x * (size_t)blockDim.x + threadIdx.x) >> 6, n_waves = ((size_t)gridDim.x * blockDim.x) >> 6;
    const int lane = threadIdx.x & 63;
    for (size_t r = wave; r < n_ids; r += n_waves) {
        float* row = g + (size_t)ids[r] * D;
        for (int d = lane; d < D; d += 64) unsafeAtomicAdd(row + d, v);
    }
}

__global__ void store_rows_kernel(float* g, const int* __restrict__ ids, size_t n_ids, int D, float v) {
    const size_t wave = (blockIdx.x * (size_t)blockDim.x + threadIdx.x) >> 6, n_waves = ((size_t)gridDim.x * blockDim.x) >> 6;
    const int lane = threadIdx.x & 63;
    for (size_t r = wave; r < n_ids; r += n_waves) {
        float* row = g + (size_t)ids[r] * D;
        for (int d = lane; d < D; d += 64) row[d] = v;
    }
}

// rows of D bf16 elements (D even): lane l adds the pairs l, l+64, ...
__global__ void atomic_bf16_rows_kernel(uint16_t* g, const int* __restrict__ ids, size_t n_ids, int D, float v) {
    const size_t wave = (blockIdx.x * (size_t)blockDim.x + threadIdx.x) >> 6, n_waves = ((size_t)gridDim.x * blockDim.x) >> 6;
    const int lane = threadIdx.x & 63;
    bf16x2_t pair;
    pair[0] = (__bf16)v;
    pair[1] = (__bf16)v;
    for (size_t r = wave; r < n_ids; r += n_waves) {
        uint16_t* row = g + (size_t)ids[r] * D;
        for (int d = 2 * lane; d < D; d += 128)
            __builtin_amdgcn_global_atomic_fadd_v2bf16(reinterpret_cast<bf16x2_t*>(row + d), pair);
    }
}

struct Timer {
    hipEvent_t e0, e1;
    Timer() { (void)hipEventCreate(&e0); (void)hipEventCreate(&e1); }
    ~Timer() { (void)hipEventDestroy(e0); (void)hipEventDestroy(e1); }
    template <typename F> double seconds_per_launch(F launch, int reps) {
        launch();
        if (hipDeviceSynchronize() != hipSuccess) return -1.0;
        (void)hipEventRecord(e0);
        for (int i = 0; i < reps; ++i) launch();
        (void)hipEventRecord(e1);
        if (hipEventSynchronize(e1) != hipSuccess) return -1.0;
        float ms = 0.0f;
        (void)hipEventElapsedTime(&ms, e0, e1);
        return ms * 1e-3 / reps;
    }
};

// xorshift64: indices into [0, span)
void fill_ids(std::vector<int>& h, size_t span, uint64_t& s) {
    for (size_t i = 0; i < h.size(); ++i) { s ^= s << 13; s ^= s >> 7; s ^= s << 17; h[i] = (int)(s % span); }
}

}  // namespace

extern "C" {

// Fills out[0..6] with GB/s (see the list at the top); table_gb = size of the table the reads
// and gathers range over (8 .. 64).  Returns 0, or a HIP error code.
int fsa_ceilings_measure(int table_gb, double* out) {
    if (table_gb < 8 || table_gb > 64 || !out) return -1;     // the copy reads the first 4 GiB, the scatters the first 8
    const size_t bytes = (size_t)table_gb << 30, copy_bytes = (size_t)4 << 30;
    uint4 *p = nullptr, *q = nullptr;
    uint32_t* sink = nullptr;
    int* ids = nullptr;
    hipError_t e;
    if ((e = hipMalloc(&p, bytes)) != hipSuccess) return (int)e;
    if ((e = hipMalloc(&q, copy_bytes)) != hipSuccess) { (void)hipFree(p); return (int)e; }
    if ((e = hipMalloc(&sink, 4)) != hipSuccess) { (void)hipFree(p); (void)hipFree(q); return (int)e; }
    const size_t n_ids = (size_t)1 << 24;
    if ((e = hipMalloc(&ids, n_ids * 4)) != hipSuccess) { (void)hipFree(p); (void)hipFree(q); (void)hipFree(sink); return (int)e; }
    (void)hipMemset(p, 1, bytes);
    (void)hipMemset(q, 0, copy_bytes);
    Timer t;
    std::vector<int> h(n_ids);
    uint64_t s = 88172645463325252ull;

    double best = 0.0;
    for (int blocks : {2048, 4096, 8192, 16384}) {
        const double sec = t.seconds_per_launch([&] { hipLaunchKernelGGL(read_kernel, dim3(blocks), dim3(256), 0, 0, p, bytes / 16, sink); }, 5);
        if (sec > 0 && bytes / sec / 1e9 > best) best = bytes / sec / 1e9;
    }
    out[0] = best;
    best = 0.0;
    for (int blocks : {2048, 8192, 32768}) {
        const double sec = t.seconds_per_launch([&] { hipLaunchKernelGGL(copy_kernel, dim3(blocks), dim3(256), 0, 0, p, q, copy_bytes / 16); }, 5);
        if (sec > 0 && 2.0 * copy_bytes / sec / 1e9 > best) best = 2.0 * copy_bytes / sec / 1e9;
    }
    out[1] = best;
    for (int k = 0; k < 2; ++k) {
        const int row_bytes = k == 0 ? 256 : 512;
        fill_ids(h, bytes / row_bytes, s);
        (void)hipMemcpy(ids, h.data(), n_ids * 4, hipMemcpyHostToDevice);
        best = 0.0;
        for (int blocks : {4096, 16384}) {
            const double sec = t.seconds_per_launch([&] { hipLaunchKernelGGL(gather_kernel, dim3(blocks), dim3(256), 0, 0, p, ids, n_ids, row_bytes / 16, sink); }, 3);
            if (sec > 0 && (double)n_ids * row_bytes / sec / 1e9 > best) best = (double)n_ids * row_bytes / sec / 1e9;
        }
        out[2 + k] = best;
    }
    // scatter patterns: 2^22 rows of 128 elements at random places of the first 8 GiB (or the whole table)
    const size_t n_rows = (size_t)1 << 22;
    const size_t span_bytes = bytes < ((size_t)8 << 30) ? bytes : ((size_t)8 << 30);
    (void)hipMemset(p, 0, span_bytes);
    h.resize(n_rows);
    fill_ids(h, span_bytes / 512, s);
    (void)hipMemcpy(ids, h.data(), n_rows * 4, hipMemcpyHostToDevice);
    double sec = t.seconds_per_launch([&] { hipLaunchKernelGGL(atomic_rows_kernel, dim3(8192), dim3(256), 0, 0, reinterpret_cast<float*>(p), ids, n_rows, 128, 1.0f); }, 3);
    out[4] = sec > 0 ? (double)n_rows * 512 / sec / 1e9 : 0.0;
    sec = t.seconds_per_launch([&] { hipLaunchKernelGGL(store_rows_kernel, dim3(8192), dim3(256), 0, 0, reinterpret_cast<float*>(p), ids, n_rows, 128, 1.0f); }, 3);
    out[6] = sec > 0 ? (double)n_rows * 512 / sec / 1e9 : 0.0;
    (void)hipMemset(p, 0, span_bytes);
    fill_ids(h, span_bytes / 256, s);
    (void)hipMemcpy(ids, h.data(), n_rows * 4, hipMemcpyHostToDevice);
    sec = t.seconds_per_launch([&] { hipLaunchKernelGGL(atomic_bf16_rows_kernel, dim3(8192), dim3(256), 0, 0, reinterpret_cast<uint16_t*>(p), ids, n_rows, 128, 0.5f); }, 3);
    out[5] = sec > 0 ? (double)n_rows * 256 / sec / 1e9 : 0.0;

    e = hipDeviceSynchronize();
    (void)hipFree(ids); (void)hipFree(sink); (void)hipFree(q); (void)hipFree(p);
    return (int)e;
}

}  // extern "C"
