// Host-side launch interface between the C ABI (fsa_api.hip) and the kernel files.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#ifdef FSA_TUNING
#include <cstdlib>
#endif

namespace fsa {

// Launch-shape overrides for sweeps.  Only a library built with -DFSA_TUNING (a separately
// named build that is never shipped) reads the environment; the product returns the default.
#ifdef FSA_TUNING
inline int tune_int(const char* name, int fallback) {
    const char* v = std::getenv(name);
    return v ? std::atoi(v) : fallback;
}
#else
constexpr int tune_int(const char*, int fallback) { return fallback; }
#endif

#ifdef FSA_TRACE
// Debug builds only (-DFSA_TRACE): per-root time stamps of the 2-hop forward go to this
// device buffer, set through fsa_debug_set_trace().
extern long long* g_trace;
#endif

// How a feature row is cut into per-lane chunks and how lanes are grouped over rows.
struct RowGeom {
    int vec_bytes;     // 16, 8, 4 or 2: bytes one lane loads per instruction
    int chunks;        // chunks per row = D * elem_bytes / vec_bytes
    int sub;           // lanes that cover one row together: min(64, pow2 >= chunks)
    int tiles;         // passes of `sub` lanes needed to cover a row
};

struct FwdArgs {
    const void* indptr; int indptr_is64; const int32_t* indices;
    const void* x; int x_kind; int64_t D;      // x_kind: 0 fp32, 1 bfloat16, 2 fp16
    const int32_t* seeds; int64_t B; int k1; int k2; int hops; uint64_t seed;
    const int32_t* ids1; const int32_t* ids2;   // replay inputs (indptr == nullptr selects replay)
    void* out; void* out_h1; int32_t* out_ids1; int32_t* out_ids2;
    RowGeom geom;
    // chained (deeper-hop) calls
    uint32_t hop_base = 0;                      // hop counter of the seeds' own rows; negative seeds = empty rows
    int32_t* out_live = nullptr;                // 2-hop: [B] number of hop-1 slots that took part
    const int32_t* slot_cnt = nullptr;          // non-null selects the slot-mean kernel: out[b] = mean of the
                                                // rows x[b*k1+j] with slot_cnt[b,j] > 0
};

struct BwdArgs {
    const void* grad_out; const void* grad_h1; const int32_t* ids1; const int32_t* ids2;
    int64_t B; int k1; int k2; int64_t D; void* grad_x;
    int grad_kind = 0;      // element type of grad_out / grad_h1: 0 fp32, 1 bfloat16, 2 fp16
    int grad_x_kind = 0;    // element type of grad_x
    const int32_t* root_valid = nullptr;   // 2-hop, chained calls: [B], a negative entry switches root b off
};

// Weighted mean: the same launches with per-edge weights (edge_w aligned with indices) and
// the sampled weights emitted / taken back next to the IDs.
struct WeightArgs {
    const float* edge_w;                        // sampling forward
    const float* w1; const float* w2;           // replay / backward inputs
    float* out_w1; float* out_w2;               // sampling forward outputs (nullable)
};

hipError_t launch_forward(const FwdArgs& a, hipStream_t stream);
hipError_t launch_forward_weighted(const FwdArgs& a, const WeightArgs& w, hipStream_t stream);
hipError_t launch_backward_weighted(const BwdArgs& a, const WeightArgs& w, hipStream_t stream);
hipError_t launch_backward(const BwdArgs& a, hipStream_t stream);
// 2-hop backward that owns each destination row (sorted, no atomics on full rows): needs a caller
// workspace; `*used` tells whether it ran (false: not eligible, nothing was launched).
size_t sorted_workspace_bytes(int64_t B, int k1, int k2, int64_t D);
hipError_t launch_backward_sorted(const BwdArgs& a, void* workspace, size_t workspace_bytes, hipStream_t stream,
                                  bool* used);
hipError_t launch_backward1_weighted(const BwdArgs& a, const float* w1, hipStream_t stream);   // 1-hop, fp32
// work[b,j,:] = (slot j took part ? grad_out[b,:] / #such slots : 0) + grad_h1[b,j,:]  (grad_h1 nullable)
hipError_t launch_deep_grad(const float* grad_out, const float* grad_h1, const int32_t* ids1, const int32_t* ids2,
                            const int32_t* ids3, float* work, int64_t B, int k1, int k2, int k3, int64_t D,
                            hipStream_t stream);

}  // namespace fsa
