// The C ABI declared in include/fsa.h: host-side validation, row geometry, dispatch.
// Nothing here allocates or synchronises; the only thing kept between calls is the device address
// of the fixed scratch array of fsa_mean3_bwd_noalloc.
#include "../../include/fsa.h"
#include "fsa_internal.h"

#include <atomic>

#ifdef FSA_TRACE
namespace fsa { long long* g_trace = nullptr; }
#endif

// Scratch of fsa_mean3_bwd_noalloc: one copy per GPU, at an address of its own on each.  In host
// code the array's name is only a handle for hipGetSymbolAddress; kernels get the looked-up pointer.
static __device__ __align__(256) float scratch[FSA_SCRATCH_FLOATS];

static constexpr int kMaxDevices = 64;
static std::atomic<float*> scratch_on_device[kMaxDevices];

// Device address of `scratch` on the current device, looked up once per device.
static float* scratch_pointer() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    float* p = scratch_on_device[dev].load(std::memory_order_acquire);
    if (!p) {
        void* sym = nullptr;
        if (hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)) != hipSuccess || !sym) {
            (void)hipGetLastError();
            return nullptr;
        }
        p = static_cast<float*>(sym);
        scratch_on_device[dev].store(p, std::memory_order_release);
    }
    return p;
}


namespace {

bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// Largest load width (bytes) that divides the row size and every pointer that is indexed by
// whole rows, then the sub-group shape that covers a row.
fsa::RowGeom row_geometry(int64_t D, int elem_bytes, const void* const* row_ptrs, int n_ptrs) {
    const int64_t row_bytes = D * elem_bytes;
    int vb = 16;
    for (; vb > elem_bytes; vb >>= 1) {
        bool ok = (row_bytes % vb) == 0;
        for (int i = 0; ok && i < n_ptrs; ++i)
            if (row_ptrs[i]) ok = aligned(row_ptrs[i], (uintptr_t)vb);
        if (ok) break;
    }
    fsa::RowGeom g;
    g.vec_bytes = vb;
    g.chunks = (int)(row_bytes / vb);
    int sub = 1;
    while (sub < g.chunks && sub < 64) sub <<= 1;
    g.sub = sub;
    g.tiles = (g.chunks + sub - 1) / sub;
    return g;
}

int check_common(int x_dtype, int64_t D, int64_t num_nodes, int64_t B) {
    if (x_dtype != FSA_F32 && x_dtype != FSA_BF16 && x_dtype != FSA_F16) return FSA_ERR_DTYPE;
    if (D <= 0 || D > (int64_t)1 << 24 || num_nodes <= 0 || num_nodes > (int64_t)INT32_MAX) return FSA_ERR_ARG;
    if (B < 0 || B > (int64_t)INT32_MAX) return FSA_ERR_ARG;
    return FSA_OK;
}

int elem_bytes(int dtype) { return dtype == FSA_F32 ? 4 : 2; }

// An error that an earlier HIP call of the caller left pending must not be reported as ours.
void drop_stale_hip_error() { (void)hipGetLastError(); }

// hipErrorInvalidValue comes from the launch code's own checks (fanouts that need more LDS than
// the device has); anything else is the runtime refusing a launch.
int status_of(hipError_t e) { return e == hipSuccess ? FSA_OK : e == hipErrorInvalidValue ? FSA_ERR_ARG : FSA_ERR_HIP; }

bool fanout_ok(int32_t k) { return k >= 1 && k <= FSA_KMAX; }

}  // namespace

extern "C" {

int fsa_sample_mean_fwd(const void* indptr, int indptr_type, const int32_t* indices,
                        int64_t num_nodes, const void* x, int x_dtype, int64_t D,
                        const int32_t* seeds, int64_t B, const int32_t* fanouts, int num_hops,
                        uint64_t seed, void* out, void* out_h1,
                        int32_t* out_ids1, int32_t* out_ids2, void* stream) {
    if (!indptr || !indices || !x || !fanouts) return FSA_ERR_NULL;
    if (B != 0 && (!seeds || !out)) return FSA_ERR_NULL;   // batch-sized arrays may be NULL when empty
    if (indptr_type != FSA_I32 && indptr_type != FSA_I64) return FSA_ERR_DTYPE;
    if (int rc = check_common(x_dtype, D, num_nodes, B)) return rc;
    if (num_hops != 1 && num_hops != 2) return FSA_ERR_ARG;
    const int32_t k1 = fanouts[0];
    const int32_t k2 = num_hops == 2 ? fanouts[1] : 0;
    if (!fanout_ok(k1) || (num_hops == 2 && !fanout_ok(k2))) return FSA_ERR_ARG;
    if (num_hops == 1 && (out_h1 || out_ids2)) return FSA_ERR_ARG;
    const int eb = elem_bytes(x_dtype);
    if (!aligned(indptr, indptr_type == FSA_I64 ? 8 : 4) || !aligned(indices, 4) || !aligned(seeds, 4) ||
        !aligned(x, eb) || !aligned(out, eb) || !aligned(out_h1, eb) ||
        !aligned(out_ids1, 4) || !aligned(out_ids2, 4))
        return FSA_ERR_ALIGN;
    if (B == 0) return FSA_OK;
    drop_stale_hip_error();

    const void* rows[3] = {x, out, out_h1};
    fsa::FwdArgs a{};
    a.indptr = indptr; a.indptr_is64 = indptr_type == FSA_I64; a.indices = indices;
    a.x = x; a.x_kind = x_dtype; a.D = D;
    a.seeds = seeds; a.B = B; a.k1 = k1; a.k2 = k2; a.hops = num_hops; a.seed = seed;
    a.ids1 = nullptr; a.ids2 = nullptr;
    a.out = out; a.out_h1 = out_h1; a.out_ids1 = out_ids1; a.out_ids2 = out_ids2;
    a.geom = row_geometry(D, eb, rows, 3);
    return status_of(fsa::launch_forward(a, static_cast<hipStream_t>(stream)));
}

int fsa_mean_replay_fwd(const void* x, int x_dtype, int64_t D, int64_t num_nodes,
                        const int32_t* ids1, const int32_t* ids2,
                        int64_t B, int32_t k1, int32_t k2,
                        void* out, void* out_h1, void* stream) {
    if (!x) return FSA_ERR_NULL;
    if (B != 0 && (!ids1 || !out)) return FSA_ERR_NULL;    // batch-sized arrays may be NULL when empty
    if (int rc = check_common(x_dtype, D, num_nodes, B)) return rc;
    if (!fanout_ok(k1) || (ids2 && !fanout_ok(k2))) return FSA_ERR_ARG;
    if (!ids2 && out_h1) return FSA_ERR_ARG;
    const int eb = elem_bytes(x_dtype);
    if (!aligned(x, eb) || !aligned(out, eb) || !aligned(out_h1, eb) || !aligned(ids1, 4) || !aligned(ids2, 4))
        return FSA_ERR_ALIGN;
    if (B == 0) return FSA_OK;
    drop_stale_hip_error();

    const void* rows[3] = {x, out, out_h1};
    fsa::FwdArgs a{};
    a.indptr = nullptr; a.indices = nullptr; a.seeds = nullptr;
    a.x = x; a.x_kind = x_dtype; a.D = D;
    a.B = B; a.k1 = k1; a.k2 = ids2 ? k2 : 0; a.hops = ids2 ? 2 : 1; a.seed = 0;
    a.ids1 = ids1; a.ids2 = ids2;
    a.out = out; a.out_h1 = out_h1; a.out_ids1 = nullptr; a.out_ids2 = nullptr;
    a.geom = row_geometry(D, eb, rows, 3);
    return status_of(fsa::launch_forward(a, static_cast<hipStream_t>(stream)));
}

int fsa_mean_bwd(const float* grad_out, const float* grad_h1,
                 const int32_t* ids1, const int32_t* ids2,
                 int64_t B, int32_t k1, int32_t k2, int64_t D,
                 float* grad_x, int64_t num_nodes, void* stream) {
    if (!grad_x) return FSA_ERR_NULL;
    if (B != 0 && (!grad_out || !ids1)) return FSA_ERR_NULL;   // batch-sized arrays may be NULL when empty
    if (int rc = check_common(FSA_F32, D, num_nodes, B)) return rc;
    if (!fanout_ok(k1) || (ids2 && !fanout_ok(k2))) return FSA_ERR_ARG;
    if (!ids2 && grad_h1) return FSA_ERR_ARG;
    if (!aligned(grad_out, 4) || !aligned(grad_h1, 4) || !aligned(grad_x, 4) || !aligned(ids1, 4) || !aligned(ids2, 4))
        return FSA_ERR_ALIGN;
    if (B == 0) return FSA_OK;
    drop_stale_hip_error();

    fsa::BwdArgs a{};
    a.grad_out = grad_out; a.grad_h1 = grad_h1; a.ids1 = ids1; a.ids2 = ids2;
    a.B = B; a.k1 = k1; a.k2 = ids2 ? k2 : 0; a.D = D; a.grad_x = grad_x;
    return status_of(fsa::launch_backward(a, static_cast<hipStream_t>(stream)));
}

int64_t fsa_mean_bwd_workspace_bytes(int64_t B, int32_t k1, int32_t k2, int64_t D) {
    if (B <= 0 || D <= 0 || !fanout_ok(k1) || !fanout_ok(k2)) return 0;
    return (int64_t)fsa::sorted_workspace_bytes(B, k1, k2, D);
}

int fsa_mean_bwd_ws(const float* grad_out, const float* grad_h1,
                    const int32_t* ids1, const int32_t* ids2,
                    int64_t B, int32_t k1, int32_t k2, int64_t D,
                    float* grad_x, int64_t num_nodes,
                    void* workspace, int64_t workspace_bytes, void* stream) {
    if (!grad_x) return FSA_ERR_NULL;
    if (B != 0 && (!grad_out || !ids1)) return FSA_ERR_NULL;
    if (int rc = check_common(FSA_F32, D, num_nodes, B)) return rc;
    if (!fanout_ok(k1) || (ids2 && !fanout_ok(k2))) return FSA_ERR_ARG;
    if (!ids2 && grad_h1) return FSA_ERR_ARG;
    if (workspace_bytes < 0) return FSA_ERR_ARG;
    if (!aligned(grad_out, 4) || !aligned(grad_h1, 4) || !aligned(grad_x, 4) || !aligned(ids1, 4) || !aligned(ids2, 4))
        return FSA_ERR_ALIGN;
    if (B == 0) return FSA_OK;
    drop_stale_hip_error();

    fsa::BwdArgs a{};
    a.grad_out = grad_out; a.grad_h1 = grad_h1; a.ids1 = ids1; a.ids2 = ids2;
    a.B = B; a.k1 = k1; a.k2 = ids2 ? k2 : 0; a.D = D; a.grad_x = grad_x;
    bool used = false;
    if (hipError_t e = fsa::launch_backward_sorted(a, workspace, (size_t)workspace_bytes, static_cast<hipStream_t>(stream), &used))
        return status_of(e);
    if (used) return FSA_OK;
    return status_of(fsa::launch_backward(a, static_cast<hipStream_t>(stream)));
}

int fsa_mean_bwd_lp(const void* grad_out, const void* grad_h1, int grad_dtype,
                    const int32_t* ids1, const int32_t* ids2,
                    int64_t B, int32_t k1, int32_t k2, int64_t D,
                    void* grad_x, int grad_x_dtype, int64_t num_nodes, void* stream) {
    if (!grad_x) return FSA_ERR_NULL;
    if (B != 0 && (!grad_out || !ids1)) return FSA_ERR_NULL;
    if (int rc = check_common(grad_dtype, D, num_nodes, B)) return rc;
    if (int rc = check_common(grad_x_dtype, D, num_nodes, B)) return rc;
    // a 16-bit grad_x takes gradients of its own type or fp32
    if (grad_x_dtype != FSA_F32 && grad_dtype != FSA_F32 && grad_dtype != grad_x_dtype) return FSA_ERR_DTYPE;
    if (!fanout_ok(k1) || (ids2 && !fanout_ok(k2))) return FSA_ERR_ARG;
    if (!ids2 && grad_h1) return FSA_ERR_ARG;
    const bool pairs = grad_x_dtype != FSA_F32;                // lanes own element pairs
    if (pairs && (D & 1)) return FSA_ERR_ARG;
    const uintptr_t g_align = pairs ? 4 : (uintptr_t)elem_bytes(grad_dtype);
    if (!aligned(grad_out, g_align) || !aligned(grad_h1, g_align) || !aligned(grad_x, 4) || !aligned(ids1, 4) ||
        !aligned(ids2, 4))
        return FSA_ERR_ALIGN;
    if (B == 0) return FSA_OK;
    drop_stale_hip_error();

    fsa::BwdArgs a{};
    a.grad_out = grad_out; a.grad_h1 = grad_h1; a.ids1 = ids1; a.ids2 = ids2;
    a.B = B; a.k1 = k1; a.k2 = ids2 ? k2 : 0; a.D = D; a.grad_x = grad_x;
    a.grad_kind = grad_dtype; a.grad_x_kind = grad_x_dtype;
    return status_of(fsa::launch_backward(a, static_cast<hipStream_t>(stream)));
}

int fsa_sample_wmean_fwd(const void* indptr, int indptr_type, const int32_t* indices,
                         const float* edge_weight, int64_t num_nodes,
                         const void* x, int x_dtype, int64_t D,
                         const int32_t* seeds, int64_t B, const int32_t* fanouts, int num_hops,
                         uint64_t seed, void* out, void* out_h1,
                         int32_t* out_ids1, int32_t* out_ids2, float* out_w1, float* out_w2,
                         void* stream) {
    if (!indptr || !indices || !edge_weight || !x || !fanouts) return FSA_ERR_NULL;
    if (B != 0 && (!seeds || !out)) return FSA_ERR_NULL;
    if (indptr_type != FSA_I32 && indptr_type != FSA_I64) return FSA_ERR_DTYPE;
    if (int rc = check_common(x_dtype, D, num_nodes, B)) return rc;
    if (num_hops != 1 && num_hops != 2) return FSA_ERR_ARG;
    const int32_t k1 = fanouts[0];
    const int32_t k2 = num_hops == 2 ? fanouts[1] : 0;
    if (!fanout_ok(k1) || (num_hops == 2 && !fanout_ok(k2))) return FSA_ERR_ARG;
    if (num_hops == 1 && (out_h1 || out_ids2 || out_w2)) return FSA_ERR_ARG;
    const int eb = elem_bytes(x_dtype);
    if (!aligned(indptr, indptr_type == FSA_I64 ? 8 : 4) || !aligned(indices, 4) || !aligned(edge_weight, 4) ||
        !aligned(seeds, 4) || !aligned(x, eb) || !aligned(out, eb) || !aligned(out_h1, eb) ||
        !aligned(out_ids1, 4) || !aligned(out_ids2, 4) || !aligned(out_w1, 4) || !aligned(out_w2, 4))
        return FSA_ERR_ALIGN;
    if (B == 0) return FSA_OK;
    drop_stale_hip_error();

    const void* rows[3] = {x, out, out_h1};
    fsa::FwdArgs a{};
    a.indptr = indptr; a.indptr_is64 = indptr_type == FSA_I64; a.indices = indices;
    a.x = x; a.x_kind = x_dtype; a.D = D;
    a.seeds = seeds; a.B = B; a.k1 = k1; a.k2 = k2; a.hops = num_hops; a.seed = seed;
    a.out = out; a.out_h1 = out_h1; a.out_ids1 = out_ids1; a.out_ids2 = out_ids2;
    a.geom = row_geometry(D, eb, rows, 3);
    fsa::WeightArgs w{};
    w.edge_w = edge_weight; w.out_w1 = out_w1; w.out_w2 = out_w2;
    return status_of(fsa::launch_forward_weighted(a, w, static_cast<hipStream_t>(stream)));
}

int fsa_wmean_replay_fwd(const void* x, int x_dtype, int64_t D, int64_t num_nodes,
                         const int32_t* ids1, const int32_t* ids2,
                         const float* w1, const float* w2,
                         int64_t B, int32_t k1, int32_t k2,
                         void* out, void* out_h1, void* stream) {
    if (!x) return FSA_ERR_NULL;
    if (B != 0 && (!ids1 || !w1 || !out || (ids2 && !w2))) return FSA_ERR_NULL;
    if (int rc = check_common(x_dtype, D, num_nodes, B)) return rc;
    if (!fanout_ok(k1) || (ids2 && !fanout_ok(k2))) return FSA_ERR_ARG;
    if (!ids2 && out_h1) return FSA_ERR_ARG;
    const int eb = elem_bytes(x_dtype);
    if (!aligned(x, eb) || !aligned(out, eb) || !aligned(out_h1, eb) || !aligned(ids1, 4) || !aligned(ids2, 4) ||
        !aligned(w1, 4) || !aligned(w2, 4))
        return FSA_ERR_ALIGN;
    if (B == 0) return FSA_OK;
    drop_stale_hip_error();

    const void* rows[3] = {x, out, out_h1};
    fsa::FwdArgs a{};
    a.x = x; a.x_kind = x_dtype; a.D = D;
    a.B = B; a.k1 = k1; a.k2 = ids2 ? k2 : 0; a.hops = ids2 ? 2 : 1;
    a.ids1 = ids1; a.ids2 = ids2; a.out = out; a.out_h1 = out_h1;
    a.geom = row_geometry(D, eb, rows, 3);
    fsa::WeightArgs w{};
    w.w1 = w1; w.w2 = w2;
    return status_of(fsa::launch_forward_weighted(a, w, static_cast<hipStream_t>(stream)));
}

int fsa_wmean_bwd(const float* grad_out, const float* grad_h1,
                  const int32_t* ids1, const int32_t* ids2,
                  const float* w1, const float* w2,
                  int64_t B, int32_t k1, int32_t k2, int64_t D,
                  float* grad_x, int64_t num_nodes, void* stream) {
    if (!grad_x) return FSA_ERR_NULL;
    if (B != 0 && (!grad_out || !ids1 || !w1 || (ids2 && !w2))) return FSA_ERR_NULL;
    if (int rc = check_common(FSA_F32, D, num_nodes, B)) return rc;
    if (!fanout_ok(k1) || (ids2 && !fanout_ok(k2))) return FSA_ERR_ARG;
    if (!ids2 && grad_h1) return FSA_ERR_ARG;
    if (!aligned(grad_out, 4) || !aligned(grad_h1, 4) || !aligned(grad_x, 4) || !aligned(ids1, 4) || !aligned(ids2, 4) ||
        !aligned(w1, 4) || !aligned(w2, 4))
        return FSA_ERR_ALIGN;
    if (B == 0) return FSA_OK;
    drop_stale_hip_error();

    fsa::BwdArgs a{};
    a.grad_out = grad_out; a.grad_h1 = grad_h1; a.ids1 = ids1; a.ids2 = ids2;
    a.B = B; a.k1 = k1; a.k2 = ids2 ? k2 : 0; a.D = D; a.grad_x = grad_x;
    fsa::WeightArgs w{};
    w.w1 = w1; w.w2 = w2;
    return status_of(fsa::launch_backward_weighted(a, w, static_cast<hipStream_t>(stream)));
}

// ---- layer-wise and three-hop variants: chains of the kernels above on one stream ----------

int fsa_sample_mean_layerwise_fwd(const void* indptr, int indptr_type, const int32_t* indices,
                                  int64_t num_nodes, const void* x, int x_dtype, int64_t D,
                                  const int32_t* seeds, int64_t B, const int32_t* fanouts,
                                  uint64_t seed, void* out, void* out_h1, void* out_m1,
                                  int32_t* out_ids1, int32_t* out_ids2, void* stream) {
    if (B != 0 && !out_m1) return FSA_ERR_NULL;
    if (x_dtype != FSA_F32 && x_dtype != FSA_BF16 && x_dtype != FSA_F16) return FSA_ERR_DTYPE;
    if (!aligned(out_m1, (uintptr_t)elem_bytes(x_dtype))) return FSA_ERR_ALIGN;
    // the two-hop call validates everything else before it launches; the one-hop call takes a
    // subset of the same arguments and draws the same hop-1 IDs (same seed, hop counter 0)
    if (int rc = fsa_sample_mean_fwd(indptr, indptr_type, indices, num_nodes, x, x_dtype, D, seeds, B, fanouts, 2,
                                     seed, out, out_h1, out_ids1, out_ids2, stream))
        return rc;
    return fsa_sample_mean_fwd(indptr, indptr_type, indices, num_nodes, x, x_dtype, D, seeds, B, fanouts, 1,
                               seed, out_m1, nullptr, nullptr, nullptr, stream);
}

namespace {

// out[b] = mean over the slots j with cnt2[b,j] > 0 of table[b*k1+j]  (table = the [B,k1,D] per-slot means)
hipError_t slot_mean(const void* table, const int32_t* cnt2, int x_dtype, int64_t D, int64_t B, int32_t k1,
                     void* out, hipStream_t stream) {
    const void* rows[2] = {table, out};
    fsa::FwdArgs a{};
    a.x = table; a.x_kind = x_dtype; a.D = D; a.B = B; a.k1 = k1; a.hops = 1;
    a.slot_cnt = cnt2; a.out = out;
    a.geom = row_geometry(D, elem_bytes(x_dtype), rows, 2);
    return fsa::launch_forward(a, stream);
}

}  // namespace

int fsa_sample_mean3_fwd(const void* indptr, int indptr_type, const int32_t* indices,
                         int64_t num_nodes, const void* x, int x_dtype, int64_t D,
                         const int32_t* seeds, int64_t B, const int32_t* fanouts, uint64_t seed,
                         void* out, void* out_h1, void* out_h2, void* out_m1,
                         int32_t* out_ids1, int32_t* out_ids2, int32_t* out_ids3, int32_t* out_cnt2,
                         void* stream) {
    if (!indptr || !indices || !x || !fanouts) return FSA_ERR_NULL;
    if (B != 0 && (!seeds || !out || !out_h1 || !out_m1 || !out_ids1 || !out_cnt2)) return FSA_ERR_NULL;
    if (indptr_type != FSA_I32 && indptr_type != FSA_I64) return FSA_ERR_DTYPE;
    if (int rc = check_common(x_dtype, D, num_nodes, B)) return rc;
    const int32_t k1 = fanouts[0], k2 = fanouts[1], k3 = fanouts[2];
    if (!fanout_ok(k1) || !fanout_ok(k2) || !fanout_ok(k3)) return FSA_ERR_ARG;
    if (B * k1 > (int64_t)INT32_MAX) return FSA_ERR_ARG;       // hop-1 slots are the roots of the inner call
    const int eb = elem_bytes(x_dtype);
    if (!aligned(indptr, indptr_type == FSA_I64 ? 8 : 4) || !aligned(indices, 4) || !aligned(seeds, 4) ||
        !aligned(x, eb) || !aligned(out, eb) || !aligned(out_h1, eb) || !aligned(out_h2, eb) || !aligned(out_m1, eb) ||
        !aligned(out_ids1, 4) || !aligned(out_ids2, 4) || !aligned(out_ids3, 4) || !aligned(out_cnt2, 4))
        return FSA_ERR_ALIGN;
    if (B == 0) return FSA_OK;
    drop_stale_hip_error();
    hipStream_t st = static_cast<hipStream_t>(stream);

    // hop 0: the seeds' rows -> ids1 and the plain hop-1 mean
    {
        const void* rows[2] = {x, out_m1};
        fsa::FwdArgs a{};
        a.indptr = indptr; a.indptr_is64 = indptr_type == FSA_I64; a.indices = indices;
        a.x = x; a.x_kind = x_dtype; a.D = D; a.seeds = seeds; a.B = B; a.k1 = k1; a.hops = 1; a.seed = seed;
        a.out = out_m1; a.out_ids1 = out_ids1;
        a.geom = row_geometry(D, eb, rows, 2);
        if (hipError_t e = fsa::launch_forward(a, st)) return status_of(e);
    }
    // hops 1 and 2: the fused two-hop kernel with the B*k1 hop-1 slots as its roots
    {
        const void* rows[3] = {x, out_h1, out_h2};
        fsa::FwdArgs a{};
        a.indptr = indptr; a.indptr_is64 = indptr_type == FSA_I64; a.indices = indices;
        a.x = x; a.x_kind = x_dtype; a.D = D; a.seeds = out_ids1; a.B = B * k1; a.k1 = k2; a.k2 = k3; a.hops = 2;
        a.seed = seed; a.hop_base = 1;
        a.out = out_h1; a.out_h1 = out_h2; a.out_ids1 = out_ids2; a.out_ids2 = out_ids3; a.out_live = out_cnt2;
        a.geom = row_geometry(D, eb, rows, 3);
        if (hipError_t e = fsa::launch_forward(a, st)) return status_of(e);
    }
    return status_of(slot_mean(out_h1, out_cnt2, x_dtype, D, B, k1, out, st));
}

int fsa_mean3_replay_fwd(const void* x, int x_dtype, int64_t D, int64_t num_nodes,
                         const int32_t* ids1, const int32_t* ids2, const int32_t* ids3,
                         int64_t B, int32_t k1, int32_t k2, int32_t k3,
                         void* out, void* out_h1, void* out_h2, void* out_m1, int32_t* out_cnt2,
                         void* stream) {
    if (!x) return FSA_ERR_NULL;
    if (B != 0 && (!ids1 || !ids2 || !ids3 || !out || !out_h1 || !out_cnt2)) return FSA_ERR_NULL;
    if (int rc = check_common(x_dtype, D, num_nodes, B)) return rc;
    if (!fanout_ok(k1) || !fanout_ok(k2) || !fanout_ok(k3)) return FSA_ERR_ARG;
    if (B * k1 > (int64_t)INT32_MAX) return FSA_ERR_ARG;
    const int eb = elem_bytes(x_dtype);
    if (!aligned(x, eb) || !aligned(out, eb) || !aligned(out_h1, eb) || !aligned(out_h2, eb) || !aligned(out_m1, eb) ||
        !aligned(ids1, 4) || !aligned(ids2, 4) || !aligned(ids3, 4) || !aligned(out_cnt2, 4))
        return FSA_ERR_ALIGN;
    if (B == 0) return FSA_OK;
    drop_stale_hip_error();
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (out_m1) {
        const void* rows[2] = {x, out_m1};
        fsa::FwdArgs a{};
        a.x = x; a.x_kind = x_dtype; a.D = D; a.B = B; a.k1 = k1; a.hops = 1; a.ids1 = ids1; a.out = out_m1;
        a.geom = row_geometry(D, eb, rows, 2);
        if (hipError_t e = fsa::launch_forward(a, st)) return status_of(e);
    }
    {
        const void* rows[3] = {x, out_h1, out_h2};
        fsa::FwdArgs a{};
        a.x = x; a.x_kind = x_dtype; a.D = D; a.seeds = ids1;      // a negative ids1 switches its slot off
        a.B = B * k1; a.k1 = k2; a.k2 = k3; a.hops = 2; a.ids1 = ids2; a.ids2 = ids3;
        a.out = out_h1; a.out_h1 = out_h2; a.out_live = out_cnt2;
        a.geom = row_geometry(D, eb, rows, 3);
        if (hipError_t e = fsa::launch_forward(a, st)) return status_of(e);
    }
    return status_of(slot_mean(out_h1, out_cnt2, x_dtype, D, B, k1, out, st));
}

namespace {

int mean3_bwd_checked(const float* grad_out, const float* grad_h1, const float* grad_h2, const float* grad_m1,
                      const int32_t* ids1, const int32_t* ids2, const int32_t* ids3,
                      int64_t B, int32_t k1, int32_t k2, int32_t k3, int64_t D,
                      float* grad_x, int64_t num_nodes) {
    if (!grad_x) return FSA_ERR_NULL;
    if (B != 0 && (!grad_out || !ids1 || !ids2 || !ids3)) return FSA_ERR_NULL;
    if (int rc = check_common(FSA_F32, D, num_nodes, B)) return rc;
    if (!fanout_ok(k1) || !fanout_ok(k2) || !fanout_ok(k3)) return FSA_ERR_ARG;
    if (B * k1 > (int64_t)INT32_MAX) return FSA_ERR_ARG;
    if (!aligned(grad_out, 4) || !aligned(grad_h1, 4) || !aligned(grad_h2, 4) || !aligned(grad_m1, 4) ||
        !aligned(grad_x, 4) || !aligned(ids1, 4) || !aligned(ids2, 4) || !aligned(ids3, 4))
        return FSA_ERR_ALIGN;
    return FSA_OK;
}

// The three launches of the three-hop backward; `work` holds B*k1*D floats.
int mean3_bwd_launch(const float* grad_out, const float* grad_h1, const float* grad_h2, const float* grad_m1,
                     const int32_t* ids1, const int32_t* ids2, const int32_t* ids3,
                     int64_t B, int32_t k1, int32_t k2, int32_t k3, int64_t D,
                     float* grad_x, float* work, hipStream_t st) {
    drop_stale_hip_error();
    if (hipError_t e = fsa::launch_deep_grad(grad_out, grad_h1, ids1, ids2, ids3, work, B, k1, k2, k3, D, st)) return status_of(e);
    {
        fsa::BwdArgs a{};
        a.grad_out = work; a.grad_h1 = grad_h2; a.ids1 = ids2; a.ids2 = ids3; a.root_valid = ids1;
        a.B = B * k1; a.k1 = k2; a.k2 = k3; a.D = D; a.grad_x = grad_x;
        if (hipError_t e = fsa::launch_backward(a, st)) return status_of(e);
    }
    if (grad_m1) {
        fsa::BwdArgs a{};
        a.grad_out = grad_m1; a.ids1 = ids1; a.B = B; a.k1 = k1; a.k2 = 0; a.D = D; a.grad_x = grad_x;
        if (hipError_t e = fsa::launch_backward(a, st)) return status_of(e);
    }
    return FSA_OK;
}

}  // namespace

int fsa_mean3_bwd(const float* grad_out, const float* grad_h1, const float* grad_h2, const float* grad_m1,
                  const int32_t* ids1, const int32_t* ids2, const int32_t* ids3,
                  int64_t B, int32_t k1, int32_t k2, int32_t k3, int64_t D,
                  float* grad_x, int64_t num_nodes, float* work, void* stream) {
    if (B != 0 && !work) return FSA_ERR_NULL;
    if (int rc = mean3_bwd_checked(grad_out, grad_h1, grad_h2, grad_m1, ids1, ids2, ids3, B, k1, k2, k3, D, grad_x, num_nodes))
        return rc;
    if (!aligned(work, 4)) return FSA_ERR_ALIGN;
    if (B == 0) return FSA_OK;
    return mean3_bwd_launch(grad_out, grad_h1, grad_h2, grad_m1, ids1, ids2, ids3, B, k1, k2, k3, D, grad_x, work,
                            static_cast<hipStream_t>(stream));
}

int fsa_mean3_bwd_noalloc(const float* grad_out, const float* grad_h1, const float* grad_h2, const float* grad_m1,
                          const int32_t* ids1, const int32_t* ids2, const int32_t* ids3,
                          int64_t B, int32_t k1, int32_t k2, int32_t k3, int64_t D,
                          float* grad_x, int64_t num_nodes, void* stream) {
    if (int rc = mean3_bwd_checked(grad_out, grad_h1, grad_h2, grad_m1, ids1, ids2, ids3, B, k1, k2, k3, D, grad_x, num_nodes))
        return rc;
    if (B == 0) return FSA_OK;
    if (B * k1 > (int64_t)FSA_SCRATCH_FLOATS / D) return FSA_ERR_SCRATCH;   // B*k1*D floats would not fit
    float* work = scratch_pointer();
    if (!work) return FSA_ERR_HIP;
    return mean3_bwd_launch(grad_out, grad_h1, grad_h2, grad_m1, ids1, ids2, ids3, B, k1, k2, k3, D, grad_x, work,
                            static_cast<hipStream_t>(stream));
}


#ifdef FSA_TRACE
// Debug builds only: device buffer [B][4] of int64 that the 2-hop forward stamps (NULL = off).
void fsa_debug_set_trace(void* device_buffer) { fsa::g_trace = static_cast<long long*>(device_buffer); }
#endif

const char* fsa_status_string(int status) {
    switch (status) {
        case FSA_OK:        return "ok";
        case FSA_ERR_NULL:  return "a required pointer is NULL";
        case FSA_ERR_ARG:   return "a size, fanout or hop count is out of range";
        case FSA_ERR_DTYPE: return "unknown element type";
        case FSA_ERR_ALIGN: return "a pointer is not aligned to its element size";
        case FSA_ERR_HIP:   return "the HIP runtime refused the launch";
        case FSA_ERR_SCRATCH: return "the call needs more scratch memory than the library's fixed array holds";
        default:            return "unknown status";
    }
}

}  // extern "C"
