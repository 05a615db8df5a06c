// CPU ORACLE -- test infrastructure only; see fsa_oracle.h for what it is and what pins it.
// Plain single-threaded C++17: no blocking, no fusion, no vectorisation tricks.  Every
// function names the passage of the paper (arXiv 2511.13645) or of the published algorithm
// it follows.
#include "fsa_oracle.h"

#include <cmath>
#include <cstring>
#include <vector>

namespace {

// ---- reading the typed inputs ---------------------------------------------------------

int64_t read_indptr(const void* indptr, int type, int64_t i) {
    if (type == ORC_I64) return static_cast<const int64_t*>(indptr)[i];
    return static_cast<int64_t>(static_cast<const int32_t*>(indptr)[i]);
}

// bfloat16 is the upper half of an IEEE binary32; widening is exact.
double bf16_bits_to_double(uint16_t bits) {
    uint32_t w = static_cast<uint32_t>(bits) << 16;
    float f;
    std::memcpy(&f, &w, sizeof f);
    return static_cast<double>(f);
}

double read_x(const void* x, int dtype, int64_t row, int64_t D, int64_t d) {
    const int64_t at = row * D + d;
    switch (dtype) {
        case ORC_X_F32:  return static_cast<double>(static_cast<const float*>(x)[at]);
        case ORC_X_BF16: return bf16_bits_to_double(static_cast<const uint16_t*>(x)[at]);
        default:         return static_cast<const double*>(x)[at];
    }
}

// Number of non-negative entries among ids[0..k-1].
int32_t count_valid(const int32_t* ids, int32_t k) {
    int32_t c = 0;
    for (int32_t i = 0; i < k; ++i) c += (ids[i] >= 0);
    return c;
}

// Sec. 3.2, first display: sum of the feature rows named by the non-negative IDs, then
// divided by their count.  Empty -> zero row.  Returns the count.
int32_t mean_of_rows(const void* x, int dtype, int64_t D, const int32_t* ids, int32_t k,
                     double* dst) {
    for (int64_t d = 0; d < D; ++d) dst[d] = 0.0;
    const int32_t cnt = count_valid(ids, k);
    if (cnt == 0) return 0;
    for (int32_t i = 0; i < k; ++i) {
        if (ids[i] < 0) continue;
        for (int64_t d = 0; d < D; ++d) dst[d] += read_x(x, dtype, ids[i], D, d);
    }
    for (int64_t d = 0; d < D; ++d) dst[d] /= static_cast<double>(cnt);
    return cnt;
}

}  // namespace

extern "C" {

// Philox4x32-10, Salmon, Moraes, Dror, Shaw, "Parallel random numbers: as easy as 1, 2, 3",
// SC'11: a round multiplies counter words 0 and 2 by two fixed odd constants, and the
// high halves are mixed with words 1 and 3 and the round key; the key advances by the
// golden-ratio and sqrt(3)-1 Weyl constants between rounds.
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    const uint64_t mult_a = 0xD2511F53u;
    const uint64_t mult_b = 0xCD9E8D57u;
    const uint32_t weyl_a = 0x9E3779B9u;
    const uint32_t weyl_b = 0xBB67AE85u;
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        if (round > 0) { k0 += weyl_a; k1 += weyl_b; }
        const uint64_t pa = mult_a * c0;
        const uint64_t pb = mult_b * c2;
        const uint32_t n0 = static_cast<uint32_t>(pb >> 32) ^ c1 ^ k0;
        const uint32_t n1 = static_cast<uint32_t>(pb);
        const uint32_t n2 = static_cast<uint32_t>(pa >> 32) ^ c3 ^ k1;
        const uint32_t n3 = static_cast<uint32_t>(pa);
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// Counter layout fixed by this build (the paper only asks for seed-controlled, repeatable
// sampling, Sec. 3.3 "Reproducibility"): counter = (node, hop, step, 0), key = seed split
// into low and high words; word 0 of the output, scaled to [0, n) by multiply-high.
uint32_t orc_draw(uint64_t seed, uint32_t node, uint32_t hop, uint32_t step, uint32_t n) {
    const uint32_t ctr[4] = {node, hop, step, 0u};
    const uint32_t key[2] = {static_cast<uint32_t>(seed), static_cast<uint32_t>(seed >> 32)};
    uint32_t r[4];
    orc_philox4x32_10(ctr, key, r);
    return static_cast<uint32_t>((static_cast<uint64_t>(r[0]) * static_cast<uint64_t>(n)) >> 32);
}

// Floyd's algorithm for a uniform k-subset of {0..deg-1} (Bentley & Floyd, CACM 1987):
// for J = deg-k .. deg-1 draw t uniform in [0, J]; insert t unless already chosen, else
// insert J.  Sec. 3.2: t = min(k, |N(v)|), so deg <= k keeps the whole row in CSR order.
int32_t orc_floyd_select(int64_t deg, int32_t k, const uint32_t* t, int64_t* pos) {
    if (deg <= 0 || k <= 0) return 0;
    if (deg <= k) {
        for (int64_t i = 0; i < deg; ++i) pos[i] = i;
        return static_cast<int32_t>(deg);
    }
    for (int32_t i = 0; i < k; ++i) {
        const int64_t J = deg - k + i;
        const int64_t cand = static_cast<int64_t>(t[i]);
        bool seen = false;
        for (int32_t m = 0; m < i; ++m) seen = seen || (pos[m] == cand);
        pos[i] = seen ? J : cand;
    }
    return k;
}

int32_t orc_sample_row(const void* indptr, int indptr_type, const int32_t* indices,
                       int64_t node, uint32_t hop, int32_t k, uint64_t seed,
                       int64_t* pos, int32_t* ids) {
    const int64_t start = read_indptr(indptr, indptr_type, node);
    const int64_t deg = read_indptr(indptr, indptr_type, node + 1) - start;
    std::vector<uint32_t> t(static_cast<size_t>(k > 0 ? k : 0), 0u);
    if (deg > k) {
        for (int32_t i = 0; i < k; ++i) {
            const int64_t J = deg - k + i;
            t[i] = orc_draw(seed, static_cast<uint32_t>(node), hop, static_cast<uint32_t>(i),
                            static_cast<uint32_t>(J + 1));
        }
    }
    std::vector<int64_t> p(static_cast<size_t>(k > 0 ? k : 0), -1);
    const int32_t cnt = orc_floyd_select(deg, k, t.data(), p.data());
    for (int32_t i = 0; i < k; ++i) {
        const bool live = i < cnt;
        if (pos) pos[i] = live ? p[i] : -1;
        if (ids) ids[i] = live ? indices[start + p[i]] : -1;
    }
    return cnt;
}

// Sec. 3.2 ("FuseSampleAgg" paragraph): for every seed sample up to k neighbors from the
// CSR row and emit their mean; for fanouts (k1,k2) emit the nested mean, leaving out hop-1
// nodes whose own neighborhood is empty from both the sum and the divisor.
int orc_sample_mean_fwd(const void* indptr, int indptr_type, const int32_t* indices,
                        int64_t num_nodes, const void* x, int x_dtype, int64_t D,
                        const int32_t* seeds, int64_t B, const int32_t* fanouts, int num_hops,
                        uint64_t seed, double* out, double* out_h1,
                        int32_t* ids1, int32_t* ids2) {
    if (!indptr || !indices || !x || !seeds || !fanouts || !out) return -1;
    if (num_hops != 1 && num_hops != 2) return -2;
    if (B < 0 || D <= 0 || num_nodes <= 0) return -2;
    const int32_t k1 = fanouts[0];
    const int32_t k2 = (num_hops == 2) ? fanouts[1] : 0;
    if (k1 <= 0 || (num_hops == 2 && k2 <= 0)) return -2;

    std::vector<int32_t> U(static_cast<size_t>(k1));
    std::vector<int32_t> W(static_cast<size_t>(k2 > 0 ? k2 : 1));
    std::vector<double> inner(static_cast<size_t>(D));

    for (int64_t b = 0; b < B; ++b) {
        const int64_t r = seeds[b];
        if (r < 0 || r >= num_nodes) return -2;
        orc_sample_row(indptr, indptr_type, indices, r, 0u, k1, seed, nullptr, U.data());
        if (ids1) std::memcpy(ids1 + b * k1, U.data(), sizeof(int32_t) * k1);
        double* out_b = out + b * D;

        if (num_hops == 1) {
            mean_of_rows(x, x_dtype, D, U.data(), k1, out_b);
            continue;
        }

        for (int64_t d = 0; d < D; ++d) out_b[d] = 0.0;
        int32_t nonempty = 0;
        for (int32_t j = 0; j < k1; ++j) {
            int32_t c2 = 0;
            if (U[j] >= 0) {
                orc_sample_row(indptr, indptr_type, indices, U[j], 1u, k2, seed, nullptr, W.data());
                c2 = mean_of_rows(x, x_dtype, D, W.data(), k2, inner.data());
            } else {
                for (int32_t i = 0; i < k2; ++i) W[i] = -1;
                for (int64_t d = 0; d < D; ++d) inner[d] = 0.0;
            }
            if (ids2) std::memcpy(ids2 + (b * k1 + j) * k2, W.data(), sizeof(int32_t) * k2);
            if (out_h1) std::memcpy(out_h1 + (b * k1 + j) * D, inner.data(), sizeof(double) * D);
            if (c2 > 0) {
                ++nonempty;
                for (int64_t d = 0; d < D; ++d) out_b[d] += inner[d];
            }
        }
        if (nonempty > 0)
            for (int64_t d = 0; d < D; ++d) out_b[d] /= static_cast<double>(nonempty);
    }
    return 0;
}

// Prop. 1 (Sec. 3.3): with the sampled IDs fixed, the output is the plain mean over the
// named feature rows, exactly what materialise-then-aggregate would give.
int orc_mean_replay_fwd(const void* x, int x_dtype, int64_t D, int64_t num_nodes,
                        const int32_t* ids1, const int32_t* ids2,
                        int64_t B, int32_t k1, int32_t k2,
                        double* out, double* out_h1) {
    if (!x || !ids1 || !out) return -1;
    if (B < 0 || D <= 0 || k1 <= 0 || num_nodes <= 0) return -2;
    if (ids2 && k2 <= 0) return -2;
    std::vector<double> inner(static_cast<size_t>(D));
    for (int64_t b = 0; b < B; ++b) {
        double* out_b = out + b * D;
        if (!ids2) {
            mean_of_rows(x, x_dtype, D, ids1 + b * k1, k1, out_b);
            continue;
        }
        for (int64_t d = 0; d < D; ++d) out_b[d] = 0.0;
        int32_t nonempty = 0;
        for (int32_t j = 0; j < k1; ++j) {
            int32_t c2 = 0;
            if (ids1[b * k1 + j] >= 0) {
                c2 = mean_of_rows(x, x_dtype, D, ids2 + (b * k1 + j) * k2, k2, inner.data());
            } else {
                for (int64_t d = 0; d < D; ++d) inner[d] = 0.0;
            }
            if (out_h1) std::memcpy(out_h1 + (b * k1 + j) * D, inner.data(), sizeof(double) * D);
            if (c2 > 0) {
                ++nonempty;
                for (int64_t d = 0; d < D; ++d) out_b[d] += inner[d];
            }
        }
        if (nonempty > 0)
            for (int64_t d = 0; d < D; ++d) out_b[d] /= static_cast<double>(nonempty);
    }
    return 0;
}

// Sec. 3.3 "Reproducibility": backward replays the saved IDs so that gradients reach the
// same neighborhoods.  The forward is linear in X, so its adjoint sends to every sampled
// row the output gradient times the weight that row had in the mean.
int orc_mean_bwd(const double* grad_out, const double* grad_h1,
                 const int32_t* ids1, const int32_t* ids2,
                 int64_t B, int32_t k1, int32_t k2, int64_t D,
                 double* grad_x, int64_t num_nodes) {
    if (!grad_out || !ids1 || !grad_x) return -1;
    if (B < 0 || D <= 0 || k1 <= 0 || num_nodes <= 0) return -2;
    if (ids2 && k2 <= 0) return -2;
    for (int64_t b = 0; b < B; ++b) {
        const double* g_b = grad_out + b * D;
        if (!ids2) {
            const int32_t cnt = count_valid(ids1 + b * k1, k1);
            for (int32_t i = 0; i < k1; ++i) {
                const int32_t u = ids1[b * k1 + i];
                if (u < 0) continue;
                for (int64_t d = 0; d < D; ++d) grad_x[static_cast<int64_t>(u) * D + d] += g_b[d] / cnt;
            }
            continue;
        }
        int32_t nonempty = 0;
        for (int32_t j = 0; j < k1; ++j)
            if (ids1[b * k1 + j] >= 0 && count_valid(ids2 + (b * k1 + j) * k2, k2) > 0) ++nonempty;
        for (int32_t j = 0; j < k1; ++j) {
            if (ids1[b * k1 + j] < 0) continue;
            const int32_t* W = ids2 + (b * k1 + j) * k2;
            const int32_t c2 = count_valid(W, k2);
            if (c2 == 0) continue;
            for (int32_t i = 0; i < k2; ++i) {
                if (W[i] < 0) continue;
                for (int64_t d = 0; d < D; ++d) {
                    double g = g_b[d] / nonempty;
                    if (grad_h1) g += grad_h1[(b * k1 + j) * D + d];
                    grad_x[static_cast<int64_t>(W[i]) * D + d] += g / c2;
                }
            }
        }
    }
    return 0;
}

// ---- weighted mean ----------------------------------------------------------------------
// Sec. 3.2 "Extension Feasibility": weighted numerators and denominators per sampled
// neighborhood.  Written out as the plain definition over the sampled (ID, weight) pairs.
static double weighted_mean_of_rows(const void* x, int dtype, int64_t D, const int32_t* ids,
                                    const float* w, int32_t k, double* dst) {
    for (int64_t d = 0; d < D; ++d) dst[d] = 0.0;
    double total = 0.0;
    for (int32_t i = 0; i < k; ++i)
        if (ids[i] >= 0) total += static_cast<double>(w[i]);
    if (!(total > 0.0)) return 0.0;
    for (int32_t i = 0; i < k; ++i) {
        if (ids[i] < 0) continue;
        const double wi = static_cast<double>(w[i]);
        for (int64_t d = 0; d < D; ++d) dst[d] += wi * read_x(x, dtype, ids[i], D, d);
    }
    for (int64_t d = 0; d < D; ++d) dst[d] /= total;
    return total;
}

int orc_wmean_replay_fwd(const void* x, int x_dtype, int64_t D, int64_t num_nodes,
                         const int32_t* ids1, const int32_t* ids2, const float* w1, const float* w2,
                         int64_t B, int32_t k1, int32_t k2, double* out, double* out_h1) {
    if (!x || !ids1 || !w1 || !out) return -1;
    if (B < 0 || D <= 0 || k1 <= 0 || num_nodes <= 0) return -2;
    if (ids2 && (k2 <= 0 || !w2)) return -2;
    std::vector<double> inner(static_cast<size_t>(D));
    for (int64_t b = 0; b < B; ++b) {
        double* out_b = out + b * D;
        if (!ids2) {
            weighted_mean_of_rows(x, x_dtype, D, ids1 + b * k1, w1 + b * k1, k1, out_b);
            continue;
        }
        for (int64_t d = 0; d < D; ++d) out_b[d] = 0.0;
        double outer_total = 0.0;
        for (int32_t j = 0; j < k1; ++j) {
            double inner_total = 0.0;
            if (ids1[b * k1 + j] >= 0) {
                inner_total = weighted_mean_of_rows(x, x_dtype, D, ids2 + (b * k1 + j) * k2,
                                                    w2 + (b * k1 + j) * k2, k2, inner.data());
            } else {
                for (int64_t d = 0; d < D; ++d) inner[d] = 0.0;
            }
            if (out_h1) std::memcpy(out_h1 + (b * k1 + j) * D, inner.data(), sizeof(double) * D);
            if (inner_total > 0.0) {
                const double a = static_cast<double>(w1[b * k1 + j]);
                outer_total += a;
                for (int64_t d = 0; d < D; ++d) out_b[d] += a * inner[d];
            }
        }
        if (outer_total > 0.0) {
            for (int64_t d = 0; d < D; ++d) out_b[d] /= outer_total;
        } else {
            for (int64_t d = 0; d < D; ++d) out_b[d] = 0.0;
        }
    }
    return 0;
}

int orc_sample_wmean_fwd(const void* indptr, int indptr_type, const int32_t* indices,
                         const float* edge_weight, int64_t num_nodes,
                         const void* x, int x_dtype, int64_t D,
                         const int32_t* seeds, int64_t B, const int32_t* fanouts, int num_hops,
                         uint64_t seed, double* out, double* out_h1,
                         int32_t* ids1, int32_t* ids2, float* w1, float* w2) {
    if (!indptr || !indices || !edge_weight || !x || !seeds || !fanouts || !out) return -1;
    if (num_hops != 1 && num_hops != 2) return -2;
    if (B < 0 || D <= 0 || num_nodes <= 0) return -2;
    const int32_t k1 = fanouts[0];
    const int32_t k2 = (num_hops == 2) ? fanouts[1] : 0;
    if (k1 <= 0 || (num_hops == 2 && k2 <= 0)) return -2;
    if (B == 0) return 0;                                     // an empty batch: nothing to sample or write
    // sample IDs and pick up the weight of every sampled edge slot, then average as in replay
    std::vector<int32_t> U(static_cast<size_t>(B) * k1, -1), W;
    std::vector<float> A(static_cast<size_t>(B) * k1, 0.0f), Wt;
    if (num_hops == 2) {
        W.assign(static_cast<size_t>(B) * k1 * k2, -1);
        Wt.assign(static_cast<size_t>(B) * k1 * k2, 0.0f);
    }
    std::vector<int64_t> pos(static_cast<size_t>(k1 > k2 ? k1 : k2));
    for (int64_t b = 0; b < B; ++b) {
        const int64_t r = seeds[b];
        if (r < 0 || r >= num_nodes) return -2;
        const int32_t c1 = orc_sample_row(indptr, indptr_type, indices, r, 0u, k1, seed, pos.data(), &U[b * k1]);
        const int64_t s0 = read_indptr(indptr, indptr_type, r);
        for (int32_t j = 0; j < c1; ++j) A[b * k1 + j] = edge_weight[s0 + pos[j]];
        if (num_hops == 1) continue;
        for (int32_t j = 0; j < c1; ++j) {
            const int64_t u = U[b * k1 + j];
            const int32_t c2 = orc_sample_row(indptr, indptr_type, indices, u, 1u, k2, seed, pos.data(),
                                              &W[(b * k1 + j) * k2]);
            const int64_t s1 = read_indptr(indptr, indptr_type, u);
            for (int32_t i = 0; i < c2; ++i) Wt[(b * k1 + j) * k2 + i] = edge_weight[s1 + pos[i]];
        }
    }
    // (an empty batch has nothing to copy: memcpy must not be handed the empty vectors' null data)
    if (ids1 && !U.empty()) std::memcpy(ids1, U.data(), sizeof(int32_t) * U.size());
    if (w1 && !A.empty()) std::memcpy(w1, A.data(), sizeof(float) * A.size());
    if (num_hops == 2) {
        if (ids2 && !W.empty()) std::memcpy(ids2, W.data(), sizeof(int32_t) * W.size());
        if (w2 && !Wt.empty()) std::memcpy(w2, Wt.data(), sizeof(float) * Wt.size());
    }
    return orc_wmean_replay_fwd(x, x_dtype, D, num_nodes, U.data(), num_hops == 2 ? W.data() : nullptr,
                                A.data(), num_hops == 2 ? Wt.data() : nullptr, B, k1, k2, out, out_h1);
}

// Adjoint of the weighted replay forward with respect to X (weights are data, not variables).
int orc_wmean_bwd(const double* grad_out, const double* grad_h1,
                  const int32_t* ids1, const int32_t* ids2, const float* w1, const float* w2,
                  int64_t B, int32_t k1, int32_t k2, int64_t D, double* grad_x, int64_t num_nodes) {
    if (!grad_out || !ids1 || !w1 || !grad_x) return -1;
    if (B < 0 || D <= 0 || k1 <= 0 || num_nodes <= 0) return -2;
    if (ids2 && (k2 <= 0 || !w2)) return -2;
    for (int64_t b = 0; b < B; ++b) {
        const double* g_b = grad_out + b * D;
        if (!ids2) {
            double total = 0.0;
            for (int32_t i = 0; i < k1; ++i)
                if (ids1[b * k1 + i] >= 0) total += static_cast<double>(w1[b * k1 + i]);
            if (!(total > 0.0)) continue;
            for (int32_t i = 0; i < k1; ++i) {
                const int32_t u = ids1[b * k1 + i];
                if (u < 0) continue;
                const double share = static_cast<double>(w1[b * k1 + i]) / total;
                for (int64_t d = 0; d < D; ++d) grad_x[static_cast<int64_t>(u) * D + d] += g_b[d] * share;
            }
            continue;
        }
        std::vector<double> inner_total(static_cast<size_t>(k1), 0.0);
        double outer_total = 0.0;
        for (int32_t j = 0; j < k1; ++j) {
            if (ids1[b * k1 + j] < 0) continue;
            for (int32_t i = 0; i < k2; ++i)
                if (ids2[(b * k1 + j) * k2 + i] >= 0) inner_total[j] += static_cast<double>(w2[(b * k1 + j) * k2 + i]);
            if (inner_total[j] > 0.0) outer_total += static_cast<double>(w1[b * k1 + j]);
        }
        for (int32_t j = 0; j < k1; ++j) {
            if (!(inner_total[j] > 0.0)) continue;
            const double outer_share = outer_total > 0.0 ? static_cast<double>(w1[b * k1 + j]) / outer_total : 0.0;
            for (int32_t i = 0; i < k2; ++i) {
                const int32_t w = ids2[(b * k1 + j) * k2 + i];
                if (w < 0) continue;
                const double share = static_cast<double>(w2[(b * k1 + j) * k2 + i]) / inner_total[j];
                for (int64_t d = 0; d < D; ++d) {
                    double g = g_b[d] * outer_share;
                    if (grad_h1) g += grad_h1[(b * k1 + j) * D + d];
                    grad_x[static_cast<int64_t>(w) * D + d] += g * share;
                }
            }
        }
    }
    return 0;
}

// ---- three hops (the nested mean of Sec. 3.2 taken one level deeper) -------------------

// Prop. 1 for three levels of saved IDs: every mean is the plain mean of the named rows, and
// an empty neighborhood leaves both the sum and the divisor of the level above.
int orc_mean3_replay_fwd(const void* x, int x_dtype, int64_t D, int64_t num_nodes,
                         const int32_t* ids1, const int32_t* ids2, const int32_t* ids3,
                         int64_t B, int32_t k1, int32_t k2, int32_t k3,
                         double* out, double* out_h1, double* out_h2, double* out_m1,
                         int32_t* cnt2) {
    if (!x || !ids1 || !ids2 || !ids3 || !out) return -1;
    if (B < 0 || D <= 0 || k1 <= 0 || k2 <= 0 || k3 <= 0 || num_nodes <= 0) return -2;
    std::vector<double> leaf_mean(static_cast<size_t>(D)), mid(static_cast<size_t>(D));
    for (int64_t b = 0; b < B; ++b) {
        double* out_b = out + b * D;
        for (int64_t d = 0; d < D; ++d) out_b[d] = 0.0;
        if (out_m1) mean_of_rows(x, x_dtype, D, ids1 + b * k1, k1, out_m1 + b * D);
        int32_t live_j = 0;
        for (int32_t j = 0; j < k1; ++j) {
            const int64_t bj = b * k1 + j;
            for (int64_t d = 0; d < D; ++d) mid[d] = 0.0;
            int32_t live_i = 0;
            for (int32_t i = 0; i < k2; ++i) {
                const int64_t bji = bj * k2 + i;
                int32_t c3 = 0;
                if (ids1[bj] >= 0 && ids2[bji] >= 0)
                    c3 = mean_of_rows(x, x_dtype, D, ids3 + bji * k3, k3, leaf_mean.data());
                else
                    for (int64_t d = 0; d < D; ++d) leaf_mean[d] = 0.0;
                if (out_h2) std::memcpy(out_h2 + bji * D, leaf_mean.data(), sizeof(double) * D);
                if (c3 > 0) {
                    ++live_i;
                    for (int64_t d = 0; d < D; ++d) mid[d] += leaf_mean[d];
                }
            }
            if (live_i > 0)
                for (int64_t d = 0; d < D; ++d) mid[d] /= static_cast<double>(live_i);
            if (cnt2) cnt2[bj] = live_i;
            if (out_h1) std::memcpy(out_h1 + bj * D, mid.data(), sizeof(double) * D);
            if (live_i > 0) {
                ++live_j;
                for (int64_t d = 0; d < D; ++d) out_b[d] += mid[d];
            }
        }
        if (live_j > 0)
            for (int64_t d = 0; d < D; ++d) out_b[d] /= static_cast<double>(live_j);
    }
    return 0;
}

// Sampling for three hops: the seed's row with hop counter 0, the rows of its sampled
// neighbors with counter 1, the rows of theirs with counter 2; then the means of the IDs.
int orc_sample_mean3_fwd(const void* indptr, int indptr_type, const int32_t* indices,
                         int64_t num_nodes, const void* x, int x_dtype, int64_t D,
                         const int32_t* seeds, int64_t B, const int32_t* fanouts, uint64_t seed,
                         double* out, double* out_h1, double* out_h2, double* out_m1,
                         int32_t* ids1, int32_t* ids2, int32_t* ids3, int32_t* cnt2) {
    if (!indptr || !indices || !x || !seeds || !fanouts || !out || !ids1 || !ids2 || !ids3) return -1;
    const int32_t k1 = fanouts[0], k2 = fanouts[1], k3 = fanouts[2];
    if (B < 0 || D <= 0 || k1 <= 0 || k2 <= 0 || k3 <= 0 || num_nodes <= 0) return -2;
    for (int64_t b = 0; b < B; ++b) {
        const int64_t r = seeds[b];
        if (r < 0 || r >= num_nodes) return -2;
        int32_t* U = ids1 + b * k1;
        orc_sample_row(indptr, indptr_type, indices, r, 0u, k1, seed, nullptr, U);
        for (int32_t j = 0; j < k1; ++j) {
            int32_t* V = ids2 + (b * k1 + j) * k2;
            if (U[j] >= 0) orc_sample_row(indptr, indptr_type, indices, U[j], 1u, k2, seed, nullptr, V);
            else for (int32_t i = 0; i < k2; ++i) V[i] = -1;
            for (int32_t i = 0; i < k2; ++i) {
                int32_t* W = ids3 + ((b * k1 + j) * k2 + i) * k3;
                if (V[i] >= 0) orc_sample_row(indptr, indptr_type, indices, V[i], 2u, k3, seed, nullptr, W);
                else for (int32_t l = 0; l < k3; ++l) W[l] = -1;
            }
        }
    }
    return orc_mean3_replay_fwd(x, x_dtype, D, num_nodes, ids1, ids2, ids3, B, k1, k2, k3,
                                out, out_h1, out_h2, out_m1, cnt2);
}

// Adjoint of orc_mean3_replay_fwd with respect to X for upstream gradients on out, out_h1,
// out_h2 and out_m1 (each nullable except grad_out), accumulated into grad_x.
int orc_mean3_bwd(const double* grad_out, const double* grad_h1, const double* grad_h2,
                  const double* grad_m1,
                  const int32_t* ids1, const int32_t* ids2, const int32_t* ids3,
                  int64_t B, int32_t k1, int32_t k2, int32_t k3, int64_t D,
                  double* grad_x, int64_t num_nodes) {
    if (!grad_out || !ids1 || !ids2 || !ids3 || !grad_x) return -1;
    if (B < 0 || D <= 0 || k1 <= 0 || k2 <= 0 || k3 <= 0 || num_nodes <= 0) return -2;
    std::vector<int32_t> c3(static_cast<size_t>(k1) * k2), live_i(static_cast<size_t>(k1));
    for (int64_t b = 0; b < B; ++b) {
        int32_t live_j = 0;
        for (int32_t j = 0; j < k1; ++j) {
            live_i[j] = 0;
            for (int32_t i = 0; i < k2; ++i) {
                const int64_t bji = (b * k1 + j) * k2 + i;
                int32_t c = 0;
                if (ids1[b * k1 + j] >= 0 && ids2[bji] >= 0) c = count_valid(ids3 + bji * k3, k3);
                c3[j * k2 + i] = c;
                if (c > 0) ++live_i[j];
            }
            if (live_i[j] > 0) ++live_j;
        }
        for (int32_t j = 0; j < k1; ++j) {
            if (live_i[j] == 0) continue;
            for (int32_t i = 0; i < k2; ++i) {
                const int32_t c = c3[j * k2 + i];
                if (c == 0) continue;
                const int64_t bji = (b * k1 + j) * k2 + i;
                for (int32_t l = 0; l < k3; ++l) {
                    const int32_t w = ids3[bji * k3 + l];
                    if (w < 0) continue;
                    for (int64_t d = 0; d < D; ++d) {
                        double g = grad_out[b * D + d] / live_j;
                        if (grad_h1) g += grad_h1[(b * k1 + j) * D + d];
                        g /= live_i[j];
                        if (grad_h2) g += grad_h2[bji * D + d];
                        grad_x[static_cast<int64_t>(w) * D + d] += g / c;
                    }
                }
            }
        }
        if (grad_m1) {
            const int32_t c1 = count_valid(ids1 + b * k1, k1);
            for (int32_t j = 0; j < k1; ++j) {
                const int32_t u = ids1[b * k1 + j];
                if (u < 0) continue;
                for (int64_t d = 0; d < D; ++d) grad_x[static_cast<int64_t>(u) * D + d] += grad_m1[b * D + d] / c1;
            }
        }
    }
    return 0;
}

void orc_round_to_bf16(const double* src, int64_t n, uint16_t* dst) {
    for (int64_t i = 0; i < n; ++i) {
        const double v = src[i];
        float f;
        if (v == 0.0 || std::isnan(v) || std::isinf(v)) {
            f = static_cast<float>(v);
        } else {
            int e;
            std::frexp(v, &e);                 // |v| = m * 2^e, m in [0.5, 1)
            int q = e - 8;                     // quantum 2^q keeps 8 significant bits
            if (q < -133) q = -133;            // bfloat16 subnormal spacing
            const double scaled = std::nearbyint(std::ldexp(v, -q));  // ties to even
            f = static_cast<float>(std::ldexp(scaled, q));            // exact in binary32
        }
        uint32_t w;
        std::memcpy(&w, &f, sizeof w);
        dst[i] = static_cast<uint16_t>(w >> 16);
    }
}

void orc_round_to_f32(const double* src, int64_t n, float* dst) {
    for (int64_t i = 0; i < n; ++i) dst[i] = static_cast<float>(src[i]);
}

}  // extern "C"
