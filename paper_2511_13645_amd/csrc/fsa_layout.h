// Index arithmetic of the forward kernels' LDS strips, shared by the kernels and the host
// launch code, and written without HIP types so that a plain C++ compiler can build it: the
// CPU tests sweep every fanout / waves-per-root combination through these functions and
// check that every offset a kernel can form stays inside the strip the host sizes.
#pragma once

#if defined(__HIPCC__)
#define FSA_HD __host__ __device__
#else
#define FSA_HD
#endif

namespace fsa {

// Draw staging of the duplicate test: 64 lanes plus the overshoot of reading it in fours.
constexpr int kDrawStripInts = 68;

FSA_HD inline int round_up4(int v) { return (v + 3) & ~3; }

// One wave's strip of the 2-hop forward, offsets in ints from the strip base.  n = nq_max * k2
// is the most leaf rows the wave's nq_max hop-1 slots can name.
struct Fwd2Layout {
    int flat;       // int2[n]   row byte offsets of the leaf rows, slot by slot; bit 63 = last row of its slot
    int meta;       // int[n]    at a slot's last row: hop-1 slot j | owned index q << 8 | count << 16
    int flat_w;     // float[n]  weighted mean only: edge weight of each listed row
    int leaf;       // int[n]    replay only: saved leaf IDs squeezed to the front of each slot
    int leaf_w;     // float[n]  weighted replay only: their weights
    int cnt2;       // int[nq_max] replay: rows per owned slot; sampling: hop-1 node of each owned slot
    int empty_q;    // int[nq_max] owned slots without rows
    int rec;        // int4[nq_max] per owned slot: row start (lo, hi), degree (replay: count), place in flat
    int slot_a;     // float[nq_max] weighted mean only: weight of the hop-0 edge of each owned slot
    int draws;      // int[kDrawStripInts] Floyd draws of the lanes, for the duplicate test
    int per_wave;   // strip size, a multiple of 4 ints so that every strip starts 16-byte aligned
};

FSA_HD inline Fwd2Layout fwd2_layout(int nq_max, int k2, bool weighted) {
    Fwd2Layout L;
    const int n = nq_max * k2;
    int o = 0;
    L.flat = o;    o += round_up4(2 * n);
    L.meta = o;    o += round_up4(n);
    L.flat_w = o;  o += weighted ? round_up4(n) : 0;
    L.leaf = o;    o += round_up4(n);
    L.leaf_w = o;  o += weighted ? round_up4(n) : 0;
    L.cnt2 = o;    o += round_up4(nq_max);
    L.empty_q = o; o += round_up4(nq_max);
    L.rec = o;     o += 4 * nq_max;
    L.slot_a = o;  o += weighted ? round_up4(nq_max) : 0;
    L.draws = o;   o += kDrawStripInts;
    L.per_wave = o;
    return L;
}

// Hop-1 slots a wave owns when `nw` waves share a root with fanout k1: j = wave + q * nw.
FSA_HD inline int owned_slots(int k1, int nw, int wave) { return wave < k1 ? (k1 - wave + nw - 1) / nw : 0; }

// Dynamic LDS of one 2-hop forward workgroup, in bytes: the strips, one live-slot count (or
// outer weight) per strip, and the floats of the cross-wave reduction (used when nw > 1).
FSA_HD inline long long fwd2_lds_bytes(int k1, int k2, int nw, int roots_per_wg, bool weighted, int sub, int ve) {
    const Fwd2Layout L = fwd2_layout((k1 + nw - 1) / nw, k2, weighted);
    const long long strips = (long long)nw * roots_per_wg;
    return 4 * (strips * L.per_wave + round_up4((int)strips)) + 4LL * nw * sub * ve;
}

// 1-hop forward: per wave 64 staged IDs (the draws of the duplicate test use the same ints
// first) and 64 staged weights.
constexpr int kFwd1StripInts = 72 + 64;

}  // namespace fsa
