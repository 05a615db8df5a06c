// Host-side bounds check of the forward kernels' LDS index arithmetic (fsa_layout.h), built by
// tests/test_layout_bounds.py with -fsanitize=address,undefined.  For every fanout pair,
// waves-per-root value and table flavour it walks the same index expressions the 2-hop kernel
// forms -- strip offsets, owned slots, (slot, step) lane mapping, flat-list places, squeezed
// leaf places, draw-strip reads -- over worst-case and random slot counts and asserts that
// each stays inside the array it addresses and inside the LDS size the host code asks for.
#include <cstdio>
#include <cstdlib>
#include <cstdint>
#include <vector>

#include "../../paper_2511_13645_amd/csrc/fsa_layout.h"

#define CHECK(cond)                                                                                  \
    do {                                                                                             \
        if (!(cond)) {                                                                               \
            std::printf("FAILED %s  (k1=%d k2=%d nw=%d weighted=%d) at line %d\n", #cond, k1, k2, nw, \
                        (int)weighted, __LINE__);                                                    \
            return 1;                                                                                \
        }                                                                                            \
    } while (0)

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd() { rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull; return (uint32_t)(rng_state >> 33); }

int main() {
    long long cases = 0;
    for (int weighted = 0; weighted < 2; ++weighted)
    for (int k1 = 1; k1 <= 64; ++k1)
    for (int k2 = 1; k2 <= 64; ++k2)
    for (int nw = 1; nw <= 8; nw *= 2) {
        if (nw > 1 && nw > k1) continue;                    // the host never picks more waves than slots
        const int nq_max = (k1 + nw - 1) / nw;
        const fsa::Fwd2Layout L = fsa::fwd2_layout(nq_max, k2, weighted != 0);
        const int n = nq_max * k2;
        // arrays in order, each inside the strip, none overlapping the next
        struct Span { int at, len; };
        const Span spans[] = {{L.flat, 2 * n}, {L.meta, n}, {L.flat_w, weighted ? n : 0}, {L.leaf, n},
                              {L.leaf_w, weighted ? n : 0}, {L.cnt2, nq_max}, {L.empty_q, nq_max},
                              {L.rec, 4 * nq_max}, {L.slot_a, weighted ? nq_max : 0}, {L.draws, fsa::kDrawStripInts}};
        int prev_end = 0;
        for (const Span& s : spans) {
            CHECK(s.at >= prev_end);
            CHECK(s.at % 4 == 0);                            // 16-byte aligned: int2 / int4 accesses
            prev_end = s.at + s.len;
        }
        CHECK(prev_end <= L.per_wave);
        CHECK(L.per_wave % 4 == 0);
        // LDS the host asks for covers every strip, the per-strip counts and the reduction floats
        for (int rpw = 1; rpw <= (nw == 1 ? 8 : 1); rpw *= 2) {
            const int sub = 64, ve = 8;                      // largest reduction footprint
            const long long bytes = fsa::fwd2_lds_bytes(k1, k2, nw, rpw, weighted != 0, sub, ve);
            const long long strips = (long long)nw * rpw;
            CHECK(bytes >= 4 * (strips * L.per_wave + strips) + 4LL * nw * sub * ve);
        }
        // lane mapping of a pass
        const int spw = 64 / k2;
        CHECK(spw >= 1 && spw * k2 <= 64);
        int owned_total = 0;
        std::vector<char> seen(k1, 0);
        for (int wave = 0; wave < nw; ++wave) {
            const int nq = fsa::owned_slots(k1, nw, wave);
            CHECK(nq >= 0 && nq <= nq_max && nq <= 64);
            owned_total += nq;
            for (int q = 0; q < nq; ++q) {
                const int j = wave + q * nw;
                CHECK(j >= 0 && j < k1 && !seen[j]);
                seen[j] = 1;
            }
            // slot counts: all full, all empty, random
            for (int trial = 0; trial < 4; ++trial) {
                std::vector<int> c(nq_max, 0);
                for (int q = 0; q < nq; ++q) c[q] = trial == 0 ? k2 : trial == 1 ? 0 : (int)(rnd() % (unsigned)(k2 + 1));
                int off = 0;
                for (int q = 0; q < nq; ++q) {
                    for (int li = 0; li < c[q]; ++li) {
                        const int at = off + li;             // flat / meta / flat_w place
                        CHECK(at >= 0 && at < n);
                        CHECK(q * k2 + li < n);              // squeezed leaf place (replay)
                    }
                    off += c[q];
                }
                CHECK(off <= n);
                // sub-group split: blocks [my_start, my_start+my_len) tile [0, total)
                for (int sub_shift = 0; sub_shift <= 6; ++sub_shift) {
                    const int nsg = 64 >> sub_shift;
                    int covered = 0;
                    for (int sg = 0; sg < nsg; ++sg) {
                        auto first_q = [&](int s) {
                            int cnt = 0, o = 0;
                            for (int q = 0; q < nq; ++q) { if (o * nsg < s * off) ++cnt; o += c[q]; }
                            return cnt;
                        };
                        int qa = first_q(sg), qb = sg == nsg - 1 ? nq : first_q(sg + 1);
                        auto start_of = [&](int q) { int o = 0; for (int i = 0; i < q; ++i) o += c[i]; return o; };
                        const int my_start = qa < nq ? start_of(qa) : off;
                        const int my_len = (qb < nq ? start_of(qb) : off) - my_start;
                        CHECK(my_len >= 0 && my_start >= 0 && my_start + my_len <= off);
                        CHECK(my_start == covered);
                        covered += my_len;
                        // clipped reads of the rolling gather
                        const int list_at = my_len > 0 ? my_start : 0;
                        const int last_i = my_len > 0 ? my_len - 1 : 0;
                        if (off > 0) CHECK(list_at + last_i < off);
                    }
                    CHECK(covered == off);
                }
            }
        }
        CHECK(owned_total == k1);
        // draw strip: lanes of segment g read entries seg_base + m0 .. m0+3 for m0 < k2 in steps of 4
        for (int lane = 0; lane < 64; ++lane) {
            const int g = lane / k2;
            const int seg_base = g < spw ? g * k2 : 0;
            const int last_m0 = ((k2 - 1) / 4) * 4;
            CHECK(seg_base + last_m0 + 3 < fsa::kDrawStripInts);
        }
        ++cases;
    }
    // hop 0 uses the draw strip with one segment of k1 lanes
    for (int k1 = 1; k1 <= 64; ++k1) {
        const int last_m0 = ((k1 - 1) / 4) * 4;
        if (last_m0 + 3 >= fsa::kDrawStripInts || last_m0 + 3 >= 72) { std::printf("FAILED hop-0 draw strip k1=%d\n", k1); return 1; }
    }
    std::printf("ok %lld cases\n", cases);
    return 0;
}
