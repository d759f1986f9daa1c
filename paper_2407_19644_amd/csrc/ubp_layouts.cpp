// Host side of the UBP library: the kernels' private re-layouts of the packed weights, each
// derived from the canonical arrays of Section 4.2 (indptr, indices, rotated values) on first
// use.  No device code here.
#include <algorithm>
#include <cstring>
#include <numeric>

#include "ubp_internal.h"

namespace ubp {

namespace {

struct Entry {
    int32_t k;     // column of W == row of X
    uint32_t mask; // stripes of the row group with a kept weight in this column
    int32_t slot;  // index into the row group's weight scratch
};

void build_one(const ubp_packed *p, StripeLayout &L, int G, int CT) {
    const int M = p->M, K = p->K, bh = p->bh, bw = p->bw;
    const int rgh = kStripe * G;
    const int RR = ring_rows(CT), PITCH = ring_pitch(CT), R = ring_slots(CT);
    L.G = G;
    L.CT = CT;
    L.nrg = (M + rgh - 1) / rgh;
    L.nch = (K + kSlotRows - 1) / kSlotRows;
    L.rg_ptr.assign((size_t)L.nrg + 1, 0);
    L.stream.clear();
    L.nsteps = 0;
    L.total_mfma = 0;
    const size_t rec_dw = 128 + 256 * (size_t)G;
    const uint16_t *vals = reinterpret_cast<const uint16_t *>(p->values.data());
    const int32_t nstart = M - bh + 1; // start rows 0..M-bh
    std::vector<int32_t> colslot((size_t)K, -1);
    std::vector<Entry> entries;
    std::vector<uint16_t> wbuf; // [entry slot][rgh]
    std::vector<int64_t> rg_weight((size_t)L.nrg, 0);
    struct Step { size_t pos, n; int cmin, cmax, rel; };
    std::vector<Step> steps;

    for (int rg = 0; rg < L.nrg; ++rg) {
        const int row0 = rg * rgh, row1 = std::min(M, row0 + rgh);
        entries.clear();
        wbuf.clear();
        // blocks whose rows [r, r+bh) meet [row0, row1): start rows in (row0-bh, row1)
        const int s0 = std::max(0, row0 - bh + 1), s1 = std::min(nstart, row1);
        for (int i = s0; i < s1; ++i) {
            for (int32_t b = p->indptr[(size_t)i]; b < p->indptr[(size_t)i + 1]; ++b) {
                const int32_t c = p->indices[(size_t)b];
                for (int q = 0; q < bw; ++q) {
                    const int k = c + q;
                    int32_t &slot = colslot[(size_t)k]; // the columns of all blocks of the row group are merged
                    if (slot < 0) {
                        slot = (int32_t)entries.size();
                        entries.push_back(Entry{k, 0u, slot});
                        wbuf.resize(wbuf.size() + (size_t)rgh, 0);
                    }
                    for (int rho = std::max(i, row0); rho < std::min(i + bh, row1); ++rho) {
                        // rotated storage: row rho of block b lives in slot rho mod bh
                        wbuf[(size_t)slot * rgh + (rho - row0)] = vals[((int64_t)b * bw + q) * bh + (rho % bh)];
                        entries[(size_t)slot].mask |= 1u << ((rho - row0) / kStripe);
                    }
                }
            }
        }
        for (const Entry &e : entries) colslot[(size_t)e.k] = -1;
        const int window = ring_window(CT);
        std::sort(entries.begin(), entries.end(), [window](const Entry &a, const Entry &b) {
            const int wa = a.k / window, wb = b.k / window;
            if (wa != wb) return wa < wb;
            if (a.mask != b.mask) return a.mask < b.mask;
            return a.k < b.k;
        });
        // steps: up to 32 entries whose X rows lie in at most R/2 + 1 consecutive ring slots
        std::vector<Step> real;
        for (size_t pos = 0; pos < entries.size();) {
            int cmin = entries[pos].k / kSlotRows, cmax = cmin;
            size_t n = 0;
            const size_t unit = 1;
            while (n + unit <= (size_t)kStep && pos + n < entries.size()) {
                const int c0 = entries[pos + n].k / kSlotRows, c1 = entries[pos + n + unit - 1].k / kSlotRows;
                const int lo = std::min(cmin, c0), hi = std::max(cmax, c1);
                if (hi - lo > R / 2) break; // at most half the ring, whatever the window size
                cmin = lo;
                cmax = hi;
                n += unit;
            }
            if (n > 8) {
                // Order inside the step is free.  One transposed LDS read serves 16 entries, 8 per
                // half wavefront, and those 8 rows hit distinct banks when their ring rows differ
                // modulo 8 (the ring's swizzle): deal the entries, sorted by that residue, round-robin
                // over the step's four groups of 8, so equal residues land in different groups.
                std::stable_sort(entries.begin() + (std::ptrdiff_t)pos, entries.begin() + (std::ptrdiff_t)(pos + n),
                                 [](const Entry &a, const Entry &b) { return (a.k & 7) < (b.k & 7); });
                std::vector<Entry> dealt(n);
                const size_t groups = (n + 7) / 8;
                size_t at[4] = {0, 8, 16, 24};
                for (size_t e = 0; e < n; ++e) {
                    size_t gsel = e % groups;
                    // a group that is already full (the last one may be shorter) passes its turn on
                    for (size_t tries = 0; tries < groups && at[gsel] >= std::min(n, 8 * (gsel + 1)); ++tries)
                        gsel = (gsel + 1) % groups;
                    dealt[at[gsel]++] = entries[pos + e];
                }
                std::copy(dealt.begin(), dealt.end(), entries.begin() + (std::ptrdiff_t)pos);
            }
            real.push_back(Step{pos, n, cmin, cmax, 0});
            pos += n;
        }
        // rel: chunks below it are read neither by the step nor by any later one
        auto set_rel = [&](std::vector<Step> &v) {
            int m = L.nch;
            for (size_t t = v.size(); t-- > 0;) {
                if (v[t].n) m = std::min(m, v[t].cmin);
                v[t].rel = m;
            }
        };
        set_rel(real);
        // The kernel gathers the rows of step t while the products of step t-1 are still being
        // issued, so at that moment it holds every chunk from rel(t-1) to cmax(t).  Two of the R
        // ring slots must stay free, or producer and consumers could wait for each other.  Where
        // two neighbouring steps lie further apart (a row group with few, scattered blocks) an
        // empty step goes between them: it reads nothing, and rel(empty) = rel(t).
        steps.clear();
        for (size_t t = 0; t < real.size(); ++t) {
            if (real[t].cmax - real[t].rel > R - 2) {
                L.G = 0; // unusable; the launcher reports UBP_ERR_UNSUPPORTED
                return;
            }
            if (t > 0 && real[t].cmax - real[t - 1].rel > R - 2) steps.push_back(Step{0, 0, 0, 0, 0});
            steps.push_back(real[t]);
        }
        // empty steps up to a multiple of the prefetch depth
        while (steps.size() % kPrefetchDepth != 0) steps.push_back(Step{0, 0, 0, 0, 0});
        set_rel(steps);

        L.rg_ptr[(size_t)rg] = (int32_t)L.nsteps;
        for (size_t si = 0; si < steps.size(); ++si) {
            const Step &st = steps[si];
            uint32_t mask = 0;
            for (size_t e = 0; e < st.n; ++e) mask |= entries[st.pos + e].mask;
            const size_t rec = L.stream.size();
            L.stream.resize(rec + rec_dw, 0u);
            // control word: the highest chunk the step reads (0 for an empty step: nothing to wait
            // for), and what may be handed back when its gather is issued: everything that no step
            // from the previous one on reads (the previous step's reads may still be in flight)
            const uint32_t ctl = (uint32_t)(st.n ? st.cmax : 0) | ((uint32_t)steps[si > 0 ? si - 1 : 0].rel << 16);
            // ring row of entry idx of this step; padding entries repeat the first row, an empty
            // step reads ring row 0 (the value is never used)
            auto ring_row = [&](size_t idx) {
                return st.n == 0 ? 0 : (idx < st.n ? entries[st.pos + idx].k : entries[st.pos].k) % RR;
            };
            auto lds_addr = [&](size_t idx, int sub) {
                const int r = ring_row(idx);
                return (uint32_t)(r * PITCH + (ring_swizzle(CT, r) << 5) + sub);
            };
            for (int lane = 0; lane < 64; ++lane) {
                // lanes 4e..4e+3 of 16-lane group g read entry 4g+e (first transposed read) and
                // entry 16+4g+e (second); each of the 4 lanes reads 8 bytes (4 pixels)
                const int g = lane / 16, t = lane % 16, e = t / 4, sub = (t % 4) * 8;
                const uint32_t lo = lds_addr((size_t)(4 * g + e), sub), hi = lds_addr((size_t)(16 + 4 * g + e), sub);
                L.stream[rec + 2 * lane] = (lo >> 3) | ((hi >> 3) << 14) | (mask << 28);
                L.stream[rec + 2 * lane + 1] = ctl;
            }
            // weight fragments: lane (n = lane mod 16, g = lane / 16) holds row 16*j + n and, in
            // element order, entries 4g..4g+3 then 16+4g..16+4g+3 (the order the reads deliver)
            uint16_t *frag = reinterpret_cast<uint16_t *>(&L.stream[rec + 128]);
            for (int j = 0; j < G; ++j) {
                if (!(mask & (1u << j))) continue;
                for (int lane = 0; lane < 64; ++lane) {
                    const int g = lane / 16, nrow = lane % 16;
                    for (int e = 0; e < 8; ++e) {
                        const size_t idx = (size_t)(e < 4 ? 4 * g + e : 16 + 4 * g + (e - 4));
                        if (idx < st.n)
                            frag[((size_t)j * 64 + lane) * 8 + e] =
                                wbuf[(size_t)entries[st.pos + idx].slot * rgh + (kStripe * j + nrow)];
                    }
                }
                ++L.total_mfma;
                ++rg_weight[(size_t)rg];
            }
            ++L.nsteps;
        }
    }
    L.rg_ptr[(size_t)L.nrg] = (int32_t)L.nsteps;
    // spare records: the kernel fetches kPrefetchDepth steps ahead without checking for the end
    L.stream.resize(L.stream.size() + rec_dw * kPrefetchDepth, 0u);
    if (L.stream.size() * sizeof(uint32_t) >= (size_t(1) << 31)) {
        L.G = 0; // the kernel addresses the stream with 32-bit byte offsets
        return;
    }
    L.rg_order.resize((size_t)L.nrg);
    std::iota(L.rg_order.begin(), L.rg_order.end(), 0);
    std::stable_sort(L.rg_order.begin(), L.rg_order.end(),
                     [&](int32_t a, int32_t b) { return rg_weight[(size_t)a] > rg_weight[(size_t)b]; });
}

// Operand tiles for the small-K kernel.  Element e of lane (n = lane mod 16, g = lane / 16) of
// tile (stripe, kt) is W[16*stripe + n][32*kt + i] with i = 4g + e for e < 4 and 16 + 4g + (e - 4)
// otherwise: the order in which two transposed LDS reads deliver 32 consecutive rows of X.
void build_tiles(const ubp_packed *p, TileLayout &T) {
    T.kt_pad = 0;
    const int M = p->M, K = p->K, bh = p->bh, bw = p->bw;
    const int kt = (K + kStep - 1) / kStep;
    // K <= 256: 2, 4, 6 or 8 tiles per stripe (held in registers at once); beyond that whole chunks
    // of 8 tiles, while the zero-filled matrix stays small
    const int kt_pad = K <= kTileMaxK ? std::max(2, ((kt + 1) / 2) * 2) : ((kt + 7) / 8) * 8;
    const int nstripes = (M + kStripe - 1) / kStripe;
    if ((int64_t)nstripes * kt_pad * 1024 > kTileMaxBytes) return;
    T.kt_pad = kt_pad;
    T.nstripes = nstripes;
    T.frags.assign((size_t)T.nstripes * T.kt_pad * 512, 0);
    const int words = (kt_pad + 31) / 32;
    T.occupied.assign((size_t)nstripes * words, 0u);
    const uint16_t *vals = reinterpret_cast<const uint16_t *>(p->values.data());
    const int32_t nstart = M - bh + 1;
    for (int i = 0; i < nstart; ++i)
        for (int32_t b = p->indptr[(size_t)i]; b < p->indptr[(size_t)i + 1]; ++b) {
            const int32_t c = p->indices[(size_t)b];
            for (int q = 0; q < bw; ++q) {
                const int k = c + q, t = k / kStep, idx = k % kStep;
                // position of entry idx inside a lane's 8 elements, and the lane group that holds it
                const int g = (idx % 16) / 4, e = (idx % 4) + (idx >= 16 ? 4 : 0);
                for (int rho = i; rho < i + bh; ++rho) {
                    const int stripe = rho / kStripe, n = rho % kStripe;
                    const uint16_t v = vals[((int64_t)b * bw + q) * bh + (rho % bh)]; // rotated storage
                    T.frags[(((size_t)stripe * T.kt_pad + t) * 64 + (size_t)(16 * g + n)) * 8 + e] = v;
                    if (v) T.occupied[(size_t)stripe * words + t / 32] |= 1u << (t % 32);
                }
            }
        }
    T.tiles_nonzero = 0;
    for (uint32_t w : T.occupied) T.tiles_nonzero += __builtin_popcount(w);
}

// ---------------------------------------------------------------- block kernel layout
struct Half {
    int32_t a;      // first row of the 16-row window of X
    int32_t b;      // block
    int32_t h;      // which 16 columns of the block
    int32_t r;      // the block's first row
    int32_t o;      // r mod 16
    bool hi;        // has rows in the stripe after the one it starts in (inside the row group)
};

// Row groups of the block layout: consecutive runs of at most G stripes.  A run costs roughly
// (halves that start in it + halves that reach into it from the stripe above) / 2 steps, and a
// workgroup lasts as long as its heaviest row group, so stripes with many blocks get short runs
// and the others long ones.  The number of runs is the smallest possible, rounded up to a whole
// number of workgroup rows of kBlkConsumers wavefronts (the spare runs cost nothing there); the
// cut minimises the sum of cubed costs.  first[g] = first stripe of run g, first[runs] = nstripes.
constexpr int kBlkConsumers = 14;

std::vector<int32_t> cut_row_groups(const ubp_packed *p, int G) {
    const int M = p->M, bh = p->bh;
    const int nstripes = (M + kStripe - 1) / kStripe;
    const int nh = (p->bw + 15) / 16;
    std::vector<int64_t> start((size_t)nstripes + 1, 0), reach((size_t)nstripes + 1, 0); // halves starting in / reaching below stripe s
    for (int i = 0; i + bh <= M; ++i) {
        const int64_t nb = p->indptr[(size_t)i + 1] - p->indptr[(size_t)i];
        start[(size_t)(i / kStripe)] += nb * nh;
        if (i % kStripe + bh > kStripe) reach[(size_t)(i / kStripe)] += nb * nh;
    }
    const int least = (nstripes + G - 1) / G;
    int runs = std::min(nstripes, (least + kBlkConsumers - 1) / kBlkConsumers * kBlkConsumers);
    std::vector<int32_t> first;
    auto fixed = [&]() {
        first.clear();
        for (int s = 0; s < nstripes; s += G) first.push_back(s);
        first.push_back(nstripes);
    };
    if (runs == least || (int64_t)runs * nstripes > (int64_t(1) << 24)) {
        fixed();
        return first;
    }
    auto cost = [&](int s0, int s1) { // stripes s0 .. s1 - 1
        int64_t c = s0 > 0 ? (reach[(size_t)s0 - 1] + 1) / 2 : 0;
        for (int s = s0; s < s1; ++s) c += (start[(size_t)s] + 1) / 2;
        return (double)c * (double)c * (double)c;
    };
    const double kInf = 1e300;
    // best[k][s]: stripes [0, s) in k runs
    std::vector<std::vector<double>> best((size_t)runs + 1, std::vector<double>((size_t)nstripes + 1, kInf));
    std::vector<std::vector<int8_t>> len((size_t)runs + 1, std::vector<int8_t>((size_t)nstripes + 1, 0));
    best[0][0] = 0.0;
    for (int k = 1; k <= runs; ++k)
        for (int s = 1; s <= nstripes; ++s)
            for (int l = 1; l <= G && l <= s; ++l) {
                const double b = best[(size_t)k - 1][(size_t)(s - l)];
                if (b >= kInf) continue;
                const double c = b + cost(s - l, s);
                if (c < best[(size_t)k][(size_t)s]) {
                    best[(size_t)k][(size_t)s] = c;
                    len[(size_t)k][(size_t)s] = (int8_t)l;
                }
            }
    if (best[(size_t)runs][(size_t)nstripes] >= kInf) {
        fixed();
        return first;
    }
    first.assign((size_t)runs + 1, 0);
    for (int k = runs, s = nstripes; k >= 1; --k) {
        first[(size_t)k] = s;
        s -= len[(size_t)k][(size_t)s];
    }
    return first;
}

void build_blk(const ubp_packed *p, BlkLayout &L, int G) {
    const int M = p->M, K = p->K, bh = p->bh, bw = p->bw;
    constexpr int CT = 4;
    const int R = ring_slots(CT);
    const int pair_span = R / 2; // chunks two halves of a step may lie apart (a wavefront then holds at most R / 2 + 2)
    L.G = G;
    L.rg_first = cut_row_groups(p, G);
    L.nrg = (int)L.rg_first.size() - 1;
    L.nch = (K + kSlotRows - 1) / kSlotRows;
    L.rg_ptr.assign((size_t)L.nrg + 1, 0);
    L.meta.clear();
    L.frags.clear();
    L.nsteps = 0;
    L.total_mfma = 0;
    L.halves = L.paired = 0;
    const uint16_t *vals = reinterpret_cast<const uint16_t *>(p->values.data());
    const int32_t nstart = M - bh + 1;
    const int nh = (bw + 15) / 16;
    std::vector<int64_t> rg_weight((size_t)L.nrg, 0);
    struct Step { int A, B, jj, cmin, cmax, rel; }; // A, B: indices into halves (-1: none); jj 15: empty
    std::vector<Half> halves;
    std::vector<Step> real, steps;
    std::vector<int> cls[kStripe + 1];

    for (int rg = 0; rg < L.nrg; ++rg) {
        const int row0 = kStripe * L.rg_first[(size_t)rg], row1 = std::min(M, kStripe * L.rg_first[(size_t)rg + 1]);
        const int cnt = L.rg_first[(size_t)rg + 1] - L.rg_first[(size_t)rg]; // stripes of this run (at most G)
        halves.clear();
        for (int j = 0; j <= G; ++j) cls[j].clear();
        const int s0 = std::max(0, row0 - bh + 1), s1 = std::min(nstart, row1);
        for (int i = s0; i < s1; ++i)
            for (int32_t b = p->indptr[(size_t)i]; b < p->indptr[(size_t)i + 1]; ++b) {
                const int t = i - row0;                      // -15 .. row1 - row0 - 1
                const int j = t >= 0 ? t / kStripe : -1;     // stripe of the row group the block starts in
                const int o = ((t % kStripe) + kStripe) % kStripe;
                const bool hi = o + bh > kStripe && j + 1 < cnt && row0 + kStripe * (j + 1) < row1;
                if (j < 0 && !hi) continue;                  // no row inside the group
                for (int h = 0; h < nh; ++h) {
                    const int a = std::min(p->indices[(size_t)b] + 16 * h, K - 16);
                    cls[j + 1].push_back((int)halves.size());
                    halves.push_back(Half{a, b, h, i, o, hi});
                }
            }
        L.halves += (int64_t)halves.size();
        // Pairs: halves of one class (same first stripe), neighbours by window row, close enough
        // for both windows to be in the ring together with room to spare.
        real.clear();
        for (int jj = 0; jj <= G; ++jj) {
            std::vector<int> &v = cls[jj];
            std::stable_sort(v.begin(), v.end(), [&](int x, int y) { return halves[(size_t)x].a < halves[(size_t)y].a; });
            for (size_t i = 0; i < v.size();) {
                const Half &A = halves[(size_t)v[i]];
                const int cmin = A.a / kSlotRows;
                if (i + 1 < v.size() && (halves[(size_t)v[i + 1]].a + 15) / kSlotRows - cmin <= pair_span) {
                    real.push_back(Step{v[i], v[i + 1], jj, cmin, (halves[(size_t)v[i + 1]].a + 15) / kSlotRows, 0});
                    L.paired += 2;
                    i += 2;
                } else {
                    real.push_back(Step{v[i], -1, jj, cmin, (A.a + 15) / kSlotRows, 0});
                    i += 1;
                }
            }
        }
        std::stable_sort(real.begin(), real.end(), [&](const Step &x, const Step &y) {
            return halves[(size_t)x.A].a < halves[(size_t)y.A].a;
        });
        // rel: chunks below it are read neither by the step nor by any later one
        auto set_rel = [&](std::vector<Step> &v) {
            int m = L.nch;
            for (size_t t = v.size(); t-- > 0;) {
                if (v[t].jj != 15) m = std::min(m, v[t].cmin);
                v[t].rel = m;
            }
        };
        set_rel(real);
        // A wavefront hands back, right after the reads of step t - 1, every chunk below rel(t);
        // while it waits for the chunks of step t it therefore holds rel(t) .. cmax(t), which is
        // at most pair_span + 2 chunks: the ring always has free slots for the producers.
        steps.clear();
        const Step empty{-1, -1, 15, 0, 0, 0};
        for (size_t t = 0; t < real.size(); ++t) {
            if (real[t].cmax - real[t].rel > R - 2) { // (cannot happen: see pair_span)
                L.G = 0;
                return;
            }
            steps.push_back(real[t]);
        }
        while (steps.size() % kPrefetchDepth != 0) steps.push_back(empty);
        set_rel(steps);

        L.rg_ptr[(size_t)rg] = (int32_t)L.nsteps;
        for (size_t si = 0; si < steps.size(); ++si) {
            const Step &st = steps[si];
            const size_t mpos = L.meta.size(), fpos = L.frags.size();
            L.meta.resize(mpos + 2, 0u);
            L.frags.resize(fpos + 256, 0u);
            const uint32_t rel = (uint32_t)(si + 1 < steps.size() ? steps[si + 1].rel : L.nch); // after this step's reads
            if (st.jj == 15) {
                L.meta[mpos + 1] = (15u << 8) | (rel << 22);
                ++L.nsteps;
                continue;
            }
            const Half &A = halves[(size_t)st.A];
            const Half *B = st.B >= 0 ? &halves[(size_t)st.B] : nullptr;
            const bool any_lo = st.jj >= 1, any_hi = A.hi || (B && B->hi);
            L.meta[mpos] = (uint32_t)A.a | ((uint32_t)(B ? B->a : A.a) << 16);
            L.meta[mpos + 1] = (uint32_t)A.o | ((uint32_t)(B ? B->o : A.o) << 4) | ((uint32_t)st.jj << 8) |
                               ((any_lo ? 1u : 0u) << 12) | ((any_hi ? 1u : 0u) << 13) | (rel << 22);
            uint16_t *frag = reinterpret_cast<uint16_t *>(&L.frags[fpos]);
            for (int lane = 0; lane < 64; ++lane) {
                const int g = lane / 16, n = lane % 16;
                for (int e = 0; e < 8; ++e) {
                    const Half *H = e < 4 ? &A : B;
                    if (!H) continue;
                    const int i = 4 * g + (e & 3);                                 // entry = window row modulo 16
                    const int rho = H->a + (((i - H->a) % 16) + 16) % 16;          // row of X
                    const int q = rho - p->indices[(size_t)H->b];                  // column of the block
                    if (q < 16 * H->h || q >= std::min(bw, 16 * H->h + 16)) continue;
                    const int d = ((n - H->o) % 16 + 16) % 16;                     // row of the block in slot n
                    if (d >= bh) continue;
                    frag[(size_t)lane * 8 + e] = vals[((int64_t)H->b * bw + q) * bh + ((H->r + d) % bh)];
                }
            }
            const int mf = (any_lo ? 1 : 0) + (any_hi ? 1 : 0);
            L.total_mfma += mf;
            rg_weight[(size_t)rg] += mf;
            ++L.nsteps;
        }
    }
    L.rg_ptr[(size_t)L.nrg] = (int32_t)L.nsteps;
    // spare records: the kernel fetches kPrefetchDepth steps ahead (and metadata 64 steps ahead)
    // without checking for the end
    L.frags.resize(L.frags.size() + (size_t)256 * kPrefetchDepth, 0u);
    L.meta.resize(L.meta.size() + (size_t)2 * 128, 0u);
    if (L.frags.size() * sizeof(uint32_t) >= (size_t(1) << 31)) {
        L.G = 0; // the kernel addresses the records with 32-bit byte offsets
        return;
    }
    L.rg_order.resize((size_t)L.nrg);
    std::iota(L.rg_order.begin(), L.rg_order.end(), 0);
    std::stable_sort(L.rg_order.begin(), L.rg_order.end(),
                     [&](int32_t a, int32_t b) { return rg_weight[(size_t)a] > rg_weight[(size_t)b]; });
    L.rg_order.insert(L.rg_order.end(), L.rg_first.begin(), L.rg_first.end());
}

} // namespace

bool blk_eligible(const ubp_packed *p) {
    return p->dtype != UBP_F32 && p->bh <= kStripe && p->K >= 16 && (p->K + kSlotRows - 1) / kSlotRows < 1023;
}

const StripeLayout &get_stripe_layout(const ubp_packed *p, int G, int CT) {
    StripeLayout &L = p->sg[layout_slot(G, CT)];
    if (!L.built) {
        L.built = true;
        L.G = 0;
        // chunk indices are 16-bit in the records
        if (p->dtype != UBP_F32 && (p->K + kSlotRows - 1) / kSlotRows <= 0xffff) build_one(p, L, G, CT);
    }
    return L;
}

const BlkLayout &get_blk_layout(const ubp_packed *p, int G) {
    BlkLayout &L = p->blk[blk_slot(G)];
    if (!L.built) {
        L.built = true;
        L.G = 0;
        if (blk_eligible(p)) build_blk(p, L, G);
    }
    return L;
}

const TileLayout &get_tile_layout(const ubp_packed *p) {
    TileLayout &T = p->tiles;
    if (!T.built) {
        T.built = true;
        T.kt_pad = 0;
        if (p->dtype != UBP_F32) build_tiles(p, T);
    }
    return T;
}

} // namespace ubp
