// Host side of the UBP library: test-mask generator, offline weight transform
// (validation, canonical ordering, indptr / indices, weight rotation) and the
// accessors of the handle.  No device code here.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>
#include <numeric>

#include "ubp_internal.h"

namespace {

// ---------------------------------------------------------------- RNG (SplitMix64)
struct SplitMix64 {
    uint64_t s;
    explicit SplitMix64(uint64_t seed) : s(seed) {}
    uint64_t next() {
        s += 0x9E3779B97F4A7C15ull;
        uint64_t z = s;
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        return z ^ (z >> 31);
    }
    // uniform in [0, n), unbiased: reject words at or above floor(2^64 / n) * n
    uint64_t bounded(uint64_t n) {
        // floor(2^64 / n) computed without 128-bit arithmetic
        uint64_t q = (~0ull) / n;
        if ((~0ull) % n == n - 1) ++q; // 2^64 is a multiple of n
        uint64_t limit = q * n;        // wraps to 0 exactly when 2^64 itself is the limit
        for (;;) {
            uint64_t x = next();
            if (limit == 0 || x < limit) return x % n;
        }
    }
};

// Occupancy bitmap of the M x K matrix.
struct CellMap {
    int64_t K;
    std::vector<uint64_t> bits;
    CellMap(int64_t M, int64_t K_) : K(K_), bits((size_t)((M * K_ + 63) / 64), 0) {}
    bool get(int64_t r, int64_t c) const {
        int64_t t = r * K + c;
        return (bits[(size_t)(t >> 6)] >> (t & 63)) & 1;
    }
    void set(int64_t r, int64_t c) {
        int64_t t = r * K + c;
        bits[(size_t)(t >> 6)] |= 1ull << (t & 63);
    }
    bool any(int32_t r, int32_t c, int32_t bh, int32_t bw) const {
        for (int32_t i = 0; i < bh; ++i)
            for (int32_t j = 0; j < bw; ++j)
                if (get(r + i, c + j)) return true;
        return false;
    }
    void paint(int32_t r, int32_t c, int32_t bh, int32_t bw) {
        for (int32_t i = 0; i < bh; ++i)
            for (int32_t j = 0; j < bw; ++j) set(r + i, c + j);
    }
};

bool block_less(const ubp_block &a, const ubp_block &b) { return a.r != b.r ? a.r < b.r : a.c < b.c; }

// Capped Zipf targets per rank: t = min(cap, lambda * rank^-s), sum == nb, integers by
// largest remainder (ties to the lower rank).
bool zipf_targets(int64_t nb, int64_t S, int64_t cap, double s, std::vector<int64_t> &t) {
    if (nb > S * cap) return false;
    std::vector<double> w((size_t)S);
    for (int64_t j = 0; j < S; ++j) w[(size_t)j] = std::pow((double)(j + 1), -s);
    std::vector<char> capped((size_t)S, 0);
    double remaining = (double)nb, lam = 0.0;
    for (;;) {
        double wsum = 0.0;
        for (int64_t j = 0; j < S; ++j)
            if (!capped[(size_t)j]) wsum += w[(size_t)j];
        if (wsum <= 0.0) break;
        lam = remaining / wsum;
        bool changed = false;
        for (int64_t j = 0; j < S; ++j)
            if (!capped[(size_t)j] && lam * w[(size_t)j] > (double)cap) {
                capped[(size_t)j] = 1;
                remaining -= (double)cap;
                changed = true;
            }
        if (!changed) break;
    }
    std::vector<double> real((size_t)S), frac((size_t)S);
    t.assign((size_t)S, 0);
    int64_t sum = 0;
    for (int64_t j = 0; j < S; ++j) {
        real[(size_t)j] = capped[(size_t)j] ? (double)cap : lam * w[(size_t)j];
        t[(size_t)j] = (int64_t)std::floor(real[(size_t)j]);
        frac[(size_t)j] = real[(size_t)j] - (double)t[(size_t)j];
        sum += t[(size_t)j];
    }
    std::vector<int64_t> order((size_t)S);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(),
                     [&](int64_t a, int64_t b) { return frac[(size_t)a] > frac[(size_t)b]; });
    int64_t left = nb - sum;
    for (int64_t i = 0; left > 0; ++i) {
        int64_t j = order[(size_t)(i % S)];
        if (t[(size_t)j] < cap) {
            ++t[(size_t)j];
            --left;
        }
    }
    return true;
}

} // namespace

extern "C" {

int64_t ubp_target_block_count(int32_t M, int32_t K, int32_t bh, int32_t bw, double density) {
    if (M < 1 || K < 1 || bh < 1 || bw < 1 || bh > M || bw > K || !(density >= 0.0 && density <= 1.0)) return -1;
    return (int64_t)std::floor(((double)M * (double)K * density) / (double)(bh * bw) + 1e-9);
}

ubp_status ubp_select_reference(int32_t M, int32_t K, int32_t bh, int32_t bw, double density, uint64_t seed,
                                int32_t mode, double zipf_s, ubp_block *out, int64_t capacity, int64_t *out_nb) {
    if (!out_nb) return UBP_ERR_INVALID_ARG;
    *out_nb = 0;
    int64_t nb = ubp_target_block_count(M, K, bh, bw, density);
    if (nb < 0 || (mode != 0 && mode != 1)) return UBP_ERR_INVALID_ARG;
    *out_nb = nb;
    if (capacity < nb || (nb > 0 && !out)) return UBP_ERR_INVALID_ARG;
    try {
        SplitMix64 rng(seed);
        CellMap occ(M, K);
        const int64_t nr = (int64_t)M - bh + 1, nc = (int64_t)K - bw + 1;
        const int64_t max_attempts = 2000 * nb + 100000;
        int64_t got_total = 0;
        auto fill = [&](int64_t count, int64_t r_base, int64_t r_span) -> bool {
            int64_t attempts = 0, got = 0;
            while (got < count) {
                if (++attempts > max_attempts) return false;
                int32_t r = (int32_t)(r_base + (int64_t)rng.bounded((uint64_t)r_span));
                int32_t c = (int32_t)rng.bounded((uint64_t)nc);
                if (occ.any(r, c, bh, bw)) continue;
                occ.paint(r, c, bh, bw);
                out[got_total++] = ubp_block{r, c};
                ++got;
            }
            return true;
        };
        if (mode == 0) {
            if (!fill(nb, 0, nr)) return UBP_ERR_INFEASIBLE;
        } else {
            const int64_t S = (nr + bh - 1) / bh;
            const int64_t cap = (int64_t)std::floor(0.375 * (double)K / (double)bw);
            std::vector<int64_t> t_rank;
            if (!zipf_targets(nb, S, cap, zipf_s, t_rank)) return UBP_ERR_INFEASIBLE;
            std::vector<int64_t> perm((size_t)S);
            std::iota(perm.begin(), perm.end(), 0);
            for (int64_t i = S - 1; i > 0; --i) std::swap(perm[(size_t)i], perm[(size_t)rng.bounded((uint64_t)i + 1)]);
            std::vector<int64_t> t_stripe((size_t)S, 0);
            for (int64_t rank = 0; rank < S; ++rank) t_stripe[(size_t)perm[(size_t)rank]] = t_rank[(size_t)rank];
            for (int64_t st = 0; st < S; ++st) {
                int64_t rows = std::min<int64_t>(bh, nr - bh * st);
                if (!fill(t_stripe[(size_t)st], bh * st, rows)) return UBP_ERR_INFEASIBLE;
            }
        }
        std::sort(out, out + nb, block_less);
    } catch (const std::bad_alloc &) {
        return UBP_ERR_ALLOC;
    }
    return UBP_OK;
}

ubp_status ubp_pack(const void *W_host, ubp_dtype dtype, int32_t M, int32_t K, int64_t ldw, int32_t bh, int32_t bw,
                    const ubp_block *blocks, int64_t nb, int32_t device, ubp_packed **out) {
    if (!out) return UBP_ERR_INVALID_ARG;
    *out = nullptr;
    if (M < 1 || K < 1 || bh < 1 || bw < 1 || nb < 0 || ldw < K || (nb > 0 && (!blocks || !W_host))) return UBP_ERR_INVALID_ARG;
    if (dtype != UBP_F32 && dtype != UBP_F16 && dtype != UBP_BF16) return UBP_ERR_INVALID_ARG;
    if (device < UBP_HOST_ONLY) return UBP_ERR_INVALID_ARG;
    ubp_packed *p = nullptr;
    try {
        // a1: bounds (the edge rule of Eq. 1), then pairwise disjointness (Eq. 2) on a cell bitmap
        for (int64_t b = 0; b < nb; ++b) {
            const ubp_block &k = blocks[b];
            if (k.r < 0 || k.c < 0 || (int64_t)k.r + bh > M || (int64_t)k.c + bw > K) return UBP_ERR_OUT_OF_BOUNDS;
        }
        {
            CellMap occ(M, K);
            for (int64_t b = 0; b < nb; ++b) {
                if (occ.any(blocks[b].r, blocks[b].c, bh, bw)) return UBP_ERR_OVERLAP;
                occ.paint(blocks[b].r, blocks[b].c, bh, bw);
            }
        }
        p = new ubp_packed();
        p->M = M; p->K = K; p->bh = bh; p->bw = bw; p->nb = nb; p->dtype = dtype;
        // canonical order: start row, then column origin
        std::vector<ubp_block> sorted(blocks, blocks + nb);
        std::sort(sorted.begin(), sorted.end(), block_less);
        // a2: metadata. indptr is indexed by START ROW (the tile row index advances by one
        // row in an unaligned kernel, Section 3.3), valid start rows are 0..M-bh.
        const int64_t nstart = (int64_t)M - bh + 1;
        p->indptr.assign((size_t)(nstart > 0 ? nstart + 1 : 1), 0);
        for (int64_t b = 0; b < nb; ++b) ++p->indptr[(size_t)sorted[(size_t)b].r + 1];
        for (size_t i = 1; i < p->indptr.size(); ++i) p->indptr[i] += p->indptr[i - 1];
        p->indices.resize((size_t)nb);
        // a3: weight rotation (Section 4.2): the weight of matrix row rho goes to slot rho mod bh
        const int64_t esz = ubp::dtype_size(dtype);
        p->values.assign((size_t)(nb * bw * bh * esz), 0);
        const uint8_t *w = static_cast<const uint8_t *>(W_host);
        for (int64_t b = 0; b < nb; ++b) {
            const int32_t r = sorted[(size_t)b].r, c = sorted[(size_t)b].c;
            p->indices[(size_t)b] = c;
            for (int32_t q = 0; q < bw; ++q)
                for (int32_t d = 0; d < bh; ++d) {
                    const int32_t rho = r + d, s = rho % bh;
                    std::memcpy(&p->values[(size_t)(((b * bw + q) * bh + s) * esz)],
                                w + ((int64_t)rho * ldw + (c + q)) * esz, (size_t)esz);
                }
        }
        if (dtype != UBP_F32) ubp::build_stripe_layouts(p);
        if (device != UBP_HOST_ONLY) {
            p->device = device;
            ubp_status st = ubp::upload(p);
            if (st != UBP_OK) {
                ubp::release_device(p);
                delete p;
                return st;
            }
        }
    } catch (const std::bad_alloc &) {
        if (p) {
            ubp::release_device(p);
            delete p;
        }
        return UBP_ERR_ALLOC;
    }
    *out = p;
    return UBP_OK;
}

const int32_t *ubp_packed_indptr(const ubp_packed *p, int64_t *len) {
    if (!p) return nullptr;
    if (len) *len = (int64_t)p->indptr.size();
    return p->indptr.data();
}

const int32_t *ubp_packed_indices(const ubp_packed *p, int64_t *len) {
    if (!p) return nullptr;
    if (len) *len = (int64_t)p->indices.size();
    return p->indices.data();
}

const void *ubp_packed_values(const ubp_packed *p, int64_t *len_elems) {
    if (!p) return nullptr;
    if (len_elems) *len_elems = p->nb * p->bw * p->bh;
    return p->values.data();
}

int64_t ubp_packed_info(const ubp_packed *p, int32_t what) {
    if (!p) return -1;
    switch (what) {
    case 0: return p->M;
    case 1: return p->K;
    case 2: return p->bh;
    case 3: return p->bw;
    case 4: return p->nb;
    case 5: return (int64_t)p->dtype;
    case 6: return p->device;
    case 7: return (int64_t)p->values.size() + (int64_t)(p->indptr.size() + p->indices.size()) * 4;
    case 8: return p->device_bytes;
    default:
        // 100 + layout slot: weight fragments (MFMA issues per 16-column tile) of that layout
        if (what >= 100 && what < 100 + ubp::kNumLayouts) return p->sg[what - 100].total_mfma;
        if (what >= 200 && what < 200 + ubp::kNumLayouts) return p->sg[what - 200].nsteps;
        if (what >= 300 && what < 300 + ubp::kNumLayouts) return p->sgn[what - 300].G ? p->sgn[what - 300].total_mfma : -1;
        if (what >= 400 && what < 400 + ubp::kNumLayouts) return p->sgn[what - 400].G ? p->sgn[what - 400].nsteps : -1;
        return -1;
    }
}

ubp_status ubp_packed_layout(const ubp_packed *p, int32_t sub_stripes, int32_t col_tiles, int32_t native,
                             int32_t *row_groups, const int32_t **rg_ptr, const int32_t **rg_order,
                             const uint32_t **stream, int64_t *stream_words) {
    if (!p || native < 1 || native > 3) return UBP_ERR_INVALID_ARG;
    if (native == 3) {
        // the dense operand tiles: row_groups = stripes, stream = the tiles as 32-bit words
        const ubp::TileLayout &T = p->tiles;
        if (T.kt_pad == 0) return UBP_ERR_UNSUPPORTED;
        if (row_groups) *row_groups = T.nstripes;
        if (rg_ptr) *rg_ptr = nullptr;
        if (rg_order) *rg_order = nullptr;
        if (stream) *stream = reinterpret_cast<const uint32_t *>(T.frags.data());
        if (stream_words) *stream_words = (int64_t)(T.frags.size() / 2);
        return UBP_OK;
    }
    const int slot = ubp::layout_slot(sub_stripes, col_tiles);
    if (slot < 0) return UBP_ERR_INVALID_ARG;
    const ubp::StripeLayout &L = native == 2 ? p->sgn[slot] : p->sg[slot];
    if (L.G == 0) return UBP_ERR_UNSUPPORTED;
    if (row_groups) *row_groups = L.nrg;
    if (rg_ptr) *rg_ptr = L.rg_ptr.data();
    if (rg_order) *rg_order = L.rg_order.data();
    if (stream) *stream = L.stream.data();
    if (stream_words) *stream_words = (int64_t)L.stream.size();
    return UBP_OK;
}

void ubp_packed_free(ubp_packed *p) {
    if (!p) return;
    ubp::release_device(p);
    delete p;
}

const char *ubp_status_string(ubp_status s) {
    switch (s) {
    case UBP_OK: return "ok";
    case UBP_ERR_INVALID_ARG: return "invalid argument";
    case UBP_ERR_OUT_OF_BOUNDS: return "block out of bounds";
    case UBP_ERR_OVERLAP: return "blocks overlap";
    case UBP_ERR_UNSUPPORTED: return "unsupported configuration";
    case UBP_ERR_INFEASIBLE: return "block selection infeasible";
    case UBP_ERR_ALLOC: return "allocation failed";
    case UBP_ERR_DEVICE: return "HIP device error";
    }
    return "unknown status";
}

} // extern "C"

// ---------------------------------------------------------------- private MFMA layout
namespace ubp {

namespace {

struct Entry {
    int32_t k;     // column of W == row of X
    uint32_t mask; // stripes of the row group with a kept weight in this column
    int32_t slot;  // index into the row group's weight scratch
    int32_t blk;   // block-native layouts: the block this column belongs to (else unused)
    int32_t off;   // block-native layouts: the block's first row minus the row group's first row
};

} // namespace

static void build_one(ubp_packed *p, StripeLayout &L, int G, int CT, bool native) {
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
    L.native = native;
    const size_t rec_dw = 128 + 256 * (size_t)(native ? 1 : G);
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
                    int32_t fresh = -1;
                    // block-native: one entry per column of every block; otherwise the columns of
                    // all blocks of the row group are merged
                    int32_t &slot = native ? fresh : colslot[(size_t)k];
                    if (slot < 0) {
                        slot = (int32_t)entries.size();
                        entries.push_back(Entry{k, 0u, slot, b, i - row0});
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
        if (!native)
            for (const Entry &e : entries) colslot[(size_t)e.k] = -1;
        const int window = ring_window(CT);
        if (native) {
            // every column of a block carries the block's stripe set and sorts with its first column
            for (size_t e = 0; e < entries.size(); e += (size_t)bw) {
                uint32_t m = 0;
                for (int q = 0; q < bw; ++q) m |= entries[e + q].mask;
                for (int q = 0; q < bw; ++q) entries[e + q].mask = m;
            }
            std::vector<size_t> order(entries.size() / (size_t)bw);
            std::iota(order.begin(), order.end(), 0);
            std::sort(order.begin(), order.end(), [&](size_t x, size_t y) {
                const Entry &a = entries[x * bw], &b = entries[y * bw];
                const int wa = a.k / window, wb = b.k / window;
                if (wa != wb) return wa < wb;
                if (a.mask != b.mask) return a.mask < b.mask;
                if (a.k != b.k) return a.k < b.k;
                return a.blk < b.blk;
            });
            std::vector<Entry> sorted;
            sorted.reserve(entries.size());
            for (size_t x : order)
                for (int q = 0; q < bw; ++q) sorted.push_back(entries[x * bw + q]);
            entries.swap(sorted);
        } else {
            std::sort(entries.begin(), entries.end(), [window](const Entry &a, const Entry &b) {
                const int wa = a.k / window, wb = b.k / window;
                if (wa != wb) return wa < wb;
                if (a.mask != b.mask) return a.mask < b.mask;
                return a.k < b.k;
            });
        }
        // steps: up to 32 entries whose X rows lie in at most R/2 + 1 consecutive ring slots
        std::vector<Step> real;
        for (size_t pos = 0; pos < entries.size();) {
            int cmin = entries[pos].k / kSlotRows, cmax = cmin;
            size_t n = 0;
            const size_t unit = native ? (size_t)bw : 1; // block-native steps hold whole blocks
            while (n + unit <= (size_t)kStep && pos + n < entries.size()) {
                const int c0 = entries[pos + n].k / kSlotRows, c1 = entries[pos + n + unit - 1].k / kSlotRows;
                const int lo = std::min(cmin, c0), hi = std::max(cmax, c1);
                if (hi - lo > R / 2) break; // at most half the ring, whatever the window size
                cmin = lo;
                cmax = hi;
                n += unit;
            }
            if (!native && n > 8) {
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
                if (!native) {
                    L.stream[rec + 2 * lane + 1] = ctl;
                } else {
                    // per lane: n - (block's first row, relative to the row group) + 64 for the block
                    // of each of its two entry quads (0 where the quad is padding: no stripe then
                    // passes the kernel's range test); bit 31 of lane l is bit l of the control word
                    auto tb = [&](size_t idx) {
                        return idx < st.n ? (uint32_t)((lane % 16) - entries[st.pos + idx].off + 64) : 0u;
                    };
                    const uint32_t bit = lane < 32 ? (ctl >> lane) & 1u : 0u;
                    L.stream[rec + 2 * lane + 1] = tb((size_t)(4 * g)) | (tb((size_t)(16 + 4 * g)) << 8) | (bit << 31);
                }
            }
            // weight fragments: lane (n = lane mod 16, g = lane / 16) holds row 16*j + n and, in
            // element order, entries 4g..4g+3 then 16+4g..16+4g+3 (the order the reads deliver)
            uint16_t *frag = reinterpret_cast<uint16_t *>(&L.stream[rec + 128]);
            if (native) {
                // one fragment for all stripes: lane (n, g) holds, for each of its 8 entries, the
                // weight of the block's row that is congruent to n modulo 16 (at most one: bh <= 16)
                for (int lane = 0; lane < 64 && st.n; ++lane) {
                    const int g = lane / 16, nrow = lane % 16;
                    for (int e = 0; e < 8; ++e) {
                        const size_t idx = (size_t)(e < 4 ? 4 * g + e : 16 + 4 * g + (e - 4));
                        if (idx >= st.n) continue;
                        uint16_t v = 0;
                        for (int j = 0; j < G; ++j) {
                            const uint16_t w = wbuf[(size_t)entries[st.pos + idx].slot * rgh + (kStripe * j + nrow)];
                            if (w) v = w;
                        }
                        frag[(size_t)lane * 8 + e] = v;
                    }
                }
                for (int j = 0; j < G; ++j)
                    if (mask & (1u << j)) {
                        ++L.total_mfma;
                        ++rg_weight[(size_t)rg];
                    }
            }
            for (int j = 0; j < G && !native; ++j) {
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
    L.sorted_steps.resize((size_t)L.nrg);
    for (int i = 0; i < L.nrg; ++i) {
        const int32_t rg = L.rg_order[(size_t)i];
        L.sorted_steps[(size_t)i] = L.rg_ptr[(size_t)rg + 1] - L.rg_ptr[(size_t)rg];
    }
}

// Operand tiles for the small-K kernel.  Element e of lane (n = lane mod 16, g = lane / 16) of
// tile (stripe, kt) is W[16*stripe + n][32*kt + i] with i = 4g + e for e < 4 and 16 + 4g + (e - 4)
// otherwise: the order in which two transposed LDS reads deliver 32 consecutive rows of X.
static void build_tiles(ubp_packed *p) {
    TileLayout &T = p->tiles;
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
                }
            }
        }
}

void build_stripe_layouts(ubp_packed *p) {
    build_tiles(p);
    if ((p->K + kSlotRows - 1) / kSlotRows > 0xffff) return; // chunk indices are 16-bit in the records
    for (int s = 0; s < kNumLayouts; ++s) build_one(p, p->sg[s], slot_G(s), slot_CT(s), false);
    // block-native layouts: a block must fit one 16-row operand (bh <= 16), whole blocks must tile
    // the 32 entries of a step and the 4 entries of a lane's quad (bw = 4, 8, 16 or 32); with one
    // stripe per wavefront there is nothing to share
    const bool eligible = p->bh <= kStripe && (p->bw == 4 || p->bw == 8 || p->bw == 16 || p->bw == 32);
    for (int s = 0; s < kNumLayouts; ++s)
        if (eligible && slot_G(s) > 1) build_one(p, p->sgn[s], slot_G(s), slot_CT(s), true);
}

} // namespace ubp
