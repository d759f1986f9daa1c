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
    case 9: return (p->nb * p->bh * p->bw + 511) / 512;
    default: break;
    }
    std::lock_guard<std::mutex> hold(p->lock);
    if (what == 8) return p->device_bytes;
    if (p->dtype == UBP_F32) return -1;
    if (what == 10 || what == 11) {
        const ubp::TileLayout &T = ubp::get_tile_layout(p);
        if (T.kt_pad == 0) return -1;
        return what == 10 ? T.tiles_nonzero : (int64_t)T.nstripes * ((p->K + ubp::kStep - 1) / ubp::kStep);
    }
    if (what >= 100 && what < 100 + ubp::kNumLayouts) {
        const ubp::StripeLayout &L = ubp::get_stripe_layout(p, ubp::slot_G(what - 100), ubp::slot_CT(what - 100));
        return L.G ? L.total_mfma : -1;
    }
    if (what >= 200 && what < 200 + ubp::kNumLayouts) {
        const ubp::StripeLayout &L = ubp::get_stripe_layout(p, ubp::slot_G(what - 200), ubp::slot_CT(what - 200));
        return L.G ? L.nsteps : -1;
    }
    if (what >= 300 && what < 312) {
        static const int kG[3] = {2, 4, 5};
        const int G = kG[(what - 300) % 3], item = (what - 300) / 3;
        if (!ubp::blk_eligible(p)) return -1;
        const ubp::BlkLayout &L = ubp::get_blk_layout(p, G);
        if (L.G == 0) return -1;
        return item == 0 ? L.total_mfma : item == 1 ? L.nsteps : item == 2 ? L.halves : L.paired;
    }
    return -1;
}

ubp_status ubp_packed_layout(const ubp_packed *p, int32_t sub_stripes, int32_t col_tiles, int32_t which,
                             int32_t *row_groups, const int32_t **rg_ptr, const int32_t **rg_order,
                             const uint32_t **stream, int64_t *stream_words, const uint32_t **meta, int64_t *meta_words) {
    if (!p || which < 1 || which > 3) return UBP_ERR_INVALID_ARG;
    if (p->dtype == UBP_F32) return UBP_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> hold(p->lock);
    if (meta) *meta = nullptr;
    if (meta_words) *meta_words = 0;
    if (which == 3) {
        // the dense operand tiles: row_groups = stripes, stream = the tiles as 32-bit words
        const ubp::TileLayout &T = ubp::get_tile_layout(p);
        if (T.kt_pad == 0) return UBP_ERR_UNSUPPORTED;
        if (row_groups) *row_groups = T.nstripes;
        if (rg_ptr) *rg_ptr = nullptr;
        if (rg_order) *rg_order = nullptr;
        if (stream) *stream = reinterpret_cast<const uint32_t *>(T.frags.data());
        if (stream_words) *stream_words = (int64_t)(T.frags.size() / 2);
        if (meta) *meta = T.occupied.data();
        if (meta_words) *meta_words = (int64_t)T.occupied.size();
        return UBP_OK;
    }
    if (which == 2) {
        if (ubp::blk_slot(sub_stripes) < 0) return UBP_ERR_INVALID_ARG;
        if (!ubp::blk_eligible(p)) return UBP_ERR_UNSUPPORTED;
        const ubp::BlkLayout &L = ubp::get_blk_layout(p, sub_stripes);
        if (L.G == 0) return UBP_ERR_UNSUPPORTED;
        if (row_groups) *row_groups = L.nrg;
        if (rg_ptr) *rg_ptr = L.rg_ptr.data();
        if (rg_order) *rg_order = L.rg_order.data();
        if (stream) *stream = L.frags.data();
        if (stream_words) *stream_words = (int64_t)L.frags.size();
        if (meta) *meta = L.meta.data();
        if (meta_words) *meta_words = (int64_t)L.meta.size();
        return UBP_OK;
    }
    const int slot = ubp::layout_slot(sub_stripes, col_tiles);
    if (slot < 0) return UBP_ERR_INVALID_ARG;
    const ubp::StripeLayout &L = ubp::get_stripe_layout(p, sub_stripes, col_tiles);
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
