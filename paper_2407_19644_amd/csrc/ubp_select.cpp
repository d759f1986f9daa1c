// Block selection on the host: which m of a layer's b candidate blocks are kept (Sections 3.1,
// 3.2 and 4.1).  Scores (Eq. 1), the greedy selector (Eq. 3), the optimal selector (Eq. 4),
// block expansion and division (Algorithms 1 and 2) and the efficacy figure (Eq. 5).
//
// The selectors return what the paper's step-by-step descriptions return, but not by those
// steps where a faster route gives the same indices:
//   greedy   : one sort by (score descending, index ascending) and one walk that skips
//              candidates a kept neighbour has shut out -- the same sequence as taking the arg max
//              m times, in O(b log b);
//   expansion: the shrinking score list is a doubly linked list over the original indices and the
//              arg max comes from a tournament tree (leftmost leaf wins a tie), so one of the m
//              rounds costs O(N log b) instead of O(b);
//   optimal  : Eq. 4's table row by row with one decision bit per cell and a walk back from
//              (b, m) instead of carrying index sets, cells that cannot lie on a path to (b, m)
//              left out: O(b m) time, b m bits.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <limits>
#include <new>
#include <numeric>
#include <vector>

#include "ubp.h"

namespace {

constexpr double kNegInf = -std::numeric_limits<double>::infinity();

inline double half_bits_to_double(uint16_t h) {
    const int sign = h >> 15, exp = (h >> 10) & 31, man = h & 1023;
    double v;
    if (exp == 0) v = std::ldexp((double)man, -24);
    else if (exp == 31) v = man ? std::numeric_limits<double>::quiet_NaN() : std::numeric_limits<double>::infinity();
    else v = std::ldexp((double)(man | 1024), exp - 25);
    return sign ? -v : v;
}

inline double bf16_bits_to_double(uint16_t h) {
    const uint32_t u = (uint32_t)h << 16;
    float f;
    std::memcpy(&f, &u, 4);
    return (double)f;
}

inline double element(const void *W, ubp_dtype dtype, int64_t at) {
    switch (dtype) {
    case UBP_F32: return (double)static_cast<const float *>(W)[at];
    case UBP_F16: return half_bits_to_double(static_cast<const uint16_t *>(W)[at]);
    default: return bf16_bits_to_double(static_cast<const uint16_t *>(W)[at]);
    }
}

bool layer_ok(const void *W, ubp_dtype dtype, int64_t ldw, int32_t M, int32_t K, int32_t bh, int32_t bw) {
    return W && (dtype == UBP_F32 || dtype == UBP_F16 || dtype == UBP_BF16) && M >= 1 && K >= 1 && bh >= 1 && bw >= 1 &&
           bh <= M && bw <= K && ldw >= K;
}

// scores may be finite or -inf; anything else (NaN, +inf) has no order the selectors could use
bool scores_ok(const double *S, int64_t b) {
    for (int64_t k = 0; k < b; ++k)
        if (!(S[k] == kNegInf || std::isfinite(S[k]))) return false;
    return true;
}

bool selector_args_ok(const double *S, int64_t b, int32_t N, int64_t m, const int64_t *I, const int64_t *count) {
    return b >= 0 && (b == 0 || S) && N >= 1 && m >= 0 && (m == 0 || I) && count;
}

// leftmost-max tournament tree over b leaves
struct Tournament {
    int64_t leaves = 1;
    std::vector<int64_t> win;          // node -> index of its best leaf, -1 for an empty subtree
    const double *S;
    Tournament(const double *scores, int64_t b) : S(scores) {
        while (leaves < b) leaves <<= 1;
        win.assign((size_t)(2 * leaves), -1);
        for (int64_t k = 0; k < b; ++k) win[(size_t)(leaves + k)] = k;
        for (int64_t v = leaves - 1; v >= 1; --v) win[(size_t)v] = better(win[(size_t)(2 * v)], win[(size_t)(2 * v + 1)]);
    }
    int64_t better(int64_t l, int64_t r) const {
        if (l < 0) return r;
        if (r < 0) return l;
        return S[r] > S[l] ? r : l;
    }
    void refresh(int64_t k, bool present) {
        int64_t v = leaves + k;
        win[(size_t)v] = present ? k : -1;
        for (v >>= 1; v >= 1; v >>= 1) win[(size_t)v] = better(win[(size_t)(2 * v)], win[(size_t)(2 * v + 1)]);
    }
    int64_t best() const { return win[1]; }
};

}  // namespace

extern "C" {

ubp_status ubp_block_scores(const void *W, ubp_dtype dtype, int64_t ldw, int32_t M, int32_t K, int32_t bh, int32_t bw,
                            int32_t aligned, double *S, int64_t b) {
    if (!layer_ok(W, dtype, ldw, M, K, bh, bw) || !S || b != (int64_t)M * (K / bw)) return UBP_ERR_INVALID_ARG;
    const int32_t groups = K / bw;
    std::vector<double> row((size_t)M);
    for (int32_t j = 0; j < groups; ++j) {
        for (int32_t i = 0; i < M; ++i) {                       // l1 norm of one row's bw weights
            double s = 0.0;
            for (int32_t q = 0; q < bw; ++q) s += std::fabs(element(W, dtype, (int64_t)i * ldw + (int64_t)j * bw + q));
            row[(size_t)i] = s;
        }
        double *out = S + (int64_t)j * M;
        for (int32_t i = 0; i < M; ++i) {
            if (i + bh > M || (aligned && i % bh)) { out[i] = kNegInf; continue; }
            double s = 0.0;
            for (int32_t t = 0; t < bh; ++t) s += row[(size_t)(i + t)];
            out[i] = s;
        }
    }
    return UBP_OK;
}

ubp_status ubp_select_greedy(const double *S, int64_t b, int32_t N, int64_t m, int64_t *I, int64_t *count) {
    if (!selector_args_ok(S, b, N, m, I, count)) return UBP_ERR_INVALID_ARG;
    *count = 0;
    if (!scores_ok(S, b)) return UBP_ERR_INVALID_ARG;
    try {
        std::vector<int64_t> order;
        order.reserve((size_t)b);
        for (int64_t k = 0; k < b; ++k)
            if (S[k] > kNegInf) order.push_back(k);
        std::sort(order.begin(), order.end(), [S](int64_t x, int64_t y) { return S[x] > S[y] || (S[x] == S[y] && x < y); });
        std::vector<unsigned char> shut((size_t)b, 0);
        int64_t got = 0;
        for (size_t at = 0; at < order.size() && got < m; ++at) {
            const int64_t k = order[at];
            if (shut[(size_t)k]) continue;
            I[got++] = k;
            const int64_t lo = std::max<int64_t>(0, k - N + 1), hi = std::min<int64_t>(b - 1, k + N - 1);
            std::memset(&shut[(size_t)lo], 1, (size_t)(hi - lo + 1));
        }
        *count = got;
    } catch (const std::bad_alloc &) {
        return UBP_ERR_ALLOC;
    }
    return UBP_OK;
}

ubp_status ubp_select_bed(const double *S_in, int64_t b, int32_t N, int64_t m, int64_t *I, int64_t *count) {
    if (!selector_args_ok(S_in, b, N, m, I, count)) return UBP_ERR_INVALID_ARG;
    *count = 0;
    if (!scores_ok(S_in, b)) return UBP_ERR_INVALID_ARG;
    if (b == 0 || m == 0) return UBP_OK;
    try {
        // ---- expansion (Algorithm 1)
        std::vector<double> S(S_in, S_in + b);
        std::vector<int64_t> prev((size_t)b), next((size_t)b), right((size_t)N);
        for (int64_t k = 0; k < b; ++k) { prev[(size_t)k] = k - 1; next[(size_t)k] = k + 1 < b ? k + 1 : -1; }
        Tournament tree(S.data(), b);
        int64_t got = 0;
        while (got < m) {
            const int64_t k = tree.best();
            if (k < 0 || S[(size_t)k] == kNegInf) break;
            // right[t] = the t-th entry after k in the list as it stands, -1 past its end
            right[0] = k;
            for (int32_t t = 1; t < N; ++t) right[(size_t)t] = right[(size_t)(t - 1)] < 0 ? -1 : next[(size_t)right[(size_t)(t - 1)]];
            // the entry n places before k becomes the block made of the n weights before k's block
            // and the N-n weights after it
            int64_t left = k;
            for (int32_t n = 1; n < N; ++n) {
                left = prev[(size_t)left];
                if (left < 0) break;
                const int64_t r = right[(size_t)(N - n)];
                const double joined = r < 0 ? kNegInf : S[(size_t)r];
                S[(size_t)left] = S[(size_t)left] + joined - S[(size_t)k];
                tree.refresh(left, true);
            }
            // k and the N-1 entries after it leave the list
            const int64_t before = prev[(size_t)k];
            int64_t last = k;
            for (int32_t t = 0; t < N && right[(size_t)t] >= 0; ++t) {
                last = right[(size_t)t];
                tree.refresh(last, false);
            }
            const int64_t after = next[(size_t)last];
            if (before >= 0) next[(size_t)before] = after;
            if (after >= 0) prev[(size_t)after] = before;
            I[got++] = k;
        }
        // ---- division (Algorithm 2)
        std::sort(I, I + got);
        int64_t next_idx = 0;
        for (int64_t at = 0; at < got; ++at) {
            const int64_t k = I[at];
            if (next_idx > k) { I[at] = next_idx; next_idx += N; }
            else { next_idx = k + N; }
        }
        *count = got;
    } catch (const std::bad_alloc &) {
        return UBP_ERR_ALLOC;
    }
    return UBP_OK;
}

ubp_status ubp_select_optimal(const double *S, int64_t b, int32_t N, int64_t m, int64_t *I, int64_t *count) {
    if (!selector_args_ok(S, b, N, m, I, count)) return UBP_ERR_INVALID_ARG;
    *count = 0;
    if (!scores_ok(S, b)) return UBP_ERR_INVALID_ARG;
    if (m == 0) return UBP_OK;
    if (m > (b + N - 1) / N) return UBP_ERR_INFEASIBLE;
    const int64_t words = (m + 63) / 64;
    if ((long double)b * (long double)words * 8.0L > 2147483648.0L) return UBP_ERR_UNSUPPORTED;   // decision bits above 2 GiB
    try {
        std::vector<uint64_t> took((size_t)(b * words), 0);
        // rows k-N .. k of T, row k at slot k mod (N+1); T[k][0] = 0, T[<=0][n>0] = -inf
        const int64_t ring = (int64_t)N + 1;
        std::vector<double> T((size_t)(ring * (m + 1)), kNegInf);
        for (int64_t r = 0; r < ring; ++r) T[(size_t)(r * (m + 1))] = 0.0;
        for (int64_t k = 1; k <= b; ++k) {
            double *cur = &T[(size_t)((k % ring) * (m + 1))];
            const double *skip_row = &T[(size_t)(((k - 1) % ring) * (m + 1))];
            const double *take_row = k - N >= 1 ? &T[(size_t)(((k - N) % ring) * (m + 1))] : nullptr;
            // cells that can lie on a path to (b, m): n <= ceil(k / N) blocks fit before k, and the
            // m - n still missing must fit into the b - k candidates after it
            const int64_t n_hi = std::min<int64_t>(m, (k + N - 1) / N);
            const int64_t n_lo = std::max<int64_t>(1, m - (b - k + N - 1) / N);
            const double s = S[k - 1];
            uint64_t *bits = &took[(size_t)((k - 1) * words)];
            for (int64_t n = n_lo; n <= n_hi; ++n) {
                const double before = take_row ? take_row[n - 1] : (n == 1 ? 0.0 : kNegInf);
                const double take = before + s, skip = k > 1 ? skip_row[n] : kNegInf;
                if (take > skip) { cur[n] = take; bits[(n - 1) >> 6] |= 1ull << ((n - 1) & 63); }
                else cur[n] = skip;
            }
            if (n_hi < m) cur[n_hi + 1] = kNegInf;      // the one cell above the band that row k+1 reads
        }
        if (T[(size_t)((b % ring) * (m + 1) + m)] == kNegInf) return UBP_ERR_INFEASIBLE;
        int64_t k = b, n = m;
        while (n > 0 && k > 0) {
            if (took[(size_t)((k - 1) * words + ((n - 1) >> 6))] >> ((n - 1) & 63) & 1) { I[--n] = k - 1; k -= N; }
            else --k;
        }
        if (n != 0) return UBP_ERR_INFEASIBLE;
        *count = m;
    } catch (const std::bad_alloc &) {
        return UBP_ERR_ALLOC;
    }
    return UBP_OK;
}

ubp_status ubp_selection_to_blocks(const int64_t *I, int64_t count, int32_t M, int32_t bw, ubp_block *blocks) {
    if (count < 0 || (count > 0 && (!I || !blocks)) || M < 1 || bw < 1) return UBP_ERR_INVALID_ARG;
    for (int64_t at = 0; at < count; ++at) {
        if (I[at] < 0 || I[at] / M > std::numeric_limits<int32_t>::max() / bw) return UBP_ERR_INVALID_ARG;
        blocks[at].r = (int32_t)(I[at] % M);
        blocks[at].c = (int32_t)(I[at] / M) * bw;
    }
    return UBP_OK;
}

ubp_status ubp_select_blocks(const void *W, ubp_dtype dtype, int64_t ldw, int32_t M, int32_t K, int32_t bh, int32_t bw,
                             double density, int32_t method, int32_t aligned, ubp_block *out, int64_t capacity,
                             int64_t *out_nb) {
    if (!layer_ok(W, dtype, ldw, M, K, bh, bw) || !out_nb || method < 0 || method > 2) return UBP_ERR_INVALID_ARG;
    *out_nb = 0;
    const int64_t m = ubp_target_block_count(M, K, bh, bw, density);
    if (m < 0) return UBP_ERR_INVALID_ARG;
    if (capacity < m || (m > 0 && !out)) { *out_nb = m; return UBP_ERR_INVALID_ARG; }
    try {
        const int64_t b = (int64_t)M * (K / bw);
        std::vector<double> S((size_t)b);
        std::vector<int64_t> I((size_t)std::max<int64_t>(m, 1));
        ubp_status rc = ubp_block_scores(W, dtype, ldw, M, K, bh, bw, aligned, S.data(), b);
        if (rc != UBP_OK) return rc;
        int64_t got = 0;
        rc = method == 0 ? ubp_select_greedy(S.data(), b, bh, m, I.data(), &got)
           : method == 1 ? ubp_select_bed(S.data(), b, bh, m, I.data(), &got)
                         : ubp_select_optimal(S.data(), b, bh, m, I.data(), &got);
        if (rc != UBP_OK) return rc;
        rc = ubp_selection_to_blocks(I.data(), got, M, bw, out);
        if (rc != UBP_OK) return rc;
        *out_nb = got;
    } catch (const std::bad_alloc &) {
        return UBP_ERR_ALLOC;
    }
    return UBP_OK;
}

ubp_status ubp_selection_efficacy(const void *W, ubp_dtype dtype, int64_t ldw, int32_t M, int32_t K, int32_t bh, int32_t bw,
                                  const ubp_block *ubp_blocks, int64_t nb, const ubp_block *abp_blocks, int64_t nb_abp,
                                  double *l1, double *efficacy) {
    if (!layer_ok(W, dtype, ldw, M, K, bh, bw) || nb < 0 || nb_abp < 0 || (nb && !ubp_blocks) || (nb_abp && !abp_blocks) ||
        !efficacy)
        return UBP_ERR_INVALID_ARG;
    try {
        auto kept = [&](const ubp_block *blocks, int64_t count, double *sum) -> ubp_status {
            std::vector<unsigned char> mark((size_t)M * (size_t)K, 0);
            for (int64_t at = 0; at < count; ++at) {
                const ubp_block o = blocks[at];
                if (o.r < 0 || o.c < 0 || o.r + bh > M || o.c + bw > K) return UBP_ERR_OUT_OF_BOUNDS;
                for (int32_t t = 0; t < bh; ++t)
                    std::memset(&mark[(size_t)(o.r + t) * K + o.c], 1, (size_t)bw);
            }
            double s = 0.0;
            for (int32_t i = 0; i < M; ++i)
                for (int32_t c = 0; c < K; ++c)
                    if (mark[(size_t)i * K + c]) s += std::fabs(element(W, dtype, (int64_t)i * ldw + c));
            *sum = s;
            return UBP_OK;
        };
        double ubp = 0.0, abp = 0.0, ep = 0.0;
        ubp_status rc = kept(ubp_blocks, nb, &ubp);
        if (rc != UBP_OK) return rc;
        rc = kept(abp_blocks, nb_abp, &abp);
        if (rc != UBP_OK) return rc;
        // element-wise pruning keeps as many weights as the unaligned selection, the largest ones
        std::vector<double> mags((size_t)M * (size_t)K);
        for (int32_t i = 0; i < M; ++i)
            for (int32_t c = 0; c < K; ++c) mags[(size_t)i * K + c] = std::fabs(element(W, dtype, (int64_t)i * ldw + c));
        const size_t keep = (size_t)std::min<int64_t>((int64_t)mags.size(), nb * bh * bw);
        std::partial_sort(mags.begin(), mags.begin() + (std::ptrdiff_t)keep, mags.end(), std::greater<double>());
        for (size_t at = 0; at < keep; ++at) ep += mags[at];
        if (l1) { l1[0] = ubp; l1[1] = abp; l1[2] = ep; }
        *efficacy = (ubp - abp) / (ep - abp);
    } catch (const std::bad_alloc &) {
        return UBP_ERR_ALLOC;
    }
    return UBP_OK;
}

}  // extern "C"
