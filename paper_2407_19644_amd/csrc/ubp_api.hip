// Device-facing entry points of the UBP library: upload of the packed weights and of the
// kernels' private layouts, the choice of kernel and launch shape, the C ABI around them.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <vector>

#include "ubp_internal.h"

namespace ubp {

struct DeviceGuard {
    int prev = -1;
    bool ok = true;
    explicit DeviceGuard(int dev) {
        if (hipGetDevice(&prev) != hipSuccess) { ok = false; prev = -1; }
        else if (prev != dev && hipSetDevice(dev) != hipSuccess) { ok = false; prev = -1; }
        if (!ok) (void)hipGetLastError(); // do not leave a sticky error for the caller's next HIP call
    }
    ~DeviceGuard() {
        if (prev >= 0) (void)hipSetDevice(prev);
    }
};

namespace {

template <class T>
bool dev_copy(T **dst, const T *src, size_t n, int64_t *bytes) {
    const size_t sz = std::max<size_t>(n, 1) * sizeof(T);
    if (hipMalloc(reinterpret_cast<void **>(dst), sz) != hipSuccess) { *dst = nullptr; return false; }
    *bytes += (int64_t)sz;
    if (n && hipMemcpy(*dst, src, n * sizeof(T), hipMemcpyHostToDevice) != hipSuccess) return false;
    return true;
}

template <class T>
bool dev_copy_vec(T **dst, const std::vector<T> &v, int64_t *bytes) { return dev_copy(dst, v.data(), v.size(), bytes); }

} // namespace

// ------------------------------------------------------------------ upload / release
ubp_status upload(ubp_packed *p) {
    int count = 0;
    if (hipGetDeviceCount(&count) != hipSuccess || p->device >= count) {
        (void)hipGetLastError();
        p->device = UBP_HOST_ONLY; // nothing was allocated; nothing to release
        return UBP_ERR_DEVICE;
    }
    DeviceGuard guard(p->device);
    if (!guard.ok) {
        p->device = UBP_HOST_ONLY;
        return UBP_ERR_DEVICE;
    }
    bool ok = true;
    ok = ok && dev_copy(&p->d_indptr, p->indptr.data(), p->indptr.size(), &p->device_bytes);
    ok = ok && dev_copy(&p->d_indices, p->indices.data(), p->indices.size(), &p->device_bytes);
    {
        const uint32_t zero = 0;
        ok = ok && dev_copy(&p->d_error, &zero, 1, &p->device_bytes);
    }
    if (!ok) {
        (void)hipGetLastError();
        return UBP_ERR_ALLOC;
    }
    return UBP_OK;
}

// (the functions below run with p->lock held and the handle's device current)
ubp_status upload_values_f32(const ubp_packed *p) {
    if (p->d_values_f32) return UBP_OK;
    // rotated values widened to fp32 (exact for fp16 and bf16) for the vector kernel
    const int64_t n = p->nb * p->bw * p->bh;
    std::vector<float> f((size_t)n);
    if (p->dtype == UBP_F32) {
        if (n) std::memcpy(f.data(), p->values.data(), (size_t)n * 4);
    } else {
        const uint16_t *h = reinterpret_cast<const uint16_t *>(p->values.data());
        for (int64_t t = 0; t < n; ++t) {
            if (p->dtype == UBP_BF16) {
                const uint32_t u = (uint32_t)h[t] << 16;
                std::memcpy(&f[(size_t)t], &u, 4);
            } else {
                _Float16 hv;
                std::memcpy(&hv, &h[t], 2);
                f[(size_t)t] = (float)hv;
            }
        }
    }
    if (!dev_copy(&p->d_values_f32, f.data(), f.size(), &p->device_bytes)) {
        (void)hipGetLastError();
        return UBP_ERR_ALLOC;
    }
    return UBP_OK;
}

ubp_status upload_stripe_layout(const ubp_packed *p, int slot) {
    StripeLayoutDev &D = p->d_sg[slot];
    if (D.uploaded) return UBP_OK;
    const StripeLayout &L = p->sg[slot];
    bool ok = dev_copy_vec(&D.rg_ptr, L.rg_ptr, &p->device_bytes) && dev_copy_vec(&D.rg_order, L.rg_order, &p->device_bytes) &&
              dev_copy_vec(&D.stream, L.stream, &p->device_bytes);
    if (!ok) {
        (void)hipGetLastError();
        return UBP_ERR_ALLOC;
    }
    D.uploaded = true;
    return UBP_OK;
}

ubp_status upload_blk_layout(const ubp_packed *p, int slot) {
    BlkLayoutDev &D = p->d_blk[slot];
    if (D.uploaded) return UBP_OK;
    const BlkLayout &L = p->blk[slot];
    bool ok = dev_copy_vec(&D.rg_ptr, L.rg_ptr, &p->device_bytes) && dev_copy_vec(&D.rg_order, L.rg_order, &p->device_bytes) &&
              dev_copy_vec(&D.meta, L.meta, &p->device_bytes) && dev_copy_vec(&D.frags, L.frags, &p->device_bytes);
    if (!ok) {
        (void)hipGetLastError();
        return UBP_ERR_ALLOC;
    }
    D.uploaded = true;
    return UBP_OK;
}

ubp_status upload_tile_layout(const ubp_packed *p) {
    TileLayoutDev &D = p->d_tiles;
    if (D.uploaded) return UBP_OK;
    const TileLayout &T = p->tiles;
    bool ok = dev_copy_vec(&D.frags, T.frags, &p->device_bytes) && dev_copy_vec(&D.occupied, T.occupied, &p->device_bytes);
    if (!ok) {
        (void)hipGetLastError();
        return UBP_ERR_ALLOC;
    }
    D.uploaded = true;
    return UBP_OK;
}

void release_device(ubp_packed *p) {
    if (!p || p->device == UBP_HOST_ONLY) return;
    DeviceGuard guard(p->device);
    if (!guard.ok) return;
    auto rel = [](auto *&ptr) {
        if (ptr) (void)hipFree(ptr);
        ptr = nullptr;
    };
    rel(p->d_indptr);
    rel(p->d_indices);
    rel(p->d_values_f32);
    rel(p->d_error);
    rel(p->d_tiles.frags);
    rel(p->d_tiles.occupied);
    for (int s = 0; s < kNumLayouts; ++s) {
        rel(p->d_sg[s].rg_ptr);
        rel(p->d_sg[s].rg_order);
        rel(p->d_sg[s].stream);
    }
    for (int s = 0; s < kNumBlkLayouts; ++s) {
        rel(p->d_blk[s].rg_ptr);
        rel(p->d_blk[s].rg_order);
        rel(p->d_blk[s].meta);
        rel(p->d_blk[s].frags);
    }
}


namespace {

// What a call resolves to: the kernel and its launch shape, every field set.
struct Shape {
    int kernel = 0;   // 1 vector, 2 gather, 4 small-K dense tiles, 5 chunked dense tiles, 6 block, 7 dense tiles through LDS
    int shape = 0;    // kernel 7: tile shape
    int G = 0, CT = 0, waves = 0, NP = 0, wg_rows = 0, rpr = 0;
    bool resident = false;
};

// Decides kernel and shape for (handle, N, alignment) and the caller's pins; builds the host image
// of the layout that shape needs (under the handle's lock).  No device work.
ubp_status resolve(const ubp_packed *p, int N, int64_t ldx_bytes, bool vec_ok, const ubp_plan &pl, Shape &s) {
    int kernel = pl.kernel;
    // the dense-tile kernels need 16-byte pieces of X rows that lie entirely inside or outside the matrix
    const bool tile_able = p->dtype != UBP_F32 && vec_ok && N % 8 == 0;
    if (kernel == 0) {
        if (p->dtype == UBP_F32) {
            kernel = 1;
        } else {
            // Whole blocks as operands where a block fills one (16-row blocks at least 16 wide) and K is
            // beyond what the ring holds at once.  Dense zero-filled tiles where most 16 x 32 tiles hold
            // a kept weight anyway (at least half of them, which small blocks reach from about a tenth
            // of the weights kept): the matrix instructions issued then stay within about twice those a
            // gather issues, and no row of X is gathered.  Otherwise gathered rows.
            const bool blk_auto = blk_eligible(p) && p->bh == kStripe && p->bw >= 16 && p->K > ring_rows(4) && vec_ok && N >= 64;
            if (blk_auto) {
                kernel = 6;
            } else if (tile_able) {
                const TileLayout &T = get_tile_layout(p);
                const int kt = (p->K + kStep - 1) / kStep;
                const bool mostly_full = T.kt_pad != 0 && 2 * T.tiles_nonzero >= (int64_t)T.nstripes * kt;
                // Among the dense-tile kernels: where every tile keeps a weight, the one that stages both
                // operands in LDS for small K or few pixels (there a weight tile fetched once per 64 pixels
                // is what costs: 4.3 against 5.3 us and 11.8 against 13.8 us on two such layers); else
                // the small-K kernel or the chunked one, which skip empty tiles.
                const bool all_full = T.kt_pad != 0 && T.tiles_nonzero == (int64_t)T.nstripes * kt;
                if (all_full && (p->K <= kTileMaxK || N <= 4096) && (int64_t)p->K * ldx_bytes < (int64_t(1) << 31)) kernel = 7;
                else if (mostly_full && p->K <= kTileMaxK) kernel = 4;
                else if (mostly_full && T.kt_pad % 4 == 0) kernel = 5;
                else kernel = 2;
            } else {
                kernel = 2;
            }
        }
    }
    if (kernel < 1 || kernel > 7) return UBP_ERR_INVALID_ARG;
    if (kernel != 1 && kernel != 3 && p->dtype == UBP_F32) return UBP_ERR_UNSUPPORTED;
    s.kernel = kernel;
    if (kernel == 1 || kernel == 3) {
        if (p->bh > 16) return UBP_ERR_UNSUPPORTED;
        int rpr = pl.rows_per_range;
        if (rpr == 0) {
            // enough row ranges to fill the chip, but each at least 4 block heights tall so
            // that re-walking bh-1 start rows stays a small fraction of the work
            const int coltiles = (N + 255) / 256;
            int ranges = std::max(1, 2048 / std::max(1, coltiles));
            rpr = std::max(4 * p->bh, (p->M + ranges - 1) / ranges);
            rpr = ((rpr + p->bh - 1) / p->bh) * p->bh;
        }
        if (rpr < 1) return UBP_ERR_INVALID_ARG;
        if ((p->M + rpr - 1) / rpr > 65535) rpr = (p->M + 65534) / 65535; // grid.y limit
        s.rpr = rpr;
        return UBP_OK;
    }
    if (kernel == 7) {
        if (!tile_able) return UBP_ERR_UNSUPPORTED;
        const TileLayout &T = get_tile_layout(p);
        if (T.kt_pad == 0) return UBP_ERR_UNSUPPORTED;
        // this kernel multiplies every tile: only for matrices whose every tile keeps a weight
        if (T.tiles_nonzero != (int64_t)T.nstripes * ((p->K + kStep - 1) / kStep)) return UBP_ERR_UNSUPPORTED;
        int best = -1;
        int64_t best_score = -1;
        for (int sh = 0; sh < kNumGemmShapes; ++sh) {
            int rows, px;
            gemm_shape(sh, &rows, &px);
            if (pl.sub_stripes && pl.sub_stripes * 16 != rows) continue;
            if (pl.col_tiles && pl.col_tiles * 16 != px) continue;
            // the largest tile that still gives about one workgroup per CU; else the most workgroups
            const int64_t wgs = (int64_t)((p->M + rows - 1) / rows) * ((N + px - 1) / px);
            const int64_t score = wgs >= 190 ? ((int64_t)1 << 40) + (int64_t)rows * px : wgs;
            if (score > best_score) {
                best_score = score;
                best = sh;
            }
        }
        if (best < 0) return UBP_ERR_UNSUPPORTED;
        int rows, px;
        gemm_shape(best, &rows, &px);
        s.shape = best;
        s.G = rows / 16;
        s.CT = px / 16;
        s.wg_rows = (p->M + rows - 1) / rows;
        s.waves = rows * px >= 128 * 256 ? 8 : 4;
        return UBP_OK;
    }
    if (kernel == 4 || kernel == 5) {
        if (!tile_able) return UBP_ERR_UNSUPPORTED;
        const TileLayout &T = get_tile_layout(p);
        if (T.kt_pad == 0) return UBP_ERR_UNSUPPORTED;
        if (kernel == 4 && p->K > kTileMaxK) return UBP_ERR_UNSUPPORTED;
        if (kernel == 5 && T.kt_pad % 4 != 0) return UBP_ERR_UNSUPPORTED;
        int CT = pl.col_tiles;
        // 64-pixel blocks halve the weight traffic per pixel; 32-pixel blocks where those would be few
        if (CT == 0) CT = kernel == 5 ? 4 : (N >= 128 * 64 ? 4 : 2);
        if (CT != 2 && CT != 4) return UBP_ERR_UNSUPPORTED;
        s.CT = CT;
        const int n_blocks = (N + 16 * CT - 1) / (16 * CT);
        int slices = pl.wg_rows;
        if (slices < 0) return UBP_ERR_INVALID_ARG;
        if (kernel == 5) {
            if (pl.waves != 0) return UBP_ERR_UNSUPPORTED; // fixed: 16 stripes' worth of multiplying wavefronts + 4 that load X
            // a workgroup's multiplying wavefronts hold 16 stripes: slices of at most 16 stripes
            // (more slices on request: each streams all of the block's X again)
            const int least = (T.nstripes + 15) / 16;
            // Fewer workgroups than half the CUs: twice the slices, and two stripes per wavefront so
            // that a workgroup still has 4 multiplying wavefronts (measured: 21 against 27 us on a
            // 256 x 2304 layer with 6272 pixels, 12.8 against 15.1 us on 1024 x 1024 with 1568)
            const bool few = slices == 0 && pl.sub_stripes == 0 && (int64_t)n_blocks * least < 128 && T.nstripes >= 2 * least * 2;
            slices = std::min(std::max(few ? 2 * least : slices, least), T.nstripes);
            s.G = pl.sub_stripes ? pl.sub_stripes : (few ? 2 : 4); // stripes per multiplying wavefront
            if (s.G != 2 && s.G != 4) return UBP_ERR_UNSUPPORTED;
        } else {
            // Workgroups of 4 wavefronts, about one and a half per CU: two share a CU and the one's
            // loading of X overlaps the other's streaming (measured better than one workgroup of 8).
            // The stripes are cut into slices to get there - every slice loads the X block again, so
            // only while a wavefront keeps at least 3 stripes.
            if (slices == 0) slices = std::max(1, std::min((int)std::lround(384.0 / n_blocks), T.nstripes / 12));
            slices = std::min(slices, T.nstripes);
        }
        const int sps = (T.nstripes + slices - 1) / slices;
        slices = (T.nstripes + sps - 1) / sps;
        if ((int64_t)n_blocks * slices > 0x7fffffff) return UBP_ERR_UNSUPPORTED;
        s.wg_rows = slices;
        if (kernel == 4) {
            s.waves = pl.waves ? pl.waves : std::min(4, sps);
            if (s.waves < 1 || s.waves > 8) return UBP_ERR_UNSUPPORTED;
        }
        return UBP_OK;
    }
    if (kernel == 6) {
        if (!blk_eligible(p) || !vec_ok || N < 64) return UBP_ERR_UNSUPPORTED;
        if (pl.col_tiles != 0 && pl.col_tiles != 4) return UBP_ERR_UNSUPPORTED;
        // 4 stripes per wavefront, or 5 (which just fits the registers) where that saves a workgroup
        // row: X is staged once per workgroup row
        int G = pl.sub_stripes;
        if (G == 0) {
            auto rows_for = [&](int g) { return ((p->M + 16 * g - 1) / (16 * g) + 13) / 14; };
            G = rows_for(5) < rows_for(4) ? 5 : 4;
        }
        if (G != 2 && G != 4 && G != 5) return UBP_ERR_UNSUPPORTED;
        const BlkLayout &L = get_blk_layout(p, G);
        if (L.G == 0) return UBP_ERR_UNSUPPORTED;
        int NP = pl.producers;
        if (NP != 0 && NP != 1 && NP != 2 && NP != 4) return UBP_ERR_UNSUPPORTED;
        int waves = pl.waves;
        // one wavefront stages about 28 GB/s: a second one as soon as a workgroup's tile is not small
        if (NP == 0) {
            NP = ((int64_t)p->K * 32 * 4 >= 64 * 1024) ? 2 : 1;
            if (waves != 0 && waves < NP + 1) NP = 1;
        }
        const int max_waves = blk_max_waves(G);
        if (waves == 0) {
            // as few workgroup rows as the wavefront limit allows; full workgroups if the last row is
            // then still at least half full, else the consumers spread evenly over the rows
            const int maxc = max_waves - NP;
            const int rows_wg = (L.nrg + maxc - 1) / maxc;
            const int last = L.nrg - (rows_wg - 1) * maxc;
            waves = (2 * last >= maxc ? maxc : (L.nrg + rows_wg - 1) / rows_wg) + NP;
        }
        if (waves < NP + 1 || waves > max_waves) return UBP_ERR_UNSUPPORTED;
        const int need_rows = (L.nrg + (waves - NP) - 1) / (waves - NP);
        if (pl.wg_rows != 0 && pl.wg_rows != need_rows) return UBP_ERR_UNSUPPORTED;
        s.G = G;
        s.CT = 4;
        s.NP = NP;
        s.waves = waves;
        s.wg_rows = need_rows;
        return UBP_OK;
    }

    // ---- gather kernel
    int CT = pl.col_tiles, G = pl.sub_stripes, waves = pl.waves, NP = pl.producers;
    if (NP != 0 && NP != 1 && NP != 2 && NP != 4) return UBP_ERR_UNSUPPORTED;
    if ((G != 0 && G != 1 && G != 2 && G != 4) || (CT != 0 && CT != 2 && CT != 4 && CT != 8)) return UBP_ERR_UNSUPPORTED;
    // Tile shape, from measurements on the benchmark layers.
    //  * Column tiles as wide as divides N (a ragged last tile takes the slow staging path),
    //    provided that still leaves a few dozen tiles: wide tiles amortise a step's fixed
    //    instruction cost over more matrix instructions.
    //  * Stripes per wavefront follow the block height: a 16-row block touches two stripes
    //    anyway, so tall row groups cost little extra zero fill and divide the staging of X by
    //    the rows a workgroup covers; for short blocks one stripe keeps the operands dense.
    if (CT == 0) {
        for (int ct = 8; ct >= 2 && CT == 0; ct /= 2)
            if (N % (16 * ct) == 0 && N / (16 * ct) >= 32) CT = ct;
        for (int ct = 8; ct >= 2 && CT == 0; ct /= 2)
            if ((N + 16 * ct - 1) / (16 * ct) >= 32) CT = ct;
        if (CT == 0) CT = 2;
    }
    if (G == 0) {
        G = p->bh >= 16 ? 4 : p->bh >= 8 ? 2 : 1;
        while (G > 1 && get_stripe_layout(p, G, CT).G == 0) G >>= 1;
    }
    const StripeLayout &L = get_stripe_layout(p, G, CT);
    if (L.G == 0) return UBP_ERR_UNSUPPORTED; // layout cannot be built for this matrix
    // one wavefront stages about 28 GB/s: a second one as soon as a workgroup's tile is not small
    if (NP == 0) {
        NP = ((int64_t)p->K * 32 * CT >= 64 * 1024) ? 2 : 1;
        if (waves != 0 && waves < NP + 1) NP = 1; // a caller who fixes a tiny workgroup gets one producer
    }
    const int max_waves = stripe_max_waves(G, CT);
    if (max_waves <= NP) return UBP_ERR_UNSUPPORTED;
    // When the ring holds all of K nothing is ever refilled and a consumer may walk several row
    // groups one after the other; the number of workgroup rows is then free.  Otherwise every
    // consumer owns exactly one row group.
    const bool resident = L.nch <= ring_slots(CT);
    int wg_rows = pl.wg_rows;
    if (wg_rows < 0) return UBP_ERR_INVALID_ARG;
    if (!resident) {
        if (waves == 0) {
            // as few workgroup rows as the wavefront limit allows; full workgroups if the last row is
            // then still at least half full (more consumers per CU measured better than even rows),
            // else the consumers spread evenly over the rows
            const int maxc = max_waves - NP;
            const int rows_wg = (L.nrg + maxc - 1) / maxc;
            const int last = L.nrg - (rows_wg - 1) * maxc;
            waves = (2 * last >= maxc ? maxc : (L.nrg + rows_wg - 1) / rows_wg) + NP; // consumers + producers
        }
        if (waves < NP + 1 || waves > max_waves) return UBP_ERR_UNSUPPORTED;
        const int need_rows = (L.nrg + (waves - NP) - 1) / (waves - NP);
        if (wg_rows != 0 && wg_rows != need_rows) return UBP_ERR_UNSUPPORTED;
        wg_rows = need_rows;
    } else {
        const int64_t ncol = (N + 16 * CT - 1) / (16 * CT);
        if (wg_rows == 0) {
            // about one workgroup per CU in a single round where the column tiles alone do not
            // fill the chip; then as few workgroup rows as give every consumer the same number
            // of row groups (no half-used passes)
            const int target = (int)std::max<int64_t>(1, 256 / std::max<int64_t>(1, ncol));
            const int nc = std::max(1, (waves ? waves : max_waves) - NP);
            const int passes = std::max(1, (L.nrg + nc * target - 1) / (nc * target));
            wg_rows = (L.nrg + nc * passes - 1) / (nc * passes);
        }
        wg_rows = std::max(1, std::min(wg_rows, std::max(1, L.nrg)));
        if (waves == 0) waves = std::min(max_waves - NP, (L.nrg + wg_rows - 1) / wg_rows) + NP;
        if (waves < NP + 1 || waves > max_waves) return UBP_ERR_UNSUPPORTED;
    }
    s.G = G;
    s.CT = CT;
    s.NP = NP;
    s.waves = waves;
    s.wg_rows = wg_rows;
    s.resident = resident;
    return UBP_OK;
}

StripeArgs stripe_args(const ubp_packed *p, const Shape &s, const void *X, int64_t ldx, int N, void *Y, int64_t ldy, bool vec_ok,
                       int ctile0, const Epilogue &ep) {
    const int slot = layout_slot(s.G, s.CT);
    const StripeLayout &L = p->sg[slot];
    const StripeLayoutDev &LD = p->d_sg[slot];
    StripeArgs a;
    a.rg_ptr = LD.rg_ptr;
    a.rg_order = LD.rg_order;
    a.stream = LD.stream;
    a.stream_bytes = (uint32_t)(L.stream.size() * sizeof(uint32_t));
    a.X = static_cast<const uint16_t *>(X);
    a.Y = Y;
    a.ldx = ldx;
    a.ldy = ldy;
    a.M = p->M;
    a.K = p->K;
    a.bh = p->bh;
    a.N = N;
    a.nrg = L.nrg;
    a.nch = L.nch;
    a.ring_bytes = std::min(ring_rows(s.CT), L.nch * kSlotRows) * ring_pitch(s.CT);
    a.err = p->d_error;
    a.ctile0 = ctile0;
    a.n_coltiles = 0;
    a.n_wgrows = s.wg_rows;
    a.n_producers = s.NP;
    a.resident = s.resident ? 1 : 0;
    a.vec_ok = vec_ok;
    a.ep = ep;
    return a;
}

// The whole of ubp_spmm_plan / ubp_spmm_prepare.  dry: everything but the launch.
ubp_status execute(const ubp_packed *p, const void *X_dev, int64_t ldx, int32_t N, void *Y_dev, int64_t ldy, ubp_dtype y_dtype,
                   void *stream, const ubp_plan *plan, bool dry, ubp_plan *chosen, const ubp_epilogue *fused) {
    if (!p || N < 0) return UBP_ERR_INVALID_ARG;
    Epilogue ep = {nullptr, 0, 0.f, 0.f};
    if (fused) {
        if (fused->activation < 0 || fused->activation > 2) return UBP_ERR_INVALID_ARG;
        if (fused->activation == 2 && !(fused->lo <= fused->hi)) return UBP_ERR_INVALID_ARG; // (also refuses NaN bounds)
        ep.bias = fused->bias_dev;
        ep.on = (fused->bias_dev != nullptr || fused->activation != 0) ? 1 : 0;
        ep.lo = fused->activation == 1 ? 0.f : fused->activation == 2 ? fused->lo : -INFINITY;
        ep.hi = fused->activation == 2 ? fused->hi : INFINITY;
    }
    if (p->device == UBP_HOST_ONLY) return UBP_ERR_INVALID_ARG;
    if (y_dtype != UBP_F32 && y_dtype != p->dtype) return UBP_ERR_INVALID_ARG;
    if (N == 0) return UBP_OK;
    if (!X_dev || !Y_dev || ldx < N || ldy < N) return UBP_ERR_INVALID_ARG;
    ubp_plan pl;
    std::memset(&pl, 0, sizeof pl);
    if (plan) pl = *plan;
    DeviceGuard guard(p->device);
    if (!guard.ok) return UBP_ERR_DEVICE;
    const size_t ysz = (y_dtype == UBP_F32) ? 4 : 2;
    const bool vec_ok = (ldx % 8 == 0) && (reinterpret_cast<uintptr_t>(X_dev) % 16 == 0) && ((ldy * ysz) % 16 == 0) &&
                        (reinterpret_cast<uintptr_t>(Y_dev) % 16 == 0);
    const bool bf16 = p->dtype == UBP_BF16, y_f32 = y_dtype == UBP_F32;

    Shape s;
    Shape tail;          // block kernel: the gather kernel's shape for a ragged last column tile
    bool has_tail = false;
    {
        // Layouts are built and uploaded on first use, under the handle's lock.  A repeated call
        // finds everything in place and allocates nothing.
        std::lock_guard<std::mutex> hold(p->lock);
        ubp_status rc = resolve(p, N, ldx * 2, vec_ok, pl, s);
        if (rc != UBP_OK) return rc;
        switch (s.kernel) {
        case 1:
        case 3: rc = upload_values_f32(p); break;
        case 2: rc = upload_stripe_layout(p, layout_slot(s.G, s.CT)); break;
        case 4:
        case 5:
        case 7: rc = upload_tile_layout(p); break;
        case 6:
            rc = upload_blk_layout(p, blk_slot(s.G));
            if (rc == UBP_OK && N % 64 != 0) {
                ubp_plan tp;
                std::memset(&tp, 0, sizeof tp);
                tp.kernel = 2;
                tp.col_tiles = 4;
                rc = resolve(p, N, ldx * 2, vec_ok, tp, tail);
                if (rc == UBP_OK) rc = upload_stripe_layout(p, layout_slot(tail.G, tail.CT));
                has_tail = true;
            }
            break;
        }
        if (rc != UBP_OK) return rc;
    }
    if (chosen) {
        std::memset(chosen, 0, sizeof *chosen);
        chosen->kernel = s.kernel;
        chosen->sub_stripes = s.G;
        chosen->col_tiles = s.CT;
        chosen->waves = s.kernel == 5 ? 16 / s.G + 4 : s.waves;
        chosen->rows_per_range = s.rpr;
        chosen->producers = s.kernel == 5 ? 4 : s.NP;
        chosen->wg_rows = s.wg_rows;
    }

    switch (s.kernel) {
    case 1:
    case 3: return launch_wros(p, X_dev, ldx, N, Y_dev, ldy, y_dtype, s.rpr, s.kernel == 3, ep, stream, dry);
    case 2: return launch_stripe(stripe_args(p, s, X_dev, ldx, N, Y_dev, ldy, vec_ok, 0, ep), bf16, y_f32, s.G, s.CT, s.waves, stream, dry);
    case 4:
    case 5:
    case 7: {
        const TileLayout &T = p->tiles;
        TileArgs a = {};
        a.frags = p->d_tiles.frags;
        a.occupied = p->d_tiles.occupied;
        a.X = static_cast<const uint16_t *>(X_dev);
        a.Y = Y_dev;
        a.ldx = ldx;
        a.ldy = ldy;
        a.M = p->M;
        a.K = p->K;
        a.N = N;
        a.nstripes = T.nstripes;
        a.err = p->d_error;
        a.ep = ep;
        a.kt_total = T.kt_pad;
        a.skip = T.tiles_nonzero != (int64_t)T.nstripes * ((p->K + kStep - 1) / kStep) ? 1 : 0; // (padding tiles aside)
        a.n_blocks = (N + 16 * s.CT - 1) / (16 * s.CT);
        a.slices = s.wg_rows;
        a.sps = (T.nstripes + s.wg_rows - 1) / s.wg_rows;
        if (s.kernel == 7) return launch_gemm(a, bf16, y_f32, s.shape, stream, dry);
        if (s.kernel == 4) return launch_xstat(a, bf16, y_f32, s.CT, T.kt_pad, s.waves, stream, dry);
        return launch_xchunk(a, bf16, y_f32, s.CT, s.G, stream, dry);
    }
    case 6: {
        const int slot = blk_slot(s.G);
        const BlkLayout &L = p->blk[slot];
        const BlkLayoutDev &LD = p->d_blk[slot];
        BlkArgs a = {};
        a.rg_ptr = LD.rg_ptr;
        a.rg_order = LD.rg_order;
        a.meta = LD.meta;
        a.frags = LD.frags;
        a.meta_bytes = (uint32_t)(L.meta.size() * sizeof(uint32_t));
        a.frag_bytes = (uint32_t)(L.frags.size() * sizeof(uint32_t));
        a.X = static_cast<const uint16_t *>(X_dev);
        a.Y = Y_dev;
        a.ldx = ldx;
        a.ldy = ldy;
        a.M = p->M;
        a.K = p->K;
        a.N = N;
        a.nrg = L.nrg;
        a.nch = L.nch;
        a.ring_bytes = std::min(ring_rows(4), L.nch * kSlotRows) * ring_pitch(4);
        a.n_coltiles = N / 64;
        a.n_wgrows = s.wg_rows;
        a.n_producers = s.NP;
        a.out_bytes = 0; // set per launch
        a.err = p->d_error;
        a.ep = ep;
        ubp_status rc = launch_blk(a, bf16, y_f32, s.G, s.waves, stream, dry);
        if (rc == UBP_OK && has_tail)
            rc = launch_stripe(stripe_args(p, tail, X_dev, ldx, N, Y_dev, ldy, vec_ok, N / 64, ep), bf16, y_f32, tail.G, tail.CT,
                               tail.waves, stream, dry);
        return rc;
    }
    }
    return UBP_ERR_INVALID_ARG;
}

} // namespace

} // namespace ubp

// ------------------------------------------------------------------ C ABI
extern "C" {

ubp_status ubp_spmm_plan(const ubp_packed *p, const void *X_dev, int64_t ldx, int32_t N, void *Y_dev, int64_t ldy,
                         ubp_dtype y_dtype, void *hip_stream, const ubp_plan *plan) {
    return ubp::execute(p, X_dev, ldx, N, Y_dev, ldy, y_dtype, hip_stream, plan, false, nullptr, nullptr);
}

ubp_status ubp_spmm(const ubp_packed *p, const void *X_dev, int64_t ldx, int32_t N, void *Y_dev, int64_t ldy,
                    ubp_dtype y_dtype, void *hip_stream) {
    return ubp::execute(p, X_dev, ldx, N, Y_dev, ldy, y_dtype, hip_stream, nullptr, false, nullptr, nullptr);
}

ubp_status ubp_spmm_fused(const ubp_packed *p, const void *X_dev, int64_t ldx, int32_t N, void *Y_dev, int64_t ldy,
                          ubp_dtype y_dtype, const ubp_epilogue *epilogue, void *hip_stream, const ubp_plan *plan) {
    return ubp::execute(p, X_dev, ldx, N, Y_dev, ldy, y_dtype, hip_stream, plan, false, nullptr, epilogue);
}

ubp_status ubp_spmm_prepare(const ubp_packed *p, const void *X_dev, int64_t ldx, int32_t N, void *Y_dev, int64_t ldy,
                            ubp_dtype y_dtype, const ubp_plan *plan, ubp_plan *chosen) {
    return ubp::execute(p, X_dev, ldx, N, Y_dev, ldy, y_dtype, nullptr, plan, true, chosen, nullptr);
}

ubp_status ubp_packed_device_error(const ubp_packed *p, uint32_t *flags) {
    if (!p || !flags || p->device == UBP_HOST_ONLY) return UBP_ERR_INVALID_ARG;
    ubp::DeviceGuard guard(p->device);
    if (!guard.ok) return UBP_ERR_DEVICE;
    if (hipMemcpy(flags, p->d_error, sizeof(uint32_t), hipMemcpyDeviceToHost) != hipSuccess) {
        (void)hipGetLastError();
        return UBP_ERR_DEVICE;
    }
    return UBP_OK;
}

ubp_status ubp_launch_floor(void *hip_stream) { return ubp::launch_floor(hip_stream); }

} // extern "C"
