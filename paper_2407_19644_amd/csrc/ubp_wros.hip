// Vector-ALU kernel of the UBP library: the paper's WROS dataflow, literally (Section 4.2).
#include "ubp_device.h"

#include <cstdint>

namespace ubp {

namespace {

// ------------------------------------------------------------------ WROS vector kernel
// Grid: x = column tiles of 256*VEC columns, y = ranges of `rpr` output rows.
// A thread owns VEC columns and BH accumulator rows (slots).  Start rows are walked in
// increasing order; the loop is unrolled by BH so that "slot = start row mod BH" is a
// compile-time register name.  After start row i is done, output row i is complete (later
// blocks start below it): its slot is stored and cleared, the other slots keep
// accumulating.  A range re-walks the BH-1 start rows above it, whose blocks reach into the
// range, and drops what those blocks add to rows it does not own.
template <typename TX, typename TY, int BH, int VEC>
__global__ __launch_bounds__(256) void wros_kernel(const int32_t *__restrict__ indptr, const int32_t *__restrict__ indices,
                                                  const float *__restrict__ vals, const TX *__restrict__ X, int64_t ldx,
                                                  TY *__restrict__ Y, int64_t ldy, int M, int N, int bw, int rpr, Epilogue ep) {
    const int col = (blockIdx.x * 256 + threadIdx.x) * VEC;
    if (col >= N) return;
    const int lo = blockIdx.y * rpr;
    const int hi = min(lo + rpr, M);
    const int last_start = M - BH; // start rows beyond this hold no block (epilogue rows)
    float acc[BH][VEC];
#pragma unroll
    for (int s = 0; s < BH; ++s)
#pragma unroll
        for (int v = 0; v < VEC; ++v) acc[s][v] = 0.f;

    const int first = max(0, lo - BH + 1);
    for (int base = (first / BH) * BH; base < hi; base += BH) {
#pragma unroll
        for (int u = 0; u < BH; ++u) {
            const int i = base + u; // start row; i mod BH == u
            if (i < first || i >= hi) continue;
            if (i <= last_start) {
                const int b1 = indptr[i + 1];
                for (int b = indptr[i]; b < b1; ++b) {
                    const int c = indices[b];
                    const float *w = vals + (int64_t)b * bw * BH;
                    for (int q = 0; q < bw; ++q) {
                        float x[VEC];
                        load_row<TX, VEC>(X + (int64_t)(c + q) * ldx + col, x);
#pragma unroll
                        for (int s = 0; s < BH; ++s) {
                            const float ws = w[q * BH + s];
#pragma unroll
                            for (int v = 0; v < VEC; ++v) acc[s][v] = fmaf(ws, x[v], acc[s][v]);
                        }
                    }
                }
            }
            if (i >= lo) {
                if (ep.on) {
                    const float b = ep.bias ? ep.bias[i] : 0.f;
#pragma unroll
                    for (int v = 0; v < VEC; ++v) acc[u][v] = epilogue_value(ep, acc[u][v], b);
                }
                store_row<TY, VEC>(Y + (int64_t)i * ldy + col, acc[u]);
            }
#pragma unroll
            for (int v = 0; v < VEC; ++v) acc[u][v] = 0.f;
        }
    }
}

// ------------------------------------------------------------------ naive dataflow (comparison only)
// The dataflow the weight rotation replaces (Section 3.3): accumulator row t always belongs to
// the output row t below the current start row.  After start row i is done, row 0 is stored, rows
// 1 .. BH-1 move up by one register row and the last one is cleared.  Same grid, same ranges, same
// loads and the same order of additions per output element as wros_kernel; the weights are read
// from the rotated array at the slot their row has there.
template <typename TX, typename TY, int BH, int VEC>
__global__ __launch_bounds__(256) void naive_kernel(const int32_t *__restrict__ indptr, const int32_t *__restrict__ indices,
                                                   const float *__restrict__ vals, const TX *__restrict__ X, int64_t ldx,
                                                   TY *__restrict__ Y, int64_t ldy, int M, int N, int bw, int rpr, Epilogue ep) {
    const int col = (blockIdx.x * 256 + threadIdx.x) * VEC;
    if (col >= N) return;
    const int lo = blockIdx.y * rpr;
    const int hi = min(lo + rpr, M);
    const int last_start = M - BH;
    float acc[BH][VEC];
#pragma unroll
    for (int t = 0; t < BH; ++t)
#pragma unroll
        for (int v = 0; v < VEC; ++v) acc[t][v] = 0.f;

    for (int i = max(0, lo - BH + 1); i < hi; ++i) {
        if (i <= last_start) {
            const int u = i % BH; // slot of the block's first row in the rotated array
            const int b1 = indptr[i + 1];
            for (int b = indptr[i]; b < b1; ++b) {
                const int c = indices[b];
                const float *w = vals + (int64_t)b * bw * BH;
                for (int q = 0; q < bw; ++q) {
                    float x[VEC];
                    load_row<TX, VEC>(X + (int64_t)(c + q) * ldx + col, x);
#pragma unroll
                    for (int t = 0; t < BH; ++t) {
                        const float wt = w[q * BH + (u + t >= BH ? u + t - BH : u + t)];
#pragma unroll
                        for (int v = 0; v < VEC; ++v) acc[t][v] = fmaf(wt, x[v], acc[t][v]);
                    }
                }
            }
        }
        if (i >= lo) {
            if (ep.on) {
                const float b = ep.bias ? ep.bias[i] : 0.f;
#pragma unroll
                for (int v = 0; v < VEC; ++v) acc[0][v] = epilogue_value(ep, acc[0][v], b);
            }
            store_row<TY, VEC>(Y + (int64_t)i * ldy + col, acc[0]);
        }
#pragma unroll
        for (int t = 0; t + 1 < BH; ++t)
#pragma unroll
            for (int v = 0; v < VEC; ++v) acc[t][v] = acc[t + 1][v];
#pragma unroll
        for (int v = 0; v < VEC; ++v) acc[BH - 1][v] = 0.f;
    }
}

template <typename TX, typename TY, int VEC>
ubp_status launch_wros_bh(const ubp_packed *p, const void *X, int64_t ldx, int N, void *Y, int64_t ldy, int rpr,
                          bool naive, const Epilogue &ep, hipStream_t st) {
    dim3 grid((unsigned)((N + 256 * VEC - 1) / (256 * VEC)), (unsigned)((p->M + rpr - 1) / rpr));
#define UBP_WROS_CASE(BH)                                                                                              \
    case BH:                                                                                                           \
        hipLaunchKernelGGL((naive ? (naive_kernel<TX, TY, BH, VEC>) : (wros_kernel<TX, TY, BH, VEC>)), grid, dim3(256), 0, \
                           st, p->d_indptr, p->d_indices, p->d_values_f32, static_cast<const TX *>(X), ldx,           \
                           static_cast<TY *>(Y), ldy, p->M, N, p->bw, rpr, ep);                                        \
        break;
    switch (p->bh) {
        UBP_WROS_CASE(1) UBP_WROS_CASE(2) UBP_WROS_CASE(3) UBP_WROS_CASE(4) UBP_WROS_CASE(5) UBP_WROS_CASE(6)
        UBP_WROS_CASE(7) UBP_WROS_CASE(8) UBP_WROS_CASE(9) UBP_WROS_CASE(10) UBP_WROS_CASE(11) UBP_WROS_CASE(12)
        UBP_WROS_CASE(13) UBP_WROS_CASE(14) UBP_WROS_CASE(15) UBP_WROS_CASE(16)
    default: return UBP_ERR_UNSUPPORTED;
    }
#undef UBP_WROS_CASE
    return hipGetLastError() == hipSuccess ? UBP_OK : UBP_ERR_DEVICE;
}

template <typename TX, typename TY>
ubp_status launch_wros_t(const ubp_packed *p, const void *X, int64_t ldx, int N, void *Y, int64_t ldy, int rpr,
                         bool naive, const Epilogue &ep, hipStream_t st) {
    // 4 columns per thread when every row of X and Y can be accessed as an aligned 4-vector
    const bool vec = (N % 4 == 0) && (ldx % 4 == 0) && (ldy % 4 == 0) &&
                     (reinterpret_cast<uintptr_t>(X) % (4 * sizeof(TX)) == 0) &&
                     (reinterpret_cast<uintptr_t>(Y) % (4 * sizeof(TY)) == 0) && N >= 2048;
    return vec ? launch_wros_bh<TX, TY, 4>(p, X, ldx, N, Y, ldy, rpr, naive, ep, st)
               : launch_wros_bh<TX, TY, 1>(p, X, ldx, N, Y, ldy, rpr, naive, ep, st);
}

} // namespace

ubp_status launch_wros(const ubp_packed *p, const void *X, int64_t ldx, int N, void *Y, int64_t ldy, ubp_dtype y_dtype,
                       int rpr, bool naive, const Epilogue &ep, void *stream, bool dry) {
    if (dry) return p->bh > 16 ? UBP_ERR_UNSUPPORTED : UBP_OK; // static LDS only: nothing to prepare
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (p->bh > 16) return UBP_ERR_UNSUPPORTED;
    switch (p->dtype) {
    case UBP_F32: return launch_wros_t<float, float>(p, X, ldx, N, Y, ldy, rpr, naive, ep, st);
    case UBP_F16:
        return y_dtype == UBP_F32 ? launch_wros_t<_Float16, float>(p, X, ldx, N, Y, ldy, rpr, naive, ep, st)
                                  : launch_wros_t<_Float16, _Float16>(p, X, ldx, N, Y, ldy, rpr, naive, ep, st);
    case UBP_BF16:
        return y_dtype == UBP_F32 ? launch_wros_t<__bf16, float>(p, X, ldx, N, Y, ldy, rpr, naive, ep, st)
                                  : launch_wros_t<__bf16, __bf16>(p, X, ldx, N, Y, ldy, rpr, naive, ep, st);
    }
    return UBP_ERR_INVALID_ARG;
}

// An empty kernel: what a launch costs on this device with nothing to do (measurement only).
__global__ void floor_kernel() {}

ubp_status launch_floor(void *stream) {
    hipLaunchKernelGGL(floor_kernel, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream));
    return hipGetLastError() == hipSuccess ? UBP_OK : UBP_ERR_DEVICE;
}

} // namespace ubp
