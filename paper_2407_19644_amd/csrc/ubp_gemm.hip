// Dense-tile kernel of the UBP library with both operands staged in LDS (fp16 / bf16), for
// layers in which every 16 x 32 tile of W keeps a weight.
//
// The small-K and chunked dense-tile kernels read every weight tile from memory once per 64
// pixels; what bounds them is the number of vector-memory instructions a CU retires.  Here a
// workgroup owns TM rows x TN pixels of Y (up to 256 x 256) for the whole of K, so that a weight
// tile is fetched once per TN pixels and a row of X once per TM output rows, and both arrive by
// direct global->LDS loads, which cost no registers and leave the wavefronts to the matrix work.
#include "ubp_device.h"

#include <cstdint>

namespace ubp {

namespace {

// Position of the 32-byte unit u (16 pixels) inside row r of a staged X tile is u ^ tile_swizzle(r):
// a transposed read covers 16 consecutive rows of one unit, and LDS has 64 four-byte banks, i.e. 8
// windows of 32 bytes; the swizzle spreads the 16 rows over all 8 (two rows per window, the minimum).
template <int UNITS> __device__ __forceinline__ constexpr int tile_swizzle(int r) {
    return UNITS >= 8 ? (r & 7) : UNITS == 4 ? ((r >> 1) & 3) : UNITS == 2 ? ((r >> 2) & 1) : 0;
}

// Workgroup = WM x WN wavefronts; wavefront (wm, wn) owns SM stripes x PN pixel tiles of 16, all
// accumulators in registers for the whole K loop (output stationary, as in the paper's kernel).
// K passes in stages of 32 rows: a stage is the TM / 16 weight tiles of that 32-column step (1 KB
// each, already in operand order) and 32 rows of X (TN pixels each, units swizzled as above), in
// one of NS LDS slots.  Every wavefront issues its share of a stage's 1 KB loads NS - 1 stages
// ahead; one barrier per stage says both "stage kt has landed" (each wavefront first waits for
// its own loads of that stage - vector memory completes in order) and "everybody is done reading
// the slot that the next loads overwrite".  Rows past K and pixels past N are loaded from
// clamped addresses: the weight tiles hold zeros beyond K, and pixels past N are not stored.
// Every tile is loaded and multiplied: the launcher takes only matrices whose every tile keeps a
// weight.  (A variant that tested one bit per tile before every load and multiplication was built
// and measured: the tests and the load counts that then vary per stage cost more than the small
// and chunked kernels lose to it, so layers with empty tiles stay with those.)
template <bool BF16, typename TY, int WM, int WN, int SM, int PN, int NS>
__global__ __launch_bounds__(WM * WN * 64) void gemm_kernel(TileArgs a) {
    constexpr int NW = WM * WN;
    constexpr int TS = WM * SM;                 // stripes per workgroup
    constexpr int UNITS = WN * PN;              // 16-pixel units per workgroup
    constexpr int TN = 16 * UNITS;
    constexpr int XROWB = 2 * TN;               // bytes of a staged row of X
    constexpr int PIECES = XROWB / 16;          // 16-byte pieces per staged row
    constexpr int RPI = 64 / PIECES;            // rows of X per 1 KB load
    static_assert(PIECES <= 64 && RPI * PIECES == 64, "a 1 KB load covers whole rows");
    constexpr int WSTAGE = TS * 1024, XSTAGE = 32 * XROWB, STAGE = WSTAGE + XSTAGE;
    constexpr int NXI = 32 / RPI;               // X loads per stage
    constexpr int NLD = TS + NXI;               // loads per stage
    static_assert(NLD % NW == 0, "every wavefront issues the same number of loads per stage");
    constexpr int PER = NLD / NW;
    extern __shared__ __attribute__((aligned(1024))) char smem[];

    // Consecutive workgroup ids go round-robin over the 8 XCDs: pixel blocks are dealt by id mod 8 and
    // the row blocks of a pixel block are neighbours on its XCD, so that X comes from memory once
    // and from that XCD's L2 for the other row blocks.
    const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
    const int nb = xcd + 8 * (local / a.slices), mb = local % a.slices;
    if (nb >= a.n_blocks) return;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int wm = wave / WN, wn = wave % WN;
    const int col0 = nb * TN;
    const int stripe0 = mb * TS;
    const int nkt = (a.K + kStep - 1) / kStep; // (the layout may pad a stripe to more tiles: those are zero)
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_address(smem));

    // ---- this wavefront's loads of a stage: load j (0 .. NLD-1) belongs to wavefront j % NW
    const int row_in = lane / PIECES, pp = lane % PIECES;
    auto issue_stage = [&](int kt, int slot) {
        const uint32_t base = lds0 + (uint32_t)(slot * STAGE);
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            const int j = wave + q * NW; // (wave-uniform)
            if (j < TS) {
                const int s = min(stripe0 + j, a.nstripes - 1);
                load16_to_lds(a.frags + ((int64_t)s * a.kt_total + kt) * 512, (uint32_t)lane * 16u, base + (uint32_t)j * 1024u);
            } else {
                const int i = j - TS;
                const int r = i * RPI + row_in;                                   // row inside the stage
                const int u = (pp >> 1) ^ tile_swizzle<UNITS>(r);                 // the unit stored at this position
                const int k = min(kt * 32 + r, a.K - 1);
                const int col = min(col0 + u * 16 + (pp & 1) * 8, a.N - 8);
                load16_to_lds(a.X, (uint32_t)(((int64_t)k * a.ldx + col) * 2), base + (uint32_t)(WSTAGE + i * 1024));
            }
        }
    };

    float4v acc[SM][PN];
#pragma unroll
    for (int i = 0; i < SM; ++i)
#pragma unroll
        for (int c = 0; c < PN; ++c) acc[i][c] = float4v{0.f, 0.f, 0.f, 0.f};

    // this lane's part in the transposed reads of pixel tile pn: rows e and 16 + e of the stage
    const int g = lane >> 4, n = lane & 15;
    const int e = 4 * g + (n >> 2);
    uint32_t xaddr[PN];
#pragma unroll
    for (int c = 0; c < PN; ++c)
        xaddr[c] = lds0 + (uint32_t)(WSTAGE + e * XROWB + (((wn * PN + c) ^ tile_swizzle<UNITS>(e)) << 5) + (n & 3) * 8);
    const uint32_t waddr = lds0 + (uint32_t)(wm * SM * 1024 + lane * 16);
    typedef __attribute__((address_space(3))) const uint4v *lds_frag_ptr;

#pragma unroll
    for (int s = 0; s < NS - 1; ++s)
        if (s < nkt) issue_stage(s, s);
    for (int kt0 = 0; kt0 < nkt; kt0 += NS) {
#pragma unroll
        for (int sl = 0; sl < NS; ++sl) { // (unrolled so that the slot is a constant)
            const int kt = kt0 + sl;
            if (kt < nkt) {
                // my loads of stage kt have landed when at most those of the later stages are outstanding
                wait_vmcnt_at_most(min(NS - 2, nkt - 1 - kt) * PER);
                lds_barrier();
                if (kt + NS - 1 < nkt) issue_stage(kt + NS - 1, (sl + NS - 1) % NS);
                uint4v wf[SM];
                short8v xf[PN];
#pragma unroll
                for (int i = 0; i < SM; ++i) wf[i] = *(lds_frag_ptr)(uintptr_t)(waddr + (uint32_t)(sl * STAGE + i * 1024));
#pragma unroll
                for (int c = 0; c < PN; ++c) {
                    const short4v p0 = lds_read_tr(xaddr[c] + (uint32_t)(sl * STAGE));
                    const short4v p1 = lds_read_tr(xaddr[c] + (uint32_t)(sl * STAGE + 16 * XROWB));
                    xf[c] = __builtin_shufflevector(p0, p1, 0, 1, 2, 3, 4, 5, 6, 7);
                }
#pragma unroll
                for (int i = 0; i < SM; ++i) {
                    const short8v wv = __builtin_bit_cast(short8v, wf[i]);
#pragma unroll
                    for (int c = 0; c < PN; ++c) acc[i][c] = mfma16<BF16>(xf[c], wv, acc[i][c]);
                }
            }
        }
    }

    // ---- stores: through 16 LDS rows of this wavefront (the stages are dead), whole rows out.
    // Lane (g, n) holds pixels 16 c + 4 g .. + 3 of row n of a stripe's tile c.
    lds_barrier(); // everybody is done with the last stage
    constexpr int YS = (int)sizeof(TY);
    constexpr int RB = 16 * PN * YS;                // bytes of one row of this wavefront's tile row
    constexpr int PR = RB / 16;                     // 16-byte pieces per row
    constexpr int RP = RB >= 256 ? 1 : 256 / RB;    // rows per 256 bytes (one pass over the banks)
    constexpr int NI = (16 * PR) / 64;              // store instructions per stripe
    static_assert(NI >= 1, "a stripe's tile row is at least 1 KB");
    char *scratch = smem + wave * (16 * RB);
    TY *Yt = static_cast<TY *>(a.Y);
    const int pcol0 = col0 + wn * PN * 16;
#pragma unroll
    for (int i = 0; i < SM; ++i) {
        const int stripe = stripe0 + wm * SM + i;
        if (a.ep.on) {
            const float b = epilogue_bias(a.ep, stripe * kStripe + n, a.M);
#pragma unroll
            for (int c = 0; c < PN; ++c) epilogue_tile(a.ep, acc[i][c], b);
        }
#pragma unroll
        for (int c = 0; c < PN; ++c) {
            const int byte = (16 * c + 4 * g) * YS;
            const int piece = (byte >> 4) ^ ((n / RP) & (PR - 1) & 7);
            char *dst = scratch + n * RB + piece * 16 + (byte & 15);
            if constexpr (YS == 4) {
                *reinterpret_cast<float4v *>(dst) = acc[i][c];
            } else {
                typedef TY ty4 __attribute__((ext_vector_type(4)));
                ty4 o;
#pragma unroll
                for (int v = 0; v < 4; ++v) o[v] = from_f32<TY>(acc[i][c][v]);
                *reinterpret_cast<ty4 *>(dst) = o;
            }
        }
        // (one wavefront writes and reads: LDS executes its instructions in order)
#pragma unroll
        for (int q = 0; q < NI; ++q) {
            const int r = q * (64 / PR) + lane / PR, lp = lane % PR;
            const uint4v o = *reinterpret_cast<const uint4v *>(scratch + r * RB + ((lp ^ ((r / RP) & (PR - 1) & 7)) << 4));
            const int row = stripe * kStripe + r;
            const int px = pcol0 + lp * (16 / YS);
            if (stripe < a.nstripes && row < a.M && px + 16 / YS <= a.N) *reinterpret_cast<uint4v *>(Yt + (int64_t)row * a.ldy + px) = o;
        }
    }
}

template <bool BF16, typename TY, int WM, int WN, int SM, int PN, int NS>
ubp_status launch_gemm_inst(const TileArgs &a, hipStream_t st, bool dry) {
    constexpr int TS = WM * SM, TN = 16 * WN * PN;
    if (a.skip) return UBP_ERR_UNSUPPORTED; // a tile keeps nothing: the kernels that test for that take the layer
    constexpr size_t lds = (size_t)NS * (TS * 1024 + 32 * 2 * TN);
    static_assert(lds <= 160 * 1024, "the stages fit LDS");
    static_assert((size_t)WM * WN * 16 * 16 * PN * 4 <= lds, "the output rows fit where the stages were");
    static LdsLimit limit; // per instantiation
    const ubp_status rc = limit.raise(reinterpret_cast<const void *>(&gemm_kernel<BF16, TY, WM, WN, SM, PN, NS>));
    if (rc != UBP_OK || dry) return rc;
    TileArgs b = a;
    b.n_blocks = (a.N + TN - 1) / TN;
    b.slices = (a.nstripes + TS - 1) / TS;
    const unsigned grid = 8u * (unsigned)((b.n_blocks + 7) / 8) * (unsigned)b.slices;
    hipLaunchKernelGGL((gemm_kernel<BF16, TY, WM, WN, SM, PN, NS>), dim3(grid), dim3(WM * WN * 64), lds, st, b);
    return hipGetLastError() == hipSuccess ? UBP_OK : UBP_ERR_DEVICE;
}

template <bool BF16, typename TY>
ubp_status launch_gemm_t(const TileArgs &a, int shape, hipStream_t st, bool dry) {
    switch (shape) {
    case 0: return launch_gemm_inst<BF16, TY, 2, 4, 8, 4, 4>(a, st, dry); // 256 rows x 256 pixels, 8 wavefronts
    case 1: return launch_gemm_inst<BF16, TY, 2, 4, 4, 4, 4>(a, st, dry); // 128 x 256, 8 wavefronts
    case 2: return launch_gemm_inst<BF16, TY, 2, 2, 4, 4, 4>(a, st, dry); // 128 x 128, 4 wavefronts
    case 3: return launch_gemm_inst<BF16, TY, 4, 1, 4, 4, 4>(a, st, dry); // 256 x 64, 4 wavefronts
    case 4: return launch_gemm_inst<BF16, TY, 2, 2, 2, 4, 4>(a, st, dry); // 64 x 128, 4 wavefronts
    case 5: return launch_gemm_inst<BF16, TY, 2, 2, 2, 2, 4>(a, st, dry); // 64 x 64, 4 wavefronts
    }
    return UBP_ERR_UNSUPPORTED;
}

} // namespace

// shape -> (rows, pixels) of a workgroup's tile
void gemm_shape(int shape, int *rows, int *pixels) {
    static const int kRows[kNumGemmShapes] = {256, 128, 128, 256, 64, 64}, kPx[kNumGemmShapes] = {256, 256, 128, 64, 128, 64};
    *rows = kRows[shape];
    *pixels = kPx[shape];
}

ubp_status launch_gemm(const TileArgs &a, bool bf16, bool y_f32, int shape, void *stream, bool dry) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (shape < 0 || shape >= kNumGemmShapes) return UBP_ERR_UNSUPPORTED;
    // the loads address X with 32-bit byte offsets
    if ((int64_t)a.K * a.ldx * 2 >= (int64_t(1) << 31)) return UBP_ERR_UNSUPPORTED;
    if (bf16) return y_f32 ? launch_gemm_t<true, float>(a, shape, st, dry) : launch_gemm_t<true, __bf16>(a, shape, st, dry);
    return y_f32 ? launch_gemm_t<false, float>(a, shape, st, dry) : launch_gemm_t<false, _Float16>(a, shape, st, dry);
}

} // namespace ubp
