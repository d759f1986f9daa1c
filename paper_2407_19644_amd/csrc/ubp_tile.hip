// Dense-tile kernels of the UBP library (fp16 / bf16): W as zero-filled 16 x 32 operand tiles
// in MFMA operand order, for layers in which nearly every such tile holds a kept weight.
#include "ubp_device.h"

#include <cstdint>

namespace ubp {

namespace {

// ------------------------------------------------------------------ small-K kernel, X stationary in registers
// Small K (<= 256): the loop nest of the paper's dataflow (section 4.2), where output rows are
// finished one after the other and leave for good.  K <= 256 means a wavefront can hold ALL of X for its 16*CT pixels as matrix
// operands in registers (KT*CT fragments of 4 registers).  So:
//  * Workgroup = NW wavefronts on ONE block of 16*CT pixels x one slice of stripes.  The block
//    of X (K rows of 32*CT bytes) is loaded once by all wavefronts together, written to LDS
//    already in the order in which the transposing reads want it (every such read then covers
//    512 consecutive bytes: no bank conflicts by construction), and every wavefront reads all
//    of it into registers.  That is the only barrier.
//  * Then wavefront w streams the stripes w, w+NW, ... of the slice: KT loads fetch a stripe's
//    weight tiles straight from memory in operand order (1 KB contiguous per instruction, each
//    tile read by exactly one wavefront of the workgroup, so LDS would add nothing), the next
//    stripe's loads are in flight while this stripe's KT*CT matrix instructions run, and the 16
//    finished rows are stored at once.  Only CT accumulator tiles are alive at any time.
// Pixels are dealt to the tiles so that a lane's results of two neighbouring tiles are 8
// consecutive 16-bit pixels (one 16-byte piece of the LDS rows through which a finished tile
// leaves, see stripe_out); for a 32-bit Y a tile is 16 consecutive pixels.
template <typename TY> struct PixelMap {
    // first pixel (in the block) of the 4 consecutive pixels that form piece p of tile c
    static constexpr bool kPairs = sizeof(TY) == 2;
    __device__ static __forceinline__ int first(int c, int p) {
        return kPairs ? 32 * (c >> 1) + 8 * p + 4 * (c & 1) : 16 * c + 4 * p;
    }
};

// SKIP: tiles that keep no weight are neither read (their load is sent past the end of the
// buffer, which returns zeros without touching memory) nor multiplied; the instantiation
// without it, for matrices whose every tile keeps a weight, has no trace of the test.
template <bool BF16, typename TY, int CT, int KT, bool SKIP>
__global__ __launch_bounds__(512) void xstat_kernel(TileArgs a) {
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const int NW = (int)(blockDim.x >> 6);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    // Consecutive workgroup ids go round-robin over the 8 XCDs: pixel blocks are dealt by id mod 8
    // and the slices of a block are neighbours on its XCD, so that the block's X is fetched from
    // memory once and found in that XCD's L2 by the other slices.
    const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
    const int block = xcd + 8 * (local / a.slices), slice = local % a.slices;
    if (block >= a.n_blocks) return;
    const int bcol0 = block * 16 * CT;

    // the first stripe's weight tiles are on their way while X is loaded
    const int s_end = min(slice * a.sps + a.sps, a.nstripes);
    int s = slice * a.sps + wave;
    const uint4v *wbase = reinterpret_cast<const uint4v *>(a.frags) + lane;
    // SKIP: lane i holds the occupancy bits (one per tile) of stripe i of the slice (at most 64)
    [[maybe_unused]] uint32_t occ_v = 0;
    [[maybe_unused]] const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t *>(a.frags), 0, a.nstripes * KT * 1024, 0x00020000);
    if constexpr (SKIP) {
        const int st = slice * a.sps + lane;
        if (lane < a.sps && st < a.nstripes) occ_v = a.occupied[st];
    }
    auto occupancy = [&](int stripe) -> uint32_t {
        if constexpr (SKIP) {
            const int i = stripe - slice * a.sps;
            if (i >= a.sps || stripe >= a.nstripes) return 0u;
            if (a.sps > 64) return a.occupied[stripe]; // (a slice too tall for one register of words: a scalar load per stripe)
            return (uint32_t)__builtin_amdgcn_readlane((int)occ_v, i & 63);
        }
        return 0xffffffffu;
    };
    auto load_w = [&](uint4v(&w)[KT], int stripe) {
        // (a stripe past the slice is clamped: loaded, never used)
        if constexpr (SKIP) {
            const uint32_t occ = occupancy(stripe);
            const uint32_t base = (uint32_t)min(stripe, a.nstripes - 1) * (uint32_t)(KT * 1024);
#pragma unroll
            for (int kt = 0; kt < KT; ++kt) {
                // (the offset of an empty tile lies beyond the buffer: zeros come back, nothing is read)
                const uint32_t vo = ((occ >> kt) & 1u) ? (uint32_t)lane * 16u : 0xfffffff0u;
                w[kt] = __builtin_bit_cast(uint4v, __builtin_amdgcn_raw_buffer_load_b128(rsrc, vo, base + (uint32_t)kt * 1024u, 0));
            }
        } else {
            const uint4v *src = wbase + (int64_t)min(stripe, a.nstripes - 1) * (KT * 64);
#pragma unroll
            for (int kt = 0; kt < KT; ++kt) w[kt] = src[kt * 64];
        }
    };
    uint4v w0[KT], w1[KT];
    load_w(w0, s);

    // ---- X block -> LDS.  LDS holds [kt][c][lo/hi half of the 32 rows][64 lanes] x 8 bytes: the
    // 8 bytes lane (g', n') supplies to the transposing read of that half = 4 pixels (piece
    // n' & 3 of tile c) of row 4 g' + (n' >> 2) of the half.
    {
        constexpr int LPR = 2 * CT;        // 16-byte pieces per block row
        constexpr int RPI = 64 / LPR;      // rows per load instruction
        constexpr int DEPTH = 8;           // loads in flight per lane (all of them for 4 wavefronts, CT = 4, K = 256)
        const int row_in = lane / LPR, q = lane % LPR;
        const int col = bcol0 + 8 * q;
        const bool col_in = col + 8 <= a.N;   // (N is a multiple of 8: a piece lies inside or outside)
        const uint16_t *src = a.X + min(col, a.N - 8);
        // (u0: first row of this wavefront's instruction, wave-uniform; an instruction lies
        // entirely inside or outside the KT * 32 rows, which are a multiple of RPI)
        // (unrolled to the batch count of a single wavefront, not a loop: in front of a loop the
        // compiler would first wait for the weight loads above)
        constexpr int BATCHES = (KT * 32 + DEPTH * RPI - 1) / (DEPTH * RPI);
#pragma unroll
        for (int b = 0; b < BATCHES; ++b) {
            const int u0 = wave * RPI + b * DEPTH * NW * RPI;
            if (u0 >= KT * 32) break;
            uint4 v[DEPTH];
#pragma unroll
            for (int d = 0; d < DEPTH; ++d) {
                // (no branch around the load - the compiler would wait for each one at the join;
                // rows past the end load row K - 1 again and are dropped below)
                const int k = u0 + d * NW * RPI + row_in;
                const uint4 x = *reinterpret_cast<const uint4 *>(src + (int64_t)min(k, a.K - 1) * a.ldx);
                v[d] = (col_in && k < a.K) ? x : uint4{0u, 0u, 0u, 0u};
            }
#pragma unroll
            for (int d = 0; d < DEPTH; ++d) {
                const int k = u0 + d * NW * RPI + row_in;
                if (u0 + d * NW * RPI < KT * 32) {
                    const int kt = k >> 5, hi = (k >> 4) & 1, gg = (k >> 2) & 3, j = k & 3;
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        // the 4 pixels 8q + 4h .. of the block: tile c, piece pc
                        int c, pc;
                        if constexpr (PixelMap<TY>::kPairs) {
                            c = 2 * (q >> 2) + h;
                            pc = q & 3;
                        } else {
                            c = q >> 1;
                            pc = 2 * (q & 1) + h;
                        }
                        char *dst = smem + (((kt * CT + c) * 2 + hi) << 9) + (gg << 7) + (j << 5) + (pc << 3);
                        *reinterpret_cast<uint2 *>(dst) = h ? uint2{v[d].z, v[d].w} : uint2{v[d].x, v[d].y};
                    }
                }
            }
        }
    }
    __syncthreads();
    short8v xf[KT][CT];
    {
        const uint32_t base = lds_address(smem) + (uint32_t)lane * 8u;
#pragma unroll
        for (int kt = 0; kt < KT; ++kt)
#pragma unroll
            for (int c = 0; c < CT; ++c) {
                const short4v p0 = lds_read_tr(base + (uint32_t)(((kt * CT + c) * 2) << 9));
                const short4v p1 = lds_read_tr(base + (uint32_t)(((kt * CT + c) * 2 + 1) << 9));
                xf[kt][c] = __builtin_shufflevector(p0, p1, 0, 1, 2, 3, 4, 5, 6, 7);
            }
    }

    // ---- stripes of the slice, NW apart
    if (s >= s_end) return;
    const int g = lane >> 4, n = lane & 15;
    char *out_lds = smem + KT * CT * 1024 + wave * (256 * CT * (int)sizeof(TY)); // behind the X block
    TY *Yt = static_cast<TY *>(a.Y);
    auto stripe_out = [&](const uint4v(&w)[KT], int stripe, bool valid) {
        [[maybe_unused]] const uint32_t occ = occupancy(stripe);
        float4v acc[CT];
#pragma unroll
        for (int c = 0; c < CT; ++c) acc[c] = float4v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kt = 0; kt < KT; ++kt) {
            if (SKIP && !((occ >> kt) & 1u)) continue; // (wave-uniform)
            const short8v wv = __builtin_bit_cast(short8v, w[kt]);
#pragma unroll
            for (int c = 0; c < CT; ++c) acc[c] = mfma16<BF16>(xf[kt][c], wv, acc[c]);
        }
        // The 16 x (16 CT) result leaves through this wavefront's own piece of LDS: in the
        // accumulators a row is spread over 4 lanes (16 bytes each per store: 64-byte runs),
        // after the detour an instruction writes whole rows of the block (RB bytes each).
        // 16-byte pieces of a row are XOR-swizzled by the row number so that the 16 lanes LDS
        // serves together hit 64 different banks on the way in and on the way out.
        if (a.ep.on) {
            const float b = epilogue_bias(a.ep, stripe * kStripe + n, a.M);
#pragma unroll
            for (int c = 0; c < CT; ++c) epilogue_tile(a.ep, acc[c], b);
        }
        constexpr int RB = 16 * CT * (int)sizeof(TY);   // bytes per row: 64, 128 or 256
        constexpr int PR = RB / 16;                     // pieces per row
        constexpr int RP = 256 / RB;                    // rows per 256 bytes (one pass over the banks)
        constexpr int NI = PR / 4;                      // pieces per lane = store instructions
#pragma unroll
        for (int jp = 0; jp < NI; ++jp) {
            uint4v o;
            if constexpr (PixelMap<TY>::kPairs) {
                typedef TY ty8 __attribute__((ext_vector_type(8)));
                ty8 t8;
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    t8[t] = from_f32<TY>(acc[2 * jp][t]);
                    t8[4 + t] = from_f32<TY>(acc[2 * jp + 1][t]);
                }
                o = __builtin_bit_cast(uint4v, t8);
            } else {
                o = __builtin_bit_cast(uint4v, acc[jp]);
            }
            const int piece = (4 * jp + g) ^ ((n / RP) & (PR - 1));
            *reinterpret_cast<uint4v *>(out_lds + n * RB + piece * 16) = o;
        }
        // (same wavefront writes and reads: LDS executes its instructions in order)
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int r = i * (64 / PR) + lane / PR, lp = lane % PR;
            const uint4v o = *reinterpret_cast<const uint4v *>(out_lds + r * RB + ((lp ^ ((r / RP) & (PR - 1))) << 4));
            const int row = stripe * kStripe + r;
            const int px = bcol0 + lp * (16 / (int)sizeof(TY));
            if (valid && row < a.M && px + 16 / (int)sizeof(TY) <= a.N)
                *reinterpret_cast<uint4v *>(Yt + (int64_t)row * a.ldy + px) = o;
        }
    };
    // Two stripes per round, no exit in the middle: a stripe past the end is computed on the
    // clamped tiles and not stored.  (The fences keep the compiler from sinking the next
    // stripe's loads below this stripe's matrix instructions to save registers.)
    for (; s < s_end; s += 2 * NW) {
        load_w(w1, s + NW);
        __builtin_amdgcn_sched_barrier(0);
        stripe_out(w0, s, true);
        load_w(w0, s + 2 * NW);
        __builtin_amdgcn_sched_barrier(0);
        stripe_out(w1, s + NW, s + NW < s_end);
    }
}

// ------------------------------------------------------------------ the same for larger K, in chunks
// xstat_kernel's scheme when K does not fit the registers: K is cut into chunks of KT * 32 rows,
// and what stays put are the accumulators - a workgroup owns 16 stripes x 16 * CT pixels for the
// whole of K (layers with few output rows, or slices of more), a multiplying wavefront SW of
// the stripes.
//  * 16 / SW wavefronts multiply, 4 more do nothing but bring X in: global -> registers -> LDS
//    (operand order, as above), requested four chunks ahead.  Separate wavefronts because a
//    wavefront's vector memory operations complete in order: a weight tile from L2 requested
//    behind rows of X from HBM is not seen before those have landed.
//  * LDS holds a ring of kChunkRing chunks.  No barrier after start-up: each loading wavefront
//    counts the chunks it has written, each multiplying wavefront the chunks it has read (every
//    one reads every chunk), a slot is rewritten when all have read it.  The wavefronts may
//    drift apart by the ring: with a barrier per chunk everybody would wait for its weight tiles
//    at the same moment and nothing would cover that wait (measured on the 3x3-convolution
//    layer: 32 us with barriers, 28.5 us without).  Every wait is bounded; one that runs out
//    raises the handle's error flag and the kernel finishes.
//  * A multiplying wavefront fetches the weight tiles of its own stripes straight from memory,
//    two (stripe, chunk) sets ahead, in three register sets that rotate; its accumulator tiles
//    leave at the end, through the wavefront's LDS rows.
constexpr int kChunkStripes = 16, kChunkProducers = 4, kChunkRing = 6;
template <bool BF16, typename TY, int CT, int KT, int SW, bool SKIP>
__global__ __launch_bounds__((kChunkStripes / SW + kChunkProducers) * 64) void xchunk_kernel(TileArgs a) {
    static_assert(SW == 2 || SW == 4, "stripes per multiplying wavefront");
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    constexpr int NWC = kChunkStripes / SW, NP = kChunkProducers, R = kChunkRing;
    constexpr int BUF = KT * CT * 1024;                           // bytes of one chunk of the block in LDS
    constexpr int OUT = 256 * CT * (int)sizeof(TY);               // 16 rows of output per multiplying wavefront
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int block = blockIdx.x % a.n_blocks, slice = blockIdx.x / a.n_blocks;
    const int bcol0 = block * 16 * CT;
    const int nch = a.kt_total / KT;
    uint32_t *written = reinterpret_cast<uint32_t *>(smem + R * BUF + NWC * OUT); // [NP] chunks written, per producer
    uint32_t *read_upto = written + 8;                                             // [NWC] chunks read, per consumer
    if (threadIdx.x < 16) written[threadIdx.x] = 0u;
    __syncthreads();
    bool broken = false;

    if (wave >= NWC) {
        // ---- producers: instruction d of producer pw covers rows (d * NP + pw) * RPI .. of a chunk
        const int pw = wave - NWC;
        constexpr int LPR = 2 * CT;                 // 16-byte pieces per block row
        constexpr int RPI = 64 / LPR;               // rows per load instruction
        constexpr int XD = KT * 32 / (NP * RPI);    // load instructions per producer and chunk
        static_assert(XD * NP * RPI == KT * 32, "a chunk's rows divide evenly over the producers");
        const int row_in = lane / LPR, q = lane % LPR;
        const int col = bcol0 + 8 * q;
        const bool col_in = col + 8 <= a.N;         // (N is a multiple of 8: a piece lies inside or outside)
        const uint16_t *xsrc = a.X + min(col, a.N - 8);
        auto load_x = [&](uint4(&v)[XD], int ch) {
            // Clamped addresses; what lies outside the matrix is zeroed when the data is written
            // to LDS - touching it here would make the wavefront wait for the load at once.
            // (Chunks past the last are loaded too and never written.)
#pragma unroll
            for (int d = 0; d < XD; ++d) {
                const int k = ch * (KT * 32) + (d * NP + pw) * RPI + row_in;
                v[d] = *reinterpret_cast<const uint4 *>(xsrc + (int64_t)min(k, a.K - 1) * a.ldx);
            }
        };
        int free_upto = R; // chunks below this may be written without asking
        auto put = [&](const uint4(&v)[XD], int ch) {
            if (ch >= free_upto && !broken) {
                // chunk ch replaces chunk ch - R: every multiplying wavefront must have read that one
                const uint32_t target = (uint32_t)(ch - R + 1);
                int spins = 0;
                for (;;) {
                    uint32_t seen = 0xffffffffu;
                    if (lane < NWC) seen = __hip_atomic_load(read_upto + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                    asm volatile("" ::: "memory");
                    if (__builtin_amdgcn_ballot_w64(seen < target) == 0) {
                        // how far the slowest one really is: saves asking again for the next chunks
                        int ahead = 1;
                        while (ahead < R && __builtin_amdgcn_ballot_w64(seen < target + (uint32_t)ahead) == 0) ++ahead;
                        free_upto = ch + ahead;
                        break;
                    }
                    if (++spins > kSpinLimit) {
                        broken = true; // reported at the end: a global atomic inside this loop would make the
                        break;         // compiler drain the loads in flight in front of it
                    }
                    __builtin_amdgcn_s_sleep(2);
                }
            }
            char *buf = smem + (ch % R) * BUF;
#pragma unroll
            for (int d = 0; d < XD; ++d) {
                const int k = (d * NP + pw) * RPI + row_in; // row inside the chunk
                const int kt = k >> 5, hi = (k >> 4) & 1, gg = (k >> 2) & 3, j = k & 3;
                const bool inside = col_in && ch * (KT * 32) + k < a.K;
                const uint4 x = inside ? v[d] : uint4{0u, 0u, 0u, 0u};
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    int c, pc;
                    if constexpr (PixelMap<TY>::kPairs) {
                        c = 2 * (q >> 2) + h;
                        pc = q & 3;
                    } else {
                        c = q >> 1;
                        pc = 2 * (q & 1) + h;
                    }
                    char *dst = buf + (((kt * CT + c) * 2 + hi) << 9) + (gg << 7) + (j << 5) + (pc << 3);
                    *reinterpret_cast<uint2 *>(dst) = h ? uint2{x.z, x.w} : uint2{x.x, x.y};
                }
            }
            // LDS executes a wavefront's operations in order: the counter follows the data
            asm volatile("" ::: "memory");
            if (lane == 0) __hip_atomic_store(written + pw, (uint32_t)(ch + 1), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        };
        // Chunk c travels in register set c % XSETS.  What a CU gets out of HBM is the bytes it has
        // in flight over the latency: four chunks (64 KB for a 64-pixel block) are on their way.
        constexpr int XSETS = 4;
        uint4 xs[XSETS][XD];
#pragma unroll
        for (int u = 0; u < XSETS; ++u) load_x(xs[u], u);
        for (int ch = 0; ch < nch;) { // (left from the middle: see the multiplying wavefronts' loop)
#pragma unroll
            for (int u = 0; u < XSETS; ++u) {
                put(xs[u], ch);
                load_x(xs[u], ch + XSETS);
                if (++ch >= nch) break;
            }
        }
        if (broken && lane == 0) atomicOr(a.err, 4u);
        return;
    }

    // ---- multiplying wavefronts
    const int s_end = min(slice * a.sps + a.sps, a.nstripes);
    const int s0 = slice * a.sps + wave * SW; // my stripes s0 .. s0 + SW - 1 (past s_end: clamped tiles, not stored)
    const uint4v *wbase = reinterpret_cast<const uint4v *>(a.frags) + lane;
    // SKIP (see xstat_kernel): lane i * words + w holds word w of the occupancy bits of my stripe i
    const int words = (a.kt_total + 31) >> 5;
    [[maybe_unused]] uint32_t occ_v = 0;
    [[maybe_unused]] const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t *>(a.frags), 0, a.nstripes * a.kt_total * 1024, 0x00020000);
    if constexpr (SKIP) {
        const int i = lane / words, w = lane % words;
        if (i < SW && s0 + i < s_end) occ_v = a.occupied[(s0 + i) * words + w];
    }
    static_assert(KT == 4, "a chunk's occupancy is one nibble");
    auto occupancy = [&](int i, int ch) -> uint32_t { // stripe s0 + i, chunk ch: bits of its KT tiles
        if constexpr (SKIP) {
            if (ch >= nch) return 0u;
            return ((uint32_t)__builtin_amdgcn_readlane((int)occ_v, (i * words + (ch >> 3)) & 63) >> ((ch & 7) * 4)) & 15u;
        }
        return 15u;
    };
    auto load_w = [&](uint4v(&w)[KT], int i, int ch) {
        const int stripe = s0 + i;
        if constexpr (SKIP) {
            const uint32_t occ = occupancy(i, ch);
            const uint32_t base = ((uint32_t)min(stripe, a.nstripes - 1) * (uint32_t)a.kt_total + (uint32_t)(min(ch, nch - 1) * KT)) * 1024u;
#pragma unroll
            for (int kt = 0; kt < KT; ++kt) {
                const uint32_t vo = ((occ >> kt) & 1u) ? (uint32_t)lane * 16u : 0xfffffff0u;
                w[kt] = __builtin_bit_cast(uint4v, __builtin_amdgcn_raw_buffer_load_b128(rsrc, vo, base + (uint32_t)kt * 1024u, 0));
            }
        } else {
            const uint4v *src = wbase + ((int64_t)min(stripe, a.nstripes - 1) * a.kt_total + min(ch, nch - 1) * KT) * 64;
#pragma unroll
            for (int kt = 0; kt < KT; ++kt) w[kt] = src[kt * 64];
        }
    };
    float4v acc[SW][CT];
#pragma unroll
    for (int i = 0; i < SW; ++i)
#pragma unroll
        for (int c = 0; c < CT; ++c) acc[i][c] = float4v{0.f, 0.f, 0.f, 0.f};
    static_assert(R == 6 && (R * SW) % 3 == 0, "the loop below walks the ring in rounds of six chunks, the weight sets in threes");
    const uint32_t lds0 = lds_address(smem) + (uint32_t)lane * 8u;
    const uint32_t lds_hi = lds0 + (uint32_t)((R / 2) * BUF);
    int ready_upto = 0; // chunks known to be written
    // Weight sets: set t = (chunk t / SW, stripe t % SW) lives in ws[t % 3] and is requested when
    // set t - 2 is about to be multiplied - two sets ahead of its use.
    uint4v ws[3][KT];
    load_w(ws[0], 0, 0);
    load_w(ws[1], 1 % SW, 1 / SW);
    // (The loop is left from the middle, not skipped through: on a path that skips the later
    // chunks and comes round again the compiler sees weight loads that were never waited for,
    // and waits for everything in flight wherever their registers are written next.)
    for (int ch = 0; ch < nch;) {
#pragma unroll
        for (int slot = 0; slot < R; ++slot) {
            if (ch >= ready_upto && !broken) {
                int spins = 0;
                for (;;) {
                    uint32_t seen = 0xffffffffu;
                    if (lane < NP) seen = __hip_atomic_load(written + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                    asm volatile("" ::: "memory");
                    static_assert(NP == 4, "four producer counters are looked at");
                    ready_upto = (int)min(min(__builtin_amdgcn_readlane(seen, 0), __builtin_amdgcn_readlane(seen, 1)),
                                          min(__builtin_amdgcn_readlane(seen, 2), __builtin_amdgcn_readlane(seen, 3)));
                    if (ch < ready_upto) break;
                    if (++spins > kSpinLimit) {
                        broken = true;
                        break;
                    }
                    __builtin_amdgcn_s_sleep(1);
                }
            }
            short8v xf[KT][CT];
            // (slot is a constant and lds0 / lds_hi live in registers throughout: the reads need no
            // address arithmetic - a fresh address register here was seen to cost a wait for all
            // weight loads in flight)
            const uint32_t base = (slot < R / 2 ? lds0 : lds_hi) + (uint32_t)((slot % (R / 2)) * BUF);
#pragma unroll
            for (int kt = 0; kt < KT; ++kt)
#pragma unroll
                for (int c = 0; c < CT; ++c) {
                    const short4v p0 = lds_read_tr(base + (uint32_t)(((kt * CT + c) * 2) << 9));
                    const short4v p1 = lds_read_tr(base + (uint32_t)(((kt * CT + c) * 2 + 1) << 9));
                    xf[kt][c] = __builtin_shufflevector(p0, p1, 0, 1, 2, 3, 4, 5, 6, 7);
                }
            // LDS executes a wavefront's operations in order: the counter store follows the reads
            asm volatile("" ::: "memory");
            if (lane == 0) __hip_atomic_store(read_upto + wave, (uint32_t)(ch + 1), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
#pragma unroll
            for (int i = 0; i < SW; ++i) {
                constexpr int kSets = 3;
                const int t = slot * SW + i;            // (compile-time: R * SW is a multiple of 3)
                const int far = i + 2;                  // set t + 2: stripe (i + 2) % SW of chunk ch + (i + 2) / SW
                load_w(ws[(t + 2) % kSets], far % SW, ch + far / SW);
                __builtin_amdgcn_sched_barrier(0);
                [[maybe_unused]] const uint32_t occ = occupancy(i, ch);
#pragma unroll
                for (int kt = 0; kt < KT; ++kt) {
                    if (SKIP && !((occ >> kt) & 1u)) continue; // (wave-uniform)
                    const short8v wv = __builtin_bit_cast(short8v, ws[t % kSets][kt]);
#pragma unroll
                    for (int c = 0; c < CT; ++c) acc[i][c] = mfma16<BF16>(xf[kt][c], wv, acc[i][c]);
                }
            }
            if (++ch >= nch) break;
        }
    }
    if (broken && lane == 0) atomicOr(a.err, 8u);

    // ---- stores, as in xstat_kernel: through 16 LDS rows of this wavefront, whole block rows out
    const int g = lane >> 4, n = lane & 15;
    constexpr int RB = 16 * CT * (int)sizeof(TY);
    constexpr int PR = RB / 16, RP = 256 / RB, NI = PR / 4;
    char *out_lds = smem + R * BUF + wave * OUT;
    TY *Yt = static_cast<TY *>(a.Y);
#pragma unroll
    for (int i = 0; i < SW; ++i) {
        const int stripe = s0 + i;
        if (a.ep.on) {
            const float b = epilogue_bias(a.ep, stripe * kStripe + n, a.M);
#pragma unroll
            for (int c = 0; c < CT; ++c) epilogue_tile(a.ep, acc[i][c], b);
        }
#pragma unroll
        for (int jp = 0; jp < NI; ++jp) {
            uint4v o;
            if constexpr (PixelMap<TY>::kPairs) {
                typedef TY ty8 __attribute__((ext_vector_type(8)));
                ty8 t8;
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    t8[t] = from_f32<TY>(acc[i][2 * jp][t]);
                    t8[4 + t] = from_f32<TY>(acc[i][2 * jp + 1][t]);
                }
                o = __builtin_bit_cast(uint4v, t8);
            } else {
                o = __builtin_bit_cast(uint4v, acc[i][jp]);
            }
            const int piece = (4 * jp + g) ^ ((n / RP) & (PR - 1));
            *reinterpret_cast<uint4v *>(out_lds + n * RB + piece * 16) = o;
        }
#pragma unroll
        for (int ii = 0; ii < NI; ++ii) {
            const int r = ii * (64 / PR) + lane / PR, lp = lane % PR;
            const uint4v o = *reinterpret_cast<const uint4v *>(out_lds + r * RB + ((lp ^ ((r / RP) & (PR - 1))) << 4));
            const int row = stripe * kStripe + r;
            const int px = bcol0 + lp * (16 / (int)sizeof(TY));
            if (stripe < s_end && row < a.M && px + 16 / (int)sizeof(TY) <= a.N)
                *reinterpret_cast<uint4v *>(Yt + (int64_t)row * a.ldy + px) = o;
        }
    }
}

// ------------------------------------------------------------------ launchers
template <bool BF16, typename TY, int CT, int KT>
ubp_status launch_xstat_inst(const TileArgs &a, int waves, hipStream_t st, bool dry) {
    // the X block, then 16 rows of output per wavefront: at most 32 + 32 KB, no attribute needed
    if (dry) return UBP_OK;
    const size_t lds = (size_t)KT * CT * 1024 + (size_t)waves * 256 * CT * sizeof(TY);
    const dim3 grid((unsigned)(8 * ((a.n_blocks + 7) / 8) * a.slices)), block((unsigned)waves * 64);
    if (a.skip) hipLaunchKernelGGL((xstat_kernel<BF16, TY, CT, KT, true>), grid, block, lds, st, a);
    else hipLaunchKernelGGL((xstat_kernel<BF16, TY, CT, KT, false>), grid, block, lds, st, a);
    return hipGetLastError() == hipSuccess ? UBP_OK : UBP_ERR_DEVICE;
}

template <bool BF16, typename TY>
ubp_status launch_xstat_t(const TileArgs &a, int CT, int KT, int waves, hipStream_t st, bool dry) {
#define UBP_XSTAT_CASE(CC, KK) \
    if (CT == CC && KT == KK) return launch_xstat_inst<BF16, TY, CC, KK>(a, waves, st, dry);
    UBP_XSTAT_CASE(2, 2) UBP_XSTAT_CASE(2, 4) UBP_XSTAT_CASE(2, 6) UBP_XSTAT_CASE(2, 8)
    UBP_XSTAT_CASE(4, 2) UBP_XSTAT_CASE(4, 4) UBP_XSTAT_CASE(4, 6) UBP_XSTAT_CASE(4, 8)
#undef UBP_XSTAT_CASE
    return UBP_ERR_UNSUPPORTED;
}

template <bool BF16, typename TY, int CT, int KT, int SW>
ubp_status launch_xchunk_inst(const TileArgs &a, hipStream_t st, bool dry) {
    constexpr int kChunkConsumers = kChunkStripes / SW;
    // the ring of chunks, 16 rows of output per multiplying wavefront, the progress counters
    const size_t lds = (size_t)kChunkRing * KT * CT * 1024 + (size_t)kChunkConsumers * 256 * CT * sizeof(TY) + 64;
    if (a.kt_total % KT != 0 || a.sps > kChunkStripes) return UBP_ERR_UNSUPPORTED;
    if (a.skip && SW * ((a.kt_total + 31) / 32) > 64) return UBP_ERR_UNSUPPORTED; // a wavefront's occupancy words sit in one register
    static LdsLimit limit_skip, limit_all; // per instantiation
    const ubp_status rc = a.skip ? limit_skip.raise(reinterpret_cast<const void *>(&xchunk_kernel<BF16, TY, CT, KT, SW, true>))
                                 : limit_all.raise(reinterpret_cast<const void *>(&xchunk_kernel<BF16, TY, CT, KT, SW, false>));
    if (rc != UBP_OK || dry) return rc;
    const dim3 grid((unsigned)(a.n_blocks * a.slices)), block((kChunkConsumers + kChunkProducers) * 64);
    if (a.skip) hipLaunchKernelGGL((xchunk_kernel<BF16, TY, CT, KT, SW, true>), grid, block, lds, st, a);
    else hipLaunchKernelGGL((xchunk_kernel<BF16, TY, CT, KT, SW, false>), grid, block, lds, st, a);
    return hipGetLastError() == hipSuccess ? UBP_OK : UBP_ERR_DEVICE;
}

template <bool BF16, typename TY>
ubp_status launch_xchunk_t(const TileArgs &a, int CT, int SW, hipStream_t st, bool dry) {
    constexpr int KT = 4; // chunks of 128 rows: X fragments, two weight sets and two chunks of X loads in 170 registers
#define UBP_XCHUNK_CASE(CC, SS) \
    if (CT == CC && SW == SS) return launch_xchunk_inst<BF16, TY, CC, KT, SS>(a, st, dry);
    UBP_XCHUNK_CASE(2, 2) UBP_XCHUNK_CASE(4, 2) UBP_XCHUNK_CASE(2, 4) UBP_XCHUNK_CASE(4, 4)
#undef UBP_XCHUNK_CASE
    return UBP_ERR_UNSUPPORTED;
}

} // namespace

ubp_status launch_xstat(const TileArgs &a, bool bf16, bool y_f32, int CT, int KT, int waves, void *stream, bool dry) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (bf16)
        return y_f32 ? launch_xstat_t<true, float>(a, CT, KT, waves, st, dry) : launch_xstat_t<true, __bf16>(a, CT, KT, waves, st, dry);
    return y_f32 ? launch_xstat_t<false, float>(a, CT, KT, waves, st, dry) : launch_xstat_t<false, _Float16>(a, CT, KT, waves, st, dry);
}

ubp_status launch_xchunk(const TileArgs &a, bool bf16, bool y_f32, int CT, int SW, void *stream, bool dry) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (bf16) return y_f32 ? launch_xchunk_t<true, float>(a, CT, SW, st, dry) : launch_xchunk_t<true, __bf16>(a, CT, SW, st, dry);
    return y_f32 ? launch_xchunk_t<false, float>(a, CT, SW, st, dry) : launch_xchunk_t<false, _Float16>(a, CT, SW, st, dry);
}

} // namespace ubp
