// Block kernel of the UBP library (fp16 / bf16, blocks of at most 16 rows): MFMA on aligned
// 16-row stripes with whole blocks as operands.
//
// A block of at most 16 rows has at most one row congruent to n modulo 16.  Stored by that
// residue - the paper's weight rotation (Section 4.2) with period 16 instead of the block
// height - ONE operand fragment serves both stripes an unaligned block reaches into: rows
// n >= o (o = first row modulo 16) belong to the stripe the block starts in, rows n < o to the
// next one, and the accumulator a row lands in is fixed at compile time, as in the paper.  The
// 16 columns of a block are rows of X; they are gathered from an LDS ring, transposed into
// operand order by the read itself.
#include "ubp_device.h"

#include <cstdint>

namespace ubp {

namespace {

constexpr int kBlkCT = 4; // 64-pixel column tiles (the ring geometry of CT = 4)


// One workgroup = NP producer wavefronts + up to 16 - NP consumer wavefronts on one tile of 64
// columns of X / Y.
//  * Producers stage X in 64-row chunks into a ring of LDS slots (ring row = X row mod 1024)
//    with direct global->LDS loads, several chunks in flight; each publishes one counter, the
//    number of chunks whose share it has landed.  Every consumer publishes one counter of its
//    own, the number of leading chunks it will not read again; a slot is refilled once all of
//    them have passed the chunk that occupies it.  No workgroup barrier after start-up.
//  * Each consumer owns one row group (a run of at most G aligned 16-row stripes; runs with many
//    blocks are shorter, so that the consumers of a workgroup carry similar loads) and keeps its
//    G x 4 output tiles in fp32 accumulators for the whole K loop (output stationary).  Its steps are a
//    contiguous run of 1 KB operand records, fetched D steps ahead into a register ring, and of
//    8-byte metadata words, fetched 64 steps at a time (one per lane) and handed out with
//    v_readlane: a step costs one vector memory instruction.
//  * A step = two half-blocks (16 columns each) that start in the same stripe: two transposed
//    LDS reads per pixel tile gather their 32 rows of X; two compares and eight selects split the
//    operand into its lower-stripe and upper-stripe part; 4 + 4 MFMAs (16x16x32).  A lane reads
//    the window row congruent to its entry number modulo 16 (the columns of a half are rotated
//    like its rows), so the ring's bank swizzle, which depends on the row modulo 8, is a lane
//    constant and an address is one select and one add away from the window's first row.
// Every wait is bounded: if one runs out the wavefront raises *err and goes on without waiting
// (wrong numbers, but the kernel always terminates).
template <bool BF16, typename TY, int G, int MAXT>
__global__ __launch_bounds__(MAXT) void blk_kernel(BlkArgs a) {
    constexpr int CT = kBlkCT;
    constexpr int NTW = 16 * CT;
    constexpr int PITCH = ring_pitch(CT);
    constexpr int PIECES = 2 * CT; // 16-byte pieces per staged row
    constexpr int R = ring_slots(CT), KS = kSlotRows, RR = ring_rows(CT);
    constexpr int D = kPrefetchDepth;
    constexpr int NINST = KS * PIECES / 64; // direct-to-LDS instructions per chunk (1 KB each)
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    uint32_t *published_p = reinterpret_cast<uint32_t *>(smem + a.ring_bytes); // [4] chunks landed, per producer
    uint32_t *released_p = published_p + 16;                                   // [16] per consumer wavefront

    // workgroup -> (column tile, workgroup row): consecutive workgroup ids go round-robin over the
    // 8 XCDs, so column tiles are dealt by id mod 8; an XCD then walks its tiles workgroup row by
    // workgroup row, so that what it runs at any time mostly shares one row's records in its L2.
    const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
    const int my_tiles = (a.n_coltiles - xcd + 7) >> 3;
    if (local >= my_tiles * a.n_wgrows) return;
    const int ctile = xcd + 8 * (local % my_tiles);
    const int wgrow = local / my_tiles;

    const int NP = a.n_producers;
    const int NC = (int)(blockDim.x >> 6) - NP; // consumer wavefronts; the last NP wavefronts produce
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int col0 = ctile * NTW;
    const int active = min(NC, a.nrg - wgrow * NC); // consumers the producers wait for

    // counters start at zero; the slots of producers that do not exist never hold anything back
    if (threadIdx.x < 32) published_p[threadIdx.x] = (threadIdx.x < 4 && (int)threadIdx.x >= NP) ? 0x7fffffffu : 0u;
    __syncthreads();

    // ------------------------------------------------------------------ producer
    if (wave >= NC) {
        const int me = wave - NC; // this producer takes instructions me, me + NP, ... of every chunk
        int published = 0;
        int free_upto = R; // chunks below this may be staged without asking: their slots are free
        bool broken = false;
        auto publish_upto = [&](int upto) {
            // relaxed on purpose: the data is known to have landed (explicit vmcnt wait); a
            // release here would make the compiler drain every load still in flight
            if (upto > published) {
                published = upto;
                if (lane == 0)
                    __hip_atomic_store(published_p + me, (uint32_t)upto, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            }
        };
        // lane w < active looks at consumer w's counter; the other lanes never hold anything back
        auto poll = [&]() -> uint32_t {
            uint32_t v = 0xffffffffu;
            if (lane < active) v = __hip_atomic_load(&released_p[lane], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            asm volatile("" ::: "memory");
            return v;
        };
        __builtin_amdgcn_s_setprio(3); // little work, but everyone else waits for it
        const int r_in = lane / PIECES, pp = lane % PIECES;
        constexpr int RPI = 64 / PIECES; // rows covered by one 1 KB instruction
        // byte offset of this lane's 16-byte piece for instruction i of a chunk, from the chunk's
        // first element
        auto piece_offset = [&](int i, int rows) {
            const int r = i * RPI + r_in;                        // row inside the chunk
            const int u = (pp >> 1) ^ ring_swizzle(CT, r);       // logical unit stored at this position
            // rows past K load the chunk's last row again (never read): every chunk then issues
            // the same number of loads, which the in-order vmcnt bookkeeping relies on
            return (uint32_t)(((int64_t)min(r, rows - 1) * a.ldx + u * 16 + (pp & 1) * 8) * 2);
        };
        // Full chunks: the swizzle depends on the row modulo 8 at most and an instruction covers 8
        // rows from a multiple of 8, so relative to the first row of ITS instruction a lane's
        // offset is the same for every instruction; the wave-uniform base moves instead.
        // (Staging through a register ring of ordinary loads instead - 24 loads of 1 KB in flight
        // per producer - was built and measured slower: 113 us against 101 us on the largest layer.)
        const uint32_t ring0 = __builtin_amdgcn_readfirstlane(lds_address(smem));
        const uint32_t voff = piece_offset(0, KS);
        const int per = NINST / NP;                    // instructions of a chunk that are mine
        const int lag = max(1, min(48 / per, R / 2));  // chunks kept in flight before they are published
        const int64_t inst_stride = (int64_t)RPI * a.ldx; // elements between the rows of two instructions
        for (int c = 0; c < a.nch; ++c) {
            const int slot = c % R;
            if (c >= free_upto && !broken) {
                // chunk c replaces chunk c - R: every consumer must have passed that one
                const uint32_t target = (uint32_t)(c - R + 1);
                uint32_t v = poll();
                if (__builtin_amdgcn_ballot_w64(v < target) != 0) {
                    // about to block: first publish every chunk already issued, the consumers
                    // this wait depends on may be waiting for one of them
                    wait_vmcnt<0>();
                    publish_upto(c);
                    int spins = 0;
                    do {
                        if (++spins > kSpinLimit) {
                            broken = true;
                            if (lane == 0) atomicOr(a.err, 1u);
                            break;
                        }
                        __builtin_amdgcn_s_sleep(2);
                        v = poll();
                    } while (__builtin_amdgcn_ballot_w64(v < target) != 0);
                }
                // how far the slowest consumer really is: saves asking again for the next chunks
                int ahead = 1;
                while (ahead < R && __builtin_amdgcn_ballot_w64(v < target + (uint32_t)ahead) == 0) ++ahead;
                free_upto = c + ahead;
            }
            const int k0 = c * KS;
            const int rows = min(KS, a.K - k0);
            const uint32_t lds0 = ring0 + (uint32_t)(slot * KS * PITCH);
            const uint16_t *base = a.X + (int64_t)k0 * a.ldx + col0; // wave-uniform
            if (rows == KS) {
                for (int i = me; i < NINST; i += NP) load16_to_lds(base + i * inst_stride, voff, lds0 + (uint32_t)i * 1024u);
            } else {
                for (int i = me; i < NINST; i += NP) load16_to_lds(base, piece_offset(i, rows), lds0 + (uint32_t)i * 1024u);
            }
            if (c + 1 - published > lag) {
                wait_vmcnt_at_most(lag * per); // vector memory completes in order: chunks <= c - lag have landed
                publish_upto(c + 1 - lag);
            }
        }
        // the tail: publish the chunks still in flight one by one as they land
        while (published < a.nch) {
            wait_vmcnt_at_most((a.nch - published - 1) * per);
            publish_upto(published + 1);
        }
        wait_vmcnt<0>();
        publish_upto(a.nch);
        return;
    }
    // Wavefront w runs on SIMD w mod 4 (in some order), and the producers, the last NP wavefronts,
    // take little of theirs: the SIMDs that host a producer have one consumer fewer and get the
    // workgroup's heaviest row groups (rg_order is sorted by decreasing work).
    int pos = wave;
    if (NP == 2 && NC == 14) pos = (wave & 2) ? (wave >> 2) * 2 + (wave & 1) : 6 + (wave >> 2) * 2 + (wave & 1);
    const int q = wgrow * NC + pos;
    if (q >= a.nrg) return; // no row group for this wavefront

    // ------------------------------------------------------------------ consumer
    const int rg = __builtin_amdgcn_readfirstlane(a.rg_order[q]);
    const int stripe0 = __builtin_amdgcn_readfirstlane(a.rg_order[a.nrg + rg]);          // the group's first stripe
    const int stripes = __builtin_amdgcn_readfirstlane(a.rg_order[a.nrg + rg + 1]) - stripe0; // at most G
    const int s_first = __builtin_amdgcn_readfirstlane(a.rg_ptr[rg]);
    const int s_all = __builtin_amdgcn_readfirstlane(a.rg_ptr[rg + 1]);

    float4v acc[G][CT];
#pragma unroll
    for (int j = 0; j < G; ++j)
#pragma unroll
        for (int c = 0; c < CT; ++c) acc[j][c] = float4v{0.f, 0.f, 0.f, 0.f};

    // Records and metadata are fetched through buffer resources: the address of a load is a
    // wave-uniform byte offset in a scalar register plus a fixed per-lane offset, so a refill
    // costs no vector ALU work.  Both arrays carry spare records at their ends: refills simply
    // read on past the row group's last step.
    const __amdgpu_buffer_rsrc_t rsrc_f =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t *>(a.frags), 0, (int)a.frag_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrc_m =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t *>(a.meta), 0, (int)a.meta_bytes, 0x00020000);
    const uint32_t lane8 = (uint32_t)lane * 8u, lane16 = (uint32_t)lane * 16u;
    uint4v wf[D];
    uint32_t rec_next = (uint32_t)s_first * 1024u;
    auto issue = [&](int d) {
        wf[d] = __builtin_bit_cast(uint4v, __builtin_amdgcn_raw_buffer_load_b128(rsrc_f, lane16, rec_next, 0));
        rec_next += 1024u;
    };
    uint32_t meta_next = (uint32_t)s_first * 8u;
    auto load_meta = [&]() {
        const uint2v m = __builtin_bit_cast(uint2v, __builtin_amdgcn_raw_buffer_load_b64(rsrc_m, lane8, meta_next, 0));
        meta_next += 512u;
        return m;
    };

    int released = 0;   // chunks this wavefront has handed back
    int ready_upto = 0; // chunks known to be resident
    bool broken = false;
    uint32_t *mine = released_p + pos; // (the producers look at positions 0 .. active - 1)
    auto wait_published = [&](int chunk) {
        if (chunk < ready_upto) return;
        int spins = 0;
        for (;;) {
            const uint32_t seen = flag_load(published_p + (lane & 3)); // unused producer slots were set to "all"
            ready_upto = (int)min(min(__builtin_amdgcn_readlane(seen, 0), __builtin_amdgcn_readlane(seen, 1)),
                                  min(__builtin_amdgcn_readlane(seen, 2), __builtin_amdgcn_readlane(seen, 3)));
            if (chunk < ready_upto) return;
            if (++spins > kSpinLimit) {
                broken = true; // reported after the step loop (no global atomic inside it)
                ready_upto = 0x7fffffff;
                return;
            }
            __builtin_amdgcn_s_sleep(1);
        }
    };
    // A counter only says "I will not read chunks below this again", so it can run ahead of the
    // producer (chunks this wavefront never reads) without harm.
    auto release_upto = [&](int upto) {
        if (upto > released) {
            released = upto;
            // relaxed + a compiler barrier: LDS executes this wavefront's operations in order, so
            // every read issued before this store is served before the store becomes visible
            asm volatile("" ::: "memory");
            if (lane == 0) __hip_atomic_store(mine, (uint32_t)upto, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
    };

    const uint32_t ring_base = __builtin_amdgcn_readfirstlane(lds_address(smem));
    const int g = lane >> 4, n = lane & 15;
    // this lane's part in a transposed read of a 16-row window: window row congruent to e modulo
    // 16, 8 bytes (4 pixels) number n & 3 of the 32-byte unit of pixel tile 0
    const uint32_t e = (uint32_t)(4 * g + (n >> 2));
    const uint32_t k0 = e * (uint32_t)PITCH + ((uint32_t)ring_swizzle(CT, (int)e) << 5) + (uint32_t)(n & 3) * 8u;

    if (s_first < s_all) {
        uint2v mcur = load_meta();
        uint2v mnext = load_meta();
#pragma unroll
        for (int d = 0; d < D; ++d) {
            issue(d);
            __builtin_amdgcn_sched_barrier(0); // same issue order as in the loop, slot by slot
        }
        // wait for them here, with a wait the compiler sees (vmcnt(0), other counters untouched):
        // loads it believes pending on registers that the loop body writes would otherwise cost a
        // wait for everything in flight at the first step of every round of the loop
        __builtin_amdgcn_s_waitcnt(0x0f70);
        {
            // nothing below the first step's windows is ever read: say so before the first wait, or
            // a row group whose first block lies beyond the ring would hold the producers back
            const uint32_t first = __builtin_amdgcn_readlane(mcur[0], 0);
            release_upto((int)(min(first & 0xffffu, first >> 16) >> 6));
        }
        int li = 0; // index of the round's first step within the metadata block
        for (int s = s_first; s < s_all; s += D) {
            if (li == 64) {
                li = 0;
                mcur = mnext;
                mnext = load_meta();
            }
#pragma unroll
            for (int d = 0; d < D; ++d) {
                const uint32_t m0 = __builtin_amdgcn_readlane(mcur[0], li + d);
                const uint32_t m1 = __builtin_amdgcn_readlane(mcur[1], li + d);
                const uint32_t aA = m0 & 0xffffu, aB = m0 >> 16;
                wait_published((int)((max(aA, aB) + 15u) >> 6));
                // ---- gather: the 16 + 16 window rows, four pixel tiles
                short8v xf[CT];
                {
                    const uint32_t rA = aA & (uint32_t)(RR - 1), rB = aB & (uint32_t)(RR - 1);
                    const uint32_t loA = ring_base + (rA & ~15u) * (uint32_t)PITCH;
                    const uint32_t hiA = ring_base + (((rA & ~15u) + 16u) & (uint32_t)(RR - 1)) * (uint32_t)PITCH;
                    const uint32_t loB = ring_base + (rB & ~15u) * (uint32_t)PITCH;
                    const uint32_t hiB = ring_base + (((rB & ~15u) + 16u) & (uint32_t)(RR - 1)) * (uint32_t)PITCH;
                    const uint32_t tA = (e < (rA & 15u) ? hiA : loA) + k0;
                    const uint32_t tB = (e < (rB & 15u) ? hiB : loB) + k0;
#pragma unroll
                    for (int c = 0; c < CT; ++c) {
                        const short4v p0 = lds_read_tr(tA ^ (uint32_t)(c << 5));
                        const short4v p1 = lds_read_tr(tB ^ (uint32_t)(c << 5));
                        xf[c] = __builtin_shufflevector(p0, p1, 0, 1, 2, 3, 4, 5, 6, 7);
                    }
                }
                // hand back the chunks that no later step reads: LDS executes this wavefront's
                // operations in order, so the reads above are served before the counter moves
                release_upto((int)(m1 >> 22));
                // ---- the operand's two parts: rows n >= o stay in the stripe the block starts in
                const uint32_t oA = m1 & 15u, oB = (m1 >> 4) & 15u;
                const uint4v f = wf[d];
                const bool inA = (uint32_t)n >= oA, inB = (uint32_t)n >= oB;
                const uint4v wl = {inA ? f[0] : 0u, inA ? f[1] : 0u, inB ? f[2] : 0u, inB ? f[3] : 0u};
                const uint4v wh = {inA ? 0u : f[0], inA ? 0u : f[1], inB ? 0u : f[2], inB ? 0u : f[3]};
                const short8v wlo = __builtin_bit_cast(short8v, wl), whi = __builtin_bit_cast(short8v, wh);
                const uint32_t jj = (m1 >> 8) & 15u;
                const bool do_hi = (m1 & 0x2000u) != 0;
#pragma unroll
                for (int j1 = 0; j1 <= G; ++j1) {
                    if (jj == (uint32_t)j1) {
                        constexpr int kLast = G - 1;
                        const int jl = j1 >= 1 ? j1 - 1 : 0, jh = j1 < G ? j1 : kLast; // (clamped: the guarded-out uses are dead code)
                        if (j1 >= 1) {
#pragma unroll
                            for (int c = 0; c < CT; ++c) acc[jl][c] = mfma16<BF16>(xf[c], wlo, acc[jl][c]);
                        }
                        if (j1 < G && do_hi) {
#pragma unroll
                            for (int c = 0; c < CT; ++c) acc[jh][c] = mfma16<BF16>(xf[c], whi, acc[jh][c]);
                        }
                    }
                }
                issue(d);
            }
            li += D;
        }
    }
    release_upto(a.nch); // the last step's reads were consumed by its MFMAs
    if (broken && lane == 0) atomicOr(a.err, 2u);

    // ---- store: lane (g = lane/16, n = lane%16) holds pixels col0 + 16*c + 4*g + v of row
    // 16*(stripe0 + j) + n, j < stripes.  Rows no block touches are stored as zeros like any other.
    TY *Yt = static_cast<TY *>(a.Y);
    // the epilogue (bias of the lane's row, clamp) is applied tile by tile on the way out
    const bool fused = a.ep.on != 0;
    if constexpr (sizeof(TY) == 2) {
        if (a.out_bytes != 0) {
            // A 16-bit tile straight from the accumulators is 8 bytes per lane, 32-byte runs per
            // row.  Through 16 LDS rows of this wavefront (16-byte pieces XOR-swizzled by the row
            // against bank conflicts; one wavefront writes and reads, LDS keeps its order) an
            // instruction stores whole rows of the tile, 16 bytes per lane.
            constexpr int RB = 16 * CT * 2;   // bytes per row of the tile
            constexpr int PR = RB / 16;       // 16-byte pieces per row
            constexpr int RP = 256 / RB;      // rows per 256 bytes (one pass over the banks)
            constexpr int NI = PR / 4;        // store instructions per stripe
            char *scratch = smem + a.ring_bytes + 32 * sizeof(uint32_t) + wave * a.out_bytes;
#pragma unroll
            for (int j = 0; j < G; ++j) {
                if (j >= stripes) break;
                const float bj = fused ? epilogue_bias(a.ep, (stripe0 + j) * kStripe + n, a.M) : 0.f;
#pragma unroll
                for (int c = 0; c < CT; ++c) {
                    typedef TY ty4 __attribute__((ext_vector_type(4)));
                    ty4 o;
                    if (fused) epilogue_tile(a.ep, acc[j][c], bj);
#pragma unroll
                    for (int v = 0; v < 4; ++v) o[v] = from_f32<TY>(acc[j][c][v]);
                    const int piece = (2 * c + (g >> 1)) ^ ((n / RP) & (PR - 1));
                    *reinterpret_cast<ty4 *>(scratch + n * RB + piece * 16 + (g & 1) * 8) = o;
                }
#pragma unroll
                for (int i = 0; i < NI; ++i) {
                    const int r = i * (64 / PR) + lane / PR, lp = lane % PR;
                    const uint4v o = *reinterpret_cast<const uint4v *>(scratch + r * RB + ((lp ^ ((r / RP) & (PR - 1))) << 4));
                    const int row = (stripe0 + j) * kStripe + r;
                    if (row < a.M) *reinterpret_cast<uint4v *>(Yt + (int64_t)row * a.ldy + col0 + lp * 8) = o;
                }
            }
            return;
        }
    }
#pragma unroll
    for (int j = 0; j < G; ++j) {
        const int row = (stripe0 + j) * kStripe + n;
        if (j >= stripes || row >= a.M) continue;
        const float bj = fused ? epilogue_bias(a.ep, row, a.M) : 0.f;
#pragma unroll
        for (int c = 0; c < CT; ++c) {
            const int px = col0 + 16 * c + 4 * g;
            TY *dst = Yt + (int64_t)row * a.ldy + px;
            if (fused) epilogue_tile(a.ep, acc[j][c], bj);
            float v[4] = {acc[j][c][0], acc[j][c][1], acc[j][c][2], acc[j][c][3]};
            store_row<TY, 4>(dst, v);
        }
    }
}

template <bool BF16, typename TY, int G, int MAXT>
ubp_status launch_blk_inst(BlkArgs a, int waves, hipStream_t st, bool dry) {
    if (waves * 64 > MAXT) return UBP_ERR_UNSUPPORTED;
    // ring + the progress counters + (16-bit Y, where it fits) the consumers' output rows
    if (sizeof(TY) == 2) {
        const size_t want = (size_t)16 * 16 * kBlkCT * 2;
        if ((size_t)a.ring_bytes + 32 * sizeof(uint32_t) + (size_t)(waves - a.n_producers) * want <= 160 * 1024) a.out_bytes = (int)want;
    }
    const size_t lds = (size_t)a.ring_bytes + 32 * sizeof(uint32_t) + (size_t)(waves - a.n_producers) * a.out_bytes;
    static LdsLimit limit; // per instantiation
    const ubp_status rc = limit.raise(reinterpret_cast<const void *>(&blk_kernel<BF16, TY, G, MAXT>));
    if (rc != UBP_OK || dry) return rc;
    const unsigned grid = 8u * (unsigned)((a.n_coltiles + 7) / 8) * (unsigned)a.n_wgrows;
    hipLaunchKernelGGL((blk_kernel<BF16, TY, G, MAXT>), dim3(grid), dim3((unsigned)waves * 64), lds, st, a);
    return hipGetLastError() == hipSuccess ? UBP_OK : UBP_ERR_DEVICE;
}

template <bool BF16, typename TY>
ubp_status launch_blk_t(const BlkArgs &a, int G, int waves, hipStream_t st, bool dry) {
    if (G == 5) return launch_blk_inst<BF16, TY, 5, 1024>(a, waves, st, dry);
    if (G == 4) return launch_blk_inst<BF16, TY, 4, 1024>(a, waves, st, dry);
    if (G == 2) return launch_blk_inst<BF16, TY, 2, 1024>(a, waves, st, dry);
    return UBP_ERR_UNSUPPORTED;
}

} // namespace

int blk_max_waves(int G) { return (G == 2 || G == 4 || G == 5) ? 16 : 0; }

ubp_status launch_blk(const BlkArgs &a, bool bf16, bool y_f32, int G, int waves, void *stream, bool dry) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    // 64 rows of ldx elements must fit the producer's 32-bit lane offsets
    if (a.ldx > (int64_t(1) << 24)) return UBP_ERR_UNSUPPORTED;
    if (bf16) return y_f32 ? launch_blk_t<true, float>(a, G, waves, st, dry) : launch_blk_t<true, __bf16>(a, G, waves, st, dry);
    return y_f32 ? launch_blk_t<false, float>(a, G, waves, st, dry) : launch_blk_t<false, _Float16>(a, G, waves, st, dry);
}

} // namespace ubp
