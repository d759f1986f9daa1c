// Gather kernel of the UBP library (fp16 / bf16): MFMA on aligned 16-row stripes, the rows of X
// that a row group needs staged in an LDS ring and read back transposed into operand order.
#include "ubp_device.h"

#include <cstdint>

namespace ubp {

namespace {

// The gather of step s+1 is issued before the MFMAs of step s (two operand buffers) except
// for the largest tile, where the second buffer would halve the wavefronts per SIMD.
constexpr bool stripe_pipelined(int G, int CT) { return G * CT < 32; }

constexpr int stripe_max_threads(int G, int CT, int D) {
    // accumulators + operand buffer(s) + D prefetched step records + addressing, in VGPRs
    // per lane; 512 per SIMD lane are shared by the wavefronts resident on the SIMD
    const int regs = 4 * G * CT + (stripe_pipelined(G, CT) ? 8 : 4) * CT + D * (2 + 4 * G) + (G == 1 ? 8 : 20);
    return regs <= 128 ? 1024 : regs <= 256 ? 512 : 256;
}

// One workgroup = 1, 2 or 4 producer wavefronts + up to 15 consumer wavefronts sharing one
// tile of 16*CT columns of X / Y.
//  * The producers stage X in 64-row chunks into a ring of LDS slots (ring row = X row mod
//    ring rows); each takes every n-th kilobyte of every chunk (one wavefront issues a direct
//    global->LDS load only every ~85 cycles, about 28 GB/s, so wide tiles need several).  FAST
//    (full column tile, 16-byte aligned rows): direct global->LDS loads, several chunks in
//    flight; otherwise (ragged last column tile, odd pitches) through registers with zero
//    fill past column N.  Each producer publishes one counter, the number of chunks whose
//    share it has landed (in order); a chunk is resident when all of them have passed it.
//    Every consumer publishes one counter of its own, the number of leading chunks it will
//    not read again; a slot is refilled once all of them have passed the chunk that occupies
//    it.  There is no workgroup barrier after start-up, so consumers drift apart by up to a
//    ring of rows and their uneven per-chunk work averages out.
//  * Each consumer owns one row group (G aligned 16-row stripes) and keeps its G*CT output
//    tiles in fp32 accumulators for the whole K loop (output stationary).  Its steps form a
//    contiguous stream of fixed-size records (LDS gather addresses, chunk bookkeeping,
//    weight fragments), fetched D steps ahead into a register ring.
//  * A step gathers 32 staged rows with two transposed LDS reads per lane and column tile
//    and issues one 16x16x32 MFMA per (stripe with nonzero weights, column tile).  The
//    gather of step s+1 is issued before the MFMAs of step s (two operand buffers), so LDS
//    latency is covered by matrix work of the same wavefront.  The product is formed
//    transposed (pixels x rows) so that a lane holds 4 consecutive pixels of one output row.
// Every wait is bounded: if one runs out the wavefront raises *err and goes on without
// waiting (wrong numbers, but the kernel always terminates).
template <bool BF16, typename TY, int G, int CT, int D, bool FAST>
__global__ __launch_bounds__(stripe_max_threads(G, CT, D)) void stripe_kernel(StripeArgs a) {
    constexpr int NTW = 16 * CT;
    constexpr int PITCH = ring_pitch(CT);
    constexpr int PIECES = 2 * CT; // 16-byte pieces per staged row
    constexpr int R = ring_slots(CT), KS = kSlotRows;
    constexpr int FG = G; // weight fragments per record
    constexpr int REC_BYTES = (128 + 256 * FG) * 4;
    constexpr int NINST = KS * PIECES / 64; // direct-to-LDS instructions per chunk (1 KB each)
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    uint32_t *published_p = reinterpret_cast<uint32_t *>(smem + a.ring_bytes); // [4] chunks landed, per producer
    uint32_t *released_p = published_p + 16;                                   // [16] per consumer wavefront

    // workgroup -> (column tile, workgroup row).  Consecutive workgroup ids go round-robin over
    // the 8 XCDs, so column tiles are dealt by id mod 8; an XCD then walks its tiles workgroup row
    // by workgroup row: the workgroups it runs at any time mostly share one row's step records,
    // which stay in its L2 (the largest layer's 6 MB of records against 4 MB of L2: 127 us instead
    // of 146 us compared with walking tile by tile, all rows of a tile together; layers whose
    // records fit anyway measure the same either way).
    const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
    const int my_tiles = (a.n_coltiles - xcd + 7) >> 3;
    if (local >= my_tiles * a.n_wgrows) return;
    const int ctile = a.ctile0 + xcd + 8 * (local % my_tiles);
    const int wgrow = local / my_tiles;

    const int NP = a.n_producers;
    const int NC = (int)(blockDim.x >> 6) - NP; // consumer wavefronts; the last NP wavefronts produce
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int col0 = ctile * NTW;
    // Ring mode: workgroup row w owns row groups (in heaviest-first order) w*NC .. w*NC+NC-1, one
    // per consumer: similar weights side by side keep the consumers of a ring in step.  Resident
    // mode: consumer v of workgroup row w walks entries (i*NC + v)*n_wgrows + w, i = 0, 1, ...
    const int q0 = a.resident ? wave * a.n_wgrows + wgrow : wgrow * NC + wave;
    const int q_step = a.resident ? NC * a.n_wgrows : a.nrg; // ring mode: one row group only
    const int active = a.resident ? NC : min(NC, a.nrg - wgrow * NC); // consumers the producers wait for (ring mode)

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
            // relaxed on purpose: the data is known to have landed (explicit vmcnt wait, or LDS
            // writes of this same wavefront, which LDS executes in order before this store); a
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
        const uint32_t ring0 = __builtin_amdgcn_readfirstlane(lds_address(smem));
        const int r_in = lane / PIECES, pp = lane % PIECES;
        constexpr int RPI = 64 / PIECES; // rows covered by one 1 KB instruction
        // FAST: byte offset of this lane's 16-byte piece for instruction i of a chunk, from the
        // chunk's first element.
        auto piece_offset = [&](int i, int rows) {
            const int r = i * RPI + r_in;                        // row inside the chunk
            const int u = (pp >> 1) ^ ring_swizzle(CT, r);       // logical unit stored at this position
            // rows past K load the chunk's last row again (never read): every chunk then issues
            // the same number of loads, which the in-order vmcnt bookkeeping relies on
            return (uint32_t)(((int64_t)min(r, rows - 1) * a.ldx + u * 16 + (pp & 1) * 8) * 2);
        };
        // Full chunks: the swizzle depends on the row modulo 8 at most and an instruction starts at
        // a multiple of 4 rows, so relative to the first row of ITS instruction a lane's offset
        // takes two values only (even / odd i); the wave-uniform base moves instead.
        const uint32_t voff_even = piece_offset(0, KS);
        const uint32_t voff_odd = NINST > 1 ? piece_offset(1, KS) - (uint32_t)((int64_t)RPI * a.ldx * 2) : voff_even;
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
            if constexpr (FAST) {
                const uint32_t lds0 = ring0 + (uint32_t)(slot * KS * PITCH);
                const uint16_t *base = a.X + (int64_t)k0 * a.ldx + col0; // wave-uniform
                if (rows == KS) {
                    for (int i = me; i < NINST; i += NP)
                        load16_to_lds(base + i * inst_stride, (i & 1) ? voff_odd : voff_even, lds0 + (uint32_t)i * 1024u);
                } else {
                    for (int i = me; i < NINST; i += NP)
                        load16_to_lds(base, piece_offset(i, rows), lds0 + (uint32_t)i * 1024u);
                }
                if (c + 1 - published > lag) {
                    wait_vmcnt_at_most(lag * per); // vector memory completes in order: chunks <= c - lag have landed
                    publish_upto(c + 1 - lag);
                }
            } else {
                for (int piece = lane + 64 * me; piece < rows * PIECES; piece += 64 * NP) {
                    const int r = piece / PIECES, q = piece % PIECES;
                    const int u = (q >> 1) ^ ring_swizzle(CT, slot * KS + r);
                    const int col = col0 + u * 16 + (q & 1) * 8;
                    const uint16_t *src = a.X + (int64_t)(k0 + r) * a.ldx + col;
                    uint4 v;
                    if (a.vec_ok && col + 8 <= a.N) {
                        v = *reinterpret_cast<const uint4 *>(src);
                    } else {
                        uint32_t e[8];
#pragma unroll
                        for (int t = 0; t < 8; ++t) e[t] = (col + t < a.N) ? (uint32_t)src[t] : 0u;
                        v = uint4{e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16)};
                    }
                    *reinterpret_cast<uint4 *>(smem + (slot * KS + r) * PITCH + q * 16) = v;
                }
                asm volatile("" ::: "memory");
                publish_upto(c + 1); // LDS executes this wavefront's writes above before the counter store
            }
        }
        // the tail: publish the chunks still in flight one by one as they land
        if constexpr (FAST) {
            while (published < a.nch) {
                wait_vmcnt_at_most((a.nch - published - 1) * per);
                publish_upto(published + 1);
            }
        }
        wait_vmcnt<0>();
        publish_upto(a.nch);
        return;
    }
    if (q0 >= a.nrg) return; // no row group for this wavefront

    // ------------------------------------------------------------------ consumer
    int q = q0;
    int rg = __builtin_amdgcn_readfirstlane(a.rg_order[q]);
    int s = __builtin_amdgcn_readfirstlane(a.rg_ptr[rg]);
    int s_all = __builtin_amdgcn_readfirstlane(a.rg_ptr[rg + 1]);

    float4v acc[G][CT];

    // Records are fetched through a buffer resource: the address of a load is the (wave-uniform)
    // byte offset of the record, kept in a scalar register and advanced by one record per step,
    // plus a fixed per-lane offset, so that a refill costs no vector ALU work.  The stream
    // carries D spare records at its end: refills run D steps ahead and simply read on past the
    // row group's last step (those records are never used).
    const __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t *>(a.stream), 0, (int)a.stream_bytes, 0x00020000);
    uint32_t info_x[D], info_y[D];
    uint4v wf[D][FG];
    uint32_t rec_next = 0;
    const uint32_t lane8 = (uint32_t)lane * 8u, lane16 = (uint32_t)lane * 16u;
    auto issue = [&](int d) {
        const uint2v inf = __builtin_bit_cast(uint2v, __builtin_amdgcn_raw_buffer_load_b64(rsrc, lane8, rec_next, 0));
        info_x[d] = inf[0];
        info_y[d] = inf[1];
#pragma unroll
        for (int j = 0; j < FG; ++j)
            wf[d][j] = __builtin_bit_cast(uint4v, __builtin_amdgcn_raw_buffer_load_b128(rsrc, lane16 + (uint32_t)(512 + j * 1024), rec_next, 0));
        rec_next += REC_BYTES;
    };

    int released = 0;   // chunks this wavefront has handed back
    int ready_upto = 0; // chunks known to be resident
    bool broken = false;
    uint32_t *mine = released_p + wave;
    auto wait_published = [&](int chunk) {
        if (chunk < ready_upto) return;
        int spins = 0;
        for (;;) {
            const uint32_t seen = flag_load(published_p + (lane & 3)); // unused producer slots were set to "all"
            ready_upto = (int)min(min(__builtin_amdgcn_readlane(seen, 0), __builtin_amdgcn_readlane(seen, 1)),
                                  min(__builtin_amdgcn_readlane(seen, 2), __builtin_amdgcn_readlane(seen, 3)));
            if (chunk < ready_upto) return;
            if (++spins > kSpinLimit) {
                broken = true; // reported after the stream loop (no global atomic inside it)
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
            // relaxed + a compiler barrier: the reads of these chunks returned before the MFMAs
            // that used them were issued, and LDS executes this wavefront's operations in order
            asm volatile("" ::: "memory");
            if (lane == 0) __hip_atomic_store(mine, (uint32_t)upto, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
    };

    // Gather of the step whose record sits in ring slot d into operand buffer b.  The record's
    // control word says which chunk must be resident and what may be handed back now (nothing
    // that the step before reads: its reads may still be in flight).  The reads are issued even
    // for an empty step (address 0, never used): the number of LDS operations between a gather
    // and its use is then the same on every path, which lets the compiler wait for exactly the
    // older gather instead of draining the newer one as well.
    constexpr bool PIPE = stripe_pipelined(G, CT);
    const uint32_t ring_base = __builtin_amdgcn_readfirstlane(lds_address(smem));
    short8v xf[PIPE ? 2 : 1][CT];
    auto stage_control = [&](int d, bool foreign, uint32_t &a_lo, uint32_t &a_hi) {
        // (foreign: the slot after the row group's last step holds another row group's record;
        // its gather is issued all the same, to valid addresses, and never used, but its control
        // word must not be acted on)
        uint32_t ctl = 0u;
        if (!foreign) ctl = __builtin_amdgcn_readfirstlane(info_y[d]);
        release_upto((int)(ctl >> 16));
        wait_published((int)(ctl & 0xffffu));
        // absolute LDS addresses: the ring starts at a multiple of 1 KB, so adding its base
        // commutes with the XOR that selects the column tile
        const uint32_t ix = info_x[d];
        a_lo = ring_base + ((ix & 0x3fffu) << 3);
        a_hi = ring_base + (((ix >> 14) & 0x3fffu) << 3);
    };
    auto stage = [&](int d, int b, bool foreign) {
        uint32_t a_lo, a_hi;
        stage_control(d, foreign, a_lo, a_hi);
#pragma unroll
        for (int c = 0; c < CT; ++c) {
            const short4v p0 = lds_read_tr(a_lo ^ (uint32_t)(c << 5));
            const short4v p1 = lds_read_tr(a_hi ^ (uint32_t)(c << 5));
            xf[b][c] = __builtin_shufflevector(p0, p1, 0, 1, 2, 3, 4, 5, 6, 7);
        }
    };
    // One stripe per wavefront: the step is straight-line code (an empty step multiplies a zero
    // fragment), and the gather of the next step is interleaved tile by tile with the MFMAs of
    // the current one.  A wavefront issues in order and an MFMA occupies the matrix pipe for 16
    // cycles: the two reads and two address operations placed behind each MFMA are then free
    // instead of queueing up after a burst of MFMAs.
    constexpr bool FUSED = PIPE && G == 1;
    auto fused = [&](int d, int dn, bool foreign) {
        uint32_t a_lo, a_hi;
        stage_control(dn, foreign, a_lo, a_hi);
        const int cb = d & 1, nb = cb ^ 1;
        const short8v wv = __builtin_bit_cast(short8v, wf[d][0]);
#pragma unroll
        for (int c = 0; c < CT; ++c) {
            const short4v p0 = lds_read_tr(a_lo ^ (uint32_t)(c << 5));
            const short4v p1 = lds_read_tr(a_hi ^ (uint32_t)(c << 5));
            xf[nb][c] = __builtin_shufflevector(p0, p1, 0, 1, 2, 3, 4, 5, 6, 7);
            acc[0][c] = mfma16<BF16>(xf[cb][c], wv, acc[0][c]);
            __builtin_amdgcn_sched_group_barrier(0x002, 2, 0); // two address operations
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0); // two LDS reads
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0); // one MFMA
        }
    };

    // The loop body is D steps with no exit in between (row groups hold a multiple of D steps,
    // the last ones possibly empty), and every step refills its ring slot unconditionally.  The number of
    // loads in flight behind a slot is then the same on every path into every step, which
    // lets the compiler wait with a partial vmcnt instead of draining the ring.
    static_assert(D == kPrefetchDepth && D % 2 == 0, "row groups are padded to a multiple of the prefetch depth");
    auto start_stream = [&]() { // first D records of the row group whose steps are s .. s_all
        rec_next = (uint32_t)s * (uint32_t)REC_BYTES;
        if (s < s_all) {
#pragma unroll
            for (int d = 0; d < D; ++d) {
                issue(d);
                __builtin_amdgcn_sched_barrier(0); // same issue order as in the loop, slot by slot
            }
            // Wait for them here, with a wait the compiler sees.  It may keep these first records
            // in other registers than the loop does and move them over; loads it believes pending
            // on registers that the loop body writes (the operand buffers) then cost a wait for
            // EVERYTHING in flight at the first step of every round of the loop - the record ring
            // was being drained every D steps.  (vmcnt(0), other counters untouched.)
            __builtin_amdgcn_s_waitcnt(0x0f70);
        }
    };
    start_stream();
    const int g = lane >> 4, n = lane & 15;
    TY *Yt = static_cast<TY *>(a.Y);
    for (;;) {
        // the row group this wavefront takes next (resident mode), looked up before the step loop:
        // the last D refills of the current row group then fetch ITS first D records, so that no
        // record latency is paid between two row groups
        const int q_next = q + q_step;
        const bool more = q_next < a.nrg;
        int rg_n = rg, s_n = s_all, s_all_n = s_all;
        if (more) {
            rg_n = __builtin_amdgcn_readfirstlane(a.rg_order[q_next]);
            s_n = __builtin_amdgcn_readfirstlane(a.rg_ptr[rg_n]);
            s_all_n = __builtin_amdgcn_readfirstlane(a.rg_ptr[rg_n + 1]);
        }
        bool handed_on = false; // the next row group's first records have been requested
#pragma unroll
        for (int j = 0; j < G; ++j)
#pragma unroll
            for (int c = 0; c < CT; ++c) acc[j][c] = float4v{0.f, 0.f, 0.f, 0.f};
        if (s < s_all) {
            if constexpr (PIPE) stage(0, 0, false);
            for (; s < s_all; s += D) {
                if (more && s + D >= s_all) {
                    rec_next = (uint32_t)s_n * (uint32_t)REC_BYTES;
                    handed_on = s_n < s_all_n;
                }
#pragma unroll
                for (int d = 0; d < D; ++d) {
                    if constexpr (FUSED) {
                        fused(d, (d + 1) % D, d + 1 == D && s + D >= s_all);
                        issue(d);
                        continue;
                    }
                    // the next step's gather first (or, with one operand buffer, this step's own)
                    if constexpr (PIPE) stage((d + 1) % D, (d + 1) & 1, d + 1 == D && s + D >= s_all);
                    else stage(d, 0, false);
                    const uint32_t mask = __builtin_amdgcn_readfirstlane(info_x[d] >> 28);
#pragma unroll
                    for (int j = 0; j < G; ++j) {
                        if (mask & (1u << j)) {
                            const short8v wv = __builtin_bit_cast(short8v, wf[d][j]);
#pragma unroll
                            for (int c = 0; c < CT; ++c) acc[j][c] = mfma16<BF16>(xf[PIPE ? (d & 1) : 0][c], wv, acc[j][c]);
                        }
                    }
                    issue(d);
                }
            }
        }
        // the next row group's first records are requested before this one's tiles are stored
        const int rg_done = rg;
        q = q_next;
        if (more) {
            rg = rg_n;
            s = s_n;
            s_all = s_all_n;
            if (!handed_on) start_stream();
        } else {
            release_upto(a.nch); // the last step's reads were consumed by its MFMAs
        }
        // ---- store: lane (g = lane/16, n = lane%16) holds pixels col0 + 16*c + 4*g + v of row
        // 16*(G*rg + j) + n.  Rows no block touches are stored as zeros like any other.
#pragma unroll
        for (int j = 0; j < G; ++j) {
            const int row = (rg_done * G + j) * kStripe + n;
            if (row >= a.M) continue;
            if (a.ep.on) {
                const float b = epilogue_bias(a.ep, row, a.M);
#pragma unroll
                for (int c = 0; c < CT; ++c) epilogue_tile(a.ep, acc[j][c], b);
            }
#pragma unroll
            for (int c = 0; c < CT; ++c) {
                const int px = col0 + 16 * c + 4 * g;
                TY *dst = Yt + (int64_t)row * a.ldy + px;
                if (a.vec_ok && px + 4 <= a.N) {
                    float v[4] = {acc[j][c][0], acc[j][c][1], acc[j][c][2], acc[j][c][3]};
                    store_row<TY, 4>(dst, v);
                } else {
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        if (px + v < a.N) dst[v] = from_f32<TY>(acc[j][c][v]);
                }
            }
        }
        if (!more) break;
    }
    if (broken && lane == 0) atomicOr(a.err, 2u);
}

// ------------------------------------------------------------------ launchers
template <bool BF16, typename TY, int G, int CT, bool FAST>
ubp_status launch_stripe_one(StripeArgs a, int ctile0, int n_coltiles, int waves, hipStream_t st, bool dry) {
    constexpr int D = kPrefetchDepth;
    const size_t lds = (size_t)a.ring_bytes + 32 * sizeof(uint32_t); // ring + the progress counters
    static LdsLimit limit; // per instantiation
    const ubp_status rc = limit.raise(reinterpret_cast<const void *>(&stripe_kernel<BF16, TY, G, CT, D, FAST>));
    if (rc != UBP_OK || dry) return rc;
    a.ctile0 = ctile0;
    a.n_coltiles = n_coltiles;
    const unsigned grid = 8u * (unsigned)((n_coltiles + 7) / 8) * (unsigned)a.n_wgrows;
    hipLaunchKernelGGL((stripe_kernel<BF16, TY, G, CT, D, FAST>), dim3(grid), dim3((unsigned)waves * 64), lds, st, a);
    return hipGetLastError() == hipSuccess ? UBP_OK : UBP_ERR_DEVICE;
}

template <bool BF16, typename TY, int G, int CT>
ubp_status launch_stripe_inst(const StripeArgs &a, int waves, hipStream_t st, bool dry) {
    if (waves * 64 > stripe_max_threads(G, CT, kPrefetchDepth)) return UBP_ERR_UNSUPPORTED;
    // full column tiles with aligned rows take the asynchronous staging path; a ragged last
    // tile (or everything, when rows are not 16-byte aligned) takes the synchronous one
    const int total = (a.N + 16 * CT - 1) / (16 * CT);
    // (the producer addresses a chunk with 32-bit lane offsets: 64 rows of ldx elements must fit)
    const int full = (a.vec_ok && a.ldx <= (int64_t(1) << 24)) ? a.N / (16 * CT) : 0;
    const int first = a.ctile0; // column tiles below this are someone else's (the block kernel's)
    ubp_status rc = UBP_OK;
    if (full > first) rc = launch_stripe_one<BF16, TY, G, CT, true>(a, first, full - first, waves, st, dry);
    if (rc == UBP_OK && total > std::max(full, first))
        rc = launch_stripe_one<BF16, TY, G, CT, false>(a, std::max(full, first), total - std::max(full, first), waves, st, dry);
    return rc;
}

template <bool BF16, typename TY>
ubp_status launch_stripe_t(const StripeArgs &a, int G, int CT, int waves, hipStream_t st, bool dry) {
#define UBP_SG_CASE(GG, CC) \
    if (G == GG && CT == CC) return launch_stripe_inst<BF16, TY, GG, CC>(a, waves, st, dry);
    UBP_SG_CASE(1, 2) UBP_SG_CASE(2, 2) UBP_SG_CASE(4, 2) UBP_SG_CASE(1, 4) UBP_SG_CASE(2, 4) UBP_SG_CASE(4, 4)
    UBP_SG_CASE(1, 8) UBP_SG_CASE(2, 8) UBP_SG_CASE(4, 8)
#undef UBP_SG_CASE
    return UBP_ERR_UNSUPPORTED;
}

} // namespace

int stripe_max_waves(int G, int CT) { return stripe_max_threads(G, CT, kPrefetchDepth) / 64; }

// a.ctile0 = first column tile this launch is responsible for (0: all of them)
ubp_status launch_stripe(const StripeArgs &a, bool bf16, bool y_f32, int G, int CT, int waves, void *stream, bool dry) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (bf16)
        return y_f32 ? launch_stripe_t<true, float>(a, G, CT, waves, st, dry) : launch_stripe_t<true, __bf16>(a, G, CT, waves, st, dry);
    return y_f32 ? launch_stripe_t<false, float>(a, G, CT, waves, st, dry) : launch_stripe_t<false, _Float16>(a, G, CT, waves, st, dry);
}

} // namespace ubp
