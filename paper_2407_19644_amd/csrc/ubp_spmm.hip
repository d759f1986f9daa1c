// Device side of the UBP library for gfx950: upload of the packed weights, the two
// SpMM kernels and their launch logic.
//
//  * wros_kernel  - vector-ALU kernel that follows the paper's WROS dataflow literally
//                   (Section 4.2): output-stationary accumulators, weights pre-rotated so
//                   that the accumulator of output row i is the compile-time slot i mod bh,
//                   one output row stored per start row, epilogue for the last bh-1 rows.
//                   Used for fp32 and as the reference GPU path for every dtype.
//  * stripe_kernel - MFMA kernel for fp16 / bf16.  A matrix instruction produces 16 output
//                   rows at once, so the accumulators are aligned 16-row stripes and an
//                   unaligned block contributes to (at most) two of them through
//                   zero-filled operand rows; the gathered X rows are staged in LDS and
//                   read back transposed (ds_read_b64_tr_b16) straight into operand order.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "ubp_internal.h"

namespace ubp {

namespace {

typedef short short4v __attribute__((ext_vector_type(4)));
typedef short short8v __attribute__((ext_vector_type(8)));
typedef _Float16 half8v __attribute__((ext_vector_type(8)));
typedef __bf16 bf8v __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));

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

template <class T>
bool dev_copy(T **dst, const T *src, size_t n, int64_t *bytes) {
    const size_t sz = std::max<size_t>(n, 1) * sizeof(T);
    if (hipMalloc(reinterpret_cast<void **>(dst), sz) != hipSuccess) { *dst = nullptr; return false; }
    *bytes += (int64_t)sz;
    if (n && hipMemcpy(*dst, src, n * sizeof(T), hipMemcpyHostToDevice) != hipSuccess) return false;
    return true;
}

// ------------------------------------------------------------------ element helpers
template <typename T> __device__ __forceinline__ float to_f32(T v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f32(float v) { return (T)v; } // round to nearest even

template <typename T, int VEC> struct VecOf { typedef T type __attribute__((ext_vector_type(VEC))); };
template <typename T> struct VecOf<T, 1> { typedef T type; };

template <typename T, int VEC>
__device__ __forceinline__ void load_row(const T *p, float (&out)[VEC]) {
    if constexpr (VEC == 1) {
        out[0] = to_f32(*p);
    } else {
        typedef typename VecOf<T, VEC>::type V;
        V v = *reinterpret_cast<const V *>(p);
#pragma unroll
        for (int t = 0; t < VEC; ++t) out[t] = to_f32((T)v[t]);
    }
}

template <typename T, int VEC>
__device__ __forceinline__ void store_row(T *p, const float (&in)[VEC]) {
    if constexpr (VEC == 1) {
        *p = from_f32<T>(in[0]);
    } else {
        typedef typename VecOf<T, VEC>::type V;
        V v;
#pragma unroll
        for (int t = 0; t < VEC; ++t) v[t] = from_f32<T>(in[t]);
        *reinterpret_cast<V *>(p) = v;
    }
}

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
                                                  TY *__restrict__ Y, int64_t ldy, int M, int N, int bw, int rpr) {
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
            if (i >= lo) store_row<TY, VEC>(Y + (int64_t)i * ldy + col, acc[u]);
#pragma unroll
            for (int v = 0; v < VEC; ++v) acc[u][v] = 0.f;
        }
    }
}

// ------------------------------------------------------------------ MFMA stripe kernel
struct StripeArgs {
    const int32_t *rg_ptr;
    const int32_t *rg_order;
    const uint32_t *stream;
    const uint16_t *X;
    void *Y;
    int64_t ldx, ldy;
    int M, K, N;
    int nrg, nch;            // row groups, 64-row chunks of X
    int ring_bytes;          // bytes of the LDS ring actually used (all of K when K is shorter than the ring)
    int ctile0, n_coltiles;  // first column tile of this launch, number of tiles in it
    int n_wgrows;
    int vec_ok;              // X and Y allow 16-byte vector access on every row
    uint32_t *err;           // set to nonzero when a bounded wait runs out
};

template <bool BF16>
__device__ __forceinline__ float4v mfma16(short8v a, short8v b, float4v c) {
    if constexpr (BF16)
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf8v, a), __builtin_bit_cast(bf8v, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8v, a), __builtin_bit_cast(half8v, b), c, 0, 0, 0);
}

__device__ __forceinline__ short4v lds_read_tr(const char *lds_base, int byte_off) {
    typedef __attribute__((address_space(3))) short4v *lds_ptr;
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(lds_base + byte_off));
}

// 16 bytes per lane from global memory straight into LDS at lds_base + 16 * lane (lds_base
// wave-uniform).  Written as inline assembly on purpose: the compiler then does not treat
// the load as a pending LDS write, which would make it wait for ALL outstanding vector
// memory operations before every LDS read.  Ordering against the LDS reads of the staged
// data is done by hand (wait_vmcnt, then the slot's ready flag).
__device__ __forceinline__ void load16_to_lds(const void *gbase, uint32_t lane_off, uint32_t lds_base) {
    // address = gbase (wave-uniform, in SGPRs) + lane_off (32-bit per-lane byte offset)
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(lane_off), "s"(gbase), "s"(lds_base));
}

__device__ __forceinline__ uint32_t lds_address(const char *p) {
    typedef __attribute__((address_space(3))) const char *lds_ptr;
    return (uint32_t)(uintptr_t)(lds_ptr)p;
}

template <int N> __device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt immediate out of range");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

__device__ __forceinline__ uint32_t flag_load(uint32_t *p) {
    return __hip_atomic_load(p, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP);
}

constexpr int kSpinLimit = 1 << 22; // polls before a wait gives up (each poll is >= 100 cycles)

constexpr int stripe_max_threads(int G, int CT, int D) {
    // accumulators + operand fragments + D prefetched step records, in VGPRs per lane
    return (4 * G * CT + 4 * CT + D * (2 + 4 * G) + 24) <= 128 ? 1024 : 512;
}

// One workgroup = one producer wavefront + up to 15 consumer wavefronts sharing one tile of
// 16*CT columns of X / Y.
//  * The producer stages X in 64-row chunks into a ring of LDS slots (ring row = X row mod
//    ring rows).  FAST (full column tile, 16-byte aligned rows): direct global->LDS loads,
//    several chunks in flight; otherwise (ragged last column tile, odd pitches) through
//    registers with zero fill past column N.  A chunk's slot is refilled only after every
//    consumer has released the chunk that occupied it (done counters), and a chunk is read
//    only after the producer has published it (ready generation numbers); there is no
//    workgroup barrier after start-up, so consumers drift apart by up to a ring of rows and
//    their uneven per-chunk work averages out.
//  * Each consumer owns one row group (G aligned 16-row stripes) and keeps its G*CT output
//    tiles in fp32 accumulators for the whole K loop (output stationary).  Its steps form a
//    contiguous stream of fixed-size records (LDS gather addresses, chunk bookkeeping,
//    weight fragments), fetched D steps ahead into a register ring.
//  * A step gathers 32 staged rows with two transposed LDS reads per lane and column tile
//    and issues one 16x16x32 MFMA per (stripe with nonzero weights, column tile).  The
//    product is formed transposed (pixels x rows) so that a lane holds 4 consecutive
//    pixels of one output row.
// Every wait is bounded: if one runs out the wavefront raises *err and goes on without
// waiting (wrong numbers, but the kernel always terminates).
template <bool BF16, typename TY, int G, int CT, int D, bool FAST>
__global__ __launch_bounds__(stripe_max_threads(G, CT, D)) void stripe_kernel(StripeArgs a) {
    constexpr int NTW = 16 * CT;
    constexpr int PITCH = ring_pitch(CT);
    constexpr int PIECES = 2 * CT; // 16-byte pieces per staged row
    constexpr int RR = ring_rows(CT), R = ring_slots(CT), KS = kSlotRows;
    constexpr int REC_DW = 128 + 256 * G;
    constexpr int NINST = KS * PIECES / 64; // direct-to-LDS instructions per chunk (1 KB each)
    constexpr int LAG = 56 / NINST;         // chunks kept in flight before their readiness is published
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    uint32_t *ready = reinterpret_cast<uint32_t *>(smem + a.ring_bytes); // [R] generation + 1 of the chunk in the slot
    uint32_t *done = ready + R;                                        // [R] releases received, all generations

    // workgroup -> (column tile, workgroup row); consecutive workgroup ids go round-robin
    // over the 8 XCDs, so tiles are dealt by id mod 8 and all row groups of one column tile
    // run on one XCD at about the same time: they share the X tile in that XCD's L2, which
    // measured better than the alternative of keeping one workgroup row's step records in L2
    // and streaming X once per workgroup row.
    const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
    const int my_tiles = (a.n_coltiles - xcd + 7) >> 3;
    if (local >= my_tiles * a.n_wgrows) return;
    const int ctile = a.ctile0 + xcd + 8 * (local / a.n_wgrows);
    const int wgrow = local % a.n_wgrows;

    const int NC = (int)(blockDim.x >> 6) - 1; // consumer wavefronts; the last wavefront produces
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int col0 = ctile * NTW;
    const int rg0 = wgrow * NC;
    const int active = min(NC, a.nrg - rg0); // consumers that own a row group

    if (threadIdx.x < 2 * R) ready[threadIdx.x] = 0u; // ready[] and done[]
    __syncthreads();

    // ------------------------------------------------------------------ producer
    if (wave == NC) {
        int published = 0;
        bool broken = false;
        auto publish_upto = [&](int upto) {
            while (published < upto) {
                // relaxed on purpose: the data is known to have landed (explicit vmcnt wait, or LDS
                // writes of this same wavefront, which LDS executes in order before this store); a
                // release here would make the compiler drain every load still in flight
                if (lane == 0)
                    __hip_atomic_store(&ready[published % R], (uint32_t)(published / R + 1), __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_WORKGROUP);
                ++published;
            }
        };
        __builtin_amdgcn_s_setprio(3); // little work, but everyone else waits for it
        const uint32_t ring0 = __builtin_amdgcn_readfirstlane(lds_address(smem));
        const int r_in = lane / PIECES, pp = lane % PIECES;
        // FAST: byte offset of this lane's 16-byte piece from the chunk's first element, for each
        // of the NINST instructions of a chunk.  The swizzle repeats every 8 rows at most, chunks
        // are 64 rows, so the offsets are the same for every chunk; only the base moves.
        uint32_t voff[NINST];
        auto piece_offset = [&](int i, int rows) {
            const int r = i * (64 / PIECES) + r_in;              // row inside the chunk
            const int u = (pp >> 1) ^ ring_swizzle(CT, r);       // logical unit stored at this position
            // rows past K load the chunk's last row again (never read): every chunk then issues
            // exactly NINST loads, which the in-order vmcnt bookkeeping relies on
            return (uint32_t)(((int64_t)min(r, rows - 1) * a.ldx + u * 16 + (pp & 1) * 8) * 2);
        };
        if constexpr (FAST) {
#pragma unroll
            for (int i = 0; i < NINST; ++i) voff[i] = piece_offset(i, KS);
        }
        for (int c = 0; c < a.nch; ++c) {
            const int slot = c % R;
            if (c >= R && !broken) {
                const uint32_t target = (uint32_t)active * (uint32_t)(c / R);
                if (flag_load(&done[slot]) < target) {
                    // about to block: first publish every chunk already issued, the consumers
                    // this wait depends on may be waiting for one of them
                    wait_vmcnt<0>();
                    publish_upto(c);
                    int spins = 0;
                    while (flag_load(&done[slot]) < target) {
                        if (++spins > kSpinLimit) {
                            broken = true;
                            if (lane == 0) atomicOr(a.err, 1u);
                            break;
                        }
                        __builtin_amdgcn_s_sleep(2);
                    }
                }
            }
            const int k0 = c * KS;
            const int rows = min(KS, a.K - k0);
            if constexpr (FAST) {
                const uint32_t lds0 = ring0 + (uint32_t)(slot * KS * PITCH);
                const uint16_t *base = a.X + (int64_t)k0 * a.ldx + col0; // wave-uniform
                if (rows == KS) {
#pragma unroll
                    for (int i = 0; i < NINST; ++i) load16_to_lds(base, voff[i], lds0 + (uint32_t)i * 1024u);
                } else {
#pragma unroll
                    for (int i = 0; i < NINST; ++i) load16_to_lds(base, piece_offset(i, rows), lds0 + (uint32_t)i * 1024u);
                }
                if (c + 1 - published > LAG) {
                    wait_vmcnt<LAG * NINST>(); // vector memory completes in order: chunks <= c - LAG have landed
                    publish_upto(c + 1 - LAG);
                }
            } else {
                for (int piece = lane; piece < rows * PIECES; piece += 64) {
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
                publish_upto(c + 1); // LDS executes this wavefront's writes above before the flag store
            }
        }
        wait_vmcnt<0>();
        publish_upto(a.nch);
        return;
    }
    if (wave >= active) return; // no row group left for this wavefront

    // ------------------------------------------------------------------ consumer
    const int rg = __builtin_amdgcn_readfirstlane(a.rg_order[rg0 + wave]);
    int s = __builtin_amdgcn_readfirstlane(a.rg_ptr[rg]);
    const int s_all = __builtin_amdgcn_readfirstlane(a.rg_ptr[rg + 1]);

    float4v acc[G][CT];
#pragma unroll
    for (int j = 0; j < G; ++j)
#pragma unroll
        for (int c = 0; c < CT; ++c) acc[j][c] = float4v{0.f, 0.f, 0.f, 0.f};

    // Record of step t: wave-uniform base (kept in SGPRs, advanced by one record per step) plus
    // a fixed per-lane offset, so that a refill costs no vector ALU work.  The stream carries D
    // spare records at its end: refills run D steps ahead and simply read on past the row
    // group's last step (those records are never used).
    uint2 info[D];
    uint4 wf[D][G];
    const char *rec_next = reinterpret_cast<const char *>(a.stream) + (int64_t)s * (REC_DW * 4);
    const uint32_t lane8 = (uint32_t)lane * 8u, lane16 = (uint32_t)lane * 16u;
    auto issue = [&](int d) {
        info[d] = *reinterpret_cast<const uint2 *>(rec_next + lane8);
#pragma unroll
        for (int j = 0; j < G; ++j) wf[d][j] = *reinterpret_cast<const uint4 *>(rec_next + 512 + j * 1024 + lane16);
        rec_next += REC_DW * 4;
    };

    int released = 0;   // chunks this wavefront has released
    int ready_upto = 0; // chunks known to be published
    bool broken = false;
    auto wait_published = [&](int chunk) {
        if (chunk < ready_upto || broken) return;
        const uint32_t want = (uint32_t)(chunk / R + 1);
        int spins = 0;
        while (flag_load(&ready[chunk % R]) < want) {
            if (++spins > kSpinLimit) {
                broken = true; // reported after the stream loop (no global atomic inside it)
                return;
            }
            __builtin_amdgcn_s_sleep(1);
        }
        ready_upto = chunk + 1;
    };
    // Releases go in chunk order, each only after the chunk has been published: the producer's
    // done counters then never contain a release of a chunk that is not in the ring yet (a
    // wavefront whose steps skip chunks would otherwise release them ahead of time and let the
    // producer refill a slot another wavefront still reads).
    auto release_upto = [&](int upto) {
        // relaxed + a compiler barrier: the reads of these chunks returned before the MFMAs that
        // used them were issued, and LDS executes this wavefront's operations in order; a release
        // would make the compiler drain the prefetch ring at every chunk
        asm volatile("" ::: "memory");
        while (released < upto) {
            wait_published(released);
            if (lane == 0)
                __hip_atomic_fetch_add(&done[released % R], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            ++released;
        }
    };

    // The loop body is D steps with no exit in between (row groups hold a multiple of D steps,
    // the last ones possibly empty), and every step refills its ring slot unconditionally.  The number of
    // loads in flight behind a slot is then the same on every path into every step, which
    // lets the compiler wait with a partial vmcnt instead of draining the ring.
    static_assert(D == kPrefetchDepth, "row groups are padded to a multiple of the prefetch depth");
    if (s < s_all) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            issue(d);
            __builtin_amdgcn_sched_barrier(0); // same issue order as in the loop, slot by slot
        }
        for (; s < s_all; s += D) {
#pragma unroll
            for (int d = 0; d < D; ++d) {
                const uint2 inf = info[d];
                const uint32_t ctl = __builtin_amdgcn_readfirstlane(inf.y);
                const int need = (int)(ctl & 0xffffu), rel = (int)(ctl >> 16);
                // first give back what no later step reads (their reads were consumed by earlier
                // MFMAs), then wait for the highest chunk this step reads; chunks are published in
                // order, so that covers every chunk of the step.  Releasing first matters: the
                // producer may need exactly those slots to bring the awaited chunk in.
                release_upto(rel);
                wait_published(need);
                const uint32_t mask = __builtin_amdgcn_readfirstlane(inf.x >> 28);
                if (mask) {
                    const int a_lo = (int)((inf.x & 0x3fffu) << 3), a_hi = (int)(((inf.x >> 14) & 0x3fffu) << 3);
                    short8v xf[CT];
#pragma unroll
                    for (int c = 0; c < CT; ++c) {
                        const short4v p0 = lds_read_tr(smem, a_lo ^ (c << 5));
                        const short4v p1 = lds_read_tr(smem, a_hi ^ (c << 5));
                        xf[c] = __builtin_shufflevector(p0, p1, 0, 1, 2, 3, 4, 5, 6, 7);
                    }
#pragma unroll
                    for (int j = 0; j < G; ++j) {
                        if (mask & (1u << j)) {
                            const short8v wv = __builtin_bit_cast(short8v, wf[d][j]);
#pragma unroll
                            for (int c = 0; c < CT; ++c) acc[j][c] = mfma16<BF16>(xf[c], wv, acc[j][c]);
                        }
                    }
                }
                issue(d);
            }
        }
    }
    if (broken && lane == 0) atomicOr(a.err, 2u);
    // the producer counts a release from every consumer for every chunk
    release_upto(a.nch);

    // ---- store: lane (g = lane/16, n = lane%16) holds pixels col0 + 16*c + 4*g + v of row
    // 16*(G*rg + j) + n.  Rows no block touches are stored as zeros like any other.
    const int g = lane >> 4, n = lane & 15;
    TY *Yt = static_cast<TY *>(a.Y);
#pragma unroll
    for (int j = 0; j < G; ++j) {
        const int row = (rg * G + j) * kStripe + n;
        if (row >= a.M) continue;
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
}

// ------------------------------------------------------------------ launchers
template <typename TX, typename TY, int VEC>
ubp_status launch_wros_bh(const ubp_packed *p, const void *X, int64_t ldx, int N, void *Y, int64_t ldy, int rpr,
                          hipStream_t st) {
    dim3 grid((unsigned)((N + 256 * VEC - 1) / (256 * VEC)), (unsigned)((p->M + rpr - 1) / rpr));
#define UBP_WROS_CASE(BH)                                                                                              \
    case BH:                                                                                                           \
        hipLaunchKernelGGL((wros_kernel<TX, TY, BH, VEC>), grid, dim3(256), 0, st, p->d_indptr, p->d_indices,         \
                           p->d_values_f32, static_cast<const TX *>(X), ldx, static_cast<TY *>(Y), ldy, p->M, N, p->bw, \
                           rpr);                                                                                       \
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
ubp_status launch_wros(const ubp_packed *p, const void *X, int64_t ldx, int N, void *Y, int64_t ldy, int rpr,
                       hipStream_t st) {
    // 4 columns per thread when every row of X and Y can be accessed as an aligned 4-vector
    const bool vec = (N % 4 == 0) && (ldx % 4 == 0) && (ldy % 4 == 0) &&
                     (reinterpret_cast<uintptr_t>(X) % (4 * sizeof(TX)) == 0) &&
                     (reinterpret_cast<uintptr_t>(Y) % (4 * sizeof(TY)) == 0) && N >= 2048;
    return vec ? launch_wros_bh<TX, TY, 4>(p, X, ldx, N, Y, ldy, rpr, st)
               : launch_wros_bh<TX, TY, 1>(p, X, ldx, N, Y, ldy, rpr, st);
}

template <bool BF16, typename TY, int G, int CT, bool FAST>
ubp_status launch_stripe_one(StripeArgs a, int ctile0, int n_coltiles, int waves, hipStream_t st) {
    constexpr int D = kPrefetchDepth;
    const size_t lds = (size_t)a.ring_bytes + 2 * ring_slots(CT) * sizeof(uint32_t);
    static size_t attr_bytes = 0; // per instantiation; the limit is only ever raised
    if (lds > attr_bytes) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(&stripe_kernel<BF16, TY, G, CT, D, FAST>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
            (void)hipGetLastError();
            return UBP_ERR_DEVICE;
        }
        attr_bytes = lds;
    }
    a.ctile0 = ctile0;
    a.n_coltiles = n_coltiles;
    const unsigned grid = 8u * (unsigned)((n_coltiles + 7) / 8) * (unsigned)a.n_wgrows;
    hipLaunchKernelGGL((stripe_kernel<BF16, TY, G, CT, D, FAST>), dim3(grid), dim3((unsigned)waves * 64), lds, st, a);
    return hipGetLastError() == hipSuccess ? UBP_OK : UBP_ERR_DEVICE;
}

template <bool BF16, typename TY, int G, int CT>
ubp_status launch_stripe_inst(const StripeArgs &a, int waves, hipStream_t st) {
    if (waves * 64 > stripe_max_threads(G, CT, kPrefetchDepth)) return UBP_ERR_UNSUPPORTED;
    // full column tiles with aligned rows take the asynchronous staging path; a ragged last
    // tile (or everything, when rows are not 16-byte aligned) takes the synchronous one
    const int total = (a.N + 16 * CT - 1) / (16 * CT);
    // (the producer addresses a chunk with 32-bit lane offsets: 64 rows of ldx elements must fit)
    const int full = (a.vec_ok && a.ldx <= (int64_t(1) << 24)) ? a.N / (16 * CT) : 0;
    ubp_status rc = UBP_OK;
    if (full > 0) rc = launch_stripe_one<BF16, TY, G, CT, true>(a, 0, full, waves, st);
    if (rc == UBP_OK && total > full)
        rc = launch_stripe_one<BF16, TY, G, CT, false>(a, full, total - full, waves, st);
    return rc;
}

template <bool BF16, typename TY>
ubp_status launch_stripe(const StripeArgs &a, int G, int CT, int waves, hipStream_t st) {
#define UBP_SG_CASE(GG, CC) \
    if (G == GG && CT == CC) return launch_stripe_inst<BF16, TY, GG, CC>(a, waves, st);
    UBP_SG_CASE(1, 2) UBP_SG_CASE(2, 2) UBP_SG_CASE(4, 2) UBP_SG_CASE(1, 4) UBP_SG_CASE(2, 4) UBP_SG_CASE(4, 4)
    UBP_SG_CASE(1, 8) UBP_SG_CASE(2, 8) UBP_SG_CASE(4, 8)
#undef UBP_SG_CASE
    return UBP_ERR_UNSUPPORTED;
}

int stripe_max_waves(int G, int CT) { return stripe_max_threads(G, CT, kPrefetchDepth) / 64; }

int env_int(const char *name, int dflt) {
    const char *v = std::getenv(name);
    return v && *v ? std::atoi(v) : dflt;
}

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
        ok = ok && dev_copy(&p->d_values_f32, f.data(), f.size(), &p->device_bytes);
    }
    {
        const uint32_t zero = 0;
        ok = ok && dev_copy(&p->d_error, &zero, 1, &p->device_bytes);
    }
    if (p->dtype != UBP_F32) {
        for (int s = 0; s < kNumLayouts && ok; ++s) {
            const StripeLayout &L = p->sg[s];
            StripeLayoutDev &D = p->d_sg[s];
            ok = ok && dev_copy(&D.rg_ptr, L.rg_ptr.data(), L.rg_ptr.size(), &p->device_bytes);
            ok = ok && dev_copy(&D.rg_order, L.rg_order.data(), L.rg_order.size(), &p->device_bytes);
            ok = ok && dev_copy(&D.stream, L.stream.data(), L.stream.size(), &p->device_bytes);
        }
    }
    if (!ok) {
        (void)hipGetLastError();
        return UBP_ERR_ALLOC;
    }
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
    for (int s = 0; s < kNumLayouts; ++s) {
        rel(p->d_sg[s].rg_ptr);
        rel(p->d_sg[s].rg_order);
        rel(p->d_sg[s].stream);
    }
}

} // namespace ubp

// ------------------------------------------------------------------ C ABI
extern "C" {

ubp_status ubp_spmm_plan(const ubp_packed *p, const void *X_dev, int64_t ldx, int32_t N, void *Y_dev, int64_t ldy,
                         ubp_dtype y_dtype, void *hip_stream, const ubp_plan *plan) {
    using namespace ubp;
    if (!p || N < 0) return UBP_ERR_INVALID_ARG;
    if (p->device == UBP_HOST_ONLY) return UBP_ERR_INVALID_ARG;
    if (y_dtype != UBP_F32 && y_dtype != p->dtype) return UBP_ERR_INVALID_ARG;
    if (N == 0) return UBP_OK;
    if (!X_dev || !Y_dev || ldx < N || ldy < N) return UBP_ERR_INVALID_ARG;
    ubp_plan pl;
    std::memset(&pl, 0, sizeof pl);
    if (plan) pl = *plan;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    DeviceGuard guard(p->device);
    if (!guard.ok) return UBP_ERR_DEVICE;

    int kernel = pl.kernel;
    if (kernel == 0) kernel = env_int("UBP_KERNEL", 0);
    if (kernel == 0) kernel = (p->dtype == UBP_F32) ? 1 : 2;
    if (kernel == 2 && p->dtype == UBP_F32) return UBP_ERR_UNSUPPORTED;
    if (kernel != 1 && kernel != 2) return UBP_ERR_INVALID_ARG;

    if (kernel == 1) {
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
        switch (p->dtype) {
        case UBP_F32: return launch_wros<float, float>(p, X_dev, ldx, N, Y_dev, ldy, rpr, st);
        case UBP_F16:
            return y_dtype == UBP_F32 ? launch_wros<_Float16, float>(p, X_dev, ldx, N, Y_dev, ldy, rpr, st)
                                      : launch_wros<_Float16, _Float16>(p, X_dev, ldx, N, Y_dev, ldy, rpr, st);
        case UBP_BF16:
            return y_dtype == UBP_F32 ? launch_wros<__bf16, float>(p, X_dev, ldx, N, Y_dev, ldy, rpr, st)
                                      : launch_wros<__bf16, __bf16>(p, X_dev, ldx, N, Y_dev, ldy, rpr, st);
        }
        return UBP_ERR_INVALID_ARG;
    }

    // ---- MFMA stripe kernel
    int CT = pl.col_tiles ? pl.col_tiles : env_int("UBP_CT", 0);
    int G = pl.sub_stripes ? pl.sub_stripes : env_int("UBP_G", 0);
    int waves = pl.waves ? pl.waves : env_int("UBP_WAVES", 0);
    if ((G != 0 && G != 1 && G != 2 && G != 4) || (CT != 0 && CT != 2 && CT != 4 && CT != 8)) return UBP_ERR_UNSUPPORTED;
    {
        // Pick the tile shape with the smallest estimated time.  What a workgroup pulls into its
        // CU (its row groups' step records plus the X tile, once per workgroup) is what bounds
        // the large layers; small layers are bounded by how many rounds of workgroups the chip
        // needs and by a workgroup's start-up and store latency.
        double best = 0.0;
        int bestG = 0, bestCT = 0;
        for (int g = 1; g <= 4; g *= 2)
            for (int ct = 2; ct <= 8; ct *= 2) {
                if ((G && g != G) || (CT && ct != CT)) continue;
                const StripeLayout &Lc = p->sg[layout_slot(g, ct)];
                if (Lc.G == 0) continue;
                const int mw = waves ? waves : stripe_max_waves(g, ct);
                if (mw < 2 || mw > stripe_max_waves(g, ct)) continue;
                const int rows_wg = (Lc.nrg + (mw - 1) - 1) / (mw - 1);           // workgroup rows
                const int nc = (Lc.nrg + rows_wg - 1) / rows_wg;                   // consumers per workgroup
                const int64_t ncol = (N + 16 * ct - 1) / (16 * ct);
                const double rec = (128 + 256 * g) * 4.0;
                const double bytes = (double)ncol * ((double)Lc.nsteps * rec + (double)rows_wg * p->K * 32.0 * ct);
                const int ring = std::min(ring_rows(ct), Lc.nch * kSlotRows) * ring_pitch(ct);
                const int wave_slots = stripe_max_threads(g, ct, kPrefetchDepth) == 1024 ? 16 : 8;
                const int resident = std::max(1, std::min((160 * 1024) / (ring + 256), wave_slots / (nc + 1)));
                const double rounds = std::ceil((double)(ncol * rows_wg) / (256.0 * resident));
                const double heaviest = Lc.sorted_steps.empty() ? 0.0 : (double)Lc.sorted_steps[0];
                const double busy = std::min(1.0, (double)(ncol * rows_wg) / 256.0); // CUs that get a workgroup
                double t = std::max(bytes / (9.0e6 * busy), rounds * (5.0 + 0.3 * heaviest)); // microseconds
                if (N % (16 * ct) != 0) t += 10.0; // the ragged last column tile takes the slow staging path
                if (bestG == 0 || t < best) {
                    best = t;
                    bestG = g;
                    bestCT = ct;
                }
            }
        if (bestG == 0) return UBP_ERR_UNSUPPORTED;
        G = bestG;
        CT = bestCT;
    }
    const int slot = layout_slot(G, CT);
    const StripeLayout &L = p->sg[slot];
    const int max_waves = stripe_max_waves(G, CT);
    if (waves == 0) {
        // as few workgroup rows as the wavefront limit allows, consumers spread evenly over them
        const int rows_wg = (L.nrg + (max_waves - 1) - 1) / (max_waves - 1);
        waves = (L.nrg + rows_wg - 1) / rows_wg + 1; // consumers + one producer
    }
    if (waves < 2 || waves > max_waves) return UBP_ERR_UNSUPPORTED;

    StripeArgs a;
    a.rg_ptr = p->d_sg[slot].rg_ptr;
    a.rg_order = p->d_sg[slot].rg_order;
    a.stream = p->d_sg[slot].stream;
    a.X = static_cast<const uint16_t *>(X_dev);
    a.Y = Y_dev;
    a.ldx = ldx;
    a.ldy = ldy;
    a.M = p->M;
    a.K = p->K;
    a.N = N;
    a.nrg = L.nrg;
    a.nch = L.nch;
    a.ring_bytes = std::min(ring_rows(CT), L.nch * kSlotRows) * ring_pitch(CT);
    a.err = p->d_error;
    a.ctile0 = 0;
    a.n_coltiles = 0;
    a.n_wgrows = (L.nrg + (waves - 1) - 1) / (waves - 1);
    const size_t ysz = (y_dtype == UBP_F32) ? 4 : 2;
    a.vec_ok = (ldx % 8 == 0) && (reinterpret_cast<uintptr_t>(X_dev) % 16 == 0) && ((ldy * ysz) % 16 == 0) &&
               (reinterpret_cast<uintptr_t>(Y_dev) % 16 == 0);
    if (p->dtype == UBP_BF16)
        return y_dtype == UBP_F32 ? launch_stripe<true, float>(a, G, CT, waves, st)
                                  : launch_stripe<true, __bf16>(a, G, CT, waves, st);
    return y_dtype == UBP_F32 ? launch_stripe<false, float>(a, G, CT, waves, st)
                              : launch_stripe<false, _Float16>(a, G, CT, waves, st);
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

ubp_status ubp_spmm(const ubp_packed *p, const void *X_dev, int64_t ldx, int32_t N, void *Y_dev, int64_t ldy,
                    ubp_dtype y_dtype, void *hip_stream) {
    return ubp_spmm_plan(p, X_dev, ldx, N, Y_dev, ldy, y_dtype, hip_stream, nullptr);
}

} // extern "C"
