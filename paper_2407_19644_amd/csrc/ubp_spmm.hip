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
typedef uint32_t uint2v __attribute__((ext_vector_type(2)));
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));

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
    uint32_t stream_bytes;   // size of the record stream (buffer-addressed: below 4 GB)
    const uint16_t *X;
    void *Y;
    int64_t ldx, ldy;
    int M, K, N, bh;
    int nrg, nch;            // row groups, 64-row chunks of X
    int ring_bytes;          // bytes of the LDS ring actually used (all of K when K is shorter than the ring)
    int ctile0, n_coltiles;  // first column tile of this launch, number of tiles in it
    int n_wgrows;
    int n_producers;         // producer wavefronts per workgroup: 1, 2 or 4 (the last wavefronts)
    int resident;            // the ring holds all of K: slots are never refilled, a consumer may walk several row groups
    int vec_ok;              // X and Y allow 16-byte vector access on every row
    int out_bytes;           // LDS bytes per consumer behind the ring and the counters for 16 rows of a
                             // 16-bit Y tile (stores then leave as whole rows of the tile); 0: none
    uint32_t *err;           // set to nonzero when a bounded wait runs out
};

template <bool BF16>
__device__ __forceinline__ float4v mfma16(short8v a, short8v b, float4v c) {
    if constexpr (BF16)
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf8v, a), __builtin_bit_cast(bf8v, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8v, a), __builtin_bit_cast(half8v, b), c, 0, 0, 0);
}

// transposed 8-byte read at an absolute LDS byte address
__device__ __forceinline__ short4v lds_read_tr(uint32_t lds_addr) {
    typedef __attribute__((address_space(3))) short4v *lds_ptr;
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(uintptr_t)lds_addr);
}

// 16 bytes per lane from global memory straight into LDS at lds_base + 16 * lane (lds_base
// wave-uniform).  Written as inline assembly on purpose: the compiler then does not treat
// the load as a pending LDS write, which would make it wait for ALL outstanding vector
// memory operations before every LDS read.  Ordering against the LDS reads of the staged
// data is done by hand (wait_vmcnt, then the producer's counter of resident chunks).
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

// waits until at most n vector memory operations of this wavefront are outstanding (n is
// wave-uniform; it is rounded down to the nearest available immediate, which only waits longer)
__device__ __forceinline__ void wait_vmcnt_at_most(int n) {
    if (n >= 48) wait_vmcnt<48>();
    else if (n >= 32) wait_vmcnt<32>();
    else if (n >= 24) wait_vmcnt<24>();
    else if (n >= 16) wait_vmcnt<16>();
    else if (n >= 12) wait_vmcnt<12>();
    else if (n >= 8) wait_vmcnt<8>();
    else if (n >= 6) wait_vmcnt<6>();
    else if (n >= 4) wait_vmcnt<4>();
    else if (n >= 3) wait_vmcnt<3>();
    else if (n >= 2) wait_vmcnt<2>();
    else if (n >= 1) wait_vmcnt<1>();
    else wait_vmcnt<0>();
}

__device__ __forceinline__ uint32_t flag_load(uint32_t *p) {
    return __hip_atomic_load(p, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP);
}

constexpr int kSpinLimit = 1 << 22; // polls before a wait gives up (each poll is >= 100 cycles)

// The gather of step s+1 is issued before the MFMAs of step s (two operand buffers) except
// for the largest tile, where the second buffer would halve the wavefronts per SIMD.
// (The block-native 16-tile shape goes without the second buffer too: with it the shape needs
// 139 registers, without it 123 - 16 wavefronts per workgroup instead of 12, 158 us against 173 us on
// the largest layer.  Two records in flight instead of four would also make room, and cost 40 %.)
constexpr bool stripe_pipelined(int G, int CT, bool NATIVE) { return NATIVE ? G * CT != 16 : G * CT < 32; }

constexpr int stripe_max_threads(int G, int CT, int D, bool NATIVE) {
    // accumulators + operand buffer(s) + D prefetched step records + addressing, in VGPRs
    // per lane; 512 per SIMD lane are shared by the wavefronts resident on the SIMD
    const int regs = 4 * G * CT + (stripe_pipelined(G, CT, NATIVE) ? 8 : 4) * CT + D * (2 + 4 * (NATIVE ? 1 : G)) +
                     (NATIVE ? 28 : G == 1 ? 8 : 20);
    // (the estimate runs high for the block-native kernel, whose fragment registers are shared by the
    // stripes: its limits are set from the compiled register counts, 123 / 138 for the two shapes
    // that change tier)
    if (NATIVE) return regs <= 136 ? 1024 : regs <= 190 ? 768 : 512;
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
template <bool BF16, typename TY, int G, int CT, int D, bool FAST, bool NATIVE>
__global__ __launch_bounds__(stripe_max_threads(G, CT, D, NATIVE)) void stripe_kernel(StripeArgs a) {
    constexpr int NTW = 16 * CT;
    constexpr int PITCH = ring_pitch(CT);
    constexpr int PIECES = 2 * CT; // 16-byte pieces per staged row
    constexpr int R = ring_slots(CT), KS = kSlotRows;
    constexpr int FG = NATIVE ? 1 : G; // weight fragments per record
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
    constexpr bool PIPE = stripe_pipelined(G, CT, NATIVE);
    const uint32_t ring_base = __builtin_amdgcn_readfirstlane(lds_address(smem));
    short8v xf[PIPE ? 2 : 1][CT];
    auto stage_control = [&](int d, bool foreign, uint32_t &a_lo, uint32_t &a_hi) {
        // (foreign: the slot after the row group's last step holds another row group's record;
        // its gather is issued all the same, to valid addresses, and never used, but its control
        // word must not be acted on)
        uint32_t ctl = 0u;
        if (!foreign) {
            // block-native records spread the control word over bit 31 of the lanes' second dwords
            if constexpr (NATIVE) ctl = (uint32_t)__builtin_amdgcn_ballot_w64((int32_t)info_y[d] < 0);
            else ctl = __builtin_amdgcn_readfirstlane(info_y[d]);
        }
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
    constexpr bool FUSED = PIPE && !NATIVE && G == 1;
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
                    // block-native: the one fragment holds, per lane, the weight of the block row that
                    // is congruent to the lane's row modulo 16; stripe j keeps an entry quad only where
                    // the block covers row 16*j + n
                    [[maybe_unused]] const int t_lo = (int)(info_y[d] & 0x7fu) - 64;
                    [[maybe_unused]] const int t_hi = (int)((info_y[d] >> 8) & 0x7fu) - 64;
#pragma unroll
                    for (int j = 0; j < G; ++j) {
                        if (mask & (1u << j)) {
                            short8v wv;
                            if constexpr (NATIVE) {
                                const uint4v f = wf[d][0];
                                const bool lo_ok = (uint32_t)(t_lo + 16 * j) < (uint32_t)a.bh;
                                const bool hi_ok = (uint32_t)(t_hi + 16 * j) < (uint32_t)a.bh;
                                const uint4v w = {lo_ok ? f[0] : 0u, lo_ok ? f[1] : 0u, hi_ok ? f[2] : 0u, hi_ok ? f[3] : 0u};
                                wv = __builtin_bit_cast(short8v, w);
                            } else {
                                wv = __builtin_bit_cast(short8v, wf[d][j]);
                            }
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
        if constexpr (sizeof(TY) == 2 && NATIVE) { // (NATIVE: the shapes with registers to spare for it)
            if (a.out_bytes != 0) {
                // A 16-bit tile straight from the accumulators is 8 bytes per lane, 32-byte runs per
                // row.  Through 16 LDS rows of this wavefront (16-byte pieces XOR-swizzled by the row
                // against bank conflicts; one wavefront writes and reads, LDS keeps its order) an
                // instruction stores whole rows of the tile, 16 bytes per lane.
                constexpr int RB = 16 * CT * 2;   // bytes per row of the tile: 64, 128 or 256
                constexpr int PR = RB / 16;       // 16-byte pieces per row
                constexpr int RP = 256 / RB;      // rows per 256 bytes (one pass over the banks)
                constexpr int NI = PR / 4;        // store instructions per stripe
                char *scratch = smem + a.ring_bytes + 32 * sizeof(uint32_t) + wave * a.out_bytes;
#pragma unroll
                for (int j = 0; j < G; ++j) {
#pragma unroll
                    for (int c = 0; c < CT; ++c) {
                        typedef TY ty4 __attribute__((ext_vector_type(4)));
                        ty4 o;
#pragma unroll
                        for (int v = 0; v < 4; ++v) o[v] = from_f32<TY>(acc[j][c][v]);
                        const int piece = (2 * c + (g >> 1)) ^ ((n / RP) & (PR - 1));
                        *reinterpret_cast<ty4 *>(scratch + n * RB + piece * 16 + (g & 1) * 8) = o;
                    }
#pragma unroll
                    for (int i = 0; i < NI; ++i) {
                        const int r = i * (64 / PR) + lane / PR, lp = lane % PR;
                        const uint4v o = *reinterpret_cast<const uint4v *>(scratch + r * RB + ((lp ^ ((r / RP) & (PR - 1))) << 4));
                        const int row = (rg_done * G + j) * kStripe + r;
                        if (row < a.M) *reinterpret_cast<uint4v *>(Yt + (int64_t)row * a.ldy + col0 + lp * 8) = o;
                    }
                }
                if (!more) break;
                continue;
            }
        }
#pragma unroll
        for (int j = 0; j < G; ++j) {
            const int row = (rg_done * G + j) * kStripe + n;
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
        if (!more) break;
    }
    if (broken && lane == 0) atomicOr(a.err, 2u);
}

// ------------------------------------------------------------------ small-K tile kernel
// For layers whose whole K dimension is a few 32-row tiles (K <= 256: pointwise convolutions
// with few input channels).  There the gather machinery above costs more than it saves: with
// 20-30 % of the weights kept in small blocks almost every 16 x 32 operand tile holds a kept
// weight.  So W is used as zero-filled operand tiles, X needs no gather, and the kernel is a
// short, fully unrolled, output-stationary loop:
//  * Workgroup = NW wavefronts on one block of NW*16*CT pixels (wavefront w owns pixel tile
//    w) x one slice of up to SMAX stripes, whose accumulators all stay in registers.
//  * The slice's weight tiles (contiguous in memory) go global -> LDS once, all wavefronts
//    taking turns at the 1 KB loads; every wavefront then reads each tile with one 16-byte
//    LDS read per lane.
//  * X is loaded by the workgroup together, block row by block row: an instruction's 64 lanes
//    cover whole rows of the block (runs of NW*32*CT bytes) instead of 16 short runs of one
//    wavefront's own columns - the memory pipeline takes a wavefront's runs one by one, and
//    it is their number, not their bytes, that costs.  Every load is issued up front; the
//    data then passes 32 rows at a time through one of two LDS staging tiles (one barrier
//    per 32 rows), from which each wavefront reads its own columns transposed into operand
//    order and multiplies them into every stripe of the slice: the MFMAs start when the
//    first 32 rows have arrived and run while the rest is still on its way.
//  * Stores leave the same way: accumulator tiles are written to LDS (the weight area, free
//    by then) and the workgroup stores whole block rows, 16 bytes per lane.
// Columns past N and rows past K are staged as zeros.  Stripes of a partial last slice are
// computed (on the slice's last real tiles) but not stored.
struct TileArgs {
    const uint16_t *frags;   // [nstripes][KT][64][8]
    const uint16_t *X;
    void *Y;
    int64_t ldx, ldy;
    int M, K, N;
    int nstripes, sps;       // stripes in all, stripes per workgroup slice (<= SMAX)
    int n_blocks;            // pixel blocks (NW tiles each)
    int slices;              // slices the stripes are cut into (xstat_kernel's workgroup order needs it)
    int kt_total;            // 32-column tiles per stripe in frags (xchunk_kernel: a multiple of its KT)
    uint32_t *err;           // the handle's error flags (bounded waits that ran out)
};

// s_barrier with only the LDS counter drained: __syncthreads() would also wait for every
// outstanding vector memory operation, i.e. for the X loads that are meant to stay in flight
__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

template <bool BF16, typename TY, int CT, int KT, int SMAX>
__global__ __launch_bounds__(512) void tile_kernel(TileArgs a) {
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const int NW = (int)(blockDim.x >> 6);                 // 1, 2, 4 or 8
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int block = blockIdx.x % a.n_blocks, slice = blockIdx.x / a.n_blocks;
    const int stripe0 = slice * a.sps;
    const int ns = min(a.sps, a.nstripes - stripe0);       // stripes of this slice
    const int bcol0 = block * NW * 16 * CT;                // first pixel of the block
    const int XRB = NW * 32 * CT;                          // bytes of one block row of X
    const int U = NW * CT;                                 // 32-byte units per block row (power of two)
    const int umask = min(U - 1, 15);
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_address(smem));
    const int w_bytes = a.sps * KT * 1024;                 // weight area, then the two staging tiles
    const int stage_bytes = 32 * XRB;
    char *stage = smem + w_bytes;

    // ---- weight tiles of the slice: global -> LDS, 1 KB per instruction, wavefronts take turns
    {
        const uint16_t *src = a.frags + (int64_t)stripe0 * KT * 512;
        const int n_kb = ns * KT;
        for (int i = wave; i < n_kb; i += NW)
            load16_to_lds(src + (int64_t)i * 512, (uint32_t)lane * 16u, lds0 + (uint32_t)i * 1024u);
    }

    // ---- X: instruction i (0 .. NW*CT-1) of a 32-row tile covers rows i*RPI .. of the block,
    // lane -> (row, 16-byte piece of the block row); wavefront w issues instructions w*CT ..
    const int LPR = 2 * U;                 // lanes (16-byte pieces) per block row
    const int RPI = 64 / LPR;              // rows per instruction (LPR <= 64)
    const int row_in = lane / LPR, piece = lane % LPR;
    uint4 v[KT][CT];
    int st_off[CT];                        // where this lane's piece of instruction i goes in a staging tile
#pragma unroll
    for (int i = 0; i < CT; ++i) {
        const int r = (wave * CT + i) * RPI + row_in; // row inside the 32-row tile
        st_off[i] = r * XRB + (((piece >> 1) ^ (r & umask)) << 5) + ((piece & 1) << 4);
    }
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) {
#pragma unroll
        for (int i = 0; i < CT; ++i) {
            const int k = kt * 32 + (wave * CT + i) * RPI + row_in;
            const int col = bcol0 + piece * 8;
            // always load (from a clamped, valid address) and zero afterwards: every wavefront then
            // has exactly KT*CT loads behind its weight loads, which the wait before the first
            // barrier counts on (N >= 8 here: a multiple of 8, and not 0)
            const bool inside = k < a.K && col + 8 <= a.N;
            const uint4 x = *reinterpret_cast<const uint4 *>(a.X + (int64_t)min(k, a.K - 1) * a.ldx + min(col, a.N - 8));
            v[kt][i] = inside ? x : uint4{0u, 0u, 0u, 0u};
        }
    }

    const int g = lane >> 4, n = lane & 15;
    uint32_t a_lo, a_hi; // this lane's two transposed reads of its wavefront's columns in staging tile 0
    {
        const int r_lo = 4 * g + (n >> 2), r_hi = 16 + r_lo, sub = (n & 3) * 8;
        const uint32_t s0 = lds_address(stage);
        a_lo = s0 + (uint32_t)(r_lo * XRB + (((wave * CT) ^ (r_lo & umask)) << 5) + sub);
        a_hi = s0 + (uint32_t)(r_hi * XRB + (((wave * CT) ^ (r_hi & umask)) << 5) + sub);
    }
    typedef __attribute__((address_space(3))) const uint4v *lds_frag_ptr;
    const uint32_t w_lane = lds0 + (uint32_t)lane * 16u;

    float4v acc[SMAX][CT];
#pragma unroll
    for (int sl = 0; sl < SMAX; ++sl)
#pragma unroll
        for (int c = 0; c < CT; ++c) acc[sl][c] = float4v{0.f, 0.f, 0.f, 0.f};

#pragma unroll
    for (int kt = 0; kt < KT; ++kt) {
        // my pieces of these 32 rows -> staging tile kt mod 2.  (The tile was last read two
        // barriers ago: nobody can still be reading it.)
        char *st = stage + (kt & 1) * stage_bytes;
#pragma unroll
        for (int i = 0; i < CT; ++i) *reinterpret_cast<uint4 *>(st + st_off[i]) = v[kt][i];
        if (kt == 0) {
            // Vector memory returns in order and the weight loads were issued before the X loads:
            // once only the X loads of the later tiles are outstanding, this wavefront's share of
            // the weight tiles has landed; after the barrier everybody's.
            wait_vmcnt<(KT - 1) * CT>();
        }
        lds_barrier();
        short8v xf[CT];
        const uint32_t off = (uint32_t)((kt & 1) * stage_bytes);
#pragma unroll
        for (int c = 0; c < CT; ++c) {
            const short4v p0 = lds_read_tr((a_lo ^ (uint32_t)(c << 5)) + off);
            const short4v p1 = lds_read_tr((a_hi ^ (uint32_t)(c << 5)) + off);
            xf[c] = __builtin_shufflevector(p0, p1, 0, 1, 2, 3, 4, 5, 6, 7);
        }
#pragma unroll
        for (int sl = 0; sl < SMAX; ++sl) {
            const int sl_c = min(sl, ns - 1); // a partial slice recomputes its last stripe (never stored)
            const uint4v w = *(lds_frag_ptr)(uintptr_t)(w_lane + (uint32_t)((sl_c * KT + kt) * 1024));
            const short8v wv = __builtin_bit_cast(short8v, w);
#pragma unroll
            for (int c = 0; c < CT; ++c) acc[sl][c] = mfma16<BF16>(xf[c], wv, acc[sl][c]);
        }
    }

    // ---- stores: tiles -> LDS (from its start: weights and staging tiles are dead) -> whole block rows
    constexpr int YS = (int)sizeof(TY);
    const int ORB = NW * 16 * CT * YS;       // bytes of one block row of Y
    const int OPR = ORB / 16;                // 16-byte pieces per block row (a power of two, >= 4)
    const int opr_shift = __builtin_ctz((unsigned)OPR);
    const int osw = min(7, OPR - 1);         // pieces of a row are XOR-swizzled by the row number against bank conflicts
    const int lds_bytes = w_bytes + 2 * stage_bytes;
    const int chunk = max(1, min(ns, lds_bytes / (16 * ORB))); // stripes that fit LDS at a time
    TY *Yt = static_cast<TY *>(a.Y);
    lds_barrier(); // everybody is done with the weights and the staging tiles
    int in_chunk = 0, first = 0; // stripes written to LDS since the last flush, first of them
#pragma unroll
    for (int sl = 0; sl < SMAX; ++sl) {
        if (sl >= ns) continue; // (no break: the loop must unroll fully, accumulators are registers)
        // lane (g, n): row n of the stripe, pixels 16c + 4g .. + 3 of wavefront w's tile
#pragma unroll
        for (int c = 0; c < CT; ++c) {
            const int byte = ((wave * CT + c) * 16 + 4 * g) * YS;
            const int pc = (byte >> 4) ^ (n & osw);
            char *dst = smem + (in_chunk * 16 + n) * ORB + pc * 16 + (byte & 15);
            if constexpr (YS == 4) {
                *reinterpret_cast<float4v *>(dst) = acc[sl][c];
            } else {
                typedef TY ty4 __attribute__((ext_vector_type(4)));
                ty4 o;
#pragma unroll
                for (int t = 0; t < 4; ++t) o[t] = from_f32<TY>(acc[sl][c][t]);
                *reinterpret_cast<ty4 *>(dst) = o;
            }
        }
        ++in_chunk;
        if (in_chunk == chunk || sl == ns - 1) {
            lds_barrier(); // the chunk is complete
            const int pieces = in_chunk * 16 * OPR;
            for (int q = wave * 64 + lane; q < pieces; q += NW * 64) {
                const int r = q >> opr_shift, pq = q & (OPR - 1);
                const uint4 o = *reinterpret_cast<const uint4 *>(smem + r * ORB + ((pq ^ (r & osw)) << 4));
                const int row = (stripe0 + first) * kStripe + r;
                const int px = bcol0 + pq * (16 / YS);
                if (row < a.M && px + 16 / YS <= a.N) *reinterpret_cast<uint4 *>(Yt + (int64_t)row * a.ldy + px) = o;
            }
            first = sl + 1;
            in_chunk = 0;
            if (sl != ns - 1) lds_barrier(); // the chunk has been read; the next one may overwrite it
        }
    }
}

// ------------------------------------------------------------------ small-K kernel, X stationary in registers
// The same operand tiles as tile_kernel, the loop nest the other way round - and closer to the
// paper's dataflow (section 4.2), where output rows are finished one after the other and leave
// for good.  K <= 256 means a wavefront can hold ALL of X for its 16*CT pixels as matrix
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

template <bool BF16, typename TY, int CT, int KT>
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
    auto load_w = [&](uint4v(&w)[KT], int stripe) {
        // (a stripe past the slice is clamped: loaded, never used)
        const uint4v *src = wbase + (int64_t)min(stripe, a.nstripes - 1) * (KT * 64);
#pragma unroll
        for (int kt = 0; kt < KT; ++kt) w[kt] = src[kt * 64];
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
        float4v acc[CT];
#pragma unroll
        for (int c = 0; c < CT; ++c) acc[c] = float4v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kt = 0; kt < KT; ++kt) {
            const short8v wv = __builtin_bit_cast(short8v, w[kt]);
#pragma unroll
            for (int c = 0; c < CT; ++c) acc[c] = mfma16<BF16>(xf[kt][c], wv, acc[c]);
        }
        // The 16 x (16 CT) result leaves through this wavefront's own piece of LDS: in the
        // accumulators a row is spread over 4 lanes (16 bytes each per store: 64-byte runs),
        // after the detour an instruction writes whole rows of the block (RB bytes each).
        // 16-byte pieces of a row are XOR-swizzled by the row number so that the 16 lanes LDS
        // serves together hit 64 different banks on the way in and on the way out.
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
template <bool BF16, typename TY, int CT, int KT, int SW>
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
    auto load_w = [&](uint4v(&w)[KT], int stripe, int ch) {
        const uint4v *src = wbase + ((int64_t)min(stripe, a.nstripes - 1) * a.kt_total + min(ch, nch - 1) * KT) * 64;
#pragma unroll
        for (int kt = 0; kt < KT; ++kt) w[kt] = src[kt * 64];
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
    load_w(ws[0], s0, 0);
    load_w(ws[1], s0 + 1, 0);
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
                load_w(ws[(t + 2) % kSets], s0 + far % SW, ch + far / SW);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int kt = 0; kt < KT; ++kt) {
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

template <bool BF16, typename TY, int CT, int KT, int SMAX>
ubp_status launch_tile_inst(const TileArgs &a, int waves, int slices, hipStream_t st) {
    const size_t lds = (size_t)a.sps * KT * 1024 + (size_t)2 * 32 * waves * 32 * CT;
    if (lds > 160 * 1024 || a.sps > SMAX) return UBP_ERR_UNSUPPORTED;
    static size_t attr_bytes = 0; // per instantiation; the limit is only ever raised
    if (lds > attr_bytes) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(&tile_kernel<BF16, TY, CT, KT, SMAX>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
            (void)hipGetLastError();
            return UBP_ERR_DEVICE;
        }
        attr_bytes = lds;
    }
    hipLaunchKernelGGL((tile_kernel<BF16, TY, CT, KT, SMAX>), dim3((unsigned)(a.n_blocks * slices)), dim3((unsigned)waves * 64),
                       lds, st, a);
    return hipGetLastError() == hipSuccess ? UBP_OK : UBP_ERR_DEVICE;
}

template <bool BF16, typename TY, int CT, int KT>
ubp_status launch_tile_ck(const TileArgs &a, int waves, int slices, hipStream_t st) {
    // the smallest accumulator set that holds the slice (unused stripes are computed all the same)
    if (a.sps <= 4) return launch_tile_inst<BF16, TY, CT, KT, 4>(a, waves, slices, st);
    if (a.sps <= 8) return launch_tile_inst<BF16, TY, CT, KT, 8>(a, waves, slices, st);
    if constexpr (CT == 2) return launch_tile_inst<BF16, TY, CT, KT, 16>(a, waves, slices, st);
    return UBP_ERR_UNSUPPORTED;
}

template <bool BF16, typename TY>
ubp_status launch_tile(const TileArgs &a, int CT, int KT, int waves, int slices, hipStream_t st) {
#define UBP_TILE_CASE(CC, KK) \
    if (CT == CC && KT == KK) return launch_tile_ck<BF16, TY, CC, KK>(a, waves, slices, st);
    UBP_TILE_CASE(2, 2) UBP_TILE_CASE(2, 4) UBP_TILE_CASE(2, 6) UBP_TILE_CASE(2, 8)
    UBP_TILE_CASE(4, 2) UBP_TILE_CASE(4, 4) UBP_TILE_CASE(4, 6) UBP_TILE_CASE(4, 8)
#undef UBP_TILE_CASE
    return UBP_ERR_UNSUPPORTED;
}

template <bool BF16, typename TY, int CT, int KT>
ubp_status launch_xstat_inst(const TileArgs &a, int waves, int slices, hipStream_t st) {
    // the X block, then 16 rows of output per wavefront: at most 32 + 32 KB, no attribute needed
    const size_t lds = (size_t)KT * CT * 1024 + (size_t)waves * 256 * CT * sizeof(TY);
    TileArgs b = a;
    b.slices = slices;
    hipLaunchKernelGGL((xstat_kernel<BF16, TY, CT, KT>), dim3((unsigned)(8 * ((a.n_blocks + 7) / 8) * slices)),
                       dim3((unsigned)waves * 64), lds, st, b);
    return hipGetLastError() == hipSuccess ? UBP_OK : UBP_ERR_DEVICE;
}

template <bool BF16, typename TY>
ubp_status launch_xstat(const TileArgs &a, int CT, int KT, int waves, int slices, hipStream_t st) {
#define UBP_XSTAT_CASE(CC, KK) \
    if (CT == CC && KT == KK) return launch_xstat_inst<BF16, TY, CC, KK>(a, waves, slices, st);
    UBP_XSTAT_CASE(2, 2) UBP_XSTAT_CASE(2, 4) UBP_XSTAT_CASE(2, 6) UBP_XSTAT_CASE(2, 8)
    UBP_XSTAT_CASE(4, 2) UBP_XSTAT_CASE(4, 4) UBP_XSTAT_CASE(4, 6) UBP_XSTAT_CASE(4, 8)
#undef UBP_XSTAT_CASE
    return UBP_ERR_UNSUPPORTED;
}

template <bool BF16, typename TY, int CT, int KT, int SW>
ubp_status launch_xchunk(const TileArgs &a, int slices, hipStream_t st) {
    constexpr int kChunkConsumers = kChunkStripes / SW;
    // the ring of chunks, 16 rows of output per multiplying wavefront, the progress counters
    const size_t lds = (size_t)kChunkRing * KT * CT * 1024 + (size_t)kChunkConsumers * 256 * CT * sizeof(TY) + 64;
    if (a.kt_total % KT != 0 || a.sps > kChunkStripes) return UBP_ERR_UNSUPPORTED;
    static size_t attr_bytes = 64 * 1024; // per instantiation; the limit is only ever raised
    if (lds > attr_bytes) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(&xchunk_kernel<BF16, TY, CT, KT, SW>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
            (void)hipGetLastError();
            return UBP_ERR_DEVICE;
        }
        attr_bytes = lds;
    }
    hipLaunchKernelGGL((xchunk_kernel<BF16, TY, CT, KT, SW>), dim3((unsigned)(a.n_blocks * slices)),
                       dim3((kChunkConsumers + kChunkProducers) * 64), lds, st, a);
    return hipGetLastError() == hipSuccess ? UBP_OK : UBP_ERR_DEVICE;
}

template <bool BF16, typename TY, int G, int CT, bool FAST, bool NATIVE>
ubp_status launch_stripe_one(StripeArgs a, int ctile0, int n_coltiles, int waves, hipStream_t st) {
    constexpr int D = kPrefetchDepth;
    // ring + the progress counters + (16-bit Y, full tiles only, where it fits) the consumers' output rows
    if (FAST && NATIVE && sizeof(TY) == 2 && a.vec_ok) {
        const size_t want = (size_t)16 * 16 * CT * 2;
        if ((size_t)a.ring_bytes + 32 * sizeof(uint32_t) + (size_t)(waves - a.n_producers) * want <= 160 * 1024) a.out_bytes = (int)want;
    }
    const size_t lds = (size_t)a.ring_bytes + 32 * sizeof(uint32_t) + (size_t)(waves - a.n_producers) * a.out_bytes;
    static size_t attr_bytes = 0; // per instantiation; the limit is only ever raised
    if (lds > attr_bytes) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(&stripe_kernel<BF16, TY, G, CT, D, FAST, NATIVE>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
            (void)hipGetLastError();
            return UBP_ERR_DEVICE;
        }
        attr_bytes = lds;
    }
    a.ctile0 = ctile0;
    a.n_coltiles = n_coltiles;
    const unsigned grid = 8u * (unsigned)((n_coltiles + 7) / 8) * (unsigned)a.n_wgrows;
    hipLaunchKernelGGL((stripe_kernel<BF16, TY, G, CT, D, FAST, NATIVE>), dim3(grid), dim3((unsigned)waves * 64), lds, st, a);
    return hipGetLastError() == hipSuccess ? UBP_OK : UBP_ERR_DEVICE;
}

template <bool BF16, typename TY, int G, int CT, bool NATIVE>
ubp_status launch_stripe_inst(const StripeArgs &a, int waves, hipStream_t st) {
    if (waves * 64 > stripe_max_threads(G, CT, kPrefetchDepth, NATIVE)) return UBP_ERR_UNSUPPORTED;
    // full column tiles with aligned rows take the asynchronous staging path; a ragged last
    // tile (or everything, when rows are not 16-byte aligned) takes the synchronous one
    const int total = (a.N + 16 * CT - 1) / (16 * CT);
    // (the producer addresses a chunk with 32-bit lane offsets: 64 rows of ldx elements must fit)
    const int full = (a.vec_ok && a.ldx <= (int64_t(1) << 24)) ? a.N / (16 * CT) : 0;
    ubp_status rc = UBP_OK;
    if (full > 0) rc = launch_stripe_one<BF16, TY, G, CT, true, NATIVE>(a, 0, full, waves, st);
    if (rc == UBP_OK && total > full)
        rc = launch_stripe_one<BF16, TY, G, CT, false, NATIVE>(a, full, total - full, waves, st);
    return rc;
}

template <bool BF16, typename TY>
ubp_status launch_stripe(const StripeArgs &a, int G, int CT, bool native, int waves, hipStream_t st) {
#define UBP_SG_CASE(GG, CC) \
    if (G == GG && CT == CC && !native) return launch_stripe_inst<BF16, TY, GG, CC, false>(a, waves, st);
    UBP_SG_CASE(1, 2) UBP_SG_CASE(2, 2) UBP_SG_CASE(4, 2) UBP_SG_CASE(1, 4) UBP_SG_CASE(2, 4) UBP_SG_CASE(4, 4)
    UBP_SG_CASE(1, 8) UBP_SG_CASE(2, 8) UBP_SG_CASE(4, 8)
#undef UBP_SG_CASE
#define UBP_SG_CASE(GG, CC) \
    if (G == GG && CT == CC && native) return launch_stripe_inst<BF16, TY, GG, CC, true>(a, waves, st);
    UBP_SG_CASE(2, 2) UBP_SG_CASE(4, 2) UBP_SG_CASE(2, 4) UBP_SG_CASE(4, 4) UBP_SG_CASE(2, 8) UBP_SG_CASE(4, 8)
#undef UBP_SG_CASE
    return UBP_ERR_UNSUPPORTED;
}

int stripe_max_waves(int G, int CT, bool native) { return stripe_max_threads(G, CT, kPrefetchDepth, native) / 64; }

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
        if (p->tiles.kt_pad) {
            ok = ok && dev_copy(&p->d_tiles.frags, p->tiles.frags.data(), p->tiles.frags.size(), &p->device_bytes);
        }
        for (int s = 0; s < kNumLayouts && ok; ++s) {
            const StripeLayout &L = p->sgn[s];
            if (L.G == 0) continue;
            StripeLayoutDev &D = p->d_sgn[s];
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
    rel(p->d_tiles.frags);
    for (int s = 0; s < kNumLayouts; ++s) {
        rel(p->d_sg[s].rg_ptr);
        rel(p->d_sg[s].rg_order);
        rel(p->d_sg[s].stream);
        rel(p->d_sgn[s].rg_ptr);
        rel(p->d_sgn[s].rg_order);
        rel(p->d_sgn[s].stream);
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
    const size_t ysz = (y_dtype == UBP_F32) ? 4 : 2;
    const bool vec_ok = (ldx % 8 == 0) && (reinterpret_cast<uintptr_t>(X_dev) % 16 == 0) && ((ldy * ysz) % 16 == 0) &&
                        (reinterpret_cast<uintptr_t>(Y_dev) % 16 == 0);
    // the small-K tile kernel needs 16-byte pieces of X rows that lie entirely inside or outside the matrix
    const bool tile_ok = p->dtype != UBP_F32 && p->tiles.kt_pad != 0 && vec_ok && N % 8 == 0;
    if (kernel == 0) {
        // Dense zero-filled tiles where most tiles hold a kept weight anyway: always for K <= 256
        // (20-30 % kept in small blocks), for larger K while at least a fifth of W is kept (the
        // 3x3-convolution layer: 28.7 us against 30.7 us with gathered rows); else gathered rows.
        const bool dense_enough = (double)p->nb * p->bh * p->bw >= 0.2 * (double)p->M * p->K;
        if (p->dtype == UBP_F32) kernel = 1;
        else if (tile_ok && p->K <= kTileMaxK) kernel = 4;
        else if (tile_ok && p->tiles.kt_pad % 4 == 0 && dense_enough) kernel = 5;
        else kernel = 2;
    }
    if (kernel >= 2 && kernel <= 5 && p->dtype == UBP_F32) return UBP_ERR_UNSUPPORTED;
    if (kernel < 1 || kernel > 5) return UBP_ERR_INVALID_ARG;
    if ((kernel == 3 || kernel == 4) && p->K > kTileMaxK) return UBP_ERR_UNSUPPORTED;
    if (kernel == 5) {
        if (!tile_ok || p->tiles.kt_pad % 4 != 0) return UBP_ERR_UNSUPPORTED;
        int CT = pl.col_tiles ? pl.col_tiles : env_int("UBP_CT", 0);
        if (CT == 0) CT = 4;
        if (CT != 2 && CT != 4) return UBP_ERR_UNSUPPORTED;
        if (pl.waves != 0) return UBP_ERR_UNSUPPORTED; // fixed: 16 stripes' worth of multiplying wavefronts + 4 that load X
        TileArgs a = {};
        a.frags = p->d_tiles.frags;
        a.X = static_cast<const uint16_t *>(X_dev);
        a.Y = Y_dev;
        a.ldx = ldx;
        a.ldy = ldy;
        a.M = p->M;
        a.K = p->K;
        a.N = N;
        a.nstripes = p->tiles.nstripes;
        a.err = p->d_error;
        a.kt_total = p->tiles.kt_pad;
        a.n_blocks = (N + 16 * CT - 1) / (16 * CT);
        // a workgroup's 8 wavefronts hold 2 stripes each: slices of at most 16 stripes (more
        // slices on request: each streams all of the block's X again)
        int slices = pl.wg_rows ? pl.wg_rows : env_int("UBP_WGROWS", 0);
        if (slices < 0) return UBP_ERR_INVALID_ARG;
        slices = std::min(std::max(slices, (a.nstripes + 15) / 16), a.nstripes);
        a.sps = (a.nstripes + slices - 1) / slices;
        slices = (a.nstripes + a.sps - 1) / a.sps;
        if ((int64_t)a.n_blocks * slices > 0x7fffffff) return UBP_ERR_UNSUPPORTED;
        constexpr int KT = 4; // chunks of 128 rows: X fragments, two weight sets and two chunks of X loads in 170 registers
        int SW = pl.sub_stripes ? pl.sub_stripes : env_int("UBP_G", 0);
        if (SW == 0) SW = 4;
#define UBP_XCHUNK_CASE(CC, KK, SS)                                                                    \
    if (CT == CC && SW == SS) {                                                                        \
        if (p->dtype == UBP_BF16)                                                                      \
            return y_dtype == UBP_F32 ? launch_xchunk<true, float, CC, KK, SS>(a, slices, st)          \
                                      : launch_xchunk<true, __bf16, CC, KK, SS>(a, slices, st);        \
        return y_dtype == UBP_F32 ? launch_xchunk<false, float, CC, KK, SS>(a, slices, st)             \
                                  : launch_xchunk<false, _Float16, CC, KK, SS>(a, slices, st);         \
    }
        UBP_XCHUNK_CASE(2, KT, 2) UBP_XCHUNK_CASE(4, KT, 2) UBP_XCHUNK_CASE(2, KT, 4) UBP_XCHUNK_CASE(4, KT, 4)
#undef UBP_XCHUNK_CASE
        return UBP_ERR_UNSUPPORTED;
    }
    if (kernel == 4) {
        if (!tile_ok) return UBP_ERR_UNSUPPORTED;
        const int KT = p->tiles.kt_pad;
        int CT = pl.col_tiles ? pl.col_tiles : env_int("UBP_CT", 0);
        // 64-pixel blocks halve the weight traffic per pixel; 32-pixel blocks where those would be few
        if (CT == 0) CT = N >= 128 * 64 ? 4 : 2;
        if (CT != 2 && CT != 4) return UBP_ERR_UNSUPPORTED;
        TileArgs a = {};
        a.frags = p->d_tiles.frags;
        a.X = static_cast<const uint16_t *>(X_dev);
        a.Y = Y_dev;
        a.ldx = ldx;
        a.ldy = ldy;
        a.M = p->M;
        a.K = p->K;
        a.N = N;
        a.nstripes = p->tiles.nstripes;
        a.err = p->d_error;
        a.kt_total = KT;
        a.n_blocks = (N + 16 * CT - 1) / (16 * CT);
        // Workgroups of 4 wavefronts, about one and a half per CU: two share a CU and the one's
        // loading of X overlaps the other's streaming (measured better than one workgroup of 8).
        // The stripes are cut into slices to get there - every slice loads the X block again, so
        // only while a wavefront keeps at least 3 stripes.
        int slices = pl.wg_rows ? pl.wg_rows : env_int("UBP_WGROWS", 0);
        if (slices < 0) return UBP_ERR_INVALID_ARG;
        if (slices == 0) slices = std::max(1, std::min((int)std::lround(384.0 / a.n_blocks), a.nstripes / 12));
        slices = std::min(slices, a.nstripes);
        a.sps = (a.nstripes + slices - 1) / slices;
        slices = (a.nstripes + a.sps - 1) / a.sps;
        int waves = pl.waves ? pl.waves : env_int("UBP_WAVES", 0);
        if (waves == 0) waves = std::min(4, a.sps);
        if (waves < 1 || waves > 8) return UBP_ERR_UNSUPPORTED;
        if ((int64_t)a.n_blocks * slices > 0x7fffffff) return UBP_ERR_UNSUPPORTED;
        if (p->dtype == UBP_BF16)
            return y_dtype == UBP_F32 ? launch_xstat<true, float>(a, CT, KT, waves, slices, st)
                                      : launch_xstat<true, __bf16>(a, CT, KT, waves, slices, st);
        return y_dtype == UBP_F32 ? launch_xstat<false, float>(a, CT, KT, waves, slices, st)
                                  : launch_xstat<false, _Float16>(a, CT, KT, waves, slices, st);
    }
    if (kernel == 3) {
        if (!tile_ok) return UBP_ERR_UNSUPPORTED;
        const int KT = p->tiles.kt_pad;
        int CT = pl.col_tiles ? pl.col_tiles : env_int("UBP_CT", 0);
        if (CT == 0) CT = 2;
        if (CT != 2 && CT != 4) return UBP_ERR_UNSUPPORTED;
        int waves = pl.waves ? pl.waves : env_int("UBP_WAVES", 0);
        if (waves == 0) waves = 8;
        if (waves != 1 && waves != 2 && waves != 4 && waves != 8) return UBP_ERR_UNSUPPORTED;
        TileArgs a = {};
        a.frags = p->d_tiles.frags;
        a.X = static_cast<const uint16_t *>(X_dev);
        a.Y = Y_dev;
        a.ldx = ldx;
        a.ldy = ldy;
        a.M = p->M;
        a.K = p->K;
        a.N = N;
        a.nstripes = p->tiles.nstripes;
        a.err = p->d_error;
        a.kt_total = KT;
        a.n_blocks = (N + waves * 16 * CT - 1) / (waves * 16 * CT);
        // Slices of stripes: a slice's accumulators must fit the registers (32 / CT stripes) and
        // its weight tiles LDS beside the wavefronts' scratch; beyond that, as many workgroups as
        // CUs where the pixel blocks alone are fewer (every slice re-reads the X block).
        int slices = pl.wg_rows ? pl.wg_rows : env_int("UBP_WGROWS", 0);
        if (slices < 0) return UBP_ERR_INVALID_ARG;
        if (slices == 0) slices = std::max(1, (int)std::lround(256.0 / a.n_blocks));
        slices = std::min(slices, a.nstripes);
        const int max_sps = std::min(32 / CT, (int)((160 * 1024 - 2 * 32 * waves * 32 * CT) / (KT * 1024)));
        if (max_sps < 1) return UBP_ERR_UNSUPPORTED;
        slices = std::max(slices, (a.nstripes + max_sps - 1) / max_sps);
        a.sps = (a.nstripes + slices - 1) / slices;
        slices = (a.nstripes + a.sps - 1) / a.sps;
        if (p->dtype == UBP_BF16)
            return y_dtype == UBP_F32 ? launch_tile<true, float>(a, CT, KT, waves, slices, st)
                                      : launch_tile<true, __bf16>(a, CT, KT, waves, slices, st);
        return y_dtype == UBP_F32 ? launch_tile<false, float>(a, CT, KT, waves, slices, st)
                                  : launch_tile<false, _Float16>(a, CT, KT, waves, slices, st);
    }

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
    int NP = pl.producers ? pl.producers : env_int("UBP_PRODUCERS", 0);
    if (NP != 0 && NP != 1 && NP != 2 && NP != 4) return UBP_ERR_UNSUPPORTED;
    int native_req = pl.native ? pl.native : env_int("UBP_NATIVE", 0); // 0 auto, 1 merged columns, 2 block-native
    if (native_req < 0 || native_req > 2) return UBP_ERR_INVALID_ARG;
    if ((G != 0 && G != 1 && G != 2 && G != 4) || (CT != 0 && CT != 2 && CT != 4 && CT != 8)) return UBP_ERR_UNSUPPORTED;
    // Block-native records by themselves only for 16-row blocks, where a block fills the shared
    // operand (shorter blocks leave rows of it empty), and then with 4 stripes x 4 column tiles per
    // wavefront: that shape fits 128 registers, so a workgroup has 14 consumers instead of 6 and X
    // is staged for 5 workgroup rows instead of 11 (largest layer: 159 us against 187 us for the
    // best merged shape).  Elsewhere the shared operand costs more vector ALU work per step
    // than the smaller records save.
    bool native = native_req == 2;
    if (native_req == 0 && p->bh == kStripe && (G == 0 || G == 4) && (CT == 0 || CT == 4) && N % 64 == 0 && N / 64 >= 32 &&
        p->sgn[layout_slot(4, 4)].G != 0 && p->sgn[layout_slot(4, 4)].nch > ring_slots(4)) {
        native = true;
        G = 4;
        CT = 4;
    }
    const StripeLayout *layouts = native ? p->sgn : p->sg;
    // Tile shape, from measurements on the four benchmark layers.
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
        while (G > 1 && layouts[layout_slot(G, CT)].G == 0) G >>= 1;
        if (native && G == 1) G = 2;
    }
    if (layouts[layout_slot(G, CT)].G == 0) return UBP_ERR_UNSUPPORTED; // layout not built for this matrix
    // one wavefront stages about 28 GB/s: a second one as soon as a workgroup's tile is not small
    if (NP == 0) {
        NP = ((int64_t)p->K * 32 * CT >= 64 * 1024) ? 2 : 1;
        if (waves != 0 && waves < NP + 1) NP = 1; // a caller who fixes a tiny workgroup gets one producer
    }
    const int slot = layout_slot(G, CT);
    const StripeLayout &L = layouts[slot];
    const int max_waves = stripe_max_waves(G, CT, native);
    if (max_waves <= NP) return UBP_ERR_UNSUPPORTED;
    // When the ring holds all of K nothing is ever refilled and a consumer may walk several row
    // groups one after the other; the number of workgroup rows is then free.  Otherwise every
    // consumer owns exactly one row group.
    const bool resident = L.nch <= ring_slots(CT);
    int wg_rows = pl.wg_rows ? pl.wg_rows : env_int("UBP_WGROWS", 0);
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

    StripeArgs a;
    const StripeLayoutDev &LD = native ? p->d_sgn[slot] : p->d_sg[slot];
    a.rg_ptr = LD.rg_ptr;
    a.rg_order = LD.rg_order;
    a.stream = LD.stream;
    a.stream_bytes = (uint32_t)(L.stream.size() * sizeof(uint32_t));
    a.X = static_cast<const uint16_t *>(X_dev);
    a.Y = Y_dev;
    a.ldx = ldx;
    a.ldy = ldy;
    a.M = p->M;
    a.K = p->K;
    a.bh = p->bh;
    a.N = N;
    a.nrg = L.nrg;
    a.nch = L.nch;
    a.ring_bytes = std::min(ring_rows(CT), L.nch * kSlotRows) * ring_pitch(CT);
    a.err = p->d_error;
    a.ctile0 = 0;
    a.n_coltiles = 0;
    a.n_wgrows = wg_rows;
    a.n_producers = NP;
    a.resident = resident ? 1 : 0;
    a.vec_ok = vec_ok;
    a.out_bytes = 0; // set per launch
    if (p->dtype == UBP_BF16)
        return y_dtype == UBP_F32 ? launch_stripe<true, float>(a, G, CT, native, waves, st)
                                  : launch_stripe<true, __bf16>(a, G, CT, native, waves, st);
    return y_dtype == UBP_F32 ? launch_stripe<false, float>(a, G, CT, native, waves, st)
                              : launch_stripe<false, _Float16>(a, G, CT, native, waves, st);
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
