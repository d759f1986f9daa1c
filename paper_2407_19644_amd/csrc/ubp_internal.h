// Internal definitions shared by the host-side packer, the layout builders and the HIP
// launch code of the UBP library.
#pragma once

#include <cstdint>
#include <mutex>
#include <vector>

#include "ubp.h"

namespace ubp {

constexpr int kStripe = 16;    // rows of one MFMA output tile (aligned row stripe)
constexpr int kStep = 32;      // gathered X rows consumed by one 16x16x32 MFMA
constexpr int kSlotRows = 64;  // X rows per slot of the LDS ring (the unit the producer stages)
constexpr int kPrefetchDepth = 4; // step records a wavefront keeps in flight; row groups hold a multiple of it
constexpr int kNumG = 3;       // stripes per wavefront: 1, 2, 4
constexpr int kNumCT = 3;      // 16-column tiles per wavefront: 2, 4, 8
constexpr int kNumLayouts = kNumG * kNumCT;

// A gather layout exists per (G, CT) the gather kernel is instantiated for; CT fixes the byte
// addresses inside the LDS ring that the records carry.
inline int layout_slot(int G, int CT) {
    const int gi = G == 1 ? 0 : G == 2 ? 1 : G == 4 ? 2 : -1;
    const int ci = CT == 2 ? 0 : CT == 4 ? 1 : CT == 8 ? 2 : -1;
    return (gi < 0 || ci < 0) ? -1 : gi * kNumCT + ci;
}
inline int slot_G(int slot) { return 1 << (slot / kNumCT); }
inline int slot_CT(int slot) { return 2 << (slot % kNumCT); }

// LDS ring geometry for a column-tile width: rows of 32*CT bytes, 128 KB in all, always a
// power-of-two number of rows so that ring row = X row mod rows.
constexpr int ring_pitch(int CT) { return 32 * CT; }
constexpr int ring_rows(int CT) { return 131072 / ring_pitch(CT); }
constexpr int ring_slots(int CT) { return ring_rows(CT) / kSlotRows; }
// Entries are grouped by stripe set inside windows of this many X rows (a quarter of the ring:
// a step may straddle two windows, and the rest of the ring is left to the drift between
// wavefronts and to the chunks the producer has in flight).
constexpr int ring_window(int CT) { return ring_rows(CT) / 4; }

// Position of the 32-byte unit u (16 pixels) inside ring row r is u ^ ring_swizzle(r): LDS
// has 64 four-byte banks, and this spreads 16 consecutive rows of one unit over all of them.
constexpr int ring_swizzle(int CT, int r) { return CT == 2 ? ((r >> 2) & 1) : CT == 4 ? ((r >> 1) & 3) : (r & 7); }

// Host image of the gather kernel's private re-layout of the packed weights, for one (G, CT).
//
// Rows are cut into row groups of 16*G aligned rows.  For a row group the columns of W
// that hold at least one kept weight in it are its "entries"; an entry is one row of X
// to gather plus the 16*G weights of that column (zero where no block covers the row).
// Entries are ordered by window of ring_window(CT) X rows, inside a window by the set of stripes
// they touch and then by column, and grouped 32 at a time into "steps" whose rows fit the
// LDS ring together.
struct StripeLayout {
    int G = 0, CT = 0; // G == 0: not usable for this matrix
    bool built = false;
    int nrg = 0;     // row groups
    int nch = 0;     // slots (chunks of kSlotRows X rows) the producer stages: ceil(K / 64)
    std::vector<int32_t> rg_ptr;     // [nrg + 1] first step of each row group (step counts are multiples of kPrefetchDepth)
    std::vector<int32_t> rg_order;   // row groups, heaviest (most MFMAs) first
    // One fixed-size record per step, (128 + 256*G) dwords, so that the address of any later
    // step is known without reading metadata:
    //   dwords 0..127 : per lane a pair {addr, ctl}
    //       addr bits 0-13 / 14-27 : LDS byte address >> 3 of the lane's two transposed reads
    //                                (ring row, swizzle and the lane's 8-byte column included;
    //                                column tile c is then reached by XOR with c << 5)
    //       addr bits 28-31        : stripes with nonzero weights in this step
    //       ctl (same in all lanes): bits 0-15 highest chunk the step reads, bits 16-31 number
    //                                of leading chunks that no step from here on reads
    //   then G x 256 dwords: weight fragment of stripe j in MFMA operand order (lane-major,
    //                        8 16-bit values per lane), all zero when the step has no weight there
    // A row group's last steps may be empty (no stripes, nothing read): they pad its step count
    // to a multiple of kPrefetchDepth so that the kernel's unrolled loop has a single exit.
    std::vector<uint32_t> stream;
    int64_t nsteps = 0;
    int64_t total_mfma = 0; // MFMA issues per 16-column tile (steps x stripes with weights)
};

// Host image of the block kernel's layout (blocks of at most 16 rows; column tiles of 64 pixels,
// i.e. the ring geometry of CT = 4), for G stripes per wavefront.
//
// Row groups are consecutive runs of at most G aligned 16-row stripes, cut so that runs with many
// blocks are short (a workgroup lasts as long as its heaviest row group).
// A block is cut into "halves" of 16 consecutive columns (a block at most 16 wide is one half).
// For a row group every half of every block that has a row in the group is an incidence.  The X rows of a half are the window [a, a + 16), a = its first column
// (moved left where the window would pass the last row of X).  A step = two halves (A, B) whose
// blocks start in the same stripe of the row group, or one half and nothing.
//   meta : 2 dwords per step
//       m0 : a_A | a_B << 16
//       m1 : bits 0-3 / 4-7  row offset o = (block's first row) mod 16 of half A / B
//            bits 8-11       jj = 1 + index of the stripe (of the row group) the blocks start in,
//                            0 when they start in the stripe above the group, 15 for an empty step
//            bit 12 / 13     some half has rows in stripe jj - 1 ("lower part", rows n >= o) /
//                            in stripe jj ("upper part", rows n < o)
//            bits 22-31      number of leading 64-row chunks of X that no later step reads
//                            (handed back as soon as this step's reads are issued)
//   frags: 256 dwords per step, the MFMA operand of both halves: lane 16 g + n holds, as 16-bit
//          element e (0..3: half A, 4..7: half B), the weight that row-slot n of the block
//          (the block row congruent to n modulo 16: the paper's rotation, Section 4.2, with
//          period 16) has in window row a + ((4 g + e - a) mod 16) - columns are rotated the same
//          way, so that the LDS row a lane reads is congruent to its entry number modulo 16.
// Steps of a row group are contiguous, ordered by the first window row, padded with empty steps
// to a multiple of kPrefetchDepth; kPrefetchDepth spare records end both arrays.
struct BlkLayout {
    int G = 0;
    bool built = false;
    int nrg = 0, nch = 0;
    std::vector<int32_t> rg_ptr;    // [nrg + 1] first step of each row group
    std::vector<int32_t> rg_order;  // [nrg] row groups, heaviest first, then [nrg + 1] the first stripe of each row group
    std::vector<int32_t> rg_first;  // the second part of rg_order while the layout is built
    std::vector<uint32_t> meta, frags;
    int64_t nsteps = 0;
    int64_t total_mfma = 0;   // MFMA issues per 16-column tile
    int64_t halves = 0, paired = 0; // incidences, and how many of them share a step with another
};

// Host image of the dense-tile kernels' layout: W as 16-row x 32-column operand tiles in MFMA
// operand order, zeros where nothing is kept, for every (stripe, 32-column tile) pair.
// kt_pad = 32-column tiles per stripe: for K <= kTileMaxK rounded up to 2, 4, 6 or 8 (such a
// stripe's tiles and a pixel block's X fit a wavefront's registers at once); for larger K
// rounded up to a multiple of 8 (chunks of 256 rows), built only while the zero-filled matrix
// stays below kTileMaxBytes.  occupied holds one bit per tile (bit kt % 32 of word
// stripe * ceil(kt_pad / 32) + kt / 32): the tile has a kept weight.
constexpr int kTileMaxK = 256;
constexpr int64_t kTileMaxBytes = 8 << 20;
struct TileLayout {
    bool built = false;
    int kt_pad = 0;                  // 0: not usable for this matrix
    int nstripes = 0;
    std::vector<uint16_t> frags;     // [nstripes][kt_pad][64 lanes][8]
    std::vector<uint32_t> occupied;
    int64_t tiles_nonzero = 0;
};

struct StripeLayoutDev {
    int32_t *rg_ptr = nullptr;
    int32_t *rg_order = nullptr;
    uint32_t *stream = nullptr;
    bool uploaded = false;
};
struct BlkLayoutDev {
    int32_t *rg_ptr = nullptr;
    int32_t *rg_order = nullptr;
    uint32_t *meta = nullptr;
    uint32_t *frags = nullptr;
    bool uploaded = false;
};
struct TileLayoutDev {
    uint16_t *frags = nullptr;
    uint32_t *occupied = nullptr;
    bool uploaded = false;
};

// ------------------------------------------------------------------ kernel arguments
// What happens to an output value between the accumulator and the store: Y = act(acc + bias[row]),
// in fp32, before the one rounding to Y's type.  on == 0: nothing.  The activation is a clamp to
// [lo, hi] (ReLU: lo = 0, hi = +inf), taken with maxNum / minNum, so that a NaN becomes lo.
struct Epilogue {
    const float *bias; // device, M floats, or null
    int on;
    float lo, hi;
};

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
    uint32_t *err;           // set to nonzero when a bounded wait runs out
    Epilogue ep;
};

struct BlkArgs {
    const int32_t *rg_ptr;
    const int32_t *rg_order;
    const uint32_t *meta;
    const uint32_t *frags;
    uint32_t meta_bytes, frag_bytes;
    const uint16_t *X;
    void *Y;
    int64_t ldx, ldy;
    int M, K, N;
    int nrg, nch;
    int ring_bytes;
    int n_coltiles;          // full 64-pixel column tiles this launch covers (from pixel 0)
    int n_wgrows;
    int n_producers;
    int out_bytes;           // LDS bytes per consumer for leaving 16-bit tiles as whole rows; 0: none
    uint32_t *err;
    Epilogue ep;
};

struct TileArgs {
    const uint16_t *frags;   // [nstripes][KT][64][8]
    const uint32_t *occupied; // one bit per tile, ceil(kt_total / 32) words per stripe
    const uint16_t *X;
    void *Y;
    int64_t ldx, ldy;
    int M, K, N;
    int nstripes, sps;       // stripes in all, stripes per workgroup slice
    int n_blocks;            // pixel blocks
    int slices;              // slices the stripes are cut into
    int kt_total;            // 32-column tiles per stripe in frags
    int skip;                // some tile keeps no weight: run the instantiation that tests the occupancy bits
    uint32_t *err;           // the handle's error flags (bounded waits that ran out)
    Epilogue ep;
};

} // namespace ubp

struct ubp_packed {
    int32_t M = 0, K = 0, bh = 0, bw = 0;
    int64_t nb = 0;
    ubp_dtype dtype = UBP_F32;
    int32_t device = UBP_HOST_ONLY;
    // canonical arrays (Section 4.2 of the paper)
    std::vector<int32_t> indptr, indices;
    std::vector<uint8_t> values; // nb*bw*bh elements of dtype, rotated
    // Private layouts, built on first use (host image) and uploaded on first use on the device;
    // guarded by `lock` because a handle is passed around as a pointer to const.
    mutable std::mutex lock;
    mutable ubp::StripeLayout sg[ubp::kNumLayouts];
    mutable ubp::BlkLayout blk[3];           // G = 2, 4, 5
    mutable ubp::TileLayout tiles;
    // device side
    int32_t *d_indptr = nullptr;
    int32_t *d_indices = nullptr;
    mutable float *d_values_f32 = nullptr; // rotated values widened to fp32 (exact), for the vector kernel
    mutable ubp::StripeLayoutDev d_sg[ubp::kNumLayouts];
    mutable ubp::BlkLayoutDev d_blk[3];
    mutable ubp::TileLayoutDev d_tiles;
    uint32_t *d_error = nullptr;   // set by a kernel whose bounded wait ran out
    mutable int64_t device_bytes = 0;
};

namespace ubp {

inline int64_t dtype_size(ubp_dtype d) { return d == UBP_F32 ? 4 : 2; }
constexpr int kNumBlkLayouts = 3;
inline int blk_slot(int G) { return G == 2 ? 0 : G == 4 ? 1 : G == 5 ? 2 : -1; }

// ---- host: layout builders (ubp_layouts.cpp).  Each builds the host image once; the caller
// holds p->lock.  A layout that cannot be built for this matrix is left marked unusable.
const StripeLayout &get_stripe_layout(const ubp_packed *p, int G, int CT);
const BlkLayout &get_blk_layout(const ubp_packed *p, int G);
const TileLayout &get_tile_layout(const ubp_packed *p);
bool blk_eligible(const ubp_packed *p);

// ---- device (HIP translation units)
ubp_status upload(ubp_packed *p);                 // canonical arrays, at pack time
void release_device(ubp_packed *p);
// upload of one private layout, on first use (caller holds p->lock); UBP_ERR_ALLOC on failure
ubp_status upload_stripe_layout(const ubp_packed *p, int slot);
ubp_status upload_blk_layout(const ubp_packed *p, int slot);
ubp_status upload_tile_layout(const ubp_packed *p);

// Launchers.  `dry` only raises the kernels' dynamic LDS limit on the current device (what a
// first launch of a shape would do), so that a later launch is nothing but a launch.
ubp_status launch_wros(const ubp_packed *p, const void *X, int64_t ldx, int N, void *Y, int64_t ldy, ubp_dtype y_dtype,
                       int rpr, bool naive, const Epilogue &ep, void *stream, bool dry);
ubp_status launch_stripe(const StripeArgs &a, bool bf16, bool y_f32, int G, int CT, int waves, void *stream, bool dry);
int stripe_max_waves(int G, int CT);
ubp_status launch_blk(const BlkArgs &a, bool bf16, bool y_f32, int G, int waves, void *stream, bool dry);
int blk_max_waves(int G);
ubp_status launch_xstat(const TileArgs &a, bool bf16, bool y_f32, int CT, int KT, int waves, void *stream, bool dry);
ubp_status launch_xchunk(const TileArgs &a, bool bf16, bool y_f32, int CT, int SW, void *stream, bool dry);
constexpr int kNumGemmShapes = 6;
void gemm_shape(int shape, int *rows, int *pixels);
ubp_status launch_gemm(const TileArgs &a, bool bf16, bool y_f32, int shape, void *stream, bool dry);
ubp_status launch_floor(void *stream);

} // namespace ubp
