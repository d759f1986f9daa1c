// Internal definitions shared by the host-side packer and the HIP launch code.
#pragma once

#include <cstdint>
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

// A layout is built for every (G, CT) the kernel is instantiated for; CT fixes the byte
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

// Host image of the MFMA kernel's private re-layout of the packed weights, for one (G, CT).
//
// Rows are cut into row groups of 16*G aligned rows.  For a row group the columns of W
// that hold at least one kept weight in it are its "entries"; an entry is one row of X
// to gather plus the 16*G weights of that column (zero where no block covers the row).
// Entries are ordered by window of ring_window(CT) X rows, inside a window by the set of stripes
// they touch and then by column, and grouped 32 at a time into "steps" whose rows fit the
// LDS ring together.
struct StripeLayout {
    int G = 0, CT = 0;
    bool native = false; // block-native record format (see below)
    int nrg = 0;     // row groups
    int nch = 0;     // slots (chunks of kSlotRows X rows) the producer stages: ceil(K / 64)
    std::vector<int32_t> rg_ptr;     // [nrg + 1] first step of each row group (step counts are multiples of kPrefetchDepth)
    std::vector<int32_t> rg_order;   // row groups, heaviest (most MFMAs) first
    std::vector<int32_t> sorted_steps; // [nrg] step count of rg_order[i] (host only: work estimates)
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
    //
    // Block-native format (bh <= 16, bw in {4, 8, 16, 32}, G > 1): columns are not merged; a step
    // holds 32 / bw whole blocks, and because a block has at most one row congruent to n modulo
    // 16, ONE fragment serves every stripe: lane (n, g) holds the weight of that row for each of
    // its entries, and the kernel zeroes it for the stripes whose row 16*j + n the block does not
    // cover.  Records are 128 + 256 dwords:
    //       addr as above;  second dword of lane l: bits 0-7 / 8-15 = n - (first row of the block
    //       of the lane's first / second entry quad, relative to the row group) + 64, or 0 for a
    //       padding quad; bit 31 = bit l of the control word (lanes 0..31)
    std::vector<uint32_t> stream;
    int64_t nsteps = 0;
    int64_t total_mfma = 0; // MFMA issues per 16-column tile (steps x stripes with weights)
};

// Host image of the dense-tile kernels' layout: W as 16-row x 32-column operand tiles in MFMA
// operand order, zeros where nothing is kept, for every (stripe, 32-column tile) pair.
// kt_pad = 32-column tiles per stripe: for K <= kTileMaxK rounded up to 2, 4, 6 or 8 (such a
// stripe's tiles and a pixel block's X fit a wavefront's registers at once); for larger K
// rounded up to a multiple of 8 (chunks of 256 rows), built only while the zero-filled matrix
// stays below kTileMaxBytes.
constexpr int kTileMaxK = 256;
constexpr int64_t kTileMaxBytes = 8 << 20;
struct TileLayout {
    int kt_pad = 0;                  // 0: not built
    int nstripes = 0;
    std::vector<uint16_t> frags;     // [nstripes][kt_pad][64 lanes][8]
};
struct TileLayoutDev {
    uint16_t *frags = nullptr;
};

struct StripeLayoutDev {
    int32_t *rg_ptr = nullptr;
    int32_t *rg_order = nullptr;
    uint32_t *stream = nullptr;
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
    // private layouts
    ubp::StripeLayout sg[ubp::kNumLayouts];
    ubp::StripeLayout sgn[ubp::kNumLayouts]; // block-native variants (G = 0 where not built)
    ubp::TileLayout tiles;                   // small-K dense-tile layout (kt_pad = 0 where not built)
    // device side
    int32_t *d_indptr = nullptr;
    int32_t *d_indices = nullptr;
    float *d_values_f32 = nullptr; // rotated values widened to fp32 (exact)
    ubp::StripeLayoutDev d_sg[ubp::kNumLayouts];
    ubp::StripeLayoutDev d_sgn[ubp::kNumLayouts];
    ubp::TileLayoutDev d_tiles;
    uint32_t *d_error = nullptr;   // set by a kernel whose bounded wait ran out
    int64_t device_bytes = 0;
};

namespace ubp {

inline int64_t dtype_size(ubp_dtype d) { return d == UBP_F32 ? 4 : 2; }

// host: builds p->sg[*] from the canonical arrays (16-bit dtypes only)
void build_stripe_layouts(ubp_packed *p);

// device (defined in the HIP translation unit)
ubp_status upload(ubp_packed *p);
void release_device(ubp_packed *p);

} // namespace ubp
