// Internal definitions shared by the host-side packer and the HIP launch code.
#pragma once

#include <cstdint>
#include <vector>

#include "ubp.h"

namespace ubp {

constexpr int kStripe = 16;     // rows of one MFMA output tile (aligned row stripe)
constexpr int kStep = 32;       // gathered X rows consumed by one 16x16x32 MFMA
constexpr int kNumG = 3;        // stripes per wavefront: 1, 2, 4
constexpr int kNumKC = 3;       // X rows staged in LDS per chunk: 256, 512, 1024
constexpr int kNumLayouts = kNumG * kNumKC;

// A layout is built for every (G, chunk rows) pair the launcher can choose.
inline int layout_slot(int G, int KC) {
    const int gi = G == 1 ? 0 : G == 2 ? 1 : G == 4 ? 2 : -1;
    const int ki = KC == 256 ? 0 : KC == 512 ? 1 : KC == 1024 ? 2 : -1;
    return (gi < 0 || ki < 0) ? -1 : gi * kNumKC + ki;
}
inline int slot_G(int slot) { return 1 << (slot / kNumKC); }
inline int slot_KC(int slot) { return 256 << (slot % kNumKC); }

// Host image of the MFMA kernel's private re-layout of the packed weights, for one
// choice of G (16-row stripes handled together by one wavefront).
//
// Rows are cut into row groups of 16*G aligned rows.  For a row group the columns of W
// that hold at least one kept weight in it are its "entries"; an entry is one row of X
// to gather plus the 16*G weights of that column (zero where no block covers the row).
// Entries are cut by chunk of chunk_rows X rows, ordered inside a chunk by the set of
// stripes they touch and then by column, and grouped 32 at a time into "steps".
struct StripeLayout {
    int G = 0;
    int chunk_rows = 0; // X rows per LDS chunk
    int nrg = 0;     // row groups
    int nch = 0;     // chunks of X rows
    std::vector<int32_t> rg_ptr;     // [nrg + 1] first step of each row group
    std::vector<int32_t> rg_order;   // row groups, heaviest (most MFMAs) first
    // One fixed-size record per step, (64 + 256*G) dwords, so that the address of any later
    // step is known without reading metadata:
    //   dwords 0..63      : per lane, bits 0-9 / 10-19 = chunk-relative X rows of the lane's two
    //                       transposed LDS reads, bits 20-23 = stripes with nonzero weights,
    //                       bit 24 = last step of its chunk (every (row group, chunk) pair has
    //                       at least one step; an empty pair gets a step with no weights)
    //   then G x 256 dwords: weight fragment of stripe j in MFMA operand order (lane-major,
    //                       8 16-bit values per lane), all zero when the step has no weight there
    std::vector<uint32_t> stream;
    int64_t nsteps = 0;
    int64_t total_mfma = 0;          // MFMA issues per 16-column tile (steps x stripes with weights)
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
    // device side
    int32_t *d_indptr = nullptr;
    int32_t *d_indices = nullptr;
    float *d_values_f32 = nullptr; // rotated values widened to fp32 (exact)
    ubp::StripeLayoutDev d_sg[ubp::kNumLayouts];
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
