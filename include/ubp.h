/*
 * ubp.h - C ABI of the unaligned block-pruned (UBP) sparse x dense product for one
 *         AMD MI355X (gfx950).
 *
 * The operation is the inference computation of a layer pruned with unaligned
 * block-wise pruning (paper: "Realizing Unaligned Block-wise Pruning for DNN
 * Acceleration on Mobile Devices", Sections 3.1, 3.3 and 4.2):
 *
 *      Y[M x N] = W_ubp[M x K] * X[K x N]
 *
 * W_ubp keeps only the weights inside non-overlapping dense bh x bw blocks whose
 * top-left origins (r, c) are arbitrary - not multiples of the block size (Section 3.1;
 * the paper's block is bh x 1, this library also takes bw > 1).  X holds one input
 * channel per row and the pixels (x batch) contiguously; Y likewise for output channels
 * (the O = W * I orientation of Section 3.3).
 *
 * All functions return a ubp_status; none throws, aborts or prints.  Unless stated
 * otherwise pointers are HOST pointers, the caller owns every buffer it passes in, and
 * the library owns only what ubp_pack returns through `out`.
 */
#ifndef UBP_H
#define UBP_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    UBP_OK = 0,
    UBP_ERR_INVALID_ARG = 1,   /* null pointer, non-positive size, bad enum, bad pitch        */
    UBP_ERR_OUT_OF_BOUNDS = 2, /* a block does not lie inside the M x K matrix                 */
    UBP_ERR_OVERLAP = 3,       /* two blocks share a cell (includes duplicates)                */
    UBP_ERR_UNSUPPORTED = 4,   /* valid request this build has no kernel for                   */
    UBP_ERR_INFEASIBLE = 5,    /* no selection with the requested number of blocks exists      */
    UBP_ERR_ALLOC = 6,         /* host or device allocation failed                             */
    UBP_ERR_DEVICE = 7         /* a HIP call failed, or no usable device                       */
} ubp_status;

typedef enum { UBP_F32 = 0, UBP_F16 = 1, UBP_BF16 = 2 } ubp_dtype;

/* Top-left origin of one kept block, 0-based: it covers rows r..r+bh-1, columns c..c+bw-1. */
typedef struct { int32_t r, c; } ubp_block;

/* Packed weights: the canonical host arrays of Section 4.2 plus device-side copies. Opaque. */
typedef struct ubp_packed ubp_packed;

#define UBP_HOST_ONLY (-1)

/*
 * Number of kept blocks for a target density: floor(M*K*density / (bh*bw) + 1e-9), the
 * count rule m = floor(b (1 - p) / N) of Section 3.1 with density = 1 - p.  Returns -1 on
 * bad arguments.
 */
int64_t ubp_target_block_count(int32_t M, int32_t K, int32_t bh, int32_t bw, double density);

/*
 * Test-mask generator (host only, deterministic in all arguments): a valid unaligned
 * block list with ubp_target_block_count() blocks, satisfying the constraints of Eq. 2
 * (no overlap) and the edge rule of Eq. 1 (no block crosses the matrix border).
 *   mode 0: seeded rejection sampling of uniform origins in [0, M-bh] x [0, K-bw].
 *   mode 1: per-stripe block counts follow a capped Zipf law with exponent zipf_s over
 *           stripes of bh start rows (heavy stripes scattered by a seeded permutation),
 *           then rejection sampling inside each stripe.
 * RNG: SplitMix64 seeded with `seed`; bounded draws by rejection (unbiased).
 * out: caller-allocated array of `capacity` blocks; *out_nb receives the count; the
 * list is sorted by (r, c).  UBP_ERR_INVALID_ARG if capacity is too small (then *out_nb
 * still receives the needed count), UBP_ERR_INFEASIBLE if sampling does not terminate.
 */
ubp_status ubp_select_reference(int32_t M, int32_t K, int32_t bh, int32_t bw, double density,
                                uint64_t seed, int32_t mode, double zipf_s,
                                ubp_block *out, int64_t capacity, int64_t *out_nb);

/*
 * Offline weight transform (Section 4.2; it runs once per layer, before inference): dense W +
 * block list -> the WROS sparse format, and, unless device == UBP_HOST_ONLY, its upload to that
 * HIP device (ordinal).
 *
 *   W_host : row-major M x K, leading dimension ldw (elements, >= K), element type dtype.
 *            Only the cells inside blocks are read.
 *   blocks : nb origins in any order.  Rejected, never repaired: UBP_ERR_OUT_OF_BOUNDS if
 *            r < 0, c < 0, r+bh > M or c+bw > K; UBP_ERR_OVERLAP if two blocks share a cell.
 *            nb == 0 is legal (Y becomes all zeros).
 * Canonical arrays (pure functions of the block SET; bits of W copied, never rounded):
 *   indptr [M-bh+2] int32 : indptr[i] = number of blocks whose start row is < i
 *                           (one entry per start row 0..M-bh, then the end sentinel);
 *   indices[nb]     int32 : column origin of each block, blocks ordered by start row and,
 *                           within a start row, by ascending column origin;
 *   values [nb*bw*bh]     : values[(b*bw + q)*bh + s] = W[rho][c_b + q] where rho is the
 *                           row of block b with rho mod bh == s  (weight rotation: the
 *                           weight of output channel i sits in slot i mod bh).
 * The kernels read private re-layouts derived from these arrays.  A re-layout is built and
 * uploaded when the first product that needs it is prepared or run (ubp_spmm_prepare,
 * ubp_spmm, ubp_spmm_plan); a handle holds only the ones that were used.
 * On error *out is NULL.  Free with ubp_packed_free.
 */
ubp_status ubp_pack(const void *W_host, ubp_dtype dtype, int32_t M, int32_t K, int64_t ldw,
                    int32_t bh, int32_t bw, const ubp_block *blocks, int64_t nb,
                    int32_t device, ubp_packed **out);

/* Read-only views of the canonical host arrays; valid until ubp_packed_free. */
const int32_t *ubp_packed_indptr(const ubp_packed *p, int64_t *len);
const int32_t *ubp_packed_indices(const ubp_packed *p, int64_t *len);
const void *ubp_packed_values(const ubp_packed *p, int64_t *len_elems);

/*
 * Y = W_ubp * X on the device the handle was packed for (Sections 3.3 and 4.2: the
 * output-stationary product; every output element is accumulated in fp32 registers and
 * written exactly once).
 *   X_dev : DEVICE pointer, row-major K x N, leading dimension ldx (elements, >= N),
 *           element type = the handle's dtype.
 *   Y_dev : DEVICE pointer, row-major M x N, leading dimension ldy (elements, >= N),
 *           element type y_dtype = UBP_F32 or the handle's dtype (fp32 accumulators are
 *           rounded to nearest-even once, at the store).  Every element of the M x N
 *           result is overwritten, rows no block touches with +0.  X and Y must not alias.
 *   hip_stream : a hipStream_t (NULL = the default stream).  The call only enqueues
 *           kernels on that stream and never synchronises.
 * Allocation: the FIRST call for a given kernel choice (which depends on N and on the
 * alignment of the pointers and pitches) builds and uploads that kernel's re-layout of W - it
 * allocates host and device memory and copies synchronously - and raises the kernel's LDS limit.
 * Every later call with the same choice does neither.  Call ubp_spmm_prepare with the same
 * arguments beforehand (for instance before capturing the stream into a graph) to have all of
 * that done up front.
 * N == 0 is a no-op.  Errors: UBP_ERR_INVALID_ARG (null pointer, N < 0, pitch < N,
 * host-only handle, y_dtype neither fp32 nor the handle's dtype), UBP_ERR_UNSUPPORTED,
 * UBP_ERR_ALLOC, UBP_ERR_DEVICE (launch failed).  Nothing is written to Y on error.
 * Non-finite X: the MFMA kernels multiply whole operand tiles, zero weights included.  An Inf
 * or NaN in a row of X therefore reaches (as NaN) outputs whose exact sum does not contain it:
 * with kernels 4, 5 and 7, every output row whose 16-row stripe keeps a weight within the aligned
 * 32 rows of X around it; with kernel 2, every row of a row group that keeps a weight in that
 * column; with kernel 6, every row of a stripe that a block reaches into whose 16-row window of X
 * (its columns, moved left at the right edge) contains it.  Kernel 1 multiplies kept weights only.
 */
ubp_status ubp_spmm(const ubp_packed *p, const void *X_dev, int64_t ldx, int32_t N,
                    void *Y_dev, int64_t ldy, ubp_dtype y_dtype, void *hip_stream);

/*
 * Same product with the kernel choice pinned (tests and tuning).  Fields set to 0 mean
 * "choose automatically"; an impossible combination returns UBP_ERR_UNSUPPORTED.
 *   kernel     : 1 = vector-ALU kernel that follows the WROS dataflow literally (any
 *                dtype, bh <= 16).
 *                3 = the same kernel with the dataflow the weight rotation replaces (Section
 *                3.3): one output row stored per start row, the other accumulator rows shifted
 *                up by one.  Never chosen automatically; it exists so that the cost of the
 *                shifting can be measured next to kernel 1 (same results bit for bit).
 *                2 = MFMA kernel on aligned 16-row stripes that gathers the rows of X a row
 *                group needs (f16 / bf16).
 *                4, 5 and 7 = MFMA kernels that use W as zero-filled 16 x 32 operand tiles; 4 and 5
 *                skip tiles that keep nothing (f16 / bf16, N a multiple of 8, 16-byte
 *                aligned rows of X and Y; col_tiles 2 or 4; wg_rows = slices the stripes are
 *                cut into, one workgroup per slice and pixel block).
 *                4 (K <= 256) keeps the X of one pixel block in registers and streams the stripes
 *                past it, 16 finished rows at a time - the order of the paper's section 4.2
 *                (waves 1..8 share a slice's stripes).
 *                5 (any K whose zero-filled W stays below 8 MB) cuts K into chunks of 128 rows
 *                that pass through LDS and the registers while the accumulators of 16 stripes
 *                stay (sub_stripes 2 or 4 = stripes per multiplying wavefront; waves fixed; by
 *                itself 4, or 2 with twice the slices where the workgroups would fill less than
 *                half the CUs).
 *                6 = MFMA kernel with whole blocks as operands, stored by row modulo 16 - the
 *                paper's rotation with period 16 (f16 / bf16, bh <= 16, 16 <= K < 65408, N >= 64,
 *                16-byte aligned rows; col_tiles 4 only; sub_stripes 2, 4 or 5 = the most stripes a
 *                wavefront's row group may have: row groups are cut shorter where many blocks start).
 *                7 = MFMA kernel on the same operand tiles with BOTH operands staged in LDS: a
 *                workgroup owns up to 256 rows x 256 pixels of Y for the whole of K (f16 / bf16,
 *                same alignment as 4 and 5; only for matrices whose every tile keeps a weight;
 *                sub_stripes x col_tiles = the workgroup's tile in units of 16 rows x 16 pixels:
 *                16 x 16, 8 x 16, 8 x 8, 16 x 4, 4 x 8 or 4 x 4; 0 = the largest that still gives
 *                about one workgroup per CU).
 *                0 picks 1 for fp32; 6 for 16-row blocks at least 16 wide when K > 1024; else, while
 *                at least half of the 16 x 32 tiles of W keep a weight, 7 (every tile keeps one, and
 *                K <= 256 or N <= 4096), 4 (K <= 256) or 5; else 2.  (3 is never picked.)
 *   sub_stripes: kernels 2 and 6, 16-row stripes per wavefront (1, 2 or 4; kernel 6: 2, 4 or 5,
 *                by itself 5 where that saves a workgroup row, else 4);
 *                kernel 5: 2 or 4.
 *   col_tiles  : kernel 2, 16-column tiles per wavefront (2, 4 or 8); kernels 4 and 5: 2 or 4;
 *                kernel 7: as above.
 *   waves      : wavefronts per workgroup (kernels 2 and 6: producers + 1 .. 16, fewer for shapes
 *                that need many registers; kernel 4 as above).
 *   rows_per_range : kernels 1 and 3, output rows owned by one workgroup row (multiple of bh).
 *   producers  : kernels 2 and 6, wavefronts of a workgroup that stage X into LDS (1, 2 or 4);
 *                the others each own a row group.
 *   wg_rows    : kernels 2 and 6, workgroups that share one column tile (each takes a share of
 *                the row groups).  Free only for kernel 2 when the staged tile holds all K rows
 *                of X at once (K <= 4096 / col_tiles); otherwise it must be 0 or
 *                ceil(row groups / (waves - producers)).  Kernels 4 and 5: slices, as above.
 */
typedef struct {
    int32_t kernel, sub_stripes, col_tiles, waves, rows_per_range, producers, wg_rows;
} ubp_plan;

ubp_status ubp_spmm_plan(const ubp_packed *p, const void *X_dev, int64_t ldx, int32_t N,
                         void *Y_dev, int64_t ldy, ubp_dtype y_dtype, void *hip_stream,
                         const ubp_plan *plan);

/*
 * The product with a fused epilogue, for callers that would otherwise run a second pass over Y
 * (a pruned convolution is followed by its bias and its activation):
 *     Y[i][j] = act( sum_k W[i][k] X[k][j] + bias[i] ),
 * bias added to the fp32 accumulator and the activation applied in fp32 before the one rounding
 * to y_dtype.  All kernels support it; nothing else about the call changes.
 *   bias_dev   : DEVICE pointer to M floats (one per output channel / row of Y), or NULL (no bias).
 *   activation : 0 none; 1 ReLU, max(v, 0); 2 clamp to [lo, hi] (requires lo <= hi, else
 *                UBP_ERR_INVALID_ARG).  max / min are IEEE maxNum / minNum: a NaN becomes the
 *                lower bound.  lo / hi are ignored for 0 and 1.
 * epilogue == NULL, or no bias and activation 0, is ubp_spmm / ubp_spmm_plan; plan may be NULL.
 */
typedef struct {
    const float *bias_dev;
    int32_t activation;
    float lo, hi;
} ubp_epilogue;

ubp_status ubp_spmm_fused(const ubp_packed *p, const void *X_dev, int64_t ldx, int32_t N,
                          void *Y_dev, int64_t ldy, ubp_dtype y_dtype, const ubp_epilogue *epilogue,
                          void *hip_stream, const ubp_plan *plan);

/*
 * Everything ubp_spmm_plan does with these arguments except the launch: resolves the kernel
 * and its shape, builds and uploads the re-layout of W that shape reads (host and device
 * allocation, synchronous copies) and raises the kernel's LDS limit.  X_dev and Y_dev are only
 * looked at for their alignment.  plan may be NULL (automatic choice, as ubp_spmm).  If chosen
 * is not NULL it receives the resolved shape, every field filled in as far as it applies.
 * After it returns UBP_OK, ubp_spmm / ubp_spmm_plan with the same arguments allocate nothing.
 */
ubp_status ubp_spmm_prepare(const ubp_packed *p, const void *X_dev, int64_t ldx, int32_t N,
                            void *Y_dev, int64_t ldy, ubp_dtype y_dtype, const ubp_plan *plan,
                            ubp_plan *chosen);

/*
 * Synchronous health check (copies one word from the device, so it waits for the work queued
 * before it on the NULL stream's terms; call it after synchronising the stream you used).
 * Every wait inside kernels 2, 5 and 6 (the ones whose wavefronts hand data to each other through
 * LDS without barriers) is bounded; a wait that runs out sets a bit here and the kernel finishes
 * with undefined Y instead of hanging.  *flags == 0 means no such event since
 * the handle was packed.
 */
ubp_status ubp_packed_device_error(const ubp_packed *p, uint32_t *flags);

/*
 * Facts about a handle, for reporting.  what:
 *   0 M, 1 K, 2 bh, 3 bw, 4 nb, 5 dtype, 6 device (-1 host only),
 *   7 bytes of the canonical arrays (values + indptr + indices),
 *   8 bytes of all device-side copies made so far,
 *   9 MFMA instructions (16 x 16 x 32) per 16 columns of X that the kept weights would fill
 *     completely: ceil(nb * bh * bw / 512) - the yardstick for the counts below.
 * The following describe private re-layouts and build the one they ask about (host memory
 * only); -1 where it does not exist for this matrix (always for fp32):
 *   10 / 11  dense operand tiles (kernels 4, 5): tiles that keep a weight = MFMAs issued per 16
 *            columns / all 16 x 32 tiles of the matrix;
 *   100 + s / 200 + s  gather layout s = 3 * log2(sub_stripes) + log2(col_tiles) - 1 (kernel 2):
 *            MFMAs issued per 16 columns / steps;
 *   300 + 3 i + g, block layout (kernel 6) for sub_stripes 2, 4, 5 (g = 0, 1, 2): i = 0 MFMAs
 *            issued per 16 columns, 1 steps, 2 half-blocks placed, 3 half-blocks that share a step
 *            with another.
 * Unknown `what` returns -1.
 */
int64_t ubp_packed_info(const ubp_packed *p, int32_t what);

/*
 * Read-only view of one of the MFMA kernels' private weight layouts (host copies, built on
 * demand; valid until ubp_packed_free), so that the host-side re-layout can be checked without
 * a GPU: decoding the records must give back the dense matrix.  Formats: comments of
 * StripeLayout, BlkLayout and TileLayout in csrc/ubp_internal.h.
 *   which = 1: gather layout (sub_stripes, col_tiles as in ubp_plan).  rg_ptr int32[row groups
 *              + 1] first step record of each row group, rg_order int32[row groups] row groups
 *              by decreasing work, stream uint32[stream_words] the step records.
 *   which = 2: block layout (sub_stripes 2, 4 or 5; col_tiles ignored).  Row groups are runs of
 *              1 .. sub_stripes consecutive 16-row stripes (short where many blocks start).
 *              rg_ptr as above; rg_order int32[2 * row groups + 1]: the row groups by decreasing
 *              work, then the first stripe of every row group and, last, the number of stripes;
 *              stream = the operand records (256 words per step), meta = 2 words per step.
 *   which = 3: the dense operand tiles (sub_stripes, col_tiles ignored).  row_groups = number
 *              of 16-row stripes, rg_ptr = rg_order = NULL, stream = [stripes][tiles per
 *              stripe][64 lanes][8] 16-bit weights as 32-bit words (tiles per stripe =
 *              stream_words / (256 * stripes)); lane 16 g + n of a tile holds row n of the
 *              stripe, columns 4 g .. 4 g + 3 and 16 + 4 g .. 16 + 4 g + 3 of the tile's 32;
 *              meta = one bit per tile (bit t % 32 of word stripe * ceil(tiles per stripe / 32)
 *              + t / 32): the tile keeps a weight.
 * Returns UBP_ERR_UNSUPPORTED when that layout does not exist for this matrix (fp32, K too
 * large, block shape not eligible).  Any output pointer may be NULL; meta / meta_words are set
 * to NULL / 0 where a layout has none.
 */
ubp_status ubp_packed_layout(const ubp_packed *p, int32_t sub_stripes, int32_t col_tiles, int32_t which,
                             int32_t *row_groups, const int32_t **rg_ptr, const int32_t **rg_order,
                             const uint32_t **stream, int64_t *stream_words,
                             const uint32_t **meta, int64_t *meta_words);

/* ---------------------------------------------------------------------------------------------
 * Block selection on the host (Sections 3.1, 3.2 and 4.1): which blocks of a dense layer to keep.
 * All pointers are host pointers; nothing here touches a device.
 *
 * Candidates.  The K columns of the M x K matrix form K / bw groups of bw consecutive columns
 * (one input channel each; a remainder of K mod bw columns belongs to no candidate).  Candidate
 * k = i + M * j is the bh x bw block with origin (row i, column j * bw), so the candidates of one
 * column group are consecutive in k and there are b = M * (K / bw) of them (Section 3.1).  Two
 * candidates of one group overlap iff their k differ by less than N = bh, which is the only
 * constraint between kept blocks (Eq. 2).
 *
 * Scores are doubles, finite or -inf; -inf marks a candidate that may never be kept.  A selector
 * given NaN or +inf returns UBP_ERR_INVALID_ARG.  Equal scores: the lower k wins.
 */

/*
 * Importance scores (Eq. 1 with the l1 norm): S[i + M*j] = sum of |W| over the block, -inf where
 * the block would cross the bottom edge (i + bh > M) and, if aligned != 0, where i is not a
 * multiple of bh (which turns every selector below into aligned block-wise pruning; remark after
 * Eq. 2).  W: row-major M x K, pitch ldw elements, read in full.  S: b = M * (K / bw) doubles,
 * caller-allocated; b is passed for checking.
 */
ubp_status ubp_block_scores(const void *W_host, ubp_dtype dtype, int64_t ldw, int32_t M, int32_t K,
                            int32_t bh, int32_t bw, int32_t aligned, double *S, int64_t b);

/*
 * The three selectors share one signature.  S: b scores (not modified).  N: block height in
 * candidates (bh).  m: blocks wanted.  I: caller-allocated, m entries; receives *count candidate
 * indices.  *count can be below m for the first two when no candidate with a score above -inf is
 * left; ubp_select_optimal returns either m indices or UBP_ERR_INFEASIBLE.
 *
 * ubp_select_greedy  (Section 3.2, Eq. 3): best remaining candidate first; a kept k shuts out
 *     k-N+1 .. k+N-1.  I is in order of selection.  O(b log b).
 * ubp_select_bed     (Section 4.1, Algorithms 1 and 2): block expansion -- the best entry of the
 *     score list is kept m times, each time the N-1 entries before it are re-scored as the blocks
 *     that join across the gap and the entry with its N-1 successors leaves the list -- then
 *     block division of the expanded runs into blocks of N.  I ascending.  O(b + m N log b).
 * ubp_select_optimal (Section 3.2, Eq. 4): the selection of exactly m non-overlapping candidates
 *     with the largest total score; of equal totals the one Eq. 4's strict comparison reaches.
 *     I ascending.  O(b m) time and b m bits of memory; UBP_ERR_UNSUPPORTED above 2 GiB of those.
 */
ubp_status ubp_select_greedy(const double *S, int64_t b, int32_t N, int64_t m, int64_t *I, int64_t *count);
ubp_status ubp_select_bed(const double *S, int64_t b, int32_t N, int64_t m, int64_t *I, int64_t *count);
ubp_status ubp_select_optimal(const double *S, int64_t b, int32_t N, int64_t m, int64_t *I, int64_t *count);

/* Candidate indices -> block origins: blocks[t] = (I[t] mod M, (I[t] div M) * bw). */
ubp_status ubp_selection_to_blocks(const int64_t *I, int64_t count, int32_t M, int32_t bw, ubp_block *blocks);

/*
 * Scores, one selector and the conversion in one call: the block list ubp_pack takes, with
 * ubp_target_block_count(M, K, bh, bw, density) blocks (fewer if the selector runs out).
 * method: 0 greedy, 1 expansion + division, 2 optimal.  aligned as in ubp_block_scores.
 * UBP_ERR_INVALID_ARG if capacity is below the target count (*out_nb then holds it).
 */
ubp_status ubp_select_blocks(const void *W_host, ubp_dtype dtype, int64_t ldw, int32_t M, int32_t K,
                             int32_t bh, int32_t bw, double density, int32_t method, int32_t aligned,
                             ubp_block *out, int64_t capacity, int64_t *out_nb);

/*
 * Efficacy of an unaligned selection (Section 5.1, Eq. 5): (|W_ubp| - |W_abp|) / (|W_ep| - |W_abp|)
 * with |W_x| the l1 norm of the weights x keeps; element-wise pruning (ep) keeps the nb*bh*bw
 * largest magnitudes.  l1 (optional, 3 doubles) receives |W_ubp|, |W_abp|, |W_ep|.  Blocks outside
 * the matrix: UBP_ERR_OUT_OF_BOUNDS; overlapping blocks count each weight once.
 */
ubp_status ubp_selection_efficacy(const void *W_host, ubp_dtype dtype, int64_t ldw, int32_t M, int32_t K,
                                  int32_t bh, int32_t bw, const ubp_block *ubp_blocks, int64_t nb,
                                  const ubp_block *abp_blocks, int64_t nb_abp, double *l1, double *efficacy);

/*
 * Enqueues an empty kernel (one wavefront, no memory access) on hip_stream: what a launch costs
 * on this device when there is nothing to do.  For measurement harnesses that report the
 * launch floor next to layers whose HBM time is below it.
 */
ubp_status ubp_launch_floor(void *hip_stream);

/* Releases host and device memory of the handle (NULL is allowed).  Must not be called
 * while a ubp_spmm using the handle is still running on the device. */
void ubp_packed_free(ubp_packed *p);

const char *ubp_status_string(ubp_status s);

#ifdef __cplusplus
}
#endif
#endif /* UBP_H */
