/*
 * paro.h - C ABI of the MI355X (gfx950) PAROAttention hot path (arXiv 2506.16054).
 *
 * The path is the attention call of a visual diffusion transformer after each head's tokens
 * have been reordered by pattern (paper Sec. 4):
 *
 *   paro_permute   (Q, K, V)        reorder tokens into one of the six (F,H,W) orders   Sec. 4.1
 *   paro_quantize  (Q, K, V)        one symmetric scale per block of `block` tokens     Sec. 4.3 (1)
 *   paro_mask_to_blocklist          static per-head bitmask -> compacted live-block list Sec. 4.2 (1),(2)
 *   paro_sparse_attn                FlashAttention-style loop over live blocks only,
 *                                   INT8 QK^T and INT8/INT4 PV with block-wise scales     Sec. 4.2 (2), 4.3
 *   paro_unpermute (O)              put output rows back into the default order          Sec. 4.1
 *
 * plus fused forms of the reorder (Sec. 4.1) and the device-side mask expansion that the
 * per-(transformer block, timestep) mask prefetch needs (Sec. 4.2 (1), App. C).
 *
 * Conventions
 *   - Every function returns 0 (PARO_OK) or a negative paro_status.  Arguments are checked on
 *     the host before anything is launched; on error nothing has been enqueued and
 *     paro_last_error() (thread-local text) says which argument was rejected.
 *   - Pointers are DEVICE pointers unless their name starts with `h_` (host).  The caller owns
 *     every buffer; the library neither allocates nor frees device memory and never
 *     synchronizes.  Device work is enqueued on `stream` (a hipStream_t passed as void*;
 *     NULL = the default stream) and the call returns immediately.
 *   - Tensors are contiguous, row-major, in the stated shape.  perm_ids, masks and block lists
 *     are per head and shared over the batch (the paper finds both prompt-invariant, Sec. 4.1/4.2).
 *   - N = F*Hg*Wg + T_text tokens; k = ceil(N / block) blocks; Npad = k * block.  Reordered
 *     tensors are padded to Npad rows (zero rows), so every block is whole in memory; padded
 *     keys never receive probability mass and padded query rows are never stored by
 *     paro_unpermute.
 */
#ifndef PARO_H
#define PARO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum paro_status {
    PARO_OK = 0,
    PARO_EINVAL = -1,       /* null pointer, bad shape, id or enum out of range            */
    PARO_EUNSUPPORTED = -2, /* valid request the kernels do not cover (see each function)  */
    PARO_EHIP = -3          /* the HIP runtime refused the launch; text in paro_last_error */
} paro_status;

typedef enum paro_dtype { PARO_F32 = 0, PARO_BF16 = 1 } paro_dtype;

/* Memory layout of a quantized (or re-laid-out) operand, per (batch, head):
 *   PARO_ROWS  codes[n][c], n in [0,Npad), c in [0,d)                      - used for Q and K
 *   PARO_VT    codes[blk][c][slot], blk in [0,k), slot in [0,block): the block is stored
 *              transposed (channel-major) with the tokens of the block in "slot" order,
 *              slot = paro_vt_slot(block, n - blk*block).  This is the order in which the PV
 *              matrix instruction consumes the key dimension, so the kernel reads V with
 *              16-byte loads and never transposes on chip.                - used for V
 * For bits == 4, two codes share a byte.  PARO_ROWS: channel 2c in bits 0-3, 2c+1 in bits 4-7.
 * PARO_VT: within each group of 8 consecutive slots, byte t (t = 0..3) holds slot 8g+t in
 * bits 0-3 and slot 8g+4+t in bits 4-7 (two's complement nibbles in [-7, 7]).
 */
typedef enum paro_layout { PARO_ROWS = 0, PARO_VT = 1 } paro_layout;

typedef struct paro_shape {
    int32_t B;      /* batch                                        */
    int32_t nh;     /* heads                                        */
    int32_t d;      /* head dimension: 64 or 128                    */
    int32_t F;      /* latent grid: frames                          */
    int32_t Hg;     /* latent grid: height                          */
    int32_t Wg;     /* latent grid: width                           */
    int32_t T_text; /* text tokens appended after the image tokens  */
    int32_t block;  /* block size for sparsity and quantization: 32 or 64 (paper: 64) */
} paro_shape;

/* ---- host-only helpers (no GPU needed) -------------------------------------------------- */

int paro_version(void);
const char* paro_strerror(int status);
const char* paro_last_error(void);

/* Shape arithmetic; return a negative status on an invalid shape. */
int64_t paro_ntokens(const paro_shape* s); /* N    */
int64_t paro_nblocks(const paro_shape* s); /* k    */
int64_t paro_npad(const paro_shape* s);    /* Npad */

/* Gather index of axis order `perm_id` (Sec. 4.1; the six orders of (F,H,W) numbered
 * lexicographically over the letters FHW, slowest axis first: 0 FHW, 1 FWH, 2 HFW, 3 HWF,
 * 4 WFH, 5 WHF).  h_idx[n'] = position in the default [F,H,W] order of the token that sits at
 * n' after the reorder; text tokens map to themselves.  h_idx has N entries (host). */
int paro_perm_index(const paro_shape* s, int perm_id, int32_t* h_idx);

/* Slot of token `i` (0 <= i < block) inside a PARO_VT block; a bijection on [0, block).
 * Returns a negative status for an unsupported block size or i out of range. */
int paro_vt_slot(int block, int i);

/* Bitmask -> compacted block list (Sec. 4.2: masks are stored as bitmasks, whole blocks are
 * skipped).  h_bitmask: [nh][ceil(k*k/8)] bytes; bit (i*k + j) of a head, LSB first in each
 * byte, says row block i attends column block j (coordinates of the REORDERED sequence).
 * h_row_ptr: [nh][k+1] offsets into h_col_idx (one array for all heads; row (h,i) owns
 * [h_row_ptr[h][i], h_row_ptr[h][i+1]) ); columns ascending within a row.  `cap` is the
 * capacity of h_col_idx in entries; *nnz_out receives the number of live blocks.  If cap is
 * too small the function returns PARO_EINVAL after writing *nnz_out, so a caller may size the
 * array with a first call (h_col_idx may then be NULL with cap 0).  All pointers are host. */
int paro_mask_to_blocklist(int nh, int k, const uint8_t* h_bitmask, int32_t* h_row_ptr,
                           int32_t* h_col_idx, int64_t cap, int64_t* nnz_out);

/* Checks a caller-made block list against what the attention kernels assume (they clamp, they do
 * not check): per head and row block the offsets are an ascending range inside [0, nnz], and the
 * column blocks of a row lie in [0, k) and are strictly ascending - the visiting order of the
 * method (Sec. 4.3 (1),(2): P is quantized per visit, so the order is part of the result), and
 * what lets the kernels treat the ragged last column block as the last entry of its row.
 * Lists made by paro_mask_to_blocklist(_device) satisfy it by construction.  Host pointers.
 * Returns PARO_OK or PARO_EINVAL with the first offending entry in paro_last_error(). */
int paro_check_blocklist(int nh, int k, const int32_t* h_row_ptr, const int32_t* h_col_idx, int64_t nnz);

/* Checks that h_order [B*nh*k] (host) is a permutation of the row blocks 0 .. B*nh*k - 1: a launch
 * order that names a row block twice leaves another one unwritten.  paro_schedule_rows' output
 * satisfies it by construction. */
int paro_check_row_order(const paro_shape* s, const int32_t* h_order);

/* Launch order of the row blocks for paro_sparse_attn (a performance hint, never a change of
 * results).  Rows of a static mask differ widely in live blocks (Sec. 4.2 (3): one threshold per
 * head), so the kernels can start the heaviest row blocks first.  h_order has B*nh*k entries;
 * entry p is the row block (b*nh + h)*k + i that runs at launch position p.  Positions are dealt
 * to the 8 XCDs in 8 contiguous ranges; inside a range, row blocks are sorted by descending live
 * count within groups of consecutive heads whose K and V operands fit one L2 (4 MB) together (so
 * the reordering never evicts the K/V tiles being reused); a range whose heads all fit together is
 * one group.  A range of several groups keeps its lightest row blocks (half as many as the XCD
 * holds workgroups, at most a quarter of the range) out of the groups and starts them last, heaviest
 * first: the launch ends when the last-started row blocks are done, and these are the shortest.
 * When every XCD's range is a whole number of (batch, head) pairs and the heads differ in live
 * blocks (one threshold per head, Sec. 4.2 (3)) so that the natural order would load some XCD more
 * than 2 % above the mean, whole heads are dealt to the ranges heaviest first, each to the range
 * with the least work that still has room; heads of equal work stay in their natural ranges.
 * bits_* size the footprint and, with d and block, name the kernel.  Host only. */
int paro_schedule_rows(const paro_shape* s, int bits_qk, int bits_pv, const int32_t* h_row_ptr,
                       int32_t* h_order);

/* ---- device entry points ---------------------------------------------------------------- */

/* Token reorder (Sec. 4.1): xp[b,h,n',:] = x[b,h,idx_h[n'],:], rows n' >= N of xp set to 0.
 *   h_perm_ids  host, [nh], values 0..5
 *   x           [B,nh,N,d]     dtype
 *   xp          [B,nh,Npad,d]  dtype   (must not alias x) */
int paro_permute(const paro_shape* s, paro_dtype dtype, const uint8_t* h_perm_ids, const void* x,
                 void* xp, void* stream);

/* Inverse reorder of the attention output (Sec. 4.1): o[b,h,idx_h[n'],:] = op[b,h,n',:], n' < N.
 *   op [B,nh,Npad,d] dtype;  o [B,nh,N,d] dtype (must not alias op) */
int paro_unpermute(const paro_shape* s, paro_dtype dtype, const uint8_t* h_perm_ids, const void* op,
                   void* o, void* stream);

/* Block-aligned symmetric quantizer (Sec. 4.3 (1)): for every (b, h, block) one group of
 * `block` tokens x d channels: absmax over rows < N; scale = absmax / qmax in binary32
 * (1.0 if absmax == 0); code = clamp(round_half_even(x / scale), -qmax, qmax) with a correctly
 * rounded binary32 divide; rows >= N give code 0.  qmax = 127 (bits 8) or 7 (bits 4).
 * bits == 16 is the unquantized mode: values are re-laid-out as bf16 without rounding beyond
 * the bf16 cast (exact for PARO_BF16 input) and all scales are 1.
 *   xp      [B,nh,Npad,d] dtype            (reordered, zero-padded input)
 *   codes   bits 8 : int8  [B,nh,Npad,d]     (PARO_ROWS)  or [B,nh,k,d,block]    (PARO_VT)
 *           bits 4 : bytes [B,nh,Npad,d/2]   (PARO_ROWS)  or [B,nh,k,d,block/2]  (PARO_VT)
 *           bits 16: bf16  same index space as bits 8
 *   scales  float32 [B,nh,k] */
int paro_quantize(const paro_shape* s, paro_dtype dtype, int bits, paro_layout layout,
                  const void* xp, void* codes, float* scales, void* stream);

/* Block-sparse attention over the live blocks of each row block (Sec. 4.2 (2), Sec. 4.3):
 * for row block i of head h, visiting its live column blocks j in the order of the list
 * (ascending), with running row maximum m, denominator l and accumulator acc:
 *     X   = (Qc_i Kc_j^T) * sq[i] * sk[j] / sqrt(d)      integer product, i32 accumulate;
 *                                                         keys >= N get -inf
 *     m'  = max(m, rowmax X);  Pt = exp(X - m');  l = l*exp(m-m') + rowsum(Pt)
 *     sP  = max(Pt over the block x block tile, rows < N) / qmax_P;  Pc = round_half_even(Pt / sP)
 *     acc = acc*exp(m-m') + sP * sv[j] * (Pc Vc_j)       integer product, i32 accumulate
 * and finally op_i = acc / l (zeros if the row block has no live block).
 *   bits_qk  8 or 4 (codes, PARO_ROWS; 4-bit codes are widened to 8 bits on chip, gfx950 has no
 *            4-bit matrix instruction) or 16 (bf16 values from paro_quantize(bits 16), PARO_ROWS)
 *   bits_pv  8 or 4 (codes, PARO_VT, P quantized to the same width) or 16 (bf16, PARO_VT, P kept
 *            in bf16);  supported pairs: qk in {8,4} with pv in {8,4}, and (16,16)
 *   q,k      [B,nh,Npad,d] as produced by paro_quantize(..., PARO_ROWS, ...)
 *   v        as produced by paro_quantize(..., PARO_VT, ...)
 *   sq,sk,sv float32 [B,nh,k] (ignored, may be NULL, when the operand is 16-bit)
 *   row_ptr  int32 [nh][k+1], col_idx int32 [nnz]: DEVICE copies of the block list; entries
 *            outside [0,nnz] / [0,k) are clamped, so a corrupt list cannot address outside the
 *            operands (the result is then meaningless but the call is memory-safe).  The columns
 *            of a row must be strictly ascending (paro_check_blocklist on the host copy verifies
 *            a list that did not come from paro_mask_to_blocklist)
 *   row_order int32 [B*nh*k], DEVICE copy of paro_schedule_rows' output, or NULL for the natural
 *            order; must be a permutation of 0..B*nh*k-1 (entries are clamped; a row block that
 *            is missing from it is not computed, one that appears twice is computed twice)
 *   op       [B,nh,Npad,d] out_dtype; rows >= N are written as zeros */
int paro_sparse_attn(const paro_shape* s, int bits_qk, int bits_pv, const void* q, const float* sq,
                     const void* k, const float* sk, const void* v, const float* sv,
                     const int32_t* row_ptr, const int32_t* col_idx, int64_t nnz,
                     const int32_t* row_order, paro_dtype out_dtype, void* op, void* stream);

/* ---- fused forms (Sec. 4.1 "Minimize Hardware Overhead"; App. C "Overhead of Permutation") ----
 * The paper removes the cost of the reorder by folding it into neighbouring kernels, so that
 * only read / write-back addresses change.  These entry points do that at both ends of the
 * path; results are bit-identical to the unfused calls they replace. */

/* paro_permute followed by paro_quantize without the intermediate tensor: the reorder happens
 * in the load addresses of the quantizer.
 *   h_perm_ids  host, [nh], values 0..5
 *   x           [B,nh,N,d] dtype, default token order
 *   codes, scales, bits, layout: exactly as paro_quantize produces them from the reordered tensor */
int paro_permute_quantize(const paro_shape* s, paro_dtype dtype, int bits, paro_layout layout,
                          const uint8_t* h_perm_ids, const void* x, void* codes, float* scales,
                          void* stream);

/* The three paro_permute_quantize calls of one attention call in a single launch: Q and K become
 * PARO_ROWS codes of bits_qk, V becomes PARO_VT codes of bits_pv, each bit-identical to the separate
 * call.  (bits_qk, bits_pv) is one of (8,8), (8,4), (4,4), (4,8), (16,16).
 *   q, k, v     [B,nh,N,d] dtype, default token order
 *   *_codes, s* as paro_quantize lays them out for the given bits and layout; none may alias an input
 *               or another output */
int paro_permute_quantize_qkv(const paro_shape* s, paro_dtype dtype, int bits_qk, int bits_pv,
                              const uint8_t* h_perm_ids, const void* q, const void* k, const void* v,
                              void* q_codes, float* sq, void* k_codes, float* sk, void* v_codes, float* sv,
                              void* stream);

/* paro_sparse_attn followed by paro_unpermute without the intermediate tensor: row n' of the
 * result is stored at row idx_h[n'] of o.  Arguments as paro_sparse_attn, plus
 *   h_perm_ids  host, [nh], values 0..5
 *   o           [B,nh,N,d] out_dtype, default token order (padded rows are not stored) */
int paro_sparse_attn_unpermuted(const paro_shape* s, int bits_qk, int bits_pv, const void* q,
                                const float* sq, const void* k, const float* sk, const void* v,
                                const float* sv, const int32_t* row_ptr, const int32_t* col_idx,
                                int64_t nnz, const int32_t* row_order, const uint8_t* h_perm_ids,
                                paro_dtype out_dtype, void* o, void* stream);

/* ---- optional pre-conditioning of K (not part of the paper's method; the paper's kernel derives from an
 * 8-bit attention kernel that has it) --------------------------------------------------------------
 * Subtracting one constant per (head, channel) from every key changes each logit of a query by the same
 * amount, so the softmax - with or without the block mask - does not see it, while the quantizer of
 * Sec. 4.3 (1) sees blocks without their common offset.
 *
 * paro_k_channel_mean: k_mean[b][h][c] = the mean of k[b][h][:, c] over the N tokens, accumulated in binary64
 * and rounded to bfloat16 (stored as float).  Any constant is valid; the coarse rounding makes this one
 * independent of the order of the additions, hence reproducible bit for bit.
 *   k       [B,nh,N,d] of dtype (device), default token order;  k_mean  float32 [B,nh,d] (device)
 * paro_permute_quantize_smoothed: paro_permute_quantize(layout PARO_ROWS) of k - k_mean, the subtraction
 * (one binary32 operation per element, real tokens only: padded rows stay zero) fused into the loads.
 *   bits 8 or 4;  codes, scales as in paro_quantize(PARO_ROWS). */
int paro_k_channel_mean(const paro_shape* s, paro_dtype dtype, const void* k, float* k_mean, void* stream);
int paro_permute_quantize_smoothed(const paro_shape* s, paro_dtype dtype, int bits, const uint8_t* h_perm_ids,
                                   const void* k, const float* k_mean, void* codes, float* scales, void* stream);

/* paro_sparse_attn_unpermuted with the reorder and quantization of Q folded in as well: the
 * quantization group of Q is the 64-token row block one workgroup owns (Sec. 4.3 (1): groups aligned
 * with the attention block), so each workgroup gathers its rows of Q by the head's axis order and
 * quantizes them to 8 bits itself; the Q codes and scales never exist in memory.  Codes and scales are
 * those of paro_permute_quantize(Q, bits 8), and the result is bit-identical to that call followed by
 * paro_sparse_attn_unpermuted(bits_qk 8) - except at d = 128 with bits_pv 8, where the two entry points run
 * different kernels whose floating-point sums associate differently: there the results agree to the
 * rounding of the output type.
 *   q_dtype  type of q;  q  [B,nh,N,d], default token order, unquantized
 *   bits_pv  8 or 4;  k, sk, v, sv and everything else as in paro_sparse_attn_unpermuted (bits_qk 8)
 * Requires block == 64 (PARO_EUNSUPPORTED otherwise). */
int paro_sparse_attn_unpermuted_rawq(const paro_shape* s, paro_dtype q_dtype, int bits_pv, const void* q,
                                     const void* k, const float* sk, const void* v, const float* sv,
                                     const int32_t* row_ptr, const int32_t* col_idx, int64_t nnz,
                                     const int32_t* row_order, const uint8_t* h_perm_ids,
                                     paro_dtype out_dtype, void* o, void* stream);

/* ---- mask prefetch (Sec. 4.2 (1), per-head masks fetched just before use; App. C "Overhead of Prefetch") ----
 * Masks differ per transformer block and timestep, so only the mask of the call at hand lives on
 * the GPU: while attention runs with one block list, the caller copies the next bitmask to the
 * device on a second stream and expands it there into a second block list (two buffers, used in
 * turn).  This entry point is that expansion; it is paro_mask_to_blocklist with every pointer on
 * the DEVICE, and produces the same row_ptr and col_idx, bit for bit.
 *   bitmask  [nh][ceil(k*k/8)] bytes, layout as paro_mask_to_blocklist; bits at or above k*k of a
 *            head are ignored
 *   row_ptr  int32 [nh][k+1], written in full
 *   col_idx  int32 [cap]; live blocks beyond `cap` entries are dropped (row_ptr still counts them:
 *            pass the same cap as `nnz` to paro_sparse_attn, which clamps).  cap = nh*k*k always
 *            suffices; cap may be 0 with col_idx NULL to obtain only row_ptr and the total.
 *   nnz_out  optional int32 on the device: receives the number of live blocks
 * The three small kernels it enqueues on `stream` read and write only these buffers; ordering
 * against the attention call that consumes (or still reads) them is the caller's, by events. */
int paro_mask_to_blocklist_device(int nh, int k, const uint8_t* bitmask, int32_t* row_ptr,
                                  int32_t* col_idx, int64_t cap, int32_t* nnz_out, void* stream);

/* The last step of paro_mask_to_blocklist_device alone, for masks whose offsets were computed
 * offline (masks are static, Sec. 4.2: `row_ptr` can be stored beside each bitmask, 4 bytes per row
 * block): writes the live columns of every row block, ascending, at the given offsets.  One small
 * kernel, so the per-step device work of the mask prefetch is a single copy and a single launch.
 *   bitmask as above;  row_ptr int32 [nh][k+1] (DEVICE), as paro_mask_to_blocklist produces it;
 *   col_idx int32 [cap]; entries whose position falls outside [0, cap) are dropped (a corrupt
 *   row_ptr cannot make the kernel write outside col_idx). */
int paro_blocklist_cols_device(int nh, int k, const uint8_t* bitmask, const int32_t* row_ptr,
                               int32_t* col_idx, int64_t cap, void* stream);

/* ---- offline calibration (Sec. 4.1 "Metric for Permutation Order"; Sec. 4.2 (3) "Efficient
 * Offline Mask Generation") -----------------------------------------------------------------
 * Run once per model on one or two calibration samples of Q and K: for each of the six axis
 * orders, statistics of the b x b blocks of the post-softmax map P = softmax(Q K^T / sqrt(d)) of
 * the reordered sequence give the two metrics of Sec. 4.1; the order with the lowest combined
 * metric is chosen per head; block sums of the chosen order, thresholded at a requested density,
 * give the head's static mask.  The map itself is never stored.
 *
 * Typical sequence, all on one stream:
 *   for t in 0..5:  paro_permute_quantize(bits 16, PARO_ROWS, perm_ids = t for every head) on Q and K
 *                   paro_calib_block_stats -> paro_calib_metrics(m_sparse6 + t*nh, m_quant6 + t*nh)
 *   paro_calib_choose -> perm_ids (copy the nh bytes to the host: the other entry points take them there)
 *   paro_permute_quantize(bits 16, chosen perm_ids) -> paro_calib_block_stats -> paro_calib_mask
 *   -> bitmask, ready for paro_mask_to_blocklist(_device). */

/* Per-block statistics of P for operands that are already reordered (Eq. (M_sparse), (M_quant)).
 * P is formed from the 16-bit operands with fp32 accumulation; entries of padded rows and
 * columns (beyond N) do not exist and enter no statistic.
 *   q16, k16   bf16 [B,nh,Npad,d] as produced by paro_(permute_)quantize(bits 16, PARO_ROWS)
 *   eps        threshold of Eq. (M_sparse) (paper: e.g. 1e-3), > 0
 *   block_sum  float32 [B,nh,k,k]  sum of |P| over the block (the block sum of Sec. 4.2 (3))
 *   block_max  float32 [B,nh,k,k]  max of |P| over the block
 *   block_cnt  int32   [B,nh,k,k]  number of entries with |P| < eps  (n_ij of Eq. (M_sparse)) */
int paro_calib_block_stats(const paro_shape* s, const void* q16, const void* k16, float eps,
                           float* block_sum, float* block_max, int32_t* block_cnt, void* stream);

/* The two metrics of one axis order per head (Eq. (M_sparse), Eq. (M_quant)), averaged over the B
 * samples:  m_sparse[h] = share of blocks with n_ij >= sigma * entries_ij (compared in binary32;
 * entries_ij = real entries of the block, b*b except in the ragged last row / column);
 * m_quant[h] = mean over blocks of max|P_ij| / mean|P_ij| (0 for an all-zero block).
 *   sigma in [0,1] (paper: e.g. 0.9);  m_sparse, m_quant: float32 [nh] */
int paro_calib_metrics(const paro_shape* s, const float* block_sum, const float* block_max,
                       const int32_t* block_cnt, float sigma, float* m_sparse, float* m_quant,
                       void* stream);

/* Combined metric (last equation of Sec. 4.1) and the chosen order per head.  The text defines
 * M_sparse as the share of sparse blocks and picks the LOWEST combined value, so the sparsity
 * term enters as the share of blocks that are not sparse, S = 1 - M_sparse:
 *   M[t][h] = alpha * S[t][h] / sum_t S[t][h] + (1 - alpha) * Mq[t][h] / sum_t Mq[t][h]
 * (a term whose normaliser is 0 is 0); perm_ids[h] = argmin_t M[t][h], lowest t on ties.
 *   m_sparse6, m_quant6  float32 [6][nh], row t = paro_calib_metrics of axis order t
 *   m_combined6          float32 [6][nh] (out);  perm_ids  uint8 [nh] (out, DEVICE) */
int paro_calib_choose(int nh, const float* m_sparse6, const float* m_quant6, float alpha,
                      float* m_combined6, uint8_t* perm_ids, void* stream);

/* Static mask of every head by block-sum thresholding with density control (Sec. 4.2 (3)):
 * among the k_img x k_img image blocks (k_img = ceil(F*Hg*Wg / block)) the
 * n_live = round_half_even(density * k_img^2) blocks with the largest block sums (added over the
 * B samples in sample order) are live; equal sums are taken in ascending i*k + j; rows and
 * columns of text blocks are always live (Sec. 4.2 (1)).  Requires k*k <= 393216, and whole image
 * blocks when text tokens follow.
 *   block_sum  float32 [B,nh,k,k] from paro_calib_block_stats on the chosen order of each head
 *   bitmask    uint8 [nh][ceil(k*k/8)] (out), layout as paro_mask_to_blocklist */
int paro_calib_mask(const paro_shape* s, const float* block_sum, float density, uint8_t* bitmask,
                    void* stream);

#ifdef __cplusplus
}
#endif
#endif /* PARO_H */
