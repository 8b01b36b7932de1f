/*
 * plora_debug.h - export of the segment-packing metadata exactly as the kernels read it (host
 * only, for tests; section 2.4: every token row goes through the adapter of its segment, so the
 * row / segment / adapter indexing is integer work that must be exact).
 *
 * The tables are derived from the description by code that is compiled for the host and the
 * device from one source; the device runs it inside the preparation kernel and writes the tables
 * into the metadata region of the workspace (byte offset ws_meta).  plora_debug_metadata runs the
 * host build and returns the same bytes, so a test can compare them with a brute-force
 * construction without a GPU, and with the workspace contents after a call on a GPU (pointer
 * fields aside: the export is built without adapter pointers, they read as zero).
 *
 * Image layout (little endian, offsets in plora_debug_info):
 *   header   { int64 T, D, K; int32 n_seg, n_adapters, n_blocks, max_r16, w_out_in, reserved;
 *              ptr at_base }   w_out_in = 1 when W is stored [d_out][d_in]; at_base = device address
 *              of the packed A_k^T buffer (zero in the export)
 *   seg[n_seg], seg_stride bytes each:
 *            { int32 row0, row1, adapter, r, rp, r16, blk0, lp; int64 h_off, hb_off, zt_off }
 *            rp = rank padded to 64, r16 = rank padded to 16, lp = length padded to 64, blk0 =
 *            index of the segment's first 128-row token block (only segments with an adapter own
 *            blocks), h_off / hb_off / zt_off = element offsets of the segment in the fp32
 *            activation [len][r], the bf16 low-rank factor [len][rp], the transposed bf16
 *            factors [r16][lp]
 *   ad[n_adapters], ad_stride bytes each:
 *            { ptr A, B, dA, dB; int32 r, rp, r16; float scale; int64 at_off, ap_off;
 *              int32 r16_off, by_tokens, seg_list0, n_own, tokens, reserved; ptr ext_b }
 *            at_off / ap_off = element offsets of A_k^T [r16][d_in] and of A_k padded
 *            [d_in][rp] (W stored [d_out][d_in]: of B_k^T padded [d_out][rp]); ext_b = the
 *            [r][N] low-rank operand of the GEMM that reads W with the contraction index as row
 *            index: B, or at_base + 2 at_off when W is stored [d_out][d_in]; r16_off = sum of r16 of the adapters before; entry i's by_tokens = the
 *            adapter with the i-th most tokens (ties: lower index first); seg_list0 / n_own =
 *            this adapter's slice of seg_list
 *   tile[n_tiles], tile_stride bytes each, one per 256 token rows:
 *            { int32 n_ext, n_own, first_seg, third_seg;
 *              2 x { int32 row0, row1, rp, r; int64 hb_off; ptr B; int64 ap_off } }
 *            n_own = segments with an adapter and at least one row that overlap the tile,
 *            first_seg / third_seg = the first / third of them (n_seg if there is none), the two
 *            records describe the first two; n_ext = the sum of rp / 64 over such segments
 *   blk_seg[n_blocks] int32: segment of each 128-row token block
 *   seg_list int32: the non-empty segments with an adapter, grouped by adapter, in segment order
 *   tile_order[n_tiles] int32: the 256-row tiles in the order the base GEMMs walk them, sorted by min(n_ext, 8),
 *            largest first, tiles of equal class in row order (tiles that run side by side are then equally long)
 */
#ifndef PLORA_DEBUG_H
#define PLORA_DEBUG_H

#include "plora.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    int64_t n_tiles;
    int32_t n_seg, n_adapters, n_blocks, max_r16;
    int32_t seg_stride, ad_stride, tile_stride, desc_words;
    uint64_t off_hdr, off_seg, off_ad, off_tile, off_blk_seg, off_seg_list, table_bytes;
    /* launch plans: contraction splits of shrink / dH, token splits and tile widths of dA / dB */
    int32_t shrink_splits, dh_splits, da_splits, da_tile_cols, db_splits, db_tile_cols;
    int32_t r16_total, n_active;     /* sum of r16 over adapters; adapters that own tokens */
    /* byte offsets of the workspace regions */
    uint64_t ws_zero, ws_meta, ws_desc, ws_at, ws_ap, ws_hb, ws_zt_h, ws_zt_g, ws_hf, ws_gf, ws_part, ws_wpart, ws_total;
    uint64_t h_elems;
    uint64_t off_tile_order;
} plora_debug_info;

/* Fills *info and, if tables_out is not NULL, copies the table image (info->table_bytes bytes;
 * cap must be at least that).  Returns 0, or -1 for an invalid description, a NULL info or a
 * short buffer.  Touches no device. */
int plora_debug_metadata(const plora_desc *desc, plora_debug_info *info, void *tables_out, size_t cap);

#ifdef __cplusplus
}
#endif
#endif /* PLORA_DEBUG_H */
