// Internal declarations shared by the host entry points and the HIP kernels of libplora.
// Not part of the public interface (that is include/plora.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "plora.h"

namespace plora {

constexpr int kSkinnyRows = 128;   // token block of the shrink / dH kernel (never straddles a segment)
constexpr int kRankPadGemm = 64;   // ranks are padded to one K-step of the GEMM in the bf16 side buffers
constexpr int kRankPadMfma = 16;   // ranks are padded to one MFMA block in the skinny kernels
constexpr int kTokPad = 64;        // segment lengths are padded to this in the transposed side buffers
constexpr int kZeroBytes = 1024;   // zero page at the head of the workspace
constexpr int kTokMaxSplits = 8;    // the dA / dB kernels split the token walk over at most this many workgroups
constexpr int kSkinnyMaxSplits = 8; // the skinny kernels split the contraction over at most this many workgroups

// One entry per segment of the call (empty and base-only segments included).
struct SegInfo {
    int32_t row0, row1;   // token rows [row0, row1)
    int32_t adapter;      // -1: base weight only
    int32_t r;            // rank of the adapter (0 if none)
    int32_t rp;           // rank padded to kRankPadGemm: row pitch of the bf16 side buffer (0 if none)
    int32_t r16;          // rank padded to kRankPadMfma
    int32_t blk0;         // index of this segment's first token block (blocks of kSkinnyRows rows)
    int32_t lp;           // segment length padded to kTokPad: row pitch of the transposed side buffers
    int64_t h_off;        // element offset of the segment in the fp32 activation  [len][r]
    int64_t hb_off;       // element offset in the bf16 side buffer                [len][rp]
    int64_t zt_off;       // element offset in the transposed bf16 side buffers    [r16][lp]
};

// One entry per adapter.
struct AdapterInfo {
    const void *A;        // [d_in][r]
    const void *B;        // [r][d_out]
    float *dA;            // [d_in][r]   (backward only)
    float *dB;            // [r][d_out]  (backward only)
    int32_t r, rp, r16;
    float scale;
    int64_t at_off;       // element offset of A^T  [r16][d_in]  in the packed-A^T buffer
    int64_t ap_off;       // element offset of A    [d_in][rp]   in the padded-A buffer
    int32_t r16_off;      // sum of r16 over the adapters before this one (row offset in dA / dB partial tiles)
    int32_t by_tokens;    // entry i: the adapter with the i-th largest token count (ties by index)
    int32_t seg_list0;    // this adapter's non-empty segments: seg_list[seg_list0 .. seg_list0 + n_own), in segment order
    int32_t n_own;
};

struct MetaHeader {
    int64_t T, D, K;
    int32_t n_seg, n_adapters;
    int32_t n_blocks;     // token blocks of kSkinnyRows rows over all segments
    int32_t max_r16;      // largest rank (padded to 16) among segments with tokens
};

// One entry per 256-row tile of the base GEMMs: the low-rank extension steps of that tile.
constexpr int kGemmTileRows = 256;
struct TileExt {
    int32_t first_seg;    // first segment with an adapter and rows that overlaps the tile (n_seg if none)
    int32_t n_ext;        // extension steps of the tile: sum over such segments of rp / 64
};

// Device view of the metadata blob (all pointers into the workspace).  Blob layout: header, seg[n_seg],
// ad[n_adapters], tile_ext[ceil(T / 256)], blk_seg[n_blocks], seg_list[non-empty segments with an adapter].
struct MetaView {
    const MetaHeader *hdr;
    const SegInfo *seg;
    const AdapterInfo *ad;
    const TileExt *tile_ext;
    const int32_t *blk_seg;   // segment of each token block of kSkinnyRows rows
    const int32_t *seg_list;  // non-empty segments grouped by adapter (see AdapterInfo)
};

// Byte offsets of the workspace regions, each 256-byte aligned.
struct WorkspaceLayout {
    size_t zero, meta, at, ap, hb, zt_h, zt_g, hf, gf, part, wpart, total;
    size_t meta_bytes;
};

struct KernelTimer;   // bench-only event bracketing, see plora_api.hip

// ---- launch wrappers implemented in the kernel files; all enqueue on `st` and return the HIP status ----

hipError_t upload_blob(void *dst_dev, const void *src_host, size_t bytes, hipStream_t st);
hipError_t clear_zero_page(void *zero_dev, hipStream_t st);
// One launch for blob + zero page + packing of A_k + transposed copy of a saved activation (each optional);
// only when prep_fits(blob_bytes).
bool prep_fits(size_t blob_bytes);
hipError_t launch_prep(const MetaHeader &h, void *meta_dev, const void *blob_host, size_t blob_bytes, void *zero_dev,
                       void *at, void *ap, bool want_at, bool want_ap, const float *hf, void *zt, hipStream_t st);

// bf16 path -------------------------------------------------------------------------------------
// Packs A_k^T (zero rows beyond r) and/or A_k padded to rp columns.
hipError_t launch_pack_bf16(const MetaView &mv, const MetaHeader &h, void *at, void *ap, bool want_at,
                            bool want_ap, hipStream_t st);
// Skinny product over token blocks: acc[t][j] = sum_c S[t][c] * Bm_k[j][c]  (c < C).
//   mode 0 (shrink): S = x (C = d_in), Bm_k = packed A_k^T;  mode 1 (dH): S = dy (C = d_out), Bm_k = B_k.
//   `part` receives the fp32 partial tiles of the contraction splits; a finishing kernel sums them and
//   writes (each optional): hf fp32 [len][r] (unscaled in mode 0); hb bf16 [len][rp] = scale_k*acc;
//   zt bf16 [r16][lp] transposed, = (zt_scaled ? scale_k : 1) * acc.
hipError_t launch_skinny_bf16(const MetaView &mv, const MetaHeader &h, int mode, const void *S, int64_t C,
                              const void *at, const void *zero, float *part, float *hf, void *hb, void *zt,
                              bool zt_scaled, hipStream_t st);
// Transposed bf16 copy of a saved fp32 activation: zt[j][t] = bf16(h[t][j]).
hipError_t launch_h_to_zt(const MetaView &mv, const MetaHeader &h, const float *hf, void *zt, hipStream_t st);
// C[T][N] = S[T][Kd] * Wop + side[T][rp] * ext_k, rounded to bf16.
//   forward : S = x,  Wop = W [Kd=d_in][N=d_out] (contraction index is the row index), ext_k = B_k [r][N]
//   backward: S = dy, Wop = W [N=d_in][Kd=d_out] (contraction index is contiguous),    ext_k = padded A_k [N][rp]
hipError_t launch_gemm_bf16(const MetaView &mv, const MetaHeader &h, bool forward, const void *S, const void *W,
                            const void *side, const void *ap, const void *zero, void *C, hipStream_t st);
// Token contraction: out_k = mult * sum_t S[t][c] * zt[j][t] over all segments of adapter k.
//   want_dA: S = x, out = dA_k[c][j], mult = 1;  else S = dy, out = dB_k[j][c], mult = scale_k.
//   n_split > 1: the token walk is split, partial tiles go through `part` ([split][r16_total][C] fp32).
hipError_t launch_tokcontract_bf16(const MetaView &mv, const MetaHeader &h, bool want_dA, const void *S,
                                   int64_t C, const void *zt, const void *zero, float *part, int n_split,
                                   int r16_total, int n_active_adapters, hipStream_t st);
int tokc_splits(const MetaHeader &h, int64_t C, int n_active_adapters);
int skinny_splits(const MetaHeader &h, int64_t C);

// fp32 path (fp64 accumulation) ---------------------------------------------------------------------
hipError_t launch_f32_lowrank(const MetaView &mv, const MetaHeader &h, int mode, const float *S, int64_t C,
                              float *out, hipStream_t st);
hipError_t launch_f32_gemm(const MetaView &mv, const MetaHeader &h, bool forward, const float *S, const float *W,
                           const float *side, float *C, hipStream_t st);
hipError_t launch_f32_wgrad(const MetaView &mv, const MetaHeader &h, bool want_dA, const float *S, int64_t C,
                            const float *side, hipStream_t st);

}  // namespace plora
