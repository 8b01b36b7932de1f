// Small helper kernels of libplora: derivation of the metadata tables from the compact description
// (which travels as a kernel argument), zero page, packing of the adapter matrices into
// MFMA-friendly bf16 buffers, transposed copy of a saved activation.
#include "plora_internal.h"

#include <cstring>
#include <mutex>

namespace plora {

// ---- per-device state ---------------------------------------------------------------------------
constexpr int kMaxDevices = 64;
static std::mutex g_dev_mu;
static int g_cu[kMaxDevices];
static bool g_lds_ok[kMaxDevices][kLdsSlots];

int device_cu_count(hipError_t *err)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) { *err = e != hipSuccess ? e : hipErrorInvalidDevice; return 0; }
    std::lock_guard<std::mutex> lock(g_dev_mu);
    if (g_cu[dev] == 0) {
        int v = 0;
        e = hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess || v < 1) { *err = e != hipSuccess ? e : hipErrorInvalidDevice; return 0; }
        g_cu[dev] = v;
    }
    *err = hipSuccess;
    return g_cu[dev];
}

hipError_t allow_full_lds(const void *kernel, int slot)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices || slot < 0 || slot >= kLdsSlots) return hipErrorInvalidValue;
    std::lock_guard<std::mutex> lock(g_dev_mu);
    if (!g_lds_ok[dev][slot]) {
        e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        g_lds_ok[dev][slot] = true;
    }
    return hipSuccess;
}

// ---- chunked upload of a compact description too long for one kernel argument ----------------------
__global__ void __launch_bounds__(256) k_upload(DescChunk c, uint32_t *dst, int n_words)
{
    for (int i = threadIdx.x; i < n_words; i += 256) dst[i] = c.w[i];
}

static hipError_t upload_words(uint32_t *dst_dev, const uint32_t *src_host, int n_words, hipStream_t st)
{
    for (int w0 = 0; w0 < n_words; w0 += kChunkWords) {
        DescChunk c;
        const int nw = n_words - w0 < kChunkWords ? n_words - w0 : kChunkWords;
        std::memcpy(c.w, src_host + w0, (size_t)nw * 4);
        hipLaunchKernelGGL(k_upload, dim3(1), dim3(256), 0, st, c, dst_dev + w0, nw);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// ---- packing of A_k ------------------------------------------------------------------------------
// at: A_k^T as [r16][D] (rows j >= r are zero) - the "row = output column, contraction contiguous"
//     operand of the shrink kernel.
// ap: A_k as [D][rp] with columns j >= r zero - the low-rank K-extension operand of the dX GEMM.
// One block handles 64 rows i of one adapter; the tile goes through LDS so that both the reads of
// A_k (contiguous in j) and the writes of A_k^T (contiguous in i) are coalesced.
struct PackJob {
    const uint16_t *A;
    int r, rp, r16;
    int64_t at_off, ap_off;
};

__device__ inline void pack_block(const PackJob &a, int64_t D, int bx, uint16_t *at, uint16_t *ap, int want_at,
                                  int want_ap, uint16_t *tile)
{
    // The 64 rows of A_k handled here are one contiguous slab of 64 r elements: copy it to LDS as it is
    // (16 bytes per thread and step), then write both layouts from there.
    const int64_t i0 = (int64_t)bx * 64;
    const int r = a.r;
    const int rows = (int)((D - i0 < 64) ? D - i0 : 64);
    const uint4 *src = reinterpret_cast<const uint4 *>(a.A + i0 * r);
    const int n_vec = rows * r / 8;                    // r * 2 bytes * rows is a multiple of 16 when rows == 64
    for (int v = threadIdx.x; v < n_vec; v += 256) reinterpret_cast<uint4 *>(tile)[v] = src[v];
    for (int e = n_vec * 8 + threadIdx.x; e < rows * r; e += 256) tile[e] = a.A[i0 * r + e];
    __syncthreads();
    if (want_at) {
        // A_k^T rows j: 64 consecutive elements each; a wave writes one row segment of 128 bytes
        uint16_t *dst = at + a.at_off;
        const int ii = threadIdx.x & 63;
        for (int j = threadIdx.x >> 6; j < a.r16; j += 4)
            if (ii < rows) dst[(int64_t)j * D + i0 + ii] = (j < r) ? tile[ii * r + j] : (uint16_t)0;
    }
    if (want_ap) {
        // padded A_k: rows of rp elements, 8 elements (16 bytes) per thread and step
        uint16_t *dst = ap + a.ap_off + i0 * a.rp;
        const int vec_per_row = a.rp / 8, lanes_per_row = 8;         // rp is a multiple of 64
        const int ii0 = threadIdx.x / lanes_per_row, l = threadIdx.x % lanes_per_row;
        for (int ii = ii0; ii < rows; ii += 256 / lanes_per_row)
            for (int v = l; v < vec_per_row; v += lanes_per_row) {
                union { uint4 q; uint16_t h[8]; } u;
#pragma unroll
                for (int t = 0; t < 8; ++t) { const int j = v * 8 + t; u.h[t] = (j < r) ? tile[ii * r + j] : (uint16_t)0; }
                reinterpret_cast<uint4 *>(dst + (int64_t)ii * a.rp)[v] = u.q;
            }
    }
}

// ---- packing of B_k when W is stored [d_out][d_in] -------------------------------------------------
// bp: B_k^T as [K][rp] with columns j >= r zero - the low-rank K-extension operand of the forward GEMM,
//     which then reads W (and with it this operand) with the contraction index contiguous.
// One block handles 64 columns n of one adapter: rows of B_k come in as 128-byte pieces, go through
// LDS, and leave as whole rows of rp elements.
struct PackBJob {
    const uint16_t *B;
    int r, rp;
    int64_t bp_off;
};

__device__ inline void pack_bt_block(const PackBJob &a, int64_t K, int bx, uint16_t *bp, uint16_t *tile)
{
    const int64_t n0 = (int64_t)bx * 64;
    const int cols = (int)((K - n0 < 64) ? K - n0 : 64);               // a multiple of 8
    const int l = threadIdx.x & 7;
    for (int j = threadIdx.x >> 3; j < a.r; j += 32) {
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (l * 8 < cols) v = *reinterpret_cast<const uint4 *>(a.B + (int64_t)j * K + n0 + l * 8);
        reinterpret_cast<uint4 *>(tile + j * 64)[l] = v;
    }
    __syncthreads();
    uint16_t *dst = bp + a.bp_off + n0 * a.rp;
    const int vec_per_row = a.rp / 8;                                   // rp is a multiple of 64
    for (int e = threadIdx.x; e < cols * vec_per_row; e += 256) {
        const int nn = e / vec_per_row, v = e % vec_per_row;
        union { uint4 q; uint16_t h[8]; } u;
#pragma unroll
        for (int t = 0; t < 8; ++t) { const int j = v * 8 + t; u.h[t] = (j < a.r) ? tile[j * 64 + nn] : (uint16_t)0; }
        reinterpret_cast<uint4 *>(dst + (int64_t)nn * a.rp)[v] = u.q;
    }
}

// ---- transposed bf16 copy of a saved fp32 activation ------------------------------------------------
__device__ inline uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// zt[j][t] = bf16(h[t][j]); rows j >= r and the padding tokens are written as zero.  One workgroup per
// (token block of kSkinnyRows rows, slice of 16 rows inside it).
struct TransposeJob {
    int len, r, r16, lp, t_block;    // segment length and rank; first token of the block inside the segment
    int64_t h_off, zt_off;
};

__device__ inline void h_to_zt_slice(const TransposeJob &g, int slice, const float *hf, uint16_t *zt, float *tile)
{
    constexpr int FR = 16;
    const int t0 = g.t_block + slice * FR;          // first token of the slice inside the segment
    if (t0 >= g.lp) return;
    int nt = g.len - t0;
    nt = nt < 0 ? 0 : (nt < FR ? nt : FR);
    // the nt rows of r floats are contiguous: flat copy, then transposed reads (thread -> rank row j, token tt)
    const float *src = hf + g.h_off + (int64_t)t0 * g.r;
    for (int e = threadIdx.x; e < nt * g.r; e += 256) tile[e] = src[e];
    __syncthreads();
    uint16_t *dst = zt + g.zt_off + t0;
    const int tt = threadIdx.x & 15;
    for (int j = threadIdx.x >> 4; j < g.r16; j += 16)
        dst[(int64_t)j * g.lp + tt] = (j < g.r && tt < nt) ? f32_to_bf16_rne(tile[tt * g.r + j]) : (uint16_t)0;
}

// ---- the preparation kernel ----------------------------------------------------------------------
// Workgroup 0 derives the metadata tables into the workspace and clears the zero page; the next
// n_pack workgroups pack the A_k, the next n_pack_b the B_k (only when W is stored [d_out][d_in]); the
// last ones make the transposed bf16 copy of a saved activation.  The packing and copy workgroups work out the few offsets they need from the compact
// description themselves, so they do not wait for workgroup 0.
struct WordsInArg {
    const DescChunk &c;
    __device__ inline uint32_t word(int i) const { return c.w[i]; }
};

constexpr int kPrepSegCopies = 64 * PLORA_MAX_RANK * 2 / (int)sizeof(SegInfo);   // segment records that fit the pack tile

template <class Src>
__device__ inline void prep_body(const DescReader<Src> &in, char *meta_dst, uint32_t *zero_page, uint16_t *at, uint16_t *ap,
                                 int want_at, int want_ap, int pack_bx, int n_pack, int pack_bx_b, int n_pack_b,
                                 const float *hf, uint16_t *zt, void *shared_mem, int32_t *sort_counts, int32_t *sort_starts)
{
    int b = blockIdx.x;
    if (b == 0) {
        zero_page[threadIdx.x] = 0u;     // kZeroBytes = 256 * 4
        const TableLayout lay = table_layout(in.T(), in.n_seg(), in.n_adapters(), in.n_blocks());
        const Tables t = tables_at(meta_dst, lay);
        // LDS of this workgroup (it packs nothing): the pack tile holds a copy of the segment records when they fit,
        // the second sort array the adapters' GEMM operands and the header; the first sort array is phase 1's scratch
        SegInfo *seg_copy = in.n_seg() <= kPrepSegCopies ? static_cast<SegInfo *>(shared_mem) : nullptr;
        AdapterGemm *ad_copy = reinterpret_cast<AdapterGemm *>(sort_starts);
        MetaHeader *hd_copy = reinterpret_cast<MetaHeader *>(ad_copy + PLORA_MAX_ADAPTERS);
        if (threadIdx.x == 0) derive_phase1(in, t, sort_counts, seg_copy, ad_copy, hd_copy);
        __threadfence_block();
        __syncthreads();
        const MetaHeader hd = *hd_copy;
        const int64_t n_tiles = (hd.T + kGemmTileRows - 1) / kGemmTileRows;
        derive_phase2(t, hd, seg_copy ? seg_copy : t.seg, ad_copy, sort_counts /* tokens */, (int)threadIdx.x, 256);
        if (in.order_is_identity()) {           // all row tiles equally long, or already in order: nothing to sort
            for (int64_t i = threadIdx.x; i < n_tiles; i += 256) t.tile_order[i] = (int32_t)i;
            return;
        }
        __threadfence_block();
        __syncthreads();                        // also: everybody is done with the token counts and the copies
        derive_phase3_count(t, n_tiles, (int)threadIdx.x, 256, sort_counts);
        __syncthreads();
        derive_phase3_scan((int)threadIdx.x, 256, sort_counts, sort_starts);
        __syncthreads();
        derive_phase3_place(t, n_tiles, (int)threadIdx.x, 256, sort_starts);
        return;
    }
    b -= 1;
    if (b < n_pack) {
        const int k = b / pack_bx;
        PackJob a;
        int64_t at_rows = 0, ap_rows = 0;
        for (int j = 0; j < k; ++j) {
            const int rj = in.ad_rank(j);
            at_rows += pad_to(rj, kRankPadMfma);
            ap_rows += pad_to(rj, kRankPadGemm);
        }
        const int64_t D = in.D();
        a.A = static_cast<const uint16_t *>(in.ad_ptr(k, 0));
        a.r = in.ad_rank(k);
        a.rp = pad_to(a.r, kRankPadGemm);
        a.r16 = pad_to(a.r, kRankPadMfma);
        a.at_off = at_rows * D;
        a.ap_off = ap_rows * D;
        pack_block(a, D, b % pack_bx, at, ap, want_at, want_ap, static_cast<uint16_t *>(shared_mem));
        return;
    }
    b -= n_pack;
    if (b < n_pack_b) {
        const int k = b / pack_bx_b;
        int64_t rows = 0;
        for (int j = 0; j < k; ++j) rows += pad_to(in.ad_rank(j), kRankPadGemm);
        const int64_t K = in.K();
        PackBJob a;
        a.B = static_cast<const uint16_t *>(in.ad_ptr(k, 1));
        a.r = in.ad_rank(k);
        a.rp = pad_to(a.r, kRankPadGemm);
        a.bp_off = rows * K;
        pack_bt_block(a, K, b % pack_bx_b, ap, static_cast<uint16_t *>(shared_mem));
        return;
    }
    b -= n_pack_b;
    const int blk = b / (kSkinnyRows / 16), slice = b % (kSkinnyRows / 16);
    // walk the segments up to the one that owns token block blk, keeping the running offsets
    const int n_seg = in.n_seg();
    int64_t h = 0, zto = 0;
    int blk0 = 0, row0 = 0;
    TransposeJob g;
    g.len = 0; g.r = 0; g.r16 = 0; g.lp = 0; g.t_block = 0; g.h_off = 0; g.zt_off = 0;
    for (int s = 0; s < n_seg; ++s) {
        const int row1 = in.seg_row1(s), a = in.seg_adapter(s);
        const int len = row1 - row0;
        row0 = row1;
        if (a < 0) continue;
        const int r = in.ad_rank(a), r16 = pad_to(r, kRankPadMfma), lp = pad_to(len, kTokPad);
        const int nb = (len + kSkinnyRows - 1) / kSkinnyRows;
        if (blk < blk0 + nb) {
            g.len = len; g.r = r; g.r16 = r16; g.lp = lp; g.t_block = (blk - blk0) * kSkinnyRows;
            g.h_off = h; g.zt_off = zto;
            break;
        }
        blk0 += nb;
        h += (int64_t)len * r;
        zto += (int64_t)r16 * lp;
    }
    h_to_zt_slice(g, slice, hf, zt, static_cast<float *>(shared_mem));
}

union PrepShared {
    uint16_t pack[64 * PLORA_MAX_RANK];
    float tr[16 * PLORA_MAX_RANK];
};

__global__ void __launch_bounds__(256) k_prep_arg(DescChunk c, char *meta_dst, uint32_t *zero_page, uint16_t *at, uint16_t *ap,
                                                 int want_at, int want_ap, int pack_bx, int n_pack, int pack_bx_b,
                                                 int n_pack_b, const float *hf, uint16_t *zt)
{
    __shared__ __attribute__((aligned(16))) PrepShared sh;
    __shared__ int32_t sort_counts[256 * kSortKeys], sort_starts[256 * kSortKeys];
    const DescReader<WordsInArg> in{WordsInArg{c}};
    prep_body(in, meta_dst, zero_page, at, ap, want_at, want_ap, pack_bx, n_pack, pack_bx_b, n_pack_b, hf, zt, &sh, sort_counts,
              sort_starts);
}

__global__ void __launch_bounds__(256) k_prep_mem(const uint32_t *desc, char *meta_dst, uint32_t *zero_page, uint16_t *at,
                                                 uint16_t *ap, int want_at, int want_ap, int pack_bx, int n_pack,
                                                 int pack_bx_b, int n_pack_b, const float *hf, uint16_t *zt)
{
    __shared__ __attribute__((aligned(16))) PrepShared sh;
    __shared__ int32_t sort_counts[256 * kSortKeys], sort_starts[256 * kSortKeys];
    const DescReader<WordsInMemory> in{WordsInMemory{desc}};
    prep_body(in, meta_dst, zero_page, at, ap, want_at, want_ap, pack_bx, n_pack, pack_bx_b, n_pack_b, hf, zt, &sh, sort_counts,
              sort_starts);
}

hipError_t launch_prep(const uint32_t *desc_host, int n_words, const MetaHeader &h, char *meta_dev, uint32_t *desc_stage,
                       void *zero_dev, void *at, void *ap, bool want_at, bool want_ap, bool want_bp, const float *hf,
                       void *zt, hipStream_t st)
{
    static_assert(kZeroBytes == 1024, "the zero page is written by one 256-thread workgroup");
    if (want_ap && want_bp) return hipErrorInvalidValue;            // both live in `ap`
    const bool pack = h.n_adapters > 0 && (want_at || want_ap);
    const int pack_bx = (int)((h.D + 63) / 64);
    const int n_pack = pack ? pack_bx * h.n_adapters : 0;
    const int pack_bx_b = (int)((h.K + 63) / 64);
    const int n_pack_b = (want_bp && h.n_adapters > 0) ? pack_bx_b * h.n_adapters : 0;
    const int n_tr = (hf && zt) ? h.n_blocks * (kSkinnyRows / 16) : 0;
    const dim3 grid((unsigned)(1 + n_pack + n_pack_b + n_tr));
    if (n_words <= kChunkWords) {
        DescChunk c;
        std::memcpy(c.w, desc_host, (size_t)n_words * 4);
        hipLaunchKernelGGL(k_prep_arg, grid, dim3(256), 0, st, c, meta_dev, static_cast<uint32_t *>(zero_dev),
                           static_cast<uint16_t *>(at), static_cast<uint16_t *>(ap), want_at ? 1 : 0, want_ap ? 1 : 0,
                           pack_bx > 0 ? pack_bx : 1, n_pack, pack_bx_b > 0 ? pack_bx_b : 1, n_pack_b, hf,
                           static_cast<uint16_t *>(zt));
        return hipGetLastError();
    }
    hipError_t e = upload_words(desc_stage, desc_host, n_words, st);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_prep_mem, grid, dim3(256), 0, st, static_cast<const uint32_t *>(desc_stage), meta_dev,
                       static_cast<uint32_t *>(zero_dev), static_cast<uint16_t *>(at), static_cast<uint16_t *>(ap),
                       want_at ? 1 : 0, want_ap ? 1 : 0, pack_bx > 0 ? pack_bx : 1, n_pack, pack_bx_b > 0 ? pack_bx_b : 1,
                       n_pack_b, hf, static_cast<uint16_t *>(zt));
    return hipGetLastError();
}

}  // namespace plora
