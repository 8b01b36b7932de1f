// Small helper kernels of libplora: metadata upload through kernel arguments, zero page, packing
// of the adapter matrices into MFMA-friendly bf16 buffers, transposed copy of a saved activation.
#include "plora_internal.h"

#include <cstring>

namespace plora {

// ---- metadata upload -------------------------------------------------------------------------
// The blob travels as a by-value kernel argument, so the host copy is consumed at launch time
// and no pinned staging buffer or host-to-device copy is needed (the call stays capturable).
constexpr int kChunkWords = 896;   // 3584 bytes per launch, below the 4 KB kernel-argument limit
struct BlobChunk { uint32_t w[kChunkWords]; };

__global__ void __launch_bounds__(256) k_upload(BlobChunk c, uint32_t *dst, int n_words)
{
    for (int i = threadIdx.x; i < n_words; i += 256) dst[i] = c.w[i];
}

hipError_t upload_blob(void *dst_dev, const void *src_host, size_t bytes, hipStream_t st)
{
    const size_t words = (bytes + 3) / 4;
    const char *src = static_cast<const char *>(src_host);
    for (size_t w0 = 0; w0 < words; w0 += kChunkWords) {
        BlobChunk c;
        const size_t nw = (words - w0 < (size_t)kChunkWords) ? words - w0 : (size_t)kChunkWords;
        const size_t b0 = w0 * 4;
        const size_t nb = (bytes - b0 < nw * 4) ? bytes - b0 : nw * 4;
        std::memset(&c, 0, sizeof(c));
        std::memcpy(c.w, src + b0, nb);
        hipLaunchKernelGGL(k_upload, dim3(1), dim3(256), 0, st, c, static_cast<uint32_t *>(dst_dev) + w0, (int)nw);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

__global__ void __launch_bounds__(256) k_zero_page(uint32_t *p)
{
    p[threadIdx.x] = 0u;   // kZeroBytes = 256 * 4
}

hipError_t clear_zero_page(void *zero_dev, hipStream_t st)
{
    static_assert(kZeroBytes == 1024, "zero page is written by one 256-thread block");
    hipLaunchKernelGGL(k_zero_page, dim3(1), dim3(256), 0, st, static_cast<uint32_t *>(zero_dev));
    return hipGetLastError();
}

// ---- packing of A_k ------------------------------------------------------------------------------
// at: A_k^T as [r16][D] (rows j >= r are zero) - the "row = output column, contraction contiguous"
//     operand of the shrink kernel.
// ap: A_k as [D][rp] with columns j >= r zero - the low-rank K-extension operand of the dX GEMM.
// One block handles 64 rows i of one adapter; the tile goes through LDS so that both the reads of
// A_k (contiguous in j) and the writes of A_k^T (contiguous in i) are coalesced.
__device__ inline void pack_block(const AdapterInfo &a, int64_t D, int bx, uint16_t *at, uint16_t *ap, int want_at,
                                  int want_ap, uint16_t *tile)
{
    // The 64 rows of A_k handled here are one contiguous slab of 64 r elements: copy it to LDS as it is
    // (16 bytes per thread and step), then write both layouts from there.
    const int64_t i0 = (int64_t)bx * 64;
    const int r = a.r;
    const int rows = (int)((D - i0 < 64) ? D - i0 : 64);
    const uint4 *src = reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(a.A) + i0 * r);
    const int n_vec = rows * r / 8;                    // r * 2 bytes * rows is a multiple of 16 when rows == 64
    for (int v = threadIdx.x; v < n_vec; v += 256) reinterpret_cast<uint4 *>(tile)[v] = src[v];
    for (int e = n_vec * 8 + threadIdx.x; e < rows * r; e += 256)
        tile[e] = static_cast<const uint16_t *>(a.A)[i0 * r + e];
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

__global__ void __launch_bounds__(256) k_pack_a(MetaView mv, uint16_t *at, uint16_t *ap, int want_at, int want_ap)
{
    __shared__ __attribute__((aligned(16))) uint16_t tile[64 * PLORA_MAX_RANK];
    const AdapterInfo a = mv.ad[blockIdx.y];
    pack_block(a, mv.hdr->D, blockIdx.x, at, ap, want_at, want_ap, tile);
}

hipError_t launch_pack_bf16(const MetaView &mv, const MetaHeader &h, void *at, void *ap, bool want_at,
                            bool want_ap, hipStream_t st)
{
    if (h.n_adapters == 0 || (!want_at && !want_ap)) return hipSuccess;
    dim3 grid((unsigned)((h.D + 63) / 64), (unsigned)h.n_adapters);
    hipLaunchKernelGGL(k_pack_a, grid, dim3(256), 0, st, mv, static_cast<uint16_t *>(at),
                       static_cast<uint16_t *>(ap), want_at ? 1 : 0, want_ap ? 1 : 0);
    return hipGetLastError();
}

// ---- transposed bf16 copy of a saved fp32 activation ------------------------------------------------
__device__ inline uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// zt[j][t] = bf16(h[t][j]); rows j >= r and the padding tokens are written as zero.  Grid: (token
// block of kSkinnyRows rows, slice of 16 rows inside it).
__device__ inline void h_to_zt_slice(const SegInfo &g, int blk, int slice, const float *hf, uint16_t *zt, float *tile)
{
    constexpr int FR = 16;
    const int t0 = (blk - g.blk0) * kSkinnyRows + slice * FR;   // first token of the slice inside the segment
    if (t0 >= g.lp) return;
    int nt = g.row1 - g.row0 - t0;
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

__global__ void __launch_bounds__(256) k_h_to_zt(MetaView mv, const float *hf, uint16_t *zt)
{
    __shared__ float tile[16 * PLORA_MAX_RANK];
    const int blk = blockIdx.x;
    const SegInfo g = mv.seg[mv.blk_seg[blk]];
    h_to_zt_slice(g, blk, blockIdx.y, hf, zt, tile);
}

hipError_t launch_h_to_zt(const MetaView &mv, const MetaHeader &h, const float *hf, void *zt, hipStream_t st)
{
    if (h.n_blocks == 0) return hipSuccess;
    hipLaunchKernelGGL(k_h_to_zt, dim3((unsigned)h.n_blocks, kSkinnyRows / 16), dim3(256), 0, st, mv, hf, static_cast<uint16_t *>(zt));
    return hipGetLastError();
}

// ---- fused preparation ---------------------------------------------------------------------------
// When the whole metadata blob fits one kernel-argument chunk, a single launch does all the small
// jobs that precede the heavy kernels: block 0 writes the blob and the zero page, the next blocks
// pack the adapter matrices, the last ones make the transposed bf16 copy of a saved activation.
// The packing and copy blocks read the metadata from the kernel argument itself, so they do not wait
// for block 0.
template <typename T> __device__ inline T read_arg(const BlobChunk &c, int byte_off)
{
    static_assert(sizeof(T) % 4 == 0, "metadata structs are made of 32-bit words");
    union { T v; uint32_t w[sizeof(T) / 4]; } u;
#pragma unroll
    for (int i = 0; i < (int)(sizeof(T) / 4); ++i) u.w[i] = c.w[byte_off / 4 + i];
    return u.v;
}

__global__ void __launch_bounds__(256) k_prep(BlobChunk c, uint32_t *meta_dst, int n_words, uint32_t *zero_page,
                                             uint16_t *at, uint16_t *ap, int want_at, int want_ap, int pack_bx,
                                             int n_pack, const float *hf, uint16_t *zt)
{
    __shared__ __attribute__((aligned(16))) union {
        uint16_t pack[64 * PLORA_MAX_RANK];
        float tr[16 * PLORA_MAX_RANK];
    } sh;
    int b = blockIdx.x;
    if (b == 0) {
        for (int i = threadIdx.x; i < n_words; i += 256) meta_dst[i] = c.w[i];
        zero_page[threadIdx.x] = 0u;     // kZeroBytes = 256 * 4
        return;
    }
    b -= 1;
    const MetaHeader hdr = read_arg<MetaHeader>(c, 0);
    const int seg_base = (int)sizeof(MetaHeader);
    const int ad_base = seg_base + hdr.n_seg * (int)sizeof(SegInfo);
    if (b < n_pack) {
        const AdapterInfo a = read_arg<AdapterInfo>(c, ad_base + (b / pack_bx) * (int)sizeof(AdapterInfo));
        pack_block(a, hdr.D, b % pack_bx, at, ap, want_at, want_ap, sh.pack);
        return;
    }
    b -= n_pack;
    const int blk = b / (kSkinnyRows / 16), slice = b % (kSkinnyRows / 16);
    const int tiles = (int)((hdr.T + kGemmTileRows - 1) / kGemmTileRows);
    const int blk_base = ad_base + hdr.n_adapters * (int)sizeof(AdapterInfo) + tiles * (int)sizeof(TileExt);
    const int s = (int)c.w[blk_base / 4 + blk];
    const SegInfo g = read_arg<SegInfo>(c, seg_base + s * (int)sizeof(SegInfo));
    h_to_zt_slice(g, blk, slice, hf, zt, sh.tr);
}

bool prep_fits(size_t blob_bytes) { return blob_bytes <= sizeof(BlobChunk); }

hipError_t launch_prep(const MetaHeader &h, void *meta_dev, const void *blob_host, size_t blob_bytes, void *zero_dev,
                       void *at, void *ap, bool want_at, bool want_ap, const float *hf, void *zt, hipStream_t st)
{
    BlobChunk c;
    std::memset(&c, 0, sizeof(c));
    std::memcpy(c.w, blob_host, blob_bytes);
    const bool pack = h.n_adapters > 0 && (want_at || want_ap);
    const int pack_bx = (int)((h.D + 63) / 64);
    const int n_pack = pack ? pack_bx * h.n_adapters : 0;
    const int n_tr = (hf && zt) ? h.n_blocks * (kSkinnyRows / 16) : 0;
    hipLaunchKernelGGL(k_prep, dim3((unsigned)(1 + n_pack + n_tr)), dim3(256), 0, st, c, static_cast<uint32_t *>(meta_dev),
                       (int)((blob_bytes + 3) / 4), static_cast<uint32_t *>(zero_dev), static_cast<uint16_t *>(at),
                       static_cast<uint16_t *>(ap), want_at ? 1 : 0, want_ap ? 1 : 0, pack_bx > 0 ? pack_bx : 1, n_pack, hf,
                       static_cast<uint16_t *>(zt));
    return hipGetLastError();
}

}  // namespace plora
