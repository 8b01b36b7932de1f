// Skinny rank-r products of the packed multi-LoRA layer on bf16 inputs (gfx950):
//   shrink  h_t = x_t A_k            (section 2.4; the first half of the low-rank update)
//   dH      g_t = scale_k dy_t B_k^T (appendix C.2, case 2)
// Both stream one big [T][C] matrix once (C = d_in or d_out) against a small per-adapter matrix
// whose rows are output columns with the contraction index contiguous (A_k^T packed, or B_k as it
// is).  They are bound by HBM; the arithmetic runs on 16x16x32 bf16 MFMA with fp32 accumulators so
// that ranks up to 128 stay far below the matrix-core roof.  The rank is never tiled (appendix C.2:
// tile the sequence and hidden dimensions, not the rank).
#include "plora_internal.h"

namespace plora {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

__device__ inline uint16_t bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

constexpr int kMB = kSkinnyRows / 16;   // 16-row MFMA blocks per token block
constexpr int kMaxNB = PLORA_MAX_RANK / 16;

// One workgroup (4 waves) per token block of kSkinnyRows rows of one segment.  The four waves split
// the contraction: wave w takes the 32-wide steps w, w+4, ...; each keeps the whole [64][r16] tile
// in registers and the partial tiles are summed through LDS at the end.
//   MODE 0: small matrix = packed A_k^T [r16][C] (rows >= r are zero),  MODE 1: B_k [r][C].
__global__ void __launch_bounds__(256) k_skinny(MetaView mv, int mode, const uint16_t *__restrict__ S, int64_t C,
                                               const uint16_t *__restrict__ at, float *__restrict__ hf,
                                               uint16_t *__restrict__ hb, uint16_t *__restrict__ zt, int zt_scaled)
{
    extern __shared__ float part[];   // [4][kSkinnyRows][LDP]
    constexpr int NB = kMaxNB;
    const int LDP = mv.hdr->max_r16 + 1;
    const int blk = blockIdx.x;
    const int n_seg = mv.hdr->n_seg;
    int s = 0;
    for (int q = 0; q < n_seg; ++q) {
        const SegInfo gq = mv.seg[q];
        if (gq.adapter >= 0 && gq.row1 > gq.row0 && blk >= gq.blk0) s = q;
    }
    const SegInfo g = mv.seg[s];
    const AdapterInfo a = mv.ad[g.adapter];
    const int t0 = (blk - g.blk0) * kSkinnyRows;
    const int len = g.row1 - g.row0;
    const int nt = (len - t0 < kSkinnyRows) ? len - t0 : kSkinnyRows;
    const int nb = g.r16 / 16;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int lm = lane & 15, kg = lane >> 4;

    const uint16_t *Bm = (mode == 0) ? at + a.at_off : static_cast<const uint16_t *>(a.B);
    const int brows = (mode == 0) ? g.r16 : g.r;     // rows of the small matrix that may be read

    const uint16_t *xrow[kMB];
    bool xok[kMB];
#pragma unroll
    for (int mb = 0; mb < kMB; ++mb) {
        const int tt = mb * 16 + lm;
        xok[mb] = tt < nt;
        xrow[mb] = S + (int64_t)(g.row0 + t0 + (xok[mb] ? tt : 0)) * C + kg * 8;
    }
    const uint16_t *brow[NB];
    bool bok[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        const int j = b * 16 + lm;
        bok[b] = j < brows;
        brow[b] = Bm + (int64_t)(bok[b] ? j : 0) * C + kg * 8;
    }

    f32x4 acc[kMB][NB];
#pragma unroll
    for (int mb = 0; mb < kMB; ++mb)
#pragma unroll
        for (int b = 0; b < NB; ++b) acc[mb][b] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int nks = (int)((C + 31) / 32);
    const bf16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll 2
    for (int ks = wave; ks < nks; ks += 4) {
        const int64_t k0 = (int64_t)ks * 32;
        const bool kok = k0 + kg * 8 < C;
        bf16x8 xf[kMB], bfr[NB];
#pragma unroll
        for (int mb = 0; mb < kMB; ++mb)
            xf[mb] = (xok[mb] && kok) ? *reinterpret_cast<const bf16x8 *>(xrow[mb] + k0) : zero8;
#pragma unroll
        for (int b = 0; b < NB; ++b)
            bfr[b] = (b < nb && bok[b] && kok) ? *reinterpret_cast<const bf16x8 *>(brow[b] + k0) : zero8;
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            if (b < nb) {
#pragma unroll
                for (int mb = 0; mb < kMB; ++mb)
                    acc[mb][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xf[mb], bfr[b], acc[mb][b], 0, 0, 0);
            }
        }
    }

    // partial tiles -> LDS.  Lane holds column j = lm, rows 4*kg + i of each 16x16 block.
    float *mine = part + (size_t)wave * kSkinnyRows * LDP;
#pragma unroll
    for (int mb = 0; mb < kMB; ++mb)
#pragma unroll
        for (int b = 0; b < NB; ++b)
            if (b < nb) {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    mine[(mb * 16 + kg * 4 + i) * LDP + b * 16 + lm] = acc[mb][b][i];
            }
    __syncthreads();

    auto total = [&](int tt, int j) -> float {
        const float *p = part + tt * LDP + j;
        return (p[0] + p[kSkinnyRows * LDP]) + (p[2 * kSkinnyRows * LDP] + p[3 * kSkinnyRows * LDP]);
    };
    const float mult = a.scale;
    const int r = g.r;
    if (hf) {   // fp32 [len][r], unscaled in mode 0 (saved activation), scaled in mode 1
        float *dst = hf + g.h_off + (int64_t)t0 * r;
        for (int e = threadIdx.x; e < nt * r; e += 256) {
            const float v = total(e / r, e % r);
            dst[e] = (mode == 0) ? v : mult * v;
        }
    }
    if (hb) {   // bf16 [len][rp], scaled, zero beyond r
        uint16_t *dst = hb + g.hb_off + (int64_t)t0 * g.rp;
        for (int e = threadIdx.x; e < nt * g.rp; e += 256) {
            const int tt = e / g.rp, j = e % g.rp;
            dst[e] = (j < r) ? bf16_rne(mult * total(tt, j)) : (uint16_t)0;
        }
    }
    if (zt) {   // bf16 [r16][lp] transposed, zero for padding tokens and rows >= r
        uint16_t *dst = zt + g.zt_off + t0;
        const float zm = zt_scaled ? mult : 1.f;
        for (int e = threadIdx.x; e < g.r16 * kSkinnyRows; e += 256) {
            const int j = e / kSkinnyRows, tt = e % kSkinnyRows;
            dst[(int64_t)j * g.lp + tt] = (j < r && tt < nt) ? bf16_rne(zm * total(tt, j)) : (uint16_t)0;
        }
    }
}

hipError_t launch_skinny_bf16(const MetaView &mv, const MetaHeader &h, int mode, const void *S, int64_t C,
                              const void *at, float *hf, void *hb, void *zt, bool zt_scaled, hipStream_t st)
{
    if (h.n_blocks == 0) return hipSuccess;
    const size_t lds = (size_t)4 * kSkinnyRows * (h.max_r16 + 1) * sizeof(float);
    static size_t lds_allowed = 0;
    if (lds > lds_allowed) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_skinny),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        lds_allowed = lds;
    }
    hipLaunchKernelGGL(k_skinny, dim3((unsigned)h.n_blocks), dim3(256), lds, st, mv, mode,
                       static_cast<const uint16_t *>(S), C, static_cast<const uint16_t *>(at), hf,
                       static_cast<uint16_t *>(hb), static_cast<uint16_t *>(zt), zt_scaled ? 1 : 0);
    return hipGetLastError();
}

}  // namespace plora
