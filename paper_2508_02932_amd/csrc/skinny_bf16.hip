// Skinny rank-r products of the packed multi-LoRA layer on bf16 inputs (gfx950):
//   shrink  h_t = x_t A_k            (section 2.4; the first half of the low-rank update)
//   dH      g_t = scale_k dy_t B_k^T (appendix C.2, case 2)
// Both stream one big [T][C] matrix once (C = d_in or d_out) against a small per-adapter matrix
// whose rows are output columns with the contraction index contiguous (A_k^T packed, or B_k as it
// is).  They are bound by HBM, so the kernel is built around keeping bytes in flight: operands go
// HBM -> LDS directly (global_load_lds) through a two-stage ring (more workgroups per compute unit
// pay more here than a deeper ring: measured), the contraction is split over
// workgroups when the batch has too few token blocks to fill the chip, and the arithmetic runs on
// 16x16x32 bf16 MFMA with fp32 accumulators so that ranks up to 128 stay far below the
// matrix-core roof.  The rank is never tiled (appendix C.2: tile the sequence and hidden
// dimensions, not the rank).  Partial tiles of the splits are summed in a fixed order by a small
// finishing kernel that also writes the bf16 copies the later kernels consume.
#include "plora_internal.h"
#include <type_traits>

namespace plora {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T *)(p))

__device__ inline uint16_t bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

constexpr int SK_BK = 64;                              // contraction elements per stage
constexpr int SK_NST = 2;                              // ring stages: 32-64 KB of LDS per workgroup, so 2-3 fit on a compute unit
constexpr int SK_XT = kSkinnyRows * SK_BK * 2;         // 16 KB: [128 tokens][64 k]
constexpr int SK_NW = kSkinnyRows / 32;                // waves per workgroup: a wave owns 32 tokens
constexpr int SK_XL = kSkinnyRows / 8 / SK_NW;         // token-tile load instructions per wave per stage (4)
constexpr int SK_MB = kSkinnyRows / 16 / SK_NW;        // 16-token MFMA blocks per wave (2)
constexpr int SK_BL = (PLORA_MAX_RANK / 8 + SK_NW - 1) / SK_NW;   // small-matrix load instructions per wave per stage, at most
constexpr int SK_MAXNB = PLORA_MAX_RANK / 16;

// s_waitcnt vmcnt(n) for a wave-uniform runtime n (the instruction takes an immediate)
__device__ inline void wait_vmcnt_dyn(int n)
{
#define W_(N) case N: __builtin_amdgcn_s_waitcnt(0x0f70 | (N & 15) | ((N >> 4) << 14)); break;
    switch (n) {
        W_(0) W_(1) W_(2) W_(3) W_(4) W_(5) W_(6) W_(7) W_(8) W_(9) W_(10) W_(11) W_(12) W_(13) W_(14) W_(15)
        W_(16) W_(17) W_(18)
    default: __builtin_amdgcn_s_waitcnt(0x0f70); break;
    }
#undef W_
}

// One workgroup (4 waves) per (token block of 128 rows of one segment, slice of the contraction).
// Stage = 64 contraction elements: the token tile [128][64] and the small-matrix tile [r16][64]
// land in LDS by direct loads (16-byte chunks XOR-swizzled by row so that MFMA operand reads are
// conflict free).  Wave w owns tokens 32w..32w+31 and every rank block, so nothing is reduced
// across waves.  Output: the fp32 partial tile [128][r16] of this slice.
//   mode 0: small matrix = packed A_k^T [r16][C] (rows >= r are zero),  mode 1: B_k [r][C].
// GROUP (mode 0 only): the small matrix of adapter k is the packed A_k^T of several projections, one below the other
// (GroupView); mv is projection 0's view, `at` is not used.
template <bool GROUP>
__global__ void __launch_bounds__(64 * SK_NW) k_skinny(MetaView mv, int mode, const uint16_t *__restrict__ S, int C,
                                               const uint16_t *__restrict__ at, const uint16_t *__restrict__ zero,
                                               float *__restrict__ part, int stages_per_split,
                                               std::conditional_t<GROUP, GroupView, NoGroup> gv)
{
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    const int blk = blockIdx.x;
    const SegInfo g = mv.seg[mv.blk_seg[blk]];
    const AdapterInfo a = mv.ad[g.adapter];
    const int t0 = (blk - g.blk0) * kSkinnyRows;
    const int nt = (g.row1 - g.row0 - t0 < kSkinnyRows) ? g.row1 - g.row0 - t0 : kSkinnyRows;
    int r16 = g.r16, max_r16;
    int p_r16[kMaxGroup];                              // GROUP: rows of each projection's block of the small matrix
    int64_t p_at[kMaxGroup];                           // ... and where the block starts in that projection's buffer
    if constexpr (GROUP) {
        r16 = 0;
#pragma unroll
        for (int p = 0; p < kMaxGroup; ++p) {
            p_r16[p] = 0; p_at[p] = 0;
            if (p < gv.n_proj) {
                const AdapterInfo ap = gv.mv[p].ad[g.adapter];
                p_r16[p] = ap.r16; p_at[p] = ap.at_off;
                r16 += ap.r16;
            }
        }
        max_r16 = gv.max_r16;
    } else {
        max_r16 = mv.hdr->max_r16;
    }
    const int nb = r16 / 16;
    const int stage_bytes = SK_XT + max_r16 * SK_BK * 2;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t lds_base = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)LDS_PTR(char, lds));

    const int n_stage_all = (C + SK_BK - 1) / SK_BK;
    const int st0 = blockIdx.y * stages_per_split;
    int n_st = n_stage_all - st0;
    n_st = n_st < stages_per_split ? n_st : stages_per_split;
    if (n_st < 0) n_st = 0;

    const uint16_t *Bm = GROUP ? nullptr : (mode == 0) ? at + a.at_off : static_cast<const uint16_t *>(a.B);
    const int brows = (mode == 0) ? r16 : g.r;       // rows of the small matrix that exist

    // ---- loader: every load instruction moves 8 rows x 128 bytes; lane -> (row 8q + lane/8, slot
    // lane%8); slot c' of row u holds chunk c' ^ ((u >> 1) & 7).  Token tile: 16 instructions, wave w
    // issues w, w+4, w+8, w+12.  Small-matrix tile: r16/8 instructions, wave w issues w, w+4, ...
    const int lrow = lane >> 3;
    const uint16_t *xp[SK_XL];
    bool xok[SK_XL];
    int xchunk[SK_XL];
#pragma unroll
    for (int jj = 0; jj < SK_XL; ++jj) {
        const int u = (wave + SK_NW * jj) * 8 + lrow;
        xchunk[jj] = (lane & 7) ^ ((u >> 1) & 7);
        xok[jj] = u < nt;
        xp[jj] = S + (int64_t)(g.row0 + t0 + (xok[jj] ? u : 0)) * C + (int64_t)st0 * SK_BK + xchunk[jj] * 8;
    }
    const int nbi = r16 / 8;                                      // small-matrix load instructions per stage
    const int my_b = (nbi > wave) ? (nbi - wave + SK_NW - 1) / SK_NW : 0;     // ... of which this wave issues my_b
    const uint16_t *bp[SK_BL];
    bool bok[SK_BL];
    int bchunk[SK_BL];
#pragma unroll
    for (int jj = 0; jj < SK_BL; ++jj) {
        const int u = (wave + SK_NW * jj) * 8 + lrow;
        bchunk[jj] = (lane & 7) ^ ((u >> 1) & 7);
        bok[jj] = u < brows;
        if constexpr (GROUP) {
            // the 8 rows of an instruction lie in one projection's block (blocks are multiples of 16 rows)
            int first = 0, cum = 0;
            const uint16_t *base = gv.small[0] + p_at[0];
#pragma unroll
            for (int p = 1; p < kMaxGroup; ++p) {
                cum += p_r16[p - 1];
                if (p < gv.n_proj && u >= cum) { first = cum; base = gv.small[p] + p_at[p]; }
            }
            bp[jj] = base + (int64_t)(bok[jj] ? u - first : 0) * C + (int64_t)st0 * SK_BK + bchunk[jj] * 8;
        } else {
            bp[jj] = Bm + (int64_t)(bok[jj] ? u : 0) * C + (int64_t)st0 * SK_BK + bchunk[jj] * 8;
        }
    }
    const int lps = SK_XL + my_b;                                     // loads per stage issued by this wave

    auto load16 = [&](const uint16_t *gp, uint32_t dst) {
        asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gp), "s"(dst));
    };
    auto issue = [&](int st) {       // stage index inside this split; ring slot st % SK_NST
        const uint32_t base = lds_base + (st % SK_NST) * stage_bytes;
        const int k0 = (st0 + st) * SK_BK;
#pragma unroll
        for (int jj = 0; jj < SK_XL; ++jj) {
            const bool ok = xok[jj] && (k0 + xchunk[jj] * 8 < C);
            load16(ok ? xp[jj] + (int64_t)st * SK_BK : zero, base + (wave + SK_NW * jj) * 1024);
        }
#pragma unroll
        for (int jj = 0; jj < SK_BL; ++jj) {
            if (jj < my_b) {
                const bool ok = bok[jj] && (k0 + bchunk[jj] * 8 < C);
                load16(ok ? bp[jj] + (int64_t)st * SK_BK : zero, base + SK_XT + (wave + SK_NW * jj) * 1024);
            }
        }
    };

    // ---- MFMA operands: lane (lm, kg) reads row lm of its block, chunk 4*ks + kg
    const int lm = lane & 15, kg = lane >> 4;
    int xoff[SK_MB];
#pragma unroll
    for (int mb = 0; mb < SK_MB; ++mb) {
        const int u = (wave * SK_MB + mb) * 16 + lm;
        xoff[mb] = u * 128 + ((kg ^ ((u >> 1) & 7)) * 16);                  // ks*4 XORs in (bit 2 of the chunk)
    }
    int boff[SK_MAXNB];
#pragma unroll
    for (int b = 0; b < SK_MAXNB; ++b) {
        const int u = b * 16 + lm;
        boff[b] = SK_XT + u * 128 + ((kg ^ ((u >> 1) & 7)) * 16);
    }
    f32x4 acc[SK_MB][SK_MAXNB];
#pragma unroll
    for (int mb = 0; mb < SK_MB; ++mb)
#pragma unroll
        for (int b = 0; b < SK_MAXNB; ++b) acc[mb][b] = f32x4{0.f, 0.f, 0.f, 0.f};

    for (int p = 0; p < SK_NST - 1; ++p)
        if (p < n_st) issue(p);
    for (int st = 0; st < n_st; ++st) {
        const int ahead = (n_st - 1 - st < SK_NST - 2) ? n_st - 1 - st : SK_NST - 2;
        wait_vmcnt_dyn(ahead * lps);             // this wave's loads of stage st have landed ...
        __builtin_amdgcn_s_waitcnt(0xc07f);      // ... its LDS reads of the slot about to be refilled are done ...
        __builtin_amdgcn_sched_barrier(0);       // (nothing may be moved across the barrier)
        __builtin_amdgcn_s_barrier();            // ... and so are everyone else's; ring slot (st-1) is free
        __builtin_amdgcn_sched_barrier(0);
        if (st + SK_NST - 1 < n_st) issue(st + SK_NST - 1);
        const char *sb = lds + (st % SK_NST) * stage_bytes;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            bf16x8 xf[SK_MB];
#pragma unroll
            for (int mb = 0; mb < SK_MB; ++mb) xf[mb] = *LDS_PTR(const bf16x8, sb + (xoff[mb] ^ (ks * 64)));
#pragma unroll
            for (int b = 0; b < SK_MAXNB; ++b) {
                if (b < nb) {
                    const bf16x8 bf = *LDS_PTR(const bf16x8, sb + (boff[b] ^ (ks * 64)));
#pragma unroll
                    for (int mb = 0; mb < SK_MB; ++mb)
                        acc[mb][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xf[mb], bf, acc[mb][b], 0, 0, 0);
                }
            }
        }
    }

    // partial tile [128][r16] of this (block, split): lane holds column 16b + lm, rows 16*(2w+mb) + 4kg + i
    float *dst = part + ((int64_t)blockIdx.y * gridDim.x + blk) * (kSkinnyRows * max_r16);
#pragma unroll
    for (int mb = 0; mb < SK_MB; ++mb)
#pragma unroll
        for (int b = 0; b < SK_MAXNB; ++b)
            if (b < nb) {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    dst[((wave * SK_MB + mb) * 16 + kg * 4 + i) * r16 + b * 16 + lm] = acc[mb][b][i];
            }
}

// Sums the partial tiles of the splits (fixed order) and writes, each optional:
//   hf fp32 [len][r]   (mode 0: the activation itself; mode 1: scaled by scale_k)
//   hb bf16 [len][rp]  scale_k * sum, zero beyond r           (K-extension operand of the GEMM)
//   zt bf16 [r16][lp]  transposed, zero for padding tokens and rows >= r; scaled if zt_scaled
// GROUP: the partial tiles are those of a fused pass (pitch = the fused rank of the segment's adapter); mv is the view of
// projection `proj`, whose columns start behind those of the projections before it.
template <bool GROUP>
__global__ void __launch_bounds__(256) k_skinny_finish(MetaView mv, int mode, const float *__restrict__ part,
                                                      int n_split, float *__restrict__ hf, uint16_t *__restrict__ hb,
                                                      uint16_t *__restrict__ zt, int zt_scaled,
                                                      std::conditional_t<GROUP, GroupView, NoGroup> gv, int proj)
{
    constexpr int FR = 16;                            // token rows per workgroup (grid.y slices of a block)
    __shared__ float tile[FR * PLORA_MAX_RANK];       // [FR][r16], pitch r16
    const int blk = blockIdx.x;
    const SegInfo g = mv.seg[mv.blk_seg[blk]];
    const float mult = mv.ad[g.adapter].scale;
    const int tb = (blk - g.blk0) * kSkinnyRows;      // first token of the block inside the segment
    const int r0 = blockIdx.y * FR;                   // first row of this slice inside the block
    const int t0 = tb + r0;
    int nt = g.row1 - g.row0 - t0;                    // valid tokens in this slice
    nt = nt < 0 ? 0 : (nt < FR ? nt : FR);
    if (t0 >= g.lp) return;                           // slice lies past the padded segment: nothing to write
    const int r = g.r, r16 = g.r16;
    if constexpr (GROUP) {
        int pitch = 0, col0 = 0;
        for (int p = 0; p < gv.n_proj; ++p) {
            const int rp16 = gv.mv[p].ad[g.adapter].r16;
            if (p < proj) col0 += rp16;
            pitch += rp16;
        }
        const int64_t tile_elems = (int64_t)kSkinnyRows * gv.max_r16;
        const int64_t split_stride = (int64_t)gridDim.x * tile_elems;
        const float *src = part + (int64_t)blk * tile_elems + (int64_t)r0 * pitch + col0;
        const int q = r16 / 4;                        // float4 per row of this projection's columns
        for (int e = threadIdx.x; e < FR * q; e += 256) {
            const int row = e / q, c4 = e - row * q;
            const float *s0 = src + row * pitch + c4 * 4;
            float4 sum = *reinterpret_cast<const float4 *>(s0);
            for (int sp = 1; sp < n_split; ++sp) {    // fixed order
                const float4 v = *reinterpret_cast<const float4 *>(s0 + sp * split_stride);
                sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;
            }
            reinterpret_cast<float4 *>(tile)[e] = sum;
        }
    } else {
        const int64_t tile_elems = (int64_t)kSkinnyRows * mv.hdr->max_r16;
        const int64_t split_stride = (int64_t)gridDim.x * tile_elems;
        // the FR rows of r16 partial sums are contiguous in every split: flat walk, four floats per thread
        const float4 *src = reinterpret_cast<const float4 *>(part + (int64_t)blk * tile_elems + (int64_t)r0 * r16);
        for (int e = threadIdx.x; e < FR * r16 / 4; e += 256) {
            float4 sum = src[e];
            for (int sp = 1; sp < n_split; ++sp) {        // fixed order
                const float4 v = src[sp * (split_stride / 4) + e];
                sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;
            }
            reinterpret_cast<float4 *>(tile)[e] = sum;
        }
    }
    __syncthreads();
    // outputs: thread -> (token tt = tid / 16, columns j = tid % 16 + 16 m), or transposed for zt
    const int hi = threadIdx.x >> 4, lo = threadIdx.x & 15;
    if (hf && hi < nt) {
        float *dst = hf + g.h_off + (int64_t)(t0 + hi) * r;
        for (int j = lo; j < r; j += 16) {
            const float v = tile[hi * r16 + j];
            dst[j] = (mode == 0) ? v : mult * v;
        }
    }
    if (hb && hi < nt) {
        uint16_t *dst = hb + g.hb_off + (int64_t)(t0 + hi) * g.rp;
        for (int j = lo; j < g.rp; j += 16) dst[j] = (j < r) ? bf16_rne(mult * tile[hi * r16 + j]) : (uint16_t)0;
    }
    if (zt) {
        uint16_t *dst = zt + g.zt_off + t0;
        const float zm = zt_scaled ? mult : 1.f;
        for (int j = hi; j < r16; j += 16)
            dst[(int64_t)j * g.lp + lo] = (j < r && lo < nt) ? bf16_rne(zm * tile[lo * r16 + j]) : (uint16_t)0;
    }
}

int skinny_splits(const MetaHeader &h, int64_t C)
{
    if (h.n_blocks == 0) return 1;
    const int n_stage_all = (int)((C + SK_BK - 1) / SK_BK);
    int want = (768 + h.n_blocks - 1) / h.n_blocks;          // aim at >= 3 workgroups per CU
    int cap = n_stage_all / 8;                                // keep at least 8 stages per split
    if (cap < 1) cap = 1;
    if (want > cap) want = cap;
    if (want > kSkinnyMaxSplits) want = kSkinnyMaxSplits;
    if (want < 1) want = 1;
    return want;
}

hipError_t launch_skinny_bf16(const MetaView &mv, const MetaHeader &h, int mode, const void *S, int64_t C,
                              const void *at, const void *zero, float *part, float *hf, void *hb, void *zt,
                              bool zt_scaled, hipStream_t st)
{
    if (h.n_blocks == 0) return hipSuccess;
    const int n_split = skinny_splits(h, C);
    const int n_stage_all = (int)((C + SK_BK - 1) / SK_BK);
    const int per = (n_stage_all + n_split - 1) / n_split;
    const size_t lds = (size_t)SK_NST * (SK_XT + h.max_r16 * SK_BK * 2);
    {
        hipError_t e = allow_full_lds(reinterpret_cast<const void *>(k_skinny<false>), 0);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(k_skinny<false>, dim3((unsigned)h.n_blocks, (unsigned)n_split), dim3(64 * SK_NW), lds, st, mv, mode,
                       static_cast<const uint16_t *>(S), (int)C, static_cast<const uint16_t *>(at),
                       static_cast<const uint16_t *>(zero), part, per, NoGroup{0});
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_skinny_finish<false>, dim3((unsigned)h.n_blocks, kSkinnyRows / 16), dim3(256), 0, st, mv, mode, part, n_split, hf,
                       static_cast<uint16_t *>(hb), static_cast<uint16_t *>(zt), zt_scaled ? 1 : 0, NoGroup{0}, 0);
    return hipGetLastError();
}

hipError_t launch_skinny_group(const GroupView &gv, const MetaHeader &hv, const void *x, int64_t C, const void *zero, float *part,
                               float *const *hf, void *const *hb, void *const *zt, hipStream_t st)
{
    if (hv.n_blocks == 0) return hipSuccess;
    if (gv.n_proj < 2 || gv.n_proj > kMaxGroup || gv.max_r16 > PLORA_MAX_RANK || hv.max_r16 != gv.max_r16) return hipErrorInvalidValue;
    const int n_split = skinny_splits(hv, C);
    const int n_stage_all = (int)((C + SK_BK - 1) / SK_BK);
    const int per = (n_stage_all + n_split - 1) / n_split;
    const size_t lds = (size_t)SK_NST * (SK_XT + gv.max_r16 * SK_BK * 2);
    {
        hipError_t e = allow_full_lds(reinterpret_cast<const void *>(k_skinny<true>), 7);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(k_skinny<true>, dim3((unsigned)hv.n_blocks, (unsigned)n_split), dim3(64 * SK_NW), lds, st, gv.mv[0], 0,
                       static_cast<const uint16_t *>(x), (int)C, static_cast<const uint16_t *>(nullptr),
                       static_cast<const uint16_t *>(zero), part, per, gv);
    hipError_t e = hipGetLastError();
    for (int p = 0; p < gv.n_proj && e == hipSuccess; ++p) {
        hipLaunchKernelGGL(k_skinny_finish<true>, dim3((unsigned)hv.n_blocks, kSkinnyRows / 16), dim3(256), 0, st, gv.mv[p], 0, part,
                           n_split, hf[p], static_cast<uint16_t *>(hb[p]), static_cast<uint16_t *>(zt[p]), 0, gv, p);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace plora
