// Base GEMM of the packed multi-LoRA layer on bf16 inputs with the low-rank term fused in as extra
// steps of the contraction loop (gfx950, MFMA 32x32x16 bf16, fp32 accumulators).
//
//   forward   y  = [x  | scale*h] . [W ; B_k]          (section 2.4:  x W + scale_k (x A_k) B_k)
//   backward  dx = [dy | g      ] . [W^T ; A_k^T]      (appendix C.2, case 4; g = scale_k dy B_k^T)
//
// The low-rank factor (h or g, bf16, rank padded to one 64-wide step) is produced by the skinny
// kernel beforehand; here it only lengthens the K loop of the tiles whose rows belong to adapter k,
// so the base output never makes an extra trip through HBM.  Row tiles are uniform over the whole
// batch; a tile that straddles segments runs the extension of each segment it touches with the
// rows of the other segments pointed at a page of zeros.
//
// Tile: 256 x 256 outputs per workgroup, 64-deep K steps, 8 waves (2 along rows x 4 along
// columns, 128 x 64 outputs each).  Operands go HBM -> LDS directly (global_load_lds, 16 bytes per
// lane) into two stages of 64 KB; the 16-byte chunks of a row are XOR-swizzled on the way in (by
// choosing which chunk each lane fetches) so that MFMA operand reads are free of bank conflicts.
// W is [d_in][d_out] row-major in both directions: backward contracts over its contiguous index
// and reads operands with ds_read_b128; forward contracts over its row index and reads operands
// with the transposing LDS load (ds_read_b64_tr_b16), so no transposed copy of W is ever made.
#include "plora_internal.h"

namespace plora {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short i16x4;
typedef __attribute__((__vector_size__(8 * sizeof(short)))) short i16x8;

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T *)(p))
#define GLB_PTR(p) ((const __attribute__((address_space(1))) void *)(p))

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int kStageBytes = (BM + BN) * BK * 2;   // 64 KB
constexpr int kATileBytes = BM * BK * 2;          // 32 KB
constexpr int kGemmLds = 2 * kStageBytes;         // 128 KB

__device__ inline uint32_t pack_bf16x2(float lo, float hi)
{
    uint32_t a = __float_as_uint(lo), b = __float_as_uint(hi);
    a += 0x7FFFu + ((a >> 16) & 1u);
    b += 0x7FFFu + ((b >> 16) & 1u);
    return (a >> 16) | (b & 0xFFFF0000u);
}

// Cursor over the low-rank extension steps of one row tile: the segments that overlap the tile,
// have an adapter and at least one row, each contributing rp/64 steps.
struct ExtCursor {
    int seg;     // current segment index (n_seg when exhausted)
    int kk;      // offset inside the padded rank of that segment
};

__device__ inline int next_ext_seg(const MetaView &mv, int from, int m0, int m1)
{
    const int n = mv.hdr->n_seg;
    int s = from;
    for (; s < n; ++s) {
        const int r0 = mv.seg[s].row0, r1 = mv.seg[s].row1;
        if (r0 >= m1) return n;
        if (mv.seg[s].adapter >= 0 && r1 > r0 && r1 > m0) return s;
    }
    return n;
}

template <bool FWD>
__global__ void __launch_bounds__(512) k_gemm(MetaView mv, const uint16_t *__restrict__ S,
                                              const uint16_t *__restrict__ W, const uint16_t *__restrict__ side,
                                              const uint16_t *__restrict__ ap, const uint16_t *__restrict__ zero,
                                              uint16_t *__restrict__ Cout, int tiles_m, int tiles_n)
{
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    const int M = (int)mv.hdr->T;
    const int Kd = (int)(FWD ? mv.hdr->D : mv.hdr->K);
    const int N = (int)(FWD ? mv.hdr->K : mv.hdr->D);
    const int ldw = (int)mv.hdr->K;
    const int n_seg = mv.hdr->n_seg;

    // ---- workgroup -> tile.  Workgroups are dealt round-robin to the 8 XCDs (each with its own L2);
    // give every XCD a contiguous range of tile ids, and walk tile ids in groups of 4 row tiles so
    // that the tiles resident on one XCD at a time share rows of S and columns of W.
    int tile = blockIdx.x;
    {
        const int nt = tiles_m * tiles_n, per = nt / 8;
        if (tile < per * 8) tile = (tile % 8) * per + tile / 8;
    }
    constexpr int GM = 4;
    int tm, tn;
    {
        const int group = tile / (GM * tiles_n), first = group * GM;
        const int gsz = (tiles_m - first < GM) ? tiles_m - first : GM;
        const int in = tile - group * GM * tiles_n;
        tm = first + in % gsz;
        tn = in / gsz;
    }
    const int m0 = tm * BM, n0 = tn * BN;
    const int m1 = (m0 + BM < M) ? m0 + BM : M;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

    // ---- loader state.  Each wave issues 4 + 4 direct-to-LDS loads of 1 KB per stage.
    // S-side tile [256 rows][8 chunks]: instruction j covers rows 8j..8j+7; lane -> (row j*8 + lane/8,
    // slot lane%8); slot c' of row q holds chunk c' ^ ((q >> 1) & 7).
    const int a_row = wave * 8 + (lane >> 3);                       // + 64*jj
    const int a_chunk = (lane & 7) ^ ((a_row >> 1) & 7);            // same for every jj (64*jj keeps bits 1..3)
    // backward W-side tile [256 n][8 chunks]: same scheme.  forward W-side tile [64 k][32 chunks]:
    // instruction j covers k rows 2j, 2j+1; lane -> (k row 2j + lane/32, slot lane%32); slot c' of
    // k row q holds chunk c' ^ (4 * (q & 3)).
    const int b_row = FWD ? wave * 2 + (lane >> 5) : a_row;        // + 16*jj (FWD) / + 64*jj
    const int b_chunk = FWD ? ((lane & 31) ^ (4 * (b_row & 3))) : a_chunk;

    const int nk_main = (Kd + BK - 1) / BK;
    ExtCursor cur;
    cur.seg = next_ext_seg(mv, 0, m0, m1);
    cur.kk = 0;

    auto issue = [&](int it, int stage) {
        char *sa = lds + stage * kStageBytes;
        char *sb = sa + kATileBytes;
        if (it < nk_main) {
            const int k0 = it * BK;
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                int row = m0 + a_row + 64 * jj;
                row = row < M ? row : M - 1;                         // rows past the end only feed outputs that are not stored
                const int kc = k0 + a_chunk * 8;
                const uint16_t *g = (kc < Kd) ? S + (int64_t)row * Kd + kc : zero;
                __builtin_amdgcn_global_load_lds(GLB_PTR(g), LDS_PTR(void, sa + (wave + 8 * jj) * 1024), 16, 0, 0);
            }
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                const uint16_t *g;
                if (FWD) {
                    const int k = k0 + b_row + 16 * jj;
                    int n = n0 + b_chunk * 8;
                    n = n < N ? n : N - 8;
                    g = (k < Kd) ? W + (int64_t)k * ldw + n : zero;
                } else {
                    int n = n0 + b_row + 64 * jj;
                    n = n < N ? n : N - 1;
                    const int kc = k0 + b_chunk * 8;
                    g = (kc < Kd) ? W + (int64_t)n * ldw + kc : zero;
                }
                __builtin_amdgcn_global_load_lds(GLB_PTR(g), LDS_PTR(void, sb + (wave + 8 * jj) * 1024), 16, 0, 0);
            }
        } else {
            // low-rank extension step of segment cur.seg at rank offset cur.kk
            const SegInfo g = mv.seg[cur.seg];
            const AdapterInfo a = mv.ad[g.adapter];
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                const int row = m0 + a_row + 64 * jj;
                const bool in = row >= g.row0 && row < g.row1;
                const uint16_t *p = in ? side + g.hb_off + (int64_t)(row - g.row0) * g.rp + cur.kk + a_chunk * 8 : zero;
                __builtin_amdgcn_global_load_lds(GLB_PTR(p), LDS_PTR(void, sa + (wave + 8 * jj) * 1024), 16, 0, 0);
            }
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                const uint16_t *p;
                if (FWD) {
                    const int j = cur.kk + b_row + 16 * jj;            // row of B_k
                    int n = n0 + b_chunk * 8;
                    n = n < N ? n : N - 8;
                    p = (j < g.r) ? static_cast<const uint16_t *>(a.B) + (int64_t)j * ldw + n : zero;
                } else {
                    int n = n0 + b_row + 64 * jj;                      // row of padded A_k
                    n = n < N ? n : N - 1;
                    p = ap + a.ap_off + (int64_t)n * g.rp + cur.kk + b_chunk * 8;
                }
                __builtin_amdgcn_global_load_lds(GLB_PTR(p), LDS_PTR(void, sb + (wave + 8 * jj) * 1024), 16, 0, 0);
            }
            cur.kk += BK;
            if (cur.kk >= g.rp) { cur.seg = next_ext_seg(mv, cur.seg + 1, m0, m1); cur.kk = 0; }
        }
    };

    // number of extension steps of this row tile
    int n_ext = 0;
    for (int s = next_ext_seg(mv, 0, m0, m1); s < n_seg; s = next_ext_seg(mv, s + 1, m0, m1))
        n_ext += mv.seg[s].rp / BK;
    const int n_it = nk_main + n_ext;

    // ---- MFMA operand addressing.  Wave (wm, wn) owns rows wm*128.. and columns wn*64..
    const int wm0 = (wave >> 2) * 128, wn0 = (wave & 3) * 64;
    const int l32 = lane & 31, kg = lane >> 5;
    // S-side operand (4 blocks of 32 rows): row q = wm0 + mi*32 + l32, chunk = ks*2 + kg
    int xoff[4];
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) {
        const int q = wm0 + mi * 32 + l32;
        xoff[mi] = q * 128 + ((kg ^ ((q >> 1) & 7)) * 16);           // chunk ks*2 XORs in separately (bits 1,2)
    }
    // W-side operand (2 blocks of 32 columns)
    int woff[2];
    const int i16 = lane & 15, g4 = lane >> 4;
#pragma unroll
    for (int ni = 0; ni < 2; ++ni) {
        if (FWD) {
            // transposing read: the 16 lanes of a group fetch a 4(k) x 16(n) block, 8 bytes each
            const int nl = wn0 + ni * 32 + (g4 & 1) * 16 + (i16 & 3) * 4;   // first column this lane fetches
            const int kr = (g4 >> 1) * 8 + (i16 >> 2);                      // + ks*16, + 4 for the second read
            woff[ni] = kr * 512 + ((((nl >> 3) ^ (4 * (kr & 3))) * 16) + (nl & 7) * 2);
        } else {
            const int q = wn0 + ni * 32 + l32;
            woff[ni] = q * 128 + ((kg ^ ((q >> 1) & 7)) * 16);
        }
    }

    f32x16 acc[2][4];
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
        for (int mi = 0; mi < 4; ++mi)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[ni][mi][i] = 0.f;

    issue(0, 0);
    for (int it = 0; it < n_it; ++it) {
        const int stage = it & 1;
        __builtin_amdgcn_s_waitcnt(0x0f70);   // vmcnt(0) (keeps lgkmcnt/expcnt fields at "don't wait")
        __syncthreads();
        if (it + 1 < n_it) issue(it + 1, stage ^ 1);
        const char *sa = lds + stage * kStageBytes;
        const char *sb = sa + kATileBytes;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            bf16x8 xf[4], wf[2];
#pragma unroll
            for (int mi = 0; mi < 4; ++mi)
                xf[mi] = *LDS_PTR(const bf16x8, sa + (xoff[mi] ^ (ks * 32)));
#pragma unroll
            for (int ni = 0; ni < 2; ++ni) {
                if (FWD) {
                    // k rows advance by 16 per ks (16*512 bytes): bits above the swizzle, plain add
                    const char *p = sb + woff[ni] + ks * 16 * 512;
                    bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(LDS_PTR(bf16x4, p));
                    bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(LDS_PTR(bf16x4, p + 4 * 512));
                    wf[ni] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                } else {
                    wf[ni] = *LDS_PTR(const bf16x8, sb + (woff[ni] ^ (ks * 32)));
                }
            }
#pragma unroll
            for (int ni = 0; ni < 2; ++ni)
#pragma unroll
                for (int mi = 0; mi < 4; ++mi)
                    acc[ni][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[ni], xf[mi], acc[ni][mi], 0, 0, 0);
        }
    }

    // ---- epilogue: MFMA rows are output columns n, MFMA columns are output rows m.
    // Lane holds, for each group i4 of 4 registers, 4 consecutive n of one m: one 8-byte store.
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) {
        const int m = m0 + wm0 + mi * 32 + l32;
        if (m >= M) continue;
        uint16_t *crow = Cout + (int64_t)m * N;
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                const int n = n0 + wn0 + ni * 32 + i4 * 8 + kg * 4;
                if (n < N) {
                    uint2 v;
                    v.x = pack_bf16x2(acc[ni][mi][i4 * 4 + 0], acc[ni][mi][i4 * 4 + 1]);
                    v.y = pack_bf16x2(acc[ni][mi][i4 * 4 + 2], acc[ni][mi][i4 * 4 + 3]);
                    *reinterpret_cast<uint2 *>(crow + n) = v;
                }
            }
    }
}

hipError_t launch_gemm_bf16(const MetaView &mv, const MetaHeader &h, bool forward, const void *S, const void *W,
                            const void *side, const void *ap, const void *zero, void *C, hipStream_t st)
{
    if (h.T == 0) return hipSuccess;
    const int64_t N = forward ? h.K : h.D;
    const int tiles_m = (int)((h.T + BM - 1) / BM), tiles_n = (int)((N + BN - 1) / BN);
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_gemm<true>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kGemmLds);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_gemm<false>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kGemmLds);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    const dim3 grid((unsigned)(tiles_m * tiles_n));
    const uint16_t *s16 = static_cast<const uint16_t *>(S), *w16 = static_cast<const uint16_t *>(W);
    const uint16_t *sd = static_cast<const uint16_t *>(side), *ap16 = static_cast<const uint16_t *>(ap);
    const uint16_t *z16 = static_cast<const uint16_t *>(zero);
    if (forward)
        hipLaunchKernelGGL(k_gemm<true>, grid, dim3(512), kGemmLds, st, mv, s16, w16, sd, ap16, z16,
                           static_cast<uint16_t *>(C), tiles_m, tiles_n);
    else
        hipLaunchKernelGGL(k_gemm<false>, grid, dim3(512), kGemmLds, st, mv, s16, w16, sd, ap16, z16,
                           static_cast<uint16_t *>(C), tiles_m, tiles_n);
    return hipGetLastError();
}

}  // namespace plora
