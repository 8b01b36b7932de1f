// Base GEMM of the packed multi-LoRA layer on bf16 inputs with the low-rank term fused in as extra
// steps of the contraction loop (gfx950, MFMA 32x32x16 bf16, fp32 accumulators).
//
//   forward   y  = [x  | scale*h] . [W ; B_k]          (section 2.4:  x W + scale_k (x A_k) B_k)
//   backward  dx = [dy | g      ] . [W^T ; A_k^T]      (appendix C.2, case 4; g = scale_k dy B_k^T)
//
// The low-rank factor (h or g, bf16, rank padded to a multiple of 64) is produced by the skinny
// kernel beforehand; here it only lengthens the K loop of the tiles whose rows belong to adapter k,
// so the base output never makes an extra trip through HBM.  Row tiles are uniform over the whole
// batch; a tile that straddles segments runs the extension of each segment it touches with the
// rows of the other segments pointed at a page of zeros.
//
// Tile: 256 x 256 outputs per workgroup, BK-deep K steps, 8 waves (2 along rows x 4 along
// columns, 128 x 64 outputs each).  Operands go HBM -> LDS directly (global_load_lds, 16 bytes per
// lane) into NST stages; the 16-byte chunks of a row are XOR-swizzled on the way in (by choosing
// which chunk each lane fetches) so that MFMA operand reads are free of bank conflicts.
// W is [d_in][d_out] row-major in both directions: backward contracts over its contiguous index
// and reads operands with ds_read_b128; forward contracts over its row index and reads operands
// with the transposing LDS load (ds_read_b64_tr_b16), so no transposed copy of W is ever made.
#include "plora_internal.h"

#include <cstdlib>
#include <type_traits>

namespace plora {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T *)(p))
#define GLB_PTR(p) ((const __attribute__((address_space(1))) void *)(p))

constexpr int BM = 256, BN = 256;

__device__ inline uint32_t pack_bf16x2(float lo, float hi)
{
    uint32_t a = __float_as_uint(lo), b = __float_as_uint(hi);
    a += 0x7FFFu + ((a >> 16) & 1u);
    b += 0x7FFFu + ((b >> 16) & 1u);
    return (a >> 16) | (b & 0xFFFF0000u);
}

// Next segment at or after `from` that overlaps rows [m0, m1), has an adapter and at least one row.
__device__ inline int next_ext_seg(const MetaView &mv, int from, int m0, int m1)
{
    const int n = mv.hdr->n_seg;
    for (int s = from; s < n; ++s) {
        const int r0 = mv.seg[s].row0, r1 = mv.seg[s].row1;
        if (r0 >= m1) return n;
        if (mv.seg[s].adapter >= 0 && r1 > r0 && r1 > m0) return s;
    }
    return n;
}

template <int N> __device__ inline void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit field");
    // gfx9 encoding: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt_hi[15:14]; other counters left at max
    __builtin_amdgcn_s_waitcnt(0x0f70 | (N & 15) | ((N >> 4) << 14));
}

// DBG is for timing experiments only: 1 = no barriers and no loads after the first stage,
// 2 = no LDS reads and no MFMAs.  0 is the product.
template <bool FWD, int BK, int NST, int DBG>
__global__ void __launch_bounds__(512) k_gemm(MetaView mv, const uint16_t *__restrict__ S,
                                              const uint16_t *__restrict__ W, const uint16_t *__restrict__ side,
                                              const uint16_t *__restrict__ ap, const uint16_t *__restrict__ zero,
                                              uint16_t *__restrict__ Cout, int tiles_m, int tiles_n)
{
    constexpr int CPR = BK / 8;                  // 16-byte chunks per S-side row
    constexpr int RPI = 64 / CPR;                // S-side rows per 1 KB load instruction
    constexpr int RP256 = 256 / (BK * 2);        // S-side rows per 256 bytes of LDS
    constexpr int NL = BM / RPI / 8;             // load instructions per wave per stage, each side
    constexpr int LPS = 2 * NL;                  // loads per wave per stage
    constexpr int kATile = BM * BK * 2;
    constexpr int kStage = (BM + BN) * BK * 2;
    constexpr int KS = BK / 16;                  // MFMA K steps per stage
    static_assert(kRankPadGemm % BK == 0, "extension steps must be whole stages");
    static_assert(NL == KS, "one S-side and one W-side load are issued after each MFMA step");
    static_assert(!FWD || BK / 2 / 8 == NL, "forward W-side tile: two k rows per load instruction");

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

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform: LDS bases stay scalar

    // ---- loader.  S-side tile [256 rows][8 chunks]: instruction q covers rows 8q..8q+7; lane ->
    // (row 8q + lane/8, slot lane%8); slot c' of row u holds chunk c' ^ ((u >> 1) & 7).
    // Wave w issues instructions w, w+8, w+16, w+24.
    const int a_row = wave * RPI + lane / CPR;                        // + 8*RPI*jj
    const int a_chunk = (lane % CPR) ^ ((a_row / RP256) % CPR);       // 8*RPI*jj / RP256 is a multiple of CPR
    // backward W-side tile [256 n][8 chunks]: same scheme.  forward W-side tile [BK k][32 chunks]:
    // instruction q covers k rows 2q, 2q+1; lane -> (k row 2q + lane/32, slot lane%32); slot c' of
    // k row u holds chunk c' ^ (4 * (u & 3)).
    const int b_row = FWD ? wave * 2 + (lane >> 5) : a_row;          // + 16*jj (FWD) / + 8*RPI*jj
    const int b_chunk = FWD ? ((lane & 31) ^ (4 * (b_row & 3))) : a_chunk;

    // running global pointers of the main K loop (rows past the end are clamped: they only feed
    // outputs that are never stored)
    const uint16_t *pa[NL], *pb[NL];
#pragma unroll
    for (int jj = 0; jj < NL; ++jj) {
        int row = m0 + a_row + 8 * RPI * jj;
        row = row < M ? row : M - 1;
        pa[jj] = S + (int64_t)row * Kd + a_chunk * 8;
        if (FWD) {
            int n = n0 + b_chunk * 8;
            n = n < N ? n : N - 8;
            pb[jj] = W + (int64_t)(b_row + 16 * jj) * ldw + n;
        } else {
            int n = n0 + b_row + 8 * RPI * jj;
            n = n < N ? n : N - 1;
            pb[jj] = W + (int64_t)n * ldw + b_chunk * 8;
        }
    }
    const int64_t pb_step = FWD ? (int64_t)BK * ldw : BK;

    const int nk_main = (Kd + BK - 1) / BK;
    int ext_seg = next_ext_seg(mv, 0, m0, m1), ext_kk = 0;
    int n_ext = 0;
    for (int s = ext_seg; s < n_seg; s = next_ext_seg(mv, s + 1, m0, m1))
        n_ext += mv.seg[s].rp / BK;
    const int n_it = nk_main + n_ext;

    // Per-lane source addresses of the 4 + 4 loads of stage `it`, in stage order (called once per
    // stage, with it = 0, 1, 2, ...).  Full main steps just hand out the running pointers; the last,
    // partial K step masks chunks past the end of the contraction with a page of zeros; the
    // low-rank extension steps of segment ext_seg read the bf16 low-rank factor of the rows that
    // belong to that segment (zeros for the other rows of the tile) and B_k or the padded A_k.
    const uint16_t *na[NL], *nb[NL];
    auto prepare = [&](int it) {
        if (it < nk_main) {
            const int k0 = it * BK;
            if (k0 + BK <= Kd) {
#pragma unroll
                for (int jj = 0; jj < NL; ++jj) { na[jj] = pa[jj]; nb[jj] = pb[jj]; }
            } else {
#pragma unroll
                for (int jj = 0; jj < NL; ++jj) {
                    na[jj] = (k0 + a_chunk * 8 < Kd) ? pa[jj] : zero;
                    const bool ok = FWD ? (k0 + b_row + 16 * jj < Kd) : (k0 + b_chunk * 8 < Kd);
                    nb[jj] = ok ? pb[jj] : zero;
                }
            }
#pragma unroll
            for (int jj = 0; jj < NL; ++jj) { pa[jj] += BK; pb[jj] += pb_step; }
        } else {
            const int sidx = __builtin_amdgcn_readfirstlane(ext_seg);
            const int kk = __builtin_amdgcn_readfirstlane(ext_kk);
            const SegInfo g = mv.seg[sidx];
            const AdapterInfo a = mv.ad[g.adapter];
#pragma unroll
            for (int jj = 0; jj < NL; ++jj) {
                const int row = m0 + a_row + 8 * RPI * jj;
                const bool in = row >= g.row0 && row < g.row1;
                na[jj] = in ? side + g.hb_off + (int64_t)(row - g.row0) * g.rp + kk + a_chunk * 8 : zero;
                if (FWD) {
                    const int j = kk + b_row + 16 * jj;                // row of B_k
                    int n = n0 + b_chunk * 8;
                    n = n < N ? n : N - 8;
                    nb[jj] = (j < g.r) ? static_cast<const uint16_t *>(a.B) + (int64_t)j * ldw + n : zero;
                } else {
                    int n = n0 + b_row + 8 * RPI * jj;                 // row of padded A_k
                    n = n < N ? n : N - 1;
                    nb[jj] = ap + a.ap_off + (int64_t)n * g.rp + kk + b_chunk * 8;
                }
            }
            ext_kk = kk + BK;
            if (ext_kk >= g.rp) { ext_seg = next_ext_seg(mv, sidx + 1, m0, m1); ext_kk = 0; }
        }
    };
    // The direct-to-LDS loads are issued through inline assembly: the compiler, which cannot tell
    // the stage being filled from the stage being read, would otherwise make every LDS read wait
    // for all of them (vmcnt(0)) and serialise the pipeline.  Ordering is explicit instead: a
    // counted s_waitcnt plus a barrier before a stage is read (wait_stage below).  M0 holds the
    // wave-uniform LDS destination; lane i lands at M0 + 16 i.
    const uint32_t lds_base = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)LDS_PTR(char, lds));
    auto load_lds16 = [&](const uint16_t *g, uint32_t dst) {
        asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(dst));
    };
    auto load_pair = [&](int stage, int jj) {
        const uint32_t sa = lds_base + stage * kStage + (wave + 8 * jj) * 1024;
        load_lds16(na[jj], sa);
        load_lds16(nb[jj], sa + kATile);
    };

    // ---- MFMA operand addressing.  Wave (wm, wn) owns rows wm*128.. and columns wn*64..
    const int wm0 = (wave >> 2) * 128, wn0 = (wave & 3) * 64;
    const int l32 = lane & 31, kg = lane >> 5;
    // S-side operand (4 blocks of 32 rows): row u = wm0 + mi*32 + l32, chunk = ks*2 + kg
    int xoff[4];
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) {
        const int u = wm0 + mi * 32 + l32;
        xoff[mi] = u * (BK * 2) + ((kg ^ ((u / RP256) % CPR)) * 16);     // ks*2 XORs in separately (bit 1 and up)
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
            const int u = wn0 + ni * 32 + l32;
            woff[ni] = u * (BK * 2) + ((kg ^ ((u / RP256) % CPR)) * 16);
        }
    }

    f32x16 acc[2][4];
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
        for (int mi = 0; mi < 4; ++mi)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[ni][mi][i] = 0.f;

    // One stage of MFMA work; with LOADS the 4 + 4 loads of the next stage (addresses in na / nb) are
    // issued one pair after each MFMA step, which keeps the memory pipe evenly fed and the waves out
    // of each other's way.
    auto compute = [&](int stage, int load_stage, auto with_loads) {
        const char *sa = lds + stage * kStage;
        const char *sb = sa + kATile;
        bf16x8 xf[2][4], wf[2][2];
        auto read_frags = [&](int ks, bf16x8 (&x)[4], bf16x8 (&w)[2]) {
#pragma unroll
            for (int mi = 0; mi < 4; ++mi)
                x[mi] = *LDS_PTR(const bf16x8, sa + (xoff[mi] ^ (ks * 32)));
#pragma unroll
            for (int ni = 0; ni < 2; ++ni) {
                if (FWD) {
                    // k rows advance by 16 per ks (16*512 bytes): bits above the swizzle, plain add
                    const char *p = sb + woff[ni] + ks * 16 * 512;
                    bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(LDS_PTR(bf16x4, p));
                    bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(LDS_PTR(bf16x4, p + 4 * 512));
                    w[ni] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                } else {
                    w[ni] = *LDS_PTR(const bf16x8, sb + (woff[ni] ^ (ks * 32)));
                }
            }
        };
        if (DBG != 2) read_frags(0, xf[0], wf[0]);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            if (DBG != 2) {
                // operands of the next MFMA step are fetched before the MFMAs of this one are issued
                if (ks + 1 < KS && DBG != 3) read_frags(ks + 1, xf[(ks + 1) & 1], wf[(ks + 1) & 1]);
#pragma unroll
                for (int ni = 0; ni < 2; ++ni)
#pragma unroll
                    for (int mi = 0; mi < 4; ++mi)
                        acc[ni][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[DBG == 3 ? 0 : (ks & 1)][ni], xf[DBG == 3 ? 0 : (ks & 1)][mi], acc[ni][mi], 0, 0, 0);
            }
            if constexpr (decltype(with_loads)::value) {
                if (DBG == 5) {          // experiment: all loads in the first half of the stage
                    if (ks * 2 < KS) { load_pair(load_stage, 2 * ks); load_pair(load_stage, 2 * ks + 1); }
                } else {
                    load_pair(load_stage, ks);
                }
            }
            // issue order inside this step: the LDS reads of the next step go out one by one behind
            // the first MFMAs
            if (DBG != 2 && DBG != 3 && DBG != 4) {
                constexpr int n_ds = FWD ? 8 : 6;
                if (ks + 1 < KS) {
#pragma unroll
                    for (int i = 0; i < n_ds; ++i) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // 1 MFMA
                        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // 1 LDS read
                    }
                    if (n_ds < 8) __builtin_amdgcn_sched_group_barrier(0x008, 8 - n_ds, 0);
                } else {
                    __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
                }
            }
        }
    };

    // NST-1 stages up front; then every pass over a stage issues the loads of the stage NST-1 ahead
    // of it (into the buffer that the previous pass has just finished reading).
    auto wait_stage = [&](int ahead) {        // loads of `ahead` later stages may stay in flight
        if (NST >= 5 && ahead >= 3) wait_vmcnt<3 * LPS>();
        else if (NST >= 4 && ahead >= 2) wait_vmcnt<2 * LPS>();
        else if (NST >= 3 && ahead >= 1) wait_vmcnt<LPS>();
        else wait_vmcnt<0>();
    };
#pragma unroll
    for (int p = 0; p < NST - 1; ++p) {
        if (p < n_it) {
            prepare(p);
#pragma unroll
            for (int jj = 0; jj < NL; ++jj) load_pair(p, jj);
        }
    }
    int it = 0;
    if (NST - 1 < n_it) prepare(NST - 1);
    for (; it + NST - 1 < n_it; ++it) {
        wait_stage(NST - 2);                  // this wave's part of stage `it` has landed ...
        if (DBG == 0 || DBG == 2 || DBG == 5) __builtin_amdgcn_s_barrier();   // ... and so has everyone else's; the buffer read last pass is free (a bare barrier: __syncthreads would drain every load in flight)
        if (DBG == 0 || DBG == 2 || DBG == 5) compute(it % NST, (it + NST - 1) % NST, std::true_type{});
        else compute(it % NST, 0, std::false_type{});
        if (it + NST < n_it) prepare(it + NST);
    }
    for (; it < n_it; ++it) {
        wait_stage(n_it - 1 - it);
        if (DBG == 0 || DBG == 2 || DBG == 5) __builtin_amdgcn_s_barrier();
        compute(it % NST, 0, std::false_type{});
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

template <bool FWD, int BK, int NST, int DBG>
static hipError_t launch_variant(const MetaView &mv, const MetaHeader &h, const void *S, const void *W,
                                 const void *side, const void *ap, const void *zero, void *C, hipStream_t st)
{
    constexpr int lds = NST * (BM + BN) * BK * 2;
    const int64_t N = FWD ? h.K : h.D;
    const int tiles_m = (int)((h.T + BM - 1) / BM), tiles_n = (int)((N + BN - 1) / BN);
    auto kern = k_gemm<FWD, BK, NST, DBG>;
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)(tiles_m * tiles_n)), dim3(512), lds, st, mv,
                       static_cast<const uint16_t *>(S), static_cast<const uint16_t *>(W),
                       static_cast<const uint16_t *>(side), static_cast<const uint16_t *>(ap),
                       static_cast<const uint16_t *>(zero), static_cast<uint16_t *>(C), tiles_m, tiles_n);
    return hipGetLastError();
}

hipError_t launch_gemm_bf16(const MetaView &mv, const MetaHeader &h, bool forward, const void *S, const void *W,
                            const void *side, const void *ap, const void *zero, void *C, hipStream_t st)
{
    if (h.T == 0) return hipSuccess;
    static int variant = -1;
    if (variant < 0) {
        const char *e = std::getenv("PLORA_GEMM_VARIANT");
        variant = e ? std::atoi(e) : 15;
    }
#define PLORA_V(FWD_) \
    if (variant == 1) return launch_variant<FWD_, 32, 4, 0>(mv, h, S, W, side, ap, zero, C, st); \
    if (variant == 2) return launch_variant<FWD_, 32, 5, 0>(mv, h, S, W, side, ap, zero, C, st); \
    if (variant == 3) return launch_variant<FWD_, 32, 3, 0>(mv, h, S, W, side, ap, zero, C, st); \
    if (variant == 11) return launch_variant<FWD_, 64, 2, 1>(mv, h, S, W, side, ap, zero, C, st); \
    if (variant == 12) return launch_variant<FWD_, 64, 2, 2>(mv, h, S, W, side, ap, zero, C, st); \
    if (variant == 13) return launch_variant<FWD_, 64, 2, 3>(mv, h, S, W, side, ap, zero, C, st); \
    if (variant == 14) return launch_variant<FWD_, 64, 2, 4>(mv, h, S, W, side, ap, zero, C, st); \
    if (variant == 15) return launch_variant<FWD_, 64, 2, 5>(mv, h, S, W, side, ap, zero, C, st); \
    if (variant == 21) return launch_variant<FWD_, 32, 4, 1>(mv, h, S, W, side, ap, zero, C, st); \
    if (variant == 22) return launch_variant<FWD_, 32, 4, 2>(mv, h, S, W, side, ap, zero, C, st); \
    return launch_variant<FWD_, 64, 2, 0>(mv, h, S, W, side, ap, zero, C, st);
    if (forward) { PLORA_V(true) }
    PLORA_V(false)
#undef PLORA_V
}

}  // namespace plora
