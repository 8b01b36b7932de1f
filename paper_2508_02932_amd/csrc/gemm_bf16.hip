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
// Tile: 256 x 256 outputs per workgroup, 64-deep K steps, 8 waves (2 along rows x 4 along
// columns, 128 x 64 outputs each).  Operands go HBM -> LDS directly (global_load_lds, 16 bytes per
// lane) into two stages of 64 KB; the 16-byte chunks of a row are XOR-swizzled on the way in (by choosing
// which chunk each lane fetches) so that MFMA operand reads are free of bank conflicts.
// W is [d_in][d_out] row-major in both directions: backward contracts over its contiguous index
// and reads operands with ds_read_b128; forward contracts over its row index and reads operands
// with the transposing LDS load (ds_read_b64_tr_b16), so no transposed copy of W is ever made.
#include "plora_internal.h"


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

constexpr int BK = 64;                       // contraction elements per stage
constexpr int CPR = BK / 8;                  // 16-byte chunks per S-side row
constexpr int RPI = 64 / CPR;                // S-side rows per 1 KB load instruction
constexpr int kATile = BM * BK * 2;          // 32 KB
constexpr int kStage = (BM + BN) * BK * 2;   // 64 KB
constexpr int kGemmLds = 2 * kStage;         // two stages
constexpr int KS = BK / 16;                  // MFMA K steps per stage (4)
static_assert(kRankPadGemm % BK == 0, "extension steps must be whole stages");
static_assert(KS == 4, "the schedule below is written for four MFMA steps per stage");

constexpr int WN = 2;                        // 32-column blocks per wave: 8 waves of 128 x 64 outputs
constexpr int AFTER = 2;                     // load pairs of the next-but-one stage issued right behind the barrier;
                                             // the rest follow behind the first MFMA step of the next stage
template <bool FWD>
__global__ void __launch_bounds__(512) k_gemm(MetaView mv, const uint16_t *__restrict__ S,
                                              const uint16_t *__restrict__ W, const uint16_t *__restrict__ side,
                                              const uint16_t *__restrict__ ap, const uint16_t *__restrict__ zero,
                                              uint16_t *__restrict__ Cout, int tiles_m, int tiles_n)
{
    constexpr int NW = 2 * (BN / (WN * 32));     // waves per workgroup
    constexpr int NL = BM / RPI / NW;            // load instructions per wave per stage, each side
    static_assert(AFTER <= NL, "");
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
    // Wave w issues instructions w, w+NW, w+2NW, ...
    const int a_row = wave * RPI + lane / CPR;                        // + 8*NW*jj
    const int a_chunk = (lane % CPR) ^ ((a_row >> 1) & 7);            // 8*NW*jj leaves bits 1..3 alone
    // backward W-side tile [256 n][8 chunks]: same scheme.  forward W-side tile [64 k][32 chunks]:
    // instruction q covers k rows 2q, 2q+1; lane -> (k row 2q + lane/32, slot lane%32); slot c' of
    // k row u holds chunk c' ^ (4 * (u & 3)).
    const int b_row = FWD ? wave * 2 + (lane >> 5) : a_row;          // + 2*NW*jj (FWD) / + 8*NW*jj
    const int b_chunk = FWD ? ((lane & 31) ^ (4 * (b_row & 3))) : a_chunk;

    // running global pointers of the main K loop (rows past the end are clamped: they only feed
    // outputs that are never stored)
    const uint16_t *pa[NL], *pb[NL];
#pragma unroll
    for (int jj = 0; jj < NL; ++jj) {
        int row = m0 + a_row + 8 * NW * jj;
        row = row < M ? row : M - 1;
        pa[jj] = S + (int64_t)row * Kd + a_chunk * 8;
        if (FWD) {
            int n = n0 + b_chunk * 8;
            n = n < N ? n : N - 8;
            pb[jj] = W + (int64_t)(b_row + 2 * NW * jj) * ldw + n;
        } else {
            int n = n0 + b_row + 8 * NW * jj;
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
                    const bool ok = FWD ? (k0 + b_row + 2 * NW * jj < Kd) : (k0 + b_chunk * 8 < Kd);
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
                const int row = m0 + a_row + 8 * NW * jj;
                const bool in = row >= g.row0 && row < g.row1;
                na[jj] = in ? side + g.hb_off + (int64_t)(row - g.row0) * g.rp + kk + a_chunk * 8 : zero;
                if (FWD) {
                    const int j = kk + b_row + 2 * NW * jj;            // row of B_k
                    int n = n0 + b_chunk * 8;
                    n = n < N ? n : N - 8;
                    nb[jj] = (j < g.r) ? static_cast<const uint16_t *>(a.B) + (int64_t)j * ldw + n : zero;
                } else {
                    int n = n0 + b_row + 8 * NW * jj;                  // row of padded A_k
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
    // counted s_waitcnt plus a bare barrier before a stage is read (__syncthreads would add a
    // fence that drains every load in flight).  M0 holds the wave-uniform LDS destination; lane i
    // lands at M0 + 16 i.
    const uint32_t lds_base = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)LDS_PTR(char, lds));
    auto load_lds16 = [&](const uint16_t *g, uint32_t dst) {
        asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(dst));
    };
    auto load_pair = [&](int buf, int jj) {
        const uint32_t sa = lds_base + buf * kStage + (wave + NW * jj) * 1024;
        load_lds16(na[jj], sa);
        load_lds16(nb[jj], sa + kATile);
    };

    // ---- MFMA operand addressing.  Wave (wm, wn) owns rows wm*128.. and columns wn*32*WN..
    constexpr int WAVES_N = BN / (WN * 32);
    const int wm0 = (wave / WAVES_N) * 128, wn0 = (wave % WAVES_N) * (WN * 32);
    const int l32 = lane & 31, kg = lane >> 5;
    // S-side operand (4 blocks of 32 rows): row u = wm0 + mi*32 + l32, chunk = ks*2 + kg
    int xoff[4];
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) {
        const int u = wm0 + mi * 32 + l32;
        xoff[mi] = u * (BK * 2) + ((kg ^ ((u >> 1) & 7)) * 16);          // ks*2 XORs in separately (bit 1 and up)
    }
    // W-side operand (WN blocks of 32 columns)
    int woff[WN];
    const int i16 = lane & 15, g4 = lane >> 4;
#pragma unroll
    for (int ni = 0; ni < WN; ++ni) {
        if (FWD) {
            // transposing read: the 16 lanes of a group fetch a 4(k) x 16(n) block, 8 bytes each
            const int nl = wn0 + ni * 32 + (g4 & 1) * 16 + (i16 & 3) * 4;   // first column this lane fetches
            const int kr = (g4 >> 1) * 8 + (i16 >> 2);                      // + ks*16, + 4 for the second read
            woff[ni] = kr * 512 + ((((nl >> 3) ^ (4 * (kr & 3))) * 16) + (nl & 7) * 2);
        } else {
            const int u = wn0 + ni * 32 + l32;
            woff[ni] = u * (BK * 2) + ((kg ^ ((u >> 1) & 7)) * 16);
        }
    }

    f32x16 acc[WN][4];
#pragma unroll
    for (int ni = 0; ni < WN; ++ni)
#pragma unroll
        for (int mi = 0; mi < 4; ++mi)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[ni][mi][i] = 0.f;

    // MFMA operands of one K step (16 deep): 4 S-side + 2 W-side fragments, double-buffered in registers
    bf16x8 xf[2][4], wf[2][WN];
    auto read_frags = [&](int buf, int ks, int f) {
        const char *sa = lds + buf * kStage;
        const char *sb = sa + kATile;
#pragma unroll
        for (int mi = 0; mi < 4; ++mi)
            xf[f][mi] = *LDS_PTR(const bf16x8, sa + (xoff[mi] ^ (ks * 32)));
#pragma unroll
        for (int ni = 0; ni < WN; ++ni) {
            if (FWD) {
                // k rows advance by 16 per ks (16*512 bytes): bits above the swizzle, plain add
                const char *p = sb + woff[ni] + ks * 16 * 512;
                bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(LDS_PTR(bf16x4, p));
                bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(LDS_PTR(bf16x4, p + 4 * 512));
                wf[f][ni] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            } else {
                wf[f][ni] = *LDS_PTR(const bf16x8, sb + (woff[ni] ^ (ks * 32)));
            }
        }
    };
    auto mfma_step = [&](int f) {
#pragma unroll
        for (int ni = 0; ni < WN; ++ni)
#pragma unroll
            for (int mi = 0; mi < 4; ++mi)
                acc[ni][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[f][ni], xf[f][mi], acc[ni][mi], 0, 0, 0);
    };
    // issue order of a step: the LDS reads of the next step go out one by one behind the first MFMAs
    auto interleave_reads = [&]() {
        constexpr int n_ds = 4 + (FWD ? 2 * WN : WN), n_mfma = 4 * WN;
#pragma unroll
        for (int i = 0; i < n_ds; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // 1 MFMA
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // 1 LDS read
        }
        if (n_ds < n_mfma) __builtin_amdgcn_sched_group_barrier(0x008, n_mfma - n_ds, 0);
    };

    // ---- schedule.  Stage p lives in buffer p % 2.  The loads of stage p+2 are issued right after the
    // barrier that ends the reading of stage p (same buffer), so they have a whole stage of MFMA work
    // to land.  That barrier sits before the last MFMA step of stage p: the operands of that step are
    // already in registers, so the first LDS reads of stage p+1 are hidden behind its MFMAs.
    prepare(0);
#pragma unroll
    for (int jj = 0; jj < NL; ++jj) load_pair(0, jj);
    if (n_it > 1) {
        prepare(1);
#pragma unroll
        for (int jj = 0; jj < NL; ++jj) load_pair(1, jj);
        wait_vmcnt<2 * NL>();                 // stage 0 landed (the 2 NL loads of stage 1 may still be in flight)
    } else {
        wait_vmcnt<0>();
    }
    if (n_it > 2) prepare(2);               // pointers of stage p+2 are ready before the barrier of stage p
    __builtin_amdgcn_s_barrier();
    read_frags(0, 0, 0);

    bool pending = false;                     // load pairs AFTER..NL-1 of the stage being fetched still to issue
    for (int p = 0; p + 1 < n_it; ++p) {
        const int buf = p & 1;
        read_frags(buf, 1, 1); mfma_step(0); interleave_reads();
        if (AFTER < NL && pending) {
#pragma unroll
            for (int jj = AFTER; jj < NL; ++jj) load_pair(buf ^ 1, jj);
        }
        read_frags(buf, 2, 0); mfma_step(1); interleave_reads();
        read_frags(buf, 3, 1); mfma_step(0); interleave_reads();
        if (p + 2 < n_it && p > 0) prepare(p + 2);
        // every read of stage p has been issued; make sure this wave's have completed, then wait for
        // stage p+1 (its loads were issued about one stage ago) and for everybody else
        wait_vmcnt<0>();
        __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0), other counters untouched
        __builtin_amdgcn_s_barrier();
        read_frags(buf ^ 1, 0, 0);
        pending = p + 2 < n_it;
        if (pending) {                        // refill the buffer that has just been released
#pragma unroll
            for (int jj = 0; jj < AFTER; ++jj) load_pair(buf, jj);
        }
        mfma_step(1);
    }
    {
        const int buf = (n_it - 1) & 1;
        read_frags(buf, 1, 1); mfma_step(0); interleave_reads();
        read_frags(buf, 2, 0); mfma_step(1); interleave_reads();
        read_frags(buf, 3, 1); mfma_step(0); interleave_reads();
        mfma_step(1);
    }
    wait_vmcnt<0>();                          // no direct-to-LDS load may outlive the workgroup

    // ---- epilogue: MFMA rows are output columns n, MFMA columns are output rows m.
    // Lane holds, for each group i4 of 4 registers, 4 consecutive n of one m: one 8-byte store.
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) {
        const int m = m0 + wm0 + mi * 32 + l32;
        if (m >= M) continue;
        uint16_t *crow = Cout + (int64_t)m * N;
#pragma unroll
        for (int ni = 0; ni < WN; ++ni)
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

template <bool FWD>
static hipError_t launch_variant(const MetaView &mv, const MetaHeader &h, const void *S, const void *W,
                                 const void *side, const void *ap, const void *zero, void *C, hipStream_t st)
{
    const int64_t N = FWD ? h.K : h.D;
    const int tiles_m = (int)((h.T + BM - 1) / BM), tiles_n = (int)((N + BN - 1) / BN);
    auto kern = k_gemm<FWD>;
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kGemmLds);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)(tiles_m * tiles_n)), dim3(512), kGemmLds, st, mv,
                       static_cast<const uint16_t *>(S), static_cast<const uint16_t *>(W),
                       static_cast<const uint16_t *>(side), static_cast<const uint16_t *>(ap),
                       static_cast<const uint16_t *>(zero), static_cast<uint16_t *>(C), tiles_m, tiles_n);
    return hipGetLastError();
}

hipError_t launch_gemm_bf16(const MetaView &mv, const MetaHeader &h, bool forward, const void *S, const void *W,
                            const void *side, const void *ap, const void *zero, void *C, hipStream_t st)
{
    if (h.T == 0) return hipSuccess;
    if (forward) return launch_variant<true>(mv, h, S, W, side, ap, zero, C, st);
    return launch_variant<false>(mv, h, S, W, side, ap, zero, C, st);
}

}  // namespace plora
