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
// rows of the other segments pointed at a page of zeros.  What a tile has to know about its
// segments comes as one record per row tile (GemmTile, derived by the preparation kernel), touched
// one tile ahead so that the fetch at the tile switch hits the scalar cache.
//
// Tile: 256 x 256 outputs per workgroup, 64-deep K steps (stages), 8 waves (2 along rows x 4 along
// columns, 128 x 64 outputs each).  Operands go HBM -> LDS directly (global_load_lds, 16 bytes per
// lane); the 16-byte chunks of a row are XOR-swizzled on the way in (by choosing which chunk each
// lane fetches) so that MFMA operand reads are free of bank conflicts.  A stage is fetched as four
// granules of 16 KB (the two row halves of the S-side tile, two halves of the W-side tile), each
// kind in its own small ring, 160 KB of LDS in all; the two waves that share a SIMD alternate
// between multiplying from registers and fetching (LDS -> registers, plus one granule HBM -> LDS).
// W is used as it lies in memory in both directions.  With W [d_in][d_out], backward contracts over
// its contiguous index and reads operands with ds_read_b128; forward contracts over its row index
// and reads operands with the transposing LDS load (ds_read_b64_tr_b16), so no transposed copy of W
// is ever made.  With W [d_out][d_in] the two forms swap roles (forward reads with ds_read_b128),
// and so do the low-rank operands: the form with the contraction index as row index takes its
// extension rows from GemmSeg::B ([r][N]: B_k, or the packed A_k^T), the other from the padded
// buffer ([N][rp]: A_k, or B_k^T).
#include "plora_internal.h"


namespace plora {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T *)(p))
#define GLB_PTR(p) ((const __attribute__((address_space(1))) void *)(p))

constexpr int BM = 256, BN = 256;

// no-ops behind the alignment point in front of the kernel's loops, per form (see the kernel)
#ifndef PLORA_GEMM_PAD_FWD
#define PLORA_GEMM_PAD_FWD 1
#endif
#ifndef PLORA_GEMM_PAD_DX
#define PLORA_GEMM_PAD_DX 4
#endif

// two floats -> packed bf16 pair, round to nearest even (one v_cvt_pk_bf16_f32 on gfx950)
__device__ inline uint32_t pack_bf16x2(float lo, float hi)
{
    typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
    typedef float v2f __attribute__((ext_vector_type(2)));
    const v2f f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, v2bf));
}

// Segment table walk for tiles that overlap more than the two segments spelled out in their GemmTile:
// the next segment at or after `from` that overlaps rows [.., m1), has an adapter and at least one row.
__device__ inline int next_ext_seg(const MetaView &mv, int n, int from, int m1)
{
    for (int s = from; s < n; ++s) {
        const int r0 = mv.seg[s].row0, r1 = mv.seg[s].row1;
        if (r0 >= m1) return n;
        if (mv.seg[s].adapter >= 0 && r1 > r0) return s;
    }
    return n;
}

__device__ inline GemmSeg load_ext_seg(const MetaView &mv, int s)
{
    const SegInfo g = mv.seg[s];
    const AdapterInfo a = mv.ad[g.adapter];
    GemmSeg q;
    q.row0 = g.row0; q.row1 = g.row1; q.rp = g.rp; q.r = g.r; q.hb_off = g.hb_off; q.B = a.ext_b; q.ap_off = a.ap_off;
    return q;
}

template <int N> __device__ inline void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit field");
    // gfx9 encoding: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt_hi[15:14]; other counters left at max
    __builtin_amdgcn_s_waitcnt(0x0f70 | (N & 15) | ((N >> 4) << 14));
}

constexpr int BK = 64;                       // contraction elements per stage
constexpr int KS = BK / 16;                  // MFMA K steps per stage (4)
constexpr int GR = 16384;                    // bytes of a granule: 128 rows x 64 k, or 32 k x 256 n
constexpr int kXL = 0, kXT = 2 * GR, kWA = 4 * GR, kWB = 7 * GR;   // rings: 2 + 2 + 3 + 3 granules
constexpr int kGemmLds = 10 * GR;            // all 160 KB of a compute unit
constexpr int WN = 2;                        // 32-column blocks per wave: 8 waves of 128 x 64 outputs
constexpr int NL = 4;                        // load instructions (1 KB each) per wave per granule
static_assert(kRankPadGemm % BK == 0, "extension steps must be whole stages");
static_assert(KS == 4 && BM == 256 && BN == 256, "the schedule below is written for this tile");
static_assert(BM == kGemmTileRows && BK == kRankPadGemm, "the per-tile extension table is built for this tile");

__device__ inline void wait_vmcnt_048(int n)
{
    if (n >= 8) wait_vmcnt<8>();
    else if (n >= 4) wait_vmcnt<4>();
    else wait_vmcnt<0>();
}

// 8 bf16 + 8 bf16 in fp32, rounded to nearest even (the accumulating epilogue)
__device__ inline uint32_t add_bf16x2(uint32_t a, uint32_t b)
{
    return pack_bf16x2(__uint_as_float(a << 16) + __uint_as_float(b << 16),
                       __uint_as_float(a & 0xffff0000u) + __uint_as_float(b & 0xffff0000u));
}

// ACC: the result is added to what Cout holds (read in the epilogue, one more rounding to bf16), for gradients of an
// input that several projections share.
template <bool FWD, bool ACC = false>
__global__ void __launch_bounds__(512) k_gemm(const GemmTile *__restrict__ tiles, const int32_t *__restrict__ order,
                                              const SegInfo *__restrict__ segs,
                                              const AdapterInfo *__restrict__ ads, const uint16_t *__restrict__ S,
                                              const uint16_t *__restrict__ W, const uint16_t *__restrict__ side,
                                              const uint16_t *__restrict__ ap, const uint16_t *__restrict__ zero,
                                              uint16_t *__restrict__ Cout, int tiles_m, int tiles_n, int M, int Kd, int N, int n_seg)
{
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    // the metadata pointers come one by one and restrict-qualified: that lets the compiler fetch the records through
    // the scalar cache (a vector load would be counted, in order, with the direct-to-LDS loads of the ring)
    MetaView mv;
    mv.hdr = nullptr; mv.seg = segs; mv.ad = ads; mv.tile = tiles; mv.blk_seg = nullptr; mv.seg_list = nullptr;
    mv.tile_order = order;
    // shapes come as kernel arguments, so the first loads do not wait for a metadata fetch.  FWD names the form of
    // the weight operand: W[Kd][N] (contraction index = row index; the forward product when W is [d_in][d_out]),
    // otherwise W[N][Kd]
    const int ldw = FWD ? N : Kd;

    // ---- workgroup -> tiles.  The grid is persistent (one workgroup per compute unit, each walks the
    // tile ids b, b + grid, b + 2 grid, ...).  Workgroups are dealt round-robin to the 8 XCDs (each with
    // its own L2); give every XCD a contiguous range of tile ids, and walk tile ids in groups of 4 row
    // tiles so that the tiles resident on one XCD at a time share rows of S and columns of W.  The
    // row tiles are taken in the order of the `order` table (sorted by their number of extension
    // steps), so that the four row tiles of a group are equally long: workgroups that stream the same
    // columns of W then stay in step, which is what makes that sharing work (tiles of unequal length
    // side by side cost about 5 % of the kernel's time).
    const int n_tiles = tiles_m * tiles_n;
    int m0 = 0, n0 = 0, m1 = 0;
    auto tile_coords = [&](int vb, int &row_tile, int &col_tile) {
        int tile = vb;
        const int per = n_tiles / 8;
        if (tile < per * 8) tile = (tile % 8) * per + tile / 8;
        constexpr int GM = kGemmGroupRows;
        const int group = tile / (GM * tiles_n), first = group * GM;
        const int gsz = (tiles_m - first < GM) ? tiles_m - first : GM;
        const int in = tile - group * GM * tiles_n;
        row_tile = order[first + in % gsz];
        col_tile = in / gsz;
    };
    auto set_tile = [&](int vb) {
        int rt, ct;
        tile_coords(vb, rt, ct);
        m0 = rt * BM;
        n0 = ct * BN;
        m1 = (m0 + BM < M) ? m0 + BM : M;
    };

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform: LDS bases stay scalar
    const int grp = wave >> 2;              // 0: leading group (tile rows 0..127), 1: trailing group (rows 128..255)
    const int w4 = wave & 3;

    // ---- loader.  The four waves of a group fetch one granule per read phase, four 1 KB instructions
    // each (instruction q = w4 + 4 jj).  The leading group fetches the S-side rows of the trailing group
    // and the second W-side half, the trailing group the S-side rows of the leading group and the first
    // W-side half (who fetches what only follows from when its ring slot comes free, see the schedule).
    // S-side granule [128 rows][8 chunks]: instruction q covers rows 8q..8q+7, lane -> (row 8q + lane/8,
    // slot lane%8), slot c' of row u holds chunk c' ^ ((u >> 1) & 7).  Backward W-side granule
    // [128 n][8 chunks]: the same.  Forward W-side granule [32 k][32 chunks]: instruction q covers k rows
    // 2q, 2q+1, lane -> (k row 2q + lane/32, slot lane%32), slot c' of k row u holds chunk c' ^ (4 (u & 3)).
    const int x_half = grp ^ 1, w_half = grp ^ 1;
    const int a_row = w4 * 8 + lane / 8;                              // + 32 jj, row inside the granule
    const int a_chunk = (lane % 8) ^ ((a_row >> 1) & 7);              // 32 jj leaves bits 1..3 alone
    const int b_row = FWD ? w4 * 2 + (lane >> 5) : a_row;             // + 8 jj (forward: k row) / + 32 jj
    const int b_chunk = FWD ? ((lane & 31) ^ (4 * (b_row & 3))) : a_chunk;

    // Full main K steps are fetched as (uniform base that advances per stage) + (per-lane byte offset
    // inside the tile that never changes).  Rows and columns past the end are clamped: they only feed
    // outputs that are never stored.
    uint32_t off_x[NL], off_w[NL];
    const char *base_x = nullptr, *base_w = nullptr;
    const int64_t step_w = FWD ? (int64_t)BK * ldw * 2 : (int64_t)BK * 2;
    auto set_addresses = [&]() {
#pragma unroll
        for (int jj = 0; jj < NL; ++jj) {
            int row = m0 + x_half * 128 + a_row + 32 * jj;
            row = row < M ? row : M - 1;
            off_x[jj] = (uint32_t)(row - m0) * (uint32_t)Kd * 2u + (uint32_t)a_chunk * 16u;
            if (FWD) {
                int n = n0 + b_chunk * 8;
                n = n < N ? n : N - 8;
                off_w[jj] = (uint32_t)(w_half * 32 + b_row + 8 * jj) * (uint32_t)ldw * 2u + (uint32_t)(n - n0) * 2u;
            } else {
                int n = n0 + w_half * 128 + b_row + 32 * jj;
                n = n < N ? n : N - 1;
                off_w[jj] = (uint32_t)(n - n0) * (uint32_t)ldw * 2u + (uint32_t)b_chunk * 16u;
            }
        }
        base_x = reinterpret_cast<const char *>(S) + (int64_t)m0 * Kd * 2;
        base_w = reinterpret_cast<const char *>(W) + (FWD ? (int64_t)n0 * 2 : (int64_t)n0 * ldw * 2);
    };

    // Stages of a tile: first one extension step per 64 padded rank columns of every segment with an
    // adapter that overlaps the rows of the tile, then the main K steps.  The extension steps come
    // first because their operands (the low-rank factor, B_k or A_k) are cold - first touched by this
    // tile - while the main operands stream: fetched in the prologue, their latency hides behind the
    // stores of the previous tile instead of stalling the end of the loop.
    const int nk_main = (Kd + BK - 1) / BK;
    int n_it = 0;
    // cursor over the extension steps: ext_pos = which of the tile's segments is being issued (0 and 1 are spelled
    // out in the tile's record, from 2 on the segment table is walked: ext_walk = index of that segment), ext_kk =
    // its next rank column.  The record is re-read where it is used - it sits
    // in the scalar cache by then - rather than held in registers, which this kernel has none to spare of.
    int ext_pos = 0, ext_kk = 0, ext_walk = 0;
    const int n_seg_all = n_seg;
    auto scan_segments = [&]() {
        const GemmTile *gt = mv.tile + __builtin_amdgcn_readfirstlane(m0 / BM);
        n_it = nk_main + gt->n_ext;
        ext_walk = gt->third_seg;
        ext_pos = 0;
        ext_kk = 0;
    };
    auto ext_segment = [&]() -> GemmSeg {
        const int pos = __builtin_amdgcn_readfirstlane(ext_pos);
        if (pos < 2) return mv.tile[__builtin_amdgcn_readfirstlane(m0 / BM)].s[pos];
        return load_ext_seg(mv, __builtin_amdgcn_readfirstlane(ext_walk));
    };
    auto ext_advance = [&]() {
        ext_kk = 0;
        if (ext_pos >= 2) ext_walk = next_ext_seg(mv, n_seg_all, ext_walk + 1, m1);   // rare: over two segments in a row tile
        ext_pos += 1;
    };

    // The direct-to-LDS loads are issued through inline assembly: the compiler, which cannot tell
    // the granule being filled from the one being read, would otherwise make every LDS read wait
    // for all of them (vmcnt(0)) and serialise the pipeline.  Ordering is explicit instead: a
    // counted s_waitcnt plus a bare barrier before a granule is read (__syncthreads would add a
    // fence that drains every load in flight).  M0 holds the wave-uniform LDS destination; lane i
    // lands at M0 + 16 i.  M0 is not named as a clobber: it is a reserved register on this target (the
    // compiler rejects it in clobber lists as undefined behaviour) in which the compiler keeps no value
    // across statements - it writes M0 itself right in front of each of its own instructions that read it.
    const uint32_t lds_base = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)LDS_PTR(char, lds));
    auto load_ptr = [&](const void *g, uint32_t dst) {
        asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(dst));
    };
    auto load_off = [&](uint32_t off, const char *base, uint32_t dst) {
        asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(off), "s"(base), "s"(dst));
    };
    // A wave fetches, stage after stage, first its W-side granule and then its S-side granule.
    // issue_w(it, slot) / issue_x(it, slot) issue the four loads of that granule of stage `it` into
    // ring slot `slot`; issue_x also moves the cursor over the low-rank extension steps.  The last,
    // partial main K step masks chunks past the end of the contraction with a page of zeros; the
    // extension steps of segment ext_seg read the bf16 low-rank factor of the rows that belong to
    // that segment (zeros for the other rows of the tile) and B_k or the padded A_k.
    auto issue_w = [&](int it, int slot) {
        const uint32_t dst = lds_base + (w_half ? kWB : kWA) + slot * GR + w4 * 1024;
        const int n_ext = n_it - nk_main;
        if (it >= n_ext) {
            const int k0 = (it - n_ext) * BK;
            const char *gw = base_w + (int64_t)(it - n_ext) * step_w;
            if (k0 + BK <= Kd) {
#pragma unroll
                for (int jj = 0; jj < NL; ++jj) load_off(off_w[jj], gw, dst + jj * 4096);
            } else {
#pragma unroll
                for (int jj = 0; jj < NL; ++jj) {
                    const bool ok = FWD ? (k0 + w_half * 32 + b_row + 8 * jj < Kd) : (k0 + b_chunk * 8 < Kd);
                    load_ptr(ok ? static_cast<const void *>(gw + off_w[jj]) : zero, dst + jj * 4096);
                }
            }
        } else {
            const int kk = __builtin_amdgcn_readfirstlane(ext_kk);
            const GemmSeg es = ext_segment();
#pragma unroll
            for (int jj = 0; jj < NL; ++jj) {
                const uint16_t *gw;
                if (FWD) {
                    const int j = kk + w_half * 32 + b_row + 8 * jj;   // row of B_k
                    int n = n0 + b_chunk * 8;
                    n = n < N ? n : N - 8;
                    // j < 128 and ldw <= 2^22: the row offset fits 32 bits
                    gw = (j < es.r) ? static_cast<const uint16_t *>(es.B) + ((uint32_t)j * (uint32_t)ldw + (uint32_t)n) : zero;
                } else {
                    int n = n0 + w_half * 128 + b_row + 32 * jj;       // row of padded A_k
                    n = n < N ? n : N - 1;
                    gw = ap + es.ap_off + (int64_t)n * es.rp + kk + b_chunk * 8;
                }
                load_ptr(gw, dst + jj * 4096);
            }
        }
    };
    auto issue_x = [&](int it, int slot) {
        const uint32_t dst = lds_base + (x_half ? kXT : kXL) + slot * GR + w4 * 1024;
        const int n_ext = n_it - nk_main;
        if (it >= n_ext) {
            const int k0 = (it - n_ext) * BK;
            const char *gx = base_x + (int64_t)k0 * 2;
            if (k0 + BK <= Kd) {
#pragma unroll
                for (int jj = 0; jj < NL; ++jj) load_off(off_x[jj], gx, dst + jj * 4096);
            } else {
#pragma unroll
                for (int jj = 0; jj < NL; ++jj) {
                    const bool ok = k0 + a_chunk * 8 < Kd;
                    load_ptr(ok ? static_cast<const void *>(gx + off_x[jj]) : zero, dst + jj * 4096);
                }
            }
        } else {
            const int kk = __builtin_amdgcn_readfirstlane(ext_kk);
            const GemmSeg es = ext_segment();
#pragma unroll
            for (int jj = 0; jj < NL; ++jj) {
                const int row = m0 + x_half * 128 + a_row + 32 * jj;
                const bool in = row >= es.row0 && row < es.row1;
                load_ptr(in ? side + es.hb_off + (int64_t)(row - es.row0) * es.rp + kk + a_chunk * 8 : zero, dst + jj * 4096);
            }
            ext_kk = kk + BK;
            if (ext_kk >= es.rp) ext_advance();
        }
    };

    // ---- MFMA operand addressing.  Wave (grp, w4) owns rows grp*128.. and columns w4*64..
    const int wm0 = grp * 128, wn0 = w4 * (WN * 32);
    const int l32 = lane & 31, kg = lane >> 5;
    // S-side operand (4 blocks of 32 rows of the wave's own granule): row u = mi*32 + l32, chunk = ks*2 + kg
    int xoff[4];
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) {
        const int u = mi * 32 + l32;
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
            const int kr = (g4 >> 1) * 8 + (i16 >> 2);                      // + 16 for the second K step, + 4 for the second read
            woff[ni] = kr * 512 + ((((nl >> 3) ^ (4 * (kr & 3))) * 16) + (nl & 7) * 2);
        } else {
            const int u = (wn0 & 127) + ni * 32 + l32;                      // row inside the wave's W-side half
            woff[ni] = u * (BK * 2) + ((kg ^ ((u >> 1) & 7)) * 16);
        }
    }

    f32x16 acc[WN][4];

    // MFMA operands of half a stage (two K steps of 16): 8 S-side + 4 W-side fragments.
    // xs: slot of the wave's S-side granule; wa, wb: slots of the two W-side halves (byte offsets in LDS).
    bf16x8 xf[2][4], wf[2][WN];
    auto read_half = [&](int xs, int wa, int wb, int h) {
        const char *sx = lds + xs;
        // forward: K half h of the stage is W-side half h; backward: the wave's columns lie in one half
        const char *sw = lds + (FWD ? (h ? wb : wa) : (wn0 >= 128 ? wb : wa));
#pragma unroll
        for (int k2 = 0; k2 < 2; ++k2) {
            const int ks = 2 * h + k2;
#pragma unroll
            for (int mi = 0; mi < 4; ++mi)
                xf[k2][mi] = *LDS_PTR(const bf16x8, sx + (xoff[mi] ^ (ks * 32)));
#pragma unroll
            for (int ni = 0; ni < WN; ++ni) {
                if (FWD) {
                    const char *p = sw + woff[ni] + k2 * 16 * 512;
                    bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(LDS_PTR(bf16x4, p));
                    bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(LDS_PTR(bf16x4, p + 4 * 512));
                    wf[k2][ni] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                } else {
                    wf[k2][ni] = *LDS_PTR(const bf16x8, sw + (woff[ni] ^ (ks * 32)));
                }
            }
        }
    };
    auto mfma_half = [&]() {
#pragma unroll
        for (int k2 = 0; k2 < 2; ++k2)
#pragma unroll
            for (int ni = 0; ni < WN; ++ni)
#pragma unroll
                for (int mi = 0; mi < 4; ++mi)
                    acc[ni][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[k2][ni], xf[k2][mi], acc[ni][mi], 0, 0, 0);
    };
    // workgroup barrier that the compiler may move nothing across: neither memory accesses nor MFMAs
    // (the phases below only work if each instruction stays in the phase it was written in)
    auto barrier = [&]() {
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("" ::: "memory");
    };

    // ---- schedule.  Time runs in phases of half a stage, one barrier each.  The two waves that share a
    // SIMD (w and w + 4) alternate roles: while one issues the 16 MFMAs of a half stage back to back
    // from registers, the other reads the operands of its next half stage from LDS and issues one
    // granule of direct loads.  The leading group reads half h of stage s in phase 4s + 2h and multiplies
    // in the next phase; the trailing group runs one phase behind.  Last reads of the granules of stage s:
    //   S rows of the leading group: phase 4s+2      S rows of the trailing group: phase 4s+3
    //   W halves: phase 4s+3
    // With rings of 2, 2, 3 and 3 slots the granules of stage s can be fetched in the phases
    //   first W half 4s-7 (trailing group), second W half 4s-6 (leading), leading S rows 4s-5 (trailing),
    //   trailing S rows 4s-4 (leading),
    // one granule per phase, each four phases or more before the phase that ends with the wait for it.
    // A wave waits, at the end of each of its read phases, until all but the last two granules it has
    // issued are complete; the barrier that follows publishes them.
    int gi = 0;                               // granules this wave has issued (stage s: W granule 2s, S granule 2s+1)
    auto wait_done = [&](int need) {          // granules 0..need of this wave complete (no-op past the last one)
        int after = gi - 1 - (need < 2 * n_it ? need : 2 * n_it - 1);
        wait_vmcnt_048(4 * (after < 0 ? 0 : after));
    };
    // Prologue of a tile: both groups fetch their granules of stages 0 and 1 (the leading group leaves the
    // S granule of stage 1 to its first read phase).
    auto prologue = [&]() {
        set_addresses();
        scan_segments();
        issue_w(0, 0); issue_x(0, 0); gi = 2;
        if (n_it > 1) {
            issue_w(1, 1); ++gi;
            if (grp == 1) { issue_x(1, 1); ++gi; }
        }
    };

    // The record of the tile after this one is touched early in the loop (two scalar loads, one per 64-byte
    // line), so that the fetch of it at the tile switch finds it in the scalar cache instead of waiting on L2.
    auto touch_next_tile = [&](int vb_now) {
        if (vb_now + (int)gridDim.x >= n_tiles) return;
        int rt, ct;
        tile_coords(vb_now + (int)gridDim.x, rt, ct);
        const int32_t *p = reinterpret_cast<const int32_t *>(mv.tile + __builtin_amdgcn_readfirstlane(rt));
        const int32_t a = p[0], b = p[16];
        asm volatile("" ::"s"(a), "s"(b));
    };

    // Placement of the loops below in the instruction stream, fixed here so that it does not move when code above
    // changes: a 256-byte boundary plus a few 4-byte no-ops.  The kernel's time depends on where its loops fall
    // inside the 32-byte windows instructions are fetched in, by up to 10 % at the largest shapes (8192 -> 28672,
    // 32768 tokens: 12.15 to 13.43 ms over the eight possible offsets for the first form, 11.50 to 12.33 ms for the
    // second) and through a second-order effect: compute units that share an instruction cache fall a few cycles out
    // of step with one another, and that decides whether the workgroups that stream the same rows of S and columns
    // of W ask the L2 for a line one after the other (one miss, the rest hits) or at the same instant (every one a
    // miss: 1.9e8 against 5.9e8 L2 misses per launch).  The offsets (PLORA_GEMM_PAD_FWD / _DX no-ops, one value per
    // form) were chosen by measurement; any change to the code from here to the end of the kernel calls for a new sweep
    // (python -m paper_2508_02932_amd.sweep_placement builds and times the eight candidates).
    asm volatile(".p2align 8\n\t.rept %0\n\ts_nop 0\n\t.endr" ::"n"(FWD ? PLORA_GEMM_PAD_FWD : PLORA_GEMM_PAD_DX) : "memory");
    int vb = blockIdx.x;
    set_tile(vb);
    prologue();
    while (true) {
#pragma unroll
    for (int ni = 0; ni < WN; ++ni)
#pragma unroll
        for (int mi = 0; mi < 4; ++mi)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[ni][mi][i] = 0.f;
    wait_done(grp == 1 ? 1 : 0);              // leading group: its S granule of stage 0 is only read in phase 1
    barrier();

    if (grp == 0) {
        // leading group
        int s3 = 0;                           // s % 3
        for (int s = 0; s < n_it; ++s) {
            const int xs = kXL + (s & 1) * GR, wa = kWA + s3 * GR, wb = kWB + s3 * GR;
            const int s3n = s3 == 2 ? 0 : s3 + 1, s3nn = s3n == 2 ? 0 : s3n + 1;
            // phase 4s: read half 0; fetch the trailing group's S rows of stage s+1
            if (s == 1) touch_next_tile(vb);
            read_half(xs, wa, wb, 0);
            if (s + 1 < n_it) { issue_x(s + 1, (s + 1) & 1); ++gi; }
            __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0): operands in registers before the roles swap
            wait_done(2 * s + 1);
            barrier();
            mfma_half();                      // phase 4s+1
            barrier();
            // phase 4s+2: read half 1; fetch the second W half of stage s+2
            read_half(xs, wa, wb, 1);
            if (s + 2 < n_it) { issue_w(s + 2, s3nn); ++gi; }
            __builtin_amdgcn_s_waitcnt(0xc07f);
            wait_done(2 * s + 2);
            barrier();
            mfma_half();                      // phase 4s+3
            barrier();
            s3 = s3n;
        }
        barrier();                            // phase 4 n_it: the trailing group multiplies its last half
    } else {
        // trailing group
        barrier();                            // phase 0
        int s3 = 0;
        for (int s = 0; s < n_it; ++s) {
            const int xs = kXT + (s & 1) * GR, wa = kWA + s3 * GR, wb = kWB + s3 * GR;
            const int s3n = s3 == 2 ? 0 : s3 + 1, s3nn = s3n == 2 ? 0 : s3n + 1;
            // phase 4s+1: read half 0; fetch the first W half of stage s+2
            if (s == 1) touch_next_tile(vb);
            read_half(xs, wa, wb, 0);
            if (s + 2 < n_it) { issue_w(s + 2, s3nn); ++gi; }
            __builtin_amdgcn_s_waitcnt(0xc07f);
            wait_done(2 * s + 2);
            barrier();
            mfma_half();                      // phase 4s+2
            barrier();
            // phase 4s+3: read half 1; fetch the leading group's S rows of stage s+2
            read_half(xs, wa, wb, 1);
            if (s + 2 < n_it) { issue_x(s + 2, s & 1); ++gi; }
            __builtin_amdgcn_s_waitcnt(0xc07f);
            wait_done(2 * s + 3);
            barrier();
            mfma_half();                      // phase 4s+4
            barrier();
            s3 = s3n;
        }
    }
    // Every LDS read of this tile has been issued and waited for: the rings are free.  Start fetching the
    // next tile before storing this one, so that its first loads fly during the stores.
    const int em0 = m0, en0 = n0;
    vb += gridDim.x;
    const bool more = vb < n_tiles;
    if (more) {
        set_tile(vb);
        prologue();
    }

    // ---- epilogue: MFMA rows are output columns n, MFMA columns are output rows m: a lane holds, for
    // each group i4 of 4 registers, 4 consecutive n of one m.  Stored straight from there, every store
    // instruction would touch 32 rows with 16 bytes each; instead each wave passes its 32 x 64 blocks
    // through 4 KB of LDS of its own (the third slots of the W rings, which the prologue of the next
    // tile does not touch) and stores whole 128-byte rows, 16 bytes per lane.
    {
        char *stg = lds + (grp == 0 ? kWA : kWB) + 2 * GR + w4 * 4096;
        // ACC: what the tile holds so far, all 16 pieces of this lane requested before the first is needed
        uint4 old[ACC ? 16 : 1];
        if constexpr (ACC) {
#pragma unroll
            for (int mi = 0; mi < 4; ++mi)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int row = (lane >> 3) + 8 * j, c = lane & 7;
                    const int m = em0 + wm0 + mi * 32 + row, n = en0 + wn0 + c * 8;
                    old[mi * 4 + j] = (m < M && n < N) ? *reinterpret_cast<const uint4 *>(Cout + (int64_t)m * N + n) : uint4{0u, 0u, 0u, 0u};
                }
        }
#pragma unroll
        for (int mi = 0; mi < 4; ++mi) {
#pragma unroll
            for (int ni = 0; ni < WN; ++ni)
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4) {
                    uint2 v;
                    v.x = pack_bf16x2(acc[ni][mi][i4 * 4 + 0], acc[ni][mi][i4 * 4 + 1]);
                    v.y = pack_bf16x2(acc[ni][mi][i4 * 4 + 2], acc[ni][mi][i4 * 4 + 3]);
                    const int chunk = ni * 4 + i4;                     // 16-byte chunk of the 128-byte row
                    *reinterpret_cast<uint2 *>(stg + l32 * 128 + ((chunk ^ (l32 & 7)) * 16) + kg * 8) = v;
                }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int row = (lane >> 3) + 8 * j, c = lane & 7;
                const uint4 v = *reinterpret_cast<const uint4 *>(stg + row * 128 + ((c ^ (row & 7)) * 16));
                const int m = em0 + wm0 + mi * 32 + row, n = en0 + wn0 + c * 8;
                if (m < M && n < N) {
                    if constexpr (ACC) {
                        const uint4 o = old[mi * 4 + j];
                        uint4 sum;
                        sum.x = add_bf16x2(o.x, v.x); sum.y = add_bf16x2(o.y, v.y);
                        sum.z = add_bf16x2(o.z, v.z); sum.w = add_bf16x2(o.w, v.w);
                        *reinterpret_cast<uint4 *>(Cout + (int64_t)m * N + n) = sum;
                    } else {
                        *reinterpret_cast<uint4 *>(Cout + (int64_t)m * N + n) = v;
                    }
                }
            }
        }
    }
    if (!more) break;
    }
    wait_vmcnt<0>();                          // no direct-to-LDS load may outlive the workgroup
}

template <bool FWD, bool ACC>
static hipError_t launch_variant(const MetaView &mv, const MetaHeader &h, int64_t Kd, int64_t N, const void *S, const void *W,
                                 const void *side, const void *ap, const void *zero, void *C, hipStream_t st)
{
    const int tiles_m = (int)((h.T + BM - 1) / BM), tiles_n = (int)((N + BN - 1) / BN);
    auto kern = k_gemm<FWD, ACC>;
    {
        hipError_t e = allow_full_lds(reinterpret_cast<const void *>(kern), (FWD ? 5 : 6) + (ACC ? 4 : 0));
        if (e != hipSuccess) return e;
    }
    // persistent grid: one workgroup per compute unit (256 on an MI355X; a workgroup takes a whole CU's LDS)
    hipError_t cu_err = hipSuccess;
    const int n_cu = device_cu_count(&cu_err);
    if (n_cu < 1) return cu_err;
    const int n_tiles = tiles_m * tiles_n;
    hipLaunchKernelGGL(kern, dim3((unsigned)(n_tiles < n_cu ? n_tiles : n_cu)), dim3(512), kGemmLds, st, mv.tile, mv.tile_order,
                       mv.seg, mv.ad,
                       static_cast<const uint16_t *>(S), static_cast<const uint16_t *>(W),
                       static_cast<const uint16_t *>(side), static_cast<const uint16_t *>(ap),
                       static_cast<const uint16_t *>(zero), static_cast<uint16_t *>(C), tiles_m, tiles_n, (int)h.T, (int)Kd,
                       (int)N, (int)h.n_seg);
    return hipGetLastError();
}

hipError_t launch_gemm_bf16(const MetaView &mv, const MetaHeader &h, bool w_rows_contract, int64_t Kd, int64_t N,
                            const void *S, const void *W, const void *side, const void *ap, const void *zero, void *C,
                            bool accumulate, hipStream_t st)
{
    if (h.T == 0) return hipSuccess;
    if (accumulate) {
        if (w_rows_contract) return launch_variant<true, true>(mv, h, Kd, N, S, W, side, ap, zero, C, st);
        return launch_variant<false, true>(mv, h, Kd, N, S, W, side, ap, zero, C, st);
    }
    if (w_rows_contract) return launch_variant<true, false>(mv, h, Kd, N, S, W, side, ap, zero, C, st);
    return launch_variant<false, false>(mv, h, Kd, N, S, W, side, ap, zero, C, st);
}

}  // namespace plora
