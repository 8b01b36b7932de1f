// Stand-alone low-rank update of the packed multi-LoRA layer on bf16 inputs (gfx950), for callers that
// compute the base product themselves:
//   forward   y_t  += scale_k (x_t A_k) B_k      (section 2.4: the low-rank half of the layer)
//   backward  dx_t += g_t A_k^T                  (appendix C.2, case 4: its low-rank half)
// C[T][N] is read, updated in fp32 and written back once (rounded to nearest even), so the kernel is
// bound by HBM: 2 x 2 bytes per element of C.  The two small operands come as the other kernels of the
// library already keep them: the bf16 low-rank factor [len][rp] of each segment (scale_k h, or g) and
// the padded, transposed small matrix [N][rp] (B_k^T, or A_k), both with zeros beyond the rank, so a
// lane fetches its MFMA operands as 16 contiguous bytes straight from L2 and the rank is never tiled
// (appendix C.2).  Only the C tile goes through LDS: it comes in by direct loads in whole 256-byte
// row pieces, is read and rewritten there in the MFMA accumulator layout, and leaves in whole row
// pieces again.  Every wave owns 32 token rows of the tile, so no workgroup barrier is needed.
#include "plora_internal.h"

namespace plora {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T *)(p))

constexpr int EX_COLS = 128;                       // columns of C per workgroup (256 bytes per row)
constexpr int EX_NW = kSkinnyRows / 32;            // 4 waves, 32 token rows each
constexpr int EX_NB = EX_COLS / 16;                // 16-column MFMA blocks per wave
constexpr int EX_LDS = kSkinnyRows * EX_COLS * 2;  // 32 KB

__device__ inline uint32_t ex_pack_bf16x2(float lo, float hi)
{
    typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
    typedef float v2f __attribute__((ext_vector_type(2)));
    const v2f f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, v2bf));
}

// One workgroup per (token block of 128 rows of one segment, 128 columns of C).
//   side : bf16 low-rank factor, segment s at side + hb_off, rows of rp elements
//   opT  : small matrices [N][rp], adapter k at opT + N * (ap_off_k / table_rows): the padded buffer laid out for N
//          rows (the tables carry the offsets for table_rows rows, i.e. table_rows * sum of rp over the adapters before)
__global__ void __launch_bounds__(64 * EX_NW) k_expand(MetaView mv, uint16_t *__restrict__ C, int N,
                                                       const uint16_t *__restrict__ side, const uint16_t *__restrict__ opT,
                                                       int64_t table_rows, const uint16_t *__restrict__ zero)
{
    __shared__ __attribute__((aligned(1024))) char lds[EX_LDS];
    const int blk = blockIdx.x;
    const SegInfo g = mv.seg[mv.blk_seg[blk]];
    const AdapterInfo a = mv.ad[g.adapter];
    const int t0 = (blk - g.blk0) * kSkinnyRows;
    const int nt = (g.row1 - g.row0 - t0 < kSkinnyRows) ? g.row1 - g.row0 - t0 : kSkinnyRows;
    const int n0 = blockIdx.y * EX_COLS;
    const int rp = g.rp;
    const int ksteps = (g.r + 31) / 32;            // 32 rank columns per MFMA; columns r .. 32 ksteps are zero on both sides

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t lds_base = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)LDS_PTR(char, lds));

    // ---- C tile -> LDS.  A load instruction moves 4 rows x 256 bytes: lane -> (row 4q + lane/16, slot lane%16); slot c'
    // of row u holds the 16-byte chunk c' ^ (u & 15), so that the 16 rows a quarter wave reads below fall into 16
    // different chunk positions.  Wave w moves and owns rows 32w .. 32w+31 (instructions q = 8w .. 8w+7).
    uint16_t *Crow0 = C + (int64_t)(g.row0 + t0) * N;
    const int lrow = lane >> 4, slot = lane & 15;
    bool ok[8];
    int64_t goff[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int u = wave * 32 + j * 4 + lrow;
        const int n = n0 + (slot ^ (u & 15)) * 8;
        ok[j] = u < nt && n < N;
        goff[j] = (int64_t)u * N + n;
        const void *src = ok[j] ? static_cast<const void *>(Crow0 + goff[j]) : static_cast<const void *>(zero);
        const uint32_t dst = lds_base + (wave * 8 + j) * 1024;
        asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(src), "s"(dst));
    }

    // ---- low-rank operands straight from memory (they sit in L2: every column tile reads the same factor rows, every
    // token block of an adapter the same small-matrix rows).  MFMA 16x16x32: the first operand's rows are columns n of
    // C, the second operand's columns are token rows, so a lane ends up with 4 consecutive n of one token.
    const int lm = lane & 15, kg = lane >> 4;
    const uint16_t *op = opT + (a.ap_off / table_rows) * (int64_t)N;      // this adapter's [N][rp]
    bf16x8 sf[2][4], bfr[2][4];
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) {
        int u = wave * 32 + tb * 16 + lm;
        u = u < nt ? u : nt - 1;                                          // clamped rows are never stored
        const uint16_t *p = side + g.hb_off + (int64_t)(t0 + u) * rp + kg * 8;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
            if (ks < ksteps) sf[tb][ks] = *reinterpret_cast<const bf16x8 *>(p + ks * 32);
    }
    auto load_block = [&](int b, bf16x8 *dst) {                           // small-matrix rows of column block b
        int n = n0 + b * 16 + lm;
        n = n < N ? n : N - 1;                                            // clamped columns are never stored
        const uint16_t *p = op + (int64_t)n * rp + kg * 8;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
            if (ks < ksteps) dst[ks] = *reinterpret_cast<const bf16x8 *>(p + ks * 32);
    };
    load_block(0, bfr[0]);
    load_block(1, bfr[1]);

    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");                    // this wave's rows of the tile are in LDS
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int b = 0; b < EX_NB; ++b) {
        bf16x8 cur[4];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) cur[ks] = bfr[b & 1][ks];
        if (b + 2 < EX_NB) load_block(b + 2, bfr[b & 1]);                 // two blocks ahead of the one being multiplied
#pragma unroll
        for (int tb = 0; tb < 2; ++tb) {
            // accumulator of (token 32w + 16tb + lm, columns 16b + 4kg .. +3): 8 bytes of the tile
            const int u = wave * 32 + tb * 16 + lm;
            const int chunk = 2 * b + (kg >> 1);
            char *cell = lds + u * 256 + ((chunk ^ (u & 15)) * 16) + (kg & 1) * 8;
            const u32x2 old = *LDS_PTR(const u32x2, cell);
            f32x4 v;
            v[0] = __uint_as_float(old.x << 16); v[1] = __uint_as_float(old.x & 0xffff0000u);
            v[2] = __uint_as_float(old.y << 16); v[3] = __uint_as_float(old.y & 0xffff0000u);
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
                if (ks < ksteps) v = __builtin_amdgcn_mfma_f32_16x16x32_bf16(cur[ks], sf[tb][ks], v, 0, 0, 0);
            u32x2 nu;
            nu.x = ex_pack_bf16x2(v[0], v[1]);
            nu.y = ex_pack_bf16x2(v[2], v[3]);
            *LDS_PTR(u32x2, cell) = nu;
        }
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");                  // the wave's own writes, before it reads them back
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const u32x4 v = *LDS_PTR(const u32x4, lds + (wave * 8 + j) * 1024 + lane * 16);
        if (ok[j]) *reinterpret_cast<u32x4 *>(Crow0 + goff[j]) = v;
    }
}

hipError_t launch_expand_bf16(const MetaView &mv, const MetaHeader &h, void *C, int64_t N, const void *side, const void *opT,
                              int64_t table_rows, const void *zero, hipStream_t st)
{
    if (h.n_blocks == 0) return hipSuccess;
    const unsigned tiles_n = (unsigned)((N + EX_COLS - 1) / EX_COLS);
    if (tiles_n > 65535u) return hipErrorInvalidValue;                   // N <= 2^22 keeps it at 32768
    hipLaunchKernelGGL(k_expand, dim3((unsigned)h.n_blocks, tiles_n), dim3(64 * EX_NW), 0, st, mv, static_cast<uint16_t *>(C),
                       (int)N, static_cast<const uint16_t *>(side), static_cast<const uint16_t *>(opT), table_rows,
                       static_cast<const uint16_t *>(zero));
    return hipGetLastError();
}

}  // namespace plora
