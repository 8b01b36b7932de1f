// Weight gradients of the packed multi-LoRA layer on bf16 inputs (gfx950): the two products that
// contract over the token axis (appendix C.2),
//   case 3   dA_k[c][j] =           sum_t x_t[c]  g_t[j]      (g carries scale_k)
//   case 1   dB_k[j][c] = scale_k * sum_t dy_t[c] h_t[j]
// summed over every segment of adapter k.  Each streams a big [T][C] matrix once (bound by HBM)
// against the small transposed bf16 factor zt[j][t] written by the skinny kernel.
//
// The token index is the slow index of the big matrix, so its MFMA operand needs a transpose; it
// is staged HBM -> LDS as it lies in memory and read with the transposing LDS load
// (ds_read_b64_tr_b16).  The rank stays whole in every tile; tiles are cut along the hidden
// dimension (128 columns per workgroup) and the workgroup walks all tokens of the adapter, so no
// partial sums ever leave the chip and the summation order is fixed.
#include "plora_internal.h"

namespace plora {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T *)(p))
#define GLB_PTR(p) ((const __attribute__((address_space(1))) void *)(p))

constexpr int TC_BC = 128;                 // columns of the big matrix per workgroup
constexpr int TC_BT = 32;                  // tokens per stage (one MFMA K step)
constexpr int TC_NST = 4;                  // LDS stages
constexpr int TC_S_BYTES = TC_BT * TC_BC * 2;             // 8 KB  [32 t][128 c]
constexpr int TC_Z_BYTES = PLORA_MAX_RANK * TC_BT * 2;    // 8 KB  [128 j][32 t]
constexpr int TC_STAGE = TC_S_BYTES + TC_Z_BYTES;
constexpr int TC_LDS = TC_NST * TC_STAGE;                 // 64 KB
constexpr int TC_NB = PLORA_MAX_RANK / 16;

struct TokCursor { int seg; int t; };      // next stage to fetch: segment index, token offset inside it

__device__ inline int next_seg_of(const MetaView &mv, int from, int k)
{
    const int n = mv.hdr->n_seg;
    for (int s = from; s < n; ++s)
        if (mv.seg[s].adapter == k && mv.seg[s].row1 > mv.seg[s].row0) return s;
    return n;
}

template <bool WANT_DA>
__global__ void __launch_bounds__(256) k_tokc(MetaView mv, const uint16_t *__restrict__ S, int C,
                                             const uint16_t *__restrict__ zt, const uint16_t *__restrict__ zero)
{
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    const int k = blockIdx.y;
    const AdapterInfo a = mv.ad[k];
    const int c0 = blockIdx.x * TC_BC;
    const int n_seg = mv.hdr->n_seg;
    const int nb = a.r16 / 16;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

    int n_steps = 0;
    for (int s = next_seg_of(mv, 0, k); s < n_seg; s = next_seg_of(mv, s + 1, k))
        n_steps += (mv.seg[s].row1 - mv.seg[s].row0 + TC_BT - 1) / TC_BT;

    // ---- loader.  Big-matrix tile [32 t][16 chunks]: instruction q covers token rows 4q..4q+3, lane ->
    // (row 4q + lane/16, slot lane%16), slot c' of row u holds chunk c' ^ (2*(u&3) + 8*((u>>3)&1)).
    // Small-factor tile [128 j][4 chunks]: instruction q covers rows 16q..16q+15, lane -> (row 16q +
    // lane/4, slot lane%4), slot c' of row u holds chunk c' ^ ((u>>2)&3).  Every wave issues exactly
    // 2 + 2 loads per stage (rows of the small factor beyond r16 fetch zeros) so that the number of
    // loads in flight per stage is a constant the wait instruction can name.
    TokCursor cur;
    cur.seg = next_seg_of(mv, 0, k);
    cur.t = 0;
    auto issue = [&](int stage) {
        char *ss = lds + stage * TC_STAGE;
        char *sz = ss + TC_S_BYTES;
        const SegInfo g = mv.seg[cur.seg];
        const int len = g.row1 - g.row0;
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
            const int q = wave + 4 * jj;
            const int u = q * 4 + (lane >> 4);
            int chunk = (lane & 15) ^ (2 * (u & 3) + 8 * ((u >> 3) & 1));
            int c = c0 + chunk * 8;
            c = c < C ? c : C - 8;                                  // columns past the end only feed outputs that are not stored
            const int t = cur.t + u;
            const uint16_t *p = (t < len) ? S + (int64_t)(g.row0 + t) * C + c : zero;
            __builtin_amdgcn_global_load_lds(GLB_PTR(p), LDS_PTR(void, ss + q * 1024), 16, 0, 0);
        }
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
            const int q = wave + 4 * jj;
            const int u = q * 16 + (lane >> 2);
            const int chunk = (lane & 3) ^ ((u >> 2) & 3);
            const uint16_t *p = (u < g.r16) ? zt + g.zt_off + (int64_t)u * g.lp + cur.t + chunk * 8 : zero + lane * 8;
            __builtin_amdgcn_global_load_lds(GLB_PTR(p), LDS_PTR(void, sz + q * 1024), 16, 0, 0);
        }
        cur.t += TC_BT;
        if (cur.t >= len) { cur.seg = next_seg_of(mv, cur.seg + 1, k); cur.t = 0; }
    };

    // ---- MFMA operands.  Wave w owns columns 32w..32w+31 (two 16-column blocks) and every rank block.
    // Transposing read of the big-matrix operand: the 16 lanes of group kg fetch the 4(t) x 16(c) block
    // at tokens kg*8 (+4 for the second read), 8 bytes each; lane i then holds column i.
    const int i16 = lane & 15, kg = lane >> 4;
    int soff[2];
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
        const int u = kg * 8 + (i16 >> 2);                            // token row fetched by this lane (first read)
        const int cl = wave * 32 + cb * 16 + (i16 & 3) * 4;           // first column fetched by this lane
        soff[cb] = u * 256 + ((((cl >> 3) ^ (2 * (u & 3) + 8 * ((u >> 3) & 1))) * 16) + (cl & 7) * 2);
    }
    // second read: token row u+4 -> (u&3) and (u>>3)&1 unchanged, plain +4*256
    int zoff[TC_NB];
#pragma unroll
    for (int b = 0; b < TC_NB; ++b) {
        const int u = b * 16 + i16;                                   // rank row j
        zoff[b] = u * 64 + ((kg ^ ((u >> 2) & 3)) * 16);
    }

    f32x4 acc[2][TC_NB];
#pragma unroll
    for (int cb = 0; cb < 2; ++cb)
#pragma unroll
        for (int b = 0; b < TC_NB; ++b) acc[cb][b] = f32x4{0.f, 0.f, 0.f, 0.f};

    for (int p = 0; p < TC_NST - 1; ++p) {
        if (p < n_steps) issue(p);
    }
    for (int it = 0; it < n_steps; ++it) {
        // loads of the stages it+1 .. it+NST-2 may stay in flight: 4 instructions each
        const int ahead = (n_steps - 1 - it < TC_NST - 2) ? n_steps - 1 - it : TC_NST - 2;
        if (ahead >= 2) __builtin_amdgcn_s_waitcnt(0x0f70 | 8);
        else if (ahead == 1) __builtin_amdgcn_s_waitcnt(0x0f70 | 4);
        else __builtin_amdgcn_s_waitcnt(0x0f70);
        __syncthreads();
        if (it + TC_NST - 1 < n_steps) issue((it + TC_NST - 1) % TC_NST);
        const char *ss = lds + (it % TC_NST) * TC_STAGE;
        const char *sz = ss + TC_S_BYTES;
        bf16x8 sf[2];
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
            bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(LDS_PTR(bf16x4, ss + soff[cb]));
            bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(LDS_PTR(bf16x4, ss + soff[cb] + 4 * 256));
            sf[cb] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        }
#pragma unroll
        for (int b = 0; b < TC_NB; ++b) {
            if (b < nb) {
                const bf16x8 zf = *LDS_PTR(const bf16x8, sz + zoff[b]);
#pragma unroll
                for (int cb = 0; cb < 2; ++cb)
                    acc[cb][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(sf[cb], zf, acc[cb][b], 0, 0, 0);
            }
        }
    }

    // ---- epilogue.  Lane holds rank column j = 16b + i16 and big-matrix columns c = cbase + 4*kg + i.
    const float mult = WANT_DA ? 1.f : a.scale;
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
        const int c = c0 + wave * 32 + cb * 16 + kg * 4;
#pragma unroll
        for (int b = 0; b < TC_NB; ++b) {
            const int j = b * 16 + i16;
            if (b < nb && j < a.r && c < C) {
                if (WANT_DA) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) a.dA[(int64_t)(c + i) * a.r + j] = acc[cb][b][i];
                } else {
                    float4 v;
                    v.x = mult * acc[cb][b][0]; v.y = mult * acc[cb][b][1];
                    v.z = mult * acc[cb][b][2]; v.w = mult * acc[cb][b][3];
                    *reinterpret_cast<float4 *>(a.dB + (int64_t)j * C + c) = v;
                }
            }
        }
    }
}

hipError_t launch_tokcontract_bf16(const MetaView &mv, const MetaHeader &h, bool want_dA, const void *S,
                                   int64_t C, const void *zt, const void *zero, hipStream_t st)
{
    if (h.n_adapters == 0) return hipSuccess;
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_tokc<true>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, TC_LDS);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_tokc<false>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, TC_LDS);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    const dim3 grid((unsigned)((C + TC_BC - 1) / TC_BC), (unsigned)h.n_adapters);
    const uint16_t *s16 = static_cast<const uint16_t *>(S), *z16 = static_cast<const uint16_t *>(zt);
    const uint16_t *zero16 = static_cast<const uint16_t *>(zero);
    if (want_dA) hipLaunchKernelGGL(k_tokc<true>, grid, dim3(256), TC_LDS, st, mv, s16, (int)C, z16, zero16);
    else hipLaunchKernelGGL(k_tokc<false>, grid, dim3(256), TC_LDS, st, mv, s16, (int)C, z16, zero16);
    return hipGetLastError();
}

}  // namespace plora
