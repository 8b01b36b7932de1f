// fp32 I/O path of the packed multi-LoRA layer.  Inputs and outputs are fp32; every sum is
// accumulated in fp64 on the vector ALU (full-rate fp64 FMA on this chip) and rounded once, so the
// result is within an ulp or two of the exact value for any problem size.  This path exists for
// the small fp32 configuration, which is launch-latency bound; the kernels are tiled through LDS
// but not tuned further.
#include "plora_internal.h"

namespace plora {

// Segment that holds row t (segments are few; a scan is cheaper than a table lookup).
__device__ inline int seg_of_row(const MetaView &mv, int t)
{
    const int n = mv.hdr->n_seg;
    for (int s = 0; s < n; ++s)
        if (t >= mv.seg[s].row0 && t < mv.seg[s].row1) return s;
    return -1;
}

// mode 0: out[t][j] = sum_c x[t][c] A_k[c][j]              (low-rank activation h, unscaled)
// mode 1: out[t][j] = scale_k sum_c dy[t][c] B_k[j][c]     (gradient case 2)
// One block per token block of kSkinnyRows rows; out is the ragged [len][r] fp32 layout.
__global__ void __launch_bounds__(256) k_f32_lowrank(MetaView mv, int mode, const float *S, int64_t C, float *out)
{
    const int blk = blockIdx.x;
    const int n_seg = mv.hdr->n_seg;
    int s = 0;
    for (int q = 0; q < n_seg; ++q) {
        const SegInfo g = mv.seg[q];
        if (g.adapter >= 0 && g.row1 > g.row0 && blk >= g.blk0) s = q;
    }
    const SegInfo g = mv.seg[s];
    const AdapterInfo a = mv.ad[g.adapter];
    const int t0 = (blk - g.blk0) * kSkinnyRows;
    const int len = g.row1 - g.row0;
    const int nt = (len - t0 < kSkinnyRows) ? len - t0 : kSkinnyRows;
    const int r = g.r;
    const float *M = static_cast<const float *>(mode == 0 ? a.A : a.B);
    for (int e = threadIdx.x; e < nt * r; e += 256) {
        const int tt = e / r, j = e % r;
        const float *srow = S + (int64_t)(g.row0 + t0 + tt) * C;
        double acc = 0.0;
        if (mode == 0) {
            for (int64_t c = 0; c < C; ++c) acc += (double)srow[c] * (double)M[c * r + j];
        } else {
            const float *brow = M + (int64_t)j * C;
            for (int64_t c = 0; c < C; ++c) acc += (double)srow[c] * (double)brow[c];
            acc *= (double)a.scale;
        }
        out[g.h_off + (int64_t)(t0 + tt) * r + j] = (float)acc;
    }
}

hipError_t launch_f32_lowrank(const MetaView &mv, const MetaHeader &h, int mode, const float *S, int64_t C,
                              float *out, hipStream_t st)
{
    if (h.n_blocks == 0) return hipSuccess;
    hipLaunchKernelGGL(k_f32_lowrank, dim3((unsigned)h.n_blocks), dim3(256), 0, st, mv, mode, S, C, out);
    return hipGetLastError();
}

// forward : C[t][n] = sum_i x[t][i]  W[i][n] + scale_k sum_j h[t][j] B_k[j][n]
// backward: C[t][i] = sum_n dy[t][n] W[i][n] +         sum_j g[t][j] A_k[i][j]     (g carries scale_k)
// 64x64 output tile per block, 4x4 outputs per thread, contraction staged through LDS 16 at a time.
// WK: the contraction index is W's row index (forward with W [d_in][d_out], backward with W [d_out][d_in]).
template <bool FWD, bool WK>
__global__ void __launch_bounds__(256) k_f32_gemm(MetaView mv, const float *S, const float *W, const float *side, float *Cout, int accumulate)
{
    __shared__ float sA[16][64 + 1];   // [kk][row]
    __shared__ float sB[16][64 + 1];   // [kk][col]
    const int64_t T = mv.hdr->T;
    const int64_t Kd = FWD ? mv.hdr->D : mv.hdr->K;   // contraction length
    const int64_t N = FWD ? mv.hdr->K : mv.hdr->D;    // output columns
    const int64_t ldw = WK ? N : Kd;                  // W is [Kd][N] or [N][Kd]
    const int64_t m0 = (int64_t)blockIdx.y * 64, n0 = (int64_t)blockIdx.x * 64;
    const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
    double acc[4][4];
    for (int i = 0; i < 4; ++i) for (int j = 0; j < 4; ++j) acc[i][j] = 0.0;

    for (int64_t k0 = 0; k0 < Kd; k0 += 16) {
        for (int e = threadIdx.x; e < 16 * 64; e += 256) {
            const int kk = e % 16, rr = e / 16;
            const int64_t t = m0 + rr, k = k0 + kk;
            sA[kk][rr] = (t < T && k < Kd) ? S[t * Kd + k] : 0.f;
        }
        for (int e = threadIdx.x; e < 16 * 64; e += 256) {
            int kk, cc;
            if (WK) { cc = e % 64; kk = e / 64; } else { kk = e % 16; cc = e / 16; }
            const int64_t k = k0 + kk, n = n0 + cc;
            float v = 0.f;
            if (k < Kd && n < N) v = WK ? W[k * ldw + n] : W[n * ldw + k];
            sB[kk][cc] = v;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            double a[4], b[4];
            for (int i = 0; i < 4; ++i) a[i] = (double)sA[kk][ty * 4 + i];
            for (int j = 0; j < 4; ++j) b[j] = (double)sB[kk][tx + 16 * j];
            for (int i = 0; i < 4; ++i) for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
        }
        __syncthreads();
    }

    for (int i = 0; i < 4; ++i) {
        const int64_t t = m0 + ty * 4 + i;
        if (t >= T) continue;
        const int s = seg_of_row(mv, (int)t);
        const SegInfo g = mv.seg[s];
        for (int j = 0; j < 4; ++j) {
            const int64_t n = n0 + tx + 16 * j;
            if (n >= N) continue;
            double v = acc[i][j];
            if (g.adapter >= 0) {
                const AdapterInfo a = mv.ad[g.adapter];
                const float *hrow = side + g.h_off + (int64_t)(t - g.row0) * g.r;
                double l = 0.0;
                if (FWD) {
                    const float *Bk = static_cast<const float *>(a.B);
                    for (int q = 0; q < g.r; ++q) l += (double)hrow[q] * (double)Bk[(int64_t)q * N + n];
                    l *= (double)a.scale;
                } else {
                    const float *Ak = static_cast<const float *>(a.A);
                    for (int q = 0; q < g.r; ++q) l += (double)hrow[q] * (double)Ak[n * g.r + q];
                }
                v += l;
            }
            if (accumulate) v += (double)Cout[t * N + n];
            Cout[t * N + n] = (float)v;
        }
    }
}

// Stand-alone low-rank update: C[t][n] += mult * sum_j side[t][j] * op_k(j, n)   (fp64 accumulation)
//   to_y : side = h (unscaled), op_k = B_k [r][N], mult = scale_k;   else side = g (carries scale_k), op_k = A_k^T, A_k [N][r]
template <bool TO_Y>
__global__ void __launch_bounds__(256) k_f32_expand(MetaView mv, float *C, int64_t N, const float *side)
{
    const int64_t t = (int64_t)blockIdx.x * 2 + threadIdx.x / 128;
    const int64_t n = (int64_t)blockIdx.y * 128 + threadIdx.x % 128;
    if (t >= mv.hdr->T || n >= N) return;
    const int s = seg_of_row(mv, (int)t);
    const SegInfo g = mv.seg[s];
    if (g.adapter < 0) return;
    const AdapterInfo a = mv.ad[g.adapter];
    const float *row = side + g.h_off + (int64_t)(t - g.row0) * g.r;
    double l = 0.0;
    if (TO_Y) {
        const float *Bk = static_cast<const float *>(a.B);
        for (int q = 0; q < g.r; ++q) l += (double)row[q] * (double)Bk[(int64_t)q * N + n];
        l *= (double)a.scale;
    } else {
        const float *Ak = static_cast<const float *>(a.A);
        for (int q = 0; q < g.r; ++q) l += (double)row[q] * (double)Ak[n * g.r + q];
    }
    C[t * N + n] = (float)((double)C[t * N + n] + l);
}

hipError_t launch_f32_expand(const MetaView &mv, const MetaHeader &h, bool to_y, float *C, const float *side, hipStream_t st)
{
    if (h.T == 0 || h.n_blocks == 0) return hipSuccess;
    const int64_t N = to_y ? h.K : h.D;
    dim3 grid((unsigned)((h.T + 1) / 2), (unsigned)((N + 127) / 128));     // N <= 2^22: at most 32768 in y
    if (to_y) hipLaunchKernelGGL(k_f32_expand<true>, grid, dim3(256), 0, st, mv, C, N, side);
    else hipLaunchKernelGGL(k_f32_expand<false>, grid, dim3(256), 0, st, mv, C, N, side);
    return hipGetLastError();
}

hipError_t launch_f32_gemm(const MetaView &mv, const MetaHeader &h, bool forward, const float *S, const float *W,
                           const float *side, float *C, bool accumulate, hipStream_t st)
{
    if (h.T == 0) return hipSuccess;
    const int acc = accumulate ? 1 : 0;
    const int64_t N = forward ? h.K : h.D;
    dim3 grid((unsigned)((N + 63) / 64), (unsigned)((h.T + 63) / 64));
    const bool wk = forward != (h.w_out_in != 0);
    if (forward && wk) hipLaunchKernelGGL((k_f32_gemm<true, true>), grid, dim3(256), 0, st, mv, S, W, side, C, acc);
    else if (forward) hipLaunchKernelGGL((k_f32_gemm<true, false>), grid, dim3(256), 0, st, mv, S, W, side, C, acc);
    else if (wk) hipLaunchKernelGGL((k_f32_gemm<false, true>), grid, dim3(256), 0, st, mv, S, W, side, C, acc);
    else hipLaunchKernelGGL((k_f32_gemm<false, false>), grid, dim3(256), 0, st, mv, S, W, side, C, acc);
    return hipGetLastError();
}

// want_dA: dA_k[c][j] = sum_t x[t][c]  g[t][j]                (case 3; g carries scale_k)
// else   : dB_k[j][c] = scale_k sum_t h[t][j] dy[t][c]        (case 1)
// summed over every segment of adapter k.  Block (x: 64 columns c, y: adapter).
__global__ void __launch_bounds__(256) k_f32_wgrad(MetaView mv, int want_dA, const float *S, int64_t C, const float *side)
{
    const int k = blockIdx.y;
    const AdapterInfo a = mv.ad[k];
    const int r = a.r;
    const int64_t c0 = (int64_t)blockIdx.x * 64;
    const int n_seg = mv.hdr->n_seg;
    for (int e = threadIdx.x; e < 64 * r; e += 256) {
        const int cc = e % 64, j = e / 64;
        const int64_t c = c0 + cc;
        if (c >= C) continue;
        double acc = 0.0;
        for (int s = 0; s < n_seg; ++s) {
            const SegInfo g = mv.seg[s];
            if (g.adapter != k) continue;
            for (int t = g.row0; t < g.row1; ++t)
                acc += (double)S[(int64_t)t * C + c] * (double)side[g.h_off + (int64_t)(t - g.row0) * r + j];
        }
        if (want_dA) a.dA[c * r + j] = (float)acc;
        else a.dB[(int64_t)j * C + c] = (float)(acc * (double)a.scale);
    }
}

hipError_t launch_f32_wgrad(const MetaView &mv, const MetaHeader &h, bool want_dA, const float *S, int64_t C,
                            const float *side, hipStream_t st)
{
    if (h.n_adapters == 0) return hipSuccess;
    dim3 grid((unsigned)((C + 63) / 64), (unsigned)h.n_adapters);
    hipLaunchKernelGGL(k_f32_wgrad, grid, dim3(256), 0, st, mv, want_dA ? 1 : 0, S, C, side);
    return hipGetLastError();
}

}  // namespace plora
