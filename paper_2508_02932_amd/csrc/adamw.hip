// Per-adapter AdamW step over all A_k and B_k of a packed multi-LoRA layer (gfx950).
//
// Packed LoRA fine-tuning keeps the adapters independent: each has its own parameters, optimizer
// state and learning rate (section 2.4; appendix B counts gradient, momentum and velocity per
// adapter for AdamW; Table 1 lists the learning rate among the per-job knobs).  The rule is the
// published AdamW, in the order the common frameworks apply it:
//     g <- grad_scale g  (the adapter's own factor: its loss normalisation or clipping coefficient)
//     theta <- theta (1 - lr wd);  m <- b1 m + (1 - b1) g;  v <- b2 v + (1 - b2) g^2;
//     theta <- theta - lr (m / (1 - b1^t)) / (sqrt(v / (1 - b2^t)) + eps)
// One launch updates up to kAdamwTensors tensors of different sizes and hyperparameters ("multi-
// tensor"): the job table travels as a kernel argument, a workgroup handles 2048 consecutive
// elements of one tensor.  Pure streaming: 16 bytes read and 12 to 16 written per element, so the
// kernel is bound by HBM.  Arithmetic in fp32; the fp32 master copy is the parameter, the copy in
// the layer's I/O type is rewritten from it (round to nearest even for bf16).
#include "plora_internal.h"

namespace plora {

constexpr int kAdamwTensors = 40;          // jobs per launch: 40 x 80 bytes fit a kernel argument
constexpr int kAdamwChunk = 2048;          // elements per workgroup

struct AdamwJob {
    void *param;            // I/O dtype copy (may be null when the master copy is all there is)
    float *master;          // fp32 parameters (null: fp32 param is updated in place)
    const float *grad;
    float *m, *v;
    uint32_t numel, chunk0; // chunk0 = index of this tensor's first workgroup in the launch
    float lr, beta1, beta2, eps, decay, c1, c2;   // decay = 1 - lr wd; c1 = 1 / (1 - beta1^t); c2 = 1 / (1 - beta2^t)
    float gscale;           // multiplier on the gradient
};
struct AdamwBatch {
    int32_t n, pad;
    AdamwJob job[kAdamwTensors];
};
static_assert(sizeof(AdamwBatch) <= 3584, "the job table must fit a kernel argument");

__device__ inline uint32_t adamw_pack_bf16x2(float lo, float hi)
{
    typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
    typedef float v2f __attribute__((ext_vector_type(2)));
    const v2f f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, v2bf));
}

__device__ inline float adamw_one(float &th, float g, float &m, float &v, const AdamwJob &j)
{
    g = j.gscale * g;
    th = th * j.decay;
    m = j.beta1 * m + (1.0f - j.beta1) * g;
    v = j.beta2 * v + (1.0f - j.beta2) * g * g;
    th = th - j.lr * (m * j.c1) / (sqrtf(v * j.c2) + j.eps);
    return th;
}

template <bool BF16>
__global__ void __launch_bounds__(256) k_adamw(AdamwBatch b)
{
    // the tensor of this workgroup: the last job whose first chunk is at or before blockIdx.x
    int t = 0;
    for (int q = 1; q < b.n; ++q)
        if (b.job[q].chunk0 <= blockIdx.x) t = q;
    const AdamwJob j = b.job[t];
    const uint32_t e0 = (blockIdx.x - j.chunk0) * kAdamwChunk;
    const uint32_t n = j.numel - e0 < (uint32_t)kAdamwChunk ? j.numel - e0 : (uint32_t)kAdamwChunk;
    float *th = j.master ? j.master + e0 : static_cast<float *>(j.param) + e0;
    const float *g = j.grad + e0;
    float *m = j.m + e0, *v = j.v + e0;
    const bool write_copy = j.master != nullptr && j.param != nullptr;
    for (uint32_t i = threadIdx.x * 4; i < n; i += 256 * 4) {
        if (i + 4 <= n) {
            float4 tv = *reinterpret_cast<const float4 *>(th + i);
            const float4 gv = *reinterpret_cast<const float4 *>(g + i);
            float4 mv = *reinterpret_cast<const float4 *>(m + i);
            float4 vv = *reinterpret_cast<const float4 *>(v + i);
            adamw_one(tv.x, gv.x, mv.x, vv.x, j);
            adamw_one(tv.y, gv.y, mv.y, vv.y, j);
            adamw_one(tv.z, gv.z, mv.z, vv.z, j);
            adamw_one(tv.w, gv.w, mv.w, vv.w, j);
            *reinterpret_cast<float4 *>(th + i) = tv;
            *reinterpret_cast<float4 *>(m + i) = mv;
            *reinterpret_cast<float4 *>(v + i) = vv;
            if (write_copy) {
                if (BF16) {
                    uint2 p;
                    p.x = adamw_pack_bf16x2(tv.x, tv.y);
                    p.y = adamw_pack_bf16x2(tv.z, tv.w);
                    *reinterpret_cast<uint2 *>(static_cast<uint16_t *>(j.param) + e0 + i) = p;
                } else {
                    *reinterpret_cast<float4 *>(static_cast<float *>(j.param) + e0 + i) = tv;
                }
            }
        } else {
            for (uint32_t q = i; q < n; ++q) {       // tail of a tensor whose size is no multiple of 4 (fp32 I/O only)
                float tq = th[q], mq = m[q], vq = v[q];
                adamw_one(tq, g[q], mq, vq, j);
                th[q] = tq; m[q] = mq; v[q] = vq;
                if (write_copy) {
                    if (BF16) static_cast<uint16_t *>(j.param)[e0 + q] = (uint16_t)(adamw_pack_bf16x2(tq, 0.f) & 0xffffu);
                    else static_cast<float *>(j.param)[e0 + q] = tq;
                }
            }
        }
    }
}

hipError_t launch_adamw(const AdamwTensor *t, int n, bool bf16, hipStream_t st)
{
    for (int i0 = 0; i0 < n; i0 += kAdamwTensors) {
        AdamwBatch b;
        b.n = 0; b.pad = 0;
        uint32_t chunks = 0;
        for (int i = i0; i < n && b.n < kAdamwTensors; ++i) {
            if (t[i].numel == 0) continue;
            AdamwJob &j = b.job[b.n++];
            j.param = t[i].param; j.master = t[i].master; j.grad = t[i].grad; j.m = t[i].m; j.v = t[i].v;
            j.numel = (uint32_t)t[i].numel; j.chunk0 = chunks;
            chunks += (uint32_t)((t[i].numel + kAdamwChunk - 1) / kAdamwChunk);
            j.lr = t[i].lr; j.beta1 = t[i].beta1; j.beta2 = t[i].beta2; j.eps = t[i].eps;
            j.decay = (float)(1.0 - (double)t[i].lr * (double)t[i].weight_decay);
            // bias corrections in double on the host: beta^t for large t is exactly what fp32 would get wrong
            double p1 = 1.0, p2 = 1.0;
            for (int s = 0; s < t[i].step && (p1 > 0.0 || p2 > 0.0); ++s) { p1 *= (double)t[i].beta1; p2 *= (double)t[i].beta2; }
            j.c1 = (float)(1.0 / (1.0 - p1));
            j.c2 = (float)(1.0 / (1.0 - p2));
            j.gscale = t[i].grad_scale;
        }
        if (chunks == 0) continue;
        if (bf16) hipLaunchKernelGGL(k_adamw<true>, dim3(chunks), dim3(256), 0, st, b);
        else hipLaunchKernelGGL(k_adamw<false>, dim3(chunks), dim3(256), 0, st, b);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace plora
