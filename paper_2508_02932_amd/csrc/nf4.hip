// Dequantisation of a base weight stored as 4-bit NormalFloat (NF4, the storage QLoRA publishes; the
// paper runs packed LoRA on such a base and notes that the LoRA computation is unchanged).
//
// Storage: the weight, flat in memory order, in blocks of 64 elements; per block one fp32 constant
// (the block's largest magnitude), per element a 4-bit index into 16 levels in [-1, 1]; two indices
// per byte, the even element in the high half.  value = level[index] * constant, one fp32
// multiplication, rounded to bf16 (nearest even) when the layer runs in bf16.
//
// On this chip the layer's GEMMs are bound by the matrix cores at fine-tuning batch sizes (tens of
// thousands of tokens), not by the bytes of W, so the weight is expanded once per call into the
// caller's workspace by this streaming kernel (4.5 bits read, 16 written per weight: about 1 % of the
// GEMM's time at 32768 tokens) and the fused GEMM runs on it unchanged, instead of spending vector-ALU
// work inside the GEMM's fetch phases, which are its critical path.
#include "plora_internal.h"

namespace plora {

// the 16 levels of the format (fp32)
__constant__ float kNf4Level[16] = {
    -1.0f, -0.6961928009986877f, -0.5250730514526367f, -0.39491748809814453f,
    -0.28444138169288635f, -0.18477343022823334f, -0.09105003625154495f, 0.0f,
    0.07958029955625534f, 0.16093020141124725f, 0.24611230194568634f, 0.33791524171829224f,
    0.44070982933044434f, 0.5626170039176941f, 0.7229568362236023f, 1.0f};

__device__ inline uint32_t nf4_pack_bf16x2(float lo, float hi)
{
    typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
    typedef float v2f __attribute__((ext_vector_type(2)));
    const v2f f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, v2bf));
}

// One thread per group of 8 elements (4 bytes of indices): a wave reads 256 contiguous bytes of indices and
// writes 1 KB (bf16) or 2 KB (fp32) of contiguous output.  8 groups share a block constant.
template <bool BF16>
__global__ void __launch_bounds__(256) k_nf4_dequant(const uint32_t *__restrict__ codes, const float *__restrict__ absmax,
                                                     void *__restrict__ out, int64_t n_groups)
{
    __shared__ float level[16];
    if (threadIdx.x < 16) level[threadIdx.x] = kNf4Level[threadIdx.x];
    __syncthreads();
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x; g < n_groups; g += stride) {
        const uint32_t c = codes[g];
        const float s = absmax[g >> 3];
        float v[8];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t b = (c >> (8 * j)) & 0xffu;            // byte j: elements 2j (high half) and 2j + 1 (low half)
            v[2 * j] = level[b >> 4] * s;
            v[2 * j + 1] = level[b & 15u] * s;
        }
        if (BF16) {
            uint4 o;
            o.x = nf4_pack_bf16x2(v[0], v[1]); o.y = nf4_pack_bf16x2(v[2], v[3]);
            o.z = nf4_pack_bf16x2(v[4], v[5]); o.w = nf4_pack_bf16x2(v[6], v[7]);
            static_cast<uint4 *>(out)[g] = o;
        } else {
            static_cast<float4 *>(out)[2 * g] = make_float4(v[0], v[1], v[2], v[3]);
            static_cast<float4 *>(out)[2 * g + 1] = make_float4(v[4], v[5], v[6], v[7]);
        }
    }
}

hipError_t launch_nf4_dequant(const void *codes, const float *absmax, int64_t n_elems, bool bf16, void *out, hipStream_t st)
{
    if (n_elems == 0) return hipSuccess;
    const int64_t n_groups = n_elems / 8;
    hipError_t cu_err = hipSuccess;
    const int n_cu = device_cu_count(&cu_err);
    if (n_cu < 1) return cu_err;
    int64_t blocks = (n_groups + 255) / 256;
    const int64_t cap = (int64_t)n_cu * 16;                      // a few workgroups per compute unit, each looping
    if (blocks > cap) blocks = cap;
    if (bf16) hipLaunchKernelGGL(k_nf4_dequant<true>, dim3((unsigned)blocks), dim3(256), 0, st, static_cast<const uint32_t *>(codes),
                                 absmax, out, n_groups);
    else hipLaunchKernelGGL(k_nf4_dequant<false>, dim3((unsigned)blocks), dim3(256), 0, st, static_cast<const uint32_t *>(codes),
                            absmax, out, n_groups);
    return hipGetLastError();
}

}  // namespace plora
