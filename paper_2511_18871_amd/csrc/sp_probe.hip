// Measured ceiling of the bf16 matrix cores on this chip, for the instruction mixes the attention
// kernels use.  Not part of the attention path: bench.py runs it beside the kernels so that their
// rates can be read against what a loop of nothing but v_mfma_f32_32x32x16_bf16 sustains
//   LDS = 0   both operands in registers,
//   LDS = 1   one operand read from LDS per MFMA (16 bytes per lane: the forward and the dq pass),
//   LDS = 2   both operands read from LDS per MFMA (the S / dP products of the dkdv pass),
// on operands the caller supplies (random values make the multipliers toggle as real data does;
// constants show the same loop without that power draw).  One workgroup of eight waves per CU, two
// waves per SIMD, like the attention kernels.
#include "../../include/sp_attn.h"
#include "sp_common.hpp"

namespace sp {
namespace {

constexpr int PROBE_MFMAS_PER_ITER = 16;

template <int LDS>
__global__ __launch_bounds__(512) void mfma_ceiling_kernel(const bf16x8* __restrict__ A, const bf16x8* __restrict__ B,
                                                           float* __restrict__ out, int iters) {
    __shared__ __attribute__((aligned(1024))) char lds[2][8 * 512 * 16];   // [A | B][operand][thread] 16 bytes
    const int tid = threadIdx.x;
    bf16x8 a[8], b[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = A[i * 512 + tid];
        b[i] = B[i * 512 + tid];
        *reinterpret_cast<bf16x8*>(&lds[0][(i * 512 + tid) * 16]) = a[i];
        *reinterpret_cast<bf16x8*>(&lds[1][(i * 512 + tid) * 16]) = b[i];
    }
    __syncthreads();
    f32x16 acc[4];
#pragma unroll
    for (int n = 0; n < 4; ++n)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[n][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
        // the fence makes the compiler read the LDS operands again in every iteration
        asm volatile("" ::: "memory");
#pragma unroll
        for (int u = 0; u < PROBE_MFMAS_PER_ITER; ++u) {
            const bf16x8 x = LDS >= 1 ? *reinterpret_cast<const bf16x8*>(&lds[0][((u % 8) * 512 + tid) * 16]) : a[u % 8];
            const bf16x8 y = LDS >= 2 ? *reinterpret_cast<const bf16x8*>(&lds[1][(((u / 2) % 8) * 512 + tid) * 16]) : b[(u / 2) % 8];
            acc[u % 4] = mfma32(x, y, acc[u % 4]);
        }
    }
    float s = 0.f;
#pragma unroll
    for (int n = 0; n < 4; ++n) s += acc[n][0] + acc[n][7];
    if (blockIdx.x == 0) out[tid] = s;          // keeps the loop alive; 512 floats
}

}  // namespace
}  // namespace sp

extern "C" sp_status sp_attn_mfma_ceiling(int32_t lds_operands, const void* a, const void* b, int32_t iters,
                                          int32_t n_blocks, float* out, void* stream) {
    if (!a || !b || !out || iters < 1 || n_blocks < 1 || lds_operands < 0 || lds_operands > 2 ||
        ((uintptr_t)a & 15) || ((uintptr_t)b & 15))
        return SP_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    const sp::bf16x8* A = (const sp::bf16x8*)a;
    const sp::bf16x8* B = (const sp::bf16x8*)b;
    if (lds_operands == 0) hipLaunchKernelGGL(sp::mfma_ceiling_kernel<0>, dim3(n_blocks), dim3(512), 0, s, A, B, out, iters);
    else if (lds_operands == 1) hipLaunchKernelGGL(sp::mfma_ceiling_kernel<1>, dim3(n_blocks), dim3(512), 0, s, A, B, out, iters);
    else hipLaunchKernelGGL(sp::mfma_ceiling_kernel<2>, dim3(n_blocks), dim3(512), 0, s, A, B, out, iters);
    return hipGetLastError() == hipSuccess ? SP_OK : SP_ERR_DEVICE;
}
