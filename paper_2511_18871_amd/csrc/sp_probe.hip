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

// What a backward in ONE pass would cost in memory atomics.  A pass that owns key tiles and produces dK, dV
// and dQ together has to add a 64 x 128 fp32 partial of dQ into a [T, Hq, 128] accumulator for every
// (128-key tile, 64-row tile, q head) it visits: 4 bytes per allowed pair and q head.  This kernel does
// nothing but those additions (no-return global_atomic_add_f32, device scope), from 512-thread workgroups
// that each add `steps` tiles: layout 0 = each half-wave covers 128 contiguous bytes of a row (what a
// kernel could arrange through LDS), layout 1 = the lanes scatter as the MFMA accumulator holds dQ^T.
template <int LAYOUT>
__global__ __launch_bounds__(512) void atomic_add_probe_kernel(float* __restrict__ buf, int n_row_tiles, int H,
                                                               int steps, int heads_per_xcd) {
    const int tid = threadIdx.x, w = tid >> 6, l = tid & 63;
    const int x = blockIdx.x & 7, j = blockIdx.x >> 3;      // XCD the block lands on, slot within it
    for (int it = 0; it < steps; ++it) {
        const int head = (x * heads_per_xcd + (j + it) % heads_per_xcd) % H;
        const int rt = (int)(((unsigned)j * 2654435761u + (unsigned)it * 40503u) % (unsigned)n_row_tiles);
        float* base = buf + ((size_t)rt * 64 * H + head) * 128;
        const size_t rs = (size_t)H * 128;
        const float v = 1.0f + it;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            int row, col;
            if (LAYOUT == 0) { row = 8 * w + 2 * (e >> 2) + (l >> 5); col = (l & 31) + 32 * (e & 3); }
            else { row = 32 * (w & 1) + (l & 31); col = 32 * (w >> 1) + 8 * (e >> 2) + 4 * (l >> 5) + (e & 3); }
            __hip_atomic_fetch_add(base + row * rs + col, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

}  // namespace
}  // namespace sp

extern "C" sp_status sp_attn_probe_atomic_add(float* buf, int64_t rows, int32_t heads, int32_t steps, int32_t n_blocks,
                                              int32_t layout, void* stream) {
    if (!buf || rows < 64 || heads < 1 || steps < 1 || n_blocks < 1 || layout < 0 || layout > 1) return SP_ERR_INVALID_ARG;
    const int n_row_tiles = (int)(rows / 64);
    const int hpx = heads >= 8 ? heads / 8 : 1;
    hipStream_t s = (hipStream_t)stream;
    if (layout == 0) hipLaunchKernelGGL(sp::atomic_add_probe_kernel<0>, dim3(n_blocks), dim3(512), 0, s, buf, n_row_tiles, heads, steps, hpx);
    else hipLaunchKernelGGL(sp::atomic_add_probe_kernel<1>, dim3(n_blocks), dim3(512), 0, s, buf, n_row_tiles, heads, steps, hpx);
    return hipGetLastError() == hipSuccess ? SP_OK : SP_ERR_DEVICE;
}

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
