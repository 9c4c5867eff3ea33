// Rotary position embedding with the shared-prompt position indices (Section 4.3,
// modification 2): the prompt keeps positions 0 .. Lp-1 and every response starts again at Lp,
// so a response token is rotated as it would be if [prompt | resp_i] were a sample of its own.
// Half-split form: with theta_i = base^(-2i/d), pair (x_i, x_{i+d/2}) at position p turns by the
// angle p * theta_i.  The rotation is orthogonal; `inverse` turns by the negative angle, which
// maps gradients with respect to rotated q / k back to gradients with respect to q / k.
//
// The kernel is a pure HBM pass (read x, write y).  A thread owns 8 consecutive pair indices of
// one token (two 16-byte loads per head for bf16), computes their 8 angles once in double
// precision (positions reach tens of thousands of radians, where an fp32 angle is already off by
// 1e-3) and applies them to every head of the token.
#include "sp_common.hpp"
#include "sp_launch.hpp"

namespace sp {
namespace {

template <typename T> struct Vec8;
template <> struct Vec8<__bf16> { typedef bf16x8 type; };
template <> struct Vec8<float> { typedef float type __attribute__((ext_vector_type(8))); };

template <typename T>
__global__ __launch_bounds__(256) void rope_kernel(const T* __restrict__ x, T* __restrict__ y,
                                                   const int* __restrict__ tab, int H, int d,
                                                   double log2_base, int inverse) {
    typedef typename Vec8<T>::type V8;
    const int half = d >> 1;
    const int tpt = half >> 3;                          // threads per token
    const int64_t T_total = tab[1];
    const int64_t tok = ((int64_t)blockIdx.x * 256 + threadIdx.x) / tpt;
    const int i0 = 8 * (int)(((int64_t)blockIdx.x * 256 + threadIdx.x) % tpt);
    if (tok >= T_total) return;
    // group of the token, then its position index
    const int g = find_group_of_token(tab, tok);
    const GroupDesc gd = load_group(tab, g);
    const int t = (int)(tok - gd.tok_base);
    const int pos = t < gd.Lp ? t : gd.Lp + (t - seg_start(gd, t));
    float c[8], s[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const double theta = exp2(-2.0 * (double)(i0 + e) / (double)d * log2_base);
        double sv, cv;
        sincos((double)pos * theta, &sv, &cv);
        c[e] = (float)cv;
        s[e] = (float)(inverse ? -sv : sv);
    }
    const T* xr = x + tok * (int64_t)H * d + i0;
    T* yr = y + tok * (int64_t)H * d + i0;
    for (int h = 0; h < H; ++h) {
        const V8 lo = *reinterpret_cast<const V8*>(xr + (int64_t)h * d);
        const V8 hi = *reinterpret_cast<const V8*>(xr + (int64_t)h * d + half);
        V8 ylo, yhi;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float a = (float)lo[e], b = (float)hi[e];
            ylo[e] = (T)(a * c[e] - b * s[e]);
            yhi[e] = (T)(a * s[e] + b * c[e]);
        }
        *reinterpret_cast<V8*>(yr + (int64_t)h * d) = ylo;
        *reinterpret_cast<V8*>(yr + (int64_t)h * d + half) = yhi;
    }
}

}  // namespace

hipError_t launch_rope(const void* x, void* y, const int* tab, int64_t total_tokens, int H, int d,
                       double base, bool inverse, bool f32, hipStream_t s) {
    const int tpt = d / 16;
    const int64_t threads = total_tokens * tpt;
    const int grid = (int)((threads + 255) / 256);
    const double l2b = log2(base);
    if (f32)
        hipLaunchKernelGGL(rope_kernel<float>, dim3(grid), dim3(256), 0, s, (const float*)x, (float*)y, tab, H, d, l2b,
                           (int)inverse);
    else
        hipLaunchKernelGGL(rope_kernel<__bf16>, dim3(grid), dim3(256), 0, s, (const __bf16*)x, (__bf16*)y, tab, H, d,
                           l2b, (int)inverse);
    return hipGetLastError();
}

}  // namespace sp
