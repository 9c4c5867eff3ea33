// Rotary position embedding with the shared-prompt position indices (Section 4.3,
// modification 2): the prompt keeps positions 0 .. Lp-1 and every response starts again at Lp,
// so a response token is rotated as it would be if [prompt | resp_i] were a sample of its own.
// Half-split form: with theta_i = base^(-2i/d), pair (x_i, x_{i+d/2}) at position p turns by the
// angle p * theta_i.  The rotation is orthogonal; `inverse` turns by the negative angle, which
// maps gradients with respect to rotated q / k back to gradients with respect to q / k.
//
// The kernel is a pure HBM pass (read x, write y).  A thread owns 8 consecutive pair indices of
// one token (two 16-byte loads per head for bf16) and evaluates their 8 angles once: the frequencies
// theta_i come from the host in double precision (a kernel argument), the product p * theta_i is
// formed and reduced to [-pi, pi] in double (positions reach tens of thousands of radians, where an
// fp32 product is already off by 1e-3), and only the reduced angle goes through the fp32 sine and
// cosine.  The same angles then serve every head of the token -- of one tensor, or of q AND k in one
// launch (sp_attn_rope_qk): one table upload, one position lookup and one set of angles for both.
#include "sp_common.hpp"
#include "sp_launch.hpp"
#include <cmath>

namespace sp {
namespace {

template <typename T> struct Vec8;
template <> struct Vec8<__bf16> { typedef bf16x8 type; };
template <> struct Vec8<float> { typedef float type __attribute__((ext_vector_type(8))); };

struct RopeFreq { double theta[64]; };      // theta_i = base^(-2 i / d), i < d / 2 <= 64

template <typename T>
__global__ __launch_bounds__(256) void rope_kernel(const T* __restrict__ x, T* __restrict__ y, int H,
                                                   const T* __restrict__ x2, T* __restrict__ y2, int H2,
                                                   const int* __restrict__ tab, int d, RopeFreq f, int inverse) {
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
        const double ang = (double)pos * f.theta[i0 + e];
        const double red = ang - 6.283185307179586476925 * rint(ang * 0.15915494309189533577);   // into [-pi, pi]
        float sv, cv;
        sincosf((float)red, &sv, &cv);
        c[e] = cv;
        s[e] = inverse ? -sv : sv;
    }
    auto rotate = [&](const T* __restrict__ xin, T* __restrict__ yout, int heads) {
        const T* xr = xin + tok * (int64_t)heads * d + i0;
        T* yr = yout + tok * (int64_t)heads * d + i0;
        for (int h = 0; h < heads; ++h) {
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
    };
    rotate(x, y, H);
    if (x2) rotate(x2, y2, H2);
}

}  // namespace

hipError_t launch_rope(const void* x, void* y, int H, const void* x2, void* y2, int H2, const int* tab,
                       int64_t total_tokens, int d, double base, bool inverse, bool f32, hipStream_t s) {
    const int tpt = d / 16;
    const int64_t threads = total_tokens * tpt;
    const int grid = (int)((threads + 255) / 256);
    RopeFreq f{};
    for (int i = 0; i < d / 2; ++i) f.theta[i] = pow(base, -2.0 * (double)i / (double)d);
    if (f32)
        hipLaunchKernelGGL(rope_kernel<float>, dim3(grid), dim3(256), 0, s, (const float*)x, (float*)y, H,
                           (const float*)x2, (float*)y2, H2, tab, d, f, (int)inverse);
    else
        hipLaunchKernelGGL(rope_kernel<__bf16>, dim3(grid), dim3(256), 0, s, (const __bf16*)x, (__bf16*)y, H,
                           (const __bf16*)x2, (__bf16*)y2, H2, tab, d, f, (int)inverse);
    return hipGetLastError();
}

}  // namespace sp
