// Response-token loss on the packed sequence (Section 4.3, modification 4: the loss is taken over
// the response tokens only, prompt rows are discarded; Section 2: the GRPO objective
// J = 1/(NG) sum_k (L_k - beta D_KL^k)).
//
//  logprob_fwd  logp[t] = z[t, y_t] - log sum_v exp z[t, v]  for response rows t; prompt rows are
//               neither read nor written.  One workgroup per row, one pass over the row with a
//               running (max, sum) per thread: a pure HBM read of T_resp * V elements.
//  logprob_bwd  dz[t, v] = g_t (1[v = y_t] - exp(z[t, v] - lse_t)); reads z, writes dz.
//  grpo         per response k (one wave): J_k = 1/|o_k| sum_t (min(r A, clip(r) A) - beta kl),
//               r = exp(logp - logp_old), kl = exp(u) - u - 1 with u = logp_ref - logp; writes
//               g[t] = dloss/dlogp[t] and J_k; a single workgroup then sums the J_k in a fixed
//               order (bitwise repeatable) into loss = -1/R sum_k J_k.
#include "sp_common.hpp"
#include "sp_launch.hpp"

namespace sp {
namespace {

template <typename T> struct Ld;
template <> struct Ld<__bf16> { typedef bf16x8 vec; static constexpr int N = 8; };
template <> struct Ld<float> { typedef f32x4 vec; static constexpr int N = 4; };

// (max, sum of exp(x - max)) merge
__device__ __forceinline__ void ms_merge(float& m, float& s, float m2, float s2) {
    const float mn = fmaxf(m, m2);
    if (mn == -INFINITY) { m = mn; s = 0.f; return; }
    s = s * __expf(m - mn) + s2 * __expf(m2 - mn);
    m = mn;
}

__device__ __forceinline__ void block_lse(float& m, float& s, float* sh) {
    for (int o = 32; o >= 1; o >>= 1) {
        const float m2 = __shfl_xor(m, o, 64), s2 = __shfl_xor(s, o, 64);
        ms_merge(m, s, m2, s2);
    }
    const int w = threadIdx.x >> 6, l = threadIdx.x & 63;
    if (l == 0) { sh[2 * w] = m; sh[2 * w + 1] = s; }
    __syncthreads();
    m = sh[0]; s = sh[1];
    for (int i = 1; i < (int)(blockDim.x >> 6); ++i) ms_merge(m, s, sh[2 * i], sh[2 * i + 1]);
}

template <typename T>
__global__ __launch_bounds__(256) void logprob_fwd_kernel(const T* __restrict__ z, const int* __restrict__ y,
                                                          float* __restrict__ logp, float* __restrict__ lse,
                                                          const int* __restrict__ tab, int64_t V) {
    __shared__ float sh[8];
    const int64_t tok = blockIdx.x;
    const GroupDesc gd = load_group(tab, find_group_of_token(tab, tok));
    if (tok - gd.tok_base < gd.Lp) return;              // prompt row: discarded
    const T* row = z + tok * V;
    float m = -INFINITY, s = 0.f;
    constexpr int N = Ld<T>::N;
    if (V % N == 0) {
        typedef typename Ld<T>::vec Vec;
        const Vec* rv = reinterpret_cast<const Vec*>(row);
        for (int64_t i = threadIdx.x; i < V / N; i += 256) {
            const Vec x = rv[i];
            float mx = (float)x[0];
#pragma unroll
            for (int e = 1; e < N; ++e) mx = fmaxf(mx, (float)x[e]);
            const float mn = fmaxf(m, mx);
            float acc = 0.f;
#pragma unroll
            for (int e = 0; e < N; ++e) acc += __expf((float)x[e] - mn);
            s = s * __expf(m - mn) + acc;
            m = mn;
        }
    } else {
        for (int64_t i = threadIdx.x; i < V; i += 256) {
            const float x = (float)row[i];
            const float mn = fmaxf(m, x);
            s = s * __expf(m - mn) + __expf(x - mn);
            m = mn;
        }
    }
    block_lse(m, s, sh);
    if (threadIdx.x == 0) {
        const float L = m + __logf(s);
        const int label = y[tok];
        lse[tok] = L;
        logp[tok] = (label >= 0 && label < V) ? (float)row[label] - L : -INFINITY;
    }
}

template <typename T>
__global__ __launch_bounds__(256) void logprob_bwd_kernel(const T* __restrict__ z, const int* __restrict__ y,
                                                          const float* __restrict__ lse, const float* __restrict__ g,
                                                          T* __restrict__ dz, const int* __restrict__ tab, int64_t V) {
    const int64_t tok = blockIdx.x;
    const GroupDesc gd = load_group(tab, find_group_of_token(tab, tok));
    if (tok - gd.tok_base < gd.Lp) return;
    const T* row = z + tok * V;
    T* out = dz + tok * V;
    const float L = lse[tok], gt = g[tok];
    const int64_t label = y[tok];
    constexpr int N = Ld<T>::N;
    if (V % N == 0) {
        typedef typename Ld<T>::vec Vec;
        const Vec* rv = reinterpret_cast<const Vec*>(row);
        Vec* ov = reinterpret_cast<Vec*>(out);
        for (int64_t i = threadIdx.x; i < V / N; i += 256) {
            const Vec x = rv[i];
            Vec d;
#pragma unroll
            for (int e = 0; e < N; ++e)
                d[e] = (T)(gt * ((i * N + e == label ? 1.f : 0.f) - __expf((float)x[e] - L)));
            ov[i] = d;
        }
    } else {
        for (int64_t i = threadIdx.x; i < V; i += 256)
            out[i] = (T)(gt * ((i == label ? 1.f : 0.f) - __expf((float)row[i] - L)));
    }
}

// one wave per response (global index k over all groups)
__global__ __launch_bounds__(256) void grpo_kernel(const float* __restrict__ logp, const float* __restrict__ old,
                                                   const float* __restrict__ ref, const float* __restrict__ adv,
                                                   float* __restrict__ g, float* __restrict__ J,
                                                   const int* __restrict__ tab, int n_resp, float eps_low,
                                                   float eps_high, float beta, float inv_R) {
    const int k = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int l = threadIdx.x & 63;
    if (k >= n_resp) return;
    // Group that holds response k.  Group g's response offsets start at table word e[3] = base + R_g + g,
    // with base the first offset word and R_g the responses in earlier groups, so R_g is read off the
    // group entries and the group is the last one with R_g <= k: a bisection (responses of empty groups
    // never match, since R_g of the next group is the same).
    const int ng = tab[0];
    const int base = TAB_HEADER + TAB_GROUP_WORDS * ng;
    int lo = 0, hi = ng;                                 // invariant: R_lo <= k, (hi == ng or R_hi > k)
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (tab[TAB_HEADER + TAB_GROUP_WORDS * mid + 3] - base - mid <= k) lo = mid; else hi = mid;
    }
    const GroupDesc gd = load_group(tab, lo);
    const int i = k - (tab[TAB_HEADER + TAB_GROUP_WORDS * lo + 3] - base - lo);
    const int b = gd.roff[i], e = gd.roff[i + 1];       // group-local token range of the response
    const float a = adv[k];
    const float inv_len = e > b ? 1.0f / (float)(e - b) : 0.f;
    float acc = 0.f;
    for (int t = b + l; t < e; t += 64) {
        const int64_t tok = (int64_t)gd.tok_base + t;
        const float lp = logp[tok];
        const float r = __expf(lp - old[tok]);
        const float un = r * a, cl = fminf(fmaxf(r, 1.0f - eps_low), 1.0f + eps_high) * a;
        const bool inside = r > 1.0f - eps_low && r < 1.0f + eps_high;
        const float surr = fminf(un, cl);
        const float d_surr = (un <= cl || inside) ? un : 0.f;      // d(r a)/dlogp = r a
        const float u = ref[tok] - lp;
        const float eu = __expf(u);
        acc += surr - beta * (eu - u - 1.0f);
        g[tok] = -inv_len * inv_R * (d_surr - beta * (1.0f - eu));
    }
    for (int o = 32; o >= 1; o >>= 1) acc += __shfl_xor(acc, o, 64);
    if (l == 0) J[k] = acc * inv_len;
}

// fixed-order sum of J[0..n) by one workgroup: thread i adds J[i], J[i+256], ... then a tree
__global__ __launch_bounds__(256) void grpo_reduce_kernel(const float* __restrict__ J, int n, float inv_R,
                                                          float* __restrict__ loss) {
    __shared__ float sh[256];
    float acc = 0.f;
    for (int i = threadIdx.x; i < n; i += 256) acc += J[i];
    sh[threadIdx.x] = acc;
    __syncthreads();
    for (int o = 128; o >= 1; o >>= 1) {
        if ((int)threadIdx.x < o) sh[threadIdx.x] += sh[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) loss[0] = -sh[0] * inv_R;
}

}  // namespace

hipError_t launch_logprob_fwd(const void* z, const int* y, float* logp, float* lse, const int* tab,
                              int64_t total_tokens, int64_t V, bool f32, hipStream_t s) {
    if (f32) hipLaunchKernelGGL(logprob_fwd_kernel<float>, dim3((unsigned)total_tokens), dim3(256), 0, s,
                                (const float*)z, y, logp, lse, tab, V);
    else hipLaunchKernelGGL(logprob_fwd_kernel<__bf16>, dim3((unsigned)total_tokens), dim3(256), 0, s,
                            (const __bf16*)z, y, logp, lse, tab, V);
    return hipGetLastError();
}

hipError_t launch_logprob_bwd(const void* z, const int* y, const float* lse, const float* g, void* dz,
                              const int* tab, int64_t total_tokens, int64_t V, bool f32, hipStream_t s) {
    if (f32) hipLaunchKernelGGL(logprob_bwd_kernel<float>, dim3((unsigned)total_tokens), dim3(256), 0, s,
                                (const float*)z, y, lse, g, (float*)dz, tab, V);
    else hipLaunchKernelGGL(logprob_bwd_kernel<__bf16>, dim3((unsigned)total_tokens), dim3(256), 0, s,
                            (const __bf16*)z, y, lse, g, (__bf16*)dz, tab, V);
    return hipGetLastError();
}

hipError_t launch_grpo(const float* logp, const float* old, const float* ref, const float* adv, float* g,
                       float* J, float* loss, const int* tab, int n_resp, int n_nonempty, float eps_low,
                       float eps_high, float beta, hipStream_t s) {
    const float inv_R = n_nonempty > 0 ? 1.0f / (float)n_nonempty : 0.f;
    if (n_resp > 0)
        hipLaunchKernelGGL(grpo_kernel, dim3((n_resp + 3) / 4), dim3(256), 0, s, logp, old, ref, adv, g, J, tab, n_resp,
                           eps_low, eps_high, beta, inv_R);
    hipLaunchKernelGGL(grpo_reduce_kernel, dim3(1), dim3(256), 0, s, J, n_resp, inv_R, loss);
    return hipGetLastError();
}

}  // namespace sp
