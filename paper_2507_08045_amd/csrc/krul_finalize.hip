// Row similarity and token-wise aggregation (Sec. 5 / Sec. 7: per-token similarities
// are added up; Sec. 4.2: the average over heads).
//
// finalize_heads: one workgroup per (conversation, pair, query head).  Each thread
// takes query rows t, t+256, ...: it merges the row's partial records of the two
// layers onto a common reference exponent, forms the cosine and (from the
// a^2 + b^2 - 2ab expansion of Sec. 7) the Euclidean distance of the two attention
// rows, and the workgroup sums over rows in a fixed tree order.
// finalize_pairs: one thread per (conversation, pair) averages the heads in order.
#include "krul_common.h"

namespace krul {
namespace {

constexpr int kThreads = 256;

__device__ inline float block_sum(float v, float *red)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    const int w = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[w] = v;
    __syncthreads();
    float s = 0.f;
    for (int i = 0; i < kThreads / 64; ++i) s += red[i];
    return s;
}

__global__ __launch_bounds__(kThreads) void finalize_heads_kernel(
    StateLayout lay, const float4 *__restrict__ state, int L, int Hq, int Hkv, int Tq,
    float *__restrict__ head_cos, float *__restrict__ head_dist)
{
    __shared__ float red[kThreads / 64];
    const int NP = L - 1;
    const int h = blockIdx.x % Hq;
    const int l = (blockIdx.x / Hq) % NP;
    const int b = blockIdx.x / (Hq * NP);
    const int g = Hq / Hkv;
    const int u = b * Hkv + h / g;
    const int P = lay.partials;

    float cos_acc = 0.f, dist_acc = 0.f;
    for (int t = threadIdx.x; t < Tq; t += kThreads) {
        const int r = (h % g) * Tq + t;
        // pass 1: common reference exponents of the two layers
        float Ma = kMInit, Mb = kMInit;
        for (int p = 0; p < P; ++p) {
            Ma = fmaxf(Ma, state[state_index(lay, u, r, p, l)].x);
            Mb = fmaxf(Mb, state[state_index(lay, u, r, p, l + 1)].x);
        }
        // pass 2: rescale and add, partials in index order
        float Za = 0.f, Na = 0.f, Zb = 0.f, Nb = 0.f, C = 0.f;
        for (int p = 0; p < P; ++p) {
            const float4 a = state[state_index(lay, u, r, p, l)];
            const float4 c = state[state_index(lay, u, r, p, l + 1)];
            const float fa = exp2f(a.x - Ma), fb = exp2f(c.x - Mb);
            Za = fmaf(a.y, fa, Za);
            Na = fmaf(a.z, fa * fa, Na);
            Zb = fmaf(c.y, fb, Zb);
            Nb = fmaf(c.z, fb * fb, Nb);
            C = fmaf(c.w, fa * fb, C);
        }
        cos_acc += C * rsqrtf(Na * Nb);
        const float ia = 1.f / Za, ib = 1.f / Zb;
        const float d2 = Na * ia * ia + Nb * ib * ib - 2.f * C * ia * ib;
        dist_acc += sqrtf(fmaxf(d2, 0.f));
    }
    const float cs = block_sum(cos_acc, red);
    const float ds = block_sum(dist_acc, red);
    if (threadIdx.x == 0) {
        head_cos[blockIdx.x] = cs / (float)Tq;
        head_dist[blockIdx.x] = ds / (float)Tq;
    }
}

__global__ void finalize_pairs_kernel(int n_pairs_total, int Hq, const float *__restrict__ head_cos,
                                      const float *__restrict__ head_dist,
                                      float *__restrict__ pair_cos, float *__restrict__ pair_dist)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_pairs_total) return;
    float cs = 0.f, ds = 0.f;
    for (int h = 0; h < Hq; ++h) {
        cs += head_cos[(size_t)i * Hq + h];
        ds += head_dist[(size_t)i * Hq + h];
    }
    pair_cos[i] = cs / (float)Hq;
    if (pair_dist) pair_dist[i] = ds / (float)Hq;
}

}  // namespace

hipError_t launch_finalize(const StateLayout &lay, const float4 *state, int B, int L, int Hq, int Hkv,
                           int Tq, float *head_cos, float *head_dist, float *pair_cos,
                           float *pair_dist, hipStream_t st)
{
    const int n_pairs_total = B * (L - 1);
    hipLaunchKernelGGL(finalize_heads_kernel, dim3(n_pairs_total * Hq), dim3(kThreads), 0, st, lay,
                       state, L, Hq, Hkv, Tq, head_cos, head_dist);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(finalize_pairs_kernel, dim3((n_pairs_total + 127) / 128), dim3(128), 0, st,
                       n_pairs_total, Hq, head_cos, head_dist, pair_cos, pair_dist);
    return hipGetLastError();
}

}  // namespace krul
