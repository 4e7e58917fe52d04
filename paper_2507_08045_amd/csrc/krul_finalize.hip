// Row similarity and token-wise aggregation (Sec. 5 / Sec. 7: per-token similarities
// are added up; Sec. 4.2: the average over heads).
//
// finalize_heads: one workgroup per (conversation, pair, query head).  A few lanes
// share each query row: they merge the row's partial records of the two layers
// onto a common reference exponent (fixed butterfly order), form the cosine and
// (from the a^2 + b^2 - 2ab expansion of Sec. 7) the Euclidean distance of the two
// attention rows, and the workgroup sums over rows in a fixed tree order.
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

// Running merge of partial records of one row for a layer pair (a = layer l, b = l+1):
// exponents Ma, Mb; Z and N2 of both layers and the cross term C, all relative to them.
struct RowAcc {
    float Ma, Za, Na, Mb, Zb, Nb, C;
};

__device__ inline void merge_into(RowAcc &r, float ma, float za, float na, float mb, float zb, float nb, float c)
{
    const float Ma = fmaxf(r.Ma, ma), Mb = fmaxf(r.Mb, mb);
    const float fa0 = exp2f(r.Ma - Ma), fa1 = exp2f(ma - Ma);
    const float fb0 = exp2f(r.Mb - Mb), fb1 = exp2f(mb - Mb);
    r.Za = r.Za * fa0 + za * fa1;
    r.Na = r.Na * (fa0 * fa0) + na * (fa1 * fa1);
    r.Zb = r.Zb * fb0 + zb * fb1;
    r.Nb = r.Nb * (fb0 * fb0) + nb * (fb1 * fb1);
    r.C = r.C * (fa0 * fb0) + c * (fa1 * fb1);
    r.Ma = Ma;
    r.Mb = Mb;
}

// G lanes of a wave (G a power of two, lanes g*(64/G) + r for g < G) share one query row:
// each merges the partials p = g, g+G, ... and a butterfly over g joins them.  Lanes with
// the same g read consecutive rows, i.e. consecutive records.
//
// PER_WAVE (few rows: all of a head's rows fit the lanes of one wave, G * Tq <= 64): every wave takes a
// (conversation, pair, query head) of its own and sums the rows by shuffles -- a decode step has one row
// per head, and a workgroup per head would be 252 idle threads and four times the workgroups.
template <bool PER_WAVE>
__global__ __launch_bounds__(kThreads) void finalize_heads_kernel(
    StateLayout lay, const float4 *__restrict__ state, int L, int Hq, int Hkv, int Tq, int G,
    int want_dist, int accumulate, int n_items, float *__restrict__ head_cos, float *__restrict__ head_dist)
{
    __shared__ float red[kThreads / 64];
    const int NP = L - 1;
    const int item = PER_WAVE ? blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6) : blockIdx.x;
    if (PER_WAVE && item >= n_items) return;   // (a whole wave: no barrier follows in this form)
    const int h = item % Hq;
    const int l = (item / Hq) % NP;
    const int b = item / (Hq * NP);
    const int g_heads = Hq / Hkv;
    const int u = b * Hkv + h / g_heads;
    const int P = lay.partials;
    const int lane = threadIdx.x & 63, wave = PER_WAVE ? 0 : threadIdx.x >> 6;
    const int RW = 64 / G;                       // rows per wave
    const int rr = lane % RW, g = lane / RW;

    float cos_acc = 0.f, dist_acc = 0.f;
    for (int t0 = 0; t0 < Tq; t0 += (PER_WAVE ? 1 : kThreads / 64) * RW) {
        const int t = t0 + wave * RW + rr;
        RowAcc acc = {kMInit, 0.f, 0.f, kMInit, 0.f, 0.f, 0.f};
        if (t < Tq) {
            const int r = (h % g_heads) * Tq + t;
            for (int p = g; p < P; p += G) {
                const float4 a = state[state_index(lay, u, r, p, l)];
                const float4 c = state[state_index(lay, u, r, p, l + 1)];
                merge_into(acc, a.x, a.y, a.z, c.x, c.y, c.z, c.w);
            }
        }
        for (int off = 32; off >= RW; off >>= 1) {
            const float ma = __shfl_xor(acc.Ma, off, 64), za = __shfl_xor(acc.Za, off, 64);
            const float na = __shfl_xor(acc.Na, off, 64), mb = __shfl_xor(acc.Mb, off, 64);
            const float zb = __shfl_xor(acc.Zb, off, 64), nb = __shfl_xor(acc.Nb, off, 64);
            const float c = __shfl_xor(acc.C, off, 64);
            merge_into(acc, ma, za, na, mb, zb, nb, c);
        }
        if (t < Tq && g == 0) {
            cos_acc += acc.C * rsqrtf(acc.Na * acc.Nb);
            if (want_dist) {   // (Z is only accumulated when the distance is asked for)
                const float ia = 1.f / acc.Za, ib = 1.f / acc.Zb;
                const float d2 = acc.Na * ia * ia + acc.Nb * ib * ib - 2.f * acc.C * ia * ib;
                dist_acc += sqrtf(fmaxf(d2, 0.f));
            }
        }
    }
    float cs = cos_acc, ds = dist_acc;
    if constexpr (PER_WAVE) {
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            cs += __shfl_xor(cs, o, 64);
            ds += __shfl_xor(ds, o, 64);
        }
    } else {
        cs = block_sum(cos_acc, red);
        ds = block_sum(dist_acc, red);
    }
    if ((PER_WAVE ? lane : (int)threadIdx.x) == 0) {
        if (accumulate) {   // token-wise running sums over several calls (Sec. 5, Sec. 7 "adds up")
            head_cos[item] += cs;
            if (want_dist) head_dist[item] += ds;
        } else {
            head_cos[item] = cs / (float)Tq;
            head_dist[item] = ds / (float)Tq;
        }
    }
}

// head values times `scale` (1 for means, 1/tokens for running sums): optionally written out as
// head scores, averaged over the heads in order into the pair scores
__global__ void finalize_pairs_kernel(int n_pairs_total, int Hq, float scale, const float *__restrict__ head_cos,
                                      const float *__restrict__ head_dist, float *__restrict__ head_out,
                                      float *__restrict__ pair_cos, float *__restrict__ pair_dist)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_pairs_total) return;
    float cs = 0.f, ds = 0.f;
    for (int h = 0; h < Hq; ++h) {
        const float c = head_cos[(size_t)i * Hq + h] * scale;
        if (head_out) head_out[(size_t)i * Hq + h] = c;
        cs += c;
        if (pair_dist) ds += head_dist[(size_t)i * Hq + h] * scale;
    }
    pair_cos[i] = cs / (float)Hq;
    if (pair_dist) pair_dist[i] = ds / (float)Hq;
}

// Initial-Recent layer test (Sec. 4.2; Alg. 1 first loop): per (conversation, layer, head) the
// mean over query rows of Zir / Z -- the attention mass on T_initial and T_recent -- from the
// partial records of each row, merged onto a common exponent like the similarity sums.
// (PER_WAVE: as for finalize_heads_kernel)
template <bool PER_WAVE>
__global__ __launch_bounds__(kThreads) void ir_heads_kernel(
    StateLayout lay, const float4 *__restrict__ state, const float *__restrict__ state_ir, int L, int Hq,
    int Hkv, int Tq, int G, int n_items, float *__restrict__ head_ir)
{
    __shared__ float red[kThreads / 64];
    const int item = PER_WAVE ? blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6) : blockIdx.x;
    if (PER_WAVE && item >= n_items) return;   // (a whole wave: no barrier follows in this form)
    const int h = item % Hq;
    const int l = (item / Hq) % L;
    const int b = item / (Hq * L);
    const int g_heads = Hq / Hkv;
    const int u = b * Hkv + h / g_heads;
    const int P = lay.partials;
    const int lane = threadIdx.x & 63, wave = PER_WAVE ? 0 : threadIdx.x >> 6;
    const int RW = 64 / G;                       // rows per wave, G lanes per row
    const int rr = lane % RW, g = lane / RW;

    float mass_acc = 0.f;
    for (int t0 = 0; t0 < Tq; t0 += (PER_WAVE ? 1 : kThreads / 64) * RW) {
        const int t = t0 + wave * RW + rr;
        float M = kMInit, Z = 0.f, I = 0.f;
        if (t < Tq) {
            const int r = (h % g_heads) * Tq + t;
            for (int pi = g; pi < P; pi += G) {
                const size_t idx = state_index(lay, u, r, pi, l);
                const float4 a = state[idx];
                const float zi = state_ir[idx];
                const float Mn = fmaxf(M, a.x);
                const float f0 = exp2f(M - Mn), f1 = exp2f(a.x - Mn);
                Z = Z * f0 + a.y * f1;
                I = I * f0 + zi * f1;
                M = Mn;
            }
        }
        for (int off = 32; off >= RW; off >>= 1) {
            const float m2 = __shfl_xor(M, off, 64), z2 = __shfl_xor(Z, off, 64), i2 = __shfl_xor(I, off, 64);
            const float Mn = fmaxf(M, m2);
            const float f0 = exp2f(M - Mn), f1 = exp2f(m2 - Mn);
            Z = Z * f0 + z2 * f1;
            I = I * f0 + i2 * f1;
            M = Mn;
        }
        if (t < Tq && g == 0) mass_acc += I / Z;
    }
    float ms = mass_acc;
    if constexpr (PER_WAVE) {
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) ms += __shfl_xor(ms, o, 64);
    } else {
        ms = block_sum(mass_acc, red);
    }
    if ((PER_WAVE ? lane : (int)threadIdx.x) == 0) head_ir[item] = ms / (float)Tq;
}

// one thread per (conversation, layer): the average over heads, and the test against gamma
__global__ void ir_layers_kernel(int n_layers_total, int Hq, float gamma, const float *__restrict__ head_ir,
                                 float *__restrict__ ir_mass, uint8_t *__restrict__ eligible)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_layers_total) return;
    float m = 0.f;
    for (int h = 0; h < Hq; ++h) m += head_ir[(size_t)i * Hq + h];
    m /= (float)Hq;
    if (ir_mass) ir_mass[i] = m;
    if (eligible) eligible[i] = m >= gamma ? 1 : 0;   // below gamma: not an Initial-Recent layer, set aside
}

}  // namespace

hipError_t launch_finalize_ir(const StateLayout &lay, const float4 *state, const float *state_ir, int B, int L,
                              int Hq, int Hkv, int Tq, float gamma, float *head_ir, float *ir_mass,
                              uint8_t *eligible, hipStream_t st)
{
    int G = 1;
    while (G < 64 && G * Tq < kThreads && G < lay.partials) G <<= 1;
    const int n_items = B * L * Hq;
    if (Tq <= 8) {   // few rows: a wave per head, G lanes per row with G * Tq <= 64
        G = 1;
        while (G * 2 * Tq <= 64 && G < lay.partials) G <<= 1;
        hipLaunchKernelGGL(ir_heads_kernel<true>, dim3((n_items + kThreads / 64 - 1) / (kThreads / 64)), dim3(kThreads),
                           0, st, lay, state, state_ir, L, Hq, Hkv, Tq, G, n_items, head_ir);
    } else {
        hipLaunchKernelGGL(ir_heads_kernel<false>, dim3(n_items), dim3(kThreads), 0, st, lay, state, state_ir, L, Hq,
                           Hkv, Tq, G, n_items, head_ir);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(ir_layers_kernel, dim3((B * L + 127) / 128), dim3(128), 0, st, B * L, Hq, gamma, head_ir,
                       ir_mass, eligible);
    return hipGetLastError();
}

hipError_t launch_finalize(const StateLayout &lay, const float4 *state, int B, int L, int Hq, int Hkv,
                           int Tq, float *head_cos, float *head_dist, float *pair_cos,
                           float *pair_dist, bool accumulate, hipStream_t st)
{
    const int n_pairs_total = B * (L - 1);
    // lanes per row: enough to keep a workgroup's 256 threads busy, at most one per partial
    int G = 1;
    while (G < 64 && G * Tq < kThreads && G < lay.partials) G <<= 1;
    const int n_items = n_pairs_total * Hq;
    if (Tq <= 8) {   // few rows: a wave per head, G lanes per row with G * Tq <= 64
        G = 1;
        while (G * 2 * Tq <= 64 && G < lay.partials) G <<= 1;
        hipLaunchKernelGGL(finalize_heads_kernel<true>, dim3((n_items + kThreads / 64 - 1) / (kThreads / 64)),
                           dim3(kThreads), 0, st, lay, state, L, Hq, Hkv, Tq, G, pair_dist != nullptr,
                           accumulate ? 1 : 0, n_items, head_cos, head_dist);
    } else {
        hipLaunchKernelGGL(finalize_heads_kernel<false>, dim3(n_items), dim3(kThreads), 0, st, lay,
                           state, L, Hq, Hkv, Tq, G, pair_dist != nullptr, accumulate ? 1 : 0, n_items, head_cos,
                           head_dist);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || accumulate || !pair_cos) return e;   // (no pair scores asked for: the caller forms them)
    hipLaunchKernelGGL(finalize_pairs_kernel, dim3((n_pairs_total + 127) / 128), dim3(128), 0, st,
                       n_pairs_total, Hq, 1.0f, head_cos, head_dist, (float *)nullptr, pair_cos, pair_dist);
    return hipGetLastError();
}

hipError_t launch_scores_from_sums(const float *head_sum, const float *head_dist_sum, int n_pairs_total,
                                   int Hq, float inv_tokens, float *pair_cos, float *head_score,
                                   float *pair_dist, hipStream_t st)
{
    hipLaunchKernelGGL(finalize_pairs_kernel, dim3((n_pairs_total + 127) / 128), dim3(128), 0, st,
                       n_pairs_total, Hq, inv_tokens, head_sum, head_dist_sum, head_score, pair_cos, pair_dist);
    return hipGetLastError();
}

}  // namespace krul
