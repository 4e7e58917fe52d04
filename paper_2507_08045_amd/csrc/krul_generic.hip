// Portable similarity kernel (fp32 VALU arithmetic; float32, bfloat16 or binary16 inputs; any head_dim
// multiple of 8).
//
// One wavefront owns one query row (conversation, query head, token) and one key
// split.  It walks its keys 64 at a time (one key per lane) and, for each group of
// 64 keys, the layers in order: logits by a plain fp32 dot product (attention
// equation of Sec. 2.1), exact online softmax statistics, and the cross term with
// the previous layer's exponentials of the same keys (Sec. 7, the "ab" term).  The
// per-layer running values live in LDS; wave shuffles do the reductions, so the
// result does not depend on timing.
#include "krul_common.h"

namespace krul {
namespace {

__device__ inline float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ inline float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

__device__ inline float bf16_to_f32(uint32_t bits16) { return __uint_as_float(bits16 << 16); }

// dot(q (LDS, fp32), key row (global)) over d elements, d % 8 == 0
template <typename T>
__device__ inline float dot_row(const float *qs, const T *krow, int d);

template <>
__device__ inline float dot_row<float>(const float *qs, const float *krow, int d)
{
    float acc = 0.f;
    const float4 *kp = reinterpret_cast<const float4 *>(krow);
    for (int i = 0; i < d / 4; ++i) {
        const float4 kv = kp[i];
        acc = fmaf(qs[4 * i + 0], kv.x, acc);
        acc = fmaf(qs[4 * i + 1], kv.y, acc);
        acc = fmaf(qs[4 * i + 2], kv.z, acc);
        acc = fmaf(qs[4 * i + 3], kv.w, acc);
    }
    return acc;
}

template <>
__device__ inline float dot_row<uint16_t>(const float *qs, const uint16_t *krow, int d)
{
    float acc = 0.f;
    const uint4 *kp = reinterpret_cast<const uint4 *>(krow);
    for (int i = 0; i < d / 8; ++i) {
        const uint4 kv = kp[i];
        const uint32_t w[4] = {kv.x, kv.y, kv.z, kv.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            acc = fmaf(qs[8 * i + 2 * j + 0], bf16_to_f32(w[j] & 0xFFFFu), acc);
            acc = fmaf(qs[8 * i + 2 * j + 1], bf16_to_f32(w[j] >> 16), acc);
        }
    }
    return acc;
}

template <>
__device__ inline float dot_row<_Float16>(const float *qs, const _Float16 *krow, int d)
{
    float acc = 0.f;
    const uint4 *kp = reinterpret_cast<const uint4 *>(krow);
    for (int i = 0; i < d / 8; ++i) {
        const uint4 kv = kp[i];
        const _Float16 *h = reinterpret_cast<const _Float16 *>(&kv);
#pragma unroll
        for (int j = 0; j < 8; ++j) acc = fmaf(qs[8 * i + j], (float)h[j], acc);
    }
    return acc;
}

template <typename T>
__device__ inline float load_as_f32(const T *p, size_t i);
template <>
__device__ inline float load_as_f32<float>(const float *p, size_t i) { return p[i]; }
template <>
__device__ inline float load_as_f32<uint16_t>(const uint16_t *p, size_t i) { return bf16_to_f32(p[i]); }
template <>
__device__ inline float load_as_f32<_Float16>(const _Float16 *p, size_t i) { return (float)p[i]; }

template <typename T>
__global__ __launch_bounds__(64) void sim_generic_kernel(SimParams p)
{
    extern __shared__ float smem[];
    float4 *st = reinterpret_cast<float4 *>(smem);   // [L] running (m, Z, N2, C)
    float *qs = smem + 4 * p.L;                      // [d] current query row
    float *st_ir = qs + p.d;                         // [L] running Zir (Initial-Recent layer test)

    const int lane = threadIdx.x;
    const int sp = blockIdx.x % p.lay.n_split;
    const size_t row = blockIdx.x / p.lay.n_split;   // (b * Hq + h) * Tq + t
    const int t = (int)(row % p.Tq);
    const int h = (int)((row / p.Tq) % p.Hq);
    const int b = (int)(row / ((size_t)p.Tq * p.Hq));
    const int kvh = h / p.g;
    const int u = b * p.Hkv + kvh;
    const int r = (h % p.g) * p.Tq + t;

    const int key_begin = sp * p.keys_per_split;
    int key_end = min(p.S, key_begin + p.keys_per_split);
    if (p.causal) key_end = min(key_end, p.S - p.Tq + t + 1);   // this row sees keys j <= S - Tq + t

    for (int l = lane; l < p.L; l += 64) {
        st[l] = make_float4(kMInit, 0.f, 0.f, 0.f);
        st_ir[l] = 0.f;
    }
    __syncthreads();

    const T *Q = static_cast<const T *>(p.q);
    const T *K = static_cast<const T *>(p.k);

    for (int key0 = key_begin; key0 < key_end; key0 += 64) {
        const int key = key0 + lane;
        const bool valid = key < key_end;
        const bool in_ir = valid && (key < p.ir_init_end || key >= p.ir_recent_begin);   // T_initial or T_recent
        float e_prev = 0.f, f_prev = 1.f;
        for (int l = 0; l < p.L; ++l) {
            const size_t qoff = ((((size_t)b * p.L + l) * p.Hq + h) * p.Tq + t) * p.d;
            __syncthreads();
            for (int i = lane; i < p.d; i += 64) qs[i] = load_as_f32<T>(Q, qoff + i);
            __syncthreads();
            float x = -INFINITY;
            if (valid) {
                const T *kl = p.k_tab ? static_cast<const T *>(p.k_tab[l]) : K + (size_t)l * p.k_stride_l;
                size_t koff = (size_t)kvh * p.k_stride_h;
                if (p.block_table)   // paged keys
                    koff += (size_t)p.block_table[(size_t)b * p.max_blocks + (key >> p.page_shift)] * p.k_stride_page +
                            (size_t)(key & ((1 << p.page_shift) - 1)) * p.k_stride_s;
                else
                    koff += (size_t)b * p.k_stride_b + (size_t)key * p.k_stride_s;
                x = dot_row<T>(qs, kl + koff, p.d) * p.c;
            }
            const float4 cur = st[l];
            const float m_new = fmaxf(cur.x, wave_max(x));
            const float f = exp2f(cur.x - m_new);
            const float e = exp2f(x - m_new);
            const float sz = wave_sum(e);
            const float sn = wave_sum(e * e);
            const float sc = wave_sum(e * e_prev);
            float si = 0.f;
            if (p.want_ir) si = wave_sum(in_ir ? e : 0.f);
            __syncthreads();
            if (lane == 0) {
                st[l] = make_float4(m_new, cur.y * f + sz, cur.z * f * f + sn, cur.w * f * f_prev + sc);
                st_ir[l] = st_ir[l] * f + si;
            }
            e_prev = e;
            f_prev = f;
        }
    }
    __syncthreads();
    for (int l = lane; l < p.L; l += 64) {
        p.state[state_index(p.lay, u, r, sp, l)] = st[l];
        if (p.want_ir) p.state_ir[state_index(p.lay, u, r, sp, l)] = st_ir[l];
    }
}

}  // namespace

hipError_t launch_sim_generic(const SimParams &p, int dtype, int n_workgroups, hipStream_t st)
{
    const size_t smem = sizeof(float) * (5 * (size_t)p.L + p.d);
    if (dtype == KRUL_F32)
        hipLaunchKernelGGL(sim_generic_kernel<float>, dim3(n_workgroups), dim3(64), smem, st, p);
    else if (dtype == KRUL_F16)
        hipLaunchKernelGGL(sim_generic_kernel<_Float16>, dim3(n_workgroups), dim3(64), smem, st, p);
    else
        hipLaunchKernelGGL(sim_generic_kernel<uint16_t>, dim3(n_workgroups), dim3(64), smem, st, p);
    return hipGetLastError();
}

}  // namespace krul
