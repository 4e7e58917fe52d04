// Greedy disjoint layer-pair selection (Alg. 1, second loop; Sec. 4.2): one workgroup per
// conversation; the method itself is select_adjacent() in krul_select_core.h.
#include "krul_common.h"
#include "krul_select_core.h"

namespace krul {
namespace {

constexpr int kSelThreads = 256;

__global__ __launch_bounds__(kSelThreads) void select_pairs_kernel(
    const float *__restrict__ pair_score, const uint8_t *__restrict__ eligible, int n_layers,
    int n_select, int32_t *__restrict__ out_pairs, int32_t *__restrict__ out_count)
{
    extern __shared__ unsigned char sel_smem[];
    const int NP = n_layers - 1;
    float *score = reinterpret_cast<float *>(sel_smem);          // [NP]
    const int b = blockIdx.x;
    for (int l = threadIdx.x; l < NP; l += kSelThreads) score[l] = pair_score[(size_t)b * NP + l];
    select_adjacent(score, eligible ? eligible + (size_t)b * n_layers : nullptr, n_layers, n_select,
                    out_pairs + (size_t)b * n_select, out_count + b, score + NP);
}

// Averages over the heads (in order, as finalize_pairs_kernel takes them: the same bits) and the greedy
// choice of one conversation per workgroup: two steps whose launches cost more than the work in them.
constexpr int kPsThreads = 1024;
constexpr int kPsLoads = (kPairsSelectMaxHeads + kPsThreads - 1) / kPsThreads;   // head values per thread

__global__ __launch_bounds__(kPsThreads) void pairs_select_kernel(PairsSelectArgs a)
{
    extern __shared__ unsigned char sel_smem[];
    const int NP = a.L - 1, n = NP * a.Hq, b = blockIdx.x;
    float *vc = reinterpret_cast<float *>(sel_smem);   // [n] head cosines of this conversation
    float *vd = vc + n;                                // [n] head distances
    float *pc = vd + n;                                // [NP] pair scores
    const float *head_cos = a.head_cos + (size_t)b * n;
    const float *head_dist = a.head_dist ? a.head_dist + (size_t)b * n : nullptr;
    {   // all loads of a thread are issued before the first is waited for: one memory latency, not one per value
        float c[kPsLoads], dd[kPsLoads];
#pragma unroll
        for (int u = 0; u < kPsLoads; ++u) {
            const int i = threadIdx.x + u * kPsThreads;
            c[u] = i < n ? head_cos[i] : 0.f;
            dd[u] = i < n && head_dist ? head_dist[i] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < kPsLoads; ++u) {
            const int i = threadIdx.x + u * kPsThreads;
            if (i < n) {
                vc[i] = c[u];
                vd[i] = dd[u];
            }
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < NP; i += kPsThreads) {
        float cs = 0.f, ds = 0.f;
#pragma unroll 8
        for (int h = 0; h < a.Hq; ++h) {
            cs += vc[i * a.Hq + h];
            if (head_dist) ds += vd[i * a.Hq + h];
        }
        a.pair_cos[(size_t)b * NP + i] = pc[i] = cs / (float)a.Hq;
        if (head_dist) a.pair_dist[(size_t)b * NP + i] = ds / (float)a.Hq;
    }
    // (select_adjacent starts with a barrier)
    select_adjacent(pc, a.eligible ? a.eligible + (size_t)b * a.L : nullptr, a.L, a.n_select,
                    a.out_pairs + (size_t)b * a.n_select, a.out_count + b, pc + NP);
}

}  // namespace

bool pairs_select_fits(int L, int Hq)
{
    return (long long)(L - 1) * Hq <= kPairsSelectMaxHeads;
}

hipError_t launch_pairs_select(const PairsSelectArgs &a, hipStream_t st)
{
    const int NP = a.L - 1;
    const size_t smem = (size_t)(2 * NP * a.Hq + NP) * sizeof(float) + select_scratch_bytes(a.L);
    if (smem > 48 * 1024) {   // more dynamic LDS than a launch may ask for without saying so first
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(pairs_select_kernel),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(pairs_select_kernel, dim3(a.B), dim3(kPsThreads), smem, st, a);
    return hipGetLastError();
}

hipError_t launch_select(const float *pair_score, const uint8_t *eligible, int batch, int n_layers,
                         int n_select, int32_t *out_pairs, int32_t *out_count, hipStream_t st)
{
    const int NP = n_layers - 1;
    const size_t smem = (size_t)NP * sizeof(float) + select_scratch_bytes(n_layers);
    hipLaunchKernelGGL(select_pairs_kernel, dim3(batch), dim3(kSelThreads), smem, st, pair_score,
                       eligible, n_layers, n_select, out_pairs, out_count);
    return hipGetLastError();
}

}  // namespace krul
