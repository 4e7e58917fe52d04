// Greedy disjoint layer-pair selection (Alg. 1, second loop; Sec. 4.2).
//
// One workgroup per conversation.  The candidates (adjacent pairs whose two layers
// are eligible) are ranked by counting: rank(l) = number of candidates that come
// before l in the order "higher score first, equal scores lower index first".  That
// is the stable descending sort the algorithm asks for, with no data-dependent
// control flow.  One thread then scans the ranked list and takes a pair iff both
// its layers are still free, until n_select pairs are held.
#include "krul_common.h"

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
    int32_t *order = reinterpret_cast<int32_t *>(score + NP);    // [NP] candidate at each rank
    uint8_t *cand = reinterpret_cast<uint8_t *>(order + NP);     // [NP]
    uint8_t *used = cand + NP;                                   // [n_layers]

    const int b = blockIdx.x;
    const float *sc = pair_score + (size_t)b * NP;
    const uint8_t *el = eligible ? eligible + (size_t)b * n_layers : nullptr;

    for (int l = threadIdx.x; l < NP; l += kSelThreads) {
        score[l] = sc[l];
        cand[l] = (!el || (el[l] && el[l + 1])) ? 1 : 0;
        order[l] = -1;
    }
    for (int l = threadIdx.x; l < n_layers; l += kSelThreads) used[l] = 0;
    __syncthreads();

    for (int l = threadIdx.x; l < NP; l += kSelThreads) {
        if (!cand[l]) continue;
        const float s = score[l];
        int rank = 0;
        for (int j = 0; j < NP; ++j) {
            if (!cand[j]) continue;
            const float sj = score[j];
            // j precedes l unless l's score is strictly higher, or equal with l first
            rank += (sj > s || (!(sj < s) && j < l)) ? 1 : 0;
        }
        order[rank] = l;
    }
    __syncthreads();

    if (threadIdx.x == 0) {
        int cnt = 0;
        for (int i = 0; i < NP && cnt < n_select; ++i) {
            const int l = order[i];
            if (l < 0) break;  // ranks are dense: first hole = end of candidates
            if (used[l] || used[l + 1]) continue;
            used[l] = used[l + 1] = 1;
            out_pairs[(size_t)b * n_select + cnt++] = l;
        }
        out_count[b] = cnt;
        for (int i = cnt; i < n_select; ++i) out_pairs[(size_t)b * n_select + i] = -1;
    }
}

}  // namespace

hipError_t launch_select(const float *pair_score, const uint8_t *eligible, int batch, int n_layers,
                         int n_select, int32_t *out_pairs, int32_t *out_count, hipStream_t st)
{
    const int NP = n_layers - 1;
    const size_t smem = (size_t)NP * (sizeof(float) + sizeof(int32_t) + 1) + n_layers;
    hipLaunchKernelGGL(select_pairs_kernel, dim3(batch), dim3(kSelThreads), smem, st, pair_score,
                       eligible, n_layers, n_select, out_pairs, out_count);
    return hipGetLastError();
}

}  // namespace krul
