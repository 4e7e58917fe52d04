// Greedy disjoint choice among adjacent layer pairs (Alg. 1, second loop; Sec. 4.2) for one
// conversation, run by all threads of a workgroup: shared by the selection kernel and by the
// kernel that averages heads and selects in one launch.
//
// The candidates (adjacent pairs whose two layers are eligible) are ranked by counting:
// rank(l) = number of candidates that come before l in the order "higher score first, equal
// scores lower index first".  That is the stable descending sort the algorithm asks for, with no
// data-dependent control flow.  One thread then scans the ranked list and takes a pair iff both
// its layers are still free, until n_select pairs are held.  A pair whose score is NaN has no
// place in that order: it is no candidate (so the order stays total and the ranks dense).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace krul {

// LDS bytes select_adjacent needs beside the scores: order [NP] int32, cand [NP], used [n_layers]
__host__ __device__ inline size_t select_scratch_bytes(int n_layers)
{
    return (size_t)(n_layers - 1) * (sizeof(int32_t) + 1) + (size_t)n_layers;
}

// score: the conversation's NP = n_layers - 1 pair scores in LDS (written before the call; the
// function starts with a barrier).  el: its eligibility bytes in global memory, or null.
// scratch: select_scratch_bytes(n_layers) bytes of LDS, 4-byte aligned.  out_pairs: n_select entries.
__device__ inline void select_adjacent(const float *score, const uint8_t *el, int n_layers, int n_select,
                                       int32_t *out_pairs, int32_t *out_count, void *scratch)
{
    const int NP = n_layers - 1;
    int32_t *order = static_cast<int32_t *>(scratch);            // [NP] candidate at each rank
    uint8_t *cand = reinterpret_cast<uint8_t *>(order + NP);     // [NP]
    uint8_t *used = cand + NP;                                   // [n_layers]
    const int nt = blockDim.x;

    for (int l = threadIdx.x; l < NP; l += nt) {
        cand[l] = (!el || (el[l] && el[l + 1])) ? 1 : 0;
        order[l] = -1;
    }
    for (int l = threadIdx.x; l < n_layers; l += nt) used[l] = 0;
    __syncthreads();

    for (int l = threadIdx.x; l < NP; l += nt) {
        const float s = score[l];
        if (!cand[l] || s != s) continue;
        int rank = 0;
#pragma unroll 8
        for (int j = 0; j < NP; ++j) {
            const float sj = score[j];
            // j precedes l unless l's score is strictly higher, or equal with l first
            rank += (cand[j] && sj == sj && (sj > s || (!(sj < s) && j < l))) ? 1 : 0;
        }
        order[rank] = l;
    }
    __syncthreads();

    if (n_layers <= 128) {
        // The scan in the first wave: its lanes hold the ranked list, the layers in use are two 64-bit
        // masks, and every step is wave-uniform (one LDS round trip in all instead of three per step).
        if (threadIdx.x < 64) {
            const int lane = threadIdx.x;
            const int o_lo = lane < NP ? order[lane] : -1, o_hi = lane + 64 < NP ? order[lane + 64] : -1;
            unsigned long long used_lo = 0, used_hi = 0;
            int cnt = 0;
            for (int i = 0; i < NP && cnt < n_select; ++i) {
                const int l = i < 64 ? __builtin_amdgcn_readlane(o_lo, i) : __builtin_amdgcn_readlane(o_hi, i - 64);
                if (l < 0) break;  // ranks are dense: first hole = end of candidates
                // layers l and l + 1 as bits of the 128-bit mask
                const unsigned long long bit_a = 1ull << (l & 63), bit_b = 1ull << ((l + 1) & 63);
                const unsigned long long m_lo = (l < 64 ? bit_a : 0) | (l + 1 < 64 ? bit_b : 0);
                const unsigned long long m_hi = (l < 64 ? 0 : bit_a) | (l + 1 < 64 ? 0 : bit_b);
                if (((used_lo & m_lo) | (used_hi & m_hi)) != 0) continue;
                used_lo |= m_lo;
                used_hi |= m_hi;
                if (lane == 0) out_pairs[cnt] = l;
                ++cnt;
            }
            if (lane == 0) *out_count = cnt;
            for (int i = cnt + lane; i < n_select; i += 64) out_pairs[i] = -1;
        }
    } else if (threadIdx.x == 0) {
        int cnt = 0;
        for (int i = 0; i < NP && cnt < n_select; ++i) {
            const int l = order[i];
            if (l < 0) break;
            if (used[l] || used[l + 1]) continue;
            used[l] = used[l + 1] = 1;
            out_pairs[cnt++] = l;
        }
        *out_count = cnt;
        for (int i = cnt; i < n_select; ++i) out_pairs[i] = -1;
    }
    __syncthreads();   // the scratch may be reused
}

}  // namespace krul
