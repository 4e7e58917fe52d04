// Similarity of EVERY two layers i > j (Alg. 1 as printed: "for every two weights A_i, A_j (i > j)",
// Sec. 4.2; the layer-by-layer similarity map of Sec. 2.3), for gfx950.
//
// For one query row the L(L-1)/2 cross terms  C_ij = sum_k e_i[k] e_j[k]  (the "ab" of Sec. 7's
// a^2 + b^2 - 2ab) are the Gram matrix  G = E E^T  of the L x S matrix E of the row's exponentials,
// a dense contraction over the keys: it goes to the matrix cores.  The layer-chained kernel of the
// adjacent reading cannot hold L layers' exponentials of a tile in registers or LDS, so here the
// exponentials ARE written out -- as the paper itself keeps the attention weights (Sec. 5) -- in
// fp16, in batches of rows sized to the workspace the caller gives:
//
//   1. weights kernel: per (128 rows of a unit, layer) two sweeps over the keys with
//      v_mfma_f32_32x32x16_bf16 logits: the row maxima, then e = 2^(x - max) <= 1, Z = sum e, and
//      the fp16 store of e.  One wave owns 32 rows and every key of them, so the maximum and Z need
//      one exchange between the two half-waves and nothing else.  K chunks of 64 keys go through a
//      double-buffered, XOR-swizzled LDS tile; the second sweep re-reads K from L2.
//      Layout of E: [32-row block][layer][32-key block][row][32 x fp16]: the 2 KB that a wave's
//      result block covers are contiguous (full-line stores), and the 64 bytes of one (row, layer,
//      key block) are what one Gram operand fetch reads.  Inside the 64 bytes the keys stand in the
//      order of the MFMA result registers; the order is the same for all layers of a row, which is
//      all a contraction over the keys needs.
//   2. Gram kernel: one workgroup per row, its four waves taking every fourth key block:
//      v_mfma_f32_32x32x16_f16 with A = B = the row's [32 layers x 16 keys] piece (lane = layer),
//      one accumulator block per pair of 32-layer blocks.  The waves' sums are added in a fixed
//      order in LDS; cos_ij = G_ij / sqrt(G_ii G_jj) and
//      dist_ij^2 = G_ii/Z_i^2 + G_jj/Z_j^2 - 2 G_ij/(Z_i Z_j) are written per row.
//   3. reduce kernel: per (unit, head of the group) the batch's rows are added, in order, to the
//      head sums; the last kernel divides by the token count, averages the heads (Sec. 4.2) and
//      mirrors the matrix.
// A portable weights kernel (one wave per row and layer, fp32 dot products) covers fp32 inputs and
// other head sizes; it writes the same layout.
//
// Also here: the greedy disjoint choice over all candidate pairs (Alg. 1, second loop).
#include <math.h>

#include "krul_common.h"

namespace krul {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kRowsPerGroup = 128;   // rows of one weights-kernel workgroup: four 32-row blocks
constexpr int kThreads = 256;

struct APParams {
    const void *q;
    const void *k;
    int B, L, Hq, Hkv, g, d, S, Tq, Rk;
    int causal;
    float c;            // scale * log2(e)
    int NRG;            // 128-row groups per unit
    int NKB;            // 32-key blocks per row
    int grg0, nrg;      // this batch: global row groups [grg0, grg0 + nrg)
    int want_dist;
    unsigned char *E;   // [nrg*4][L][NKB][32][64 bytes]
    float *rowZ;        // [nrg*128][L]
    float *row_cos;     // [nrg*128][L*L]  (entries i > j)
    float *row_dist;    // same, or unused
    float *head_cos;    // [B][Hq][L*L] running sums over the rows of a head
    float *head_dist;
};

__device__ inline size_t e_block_offset(const APParams &p, int rbl, int l, int kb)
{
    return ((((size_t)rbl * p.L + l) * p.NKB + kb) * 32) * 64;
}

// Row-dependent XOR applied to the 16-byte piece index inside an LDS tile of key rows, so that the
// 16-byte operand reads of consecutive rows fall into different bank groups.
template <int D>
__device__ inline int swz(int row)
{
    return D == 128 ? (row & 15) : ((row >> 1) & 7);
}

__device__ inline uint32_t pack_f16(float a, float b)
{
    const f16x2 h = {(_Float16)a, (_Float16)b};   // round to nearest even
    return __builtin_bit_cast(uint32_t, h);
}

// ------------------------------------------------------------------------------------------------
// 1. weights kernel (bf16, head_dim 64 or 128)
template <int D>
__global__ __launch_bounds__(kThreads) void ap_weights_mfma_kernel(APParams p)
{
    constexpr int KS = D / 16, PPR = D / 8, ROWB = D * 2, CHK = 64, SLOT = CHK * ROWB;
    constexpr int NLD = CHK * PPR / kThreads;
    __shared__ __attribute__((aligned(16))) unsigned char kl[2][SLOT];

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, half = lane >> 5, n = lane & 31;
    const int l = blockIdx.x % p.L;
    const int rgl = blockIdx.x / p.L;
    const int grg = p.grg0 + rgl;
    const int u = grg / p.NRG, rg = grg % p.NRG;
    const int b = u / p.Hkv, kvh = u % p.Hkv;
    const int rbl = rgl * 4 + w;
    const int r = (rg * 4 + w) * 32 + n;            // row of the unit: head-in-group * Tq + t
    const bool blk_ok = (rg * 4 + w) * 32 < p.Rk;   // this wave has rows at all
    const bool row_ok = r < p.Rk;
    const int S = p.S;
    const int row_end = row_ok ? (p.causal ? S - p.Tq + r % p.Tq + 1 : S) : 0;   // keys [0, row_end) are seen

    // query rows of a unit are contiguous in r: [b][l][kvh*g + r / Tq][r % Tq][D]
    const uint16_t *Qg = static_cast<const uint16_t *>(p.q);
    const uint16_t *qrow = Qg + ((((size_t)b * p.L + l) * p.Hq + (size_t)kvh * p.g) * p.Tq + (size_t)(row_ok ? r : 0)) * D;
    bf16x8 qf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (row_ok) v = *reinterpret_cast<const uint4 *>(qrow + ks * 16 + half * 8);
        qf[ks] = __builtin_bit_cast(bf16x8, v);
    }
    const uint16_t *kbase = static_cast<const uint16_t *>(p.k) + ((((size_t)b * p.L + l) * p.Hkv + kvh) * (size_t)S) * D;

    // staging: piece id = i*256 + tid -> key row id / PPR, 16-byte piece id % PPR
    uint4 stage[NLD];
    auto load_chunk = [&](int c) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int id = i * kThreads + tid, row = id / PPR, pc = id % PPR;
            const int key = c * CHK + row;
            stage[i] = key < S ? *reinterpret_cast<const uint4 *>(kbase + (size_t)key * D + pc * 8)
                               : make_uint4(0u, 0u, 0u, 0u);
        }
    };
    auto store_chunk = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int id = i * kThreads + tid, row = id / PPR, pc = id % PPR;
            *reinterpret_cast<uint4 *>(&kl[buf][row * ROWB + ((pc ^ swz<D>(row)) << 4)]) = stage[i];
        }
    };
    // logits of the 32 keys of block kb of a chunk against this wave's 32 rows: lane (n, half) gets
    // row n, keys 8*(v/4) + 4*half + v%4
    auto logits = [&](int buf, int kb) __attribute__((always_inline)) -> f32x16 {
        f32x16 a;
#pragma unroll
        for (int v = 0; v < 16; ++v) a[v] = 0.f;
        const int row = kb * 32 + n;
        const unsigned char *rp = &kl[buf][row * ROWB];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const bf16x8 ka = *reinterpret_cast<const bf16x8 *>(rp + (((2 * ks + half) ^ swz<D>(row)) << 4));
            a = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qf[ks], a, 0, 0, 0);
        }
        return a;
    };

    const int nchunks = (S + CHK - 1) / CHK;
    float mx = -INFINITY, M = 0.f, z = 0.f;
    for (int sweep = 0; sweep < 2; ++sweep) {
        load_chunk(0);
        store_chunk(0);
        __syncthreads();
        for (int c = 0; c < nchunks; ++c) {
            const int buf = c & 1;
            if (c + 1 < nchunks) load_chunk(c + 1);
            if (blk_ok) {
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) {
                    const int key0 = c * CHK + kb * 32;
                    if (key0 >= S) break;   // (the last chunk may hold one block only: E has no room for another)
                    f32x16 a = logits(buf, kb);
                    if (__any(key0 + 32 > row_end)) {   // some row of the wave does not see all 32 keys
                        const int lim = row_end - key0 - 4 * half;
#pragma unroll
                        for (int v = 0; v < 16; ++v)
                            if (8 * (v >> 2) + (v & 3) >= lim) a[v] = -INFINITY;
                    }
                    if (sweep == 0) {
#pragma unroll
                        for (int v = 0; v < 16; ++v) mx = fmaxf(mx, a[v]);
                    } else {
                        uint32_t pk[8];
#pragma unroll
                        for (int v = 0; v < 16; v += 2) {
                            const float e0 = __builtin_amdgcn_exp2f(fmaf(a[v], p.c, -M));
                            const float e1 = __builtin_amdgcn_exp2f(fmaf(a[v + 1], p.c, -M));
                            z += e0 + e1;
                            pk[v >> 1] = pack_f16(e0, e1);
                        }
                        if (row_ok) {
                            uint4 *dst = reinterpret_cast<uint4 *>(p.E + e_block_offset(p, rbl, l, c * 2 + kb) + n * 64 + half * 32);
                            dst[0] = make_uint4(pk[0], pk[1], pk[2], pk[3]);
                            dst[1] = make_uint4(pk[4], pk[5], pk[6], pk[7]);
                        }
                    }
                }
            }
            if (c + 1 < nchunks) store_chunk(buf ^ 1);
            __syncthreads();
        }
        if (sweep == 0) {
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            M = row_ok ? mx * p.c : 0.f;   // (c > 0: the largest logit gives the largest exponent)
        }
    }
    z += __shfl_xor(z, 32, 64);
    if (row_ok && half == 0) p.rowZ[((size_t)rbl * 32 + n) * p.L + l] = z;
}

// Portable weights kernel: one wave per (row of the batch, layer); lane = key.
template <typename T>
__device__ inline float load_f32(const T *ptr, size_t i);
template <>
__device__ inline float load_f32<float>(const float *ptr, size_t i) { return ptr[i]; }
template <>
__device__ inline float load_f32<uint16_t>(const uint16_t *ptr, size_t i) { return __uint_as_float((uint32_t)ptr[i] << 16); }

template <typename T>
__global__ __launch_bounds__(64) void ap_weights_generic_kernel(APParams p)
{
    extern __shared__ float qs[];   // [d]
    const int lane = threadIdx.x;
    const int l = blockIdx.x % p.L;
    const int rowl = blockIdx.x / p.L;
    const int rbl = rowl >> 5, n = rowl & 31;
    const int grb = p.grg0 * 4 + rbl;
    const int u = grb / (p.NRG * 4), rb = grb % (p.NRG * 4);
    const int r = rb * 32 + n;
    if (r >= p.Rk) return;
    const int b = u / p.Hkv, kvh = u % p.Hkv;
    const int hq = kvh * p.g + r / p.Tq, t = r % p.Tq;
    const int S = p.S, d = p.d;
    const int row_end = p.causal ? S - p.Tq + t + 1 : S;
    const T *Q = static_cast<const T *>(p.q);
    const T *K = static_cast<const T *>(p.k);
    const size_t qoff = ((((size_t)b * p.L + l) * p.Hq + hq) * p.Tq + t) * d;
    const size_t koff = ((((size_t)b * p.L + l) * p.Hkv + kvh) * (size_t)S) * d;
    for (int i = lane; i < d; i += 64) qs[i] = load_f32<T>(Q, qoff + i);
    __syncthreads();

    auto logit = [&](int key) -> float {
        float acc = 0.f;
        for (int i = 0; i < d; ++i) acc = fmaf(qs[i], load_f32<T>(K, koff + (size_t)key * d + i), acc);
        return acc * p.c;
    };
    float mx = -INFINITY;
    for (int key = lane; key < row_end; key += 64) mx = fmaxf(mx, logit(key));
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
    float z = 0.f;
    _Float16 *E = reinterpret_cast<_Float16 *>(p.E);
    for (int key = lane; key < p.NKB * 32; key += 64) {
        const float e = key < row_end ? exp2f(logit(key) - mx) : 0.f;
        z += e;
        E[(e_block_offset(p, rbl, l, key >> 5) + (size_t)n * 64) / 2 + (key & 31)] = (_Float16)e;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) z += __shfl_xor(z, o, 64);
    if (lane == 0) p.rowZ[((size_t)rbl * 32 + n) * p.L + l] = z;
}

// ------------------------------------------------------------------------------------------------
// 2. Gram kernel: one workgroup per row of the batch.  NB = 32-layer blocks (L <= 32*NB).
template <int NB>
__global__ __launch_bounds__(kThreads) void ap_gram_kernel(APParams p)
{
    extern __shared__ float G[];   // [Lp][Lp], Lp = 32*NB; blocks (bi >= bj) are filled
    constexpr int Lp = 32 * NB, NACC = NB * (NB + 1) / 2;
    const int rowl = blockIdx.x, rbl = rowl >> 5, row32 = rowl & 31;
    const int grb = p.grg0 * 4 + rbl;
    const int rb = grb % (p.NRG * 4);
    if (rb * 32 + row32 >= p.Rk) return;   // (the whole workgroup)
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, m = lane & 31, kg = lane >> 5;
    const int L = p.L;

    const unsigned char *src[NB];
    bool lok[NB];
#pragma unroll
    for (int lb = 0; lb < NB; ++lb) {
        const int l = lb * 32 + m;
        lok[lb] = l < L;
        src[lb] = p.E + e_block_offset(p, rbl, lok[lb] ? l : 0, 0) + row32 * 64 + kg * 32;
    }
    f32x16 acc[NACC];
#pragma unroll
    for (int a = 0; a < NACC; ++a)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[a][v] = 0.f;

    for (int i = tid; i < Lp * Lp; i += kThreads) G[i] = 0.f;

    constexpr int UNR = NB == 1 ? 4 : (NB == 2 ? 2 : 1);
    const int NKB = p.NKB;
    for (int kb0 = w; kb0 < NKB; kb0 += 4 * UNR) {
        uint4 raw[UNR][NB][2];
#pragma unroll
        for (int uu = 0; uu < UNR; ++uu) {
            const int kb = kb0 + 4 * uu;
#pragma unroll
            for (int lb = 0; lb < NB; ++lb) {
                raw[uu][lb][0] = raw[uu][lb][1] = make_uint4(0u, 0u, 0u, 0u);
                if (lok[lb] && kb < NKB) {
                    const uint4 *s4 = reinterpret_cast<const uint4 *>(src[lb] + (size_t)kb * 2048);
                    raw[uu][lb][0] = s4[0];
                    raw[uu][lb][1] = s4[1];
                }
            }
        }
#pragma unroll
        for (int uu = 0; uu < UNR; ++uu) {
            int a = 0;
#pragma unroll
            for (int bi = 0; bi < NB; ++bi)
#pragma unroll
                for (int bj = 0; bj <= bi; ++bj, ++a)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[a] = __builtin_amdgcn_mfma_f32_32x32x16_f16(
                            __builtin_bit_cast(f16x8, raw[uu][bi][j]), __builtin_bit_cast(f16x8, raw[uu][bj][j]),
                            acc[a], 0, 0, 0);
        }
    }
    // the four waves' sums, added in wave order: result element v of lane (m, kg) is
    // G[bi*32 + 8*(v/4) + 4*kg + v%4][bj*32 + m]
    for (int round = 0; round < 4; ++round) {
        __syncthreads();
        if (w == round) {
            int a = 0;
#pragma unroll
            for (int bi = 0; bi < NB; ++bi)
#pragma unroll
                for (int bj = 0; bj <= bi; ++bj, ++a)
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        G[(bi * 32 + 8 * (v >> 2) + 4 * kg + (v & 3)) * Lp + bj * 32 + m] += acc[a][v];
        }
    }
    __syncthreads();
    const float *Z = p.rowZ + (size_t)rowl * L;
    float *oc = p.row_cos + (size_t)rowl * L * L;
    float *od = p.row_dist + (size_t)rowl * L * L;
    for (int e = tid; e < L * L; e += kThreads) {
        const int i = e / L, j = e % L;
        if (i <= j) continue;
        const float gij = G[i * Lp + j], gii = G[i * Lp + i], gjj = G[j * Lp + j];
        oc[e] = gij * rsqrtf(gii * gjj);
        if (p.want_dist) {
            const float zi = 1.f / Z[i], zj = 1.f / Z[j];
            od[e] = sqrtf(fmaxf(gii * zi * zi + gjj * zj * zj - 2.f * gij * zi * zj, 0.f));
        }
    }
}

// ------------------------------------------------------------------------------------------------
// 3. rows -> head sums (one workgroup column per (unit of the batch, head of the group))
__global__ __launch_bounds__(kThreads) void ap_reduce_kernel(APParams p, int u0)
{
    const int LL = p.L * p.L;
    const int e = blockIdx.y * kThreads + threadIdx.x;
    const int hg = blockIdx.x % p.g, u = u0 + blockIdx.x / p.g;
    // rows of unit u that this batch holds, and those of them that belong to head hg
    const int rg_lo = max(p.grg0, u * p.NRG) - u * p.NRG;
    const int rg_hi = min(p.grg0 + p.nrg, (u + 1) * p.NRG) - u * p.NRG;
    const int r_lo = max(rg_lo * kRowsPerGroup, hg * p.Tq);
    const int r_hi = min(min(rg_hi * kRowsPerGroup, p.Rk), (hg + 1) * p.Tq);
    if (e >= LL || r_lo >= r_hi) return;
    const int i = e / p.L, j = e % p.L;
    if (i <= j) return;
    const int b = u / p.Hkv, hq = (u % p.Hkv) * p.g + hg;
    const size_t o = ((size_t)b * p.Hq + hq) * LL + e;
    // the rows are added one by one to the running sum, so that the result does not depend on where
    // the batches are cut
    float cs = p.head_cos[o], ds = p.want_dist ? p.head_dist[o] : 0.f;
    for (int r = r_lo; r < r_hi; ++r) {
        const size_t rowl = (size_t)(u * p.NRG + r / kRowsPerGroup - p.grg0) * kRowsPerGroup + r % kRowsPerGroup;
        cs += p.row_cos[rowl * LL + e];
        if (p.want_dist) ds += p.row_dist[rowl * LL + e];
    }
    p.head_cos[o] = cs;
    if (p.want_dist) p.head_dist[o] = ds;
}

__global__ void ap_fill_kernel(float *ptr, size_t n, float v)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) ptr[i] = v;
}

// head sums -> means over tokens, average over heads, mirrored matrices with cos 1 / distance 0 on
// the diagonal.  One thread per (conversation, i, j).
__global__ void ap_final_kernel(int B, int L, int Hq, float inv_tokens, const float *__restrict__ head_cos,
                                const float *__restrict__ head_dist, float *__restrict__ pair_cos,
                                float *__restrict__ pair_dist, float *__restrict__ head_out)
{
    const int LL = L * L;
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)B * LL) return;
    const int b = (int)(idx / LL), e = (int)(idx % LL), i = e / L, j = e % L;
    const int lo = i > j ? e : j * L + i;   // the entry below the diagonal holds the sums
    float cs = 0.f, ds = 0.f;
    for (int h = 0; h < Hq; ++h) {
        const size_t o = ((size_t)b * Hq + h) * LL;
        const float c = i == j ? 1.f : head_cos[o + lo] * inv_tokens;
        cs += c;
        if (head_out) head_out[o + e] = c;
        if (pair_dist) ds += i == j ? 0.f : head_dist[o + lo] * inv_tokens;
    }
    pair_cos[idx] = cs / (float)Hq;
    if (pair_dist) pair_dist[idx] = ds / (float)Hq;
}

// ------------------------------------------------------------------------------------------------
// Greedy choice over all candidate pairs: n_select rounds of "best free pair", which is what one
// scan of the stably sorted list takes.  Order: key ascending (distance, or minus similarity),
// equal keys by lower j, then lower i.
constexpr int kSelThreads = 256;

__global__ __launch_bounds__(kSelThreads) void select_all_kernel(
    const float *__restrict__ score, int closer_is_smaller, const uint8_t *__restrict__ eligible,
    int L, int n_select, int32_t *__restrict__ out_pairs, int32_t *__restrict__ out_count)
{
    extern __shared__ unsigned char sm[];
    uint8_t *used = sm;                                                      // [L]: shared already, or not eligible
    float *bkey = reinterpret_cast<float *>(sm + ((L + 15) & ~15));          // [waves]
    int *brank = reinterpret_cast<int *>(bkey + kSelThreads / 64);           // [waves]
    __shared__ int chosen;
    const int b = blockIdx.x, tid = threadIdx.x;
    const float *sc = score + (size_t)b * L * L;
    for (int l = tid; l < L; l += kSelThreads) used[l] = eligible ? (eligible[(size_t)b * L + l] ? 0 : 1) : 0;
    __syncthreads();
    int cnt = 0;
    for (; cnt < n_select; ++cnt) {
        float best = INFINITY;
        int rank = INT32_MAX;   // j * L + i of the best candidate
        for (int e = tid; e < L * L; e += kSelThreads) {
            const int i = e / L, j = e % L;
            if (i <= j || used[i] || used[j]) continue;
            const float key = closer_is_smaller ? sc[e] : -sc[e];
            const int rk = j * L + i;
            if (rank == INT32_MAX || key < best || (key == best && rk < rank)) {
                best = key;
                rank = rk;
            }
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const float ob = __shfl_xor(best, o, 64);
            const int orank = __shfl_xor(rank, o, 64);
            if (orank != INT32_MAX && (rank == INT32_MAX || ob < best || (ob == best && orank < rank))) {
                best = ob;
                rank = orank;
            }
        }
        if ((tid & 63) == 0) {
            bkey[tid >> 6] = best;
            brank[tid >> 6] = rank;
        }
        __syncthreads();
        if (tid == 0) {
            float kb = bkey[0];
            int rk = brank[0];
            for (int wv = 1; wv < kSelThreads / 64; ++wv)
                if (brank[wv] != INT32_MAX && (rk == INT32_MAX || bkey[wv] < kb || (bkey[wv] == kb && brank[wv] < rk))) {
                    kb = bkey[wv];
                    rk = brank[wv];
                }
            chosen = rk;
            if (rk != INT32_MAX) {
                const int j = rk / L, i = rk % L;
                used[i] = used[j] = 1;
                out_pairs[((size_t)b * n_select + cnt) * 2] = j;
                out_pairs[((size_t)b * n_select + cnt) * 2 + 1] = i;
            }
        }
        __syncthreads();
        if (chosen == INT32_MAX) break;   // no free candidate is left
        __syncthreads();
    }
    if (tid == 0) {
        out_count[b] = cnt;
        for (int a = cnt; a < n_select; ++a)
            out_pairs[((size_t)b * n_select + a) * 2] = out_pairs[((size_t)b * n_select + a) * 2 + 1] = -1;
    }
}

size_t align_up(size_t v) { return (v + 255) & ~(size_t)255; }

struct APPlan {
    int NRG, NKB, total_rg, nrg_batch;
    size_t head_cos_off, head_dist_off, rowz_off, row_cos_off, row_dist_off, e_off, total_bytes;
    bool mfma;
};

// Sizes for a batch of nrg row groups.
void ap_layout(const krul_shape_t *s, int nrg, APPlan *pl)
{
    const size_t L = s->n_layers, LL = L * L;
    const size_t heads = (size_t)s->batch * s->n_q_heads * LL * sizeof(float);
    const size_t rows = (size_t)nrg * kRowsPerGroup;
    size_t off = 0;
    pl->head_cos_off = off; off += align_up(heads);
    pl->head_dist_off = off; off += align_up(heads);
    pl->rowz_off = off; off += align_up(rows * L * sizeof(float));
    pl->row_cos_off = off; off += align_up(rows * LL * sizeof(float));
    pl->row_dist_off = off; off += align_up(rows * LL * sizeof(float));
    pl->e_off = off; off += align_up((size_t)nrg * 4 * L * pl->NKB * 2048);
    pl->total_bytes = off;
    pl->nrg_batch = nrg;
}

constexpr int kMaxLayersAllPairs = 128;
constexpr size_t kDefaultBudget = (size_t)2 << 30;

// Validate and size: the largest batch of row groups whose workspace fits max_bytes (0: a default
// budget), at least one group.  Returns a krul_status_t.
int ap_plan(const krul_shape_t *s, size_t max_bytes, APPlan *pl)
{
    const int rc = check_shape(s);
    if (rc != KRUL_OK) return rc;
    if (s->n_layers > kMaxLayersAllPairs) return KRUL_EUNSUPPORTED;
    const long long g = s->n_q_heads / s->n_kv_heads, Rk = g * s->n_query;
    if (Rk > INT32_MAX || (long long)s->batch * s->n_q_heads * s->n_query > INT32_MAX) return KRUL_EUNSUPPORTED;
    pl->NRG = (int)((Rk + kRowsPerGroup - 1) / kRowsPerGroup);
    pl->NKB = (s->n_hist + 31) / 32;
    const long long total = (long long)s->batch * s->n_kv_heads * pl->NRG;
    if (total * kRowsPerGroup > INT32_MAX / 4) return KRUL_EUNSUPPORTED;
    pl->total_rg = (int)total;
    pl->mfma = s->dtype == KRUL_BF16 && (s->head_dim == 64 || s->head_dim == 128) &&
               !(s->flags & KRUL_FLAG_GENERIC_KERNEL);
    if (s->n_hist * (long long)s->head_dim * 4 >= (1ll << 31)) return KRUL_EUNSUPPORTED;
    const size_t budget = max_bytes ? max_bytes : kDefaultBudget;
    ap_layout(s, 1, pl);
    const size_t fixed = pl->rowz_off;   // the head sums do not grow with the batch
    const size_t per_group = pl->total_bytes - fixed;
    long long nrg = budget > fixed ? (long long)((budget - fixed) / per_group) : 0;
    if (nrg < 1) nrg = 1;
    if (nrg > total) nrg = total;
    ap_layout(s, (int)nrg, pl);
    while (pl->total_bytes > budget && nrg > 1) ap_layout(s, (int)--nrg, pl);   // (alignment padding)
    return KRUL_OK;
}

}  // namespace

size_t all_pairs_workspace(const krul_shape_t *s, size_t max_bytes)
{
    APPlan pl;
    if (ap_plan(s, max_bytes, &pl) != KRUL_OK) return 0;
    return pl.total_bytes;
}

int run_all_pairs(const krul_shape_t *s, const void *q, const void *k, float *pair_score, float *pair_dist,
                  float *head_score, void *workspace, size_t workspace_bytes, hipStream_t st)
{
    APPlan pl;
    int rc = ap_plan(s, 0, &pl);
    if (rc != KRUL_OK) return rc;
    if (!q || !k || !pair_score) return KRUL_EINVAL;
    if (((uintptr_t)q | (uintptr_t)k) & 15) return KRUL_EINVAL;
    if (((uintptr_t)pair_score | (uintptr_t)pair_dist | (uintptr_t)head_score) & 3) return KRUL_EINVAL;
    if (!workspace || ((uintptr_t)workspace & 255)) return KRUL_EWORKSPACE;
    // the batch is what the caller's workspace holds: the smallest (one row group) must fit
    {
        APPlan one = pl;
        ap_layout(s, 1, &one);
        if (workspace_bytes < one.total_bytes) return KRUL_EWORKSPACE;
        rc = ap_plan(s, workspace_bytes, &pl);
        if (rc != KRUL_OK) return rc;
        if (pl.total_bytes > workspace_bytes) return KRUL_EWORKSPACE;
    }
    unsigned char *ws = static_cast<unsigned char *>(workspace);
    APParams p;
    p.q = q;
    p.k = k;
    p.B = s->batch;
    p.L = s->n_layers;
    p.Hq = s->n_q_heads;
    p.Hkv = s->n_kv_heads;
    p.g = p.Hq / p.Hkv;
    p.d = s->head_dim;
    p.S = s->n_hist;
    p.Tq = s->n_query;
    p.Rk = p.g * p.Tq;
    p.causal = (s->flags & KRUL_FLAG_CAUSAL) != 0;
    const float scale = s->scale > 0.f ? s->scale : 1.0f / sqrtf((float)s->head_dim);
    p.c = scale * 1.4426950408889634f;
    p.NRG = pl.NRG;
    p.NKB = pl.NKB;
    p.want_dist = pair_dist != nullptr;
    p.E = ws + pl.e_off;
    p.rowZ = reinterpret_cast<float *>(ws + pl.rowz_off);
    p.row_cos = reinterpret_cast<float *>(ws + pl.row_cos_off);
    p.row_dist = reinterpret_cast<float *>(ws + pl.row_dist_off);
    p.head_cos = reinterpret_cast<float *>(ws + pl.head_cos_off);
    p.head_dist = reinterpret_cast<float *>(ws + pl.head_dist_off);

    const int L = p.L, LL = L * L;
    const size_t n_head = (size_t)p.B * p.Hq * LL;
    hipLaunchKernelGGL(ap_fill_kernel, dim3((unsigned)((n_head + 255) / 256)), dim3(256), 0, st, p.head_cos, n_head, 0.f);
    if (p.want_dist)
        hipLaunchKernelGGL(ap_fill_kernel, dim3((unsigned)((n_head + 255) / 256)), dim3(256), 0, st, p.head_dist, n_head, 0.f);
    if (hipGetLastError() != hipSuccess) return KRUL_ELAUNCH;

    const int NB = (L + 31) / 32;
    const size_t gram_smem = (size_t)(32 * NB) * (32 * NB) * sizeof(float);
    for (int g0 = 0; g0 < pl.total_rg; g0 += pl.nrg_batch) {
        p.grg0 = g0;
        p.nrg = pl.nrg_batch < pl.total_rg - g0 ? pl.nrg_batch : pl.total_rg - g0;
        const int rows = p.nrg * kRowsPerGroup;
        if (pl.mfma) {
            if (p.d == 128)
                hipLaunchKernelGGL(ap_weights_mfma_kernel<128>, dim3(p.nrg * L), dim3(kThreads), 0, st, p);
            else
                hipLaunchKernelGGL(ap_weights_mfma_kernel<64>, dim3(p.nrg * L), dim3(kThreads), 0, st, p);
        } else if (s->dtype == KRUL_F32) {
            hipLaunchKernelGGL(ap_weights_generic_kernel<float>, dim3(rows * L), dim3(64), p.d * sizeof(float), st, p);
        } else {
            hipLaunchKernelGGL(ap_weights_generic_kernel<uint16_t>, dim3(rows * L), dim3(64), p.d * sizeof(float), st, p);
        }
        switch (NB) {
        case 1: hipLaunchKernelGGL(ap_gram_kernel<1>, dim3(rows), dim3(kThreads), gram_smem, st, p); break;
        case 2: hipLaunchKernelGGL(ap_gram_kernel<2>, dim3(rows), dim3(kThreads), gram_smem, st, p); break;
        case 3: hipLaunchKernelGGL(ap_gram_kernel<3>, dim3(rows), dim3(kThreads), gram_smem, st, p); break;
        default: hipLaunchKernelGGL(ap_gram_kernel<4>, dim3(rows), dim3(kThreads), gram_smem, st, p); break;
        }
        const int u0 = g0 / p.NRG, u1 = (g0 + p.nrg - 1) / p.NRG;
        hipLaunchKernelGGL(ap_reduce_kernel, dim3((u1 - u0 + 1) * p.g, (LL + kThreads - 1) / kThreads), dim3(kThreads),
                           0, st, p, u0);
        if (hipGetLastError() != hipSuccess) return KRUL_ELAUNCH;
    }
    const size_t n_out = (size_t)p.B * LL;
    hipLaunchKernelGGL(ap_final_kernel, dim3((unsigned)((n_out + 255) / 256)), dim3(256), 0, st, p.B, L, p.Hq,
                       1.0f / (float)p.Tq, p.head_cos, p.head_dist, pair_score, pair_dist, head_score);
    return hipGetLastError() == hipSuccess ? KRUL_OK : KRUL_ELAUNCH;
}

hipError_t launch_select_all(const float *score, int closer_is_smaller, const uint8_t *eligible, int batch,
                             int n_layers, int n_select, int32_t *out_pairs, int32_t *out_count, hipStream_t st)
{
    const size_t smem = ((n_layers + 15) & ~15) + (kSelThreads / 64) * (sizeof(float) + sizeof(int));
    hipLaunchKernelGGL(select_all_kernel, dim3(batch), dim3(kSelThreads), smem, st, score, closer_is_smaller,
                       eligible, n_layers, n_select, out_pairs, out_count);
    return hipGetLastError();
}

}  // namespace krul
