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
//   1. weights kernel: a workgroup owns a row group of a unit -- 1, 2, 4 or 8 32-row blocks with
//      the rows a kv head has: up to four waves, each with one or two blocks --, one layer, and a
//      run of key splits of 128 keys.  Per split: the keys go to one of two XOR-swizzled LDS
//      buffers by buffer_load ... lds (the next split's are already in flight), one barrier,
//      v_mfma_f32_32x32x16_bf16 logits of all 128 keys into registers, their maximum m (one exchange
//      between the two half-waves: a wave owns all 128 keys of its 32 rows), e = 2^(x - m) <= 1,
//      Z = sum e, and the fp16 store of e.  m and Z are kept per (row, layer, split).
//      Layout of E: [32-row block][32-key block][layer][row][32 x fp16]: the 2 KB that a wave's
//      result block covers are contiguous (full-line stores), the L x 2 KB of a key block are
//      contiguous for the Gram kernel, and the 64 bytes of one (row, layer, key block) are what one
//      Gram operand fetch reads.  Inside the 64 bytes the keys stand in the order of the MFMA result
//      registers; the order is the same for all layers of a row, which is all a contraction over
//      the keys needs.
//   2. scale kernel: per (row, layer) the splits' exponents are replaced by their factors to the
//      largest, 2^(m_s - max), and Z is summed at that common exponent.
//   3. Gram kernel: a workgroup takes the rows of a 32-row block (each wave a few) and a range of
//      key blocks; v_mfma_f32_32x32x16_f16 with A = B = the row's [32 layers x 16 keys] piece
//      (lane = layer) scaled by the split's factor, one accumulator block per pair of 32-layer
//      blocks; the partial matrices of the key ranges are written out.
//   4. row kernel: per row the partial matrices are added in order; cos_ij = G_ij / sqrt(G_ii G_jj)
//      and dist_ij^2 = G_ii/Z_i^2 + G_jj/Z_j^2 - 2 G_ij/(Z_i Z_j).
//   5. reduce kernel: per (unit, head of the group) the batch's rows are added, one by one, to the
//      head sums (so the result does not depend on the batch size); the last kernel divides by the
//      token count, averages the heads (Sec. 4.2) and mirrors the matrix.
// A portable weights kernel (one wave per row and layer, fp32 dot products, no key splits) covers
// fp32 inputs and other head sizes; it writes the same layout.
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

constexpr int kThreads = 256;
constexpr int kDumpBlocks = 128;     // 2 KB blocks of the area that takes stores with no place of their own
constexpr int kKeysPerSplit = 128;   // keys of one step of a weights-kernel workgroup (an LDS buffer)

struct APParams {
    const void *q;
    const void *k;
    int B, L, Hq, Hkv, g, d, S, Tq, Rk;
    int causal;
    KeyAddr ka;         // where the keys are (dense: ka.k; in place: per-layer table, strides, pages)
    float c;            // scale * log2(e)
    int NW;             // 32-row blocks per row group (1, 2, 4 or 8: the waves of a weights-kernel workgroup
                        // times the blocks each takes)
    int NRG;            // row groups per unit
    int NKB;            // 32-key blocks per row
    int nsplit, kps;    // key splits of the weights kernel, keys per split (a multiple of 32)
    int tpw;            // key splits that one weights-kernel workgroup walks
    int grg0, nrg;      // this batch: global row groups [grg0, grg0 + nrg)
    int want_dist;
    unsigned char *dump;   // [kDumpBlocks][2 KB]
    unsigned char *E;   // [nrg*NW][NKB][L][32][64 bytes]; e = 2^(x - m) with m of the row, layer and key split
    float *rowM;        // [nrg*NW*32][nsplit][L]  reference exponent m; then the factor 2^(m - largest m of the row, layer)
    float *rowZ;        // [nrg*NW*32][nsplit][L]  sum of e over the split's keys
    float *rowZt;       // [nrg*NW*32][L]          1 / (sum of e over all keys, at the common exponent)
    float *Gpart;       // [nrg*NW*32][ksp][NACC*1024] partial Gram matrices, result-register order
    float *row_cos;     // [nrg*NW*32][L*L]  (entries i > j)
    float *row_dist;    // same, or unused
    float *head_cos;    // [B][Hq][kClasses][L*L] running sums over the rows of a head, by class of token index
    float *head_dist;
};

__device__ inline size_t e_block_offset(const APParams &p, int rbl, int l, int kb)
{
    return ((((size_t)rbl * p.NKB + kb) * p.L + l) * 32) * 64;
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
// NW waves, each with RB 32-row blocks (taken one after the other against the same keys in LDS): a
// row group is NW*RB blocks.
// INPLACE: the keys are read where the caller keeps them (one allocation or page pool per layer, strides,
// a block table) instead of from the dense layout.
template <int D, int NW, int RB, bool F16, bool INPLACE>
__global__ __launch_bounds__(NW * 64, NW == 4 ? 2 : 1) void ap_weights_mfma_kernel(APParams p)
{
    constexpr int KS = D / 16, ROWB = D * 2, KR = kKeysPerSplit, NKBW = KR / 32;
    [[maybe_unused]] constexpr int PPR = D / 8;
    __shared__ __attribute__((aligned(16))) unsigned char kl[2][KR * ROWB];

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, half = lane >> 5, n = lane & 31;
    const int nkc = (p.nsplit + p.tpw - 1) / p.tpw;   // workgroups along the keys
    // key chunks vary fastest, then layers: the workgroups that run at the same time fill one row
    // group's part of E densely (the order with the row groups fastest, which would share the keys
    // between them, measured 20 % slower)
    const int kc = blockIdx.x % nkc;
    const int l = (blockIdx.x / nkc) % p.L;
    const int rgl = blockIdx.x / (nkc * p.L);
    const int grg = p.grg0 + rgl;
    const int u = grg / p.NRG, rg = grg % p.NRG;
    const int b = u / p.Hkv, kvh = u % p.Hkv;
    const int S = p.S;
    int rbl[RB], row_end[RB];
    bool row_ok[RB];
#pragma unroll
    for (int j = 0; j < RB; ++j) {
        rbl[j] = (rgl * NW + w) * RB + j;
        const int r = ((rg * NW + w) * RB + j) * 32 + n;   // row of the unit: head-in-group * Tq + t
        row_ok[j] = r < p.Rk;
        row_end[j] = row_ok[j] ? (p.causal ? S - p.Tq + r % p.Tq + 1 : S) : 0;   // keys [0, row_end) are seen
    }

    // This workgroup walks the key splits [t0, t1) of its rows and layer, KR keys each.  The keys of
    // split t+1 are copied into the other LDS buffer while split t is worked on.
    const int t0 = kc * p.tpw, t1 = min(p.nsplit, t0 + p.tpw);
    // dense: this unit's keys of layer l; in place: the layer's allocation at this unit's kv head (and
    // conversation, unless a block table says where its keys are)
    typedef const __attribute__((address_space(4))) unsigned long long *const_u64_ptr;   // constant memory: scalar loads
    typedef const __attribute__((address_space(4))) int *const_i32_ptr;
    [[maybe_unused]] const uint16_t *klayer =
        INPLACE ? (p.ka.k_tab ? (const uint16_t *)(uintptr_t)((const_u64_ptr)(uintptr_t)p.ka.k_tab)[l]
                              : static_cast<const uint16_t *>(p.ka.k) + (size_t)l * p.ka.stride_l) +   // (dense, head size below D)
                      (size_t)kvh * p.ka.stride_h + (p.ka.block_table ? 0 : (size_t)b * p.ka.stride_b)
                : static_cast<const uint16_t *>(p.k) + ((((size_t)b * p.L + l) * p.Hkv + kvh) * (size_t)S) * D;
    [[maybe_unused]] const unsigned k_row_bytes = INPLACE ? (unsigned)p.ka.stride_s * 2u : (unsigned)ROWB;
    // head size in memory (INPLACE: any multiple of 8 up to D; the pieces a shorter row does not have are left
    // to lanes whose offset lies past every range: they fetch nothing and write zero)
    [[maybe_unused]] const int dq = INPLACE ? p.d : D;
    [[maybe_unused]] const unsigned d_bytes = (unsigned)dq * 2u, pp_real = (unsigned)dq >> 3;
    constexpr unsigned kNoFetch = 0x7FFFFFF0u;
    // The keys go HBM -> LDS directly (buffer_load ... lds, no staging registers):
    // wave-instruction j fills the 1 KB at j*1024 (RPI key rows), lane by lane, so each lane fetches
    // the 16-byte piece that belongs at its LDS position (the XOR swizzle applied on the global
    // side); rows past the split's end are outside the descriptor's range and read as zero.
    auto copy_keys = [&](int t, int buf) __attribute__((always_inline)) {
#if defined(__HIP_DEVICE_COMPILE__)   // (the host pass only needs the kernel's launch stub)
        constexpr int RPI = 64 / PPR, NI = KR / RPI / NW;
        const int kn = min(KR, S - t * KR);
        if constexpr (INPLACE) {
            if (p.ka.block_table) {
                // pages: a copy instruction's RPI keys lie in one page (pages hold a power of two >= 8 keys);
                // it looks its page up (scalar load) and gets a descriptor of its own: all its keys or none
                // (a page has room for all its keys; the ones past the last are masked like any unseen key)
                const const_i32_ptr page_row = (const_i32_ptr)(uintptr_t)(p.ka.block_table + (size_t)b * p.ka.max_blocks);
#pragma unroll
                for (int jj = 0; jj < NI; ++jj) {
                    const int j = __builtin_amdgcn_readfirstlane(w) * NI + jj;
                    const int krow = t * KR + j * RPI, kcl = min(krow, S - 1);
                    const uint16_t *base = klayer + (size_t)page_row[kcl >> p.ka.page_shift] * p.ka.stride_page +
                                           (size_t)(kcl & ((1 << p.ka.page_shift) - 1)) * p.ka.stride_s;
                    const unsigned bytes = krow < S ? (unsigned)(RPI - 1) * k_row_bytes + d_bytes : 0u;
                    const __amdgpu_buffer_rsrc_t rsrc =
                        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(base), 0, (int)bytes, 0x00020000);
                    const int row = j * RPI + lane / PPR;
                    const unsigned pj = (unsigned)((lane % PPR) ^ swz<D>(row));
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(
                        rsrc, (__attribute__((address_space(3))) void *)(&kl[buf][0] + j * 1024), 16,
                        (int)(pj < pp_real ? (unsigned)(lane / PPR) * k_row_bytes + (pj << 4) : kNoFetch), 0, 0, 0);
                }
            } else {
                // strides: one descriptor for the split, the row pitch a run-time value
                const uintptr_t ka = (uintptr_t)(klayer + (size_t)t * KR * p.ka.stride_s);
                const uint16_t *kb_u = (const uint16_t *)(((uintptr_t)(unsigned)__builtin_amdgcn_readfirstlane((int)(ka >> 32)) << 32) |
                                                          (uintptr_t)(unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)ka));
                const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
                    const_cast<uint16_t *>(kb_u), 0,
                    __builtin_amdgcn_readfirstlane(kn > 0 ? (int)((unsigned)(kn - 1) * k_row_bytes + d_bytes) : 0), 0x00020000);
#pragma unroll
                for (int jj = 0; jj < NI; ++jj) {
                    const int j = __builtin_amdgcn_readfirstlane(w) * NI + jj;
                    const int row = j * RPI + lane / PPR;
                    const unsigned pj = (unsigned)((lane % PPR) ^ swz<D>(row));
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(
                        rsrc, (__attribute__((address_space(3))) void *)(&kl[buf][0] + j * 1024), 16,
                        (int)(pj < pp_real ? (unsigned)row * k_row_bytes + (pj << 4) : kNoFetch), 0, 0, 0);
                }
            }
            return;
        }
        const uintptr_t ka = (uintptr_t)(klayer + (size_t)t * KR * D);   // wave-uniform: a scalar descriptor
        const uint16_t *kb_u = (const uint16_t *)(((uintptr_t)(unsigned)__builtin_amdgcn_readfirstlane((int)(ka >> 32)) << 32) |
                                                  (uintptr_t)(unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)ka));
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint16_t *>(kb_u), 0, __builtin_amdgcn_readfirstlane(kn * ROWB), 0x00020000);
#pragma unroll
        for (int jj = 0; jj < NI; ++jj) {
            const int j = __builtin_amdgcn_readfirstlane(w) * NI + jj;
            const int row = j * RPI + lane / PPR, pos = lane % PPR;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(
                rsrc, (__attribute__((address_space(3))) void *)(&kl[buf][0] + j * 1024), 16,
                row * ROWB + ((pos ^ swz<D>(row)) << 4), 0, 0, 0);
        }
#endif
    };
    copy_keys(t0, 0);
    // query rows of a unit are contiguous in r: [b][l][kvh*g + r / Tq][r % Tq][D]
    const uint16_t *Qg = static_cast<const uint16_t *>(p.q);
    bf16x8 qf[RB][KS];
#pragma unroll
    for (int j = 0; j < RB; ++j) {
        const int r = ((rg * NW + w) * RB + j) * 32 + n;
        const uint16_t *qrow = Qg + ((((size_t)b * p.L + l) * p.Hq + (size_t)kvh * p.g) * p.Tq + (size_t)(row_ok[j] ? r : 0)) * dq;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            uint4 v = make_uint4(0u, 0u, 0u, 0u);   // (zero: rows that do not exist, elements past the head size)
            if (row_ok[j] && ks * 16 + half * 8 < dq) v = *reinterpret_cast<const uint4 *>(qrow + ks * 16 + half * 8);
            qf[j][ks] = __builtin_bit_cast(bf16x8, v);
        }
    }

    // The query rows and the first split's keys have arrived before the loop starts.  Inside it a
    // split's copy is followed by the RB*kStores stores of the split before it, all unconditional
    // (addresses are redirected instead); memory operations complete in the order issued, so "at
    // most kStores - 2 outstanding" means this wave's part of split t has landed, without waiting
    // for the newest stores.
    constexpr int kStores = 2 * NKBW + 2;
    static_assert(kStores - 2 == 8, "the wait below is written for eight");
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
    for (int t = t0; t < t1; ++t) {
        const int buf = (t - t0) & 1;
        __builtin_amdgcn_s_waitcnt(0x0F78);   // vmcnt(8)
        // the keys of split t are in LDS; every wave has finished reading the other buffer (split t-1)
        __syncthreads();
        if (t + 1 < t1) copy_keys(t + 1, buf ^ 1);

        const int k0 = t * KR, kn = min(KR, S - k0), nkb = (kn + 31) / 32;
#pragma unroll
        for (int j = 0; j < RB; ++j) {
        // logits of the 32 keys of block kb against this wave's 32 rows: lane (n, half) gets row n,
        // keys 8*(v/4) + 4*half + v%4 of the block; keys the row does not see are set to -inf.  The
        // logits of all KR keys stay in registers between the maximum and the exponentials.
        f32x16 x[NKBW];
        float mx = -INFINITY;
#pragma unroll
        for (int kb = 0; kb < NKBW; ++kb) {
            {
                f32x16 a;
#pragma unroll
                for (int v = 0; v < 16; ++v) a[v] = 0.f;
                const int row = kb * 32 + n;
                const unsigned char *rp = &kl[buf][row * ROWB];
                bf16x8 ka[KS];   // all operand reads first: one LDS latency per block, not one per MFMA
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
                    ka[ks] = *reinterpret_cast<const bf16x8 *>(rp + (((2 * ks + half) ^ swz<D>(row)) << 4));
                // (the empty statements keep the compiler from moving the reads back between the MFMAs)
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(ka[ks]));
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    if constexpr (F16)   // IEEE binary16 inputs: same layout, same rate
                        a = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, ka[ks]),
                                                                   __builtin_bit_cast(f16x8, qf[j][ks]), a, 0, 0, 0);
                    else
                        a = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[ks], qf[j][ks], a, 0, 0, 0);
                }
                const int key0 = k0 + kb * 32;
                if (__any(key0 + 32 > row_end[j])) {   // some row of the wave does not see all 32 keys
                    const int lim = row_end[j] - key0 - 4 * half;
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        if (8 * (v >> 2) + (v & 3) >= lim) a[v] = -INFINITY;
                }
#pragma unroll
                for (int v = 0; v < 16; ++v) mx = fmaxf(mx, a[v]);
                x[kb] = a;
            }
        }
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        // (c > 0: the largest logit gives the largest exponent.)  A row that sees none of this split's
        // keys (causal reading) gets e = 0 everywhere and the "no key yet" exponent.
        const float M = mx > -INFINITY ? mx * p.c : 0.f;
        float z = 0.f;
#pragma unroll
        for (int kb = 0; kb < NKBW; ++kb) {
            {
                uint32_t pk[8];
#pragma unroll
                for (int v = 0; v < 16; v += 2) {
                    const float e0 = __builtin_amdgcn_exp2f(fmaf(x[kb][v], p.c, -M));
                    const float e1 = __builtin_amdgcn_exp2f(fmaf(x[kb][v + 1], p.c, -M));
                    z += e0 + e1;
                    pk[v >> 1] = pack_f16(e0, e1);
                }
                // a block past the last key has no place in E: its zeros go to a dump area.  Rows
                // that do not exist (and the blocks of a wave without rows) have theirs and are
                // never read.
                unsigned char *blk = kb < nkb ? p.E + e_block_offset(p, rbl[j], l, t * NKBW + kb)
                                              : p.dump + (size_t)((blockIdx.x * NW + w) & (kDumpBlocks - 1)) * 2048;
                uint4 *dst = reinterpret_cast<uint4 *>(blk + n * 64 + half * 32);
                dst[0] = make_uint4(pk[0], pk[1], pk[2], pk[3]);
                dst[1] = make_uint4(pk[4], pk[5], pk[6], pk[7]);
            }
        }
        z += __shfl_xor(z, 32, 64);
        {   // (both half-waves hold the same values and write them to the same place)
            const size_t o = (((size_t)rbl[j] * 32 + n) * p.nsplit + t) * p.L + l;
            p.rowM[o] = mx > -INFINITY ? M : kMInit;
            p.rowZ[o] = z;
        }
        }
    }
}


// Portable weights kernel: one wave per (row of the batch, layer); lane = key.
template <typename T>
__device__ inline float load_f32(const T *ptr, size_t i);
template <>
__device__ inline float load_f32<float>(const float *ptr, size_t i) { return ptr[i]; }
template <>
__device__ inline float load_f32<uint16_t>(const uint16_t *ptr, size_t i) { return __uint_as_float((uint32_t)ptr[i] << 16); }
template <>
__device__ inline float load_f32<_Float16>(const _Float16 *ptr, size_t i) { return (float)ptr[i]; }

template <typename T>
__global__ __launch_bounds__(64) void ap_weights_generic_kernel(APParams p)
{
    extern __shared__ float qs[];   // [d]
    const int lane = threadIdx.x;
    const int l = blockIdx.x % p.L;
    const int rowl = blockIdx.x / p.L;
    const int rbl = rowl >> 5, n = rowl & 31;
    const int grb = p.grg0 * p.NW + rbl;
    const int u = grb / (p.NRG * p.NW), rb = grb % (p.NRG * p.NW);
    const int r = rb * 32 + n;
    if (r >= p.Rk) return;
    const int b = u / p.Hkv, kvh = u % p.Hkv;
    const int hq = kvh * p.g + r / p.Tq, t = r % p.Tq;
    const int S = p.S, d = p.d;
    const int row_end = p.causal ? S - p.Tq + t + 1 : S;
    const T *Q = static_cast<const T *>(p.q);
    const T *K = p.ka.k_tab ? static_cast<const T *>(p.ka.k_tab[l]) : static_cast<const T *>(p.ka.k) + (size_t)l * p.ka.stride_l;
    const size_t qoff = ((((size_t)b * p.L + l) * p.Hq + hq) * p.Tq + t) * d;
    auto key_off = [&](int key) -> size_t {   // (see KeyAddr)
        if (p.ka.block_table)
            return (size_t)p.ka.block_table[(size_t)b * p.ka.max_blocks + (key >> p.ka.page_shift)] * p.ka.stride_page +
                   (size_t)kvh * p.ka.stride_h + (size_t)(key & ((1 << p.ka.page_shift) - 1)) * p.ka.stride_s;
        return (size_t)b * p.ka.stride_b + (size_t)kvh * p.ka.stride_h + (size_t)key * p.ka.stride_s;
    };
    for (int i = lane; i < d; i += 64) qs[i] = load_f32<T>(Q, qoff + i);
    __syncthreads();

    auto logit = [&](int key) -> float {
        float acc = 0.f;
        const size_t koff = key_off(key);
        for (int i = 0; i < d; ++i) acc = fmaf(qs[i], load_f32<T>(K, koff + i), acc);
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
    if (lane == 0) {   // (this kernel does not split the keys: nsplit is 1)
        p.rowM[((size_t)rbl * 32 + n) * p.L + l] = mx;
        p.rowZ[((size_t)rbl * 32 + n) * p.L + l] = z;
    }
}

// 2. The key splits' exponents of a (row, layer) are replaced by their factors
// against the largest, 2^(m_s - max m), and Z is summed at that common exponent.  One workgroup
// per row of the batch.
__global__ __launch_bounds__(kThreads) void ap_scale_kernel(APParams p)
{
    __shared__ float red[kThreads];
    const int rowl = blockIdx.x;
    const int grb = p.grg0 * p.NW + (rowl >> 5);
    if ((grb % (p.NRG * p.NW)) * 32 + (rowl & 31) >= p.Rk) return;   // no such row
    // thread = (group gi of key splits, layer l): Lq layers side by side, kThreads / Lq groups
    const int Lq = p.L <= 32 ? 32 : (p.L <= 64 ? 64 : 128), NG = kThreads / Lq;
    const int l = threadIdx.x % Lq, gi = threadIdx.x / Lq;
    const bool ok = l < p.L;
    float *pm = p.rowM + (size_t)rowl * p.nsplit * p.L + l;
    const float *pz = p.rowZ + (size_t)rowl * p.nsplit * p.L + l;
    float mxv = kMInit;
    if (ok)
        for (int sp = gi; sp < p.nsplit; sp += NG) mxv = fmaxf(mxv, pm[(size_t)sp * p.L]);
    red[threadIdx.x] = mxv;
    __syncthreads();
    for (int g2 = 0; g2 < NG; ++g2) mxv = fmaxf(mxv, red[g2 * Lq + l]);
    __syncthreads();
    float z = 0.f;
    if (ok)
        for (int sp = gi; sp < p.nsplit; sp += NG) {
            const float f = exp2f(pm[(size_t)sp * p.L] - mxv);
            z += pz[(size_t)sp * p.L] * f;
            pm[(size_t)sp * p.L] = f;
        }
    red[threadIdx.x] = z;
    __syncthreads();
    if (ok && gi == 0) {
        float zt = 0.f;
        for (int g2 = 0; g2 < NG; ++g2) zt += red[g2 * Lq + l];   // fixed order
        p.rowZt[(size_t)rowl * p.L + l] = 1.f / zt;
    }
}

// ------------------------------------------------------------------------------------------------
// 3. Gram kernel.  A workgroup of WV waves takes WV*RPW rows of one 32-row block (wave w the rows
// w*RPW ..) and the key blocks [y*kb_per, (y+1)*kb_per) of them: all its waves walk the same key
// blocks at about the same time, so that what it fetches of a (layer, key block) is one contiguous
// run.  NB = 32-layer blocks (L <= 32*NB).  The sums go to Gpart[row][y] in result-register order
// (block a, register v, lane): element v of lane (m, kg) of block (bi, bj) is
// G[bi*32 + 8*(v/4) + 4*kg + v%4][bj*32 + m].
template <int NB, int RPW, int WV>
__global__ __launch_bounds__(WV * 64) void ap_gram_kernel(APParams p, int ksp, int kb_per)
{
    constexpr int NACC = NB * (NB + 1) / 2, RWG = WV * RPW;
    const int sub = blockIdx.x % (32 / RWG), rbl = blockIdx.x / (32 / RWG), y = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, m = lane & 31, kg = lane >> 5;
    const int grb = p.grg0 * p.NW + rbl;
    const int rb = grb % (p.NRG * p.NW);
    const int row0 = sub * RWG + w * RPW;           // first row (of the 32-row block) of this wave
    const int L = p.L, nsplit = p.nsplit;
    int nrows = p.Rk - (rb * 32 + row0);            // rows of this wave that exist
    nrows = nrows < 0 ? 0 : (nrows > RPW ? RPW : nrows);
    if (nrows == 0) return;

    const unsigned char *src[NB];
    bool lok[NB];
#pragma unroll
    for (int lb = 0; lb < NB; ++lb) {
        const int l = lb * 32 + m;
        lok[lb] = l < L;
        src[lb] = p.E + e_block_offset(p, rbl, lok[lb] ? l : 0, 0) + row0 * 64 + kg * 32;
    }
    f32x16 acc[RPW][NACC];
#pragma unroll
    for (int rr = 0; rr < RPW; ++rr)
#pragma unroll
        for (int a = 0; a < NACC; ++a)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[rr][a][v] = 0.f;

    const int bps = p.kps / 32;   // key blocks per key split of the weights kernel
    const int kb_begin = y * kb_per, kb_end = min(p.NKB, kb_begin + kb_per);
    int cur_sp = -1;
    f16x8 fsc[RPW][NB];
    // the operands of key block kb+1 are fetched while those of kb are multiplied
    uint4 raw[2][RPW][NB][2];
    auto fetch = [&](int kb, uint4 (&dst)[RPW][NB][2]) __attribute__((always_inline)) {
#pragma unroll
        for (int rr = 0; rr < RPW; ++rr)
#pragma unroll
            for (int lb = 0; lb < NB; ++lb) {
                dst[rr][lb][0] = dst[rr][lb][1] = make_uint4(0u, 0u, 0u, 0u);
                if (lok[lb] && rr < nrows) {
                    const uint4 *s4 = reinterpret_cast<const uint4 *>(src[lb] + (size_t)kb * L * 2048 + rr * 64);
                    dst[rr][lb][0] = s4[0];
                    dst[rr][lb][1] = s4[1];
                }
            }
    };
    auto multiply = [&](int kb, const uint4 (&cur)[RPW][NB][2]) __attribute__((always_inline)) {
        if (nsplit > 1 && kb / bps != cur_sp) {   // a new key split: its factors to the common exponents
            cur_sp = kb / bps;
#pragma unroll
            for (int rr = 0; rr < RPW; ++rr)
#pragma unroll
                for (int lb = 0; lb < NB; ++lb) {
                    float f = 0.f;
                    if (lok[lb] && rr < nrows)
                        f = p.rowM[(((size_t)rbl * 32 + row0 + rr) * nsplit + cur_sp) * L + lb * 32 + m];
                    const _Float16 fh = (_Float16)f;
                    fsc[rr][lb] = f16x8{fh, fh, fh, fh, fh, fh, fh, fh};
                }
        }
        f16x8 op[RPW][NB][2];
#pragma unroll
        for (int rr = 0; rr < RPW; ++rr)
#pragma unroll
            for (int lb = 0; lb < NB; ++lb)
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    op[rr][lb][j] = __builtin_bit_cast(f16x8, cur[rr][lb][j]);
                    if (nsplit > 1) op[rr][lb][j] = op[rr][lb][j] * fsc[rr][lb];
                }
#pragma unroll
        for (int rr = 0; rr < RPW; ++rr) {
            int a = 0;
#pragma unroll
            for (int bi = 0; bi < NB; ++bi)
#pragma unroll
                for (int bj = 0; bj <= bi; ++bj, ++a)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[rr][a] = __builtin_amdgcn_mfma_f32_32x32x16_f16(op[rr][bi][j], op[rr][bj][j], acc[rr][a], 0, 0, 0);
        }
    };
    if (kb_begin < kb_end) fetch(kb_begin, raw[0]);
    for (int kb = kb_begin; kb < kb_end; kb += 2) {
        if (kb + 1 < kb_end) fetch(kb + 1, raw[1]);
        multiply(kb, raw[0]);
        if (kb + 1 < kb_end) {
            if (kb + 2 < kb_end) fetch(kb + 2, raw[0]);
            multiply(kb + 1, raw[1]);
        }
    }
#pragma unroll
    for (int rr = 0; rr < RPW; ++rr) {
        if (rr >= nrows) break;
        float *dst = p.Gpart + (((size_t)rbl * 32 + row0 + rr) * ksp + y) * (NACC * 1024) + lane;
#pragma unroll
        for (int a = 0; a < NACC; ++a)
#pragma unroll
            for (int v = 0; v < 16; ++v) dst[a * 1024 + v * 64] = acc[rr][a][v];
    }
}

// 4. One workgroup per row of the batch: the row's partial Gram matrices are added in order and
// cos_ij, dist_ij are written for i > j.
__global__ __launch_bounds__(kThreads) void ap_row_final_kernel(APParams p, int ksp)
{
    extern __shared__ float sm_rf[];
    const int L = p.L, NB = (L + 31) / 32, NACC = NB * (NB + 1) / 2;
    float *Gs = sm_rf;                 // [NACC*1024]
    float *Zs = Gs + NACC * 1024;      // [L]: 1 / Z of the layer
    const int rowl = blockIdx.x, rbl = rowl >> 5, row32 = rowl & 31;
    const int grb = p.grg0 * p.NW + rbl;
    const int rb = grb % (p.NRG * p.NW);
    if (rb * 32 + row32 >= p.Rk) return;
    const int tid = threadIdx.x;
    const float *gp = p.Gpart + (size_t)rowl * ksp * (NACC * 1024);
    for (int i = tid; i < NACC * 1024; i += kThreads) {
        float g = 0.f;
        int y = 0;
        for (; y + 8 <= ksp; y += 8) {   // eight loads in flight, added in order
            float t[8];
#pragma unroll
            for (int k2 = 0; k2 < 8; ++k2) t[k2] = gp[(size_t)(y + k2) * (NACC * 1024) + i];
#pragma unroll
            for (int k2 = 0; k2 < 8; ++k2) g += t[k2];
        }
        for (; y < ksp; ++y) g += gp[(size_t)y * (NACC * 1024) + i];
        Gs[i] = g;
    }
    for (int l = tid; l < L; l += kThreads) Zs[l] = p.rowZt[(size_t)rowl * L + l];
    __syncthreads();
    auto G = [&](int i, int j) -> float {   // i >= j
        const int bi = i >> 5, bj = j >> 5, ii = i & 31;
        const int a = bi * (bi + 1) / 2 + bj;
        const int v = ((ii >> 3) << 2) | (ii & 3), kg = (ii >> 2) & 1;
        return Gs[a * 1024 + v * 64 + kg * 32 + (j & 31)];
    };
    float *oc = p.row_cos + (size_t)rowl * L * L;
    float *od = p.row_dist + (size_t)rowl * L * L;
    for (int e = tid; e < L * L; e += kThreads) {
        const int i = e / L, j = e % L;
        if (i <= j) continue;
        const float gij = G(i, j), gii = G(i, i), gjj = G(j, j);
        oc[e] = gij * rsqrtf(gii * gjj);
        if (p.want_dist) {
            const float zi = Zs[i], zj = Zs[j];
            od[e] = sqrtf(fmaxf(gii * zi * zi + gjj * zj * zj - 2.f * gij * zi * zj, 0.f));
        }
    }
}

// ------------------------------------------------------------------------------------------------
// 5. rows -> head sums.  The rows of a head fall into kClasses classes by token index (t % kClasses);
// a thread owns one matrix entry of one class of one head and adds that class's rows of the batch,
// one by one in order, to the class's running sum: each sum sees its rows in the same order
// wherever the batches are cut, so the result does not depend on the batch size.
constexpr int kClasses = 8;

__global__ __launch_bounds__(kThreads) void ap_reduce_kernel(APParams p, int u0)
{
    const int LL = p.L * p.L;
    const int e = blockIdx.y * kThreads + threadIdx.x;
    const int cls = blockIdx.z;
    const int hg = blockIdx.x % p.g, u = u0 + blockIdx.x / p.g;
    // rows of unit u that this batch holds, and those of them that belong to head hg
    const int rg_lo = max(p.grg0, u * p.NRG) - u * p.NRG;
    const int rg_hi = min(p.grg0 + p.nrg, (u + 1) * p.NRG) - u * p.NRG;
    const int rpg = p.NW * 32;   // rows per row group
    const int r_lo = max(rg_lo * rpg, hg * p.Tq);
    const int r_hi = min(min(rg_hi * rpg, p.Rk), (hg + 1) * p.Tq);
    if (e >= LL || r_lo >= r_hi) return;
    const int i = e / p.L, j = e % p.L;
    if (i <= j) return;
    const int b = u / p.Hkv, hq = (u % p.Hkv) * p.g + hg;
    const size_t o = (((size_t)b * p.Hq + hq) * kClasses + cls) * LL + e;
    float cs = p.head_cos[o], ds = p.want_dist ? p.head_dist[o] : 0.f;
    auto rowl_of = [&](int r) -> size_t { return (size_t)(u * p.NRG + r / rpg - p.grg0) * rpg + r % rpg; };
    // first row of the range whose token index t = r - hg*Tq is in this class
    int r = r_lo + ((cls - (r_lo - hg * p.Tq)) % kClasses + kClasses) % kClasses;
    for (; r + 3 * kClasses < r_hi; r += 4 * kClasses) {   // four rows in flight, added in order
        float tc[4], td[4];
#pragma unroll
        for (int k2 = 0; k2 < 4; ++k2) {
            const size_t rowl = rowl_of(r + k2 * kClasses);
            tc[k2] = p.row_cos[rowl * LL + e];
            td[k2] = p.want_dist ? p.row_dist[rowl * LL + e] : 0.f;
        }
#pragma unroll
        for (int k2 = 0; k2 < 4; ++k2) {
            cs += tc[k2];
            ds += td[k2];
        }
    }
    for (; r < r_hi; r += kClasses) {
        const size_t rowl = rowl_of(r);
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
// the diagonal.  A workgroup takes 8 entries (conversation, i, j); 32 threads share an entry's heads
// (h = lane, lane + 32, ...) and their sums are added in lane order.
__global__ __launch_bounds__(kThreads) void ap_final_kernel(int B, int L, int Hq, float inv_tokens,
                                                            const float *__restrict__ head_cos,
                                                            const float *__restrict__ head_dist,
                                                            float *__restrict__ pair_cos, float *__restrict__ pair_dist,
                                                            float *__restrict__ head_out)
{
    __shared__ float sc[32][8], sd[32][8];
    const int LL = L * L;
    const int el = threadIdx.x & 7, hl = threadIdx.x >> 3;
    const size_t idx = (size_t)blockIdx.x * 8 + el;
    const bool ok = idx < (size_t)B * LL;
    float cs = 0.f, ds = 0.f;
    if (ok) {
        const int b = (int)(idx / LL), e = (int)(idx % LL), i = e / L, j = e % L;
        const int lo = i > j ? e : j * L + i;   // the entry below the diagonal holds the sums
        for (int h = hl; h < Hq; h += 32) {
            const size_t o = ((size_t)b * Hq + h) * LL, oc = o * kClasses + lo;
            float hc = 0.f, hd = 0.f;   // the classes' sums, in order
            if (i != j) {
#pragma unroll
                for (int cl = 0; cl < kClasses; ++cl) {
                    hc += head_cos[oc + (size_t)cl * LL];
                    if (pair_dist) hd += head_dist[oc + (size_t)cl * LL];
                }
            }
            const float c = i == j ? 1.f : hc * inv_tokens;
            cs += c;
            if (head_out) head_out[o + e] = c;
            ds += hd * inv_tokens;
        }
    }
    sc[hl][el] = cs;
    sd[hl][el] = ds;
    __syncthreads();
    if (ok && hl == 0) {
        float c = 0.f, d = 0.f;
        for (int k2 = 0; k2 < 32; ++k2) {
            c += sc[k2][el];
            d += sd[k2][el];
        }
        pair_cos[idx] = c / (float)Hq;
        if (pair_dist) pair_dist[idx] = d / (float)Hq;
    }
}

// ------------------------------------------------------------------------------------------------
// Greedy choice over all candidate pairs: n_select rounds of "best free pair", which is what one
// scan of the stably sorted list takes.  Order: key ascending (distance, or minus similarity),
// equal keys by lower j, then lower i.
constexpr int kSelThreads = 256;
constexpr int kSelLdsLayers = 96;   // up to this many layers the ordering keys are kept in LDS

__global__ __launch_bounds__(kSelThreads) void select_all_kernel(
    const float *__restrict__ score, int closer_is_smaller, const uint8_t *__restrict__ eligible,
    int L, int n_select, int32_t *__restrict__ out_pairs, int32_t *__restrict__ out_count)
{
    extern __shared__ unsigned char sm[];
    uint8_t *used = sm;                                                      // [L]: shared already, or not eligible
    float *bkey = reinterpret_cast<float *>(sm + ((L + 15) & ~15));          // [waves]
    int *brank = reinterpret_cast<int *>(bkey + kSelThreads / 64);           // [waves]
    float *keys = reinterpret_cast<float *>(brank + kSelThreads / 64);       // [L*L] if L <= kSelLdsLayers
    __shared__ int chosen;
    const int b = blockIdx.x, tid = threadIdx.x;
    const float *sc = score + (size_t)b * L * L;
    const bool in_lds = L <= kSelLdsLayers;
    for (int l = tid; l < L; l += kSelThreads) used[l] = eligible ? (eligible[(size_t)b * L + l] ? 0 : 1) : 0;
    if (in_lds) {   // (four loads in flight per thread: one memory latency per four entries)
        for (int e0 = 0; e0 < L * L; e0 += 4 * kSelThreads) {
            float v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int e = e0 + u * kSelThreads + tid;
                v[u] = e < L * L ? sc[e] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int e = e0 + u * kSelThreads + tid;
                if (e < L * L) keys[e] = closer_is_smaller ? v[u] : -v[u];
            }
        }
    }
    __syncthreads();
    int cnt = 0;
    if (L <= 128 && in_lds) {
        // Ordering keys in LDS (at most 96 layers): the layers in use are two 64-bit masks that every thread keeps for itself, and
        // every thread works out the round's winner from the waves' candidates -- one barrier a round
        // (the waves' candidates alternate between two sets of slots), no thread waits for thread 0.
        const int ln = tid & 63;
        unsigned long long used_lo = __ballot(ln < L && used[ln < L ? ln : 0]);
        unsigned long long used_hi = __ballot(ln + 64 < L && used[ln + 64 < L ? ln + 64 : 0]);
        auto is_used = [&](int l) { return ((l < 64 ? used_lo : used_hi) >> (l & 63)) & 1ull; };
        float *bk2 = keys + L * L;                                  // [2][waves]
        int *br2 = reinterpret_cast<int *>(bk2 + 2 * (kSelThreads / 64));
        for (; cnt < n_select; ++cnt) {
            float best = INFINITY;
            int rank = INT32_MAX;   // j * L + i of the best candidate
            for (int e = tid; e < L * L; e += kSelThreads) {
                const int i = e / L, j = e % L;
                if (i <= j || is_used(i) || is_used(j)) continue;
                const float key = keys[e];
                if (key != key) continue;   // a NaN score: no candidate
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
            const int set = (cnt & 1) * (kSelThreads / 64);
            if ((tid & 63) == 0) {
                bk2[set + (tid >> 6)] = best;
                br2[set + (tid >> 6)] = rank;
            }
            __syncthreads();
            float kb = bk2[set];
            int rk = br2[set];
#pragma unroll
            for (int wv = 1; wv < kSelThreads / 64; ++wv) {
                const float ob = bk2[set + wv];
                const int orank = br2[set + wv];
                if (orank != INT32_MAX && (rk == INT32_MAX || ob < kb || (ob == kb && orank < rk))) {
                    kb = ob;
                    rk = orank;
                }
            }
            if (rk == INT32_MAX) break;   // no free candidate is left
            const int j = rk / L, i = rk % L;
            (i < 64 ? used_lo : used_hi) |= 1ull << (i & 63);
            (j < 64 ? used_lo : used_hi) |= 1ull << (j & 63);
            if (tid == 0) {
                out_pairs[((size_t)b * n_select + cnt) * 2] = j;
                out_pairs[((size_t)b * n_select + cnt) * 2 + 1] = i;
            }
        }
    } else
    for (; cnt < n_select; ++cnt) {
        float best = INFINITY;
        int rank = INT32_MAX;   // j * L + i of the best candidate
        for (int e = tid; e < L * L; e += kSelThreads) {
            const int i = e / L, j = e % L;
            if (i <= j || used[i] || used[j]) continue;
            const float key = in_lds ? keys[e] : (closer_is_smaller ? sc[e] : -sc[e]);
            if (key != key) continue;   // a NaN score: no candidate
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
    int NW, NRG, NKB, nsplit, kps, tpw, total_rg, nrg_batch, ksp, kb_per;
    size_t head_cos_off, head_dist_off, dump_off, rowm_off, rowz_off, rowzt_off, gpart_off, row_cos_off, row_dist_off, e_off, total_bytes;
    bool mfma;
};

constexpr int kGramTargetWorkgroups = 512;

// Sizes for a batch of nrg row groups (NW, NRG, NKB, nsplit must be set).
void ap_layout(const krul_shape_t *s, int nrg, APPlan *pl)
{
    const size_t L = s->n_layers, LL = L * L, NB = (L + 31) / 32, NACC = NB * (NB + 1) / 2;
    const size_t heads = (size_t)s->batch * s->n_q_heads * kClasses * LL * sizeof(float);
    const size_t rows = (size_t)nrg * pl->NW * 32;
    // the Gram kernel splits the keys until it has enough workgroups, but keeps at least 16 key blocks
    // per workgroup so that the partial matrices stay small beside the weights
    const long long row_wgs = (long long)nrg * pl->NW * (NB == 1 ? 1 : (NB == 2 ? 2 : (NB == 3 ? 4 : 8)));
    long long ksp = (kGramTargetWorkgroups + row_wgs - 1) / row_wgs;
    const long long ksp_max = pl->NKB / 16 > 1 ? pl->NKB / 16 : 1;
    if (ksp > ksp_max) ksp = ksp_max;
    if (ksp > 64) ksp = 64;
    pl->kb_per = (int)((pl->NKB + ksp - 1) / ksp);
    pl->ksp = (pl->NKB + pl->kb_per - 1) / pl->kb_per;
    size_t off = 0;
    pl->head_cos_off = off; off += align_up(heads);
    pl->head_dist_off = off; off += align_up(heads);
    pl->dump_off = off; off += align_up((size_t)kDumpBlocks * 2048);
    pl->rowm_off = off; off += align_up(rows * L * pl->nsplit * sizeof(float));
    pl->rowz_off = off; off += align_up(rows * L * pl->nsplit * sizeof(float));
    pl->rowzt_off = off; off += align_up(rows * L * sizeof(float));
    pl->gpart_off = off; off += align_up(rows * pl->ksp * NACC * 1024 * sizeof(float));
    pl->row_cos_off = off; off += align_up(rows * LL * sizeof(float));
    pl->row_dist_off = off; off += align_up(rows * LL * sizeof(float));
    pl->e_off = off; off += align_up((size_t)nrg * pl->NW * L * pl->NKB * 2048);
    pl->total_bytes = off;
    pl->nrg_batch = nrg;
}

constexpr int kMaxLayersAllPairs = 128;
constexpr size_t kDefaultBudget = (size_t)4 << 30;

// Validate and size: the largest batch of row groups whose workspace fits max_bytes (0: a default
// budget), at least one group.  Returns a krul_status_t.
int ap_plan(const krul_shape_t *s, size_t max_bytes, APPlan *pl)
{
    const int rc = check_shape(s);
    if (rc != KRUL_OK) return rc;
    if (s->n_layers > kMaxLayersAllPairs) return KRUL_EUNSUPPORTED;
    const long long g = s->n_q_heads / s->n_kv_heads, Rk = g * s->n_query;
    if (Rk > INT32_MAX || (long long)s->batch * s->n_q_heads * s->n_query > INT32_MAX) return KRUL_EUNSUPPORTED;
    if (s->n_hist * (long long)s->head_dim * 4 >= (1ll << 31)) return KRUL_EUNSUPPORTED;
    const long long NRB = (Rk + 31) / 32;   // 32-row blocks per unit
    pl->NW = NRB >= 6 ? 8 : (NRB >= 3 ? 4 : (int)NRB);
    pl->NRG = (int)((NRB + pl->NW - 1) / pl->NW);
    pl->NKB = (s->n_hist + 31) / 32;
    const long long total = (long long)s->batch * s->n_kv_heads * pl->NRG;
    if (total * pl->NW * 32 > INT32_MAX / 4) return KRUL_EUNSUPPORTED;
    pl->total_rg = (int)total;
    pl->mfma = (s->dtype == KRUL_BF16 || s->dtype == KRUL_F16) && s->head_dim <= 128 &&
               !(s->flags & KRUL_FLAG_GENERIC_KERNEL);
    // key splits of the weights kernel: one per kKeysPerSplit keys (the portable kernel does not split)
    if (pl->mfma) {
        pl->kps = kKeysPerSplit;
        pl->nsplit = (s->n_hist + kKeysPerSplit - 1) / kKeysPerSplit;
        // a workgroup walks up to 8 splits, fewer while that leaves fewer than 2048 workgroups
        const long long wg1 = total * s->n_layers;
        long long tpw = wg1 * pl->nsplit / 2048;
        pl->tpw = (int)(tpw < 1 ? 1 : (tpw > 8 ? 8 : tpw));
    } else {
        pl->nsplit = 1;
        pl->tpw = 1;
        pl->kps = pl->NKB * 32;
    }

    const size_t budget = max_bytes ? max_bytes : kDefaultBudget;
    // the largest batch that fits (the size grows with the batch but for the partial matrices, whose
    // number per row shrinks as the batch grows: bisect, then step down if need be)
    long long lo = 1, hi = total;
    while (lo < hi) {
        const long long mid = (lo + hi + 1) / 2;
        ap_layout(s, (int)mid, pl);
        if (pl->total_bytes <= budget) lo = mid; else hi = mid - 1;
    }
    ap_layout(s, (int)lo, pl);
    while (pl->total_bytes > budget && lo > 1) ap_layout(s, (int)--lo, pl);
    return KRUL_OK;
}

template <int D, bool F16>
void launch_weights(const APParams &p, hipStream_t st)
{
    const dim3 grid(p.nrg * p.L * ((p.nsplit + p.tpw - 1) / p.tpw));
    if (p.ka.k_tab || p.d != D) {
        switch (p.NW) {
        case 1: hipLaunchKernelGGL((ap_weights_mfma_kernel<D, 1, 1, F16, true>), grid, dim3(64), 0, st, p); break;
        case 2: hipLaunchKernelGGL((ap_weights_mfma_kernel<D, 2, 1, F16, true>), grid, dim3(128), 0, st, p); break;
        case 4: hipLaunchKernelGGL((ap_weights_mfma_kernel<D, 4, 1, F16, true>), grid, dim3(256), 0, st, p); break;
        default: hipLaunchKernelGGL((ap_weights_mfma_kernel<D, 4, 2, F16, true>), grid, dim3(256), 0, st, p); break;
        }
        return;
    }
    switch (p.NW) {
    case 1: hipLaunchKernelGGL((ap_weights_mfma_kernel<D, 1, 1, F16, false>), grid, dim3(64), 0, st, p); break;
    case 2: hipLaunchKernelGGL((ap_weights_mfma_kernel<D, 2, 1, F16, false>), grid, dim3(128), 0, st, p); break;
    case 4: hipLaunchKernelGGL((ap_weights_mfma_kernel<D, 4, 1, F16, false>), grid, dim3(256), 0, st, p); break;
    default: hipLaunchKernelGGL((ap_weights_mfma_kernel<D, 4, 2, F16, false>), grid, dim3(256), 0, st, p); break;
    }
}

}  // namespace

size_t all_pairs_workspace(const krul_shape_t *s, size_t max_bytes)
{
    APPlan pl;
    if (ap_plan(s, max_bytes, &pl) != KRUL_OK) return 0;
    return pl.total_bytes;
}

int run_all_pairs(const krul_shape_t *s, const void *q, const void *k, const krul_k_layout_t *kl,
                  const krul_k_pages_t *kp, float *pair_score, float *pair_dist, float *head_score,
                  void *workspace, size_t workspace_bytes, hipStream_t st)
{
    APPlan pl;
    int rc = ap_plan(s, 1, &pl);   // the smallest batch: one row group
    if (rc != KRUL_OK) return rc;
    if (!q || !pair_score) return KRUL_EINVAL;
    if ((uintptr_t)q & 15) return KRUL_EINVAL;
    if (((uintptr_t)pair_score | (uintptr_t)pair_dist | (uintptr_t)head_score) & 3) return KRUL_EINVAL;
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < pl.total_bytes) return KRUL_EWORKSPACE;
    // the batch is what the caller's workspace holds
    rc = ap_plan(s, workspace_bytes, &pl);
    if (rc != KRUL_OK) return rc;
    if (pl.total_bytes > workspace_bytes) return KRUL_EWORKSPACE;

    unsigned char *ws = static_cast<unsigned char *>(workspace);
    APParams p;
    p.q = q;
    p.k = k;
    rc = resolve_keys(s, pl.mfma, false, k, kl, kp, &p.ka);
    if (rc != KRUL_OK) return rc;
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
    p.NW = pl.NW;
    p.NRG = pl.NRG;
    p.NKB = pl.NKB;
    p.nsplit = pl.nsplit;
    p.kps = pl.kps;
    p.tpw = pl.tpw;
    p.want_dist = pair_dist != nullptr;
    p.E = ws + pl.e_off;
    p.dump = ws + pl.dump_off;
    p.rowM = reinterpret_cast<float *>(ws + pl.rowm_off);
    p.rowZ = reinterpret_cast<float *>(ws + pl.rowz_off);
    p.rowZt = reinterpret_cast<float *>(ws + pl.rowzt_off);
    p.Gpart = reinterpret_cast<float *>(ws + pl.gpart_off);
    p.row_cos = reinterpret_cast<float *>(ws + pl.row_cos_off);
    p.row_dist = reinterpret_cast<float *>(ws + pl.row_dist_off);
    p.head_cos = reinterpret_cast<float *>(ws + pl.head_cos_off);
    p.head_dist = reinterpret_cast<float *>(ws + pl.head_dist_off);

    const int L = p.L, LL = L * L;
    const size_t n_head = (size_t)p.B * p.Hq * kClasses * LL;
    // (the two areas of running sums lie one after the other in the workspace: one launch clears both)
    const size_t n_fill = p.want_dist ? (size_t)(p.head_dist - p.head_cos) + n_head : n_head;
    hipLaunchKernelGGL(ap_fill_kernel, dim3((unsigned)((n_fill + 255) / 256)), dim3(256), 0, st, p.head_cos, n_fill, 0.f);
    if (hipGetLastError() != hipSuccess) return KRUL_ELAUNCH;

    const int NB = (L + 31) / 32, NACC = NB * (NB + 1) / 2;
    const size_t rf_smem = ((size_t)NACC * 1024 + L) * sizeof(float);
    for (int g0 = 0; g0 < pl.total_rg; g0 += pl.nrg_batch) {
        p.grg0 = g0;
        p.nrg = pl.nrg_batch < pl.total_rg - g0 ? pl.nrg_batch : pl.total_rg - g0;
        const int rblocks = p.nrg * p.NW, rows = rblocks * 32;
        if (pl.mfma) {
            const bool f16 = s->dtype == KRUL_F16;
            if (p.d > 64)   // (head sizes below the kernel's ride zero-padded in LDS: the in-place form)
                f16 ? launch_weights<128, true>(p, st) : launch_weights<128, false>(p, st);
            else
                f16 ? launch_weights<64, true>(p, st) : launch_weights<64, false>(p, st);
        } else if (s->dtype == KRUL_F32) {
            hipLaunchKernelGGL(ap_weights_generic_kernel<float>, dim3(rows * L), dim3(64), p.d * sizeof(float), st, p);
        } else if (s->dtype == KRUL_F16) {
            hipLaunchKernelGGL(ap_weights_generic_kernel<_Float16>, dim3(rows * L), dim3(64), p.d * sizeof(float), st, p);
        } else {
            hipLaunchKernelGGL(ap_weights_generic_kernel<uint16_t>, dim3(rows * L), dim3(64), p.d * sizeof(float), st, p);
        }
        hipLaunchKernelGGL(ap_scale_kernel, dim3(rows), dim3(kThreads), 0, st, p);
        switch (NB) {
        case 1: hipLaunchKernelGGL((ap_gram_kernel<1, 4, 8>), dim3(rblocks, pl.ksp), dim3(512), 0, st, p, pl.ksp, pl.kb_per); break;
        case 2: hipLaunchKernelGGL((ap_gram_kernel<2, 2, 8>), dim3(rblocks * 2, pl.ksp), dim3(512), 0, st, p, pl.ksp, pl.kb_per); break;
        case 3: hipLaunchKernelGGL((ap_gram_kernel<3, 1, 8>), dim3(rblocks * 4, pl.ksp), dim3(512), 0, st, p, pl.ksp, pl.kb_per); break;
        default: hipLaunchKernelGGL((ap_gram_kernel<4, 1, 4>), dim3(rblocks * 8, pl.ksp), dim3(256), 0, st, p, pl.ksp, pl.kb_per); break;
        }
        hipLaunchKernelGGL(ap_row_final_kernel, dim3(rows), dim3(kThreads), rf_smem, st, p, pl.ksp);
        const int u0 = g0 / p.NRG, u1 = (g0 + p.nrg - 1) / p.NRG;
        hipLaunchKernelGGL(ap_reduce_kernel, dim3((u1 - u0 + 1) * p.g, (LL + kThreads - 1) / kThreads, kClasses), dim3(kThreads),
                           0, st, p, u0);
        if (hipGetLastError() != hipSuccess) return KRUL_ELAUNCH;
    }
    const size_t n_out = (size_t)p.B * LL;
    hipLaunchKernelGGL(ap_final_kernel, dim3((unsigned)((n_out + 7) / 8)), dim3(kThreads), 0, st, p.B, L, p.Hq,
                       1.0f / (float)p.Tq, p.head_cos, p.head_dist, pair_score, pair_dist, head_score);
    return hipGetLastError() == hipSuccess ? KRUL_OK : KRUL_ELAUNCH;
}

hipError_t launch_select_all(const float *score, int closer_is_smaller, const uint8_t *eligible, int batch,
                             int n_layers, int n_select, int32_t *out_pairs, int32_t *out_count, hipStream_t st)
{
    const size_t smem = ((n_layers + 15) & ~15) + (kSelThreads / 64) * (sizeof(float) + sizeof(int));
    // (+ two sets of per-wave candidates for the one-barrier rounds)
    const size_t smem_keys = n_layers <= kSelLdsLayers
                                 ? (size_t)n_layers * n_layers * sizeof(float) + 2 * (kSelThreads / 64) * (sizeof(float) + sizeof(int))
                                 : 0;
    hipLaunchKernelGGL(select_all_kernel, dim3(batch), dim3(kSelThreads), smem + smem_keys, st, score, closer_is_smaller,
                       eligible, n_layers, n_select, out_pairs, out_count);
    return hipGetLastError();
}

}  // namespace krul
