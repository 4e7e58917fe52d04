// bf16 MFMA similarity kernel for gfx950 (CDNA4).
//
// Work decomposition.  A "unit" is one (conversation, kv head): its (Hq/Hkv)*Tq
// query rows all read the same keys.  A workgroup (4 wavefronts) owns R_WG rows of a
// unit and one contiguous key split; it walks the split in key tiles of KT keys and,
// inside a tile, the layers 0..L-1 in order, so that every layer's logits are formed
// exactly once and the previous layer's exponentials of the same keys are still in
// registers when the cross term (the "ab" of Sec. 7's a^2 + b^2 - 2ab) is taken.
//
// Per layer step the K tile arrives in chunks of CH = 32*WK keys: global -> registers
// -> LDS (row stride padded by 16 bytes, which spreads 16 consecutive rows over all
// banks for 16-byte reads), double buffered, one barrier per chunk.  Each wave takes
// one 32-key block of the chunk and RB blocks of 32 query rows:
//     S^T (32 keys x 32 rows) = K_blk (32 x d) * Q_blk^T (d x 32)
// with v_mfma_f32_32x32x16_bf16, A = keys (from LDS), B = query rows (held in
// registers for the whole layer step).  In the result every lane owns ONE query row
// (column lane%32) and 16 keys, so all softmax reductions are lane-local: no
// cross-lane traffic in the loop.  Lanes l and l+32 and the WK waves along the keys
// are independent partials of a row, merged once after the last tile.
//
// Online softmax uses a lazily updated reference exponent m per (lane, layer): it is
// raised only when a logit exceeds it by more than kLazy (in log2 units); then the
// running sums, and the exponentials of the current layer already produced in this
// tile, are rescaled.  Cosine and distance are invariant to the choice of m, and
// e = 2^(x-m) <= 2^kLazy keeps every sum far inside fp32 range.
#include "krul_common.h"

namespace krul {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr float kLazy = 16.0f;

template <int D_, int WR_, int WK_, int RB_, int NKB_>
struct Cfg {
    static constexpr int D = D_, WR = WR_, WK = WK_, RB = RB_, NKB = NKB_;
    static constexpr int NW = WR * WK;
    static constexpr int THREADS = NW * 64;
    static constexpr int R_WG = WR * RB * 32;
    static constexpr int CH = WK * 32;             // keys per chunk
    static constexpr int KT = CH * NKB;            // keys per tile
    static constexpr int KS = D / 16;              // MFMA k-steps per 32x32 block
    static constexpr int ROWB = D * 2 + 16;        // LDS row stride, bytes
    static constexpr int CHUNK_BYTES = CH * ROWB;
    static constexpr int PIECES_PER_ROW = D / 8;   // 16-byte pieces per key row
    static constexpr int NLD = CH * PIECES_PER_ROW / THREADS;  // pieces per thread per chunk
    static_assert(NW == 4, "four waves per workgroup");
    static_assert(CH * PIECES_PER_ROW % THREADS == 0, "chunk must split evenly over threads");
};

// Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous range of
// logical ids so that workgroups sharing K (neighbouring row tiles) share an L2.
__device__ inline int xcd_remap(int bid, int n)
{
    const int q = n >> 3, rem = n & 7, x = bid & 7;
    return x * q + min(x, rem) + (bid >> 3);
}

template <class C>
__global__ __launch_bounds__(C::THREADS, 2) void sim_mfma_kernel(SimParams p)
{
    constexpr int D = C::D, WK = C::WK, RB = C::RB, NKB = C::NKB, KS = C::KS, NLD = C::NLD;
    __shared__ __attribute__((aligned(16))) unsigned char lds[2][C::CHUNK_BYTES];
    __shared__ float red[C::NW][RB][4][32];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wr = wave / WK, wk = wave % WK, half = lane >> 5, l32 = lane & 31;

    const int wg = xcd_remap(blockIdx.x, gridDim.x);
    const int nrt = p.lay.n_row_tiles, nsplit = p.lay.n_split;
    const int rt = wg % nrt, sp = (wg / nrt) % nsplit, u = wg / (nrt * nsplit);
    const int b = u / p.Hkv, kvh = u % p.Hkv;
    const int L = p.L, S = p.S, Rk = p.lay.rows_per_unit;

    const int key_begin = sp * p.keys_per_split;
    const int key_end = min(S, key_begin + p.keys_per_split);
    const int ntiles = (key_end - key_begin + C::KT - 1) / C::KT;
    const int nchunks = ntiles * L * NKB;

    // ---- query rows of this lane (clamped; rows past the unit are never read back)
    const uint16_t *Qg = static_cast<const uint16_t *>(p.q);
    const uint16_t *Kg = static_cast<const uint16_t *>(p.k);
    const size_t q_layer_stride = (size_t)p.Hq * p.Tq * D;
    const size_t k_layer_stride = (size_t)p.Hkv * S * D;
    const uint16_t *qptr[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const int r = min(rt * C::R_WG + (wr * RB + rb) * 32 + l32, Rk - 1);
        qptr[rb] = Qg + ((size_t)b * L * p.Hq * p.Tq + (size_t)kvh * Rk + r) * D + half * 8;
    }
    const uint16_t *kbase = Kg + ((size_t)b * L * p.Hkv + kvh) * (size_t)S * D;

    // ---- chunk staging: piece i = tid + j*THREADS -> key i / (D/8), 16-byte piece i % (D/8)
    uint4 stg[NLD];
    int pf_tile = 0, pf_l = 0, pf_c = 0;   // position of the next chunk to fetch
    auto fetch_chunk = [&]() {
        const int key0 = key_begin + pf_tile * C::KT + pf_c * C::CH;
        const uint16_t *src = kbase + (size_t)pf_l * k_layer_stride;
#pragma unroll
        for (int j = 0; j < NLD; ++j) {
            const int i = tid + j * C::THREADS;
            const int key = min(key0 + i / C::PIECES_PER_ROW, S - 1);
            stg[j] = *reinterpret_cast<const uint4 *>(src + (size_t)key * D + (i % C::PIECES_PER_ROW) * 8);
        }
        if (++pf_c == NKB) {
            pf_c = 0;
            if (++pf_l == L) {
                pf_l = 0;
                ++pf_tile;
            }
        }
    };
    auto stage_chunk = [&](int buf) {
#pragma unroll
        for (int j = 0; j < NLD; ++j) {
            const int i = tid + j * C::THREADS;
            *reinterpret_cast<uint4 *>(&lds[buf][(i / C::PIECES_PER_ROW) * C::ROWB + (i % C::PIECES_PER_ROW) * 16]) = stg[j];
        }
    };

    bf16x8 qf[RB][KS];
    auto load_q = [&](int l) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                qf[rb][ks] = *reinterpret_cast<const bf16x8 *>(qptr[rb] + (size_t)l * q_layer_stride + ks * 16);
    };

    // per-lane spill records (only used when the split spans several tiles)
    float4 *spill = p.spill;
    auto spill_index = [&](int l, int rb) -> size_t {
        return (((((size_t)wg * L + l) * C::NW + wave) * RB + rb) << 6) + lane;
    };

    float e[RB][NKB][16];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int c = 0; c < NKB; ++c)
#pragma unroll
            for (int v = 0; v < 16; ++v) e[rb][c][v] = 0.f;

    // ---- prologue of the chunk pipeline
    fetch_chunk();
    stage_chunk(0);
    if (nchunks > 1) fetch_chunk();
    load_q(0);
    __syncthreads();

    const float cs = p.c;
    int n = 0;
    float f_prev[RB], mrg_prev[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) f_prev[rb] = mrg_prev[rb] = 1.f;

    for (int tile = 0; tile < ntiles; ++tile) {
        const int tile_key0 = key_begin + tile * C::KT;
        const bool ragged = tile_key0 + C::KT > key_end;
        const bool last_tile = tile == ntiles - 1;
        for (int l = 0; l < L; ++l) {
            float4 rec[RB];
            float mcur[RB], tz[RB], tn[RB], tc[RB];
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                rec[rb] = tile > 0 ? spill[spill_index(l, rb)] : make_float4(kMInit, 0.f, 0.f, 0.f);
                mcur[rb] = rec[rb].x;
                tz[rb] = tn[rb] = tc[rb] = 0.f;
            }
#pragma unroll
            for (int c = 0; c < NKB; ++c) {
                const int buf = n & 1;
                if (n + 1 < nchunks) stage_chunk(buf ^ 1);
                if (n + 2 < nchunks) fetch_chunk();

                f32x16 acc[RB];
#pragma unroll
                for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[rb][v] = 0.f;
                const unsigned char *kb = &lds[buf][(wk * 32 + l32) * C::ROWB + half * 16];
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const bf16x8 a = *reinterpret_cast<const bf16x8 *>(kb + ks * 32);
#pragma unroll
                    for (int rb = 0; rb < RB; ++rb)
                        acc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[rb][ks], acc[rb], 0, 0, 0);
                }
                if (c == NKB - 1) load_q(l + 1 == L ? 0 : l + 1);   // next step's query rows

#pragma unroll
                for (int rb = 0; rb < RB; ++rb) {
                    if (ragged) {
                        const int kb0 = tile_key0 + c * C::CH + wk * 32 + half * 4;
#pragma unroll
                        for (int v = 0; v < 16; ++v)
                            if (kb0 + 8 * (v >> 2) + (v & 3) >= key_end) acc[rb][v] = -INFINITY;
                    }
                    float tmax = acc[rb][0];
#pragma unroll
                    for (int v = 1; v < 16; ++v) tmax = fmaxf(tmax, acc[rb][v]);
                    const float xm = tmax * cs;
                    if (__any(xm > mcur[rb] + kLazy)) {
                        const float mnew = fmaxf(mcur[rb], xm);
                        const float f = __builtin_amdgcn_exp2f(mcur[rb] - mnew);
                        tz[rb] *= f;
                        tn[rb] *= f * f;
                        tc[rb] *= f;
#pragma unroll
                        for (int cc = 0; cc < c; ++cc)
#pragma unroll
                            for (int v = 0; v < 16; ++v) e[rb][cc][v] *= f;
                        mcur[rb] = mnew;
                    }
                    const float negm = -mcur[rb];
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const float ev = __builtin_amdgcn_exp2f(fmaf(acc[rb][v], cs, negm));
                        tz[rb] += ev;
                        tn[rb] = fmaf(ev, ev, tn[rb]);
                        tc[rb] = fmaf(ev, e[rb][c][v], tc[rb]);
                        e[rb][c][v] = ev;
                    }
                }
                __syncthreads();
                ++n;
            }

            // ---- fold this tile's sums into the running record of layer l
            float4 out[RB];
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                const float F = __builtin_amdgcn_exp2f(rec[rb].x - mcur[rb]);
                out[rb].x = mcur[rb];
                out[rb].y = fmaf(rec[rb].y, F, tz[rb]);
                out[rb].z = fmaf(rec[rb].z, F * F, tn[rb]);
                out[rb].w = fmaf(rec[rb].w, F * f_prev[rb], tc[rb]);
                f_prev[rb] = F;
            }
            if (!last_tile) {
#pragma unroll
                for (int rb = 0; rb < RB; ++rb) spill[spill_index(l, rb)] = out[rb];
            } else {
                // ---- merge the 2*WK partials of each row: common exponent, then sums
                float mh[RB];
#pragma unroll
                for (int rb = 0; rb < RB; ++rb) {
                    mh[rb] = fmaxf(out[rb].x, __shfl_xor(out[rb].x, 32, 64));
                    if (half == 0) red[wave][rb][0][l32] = mh[rb];
                }
                __syncthreads();
                float zs[RB], ns[RB], cc2[RB], M[RB];
#pragma unroll
                for (int rb = 0; rb < RB; ++rb) {
                    M[rb] = red[wr * WK][rb][0][l32];
#pragma unroll
                    for (int w2 = 1; w2 < WK; ++w2) M[rb] = fmaxf(M[rb], red[wr * WK + w2][rb][0][l32]);
                    const float f = __builtin_amdgcn_exp2f(out[rb].x - M[rb]);
                    float z = out[rb].y * f, nn = out[rb].z * f * f, cc = out[rb].w * f * mrg_prev[rb];
                    mrg_prev[rb] = f;
                    z += __shfl_xor(z, 32, 64);
                    nn += __shfl_xor(nn, 32, 64);
                    cc += __shfl_xor(cc, 32, 64);
                    zs[rb] = z;
                    ns[rb] = nn;
                    cc2[rb] = cc;
                }
                __syncthreads();
#pragma unroll
                for (int rb = 0; rb < RB; ++rb)
                    if (half == 0) {
                        red[wave][rb][1][l32] = zs[rb];
                        red[wave][rb][2][l32] = ns[rb];
                        red[wave][rb][3][l32] = cc2[rb];
                    }
                __syncthreads();
                if (wk == 0 && half == 0) {
#pragma unroll
                    for (int rb = 0; rb < RB; ++rb) {
                        float z = 0.f, nn = 0.f, cc = 0.f;
#pragma unroll
                        for (int w2 = 0; w2 < WK; ++w2) {
                            z += red[wr * WK + w2][rb][1][l32];
                            nn += red[wr * WK + w2][rb][2][l32];
                            cc += red[wr * WK + w2][rb][3][l32];
                        }
                        const size_t idx = ((size_t)wg * L + l) * C::R_WG + (wr * RB + rb) * 32 + l32;
                        p.state[idx] = make_float4(M[rb], z, nn, cc);
                    }
                }
                __syncthreads();
            }
        }
    }
}

template <class C>
hipError_t launch_cfg(const SimParams &p, int n_workgroups, hipStream_t st)
{
    hipLaunchKernelGGL(sim_mfma_kernel<C>, dim3(n_workgroups), dim3(C::THREADS), 0, st, p);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_sim_mfma(const SimParams &p, int n_workgroups, hipStream_t st)
{
    const bool d128 = p.d == 128;
    switch (p.lay.variant) {
    case kMfmaWide:
        return d128 ? launch_cfg<Cfg<128, 2, 2, 2, 2>>(p, n_workgroups, st)
                    : launch_cfg<Cfg<64, 2, 2, 2, 2>>(p, n_workgroups, st);
    case kMfmaMid:
        return d128 ? launch_cfg<Cfg<128, 1, 4, 2, 2>>(p, n_workgroups, st)
                    : launch_cfg<Cfg<64, 1, 4, 2, 2>>(p, n_workgroups, st);
    case kMfmaSlim:
        return d128 ? launch_cfg<Cfg<128, 1, 4, 1, 4>>(p, n_workgroups, st)
                    : launch_cfg<Cfg<64, 1, 4, 1, 4>>(p, n_workgroups, st);
    default:
        return hipErrorInvalidValue;
    }
}

}  // namespace krul
