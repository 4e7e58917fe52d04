// bf16 MFMA similarity kernel for gfx950 (CDNA4).
//
// Work decomposition.  A "unit" is one (conversation, kv head): its (Hq/Hkv)*Tq
// query rows all read the same keys.  A workgroup (4 or 8 wavefronts) owns R_WG rows of a
// unit and one contiguous key split; it walks the split in key tiles of KT keys and,
// inside a tile, the layers 0..L-1 in order, so that every layer's logits are formed
// exactly once and the previous layer's exponentials of the same keys are still in
// registers when the cross term (the "ab" of Sec. 7's a^2 + b^2 - 2ab) is taken.
//
// K stream.  Per layer step the K tile arrives in NC chunks of CH keys.  Chunks are
// copied HBM -> LDS by buffer_load_dwordx4 ... lds (no register staging) into a ring of
// NBUF slots, NBUF-1 chunks ahead of the compute; one s_waitcnt + s_barrier per chunk
// publishes a slot.  Every slot is its own LDS object and every use names its slot
// statically, so the compiler can tell a copy in flight from the slot being read and
// adds no waits of its own.  Inside a slot 16-byte pieces are XOR-swizzled by row so
// that the 16-byte MFMA operand reads of 16 consecutive rows hit 16 different bank
// groups (the swizzle is applied on the global side: each lane fetches the piece that
// belongs in its LDS position).
//
// Math.  Per chunk each wave takes KBW blocks of 32 keys and RB blocks of 32 query rows:
//     S^T (32 keys x 32 rows) = K_blk (32 x d) * Q_blk^T (d x 32)
// with v_mfma_f32_32x32x16_bf16, A = keys (from LDS), B = query rows (registers, loaded
// once per layer step straight from global memory).  In the result every lane owns ONE
// query row (column lane%32) and 16 keys, so all softmax reductions are lane-local: no
// cross-lane traffic in the loop.  Lanes l and l+32 and the WK waves along the keys
// are independent partials of a row, merged once after the last tile.
//
// Online softmax uses a lazily updated reference exponent m per (lane, layer): it is
// raised only when a logit exceeds it by more than kLazy (in log2 units); the running
// sums Z and N2 are then rescaled.  The exponentials kept for the next layer's cross
// term are NOT rescaled: each 32-key block remembers the exponent it was formed under,
// the block's dot product with the next layer is kept apart, and the per-block factors
// of both layers are applied when the layer step ends.  Cosine and distance are
// invariant to the choice of m, and e = 2^(x-m) <= 2^kLazy keeps every sum far inside
// fp32 range.
#include "krul_common.h"

namespace krul {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr float kLazy = 16.0f;

template <int D_, int WR_, int WK_, int RB_, int KBW_, int NC_, int NBUF_>
struct Cfg {
    static constexpr int D = D_, WR = WR_, WK = WK_, RB = RB_, KBW = KBW_, NC = NC_, NBUF = NBUF_;
    static constexpr int NW = WR * WK;
    static constexpr int THREADS = NW * 64;
    static constexpr int R_WG = WR * RB * 32;      // query rows per workgroup
    static constexpr int CH = WK * KBW * 32;       // keys per chunk
    static constexpr int KT = CH * NC;             // keys per tile
    static constexpr int NBLK = NC * KBW;          // 32-key blocks per wave per tile
    static constexpr int KS = D / 16;              // MFMA k-steps per 32x32 block
    static constexpr int PPR = D / 8;              // 16-byte pieces per key row
    static constexpr int SLOT_BYTES = CH * D * 2;
    static constexpr int NLD = CH * PPR / THREADS; // direct-to-LDS loads per thread per chunk
    static constexpr int PF = NBUF - 1;            // chunks in flight ahead of the compute
    static_assert(NW == 4 || NW == 8, "four or eight waves per workgroup");
    static_assert(CH * PPR % THREADS == 0, "chunk must split evenly over threads");
    static_assert(NBUF == NC || NBUF == 2 * NC, "ring must be one or two tiles deep");
    static_assert(NBUF >= 2 && NBUF <= 4, "two to four ring slots");
    static_assert(D == 64 || D == 128, "head_dim 64 or 128");
};

// s_waitcnt immediates (gfx9 encoding: vmcnt [3:0]+[15:14], expcnt [6:4], lgkmcnt [11:8]).
constexpr int wait_vm(int n) { return (n & 15) | ((n >> 4) << 14) | 0x0F70; }
constexpr int kWaitLgkm0 = 0xC07F;

// Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous range of
// logical ids so that workgroups sharing K (neighbouring row tiles) share an L2.
__device__ inline int xcd_remap(int bid, int n)
{
    const int q = n >> 3, rem = n & 7, x = bid & 7;
    return x * q + min(x, rem) + (bid >> 3);
}

// Row-dependent XOR applied to the piece index inside an LDS slot.
template <int D>
__device__ inline int swz(int row)
{
    return D == 128 ? (row & 15) : ((row >> 1) & 7);
}

template <class C>
__global__ __launch_bounds__(C::THREADS, 2) void sim_mfma_kernel(SimParams p)
{
    constexpr int D = C::D, WK = C::WK, RB = C::RB, KBW = C::KBW, NC = C::NC, KS = C::KS;
    constexpr int NLD = C::NLD, NBUF = C::NBUF, PF = C::PF, PPR = C::PPR, NBLK = C::NBLK;
    __shared__ __attribute__((aligned(1024))) unsigned char ring0[C::SLOT_BYTES];
    __shared__ __attribute__((aligned(1024))) unsigned char ring1[C::SLOT_BYTES];
    __shared__ __attribute__((aligned(1024))) unsigned char ring2[NBUF > 2 ? C::SLOT_BYTES : 16];
    __shared__ __attribute__((aligned(1024))) unsigned char ring3[NBUF > 3 ? C::SLOT_BYTES : 16];
    __shared__ float red[C::NW][RB][4][32];
    auto slot_ptr = [&](int i) __attribute__((always_inline)) -> unsigned char * {
        switch (i) {   // i is a constant at every call site once the loops are unrolled
        case 0: return ring0;
        case 1: return ring1;
        case 2: return ring2;
        default: return ring3;
        }
    };

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keep it scalar
    const int wr = wave / WK, wk = wave % WK, half = lane >> 5, l32 = lane & 31;

    const int wg = xcd_remap(blockIdx.x, gridDim.x);
    const int nrt = p.lay.n_row_tiles, nsplit = p.lay.n_split;
    const int rt = wg % nrt, sp = (wg / nrt) % nsplit, u = wg / (nrt * nsplit);
    const int b = u / p.Hkv, kvh = u % p.Hkv;
    const int L = p.L, S = p.S, Rk = p.lay.rows_per_unit;

    const int key_begin = sp * p.keys_per_split;
    const int key_end = min(S, key_begin + p.keys_per_split);
    const int ntiles = (key_end - key_begin + C::KT - 1) / C::KT;
    const int nchunks = ntiles * L * NC;

    // ---- query rows of this lane (clamped; rows past the unit are never read back)
    const uint16_t *Qg = static_cast<const uint16_t *>(p.q);
    const uint16_t *Kg = static_cast<const uint16_t *>(p.k);
    const size_t q_layer_stride = (size_t)p.Hq * p.Tq * D;
    const size_t k_layer_stride = (size_t)p.Hkv * S * D;
    const uint16_t *qbase = Qg + ((size_t)b * L * p.Hq * p.Tq + (size_t)kvh * Rk) * D;
    unsigned qoff[RB];   // element offset of this lane's query row inside a layer
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
        qoff[rb] = (unsigned)(min(rt * C::R_WG + (wr * RB + rb) * 32 + l32, Rk - 1) * D + half * 8);
    const uint16_t *kbase = Kg + ((size_t)b * L * p.Hkv + kvh) * (size_t)S * D;

    // ---- K ring: wave-instruction j of this wave fills granules [(wave*NLD+j)*64, +64)
    // of a slot; the lane at granule g = row*PPR + pc fetches piece pc ^ swz(row) of row.
    // One wave-instruction covers 64/PPR whole rows (1 KB).  For instruction j the row is
    // ld_row0 + j*(64/PPR) (the j*1 KB step goes into the scalar offset of the load);
    // j*(64/PPR) occupies bits of the row number that are zero in
    // ld_row0 (all extents are powers of two), so the swizzle of row j is that of row 0
    // with xj(j) xor-ed in: one register (ld_off0) describes all of a lane's copies.
    constexpr int RPI = 64 / PPR;   // rows per wave-instruction
    const int ld_row0 = wave * NLD * RPI + lane / PPR;
    const int ld_colb0 = ((lane % PPR) ^ swz<D>(ld_row0)) * 16;
    const unsigned ld_off0 = (unsigned)(ld_row0 * (D * 2) + ld_colb0);   // unsigned: base + 32-bit offset addressing
    auto xj = [](int j) -> unsigned { return (unsigned)((D == 128 ? ((j * RPI) & 15) : (((j * RPI) >> 1) & 7)) * 16); };
    int pf_tile = 0, pf_l = 0, pf_c = 0;   // next chunk to fetch
    auto issue_chunk = [&](int slot) __attribute__((always_inline)) {
        unsigned char *dst = slot_ptr(slot);
        const int key0 = key_begin + pf_tile * C::KT + pf_c * C::CH;
        // Buffer addressing: a scalar descriptor for the rest of this layer's keys (rows past
        // the last key are out of range and are not fetched), one 32-bit offset per lane.
        const uint16_t *src = kbase + (size_t)pf_l * k_layer_stride + (size_t)key0 * D;
        const unsigned bytes = (unsigned)max(S - key0, 0) * (unsigned)(D * 2);
        const __amdgpu_buffer_rsrc_t rsrc =
            __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(src), 0, (int)bytes, 0x00020000);
#pragma unroll
        for (int j = 0; j < NLD; ++j)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(
                rsrc, (__attribute__((address_space(3))) void *)(dst + (wave * NLD + j) * 1024), 16,
                (int)(ld_off0 ^ xj(j)), j * 1024, 0, 0);
        // (the counters are wave-uniform; say so, to keep them in scalar registers)
        pf_c = pf_c + 1;
        if (pf_c == NC) {
            pf_c = 0;
            pf_l = pf_l + 1;
            if (pf_l == L) {
                pf_l = 0;
                pf_tile = pf_tile + 1;
            }
        }
    };

    bf16x8 qf[RB][KS];
    auto load_q = [&](int l) __attribute__((always_inline)) {
        const uint16_t *ql = qbase + (size_t)l * q_layer_stride;
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                qf[rb][ks] = *reinterpret_cast<const bf16x8 *>(ql + qoff[rb] + ks * 16);
    };

    // per-lane running records between key tiles (only when the split spans several tiles)
    float4 *spill = p.spill;
    auto spill_index = [&](int l, int rb) -> size_t {
        return (((((size_t)wg * L + l) * C::NW + wave) * RB + rb) << 6) + lane;
    };

    float e[RB][NBLK][16];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int c = 0; c < NBLK; ++c)
#pragma unroll
            for (int v = 0; v < 16; ++v) e[rb][c][v] = 0.f;

    // LDS read offset of this lane inside a 32-key block: row l32, piece (2*ks + half) ^ swz
    // = l32*(D*2) + (((2*ks) ^ a_hs) << 4) = a_base ^ (ks << 5), a_hs = half ^ swz(l32)
    const int a_base = l32 * (D * 2) + ((half ^ swz<D>(l32)) << 4);

    // ---- prologue: PF chunks in flight, query rows of layer 0
    int n_issued = 0, n_done = 0;
#pragma unroll
    for (int i = 0; i < PF; ++i)
        if (n_issued < nchunks) {
            issue_chunk(i);
            ++n_issued;
        }
    load_q(0);

    const float cs = p.c;
    float f_prev[RB], mrg_prev[RB];
    float sprev[RB][NBLK];    // previous layer step: 2^(block exponent - final exponent)
    bool raised_prev = false;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        f_prev[rb] = mrg_prev[rb] = 1.f;
#pragma unroll
        for (int k2 = 0; k2 < NBLK; ++k2) sprev[rb][k2] = 1.f;
    }

    int step = 0;   // layer steps done; its parity selects the ring half when NBUF == 2*NC
    for (int tile = 0; tile < ntiles; ++tile) {
        const int tile_key0 = key_begin + tile * C::KT;
        const bool ragged = tile_key0 + C::KT > key_end;
        const bool last_tile = tile == ntiles - 1;

        // One layer step; par (the step's parity) is a constant in each inlined copy, so
        // every ring slot named below is a fixed LDS object.
        auto layer_step = [&](const int par, const int l) __attribute__((always_inline)) {
            float4 rec[RB];
            float mcur[RB], tz[RB], tn[RB];
            float mb[RB][NBLK], dot[RB][NBLK];   // per block: exponent used, dot with previous layer
            bool raised = false;                 // some lane raised m during this step (wave-uniform)
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                rec[rb] = tile > 0 ? spill[spill_index(l, rb)] : make_float4(kMInit, 0.f, 0.f, 0.f);
                mcur[rb] = rec[rb].x;
                tz[rb] = tn[rb] = 0.f;
            }
            const int ring_half = (NBUF == NC) ? 0 : par * NC;
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                // Chunk (step, c) must have landed.  Loads return in order, so it is enough
                // that no more loads are outstanding than the younger chunks account for.
                // At the first chunk of a step the query rows loaded during the previous chunk
                // (issued before that chunk's copy) must be complete too: allow one younger
                // chunk only, which also tells the compiler's wait pass that they have landed.
                const int younger = n_issued - 1 - n_done;
                if (PF >= 3 && younger >= 2 && c != 0)
                    __builtin_amdgcn_s_waitcnt(wait_vm(2 * NLD));
                else if (PF >= 2 && younger >= 1)
                    __builtin_amdgcn_s_waitcnt(wait_vm(NLD));
                else
                    __builtin_amdgcn_s_waitcnt(wait_vm(0));
                __builtin_amdgcn_s_barrier();
                n_done = n_done + 1;
                const bool more = n_issued < nchunks;
                if (c != NC - 1 && more) {
                    issue_chunk((ring_half + c + PF) % NBUF);
                    n_issued = n_issued + 1;
                }

                const unsigned char *slot = slot_ptr(ring_half + c);
                // Logits of all this wave's blocks first, the independent accumulator chains
                // interleaved so that no MFMA waits for the one issued just before it ...
                f32x16 acc[KBW][RB];
#pragma unroll
                for (int kb = 0; kb < KBW; ++kb)
#pragma unroll
                    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                        for (int v = 0; v < 16; ++v) acc[kb][rb][v] = 0.f;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                    for (int kb = 0; kb < KBW; ++kb) {
                        const unsigned char *kbp = slot + (wk * KBW + kb) * 32 * (D * 2);
                        const bf16x8 a = *reinterpret_cast<const bf16x8 *>(kbp + (a_base ^ (ks << 5)));
#pragma unroll
                        for (int rb = 0; rb < RB; ++rb)
                            acc[kb][rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[rb][ks], acc[kb][rb], 0, 0, 0);
                    }
                if (c == NC - 1) {
                    // the old query rows are dead once the MFMAs above have issued
                    load_q(l + 1 == L ? 0 : l + 1);   // next step's query rows
                    if (more) {                        // ring loads stay the youngest loads
                        issue_chunk((ring_half + c + PF) % NBUF);
                        n_issued = n_issued + 1;
                    }
                }

                // ... then the softmax statistics and cross terms, block by block.
#pragma unroll
                for (int kb = 0; kb < KBW; ++kb) {
                    const int blk = c * KBW + kb;
#pragma unroll
                    for (int rb = 0; rb < RB; ++rb) {
                        if (ragged) {
                            // keys at or past key_end: element v of this lane is key kb0 + 8*(v/4) + v%4
                            int lim = key_end - (tile_key0 + c * C::CH + (wk * KBW + kb) * 32 + half * 4);
                            asm volatile("" : "+v"(lim));   // keep the 16 compares here, not hoisted
#pragma unroll
                            for (int v = 0; v < 16; ++v)
                                if (8 * (v >> 2) + (v & 3) >= lim) acc[kb][rb][v] = -INFINITY;
                        }
                        float tmax = acc[kb][rb][0];
#pragma unroll
                        for (int v = 1; v < 16; ++v) tmax = fmaxf(tmax, acc[kb][rb][v]);
                        const float xm = tmax * cs;
                        if (__any(xm > mcur[rb] + kLazy)) {
                            const float mnew = fmaxf(mcur[rb], xm);
                            const float f = __builtin_amdgcn_exp2f(mcur[rb] - mnew);
                            tz[rb] *= f;
                            tn[rb] *= f * f;
                            mcur[rb] = mnew;
                            raised = true;
                        }
                        mb[rb][blk] = mcur[rb];
                        const float negm = -mcur[rb];
                        float bz = 0.f, bn = 0.f, bd = 0.f;
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            const float ev = __builtin_amdgcn_exp2f(fmaf(acc[kb][rb][v], cs, negm));
                            bz += ev;
                            bn = fmaf(ev, ev, bn);
                            bd = fmaf(ev, e[rb][blk][v], bd);
                            e[rb][blk][v] = ev;
                        }
                        tz[rb] += bz;
                        tn[rb] += bn;
                        dot[rb][blk] = bd;
                    }
                }
            }

            // ---- cross term of this tile: block dots, each brought to the final exponents of
            // both layers (the factors are 1 unless some m was raised in this or the last step)
            float tc[RB];
            if (raised || raised_prev) {
#pragma unroll
                for (int rb = 0; rb < RB; ++rb) {
                    tc[rb] = 0.f;
#pragma unroll
                    for (int k2 = 0; k2 < NBLK; ++k2) {
                        const float sc = __builtin_amdgcn_exp2f(mb[rb][k2] - mcur[rb]);
                        tc[rb] = fmaf(dot[rb][k2], sc * sprev[rb][k2], tc[rb]);
                        sprev[rb][k2] = sc;
                    }
                }
            } else {
#pragma unroll
                for (int rb = 0; rb < RB; ++rb) {
                    tc[rb] = 0.f;
#pragma unroll
                    for (int k2 = 0; k2 < NBLK; ++k2) tc[rb] += dot[rb][k2];
                }
            }
            raised_prev = raised;

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
                float M[RB];
#pragma unroll
                for (int rb = 0; rb < RB; ++rb) M[rb] = fmaxf(out[rb].x, __shfl_xor(out[rb].x, 32, 64));
                if (WK > 1) {
#pragma unroll
                    for (int rb = 0; rb < RB; ++rb)
                        red[wave][rb][0][l32] = M[rb];   // both half-waves hold the same value
                    __builtin_amdgcn_s_waitcnt(kWaitLgkm0);
                    __builtin_amdgcn_s_barrier();
#pragma unroll
                    for (int rb = 0; rb < RB; ++rb) {
                        M[rb] = red[wr * WK][rb][0][l32];
#pragma unroll
                        for (int w2 = 1; w2 < WK; ++w2) M[rb] = fmaxf(M[rb], red[wr * WK + w2][rb][0][l32]);
                    }
                }
                float zs[RB], ns[RB], cc2[RB];
#pragma unroll
                for (int rb = 0; rb < RB; ++rb) {
                    const float f = __builtin_amdgcn_exp2f(out[rb].x - M[rb]);
                    float z = out[rb].y * f, nn = out[rb].z * f * f, cc = out[rb].w * f * mrg_prev[rb];
                    mrg_prev[rb] = f;
                    zs[rb] = z + __shfl_xor(z, 32, 64);
                    ns[rb] = nn + __shfl_xor(nn, 32, 64);
                    cc2[rb] = cc + __shfl_xor(cc, 32, 64);
                }
                if (WK > 1) {
#pragma unroll
                    for (int rb = 0; rb < RB; ++rb) {   // both half-waves hold the same sums
                        red[wave][rb][1][l32] = zs[rb];
                        red[wave][rb][2][l32] = ns[rb];
                        red[wave][rb][3][l32] = cc2[rb];
                    }
                    __builtin_amdgcn_s_waitcnt(kWaitLgkm0);
                    __builtin_amdgcn_s_barrier();
#pragma unroll
                    for (int rb = 0; rb < RB; ++rb) {
                        zs[rb] = ns[rb] = cc2[rb] = 0.f;
#pragma unroll
                        for (int w2 = 0; w2 < WK; ++w2) {
                            zs[rb] += red[wr * WK + w2][rb][1][l32];
                            ns[rb] += red[wr * WK + w2][rb][2][l32];
                            cc2[rb] += red[wr * WK + w2][rb][3][l32];
                        }
                    }
                    // red is next written after the following layer step's chunk barriers
                }
                if (wk == 0) {   // wave-uniform; lanes l and l+32 store the same record
#pragma unroll
                    for (int rb = 0; rb < RB; ++rb) {
                        const size_t idx = ((size_t)wg * L + l) * C::R_WG + (wr * RB + rb) * 32 + l32;
                        p.state[idx] = make_float4(M[rb], zs[rb], ns[rb], cc2[rb]);
                    }
                }
            }
        };

        for (int l = 0; l < L; ++l, ++step) {
            if (NBUF == NC || !(step & 1))
                layer_step(0, l);
            else
                layer_step(1, l);
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

// Tile shapes (rows x keys per workgroup tile) must match make_plan().
//           D  WR WK RB KBW NC NBUF
typedef Cfg<128, 4, 1, 1, 2, 2, 2> Wide128;   // 128 x 128, 4 waves, ring 2 x  64 keys ( 32 KB)
typedef Cfg<64, 4, 1, 1, 2, 2, 2> Wide64;
typedef Cfg<128, 2, 4, 1, 2, 2, 2> Mid128;    //  64 x 512, 8 waves, ring 2 x 256 keys (128 KB)
typedef Cfg<64, 2, 4, 1, 2, 2, 4> Mid64;      //  64 x 512, 8 waves, ring 4 x 256 keys (128 KB)
typedef Cfg<128, 1, 8, 1, 1, 2, 2> Slim128;   //  32 x 512, 8 waves, ring 2 x 256 keys (128 KB)
typedef Cfg<64, 1, 8, 1, 1, 2, 4> Slim64;     //  32 x 512, 8 waves, ring 4 x 256 keys (128 KB)

hipError_t launch_sim_mfma(const SimParams &p, int n_workgroups, hipStream_t st)
{
    const bool d128 = p.d == 128;
    switch (p.lay.variant) {
    case kMfmaWide:
        return d128 ? launch_cfg<Wide128>(p, n_workgroups, st) : launch_cfg<Wide64>(p, n_workgroups, st);
    case kMfmaMid:
        return d128 ? launch_cfg<Mid128>(p, n_workgroups, st) : launch_cfg<Mid64>(p, n_workgroups, st);
    case kMfmaSlim:
        return d128 ? launch_cfg<Slim128>(p, n_workgroups, st) : launch_cfg<Slim64>(p, n_workgroups, st);
    default:
        return hipErrorInvalidValue;
    }
}

}  // namespace krul
