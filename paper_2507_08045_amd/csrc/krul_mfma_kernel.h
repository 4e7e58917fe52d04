// 16-bit (bfloat16 or IEEE binary16) MFMA similarity kernel for gfx950 (CDNA4).
//
// Work decomposition.  A "unit" is one (conversation, kv head): its (Hq/Hkv)*Tq
// query rows all read the same keys.  A workgroup (8 wavefronts, WR x WK) owns R_WG rows
// of a unit and one contiguous key split; it walks the split in key tiles of KT keys and,
// inside a tile, the layers 0..L-1 in order, so that every layer's logits are formed
// exactly once and the previous layer's exponentials of the same keys are still in
// registers when the cross term (the "ab" of Sec. 7's a^2 + b^2 - 2ab) is taken.
//
// Streams.  A key tile is NC chunks of CH keys; chunk c of a layer step lives in ring slot
// c.  Chunks, and the next layer's query rows, are copied HBM -> LDS by
// buffer_load_dwordx4 ... lds (no register staging); the copy issued while chunk c of a
// step is worked on is chunk c of the next step, i.e. NC-1 chunks ahead.  One count-based
// s_waitcnt + one s_barrier per chunk publish a slot.  Every slot is its own LDS object
// and every use names its slot statically, so the compiler can tell a copy in flight
// from the slot being read and adds no waits of its own.  Inside a slot 16-byte pieces
// are XOR-swizzled by row so that the 16-byte MFMA operand reads of 16 consecutive rows
// hit 16 different bank groups (the swizzle is applied on the global side: each lane
// fetches the piece that belongs in its LDS position).
//
// Math.  Per chunk each wave takes KBW blocks of 32 keys against its 32 query rows:
//     S^T (32 keys x 32 rows) = K_blk (32 x d) * Q_blk^T (d x 32)
// with v_mfma_f32_32x32x16_bf16, A = keys (from LDS), B = query rows (registers, read once
// per layer step from their LDS staging area).  In the result every lane owns ONE query
// row (column lane%32) and 16 keys, so all softmax sums are lane-local: no cross-lane
// traffic in the loop.  Lanes l and l+32 and the WK waves along the keys are independent
// partials of a row, merged one step late by the first wave of each wave row.
//
// Software pipeline.  While a wave takes the exponentials of chunk c's block it issues the
// MFMA chain that forms chunk c+1's logits (double-buffered accumulators); the order
// "one MFMA, the vector work of 16/KS logits, ..." is pinned with empty asm statements.
//
// Online softmax uses a reference exponent m per (lane, layer) that is only raised when
// it has to be: a block is taken under the current m and, if its sum of squares shows an
// exponential above 2^kLazy (or an overflow), m is raised to the block maximum, the
// running sums are rescaled and the block is redone.  The exponentials kept for the next
// layer's cross term are NOT rescaled: each 32-key block remembers the exponent it was
// formed under, the block's dot product with the next layer is kept apart, and the
// per-block factors of both layers are applied when the layer step ends.  Cosine and
// distance are invariant to the choice of m, and e = 2^(x-m) <= 2^kLazy keeps every sum
// far inside fp32 range.
#pragma once
#include "krul_common.h"

namespace krul {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;   // eight 16-bit elements (bfloat16, or binary16 bits)
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr float kLazy = 16.0f;
constexpr float kBig = 4294967296.0f;   // 2^(2*kLazy): bound on a block's sum of squared exponentials

template <int D_, int WR_, int WK_, int KBW_, int NC_>
struct Cfg {
    static constexpr int D = D_, WR = WR_, WK = WK_, KBW = KBW_;
    static constexpr int NC = NC_;                 // chunks per key tile = ring slots
    static constexpr int PF = NC - 1;              // chunks in flight ahead of the MFMAs
    static constexpr int NW = WR * WK;
    static constexpr int THREADS = NW * 64;
    static constexpr int R_WG = WR * 32;           // query rows per workgroup
    static constexpr int CH = WK * KBW * 32;       // keys per chunk
    static constexpr int KT = CH * NC;             // keys per tile
    static constexpr int NBLK = NC * KBW;          // 32-key blocks per wave per tile
    static constexpr int KS = D / 16;              // MFMA k-steps per 32x32 block
    static constexpr int PPR = D / 8;              // 16-byte pieces per row
    static constexpr int RPI = 64 / PPR;           // rows covered by one 1 KB wave-instruction
    static constexpr int SLOT_BYTES = CH * D * 2;
    static constexpr int SLOT_ALIGN = SLOT_BYTES < 16384 ? SLOT_BYTES : 16384;
    static constexpr int NLD = CH * PPR / THREADS; // direct-to-LDS loads per thread per chunk
    static constexpr int QBYTES = 32 * D * 2;      // the 32 query rows of one wave row
    static constexpr int NQI = 32 / RPI;           // wave-instructions that copy them
    static constexpr int QPW = (NQI + WK - 1) / WK;   // ... of which each of the WK waves issues
    static_assert(NW == 4 || NW == 8, "four or eight waves per workgroup");
    static_assert(CH * PPR % THREADS == 0, "chunk must split evenly over threads");
    static_assert(D == 64 || D == 128, "head_dim 64 or 128");
    static_assert(NC == 2 || NC == 4, "two or four chunks per tile");
    static_assert(NC == 2 || WK * QPW == NQI, "every wave must issue the same number of copies");
};

// s_waitcnt immediates (gfx9 encoding: vmcnt [3:0]+[15:14], expcnt [6:4], lgkmcnt [11:8]).
constexpr int wait_vm(int n) { return (n & 15) | ((n >> 4) << 14) | 0x0F70; }
constexpr int wait_vm_lgkm0(int n) { return (n & 15) | ((n >> 4) << 14) | 0x0070; }   // ... and lgkmcnt(0)
constexpr int kWaitLgkm0 = 0xC07F;

// Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous range of
// logical ids so that workgroups sharing K (neighbouring row tiles) share an L2.
__device__ inline int xcd_remap(int bid, int n)
{
    const int q = n >> 3, rem = n & 7, x = bid & 7;
    return x * q + min(x, rem) + (bid >> 3);
}

// Row-dependent XOR applied to the piece index inside an LDS tile of rows.
template <int D>
__device__ inline int swz(int row)
{
    return D == 128 ? (row & 15) : ((row >> 1) & 7);
}

// MODE 0: cosine only; 1: also Z = sum e (needed for the distance); 2: also Zir = sum of e over the
// initial and recent keys (the Initial-Recent layer test of Sec. 4.2), which needs Z too
// A wave-uniform address, said to be so: descriptors built from it then stay in scalar registers.
__device__ inline const uint16_t *uniform_ptr(const uint16_t *ptr)
{
    const uintptr_t a = (uintptr_t)ptr;
    return (const uint16_t *)(((uintptr_t)(unsigned)__builtin_amdgcn_readfirstlane((int)(a >> 32)) << 32) |
                              (uintptr_t)(unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)a));
}

// One 32x32x16 step on eight 16-bit elements per lane and operand: bfloat16, or (F16) IEEE binary16 --
// same operand layout, same rate, so the kernel is the same for both.
template <bool F16>
__device__ inline f32x16 mfma_16bit(bf16x8 a, bf16x8 b, f32x16 c)
{
    if constexpr (F16)
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// KA: how the keys are addressed.  0: dense [B][L][Hkv][S][d].  1: one allocation per layer (a device
// table of pointers) and strides between conversations, kv heads and keys.  2: one pool of pages per
// layer, a block table per conversation, strides between pages, kv heads and the keys of a page.
template <class C, int MODE, int KA, bool F16>
__global__ __launch_bounds__(C::THREADS, 2) void sim_mfma_kernel(SimParams p)
{
    constexpr int D = C::D, WK = C::WK, KBW = C::KBW, NC = C::NC, KS = C::KS;
    constexpr bool WZ = MODE >= 1, IR = MODE == 2;
    constexpr int NLD = C::NLD, PPR = C::PPR, NBLK = C::NBLK, RPI = C::RPI, PF = C::PF;
    // (the larger alignment puts the ring first in the workgroup's LDS, within reach of the
    // 16-bit offset field of the operand reads)
    __shared__ __attribute__((aligned(C::SLOT_ALIGN))) unsigned char ring0[C::SLOT_BYTES];
    __shared__ __attribute__((aligned(C::SLOT_ALIGN))) unsigned char ring1[C::SLOT_BYTES];
    __shared__ __attribute__((aligned(C::SLOT_ALIGN))) unsigned char ring2[NC > 2 ? C::SLOT_BYTES : 16];
    __shared__ __attribute__((aligned(C::SLOT_ALIGN))) unsigned char ring3[NC > 2 ? C::SLOT_BYTES : 16];
    __shared__ __attribute__((aligned(1024))) unsigned char qlds[C::WR * C::QBYTES];
    __shared__ float4 part[C::NW][64];   // every lane's record of the last step (m, Z, N2, C)
    __shared__ float part_ir[IR ? C::NW : 1][64];   // ... and its Zir
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

    const int nrt = p.lay.n_row_tiles, nsplit = p.lay.n_split;
    int rt, sp, u;
    {
        // the XCD's next workgroup in its contiguous range of logical ids; inside a unit the ids run patch
        // by patch (see patch_rows()), inside a patch row tile first
        const int w = xcd_remap(blockIdx.x, gridDim.x);
        const int per_unit = nrt * nsplit, r = w % per_unit;
        u = w / per_unit;
        const int pr = patch_rows(nrt, nsplit);
        if (pr) {
            const int ps = 32 / pr, j = r % 32, pt = r / 32, prt = pt % (nrt / pr), psp = pt / (nrt / pr);
            rt = prt * pr + j % pr;
            sp = psp * ps + j / pr;
        } else {
            rt = r % nrt;
            sp = r / nrt;
        }
    }
    // where this workgroup's records go: by (unit, key split, row tile), whatever order the workgroups run in
    const int wg = (u * nsplit + sp) * nrt + rt;
    const int b = u / p.Hkv, kvh = u % p.Hkv;
    const int L = p.L, S = p.S, Rk = p.lay.rows_per_unit;

    const int key_begin = sp * p.keys_per_split;
    int key_end = min(S, key_begin + p.keys_per_split);
    if (p.causal) {
        // no row of this workgroup sees a key past the last position among its rows: stop there
        // (at least one key stays, so that every row still gets its -- then empty -- records)
        const int r_lo = rt * C::R_WG, r_hi = min(r_lo + C::R_WG, Rk) - 1;
        const int t_max = r_lo / p.Tq != r_hi / p.Tq ? p.Tq - 1 : r_hi % p.Tq;
        key_end = max(min(key_end, S - p.Tq + t_max + 1), key_begin + 1);
    }
    // causal reading: this lane's query row t (of its head's Tq rows) sees the keys j < row_end
    const int row_end = p.causal ? S - p.Tq + min(rt * C::R_WG + wr * 32 + l32, Rk - 1) % p.Tq + 1 : S;
    const int ntiles = (key_end - key_begin + C::KT - 1) / C::KT;
    const int nsteps = ntiles * L;          // layer steps; at least 2
    const int nchunks = nsteps * NC;        // at least 4

    const uint16_t *Qg = static_cast<const uint16_t *>(p.q);
    const uint16_t *Kg = static_cast<const uint16_t *>(p.k);
    constexpr bool SK = KA != 0;   // keys with strides, layers from a table
    // Head size in memory: the kernel's D, or (SK) any multiple of 8 up to it.  Rows are copied piece by
    // piece into the D-wide LDS rows; the pieces a shorter row does not have are left to lanes whose
    // offset lies outside every range, which fetch nothing and write zero, so the MFMAs run over D as ever.
    const int dq = SK ? p.d : D;
    [[maybe_unused]] const unsigned d_bytes = (unsigned)dq * 2u;
    [[maybe_unused]] const unsigned pp_real = (unsigned)dq >> 3;   // 16-byte pieces of a row in memory
    constexpr unsigned kNoFetch = 0x7FFFFFF0u;
    const size_t q_layer_stride = (size_t)p.Hq * p.Tq * dq;
    // Keys of layer l, this unit: k_layer(l) + k_tile_off, where k_tile_off leads to the unit's first key
    // of the tile being fetched (see SimParams).  Layer and tile advance by additions, so that the dense
    // layout costs no multiplications inside the loop.
    const size_t k_stride_s = SK ? (size_t)p.k_stride_s : (size_t)D;
    // (paged: the page and the key inside it are added per copy instruction; only the head is fixed)
    size_t k_tile_off = KA == 2 ? (size_t)kvh * p.k_stride_h
                                : (size_t)b * p.k_stride_b + (size_t)kvh * p.k_stride_h + (size_t)key_begin * k_stride_s;
    const size_t k_tile_step = KA == 2 ? 0 : (size_t)C::KT * k_stride_s;
    const uint16_t *k_dense = Kg;   // dense layout: the layer being fetched starts here
    auto k_layer = [&](int l) __attribute__((always_inline)) -> const uint16_t * {
        // the table is read as constant memory at a uniform address: a scalar load, which takes no place in
        // the vector-memory queue that the ring's waits count
        typedef const __attribute__((address_space(4))) unsigned long long *const_u64_ptr;
        // (SK without a table: the dense layout with a head size below D)
        return SK && p.k_tab ? (const uint16_t *)(uintptr_t)((const_u64_ptr)(uintptr_t)p.k_tab)[l] : k_dense;
    };
    const unsigned k_row_bytes = (unsigned)k_stride_s * 2u;   // (dense: 2*D, the swizzle bits stay clear)
    const unsigned k_chunk_bytes = (unsigned)C::CH * k_row_bytes;   // (a layer's keys of one head span < 2 GiB)

    // ---- direct-to-LDS copies.  One wave-instruction moves 1 KB = RPI whole rows: the lane
    // at LDS granule g = row*PPR + pc fetches piece pc ^ swz(row) of its row (the swizzle is
    // applied on the global side).  For instruction j of a lane the row is row0 + j*RPI;
    // j*RPI occupies bits of the row number that are zero in row0 (all extents are powers
    // of two), so its swizzle is that of row0 with xj(j) xor-ed in, and the j*1 KB step goes
    // into the scalar offset of the load: one register per lane describes all its copies.
    auto xj = [](int j) -> unsigned { return (unsigned)((D == 128 ? ((j * RPI) & 15) : (((j * RPI) >> 1) & 7)) * 16); };

    // K ring: wave-instruction j of this wave fills granules [(wave*NLD+j)*64, +64) of a slot.
    const int ld_row0 = wave * NLD * RPI + lane / PPR;
    [[maybe_unused]] const unsigned ld_off0 = (unsigned)ld_row0 * k_row_bytes + (unsigned)(((lane % PPR) ^ swz<D>(ld_row0)) * 16);
    // The chunk copied during chunk c of a step is chunk c of the NEXT step (PF + 1 = NC chunks
    // later), so per step one base address serves all its copies: that of the next step's
    // layer and key tile (fetch_k), with the tile's first key (fetch_key0).
    const uint16_t *fetch_k = uniform_ptr(k_layer(0) + k_tile_off);
    int fetch_key0 = key_begin;
    // SK: the lane offset of copy instruction j, worked out piece by piece (any row pitch, any head size):
    // the lane's LDS granule holds piece pj of its row, if the row has it
    [[maybe_unused]] auto k_lane_off = [&](int j, unsigned row_off) -> unsigned {
        const unsigned pj = (unsigned)((lane % PPR) ^ swz<D>(ld_row0)) ^ (xj(j) >> 4);
        return pj < pp_real ? row_off + pj * 16u : kNoFetch;
    };
    // Paged keys: a copy instruction moves RPI whole keys, which lie in one page (pages hold a power of
    // two >= 8 keys and tiles start on multiples of them); its page comes from the conversation's block
    // table by a scalar load, and it gets a descriptor of its own, bounded by the keys that exist.
    // (On this chip the scalar offset of a buffer instruction takes part in the range check, like the
    // lane offset: the dense path below relies on that.)
    typedef const __attribute__((address_space(4))) int *const_i32_ptr;
    const const_i32_ptr page_row = KA == 2 ? (const_i32_ptr)(uintptr_t)(p.block_table + (size_t)b * p.max_blocks) : nullptr;
    // Where each copy instruction of a tile starts, relative to the layer's pool (wave-uniform, in scalar
    // registers).  Every layer has the same pages, so the table is read once per tile, not once per
    // layer step: a lookup inside the step would make the wave wait for the scalar load at every chunk.
    long long page_off[KA == 2 ? NC : 1][KA == 2 ? NLD : 1];   // in elements
    auto load_pages = [&](int tile_key0) __attribute__((always_inline)) {
        if constexpr (KA == 2) {
            const int wave_u = __builtin_amdgcn_readfirstlane(wave);
#pragma unroll
            for (int c = 0; c < NC; ++c)
#pragma unroll
                for (int j = 0; j < NLD; ++j) {
                    const int kcl = min(tile_key0 + c * C::CH + (wave_u * NLD + j) * RPI, S - 1);   // (stay inside the table row)
                    page_off[c][j] = (long long)page_row[kcl >> p.page_shift] * p.k_stride_page +
                                     (long long)(kcl & ((1 << p.page_shift) - 1)) * (long long)k_stride_s;
                }
        }
    };
    load_pages(key_begin);
    const unsigned page_copy_bytes = (unsigned)(RPI - 1) * k_row_bytes + d_bytes;
    auto issue_chunk = [&](int c, bool live) __attribute__((always_inline)) {
        unsigned char *dst = slot_ptr(c);
        const int key0 = fetch_key0 + c * C::CH;
        if constexpr (KA == 2) {
            const int wave_u = __builtin_amdgcn_readfirstlane(wave);
#pragma unroll
            for (int j = 0; j < NLD; ++j) {
                const int krow = key0 + (wave_u * NLD + j) * RPI;        // first key of this instruction
                const uint16_t *base = fetch_k + page_off[c][j];
                // All RPI keys or none: a page has room for all its keys, so the ones past the last key of
                // the conversation can be read (they are masked like any key a row does not see), and the
                // range needs no arithmetic.  (A clamp to the keys that exist would also be selected as a
                // vector instruction, which makes the descriptor a per-lane value issued in a retry loop.)
                const unsigned bytes = live && krow < S ? page_copy_bytes : 0u;
                const __amdgpu_buffer_rsrc_t rsrc =
                    __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(base), 0, (int)bytes, 0x00020000);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(
                    rsrc, (__attribute__((address_space(3))) void *)(dst + (wave * NLD + j) * 1024), 16,
                    (int)k_lane_off(j, (unsigned)(lane / PPR) * k_row_bytes), 0, 0, 0);
            }
            return;
        }
        // Buffer addressing: a scalar descriptor for the rest of this layer's keys (rows past
        // the last key are out of range and are not fetched), one 32-bit offset per lane.
        // (a chunk past the end of the split gets an empty range: nothing is fetched)
        const unsigned bytes = live && key0 < S ? (unsigned)(S - key0 - 1) * k_row_bytes + (SK ? d_bytes : (unsigned)(D * 2)) : 0u;
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint16_t *>(fetch_k + (c * k_chunk_bytes) / 2), 0, (int)bytes, 0x00020000);
#pragma unroll
        for (int j = 0; j < NLD; ++j)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(
                rsrc, (__attribute__((address_space(3))) void *)(dst + (wave * NLD + j) * 1024), 16,
                SK ? (int)k_lane_off(j, (unsigned)ld_row0 * k_row_bytes) : (int)(ld_off0 ^ xj(j)),
                (int)(j * RPI * k_row_bytes), 0, 0);
    };

    // Query rows: the 32 rows of wave row wr are staged in LDS (laid out like a 32-key block)
    // by the WK waves that share them, one layer step ahead, and read into registers from
    // there.  Rows past the end of the unit are out of the descriptor's range: they are not
    // fetched, their results are never read back.
    const int r0 = rt * C::R_WG + wr * 32;
    const int q_rows = min(max(Rk - r0, 0), 32);
    const uint16_t *qbase = uniform_ptr(Qg + ((size_t)b * L * p.Hq * p.Tq + (size_t)kvh * Rk + (size_t)(q_rows ? r0 : 0)) * dq);
    [[maybe_unused]] const unsigned q_off0 = (unsigned)((lane / PPR) * (D * 2) + (((lane % PPR) ^ swz<D>(lane / PPR)) * 16));
    const uint16_t *fetch_q = qbase;   // query rows of the next step's layer
    auto issue_q = [&](bool live) __attribute__((always_inline)) {
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint16_t *>(fetch_q), 0, __builtin_amdgcn_readfirstlane(live ? q_rows * (int)(SK ? d_bytes : (unsigned)(D * 2)) : 0), 0x00020000);
        unsigned char *dst = qlds + wr * C::QBYTES;
#pragma unroll
        for (int jj = 0; jj < C::QPW; ++jj) {
            const int j = wk * C::QPW + jj;
            if (j < C::NQI) {
                if constexpr (SK) {   // piece by piece, as for the keys
                    const unsigned pj = (unsigned)((lane % PPR) ^ swz<D>(lane / PPR)) ^ (xj(j) >> 4);
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(
                        rsrc, (__attribute__((address_space(3))) void *)(dst + j * 1024), 16,
                        (int)(pj < pp_real ? (unsigned)(lane / PPR) * d_bytes + pj * 16u : kNoFetch),
                        (int)((unsigned)(j * RPI) * d_bytes), 0, 0);
                } else {
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(
                        rsrc, (__attribute__((address_space(3))) void *)(dst + j * 1024), 16,
                        (int)(q_off0 ^ xj(j)), j * 1024, 0, 0);
                }
            }
        }
    };

    // LDS read offset of this lane inside a 32-row block: row l32, piece (2*ks + half) ^ swz
    // = l32*(D*2) + (((2*ks) ^ a_hs) << 4) = a_base ^ (ks << 5), a_hs = half ^ swz(l32)
    const int a_base = l32 * (D * 2) + ((half ^ swz<D>(l32)) << 4);
    // ... and the same inside this wave's first 32-key block of a chunk (a whole number of
    // 32-row blocks further on: the bits the k-step toggles are not touched)
    const int ka_base = a_base + wk * KBW * 32 * (D * 2);

    bf16x8 qf[KS];
    auto read_q = [&]() __attribute__((always_inline)) {
        const unsigned char *src = qlds + wr * C::QBYTES;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[ks] = *reinterpret_cast<const bf16x8 *>(src + (a_base ^ (ks << 5)));
    };
    // logits of 32-key block kb of the chunk in `slot` for this lane's query row
    auto logits = [&](const unsigned char *slot, int kb) __attribute__((always_inline)) -> f32x16 {
        const unsigned char *kbp = slot + kb * 32 * (D * 2);
        f32x16 a;
#pragma unroll
        for (int v = 0; v < 16; ++v) a[v] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            a = mfma_16bit<F16>(*reinterpret_cast<const bf16x8 *>(kbp + (ka_base ^ (ks << 5))), qf[ks], a);
        return a;
    };

    // Splits that span several key tiles: a row's running record (layer l, all keys so far) is the row
    // record the merge below stores after every tile; at the next tile ONE of the row's partials -- the
    // first half-wave of the first wave along the keys -- takes it up again, the others start empty.
    const bool carries = wk == 0 && half == 0;
    const size_t row_rec = (size_t)wg * L * C::R_WG + wr * 32 + l32;   // + l * R_WG: this lane's row, layer l

    float e[NBLK][16];
#pragma unroll
    for (int c = 0; c < NBLK; ++c)
#pragma unroll
        for (int v = 0; v < 16; ++v) e[c][v] = 0.f;

    // ---- prologue: query rows of layer 0 and the first NC chunks (there are at least 2*NC);
    // logits of chunk 0
    issue_q(true);
#pragma unroll
    for (int i = 0; i < NC; ++i) issue_chunk(i, true);
    __builtin_amdgcn_s_waitcnt(wait_vm(PF * NLD));   // all but the chunks after chunk 0 (loads return in order)
    __builtin_amdgcn_s_barrier();
    read_q();
    f32x16 acc[2][KBW];
#pragma unroll
    for (int kb = 0; kb < KBW; ++kb) acc[0][kb] = logits(slot_ptr(0), kb);

    const float cs = p.c;
    float f_prev = 1.f;
    float sprev[NBLK];    // previous layer step: 2^(block exponent - final exponent)
    bool raised_prev = false;
#pragma unroll
    for (int k2 = 0; k2 < NBLK; ++k2) sprev[k2] = 1.f;

    int step = 0;   // layer steps done
    // The 2*WK partials of a row (two half-waves, WK waves) are merged one step late, so that
    // the merge costs no barrier of its own: at the end of a step every lane posts its record
    // in LDS; after the next chunk barrier the first wave of each wave row brings the partials
    // of its rows onto their common exponent, adds them in a fixed order and stores the row
    // records (after every tile: the stored record is also the running record the next tile starts from).  The cross term of partial p carries the exponents of two layers: gprev[p] is
    // the factor that took p's exponent of the previous layer onto that layer's merged one.
    float gprev[2 * WK];
#pragma unroll
    for (int pi = 0; pi < 2 * WK; ++pi) gprev[pi] = 1.f;
    int mg_l = 0;
    bool mg_on = false;   // a merge is pending (uniform over the workgroup)
    auto merge_rows = [&]() __attribute__((always_inline)) {
        float4 pp[2 * WK];
#pragma unroll
        for (int pi = 0; pi < 2 * WK; ++pi) pp[pi] = part[wr * WK + (pi >> 1)][(pi & 1) * 32 + l32];
        float M = pp[0].x;
#pragma unroll
        for (int pi = 1; pi < 2 * WK; ++pi) M = fmaxf(M, pp[pi].x);
        float zs = 0.f, ns = 0.f, cc = 0.f, zir = 0.f;
#pragma unroll
        for (int pi = 0; pi < 2 * WK; ++pi) {
            const float f = __builtin_amdgcn_exp2f(pp[pi].x - M);
            if (IR) zir = fmaf(part_ir[wr * WK + (pi >> 1)][(pi & 1) * 32 + l32], f, zir);
            zs = fmaf(pp[pi].y, f, zs);
            ns = fmaf(pp[pi].z, f * f, ns);
            cc = fmaf(pp[pi].w, f * gprev[pi], cc);
            gprev[pi] = f;
        }
        // lanes l and l+32 hold, and store, the same record
        p.state[((size_t)wg * L + mg_l) * C::R_WG + wr * 32 + l32] = make_float4(M, zs, ns, cc);
        if (IR) p.state_ir[((size_t)wg * L + mg_l) * C::R_WG + wr * 32 + l32] = zir;
    };
    // running record of the coming step (its previous tile's), fetched one step ahead
    float4 rec_pre = make_float4(kMInit, 0.f, 0.f, 0.f);
    float rec_ir_pre = 0.f;
    for (int tile = 0; tile < ntiles; ++tile) {
        const int tile_key0 = key_begin + tile * C::KT;
        // keys of this tile to be masked out: past the end of the split, or (causal reading) past
        // the own position of some row of this wave
        const bool ragged = tile_key0 + C::KT > key_end || (p.causal && __any(tile_key0 + C::KT > row_end));

        for (int l = 0; l < L; ++l, ++step) {
            const float4 rec = rec_pre;
            const float rec_ir = rec_ir_pre;
            float tzir = 0.f;
            // the step after this one: its layer and tile, and where its keys and query rows are
            const bool has_next = step + 1 < nsteps;
            const int ln = l + 1 == L ? 0 : l + 1;
            const int tn_ = l + 1 == L ? tile + 1 : tile;
            fetch_key0 = key_begin + tn_ * C::KT;
            if (l + 1 == L) {
                k_tile_off += k_tile_step;
                k_dense = Kg;
                if (has_next) load_pages(fetch_key0);
            } else {
                k_dense += p.k_stride_l;
            }
            fetch_k = uniform_ptr(k_layer(ln) + k_tile_off);
            fetch_q = qbase + (size_t)ln * q_layer_stride;
            float mcur = rec.x, tz = 0.f, tn = 0.f;
            float mb[NBLK], dot[NBLK];   // per block: exponent used, dot with previous layer
            bool raised = false;         // some lane raised m during this step (wave-uniform)
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                // The chunk after this one (copied PF chunks ago) and, before the last chunk of a
                // step, the next layer's query rows must have landed; past the barrier every wave
                // has finished reading this chunk from its slot, which is then refilled.  Loads
                // return in order: it is enough that no more are outstanding than were issued
                // after the ones needed -- the copies of the PF-1 chunks issued since, and, in
                // the chunks between a step's first and last, the copies of the query rows
                // (issued during the first, needed at the last).  Record stores in flight only
                // make this wait a little longer than needed.
                if (c != 0 && c != NC - 1)
                    __builtin_amdgcn_s_waitcnt(wait_vm_lgkm0((PF - 1) * NLD + C::QPW));
                else
                    __builtin_amdgcn_s_waitcnt(wait_vm_lgkm0((PF - 1) * NLD));
                __builtin_amdgcn_s_barrier();
                if (c == 0 && mg_on) {
                    if (wk == 0) merge_rows();
                    mg_on = false;
                }
                if (c == 0) {
                    // The next step's running record was stored L-2 steps ago or earlier (by this lane, in
                    // merge_rows).
                    rec_pre = make_float4(kMInit, 0.f, 0.f, 0.f);
                    rec_ir_pre = 0.f;
                    if (tn_ > 0 && has_next && carries) {
                        if (L < 5) __builtin_amdgcn_s_waitcnt(wait_vm(0));   // (then it may still be on its way)
                        rec_pre = p.state[row_rec + (size_t)ln * C::R_WG];
                        if (IR) rec_ir_pre = p.state_ir[row_rec + (size_t)ln * C::R_WG];
                    }
                }
                if (c == NC - 1) read_q();   // every wave has the old rows in use no more
                const unsigned char *nslot = slot_ptr((c + 1) % NC);

                if (ragged) {
                    // keys at or past key_end: element v of a lane is key kb0 + 8*(v/4) + v%4
#pragma unroll
                    for (int kb = 0; kb < KBW; ++kb) {
                        int lim = min(key_end, row_end) - (tile_key0 + c * C::CH + (wk * KBW + kb) * 32 + half * 4);
                        asm volatile("" : "+v"(lim));   // keep the 16 compares here, not hoisted
#pragma unroll
                        for (int v = 0; v < 16; ++v)
                            if (8 * (v >> 2) + (v & 3) >= lim) acc[c & 1][kb][v] = -INFINITY;
                    }
                }
#pragma unroll
                for (int kb = 0; kb < KBW; ++kb) {
                    const int blk = c * KBW + kb;
                    f32x16 &x = acc[c & 1][kb];
                    if (blk == 0) {
                        // first block of a step: bring the reference exponent (which starts from
                        // "no key seen", or from the previous tile's) up to this block's maximum
                        // before use; no sums of this step exist yet that would need rescaling
                        float tmax = x[0];
#pragma unroll
                        for (int v = 1; v < 16; ++v) tmax = fmaxf(tmax, x[v]);
                        mcur = fmaxf(mcur, tmax * cs);
                    }
                    // The next chunk's logits of this block are formed while this block's
                    // exponentials are taken: independent work for the matrix and vector units.
                    // All operands are read up front, so that no MFMA waits for LDS; the copies of
                    // this iteration are issued here as well: the next step's chunk c into the slot
                    // this chunk was read from, the next step's query rows.
                    bf16x8 aop[KS];
                    {
                        const unsigned char *kbp = nslot + kb * 32 * (D * 2);
#pragma unroll
                        for (int ks = 0; ks < KS; ++ks)
                            aop[ks] = *reinterpret_cast<const bf16x8 *>(kbp + (ka_base ^ (ks << 5)));
                    }
                    if (kb == 0) issue_chunk(c, has_next);
                    if (c == 0 && kb == KBW - 1) issue_q(has_next);
                    // Exponentials under the current reference exponent; if one of them turns out
                    // large (above 2^kLazy, or overflowed) the exponent is raised to the block's
                    // maximum, the running sums are rescaled, and the block is taken again.
                    // One MFMA, then the vector work of 16/KS logits, and so on: the empty asm
                    // statements keep that order (the compiler would issue the MFMAs back to back,
                    // each waiting for the one before, and the vector work after them).
                    f32x16 nx;
#pragma unroll
                    for (int v = 0; v < 16; ++v) nx[v] = 0.f;
                    float ev[16];
                    float bz = 0.f, bn = 0.f, bd = 0.f;
                    {
                        const float negm = -mcur;
                        constexpr int VPK = 16 / KS;
#pragma unroll
                        for (int ks = 0; ks < KS; ++ks) {
                            nx = mfma_16bit<F16>(aop[ks], qf[ks], nx);
                            asm volatile("" : "+v"(nx));
#pragma unroll
                            for (int v = ks * VPK; v < (ks + 1) * VPK; ++v) {
                                ev[v] = __builtin_amdgcn_exp2f(fmaf(x[v], cs, negm));
                                if (WZ) bz += ev[v];
                                bn = fmaf(ev[v], ev[v], bn);
                                bd = fmaf(ev[v], e[blk][v], bd);
                            }
                            if (ks + 1 < KS) asm volatile("" : "+v"(bz), "+v"(bn), "+v"(bd));
                        }
                    }
                    acc[(c + 1) & 1][kb] = nx;
                    asm volatile("" : "+v"(bz), "+v"(bn), "+v"(bd));   // the sums are taken here, beside the MFMAs
                    if (__any(!(bn <= kBig))) {
                        float tmax = x[0];
#pragma unroll
                        for (int v = 1; v < 16; ++v) tmax = fmaxf(tmax, x[v]);
                        const float mnew = fmaxf(mcur, tmax * cs);
                        const float f = __builtin_amdgcn_exp2f(mcur - mnew);
                        tz *= f;
                        tzir *= f;
                        tn *= f * f;
                        mcur = mnew;
                        raised = true;
                        const float negm = -mcur;
                        bz = bn = bd = 0.f;
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            ev[v] = __builtin_amdgcn_exp2f(fmaf(x[v], cs, negm));
                            if (WZ) bz += ev[v];
                            bn = fmaf(ev[v], ev[v], bn);
                            bd = fmaf(ev[v], e[blk][v], bd);
                        }
                    }
                    mb[blk] = mcur;
#pragma unroll
                    for (int v = 0; v < 16; ++v) e[blk][v] = ev[v];
                    tz += bz;
                    if (IR) {
                        // keys of this block inside T_initial or T_recent: all, none, or some
                        const int kb0 = tile_key0 + c * C::CH + (wk * KBW + kb) * 32;
                        if (kb0 + 32 <= p.ir_init_end || kb0 >= p.ir_recent_begin) {
                            tzir += bz;
                        } else if (!(kb0 >= p.ir_init_end && kb0 + 32 <= p.ir_recent_begin)) {
                            float bir = 0.f;   // element v of this lane is key kb0 + 8*(v/4) + 4*half + v%4
#pragma unroll
                            for (int v = 0; v < 16; ++v) {
                                const int key = kb0 + 8 * (v >> 2) + 4 * half + (v & 3);
                                if (key < p.ir_init_end || key >= p.ir_recent_begin) bir += ev[v];
                            }
                            tzir += bir;
                        }
                    }
                    tn += bn;
                    dot[blk] = bd;
                }
            }

            // ---- cross term of this tile: block dots, each brought to the final exponents of
            // both layers (the factors are 1 unless some m was raised in this or the last step)
            float tc = 0.f;
            if (raised || raised_prev) {
#pragma unroll
                for (int k2 = 0; k2 < NBLK; ++k2) {
                    const float sc = __builtin_amdgcn_exp2f(mb[k2] - mcur);
                    tc = fmaf(dot[k2], sc * sprev[k2], tc);
                    sprev[k2] = sc;
                }
            } else {
#pragma unroll
                for (int k2 = 0; k2 < NBLK; ++k2) tc += dot[k2];
            }
            raised_prev = raised;

            // ---- fold this tile's sums into the running record of layer l
            float4 out;
            float out_ir = 0.f;
            {
                const float F = __builtin_amdgcn_exp2f(rec.x - mcur);
                if (IR) out_ir = fmaf(rec_ir, F, tzir);
                out.x = mcur;
                out.y = fmaf(rec.y, F, tz);
                out.z = fmaf(rec.z, F * F, tn);
                out.w = fmaf(rec.w, F * f_prev, tc);
                f_prev = F;
            }
            // ---- post this lane's record; the merge follows during the next step
            part[wave][lane] = out;
            if (IR) part_ir[wave][lane] = out_ir;
            mg_l = l;
            mg_on = true;
        }
    }
    // the last step's merge
    if (mg_on) {
        __builtin_amdgcn_s_waitcnt(kWaitLgkm0);
        __builtin_amdgcn_s_barrier();
        if (wk == 0) merge_rows();
    }
}

template <class C, int KA, bool F16>
hipError_t launch_mode(const SimParams &p, int n_workgroups, hipStream_t st)
{
    const dim3 grid(n_workgroups), block(C::THREADS);
    if (p.want_ir)
        hipLaunchKernelGGL((sim_mfma_kernel<C, 2, KA, F16>), grid, block, 0, st, p);
    else if (p.want_dist)
        hipLaunchKernelGGL((sim_mfma_kernel<C, 1, KA, F16>), grid, block, 0, st, p);
    else
        hipLaunchKernelGGL((sim_mfma_kernel<C, 0, KA, F16>), grid, block, 0, st, p);
    return hipGetLastError();
}

template <class C, bool F16>
hipError_t launch_cfg_t(const SimParams &p, int n_workgroups, hipStream_t st)
{
    if (p.block_table) return launch_mode<C, 2, F16>(p, n_workgroups, st);   // keys in pages
    // keys in per-layer allocations, with strides -- or dense, with a head size below the kernel's
    if (p.k_tab || p.d != C::D) return launch_mode<C, 1, F16>(p, n_workgroups, st);
    return launch_mode<C, 0, F16>(p, n_workgroups, st);
}

template <class C>
hipError_t launch_cfg(const SimParams &p, int n_workgroups, hipStream_t st)
{
    return p.f16 ? launch_cfg_t<C, true>(p, n_workgroups, st) : launch_cfg_t<C, false>(p, n_workgroups, st);
}

}  // namespace
}  // namespace krul
