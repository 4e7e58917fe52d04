// The many-query form of the 16-bit matrix-core similarity kernel: 256 query rows x 256 keys per workgroup
// tile, head_dim 128, dense keys, cosine (and optionally the distance's plain sum), no mask.
//
// Same method as sim_mfma_kernel (krul_mfma_kernel.h: layer-chained walk, logits of 32 keys x 32 rows per MFMA
// chain with a query row per lane, lazy reference exponent, row records merged one step late), with three
// changes that the many-query problems pay for:
//
//  * Every wave owns TWO 32-row blocks of query rows (64 rows, both in registers).  A block of keys read from
//    LDS feeds two MFMA chains, so a logit costs half the operand reads, and while the vector units take the
//    exponentials of one row block's logits the matrix cores form the other's: the two accumulators are each
//    other's double buffer.
//  * The previous layer's exponentials, kept for the cross term (the "ab" of Sec. 7's a^2 + b^2 - 2ab), are
//    stored as IEEE binary16 pairs (e <= 2^15, round to nearest: 2^-11 relative, read back by v_fma_mix_f32
//    with no unpacking).  That halves their registers, which is what lets a workgroup hold 256 x 256 logits'
//    worth of them: per logit the workgroup then fetches 2 bytes of keys and query rows instead of 3.
//    The sums of squares and the running sums use the unrounded fp32 values; only the cross term sees the
//    rounding, and it moves a cosine by at most 2^-11 of itself.
//  * All blocks of a layer step are kept on ONE exponent, and the check comes BEFORE the exponentials: a block's
//    exponents a = x*c - m are formed first (in place, in the accumulator registers) and their maximum taken; if
//    it is above 15 the lane's reference exponent is raised to it and the step's sums and the blocks already
//    stored are rescaled on the spot (rare; exact: powers of two).  So no exponential can overflow, no block is
//    ever taken twice, no per-block exponents are carried, and the exponentials can replace the previous layer's
//    in their registers as they are formed.
//
// Streams, ring slots, count-based waits, the XOR swizzle and the patch numbering of workgroups are those of
// sim_mfma_kernel.  A layer step is four chunks of 64 keys; per chunk a wave runs two phases, (c, 0) and
// (c, 1): in phase (c, r) the MFMA chain of row block r on chunk c runs beside the vector work of the unit
// before it -- (c-1, 1) for r = 0, (c, 0) for r = 1.  The key operands of chunk c+1 replace those of chunk c
// register by register during phase (c, 1), as the last chain that needs them passes.  The loop body is
// "barrier, phase (c, 1), phase (c+1, 0)"; the first phase (0, 0) is the prologue.
#include "krul_mfma_kernel.h"

namespace krul {
namespace {

typedef _Float16 h16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr float kLazyMax = 15.0f;   // exponentials stay below 2^15: inside binary16 range, their squares far inside fp32's

// MODE 0: cosine only; 1: also Z = sum e (the distance needs it)
template <int MODE, bool F16>
__global__ __launch_bounds__(512, 2) void sim_big_kernel(SimParams p)
{
    constexpr int D = 128, NC = 4, CH = 64, KT = NC * CH, KS = 8, NLD = 2, RPI = 4, PPR = 16;
    constexpr int R_WG = 256, SLOT_BYTES = CH * D * 2, QWR_BYTES = 64 * D * 2;
    constexpr bool WZ = MODE >= 1;
    __shared__ __attribute__((aligned(16384))) unsigned char ring0[SLOT_BYTES];
    __shared__ __attribute__((aligned(16384))) unsigned char ring1[SLOT_BYTES];
    __shared__ __attribute__((aligned(16384))) unsigned char ring2[SLOT_BYTES];
    __shared__ __attribute__((aligned(16384))) unsigned char ring3[SLOT_BYTES];
    __shared__ __attribute__((aligned(1024))) unsigned char qlds[4 * QWR_BYTES];
    __shared__ float4 part[8][2][64];   // every lane's record of the last step, per row block
    __shared__ __attribute__((aligned(1024))) float4 runl[8][64];   // per wave: the running records (all tiles before this one) of the 32 rows it merges
    __shared__ float gl[8][5][32];      // per wave and partial: last step's merge factors
    auto slot_ptr = [&](int i) __attribute__((always_inline)) -> unsigned char * {
        switch (i & 3) {
        case 0: return ring0;
        case 1: return ring1;
        case 2: return ring2;
        default: return ring3;
        }
    };

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wr = wave >> 1, wk = wave & 1, half = lane >> 5, l32 = lane & 31;

    const int nrt = p.lay.n_row_tiles, nsplit = p.lay.n_split;
    int rt, sp, u;
    {
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
    const int wg = (u * nsplit + sp) * nrt + rt;
    const int b = u / p.Hkv, kvh = u % p.Hkv;
    const int L = p.L, S = p.S, Rk = p.lay.rows_per_unit;
    const int key_begin = sp * p.keys_per_split;
    const int key_end = min(S, key_begin + p.keys_per_split);
    const int ntiles = (key_end - key_begin + KT - 1) / KT;
    const int nsteps = ntiles * L;

    const uint16_t *Qg = static_cast<const uint16_t *>(p.q);
    const uint16_t *Kg = static_cast<const uint16_t *>(p.k);
    const size_t q_layer_stride = (size_t)p.Hq * p.Tq * D;
    const uint16_t *k_unit = Kg + (size_t)b * p.k_stride_b + (size_t)kvh * p.k_stride_h + (size_t)key_begin * D;
    constexpr unsigned k_row_bytes = D * 2, k_chunk_bytes = CH * D * 2;

    auto xj = [](int j) -> unsigned { return (unsigned)(((j * RPI) & 15) * 16); };
    // ---- key chunks: wave-instruction j of this wave fills granules [(wave*NLD+j)*64, +64) of a slot
    const int ld_row0 = wave * NLD * RPI + lane / PPR;
    const unsigned ld_off0 = (unsigned)ld_row0 * k_row_bytes + (unsigned)(((lane % PPR) ^ swz<D>(ld_row0)) * 16);
    const uint16_t *fetch_k = uniform_ptr(k_unit);   // the next step's layer and tile
    int fetch_key0 = key_begin;
    // (one copy instruction at a time: the copies of a step are spread over its phases, a few MFMAs apart, so that
    // the CU's queue of memory requests never holds a burst -- a wave whose copy finds the queue full stands
    // still until there is room, with its matrix and vector work)
    auto issue_chunk = [&](int c, int j, bool live) __attribute__((always_inline)) {
        unsigned char *dst = slot_ptr(c);
        const int key0 = fetch_key0 + c * CH;
        const unsigned bytes = live && key0 < S ? (unsigned)(S - key0) * k_row_bytes : 0u;
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint16_t *>(fetch_k + (c * k_chunk_bytes) / 2), 0, (int)bytes, 0x00020000);
        unsigned off = ld_off0;
        asm volatile("" : "+v"(off));   // (the per-instruction offsets are formed here, not kept over the loop)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            rsrc, (__attribute__((address_space(3))) void *)(dst + (wave * NLD + j) * 1024), 16,
            (int)(off ^ xj(j)), (int)(j * RPI * k_row_bytes), 0, 0);
    };
    // ---- query rows: the 64 rows of wave row wr, staged as two 32-row blocks laid out like key blocks, copied
    // by the two waves that share them (eight wave-instructions each)
    const int r0 = rt * R_WG + wr * 64;
    const int q_rows = min(max(Rk - r0, 0), 64);
    const uint16_t *qbase = uniform_ptr(Qg + ((size_t)b * L * p.Hq * p.Tq + (size_t)kvh * Rk + (size_t)(q_rows ? r0 : 0)) * D);
    const unsigned q_off0 = (unsigned)((lane / PPR) * (D * 2) + (((lane % PPR) ^ swz<D>(lane / PPR)) * 16));
    const uint16_t *fetch_q = qbase;
    auto issue_q = [&](int jj, bool live) __attribute__((always_inline)) {   // jj: which of this wave's eight
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint16_t *>(fetch_q), 0, __builtin_amdgcn_readfirstlane(live ? q_rows * (D * 2) : 0), 0x00020000);
        unsigned char *dst = qlds + wr * QWR_BYTES;
        unsigned off = q_off0;
        asm volatile("" : "+v"(off));
        const int j = wk * 8 + jj;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            rsrc, (__attribute__((address_space(3))) void *)(dst + j * 1024), 16, (int)(off ^ xj(j)), j * 1024, 0, 0);
    };

    const int a_base = l32 * (D * 2) + ((half ^ swz<D>(l32)) << 4);
    const int ka_base = a_base + wk * 32 * (D * 2);   // this wave's 32 keys of a chunk
    // LDS offsets of this lane's eight operand pieces inside a chunk (the XOR swizzle makes them per-lane values);
    // a slot's place goes into the instruction's offset field.  The query rows are read at the same offsets plus
    // a wave-uniform distance that is added at the read (kept out of registers: see q_delta()).
    auto kaddr_of = [&](int ks) __attribute__((always_inline)) -> int {
        int flip = ks << 5;
        asm volatile("" : "+s"(flip));   // (opaque: the offset is formed at the read, by one XOR, not kept over the loop)
        return ka_base ^ flip;
    };
    bf16x8 qf[2][KS], aop[KS];
    auto read_q = [&](int rb) __attribute__((always_inline)) {
        // (opaque to the compiler, so that the eight sums are formed here and not kept in registers over the loop)
        int delta = (wr * QWR_BYTES + rb * (32 * D * 2)) - wk * 32 * (D * 2);
        asm volatile("" : "+s"(delta));
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[rb][ks] = *reinterpret_cast<const bf16x8 *>(qlds + (kaddr_of(ks) + delta));
    };

    // the previous layer's exponentials of this tile, per row block and chunk, as binary16 pairs
    h16x2 e2[2][NC][8];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int c = 0; c < NC; ++c)
#pragma unroll
            for (int i = 0; i < 8; ++i) e2[rb][c][i] = h16x2{(_Float16)0.f, (_Float16)0.f};

    // per row block: this step's reference exponent and sums (of this tile only: a row's running record over the
    // tiles before joins in the merge, as one more partial)
    float mcur[2], tz[2], tn[2], td[2];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
        mcur[rb] = kMInit;
        tz[rb] = tn[rb] = td[rb] = 0.f;
    }
    const float cs = p.c;

    // ---- merge of a row's partials, one step late: the tile's four (two half-waves, two waves along the keys) and,
    // from the second tile on, the row's running record over the tiles before (copied into runl a step ahead).
    // The result is stored as the row record: the final one after the last tile, the running one before.  The
    // two waves of a wave row share the work: wave (wr, wk) merges row block wk.  gl: factors that took each
    // partial's exponent of the previous layer onto that layer's merged one (the cross term carries two layers'
    // exponents); kept in LDS -- registers are what this kernel is short of.
    if (half == 0)
#pragma unroll
        for (int i = 0; i < 5; ++i) gl[wave][i][l32] = 1.f;
    const size_t my_rec = (size_t)wg * L * R_WG + wr * 64 + wk * 32;   // + l * R_WG: first of the 32 rows this wave merges
    auto merge_rows = [&](int l_of, bool with_run) __attribute__((always_inline)) {
        if (half == 0) {   // (one lane per row)
            const float4 *pr[5];
#pragma unroll
            for (int pi = 0; pi < 4; ++pi) pr[pi] = &part[wr * 2 + (pi >> 1)][wk][(pi & 1) * 32 + l32];
            pr[4] = &runl[wave][l32];
            float M = pr[0]->x;
#pragma unroll
            for (int pi = 1; pi < 4; ++pi) M = fmaxf(M, pr[pi]->x);
            if (with_run) M = fmaxf(M, pr[4]->x);
            float zs = 0.f, ns = 0.f, cc = 0.f;
#pragma unroll
            for (int pi = 0; pi < 5; ++pi) {
                if (pi == 4 && !with_run) {
                    gl[wave][pi][l32] = 0.f;
                    break;
                }
                const float4 v = *pr[pi];
                const float f = __builtin_amdgcn_exp2f(v.x - M);
                zs = fmaf(v.y, f, zs);
                ns = fmaf(v.z, f * f, ns);
                cc = fmaf(v.w, f * gl[wave][pi][l32], cc);
                gl[wave][pi][l32] = f;
            }
            p.state[my_rec + l32 + (size_t)l_of * R_WG] = make_float4(M, zs, ns, cc);
        }
    };
    // the running records of layer l_of of the 32 rows this wave merges (512 bytes) -> runl[wave], by one copy
    // instruction; read past the L1 (this wave stored them a tile ago)
    auto fetch_run = [&](int l_of, bool live) __attribute__((always_inline)) {
        const uint16_t *src = uniform_ptr(reinterpret_cast<const uint16_t *>(p.state + my_rec + (size_t)l_of * R_WG));
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(src), 0, live ? 512 : 0, 0x00020000);
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (__attribute__((address_space(3))) void *)(&runl[wave][0]), 16,
                                                 lane * 16, 0, 0, 1 /* glc */);
    };
    // ---- the end of a layer step for row block rb: post this lane's sums over the tile
    auto end_step = [&](int rb) __attribute__((always_inline)) {
        part[wave][rb][lane] = make_float4(mcur[rb], tz[rb], tn[rb], td[rb]);
        mcur[rb] = kMInit;
        tz[rb] = tn[rb] = td[rb] = 0.f;
    };

    f32x16 acc[2];
    // ---- the vector work of one unit: chunk c of row block rb, logits in acc[rb], turned in place into exponents
    // a = x*c - m and then into exponentials.  The exponent's reference m is only raised when it has to be: if
    // some a of the block exceeds kLazyMax (checked before any exponential is taken, so nothing can overflow, not
    // even the binary16 copies), the lane's m goes up to the block's maximum and the step's sums and the blocks
    // already stored follow (exact: powers of two).  unit_pair is called between the MFMAs of the chain that runs
    // beside the unit, two logits per call.
    float bz, bn, bd;
    auto unit_begin = [&](int c, int rb, bool ragged, int lim) __attribute__((always_inline)) {
        f32x16 &x = acc[rb];
        if (ragged) {   // (a tile with keys at or past the end of the split) element v of a lane is key 8*(v/4) + v%4 (+ 4*half, in lim)
            asm volatile("" : "+v"(lim));   // keep the compares here
#pragma unroll
            for (int v = 0; v < 16; ++v)
                if (8 * (v >> 2) + (v & 3) >= lim) x[v] = -INFINITY;
        }
        if (c == 0) {
            // first block of a step: no sums yet, and m may still be "no key seen": take the block's maximum
            float tmax = x[0];
#pragma unroll
            for (int v = 1; v < 16; ++v) tmax = fmaxf(tmax, x[v]);
            mcur[rb] = fmaxf(mcur[rb], tmax * cs);
            const float negm = -mcur[rb];
#pragma unroll
            for (int v = 0; v < 16; ++v) x[v] = fmaf(x[v], cs, negm);
        } else {
            const float negm = -mcur[rb];
#pragma unroll
            for (int v = 0; v < 16; ++v) x[v] = fmaf(x[v], cs, negm);
            float amax = x[0];
#pragma unroll
            for (int v = 1; v < 16; ++v) amax = fmaxf(amax, x[v]);
            if (__any(amax > kLazyMax)) {
                const float up = amax > kLazyMax ? amax : 0.f;   // this lane's m goes up by `up`
                const float f = __builtin_amdgcn_exp2f(-up);
#pragma unroll
                for (int v = 0; v < 16; ++v) x[v] -= up;
                mcur[rb] += up;
                tz[rb] *= f;
                tn[rb] *= f * f;
                td[rb] *= f;
                const h16x2 fh = h16x2{(_Float16)f, (_Float16)f};
#pragma unroll
                for (int cc = 0; cc < NC; ++cc)
                    if (cc < c) {
#pragma unroll
                        for (int i = 0; i < 8; ++i) e2[rb][cc][i] *= fh;
                    }
            }
        }
        bz = bn = bd = 0.f;
    };
    auto unit_pair = [&](int c, int rb, int ks) __attribute__((always_inline)) {
        f32x16 &x = acc[rb];
        const float ea = __builtin_amdgcn_exp2f(x[2 * ks]);
        const float eb = __builtin_amdgcn_exp2f(x[2 * ks + 1]);
        if (WZ) bz += ea + eb;
        bn = fmaf(ea, ea, bn);
        bn = fmaf(eb, eb, bn);
        bd = fmaf(ea, (float)e2[rb][c][ks].x, bd);
        bd = fmaf(eb, (float)e2[rb][c][ks].y, bd);
        e2[rb][c][ks] = __builtin_convertvector((f32x2{ea, eb}), h16x2);
    };
    auto unit_end = [&](int c, int rb) __attribute__((always_inline)) {
        tz[rb] += bz;
        tn[rb] += bn;
        td[rb] += bd;
    };

    // ---- prologue: query rows of layer 0, the four chunks of the first step; operands of chunk 0; the logits
    // of the first unit
#pragma unroll
    for (int jj = 0; jj < 8; ++jj) issue_q(jj, true);
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        issue_chunk(c, 0, true);
        issue_chunk(c, 1, true);
    }
    __builtin_amdgcn_s_waitcnt(wait_vm((NC - 1) * NLD));   // query rows and chunk 0 have landed
    __builtin_amdgcn_s_barrier();
    read_q(0);
    read_q(1);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) aop[ks] = *reinterpret_cast<const bf16x8 *>(ring0 + kaddr_of(ks));
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[0][v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) acc[0] = mfma_16bit<F16>(aop[ks], qf[0][ks], acc[0]);

    int l = 0, tile = 0;
    for (int step = 0; step < nsteps; ++step) {
        const bool has_next = step + 1 < nsteps;
        const int ln = l + 1 == L ? 0 : l + 1;
        const int tn_ = l + 1 == L ? tile + 1 : tile;
        const int tile_key0 = key_begin + tile * KT;
        const bool ragged = tile_key0 + KT > key_end;
        // where the next step's keys and query rows are
        fetch_key0 = key_begin + tn_ * KT;
        fetch_k = uniform_ptr(k_unit + (size_t)ln * p.k_stride_l + (size_t)tn_ * KT * D);
        fetch_q = qbase + (size_t)ln * q_layer_stride;

#pragma unroll
        for (int c = 0; c < NC; ++c) {
            // ---- Chunk c+1 of this step (for c = 3: chunk 0 of the next step, and the next layer's query rows) must
            // have landed, for every wave.  Loads return in order, so it is enough that no more are outstanding
            // than were issued after the ones needed.  A wave's copies over a step, in issue order (K: a key chunk
            // of the next step, two instructions a and b; Q: one of eight instructions for the next layer's query
            // rows; R: the record store and copy of the merge):
            //   (0,1) R R K0a Q K0b Q   (1,0) Q Q   (1,1) K1a Q K1b Q   (2,0) Q Q   (2,1) K2a K2b   (3,1) K3a K3b
            // After the chunk needed at c = 0 (K1b of the step before) came 7; at c = 1 (K2b) 8 or more; at c = 2
            // (K3b) 12 or more; at c = 3 (K0b and the last Q) 2.  In the first step the chunks come from the
            // prologue, back to back: 4 after K1b.
            if (c == 0) {
                if (step == 0) __builtin_amdgcn_s_waitcnt(wait_vm_lgkm0(4));
                else __builtin_amdgcn_s_waitcnt(wait_vm_lgkm0(7));
            } else if (c == 1) {
                __builtin_amdgcn_s_waitcnt(wait_vm_lgkm0(8));
            } else if (c == 2) {
                __builtin_amdgcn_s_waitcnt(wait_vm_lgkm0(12));
            } else {
                __builtin_amdgcn_s_waitcnt(wait_vm_lgkm0(2));
            }
            __builtin_amdgcn_s_barrier();
            // ======== phase (c, 1): logits of row block 1 on chunk c beside the exponentials of (c, 0); the
            // operands of the next chunk replace this chunk's as the chain passes
            {
                if (c == 0) {
                    // The step before is complete in LDS: merge it, with its layer's running record if its tile
                    // was not the first.  Then copy in the running record this step's merge will need (stored
                    // L-1 steps ago or earlier by this wave; the reads of runl above have returned: the merge
                    // used them).
                    if (step > 0) merge_rows(l == 0 ? L - 1 : l - 1, (l == 0 ? tile - 1 : tile) > 0);
                    if (L < 5) __builtin_amdgcn_s_waitcnt(wait_vm(0));
                    __builtin_amdgcn_s_waitcnt(kWaitLgkm0);
                    fetch_run(l, tile > 0);
                }
                // the next step's chunk c goes into the slot whose operands every wave holds by now; its query rows
                // into the staging area every wave has read (see the issue order above)
                issue_chunk(c, 0, has_next);
                issue_chunk(c, 1, has_next);
                if (c <= 1) {
                    issue_q(c * 4, has_next);
                    issue_q(c * 4 + 1, has_next);
                }
                if (c == NC - 1) read_q(0);        // the next step's rows of block 0 (the last chain on the old ones has been issued)
                unit_begin(c, 0, ragged, key_end - (tile_key0 + c * CH + wk * 32 + half * 4));
                const unsigned char *nslot = slot_ptr(c + 1);
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[1][v] = 0.f;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    acc[1] = mfma_16bit<F16>(aop[ks], qf[1][ks], acc[1]);
                    asm volatile("" : "+v"(acc[1]));
                    aop[ks] = *reinterpret_cast<const bf16x8 *>(nslot + kaddr_of(ks));
                    unit_pair(c, 0, ks);
                    asm volatile("" : "+v"(bn), "+v"(bd));
                }
                unit_end(c, 0);
                if (c == NC - 1) end_step(0);
            }
            // ======== phase (c+1, 0) -- for c = 3: (0, 0) of the next step --: logits of row block 0 on the next chunk
            // beside the exponentials of (c, 1).  (After the last step the chain runs on stale operands; nothing
            // reads its result.)
            {
                if (c == NC - 1) read_q(1);        // the next step's rows of block 1
                if (c <= 1) {
                    issue_q(c * 4 + 2, has_next);
                    issue_q(c * 4 + 3, has_next);
                }
                unit_begin(c, 1, ragged, key_end - (tile_key0 + c * CH + wk * 32 + half * 4));
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[0][v] = 0.f;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    acc[0] = mfma_16bit<F16>(aop[ks], qf[0][ks], acc[0]);
                    asm volatile("" : "+v"(acc[0]));
                    unit_pair(c, 1, ks);
                    asm volatile("" : "+v"(bn), "+v"(bd));
                }
                unit_end(c, 1);
                if (c == NC - 1) end_step(1);
            }
        }
        l = ln;
        tile = tn_;
    }
    // ---- the last step's merge
    __builtin_amdgcn_s_waitcnt(wait_vm_lgkm0(0));
    __builtin_amdgcn_s_barrier();
    merge_rows(L - 1, ntiles > 1);
}

}  // namespace

hipError_t launch_sim_mfma_big(const SimParams &p, int n_workgroups, hipStream_t st)
{
    const dim3 grid(n_workgroups), block(512);
    if (p.want_dist) {
        if (p.f16) hipLaunchKernelGGL((sim_big_kernel<1, true>), grid, block, 0, st, p);
        else hipLaunchKernelGGL((sim_big_kernel<1, false>), grid, block, 0, st, p);
    } else {
        if (p.f16) hipLaunchKernelGGL((sim_big_kernel<0, true>), grid, block, 0, st, p);
        else hipLaunchKernelGGL((sim_big_kernel<0, false>), grid, block, 0, st, p);
    }
    return hipGetLastError();
}

}  // namespace krul
