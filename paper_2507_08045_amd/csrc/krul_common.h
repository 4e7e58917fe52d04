// Internal declarations shared by the translation units of libkrul (not installed).
//
// Data flow of krul_pair_similarity (Sec. 5 / Sec. 7 of the paper: similarity is
// accumulated token-wise, attention weights are never kept):
//   1. a similarity kernel walks the history keys tile by tile and, inside a tile,
//      the layers in order.  For each (row, layer) it maintains the online-softmax
//      statistics  m (reference exponent), Z = sum e, N2 = sum e^2  with
//      e = 2^(x - m), x = logit * scale * log2(e); for each adjacent pair it
//      maintains the cross term  C = sum e_l * e_{l+1}  (the "-2ab" term of the
//      a^2 + b^2 - 2ab expansion in Sec. 7).  A row's keys may be spread over several
//      independent "partials" (lanes, waves, key splits).  Partials inside a
//      workgroup are merged there; each key split writes one record per (row,
//      layer), float4 (m, Z, N2, C(l-1,l)), to the state area of the workspace.
//   2. the finalize kernel merges a row's partials (rescaling to the common
//      reference exponent), forms cos = C / sqrt(N2_l N2_{l+1}) and
//      dist^2 = N2_l/Z_l^2 + N2_{l+1}/Z_{l+1}^2 - 2C/(Z_l Z_{l+1}), and averages over
//      the query rows of a head in a fixed order;
//   3. the pair kernel averages over heads.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "krul.h"

namespace krul {

// Reference exponent of a partial that has seen no key yet: finite, so that
// differences of exponents never give inf - inf.
constexpr float kMInit = -1.0e30f;

enum Variant : int {
    kGeneric = 0,   // portable VALU kernel: one wave per (row, key split)
    kMfmaWide = 1,  // bf16 MFMA, 128 rows x 256 keys per workgroup tile (4x2 waves)
    kMfmaMid = 2,   // bf16 MFMA,  64 rows x 512 keys per workgroup tile (2x4 waves)
    kMfmaSlim = 3,  // bf16 MFMA,  32 rows x 512 keys per workgroup tile (1x8 waves)
    kMfmaSlimDeep = 4,   // bf16 MFMA,  32 rows x 512 keys (1x4 waves, three chunks of keys in flight)
    kMfmaSlimShort = 5,  // bf16 MFMA,  32 rows x 256 keys (1x4 waves, two workgroups per CU)
    kMfmaMidShort = 6,   // bf16 MFMA,  64 rows x 128 keys (2x2 waves)
    kMfmaWideShort = 7,  // bf16 MFMA, 128 rows x 128 keys (4x2 waves)
    kMfmaBig = 8,        // bf16 MFMA, 256 rows x 256 keys (4x2 waves, two 32-row blocks per wave): krul_mfma_big.hip
};

// How the state records of one launch are laid out; used by the producer kernels
// and by the finalize kernel.
struct StateLayout {
    int variant;
    int n_layers;
    int rows_per_unit;   // Rk = (Hq/Hkv) * Tq rows share one kv head
    int n_split;         // key splits (workgroups along the keys)
    int n_row_tiles;     // workgroups along the rows of a unit (MFMA variants)
    int wr, wk, rb;      // wave grid and 32-row blocks per wave (MFMA variants)
    int partials;        // records per (row, layer)
};

struct Plan {
    StateLayout lay;
    int keys_per_split;  // multiple of the key tile for MFMA variants
    int n_workgroups;
    float c;             // scale * log2(e)
    size_t state_bytes;  // merged partial records (float4), read by the finalize kernel
    size_t head_cos_off, head_dist_off, total_bytes;
    // Initial-Recent layer test only: one float per record beside state, head means
    size_t state_ir_off, head_ir_off;
};

// Host: choose kernel and decomposition for a validated shape.  Returns a
// krul_status_t.
// plain_keys: the keys are dense and no mask or Initial-Recent test is asked for -- what the many-query kernel
// (kMfmaBig) takes; the plan (and so the workspace) may differ with it.
int make_plan(const krul_shape_t *s, Plan *plan, bool want_ir = false, bool plain_keys = false);

struct SimParams {
    const void *q;
    const void *k;
    float4 *state;   // partial records, indexed by state_index() (MFMA variants: also a split's running records
                     // between its key tiles)
    int B, L, Hq, Hkv, g, d, S, Tq;
    int keys_per_split;
    float c;
    int want_dist;   // the distance is asked for: Z = sum e must be accumulated too
    // Initial-Recent layer test (Sec. 4.2, Alg. 1 first loop): Zir = sum of e over the keys
    // [0, ir_init_end) and [ir_recent_begin, S), one float per record, laid out like state
    int want_ir;
    int causal;   // row t sees keys j <= S - Tq + t (KRUL_FLAG_CAUSAL)
    int f16;      // the 16-bit inputs are IEEE binary16, not bfloat16 (MFMA variants)
    // Where the keys are (elements of the storage type): layer l starts at k_tab[l] if k_tab is
    // set (a device array of device pointers), else at k + l * k_stride_l; inside a layer the key
    // (b, kv head, j) starts at b * k_stride_b + kvh * k_stride_h + j * k_stride_s, head_dim contiguous.
    const void *const *k_tab;
    long long k_stride_l, k_stride_b, k_stride_h, k_stride_s;
    // Paged keys (k_tab set as well: one pool of pages per layer): key j of conversation b is key
    // j % 2^page_shift of page block_table[b * max_blocks + (j >> page_shift)]; a page starts k_stride_page
    // elements after the one before, its keys are k_stride_s apart, kv heads k_stride_h.
    const int *block_table;
    int page_shift, max_blocks;
    long long k_stride_page;
    int ir_init_end, ir_recent_begin;
    float *state_ir;
    StateLayout lay;
};

// Head averages and the greedy choice in one kernel, a workgroup per conversation (krul_pair_similarity_select).
struct PairsSelectArgs {
    const float *head_cos, *head_dist;   // [B][L-1][Hq]; head_dist may be null
    float *pair_cos, *pair_dist;         // [B][L-1]; pair_dist may be null
    const uint8_t *eligible;             // [B][L] or null
    int B, L, Hq, n_select;
    int32_t *out_pairs, *out_count;
};
constexpr int kPairsSelectMaxHeads = 16384;   // (L-1) * Hq head values that one workgroup averages and ranks

// Host: shape checks common to all entry points.  Returns a krul_status_t.
int check_shape(const krul_shape_t *s);

// Where the keys are, in the kernels' terms (elements of the storage type): layer l starts at k_tab[l] if
// k_tab is set (a device array of device pointers), else at k + l * stride_l; inside a layer the key
// (b, kv head, j) starts at b * stride_b + kvh * stride_h + j * stride_s -- or, if block_table is set, at
// block_table[b * max_blocks + (j >> page_shift)] * stride_page + kvh * stride_h + (j & (2^page_shift - 1)) * stride_s.
struct KeyAddr {
    const void *k;
    const void *const *k_tab;
    long long stride_l, stride_b, stride_h, stride_s;
    const int *block_table;
    int page_shift, max_blocks;
    long long stride_page;
};
// Host: validate one source of keys (exactly one of k, kl, kp set) for a checked shape and put it in the
// kernels' terms.  mfma: the matrix-core kernels will read it (their row swizzle and 32-bit offsets add
// limits); dense_2gib: ... and address a layer's keys of one head with 32-bit offsets.  Returns a krul_status_t.
int resolve_keys(const krul_shape_t *s, bool mfma, bool dense_2gib, const void *k, const krul_k_layout_t *kl,
                 const krul_k_pages_t *kp, KeyAddr *out);

// Similarity of every two layers (krul_allpairs.hip).  all_pairs_workspace: bytes for the largest batch
// of rows that fits max_bytes (0: a default budget), 0 if the shape is not supported.  run_all_pairs
// validates, enqueues everything on st and returns a krul_status_t.
size_t all_pairs_workspace(const krul_shape_t *s, size_t max_bytes);
int run_all_pairs(const krul_shape_t *s, const void *q, const void *k, const krul_k_layout_t *kl,
                  const krul_k_pages_t *kp, float *pair_score, float *pair_dist, float *head_score,
                  void *workspace, size_t workspace_bytes, hipStream_t st);
hipError_t launch_select_all(const float *score, int closer_is_smaller, const uint8_t *eligible, int batch,
                             int n_layers, int n_select, int32_t *out_pairs, int32_t *out_count, hipStream_t st);

// Launchers (each returns hipError_t of the launch).
hipError_t launch_sim_generic(const SimParams &p, int dtype, int n_workgroups, hipStream_t st);
hipError_t launch_sim_mfma(const SimParams &p, int n_workgroups, hipStream_t st);
hipError_t launch_sim_mfma_big(const SimParams &p, int n_workgroups, hipStream_t st);
// accumulate: add the sums over rows to head_cos / head_dist (head_dist may then be null) and write no
// pair scores; otherwise write the means and the pair scores (pair_dist may be null: no distances;
// pair_cos may be null: head values only, head_dist filled iff pair_dist is set).
hipError_t launch_finalize(const StateLayout &lay, const float4 *state, int B, int L, int Hq, int Hkv,
                           int Tq, float *head_cos, float *head_dist, float *pair_cos,
                           float *pair_dist, bool accumulate, hipStream_t st);
// Pair scores from head scores and the selection, one workgroup per conversation
// (pairs_select_fits says whether a conversation's head values fit one).
bool pairs_select_fits(int L, int Hq);
hipError_t launch_pairs_select(const PairsSelectArgs &a, hipStream_t st);
// head sums -> head and pair scores (head_dist_sum, head_score, pair_dist may be null)
hipError_t launch_scores_from_sums(const float *head_sum, const float *head_dist_sum, int n_pairs_total,
                                   int Hq, float inv_tokens, float *pair_cos, float *head_score,
                                   float *pair_dist, hipStream_t st);
// Initial-Recent mass per layer from the (m, Z) records and the Zir values: mean over rows and heads of
// Zir / Z; eligible = (mass >= gamma).  head_ir is scratch [B][L][Hq]; ir_mass or eligible may be null.
hipError_t launch_finalize_ir(const StateLayout &lay, const float4 *state, const float *state_ir, int B, int L,
                              int Hq, int Hkv, int Tq, float gamma, float *head_ir, float *ir_mass,
                              uint8_t *eligible, hipStream_t st);
hipError_t launch_select(const float *pair_score, const uint8_t *eligible, int batch, int n_layers,
                         int n_select, int32_t *out_pairs, int32_t *out_count, hipStream_t st);

// Workgroups of the matrix-core kernels that run side by side on one XCD (32 CUs, one 4 MB L2) are dealt
// a PATCH of one unit's (row tile, key split) grid: patch_rows() row tiles by 32 / patch_rows() key
// splits.  The workgroups of a patch row read the same query rows and those of a patch column the same
// keys, at about the same time, so most of both streams is found in the L2 and comes from HBM once per
// patch instead of once per workgroup.  The patch shape used is the one that divides the unit's grid;
// patch_rows() returns 0 if none does (then workgroups are numbered row tile first, as without patches).
__host__ __device__ inline int patch_rows(int n_row_tiles, int n_split)
{
    for (int pr = 8; pr >= 1; pr >>= 1)
        if (n_row_tiles % pr == 0 && n_split % (32 / pr) == 0) return pr;
    return 0;
}

// Index (in float4 records) of the record of partial p of row r of unit u
// (u = b * Hkv + kv head; r = head-in-group * Tq + t) for layer l.
__host__ __device__ inline size_t state_index(const StateLayout &y, int u, int r, int p, int l)
{
    if (y.variant == kGeneric) {
        const size_t grow = (size_t)u * y.rows_per_unit + r;
        return (grow * y.n_split + p) * y.n_layers + l;
    }
    // MFMA variants: one record per (workgroup, layer, row); partial p = key split
    const int r_wg = y.wr * y.rb * 32;
    const int rt = r / r_wg, rr = r % r_wg;
    const size_t wg = ((size_t)u * y.n_split + p) * y.n_row_tiles + rt;
    return (wg * y.n_layers + l) * r_wg + rr;
}

}  // namespace krul
