// C ABI of libkrul: argument checks, kernel choice, launches.  See include/krul.h for
// the contract of each entry point.
#include <math.h>

#include <mutex>

#include "krul_common.h"

namespace krul {
namespace {

constexpr int kTargetWorkgroups = 512;   // two eight-wave workgroups for each of 256 CUs
constexpr size_t kAlign = 256;

size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

}  // namespace

int check_shape(const krul_shape_t *s)
{
    if (!s) return KRUL_EINVAL;
    if (s->dtype != KRUL_F32 && s->dtype != KRUL_BF16 && s->dtype != KRUL_F16) return KRUL_EDTYPE;
    if (s->batch <= 0 || s->n_layers < 2 || s->n_q_heads <= 0 || s->n_kv_heads <= 0 ||
        s->head_dim <= 0 || s->n_hist <= 0 || s->n_query <= 0)
        return KRUL_EINVAL;
    if (s->n_q_heads % s->n_kv_heads != 0) return KRUL_EINVAL;
    if (!(s->scale >= 0.f) || !isfinite(s->scale)) return KRUL_EINVAL;
    if (s->flags & ~(KRUL_FLAG_CAUSAL | KRUL_FLAG_GENERIC_KERNEL | KRUL_FLAG_SINGLE_SPLIT)) return KRUL_EINVAL;
    if ((s->flags & KRUL_FLAG_CAUSAL) && s->n_hist < s->n_query) return KRUL_EINVAL;
    if (s->head_dim % 8 != 0 || s->head_dim > 256) return KRUL_EUNSUPPORTED;
    if (s->n_layers > 2048) return KRUL_EUNSUPPORTED;
    return KRUL_OK;
}


int make_plan(const krul_shape_t *s, Plan *pl, bool want_ir, bool plain_keys)
{
    const int rc = check_shape(s);
    if (rc != KRUL_OK) return rc;
    const long long B = s->batch, L = s->n_layers, Hq = s->n_q_heads, Hkv = s->n_kv_heads;
    const long long S = s->n_hist, Tq = s->n_query, g = Hq / Hkv, Rk = g * Tq;
    if (Rk > INT32_MAX || B * Hq * Tq > INT32_MAX) return KRUL_EUNSUPPORTED;

    const float scale = s->scale > 0.f ? s->scale : 1.0f / sqrtf((float)s->head_dim);
    pl->c = scale * 1.4426950408889634f;
    StateLayout &y = pl->lay;
    y.n_layers = (int)L;
    y.rows_per_unit = (int)Rk;

    // 16-bit inputs with a head size up to 128 take the matrix cores (64 and 128 as they are, the sizes between
    // zero-padded to the next of the two inside LDS)
    const bool mfma = (s->dtype == KRUL_BF16 || s->dtype == KRUL_F16) && s->head_dim <= 128 &&
                      !(s->flags & KRUL_FLAG_GENERIC_KERNEL);
    long long n_wg, records;
    if (mfma) {
        int kt;
        // Which shape of workgroup tile (rows x keys).  A shape's ordinary form is for problems that give
        // the 256 CUs about a round of workgroups (w below) or more; with fewer, a "short" form with fewer
        // keys per tile makes two to four times as many workgroups (measured, one conversation of
        // Llama-3-8B shape: 64 query tokens over 2048 keys 92 -> 64 us, 16 over 4096 96 -> 63 us, one over
        // 4096 82 -> 64 us).  The thresholds are where the two forms measured equal.
        if (Rk <= 32) {
            // Decode steps, bound by the stream of keys.  With two or more rounds of workgroups, four waves
            // with three chunks of keys in flight do better than eight waves with one (+2..4 %, +6 % at
            // head_dim 64).
            const long long w = B * Hkv * ((S + 511) / 512);
            if (w <= 192) { y.variant = kMfmaSlimShort; y.wr = 1; y.wk = 4; y.rb = 1; kt = 256; }
            else if (w >= 512) { y.variant = kMfmaSlimDeep; y.wr = 1; y.wk = 4; y.rb = 1; kt = 512; }
            else { y.variant = kMfmaSlim; y.wr = 1; y.wk = 8; y.rb = 1; kt = 512; }
        } else if (Rk <= 64) {
            const long long w = B * Hkv * ((S + 511) / 512);
            if (w <= 128) { y.variant = kMfmaMidShort; y.wr = 2; y.wk = 2; y.rb = 1; kt = 128; }
            else { y.variant = kMfmaMid; y.wr = 2; y.wk = 4; y.rb = 1; kt = 512; }
        } else {
            const long long w = B * Hkv * ((Rk + 127) / 128) * ((S + 255) / 256);
            // Many query rows on a large problem: 256 x 256 tiles (two 32-row blocks per wave, the previous layer's
            // exponentials kept as binary16 pairs) move a third fewer bytes per logit and read half the operands.
            // Taken when the rows fill 256-row tiles well and there are two rounds of workgroups or more.
            const long long nrt_big = (Rk + 255) / 256, w_big = B * Hkv * nrt_big * ((S + 255) / 256);
            const bool big = plain_keys && !want_ir && !(s->flags & KRUL_FLAG_CAUSAL) && s->head_dim == 128 &&
                             nrt_big * 256 * 7 <= Rk * 8 && w_big >= 512;
            if (big) { y.variant = kMfmaBig; y.wr = 4; y.wk = 2; y.rb = 2; kt = 256; }
            else if (w <= 128) { y.variant = kMfmaWideShort; y.wr = 4; y.wk = 2; y.rb = 1; kt = 128; }
            else { y.variant = kMfmaWide; y.wr = 4; y.wk = 2; y.rb = 1; kt = 256; }
        }
        const long long r_wg = y.wr * y.rb * 32;
        const long long nrt = (Rk + r_wg - 1) / r_wg;
        const long long units = B * Hkv * nrt;
        const long long tiles = (S + kt - 1) / kt;
        // the wide tile's workgroups are resident one per CU: aim for one round of them
        const bool wide = y.variant == kMfmaWide || y.variant == kMfmaWideShort || y.variant == kMfmaBig;
        const long long target = wide ? kTargetWorkgroups / 2 : kTargetWorkgroups;
        long long want = (target + units - 1) / units;
        // The narrow tiles are bound by the stream of keys: there a split of several tiles, which
        // parks its running records in memory between tiles, costs a quarter of the bandwidth (a decode
        // step over 131072 tokens: 57 % of 8 TB/s against 74 % with one tile per split), and the
        // partial records stay below 1 % of the key bytes.  So: one tile per split, up to 1024 splits.
        if (!wide && want < 1024) want = 1024;
        // The wide tile on a large problem: four key splits (or more) per row tile, so that the workgroups
        // running side by side on an XCD form patches of 8 row tiles x 4 key splits (patch_rows()) and share
        // both their query rows and their keys through the L2 -- as long as a split keeps four tiles or more
        if ((y.variant == kMfmaWide || y.variant == kMfmaBig) && want < 4 && tiles >= 16 && nrt % 8 == 0) want = 4;
        if (want < 1 || (s->flags & KRUL_FLAG_SINGLE_SPLIT)) want = 1;
        long long nsplit = want < tiles ? want : tiles;
        const long long tps = (tiles + nsplit - 1) / nsplit;
        nsplit = (tiles + tps - 1) / tps;
        y.n_row_tiles = (int)nrt;
        y.n_split = (int)nsplit;
        y.partials = (int)nsplit;
        pl->keys_per_split = (int)(tps * kt);
        n_wg = units * nsplit;
        records = n_wg * L * r_wg;
    } else {
        y.variant = kGeneric;
        y.wr = y.wk = y.rb = 1;
        y.n_row_tiles = 1;
        const long long rows = B * Hq * Tq;
        long long want = (2048 + rows - 1) / rows;
        const long long max_split = (S + 255) / 256;
        long long nsplit = want < max_split ? want : max_split;
        if (nsplit < 1 || (s->flags & KRUL_FLAG_SINGLE_SPLIT)) nsplit = 1;
        long long kps = ((S + nsplit - 1) / nsplit + 63) / 64 * 64;
        nsplit = (S + kps - 1) / kps;
        y.n_split = (int)nsplit;
        y.partials = (int)nsplit;
        pl->keys_per_split = (int)kps;
        n_wg = rows * nsplit;
        records = n_wg * L;
    }
    if (n_wg > INT32_MAX) return KRUL_EUNSUPPORTED;
    pl->n_workgroups = (int)n_wg;
    pl->state_bytes = round_up((size_t)records * sizeof(float4), kAlign);
    const size_t head_bytes = round_up((size_t)(B * (L - 1) * Hq) * sizeof(float), kAlign);
    pl->head_cos_off = pl->state_bytes;
    pl->head_dist_off = pl->head_cos_off + head_bytes;
    pl->total_bytes = pl->head_dist_off + head_bytes;
    pl->state_ir_off = pl->head_ir_off = 0;
    if (want_ir) {
        pl->state_ir_off = pl->total_bytes;
        pl->head_ir_off = pl->state_ir_off + round_up((size_t)records * sizeof(float), kAlign);
        pl->total_bytes = pl->head_ir_off + round_up((size_t)(B * L * Hq) * sizeof(float), kAlign);
    }
    return KRUL_OK;
}

int resolve_keys(const krul_shape_t *s, bool mfma, bool dense_2gib, const void *k, const krul_k_layout_t *kl,
                 const krul_k_pages_t *kp, KeyAddr *out)
{
    if ((k != nullptr) + (kl != nullptr) + (kp != nullptr) != 1) return KRUL_EINVAL;
    const long long d = s->head_dim, S = s->n_hist;
    KeyAddr a = {};
    if (k) {
        if ((uintptr_t)k & 15) return KRUL_EINVAL;
        if (mfma && dense_2gib && S * d * 2 >= (1ll << 31)) return KRUL_EUNSUPPORTED;
        a.k = k;
        a.stride_l = (long long)s->n_kv_heads * S * d;
        a.stride_b = (long long)s->n_layers * s->n_kv_heads * S * d;
        a.stride_h = S * d;
        a.stride_s = d;
    } else if (kl) {
        if (!kl->k_layers || ((uintptr_t)kl->k_layers & 7)) return KRUL_EINVAL;
        const long long sb = s->batch > 1 ? kl->k_stride_b : 8;   // (not used for one conversation)
        if (sb <= 0 || kl->k_stride_h <= 0 || kl->k_stride_s < d || ((sb | kl->k_stride_h | kl->k_stride_s) & 7))
            return KRUL_EINVAL;
        // the matrix-core kernels' 32-bit offsets and ranges need a layer's keys of one head to span
        // less than 2 GiB
        if (mfma && (kl->k_stride_s >= (1ll << 23) ||
                     (dense_2gib && kl->k_stride_s * 2 * S >= (1ll << 31))))
            return KRUL_EUNSUPPORTED;
        a.k_tab = kl->k_layers;
        a.stride_b = s->batch > 1 ? kl->k_stride_b : 0;
        a.stride_h = kl->k_stride_h;
        a.stride_s = kl->k_stride_s;
    } else {
        if (!kp->k_layers || !kp->block_table || ((uintptr_t)kp->k_layers & 7) || ((uintptr_t)kp->block_table & 3))
            return KRUL_EINVAL;
        const int bs = kp->block_size;
        if (bs < 8 || (bs & (bs - 1)) || kp->max_blocks < (S + bs - 1) / bs || kp->k_stride_block <= 0 ||
            kp->k_stride_h <= 0 || kp->k_stride_s < d || ((kp->k_stride_block | kp->k_stride_h | kp->k_stride_s) & 7))
            return KRUL_EINVAL;
        // (32-bit byte offsets over the keys one copy instruction moves)
        if (mfma && kp->k_stride_s >= (1ll << 27)) return KRUL_EUNSUPPORTED;
        a.k_tab = kp->k_layers;
        a.block_table = kp->block_table;
        a.max_blocks = kp->max_blocks;
        for (a.page_shift = 3; (1 << a.page_shift) < bs; ++a.page_shift) {}
        a.stride_page = kp->k_stride_block;
        a.stride_h = kp->k_stride_h;
        a.stride_s = kp->k_stride_s;
    }
    *out = a;
    return KRUL_OK;
}

}  // namespace krul

using namespace krul;

namespace {
__global__ __launch_bounds__(256) void calibration_copy_kernel(const uint4 *__restrict__ src,
                                                               uint4 *__restrict__ dst, size_t n)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}
}  // namespace

namespace {
// Selection asked for in the same call (krul_pair_similarity_select).
struct SelectArgs {
    const uint8_t *eligible;
    int n_select;
    int32_t *out_pairs, *out_count;
};

// The one implementation behind the similarity entry points.  ir: also run the Initial-Recent layer
// test (gamma, ir_mass, eligible as for krul_pair_similarity_ir).
// accumulate: head_score / pair_dist are the caller's running sums [B][L-1][Hq] (see
// krul_pair_similarity_accumulate) and pair_score is unused.
int run_similarity(const krul_shape_t *shape, const void *q, const void *k, float *pair_score,
                   float *head_score, float *pair_dist, bool ir, float gamma, float *ir_mass,
                   uint8_t *eligible, void *workspace, size_t workspace_bytes, void *stream,
                   void *event_begin, void *event_end, bool accumulate = false,
                   const krul_k_layout_t *kl = nullptr, const krul_k_pages_t *kp = nullptr,
                   const SelectArgs *sel = nullptr)
{
    Plan pl;
    const int rc = make_plan(shape, &pl, ir, k != nullptr && !kl && !kp);
    if (rc != KRUL_OK) return rc;
    if (!q || (accumulate ? !head_score : !pair_score)) return KRUL_EINVAL;
    if (ir && (shape->flags & KRUL_FLAG_CAUSAL)) return KRUL_EUNSUPPORTED;
    if ((uintptr_t)q & 15) return KRUL_EINVAL;
    if (((uintptr_t)pair_score | (uintptr_t)head_score | (uintptr_t)pair_dist | (uintptr_t)ir_mass) & 3)
        return KRUL_EINVAL;
    if (ir && (!(gamma >= 0.f) || !isfinite(gamma) || (!ir_mass && !eligible))) return KRUL_EINVAL;
    if (!workspace || ((uintptr_t)workspace & (kAlign - 1)) || workspace_bytes < pl.total_bytes)
        return KRUL_EWORKSPACE;

    hipStream_t st = static_cast<hipStream_t>(stream);
    unsigned char *ws = static_cast<unsigned char *>(workspace);
    SimParams p;
    p.q = q;
    p.state = reinterpret_cast<float4 *>(ws);
    p.B = shape->batch;
    p.L = shape->n_layers;
    p.Hq = shape->n_q_heads;
    p.Hkv = shape->n_kv_heads;
    p.g = p.Hq / p.Hkv;
    p.d = shape->head_dim;
    p.S = shape->n_hist;
    p.Tq = shape->n_query;
    p.keys_per_split = pl.keys_per_split;
    p.c = pl.c;
    p.want_dist = pair_dist != nullptr || ir;   // the test needs Z as well
    p.want_ir = ir;
    p.causal = (shape->flags & KRUL_FLAG_CAUSAL) != 0;
    p.f16 = shape->dtype == KRUL_F16;
    // T_initial = T[:10% s], T_recent = T[90% s:] (Sec. 4.2): keys [0, floor(0.1 S)) and [floor(0.9 S), S)
    p.ir_init_end = (int)floor(0.1 * (double)p.S);
    p.ir_recent_begin = (int)floor(0.9 * (double)p.S);
    p.state_ir = reinterpret_cast<float *>(ws + pl.state_ir_off);
    p.lay = pl.lay;
    {
        KeyAddr ka;
        const int krc = resolve_keys(shape, pl.lay.variant != kGeneric, true, k, kl, kp, &ka);
        if (krc != KRUL_OK) return krc;
        p.k = ka.k;
        p.k_tab = ka.k_tab;
        p.k_stride_l = ka.stride_l;
        p.k_stride_b = ka.stride_b;
        p.k_stride_h = ka.stride_h;
        p.k_stride_s = ka.stride_s;
        p.block_table = ka.block_table;
        p.page_shift = ka.page_shift;
        p.max_blocks = ka.max_blocks;
        p.k_stride_page = ka.stride_page;
    }

    if (event_begin && hipEventRecord(static_cast<hipEvent_t>(event_begin), st) != hipSuccess)
        return KRUL_ELAUNCH;
    hipError_t e = pl.lay.variant == kGeneric
                       ? launch_sim_generic(p, shape->dtype, pl.n_workgroups, st)
                       : launch_sim_mfma(p, pl.n_workgroups, st);
    if (e != hipSuccess) return KRUL_ELAUNCH;
    if (event_end && hipEventRecord(static_cast<hipEvent_t>(event_end), st) != hipSuccess)
        return KRUL_ELAUNCH;
    float *head_cos = head_score ? head_score : reinterpret_cast<float *>(ws + pl.head_cos_off);
    float *head_dist = accumulate ? pair_dist : reinterpret_cast<float *>(ws + pl.head_dist_off);
    if (sel && pairs_select_fits(p.L, p.Hq)) {   // head scores, then pairs and selection in one small launch
        e = launch_finalize(pl.lay, p.state, p.B, p.L, p.Hq, p.Hkv, p.Tq, head_cos, head_dist, nullptr,
                            pair_dist, false, st);
        if (e == hipSuccess) {
            const PairsSelectArgs a = {head_cos, pair_dist ? head_dist : nullptr, pair_score, pair_dist, sel->eligible,
                                       p.B, p.L, p.Hq, sel->n_select, sel->out_pairs, sel->out_count};
            e = launch_pairs_select(a, st);
        }
        return e == hipSuccess ? KRUL_OK : KRUL_ELAUNCH;
    }
    e = launch_finalize(pl.lay, p.state, p.B, p.L, p.Hq, p.Hkv, p.Tq, head_cos, head_dist,
                        pair_score, pair_dist, accumulate, st);
    if (e != hipSuccess) return KRUL_ELAUNCH;
    if (sel) {
        e = launch_select(pair_score, sel->eligible, p.B, p.L, sel->n_select, sel->out_pairs, sel->out_count, st);
        if (e != hipSuccess) return KRUL_ELAUNCH;
    }
    if (ir) {
        e = launch_finalize_ir(pl.lay, p.state, p.state_ir, p.B, p.L, p.Hq, p.Hkv, p.Tq, gamma,
                               reinterpret_cast<float *>(ws + pl.head_ir_off), ir_mass, eligible, st);
        if (e != hipSuccess) return KRUL_ELAUNCH;
    }
    return KRUL_OK;
}
}  // namespace

extern "C" {

int krul_calibration_copy(const void *src, void *dst, size_t bytes, void *stream)
{
    if (!src || !dst || bytes == 0 || (bytes & 15) || (((uintptr_t)src | (uintptr_t)dst) & 15))
        return KRUL_EINVAL;
    hipLaunchKernelGGL(calibration_copy_kernel, dim3(256 * 8), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint4 *>(src), static_cast<uint4 *>(dst), bytes / 16);
    return hipGetLastError() == hipSuccess ? KRUL_OK : KRUL_ELAUNCH;
}

int krul_pair_similarity_plan(const krul_shape_t *shape, int32_t *n_workgroups, int32_t *n_key_splits)
{
    Plan pl;
    const int rc = make_plan(shape, &pl, false, true);
    if (rc != KRUL_OK) return rc;
    if (n_workgroups) *n_workgroups = pl.n_workgroups;
    if (n_key_splits) *n_key_splits = pl.lay.n_split;
    return pl.lay.variant;
}

size_t krul_pair_similarity_workspace(const krul_shape_t *shape)
{
    // enough for the call on dense keys and for the calls on keys read in place (their plans may differ)
    Plan pl, pl_dense;
    if (make_plan(shape, &pl) != KRUL_OK || make_plan(shape, &pl_dense, false, true) != KRUL_OK) return 0;
    return pl.total_bytes > pl_dense.total_bytes ? pl.total_bytes : pl_dense.total_bytes;
}

int krul_pair_similarity(const krul_shape_t *shape, const void *q, const void *k,
                         float *pair_score, float *head_score, float *pair_dist,
                         void *workspace, size_t workspace_bytes, void *stream)
{
    return krul_pair_similarity_timed(shape, q, k, pair_score, head_score, pair_dist, workspace,
                                      workspace_bytes, stream, nullptr, nullptr);
}

int krul_pair_similarity_timed(const krul_shape_t *shape, const void *q, const void *k,
                               float *pair_score, float *head_score, float *pair_dist,
                               void *workspace, size_t workspace_bytes, void *stream,
                               void *event_begin, void *event_end)
{
    return run_similarity(shape, q, k, pair_score, head_score, pair_dist, false, 0.f, nullptr, nullptr,
                          workspace, workspace_bytes, stream, event_begin, event_end);
}

}  // extern "C"

namespace {
// The scratch area of krul_pair_similarity_static: device memory the code object brings along, one copy
// per GPU.  In host code the array's name only stands for the symbol; its device address is asked for
// once per GPU (that GPU current) and kept.
static __device__ __align__(256) unsigned char scratch[KRUL_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
std::mutex scratch_mutex;
void *scratch_ptr[kMaxDevices];   // by device ordinal; null until the first call on that device

int static_scratch(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return KRUL_ELAUNCH;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return KRUL_ELAUNCH;
        scratch_ptr[dev] = ptr;
    }
    *out = scratch_ptr[dev];
    return KRUL_OK;
}
}  // namespace

extern "C" {

int krul_pair_similarity_static(const krul_shape_t *shape, const void *q, const void *k,
                                float *pair_score, float *head_score, float *pair_dist, void *stream)
{
    Plan pl;
    const int rc = make_plan(shape, &pl, false, true);
    if (rc != KRUL_OK) return rc;
    if (pl.total_bytes > (size_t)KRUL_STATIC_SCRATCH_BYTES) return KRUL_ESCRATCH;
    void *ptr = nullptr;
    const int src = static_scratch(&ptr);
    if (src != KRUL_OK) return src;
    // Nothing in the area has to start at zero: every record the finalize kernels read is written by the
    // similarity kernel of the same call first.
    return run_similarity(shape, q, k, pair_score, head_score, pair_dist, false, 0.f, nullptr, nullptr,
                          ptr, (size_t)KRUL_STATIC_SCRATCH_BYTES, stream, nullptr, nullptr);
}

int krul_pair_similarity_strided(const krul_shape_t *shape, const void *q, const krul_k_layout_t *k_layout,
                                 float *pair_score, float *head_score, float *pair_dist,
                                 void *workspace, size_t workspace_bytes, void *stream)
{
    if (!k_layout) return KRUL_EINVAL;
    return run_similarity(shape, q, nullptr, pair_score, head_score, pair_dist, false, 0.f, nullptr, nullptr,
                          workspace, workspace_bytes, stream, nullptr, nullptr, false, k_layout);
}

namespace {
// exactly one source of keys
bool one_source(const krul_keys_t *keys)
{
    return keys && (keys->dense != nullptr) + (keys->strided != nullptr) + (keys->paged != nullptr) == 1;
}
}  // namespace

int krul_all_pairs_similarity_in_place(const krul_shape_t *shape, const void *q, const krul_keys_t *keys,
                                       float *pair_score_all, float *pair_dist_all, float *head_score_all,
                                       void *workspace, size_t workspace_bytes, void *stream)
{
    if (!one_source(keys)) return KRUL_EINVAL;
    return run_all_pairs(shape, q, keys->dense, keys->strided, keys->paged, pair_score_all, pair_dist_all,
                         head_score_all, workspace, workspace_bytes, static_cast<hipStream_t>(stream));
}

size_t krul_all_pairs_workspace(const krul_shape_t *shape, size_t max_bytes)
{
    return all_pairs_workspace(shape, max_bytes);
}

int krul_all_pairs_similarity(const krul_shape_t *shape, const void *q, const void *k,
                              float *pair_score_all, float *pair_dist_all, float *head_score_all,
                              void *workspace, size_t workspace_bytes, void *stream)
{
    return run_all_pairs(shape, q, k, nullptr, nullptr, pair_score_all, pair_dist_all, head_score_all, workspace,
                         workspace_bytes, static_cast<hipStream_t>(stream));
}

int krul_select_pairs_all(const float *score, int32_t closer_is_smaller, const uint8_t *eligible,
                          int32_t batch, int32_t n_layers, int32_t n_select,
                          int32_t *out_pairs, int32_t *out_count, void *stream)
{
    if (!score || !out_count || batch <= 0 || n_layers < 2 || n_select < 0 || n_select > n_layers / 2 ||
        (n_select > 0 && !out_pairs))
        return KRUL_EINVAL;
    if (((uintptr_t)score | (uintptr_t)out_pairs | (uintptr_t)out_count) & 3) return KRUL_EINVAL;
    if (n_layers > 1024) return KRUL_EUNSUPPORTED;   // (n_select rounds over n_layers^2 entries)
    const hipError_t e = launch_select_all(score, closer_is_smaller, eligible, batch, n_layers, n_select, out_pairs,
                                           out_count, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? KRUL_OK : KRUL_ELAUNCH;
}

int krul_pair_similarity_select(const krul_shape_t *shape, const void *q, const void *k,
                                const uint8_t *eligible, int32_t n_select,
                                float *pair_score, float *head_score, float *pair_dist,
                                int32_t *out_pairs, int32_t *out_count,
                                void *workspace, size_t workspace_bytes, void *stream,
                                void *event_begin, void *event_end)
{
    if (!shape || !out_count || n_select < 0 || n_select > shape->n_layers / 2 || (n_select > 0 && !out_pairs))
        return KRUL_EINVAL;
    if (((uintptr_t)out_pairs | (uintptr_t)out_count) & 3) return KRUL_EINVAL;
    const SelectArgs sel = {eligible, n_select, out_pairs, out_count};
    return run_similarity(shape, q, k, pair_score, head_score, pair_dist, false, 0.f, nullptr, nullptr,
                          workspace, workspace_bytes, stream, event_begin, event_end, false, nullptr, nullptr, &sel);
}

int krul_pair_similarity_paged(const krul_shape_t *shape, const void *q, const krul_k_pages_t *k_pages,
                               float *pair_score, float *head_score, float *pair_dist,
                               void *workspace, size_t workspace_bytes, void *stream)
{
    if (!k_pages) return KRUL_EINVAL;
    return run_similarity(shape, q, nullptr, pair_score, head_score, pair_dist, false, 0.f, nullptr, nullptr,
                          workspace, workspace_bytes, stream, nullptr, nullptr, false, nullptr, k_pages);
}

int krul_pair_similarity_accumulate(const krul_shape_t *shape, const void *q, const void *k,
                                    float *head_sum, float *head_dist_sum,
                                    void *workspace, size_t workspace_bytes, void *stream)
{
    return run_similarity(shape, q, k, nullptr, head_sum, head_dist_sum, false, 0.f, nullptr, nullptr,
                          workspace, workspace_bytes, stream, nullptr, nullptr, true);
}

int krul_pair_similarity_accumulate_in_place(const krul_shape_t *shape, const void *q, const krul_keys_t *keys,
                                             float *head_sum, float *head_dist_sum,
                                             void *workspace, size_t workspace_bytes, void *stream)
{
    if (!one_source(keys)) return KRUL_EINVAL;
    return run_similarity(shape, q, keys->dense, nullptr, head_sum, head_dist_sum, false, 0.f, nullptr, nullptr,
                          workspace, workspace_bytes, stream, nullptr, nullptr, true, keys->strided, keys->paged);
}

int krul_pair_similarity_ir_in_place(const krul_shape_t *shape, const void *q, const krul_keys_t *keys, float gamma,
                                     float *pair_score, float *head_score, float *pair_dist,
                                     float *ir_mass, uint8_t *eligible,
                                     void *workspace, size_t workspace_bytes, void *stream)
{
    if (!one_source(keys)) return KRUL_EINVAL;
    return run_similarity(shape, q, keys->dense, pair_score, head_score, pair_dist, true, gamma, ir_mass, eligible,
                          workspace, workspace_bytes, stream, nullptr, nullptr, false, keys->strided, keys->paged);
}

int krul_pair_scores_from_sums(const float *head_sum, const float *head_dist_sum,
                               int32_t batch, int32_t n_layers, int32_t n_q_heads, float n_tokens,
                               float *pair_score, float *head_score, float *pair_dist, void *stream)
{
    if (!head_sum || !pair_score || batch <= 0 || n_layers < 2 || n_q_heads <= 0 || !(n_tokens > 0.f) ||
        !isfinite(n_tokens) || (pair_dist && !head_dist_sum))
        return KRUL_EINVAL;
    if (((uintptr_t)head_sum | (uintptr_t)head_dist_sum | (uintptr_t)pair_score | (uintptr_t)head_score |
         (uintptr_t)pair_dist) & 3)
        return KRUL_EINVAL;
    const hipError_t e = launch_scores_from_sums(head_sum, head_dist_sum, batch * (n_layers - 1), n_q_heads,
                                                 1.0f / n_tokens, pair_score, head_score, pair_dist,
                                                 static_cast<hipStream_t>(stream));
    return e == hipSuccess ? KRUL_OK : KRUL_ELAUNCH;
}

size_t krul_pair_similarity_ir_workspace(const krul_shape_t *shape)
{
    Plan pl;
    if (make_plan(shape, &pl, true) != KRUL_OK) return 0;
    return pl.total_bytes;
}

int krul_pair_similarity_ir(const krul_shape_t *shape, const void *q, const void *k, float gamma,
                            float *pair_score, float *head_score, float *pair_dist,
                            float *ir_mass, uint8_t *eligible,
                            void *workspace, size_t workspace_bytes, void *stream)
{
    return run_similarity(shape, q, k, pair_score, head_score, pair_dist, true, gamma, ir_mass, eligible,
                          workspace, workspace_bytes, stream, nullptr, nullptr);
}

int krul_select_pairs(const float *pair_score, const uint8_t *eligible,
                      int32_t batch, int32_t n_layers, int32_t n_select,
                      int32_t *out_pairs, int32_t *out_count, void *stream)
{
    if (!pair_score || !out_count || batch <= 0 || n_layers < 2 || n_select < 0 ||
        n_select > n_layers / 2 || (n_select > 0 && !out_pairs))
        return KRUL_EINVAL;
    if (((uintptr_t)pair_score | (uintptr_t)out_pairs | (uintptr_t)out_count) & 3) return KRUL_EINVAL;
    if (n_layers > 4096) return KRUL_EUNSUPPORTED;
    const hipError_t e = launch_select(pair_score, eligible, batch, n_layers, n_select, out_pairs,
                                       out_count, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? KRUL_OK : KRUL_ELAUNCH;
}

int32_t krul_n_select_from_ratio(int32_t n_layers, float r_l)
{
    if (n_layers < 2 || !(r_l > 0.f)) return 0;
    const double want = ceil((double)n_layers * (double)r_l / 2.0 - 1e-9);
    const int32_t cap = n_layers / 2;
    return want > cap ? cap : (int32_t)want;
}

const char *krul_strerror(int status)
{
    switch (status) {
    case KRUL_OK: return "ok";
    case KRUL_EINVAL: return "invalid argument";
    case KRUL_EDTYPE: return "unknown dtype";
    case KRUL_EWORKSPACE: return "workspace missing, misaligned or too small";
    case KRUL_ELAUNCH: return "kernel launch failed";
    case KRUL_EUNSUPPORTED: return "no kernel for this shape";
    case KRUL_ESCRATCH: return "the problem needs more scratch memory than the library's built-in area holds";
    default: return "unknown status";
    }
}

}  // extern "C"
