// Offline-phase host helpers: BN folding, weight packing, launch planning.
// (Paper, "Offline Phase": everything that can be prepared before a task is
// released is prepared once.)
#include <algorithm>
#include <cmath>
#include <cstring>

#include "internal.h"

namespace sgprs {

int check_conv_desc(const sgprs_conv_desc_t* d)
{
    if (!d) return fail(SGPRS_ERR_INVALID_ARG, "conv desc is NULL");
    if (!dtype_ok(d->dtype)) return fail(SGPRS_ERR_UNSUPPORTED, "dtype %d", d->dtype);
    if (d->n <= 0 || d->h <= 0 || d->w <= 0 || d->cin <= 0 || d->cout <= 0 || d->r <= 0 || d->s <= 0 ||
        d->stride <= 0 || d->pad < 0)
        return fail(SGPRS_ERR_INVALID_ARG, "non-positive conv dimension");
    if (d->h + 2 * d->pad < d->r || d->w + 2 * d->pad < d->s)
        return fail(SGPRS_ERR_INVALID_ARG, "kernel larger than padded input");
    if (!is_stem(*d) && !is_igemm(*d))
        return fail(SGPRS_ERR_UNSUPPORTED,
                    "conv %dx%d stride %d pad %d cin %d: supported are 1x1/3x3 stride 1/2 with "
                    "cin %% 32 == 0 and the 7x7 stride-2 pad-3 3-channel stem",
                    d->r, d->s, d->stride, d->pad, d->cin);
    if (d->cout % 64) return fail(SGPRS_ERR_UNSUPPORTED, "cout %d must be a multiple of 64", d->cout);
    if (is_igemm(*d) && d->dtype == SGPRS_BF16 && d->cin % 64)
        return fail(SGPRS_ERR_UNSUPPORTED, "bf16 conv needs cin %% 64 == 0 (got %d)", d->cin);
    const long long p = out_dim(d->h, d->r, d->stride, d->pad), q = out_dim(d->w, d->s, d->stride, d->pad);
    const long long in_el = (long long)d->n * d->h * d->w * d->cin, out_el = (long long)d->n * p * q * d->cout;
    if (in_el >= (1ll << 31) || out_el >= (1ll << 31))
        return fail(SGPRS_ERR_UNSUPPORTED, "tensor with 2^31 or more elements");
    return SGPRS_OK;
}

static size_t packed_elems(const sgprs_conv_desc_t& d)
{
    return is_stem(d) ? (size_t)d.cout * kStemK : (size_t)d.cout * d.r * d.s * d.cin;
}

// Position of w[k][c][r][s] in the packed array, or -1 for "not stored".
static inline size_t packed_index(const sgprs_conv_desc_t& d, int k, int c, int r, int s)
{
    if (is_stem(d)) return (size_t)k * kStemK + (size_t)r * kStemTapRow + s * 4 + c;
    return (((size_t)k * d.r + r) * d.s + s) * d.cin + c;
}

// Rough cost model (microseconds) used to pick a tile shape and split-K
// factor.  It only has to rank candidates; absolute accuracy is irrelevant.
struct Tile { int bm, bn; double eff; };
static const Tile kTiles[] = {{128, 128, 1.0}, {128, 64, 0.85}, {64, 64, 0.6}, {32, 128, 0.5}};

int igemm_num_variants() { return (int)(sizeof(kTiles) / sizeof(kTiles[0])); }

// Tuning overrides: written by sgprs_conv_tuning_override, read by whatever thread plans a launch
// (the lane launcher threads of a periodic run among them), hence atomics.
std::atomic<int> g_conv_force_kind{-1};
std::atomic<int> g_igemm_force_variant{-1};
std::atomic<int> g_igemm_force_splits{0};

std::atomic<int> g_plan_generation{0};

static ConvPlan plan_conv_uncached(const sgprs_conv_desc_t& d, int cus, bool has_residual);

ConvPlan plan_conv(const sgprs_conv_desc_t& d, int cus, bool has_residual)
{
    struct Key { sgprs_conv_desc_t d; int cus, res, gen; };
    static thread_local PlanMemo<Key, ConvPlan> local;
    static SharedPlanMemo<Key, ConvPlan> memo;
    Key k;
    memset(&k, 0, sizeof(k));
    k.d = d; k.cus = cus; k.res = has_residual; k.gen = g_plan_generation.load();
    return memo.get(local, k, [&]() { return plan_conv_uncached(d, cus, has_residual); });
}

static ConvPlan plan_conv_uncached(const sgprs_conv_desc_t& d, int cus, bool has_residual)
{
    const int force_kind = g_conv_force_kind.load(), force_variant = g_igemm_force_variant.load(),
              force_splits = g_igemm_force_splits.load();
    if (force_kind == -1) {
        int rows = 0;
        if (plan_rows(d, cus < 1 ? 1 : cus, &rows)) {
            ConvPlan p;
            p.kind = 3; p.variant = rows; p.splits = 1;
            p.bm = 1;  // marks a valid plan
            return p;
        }
    }
    if (force_kind != 0) {
        int v = 0, s = 1;
        if (plan_patch(d, cus < 1 ? 1 : cus, &v, &s)) {
            ConvPlan p;
            p.kind = 1; p.variant = v; p.splits = s;
            p.bm = 1;  // marks a valid plan
            return p;
        }
        if (force_kind != 1 && !has_residual && plan_s2patch(d, cus < 1 ? 1 : cus, &v)) {
            ConvPlan p;
            p.kind = 2; p.variant = v; p.splits = 1;
            p.bm = 1;
            return p;
        }
    }
    const int P = out_dim(d.h, d.r, d.stride, d.pad), Q = out_dim(d.w, d.s, d.stride, d.pad);
    const long long M = (long long)d.n * P * Q;
    const int kt_el = d.dtype == SGPRS_BF16 ? 64 : 32;
    const int ktiles = d.r * d.s * d.cin / kt_el;
    // time of one 128x128 tile over one k-tile on one CU at a realistic rate
    const double us_per_ktile_128 = d.dtype == SGPRS_BF16 ? 0.45 : 1.8;
    ConvPlan best;
    double best_cost = 1e30;
    if (cus < 1) cus = 1;
    for (int v = 0; v < igemm_num_variants(); ++v) {
        Tile t = kTiles[v];
        if (d.cout % t.bn) continue;
        // few output pixels (batch-1 layers of 28x28 and below): the 32-row tile wastes the fewest
        // rows and gives split-K the most workgroups; measured 3-7 % faster than 64x64 there
        if (t.bm == 32 && M <= 1024) t.eff = 0.8;
        if (force_variant >= 0 && force_variant < igemm_num_variants() && v != force_variant &&
            d.cout % kTiles[force_variant].bn == 0)
            continue;
        const long long gm = (M + t.bm - 1) / t.bm, gn = d.cout / t.bn;
        const long long blocks = gm * gn;
        const int occ = 2;  // workgroups resident per CU
        for (int s = 1; s <= 32; s *= 2) {
            if (s > 1 && ktiles / s < 2) break;
            // a forced split factor applies where the shape allows it (else the planner's own choice stands)
            if (force_variant >= 0 && force_splits > 1 && s != force_splits &&
                ktiles / force_splits >= 2)
                continue;
            if (force_variant >= 0 && force_splits == 1 && s != 1) continue;
            const int kt_per = (ktiles + s - 1) / s;
            if (s > 1 && (long long)(s - 1) * kt_per >= ktiles) continue;  // an empty split
            const double per_block =
                kt_per * us_per_ktile_128 * (t.bm * t.bn / 16384.0) / t.eff * occ + 2.0;
            const long long rounds = (blocks * s + (long long)cus * occ - 1) / ((long long)cus * occ);
            double cost = rounds * per_block;
            if (s > 1) {
                const double bytes = (double)M * d.cout * 4.0 * (s + 1);
                cost += 4.0 + bytes / (3.0e6 * cus / 256.0);
            }
            if (cost < best_cost) {
                best_cost = cost;
                best.variant = v; best.bm = t.bm; best.bn = t.bn; best.splits = s; best.ktiles = ktiles;
                best.grid_m = (int)gm; best.grid_n = (int)gn;
            }
        }
    }
    return best;
}

size_t conv_workspace_bytes(const sgprs_conv_desc_t& d, const ConvPlan& p)
{
    if (p.splits <= 1) return 0;
    const int P = out_dim(d.h, d.r, d.stride, d.pad), Q = out_dim(d.w, d.s, d.stride, d.pad);
    return (size_t)p.splits * d.n * P * Q * d.cout * sizeof(float);
}

}  // namespace sgprs

using namespace sgprs;

extern "C" {

int sgprs_fold_bn(const float* gamma, const float* beta, const float* mean, const float* var, float eps,
                  int c, float* scale, float* shift)
{
    if (!gamma || !beta || !mean || !var || !scale || !shift)
        return fail(SGPRS_ERR_INVALID_ARG, "NULL BN vector");
    if (c <= 0) return fail(SGPRS_ERR_INVALID_ARG, "c %d <= 0", c);
    for (int i = 0; i < c; ++i) {
        const double v = (double)var[i] + (double)eps;
        if (!(v > 0.0)) return fail(SGPRS_ERR_INVALID_ARG, "var[%d]+eps = %g is not positive", i, v);
        const double sc = (double)gamma[i] / std::sqrt(v);
        scale[i] = (float)sc;
        shift[i] = (float)((double)beta[i] - (double)mean[i] * sc);
    }
    return SGPRS_OK;
}

int sgprs_conv_packed_weight_bytes(const sgprs_conv_desc_t* d, size_t* bytes)
{
    int rc = check_conv_desc(d);
    if (rc) return rc;
    if (!bytes) return fail(SGPRS_ERR_INVALID_ARG, "bytes is NULL");
    *bytes = packed_elems(*d) * dtype_size(d->dtype);
    return SGPRS_OK;
}

int sgprs_pack_conv_weights(const sgprs_conv_desc_t* d, const float* w, void* packed, size_t bytes)
{
    int rc = check_conv_desc(d);
    if (rc) return rc;
    if (!w || !packed) return fail(SGPRS_ERR_INVALID_ARG, "NULL weight pointer");
    const size_t need = packed_elems(*d) * dtype_size(d->dtype);
    if (bytes < need) return fail(SGPRS_ERR_INVALID_ARG, "packed buffer %zu < %zu bytes", bytes, need);
    memset(packed, 0, need);
    for (int k = 0; k < d->cout; ++k)
        for (int c = 0; c < d->cin; ++c)
            for (int r = 0; r < d->r; ++r)
                for (int s = 0; s < d->s; ++s) {
                    const float v = w[(((size_t)k * d->cin + c) * d->r + r) * d->s + s];
                    const size_t o = packed_index(*d, k, c, r, s);
                    if (d->dtype == SGPRS_BF16) ((uint16_t*)packed)[o] = f32_to_bf16_bits(v);
                    else ((float*)packed)[o] = v;
                }
    return SGPRS_OK;
}

int sgprs_unpack_conv_weights(const sgprs_conv_desc_t* d, const void* packed, size_t bytes, float* w)
{
    int rc = check_conv_desc(d);
    if (rc) return rc;
    if (!w || !packed) return fail(SGPRS_ERR_INVALID_ARG, "NULL weight pointer");
    const size_t need = packed_elems(*d) * dtype_size(d->dtype);
    if (bytes < need) return fail(SGPRS_ERR_INVALID_ARG, "packed buffer %zu < %zu bytes", bytes, need);
    for (int k = 0; k < d->cout; ++k)
        for (int c = 0; c < d->cin; ++c)
            for (int r = 0; r < d->r; ++r)
                for (int s = 0; s < d->s; ++s) {
                    const size_t o = packed_index(*d, k, c, r, s);
                    w[(((size_t)k * d->cin + c) * d->r + r) * d->s + s] =
                        d->dtype == SGPRS_BF16 ? bf16_bits_to_f32(((const uint16_t*)packed)[o])
                                               : ((const float*)packed)[o];
                }
    return SGPRS_OK;
}

int sgprs_conv2d_workspace(const sgprs_conv_desc_t* d, int partition_cus, size_t* bytes)
{
    int rc = check_conv_desc(d);
    if (rc) return rc;
    if (!bytes) return fail(SGPRS_ERR_INVALID_ARG, "bytes is NULL");
    if (partition_cus <= 0) return fail(SGPRS_ERR_INVALID_ARG, "partition_cus %d <= 0", partition_cus);
    // the plan may depend on whether a residual is passed: enough for either
    *bytes = is_stem(*d) ? 0 : std::max(conv_workspace_bytes(*d, plan_conv(*d, partition_cus, false)),
                                        conv_workspace_bytes(*d, plan_conv(*d, partition_cus, true)));
    return SGPRS_OK;
}

int sgprs_conv2d_plan(const sgprs_conv_desc_t* d, int partition_cus, int has_residual, int* family, int* detail)
{
    int rc = check_conv_desc(d);
    if (rc) return rc;
    if (!family || !detail) return fail(SGPRS_ERR_INVALID_ARG, "family or detail is NULL");
    if (partition_cus <= 0) return fail(SGPRS_ERR_INVALID_ARG, "partition_cus %d <= 0", partition_cus);
    if (is_stem(*d)) {
        *family = 4; *detail = 0;
        return SGPRS_OK;
    }
    const ConvPlan p = plan_conv(*d, partition_cus, has_residual != 0);
    if (p.bm == 0) return fail(SGPRS_ERR_UNSUPPORTED, "no tile shape fits cout %d", d->cout);
    *family = p.kind; *detail = p.variant;
    return SGPRS_OK;
}

}  // extern "C"
