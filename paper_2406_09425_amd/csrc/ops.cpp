// Per-operator entry points: argument validation, then enqueue on the
// partition's stream.  A call that fails validation enqueues nothing.
#include "internal.h"

namespace sgprs {

thread_local hipEvent_t tl_start = nullptr, tl_stop = nullptr;

Profiler::~Profiler()
{
    for (hipEvent_t e : event_pool) (void)hipEventDestroy(e);
}

int Profiler::begin(hipStream_t s, int kind, int variant, double flops, double bytes)
{
    while (event_pool.size() < next_event + 2) {
        hipEvent_t e;
        // no system-scope release at the event: a full L2 write-back between kernels would slow down
        // the memory-heavy ones and the profile would not show the kernels as they run unprofiled
        SGPRS_HIP(hipEventCreateWithFlags(&e, hipEventDisableSystemFence));
        event_pool.push_back(e);
    }
    // Both events ride on the kernel's own dispatch packet (hipExtLaunchKernelGGL):
    // start..stop is the kernel alone, as a profiler's kernel trace reports it,
    // without the gap to the previous kernel.
    KernelRecord r;
    r.kind = kind; r.variant = variant; r.flops = flops; r.bytes = bytes;
    r.start = event_pool[next_event++];
    r.stop = event_pool[next_event++];
    recs.push_back(r);
    tl_start = r.start;
    tl_stop = r.stop;
    prev = r.stop;
    (void)s;
    return SGPRS_OK;
}

int Profiler::end(hipStream_t)
{
    tl_start = nullptr;
    tl_stop = nullptr;
    return SGPRS_OK;
}

static bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

}  // namespace sgprs

using namespace sgprs;

extern "C" {

int sgprs_conv2d(const sgprs_conv_desc_t* d, const void* x, const void* w_packed, const float* scale,
                 const float* shift, const void* residual, void* y, void* workspace, size_t workspace_bytes,
                 sgprs_pool_t* pool, int partition)
{
    int rc = check_conv_desc(d);
    if (rc) return rc;
    hipStream_t stream;
    int cus = 0;
    if ((rc = resolve(pool, partition, &stream, &cus))) return rc;
    if (!x || !w_packed || !scale || !shift || !y) return fail(SGPRS_ERR_INVALID_ARG, "NULL tensor pointer");
    if (!aligned16(x) || !aligned16(w_packed) || !aligned16(y) || !aligned16(residual) || !aligned16(scale) ||
        !aligned16(shift) || !aligned16(workspace))
        return fail(SGPRS_ERR_INVALID_ARG, "tensor pointers must be 16-byte aligned");
    if (x == y || (residual && residual == y)) return fail(SGPRS_ERR_INVALID_ARG, "y must not alias x or residual");
    if (is_stem(*d)) {
        if (residual) return fail(SGPRS_ERR_UNSUPPORTED, "stem conv takes no residual");
        return launch_stem(*d, x, w_packed, scale, shift, y, stream, cus, nullptr);
    }
    return launch_conv(*d, x, w_packed, scale, shift, residual, y, workspace, workspace_bytes, stream, cus, nullptr);
}

int sgprs_conv_tuning_override(int kind, int variant, int splits)
{
    if (kind < -1 || kind > 5) return fail(SGPRS_ERR_INVALID_ARG, "kind %d outside [-1,5]", kind);
    if (kind == 3 && (variant < 0 || variant > s2patch_num_variants()))
        return fail(SGPRS_ERR_INVALID_ARG, "stride-2 patch variant %d outside [0,%d]", variant, s2patch_num_variants());
    g_plan_generation.fetch_add(1);
    s2patch_force(kind == 3 ? variant : kind == 0 ? 2 : -1);
    stem_pool_force(kind == 4 ? 1 : -1);
    rows_force_off(kind == 5);
    g_conv_force_kind = kind >= 2 ? -1 : kind;
    g_igemm_force_variant = kind == 2 ? variant : -1;
    g_igemm_force_splits = kind == 2 ? splits : 0;
    patch_force(kind == 1 ? variant : -1, splits);
    return SGPRS_OK;
}

int sgprs_maxpool2d(int dtype, int n, int h, int w, int c, const void* x, void* y, sgprs_pool_t* pool,
                    int partition)
{
    hipStream_t stream;
    int cus = 0, rc;
    if ((rc = resolve(pool, partition, &stream, &cus))) return rc;
    if (!dtype_ok(dtype)) return fail(SGPRS_ERR_UNSUPPORTED, "dtype %d", dtype);
    if (n <= 0 || h <= 0 || w <= 0 || c <= 0) return fail(SGPRS_ERR_INVALID_ARG, "non-positive dimension");
    if (c % (dtype == SGPRS_BF16 ? 8 : 4)) return fail(SGPRS_ERR_UNSUPPORTED, "c %d not a multiple of the vector width", c);
    if ((long long)n * h * w * c >= (1ll << 31)) return fail(SGPRS_ERR_UNSUPPORTED, "tensor with 2^31 or more elements");
    if (!x || !y || !aligned16(x) || !aligned16(y) || x == y)
        return fail(SGPRS_ERR_INVALID_ARG, "x and y must be distinct, non-NULL and 16-byte aligned");
    return launch_maxpool(dtype, n, h, w, c, x, y, stream, cus, nullptr);
}

int sgprs_bn_relu(int dtype, size_t pixels, int c, const void* x, const float* scale, const float* shift,
                  void* y, sgprs_pool_t* pool, int partition)
{
    hipStream_t stream;
    int cus = 0, rc;
    if ((rc = resolve(pool, partition, &stream, &cus))) return rc;
    if (!dtype_ok(dtype)) return fail(SGPRS_ERR_UNSUPPORTED, "dtype %d", dtype);
    if (pixels == 0 || c <= 0) return fail(SGPRS_ERR_INVALID_ARG, "empty tensor");
    if (c % (dtype == SGPRS_BF16 ? 8 : 4)) return fail(SGPRS_ERR_UNSUPPORTED, "c %d not a multiple of the vector width", c);
    if (pixels >= (1ull << 31) / (size_t)c || c / (dtype == SGPRS_BF16 ? 8 : 4) >= 65536)
        return fail(SGPRS_ERR_UNSUPPORTED, "tensor with 2^31 or more elements, or 65536 or more channel vectors");
    if (!x || !y || !scale || !shift || !aligned16(x) || !aligned16(y))
        return fail(SGPRS_ERR_INVALID_ARG, "pointers must be non-NULL and 16-byte aligned");
    return launch_bn_relu(dtype, pixels, c, x, scale, shift, y, stream, cus, nullptr);
}

int sgprs_add_relu(int dtype, size_t count, const void* a, const void* b, void* y, int relu, sgprs_pool_t* pool,
                   int partition)
{
    hipStream_t stream;
    int cus = 0, rc;
    if ((rc = resolve(pool, partition, &stream, &cus))) return rc;
    if (!dtype_ok(dtype)) return fail(SGPRS_ERR_UNSUPPORTED, "dtype %d", dtype);
    if (count == 0 || count % 8) return fail(SGPRS_ERR_INVALID_ARG, "count %zu must be a positive multiple of 8", count);
    if (count >= (1ull << 31)) return fail(SGPRS_ERR_UNSUPPORTED, "tensor with 2^31 or more elements");
    if (!a || !b || !y || !aligned16(a) || !aligned16(b) || !aligned16(y))
        return fail(SGPRS_ERR_INVALID_ARG, "pointers must be non-NULL and 16-byte aligned");
    return launch_add_relu(dtype, count, a, b, y, relu, stream, cus, nullptr);
}

int sgprs_avgpool_fc(int dtype, int n, int hw, int cin, int cout, const void* x, const void* w, const float* bias,
                     float* logits, float* workspace, sgprs_pool_t* pool, int partition)
{
    hipStream_t stream;
    int cus = 0, rc;
    if ((rc = resolve(pool, partition, &stream, &cus))) return rc;
    if (!dtype_ok(dtype)) return fail(SGPRS_ERR_UNSUPPORTED, "dtype %d", dtype);
    if (n <= 0 || hw <= 0 || cout <= 0) return fail(SGPRS_ERR_INVALID_ARG, "non-positive dimension");
    if (n > 65535 || cout > (1 << 20) || (long long)n * hw * cin >= (1ll << 31))
        return fail(SGPRS_ERR_UNSUPPORTED, "more than 65535 images, 2^20 outputs or 2^31 input elements");
    if (cin != 512 && cin != 1024 && cin != 2048)
        return fail(SGPRS_ERR_UNSUPPORTED, "cin %d: supported are 512, 1024, 2048", cin);
    if (!x || !w || !logits || !workspace || !aligned16(x) || !aligned16(w) || !aligned16(workspace))
        return fail(SGPRS_ERR_INVALID_ARG, "pointers must be non-NULL and 16-byte aligned");
    return launch_avgpool_fc(dtype, n, hw, cin, cout, x, w, bias, logits, workspace, stream, cus, nullptr);
}

int sgprs_global_avgpool(int dtype, int n, int hw, int c, const void* x, float* pooled, sgprs_pool_t* pool, int partition)
{
    hipStream_t stream;
    int cus = 0, rc;
    if ((rc = resolve(pool, partition, &stream, &cus))) return rc;
    if (!dtype_ok(dtype)) return fail(SGPRS_ERR_UNSUPPORTED, "dtype %d", dtype);
    if (n <= 0 || hw <= 0) return fail(SGPRS_ERR_INVALID_ARG, "non-positive dimension");
    if (n > 65535 || (long long)n * hw * c >= (1ll << 31))
        return fail(SGPRS_ERR_UNSUPPORTED, "more than 65535 images or 2^31 input elements");
    if (c != 512 && c != 1024 && c != 2048) return fail(SGPRS_ERR_UNSUPPORTED, "c %d: supported are 512, 1024, 2048", c);
    if (!x || !pooled || !aligned16(x) || !aligned16(pooled) || (const void*)pooled == x)
        return fail(SGPRS_ERR_INVALID_ARG, "x and pooled must be distinct, non-NULL and 16-byte aligned");
    return launch_avgpool(dtype, n, hw, c, x, pooled, stream, nullptr);
}

int sgprs_avgpool_fc_static(int dtype, int n, int hw, int cin, int cout, const void* x, const void* w, const float* bias,
                            float* logits, sgprs_pool_t* pool, int partition)
{
    hipStream_t stream;
    int cus = 0, rc;
    if ((rc = resolve(pool, partition, &stream, &cus))) return rc;
    if (!dtype_ok(dtype)) return fail(SGPRS_ERR_UNSUPPORTED, "dtype %d", dtype);
    if (n <= 0 || hw <= 0 || cout <= 0) return fail(SGPRS_ERR_INVALID_ARG, "non-positive dimension");
    if (n > 65535 || cout > (1 << 20) || (long long)n * hw * cin >= (1ll << 31))
        return fail(SGPRS_ERR_UNSUPPORTED, "more than 65535 images, 2^20 outputs or 2^31 input elements");
    if (cin != 512 && cin != 1024 && cin != 2048)
        return fail(SGPRS_ERR_UNSUPPORTED, "cin %d: supported are 512, 1024, 2048", cin);
    if ((size_t)n * (size_t)cin > kStaticScratchFloats)
        return fail(SGPRS_ERR_UNSUPPORTED, "n * cin = %zu pooled values exceed the static scratch of %zu", (size_t)n * (size_t)cin,
                    kStaticScratchFloats);
    if (!x || !w || !logits || !aligned16(x) || !aligned16(w))
        return fail(SGPRS_ERR_INVALID_ARG, "pointers must be non-NULL and 16-byte aligned");
    float* ws = nullptr;
    if ((rc = static_scratch(pool->device, &ws))) return rc;
    return launch_avgpool_fc(dtype, n, hw, cin, cout, x, w, bias, logits, ws, stream, cus, nullptr);
}

}  // extern "C"
