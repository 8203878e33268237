// Context pool: n_p partitions realised as CU-masked HIP streams, plus the
// library's status/error plumbing.  (Paper, "Task Model": context pool CP with
// n_p contexts of a fixed number of compute units each; "Simulation Results":
// over-subscribed pools.)
#include <cstring>
#include <new>

#include "internal.h"

namespace sgprs {

static thread_local char g_err[512] = "";

int fail(int status, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return status;
}

int resolve(sgprs_pool_t* pool, int partition, hipStream_t* stream, int* cus)
{
    if (!pool) return fail(SGPRS_ERR_INVALID_ARG, "pool is NULL");
    if (partition < 0 || partition >= (int)pool->parts.size())
        return fail(SGPRS_ERR_INVALID_ARG, "partition %d outside [0,%d)", partition,
                    (int)pool->parts.size());
    *stream = pool->parts[partition].stream;
    *cus = pool->parts[partition].cus;
    return SGPRS_OK;
}

static int popcount_mask(const std::vector<uint32_t>& m)
{
    int c = 0;
    for (uint32_t w : m) c += __builtin_popcount(w);
    return c;
}

// Number of accelerator dies: MI300/MI350-class parts expose 8 dies of
// total/8 CUs behind one device; anything that does not divide evenly is
// treated as a single die.
static int guess_xcds(int total_cus)
{
    return (total_cus >= 64 && total_cus % 8 == 0) ? 8 : 1;
}

static int device_cus(int device, int* total)
{
    int n = 0;
    hipError_t e = hipGetDeviceCount(&n);
    if (e != hipSuccess || n <= 0) {
        (void)hipGetLastError();
        return fail(SGPRS_ERR_NO_DEVICE, "no HIP device available (%s)",
                    e == hipSuccess ? "count is 0" : hipGetErrorString(e));
    }
    if (device < 0 || device >= n)
        return fail(SGPRS_ERR_INVALID_ARG, "device %d outside [0,%d)", device, n);
    SGPRS_HIP(hipDeviceGetAttribute(total, hipDeviceAttributeMultiprocessorCount, device));
    return SGPRS_OK;
}

static int make_pool(int device, int total, const std::vector<std::vector<uint32_t>>& masks,
                     int cus_per_partition, sgprs_pool_t** out)
{
    sgprs_pool* p = new (std::nothrow) sgprs_pool;
    if (!p) return fail(SGPRS_ERR_OOM, "out of host memory");
    p->device = device;
    p->total_cus = total;
    p->n_xcd = guess_xcds(total);
    p->cus_per_partition = cus_per_partition;
    int prev = 0;
    (void)hipGetDevice(&prev);
    hipError_t e = hipSetDevice(device);
    for (size_t i = 0; e == hipSuccess && i < masks.size(); ++i) {
        Partition part;
        part.mask = masks[i];
        part.cus = popcount_mask(part.mask);
        e = hipExtStreamCreateWithCUMask(&part.stream, (uint32_t)part.mask.size(), part.mask.data());
        if (e == hipSuccess) p->parts.push_back(part);
    }
    (void)hipSetDevice(prev);
    if (e != hipSuccess) {
        for (auto& q : p->parts) (void)hipStreamDestroy(q.stream);
        delete p;
        return fail(SGPRS_ERR_HIP, "creating a CU-masked stream failed: %s", hipGetErrorString(e));
    }
    *out = p;
    return SGPRS_OK;
}

}  // namespace sgprs

using namespace sgprs;

extern "C" {

const char* sgprs_status_string(int s)
{
    switch (s) {
        case SGPRS_OK: return "ok";
        case SGPRS_ERR_INVALID_ARG: return "invalid argument";
        case SGPRS_ERR_NO_DEVICE: return "no device";
        case SGPRS_ERR_HIP: return "HIP runtime error";
        case SGPRS_ERR_OOM: return "out of memory";
        case SGPRS_ERR_UNSUPPORTED: return "unsupported shape or dtype";
        case SGPRS_ERR_OVERSUBSCRIBED: return "pool larger than the device";
        default: return "unknown status";
    }
}

const char* sgprs_last_error(void) { return g_err; }

int sgprs_version(void) { return 100; }

int sgprs_build_cu_mask(int total_cus, int n_xcd, int cus, int partition, int blocked_layout,
                        uint32_t* words, int n_words)
{
    if (!words) return fail(SGPRS_ERR_INVALID_ARG, "words is NULL");
    if (total_cus <= 0 || n_xcd <= 0 || total_cus % n_xcd)
        return fail(SGPRS_ERR_INVALID_ARG, "total_cus %d not a multiple of n_xcd %d", total_cus, n_xcd);
    if (cus < n_xcd || cus > total_cus || cus % n_xcd)
        return fail(SGPRS_ERR_INVALID_ARG, "cus %d must be a multiple of %d in [%d,%d]", cus, n_xcd,
                    n_xcd, total_cus);
    if (partition < 0) return fail(SGPRS_ERR_INVALID_ARG, "partition %d < 0", partition);
    if (n_words < (total_cus + 31) / 32 || n_words > SGPRS_MAX_MASK_WORDS)
        return fail(SGPRS_ERR_INVALID_ARG, "n_words %d does not fit %d CUs", n_words, total_cus);
    const int per_xcd = total_cus / n_xcd, take = cus / n_xcd;
    memset(words, 0, sizeof(uint32_t) * n_words);
    for (int x = 0; x < n_xcd; ++x)
        for (int j = 0; j < take; ++j) {
            const int slot = (int)(((long long)partition * take + j) % per_xcd);
            const int bit = blocked_layout ? x * per_xcd + slot : slot * n_xcd + x;
            words[bit >> 5] |= 1u << (bit & 31);
        }
    return SGPRS_OK;
}

int sgprs_pool_create(int device, int n_p, int cus, unsigned flags, sgprs_pool_t** out)
{
    if (!out) return fail(SGPRS_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    if (n_p <= 0 || n_p > 1024) return fail(SGPRS_ERR_INVALID_ARG, "n_p %d outside [1,1024]", n_p);
    if (flags & ~(SGPRS_POOL_OVERSUBSCRIBE | SGPRS_POOL_BLOCKED_LAYOUT))
        return fail(SGPRS_ERR_INVALID_ARG, "unknown flags 0x%x", flags);
    int total = 0;
    int rc = device_cus(device, &total);
    if (rc) return rc;
    const int n_xcd = guess_xcds(total);
    if (cus <= 0 || cus > total || cus % n_xcd)
        return fail(SGPRS_ERR_INVALID_ARG, "cus_per_partition %d must be a multiple of %d in [%d,%d]",
                    cus, n_xcd, n_xcd, total);
    if ((long long)n_p * cus > total && !(flags & SGPRS_POOL_OVERSUBSCRIBE))
        return fail(SGPRS_ERR_OVERSUBSCRIBED, "%d partitions x %d CUs > %d CUs; pass SGPRS_POOL_OVERSUBSCRIBE",
                    n_p, cus, total);
    const int n_words = (total + 31) / 32;
    std::vector<std::vector<uint32_t>> masks(n_p, std::vector<uint32_t>(n_words));
    for (int p = 0; p < n_p; ++p) {
        rc = sgprs_build_cu_mask(total, n_xcd, cus, p, (flags & SGPRS_POOL_BLOCKED_LAYOUT) ? 1 : 0,
                                 masks[p].data(), n_words);
        if (rc) return rc;
    }
    return make_pool(device, total, masks, cus, out);
}

int sgprs_pool_create_masks(int device, int n_p, const uint32_t* masks, int words_per_mask,
                            sgprs_pool_t** out)
{
    if (!out) return fail(SGPRS_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    if (!masks) return fail(SGPRS_ERR_INVALID_ARG, "masks is NULL");
    if (n_p <= 0 || n_p > 1024) return fail(SGPRS_ERR_INVALID_ARG, "n_p %d outside [1,1024]", n_p);
    if (words_per_mask <= 0 || words_per_mask > SGPRS_MAX_MASK_WORDS)
        return fail(SGPRS_ERR_INVALID_ARG, "words_per_mask %d outside [1,%d]", words_per_mask,
                    SGPRS_MAX_MASK_WORDS);
    int total = 0;
    int rc = device_cus(device, &total);
    if (rc) return rc;
    const int n_words = (total + 31) / 32;
    std::vector<std::vector<uint32_t>> m(n_p, std::vector<uint32_t>(n_words, 0u));
    for (int p = 0; p < n_p; ++p) {
        for (int i = 0; i < words_per_mask; ++i) {
            uint32_t w = masks[(size_t)p * words_per_mask + i];
            if (i >= n_words) continue;  // bits beyond the device are ignored
            if (i == n_words - 1 && total % 32) w &= (1u << (total % 32)) - 1u;
            m[p][i] = w;
        }
        if (popcount_mask(m[p]) == 0)
            return fail(SGPRS_ERR_INVALID_ARG, "mask of partition %d selects no CU", p);
        // The hardware hands the workgroups of a launch to the dies in turn, and mask bit i selects a
        // CU of die i % n_xcd: a stream whose mask leaves a die without CUs cannot run there (the
        // driver refuses to create it), so it is rejected here with a message that says why.
        const int n_xcd = guess_xcds(total);
        for (int x = 0; x < n_xcd; ++x) {
            bool any = false;
            for (int bit = x; bit < total && !any; bit += n_xcd) any = (m[p][bit >> 5] >> (bit & 31)) & 1u;
            if (!any)
                return fail(SGPRS_ERR_INVALID_ARG, "mask of partition %d selects no CU on die %d (bits %d, %d, ...): every one of the %d dies needs one",
                            p, x, x, x + n_xcd, n_xcd);
        }
    }
    return make_pool(device, total, m, 0, out);
}

int sgprs_pool_destroy(sgprs_pool_t* pool)
{
    if (!pool) return fail(SGPRS_ERR_INVALID_ARG, "pool is NULL");
    int rc = SGPRS_OK;
    for (auto& p : pool->parts) {
        if (hipStreamSynchronize(p.stream) != hipSuccess) rc = SGPRS_ERR_HIP;
        if (hipStreamDestroy(p.stream) != hipSuccess) rc = SGPRS_ERR_HIP;
    }
    delete pool;
    return rc ? fail(rc, "destroying a partition stream failed") : SGPRS_OK;
}

int sgprs_pool_info(const sgprs_pool_t* pool, int* n_p, int* cus, int* total, int* n_xcd)
{
    if (!pool) return fail(SGPRS_ERR_INVALID_ARG, "pool is NULL");
    if (n_p) *n_p = (int)pool->parts.size();
    if (cus) *cus = pool->cus_per_partition;
    if (total) *total = pool->total_cus;
    if (n_xcd) *n_xcd = pool->n_xcd;
    return SGPRS_OK;
}

int sgprs_pool_partition_cus(const sgprs_pool_t* pool, int partition, int* cus)
{
    hipStream_t s;
    int c = 0;
    int rc = resolve(const_cast<sgprs_pool_t*>(pool), partition, &s, &c);
    if (rc) return rc;
    if (!cus) return fail(SGPRS_ERR_INVALID_ARG, "cus is NULL");
    *cus = c;
    return SGPRS_OK;
}

int sgprs_pool_get_mask(const sgprs_pool_t* pool, int partition, uint32_t* words, int n_words)
{
    hipStream_t s;
    int c = 0;
    int rc = resolve(const_cast<sgprs_pool_t*>(pool), partition, &s, &c);
    if (rc) return rc;
    const auto& m = pool->parts[partition].mask;
    if (!words || n_words < (int)m.size())
        return fail(SGPRS_ERR_INVALID_ARG, "need room for %d mask words", (int)m.size());
    memset(words, 0, sizeof(uint32_t) * n_words);
    memcpy(words, m.data(), sizeof(uint32_t) * m.size());
    return SGPRS_OK;
}

void* sgprs_pool_stream(const sgprs_pool_t* pool, int partition)
{
    hipStream_t s = nullptr;
    int c = 0;
    if (resolve(const_cast<sgprs_pool_t*>(pool), partition, &s, &c)) return nullptr;
    return (void*)s;
}

int sgprs_partition_sync(sgprs_pool_t* pool, int partition)
{
    hipStream_t s;
    int c = 0;
    int rc = resolve(pool, partition, &s, &c);
    if (rc) return rc;
    SGPRS_HIP(hipStreamSynchronize(s));
    return SGPRS_OK;
}

int sgprs_pool_sync(sgprs_pool_t* pool)
{
    if (!pool) return fail(SGPRS_ERR_INVALID_ARG, "pool is NULL");
    for (auto& p : pool->parts) SGPRS_HIP(hipStreamSynchronize(p.stream));
    return SGPRS_OK;
}

int sgprs_partition_probe(sgprs_pool_t* pool, int partition, int n_blocks, int spin_cycles,
                          uint32_t* out)
{
    hipStream_t s;
    int c = 0;
    int rc = resolve(pool, partition, &s, &c);
    if (rc) return rc;
    if (!out) return fail(SGPRS_ERR_INVALID_ARG, "out is NULL");
    if (n_blocks <= 0 || n_blocks > 65536)
        return fail(SGPRS_ERR_INVALID_ARG, "n_blocks %d outside [1,65536]", n_blocks);
    if (spin_cycles < 0 || spin_cycles > 10000000)
        return fail(SGPRS_ERR_INVALID_ARG, "spin_cycles %d outside [0,1e7]", spin_cycles);
    return launch_probe(n_blocks, spin_cycles, out, s);
}

int sgprs_partition_probe_graph(sgprs_pool_t* pool, int partition, int n_blocks, int spin_cycles, uint32_t* out)
{
    hipStream_t s;
    int c = 0;
    int rc = resolve(pool, partition, &s, &c);
    if (rc) return rc;
    if (!out) return fail(SGPRS_ERR_INVALID_ARG, "out is NULL");
    if (n_blocks <= 0 || n_blocks > 65536)
        return fail(SGPRS_ERR_INVALID_ARG, "n_blocks %d outside [1,65536]", n_blocks);
    if (spin_cycles < 0 || spin_cycles > 10000000)
        return fail(SGPRS_ERR_INVALID_ARG, "spin_cycles %d outside [0,1e7]", spin_cycles);
    SGPRS_HIP(hipStreamBeginCapture(s, hipStreamCaptureModeThreadLocal));
    rc = launch_probe(n_blocks, spin_cycles, out, s);
    hipGraph_t g = nullptr;
    const hipError_t e = hipStreamEndCapture(s, &g);
    if (rc || e != hipSuccess || !g) {
        (void)hipGetLastError();
        if (g) (void)hipGraphDestroy(g);
        return rc ? rc : fail(SGPRS_ERR_HIP, "stream capture failed: %s", hipGetErrorString(e));
    }
    hipGraphExec_t x = nullptr;
    hipError_t e2 = hipGraphInstantiate(&x, g, nullptr, nullptr, 0);
    if (e2 == hipSuccess) e2 = hipGraphLaunch(x, s);
    if (e2 == hipSuccess) e2 = hipStreamSynchronize(s);
    if (x) (void)hipGraphExecDestroy(x);
    (void)hipGraphDestroy(g);
    if (e2 != hipSuccess) return fail(SGPRS_ERR_HIP, "graph launch failed: %s", hipGetErrorString(e2));
    return SGPRS_OK;
}

int sgprs_mfma_probe(sgprs_pool_t* pool, int partition, int random_data, int steps, uint64_t* out)
{
    hipStream_t s;
    int c = 0;
    int rc = resolve(pool, partition, &s, &c);
    if (rc) return rc;
    if (!out) return fail(SGPRS_ERR_INVALID_ARG, "out is NULL");
    if (steps <= 0 || steps > 1000000) return fail(SGPRS_ERR_INVALID_ARG, "steps %d outside [1,1e6]", steps);
    return launch_mfma_probe(c, steps, random_data != 0, (unsigned long long*)out, s);
}

int sgprs_load_probe(sgprs_pool_t* pool, int partition, const void* buf, size_t buf_bytes, size_t region_bytes, int iters,
                     uint32_t* out)
{
    hipStream_t s;
    int c = 0;
    int rc = resolve(pool, partition, &s, &c);
    if (rc) return rc;
    if (!buf || !out || ((uintptr_t)buf & 15)) return fail(SGPRS_ERR_INVALID_ARG, "buf must be 16-byte aligned, buf and out non-NULL");
    if (region_bytes < (16u << 10) || region_bytes > (1u << 30) || (region_bytes & (region_bytes - 1)))
        return fail(SGPRS_ERR_INVALID_ARG, "region_bytes %zu is not a power of two in [16 KiB, 1 GiB]", region_bytes);
    if (buf_bytes < region_bytes || buf_bytes % region_bytes)
        return fail(SGPRS_ERR_INVALID_ARG, "buf_bytes %zu is not a positive multiple of region_bytes %zu", buf_bytes, region_bytes);
    if (iters <= 0 || iters > 1000000) return fail(SGPRS_ERR_INVALID_ARG, "iters %d outside [1,1e6]", iters);
    return launch_load_probe(c, buf, buf_bytes, (unsigned)region_bytes, iters, out, s);
}

}  // extern "C"
