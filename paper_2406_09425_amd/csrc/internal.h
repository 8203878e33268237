// Internal declarations shared by the host and kernel translation units of
// libsgprs.  Nothing here is part of the ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <atomic>
#include <hip/hip_ext.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <string>
#include <cstring>
#include <utility>
#include <mutex>
#include <vector>

#include "sgprs.h"

namespace sgprs {

// ---- error reporting -------------------------------------------------------
int fail(int status, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

#define SGPRS_HIP(call)                                                                   \
    do {                                                                                  \
        hipError_t e_ = (call);                                                           \
        if (e_ != hipSuccess)                                                             \
            return ::sgprs::fail(SGPRS_ERR_HIP, "%s failed: %s (%s:%d)", #call,           \
                                 hipGetErrorString(e_), __FILE__, __LINE__);              \
    } while (0)

// CU-masked streams that may be busy at once without the throughput of all of them collapsing
// (measured on MI355X: eight batch-1 tasks reach 20 k images/s over 4 busy partitions of a pool of 8,
// 8-9 k over 5, 6 or 8, whatever the partition size; idle partitions cost nothing).
constexpr int kMaxBusyQueues = 4;

// ---- pool ------------------------------------------------------------------
struct Partition {
    hipStream_t stream = nullptr;
    std::vector<uint32_t> mask;
    int cus = 0;
};

}  // namespace sgprs

struct sgprs_pool {
    int device = 0;
    int total_cus = 0;
    int n_xcd = 1;
    int cus_per_partition = 0;  // 0 when created from explicit masks of mixed size
    std::vector<sgprs::Partition> parts;
};

namespace sgprs {

// validates pool/partition, returns the stream and CU count
int resolve(sgprs_pool_t* pool, int partition, hipStream_t* stream, int* cus);

inline size_t dtype_size(int dtype) { return dtype == SGPRS_BF16 ? 2 : 4; }
inline bool dtype_ok(int dtype) { return dtype == SGPRS_F32 || dtype == SGPRS_BF16; }

// Device side: two fp32 values to one dword of bf16 (round to nearest even, a single packed
// conversion), then the optional ReLU on the packed pair as a signed 16-bit maximum against
// `floor16x2`: 0 for a ReLU (negative values and -0 carry the sign bit, read as negative integers
// and become +0; rounding keeps the sign, so this equals clamping before the conversion),
// 0x80008000 for none (the smallest 16-bit integer twice: every pattern passes unchanged).
__device__ __forceinline__ unsigned pack_bf16x2_relu(float lo, float hi, unsigned floor16x2)
{
    typedef float pk_f32x2 __attribute__((ext_vector_type(2)));
    typedef __bf16 pk_bf16x2 __attribute__((ext_vector_type(2)));
    typedef short pk_s16x2 __attribute__((ext_vector_type(2)));
    const pk_f32x2 f = {lo, hi};
    const pk_s16x2 b = __builtin_bit_cast(pk_s16x2, __builtin_convertvector(f, pk_bf16x2));
    return __builtin_bit_cast(unsigned, __builtin_elementwise_max(b, __builtin_bit_cast(pk_s16x2, floor16x2)));
}
constexpr unsigned kReluFloor = 0u, kNoReluFloor = 0x80008000u;

// host bf16 conversion, round to nearest even
inline uint16_t f32_to_bf16_bits(float f)
{
    uint32_t u;
    __builtin_memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);  // quiet NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
inline float bf16_bits_to_f32(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    __builtin_memcpy(&f, &u, 4);
    return f;
}

// ---- convolution -----------------------------------------------------------
// Stem layout constants: 7 tap rows, each 7 taps x 4 channel slots (3 real
// channels + 1 zero) = 28 elements padded to 32.
constexpr int kStemTapRow = 32;
constexpr int kStemK = 7 * kStemTapRow;  // 224

inline bool is_stem(const sgprs_conv_desc_t& d)
{
    return d.cin == 3 && d.r == 7 && d.s == 7 && d.stride == 2 && d.pad == 3;
}
inline bool is_igemm(const sgprs_conv_desc_t& d)
{
    return d.cin % 32 == 0 && d.r == d.s && (d.r == 1 || d.r == 3) && (d.stride == 1 || d.stride == 2);
}
int check_conv_desc(const sgprs_conv_desc_t* d);
inline int out_dim(int in, int k, int stride, int pad) { return (in + 2 * pad - k) / stride + 1; }

// Small memo for launch planning: the same few shapes are planned again on every launch, and the
// geometry searches behind a plan walk all row tiles.  Keys are plain structs compared bytewise
// (fill them with memset first); the oldest entries are dropped.
template <class K, class V, int CAP = 128> struct PlanMemo {
    std::vector<std::pair<K, V>> items;
    const V* find(const K& k)
    {
        for (size_t i = 0; i < items.size(); ++i)
            if (!memcmp(&items[i].first, &k, sizeof(K))) {
                if (i >= 8) {  // entries in use drift to the front
                    std::swap(items[i], items[i / 2]);
                    i /= 2;
                }
                return &items[i].second;
            }
        return nullptr;
    }
    void put(const K& k, const V& v)
    {
        if ((int)items.size() >= CAP) items.erase(items.begin(), items.begin() + CAP / 2);
        items.emplace_back(k, v);
    }
};
// Two levels: a memo per thread, read without a lock, in front of one per process behind a mutex,
// so that a thread that has never planned (a launcher thread just created) copies what another
// thread worked out instead of searching again.
template <class K, class V, int CAP = 128> struct SharedPlanMemo {
    std::mutex mu;
    PlanMemo<K, V, CAP> shared;
    template <class F> V get(PlanMemo<K, V, CAP>& local, const K& k, F compute)
    {
        if (const V* hit = local.find(k)) return *hit;
        V v;
        {
            std::lock_guard<std::mutex> guard(mu);
            if (const V* hit = shared.find(k)) v = *hit;
            else {
                v = compute();
                shared.put(k, v);
            }
        }
        local.put(k, v);
        return v;
    }
};
extern std::atomic<int> g_plan_generation;  // bumped whenever a tuning override changes what the planners return

// Tile configuration of one implicit-GEMM launch.
struct ConvPlan {
    int kind = 0;      // 0: implicit GEMM, 1: LDS-patch 3x3 kernel, 2: its stride-2 variant, 3: row streaming
    int variant = 0;   // index into the kernel's tile table (row streaming: output rows per stream and job)
    int bm = 0, bn = 0;
    int splits = 1;    // split-K factor (grid.z)
    int ktiles = 0;    // total k-tiles of 128 bytes
    int grid_m = 0, grid_n = 0;
};
// Chooses tile shape and split-K factor from the GEMM shape and the CU count of
// the partition the launch will run on.
// (has_residual: kernels without a residual input are left out).
ConvPlan plan_conv(const sgprs_conv_desc_t& d, int partition_cus, bool has_residual = false);
size_t conv_workspace_bytes(const sgprs_conv_desc_t& d, const ConvPlan& p);

struct KernelRecord {
    int kind = 0, variant = 0;
    double flops = 0, bytes = 0;
    hipEvent_t start = nullptr, stop = nullptr;
};
// Optional per-launch timing hook.  begin() appends a record and publishes its
// stop event in tl_stop; the next kernel launch (SGPRS_LAUNCH) attaches it to
// its own dispatch, so it carries the kernel's completion time.  A record's
// start is the stop event of the kernel queued just before it on the same
// stream (kernels of a run are queued back to back), or a plain event when
// there is none: separately recorded event packets would add microseconds of
// their own latency to every interval.
extern thread_local hipEvent_t tl_start, tl_stop;
// (Plain launches when no timing is attached: those are what stream capture records.)
#define SGPRS_LAUNCH(kernel, grid, block, lds, stream, ...)                                                             \
    do {                                                                                                                \
        if (::sgprs::tl_start || ::sgprs::tl_stop)                                                                      \
            hipExtLaunchKernelGGL(kernel, grid, block, lds, stream, ::sgprs::tl_start, ::sgprs::tl_stop, 0, __VA_ARGS__); \
        else                                                                                                            \
            hipLaunchKernelGGL(kernel, grid, block, lds, stream, __VA_ARGS__);                                          \
    } while (0)
struct Profiler {
    bool on = false;
    std::vector<KernelRecord> recs;      // records of the stage being run
    std::vector<hipEvent_t> event_pool;  // reused events
    size_t next_event = 0;
    hipEvent_t prev = nullptr;           // completion event of the previous kernel on this stream
    int begin(hipStream_t s, int kind, int variant, double flops, double bytes);
    int end(hipStream_t s);
    void reset(hipEvent_t prev_stop = nullptr) { recs.clear(); next_event = 0; prev = prev_stop; }
    ~Profiler();
};

enum KernelKind { kKindIgemm = 0, kKindStem = 1, kKindReduce = 2, kKindMaxpool = 3, kKindAvgpool = 4,
                  kKindFc = 5, kKindBnRelu = 6, kKindAdd = 7, kKindPatch = 8, kKindStemPool = 9,
                  kKindIgemmPair = 10, kKindS2Patch = 11, kKindRows = 12 };

// launchers (device pointers; validated by callers)
int launch_conv(const sgprs_conv_desc_t& d, const void* x, const void* w, const float* scale,
                const float* shift, const void* residual, void* y, void* ws, size_t ws_bytes,
                hipStream_t stream, int cus, Profiler* prof);
int launch_stem(const sgprs_conv_desc_t& d, const void* x, const void* w, const float* scale,
                const float* shift, void* y, hipStream_t stream, int cus, Profiler* prof);
int launch_maxpool(int dtype, int n, int h, int w, int c, const void* x, void* y, hipStream_t stream,
                   int cus, Profiler* prof);
int launch_bn_relu(int dtype, size_t pixels, int c, const void* x, const float* scale,
                   const float* shift, void* y, hipStream_t stream, int cus, Profiler* prof);
int launch_add_relu(int dtype, size_t count, const void* a, const void* b, void* y, int relu,
                    hipStream_t stream, int cus, Profiler* prof);
int launch_avgpool(int dtype, int n, int hw, int cin, const void* x, float* pooled, hipStream_t stream, Profiler* prof);
int launch_avgpool_fc(int dtype, int n, int hw, int cin, int cout, const void* x, const void* w,
                      const float* bias, float* logits, float* ws, hipStream_t stream, int cus,
                      Profiler* prof);
// Device address of this GPU's static pooled-vector scratch (kStaticScratchFloats fp32), looked up
// on first use; nothing is allocated.
constexpr size_t kStaticScratchFloats = 64 * 2048;
constexpr int kMaxStaticScratchDevices = 16;
int static_scratch(int device, float** out);
int launch_probe(int n_blocks, int spin_cycles, uint32_t* out, hipStream_t stream);
int launch_mfma_probe(int cus, int steps, int random_data, unsigned long long* out, hipStream_t stream);
int launch_load_probe(int cus, const void* buf, size_t buf_bytes, unsigned region, int iters, unsigned* out, hipStream_t stream);
// stage 0 fused: conv7x7/2 + BN + ReLU + max-pool 3x3/2
bool stem_pool_applicable(int dtype, int n, int h, int w, int cus);
// wts: the stem layout of sgprs_pack_conv_weights; wts_rows: the bf16 [64][176] tap-row layout of
// pack_stem_rows (may be NULL: then the kernel that reads wts runs)
constexpr int kStemRowsK = 176;
void pack_stem_rows(const float* oihw, uint16_t* out);
void stem_pool_force(int v);  // -1 automatic, 1: never the packed-row kernel
int launch_stem_pool(int dtype, int n, int h, int w, const void* x, const void* wts, const void* wts_rows,
                     const float* scale, const float* shift, void* y, hipStream_t stream, int cus, Profiler* prof);

// LDS-patch 3x3 kernel (bf16, stride 1)
bool plan_patch(const sgprs_conv_desc_t& d, int cus, int* variant, int* splits);
void patch_force(int variant, int splits);
const char* patch_variant_name(int variant);
int launch_conv3x3_patch(const sgprs_conv_desc_t& d, int variant, int splits, const void* x, const void* w,
                         const float* scale, const float* shift, const void* residual, void* y, void* ws,
                         size_t ws_bytes, hipStream_t stream, int cus, Profiler* prof);
int launch_splitk_reduce(int dtype, const float* partial, int splits, size_t total, int cout, const float* scale,
                         const float* shift, const void* res, void* y, int relu, hipStream_t stream);
// LDS-patch 3x3 stride-2 kernel (bf16), alone or together with the block's 1x1 stride-2 shortcut
bool plan_s2patch(const sgprs_conv_desc_t& d, int cus, int* variant);
void s2patch_force(int v);
int s2patch_num_variants();
const char* s2patch_variant_name(int variant);
int launch_conv3x3s2_patch(const sgprs_conv_desc_t& d, int variant, const void* x, const void* w, const float* scale,
                           const float* shift, void* y, const sgprs_conv_desc_t* d2, const void* w2, const float* scale2,
                           const float* shift2, void* y2, hipStream_t stream, int cus, Profiler* prof);
// row-streaming 3x3 kernel (bf16, 64 -> 64 channels, 56-pixel rows)
bool plan_rows(const sgprs_conv_desc_t& d, int cus, int* rows_per_stream);
void rows_force_off(bool off);
int launch_conv3x3_rows(const sgprs_conv_desc_t& d, int rows_per_stream, const void* x, const void* w, const float* scale,
                        const float* shift, const void* residual, void* y, hipStream_t stream, int cus, Profiler* prof);
// tuning override: kind -1 automatic, 0 implicit GEMM only, 1 force patch (variant, splits)
extern std::atomic<int> g_conv_force_kind;
extern std::atomic<int> g_igemm_force_variant, g_igemm_force_splits;

const char* igemm_variant_name(int v);
const char* igemm_pair_variant_name(int v);
int launch_conv_pair(const sgprs_conv_desc_t& d0, const void* w0, const float* scale0, const float* shift0, void* y0,
                     const sgprs_conv_desc_t& d1, const void* w1, const float* scale1, const float* shift1, void* y1,
                     const void* x, hipStream_t stream, int cus, Profiler* prof, bool* done);
int igemm_num_variants();

}  // namespace sgprs
