// Task tau_i = one ResNet18 instance and its six stages tau_i^0..5 (paper,
// "Task Model" and "Simulation Results": ResNet18 on a 224x224 input, each
// task divided into six stages).  Creating the task is the offline phase
// (fold BN, round, pack, upload); sgprs_stage_run / sgprs_task_run only
// enqueue kernels on partition streams.
#include <algorithm>
#include <cstring>
#include <new>

#include "internal.h"

namespace {

// Replaying costs about 5 us of GPU time per launch and saves 50-90 us of host time: it pays when
// one host thread feeds several partitions with short inferences, not for one long batch.
constexpr int kReplayMaxBatch = 8;

using namespace sgprs;

// cin, cout, kernel, stride, pad, input height -- forward order
struct ConvSpec { int cin, cout, k, stride, pad, h; };
const ConvSpec kConvs[SGPRS_RESNET18_CONVS] = {
    {3, 64, 7, 2, 3, 224},
    {64, 64, 3, 1, 1, 56},   {64, 64, 3, 1, 1, 56},   {64, 64, 3, 1, 1, 56},   {64, 64, 3, 1, 1, 56},
    {64, 128, 3, 2, 1, 56},  {128, 128, 3, 1, 1, 28}, {64, 128, 1, 2, 0, 56},  {128, 128, 3, 1, 1, 28}, {128, 128, 3, 1, 1, 28},
    {128, 256, 3, 2, 1, 28}, {256, 256, 3, 1, 1, 14}, {128, 256, 1, 2, 0, 28}, {256, 256, 3, 1, 1, 14}, {256, 256, 3, 1, 1, 14},
    {256, 512, 3, 2, 1, 14}, {512, 512, 3, 1, 1, 7},  {256, 512, 1, 2, 0, 14}, {512, 512, 3, 1, 1, 7},  {512, 512, 3, 1, 1, 7},
};
// per-image C,H,W at each stage boundary: [j] = input of stage j, [j+1] = its output
const int kStageDims[7][3] = {{3, 224, 224}, {64, 56, 56}, {64, 56, 56}, {128, 28, 28},
                              {256, 14, 14}, {512, 7, 7},  {1000, 1, 1}};
constexpr int kFcIn = 512, kFcOut = 1000;

struct ConvLayer {
    sgprs_conv_desc_t d;
    void* w = nullptr;
    float* scale = nullptr;
    float* shift = nullptr;
};

}  // namespace

struct sgprs_task {
    int device = 0, dtype = 0, max_batch = 0;
    ConvLayer conv[SGPRS_RESNET18_CONVS];
    void* fc_w = nullptr;
    float* fc_b = nullptr;
    void* stem_w_rows = nullptr;  // bf16 only: the stem weights in the packed-row kernel's layout
    void* stem_out = nullptr;
    void* tmp[3] = {nullptr, nullptr, nullptr};
    void* stage_out[5] = {nullptr, nullptr, nullptr, nullptr, nullptr};
    float* pooled = nullptr;
    void* splitk = nullptr;
    size_t splitk_bytes = 0;
    std::vector<void*> allocs;
    sgprs::Profiler prof[SGPRS_RESNET18_STAGES];
    bool profiling = false;
    hipEvent_t chain[SGPRS_RESNET18_STAGES] = {};
    // Whole-task launches with the same arguments are captured into a HIP graph the second time
    // they are seen and replayed from then on (one host call instead of 20-33 kernel launches).
    struct Replay {
        int batch = 0, partition = 0;
        const void* in = nullptr;
        float* logits = nullptr;
        const sgprs_pool_t* pool = nullptr;
        hipStream_t stream = nullptr;
        int generation = 0;  // tuning-override generation the capture was made under
        int seen = 0;
        hipGraph_t graph = nullptr;
        hipGraphExec_t exec = nullptr;
    };
    std::vector<Replay> replays;
    int graph_mode = -1;     // -1: replay batches up to kReplayMaxBatch, 0: never, 1: always
    bool use_graphs = true;  // cleared when a capture fails
};

namespace {

int dev_alloc(sgprs_task* t, size_t bytes, void** out)
{
    void* p = nullptr;
    hipError_t e = hipMalloc(&p, bytes ? bytes : 16);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return fail(e == hipErrorOutOfMemory ? SGPRS_ERR_OOM : SGPRS_ERR_HIP, "hipMalloc(%zu): %s", bytes,
                    hipGetErrorString(e));
    }
    t->allocs.push_back(p);
    *out = p;
    return SGPRS_OK;
}

int upload(sgprs_task* t, const void* host, size_t bytes, void** out)
{
    int rc = dev_alloc(t, bytes, out);
    if (rc) return rc;
    SGPRS_HIP(hipMemcpy(*out, host, bytes, hipMemcpyHostToDevice));
    return SGPRS_OK;
}

void drop_replay(sgprs_task::Replay& r)
{
    if (r.exec) (void)hipGraphExecDestroy(r.exec);
    if (r.graph) (void)hipGraphDestroy(r.graph);
    r.exec = nullptr;
    r.graph = nullptr;
}

void destroy_task(sgprs_task* t)
{
    for (auto& r : t->replays) drop_replay(r);
    for (void* p : t->allocs) (void)hipFree(p);
    if (t->splitk) (void)hipFree(t->splitk);
    for (hipEvent_t e : t->chain)
        if (e) (void)hipEventDestroy(e);
    delete t;
}

size_t splitk_need(const sgprs_task* t, int first, int last, int batch, int cus)
{
    size_t need = 0;
    for (int i = first; i <= last; ++i) {
        if (is_stem(t->conv[i].d)) continue;
        sgprs_conv_desc_t d = t->conv[i].d;
        d.n = batch;
        need = std::max(need, std::max(conv_workspace_bytes(d, plan_conv(d, cus, false)), conv_workspace_bytes(d, plan_conv(d, cus, true))));
    }
    return need;
}

// Grows the split-K scratch if this (batch, partition size) needs more than
// any earlier run.  Growing waits for the stream and reallocates, so it only
// happens on the first run of a new shape.
int ensure_splitk(sgprs_task* t, size_t need, hipStream_t stream)
{
    if (need <= t->splitk_bytes) return SGPRS_OK;
    SGPRS_HIP(hipStreamSynchronize(stream));
    // captured graphs hold the old scratch pointer and go with it; they may have been launched on
    // other streams, so the whole device is drained first (this path runs once per new shape)
    if (!t->replays.empty()) {
        SGPRS_HIP(hipDeviceSynchronize());
        for (auto& r : t->replays) drop_replay(r);
        t->replays.clear();
    }
    if (t->splitk) SGPRS_HIP(hipFree(t->splitk));
    t->splitk = nullptr;
    t->splitk_bytes = 0;
    hipError_t e = hipMalloc(&t->splitk, need);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return fail(SGPRS_ERR_OOM, "hipMalloc(%zu) for split-K scratch: %s", need, hipGetErrorString(e));
    }
    t->splitk_bytes = need;
    return SGPRS_OK;
}

int run_conv(sgprs_task* t, int i, int batch, const void* x, const void* res, void* y, int relu, hipStream_t s,
             int cus, Profiler* prof)
{
    sgprs_conv_desc_t d = t->conv[i].d;
    d.n = batch;
    d.relu = relu;
    if (is_stem(d)) return launch_stem(d, x, t->conv[i].w, t->conv[i].scale, t->conv[i].shift, y, s, cus, prof);
    return launch_conv(d, x, t->conv[i].w, t->conv[i].scale, t->conv[i].shift, res, y, t->splitk, t->splitk_bytes, s,
                       cus, prof);
}

// BasicBlock: out = ReLU(BN2(conv2(ReLU(BN1(conv1(x))))) + shortcut(x)); the
// shortcut is x or BN(conv1x1/2(x)).  BN, the add and both ReLUs are fused
// into the convolutions' epilogues.
int run_block(sgprs_task* t, int c1, int c2, int down, int batch, const void* x, void* out, hipStream_t s, int cus,
              Profiler* prof)
{
    int rc;
    const void* shortcut = x;
    bool paired = false;
    if (down >= 0) {  // conv1 and the shortcut's 1x1 convolution read the same input: one launch when the plans allow
        sgprs_conv_desc_t d0 = t->conv[c1].d, d1 = t->conv[down].d;
        d0.n = d1.n = batch; d0.relu = 1; d1.relu = 0;
        int sv = 0;
        if (!d0.relu || d1.cout != d0.cout || !plan_s2patch(d0, cus, &sv)) sv = -1;
        if (sv >= 0) {
            if ((rc = launch_conv3x3s2_patch(d0, sv, x, t->conv[c1].w, t->conv[c1].scale, t->conv[c1].shift, t->tmp[0], &d1,
                                             t->conv[down].w, t->conv[down].scale, t->conv[down].shift, t->tmp[1], s, cus, prof)))
                return rc;
            paired = true;
        } else if ((rc = launch_conv_pair(d0, t->conv[c1].w, t->conv[c1].scale, t->conv[c1].shift, t->tmp[0], d1,
                                   t->conv[down].w, t->conv[down].scale, t->conv[down].shift, t->tmp[1], x, s, cus, prof,
                                   &paired)))
            return rc;
        shortcut = t->tmp[1];
    }
    if (!paired) {
        if ((rc = run_conv(t, c1, batch, x, nullptr, t->tmp[0], 1, s, cus, prof))) return rc;
        if (down >= 0 && (rc = run_conv(t, down, batch, x, nullptr, t->tmp[1], 0, s, cus, prof))) return rc;
    }
    return run_conv(t, c2, batch, t->tmp[0], shortcut, out, 1, s, cus, prof);
}

int run_stage(sgprs_task* t, int j, int batch, const void* in, void* out, hipStream_t s, int cus,
              hipEvent_t prev_stop = nullptr)
{
    Profiler* prof = &t->prof[j];
    prof->on = t->profiling;
    prof->reset(prev_stop);
    int rc;
    if (j == 0) {
        if (stem_pool_applicable(t->dtype, batch, 224, 224, cus))
            return launch_stem_pool(t->dtype, batch, 224, 224, in, t->conv[0].w, t->stem_w_rows, t->conv[0].scale, t->conv[0].shift, out, s,
                                    cus, prof);
        if ((rc = run_conv(t, 0, batch, in, nullptr, t->stem_out, 1, s, cus, prof))) return rc;
        return launch_maxpool(t->dtype, batch, 112, 112, 64, t->stem_out, out, s, cus, prof);
    }
    if (j == 5)
        return launch_avgpool_fc(t->dtype, batch, 49, kFcIn, kFcOut, in, t->fc_w, t->fc_b, (float*)out, t->pooled, s,
                                 cus, prof);
    const int first = j == 1 ? 1 : 5 + 5 * (j - 2);
    const int last = j == 1 ? 4 : first + 4;
    if ((rc = ensure_splitk(t, splitk_need(t, first, last, batch, cus), s))) return rc;
    if (j == 1) {
        if ((rc = run_block(t, 1, 2, -1, batch, in, t->tmp[2], s, cus, prof))) return rc;
        return run_block(t, 3, 4, -1, batch, t->tmp[2], out, s, cus, prof);
    }
    if ((rc = run_block(t, first, first + 1, first + 2, batch, in, t->tmp[2], s, cus, prof))) return rc;
    return run_block(t, first + 3, first + 4, -1, batch, t->tmp[2], out, s, cus, prof);
}

size_t stage_bytes(const sgprs_task* t, int boundary, int batch)
{
    const int* d = kStageDims[boundary];
    const size_t el = (size_t)batch * d[0] * d[1] * d[2];
    return el * (boundary == 6 ? sizeof(float) : dtype_size(t->dtype));
}

int check_task_call(const sgprs_task* t, int stage, int batch)
{
    if (!t) return fail(SGPRS_ERR_INVALID_ARG, "task is NULL");
    if (stage < 0 || stage >= SGPRS_RESNET18_STAGES)
        return fail(SGPRS_ERR_INVALID_ARG, "stage %d outside [0,%d)", stage, SGPRS_RESNET18_STAGES);
    if (batch <= 0 || batch > t->max_batch)
        return fail(SGPRS_ERR_INVALID_ARG, "batch %d outside [1,%d]", batch, t->max_batch);
    return SGPRS_OK;
}

}  // namespace

extern "C" {

int sgprs_task_create_resnet18(int device, int dtype, int max_batch, const sgprs_resnet18_params_t* hp,
                               sgprs_task_t** out)
{
    if (!out) return fail(SGPRS_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    if (!hp) return fail(SGPRS_ERR_INVALID_ARG, "host_params is NULL");
    if (!dtype_ok(dtype)) return fail(SGPRS_ERR_UNSUPPORTED, "dtype %d", dtype);
    if (max_batch <= 0 || max_batch > 512) return fail(SGPRS_ERR_INVALID_ARG, "max_batch %d outside [1,512]", max_batch);
    for (int i = 0; i < SGPRS_RESNET18_CONVS; ++i)
        if (!hp->conv_w[i] || !hp->bn_gamma[i] || !hp->bn_beta[i] || !hp->bn_mean[i] || !hp->bn_var[i])
            return fail(SGPRS_ERR_INVALID_ARG, "NULL parameter pointer for conv %d", i);
    if (!hp->fc_w) return fail(SGPRS_ERR_INVALID_ARG, "fc_w is NULL");
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev <= 0) {
        (void)hipGetLastError();
        return fail(SGPRS_ERR_NO_DEVICE, "no HIP device available");
    }
    if (device < 0 || device >= ndev) return fail(SGPRS_ERR_INVALID_ARG, "device %d outside [0,%d)", device, ndev);
    SGPRS_HIP(hipSetDevice(device));

    sgprs_task* t = new (std::nothrow) sgprs_task;
    if (!t) return fail(SGPRS_ERR_OOM, "out of host memory");
    t->device = device; t->dtype = dtype; t->max_batch = max_batch;
    int rc = SGPRS_OK;
    std::vector<unsigned char> packed;
    std::vector<float> scale, shift;
    for (int i = 0; i < SGPRS_RESNET18_CONVS && !rc; ++i) {
        const ConvSpec& cs = kConvs[i];
        sgprs_conv_desc_t& d = t->conv[i].d;
        d.n = max_batch; d.h = cs.h; d.w = cs.h; d.cin = cs.cin; d.cout = cs.cout; d.r = cs.k; d.s = cs.k;
        d.stride = cs.stride; d.pad = cs.pad; d.dtype = dtype; d.relu = 0;
        size_t bytes = 0;
        if ((rc = sgprs_conv_packed_weight_bytes(&d, &bytes))) break;
        packed.resize(bytes);
        if ((rc = sgprs_pack_conv_weights(&d, hp->conv_w[i], packed.data(), bytes))) break;
        scale.resize(cs.cout); shift.resize(cs.cout);
        if ((rc = sgprs_fold_bn(hp->bn_gamma[i], hp->bn_beta[i], hp->bn_mean[i], hp->bn_var[i], hp->bn_eps, cs.cout,
                                scale.data(), shift.data())))
            break;
        if ((rc = upload(t, packed.data(), bytes, &t->conv[i].w))) break;
        if ((rc = upload(t, scale.data(), cs.cout * sizeof(float), (void**)&t->conv[i].scale))) break;
        if ((rc = upload(t, shift.data(), cs.cout * sizeof(float), (void**)&t->conv[i].shift))) break;
        if (i == 0 && dtype == SGPRS_BF16) {
            std::vector<uint16_t> rows((size_t)64 * kStemRowsK);
            pack_stem_rows(hp->conv_w[0], rows.data());
            rc = upload(t, rows.data(), rows.size() * 2, &t->stem_w_rows);
        }
    }
    if (!rc) {
        const size_t n = (size_t)kFcOut * kFcIn;
        if (dtype == SGPRS_BF16) {
            std::vector<uint16_t> w16(n);
            for (size_t i = 0; i < n; ++i) w16[i] = f32_to_bf16_bits(hp->fc_w[i]);
            rc = upload(t, w16.data(), n * 2, &t->fc_w);
        } else {
            rc = upload(t, hp->fc_w, n * 4, &t->fc_w);
        }
    }
    if (!rc && hp->fc_b) rc = upload(t, hp->fc_b, kFcOut * sizeof(float), (void**)&t->fc_b);
    const size_t es = dtype_size(dtype);
    if (!rc) rc = dev_alloc(t, (size_t)max_batch * 112 * 112 * 64 * es, &t->stem_out);
    for (int i = 0; i < 3 && !rc; ++i) rc = dev_alloc(t, (size_t)max_batch * 56 * 56 * 64 * es, &t->tmp[i]);
    for (int j = 0; j < 5 && !rc; ++j) rc = dev_alloc(t, stage_bytes(t, j + 1, max_batch), &t->stage_out[j]);
    if (!rc) rc = dev_alloc(t, (size_t)max_batch * kFcIn * sizeof(float), (void**)&t->pooled);
    if (!rc) {
        int total = 0;
        if (hipDeviceGetAttribute(&total, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess) total = 256;
        size_t need = 0;
        for (int cus = 8; cus <= total; cus += 8)
            for (int b : {1, max_batch}) need = std::max(need, splitk_need(t, 1, SGPRS_RESNET18_CONVS - 1, b, cus));
        if (need) rc = ensure_splitk(t, need, nullptr);
    }
    for (int j = 0; j < SGPRS_RESNET18_STAGES && !rc; ++j)
        if (hipEventCreateWithFlags(&t->chain[j], hipEventDisableTiming) != hipSuccess)
            rc = fail(SGPRS_ERR_HIP, "hipEventCreate failed");
    if (rc) {
        destroy_task(t);
        return rc;
    }
    *out = t;
    return SGPRS_OK;
}

int sgprs_task_destroy(sgprs_task_t* t)
{
    if (!t) return fail(SGPRS_ERR_INVALID_ARG, "task is NULL");
    (void)hipDeviceSynchronize();
    destroy_task(t);
    return SGPRS_OK;
}

int sgprs_task_num_stages(const sgprs_task_t* t)
{
    if (!t) return fail(SGPRS_ERR_INVALID_ARG, "task is NULL");
    return SGPRS_RESNET18_STAGES;
}

int sgprs_task_stage_io(const sgprs_task_t* t, int stage, int batch, size_t* in_bytes, size_t* out_bytes,
                        int in_nchw[4], int out_nchw[4])
{
    int rc = check_task_call(t, stage, batch);
    if (rc) return rc;
    if (in_bytes) *in_bytes = stage_bytes(t, stage, batch);
    if (out_bytes) *out_bytes = stage_bytes(t, stage + 1, batch);
    if (in_nchw) { in_nchw[0] = batch; for (int i = 0; i < 3; ++i) in_nchw[1 + i] = kStageDims[stage][i]; }
    if (out_nchw) { out_nchw[0] = batch; for (int i = 0; i < 3; ++i) out_nchw[1 + i] = kStageDims[stage + 1][i]; }
    return SGPRS_OK;
}

int sgprs_stage_run(sgprs_task_t* t, int stage, int batch, const void* in, void* out, sgprs_pool_t* pool,
                    int partition)
{
    int rc = check_task_call(t, stage, batch);
    if (rc) return rc;
    hipStream_t s;
    int cus = 0;
    if ((rc = resolve(pool, partition, &s, &cus))) return rc;
    if (!in || !out || ((uintptr_t)in & 15) || ((uintptr_t)out & 15) || in == out)
        return fail(SGPRS_ERR_INVALID_ARG, "in and out must be distinct, non-NULL and 16-byte aligned");
    if (pool->device != t->device) return fail(SGPRS_ERR_INVALID_ARG, "pool and task live on different devices");
    return run_stage(t, stage, batch, in, out, s, cus);
}

int sgprs_task_run(sgprs_task_t* t, int batch, const void* in, float* logits, sgprs_pool_t* pool, int partition,
                   const int* pps)
{
    int rc = check_task_call(t, 0, batch);
    if (rc) return rc;
    if (!in || !logits || ((uintptr_t)in & 15) || ((uintptr_t)logits & 15))
        return fail(SGPRS_ERR_INVALID_ARG, "in and logits must be non-NULL and 16-byte aligned");
    hipStream_t s[SGPRS_RESNET18_STAGES];
    int cus[SGPRS_RESNET18_STAGES];
    for (int j = 0; j < SGPRS_RESNET18_STAGES; ++j)
        if ((rc = resolve(pool, pps ? pps[j] : partition, &s[j], &cus[j]))) return rc;
    if (pool->device != t->device) return fail(SGPRS_ERR_INVALID_ARG, "pool and task live on different devices");

    // ---- graph replay: one partition, no per-kernel timing ----
    bool one_stream = true;
    for (int j = 1; j < SGPRS_RESNET18_STAGES; ++j) one_stream = one_stream && s[j] == s[0];
    sgprs_task::Replay* rp = nullptr;
    if (t->use_graphs && one_stream && !t->profiling &&
        (t->graph_mode == 1 || (t->graph_mode < 0 && batch <= kReplayMaxBatch))) {
        // the split-K scratch must neither grow while capturing nor move under a captured graph
        for (int j = 1; j <= 4; ++j) {
            const int first = j == 1 ? 1 : 5 + 5 * (j - 2), last = j == 1 ? 4 : first + 4;
            if ((rc = ensure_splitk(t, splitk_need(t, first, last, batch, cus[j]), s[0]))) return rc;
        }
        for (auto& r : t->replays)
            if (r.batch == batch && r.in == in && r.logits == logits && r.pool == pool && r.stream == s[0] &&
                r.generation == g_plan_generation)
                rp = &r;
        if (!rp) {
            if (t->replays.size() >= 8) {  // a handful of argument sets per task; the oldest goes
                drop_replay(t->replays.front());
                t->replays.erase(t->replays.begin());
            }
            sgprs_task::Replay r;
            r.batch = batch; r.partition = partition; r.in = in; r.logits = logits; r.pool = pool; r.stream = s[0];
            r.generation = g_plan_generation;
            t->replays.push_back(r);
            rp = &t->replays.back();
        }
        if (rp->exec) {
            SGPRS_HIP(hipGraphLaunch(rp->exec, s[0]));
            return SGPRS_OK;
        }
        ++rp->seen;
    }
    // The second sighting of an argument set is captured (the first ran eagerly, so every one-time
    // set-up, allocation and attribute call is behind us); a failed capture switches replay off.
    const bool capture = rp && rp->seen == 2;
    if (capture) {
        if (hipStreamBeginCapture(s[0], hipStreamCaptureModeThreadLocal) != hipSuccess) {
            (void)hipGetLastError();
            t->use_graphs = false;
            rp = nullptr;
        }
    }
    const bool capturing = capture && rp;
    for (int j = 0; j < SGPRS_RESNET18_STAGES; ++j) {
        if (j > 0 && s[j] != s[j - 1]) {
            SGPRS_HIP(hipEventRecord(t->chain[j], s[j - 1]));
            SGPRS_HIP(hipStreamWaitEvent(s[j], t->chain[j], 0));
        }
        const void* src = j == 0 ? in : t->stage_out[j - 1];
        void* dst = j == 5 ? (void*)logits : t->stage_out[j];
        // profiling: a stage on the same stream as its predecessor times its first
        // kernel from the predecessor's last completion event
        hipEvent_t prev = nullptr;
        if (t->profiling && j > 0 && s[j] == s[j - 1] && !t->prof[j - 1].recs.empty()) prev = t->prof[j - 1].recs.back().stop;
        if ((rc = run_stage(t, j, batch, src, dst, s[j], cus[j], prev))) break;
    }
    if (capturing) {
        hipGraph_t g = nullptr;
        const hipError_t e = hipStreamEndCapture(s[0], &g);
        hipGraphExec_t x = nullptr;
        if (!rc && e == hipSuccess && g && hipGraphInstantiate(&x, g, nullptr, nullptr, 0) == hipSuccess) {
            rp->graph = g;
            rp->exec = x;
            SGPRS_HIP(hipGraphLaunch(x, s[0]));
            return SGPRS_OK;
        }
        (void)hipGetLastError();
        if (g) (void)hipGraphDestroy(g);
        t->use_graphs = false;  // nothing was executed while capturing: run this call eagerly
        if (rc) return rc;
        return sgprs_task_run(t, batch, in, logits, pool, partition, pps);
    }
    return rc;
}

const void* sgprs_task_stage_output(const sgprs_task_t* t, int stage)
{
    if (!t || stage < 0 || stage > 4) {
        fail(SGPRS_ERR_INVALID_ARG, "stage %d outside [0,4] or task NULL", stage);
        return nullptr;
    }
    return t->stage_out[stage];
}

int sgprs_task_set_graph_replay(sgprs_task_t* t, int on)
{
    if (!t) return fail(SGPRS_ERR_INVALID_ARG, "task is NULL");
    if (on < -1 || on > 1) return fail(SGPRS_ERR_INVALID_ARG, "mode %d outside [-1,1]", on);
    t->graph_mode = on;
    return SGPRS_OK;
}

int sgprs_task_set_profiling(sgprs_task_t* t, int on)
{
    if (!t) return fail(SGPRS_ERR_INVALID_ARG, "task is NULL");
    t->profiling = on != 0;
    return SGPRS_OK;
}

int sgprs_task_kernel_times(sgprs_task_t* t, int stage, int* count, int* kind, int* variant, float* ms,
                            double* flops, double* bytes)
{
    int rc = check_task_call(t, stage, 1);
    if (rc) return rc;
    if (!count) return fail(SGPRS_ERR_INVALID_ARG, "count is NULL");
    const auto& recs = t->prof[stage].recs;
    const int cap = *count;
    *count = (int)recs.size();
    if (cap < (int)recs.size()) return fail(SGPRS_ERR_INVALID_ARG, "room for %d records, %d needed", cap, *count);
    for (size_t i = 0; i < recs.size(); ++i) {
        float t_ms = 0.f;
        SGPRS_HIP(hipEventElapsedTime(&t_ms, recs[i].start, recs[i].stop));
        if (kind) kind[i] = recs[i].kind;
        if (variant) variant[i] = recs[i].variant;
        if (ms) ms[i] = t_ms;
        if (flops) flops[i] = recs[i].flops;
        if (bytes) bytes[i] = recs[i].bytes;
    }
    return SGPRS_OK;
}

const char* sgprs_kernel_name(int kind, int variant)
{
    switch (kind) {
        case kKindIgemm: return igemm_variant_name(variant);
        case kKindIgemmPair: return igemm_pair_variant_name(variant);
        case kKindPatch: return patch_variant_name(variant);
        case kKindS2Patch: return s2patch_variant_name(variant);
        case kKindRows: return "conv3x3_rows_kernel";
        case kKindStem: return "conv_stem_kernel";
        case kKindStemPool:
            return variant == 2 ? "stem_pool_packed_kernel" : variant == SGPRS_BF16 ? "stem_pool_kernel<1>" : "stem_pool_kernel<0>";
        case kKindReduce: return "splitk_reduce_kernel";
        case kKindMaxpool: return "maxpool3x3s2_kernel";
        case kKindAvgpool: return "avgpool_kernel";
        case kKindFc: return variant >= 4 ? "fc_mfma_kernel" : variant >= 2 ? "avgpool_fc_kernel" : "fc_kernel";
        case kKindBnRelu: return "bn_relu_kernel";
        case kKindAdd: return "add_relu_kernel";
        default: return "?";
    }
}

}  // extern "C"
