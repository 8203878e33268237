// 3x3 stride-1 pad-1 convolution, bf16, 64 -> 64 channels on 56-pixel rows: row streaming with
// the weights stationary in registers.
//
// The LDS-patch kernel stages a tile's input patch and streams or keeps the weights in LDS; every
// MFMA then needs two LDS fragment reads.  For the 64 -> 64 layers the whole filter of 16 output
// channels is 72 VGPRs, so here a wavefront keeps its filter slice in registers for the whole
// launch and only the pixels come from LDS:
//
//  * one workgroup of 8 wavefronts per CU; a job is S output rows of two row streams of one image
//    (rows r0 .. r0+S-1 and r0+S .. r0+2S-1), handled as one "virtual row" of 2 x 56 = 112 pixels
//    = 7 MFMA column tiles of 16 pixels; wavefront w owns output channels 16*(w%4) .. +15 and
//    tiles 0-3 (w < 4) or 4-6 (w >= 4), so the two wavefronts of a SIMD split the row 4 : 3;
//  * MFMA 16x16x32 with A = weights (row = output channel) and B = pixels; a step t reads input
//    row t-1 of both streams from a four-slot LDS ring and feeds three accumulator sets: output
//    rows t (filter row 0), t-1 (filter row 1) and t-2 (filter row 2).  The accumulators keep their
//    roles: a row moves from one set to the next by being the addend of the first MFMA of the next
//    role, so one loop body serves every step;
//  * input rows, the residual and the output rows move as whole 16-byte units, 1 KiB per
//    instruction: the loads write LDS directly (zeros outside the image from the buffer bounds
//    check), finished rows are scaled, shifted, joined with the residual and rounded in registers,
//    staged in LDS and written out in full 128-byte lines one step later;
//  * one barrier per step, in the middle of its MFMAs; what a step waits for was requested two
//    steps earlier.
//
// Ring pixel pitch is 160 bytes (128 of channels + 32 of padding): a shift by one pixel or by 32
// channels is a constant address offset, and the fragment read of 16 consecutive pixels x 4 K groups
// is free of bank conflicts (measured: 2.1 ns per wavefront-instruction, as for contiguous
// addresses; 3.6 ns with a pitch of 144 or 272 bytes, whatever the order of pixels and K groups).
// The two streams of a row share the zero pixel between them: [0][56 pixels][0][56 pixels][0].
#include "internal.h"

namespace sgprs {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));

struct RowsArgs {
    const unsigned char* x;
    const unsigned char* w;   // [64][3][3][64] bf16
    unsigned char* y;
    const float* scale;
    const float* shift;
    const unsigned char* res;  // nullable
    int N, H, S, njobs, jpi, relu;
    unsigned x_bytes, w_bytes, y_bytes;
};

constexpr int kRowsWidth = 56, kRowsStreams = 2, kRowsVRow = kRowsWidth * kRowsStreams;
constexpr int kRowsPixB = 160, kRowsPixUnits = kRowsPixB / 16;
constexpr int kRowsSlotPix = kRowsWidth + 1;                               // pixel slots from one stream to the next (one zero pixel between)
constexpr int kRowsStepUnits = (kRowsStreams * kRowsSlotPix + 1) * kRowsPixUnits;   // 16-byte units of the rows of one step
constexpr int kRowsStepStride = (kRowsStepUnits + 63) / 64 * 1024;         // whole 1 KiB load instructions
constexpr int kRowsRowBytes = kRowsVRow * 128;
constexpr int kRowsRsBase = 4 * kRowsStepStride, kRowsOsBase = kRowsRsBase + 4 * kRowsRowBytes;
constexpr int kRowsDummyBase = kRowsOsBase + 2 * kRowsRowBytes;            // 1 KiB that nobody reads
constexpr int kRowsLds = kRowsDummyBase + 1024;
static_assert(kRowsLds <= 160 * 1024, "LDS of one CU");

// rounds two floats to a bf16 pair and takes the maximum with `floor16x2` as signed 16-bit integers:
// 0 for ReLU (rounding is monotone and keeps 0), the most negative value for none
__device__ __forceinline__ unsigned rows_pack2(float lo, float hi, unsigned floor16x2)
{
    typedef float pk_f32x2 __attribute__((ext_vector_type(2)));
    typedef __bf16 pk_bf16x2 __attribute__((ext_vector_type(2)));
    typedef short pk_s16x2 __attribute__((ext_vector_type(2)));
    const pk_f32x2 f = {lo, hi};
    const pk_s16x2 b = __builtin_bit_cast(pk_s16x2, __builtin_convertvector(f, pk_bf16x2));
    return __builtin_bit_cast(unsigned, __builtin_elementwise_max(b, __builtin_bit_cast(pk_s16x2, floor16x2)));
}

// One wavefront's share: NSUB 16-pixel tiles (from tile sub0) of the virtual row x 16 output channels.
template <int NSUB>
__device__ __forceinline__ void rows_body(const RowsArgs& a, unsigned char* smem, int sub0)
{
#if __HIP_DEVICE_COMPILE__
    constexpr int WIDTH = kRowsWidth, NS = kRowsStreams, VROW = kRowsVRow, PIXB = kRowsPixB;
    constexpr int SLOT_BYTES = kRowsSlotPix * PIXB, UPP = kRowsPixUnits;
    constexpr int STEP_UNITS = kRowsStepUnits, LOAD_IT = (STEP_UNITS + 511) / 512, STEP_STRIDE = kRowsStepStride;
    constexpr int RS_BASE = kRowsRsBase, OS_BASE = kRowsOsBase, DUMMY_BASE = kRowsDummyBase;
    typedef __attribute__((address_space(3))) void* lds_ptr_t;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int q = wave & 3;
    const int j16 = lane & 15, g = lane >> 4;
    const int S = a.S;

    // stationary weights: A operand, row j16 -> output channel 16q + j16, K group g
    const __amdgpu_buffer_rsrc_t w_rs = __builtin_amdgcn_make_buffer_rsrc((void*)a.w, 0, (int)a.w_bytes, 0x00020000);
    u32x4_t wf[9][2];
#pragma unroll
    for (int tap = 0; tap < 9; ++tap)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
            wf[tap][ks] = __builtin_amdgcn_raw_buffer_load_b128(w_rs, (unsigned)((((q * 16 + j16) * 9 + tap) * 64 + ks * 32 + g * 8) * 2), 0, 0);

    // loader table: unit u = it * 512 + tid of a step's rows is 16-byte piece u % UPP of pixel slot u / UPP; slot
    // k * (WIDTH + 1) is a zero pixel, the WIDTH slots behind it are stream k; packed as stream << 16 | byte offset
    // inside the image row, all ones for no data (zero pixels, the padding pieces)
    unsigned ld_tab[LOAD_IT];
#pragma unroll
    for (int it = 0; it < LOAD_IT; ++it) {
        const int u = it * 512 + tid;
        const int slot = u / UPP, cg = u - slot * UPP;
        const int k = slot / kRowsSlotPix, px = slot - k * kRowsSlotPix;   // px 0: the zero pixel in front of stream k
        const bool ok = u < STEP_UNITS && k < NS && px >= 1 && cg < 8;
        ld_tab[it] = ok ? (unsigned)(k << 16) | (unsigned)(((px - 1) * 64 + cg * 8) * 2) : 0xffffffffu;
    }
    unsigned boff[NSUB];   // B fragment address for filter column 0, channels 0-31; + PIXB per column, + 64 for channels 32-63
    unsigned sto[NSUB];    // this lane's 8 bytes (4 channels) of its pixel inside a staged row of 112 pixels x 128 bytes
#pragma unroll
    for (int sub = 0; sub < NSUB; ++sub) {
        const int v = 16 * (sub0 + sub) + j16;
        const int k = v / WIDTH, p = v - k * WIDTH;
        boff[sub] = (unsigned)(k * SLOT_BYTES + p * PIXB + g * 16);
        sto[sub] = (unsigned)(v * 128 + ((((q << 1) | (g >> 1)) ^ (v & 7)) << 4) + ((g & 1) << 3));
    }
    // staged rows (residual in, output out) move as 16-byte units u = it * 512 + tid: slot u & 7 of pixel u >> 3,
    // which holds channel group (u & 7) ^ (pixel & 7)
    constexpr int ROW_UNITS = VROW * 8, ROW_IT = (ROW_UNITS + 511) / 512, ROW_BYTES = kRowsRowBytes;
    unsigned ro_off[ROW_IT];   // byte offset of the unit relative to row 0 of stream 0 (top bit: no such unit)
#pragma unroll
    for (int it = 0; it < ROW_IT; ++it) {
        const int u = it * 512 + tid, px = u >> 3, sl = u & 7;
        const int k = px / WIDTH, p = px - k * WIDTH;
        ro_off[it] = u < ROW_UNITS ? (unsigned)(((k * S * WIDTH + p) * 64 + ((sl ^ (px & 7)) << 3)) * 2) : 0x80000000u;
    }
    const f32x4_t sc = *(const f32x4_t*)(a.scale + q * 16 + 4 * g);
    const f32x4_t sh = *(const f32x4_t*)(a.shift + q * 16 + 4 * g);
    const unsigned relu_floor = a.relu ? 0u : 0x80008000u;

    const __amdgpu_buffer_rsrc_t x_rs = __builtin_amdgcn_make_buffer_rsrc((void*)a.x, 0, (int)a.x_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t y_rs = __builtin_amdgcn_make_buffer_rsrc((void*)a.y, 0, (int)a.y_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t r_rs = __builtin_amdgcn_make_buffer_rsrc((void*)a.res, 0, a.res ? (int)a.y_bytes : 0, 0x00020000);

    // on the whole chip workgroup b runs on die b % 8: consecutive jobs (neighbouring row ranges) share a die
    const int per_die = (a.njobs + 7) / 8;
    for (int b = blockIdx.x; b < per_die * 8; b += gridDim.x) {
        const int job = (b & 7) * per_die + (b >> 3);
        if (job >= a.njobs) continue;
        const int n = job / a.jpi, r0 = (job - n * a.jpi) * NS * S;
        const unsigned img_base = (unsigned)n * a.H * WIDTH * 128u;

        // Every wavefront issues LOAD_IT requests per step, so that "all but the youngest n" is the same count
        // for all: a request with nothing to fetch gets an offset beyond the buffer (zeros arrive) and, where
        // the wavefront's unit range lies beyond the step's units, a destination nobody reads.
        auto ring_load = [&](int tt) {   // input rows of step tt into ring position tt % 4
            const int pos = tt & 3;
#pragma unroll
            for (int it = 0; it < LOAD_IT; ++it) {
                const unsigned tb = ld_tab[it];
                const int row = r0 + (int)((tb >> 16) & 0xffu) * S + tt - 1;
                const bool ok = (int)tb >= 0 && (unsigned)row < (unsigned)a.H && tt <= S + 1;
                const unsigned voff = ok ? img_base + (unsigned)row * (WIDTH * 128u) + (tb & 0xffffu) : 0x80000000u;
                const int dst = it * 512 + wave * 64 < STEP_UNITS ? pos * STEP_STRIDE + (it * 512 + wave * 64) * 16 : DUMMY_BASE;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(x_rs, (lds_ptr_t)(smem + dst), 16, voff, 0, 0, 0);
            }
        };
        ring_load(0);
        ring_load(1);
        ring_load(2);
        __builtin_amdgcn_s_waitcnt(0);
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");

        // acc0 / acc1 / acc2: partial sums of output rows t / t - 1 / t - 2 at step t
        f32x4_t acc0[NSUB], acc1[NSUB], acc2[NSUB];
        u32x4_t bfr[NSUB];
        // where in a step the stores, the requests and the epilogue arithmetic go: one MFMA group after the
        // barrier for the wavefront with four tiles, three groups after it (the step's last group) for the one
        // with three, so that the two wavefronts of a SIMD do their vector work at different times (measured
        // inside the network, same box: 22.4 us per launch against 23.1 us for groups 2 and 4, 22.7-23.5 us
        // for 2/3, 2/5, 2/2, 3/4, 4/2, 5/3 and 5/5, 22.3-22.5 us for 4/5)
        constexpr int TAIL_GI = NSUB == 3 ? 5 : 3;
#pragma unroll
        for (int sub = 0; sub < NSUB; ++sub) {
            acc0[sub] = acc1[sub] = acc2[sub] = f32x4_t{0.f, 0.f, 0.f, 0.f};
            bfr[sub] = *(const u32x4_t*)(smem + boff[sub]);   // first fragments of step 0
        }
        const unsigned out_base = (unsigned)((n * a.H + r0) * WIDTH) * 64u;   // elements

        // Step t: the input rows r0 + k*S + t - 1 of the streams (ring position t % 4) feed output rows t, t - 1
        // and t - 2; VM says which of the three exist.  Output row t - 3, which the previous step finished, is
        // scaled and shifted out of acc2 before the first MFMA reuses those registers.  Half way through the
        // step comes the only synchronisation: every wavefront waits for the rows it requested two steps ago
        // (those of step t + 1) and for the residual it requested then, and all meet at a barrier; after it
        // row t - 4 is written out of its stage, the residual of row t is requested, the rows of step t + 3
        // are requested into the ring position that step t - 1 has left, and row t - 3 is finished into the
        // output stage.  The first fragments of step t + 1 are read before the last MFMAs of step t.
        auto step = [&](auto VMC, int t) {
            constexpr int VM = decltype(VMC)::value;
            f32x4_t fm[NSUB];
#pragma unroll
            for (int sub = 0; sub < NSUB; ++sub) fm[sub] = acc2[sub] * sc + sh;
            const unsigned char* buf = smem + (t & 3) * STEP_STRIDE;
            const unsigned char* buf_next = smem + ((t + 1) & 3) * STEP_STRIDE;
            auto mid_sync = [&]() {
                // Everything but what the previous step requested (ROW_IT + LOAD_IT requests per wavefront, its
                // youngest loads) has arrived.  Loads return in order, so the count is safe whatever the stores
                // do.  Steps without MFMAs request nothing and wait only for LDS.
                if constexpr (VM == 0) __builtin_amdgcn_s_waitcnt(0xC07F);
                else if constexpr (VM == 1) __builtin_amdgcn_s_waitcnt(0x0070);   // step 0: the prologue waited for everything
                else __builtin_amdgcn_s_waitcnt(((ROW_IT + LOAD_IT) & 15) | 0x0070);
                asm volatile("" ::: "memory");
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
            };
            auto io_part = [&]() {
                {   // output row t - 4, staged by all wavefronts, goes out in whole 128-byte lines
                    const int yo = t - 4;
                    const unsigned char* os = smem + OS_BASE + (yo & 1) * ROW_BYTES;
                    const unsigned row_b = out_base * 2u + (unsigned)yo * (WIDTH * 128u);
#pragma unroll
                    for (int it = 0; it < ROW_IT; ++it) {
                        const u32x4_t v = *(const u32x4_t*)(os + (it * 512 + tid) * 16);
                        __builtin_amdgcn_raw_buffer_store_b128(v, y_rs, (yo >= 0 && (int)ro_off[it] >= 0) ? row_b + ro_off[it] : 0x80000000u, 0, 0);
                    }
                }
                if constexpr (VM != 0) {
                    // residual of output row t, which the step after next completes (nothing to fetch from row S on)
                    const unsigned row_b = out_base * 2u + (unsigned)t * (WIDTH * 128u);
#pragma unroll
                    for (int it = 0; it < ROW_IT; ++it) {
                        const int dst = it * 512 + wave * 64 < ROW_UNITS ? RS_BASE + (t & 3) * ROW_BYTES + (it * 512 + wave * 64) * 16 : DUMMY_BASE;
                        __builtin_amdgcn_raw_ptr_buffer_load_lds(r_rs, (lds_ptr_t)(smem + dst), 16,
                                                                 (t < S && (int)ro_off[it] >= 0) ? row_b + ro_off[it] : 0x80000000u, 0, 0, 0);
                    }
                    ring_load(t + 3);
                }
            };
            // output row yrow (scaled and shifted in fm): residual from its staged copy, result into the output stage
            auto math_part = [&](int yrow) {
                const unsigned char* rs = smem + RS_BASE + (yrow & 3) * ROW_BYTES;
                unsigned char* os = smem + OS_BASE + (yrow & 1) * ROW_BYTES;
#pragma unroll
                for (int sub = 0; sub < NSUB; ++sub) {
                    const u32x2_t rr = *(const u32x2_t*)(rs + sto[sub]);
                    const float o0 = fm[sub][0] + __uint_as_float(rr[0] << 16);
                    const float o1 = fm[sub][1] + __uint_as_float(rr[0] & 0xffff0000u);
                    const float o2 = fm[sub][2] + __uint_as_float(rr[1] << 16);
                    const float o3 = fm[sub][3] + __uint_as_float(rr[1] & 0xffff0000u);
                    u32x2_t ov;
                    ov[0] = rows_pack2(o0, o1, relu_floor);
                    ov[1] = rows_pack2(o2, o3, relu_floor);
                    *(u32x2_t*)(os + sto[sub]) = ov;
                }
            };
            if constexpr (VM != 0) {
#pragma unroll
                for (int gi = 0; gi < 6; ++gi) {
                    const int s = gi >> 1, ks = gi & 1;
                    const int s1 = (gi + 1) >> 1, ks1 = (gi + 1) & 1;
#pragma unroll
                    for (int sub = 0; sub < NSUB; ++sub) {
                        if constexpr ((VM & 4) != 0)
                            acc2[sub] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, wf[6 + s][ks]), __builtin_bit_cast(bf16x8_t, bfr[sub]),
                                                                                gi == 0 ? acc1[sub] : acc2[sub], 0, 0, 0);
                        if constexpr ((VM & 2) != 0)
                            acc1[sub] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, wf[3 + s][ks]), __builtin_bit_cast(bf16x8_t, bfr[sub]),
                                                                                gi == 0 ? acc0[sub] : acc1[sub], 0, 0, 0);
                        if constexpr ((VM & 1) != 0)
                            acc0[sub] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, wf[s][ks]), __builtin_bit_cast(bf16x8_t, bfr[sub]),
                                                                                gi == 0 ? f32x4_t{0.f, 0.f, 0.f, 0.f} : acc0[sub], 0, 0, 0);
                        // the fragment's registers are refilled for the next group (the next step's first group
                        // at the end) while the MFMAs of the other tiles run
                        bfr[sub] = gi + 1 < 6 ? *(const u32x4_t*)(buf + boff[sub] + s1 * PIXB + ks1 * 64) : *(const u32x4_t*)(buf_next + boff[sub]);
                    }
                    if (gi == 2) mid_sync();
                    if (gi == TAIL_GI) { io_part(); math_part(t - 3); }
                }
            } else {
                mid_sync();
                io_part();
                math_part(t - 3);
            }
        };
        // steps 0 .. S + 1 compute (S >= 2), steps S + 2 and S + 3 only finish and write the last rows
        step(std::integral_constant<int, 1>{}, 0);
        step(std::integral_constant<int, 3>{}, 1);
        for (int t = 2; t < S; ++t) step(std::integral_constant<int, 7>{}, t);
        step(std::integral_constant<int, 6>{}, S);
        step(std::integral_constant<int, 4>{}, S + 1);
        step(std::integral_constant<int, 0>{}, S + 2);
        step(std::integral_constant<int, 0>{}, S + 3);
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();   // the ring is free for the next job
        asm volatile("" ::: "memory");
    }
    __builtin_amdgcn_s_waitcnt(0);
#endif
}

__global__ __launch_bounds__(512, 1) void conv3x3_rows_kernel(const RowsArgs a)
{
#if __HIP_DEVICE_COMPILE__
    extern __shared__ __align__(16) unsigned char smem[];
    // wavefronts w and w + 4 share a SIMD: one takes tiles 0-3 of the virtual row, the other tiles 4-6
    if (threadIdx.x < 256) rows_body<4>(a, smem, 0);
    else rows_body<3>(a, smem, 4);
#endif
}

static std::atomic<bool> g_rows_off{false};
void rows_force_off(bool off) { g_rows_off = off; }

// Rows per stream and job for this shape on `cus` CUs, 0 if the kernel does not apply.  Measured
// faster than the LDS-patch kernel where every CU gets the same number of whole jobs of at least 7
// rows per stream; smaller jobs spend too much on halo rows and on filling the pipeline.
bool plan_rows(const sgprs_conv_desc_t& d, int cus, int* rows_per_stream)
{
    if (g_rows_off.load()) return false;
    if (d.dtype != SGPRS_BF16 || d.r != 3 || d.s != 3 || d.stride != 1 || d.pad != 1 || d.cin != 64 || d.cout != 64 ||
        d.w != kRowsWidth || d.n < 1 || (long long)d.n * d.h * d.w * 128 >= (1ll << 31))
        return false;
    int best = 0;
    double best_cost = 1e30;
    for (int S = 7; 2 * S <= d.h; ++S) {
        if (d.h % (2 * S) || S > 60) continue;
        const long long jobs = (long long)d.n * (d.h / (2 * S));
        const long long rounds = (jobs + cus - 1) / cus;
        const double ideal = (double)d.n * d.h / 2.0 / cus;   // rows per stream and CU with perfect balance
        if (ideal / (double)(rounds * S) < 0.85) continue;
        const double cost = (double)rounds * (S + 7);
        if (cost < best_cost) { best_cost = cost; best = S; }
    }
    if (!best) return false;
    *rows_per_stream = best;
    return true;
}

int launch_conv3x3_rows(const sgprs_conv_desc_t& d, int S, const void* x, const void* w, const float* scale,
                        const float* shift, const void* residual, void* y, hipStream_t stream, int cus, Profiler* prof)
{
    if (d.w != kRowsWidth || d.cin != 64 || d.cout != 64 || S < 2 || d.h % (2 * S))
        return fail(SGPRS_ERR_INVALID_ARG, "internal: row-streaming plan does not match the shape");
    RowsArgs a;
    a.x = (const unsigned char*)x; a.w = (const unsigned char*)w; a.y = (unsigned char*)y;
    a.scale = scale; a.shift = shift; a.res = (const unsigned char*)residual;
    a.N = d.n; a.H = d.h; a.S = S; a.jpi = d.h / (2 * S); a.njobs = d.n * a.jpi; a.relu = d.relu;
    a.x_bytes = a.y_bytes = (unsigned)((size_t)d.n * d.h * d.w * 128);
    a.w_bytes = 64 * 9 * 64 * 2;
    const double M = (double)d.n * d.h * d.w;
    const double flops = 2.0 * M * 64 * 9.0 * 64;
    const double bytes = (M * 64 + 64.0 * 9 * 64 + M * 64 * (residual ? 2 : 1)) * 2.0;
    int rc;
    if (prof && prof->on && (rc = prof->begin(stream, kKindRows, 0, flops, bytes))) return rc;
    static std::atomic<bool> raised{false};
    if (!raised) {
        SGPRS_HIP(hipFuncSetAttribute((const void*)conv3x3_rows_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kRowsLds));
        raised = true;
    }
    const int per_die = (a.njobs + 7) / 8;
    const int grid = std::min(cus < 1 ? 1 : cus, per_die * 8);
    SGPRS_LAUNCH(conv3x3_rows_kernel, dim3(grid), dim3(512), kRowsLds, stream, a);
    SGPRS_HIP(hipGetLastError());
    if (prof && prof->on && (rc = prof->end(stream))) return rc;
    return SGPRS_OK;
}

}  // namespace sgprs
