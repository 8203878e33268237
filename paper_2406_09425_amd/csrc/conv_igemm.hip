// Convolution as implicit GEMM on the gfx950 matrix cores.
//
// The paper's "GPU Speedup Analysis" singles out convolution as the operation
// that dominates ResNet18; it really is a dense contraction, so it goes to
// MFMA:  C[m][n] = sum_k A[m][k] * B[n][k]  with
//   m = output pixel (image, p, q), n = output channel, k = (r, s, c),
//   A gathered on the fly from the NHWC input (zero outside the image),
//   B = weights packed [cout][r][s][cin].
// A k-tile is 128 bytes of one filter tap (64 bf16 / 32 fp32 channels), so a
// tile row is one contiguous run of channels of one input pixel.
//
// Per workgroup (256 threads = 4 wavefronts of 64): a BM x BN output tile,
// A and B k-tiles staged in LDS (two stages, filled by buffer loads that write
// LDS directly while the other stage feeds the MFMAs), XOR-swizzled 16-byte
// chunks so that fragment reads are bank-conflict free.  The epilogue applies
// the folded BN scale/shift, the residual and ReLU in fp32 and stores in the
// activation dtype.  With split-K each z-slice of the grid writes fp32 partial
// tiles and a second kernel sums the slices in a fixed order and applies the
// same epilogue, which keeps results bitwise reproducible.
#include "internal.h"

namespace sgprs {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

struct IgemmArgs {
    const unsigned char* x;
    const unsigned char* w;
    unsigned char* y;
    const float* scale;
    const float* shift;
    const unsigned char* res;
    float* partial;
    int H, W, Cin, Cout, P, Q, R, S, stride, pad;
    int M, PQ;
    unsigned pq_mul, q_mul;  // m / PQ and rem / Q as multiply-high and shift (shift -1: divisor 1)
    int pq_sh, q_sh;
    int ktiles, kt_per_split, cin_tiles;
    int relu;
    unsigned x_bytes, w_bytes;  // buffer-descriptor bounds of x and w
};

__device__ __forceinline__ float bf16_to_f32(unsigned short b) { return __uint_as_float((unsigned)b << 16); }
__device__ __forceinline__ unsigned short f32_to_bf16(float f)
{
    __bf16 h = (__bf16)f;  // round to nearest even
    return __builtin_bit_cast(unsigned short, h);
}

template <int DT> struct Store;
template <> struct Store<SGPRS_F32> {
    static __device__ __forceinline__ float load(const unsigned char* p, size_t i) { return ((const float*)p)[i]; }
    static __device__ __forceinline__ void store(unsigned char* p, size_t i, float v) { ((float*)p)[i] = v; }
};
template <> struct Store<SGPRS_BF16> {
    static __device__ __forceinline__ float load(const unsigned char* p, size_t i)
    {
        return bf16_to_f32(((const unsigned short*)p)[i]);
    }
    static __device__ __forceinline__ void store(unsigned char* p, size_t i, float v)
    {
        ((unsigned short*)p)[i] = f32_to_bf16(v);
    }
};

// m / d for 0 <= m < 2^31 with the constants of fast_div_constants().
__device__ __forceinline__ int fast_div(int m, unsigned mul, int sh)
{
    return sh < 0 ? m : (int)(__umulhi((unsigned)m, mul) >> sh);
}

__device__ __forceinline__ int swz(int row, int chunk) { return row * 128 + ((chunk ^ (row & 7)) << 4); }

// Pipeline depth (LDS stages).  Three and four stages measured the same as two,
// at batch 64 (where they also cost workgroups per CU) and at batch 1: the loop
// is bound by its instruction stream and by per-tile fixed costs, not by load
// latency or L2 -> LDS bandwidth.
template <int BM, int BN> struct IgemmStages { static constexpr int value = 2; };

// One BM x BN output tile: tile column bx, channel block by, split-K slice bz.
//
// The k-tiles move global -> LDS directly (buffer loads with the LDS bit; one
// wavefront instruction fills 8 swizzled rows = 1 KiB), NS stages deep: while
// k-tile kt feeds the MFMAs, k-tiles kt+1 .. kt+NS-2 are in flight and the
// loads of kt+NS-1 are issued.  Taps outside the image get a buffer offset
// beyond the descriptor's size, for which the hardware returns zeros; k-tiles
// past the end use a descriptor of size 0.  Every stage issues the same number
// of loads, so "k-tile kt has landed" is a fixed vmcnt.
template <int DT, int BM, int BN, int WM, int WN, bool SPLIT>
__device__ __forceinline__ void igemm_tile(const IgemmArgs& a, int bx, int by, int bz)
{
    constexpr int ES = DT == SGPRS_BF16 ? 2 : 4;  // element size
    constexpr int KT = 128 / ES;                  // elements per k-tile row
    constexpr int CH = 16 / ES;                   // elements per 16-byte chunk
    constexpr int WTM = BM / WM, WTN = BN / WN;   // wavefront tile
    constexpr int TM = WTM / 32, TN = WTN / 32;   // 32x32 MFMA tiles per wavefront
    constexpr int A_IT = BM / 32, B_IT = BN / 32; // load instructions per thread and stage
    constexpr int STAGE = (BM + BN) * 128;
    constexpr int NS = IgemmStages<BM, BN>::value;
    constexpr int LPS = A_IT + B_IT;
    static_assert(WM * WN == 4 && TM >= 1 && TN >= 1, "tile shape");
    static_assert((NS - 2) * LPS <= 63, "vmcnt range");

    extern __shared__ __align__(16) unsigned char smem[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform: LDS destinations stay in scalar registers
    const int wm = wave / WN, wn = wave % WN;
    const int m0 = bx * BM, n0 = by * BN;
    const int kt_begin = bz * a.kt_per_split;
    const int kt_end = min(kt_begin + a.kt_per_split, a.ktiles);
    const int K = a.ktiles * KT;

    // ---- loader bookkeeping: instruction i of this wavefront fills rows
    // i*32 + wave*8 .. +7 of a stage; this lane's LDS slot (lane & 7) of row
    // lane >> 3 holds global chunk (lane & 7) ^ (lane >> 3) (the swizzle).
    // Per row: the byte offset of tap (0, 0) and which filter rows (bits 0..)
    // and columns (bits 16..) fall inside the image.
    const int lrow = wave * 8 + (lane >> 3), gchunk = (lane & 7) ^ (lane >> 3);
    int a_base[A_IT];
    unsigned a_in[A_IT];
#pragma unroll
    for (int i = 0; i < A_IT; ++i) {
        const int m = m0 + lrow + 32 * i;
        a_base[i] = 0;
        a_in[i] = 0;  // rows past M: every tap falls outside
        if (m < a.M) {
            const int n = fast_div(m, a.pq_mul, a.pq_sh), rem = m - n * a.PQ;
            const int p = fast_div(rem, a.q_mul, a.q_sh), q = rem - p * a.Q;
            const int h0 = p * a.stride - a.pad, w0 = q * a.stride - a.pad;
            a_base[i] = (((n * a.H + h0) * a.W + w0) * a.Cin + gchunk * CH) * ES;
#pragma unroll
            for (int t = 0; t < 3; ++t) {  // filters are at most 3x3 here
                a_in[i] |= (unsigned)(t < a.R && (unsigned)(h0 + t) < (unsigned)a.H) << t;
                a_in[i] |= (unsigned)(t < a.S && (unsigned)(w0 + t) < (unsigned)a.W) << (16 + t);
            }
        }
    }
    unsigned b_off[B_IT];
#pragma unroll
    for (int i = 0; i < B_IT; ++i) b_off[i] = (unsigned)((n0 + lrow + 32 * i) * K + gchunk * CH) * ES;

    // The issue cursor walks the k-tiles in order: channel tile ic of tap (ir, is).  The lanes'
    // offsets change only when the tap does; the channel tile goes into the scalar offset.
    int ic = 0, ir = 0, is = 0;
    if (kt_begin) {  // split-K slices start somewhere inside the filter
        const int tap = kt_begin / a.cin_tiles;
        ic = kt_begin - tap * a.cin_tiles;
        ir = tap / a.S;
        is = tap - ir * a.S;
    }
    unsigned a_voff[A_IT];
    auto enter_tap = [&]() {
        const int tap_off = (ir * a.W + is) * a.Cin * ES;
        const unsigned need = (1u << ir) | (0x10000u << is);
#pragma unroll
        for (int i = 0; i < A_IT; ++i)
            a_voff[i] = (a_in[i] & need) == need ? (unsigned)(a_base[i] + tap_off) : 0x80000000u;
    };
    enter_tap();
    // Loads of k-tile kt straight into LDS stage `stage`: A_IT instructions for the input rows,
    // B_IT for the weight rows.  Past kt_end the descriptors have size 0 and nothing is fetched.
    auto issue_stage = [&](int kt, int stage) {
#if __HIP_DEVICE_COMPILE__  // the buffer-resource builtins exist in the device pass only
        typedef __attribute__((address_space(3))) void* lds_ptr_t;
        const bool live = kt < kt_end;
        const __amdgpu_buffer_rsrc_t x_rs = __builtin_amdgcn_make_buffer_rsrc((void*)a.x, 0, live ? (int)a.x_bytes : 0, 0x00020000);
        const __amdgpu_buffer_rsrc_t w_rs = __builtin_amdgcn_make_buffer_rsrc((void*)a.w, 0, live ? (int)a.w_bytes : 0, 0x00020000);
        unsigned char* As = smem + stage * STAGE;
#pragma unroll
        for (int i = 0; i < A_IT; ++i)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(x_rs, (lds_ptr_t)(As + (i * 32 + wave * 8) * 128), 16, a_voff[i], ic * 128, 0, 0);
#pragma unroll
        for (int i = 0; i < B_IT; ++i)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(w_rs, (lds_ptr_t)(As + (BM + i * 32 + wave * 8) * 128), 16, b_off[i],
                                                     (live ? kt : 0) * 128, 0, 0);
        if (++ic == a.cin_tiles) {
            ic = 0;
            if (++is == a.S) { is = 0; ++ir; }
            enter_tap();
        }
#endif
    };

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    const int frow = lane & 31, fhalf = lane >> 5;
    // fragment addresses inside a stage, one per k-step (k-step ks flips bits 5-6); the
    // 32-row tiles below and the stage are constant offsets from them
    unsigned fa_off[4], fb_off[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        fa_off[ks] = swz(wm * WTM + frow, fhalf) ^ (ks << 5);
        fb_off[ks] = BM * 128 + (swz(wn * WTN + frow, fhalf) ^ (ks << 5));
    }

    auto compute_stage = [&](int stage) {
        const unsigned char* St = smem + stage * STAGE;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            u32x4_t af[TM], bf[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) af[i] = *(const u32x4_t*)(St + fa_off[ks] + i * 32 * 128);
#pragma unroll
            for (int j = 0; j < TN; ++j) bf[j] = *(const u32x4_t*)(St + fb_off[ks] + j * 32 * 128);
            if constexpr (DT == SGPRS_BF16) {
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            __builtin_bit_cast(bf16x8_t, af[i]), __builtin_bit_cast(bf16x8_t, bf[j]),
                            acc[i][j], 0, 0, 0);
            } else {
#pragma unroll
                for (int u = 0; u < 4; ++u)
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int j = 0; j < TN; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(
                                __uint_as_float(af[i][u]), __uint_as_float(bf[j][u]), acc[i][j], 0, 0, 0);
            }
        }
    };

#pragma unroll
    for (int q = 0; q < NS - 1; ++q) issue_stage(kt_begin + q, q);
    // NS k-tiles per trip, so that every stage index below is a constant
    auto k_tile = [&](int kt, int st) {
        // k-tile kt has landed once at most the NS-2 younger stages are outstanding
        __builtin_amdgcn_s_waitcnt(((NS - 2) * LPS & 15) | (((NS - 2) * LPS >> 4) << 14) | 0x0F70);
        __syncthreads();  // ... for every thread; and the stage read last iteration is free
        issue_stage(kt + NS - 1, (st + NS - 1) % NS);
        compute_stage(st);
    };
    int kt = kt_begin;
    for (; kt + NS <= kt_end; kt += NS) {
#pragma unroll
        for (int st = 0; st < NS; ++st) k_tile(kt + st, st);
    }
#pragma unroll
    for (int st = 0; st < NS - 1; ++st)
        if (kt + st < kt_end) k_tile(kt + st, st);
    // drain the (empty) loads still in flight before the staging area becomes scratch
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();

    // ---- epilogue.  32x32 accumulator layout: column = lane % 32,
    // row = 8*(e/4) + 4*(lane/32) + e%4 for register e.
    // Each wavefront transposes one 32-row x WTN-column piece at a time through
    // its own LDS scratch (the k-loop ended with a barrier, so the staging
    // buffers are free); afterwards a lane owns 8 consecutive channels of one
    // output pixel and moves 16 (bf16) or 32 (fp32) contiguous bytes.
    constexpr int SROW = WTN + 4;  // padded scratch row, floats
    constexpr int LPR = WTN / 8;   // lanes per row in the read-back
    constexpr int RPP = 64 / LPR;  // rows per pass
    constexpr int NPASS = 32 / RPP;
    static_assert(4 * 32 * SROW * 4 <= NS * STAGE, "epilogue scratch fits the staging buffers");
    float* scr = (float*)smem + wave * 32 * SROW;
    const int c8 = (lane % LPR) * 8, rsub = lane / LPR;
    const int nb = n0 + wn * WTN + c8;
    f32x4_t sc0 = {1.f, 1.f, 1.f, 1.f}, sc1 = sc0, sh0 = {0.f, 0.f, 0.f, 0.f}, sh1 = sh0;
    if constexpr (!SPLIT) {
        sc0 = *(const f32x4_t*)(a.scale + nb); sc1 = *(const f32x4_t*)(a.scale + nb + 4);
        sh0 = *(const f32x4_t*)(a.shift + nb); sh1 = *(const f32x4_t*)(a.shift + nb + 4);
    }
    // The residual rows are requested up front, unconditionally and from clamped
    // (always valid) rows, so that all of them are in flight together instead
    // of one round trip per pass.
    constexpr int RV = DT == SGPRS_F32 ? 2 : 1;
    u32x4_t rres[TM][NPASS][RV];
    const bool has_res = !SPLIT && a.res != nullptr;
    const unsigned relu_floor = a.relu ? kReluFloor : kNoReluFloor;
    if (has_res) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int pass = 0; pass < NPASS; ++pass) {
                const int m = min(m0 + wm * WTM + i * 32 + pass * RPP + rsub, a.M - 1);
                const unsigned char* rp = a.res + ((size_t)m * a.Cout + nb) * ES;
#pragma unroll
                for (int v = 0; v < RV; ++v) rres[i][pass][v] = *(const u32x4_t*)(rp + 16 * v);
            }
    }
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e)
                scr[(8 * (e >> 2) + 4 * fhalf + (e & 3)) * SROW + j * 32 + frow] = acc[i][j][e];
#pragma unroll
        for (int pass = 0; pass < NPASS; ++pass) {
            const int rr = pass * RPP + rsub;
            const int m = m0 + wm * WTM + i * 32 + rr;
            f32x4_t v0 = *(const f32x4_t*)(scr + rr * SROW + c8);
            f32x4_t v1 = *(const f32x4_t*)(scr + rr * SROW + c8 + 4);
            if (m >= a.M) continue;
            if constexpr (SPLIT) {
                float* dst = a.partial + ((size_t)bz * a.M + m) * a.Cout + nb;
                *(f32x4_t*)dst = v0;
                *(f32x4_t*)(dst + 4) = v1;
            } else {
                const size_t o = (size_t)m * a.Cout + nb;
                v0 = v0 * sc0 + sh0;
                v1 = v1 * sc1 + sh1;
                if constexpr (DT == SGPRS_F32) {
                    if (has_res) {
                        v0 += __builtin_bit_cast(f32x4_t, rres[i][pass][0]);
                        v1 += __builtin_bit_cast(f32x4_t, rres[i][pass][RV - 1]);
                    }
                    if (a.relu) {
#pragma unroll
                        for (int u = 0; u < 4; ++u) { v0[u] = fmaxf(v0[u], 0.f); v1[u] = fmaxf(v1[u], 0.f); }
                    }
                    *(f32x4_t*)(a.y + o * 4) = v0;
                    *(f32x4_t*)(a.y + o * 4 + 16) = v1;
                } else {
                    float v[8] = {v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
                    u32x4_t rv = {0u, 0u, 0u, 0u};
                    if (has_res) rv = rres[i][pass][0];
                    u32x4_t ov;
                    if (has_res) {  // uniform: launches without a residual skip its unpacking and additions
#pragma unroll
                        for (int u = 0; u < 4; ++u) {
                            const float lo = v[2 * u] + __uint_as_float(rv[u] << 16);
                            const float hi = v[2 * u + 1] + __uint_as_float(rv[u] & 0xffff0000u);
                            ov[u] = pack_bf16x2_relu(lo, hi, relu_floor);
                        }
                    } else {
#pragma unroll
                        for (int u = 0; u < 4; ++u) ov[u] = pack_bf16x2_relu(v[2 * u], v[2 * u + 1], relu_floor);
                    }
                    *(u32x4_t*)(a.y + o * 2) = ov;
                }
            }
        }
    }
}

template <int DT, int BM, int BN, int WM, int WN, bool SPLIT>
__global__ __launch_bounds__(256) void conv_igemm_kernel(const IgemmArgs a)
{
    const int bx = blockIdx.x, by = blockIdx.y, bz = blockIdx.z;
    igemm_tile<DT, BM, BN, WM, WN, SPLIT>(a, bx, by, bz);
}

// Two convolutions of the same input in one launch (a BasicBlock's first 3x3
// convolution and the 1x1 convolution of its shortcut, which reads the centre
// tap of the same windows): workgroups [0, tiles0) run the first problem, the
// rest the second.  Neither depends on the other, so the short second problem
// fills the tail of the first instead of paying a launch of its own.
template <int DT, int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(256) void conv_igemm_pair_kernel(const IgemmArgs a0, const IgemmArgs a1, int grid_n0,
                                                              int tiles0, int slots0, int grid_n1, int tiles1)
{
    // Workgroup b runs on die b % 8.  Each die takes a contiguous range of row tiles with all
    // their channel blocks (of both problems), so that a die's L2 fetches its input rows once and
    // workgroups launched back to back share them; slots0 and the grid are multiples of 8, the
    // surplus workgroups leave at once.
    const int b = blockIdx.x, die = b & 7;
    if (b < slots0) {
        const int t = die * (slots0 >> 3) + (b >> 3);
        if (t < tiles0) igemm_tile<DT, BM, BN, WM, WN, false>(a0, t / grid_n0, t % grid_n0, 0);
    } else {
        const int slots1 = gridDim.x - slots0;
        const int t = die * (slots1 >> 3) + ((b - slots0) >> 3);
        if (t < tiles1) igemm_tile<DT, BM, BN, WM, WN, false>(a1, t / grid_n1, t % grid_n1, 0);
    }
}

// Second pass of split-K: sums the slices in index order, then scale/shift,
// residual, ReLU.  One thread per 4 consecutive output channels.
template <int DT>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ partial, int splits,
                                                            size_t total, int Cout,
                                                            const float* __restrict__ scale,
                                                            const float* __restrict__ shift,
                                                            const unsigned char* __restrict__ res,
                                                            unsigned char* __restrict__ y, int relu)
{
    const size_t i4 = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i4 >= total) return;
    f32x4_t s = *(const f32x4_t*)(partial + i4);
    for (int z = 1; z < splits; ++z) {
        const f32x4_t t = *(const f32x4_t*)(partial + (size_t)z * total + i4);
        s += t;
    }
    const int n = (int)(i4 % Cout);
    const f32x4_t sc = *(const f32x4_t*)(scale + n), sh = *(const f32x4_t*)(shift + n);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        float v = s[e] * sc[e] + sh[e];
        if (res) v += Store<DT>::load(res, i4 + e);
        if (relu) v = fmaxf(v, 0.f);
        Store<DT>::store(y, i4 + e, v);
    }
}

// ---- launch ----------------------------------------------------------------
template <int DT, int BM, int BN, int WM, int WN>
static int launch_variant(const IgemmArgs& a, const ConvPlan& p, hipStream_t stream)
{
    const dim3 grid(p.grid_m, p.grid_n, p.splits), block(256);
    const size_t lds = (size_t)IgemmStages<BM, BN>::value * (BM + BN) * 128;
    static std::atomic<bool> raised{false};  // more than the default 64 KiB of dynamic LDS needs an opt-in per kernel
    if (!raised) {
        SGPRS_HIP(hipFuncSetAttribute((const void*)conv_igemm_kernel<DT, BM, BN, WM, WN, true>,
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        SGPRS_HIP(hipFuncSetAttribute((const void*)conv_igemm_kernel<DT, BM, BN, WM, WN, false>,
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        raised = true;
    }
    if (p.splits > 1)
        SGPRS_LAUNCH((conv_igemm_kernel<DT, BM, BN, WM, WN, true>), grid, block, lds, stream, a);
    else
        SGPRS_LAUNCH((conv_igemm_kernel<DT, BM, BN, WM, WN, false>), grid, block, lds, stream, a);
    SGPRS_HIP(hipGetLastError());
    return SGPRS_OK;
}

template <int DT>
static int launch_dtype(const IgemmArgs& a, const ConvPlan& p, hipStream_t stream)
{
    switch (p.variant) {
        case 0: return launch_variant<DT, 128, 128, 2, 2>(a, p, stream);
        case 1: return launch_variant<DT, 128, 64, 2, 2>(a, p, stream);
        case 2: return launch_variant<DT, 64, 64, 2, 2>(a, p, stream);
        case 3: return launch_variant<DT, 32, 128, 1, 4>(a, p, stream);
        default: return fail(SGPRS_ERR_INVALID_ARG, "bad igemm variant %d", p.variant);
    }
}

template <int DT, int BM, int BN, int WM, int WN>
static int launch_pair_variant(const IgemmArgs& a0, const ConvPlan& p0, const IgemmArgs& a1, const ConvPlan& p1,
                               hipStream_t stream)
{
    const int tiles0 = p0.grid_m * p0.grid_n, tiles1 = p1.grid_m * p1.grid_n;
    const size_t lds = (size_t)IgemmStages<BM, BN>::value * (BM + BN) * 128;
    static std::atomic<bool> raised{false};
    if (!raised) {
        SGPRS_HIP(hipFuncSetAttribute((const void*)conv_igemm_pair_kernel<DT, BM, BN, WM, WN>,
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        raised = true;
    }
    const int slots0 = (tiles0 + 7) / 8 * 8, slots1 = (tiles1 + 7) / 8 * 8;
    SGPRS_LAUNCH((conv_igemm_pair_kernel<DT, BM, BN, WM, WN>), dim3(slots0 + slots1), dim3(256), lds, stream, a0, a1, p0.grid_n, tiles0, slots0,
                 p1.grid_n, tiles1);
    SGPRS_HIP(hipGetLastError());
    return SGPRS_OK;
}

template <int DT>
static int launch_pair_dtype(const IgemmArgs& a0, const ConvPlan& p0, const IgemmArgs& a1, const ConvPlan& p1,
                             hipStream_t stream)
{
    switch (p0.variant) {
        case 0: return launch_pair_variant<DT, 128, 128, 2, 2>(a0, p0, a1, p1, stream);
        case 1: return launch_pair_variant<DT, 128, 64, 2, 2>(a0, p0, a1, p1, stream);
        case 2: return launch_pair_variant<DT, 64, 64, 2, 2>(a0, p0, a1, p1, stream);
        case 3: return launch_pair_variant<DT, 32, 128, 1, 4>(a0, p0, a1, p1, stream);
        default: return fail(SGPRS_ERR_INVALID_ARG, "bad igemm variant %d", p0.variant);
    }
}

static const int kIgemmShape[4][4] = {{128, 128, 2, 2}, {128, 64, 2, 2}, {64, 64, 2, 2}, {32, 128, 1, 4}};

// Name as a profiler prints it: v = tile variant + 8 * dtype.
const char* igemm_pair_variant_name(int v)
{
    static char buf[8][96];
    static int next = 0;
    if (v < 0 || v >= 16 || (v & 7) >= 4) return "?";
    const int* t = kIgemmShape[v & 7];
    char* out = buf[next++ & 7];
    snprintf(out, 96, "conv_igemm_pair_kernel<%d, %d, %d, %d, %d>", (v >> 3) & 1, t[0], t[1], t[2], t[3]);
    return out;
}

// Name as a profiler prints it: v = tile variant + 8 * dtype + 16 * split.
const char* igemm_variant_name(int v)
{
    static char buf[8][96];
    static int next = 0;
    if (v < 0 || v >= 32 || (v & 7) >= 4) return "?";
    const int* t = kIgemmShape[v & 7];
    char* out = buf[next++ & 7];
    snprintf(out, 96, "conv_igemm_kernel<%d, %d, %d, %d, %d, %s>", (v >> 3) & 1, t[0], t[1], t[2], t[3],
             (v & 16) ? "true" : "false");
    return out;
}

int launch_splitk_reduce(int dtype, const float* partial, int splits, size_t total, int cout, const float* scale,
                         const float* shift, const void* res, void* y, int relu, hipStream_t stream)
{
    const unsigned blocks = (unsigned)((total / 4 + 255) / 256);
    if (dtype == SGPRS_BF16)
        SGPRS_LAUNCH(splitk_reduce_kernel<SGPRS_BF16>, dim3(blocks), dim3(256), 0, stream, partial, splits, total,
                           cout, scale, shift, (const unsigned char*)res, (unsigned char*)y, relu);
    else
        SGPRS_LAUNCH(splitk_reduce_kernel<SGPRS_F32>, dim3(blocks), dim3(256), 0, stream, partial, splits, total,
                           cout, scale, shift, (const unsigned char*)res, (unsigned char*)y, relu);
    SGPRS_HIP(hipGetLastError());
    return SGPRS_OK;
}

// Kernel arguments for plan p; false if the plan does not match the shape
// (the host-side checks the kernel relies on).
// Constants for fast_div: with L = ceil(log2 d) and mul = ceil(2^(31+L) / d) < 2^32,
// floor(m / d) = (m * mul) >> (31 + L) for every 0 <= m < 2^31.
static void fast_div_constants(int d, unsigned* mul, int* sh)
{
    if (d <= 1) { *mul = 0; *sh = -1; return; }
    int L = 1;
    while ((1ll << L) < d) ++L;
    *mul = (unsigned)(((1ull << (31 + L)) + (unsigned)d - 1) / (unsigned)d);
    *sh = L - 1;
}

static bool fill_igemm_args(const sgprs_conv_desc_t& d, const ConvPlan& p, const void* x, const void* w,
                            const float* scale, const float* shift, const void* residual, void* y, void* ws,
                            IgemmArgs* out)
{
    const int es = (int)dtype_size(d.dtype), kt_el = 128 / es;
    IgemmArgs& a = *out;
    a.x = (const unsigned char*)x; a.w = (const unsigned char*)w; a.y = (unsigned char*)y;
    a.scale = scale; a.shift = shift; a.res = (const unsigned char*)residual; a.partial = (float*)ws;
    a.H = d.h; a.W = d.w; a.Cin = d.cin; a.Cout = d.cout;
    a.P = out_dim(d.h, d.r, d.stride, d.pad); a.Q = out_dim(d.w, d.s, d.stride, d.pad);
    a.R = d.r; a.S = d.s; a.stride = d.stride; a.pad = d.pad;
    a.PQ = a.P * a.Q; a.M = d.n * a.PQ;
    fast_div_constants(a.PQ, &a.pq_mul, &a.pq_sh);
    fast_div_constants(a.Q, &a.q_mul, &a.q_sh);
    if (d.r > 3 || d.s > 3) return false;  // the tap masks of the loader hold 3 rows and 3 columns
    a.ktiles = p.ktiles; a.kt_per_split = (p.ktiles + p.splits - 1) / p.splits;
    a.cin_tiles = d.cin / kt_el; a.relu = d.relu;
    // x and w are addressed through 31-bit buffer offsets
    const long long xb = (long long)d.n * d.h * d.w * d.cin * es, wb = (long long)d.cout * d.r * d.s * d.cin * es;
    if (xb >= (1ll << 31) || wb >= (1ll << 31)) return false;
    a.x_bytes = (unsigned)xb; a.w_bytes = (unsigned)wb;
    return !(d.cin % kt_el || d.cout % p.bn || p.grid_m != (a.M + p.bm - 1) / p.bm || p.grid_n != d.cout / p.bn ||
             (long long)(p.splits - 1) * a.kt_per_split >= p.ktiles);
}

// Both convolutions in one launch when both plans are the same implicit-GEMM
// tile without split-K; *done = false (and nothing launched) otherwise.
int launch_conv_pair(const sgprs_conv_desc_t& d0, const void* w0, const float* scale0, const float* shift0, void* y0,
                     const sgprs_conv_desc_t& d1, const void* w1, const float* scale1, const float* shift1, void* y1,
                     const void* x, hipStream_t stream, int cus, Profiler* prof, bool* done)
{
    *done = false;
    if (d0.dtype != d1.dtype || d0.n != d1.n || d0.h != d1.h || d0.w != d1.w || d0.cin != d1.cin) return SGPRS_OK;
    const ConvPlan p0 = plan_conv(d0, cus);
    ConvPlan p1 = plan_conv(d1, cus);
    if (p0.bm == 0 || p0.kind != 0 || p0.splits != 1 || p1.bm == 0 || p1.kind != 0) return SGPRS_OK;
    // the second problem takes the first one's tile shape
    const int es = (int)dtype_size(d1.dtype);
    const long long M1 = (long long)d1.n * out_dim(d1.h, d1.r, d1.stride, d1.pad) * out_dim(d1.w, d1.s, d1.stride, d1.pad);
    if (d1.cout % p0.bn) return SGPRS_OK;
    p1.variant = p0.variant; p1.bm = p0.bm; p1.bn = p0.bn; p1.splits = 1;
    p1.grid_m = (int)((M1 + p0.bm - 1) / p0.bm); p1.grid_n = d1.cout / p0.bn;
    p1.ktiles = d1.r * d1.s * d1.cin / (128 / es);
    IgemmArgs a0, a1;
    if (!fill_igemm_args(d0, p0, x, w0, scale0, shift0, nullptr, y0, nullptr, &a0) ||
        !fill_igemm_args(d1, p1, x, w1, scale1, shift1, nullptr, y1, nullptr, &a1))
        return fail(SGPRS_ERR_INVALID_ARG, "internal: launch plan does not match the shape");
    const double flops = 2.0 * a0.M * d0.cout * (double)d0.r * d0.s * d0.cin + 2.0 * a1.M * d1.cout * (double)d1.r * d1.s * d1.cin;
    const double bytes = ((double)d0.n * d0.h * d0.w * d0.cin + (double)d0.cout * d0.r * d0.s * d0.cin +
                          (double)d1.cout * d1.r * d1.s * d1.cin + (double)a0.M * d0.cout + (double)a1.M * d1.cout) * es;
    int rc;
    if (prof && prof->on && (rc = prof->begin(stream, kKindIgemmPair, d0.dtype * 8 + p0.variant, flops, bytes))) return rc;
    rc = d0.dtype == SGPRS_BF16 ? launch_pair_dtype<SGPRS_BF16>(a0, p0, a1, p1, stream)
                                : launch_pair_dtype<SGPRS_F32>(a0, p0, a1, p1, stream);
    if (rc) return rc;
    if (prof && prof->on && (rc = prof->end(stream))) return rc;
    *done = true;
    return SGPRS_OK;
}

int launch_conv(const sgprs_conv_desc_t& d, const void* x, const void* w, const float* scale,
                const float* shift, const void* residual, void* y, void* ws, size_t ws_bytes,
                hipStream_t stream, int cus, Profiler* prof)
{
    const ConvPlan p = plan_conv(d, cus, residual != nullptr);
    if (p.bm == 0) return fail(SGPRS_ERR_UNSUPPORTED, "no tile shape fits cout %d", d.cout);
    if (p.kind == 1)
        return launch_conv3x3_patch(d, p.variant, p.splits, x, w, scale, shift, residual, y, ws, ws_bytes, stream, cus,
                                    prof);
    if (p.kind == 3) return launch_conv3x3_rows(d, p.variant, x, w, scale, shift, residual, y, stream, cus, prof);
    if (p.kind == 2) {
        return launch_conv3x3s2_patch(d, p.variant, x, w, scale, shift, y, nullptr, nullptr, nullptr, nullptr, nullptr, stream, cus,
                                      prof);
    }
    const size_t need = conv_workspace_bytes(d, p);
    if (need > ws_bytes || (need && !ws))
        return fail(SGPRS_ERR_INVALID_ARG, "split-K workspace %zu bytes needed, %zu given", need, ws_bytes);
    const int es = (int)dtype_size(d.dtype);
    IgemmArgs a;
    if (!fill_igemm_args(d, p, x, w, scale, shift, residual, y, ws, &a))
        return fail(SGPRS_ERR_INVALID_ARG, "internal: launch plan does not match the shape");
    const double flops = 2.0 * a.M * d.cout * (double)d.r * d.s * d.cin;
    const double bytes = ((double)d.n * d.h * d.w * d.cin + (double)d.cout * d.r * d.s * d.cin +
                          (double)a.M * d.cout * (residual ? 2 : 1)) * es;
    int rc;
    if (prof && prof->on && (rc = prof->begin(stream, kKindIgemm, d.dtype * 8 + p.variant + (p.splits > 1 ? 16 : 0), flops, bytes))) return rc;
    rc = d.dtype == SGPRS_BF16 ? launch_dtype<SGPRS_BF16>(a, p, stream) : launch_dtype<SGPRS_F32>(a, p, stream);
    if (rc) return rc;
    if (prof && prof->on && (rc = prof->end(stream))) return rc;
    if (p.splits > 1) {
        const size_t total = (size_t)a.M * d.cout;
        if (prof && prof->on &&
            (rc = prof->begin(stream, kKindReduce, d.dtype, 0.0, (double)total * 4.0 * p.splits + total * es)))
            return rc;
        if ((rc = launch_splitk_reduce(d.dtype, a.partial, p.splits, total, d.cout, scale, shift, a.res, a.y, d.relu,
                                       stream)))
            return rc;
        if (prof && prof->on && (rc = prof->end(stream))) return rc;
    }
    return SGPRS_OK;
}

}  // namespace sgprs
