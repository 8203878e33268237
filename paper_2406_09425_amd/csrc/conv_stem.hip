// Stem convolution: 7x7, stride 2, pad 3, 3 -> 64 channels, NHWC input.
//
// With 3 input channels the reduction length is only 147, and a k-tile of one
// tap would be 3 elements, so the generic implicit-GEMM loader does not fit.
// Here a workgroup stages the input patch of its TP x 16 output pixels in LDS
// once, zero-filled outside the image and with every pixel widened to 4
// channel slots, so that the 7 taps of one filter row are 28 contiguous,
// 16-byte aligned elements; the weights are packed to match (7 rows of 32,
// zeros in the unused slots) and also sit in LDS.  MFMA fragments are read
// straight from the patch: no predicates in the reduction loop.
// The op is bound by writing its 64 x 112 x 112 output, not by the MFMAs, so
// the 147/224 useful-k ratio costs little.
#include "internal.h"

namespace sgprs {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

struct StemArgs {
    const unsigned char* x;
    const unsigned char* w;
    unsigned char* y;
    const float* scale;
    const float* shift;
    int N, H, W, P, Q;
    int tiles_p, tiles_q, ntiles;
    int relu;
};

constexpr int kTQ = 16;                  // output columns per tile
constexpr int kPatchW = 2 * kTQ + 6;     // input columns staged (one spare for the padded 8th tap)

template <int DT, int TP>
__global__ __launch_bounds__(256) void conv_stem_kernel(const StemArgs a)
{
    constexpr int ES = DT == SGPRS_BF16 ? 2 : 4;
    constexpr int PIX = 4 * ES;                 // bytes per staged pixel (4 channel slots)
    constexpr int PATCH_H = 2 * TP + 5;
    constexpr int PATCH_BYTES = ((PATCH_H * kPatchW * PIX + 15) / 16) * 16;
    constexpr int WROW = kStemK * ES + 16;      // padded weight row: conflict-free fragment reads
    constexpr int BM = TP * kTQ;                // 128 or 64 output pixels
    constexpr int WM = BM / 32 >= 4 ? 4 : 2, WN = 4 / WM;
    constexpr int TM = BM / WM / 32, TN = 64 / WN / 32;
    static_assert(TM == 1 && TN >= 1, "tile shape");

    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char* Ws = smem;
    unsigned char* Ps = smem + 64 * WROW;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int frow = lane & 31, fhalf = lane >> 5;

    // weights -> LDS, once per workgroup
    for (int i = tid; i < 64 * (kStemK * ES / 16); i += 256) {
        const int row = i / (kStemK * ES / 16), ch = i - row * (kStemK * ES / 16);
        *(u32x4_t*)(Ws + row * WROW + ch * 16) = *(const u32x4_t*)(a.w + ((size_t)row * kStemK * ES) + ch * 16);
    }

    for (int tile = blockIdx.x; tile < a.ntiles; tile += gridDim.x) {
        const int n = tile / (a.tiles_p * a.tiles_q), t2 = tile - n * (a.tiles_p * a.tiles_q);
        const int p0 = (t2 / a.tiles_q) * TP, q0 = (t2 % a.tiles_q) * kTQ;
        const int h_base = 2 * p0 - 3, w_base = 2 * q0 - 3;

        __syncthreads();  // previous tile's fragment reads are done
        for (int i = tid; i < PATCH_H * kPatchW; i += 256) {
            const int pr = i / kPatchW, pc = i - pr * kPatchW;
            const int ih = h_base + pr, iw = w_base + pc;
            const bool ok = (unsigned)ih < (unsigned)a.H && (unsigned)iw < (unsigned)a.W;
            const size_t g = ((size_t)(n * a.H + (ok ? ih : 0)) * a.W + (ok ? iw : 0)) * 3;
            if constexpr (DT == SGPRS_BF16) {
                const unsigned short* xp = (const unsigned short*)a.x + g;
                unsigned short v0 = 0, v1 = 0, v2 = 0;
                if (ok) { v0 = xp[0]; v1 = xp[1]; v2 = xp[2]; }
                uint2 o;
                o.x = (unsigned)v0 | ((unsigned)v1 << 16);
                o.y = (unsigned)v2;
                *(uint2*)(Ps + i * PIX) = o;
            } else {
                const float* xp = (const float*)a.x + g;
                float4 o = {0.f, 0.f, 0.f, 0.f};
                if (ok) { o.x = xp[0]; o.y = xp[1]; o.z = xp[2]; }
                *(float4*)(Ps + i * PIX) = o;
            }
        }
        __syncthreads();

        f32x16_t acc[TN];
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;

        // this lane's output pixel inside the tile (A-fragment row)
        const int pix = wm * 32 + frow;
        const int pp = pix / kTQ, qq = pix % kTQ;
        const unsigned char* prow = Ps + ((2 * pp) * kPatchW + 2 * qq) * PIX;
        const unsigned char* wbase = Ws + (wn * (64 / WN) + frow) * WROW;

#pragma unroll
        for (int r = 0; r < 7; ++r) {
            if constexpr (DT == SGPRS_BF16) {
                // tap row = 32 elements = 4 chunks of 8; one MFMA eats 2 chunks
#pragma unroll
                for (int ks = 0; ks < 2; ++ks) {
                    const int chunk = 2 * ks + fhalf;
                    const u32x4_t af = *(const u32x4_t*)(prow + r * kPatchW * PIX + chunk * 16);
#pragma unroll
                    for (int j = 0; j < TN; ++j) {
                        const u32x4_t bf = *(const u32x4_t*)(wbase + j * 32 * WROW + (r * kStemTapRow * ES) + chunk * 16);
                        acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, af),
                                                                       __builtin_bit_cast(bf16x8_t, bf), acc[j], 0, 0, 0);
                    }
                }
            } else {
                // tap row = 32 floats = 8 chunks of 4 (one tap each); a pair of
                // chunks feeds 4 MFMAs of k = 2
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    const int chunk = 2 * ks + fhalf;
                    const u32x4_t af = *(const u32x4_t*)(prow + r * kPatchW * PIX + chunk * 16);
#pragma unroll
                    for (int j = 0; j < TN; ++j) {
                        const u32x4_t bf = *(const u32x4_t*)(wbase + j * 32 * WROW + (r * kStemTapRow * ES) + chunk * 16);
#pragma unroll
                        for (int u = 0; u < 3; ++u)  // slot 3 is the zero channel
                            acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(af[u]), __uint_as_float(bf[u]),
                                                                         acc[j], 0, 0, 0);
                    }
                }
            }
        }

        // epilogue: column = lane%32 -> channel, row -> pixel in tile
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int k = wn * (64 / WN) + j * 32 + frow;
            const float sc = a.scale[k], sh = a.shift[k];
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int opix = wm * 32 + 8 * (e >> 2) + 4 * fhalf + (e & 3);
                const int p = p0 + opix / kTQ, q = q0 + opix % kTQ;
                if (p >= a.P || q >= a.Q) continue;
                float v = acc[j][e] * sc + sh;
                if (a.relu) v = fmaxf(v, 0.f);
                const size_t o = ((size_t)(n * a.P + p) * a.Q + q) * 64 + k;
                if constexpr (DT == SGPRS_BF16) {
                    __bf16 hv = (__bf16)v;
                    ((unsigned short*)a.y)[o] = __builtin_bit_cast(unsigned short, hv);
                } else {
                    ((float*)a.y)[o] = v;
                }
            }
        }
    }
}

template <int DT, int TP>
static int launch_stem_variant(const StemArgs& a, int grid, hipStream_t stream)
{
    constexpr int ES = DT == SGPRS_BF16 ? 2 : 4;
    constexpr int PATCH_BYTES = (((2 * TP + 5) * kPatchW * 4 * ES + 15) / 16) * 16;
    const size_t lds = 64 * (kStemK * ES + 16) + PATCH_BYTES;
    static std::atomic<bool> raised{false};  // more than 64 KB of dynamic LDS needs an explicit opt-in
    if (lds > 65536 && !raised) {
        SGPRS_HIP(hipFuncSetAttribute((const void*)conv_stem_kernel<DT, TP>,
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        raised = true;
    }
    SGPRS_LAUNCH((conv_stem_kernel<DT, TP>), dim3(grid), dim3(256), lds, stream, a);
    SGPRS_HIP(hipGetLastError());
    return SGPRS_OK;
}

int launch_stem(const sgprs_conv_desc_t& d, const void* x, const void* w, const float* scale,
                const float* shift, void* y, hipStream_t stream, int cus, Profiler* prof)
{
    if (d.cout != 64) return fail(SGPRS_ERR_UNSUPPORTED, "stem conv needs cout == 64 (got %d)", d.cout);
    StemArgs a;
    a.x = (const unsigned char*)x; a.w = (const unsigned char*)w; a.y = (unsigned char*)y;
    a.scale = scale; a.shift = shift;
    a.N = d.n; a.H = d.h; a.W = d.w;
    a.P = out_dim(d.h, 7, 2, 3); a.Q = out_dim(d.w, 7, 2, 3);
    a.relu = d.relu;
    a.tiles_q = (a.Q + kTQ - 1) / kTQ;
    // 8-row tiles unless that leaves CUs idle
    const long long tiles8 = (long long)d.n * ((a.P + 7) / 8) * a.tiles_q;
    const int tp = tiles8 >= 2ll * cus ? 8 : 4;
    a.tiles_p = (a.P + tp - 1) / tp;
    const long long nt = (long long)d.n * a.tiles_p * a.tiles_q;
    if (nt >= (1ll << 31)) return fail(SGPRS_ERR_UNSUPPORTED, "too many stem tiles");
    a.ntiles = (int)nt;
    const int grid = (int)std::min<long long>(nt, 4ll * cus);
    const double flops = 2.0 * d.n * a.P * a.Q * 64.0 * 147.0;
    const double bytes = ((double)d.n * d.h * d.w * 3 + 64.0 * 147 + (double)d.n * a.P * a.Q * 64) * dtype_size(d.dtype);
    int rc;
    if (prof && prof->on && (rc = prof->begin(stream, kKindStem, d.dtype * 2 + (tp == 8 ? 0 : 1), flops, bytes))) return rc;
    if (d.dtype == SGPRS_BF16)
        rc = tp == 8 ? launch_stem_variant<SGPRS_BF16, 8>(a, grid, stream) : launch_stem_variant<SGPRS_BF16, 4>(a, grid, stream);
    else
        rc = tp == 8 ? launch_stem_variant<SGPRS_F32, 8>(a, grid, stream) : launch_stem_variant<SGPRS_F32, 4>(a, grid, stream);
    if (rc) return rc;
    if (prof && prof->on && (rc = prof->end(stream))) return rc;
    return SGPRS_OK;
}

}  // namespace sgprs
