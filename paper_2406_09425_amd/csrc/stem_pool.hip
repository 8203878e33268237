// Stage 0 in one kernel: conv 7x7/2 (3 -> 64) + folded BN + ReLU + max-pool 3x3/2.
//
// The stem's 64 x 112 x 112 output is the largest tensor of the network; written
// out and read back by a separate pooling kernel it costs more HBM traffic than
// everything else in the stage.  Here a workgroup owns 7 x 8 pooled pixels.  It
// computes the 15 x 17 conv pixels they depend on (255 rows of a 256-row MFMA
// tile; the overlap between neighbouring tiles is recomputed), keeps them in
// LDS, pools there and writes only the pooled 16-byte vectors.
//
// As in the stand-alone stem kernel the input patch is staged in LDS with 4
// channel slots per pixel and zero fill outside the image, and the weights sit
// in LDS in the matching 7 x 32 tap-row layout.  The MFMA operands are swapped
// (weights as the row operand, pixels as the column operand) so that a lane's
// accumulator registers hold 4 consecutive channels of one pixel, which go to
// the LDS staging area as one 8-byte (bf16) or 16-byte (fp32) write.
// Positions outside the conv output hold -inf (fp32) or 0 (bf16, where the
// post-ReLU values are pooled as unsigned bit patterns) in the staging area, so
// padding never wins the maximum.
#include "internal.h"

namespace sgprs {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
typedef unsigned short u16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

struct StemPoolArgs {
    const unsigned char* x;
    const unsigned char* w;
    unsigned char* y;
    const float* scale;
    const float* shift;
    int N, H, W;      // input
    int P, Q;         // conv output
    int PP, PQ;       // pooled output
    int tiles_p, tiles_q, ntiles;
};

constexpr int kPoolTP = 7, kPoolTQ = 8;           // pooled pixels per tile
constexpr int kConvR = 2 * kPoolTP + 1;           // 15 conv rows
constexpr int kConvC = 2 * kPoolTQ + 1;           // 17 conv columns
constexpr int kInR = 2 * kConvR + 5;              // 35 input rows
constexpr int kInC = 2 * kConvC + 6;              // 40 input columns (one spare for the padded 8th tap)

template <int DT>
__global__ __launch_bounds__(256) void stem_pool_kernel(const StemPoolArgs a)
{
    constexpr int ES = DT == SGPRS_BF16 ? 2 : 4;
    constexpr int PIX = 4 * ES;                      // staged input pixel: 4 channel slots
    constexpr int WROW = kStemK * ES + 16;           // padded weight row
    constexpr int W_BYTES = 64 * WROW;
    constexpr int SROWB = 64 * ES + 16;              // staged conv pixel: 64 channels + pad
    constexpr int PATCH_BYTES = kInR * kInC * PIX;
    constexpr int STG_BYTES = 256 * SROWB;
    constexpr int BUF_BYTES = PATCH_BYTES > STG_BYTES ? PATCH_BYTES : STG_BYTES;

    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char* Ws = smem;
    unsigned char* Ps = smem + W_BYTES;              // patch, later the conv staging area

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int frow = lane & 31, fhalf = lane >> 5;

    for (int i = tid; i < 64 * (kStemK * ES / 16); i += 256) {
        const int row = i / (kStemK * ES / 16), ch = i - row * (kStemK * ES / 16);
        *(u32x4_t*)(Ws + row * WROW + ch * 16) = *(const u32x4_t*)(a.w + (size_t)row * kStemK * ES + ch * 16);
    }

    // The next tile's input patch is fetched into registers while the current
    // tile computes: PF_IT pixels per thread, 3 channels each.
    constexpr int PF_IT = (kInR * kInC + 255) / 256;
    unsigned pf_lo[PF_IT], pf_hi[PF_IT], pf_x[DT == SGPRS_BF16 ? 1 : PF_IT];
    auto fetch_patch = [&](int tile) {
        const int n = tile / (a.tiles_p * a.tiles_q), t2 = tile - n * (a.tiles_p * a.tiles_q);
        const int pp0 = (t2 / a.tiles_q) * kPoolTP, pq0 = (t2 % a.tiles_q) * kPoolTQ;
        const int h_base = 2 * (2 * pp0 - 1) - 3, w_base = 2 * (2 * pq0 - 1) - 3;
#pragma unroll
        for (int it = 0; it < PF_IT; ++it) {
            const int i = it * 256 + tid;
            const int pr = i / kInC, pc = i - pr * kInC;
            const int ih = h_base + pr, iw = w_base + pc;
            const bool ok = i < kInR * kInC && (unsigned)ih < (unsigned)a.H && (unsigned)iw < (unsigned)a.W;
            const size_t g = ((size_t)(n * a.H + (ok ? ih : 0)) * a.W + (ok ? iw : 0)) * 3;
            if constexpr (DT == SGPRS_BF16) {
                const unsigned short* xp = (const unsigned short*)a.x + g;
                // unconditional loads from a clamped (always valid) pixel, zeroed afterwards:
                // nothing waits on a branch, all loads of the patch are in flight together
                const unsigned v0 = xp[0], v1 = xp[1], v2 = xp[2];
                pf_lo[it] = ok ? v0 | (v1 << 16) : 0u;
                pf_hi[it] = ok ? v2 : 0u;
            } else {
                const unsigned* xp = (const unsigned*)a.x + g;
                const unsigned v0 = xp[0], v1 = xp[1], v2 = xp[2];
                pf_lo[it] = ok ? v0 : 0u; pf_hi[it] = ok ? v1 : 0u; pf_x[it] = ok ? v2 : 0u;
            }
        }
    };
    auto store_patch = [&]() {
#pragma unroll
        for (int it = 0; it < PF_IT; ++it) {
            const int i = it * 256 + tid;
            if (i >= kInR * kInC) continue;
            if constexpr (DT == SGPRS_BF16) {
                u32x2_t o = {pf_lo[it], pf_hi[it]};
                *(u32x2_t*)(Ps + i * PIX) = o;
            } else {
                u32x4_t o = {pf_lo[it], pf_hi[it], pf_x[it], 0u};
                *(u32x4_t*)(Ps + i * PIX) = o;
            }
        }
    };

    // this lane's BN scale / shift: accumulator register 4g+u of channel tile i is channel 32i + 8g + 4*fhalf + u
    f32x4_t sc[2][4], sh[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            sc[i][g] = *(const f32x4_t*)(a.scale + 32 * i + 8 * g + 4 * fhalf);
            sh[i][g] = *(const f32x4_t*)(a.shift + 32 * i + 8 * g + 4 * fhalf);
        }

    if ((int)blockIdx.x < a.ntiles) fetch_patch(blockIdx.x);
    for (int tile = blockIdx.x; tile < a.ntiles; tile += gridDim.x) {
        const int n = tile / (a.tiles_p * a.tiles_q), t2 = tile - n * (a.tiles_p * a.tiles_q);
        const int pp0 = (t2 / a.tiles_q) * kPoolTP, pq0 = (t2 % a.tiles_q) * kPoolTQ;
        const int cr0 = 2 * pp0 - 1, cc0 = 2 * pq0 - 1;   // first conv row / column of the tile

        __syncthreads();  // the previous tile's pooling reads are done
        store_patch();
        __syncthreads();
        if (tile + (int)gridDim.x < a.ntiles) fetch_patch(tile + gridDim.x);

        // accumulators: [channel tile i][pixel tile j]; this wavefront owns conv
        // pixels 64*wave .. 64*wave+63 of the tile (pixel t = row*17 + column)
        f32x16_t acc[2][2];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

        int poff[2];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            int t = wave * 64 + j * 32 + frow;
            if (t >= kConvR * kConvC) t = 0;  // the one padding row of the 256-row tile: computed, never used
            const int cr = t / kConvC, cc = t - cr * kConvC;
            poff[j] = ((2 * cr) * kInC + 2 * cc) * PIX;
        }
        const unsigned char* wbase = Ws + frow * WROW;

#pragma unroll
        for (int r = 0; r < 7; ++r) {
            constexpr int KSTEPS = DT == SGPRS_BF16 ? 2 : 4;
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks) {
                const int chunk = 2 * ks + fhalf;
                u32x4_t pf[2], wf[2];
#pragma unroll
                for (int j = 0; j < 2; ++j) pf[j] = *(const u32x4_t*)(Ps + poff[j] + r * kInC * PIX + chunk * 16);
#pragma unroll
                for (int i = 0; i < 2; ++i) wf[i] = *(const u32x4_t*)(wbase + i * 32 * WROW + r * kStemTapRow * ES + chunk * 16);
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        if constexpr (DT == SGPRS_BF16) {
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, wf[i]),
                                                                              __builtin_bit_cast(bf16x8_t, pf[j]), acc[i][j], 0, 0, 0);
                        } else {
#pragma unroll
                            for (int u = 0; u < 3; ++u)  // slot 3 is the zero channel
                                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(wf[i][u]), __uint_as_float(pf[j][u]),
                                                                                acc[i][j], 0, 0, 0);
                        }
                    }
            }
        }

        __syncthreads();  // every wavefront is done with the patch: reuse it as the staging area

        // accumulator register e: column lane%32 = pixel, row 8*(e/4) + 4*(lane/32) + e%4 = channel
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int t = wave * 64 + j * 32 + frow;
            const int cr = t / kConvC, cc = t - cr * kConvC;
            const int crow = cr0 + cr, ccol = cc0 + cc;
            const bool ok = t < kConvR * kConvC && (unsigned)crow < (unsigned)a.P && (unsigned)ccol < (unsigned)a.Q;
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int c = 32 * i + 8 * g + 4 * fhalf;
                    float v[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) v[u] = fmaxf(acc[i][j][4 * g + u] * sc[i][g][u] + sh[i][g][u], 0.f);
                    if constexpr (DT == SGPRS_BF16) {
                        // After the ReLU every value is >= 0, so pooling can compare bf16 bit
                        // patterns as unsigned integers and positions outside the conv output
                        // hold 0: each pooling window has a real pixel, so 0 never wins wrongly.
                        // The sign bit is cleared so that a -0 cannot compare as large.
                        const f32x2_t p0 = {v[0], v[1]}, p1 = {v[2], v[3]};
                        const unsigned keep = ok ? 0x7fff7fffu : 0u;
                        u32x2_t o = {__builtin_bit_cast(unsigned, __builtin_convertvector(p0, bf16x2_t)) & keep,
                                     __builtin_bit_cast(unsigned, __builtin_convertvector(p1, bf16x2_t)) & keep};
                        *(u32x2_t*)(Ps + t * SROWB + c * 2) = o;
                    } else {
                        f32x4_t o = {ok ? v[0] : -INFINITY, ok ? v[1] : -INFINITY, ok ? v[2] : -INFINITY, ok ? v[3] : -INFINITY};
                        *(f32x4_t*)(Ps + t * SROWB + c * 4) = o;
                    }
                }
        }
        __syncthreads();

        // pooling: one item = (pooled pixel, 16-byte channel group)
        constexpr int GROUPS = 64 * ES / 16;
        for (int it = tid; it < kPoolTP * kPoolTQ * GROUPS; it += 256) {
            const int grp = it % GROUPS, px = it / GROUPS;
            const int lp = px / kPoolTQ, lq = px - lp * kPoolTQ;
            const int gp = pp0 + lp, gq = pq0 + lq;
            if (gp >= a.PP || gq >= a.PQ) continue;
            const unsigned char* base = Ps + ((2 * lp) * kConvC + 2 * lq) * SROWB + grp * 16;
            u32x4_t m = *(const u32x4_t*)base;
#pragma unroll
            for (int rs = 1; rs < 9; ++rs) {
                const u32x4_t t = *(const u32x4_t*)(base + ((rs / 3) * kConvC + rs % 3) * SROWB);
                if constexpr (DT == SGPRS_BF16) {
                    // whole-vector form: eight unsigned 16-bit maxima per tap
                    m = __builtin_bit_cast(u32x4_t, __builtin_elementwise_max(__builtin_bit_cast(u16x8_t, m),
                                                                              __builtin_bit_cast(u16x8_t, t)));
                } else {
#pragma unroll
                    for (int u = 0; u < 4; ++u) m[u] = __float_as_uint(fmaxf(__uint_as_float(m[u]), __uint_as_float(t[u])));
                }
            }
            *(u32x4_t*)(a.y + (((size_t)(n * a.PP + gp) * a.PQ + gq) * 64) * ES + grp * 16) = m;
        }
    }
}

bool stem_pool_applicable(int dtype, int n, int h, int w, int cus)
{
    const int P = out_dim(h, 7, 2, 3), Q = out_dim(w, 7, 2, 3);
    const int PP = (P - 1) / 2 + 1, PQ = (Q - 1) / 2 + 1;
    const long long tiles = (long long)n * ((PP + kPoolTP - 1) / kPoolTP) * ((PQ + kPoolTQ - 1) / kPoolTQ);
    // smaller launches keep the finer-grained two-kernel path; in bf16 the fused kernel wins down
    // to one image (9.4 us against 8.5 + 4.9 us at batch 1), in fp32 it does not (17.9 against 16.3)
    return dtype == SGPRS_BF16 ? tiles >= 32 : tiles >= 2ll * cus;
}

int launch_stem_pool(int dtype, int n, int h, int w, const void* x, const void* wts, const float* scale,
                     const float* shift, void* y, hipStream_t stream, int cus, Profiler* prof)
{
    StemPoolArgs a;
    a.x = (const unsigned char*)x; a.w = (const unsigned char*)wts; a.y = (unsigned char*)y;
    a.scale = scale; a.shift = shift;
    a.N = n; a.H = h; a.W = w;
    a.P = out_dim(h, 7, 2, 3); a.Q = out_dim(w, 7, 2, 3);
    a.PP = (a.P - 1) / 2 + 1; a.PQ = (a.Q - 1) / 2 + 1;
    a.tiles_p = (a.PP + kPoolTP - 1) / kPoolTP; a.tiles_q = (a.PQ + kPoolTQ - 1) / kPoolTQ;
    const long long nt = (long long)n * a.tiles_p * a.tiles_q;
    if (nt >= (1ll << 31)) return fail(SGPRS_ERR_UNSUPPORTED, "too many stem tiles");
    a.ntiles = (int)nt;
    const int es = (int)dtype_size(dtype);
    const int patch = kInR * kInC * 4 * es, stg = 256 * (64 * es + 16);
    const size_t lds = 64 * (kStemK * es + 16) + (patch > stg ? patch : stg);
    const int occ = lds <= 80 * 1024 ? 2 : 1;
    const int grid = (int)std::min<long long>(nt, (long long)cus * occ);
    const double flops = 2.0 * n * a.P * a.Q * 64.0 * 147.0;
    const double bytes = ((double)n * h * w * 3 + 64.0 * 147 + (double)n * a.PP * a.PQ * 64) * es;
    int rc;
    if (prof && prof->on && (rc = prof->begin(stream, kKindStemPool, dtype, flops, bytes))) return rc;
    static std::atomic<bool> raised[2] = {{false}, {false}};
    if (dtype == SGPRS_BF16) {
        if (!raised[1]) {
            SGPRS_HIP(hipFuncSetAttribute((const void*)stem_pool_kernel<SGPRS_BF16>,
                                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
            raised[1] = true;
        }
        SGPRS_LAUNCH(stem_pool_kernel<SGPRS_BF16>, dim3(grid), dim3(256), lds, stream, a);
    } else {
        if (!raised[0]) {
            SGPRS_HIP(hipFuncSetAttribute((const void*)stem_pool_kernel<SGPRS_F32>,
                                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
            raised[0] = true;
        }
        SGPRS_LAUNCH(stem_pool_kernel<SGPRS_F32>, dim3(grid), dim3(256), lds, stream, a);
    }
    SGPRS_HIP(hipGetLastError());
    if (prof && prof->on && (rc = prof->end(stream))) return rc;
    return SGPRS_OK;
}

}  // namespace sgprs
