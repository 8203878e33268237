// Memory-bound operators of the ResNet18 stages: max pooling, folded BN+ReLU,
// residual add, global average pool and the fully connected layer (the
// "max pooling" and "other operations" of the paper's "GPU Speedup
// Analysis"), plus the partition placement probe.  All of them move 16 bytes
// per lane per access, coalesced along the NHWC channel axis; none of them is
// a contraction worth the matrix cores except the batched FC, which is tiny.
#include "internal.h"

namespace sgprs {

typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

// 16 bytes of activations as floats: 4 (fp32) or 8 (bf16) lanes.
template <int DT> struct Vec;
template <> struct Vec<SGPRS_F32> {
    static constexpr int N = 4;
    float v[4];
    __device__ __forceinline__ void load(const void* p, size_t vec_index)
    {
        const f32x4_t t = ((const f32x4_t*)p)[vec_index];
        v[0] = t[0]; v[1] = t[1]; v[2] = t[2]; v[3] = t[3];
    }
    __device__ __forceinline__ void store(void* p, size_t vec_index) const
    {
        f32x4_t t = {v[0], v[1], v[2], v[3]};
        ((f32x4_t*)p)[vec_index] = t;
    }
    // streaming forms for data touched once: they do not displace reusable lines from L2
    __device__ __forceinline__ void load_nt(const void* p, size_t vec_index)
    {
        const f32x4_t t = __builtin_nontemporal_load((const f32x4_t*)p + vec_index);
        v[0] = t[0]; v[1] = t[1]; v[2] = t[2]; v[3] = t[3];
    }
    __device__ __forceinline__ void store_nt(void* p, size_t vec_index) const
    {
        f32x4_t t = {v[0], v[1], v[2], v[3]};
        __builtin_nontemporal_store(t, (f32x4_t*)p + vec_index);
    }
};
template <> struct Vec<SGPRS_BF16> {
    static constexpr int N = 8;
    float v[8];
    __device__ __forceinline__ void load(const void* p, size_t vec_index)
    {
        const u32x4_t t = ((const u32x4_t*)p)[vec_index];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = __uint_as_float(t[i] << 16);
            v[2 * i + 1] = __uint_as_float(t[i] & 0xffff0000u);
        }
    }
    __device__ __forceinline__ void store(void* p, size_t vec_index) const
    {
        u32x4_t t;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const __bf16 lo = (__bf16)v[2 * i], hi = (__bf16)v[2 * i + 1];  // nearest even
            t[i] = (unsigned)__builtin_bit_cast(unsigned short, lo) |
                   ((unsigned)__builtin_bit_cast(unsigned short, hi) << 16);
        }
        ((u32x4_t*)p)[vec_index] = t;
    }
    __device__ __forceinline__ void load_nt(const void* p, size_t vec_index)
    {
        const u32x4_t t = __builtin_nontemporal_load((const u32x4_t*)p + vec_index);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = __uint_as_float(t[i] << 16);
            v[2 * i + 1] = __uint_as_float(t[i] & 0xffff0000u);
        }
    }
    __device__ __forceinline__ void store_nt(void* p, size_t vec_index) const
    {
        u32x4_t t;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const __bf16 lo = (__bf16)v[2 * i], hi = (__bf16)v[2 * i + 1];  // nearest even
            t[i] = (unsigned)__builtin_bit_cast(unsigned short, lo) |
                   ((unsigned)__builtin_bit_cast(unsigned short, hi) << 16);
        }
        __builtin_nontemporal_store(t, (u32x4_t*)p + vec_index);
    }
};

// ---- max pool 3x3 stride 2 pad 1 -------------------------------------------
// One thread = one 16-byte channel vector of two vertically adjacent output
// pixels: the five input rows they need are read once (the middle row is
// shared), 15 loads for 2 outputs.  All index arithmetic is 32-bit.
template <int DT>
__global__ __launch_bounds__(256) void maxpool3x3s2_kernel(const void* __restrict__ x, void* __restrict__ y,
                                                           int H, int W, int C, int P, int Q, unsigned total_items)
{
    constexpr int N = Vec<DT>::N;
    // Workgroup b runs on die b % 8: give each die a contiguous band of the
    // output so that input rows shared by neighbouring output rows hit in that
    // die's L2 instead of being fetched once per die.
    const unsigned per_die = (gridDim.x + 7) / 8;
    const unsigned vb = (blockIdx.x % 8) * per_die + blockIdx.x / 8;
    const unsigned idx = vb * 256 + threadIdx.x;
    if (idx >= total_items) return;
    const unsigned cv = C / N, P2 = (P + 1) / 2;
    const unsigned c = idx % cv;
    unsigned t = idx / cv;
    const int q = (int)(t % Q);
    t /= Q;
    const int p0 = 2 * (int)(t % P2);
    const int n = (int)(t / P2);
    // All 15 loads are issued unconditionally from clamped (always valid)
    // coordinates so that they are in flight together; taps outside the image
    // are replaced by -inf afterwards (padding never wins).
    Vec<DT> v[5][3];
    bool rok[5], cok[3];
#pragma unroll
    for (int r = 0; r < 5; ++r) {
        const int ih = 2 * p0 - 1 + r;
        rok[r] = (unsigned)ih < (unsigned)H;
        const int ihc = min(max(ih, 0), H - 1);
#pragma unroll
        for (int s = 0; s < 3; ++s) {
            const int iw = 2 * q - 1 + s;
            cok[s] = (unsigned)iw < (unsigned)W;
            const int iwc = min(max(iw, 0), W - 1);
            // the three middle rows belong to this thread's two outputs alone: streamed past the caches;
            // the outer two are shared with the neighbouring output rows (other workgroups) and stay cached
            if (r >= 1 && r <= 3) v[r][s].load_nt(x, ((size_t)(n * H + ihc) * W + iwc) * cv + c);
            else v[r][s].load(x, ((size_t)(n * H + ihc) * W + iwc) * cv + c);
        }
    }
    Vec<DT> m0, m1;
#pragma unroll
    for (int i = 0; i < N; ++i) { m0.v[i] = -INFINITY; m1.v[i] = -INFINITY; }
#pragma unroll
    for (int r = 0; r < 5; ++r) {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            float rm = -INFINITY;  // horizontal maximum of this input row's three taps
#pragma unroll
            for (int s = 0; s < 3; ++s) rm = fmaxf(rm, (rok[r] && cok[s]) ? v[r][s].v[i] : -INFINITY);
            if (r <= 2) m0.v[i] = fmaxf(m0.v[i], rm);
            if (r >= 2) m1.v[i] = fmaxf(m1.v[i], rm);
        }
    }
    m0.store_nt(y, ((size_t)(n * P + p0) * Q + q) * cv + c);
    if (p0 + 1 < P) m1.store_nt(y, ((size_t)(n * P + p0 + 1) * Q + q) * cv + c);
}

// ---- y = max(0, scale*x + shift) -------------------------------------------
template <int DT>
__global__ __launch_bounds__(256) void bn_relu_kernel(const void* __restrict__ x, void* __restrict__ y,
                                                      const float* __restrict__ scale,
                                                      const float* __restrict__ shift, int C, size_t total_vec)
{
    constexpr int N = Vec<DT>::N;
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total_vec) return;
    // (block * 256 + thread) mod cv without a 64-bit division
    const unsigned cv = C / N;
    const int c0 = (int)((((unsigned)(blockIdx.x % cv) * (256u % cv)) + threadIdx.x) % cv) * N;
    Vec<DT> t;
    t.load_nt(x, idx);
#pragma unroll
    for (int i = 0; i < N; ++i) t.v[i] = fmaxf(t.v[i] * scale[c0 + i] + shift[c0 + i], 0.f);
    t.store_nt(y, idx);
}

// ---- y = a + b (ReLU optional) ---------------------------------------------
template <int DT>
__global__ __launch_bounds__(256) void add_relu_kernel(const void* __restrict__ a, const void* __restrict__ b,
                                                       void* __restrict__ y, int relu, size_t total_vec)
{
    constexpr int N = Vec<DT>::N;
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total_vec) return;
    Vec<DT> s, t;
    s.load_nt(a, idx);
    t.load_nt(b, idx);
#pragma unroll
    for (int i = 0; i < N; ++i) {
        s.v[i] += t.v[i];
        if (relu) s.v[i] = fmaxf(s.v[i], 0.f);
    }
    s.store_nt(y, idx);
}

// ---- global average pool: x [n][hw][c] -> v [n][c] fp32 ---------------------
// One workgroup per (image, 64 channel vectors): the four wavefronts take
// every fourth position, partial sums meet in LDS and are added in wavefront
// order, so the result does not depend on timing.
template <int DT>
__global__ __launch_bounds__(256) void avgpool_kernel(const void* __restrict__ x, float* __restrict__ v, int HW,
                                                      int C)
{
    constexpr int N = Vec<DT>::N;
    __shared__ float part[4][64][N];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int cv = C / N;
    const int c = blockIdx.x * 64 + lane;
    const size_t n = blockIdx.y;
    float s[N];
#pragma unroll
    for (int i = 0; i < N; ++i) s[i] = 0.f;
    if (c < cv) {
        int j = wave;
        for (; j + 12 < HW; j += 16) {  // four positions per round trip
            Vec<DT> t[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) t[u].load(x, (n * HW + j + 4 * u) * cv + c);
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int i = 0; i < N; ++i) s[i] += t[u].v[i];
        }
        for (; j < HW; j += 4) {
            Vec<DT> t;
            t.load(x, (n * HW + j) * cv + c);
#pragma unroll
            for (int i = 0; i < N; ++i) s[i] += t.v[i];
        }
    }
#pragma unroll
    for (int i = 0; i < N; ++i) part[wave][lane][i] = s[i];
    __syncthreads();
    if (wave == 0 && c < cv) {
        const float hw = (float)HW;
#pragma unroll
        for (int i = 0; i < N; ++i)
            v[(n * cv + c) * N + i] = (((part[0][lane][i] + part[1][lane][i]) + part[2][lane][i]) + part[3][lane][i]) / hw;
    }
}

// ---- the same for many images ------------------------------------------------
// One wavefront per (image, 64 channel vectors), four images per workgroup, nothing shared: a lane
// keeps four partial sums, over the positions j = 0, 1, 2, 3 (mod 4) in rising order, and adds them as
// ((p0 + p1) + p2) + p3: the arithmetic of the one-launch kernel below, whose four wavefronts take one
// residue each.  Up to 28 positions are in flight per round trip; the data is touched once (streamed).
template <int DT>
__global__ __launch_bounds__(256) void avgpool_stream_kernel(const void* __restrict__ x, float* __restrict__ v, int HW,
                                                             int C, int Nimg)
{
    constexpr int N = Vec<DT>::N, B = 28;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int cv = C / N;
    const int c = blockIdx.x * 64 + lane;
    const size_t n = (size_t)blockIdx.y * 4 + wave;
    if (n >= (size_t)Nimg || c >= cv) return;
    float p[4][N];
#pragma unroll
    for (int w = 0; w < 4; ++w)
#pragma unroll
        for (int i = 0; i < N; ++i) p[w][i] = 0.f;
    for (int j0 = 0; j0 < HW; j0 += B) {
        Vec<DT> t[B];
#pragma unroll
        for (int u = 0; u < B; ++u) t[u].load_nt(x, (n * HW + min(j0 + u, HW - 1)) * cv + c);
#pragma unroll
        for (int u = 0; u < B; ++u)
            if (j0 + u < HW) {
#pragma unroll
                for (int i = 0; i < N; ++i) p[u & 3][i] += t[u].v[i];   // (B is a multiple of 4: position j feeds partial sum j & 3)
            }
    }
    const float hw = (float)HW;
#pragma unroll
    for (int i = 0; i < N; ++i) v[(n * cv + c) * N + i] = (((p[0][i] + p[1][i]) + p[2][i]) + p[3][i]) / hw;
}

// ---- avg-pool + FC in one launch, for a few images ---------------------------------
// Every workgroup pools its image once more (the 50 KB come from the L2) with exactly the
// arithmetic of avgpool_kernel, keeps the vector in LDS, and its four wavefronts then compute
// four output rows each with exactly the arithmetic of fc_kernel: one kernel less at batch 1-8,
// the same bits.
template <int DT, int CPL /* 512-element passes */>
__global__ __launch_bounds__(256) void avgpool_fc_kernel(const void* __restrict__ x, const void* __restrict__ w,
                                                         const float* __restrict__ bias, float* __restrict__ y, int HW,
                                                         int Cout)
{
    constexpr int N = Vec<DT>::N, C = CPL * 512, CV = C / N, VP = CV / 64, R = 4;
    __shared__ float part[4][CV][N];
    __shared__ __align__(16) float pooled[C];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const size_t n = blockIdx.y;
    // the weight rows do not depend on the pooling: fetch them first so both latencies overlap
    float wr[R][CPL][8];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int o = min((int)(blockIdx.x * 4 + wave) * R + r, Cout - 1);
#pragma unroll
        for (int j = 0; j < CPL; ++j) {
            const size_t e0 = (size_t)o * C + j * 512 + lane * 8;
            if constexpr (DT == SGPRS_BF16) {
                Vec<SGPRS_BF16> t;
                t.load(w, e0 / 8);
#pragma unroll
                for (int i = 0; i < 8; ++i) wr[r][j][i] = t.v[i];
            } else {
                Vec<SGPRS_F32> t0, t1;
                t0.load(w, e0 / 4);
                t1.load(w, e0 / 4 + 1);
#pragma unroll
                for (int i = 0; i < 4; ++i) { wr[r][j][i] = t0.v[i]; wr[r][j][4 + i] = t1.v[i]; }
            }
        }
    }
#pragma unroll
    for (int vp = 0; vp < VP; ++vp) {
        const int c = vp * 64 + lane;
        float s[N];
#pragma unroll
        for (int i = 0; i < N; ++i) s[i] = 0.f;
        int j = wave;
        for (; j + 12 < HW; j += 16) {
            Vec<DT> t[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) t[u].load(x, (n * HW + j + 4 * u) * CV + c);
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int i = 0; i < N; ++i) s[i] += t[u].v[i];
        }
        for (; j < HW; j += 4) {
            Vec<DT> t;
            t.load(x, (n * HW + j) * CV + c);
#pragma unroll
            for (int i = 0; i < N; ++i) s[i] += t.v[i];
        }
#pragma unroll
        for (int i = 0; i < N; ++i) part[wave][c][i] = s[i];
    }
    __syncthreads();
    const float hw = (float)HW;
    for (int e = threadIdx.x; e < C; e += 256) {
        const int c = e / N, i = e % N;
        pooled[e] = (((part[0][c][i] + part[1][c][i]) + part[2][c][i]) + part[3][c][i]) / hw;
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int o = (blockIdx.x * 4 + wave) * R + r;
        if (o >= Cout) break;
        float sum = 0.f;
#pragma unroll
        for (int j = 0; j < CPL; ++j) {
            const f32x4_t v0 = *(const f32x4_t*)(pooled + j * 512 + lane * 8), v1 = *(const f32x4_t*)(pooled + j * 512 + lane * 8 + 4);
#pragma unroll
            for (int i = 0; i < 4; ++i) sum += wr[r][j][i] * v0[i];
#pragma unroll
            for (int i = 0; i < 4; ++i) sum += wr[r][j][4 + i] * v1[i];
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off, 64);
        if (lane == 0) y[n * Cout + o] = sum + (bias ? bias[o] : 0.f);
    }
}

// ---- FC: logits[n][o] = sum_c w[o][c] v[n][c] + b[o] ------------------------
// One wavefront per output row o; its weights stay in registers (8 per lane per
// 512 inputs) while it walks a chunk of images; wavefront reduction by
// cross-lane shuffles.
template <int DT, int CPL /* 512-element passes */>
__global__ __launch_bounds__(256) void fc_kernel(const float* __restrict__ v, const void* __restrict__ w,
                                                 const float* __restrict__ bias, float* __restrict__ y, int Nimg,
                                                 int Cin, int Cout, int img_per_block)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int o = blockIdx.x * 4 + wave;
    if (o >= Cout) return;
    float wr[CPL][8];
#pragma unroll
    for (int j = 0; j < CPL; ++j) {
        const size_t e0 = (size_t)o * Cin + j * 512 + lane * 8;
        if constexpr (DT == SGPRS_BF16) {
            Vec<SGPRS_BF16> t;
            t.load(w, e0 / 8);
#pragma unroll
            for (int i = 0; i < 8; ++i) wr[j][i] = t.v[i];
        } else {
            Vec<SGPRS_F32> t0, t1;
            t0.load(w, e0 / 4);
            t1.load(w, e0 / 4 + 1);
#pragma unroll
            for (int i = 0; i < 4; ++i) { wr[j][i] = t0.v[i]; wr[j][4 + i] = t1.v[i]; }
        }
    }
    const float b = bias ? bias[o] : 0.f;
    const int n_begin = blockIdx.y * img_per_block;
    const int n_end = min(n_begin + img_per_block, Nimg);
    // G images at a time: their vector loads are in flight together (one image per round trip made
    // the kernel latency-bound), images past the end re-read the last one and are dropped.  A dot
    // product is summed in the same order whatever G is.
    constexpr int G = CPL == 1 ? 8 : 4;   // (512 inputs: the whole block of eight images at once, together with the weights)
    for (int n0 = n_begin; n0 < n_end; n0 += G) {
        f32x4_t v0[G][CPL], v1[G][CPL];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const int n = min(n0 + g, n_end - 1);
#pragma unroll
            for (int j = 0; j < CPL; ++j) {
                const f32x4_t* vp = (const f32x4_t*)(v + (size_t)n * Cin + j * 512 + lane * 8);
                v0[g][j] = vp[0];
                v1[g][j] = vp[1];
            }
        }
        float s[G];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            s[g] = 0.f;
#pragma unroll
            for (int j = 0; j < CPL; ++j) {
#pragma unroll
                for (int i = 0; i < 4; ++i) s[g] += wr[j][i] * v0[g][j][i];
#pragma unroll
                for (int i = 0; i < 4; ++i) s[g] += wr[j][4 + i] * v1[g][j][i];
            }
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1)
#pragma unroll
            for (int g = 0; g < G; ++g) s[g] += __shfl_xor(s[g], off, 64);
#pragma unroll
        for (int g = 0; g < G; ++g)
            if (lane == 0 && n0 + g < n_end) y[(size_t)(n0 + g) * Cout + o] = s[g] + b;
    }
}

// ---- FC on the matrix cores, for batches of 32 images and more (bf16 weights) ------------
// logits[n][o] = sum_c w[o][c] v[n][c] + b[o] as 32 x 32 tiles of MFMA 32x32x16: rows = outputs
// (weights straight from memory, 16 bytes per lane), columns = images.  The pooled vectors stay
// fp32: each value goes in as a bf16 head plus a bf16 remainder (two MFMAs; products of two bf16
// are exact in fp32, so what is lost is below 2^-17 of a value).  The four wavefronts of a
// workgroup split the inputs of one tile and add their partial tiles through LDS in wavefront
// order, so the result does not depend on timing.
typedef __bf16 fc_bf16x8_t __attribute__((ext_vector_type(8)));
typedef float fc_f32x16_t __attribute__((ext_vector_type(16)));
__global__ __launch_bounds__(256) void fc_mfma_kernel(const float* __restrict__ v, const void* __restrict__ w,
                                                      const float* __restrict__ bias, float* __restrict__ y, int Nimg,
                                                      int Cin, int Cout)
{
    __shared__ f32x4_t part[4][4][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int frow = lane & 31, half = lane >> 5;
    const int o0 = blockIdx.x * 32, n0 = blockIdx.y * 32;
    const int o = min(o0 + frow, Cout - 1), n = min(n0 + frow, Nimg - 1);   // rows and columns past the end repeat the last one
    const int kq = Cin / 4, k0 = wave * kq + half * 8;
    const unsigned short* wp = (const unsigned short*)w + (size_t)o * Cin + k0;
    const float* vp = v + (size_t)n * Cin + k0;
    fc_f32x16_t acc;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0.f;
    for (int kb = 0; kb < kq; kb += 128) {   // eight k-steps per round trip
        u32x4_t a[8];
        f32x4_t b0[8], b1[8];
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            a[s] = *(const u32x4_t*)(wp + kb + s * 16);
            b0[s] = *(const f32x4_t*)(vp + kb + s * 16);
            b1[s] = *(const f32x4_t*)(vp + kb + s * 16 + 4);
        }
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            fc_bf16x8_t hi, lo;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const float f = i < 4 ? b0[s][i] : b1[s][i - 4];
                hi[i] = (__bf16)f;
                lo[i] = (__bf16)(f - (float)hi[i]);
            }
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(fc_bf16x8_t, a[s]), hi, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(fc_bf16x8_t, a[s]), lo, acc, 0, 0, 0);
        }
    }
    // accumulator register 4q + u: output o0 + 8q + 4 * half + u of image n0 + frow
#pragma unroll
    for (int q = 0; q < 4; ++q) part[wave][q][lane] = f32x4_t{acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]};
    __syncthreads();
    {
        const int q = wave, ob = o0 + 8 * q + 4 * half;
        f32x4_t r = ((part[0][q][lane] + part[1][q][lane]) + part[2][q][lane]) + part[3][q][lane];
        if (n0 + frow < Nimg && ob < Cout) {   // (Cout is a multiple of 4: a group of four is inside or outside as a whole)
            if (bias) r += *(const f32x4_t*)(bias + ob);
            *(f32x4_t*)(y + (size_t)(n0 + frow) * Cout + ob) = r;
        }
    }
}

// ---- placement probe --------------------------------------------------------
__global__ __launch_bounds__(64) void probe_kernel(uint32_t* out, int spin)
{
    const long long t0 = clock64();
    while (clock64() - t0 < (long long)spin) {}
    if (threadIdx.x == 0) {
        out[2 * blockIdx.x] = __builtin_amdgcn_s_getreg((3 << 11) | 20);      // XCC_ID[3:0]
        out[2 * blockIdx.x + 1] = __builtin_amdgcn_s_getreg((31 << 11) | 4);  // HW_ID
    }
}

// ---- launchers --------------------------------------------------------------
#define PROF_BEGIN(kind, variant, flops, bytes)                                                     \
    do {                                                                                            \
        int rc_ = SGPRS_OK;                                                                         \
        if (prof && prof->on && (rc_ = prof->begin(stream, kind, variant, flops, bytes))) return rc_; \
    } while (0)
#define PROF_END()                                                          \
    do {                                                                    \
        int rc_ = SGPRS_OK;                                                 \
        if (prof && prof->on && (rc_ = prof->end(stream))) return rc_;      \
    } while (0)

constexpr int kAvgpoolStreamMin = 512;
static unsigned blocks_for(size_t n) { return (unsigned)((n + 255) / 256); }

int launch_maxpool(int dtype, int n, int h, int w, int c, const void* x, void* y, hipStream_t stream, int,
                   Profiler* prof)
{
    const int P = (h - 1) / 2 + 1, Q = (w - 1) / 2 + 1;
    const int vec = dtype == SGPRS_BF16 ? 8 : 4;
    const unsigned total = (unsigned)((size_t)n * ((P + 1) / 2) * Q * (c / vec));  // two output rows per thread
    const double bytes = ((double)n * h * w * c + (double)n * P * Q * c) * dtype_size(dtype);
    PROF_BEGIN(kKindMaxpool, dtype, 0.0, bytes);
    const unsigned nblk = (blocks_for(total) + 7) / 8 * 8;  // whole multiple of the die count
    if (dtype == SGPRS_BF16)
        SGPRS_LAUNCH(maxpool3x3s2_kernel<SGPRS_BF16>, dim3(nblk), dim3(256), 0, stream, x, y, h, w,
                           c, P, Q, total);
    else
        SGPRS_LAUNCH(maxpool3x3s2_kernel<SGPRS_F32>, dim3(nblk), dim3(256), 0, stream, x, y, h, w,
                           c, P, Q, total);
    SGPRS_HIP(hipGetLastError());
    PROF_END();
    return SGPRS_OK;
}

int launch_bn_relu(int dtype, size_t pixels, int c, const void* x, const float* scale, const float* shift,
                   void* y, hipStream_t stream, int, Profiler* prof)
{
    const int vec = dtype == SGPRS_BF16 ? 8 : 4;
    const size_t total = pixels * (c / vec);
    PROF_BEGIN(kKindBnRelu, dtype, 2.0 * pixels * c, 2.0 * pixels * c * dtype_size(dtype));
    if (dtype == SGPRS_BF16)
        SGPRS_LAUNCH(bn_relu_kernel<SGPRS_BF16>, dim3(blocks_for(total)), dim3(256), 0, stream, x, y, scale,
                           shift, c, total);
    else
        SGPRS_LAUNCH(bn_relu_kernel<SGPRS_F32>, dim3(blocks_for(total)), dim3(256), 0, stream, x, y, scale,
                           shift, c, total);
    SGPRS_HIP(hipGetLastError());
    PROF_END();
    return SGPRS_OK;
}

int launch_add_relu(int dtype, size_t count, const void* a, const void* b, void* y, int relu,
                    hipStream_t stream, int, Profiler* prof)
{
    const int vec = dtype == SGPRS_BF16 ? 8 : 4;
    const size_t total = count / vec;
    PROF_BEGIN(kKindAdd, dtype, (double)count, 3.0 * count * dtype_size(dtype));
    if (dtype == SGPRS_BF16)
        SGPRS_LAUNCH(add_relu_kernel<SGPRS_BF16>, dim3(blocks_for(total)), dim3(256), 0, stream, a, b, y, relu,
                           total);
    else
        SGPRS_LAUNCH(add_relu_kernel<SGPRS_F32>, dim3(blocks_for(total)), dim3(256), 0, stream, a, b, y, relu,
                           total);
    SGPRS_HIP(hipGetLastError());
    PROF_END();
    return SGPRS_OK;
}

// Global average pool alone: x [n][hw][c] -> v fp32 [n][c].
int launch_avgpool(int dtype, int n, int hw, int cin, const void* x, float* ws, hipStream_t stream, Profiler* prof)
{
    const int vec = dtype == SGPRS_BF16 ? 8 : 4;
    const size_t es = dtype_size(dtype);
    PROF_BEGIN(kKindAvgpool, dtype, (double)n * hw * cin, (double)n * hw * cin * es + (double)n * cin * 4);
    if (n >= kAvgpoolStreamMin) {   // many images: one wavefront per image, no LDS, no barrier (the same bits)
        const dim3 pgrid((cin / vec + 63) / 64, (n + 3) / 4);
        if (dtype == SGPRS_BF16)
            SGPRS_LAUNCH(avgpool_stream_kernel<SGPRS_BF16>, pgrid, dim3(256), 0, stream, x, ws, hw, cin, n);
        else
            SGPRS_LAUNCH(avgpool_stream_kernel<SGPRS_F32>, pgrid, dim3(256), 0, stream, x, ws, hw, cin, n);
    } else {
        const dim3 pgrid((cin / vec + 63) / 64, n);
        if (dtype == SGPRS_BF16)
            SGPRS_LAUNCH(avgpool_kernel<SGPRS_BF16>, pgrid, dim3(256), 0, stream, x, ws, hw, cin);
        else
            SGPRS_LAUNCH(avgpool_kernel<SGPRS_F32>, pgrid, dim3(256), 0, stream, x, ws, hw, cin);
    }
    SGPRS_HIP(hipGetLastError());
    PROF_END();
    return SGPRS_OK;
}

int launch_avgpool_fc(int dtype, int n, int hw, int cin, int cout, const void* x, const void* w,
                      const float* bias, float* logits, float* ws, hipStream_t stream, int, Profiler* prof)
{
    const int vec = dtype == SGPRS_BF16 ? 8 : 4;
    const size_t es = dtype_size(dtype);
    if (n <= 8 && (cin == 512 || cin == 1024)) {  // a few images: one launch (its bits equal the two-kernel path's)
        const dim3 fgrid((cout + 15) / 16, n);
        PROF_BEGIN(kKindFc, 2 + dtype, 2.0 * n * cin * cout,
                   (double)cin * cout * es + (double)n * hw * cin * es + (double)n * cout * 4);
        if (dtype == SGPRS_BF16) {
            if (cin == 512) SGPRS_LAUNCH((avgpool_fc_kernel<SGPRS_BF16, 1>), fgrid, dim3(256), 0, stream, x, w, bias, logits, hw, cout);
            else SGPRS_LAUNCH((avgpool_fc_kernel<SGPRS_BF16, 2>), fgrid, dim3(256), 0, stream, x, w, bias, logits, hw, cout);
        } else {
            if (cin == 512) SGPRS_LAUNCH((avgpool_fc_kernel<SGPRS_F32, 1>), fgrid, dim3(256), 0, stream, x, w, bias, logits, hw, cout);
            else SGPRS_LAUNCH((avgpool_fc_kernel<SGPRS_F32, 2>), fgrid, dim3(256), 0, stream, x, w, bias, logits, hw, cout);
        }
        SGPRS_HIP(hipGetLastError());
        PROF_END();
        return SGPRS_OK;
    }
    int rc = launch_avgpool(dtype, n, hw, cin, x, ws, stream, prof);
    if (rc) return rc;

    if (dtype == SGPRS_BF16 && n >= 32 && cout % 4 == 0 && cin % 512 == 0) {   // enough images for 32 x 32 tiles on the matrix cores
        PROF_BEGIN(kKindFc, 4, 2.0 * n * cin * cout, (double)cin * cout * es + (double)n * (cin + cout) * 4);
        SGPRS_LAUNCH(fc_mfma_kernel, dim3((cout + 31) / 32, (n + 31) / 32), dim3(256), 0, stream, (const float*)ws, w, bias, logits, n, cin, cout);
        SGPRS_HIP(hipGetLastError());
        PROF_END();
        return SGPRS_OK;
    }
    const int img_per_block = 8;
    const dim3 grid((cout + 3) / 4, (n + img_per_block - 1) / img_per_block);
    const int cpl = cin / 512;
    PROF_BEGIN(kKindFc, dtype, 2.0 * n * cin * cout, (double)cin * cout * es + (double)n * (cin + cout) * 4);
#define FC_LAUNCH(DT, CPL)                                                                                  \
    SGPRS_LAUNCH((fc_kernel<DT, CPL>), grid, dim3(256), 0, stream, (const float*)ws, w, bias, logits, n, cin, \
                       cout, img_per_block)
    if (dtype == SGPRS_BF16) {
        if (cpl == 1) FC_LAUNCH(SGPRS_BF16, 1); else if (cpl == 2) FC_LAUNCH(SGPRS_BF16, 2); else FC_LAUNCH(SGPRS_BF16, 4);
    } else {
        if (cpl == 1) FC_LAUNCH(SGPRS_F32, 1); else if (cpl == 2) FC_LAUNCH(SGPRS_F32, 2); else FC_LAUNCH(SGPRS_F32, 4);
    }
#undef FC_LAUNCH
    SGPRS_HIP(hipGetLastError());
    PROF_END();
    return SGPRS_OK;
}

// ---- pooled-vector scratch for callers that cannot allocate ------------------
// One array per GPU, held until the process ends.  In host code the array's
// name is only a stand-in: the device address is looked up once per device,
// with that device current, and kept.
static __device__ __align__(256) float scratch[kStaticScratchFloats];
static std::mutex g_scratch_mu;
static float* g_scratch_ptr[kMaxStaticScratchDevices];

int static_scratch(int device, float** out)
{
    if (device < 0 || device >= kMaxStaticScratchDevices)
        return fail(SGPRS_ERR_UNSUPPORTED, "device %d: the static scratch covers devices 0..%d", device, kMaxStaticScratchDevices - 1);
    std::lock_guard<std::mutex> guard(g_scratch_mu);
    if (!g_scratch_ptr[device]) {
        int prev = 0;
        SGPRS_HIP(hipGetDevice(&prev));
        if (prev != device) SGPRS_HIP(hipSetDevice(device));
        void* p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (prev != device) (void)hipSetDevice(prev);
        if (e != hipSuccess || !p)
            return fail(SGPRS_ERR_HIP, "hipGetSymbolAddress(scratch) failed on device %d: %s", device, hipGetErrorString(e));
        g_scratch_ptr[device] = (float*)p;
    }
    *out = g_scratch_ptr[device];
    return SGPRS_OK;
}

int launch_probe(int n_blocks, int spin_cycles, uint32_t* out, hipStream_t stream)
{
    SGPRS_LAUNCH(probe_kernel, dim3(n_blocks), dim3(64), 0, stream, out, spin_cycles);
    SGPRS_HIP(hipGetLastError());
    return SGPRS_OK;
}

}  // namespace sgprs
