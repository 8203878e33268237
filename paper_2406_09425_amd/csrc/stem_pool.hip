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
typedef short i16x2_t __attribute__((ext_vector_type(2)));

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

// ---------------------------------------------------------------------------------------------
// bf16 variant with packed input rows.
//
// In the kernel above every wavefront re-reads all weights from LDS for each tile, the 4-slot pixel
// layout pads K from 147 to 224, and the patch goes through registers and LDS stores.  Here
//  * the weights are stationary in registers (88 VGPRs: 2 channel tiles x 11 K-steps), loaded once
//    per workgroup from a [64][176] layout prepared at task creation;
//  * the input patch keeps the image's own 3-channel packing: 35 rows of 17 16-byte pieces are
//    copied global -> LDS by the load unit itself (zero fill outside the image comes from the
//    buffer bounds check), double buffered so that the next tile's patch lands during this
//    tile's arithmetic;
//  * a pixel's K-run for tap row r is the 24 consecutive bf16 that start one element before its
//    first tap (elements 0, 22, 23 meet zero weights), so K = 7 x 24 = 168 (+8 zero) = 176 and
//    the run starts on a 4-byte boundary;
//  * BN scale / shift live in LDS, and there are two barriers per tile instead of four.
// Element 0 / 22 / 23 of a run are real neighbouring inputs multiplied by zero weights: the
// result equals the plain definition for finite inputs (a non-finite input pixel would also
// reach the output columns next to its window).
constexpr int kRowPitch = 272;                       // 17 pieces of 16 bytes per staged input row
constexpr int kRowUnits = kInR * 17;                 // 595 pieces per patch
constexpr int kPatchPitch = 640 * 16;                // 3 rounds of 256 lanes, the tail lands as zeros (row 35, 36)
constexpr int kPackedK = 176;

typedef unsigned int u32x4a4_t __attribute__((ext_vector_type(4), aligned(4)));
typedef __attribute__((address_space(3))) void* lds_ptr_t;

__global__ __launch_bounds__(256, 2) void stem_pool_packed_kernel(const StemPoolArgs a, const unsigned x_bytes)
{
    constexpr int SROWB = 64 * 2 + 16;
    constexpr int STG_BASE = 2 * kPatchPitch;
    constexpr int SC_BASE = STG_BASE + 256 * SROWB;

    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int frow = lane & 31, fhalf = lane >> 5;

    const __amdgpu_buffer_rsrc_t x_rs = __builtin_amdgcn_make_buffer_rsrc((void*)a.x, 0, (int)x_bytes, 0x00020000);
    const int row_bytes = a.W * 6;
    // Workgroup b runs on die b % 8 (whole chip; on a masked partition the dies of the mask take
    // turns the same way).  Each die walks its own contiguous eighth of the tiles, so neighbouring
    // tiles, whose input patches overlap by a quarter, meet in one L2 and the overlap is fetched
    // from HBM once.
    int first_tile = blockIdx.x, tile_step = gridDim.x, tile_end = a.ntiles;
    if (gridDim.x % 8 == 0) {
        const int per_die = (a.ntiles + 7) / 8, die = blockIdx.x & 7;
        first_tile = die * per_die + ((int)blockIdx.x >> 3);
        tile_step = (int)gridDim.x >> 3;
        tile_end = min((die + 1) * per_die, a.ntiles);
    }
    // A tile is (image n, tile row tp, tile column tq).  The walk tile += tile_step is kept in
    // that form with carries, so that no tile costs an integer division.
    struct TilePos { int n, tp, tq; };
    const int per_image = a.tiles_p * a.tiles_q;
    const int step_n = tile_step / per_image, step_r = tile_step - step_n * per_image;
    const int step_p = step_r / a.tiles_q, step_q = step_r - step_p * a.tiles_q;
    auto advance = [&](TilePos t) {
        t.tq += step_q;
        if (t.tq >= a.tiles_q) { t.tq -= a.tiles_q; ++t.tp; }
        t.tp += step_p;
        if (t.tp >= a.tiles_p) { t.tp -= a.tiles_p; ++t.n; }
        t.n += step_n;
        return t;
    };
    // The patch of a tile: 16-byte piece u = it * 256 + tid is piece u % 17 of input row u / 17.  Offsets
    // first (vector arithmetic), then one load instruction per round, so that the loads can be
    // placed between the MFMAs of the tile before (issued back to back they stall on the address queue).
    auto patch_offsets = [&](const TilePos t, unsigned (&off)[3]) {
        const int n = t.n, pp0 = t.tp * kPoolTP, pq0 = t.tq * kPoolTQ;
        const int h_base = 4 * pp0 - 5, b_base = 24 * pq0 - 32;  // first input row; byte of the first piece in its row
#pragma unroll
        for (int it = 0; it < 3; ++it) {
            const int u = it * 256 + tid;
            const int row = u / 17, seg = u - row * 17;
            const int ih = h_base + row, b = b_base + 16 * seg;
            const bool ok = u < kRowUnits && seg < 16 && (unsigned)ih < (unsigned)a.H && (unsigned)b < (unsigned)row_bytes;
            off[it] = ok ? (unsigned)((n * a.H + ih) * row_bytes + b) : 0x80000000u;
        }
    };
    auto patch_load = [&](int it, const unsigned (&off)[3], int buf) {
        if (it == 2 && wave >= 2) return;            // 640 piece slots: the third round is half a round
        __builtin_amdgcn_raw_ptr_buffer_load_lds(x_rs, (lds_ptr_t)(smem + buf * kPatchPitch + (it * 256 + wave * 64) * 16), 16,
                                                 off[it], 0, 0, 0);
    };
    TilePos cur;
    cur.n = first_tile / per_image;
    cur.tp = (first_tile - cur.n * per_image) / a.tiles_q;
    cur.tq = first_tile - cur.n * per_image - cur.tp * a.tiles_q;
    unsigned poffs[3];
    if (first_tile < tile_end) {
        patch_offsets(cur, poffs);
#pragma unroll
        for (int it = 0; it < 3; ++it) patch_load(it, poffs, 0);
    }

    if (tid < 32) {
        const int c4 = (tid & 15) * 4;
        const float* src = tid < 16 ? a.scale : a.shift;
        *(f32x4_t*)(smem + SC_BASE + (tid < 16 ? 0 : 256) + c4 * 4) = *(const f32x4_t*)(src + c4);
    }

    // stationary weights: A fragment of channel tile i, K-step ks = 16 bytes at [32i + frow][(2ks + fhalf) * 8]
    u32x4_t wreg[2][11];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int ks = 0; ks < 11; ++ks)
            wreg[i][ks] = *(const u32x4_t*)(a.w + (size_t)(32 * i + frow) * (kPackedK * 2) + (2 * ks + fhalf) * 16);

    // this lane's two conv pixels: byte offset of their K-run for tap row 0 inside a patch
    int poff[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        int t = wave * 64 + j * 32 + frow;
        if (t >= kConvR * kConvC) t = 0;             // the one padding row of the 256-row tile: computed, never used
        const int cr = t / kConvC, cc = t - cr * kConvC;
        poff[j] = (2 * cr) * kRowPitch + 12 * cc;
    }

    int buf = 0;
    for (int tile = first_tile; tile < tile_end; tile += tile_step, buf ^= 1) {
        const int n = cur.n, pp0 = cur.tp * kPoolTP, pq0 = cur.tq * kPoolTQ;
        cur = advance(cur);
        const int cr0 = 2 * pp0 - 1, cc0 = 2 * pq0 - 1;

        __builtin_amdgcn_s_waitcnt(0);               // this tile's patch has landed (and the last tile's stores have left)
        __syncthreads();                             // ... for every wavefront; the last tile's pooling reads are done
        const bool has_next = tile + tile_step < tile_end;
        if (has_next) patch_offsets(cur, poffs);

        f32x16_t acc[2][2];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

        // K group kg = 2ks + fhalf covers tap row kg / 3, 16-byte part kg % 3.  The upper half-wave
        // is one group ahead: 16 bytes further, or 240 (next tap row, part 0) when kg % 3 == 2.
        const unsigned char* P = smem + buf * kPatchPitch;
        const unsigned char *b0[2], *bA[2], *bB[2];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            b0[j] = P + poff[j];
            bA[j] = b0[j] + fhalf * 16;
            bB[j] = b0[j] + fhalf * (kRowPitch - 32);
        }
        // B fragments are read one K-step ahead of the MFMAs that use them
        auto read_b = [&](int ks, u32x4_t (&pf)[2]) {
            const int kg = 2 * ks, off = (kg / 3) * kRowPitch + (kg % 3) * 16;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                // the last step's upper group (21) has zero weights: it re-reads group 20
                const unsigned char* src = ks == 10 ? b0[j] : kg % 3 == 2 ? bB[j] : bA[j];
                pf[j] = *(const u32x4a4_t*)(src + off);
            }
        };
        constexpr int STEM_DEPTH = 1;   // deeper prefetch measured no faster
        u32x4_t pf[STEM_DEPTH + 1][2];
#pragma unroll
        for (int d = 0; d < STEM_DEPTH; ++d) read_b(d, pf[d]);
#pragma unroll
        for (int ks = 0; ks < 11; ++ks) {
            if (ks + STEM_DEPTH < 11) read_b(ks + STEM_DEPTH, pf[(ks + STEM_DEPTH) % (STEM_DEPTH + 1)]);
            if (has_next && ks % 3 == 1 && ks < 9) patch_load(ks / 3, poffs, buf ^ 1);   // the next tile's patch: K-steps 1, 4, 7
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, wreg[i][ks]),
                                                                      __builtin_bit_cast(bf16x8_t, pf[ks % (STEM_DEPTH + 1)][j]),
                                                                      acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }

        // Accumulator register e: column lane%32 = pixel, row 8*(e/4) + 4*(lane/32) + e%4 = channel.
        // Scale and shift of the next channel group are read from LDS while this one is computed.
        // ReLU is taken after the rounding, on the bf16 pair as signed 16-bit integers (rounding
        // is monotone and keeps 0, so the order does not matter); the staged values are then
        // non-negative bit patterns, which the pooling compares as unsigned integers.  Positions
        // outside the conv output are cleared to 0 afterwards: each pooling window has a real pixel,
        // so 0 never wins wrongly.
        int tpix[2];
        bool keep[2];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int t = wave * 64 + j * 32 + frow;
            const int cr = t / kConvC, cc = t - cr * kConvC;
            const int crow = cr0 + cr, ccol = cc0 + cc;
            const bool ok = t < kConvR * kConvC && (unsigned)crow < (unsigned)a.P && (unsigned)ccol < (unsigned)a.Q;
            keep[j] = ok;
            tpix[j] = t;
        }
        const unsigned char* scp = smem + SC_BASE + 16 * fhalf;
        f32x4_t sc_n = *(const f32x4_t*)scp, sh_n = *(const f32x4_t*)(scp + 256);
#pragma unroll
        for (int ig = 0; ig < 8; ++ig) {
            const int i = ig >> 2, g = ig & 3;
            const f32x4_t sc = sc_n, sh = sh_n;
            if (ig + 1 < 8) {
                sc_n = *(const f32x4_t*)(scp + (ig + 1) * 32);
                sh_n = *(const f32x4_t*)(scp + 256 + (ig + 1) * 32);
            }
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                float v[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) v[u] = acc[i][j][4 * g + u] * sc[u] + sh[u];
                const f32x2_t p0 = {v[0], v[1]}, p1 = {v[2], v[3]};
                const i16x2_t zero = {0, 0};
                const i16x2_t r0 = __builtin_elementwise_max(__builtin_bit_cast(i16x2_t, __builtin_convertvector(p0, bf16x2_t)), zero);
                const i16x2_t r1 = __builtin_elementwise_max(__builtin_bit_cast(i16x2_t, __builtin_convertvector(p1, bf16x2_t)), zero);
                u32x2_t o = {__builtin_bit_cast(unsigned, r0), __builtin_bit_cast(unsigned, r1)};
                *(u32x2_t*)(smem + STG_BASE + tpix[j] * SROWB + (32 * i + 8 * g + 4 * fhalf) * 2) = o;
            }
        }
        // border tiles only: a lane whose pixel lies outside the conv output clears what it staged
        // (both half-waves of a pixel take the branch together and write the same zeros)
#pragma unroll
        for (int j = 0; j < 2; ++j)
            if (!keep[j]) {
                const u32x4_t z = {0u, 0u, 0u, 0u};
#pragma unroll
                for (int q = 0; q < 8; ++q) *(u32x4_t*)(smem + STG_BASE + tpix[j] * SROWB + q * 16) = z;
            }
        __syncthreads();

        // pooling: one item = (pooled pixel, 16-byte channel group); 448 items, two per thread (the
        // second only for threads 0..191), the 18 LDS reads of both in flight together
        {
            constexpr int ITEMS = kPoolTP * kPoolTQ * 8;
            u32x4_t m[2];
            const unsigned char* base[2];
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                const int it = tid + 256 * k < ITEMS ? tid + 256 * k : tid;
                const int px = it >> 3, lp = px / kPoolTQ, lq = px - lp * kPoolTQ;
                base[k] = smem + STG_BASE + ((2 * lp) * kConvC + 2 * lq) * SROWB + (it & 7) * 16;
                m[k] = *(const u32x4_t*)base[k];
            }
#pragma unroll
            for (int rs = 1; rs < 9; ++rs)
#pragma unroll
                for (int k = 0; k < 2; ++k) {
                    const u32x4_t t = *(const u32x4_t*)(base[k] + ((rs / 3) * kConvC + rs % 3) * SROWB);
                    m[k] = __builtin_bit_cast(u32x4_t, __builtin_elementwise_max(__builtin_bit_cast(u16x8_t, m[k]), __builtin_bit_cast(u16x8_t, t)));
                }
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                const int it = tid + 256 * k;
                const int px = it >> 3, lp = px / kPoolTQ, lq = px - lp * kPoolTQ;
                const int gp = pp0 + lp, gq = pq0 + lq;
                if (it < ITEMS && gp < a.PP && gq < a.PQ)
                    *(u32x4_t*)(a.y + (((size_t)(n * a.PP + gp) * a.PQ + gq) * 64) * 2 + (it & 7) * 16) = m[k];
            }
        }
    }
    __builtin_amdgcn_s_waitcnt(0);
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

std::atomic<int> g_stem_pool_force{-1};
void stem_pool_force(int v) { g_stem_pool_force = v; }

void pack_stem_rows(const float* oihw, uint16_t* out)
{
    // [64][176]: tap row r occupies 24 elements, element 1 + 3s + c is tap (r, s) of input channel c
    std::fill(out, out + 64 * kPackedK, (uint16_t)0);
    for (int k = 0; k < 64; ++k)
        for (int c = 0; c < 3; ++c)
            for (int r = 0; r < 7; ++r)
                for (int s2 = 0; s2 < 7; ++s2)
                    out[k * kPackedK + r * 24 + 1 + 3 * s2 + c] = f32_to_bf16_bits(oihw[((k * 3 + c) * 7 + r) * 7 + s2]);
}

int launch_stem_pool(int dtype, int n, int h, int w, const void* x, const void* wts, const void* wts_rows,
                     const float* scale, const float* shift, void* y, hipStream_t stream, int cus, Profiler* prof)
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
    static std::atomic<bool> raised[3] = {{false}, {false}, {false}};
    const long long x_bytes = (long long)n * h * w * 6;
    const bool packed = dtype == SGPRS_BF16 && wts_rows && w % 8 == 0 && ((uintptr_t)x & 15) == 0 && x_bytes < (1ll << 31) &&
                        g_stem_pool_force.load() != 1;
    if (prof && prof->on && (rc = prof->begin(stream, kKindStemPool, packed ? 2 : dtype, flops, bytes))) return rc;
    if (packed) {
        a.w = (const unsigned char*)wts_rows;
        constexpr int lds_rows = 2 * kPatchPitch + 256 * (64 * 2 + 16) + 512;
        if (!raised[2]) {
            SGPRS_HIP(hipFuncSetAttribute((const void*)stem_pool_packed_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                          lds_rows));
            raised[2] = true;
        }
        SGPRS_LAUNCH(stem_pool_packed_kernel, dim3((int)std::min<long long>(nt, 2ll * cus)), dim3(256), lds_rows, stream, a,
                     (unsigned)x_bytes);
    } else if (dtype == SGPRS_BF16) {
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
