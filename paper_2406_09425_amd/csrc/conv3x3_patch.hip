// 3x3 stride-1 pad-1 convolution, bf16, with the input patch staged in LDS.
//
// A plain implicit GEMM re-reads every input pixel once per filter tap; at
// ResNet18's shapes that makes the kernel bound by L2->CU traffic long before
// the matrix cores are busy.  Here a workgroup owns TR whole output rows
// (TR*W <= BM pixels, rows counted across the batch) and 64 output channels.
// For each chunk of KC input channels it stages in LDS
//   * the input patch: the TR+2 (plus image-boundary padding) input rows of
//     width W+2, zero filled outside the image, read once and reused by all
//     nine taps, and
//   * the weights of that chunk for its 64 channels and all nine taps,
// and then runs 9 * KC/16 MFMA k-steps straight out of LDS with no predicates,
// while the next chunk's patch and weights are on their way into the other LDS
// buffer.  Workgroups are persistent over their work items; when a layer has
// two chunks and a single channel block (64->64) the weights stay resident in
// LDS for the whole launch.
//
// Rows are addressed in an "extended" row space in which every image has one
// zero row above and below it: output row g = n*H + p maps to extended row
// e(g) = g + 2*(g/H) + 1 and needs extended rows e-1, e, e+1; a run of output
// rows therefore needs a contiguous run of extended rows, even across images.
#include "internal.h"
#include "patch_items.h"

namespace sgprs {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

struct PatchArgs {
    const unsigned char* x;
    const unsigned char* w;
    unsigned char* y;
    const float* scale;
    const float* shift;
    const unsigned char* res;
    float* partial;
    int H, W, Cin, Cout, NH;  // NH = N*H output rows in total
    int PW, HE;               // W+2, H+2
    unsigned mW, mPW, mHE, mH;  // ceil(2^32/d) multipliers for exact division
    int TR;                   // output rows per tile
    int n_mtiles, n_ntiles, n_chunks, chunks_per_split, splits;
    int xcd_groups;           // > 0: work items are laid out so that one die keeps one channel block
    int n_slots;              // size of the (possibly padded) work-item index space
    int relu;
    unsigned x_bytes, w_bytes, y_bytes;  // sizes of x, w and y (buffer-descriptor bounds of the direct-to-LDS kernel)
};

__device__ __forceinline__ unsigned fdiv(unsigned x, unsigned magic) { return __umulhi(x, magic); }

// ---- the kernel --------------------------------------------------------------------
// Tiles of 512, 256 or 128 rows x 64 channels, chunks of 32 (or 16) channels.  The
// global loads write LDS directly (buffer loads with the LDS bit: 64 lanes x 16
// bytes land in one contiguous KiB), so no registers, no LDS-store instructions
// and no address arithmetic are spent on staging.  Two LDS buffers: while the
// MFMAs of step t (one chunk of one work item) read buffer t % 2, the loads of
// step t+1 are issued into the other one, one per MFMA k-step.  Out-of-image
// pixels get a buffer offset beyond the descriptor's size, for which the
// hardware returns zeros: the zero halo costs no branch and no select.
//
// LDS layout: pixel p of the patch occupies bytes [64p, 64p+64) as four 16-byte
// slots; slot s holds channel group s ^ f(p), f(p) = bit-swap of (p >> 2) & 3,
// so that 16 consecutive pixels of one group, or 8 consecutive pixels of two
// adjacent groups, touch 16 distinct 16-byte bank groups without padding.  The
// weights use the same rule with the output channel in the place of p.
// With two chunks and one channel block (64 -> 64 layers) all weights stay
// resident (STAT) and only the patch is double buffered.
constexpr int kPatchCap512 = 672;  // patch capacity (pixels) of the 512-row tile
__host__ __device__ constexpr int s2_patch_cap(int bm) { return bm == 256 ? 1344 : 704; }  // stride-2 kernel: four parity planes
__device__ __forceinline__ unsigned dl_swz(unsigned p) { return ((p >> 3) & 1u) | ((p >> 1) & 2u); }
// The same with 16-channel chunks (32-byte pixels, two slots): slot s holds group s ^ ((p >> 3) & 1),
// conflict-free for 16 consecutive pixels of one group and for 8 pixels x both groups.
template <int SL> __device__ __forceinline__ unsigned dl_swz_sl(unsigned p) { return SL == 4 ? dl_swz(p) : (p >> 3) & 1u; }

template <int BM, int KC, bool STAT, bool SPLIT, int NW = 4>
__global__ __launch_bounds__(NW * 64, (KC == 16 ? 2 : 1)) void conv3x3_patch_dl_kernel(const PatchArgs a)
{
#if __HIP_DEVICE_COMPILE__  // the buffer-resource builtins exist in the device pass only; the host needs just the stub
    constexpr int BN = 64, NT = NW * 64;
    static_assert(NW == 4 || (NW == 8 && (BM == 256 || BM == 512) && KC == 32), "wavefront counts");
    static_assert((BM == 512 || BM == 256 || BM == 128) && (KC == 32 || KC == 16) && !(KC == 16 && (STAT || BM != 256)) &&
                      !(BM == 512 && NW != 8),
                  "tile shapes");
    constexpr int PB = KC * 2, SL = PB / 16;     // bytes and 16-byte slots per pixel of one chunk
    // wavefront grid: 4 x 1 or 2 x 2 (each wavefront 64 rows x 64 / WNW channels), or 8 x 1 with 32 rows each
    // (two wavefronts per SIMD: one's waits and epilogue arithmetic overlap the other's MFMAs); with
    // 512-row tiles those 8 wavefronts own 64 rows each, i.e. 2 x 2 MFMA tiles and one LDS fragment
    // read per MFMA instead of one and a half
    constexpr int WMW = NW == 8 ? 8 : BM / 64, WNW = NW / WMW, WTM = BM / WMW;
    // patch capacity in pixels: twice the tile for the small tiles; the 512-row tile has to share
    // the 160 KB with two weight buffers and gets what is left (enough for 18 rows of a 28-wide
    // image plus halo across one image border, or 8 rows of a 56-wide one)
    constexpr int PCAP_PIX = BM == 512 ? kPatchCap512 : 2 * BM;
    constexpr int P_UNITS = PCAP_PIX * SL, P_IT = (P_UNITS + NT - 1) / NT;  // the last patch slot may cover only some wavefronts
    static_assert(P_UNITS % 64 == 0, "whole-wavefront patch loads");
    constexpr int W_UNITS = BN * 9 * SL, W_IT = (W_UNITS + NT - 1) / NT;  // the last weight slot may cover only some wavefronts
    constexpr int P_BYTES = PCAP_PIX * PB, W_BYTES = BN * 9 * PB, WROW = 9 * PB;
    // LDS map.  32-channel chunks: [patch 0][pad][patch 1][pad][weights 0][weights 1] (the patch
    // fragment reads keep 16-bit immediate offsets; the pad lets the epilogue scratch overhang
    // the patch area).  16-channel chunks: [patch 0][weights 0][patch 1][weights 1], one stage
    // being exactly the size of the epilogue scratch, so that two workgroups fit one CU.
    constexpr int P_PITCH = KC == 32 ? P_BYTES + (BM == 512 ? 0 : 4096) : P_BYTES + W_BYTES;
    constexpr int W_BASE = KC == 32 ? 2 * P_PITCH : P_BYTES, W_PITCH = KC == 32 ? W_BYTES : P_PITCH;
    constexpr int PF_BASE = BM == 512 ? W_BASE + 2 * W_PITCH : P_BYTES;  // 256 bytes per wavefront that nobody reads
    constexpr int WTN = BN / WNW, TM = WTM / 32, TN = WTN / 32, KS = KC / 16, NSTEP = 9 * KS;
    constexpr int SCR_ROWS = NW == 8 ? 16 : 32;  // rows a wavefront transposes through its LDS scratch at a time
    constexpr int SROW = WTN + 4, LPR = WTN / 8, RPP = 64 / LPR, NPASS = 32 / RPP;
    static_assert(NSTEP >= P_IT + W_IT, "loader slots");
    static_assert(NW * SCR_ROWS * SROW * 4 <= P_PITCH, "epilogue scratch fits the patch buffer and what follows it");
    typedef __attribute__((address_space(3))) void* lds_ptr_t;

    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int frow = lane & 31, fhalf = lane >> 5;
    const int wm = wave / WNW, wn = wave % WNW;
    static_assert(!(STAT && SPLIT), "resident weights are for whole-K items");
    // whether the residual and the BN vectors are requested before the last step's MFMAs (registers permitting) or in the epilogue
    constexpr bool EARLY_RES = KC == 32 && BM != 512;

    // weight loader: 16-byte unit u = it * 256 + tid is slot u % SL of tap (u / SL) % 9 of row u / (9 * SL)
    unsigned w_voff[W_IT];
#pragma unroll
    for (int it = 0; it < W_IT; ++it) {
        const unsigned u = it * NT + tid, row = u / (9 * SL), rem = u % (9 * SL);
        w_voff[it] = ((row * 9 + rem / SL) * (unsigned)a.Cin + (((rem % SL) ^ dl_swz_sl<SL>(row)) * 8)) * 2u;
    }
    // Work items blockIdx.x + k * gridDim.x; an item is n_chunks steps (n_chunks is
    // even, so every item starts on buffer 0 and ends on buffer 1).
    int item = blockIdx.x;
    PatchItem cur = next_item(a, item, (int)gridDim.x);
    if (!cur.valid) return;

    const __amdgpu_buffer_rsrc_t w_rs = __builtin_amdgcn_make_buffer_rsrc((void*)a.w, 0, (int)a.w_bytes, 0x00020000);
    if constexpr (STAT) {  // both weight chunks resident
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int it = 0; it < W_IT; ++it)
                if (it * NT + wave * 64 < W_UNITS)  // the last slot covers only some wavefronts
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(w_rs, (lds_ptr_t)(smem + W_BASE + c * W_PITCH + (it * NT + wave * 64) * 16),
                                                             16, w_voff[it], c * KC * 2, 0, 0);
    }
    const int cb0 = SPLIT ? cur.split * a.chunks_per_split : 0;  // split-K slice s of an item covers chunks s * chunks_per_split ...
    if constexpr (!STAT) {  // first step's weights: requested before the patch tables are worked out
        const int ws = (cur.ntile * BN * 9 * a.Cin + cb0 * KC) * 2;
#pragma unroll
        for (int it = 0; it < W_IT; ++it)
            if (it * NT + wave * 64 < W_UNITS)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(w_rs, (lds_ptr_t)(smem + W_BASE + (it * NT + wave * 64) * 16), 16, w_voff[it], ws, 0, 0);
    }

    // patch loader: unit u is slot u % SL of patch pixel u / SL
    int p_row[P_IT], p_col[P_IT];
    unsigned p_grp[P_IT];
#pragma unroll
    for (int it = 0; it < P_IT; ++it) {
        const unsigned u = it * NT + tid, pix = u / SL;
        p_row[it] = fdiv(pix, a.mPW);
        p_col[it] = pix - p_row[it] * a.PW;
        p_grp[it] = (((u % SL) ^ dl_swz_sl<SL>(pix)) * 8) * 2u;
    }
    unsigned p_voff[P_IT];  // byte offset of each unit's source inside x for the item being loaded
    unsigned p_next[P_IT];  // the same for the item after the current one
    auto patch_offsets = [&](int mtile, unsigned (&voff)[P_IT]) {
        const int g0 = mtile * a.TR;
        const int g1 = min(g0 + a.TR, a.NH) - 1;
        const int E0 = g0 + 2 * (int)fdiv(g0, a.mH);
        const int R = (g1 + 2 * (int)fdiv(g1, a.mH) + 2) - E0 + 1;
#pragma unroll
        for (int it = 0; it < P_IT; ++it) {
            const int E = E0 + p_row[it];
            const int n = fdiv(E, a.mHE);
            const int hh = E - n * a.HE - 1;
            const bool ok = p_row[it] < R && (unsigned)hh < (unsigned)a.H && p_col[it] >= 1 && p_col[it] <= a.W;
            voff[it] = ok ? ((unsigned)((n * a.H + hh) * a.W + p_col[it] - 1) * (unsigned)a.Cin) * 2u + p_grp[it]
                          : 0x80000000u;
        }
    };

    // first step's patch
    patch_offsets(cur.mtile, p_voff);
    {
        const __amdgpu_buffer_rsrc_t x_rs = __builtin_amdgcn_make_buffer_rsrc((void*)a.x, 0, (int)a.x_bytes, 0x00020000);
#pragma unroll
        for (int it = 0; it < P_IT; ++it)
            if (it * NT + wave * 64 < P_UNITS)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(x_rs, (lds_ptr_t)(smem + (it * NT + wave * 64) * 16), 16, p_voff[it],
                                                         cb0 * KC * 2, 0, 0);
    }
    // (they land while the first item's addresses are set up; the wait is inside the item loop)

    const int c8 = (lane % LPR) * 8, rsub = lane / LPR;
    // this lane's weight rows: byte offset inside a weight buffer for k-step parity 0 / 1
    unsigned wb[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) wb[ks] = (wn * WTN + frow) * WROW + (((ks * 2 + fhalf) ^ dl_swz_sl<SL>(frow)) << 4);

    bool first_item = true;
    for (;;) {
        // ---- this work item
        const int g0 = cur.mtile * a.TR;
        const int rows_here = min(a.TR, a.NH - g0);
        const int m_lim = rows_here * a.W;
        const int nbase = cur.ntile * BN + wn * WTN + c8;
        unsigned aoff[TM][9];  // this lane's patch fragment address for every tap (k-step parity 0)
        {
            const int E0 = g0 + 2 * (int)fdiv(g0, a.mH);
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int tt = wm * WTM + i * 32 + frow;
                const int pr = fdiv(tt, a.mW), q = tt - pr * a.W;
                const bool ok = pr < rows_here;
                const int g = g0 + (ok ? pr : 0);
                const int e1 = g + 2 * (int)fdiv(g, a.mH);
                const unsigned pp = (unsigned)((e1 - E0) * a.PW + (ok ? q : 0));
#pragma unroll
                for (int tap = 0; tap < 9; ++tap) {
                    const unsigned p = pp + (tap / 3) * a.PW + (tap % 3);
                    aoff[i][tap] = p * PB + ((fhalf ^ dl_swz_sl<SL>(p)) << 4);
                }
            }
        }
        // tile row -> output pixel of this item, or -1 past the item's rows
        auto tile_pixel = [&](int tt) { return tt < m_lim ? tt : -1; };
        // y and the residual go through buffer descriptors: 32-bit offsets, rows past the item get an
        // offset beyond the bound (loads return 0, stores are dropped), no residual = a bound of 0
        const __amdgpu_buffer_rsrc_t y_rs = __builtin_amdgcn_make_buffer_rsrc((void*)a.y, 0, (int)a.y_bytes, 0x00020000);
        const __amdgpu_buffer_rsrc_t res_rs = __builtin_amdgcn_make_buffer_rsrc((void*)a.res, 0, a.res ? (int)a.y_bytes : 0, 0x00020000);
        auto out_off = [&](int px) { return px >= 0 ? (unsigned)((g0 * a.W + px) * a.Cout + nbase) * 2u : 0x80000000u; };
        f32x16_t acc[TM][TN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

        // the item after this one (its first step is loaded during this item's last step)
        int nxt_index = item + (int)gridDim.x;
        const PatchItem nxt = next_item(a, nxt_index, (int)gridDim.x);
        if (nxt.valid) patch_offsets(nxt.mtile, p_next);
        // this item's chunks [cb, ce): an even count, so it starts on buffer 0 and ends on buffer 1
        const int cb = SPLIT ? cur.split * a.chunks_per_split : 0;
        const int ce = SPLIT ? min(cb + a.chunks_per_split, a.n_chunks) : a.n_chunks;
        const int nxt_cb = SPLIT ? nxt.split * a.chunks_per_split : 0;

        f32x4_t sc0 = {1.f, 1.f, 1.f, 1.f}, sc1 = sc0, sh0 = {0.f, 0.f, 0.f, 0.f}, sh1 = sh0;
        u32x4_t rres[TM][NPASS];

        if (first_item) {  // the first step's data: every later step is awaited at the end of the step before it
            __builtin_amdgcn_s_waitcnt(0);
            __syncthreads();
            first_item = false;
        }

        // One step: MFMAs of chunk `chunk` from buffer BUF; loads of the following step into the other buffer.
        auto step = [&](auto BUFC, int chunk) {
            constexpr int BUF = decltype(BUFC)::value;
            const bool last = BUF == 1 && chunk == ce - 1;
            const bool has1 = !last || nxt.valid;
            if (last && nxt.valid) {
#pragma unroll
                for (int it = 0; it < P_IT; ++it) p_voff[it] = p_next[it];
            }
            // without a following step the descriptors have size 0: the loads fetch nothing
            const __amdgpu_buffer_rsrc_t x_rs = __builtin_amdgcn_make_buffer_rsrc((void*)a.x, 0, has1 ? (int)a.x_bytes : 0, 0x00020000);
            const __amdgpu_buffer_rsrc_t wn_rs = __builtin_amdgcn_make_buffer_rsrc((void*)a.w, 0, has1 ? (int)a.w_bytes : 0, 0x00020000);
            const int chunk1 = last ? nxt_cb : chunk + 1;
            const int xs1 = chunk1 * KC * 2;
            const int ws1 = ((last ? nxt.ntile : cur.ntile) * BN * 9 * a.Cin + chunk1 * KC) * 2;
            auto issue_slot = [&](int k) {
                if (k < P_IT) {
                    if (k * NT + wave * 64 < P_UNITS)
                        __builtin_amdgcn_raw_ptr_buffer_load_lds(x_rs, (lds_ptr_t)(smem + (BUF ^ 1) * P_PITCH + (k * NT + wave * 64) * 16),
                                                                 16, p_voff[k < P_IT ? k : 0], xs1, 0, 0);
                } else if (!STAT && k - P_IT < W_IT && (k - P_IT) * NT + wave * 64 < W_UNITS)
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(wn_rs, (lds_ptr_t)(smem + W_BASE + (BUF ^ 1) * W_PITCH + ((k - P_IT) * NT + wave * 64) * 16),
                                                             16, w_voff[k - P_IT < W_IT && k >= P_IT ? k - P_IT : 0], ws1, 0, 0);
            };
            if constexpr (KC == 32 && BUF == 0) {
                // First step of an item: touch every cache line of the NEXT item's patch (4 bytes per
                // unit into an unused LDS pad), one step before its real loads are issued.  Inputs
                // that do not fit the L2 come from HBM with a latency of two to three steps; this
                // way the real loads find their lines in (or on their way to) the L2.
                if (chunk == cb && nxt.valid) {
                    const __amdgpu_buffer_rsrc_t pf_rs = __builtin_amdgcn_make_buffer_rsrc((void*)a.x, 0, (int)a.x_bytes, 0x00020000);
                    const int lines = min(a.Cin >> 6, 2);  // 128-byte lines per pixel that are worth the extra instructions
                    for (int l = 0; l < lines; ++l)
#pragma unroll
                        for (int it = 0; it < P_IT; ++it)
                            if (it * NT + wave * 64 < P_UNITS)
                                __builtin_amdgcn_raw_ptr_buffer_load_lds(pf_rs, (lds_ptr_t)(smem + PF_BASE + wave * 256), 4, p_next[it],
                                                                         l * 128 + nxt_cb * KC * 2, 0, 0);
                }
            }
            if constexpr (!SPLIT && BM == 512 && BUF == 1 && WNW == 1) {
                // No registers to spare for the residual here: touch this wavefront's residual lines instead
                // (one 128-byte line per output row, 4 bytes each into the unused pad), so that the
                // epilogue's loads hit in the L2.
                if (last && a.res) {
                    const __amdgpu_buffer_rsrc_t r_rs = __builtin_amdgcn_make_buffer_rsrc((void*)a.res, 0, (int)a.y_bytes, 0x00020000);
#pragma unroll
                    for (int r = 0; r < WTM / 64; ++r) {
                        const int px = tile_pixel(wm * WTM + r * 64 + lane);
                        const unsigned off = px >= 0 ? (unsigned)((g0 * a.W + px) * a.Cout + cur.ntile * BN) * 2u : 0x80000000u;
                        __builtin_amdgcn_raw_ptr_buffer_load_lds(r_rs, (lds_ptr_t)(smem + PF_BASE + wave * 256), 4, off, 0, 0, 0);
                    }
                }
            }
            if (!SPLIT && EARLY_RES && BUF == 1 && last) {  // epilogue operands, requested now so that they arrive during the MFMAs
                sc0 = *(const f32x4_t*)(a.scale + nbase); sc1 = *(const f32x4_t*)(a.scale + nbase + 4);
                sh0 = *(const f32x4_t*)(a.shift + nbase); sh1 = *(const f32x4_t*)(a.shift + nbase + 4);
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int pass = 0; pass < NPASS; ++pass) {
                        rres[i][pass] = __builtin_amdgcn_raw_buffer_load_b128(
                            res_rs, out_off(tile_pixel(wm * WTM + i * 32 + pass * RPP + rsub)), 0, 0);
                    }
            }
            // MFMA loop: 9 * KS k-steps, fragments fetched two k-steps ahead, one load slot per k-step
            const unsigned char* pbuf = smem + BUF * P_PITCH;
            const unsigned char* wbuf = smem + W_BASE + (STAT ? chunk : BUF) * W_PITCH;  // STAT: two chunks in all
            // fragments are read AHEAD k-steps before their MFMAs; with two workgroups per CU the other
            // workgroup hides LDS latency and registers are scarce, so one k-step ahead is enough there
            constexpr int AHEAD = 2, SETS = AHEAD + 1;
            u32x4_t fa[SETS][TM], fb[SETS][TN];
            auto load_frags = [&](int set, int st) {
                const int tap = st / KS, ks = st % KS;
#pragma unroll
                for (int i = 0; i < TM; ++i) fa[set][i] = *(const u32x4_t*)(pbuf + (aoff[i][tap] ^ (ks << 5)));
#pragma unroll
                for (int j = 0; j < TN; ++j) fb[set][j] = *(const u32x4_t*)(wbuf + wb[ks] + j * 32 * WROW + tap * PB);
            };
#pragma unroll
            for (int q = 0; q < AHEAD; ++q) load_frags(q, q);
#pragma unroll
            for (int st = 0; st < NSTEP; ++st) {
                __builtin_amdgcn_sched_barrier(0);  // keep the read-ahead order of the LDS reads
                if (st + AHEAD < NSTEP) load_frags((st + AHEAD) % SETS, st + AHEAD);
                issue_slot(st);  // one per k-step: issuing them faster only stalls on the address queue
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            __builtin_bit_cast(bf16x8_t, fa[st % SETS][i]), __builtin_bit_cast(bf16x8_t, fb[st % SETS][j]),
                            acc[i][j], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            // the following step's data has landed, and nobody reads this buffer any more
            __builtin_amdgcn_s_waitcnt(0);
            __syncthreads();
        };
        for (int chunk = cb; chunk < ce; chunk += 2) {
            step(std::integral_constant<int, 0>{}, chunk);
            step(std::integral_constant<int, 1>{}, chunk + 1);
        }

        {   // epilogue through the patch area of buffer 1 (the next item's first step sits in buffer 0)
            float* scr = (float*)(smem + P_PITCH) + wave * SCR_ROWS * SROW;
            const unsigned relu_floor = a.relu ? kReluFloor : kNoReluFloor;
            if constexpr (!SPLIT && !EARLY_RES) {  // registers are scarce here: the operands are fetched now, the other wavefronts of the CU cover the wait
                sc0 = *(const f32x4_t*)(a.scale + nbase); sc1 = *(const f32x4_t*)(a.scale + nbase + 4);
                sh0 = *(const f32x4_t*)(a.shift + nbase); sh1 = *(const f32x4_t*)(a.shift + nbase + 4);
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int pass = 0; pass < NPASS; ++pass) {
                        rres[i][pass] = __builtin_amdgcn_raw_buffer_load_b128(
                            res_rs, out_off(tile_pixel(wm * WTM + i * 32 + pass * RPP + rsub)), 0, 0);
                    }
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int h = 0; h < 32 / SCR_ROWS; ++h) {  // accumulator registers 8h .. 8h+7 are rows 16h .. 16h+15 of the tile
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int e = 0; e < 16; ++e)
                        if (SCR_ROWS == 32 || (e >> 3) == h)
                            scr[(8 * (e >> 2) + 4 * fhalf + (e & 3) - h * SCR_ROWS) * SROW + j * 32 + frow] = acc[i][j][e];
#pragma unroll
                for (int pp = 0; pp < SCR_ROWS / RPP; ++pp) {
                    const int pass = h * (SCR_ROWS / RPP) + pp;
                    const int rr = pp * RPP + rsub;
                    const int px = tile_pixel(wm * WTM + i * 32 + pass * RPP + rsub);
                    f32x4_t v0 = *(const f32x4_t*)(scr + rr * SROW + c8);
                    f32x4_t v1 = *(const f32x4_t*)(scr + rr * SROW + c8 + 4);
                    if constexpr (SPLIT) {  // fp32 partial sums; scale, shift, residual and ReLU happen in the reduction
                        if (px >= 0) {
                            const size_t m = (size_t)g0 * a.W + px;
                            float* dst = a.partial + ((size_t)cur.split * a.NH * a.W + m) * a.Cout + nbase;
                            *(f32x4_t*)dst = v0;
                            *(f32x4_t*)(dst + 4) = v1;
                        }
                    } else {
                        const u32x4_t rv = rres[i][pass];
                        v0 = v0 * sc0 + sh0;
                        v1 = v1 * sc1 + sh1;
                        float v[8] = {v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
                        u32x4_t ov;
#pragma unroll
                        for (int u = 0; u < 4; ++u) {
                            const float lo = v[2 * u] + __uint_as_float(rv[u] << 16);
                            const float hi = v[2 * u + 1] + __uint_as_float(rv[u] & 0xffff0000u);
                            ov[u] = pack_bf16x2_relu(lo, hi, relu_floor);
                        }
                        __builtin_amdgcn_raw_buffer_store_b128(ov, y_rs, out_off(px), 0, 0);  // rows past the item: dropped
                    }
                }
            }
        }
        if (!nxt.valid) break;
        __syncthreads();  // the scratch area is free again before the next item's loads target it
        item = nxt_index;
        cur = nxt;
    }
#endif
}

// ---- stride-2 variant -------------------------------------------------------------
// 3x3 stride-2 pad-1 (the first convolution of a down-sampling block), optionally
// together with the block's shortcut, a 1x1 stride-2 convolution of the same
// input: the shortcut's operand x[2p][2q] is the 3x3's centre tap, so it costs
// one more k-step per chunk on a second accumulator and no loads of x at all.
// As an implicit GEMM these layers move 15-30 KB from the L2 per MFLOP and are
// bound by that; the patch moves 12-17.
//
// The patch is kept as four parity planes: extended row e (one zero row above
// every image, one unused row below, so that an image is H + 2 = even rows) and
// extended column c go to plane (e & 1, c & 1), position (e >> 1, c >> 1).
// Output (p, q), tap (r, s) needs extended (2p + r, 2q + s), i.e. plane
// (r & 1, s & 1) at (p + (r >> 1), q + (s >> 1)): consecutive output pixels read
// consecutive plane pixels, exactly as with stride 1, and the same swizzle
// applies.  In half-row units an output row g = n * Ho + p sits at
// hb(g) = g + g / Ho; a run of output rows needs plane rows hb(g0) .. hb(g1) + 1.
// Chunks are 16 channels (a 256-pixel tile's patch is 1100-1350 pixels).
struct S2Args {
    const unsigned char* x;
    const unsigned char* w;
    const unsigned char* w2;  // shortcut weights [Cout][Cin], or nullptr
    unsigned char* y;
    unsigned char* y2;
    const float* scale;
    const float* shift;
    const float* scale2;
    const float* shift2;
    int H, W, Cin, Cout, Ho, Wo, NHo;  // NHo = N * Ho output rows in total
    int PWh, HE;                       // Wo + 1, H + 2
    unsigned mWo, mPWh, mHE, mHo;      // ceil(2^32/d) multipliers for exact division
    int TR, n_mtiles, n_ntiles, n_chunks, splits, xcd_groups, n_slots, relu;
    unsigned x_bytes, w_bytes, w2_bytes;
};

template <int BM, int NW, bool PAIR>
__global__ __launch_bounds__(NW * 64, 1) void conv3x3s2_patch_kernel(const S2Args a)
{
#if __HIP_DEVICE_COMPILE__
    constexpr int BN = 64, NT = NW * 64, KC = 16, PB = 32, SL = 2;
    static_assert((BM == 256 && NW == 8) || (BM == 128 && NW == 4), "tile shapes");
    constexpr int WMW = NW == 8 ? 8 : BM / 64, WNW = NW / WMW, WTM = BM / WMW, WTN = BN / WNW, TM = WTM / 32, TN = WTN / 32;
    constexpr int PCAP_PIX = s2_patch_cap(BM), PPL = PCAP_PIX / 4;  // pixels per parity plane
    static_assert(PPL % 16 == 0, "plane pitch keeps the swizzle phase");
    constexpr int P_UNITS = PCAP_PIX * SL, W_UNITS = BN * 9 * SL, W2_UNITS = PAIR ? BN * SL : 0;
    constexpr int P_IT = (P_UNITS + NT - 1) / NT, W_IT = (W_UNITS + NT - 1) / NT, W2_IT = PAIR ? 1 : 0;
    constexpr int P_BYTES = PCAP_PIX * PB, W_BYTES = BN * 9 * PB, W2_BYTES = BN * PB, WROW = 9 * PB;
    constexpr int STAGE = P_BYTES + W_BYTES + W2_BYTES, W_BASE = P_BYTES, W2_BASE = P_BYTES + W_BYTES;
    constexpr int NSTEP = PAIR ? 10 : 9;                            // nine taps, then the shortcut on the centre tap's fragments
    constexpr int SPS = (P_IT + W_IT + W2_IT + NSTEP - 1) / NSTEP;  // load slots per k-step
    constexpr int SCR_ROWS = NW == 8 ? 16 : 32;
    constexpr int SROW = WTN + 4, LPR = WTN / 8, RPP = 64 / LPR, NPASS = 32 / RPP;
    static_assert(NW * SCR_ROWS * SROW * 4 <= P_BYTES, "epilogue scratch fits the patch area");
    typedef __attribute__((address_space(3))) void* lds_ptr_t;

    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int frow = lane & 31, fhalf = lane >> 5;
    const int wm = wave / WNW, wn = wave % WNW;

    int item = blockIdx.x;
    PatchItem cur = next_item(a, item, (int)gridDim.x);
    if (!cur.valid) return;

    // weight loaders: 16-byte unit u is slot u % 2 of tap (u / 2) % 9 of row u / 18 (shortcut: slot u % 2 of row u / 2)
    unsigned w_voff[W_IT], w2_voff = 0;
#pragma unroll
    for (int it = 0; it < W_IT; ++it) {
        const unsigned u = it * NT + tid, row = u / (9 * SL), rem = u % (9 * SL);
        w_voff[it] = ((row * 9 + rem / SL) * (unsigned)a.Cin + (((rem % SL) ^ dl_swz_sl<SL>(row)) * 8)) * 2u;
    }
    if constexpr (PAIR) w2_voff = ((unsigned)(tid / SL) * (unsigned)a.Cin + (((tid % SL) ^ dl_swz_sl<SL>(tid / SL)) * 8)) * 2u;
    // patch loader: unit u is slot u % 2 of patch pixel u / 2 = plane pix / PPL, plane row and column from the rest
    unsigned p_tab[P_IT];  // plane << 16 | plane row << 8 | plane column
    unsigned p_grp[P_IT];
#pragma unroll
    for (int it = 0; it < P_IT; ++it) {
        const unsigned u = it * NT + tid, pix = u / SL, pl = pix / PPL, rem = pix % PPL;
        const unsigned prow = fdiv(rem, a.mPWh), pcol = rem - prow * a.PWh;
        p_tab[it] = pl << 16 | prow << 8 | pcol;
        p_grp[it] = (((u % SL) ^ dl_swz_sl<SL>(pix)) * 8) * 2u;
    }
    unsigned p_voff[P_IT], p_next[P_IT];
    auto patch_offsets = [&](int mtile, unsigned (&voff)[P_IT]) {
        const int g0 = mtile * a.TR;
        const int g1 = min(g0 + a.TR, a.NHo) - 1;
        const int hb0 = g0 + (int)fdiv(g0, a.mHo);
        const int R2 = g1 + (int)fdiv(g1, a.mHo) - hb0 + 2;
#pragma unroll
        for (int it = 0; it < P_IT; ++it) {
            const int pl = p_tab[it] >> 16, prow = (p_tab[it] >> 8) & 255, pcol = p_tab[it] & 255;
            const int E = 2 * (hb0 + prow) + (pl >> 1);
            const int n = fdiv(E, a.mHE);
            const int hh = E - n * a.HE - 1;
            const int ww = 2 * pcol + (pl & 1) - 1;
            const bool ok = pl < 4 && prow < R2 && (unsigned)hh < (unsigned)a.H && (unsigned)ww < (unsigned)a.W;
            voff[it] = ok ? ((unsigned)((n * a.H + hh) * a.W + ww) * (unsigned)a.Cin) * 2u + p_grp[it] : 0x80000000u;
        }
    };
    // One load slot of the step (chunk, channel block ntile, patch offsets voff) into stage `stage`.
    auto issue_slot = [&](int k, int stage, const unsigned (&voff)[P_IT], int ntile, int chunk, bool live) {
        unsigned char* st = smem + stage * STAGE;
        if (k < P_IT) {
            if (k * NT + wave * 64 < P_UNITS) {
                const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void*)a.x, 0, live ? (int)a.x_bytes : 0, 0x00020000);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_ptr_t)(st + (k * NT + wave * 64) * 16), 16, voff[k < P_IT ? k : 0],
                                                         chunk * KC * 2, 0, 0);
            }
        } else if (k < P_IT + W_IT) {
            const int kk = k - P_IT;
            if (kk * NT + wave * 64 < W_UNITS) {
                const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void*)a.w, 0, live ? (int)a.w_bytes : 0, 0x00020000);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_ptr_t)(st + W_BASE + (kk * NT + wave * 64) * 16), 16,
                                                         w_voff[kk >= 0 && kk < W_IT ? kk : 0], (ntile * BN * 9 * a.Cin + chunk * KC) * 2, 0, 0);
            }
        } else if (PAIR && k == P_IT + W_IT) {
            if (wave * 64 < W2_UNITS) {
                const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void*)a.w2, 0, live ? (int)a.w2_bytes : 0, 0x00020000);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_ptr_t)(st + W2_BASE + wave * 64 * 16), 16, w2_voff,
                                                         (ntile * BN * a.Cin + chunk * KC) * 2, 0, 0);
            }
        }
    };

    patch_offsets(cur.mtile, p_voff);
#pragma unroll
    for (int k = 0; k < P_IT + W_IT + W2_IT; ++k) issue_slot(k, 0, p_voff, cur.ntile, 0, true);

    const int c8 = (lane % LPR) * 8, rsub = lane / LPR;
    const unsigned wrow = wn * WTN + frow;
    const unsigned wb = wrow * WROW + ((fhalf ^ dl_swz_sl<SL>(wrow)) << 4);
    const unsigned wb2 = wrow * PB + ((fhalf ^ dl_swz_sl<SL>(wrow)) << 4);

    bool first_item = true;
    for (;;) {
        const int g0 = cur.mtile * a.TR;
        const int rows_here = min(a.TR, a.NHo - g0);
        const int m_lim = rows_here * a.Wo;
        const int nbase = cur.ntile * BN + wn * WTN + c8;
        unsigned aoff[TM][9];
        {
            const int hb0 = g0 + (int)fdiv(g0, a.mHo);
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int tt = wm * WTM + i * 32 + frow;
                const int pr = fdiv(tt, a.mWo), q = tt - pr * a.Wo;
                const bool ok = pr < rows_here;
                const int g = g0 + (ok ? pr : 0);
                const int rowb = g + (int)fdiv(g, a.mHo) - hb0;
#pragma unroll
                for (int tap = 0; tap < 9; ++tap) {
                    const int r = tap / 3, sx = tap % 3;
                    const unsigned p = ((r & 1) * 2 + (sx & 1)) * PPL + (rowb + (r >> 1)) * a.PWh + (ok ? q : 0) + (sx >> 1);
                    aoff[i][tap] = p * PB + ((fhalf ^ dl_swz_sl<SL>(p)) << 4);
                }
            }
        }
        f32x16_t acc[TM][TN], acc2[PAIR ? TM : 1][PAIR ? TN : 1];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    acc[i][j][e] = 0.f;
                    if constexpr (PAIR) acc2[i][j][e] = 0.f;
                }

        int nxt_index = item + (int)gridDim.x;
        const PatchItem nxt = next_item(a, nxt_index, (int)gridDim.x);
        if (nxt.valid) patch_offsets(nxt.mtile, p_next);

        if (first_item) {
            __builtin_amdgcn_s_waitcnt(0);
            __syncthreads();
            first_item = false;
        }

        auto step = [&](auto BUFC, int chunk) {
            constexpr int BUF = decltype(BUFC)::value;
            const bool last = BUF == 1 && chunk == a.n_chunks - 1;
            const bool live = !last || nxt.valid;
            if (last && nxt.valid) {
#pragma unroll
                for (int it = 0; it < P_IT; ++it) p_voff[it] = p_next[it];
            }
            const int chunk1 = last ? 0 : chunk + 1;
            const int ntile1 = last ? nxt.ntile : cur.ntile;
            const unsigned char* pbuf = smem + BUF * STAGE;
            const unsigned char* wbuf = pbuf + W_BASE;
            constexpr int AHEAD = 2, SETS = AHEAD + 1;
            u32x4_t fa[SETS][TM], fb[SETS][TN];
            auto load_frags = [&](int set, int st) {
                const int tap = st < 9 ? st : 4;
#pragma unroll
                for (int i = 0; i < TM; ++i) fa[set][i] = *(const u32x4_t*)(pbuf + aoff[i][tap]);
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    fb[set][j] = st < 9 ? *(const u32x4_t*)(wbuf + wb + j * 32 * WROW + tap * PB)
                                        : *(const u32x4_t*)(pbuf + W2_BASE + wb2 + j * 32 * PB);
            };
#pragma unroll
            for (int q = 0; q < AHEAD; ++q) load_frags(q, q);
#pragma unroll
            for (int st = 0; st < NSTEP; ++st) {
                __builtin_amdgcn_sched_barrier(0);
                if (st + AHEAD < NSTEP) load_frags((st + AHEAD) % SETS, st + AHEAD);
#pragma unroll
                for (int k = st * SPS; k < (st + 1) * SPS; ++k) issue_slot(k, BUF ^ 1, p_voff, ntile1, chunk1, live);
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) {
                        if (st < 9)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                                __builtin_bit_cast(bf16x8_t, fa[st % SETS][i]), __builtin_bit_cast(bf16x8_t, fb[st % SETS][j]),
                                acc[i][j], 0, 0, 0);
                        else if constexpr (PAIR)
                            acc2[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                                __builtin_bit_cast(bf16x8_t, fa[st % SETS][i]), __builtin_bit_cast(bf16x8_t, fb[st % SETS][j]),
                                acc2[i][j], 0, 0, 0);
                    }
            }
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_waitcnt(0);
            __syncthreads();
        };
        for (int chunk = 0; chunk < a.n_chunks; chunk += 2) {
            step(std::integral_constant<int, 0>{}, chunk);
            step(std::integral_constant<int, 1>{}, chunk + 1);
        }

        {   // epilogue through the patch area of stage 1 (the next item's first step sits in stage 0)
            float* scr = (float*)(smem + STAGE) + wave * SCR_ROWS * SROW;
            auto write_out = [&](f32x16_t (&av)[TM][TN], const float* scale, const float* shift, unsigned char* y, bool relu) {
                const f32x4_t sc0 = *(const f32x4_t*)(scale + nbase), sc1 = *(const f32x4_t*)(scale + nbase + 4);
                const f32x4_t sh0 = *(const f32x4_t*)(shift + nbase), sh1 = *(const f32x4_t*)(shift + nbase + 4);
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int h = 0; h < 32 / SCR_ROWS; ++h) {
#pragma unroll
                        for (int j = 0; j < TN; ++j)
#pragma unroll
                            for (int e = 0; e < 16; ++e)
                                if (SCR_ROWS == 32 || (e >> 3) == h)
                                    scr[(8 * (e >> 2) + 4 * fhalf + (e & 3) - h * SCR_ROWS) * SROW + j * 32 + frow] = av[i][j][e];
#pragma unroll
                        for (int pp = 0; pp < SCR_ROWS / RPP; ++pp) {
                            const int pass = h * (SCR_ROWS / RPP) + pp;
                            const int rr = pp * RPP + rsub;
                            const int tt = wm * WTM + i * 32 + pass * RPP + rsub;
                            f32x4_t v0 = *(const f32x4_t*)(scr + rr * SROW + c8);
                            f32x4_t v1 = *(const f32x4_t*)(scr + rr * SROW + c8 + 4);
                            if (tt < m_lim) {
                                const size_t m = (size_t)g0 * a.Wo + tt;
                                v0 = v0 * sc0 + sh0;
                                v1 = v1 * sc1 + sh1;
                                float v[8] = {v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
                                u32x4_t ov;
#pragma unroll
                                for (int u = 0; u < 4; ++u) {
                                    ov[u] = pack_bf16x2_relu(v[2 * u], v[2 * u + 1], relu ? kReluFloor : kNoReluFloor);
                                }
                                *(u32x4_t*)(y + (m * a.Cout + nbase) * 2) = ov;
                            }
                        }
                    }
            };
            write_out(acc, a.scale, a.shift, a.y, a.relu != 0);
            if constexpr (PAIR) write_out(acc2, a.scale2, a.shift2, a.y2, false);
        }
        if (!nxt.valid) break;
        __syncthreads();
        item = nxt_index;
        cur = nxt;
    }
#endif
}

// ---- host side ---------------------------------------------------------------
static unsigned magic_for(unsigned d) { return (unsigned)((0x100000000ull + d - 1) / d); }

struct PatchVariant { int bm, bn, kc; };
static const PatchVariant kPatchVariants[] = {{256, 64, 32}, {128, 64, 32}, {256, 64, 16}, {256, 64, 32}, {512, 64, 32}};
constexpr int kNumPatchVariants = 5;
constexpr int kPatchDlVariant = 0;       // 256-row tiles, 4 wavefronts
constexpr int kPatchDlSmallVariant = 1;  // 128-row tiles, for layers with few row tiles
constexpr int kPatchDlPairVariant = 2;   // 16-channel chunks: half the LDS, two workgroups per CU
constexpr int kPatchDlWideVariant = 3;   // 256-row tiles, 8 wavefronts of 32 rows: two per SIMD
constexpr int kPatchDlTallVariant = 4;   // 512-row tiles, 8 wavefronts of 64 rows
int patch_num_variants() { return kNumPatchVariants; }

// Name as a profiler prints it: v = tile variant + 16 * stationary + 32 * split.
const char* patch_variant_name(int v)
{
    static char buf[8][96];
    static int next = 0;
    const int tv = v & 15;
    if (tv >= kNumPatchVariants) return "?";
    const PatchVariant& pv = kPatchVariants[tv];
    char* out = buf[next++ & 7];
    snprintf(out, 96, "conv3x3_patch_dl_kernel<%d, %d, %s, %s, %d>", pv.bm, pv.kc, (v & 16) ? "true" : "false",
             (v & 32) ? "true" : "false", tv >= kPatchDlWideVariant ? 8 : 4);
    return out;
}

bool patch_eligible(const sgprs_conv_desc_t& d)
{
    return d.dtype == SGPRS_BF16 && d.r == 3 && d.s == 3 && d.stride == 1 && d.pad == 1 && d.cin % 64 == 0 &&
           d.cout % 64 == 0 && d.w <= 128 && d.w >= 2 && d.h >= 2 && (long long)d.n * d.h * (d.w + 2) * 8 < (1ll << 24);
}

// Fills the tile geometry of variant v for this shape; false if it does not fit.
static bool patch_geometry_uncached(const sgprs_conv_desc_t& d, int v, int splits, PatchArgs* a);
static bool patch_geometry(const sgprs_conv_desc_t& d, int v, int splits, PatchArgs* a)
{
    struct Key { sgprs_conv_desc_t d; int v, splits; };
    struct Val { bool ok; PatchArgs a; };
    static thread_local PlanMemo<Key, Val, 512> local;
    static SharedPlanMemo<Key, Val, 512> memo;
    Key k;
    memset(&k, 0, sizeof(k));
    k.d = d; k.v = v; k.splits = splits;
    const Val hit = memo.get(local, k, [&]() {
        Val nv;
        memset(&nv, 0, sizeof(nv));
        nv.ok = patch_geometry_uncached(d, v, splits, &nv.a);
        return nv;
    });
    if (hit.ok) *a = hit.a;
    return hit.ok;
}
static bool patch_geometry_uncached(const sgprs_conv_desc_t& d, int v, int splits, PatchArgs* a)
{
    const PatchVariant& pv = kPatchVariants[v];
    if (d.cout % pv.bn || d.cin % pv.kc || d.w > pv.bm) return false;
    // x, w and the residual are addressed through 31-bit buffer offsets
    if (((long long)d.n * d.h * d.w * d.cin * 2 >= (1ll << 31) || (long long)d.n * d.h * d.w * d.cout * 2 >= (1ll << 31) ||
                                 (long long)d.cout * 9 * d.cin * 2 >= (1ll << 31)))
        return false;
    const int NH = d.n * d.h;
    const int cap = pv.bm == 512 ? kPatchCap512 : 2 * pv.bm;  // patch capacity in pixels
    // the most output rows per tile whose patch (halo rows included, also across image borders) fits
    int TR = pv.bm / d.w, n_mtiles = 0;
    for (; TR >= 1; --TR) {
        n_mtiles = (NH + TR - 1) / TR;
        int rmax = 0;
        for (int t = 0; t < n_mtiles; ++t) {
            const int g0 = t * TR, g1 = std::min(g0 + TR, NH) - 1;
            rmax = std::max(rmax, (g1 + 2 * (g1 / d.h) + 2) - (g0 + 2 * (g0 / d.h)) + 1);
        }
        if (rmax * (d.w + 2) <= cap) break;
        if (pv.bm != 512) return false;  // the smaller tiles keep their full-height geometry or decline
    }
    if (TR < 1 || (pv.bm == 512 && TR * d.w * 4 < pv.bm * 3)) return false;  // a 512-row tile less than three quarters full is not worth it
    const int n_chunks = d.cin / pv.kc;
    if (splits < 1 || splits > n_chunks) return false;
    const int cps = (n_chunks + splits - 1) / splits;
    if ((splits - 1) * cps >= n_chunks) return false;
    // the direct-to-LDS kernel alternates two buffers and wants an even number of chunks per item
    if (n_chunks % 2 || (splits > 1 && (cps % 2 || n_chunks % cps))) return false;
    // exactness of the multiply-high divisions: dividend * divisor < 2^32
    const unsigned long long lim = 1ull << 32;
    if ((unsigned long long)(NH + 2 * d.n + 4) * (d.h + 2) >= lim || (unsigned long long)(cap + 256) * (d.w + 2) >= lim) return false;
    a->H = d.h; a->W = d.w; a->Cin = d.cin; a->Cout = d.cout; a->NH = NH;
    a->PW = d.w + 2; a->HE = d.h + 2;
    a->mW = magic_for(d.w); a->mPW = magic_for(d.w + 2); a->mHE = magic_for(d.h + 2); a->mH = magic_for(d.h);
    a->TR = TR; a->n_mtiles = n_mtiles; a->n_ntiles = d.cout / pv.bn; a->n_chunks = n_chunks;
    a->chunks_per_split = cps; a->splits = splits; a->relu = d.relu;
    patch_index_space(n_mtiles, a->n_ntiles, splits, &a->xcd_groups, &a->n_slots);
    return true;
}

static std::atomic<int> g_force_variant{-1}, g_force_splits{0};
void patch_force(int variant, int splits) { g_force_variant = variant; g_force_splits = splits; }

// Picks the tile variant: the candidate with the smallest estimated time
// rounds(items / CUs) * (chunks * cost-per-chunk + cost-per-item); the costs (in
// microseconds, whole-GPU measurements at batch 64) only rank candidates.
// When a shape offers too few work items to fill the partition and is deep in K
// this kernel declines and the implicit-GEMM path (with its split-K) takes over.
bool plan_patch(const sgprs_conv_desc_t& d, int cus, int* variant, int* splits)
{
    if (!patch_eligible(d)) return false;
    PatchArgs a;
    const int fv = g_force_variant.load(), fs = g_force_splits.load();
    if (fv >= 0) {
        if (fv >= kNumPatchVariants || !patch_geometry(d, fv, std::max(1, fs), &a)) return false;
        *variant = fv; *splits = std::max(1, fs);
        return true;
    }
    // {variant, microseconds per chunk, microseconds per work item}
    static const struct { int v; double step, item; } cand[] = {
        {kPatchDlTallVariant, 2.4, 6.0}, {kPatchDlWideVariant, 1.5, 4.3}, {kPatchDlVariant, 1.65, 5.0}, {kPatchDlSmallVariant, 1.0, 4.5}};
    double best = 1e30;
    bool found = false;
    for (const auto& c : cand) {
        // split-K (fp32 partial sums plus a reduction pass) for shapes with too few work items to
        // occupy the partition
        for (int sp = 1; sp <= 2; ++sp) {
            if (!patch_geometry(d, c.v, sp, &a)) continue;
            const long long items = (long long)a.n_mtiles * a.n_ntiles * sp;
            // far fewer items than CUs: the partition's time is one workgroup's serial K loop. A shallow
            // one (up to four chunks, Cin <= 128) is over before a split implicit GEMM plus its reduction
            // pass would be (batch 1 on 256 CUs: 6.0 against 6.9-9.8 us at 56x56x64, 7.8 against 10.2 us
            // at 28x28x128); a deep one is left to the implicit GEMM's wider split-K
            if (items * 3 < cus && (sp > 1 || a.chunks_per_split > 4)) continue;
            const long long rounds = (items + cus - 1) / cus;
            double cost = rounds * (a.chunks_per_split * c.step + c.item);
            if (sp > 1) cost += 9.0 + (double)d.n * d.h * d.w * d.cout * 4.0 * (sp + 1) / (3.0e6 * cus / 256.0);
            if (cost < best) { best = cost; *variant = c.v; *splits = sp; found = true; }
        }
    }
    return found;
}

size_t patch_workspace_bytes(const sgprs_conv_desc_t& d, int splits)
{
    return splits > 1 ? (size_t)splits * d.n * d.h * d.w * d.cout * sizeof(float) : 0;
}

template <int BM, int KC, int NW = 4>
static int launch_patch_dl(const PatchArgs& a, int grid, hipStream_t stream)
{
    constexpr int kLds = BM == 512 ? 2 * kPatchCap512 * 64 + 2 * 64 * 9 * 64 + 8 * 256
                         : KC == 32 ? 2 * (2 * BM * 64 + 4096) + 2 * 64 * 9 * 64
                                    : 2 * (2 * BM * 32 + 64 * 9 * 32);
    static_assert(kLds <= 160 * 1024, "LDS of one CU");
    constexpr bool kStatOk = KC == 32;  // resident weights need room for every chunk
    static std::atomic<bool> raised{false};
    if (!raised) {
        if constexpr (kStatOk)
            SGPRS_HIP(hipFuncSetAttribute((const void*)conv3x3_patch_dl_kernel<BM, KC, kStatOk, false, NW>,
                                          hipFuncAttributeMaxDynamicSharedMemorySize, kLds));
        SGPRS_HIP(hipFuncSetAttribute((const void*)conv3x3_patch_dl_kernel<BM, KC, false, false, NW>,
                                      hipFuncAttributeMaxDynamicSharedMemorySize, kLds));
        SGPRS_HIP(hipFuncSetAttribute((const void*)conv3x3_patch_dl_kernel<BM, KC, false, true, NW>,
                                      hipFuncAttributeMaxDynamicSharedMemorySize, kLds));
        raised = true;
    }
    const dim3 block(NW * 64);
    if (a.splits > 1)
        SGPRS_LAUNCH((conv3x3_patch_dl_kernel<BM, KC, false, true, NW>), dim3(grid), block, kLds, stream, a);
    else if (kStatOk && a.n_chunks == 2 && a.n_ntiles == 1)
        SGPRS_LAUNCH((conv3x3_patch_dl_kernel<BM, KC, kStatOk, false, NW>), dim3(grid), block, kLds, stream, a);
    else
        SGPRS_LAUNCH((conv3x3_patch_dl_kernel<BM, KC, false, false, NW>), dim3(grid), block, kLds, stream, a);
    SGPRS_HIP(hipGetLastError());
    return SGPRS_OK;
}

int launch_splitk_reduce(int dtype, const float* partial, int splits, size_t total, int cout, const float* scale,
                         const float* shift, const void* res, void* y, int relu, hipStream_t stream);

int launch_conv3x3_patch(const sgprs_conv_desc_t& d, int variant, int splits, const void* x, const void* w,
                         const float* scale, const float* shift, const void* residual, void* y, void* ws,
                         size_t ws_bytes, hipStream_t stream, int cus, Profiler* prof)
{
    PatchArgs a;
    if (variant < 0 || variant >= kNumPatchVariants || !patch_eligible(d) || !patch_geometry(d, variant, splits, &a))
        return fail(SGPRS_ERR_INVALID_ARG, "internal: patch plan does not match the shape");
    const size_t need = patch_workspace_bytes(d, splits);
    if (need > ws_bytes || (need && !ws))
        return fail(SGPRS_ERR_INVALID_ARG, "split-K workspace %zu bytes needed, %zu given", need, ws_bytes);
    a.x = (const unsigned char*)x; a.w = (const unsigned char*)w; a.y = (unsigned char*)y;
    a.scale = scale; a.shift = shift; a.res = (const unsigned char*)residual; a.partial = (float*)ws;
    a.x_bytes = (unsigned)((size_t)d.n * d.h * d.w * d.cin * 2); a.w_bytes = (unsigned)((size_t)d.cout * 9 * d.cin * 2);
    a.y_bytes = (unsigned)((size_t)d.n * d.h * d.w * d.cout * 2);
    const int occ = variant == kPatchDlPairVariant ? 2 : 1;  // small enough for two workgroups per CU
    // a multiple of 8 keeps every workgroup on one die across its items
    int grid = (int)std::min<long long>(a.n_slots, (long long)cus * occ);
    if (a.xcd_groups && grid >= 8) grid -= grid % 8;
    const bool stat = variant != kPatchDlPairVariant && a.n_chunks == 2 && a.n_ntiles == 1 && a.splits == 1;  // resident weights
    const double M = (double)d.n * d.h * d.w;
    const double flops = 2.0 * M * d.cout * 9.0 * d.cin;
    const double bytes = (M * d.cin + (double)d.cout * 9 * d.cin + M * d.cout * (residual ? 2 : 1)) * 2.0;
    int rc;
    if (prof && prof->on && (rc = prof->begin(stream, kKindPatch, variant + (stat ? 16 : 0) + (splits > 1 ? 32 : 0), flops, bytes))) return rc;
    switch (variant) {
        case kPatchDlVariant: rc = launch_patch_dl<256, 32>(a, grid, stream); break;
        case kPatchDlSmallVariant: rc = launch_patch_dl<128, 32>(a, grid, stream); break;
        case kPatchDlPairVariant: rc = launch_patch_dl<256, 16>(a, grid, stream); break;
        case kPatchDlWideVariant: rc = launch_patch_dl<256, 32, 8>(a, grid, stream); break;
        default: rc = launch_patch_dl<512, 32, 8>(a, grid, stream); break;
    }
    if (rc) return rc;
    if (prof && prof->on && (rc = prof->end(stream))) return rc;
    if (splits > 1) {
        const size_t total = (size_t)M * d.cout;
        if (prof && prof->on &&
            (rc = prof->begin(stream, kKindReduce, d.dtype, 0.0, (double)total * 4.0 * splits + total * 2.0)))
            return rc;
        if ((rc = launch_splitk_reduce(d.dtype, a.partial, splits, total, d.cout, scale, shift, residual, y, d.relu, stream)))
            return rc;
        if (prof && prof->on && (rc = prof->end(stream))) return rc;
    }
    return SGPRS_OK;
}

// ---- stride-2 variant: host side ---------------------------------------------------
struct S2Variant { int bm, nw; };
static const S2Variant kS2Variants[] = {{256, 8}, {128, 4}};
constexpr int kNumS2Variants = 2;
static std::atomic<int> g_s2_force{-1};  // -1 automatic, 0 / 1 that tile where the shape allows it, 2 never
void s2patch_force(int v) { g_s2_force = v; }
int s2patch_num_variants() { return kNumS2Variants; }

// Name as a profiler prints it: v = tile variant + 4 * paired.
const char* s2patch_variant_name(int v)
{
    static char buf[4][64];
    static int next = 0;
    if (v < 0 || (v & 3) >= kNumS2Variants) return "?";
    char* out = buf[next++ & 3];
    snprintf(out, 64, "conv3x3s2_patch_kernel<%d, %d, %s>", kS2Variants[v & 3].bm, kS2Variants[v & 3].nw, (v & 4) ? "true" : "false");
    return out;
}

static bool s2patch_eligible(const sgprs_conv_desc_t& d)
{
    return d.dtype == SGPRS_BF16 && d.r == 3 && d.s == 3 && d.stride == 2 && d.pad == 1 && d.h % 2 == 0 && d.w % 2 == 0 &&
           d.h >= 2 && d.w >= 2 && d.w <= 128 && d.h <= 252 && d.cin % 32 == 0 && d.cout % 64 == 0 &&
           (long long)d.n * d.h * d.w * d.cin * 2 < (1ll << 31) && (long long)d.cout * 9 * d.cin * 2 < (1ll << 31) &&
           (long long)d.n * (d.h + 2) * (d.h + 2) < (1ll << 30);
}

static bool s2patch_geometry_uncached(const sgprs_conv_desc_t& d, int v, S2Args* a);
static bool s2patch_geometry(const sgprs_conv_desc_t& d, int v, S2Args* a)
{
    struct Key { sgprs_conv_desc_t d; int v; };
    struct Val { bool ok; S2Args a; };
    static thread_local PlanMemo<Key, Val, 64> local;
    static SharedPlanMemo<Key, Val, 64> memo;
    Key k;
    memset(&k, 0, sizeof(k));
    k.d = d; k.v = v;
    const Val hit = memo.get(local, k, [&]() {
        Val nv;
        memset(&nv, 0, sizeof(nv));
        nv.ok = s2patch_geometry_uncached(d, v, &nv.a);
        return nv;
    });
    if (hit.ok) *a = hit.a;
    return hit.ok;
}
static bool s2patch_geometry_uncached(const sgprs_conv_desc_t& d, int v, S2Args* a)
{
    const int bm = kS2Variants[v].bm;
    const int Ho = d.h / 2, Wo = d.w / 2, NHo = d.n * Ho, PWh = Wo + 1;
    if (Wo > bm) return false;
    const int ppl = s2_patch_cap(bm) / 4;
    int TR = bm / Wo, n_mtiles = 0;
    for (; TR >= 1; --TR) {  // the most output rows per tile whose plane rows (one more than output rows, plus one per image border) fit
        n_mtiles = (NHo + TR - 1) / TR;
        int rmax = 0;
        for (int t = 0; t < n_mtiles; ++t) {
            const int g0 = t * TR, g1 = std::min(g0 + TR, NHo) - 1;
            rmax = std::max(rmax, (g1 + g1 / Ho) - (g0 + g0 / Ho) + 2);
        }
        if (rmax * PWh <= ppl && rmax < 256) break;
    }
    if (TR < 1 || TR * Wo * 2 < bm) return false;  // a tile less than half full is left to the implicit GEMM
    a->H = d.h; a->W = d.w; a->Cin = d.cin; a->Cout = d.cout; a->Ho = Ho; a->Wo = Wo; a->NHo = NHo;
    a->PWh = PWh; a->HE = d.h + 2;
    a->mWo = magic_for(Wo); a->mPWh = magic_for(PWh); a->mHE = magic_for(d.h + 2); a->mHo = magic_for(Ho);
    a->TR = TR; a->n_mtiles = n_mtiles; a->n_ntiles = d.cout / 64; a->n_chunks = d.cin / 16; a->splits = 1;
    a->relu = d.relu;
    patch_index_space(n_mtiles, a->n_ntiles, 1, &a->xcd_groups, &a->n_slots);
    return true;
}

// The stride-2 kernel runs only when asked for (tuning override): measured at batch 64 on 256 CUs
// it takes 25-28 / 20-23 / 26-28 us for the three down-sampling blocks of ResNet18 against
// 24 / 22 / 24-26 us for the paired implicit GEMM.  Its patch moves fewer bytes from the L2, but in
// 32-byte pieces (16 channels of every other pixel), and a step of nine or ten k-steps is too
// short for its barrier; chunks of 32 channels would need 172 KB of LDS.
bool plan_s2patch(const sgprs_conv_desc_t& d, int cus, int* variant)
{
    (void)cus;
    const int force = g_s2_force.load();
    if (force < 0 || force >= kNumS2Variants || !s2patch_eligible(d)) return false;
    S2Args a;
    if (!s2patch_geometry(d, force, &a)) return false;
    *variant = force;
    return true;
}

template <int BM, int NW>
static int launch_s2_variant(const S2Args& a, int grid, hipStream_t stream)
{
    constexpr int kLds = 2 * (s2_patch_cap(BM) * 32 + 64 * 9 * 32 + 64 * 32);
    static_assert(kLds <= 160 * 1024, "LDS of one CU");
    static std::atomic<bool> raised{false};
    if (!raised) {
        SGPRS_HIP(hipFuncSetAttribute((const void*)conv3x3s2_patch_kernel<BM, NW, true>, hipFuncAttributeMaxDynamicSharedMemorySize, kLds));
        SGPRS_HIP(hipFuncSetAttribute((const void*)conv3x3s2_patch_kernel<BM, NW, false>, hipFuncAttributeMaxDynamicSharedMemorySize, kLds));
        raised = true;
    }
    if (a.w2)
        SGPRS_LAUNCH((conv3x3s2_patch_kernel<BM, NW, true>), dim3(grid), dim3(NW * 64), kLds, stream, a);
    else
        SGPRS_LAUNCH((conv3x3s2_patch_kernel<BM, NW, false>), dim3(grid), dim3(NW * 64), kLds, stream, a);
    SGPRS_HIP(hipGetLastError());
    return SGPRS_OK;
}

// d: the 3x3 stride-2 convolution; d2 (may be null): the 1x1 stride-2 shortcut on the same input.
int launch_conv3x3s2_patch(const sgprs_conv_desc_t& d, int variant, const void* x, const void* w, const float* scale,
                           const float* shift, void* y, const sgprs_conv_desc_t* d2, const void* w2, const float* scale2,
                           const float* shift2, void* y2, hipStream_t stream, int cus, Profiler* prof)
{
    S2Args a;
    if (variant < 0 || variant >= kNumS2Variants || !s2patch_eligible(d) || !s2patch_geometry(d, variant, &a))
        return fail(SGPRS_ERR_INVALID_ARG, "internal: stride-2 patch plan does not match the shape");
    if (d2 && (d2->dtype != d.dtype || d2->n != d.n || d2->h != d.h || d2->w != d.w || d2->cin != d.cin || d2->cout != d.cout ||
               d2->r != 1 || d2->s != 1 || d2->stride != 2 || d2->pad != 0 || d2->relu))
        return fail(SGPRS_ERR_INVALID_ARG, "internal: shortcut does not match the 3x3 convolution");
    a.x = (const unsigned char*)x; a.w = (const unsigned char*)w; a.y = (unsigned char*)y;
    a.scale = scale; a.shift = shift;
    a.w2 = d2 ? (const unsigned char*)w2 : nullptr; a.y2 = (unsigned char*)y2; a.scale2 = scale2; a.shift2 = shift2;
    a.x_bytes = (unsigned)((size_t)d.n * d.h * d.w * d.cin * 2); a.w_bytes = (unsigned)((size_t)d.cout * 9 * d.cin * 2);
    a.w2_bytes = (unsigned)((size_t)d.cout * d.cin * 2);
    int grid = (int)std::min<long long>(a.n_slots, (long long)cus);
    if (a.xcd_groups && grid >= 8) grid -= grid % 8;
    const double M = (double)a.NHo * a.Wo;
    const double flops = 2.0 * M * d.cout * (9.0 + (d2 ? 1.0 : 0.0)) * d.cin;
    const double bytes = ((double)d.n * d.h * d.w * d.cin + (double)d.cout * (9 + (d2 ? 1 : 0)) * d.cin + M * d.cout * (d2 ? 2 : 1)) * 2.0;
    int rc;
    if (prof && prof->on && (rc = prof->begin(stream, kKindS2Patch, variant + (d2 ? 4 : 0), flops, bytes))) return rc;
    rc = variant == 0 ? launch_s2_variant<256, 8>(a, grid, stream) : launch_s2_variant<128, 4>(a, grid, stream);
    if (rc) return rc;
    if (prof && prof->on && (rc = prof->end(stream))) return rc;
    return SGPRS_OK;
}

}  // namespace sgprs
