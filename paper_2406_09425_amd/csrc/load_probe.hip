// Sustained-rate probe for the load path of the convolution kernels: 16-byte
// buffer loads that go straight into LDS (the instruction that feeds every
// MFMA kernel here), eight wavefronts per CU, eight loads of 1 KiB per
// wavefront in flight, nothing else.  Every workgroup walks its own region of
// a caller-supplied buffer over and over; the region size decides where the
// data comes from: all regions together inside the L2s, or beyond them (memory
// -side cache and HBM).  What it reaches is the ceiling for the prologues,
// epilogues and k-tile streams of the kernels built on that instruction.
#include "internal.h"

namespace sgprs {

constexpr int kLoadProbeLds = 64 * 1024;  // one iteration = 8 wavefronts x 8 loads x 1 KiB

__global__ __launch_bounds__(512, 1) void load_probe_kernel(const unsigned char* __restrict__ buf, unsigned long long buf_bytes,
                                                            unsigned region, int iters, unsigned* __restrict__ out)
{
    extern __shared__ __align__(16) unsigned char smem[];
#if __HIP_DEVICE_COMPILE__  // the buffer-resource builtins exist in the device pass only
    typedef __attribute__((address_space(3))) void* lds_ptr_t;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const unsigned char* base = buf + ((unsigned long long)blockIdx.x * region) % buf_bytes;
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, (int)region, 0x00020000);
    unsigned off = wave * 8192 + lane * 16;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 8; ++u)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_ptr_t)(smem + (wave * 8 + u) * 1024), 16,
                                                     (off + u * 1024) & (region - 1), 0, 0, 0);
        __builtin_amdgcn_s_waitcnt(8 | 0x0F70);  // the previous iteration's loads have landed, this one's stay in flight
        off += kLoadProbeLds;
    }
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    // checksum of what the last iteration left in LDS: proves that the loads ran
    unsigned s = 0;
    for (int i = threadIdx.x; i < kLoadProbeLds / 4; i += 512) s += ((const unsigned*)smem)[i];
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) s += __shfl_xor(s, o, 64);
    __syncthreads();
    if (lane == 0) ((unsigned*)smem)[wave] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned t = 0;
        for (int w = 0; w < 8; ++w) t += ((const unsigned*)smem)[w];
        out[blockIdx.x] = t;
    }
#endif
}

int launch_load_probe(int cus, const void* buf, size_t buf_bytes, unsigned region, int iters, unsigned* out, hipStream_t stream)
{
    SGPRS_LAUNCH(load_probe_kernel, dim3(cus), dim3(512), kLoadProbeLds, stream, (const unsigned char*)buf,
                 (unsigned long long)buf_bytes, region, iters, out);
    SGPRS_HIP(hipGetLastError());
    return SGPRS_OK;
}

}  // namespace sgprs
