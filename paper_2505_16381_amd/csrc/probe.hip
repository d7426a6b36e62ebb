// Measurement aid: register-resident MFMA chain, for calibrating "percent of peak" against the rate the
// matrix pipes deliver at the clock the chip holds under that load (the datasheet figure assumes 2.4 GHz).
// The clock depends on the power the products draw, and that on the operands: with smooth, slowly varying
// operands the chain runs at about 2.1 PFLOP/s, with operands of random sign and significand -- what the
// method's kernels multiply -- at about 1.6 PFLOP/s.  Both patterns are offered.
#include "../../include/path_attn.h"
#include "path_common.h"

namespace path {

// fp16 value of random sign, exponent field 13..16 (0.25 <= |x| < 4) and random significand from a hash of n
__device__ __forceinline__ half_t random_half(unsigned n) {
    n = n * 747796405u + 2891336453u;
    n = ((n >> ((n >> 28) + 4)) ^ n) * 277803737u;
    n = (n >> 22) ^ n;
    const unsigned short bits = (unsigned short)((n & 0x8000u) | ((13u + ((n >> 10) & 3u)) << 10) | (n & 0x3ffu));
    return __builtin_bit_cast(half_t, bits);
}

template <int NW>
__global__ __launch_bounds__(64 * NW) void mfma_probe_kernel(float* sink, int iters, int random_operands) {
    const int lane = threadIdx.x & 63;
    halfx8 a[4], b[4];
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            if (random_operands) {
                a[s][e] = random_half((threadIdx.x * 4 + s) * 8 + e);
                b[s][e] = random_half(0x10000u + (threadIdx.x * 4 + s) * 8 + e);
            } else {
                a[s][e] = (half_t)(0.001f * (lane + s + e));
                b[s][e] = (half_t)(0.001f * (s + 2 * e));
            }
        }
    f32x16 acc[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) acc[s] = zero16();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int s = 0; s < 4; ++s) acc[s] = Tr<half_t>::mma(a[s], b[u], acc[s]);
    }
    float r = 0.f;
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int j = 0; j < 16; ++j) r += acc[s][j];
    sink[(size_t)blockIdx.x * 256 + (threadIdx.x & 255)] = r;      // (waves of a workgroup beyond the fourth share slots: nobody reads them)
}

}  // namespace path

extern "C" double path_probe_mfma_flops(int waves_per_simd, int iters) {
    return 256.0 * 4 * waves_per_simd * (double)iters * 16 * 2.0 * 32 * 32 * 16;
}

extern "C" path_status_t path_probe_mfma(void* sink, int waves_per_simd, int iters, void* stream) {
    return path_probe_mfma_operands(sink, waves_per_simd, iters, 0, stream);
}

extern "C" path_status_t path_probe_mfma_operands(void* sink, int waves_per_simd, int iters, int random_operands, void* stream) {
    if (!sink) return PATH_ERR_NULL;
    if ((waves_per_simd != 1 && waves_per_simd != 2 && waves_per_simd != 4) || iters < 1) return PATH_ERR_SHAPE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    float* out = static_cast<float*>(sink);
    (void)hipGetLastError();
    // one workgroup per CU (256 of them): a workgroup of 4 * waves_per_simd waves puts waves_per_simd on each SIMD
    if (waves_per_simd == 1) hipLaunchKernelGGL((path::mfma_probe_kernel<4>), dim3(256), dim3(256), 0, st, out, iters, random_operands);
    else if (waves_per_simd == 2) hipLaunchKernelGGL((path::mfma_probe_kernel<8>), dim3(256), dim3(512), 0, st, out, iters, random_operands);
    else hipLaunchKernelGGL((path::mfma_probe_kernel<16>), dim3(256), dim3(1024), 0, st, out, iters, random_operands);
    return hipGetLastError() == hipSuccess ? PATH_OK : PATH_ERR_HIP;
}
