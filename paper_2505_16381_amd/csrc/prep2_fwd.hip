// Second blocking level of the forward (not in the paper; it follows from the
// associativity the paper uses in Sec. 3.2 for the cross-block term): inside a
// super-block of SBC chunks the boundary-adjusted keys are carried further, to
// the super-block's right edge, and the chunk products are multiplied up,
//
//     R_c = P_last ... P_{c+1}         (R_last = I),      R_{c-1} = R_c P_c
//     Kb2_c = Kb_c R_c^T ,             P_superblock = R_{first-1} ,
//
// so that the sweep applies ONE d x d product per super-block instead of one
// per chunk.  With E_c = I - R_c:  E_{c-1} = E_c + dP_c - E_c dP_c  and
// Kb2_c = Kb_c - Kb_c E_c^T.  E is kept in fp32 registers; only its operand
// copy (LDS) is rounded.  One workgroup per (batch*head, super-block).
#include "path_common.h"

namespace path {

template <typename TIO, int D> struct Prep2Cfg {
    typedef typename Compute<TIO>::type T;
    static constexpr int FE = Tr<T>::FE;
    static constexpr int LDE = D + FE;
    static constexpr size_t smem_bytes = (size_t)D * LDE * sizeof(T);
};

template <typename TIO, int D>
__global__ __launch_bounds__(256) void prep2_fwd_kernel(FwdParams p) {
    using C = Prep2Cfg<TIO, D>;
    using T = typename C::T;
    using Frag = typename Tr<T>::Frag;
    using Vec4 = typename Tr<T>::Vec4;
    constexpr int FE = C::FE, KW = Tr<T>::KW, LDE = C::LDE;
    constexpr int SPB = 32 / KW, DB = D / 32, NE = DB * DB / 4, NK = 2 * DB / 4;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    T* Es = reinterpret_cast<T*>(smem);        // operand copy of E, row-major [a][m]

    const int sb = blockIdx.x, bh = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, h = lane >> 5, l32 = lane & 31;
    const int NC = p.NC;
    const int c0 = sb * SBC;
    const int clast = (c0 + SBC - 1 < NC) ? c0 + SBC - 1 : NC - 1;

    f32x16 Em[NE];
#pragma unroll
    for (int o = 0; o < NE; ++o) Em[o] = zero16();

    for (int c = clast; c >= c0; --c) {
        const size_t bhc = (size_t)bh * NC + c;
        const T* kn = reinterpret_cast<const T*>(p.knat) + bhc * CHUNK * D;       // Kb_c [s][b]
        const T* dpt = reinterpret_cast<const T*>(p.dptnat) + bhc * (size_t)D * D;  // dP_c^T [b][m]
        Frag* k2 = reinterpret_cast<Frag*>(reinterpret_cast<T*>(p.kt2) + bhc * (size_t)CHUNK * D);
        if (c == clast) {
            const Frag* k1 = reinterpret_cast<const Frag*>(reinterpret_cast<const T*>(p.kt) + bhc * (size_t)CHUNK * D);
            for (int idx = tid; idx < CHUNK * D / FE; idx += 256) k2[idx] = k1[idx];
        } else {
            // Kb2^T[cc][s] = Kb^T[cc][s] - sum_b E[cc][b] Kb[s][b]   (acc rows cc, lane s)
#pragma unroll
            for (int o = 0; o < NK; ++o) {
                const int blk = wv + 4 * o, cb = blk >> 1, sb2 = blk & 1;
                f32x16 acc = gemm32<T, D>(Es, LDE, 32 * cb, kn, D, 32 * sb2, l32, h, zero16());
                const T* krow = kn + (size_t)(32 * sb2 + l32) * D + 32 * cb + 4 * h;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const Vec4 k4 = *reinterpret_cast<const Vec4*>(krow + 8 * g);
#pragma unroll
                    for (int r = 0; r < 4; ++r) acc[4 * g + r] = (float)k4[r] - acc[4 * g + r];
                }
                Frag fr[SPB];
                pack_block<T>(acc, fr);
#pragma unroll
                for (int s2 = 0; s2 < SPB; ++s2) k2[((size_t)sb2 * (D / KW) + cb * SPB + s2) * 64 + lane] = fr[s2];
            }
        }
        // E <- E + dP_c - E dP_c   (acc rows a, lane b)
#pragma unroll
        for (int o = 0; o < NE; ++o) {
            const int blk = wv + 4 * o, ab = blk / DB, bb = blk % DB;
            f32x16 acc = zero16();
            if (c != clast) acc = gemm32<T, D>(Es, LDE, 32 * ab, dpt, D, 32 * bb, l32, h, zero16());
            const T* drow = dpt + (size_t)(32 * bb + l32) * D + 32 * ab + 4 * h;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const Vec4 d4 = *reinterpret_cast<const Vec4*>(drow + 8 * g);
#pragma unroll
                for (int r = 0; r < 4; ++r) Em[o][4 * g + r] += (float)d4[r] - acc[4 * g + r];
            }
        }
        __syncthreads();      // every read of the old operand copy is done
        if (c > c0) {
#pragma unroll
            for (int o = 0; o < NE; ++o) {
                const int blk = wv + 4 * o, ab = blk / DB, bb = blk % DB;
#pragma unroll
                for (int jj = 0; jj < 16; ++jj) Es[(32 * ab + acc_row(jj, h)) * LDE + 32 * bb + l32] = (T)Em[o][jj];
            }
        }
        __syncthreads();
    }
    // -(I - P_superblock) as a fragment-order tile: rows = output column b, contraction = a
    Frag* dst = reinterpret_cast<Frag*>(reinterpret_cast<T*>(p.dp2) + ((size_t)bh * gridDim.x + sb) * (size_t)D * D);
#pragma unroll
    for (int o = 0; o < NE; ++o) {
        const int blk = wv + 4 * o, ab = blk / DB, bb = blk % DB;
        f32x16 acc;
#pragma unroll
        for (int jj = 0; jj < 16; ++jj) acc[jj] = -Em[o][jj];
        Frag fr[SPB];
        pack_block<T>(acc, fr);
#pragma unroll
        for (int s = 0; s < SPB; ++s) dst[((size_t)bb * (D / KW) + ab * SPB + s) * 64 + lane] = fr[s];
    }
}

template <typename TIO, int D>
hipError_t launch_prep2_fwd_t(const FwdParams& p, hipStream_t stream) {
    using C = Prep2Cfg<TIO, D>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&prep2_fwd_kernel<TIO, D>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::smem_bytes);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    dim3 grid((p.NC + SBC - 1) / SBC, p.B * p.H);
    const size_t bytes = C::smem_bytes;
    hipLaunchKernelGGL((prep2_fwd_kernel<TIO, D>), grid, dim3(256), bytes, stream, p);
    return hipGetLastError();
}

hipError_t launch_prep2_fwd(const FwdParams& p, int d, int is_bf16, hipStream_t stream) {
    if (is_bf16) return d == 64 ? launch_prep2_fwd_t<bf16_t, 64>(p, stream) : launch_prep2_fwd_t<bf16_t, 128>(p, stream);
    return d == 64 ? launch_prep2_fwd_t<float, 64>(p, stream) : launch_prep2_fwd_t<float, 128>(p, stream);
}

}  // namespace path
