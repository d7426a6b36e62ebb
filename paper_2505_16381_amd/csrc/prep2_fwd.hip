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
// Kb2_c = Kb_c - Kb_c E_c^T.
//
// One workgroup per (batch*head, super-block).  E is kept TRANSPOSED in fp32
// registers (rows b, lane a): in that layout its operand copy is directly the
// fragment-order tile (rows a, contraction b) that both products need -- as the
// A operand of the key transport and as the B operand of the update -- and the
// other operands are the fragment tiles the chunk kernel already wrote (keys and
// -dP), read straight from global memory; where -dP is needed element-wise in the
// transposed register layout it is transposed through the matrix unit.
#include "path_common.h"

namespace path {

template <typename TIO, int D> struct Prep2Cfg {
    typedef typename Compute<TIO>::type T;
    static constexpr int KV_FRAGS = CHUNK * D / Tr<T>::FE, DP_FRAGS = D * D / Tr<T>::FE;
    static constexpr int NBUF = sizeof(T) == 2 ? 2 : 1;      // fp32 tiles: one stage only fits
    // operand copy of E (fragment order) + NBUF stages of (key tile | -dP tile) of a chunk
    static constexpr size_t smem_bytes = (size_t)D * D * sizeof(T) + (size_t)NBUF * (KV_FRAGS + DP_FRAGS) * 16;
};

// BWD: also write the backward-only outputs (compile-time, so the forward carries none of that code).
template <typename TIO, int D, bool BWD>
__global__ __launch_bounds__(256) void prep2_fwd_kernel(FwdParams p) {
    using T = typename Compute<TIO>::type;
    using Frag = typename Tr<T>::Frag;
    constexpr int FE = Tr<T>::FE, KW = Tr<T>::KW;
    constexpr int SPB = 32 / KW, DB = D / 32, DS = D / KW, NE = DB * DB / 4, NK = 2 * DB / 4;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    Frag* Es = reinterpret_cast<Frag*>(smem);      // tile (rows a, contraction b) of E

    const int sb = blockIdx.x, bh = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wv = __builtin_amdgcn_readfirstlane(tid >> 6), h = lane >> 5, l32 = lane & 31;
    const int NC = p.NC;                                                   // chunks per head in the workspace arrays
    const int NCown = (seq_len(p.ul, bh, p.L) + CHUNK - 1) / CHUNK;        // this head's own (packed batches: may be fewer)
    const int c0 = sb * SBC;
    if (c0 >= NCown) return;
    const int clast = (c0 + SBC - 1 < NCown) ? c0 + SBC - 1 : NCown - 1;

    Frag idf[SPB];
    identity_frags<T>(idf, l32, h);
    f32x16 Fm[NE];      // E^T: block o = (rows b-block bb, lane a-block ab), blk = wv + 4*o, bb = blk / DB, ab = blk % DB

    // the chunk's key and -dP tiles are copied to LDS (direct-to-LDS), one chunk ahead where two stages fit
    constexpr int KVF = Prep2Cfg<TIO, D>::KV_FRAGS, DPF = Prep2Cfg<TIO, D>::DP_FRAGS, NBUF = Prep2Cfg<TIO, D>::NBUF;
    Frag* stage = Es + DPF;
    auto issue = [&](int c) {
        const size_t bhc = (size_t)bh * NC + c;
        Frag* buf = stage + (size_t)(c & (NBUF - 1)) * (KVF + DPF);
        async_copy_tile<256, KVF>(reinterpret_cast<const Frag*>(reinterpret_cast<const T*>(p.kt) + bhc * (size_t)CHUNK * D), buf, tid, wv);
        async_copy_tile<256, DPF>(reinterpret_cast<const Frag*>(reinterpret_cast<const T*>(p.dp) + bhc * (size_t)D * D), buf + KVF, tid, wv);
    };
    if (NBUF == 2) issue(clast);
    for (int c = clast; c >= c0; --c) {
        const size_t bhc = (size_t)bh * NC + c;
        if (NBUF == 2) {
            wait_async_and_sync();             // chunk c has landed; everyone is done with chunk c+1
            if (c > c0) issue(c - 1);
        } else {
            __syncthreads();
            issue(c);
            wait_async_and_sync();
        }
        const Frag* k1 = stage + (size_t)(c & (NBUF - 1)) * (KVF + DPF);
        const Frag* dpn = k1 + KVF;                                                                                  // (rows b, contr a) = -dP[a][b]
        Frag* k2 = reinterpret_cast<Frag*>(reinterpret_cast<T*>(p.kt2) + bhc * (size_t)CHUNK * D);
        // (the transposed arrangement of the second-level keys: fp32 operands only, as for the chunk-level ones)
        Frag* k2T = (BWD && p.kt2T && sizeof(T) == 4) ? reinterpret_cast<Frag*>(reinterpret_cast<T*>(p.kt2T) + bhc * (size_t)CHUNK * D) : nullptr;
        if (BWD && p.rm) {      // backward only: R_c = I - E_c, row-major [a][b]
            typedef typename Tr<T>::Vec4 TVec4;
            T* rdst = reinterpret_cast<T*>(p.rm) + bhc * (size_t)D * D;
#pragma unroll
            for (int o = 0; o < NE; ++o) {
                const int blk = wv + 4 * o, bb = blk / DB, ab = blk % DB;
                const int a = 32 * ab + l32;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    TVec4 o4;
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int b = 32 * bb + 8 * g + 4 * h + r;
                        const float e = (c == clast) ? 0.f : Fm[o][4 * g + r];
                        o4[r] = (T)((a == b ? 1.f : 0.f) - e);
                    }
                    *reinterpret_cast<TVec4*>(rdst + (size_t)a * D + 32 * bb + 8 * g + 4 * h) = o4;
                }
            }
        }
        if (c == clast) {
            for (int idx = tid; idx < CHUNK * D / FE; idx += 256) k2[idx] = k1[idx];
            if (k2T) {
                const Frag* k1T = reinterpret_cast<const Frag*>(reinterpret_cast<const T*>(p.ktT) + bhc * (size_t)CHUNK * D);
                for (int idx = tid; idx < CHUNK * D / FE; idx += 256) __builtin_nontemporal_store(k1T[idx], &k2T[idx]);
            }
        } else {
            // Kb2^T[cc][s] = Kb^T[cc][s] - sum_b E[cc][b] Kb[s][b]   (registers rows cc, lane s)
#pragma unroll
            for (int o = 0; o < NK; ++o) {
                const int blk = wv + 4 * o, cb = blk >> 1, sb2 = blk & 1;
                f32x16 acc = zero16();
#pragma unroll
                for (int s = 0; s < DS; ++s) acc = Tr<T>::mma(Es[(cb * DS + s) * 64 + lane], k1[((size_t)sb2 * DS + s) * 64 + lane], acc);
                Frag fr[SPB];
#pragma unroll
                for (int s2 = 0; s2 < SPB; ++s2) {
                    const Frag kf = k1[((size_t)sb2 * DS + cb * SPB + s2) * 64 + lane];
#pragma unroll
                    for (int e = 0; e < FE; ++e) fr[s2][e] = (T)((float)kf[e] - acc[s2 * FE + e]);
                }
#pragma unroll
                for (int s2 = 0; s2 < SPB; ++s2) __builtin_nontemporal_store(fr[s2], &k2[((size_t)sb2 * DS + cb * SPB + s2) * 64 + lane]);
                if (k2T) {     // backward only: the arrangement (rows cc, contraction s)
                    const f32x16 tr = transpose32<T>(fr, idf);      // rows s, lane cc
                    Frag ft[SPB];
                    pack_block<T>(tr, ft);
#pragma unroll
                    for (int s2 = 0; s2 < SPB; ++s2) __builtin_nontemporal_store(ft[s2], &k2T[((size_t)cb * (CHUNK / KW) + sb2 * SPB + s2) * 64 + lane]);
                }
            }
        }
        // E^T <- E^T + dP^T - dP^T E^T   (registers rows b, lane a)
#pragma unroll
        for (int o = 0; o < NE; ++o) {
            const int blk = wv + 4 * o, bb = blk / DB, ab = blk % DB;
            f32x16 acc = zero16();
            if (c != clast) {
#pragma unroll
                for (int s = 0; s < DS; ++s) acc = Tr<T>::mma(dpn[((size_t)bb * DS + s) * 64 + lane], Es[(ab * DS + s) * 64 + lane], acc);
            }
            // -dP[a][b] in this block's register layout (rows b, lane a): the tile piece (rows b,
            // contraction a) transposed through the matrix unit
            Frag dfr[SPB];
#pragma unroll
            for (int s2 = 0; s2 < SPB; ++s2) dfr[s2] = dpn[((size_t)bb * DS + ab * SPB + s2) * 64 + lane];
            const f32x16 dpT = transpose32<T>(dfr, idf);
#pragma unroll
            for (int jj = 0; jj < 16; ++jj) {
                const float prev = (c == clast) ? 0.f : Fm[o][jj];
                Fm[o][jj] = prev - dpT[jj] + acc[jj];
            }
        }
        __syncthreads();      // every read of the old operand copy is done
        if (c > c0) {
#pragma unroll
            for (int o = 0; o < NE; ++o) {
                const int blk = wv + 4 * o, bb = blk / DB, ab = blk % DB;
                Frag fr[SPB];
                pack_block<T>(Fm[o], fr);
#pragma unroll
                for (int s2 = 0; s2 < SPB; ++s2) Es[(ab * DS + bb * SPB + s2) * 64 + lane] = fr[s2];
            }
        }
        __syncthreads();
    }
    // -(I - P_superblock) as the sweep's tile (rows b, contraction a): E itself (rows a, lane b) is the
    // transpose of what the registers hold -- taken through the matrix unit.
    Frag* dst = reinterpret_cast<Frag*>(reinterpret_cast<T*>(p.dp2) + ((size_t)bh * gridDim.x + sb) * (size_t)D * D);
#pragma unroll
    for (int o = 0; o < NE; ++o) {
        const int blk = wv + 4 * o, bb = blk / DB, ab = blk % DB;
        Frag fin[SPB];
        pack_block<T>(Fm[o], fin);                              // tile piece (rows a, contraction b)
        if (BWD && p.dpt2 && sizeof(T) == 4) {      // backward, fp32 operands only: -(I - P_superblock) in the arrangement (rows a, contraction b)
            Frag* dt = reinterpret_cast<Frag*>(reinterpret_cast<T*>(p.dpt2) + ((size_t)bh * gridDim.x + sb) * (size_t)D * D);
#pragma unroll
            for (int s = 0; s < SPB; ++s) {
                Frag ng;
#pragma unroll
                for (int e = 0; e < FE; ++e) ng[e] = (T)(-(float)fin[s][e]);
                __builtin_nontemporal_store(ng, &dt[((size_t)ab * DS + bb * SPB + s) * 64 + lane]);
            }
        }
        f32x16 tr = transpose32<T>(fin, idf);                   // rows a, lane b
#pragma unroll
        for (int jj = 0; jj < 16; ++jj) tr[jj] = -tr[jj];
        Frag fr[SPB];
        pack_block<T>(tr, fr);
#pragma unroll
        for (int s = 0; s < SPB; ++s) __builtin_nontemporal_store(fr[s], &dst[((size_t)bb * DS + ab * SPB + s) * 64 + lane]);
    }
}

template <typename TIO, int D, bool BWD>
hipError_t launch_prep2_fwd_b(const FwdParams& p, hipStream_t stream) {
    using C = Prep2Cfg<TIO, D>;
    // set once per process; a function-local static is initialised under the language's own lock
    static const hipError_t attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&prep2_fwd_kernel<TIO, D, BWD>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::smem_bytes);
    if (attr_err != hipSuccess) return attr_err;
    dim3 grid((p.NC + SBC - 1) / SBC, p.B * p.H);
    const size_t bytes = C::smem_bytes;
    hipLaunchKernelGGL((prep2_fwd_kernel<TIO, D, BWD>), grid, dim3(256), bytes, stream, p);
    return hipGetLastError();
}
template <typename TIO, int D>
hipError_t launch_prep2_fwd_t(const FwdParams& p, hipStream_t stream) {
    return p.rm ? launch_prep2_fwd_b<TIO, D, true>(p, stream) : launch_prep2_fwd_b<TIO, D, false>(p, stream);
}

hipError_t launch_prep2_fwd(const FwdParams& p, int d, int is_bf16, hipStream_t stream) {
    if (is_bf16) return d == 64 ? launch_prep2_fwd_t<bf16_t, 64>(p, stream) : launch_prep2_fwd_t<bf16_t, 128>(p, stream);
    return d == 64 ? launch_prep2_fwd_t<float, 64>(p, stream) : launch_prep2_fwd_t<float, 128>(p, stream);
}

}  // namespace path
