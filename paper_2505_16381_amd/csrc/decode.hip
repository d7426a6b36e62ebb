// Decode path of PaTH attention (paper Sec. 3.4 "Efficient Inference").
//
//  * Key prefill (the section's second formula): the cache a prompt leaves behind holds
//    k_i^(l) = H_l ... H_{i+1} k_i.  Blockwise with suffix products, on top of what the forward's
//    preprocessing already wrote: Kb2_c (keys carried to their super-block's right edge) and
//    -dP2_J = -(I - P_superblock J).  With E = I - R (R = P2_last ... P2_{J+1}) kept transposed in
//    fp32 registers,
//        K^(l)_c = Kb2_c - Kb2_c E^T ,      E <- E + dP2_J - E dP2_J ,
//    exactly the second level's own recurrence one level up (see prep2_fwd.hip), so the cost is
//    linear in l.  One workgroup per (head, super-block): it runs the d x d recurrence from the
//    right end down to its own super-block (a few small products per step, the same for every
//    workgroup of the head, hence the same E) and carries only its own super-block's keys.
//    Results go row-major into the key cache, in the cache's storage type.
//
//  * Decode step (the section's first equation): when token t arrives every cached key is
//    refreshed in place, k_i <- k_i - beta_t (w_t . k_i) w_t, and attention of q_t over the
//    refreshed cache is ordinary softmax attention.  Both happen in ONE pass over the key cache
//    (read k, write k, read v: 3 n d elements per head -- HBM-bound), split over the cached
//    positions; a second small kernel merges the splits, adds the arriving token's own key and
//    value, and appends them to the caches.
//
//  * PaTH-FoX at decode time (Sec. 2.2 extension): with the running sums c_i of the log gates kept beside the
//    caches, key i's logit gets c_t - c_i, c_t = c_{t-1} + log f_t; the arriving token's own logit gets nothing
//    and its sum is appended (GATES instantiations of the two kernels).
#include "path_common.h"
#include "decode_decl.h"

namespace path {

// ---------------------------------------------------------------------------------------
template <typename TIO, int D> struct PrefillCfg {
    typedef typename Compute<TIO>::type T;
    static constexpr int KV_FRAGS = CHUNK * D / Tr<T>::FE, DP_FRAGS = D * D / Tr<T>::FE;
    // operand copy of E | -dP2 tile of the super-block | one key tile
    static constexpr size_t smem_bytes = (size_t)(2 * DP_FRAGS + KV_FRAGS) * 16;
};

template <typename TIO, int D>
__global__ __launch_bounds__(256) void key_prefill_kernel(PrefillArgs a) {
    using T = typename Compute<TIO>::type;
    using Frag = typename Tr<T>::Frag;
    typedef typename Tr<TIO>::Vec4 OVec4;
    constexpr int FE = Tr<T>::FE, KW = Tr<T>::KW;
    constexpr int SPB = 32 / KW, DB = D / 32, DS = D / KW, NE = DB * DB / 4, NK = 2 * DB / 4;
    constexpr int KVF = PrefillCfg<TIO, D>::KV_FRAGS, DPF = PrefillCfg<TIO, D>::DP_FRAGS;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    Frag* Es = reinterpret_cast<Frag*>(smem);      // tile (rows a, contraction b) of E
    Frag* sDP = Es + DPF;                          // -dP2 tile (rows b, contraction a)
    Frag* sK = sDP + DPF;                          // Kb2 tile of the current chunk (rows s, contraction c)

    const int bh = blockIdx.x, Jme = blockIdx.y;   // this workgroup carries the keys of super-block Jme
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, h = lane >> 5, l32 = lane & 31;
    const int NC = a.NC, L = a.L, nsb = (NC + SBC - 1) / SBC;
    if (Jme >= nsb) return;

    Frag idf[SPB];
    identity_frags<T>(idf, l32, h);
    f32x16 Fm[NE];      // E^T: block o = (rows b-block bb, lane a-block ab), blk = wv + 4*o

    for (int J = nsb - 1; J >= Jme; --J) {
        const bool lastsb = J == nsb - 1;          // E = 0: plain copy
        const int c0 = J * SBC, c1 = (c0 + SBC < NC) ? c0 + SBC : NC;
        if (J > Jme) {                             // on the way down: only the product of super-block J
            __syncthreads();                       // sDP is free
            async_copy_tile<256, DPF>(reinterpret_cast<const Frag*>(reinterpret_cast<const T*>(a.dp2) + ((size_t)bh * nsb + J) * (size_t)D * D), sDP, tid, wv);
            wait_async_and_sync();
        }
        for (int c = c0; c < c1 && J == Jme; ++c) {
            const size_t bhc = (size_t)bh * NC + c;
            __syncthreads();                       // sK is free (and, first time round, Es is written)
            async_copy_tile<256, KVF>(reinterpret_cast<const Frag*>(reinterpret_cast<const T*>(a.kt2) + bhc * (size_t)CHUNK * D), sK, tid, wv);
            wait_async_and_sync();
            // K^(l)^T[cc][s] = Kb2^T[cc][s] - sum_b E[cc][b] Kb2[s][b]   (registers rows cc, lane s)
#pragma unroll
            for (int o = 0; o < NK; ++o) {
                const int blk = wv + 4 * o, cb = blk >> 1, sb2 = blk & 1;
                f32x16 acc = zero16();
                if (!lastsb) {
#pragma unroll
                    for (int s = 0; s < DS; ++s) acc = Tr<T>::mma(Es[(cb * DS + s) * 64 + lane], sK[((size_t)sb2 * DS + s) * 64 + lane], acc);
                }
                const int s = 32 * sb2 + l32, tok = c * CHUNK + s;
                if (tok < L) {
                    TIO* dst = reinterpret_cast<TIO*>(a.kcache) + ((size_t)bh * a.Lmax + tok) * D + 32 * cb + 4 * h;
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        // accumulator register jj = 4g + r holds column 32cb + 8g + 4h + r of key s; the tile's
                        // fragment order keeps that same element at slab jj / FE, position jj % FE of this lane
                        OVec4 o4;
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            const int jj = 4 * g + r;
                            const Frag kf = sK[((size_t)sb2 * DS + cb * SPB + jj / FE) * 64 + lane];
                            o4[r] = (TIO)((float)kf[jj % FE] - acc[jj]);
                        }
                        *reinterpret_cast<OVec4*>(dst + 8 * g) = o4;
                    }
                }
            }
        }
        if (J == Jme) break;
        // E^T <- E^T + dP2^T - dP2^T E^T   (registers rows b, lane a)
#pragma unroll
        for (int o = 0; o < NE; ++o) {
            const int blk = wv + 4 * o, bb = blk / DB, ab = blk % DB;
            f32x16 acc = zero16();
            if (!lastsb) {
#pragma unroll
                for (int s = 0; s < DS; ++s) acc = Tr<T>::mma(sDP[((size_t)bb * DS + s) * 64 + lane], Es[(ab * DS + s) * 64 + lane], acc);
            }
            Frag dfr[SPB];
#pragma unroll
            for (int s2 = 0; s2 < SPB; ++s2) dfr[s2] = sDP[((size_t)bb * DS + ab * SPB + s2) * 64 + lane];
            const f32x16 dpT = transpose32<T>(dfr, idf);
#pragma unroll
            for (int jj = 0; jj < 16; ++jj) {
                const float prev = lastsb ? 0.f : Fm[o][jj];
                Fm[o][jj] = prev - dpT[jj] + acc[jj];
            }
        }
        __syncthreads();      // every read of the old operand copy is done
#pragma unroll
        for (int o = 0; o < NE; ++o) {
            const int blk = wv + 4 * o, bb = blk / DB, ab = blk % DB;
            Frag fr[SPB];
            pack_block<T>(Fm[o], fr);
#pragma unroll
            for (int s2 = 0; s2 < SPB; ++s2) Es[(ab * DS + bb * SPB + s2) * 64 + lane] = fr[s2];
        }
    }
}

// ---------------------------------------------------------------------------------------
// One pass over the cached keys of a split: refresh, logit, online softmax, P V.
// A key is handled by LPK = D/8 consecutive lanes (8 elements each); a wave takes 64/LPK keys
// per round.  Partial results (m, l, o[D]) per split go to the workspace.
template <typename TIO, int D, bool GATES>
__global__ __launch_bounds__(256) void decode_partial_kernel(DecodeArgs a) {
    constexpr int LPK = D / 8, KPW = 64 / LPK, GROUPS = 4 * KPW;
    typedef TIO Vec8 __attribute__((ext_vector_type(8)));
    __shared__ float red_m[GROUPS], red_l[GROUPS];
    __shared__ float red_o[GROUPS][D];

    const int split = blockIdx.x, bh = blockIdx.y, nsplit = gridDim.x;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int grp = lane / LPK, sub = lane % LPK;                 // key within the wave's round; 8-element slice
    const int n = a.n;
    const int i_begin = (int)((long long)n * split / nsplit), i_end = (int)((long long)n * (split + 1) / nsplit);

    float q8[8], w8[8];
    {
        const Vec8 qv = *reinterpret_cast<const Vec8*>(reinterpret_cast<const TIO*>(a.q) + (size_t)bh * D + 8 * sub);
        const Vec8 wv8 = *reinterpret_cast<const Vec8*>(reinterpret_cast<const TIO*>(a.w) + (size_t)bh * D + 8 * sub);
#pragma unroll
        for (int e = 0; e < 8; ++e) { q8[e] = (float)qv[e]; w8[e] = (float)wv8[e]; }
    }
    const float beta = (float)reinterpret_cast<const TIO*>(a.beta)[bh];
    const float* cc = GATES ? a.ccache + (size_t)bh * a.Lmax : nullptr;
    const float c_t = GATES ? (n > 0 ? cc[n - 1] : 0.f) + (float)reinterpret_cast<const TIO*>(a.log_f)[bh] : 0.f;
    auto group_sum = [&](float x) {
#pragma unroll
        for (int off = 1; off < LPK; off <<= 1) x += __shfl_xor(x, off);
        return x;
    };

    TIO* kc = reinterpret_cast<TIO*>(a.kcache) + (size_t)bh * a.Lmax * D + 8 * sub;
    const TIO* vc = reinterpret_cast<const TIO*>(a.vcache) + (size_t)bh * a.Lmax * D + 8 * sub;
    float m = -INFINITY, l = 0.f, acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;

    for (int i0 = i_begin + wv * KPW; i0 < i_end; i0 += GROUPS) {
        const int i = i0 + grp;
        const bool ok = i < i_end;
        float k8[8], v8[8];
        if (ok) {
            const Vec8 kv = *reinterpret_cast<const Vec8*>(kc + (size_t)i * D);
            const Vec8 vv = *reinterpret_cast<const Vec8*>(vc + (size_t)i * D);
#pragma unroll
            for (int e = 0; e < 8; ++e) { k8[e] = (float)kv[e]; v8[e] = (float)vv[e]; }
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) { k8[e] = 0.f; v8[e] = 0.f; }
        }
        float wk = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) wk += w8[e] * k8[e];
        wk = group_sum(wk);
        // refreshed key, rounded to the cache's storage type: the stored value is the state, and
        // the logit is taken against it
        Vec8 kn;
        float qk = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            kn[e] = (TIO)(k8[e] - beta * wk * w8[e]);
            qk += q8[e] * (float)kn[e];
        }
        qk = group_sum(qk);
        if (ok) {
            *reinterpret_cast<Vec8*>(kc + (size_t)i * D) = kn;
            const float s = GATES ? a.scale * qk + (c_t - cc[i]) : a.scale * qk;
            const float mn = fmaxf(m, s);
            const float alpha = __expf(m - mn), pr = __expf(s - mn);      // m = -inf first time: alpha = 0
            l = l * alpha + pr;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] = acc[e] * alpha + pr * v8[e];
            m = mn;
        }
    }
    // merge the lane groups of the workgroup
    const int g = wv * KPW + grp;
    if (sub == 0) { red_m[g] = m; red_l[g] = l; }
#pragma unroll
    for (int e = 0; e < 8; ++e) red_o[g][8 * sub + e] = acc[e];
    __syncthreads();
    if (tid < D) {
        float M = -INFINITY;
        for (int gg = 0; gg < GROUPS; ++gg) M = fmaxf(M, red_m[gg]);
        float Ls = 0.f, O = 0.f;
        for (int gg = 0; gg < GROUPS; ++gg) {
            const float sc = (red_m[gg] == -INFINITY) ? 0.f : __expf(red_m[gg] - M);
            Ls += red_l[gg] * sc;
            O += red_o[gg][tid] * sc;
        }
        float* part = a.partial + ((size_t)bh * nsplit + split) * (D + 2);
        part[2 + tid] = O;
        if (tid == 0) { part[0] = M; part[1] = Ls; }
    }
}

// Merge the splits, add the arriving token's own key/value, normalise; append to the caches.
template <typename TIO, int D, bool GATES>
__global__ __launch_bounds__(D) void decode_combine_kernel(DecodeArgs a, int nsplit) {
    __shared__ float sq[D];
    const int bh = blockIdx.x, c = threadIdx.x;
    const float qc = (float)reinterpret_cast<const TIO*>(a.q)[(size_t)bh * D + c];
    const TIO kt = reinterpret_cast<const TIO*>(a.k)[(size_t)bh * D + c];
    const TIO vt = reinterpret_cast<const TIO*>(a.v)[(size_t)bh * D + c];
    sq[c] = qc * (float)kt;
    __syncthreads();
    for (int off = D / 2; off > 0; off >>= 1) {
        if (c < off) sq[c] += sq[c + off];
        __syncthreads();
    }
    const float s_new = a.scale * sq[0];
    const float* part = a.partial + (size_t)bh * nsplit * (D + 2);
    float M = s_new;
    for (int s = 0; s < nsplit; ++s) M = fmaxf(M, part[(size_t)s * (D + 2)]);
    float Ls = __expf(s_new - M), O = Ls * (float)vt;
    for (int s = 0; s < nsplit; ++s) {
        const float ms = part[(size_t)s * (D + 2)];
        const float sc = (ms == -INFINITY) ? 0.f : __expf(ms - M);
        Ls += part[(size_t)s * (D + 2) + 1] * sc;
        O += part[(size_t)s * (D + 2) + 2 + c] * sc;
    }
    reinterpret_cast<TIO*>(a.o)[(size_t)bh * D + c] = (TIO)(O / Ls);
    if (c == 0) a.lse[bh] = M + __logf(Ls);
    reinterpret_cast<TIO*>(a.kcache)[((size_t)bh * a.Lmax + a.n) * D + c] = kt;
    reinterpret_cast<TIO*>(a.vcache)[((size_t)bh * a.Lmax + a.n) * D + c] = vt;
    if (GATES && c == 0) {      // the arriving token's running gate sum joins the cache (its own logit carries no gate)
        float* cc = a.ccache + (size_t)bh * a.Lmax;
        cc[a.n] = (a.n > 0 ? cc[a.n - 1] : 0.f) + (float)reinterpret_cast<const TIO*>(a.log_f)[bh];
    }
}

// ---------------------------------------------------------------------------------------
template <typename TIO, int D>
static hipError_t launch_prefill_t(const PrefillArgs& a, int BH, hipStream_t st) {
    const size_t bytes = PrefillCfg<TIO, D>::smem_bytes;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&key_prefill_kernel<TIO, D>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((key_prefill_kernel<TIO, D>), dim3(BH, (a.NC + SBC - 1) / SBC), dim3(256), bytes, st, a);
    return hipGetLastError();
}
hipError_t launch_key_prefill(const PrefillArgs& a, int BH, int d, int is_bf16, hipStream_t st) {
    if (is_bf16) return d == 64 ? launch_prefill_t<bf16_t, 64>(a, BH, st) : launch_prefill_t<bf16_t, 128>(a, BH, st);
    return d == 64 ? launch_prefill_t<float, 64>(a, BH, st) : launch_prefill_t<float, 128>(a, BH, st);
}

int decode_num_splits(int BH, int n) {
    int s = (1024 + BH - 1) / BH;                 // about four workgroups per CU
    if (s > DECODE_MAX_SPLITS) s = DECODE_MAX_SPLITS;
    const int by_len = (n + 127) / 128;           // at least ~128 keys per split
    if (s > by_len) s = by_len;
    return s < 1 ? 1 : s;
}

template <typename TIO, int D, bool GATES>
static hipError_t launch_decode_g(const DecodeArgs& a, int BH, hipStream_t st) {
    const int nsplit = decode_num_splits(BH, a.n);
    hipLaunchKernelGGL((decode_partial_kernel<TIO, D, GATES>), dim3(nsplit, BH), dim3(256), 0, st, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((decode_combine_kernel<TIO, D, GATES>), dim3(BH), dim3(D), 0, st, a, nsplit);
    return hipGetLastError();
}
template <typename TIO, int D>
static hipError_t launch_decode_t(const DecodeArgs& a, int BH, hipStream_t st) {
    return a.ccache ? launch_decode_g<TIO, D, true>(a, BH, st) : launch_decode_g<TIO, D, false>(a, BH, st);
}
hipError_t launch_decode_step(const DecodeArgs& a, int BH, int d, int is_bf16, hipStream_t st) {
    if (is_bf16) return d == 64 ? launch_decode_t<bf16_t, 64>(a, BH, st) : launch_decode_t<bf16_t, 128>(a, BH, st);
    return d == 64 ? launch_decode_t<float, 64>(a, BH, st) : launch_decode_t<float, 128>(a, BH, st);
}

}  // namespace path
