// Backward of PaTH attention.  The paper gives no backward pass; this is the
// reverse-mode derivative of the blockwise forward (Sec. 3.2-3.3), organised as
//
//   1. prep (forward kernel, extra row-major outputs) and a states-only sweep:
//      Xs(i,j) = query state of chunk i as used against key chunk j < i.
//   2. bwd_delta:    delta_t = dO_t . o_t.
//   3. bwd_adjoint:  per query chunk i, left-to-right over key chunks j:
//        dS = scale * P o (dO V_j^T - delta),   P = exp(scale * Xs Kb_j^T - lse)
//        g(i,j) = dS Kb_j + g(i,j-1) (I - dP_j)^T          (g(i,-1) = 0)
//      g(i,i-1) is the gradient of the boundary-adjusted queries Qb_i.
//   4. bwd_keyside:  per key chunk j, over query chunks i > j (no atomics):
//        dV_j += P^T dO_i,  dKb_j += dS^T Xs(i,j),  ddP_j -= Xs(i,j)^T g(i,j-1).
//   5. chunk transform adjoint (Qb, Kb, dP, Sd -> q, k, w, beta): a short
//      sequence of batched 64x64xd products (batched_gemm) and elementwise steps.
//
// Steps 3 and 4 read their operands row-major from the workspace and stage the
// transposed copies they need through LDS.
#include "path_common.h"
#include "bwd_decl.h"

namespace path {

// ---------------------------------------------------------------------------------------
template <typename TIO, int D>
__global__ __launch_bounds__(256) void bwd_delta_kernel(BwdParams p) {
    const int chunk = blockIdx.x, bh = blockIdx.y, tid = threadIdx.x;
    const int row = tid >> 2, part = tid & 3;
    const int tg = chunk * CHUNK + row;
    float s = 0.f;
    if (tg < p.L) {
        const TIO* a = reinterpret_cast<const TIO*>(p.o) + ((size_t)bh * p.L + tg) * D + part * (D / 4);
        const TIO* b = reinterpret_cast<const TIO*>(p.dO) + ((size_t)bh * p.L + tg) * D + part * (D / 4);
#pragma unroll
        for (int c = 0; c < D / 4; ++c) s += (float)a[c] * (float)b[c];
    }
    s += __shfl_xor(s, 1);
    s += __shfl_xor(s, 2);
    if (part == 0) p.delta[(size_t)bh * p.NC * CHUNK + tg] = s;
}

// ---------------------------------------------------------------------------------------
template <typename TIO, int D> struct AdjCfg {
    typedef typename Compute<TIO>::type T;
    static constexpr int FE = Tr<T>::FE;
    static constexpr int LDD = D + FE, LDC = CHUNK + FE;
    static constexpr size_t smem_bytes = ((size_t)CHUNK * LDD + (size_t)CHUNK * LDC) * sizeof(T) + 2 * CHUNK * 4;
};

template <typename TIO, int D>
__global__ __launch_bounds__(256) void bwd_adjoint_kernel(BwdParams p) {
    using C = AdjCfg<TIO, D>;
    using T = typename C::T;
    constexpr int FE = C::FE, LDD = C::LDD, LDC = C::LDC;
    constexpr int DB = D / 32, NOWN = 2 * DB / 4;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    T* gT = reinterpret_cast<T*>(smem);                 // g(i,j-1), rows t
    T* dST = gT + CHUNK * LDD;                          // dS[t][s]
    float* lse2 = reinterpret_cast<float*>(dST + CHUNK * LDC);
    float* dl = lse2 + CHUNK;

    const int i = blockIdx.x, bh = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, h = lane >> 5, l32 = lane & 31;
    const int L = p.L, NC = p.NC;
    const size_t Lp = (size_t)NC * CHUNK, npairs = (size_t)NC * (NC - 1) / 2;
    const float sl2 = p.scale * 1.44269504088896340736f;

    f32x16 gm[NOWN];
#pragma unroll
    for (int o = 0; o < NOWN; ++o) gm[o] = zero16();

    for (int idx = tid; idx < CHUNK * LDD; idx += 256) gT[idx] = (T)0.f;
    if (tid < CHUNK) {
        const int tg = i * CHUNK + tid;
        lse2[tid] = (tg < L) ? p.lse[(size_t)bh * L + tg] * 1.44269504088896340736f : 0.f;
        dl[tid] = p.delta[(size_t)bh * Lp + tg];
    }
    __syncthreads();

    const int tb = wv >> 1, sb = wv & 1;
    const int trow = i * CHUNK + 32 * tb + l32;
    const TIO* dop = reinterpret_cast<const TIO*>(p.dO) + ((size_t)bh * L + (trow < L ? trow : L - 1)) * D + FE * h;

    for (int j = 0; j < i; ++j) {
        const T* xst = reinterpret_cast<const T*>(p.xs) + ((size_t)bh * npairs + pair_slot(i, j)) * CHUNK * D;
        const T* kn = reinterpret_cast<const T*>(p.knat) + ((size_t)bh * NC + j) * CHUNK * D;
        const T* ktn = reinterpret_cast<const T*>(p.ktnat) + ((size_t)bh * NC + j) * CHUNK * D;
        const T* dpn = reinterpret_cast<const T*>(p.dpnat) + ((size_t)bh * NC + j) * D * D;
        const TIO* vp = reinterpret_cast<const TIO*>(p.v) + ((size_t)bh * L + j * CHUNK + 32 * sb + l32) * D + FE * h;

        f32x16 S = gemm_rows<T, D>(xst + (size_t)(32 * tb + l32) * D + FE * h,
                                   kn + (size_t)(32 * sb + l32) * D + FE * h, zero16());
        f32x16 dP = gemm_rows<TIO, D>(dop, vp, zero16());
#pragma unroll
        for (int jj = 0; jj < 16; ++jj) {
            const int t = 32 * tb + acc_row(jj, h);
            const float P = (i * CHUNK + t < L) ? __builtin_amdgcn_exp2f(S[jj] * sl2 - lse2[t]) : 0.f;
            dST[t * LDC + 32 * sb + l32] = (T)(P * (dP[jj] - dl[t]) * p.scale);
        }
        __syncthreads();
#pragma unroll
        for (int o = 0; o < NOWN; ++o) {
            const int blk = wv + 4 * o, tb2 = blk / DB, cb = blk % DB;
            f32x16 a1 = gemm32<T, CHUNK>(dST, LDC, 32 * tb2, ktn, CHUNK, 32 * cb, l32, h, zero16());
            f32x16 a2 = gemm32<T, D>(gT, LDD, 32 * tb2, dpn, D, 32 * cb, l32, h, zero16());
#pragma unroll
            for (int jj = 0; jj < 16; ++jj) gm[o][jj] += a1[jj] - a2[jj];
        }
        __syncthreads();
        T* gst = reinterpret_cast<T*>(p.gs) + ((size_t)bh * npairs + pair_slot(i, j + 1 < i ? j + 1 : j)) * CHUNK * D;
        const bool store = j + 1 < i;
#pragma unroll
        for (int o = 0; o < NOWN; ++o) {
            const int blk = wv + 4 * o, tb2 = blk / DB, cb = blk % DB;
#pragma unroll
            for (int jj = 0; jj < 16; ++jj) {
                const int t = 32 * tb2 + acc_row(jj, h), c = 32 * cb + l32;
                const T v = (T)gm[o][jj];
                gT[t * LDD + c] = v;
                if (store) gst[(size_t)t * D + c] = v;
            }
        }
        __syncthreads();
    }
#pragma unroll
    for (int o = 0; o < NOWN; ++o) {
        const int blk = wv + 4 * o, tb2 = blk / DB, cb = blk % DB;
#pragma unroll
        for (int jj = 0; jj < 16; ++jj)
            p.dqb[((size_t)bh * Lp + i * CHUNK + 32 * tb2 + acc_row(jj, h)) * D + 32 * cb + l32] = gm[o][jj];
    }
}

// ---------------------------------------------------------------------------------------
template <typename TIO, int D> struct KeyCfg {
    typedef typename Compute<TIO>::type T;
    static constexpr int FE = Tr<T>::FE;
    static constexpr int LDC = CHUNK + FE;
    static constexpr size_t smem_bytes = (size_t)D * LDC * (2 * sizeof(T) + sizeof(TIO)) +
                                         (size_t)CHUNK * LDC * (sizeof(T) + sizeof(TIO)) + 2 * CHUNK * 4;
};

template <typename TIO, int D>
__global__ __launch_bounds__(256) void bwd_keyside_kernel(BwdParams p) {
    using C = KeyCfg<TIO, D>;
    using T = typename C::T;
    using Frag = typename Tr<T>::Frag;
    using FragIO = typename Tr<TIO>::Frag;
    constexpr int FE = C::FE, LDC = C::LDC;
    constexpr int DB = D / 32, NOWN = 2 * DB / 4, NDP = DB * DB / 4;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    T* Xt = reinterpret_cast<T*>(smem);                       // [c][t]
    T* Gt = Xt + D * LDC;                                     // [b][t]
    TIO* dOt = reinterpret_cast<TIO*>(Gt + D * LDC);          // [c][t]
    TIO* Pt = dOt + D * LDC;                                  // [s][t]
    T* dSt = reinterpret_cast<T*>(Pt + CHUNK * LDC);          // [s][t]
    float* lse2 = reinterpret_cast<float*>(dSt + CHUNK * LDC);
    float* dl = lse2 + CHUNK;

    const int j = blockIdx.x, bh = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, h = lane >> 5, l32 = lane & 31;
    const int L = p.L, NC = p.NC;
    const size_t Lp = (size_t)NC * CHUNK, npairs = (size_t)NC * (NC - 1) / 2;
    const float sl2 = p.scale * 1.44269504088896340736f;

    f32x16 dV[NOWN], dK[NOWN], dDP[NDP];
#pragma unroll
    for (int o = 0; o < NOWN; ++o) { dV[o] = zero16(); dK[o] = zero16(); }
#pragma unroll
    for (int o = 0; o < NDP; ++o) dDP[o] = zero16();

    const int tb = wv >> 1, sb = wv & 1;
    const T* kn = reinterpret_cast<const T*>(p.knat) + ((size_t)bh * NC + j) * CHUNK * D;
    // rows of V_j: chunk j < NC-1 is always complete when the loop below runs
    const TIO* vp = reinterpret_cast<const TIO*>(p.v) + ((size_t)bh * L + j * CHUNK + 32 * sb + l32) * D + FE * h;

    for (int i = j + 1; i < NC; ++i) {
        const T* xst = reinterpret_cast<const T*>(p.xs) + ((size_t)bh * npairs + pair_slot(i, j)) * CHUNK * D;
        const T* gst = reinterpret_cast<const T*>(p.gs) + ((size_t)bh * npairs + pair_slot(i, j)) * CHUNK * D;
        for (int idx = tid; idx < CHUNK * (D / FE); idx += 256) {
            const int row = idx / (D / FE), cf = idx % (D / FE);
            const int tg = i * CHUNK + row;
            const Frag xv = ld_frag<T>(xst + (size_t)row * D + cf * FE);
            Frag gv = Tr<T>::zero();
            if (j >= 1) gv = ld_frag<T>(gst + (size_t)row * D + cf * FE);
            FragIO ov = Tr<TIO>::zero();
            if (tg < L) ov = ld_frag<TIO>(reinterpret_cast<const TIO*>(p.dO) + ((size_t)bh * L + tg) * D + cf * FE);
#pragma unroll
            for (int e = 0; e < FE; ++e) {
                Xt[(cf * FE + e) * LDC + row] = xv[e];
                Gt[(cf * FE + e) * LDC + row] = gv[e];
                dOt[(cf * FE + e) * LDC + row] = ov[e];
            }
        }
        if (tid < CHUNK) {
            const int tg = i * CHUNK + tid;
            lse2[tid] = (tg < L) ? p.lse[(size_t)bh * L + tg] * 1.44269504088896340736f : 0.f;
            dl[tid] = p.delta[(size_t)bh * Lp + tg];
        }
        __syncthreads();

        const int trow = i * CHUNK + 32 * tb + l32;
        const TIO* dop = reinterpret_cast<const TIO*>(p.dO) + ((size_t)bh * L + (trow < L ? trow : L - 1)) * D + FE * h;
        f32x16 S = gemm_rows<T, D>(xst + (size_t)(32 * tb + l32) * D + FE * h,
                                   kn + (size_t)(32 * sb + l32) * D + FE * h, zero16());
        f32x16 dP = gemm_rows<TIO, D>(dop, vp, zero16());
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            typename Tr<TIO>::Vec4 p4;
            typename Tr<T>::Vec4 s4;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int t = 32 * tb + 8 * g + 4 * h + r;
                const float P = (i * CHUNK + t < L) ? __builtin_amdgcn_exp2f(S[4 * g + r] * sl2 - lse2[t]) : 0.f;
                p4[r] = (TIO)P;
                s4[r] = (T)(P * (dP[4 * g + r] - dl[t]) * p.scale);
            }
            *reinterpret_cast<typename Tr<TIO>::Vec4*>(Pt + (32 * sb + l32) * LDC + 32 * tb + 8 * g + 4 * h) = p4;
            *reinterpret_cast<typename Tr<T>::Vec4*>(dSt + (32 * sb + l32) * LDC + 32 * tb + 8 * g + 4 * h) = s4;
        }
        __syncthreads();
#pragma unroll
        for (int o = 0; o < NOWN; ++o) {
            const int blk = wv + 4 * o, sb2 = blk / DB, cb = blk % DB;
            dV[o] = gemm32<TIO, CHUNK>(Pt, LDC, 32 * sb2, dOt, LDC, 32 * cb, l32, h, dV[o]);
            dK[o] = gemm32<T, CHUNK>(dSt, LDC, 32 * sb2, Xt, LDC, 32 * cb, l32, h, dK[o]);
        }
        if (j >= 1) {
#pragma unroll
            for (int o = 0; o < NDP; ++o) {
                const int blk = wv + 4 * o, ab = blk / DB, bb = blk % DB;
                dDP[o] = gemm32<T, CHUNK>(Xt, LDC, 32 * ab, Gt, LDC, 32 * bb, l32, h, dDP[o]);
            }
        }
        __syncthreads();
    }
#pragma unroll
    for (int o = 0; o < NOWN; ++o) {
        const int blk = wv + 4 * o, sb2 = blk / DB, cb = blk % DB;
#pragma unroll
        for (int jj = 0; jj < 16; ++jj) {
            const size_t off = ((size_t)bh * Lp + j * CHUNK + 32 * sb2 + acc_row(jj, h)) * D + 32 * cb + l32;
            p.dvp[off] = dV[o][jj];
            p.dkb[off] = dK[o][jj];
        }
    }
#pragma unroll
    for (int o = 0; o < NDP; ++o) {
        const int blk = wv + 4 * o, ab = blk / DB, bb = blk % DB;
#pragma unroll
        for (int jj = 0; jj < 16; ++jj)
            p.ddp[(((size_t)bh * NC + j) * D + 32 * ab + acc_row(jj, h)) * D + 32 * bb + l32] = -dDP[o][jj];
    }
}

// ---------------------------------------------------------------------------------------
// Batched small product for the chunk-transform adjoint, one workgroup per (chunk, bh):
//   C[m][n] = mask( alpha * sum_k A[m][k] B[n][k] + Cin[m][n] )
// Operands are addressed with explicit strides (so either orientation of a stored
// matrix can be used), converted to the operand type while being staged in LDS.
template <typename TIO>
__device__ __forceinline__ float load_el(const MatRef& r, long long off) {
    typedef typename Compute<TIO>::type T;
    if (r.type == EL_F32) return reinterpret_cast<const float*>(r.p)[off];
    if (r.type == EL_OP) return (float)reinterpret_cast<const T*>(r.p)[off];
    return (float)reinterpret_cast<const TIO*>(r.p)[off];
}

template <typename TIO>
__device__ __forceinline__ void stage_mat(const MatRef& r, typename Compute<TIO>::type* dst, int ld, int R, int K,
                                          int bh, int chunk, int L, int tid) {
    typedef typename Compute<TIO>::type T;
    const long long base = bh * r.s_bh + chunk * r.s_ch;
    const int ntok = L - chunk * CHUNK;     // tokens of this chunk that exist
    for (int idx = tid; idx < R * K; idx += 256) {
        int m, k;
        if (r.ks == 1) { m = idx / K; k = idx % K; } else { k = idx / R; m = idx % R; }
        const bool ok = (r.tok == TOK_NONE) || ((r.tok == TOK_ROW ? m : k) < ntok);
        const float v = ok ? load_el<TIO>(r, base + (long long)m * r.rs + (long long)k * r.ks) : 0.f;
        dst[m * ld + k] = (T)v;
    }
}

template <typename TIO>
__global__ __launch_bounds__(256) void batched_gemm_kernel(GemmArgs a) {
    typedef typename Compute<TIO>::type T;
    constexpr int FE = Tr<T>::FE, KW = Tr<T>::KW;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int ld = a.K + FE;
    T* As = reinterpret_cast<T*>(smem);
    T* Bs = As + a.M * ld;
    const int chunk = blockIdx.x, bh = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, h = lane >> 5, l32 = lane & 31;
    stage_mat<TIO>(a.A, As, ld, a.M, a.K, bh, chunk, a.L, tid);
    stage_mat<TIO>(a.B, Bs, ld, a.N, a.K, bh, chunk, a.L, tid);
    __syncthreads();
    const int nb = a.N / 32, nblk = (a.M / 32) * nb;
    const long long cbase = bh * a.c_bh + chunk * a.c_ch;
    for (int blk = wv; blk < nblk; blk += 4) {
        const int mb = blk / nb, cb = blk % nb;
        const T* ap = As + (32 * mb + l32) * ld + FE * h;
        const T* bp = Bs + (32 * cb + l32) * ld + FE * h;
        f32x16 acc = zero16();
        for (int k0 = 0; k0 < a.K; k0 += KW) acc = Tr<T>::mma(ld_frag<T>(ap + k0), ld_frag<T>(bp + k0), acc);
#pragma unroll
        for (int jj = 0; jj < 16; ++jj) {
            const int m = 32 * mb + acc_row(jj, h), n = 32 * cb + l32;
            const long long off = cbase + (long long)m * a.crs + (long long)n * a.ccs;
            float v = a.alpha * acc[jj];
            if (a.Cin) v += a.Cin[off];
            if ((a.mask == MASK_TRIL && n > m) || (a.mask == MASK_SLOWER && n >= m)) v = 0.f;
            a.C[off] = v;
        }
    }
}

// ---------------------------------------------------------------------------------------
// Diagonal block: P = exp(scale*Sd - lse) on key <= query, dSd = scale * P (dPd - delta).
__global__ __launch_bounds__(256) void bwd_diag_kernel(DiagArgs a) {
    const int chunk = blockIdx.x, bh = blockIdx.y;
    const size_t base = ((size_t)bh * a.NC + chunk) * 4096;
    for (int idx = threadIdx.x; idx < 4096; idx += 256) {
        const int t = idx >> 6, s = idx & 63, tg = chunk * CHUNK + t;
        float P = 0.f, ds = 0.f;
        if (s <= t && tg < a.L) {
            P = __expf(a.scale * a.sdm[base + idx] - a.lse[(size_t)bh * a.L + tg]);
            ds = a.scale * P * (a.dpd[base + idx] - a.delta[(size_t)bh * a.NC * CHUNK + tg]);
        }
        a.pd[base + idx] = P;
        a.dsd[base + idx] = ds;
    }
}

// dbeta_a = R[a][a] + sum_s M[a][s] G[a][s];  dGs = diag(beta) M + (diag(beta) M)^T.
template <typename TIO>
__global__ __launch_bounds__(256) void bwd_beta_kernel(BetaArgs a) {
    __shared__ float bs[CHUNK];
    const int chunk = blockIdx.x, bh = blockIdx.y, tid = threadIdx.x;
    const size_t base = ((size_t)bh * a.NC + chunk) * 4096;
    if (tid < CHUNK) {
        const int tg = chunk * CHUNK + tid;
        bs[tid] = (tg < a.L) ? (float)reinterpret_cast<const TIO*>(a.beta)[(size_t)bh * a.L + tg] : 0.f;
    }
    __syncthreads();
    for (int idx = tid; idx < 4096; idx += 256) {
        const int r = idx >> 6, c = idx & 63;
        a.dgs[base + idx] = bs[r] * a.m[base + idx] + bs[c] * a.m[base + c * 64 + r];
    }
    if (tid < CHUNK) {
        float s = a.r[base + tid * 64 + tid];
        for (int c = 0; c < tid; ++c) s += a.m[base + tid * 64 + c] * a.g[base + tid * 64 + c];
        a.dbf[(size_t)bh * a.NC * CHUNK + chunk * CHUNK + tid] = s;
    }
}

// fp32 [BH][Lp][d] -> I/O type [BH][L][d]; dbeta likewise.
template <typename TIO>
__global__ __launch_bounds__(256) void bwd_store_kernel(OutArgs a) {
    const int chunk = blockIdx.x, bh = blockIdx.y, tid = threadIdx.x;
    const size_t Lp = (size_t)a.NC * CHUNK;
    for (int idx = tid; idx < CHUNK * a.d; idx += 256) {
        const int t = idx / a.d, c = idx % a.d, tg = chunk * CHUNK + t;
        if (tg >= a.L) continue;
        const size_t src = ((size_t)bh * Lp + tg) * a.d + c, dst = ((size_t)bh * a.L + tg) * a.d + c;
        reinterpret_cast<TIO*>(a.dq)[dst] = (TIO)a.dqf[src];
        reinterpret_cast<TIO*>(a.dk)[dst] = (TIO)a.dkf[src];
        reinterpret_cast<TIO*>(a.dv)[dst] = (TIO)a.dvf[src];
        reinterpret_cast<TIO*>(a.dw)[dst] = (TIO)a.dwf[src];
    }
    if (tid < CHUNK && chunk * CHUNK + tid < a.L)
        reinterpret_cast<TIO*>(a.dbeta)[(size_t)bh * a.L + chunk * CHUNK + tid] = (TIO)a.dbf[(size_t)bh * Lp + chunk * CHUNK + tid];
}

// ---------------------------------------------------------------------------------------
template <typename K> static hipError_t set_smem(K kernel, size_t bytes) {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

template <typename TIO, int D>
static hipError_t launch_scan_t(const BwdParams& p, hipStream_t st) {
    dim3 grid(p.NC, p.B * p.H);
    hipError_t e;
    hipLaunchKernelGGL((bwd_delta_kernel<TIO, D>), grid, dim3(256), 0, st, p);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    const size_t adj_bytes = AdjCfg<TIO, D>::smem_bytes, key_bytes = KeyCfg<TIO, D>::smem_bytes;
    if ((e = set_smem(&bwd_adjoint_kernel<TIO, D>, adj_bytes)) != hipSuccess) return e;
    hipLaunchKernelGGL((bwd_adjoint_kernel<TIO, D>), grid, dim3(256), adj_bytes, st, p);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if ((e = set_smem(&bwd_keyside_kernel<TIO, D>, key_bytes)) != hipSuccess) return e;
    hipLaunchKernelGGL((bwd_keyside_kernel<TIO, D>), grid, dim3(256), key_bytes, st, p);
    return hipGetLastError();
}

hipError_t launch_bwd_scan(const BwdParams& p, int d, int is_bf16, hipStream_t st) {
    if (is_bf16) return d == 64 ? launch_scan_t<bf16_t, 64>(p, st) : launch_scan_t<bf16_t, 128>(p, st);
    return d == 64 ? launch_scan_t<float, 64>(p, st) : launch_scan_t<float, 128>(p, st);
}

hipError_t launch_batched_gemm(const GemmArgs& a, int BH, int is_bf16, hipStream_t st) {
    const size_t es = is_bf16 ? 2 : 4, fe = is_bf16 ? 8 : 4;
    const size_t bytes = (size_t)(a.M + a.N) * (a.K + fe) * es;
    dim3 grid(a.NC, BH);
    hipError_t e;
    if (is_bf16) {
        if ((e = set_smem(&batched_gemm_kernel<bf16_t>, 160 * 1024)) != hipSuccess) return e;
        hipLaunchKernelGGL((batched_gemm_kernel<bf16_t>), grid, dim3(256), bytes, st, a);
    } else {
        if ((e = set_smem(&batched_gemm_kernel<float>, 160 * 1024)) != hipSuccess) return e;
        hipLaunchKernelGGL((batched_gemm_kernel<float>), grid, dim3(256), bytes, st, a);
    }
    return hipGetLastError();
}

hipError_t launch_bwd_diag(const DiagArgs& a, int BH, hipStream_t st) {
    hipLaunchKernelGGL(bwd_diag_kernel, dim3(a.NC, BH), dim3(256), 0, st, a);
    return hipGetLastError();
}

hipError_t launch_bwd_beta(const BetaArgs& a, int BH, int is_bf16, hipStream_t st) {
    if (is_bf16) hipLaunchKernelGGL((bwd_beta_kernel<bf16_t>), dim3(a.NC, BH), dim3(256), 0, st, a);
    else hipLaunchKernelGGL((bwd_beta_kernel<float>), dim3(a.NC, BH), dim3(256), 0, st, a);
    return hipGetLastError();
}

hipError_t launch_bwd_store(const OutArgs& a, int BH, int is_bf16, hipStream_t st) {
    if (is_bf16) hipLaunchKernelGGL((bwd_store_kernel<bf16_t>), dim3(a.NC, BH), dim3(256), 0, st, a);
    else hipLaunchKernelGGL((bwd_store_kernel<float>), dim3(a.NC, BH), dim3(256), 0, st, a);
    return hipGetLastError();
}

}  // namespace path
