// Adjoint of the chunk transform (the UT transform of Sec. 3.2 and the diagonal block of
// Sec. 3.3), fused: one workgroup per (chunk, head) for 2-byte operand types.  The paper gives
// no backward; with the chunk's matrices (rows = the 64 tokens of the chunk)
//
//   F   strictly-lower part of the boundary-adjusted query transform,  Y = solved W-side block,
//   N, Gk, A^-1 from the UT transform,  U = T^-1-transformed W (dP = W^T U),  Sd the raw diagonal logits,
//
// the gradients that arrive are dQb, dKb (boundary-adjusted queries / keys), ddP (chunk product),
// dV' (off-diagonal part of dV), and the steps are
//
//   dPd = dO V^T;  P = exp(scale Sd - lse) (key <= query);  dSd = scale P o (dPd - delta)
//   dV  = dV' + P^T dO
//   dF  = tril(-dSd Y^T - dQb U^T)            dY = -F^T dSd - W dKb^T
//   dU  = -F^T dQb + W ddP                     dN = dY Gk^T + dU W^T
//   dGk = sl(N^T dY)     R = A^-T dN     M = sl(-R N^T)     dGs = diag(beta) M + (diag(beta) M)^T
//   dbeta_a = R_aa + sum_s M_as G_as
//   dQ  = dQb + dSd K + dF W
//   dK  = dKb + dSd^T Q + dGk^T W
//   dW  = -Y dKb + U ddP^T + dF^T Q + dGk K + N^T dU + dGs W
//
// (sl = strictly lower part).  Every matrix is staged ONCE into LDS in the layout it has in
// memory (converted to the operand type); a product whose contraction runs along the rows of a
// stored matrix takes its 16-byte fragments with two transposing LDS reads instead of keeping a
// transposed copy.  dK and dW accumulate in registers across the whole kernel; the 64 x 64
// intermediates never leave LDS.  Per chunk the kernel reads about 0.46 MB and writes the four
// gradients, against about 1.5 MB for the same steps run as separate staged products.
#include "path_common.h"
#include "bwd_decl.h"

namespace path {
namespace {

constexpr int CA_NT = 512;       // threads per workgroup (8 waves)

template <typename TIO, int D> struct CaCfg {
    typedef typename Compute<TIO>::type T;
    static_assert(sizeof(T) == 2, "fused chunk adjoint: 2-byte operand types only");
    static constexpr int LDD = D + 8;          // pitch of a [..][D] tile (elements)
    static constexpr int LDC = CHUNK + 8;      // pitch of a [..][64] tile
    static constexpr int BIG = (64 * LDD > D * LDC ? 64 * LDD : D * LDC) * 2;   // bytes of a 64 x D or D x 64 tile
    static constexpr int SMALL = 64 * LDC * 2;
    static constexpr int LDM = 65;             // pitch of the fp32 copy of M
    // byte offsets: W | X0 X3 (adjacent: ddP spans both) | X1 | X2 | Y0..Y4 | misc
    static constexpr int XW = 0, X0 = BIG, X3 = 2 * BIG, X1 = 3 * BIG, X2 = 4 * BIG;
    static constexpr int Y0 = 5 * BIG, Y1 = Y0 + SMALL, Y2 = Y1 + SMALL, Y3 = Y2 + SMALL, Y4 = Y3 + SMALL;
    static constexpr int MISC = Y4 + SMALL;
    static constexpr int TOTAL = MISC + 2048;
    static_assert(D * LDD * 2 <= 2 * BIG, "ddP tile must fit X0+X3");
    static_assert(64 * LDM * 4 <= 2 * BIG, "fp32 M must fit X0+X3");
    static_assert(TOTAL <= 160 * 1024, "LDS budget");
};

// ROWS x COLS elements of type S from global memory (row-major, `stride` elements between rows), 8 per
// thread and step, held in registers between load() and store(); rows >= nvalid are zero.
template <typename S, int ROWS, int COLS> struct GTile {
    static constexpr int NV = ROWS * COLS / 8 / CA_NT;
    static_assert(NV >= 1 && NV * 8 * CA_NT == ROWS * COLS, "tile must be a multiple of the workgroup's reach");
    typedef S Vec8 __attribute__((ext_vector_type(8)));
    Vec8 v[NV];
    __device__ __forceinline__ void load(const S* src, int stride, int nvalid, int tid) {
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            const int idx = tid + u * CA_NT, r = idx / (COLS / 8), c = (idx % (COLS / 8)) * 8;
            if (r < nvalid) v[u] = *reinterpret_cast<const Vec8*>(src + r * stride + c);
            else
#pragma unroll
                for (int e = 0; e < 8; ++e) v[u][e] = (S)0.f;
        }
    }
    template <typename T, bool NEG> __device__ __forceinline__ void store(T* dst, int ld, int tid) const {
        typedef T TVec8 __attribute__((ext_vector_type(8)));
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            const int idx = tid + u * CA_NT, r = idx / (COLS / 8), c = (idx % (COLS / 8)) * 8;
            TVec8 o;
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = (T)(NEG ? -(float)v[u][e] : (float)v[u][e]);
            *reinterpret_cast<TVec8*>(dst + r * ld + c) = o;
        }
    }
};

// One 32x32 accumulator block -> LDS, stored [m][n] in the operand type.
template <typename T>
__device__ __forceinline__ void st_block(T* dst, int ld, int r0, int c0, const f32x16& acc, int l32, int h) {
#pragma unroll
    for (int jj = 0; jj < 16; ++jj) dst[(r0 + acc_row(jj, h)) * ld + c0 + l32] = (T)acc[jj];
}

template <typename TIO, int D, bool FOX, bool STRIDED>
__global__ __launch_bounds__(CA_NT) void chunk_fused_kernel(ChunkFusedArgs a) {
    using C = CaCfg<TIO, D>;
    typedef typename C::T T;
    constexpr int LDD = C::LDD, LDC = C::LDC, LDM = C::LDM;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    T* XW = reinterpret_cast<T*>(smem + C::XW);
    T* X0 = reinterpret_cast<T*>(smem + C::X0);
    T* X1 = reinterpret_cast<T*>(smem + C::X1);
    T* X2 = reinterpret_cast<T*>(smem + C::X2);
    T* X3 = reinterpret_cast<T*>(smem + C::X3);
    T* Y0 = reinterpret_cast<T*>(smem + C::Y0);
    T* Y1 = reinterpret_cast<T*>(smem + C::Y1);
    T* Y2 = reinterpret_cast<T*>(smem + C::Y2);
    T* Y3 = reinterpret_cast<T*>(smem + C::Y3);
    T* Y4 = reinterpret_cast<T*>(smem + C::Y4);
    float* Mf = reinterpret_cast<float*>(smem + C::X0);      // fp32 M, after ddP is dead
    float* misc = reinterpret_cast<float*>(smem + C::MISC);
    float *lse_s = misc, *delta_s = misc + 64, *beta_s = misc + 128, *rdiag = misc + 192, *colsum = misc + 256, *cum_s = misc + 384;

    const int chunk = blockIdx.x, bh = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, h = lane >> 5, l32 = lane & 31;
    const int L = seq_len(a.ul, bh, a.L), NC = a.NC;      // this head's own length; NC: chunks per head in the workspace arrays
    if (chunk * CHUNK >= L) return;                        // (packed batch: a shorter sequence has fewer chunks)
    const int ntok = (L - chunk * CHUNK < CHUNK) ? L - chunk * CHUNK : CHUNK;
    const size_t Lp = (size_t)NC * CHUNK;
    const long long ubase = user_vec(a.ul, bh, (long long)chunk * CHUNK);    // the caller's tensors: row of the chunk's first token
    const int TS = STRIDED ? (int)a.ul.vt : D;                                // ... and their token stride (a compile-time
                                                                              // constant unless the layout interleaves heads)
    const size_t pbase = ((size_t)bh * Lp + (size_t)chunk * CHUNK) * D;      // padded [Lp][d] workspace tensors
    const size_t cbase = ((size_t)bh * NC + chunk) * 4096;                   // 64 x 64 per chunk
    const size_t tpad = (size_t)bh * Lp + (size_t)chunk * CHUNK;             // per-token, padded
    const TIO* qg = reinterpret_cast<const TIO*>(a.q) + ubase;
    const TIO* kg = reinterpret_cast<const TIO*>(a.k) + ubase;
    const TIO* vg = reinterpret_cast<const TIO*>(a.v) + ubase;
    const TIO* wg = reinterpret_cast<const TIO*>(a.w) + ubase;
    const TIO* dog = reinterpret_cast<const TIO*>(a.d_o) + ubase;
    const T* utmg = reinterpret_cast<const T*>(a.utm) + ((size_t)bh * NC + chunk) * D * CHUNK;
    const float* ddpg = a.ddp + ((size_t)bh * NC + chunk) * D * D;

    // wave -> 32x32 block of a 64 x D result (all 8 waves for D = 128) and of a 64 x 64 result (waves 0..3)
    constexpr int NBD = D / 32;
    const bool actD = wv < 2 * NBD, act6 = wv < 4;
    const int mbD = wv / NBD, cbD = wv % NBD, mb6 = (wv >> 1) & 1, cb6 = wv & 1;

    auto cin = [&](const float* g, f32x16& acc) {       // accumulator block (mbD, cbD) from a padded fp32 [64][D] tensor
#pragma unroll
        for (int jj = 0; jj < 16; ++jj) acc[jj] = g[(size_t)(32 * mbD + acc_row(jj, h)) * D + 32 * cbD + l32];
    };
    auto out_user = [&](void* base, const f32x16& acc) {   // ... to a user gradient, rows of existing tokens only
        TIO* g = reinterpret_cast<TIO*>(base) + ubase;
#pragma unroll
        for (int jj = 0; jj < 16; ++jj) {
            const int t = 32 * mbD + acc_row(jj, h);
            if (t < ntok) g[t * TS + 32 * cbD + l32] = (TIO)acc[jj];
        }
    };

    // ---- stage W, dO, V; per-token scalars ---------------------------------------------------
    GTile<TIO, 64, D> tW, tdO, tV;
    tW.load(wg, TS, ntok, tid);
    tdO.load(dog, TS, ntok, tid);
    tV.load(vg, TS, ntok, tid);
    if (tid < CHUNK) {
        const bool ok = tid < ntok;
        lse_s[tid] = ok ? a.lse[user_scl(a.ul, bh, chunk * CHUNK + tid)] : 0.f;
        delta_s[tid] = a.delta[tpad + tid];
        beta_s[tid] = ok ? (float)reinterpret_cast<const TIO*>(a.beta)[user_scl(a.ul, bh, chunk * CHUNK + tid)] : 0.f;
        if (FOX) { cum_s[tid] = a.cum[tpad + tid]; colsum[tid] = 0.f; colsum[CHUNK + tid] = 0.f; }
    }
    float sd[16];                                   // raw diagonal logits of this wave's block
    if (act6) {
#pragma unroll
        for (int jj = 0; jj < 16; ++jj) sd[jj] = a.sdm[cbase + (size_t)(32 * mb6 + acc_row(jj, h)) * 64 + 32 * cb6 + l32];
    }
    tW.template store<T, false>(XW, LDD, tid);
    tdO.template store<T, false>(X0, LDD, tid);
    tV.template store<T, false>(X1, LDD, tid);
    f32x16 accV, accK, accQ, accW = zero16();
    if (actD) cin(a.dvp + pbase, accV);
    GTile<TIO, 64, D> tQ;
    tQ.load(qg, TS, ntok, tid);
    GTile<T, 64, 64> tY;
    tY.load(reinterpret_cast<const T*>(a.ytm) + cbase, 64, 64, tid);
    GTile<float, 64, D> tdQb;
    tdQb.load(a.dqb + pbase, D, 64, tid);
    GTile<T, D, 64> tU;
    tU.load(utmg, 64, D, tid);
    __syncthreads();

    // ---- dPd = dO V^T; P, dSd (diagonal block) -> Y0 = P, Y1 = dSd, both [query][key] ----------
    if (act6) {
        f32x16 acc = zero16();
        mm<T, D, false, false>(acc, X0, LDD, 32 * mb6, X1, LDD, 32 * cb6, l32, h);
        const int s = 32 * cb6 + l32;
        float csum = 0.f;
#pragma unroll
        for (int jj = 0; jj < 16; ++jj) {
            const int t = 32 * mb6 + acc_row(jj, h);
            float P = 0.f, ds = 0.f;
            if (s <= t && t < ntok) {
                float z = a.scale * sd[jj] - lse_s[t];
                if (FOX) z += (cum_s[t] - cum_s[s]) * 0.69314718055994530942f;     // gate sums are kept in base-2 units
                P = __expf(z);
                const float dz = P * (acc[jj] - delta_s[t]);
                ds = a.scale * dz;
                if (FOX) { csum += dz; atomicAdd(colsum + CHUNK + t, dz); }
            }
            Y0[t * LDC + s] = (T)P;
            Y1[t * LDC + s] = (T)ds;
        }
        if (FOX) atomicAdd(colsum + s, csum);
    }
    GTile<float, 64, D> tdKb;
    tdKb.load(a.dkb + pbase, D, 64, tid);
    __syncthreads();
    if (FOX && tid < CHUNK) {        // the diagonal block's column and row sums of the logit gradient
        a.dcol[tpad + tid] += colsum[tid];
        a.drow[tpad + tid] += colsum[CHUNK + tid];
    }

    // ---- dV = dV' + P^T dO ---------------------------------------------------------------------
    if (actD) {
        mm<T, 64, true, true>(accV, Y0, LDC, 32 * mbD, X0, LDD, 32 * cbD, l32, h);
        out_user(a.dv, accV);
        cin(a.dkb + pbase, accK);
    }
    __syncthreads();                 // dO (X0), V (X1), P (Y0) are free
    tQ.template store<T, false>(X0, LDD, tid);
    tY.template store<T, true>(Y0, LDC, tid);          // -Y^T as stored ([r][s])
    tdQb.template store<T, true>(X1, LDD, tid);        // -dQb
    tU.template store<T, false>(X2, LDC, tid);         // U as stored: [feature][token]
    if (actD) cin(a.dqb + pbase, accQ);
    GTile<TIO, 64, D> tK;
    tK.load(kg, TS, ntok, tid);
    GTile<T, 64, 64> tF;
    tF.load(reinterpret_cast<const T*>(a.fm) + cbase, 64, 64, tid);
    __syncthreads();

    // ---- dK = dKb + dSd^T Q (kept open);  dF = tril(-dSd Y^T - dQb U^T) -> Y2 --------------------
    if (actD) mm<T, 64, true, true>(accK, Y1, LDC, 32 * mbD, X0, LDD, 32 * cbD, l32, h);
    if (act6) {
        f32x16 acc = zero16();
        mm<T, 64, false, true>(acc, Y1, LDC, 32 * mb6, Y0, LDC, 32 * cb6, l32, h);
        mm<T, D, false, true>(acc, X1, LDD, 32 * mb6, X2, LDC, 32 * cb6, l32, h);
#pragma unroll
        for (int jj = 0; jj < 16; ++jj)
            if (32 * cb6 + l32 > 32 * mb6 + acc_row(jj, h)) acc[jj] = 0.f;
        st_block<T>(Y2, LDC, 32 * mb6, 32 * cb6, acc, l32, h);
    }
    tdKb.template store<T, false>(X3, LDD, tid);
    GTile<float, D, D> tDD;
    tDD.load(ddpg, D, D, tid);
    __syncthreads();

    // ---- dW = dF^T Q - Y dKb (kept open) ----------------------------------------------------------
    if (actD) {
        mm<T, 64, true, true>(accW, Y2, LDC, 32 * mbD, X0, LDD, 32 * cbD, l32, h);
        mm<T, 64, true, true>(accW, Y0, LDC, 32 * mbD, X3, LDD, 32 * cbD, l32, h);
    }
    __syncthreads();                 // Q (X0) and Y (Y0) are free
    tK.template store<T, false>(X0, LDD, tid);
    tF.template store<T, false>(Y3, LDC, tid);
    GTile<T, 64, 64> tN, tG;
    tN.load(reinterpret_cast<const T*>(a.nm) + cbase, 64, 64, tid);
    tG.load(reinterpret_cast<const T*>(a.gktm) + cbase, 64, 64, tid);
    __syncthreads();

    // ---- dQ = dQb + dSd K + dF W;  dY = -(F^T dSd + W dKb^T) -> Y4 ---------------------------------
    if (actD) {
        mm<T, 64, false, true>(accQ, Y1, LDC, 32 * mbD, X0, LDD, 32 * cbD, l32, h);
        mm<T, 64, false, true>(accQ, Y2, LDC, 32 * mbD, XW, LDD, 32 * cbD, l32, h);
        out_user(a.dq, accQ);
    }
    if (act6) {
        f32x16 acc = zero16();
        mm<T, 64, true, true>(acc, Y3, LDC, 32 * mb6, Y1, LDC, 32 * cb6, l32, h);
        mm<T, D, false, false>(acc, XW, LDD, 32 * mb6, X3, LDD, 32 * cb6, l32, h);
#pragma unroll
        for (int jj = 0; jj < 16; ++jj) acc[jj] = -acc[jj];
        st_block<T>(Y4, LDC, 32 * mb6, 32 * cb6, acc, l32, h);
    }
    GTile<T, 64, 64> tA;
    tA.load(reinterpret_cast<const T*>(a.aim) + cbase, 64, 64, tid);
    tK.load(kg, TS, ntok, tid);       // K once more, for dGk K at the end
    __syncthreads();                 // K (X0), dKb (X3), dSd (Y1), dF (Y2) are free
    tDD.template store<T, false>(X0, LDD, tid);        // ddP [a][b], spans X0 and X3
    tN.template store<T, false>(Y0, LDC, tid);
    tG.template store<T, false>(Y1, LDC, tid);
    __syncthreads();

    // ---- dU = -F^T dQb + W ddP;  dW += U ddP^T ---------------------------------------------------
    f32x16 accU = zero16();
    if (actD) {
        mm<T, 64, true, true>(accU, Y3, LDC, 32 * mbD, X1, LDD, 32 * cbD, l32, h);
        mm<T, D, false, true>(accU, XW, LDD, 32 * mbD, X0, LDD, 32 * cbD, l32, h);
        mm<T, D, true, false>(accW, X2, LDC, 32 * mbD, X0, LDD, 32 * cbD, l32, h);
    }
    __syncthreads();                 // every wave is done with dQb (X1), U (X2)
    if (actD) st_block<T>(X1, LDD, 32 * mbD, 32 * cbD, accU, l32, h);       // dU [token][feature]
    tK.template store<T, false>(X2, LDD, tid);
    __syncthreads();

    // ---- dW += N^T dU;  dN = dY Gk^T + dU W^T -> Y3 ------------------------------------------------
    if (actD) mm<T, 64, true, true>(accW, Y0, LDC, 32 * mbD, X1, LDD, 32 * cbD, l32, h);
    if (act6) {
        f32x16 acc = zero16();
        mm<T, 64, false, true>(acc, Y4, LDC, 32 * mb6, Y1, LDC, 32 * cb6, l32, h);
        mm<T, D, false, false>(acc, X1, LDD, 32 * mb6, XW, LDD, 32 * cb6, l32, h);
        st_block<T>(Y3, LDC, 32 * mb6, 32 * cb6, acc, l32, h);
    }
    float gv[8];                     // G of the rows this wave reduces for dbeta (row wv + 8 i, column lane)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int r = wv + 8 * i;
        gv[i] = (lane < r) ? a.gm[cbase + (size_t)r * 64 + lane] : 0.f;
    }
    __syncthreads();                 // dN visible; Gk (Y1) is free

    // ---- dGk = sl(N^T dY) -> Y1 ----------------------------------------------------------------------
    if (act6) {
        f32x16 acc = zero16();
        mm<T, 64, true, true>(acc, Y0, LDC, 32 * mb6, Y4, LDC, 32 * cb6, l32, h);
#pragma unroll
        for (int jj = 0; jj < 16; ++jj)
            if (32 * cb6 + l32 >= 32 * mb6 + acc_row(jj, h)) acc[jj] = 0.f;
        st_block<T>(Y1, LDC, 32 * mb6, 32 * cb6, acc, l32, h);
    }
    __syncthreads();                 // dY (Y4) is free
    tA.template store<T, false>(Y4, LDC, tid);
    __syncthreads();

    // ---- R = A^-T dN -> Y2 (operand) and its diagonal (fp32) ----------------------------------------
    if (act6) {
        f32x16 acc = zero16();
        mm<T, 64, true, true>(acc, Y4, LDC, 32 * mb6, Y3, LDC, 32 * cb6, l32, h);
        st_block<T>(Y2, LDC, 32 * mb6, 32 * cb6, acc, l32, h);
        if (mb6 == cb6) {
#pragma unroll
            for (int jj = 0; jj < 16; ++jj)
                if (acc_row(jj, h) == l32) rdiag[32 * mb6 + l32] = acc[jj];
        }
    }
    __syncthreads();

    // ---- M = sl(-R N^T) -> fp32 in LDS ---------------------------------------------------------------
    if (act6) {
        f32x16 acc = zero16();
        mm<T, 64, false, false>(acc, Y2, LDC, 32 * mb6, Y0, LDC, 32 * cb6, l32, h);
#pragma unroll
        for (int jj = 0; jj < 16; ++jj) {
            const int m = 32 * mb6 + acc_row(jj, h), n = 32 * cb6 + l32;
            Mf[m * LDM + n] = (n >= m) ? 0.f : -acc[jj];
        }
    }
    __syncthreads();

    // ---- dGs = diag(beta) M + (diag(beta) M)^T -> Y3;  dbeta ------------------------------------------
    for (int idx = tid; idx < 4096; idx += CA_NT) {
        const int r = idx >> 6, c = idx & 63;
        Y3[r * LDC + c] = (T)(beta_s[r] * Mf[r * LDM + c] + beta_s[c] * Mf[c * LDM + r]);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int r = wv + 8 * i;
        float s = Mf[r * LDM + lane] * gv[i];           // M is zero on and above the diagonal, gv outside lane < r
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off);
        if (lane == 0 && r < ntok)
            reinterpret_cast<TIO*>(a.dbeta)[user_scl(a.ul, bh, chunk * CHUNK + r)] = (TIO)(s + rdiag[r]);
    }
    __syncthreads();

    // ---- dK += dGk^T W;  dW += dGs W + dGk K ------------------------------------------------------------
    if (actD) {
        mm<T, 64, true, true>(accK, Y1, LDC, 32 * mbD, XW, LDD, 32 * cbD, l32, h);
        out_user(a.dk, accK);
        mm<T, 64, false, true>(accW, Y3, LDC, 32 * mbD, XW, LDD, 32 * cbD, l32, h);
        mm<T, 64, false, true>(accW, Y1, LDC, 32 * mbD, X2, LDD, 32 * cbD, l32, h);
        out_user(a.dw, accW);
    }
}

template <typename TIO, int D, bool FOX, bool STRIDED>
hipError_t launch_s(const ChunkFusedArgs& a, int BH, hipStream_t st) {
    using C = CaCfg<TIO, D>;
    // set once per process; a function-local static is initialised under the language's own lock
    static const hipError_t attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&chunk_fused_kernel<TIO, D, FOX, STRIDED>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::TOTAL);
    if (attr_err != hipSuccess) return attr_err;
    hipLaunchKernelGGL((chunk_fused_kernel<TIO, D, FOX, STRIDED>), dim3(a.NC, BH), dim3(CA_NT), (size_t)C::TOTAL, st, a);
    return hipGetLastError();
}
template <typename TIO, int D, bool FOX>
hipError_t launch_t(const ChunkFusedArgs& a, int BH, hipStream_t st) {
    return a.ul.vt != D ? launch_s<TIO, D, FOX, true>(a, BH, st) : launch_s<TIO, D, FOX, false>(a, BH, st);
}


// ---------------------------------------------------------------------------------------
// Adjoint of the second blocking level (Kb2_c = Kb_c R_c^T, R_{c-1} = R_c P_c with R_last = I,
// P_superblock = R_{first-1}; P_c = I - dP_c, dP_c = W_c^T U_c), fused: one workgroup per
// (super-block J, head) walks the chunks c = first .. last with the gradient G of R_{c-1} in
// accumulator registers (start: the gradient of P_superblock from the far ddP kernel),
//     ddP_c -= R_c^T G                              (d x d x d)
//     dKb_c += dKb2_c R_c                           (64 x d x d)
//     G     <- G - (G U_c^T) W_c + dKb2_c^T Kb_c     (c < last)
// The five operands of a chunk are fetched into registers one chunk ahead and staged in LDS as
// they lie in memory (16-byte writes, no bank conflicts); products that contract along the rows
// of a stored matrix take their fragments with transposing LDS reads.
template <typename TIO, int D> struct SbCfg {
    typedef typename Compute<TIO>::type T;
    static constexpr int LDD = D + 8, LDC = CHUNK + 8;
    static constexpr int DD = D * LDD * 2, TD = 64 * LDD * 2, DT = D * LDC * 2;     // bytes: d x d, 64 x d, d x 64 tiles
    static constexpr int R_ = 0, G_ = DD, K2 = 2 * DD, U_ = K2 + TD, W_ = U_ + DT, KB = W_ + TD, T1 = KB + TD;
    static constexpr int TOTAL = T1 + DT;
    static_assert(TOTAL <= 160 * 1024, "LDS budget");
};

template <typename TIO, int D, bool STRIDED>
__global__ __launch_bounds__(CA_NT) void sb_chain_kernel(SbChainArgs a) {
    using C = SbCfg<TIO, D>;
    typedef typename C::T T;
    constexpr int LDD = C::LDD, LDC = C::LDC, DB = D / 32;
    constexpr int NOWN = (DB * DB + 7) / 8;          // d x d blocks per wave: blocks wv, wv + 8, ...
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    T* sR = reinterpret_cast<T*>(smem + C::R_);       // R_c [k][x]
    T* sG = reinterpret_cast<T*>(smem + C::G_);       // G [a][b]
    T* sK2 = reinterpret_cast<T*>(smem + C::K2);      // dKb2_c [s][a]
    T* sU = reinterpret_cast<T*>(smem + C::U_);       // U_c as stored: [feature][token]
    T* sW = reinterpret_cast<T*>(smem + C::W_);       // W_c [t][b]
    T* sKb = reinterpret_cast<T*>(smem + C::KB);      // Kb_c [s][b]
    T* sT1 = reinterpret_cast<T*>(smem + C::T1);      // -(G U^T) [a][t]

    const int J = blockIdx.x, bh = blockIdx.y, NC = a.NC;           // NC: chunks per head in the workspace arrays
    const int L = seq_len(a.ul, bh, a.L), NCo = (L + CHUNK - 1) / CHUNK;   // this head's own length and chunks
    const int tid = threadIdx.x, lane = tid & 63, wv = __builtin_amdgcn_readfirstlane(tid >> 6), h = lane >> 5, l32 = lane & 31;
    const int c0 = J * SBC;
    if (c0 >= NCo) return;                            // (packed batch: a shorter sequence has fewer super-blocks)
    const int clast = (c0 + SBC - 1 < NCo) ? c0 + SBC - 1 : NCo - 1;
    const int TS = STRIDED ? (int)a.ul.vt : D;        // token stride of W
    const bool act = wv < 2 * DB;                     // 64 x d and d x 64 results: one block per wave
    const int hb = act ? wv / DB : 0, db = wv % DB;   // ... block (hb, db) of a 64 x d result, (db, hb) of a d x 64 one

    f32x16 G[NOWN];
    {
        const float* src = a.dchain + ((size_t)bh * (NC + 1) + c0) * D * D;
#pragma unroll
        for (int o = 0; o < NOWN; ++o) {
            const int blk = wv + 8 * o, ab = blk / DB, bb = blk % DB;
            if (blk < DB * DB) {
#pragma unroll
                for (int jj = 0; jj < 16; ++jj) G[o][jj] = src[(size_t)(32 * ab + acc_row(jj, h)) * D + 32 * bb + l32];
            }
        }
    }
    GTile<T, D, D> tR;
    GTile<float, 64, D> tK2;
    GTile<T, D, 64> tU;
    GTile<TIO, 64, D> tW;
    GTile<T, 64, D> tKb;
    auto fetch = [&](int c) {
        const size_t bhc = (size_t)bh * NC + c;
        const int ntok = (L - c * CHUNK < CHUNK) ? L - c * CHUNK : CHUNK;
        tR.load(reinterpret_cast<const T*>(a.rm) + bhc * D * D, D, D, tid);
        tK2.load(a.dk2 + bhc * CHUNK * D, D, 64, tid);
        if (c < clast) {
            tU.load(reinterpret_cast<const T*>(a.utm) + bhc * D * CHUNK, 64, D, tid);
            tW.load(reinterpret_cast<const TIO*>(a.w) + user_vec(a.ul, bh, (long long)c * CHUNK), TS, ntok, tid);
            tKb.load(reinterpret_cast<const T*>(a.kbm) + bhc * CHUNK * D, D, 64, tid);
        }
    };
    fetch(c0);
    for (int c = c0; c <= clast; ++c) {
        const size_t bhc = (size_t)bh * NC + c;
        __syncthreads();                              // the previous chunk's reads are done
        tR.template store<T, false>(sR, LDD, tid);
        tK2.template store<T, false>(sK2, LDD, tid);
        if (c < clast) {
            tU.template store<T, false>(sU, LDC, tid);
            tW.template store<T, false>(sW, LDD, tid);
            tKb.template store<T, false>(sKb, LDD, tid);
        }
#pragma unroll
        for (int o = 0; o < NOWN; ++o) {
            const int blk = wv + 8 * o, ab = blk / DB, bb = blk % DB;
            if (blk < DB * DB) st_block<T>(sG, LDD, 32 * ab, 32 * bb, G[o], l32, h);
        }
        if (c < clast) fetch(c + 1);
        // The two results of this step are added to what the key-side kernels left in ddP_c and dKb_c: every
        // element has exactly one writer here, so a plain read-modify-write does (hardware atomic adds, tried
        // first because they need no old value, ran at the L2's atomic rate and doubled the kernel's time).
        // The old values are requested well before they are used: those of the wave's first ddP block and of
        // its dKb block now, those of its second ddP block after the first is stored -- that block's product
        // is taken last, after the update of G (R and this step's G stay in LDS until the next step).
        static_assert(NOWN <= 2, "two d x d blocks per wave at most");
        float* const ddp_dst = a.ddp + bhc * (size_t)D * D;
        float* const dkb_dst = a.dkb + (bhc * CHUNK) * (size_t)D;
        auto ddp_load = [&](int o, f32x16& old) {
            const int blk = wv + 8 * o, xb = blk / DB, bb = blk % DB;
            if (blk < DB * DB) {
#pragma unroll
                for (int jj = 0; jj < 16; ++jj) old[jj] = ddp_dst[(size_t)(32 * xb + acc_row(jj, h)) * D + 32 * bb + l32];
            }
        };
        // ddP_c[x][b] -= sum_k R[k][x] G[k][b]
        auto ddp_block = [&](int o, const f32x16& old) {
            const int blk = wv + 8 * o, xb = blk / DB, bb = blk % DB;
            if (blk < DB * DB) {
                f32x16 acc = zero16();
                mm<T, D, true, true>(acc, sR, LDD, 32 * xb, sG, LDD, 32 * bb, l32, h);
#pragma unroll
                for (int jj = 0; jj < 16; ++jj) ddp_dst[(size_t)(32 * xb + acc_row(jj, h)) * D + 32 * bb + l32] = old[jj] - acc[jj];
            }
        };
        f32x16 ddp_old, dkb_old;
        ddp_load(0, ddp_old);
        if (act) {
#pragma unroll
            for (int jj = 0; jj < 16; ++jj) dkb_old[jj] = dkb_dst[(size_t)(32 * hb + acc_row(jj, h)) * D + 32 * db + l32];
        }
        __syncthreads();
        ddp_block(0, ddp_old);
        if (NOWN > 1) ddp_load(1, ddp_old);
        // dKb_c[s][b] += sum_a dKb2[s][a] R[a][b]
        if (act) {
            f32x16 acc = zero16();
            mm<T, D, false, true>(acc, sK2, LDD, 32 * hb, sR, LDD, 32 * db, l32, h);
#pragma unroll
            for (int jj = 0; jj < 16; ++jj) dkb_dst[(size_t)(32 * hb + acc_row(jj, h)) * D + 32 * db + l32] = dkb_old[jj] + acc[jj];
        }
        if (c == clast) {
            if (NOWN > 1) ddp_block(1, ddp_old);
            break;
        }
        // T1[a][t] = sum_k G[a][k] U[t][k]
        if (act) {
            f32x16 acc = zero16();
            mm<T, D, false, true>(acc, sG, LDD, 32 * db, sU, LDC, 32 * hb, l32, h);
#pragma unroll
            for (int jj = 0; jj < 16; ++jj) acc[jj] = -acc[jj];
            st_block<T>(sT1, LDC, 32 * db, 32 * hb, acc, l32, h);
        }
        __syncthreads();
        // G += -T1 W + dKb2^T Kb
#pragma unroll
        for (int o = 0; o < NOWN; ++o) {
            const int blk = wv + 8 * o, ab = blk / DB, bb = blk % DB;
            if (blk < DB * DB) {
                mm<T, 64, false, true>(G[o], sT1, LDC, 32 * ab, sW, LDD, 32 * bb, l32, h);
                mm<T, 64, true, true>(G[o], sK2, LDD, 32 * ab, sKb, LDD, 32 * bb, l32, h);
            }
        }
        if (NOWN > 1) ddp_block(1, ddp_old);
    }
}

template <typename TIO, int D, bool STRIDED>
hipError_t launch_sb_s(const SbChainArgs& a, int BH, hipStream_t st) {
    using C = SbCfg<TIO, D>;
    // set once per process; a function-local static is initialised under the language's own lock
    static const hipError_t attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&sb_chain_kernel<TIO, D, STRIDED>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::TOTAL);
    if (attr_err != hipSuccess) return attr_err;
    hipLaunchKernelGGL((sb_chain_kernel<TIO, D, STRIDED>), dim3((a.NC + SBC - 1) / SBC, BH), dim3(CA_NT), (size_t)C::TOTAL, st, a);
    return hipGetLastError();
}
template <typename TIO, int D>
hipError_t launch_sb_t(const SbChainArgs& a, int BH, hipStream_t st) {
    return a.ul.vt != D ? launch_sb_s<TIO, D, true>(a, BH, st) : launch_sb_s<TIO, D, false>(a, BH, st);
}

}  // namespace

hipError_t launch_bwd_sb_chain(const SbChainArgs& a, int BH, int d, hipStream_t st) {
    return d == 64 ? launch_sb_t<bf16_t, 64>(a, BH, st) : launch_sb_t<bf16_t, 128>(a, BH, st);
}

hipError_t launch_chunk_fused(const ChunkFusedArgs& a, int BH, int d, hipStream_t st) {
    const bool fox = a.cum != nullptr;
    if (d == 64) return fox ? launch_t<bf16_t, 64, true>(a, BH, st) : launch_t<bf16_t, 64, false>(a, BH, st);
    return fox ? launch_t<bf16_t, 128, true>(a, BH, st) : launch_t<bf16_t, 128, false>(a, BH, st);
}

}  // namespace path
