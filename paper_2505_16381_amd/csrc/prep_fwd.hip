// Chunk preprocessing of PaTH attention (paper Sec. 3.2: UT transform of a
// chunk, boundary-adjusted queries and keys, chunk transition product).
//
// One workgroup (4 waves) per (batch*head, chunk of 64 tokens).  With
// Q, K, W the chunk's rows and beta its transition strengths:
//
//   G   = W W^T                       A = I + strictLower(diag(beta) G)
//   N   = A^{-1} diag(beta)           (the chunk's "T^{-1}", Sec. 3 UT paragraph)
//   U   = N W                         dP = W^T U   (chunk product P = I - dP)
//   F   = tril(Q W^T)                 Y  = N strictLower(W K^T)
//   Qb  = Q - F U                     Kb = K - Y^T W            (Sec. 3.2 matrix forms)
//   Sd  = Q K^T - F Y                 (diagonal block logits, Sec. 3.2 case i = j)
//
// The triangular system is solved by forward substitution in fp32 (never
// through 1/beta, so beta = 0 is regular); everything else is MFMA.
// Outputs go to the workspace in the layouts the sweep kernel consumes
// without any shuffling: K-tile, V^T-tile and -dP-tile in fragment order,
// Qb and Sd in accumulator order (fp32).  Rows past L are treated as
// beta = 0, w = k = q = v = 0.
#include "path_common.h"

namespace path {

// TIO: storage type of the inputs; T = Compute<TIO>::type: operand type of the transform.
template <typename TIO, int D> struct PrepCfg {
    typedef typename Compute<TIO>::type T;
    static constexpr int FE = Tr<T>::FE;
    static constexpr int KW = Tr<T>::KW;
    static constexpr int LDD = D + FE;                 // padded length-D rows
    static constexpr int LDC = CHUNK + FE;             // padded length-64 rows
    static constexpr int LDA = CHUNK + 4;              // fp32 solve matrix
    static constexpr int LDH = 32 + 4;                 // fp32 32x32 helpers of the blocked inverse
    // Q and K are not staged: their operand fragments come straight from global memory (the chunk's rows are
    // read a few times, out of L2), converted to the operand type on the way.
    //
    // 2-byte operands use a compact map (81 KB: TWO workgroups per CU, so that the barriers and the
    // half-empty phases of one overlap the work of the other -- the kernel is a chain of short dependent
    // phases, not a stream): U^T has the space a transposed copy of W would take; where it is large enough
    // (d = 128) the fp32 inverse A^{-1} lives there before U^T is written; F, needed only by the output phase,
    // is computed there and takes the place of the fp32 matrix A, which is dead by then.
    // fp32 operands keep separate blocks (N overwrites A^{-1} in place; one workgroup per CU).
    static constexpr bool COMPACT = sizeof(T) == 2;
    static constexpr int WSUT = COMPACT ? CHUNK * LDD : ((CHUNK * LDD > D * LDC) ? CHUNK * LDD : D * LDC);   // fp32: U^T re-uses W's rows
    // element offsets (in T) -- every block is a multiple of 16 bytes
    static constexpr size_t off_ws = 0;                               // W rows (fp32: later U^T)
    static constexpr size_t off_wt = off_ws + WSUT;                   // fp32: W^T; 2-byte: U^T
    static constexpr size_t off_f_sep = off_wt + (size_t)D * LDC;     // F (fp32 map)
    static constexpr size_t off_gk = COMPACT ? off_wt + (size_t)D * LDC : off_f_sep + (size_t)CHUNK * LDC;     // (strictLower(W K^T))^T
    static constexpr size_t off_yt = off_gk + (size_t)CHUNK * LDC;    // Y^T
    static constexpr size_t off_nt = off_yt + (size_t)CHUNK * LDC;    // N (operand precision)
    static constexpr bool NT_IN_XF = sizeof(T) == 4;                  // fp32: N overwrites A^{-1} in place (same shape)
    static constexpr size_t t_elems = off_nt + (NT_IN_XF ? 0 : (size_t)CHUNK * LDC);
    static constexpr size_t off_af_bytes = ((t_elems * sizeof(T) + 15) / 16) * 16;   // fp32 A / solve
    static constexpr size_t off_f = COMPACT ? off_af_bytes / sizeof(T) : off_f_sep;  // F (2-byte: in A's place, from phase 4 on)
    static constexpr size_t off_beta_bytes = off_af_bytes + (size_t)CHUNK * LDA * 4;
    static constexpr bool XF_IN_UT = COMPACT && (size_t)D * LDC * sizeof(T) >= (size_t)CHUNK * LDA * 4;
    static constexpr size_t off_xf_bytes = XF_IN_UT ? off_wt * sizeof(T) : off_beta_bytes + CHUNK * 4;   // A^{-1}, fp32 [64][LDA]
    // the two 32x32 fp32 helpers live in Y^T's space (Y^T is written only after the inverse is done)
    static constexpr size_t off_xt1_bytes = off_yt * sizeof(T);                       // (A^{-1})_11^T
    static constexpr size_t off_tt_bytes = off_xt1_bytes + (size_t)32 * LDH * 4;      // (A_21 (A^{-1})_11)^T
    static_assert(2 * 32 * LDH * 4 <= CHUNK * LDC * sizeof(T), "helpers must fit in Y^T");
    static_assert(!COMPACT || (size_t)CHUNK * LDC * sizeof(T) <= (size_t)CHUNK * LDA * 4, "F must fit in A's place");
    static constexpr size_t smem_bytes = XF_IN_UT ? off_beta_bytes + CHUNK * 4 : off_xf_bytes + (size_t)CHUNK * LDA * 4;
    static_assert(!COMPACT || smem_bytes <= 80 * 1024, "two workgroups per CU");
    static constexpr int WGS_PER_CU = COMPACT ? 2 : 1;
};

// BWD: also write the backward-only outputs (all of them; their pointers are set).  A compile-time
// switch, so that the forward's instantiation carries none of that code.
template <typename TIO, int D, bool BWD, bool STRIDED>
__global__ __launch_bounds__(256, (PrepCfg<TIO, D>::WGS_PER_CU)) void prep_fwd_kernel(FwdParams p) {
    using C = PrepCfg<TIO, D>;
    using T = typename C::T;
    using Frag = typename Tr<T>::Frag;
    using FragV = typename Tr<TIO>::Frag;
    using Vec4 = typename Tr<T>::Vec4;
    constexpr int FE = C::FE, KW = C::KW, LDD = C::LDD, LDC = C::LDC, LDA = C::LDA;
    constexpr int SPB = 32 / KW;   // slabs per 32-index block

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    T* sT = reinterpret_cast<T*>(smem);
    T* Ws = sT + C::off_ws;
    // 16-bit operands: products with W^T take their fragments from the rows of W with transposing LDS reads, and
    // U^T has the space a transposed copy of W would need.  fp32 operands (no such read): W^T is written out,
    // element by element, while the chunk is staged, and U^T re-uses W's rows once phase 1 is over.
    constexpr bool WTR = sizeof(T) == 2;
    T* Wt = sT + C::off_wt;
    T* Ut = WTR ? Wt : Ws;
    T* Fs = sT + C::off_f;
    T* Gk = sT + C::off_gk;
    T* Yt = sT + C::off_yt;
    T* Nt = C::NT_IN_XF ? reinterpret_cast<T*>(smem + C::off_xf_bytes) : sT + C::off_nt;
    static_assert(!C::NT_IN_XF || C::LDC == C::LDA, "in-place N needs equal row pitch");
    float* Af = reinterpret_cast<float*>(smem + C::off_af_bytes);
    float* bs = reinterpret_cast<float*>(smem + C::off_beta_bytes);
    float* Xf = reinterpret_cast<float*>(smem + C::off_xf_bytes);
    float* XT1 = reinterpret_cast<float*>(smem + C::off_xt1_bytes);
    float* TT = reinterpret_cast<float*>(smem + C::off_tt_bytes);
    constexpr int LDH = C::LDH;
    constexpr bool COMPACT = C::COMPACT;

    const int chunk = blockIdx.x, bh = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, h = lane >> 5, l32 = lane & 31;
    const int L = seq_len(p.ul, bh, p.L), NC = p.NC;      // this head's own length; NC: chunks per head in the workspace arrays
    const int t0 = chunk * CHUNK;
    if (t0 >= L) return;                                   // (packed batch: a shorter sequence has fewer chunks)
    const int nvalid = (L - t0 < CHUNK) ? (L - t0) : CHUNK;
    const long long rowbase = user_vec(p.ul, bh, t0);       // the caller's layout: token stride TS between rows
    // token stride of the caller's tensors; a compile-time constant unless the layout interleaves heads
    // (then every row address costs vector arithmetic instead of an immediate offset)
    const int TS = STRIDED ? (int)p.ul.vt : D;
    const TIO* Qg = reinterpret_cast<const TIO*>(p.q) + rowbase;
    const TIO* Kg = reinterpret_cast<const TIO*>(p.k) + rowbase;
    const TIO* Vg = reinterpret_cast<const TIO*>(p.v) + rowbase;
    const TIO* Wg = reinterpret_cast<const TIO*>(p.w) + rowbase;
    const TIO* Bg = reinterpret_cast<const TIO*>(p.beta) + user_scl(p.ul, bh, t0);

    // V is only re-arranged (tiles V^T and, for the backward, V): the wave's elements of both, fetched at the
    // start and held in registers until the output phase.
    constexpr int NBV = (D / 32) * 2 / 4;           // 32x32 blocks of a 64 x d tile per wave
    typedef typename Tr<TIO>::Vec4 VecIO4;
    TIO vt_r[NBV][16];                              // V^T blocks: registers rows s, lane c
    VecIO4 vk_r[BWD ? NBV : 1][4];                  // V blocks: registers rows c (4 consecutive per load), lane s
    auto load_v = [&]() {
#pragma unroll
        for (int i = 0; i < NBV; ++i) {
            const int blk = wv + 4 * i;
            const int cb = blk >> 1, sb = blk & 1;
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const int s = 32 * sb + acc_row(j, h);
                vt_r[i][j] = (s < nvalid) ? Vg[s * TS + 32 * cb + l32] : (TIO)0.f;
            }
            if (BWD && p.ktT) {
                const int s = 32 * sb + l32;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) vk_r[i][g][r] = (TIO)0.f;
                    if (s < nvalid) vk_r[i][g] = *reinterpret_cast<const VecIO4*>(Vg + s * TS + 32 * cb + 8 * g + 4 * h);
                }
            }
        }
    };

    // ---- phase 0: stage the chunk (zero rows past L) ---------------------------
    // All of a thread's loads are issued before the first conversion, so their latencies overlap.
    {
        typedef typename Tr<TIO>::Frag FragIO;
        constexpr int NIT = CHUNK * (D / FE) / 256;
        FragIO wr[NIT];
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const int idx = tid + it * 256, row = idx / (D / FE), cf = idx % (D / FE);
            if (row < nvalid) wr[it] = ld_frag<TIO>(Wg + row * TS + cf * FE);
        }
        load_v();                     // needed only at the very end: in flight during everything in between
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const int idx = tid + it * 256, row = idx / (D / FE), cf = idx % (D / FE);
            Frag wv_ = Tr<T>::zero();
            if (row < nvalid) wv_ = cvt_frag<T, TIO>(wr[it]);
            *reinterpret_cast<Frag*>(Ws + row * LDD + cf * FE) = wv_;
            if (!WTR)
#pragma unroll
                for (int e = 0; e < FE; ++e) Wt[(cf * FE + e) * LDC + row] = wv_[e];
        }
    }
    if (tid < CHUNK) bs[tid] = (tid < nvalid) ? (float)Bg[tid * (int)p.ul.st] : 0.f;
    __syncthreads();

    // Q and K are read from global memory.  Rows past L must not be touched: those lanes are redirected to
    // row 0 and their products masked out by the zero W / the explicit masks below.

    const int bi = wv >> 1, bj = wv & 1;   // this wave's 32x32 block of a 64x64 result
    const size_t bhc = (size_t)bh * NC + chunk;

    // Row of Q/K this lane supplies as an operand row (clamped for the global path).
    auto qk_row = [&](int r) { return r < nvalid ? r : 0; };
    auto qk_ok = [&](int r) { return r < nvalid; };
    // operand fragment of row r of Q or K: the FE elements from column k on
    auto qk_frag = [&](const TIO* base, int r, int k) { return cvt_frag<T, TIO>(ld_frag<TIO>(base + (size_t)qk_row(r) * TS + k)); };
    // F block: rows t (Q), cols t' (W); keep t' <= t.
    auto f_block = [&]() {
        const int ar = 32 * (wv >> 1) + l32, bjj = wv & 1;
        f32x16 acc = zero16();
        const T* bp = Ws + (size_t)(32 * bjj + l32) * LDD + FE * h;
#pragma unroll
        for (int k0 = 0; k0 < D; k0 += KW) acc = Tr<T>::mma(qk_frag(Qg, ar, k0 + FE * h), ld_frag<T>(bp + k0), acc);
        const int tp = 32 * bjj + l32;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int t = 32 * (wv >> 1) + acc_row(j, h);
            Fs[t * LDC + tp] = (tp <= t && t < nvalid) ? (T)acc[j] : (T)0.f;
        }
    };

    // (W^T block cb) x (rows xr0.. of X)^T and (rows xr0.. of X) x (W^T block cb)^T, contraction over the chunk's tokens
    auto wt_times = [&](int cb, const T* X, int xr0) {
        if constexpr (WTR) {
            f32x16 acc = zero16();
            mm<T, CHUNK, true, false>(acc, Ws, LDD, 32 * cb, X, LDC, xr0, l32, h);
            return acc;
        } else {
            return gemm32<T, CHUNK>(Wt, LDC, 32 * cb, X, LDC, xr0, l32, h, zero16());
        }
    };
    auto times_wt = [&](const T* X, int xr0, int cb) {
        if constexpr (WTR) {
            f32x16 acc = zero16();
            mm<T, CHUNK, false, true>(acc, X, LDC, xr0, Ws, LDD, 32 * cb, l32, h);
            return acc;
        } else {
            return gemm32<T, CHUNK>(X, LDC, xr0, Wt, LDC, 32 * cb, l32, h, zero16());
        }
    };

    // ---- phase 1: products of the inputs ----------------------------------------
    // G block -> Af[t][s] = beta_t G[t][s] for s < t, else 0.
    {
        f32x16 acc = gemm32<T, D>(Ws, LDD, 32 * bi, Ws, LDD, 32 * bj, l32, h, zero16());
        const int s = 32 * bj + l32;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int t = 32 * bi + acc_row(j, h);
            Af[t * LDA + s] = (s < t) ? bs[t] * acc[j] : 0.f;
            if (BWD && p.gm) p.gm[bhc * 4096 + t * 64 + s] = acc[j];
        }
    }
    if (!COMPACT) f_block();          // (2-byte operands: at the start of phase 4, in A's place)
    // Gk block: rows t' (W), cols s (K); stored transposed Gk[s][t'], keep t' > s.
    {
        f32x16 acc = zero16();
        {
            const T* ap = Ws + (size_t)(32 * bi + l32) * LDD + FE * h;
#pragma unroll
            for (int k0 = 0; k0 < D; k0 += KW) acc = Tr<T>::mma(ld_frag<T>(ap + k0), qk_frag(Kg, 32 * bj + l32, k0 + FE * h), acc);
        }
        const int s = 32 * bj + l32;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            Vec4 v4;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int tp = 32 * bi + 8 * g + 4 * h + r;
                v4[r] = (tp > s && qk_ok(s)) ? (T)acc[4 * g + r] : (T)0.f;
            }
            *reinterpret_cast<Vec4*>(Gk + s * LDC + 32 * bi + 8 * g + 4 * h) = v4;
        }
    }
    // K Q^T block (rows s = keys, cols t = queries): first term of Sd^T, kept in registers.
    f32x16 accS = zero16();
    {
#pragma unroll
        for (int k0 = 0; k0 < D; k0 += KW) accS = Tr<T>::mma(qk_frag(Kg, 32 * bi + l32, k0 + FE * h), qk_frag(Qg, 32 * bj + l32, k0 + FE * h), accS);
    }
    __syncthreads();

    // ---- phase 2: X = A^{-1} (A unit lower triangular), then N = X diag(beta) --------------
    // Blocked: the two 32x32 diagonal blocks by forward substitution (waves 0 and 1, one
    // lane per column -- a column of the inverse depends only on itself), the off-diagonal
    // block X_21 = -X_22 (A_21 X_11) by two fp32 MFMA products.
    if (wv < 2) {
        if (lane < 32) {
            const int r0 = 32 * wv, c = lane;
            float n[32];
#pragma unroll
            for (int t = 0; t < 32; ++t) n[t] = 0.f;
#pragma unroll
            for (int t = 0; t < 32; ++t) {
                float a0 = (t == c) ? 1.f : 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
#pragma unroll
                for (int s4 = 0; s4 < (t + 3) / 4; ++s4) {
                    const f32x4 a4 = *reinterpret_cast<const f32x4*>(Af + (r0 + t) * LDA + r0 + 4 * s4);   // zeros for s >= t
                    a0 -= a4[0] * n[4 * s4 + 0];
                    a1 -= a4[1] * n[4 * s4 + 1];
                    a2 -= a4[2] * n[4 * s4 + 2];
                    a3 -= a4[3] * n[4 * s4 + 3];
                }
                const float acc = (a0 + a1) + (a2 + a3);
                n[t] = acc;
                Xf[(r0 + t) * LDA + r0 + c] = acc;
                if (wv == 0) XT1[c * LDH + t] = acc;
            }
        }
    } else if (wv == 2) {
        for (int idx = lane; idx < 32 * 32; idx += 64) Xf[(idx >> 5) * LDA + 32 + (idx & 31)] = 0.f;   // upper-right block
    }
    __syncthreads();
    if (wv == 0) {      // T = A_21 X_11, stored transposed
        f32x16 acc = gemm32<float, 32>(Af + 32 * LDA, LDA, 0, XT1, LDH, 0, l32, h, zero16());
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            f32x4 v4;
#pragma unroll
            for (int r = 0; r < 4; ++r) v4[r] = acc[4 * g + r];
            *reinterpret_cast<f32x4*>(TT + l32 * LDH + 8 * g + 4 * h) = v4;
        }
    }
    __syncthreads();
    if (wv == 0) {      // X_21 = -X_22 T
        f32x16 acc = gemm32<float, 32>(Xf + 32 * LDA + 32, LDA, 0, TT, LDH, 0, l32, h, zero16());
#pragma unroll
        for (int j = 0; j < 16; ++j) Xf[(32 + acc_row(j, h)) * LDA + l32] = -acc[j];
    }
    __syncthreads();
    for (int idx = tid; idx < CHUNK * CHUNK; idx += 256) {
        const int t = idx >> 6, c = idx & 63;
        const float x = Xf[t * LDA + c];
        Nt[t * LDC + c] = (T)(x * bs[c]);
        if (BWD && p.aim) reinterpret_cast<T*>(p.aim)[bhc * 4096 + idx] = (T)x;
    }
    __syncthreads();

    // ---- phase 3: U^T = W^T N^T  and  Y^T -----------------------------------------
    // Y block: rows t (N), cols s (Gk rows); stored transposed Yt[s][t].
    {
        f32x16 acc = gemm32<T, CHUNK>(Nt, LDC, 32 * bi, Gk, LDC, 32 * bj, l32, h, zero16());
        const int s = 32 * bj + l32;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            Vec4 v4;
#pragma unroll
            for (int r = 0; r < 4; ++r) v4[r] = (T)acc[4 * g + r];
            *reinterpret_cast<Vec4*>(Yt + s * LDC + 32 * bi + 8 * g + 4 * h) = v4;
        }
    }
    // U^T blocks: rows c (W^T), cols t (N rows).  (fp32 operands: Ut aliases Ws, all reads of Ws are done.)
    {
        f32x16 accU[D / 64];
#pragma unroll
        for (int i = 0; i < D / 64; ++i) {
            const int blk = wv + 4 * i;                 // (D/32)*2 blocks over 4 waves
            const int cb = blk >> 1, tb = blk & 1;
            accU[i] = wt_times(cb, Nt, 32 * tb);
        }
        __syncthreads();                                 // nobody still reads Ws (phase 1) -- and keeps phases apart
#pragma unroll
        for (int i = 0; i < D / 64; ++i) {
            const int blk = wv + 4 * i;
            const int cb = blk >> 1, tb = blk & 1;
#pragma unroll
            for (int j = 0; j < 16; ++j) Ut[(32 * cb + acc_row(j, h)) * LDC + 32 * tb + l32] = (T)accU[i][j];
        }
    }
    __syncthreads();

    // ---- phase 4: outputs -----------------------------------------------------------
    if (COMPACT) {       // F, into the space of the fp32 matrix A (dead since the inverse)
        f_block();
        __syncthreads();
    }
    if (BWD && p.fm) {   // backward: keep the chunk's matrices (row-major, operand type)
        T* fm = reinterpret_cast<T*>(p.fm) + bhc * 4096;
        T* gk = reinterpret_cast<T*>(p.gktm) + bhc * 4096;
        T* nm = reinterpret_cast<T*>(p.nm) + bhc * 4096;
        T* yt = reinterpret_cast<T*>(p.ytm) + bhc * 4096;
        T* ut = reinterpret_cast<T*>(p.utm) + bhc * (size_t)D * 64;
        // 16 bytes per lane (the LDS rows are 16-byte aligned: LDC * sizeof(T) is a multiple of 16)
        typedef T RowVec __attribute__((ext_vector_type(16 / sizeof(T))));
        constexpr int VE = 16 / (int)sizeof(T), VPR = 64 / VE;
        static_assert((LDC * sizeof(T)) % 16 == 0, "aligned rows");
        for (int idx = tid; idx < 64 * VPR; idx += 256) {
            const int r = idx / VPR, c = (idx % VPR) * VE;
            __builtin_nontemporal_store(*reinterpret_cast<const RowVec*>(Fs + r * LDC + c), reinterpret_cast<RowVec*>(fm + r * 64 + c));
            __builtin_nontemporal_store(*reinterpret_cast<const RowVec*>(Gk + r * LDC + c), reinterpret_cast<RowVec*>(gk + r * 64 + c));
            __builtin_nontemporal_store(*reinterpret_cast<const RowVec*>(Nt + r * LDC + c), reinterpret_cast<RowVec*>(nm + r * 64 + c));
            __builtin_nontemporal_store(*reinterpret_cast<const RowVec*>(Yt + r * LDC + c), reinterpret_cast<RowVec*>(yt + r * 64 + c));
        }
        for (int idx = tid; idx < D * VPR; idx += 256) {
            const int r = idx / VPR, c = (idx % VPR) * VE;
            __builtin_nontemporal_store(*reinterpret_cast<const RowVec*>(Ut + r * LDC + c), reinterpret_cast<RowVec*>(ut + r * 64 + c));
        }
    }
    // (a) Sd^T = K Q^T - Y^T F^T, accumulator order: [bhc][qb][kb][g][lane][4]
    {
        f32x16 corr = gemm32<T, CHUNK>(Yt, LDC, 32 * bi, Fs, LDC, 32 * bj, l32, h, zero16());
        float* dst = p.sd + (bhc * 4 + (size_t)(bj * 2 + bi)) * 1024;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            f32x4 v4;
#pragma unroll
            for (int r = 0; r < 4; ++r) v4[r] = accS[4 * g + r] - corr[4 * g + r];
            __builtin_nontemporal_store(v4, reinterpret_cast<f32x4*>(dst + (g * 64 + lane) * 4));
            if (BWD && p.sdm) *reinterpret_cast<f32x4*>(p.sdm + bhc * 4096 + (32 * bj + l32) * 64 + 32 * bi + 8 * g + 4 * h) = v4;
        }
    }
    // (b) -dP tile (rows = output column b of dP, contraction = a): acc rows a, cols b.
    {
        Frag* dst = reinterpret_cast<Frag*>(reinterpret_cast<T*>(p.dp) + bhc * (size_t)D * D);
        constexpr int NB = (D / 32) * (D / 32);
#pragma unroll
        for (int i = 0; i < NB / 4; ++i) {
            const int blk = wv + 4 * i;
            const int ab = blk / (D / 32), bb = blk % (D / 32);
            f32x16 acc = wt_times(ab, Ut, 32 * bb);
#pragma unroll
            for (int j = 0; j < 16; ++j) acc[j] = -acc[j];
            Frag fr[SPB];
            pack_block<T>(acc, fr);
#pragma unroll
            for (int s = 0; s < SPB; ++s) __builtin_nontemporal_store(fr[s], &dst[((size_t)bb * (D / KW) + ab * SPB + s) * 64 + lane]);
        }
    }
    // (c) Kb tile (rows = key s, contraction = c): acc rows c, cols s;  Kb^T = K^T - W^T Y.
    // (d) Qb in accumulator order (rows c, cols t): Qb^T = Q^T - U^T F^T.
    {
        Frag* kdst = reinterpret_cast<Frag*>(reinterpret_cast<T*>(p.kt) + bhc * (size_t)CHUNK * D);
        constexpr int NB = (D / 32) * 2;
#pragma unroll
        for (int i = 0; i < NB / 4; ++i) {
            const int blk = wv + 4 * i;
            const int cb = blk >> 1, sb = blk & 1;
            f32x16 acc = wt_times(cb, Yt, 32 * sb);
            const int s = 32 * sb + l32;
            const TIO* krow = Kg + (size_t)qk_row(s) * TS + 32 * cb + 4 * h;
            const bool ok = qk_ok(s);
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const VecIO4 k4 = *reinterpret_cast<const VecIO4*>(krow + 8 * g);
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[4 * g + r] = (ok ? (float)k4[r] : 0.f) - acc[4 * g + r];
            }
            Frag fr[SPB];
            pack_block<T>(acc, fr);
#pragma unroll
            for (int s2 = 0; s2 < SPB; ++s2) __builtin_nontemporal_store(fr[s2], &kdst[((size_t)sb * (D / KW) + cb * SPB + s2) * 64 + lane]);
            if (BWD && p.kbm) {       // backward only: the same keys row-major [token][c]
                typedef typename Tr<T>::Vec4 TVec4;
                T* kb = reinterpret_cast<T*>(p.kbm) + (bhc * CHUNK + s) * (size_t)D + 32 * cb + 4 * h;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    TVec4 o4;
#pragma unroll
                    for (int r = 0; r < 4; ++r) o4[r] = (T)acc[4 * g + r];
                    *reinterpret_cast<TVec4*>(kb + 8 * g) = o4;
                }
            }
        }
#pragma unroll
        for (int i = 0; i < NB / 4; ++i) {
            const int blk = wv + 4 * i;
            const int cb = blk >> 1, tb = blk & 1;
            f32x16 acc = gemm32<T, CHUNK>(Ut, LDC, 32 * cb, Fs, LDC, 32 * tb, l32, h, zero16());
            const int t = 32 * tb + l32;
            const TIO* qrow = Qg + (size_t)qk_row(t) * TS + 32 * cb + 4 * h;
            const bool ok = qk_ok(t);
            // xinit: [bh][query block of 32][d block][g][lane][4]
            float* xdst = p.xinit + ((((size_t)bh * NC + chunk) * 2 + tb) * (D / 32) + cb) * 1024;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const VecIO4 q4 = *reinterpret_cast<const VecIO4*>(qrow + 8 * g);
                f32x4 v4;
#pragma unroll
                for (int r = 0; r < 4; ++r) v4[r] = (ok ? (float)q4[r] : 0.f) - acc[4 * g + r];
                __builtin_nontemporal_store(v4, reinterpret_cast<f32x4*>(xdst + (g * 64 + lane) * 4));
            }
        }
        // (e) V^T tile (rows = c, contraction = key s): plain re-layout of V.
        FragV* vdst = reinterpret_cast<FragV*>(reinterpret_cast<TIO*>(p.vt) + bhc * (size_t)CHUNK * D);
#pragma unroll
        for (int i = 0; i < NB / 4; ++i) {
            const int blk = wv + 4 * i;
            const int cb = blk >> 1, sb = blk & 1;
            f32x16 acc;
#pragma unroll
            for (int j = 0; j < 16; ++j) acc[j] = (float)vt_r[i][j];
            FragV fr[SPB];
            pack_block<TIO>(acc, fr);
#pragma unroll
            for (int s2 = 0; s2 < SPB; ++s2) __builtin_nontemporal_store(fr[s2], &vdst[(((size_t)sb * (D / 32) + cb) * SPB + s2) * 64 + lane]);   // [key half][d block][slab]
        }
        if (BWD && p.dpt && sizeof(T) == 4) {
            // -dP in the transposed arrangement (rows c, contraction b) = -dP[c][b]: accumulate with rows b,
            // lane c.  Read by the backward's adjoint scan for fp32 operands (the 16-bit one transposes in LDS).
            Frag* pdst = reinterpret_cast<Frag*>(reinterpret_cast<T*>(p.dpt) + bhc * (size_t)D * D);
            constexpr int NBP = (D / 32) * (D / 32);
#pragma unroll
            for (int i = 0; i < NBP / 4; ++i) {
                const int blk = wv + 4 * i;
                const int bb = blk / (D / 32), cb = blk % (D / 32);
                f32x16 acc = times_wt(Ut, 32 * bb, cb);
#pragma unroll
                for (int j = 0; j < 16; ++j) acc[j] = -acc[j];
                Frag fr[SPB];
                pack_block<T>(acc, fr);
#pragma unroll
                for (int s2 = 0; s2 < SPB; ++s2) __builtin_nontemporal_store(fr[s2], &pdst[((size_t)cb * (D / KW) + bb * SPB + s2) * 64 + lane]);
            }
        }
        if (BWD && p.ktT) {
            // ---- backward-only tiles ------------------------------------------------------------
            constexpr int QS = CHUNK / KW;
            // ktT (rows c, contraction s) = Kb[s][c]: accumulate with rows s, lane c.  fp32 operands only: the 16-bit
            // adjoint scan reads these fragments out of the key tile with transposing LDS reads.
            Frag* tdst = reinterpret_cast<Frag*>(reinterpret_cast<T*>(p.ktT) + bhc * (size_t)CHUNK * D);
#pragma unroll
            for (int i = 0; i < (sizeof(T) == 4 ? NB / 4 : 0); ++i) {
                const int blk = wv + 4 * i;
                const int cb = blk >> 1, sb = blk & 1;
                f32x16 acc = times_wt(Yt, 32 * sb, cb);
                const int c = 32 * cb + l32;
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    const int s = 32 * sb + acc_row(j, h);
                    const float kv = qk_ok(s) ? (float)Kg[(size_t)qk_row(s) * TS + c] : 0.f;
                    acc[j] = kv - acc[j];
                }
                Frag fr[SPB];
                pack_block<T>(acc, fr);
#pragma unroll
                for (int s2 = 0; s2 < SPB; ++s2) __builtin_nontemporal_store(fr[s2], &tdst[((size_t)cb * QS + sb * SPB + s2) * 64 + lane]);
            }
            // vk (rows s, contraction c) = V[s][c] (I/O type): registers rows c, lane s
            FragV* vkd = reinterpret_cast<FragV*>(reinterpret_cast<TIO*>(p.vk) + bhc * (size_t)CHUNK * D);
#pragma unroll
            for (int i = 0; i < NB / 4; ++i) {
                const int blk = wv + 4 * i;
                const int cb = blk >> 1, sb = blk & 1;
                f32x16 acc;
#pragma unroll
                for (int j = 0; j < 16; ++j) acc[j] = (float)vk_r[i][j >> 2][j & 3];
                FragV fr[SPB];
                pack_block<TIO>(acc, fr);
#pragma unroll
                for (int s2 = 0; s2 < SPB; ++s2) __builtin_nontemporal_store(fr[s2], &vkd[((size_t)sb * (D / KW) + cb * SPB + s2) * 64 + lane]);
            }
        }
    }
}

template <typename T, int D, bool BWD, bool STRIDED>
hipError_t launch_prep_fwd_s(const FwdParams& p, hipStream_t stream) {
    using C = PrepCfg<T, D>;
    static_assert(sizeof(typename C::T) == sizeof(T), "tile sizes assume equal operand and I/O width");
    // set once per process; a function-local static is initialised under the language's own lock
    static const hipError_t attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&prep_fwd_kernel<T, D, BWD, STRIDED>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::smem_bytes);
    if (attr_err != hipSuccess) return attr_err;
    dim3 grid(p.NC, p.B * p.H);
    hipLaunchKernelGGL((prep_fwd_kernel<T, D, BWD, STRIDED>), grid, dim3(256), C::smem_bytes, stream, p);
    return hipGetLastError();
}
template <typename T, int D, bool BWD>
hipError_t launch_prep_fwd_b(const FwdParams& p, hipStream_t stream) {
    return p.ul.vt != D ? launch_prep_fwd_s<T, D, BWD, true>(p, stream) : launch_prep_fwd_s<T, D, BWD, false>(p, stream);
}
template <typename T, int D>
hipError_t launch_prep_fwd_t(const FwdParams& p, hipStream_t stream) {
    return p.fm ? launch_prep_fwd_b<T, D, true>(p, stream) : launch_prep_fwd_b<T, D, false>(p, stream);
}

hipError_t launch_prep_fwd(const FwdParams& p, int d, int is_bf16, hipStream_t stream) {
    if (is_bf16) return d == 64 ? launch_prep_fwd_t<bf16_t, 64>(p, stream) : launch_prep_fwd_t<bf16_t, 128>(p, stream);
    return d == 64 ? launch_prep_fwd_t<float, 64>(p, stream) : launch_prep_fwd_t<float, 128>(p, stream);
}

}  // namespace path
