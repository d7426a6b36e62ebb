// Right-to-left sweep of PaTH attention (paper Sec. 3.3, boxed workflow):
// for a resident query tile, walk the key chunks from the diagonal down to
// chunk 0; per chunk take the logits against the boundary-adjusted keys,
// update the online softmax and the output accumulator, then apply the
// chunk's transition product to the query state.
//
// Layout of the computation (everything transposed so that activations stay
// in registers): wave = 32 queries = 32 MFMA columns; per key chunk j
//
//     S^T (64 x 32)  = Kb_j   X^T          A = Kb tile (LDS),   B = X   (registers)
//     O^T (D x 32)  += V_j^T  P^T          A = V^T tile (LDS),  B = P   (registers)
//     X^T (D x 32)  += (-dP_j)^T X^T       A = -dP tile (LDS),  B = X   (registers)
//
// Keys run along accumulator registers, so the softmax row statistics are
// per-lane reductions plus one exchange between the two half-waves.  The
// query state keeps an fp32 master (the accumulator of the third product);
// it is rounded to the operand type only as an MFMA input.  The diagonal
// chunk's logits come precomputed (fp32) from the preprocessing kernel.
#include "path_common.h"

namespace path {

template <typename T, int D> struct FwdCfg {
    static constexpr int FE = Tr<T>::FE;
    static constexpr int KW = Tr<T>::KW;
    static constexpr int KV_FRAGS = CHUNK * D / FE;     // fragments per K / V^T tile
    static constexpr int DP_FRAGS = D * D / FE;         // fragments per -dP tile
    static constexpr size_t smem_bytes = (size_t)(2 * KV_FRAGS + DP_FRAGS) * 16;
};

// TIO: storage type of v and o (and of P as an operand); T: operand type of X, Kb, dP.
// STATES_ONLY (backward): no logits, softmax or output; instead the query state of
// every (query block, key chunk) pair is written row-major to p.xs for the backward.
template <typename TIO, int D, bool STATES_ONLY>
__global__ __launch_bounds__(256) void attn_fwd_kernel(FwdParams p) {
    using C = FwdCfg<TIO, D>;
    using T = typename Compute<TIO>::type;
    using Frag = typename Tr<T>::Frag;
    using FragV = typename Tr<TIO>::Frag;
    using Vec4 = typename Tr<TIO>::Vec4;
    constexpr int KW = C::KW;
    constexpr int SPB = 32 / KW;       // slabs per 32-index block
    constexpr int DB = D / 32;         // 32-row blocks along d
    constexpr int DS = D / KW;         // slabs along d
    constexpr int CS = CHUNK / KW;     // slabs along the 64 keys of a chunk

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    Frag* sK = reinterpret_cast<Frag*>(smem);
    FragV* sV = reinterpret_cast<FragV*>(sK + C::KV_FRAGS);
    Frag* sP = sK + 2 * C::KV_FRAGS;

    const int BH = p.B * p.H, L = p.L, NC = p.NC;
    const int ntiles = (NC + 1) / 2;
    // heaviest (right-most) query tiles first; the heads of one tile index are adjacent
    const int tile = ntiles - 1 - (int)(blockIdx.x / BH);
    const int bh = blockIdx.x % BH;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, h = lane >> 5, l32 = lane & 31;

    const int qblk = tile * 4 + wv;            // 32-query block of this wave
    const int cq = qblk >> 1;                  // its chunk
    const int qb = qblk & 1;                   // which half of the chunk
    const bool active = cq < NC;
    const int jtop = (2 * tile + 1 < NC) ? 2 * tile + 1 : NC - 1;

    const float sl2 = p.scale * 1.44269504088896340736f;    // logits in base-2 units

    // ---- query state: fp32 master Xm (accumulator layout) + operand copy Xb -----
    f32x16 Xm[DB];
    Frag Xb[DS];
    f32x16 O[DB];
#pragma unroll
    for (int b = 0; b < DB; ++b) { Xm[b] = zero16(); O[b] = zero16(); }
    if (active) {
        const float* xs = p.xinit + ((size_t)bh * NC * 2 + qblk) * (size_t)DB * 1024;
#pragma unroll
        for (int b = 0; b < DB; ++b)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const f32x4 v4 = *reinterpret_cast<const f32x4*>(xs + ((size_t)b * 4 + g) * 256 + lane * 4);
#pragma unroll
                for (int r = 0; r < 4; ++r) Xm[b][4 * g + r] = v4[r];
            }
    }
#pragma unroll
    for (int b = 0; b < DB; ++b) pack_block<T>(Xm[b], Xb + b * SPB);

    float m_run = -INFINITY;    // running max of the base-2 logits of this lane's query
    float l_run = 0.f;          // running sum over the keys THIS half-wave holds

    const T* ktg = reinterpret_cast<const T*>(p.kt) + (size_t)bh * NC * CHUNK * D;
    const TIO* vtg = reinterpret_cast<const TIO*>(p.vt) + (size_t)bh * NC * CHUNK * D;
    const T* dpg = reinterpret_cast<const T*>(p.dp) + (size_t)bh * NC * D * D;

    for (int j = jtop; j >= 0; --j) {
        // ---- stage tiles of chunk j ---------------------------------------------
        const bool need_dp = j < jtop && j > 0;     // some wave of the tile lies right of chunk j
        __syncthreads();
        {
            if (!STATES_ONLY) {
                const Frag* gk = reinterpret_cast<const Frag*>(ktg + (size_t)j * CHUNK * D);
                const FragV* gv = reinterpret_cast<const FragV*>(vtg + (size_t)j * CHUNK * D);
#pragma unroll
                for (int i = 0; i < C::KV_FRAGS / 256; ++i) {
                    sK[i * 256 + tid] = gk[i * 256 + tid];
                    sV[i * 256 + tid] = gv[i * 256 + tid];
                }
            }
            if (need_dp) {
                const Frag* gp = reinterpret_cast<const Frag*>(dpg + (size_t)j * D * D);
#pragma unroll
                for (int i = 0; i < C::DP_FRAGS / 256; ++i) sP[i * 256 + tid] = gp[i * 256 + tid];
            }
        }
        __syncthreads();
        if (!active || j > cq) continue;

        if (STATES_ONLY) {
            if (j == cq) continue;
            // state of this wave's 32 queries against key chunk j, as two fragment-order tiles of
            // the pair (cq, j): xs (rows q, contraction c) is the operand copy itself; xsT (rows c,
            // contraction q) is its transpose, taken through the matrix unit.
            {
                const size_t slot = ((size_t)bh * NC * (NC - 1) / 2 + pair_slot(cq, j)) * (size_t)CHUNK * D;
                Frag* xd = reinterpret_cast<Frag*>(reinterpret_cast<T*>(p.xs) + slot);
#pragma unroll
                for (int s = 0; s < DS; ++s) xd[((size_t)qb * DS + s) * 64 + lane] = Xb[s];
                Frag* xt = reinterpret_cast<Frag*>(reinterpret_cast<T*>(p.xsT) + slot);
                Frag idf[SPB];
                identity_frags<T>(idf, l32, h);
#pragma unroll
                for (int b = 0; b < DB; ++b) {
                    const f32x16 tr = transpose32<T>(Xb + b * SPB, idf);     // rows q, lane c (block b)
                    Frag fr[SPB];
                    pack_block<T>(tr, fr);
#pragma unroll
                    for (int s2 = 0; s2 < SPB; ++s2) xt[((size_t)b * (CHUNK / KW) + qb * SPB + s2) * 64 + lane] = fr[s2];
                }
            }
            if (j > 0) {
#pragma unroll
                for (int b = 0; b < DB; ++b)
#pragma unroll
                    for (int s = 0; s < DS; ++s) Xm[b] = Tr<T>::mma(sP[(b * DS + s) * 64 + lane], Xb[s], Xm[b]);
#pragma unroll
                for (int b = 0; b < DB; ++b) pack_block<T>(Xm[b], Xb + b * SPB);
            }
            continue;
        }

        // ---- logits S^T: two 32-key blocks ----------------------------------------
        f32x16 S[2];
        if (j == cq) {
            // diagonal chunk: precomputed Q K^T - F Y, causal mask key <= query
            const float* sd = p.sd + (((size_t)bh * NC + j) * 4 + (size_t)qb * 2) * 1024;
            const int tq = 32 * qb + l32;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const f32x4 v4 = *reinterpret_cast<const f32x4*>(sd + ((size_t)kb * 4 + g) * 256 + lane * 4);
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int sk = 32 * kb + 8 * g + 4 * h + r;
                        S[kb][4 * g + r] = (sk <= tq) ? v4[r] * sl2 : -INFINITY;
                    }
                }
        } else {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                f32x16 acc = zero16();
#pragma unroll
                for (int s = 0; s < DS; ++s) acc = Tr<T>::mma(sK[(kb * DS + s) * 64 + lane], Xb[s], acc);
#pragma unroll
                for (int jj = 0; jj < 16; ++jj) acc[jj] *= sl2;
                S[kb] = acc;
            }
        }

        // ---- online softmax (base 2) ------------------------------------------------
        float mloc = S[0][0];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int jj = 0; jj < 16; ++jj) mloc = fmaxf(mloc, S[kb][jj]);
        mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
        const float m_new = fmaxf(m_run, mloc);         // finite: the diagonal chunk comes first
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        float rs = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int jj = 0; jj < 16; ++jj) {
                const float e = __builtin_amdgcn_exp2f(S[kb][jj] - m_new);
                S[kb][jj] = e;
                rs += e;
            }
        l_run = l_run * alpha + rs;
        m_run = m_new;
        FragV Pb[CS];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) pack_block<TIO>(S[kb], Pb + kb * SPB);

        // ---- O^T = alpha O^T + V^T P^T -------------------------------------------------
#pragma unroll
        for (int b = 0; b < DB; ++b) {
#pragma unroll
            for (int jj = 0; jj < 16; ++jj) O[b][jj] *= alpha;
#pragma unroll
            for (int s = 0; s < CS; ++s) O[b] = Tr<TIO>::mma(sV[(b * CS + s) * 64 + lane], Pb[s], O[b]);
        }

        // ---- X <- X (I - dP_j): only if keys further left will still be visited -------
        if (j < cq && j > 0) {
#pragma unroll
            for (int b = 0; b < DB; ++b)
#pragma unroll
                for (int s = 0; s < DS; ++s) Xm[b] = Tr<T>::mma(sP[(b * DS + s) * 64 + lane], Xb[s], Xm[b]);
#pragma unroll
            for (int b = 0; b < DB; ++b) pack_block<T>(Xm[b], Xb + b * SPB);
        }
    }

    // ---- epilogue: normalise, store o and lse (paper Sec. 3.3 last step) -----------------
    if (!active || STATES_ONLY) return;
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    const float inv = 1.f / l_tot;
    const int tq = qblk * 32 + l32;
    if (tq < L) {
        TIO* orow = reinterpret_cast<TIO*>(p.o) + ((size_t)bh * L + tq) * D + 4 * h;
#pragma unroll
        for (int b = 0; b < DB; ++b)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                Vec4 v4;
#pragma unroll
                for (int r = 0; r < 4; ++r) v4[r] = (TIO)(O[b][4 * g + r] * inv);
                *reinterpret_cast<Vec4*>(orow + 32 * b + 8 * g) = v4;
            }
        if (h == 0) p.lse[(size_t)bh * L + tq] = (m_run + __builtin_amdgcn_logf(l_tot)) * 0.69314718055994530942f;
    }
}

template <typename T, int D, bool STATES_ONLY>
hipError_t launch_attn_fwd_t(const FwdParams& p, hipStream_t stream) {
    using C = FwdCfg<T, D>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_fwd_kernel<T, D, STATES_ONLY>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::smem_bytes);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int ntiles = (p.NC + 1) / 2;
    dim3 grid((unsigned)(ntiles * p.B * p.H));
    hipLaunchKernelGGL((attn_fwd_kernel<T, D, STATES_ONLY>), grid, dim3(256), C::smem_bytes, stream, p);
    return hipGetLastError();
}

// Backward helper: the same sweep, query states only (written to p.xs).
hipError_t launch_attn_states(const FwdParams& p, int d, int is_bf16, hipStream_t stream) {
    if (is_bf16) return d == 64 ? launch_attn_fwd_t<bf16_t, 64, true>(p, stream) : launch_attn_fwd_t<bf16_t, 128, true>(p, stream);
    return d == 64 ? launch_attn_fwd_t<float, 64, true>(p, stream) : launch_attn_fwd_t<float, 128, true>(p, stream);
}

}  // namespace path
