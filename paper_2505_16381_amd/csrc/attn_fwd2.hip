// Forward sweep of PaTH attention, two blocking levels (paper Sec. 3.3 workflow;
// the second level is this library's own, see prep2_fwd.hip).
//
// One workgroup = 4 waves = 128 queries = two chunks; wave w owns the 32-query
// half (w & 1) of chunk 2*tile + (w >> 1).  A wave's working set fits the 256
// architectural VGPRs and a workgroup uses 64 KB of LDS, so TWO workgroups share
// a CU: they are not synchronised with each other, and the vector work (softmax)
// of one runs under the matrix work of the other.  Everything is transposed so
// that activations stay in registers:
//
//     S^T (32 keys x 32 q)  = Kb   X^T        A = key tile (LDS),  B = X (registers)
//     O^T (d x 32 q)       += V^T  P^T        A = V^T tile (LDS),  B = P (registers)
//     X^T (d x 32 q)       += (-dP)^T X^T     A = -dP tile (LDS),  B = X (registers)
//
// The key axis is walked right to left in stages of 32 keys (half a chunk),
// double buffered with direct-to-LDS loads, one barrier per stage.  Phase A
// (chunks of the query tile's own super-block): chunk-level keys, one state
// update per chunk; the wave's own chunk uses the precomputed diagonal logits.
// Phase B (super-blocks further left): keys carried to the super-block edge,
// ONE state update per super-block.  Workgroups are numbered so that one XCD
// works through the query tiles of one head at a time (its K/V/dP stay in that
// XCD's L2), heaviest tile first.
#include <type_traits>

#include "path_common.h"

namespace path {

#ifndef FWD2_CPT
#define FWD2_CPT 2                  // query chunks per workgroup (two waves each); 4 was tried: 6 % slower
#endif
constexpr int FWD2_THREADS = 128 * FWD2_CPT;

template <typename TIO, int D> struct Fwd2Cfg {
    typedef typename Compute<TIO>::type T;
    static constexpr int FE = Tr<T>::FE;
    static constexpr int HALF_FRAGS = 32 * D / FE;      // fragments of 32 keys of a key tile / V^T tile
    static constexpr int DP_FRAGS = D * D / FE;         // fragments per -dP tile
    static constexpr size_t smem_bytes = (size_t)(4 * HALF_FRAGS + DP_FRAGS) * 16 + 256;   // 2 stages x (K|V) + dP + 2 x 32 gate sums
};

__device__ __forceinline__ void wait_tiles_and_sync() {
    __builtin_amdgcn_s_waitcnt(0x0000);   // vmcnt(0) expcnt(0) lgkmcnt(0): this wave's tile loads have landed
    __syncthreads();
}

// FOX (PaTH-FoX, paper Sec. 2.2 extension): the logit of key j gets - c_j (c = cumulative log of the
// forget gates, here in base-2 units); the query's own + c_i cancels in the softmax and is added
// to the log-sum-exp at the end.
//
// EMIT (forward of a training pair): the query states the backward needs are written on the way,
// in the arrangement of the backward's own states sweep (see states_bwd.hip): whenever a wave
// meets a new key block -- a chunk j < cq of its own super-block, or a super-block further left --
// it stores its state as the tiles xs and xsT of the pair (cq, block).
//
// RING (sequence-parallel forward, Sec. 3.5): 1 = the sweep over a device's own segment; it also applies the
// product of the segment's first chunk / super-block at the end (the query state then stands at the segment's left
// edge, ready for the keys of the segment before) and stores its registers instead of writing o and lse.
// 2 = one hop: the registers are loaded, all chunks of an earlier segment are swept as "far" blocks (second-level
// keys, one product per super-block, the first one's included), and the registers are stored again.
template <typename TIO, int D, bool FOX, bool EMIT, int RING = 0>
__global__ __launch_bounds__(FWD2_THREADS, 512 / FWD2_THREADS) void attn_fwd2_kernel(FwdParams p) {
    using C = Fwd2Cfg<TIO, D>;
    using T = typename C::T;
    using Frag = typename Tr<T>::Frag;
    using FragV = typename Tr<TIO>::Frag;
    using Vec4 = typename Tr<TIO>::Vec4;
    constexpr int KW = Tr<T>::KW;
    constexpr int SPB = 32 / KW, DB = D / 32, DS = D / KW;
    constexpr int HF = C::HALF_FRAGS, DPF = C::DP_FRAGS;
    constexpr bool HAS_MASTER = sizeof(T) == 2;      // fp32 operands are their own master copy

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    Frag* sKV = reinterpret_cast<Frag*>(smem);                  // [2 stages][K half | V half]
    Frag* sP = sKV + 4 * HF;                                    // -dP tile
    float* sC = reinterpret_cast<float*>(sP + DPF);             // FOX: [2 stages][32] gate sums of the stage's keys

    const int BH = p.B * p.H, NC = p.NC;            // NC: chunks per head in the workspace arrays and in the grid's numbering
    const int NCq = RING == 2 ? p.NCq : NC;         // chunks of the query side (a hop's keys belong to another segment)
    const int ntiles = (NCq + FWD2_CPT - 1) / FWD2_CPT;
    // XCD-aware numbering: workgroup b runs on XCD b % 8; that XCD takes heads xcd, xcd+8, ...
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    // (the division runs on the vector unit; its result, uniform over the workgroup, goes back to scalar
    // registers, so that everything derived from it -- loop bounds, tile addresses -- is scalar arithmetic)
    const int bh = __builtin_amdgcn_readfirstlane((slot / ntiles) * 8 + xcd);
    const int tile = __builtin_amdgcn_readfirstlane(ntiles - 1 - slot % ntiles);
    if (bh >= BH) return;
    const int tid = threadIdx.x, lane = tid & 63, wv = __builtin_amdgcn_readfirstlane(tid >> 6), h = lane >> 5, l32 = lane & 31;

    const int L = seq_len(p.ul, bh, p.L);
    const int NCown = RING == 2 ? NCq : (L + CHUNK - 1) / CHUNK;     // this head's own length (packed batches: may be shorter)
    if (tile * FWD2_CPT >= NCown) return;
    const int cq = tile * FWD2_CPT + (wv >> 1);     // this wave's chunk
    const int qb = wv & 1;                          // ... and which 32-query half of it
    const bool active = cq < NCown;
    // (a hop sweeps every chunk of the other segment, all of them as far blocks)
    const int jtop = RING == 2 ? NC - 1 : ((tile * FWD2_CPT + FWD2_CPT - 1 < NCown) ? tile * FWD2_CPT + FWD2_CPT - 1 : NCown - 1);
    static_assert(SBC % FWD2_CPT == 0, "a tile must lie in one super-block");
    const int jsb = RING == 2 ? NC : (tile * FWD2_CPT / SBC) * SBC;  // first chunk of the tile's own super-block
    const int nsb = (NC + SBC - 1) / SBC;
    const float sl2 = p.scale * 1.44269504088896340736f;

    // ---- query state (fp32 master + operand copy), output accumulator, softmax statistics ----
    f32x16 O[DB], Xm[HAS_MASTER ? DB : 1];
    Frag Xh[DS];
    float m_run = -INFINITY, l_run = 0.f;           // m in base-2 logit units
    float* const rec = RING ? p.ring_state + (((size_t)bh * NCq + cq) * 2 + qb) * ring_rec_floats(D) : nullptr;
    // PaTH-FoX in a hop: the gate sums of the other segment count from ITS start.  With T its total and g the totals of
    // the segments already passed, key j's logit gets g + T - c_j (the query's own + c_i, local to its segment, is added
    // at the end as always).
    float goff = 0.f, koff = 0.f;
    if (RING == 2 && active) {
        m_run = rec[2 * DB * 1024 + lane]; l_run = rec[2 * DB * 1024 + 64 + lane];
        if (FOX) { goff = rec[2 * DB * 1024 + 128 + lane]; koff = goff + p.cum[(size_t)bh * NC * CHUNK + (size_t)NC * CHUNK - 1]; }
    }
#pragma unroll
    for (int b = 0; b < DB; ++b) {
        O[b] = zero16();
        f32x16 x = zero16();
        if (RING == 2 && active) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const f32x4 o4 = *reinterpret_cast<const f32x4*>(rec + (size_t)(DB + b) * 1024 + g * 256 + lane * 4);
#pragma unroll
                for (int r = 0; r < 4; ++r) O[b][4 * g + r] = o4[r];
            }
        }
        if (active) {
            const float* xs = RING == 2 ? rec + (size_t)b * 1024
                                        : p.xinit + (((size_t)bh * NC + cq) * 2 + qb) * (size_t)DB * 1024 + (size_t)b * 1024;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const f32x4 v4 = *reinterpret_cast<const f32x4*>(xs + g * 256 + lane * 4);
#pragma unroll
                for (int r = 0; r < 4; ++r) x[4 * g + r] = v4[r];
            }
        }
        if (HAS_MASTER) Xm[b] = x;
        pack_block<T>(x, Xh + b * SPB);
    }

    const T* ktg = reinterpret_cast<const T*>(p.kt) + (size_t)bh * NC * CHUNK * D;
    const T* kt2g = reinterpret_cast<const T*>(p.kt2) + (size_t)bh * NC * CHUNK * D;
    const TIO* vtg = reinterpret_cast<const TIO*>(p.vt) + (size_t)bh * NC * CHUNK * D;
    const T* dpg = reinterpret_cast<const T*>(p.dp) + (size_t)bh * NC * D * D;
    const T* dp2g = reinterpret_cast<const T*>(p.dp2) + (size_t)bh * nsb * D * D;

    // Stage u = 0, 1, ...: chunk j = jtop - u/2, key half kb = u % 2, LDS buffer u % 2.
    const int nstage = 2 * (jtop + 1);
    auto issue_kv = [&](int u) {
        const int j = jtop - (u >> 1), kb = u & 1;
        Frag* buf = sKV + (size_t)(u & 1) * 2 * HF;
        const T* kg = (j >= jsb ? ktg : kt2g) + (size_t)j * CHUNK * D;
        async_copy_tile<FWD2_THREADS, HF>(reinterpret_cast<const Frag*>(kg) + kb * HF, buf, tid, wv);
        async_copy_tile<FWD2_THREADS, HF>(reinterpret_cast<const Frag*>(vtg + (size_t)j * CHUNK * D) + kb * HF, buf + HF, tid, wv);
        if (FOX && tid < 8)      // 32 floats, 16 bytes per lane
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(p.cum + (size_t)bh * NC * CHUNK + (size_t)j * CHUNK + 32 * kb + 4 * tid),
                                             (__attribute__((address_space(3))) void*)(sC + (u & 1) * 32), 16, 0, 0);
    };
    // the product applied after chunk j (if any): loaded while the chunk's first half is
    // processed (sP is free then: the previous update ended before this stage's barrier)
    auto issue_dp = [&](int j) {
        if (j >= jsb) {
            if (j < jtop && (j > 0 || RING)) async_copy_tile<FWD2_THREADS, DPF>(reinterpret_cast<const Frag*>(dpg + (size_t)j * D * D), sP, tid, wv);
        } else if (j % SBC == 0 && (j > 0 || RING)) {
            async_copy_tile<FWD2_THREADS, DPF>(reinterpret_cast<const Frag*>(dp2g + (size_t)(j / SBC) * D * D), sP, tid, wv);
        }
    };

    // One stage of an active wave (chunk j <= cq).  DIAG: the wave's own chunk (precomputed logits, causal mask,
    // no state update after it); otherwise a chunk further left.
    auto stage = [&](int u, auto diag_tag) {
        constexpr bool DIAG = decltype(diag_tag)::value;
        const int j = jtop - (u >> 1), kb = u & 1;
        const Frag* sK = sKV + (size_t)(u & 1) * 2 * HF;
        const FragV* sV = reinterpret_cast<const FragV*>(sK + HF);
        if (!DIAG) {
            if (EMIT && kb == 0 && (j >= jsb || (j % SBC) == SBC - 1)) {
                constexpr int QS = CHUNK / KW;
                const size_t slot = ((size_t)bh * num_block_slots(NC) + block_slot(cq, j >= jsb ? j : j - (SBC - 1), NC)) * (size_t)CHUNK * D;
                Frag* xd = reinterpret_cast<Frag*>(reinterpret_cast<T*>(p.xs) + slot);
#pragma unroll
                for (int s = 0; s < DS; ++s) __builtin_nontemporal_store(Xh[s], &xd[((size_t)qb * DS + s) * 64 + lane]);     // streamed: keep the key/value tiles in L2
                if (sizeof(T) == 4 || j < jsb) {     // (16-bit operands: the near blocks' consumer transposes xs itself)
                    Frag* xt = reinterpret_cast<Frag*>(reinterpret_cast<T*>(p.xsT) + slot);
                    Frag idf[SPB];
                    identity_frags<T>(idf, l32, h);
#pragma unroll
                    for (int b = 0; b < DB; ++b) {
                        const f32x16 tr = transpose32<T>(Xh + b * SPB, idf);     // rows q, lane c (block b)
                        Frag fr[SPB];
                        pack_block<T>(tr, fr);
#pragma unroll
                        for (int s2 = 0; s2 < SPB; ++s2) __builtin_nontemporal_store(fr[s2], &xt[((size_t)b * QS + qb * SPB + s2) * 64 + lane]);
                    }
                }
            }
        }

        // ---- logits of 32 keys (raw, unscaled) -------------------------------------------
        f32x16 S;
        if (DIAG) {                       // own chunk: precomputed Q K^T - F Y, causal mask
            const float* diag = p.sd + ((size_t)bh * NC + j) * 4096 + ((size_t)qb * 2 + kb) * 1024;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const f32x4 v4 = *reinterpret_cast<const f32x4*>(diag + g * 256 + lane * 4);
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int sk = 32 * kb + 8 * g + 4 * h + r, tq = 32 * qb + l32;
                    S[4 * g + r] = (sk <= tq) ? v4[r] : -INFINITY;
                }
            }
        } else {
            S = zero16();
#pragma unroll
            for (int s = 0; s < DS; ++s) S = Tr<T>::mma(sK[s * 64 + lane], Xh[s], S);
        }

        // ---- online softmax.  Fast path: exponentiate against the current reference maximum
        // without looking at the block's own maximum; only if a lane's partial row sum is not
        // below 2^16 (a logit beat the reference by more than ~16 bits, or overflowed), or on
        // the wave's first block, take the slow path: find the block maximum, move the
        // reference, rescale O and l, and exponentiate again.  Probabilities may thus be as
        // large as 2^16, which bf16/fp32 operands and the fp32 sums hold without loss.
        {
            f32x16 E;
            float rs = 0.f;
            if (FOX) {            // T = logit in base-2 units minus the key's gate sum; then as below with scale 1
                const float* ck = sC + (u & 1) * 32 + 4 * h;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const f32x4 c4 = *reinterpret_cast<const f32x4*>(ck + 8 * g);
#pragma unroll
                    for (int r = 0; r < 4; ++r) S[4 * g + r] = __builtin_fmaf(S[4 * g + r], sl2, (RING == 2 ? koff : 0.f) - c4[r]);
                }
            }
            const float sl = FOX ? 1.f : sl2;
            bool slow = DIAG && kb == 0;                // first block of this wave: no reference yet
            if (!slow) {
                const float mneg = -m_run;
#pragma unroll
                for (int jj = 0; jj < 16; ++jj) {
                    E[jj] = __builtin_amdgcn_exp2f(FOX ? S[jj] + mneg : __builtin_fmaf(S[jj], sl2, mneg));
                    rs += E[jj];
                }
                slow = __builtin_amdgcn_ballot_w64(!(rs < 65536.f)) != 0;
            }
            if (slow) {
                float mloc = fmaxf(S[0], S[1]);
#pragma unroll
                for (int jj = 2; jj < 16; jj += 2) mloc = fmaxf(mloc, fmaxf(S[jj], S[jj + 1]));
                mloc = fmaxf(mloc, __shfl_xor(mloc, 32)) * sl;
                const float m_new = fmaxf(m_run, mloc);     // finite: the first block holds the diagonal
                const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
                m_run = m_new;
                l_run *= alpha;
#pragma unroll
                for (int b = 0; b < DB; ++b)
#pragma unroll
                    for (int jj = 0; jj < 16; ++jj) O[b][jj] *= alpha;
                rs = 0.f;
#pragma unroll
                for (int jj = 0; jj < 16; ++jj) {
                    E[jj] = __builtin_amdgcn_exp2f(FOX ? S[jj] - m_new : __builtin_fmaf(S[jj], sl2, -m_new));
                    rs += E[jj];
                }
            }
            l_run += rs;
            S = E;
        }
        FragV Pb[SPB];
        pack_block<TIO>(S, Pb);

        // ---- O^T += V^T P^T ------------------------------------------------------------------
#pragma unroll
        for (int b = 0; b < DB; ++b)
#pragma unroll
            for (int s = 0; s < SPB; ++s) O[b] = Tr<TIO>::mma(sV[(b * SPB + s) * 64 + lane], Pb[s], O[b]);

        if (!DIAG) {
            // ---- X <- X (I - dP) after the chunk (phase A) / after the super-block (phase B) -------
            const bool upd = kb == 1 && (j > 0 || RING) && (j >= jsb || (j % SBC) == 0);
            if (upd) {
                f32x16 Xn[DB];
#pragma unroll
                for (int b = 0; b < DB; ++b) {
                    if (HAS_MASTER) Xn[b] = Xm[b];
                    else
#pragma unroll
                        for (int jj = 0; jj < 16; ++jj) Xn[b][jj] = (float)Xh[b * SPB + jj / Tr<T>::FE][jj % Tr<T>::FE];
                }
#pragma unroll
                for (int b = 0; b < DB; ++b)
#pragma unroll
                    for (int s = 0; s < DS; ++s) Xn[b] = Tr<T>::mma(sP[(b * DS + s) * 64 + lane], Xh[s], Xn[b]);
#pragma unroll
                for (int b = 0; b < DB; ++b) {
                    if (HAS_MASTER) Xm[b] = Xn[b];
                    pack_block<T>(Xn[b], Xh + b * SPB);
                }
            }
        }
    };
    // Every wave passes the same nstage barriers: as a bystander (stages right of its own chunk: it only helps
    // with the tile copies), through its own chunk (two stages), then the steady state.
    auto top_of_stage = [&](int u) {
        wait_tiles_and_sync();            // stage u has landed; everyone is done with stage u-1
        if (u + 1 < nstage) issue_kv(u + 1);
        if ((u & 1) == 0) issue_dp(jtop - (u >> 1));
    };
    const int u0 = RING == 2 ? (active ? 0 : nstage) : (active ? 2 * (jtop - cq) : nstage);      // this wave's first stage
    issue_kv(0);
    int u = 0;
    for (; u < u0; ++u) top_of_stage(u);
    if (active) {
        if (RING != 2) {
            top_of_stage(u); stage(u, std::true_type{}); ++u;
            top_of_stage(u); stage(u, std::true_type{}); ++u;
        }
        for (; u < nstage; ++u) {
            top_of_stage(u);
            stage(u, std::false_type{});
        }
    }
    if (RING) {
        // the registers go to memory as they are (fp32): the next hop, or the final normalisation, continues from them
        if (!active) return;
#pragma unroll
        for (int b = 0; b < DB; ++b)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                f32x4 x4, o4;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int jj = 4 * g + r;
                    x4[r] = HAS_MASTER ? Xm[HAS_MASTER ? b : 0][jj] : (float)Xh[b * SPB + jj / Tr<T>::FE][jj % Tr<T>::FE];
                    o4[r] = O[b][jj];
                }
                *reinterpret_cast<f32x4*>(rec + (size_t)b * 1024 + g * 256 + lane * 4) = x4;
                *reinterpret_cast<f32x4*>(rec + (size_t)(DB + b) * 1024 + g * 256 + lane * 4) = o4;
            }
        rec[2 * DB * 1024 + lane] = m_run;
        rec[2 * DB * 1024 + 64 + lane] = l_run;
        rec[2 * DB * 1024 + 128 + lane] = (RING == 2 && FOX) ? koff : 0.f;
        return;
    }

    // ---- epilogue: normalise, store o and lse (paper Sec. 3.3, last step) ---------------------
    if (!active) return;
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    const float inv = 1.f / l_tot;
    const int tq = cq * CHUNK + 32 * qb + l32;
    if (tq < L) {
        TIO* orow = reinterpret_cast<TIO*>(p.o) + user_vec(p.ul, bh, tq) + 4 * h;
#pragma unroll
        for (int b = 0; b < DB; ++b)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                Vec4 v4;
#pragma unroll
                for (int r = 0; r < 4; ++r) v4[r] = (TIO)(O[b][4 * g + r] * inv);
                *reinterpret_cast<Vec4*>(orow + 32 * b + 8 * g) = v4;
            }
        const float ci = FOX ? p.cum[(size_t)bh * NC * CHUNK + tq] : 0.f;
        if (h == 0) p.lse[user_scl(p.ul, bh, tq)] = (m_run + __builtin_amdgcn_logf(l_tot) + ci) * 0.69314718055994530942f;
    }
}

template <typename TIO, int D, bool FOX, bool EMIT, int RING = 0>
hipError_t launch_attn_fwd2_f(const FwdParams& p, hipStream_t stream) {
    using C = Fwd2Cfg<TIO, D>;
    // set once per process; a function-local static is initialised under the language's own lock
    static const hipError_t attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_fwd2_kernel<TIO, D, FOX, EMIT, RING>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::smem_bytes);
    if (attr_err != hipSuccess) return attr_err;
    const int ntiles = ((RING == 2 ? p.NCq : p.NC) + FWD2_CPT - 1) / FWD2_CPT;
    const int BH = p.B * p.H;
    dim3 grid((unsigned)(((BH + 7) / 8) * 8 * ntiles));
    const size_t bytes = C::smem_bytes;
    hipLaunchKernelGGL((attn_fwd2_kernel<TIO, D, FOX, EMIT, RING>), grid, dim3(FWD2_THREADS), bytes, stream, p);
    return hipGetLastError();
}
template <typename TIO, int D>
hipError_t launch_attn_fwd2_t(const FwdParams& p, hipStream_t stream) {
    if (p.ring == 1) return p.cum ? launch_attn_fwd2_f<TIO, D, true, false, 1>(p, stream) : launch_attn_fwd2_f<TIO, D, false, false, 1>(p, stream);
    if (p.ring == 2) return p.cum ? launch_attn_fwd2_f<TIO, D, true, false, 2>(p, stream) : launch_attn_fwd2_f<TIO, D, false, false, 2>(p, stream);
    if (p.emit_states) return p.cum ? launch_attn_fwd2_f<TIO, D, true, true>(p, stream) : launch_attn_fwd2_f<TIO, D, false, true>(p, stream);
    return p.cum ? launch_attn_fwd2_f<TIO, D, true, false>(p, stream) : launch_attn_fwd2_f<TIO, D, false, false>(p, stream);
}

// Sequence-parallel forward, last step: o = O / l and lse = m + log l from the stored registers (the sweep's own
// epilogue, on what the last hop left).  One wave per (head, chunk, 32-query half).
template <typename TIO, int D>
__global__ __launch_bounds__(64) void ring_finish_kernel(FwdParams p) {
    using Vec4 = typename Tr<TIO>::Vec4;
    constexpr int DB = D / 32;
    const int lane = threadIdx.x, h = lane >> 5, l32 = lane & 31;
    const int cq = blockIdx.x >> 1, qb = blockIdx.x & 1, bh = blockIdx.y;
    const float* rec = p.ring_state + (((size_t)bh * p.NC + cq) * 2 + qb) * ring_rec_floats(D);
    const float m_run = rec[2 * DB * 1024 + lane], l_run = rec[2 * DB * 1024 + 64 + lane];
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    const float inv = 1.f / l_tot;
    const int tq = cq * CHUNK + 32 * qb + l32;
    if (tq >= p.L) return;
    TIO* orow = reinterpret_cast<TIO*>(p.o) + user_vec(p.ul, bh, tq) + 4 * h;
#pragma unroll
    for (int b = 0; b < DB; ++b)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const f32x4 o4 = *reinterpret_cast<const f32x4*>(rec + (size_t)(DB + b) * 1024 + g * 256 + lane * 4);
            Vec4 v4;
#pragma unroll
            for (int r = 0; r < 4; ++r) v4[r] = (TIO)(o4[r] * inv);
            *reinterpret_cast<Vec4*>(orow + 32 * b + 8 * g) = v4;
        }
    const float ci = p.cum ? p.cum[(size_t)bh * p.NC * CHUNK + tq] : 0.f;      // PaTH-FoX: the query's own gate sum, inside its segment
    if (h == 0) p.lse[user_scl(p.ul, bh, tq)] = (m_run + __builtin_amdgcn_logf(l_tot) + ci) * 0.69314718055994530942f;
}
template <typename TIO, int D>
static hipError_t launch_ring_finish_t(const FwdParams& p, hipStream_t stream) {
    hipLaunchKernelGGL((ring_finish_kernel<TIO, D>), dim3(2 * p.NC, p.B * p.H), dim3(64), 0, stream, p);
    return hipGetLastError();
}
hipError_t launch_ring_finish(const FwdParams& p, int d, int is_bf16, hipStream_t stream) {
    if (is_bf16) return d == 64 ? launch_ring_finish_t<bf16_t, 64>(p, stream) : launch_ring_finish_t<bf16_t, 128>(p, stream);
    return d == 64 ? launch_ring_finish_t<float, 64>(p, stream) : launch_ring_finish_t<float, 128>(p, stream);
}

hipError_t launch_attn_fwd2(const FwdParams& p, int d, int is_bf16, hipStream_t stream) {
    if (is_bf16) return d == 64 ? launch_attn_fwd2_t<bf16_t, 64>(p, stream) : launch_attn_fwd2_t<bf16_t, 128>(p, stream);
    return d == 64 ? launch_attn_fwd2_t<float, 64>(p, stream) : launch_attn_fwd2_t<float, 128>(p, stream);
}

}  // namespace path
