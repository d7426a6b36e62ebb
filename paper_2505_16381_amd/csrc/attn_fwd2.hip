// Forward sweep of PaTH attention, two blocking levels (paper Sec. 3.3 workflow;
// the second level is this library's own, see prep2_fwd.hip).
//
// One workgroup = 256 queries = one super-block of SBC = 4 chunks; wave w owns
// chunk 4*tile + w (64 queries = two 32-column MFMA blocks, so every operand
// fragment read from LDS feeds two MFMAs).  Everything is transposed so that
// activations stay in registers:
//
//     S^T (64 keys x 64 q)  = Kb   X^T        A = key tile (LDS),  B = X (registers)
//     O^T (d x 64 q)       += V^T  P^T        A = V^T tile (LDS),  B = P (registers)
//     X^T (d x 64 q)       += (-dP)^T X^T     A = -dP tile (LDS),  B = X (registers)
//
// Phase A (inside the query tile's own super-block): chunk by chunk, with the
// chunk-level keys and one state update per chunk; the wave's own chunk uses
// the precomputed diagonal logits.  Phase B (super-blocks further left): keys
// carried to the super-block edge, ONE state update per super-block.  Tiles
// stream global -> LDS with direct-to-LDS loads, double buffered, one barrier
// per key chunk.  Workgroups are numbered so that one XCD works through the
// query tiles of one head at a time (its K/V/dP stay in that XCD's L2),
// heaviest tile first.
#include "path_common.h"

namespace path {

template <typename TIO, int D, int NBUF> struct Fwd2Cfg {
    typedef typename Compute<TIO>::type T;
    static constexpr int FE = Tr<T>::FE;
    static constexpr int KV_FRAGS = CHUNK * D / FE;     // fragments per key tile / V^T tile
    static constexpr int DP_FRAGS = D * D / FE;         // fragments per -dP tile
    static constexpr size_t smem_bytes = (size_t)(2 * NBUF * KV_FRAGS + DP_FRAGS) * 16;
};

// Linear copy of nfrag 16-byte fragments global -> LDS, asynchronous (direct-to-LDS):
// wave wv moves fragments [i*256 + 64*wv, +64) of every 256-fragment group.
template <typename Frag>
__device__ __forceinline__ void async_tile(const Frag* g, Frag* s, int nfrag, int tid, int wv) {
    for (int i = 0; i < nfrag; i += 256)
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(g + i + tid),
                                         (__attribute__((address_space(3))) void*)(s + i + 64 * wv), 16, 0, 0);
}

__device__ __forceinline__ void wait_tiles_and_sync() {
    __builtin_amdgcn_s_waitcnt(0x0000);   // vmcnt(0) expcnt(0) lgkmcnt(0): this wave's tile loads have landed
    __syncthreads();
}

template <typename TIO, int D, int NBUF>
__global__ __launch_bounds__(256) void attn_fwd2_kernel(FwdParams p) {
    using C = Fwd2Cfg<TIO, D, NBUF>;
    using T = typename C::T;
    using Frag = typename Tr<T>::Frag;
    using FragV = typename Tr<TIO>::Frag;
    using Vec4 = typename Tr<TIO>::Vec4;
    constexpr int KW = Tr<T>::KW;
    constexpr int SPB = 32 / KW, DB = D / 32, DS = D / KW, CS = CHUNK / KW;
    constexpr int KVF = C::KV_FRAGS, DPF = C::DP_FRAGS;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    Frag* sKV = reinterpret_cast<Frag*>(smem);                  // [NBUF][K tile | V tile]
    Frag* sP = sKV + 2 * NBUF * KVF;                            // -dP tile

    const int BH = p.B * p.H, L = p.L, NC = p.NC;
    const int ntiles = (NC + SBC - 1) / SBC;
    // XCD-aware numbering: workgroup b runs on XCD b % 8; that XCD takes heads xcd, xcd+8, ...
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int bh = (slot / ntiles) * 8 + xcd;
    const int tile = ntiles - 1 - slot % ntiles;
    if (bh >= BH) return;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, h = lane >> 5, l32 = lane & 31;

    const int cq = tile * SBC + wv;                 // this wave's chunk
    const bool active = cq < NC;
    const int jtop = (tile * SBC + SBC - 1 < NC) ? tile * SBC + SBC - 1 : NC - 1;
    const float sl2 = p.scale * 1.44269504088896340736f;

    // ---- query state (fp32 master + operand copy), output accumulator, softmax statistics ----
    f32x16 Xm[2][DB], O[2][DB];
    Frag Xb[2][DS];
    float m_run[2] = {-INFINITY, -INFINITY}, l_run[2] = {0.f, 0.f};
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int b = 0; b < DB; ++b) { Xm[qb][b] = zero16(); O[qb][b] = zero16(); }
    if (active) {
        const float* xs = p.xinit + ((size_t)bh * NC + cq) * 2 * (size_t)DB * 1024;
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int b = 0; b < DB; ++b)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const f32x4 v4 = *reinterpret_cast<const f32x4*>(xs + (((size_t)qb * DB + b) * 4 + g) * 256 + lane * 4);
#pragma unroll
                    for (int r = 0; r < 4; ++r) Xm[qb][b][4 * g + r] = v4[r];
                }
    }
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int b = 0; b < DB; ++b) pack_block<T>(Xm[qb][b], Xb[qb] + b * SPB);

    const T* ktg = reinterpret_cast<const T*>(p.kt) + (size_t)bh * NC * CHUNK * D;
    const T* kt2g = reinterpret_cast<const T*>(p.kt2) + (size_t)bh * NC * CHUNK * D;
    const TIO* vtg = reinterpret_cast<const TIO*>(p.vt) + (size_t)bh * NC * CHUNK * D;
    const T* dpg = reinterpret_cast<const T*>(p.dp) + (size_t)bh * NC * D * D;
    const T* dp2g = reinterpret_cast<const T*>(p.dp2) + (size_t)bh * ntiles * D * D;

    // one key chunk: logits (or the given diagonal logits), online softmax, O += V^T P^T
    auto attend = [&](const Frag* sK, const FragV* sV, const float* diag) {
        f32x16 S[2][2];     // [query block][key block]
        if (diag) {
#pragma unroll
            for (int qb = 0; qb < 2; ++qb)
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const f32x4 v4 = *reinterpret_cast<const f32x4*>(diag + (((size_t)qb * 2 + kb) * 4 + g) * 256 + lane * 4);
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            const int sk = 32 * kb + 8 * g + 4 * h + r, tq = 32 * qb + l32;
                            S[qb][kb][4 * g + r] = (sk <= tq) ? v4[r] * sl2 : -INFINITY;
                        }
                    }
        } else {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                f32x16 a0 = zero16(), a1 = zero16();
#pragma unroll
                for (int s = 0; s < DS; ++s) {
                    const Frag a = sK[(kb * DS + s) * 64 + lane];
                    a0 = Tr<T>::mma(a, Xb[0][s], a0);
                    a1 = Tr<T>::mma(a, Xb[1][s], a1);
                }
#pragma unroll
                for (int jj = 0; jj < 16; ++jj) { a0[jj] *= sl2; a1[jj] *= sl2; }
                S[0][kb] = a0; S[1][kb] = a1;
            }
        }
        FragV Pb[2][CS];
        float alpha[2];
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            float mloc = S[qb][0][0];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int jj = 0; jj < 16; ++jj) mloc = fmaxf(mloc, S[qb][kb][jj]);
            mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
            const float m_new = fmaxf(m_run[qb], mloc);      // finite: the diagonal chunk comes first
            alpha[qb] = __builtin_amdgcn_exp2f(m_run[qb] - m_new);
            float rs = 0.f;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int jj = 0; jj < 16; ++jj) {
                    const float e = __builtin_amdgcn_exp2f(S[qb][kb][jj] - m_new);
                    S[qb][kb][jj] = e;
                    rs += e;
                }
            l_run[qb] = l_run[qb] * alpha[qb] + rs;
            m_run[qb] = m_new;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) pack_block<TIO>(S[qb][kb], Pb[qb] + kb * SPB);
        }
#pragma unroll
        for (int b = 0; b < DB; ++b) {
#pragma unroll
            for (int jj = 0; jj < 16; ++jj) { O[0][b][jj] *= alpha[0]; O[1][b][jj] *= alpha[1]; }
#pragma unroll
            for (int s = 0; s < CS; ++s) {
                const FragV a = sV[(b * CS + s) * 64 + lane];
                O[0][b] = Tr<TIO>::mma(a, Pb[0][s], O[0][b]);
                O[1][b] = Tr<TIO>::mma(a, Pb[1][s], O[1][b]);
            }
        }
    };
    // X <- X (I - dP) with the -dP tile in sP
    auto update = [&]() {
#pragma unroll
        for (int b = 0; b < DB; ++b)
#pragma unroll
            for (int s = 0; s < DS; ++s) {
                const Frag a = sP[(b * DS + s) * 64 + lane];
                Xm[0][b] = Tr<T>::mma(a, Xb[0][s], Xm[0][b]);
                Xm[1][b] = Tr<T>::mma(a, Xb[1][s], Xm[1][b]);
            }
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int b = 0; b < DB; ++b) pack_block<T>(Xm[qb][b], Xb[qb] + b * SPB);
    };

    // ---- phase A: the tile's own super-block, chunk granularity -----------------------------
    for (int j = jtop; j >= tile * SBC; --j) {
        const bool need_dp = j < jtop && j > 0;       // some wave lies right of chunk j and goes on
        __syncthreads();                               // previous step's LDS reads are done
        async_tile(reinterpret_cast<const Frag*>(ktg + (size_t)j * CHUNK * D), sKV, KVF, tid, wv);
        async_tile(reinterpret_cast<const Frag*>(vtg + (size_t)j * CHUNK * D), sKV + KVF, KVF, tid, wv);
        if (need_dp) async_tile(reinterpret_cast<const Frag*>(dpg + (size_t)j * D * D), sP, DPF, tid, wv);
        wait_tiles_and_sync();
        if (!active || j > cq) continue;
        const float* diag = (j == cq) ? p.sd + ((size_t)bh * NC + j) * 4096 : nullptr;
        attend(sKV, reinterpret_cast<const FragV*>(sKV + KVF), diag);
        if (j < cq && j > 0) update();
    }

    // ---- phase B: super-blocks to the left, one state update per super-block ------------------
    // chunk sequence j = tile*SBC - 1 ... 0; buffer of chunk j is j % NBUF
    const int jfirst = tile * SBC - 1;
    if (NBUF == 2 && jfirst >= 0) {
        __syncthreads();                               // phase A's reads of buffer 0/1 and sP are done
        Frag* buf = sKV + (size_t)(jfirst & 1) * 2 * KVF;
        async_tile(reinterpret_cast<const Frag*>(kt2g + (size_t)jfirst * CHUNK * D), buf, KVF, tid, wv);
        async_tile(reinterpret_cast<const Frag*>(vtg + (size_t)jfirst * CHUNK * D), buf + KVF, KVF, tid, wv);
    }
    for (int j = jfirst; j >= 0; --j) {
        Frag* buf = sKV + (size_t)(NBUF == 2 ? (j & 1) : 0) * 2 * KVF;
        const bool sb_start = (j % SBC) == SBC - 1, sb_end = (j % SBC) == 0;
        if (NBUF == 2) {
            wait_tiles_and_sync();                     // chunk j has landed; everyone is done with chunk j+1
            if (j > 0) {
                Frag* nxt = sKV + (size_t)((j - 1) & 1) * 2 * KVF;
                async_tile(reinterpret_cast<const Frag*>(kt2g + (size_t)(j - 1) * CHUNK * D), nxt, KVF, tid, wv);
                async_tile(reinterpret_cast<const Frag*>(vtg + (size_t)(j - 1) * CHUNK * D), nxt + KVF, KVF, tid, wv);
            }
            if (sb_start && j >= SBC)                  // this super-block's product, used at its last chunk
                async_tile(reinterpret_cast<const Frag*>(dp2g + (size_t)(j / SBC) * D * D), sP, DPF, tid, wv);
        } else {
            __syncthreads();
            async_tile(reinterpret_cast<const Frag*>(kt2g + (size_t)j * CHUNK * D), buf, KVF, tid, wv);
            async_tile(reinterpret_cast<const Frag*>(vtg + (size_t)j * CHUNK * D), buf + KVF, KVF, tid, wv);
            if (sb_end && j >= SBC)
                async_tile(reinterpret_cast<const Frag*>(dp2g + (size_t)(j / SBC) * D * D), sP, DPF, tid, wv);
            wait_tiles_and_sync();
        }
        if (!active) continue;
        attend(buf, reinterpret_cast<const FragV*>(buf + KVF), nullptr);
        if (sb_end && j > 0) update();
    }

    // ---- epilogue: normalise, store o and lse (paper Sec. 3.3, last step) ---------------------
    if (!active) return;
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        const float l_tot = l_run[qb] + __shfl_xor(l_run[qb], 32);
        const float inv = 1.f / l_tot;
        const int tq = cq * CHUNK + 32 * qb + l32;
        if (tq < L) {
            TIO* orow = reinterpret_cast<TIO*>(p.o) + ((size_t)bh * L + tq) * D + 4 * h;
#pragma unroll
            for (int b = 0; b < DB; ++b)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    Vec4 v4;
#pragma unroll
                    for (int r = 0; r < 4; ++r) v4[r] = (TIO)(O[qb][b][4 * g + r] * inv);
                    *reinterpret_cast<Vec4*>(orow + 32 * b + 8 * g) = v4;
                }
            if (h == 0) p.lse[(size_t)bh * L + tq] = (m_run[qb] + __builtin_amdgcn_logf(l_tot)) * 0.69314718055994530942f;
        }
    }
}

template <typename TIO, int D, int NBUF>
hipError_t launch_attn_fwd2_t(const FwdParams& p, hipStream_t stream) {
    using C = Fwd2Cfg<TIO, D, NBUF>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_fwd2_kernel<TIO, D, NBUF>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::smem_bytes);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int ntiles = (p.NC + SBC - 1) / SBC;
    const int BH = p.B * p.H;
    dim3 grid((unsigned)(((BH + 7) / 8) * 8 * ntiles));
    const size_t bytes = C::smem_bytes;
    hipLaunchKernelGGL((attn_fwd2_kernel<TIO, D, NBUF>), grid, dim3(256), bytes, stream, p);
    return hipGetLastError();
}

hipError_t launch_attn_fwd2(const FwdParams& p, int d, int is_bf16, hipStream_t stream) {
    if (is_bf16) return d == 64 ? launch_attn_fwd2_t<bf16_t, 64, 2>(p, stream) : launch_attn_fwd2_t<bf16_t, 128, 2>(p, stream);
    return d == 64 ? launch_attn_fwd2_t<float, 64, 2>(p, stream) : launch_attn_fwd2_t<float, 128, 1>(p, stream);
}

}  // namespace path
