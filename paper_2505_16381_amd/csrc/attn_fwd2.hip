// Forward sweep of PaTH attention, two blocking levels (paper Sec. 3.3 workflow;
// the second level is this library's own, see prep2_fwd.hip).
//
// One workgroup = 8 waves = 256 queries = one super-block of SBC = 4 chunks; waves
// 2c and 2c+1 own the two 32-query halves of chunk 4*tile + c.  Two waves share a
// SIMD, so the vector work (softmax) of one runs under the matrix work of the other;
// each wave's working set fits the 256 architectural VGPRs (no accumulator-register
// copies).  Everything is transposed so that activations stay in registers:
//
//     S^T (64 keys x 32 q)  = Kb   X^T        A = key tile (LDS),  B = X (registers)
//     O^T (d x 32 q)       += V^T  P^T        A = V^T tile (LDS),  B = P (registers)
//     X^T (d x 32 q)       += (-dP)^T X^T     A = -dP tile (LDS),  B = X (registers)
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
// wave wv moves fragments [i*512 + 64*wv, +64) of every 512-fragment group.
constexpr int FWD2_THREADS = 512;
template <typename Frag>
__device__ __forceinline__ void async_tile(const Frag* g, Frag* s, int nfrag, int tid, int wv) {
    for (int i = 0; i < nfrag; i += FWD2_THREADS)
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(g + i + tid),
                                         (__attribute__((address_space(3))) void*)(s + i + 64 * wv), 16, 0, 0);
}

__device__ __forceinline__ void wait_tiles_and_sync() {
    __builtin_amdgcn_s_waitcnt(0x0000);   // vmcnt(0) expcnt(0) lgkmcnt(0): this wave's tile loads have landed
    __syncthreads();
}

template <typename TIO, int D, int NBUF>
__global__ __launch_bounds__(FWD2_THREADS) void attn_fwd2_kernel(FwdParams p) {
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

    const int cq = tile * SBC + (wv >> 1);          // this wave's chunk
    const int qb = wv & 1;                          // ... and which 32-query half of it
    const bool active = cq < NC;
    const int jtop = (tile * SBC + SBC - 1 < NC) ? tile * SBC + SBC - 1 : NC - 1;
    const float sl2 = p.scale * 1.44269504088896340736f;

    // ---- query state, output accumulator, softmax statistics -----------------------------------
    // The state is kept as two operand-type fragments per slab, X = Xh + Xl (Xl = what
    // rounding X to the operand type lost): Xh is the MFMA operand, and the pair restores
    // the fp32 value when the state is updated, at two thirds of the registers of an fp32
    // master plus operand copy.  (fp32 I/O: Xh is exact, Xl unused.)
    constexpr bool HAS_LO = sizeof(T) == 2;
    f32x16 O[DB];
    Frag Xh[DS], Xl[HAS_LO ? DS : 1];
    float m_run = -INFINITY, l_run = 0.f;           // m in base-2 logit units
    auto split_state = [&](int b, const f32x16& x) {
        pack_block<T>(x, Xh + b * SPB);
        if (HAS_LO) {
            f32x16 r;
#pragma unroll
            for (int jj = 0; jj < 16; ++jj) r[jj] = x[jj] - (float)Xh[b * SPB + jj / Tr<T>::FE][jj % Tr<T>::FE];
            pack_block<T>(r, Xl + b * SPB);
        }
    };
#pragma unroll
    for (int b = 0; b < DB; ++b) {
        O[b] = zero16();
        f32x16 x = zero16();
        if (active) {
            const float* xs = p.xinit + (((size_t)bh * NC + cq) * 2 + qb) * (size_t)DB * 1024 + (size_t)b * 1024;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const f32x4 v4 = *reinterpret_cast<const f32x4*>(xs + g * 256 + lane * 4);
#pragma unroll
                for (int r = 0; r < 4; ++r) x[4 * g + r] = v4[r];
            }
        }
        split_state(b, x);
    }

    const T* ktg = reinterpret_cast<const T*>(p.kt) + (size_t)bh * NC * CHUNK * D;
    const T* kt2g = reinterpret_cast<const T*>(p.kt2) + (size_t)bh * NC * CHUNK * D;
    const TIO* vtg = reinterpret_cast<const TIO*>(p.vt) + (size_t)bh * NC * CHUNK * D;
    const T* dpg = reinterpret_cast<const T*>(p.dp) + (size_t)bh * NC * D * D;
    const T* dp2g = reinterpret_cast<const T*>(p.dp2) + (size_t)bh * ntiles * D * D;

    // Online softmax of one 32-key block (raw logits S) -> P fragments.  The reference
    // maximum is only moved when the block's maximum exceeds it by more than 2^16 (so O
    // and l are rescaled practically never after the first block); probabilities may then
    // be as large as 2^16, which bf16/fp32 operands and the fp32 sums hold without loss.
    auto softmax_block = [&](f32x16& S, FragV (&Pb)[SPB]) {
        float mloc = fmaxf(S[0], S[1]);
#pragma unroll
        for (int jj = 2; jj < 16; jj += 2) mloc = fmaxf(mloc, fmaxf(S[jj], S[jj + 1]));
        mloc = fmaxf(mloc, __shfl_xor(mloc, 32)) * sl2;
        const bool move = mloc - m_run > 16.f;          // true on the first block (m_run = -inf)
        if (__builtin_amdgcn_ballot_w64(move) != 0) {
            const float m_new = move ? mloc : m_run;
            const float alpha = move ? __builtin_amdgcn_exp2f(m_run - m_new) : 1.f;
            m_run = m_new;
            l_run *= alpha;
#pragma unroll
            for (int b = 0; b < DB; ++b)
#pragma unroll
                for (int jj = 0; jj < 16; ++jj) O[b][jj] *= alpha;
        }
        const float mneg = -m_run;
        float rs = 0.f;
#pragma unroll
        for (int jj = 0; jj < 16; ++jj) {
            const float e = __builtin_amdgcn_exp2f(__builtin_fmaf(S[jj], sl2, mneg));
            S[jj] = e;
            rs += e;
        }
        l_run += rs;
        pack_block<TIO>(S, Pb);
    };
    // one key chunk: logits (or the given diagonal logits) per 32-key block, softmax, O += V^T P^T
    auto attend = [&](const Frag* sK, const FragV* sV, const float* diag) {
        f32x16 S[2];        // [key block], raw (unscaled) logits
        if (diag) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const f32x4 v4 = *reinterpret_cast<const f32x4*>(diag + (((size_t)qb * 2 + kb) * 4 + g) * 256 + lane * 4);
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int sk = 32 * kb + 8 * g + 4 * h + r, tq = 32 * qb + l32;
                        S[kb][4 * g + r] = (sk <= tq) ? v4[r] : -INFINITY;
                    }
                }
        } else {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                f32x16 a0 = zero16();
#pragma unroll
                for (int s = 0; s < DS; ++s) a0 = Tr<T>::mma(sK[(kb * DS + s) * 64 + lane], Xh[s], a0);
                S[kb] = a0;
            }
        }
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            FragV Pb[SPB];
            softmax_block(S[kb], Pb);
#pragma unroll
            for (int b = 0; b < DB; ++b)
#pragma unroll
                for (int s = 0; s < SPB; ++s) O[b] = Tr<TIO>::mma(sV[(b * CS + kb * SPB + s) * 64 + lane], Pb[s], O[b]);
        }
    };
    // X <- X (I - dP) with the -dP tile in sP
    auto update = [&]() {
        f32x16 Xn[DB];
#pragma unroll
        for (int b = 0; b < DB; ++b)
#pragma unroll
            for (int jj = 0; jj < 16; ++jj) {
                float x = (float)Xh[b * SPB + jj / Tr<T>::FE][jj % Tr<T>::FE];
                if (HAS_LO) x += (float)Xl[b * SPB + jj / Tr<T>::FE][jj % Tr<T>::FE];
                Xn[b][jj] = x;
            }
#pragma unroll
        for (int b = 0; b < DB; ++b)
#pragma unroll
            for (int s = 0; s < DS; ++s) Xn[b] = Tr<T>::mma(sP[(b * DS + s) * 64 + lane], Xh[s], Xn[b]);
#pragma unroll
        for (int b = 0; b < DB; ++b) split_state(b, Xn[b]);
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
    const float l_tot = l_run + __shfl_xor(l_run, 32);
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
                for (int r = 0; r < 4; ++r) v4[r] = (TIO)(O[b][4 * g + r] * inv);
                *reinterpret_cast<Vec4*>(orow + 32 * b + 8 * g) = v4;
            }
        if (h == 0) p.lse[(size_t)bh * L + tq] = (m_run + __builtin_amdgcn_logf(l_tot)) * 0.69314718055994530942f;
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
    hipLaunchKernelGGL((attn_fwd2_kernel<TIO, D, NBUF>), grid, dim3(FWD2_THREADS), bytes, stream, p);
    return hipGetLastError();
}

hipError_t launch_attn_fwd2(const FwdParams& p, int d, int is_bf16, hipStream_t stream) {
    if (is_bf16) return d == 64 ? launch_attn_fwd2_t<bf16_t, 64, 2>(p, stream) : launch_attn_fwd2_t<bf16_t, 128, 2>(p, stream);
    return d == 64 ? launch_attn_fwd2_t<float, 64, 2>(p, stream) : launch_attn_fwd2_t<float, 128, 1>(p, stream);
}

}  // namespace path
