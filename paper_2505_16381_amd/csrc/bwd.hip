// Backward of PaTH attention.  The paper gives no backward pass; this is the
// reverse-mode derivative of the blockwise forward (Sec. 3.2-3.3), organised as
//
//   1. prep and prep2 (forward kernels, extra outputs) and a states-only sweep:
//      Xs(i,blk) = query state of chunk i as used against key block blk.  Key blocks follow the
//      forward's two blocking levels: the chunks of i's own super-block one by one ("near", keys
//      Kb, product dP_j), the super-blocks further left as a whole ("far": one state for the
//      super-block's SBC chunks, second-level keys Kb2, product dP2 = I - P_superblock).
//   2. bwd_dotile:   delta_t = dO_t . o_t, and dO as operand tiles.
//   3. bwd_adjoint2: per query chunk i, left-to-right over key chunks j:
//        dS = scale * P o (dO V_j^T - delta),   P = exp(scale * Xs Kb_j^T - lse)
//        g(i,j) = dS Kb_j + g(i,j-1) (I - dP_j)^T          (g(i,-1) = 0)
//      g(i,i-1) is the gradient of the boundary-adjusted queries Qb_i.
//   4. bwd_keyside2 / bwd_ddp: per key chunk j, over query chunks i > j (no atomics):
//        dV_j += P^T dO_i,  dKb_j += dS^T Xs(i,j),  ddP_j -= Xs(i,j)^T g(i,j-1).
//   5. adjoint of the second level (dKb2, ddP2 -> dKb, ddP) and of the chunk transform
//      (Qb, Kb, dP, Sd -> q, k, w, beta): short sequences of batched products (batched_gemm)
//      and elementwise steps, driven from the host code.
//
// Steps 3 and 4 follow the forward's scheme: activations stay in registers in
// transposed form, streamed operands are fragment-order tiles (written by prep, the
// states sweep and bwd_dotile), and the transposes that a change of contraction axis
// needs are taken through the matrix unit (product with an identity operand).
#include <type_traits>

#include "path_common.h"
#include "bwd_decl.h"

namespace path {

// ---------------------------------------------------------------------------------------
// Per query chunk: delta_t = dO_t . o_t, the row constants of the softmax, and dO as two
// fragment-order tiles (I/O type; rows past L are zero):
//   doq (rows q, contraction c)  and  doT (rows c, contraction q).
// dO is read once, in 16-byte vectors, and staged in LDS; both tiles are built from there.
template <typename TIO, int D, bool STRIDED>
__global__ __launch_bounds__(256) void bwd_dotile_kernel(BwdParams p) {
    using FragV = typename Tr<TIO>::Frag;
    constexpr int KW = Tr<TIO>::KW, SPB = 32 / KW, DB = D / 32, QS = CHUNK / KW;
    constexpr int VE = 16 / (int)sizeof(TIO), VPR = D / VE, LD = D + VE;      // vector length, vectors per row, LDS pitch
    typedef TIO Vec __attribute__((ext_vector_type(VE)));
    __shared__ __attribute__((aligned(16))) TIO sdo[CHUNK * LD];
    const int i = blockIdx.x, bh = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wv = __builtin_amdgcn_readfirstlane(tid >> 6), h = lane >> 5, l32 = lane & 31;
    const int L = seq_len(p.ul, bh, p.L), NC = p.NC;      // this head's own length; NC: chunks per head in the workspace arrays
    if (i * CHUNK >= L) return;                            // (packed batch: a shorter sequence has fewer chunks)
    const long long tok0 = user_vec(p.ul, bh, (long long)i * CHUNK);
    const TIO* dO = reinterpret_cast<const TIO*>(p.dO) + tok0;
    const TIO* O = reinterpret_cast<const TIO*>(p.o) + tok0;
    const int TS = STRIDED ? (int)p.ul.vt : D;       // token stride: a compile-time constant unless heads are interleaved
    const int nvalid = (L - i * CHUNK < CHUNK) ? L - i * CHUNK : CHUNK;
#pragma unroll
    for (int idx = tid; idx < CHUNK * VPR; idx += 256) {
        const int row = idx / VPR, v = idx % VPR;
        Vec a, b;
#pragma unroll
        for (int e = 0; e < VE; ++e) { a[e] = (TIO)0.f; b[e] = (TIO)0.f; }
        if (row < nvalid) {
            a = *reinterpret_cast<const Vec*>(dO + (size_t)row * TS + v * VE);
            b = *reinterpret_cast<const Vec*>(O + (size_t)row * TS + v * VE);
        }
        *reinterpret_cast<Vec*>(sdo + row * LD + v * VE) = a;
        float s = 0.f;
#pragma unroll
        for (int e = 0; e < VE; ++e) s += (float)a[e] * (float)b[e];
#pragma unroll
        for (int m = 1; m < VPR; m <<= 1) s += __shfl_xor(s, m);     // the VPR lanes of a row are neighbours
        if (v == 0) {
            const int tg = i * CHUNK + row;
            p.delta[(size_t)bh * NC * CHUNK + tg] = s;
            // log-sum-exp in base-2 units; with gates (PaTH-FoX) minus the query's own gate sum, so that
            // P = exp2(scale2 * s - c_key - lse2p)
            p.lse2p[(size_t)bh * NC * CHUNK + tg] = (row < nvalid) ? p.lse[user_scl(p.ul, bh, tg)] * 1.44269504088896340736f - (p.cum ? p.cum[(size_t)bh * NC * CHUNK + tg] : 0.f) : 3.0e38f;      // rows past L: P = exp2(-huge) = 0
        }
    }
    __syncthreads();
    FragV* dq = reinterpret_cast<FragV*>(reinterpret_cast<TIO*>(p.doq) + ((size_t)bh * NC + i) * CHUNK * D);
    FragV* dt = reinterpret_cast<FragV*>(reinterpret_cast<TIO*>(p.doT) + ((size_t)bh * NC + i) * CHUNK * D);
    for (int blk = wv; blk < 2 * DB; blk += 4) {
        const int cb = blk >> 1, qb = blk & 1;
        f32x16 a, b;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            a[j] = (float)sdo[(32 * qb + l32) * LD + 32 * cb + acc_row(j, h)];      // registers rows c, lane q
            b[j] = (float)sdo[(32 * qb + acc_row(j, h)) * LD + 32 * cb + l32];      // registers rows q, lane c
        }
        FragV fa[SPB], fb[SPB];
        pack_block<TIO>(a, fa);
        pack_block<TIO>(b, fb);
#pragma unroll
        for (int s = 0; s < SPB; ++s) {
            __builtin_nontemporal_store(fa[s], &dq[((size_t)qb * (D / KW) + cb * SPB + s) * 64 + lane]);
            __builtin_nontemporal_store(fb[s], &dt[((size_t)cb * QS + qb * SPB + s) * 64 + lane]);
        }
    }
}

// ---------------------------------------------------------------------------------------
// Adjoint scan.  One workgroup = 4 waves = two query chunks; wave w owns the 32-query half
// (w & 1) of chunk 2*tile + (w >> 1), exactly as in the states sweep.  Everything is transposed
// (wave = 32 queries = the MFMA columns), so the adjoint state g^T (rows c, lane q) stays in
// registers across the key chunks j = 0 .. cq-1:
//     S^T  = Kb_j Xs^T            A = kt tile,   B = Xs fragments (loaded per pair)
//     dP^T = V_j dO^T             A = vk tile,   B = dO fragments (resident)
//     dS^T = scale * P o (dP^T - delta),   P = exp(scale S^T - lse)
//     g^T <- g^T + Kb_j^T dS^T - dP_j g^T      A = ktT tile / dpt tile,  B = dS^T / g^T (registers)
// After step j the state is also written, transposed through the matrix unit, as the tile
// gT (rows b, contraction q) of pair (cq, j+1) for the key-side kernels.
// This kernel runs fp32 operands (one workgroup per CU, one stage of tiles); 16-bit operands use
// bwd_adjoint2_lite_kernel below (two workgroups per CU).
template <typename TIO, int D> struct Adj2Cfg {
    typedef typename Compute<TIO>::type T;
    static constexpr int FE = Tr<T>::FE;
    static constexpr int KV_FRAGS = CHUNK * D / FE, DP_FRAGS = D * D / FE;
    static constexpr int NBUF = (sizeof(T) == 2) ? 2 : 1;
    static constexpr int STAGE_FRAGS = 3 * KV_FRAGS + DP_FRAGS;                    // kt | vk | ktT | dpt
    static constexpr size_t smem_bytes = (size_t)NBUF * STAGE_FRAGS * 16;
};

template <typename TIO, int D, bool FOX>
__global__ __launch_bounds__(256) void bwd_adjoint2_kernel(BwdParams p) {
    using C = Adj2Cfg<TIO, D>;
    using T = typename C::T;
    using Frag = typename Tr<T>::Frag;
    using FragV = typename Tr<TIO>::Frag;
    constexpr int KW = Tr<T>::KW, SPB = 32 / KW, DB = D / 32, DS = D / KW, QS = CHUNK / KW;
    constexpr int KVF = C::KV_FRAGS, DPF = C::DP_FRAGS;

    constexpr int NBUF = C::NBUF, STF = C::STAGE_FRAGS;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    Frag* sbase = reinterpret_cast<Frag*>(smem);

    const int BH = p.B * p.H, NC = p.NC;
    const int ntiles = (NC + 1) / 2;
    // XCD-aware numbering: workgroup n runs on XCD n % 8; that XCD takes heads xcd, xcd+8, ... one
    // after the other, all tiles of a head together (heaviest first).  They walk the key chunks
    // from 0 upwards at the same pace, so each tile is fetched once per head into that XCD's L2.
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int bh = __builtin_amdgcn_readfirstlane((slot / ntiles) * 8 + xcd);        // (divisions run on the vector unit:
    const int tile = __builtin_amdgcn_readfirstlane(ntiles - 1 - slot % ntiles);     // back to scalar registers)
    if (bh >= BH) return;
    const int tid = threadIdx.x, lane = tid & 63, wv = __builtin_amdgcn_readfirstlane(tid >> 6), h = lane >> 5, l32 = lane & 31;
    const int NCo = (seq_len(p.ul, bh, p.L) + CHUNK - 1) / CHUNK;          // this head's own chunks (NC: per head in the workspace arrays)
    if (tile * 2 >= NCo) return;
    const int cq = tile * 2 + (wv >> 1), qb = wv & 1;
    const bool active = cq < NCo;
    const int jmax = ((tile * 2 + 1 < NCo) ? tile * 2 + 1 : NCo - 1) - 1;   // last key chunk any wave needs
    const int jsb = (tile * 2 / SBC) * SBC;                                // first chunk of the tile's own super-block
    const size_t Lp = (size_t)NC * CHUNK, nslots = num_block_slots(NC);
    const float sl2 = p.scale * 1.44269504088896340736f;
    const int tq = cq * CHUNK + 32 * qb + l32;                             // this lane's query

    // resident: dO fragments of the wave's 32 queries, lse and delta of the lane's query
    FragV dOb[DS];
    float lse2 = 0.f, dl = 0.f;
    float drow = 0.f;       // PaTH-FoX: this query's row sum of the logit gradient (off-diagonal part)
    if (active) {
        const FragV* dq = reinterpret_cast<const FragV*>(reinterpret_cast<const TIO*>(p.doq) + ((size_t)bh * NC + cq) * CHUNK * D);
#pragma unroll
        for (int s = 0; s < DS; ++s) dOb[s] = dq[((size_t)qb * DS + s) * 64 + lane];
        // base-2 units (PaTH-FoX: minus the query's gate sum); rows past L hold a huge value, so that their
        // P = exp2(-huge) = 0 without a mask.  log2(scale) is folded in: the exponential then yields scale * P,
        // which is all the logit gradient dS = scale * P o (dP - delta) needs.
        lse2 = p.lse2p[(size_t)bh * Lp + tq] - __builtin_log2f(p.scale);
        dl = p.delta[(size_t)bh * Lp + tq];
    }
    f32x16 Gm[DB];
    Frag Gb[DS];
#pragma unroll
    for (int b = 0; b < DB; ++b) { Gm[b] = zero16(); pack_block<T>(Gm[b], Gb + b * SPB); }
    Frag idf[SPB];
    identity_frags<T>(idf, l32, h);

    // Step j handles key chunk j: far (j < jsb: second-level keys, state and product of its
    // super-block) or near (chunk-level keys, state and product of the chunk).
    const int nsb = (NC + SBC - 1) / SBC;
    // The four tiles of chunk j are requested in four parts (part = -1: all at once).  With two
    // stage buffers the parts of the NEXT chunk are spread over the current chunk's work: the
    // direct-to-LDS path takes about 32 B/clk per CU, and a wave that issues a whole stage at
    // once sits in the issue queue for that long.
    auto issue = [&](int j, int part) {
        Frag* buf = sbase + (size_t)(j & (NBUF - 1)) * STF;
        const size_t bhc = (size_t)bh * NC + j;
        const bool far = j < jsb;
        if (part < 0 || part == 0)
            async_copy_tile<256, KVF>(reinterpret_cast<const Frag*>(reinterpret_cast<const T*>(far ? p.kt2 : p.kt) + bhc * CHUNK * D), buf, tid, wv);
        if (part < 0 || part == 1)
            async_copy_tile<256, KVF>(reinterpret_cast<const Frag*>(reinterpret_cast<const TIO*>(p.vk) + bhc * CHUNK * D), buf + KVF, tid, wv);
        if (part < 0 || part == 2)
            async_copy_tile<256, KVF>(reinterpret_cast<const Frag*>(reinterpret_cast<const T*>(far ? p.kt2T : p.ktT) + bhc * CHUNK * D), buf + 2 * KVF, tid, wv);
        if ((part < 0 || part == 3) && j > 0) {
            if (!far)
                async_copy_tile<256, DPF>(reinterpret_cast<const Frag*>(reinterpret_cast<const T*>(p.dpt) + bhc * (size_t)D * D), buf + 3 * KVF, tid, wv);
            else if (j % SBC == 0)
                async_copy_tile<256, DPF>(reinterpret_cast<const Frag*>(reinterpret_cast<const T*>(p.dpt2) + ((size_t)bh * nsb + j / SBC) * (size_t)D * D), buf + 3 * KVF, tid, wv);
        }
    };
    auto block_start = [&](int j) { return j >= jsb || j % SBC == 0; };
    // the wave's own state fragments of the block that starts at chunk j: fetched one step ahead
    auto load_x = [&](int j, Frag* x) {
        const size_t slot = ((size_t)bh * nslots + block_slot(cq, j, NC)) * (size_t)CHUNK * D;
        const Frag* xg = reinterpret_cast<const Frag*>(reinterpret_cast<const T*>(p.xs) + slot);
#pragma unroll
        for (int s = 0; s < DS; ++s) x[s] = __builtin_nontemporal_load(&xg[((size_t)qb * DS + s) * 64 + lane]);     // read once: leave L2 to the key tiles
    };
    Frag Xnext[DS], Xb[DS];
#pragma unroll
    for (int s = 0; s < DS; ++s) { Xnext[s] = Tr<T>::zero(); Xb[s] = Tr<T>::zero(); }
    if (active && cq > 0) load_x(0, Xnext);
    if (jmax >= 0 && NBUF == 2) issue(0, -1);

    for (int j = 0; j <= jmax; ++j) {
        const bool spread = NBUF == 2 && j + 1 <= jmax;     // request chunk j+1 while working on chunk j
        if (NBUF == 2) {
            wait_async_and_sync();                 // chunk j has landed; everyone is done with chunk j-1
            if (spread) issue(j + 1, 0);
        } else {
            __syncthreads();
            issue(j, -1);
            wait_async_and_sync();
        }
        if (!active || j >= cq) {
            if (spread) { issue(j + 1, 1); issue(j + 1, 2); issue(j + 1, 3); }
            continue;
        }
        const Frag* sK = sbase + (size_t)(j & (NBUF - 1)) * STF;
        const FragV* sV = reinterpret_cast<const FragV*>(sK + KVF);
        const Frag* sKT = sK + 2 * KVF;
        const Frag* sDP = sK + 3 * KVF;

        const bool first = block_start(j);          // first chunk of its block: new state, product applied to g
        if (first) {
#pragma unroll
            for (int s = 0; s < DS; ++s) Xb[s] = Xnext[s];
        }
        const bool next_starts = j + 1 < cq && block_start(j + 1);
        if (next_starts) load_x(j + 1, Xnext);

        Frag dSb[QS];
        {
    #pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                f32x16 S = zero16(), dP = zero16();
                // operand fragments are fetched in batches ahead of the products that use them
    #pragma unroll
                for (int s0 = 0; s0 < DS; s0 += 4) {
                    Frag ka[4];
                    FragV va[4];
    #pragma unroll
                    for (int u = 0; u < 4; ++u) { ka[u] = sK[(kb * DS + s0 + u) * 64 + lane]; va[u] = sV[(kb * DS + s0 + u) * 64 + lane]; }
    #pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        S = Tr<T>::mma(ka[u], Xb[s0 + u], S);
                        dP = Tr<TIO>::mma(va[u], dOb[s0 + u], dP);
                    }
                }
                f32x4 ck4[4];
                if (FOX) {      // gate sums of the 16 keys this lane holds (rows 8g + 4h + r of the 32-key block)
                    const float* ck = p.cum + (size_t)bh * Lp + (size_t)j * CHUNK + 32 * kb + 4 * h;
    #pragma unroll
                    for (int g = 0; g < 4; ++g) ck4[g] = *reinterpret_cast<const f32x4*>(ck + 8 * g);
                }
    #pragma unroll
                for (int jj = 0; jj < 16; ++jj) {
                    const float arg = __builtin_fmaf(S[jj], sl2, -lse2) - (FOX ? ck4[jj >> 2][jj & 3] : 0.f);
                    const float ds = __builtin_amdgcn_exp2f(arg) * (dP[jj] - dl);      // scale * P * (dP - delta)
                    if (FOX) drow += ds;
                    S[jj] = ds;
                }
                pack_block<T>(S, dSb + kb * SPB);
                if (spread) issue(j + 1, 1 + kb);
            }
            if (spread) issue(j + 1, 3);
    #pragma unroll
            for (int b = 0; b < DB; b += 2) {
                Frag ta[2 * QS];
    #pragma unroll
                for (int u = 0; u < 2 * QS; ++u) ta[u] = sKT[((b + u / QS) * QS + u % QS) * 64 + lane];
    #pragma unroll
                for (int u = 0; u < 2 * QS; ++u) Gm[b + u / QS] = Tr<T>::mma(ta[u], dSb[u % QS], Gm[b + u / QS]);
            }
        }
        if (j > 0 && first) {
#pragma unroll
            for (int b = 0; b < DB; ++b)
#pragma unroll
                for (int s0 = 0; s0 < DS; s0 += 8) {
                    constexpr int NB8 = DS < 8 ? DS : 8;
                    Frag pa[NB8];
#pragma unroll
                    for (int u = 0; u < NB8; ++u) pa[u] = sDP[(b * DS + s0 + u) * 64 + lane];
#pragma unroll
                    for (int u = 0; u < NB8; ++u) Gm[b] = Tr<T>::mma(pa[u], Gb[s0 + u], Gm[b]);
                }
        }
        if (next_starts) {     // g after this block: operand copy for the next block's product, and
                               // tile gT (rows b, contraction q) of the pair (cq, next block)
#pragma unroll
            for (int b = 0; b < DB; ++b) pack_block<T>(Gm[b], Gb + b * SPB);
            const size_t slot2 = ((size_t)bh * nslots + block_slot(cq, j + 1, NC)) * (size_t)CHUNK * D;
            Frag* gt = reinterpret_cast<Frag*>(reinterpret_cast<T*>(p.gs) + slot2);
#pragma unroll
            for (int b = 0; b < DB; ++b) {
                const f32x16 tr = transpose32<T>(Gb + b * SPB, idf);       // rows q, lane b
                Frag fr[SPB];
                pack_block<T>(tr, fr);
#pragma unroll
                for (int s2 = 0; s2 < SPB; ++s2) __builtin_nontemporal_store(fr[s2], &gt[((size_t)b * QS + qb * SPB + s2) * 64 + lane]);   // streamed: the key tiles stay in L2
            }
        }
    }
    if (FOX && active) {    // the two half-waves hold different keys of the same query
        drow += __shfl_xor(drow, 32);
        if (h == 0) p.drow[(size_t)bh * Lp + tq] = drow / p.scale;      // the sums above carry the factor scale
    }
    // dQb of the wave's queries: row-major fp32 [q][c] from registers (rows c, lane q)
    if (active) {
        float* dst = p.dqb + ((size_t)bh * Lp + tq) * D + 4 * h;
#pragma unroll
        for (int b = 0; b < DB; ++b)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                f32x4 v4;
#pragma unroll
                for (int r = 0; r < 4; ++r) v4[r] = Gm[b][4 * g + r];
                *reinterpret_cast<f32x4*>(dst + 32 * b + 8 * g) = v4;
            }
    }
}

// ---------------------------------------------------------------------------------------
// Fragment of the TRANSPOSE of a fragment-order tile (rows q in 32-row halves of DS slabs,
// contraction c).  Element e of a fragment belongs to contraction index 16 s + acc_row(e, h) of
// its slab s, in both tiles, so the lane needs tile[q = 16 qs + acc_row(e, h)][c = 32 b + l32],
// e = 0..7: two transposing reads, of rows 16 qs + 4 h + 0..3 and the same + 8 (in each block of
// 16 lanes, lane i points at 4 consecutive c of row .. + i/4 and receives column i of the four rows).
template <typename E, int DS>
__device__ __forceinline__ typename Tr<E>::Frag ld_tile_frag_tr(const E* tile, int qs, int b, int l32, int h) {
    static_assert(sizeof(E) == 2, "16-bit transposing reads");
    typedef short v4s __attribute__((ext_vector_type(4)));
    const int i = l32 & 15;
    const E* p = tile + (size_t)((((qs >> 1) * DS + 2 * b + (l32 >> 4)) * 64 + (i & 1) * 32 + 16 * (qs & 1) + 4 * h + (i >> 2)) * 8 + 4 * ((i >> 1) & 1));
    union { v4s v[2]; typename Tr<E>::Frag f; } u;
    u.v[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s*)(p));
    u.v[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s*)(p + 64));
    return u.f;
}

// ---------------------------------------------------------------------------------------
// The adjoint scan for 16-bit operands with TWO workgroups per CU: the same arithmetic as
// bwd_adjoint2_kernel, arranged to fit 256 registers per wave and one 80 KB stage per workgroup, so that
// the second workgroup's waves fill the gaps of the first (tile requests, LDS latencies, the dependent
// chain logits -> exponentials -> update) instead of hand-interleaved halves of one wave.  Per step: one
// request for the chunk's four tiles, no prefetch; the state fragments of a new block are fetched while
// those tiles are on their way; the operand copy of g exists only while a block boundary needs it.
// The fragments of Kb^T for g^T += Kb^T dS^T are read out of the key tile itself with transposing LDS reads
// (three tiles per step instead of four: the transposed key tiles are neither written nor copied; as a fourth
// tile they cost 4 % of this kernel), and likewise the fragments of -dP in the arrangement (rows a, contraction b)
// out of the forward's tile (rows b, contraction a): p.dpt / p.dpt2 point at the FORWARD's tiles here.  No copy is in
// flight while a step computes, so those reads wait for nothing.
template <typename TIO, int D, bool FOX>
__global__ __launch_bounds__(256, 2) void bwd_adjoint2_lite_kernel(BwdParams p) {
    using C = Adj2Cfg<TIO, D>;
    using T = typename C::T;
    using Frag = typename Tr<T>::Frag;
    using FragV = typename Tr<TIO>::Frag;
    static_assert(sizeof(T) == 2, "16-bit operands");
    constexpr int KW = Tr<T>::KW, SPB = 32 / KW, DB = D / 32, DS = D / KW, QS = CHUNK / KW;
    constexpr int KVF = C::KV_FRAGS, DPF = C::DP_FRAGS;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    Frag* sK = reinterpret_cast<Frag*>(smem);
    const FragV* sV = reinterpret_cast<const FragV*>(sK + KVF);
    const Frag* sDP = sK + 2 * KVF;

    const int BH = p.B * p.H, NC = p.NC;
    const int ntiles = (NC + 1) / 2;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;        // numbering as in bwd_adjoint2_kernel
    const int bh = __builtin_amdgcn_readfirstlane((slot / ntiles) * 8 + xcd);        // (divisions run on the vector unit:
    const int tile = __builtin_amdgcn_readfirstlane(ntiles - 1 - slot % ntiles);     // back to scalar registers)
    if (bh >= BH) return;
    const int tid = threadIdx.x, lane = tid & 63, wv = __builtin_amdgcn_readfirstlane(tid >> 6), h = lane >> 5, l32 = lane & 31;
    const int NCo = (seq_len(p.ul, bh, p.L) + CHUNK - 1) / CHUNK;          // this head's own chunks (NC: per head in the workspace arrays)
    if (tile * 2 >= NCo) return;
    const int cq = tile * 2 + (wv >> 1), qb = wv & 1;
    const bool active = cq < NCo;
    const int jmax = ((tile * 2 + 1 < NCo) ? tile * 2 + 1 : NCo - 1) - 1;
    const int jsb = (tile * 2 / SBC) * SBC;
    const size_t Lp = (size_t)NC * CHUNK, nslots = num_block_slots(NC);
    const float sl2 = p.scale * 1.44269504088896340736f;
    const int tq = cq * CHUNK + 32 * qb + l32;
    const int nsb = (NC + SBC - 1) / SBC;

    FragV dOb[DS];
    float lse2 = 0.f, dl = 0.f, drow = 0.f;
    if (active) {
        const FragV* dq = reinterpret_cast<const FragV*>(reinterpret_cast<const TIO*>(p.doq) + ((size_t)bh * NC + cq) * CHUNK * D);
#pragma unroll
        for (int s = 0; s < DS; ++s) dOb[s] = dq[((size_t)qb * DS + s) * 64 + lane];
        lse2 = p.lse2p[(size_t)bh * Lp + tq] - __builtin_log2f(p.scale);     // the exponential then yields scale * P
        dl = p.delta[(size_t)bh * Lp + tq];
    }
    f32x16 Gm[DB];
    Frag Xb[DS];
#pragma unroll
    for (int b = 0; b < DB; ++b) Gm[b] = zero16();
#pragma unroll
    for (int s = 0; s < DS; ++s) Xb[s] = Tr<T>::zero();
    auto block_start = [&](int j) { return j >= jsb || j % SBC == 0; };

    for (int j = 0; j <= jmax; ++j) {
        const bool far = j < jsb;
        const bool mine = active && j < cq;
        const bool first = block_start(j);
        __syncthreads();                           // everyone is done with the previous chunk's tiles
        {
            const size_t bhc = (size_t)bh * NC + j;
            async_copy_tile<256, KVF>(reinterpret_cast<const Frag*>(reinterpret_cast<const T*>(far ? p.kt2 : p.kt) + bhc * CHUNK * D), sK, tid, wv);
            async_copy_tile<256, KVF>(reinterpret_cast<const Frag*>(reinterpret_cast<const TIO*>(p.vk) + bhc * CHUNK * D), sK + KVF, tid, wv);
            if (j > 0 && first) {
                const T* src = far ? reinterpret_cast<const T*>(p.dpt2) + ((size_t)bh * nsb + j / SBC) * (size_t)D * D
                                   : reinterpret_cast<const T*>(p.dpt) + bhc * (size_t)D * D;
                async_copy_tile<256, DPF>(reinterpret_cast<const Frag*>(src), sK + 2 * KVF, tid, wv);
            }
        }
        if (mine && first) {                       // the state of the block that starts here
            const size_t xslot = ((size_t)bh * nslots + block_slot(cq, j, NC)) * (size_t)CHUNK * D;
            const Frag* xg = reinterpret_cast<const Frag*>(reinterpret_cast<const T*>(p.xs) + xslot);
#pragma unroll
            for (int s = 0; s < DS; ++s) Xb[s] = __builtin_nontemporal_load(&xg[((size_t)qb * DS + s) * 64 + lane]);
        }
        wait_async_and_sync();
        if (!mine) continue;

        if (j > 0 && first) {                      // g <- g (I - dP_blk)^T: the product with the state before this step
            Frag Gb[DS];
#pragma unroll
            for (int b = 0; b < DB; ++b) pack_block<T>(Gm[b], Gb + b * SPB);
#pragma unroll
            for (int b = 0; b < DB; ++b)
#pragma unroll
                for (int s0 = 0; s0 < DS; s0 += 4) {
                    Frag pa[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) pa[u] = ld_tile_frag_tr<T, DS>(reinterpret_cast<const T*>(sDP), s0 + u, b, l32, h);
#pragma unroll
                    for (int u = 0; u < 4; ++u) Gm[b] = Tr<T>::mma(pa[u], Gb[s0 + u], Gm[b]);
                }
        }
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            f32x16 S = zero16(), dP = zero16();
#pragma unroll
            for (int s0 = 0; s0 < DS; s0 += 2) {
                Frag ka[2];
                FragV va[2];
#pragma unroll
                for (int u = 0; u < 2; ++u) { ka[u] = sK[(kb * DS + s0 + u) * 64 + lane]; va[u] = sV[(kb * DS + s0 + u) * 64 + lane]; }
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    S = Tr<T>::mma(ka[u], Xb[s0 + u], S);
                    dP = Tr<TIO>::mma(va[u], dOb[s0 + u], dP);
                }
            }
            f32x4 ck4[4];
            if (FOX) {      // gate sums of the 16 keys this lane holds (rows 8g + 4h + r of the 32-key block)
                const float* ck = p.cum + (size_t)bh * Lp + (size_t)j * CHUNK + 32 * kb + 4 * h;
#pragma unroll
                for (int g = 0; g < 4; ++g) ck4[g] = *reinterpret_cast<const f32x4*>(ck + 8 * g);
            }
#pragma unroll
            for (int jj = 0; jj < 16; ++jj) {
                const float arg = __builtin_fmaf(S[jj], sl2, -lse2) - (FOX ? ck4[jj >> 2][jj & 3] : 0.f);
                const float ds = __builtin_amdgcn_exp2f(arg) * (dP[jj] - dl);      // scale * P * (dP - delta)
                if (FOX) drow += ds;
                S[jj] = ds;
            }
            Frag dSh[SPB];
            pack_block<T>(S, dSh);
            // g^T += Kb^T dS^T, the 32 keys of this half
#pragma unroll
            for (int b = 0; b < DB; ++b) {
                Frag ta[SPB];
#pragma unroll
                for (int u = 0; u < SPB; ++u) ta[u] = ld_tile_frag_tr<T, DS>(reinterpret_cast<const T*>(sK), kb * SPB + u, b, l32, h);
#pragma unroll
                for (int u = 0; u < SPB; ++u) Gm[b] = Tr<T>::mma(ta[u], dSh[u], Gm[b]);
            }
        }
        if (j + 1 < cq && block_start(j + 1)) {    // g after this block: tile gT (rows b, contraction q) of the pair (cq, next block)
            Frag idf[SPB];
            identity_frags<T>(idf, l32, h);
            const size_t slot2 = ((size_t)bh * nslots + block_slot(cq, j + 1, NC)) * (size_t)CHUNK * D;
            Frag* gt = reinterpret_cast<Frag*>(reinterpret_cast<T*>(p.gs) + slot2);
#pragma unroll
            for (int b = 0; b < DB; ++b) {
                Frag gb[SPB];
                pack_block<T>(Gm[b], gb);
                const f32x16 tr = transpose32<T>(gb, idf);       // rows q, lane b
                Frag fr[SPB];
                pack_block<T>(tr, fr);
#pragma unroll
                for (int s2 = 0; s2 < SPB; ++s2) __builtin_nontemporal_store(fr[s2], &gt[((size_t)b * QS + qb * SPB + s2) * 64 + lane]);
            }
        }
    }
    if (FOX && active) {
        drow += __shfl_xor(drow, 32);
        if (h == 0) p.drow[(size_t)bh * Lp + tq] = drow / p.scale;
    }
    if (active) {
        float* dst = p.dqb + ((size_t)bh * Lp + tq) * D + 4 * h;
#pragma unroll
        for (int b = 0; b < DB; ++b)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                f32x4 v4;
#pragma unroll
                for (int r = 0; r < 4; ++r) v4[r] = Gm[b][4 * g + r];
                *reinterpret_cast<f32x4*>(dst + 32 * b + 8 * g) = v4;
            }
    }
}

// ---------------------------------------------------------------------------------------
// Key-side reduction of dV and dKb.  One workgroup per key chunk j; wave w owns the 32 keys of
// half (w & 1) (= the MFMA columns) and the 32-query half (w >> 1) of every query chunk i > j
// of the kernel's range -- near (FAR = false): the chunks i > j of j's own super-block, keys Kb,
// results dKb and dV; far (FAR = true): all chunks of the super-blocks to the right, keys Kb2,
// results dKb2 and dV added to the near part (the near kernel runs first):
//     S  = Xs Kb_j^T              A = xs tile,   B = Kb fragments (resident)
//     dP = dO V_j^T               A = doq tile,  B = V fragments (resident)
//     dV^T  += dO^T P             A = doT tile,  B = P   (registers)
//     dKb^T += Xs^T dS            A = xsT tile,  B = dS  (registers)
// The two query halves are summed through LDS at the end (no atomics).
//
// With 16-bit operands the near kernel also takes the near part of ddP_j (see bwd_ddp_kernel):
//     ddP_j -= Xs^T g               A = xsT tile,  B = gT tile
// over the same pairs (i, j), whose xsT tile it has staged anyway.  The gT tile takes the LDS
// space of the doT tile; the dO^T fragments are then read out of the doq tile with the
// transposing LDS read.
//
template <typename TIO, int D> struct Key2Cfg {
    typedef typename Compute<TIO>::type T;
    static constexpr int FE = Tr<T>::FE;
    static constexpr int KV_FRAGS = CHUNK * D / FE;
    static constexpr int NBUF = (sizeof(T) == 2) ? 2 : 1;                     // fp32 tiles are too big to double-buffer
    static constexpr int STAGE_FRAGS = 4 * KV_FRAGS + 32;                     // xs | xsT | doq | doT (near, 16-bit: gT) | lse2 | delta
    static constexpr size_t tile_bytes = (size_t)NBUF * STAGE_FRAGS * 16;
    static constexpr size_t red_bytes = (size_t)2 * 2 * (D / 32) * 1024 * 4 + 256;   // dV, dKb (and FOX column sums) of the two upper waves
    static constexpr size_t smem_bytes = tile_bytes > red_bytes ? tile_bytes : red_bytes;
};

template <typename TIO, int D, bool FAR, bool FOX>
__global__ __launch_bounds__(256) void bwd_keyside2_kernel(BwdParams p) {
    using C = Key2Cfg<TIO, D>;
    using T = typename C::T;
    using Frag = typename Tr<T>::Frag;
    using FragV = typename Tr<TIO>::Frag;
    constexpr int KW = Tr<T>::KW, SPB = 32 / KW, DB = D / 32, DS = D / KW, QS = CHUNK / KW;
    constexpr int KVF = C::KV_FRAGS, NBUF = C::NBUF, STF = C::STAGE_FRAGS;
    constexpr bool NFUSE = !FAR && sizeof(T) == 2;          // the near part of ddP is taken here too
    constexpr int NOWN = NFUSE ? DB * DB / 4 : 1;           // its 32x32 blocks per wave

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    Frag* sbase = reinterpret_cast<Frag*>(smem);

    // Workgroup numbering (1-D grid): workgroup n runs on XCD n % 8.  XCD x takes the heads
    // bh = x (mod 8), and the workgroups of one super-block get consecutive numbers on it:
    // they stream the same far states and dO tiles at the same time, out of that XCD's L2.
    // Super-blocks with the most query chunks to their right come first.
    // Near: one key chunk per workgroup, wave w = key half (w & 1) x query half (w >> 1).
    // Far: TWO key chunks per workgroup (they share every staged tile), wave w = key half (w & 1)
    // of chunk j + (w >> 1), both query halves in turn.
    constexpr int CPW = FAR ? 2 : 1, NPOS = SBC / CPW;
    const int NC = p.NC;                                        // chunks per head in the workspace arrays and the grid's numbering
    const int nsb_g = (NC + SBC - 1) / SBC;
    const int xcd = blockIdx.x & 7, kk = blockIdx.x >> 3;
    // (the divisions run on the vector unit; their results go back to scalar registers)
    const int j = __builtin_amdgcn_readfirstlane((kk / NPOS % nsb_g) * SBC + (kk % NPOS) * CPW);       // first key chunk of the workgroup
    const int bh = __builtin_amdgcn_readfirstlane((kk / (NPOS * nsb_g)) * 8 + xcd);
    if (bh >= p.B * p.H) return;
    const int NCo = (seq_len(p.ul, bh, p.L) + CHUNK - 1) / CHUNK;      // this head's own chunks
    if (j >= NCo) return;
    const int tid = threadIdx.x, lane = tid & 63, wv = __builtin_amdgcn_readfirstlane(tid >> 6), h = lane >> 5, l32 = lane & 31;
    const int kh = wv & 1;
    const int jw = FAR ? j + (wv >> 1) : j;                            // this wave's key chunk
    const bool wactive = jw < NCo;
    const size_t Lp = (size_t)NC * CHUNK, nslots = num_block_slots(NC);
    const float sl2 = p.scale * 1.44269504088896340736f;
    const int sb_end = (j / SBC + 1) * SBC;                       // first chunk right of j's super-block
    const int i0 = FAR ? sb_end : j + 1;
    const int i1 = FAR ? NCo : (sb_end < NCo ? sb_end : NCo);

    Frag Kb[DS];
    FragV Vb[DS];
    {
        const int jl = wactive ? jw : j;
        const Frag* kg = reinterpret_cast<const Frag*>(reinterpret_cast<const T*>(FAR ? p.kt2 : p.kt) + ((size_t)bh * NC + jl) * CHUNK * D);
        const FragV* vg = reinterpret_cast<const FragV*>(reinterpret_cast<const TIO*>(p.vk) + ((size_t)bh * NC + jl) * CHUNK * D);
#pragma unroll
        for (int s = 0; s < DS; ++s) { Kb[s] = kg[((size_t)kh * DS + s) * 64 + lane]; Vb[s] = vg[((size_t)kh * DS + s) * 64 + lane]; }
    }
    f32x16 dVt[DB], dKt[DB];
#pragma unroll
    for (int b = 0; b < DB; ++b) { dVt[b] = zero16(); dKt[b] = zero16(); }
    f32x16 ddPa[NOWN];
#pragma unroll
    for (int o = 0; o < NOWN; ++o) ddPa[o] = zero16();
    // PaTH-FoX: this lane's key has gate sum ckj; dcol collects the column sum of the logit gradient
    const int key_tok = (wactive ? jw : j) * CHUNK + 32 * kh + l32;
    const float ckj = FOX ? p.cum[(size_t)bh * Lp + key_tok] : 0.f;
    float dcol = 0.f;

    // all operands of query chunk i, asynchronously, into stage buffer (i & (NBUF-1))
    // part = -1: everything; 0..3: one tile each (the requests for the next chunk are spread over
    // the current chunk's work, see the adjoint scan)
    auto issue = [&](int i, int part) {
        Frag* buf = sbase + (size_t)(i & (NBUF - 1)) * STF;
        const size_t slot = ((size_t)bh * nslots + block_slot(i, j, NC)) * (size_t)CHUNK * D;
        const size_t bhi = ((size_t)bh * NC + i) * CHUNK * D;
        if (part < 0 || part == 0)
            async_copy_tile<256, KVF>(reinterpret_cast<const Frag*>(reinterpret_cast<const T*>(p.xs) + slot), buf, tid, wv);
        if ((part < 0 || part == 2) && !NFUSE)       // (near, 16-bit: Xs^T fragments are read out of the xs tile)
            async_copy_tile<256, KVF>(reinterpret_cast<const Frag*>(reinterpret_cast<const T*>(p.xsT) + slot), buf + KVF, tid, wv);
        if (part < 0 || part == 1)
            async_copy_tile<256, KVF>(reinterpret_cast<const Frag*>(reinterpret_cast<const TIO*>(p.doq) + bhi), buf + 2 * KVF, tid, wv);
        if (part < 0 || part == 3) {
            if (NFUSE) async_copy_tile<256, KVF>(reinterpret_cast<const Frag*>(reinterpret_cast<const T*>(p.gs) + slot), buf + 3 * KVF, tid, wv);
            else async_copy_tile<256, KVF>(reinterpret_cast<const Frag*>(reinterpret_cast<const TIO*>(p.doT) + bhi), buf + 3 * KVF, tid, wv);
        }
        if ((part < 0 || part == 0) && tid < 32) {     // 64 floats of lse2 (lanes 0-15) and of delta (lanes 16-31): 16 bytes per lane
            const float* src = (tid < 16 ? p.lse2p : p.delta) + (size_t)bh * Lp + (size_t)i * CHUNK + 4 * (tid & 15);
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                             (__attribute__((address_space(3))) void*)(buf + 4 * KVF), 16, 0, 0);
        }
    };

    if (i0 < i1 && NBUF == 2) issue(i0, -1);
    for (int i = i0; i < i1; ++i) {
        const bool spread = NBUF == 2 && i + 1 < i1 && FAR;       // far: two rounds of work per chunk to spread over
        if (NBUF == 2) {
            wait_async_and_sync();                 // chunk i has landed; everyone is done with chunk i-1
            if (i + 1 < i1) issue(i + 1, spread ? 0 : -1);
        } else {
            __syncthreads();
            issue(i, -1);
            wait_async_and_sync();
        }
        const Frag* sX = sbase + (size_t)(i & (NBUF - 1)) * STF;
        const Frag* sXT = sX + KVF;
        const FragV* sDQ = reinterpret_cast<const FragV*>(sX + 2 * KVF);
        const FragV* sDT = reinterpret_cast<const FragV*>(sX + 3 * KVF);
        const float* lse2 = reinterpret_cast<const float*>(sX + 4 * KVF);
        const float* dl = lse2 + CHUNK;

        // The three parts of the work on a 32-query half: logits and dP (16 products), the element-wise
        // part, and the updates of dV^T and dKb^T (32 products).
        auto sdp = [&](int qh, f32x16& S, f32x16& dP) {
            S = zero16(); dP = zero16();                           // rows q (half qh), lane s
            // operand fragments are fetched in batches ahead of the products that use them
#pragma unroll
            for (int s0 = 0; s0 < DS; s0 += 4) {
                Frag xa[4];
                FragV da[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) { xa[u] = sX[(qh * DS + s0 + u) * 64 + lane]; da[u] = sDQ[(qh * DS + s0 + u) * 64 + lane]; }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    S = Tr<T>::mma(xa[u], Kb[s0 + u], S);
                    dP = Tr<TIO>::mma(da[u], Vb[s0 + u], dP);
                }
            }
        };
        auto soft = [&](int qh, f32x16& S, const f32x16& dP, FragV* Pb, Frag* dSb) {
            // Rows past L need no mask: their padded lse2p is huge, so P = exp2(-huge) = 0.
            f32x4 ls[4], dls[4];
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                ls[g] = *reinterpret_cast<const f32x4*>(lse2 + 32 * qh + 8 * g + 4 * h);
                dls[g] = *reinterpret_cast<const f32x4*>(dl + 32 * qh + 8 * g + 4 * h);
            }
            f32x16 Pm;
#pragma unroll
            for (int jj = 0; jj < 16; ++jj) {
                const float P = __builtin_amdgcn_exp2f(__builtin_fmaf(S[jj], sl2, -ls[jj >> 2][jj & 3]) - ckj);
                Pm[jj] = P;
                const float dz = P * (dP[jj] - dls[jj >> 2][jj & 3]);
                if (FOX) dcol += dz;
                S[jj] = dz;                 // the factor scale of dS is applied to the finished dKb sums
            }
            pack_block<TIO>(Pm, Pb);
            pack_block<T>(S, dSb);
        };
        auto upd = [&](int qh, const FragV* Pb, const Frag* dSb) {
#pragma unroll
            for (int b = 0; b < DB; b += 2) {
                FragV ta[2 * SPB];
                Frag tb[2 * SPB];
#pragma unroll
                for (int u = 0; u < 2 * SPB; ++u) {
                    ta[u] = sDT[((b + u / SPB) * QS + qh * SPB + u % SPB) * 64 + lane];
                    tb[u] = sXT[((b + u / SPB) * QS + qh * SPB + u % SPB) * 64 + lane];
                }
#pragma unroll
                for (int u = 0; u < 2 * SPB; ++u) {
                    dVt[b + u / SPB] = Tr<TIO>::mma(ta[u], Pb[u % SPB], dVt[b + u / SPB]);
                    dKt[b + u / SPB] = Tr<T>::mma(tb[u], dSb[u % SPB], dKt[b + u / SPB]);
                }
            }
        };
        if (FAR && sizeof(T) == 2) {
            // Both query halves, software-pipelined by hand: the element-wise part of one half is
            // interleaved, element by element, with the products of the other (one wave per SIMD:
            // nothing else hides it).  The scheduling barriers keep the compiler from undoing the order.
            f32x16 S0 = zero16(), dP0 = zero16(), S1 = zero16(), dP1 = zero16(), Pm;
            FragV Pb0[SPB], Pb1[SPB];
            Frag dSb0[SPB], dSb1[SPB];
            f32x4 ls0[4], dls0[4], ls1[4], dls1[4];
            // Rows past L need no mask: their padded lse2p is huge, so P = exp2(-huge) = 0.
            // The empty asm statements pin the element's arithmetic between the two products around it
            // (they are ordered with the scheduling barriers; plain arithmetic alone is not).
            auto elem = [&](int jj, f32x16& S, const f32x16& dP, const f32x4* ls, const f32x4* dls) {
                float sv = S[jj], dv = dP[jj];
                asm volatile("" : "+v"(sv), "+v"(dv));
                const float P = __builtin_amdgcn_exp2f(__builtin_fmaf(sv, sl2, -ls[jj >> 2][jj & 3]) - ckj);
                const float dz = P * (dv - dls[jj >> 2][jj & 3]);
                if (FOX) dcol += dz;
                float ds = dz, pv = P;      // the factor scale of dS is applied to the finished dKb sums
                asm volatile("" : "+v"(ds), "+v"(pv));
                Pm[jj] = pv;
                S[jj] = ds;
            };
            Frag xa0[DS], xa1[DS], tb0[DB * SPB], tb1[DB * SPB];
            FragV da0[DS], da1[DS], ta0[DB * SPB], ta1[DB * SPB];
#pragma unroll
            for (int u = 0; u < DS; ++u) { xa0[u] = sX[u * 64 + lane]; da0[u] = sDQ[u * 64 + lane]; }
            __builtin_amdgcn_sched_barrier(0);
            // logits and dP of half 0
#pragma unroll
            for (int u = 0; u < DS; ++u) {
                S0 = Tr<T>::mma(xa0[u], Kb[u], S0);
                dP0 = Tr<TIO>::mma(da0[u], Vb[u], dP0);
            }
            __builtin_amdgcn_sched_barrier(0);
            if (spread) issue(i + 1, 1);
            // logits and dP of half 1  ||  element-wise part of half 0
#pragma unroll
            for (int u = 0; u < DS; ++u) { xa1[u] = sX[(DS + u) * 64 + lane]; da1[u] = sDQ[(DS + u) * 64 + lane]; }
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                ls0[g] = *reinterpret_cast<const f32x4*>(lse2 + 8 * g + 4 * h);
                dls0[g] = *reinterpret_cast<const f32x4*>(dl + 8 * g + 4 * h);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < DS; ++u) {
                S1 = Tr<T>::mma(xa1[u], Kb[u], S1);
                __builtin_amdgcn_sched_barrier(0);
                if (2 * u < 16) elem(2 * u, S0, dP0, ls0, dls0);
                __builtin_amdgcn_sched_barrier(0);
                dP1 = Tr<TIO>::mma(da1[u], Vb[u], dP1);
                __builtin_amdgcn_sched_barrier(0);
                if (2 * u + 1 < 16) elem(2 * u + 1, S0, dP0, ls0, dls0);
                __builtin_amdgcn_sched_barrier(0);
            }
            if (DS < 8) {
#pragma unroll
                for (int jj = 2 * DS; jj < 16; ++jj) elem(jj, S0, dP0, ls0, dls0);
            }
            pack_block<TIO>(Pm, Pb0);
            pack_block<T>(S0, dSb0);
            if (spread) issue(i + 1, 3);
            // dV^T, dKb^T of half 0  ||  element-wise part of half 1
#pragma unroll
            for (int u = 0; u < DB * SPB; ++u) {
                ta0[u] = sDT[((u / SPB) * QS + u % SPB) * 64 + lane];
                tb0[u] = sXT[((u / SPB) * QS + u % SPB) * 64 + lane];
            }
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                ls1[g] = *reinterpret_cast<const f32x4*>(lse2 + 32 + 8 * g + 4 * h);
                dls1[g] = *reinterpret_cast<const f32x4*>(dl + 32 + 8 * g + 4 * h);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < DB * SPB; ++u) {
                dVt[u / SPB] = Tr<TIO>::mma(ta0[u], Pb0[u % SPB], dVt[u / SPB]);
                __builtin_amdgcn_sched_barrier(0);
                if (2 * u < 16) elem(2 * u, S1, dP1, ls1, dls1);
                __builtin_amdgcn_sched_barrier(0);
                dKt[u / SPB] = Tr<T>::mma(tb0[u], dSb0[u % SPB], dKt[u / SPB]);
                __builtin_amdgcn_sched_barrier(0);
                if (2 * u + 1 < 16) elem(2 * u + 1, S1, dP1, ls1, dls1);
                __builtin_amdgcn_sched_barrier(0);
            }
            if (DB * SPB < 8) {
#pragma unroll
                for (int jj = 2 * DB * SPB; jj < 16; ++jj) elem(jj, S1, dP1, ls1, dls1);
            }
            pack_block<TIO>(Pm, Pb1);
            pack_block<T>(S1, dSb1);
            if (spread) issue(i + 1, 2);
            // dV^T, dKb^T of half 1
#pragma unroll
            for (int u = 0; u < DB * SPB; ++u) {
                ta1[u] = sDT[((u / SPB) * QS + SPB + u % SPB) * 64 + lane];
                tb1[u] = sXT[((u / SPB) * QS + SPB + u % SPB) * 64 + lane];
            }
#pragma unroll
            for (int u = 0; u < DB * SPB; ++u) {
                dVt[u / SPB] = Tr<TIO>::mma(ta1[u], Pb1[u % SPB], dVt[u / SPB]);
                dKt[u / SPB] = Tr<T>::mma(tb1[u], dSb1[u % SPB], dKt[u / SPB]);
            }
        } else {
#pragma unroll
            for (int qq = 0; qq < CPW; ++qq) {
                const int qh = FAR ? qq : (wv >> 1);
                f32x16 S, dP;
                FragV Pb[SPB];
                Frag dSb[SPB];
                sdp(qh, S, dP);
                if (FAR && spread) issue(i + 1, qq == 0 ? 1 : 3);
                soft(qh, S, dP, Pb, dSb);
                if constexpr (NFUSE) {
                    // dV^T, dKb^T and the wave's ddP blocks, one 32-row block b of Xs^T at a time: its four
                    // fragments (all 64 queries) serve ddP, and the two of the wave's own query half serve dKb^T --
                    // every fragment is read from LDS once per step (the reads, not the products, bound this loop).
                    // The wave's ddP blocks wv, wv + 4, ... all lie in column block bb of g (d = 128: one per row
                    // block b; d = 64: the single block (wv / 2, wv % 2)), whose fragments are read once too.
                    static_assert(DB == 4 || DB == 2, "block ownership below");
                    // The wave's own query half comes first, the other one second, both by address (qh is uniform over
                    // the wave): no selects between registers.  Chunk 0 has no transform to the left of it: its sums
                    // are taken like the others (its adjoint-state tile is valid memory, whatever it holds) and
                    // written as zeros at the end -- a test here would put the accumulators behind a branch, and
                    // the compiler then copies them between the register files around every product.
                    const Frag* sG = sX + 3 * KVF;
                    const int bb = DB == 4 ? wv : (wv & 1);
                    const int own = qh * SPB, oth = (1 - qh) * SPB;
                    Frag fbo[SPB], fbx[SPB];
#pragma unroll
                    for (int u = 0; u < SPB; ++u) { fbo[u] = sG[(bb * QS + own + u) * 64 + lane]; fbx[u] = sG[(bb * QS + oth + u) * 64 + lane]; }
#pragma unroll
                    for (int b = 0; b < DB; ++b) {
                        Frag fo[SPB], fx[SPB];
                        FragV ta[SPB];
#pragma unroll
                        for (int u = 0; u < SPB; ++u) {
                            fo[u] = ld_tile_frag_tr<T, DS>(reinterpret_cast<const T*>(sX), own + u, b, l32, h);
                            fx[u] = ld_tile_frag_tr<T, DS>(reinterpret_cast<const T*>(sX), oth + u, b, l32, h);
                            ta[u] = ld_tile_frag_tr<TIO, DS>(reinterpret_cast<const TIO*>(sDQ), own + u, b, l32, h);
                        }
#pragma unroll
                        for (int u = 0; u < SPB; ++u) {
                            dVt[b] = Tr<TIO>::mma(ta[u], Pb[u], dVt[b]);
                            dKt[b] = Tr<T>::mma(fo[u], dSb[u], dKt[b]);
                        }
                        if (DB == 4 || b == (wv >> 1)) {
                            constexpr int NO = DB == 4 ? DB : 1;
#pragma unroll
                            for (int o = 0; o < NO; ++o)
                                if (DB != 4 || o == b) {
#pragma unroll
                                    for (int u = 0; u < SPB; ++u) {
                                        ddPa[o] = Tr<T>::mma(fo[u], fbo[u], ddPa[o]);
                                        ddPa[o] = Tr<T>::mma(fx[u], fbx[u], ddPa[o]);
                                    }
                                }
                        }
                    }
                } else {
                    upd(qh, Pb, dSb);
                }
                if (FAR && spread && qq == 0) issue(i + 1, 2);
            }
        }
    }
    if (NFUSE) {
#pragma unroll
        for (int o = 0; o < NOWN; ++o) {
            const int blk = wv + 4 * o, ab = blk / DB, bb = blk % DB;
#pragma unroll
            for (int jj = 0; jj < 16; ++jj)
                __builtin_nontemporal_store(j >= 1 ? -ddPa[o][jj] : 0.f, &p.ddp[((size_t)bh * NC + j) * D * D + (size_t)(32 * ab + acc_row(jj, h)) * D + 32 * bb + l32]);
        }
    }
    if (FAR) {
        // each wave holds the complete sums of its 32 keys: write row-major fp32 [s][c] from
        // registers (rows c, lane s); dV is added to the near part
        if (!wactive) return;
        if (FOX) {           // the two half-waves hold different query rows of the same keys
            dcol += __shfl_xor(dcol, 32);
            if (h == 0) p.dcol[(size_t)bh * Lp + key_tok] += dcol;      // added to the near part
        }
        const size_t row = ((size_t)bh * Lp + jw * CHUNK + 32 * kh + l32) * D + 4 * h;
#pragma unroll
        for (int b = 0; b < DB; ++b)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                f32x4 v4 = *reinterpret_cast<const f32x4*>(p.dvp + row + 32 * b + 8 * g), k4;
#pragma unroll
                for (int r = 0; r < 4; ++r) { v4[r] += dVt[b][4 * g + r]; k4[r] = p.scale * dKt[b][4 * g + r]; }
                *reinterpret_cast<f32x4*>(p.dvp + row + 32 * b + 8 * g) = v4;
                *reinterpret_cast<f32x4*>(p.dk2 + row + 32 * b + 8 * g) = k4;
            }
        return;
    }
    const int qh = wv >> 1;
    // sum the two query halves, write row-major fp32 [s][c] from registers (rows c, lane s)
    __syncthreads();
    float* red = reinterpret_cast<float*>(smem);
    float* redc = red + 2 * 2 * DB * 1024;       // FOX: column sums of the upper waves
    if (FOX) dcol += __shfl_xor(dcol, 32);
    if (qh == 1) {
#pragma unroll
        for (int b = 0; b < DB; ++b)
#pragma unroll
            for (int jj = 0; jj < 16; ++jj) {
                red[((kh * 2 + 0) * DB + b) * 1024 + jj * 64 + lane] = dVt[b][jj];
                red[((kh * 2 + 1) * DB + b) * 1024 + jj * 64 + lane] = dKt[b][jj];
            }
        if (FOX && h == 0) redc[kh * 32 + l32] = dcol;
    }
    __syncthreads();
    if (FOX && qh == 0 && h == 0) p.dcol[(size_t)bh * Lp + key_tok] = dcol + redc[kh * 32 + l32];
    if (qh == 0) {
        const size_t row = ((size_t)bh * Lp + j * CHUNK + 32 * kh + l32) * D + 4 * h;
#pragma unroll
        for (int b = 0; b < DB; ++b)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                f32x4 v4, k4;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    v4[r] = dVt[b][4 * g + r] + red[((kh * 2 + 0) * DB + b) * 1024 + (4 * g + r) * 64 + lane];
                    k4[r] = p.scale * (dKt[b][4 * g + r] + red[((kh * 2 + 1) * DB + b) * 1024 + (4 * g + r) * 64 + lane]);
                }
                *reinterpret_cast<f32x4*>(p.dvp + row + 32 * b + 8 * g) = v4;
                *reinterpret_cast<f32x4*>(p.dkb + row + 32 * b + 8 * g) = k4;
            }
    }
}

// ---------------------------------------------------------------------------------------
// ddP_blk[a][b] = - sum_i sum_q Xs(i,blk)[q][a] g(i, block before blk)[q][b]: one workgroup per key
// block, a plain product over the stacked query axis of the tiles xsT and gT (contraction q),
// staged through LDS.  Near (FAR = false): block = chunk j, queries = the chunks i > j of j's
// super-block, result ddP_j.  Far (FAR = true): block = super-block J, queries = all chunks
// right of it; the result is stored with the opposite sign -- the gradient with respect to
// P_superblock = I - dP2 -- where the adjoint of the second level starts its chain: entry 4J of
// the per-head array dchain (entry c+1 belongs to chunk c; entry 0 is zero).
template <typename TIO, int D> struct DdpCfg {
    typedef typename Compute<TIO>::type T;
    static constexpr int KV_FRAGS = CHUNK * D / Tr<T>::FE;
    static constexpr int NBUF = 2;
    static constexpr size_t smem_bytes = (size_t)NBUF * 2 * KV_FRAGS * 16;     // NBUF x (xsT | gT)
};

template <typename TIO, int D, bool FAR>
__global__ __launch_bounds__(256) void bwd_ddp_kernel(BwdParams p) {
    using C = DdpCfg<TIO, D>;
    using T = typename Compute<TIO>::type;
    using Frag = typename Tr<T>::Frag;
    constexpr int KW = Tr<T>::KW, DB = D / 32, QS = CHUNK / KW, NOWN = DB * DB / 4, KVF = C::KV_FRAGS;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    Frag* sbase = reinterpret_cast<Frag*>(smem);
    const int j = blockIdx.x, bh = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wv = __builtin_amdgcn_readfirstlane(tid >> 6), h = lane >> 5, l32 = lane & 31;
    const int NC = p.NC;                                          // chunks per head in the workspace arrays
    const int NCo = (seq_len(p.ul, bh, p.L) + CHUNK - 1) / CHUNK;  // this head's own chunks
    const size_t nslots = num_block_slots(NC);
    const int cj = FAR ? j * SBC : j;                             // a key chunk of the block
    const int sb_end = (cj / SBC + 1) * SBC;
    const int i0 = FAR ? sb_end : j + 1;
    const int i1 = FAR ? NCo : (sb_end < NCo ? sb_end : NCo);       // (no queries to the right: the sums are zero)
    f32x16 acc[NOWN];
#pragma unroll
    for (int o = 0; o < NOWN; ++o) acc[o] = zero16();
    if (j >= 1) {
        auto issue = [&](int i) {
            Frag* buf = sbase + (size_t)(i & 1) * 2 * KVF;
            const size_t slot = ((size_t)bh * nslots + block_slot(i, cj, NC)) * (size_t)CHUNK * D;
            async_copy_tile<256, KVF>(reinterpret_cast<const Frag*>(reinterpret_cast<const T*>(p.xsT) + slot), buf, tid, wv);
            async_copy_tile<256, KVF>(reinterpret_cast<const Frag*>(reinterpret_cast<const T*>(p.gs) + slot), buf + KVF, tid, wv);
        };
        if (i0 < i1) issue(i0);
        for (int i = i0; i < i1; ++i) {
            wait_async_and_sync();                 // pair (i, j) has landed; everyone is done with pair (i-1, j)
            if (i + 1 < i1) issue(i + 1);
            const Frag* xt = sbase + (size_t)(i & 1) * 2 * KVF;
            const Frag* gt = xt + KVF;
#pragma unroll
            for (int o = 0; o < NOWN; ++o) {
                const int blk = wv + 4 * o, ab = blk / DB, bb = blk % DB;
                Frag fa[QS], fb[QS];
#pragma unroll
                for (int s = 0; s < QS; ++s) { fa[s] = xt[(ab * QS + s) * 64 + lane]; fb[s] = gt[(bb * QS + s) * 64 + lane]; }
#pragma unroll
                for (int s = 0; s < QS; ++s) acc[o] = Tr<T>::mma(fa[s], fb[s], acc[o]);
            }
        }
    }
#pragma unroll
    for (int o = 0; o < NOWN; ++o) {
        const int blk = wv + 4 * o, ab = blk / DB, bb = blk % DB;
#pragma unroll
        for (int jj = 0; jj < 16; ++jj) {
            const size_t el = (size_t)(32 * ab + acc_row(jj, h)) * D + 32 * bb + l32;
            if (FAR) p.dchain[((size_t)bh * (NC + 1) + (size_t)j * SBC) * D * D + el] = acc[o][jj];
            else p.ddp[((size_t)bh * NC + j) * D * D + el] = -acc[o][jj];
        }
    }
}

// ---------------------------------------------------------------------------------------
// Batched small product for the chunk-transform adjoint, one workgroup per (chunk, bh):
//   C[m][n] = mask( alpha * sum_k A[m][k] B[n][k] + Cin[m][n] )
// Operands are addressed with explicit strides (so either orientation of a stored
// matrix can be used), converted to the operand type while being staged in LDS.
// Stage R x K elements of one operand into LDS (row-major, pitch ld, operand type), eight
// elements per thread along whichever index is contiguous in memory (one 16/32-byte load).
// NB: how many 8-element vectors a thread loads before it converts and stores any of them.
// 1 keeps the register count low (kernels that rely on several workgroups per CU); 4 overlaps
// the load latencies (kernels with one workgroup per CU and registers to spare).
template <typename TIO, typename E, int NB = 1>
__device__ __forceinline__ void stage_mat_t(const MatRef& r, typename Compute<TIO>::type* dst, int ld, int R, int K,
                                            long long base, int ntok, int tid, float mul = 1.f) {
    typedef typename Compute<TIO>::type T;
    const E* src = reinterpret_cast<const E*>(r.p) + base;
    typedef E Vec8 __attribute__((ext_vector_type(8)));
    if (NB == 1) {
        if (r.ks == 1) {                       // contraction index contiguous
            const int kg = K / 8;
            for (int idx = tid; idx < R * kg; idx += 256) {
                const int m = idx / kg, k0 = (idx % kg) * 8;
                Vec8 v;
                const bool row_ok = r.tok != TOK_ROW || m < ntok;
                if (row_ok) v = *reinterpret_cast<const Vec8*>(src + (long long)m * r.rs + k0);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const bool ok = row_ok && (r.tok != TOK_K || k0 + e < ntok);
                    dst[m * ld + k0 + e] = ok ? (T)((float)v[e] * mul) : (T)0.f;
                }
            }
        } else {                               // row index contiguous (rs == 1)
            const int mg = R / 8;
            for (int idx = tid; idx < K * mg; idx += 256) {
                const int k = idx / mg, m0 = (idx % mg) * 8;
                Vec8 v;
                const bool k_ok = r.tok != TOK_K || k < ntok;
                if (k_ok) v = *reinterpret_cast<const Vec8*>(src + (long long)k * r.ks + m0);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const bool ok = k_ok && (r.tok != TOK_ROW || m0 + e < ntok);
                    dst[(m0 + e) * ld + k] = ok ? (T)((float)v[e] * mul) : (T)0.f;
                }
            }
        }
        return;
    }
    // A thread moves vectors of 8 elements along whichever index is contiguous in memory
    // (vectors per line: K/8 or R/8, a power of two).
    const bool kcontig = r.ks == 1;
    const int vlen = (kcontig ? K : R) / 8, sh = __ffs(vlen) - 1, nvec = R * K / 8;
    const long long lstride = kcontig ? r.rs : r.ks;
    for (int i0 = tid; i0 < nvec; i0 += 256 * NB) {
        Vec8 v[NB];
        bool ok_line[NB];
#pragma unroll
        for (int u = 0; u < NB; ++u) {
            const int idx = i0 + u * 256, line = idx >> sh, pos = (idx & (vlen - 1)) * 8;
            ok_line[u] = idx < nvec && (kcontig ? (r.tok != TOK_ROW || line < ntok) : (r.tok != TOK_K || line < ntok));
            if (ok_line[u]) v[u] = *reinterpret_cast<const Vec8*>(src + line * lstride + pos);
        }
#pragma unroll
        for (int u = 0; u < NB; ++u) {
            const int idx = i0 + u * 256, line = idx >> sh, pos = (idx & (vlen - 1)) * 8;
            if (idx >= nvec) break;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                // the index that runs along the vector is a token when it is k (kcontig, TOK_K) or a row (TOK_ROW)
                const bool ok = ok_line[u] && ((kcontig ? r.tok != TOK_K : r.tok != TOK_ROW) || pos + e < ntok);
                const T val = ok ? (T)((float)v[u][e] * mul) : (T)0.f;
                if (kcontig) dst[line * ld + pos + e] = val;
                else dst[(pos + e) * ld + line] = val;
            }
        }
    }
}

template <typename TIO, int NB = 1>
__device__ __forceinline__ void stage_mat(const MatRef& r, const UserLayout& ul, typename Compute<TIO>::type* dst, int ld, int R, int K,
                                          int bh, int chunk, int L, int tid, float mul = 1.f) {
    typedef typename Compute<TIO>::type T;
    const long long base = r.user ? user_vec(ul, bh, (long long)chunk * CHUNK) : bh * r.s_bh + chunk * r.s_ch;
    const int ntok = L - chunk * CHUNK;     // tokens of this chunk that exist
    if (r.type == EL_F32) stage_mat_t<TIO, float, NB>(r, dst, ld, R, K, base, ntok, tid, mul);
    else if (r.type == EL_OP) stage_mat_t<TIO, T, NB>(r, dst, ld, R, K, base, ntok, tid, mul);
    else stage_mat_t<TIO, TIO, NB>(r, dst, ld, R, K, base, ntok, tid, mul);
}

template <typename TIO>
__global__ __launch_bounds__(256) void batched_gemm_kernel(GemmArgs a) {
    typedef typename Compute<TIO>::type T;
    constexpr int FE = Tr<T>::FE, KW = Tr<T>::KW;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int ld = a.K + FE;
    T* As = reinterpret_cast<T*>(smem);
    T* Bs = As + a.M * ld;
    const int chunk = blockIdx.x * a.cmul + a.cadd, bh = blockIdx.y;
    const int Lown = seq_len(a.ul, bh, a.L);               // this head's own length (packed batches: may be shorter than a.L)
    if (chunk >= a.NC || chunk * CHUNK >= Lown) return;
    const int tid = threadIdx.x, lane = tid & 63, wv = __builtin_amdgcn_readfirstlane(tid >> 6), h = lane >> 5, l32 = lane & 31;
    stage_mat<TIO>(a.A, a.ul, As, ld, a.M, a.K, bh, chunk, Lown, tid);
    stage_mat<TIO>(a.B, a.ul, Bs, ld, a.N, a.K, bh, chunk, Lown, tid);
    __syncthreads();
    const int nb = a.N / 32, nblk = (a.M / 32) * nb;
    const long long cbase = bh * a.c_bh + chunk * a.c_ch;
    for (int blk = wv; blk < nblk; blk += 4) {
        const int mb = blk / nb, cb = blk % nb;
        const T* ap = As + (32 * mb + l32) * ld + FE * h;
        const T* bp = Bs + (32 * cb + l32) * ld + FE * h;
        f32x16 acc = zero16();
        for (int k0 = 0; k0 < a.K; k0 += 4 * KW) {        // K is a multiple of 64
            typename Tr<T>::Frag fa[4], fb[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) { fa[u] = ld_frag<T>(ap + k0 + u * KW); fb[u] = ld_frag<T>(bp + k0 + u * KW); }
#pragma unroll
            for (int u = 0; u < 4; ++u) acc = Tr<T>::mma(fa[u], fb[u], acc);
        }
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
// Element-wise steps of the chunk-transform adjoint (device functions of the fused kernel).
// Diagonal block: P = exp(scale*Sd - lse) on key <= query, dSd = scale * P (dPd - delta).
template <typename TIO, bool FOX>
__device__ __forceinline__ void chunk_diag(const DiagArgs& a, const UserLayout& ul, float* colsum, int chunk, int bh, int tid) {
    typedef typename Compute<TIO>::type T;
    const size_t base = ((size_t)bh * a.NC + chunk) * 4096;
    if (FOX) {
        if (tid < 2 * CHUNK) colsum[tid] = 0.f;
        __syncthreads();
    }
    for (int idx = tid; idx < 4096; idx += 256) {
        const int t = idx >> 6, s = idx & 63, tg = chunk * CHUNK + t;
        float P = 0.f, ds = 0.f;
        if (s <= t && tg < seq_len(ul, bh, a.L)) {
            float z = a.scale * a.sdm[base + idx] - a.lse[user_scl(ul, bh, tg)];
            if (FOX) {     // PaTH-FoX: + c_t - c_s (the gate sums are kept in base-2 units)
                const float* c = a.cum + (size_t)bh * a.NC * CHUNK + (size_t)chunk * CHUNK;
                z += (c[t] - c[s]) * 0.69314718055994530942f;
            }
            P = __expf(z);
            const float dz = P * (a.dpd[base + idx] - a.delta[(size_t)bh * a.NC * CHUNK + tg]);
            ds = a.scale * dz;
            if (FOX) { atomicAdd(colsum + s, dz); atomicAdd(colsum + CHUNK + t, dz); }      // LDS: column and row sums of the block
        }
        reinterpret_cast<T*>(a.pd)[base + idx] = (T)P;
        reinterpret_cast<T*>(a.dsd)[base + idx] = (T)ds;
    }
    if (FOX) {
        __syncthreads();
        if (tid < CHUNK) {
            a.dcol[(size_t)bh * a.NC * CHUNK + (size_t)chunk * CHUNK + tid] += colsum[tid];
            a.drow[(size_t)bh * a.NC * CHUNK + (size_t)chunk * CHUNK + tid] += colsum[CHUNK + tid];
        }
    }
}

// dbeta_a = R[a][a] + sum_s M[a][s] G[a][s];  dGs = diag(beta) M + (diag(beta) M)^T.
template <typename TIO>
__device__ __forceinline__ void chunk_beta(const BetaArgs& a, const UserLayout& ul, float* bs, int chunk, int bh, int tid) {
    const size_t base = ((size_t)bh * a.NC + chunk) * 4096;
    if (tid < CHUNK) {
        const int tg = chunk * CHUNK + tid;
        bs[tid] = (tg < seq_len(ul, bh, a.L)) ? (float)reinterpret_cast<const TIO*>(a.beta)[user_scl(ul, bh, tg)] : 0.f;
    }
    __syncthreads();
    for (int idx = tid; idx < 4096; idx += 256) {
        const int r = idx >> 6, c = idx & 63;
        reinterpret_cast<typename Compute<TIO>::type*>(a.dgs)[base + idx] = (typename Compute<TIO>::type)(bs[r] * a.m[base + idx] + bs[c] * a.m[base + c * 64 + r]);
    }
    if (tid < CHUNK) {
        float s = a.r[base + tid * 64 + tid];
        for (int c = 0; c < tid; ++c) s += a.m[base + tid * 64 + c] * a.g[base + tid * 64 + c];
        a.dbf[(size_t)bh * a.NC * CHUNK + chunk * CHUNK + tid] = s;
    }
}

// fp32 [BH][Lp][d] -> I/O type [BH][L][d]; dbeta likewise.
template <typename TIO>
__device__ __forceinline__ void chunk_store(const OutArgs& a, const UserLayout& ul, int chunk, int bh, int tid) {
    const size_t Lp = (size_t)a.NC * CHUNK;
    const int Lown = seq_len(ul, bh, a.L);
    for (int idx = tid; idx < CHUNK * a.d; idx += 256) {
        const int t = idx / a.d, c = idx % a.d, tg = chunk * CHUNK + t;
        if (tg >= Lown) continue;
        const size_t src = ((size_t)bh * Lp + tg) * a.d + c, dst = (size_t)(user_vec(ul, bh, tg) + c);
        reinterpret_cast<TIO*>(a.dq)[dst] = (TIO)a.dqf[src];
        reinterpret_cast<TIO*>(a.dk)[dst] = (TIO)a.dkf[src];
        reinterpret_cast<TIO*>(a.dv)[dst] = (TIO)a.dvf[src];
        reinterpret_cast<TIO*>(a.dw)[dst] = (TIO)a.dwf[src];
    }
    if (tid < CHUNK && chunk * CHUNK + tid < Lown)
        reinterpret_cast<TIO*>(a.dbeta)[user_scl(ul, bh, chunk * CHUNK + tid)] = (TIO)a.dbf[(size_t)bh * Lp + chunk * CHUNK + tid];
}

// The fused adjoint of the chunk transform: one workgroup per (chunk, head) runs the program.
// Results that later steps read go through global memory (they stay in L2); a chain of
// products that add into the same result keeps it in accumulator registers.
#ifndef CHUNK_NB
#define CHUNK_NB 1
#endif
// FOX: the diagonal-block step also applies the gate sums and collects row/column sums (PaTH-FoX).
template <typename TIO, bool FOX>
__global__ __launch_bounds__(256, 3) void chunk_adjoint_kernel(ChunkProgram pr) {
    typedef typename Compute<TIO>::type T;
    constexpr int FE = Tr<T>::FE, KW = Tr<T>::KW;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int chunk = blockIdx.x, bh = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wv = __builtin_amdgcn_readfirstlane(tid >> 6), h = lane >> 5, l32 = lane & 31;
    const int Lown = seq_len(pr.ul, bh, pr.L);             // this head's own length (packed batches: may be shorter than pr.L)
    if (chunk * CHUNK >= Lown) return;
    f32x16 acc[2];
    for (int i = 0; i < pr.n; ++i) {
        const ChunkOp& op = pr.ops[i];
        __syncthreads();       // earlier steps' results are visible to the whole workgroup; LDS is free
        if (op.kind == OP_DIAG) { chunk_diag<TIO, FOX>(pr.diag, pr.ul, reinterpret_cast<float*>(smem), chunk, bh, tid); continue; }
        if (op.kind == OP_BETA) { chunk_beta<TIO>(pr.beta, pr.ul, reinterpret_cast<float*>(smem), chunk, bh, tid); continue; }
        if (op.kind == OP_STORE) { chunk_store<TIO>(pr.out, pr.ul, chunk, bh, tid); continue; }
        // M = 64 for every product of the list; N = 64 or 128.  Results are handled in halves of 64
        // columns (one 32x32 block per wave and half), the B operand is staged half by half, so a
        // workgroup needs (64 + 64) x (K + pad) operand elements of LDS and four workgroups fit a CU.
        const int N = op.N, K = op.K, ld = K + FE;
        T* As = reinterpret_cast<T*>(smem);
        T* Bs = As + CHUNK * ld;
        stage_mat<TIO, CHUNK_NB>(op.A, pr.ul, As, ld, CHUNK, K, bh, chunk, Lown, tid, op.alpha);
        const long long cbase = bh * op.c_bh + chunk * op.c_ch;
        const int mb = wv >> 1;
#pragma unroll
        for (int o = 0; o < 2; ++o) {
            if (64 * o >= N) break;
            if (o > 0) __syncthreads();                    // the first half's fragments have been read
            MatRef bhalf = op.B;                           // rows 64*o .. 64*o+63 of B (features, never tokens)
            bhalf.p = reinterpret_cast<const char*>(op.B.p) + (size_t)(64 * o) * op.B.rs * (op.B.type == EL_F32 ? 4 : sizeof(T));
            stage_mat<TIO, CHUNK_NB>(bhalf, pr.ul, Bs, ld, 64, K, bh, chunk, Lown, tid);
            __syncthreads();
            const int cb = 2 * o + (wv & 1), cbl = wv & 1;
            if (op.first) {
                if (op.Cin) {
#pragma unroll
                    for (int jj = 0; jj < 16; ++jj)
                        acc[o][jj] = op.Cin[cbase + (long long)(32 * mb + acc_row(jj, h)) * op.crs + 32 * cb + l32];
                } else {
                    acc[o] = zero16();
                }
            }
            const T* ap = As + (32 * mb + l32) * ld + FE * h;
            const T* bp = Bs + (32 * cbl + l32) * ld + FE * h;
            for (int k0 = 0; k0 < K; k0 += 4 * KW) {        // K is a multiple of 64
                typename Tr<T>::Frag fa[4], fb[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) { fa[u] = ld_frag<T>(ap + k0 + u * KW); fb[u] = ld_frag<T>(bp + k0 + u * KW); }
#pragma unroll
                for (int u = 0; u < 4; ++u) acc[o] = Tr<T>::mma(fa[u], fb[u], acc[o]);
            }
            if (op.last) {
#pragma unroll
                for (int jj = 0; jj < 16; ++jj) {
                    const int m = 32 * mb + acc_row(jj, h), n = 32 * cb + l32;
                    float v = acc[o][jj];
                    if ((op.mask == MASK_TRIL && n > m) || (op.mask == MASK_SLOWER && n >= m)) v = 0.f;
                    if (op.c_op) reinterpret_cast<T*>(op.C)[cbase + (long long)m * op.crs + n] = (T)v;
                    else op.C[cbase + (long long)m * op.crs + n] = v;
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
template <typename K> static hipError_t set_smem(K kernel, size_t bytes) {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

// stages: which of the kernels to launch (BWD_STAGE_* bits; all of them is the whole pass, in this order)
template <typename TIO, int D>
static hipError_t launch_scan_t(const BwdParams& p, int stages, hipStream_t st) {
    dim3 grid(p.NC, p.B * p.H);
    hipError_t e = hipSuccess;
    if (stages & BWD_STAGE_SCAN) {
        if (p.ul.vt != D) hipLaunchKernelGGL((bwd_dotile_kernel<TIO, D, true>), grid, dim3(256), 0, st, p);
        else hipLaunchKernelGGL((bwd_dotile_kernel<TIO, D, false>), grid, dim3(256), 0, st, p);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    const size_t adj_bytes = Adj2Cfg<TIO, D>::smem_bytes, key_bytes = Key2Cfg<TIO, D>::smem_bytes;
    const int ntiles = (p.NC + 1) / 2;
    const int BH = p.B * p.H, nsb = (p.NC + SBC - 1) / SBC;
    const dim3 grid_adj((unsigned)(8 * ((BH + 7) / 8) * ntiles));
    const dim3 grid_key((unsigned)(8 * ((BH + 7) / 8) * nsb * SBC)), grid_key_far((unsigned)(8 * ((BH + 7) / 8) * nsb * (SBC / 2)));
    if (p.cum) {       // PaTH-FoX instantiations
        if (stages & BWD_STAGE_SCAN) {
            if constexpr (sizeof(typename Compute<TIO>::type) == 2) {
                const size_t lite_bytes = (size_t)(2 * Adj2Cfg<TIO, D>::KV_FRAGS + Adj2Cfg<TIO, D>::DP_FRAGS) * 16;      // kt | vk | dpt
                if ((e = set_smem(&bwd_adjoint2_lite_kernel<TIO, D, true>, lite_bytes)) != hipSuccess) return e;
                hipLaunchKernelGGL((bwd_adjoint2_lite_kernel<TIO, D, true>), grid_adj, dim3(256), lite_bytes, st, p);
            } else {
                if ((e = set_smem(&bwd_adjoint2_kernel<TIO, D, true>, adj_bytes)) != hipSuccess) return e;
                hipLaunchKernelGGL((bwd_adjoint2_kernel<TIO, D, true>), grid_adj, dim3(256), adj_bytes, st, p);
            }
            if ((e = hipGetLastError()) != hipSuccess) return e;
        }
        if ((e = set_smem(&bwd_keyside2_kernel<TIO, D, false, true>, key_bytes)) != hipSuccess) return e;
        if ((e = set_smem(&bwd_keyside2_kernel<TIO, D, true, true>, key_bytes)) != hipSuccess) return e;
        if (stages & BWD_STAGE_KEYS_NEAR) hipLaunchKernelGGL((bwd_keyside2_kernel<TIO, D, false, true>), grid_key, dim3(256), key_bytes, st, p);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        if (stages & BWD_STAGE_KEYS_FAR) hipLaunchKernelGGL((bwd_keyside2_kernel<TIO, D, true, true>), grid_key_far, dim3(256), key_bytes, st, p);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    } else {
        if (stages & BWD_STAGE_SCAN) {
            if constexpr (sizeof(typename Compute<TIO>::type) == 2) {
                const size_t lite_bytes = (size_t)(2 * Adj2Cfg<TIO, D>::KV_FRAGS + Adj2Cfg<TIO, D>::DP_FRAGS) * 16;      // kt | vk | dpt
                if ((e = set_smem(&bwd_adjoint2_lite_kernel<TIO, D, false>, lite_bytes)) != hipSuccess) return e;
                hipLaunchKernelGGL((bwd_adjoint2_lite_kernel<TIO, D, false>), grid_adj, dim3(256), lite_bytes, st, p);
            } else {
                if ((e = set_smem(&bwd_adjoint2_kernel<TIO, D, false>, adj_bytes)) != hipSuccess) return e;
                hipLaunchKernelGGL((bwd_adjoint2_kernel<TIO, D, false>), grid_adj, dim3(256), adj_bytes, st, p);
            }
            if ((e = hipGetLastError()) != hipSuccess) return e;
        }
        if ((e = set_smem(&bwd_keyside2_kernel<TIO, D, false, false>, key_bytes)) != hipSuccess) return e;
        if ((e = set_smem(&bwd_keyside2_kernel<TIO, D, true, false>, key_bytes)) != hipSuccess) return e;
        if (stages & BWD_STAGE_KEYS_NEAR) hipLaunchKernelGGL((bwd_keyside2_kernel<TIO, D, false, false>), grid_key, dim3(256), key_bytes, st, p);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        if (stages & BWD_STAGE_KEYS_FAR) hipLaunchKernelGGL((bwd_keyside2_kernel<TIO, D, true, false>), grid_key_far, dim3(256), key_bytes, st, p);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    const size_t ddp_bytes = DdpCfg<TIO, D>::smem_bytes;
    if ((e = set_smem(&bwd_ddp_kernel<TIO, D, false>, ddp_bytes)) != hipSuccess) return e;
    if ((e = set_smem(&bwd_ddp_kernel<TIO, D, true>, ddp_bytes)) != hipSuccess) return e;
    if (!(stages & BWD_STAGE_DDP)) return hipSuccess;
    if (sizeof(typename Compute<TIO>::type) != 2)       // 16-bit operands: the near key-side kernel has written ddP
        hipLaunchKernelGGL((bwd_ddp_kernel<TIO, D, false>), grid, dim3(256), ddp_bytes, st, p);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    const dim3 grid_sb((p.NC + SBC - 1) / SBC, p.B * p.H);
    hipLaunchKernelGGL((bwd_ddp_kernel<TIO, D, true>), grid_sb, dim3(256), ddp_bytes, st, p);
    return hipGetLastError();
}

hipError_t launch_bwd_scan(const BwdParams& p, int d, int is_bf16, int stages, hipStream_t st) {
    if (is_bf16) return d == 64 ? launch_scan_t<bf16_t, 64>(p, stages, st) : launch_scan_t<bf16_t, 128>(p, stages, st);
    return d == 64 ? launch_scan_t<float, 64>(p, stages, st) : launch_scan_t<float, 128>(p, stages, st);
}

hipError_t launch_batched_gemm(const GemmArgs& a, int BH, int is_bf16, hipStream_t st) {
    const size_t es = is_bf16 ? 2 : 4, fe = is_bf16 ? 8 : 4;
    const size_t bytes = (size_t)(a.M + a.N) * (a.K + fe) * es;
    dim3 grid(a.gridx, BH);
    // set once per process; function-local statics are initialised under the language's own lock
    static const hipError_t attr_bf = set_smem(&batched_gemm_kernel<bf16_t>, 160 * 1024);
    static const hipError_t attr_f32 = set_smem(&batched_gemm_kernel<float>, 160 * 1024);
    if ((is_bf16 ? attr_bf : attr_f32) != hipSuccess) return is_bf16 ? attr_bf : attr_f32;
    if (is_bf16) hipLaunchKernelGGL((batched_gemm_kernel<bf16_t>), grid, dim3(256), bytes, st, a);
    else hipLaunchKernelGGL((batched_gemm_kernel<float>), grid, dim3(256), bytes, st, a);
    return hipGetLastError();
}

hipError_t launch_chunk_adjoint(const ChunkProgram& pr, int BH, int is_bf16, hipStream_t st) {
    const size_t es = is_bf16 ? 2 : 4, fe = is_bf16 ? 8 : 4;
    size_t bytes = 1024;
    for (int i = 0; i < pr.n; ++i) {
        if (pr.ops[i].kind != OP_PRODUCT) continue;
        const size_t b = (size_t)(CHUNK + CHUNK) * (pr.ops[i].K + fe) * es;      // A and half of B
        if (b > bytes) bytes = b;
    }
    const bool fox = pr.diag.cum != nullptr;
    hipError_t e;
    dim3 grid(pr.NC, BH);
#define LAUNCH_CHUNK_ADJ(TT, FF)                                                                  \
    do {                                                                                          \
        if ((e = set_smem(&chunk_adjoint_kernel<TT, FF>, 160 * 1024)) != hipSuccess) return e;    \
        hipLaunchKernelGGL((chunk_adjoint_kernel<TT, FF>), grid, dim3(256), bytes, st, pr);       \
    } while (0)
    if (is_bf16) { if (fox) LAUNCH_CHUNK_ADJ(bf16_t, true); else LAUNCH_CHUNK_ADJ(bf16_t, false); }
    else { if (fox) LAUNCH_CHUNK_ADJ(float, true); else LAUNCH_CHUNK_ADJ(float, false); }
#undef LAUNCH_CHUNK_ADJ
    return hipGetLastError();
}

}  // namespace path
