// Shared device-side definitions of the PaTH attention kernels (gfx950 only).
//
// Register/fragment conventions used by every kernel
// --------------------------------------------------
// All contractions run on the 32x32 MFMA tile of a 64-lane wavefront.  Lane
// l = 32*h + c (h = l/32, c = l%32) owns column c of the 32x32 fp32 result;
// its 16 accumulator registers j = 0..15 hold rows
//
//        acc_row(j, h) = 8*(j/4) + 4*h + (j%4).
//
// An operand fragment is 16 bytes per lane: FE = 8 bf16 or 4 fp32 elements.
// One "slab" is what one fragment pair contracts: KW = 2*FE indices
// (bf16: one v_mfma_f32_32x32x16_bf16; fp32: four v_mfma_f32_32x32x2_f32).
//
// Activations (query state X, probabilities P) never leave registers: a
// result in accumulator layout is re-used as the B operand of the next
// contraction by packing registers [s*FE, (s+1)*FE) of a 32-row block into
// slab s.  That fixes which contraction index sits in which fragment element,
//
//        index(block b, slab s, half h, element e) = 32*b + acc_row(s*FE+e, h),
//
// so the other operand (K, V^T, chunk products), which streams through LDS,
// is stored by the preprocessing kernel in exactly that order ("fragment
// order"): fragment ((rb*(Kc/KW) + slab)*64 + lane) of a tile with rows
// 32*rb + c and Kc contraction indices.  Lanes then read consecutive 16-byte
// fragments: conflict-free LDS reads and linear global->LDS copies.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace path {

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 half_t;
typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));
typedef _Float16 halfx4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int CHUNK = 64;      // tokens per chunk (UT transform block)
#ifndef PATH_SBC
#define PATH_SBC 16            // measured at B=4, H=16, L=8192, d=128: 8 -> +0.35 ms per training step, 32 -> +0.65 ms
#endif
constexpr int SBC = PATH_SBC;  // chunks per super-block (second blocking level of the forward sweep)

__device__ __forceinline__ int acc_row(int j, int h) { return 8 * (j >> 2) + 4 * h + (j & 3); }

template <typename T> struct Tr;

template <> struct Tr<bf16_t> {
    static constexpr int FE = 8;    // elements per 16-byte fragment
    static constexpr int KW = 16;   // contraction indices per slab
    typedef bf16x8 Frag;
    typedef bf16x4 Vec4;            // 4 consecutive elements
    static __device__ __forceinline__ f32x16 mma(Frag a, Frag b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
    // slab s of a 32-row accumulator block as an operand fragment
    template <int S> static __device__ __forceinline__ Frag pack(const f32x16& a) {
        Frag f;
#pragma unroll
        for (int e = 0; e < 8; ++e) f[e] = (bf16_t)a[S * 8 + e];
        return f;
    }
    static __device__ __forceinline__ Frag zero() { Frag f; for (int e = 0; e < 8; ++e) f[e] = (bf16_t)0.0f; return f; }
};

template <> struct Tr<half_t> {
    static constexpr int FE = 8;
    static constexpr int KW = 16;
    typedef halfx8 Frag;
    typedef halfx4 Vec4;
    static __device__ __forceinline__ f32x16 mma(Frag a, Frag b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
    }
    template <int S> static __device__ __forceinline__ Frag pack(const f32x16& a) {
        Frag f;
#pragma unroll
        for (int e = 0; e < 8; ++e) f[e] = (half_t)a[S * 8 + e];
        return f;
    }
    static __device__ __forceinline__ Frag zero() { Frag f; for (int e = 0; e < 8; ++e) f[e] = (half_t)0.0f; return f; }
};

template <> struct Tr<float> {
    static constexpr int FE = 4;
    static constexpr int KW = 8;
    typedef f32x4 Frag;
    typedef f32x4 Vec4;
    static __device__ __forceinline__ f32x16 mma(Frag a, Frag b, f32x16 c) {
#pragma unroll
        for (int e = 0; e < 4; ++e) c = __builtin_amdgcn_mfma_f32_32x32x2f32(a[e], b[e], c, 0, 0, 0);
        return c;
    }
    template <int S> static __device__ __forceinline__ Frag pack(const f32x16& a) {
        Frag f;
#pragma unroll
        for (int e = 0; e < 4; ++e) f[e] = a[S * 4 + e];
        return f;
    }
    static __device__ __forceinline__ Frag zero() { Frag f = {0.f, 0.f, 0.f, 0.f}; return f; }
};

// Operand type of the TRANSPORTED quantities (query state, boundary-adjusted
// keys, chunk products and everything inside the chunk transform) for a given
// I/O type.  With bf16 I/O these are carried in fp16: they are not
// representable in the input precision, and their rounding -- not the
// inputs' -- sets the error of the logits; bf16's 8 significand bits leave the
// log-sum-exp about 1.1e-3..2.8e-3 off, fp16's 11 bits about 2e-4, at the same
// MFMA rate.  (The method's transitions are contractions for beta in [0,2],
// |w| <= 1, so these operands are bounded by the norms of q and k, which must
// stay below the fp16 maximum 65504.)  P and V stay in the I/O type.
template <typename TIO> struct Compute { typedef TIO type; };
template <> struct Compute<bf16_t> { typedef half_t type; };

template <typename TO, typename TI>
__device__ __forceinline__ typename Tr<TO>::Frag cvt_frag(const typename Tr<TI>::Frag& f) {
    typename Tr<TO>::Frag o;
#pragma unroll
    for (int e = 0; e < Tr<TI>::FE; ++e) o[e] = (TO)(float)f[e];
    return o;
}

// Number of slabs in a 32-index block / in Kc indices.
template <typename T> constexpr int slabs_per_block() { return 32 / Tr<T>::KW; }

// All slabs of one 32-row accumulator block -> operand fragments dst[0 .. 32/KW).
template <typename T> __device__ __forceinline__ void pack_block(const f32x16& a, typename Tr<T>::Frag* dst);
template <> __device__ __forceinline__ void pack_block<bf16_t>(const f32x16& a, bf16x8* dst) {
    dst[0] = Tr<bf16_t>::pack<0>(a);
    dst[1] = Tr<bf16_t>::pack<1>(a);
}
template <> __device__ __forceinline__ void pack_block<half_t>(const f32x16& a, halfx8* dst) {
    dst[0] = Tr<half_t>::pack<0>(a);
    dst[1] = Tr<half_t>::pack<1>(a);
}
template <> __device__ __forceinline__ void pack_block<float>(const f32x16& a, f32x4* dst) {
    dst[0] = Tr<float>::pack<0>(a);
    dst[1] = Tr<float>::pack<1>(a);
    dst[2] = Tr<float>::pack<2>(a);
    dst[3] = Tr<float>::pack<3>(a);
}

__device__ __forceinline__ f32x16 zero16() {
    f32x16 z;
#pragma unroll
    for (int j = 0; j < 16; ++j) z[j] = 0.f;
    return z;
}

template <typename T>
__device__ __forceinline__ typename Tr<T>::Frag ld_frag(const T* p) {
    return *reinterpret_cast<const typename Tr<T>::Frag*>(p);
}

// acc += A[arow0 + c][0..Kc) . B[brow0 + c'][0..Kc)  for a 32x32 block; both
// operands are stored with the contraction index contiguous.
template <typename T, int Kc>
__device__ __forceinline__ f32x16 gemm32(const T* A, int lda, int arow0, const T* Bm, int ldb,
                                         int brow0, int l32, int h, f32x16 acc) {
    constexpr int FE = Tr<T>::FE, KW = Tr<T>::KW;
    const T* ap = A + (size_t)(arow0 + l32) * lda + FE * h;
    const T* bp = Bm + (size_t)(brow0 + l32) * ldb + FE * h;
#pragma unroll
    for (int k0 = 0; k0 < Kc; k0 += KW) acc = Tr<T>::mma(ld_frag<T>(ap + k0), ld_frag<T>(bp + k0), acc);
    return acc;
}

// Same with lane-specific row pointers (already offset by the row and by FE*h).
template <typename T, int Kc>
__device__ __forceinline__ f32x16 gemm_rows(const T* ap, const T* bp, f32x16 acc) {
    constexpr int KW = Tr<T>::KW;
#pragma unroll
    for (int k0 = 0; k0 < Kc; k0 += KW) acc = Tr<T>::mma(ld_frag<T>(ap + k0), ld_frag<T>(bp + k0), acc);
    return acc;
}

// Operand fragment of a matrix stored [k][row] (row contiguous) for the lane (l32, h) of a 32x32x16 product:
// the eight values X[kk + 8h + e][r0 + l32], e = 0..7.  Two transposing LDS reads (ds_read_b64_tr_b16): in
// each block of 16 lanes, lane j supplies the address of four consecutive values, and lane i receives
// element i % 4 of the chunks of lanes i/4, 4 + i/4, 8 + i/4, 12 + i/4.  With lane j pointing at
// X[kb + j/4][rb + 4 (j%4)], lane i therefore gets X[kb + e][rb + i], e = 0..3.
template <typename T>
__device__ __forceinline__ typename Tr<T>::Frag ld_frag_tr(const T* X, int ld, int kk, int r0, int l32, int h) {
    static_assert(sizeof(T) == 2, "16-bit transposing reads");
    typedef short v4s __attribute__((ext_vector_type(4)));
    const int j = l32 & 15;
    const T* p = X + (kk + 8 * h + (j >> 2)) * ld + r0 + (l32 & 16) + 4 * (j & 3);
    union { v4s v[2]; typename Tr<T>::Frag f; } u;
    u.v[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s*)(p));
    u.v[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s*)(p + 4 * ld));
    return u.f;
}

// acc[m][n] += sum_k A(m,k) B(n,k) for one 32x32 block (rows ar0.., columns br0..).
// TA == false: A is stored [m][k] (16-byte fragment reads); TA == true: A is stored [k][m] (transposing reads).  Same for B.
template <typename T, int K, bool TA, bool TB>
__device__ __forceinline__ void mm(f32x16& acc, const T* A, int lda, int ar0, const T* B, int ldb, int br0, int l32, int h) {
    // four slabs (64 contraction indices) at a time: their fragments are fetched ahead of the four products
#pragma unroll
    for (int k0 = 0; k0 < K; k0 += 64) {
        typename Tr<T>::Frag fa[4], fb[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int k = k0 + 16 * s + 8 * h;
            if (TA) {
                fa[s] = ld_frag_tr<T>(A, lda, k0 + 16 * s, ar0, l32, h);
            } else {
                fa[s] = ld_frag<T>(A + (ar0 + l32) * lda + k);
            }
            if (TB) {
                fb[s] = ld_frag_tr<T>(B, ldb, k0 + 16 * s, br0, l32, h);
            } else {
                fb[s] = ld_frag<T>(B + (br0 + l32) * ldb + k);
            }
        }
#pragma unroll
        for (int s = 0; s < 4; ++s) acc = Tr<T>::mma(fa[s], fb[s], acc);
    }
}

// Linear copy of NFRAG 16-byte fragments global -> LDS, asynchronous (direct-to-LDS), by a workgroup of
// NT threads.  One instruction moves 64 consecutive fragments (lane = fragment); wave wv takes the
// groups wv*NPT .. wv*NPT + NPT-1 (NPT = NFRAG / NT), which are 1 KB apart, so that one
// global address and one LDS base per four groups do: the instruction's immediate offset (added to both
// sides, at most 4095) covers the rest.
template <int NT, int NFRAG, typename Frag>
__device__ __forceinline__ void async_copy_tile(const Frag* g, Frag* s, int tid, int wv) {
    static_assert(sizeof(Frag) == 16 && NFRAG % 64 == 0 && (NFRAG % NT == 0 || NFRAG < NT), "whole groups of fragments");
    const int lane = tid & 63;
    if (NFRAG < NT) {          // fewer groups than waves: the first NFRAG/64 waves take one each (wave-uniform test)
        if (wv * 64 < NFRAG)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(reinterpret_cast<const char*>(g) + (unsigned)((wv * 64 + lane) * 16)),
                                             (__attribute__((address_space(3))) void*)(s + wv * 64), 16, 0, 0);
        return;
    }
    constexpr int NPT = NFRAG / NT > 0 ? NFRAG / NT : 1;
#pragma unroll
    for (int i0 = 0; i0 < NPT; i0 += 4) {
        const char* ga = reinterpret_cast<const char*>(g) + (unsigned)(((wv * NPT + i0) * 64 + lane) * 16);
        Frag* sa = s + (wv * NPT + i0) * 64;
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)ga, (__attribute__((address_space(3))) void*)sa, 16, 0, 0);
        if (i0 + 1 < NPT) __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)ga, (__attribute__((address_space(3))) void*)sa, 16, 1024, 0);
        if (i0 + 2 < NPT) __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)ga, (__attribute__((address_space(3))) void*)sa, 16, 2048, 0);
        if (i0 + 3 < NPT) __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)ga, (__attribute__((address_space(3))) void*)sa, 16, 3072, 0);
    }
}
__device__ __forceinline__ void wait_async_and_sync() {
    __builtin_amdgcn_s_waitcnt(0x0000);   // vmcnt(0) expcnt(0) lgkmcnt(0): this wave's copies have landed
    __syncthreads();
}

// Identity operand for transposing a 32x32 block through the matrix unit: with the block given as
// an A operand (rows r, contraction k; i.e. packed from accumulators that hold it as rows k, lane r),
// D = A * I comes out with rows r, lane k -- the transposed register layout.  Slab s of the identity
// B operand for lane (column l32, half h): element e is 1 where the contraction index equals l32.
template <typename T>
__device__ __forceinline__ void identity_frags(typename Tr<T>::Frag* id, int l32, int h) {
    constexpr int FE = Tr<T>::FE, SPB = 32 / Tr<T>::KW;
#pragma unroll
    for (int s = 0; s < SPB; ++s)
#pragma unroll
        for (int e = 0; e < FE; ++e) id[s][e] = (T)((acc_row(s * FE + e, h) == l32) ? 1.f : 0.f);
}
// out (rows r, lane k) = transpose of the 32x32 block whose operand fragments (rows r, contraction k) are a[0..SPB)
template <typename T>
__device__ __forceinline__ f32x16 transpose32(const typename Tr<T>::Frag* a, const typename Tr<T>::Frag* id) {
    f32x16 o = zero16();
#pragma unroll
    for (int s = 0; s < 32 / Tr<T>::KW; ++s) o = Tr<T>::mma(a[s], id[s], o);
    return o;
}

// Workspace carve-up shared by host launch code and kernels (byte offsets, 256-aligned).
struct FwdWorkspace {
    size_t kt, vt, dp, xinit, sd, kt2, dp2, cum, total;
};

// Layout of the caller's tensors: element strides of the batch, head and token index, for the
// [.,.,.,d] tensors (q, k, v, w, o and the gradients; d contiguous) and for the per-token scalars
// (beta, lse, log f and their gradients).  [B,H,L,d]: {H*L*d, L*d, d | H*L, L, 1};
// [B,L,H,d]: {L*H*d, d, H*d | L*H, 1, H}.  H = heads per batch entry (bh = b * H + h).
// bh0: the kernels of one launch may work on a slice of the heads (a backward that passes over the heads in
// groups to bound its workspace); they number their heads from 0, and head bh of the launch is head bh0 + bh of
// the caller's tensors.
// cu (device pointer, NULL for batches of one length): packed variable-length batches [T,H,d] / [T,H].  Batch
// entry b is the sequence of the tokens cu[b] .. cu[b+1]-1; its length replaces the launch's L in every bound
// (the launch's L and chunk count remain the STRIDES of the workspace arrays, sized for the longest sequence),
// and its tensors start at token cu[b] (vt, st are the token strides; vb, sb are not used).
struct UserLayout {
    long long vb, vh, vt, sb, sh, st;
    int H;
    int bh0;
    const int* cu;
};
__device__ __forceinline__ long long user_vec(const UserLayout& u, int bh, long long t) {
    bh += u.bh0;
    if (u.cu) return ((long long)u.cu[bh / u.H] + t) * u.vt + (bh % u.H) * u.vh;
    return (bh / u.H) * u.vb + (bh % u.H) * u.vh + t * u.vt;
}
__device__ __forceinline__ long long user_scl(const UserLayout& u, int bh, long long t) {
    bh += u.bh0;
    if (u.cu) return ((long long)u.cu[bh / u.H] + t) * u.st + (bh % u.H) * u.sh;
    return (bh / u.H) * u.sb + (bh % u.H) * u.sh + t * u.st;
}
// length of head bh's sequence: the launch's L, or the head's own in a packed batch
__device__ __forceinline__ int seq_len(const UserLayout& u, int bh, int L) {
    if (!u.cu) return L;
    const int b = (bh + u.bh0) / u.H;
    return u.cu[b + 1] - u.cu[b];
}

struct FwdParams {
    UserLayout ul;
    const void *q, *k, *v, *w, *beta;
    void* o;
    float* lse;
    void *kt, *vt, *dp;   // fragment-order tiles written by prep, read by the sweep
    void *kt2, *dp2;      // second level: keys carried to their super-block's right edge; -(I - P_superblock)
    void *dpt;            // backward only: -dP per chunk in the transposed arrangement (rows a, contraction b) = -dP[a][b]
    float *xinit, *sd;    // accumulator-order fp32 tiles
    const float* cum;     // PaTH-FoX only (else NULL): [BH][64*NC] cumulative log2 of the forget gates, log2(e) * sum_{s<=t} log f_s
    int B, H, L, NC;      // NC = number of 64-token chunks = ceil(L/64)
    float scale;
    // Backward only (NULL in the forward), all in fragment order:
    //   per chunk:  ktT (rows c, contraction s) = Kb[s][c];  vk (rows s, contraction c) = V[s][c] (I/O type);
    //               kt2T: the same arrangement of the second-level keys Kb2;
    //   per super-block: dpt2 (rows a, contraction b) = -(I - P_superblock)[a][b];
    //   per pair (query chunk i, key block), slot block_slot(i, c): xs (rows q, contraction c) and
    //               xsT (rows c, contraction q): the query state of chunk i as used against the block.
    void *ktT, *vk, *xs, *xsT, *kt2T, *dpt2;
    int emit_states;      // forward sweep of a training pair: also write xs and xsT
    // Backward only: per-chunk matrices of the transform, row-major 64x64 (operand type) --
    // fm = F[t][t'], gktm[s][t'] = strictLower(W K^T)[t'][s], nm = N, aim = A^{-1},
    // ytm[s][t] = Y[t][s]; utm [d][64]: utm[c][t] = U[t][c]; fp32: gm = W W^T, sdm[t][s] = Sd;
    // kbm [Lp][d]: boundary-adjusted keys Kb (rows past L zero); rm [d][d] per chunk: R_c of
    // the second level (operand type).
    void *fm, *gktm, *nm, *aim, *ytm, *utm, *kbm, *rm;
    float *gm, *sdm;
    // Sequence-parallel forward (one device's share of the ring of Sec. 3.5): the sweep's per-query registers --
    // the query state carried to the left edge of what has been attended so far, the unnormalised output, the
    // running maximum and row sum -- kept in memory between the calls.  ring: 0 = ordinary forward; 1 = sweep over
    // the device's own segment, leaving the registers in ring_state; 2 = one hop: the registers are loaded, every
    // key of an earlier segment (whose tiles kt2, vt, dp2 this structure then points at; NC = ITS chunk count) is
    // attended, and they are stored again.  NCq: chunks of the query side (ring = 2 only; else NC).
    float* ring_state;
    int ring, NCq;
};
// ring_state: per (head, query chunk, 32-query half) one record of RING_REC(d) floats, each quantity as the sweep
// holds it: [X: d/32 blocks][O: d/32 blocks] of 1024 floats (register g*4+r of lane l at g*256 + l*4 + r), then the
// running maximum and the row sum per lane (64 + 64), then (PaTH-FoX; zero otherwise) the sum of the gate logarithms
// of the segments passed so far, in base-2 units, once per lane (64).
__host__ __device__ constexpr size_t ring_rec_floats(int d) { return (size_t)2 * (d / 32) * 1024 + 192; }

// Key blocks of the backward, for query chunk i (own super-block I = i / SBC): the chunks
// SBC*I <= j < i one by one ("near"), and the super-blocks J < I as a whole ("far": the state is
// the one at the super-block's right edge, the keys are the second-level keys).  Per head the
// state arrays hold the near slots [0, NC*(SBC-1)) first, then the far slots.
__host__ __device__ __forceinline__ size_t far_base(int i) {
    const size_t I = (size_t)(i / SBC);
    return (size_t)SBC * (I * (I - 1) / 2) + (size_t)(i % SBC) * I;
}
__host__ __device__ __forceinline__ size_t num_block_slots(int NC) { return (size_t)NC * (SBC - 1) + far_base(NC); }
// slot of (query chunk i, block holding key chunk c < i)
__host__ __device__ __forceinline__ size_t block_slot(int i, int c, int NC) {
    const int jsb = (i / SBC) * SBC;
    if (c >= jsb) return (size_t)i * (SBC - 1) + (c - jsb);
    return (size_t)NC * (SBC - 1) + far_base(i) + (size_t)(c / SBC);
}

}  // namespace path
