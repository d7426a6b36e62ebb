// Query states for the backward of PaTH attention: the right-to-left sweep of the forward
// (paper Sec. 3.3 workflow) without logits or outputs.  For every query chunk i it writes the
// state used against each key block of the backward -- the chunks of i's own super-block one
// by one, the super-blocks further left as a whole (second blocking level, see prep2_fwd.hip) --
// as two fragment-order tiles per (chunk, block) pair: xs (rows q, contraction c), which is
// the operand copy of the state itself, and xsT (rows c, contraction q), its transpose taken
// through the matrix unit (with 16-bit operands only for the far blocks: the near blocks'
// consumer reads xs with the transposing LDS read instead).
//
// One workgroup = 4 waves = two query chunks; wave w owns the 32-query half (w & 1) of chunk
// 2*tile + (w >> 1).  The state keeps an fp32 master; per step one -dP tile (chunk or
// super-block level) is streamed through LDS, double buffered.
#include "path_common.h"

namespace path {

template <typename TIO, int D> struct StatesCfg {
    typedef typename Compute<TIO>::type T;
    static constexpr int DP_FRAGS = D * D / Tr<T>::FE;
    static constexpr size_t smem_bytes = (size_t)2 * DP_FRAGS * 16;
};

template <typename TIO, int D>
__global__ __launch_bounds__(256) void bwd_states_kernel(FwdParams p) {
    using C = StatesCfg<TIO, D>;
    using T = typename C::T;
    using Frag = typename Tr<T>::Frag;
    constexpr int KW = Tr<T>::KW, SPB = 32 / KW, DB = D / 32, DS = D / KW, QS = CHUNK / KW, DPF = C::DP_FRAGS;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    Frag* sP = reinterpret_cast<Frag*>(smem);

    const int BH = p.B * p.H, NC = p.NC;
    const int ntiles = (NC + 1) / 2;
    // (divisions run on the vector unit; the results, uniform over the workgroup, go back to scalar registers)
    const int tile = __builtin_amdgcn_readfirstlane(ntiles - 1 - (int)(blockIdx.x / BH));      // heaviest (right-most) tiles first
    const int bh = __builtin_amdgcn_readfirstlane((int)(blockIdx.x % BH));
    const int tid = threadIdx.x, lane = tid & 63, wv = __builtin_amdgcn_readfirstlane(tid >> 6), h = lane >> 5, l32 = lane & 31;
    const int NCown = (seq_len(p.ul, bh, p.L) + CHUNK - 1) / CHUNK;   // this head's own chunks (NC: per head in the workspace arrays)
    if (tile * 2 >= NCown) return;
    const int cq = tile * 2 + (wv >> 1), qb = wv & 1;
    const bool active = cq < NCown;
    const int ctop = (tile * 2 + 1 < NCown) ? tile * 2 + 1 : NCown - 1;     // right-most chunk of the tile
    const int I = (tile * 2) / SBC, jsb = I * SBC;                    // both chunks lie in super-block I
    const int nnear = ctop - jsb;                                     // near steps: j = ctop-1 .. jsb
    const int nsteps = nnear + I;                                     // then far steps: J = I-1 .. 0
    const size_t nslots = num_block_slots(NC);
    const int nsb = (NC + SBC - 1) / SBC;

    f32x16 Xm[DB];
    Frag Xb[DS];
#pragma unroll
    for (int b = 0; b < DB; ++b) {
        Xm[b] = zero16();
        if (active) {
            const float* xs = p.xinit + (((size_t)bh * NC + cq) * 2 + qb) * (size_t)DB * 1024 + (size_t)b * 1024;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const f32x4 v4 = *reinterpret_cast<const f32x4*>(xs + g * 256 + lane * 4);
#pragma unroll
                for (int r = 0; r < 4; ++r) Xm[b][4 * g + r] = v4[r];
            }
        }
        pack_block<T>(Xm[b], Xb + b * SPB);
    }
    Frag idf[SPB];
    identity_frags<T>(idf, l32, h);

    const T* dpg = reinterpret_cast<const T*>(p.dp) + (size_t)bh * NC * D * D;
    const T* dp2g = reinterpret_cast<const T*>(p.dp2) + (size_t)bh * nsb * D * D;
    // the -dP tile applied after step k (none after the left-most chunk / super-block)
    auto issue = [&](int k) {
        const T* src;
        if (k < nnear) {
            const int j = ctop - 1 - k;
            if (j == 0) return;
            src = dpg + (size_t)j * D * D;
        } else {
            const int J = I - 1 - (k - nnear);
            if (J == 0) return;
            src = dp2g + (size_t)J * D * D;
        }
        async_copy_tile<256, DPF>(reinterpret_cast<const Frag*>(src), sP + (size_t)(k & 1) * DPF, tid, wv);
    };

    if (nsteps > 0) issue(0);
    for (int k = 0; k < nsteps; ++k) {
        wait_async_and_sync();                 // tile k has landed; everyone is done with tile k-1
        if (k + 1 < nsteps) issue(k + 1);
        const bool near = k < nnear;
        const int c = near ? ctop - 1 - k : (I - 1 - (k - nnear)) * SBC;     // a key chunk of the block
        if (!active || (near && c >= cq)) continue;
        {
            const size_t slot = ((size_t)bh * nslots + block_slot(cq, c, NC)) * (size_t)CHUNK * D;
            Frag* xd = reinterpret_cast<Frag*>(reinterpret_cast<T*>(p.xs) + slot);
#pragma unroll
            for (int s = 0; s < DS; ++s) __builtin_nontemporal_store(Xb[s], &xd[((size_t)qb * DS + s) * 64 + lane]);
            Frag* xt = reinterpret_cast<Frag*>(reinterpret_cast<T*>(p.xsT) + slot);
            if (sizeof(T) == 4 || !near)       // (16-bit operands: the near blocks' consumer transposes xs itself)
#pragma unroll
            for (int b = 0; b < DB; ++b) {
                const f32x16 tr = transpose32<T>(Xb + b * SPB, idf);     // rows q, lane c (block b)
                Frag fr[SPB];
                pack_block<T>(tr, fr);
#pragma unroll
                for (int s2 = 0; s2 < SPB; ++s2) __builtin_nontemporal_store(fr[s2], &xt[((size_t)b * QS + qb * SPB + s2) * 64 + lane]);
            }
        }
        if (c > 0) {                           // X <- X (I - dP) of the chunk / super-block just left
            const Frag* tp = sP + (size_t)(k & 1) * DPF;
#pragma unroll
            for (int b = 0; b < DB; ++b)
#pragma unroll
                for (int s0 = 0; s0 < DS; s0 += 4) {
                    Frag pa[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) pa[u] = tp[(b * DS + s0 + u) * 64 + lane];
#pragma unroll
                    for (int u = 0; u < 4; ++u) Xm[b] = Tr<T>::mma(pa[u], Xb[s0 + u], Xm[b]);
                }
#pragma unroll
            for (int b = 0; b < DB; ++b) pack_block<T>(Xm[b], Xb + b * SPB);
        }
    }
}

template <typename TIO, int D>
static hipError_t launch_states_t(const FwdParams& p, hipStream_t stream) {
    using C = StatesCfg<TIO, D>;
    // set once per process; a function-local static is initialised under the language's own lock
    static const hipError_t attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&bwd_states_kernel<TIO, D>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::smem_bytes);
    if (attr_err != hipSuccess) return attr_err;
    const int ntiles = (p.NC + 1) / 2;
    const size_t bytes = C::smem_bytes;
    hipLaunchKernelGGL((bwd_states_kernel<TIO, D>), dim3((unsigned)(ntiles * p.B * p.H)), dim3(256), bytes, stream, p);
    return hipGetLastError();
}

hipError_t launch_attn_states(const FwdParams& p, int d, int is_bf16, hipStream_t stream) {
    if (is_bf16) return d == 64 ? launch_states_t<bf16_t, 64>(p, stream) : launch_states_t<bf16_t, 128>(p, stream);
    return d == 64 ? launch_states_t<float, 64>(p, stream) : launch_states_t<float, 128>(p, stream);
}

}  // namespace path
