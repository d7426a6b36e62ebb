// PaTH-FoX helper (paper Sec. 2.2, "Extension: PaTH-FoX"): the gate product prod_{s=j+1..i} f_s
// enters the logit as c_i - c_j with c_t = sum_{s<=t} log f_s.  One kernel does both scans that
// the forward and the backward need, per head, in fp32:
//   forward:  cum[t]   = scale_out * sum_{s<=t} x[s]      (inclusive; x = log f, scale_out = log2 e)
//   backward: dlogf[s] = sum_{t<s} (y[t] - r[t])          (exclusive; y = column sums, r = row sums of the logit gradient)
// One workgroup per head; a thread owns a contiguous run of the row.
#include "path_common.h"
#include "fox_decl.h"

namespace path {

template <typename TIN, typename TOUT>
__global__ __launch_bounds__(256) void fox_scan_kernel(ScanArgs a) {
    __shared__ float part[256];
    const int bh = blockIdx.x, tid = threadIdx.x;
    // packed batches: this head's own length bounds what is read, and what is written to a tensor of the caller
    const int Lown = seq_len(a.ul, bh, a.n_in);
    const int n_in = a.n_in < Lown ? a.n_in : Lown, n_out = (a.out_user && Lown < a.n_out) ? Lown : a.n_out;
    const int per = (n_out + 255) / 256;
    const int t0 = tid * per, t1 = (t0 + per < n_out) ? t0 + per : n_out;
    const TIN* x = reinterpret_cast<const TIN*>(a.in) + (a.in_user ? user_scl(a.ul, bh, 0) : (long long)bh * a.in_stride);
    TOUT* y = reinterpret_cast<TOUT*>(a.out) + (a.out_user ? user_scl(a.ul, bh, 0) : (long long)bh * a.out_stride);
    const long long xs = a.in_user ? a.ul.st : 1, ys = a.out_user ? a.ul.st : 1;        // token strides
    const float* mi = a.minus ? a.minus + (size_t)bh * a.in_stride : nullptr;
    auto val = [&](int t) { return (t < n_in) ? (float)x[t * xs] - (mi ? mi[t] : 0.f) : 0.f; };
    float s = 0.f;
    for (int t = t0; t < t1; ++t) s += val(t);
    part[tid] = s;
    __syncthreads();
    // exclusive scan of the 256 partial sums (Hillis-Steele on a copy)
    float run = s;
    for (int off = 1; off < 256; off <<= 1) {
        const float other = (tid >= off) ? part[tid - off] : 0.f;
        __syncthreads();
        run += other;
        part[tid] = run;
        __syncthreads();
    }
    float acc = run - s;                       // sum of everything before this thread's run
    for (int t = t0; t < t1; ++t) {
        const float v = val(t);
        if (a.inclusive) { acc += v; y[t * ys] = (TOUT)(acc * a.scale_out); }
        else { y[t * ys] = (TOUT)(acc * a.scale_out); acc += v; }
    }
}

hipError_t launch_fox_scan(const ScanArgs& a, int BH, int in_type, int out_type, hipStream_t st) {
    // types: 0 = float, 1 = bf16
    if (in_type == 0 && out_type == 0) hipLaunchKernelGGL((fox_scan_kernel<float, float>), dim3(BH), dim3(256), 0, st, a);
    else if (in_type == 1 && out_type == 0) hipLaunchKernelGGL((fox_scan_kernel<bf16_t, float>), dim3(BH), dim3(256), 0, st, a);
    else if (in_type == 0 && out_type == 1) hipLaunchKernelGGL((fox_scan_kernel<float, bf16_t>), dim3(BH), dim3(256), 0, st, a);
    else hipLaunchKernelGGL((fox_scan_kernel<bf16_t, bf16_t>), dim3(BH), dim3(256), 0, st, a);
    return hipGetLastError();
}

}  // namespace path
