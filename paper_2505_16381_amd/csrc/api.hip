// C ABI of the PaTH attention library: argument checks, workspace carve-up,
// kernel launches on the caller's stream.  No allocation, no synchronisation.
#include "../../include/path_attn.h"
#include "path_common.h"

namespace path {
hipError_t launch_prep_fwd(const FwdParams& p, int d, int is_bf16, hipStream_t stream);
hipError_t launch_attn_fwd(const FwdParams& p, int d, int is_bf16, hipStream_t stream);

static size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

static bool shape_ok(int B, int H, int L, int d) {
    if (B < 1 || H < 1 || L < 1) return false;
    if (d != 64 && d != 128) return false;
    if ((long long)B * H > 65535) return false;               // grid.y of the chunk kernels
    if ((long long)B * H * L > (1LL << 31) / 4) return false;  // 32-bit tile counters
    return true;
}

static FwdWorkspace fwd_workspace(int B, int H, int L, int d, size_t es) {
    const size_t BH = (size_t)B * H, NC = (size_t)(L + CHUNK - 1) / CHUNK, Lp = NC * CHUNK;
    FwdWorkspace w;
    size_t off = 0;
    w.kt = off;    off = align256(off + BH * Lp * d * es);
    w.vt = off;    off = align256(off + BH * Lp * d * es);
    w.dp = off;    off = align256(off + BH * NC * d * d * es);
    w.xinit = off; off = align256(off + BH * Lp * d * 4);
    w.sd = off;    off = align256(off + BH * NC * CHUNK * CHUNK * 4);
    w.total = off;
    return w;
}
}  // namespace path

using namespace path;

extern "C" const char* path_status_str(path_status_t s) {
    switch (s) {
        case PATH_OK: return "PATH_OK";
        case PATH_ERR_NULL: return "PATH_ERR_NULL";
        case PATH_ERR_SHAPE: return "PATH_ERR_SHAPE";
        case PATH_ERR_DTYPE: return "PATH_ERR_DTYPE";
        case PATH_ERR_UNSUPPORTED: return "PATH_ERR_UNSUPPORTED";
        case PATH_ERR_WORKSPACE: return "PATH_ERR_WORKSPACE";
        case PATH_ERR_HIP: return "PATH_ERR_HIP";
        case PATH_ERR_ALIGN: return "PATH_ERR_ALIGN";
    }
    return "PATH_ERR_UNKNOWN";
}

extern "C" size_t path_attn_workspace_bytes(int B, int H, int L, int d, path_dtype_t dt, int for_backward) {
    if (!shape_ok(B, H, L, d)) return 0;
    if (dt != PATH_F32 && dt != PATH_BF16) return 0;
    const size_t es = dt == PATH_BF16 ? 2 : 4;
    if (for_backward) return 0;   // backward: not built yet
    return fwd_workspace(B, H, L, d, es).total;
}

extern "C" path_status_t path_attn_fwd_workspace_layout(int B, int H, int L, int d, path_dtype_t dt,
                                                        size_t offsets[6]) {
    if (!offsets) return PATH_ERR_NULL;
    if (dt != PATH_F32 && dt != PATH_BF16) return PATH_ERR_DTYPE;
    if (!shape_ok(B, H, L, d)) return PATH_ERR_SHAPE;
    const FwdWorkspace ws = fwd_workspace(B, H, L, d, dt == PATH_BF16 ? 2 : 4);
    offsets[0] = ws.kt; offsets[1] = ws.vt; offsets[2] = ws.dp; offsets[3] = ws.xinit; offsets[4] = ws.sd;
    offsets[5] = ws.total;
    return PATH_OK;
}

static bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) != 0; }

extern "C" path_status_t path_attn_fwd(const void* q, const void* k, const void* v, const void* w,
                                       const void* beta, void* o, float* lse, int B, int H, int L, int d,
                                       int causal, float scale, path_dtype_t dt, void* workspace,
                                       size_t workspace_bytes, void* stream) {
    if (!q || !k || !v || !w || !beta || !o || !lse || !workspace) return PATH_ERR_NULL;
    if (dt != PATH_F32 && dt != PATH_BF16) return PATH_ERR_DTYPE;
    if (!shape_ok(B, H, L, d)) return PATH_ERR_SHAPE;
    if (!causal) return PATH_ERR_UNSUPPORTED;
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(w) || misaligned(o)) return PATH_ERR_ALIGN;
    const size_t es = dt == PATH_BF16 ? 2 : 4;
    const FwdWorkspace ws = fwd_workspace(B, H, L, d, es);
    if (workspace_bytes < ws.total || (reinterpret_cast<uintptr_t>(workspace) & 255)) return PATH_ERR_WORKSPACE;

    unsigned char* base = static_cast<unsigned char*>(workspace);
    FwdParams p;
    p.q = q; p.k = k; p.v = v; p.w = w; p.beta = beta; p.o = o; p.lse = lse;
    p.kt = base + ws.kt; p.vt = base + ws.vt; p.dp = base + ws.dp;
    p.xinit = reinterpret_cast<float*>(base + ws.xinit);
    p.sd = reinterpret_cast<float*>(base + ws.sd);
    p.B = B; p.H = H; p.L = L; p.NC = (L + CHUNK - 1) / CHUNK; p.scale = scale;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (launch_prep_fwd(p, d, dt == PATH_BF16, st) != hipSuccess) return PATH_ERR_HIP;
    if (launch_attn_fwd(p, d, dt == PATH_BF16, st) != hipSuccess) return PATH_ERR_HIP;
    return PATH_OK;
}

extern "C" path_status_t path_attn_bwd(const void* q, const void* k, const void* v, const void* w,
                                       const void* beta, const void* o, const float* lse, const void* d_o,
                                       void* dq, void* dk, void* dv, void* dw, void* dbeta, int B, int H,
                                       int L, int d, int causal, float scale, path_dtype_t dt,
                                       void* workspace, size_t workspace_bytes, void* stream) {
    (void)q; (void)k; (void)v; (void)w; (void)beta; (void)o; (void)lse; (void)d_o; (void)dq; (void)dk;
    (void)dv; (void)dw; (void)dbeta; (void)B; (void)H; (void)L; (void)d; (void)causal; (void)scale;
    (void)dt; (void)workspace; (void)workspace_bytes; (void)stream;
    return PATH_ERR_UNSUPPORTED;
}
