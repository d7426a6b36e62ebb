// C ABI of the PaTH attention library: argument checks, workspace carve-up,
// kernel launches on the caller's stream.  No allocation, no synchronisation.
#include <cstdio>
#include "../../include/path_attn.h"
#include <mutex>
#include <type_traits>

#include "path_common.h"

namespace path {
hipError_t launch_prep_fwd(const FwdParams& p, int d, int is_bf16, hipStream_t stream);

hipError_t launch_prep2_fwd(const FwdParams& p, int d, int is_bf16, hipStream_t stream);
hipError_t launch_attn_fwd2(const FwdParams& p, int d, int is_bf16, hipStream_t stream);
hipError_t launch_ring_finish(const FwdParams& p, int d, int is_bf16, hipStream_t stream);
hipError_t launch_attn_states(const FwdParams& p, int d, int is_bf16, hipStream_t stream);
}  // namespace path
#include "bwd_decl.h"
#include "decode_decl.h"
#include "fox_decl.h"
namespace path {

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
    const size_t NSB = (NC + SBC - 1) / SBC;
    w.kt2 = off;    off = align256(off + BH * Lp * d * es);
    w.dp2 = off;    off = align256(off + BH * NSB * d * d * es);
    w.cum = off;    off = align256(off + BH * Lp * 4);          // PaTH-FoX: cumulative log2 gates
    w.total = off;
    return w;
}
// Backward workspace: the forward's five regions first (same carve-up), then everything else.
struct BwdWorkspace {
    FwdWorkspace f;
    size_t ktT, vk, dpt, doq, doT, xs, xsT, gs, fm, gktm, nm, aim, ytm, utm, gm, sdm, delta, lse2p, dqb, dkb, dvp, ddp;
    size_t kt2T, dpt2, kbm, rm, dk2, dchain, t1;       // second level and its adjoint
    size_t dcol, drow;                                 // PaTH-FoX: column and row sums of the logit gradient
    size_t dpd, pd, dsd, df, dy, dn, dgk, rr, mm, dgs, du, dqf, dkf, dwf, dbf, total;
};

static BwdWorkspace bwd_workspace(int B, int H, int L, int d, size_t es) {
    const size_t BH = (size_t)B * H, NC = (size_t)(L + CHUNK - 1) / CHUNK, Lp = NC * CHUNK;
    const size_t nslots = num_block_slots((int)NC), NSB = (NC + SBC - 1) / SBC;
    BwdWorkspace w;
    w.f = fwd_workspace(B, H, L, d, es);
    size_t off = w.f.total;
    auto take = [&](size_t& field, size_t bytes) { field = off; off = align256(off + bytes); };
    // (the transposed key tiles ktT, kt2T exist for fp32 operands only: the 16-bit adjoint scan transposes in LDS)
    take(w.ktT, (es == 4 ? 1 : 0) * BH * Lp * d * es);
    for (size_t* f : {&w.vk, &w.doq, &w.doT}) take(*f, BH * Lp * d * es);
    take(w.dpt, (es == 4 ? 1 : 0) * BH * NC * d * d * es);       // (fp32 operands only, like ktT)
    for (size_t* f : {&w.xs, &w.xsT, &w.gs}) take(*f, BH * nslots * CHUNK * d * es);
    take(w.kt2T, (es == 4 ? 1 : 0) * BH * Lp * d * es);
    take(w.dpt2, (es == 4 ? 1 : 0) * BH * NSB * d * d * es);
    take(w.kbm, BH * Lp * d * es);
    take(w.rm, BH * NC * d * d * es);
    take(w.dk2, BH * Lp * d * 4);
    take(w.dchain, BH * (NC + 1) * d * d * 4);
    // (regions only the fp32-operand path uses -- the second level's chain and the chunk-transform adjoint as
    //  staged products -- have size zero for 2-byte operands, whose fused kernels keep these in LDS)
    const size_t staged = es == 4 ? 1 : 0;
    take(w.t1, staged * BH * NC * d * CHUNK * 4);
    take(w.dcol, BH * Lp * 4);
    take(w.drow, BH * Lp * 4);
    for (size_t* f : {&w.fm, &w.gktm, &w.nm, &w.aim, &w.ytm}) take(*f, BH * NC * 4096 * es);
    take(w.utm, BH * NC * d * CHUNK * es);
    take(w.gm, BH * NC * 4096 * 4);
    take(w.sdm, BH * NC * 4096 * 4);
    take(w.delta, BH * Lp * 4);
    take(w.lse2p, BH * Lp * 4);
    for (size_t* f : {&w.dqb, &w.dkb, &w.dvp}) take(*f, BH * Lp * d * 4);
    take(w.ddp, BH * NC * d * d * 4);
    for (size_t* f : {&w.dpd, &w.pd, &w.dsd, &w.df, &w.dy, &w.dn, &w.dgk, &w.rr, &w.mm, &w.dgs}) take(*f, staged * BH * NC * 4096 * 4);
    for (size_t* f : {&w.du, &w.dqf, &w.dkf, &w.dwf}) take(*f, staged * BH * Lp * d * 4);
    take(w.dbf, staged * BH * Lp * 4);
    w.total = off;
    return w;
}
}  // namespace path

using namespace path;

// Last HIP failure seen by an entry point on this thread: "<step>: <hip error name>".
static thread_local char g_last_error[160] = "";

static bool hip_ok(hipError_t e, const char* step) {
    if (e == hipSuccess) return true;
    snprintf(g_last_error, sizeof g_last_error, "%s: %s (%d)", step, hipGetErrorName(e), static_cast<int>(e));
    return false;
}

// The runtime keeps one "last error" per thread, shared with every other user of it in the process; a
// value left there by someone else must not be taken for a failed launch of ours.  It is cleared on
// entry and noted, so that the caller can still see it.
static void clear_inherited_error() {
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        snprintf(g_last_error, sizeof g_last_error, "inherited and cleared on entry: %s (%d)", hipGetErrorName(e),
                 static_cast<int>(e));
}

extern "C" const char* path_attn_last_error(void) { return g_last_error; }

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
    if (for_backward) return bwd_workspace(B, H, L, d, es).total;
    return fwd_workspace(B, H, L, d, es).total;
}

static int heads_per_pass(int B, int H, int L, int d, size_t es, size_t bytes);

extern "C" size_t path_attn_bwd_workspace_bytes_for_heads(int B, int H, int L, int d, path_dtype_t dt, int heads) {
    if (!shape_ok(B, H, L, d) || (dt != PATH_F32 && dt != PATH_BF16) || heads < 1) return 0;
    if (heads > B * H) heads = B * H;
    return bwd_workspace(1, heads, L, d, dt == PATH_BF16 ? 2 : 4).total;
}

extern "C" int path_attn_bwd_heads_per_pass(int B, int H, int L, int d, path_dtype_t dt, size_t workspace_bytes) {
    if (!shape_ok(B, H, L, d) || (dt != PATH_F32 && dt != PATH_BF16)) return 0;
    return heads_per_pass(B, H, L, d, dt == PATH_BF16 ? 2 : 4, workspace_bytes);
}

extern "C" path_status_t path_attn_fwd_workspace_layout(int B, int H, int L, int d, path_dtype_t dt,
                                                        size_t offsets[6]) {
    if (!offsets) return PATH_ERR_NULL;
    if (dt != PATH_F32 && dt != PATH_BF16) return PATH_ERR_DTYPE;
    if (!shape_ok(B, H, L, d)) return PATH_ERR_SHAPE;
    const FwdWorkspace ws = fwd_workspace(B, H, L, d, dt == PATH_BF16 ? 2 : 4);
    offsets[0] = ws.kt; offsets[1] = ws.vt; offsets[2] = ws.dp; offsets[3] = ws.xinit; offsets[4] = ws.sd;
    offsets[5] = ws.kt2;   // end of the fifth region
    return PATH_OK;
}

static bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) != 0; }

// Strides of the caller's tensors for one of the two layouts of the ABI.
static bool layout_ok(int layout) { return layout == PATH_LAYOUT_BHLD || layout == PATH_LAYOUT_BLHD; }
static UserLayout layout_of(int layout, int H, int L, int d) {
    UserLayout u;
    u.H = H;
    u.bh0 = 0;
    u.cu = nullptr;
    if (layout == PATH_LAYOUT_BLHD) {
        u.vb = (long long)L * H * d; u.vh = d; u.vt = (long long)H * d;
        u.sb = (long long)L * H; u.sh = 1; u.st = H;
    } else {
        u.vb = (long long)H * L * d; u.vh = (long long)L * d; u.vt = d;
        u.sb = (long long)H * L; u.sh = L; u.st = 1;
    }
    return u;
}

static path_status_t fwd_setup(FwdParams& p, const UserLayout& ul, int B, int H, int L, int d, path_dtype_t dt, void* workspace,
                               size_t workspace_bytes) {
    if (!workspace) return PATH_ERR_NULL;
    if (dt != PATH_F32 && dt != PATH_BF16) return PATH_ERR_DTYPE;
    if (!shape_ok(B, H, L, d)) return PATH_ERR_SHAPE;
    const FwdWorkspace ws = fwd_workspace(B, H, L, d, dt == PATH_BF16 ? 2 : 4);
    if (workspace_bytes < ws.total || (reinterpret_cast<uintptr_t>(workspace) & 255)) return PATH_ERR_WORKSPACE;
    unsigned char* base = static_cast<unsigned char*>(workspace);
    p.kt = base + ws.kt; p.vt = base + ws.vt; p.dp = base + ws.dp;
    p.xinit = reinterpret_cast<float*>(base + ws.xinit);
    p.sd = reinterpret_cast<float*>(base + ws.sd);
    p.kt2 = base + ws.kt2; p.dp2 = base + ws.dp2;
    p.dpt = nullptr;                                         // transposed -dP tile: backward only
    p.cum = nullptr;                                         // set by the PaTH-FoX entry points
    p.B = B; p.H = H; p.L = L; p.NC = (L + CHUNK - 1) / CHUNK;
    p.ul = ul;
    return PATH_OK;
}

// PaTH-FoX: cum[t] = log2(e) * sum_{s<=t} log f_s per head, fp32, padded to whole chunks.
static hipError_t launch_gate_sums(const void* log_f, const UserLayout& ul, float* cum, int B, int H, int L, path_dtype_t dt, hipStream_t st) {
    const int Lp = ((L + CHUNK - 1) / CHUNK) * CHUNK;
    ScanArgs a{log_f, nullptr, cum, L, Lp, L, Lp, 1, 1.44269504088896340736f, 1, 0, ul};
    return launch_fox_scan(a, B * H, dt == PATH_BF16 ? 1 : 0, 0, st);
}

// Forward of plain PaTH (log_f == NULL) and of PaTH-FoX: stage 0 = everything, 1 = the two transforms
// (and the gate sums), 2 = the sweep (with_gates tells whether gate sums are in the workspace).
static path_status_t fwd_impl(int stage, const UserLayout& ul, const void* q, const void* k, const void* v, const void* w,
                              const void* beta, const void* log_f, int with_gates, void* o, float* lse, int B, int H, int L,
                              int d, int causal, float scale, path_dtype_t dt, void* workspace, size_t workspace_bytes,
                              void* stream) {
    if (stage != 2 && (!q || !k || !v || !w || !beta)) return PATH_ERR_NULL;
    if (stage != 1 && (!o || !lse)) return PATH_ERR_NULL;
    if (!workspace) return PATH_ERR_NULL;
    if (dt != PATH_F32 && dt != PATH_BF16) return PATH_ERR_DTYPE;
    if (!shape_ok(B, H, L, d)) return PATH_ERR_SHAPE;
    if (!causal || (stage != 1 && !(scale > 0.f))) return PATH_ERR_UNSUPPORTED;     // the online softmax tracks max(s) * scale
    FwdParams p = {};
    const path_status_t st = fwd_setup(p, ul, B, H, L, d, dt, workspace, workspace_bytes);
    if (st != PATH_OK) return st;
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(w) || misaligned(o)) return PATH_ERR_ALIGN;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    const FwdWorkspace ws = fwd_workspace(B, H, L, d, dt == PATH_BF16 ? 2 : 4);
    float* cum = reinterpret_cast<float*>(static_cast<unsigned char*>(workspace) + ws.cum);
    clear_inherited_error();
    if (stage != 2) {
        p.q = q; p.k = k; p.v = v; p.w = w; p.beta = beta;
        if (!hip_ok(launch_prep_fwd(p, d, dt == PATH_BF16, hs), "chunk transform")) return PATH_ERR_HIP;
        // (the sweep reads the second level only when there is a super-block to the left; the key
        // prefill of the decode path reads it always)
        if (!hip_ok(launch_prep2_fwd(p, d, dt == PATH_BF16, hs), "second-level transform")) return PATH_ERR_HIP;
        if (log_f && !hip_ok(launch_gate_sums(log_f, ul, cum, B, H, L, dt, hs), "gate sums")) return PATH_ERR_HIP;
    }
    if (stage != 1) {
        p.o = o; p.lse = lse; p.scale = scale; p.cum = (log_f || with_gates) ? cum : nullptr;
        if (!hip_ok(launch_attn_fwd2(p, d, dt == PATH_BF16, hs), "forward sweep")) return PATH_ERR_HIP;
    }
    return PATH_OK;
}

extern "C" path_status_t path_attn_fwd_prep(const void* q, const void* k, const void* v, const void* w,
                                            const void* beta, int B, int H, int L, int d, path_dtype_t dt,
                                            void* workspace, size_t workspace_bytes, void* stream) {
    return fwd_impl(1, layout_of(PATH_LAYOUT_BHLD, H, L, d), q, k, v, w, beta, nullptr, 0, nullptr, nullptr, B, H, L, d, 1, 1.f, dt,
                    workspace, workspace_bytes, stream);
}

extern "C" path_status_t path_attn_fwd_sweep(void* o, float* lse, int B, int H, int L, int d, float scale,
                                             path_dtype_t dt, void* workspace, size_t workspace_bytes,
                                             void* stream) {
    return fwd_impl(2, layout_of(PATH_LAYOUT_BHLD, H, L, d), nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0, o, lse, B, H, L, d, 1,
                    scale, dt, workspace, workspace_bytes, stream);
}

extern "C" path_status_t path_attn_fwd(const void* q, const void* k, const void* v, const void* w,
                                       const void* beta, void* o, float* lse, int B, int H, int L, int d,
                                       int causal, float scale, path_dtype_t dt, void* workspace,
                                       size_t workspace_bytes, void* stream) {
    return fwd_impl(0, layout_of(PATH_LAYOUT_BHLD, H, L, d), q, k, v, w, beta, nullptr, 0, o, lse, B, H, L, d, causal, scale, dt,
                    workspace, workspace_bytes, stream);
}

// ---- sequence-parallel forward: one device's share of the ring (paper Sec. 3.5) ------------------------------
extern "C" size_t path_attn_ring_state_bytes(int B, int H, int L, int d) {
    if (!shape_ok(B, H, L, d)) return 0;
    const size_t NC = (size_t)(L + CHUNK - 1) / CHUNK;
    return (size_t)B * H * NC * 2 * ring_rec_floats(d) * sizeof(float);
}

// The regions of a segment's workspace that a hop reads -- what has to travel between devices: second-level keys,
// values, super-block products and (PaTH-FoX) the gate sums, as byte offsets into the workspace and lengths.
extern "C" path_status_t path_attn_ring_regions(int B, int H, int L, int d, path_dtype_t dt, size_t offsets[4], size_t bytes[4]) {
    if (!offsets || !bytes) return PATH_ERR_NULL;
    if (dt != PATH_F32 && dt != PATH_BF16) return PATH_ERR_DTYPE;
    if (!shape_ok(B, H, L, d)) return PATH_ERR_SHAPE;
    const size_t es = dt == PATH_BF16 ? 2 : 4;
    const FwdWorkspace ws = fwd_workspace(B, H, L, d, es);
    const size_t BH = (size_t)B * H, NC = (size_t)(L + CHUNK - 1) / CHUNK, Lp = NC * CHUNK, NSB = (NC + SBC - 1) / SBC;
    offsets[0] = ws.kt2; bytes[0] = BH * Lp * d * es;
    offsets[1] = ws.vt;  bytes[1] = BH * Lp * d * es;
    offsets[2] = ws.dp2; bytes[2] = BH * NSB * d * d * es;
    offsets[3] = ws.cum; bytes[3] = BH * Lp * 4;
    return PATH_OK;
}

extern "C" path_status_t path_attn_ring_local(const void* q, const void* k, const void* v, const void* w, const void* beta,
                                              const void* log_f, void* state, int B, int H, int L, int d, float scale,
                                              path_dtype_t dt, void* workspace, size_t workspace_bytes, void* stream) {
    if (!q || !k || !v || !w || !beta || !state || !workspace) return PATH_ERR_NULL;
    if (!(scale > 0.f)) return PATH_ERR_UNSUPPORTED;
    FwdParams p = {};
    const path_status_t st = fwd_setup(p, layout_of(PATH_LAYOUT_BHLD, H, L, d), B, H, L, d, dt, workspace, workspace_bytes);
    if (st != PATH_OK) return st;
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(w) || misaligned(state)) return PATH_ERR_ALIGN;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    clear_inherited_error();
    p.q = q; p.k = k; p.v = v; p.w = w; p.beta = beta;
    if (!hip_ok(launch_prep_fwd(p, d, dt == PATH_BF16, hs), "chunk transform")) return PATH_ERR_HIP;
    if (!hip_ok(launch_prep2_fwd(p, d, dt == PATH_BF16, hs), "second-level transform")) return PATH_ERR_HIP;
    if (log_f) {      // PaTH-FoX: gate sums counted from the segment's start
        float* cum = reinterpret_cast<float*>(static_cast<unsigned char*>(workspace) + fwd_workspace(B, H, L, d, dt == PATH_BF16 ? 2 : 4).cum);
        if (!hip_ok(launch_gate_sums(log_f, p.ul, cum, B, H, L, dt, hs), "gate sums")) return PATH_ERR_HIP;
        p.cum = cum;
    }
    p.scale = scale; p.ring = 1; p.ring_state = static_cast<float*>(state); p.NCq = p.NC;
    if (!hip_ok(launch_attn_fwd2(p, d, dt == PATH_BF16, hs), "sweep of the own segment")) return PATH_ERR_HIP;
    return PATH_OK;
}

extern "C" path_status_t path_attn_ring_hop(void* state, int B, int H, int Lq, const void* remote_workspace,
                                            size_t remote_workspace_bytes, int Lk, int d, int with_gates, float scale,
                                            path_dtype_t dt, void* stream) {
    if (!state || !remote_workspace) return PATH_ERR_NULL;
    if (!(scale > 0.f)) return PATH_ERR_UNSUPPORTED;
    if (!shape_ok(B, H, Lq, d)) return PATH_ERR_SHAPE;
    if (Lk % CHUNK != 0) {      // padded keys of a ragged segment would be attended: only the LAST segment may be ragged, and it is nobody's earlier segment
        snprintf(g_last_error, sizeof g_last_error, "path_attn_ring_hop: the earlier segment's length %d is not a multiple of 64", Lk);
        return PATH_ERR_SHAPE;
    }
    FwdParams p = {};
    // the earlier segment's tiles: its workspace as path_attn_ring_local laid it out (the sweep reads kt2, vt, dp2)
    const path_status_t st = fwd_setup(p, layout_of(PATH_LAYOUT_BHLD, H, Lk, d), B, H, Lk, d, dt, const_cast<void*>(remote_workspace),
                                       remote_workspace_bytes);
    if (st != PATH_OK) return st;
    if (misaligned(state)) return PATH_ERR_ALIGN;
    clear_inherited_error();
    if (with_gates)
        p.cum = reinterpret_cast<const float*>(static_cast<const unsigned char*>(remote_workspace) + fwd_workspace(B, H, Lk, d, dt == PATH_BF16 ? 2 : 4).cum);
    p.scale = scale; p.ring = 2; p.ring_state = static_cast<float*>(state); p.NCq = (Lq + CHUNK - 1) / CHUNK;
    if (!hip_ok(launch_attn_fwd2(p, d, dt == PATH_BF16, static_cast<hipStream_t>(stream)), "ring hop")) return PATH_ERR_HIP;
    return PATH_OK;
}

extern "C" path_status_t path_attn_ring_finish(const void* state, void* o, float* lse, int B, int H, int L, int d,
                                               path_dtype_t dt, const void* gates_workspace, size_t gates_workspace_bytes,
                                               void* stream) {
    if (!state || !o || !lse) return PATH_ERR_NULL;
    if (dt != PATH_F32 && dt != PATH_BF16) return PATH_ERR_DTYPE;
    if (!shape_ok(B, H, L, d)) return PATH_ERR_SHAPE;
    if (misaligned(state) || misaligned(o)) return PATH_ERR_ALIGN;
    FwdParams p = {};
    if (gates_workspace) {      // PaTH-FoX: the segment's own gate sums, where path_attn_ring_local left them
        const FwdWorkspace ws = fwd_workspace(B, H, L, d, dt == PATH_BF16 ? 2 : 4);
        if (gates_workspace_bytes < ws.total || (reinterpret_cast<uintptr_t>(gates_workspace) & 255)) return PATH_ERR_WORKSPACE;
        p.cum = reinterpret_cast<const float*>(static_cast<const unsigned char*>(gates_workspace) + ws.cum);
    }
    p.ul = layout_of(PATH_LAYOUT_BHLD, H, L, d);
    p.B = B; p.H = H; p.L = L; p.NC = (L + CHUNK - 1) / CHUNK;
    p.o = o; p.lse = lse; p.ring_state = const_cast<float*>(static_cast<const float*>(state));
    clear_inherited_error();
    if (!hip_ok(launch_ring_finish(p, d, dt == PATH_BF16, static_cast<hipStream_t>(stream)), "ring normalisation")) return PATH_ERR_HIP;
    return PATH_OK;
}

extern "C" path_status_t path_attn_fox_fwd(const void* q, const void* k, const void* v, const void* w,
                                           const void* beta, const void* log_f, void* o, float* lse, int B, int H,
                                           int L, int d, int causal, float scale, path_dtype_t dt, void* workspace,
                                           size_t workspace_bytes, void* stream) {
    if (!log_f) return PATH_ERR_NULL;
    return fwd_impl(0, layout_of(PATH_LAYOUT_BHLD, H, L, d), q, k, v, w, beta, log_f, 1, o, lse, B, H, L, d, causal, scale, dt,
                    workspace, workspace_bytes, stream);
}

// Backward of plain PaTH (log_f == NULL) and of PaTH-FoX (log_f, dlog_f given), and the forward of the
// training pair, which runs the backward's instantiations of the two transforms so that the backward
// can start from what they left in the workspace.
enum BwdMode { BWD_FULL = 0,        // transforms + backward (path_attn_bwd)
               BWD_FWD_ONLY = 1,    // transforms + forward sweep, everything the backward needs stays in the workspace
               BWD_RESUME = 2,      // backward without the transforms (the workspace is as BWD_FWD_ONLY left it)
               BWD_FWD_PREP = 3,    // the two halves of BWD_FWD_ONLY as separate calls: transforms ...
               BWD_FWD_SWEEP = 4 }; // ... and the forward sweep
static path_status_t bwd_run(BwdMode mode, int stages, const UserLayout& ul, const void* q, const void* k, const void* v, const void* w,
                             const void* beta, const void* log_f, const void* o, const float* lse, const void* d_o,
                             void* dq, void* dk, void* dv, void* dw, void* dbeta, void* dlog_f, int B, int H,
                             int L, int d, float scale, path_dtype_t dt, void* workspace, void* stream);

// Heads per pass of a self-contained backward in a workspace of `bytes`: all B*H if they fit, else the largest
// number of heads whose workspace does (0: not even one).
static int heads_per_pass(int B, int H, int L, int d, size_t es, size_t bytes) {
    const int BH = B * H;
    if (bwd_workspace(1, BH, L, d, es).total <= bytes) return BH;
    int lo = 0, hi = BH;                               // the size grows with the number of heads
    while (hi - lo > 1) {
        const int mid = (lo + hi) / 2;
        if (bwd_workspace(1, mid, L, d, es).total <= bytes) lo = mid; else hi = mid;
    }
    return lo;
}

static path_status_t bwd_impl(BwdMode mode, int stages, const UserLayout& ul, const void* q, const void* k, const void* v, const void* w,
                              const void* beta, const void* log_f, const void* o, const float* lse, const void* d_o,
                              void* dq, void* dk, void* dv, void* dw, void* dbeta, void* dlog_f, int B, int H,
                              int L, int d, int causal, float scale, path_dtype_t dt,
                              void* workspace, size_t workspace_bytes, void* stream) {
    if (!workspace) return PATH_ERR_NULL;
    if (mode != BWD_FWD_SWEEP && (!q || !k || !v || !w || !beta)) return PATH_ERR_NULL;
    if (mode != BWD_FWD_PREP && (!o || !lse)) return PATH_ERR_NULL;
    const bool fwd_mode = mode == BWD_FWD_ONLY || mode == BWD_FWD_PREP || mode == BWD_FWD_SWEEP;
    if (!fwd_mode) {
        if (!d_o || !dq || !dk || !dv || !dw || !dbeta) return PATH_ERR_NULL;
        if ((log_f == nullptr) != (dlog_f == nullptr)) return PATH_ERR_NULL;
    }
    if (dt != PATH_F32 && dt != PATH_BF16) return PATH_ERR_DTYPE;
    if (!shape_ok(B, H, L, d)) return PATH_ERR_SHAPE;
    if (!causal || !(scale > 0.f)) return PATH_ERR_UNSUPPORTED;
    const void* al[] = {q, k, v, w, o, d_o, dq, dk, dv, dw};
    for (const void* ptr : al) if (misaligned(ptr)) return PATH_ERR_ALIGN;      // (NULL is aligned)
    const size_t es = dt == PATH_BF16 ? 2 : 4;
    if (reinterpret_cast<uintptr_t>(workspace) & 255) return PATH_ERR_WORKSPACE;
    clear_inherited_error();
    if (mode != BWD_FULL) {            // the halves of a training pair share everything in the workspace: all heads at once
        if (workspace_bytes < bwd_workspace(B, H, L, d, es).total) return PATH_ERR_WORKSPACE;
        return bwd_run(mode, stages, ul, q, k, v, w, beta, log_f, o, lse, d_o, dq, dk, dv, dw, dbeta, dlog_f, B, H, L, d, scale, dt, workspace, stream);
    }
    // The self-contained backward passes over the heads in groups of as many as the workspace holds: the heads are
    // independent problems, so a smaller workspace costs launches, not arithmetic.
    const int BH = B * H, G = heads_per_pass(B, H, L, d, es, workspace_bytes);
    if (G < 1) return PATH_ERR_WORKSPACE;
    for (int bh0 = 0; bh0 < BH; bh0 += G) {
        UserLayout ug = ul;
        ug.bh0 = bh0;
        const path_status_t st = bwd_run(mode, stages, ug, q, k, v, w, beta, log_f, o, lse, d_o, dq, dk, dv, dw, dbeta, dlog_f,
                                         1, BH - bh0 < G ? BH - bh0 : G, L, d, scale, dt, workspace, stream);
        if (st != PATH_OK) return st;
    }
    return PATH_OK;
}

// One pass: the heads ul.bh0 .. ul.bh0 + B*H - 1 of the caller's tensors, numbered from 0 in the workspace.
static path_status_t bwd_run(BwdMode mode, int stages, const UserLayout& ul, const void* q, const void* k, const void* v, const void* w,
                             const void* beta, const void* log_f, const void* o, const float* lse, const void* d_o,
                             void* dq, void* dk, void* dv, void* dw, void* dbeta, void* dlog_f, int B, int H,
                             int L, int d, float scale, path_dtype_t dt, void* workspace, void* stream) {
    const bool fwd_mode = mode == BWD_FWD_ONLY || mode == BWD_FWD_PREP || mode == BWD_FWD_SWEEP;
    const int bf = dt == PATH_BF16;
    const size_t es = bf ? 2 : 4;
    const BwdWorkspace ws = bwd_workspace(B, H, L, d, es);
    unsigned char* base = static_cast<unsigned char*>(workspace);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int NC = (L + CHUNK - 1) / CHUNK, BH = B * H;
    const long long Lp = (long long)NC * CHUNK;
    auto F = [&](size_t off) { return reinterpret_cast<float*>(base + off); };

    // 1. chunk transform (forward kernel, with the row-major extras) and query states
    FwdParams fp = {};
    fp.q = q; fp.k = k; fp.v = v; fp.w = w; fp.beta = beta;
    fp.kt = base + ws.f.kt; fp.vt = base + ws.f.vt; fp.dp = base + ws.f.dp;
    fp.xinit = F(ws.f.xinit); fp.sd = F(ws.f.sd);
    fp.kt2 = base + ws.f.kt2; fp.dp2 = base + ws.f.dp2;
    fp.kt2T = base + ws.kt2T; fp.dpt2 = base + ws.dpt2; fp.kbm = base + ws.kbm; fp.rm = base + ws.rm;
    fp.B = B; fp.H = H; fp.L = L; fp.NC = NC; fp.scale = scale; fp.ul = ul;
    fp.ktT = base + ws.ktT; fp.vk = base + ws.vk; fp.dpt = base + ws.dpt; fp.xs = base + ws.xs; fp.xsT = base + ws.xsT;
    fp.fm = base + ws.fm; fp.gktm = base + ws.gktm; fp.nm = base + ws.nm; fp.aim = base + ws.aim;
    fp.ytm = base + ws.ytm; fp.utm = base + ws.utm; fp.gm = F(ws.gm); fp.sdm = F(ws.sdm);
    float* cum = log_f ? F(ws.f.cum) : nullptr;
    if (mode != BWD_RESUME && mode != BWD_FWD_SWEEP) {
        if (log_f && !hip_ok(launch_gate_sums(log_f, ul, cum, B, H, L, dt, st), "gate sums (backward)")) return PATH_ERR_HIP;
        if (!hip_ok(launch_prep_fwd(fp, d, bf, st), "chunk transform (backward)")) return PATH_ERR_HIP;
        if (!hip_ok(launch_prep2_fwd(fp, d, bf, st), "second-level transform (backward)")) return PATH_ERR_HIP;
    }
    if (mode == BWD_FWD_PREP) return PATH_OK;
    if (fwd_mode) {
        fp.o = const_cast<void*>(o); fp.lse = const_cast<float*>(lse); fp.cum = cum;
        fp.emit_states = 1;            // the sweep leaves the query states for the backward of the pair
        if (!hip_ok(launch_attn_fwd2(fp, d, bf, st), "forward sweep (training pair)")) return PATH_ERR_HIP;
        return PATH_OK;
    }
    if (mode != BWD_RESUME && NC > 1 && !hip_ok(launch_attn_states(fp, d, bf, st), "query states")) return PATH_ERR_HIP;

    // 2.-4. delta, adjoint scan over key chunks, key-side reductions
    BwdParams bp = {};
    bp.q = q; bp.k = k; bp.v = v; bp.w = w; bp.beta = beta; bp.o = o; bp.dO = d_o; bp.lse = lse;
    bp.kt = fp.kt; bp.vk = fp.vk; bp.ktT = fp.ktT; bp.xs = fp.xs; bp.xsT = fp.xsT;
    bp.kt2 = fp.kt2; bp.kt2T = fp.kt2T;
    // the 16-bit adjoint scan reads the transposed arrangements out of the forward's own product tiles
    bp.dpt = bf ? fp.dp : fp.dpt; bp.dpt2 = bf ? fp.dp2 : fp.dpt2; bp.dk2 = F(ws.dk2); bp.dchain = F(ws.dchain);
    bp.doq = base + ws.doq; bp.doT = base + ws.doT; bp.gs = base + ws.gs;
    bp.delta = F(ws.delta); bp.lse2p = F(ws.lse2p); bp.dqb = F(ws.dqb); bp.dkb = F(ws.dkb); bp.dvp = F(ws.dvp); bp.ddp = F(ws.ddp);
    bp.B = B; bp.H = H; bp.L = L; bp.NC = NC; bp.scale = scale; bp.ul = ul;
    bp.cum = cum; bp.dcol = cum ? F(ws.dcol) : nullptr; bp.drow = cum ? F(ws.drow) : nullptr;
    if (!hip_ok(launch_bwd_scan(bp, d, bf, stages, st), "backward pair kernels")) return PATH_ERR_HIP;
    if (!(stages & BWD_STAGE_CHUNK)) return PATH_OK;

    // 5. adjoint of the chunk transform
    const long long c_bh = (long long)NC * 4096, c_ch = 4096;          // 64x64 per chunk
    const long long t_bh = Lp * d, t_ch = (long long)CHUNK * d;        // padded token-major [Lp][d]
    auto chunk_n = [&](const void* p, int type) { return MatRef{p, c_bh, c_ch, 64, 1, type, TOK_NONE}; };   // [r][k]
    auto chunk_t = [&](const void* p, int type) { return MatRef{p, c_bh, c_ch, 1, 64, type, TOK_NONE}; };   // [k][r]
    auto tokws_n = [&](const void* p) { return MatRef{p, t_bh, t_ch, d, 1, EL_F32, TOK_NONE}; };            // rows = tokens
    auto tokws_t = [&](const void* p) { return MatRef{p, t_bh, t_ch, 1, d, EL_F32, TOK_NONE}; };            // k = tokens
    const int uts = (int)ul.vt;                                         // token stride of the caller's tensors
    auto user_n = [&](const void* p) { return MatRef{p, 0, 0, uts, 1, EL_IO, TOK_ROW, 1}; };
    auto user_t = [&](const void* p) { return MatRef{p, 0, 0, 1, uts, EL_IO, TOK_K, 1}; };
    const MatRef U_rows{base + ws.utm, (long long)NC * d * CHUNK, (long long)d * CHUNK, 1, 64, EL_OP, TOK_NONE};  // U[t'][c]
    const MatRef ddp_kfirst{F(ws.ddp), (long long)NC * d * d, (long long)d * d, 1, d, EL_F32, TOK_NONE};   // (n=c, k=a): ddP[a][c]
    const MatRef ddp_nfirst{F(ws.ddp), (long long)NC * d * d, (long long)d * d, d, 1, EL_F32, TOK_NONE};   // (n=c, k=b): ddP[c][b]

    bool ok = true;
    int cmul = 1, cadd = 0;          // which chunks the following products run on: x * cmul + cadd
    auto gemm = [&](float* C, int tokC, const float* Cin, MatRef A, MatRef Bm, int M, int N, int K, float alpha, int mask) {
        if (!ok) return;
        GemmArgs a;
        a.A = A; a.B = Bm; a.C = C; a.Cin = Cin;
        a.ccs = 1;
        switch (tokC) {      // layout of C (and Cin)
            case OUT_TOK:  a.c_bh = t_bh; a.c_ch = t_ch; a.crs = d; break;                                    // tokens x d
            case OUT_DD:   a.c_bh = (long long)NC * d * d; a.c_ch = (long long)d * d; a.crs = d; break;       // d x d per chunk
            case OUT_DD1:  a.c_bh = (long long)(NC + 1) * d * d; a.c_ch = (long long)d * d; a.crs = d; break; // ... in an array of NC+1
            case OUT_D64:  a.c_bh = (long long)NC * d * CHUNK; a.c_ch = (long long)d * CHUNK; a.crs = 64; break;   // d x 64 per chunk
            default:       a.c_bh = c_bh; a.c_ch = c_ch; a.crs = 64; break;                                   // 64 x 64 per chunk
        }
        a.M = M; a.N = N; a.K = K; a.alpha = alpha; a.mask = mask; a.NC = NC; a.L = L;
        a.cmul = cmul; a.cadd = cadd; a.gridx = cmul == 1 ? NC : (NC + cmul - 1) / cmul; a.ul = ul;
        ok = hip_ok(launch_batched_gemm(a, BH, bf, st), "chunk-transform adjoint product");
    };
    float *dpd = F(ws.dpd), *pd = F(ws.pd), *dsd = F(ws.dsd), *df = F(ws.df), *dy = F(ws.dy), *dn = F(ws.dn);
    float *dgk = F(ws.dgk), *rr = F(ws.rr), *mm = F(ws.mm), *dgs = F(ws.dgs), *du = F(ws.du);
    float *dqf = F(ws.dqf), *dkf = F(ws.dkf), *dwf = F(ws.dwf), *dbf = F(ws.dbf);
    float *dqb = bp.dqb, *dkb = bp.dkb, *dvp = bp.dvp;
    void *fm = fp.fm, *gktm = fp.gktm, *nm = fp.nm, *aim = fp.aim, *ytm = fp.ytm;

    // 5a. adjoint of the second level (Kb2_c = Kb_c R_c^T, R_{c-1} = R_c P_c, P_superblock = R_{first-1}),
    // position by position inside the super-blocks, all super-blocks at once.  dchain entry c+1 is
    // the gradient of R_c; entry 4J (gradient of P_superblock J) comes from the far ddP kernel.
    //     ddP_c  -= R_c^T D_{c-1}
    //     D_c     = D_{c-1} (I - dP_c)^T + dKb2_c^T Kb_c          dP_c = W_c^T U_c
    //     dKb_c  += dKb2_c R_c
    if (NC > SBC && bf) {         // fused kernel (2-byte operand types)
        SbChainArgs sa{base + ws.rm, base + ws.kbm, base + ws.utm, w, F(ws.dk2), F(ws.dchain), F(ws.ddp), dkb, L, NC, ul};
        ok = hip_ok(launch_bwd_sb_chain(sa, BH, d, st), "second-level adjoint");
    } else if (NC > SBC) {        // the same chain as a sequence of batched products (fp32 operands)
        const long long dd = (long long)d * d, dd_bh = (long long)NC * dd, ch_bh = (long long)(NC + 1) * dd;
        float* dch = F(ws.dchain);
        float* t1 = F(ws.t1);
        float* dk2 = F(ws.dk2);
        cmul = SBC;
        for (int cl = 0; cl < SBC && ok; ++cl) {
            cadd = cl;
            const MatRef Dprev_kfirst{dch, ch_bh, dd, 1, d, EL_F32, TOK_NONE};          // (n=b, k): D_{c-1}[k][b]
            const MatRef Dprev_rows{dch, ch_bh, dd, d, 1, EL_F32, TOK_NONE};            // (m=a, k): D_{c-1}[a][k]
            const MatRef R_kfirst{base + ws.rm, dd_bh, dd, 1, d, EL_OP, TOK_NONE};       // (m=a, k): R_c[k][a]  /  (n=b, k=a): R_c[a][b]
            gemm(F(ws.ddp), OUT_DD, F(ws.ddp), R_kfirst, Dprev_kfirst, d, d, d, -1.f, MASK_NONE);
            if (cl + 1 < SBC) {
                // T1 = D_{c-1} U_c^T  (d x 64),  D_c = D_{c-1} - T1 W_c + dKb2_c^T Kb_c
                gemm(t1, OUT_D64, nullptr, Dprev_rows, U_rows, d, 64, d, 1.f, MASK_NONE);
                const MatRef T1_rows{t1, (long long)NC * d * CHUNK, (long long)d * CHUNK, 64, 1, EL_F32, TOK_NONE};
                gemm(dch + dd, OUT_DD1, dch, T1_rows, user_t(w), d, d, 64, -1.f, MASK_NONE);
                const MatRef dk2_t{dk2, t_bh, t_ch, 1, d, EL_F32, TOK_NONE};             // (m=a, k=s): dKb2[s][a]
                const MatRef kb_t{base + ws.kbm, t_bh, t_ch, 1, d, EL_OP, TOK_NONE};     // (n=b, k=s): Kb[s][b]
                gemm(dch + dd, OUT_DD1, dch + dd, dk2_t, kb_t, d, d, 64, 1.f, MASK_NONE);
            }
            const MatRef dk2_n{dk2, t_bh, t_ch, d, 1, EL_F32, TOK_NONE};                 // (m=s, k=a): dKb2[s][a]
            gemm(dkb, OUT_TOK, dkb, dk2_n, R_kfirst, 64, d, d, 1.f, MASK_NONE);
        }
        cmul = 1; cadd = 0;
    }

    // 5b. adjoint of the chunk transform: one fused kernel runs this list per (chunk, head).
    // Chains of products that add into the same result are consecutive.
    if (!ok) return PATH_ERR_HIP;
    if (bf) {      // 2-byte operand types: the hand-fused kernel
        ChunkFusedArgs ca{ul, q, k, v, w, beta, d_o, lse, bp.delta, fp.sdm, fp.gm, fp.fm, fp.gktm, fp.nm, fp.aim, fp.ytm,
                          base + ws.utm, bp.dqb, bp.dkb, bp.dvp, F(ws.ddp), dq, dk, dv, dw, dbeta, bp.cum, bp.dcol, bp.drow,
                          L, NC, scale};
        ok = hip_ok(launch_chunk_fused(ca, BH, d, st), "chunk-transform adjoint");
        if (ok && log_f) {
            ScanArgs sa{bp.dcol, bp.drow, dlog_f, (int)Lp, L, L, L, 0, 1.f, 0, 1, ul};
            ok = hip_ok(launch_fox_scan(sa, BH, 0, 1, st), "gate gradient");
        }
        return ok ? PATH_OK : PATH_ERR_HIP;
    }
    ChunkProgram pr = {};
    pr.L = L; pr.NC = NC; pr.ul = ul;
    bool chain_open = false;
    // one product: C (+)= alpha A B^T; `first` opens a chain (from Cin or zero), `last` masks and writes C
    // results that are only read as matrix operands (marked OP) are stored in the operand type: half the bytes
    // for 2-byte operands, and the same values the staging would produce from a float copy
    bool as_op = false;
    auto prod = [&](float* C, int out, const float* Cin, MatRef A, MatRef Bm, int M, int N, int K, float alpha, int mask,
                    bool first, bool last) {
        ChunkOp& o = pr.ops[pr.n++];
        o.kind = OP_PRODUCT; o.A = A; o.B = Bm; o.C = C; o.Cin = Cin;
        if (out == OUT_TOK) { o.c_bh = t_bh; o.c_ch = t_ch; o.crs = d; }
        else { o.c_bh = c_bh; o.c_ch = c_ch; o.crs = 64; }
        o.M = (short)M; o.N = (short)N; o.K = (short)K; o.alpha = alpha; o.mask = (unsigned char)mask;
        o.first = first; o.last = last; o.c_op = as_op;
        chain_open = !last;
    };
    auto special = [&](int kind) { pr.ops[pr.n++].kind = (unsigned char)kind; };
    pr.diag = DiagArgs{fp.sdm, dpd, bp.delta, lse, pd, dsd, L, NC, scale, bp.cum, bp.dcol, bp.drow};
    pr.beta = BetaArgs{rr, mm, fp.gm, beta, dgs, dbf, L, NC};
    pr.out = OutArgs{dqf, dkf, dvp, dwf, dbf, dq, dk, dv, dw, dbeta, L, NC, d};

    prod(dpd, OUT_C64, nullptr, user_n(d_o), user_n(v), 64, 64, d, 1.f, MASK_NONE, true, true);              // dPd = dO V^T
    special(OP_DIAG);                                                                                          // P, dSd
    prod(dvp, OUT_TOK, dvp, chunk_t(pd, EL_OP), user_t(d_o), 64, d, 64, 1.f, MASK_NONE, true, true);         // dV += P^T dO
    prod(dqf, OUT_TOK, dqb, chunk_n(dsd, EL_OP), user_t(k), 64, d, 64, 1.f, MASK_NONE, true, true);          // dQ = dQb + dSd K
    prod(dkf, OUT_TOK, dkb, chunk_t(dsd, EL_OP), user_t(q), 64, d, 64, 1.f, MASK_NONE, true, true);          // dK = dKb + dSd^T Q
    as_op = true;
    prod(df, OUT_C64, nullptr, chunk_n(dsd, EL_OP), chunk_t(ytm, EL_OP), 64, 64, 64, -1.f, MASK_TRIL, true, false);   // dF = tril(-dSd Y^T
    prod(df, OUT_C64, nullptr, tokws_n(dqb), U_rows, 64, 64, d, -1.f, MASK_TRIL, false, true);                         //          - dQb U^T)
    prod(dy, OUT_C64, nullptr, chunk_t(fm, EL_OP), chunk_t(dsd, EL_OP), 64, 64, 64, -1.f, MASK_NONE, true, false);    // dY = -F^T dSd
    prod(dy, OUT_C64, nullptr, user_n(w), tokws_n(dkb), 64, 64, d, -1.f, MASK_NONE, false, true);                      //      - W dKb^T
    prod(du, OUT_TOK, nullptr, chunk_t(fm, EL_OP), tokws_t(dqb), 64, d, 64, -1.f, MASK_NONE, true, false);             // dU = -F^T dQb
    prod(du, OUT_TOK, nullptr, user_n(w), ddp_kfirst, 64, d, d, 1.f, MASK_NONE, false, true);                          //      + W ddP
    prod(dn, OUT_C64, nullptr, chunk_n(dy, EL_OP), chunk_t(gktm, EL_OP), 64, 64, 64, 1.f, MASK_NONE, true, false);    // dN = dY Gk^T
    prod(dn, OUT_C64, nullptr, MatRef{du, t_bh, t_ch, d, 1, EL_OP, TOK_NONE}, user_n(w), 64, 64, d, 1.f, MASK_NONE, false, true);                        //      + dU W^T
    prod(dgk, OUT_C64, nullptr, chunk_t(nm, EL_OP), chunk_t(dy, EL_OP), 64, 64, 64, 1.f, MASK_SLOWER, true, true);    // dGk = sl(N^T dY)
    as_op = false;      // R and M are also read element-wise (dbeta)
    prod(rr, OUT_C64, nullptr, chunk_t(aim, EL_OP), chunk_t(dn, EL_OP), 64, 64, 64, 1.f, MASK_NONE, true, true);      // R = A^-T dN
    prod(mm, OUT_C64, nullptr, chunk_n(rr, EL_F32), chunk_n(nm, EL_OP), 64, 64, 64, -1.f, MASK_SLOWER, true, true);    // M = sl(-R N^T)
    special(OP_BETA);                                                                                          // dGs, dbeta
    prod(dwf, OUT_TOK, nullptr, chunk_t(ytm, EL_OP), tokws_t(dkb), 64, d, 64, -1.f, MASK_NONE, true, false);           // dW = -Y dKb
    prod(dwf, OUT_TOK, nullptr, U_rows, ddp_nfirst, 64, d, d, 1.f, MASK_NONE, false, false);                           //    + U ddP^T
    prod(dwf, OUT_TOK, nullptr, chunk_t(df, EL_OP), user_t(q), 64, d, 64, 1.f, MASK_NONE, false, false);              //    + dF^T Q
    prod(dwf, OUT_TOK, nullptr, chunk_n(dgk, EL_OP), user_t(k), 64, d, 64, 1.f, MASK_NONE, false, false);             //    + dGk K
    prod(dwf, OUT_TOK, nullptr, chunk_t(nm, EL_OP), MatRef{du, t_bh, t_ch, 1, d, EL_OP, TOK_NONE}, 64, d, 64, 1.f, MASK_NONE, false, false);             //    + N^T dU
    prod(dwf, OUT_TOK, nullptr, chunk_n(dgs, EL_OP), user_t(w), 64, d, 64, 1.f, MASK_NONE, false, true);              //    + (dG+dG^T) W
    prod(dqf, OUT_TOK, dqf, chunk_n(df, EL_OP), user_t(w), 64, d, 64, 1.f, MASK_NONE, true, true);           // dQ += dF W
    prod(dkf, OUT_TOK, dkf, chunk_t(dgk, EL_OP), user_t(w), 64, d, 64, 1.f, MASK_NONE, true, true);          // dK += dGk^T W
    special(OP_STORE);                                                                                         // to the I/O dtype
    if (chain_open || pr.n > MAX_CHUNK_OPS) return PATH_ERR_HIP;
    ok = hip_ok(launch_chunk_adjoint(pr, BH, bf, st), "chunk-transform adjoint");
    if (ok && log_f) {
        // dlog f_s = sum over the pairs j < s <= i of the logit gradient = (column sums left of s) - (row sums
        // above s).  The row sums vanish in exact arithmetic; subtracting them as computed removes the error that
        // delta = dO . o (o rounded to the I/O type) puts into every row, which the prefix sum would pile up.
        ScanArgs sa{bp.dcol, bp.drow, dlog_f, (int)Lp, L, L, L, 0, 1.f, 0, 1, ul};
        ok = hip_ok(launch_fox_scan(sa, BH, 0, bf ? 1 : 0, st), "gate gradient");
    }
    return ok ? PATH_OK : PATH_ERR_HIP;
}

extern "C" size_t path_decode_workspace_bytes(int B, int H, int d) {
    if (B < 1 || H < 1 || (d != 64 && d != 128)) return 0;
    return align256((size_t)B * H * DECODE_MAX_SPLITS * (d + 2) * 4);
}

extern "C" path_status_t path_key_prefill(const void* v, int B, int H, int L, int d, path_dtype_t dt,
                                          const void* fws, size_t fws_bytes,
                                          void* kcache, void* vcache, int Lmax, void* stream) {
    if (!v || !fws || !kcache || !vcache) return PATH_ERR_NULL;
    if (dt != PATH_F32 && dt != PATH_BF16) return PATH_ERR_DTYPE;
    if (!shape_ok(B, H, L, d) || L > Lmax) return PATH_ERR_SHAPE;
    const size_t es = dt == PATH_BF16 ? 2 : 4;
    const FwdWorkspace ws = fwd_workspace(B, H, L, d, es);
    if (fws_bytes < ws.total || (reinterpret_cast<uintptr_t>(fws) & 255)) return PATH_ERR_WORKSPACE;
    if (misaligned(v) || misaligned(kcache) || misaligned(vcache)) return PATH_ERR_ALIGN;
    const unsigned char* base = static_cast<const unsigned char*>(fws);
    hipStream_t st = static_cast<hipStream_t>(stream);
    clear_inherited_error();
    PrefillArgs a{base + ws.kt2, base + ws.dp2, kcache, L, (L + CHUNK - 1) / CHUNK, Lmax};
    if (!hip_ok(launch_key_prefill(a, B * H, d, dt == PATH_BF16, st), "key prefill")) return PATH_ERR_HIP;
    // values: rows [0, L) of every head, unchanged
    if (!hip_ok(hipMemcpy2DAsync(vcache, (size_t)Lmax * d * es, v, (size_t)L * d * es, (size_t)L * d * es, (size_t)B * H,
                                 hipMemcpyDeviceToDevice, st), "value cache copy"))
        return PATH_ERR_HIP;
    return PATH_OK;
}

extern "C" path_status_t path_decode_step(const void* q, const void* k, const void* v, const void* w,
                                          const void* beta, void* kcache, void* vcache, int n, int Lmax,
                                          void* o, float* lse, int B, int H, int d, float scale,
                                          path_dtype_t dt, void* workspace, size_t workspace_bytes,
                                          void* stream) {
    if (!q || !k || !v || !w || !beta || !kcache || !vcache || !o || !lse || !workspace) return PATH_ERR_NULL;
    if (dt != PATH_F32 && dt != PATH_BF16) return PATH_ERR_DTYPE;
    if (B < 1 || H < 1 || (d != 64 && d != 128) || (long long)B * H > 65535 || n < 0 || n >= Lmax) return PATH_ERR_SHAPE;
    if (!(scale > 0.f)) return PATH_ERR_UNSUPPORTED;
    if (workspace_bytes < path_decode_workspace_bytes(B, H, d) || (reinterpret_cast<uintptr_t>(workspace) & 255))
        return PATH_ERR_WORKSPACE;
    const void* al[] = {q, k, v, w, kcache, vcache, o};
    for (const void* ptr : al) if (misaligned(ptr)) return PATH_ERR_ALIGN;
    clear_inherited_error();
    DecodeArgs a{q, k, v, w, beta, kcache, vcache, o, lse, static_cast<float*>(workspace), n, Lmax, scale, nullptr, nullptr};
    if (!hip_ok(launch_decode_step(a, B * H, d, dt == PATH_BF16, static_cast<hipStream_t>(stream)), "decode step"))
        return PATH_ERR_HIP;
    return PATH_OK;
}

// PaTH-FoX at decode time: the running sums of the log gates are a third cache.
extern "C" path_status_t path_gate_prefill(const void* log_f, int B, int H, int L, path_dtype_t dt, float* ccache, int Lmax,
                                           void* stream) {
    if (!log_f || !ccache) return PATH_ERR_NULL;
    if (dt != PATH_F32 && dt != PATH_BF16) return PATH_ERR_DTYPE;
    if (B < 1 || H < 1 || L < 1 || L > Lmax || (long long)B * H > 65535) return PATH_ERR_SHAPE;
    clear_inherited_error();
    ScanArgs a{log_f, nullptr, ccache, L, Lmax, L, L, 1, 1.f, 0, 0, layout_of(PATH_LAYOUT_BHLD, H, L, 64)};
    if (!hip_ok(launch_fox_scan(a, B * H, dt == PATH_BF16 ? 1 : 0, 0, static_cast<hipStream_t>(stream)), "gate sums of the prompt"))
        return PATH_ERR_HIP;
    return PATH_OK;
}

extern "C" path_status_t path_decode_step_fox(const void* q, const void* k, const void* v, const void* w,
                                              const void* beta, const void* log_f, void* kcache, void* vcache,
                                              float* ccache, int n, int Lmax, void* o, float* lse, int B, int H, int d,
                                              float scale, path_dtype_t dt, void* workspace, size_t workspace_bytes,
                                              void* stream) {
    if (!q || !k || !v || !w || !beta || !log_f || !kcache || !vcache || !ccache || !o || !lse || !workspace) return PATH_ERR_NULL;
    if (dt != PATH_F32 && dt != PATH_BF16) return PATH_ERR_DTYPE;
    if (B < 1 || H < 1 || (d != 64 && d != 128) || (long long)B * H > 65535 || n < 0 || n >= Lmax) return PATH_ERR_SHAPE;
    if (!(scale > 0.f)) return PATH_ERR_UNSUPPORTED;
    if (workspace_bytes < path_decode_workspace_bytes(B, H, d) || (reinterpret_cast<uintptr_t>(workspace) & 255))
        return PATH_ERR_WORKSPACE;
    const void* al[] = {q, k, v, w, kcache, vcache, o};
    for (const void* ptr : al) if (misaligned(ptr)) return PATH_ERR_ALIGN;
    clear_inherited_error();
    DecodeArgs a{q, k, v, w, beta, kcache, vcache, o, lse, static_cast<float*>(workspace), n, Lmax, scale, log_f, ccache};
    if (!hip_ok(launch_decode_step(a, B * H, d, dt == PATH_BF16, static_cast<hipStream_t>(stream)), "gated decode step"))
        return PATH_ERR_HIP;
    return PATH_OK;
}

// ---- decode step for callers that cannot allocate: the split partials live in a device array of the library ----
//
// One copy of the array exists on every GPU the library is loaded on; host code must not use the array's name as
// an address (it is a host-side stand-in): the device address is looked up once per device and kept.
static __device__ __align__(256) unsigned char scratch[PATH_DECODE_STATIC_BYTES];
static constexpr int MAX_DEVICES = 64;
static std::mutex g_scratch_lock;
static void* g_scratch_ptr[MAX_DEVICES] = {};      // per device: address of `scratch` there

// Address of the array on the current device (looked up on the first call on that device), or NULL with the
// reason in the thread's last-error text.
static void* scratch_on_current_device() {
    int dev = -1;
    if (!hip_ok(hipGetDevice(&dev), "static scratch: current device")) return nullptr;
    if (dev < 0 || dev >= MAX_DEVICES) {
        snprintf(g_last_error, sizeof g_last_error, "static scratch: device index %d outside [0, %d)", dev, MAX_DEVICES);
        return nullptr;
    }
    std::lock_guard<std::mutex> guard(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (!hip_ok(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)), "static scratch: symbol address")) return nullptr;
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}

extern "C" size_t path_decode_static_scratch_bytes(void) { return PATH_DECODE_STATIC_BYTES; }

extern "C" path_status_t path_decode_step_static(const void* q, const void* k, const void* v, const void* w,
                                                 const void* beta, void* kcache, void* vcache, int n, int Lmax,
                                                 void* o, float* lse, int B, int H, int d, float scale,
                                                 path_dtype_t dt, void* stream) {
    if (!q || !k || !v || !w || !beta || !kcache || !vcache || !o || !lse) return PATH_ERR_NULL;
    if (dt != PATH_F32 && dt != PATH_BF16) return PATH_ERR_DTYPE;
    if (B < 1 || H < 1 || (d != 64 && d != 128) || (long long)B * H > 65535 || n < 0 || n >= Lmax) return PATH_ERR_SHAPE;
    if (!(scale > 0.f)) return PATH_ERR_UNSUPPORTED;
    const size_t need = path_decode_workspace_bytes(B, H, d);
    if (need > PATH_DECODE_STATIC_BYTES) {
        snprintf(g_last_error, sizeof g_last_error, "static scratch: B*H = %lld at d = %d needs %zu bytes, the array holds %zu",
                 (long long)B * H, d, need, (size_t)PATH_DECODE_STATIC_BYTES);
        return PATH_ERR_WORKSPACE;
    }
    const void* al[] = {q, k, v, w, kcache, vcache, o};
    for (const void* ptr : al) if (misaligned(ptr)) return PATH_ERR_ALIGN;
    clear_inherited_error();
    void* ws = scratch_on_current_device();
    if (!ws) return PATH_ERR_HIP;
    // (nothing in the array has to start at zero: every split writes its whole record before the merge reads it)
    DecodeArgs a{q, k, v, w, beta, kcache, vcache, o, lse, static_cast<float*>(ws), n, Lmax, scale, nullptr, nullptr};
    if (!hip_ok(launch_decode_step(a, B * H, d, dt == PATH_BF16, static_cast<hipStream_t>(stream)), "decode step (static scratch)"))
        return PATH_ERR_HIP;
    return PATH_OK;
}

extern "C" path_status_t path_attn_bwd(const void* q, const void* k, const void* v, const void* w,
                                       const void* beta, const void* o, const float* lse, const void* d_o,
                                       void* dq, void* dk, void* dv, void* dw, void* dbeta, int B, int H,
                                       int L, int d, int causal, float scale, path_dtype_t dt,
                                       void* workspace, size_t workspace_bytes, void* stream) {
    return bwd_impl(BWD_FULL, BWD_STAGE_ALL, layout_of(PATH_LAYOUT_BHLD, H, L, d), q, k, v, w, beta, nullptr, o, lse, d_o, dq, dk, dv, dw, dbeta, nullptr, B, H, L, d, causal, scale, dt,
                    workspace, workspace_bytes, stream);
}

extern "C" path_status_t path_attn_fox_bwd(const void* q, const void* k, const void* v, const void* w,
                                           const void* beta, const void* log_f, const void* o, const float* lse,
                                           const void* d_o, void* dq, void* dk, void* dv, void* dw, void* dbeta,
                                           void* dlog_f, int B, int H, int L, int d, int causal, float scale,
                                           path_dtype_t dt, void* workspace, size_t workspace_bytes, void* stream) {
    if (!log_f || !dlog_f) return PATH_ERR_NULL;
    return bwd_impl(BWD_FULL, BWD_STAGE_ALL, layout_of(PATH_LAYOUT_BHLD, H, L, d), q, k, v, w, beta, log_f, o, lse, d_o, dq, dk, dv, dw, dbeta, dlog_f, B, H, L, d, causal, scale, dt,
                    workspace, workspace_bytes, stream);
}

extern "C" path_status_t path_attn_train_fwd(const void* q, const void* k, const void* v, const void* w,
                                             const void* beta, const void* log_f, void* o, float* lse,
                                             int B, int H, int L, int d, int causal, float scale,
                                             path_dtype_t dt, void* workspace, size_t workspace_bytes, void* stream) {
    return bwd_impl(BWD_FWD_ONLY, BWD_STAGE_ALL, layout_of(PATH_LAYOUT_BHLD, H, L, d), q, k, v, w, beta, log_f, o, lse, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr,
                    B, H, L, d, causal, scale, dt, workspace, workspace_bytes, stream);
}

extern "C" path_status_t path_attn_train_fwd_prep(const void* q, const void* k, const void* v, const void* w,
                                                  const void* beta, const void* log_f, int B, int H, int L, int d,
                                                  path_dtype_t dt, void* workspace, size_t workspace_bytes, void* stream) {
    return bwd_impl(BWD_FWD_PREP, BWD_STAGE_ALL, layout_of(PATH_LAYOUT_BHLD, H, L, d), q, k, v, w, beta, log_f, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr,
                    nullptr, B, H, L, d, 1, 1.f, dt, workspace, workspace_bytes, stream);
}

extern "C" path_status_t path_attn_train_fwd_sweep(void* o, float* lse, int with_gates, int B, int H, int L, int d, float scale,
                                                   path_dtype_t dt, void* workspace, size_t workspace_bytes, void* stream) {
    // (log_f itself is not read here: the gate sums are in the workspace; any non-NULL value selects them)
    return bwd_impl(BWD_FWD_SWEEP, BWD_STAGE_ALL, layout_of(PATH_LAYOUT_BHLD, H, L, d), nullptr, nullptr, nullptr, nullptr, nullptr, with_gates ? workspace : nullptr, o, lse, nullptr,
                    nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, B, H, L, d, 1, scale, dt, workspace, workspace_bytes, stream);
}

extern "C" path_status_t path_attn_train_bwd(const void* q, const void* k, const void* v, const void* w,
                                             const void* beta, const void* log_f, const void* o, const float* lse,
                                             const void* d_o, void* dq, void* dk, void* dv, void* dw, void* dbeta,
                                             void* dlog_f, int B, int H, int L, int d, int causal, float scale,
                                             path_dtype_t dt, void* workspace, size_t workspace_bytes, void* stream) {
    return bwd_impl(BWD_RESUME, BWD_STAGE_ALL, layout_of(PATH_LAYOUT_BHLD, H, L, d), q, k, v, w, beta, log_f, o, lse, d_o, dq, dk, dv, dw, dbeta, dlog_f, B, H, L, d, causal, scale, dt,
                    workspace, workspace_bytes, stream);
}

extern "C" path_status_t path_attn_train_bwd_stages(int stages, const void* q, const void* k, const void* v, const void* w,
                                                    const void* beta, const void* log_f, const void* o, const float* lse,
                                                    const void* d_o, void* dq, void* dk, void* dv, void* dw, void* dbeta,
                                                    void* dlog_f, int B, int H, int L, int d, int causal, float scale,
                                                    path_dtype_t dt, void* workspace, size_t workspace_bytes, void* stream) {
    if (stages <= 0 || (stages & ~BWD_STAGE_ALL)) return PATH_ERR_UNSUPPORTED;
    return bwd_impl(BWD_RESUME, stages, layout_of(PATH_LAYOUT_BHLD, H, L, d), q, k, v, w, beta, log_f, o, lse, d_o, dq, dk, dv, dw, dbeta, dlog_f, B, H, L, d, causal, scale, dt,
                    workspace, workspace_bytes, stream);
}

// ---- the same computations on [B,L,H,d] tensors, and on packed variable-length batches ------------------

extern "C" path_status_t path_attn_fwd_layout(const void* q, const void* k, const void* v, const void* w,
                                              const void* beta, const void* log_f, void* o, float* lse,
                                              int B, int H, int L, int d, path_layout_t layout, int causal, float scale,
                                              path_dtype_t dt, void* workspace, size_t workspace_bytes, void* stream) {
    if (!layout_ok(layout)) return PATH_ERR_UNSUPPORTED;
    return fwd_impl(0, layout_of(layout, H, L, d), q, k, v, w, beta, log_f, log_f != nullptr, o, lse, B, H, L, d, causal, scale, dt,
                    workspace, workspace_bytes, stream);
}

extern "C" path_status_t path_attn_bwd_layout(const void* q, const void* k, const void* v, const void* w,
                                              const void* beta, const void* log_f, const void* o, const float* lse,
                                              const void* d_o, void* dq, void* dk, void* dv, void* dw, void* dbeta,
                                              void* dlog_f, int B, int H, int L, int d, path_layout_t layout, int causal,
                                              float scale, path_dtype_t dt, void* workspace, size_t workspace_bytes,
                                              void* stream) {
    if (!layout_ok(layout)) return PATH_ERR_UNSUPPORTED;
    return bwd_impl(BWD_FULL, BWD_STAGE_ALL, layout_of(layout, H, L, d), q, k, v, w, beta, log_f, o, lse, d_o, dq, dk, dv, dw, dbeta, dlog_f,
                    B, H, L, d, causal, scale, dt, workspace, workspace_bytes, stream);
}

// Packed sequences [T,H,d]: ONE set of launches for the whole batch.  Sequence s is batch entry s of a problem
// with B = nseq whose workspace arrays are sized for the longest sequence; the kernels take every bound from the
// entry's own length (a device copy of cu_seqlens, kept at the start of the workspace) and address the caller's
// tensors from token cu_seqlens[s] on.  Workgroups beyond a shorter sequence's last chunk exit at once.
static bool varlen_ok(const int* cu, int nseq, int* lmax) {
    if (!cu || nseq < 1 || cu[0] != 0) return false;
    int m = 0;
    for (int s = 0; s < nseq; ++s) {
        const int len = cu[s + 1] - cu[s];
        if (len < 1) return false;
        if (len > m) m = len;
    }
    *lmax = m;
    return true;
}
static size_t cu_table_bytes(int nseq) { return align256((size_t)(nseq + 1) * sizeof(int)); }
static UserLayout varlen_layout(int H, int d, const int* cu_device) {
    UserLayout u;
    u.H = H; u.bh0 = 0; u.cu = cu_device;
    u.vb = 0; u.vh = d; u.vt = (long long)H * d;
    u.sb = 0; u.sh = 1; u.st = H;
    return u;
}
// copies the table to the head of the workspace (the host array may be pageable: the runtime stages it before
// the call returns) and splits the workspace
static path_status_t varlen_setup(const int* cu, int nseq, int H, int d, path_dtype_t dt, void* workspace, size_t workspace_bytes,
                                  void* stream, int* lmax, UserLayout* ul, void** rest, size_t* rest_bytes) {
    if (dt != PATH_F32 && dt != PATH_BF16) return PATH_ERR_DTYPE;
    if (!varlen_ok(cu, nseq, lmax) || !shape_ok(nseq, H, *lmax, d)) return PATH_ERR_SHAPE;
    if (!workspace) return PATH_ERR_NULL;
    const size_t tb = cu_table_bytes(nseq);
    if (workspace_bytes <= tb || (reinterpret_cast<uintptr_t>(workspace) & 255)) return PATH_ERR_WORKSPACE;
    clear_inherited_error();
    if (!hip_ok(hipMemcpyAsync(workspace, cu, (size_t)(nseq + 1) * sizeof(int), hipMemcpyHostToDevice, static_cast<hipStream_t>(stream)),
                "sequence table copy"))
        return PATH_ERR_HIP;
    *ul = varlen_layout(H, d, static_cast<const int*>(workspace));
    *rest = static_cast<unsigned char*>(workspace) + tb;
    *rest_bytes = workspace_bytes - tb;
    return PATH_OK;
}

extern "C" size_t path_attn_varlen_workspace_bytes(const int* cu_seqlens, int nseq, int H, int d, path_dtype_t dt,
                                                   int for_backward) {
    int lmax = 0;
    if (!varlen_ok(cu_seqlens, nseq, &lmax)) return 0;
    const size_t body = path_attn_workspace_bytes(nseq, H, lmax, d, dt, for_backward);
    return body ? cu_table_bytes(nseq) + body : 0;
}

extern "C" path_status_t path_attn_varlen_fwd(const void* q, const void* k, const void* v, const void* w,
                                              const void* beta, const void* log_f, void* o, float* lse,
                                              const int* cu_seqlens, int nseq, int H, int d, int causal, float scale,
                                              path_dtype_t dt, void* workspace, size_t workspace_bytes, void* stream) {
    int lmax = 0;
    UserLayout ul;
    void* rest = nullptr;
    size_t rest_bytes = 0;
    const path_status_t st = varlen_setup(cu_seqlens, nseq, H, d, dt, workspace, workspace_bytes, stream, &lmax, &ul, &rest, &rest_bytes);
    if (st != PATH_OK) return st;
    return fwd_impl(0, ul, q, k, v, w, beta, log_f, log_f != nullptr, o, lse, nseq, H, lmax, d, causal, scale, dt, rest, rest_bytes, stream);
}

extern "C" path_status_t path_attn_varlen_bwd(const void* q, const void* k, const void* v, const void* w,
                                              const void* beta, const void* log_f, const void* o, const float* lse,
                                              const void* d_o, void* dq, void* dk, void* dv, void* dw, void* dbeta,
                                              void* dlog_f, const int* cu_seqlens, int nseq, int H, int d, int causal,
                                              float scale, path_dtype_t dt, void* workspace, size_t workspace_bytes,
                                              void* stream) {
    int lmax = 0;
    UserLayout ul;
    void* rest = nullptr;
    size_t rest_bytes = 0;
    const path_status_t st = varlen_setup(cu_seqlens, nseq, H, d, dt, workspace, workspace_bytes, stream, &lmax, &ul, &rest, &rest_bytes);
    if (st != PATH_OK) return st;
    return bwd_impl(BWD_FULL, BWD_STAGE_ALL, ul, q, k, v, w, beta, log_f, o, lse, d_o, dq, dk, dv, dw, dbeta, dlog_f, nseq, H, lmax, d,
                    causal, scale, dt, rest, rest_bytes, stream);
}
