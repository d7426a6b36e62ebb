// Host/device argument structs of the backward kernels and their launchers.
#pragma once
#include "path_common.h"

namespace path {

struct BwdParams {
    UserLayout ul;                     // layout of q .. dO, lse and of the gradients
    const void *q, *k, *v, *w, *beta, *o, *dO;
    const float* lse;
    const void *kt, *vk, *ktT, *dpt;   // per-chunk fragment tiles from the chunk transform
    const void *kt2, *kt2T, *dpt2;     // second-level tiles: keys per chunk, -(I - P_superblock) per super-block
    const void *xs, *xsT;              // per-(chunk, key block) query-state tiles from the states sweep
    void *doq, *doT;                   // per-chunk dO tiles (I/O type)
    void* gs;                          // per-pair adjoint-state tiles gT (rows b, contraction q): g(i,j-1) at slot (i,j)
    float *delta;             // [BH][Lp]
    float *lse2p;             // [BH][Lp]: lse * log2(e), zero past L
    float *dqb, *dkb, *dvp;   // [BH][Lp][d] fp32: dQb, dKb, dV (off-diagonal part)
    float *ddp;               // [BH][NC][d][d] fp32: ddP[a][b]
    float *dk2;               // [BH][Lp][d] fp32: dKb2 (gradient of the second-level keys)
    float *dchain;            // [BH][NC+1][d][d] fp32: chain of the second level's adjoint, entry c+1 for chunk c
    const float* cum;         // PaTH-FoX only (else NULL): [BH][Lp] cumulative log2 gates
    float* dcol;              // PaTH-FoX only: [BH][Lp] column sums of the logit gradient
    float* drow;              // PaTH-FoX only: [BH][Lp] row sums of the logit gradient (zero in exact arithmetic)
    int B, H, L, NC;
    float scale;
};

enum { EL_F32 = 0, EL_OP = 1, EL_IO = 2 };           // element type: float, operand type, I/O type
enum { TOK_NONE = 0, TOK_ROW = 1, TOK_K = 2 };       // which index (if any) is a token of the chunk (zero past L)
enum { MASK_NONE = 0, MASK_TRIL = 1, MASK_SLOWER = 2 };

struct MatRef {
    const void* p;
    long long s_bh, s_ch;   // element strides per (batch*head) and per chunk
    int rs, ks;             // element strides of the row (m or n) and contraction index
    int type, tok;
    int user;               // one of the caller's [.,.,.,d] tensors: the base follows the UserLayout instead of s_bh, s_ch
};

struct GemmArgs {
    MatRef A, B;
    float* C;
    const float* Cin;
    long long c_bh, c_ch;
    int crs, ccs;
    int M, N, K;
    float alpha;
    int mask;
    int NC, L;
    int cmul, cadd, gridx;  // workgroup x handles chunk x * cmul + cadd (skipped if >= NC); gridx workgroups per head
    UserLayout ul;
};

// Adjoint of the second blocking level, one workgroup per (super-block, head).
struct SbChainArgs {
    const void* rm;      // [BH][NC][d][d] operand type: R_c row-major
    const void* kbm;     // [BH][Lp][d] operand type: Kb
    const void* utm;     // [BH][NC][d][64] operand type: utm[c][t] = U[t][c]
    const void* w;       // [BH][L][d] I/O type
    const float* dk2;    // [BH][Lp][d]
    const float* dchain; // [BH][NC+1][d][d]: entry 4J = gradient of P_superblock J
    float* ddp;          // [BH][NC][d][d]   (updated)
    float* dkb;          // [BH][Lp][d]      (updated)
    int L, NC;
    UserLayout ul;       // layout of w
};

struct DiagArgs {
    const float *sdm, *dpd, *delta, *lse;
    void *pd, *dsd;       // operand type (read only as matrix operands)
    int L, NC;
    float scale;
    const float* cum;     // PaTH-FoX only (else NULL)
    float* dcol;          // PaTH-FoX only: the diagonal block's column sums are ADDED here
    float* drow;          // PaTH-FoX only: ... and its row sums here
};
struct BetaArgs {
    const float *r, *m, *g;
    const void* beta;
    void* dgs;            // operand type
    float* dbf;
    int L, NC;
};
struct OutArgs {
    const float *dqf, *dkf, *dvf, *dwf, *dbf;
    void *dq, *dk, *dv, *dw, *dbeta;
    int L, NC, d;
};

// Adjoint of the chunk transform as ONE kernel: every workgroup (chunk, head) runs the same
// list of steps.  A step is one product of a chain  acc (+)= alpha * A B^T  (the chain's first
// step starts from Cin or zero, its last step masks and writes C), or one of the element-wise
// specials between the chains.
enum { OP_PRODUCT = 0, OP_DIAG = 1, OP_BETA = 2, OP_STORE = 3 };
enum { OUT_C64 = 0, OUT_TOK = 1, OUT_DD = 2, OUT_DD1 = 3, OUT_D64 = 4 };   // layout of a product's result
struct ChunkOp {
    MatRef A, B;
    float* C;
    const float* Cin;
    long long c_bh, c_ch;
    int crs;
    short M, N, K;
    float alpha;
    unsigned char mask, first, last, kind;
    unsigned char c_op;      // the result is stored in the operand type (it is only read as an operand), not as float
};
constexpr int MAX_CHUNK_OPS = 26;
struct ChunkProgram {
    UserLayout ul;           // layout of the caller's tensors (operands marked `user`, lse, beta, the outputs)
    ChunkOp ops[MAX_CHUNK_OPS];
    int n;
    DiagArgs diag;
    BetaArgs beta;
    OutArgs out;
    int L, NC;
};
hipError_t launch_chunk_adjoint(const ChunkProgram& pr, int BH, int is_bf16, hipStream_t st);

// The same steps as one hand-fused kernel (2-byte operand types): every input is a plain pointer.
struct ChunkFusedArgs {
    UserLayout ul;                               // layout of q .. d_o, lse and of the outputs
    const void *q, *k, *v, *w, *beta, *d_o;      // I/O type, the caller's layout
    const float *lse, *delta;                    // the caller's layout; [BH][Lp]
    const float *sdm, *gm;                       // [BH][NC][64][64]: raw diagonal logits, G
    const void *fm, *gktm, *nm, *aim, *ytm;      // operand type, [BH][NC][64][64]
    const void* utm;                             // operand type, [BH][NC][d][64]
    const float *dqb, *dkb, *dvp;                // [BH][Lp][d]
    const float* ddp;                            // [BH][NC][d][d]
    void *dq, *dk, *dv, *dw, *dbeta;             // I/O type
    const float* cum;                            // PaTH-FoX only (else NULL)
    float *dcol, *drow;
    int L, NC;
    float scale;
};
hipError_t launch_chunk_fused(const ChunkFusedArgs& a, int BH, int d, hipStream_t st);

// Stages of the backward after the transforms, as bits (the public PATH_BWD_STAGE_* values of the header):
// dO tiles + adjoint scan | near key-side | far key-side | far (fp32: and near) ddP | second-level chain and
// chunk-transform adjoint.  launch_bwd_scan runs the first four as asked, in this order.
enum { BWD_STAGE_SCAN = 1, BWD_STAGE_KEYS_NEAR = 2, BWD_STAGE_KEYS_FAR = 4, BWD_STAGE_DDP = 8, BWD_STAGE_CHUNK = 16, BWD_STAGE_ALL = 31 };
hipError_t launch_bwd_scan(const BwdParams& p, int d, int is_bf16, int stages, hipStream_t st);
hipError_t launch_batched_gemm(const GemmArgs& a, int BH, int is_bf16, hipStream_t st);
hipError_t launch_bwd_sb_chain(const SbChainArgs& a, int BH, int d, hipStream_t st);    // 2-byte operand types only

}  // namespace path
