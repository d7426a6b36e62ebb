// Argument structs and launchers of the decode-path kernels.
#pragma once
#include "path_common.h"

namespace path {

constexpr int DECODE_MAX_SPLITS = 64;

struct PrefillArgs {
    const void *kt2, *dp2;   // second-level tiles of the forward workspace
    void* kcache;            // [BH][Lmax][d], cache storage type
    int L, NC, Lmax;
};

struct DecodeArgs {
    const void *q, *k, *v, *w, *beta;   // the arriving token: [BH][d], beta [BH]
    void *kcache, *vcache;              // [BH][Lmax][d]
    void* o;                            // [BH][d]
    float* lse;                         // [BH]
    float* partial;                     // [BH][splits][d + 2]: m, l, o
    int n, Lmax;                        // cached tokens before the step
    float scale;
    // PaTH-FoX (NULL for plain PaTH): the arriving token's log gate [BH] (I/O type) and the running sums
    // c_i = sum_{s<=i} log f_s of the cached tokens, fp32 [BH][Lmax], natural logarithm; the step appends c_n
    const void* log_f;
    float* ccache;
};

hipError_t launch_key_prefill(const PrefillArgs& a, int BH, int d, int is_bf16, hipStream_t st);
hipError_t launch_decode_step(const DecodeArgs& a, int BH, int d, int is_bf16, hipStream_t st);
int decode_num_splits(int BH, int n);

}  // namespace path
