// Internal: the plan the host derives from an fle_problem and hands to the kernels.
// Shared by the HIP-free host translation unit and the kernel translation unit.
#pragma once
#include <stddef.h>
#include <stdint.h>

#include "fle.h"

namespace fle {

// One epilogue op as the kernels see it (pointers are device pointers).
struct DevOp {
    int32_t kind;
    float alpha;
    const void *p0;
    const void *p1;
    int64_t ld;
};

// The op list split at its (single, optional) row reduction.
struct DevEpilogue {
    int32_t n_pre;     // elementwise ops applied in the GEMM kernel's registers
    int32_t n_post;    // elementwise ops applied by the finalize pass, after the row op
    int32_t row_kind;  // FLE_LAYERNORM / FLE_SOFTMAX / FLE_LOGSUMEXP, or -1
    int32_t dtype;     // fle_dtype of b, residual / store operands, gamma, beta and out (fp8 problems: FLE_BF16)
    const void *bias;  // b[N] or nullptr
    DevOp row;         // valid when row_kind >= 0
    DevOp pre[FLE_MAX_OPS];
    DevOp post[FLE_MAX_OPS];
    // a second row reduction later in the list: the finalize pass hands its values over in fp32, a third pass
    // (second_row_op) reduces, normalises and applies the ops behind it
    int32_t row2_kind;  // FLE_LAYERNORM / FLE_SOFTMAX / FLE_LOGSUMEXP, or -1
    int32_t n_post2;
    DevOp row2;
    DevOp post2[FLE_MAX_OPS];
};

enum Variant { V_AUTO = 0, V_GENERAL = 1, V_TILED = 2, V_SKINNY = 3, V_TILED_256 = 4, V_TILED_128 = 5, V_SKINNY_128 = 6, V_SKINNY_256 = 7, V_SKINNY_SEQ = 8, V_THIN = 9 };

// Where the GEMM pass writes its (pre-row-op) values.
enum Staging {
    ST_NONE = 0,  // no row op: final values go straight to out; or logsumexp: nothing staged
    ST_OUT = 1,   // staged in out itself (storage dtype), finalize rewrites it in place
    ST_WS = 2     // staged as fp32 [M,N] in the workspace
};

struct Plan {
    int32_t variant;
    int32_t bm, bn, bk;      // block tile: rows of x, rows of W, K step
    int32_t part_cols;       // columns covered by one row-reduction partial
    int32_t np;              // partials per row = ceil(N / part_cols)
    int32_t staging;
    int32_t stage_rel;       // 2-byte row op staged in out as v - (mean / maximum of v's partial)
    int32_t edge;            // tiled kernel: the epilogue must access b / residual / out one element at a time
    int32_t split_k;         // workgroups along K per tile (1: none); > 1 adds fp32 slabs and a reduction pass
    int32_t groups;          // grouped problem: number of row groups (tiles_m is then an upper bound); 0 otherwise
    int32_t w_stream;        // grouped problem with about one tile row per group: W panels are read once (non-temporal copies)
    int32_t op_dtype;        // fle_dtype of x and W (differs from epi.dtype for fp8 problems only)
    int32_t mx;              // fp8 problem whose operands carry block scales (FLE_MXSCALE)
    const void *x_scale, *w_scale;
    int32_t ln_pre;          // LayerNorm of x over K in front of the multiplication (FLE_LAYERNORM_PRE): LN_PRE_*
    const void *ln_gamma, *ln_beta;
    float ln_eps;
    size_t ws_xhat_off;      // LN_PRE_PASS: the normalised copy of x, [M][K] of the dtype
    int64_t tiles_m, tiles_n;
    size_t ws_part_off, ws_y_off, ws_slab_off, ws_mid_off, ws_total;  // (ws_mid: fp32 [M,N] between two row ops)
    DevEpilogue epi;
};

enum { LN_PRE_NONE = 0, LN_PRE_FUSED = 1, LN_PRE_PASS = 2 };  // inside the dot-product kernel / a pass of its own in front of the GEMM kernel

// Validates p (everything except workspace size) and fills plan.  Host only, no HIP calls.
// groups: nullptr for a plain problem, else the row groups of a grouped one.
fle_status make_plan(const fle_problem *p, int forced_variant, int forced_split, Plan *plan, const fle_groups *groups = nullptr);

// Records the calling thread's error detail; returns s.
fle_status fail(fle_status s, const char *fmt, ...);

// Implemented in the kernel translation unit: enqueue the planned kernels.
fle_status launch(const fle_problem *p, const Plan &plan, const fle_groups *groups = nullptr);

// Implemented in the kernel translation unit: the address, on the current device, of the library's static
// scratch array of FLE_STATIC_SCRATCH_BYTES (looked up once per device; no allocation).
fle_status static_scratch(void **ptr);

// Implemented in the kernel translation unit: enqueue the persistent perceptron kernel for an already validated
// chain (sync: the barrier words; acts: one activation buffer per layer boundary, act_stride bytes apart; all in the workspace).
fle_status launch_chain(const fle_chain *p, void *sync, void *acts, size_t act_stride);

// Implemented in the kernel translation unit: enqueue the attention kernel for an already validated problem.
fle_status launch_attention(const fle_attention *p);

}  // namespace fle
