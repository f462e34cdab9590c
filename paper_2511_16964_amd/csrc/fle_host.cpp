// Host side of libfle: argument validation, epilogue grammar, kernel planning and the C ABI.
// This translation unit makes no HIP call, so everything it decides is testable without a GPU.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>

#include "fle_plan.h"

namespace fle {

static thread_local char g_error[512] = "";
// The calling thread's most recent plan; its text is only formatted when fle_last_plan asks for it.
static thread_local Plan g_plan;
static thread_local bool g_have_plan = false;
static thread_local int g_forced = V_AUTO;
static thread_local int g_split = 0;

fle_status fail(fle_status s, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof g_error, fmt, ap);
    va_end(ap);
    return s;
}

static inline bool is_row_op(int k) { return k == FLE_LAYERNORM || k == FLE_SOFTMAX || k == FLE_LOGSUMEXP; }
static inline size_t esize(int dtype) { return dtype == FLE_F32 ? 4 : 2; }
static inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
static inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Half-open byte ranges [a, a+na) and [b, b+nb) intersect.
static bool overlaps(const void *a, size_t na, const void *b, size_t nb) {
    if (!a || !b || na == 0 || nb == 0) return false;
    uintptr_t pa = reinterpret_cast<uintptr_t>(a), pb = reinterpret_cast<uintptr_t>(b);
    return pa < pb + nb && pb < pa + na;
}

static size_t span_bytes(int64_t rows, int64_t cols, int64_t ld, size_t es) {
    if (rows <= 0 || cols <= 0) return 0;
    return (static_cast<size_t>(rows - 1) * static_cast<size_t>(ld) + static_cast<size_t>(cols)) * es;
}

// Grouped problems with at most this many rows per group on average read nearly every W panel once: their W
// copies carry the non-temporal hint (32 groups of 4096 x 4096, 512 rows in all: 187 -> 174 us back to back,
// 249 -> 185 us from cold caches; at 128 rows per group the hint costs 3 % back to back, so the limit is 64).
static const int64_t kGroupedStreamRows = 64;

static fle_status make_plan_core(const fle_problem *p, int forced, int forced_split, Plan *plan, const fle_groups *grp);

// A list that starts with FLE_LAYERNORM_PRE: the rest of the list is planned as a problem of its own, first on x as
// it is.  If that gives the dot-product kernel for a few rows, the kernel normalises in its own sweep and nothing else
// changes.  Otherwise a pass writes the normalised rows into the workspace and the rest is planned again for that
// copy (contiguous and aligned whatever x looks like).
fle_status make_plan(const fle_problem *p, int forced, int forced_split, Plan *plan, const fle_groups *grp) {
    if (!p) return fail(FLE_ERR_NULL, "problem is NULL");
    bool ln_pre = false;
    if (p->n_ops > 0 && p->n_ops <= FLE_MAX_OPS && p->ops)
        for (int i = 0; i < p->n_ops; ++i)
            if (p->ops[i].kind == FLE_LAYERNORM_PRE) {
                if (i != 0) return fail(FLE_ERR_UNSUPPORTED, "op %d: the LayerNorm of x must be the first entry of the list", i);
                ln_pre = true;
            }
    if (!ln_pre) return make_plan_core(p, forced, forced_split, plan, grp);
    const fle_op &op = p->ops[0];
    if (grp) return fail(FLE_ERR_UNSUPPORTED, "op 0: grouped problems take no LayerNorm of x");
    if (p->dtype == FLE_F8E4M3) return fail(FLE_ERR_UNSUPPORTED, "op 0: fp8 operands take no LayerNorm of x");
    if (!(op.alpha >= 0.0f && std::isfinite(op.alpha))) return fail(FLE_ERR_OP, "op 0: layernorm eps must be finite and >= 0");
    if (p->K < 1) return fail(FLE_ERR_SHAPE, "op 0: a LayerNorm of x needs K >= 1");
    fle_problem q = *p;
    q.ops = p->ops + 1;
    q.n_ops = p->n_ops - 1;
    fle_status s = make_plan_core(&q, forced, forced_split, plan, nullptr);
    if (s != FLE_OK && !(s == FLE_ERR_UNSUPPORTED && forced != V_AUTO)) return s;  // (a forced kernel may only fit the copy)
    const size_t es = p->dtype == FLE_F32 ? 4 : 2;
    if (!aligned(op.p0, es) || !aligned(op.p1, es)) return fail(FLE_ERR_ALIGN, "op 0: gamma/beta not aligned to the element size");
    if (p->M > 0 && p->out) {
        const size_t ob = (plan->epi.row_kind == FLE_LOGSUMEXP || plan->epi.row2_kind == FLE_LOGSUMEXP) ? size_t(p->M) * es : span_bytes(p->M, p->N, p->ldo, es);
        if (overlaps(p->out, ob, op.p0, size_t(p->K) * es) || overlaps(p->out, ob, op.p1, size_t(p->K) * es)) return fail(FLE_ERR_UNSUPPORTED, "op 0: out overlaps gamma or beta");
    }
    const bool fused = s == FLE_OK && plan->variant == V_THIN && plan->bm == 8 && p->M <= 4;  // (8 fp32 rows with the extra sums need more than 256 registers)
    if (!fused) {
        q.x = reinterpret_cast<const void *>(uintptr_t(256));  // stands for the copy: aligned, rows contiguous, overlapping nothing
        q.ldx = p->K;
        s = make_plan_core(&q, forced, forced_split, plan, nullptr);
        if (s != FLE_OK) return s;
        plan->ws_xhat_off = plan->ws_total;
        plan->ws_total = round_up(plan->ws_total + size_t(p->M) * size_t(p->K) * es, 256);
    }
    plan->ln_pre = fused ? LN_PRE_FUSED : LN_PRE_PASS;
    plan->ln_gamma = op.p0;
    plan->ln_beta = op.p1;
    plan->ln_eps = op.alpha;
    return FLE_OK;
}

static fle_status make_plan_core(const fle_problem *p, int forced, int forced_split, Plan *plan, const fle_groups *grp) {
    if (!p) return fail(FLE_ERR_NULL, "problem is NULL");
    std::memset(plan, 0, sizeof *plan);
    if (p->dtype != FLE_F32 && p->dtype != FLE_BF16 && p->dtype != FLE_F16 && p->dtype != FLE_F8E4M3)
        return fail(FLE_ERR_OP, "dtype %d is not FLE_F32, FLE_BF16, FLE_F16 or FLE_F8E4M3", p->dtype);
    const bool f8 = p->dtype == FLE_F8E4M3;
    const int64_t M = p->M, N = p->N, K = p->K;
    const int64_t kLimit = int64_t(1) << 40;
    if (M < 0 || N < 1 || K < 0) return fail(FLE_ERR_SHAPE, "need M >= 0, N >= 1, K >= 0 (got %lld, %lld, %lld)", (long long)M, (long long)N, (long long)K);
    if (M > kLimit || N > (int64_t(1) << 30) || K > (int64_t(1) << 30)) return fail(FLE_ERR_SHAPE, "size too large");
    if (p->n_ops < 0 || p->n_ops > FLE_MAX_OPS) return fail(FLE_ERR_OP, "n_ops %d outside 0..%d", p->n_ops, FLE_MAX_OPS);
    if (p->n_ops > 0 && !p->ops) return fail(FLE_ERR_NULL, "ops is NULL with n_ops %d", p->n_ops);

    const int64_t G = grp ? grp->n_groups : 0;
    if (grp) {
        if (G < 1 || G > 65536) return fail(FLE_ERR_SHAPE, "n_groups %lld outside 1..65536", (long long)G);
        if (grp->w_group_stride < 0 || grp->b_group_stride < 0 || grp->w_group_stride > kLimit || grp->b_group_stride > kLimit) return fail(FLE_ERR_SHAPE, "group strides must be >= 0");
        if (M > 0 && !grp->row_offsets) return fail(FLE_ERR_NULL, "row_offsets is NULL");
        if (!aligned(grp->row_offsets, 8)) return fail(FLE_ERR_ALIGN, "row_offsets is not aligned to 8 bytes");
    }
    plan->groups = int32_t(G);

    DevEpilogue &e = plan->epi;
    e.row_kind = -1;
    e.row2_kind = -1;
    e.dtype = f8 ? int32_t(FLE_BF16) : p->dtype;  // fp8 problems: everything but x and W is bf16
    e.bias = p->b;
    plan->op_dtype = p->dtype;
    const size_t es = esize(e.dtype);      // bytes per element of b, residual / store operands, gamma, beta, out
    const size_t xs = f8 ? 1 : es;         // bytes per element of x and W
    for (int i = 0; i < p->n_ops; ++i) {
        const fle_op &op = p->ops[i];
        if (op.kind < FLE_BIAS || op.kind > FLE_LAYERNORM_PRE) return fail(FLE_ERR_OP, "op %d: unknown kind %d", i, op.kind);
        if (op.kind == FLE_LAYERNORM_PRE) return fail(FLE_ERR_UNSUPPORTED, "op %d: the LayerNorm of x must be the first entry of the list", i);
        if (op.kind == FLE_MXSCALE) {  // not an epilogue op: says how x and W are to be read
            if (i != 0) return fail(FLE_ERR_UNSUPPORTED, "op %d: the block scales of x and W must be the first entry of the list", i);
            if (!f8) return fail(FLE_ERR_UNSUPPORTED, "op %d: block scales need FLE_F8E4M3 operands", i);
            if (grp) return fail(FLE_ERR_UNSUPPORTED, "op %d: grouped problems take no block scales", i);
            if (K % 128 != 0) return fail(FLE_ERR_UNSUPPORTED, "op %d: block scales need K to be a multiple of 128 (got %lld)", i, (long long)K);
            if ((!op.p0 || !op.p1) && M > 0 && K > 0) return fail(FLE_ERR_NULL, "op %d: a block-scale pointer is NULL", i);
            if (!aligned(op.p0, 4) || !aligned(op.p1, 4)) return fail(FLE_ERR_ALIGN, "op %d: block scales must be 4-byte aligned", i);
            plan->mx = 1;
            plan->x_scale = op.p0;
            plan->w_scale = op.p1;
            continue;
        }
        if (e.row_kind == FLE_LOGSUMEXP || e.row2_kind == FLE_LOGSUMEXP) return fail(FLE_ERR_UNSUPPORTED, "op %d follows logsumexp, which must be last", i);
        DevOp d{op.kind, op.alpha, op.p0, op.p1, op.ld};
        if (is_row_op(op.kind)) {
            if (e.row2_kind >= 0) return fail(FLE_ERR_UNSUPPORTED, "op %d: a third row reduction in one list is not supported", i);
            if (e.row_kind >= 0 && grp) return fail(FLE_ERR_UNSUPPORTED, "op %d: grouped problems take one row reduction", i);
            if (op.kind == FLE_LAYERNORM && !(op.alpha >= 0.0f && std::isfinite(op.alpha))) return fail(FLE_ERR_OP, "op %d: layernorm eps must be finite and >= 0", i);
            if (e.row_kind >= 0) { e.row2_kind = op.kind; e.row2 = d; }
            else { e.row_kind = op.kind; e.row = d; }
            continue;
        }
        if (op.kind == FLE_BIAS && !p->b && M > 0) return fail(FLE_ERR_NULL, "op %d: bias listed but b is NULL", i);
        if (op.kind == FLE_SCALE && !std::isfinite(op.alpha)) return fail(FLE_ERR_OP, "op %d: scale factor is not finite", i);
        if (op.kind == FLE_RESIDUAL || op.kind == FLE_STORE) {
            const char *what = op.kind == FLE_STORE ? "store" : "residual";
            if (!op.p0 && M > 0) return fail(FLE_ERR_NULL, "op %d: %s pointer is NULL", i, what);
            if (op.ld < N) return fail(FLE_ERR_SHAPE, "op %d: %s ld %lld < N %lld", i, what, (long long)op.ld, (long long)N);
            if (op.ld > kLimit) return fail(FLE_ERR_SHAPE, "op %d: %s ld too large", i, what);
            if (op.kind == FLE_STORE && e.row_kind >= 0) return fail(FLE_ERR_UNSUPPORTED, "op %d: a store after the row op is not supported", i);
        }
        if (e.row_kind < 0) e.pre[e.n_pre++] = d;
        else if (e.row2_kind < 0) e.post[e.n_post++] = d;
        else e.post2[e.n_post2++] = d;
    }
    const bool lse = e.row_kind == FLE_LOGSUMEXP || e.row2_kind == FLE_LOGSUMEXP;  // out is [M]
    if (p->ldx < K || p->ldw < K) return fail(FLE_ERR_SHAPE, "ldx %lld / ldw %lld smaller than K %lld", (long long)p->ldx, (long long)p->ldw, (long long)K);
    if (!lse && p->ldo < N) return fail(FLE_ERR_SHAPE, "ldo %lld < N %lld", (long long)p->ldo, (long long)N);
    if (p->ldx > kLimit || p->ldw > kLimit || p->ldo > kLimit) return fail(FLE_ERR_SHAPE, "leading dimension too large");
    if (M > 0) {
        if (!p->out) return fail(FLE_ERR_NULL, "out is NULL");
        if (K > 0 && (!p->x || !p->w)) return fail(FLE_ERR_NULL, "x or w is NULL");
        // element alignment is the only hard requirement
        if (!aligned(p->x, xs) || !aligned(p->w, xs) || !aligned(p->out, es) || !aligned(p->b, es)) return fail(FLE_ERR_ALIGN, "a pointer is not aligned to its element size");
        const size_t out_bytes = lse ? size_t(M) * es : span_bytes(M, N, p->ldo, es);
        const size_t w_bytes = span_bytes(N, K, p->ldw, xs) + (grp ? size_t(G - 1) * size_t(grp->w_group_stride) * xs : 0);
        const size_t b_bytes = size_t(N) * es + (grp ? size_t(G - 1) * size_t(grp->b_group_stride) * es : 0);
        if (overlaps(p->out, out_bytes, p->x, span_bytes(M, K, p->ldx, xs)) || overlaps(p->out, out_bytes, p->w, w_bytes) || overlaps(p->out, out_bytes, p->b, b_bytes))
            return fail(FLE_ERR_UNSUPPORTED, "out overlaps x, w or b");
        if (plan->mx && (overlaps(p->out, out_bytes, plan->x_scale, size_t(M) * size_t(K / 32)) || overlaps(p->out, out_bytes, plan->w_scale, size_t(N) * size_t(K / 32)) ||
                         overlaps(p->workspace, p->workspace_bytes, plan->x_scale, size_t(M) * size_t(K / 32)) || overlaps(p->workspace, p->workspace_bytes, plan->w_scale, size_t(N) * size_t(K / 32))))
            return fail(FLE_ERR_UNSUPPORTED, "out or the workspace overlaps the block scales");
        if (grp && (overlaps(p->out, out_bytes, grp->row_offsets, size_t(G + 1) * 8) || overlaps(p->workspace, p->workspace_bytes, grp->row_offsets, size_t(G + 1) * 8)))
            return fail(FLE_ERR_UNSUPPORTED, "out or the workspace overlaps row_offsets");
        for (int i = 0; i < p->n_ops; ++i) {
            const fle_op &op = p->ops[i];
            if (op.kind == FLE_RESIDUAL) {
                if (!aligned(op.p0, es)) return fail(FLE_ERR_ALIGN, "op %d: residual pointer not aligned to its element size", i);
                const bool same = op.p0 == p->out && op.ld == p->ldo && !lse;
                if (!same && overlaps(p->out, out_bytes, op.p0, span_bytes(M, N, op.ld, es))) return fail(FLE_ERR_UNSUPPORTED, "op %d: out overlaps the residual without being identical to it", i);
            } else if (op.kind == FLE_STORE) {
                if (!aligned(op.p0, es)) return fail(FLE_ERR_ALIGN, "op %d: store pointer not aligned to its element size", i);
                const size_t t_bytes = span_bytes(M, N, op.ld, es);
                bool clash = overlaps(op.p0, t_bytes, p->out, out_bytes) || overlaps(op.p0, t_bytes, p->x, span_bytes(M, K, p->ldx, xs)) ||
                             overlaps(op.p0, t_bytes, p->w, w_bytes) || overlaps(op.p0, t_bytes, p->b, b_bytes) ||
                             overlaps(op.p0, t_bytes, p->workspace, p->workspace_bytes) || (grp && overlaps(op.p0, t_bytes, grp->row_offsets, size_t(G + 1) * 8));
                for (int j = 0; j < p->n_ops && !clash; ++j) {
                    const fle_op &o2 = p->ops[j];
                    if (j == i) continue;
                    if (o2.kind == FLE_RESIDUAL || o2.kind == FLE_STORE) clash = overlaps(op.p0, t_bytes, o2.p0, span_bytes(M, N, o2.ld, es));
                    else if (o2.kind == FLE_LAYERNORM) clash = overlaps(op.p0, t_bytes, o2.p0, size_t(N) * es) || overlaps(op.p0, t_bytes, o2.p1, size_t(N) * es);
                }
                if (clash) return fail(FLE_ERR_UNSUPPORTED, "op %d: the store target overlaps another operand, out or the workspace", i);
            } else if (op.kind == FLE_LAYERNORM) {
                if (!aligned(op.p0, es) || !aligned(op.p1, es)) return fail(FLE_ERR_ALIGN, "op %d: gamma/beta not aligned to the element size", i);
                if (overlaps(p->out, out_bytes, op.p0, size_t(N) * es) || overlaps(p->out, out_bytes, op.p1, size_t(N) * es)) return fail(FLE_ERR_UNSUPPORTED, "op %d: out overlaps gamma or beta", i);
            }
        }
        if (p->workspace && overlaps(p->out, out_bytes, p->workspace, p->workspace_bytes)) return fail(FLE_ERR_UNSUPPORTED, "out overlaps the workspace");
    }

    // ---- kernel variant
    const bool f32 = p->dtype == FLE_F32;
    // The tiled kernels copy 16-byte chunks and read / write groups of 4 consecutive columns.
    const int64_t chunk = 16 / int64_t(xs);                  // x / W elements per 16-byte chunk: 16 fp8, 8 bf16, 4 fp32
    const size_t vec4 = 4 * es;                              // alignment of a 4-column group
    const int64_t ld_max = (int64_t(1) << 22) / int64_t(es); // 32-bit byte offsets inside a 256-row tile (epilogue operands)
    const int64_t ldx_max = (int64_t(1) << 22) / int64_t(xs);  // (x and W)
    bool res_ok = true, post_res_alias_out = false;
    for (int i = 0; i < e.n_pre; ++i) {
        if ((e.pre[i].kind == FLE_RESIDUAL || e.pre[i].kind == FLE_STORE) && !(aligned(e.pre[i].p0, vec4) && e.pre[i].ld % 4 == 0 && e.pre[i].ld < ld_max)) res_ok = false;
    }
    for (int i = 0; i < e.n_post; ++i)
        if (e.post[i].kind == FLE_RESIDUAL && e.post[i].p0 == p->out) post_res_alias_out = true;
    for (int i = 0; i < e.n_post2; ++i)
        if (e.post2[i].kind == FLE_RESIDUAL && e.post2[i].p0 == p->out) post_res_alias_out = true;
    // x and W rows must be whole, aligned 16-byte chunks; everything the epilogue touches may be ragged
    // (the kernel then has an element-wise epilogue)
    const bool tiled_ok = K >= chunk && K % chunk == 0 && aligned(p->x, 16) && aligned(p->w, 16) && p->ldx % chunk == 0 && p->ldw % chunk == 0 &&
                          p->ldx < ldx_max && p->ldw < ldx_max && (!grp || grp->w_group_stride % chunk == 0);
    const bool vec_epi = N % 4 == 0 && (lse || (aligned(p->out, vec4) && p->ldo % 4 == 0)) && aligned(p->b, vec4) && res_ok && (!grp || grp->b_group_stride % 4 == 0);
    if (grp) {
        // Grouped problems run on the tiled kernels only, one workgroup per tile over the whole K.  A group's
        // tile rows start at its first row, so with rows spread over G groups about G / 2 tile rows are
        // partly empty: the 256 tile (1.45 us per K step for 4 times the outputs of a 128 tile, which costs
        // 0.85 / 2 with two workgroups per CU) only pays when groups hold several hundred rows.
        if (forced != V_AUTO && forced != V_TILED && forced != V_TILED_256 && forced != V_TILED_128) return fail(FLE_ERR_UNSUPPORTED, "grouped problems run on the tiled kernels only");
        if (forced_split > 1) return fail(FLE_ERR_UNSUPPORTED, "grouped problems are not split along K");
        if (!tiled_ok) return fail(FLE_ERR_UNSUPPORTED, "a grouped problem needs x and W rows made of whole, 16-byte aligned chunks (K, the leading dimensions and the W group stride multiples of 16 bytes)");
        if (forced == V_AUTO || forced == V_TILED) {
            auto cost = [&](int tile) -> double {
                const double wgs = (double(M) / tile + 0.5 * double(G)) * double((N + tile - 1) / tile);
                const double slots = tile == 128 ? 512.0 : 256.0;
                const double per_step = p->dtype == FLE_F32 ? (tile == 256 ? 7.8 : 3.9) : (tile == 256 ? 1.45 : 0.85);
                return (wgs > slots ? wgs / slots : 1.0) * per_step;
            };
            forced = (M > 128 && N > 128 && cost(256) < cost(128)) ? V_TILED_256 : V_TILED_128;
        }
        forced_split = 1;
    }
    if (f8) {  // fp8 operands exist on the tiled kernels only
        if (forced != V_AUTO && forced != V_TILED && forced != V_TILED_256 && forced != V_TILED_128) return fail(FLE_ERR_UNSUPPORTED, "fp8 problems run on the tiled kernels only");
        if (!tiled_ok) return fail(FLE_ERR_UNSUPPORTED, "an fp8 problem needs x and W rows made of whole, 16-byte aligned chunks (K and the leading dimensions multiples of 16 elements, K >= 16)");
        if (forced == V_AUTO) forced = V_TILED;
    }
    int variant = forced, forced_tile = 0;
    if (variant == V_TILED_256 || variant == V_TILED_128) {
        forced_tile = variant == V_TILED_256 ? 256 : 128;
        variant = V_TILED;
    }
    int forced_bk = 0;
    bool forced_seq = false;
    if (variant == V_SKINNY_128 || variant == V_SKINNY_256 || variant == V_SKINNY_SEQ) {
        forced_bk = variant == V_SKINNY_128 ? 128 : 256;
        forced_seq = variant == V_SKINNY_SEQ;
        variant = V_SKINNY;
    }
    const bool skinny_ok = !f8 && tiled_ok && vec_epi && M <= 256 && K % (f32 ? 32 : 64) == 0;  // a K step is at least 128 bytes of every row
    const bool thin_ok = !f8 && tiled_ok && M >= 1 && M <= 32;  // element-wise epilogue: nothing else needs alignment

    // Tile and split of K of the tiled kernel together, by a coarse time model (microseconds) fitted
    // to measured runs.  bf16: a K step (128 bytes of every row) costs a 256 tile 1.45, a 128 tile 0.85
    // with two workgroups per CU and 0.6 alone.  fp32: the matrix pipe bounds a K step at 7.8 / 3.9 /
    // 1.95.  Filling the pipeline and the epilogue cost about 15 us (256 tile) or 6 us;
    // workgroups beyond the 256 (512) that are resident at once wait for a second round; a split adds
    // a launch and 8 S M N bytes of slab traffic at about 6 TB/s (the slabs mostly stay in the
    // last-level cache).
    const int64_t tiled_steps = (K * int64_t(xs) + 127) / 128;
    auto tiled_cost = [&](int tile, int64_t sp) -> double {
        const int64_t tiles = ((M + tile - 1) / tile) * ((N + tile - 1) / tile), wgs = tiles * sp;
        const int64_t slots = tile == 128 ? 512 : 256, rounds = (wgs + slots - 1) / slots;
        // (a 256 tile whose K is split over no more workgroups than there are CUs measured 1.3 per step: 768 .. 2048 x
        // 4096 x 16384 with K split in 2 or 4 came out 10 - 26 % ahead of the 128 tile where 1.45 said the opposite)
        const double per_step = f32 ? (tile == 256 ? 7.8 : wgs > 256 ? 3.9 : 1.95) : (tile == 256 ? (sp > 1 && wgs <= 256 ? 1.3 : 1.45) : wgs > 256 ? 0.85 : 0.6);
        // in K steps; two co-resident 128 tiles hide part of each other's epilogue
        const double fixed = f32 ? (tile == 256 ? 1.5 : 3.5) : (tile == 256 ? 10.5 : wgs > 256 ? 7.0 : 8.0);
        double t = double(rounds) * (double((tiled_steps + sp - 1) / sp) + fixed) * per_step;
        if (sp > 1) t += 4.0 + 8.0 * double(sp) * double(M) * double(N) / 6.0e6;
        return t;
    };
    int best_tile = 0, best_split = 1;
    double best = 0.0;
    if (tiled_ok && M > 0) {
        static const int kSplits[] = {1, 2, 3, 4, 6, 8, 12, 16};
        for (int tile = 128; tile <= 256; tile += 128) {
            if (forced_tile ? tile != forced_tile : (tile == 256 && !(M > 128 && N > 128))) continue;
            for (int sp : kSplits) {
                if (forced_split > 0 ? sp != 1 : (sp > 1 && (sp * 4 > tiled_steps || int64_t(sp) * M * (N + 3) * 4 > (int64_t(128) << 20)))) continue;
                const double t = tiled_cost(tile, sp);
                if (!best_tile || t < best) { best = t; best_tile = tile; best_split = sp; }
            }
        }
    }
    if (!best_tile) best_tile = forced_tile ? forced_tile : 128;
    if (variant == V_AUTO) {
        // W is worth streaming: always for a small M; up to 128 rows when W (256 MB or more) cannot stay in the
        // Infinity Cache anyway (measured: 128 x 32768 x 8192 124 us against 156 us tiled; at 134 MB the tiled
        // kernel wins warm and cold; 8 sub-blocks are slower than the tiled kernel everywhere)
        // A few rows against a whole weight matrix (a perceptron layer at batch 1 .. 32): the thin kernels, where
        // they measured faster than what follows.  Dot-product form: fp32 up to 8 rows from 512 x 1024 weights on
        // (4096^2 at one row: 16 us against 33 us general; 1024 x 32768: 46 against 110); 2-byte dtypes up to 4
        // rows while the skinny kernel would need a split of K and a second launch (4096^2: 8.5-9.6 us against
        // 12.5), i.e. up to 2^24 weights (any size for a single row: 32768 x 8192 85 us against 91), with rows of
        // 2048 or more beyond 2^22.  MFMA form: 2-byte dtypes, 5 .. 32 rows,
        // 2^20 .. 2^23 weights (2048^2 at 16 rows: 7.9 us against 10.4).
        const int64_t nk = N * K;
        const bool gemv_auto = thin_ok && M <= (f32 ? 8 : 4) && nk >= (int64_t(1) << 19) &&
                               (f32 || ((M == 1 || nk <= (int64_t(1) << 24)) && (nk <= (int64_t(1) << 22) || K >= 2048)));
        const bool thin_auto = thin_ok && !f32 && M > 4 && nk >= (int64_t(1) << 20) && nk <= (int64_t(1) << 23);
        if ((gemv_auto || thin_auto) && forced_split <= 1) variant = V_THIN;
        // (fp32 operands keep the matrix pipe about as busy as the memory system: worth it from 2^24 weights on,
        // 2^25 up to 16 rows where the general kernel's 16 x 16 tiles are as fast; 8192^2 at 16 rows 83 -> 60 us)
        // 65 .. 128 rows of a 2-byte dtype: the skinny kernel with 64 rows at once on a 128-wide K step.  Measured with
        // the weights coming from memory, as they do when a layer is used once per pass: 128 x 16384 x 4096 42.5 us
        // against 77.0 us for the 128 tile with K split, 128 x 4096 x 16384 50.4 against 74.4, 128 x 4096 x 4096 20.7
        // against 28.2; in a back-to-back loop, where up to 256 MB of weights stay in the Infinity Cache for the
        // tiled kernel's cacheable copies, within 12 % either way.  (192 .. 256 rows: 20 - 35 % faster from memory
        // but 35 - 50 % slower back to back; left to the tuned table.)
        else if (skinny_ok && !f32 && M > 64 && M <= 128 && K % 128 == 0 && N >= 2048 && N * K >= (int64_t(1) << 22) && forced_split <= 1) {
            variant = V_SKINNY;
            forced_bk = 128;
        }
        else if (skinny_ok && ((M <= 64 && N >= 2048 && N * K >= (int64_t(1) << (f32 ? (M <= 16 ? 25 : 24) : 22))) || (!f32 && M <= 128 && K % 256 == 0 && N >= 8192 && N * K >= (int64_t(1) << 27)))) variant = V_SKINNY;
        else {
            // The general kernel: about 4 us of launch and latency, then either its throughput (55 TFLOP/s on
            // fp32 operands, 70 on bf16) or, for few workgroups and a long K, the serial chain of one
            // workgroup (1.25 us per 256 of K; up to 4 workgroups per CU are resident).
            const int64_t gt = (M <= 16 || ((M + 31) / 32) * ((N + 31) / 32) < 128) ? 16 : 32;
            const int64_t gw = ((M + gt - 1) / gt) * ((N + gt - 1) / gt);
            const double chain = double((gw + 1023) / 1024) * double((K + 255) / 256) * 1.25;
            const double rate = 2.0 * double(M) * double(N) * double(K) / (f32 ? 55.0e6 : 70.0e6);
            const double general = 4.0 + (chain > rate ? chain : rate);
            // a forced split only exists on the tiled and skinny kernels
            variant = (tiled_ok && M > 0 && (best < general || forced_split > 1)) ? V_TILED : V_GENERAL;
        }
    }
    if (variant == V_SKINNY && !skinny_ok) return fail(FLE_ERR_UNSUPPORTED, "the skinny kernel needs M <= 256, K a multiple of 128 bytes and everything the tiled kernel needs");
    if (variant == V_TILED && !tiled_ok) return fail(FLE_ERR_UNSUPPORTED, "the tiled MFMA kernel needs x and W rows made of whole, 16-byte aligned chunks (K and the leading dimensions multiples of 16 bytes)");
    if (variant == V_THIN && !thin_ok) return fail(FLE_ERR_UNSUPPORTED, "the thin kernel needs M <= 32 and everything the tiled kernel needs of x and W");
    if (variant == V_THIN && forced_split > 1) return fail(FLE_ERR_UNSUPPORTED, "the thin kernel does not split K");
    if (variant != V_TILED && variant != V_GENERAL && variant != V_SKINNY && variant != V_THIN) return fail(FLE_ERR_OP, "unknown forced variant %d", variant);
    plan->variant = variant;
    plan->edge = 0;
    int auto_split = 0;  // chosen with the tile (tiled kernel); 0: decided below
    if (variant == V_SKINNY) {
        // The widest K step that fits two stages wins on an MI355X: 512-byte runs per W row stream at
        // 6.0 TB/s where 128- and 256-byte runs reach 4.5 TB/s.  forced 64 keeps the narrow ring for comparison.
        int bk = forced_bk ? forced_bk : 256;  // in 2-byte elements; fp32 operands take half as many for the same bytes
        if (forced == V_SKINNY) bk = 64;
        const int per = f32 ? 2 : 1;
        while (bk > 64 && K % (bk / per) != 0) bk /= 2;
        // Row blocks of 32.  More than 32 rows: one block of 64, 128 or 256 rows whose 32-row sub-blocks take
        // turns on a 256-wide W stage (automatic choice; with fewer than 64 W tiles the chip is not full and
        // more, smaller workgroups do better), or, on request, 64 rows at once on a 128-wide K step; a forced
        // 256-wide K step keeps blocks of 32 (one workgroup each) for comparison.
        plan->bm = 32;
        if (f32) { /* row blocks of 32 only */ }
        else if (M > 32 && forced_bk == 128 && bk == 128) plan->bm = 64;
        else if (M > 32 && bk == 256 && (forced_seq || (forced == V_AUTO && N >= 8192))) plan->bm = M <= 64 ? 64 : M <= 128 ? 128 : 256;
        plan->bn = 128;
        plan->bk = bk / per;
        plan->part_cols = 32;  // one partial per wave tile
    } else if (variant == V_THIN) {
        // few rows: dot products on row-contiguous loads (the vector ALU keeps up with HBM to 4 rows of a 2-byte
        // dtype, 8 of fp32); else the 16x16 MFMA
        plan->bm = M <= (f32 ? 8 : 4) ? 8 : M <= 16 ? 16 : 32;
        plan->bn = 16;
        plan->bk = int32_t(64 / es);  // MFMA form: one step is 64 bytes of every row
        if (plan->bm == 8) {
            // dot-product form: the field holds the W rows per wave instead.  One row of x against many long rows
            // of W: one W row per wave and 16 waves per workgroup keep more loads in flight (fp32 8192^2: 53 ->
            // 47 us; bf16 32768 x 8192: 91 -> 85 us); with more x rows or few W rows 4 per wave are faster.
            plan->bk = (M == 1 && N >= 4096 && K >= 2048) ? 1 : 4;
        }
        plan->part_cols = 16;
    } else if (variant == V_TILED) {
        plan->bm = plan->bn = best_tile;
        plan->bk = f32 ? 32 : f8 ? 128 : 64;
        plan->part_cols = plan->bn / 2;  // one partial per wave column
        plan->edge = vec_epi ? 0 : 1;
        auto_split = best_split;
    } else {
        // 32 x 32 tiles; 16 x 16 when those would give fewer than 128 workgroups (tiny, latency-bound problems)
        const int64_t t32 = ((M + 31) / 32) * ((N + 31) / 32);
        plan->bm = plan->bn = (M <= 16 || t32 < 128) ? 16 : 32;  // (up to 16 rows a 32-row tile would be half empty)
        plan->bk = 16;
        plan->part_cols = 16;
    }
    plan->tiles_m = (M + plan->bm - 1) / plan->bm;
    if (grp) {  // every group may end in a partly filled tile row; the kernel finds the actual count
        plan->tiles_m = M / plan->bm + G;
        if (plan->tiles_m > M) plan->tiles_m = M;
        plan->w_stream = (plan->bm == 128 && M <= G * kGroupedStreamRows) ? 1 : 0;
    }
    plan->tiles_n = (N + plan->bn - 1) / plan->bn;
    if (plan->tiles_m * plan->tiles_n > (int64_t(1) << 31) - 1) return fail(FLE_ERR_SHAPE, "too many tiles for one launch");

    // ---- split K: few tiles and a long K leave most of the chip idle, so several workgroups share
    // a tile, each over its own K range, writing fp32 slabs that a reduction pass sums in slab order
    // (deterministic).
    plan->split_k = 1;
    if (variant != V_GENERAL && variant != V_THIN && M > 0) {
        const int64_t steps = variant == V_TILED ? tiled_steps : K / plan->bk;
        int64_t s = 1;
        if (forced_split > 0) s = forced_split;
        else if (auto_split > 0) s = auto_split;
        else {  // skinny kernel: fill the chip as long as every workgroup keeps at least 512 of K
            const int64_t tiles = plan->tiles_m * plan->tiles_n;
            const int64_t min_steps = 512 / plan->bk > 2 ? 512 / plan->bk : 2;
            if (tiles * 2 <= 256) {
                s = 256 / tiles;
                if (s > steps / min_steps) s = steps / min_steps;
                if (s > 16) s = 16;
            }
        }
        if (s > steps) s = steps;
        if (s > 64) s = 64;
        if (s < 1) s = 1;
        plan->split_k = int32_t(s);
        if (s > 1) plan->part_cols = 256;  // the reduction pass owns the partials
    }

    // ---- staging and workspace
    size_t off = 0;
    plan->staging = ST_NONE;
    plan->stage_rel = 0;
    if (e.row_kind >= 0) {
        plan->np = int32_t((N + plan->part_cols - 1) / plan->part_cols);
        plan->ws_part_off = off;
        off = round_up(off + size_t(M) * size_t(plan->np) * 2 * sizeof(float), 256);
        if (e.row_kind != FLE_LOGSUMEXP) {
            // Staged in out itself unless a trailing residual aliases out (or out is the [M] vector of a logsumexp
            // that comes second).  A 2-byte dtype stages v minus the
            // statistic of v's partial (its mean for LayerNorm, its maximum for softmax), which the finalize pass
            // adds back in fp32: the rounding error of the staged value is then relative to the distance from that
            // statistic, not to v itself (a row of mean 100 and deviation 0.01 keeps its deviations; exp() of a
            // distance d <= 0 is off by at most |d| 2^-9, negligible where the probability is not).
            const bool in_out = !post_res_alias_out && !lse;
            plan->staging = in_out ? ST_OUT : ST_WS;
            plan->stage_rel = (in_out && p->dtype != FLE_F32) ? 1 : 0;
            if (!in_out) {
                plan->ws_y_off = off;
                off = round_up(off + size_t(M) * size_t(N) * sizeof(float), 256);
            }
        }
    }
    if (e.row2_kind >= 0) {  // the values between the two row reductions, fp32 [M,N]
        plan->ws_mid_off = off;
        off = round_up(off + size_t(M) * size_t(N) * sizeof(float), 256);
    }
    if (plan->split_k > 1) {
        plan->ws_slab_off = off;
        off = round_up(off + size_t(plan->split_k) * size_t(M) * size_t((N + 3) / 4 * 4) * sizeof(float), 256);
    }
    plan->ws_total = M > 0 ? off : 0;
    return FLE_OK;
}

}  // namespace fle

using namespace fle;

static void format_plan(const Plan &plan, char *buf, size_t n) {
    const char *dt = plan.op_dtype == FLE_F32 ? "f32" : plan.op_dtype == FLE_F16 ? "f16" : plan.op_dtype == FLE_F8E4M3 ? (plan.mx ? "f8mx" : "f8") : "bf16";
    snprintf(buf, n, "variant=%s_%s_%s%s%s tile=%dx%dx%d tiles=%lldx%lld split_k=%d row_op=%d np=%d staging=%s workspace=%zu%s",
             plan.variant == V_TILED ? (plan.groups ? "grouped_tiled" : "tiled") : plan.variant == V_SKINNY ? "skinny" : plan.variant == V_THIN ? "thin" : "general", dt,
             plan.variant == V_THIN && plan.bm == 8 ? "dot" : "mfma",
             plan.edge ? "+edge" : "", plan.w_stream ? "+wstream" : "", plan.bm, plan.bn, plan.bk, (long long)plan.tiles_m, (long long)plan.tiles_n, plan.split_k, plan.epi.row_kind,
             plan.np, plan.staging == ST_OUT ? "out" : plan.staging == ST_WS ? "workspace_f32" : "none", plan.ws_total,
             plan.ln_pre == LN_PRE_FUSED ? " ln_pre=fused" : plan.ln_pre == LN_PRE_PASS ? " ln_pre=pass" : "");
}

static fle_status check_workspace(const fle_problem *p, const Plan &plan) {
    if (plan.ws_total == 0) return FLE_OK;
    if (!p->workspace) return fail(FLE_ERR_WORKSPACE, "workspace is NULL but %zu bytes are needed", plan.ws_total);
    if (p->workspace_bytes < plan.ws_total) return fail(FLE_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", p->workspace_bytes, plan.ws_total);
    if (reinterpret_cast<uintptr_t>(p->workspace) % 256 != 0) return fail(FLE_ERR_ALIGN, "workspace must be 256-byte aligned");
    return FLE_OK;
}

// ------------------------------------------------------------------ attention
// Elements spanned by B sequences of T tokens of HD elements with token stride ld and sequence stride sb,
// or 0 if the two strides make tokens of different sequences collide.
static int64_t attention_extent(int64_t B, int64_t T, int64_t HD, int64_t ld, int64_t sb) {
    const bool seq_major = sb >= (T - 1) * ld + HD, token_major = sb >= HD && ld >= (B - 1) * sb + HD;
    if (B > 1 && !seq_major && !token_major) return 0;
    return (B - 1) * sb + (T - 1) * ld + HD;
}

static fle_status check_attention(const fle_attention *p) {
    if (!p) return fail(FLE_ERR_NULL, "attention problem is NULL");
    if (p->dtype != FLE_BF16 && p->dtype != FLE_F16) return fail(FLE_ERR_UNSUPPORTED, "attention takes FLE_BF16 or FLE_F16 (got dtype %d)", p->dtype);
    if (p->B < 0 || p->H < 1 || p->T < 1 || p->Tk < 0) return fail(FLE_ERR_SHAPE, "need B >= 0, H >= 1, T >= 1, Tk >= 0 (got %lld, %lld, %lld, %lld)", (long long)p->B, (long long)p->H, (long long)p->T, (long long)p->Tk);
    if (p->D != 32 && p->D != 64 && p->D != 128 && p->D != 256) return fail(FLE_ERR_UNSUPPORTED, "head dimension %lld is not 32, 64, 128 or 256", (long long)p->D);
    if (p->causal < 0) return fail(FLE_ERR_OP, "causal must be 0, 1 or a group size (got %d)", p->causal);
    if (p->B > 65535 || p->H > 65535) return fail(FLE_ERR_SHAPE, "B and H are limited to 65535");
    const int64_t Tk = p->Tk > 0 ? p->Tk : p->T;
    if (p->T > (int64_t(1) << 24) || Tk > (int64_t(1) << 24)) return fail(FLE_ERR_SHAPE, "T and Tk are limited to 2^24");
    if (p->causal && Tk < p->T) return fail(FLE_ERR_SHAPE, "a causal mask needs Tk >= T (got Tk = %lld, T = %lld)", (long long)Tk, (long long)p->T);
    if ((p->T + 127) / 128 * p->H * p->B >= (int64_t(1) << 31)) return fail(FLE_ERR_SHAPE, "B * H * T / 128 is limited to 2^31 workgroups");
    const int64_t HD = p->H * p->D;
    const int64_t kLimit = int64_t(1) << 40;
    if (p->ldq < HD || p->ldk < HD || p->ldv < HD || p->ldo < HD) return fail(FLE_ERR_SHAPE, "a token stride is smaller than H*D = %lld", (long long)HD);
    if (p->ldq > kLimit || p->ldk > kLimit || p->ldv > kLimit || p->ldo > kLimit) return fail(FLE_ERR_SHAPE, "token stride too large");
    if (p->sbq < 0 || p->sbk < 0 || p->sbv < 0 || p->sbo < 0 || p->sbq > kLimit || p->sbk > kLimit || p->sbv > kLimit || p->sbo > kLimit)
        return fail(FLE_ERR_SHAPE, "sequence strides must be >= 0 (0 = packed)");
    // the kernel addresses the Q, K and V of one sequence with 32-bit byte offsets
    if ((p->T + 256) * p->ldq * 2 >= (int64_t(1) << 31) || (Tk + 64) * (p->ldk > p->ldv ? p->ldk : p->ldv) * 2 >= (int64_t(1) << 31))
        return fail(FLE_ERR_SHAPE, "one sequence's Q, K or V spans 2 GiB or more");
    if (!(p->scale >= 0.0f) || std::isinf(p->scale)) return fail(FLE_ERR_OP, "scale must be finite and > 0 (or 0 for 1/sqrt(D))");
    if (p->B == 0) return FLE_OK;
    if (!p->q || !p->k || !p->v || !p->o) return fail(FLE_ERR_NULL, "q, k, v or o is NULL");
    if (!aligned(p->q, 16) || !aligned(p->k, 16) || !aligned(p->v, 16)) return fail(FLE_ERR_ALIGN, "q, k and v must be 16-byte aligned");
    if (p->ldq % 8 || p->ldk % 8 || p->ldv % 8 || p->sbq % 8 || p->sbk % 8 || p->sbv % 8) return fail(FLE_ERR_ALIGN, "the strides of q, k and v must be multiples of 8 elements");
    if (!aligned(p->o, 8) || p->ldo % 4 || p->sbo % 4) return fail(FLE_ERR_ALIGN, "o must be 8-byte aligned and its strides multiples of 4 elements");
    const int64_t eq = attention_extent(p->B, p->T, HD, p->ldq, p->sbq > 0 ? p->sbq : p->T * p->ldq);
    const int64_t ek = attention_extent(p->B, Tk, HD, p->ldk, p->sbk > 0 ? p->sbk : Tk * p->ldk);
    const int64_t ev = attention_extent(p->B, Tk, HD, p->ldv, p->sbv > 0 ? p->sbv : Tk * p->ldv);
    const int64_t eo = attention_extent(p->B, p->T, HD, p->ldo, p->sbo > 0 ? p->sbo : p->T * p->ldo);
    if (!eq || !ek || !ev || !eo) return fail(FLE_ERR_SHAPE, "token and sequence strides make sequences collide");
    const size_t no = size_t(eo) * 2;
    if (overlaps(p->o, no, p->q, size_t(eq) * 2) || overlaps(p->o, no, p->k, size_t(ek) * 2) || overlaps(p->o, no, p->v, size_t(ev) * 2))
        return fail(FLE_ERR_UNSUPPORTED, "o overlaps q, k or v");
    return FLE_OK;
}

// The three stages of an attention block and where their intermediates sit in the workspace.
struct BlockParts {
    fle_problem proj, outp;
    fle_attention att;
    fle_op proj_ops[1], out_ops[2];
    Plan proj_plan, out_plan;
    size_t qkv_off, a_off, sub_off, total;
};

static fle_status plan_block(const fle_attention_block *p, BlockParts *bp) {
    if (!p) return fail(FLE_ERR_NULL, "attention block is NULL");
    if (p->dtype != FLE_BF16 && p->dtype != FLE_F16) return fail(FLE_ERR_UNSUPPORTED, "attention takes FLE_BF16 or FLE_F16 (got dtype %d)", p->dtype);
    if (p->B < 0 || p->T < 1 || p->C < 1 || p->H < 1) return fail(FLE_ERR_SHAPE, "need B >= 0, T >= 1, C >= 1, H >= 1");
    if (p->B > 65535 || p->T > (int64_t(1) << 24) || p->C > (int64_t(1) << 24)) return fail(FLE_ERR_SHAPE, "size too large");
    if (p->C % p->H) return fail(FLE_ERR_SHAPE, "C = %lld is not a multiple of H = %lld", (long long)p->C, (long long)p->H);
    const int64_t D = p->C / p->H, rows = p->B * p->T, C = p->C;
    std::memset(bp, 0, sizeof *bp);
    bp->qkv_off = 0;
    bp->a_off = round_up(size_t(rows) * size_t(3 * C) * 2, 256);
    bp->sub_off = bp->a_off + round_up(size_t(rows) * size_t(C) * 2, 256);
    char *ws = reinterpret_cast<char *>(p->workspace);
    char *qkv = ws ? ws + bp->qkv_off : nullptr, *a = ws ? ws + bp->a_off : nullptr;

    fle_problem &pj = bp->proj;
    pj.M = rows; pj.N = 3 * C; pj.K = C; pj.dtype = p->dtype;
    pj.x = p->x; pj.ldx = C; pj.w = p->w_qkv; pj.ldw = C; pj.b = p->b_qkv;
    pj.out = qkv;
    pj.ldo = 3 * C;
    if (p->b_qkv) { bp->proj_ops[0].kind = FLE_BIAS; pj.n_ops = 1; }
    pj.ops = bp->proj_ops;
    pj.stream = p->stream;

    fle_attention &at = bp->att;
    at.dtype = p->dtype; at.causal = p->causal; at.B = p->B; at.H = p->H; at.T = p->T; at.D = D;
    at.q = qkv; at.k = qkv ? qkv + C * 2 : nullptr; at.v = qkv ? qkv + 2 * C * 2 : nullptr;
    at.ldq = at.ldk = at.ldv = 3 * C;
    at.o = a; at.ldo = C; at.scale = 0.0f; at.stream = p->stream;

    fle_problem &po = bp->outp;
    po.M = rows; po.N = C; po.K = C; po.dtype = p->dtype;
    po.x = a; po.ldx = C; po.w = p->w_o; po.ldw = C; po.b = p->b_o;
    po.out = p->out; po.ldo = C;
    int n = 0;
    if (p->b_o) bp->out_ops[n++].kind = FLE_BIAS;
    if (p->residual) { bp->out_ops[n].kind = FLE_RESIDUAL; bp->out_ops[n].p0 = p->residual; bp->out_ops[n].ld = C; ++n; }
    po.ops = bp->out_ops; po.n_ops = n;
    po.stream = p->stream;

    if (D != 32 && D != 64 && D != 128 && D != 256) return fail(FLE_ERR_UNSUPPORTED, "head dimension C / H = %lld is not 32, 64, 128 or 256", (long long)D);
    if (rows > 0 && (!p->x || !p->w_qkv || !p->w_o || !p->out)) return fail(FLE_ERR_NULL, "x, w_qkv, w_o or out is NULL");
    if (rows > 0) {
        // the output projection checks out against its own operands; the first stage's are checked here
        const size_t n_out = size_t(rows) * size_t(C) * 2;
        if (overlaps(p->out, n_out, p->w_qkv, size_t(3 * C) * size_t(C) * 2) || overlaps(p->out, n_out, p->b_qkv, size_t(3 * C) * 2))
            return fail(FLE_ERR_UNSUPPORTED, "out overlaps w_qkv or b_qkv");
        if (overlaps(p->out, n_out, p->x, n_out) && !(p->out == p->x && p->residual == p->x))
            return fail(FLE_ERR_UNSUPPORTED, "out overlaps x (allowed only when x is also the residual, exactly)");
    }
    fle_status s;
    if (ws) {
        s = make_plan(&pj, V_AUTO, 0, &bp->proj_plan);
        if (s == FLE_OK) s = check_attention(&at);
        if (s == FLE_OK) s = make_plan(&po, V_AUTO, 0, &bp->out_plan);
        if (s != FLE_OK) return s;
        if (rows > 0 && overlaps(p->out, size_t(rows) * size_t(C) * 2, ws, p->workspace_bytes)) return fail(FLE_ERR_UNSUPPORTED, "out overlaps the workspace");
    } else {
        // No workspace yet (validation, sizing): the intermediates get a stand-in address that is never
        // dereferenced; the plans of the two projections do not depend on where qkv and a will live.
        fle_problem t1 = pj, t2 = po;
        t1.out = reinterpret_cast<void *>(uintptr_t(256));
        t2.x = reinterpret_cast<const void *>(uintptr_t(256));
        s = make_plan(&t1, V_AUTO, 0, &bp->proj_plan);
        if (s == FLE_OK) s = make_plan(&t2, V_AUTO, 0, &bp->out_plan);
        if (s != FLE_OK) return s;
    }
    const size_t sub = bp->proj_plan.ws_total > bp->out_plan.ws_total ? bp->proj_plan.ws_total : bp->out_plan.ws_total;
    bp->total = bp->sub_off + round_up(sub, 256);
    pj.workspace = ws ? ws + bp->sub_off : nullptr; pj.workspace_bytes = round_up(sub, 256);
    po.workspace = pj.workspace; po.workspace_bytes = pj.workspace_bytes;
    return FLE_OK;
}

// ------------------------------------------------------------------ perceptron chain
static const size_t kChainSyncBytes = 2560;  // the barrier state at the start of the workspace: 20 lines of 128 bytes
static fle_status check_chain(const fle_chain *p, size_t *act_bytes) {
    if (!p) return fail(FLE_ERR_NULL, "chain is NULL");
    if (p->dtype != FLE_F32 && p->dtype != FLE_BF16 && p->dtype != FLE_F16) return fail(FLE_ERR_OP, "dtype %d is not FLE_F32, FLE_BF16 or FLE_F16", p->dtype);
    if (p->n_layers < 1 || p->n_layers > FLE_CHAIN_MAX_LAYERS) return fail(FLE_ERR_SHAPE, "n_layers %d outside 1..%d", p->n_layers, FLE_CHAIN_MAX_LAYERS);
    if (!p->layers || !p->x || !p->out) return fail(FLE_ERR_NULL, "layers, x or out is NULL");
    if (p->w_dtype != p->dtype && !(p->dtype == FLE_F32 && (p->w_dtype == FLE_BF16 || p->w_dtype == FLE_F16)))
        return fail(FLE_ERR_UNSUPPORTED, "w_dtype %d must equal dtype %d, or be a 2-byte dtype under FLE_F32", p->w_dtype, p->dtype);
    const size_t es = esize(p->dtype), ws_ = esize(p->w_dtype);
    if (!aligned(p->x, 16)) return fail(FLE_ERR_ALIGN, "x must be 16-byte aligned");
    int64_t widest = 0;
    for (int l = 0; l < p->n_layers; ++l) {
        const fle_chain_layer &L = p->layers[l];
        if (L.n < 1 || L.k < 1 || L.n > (int64_t(1) << 24) || L.k > (int64_t(1) << 24)) return fail(FLE_ERR_SHAPE, "layer %d: n and k must be in 1 .. 2^24", l);
        if (l > 0 && L.k != p->layers[l - 1].n) return fail(FLE_ERR_SHAPE, "layer %d takes %lld inputs but layer %d gives %lld", l, (long long)L.k, l - 1, (long long)p->layers[l - 1].n);
        if ((size_t(L.k) * ws_) % 16) return fail(FLE_ERR_ALIGN, "layer %d: a row of W must be a multiple of 16 bytes", l);
        if (!L.w) return fail(FLE_ERR_NULL, "layer %d: w is NULL", l);
        if (!aligned(L.w, 16)) return fail(FLE_ERR_ALIGN, "layer %d: w must be 16-byte aligned", l);
        if (L.act != -1 && L.act != FLE_RELU && L.act != FLE_GELU_ERF && L.act != FLE_GELU_TANH) return fail(FLE_ERR_OP, "layer %d: activation %d is not -1, RELU, GELU_ERF or GELU_TANH", l, L.act);
        if (overlaps(p->out, size_t(p->layers[p->n_layers - 1].n) * es, L.w, size_t(L.n) * size_t(L.k) * ws_)) return fail(FLE_ERR_UNSUPPORTED, "out overlaps the weights of layer %d", l);
        if (l + 1 < p->n_layers && L.n > widest) widest = L.n;
    }
    if (overlaps(p->out, size_t(p->layers[p->n_layers - 1].n) * es, p->x, size_t(p->layers[0].k) * es) && p->n_layers > 1)
        return fail(FLE_ERR_UNSUPPORTED, "out overlaps x");
    *act_bytes = round_up(size_t(widest) * es, 256);
    return FLE_OK;
}

extern "C" {

fle_status fle_validate(const fle_problem *p) {
    Plan plan;
    return make_plan(p, g_forced, g_split, &plan);
}

fle_status fle_workspace_size(const fle_problem *p, size_t *bytes_out) {
    if (!bytes_out) return fail(FLE_ERR_NULL, "bytes_out is NULL");
    Plan plan;
    fle_status s = make_plan(p, g_forced, g_split, &plan);
    if (s != FLE_OK) return s;
    *bytes_out = plan.ws_total;
    g_plan = plan;
    g_have_plan = true;
    return FLE_OK;
}

fle_status fle_run(const fle_problem *p) {
    Plan plan;
    fle_status s = make_plan(p, g_forced, g_split, &plan);
    if (s != FLE_OK) return s;
    if (p->M == 0) return FLE_OK;
    s = check_workspace(p, plan);
    if (s == FLE_OK) s = launch(p, plan);
    if (s == FLE_OK) {
        g_plan = plan;
        g_have_plan = true;
    }
    return s;
}

// A plan choice is valid when it names a variant the force knob knows and a split in 0 .. 64.
static fle_status check_choice(const fle_plan_choice *c) {
    if (!c) return fail(FLE_ERR_NULL, "plan choice is NULL");
    if (c->variant < V_AUTO || c->variant > V_THIN) return fail(FLE_ERR_OP, "plan choice: unknown variant %d", c->variant);
    if (c->split < 0 || c->split > 64) return fail(FLE_ERR_OP, "plan choice: split %d outside 0..64", c->split);
    return FLE_OK;
}

fle_status fle_workspace_size_with(const fle_problem *p, const fle_plan_choice *c, size_t *bytes_out) {
    if (!bytes_out) return fail(FLE_ERR_NULL, "bytes_out is NULL");
    fle_status s = check_choice(c);
    if (s != FLE_OK) return s;
    Plan plan;
    s = make_plan(p, c->variant, c->split, &plan);
    if (s != FLE_OK) return s;
    *bytes_out = plan.ws_total;
    g_plan = plan;
    g_have_plan = true;
    return FLE_OK;
}

fle_status fle_run_with(const fle_problem *p, const fle_plan_choice *c) {
    fle_status s = check_choice(c);
    if (s != FLE_OK) return s;
    Plan plan;
    s = make_plan(p, c->variant, c->split, &plan);
    if (s != FLE_OK) return s;
    if (p->M == 0) return FLE_OK;
    s = check_workspace(p, plan);
    if (s == FLE_OK) s = launch(p, plan);
    if (s == FLE_OK) {
        g_plan = plan;
        g_have_plan = true;
    }
    return s;
}

fle_status fle_run_static(const fle_problem *p) {
    if (!p) return fail(FLE_ERR_NULL, "problem is NULL");
    fle_problem q = *p;
    q.workspace = nullptr;  // the caller's workspace fields are ignored
    q.workspace_bytes = 0;
    Plan plan;
    fle_status s = make_plan(&q, g_forced, g_split, &plan);
    if (s != FLE_OK) return s;
    if (q.M == 0) return FLE_OK;
    if (plan.ws_total > size_t(FLE_STATIC_SCRATCH_BYTES))
        return fail(FLE_ERR_WORKSPACE, "this problem needs %zu bytes of scratch, the static array holds %zu: use fle_run with a workspace", plan.ws_total,
                    size_t(FLE_STATIC_SCRATCH_BYTES));
    if (plan.ws_total > 0) {
        void *ptr = nullptr;
        s = static_scratch(&ptr);
        if (s != FLE_OK) return s;
        q.workspace = ptr;
        q.workspace_bytes = size_t(FLE_STATIC_SCRATCH_BYTES);
        s = make_plan(&q, g_forced, g_split, &plan);  // again with the scratch in place: no operand may reach into it
        if (s == FLE_OK) s = check_workspace(&q, plan);
        if (s != FLE_OK) return s;
    }
    s = launch(&q, plan);
    if (s == FLE_OK) {
        g_plan = plan;
        g_have_plan = true;
    }
    return s;
}

static fle_status check_groups(const fle_groups *g) { return g ? FLE_OK : fail(FLE_ERR_NULL, "groups is NULL"); }

fle_status fle_validate_grouped(const fle_problem *p, const fle_groups *g) {
    Plan plan;
    fle_status s = check_groups(g);
    return s != FLE_OK ? s : make_plan(p, g_forced, g_split, &plan, g);
}

fle_status fle_workspace_size_grouped(const fle_problem *p, const fle_groups *g, size_t *bytes_out) {
    if (!bytes_out) return fail(FLE_ERR_NULL, "bytes_out is NULL");
    Plan plan;
    fle_status s = check_groups(g);
    if (s == FLE_OK) s = make_plan(p, g_forced, g_split, &plan, g);
    if (s != FLE_OK) return s;
    *bytes_out = plan.ws_total;
    g_plan = plan;
    g_have_plan = true;
    return FLE_OK;
}

fle_status fle_run_grouped(const fle_problem *p, const fle_groups *g) {
    Plan plan;
    fle_status s = check_groups(g);
    if (s == FLE_OK) s = make_plan(p, g_forced, g_split, &plan, g);
    if (s != FLE_OK) return s;
    if (p->M == 0) return FLE_OK;
    s = check_workspace(p, plan);
    if (s == FLE_OK) s = launch(p, plan, g);
    if (s == FLE_OK) {
        g_plan = plan;
        g_have_plan = true;
    }
    return s;
}

fle_status fle_attention_validate(const fle_attention *p) { return check_attention(p); }

fle_status fle_attention_run(const fle_attention *p) {
    fle_status s = check_attention(p);
    if (s != FLE_OK || p->B == 0) return s;
    return launch_attention(p);
}

fle_status fle_attention_block_validate(const fle_attention_block *p) {
    BlockParts bp;
    if (!p) return fail(FLE_ERR_NULL, "attention block is NULL");
    fle_attention_block t = *p;
    t.workspace = nullptr;  // validation does not look at the workspace
    return plan_block(&t, &bp);
}

fle_status fle_attention_block_workspace_size(const fle_attention_block *p, size_t *bytes_out) {
    if (!bytes_out) return fail(FLE_ERR_NULL, "bytes_out is NULL");
    if (!p) return fail(FLE_ERR_NULL, "attention block is NULL");
    BlockParts bp;
    fle_attention_block t = *p;
    t.workspace = nullptr;
    fle_status s = plan_block(&t, &bp);
    if (s == FLE_OK) *bytes_out = bp.total;
    return s;
}

fle_status fle_attention_block_run(const fle_attention_block *p) {
    BlockParts bp;
    if (!p) return fail(FLE_ERR_NULL, "attention block is NULL");
    {
        fle_attention_block t = *p;
        t.workspace = nullptr;
        fle_status s = plan_block(&t, &bp);
        if (s != FLE_OK) return s;
    }
    if (p->B == 0) return FLE_OK;
    if (!p->workspace) return fail(FLE_ERR_WORKSPACE, "workspace is NULL but %zu bytes are needed", bp.total);
    if (p->workspace_bytes < bp.total) return fail(FLE_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", p->workspace_bytes, bp.total);
    if (reinterpret_cast<uintptr_t>(p->workspace) % 256 != 0) return fail(FLE_ERR_ALIGN, "workspace must be 256-byte aligned");
    fle_status s = plan_block(p, &bp);
    if (s != FLE_OK) return s;
    s = check_workspace(&bp.proj, bp.proj_plan);
    if (s == FLE_OK) s = check_workspace(&bp.outp, bp.out_plan);
    if (s == FLE_OK) s = launch(&bp.proj, bp.proj_plan);
    if (s == FLE_OK) s = launch_attention(&bp.att);
    if (s == FLE_OK) s = launch(&bp.outp, bp.out_plan);
    if (s == FLE_OK) {
        g_plan = bp.out_plan;
        g_have_plan = true;
    }
    return s;
}

fle_status fle_chain_validate(const fle_chain *p) {
    size_t act = 0;
    return check_chain(p, &act);
}

fle_status fle_chain_workspace_size(const fle_chain *p, size_t *bytes_out) {
    if (!bytes_out) return fail(FLE_ERR_NULL, "bytes_out is NULL");
    size_t act = 0;
    fle_status s = check_chain(p, &act);
    if (s == FLE_OK) *bytes_out = kChainSyncBytes + size_t(p->n_layers - 1) * act;
    return s;
}

fle_status fle_chain_run(const fle_chain *p) {
    size_t act = 0;
    fle_status s = check_chain(p, &act);
    if (s != FLE_OK) return s;
    char *ws = reinterpret_cast<char *>(p->workspace);
    const size_t need = kChainSyncBytes + size_t(p->n_layers - 1) * act;
    if (!ws) return fail(FLE_ERR_WORKSPACE, "workspace is NULL but %zu bytes are needed", need);
    if (p->workspace_bytes < need) return fail(FLE_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", p->workspace_bytes, need);
    if (reinterpret_cast<uintptr_t>(ws) % 256 != 0) return fail(FLE_ERR_ALIGN, "workspace must be 256-byte aligned");
    const size_t es = esize(p->dtype);
    if (overlaps(ws, need, p->x, size_t(p->layers[0].k) * es) || overlaps(ws, need, p->out, size_t(p->layers[p->n_layers - 1].n) * es))
        return fail(FLE_ERR_UNSUPPORTED, "the workspace overlaps x or out");
    return launch_chain(p, ws, ws + kChainSyncBytes, act);
}

const char *fle_status_string(fle_status s) {
    switch (s) {
    case FLE_OK: return "ok";
    case FLE_ERR_NULL: return "required pointer is NULL";
    case FLE_ERR_SHAPE: return "invalid shape or leading dimension";
    case FLE_ERR_ALIGN: return "misaligned pointer or leading dimension";
    case FLE_ERR_OP: return "invalid epilogue op";
    case FLE_ERR_UNSUPPORTED: return "unsupported combination";
    case FLE_ERR_WORKSPACE: return "workspace missing or too small";
    case FLE_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}

const char *fle_last_error(void) { return g_error; }

fle_status fle_last_plan(char *buf, size_t n) {
    if (!buf || n == 0) return fail(FLE_ERR_NULL, "buf is NULL or empty");
    if (g_have_plan) format_plan(g_plan, buf, n);
    else buf[0] = 0;
    return FLE_OK;
}

void fle_force_variant(int variant) { g_forced = variant; }

void fle_force_split(int split) { g_split = split < 0 ? 0 : split; }

int fle_version(void) { return 900; }  // 0.9.0: fp8 operands, two row reductions, per-call plan choice (0.8.0: fle_run_static; 0.7.0: store op; 0.6.0: perceptron chain; 0.5.0: attention; 0.4.0: thin kernels; 0.3.0: grouped problems)

}  // extern "C"
