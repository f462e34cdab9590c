/*
 * fle.h -- C ABI of libfle: fused linear + epilogue for AMD MI355X (gfx950).
 *
 *     out = epilogue( x[M,K] * W[N,K]^T )
 *
 * The operator is the fusion pattern that arXiv 2511.16964 reports as a
 * recurring source of speedup over PyTorch eager (Section 5.3: fusing a
 * matmul with the elementwise and reduction ops that follow it into one
 * kernel removes the intermediate tensors' memory traffic and the extra
 * launches).  The epilogue is an ordered list drawn from
 * {bias, scale, ReLU, GELU-erf, GELU-tanh, residual add, LayerNorm over N,
 * row softmax, row logsumexp}; each op has PyTorch-eager semantics, and the
 * result equals the unfused composition up to floating-point rounding (the
 * comparison the paper's evaluator makes, Appendix A).
 *
 * Conventions
 *   - All tensors are row-major.  W is [N,K] (the nn.Linear weight layout).
 *   - One dtype per problem for x, W, b, residual, gamma, beta and out:
 *     FLE_F32, FLE_BF16 or FLE_F16 (FLE_F8E4M3: x and W in fp8, the rest in bf16).
 *     Products are accumulated in fp32, the whole epilogue runs in fp32, and the
 *     result is rounded once (round-to-nearest-even) to the output dtype.
 *   - Pointers inside fle_problem and fle_op are DEVICE pointers unless
 *     stated otherwise; the structs themselves and the ops array live on the
 *     HOST and are only read during the call.
 *   - The caller owns every buffer; the library allocates, frees and keeps
 *     nothing on the device.  Buffers must stay valid until the work
 *     enqueued on `stream` has completed.
 *   - No function throws or aborts; errors come back as fle_status and a
 *     thread-local message (fle_last_error).  On any error nothing has been
 *     enqueued.
 *   - Results are bitwise reproducible for a given problem: no floating-point
 *     atomics, fixed reduction order.
 */
#ifndef FLE_H
#define FLE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FLE_OK = 0,
    FLE_ERR_NULL = 1,        /* a required pointer is NULL                               */
    FLE_ERR_SHAPE = 2,       /* negative size, leading dimension too small, size overflow */
    FLE_ERR_ALIGN = 3,       /* a pointer or leading dimension breaks the alignment rule */
    FLE_ERR_OP = 4,          /* unknown op kind, bad op argument, too many ops           */
    FLE_ERR_UNSUPPORTED = 5, /* valid math, but outside the accepted epilogue grammar    */
    FLE_ERR_WORKSPACE = 6,   /* workspace missing or smaller than fle_workspace_size     */
    FLE_ERR_HIP = 7          /* the HIP runtime refused a launch                         */
} fle_status;

typedef enum {
    FLE_F32 = 0,
    FLE_BF16 = 1,
    FLE_F16 = 2,
    FLE_F8E4M3 = 3 /* x and W in OCP 8-bit floating point (e4m3: 4 exponent bits, 3 mantissa bits, no infinities, the
                      torch.float8_e4m3fn encoding); b, residual and store operands, gamma, beta and out in bf16.
                      Products of the stored values are accumulated in fp32 exactly as for the wider dtypes, on
                      the fp8 matrix instructions (twice the bf16 rate, half the bytes per operand element): the
                      precision reduction that the paper's analysis names as its most effective single pattern
                      (Section 5.3) and that its tolerance admits (Appendix A).  Per-tensor scale factors of x
                      and W are applied by listing FLE_SCALE with their product as the first op.  fp8 problems
                      run on the tiled kernels only: x and W 16-byte aligned, K and the row strides multiples of
                      16 elements; otherwise FLE_ERR_UNSUPPORTED.                                             */
} fle_dtype;

typedef enum {
    FLE_BIAS = 0,      /* v += b[n]                                  (needs problem.b)     */
    FLE_SCALE = 1,     /* v *= alpha                                                        */
    FLE_RELU = 2,      /* v = max(v, 0); NaN stays NaN                                      */
    FLE_GELU_ERF = 3,  /* v = 0.5 v (1 + erf(v / sqrt 2))            (approximate='none')  */
    FLE_GELU_TANH = 4, /* v = 0.5 v (1 + tanh(sqrt(2/pi) (v + 0.044715 v^3)))               */
    FLE_RESIDUAL = 5,  /* v += r[m,n]                                (p0 = r, ld)          */
    FLE_LAYERNORM = 6, /* over n: (v - mean) / sqrt(biased var + alpha) * gamma[n] + beta[n];
                          p0 = gamma or NULL (1), p1 = beta or NULL (0), alpha = eps        */
    FLE_SOFTMAX = 7,   /* over n: exp(v - max) / sum exp(v - max)                           */
    FLE_LOGSUMEXP = 8, /* over n: max + log sum exp(v - max); out becomes [M]; last op only */
    FLE_MXSCALE = 10,  /* not an epilogue step: says that the FLE_F8E4M3 operands are block-scaled (OCP microscaling,
                          MXFP8): every 32 consecutive k of a row of x and of W share a power-of-two scale, stored
                          as one byte e (E8M0: the scale is 2^(e - 127); e = 255 marks NaN).  p0 = scales of x,
                          device [M][K/32] bytes, p1 = scales of W, device [N][K/32] bytes, rows contiguous, both
                          4-byte aligned.  out = epilogue( (x * scale_x) (W * scale_W)^T ), with the products formed
                          and summed on the matrix instruction's block-scaled form.  First entry of the list only;
                          K a multiple of 128; plain problems only (fle_run*, not the grouped form).  This is the
                          finer-grained of the reduced-precision formats the paper's tolerance admits (Section 5.3,
                          Appendix A); per-tensor scales need no such entry (FLE_SCALE).                       */
    FLE_LAYERNORM_PRE = 11, /* not an epilogue step: LayerNorm over K of every row of x in front of the multiplication,
                          out = epilogue( LN(x) W^T ) with LN(x)[m,k] = (x[m,k] - mean_m) / sqrt(biased var_m + alpha)
                          * gamma[k] + beta[k]; p0 = gamma[K] or NULL (1), p1 = beta[K] or NULL (0), alpha = eps
                          (the normalisation -> projection pairs of a transformer block, Section 5.3).  First entry
                          of the list only; FLE_F32, FLE_BF16 and FLE_F16; plain problems only.  For up to 4 rows of
                          x on the dot-product kernel the statistics and the normalisation are part of
                          that kernel's one sweep over W: one launch in place of two, where launches are most of
                          the time.  Every other shape gets a pass that writes LN(x), rounded to the dtype as the
                          unfused composition rounds it, into M * K more elements of workspace, which the usual
                          kernels then read (inside the K loop of a compute-bound kernel the normalisation costs
                          more than that pass).                                                                */
    FLE_STORE = 9      /* t[m,n] = v, rounded to the dtype; v itself goes on unchanged (p0 = t, ld).
                          Allowed before the row op (or anywhere in a list without one).  It is how
                          one call hands over both a value and its normalisation, e.g. bias, residual,
                          STORE, LAYERNORM gives x + f(x) in t and its LayerNorm in out: what a
                          pre-norm transformer layer needs from the call that ends the previous block */
} fle_op_kind;

#define FLE_MAX_OPS 8

typedef struct {
    int32_t kind;   /* fle_op_kind */
    float alpha;    /* SCALE: factor.  LAYERNORM, LAYERNORM_PRE: eps.  Otherwise ignored.  */
    const void *p0; /* RESIDUAL: r[M,N] (device).  LAYERNORM: gamma[N] (device) or NULL.
                       STORE: t[M,N] (device, written; must not overlap any other operand).
                       MXSCALE: block scales of x (device).  LAYERNORM_PRE: gamma[K] or NULL */
    const void *p1; /* LAYERNORM: beta[N] (device) or NULL.  MXSCALE: block scales of W.
                       LAYERNORM_PRE: beta[K] (device) or NULL                              */
    int64_t ld;     /* RESIDUAL / STORE: row stride of r / t in elements (>= N).           */
} fle_op;

typedef struct {
    int64_t M, N, K;        /* M >= 0, N >= 1, K >= 0.  M == 0 is a valid no-op.           */
    int32_t dtype;          /* fle_dtype                                                    */
    const void *x;          /* device [M,K], row stride ldx >= K elements                   */
    int64_t ldx;
    const void *w;          /* device [N,K], row stride ldw >= K elements                   */
    int64_t ldw;
    const void *b;          /* device [N], or NULL when no FLE_BIAS op is listed            */
    void *out;              /* device [M,N] with row stride ldo >= N, or [M] contiguous
                               (ldo ignored) when the list ends in FLE_LOGSUMEXP            */
    int64_t ldo;
    const fle_op *ops;      /* host array of n_ops entries, applied in order                */
    int32_t n_ops;          /* 0 .. FLE_MAX_OPS                                             */
    void *workspace;        /* device scratch of at least fle_workspace_size() bytes,
                               256-byte aligned; may be NULL when that size is 0.  Its
                               contents are undefined afterwards; it needs no clearing.     */
    size_t workspace_bytes;
    void *stream;           /* hipStream_t (NULL = the default stream)                      */
} fle_problem;

/*
 * Accepted epilogue grammar:   [ MXSCALE | LAYERNORM_PRE ]  elementwise*  [ rowop  elementwise*  [ rowop  elementwise* ] ]
 * with rowop = LAYERNORM | SOFTMAX | LOGSUMEXP and elementwise = BIAS | SCALE | RELU | GELU_ERF |
 * GELU_TANH | RESIDUAL | STORE (STORE only before the first row op); nothing follows LOGSUMEXP.  A
 * list with two row ops (e.g. LAYERNORM, SOFTMAX: a normalised layer's class probabilities) costs
 * M * N * 4 more workspace bytes and a third pass over the rows; the values between the two
 * reductions stay in fp32.  A third row op gives FLE_ERR_UNSUPPORTED, as does a second one in a
 * grouped problem.
 *
 * Alignment rule: no alignment is required for correctness.  The fast kernels (tiled MFMA
 * kernels for every dtype; the skinny and thin kernels that stream W for up to 256, 32 or 8
 * rows of x) are taken when x and W are 16-byte aligned and K and their row strides are
 * multiples of 16 bytes (8 bf16 or fp16 / 4 fp32 elements); N, out, b and the residual may then be
 * ragged or misaligned (the kernel switches to an element-wise epilogue).  Other problems
 * run on a slower general kernel.  Problems with few output tiles and a long K are split
 * along K over several workgroups; the partial sums go through the workspace and are added
 * in a fixed order, so the result stays reproducible.
 * `out` may alias a residual operand only exactly (same pointer and stride); it must not
 * overlap x, W, b, gamma, beta or the workspace.
 */

/* Host only (no HIP call).  Checks everything fle_run checks except the workspace size. */
fle_status fle_validate(const fle_problem *p);

/* Host only.  Bytes of device scratch fle_run needs for this problem (0 for purely
 * elementwise epilogues unless K is split). */
fle_status fle_workspace_size(const fle_problem *p, size_t *bytes_out);

/* Validates, then enqueues one to three kernels on p->stream and returns without
 * synchronising.  Never allocates or frees device memory. */
fle_status fle_run(const fle_problem *p);

/*
 * The plan (kernel family, tile, split of K) that fle_run derives from a cost model can also be given by the
 * caller, per call and without any state in the library: this is how a table made by an offline tuning run is
 * applied (the paper credits autotuned tile choices for many of its best solutions, Section 5.2 and the appendix
 * on outlier tasks; the package's autotune module measures every candidate plan of a list of shapes on the GPU at
 * hand and writes such a table).  variant and split mean what fle_force_variant and fle_force_split document
 * (0 = the library's own choice for that part).  c NULL gives FLE_ERR_NULL, values outside the ranges below
 * FLE_ERR_OP, a choice that cannot run the problem FLE_ERR_UNSUPPORTED; nothing is enqueued then.  The thread's
 * fle_force_* knobs are not read.  Results do not depend on the plan beyond floating-point summation order.
 */
typedef struct {
    int32_t variant; /* 0 .. 9 as for fle_force_variant */
    int32_t split;   /* 0 = automatic, 1 = none, S > 1 = S workgroups per output tile (at most 64) */
} fle_plan_choice;
fle_status fle_workspace_size_with(const fle_problem *p, const fle_plan_choice *c, size_t *bytes_out);
fle_status fle_run_with(const fle_problem *p, const fle_plan_choice *c);

/*
 * fle_run for callers that cannot allocate device memory or cannot bring a workspace: code inside a HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  p->workspace and
 * p->workspace_bytes are ignored; the scratch that fle_run takes from the workspace (row-reduction
 * partials, fp32 staging, split-K slabs) lives instead in a static device array of
 * FLE_STATIC_SCRATCH_BYTES that is part of the library's code object (every GPU the library runs on
 * holds its own copy until the process ends).  The call allocates and frees nothing and never
 * synchronises; its first call on a device looks the array's address up once
 * (hipGetSymbolAddress), so make that first call outside a graph capture.
 * A problem whose fle_workspace_size exceeds FLE_STATIC_SCRATCH_BYTES is refused with
 * FLE_ERR_WORKSPACE and nothing is enqueued.  Results are bit-identical to fle_run's.
 * Every call on one GPU shares that GPU's array: calls that overlap in time on one GPU (different
 * streams, different threads) race on it and must be serialised by the caller.  Nothing in the array has
 * to start at zero, and a call leaves its contents undefined.
 */
#define FLE_STATIC_SCRATCH_BYTES (16u << 20)
fle_status fle_run_static(const fle_problem *p);

/*
 * Grouped form: the rows of x are cut into G consecutive groups and group g is multiplied by its
 * own weight matrix W_g (and gets its own bias b_g), all in one launch.  This is the layout of a
 * mixture-of-experts layer after the tokens have been sorted by expert; the paper's appendix on
 * outlier tasks (Level 5, the mixture-of-experts task) reports that replacing the loop over experts
 * by one grouped matrix multiplication over packed expert weights is what gave its ~10x there.
 *
 *     out[m, :] = epilogue( x[m, :] * W_g^T ),   row_offsets[g] <= m < row_offsets[g+1]
 *
 * The fle_problem describes the stacked operands: M is the total number of rows, x / out / every
 * residual operand are [M, ...] as in the plain form, p->w points to W_0 and p->b to b_0.  The
 * epilogue (any list the plain form accepts) is the same for every group; LayerNorm's gamma / beta
 * are shared.
 */
typedef struct {
    int32_t n_groups;           /* G, 1 .. 65536                                                  */
    const int64_t *row_offsets; /* DEVICE array of G + 1 entries, non-decreasing, [0] = 0 and
                                   [G] = M; group g owns rows [g] .. [g+1] - 1 (possibly none).
                                   Read by the kernel only, so a routing kernel may still be
                                   writing it on the same stream when the call is made.  Entries
                                   are clamped to 0 .. M and to be non-decreasing before use, so a
                                   malformed array never causes an out-of-bounds access; rows that
                                   no group owns are left undefined in out.                       */
    int64_t w_group_stride;     /* elements from W_g to W_g+1 (N * ldw for packed weights); a
                                   multiple of 16 bytes                                           */
    int64_t b_group_stride;     /* elements from b_g to b_g+1 (0: one bias for all groups)        */
} fle_groups;

/* As fle_validate / fle_workspace_size / fle_run, for a grouped problem.  Grouped problems run on the
 * tiled MFMA kernels only: x and W must satisfy that path's 16-byte rule (see above), otherwise
 * FLE_ERR_UNSUPPORTED; K is never split.  The structs are read during the call only. */
fle_status fle_validate_grouped(const fle_problem *p, const fle_groups *g);
fle_status fle_workspace_size_grouped(const fle_problem *p, const fle_groups *g, size_t *bytes_out);
fle_status fle_run_grouped(const fle_problem *p, const fle_groups *g);

/*
 * Scaled dot-product attention, forward, with the causal mask applied on the fly:
 *
 *     o[b,t,h,:] = sum_j softmax_j( scale * q[b,t,h,:] . k[b,j,h,:] ) * v[b,j,h,:]      (j <= t when causal)
 *
 * The mask can also be causal over groups of G consecutive tokens: query t then sees every key of its own
 * and of earlier groups, j < (t / G + 1) * G -- the causal mask of a sequence made of frames or patches
 * whose tokens are not ordered among themselves.
 *
 * The paper's task-wise analysis (Section 5.3) and its appendix on Level 3-pike and Level 5 outliers
 * name a flash-attention kernel, fused with the input and output projections and masking causally
 * without a materialised mask, as the largest recurring speedup over eager PyTorch.  Operands are
 * token-major, the layout a fused QKV projection writes: element (b,t,h,d) of q is at
 * q[(b*T + t)*ldq + h*D + d], likewise k, v, o, so q, k and v may be the three column thirds of one
 * [B*T, 3*H*D] matrix (ldq = ldk = ldv = 3*H*D) and o is ready to be the x of the output projection.
 * The score matrix never reaches memory: one kernel walks the keys with a running maximum and sum
 * (fp32 statistics and accumulation; the probabilities are rounded to the storage dtype for the
 * second product, as the values are).
 */
typedef struct {
    int32_t dtype;         /* FLE_BF16 or FLE_F16                                                  */
    int32_t causal;        /* 0: every key; 1: query t sees keys 0 .. t; G > 1: keys below (t/G + 1)*G */
    int64_t B, H, T, D;    /* batch, heads, queries per sequence (>= 1), head dimension (32, 64, 128 or 256) */
    const void *q, *k, *v; /* DEVICE, 16-byte aligned                                               */
    int64_t ldq, ldk, ldv; /* elements between consecutive tokens, >= H*D, multiples of 8           */
    void *o;               /* DEVICE, 8-byte aligned; must not overlap q, k or v                    */
    int64_t ldo;           /* >= H*D, a multiple of 4                                               */
    float scale;           /* > 0, or 0 for 1/sqrt(D)                                               */
    void *stream;          /* hipStream_t (NULL = the default stream)                               */
    int64_t Tk;            /* keys per sequence, or 0 for T.  Under a mask the queries are the last
                              T of the Tk positions (query t stands at t + Tk - T; needs Tk >= T),
                              the case of keys kept from earlier calls                               */
    int64_t sbq, sbk, sbv, sbo; /* elements between consecutive sequences, or 0 for packed
                              sequences (T*ldq, Tk*ldk, Tk*ldv, T*ldo).  Same multiples as the token
                              strides.  Either the sequences follow each other (stride >= one
                              sequence's extent) or the tokens of all sequences interleave
                              (sequence-first layouts: token stride >= B sequence strides)           */
} fle_attention;

/* Host only (no HIP call): checks everything fle_attention_run checks. */
fle_status fle_attention_validate(const fle_attention *p);

/* Validates, then enqueues one kernel on p->stream and returns without synchronising.  Needs no
 * workspace and never allocates.  B == 0 is a valid no-op. */
fle_status fle_attention_run(const fle_attention *p);

/*
 * A whole self-attention block in three launches that share no host synchronisation:
 *
 *     qkv = x w_qkv^T + b_qkv          [B*T, 3C]   (fused linear, columns are q | k | v, each H heads of D = C/H)
 *     a   = attention(q, k, v)         [B*T, C]    (fle_attention_run reading the thirds of qkv in place)
 *     out = a w_o^T + b_o (+ residual) [B*T, C]    (fused linear with its epilogue)
 *
 * All operands are row-major and packed (row strides C, 3C as above); qkv and a live in the workspace.
 */
typedef struct {
    int32_t dtype;        /* FLE_BF16 or FLE_F16                                          */
    int32_t causal;       /* as fle_attention.causal                                      */
    int64_t B, T, C, H;   /* C = H * D with D = 32, 64, 128 or 256                        */
    const void *x;        /* DEVICE [B*T, C]                                              */
    const void *w_qkv;    /* DEVICE [3C, C]                                               */
    const void *b_qkv;    /* DEVICE [3C] or NULL                                          */
    const void *w_o;      /* DEVICE [C, C]                                                */
    const void *b_o;      /* DEVICE [C] or NULL                                           */
    const void *residual; /* DEVICE [B*T, C] or NULL; may be x                            */
    void *out;            /* DEVICE [B*T, C]; may alias residual exactly, nothing else    */
    void *workspace;      /* DEVICE, 256-byte aligned, fle_attention_block_workspace_size bytes */
    size_t workspace_bytes;
    void *stream;
} fle_attention_block;

fle_status fle_attention_block_validate(const fle_attention_block *p);
fle_status fle_attention_block_workspace_size(const fle_attention_block *p, size_t *bytes_out);
/* Enqueues the three stages on p->stream.  On an error from a later stage the earlier ones may
 * already be enqueued (they only write the workspace). */
fle_status fle_attention_block_run(const fle_attention_block *p);

/*
 * A whole perceptron at batch 1 in one persistent launch: a chain of layers
 *
 *     h_0 = x,   h_{l+1} = act_l( W_l h_l + b_l ),   out = h_L
 *
 * The paper's MLP tasks run at batch 1 on small layers, where launches and the refill of the memory
 * pipeline between dependent launches dominate (appendix on task refinement: such tasks were noisy
 * or dropped for being launch-bound), and its task-wise analysis names fusing a whole model into a
 * single kernel as a recurring winner.  One launch keeps at most one workgroup resident per CU,
 * separates the layers by a grid-wide barrier and requests the next layer's first weights before the
 * barrier.  Intermediate activations are rounded to the storage dtype, as separate calls would.
 * The barrier's waits are bounded: should the workgroups ever not be resident together (another
 * kernel holding CUs that never finishes), the call ends instead of hanging: the error word (see
 * workspace) becomes non-zero and every workgroup that gave up fills its share of out with NaN, so
 * such a call cannot be mistaken for a result.
 */
typedef struct {
    const void *w;  /* DEVICE [n, k] row-major and packed (row stride k), 16-byte aligned            */
    const void *b;  /* DEVICE [n] or NULL                                                            */
    int64_t n, k;   /* k inputs -> n outputs; k must equal the previous layer's n; a W row (k weights)
                       must be a multiple of 16 bytes (4 fp32 / 8 bf16 or fp16 weights)              */
    int32_t act;    /* -1: none, or FLE_RELU, FLE_GELU_ERF, FLE_GELU_TANH                            */
} fle_chain_layer;

#define FLE_CHAIN_MAX_LAYERS 16

typedef struct {
    int32_t dtype;                 /* FLE_F32, FLE_BF16 or FLE_F16: x, every b, the activations, out */
    int32_t n_layers;              /* 1 .. FLE_CHAIN_MAX_LAYERS                                      */
    const fle_chain_layer *layers; /* HOST array                                                     */
    const void *x;                 /* DEVICE [layers[0].k], 16-byte aligned                          */
    void *out;                     /* DEVICE [layers[n_layers-1].n]                                  */
    void *workspace;               /* DEVICE, 256-byte aligned, fle_chain_workspace_size bytes: 2560
                                      bytes of barrier state, then one activation buffer per layer boundary.
                                      The barrier state must be ZERO before the first call; every
                                      call leaves it zero, except the 32-bit error word at byte 256,
                                      which becomes 1 if a barrier wait ran out.  While that word is
                                      non-zero every call on this workspace gives up at its first wait
                                      (out becomes NaN): zero all 2560 bytes again before the next
                                      call.  Calls that share a workspace must not overlap in time   */
    size_t workspace_bytes;
    void *stream;
    int32_t w_dtype;               /* dtype of every W: equal to dtype, or FLE_BF16 / FLE_F16 under
                                      dtype = FLE_F32 (weights stored in reduced precision, everything
                                      else fp32: the kernel is bound by the weight bytes, and the
                                      paper's appendix on correctness notes that its 1e-2 tolerance
                                      admits such precision reduction)                               */
} fle_chain;

fle_status fle_chain_validate(const fle_chain *p);
fle_status fle_chain_workspace_size(const fle_chain *p, size_t *bytes_out);
/* Enqueues one kernel on p->stream.  Never allocates or synchronises. */
fle_status fle_chain_run(const fle_chain *p);

/* Static description of a status code. */
const char *fle_status_string(fle_status s);

/* Detail text of the calling thread's most recent failing call ("" if none). */
const char *fle_last_error(void);

/* Human-readable plan (kernel variant, tile, grid) of the calling thread's most recent
 * successful fle_run or fle_workspace_size (or their grouped forms), copied into buf (NUL-terminated,
 * truncated to n).  "tile=AxBxC" is rows of x, rows of W and the K step in elements; for the
 * dot-product thin kernel ("thin_*_dot") C is the number of W rows per wave instead. */
fle_status fle_last_plan(char *buf, size_t n);

/* The two calls below are knobs for tests and tuning, not part of the operator: they keep a setting per
 * calling thread (the only mutable state of the library besides the error text and the last plan) that
 * stays in force until it is set back to 0, so a product call path should never touch them.
 *
 * Force a kernel variant for the calling thread's next calls:
 * 0 = automatic, 1 = general kernel, 2 = tiled MFMA kernel (automatic tile), 3 = skinny kernel
 * (bf16 / fp16, M <= 256) with a K step of 64, 4 = tiled with the 256x256 tile, 5 = tiled with
 * the 128x128 tile, 6 / 7 = skinny kernel with a K step of 128 / 256, 8 = skinny kernel with one
 * row block of up to 256 rows whose 32-row sub-blocks take turns on a 256-wide K step, 9 = thin kernel
 * (M <= 32: 16-row W tiles streamed without LDS staging, every dtype).
 * A forced variant that cannot run the problem gives FLE_ERR_UNSUPPORTED from fle_run.  Grouped
 * problems accept 0, 2, 4 and 5. */
void fle_force_variant(int variant);

/* Force the split of K for the calling thread's next calls on the tiled and skinny kernels (a test
 * and tuning knob like fle_force_variant): 0 = automatic, 1 = no split, S > 1 = S workgroups per output tile, each
 * over its own K range, summed in a fixed order by a reduction pass (capped at the number of
 * K steps and at 64).  A split needs S * M * N * 4 more workspace bytes; fle_workspace_size
 * reports them. */
void fle_force_split(int split);

/* Library version: major * 10000 + minor * 100 + patch. */
int fle_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FLE_H */
