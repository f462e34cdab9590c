// Device side of libfle: hand-written gfx950 (CDNA4) kernels and their launcher.
//
//   fle_gemm_tiled.h     gemm_tiled_256 / _128 (+ _grouped_): LDS-tiled MFMA GEMM (bf16, fp16, fp32) with the epilogue fused
//   fle_gemm_skinny.h    gemm_bf16_skinny: HBM-bound GEMM for few rows, W staged through LDS in long contiguous runs
//                        (row blocks of 32; bf16 / fp16 also 64 .. 256)
//   fle_gemm_thin.h      gemm_gemv (M <= 4 / 8, row-contiguous loads and dot products), gemm_thin (M <= 32, 16-row W tiles on
//                        the 16x16 MFMA): streams over W without LDS staging, every dtype
//   fle_gemm_general.h   gemm_general: any shape / alignment / dtype, small tiles, in-block split of K
//   fle_rowops.h         finalize_rows / finalize_lse (second pass of a row reduction + trailing ops),
//                        reduce_slabs (ordered sum of split-K slabs + the ops before the row op)
//   fle_device_common.h  argument structs, dtype-aware loads / stores, elementwise ops, partial statistics
//
// Orientation used by every GEMM kernel: the W tile is MFMA operand A and the x tile is
// operand B, so the accumulator holds a tile of out^T.  In the MFMA result layout a lane owns
// one column and groups of four consecutive rows; with this orientation a lane therefore owns
// one output row m and groups of four consecutive n: stores, bias and residual accesses are
// 8-byte vectors, and a row reduction is in-register work plus one cross-lane exchange.
#include "fle_device_common.h"
#include "fle_gemm_general.h"
#include "fle_gemm_skinny.h"
#include "fle_gemm_thin.h"
#include "fle_attention.h"
#include "fle_chain.h"
#include "fle_gemm_tiled.h"
#include "fle_rowops.h"

#include <atomic>

namespace fle {

// ------------------------------------------------------------------ static scratch (fle_run_static)
// Device memory for callers that cannot allocate: part of the code object, one copy per GPU.  In host code
// the array's name is only a handle for hipGetSymbolAddress; kernels and copies get the looked-up address.
static __device__ __align__(256) unsigned char scratch[FLE_STATIC_SCRATCH_BYTES];
static constexpr int kMaxDevices = 64;
static std::atomic<void *> g_scratch_ptr[kMaxDevices];

fle_status static_scratch(void **ptr) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return fail(FLE_ERR_HIP, "cannot query the current device");
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {  // once per device, with that device current (two threads racing here look up the same address)
        const hipError_t err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (err != hipSuccess || !p) return fail(FLE_ERR_HIP, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(err));
        g_scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *ptr = p;
    return FLE_OK;
}

// ------------------------------------------------------------------ launcher
static fle_status check_launch(const char *what) {
    const hipError_t err = hipGetLastError();
    if (err != hipSuccess) return fail(FLE_ERR_HIP, "%s: %s", what, hipGetErrorString(err));
    return FLE_OK;
}

fle_status launch(const fle_problem *p, const Plan &plan, const fle_groups *grp) {
    hipStream_t stream = reinterpret_cast<hipStream_t>(p->stream);
    const DevEpilogue &e = plan.epi;
    char *ws = reinterpret_cast<char *>(p->workspace);
    const bool bf16 = p->dtype != FLE_F32;  // 2-byte operands (bf16 or fp16)
    const size_t es = bf16 ? 2 : 4;

    GemmArgs g{};
    g.M = p->M; g.N = p->N; g.K = p->K;
    g.x = p->x; g.ldx = p->ldx; g.w = p->w; g.ldw = p->ldw;
    g.np = plan.np;
    g.partials = e.row_kind >= 0 ? reinterpret_cast<float *>(ws + plan.ws_part_off) : nullptr;
    g.tiles_m = int32_t(plan.tiles_m); g.tiles_n = int32_t(plan.tiles_n);
    g.epi = e;
    g.x_scale = plan.x_scale;
    g.w_scale = plan.w_scale;
    if (plan.ln_pre == LN_PRE_FUSED) {
        g.ln_gamma = plan.ln_gamma; g.ln_beta = plan.ln_beta; g.ln_eps = plan.ln_eps;
    } else if (plan.ln_pre == LN_PRE_PASS) {
        // the normalised copy of x, rows contiguous, which the GEMM kernel then reads in place of x
        LnArgs l{};
        l.M = p->M; l.K = p->K; l.x = p->x; l.ldx = p->ldx; l.gamma = plan.ln_gamma; l.beta = plan.ln_beta; l.eps = plan.ln_eps;
        l.dtype = p->dtype; l.dst = ws + plan.ws_xhat_off;
        const uintptr_t all = reinterpret_cast<uintptr_t>(p->x) | reinterpret_cast<uintptr_t>(plan.ln_gamma) | reinterpret_cast<uintptr_t>(plan.ln_beta) | uintptr_t(p->ldx * int64_t(es));
        l.vec = (all % 16 == 0 && p->K % int64_t(16 / es) == 0) ? 1 : 0;
        if (p->M > 0 && p->K > 0) {
            const bool in_regs = l.vec && p->K <= 16384;  // one wave per row, four rows per workgroup
            const int64_t wgs_ln = in_regs ? (p->M + 3) / 4 : p->M;
            void (*lnk)(LnArgs) = p->dtype == FLE_F32 ? ln_prologue<FLE_F32> : p->dtype == FLE_F16 ? ln_prologue<FLE_F16> : ln_prologue<FLE_BF16>;
            hipLaunchKernelGGL(lnk, dim3(uint32_t(wgs_ln < 65536 ? wgs_ln : 65536)), dim3(256), 0, stream, l);
            const fle_status ls = check_launch("LayerNorm pass launch");
            if (ls != FLE_OK) return ls;
        }
        g.x = l.dst; g.ldx = p->K;
    }
    if (e.row_kind < 0 || plan.staging == ST_OUT) { g.dst = p->out; g.ldd = p->ldo; g.dst_f32 = 0; g.dst_rel = plan.stage_rel; }
    else if (plan.staging == ST_WS) { g.dst = ws + plan.ws_y_off; g.ldd = p->N; g.dst_f32 = 1; }
    else { g.dst = nullptr; g.ldd = 0; g.dst_f32 = 0; }

    // Split K: the GEMM writes bare fp32 slabs; reduce_slabs takes over dst, the pre-ops and the partials.
    RedArgs r{};
    const bool split = plan.split_k > 1;
    if (split) {
        r.M = p->M; r.N = p->N;
        r.slabs = reinterpret_cast<const float *>(ws + plan.ws_slab_off);
        r.ld_slab = (p->N + 3) / 4 * 4;
        r.stride = p->M * r.ld_slab;
        r.vec = plan.edge ? 0 : 1;
        r.S = plan.split_k;
        r.dst = g.dst; r.ldd = g.ldd; r.dst_f32 = g.dst_f32; r.dst_rel = g.dst_rel;
        r.np = plan.np; r.partials = g.partials;
        r.epi = e;
        g.dst = ws + plan.ws_slab_off; g.ldd = r.ld_slab; g.dst_f32 = 1; g.dst_rel = 0;
        g.split_stride = r.stride * int64_t(sizeof(float));
        g.partials = nullptr;
        g.epi.n_pre = 0; g.epi.n_post = 0; g.epi.row_kind = -1;
    }
    // skinny kernel: W tiles in groups of 8 (one per XCD), each with all its row blocks
    const int64_t wgs = plan.variant == V_SKINNY ? (plan.tiles_n + 7) / 8 * 8 * plan.tiles_m : plan.tiles_m * plan.tiles_n;
    const dim3 grid{uint32_t(wgs), uint32_t(plan.split_k)};
    if (plan.variant == V_SKINNY) {
        auto pick = [&](auto dt_c) -> void (*)(GemmArgs) {
            constexpr int DT = decltype(dt_c)::value;
            if (plan.bm == 32) return plan.bk == 256 ? gemm_bf16_skinny<1, 256, DT> : plan.bk == 128 ? gemm_bf16_skinny<1, 128, DT> : gemm_bf16_skinny<1, 64, DT>;
            // larger row blocks: 32-row sub-blocks in turn on a 256-wide K step, or (64 rows) both at once on a 128-wide one
            if (plan.bk == 128) return gemm_bf16_skinny<2, 128, DT>;
            return plan.bm == 64 ? gemm_bf16_skinny<2, 256, DT, true> : plan.bm == 128 ? gemm_bf16_skinny<4, 256, DT, true> : gemm_bf16_skinny<8, 256, DT, true>;
        };
        void (*kern)(GemmArgs);
        if (p->dtype == FLE_F32)  // row blocks of 32 only; the K step is half as many elements for the same bytes
            kern = plan.bk == 128 ? gemm_bf16_skinny<1, 128, FLE_F32> : plan.bk == 64 ? gemm_bf16_skinny<1, 64, FLE_F32> : gemm_bf16_skinny<1, 32, FLE_F32>;
        else
            kern = p->dtype == FLE_F16 ? pick(std::integral_constant<int, FLE_F16>{}) : pick(std::integral_constant<int, FLE_BF16>{});
        hipLaunchKernelGGL(kern, grid, dim3(256), 0, stream, g);
    } else if (plan.variant == V_THIN) {
        // dot-product form: 4 rows of W per wave, or (one row of x, many rows of W) one per wave and 16 waves
        const bool wide = plan.bm <= 8 && plan.bk == 1;  // (the plan's K step field carries the rows per wave for this form)
        auto pick = [&](auto dt_c) -> void (*)(GemmArgs) {
            constexpr int DT = decltype(dt_c)::value;
            if (plan.bm <= 8) {  // (the planner gives 5 .. 8 rows to this form for fp32 only)
                if (plan.ln_pre == LN_PRE_FUSED) {  // (the planner fuses up to 4 rows)
                    if (wide) return gemm_gemv<DT, 1, 1, true>;
                    return p->M <= 1 ? gemm_gemv<DT, 1, 4, true> : p->M <= 2 ? gemm_gemv<DT, 2, 4, true> : gemm_gemv<DT, 4, 4, true>;
                }
                if constexpr (DT == FLE_F32)
                    if (p->M > 4) return gemm_gemv<DT, 8, 4>;
                if (wide) return gemm_gemv<DT, 1, 1>;
                return p->M <= 1 ? gemm_gemv<DT, 1, 4> : p->M <= 2 ? gemm_gemv<DT, 2, 4> : gemm_gemv<DT, 4, 4>;
            }
            return plan.bm == 16 ? gemm_thin<DT, 1> : gemm_thin<DT, 2>;
        };
        void (*kern)(GemmArgs) = p->dtype == FLE_F32 ? pick(std::integral_constant<int, FLE_F32>{})
                                 : p->dtype == FLE_F16 ? pick(std::integral_constant<int, FLE_F16>{}) : pick(std::integral_constant<int, FLE_BF16>{});
        const uint32_t threads = wide ? 1024u : 256u;
        hipLaunchKernelGGL(kern, dim3(uint32_t(plan.tiles_n)), dim3(threads), 0, stream, g);
    } else if (plan.variant == V_TILED && grp) {
        const bool edge = plan.edge != 0;
        const int64_t xs = plan.op_dtype == FLE_F8E4M3 ? 1 : int64_t(es);  // bytes per element of W
        GroupArgs ga{grp->row_offsets, grp->n_groups, grp->w_group_stride * xs, grp->b_group_stride * int64_t(es)};
        auto pick = [&](auto dt_c) -> void (*)(GemmArgs, GroupArgs) {
            constexpr int DT = decltype(dt_c)::value;
            if (plan.bm == 256) return edge ? gemm_tiled_grouped_256<DT, true> : gemm_tiled_grouped_256<DT, false>;
            if (plan.w_stream) return edge ? gemm_tiled_grouped_128<DT, true, true> : gemm_tiled_grouped_128<DT, false, true>;
            return edge ? gemm_tiled_grouped_128<DT, true, false> : gemm_tiled_grouped_128<DT, false, false>;
        };
        void (*kern)(GemmArgs, GroupArgs) = p->dtype == FLE_F32 ? pick(std::integral_constant<int, FLE_F32>{})
                                            : p->dtype == FLE_F16 ? pick(std::integral_constant<int, FLE_F16>{})
                                            : p->dtype == FLE_F8E4M3 ? pick(std::integral_constant<int, FLE_F8E4M3>{}) : pick(std::integral_constant<int, FLE_BF16>{});
        hipLaunchKernelGGL(kern, grid, dim3(256), 0, stream, g, ga);
    } else if (plan.variant == V_TILED) {
        // split K writes fp32 slabs with a padded leading dimension: vector stores whatever out looks like
        const bool edge = plan.edge && !split;
        void (*kern)(GemmArgs);
        auto pick = [&](auto dt_c) -> void (*)(GemmArgs) {
            constexpr int DT = decltype(dt_c)::value;
            if (plan.bm == 256) return edge ? gemm_tiled_256<DT, true> : gemm_tiled_256<DT, false>;
            return edge ? gemm_tiled_128<DT, true> : gemm_tiled_128<DT, false>;
        };
        if (p->dtype == FLE_F32) kern = pick(std::integral_constant<int, FLE_F32>{});
        else if (p->dtype == FLE_F16) kern = pick(std::integral_constant<int, FLE_F16>{});
        else if (p->dtype == FLE_F8E4M3 && plan.mx)
            kern = plan.bm == 256 ? (edge ? gemm_tiled_256<FLE_F8E4M3, true, 32, -1, true> : gemm_tiled_256<FLE_F8E4M3, false, 32, -1, true>)
                                  : (edge ? gemm_tiled_128<FLE_F8E4M3, true, 32, -1, true> : gemm_tiled_128<FLE_F8E4M3, false, 32, -1, true>);
        else if (p->dtype == FLE_F8E4M3) kern = pick(std::integral_constant<int, FLE_F8E4M3>{});
        else kern = pick(std::integral_constant<int, FLE_BF16>{});
        hipLaunchKernelGGL(kern, grid, dim3(256), 0, stream, g);
    } else {
        // vector loads need 4-element groups that never straddle K and rows that keep the alignment
        const size_t va = bf16 ? 8 : 16;
        const bool vec = p->K % 4 == 0 && reinterpret_cast<uintptr_t>(p->x) % va == 0 && reinterpret_cast<uintptr_t>(p->w) % va == 0 &&
                         p->ldx % 4 == 0 && p->ldw % 4 == 0;
        auto pick = [&](auto dt_c) -> void (*)(GemmArgs) {
            constexpr int DT = decltype(dt_c)::value;
            if (plan.bm == 32) return vec ? gemm_general<DT, true, 2> : gemm_general<DT, false, 2>;
            return vec ? gemm_general<DT, true, 1> : gemm_general<DT, false, 1>;
        };
        void (*kern)(GemmArgs) = p->dtype == FLE_F32 ? pick(std::integral_constant<int, FLE_F32>{})
                                 : p->dtype == FLE_F16 ? pick(std::integral_constant<int, FLE_F16>{}) : pick(std::integral_constant<int, FLE_BF16>{});
        hipLaunchKernelGGL(kern, grid, dim3(256), 0, stream, g);
    }
    fle_status s = check_launch("GEMM kernel launch");
    if (s == FLE_OK && split) {
        const int64_t want = (p->M * ((p->N + 255) / 256) + 3) / 4;
        hipLaunchKernelGGL(reduce_slabs, dim3(uint32_t(want < (int64_t(1) << 20) ? want : (int64_t(1) << 20))), dim3(256), 0, stream, r);
        s = check_launch("split-K reduction launch");
    }
    if (s != FLE_OK || e.row_kind < 0) return s;

    FinArgs f{};
    f.M = p->M; f.N = p->N;
    f.np = plan.np; f.part_cols = plan.part_cols;
    f.part_shift = 0;
    while ((1 << f.part_shift) < plan.part_cols) ++f.part_shift;
    if ((1 << f.part_shift) != plan.part_cols) return fail(FLE_ERR_UNSUPPORTED, "internal: partial width %d is not a power of two", plan.part_cols);
    f.partials = split ? r.partials : g.partials;
    f.out = p->out; f.ldo = p->ldo;
    f.epi = e;
    if (grp && grp->b_group_stride != 0) {  // a bias op after the row op needs the row's group
        for (int o = 0; o < e.n_post; ++o)
            if (e.post[o].kind == FLE_BIAS) {
                f.row_offsets = grp->row_offsets;
                f.n_groups = grp->n_groups;
                f.b_stride_bytes = grp->b_group_stride * int64_t(es);
            }
    }
    if (e.row_kind == FLE_LOGSUMEXP) {
        hipLaunchKernelGGL(finalize_lse, dim3(uint32_t((p->M + 3) / 4)), dim3(256), 0, stream, f);
        return check_launch("logsumexp finalize launch");
    }
    const bool two = e.row2_kind >= 0;  // a second row reduction: this pass hands its values over in fp32
    if (two) { f.out = ws + plan.ws_mid_off; f.ldo = p->N; f.out_f32 = 1; }
    if (split) { f.y = r.dst; f.ldy = r.ldd; f.y_f32 = r.dst_f32; }
    else { f.y = g.dst; f.ldy = g.ldd; f.y_f32 = g.dst_f32; }
    f.y_rel = plan.stage_rel;
    const size_t ysz = f.y_f32 ? 4 : es;
    const bool vec = p->N % 8 == 0 && f.ldy % 8 == 0 && f.ldo % 8 == 0 && reinterpret_cast<uintptr_t>(f.y) % (8 * ysz) == 0 &&
                     reinterpret_cast<uintptr_t>(f.out) % (8 * (two ? 4 : es)) == 0;
    // vector path also needs 16-byte aligned gamma / beta
    const bool gb_ok = reinterpret_cast<uintptr_t>(e.row.p0) % (8 * es) == 0 && reinterpret_cast<uintptr_t>(e.row.p1) % (8 * es) == 0;
    const int64_t items = p->M * ((p->N + 2047) / 2048);
    const int64_t want = (items + 3) / 4;
    const dim3 fgrid(uint32_t(want < (int64_t(1) << 20) ? want : (int64_t(1) << 20)));
    void (*fin)(FinArgs);
    const int fdt = e.dtype;
    if (e.row_kind == FLE_LAYERNORM)
        fin = !(vec && gb_ok) ? finalize_rows<false, true>
              : fdt == FLE_BF16 ? finalize_rows<true, true, FLE_BF16> : fdt == FLE_F16 ? finalize_rows<true, true, FLE_F16> : finalize_rows<true, true, FLE_F32>;
    else
        fin = !(vec && gb_ok) ? finalize_rows<false, false>
              : fdt == FLE_BF16 ? finalize_rows<true, false, FLE_BF16> : fdt == FLE_F16 ? finalize_rows<true, false, FLE_F16> : finalize_rows<true, false, FLE_F32>;
    hipLaunchKernelGGL(fin, fgrid, dim3(256), 0, stream, f);
    s = check_launch("row finalize launch");
    if (s != FLE_OK || !two) return s;
    Row2Args r2{};
    r2.M = p->M; r2.N = p->N;
    r2.v = reinterpret_cast<const float *>(ws + plan.ws_mid_off);
    r2.out = p->out; r2.ldo = p->ldo;
    r2.epi = e;
    hipLaunchKernelGGL(second_row_op, dim3(uint32_t(p->M < (int64_t(1) << 16) ? p->M : (int64_t(1) << 16))), dim3(256), 0, stream, r2);
    return check_launch("second row reduction launch");
}

template <int DT, int D>
static void launch_attention_dt(const fle_attention *p, const AttnArgs &a, hipStream_t stream) {
    // One query tile per wave, 128 queries per workgroup: two (D = 128) or three (D <= 64) waves per SIMD, so
    // that one wave's softmax arithmetic runs under another's MFMAs.  Two tiles per wave halve the LDS reads
    // per MFMA but leave one wave per SIMD at D = 128, and measured 10 - 35 % slower there (equal at D = 64).
    hipLaunchKernelGGL((flash_attention<DT, D, 1>), dim3(uint32_t((p->T + 127) / 128 * p->H * p->B)), dim3(256), 0, stream, a);
}

fle_status launch_attention(const fle_attention *p) {
    hipStream_t stream = reinterpret_cast<hipStream_t>(p->stream);
    AttnArgs a;
    a.q = p->q; a.k = p->k; a.v = p->v; a.o = p->o;
    a.ldq = p->ldq; a.ldk = p->ldk; a.ldv = p->ldv; a.ldo = p->ldo;
    const int64_t Tk = p->Tk > 0 ? p->Tk : p->T;
    a.sbq = p->sbq > 0 ? p->sbq : p->T * p->ldq; a.sbo = p->sbo > 0 ? p->sbo : p->T * p->ldo;
    a.sbk = p->sbk > 0 ? p->sbk : Tk * p->ldk; a.sbv = p->sbv > 0 ? p->sbv : Tk * p->ldv;
    a.T = int32_t(p->T); a.Tk = int32_t(Tk); a.H = int32_t(p->H); a.B = int32_t(p->B); a.causal = p->causal;
    const float scale = p->scale > 0.0f ? p->scale : 1.0f / sqrtf(float(p->D));
    a.scale_log2e = scale * 1.44269504088896340736f;
    const bool f16 = p->dtype == FLE_F16;
    switch (p->D) {
    case 32: f16 ? launch_attention_dt<FLE_F16, 32>(p, a, stream) : launch_attention_dt<FLE_BF16, 32>(p, a, stream); break;
    case 64: f16 ? launch_attention_dt<FLE_F16, 64>(p, a, stream) : launch_attention_dt<FLE_BF16, 64>(p, a, stream); break;
    case 128: f16 ? launch_attention_dt<FLE_F16, 128>(p, a, stream) : launch_attention_dt<FLE_BF16, 128>(p, a, stream); break;
    default: f16 ? launch_attention_dt<FLE_F16, 256>(p, a, stream) : launch_attention_dt<FLE_BF16, 256>(p, a, stream); break;
    }
    return check_launch("flash_attention");
}

fle_status launch_chain(const fle_chain *p, void *sync, void *acts, size_t act_stride) {
    hipStream_t stream = reinterpret_cast<hipStream_t>(p->stream);
    ChainArgs a;
    a.n_layers = p->n_layers;
    a.x = p->x; a.out = p->out; a.sync = reinterpret_cast<uint32_t *>(sync);
    for (int l = 0; l < kChainMaxLayers; ++l) a.act[l] = acts ? reinterpret_cast<char *>(acts) + size_t(l) * act_stride : nullptr;
    int64_t widest = 0;
    for (int l = 0; l < p->n_layers; ++l) {
        a.layer[l].w = p->layers[l].w; a.layer[l].bias = p->layers[l].b;
        a.layer[l].n = int32_t(p->layers[l].n); a.layer[l].k = int32_t(p->layers[l].k); a.layer[l].act = p->layers[l].act;
        if (p->layers[l].n > widest) widest = p->layers[l].n;
    }
    // at most one workgroup of 16 waves per CU (a CU holds two), so that every workgroup is resident while the
    // others wait at a barrier; fewer when no layer has 16 rows for each
    static thread_local int cu_count[64] = {0};  // per device: CUs (queried once per thread and device)
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return fail(FLE_ERR_HIP, "cannot query the current device");
    if (cu_count[dev] == 0 && (hipDeviceGetAttribute(&cu_count[dev], hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cu_count[dev] < 1)) {
        cu_count[dev] = 0;
        return fail(FLE_ERR_HIP, "cannot query the device's CU count");
    }
    const int cus = cu_count[dev];
    const int64_t want = (widest + 15) / 16;
    const uint32_t grid = uint32_t(want < cus ? want : cus);
    if (p->dtype == FLE_F32) {
        if (p->w_dtype == FLE_BF16) hipLaunchKernelGGL((mlp_chain<FLE_F32, FLE_BF16>), dim3(grid), dim3(1024), 0, stream, a);
        else if (p->w_dtype == FLE_F16) hipLaunchKernelGGL((mlp_chain<FLE_F32, FLE_F16>), dim3(grid), dim3(1024), 0, stream, a);
        else hipLaunchKernelGGL((mlp_chain<FLE_F32, FLE_F32>), dim3(grid), dim3(1024), 0, stream, a);
    } else if (p->dtype == FLE_F16) {
        hipLaunchKernelGGL((mlp_chain<FLE_F16, FLE_F16>), dim3(grid), dim3(1024), 0, stream, a);
    } else {
        hipLaunchKernelGGL((mlp_chain<FLE_BF16, FLE_BF16>), dim3(grid), dim3(1024), 0, stream, a);
    }
    return check_launch("mlp_chain");
}

}  // namespace fle
