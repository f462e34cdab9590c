// Device-side types and helpers shared by every libfle kernel: vector types, kernel argument structs,
// dtype-aware loads and stores, the elementwise ops, and the row-reduction partials.
#pragma once
#include <hip/hip_runtime.h>

#include <type_traits>

#include "fle_plan.h"

namespace fle {


typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(4))) _Float16 f16x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((address_space(3))) void lds_void;

struct GemmArgs {
    int64_t M, N, K;
    const void *x;
    int64_t ldx;
    const void *w;
    int64_t ldw;
    void *dst;  // where the values after the pre-ops go (nullptr: nowhere, logsumexp)
    int64_t ldd;
    int32_t dst_f32;  // dst holds fp32 regardless of the storage dtype (workspace staging)
    int32_t dst_rel;  // row op staged in a 2-byte dtype: store v - (mean / maximum of v's partial); the finalize pass adds it back in fp32
    int32_t np;       // row-reduction partials per row
    float *partials;  // [M][np][2], or nullptr without a row op
    int32_t tiles_m, tiles_n;
    int64_t split_stride;  // split K (gridDim.y > 1): workgroup row y owns a K range and writes dst + y * split_stride bytes
    const void *x_scale, *w_scale;  // block-scaled fp8 operands: one E8M0 byte per 32 consecutive k, [M][K/32] and [N][K/32]
    const void *ln_gamma, *ln_beta;  // LayerNorm of x over K in front of the multiplication, done by the kernel itself
    float ln_eps;                    // (dot-product kernel for a few rows of x only); gamma / beta [K] or nullptr
    DevEpilogue epi;
};

// LayerNorm of the rows of x over K, written to a contiguous copy (the pass in front of the GEMM kernels).
struct LnArgs {
    int64_t M, K;
    const void *x;
    int64_t ldx;
    const void *gamma, *beta;  // [K] or nullptr
    float eps;
    int32_t dtype;
    int32_t vec;               // rows, gamma and beta allow 16-byte accesses of 8 (2-byte dtypes) or 4 (fp32) elements
    void *dst;                 // [M][K], rows contiguous
};

// Sum of the split-K slabs followed by the ops before the row op (reduce_slabs).
struct RedArgs {
    int64_t M, N;
    const float *slabs;  // [S][M][N] fp32
    int64_t stride;      // elements between slabs
    int64_t ld_slab;     // elements between slab rows (N rounded up to a multiple of 4)
    int32_t S;
    int32_t vec;         // b, residual and dst allow 4-column vector accesses
    int32_t dst_f32;
    int32_t dst_rel;     // as GemmArgs::dst_rel
    void *dst;           // as GemmArgs::dst
    int64_t ldd;
    int32_t np;
    float *partials;     // one partial per (row, 256 columns)
    DevEpilogue epi;
};

struct FinArgs {
    int64_t M, N;
    const void *y;  // staged values: storage dtype (may alias out) or fp32
    int64_t ldy;
    int32_t y_f32;
    int32_t y_rel;  // staged values are relative to the mean / maximum of their partial (2-byte dtypes)
    int32_t np, part_cols;
    int32_t part_shift;  // log2(part_cols): the planner only uses powers of two
    const float *partials;
    void *out;
    int64_t ldo;
    int32_t out_f32;  // out holds fp32 regardless of the storage dtype (the values handed to a second row reduction)
    // grouped problems whose list has a bias op after the row op: the row's group selects the bias
    const int64_t *row_offsets;  // [n_groups + 1] (device), or nullptr
    int32_t n_groups;
    int64_t b_stride_bytes;
    DevEpilogue epi;
};

// Second row reduction of a list (second_row_op): v[M,N] fp32 in, out in the storage dtype.
struct Row2Args {
    int64_t M, N;
    const float *v;  // [M][N] fp32, packed rows
    void *out;       // [M][ldo], or [M] for logsumexp
    int64_t ldo;
    DevEpilogue epi; // row2_kind, row2, post2 (and bias, dtype)
};

// ------------------------------------------------------------------ scalar helpers
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

__device__ __forceinline__ float ld_elem(const void *p, int64_t i, int dtype) {
    if (dtype == FLE_BF16) return bf16_bits_to_f32(reinterpret_cast<const uint16_t *>(p)[i]);
    if (dtype == FLE_F16) return float(reinterpret_cast<const _Float16 *>(p)[i]);
    return reinterpret_cast<const float *>(p)[i];
}

__device__ __forceinline__ void st_elem(void *p, int64_t i, int dtype, float v) {
    if (dtype == FLE_BF16)
        reinterpret_cast<__bf16 *>(p)[i] = static_cast<__bf16>(v);
    else if (dtype == FLE_F16)
        reinterpret_cast<_Float16 *>(p)[i] = static_cast<_Float16>(v);
    else
        reinterpret_cast<float *>(p)[i] = v;
}

__device__ __forceinline__ f32x4 ld4_bf16(const void *p) {  // p is 8-byte aligned
    const uint2 u = *reinterpret_cast<const uint2 *>(p);
    f32x4 r;
    r[0] = __uint_as_float(u.x << 16);
    r[1] = __uint_as_float(u.x & 0xffff0000u);
    r[2] = __uint_as_float(u.y << 16);
    r[3] = __uint_as_float(u.y & 0xffff0000u);
    return r;
}

// 4 consecutive elements at element index i of p as fp32 (p + i aligned to 4 elements).  DT: fle_dtype.
template <int DT>
__device__ __forceinline__ f32x4 ld4(const void *p, int64_t i) {
    if constexpr (DT == FLE_F32) return *reinterpret_cast<const f32x4 *>(reinterpret_cast<const float *>(p) + i);
    else if constexpr (DT == FLE_F16) return __builtin_convertvector(*reinterpret_cast<const f16x4 *>(reinterpret_cast<const _Float16 *>(p) + i), f32x4);
    else return ld4_bf16(reinterpret_cast<const uint16_t *>(p) + i);
}
__device__ __forceinline__ f32x4 ld4_rt(const void *p, int64_t i, int dtype) {  // dtype known at run time only
    if (dtype == FLE_F32) return ld4<FLE_F32>(p, i);
    if (dtype == FLE_F16) return ld4<FLE_F16>(p, i);
    return ld4<FLE_BF16>(p, i);
}

// 4 fp32 values rounded (to nearest even) to a 2-byte dtype and packed into 8 bytes.
template <int DT>
__device__ __forceinline__ u32x2 pack4(f32x4 v) {
    static_assert(DT == FLE_BF16 || DT == FLE_F16, "2-byte dtypes only");
    if constexpr (DT == FLE_F16) return __builtin_bit_cast(u32x2, __builtin_convertvector(v, f16x4));
    else return __builtin_bit_cast(u32x2, __builtin_convertvector(v, bf16x4));
}
__device__ __forceinline__ u32x2 pack4_rt(f32x4 v, int dtype) { return dtype == FLE_F16 ? pack4<FLE_F16>(v) : pack4<FLE_BF16>(v); }

__device__ __forceinline__ float relu_f(float v) { return v < 0.0f ? 0.0f : v; }  // NaN stays NaN

// GELU with the exact-erf definition.  erfc(|x|) = t (a1 + t (a2 + t (a3 + t (a4 + t a5)))) exp(-x^2),
// t = 1 / (1 + p |x|)  (Abramowitz & Stegun 7.1.26, |error| <= 1.5e-7), and
// 1 + erf(x) = erfc(|x|) for x < 0, 2 - erfc(|x|) otherwise: no cancellation in the left tail.
// (Constants folded: |v| / sqrt 2 into p, the final 1/2 into the coefficients, exp(-v^2 / 2) as 2^(v v (-log2 e / 2));
// h = erfc(|v| / sqrt 2) / 2, and the result is v h for v < 0, v - v h otherwise: 13 plain and 2 quarter-rate
// instructions per value, which at 256 values per lane is most of what this epilogue costs a 256 x 256 tile.)
__device__ __forceinline__ float gelu_erf_f(float v) {
    const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f * 0.70710678118654752f, fabsf(v), 1.0f));
    float p = fmaf(t, 0.5f * 1.061405429f, 0.5f * -1.453152027f);
    p = fmaf(t, p, 0.5f * 1.421413741f);
    p = fmaf(t, p, 0.5f * -0.284496736f);
    p = fmaf(t, p, 0.5f * 0.254829592f);
    const float h = p * t * __builtin_amdgcn_exp2f(v * v * (-0.5f * 1.4426950408889634f));
    const float r = v * h;
    return v < 0.0f ? r : v - r;
}

// 0.5 v (1 + tanh u) == v / (1 + exp(-2u)),  u = sqrt(2/pi) (v + 0.044715 v^3)
// (exp(-2u) as 2^(v (1 + 0.044715 v^2) k), k = -2 sqrt(2/pi) log2 e: 6 plain and 2 quarter-rate instructions per value)
__device__ __forceinline__ float gelu_tanh_f(float v) {
    const float w = fmaf(0.044715f * v, v, 1.0f);
    const float e = __builtin_amdgcn_exp2f(v * w * (-2.0f * 0.7978845608028654f * 1.4426950408889634f));
    return v * __builtin_amdgcn_rcpf(1.0f + e);
}

// One elementwise op on one value at (m, n).
__device__ __forceinline__ float apply_op(const DevOp &op, float v, int64_t m, int64_t n, const void *bias, int dtype) {
    switch (op.kind) {
    case FLE_BIAS: return v + ld_elem(bias, n, dtype);
    case FLE_SCALE: return v * op.alpha;
    case FLE_RELU: return relu_f(v);
    case FLE_GELU_ERF: return gelu_erf_f(v);
    case FLE_GELU_TANH: return gelu_tanh_f(v);
    case FLE_RESIDUAL: return v + ld_elem(op.p0, m * op.ld + n, dtype);
    case FLE_STORE: st_elem(const_cast<void *>(op.p0), m * op.ld + n, dtype, v); return v;
    default: return v;
    }
}

// ------------------------------------------------------------------ row-reduction partials
// LayerNorm partial over c values: (mean, M2 = sum (v - mean)^2); the count is implied by the
// partial's position.  Softmax / logsumexp partial: (max, sum exp(v - max)).
struct Stat {
    float n, a, b;  // n = count (LayerNorm only); (a, b) = (mean, M2) or (max, sum)
};

__device__ __forceinline__ Stat combine_ln(const Stat &p, const Stat &q) {
    if (q.n == 0.0f) return p;
    if (p.n == 0.0f) return q;
    Stat r;
    r.n = p.n + q.n;
    const float d = q.a - p.a;
    // (one hardware reciprocal, 1 ulp, in place of two IEEE divisions of a dozen instructions each: the combine runs
    // seven times per wave of the finalize pass and was half of its vector-ALU work)
    const float w = q.n * __builtin_amdgcn_rcpf(r.n);
    r.a = fmaf(d, w, p.a);
    r.b = p.b + q.b + d * d * (p.n * w);
    return r;
}

__device__ __forceinline__ Stat combine_sm(const Stat &p, const Stat &q) {
    Stat r;
    r.n = 0.0f;
    r.a = fmaxf(p.a, q.a);
    const float sp = p.b == 0.0f ? 0.0f : p.b * __expf(p.a - r.a);
    const float sq = q.b == 0.0f ? 0.0f : q.b * __expf(q.a - r.a);
    r.b = sp + sq;
    return r;
}

// All lanes of a wave end up with the combination of every partial of `row`, in a fixed order.
// LayerNorm: Chan's update, lane-serial then a butterfly.  Softmax / logsumexp: the row maximum first
// (exact in any order), then every partial sum rescaled to it once and added lane-serially and by
// butterfly: one exp per partial instead of two per pairwise combine.
// first: (LayerNorm) partial `lane` of the row if the caller has already loaded it (with the rest of what it reads), else nullptr.
template <bool LN>
__device__ __forceinline__ Stat reduce_partials(const float *partials, int64_t row, int np, int part_cols, int64_t N, int lane, const float2 *first = nullptr) {
    Stat s;
    s.n = 0.0f;
    s.a = LN ? 0.0f : -INFINITY;
    s.b = 0.0f;
    const float *pr = partials + row * np * 2;
    if (LN) {  // few partials per row (N / 64 or fewer): one load per lane and round
        for (int p = lane; p < np; p += 64) {
            Stat q;
            const int64_t left = N - int64_t(p) * part_cols;
            q.n = float(left < part_cols ? left : part_cols);
            if (first && p == lane) {
                q.a = first->x;
                q.b = first->y;
            } else {
                q.a = pr[2 * p];
                q.b = pr[2 * p + 1];
            }
            s = combine_ln(s, q);
        }
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            Stat o;
            o.n = __shfl_xor(s.n, d);
            o.a = __shfl_xor(s.a, d);
            o.b = __shfl_xor(s.b, d);
            const bool upper = (lane & d) != 0;  // both partners combine (lower lane, upper lane): identical results
            const Stat lo = upper ? o : s, hi = upper ? s : o;
            s = combine_ln(lo, hi);
        }
        return s;
    }
    // softmax / logsumexp: a lane takes partials lane, lane + 64, ...; up to 16 loads go out together so
    // that their latencies overlap (a row of a 32768-column softmax has 1024 partials, 16 per lane)
    constexpr int B = 16;
    if (np <= 64 * B) {  // one batch: keep the partials in registers between the two sweeps
        float2 buf[B];
#pragma unroll
        for (int j = 0; j < B; ++j) {
            const int p = j * 64 + lane;
            buf[j] = make_float2(-INFINITY, 0.0f);
            if (j * 64 < np && p < np) buf[j] = *reinterpret_cast<const float2 *>(pr + 2 * p);  // outer test is wave-uniform
        }
        float mx = -INFINITY;
#pragma unroll
        for (int j = 0; j < B; ++j) mx = fmaxf(mx, buf[j].x);
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) mx = fmaxf(mx, __shfl_xor(mx, d));
        float sum = 0.0f;
#pragma unroll
        for (int j = 0; j < B; ++j)
            if (j * 64 < np && buf[j].y != 0.0f) sum += buf[j].y * __expf(buf[j].x - mx);
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) sum += __shfl_xor(sum, d);  // partners add the same two numbers: identical in every lane
        s.a = mx;
        s.b = sum;
        return s;
    }
    float mx = -INFINITY;
    for (int p = lane; p < np; p += 64) mx = fmaxf(mx, pr[2 * p]);
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) mx = fmaxf(mx, __shfl_xor(mx, d));
    float sum = 0.0f;
    for (int p = lane; p < np; p += 64) {
        const float2 q = *reinterpret_cast<const float2 *>(pr + 2 * p);
        if (q.y != 0.0f) sum += q.y * __expf(q.x - mx);
    }
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) sum += __shfl_xor(sum, d);
    s.a = mx;
    s.b = sum;
    return s;
}

template <int N>
__device__ __forceinline__ void wait_vmcnt() {  // s_waitcnt vmcnt(N), other counters untouched
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | 0x0F70);
}


}  // namespace fle
