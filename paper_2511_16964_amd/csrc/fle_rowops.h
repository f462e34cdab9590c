// Second passes: finalize of LayerNorm / softmax / logsumexp, and the split-K reduction.
#pragma once
#include "fle_device_common.h"

namespace fle {

// ------------------------------------------------------------------ finalize passes
// One wave per (row, 2048-column chunk).  The wave combines the row's partials itself (one
// per lane, then a fixed butterfly: identical result in every lane), issues all of its
// 16-byte loads of staged y at once, normalises, applies the trailing elementwise ops, rounds
// and writes 16-byte vectors.
__device__ __forceinline__ void ld8(const void *p, int64_t i, int dtype, float (&v)[8]) {  // 8 elements at index i
    if (dtype == FLE_F32) {
        const f32x4 *src = reinterpret_cast<const f32x4 *>(reinterpret_cast<const float *>(p) + i);
        const f32x4 u0 = src[0], u1 = src[1];
#pragma unroll
        for (int e = 0; e < 4; ++e) { v[e] = u0[e]; v[4 + e] = u1[e]; }
    } else if (dtype == FLE_F16) {
        const f16x8 u = *reinterpret_cast<const f16x8 *>(reinterpret_cast<const _Float16 *>(p) + i);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = float(u[e]);
    } else {
        const uint4 u = *reinterpret_cast<const uint4 *>(reinterpret_cast<const uint16_t *>(p) + i);
        const uint32_t wv[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) { v[2 * e] = __uint_as_float(wv[e] << 16); v[2 * e + 1] = __uint_as_float(wv[e] & 0xffff0000u); }
    }
}
// 8 fp32 values rounded to a 2-byte dtype, stored as one 16-byte vector at element index i.
__device__ __forceinline__ void st8_2byte(void *p, int64_t i, int dtype, const float (&v)[8]) {
    u32x4 o;
    if (dtype == FLE_F16) {
        f16x8 h;
#pragma unroll
        for (int e = 0; e < 8; ++e) h[e] = static_cast<_Float16>(v[e]);
        o = __builtin_bit_cast(u32x4, h);
    } else {
        bf16x8 h;
#pragma unroll
        for (int e = 0; e < 8; ++e) h[e] = static_cast<__bf16>(v[e]);
        o = __builtin_bit_cast(u32x4, h);
    }
    *reinterpret_cast<u32x4 *>(reinterpret_cast<uint16_t *>(p) + i) = o;
}

// 16 bytes of a 2-byte dtype (known at run time) as 8 fp32 values.
__device__ __forceinline__ void unpack8_2byte(const u32x4 r, int dtype, float (&v)[8]) {
    if (dtype == FLE_F16) {
        const f16x8 h = __builtin_bit_cast(f16x8, r);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = float(h[e]);
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) { v[2 * e] = __uint_as_float(r[e] << 16); v[2 * e + 1] = __uint_as_float(r[e] & 0xffff0000u); }
    }
}

// LNK: LayerNorm (true) or softmax (false); separate kernels so that each gets its own register budget.
// DT: the storage dtype when known at compile time (the vector forms: the conversions then carry no run-time
// choice), -1: read from the arguments.
template <bool VEC, bool LNK, int DT = -1>
__global__ __launch_bounds__(256) void finalize_rows(const FinArgs a) {
    constexpr int CH = 2048, IT = CH / 512;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int dtype = DT >= 0 ? DT : a.epi.dtype;
    const bool f32 = dtype == FLE_F32;
    constexpr bool ln = LNK;
    const int64_t N = a.N;
    const int64_t chunks = (N + CH - 1) / CH, items = a.M * chunks;
    // item -> (row, first column).  (64-bit divisions cost over a hundred vector instructions each; so does the
    // run-time choice of conversions that a dtype known at compile time avoids: c3's pass 34.4 -> 31.5 us with the
    // cheaper combine of the partials.  Walking several items per wave with the next item's loads ahead: 34.1 us.)
    auto place = [&](int64_t item, int64_t &row, int64_t &c0) {
        if (items <= 0x7fffffff) {
            const uint32_t r32 = uint32_t(item) / uint32_t(chunks);
            row = r32;
            c0 = int64_t(uint32_t(item) - r32 * uint32_t(chunks)) * CH;
        } else {
            row = item / chunks;
            c0 = (item % chunks) * CH;
        }
    };
    for (int64_t item = int64_t(blockIdx.x) * 4 + wave; item < items; item += int64_t(gridDim.x) * 4) {
        int64_t row;
        int64_t c0;
        place(item, row, c0);
        const int64_t c1 = c0 + CH < N ? c0 + CH : N;
        // Everything the item reads goes out in one batch in front of the combine of the partials, as loaded
        // (conversions later) and without a branch around any of it: a vector past the end of the row re-reads
        // the row's last one.  (Loads inside per-vector conditions, each converted where it stood, came out as
        // load, wait, convert, load, wait, convert: four round trips to memory per wave instead of one.)
        float y[IT][8];
        [[maybe_unused]] u32x4 yr[VEC ? IT : 1][2], gr[VEC && LNK ? IT : 1], br[VEC && LNK ? IT : 1];
        [[maybe_unused]] float pmean[IT];
        const bool yf = f32 || a.y_f32;                       // staged values are fp32
        constexpr bool early_gb = VEC && LNK && DT >= 0 && DT != FLE_F32;   // gamma / beta of a 2-byte dtype: 4 registers per vector
        [[maybe_unused]] float2 part_first = make_float2(0.0f, 0.0f);
        if (VEC) {
            if constexpr (LNK) {  // this lane's partial of the row, in the same batch
                if (lane < a.np) part_first = *reinterpret_cast<const float2 *>(a.partials + (row * a.np + lane) * 2);
            }
            int64_t nc[IT];
#pragma unroll
            for (int it = 0; it < IT; ++it) {
                const int64_t n = c0 + it * 512 + lane * 8;
                nc[it] = n < c1 ? n : c1 - 8;
            }
            if (yf) {
#pragma unroll
                for (int it = 0; it < IT; ++it) {
                    const u32x4 *q = reinterpret_cast<const u32x4 *>(reinterpret_cast<const float *>(a.y) + row * a.ldy + nc[it]);
                    yr[it][0] = q[0];
                    yr[it][1] = q[1];
                }
            } else {
#pragma unroll
                for (int it = 0; it < IT; ++it) yr[it][0] = *reinterpret_cast<const u32x4 *>(reinterpret_cast<const uint16_t *>(a.y) + row * a.ldy + nc[it]);
            }
            if (a.y_rel) {
#pragma unroll
                for (int it = 0; it < IT; ++it) pmean[it] = a.partials[(row * a.np + (nc[it] >> a.part_shift)) * 2];
            }
            if constexpr (early_gb) {
                if (a.epi.row.p0) {
#pragma unroll
                    for (int it = 0; it < IT; ++it) gr[it] = *reinterpret_cast<const u32x4 *>(reinterpret_cast<const uint16_t *>(a.epi.row.p0) + nc[it]);
                }
                if (a.epi.row.p1) {
#pragma unroll
                    for (int it = 0; it < IT; ++it) br[it] = *reinterpret_cast<const u32x4 *>(reinterpret_cast<const uint16_t *>(a.epi.row.p1) + nc[it]);
                }
            }
        }
        float sub, mul;  // out = (y - sub) * mul  (LayerNorm),  exp(y - sub) * mul  (softmax)
        if (ln) {
            const Stat s = reduce_partials<true>(a.partials, row, a.np, a.part_cols, N, lane, VEC ? &part_first : nullptr);
            sub = s.a;
            mul = rsqrtf(s.b / float(N) + a.epi.row.alpha);
        } else {
            const Stat s = reduce_partials<false>(a.partials, row, a.np, a.part_cols, N, lane);
            sub = s.a;
            mul = 1.0f / s.b;
        }
        // the bias of this row: of its group for a grouped problem (the last group whose first row is <= row:
        // empty groups share their offset with the next one), else the problem's
        const void *bias = a.epi.bias;
        if (a.row_offsets && bias) {
            int lo = 0, hi = a.n_groups;  // invariant: offsets[lo] <= row (offsets[0] counts as 0), offsets[hi] > row or hi == n_groups
            while (hi - lo > 1) {
                const int mid = (lo + hi) / 2;
                if (a.row_offsets[mid] <= row) lo = mid;
                else hi = mid;
            }
            bias = reinterpret_cast<const char *>(bias) + int64_t(lo) * a.b_stride_bytes;
        }
        auto post = [&](float v, int64_t n) -> float {
            for (int o = 0; o < a.epi.n_post; ++o) v = apply_op(a.epi.post[o], v, row, n, bias, dtype);
            return v;
        };
        if (VEC) {
#pragma unroll
            for (int it = 0; it < IT; ++it) {
                const int64_t n = c0 + it * 512 + lane * 8;
                if (n < c1) {
                    float *v = y[it];
                    if (yf) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) { v[e] = __uint_as_float(yr[it][0][e]); v[4 + e] = __uint_as_float(yr[it][1][e]); }
                    } else {
                        unpack8_2byte(yr[it][0], dtype, y[it]);
                    }
                    // staged relative to the statistic (mean / maximum) of the partial the 8 columns lie in (part_cols is a multiple of 8)
                    const float shift = a.y_rel ? sub - pmean[it] : sub;
                    if (ln) {
                        float g[8], be[8];
#pragma unroll
                        for (int e = 0; e < 8; ++e) { g[e] = 1.0f; be[e] = 0.0f; }
                        if constexpr (early_gb) {
                            if (a.epi.row.p0) unpack8_2byte(gr[it], dtype, g);
                            if (a.epi.row.p1) unpack8_2byte(br[it], dtype, be);
                        } else {
                            if (a.epi.row.p0) ld8(a.epi.row.p0, n, dtype, g);
                            if (a.epi.row.p1) ld8(a.epi.row.p1, n, dtype, be);
                        }
#pragma unroll
                        for (int e = 0; e < 8; ++e) v[e] = (v[e] - shift) * mul * g[e] + be[e];
                    } else {
#pragma unroll
                        for (int e = 0; e < 8; ++e) v[e] = __expf(v[e] - shift) * mul;
                    }
                    if (a.epi.n_post > 0) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) v[e] = post(v[e], n + e);
                    }
                    if (f32 || a.out_f32) {
                        f32x4 *dstp = reinterpret_cast<f32x4 *>(reinterpret_cast<float *>(a.out) + row * a.ldo + n);
                        dstp[0] = f32x4{v[0], v[1], v[2], v[3]};
                        dstp[1] = f32x4{v[4], v[5], v[6], v[7]};
                    } else {
                        st8_2byte(a.out, row * a.ldo + n, dtype, y[it]);
                    }
                }
            }
        } else {
            auto one = [&](int64_t n) {  // one element
                const float yv = ld_elem(a.y, row * a.ldy + n, a.y_f32 ? FLE_F32 : dtype);
                float v;
                const float shift = a.y_rel ? sub - a.partials[(row * a.np + (n >> a.part_shift)) * 2] : sub;
                if (ln) {
                    v = (yv - shift) * mul;
                    if (a.epi.row.p0) v *= ld_elem(a.epi.row.p0, n, dtype);
                    if (a.epi.row.p1) v += ld_elem(a.epi.row.p1, n, dtype);
                } else {
                    v = __expf(yv - shift) * mul;
                }
                st_elem(a.out, row * a.ldo + n, a.out_f32 ? FLE_F32 : dtype, post(v, n));
            };
            // bf16 rows whose staged values and outputs share their offset within a 16-byte line (always so
            // when staged in out itself): skip h elements to the next line boundary, then whole lines as
            // 16-byte vectors.  Chunk k takes elements h + 2048 k ... of the row, chunk 0 also the first h.
            const uintptr_t ya = reinterpret_cast<uintptr_t>(a.y) + uintptr_t(row * a.ldy) * 2;
            const uintptr_t oa = reinterpret_cast<uintptr_t>(a.out) + uintptr_t(row * a.ldo) * 2;
            if (!f32 && !a.y_f32 && !a.out_f32 && ((ya ^ oa) & 15) == 0 && (ya & 1) == 0) {
                const int h = int(((16 - (ya & 15)) & 15) >> 1);
                if (c0 == 0 && lane < h && lane < N) one(lane);
#pragma unroll
                for (int it = 0; it < IT; ++it) {
                    const int64_t n = h + c0 + (it * 64 + lane) * 8;
                    if (n + 8 <= N) {
                        float v[8];
                        ld8(a.y, row * a.ldy + n, dtype, v);
                        float s0 = sub, s1 = sub;
                        const int64_t p0 = (n >> a.part_shift), p1 = ((n + 7) >> a.part_shift);  // the 8 columns may straddle two partials
                        if (a.y_rel) {
                            s0 = sub - a.partials[(row * a.np + p0) * 2];
                            s1 = sub - a.partials[(row * a.np + p1) * 2];
                        }
                        if (ln) {
#pragma unroll
                            for (int e = 0; e < 8; ++e) {
                                v[e] = (v[e] - (((n + e) >> a.part_shift) == p0 ? s0 : s1)) * mul;
                                if (a.epi.row.p0) v[e] *= ld_elem(a.epi.row.p0, n + e, dtype);
                                if (a.epi.row.p1) v[e] += ld_elem(a.epi.row.p1, n + e, dtype);
                            }
                        } else {
#pragma unroll
                            for (int e = 0; e < 8; ++e) v[e] = __expf(v[e] - (((n + e) >> a.part_shift) == p0 ? s0 : s1)) * mul;
                        }
                        if (a.epi.n_post > 0) {
#pragma unroll
                            for (int e = 0; e < 8; ++e) v[e] = post(v[e], n + e);
                        }
                        st8_2byte(a.out, row * a.ldo + n, dtype, v);
                    } else {
                        for (int64_t nn = n; nn < N; ++nn) one(nn);  // the row's last, partial line (one lane at most)
                    }
                }
            } else {
                for (int64_t n = c0 + lane; n < c1; n += 64) one(n);
            }
        }
    }
}

// logsumexp: one wave per row, out[row] = max + log(sum).
__global__ __launch_bounds__(256) void finalize_lse(const FinArgs a) {
    const int lane = threadIdx.x & 63;
    const int64_t row = int64_t(blockIdx.x) * 4 + (threadIdx.x >> 6);
    if (row >= a.M) return;
    const Stat s = reduce_partials<false>(a.partials, row, a.np, a.part_cols, a.N, lane);
    if (lane == 0) st_elem(a.out, row, a.epi.dtype, s.a + __logf(s.b));
}

// ------------------------------------------------------------------ a second row reduction in the list
// One workgroup per row: the values behind the first row reduction (and the ops that follow it) arrive in fp32;
// three sweeps over the row (it stays in the L2): mean or maximum, then sum of squared deviations or of
// exponentials, then normalise, apply the ops behind the reduction, round and store.  Sums are formed per thread
// in index order, across the wave by a fixed butterfly and across the four waves in wave order: reproducible.
__device__ __forceinline__ float block_allreduce(float v, bool max, float *lds) {
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const float o = __shfl_xor(v, d);
        v = max ? fmaxf(v, o) : v + o;
    }
    const int wave = threadIdx.x >> 6;
    __syncthreads();  // (the previous use of lds is over)
    if ((threadIdx.x & 63) == 0) lds[wave] = v;
    __syncthreads();
    float r = lds[0];
    for (int w = 1; w < 4; ++w) r = max ? fmaxf(r, lds[w]) : r + lds[w];
    return r;
}

__global__ __launch_bounds__(256) void second_row_op(const Row2Args a) {
    __shared__ float lds[4];
    const int64_t N = a.N;
    const int dtype = a.epi.dtype;
    const int kind = a.epi.row2_kind;
    for (int64_t row = blockIdx.x; row < a.M; row += gridDim.x) {
        const float *v = a.v + row * N;
        float sub, mul;
        if (kind == FLE_LAYERNORM) {
            float s = 0.0f;
            for (int64_t n = threadIdx.x; n < N; n += 256) s += v[n];
            const float mean = block_allreduce(s, false, lds) / float(N);
            float m2 = 0.0f;
            for (int64_t n = threadIdx.x; n < N; n += 256) m2 += (v[n] - mean) * (v[n] - mean);
            m2 = block_allreduce(m2, false, lds);
            sub = mean;
            mul = rsqrtf(m2 / float(N) + a.epi.row2.alpha);
        } else {
            float mx = -INFINITY;
            for (int64_t n = threadIdx.x; n < N; n += 256) mx = fmaxf(mx, v[n]);
            mx = block_allreduce(mx, true, lds);
            float se = 0.0f;
            for (int64_t n = threadIdx.x; n < N; n += 256) se += __expf(v[n] - mx);
            se = block_allreduce(se, false, lds);
            sub = mx;
            mul = 1.0f / se;
            if (kind == FLE_LOGSUMEXP) {
                if (threadIdx.x == 0) st_elem(a.out, row, dtype, mx + __logf(se));
                continue;
            }
        }
        for (int64_t n = threadIdx.x; n < N; n += 256) {
            float o;
            if (kind == FLE_LAYERNORM) {
                o = (v[n] - sub) * mul;
                if (a.epi.row2.p0) o *= ld_elem(a.epi.row2.p0, n, dtype);
                if (a.epi.row2.p1) o += ld_elem(a.epi.row2.p1, n, dtype);
            } else {
                o = __expf(v[n] - sub) * mul;
            }
            for (int q = 0; q < a.epi.n_post2; ++q) o = apply_op(a.epi.post2[q], o, row, n, a.epi.bias, dtype);
            st_elem(a.out, row * a.ldo + n, dtype, o);
        }
    }
}

// ------------------------------------------------------------------ LayerNorm of x in front of the multiplication
// Writes (x - mean) rstd gamma + beta, rounded to the dtype, into a contiguous copy of x that the GEMM kernels read.
// Rows of up to 16384 elements whose operands allow 16-byte accesses: one wave per row, reductions by butterflies
// alone.  Other rows: one workgroup per row, element by element.  Three sweeps in both forms (mean, squared
// deviations, result); the row stays in cache after the first.  Sums per lane in
// index order, then a fixed butterfly (and the waves in wave order): reproducible.
__device__ __forceinline__ float wave_allreduce_sum(float v) {
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) v += __shfl_xor(v, d);
    return v;
}

// 16 bytes as fp32 values (DT: fle_dtype; 4 values of fp32, else 8).
template <int DT>
__device__ __forceinline__ void unpack_vec(const u32x4 r, float (&v)[8]) {
    if constexpr (DT == FLE_F32) {
#pragma unroll
        for (int e = 0; e < 4; ++e) { v[e] = __uint_as_float(r[e]); v[4 + e] = 0.0f; }
    } else if constexpr (DT == FLE_F16) {
        const f16x8 h = __builtin_bit_cast(f16x8, r);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = float(h[e]);
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) { v[2 * e] = __uint_as_float(r[e] << 16); v[2 * e + 1] = __uint_as_float(r[e] & 0xffff0000u); }
    }
}

template <int DT>
__global__ __launch_bounds__(256) void ln_prologue(const LnArgs a) {
    __shared__ float lds[4];
    const int64_t K = a.K;
    constexpr int dtype = DT;
    constexpr int W = DT == FLE_F32 ? 4 : 8;  // elements per 16 bytes
    constexpr int ES = DT == FLE_F32 ? 4 : 2;
    constexpr int NVR = 8;  // vectors of 16 bytes per lane that the register form holds: rows of up to 4096 (fp32: 2048) elements
    if (a.vec && K <= int64_t(64) * W * NVR) {
        // One wave per row, the row read once: all of a lane's vectors requested in one batch, without a branch (a
        // vector past the end of the row re-reads the row's last one and is left out of the sums), and kept as
        // loaded, 4 registers each; each of the three phases converts them anew.  gamma and beta come in two batches
        // of four vectors each.
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
        for (int64_t row = int64_t(blockIdx.x) * 4 + wave; row < a.M; row += int64_t(gridDim.x) * 4) {
            const char *src = reinterpret_cast<const char *>(a.x) + row * a.ldx * ES;
            u32x4 raw[NVR];
            int64_t kc[NVR];
#pragma unroll
            for (int i = 0; i < NVR; ++i) {
                const int64_t k = (int64_t(i) * 64 + lane) * W;
                kc[i] = k < K ? k : K - W;
                raw[i] = *reinterpret_cast<const u32x4 *>(src + kc[i] * ES);
            }
            float s = 0.0f;
#pragma unroll
            for (int i = 0; i < NVR; ++i) {
                float v[8];
                unpack_vec<DT>(raw[i], v);
                float part = 0.0f;
#pragma unroll
                for (int e = 0; e < W; ++e) part += v[e];
                s += (int64_t(i) * 64 + lane) * W < K ? part : 0.0f;
            }
            const float mean = wave_allreduce_sum(s) / float(K);
            float m2 = 0.0f;
#pragma unroll
            for (int i = 0; i < NVR; ++i) {
                float v[8];
                unpack_vec<DT>(raw[i], v);
                float part = 0.0f;
#pragma unroll
                for (int e = 0; e < W; ++e) part += (v[e] - mean) * (v[e] - mean);
                m2 += (int64_t(i) * 64 + lane) * W < K ? part : 0.0f;
            }
            const float rstd = rsqrtf(wave_allreduce_sum(m2) / float(K) + a.eps);
#pragma unroll
            for (int h = 0; h < NVR; h += 4) {
                u32x4 gr[4], br[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    gr[j] = br[j] = u32x4{0u, 0u, 0u, 0u};
                    if (a.gamma) gr[j] = *reinterpret_cast<const u32x4 *>(reinterpret_cast<const char *>(a.gamma) + kc[h + j] * ES);
                    if (a.beta) br[j] = *reinterpret_cast<const u32x4 *>(reinterpret_cast<const char *>(a.beta) + kc[h + j] * ES);
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int64_t k = (int64_t(h + j) * 64 + lane) * W;
                    float v[8], g[8], be[8], o[8];
                    unpack_vec<DT>(raw[h + j], v);
#pragma unroll
                    for (int e = 0; e < 8; ++e) { g[e] = 1.0f; be[e] = 0.0f; }
                    if (a.gamma) unpack_vec<DT>(gr[j], g);
                    if (a.beta) unpack_vec<DT>(br[j], be);
#pragma unroll
                    for (int e = 0; e < 8; ++e) o[e] = (v[e] - mean) * rstd * g[e] + be[e];
                    if (k < K) {
                        if constexpr (DT == FLE_F32) *reinterpret_cast<f32x4 *>(reinterpret_cast<float *>(a.dst) + row * K + k) = f32x4{o[0], o[1], o[2], o[3]};
                        else st8_2byte(a.dst, row * K + k, dtype, o);
                    }
                }
            }
        }
        return;
    }
    if (a.vec && K <= 16384) {
        // (longer rows) one wave per row, three sweeps of 16-byte loads; the second and third find the row in the CU's own cache
        // (holding it in registers instead, 128 of them at 8192 elements, left one or two waves per SIMD and
        // nothing to cover the loads: 42 us against torch's 23 on 4096 x 4096)
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
        for (int64_t row = int64_t(blockIdx.x) * 4 + wave; row < a.M; row += int64_t(gridDim.x) * 4) {
            const char *src = reinterpret_cast<const char *>(a.x) + row * a.ldx * ES;
            float s = 0.0f;
#pragma unroll 4
            for (int64_t k = int64_t(lane) * W; k < K; k += 64 * W) {
                float v[8];
                unpack_vec<DT>(*reinterpret_cast<const u32x4 *>(src + k * ES), v);
#pragma unroll
                for (int e = 0; e < W; ++e) s += v[e];
            }
            const float mean = wave_allreduce_sum(s) / float(K);
            float m2 = 0.0f;
#pragma unroll 4
            for (int64_t k = int64_t(lane) * W; k < K; k += 64 * W) {
                float v[8];
                unpack_vec<DT>(*reinterpret_cast<const u32x4 *>(src + k * ES), v);
#pragma unroll
                for (int e = 0; e < W; ++e) m2 += (v[e] - mean) * (v[e] - mean);
            }
            const float rstd = rsqrtf(wave_allreduce_sum(m2) / float(K) + a.eps);
#pragma unroll 2
            for (int64_t k = int64_t(lane) * W; k < K; k += 64 * W) {
                float v[8], g[8], be[8], o[8];
                unpack_vec<DT>(*reinterpret_cast<const u32x4 *>(src + k * ES), v);
#pragma unroll
                for (int e = 0; e < 8; ++e) { g[e] = 1.0f; be[e] = 0.0f; }
                if (a.gamma) unpack_vec<DT>(*reinterpret_cast<const u32x4 *>(reinterpret_cast<const char *>(a.gamma) + k * ES), g);
                if (a.beta) unpack_vec<DT>(*reinterpret_cast<const u32x4 *>(reinterpret_cast<const char *>(a.beta) + k * ES), be);
#pragma unroll
                for (int e = 0; e < 8; ++e) o[e] = (v[e] - mean) * rstd * g[e] + be[e];
                if constexpr (DT == FLE_F32) *reinterpret_cast<f32x4 *>(reinterpret_cast<float *>(a.dst) + row * K + k) = f32x4{o[0], o[1], o[2], o[3]};
                else st8_2byte(a.dst, row * K + k, dtype, o);
            }
        }
        return;
    }
    for (int64_t row = blockIdx.x; row < a.M; row += gridDim.x) {
        const int64_t base = row * a.ldx;
        auto sweep = [&](auto &&f) {  // f(k, value) for this thread's elements of the row, in index order
            for (int64_t k = threadIdx.x; k < K; k += 256) f(k, ld_elem(a.x, base + k, dtype));
        };
        float s = 0.0f;
        sweep([&](int64_t, float v) { s += v; });
        const float mean = block_allreduce(s, false, lds) / float(K);
        float m2 = 0.0f;
        sweep([&](int64_t, float v) { m2 += (v - mean) * (v - mean); });
        const float rstd = rsqrtf(block_allreduce(m2, false, lds) / float(K) + a.eps);
        sweep([&](int64_t k, float v) {
            float o = (v - mean) * rstd;
            if (a.gamma) o *= ld_elem(a.gamma, k, dtype);
            if (a.beta) o += ld_elem(a.beta, k, dtype);
            st_elem(a.dst, row * K + k, dtype, o);
        });
    }
}

// ------------------------------------------------------------------ split-K reduction
// One wave per (row, 256-column chunk), a lane per 4 consecutive columns: sums the S fp32 slabs
// in slab order, applies the ops that precede the row op, writes the value (final, or staged
// for the finalize pass) and, with a row op, the chunk's partial.
template <bool MAX>
__device__ __forceinline__ float wave_allreduce(float v) {
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const float o = __shfl_xor(v, d);
        v = MAX ? fmaxf(v, o) : v + o;
    }
    return v;
}

__global__ __launch_bounds__(256) void reduce_slabs(const RedArgs a) {
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t N = a.N;
    const int dtype = a.epi.dtype;
    const bool f32 = dtype == FLE_F32;
    const bool vec = a.vec != 0;  // 4-column vector accesses to b, residual and dst are possible
    const int64_t chunks = (N + 255) / 256, items = a.M * chunks;
    for (int64_t item = int64_t(blockIdx.x) * 4 + wave; item < items; item += int64_t(gridDim.x) * 4) {
        const int64_t row = item / chunks, c0 = (item % chunks) * 256;
        const int64_t n = c0 + lane * 4;
        const bool ok = n < N;  // at least the first of this lane's four columns exists
        bool okc[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) okc[e] = n + e < N;
        f32x4 v = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
        if (ok) {
            const float *src = a.slabs + row * a.ld_slab + n;  // slab rows are padded to whole groups of four
            int s = 0;
            for (; s + 4 <= a.S; s += 4) {
                const f32x4 u0 = *reinterpret_cast<const f32x4 *>(src + (s + 0) * a.stride);
                const f32x4 u1 = *reinterpret_cast<const f32x4 *>(src + (s + 1) * a.stride);
                const f32x4 u2 = *reinterpret_cast<const f32x4 *>(src + (s + 2) * a.stride);
                const f32x4 u3 = *reinterpret_cast<const f32x4 *>(src + (s + 3) * a.stride);
                v = (((v + u0) + u1) + u2) + u3;
            }
            for (; s < a.S; ++s) v += *reinterpret_cast<const f32x4 *>(src + s * a.stride);
            auto add4 = [&](const void *ptr, int64_t idx) {
                if (vec) {
                    v += ld4_rt(ptr, idx, dtype);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (okc[e]) v[e] += ld_elem(ptr, idx + e, dtype);
                }
            };
            for (int o = 0; o < a.epi.n_pre; ++o) {
                const DevOp op = a.epi.pre[o];
                switch (op.kind) {
                case FLE_BIAS: add4(a.epi.bias, n); break;
                case FLE_SCALE: v *= op.alpha; break;
                case FLE_RELU:
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = relu_f(v[e]);
                    break;
                case FLE_GELU_ERF:
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = gelu_erf_f(v[e]);
                    break;
                case FLE_GELU_TANH:
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = gelu_tanh_f(v[e]);
                    break;
                case FLE_RESIDUAL: add4(op.p0, row * op.ld + n); break;
                case FLE_STORE: {  // a copy of the values as they stand, rounded to the dtype
                    void *tp = const_cast<void *>(op.p0);
                    if (!vec) {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (okc[e]) st_elem(tp, row * op.ld + n + e, dtype, v[e]);
                    } else if (f32) {
                        *reinterpret_cast<f32x4 *>(reinterpret_cast<float *>(tp) + row * op.ld + n) = v;
                    } else {
                        *reinterpret_cast<u32x2 *>(reinterpret_cast<uint16_t *>(tp) + row * op.ld + n) = pack4_rt(v, dtype);
                    }
                    break;
                }
                default: break;
                }
            }
        }
        if (a.epi.row_kind >= 0) {
            float s0, s1;
            if (a.epi.row_kind == FLE_LAYERNORM) {
                const float cnt = float(N - c0 < 256 ? N - c0 : 256);
                float sum = 0.0f;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (okc[e]) sum += v[e];
                const float mean = wave_allreduce<false>(sum) / cnt;
                float m2 = 0.0f;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (okc[e]) m2 += (v[e] - mean) * (v[e] - mean);
                s0 = mean;
                s1 = wave_allreduce<false>(m2);
            } else {
                float mx = -INFINITY;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (okc[e]) mx = fmaxf(mx, v[e]);
                mx = wave_allreduce<true>(mx);
                float se = 0.0f;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (okc[e]) se += __expf(v[e] - mx);
                s0 = mx;
                s1 = wave_allreduce<false>(se);
            }
            if (lane == 0) *reinterpret_cast<float2 *>(a.partials + (row * a.np + c0 / 256) * 2) = make_float2(s0, s1);
            if (a.dst_rel) v -= s0;
        }
        if (a.dst && ok) {
            const bool d32 = a.dst_f32 || f32;
            if (!vec) {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (okc[e]) st_elem(a.dst, row * a.ldd + n + e, d32 ? FLE_F32 : dtype, v[e]);
            } else if (d32) {
                *reinterpret_cast<f32x4 *>(reinterpret_cast<float *>(a.dst) + row * a.ldd + n) = v;
            } else {
                *reinterpret_cast<u32x2 *>(reinterpret_cast<uint16_t *>(a.dst) + row * a.ldd + n) = pack4_rt(v, dtype);
            }
        }
    }
}

}  // namespace fle
