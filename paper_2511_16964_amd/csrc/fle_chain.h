// A whole perceptron (a chain of Linear + bias + activation layers) at batch 1 in one persistent launch.
#pragma once
#include "fle_gemm_thin.h"

namespace fle {

constexpr int kChainMaxLayers = 16;

struct ChainLayer {
    const void *w;     // [n, k], packed rows
    const void *bias;  // [n] or nullptr
    int32_t n, k;
    int32_t act;       // -1, FLE_RELU, FLE_GELU_ERF or FLE_GELU_TANH
};

struct ChainArgs {
    int32_t n_layers;
    const void *x;     // [k of layer 0]
    void *out;         // [n of the last layer]
    void *act[kChainMaxLayers];  // act[l]: output of layer l < n_layers - 1 (storage dtype), every one a buffer of its own
    uint32_t *sync;    // grid barrier state (20 lines of 128 bytes, see chain_barrier); all zero between calls
    ChainLayer layer[kChainMaxLayers];
};

// Every layer is a matrix-vector product that streams its weight matrix once, exactly as the dot-product thin
// kernel does for a single layer: a wave owns one W row at a time and all of K, keeps two register batches of
// 2 KB of the row in flight, multiplies in fp32 and sums over its 64 lanes; lane 0 adds the bias, applies the
// activation and stores the element in the storage dtype.  What the single launch adds: the workgroups stay
// resident (at most one per CU, 58 registers per lane and no LDS, so all of them fit on the chip at once), a
// grid-wide barrier separates the layers, and the first weight batch of the next layer is requested before a
// workgroup enters that barrier, so the weight stream of layer l + 1 is already under way while the last
// workgroups finish layer l: the cost of draining and refilling the memory pipeline between two dependent
// launches is what bounds a 64 MB layer.
//
// The barrier: thread 0 of a workgroup counts itself in; the last arrival resets the counts and publishes the
// new generation, the others wait for it.  Nothing here flushes or invalidates a cache.  The activations are the
// only data that cross the barrier.  They are stored with device scope (written through to memory), and every
// storing wave waits for its own stores to be acknowledged (vmcnt(0)) before its workgroup arrives, so the order
// store -> arrive is explicit; relaxed device-scope atomics are then enough (a version with release / acquire
// fences, an L2 write-back and invalidation per workgroup and barrier, cost 30 us per layer).  They are loaded
// with ordinary cached loads: every layer writes a buffer of its own that no workgroup has read earlier in the
// launch, so no XCD's L2 can hold an older copy of a line; across launches the same holds because a kernel
// starts with clean (invalidated) L2s.  Every wait is bounded: a workgroup that gives up raises the error word,
// which ends all later waits at once, fills its share of the output with NaN and leaves, so the kernel always
// terminates, and a call whose workgroups were not all resident cannot be mistaken for a result.  The last
// workgroup to finish the kernel puts the counters and generations back to zero (the error word stays).
constexpr uint32_t kChainSpinLimit = 1u << 21;

// st: 32-bit words, one 128-byte line each: line 0 = arrivals of the group leaders, line 1 = finished workgroups,
// line 2 = error, lines 4 .. 11 = arrivals within group g, lines 12 .. 19 = generation as seen by group g.
// Two levels, because device-scope atomics on one address are served one after another (256 arrivals on one
// counter cost about 10 us): a workgroup arrives at its group's counter (group = workgroup index mod 8), the
// last of a group arrives at the top counter, the last of those publishes the new generation to every group.
constexpr int kChainGroups = 8;
__device__ __forceinline__ uint32_t *chain_word(uint32_t *st, int line) { return st + line * 32; }

// Returns false (to every thread of the workgroup) if the wait was given up.
__device__ __forceinline__ bool chain_barrier(uint32_t *st, uint32_t n_wg, uint32_t target_gen) {
    int gave_up = 0;
    __syncthreads();  // every wave of the workgroup has waited for its activation stores (see the caller)
    if (threadIdx.x == 0) {
        const int g = int(blockIdx.x) % kChainGroups;
        const uint32_t n_groups = n_wg < uint32_t(kChainGroups) ? n_wg : uint32_t(kChainGroups);
        const uint32_t in_group = (n_wg - uint32_t(g) + kChainGroups - 1) / kChainGroups;  // workgroups with this index mod 8
        bool release = false;
        if (__hip_atomic_fetch_add(chain_word(st, 4 + g), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == in_group - 1) {
            __hip_atomic_store(chain_word(st, 4 + g), 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (__hip_atomic_fetch_add(chain_word(st, 0), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == n_groups - 1) {
                __hip_atomic_store(chain_word(st, 0), 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                release = true;
            }
        }
        if (release) {
            __builtin_amdgcn_s_waitcnt(0);  // the resets are out before anybody can arrive again
            for (uint32_t q = 0; q < n_groups; ++q)
                __hip_atomic_store(chain_word(st, 12 + int(q)), target_gen, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        } else {
            uint32_t spins = 0;
            while (__hip_atomic_load(chain_word(st, 12 + g), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target_gen) {
                if (++spins > kChainSpinLimit || __hip_atomic_load(chain_word(st, 2), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) {
                    __hip_atomic_store(chain_word(st, 2), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    gave_up = 1;
                    break;
                }
                __builtin_amdgcn_s_sleep(1);
            }
        }
    }
    return __syncthreads_or(gave_up) == 0;
}

// One element of an activation vector, stored with device scope (written through, visible to every XCD).
template <int DT>
__device__ __forceinline__ void store_activation(void *dst, int64_t i, float v) {
    if constexpr (DT == FLE_F32) {
        __hip_atomic_store(reinterpret_cast<uint32_t *>(dst) + i, __float_as_uint(v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    } else {
        uint16_t bits;
        if constexpr (DT == FLE_F16) bits = __builtin_bit_cast(uint16_t, static_cast<_Float16>(v));
        else bits = __builtin_bit_cast(uint16_t, static_cast<__bf16>(v));
        __hip_atomic_store(reinterpret_cast<uint16_t *>(dst) + i, bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// DT: dtype of the activations, biases and the output; DW: dtype of the weights (DT, or a 2-byte dtype under
// fp32 activations: reduced-precision weights halve the bytes that bound this kernel).
template <int DT, int DW>
__global__ __launch_bounds__(1024) void mlp_chain(const ChainArgs a) {
    static_assert(DW == DT || (DT == FLE_F32 && DW != FLE_F32), "weights in the activations' dtype, or 2-byte weights under fp32");
    constexpr int ES = DW == FLE_F32 ? 4 : 2;   // bytes per weight
    constexpr int EX = DT == FLE_F32 ? 4 : 2;   // bytes per activation
    constexpr int XW = EX / ES;                 // 16-byte pieces of x that go with 16 bytes of W
    constexpr int D = 2;  // 1 KB blocks of a row per register batch
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    struct Batch {
        u32x4 w[D], x[D][XW];
    };
    // the first row of this wave in a layer, its buffer resource, and the loads of K blocks j D .. j D + D - 1
    auto w_rsrc = [&](const ChainLayer &L, int row) {
        const bool live = row < L.n;
        return __builtin_amdgcn_make_buffer_rsrc(
            const_cast<char *>(reinterpret_cast<const char *>(L.w) + (live ? int64_t(row) * L.k * ES : 0)), 0,
            live ? uint32_t(L.k * ES) : 0u, 0x00020000);
    };
    auto load_w = [&](Batch &b, const __amdgpu_buffer_rsrc_t &rw, uint32_t kbytes, uint32_t j) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            const uint32_t col = (j * D + d) * 1024 + uint32_t(lane) * 16;
            b.w[d] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rw, col < kbytes ? col : 0x80000000u, 0, 2));
        }
    };
    // the x elements that go with W bytes col .. col + 15 start at byte col * XW
    auto load_x = [&](Batch &b, const __amdgpu_buffer_rsrc_t &rx, uint32_t kbytes, uint32_t j) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            const uint32_t col = (j * D + d) * 1024 + uint32_t(lane) * 16;
#pragma unroll
            for (int h = 0; h < XW; ++h)
                b.x[d][h] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rx, col < kbytes ? col * XW + 16 * h : 0x80000000u, 0, 0));
        }
    };

    Batch b0, b1;
    bool have_w0 = false;  // b0.w and b1.w already hold the first two weight batches of this wave's first row of the layer
    for (int l = 0; l < a.n_layers; ++l) {
        const ChainLayer &L = a.layer[l];
        const void *src = l == 0 ? a.x : a.act[l - 1];
        void *dst = l + 1 == a.n_layers ? a.out : a.act[l];
        const uint32_t kbytes = uint32_t(L.k) * ES;  // of a W row
        const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(src), 0, uint32_t(L.k) * EX, 0x00020000);
        const uint32_t blocks = (kbytes + 1023) / 1024, batches = (blocks + D - 1) / D;
        for (int row = int(blockIdx.x) * 16 + wave; row < L.n; row += int(gridDim.x) * 16) {
            const __amdgpu_buffer_rsrc_t rw = w_rsrc(L, row);
            if (!have_w0) load_w(b0, rw, kbytes, 0);
            const bool have_w1 = have_w0;
            have_w0 = false;
            load_x(b0, rx, kbytes, 0);
            float acc = 0.0f;
            auto multiply = [&](const Batch &b) {
#pragma unroll
                for (int d = 0; d < D; ++d) {
                    const Unpacked<DW> w = unpack16<DW>(b.w[d]);
                    if constexpr (XW == 1) {
                        const Unpacked<DT> x = unpack16<DT>(b.x[d][0]);
#pragma unroll
                        for (int e = 0; e < (DW == FLE_F32 ? 4 : 8); ++e) acc = fmaf(w.v[e], x.v[e], acc);
                    } else {  // 8 two-byte weights against 8 fp32 activations
#pragma unroll
                        for (int e = 0; e < 8; ++e) acc = fmaf(w.v[e], __uint_as_float(b.x[d][e / 4][e % 4]), acc);
                    }
                }
            };
            for (uint32_t j = 0; j < batches; j += 2) {
                if (!(have_w1 && j == 0)) load_w(b1, rw, kbytes, j + 1);
                load_x(b1, rx, kbytes, j + 1);
                __builtin_amdgcn_sched_barrier(0);
                multiply(b0);
                __builtin_amdgcn_sched_barrier(0);
                load_w(b0, rw, kbytes, j + 2);
                load_x(b0, rx, kbytes, j + 2);
                __builtin_amdgcn_sched_barrier(0);
                multiply(b1);
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) acc += __shfl_xor(acc, d);
            if (lane == 0) {
                float v = acc;
                if (L.bias) v += ld_elem(L.bias, row, DT);
                if (L.act == FLE_RELU) v = relu_f(v);
                else if (L.act == FLE_GELU_ERF) v = gelu_erf_f(v);
                else if (L.act == FLE_GELU_TANH) v = gelu_tanh_f(v);
                if (l + 1 == a.n_layers) st_elem(dst, row, DT, v);
                else store_activation<DT>(dst, row, v);
            }
        }
        if (l + 1 < a.n_layers) {
            // this wave's activation stores have reached memory before its workgroup arrives at the barrier
            // (and before the loads below, which stay in flight across it, join the same counter)
            wait_vmcnt<0>();
            // request the first two weight batches of the next layer's first row before waiting for the other workgroups
            const ChainLayer &Ln = a.layer[l + 1];
            const int row = int(blockIdx.x) * 16 + wave;
            if (row < Ln.n) {
                const __amdgpu_buffer_rsrc_t rn = w_rsrc(Ln, row);
                load_w(b0, rn, uint32_t(Ln.k) * ES, 0);
                load_w(b1, rn, uint32_t(Ln.k) * ES, 1);
                have_w0 = true;
            }
            if (!chain_barrier(a.sync, gridDim.x, uint32_t(l + 1))) {  // layer l is complete and visible everywhere, or:
                // the wait was given up: this workgroup's share of the result becomes NaN and it computes no further
                const ChainLayer &Le = a.layer[a.n_layers - 1];
                if (lane == 0)
                    for (int row = int(blockIdx.x) * 16 + wave; row < Le.n; row += int(gridDim.x) * 16) st_elem(a.out, row, DT, __builtin_nanf(""));
                break;
            }
        }
    }
    // the last workgroup to get here puts the barrier state back to zero (the error word stays if raised)
    if (threadIdx.x == 0 && a.n_layers > 1) {
        if (__hip_atomic_fetch_add(chain_word(a.sync, 1), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == gridDim.x - 1) {
            __hip_atomic_store(chain_word(a.sync, 1), 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(chain_word(a.sync, 0), 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            for (int q = 0; q < kChainGroups; ++q) {
                __hip_atomic_store(chain_word(a.sync, 4 + q), 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(chain_word(a.sync, 12 + q), 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
}

}  // namespace fle
