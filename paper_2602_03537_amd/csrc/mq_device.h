// Device-side pieces shared by the vector-ALU kernel (mq_linear.hip) and the
// MFMA kernel (mq_gemm.hip): the persistent schedule over all tiles of a stack
// and the deterministic split-K hand-off.
//
// Schedule.  ("wavefront w" below is a schedule share, a "worker": a wave may serve several.)
// A layer is CB x RB x G tiles (column chunk, row block of 64 rows,
// group of 128 columns; CB = 1 unless the batch is served 16 columns at a time).
// Tiles of all layers form one line in "cost" space (cost ~ bytes of a tile);
// wavefront w owns the tiles whose start lies in [w*C/W, (w+1)*C/W): a
// contiguous run, group index fastest, i.e. a contiguous piece of packed
// memory, while the wave keeps fp32 running sums for its current row block.
//
// Split-K.  When a run ends inside a row block the wave leaves its partial sums
// in a slot of its own and adds the number of groups it covered to the row
// block's counter; whoever brings the counter to G adds the slots up in wave
// order (so the result does not depend on timing), writes y and resets the
// counter.  Nobody waits for anybody.
#pragma once
#include "mq_internal.h"
#include "mq_static_for.h"

namespace mq {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// Pointers inside LayerDesc arrive as plain 64-bit values, so the compiler would treat
// them as generic ("flat") addresses, whose loads cannot be counted separately from LDS
// traffic and force full waits.  Everything here lives in global memory: say so.
#define MQ_GLOBAL __attribute__((address_space(1)))
#define MQ_LDS __attribute__((address_space(3)))
template <class T> __device__ __forceinline__ const T MQ_GLOBAL *gl(const T *p) { return (const T MQ_GLOBAL *)p; }
template <class T> __device__ __forceinline__ T MQ_GLOBAL *gl(T *p) { return (T MQ_GLOBAL *)p; }
typedef const uint32_t __attribute__((address_space(4))) *cptr32;  // scalar (SGPR) loads

__device__ __forceinline__ cptr32 as_const(const void *p) { return (cptr32)(uintptr_t)p; }

// bf16 activations and outputs (LayerDesc::flags).  A bf16 value inside the fp16 range is an fp16 value with mantissa
// bits to spare, so activations are converted where they are consumed and every product stays exact; beyond +-65504
// they become infinities, below 2^-14 they keep what fp16 subnormals can hold.  Outputs are the fp32 sums rounded to
// nearest even in the type asked for.
constexpr int kFlagXBf16 = 1, kFlagYBf16 = 2;
__device__ __forceinline__ uint32_t bf16_pair_to_f16_pair(uint32_t v) {
    const float lo = __builtin_bit_cast(float, v << 16), hi = __builtin_bit_cast(float, v & 0xFFFF0000u);
    const half2_t h = {(_Float16)lo, (_Float16)hi};
    return __builtin_bit_cast(uint32_t, h);
}
// (for the activation prep kernels of the matrix-core paths, where the conversion costs nothing that matters; the
// vector-ALU kernels read activations that xcvt_kernel has converted ahead of them: computed both ways and selected per
// tile, the conversion costs the ALU-bound 2-bit tiles 3 %, branched around 10 %)
__device__ __forceinline__ uint32_t x_pair(uint32_t v, int flags) { return flags & kFlagXBf16 ? bf16_pair_to_f16_pair(v) : v; }

__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
    uint32_t b = __builtin_bit_cast(uint32_t, f);
    if ((b & 0x7F800000u) == 0x7F800000u) return (uint16_t)((b >> 16) | ((b & 0xFFFFu) ? 0x40u : 0u));  // Inf, NaN stays NaN
    b += 0x7FFFu + ((b >> 16) & 1u);
    return (uint16_t)(b >> 16);
}
// the 16 bits stored for output value v
__device__ __forceinline__ uint16_t y_bits(float v, int flags) {
    return flags & kFlagYBf16 ? f32_to_bf16_bits(v) : __builtin_bit_cast(uint16_t, (_Float16)v);
}
__device__ __forceinline__ void store_y(_Float16 *y, size_t idx, float v, int flags) {
    gl(reinterpret_cast<uint16_t *>(y))[idx] = y_bits(v, flags);
}

__device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float c) {
    return __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, a), __builtin_bit_cast(half2_t, b), c, false);
}

template <int CTRL> __device__ __forceinline__ float dpp_add(float v) {
    const int t = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false);
    return v + __builtin_bit_cast(float, t);
}
// Sum over the 64 lanes, result in every lane.
__device__ __forceinline__ float wave_sum(float v) {
    v = dpp_add<0xB1>(v);   // quad_perm [1,0,3,2]
    v = dpp_add<0x4E>(v);   // quad_perm [2,3,0,1]
    v = dpp_add<0x141>(v);  // row_half_mirror
    v = dpp_add<0x140>(v);  // row_mirror: every lane of a 16-lane row holds the row total
    v += __shfl_xor(v, 16);
    v += __shfl_xor(v, 32);
    return v;
}

__device__ __forceinline__ LayerDesc load_desc(const LayerDesc *p) {
    constexpr int ND = sizeof(LayerDesc) / 4;
    static_assert(sizeof(LayerDesc) % 4 == 0, "descriptor is read as dwords");
    uint32_t w[ND];
    cptr32 c = as_const(p);
#pragma unroll
    for (int i = 0; i < ND; ++i) w[i] = c[i];
    LayerDesc d;
    __builtin_memcpy(&d, w, sizeof(d));
    return d;
}

// wave that owns the tile starting at cost position pos
__device__ __forceinline__ int wave_of(uint64_t pos, uint64_t nw, uint64_t ctot) {
    return (int)(((pos + 1) * nw - 1) / ctot);
}

// Walk the tiles of schedule share `worker`: f(L, u_begin, u_end) is called once per layer
// the share touches, with tile indices in [0, CB*RB*G) of that layer.
template <class F> __device__ __forceinline__ void walk_tiles(const StackParams &p, int worker, F &&f) {
    const uint64_t b_lo = (uint64_t)worker * p.cost_total / (uint64_t)p.nworkers;
    const uint64_t b_hi = (uint64_t)(worker + 1) * p.cost_total / (uint64_t)p.nworkers;
    int li = 0;
    if (p.table) {  // last layer whose cost_start <= b_lo
        int lo = 0, hi = p.n_layers - 1;
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            const uint64_t cs = load_desc(p.table + mid).cost_start;
            if (cs <= b_lo) lo = mid; else hi = mid - 1;
        }
        li = lo;
    }
    uint64_t pos = b_lo;
    while (li < p.n_layers) {
        const LayerDesc L = p.table ? load_desc(p.table + li) : p.single;
        const uint64_t layer_end = L.cost_start + (uint64_t)L.CB * L.RB * L.G * L.cost;
        if (pos < layer_end) {
            const uint64_t hi = b_hi < layer_end ? b_hi : layer_end;
            const int u_begin = (int)((pos - L.cost_start + L.cost - 1) / L.cost);
            const int u_end = (int)((hi - L.cost_start + L.cost - 1) / L.cost);
            if (u_begin < u_end) f(L, u_begin, u_end);
        }
        if (b_hi <= layer_end) break;
        pos = layer_end;
        ++li;
    }
}

// End of a wave's run inside row block (chunk c, rb): groups [ga, gb) are in acc[NV] (per lane).
// Complete row block -> final(acc).  Otherwise publish the partial sums; the last
// contributor sums all slots in wave order and calls final(total).
//   cnt     : the row block's counter
//   a       : cost position of the row block's first tile
// Partial sums travel through agent-scope atomic stores/loads (write-through, cache
// bypassing), so no whole-L2 write-back or invalidate is needed to publish them.
template <int NV, class Final>
__device__ __forceinline__ void finish_row_block(const LayerDesc &L, const StackParams &p, int32_t *cnt, uint64_t a,
                                                 int ga, int gb, float (&acc)[NV], int worker, int lane, Final &&final) {
    if (ga == 0 && gb == L.G) {
        final(acc);
        return;
    }
    const int slot = ga == 0 ? 1 : 0;  // the wave holding a row block's first tile uses slot 1
    const size_t slot_floats = (size_t)p.slot_floats;
    float MQ_GLOBAL *mine = gl(p.part + (size_t)(worker * 2 + slot) * slot_floats + lane);
#pragma unroll
    for (int v = 0; v < NV; ++v) __hip_atomic_store(mine + v * 64, acc[v], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    // the write-through stores must have been acknowledged before the counter moves
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    int old = 0;
    if (lane == 0) old = __hip_atomic_fetch_add(gl(cnt), gb - ga, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    old = __builtin_amdgcn_readfirstlane(old);
    if (old + (gb - ga) != L.G) return;
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    const int w_lo = wave_of(a, p.nworkers, p.cost_total);
    const int w_hi = wave_of(a + (uint64_t)(L.G - 1) * L.cost, p.nworkers, p.cost_total);
    // Fixed summation order (w_lo's slot 1, then slot 0 of w_lo+1 .. w_hi); loads are issued
    // in batches so that their round trips overlap.
    constexpr int kBatch = NV >= 8 ? 8 : 16;  // slots fetched per round trip (NV * kBatch registers)
    float tot[NV];
    const float MQ_GLOBAL *first = gl(p.part + (size_t)(w_lo * 2 + 1) * slot_floats + lane);
#pragma unroll
    for (int v = 0; v < NV; ++v) tot[v] = __hip_atomic_load(first + v * 64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    for (int w0 = w_lo + 1; w0 <= w_hi; w0 += kBatch) {
        float t[kBatch][NV];
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
            const int w = w0 + j <= w_hi ? w0 + j : w_hi;
            const float MQ_GLOBAL *src = gl(p.part + (size_t)(w * 2) * slot_floats + lane);
#pragma unroll
            for (int v = 0; v < NV; ++v)
                t[j][v] = __hip_atomic_load(src + v * 64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
#pragma unroll
        for (int j = 0; j < kBatch; ++j)
            if (w0 + j <= w_hi) {
#pragma unroll
                for (int v = 0; v < NV; ++v) tot[v] += t[j][v];
            }
    }
    final(tot);
    if (lane == 0) __hip_atomic_store(gl(cnt), 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

}  // namespace mq
