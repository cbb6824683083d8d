// Sliced, group-dequantised linear layer  y = x * W_D^T  (Section 4 of the paper)
// for batch sizes served by the vector ALUs, and the mixed-precision stack of
// such layers (Section 3.3), as ONE persistent kernel.
//
// Work decomposition.  A layer is RB x G tiles (64 rows x one group of 128
// columns, mq_layout.h).  Tiles of all layers form one line in "cost" space
// (cost ~ bytes of a tile); wavefront w owns the tiles whose start lies in
// [w*C/W, (w+1)*C/W), i.e. a contiguous run of tiles, group index fastest, so a
// wave streams a contiguous piece of packed memory and keeps one fp32 running
// sum per row (lane) while it walks along K.  When a run ends inside a row block
// the wave leaves its partial sums in a slot of its own and bumps the row
// block's counter; whoever brings the counter to G adds the slots up in wave
// order (so the result does not depend on timing) and writes y.  Nobody waits.
//
// Arithmetic per tile and lane (one row, one group g):
//   D   = sum_k x[k] * t[k]            t = r-bit code, via fp16-subnormal fields
//   y  += scale * (2^(8-r) * D - zero * X_g),   X_g = sum_{k in g} x[k]
// which is  sum_k x[k] * scale * (S[k] - zero)  with S = t * 2^(8-r)  (Eq. 1's
// rescale), the zero-offset and scale applied once per group instead of per weight.
#include "mq_internal.h"
#include "mq_static_for.h"

namespace mq {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef const uint32_t __attribute__((address_space(4))) *cptr32;  // scalar (SGPR) loads

__device__ __forceinline__ cptr32 as_const(const void *p) { return (cptr32)(uintptr_t)p; }

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

template <int R> struct TileRegs {
    uint32_t w[4 * R];
    _Float16 s, z;
};

template <int R> __device__ __forceinline__ void load_tile(TileRegs<R> &t, const LayerDesc &L, int u, int lane) {
    const uint4 *src = L.Wp + (size_t)u * (R * 64) + lane;
#pragma unroll
    for (int i = 0; i < R; ++i) {
        const uint4 v = src[i * 64];
        t.w[4 * i] = v.x; t.w[4 * i + 1] = v.y; t.w[4 * i + 2] = v.z; t.w[4 * i + 3] = v.w;
    }
    t.s = L.st[(size_t)u * 64 + lane];
    t.z = L.zt[(size_t)u * 64 + lane];
}

// Partial or complete result of a row block: store / combine (see file header).
template <int M>
__device__ __forceinline__ void flush_rows(const LayerDesc &L, const StackParams &p, int rb, int ga, int gb,
                                           const float (&yacc)[M], int wave, int lane) {
    const int row = rb * kRowBlock + lane;
    if (ga == 0 && gb == L.G) {
#pragma unroll
        for (int m = 0; m < M; ++m)
            if (row < L.N) L.y[(size_t)m * L.N + row] = (_Float16)yacc[m];
        return;
    }
    const int slot = ga == 0 ? 1 : 0;  // the wave holding a row block's first tile uses slot 1
    // Partial sums travel through agent-scope atomic stores/loads (write-through, cache
    // bypassing), so no whole-L2 write-back or invalidate is needed to publish them.
    float *mine = p.part + ((size_t)(wave * 2 + slot) * M) * 64 + lane;
#pragma unroll
    for (int m = 0; m < M; ++m) __hip_atomic_store(mine + m * 64, yacc[m], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    // the write-through stores must have been acknowledged before the counter moves
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    int old = 0;
    int32_t *cnt = p.cnt + L.cnt_off + rb;
    if (lane == 0) old = __hip_atomic_fetch_add(cnt, gb - ga, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    old = __builtin_amdgcn_readfirstlane(old);
    if (old + (gb - ga) != L.G) return;
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    const uint64_t a = L.cost_start + (uint64_t)rb * L.G * L.cost;
    const int w_lo = wave_of(a, p.nwaves, p.cost_total);
    const int w_hi = wave_of(a + (uint64_t)(L.G - 1) * L.cost, p.nwaves, p.cost_total);
    // Fixed summation order (w_lo's slot 1, then slot 0 of w_lo+1 .. w_hi); loads are issued
    // in batches so that their round trips overlap.
    constexpr int kBatch = 16;
#pragma unroll
    for (int m = 0; m < M; ++m) {
        float tot = __hip_atomic_load(p.part + ((size_t)(w_lo * 2 + 1) * M + m) * 64 + lane, __ATOMIC_RELAXED,
                                      __HIP_MEMORY_SCOPE_AGENT);
        for (int w0 = w_lo + 1; w0 <= w_hi; w0 += kBatch) {
            float v[kBatch];
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
                const int w = w0 + j <= w_hi ? w0 + j : w_hi;
                v[j] = __hip_atomic_load(p.part + ((size_t)(w * 2) * M + m) * 64 + lane, __ATOMIC_RELAXED,
                                         __HIP_MEMORY_SCOPE_AGENT);
            }
#pragma unroll
            for (int j = 0; j < kBatch; ++j)
                if (w0 + j <= w_hi) tot += v[j];
        }
        if (row < L.N) L.y[(size_t)m * L.N + row] = (_Float16)tot;
    }
    if (lane == 0) __hip_atomic_store(cnt, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int R, int M>
__device__ __forceinline__ void tile_math(const TileRegs<R> &t, const LayerDesc &L, int g, int lane, float (&yacc)[M]) {
    using T = Layout<R>;
    constexpr int NU = 4 * R / T::UD;
    float xg[M];
    cptr32 xs[M];
#pragma unroll
    for (int m = 0; m < M; ++m) {
        const _Float16 *xrow = L.x + (size_t)m * L.K + (size_t)g * kGroup;
        const uint32_t xl = reinterpret_cast<const uint32_t *>(xrow)[lane];
        xg[m] = wave_sum(dot2(xl, 0x3C003C00u, 0.f));  // (1.0, 1.0)
        xs[m] = as_const(xrow);
    }
    float acc[M][T::NKEYS];
#pragma unroll
    for (int m = 0; m < M; ++m)
#pragma unroll
        for (int k = 0; k < T::NKEYS; ++k) acc[m][k] = 0.f;

    static_for<NU>([&](auto un) {
        static_for<T::NOPS>([&](auto oi) {
            constexpr Op o = T::op(oi);
            constexpr int key = key_index<R>(oi);
            uint32_t v = t.w[un * T::UD + o.dw];
            if constexpr (o.sh != 0) v >>= o.sh;
            v &= (uint32_t)o.mask * 0x10001u;
#pragma unroll
            for (int m = 0; m < M; ++m) acc[m][key] = dot2(v, xs[m][un * T::PPU + o.pair], acc[m][key]);
        });
    });
    const float s = (float)t.s, z = (float)t.z;
#pragma unroll
    for (int m = 0; m < M; ++m) {
        float d = 0.f;
        static_for<T::NKEYS>([&](auto k) {
            // field value = digit * 2^(key-24); back to code units, then Eq. 1's rescale 2^(8-r)
            d = fmaf(acc[m][k], __builtin_ldexpf(1.f, 24 - T::key(k) + kC - R), d);
        });
        yacc[m] = fmaf(s, fmaf(-z, xg[m], d), yacc[m]);
    }
}

// Tiles [u_begin, u_end) of one layer, owned by this wave.
template <int R, int M>
__device__ __forceinline__ void run_units(const LayerDesc &L, const StackParams &p, int u_begin, int u_end, int wave,
                                          int lane) {
    int rb = u_begin / L.G;
    int g = u_begin - rb * L.G;
    int ga = g;
    float yacc[M];
#pragma unroll
    for (int m = 0; m < M; ++m) yacc[m] = 0.f;

    TileRegs<R> cur, nxt;
    load_tile<R>(cur, L, u_begin, lane);
    for (int u = u_begin; u < u_end; ++u) {
        if (u + 1 < u_end) load_tile<R>(nxt, L, u + 1, lane);
        tile_math<R, M>(cur, L, g, lane, yacc);
        ++g;
        if (g == L.G || u + 1 == u_end) {
            flush_rows<M>(L, p, rb, ga, g, yacc, wave, lane);
            ++rb;
            g = 0;
            ga = 0;
#pragma unroll
            for (int m = 0; m < M; ++m) yacc[m] = 0.f;
        }
        cur = nxt;
    }
}

template <int M> __global__ __launch_bounds__(256) void stack_kernel(const StackParams p) {
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)((blockIdx.x * blockDim.x + threadIdx.x) >> 6));
    if (wave >= p.nwaves) return;
    const uint64_t b_lo = (uint64_t)wave * p.cost_total / (uint64_t)p.nwaves;
    const uint64_t b_hi = (uint64_t)(wave + 1) * p.cost_total / (uint64_t)p.nwaves;

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
        const uint64_t layer_end = L.cost_start + (uint64_t)L.RB * L.G * L.cost;
        if (pos < layer_end) {
            const uint64_t hi = b_hi < layer_end ? b_hi : layer_end;
            const int u_begin = (int)((pos - L.cost_start + L.cost - 1) / L.cost);
            const int u_end = (int)((hi - L.cost_start + L.cost - 1) / L.cost);
            if (u_begin < u_end) {
                switch (L.r) {
                    case 2: run_units<2, M>(L, p, u_begin, u_end, wave, lane); break;
                    case 3: run_units<3, M>(L, p, u_begin, u_end, wave, lane); break;
                    case 4: run_units<4, M>(L, p, u_begin, u_end, wave, lane); break;
                    case 6: run_units<6, M>(L, p, u_begin, u_end, wave, lane); break;
                    default: run_units<8, M>(L, p, u_begin, u_end, wave, lane); break;
                }
            }
        }
        if (b_hi <= layer_end) break;
        pos = layer_end;
        ++li;
    }
}

bool linear_supports_m(int64_t M) { return M >= 1 && M <= 4; }

template <int M> static int resident_waves() {
    static int cached = 0;
    if (cached) return cached;
    int dev = 0, cus = 0, blocks = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&blocks, stack_kernel<M>, 256, 0) != hipSuccess) return 0;
    if (blocks < 1) blocks = 1;
    int w = cus * blocks * 4;
    if (w > kMaxWaves) w = kMaxWaves;
    cached = w;
    return w;
}

template <int M> static hipError_t launch_stack_m(StackParams p, int max_cost, hipStream_t s) {
    int hw = resident_waves<M>();
    if (hw <= 0) return hipErrorUnknown;
    // every wave's share must be at least one tile long, so that each wave between the
    // first and last contributor of a row block really owns a tile of it
    uint64_t cap = p.cost_total / (uint64_t)max_cost;
    if (cap < 1) cap = 1;
    p.nwaves = (int)(cap < (uint64_t)hw ? cap : (uint64_t)hw);
    const unsigned blocks = (unsigned)((p.nwaves + 3) / 4);
    (void)hipGetLastError();  // drop stale errors of earlier, unrelated calls
    hipLaunchKernelGGL(stack_kernel<M>, dim3(blocks), dim3(256), 0, s, p);
    return hipGetLastError();
}

hipError_t launch_stack(StackParams p, int max_cost, hipStream_t s) {
    switch (p.M) {
        case 1: return launch_stack_m<1>(p, max_cost, s);
        case 2: return launch_stack_m<2>(p, max_cost, s);
        case 3: return launch_stack_m<3>(p, max_cost, s);
        case 4: return launch_stack_m<4>(p, max_cost, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace mq
