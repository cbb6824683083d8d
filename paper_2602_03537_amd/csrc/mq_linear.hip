// Sliced, group-dequantised linear layer  y = x * W_D^T  (Section 4 of the paper)
// for batch sizes served by the vector ALUs (M <= 4), and the mixed-precision
// stack of such layers (Section 3.3), as ONE persistent kernel.  Schedule and
// split-K hand-off: mq_device.h.
//
// Arithmetic per tile and lane (one row, one group g):
//   D   = sum_k x[k] * t[k]            t = r-bit code, via fp16-subnormal fields
//   y  += scale * (2^(8-r) * D - zero * X_g),   X_g = sum_{k in g} x[k]
// which is  sum_k x[k] * scale * (S[k] - zero)  with S = t * 2^(8-r)  (Eq. 1's
// rescale), the zero-offset and scale applied once per group instead of per weight.
#include "mq_device.h"

namespace mq {

template <int R> struct TileRegs {
    uint32_t w[4 * R];
    _Float16 s, z;
};

template <int R> __device__ __forceinline__ void load_tile(TileRegs<R> &t, const LayerDesc &L, int u, int lane) {
    const u32x4 MQ_GLOBAL *src = gl(reinterpret_cast<const u32x4 *>(L.Wp) + (size_t)u * (R * 64) + lane);
#pragma unroll
    for (int i = 0; i < R; ++i) {
        const u32x4 v = src[i * 64];
        t.w[4 * i] = v.x; t.w[4 * i + 1] = v.y; t.w[4 * i + 2] = v.z; t.w[4 * i + 3] = v.w;
    }
    t.s = gl(L.st)[(size_t)u * 64 + lane];
    t.z = gl(L.zt)[(size_t)u * 64 + lane];
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
        const uint32_t xl = gl(reinterpret_cast<const uint32_t *>(xrow))[lane];
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
            const int row = rb * kRowBlock + lane;
            finish_row_block<M>(L, p, p.cnt + L.cnt_off + rb, L.cost_start + (uint64_t)rb * L.G * L.cost, ga, g, yacc,
                                wave, lane, [&](const float(&tot)[M]) {
#pragma unroll
                                    for (int m = 0; m < M; ++m)
                                        if (row < L.N) gl(L.y)[(size_t)m * L.N + row] = (_Float16)tot[m];
                                });
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
    walk_tiles(p, wave, [&](const LayerDesc &L, int u_begin, int u_end) {
        switch (L.r) {
            case 2: run_units<2, M>(L, p, u_begin, u_end, wave, lane); break;
            case 3: run_units<3, M>(L, p, u_begin, u_end, wave, lane); break;
            case 4: run_units<4, M>(L, p, u_begin, u_end, wave, lane); break;
            case 6: run_units<6, M>(L, p, u_begin, u_end, wave, lane); break;
            default: run_units<8, M>(L, p, u_begin, u_end, wave, lane); break;
        }
    });
}

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
