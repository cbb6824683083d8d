// Slice, pack, unpack and meta re-tiling kernels (load-time steps of the path), and the
// run-time re-slice of a resident parent.
//   slice   : Eq. 1 (Section 2), elementwise on bytes
//   pack    : Section 4's offline reorder, into the tile layout of mq_layout.h
//   reslice : Eq. 1 + pack on a parent that is already in the tile layout (8-bit pack)
#include "mq_internal.h"
#include "mq_static_for.h"

namespace mq {

// ------------------------------------------------------------------ slice
// Eq. 1 with round-half-up: t = min((q + 2^(c-r-1)) >> (c-r), 2^r - 1); S = t << (c-r).
__device__ __forceinline__ uint32_t slice_byte(uint32_t q, int cmask, int sh, int half, int tmax) {
    q &= cmask;
    uint32_t t = (q + half) >> sh;
    t = t < (uint32_t)tmax ? t : (uint32_t)tmax;
    return t << sh;
}

// in == out (in place) is allowed: every element is read and then written by the same lane.
__global__ __launch_bounds__(256) void slice_kernel(const uint8_t *in, uint8_t *out, int64_t n, int cmask, int sh, int half,
                                                    int tmax, int vec) {
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    int64_t nvec = vec ? n / 16 : 0;
    for (int64_t i = tid; i < nvec; i += stride) {
        uint4 v = reinterpret_cast<const uint4 *>(in)[i];
        uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint32_t o = 0;
#pragma unroll
            for (int b = 0; b < 4; ++b) o |= slice_byte((w[j] >> (8 * b)) & 0xFF, cmask, sh, half, tmax) << (8 * b);
            w[j] = o;
        }
        reinterpret_cast<uint4 *>(out)[i] = make_uint4(w[0], w[1], w[2], w[3]);
    }
    for (int64_t i = nvec * 16 + tid; i < n; i += stride) out[i] = (uint8_t)slice_byte(in[i], cmask, sh, half, tmax);
}

hipError_t launch_slice(const uint8_t *parent, int64_t n, int c, int r, uint8_t *out, hipStream_t s) {
    if (n == 0) return hipSuccess;
    const int sh = c - r;
    const int half = sh ? (1 << (sh - 1)) : 0;
    const int vec = ((reinterpret_cast<uintptr_t>(parent) | reinterpret_cast<uintptr_t>(out)) & 15) == 0;
    int64_t work = vec ? (n + 15) / 16 : n;
    int64_t blocks = (work + 255) / 256;
    if (blocks > 256 * 64) blocks = 256 * 64;
    return launch(slice_kernel, dim3((unsigned)blocks), dim3(256), 0, s, parent, out, n, (1 << c) - 1, sh, half,
                  (1 << r) - 1, vec);
}

// ------------------------------------------------------------------ pack
// One thread per (row block, group, lane): reads its row's 128 codes, emits 4R dwords.
// SL: the input is the unsliced 8-bit parent and Eq. 1 is applied on the way (slice + pack fused).
template <int R, bool SL>
__global__ __launch_bounds__(256) void pack_kernel(const uint8_t *__restrict__ S, uint4 *__restrict__ packed, int N,
                                                   int64_t K, int G, int64_t ntiles) {
    using T = Layout<R>;
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int lane = threadIdx.x & 63;
    const int64_t tile = tid >> 6;
    if (tile >= ntiles) return;
    const int64_t rb = tile / G;
    const int g = (int)(tile - rb * G);
    const int64_t n = rb * kRowBlock + lane;

    uint8_t code[kGroup];
    if (n < N) {
        const uint8_t *src = S + n * K + (int64_t)g * kGroup;
#pragma unroll
        for (int i = 0; i < kGroup; ++i) {
            if constexpr (SL && R < kC) {
                const uint32_t t = ((uint32_t)src[i] + (1u << (kC - R - 1))) >> (kC - R);
                code[i] = (uint8_t)(t < (1u << R) - 1 ? t : (1u << R) - 1);
            } else {
                code[i] = src[i] >> (kC - R);
            }
        }
    } else {
#pragma unroll
        for (int i = 0; i < kGroup; ++i) code[i] = 0;
    }

    uint32_t dw[4 * R];
#pragma unroll
    for (int i = 0; i < 4 * R; ++i) dw[i] = 0;
    constexpr int NU = 4 * R / T::UD;
    static_for<NU>([&](auto un) {
        static_for<T::NOPS>([&](auto oi) {
            constexpr Op o = T::op(oi);
            constexpr int p = ctz16(o.mask);
            constexpr uint32_t fm = (uint32_t)(o.mask >> p);
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const uint32_t t = code[2 * (un * T::PPU + o.pair) + h];
                dw[un * T::UD + o.dw] |= ((t >> o.d) & fm) << (p + o.sh + 16 * h);
            }
        });
    });
    uint4 *dst = packed + tile * (R * 64) + lane;
#pragma unroll
    for (int i = 0; i < R; ++i) dst[i * 64] = make_uint4(dw[4 * i], dw[4 * i + 1], dw[4 * i + 2], dw[4 * i + 3]);
}

// ------------------------------------------------------------------ re-slice
// Tile layout in (the 8-bit pack of the parent), tile layout out (r bits): one thread per (tile, lane).
// A lane dword of the parent holds pair 2j in the low bytes of its halves and pair 2j+1 in the high
// bytes; Eq. 1 is applied to both columns of a pair at once in their 16-bit containers, and the r-bit
// indices go to their fields of Layout<R> with the same shifts for both halves.
typedef uint16_t u16x2 __attribute__((ext_vector_type(2)));
template <int R> __device__ __forceinline__ uint32_t slice_pair_index(uint32_t v) {
    if constexpr (R == kC) return v;
    constexpr int sh = kC - R;
    u16x2 t = __builtin_bit_cast(u16x2, v + (0x10001u << (sh - 1)));
    t = t >> (uint16_t)sh;
    const u16x2 cap = {(uint16_t)((1 << R) - 1), (uint16_t)((1 << R) - 1)};
    t = __builtin_elementwise_min(t, cap);
    return __builtin_bit_cast(uint32_t, t);
}

// one lane's share of a tile: 8 16-byte pieces of the parent in, R pieces out
template <int R>
__device__ __forceinline__ void reslice_tile(const uint4 *__restrict__ src, uint4 *__restrict__ dst) {
    using T = Layout<R>;
    // both sides are touched once: non-temporal (streaming) loads and stores
    typedef uint32_t v4u __attribute__((ext_vector_type(4)));
    uint32_t q[4 * kC];
#pragma unroll
    for (int i = 0; i < kC; ++i) {
        const v4u v = __builtin_nontemporal_load(reinterpret_cast<const v4u *>(src) + i * 64);
        q[4 * i] = v.x; q[4 * i + 1] = v.y; q[4 * i + 2] = v.z; q[4 * i + 3] = v.w;
    }
    uint32_t dw[4 * R];
#pragma unroll
    for (int i = 0; i < 4 * R; ++i) dw[i] = 0;
    constexpr int NU = 4 * R / T::UD;
    static_for<NU>([&](auto un) {
        static_for<T::NOPS>([&](auto oi) {
            constexpr Op o = T::op(oi);
            constexpr int pidx = un * T::PPU + o.pair;  // activation pair of the group, 0..63
            constexpr int p = ctz16(o.mask);
            constexpr uint32_t fm = (uint32_t)(o.mask >> p) * 0x10001u;
            const uint32_t two = pidx & 1 ? (q[pidx >> 1] >> 8) & 0x00FF00FFu : q[pidx >> 1] & 0x00FF00FFu;
            uint32_t t = slice_pair_index<R>(two);
            if constexpr (o.d != 0) t >>= o.d;
            if constexpr (popc16(o.mask) != R) t &= fm;
            dw[un * T::UD + o.dw] |= t << (p + o.sh);
        });
    });
#pragma unroll
    for (int i = 0; i < R; ++i) {
        const v4u v = {dw[4 * i], dw[4 * i + 1], dw[4 * i + 2], dw[4 * i + 3]};
        __builtin_nontemporal_store(v, reinterpret_cast<v4u *>(dst) + i * 64);
    }
}

template <int R>
__global__ __launch_bounds__(256) void reslice_kernel(const uint4 *__restrict__ parent8, uint4 *__restrict__ packed,
                                                      int64_t ntiles) {
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int lane = threadIdx.x & 63;
    const int64_t tile = tid >> 6;
    if (tile >= ntiles) return;
    reslice_tile<R>(parent8 + tile * (kC * 64) + lane, packed + tile * (R * 64) + lane);
}

// Several layers in one launch (small layers are launch-bound one by one): tiles of all jobs form one line,
// a wave finds its job in the table that travels with the launch.
struct ResliceJobs {
    const uint4 *src[kResliceBatch];
    uint4 *dst[kResliceBatch];
    int64_t tile_end[kResliceBatch];  // running sum of tiles
    int32_t r[kResliceBatch];
    int32_t n;
};
__global__ __launch_bounds__(256) void reslice_many_kernel(const ResliceJobs jobs) {
    const int lane = threadIdx.x & 63;
    const int64_t tile = (int64_t)blockIdx.x * 4 + __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    // the table is searched with compile-time indices only (a run-time index would move it to scratch memory)
    const uint4 *src = nullptr;
    uint4 *dst = nullptr;
    int r = 0;
    int64_t t = 0;
#pragma unroll
    for (int j = 0; j < kResliceBatch; ++j) {
        const int64_t lo = j ? jobs.tile_end[j - 1] : 0;
        if (j < jobs.n && tile >= lo && tile < jobs.tile_end[j]) {
            src = jobs.src[j];
            dst = jobs.dst[j];
            r = jobs.r[j];
            t = tile - lo;
        }
    }
    if (!src) return;  // past the last tile
    src += t * (kC * 64) + lane;
    switch (r) {
        case 2: reslice_tile<2>(src, dst + t * (2 * 64) + lane); break;
        case 3: reslice_tile<3>(src, dst + t * (3 * 64) + lane); break;
        case 4: reslice_tile<4>(src, dst + t * (4 * 64) + lane); break;
        case 6: reslice_tile<6>(src, dst + t * (6 * 64) + lane); break;
        default: reslice_tile<8>(src, dst + t * (8 * 64) + lane); break;
    }
}

template <int R>
__global__ __launch_bounds__(256) void unpack_kernel(const uint4 *__restrict__ packed, uint8_t *__restrict__ S, int N,
                                                     int64_t K, int G, int64_t ntiles) {
    using T = Layout<R>;
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int lane = threadIdx.x & 63;
    const int64_t tile = tid >> 6;
    if (tile >= ntiles) return;
    const int64_t rb = tile / G;
    const int g = (int)(tile - rb * G);
    const int64_t n = rb * kRowBlock + lane;
    if (n >= N) return;

    uint32_t dw[4 * R];
    const uint4 *src = packed + tile * (R * 64) + lane;
#pragma unroll
    for (int i = 0; i < R; ++i) {
        const uint4 v = src[i * 64];
        dw[4 * i] = v.x; dw[4 * i + 1] = v.y; dw[4 * i + 2] = v.z; dw[4 * i + 3] = v.w;
    }
    uint8_t code[kGroup];
#pragma unroll
    for (int i = 0; i < kGroup; ++i) code[i] = 0;
    constexpr int NU = 4 * R / T::UD;
    static_for<NU>([&](auto un) {
        static_for<T::NOPS>([&](auto oi) {
            constexpr Op o = T::op(oi);
            constexpr int p = ctz16(o.mask);
            constexpr uint32_t fm = (uint32_t)(o.mask >> p);
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const uint32_t f = (dw[un * T::UD + o.dw] >> (p + o.sh + 16 * h)) & fm;
                code[2 * (un * T::PPU + o.pair) + h] |= (uint8_t)(f << o.d);
            }
        });
    });
    uint8_t *dst = S + n * K + (int64_t)g * kGroup;
#pragma unroll
    for (int i = 0; i < kGroup; ++i) dst[i] = (uint8_t)(code[i] << (kC - R));
}

template <int R, bool SL>
static hipError_t launch_pack_r(const uint8_t *S, int64_t N, int64_t K, uint4 *packed, hipStream_t s) {
    const int G = (int)(K / kGroup);
    const int64_t ntiles = pad_rows(N) / kRowBlock * G;
    const int64_t blocks = (ntiles * 64 + 255) / 256;
    if (blocks > (int64_t)0x7fffffff) return hipErrorInvalidValue;  // beyond one grid dimension
    return launch((pack_kernel<R, SL>), dim3((unsigned)blocks), dim3(256), 0, s, S, packed, (int)N, K, G, ntiles);
}
template <int R>
static hipError_t launch_reslice_r(const uint4 *parent8, int64_t N, int64_t K, uint4 *packed, hipStream_t s) {
    const int64_t ntiles = pad_rows(N) / kRowBlock * (K / kGroup);
    const int64_t blocks = (ntiles * 64 + 255) / 256;
    if (blocks > (int64_t)0x7fffffff) return hipErrorInvalidValue;  // beyond one grid dimension
    return launch(reslice_kernel<R>, dim3((unsigned)blocks), dim3(256), 0, s, parent8, packed, ntiles);
}
template <int R>
static hipError_t launch_unpack_r(const uint4 *packed, int64_t N, int64_t K, uint8_t *S, hipStream_t s) {
    const int G = (int)(K / kGroup);
    const int64_t ntiles = pad_rows(N) / kRowBlock * G;
    const int64_t blocks = (ntiles * 64 + 255) / 256;
    if (blocks > (int64_t)0x7fffffff) return hipErrorInvalidValue;  // beyond one grid dimension
    return launch(unpack_kernel<R>, dim3((unsigned)blocks), dim3(256), 0, s, packed, S, (int)N, K, G, ntiles);
}

hipError_t launch_pack(const uint8_t *S, int64_t N, int64_t K, int r, uint4 *packed, hipStream_t s) {
    switch (r) {
        case 2: return launch_pack_r<2, false>(S, N, K, packed, s);
        case 3: return launch_pack_r<3, false>(S, N, K, packed, s);
        case 4: return launch_pack_r<4, false>(S, N, K, packed, s);
        case 6: return launch_pack_r<6, false>(S, N, K, packed, s);
        case 8: return launch_pack_r<8, false>(S, N, K, packed, s);
    }
    return hipErrorInvalidValue;
}
hipError_t launch_slice_pack(const uint8_t *parent, int64_t N, int64_t K, int r, uint4 *packed, hipStream_t s) {
    switch (r) {
        case 2: return launch_pack_r<2, true>(parent, N, K, packed, s);
        case 3: return launch_pack_r<3, true>(parent, N, K, packed, s);
        case 4: return launch_pack_r<4, true>(parent, N, K, packed, s);
        case 6: return launch_pack_r<6, true>(parent, N, K, packed, s);
        case 8: return launch_pack_r<8, true>(parent, N, K, packed, s);
    }
    return hipErrorInvalidValue;
}
hipError_t launch_reslice_many(const uint4 *const *src, uint4 *const *dst, const int64_t *N, const int64_t *K,
                               const int *r, int n, hipStream_t s) {
    for (int j0 = 0; j0 < n; j0 += kResliceBatch) {
        ResliceJobs jobs{};
        int64_t tiles = 0;
        jobs.n = n - j0 < kResliceBatch ? n - j0 : kResliceBatch;
        for (int j = 0; j < jobs.n; ++j) {
            jobs.src[j] = src[j0 + j];
            jobs.dst[j] = dst[j0 + j];
            jobs.r[j] = r[j0 + j];
            tiles += pad_rows(N[j0 + j]) / kRowBlock * (K[j0 + j] / kGroup);
            jobs.tile_end[j] = tiles;
        }
        const int64_t blocks = (tiles * 64 + 255) / 256;
        if (blocks > (int64_t)0x7fffffff) return hipErrorInvalidValue;  // beyond one grid dimension
        const hipError_t e = launch(reslice_many_kernel, dim3((unsigned)blocks), dim3(256), 0, s, jobs);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}
hipError_t launch_reslice(const uint4 *parent8, int64_t N, int64_t K, int r, uint4 *packed, hipStream_t s) {
    switch (r) {
        case 2: return launch_reslice_r<2>(parent8, N, K, packed, s);
        case 3: return launch_reslice_r<3>(parent8, N, K, packed, s);
        case 4: return launch_reslice_r<4>(parent8, N, K, packed, s);
        case 6: return launch_reslice_r<6>(parent8, N, K, packed, s);
        case 8: return launch_reslice_r<8>(parent8, N, K, packed, s);
    }
    return hipErrorInvalidValue;
}
hipError_t launch_unpack(const uint4 *packed, int64_t N, int64_t K, int r, uint8_t *S, hipStream_t s) {
    switch (r) {
        case 2: return launch_unpack_r<2>(packed, N, K, S, s);
        case 3: return launch_unpack_r<3>(packed, N, K, S, s);
        case 4: return launch_unpack_r<4>(packed, N, K, S, s);
        case 6: return launch_unpack_r<6>(packed, N, K, S, s);
        case 8: return launch_unpack_r<8>(packed, N, K, S, s);
    }
    return hipErrorInvalidValue;
}

// ------------------------------------------------------------------ meta
// [N, G] -> [RB][G][64]; pad rows get scale 0 / zero 0.
__global__ __launch_bounds__(256) void pack_meta_kernel(const _Float16 *__restrict__ sc, const _Float16 *__restrict__ zr,
                                                        _Float16 *__restrict__ st, _Float16 *__restrict__ zt, int64_t N,
                                                        int64_t G, int64_t total) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const int lane = (int)(i & 63);
    const int64_t tile = i >> 6;
    const int64_t rb = tile / G;
    const int64_t g = tile - rb * G;
    const int64_t n = rb * kRowBlock + lane;
    st[i] = n < N ? sc[n * G + g] : (_Float16)0.f;
    if (zt) zt[i] = n < N ? zr[n * G + g] : (_Float16)0.f;  // a symmetric layer has no zero-offsets to tile
}

hipError_t launch_pack_meta(const _Float16 *sc, const _Float16 *zr, int64_t N, int64_t G, _Float16 *st, _Float16 *zt,
                            hipStream_t s) {
    const int64_t total = pad_rows(N) * G;
    return launch(pack_meta_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, sc, zr, st, zt, N, G,
                       total);
}

__global__ __launch_bounds__(256) void fill_zero_kernel(uint32_t *p, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}
hipError_t launch_fill_zero(void *p, size_t bytes, hipStream_t s) {
    const size_t n = bytes / 4;
    if (!n) return hipSuccess;
    return launch(fill_zero_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, (uint32_t *)p, n);
}

// ------------------------------------------------------------------ descriptor table of a stack plan
// The table reaches the device inside kernel arguments, kDescPerLaunch descriptors per launch: the runtime copies
// arguments when a launch is enqueued, so no host buffer has to outlive the call and nothing is waited for.
constexpr int kDescPerLaunch = 32;
constexpr int kDescDwords = sizeof(LayerDesc) / 4;
struct DescChunk {
    uint32_t w[kDescPerLaunch * kDescDwords];
};
static_assert(sizeof(DescChunk) + 16 <= 4096, "kernel arguments are limited to 4 KiB");

__global__ __launch_bounds__(256) void write_table_kernel(const DescChunk chunk, uint32_t *dst, int ndw) {
    for (int i = (int)threadIdx.x; i < ndw; i += 256) dst[i] = chunk.w[i];
}

hipError_t launch_write_table(const LayerDesc *table, int n, LayerDesc *dst, hipStream_t s) {
    for (int i0 = 0; i0 < n; i0 += kDescPerLaunch) {
        const int cnt = n - i0 < kDescPerLaunch ? n - i0 : kDescPerLaunch;
        DescChunk c{};
        __builtin_memcpy(c.w, table + i0, (size_t)cnt * sizeof(LayerDesc));
        const hipError_t e = launch(write_table_kernel, dim3(1), dim3(256), 0, s, c,
                                    reinterpret_cast<uint32_t *>(dst + i0), cnt * kDescDwords);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// ------------------------------------------------------------------ measurement aid: what a plain read achieves
// Every wave streams a contiguous share of the buffer with eight non-temporal 16-byte loads per lane in flight and
// folds what it read into one word (so that nothing can be dropped); the rate of this kernel is the read bandwidth
// the linear kernels are measured against, next to the published peak.
__global__ __launch_bounds__(256) void read_probe_kernel(const uint4 *buf, size_t n16, uint32_t *out) {
    typedef uint32_t v4u __attribute__((ext_vector_type(4)));
    constexpr int U = 8;
    const int lane = threadIdx.x & 63;
    const size_t wave = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const size_t nw = ((size_t)gridDim.x * blockDim.x) >> 6;
    const v4u __attribute__((address_space(1))) *g = (const v4u __attribute__((address_space(1))) *)buf;
    const size_t chunk = (size_t)U * 64;
    const size_t per = ((n16 + nw - 1) / nw + chunk - 1) / chunk * chunk;  // whole chunks, shares cover the buffer
    const size_t lo = wave * per < n16 ? wave * per : n16;
    const size_t hi = lo + per < n16 ? lo + per : n16;
    v4u acc = {0, 0, 0, 0};
    size_t base = lo;
    for (; base + chunk <= hi; base += chunk) {
        v4u v[U];
#pragma unroll
        for (int i = 0; i < U; ++i) v[i] = __builtin_nontemporal_load(g + base + i * 64 + lane);
#pragma unroll
        for (int i = 0; i < U; ++i) acc ^= v[i];
    }
    for (base += lane; base < hi; base += 64) acc ^= __builtin_nontemporal_load(g + base);
    uint32_t r = acc.x ^ acc.y ^ acc.z ^ acc.w;
#pragma unroll
    for (int off = 32; off; off >>= 1) r ^= __shfl_xor(r, off);
    if (lane == 0) __hip_atomic_fetch_xor(out, r, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

hipError_t launch_read_probe(const void *buf, size_t bytes, uint32_t *out, hipStream_t s) {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return hipErrorUnknown;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) return hipErrorUnknown;
    return launch(read_probe_kernel, dim3((unsigned)(cus * 4)), dim3(256), 0, s, static_cast<const uint4 *>(buf), bytes / 16, out);
}

}  // namespace mq
