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

// How a wave gets the 64 activation pairs of a group (they are the same for every lane):
//   kXScalar : scalar loads into SGPRs at the start of the tile's math (short latency while x
//              sits in the scalar cache; exposed when it does not)
//   kXLds    : each lane fetches ONE pair together with the tile (one tile ahead, like the
//              weights), drops it into the wave's 256 bytes of LDS and all lanes read the
//              pairs back with broadcast ds_read_b128: no scalar-cache dependence at all
enum XPath { kXScalar = 0, kXLds = 1 };

template <int R, int M> struct TileRegs {
    uint32_t w[4 * R];
    _Float16 s, z;
    uint32_t xl[M];  // lane l's pair (x[2l], x[2l+1]) of the group: X_g, and the kXLds path
};

// weights, scale and zero-offset of tile u
template <int R, int M>
__device__ __forceinline__ void load_tile_w(TileRegs<R, M> &t, const LayerDesc &L, int u, int lane) {
    // Weights, scales and zeros are read exactly once per call: non-temporal loads (streaming hint) keep them from
    // displacing anything in the caches and, measured with a plain read kernel on this chip, stream at 7.0 TB/s where
    // ordinary loads reach 6.2.  The activations below are shared by every wave and stay ordinary loads.
    const u32x4 MQ_GLOBAL *src = gl(reinterpret_cast<const u32x4 *>(L.Wp) + (size_t)u * (R * 64) + lane);
#pragma unroll
    for (int i = 0; i < R; ++i) {
        const u32x4 v = __builtin_nontemporal_load(src + i * 64);
        t.w[4 * i] = v.x; t.w[4 * i + 1] = v.y; t.w[4 * i + 2] = v.z; t.w[4 * i + 3] = v.w;
    }
    t.s = __builtin_nontemporal_load(gl(L.st) + (size_t)u * 64 + lane);
    // A symmetric layer has no zero-offset array: its zt is a few lines of 64 x 128.0 inside the library and zmask
    // folds every tile onto them (cache hits, no HBM traffic).  The load is neither branched around nor selected -- either
    // costs the ALU-bound 2-bit tiles and the mixed Llama-3-70B stack 3-9 % -- and an asymmetric layer pays one scalar AND.
    t.z = __builtin_nontemporal_load(gl(L.zt) + (size_t)(u & L.zmask) * 64 + lane);
}
// the lane's activation pair of group g, per batch row.  fresh: x was written by other workgroups of this very launch
// (a chained stack): the loads go to where the whole device sees memory, past whatever this compute die's caches hold.
template <int R, int M>
__device__ __forceinline__ void load_tile_x(TileRegs<R, M> &t, const LayerDesc &L, int g, int lane, bool fresh = false) {
#pragma unroll
    for (int m = 0; m < M; ++m) {
        const uint32_t MQ_GLOBAL *src = gl(reinterpret_cast<const uint32_t *>(L.x + (size_t)m * L.K + (size_t)g * kGroup)) + lane;
        t.xl[m] = fresh ? __hip_atomic_load(src, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : *src;
    }
}
template <int R, int M>
__device__ __forceinline__ void load_tile(TileRegs<R, M> &t, const LayerDesc &L, int u, int g, int lane) {
    load_tile_w<R, M>(t, L, u, lane);
    load_tile_x<R, M>(t, L, g, lane);
}

// Eq. 1 on the two 8-bit codes of a masked pair (one per 16-bit half), in 8-bit units:
//   S = min((q + 2^(sh-1)) & ~(2^sh - 1), 256 - 2^sh),  sh = 8 - rs
// (rounding half up; q + 2^(sh-1) < 256 + 2^sh, so the only value above the top code is 256 itself).
typedef uint16_t u16x2 __attribute__((ext_vector_type(2)));
struct SliceConst {
    uint32_t half2, keep2;
    u16x2 cap2;
};
__device__ __forceinline__ SliceConst slice_const(int rs) {
    const uint32_t low = (1u << (kC - rs)) - 1;  // the bits Eq. 1 drops
    const uint16_t cap = (uint16_t)(255u - low);
    return {((low + 1) >> 1) * 0x10001u, (0x1FFu & ~low) * 0x10001u, {cap, cap}};
}
__device__ __forceinline__ uint32_t slice_pair(uint32_t v, const SliceConst &c) {
    const u16x2 t = __builtin_bit_cast(u16x2, (v + c.half2) & c.keep2);
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_min(t, c.cap2));
}

// xlds: this wave's M x 64 dwords of LDS (kXLds only)
// SL (R == 8 only): the tile holds the unsliced parent; its codes are sliced to L.rs bits first.
template <int R, int M, int XP, bool SL = false>
__device__ __forceinline__ void tile_math(const TileRegs<R, M> &t, const LayerDesc &L, int g, int lane,
                                          uint32_t *xlds, float (&yacc)[M]) {
    using T = Layout<R>;
    static_assert(!SL || R == kC, "slicing in registers starts from the 8-bit parent");
    constexpr int NU = 4 * R / T::UD;
    const SliceConst sc = slice_const(SL ? L.rs : kC);
    float xg[M];
    cptr32 xs[M];
#pragma unroll
    for (int m = 0; m < M; ++m) {
        const uint32_t xl = t.xl[m];
        xg[m] = wave_sum(dot2(xl, 0x3C003C00u, 0.f));  // (1.0, 1.0)
        if constexpr (XP == kXLds)
            xlds[m * 64 + lane] = xl;
        else
            xs[m] = as_const(L.x + (size_t)m * L.K + (size_t)g * kGroup);
    }
    float acc[M][T::NKEYS];
#pragma unroll
    for (int m = 0; m < M; ++m)
#pragma unroll
        for (int k = 0; k < T::NKEYS; ++k) acc[m][k] = 0.f;

    if constexpr (XP == kXLds) {
        // quad by quad of activation pairs: one broadcast 16-byte LDS read serves four pairs
        static_for<16>([&](auto qi) {
            u32x4 xq[M];
#pragma unroll
            for (int m = 0; m < M; ++m) xq[m] = reinterpret_cast<const u32x4 *>(xlds + m * 64)[qi];
            static_for<NU>([&](auto un) {
                static_for<T::NOPS>([&](auto oi) {
                    constexpr Op o = T::op(oi);
                    constexpr int pidx = un * T::PPU + o.pair;
                    if constexpr (pidx / 4 == qi) {
                        constexpr int key = key_index<R>(oi);
                        uint32_t v = t.w[un * T::UD + o.dw];
                        if constexpr (o.sh != 0) v >>= o.sh;
                        v &= (uint32_t)o.mask * 0x10001u;
                        if constexpr (SL) v = slice_pair(v, sc);
#pragma unroll
                        for (int m = 0; m < M; ++m) acc[m][key] = dot2(v, xq[m][pidx % 4], acc[m][key]);
                    }
                });
            });
        });
    } else {
        static_for<NU>([&](auto un) {
            static_for<T::NOPS>([&](auto oi) {
                constexpr Op o = T::op(oi);
                constexpr int key = key_index<R>(oi);
                uint32_t v = t.w[un * T::UD + o.dw];
                if constexpr (o.sh != 0) v >>= o.sh;
                v &= (uint32_t)o.mask * 0x10001u;
                if constexpr (SL) v = slice_pair(v, sc);
#pragma unroll
                for (int m = 0; m < M; ++m) acc[m][key] = dot2(v, xs[m][un * T::PPU + o.pair], acc[m][key]);
            });
        });
    }
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

// Tiles a wave keeps in flight ahead of the one it is working on.  A wave with one small tile
// in flight cannot pull more than tile_bytes / memory_latency (1.3 GB/s at r = 2), less than
// its fair share of HBM once wider layers free bandwidth, so narrow tiles are fetched deeper:
// about 8 KB per wave in flight at every width.
template <int R> struct PrefetchDepth {
    static constexpr int value = R <= 2 ? 4 : R == 3 ? 3 : R <= 6 ? 2 : 1;
};

// Tiles [u_begin, u_end) of one layer, owned by share `wave`.
template <int R, int M, int XP, bool SL = false>
__device__ __forceinline__ void run_units(const LayerDesc &L, const StackParams &p, int u_begin, int u_end, int wave,
                                          int lane, uint32_t *xlds) {
    constexpr int D = PrefetchDepth<R>::value, NB = D + 1;
    int rb = u_begin / L.G;
    int g = u_begin - rb * L.G;
    int ga = g;
    float yacc[M];
#pragma unroll
    for (int m = 0; m < M; ++m) yacc[m] = 0.f;

    // ring of NB tile buffers with compile-time indices (no register copies, which would wait
    // for the loads); past the end of the run the last tile is fetched again instead of
    // branching around the loads
    TileRegs<R, M> buf[NB];
    int u_pf = u_begin, g_pf = g;
    auto prefetch = [&](TileRegs<R, M> &t) {
        load_tile<R, M>(t, L, u_pf, g_pf, lane);
        if (u_pf + 1 < u_end) {
            ++u_pf;
            g_pf = g_pf + 1 == L.G ? 0 : g_pf + 1;
        }
    };
    static_for<D>([&](auto j) { prefetch(buf[j]); });
    int u = u_begin;
    while (u < u_end) {
        static_for<NB>([&](auto j) {
            if (u >= u_end) return;
            prefetch(buf[(j + D) % NB]);
            tile_math<R, M, XP, SL>(buf[j], L, g, lane, xlds, yacc);
            ++g;
            ++u;
            if (g == L.G || u == u_end) {
                const int row = rb * kRowBlock + lane;
                finish_row_block<M>(L, p, p.cnt + L.cnt_off + rb, L.cost_start + (uint64_t)rb * L.G * L.cost, ga, g,
                                    yacc, wave, lane, [&](const float(&tot)[M]) {
#pragma unroll
                                        for (int m = 0; m < M; ++m)
                                            if (row < L.N) store_y(L.y, (size_t)m * L.N + row, tot[m], L.flags);
                                    });
                ++rb;
                g = 0;
                ga = 0;
#pragma unroll
                for (int m = 0; m < M; ++m) yacc[m] = 0.f;
            }
        });
    }
}

// SL: every layer of the stack is computed from its resident 8-bit parent (LayerDesc::rs).
template <int M, int XP, bool SL = false> __global__ __launch_bounds__(256) void stack_kernel(const StackParams p) {
    __shared__ __attribute__((aligned(16))) uint32_t xlds_all[XP == kXLds ? 4 * M * 64 : 4];
    uint32_t *xlds = xlds_all + (XP == kXLds ? (threadIdx.x >> 6) * M * 64 : 0);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)((blockIdx.x * blockDim.x + threadIdx.x) >> 6));
    if (wave >= p.nwaves) return;
    for (int worker = wave; worker < p.nworkers; worker += p.nwaves) {
        walk_tiles(p, worker, [&](const LayerDesc &L, int u_begin, int u_end) {
            if constexpr (SL) {
                run_units<8, M, XP, true>(L, p, u_begin, u_end, worker, lane, xlds);
            } else {
                switch (L.r) {
                    case 2: run_units<2, M, XP>(L, p, u_begin, u_end, worker, lane, xlds); break;
                    case 3: run_units<3, M, XP>(L, p, u_begin, u_end, worker, lane, xlds); break;
                    case 4: run_units<4, M, XP>(L, p, u_begin, u_end, worker, lane, xlds); break;
                    case 6: run_units<6, M, XP>(L, p, u_begin, u_end, worker, lane, xlds); break;
                    default: run_units<8, M, XP>(L, p, u_begin, u_end, worker, lane, xlds); break;
                }
            }
        });
    }
}

// ------------------------------------------------------------------ one layer, low latency
// mq_linear on a single layer is latency- rather than bandwidth-bound for Llama-sized
// matrices (a 4096 x 4096 layer at r = 4 is 8 MB: one microsecond of HBM time), so the
// single-layer entry point uses a launch shaped for the shortest dependency chain instead of
// the streaming schedule above: one workgroup per (row block, K slice); its W waves take the
// slice's groups round-robin (all their loads are in flight at once), add their lane sums up
// through LDS in wave order, and -- only if K is cut into KS > 1 slices -- hand over to the
// last-arriving slice through KS slots (same deterministic protocol as the stack kernel, with
// KS <= 8 contributors instead of up to G).
// Body shared by the single-layer kernel and the small-stack kernel below.  blk = index of this workgroup among the
// layer's RB * KS workgroups, slot0 = index of the layer's first partial-sum slot, cnt = the layer's row-block counters.
// A layer of a chained small stack that reads what earlier layers of the same launch write (LayerDesc::chain): its
// workgroups fetch their first weights, wait until the finished-row-block counters of all earlier stages have reached
// their totals, and only then read activations.  Nobody can wait for ever: the launch shape keeps every workgroup of
// the stack resident at one time (checked when the stack is planned), so the workgroups waited for are running, and
// they wait for strictly earlier layers only; the number of polls is bounded on top of that (a wait that runs out goes
// on with whatever x holds).  Visibility follows the split-K hand-over's protocol: in a chained stack every y is stored
// through to device-wide memory and acknowledged before its row block is counted, and a layer that has waited reads
// its activations with device-scope loads -- no cache-wide write-back or invalidation anywhere (one per row block and
// one per waiting wave made the chained launch 2.6 times slower than the launches it replaces).
constexpr int kChainPolls = 1 << 20;
// What a workgroup of a chained small stack needs besides its descriptor (all of it uniform over the launch and held
// in scalar registers): the counters, the totals of the stages before the layer's own, and the launch's total.
struct ChainCtl {
    int32_t *counters;         // kChainCounters of them; nullptr: the stack is not chained
    const int32_t *stage_rb;   // row blocks per stage (kernel arguments)
    int32_t total;
};
__device__ __forceinline__ void chain_wait(const ChainCtl &c, int stage) {
    for (int s = 0; s < stage; ++s) {
        const int32_t MQ_GLOBAL *ctr = gl(c.counters + s);
        const int want = c.stage_rb[s];
        for (int polls = 0; polls < kChainPolls; ++polls) {
            if (__hip_atomic_load(ctr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= want) break;
            __builtin_amdgcn_s_sleep(2);
        }
    }
}
// by the wave that has just stored a row block of y
__device__ __forceinline__ void chain_announce(const ChainCtl &c, int stage, int lane) {
    // the write-through stores of y must have been acknowledged before the counters move
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    if (lane != 0) return;
    int32_t MQ_GLOBAL *ctr = gl(c.counters);
    __hip_atomic_fetch_add(ctr + stage, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    // every row block of the launch is counted once more in the last counter; whoever completes it is the last to
    // touch the counters (each waiter has contributed to a row block counted here, after its wait) and zeroes them
    const int old = __hip_atomic_fetch_add(ctr + kSmallStackLayers, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (old + 1 == c.total)
        for (int i = 0; i < kChainCounters; ++i) __hip_atomic_store(ctr + i, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// CH: the launch is a chained small stack (`chain` is live); the plain variants carry none of its code
template <int R, int M, int XP, bool SL, bool CH = false>
__device__ __forceinline__ void linear_rb_body(const LayerDesc &L, const int KS, const int blk, const int slot0,
                                               float *part, int32_t *cnt, float (*red)[M][64], uint32_t *xlds_all,
                                               const ChainCtl chain = ChainCtl{nullptr, nullptr, 0}) {
    uint32_t *xlds = xlds_all + (XP == kXLds ? (threadIdx.x >> 6) * M * 64 : 0);
    const int lane = threadIdx.x & 63;
    const int w = threadIdx.x >> 6, W = blockDim.x >> 6;
    const int rb = blk / KS, ks = blk - rb * KS;
    const int g_lo = (int)((int64_t)ks * L.G / KS), g_hi = (int)((int64_t)(ks + 1) * L.G / KS);
    float yacc[M];
#pragma unroll
    for (int m = 0; m < M; ++m) yacc[m] = 0.f;
    int g = g_lo + w;
    const bool waits = CH && (L.chain & kChainWaits);
    TileRegs<R, M> cur, nxt;
    if (g < g_hi) load_tile_w<R, M>(cur, L, rb * L.G + g, lane);
    bool have_nxt = false;  // a waiting layer has the weights of its second tile on their way, too, before it waits
    if constexpr (CH) {
        if (waits) {  // uniform over the workgroup
            if (g + W < g_hi) {
                load_tile_w<R, M>(nxt, L, rb * L.G + g + W, lane);
                have_nxt = true;
            }
            if (w == 0) chain_wait(chain, L.chain & 0xFF);
            __syncthreads();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
        }
    }
    if (g < g_hi) {
        load_tile_x<R, M>(cur, L, g, lane, waits);
        while (true) {
            const int g2 = g + W;
            if (g2 < g_hi) {
                if (!have_nxt) load_tile_w<R, M>(nxt, L, rb * L.G + g2, lane);
                have_nxt = false;
                load_tile_x<R, M>(nxt, L, g2, lane, waits);
            }
            tile_math<R, M, XP, SL>(cur, L, g, lane, xlds, yacc);
            if (g2 >= g_hi) break;
            cur = nxt;
            g = g2;
        }
    }
#pragma unroll
    for (int m = 0; m < M; ++m) red[w][m][lane] = yacc[m];
    __syncthreads();
    if (w != 0) return;
    float tot[M];
#pragma unroll
    for (int m = 0; m < M; ++m) {
        tot[m] = red[0][m][lane];
        for (int i = 1; i < W; ++i) tot[m] += red[i][m][lane];
    }
    const int row = rb * kRowBlock + lane;
    if (KS > 1) {
        float MQ_GLOBAL *mine = gl(part + ((size_t)(slot0 + blk) * M) * 64 + lane);
#pragma unroll
        for (int m = 0; m < M; ++m) __hip_atomic_store(mine + m * 64, tot[m], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        // the write-through stores must have been acknowledged before the counter moves
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        int old = 0;
        if (lane == 0) old = __hip_atomic_fetch_add(gl(cnt + rb), 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        old = __builtin_amdgcn_readfirstlane(old);
        if (old != KS - 1) return;
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
        const float MQ_GLOBAL *src = gl(part + ((size_t)(slot0 + rb * KS) * M) * 64 + lane);
        float v[8][M];
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int m = 0; m < M; ++m)
                v[i][m] = __hip_atomic_load(src + ((size_t)(i < KS ? i : KS - 1) * M + m) * 64, __ATOMIC_RELAXED,
                                            __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
        for (int m = 0; m < M; ++m) {
            tot[m] = v[0][m];
#pragma unroll
            for (int i = 1; i < 8; ++i)
                if (i < KS) tot[m] += v[i][m];
        }
        if (lane == 0) __hip_atomic_store(gl(cnt + rb), 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if constexpr (CH) {
#pragma unroll
        for (int m = 0; m < M; ++m)
            if (row < L.N)
                __hip_atomic_store(gl(reinterpret_cast<uint16_t *>(L.y)) + (size_t)m * L.N + row, y_bits(tot[m], L.flags),
                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        chain_announce(chain, L.chain & 0xFF, lane);
        return;
    }
#pragma unroll
    for (int m = 0; m < M; ++m)
        if (row < L.N) store_y(L.y, (size_t)m * L.N + row, tot[m], L.flags);
}

template <int R, int M, int XP, bool SL = false>
__global__ __launch_bounds__(1024) void linear_rb_kernel(const LayerDesc L, const int KS, float *part, int32_t *cnt) {
    __shared__ float red[16][M][64];
    __shared__ __attribute__((aligned(16))) uint32_t xlds_all[XP == kXLds ? 16 * M * 64 : 4];
    linear_rb_body<R, M, XP, SL>(L, KS, (int)blockIdx.x, 0, part, cnt, red, xlds_all);
}

// Launch shape, from sweeps on Llama-2-7B / Llama-3-70B shapes (cold weights): enough K slices
// that (a) there are >= 256 workgroups when there are few row blocks and (b) no wave owns more
// than about two tiles; at most 8 slices, each at least 4 groups long.
__host__ __device__ static inline int pick_k_slices(const LayerDesc &L) {
    const int cover = L.RB >= 128 ? 1 : (256 + L.RB - 1) / L.RB;
    const int depth = (L.G + 31) / 32;
    int ks = cover > depth ? cover : depth;
    if (ks > 8) ks = 8;
    while (ks > 1 && L.G / ks < 4) --ks;
    return ks < 1 ? 1 : ks;
}

// K slices of a layer inside a small stack: as alone, but no more than the stack's launch shape allows
__host__ __device__ static inline int stack_k_slices(const LayerDesc &L, int ks_cap) {
    const int ks = pick_k_slices(L);
    return ks_cap > 0 && ks > ks_cap ? ks_cap : ks;
}

// Waves per workgroup for a K slice of per_block groups (sweeps on the Llama-2-7B shapes, r = 2, 4, 8: 16 waves from 16
// groups on, e.g. 4096 x 11008 in four slices of 21-22 groups: 8.3 / 9.6 / 12.9 -> 7.9 / 9.1 / 11.8 us)
static int rb_waves(const LayerDesc &L, int KS) {
    const int per_block = (L.G + KS - 1) / KS;
    return (per_block >= 16 || (KS == 1 && per_block >= 12)) ? 16 : per_block >= 6 ? 8 : 4;
}

template <int R, int M, bool SL = false>
static hipError_t launch_linear_rb_rm(const LayerDesc &L, float *part, int32_t *cnt, hipStream_t s) {
    const int KS = pick_k_slices(L);
    const int W = rb_waves(L, KS);
    return launch((linear_rb_kernel<R, M, kXLds, SL>), dim3((unsigned)(L.RB * KS)), dim3(64 * W), 0, s, L, KS, part,
                       cnt);
}
template <int M> static hipError_t launch_linear_rb_m(const LayerDesc &L, float *part, int32_t *cnt, hipStream_t s) {
    if (L.rs) return launch_linear_rb_rm<8, M, true>(L, part, cnt, s);
    switch (L.r) {
        case 2: return launch_linear_rb_rm<2, M>(L, part, cnt, s);
        case 3: return launch_linear_rb_rm<3, M>(L, part, cnt, s);
        case 4: return launch_linear_rb_rm<4, M>(L, part, cnt, s);
        case 6: return launch_linear_rb_rm<6, M>(L, part, cnt, s);
        case 8: return launch_linear_rb_rm<8, M>(L, part, cnt, s);
    }
    return hipErrorInvalidValue;
}
// The low-latency shape pays off while a wave owns few tiles; big layers stream better under
// the persistent schedule.  Slots needed: RB * KS * M * 64 floats (KS <= 8).
bool linear_rb_fits(const LayerDesc &L, size_t part_bytes) {
    if ((int64_t)L.RB * L.G > 12288) return false;
    return (size_t)L.RB * 8 * (size_t)L.M * 64 * sizeof(float) <= part_bytes;
}
hipError_t launch_linear_rb(const LayerDesc &L, float *part, int32_t *cnt, hipStream_t s) {
    switch (L.M) {
        case 1: return launch_linear_rb_m<1>(L, part, cnt, s);
        case 2: return launch_linear_rb_m<2>(L, part, cnt, s);
        case 3: return launch_linear_rb_m<3>(L, part, cnt, s);
        case 4: return launch_linear_rb_m<4>(L, part, cnt, s);
    }
    return hipErrorInvalidValue;
}

// The same shape for a SMALL stack (the linears of a decoder block that share their input, say): the workgroups of all
// layers in one launch; a workgroup finds its layer and its descriptor in the kernel arguments (at most 16 layers).
template <int M, int XP, bool SL, bool CH = false>
__global__ __launch_bounds__(1024) void linear_rb_stack_kernel(const StackParams p, const SmallTable t) {
    __shared__ float red[16][M][64];
    __shared__ __attribute__((aligned(16))) uint32_t xlds_all[XP == kXLds ? 16 * M * 64 : 4];
    // the grid holds exactly sum(RB * KS) workgroups; each layer's first one and the descriptors come with the kernel
    // arguments, so a workgroup reads nothing from device memory before its tiles (a walk along the table there was a
    // chain of dependent loads, 0.5 us each and 1.2 us for the first)
    int li = 0;
#pragma unroll
    for (int i = 1; i < 16; ++i)
        if (i < p.n_layers && (int)blockIdx.x >= p.ll_start[i]) li = i;
    const int slot0 = p.ll_start[li], blk = (int)blockIdx.x - slot0;
    const LayerDesc L = t.d[li];
    const int KS = stack_k_slices(L, p.ks_cap);
    int32_t *cnt = p.cnt + L.cnt_off;
    const ChainCtl chain{CH ? p.cnt + p.chain_off : nullptr, p.stage_rb, p.chain_total};
    if constexpr (SL) {
        linear_rb_body<8, M, XP, true, CH>(L, KS, blk, slot0, p.part, cnt, red, xlds_all, chain);
    } else {
        switch (L.r) {
            case 2: linear_rb_body<2, M, XP, false, CH>(L, KS, blk, slot0, p.part, cnt, red, xlds_all, chain); break;
            case 3: linear_rb_body<3, M, XP, false, CH>(L, KS, blk, slot0, p.part, cnt, red, xlds_all, chain); break;
            case 4: linear_rb_body<4, M, XP, false, CH>(L, KS, blk, slot0, p.part, cnt, red, xlds_all, chain); break;
            case 6: linear_rb_body<6, M, XP, false, CH>(L, KS, blk, slot0, p.part, cnt, red, xlds_all, chain); break;
            default: linear_rb_body<8, M, XP, false, CH>(L, KS, blk, slot0, p.part, cnt, red, xlds_all, chain); break;
        }
    }
}

// workgroups of `waves` waves of the small-stack kernel that the device holds at one time
template <int M, bool SL, bool CH = false> static int rb_stack_resident(int waves) {
    static int cached[3] = {0, 0, 0};
    const int slot = waves == 16 ? 0 : waves == 8 ? 1 : 2;
    if (cached[slot]) return cached[slot];
    int dev = 0, cus = 0, b = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&b, linear_rb_stack_kernel<M, kXLds, SL, CH>, 64 * waves, 0) != hipSuccess)
        return 0;
    cached[slot] = cus * (b < 1 ? 1 : b);
    return cached[slot];
}
template <int M> static int rb_stack_resident_v(bool from_parent, bool chained, int waves) {
    if constexpr (M <= kChainMaxM) {
        if (chained) return from_parent ? rb_stack_resident<M, true, true>(waves) : rb_stack_resident<M, false, true>(waves);
    }
    return from_parent ? rb_stack_resident<M, true>(waves) : rb_stack_resident<M, false>(waves);
}
// chained: the variant of the kernel whose layers may wait for each other (it is the one whose residency matters then)
static int rb_stack_resident_m(int M, bool from_parent, bool chained, int waves) {
    switch (M) {
        case 1: return rb_stack_resident_v<1>(from_parent, chained, waves);
        case 2: return rb_stack_resident_v<2>(from_parent, chained, waves);
        case 3: return rb_stack_resident_v<3>(from_parent, chained, waves);
        default: return rb_stack_resident_v<4>(from_parent, false, waves);
    }
}

// A stack is "small" when all its layers together still fit the low-latency shape (same bound as for one layer).
// Returns the launch shape: workgroups = sum of RB * KS, waves per workgroup = the most any layer wants -- unless the
// device cannot hold all those workgroups at one time: the ones left over would start when the first have finished,
// and a launch this short then takes half as long again (three 4096 x 4096 layers: 768 workgroups of 8 waves where 512
// fit).  Then first the waves per workgroup are halved (a wave takes more tiles), then the K slices.
bool linear_rb_stack_shape(const LayerDesc *table, int n_layers, size_t part_bytes, bool from_parent, bool chained,
                           int *blocks, int *waves, int *ks_cap, int32_t *ll_start, bool *all_resident) {
    if (n_layers > kSmallStackLayers || table[0].M > kValuMaxM) return false;
    int64_t tiles = 0, slots = 0;
    for (int i = 0; i < n_layers; ++i) {
        tiles += (int64_t)table[i].RB * table[i].G;
        slots += (int64_t)table[i].RB * 8;
    }
    if (tiles > 12288 || (size_t)slots * (size_t)table[0].M * 64 * sizeof(float) > part_bytes) return false;
    auto shape = [&](int cap, int *nb, int *W) {
        *nb = 0;
        *W = 4;
        for (int i = 0; i < n_layers; ++i) {
            const int ks = stack_k_slices(table[i], cap);
            *nb += table[i].RB * ks;
            const int w = rb_waves(table[i], ks);
            if (w > *W) *W = w;
        }
    };
    // A chained stack is a chain of dependent steps: what counts is the length of one step, and a row block that is
    // not cut along K needs no hand-over through device memory (three round trips) before its y can be announced.
    int nb = 0, W = 4, cap = chained ? 1 : 0;
    shape(cap, &nb, &W);
    *all_resident = false;
    for (;;) {
        const int fit = rb_stack_resident_m(table[0].M, from_parent, chained, W);
        if (fit > 0 && nb <= fit) *all_resident = true;
        if (fit <= 0 || nb <= fit) break;
        if (W > 4) { W /= 2; continue; }
        const int next = cap == 0 ? 4 : cap / 2;
        if (next < 1) break;
        cap = next;
        shape(cap, &nb, &W);
    }
    *blocks = nb;
    *waves = W;
    *ks_cap = cap;
    int start = 0;
    for (int i = 0; i < 16; ++i) {
        ll_start[i] = start;
        if (i < n_layers) start += table[i].RB * stack_k_slices(table[i], cap);
    }
    return true;
}

template <int M> static hipError_t launch_linear_rb_stack_m(const StackParams &p, const SmallTable &t, int blocks, int waves,
                                                            bool from_parent, hipStream_t s) {
    if constexpr (M <= kChainMaxM) {
        if (p.chain_total) {
            if (from_parent)
                return launch((linear_rb_stack_kernel<M, kXLds, true, true>), dim3((unsigned)blocks), dim3(64 * waves), 0, s, p, t);
            return launch((linear_rb_stack_kernel<M, kXLds, false, true>), dim3((unsigned)blocks), dim3(64 * waves), 0, s, p, t);
        }
    }
    if (p.chain_total) return hipErrorInvalidValue;  // refused when the stack was planned
    if (from_parent)
        return launch((linear_rb_stack_kernel<M, kXLds, true>), dim3((unsigned)blocks), dim3(64 * waves), 0, s, p, t);
    return launch((linear_rb_stack_kernel<M, kXLds, false>), dim3((unsigned)blocks), dim3(64 * waves), 0, s, p, t);
}
hipError_t launch_linear_rb_stack(const StackParams &p, const SmallTable &t, int blocks, int waves, bool from_parent,
                                  hipStream_t s) {
    switch (p.M) {
        case 1: return launch_linear_rb_stack_m<1>(p, t, blocks, waves, from_parent, s);
        case 2: return launch_linear_rb_stack_m<2>(p, t, blocks, waves, from_parent, s);
        case 3: return launch_linear_rb_stack_m<3>(p, t, blocks, waves, from_parent, s);
        case 4: return launch_linear_rb_stack_m<4>(p, t, blocks, waves, from_parent, s);
    }
    return hipErrorInvalidValue;
}

// blocks (of 4 waves) the device keeps resident per compute unit, and the number of units
template <int M, int XP, bool SL> static bool residency(int &cus, int &blocks) {
    static int c_cus = 0, c_blocks = 0;
    if (!c_cus) {
        int dev = 0, a = 0, b = 0;
        if (hipGetDevice(&dev) != hipSuccess) return false;
        if (hipDeviceGetAttribute(&a, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return false;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&b, stack_kernel<M, XP, SL>, 256, 0) != hipSuccess) return false;
        if (b < 1) b = 1;
        while (a * b * 4 > kMaxWaves) --b;
        c_cus = a;
        c_blocks = b;
    }
    cus = c_cus;
    blocks = c_blocks;
    return true;
}

template <int M, int XP, bool SL> static hipError_t launch_stack_mx(StackParams p, int max_cost, hipStream_t s) {
    int cus = 0, blocks = 0;
    if (!residency<M, XP, SL>(cus, blocks)) return hipErrorUnknown;
    int hw = cus * blocks * 4;
    if (p.worker_cap && hw > p.worker_cap) hw = p.worker_cap;
    const uint64_t max_workers = p.worker_cap ? (uint64_t)p.worker_cap : (uint64_t)max_workers_valu(M);
    // every share must be at least one tile long, so that each share between the first
    // and last contributor of a row block really owns a tile of it
    uint64_t cap = p.cost_total / (uint64_t)max_cost;
    if (cap < 1) cap = 1;
    p.nwaves = (int)(cap < (uint64_t)hw ? cap : (uint64_t)hw);
    // A single big layer at batch 1 is over in 25-50 us: with every resident wave a share is only a few tiles
    // long and each row block is handed over many times.  A quarter of the waves still saturates HBM for that
    // long (each keeps its 8 KB in flight) and takes 10-25 % off the call (measured on the Llama-3-70B MLP shapes).
    if (!p.table && M == 1 && p.nwaves > 2048) p.nwaves = 2048;
    // Several interleaved shares per wave even out layers of different width (a wave serves
    // shares w, w + nwaves, ...), but every share ends with up to two hand-overs of a few
    // microseconds, so shares stay at least ~128 tiles long (measured: Llama-2-7B stacks are
    // best with one share per wave, Llama-3-70B stacks gain 15 % from eight).
    uint64_t spw = p.cost_total / ((uint64_t)max_cost * 128 * (uint64_t)p.nwaves);  // whole shares per wave
    if (spw > (uint64_t)kSharesPerWave) spw = kSharesPerWave;
    while (spw > 1 && spw * (uint64_t)p.nwaves > max_workers) --spw;
    if (spw < 1) spw = 1;
    p.nworkers = (int)(spw * (uint64_t)p.nwaves);
    const unsigned nblocks = (unsigned)((p.nwaves + 3) / 4);
    return launch((stack_kernel<M, XP, SL>), dim3(nblocks), dim3(256), 0, s, p);
}
template <int M> static hipError_t launch_stack_m(StackParams p, int max_cost, bool from_parent, hipStream_t s) {
    // kXLds: measured 1-3 % (stack) to 20 % (single calls) faster than kXScalar
    return from_parent ? launch_stack_mx<M, kXLds, true>(p, max_cost, s) : launch_stack_mx<M, kXLds, false>(p, max_cost, s);
}

hipError_t launch_stack(StackParams p, int max_cost, bool from_parent, hipStream_t s) {
    switch (p.M) {
        case 1: return launch_stack_m<1>(p, max_cost, from_parent, s);
        case 2: return launch_stack_m<2>(p, max_cost, from_parent, s);
        case 3: return launch_stack_m<3>(p, max_cost, from_parent, s);
        case 4: return launch_stack_m<4>(p, max_cost, from_parent, s);
    }
    return hipErrorInvalidValue;
}

// ------------------------------------------------------------------ bf16 activations for the kernels above
// One small launch ahead of a vector-ALU launch whose layers (some of them) take bf16 activations: those layers'
// activations (LayerDesc::x_bf16) go, as fp16, to the room the workspace keeps for them, which is where LayerDesc::x of
// such a layer points: the kernels above never see the difference.  32 workgroups per layer; layers without the flag
// return at once.
constexpr int kXcvtBlocks = 32;
__global__ __launch_bounds__(256) void xcvt_kernel(const StackParams p) {
    const int li = (int)(blockIdx.x / kXcvtBlocks), bx = (int)(blockIdx.x % kXcvtBlocks);
    const LayerDesc L = p.table ? load_desc(p.table + li) : p.single;
    if (!(L.flags & kFlagXBf16)) return;
    const uint32_t MQ_GLOBAL *src = gl(reinterpret_cast<const uint32_t *>(L.x_bf16));
    uint32_t MQ_GLOBAL *dst = gl(reinterpret_cast<uint32_t *>(const_cast<_Float16 *>(L.x)));
    const int64_t pairs = (int64_t)L.M * L.K / 2;
    for (int64_t i = (int64_t)bx * 256 + threadIdx.x; i < pairs; i += (int64_t)kXcvtBlocks * 256)
        dst[i] = bf16_pair_to_f16_pair(src[i]);
}
hipError_t launch_xcvt(const StackParams &p, hipStream_t s) {
    return launch(xcvt_kernel, dim3((unsigned)(p.n_layers * kXcvtBlocks)), dim3(256), 0, s, p);
}

}  // namespace mq
