// Small / medium batch (4 < M <= 256): the same sliced linear layer on the
// matrix cores (Section 4 of the paper switches to TensorCores from batch 8;
// here the switch is at M = 5).  Same packed tiles, same persistent schedule and
// split-K hand-off (mq_device.h) as the vector-ALU kernel.
//
// MFMA mapping.  v_mfma_f32_32x32x16_f16 computes D[32x32] += A[32x16] * B[16x32];
// lane l supplies A[l%32][8*(l/32) .. +7] and B[8*(l/32) .. +7][l%32].  In the tile
// layout lane l owns row l of the 64-row tile, and four masked dwords of a lane
// (the same bit-field of four units) are eight fp16 subnormals = eight columns
// k_0..k_7 of that row, i.e. already a valid A operand: lanes 0..31 feed tile
// rows 0..31 as the first k-half, lanes 32..63 feed tile rows 32..63 as the
// second k-half, both halves carrying the SAME eight columns.  B separates the
// two halves again: for output column j < 16 it holds x[j][k_e] in the first
// k-half and zero in the second, for j >= 16 the other way round.  Then
//   D[i][j]      = sum_e W[row i     ][k_e] * x[j     ][k_e]     (j <  16)
//   D[i][j]      = sum_e W[row 32 + i][k_e] * x[j - 16][k_e]     (j >= 16)
// so one MFMA handles 64 rows x 8 columns of W x 16 batch rows (half of B is
// zeros: the price of sharing one weight layout with the batch-1 kernel).
// The B operands are prepared once per call by xprep_kernel into the order the
// MFMAs consume them; lanes whose B is zero read out of range of a buffer
// resource, which returns 0 without touching memory.
//
// A batch of more than 16 rows is served in chunks of 16 columns; a chunk is
// scheduled like a layer of its own (chunk index slowest).
//
// One accumulator per tile.  A masked field is the fp16 subnormal digit * 2^(p-24) and stands for
// digit * 2^d of the code (p = position of the field in its half, d = first code bit it carries), so
// fields with different p - d ("keys") would need accumulators of their own.  Instead the B operand
// of each MFMA is the activations times 2^(e - (p - d)): every MFMA of a tile then adds
// code-part * x * 2^(e-24) into the SAME 32x32 accumulator, and no vector instruction touches the
// accumulator before the group is complete.  e is a block exponent chosen by the prep kernel per
// (chunk, group, batch column) so that the largest |x| of the group lands in [2^14, 2^15): the scaling
// is exact for every element within 2^-22 of the group's largest (smaller ones lose low bits worth
// less than 2^-38 of the largest product: far below the fp32 accumulation itself).
// The zero-offset rides on the matrix core as well: one more MFMA per tile multiplies the row's zero
// (A = z * 2^(r-17), exact for every zero >= 2) by -X_g * 2^(e-15) split into three fp16 pieces
// (relative error 2^-33), so that D = 2^(e+r-32) * sum_k x_k * (S_k - z).  Per group and accumulator
// element what is left for the vector ALUs is  y += scale * (F * D),  F = 2^(32-r-e)  from the prep
// kernel: integer codes stay exact and scales are never rounded to fp16, as on the vector-ALU path.
#include "mq_device.h"

namespace mq {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float16_t __attribute__((ext_vector_type(16)));
typedef u32x4 uint4_t;

template <int R> struct Mfma {
    using T = Layout<R>;
    static constexpr int NU = 4 * R / T::UD;       // units per lane and tile
    static constexpr int NQ = NU / 4;              // unit quads
    static constexpr int NMF = NQ * T::NOPS;       // MFMAs per tile
    static_assert(NU % 4 == 0, "units must come in quads");
};

// ------------------------------------------------------------------ activation prep
// One wave per (layer, chunk, group): writes the B operands of the NMF MFMAs of a tile
// (16 columns x 8 halves each) and the per-column group sums X_g.  Branch-free: columns
// beyond M read column 0 and are masked to zero, all loads are issued before the stores.
template <int CTRL> __device__ __forceinline__ float dpp_max(float v) {
    const int t = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false);
    return fmaxf(v, __builtin_bit_cast(float, t));
}
// (x_lo, x_hi) * scale, a power of two, back to an fp16 pair (exact unless a result is subnormal)
__device__ __forceinline__ uint32_t scale_pair(uint32_t v, float scale) {
    const half2_t h = __builtin_bit_cast(half2_t, v);
    const half2_t o = {(_Float16)((float)h.x * scale), (_Float16)((float)h.y * scale)};
    return __builtin_bit_cast(uint32_t, o);
}
template <int R> __device__ __forceinline__ void xprep_job(const LayerDesc &L, int c, int g, int lane) {
    using T = Layout<R>;
    constexpr int NMF = Mfma<R>::NMF;
    const int m = lane >> 2, j = lane & 3;
    const int col = c * kChunkCols + m;
    const uint32_t live = col < L.M ? 0xFFFFFFFFu : 0u;
    const uint32_t MQ_GLOBAL *xrow =
        gl(reinterpret_cast<const uint32_t *>(L.x + (size_t)(live ? col : 0) * L.K) + (size_t)g * 64);
    uint32_t MQ_GLOBAL *out =
        gl(reinterpret_cast<uint32_t *>(const_cast<uint4 *>(L.xt)) + ((size_t)(c * L.G + g) * (NMF + 1)) * 64 + lane);
    uint32_t v[NMF];
    static_for<NMF>([&](auto mf) {
        constexpr int Q = mf / T::NOPS;
        constexpr Op o = T::op(mf % T::NOPS);
        // dword j of the lane's operand = activation pair of unit 4Q+j, field o
        v[mf] = xrow[(4 * Q + j) * T::PPU + o.pair] & live;
    });
    uint32_t q[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) q[i] = xrow[j * 16 + i] & live;
    // X_g and the largest |x| of column m: lanes 4m..4m+3 each cover a quarter of the group
    float s = 0.f, amax = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        s = dot2(q[i], 0x3C003C00u, s);
        const half2_t h = __builtin_bit_cast(half2_t, q[i] & 0x7FFF7FFFu);
        amax = fmaxf(amax, fmaxf((float)h.x, (float)h.y));
    }
    s = dpp_add<0xB1>(s);
    s = dpp_add<0x4E>(s);
    amax = dpp_max<0xB1>(amax);
    amax = dpp_max<0x4E>(amax);
    // block exponent: amax * 2^e in [2^14, 2^15) (amax = 0 or subnormal: as if it were the smallest normal)
    int ex = (int)((__builtin_bit_cast(uint32_t, amax) >> 23) & 0xFF) - 127;  // floor(log2(amax)) for normal fp32
    if (ex < -14) ex = -14;
    if (ex > 15) ex = 15;  // Inf / NaN in, garbage out, but no undefined shifts
    const int e = 14 - ex;
    const float base = __builtin_ldexpf(1.f, e);
    static_for<NMF>([&](auto mf) {
        constexpr Op o = T::op(mf % T::NOPS);
        constexpr int key = ctz16(o.mask) - o.d;
        out[mf * 64] = scale_pair(v[mf], base * __builtin_ldexpf(1.f, -key));
    });
    // the zero-offset block: -X_g * 2^(e-15) in three fp16 pieces (hi, mid, lo), then zeros
    const float xs = -s * base * 0x1p-15f;
    const _Float16 p0 = (_Float16)xs;
    const float r1 = xs - (float)p0;
    const _Float16 p1 = (_Float16)r1;
    const _Float16 p2 = (_Float16)(r1 - (float)p1);
    const half2_t d0 = {p0, p1}, d1 = {p2, (_Float16)0.f};
    out[NMF * 64] = j == 0 ? __builtin_bit_cast(uint32_t, d0) : j == 1 ? __builtin_bit_cast(uint32_t, d1) : 0u;
    // F = 2^(32 - r - e): what turns the accumulator back into code units times Eq. 1's rescale
    if (j == 0) gl(const_cast<float *>(L.xsum))[(size_t)(c * L.G + g) * kChunkCols + m] = __builtin_ldexpf(1.f, 32 - R - e);
}

__global__ __launch_bounds__(256) void xprep_kernel(const StackParams p) {
    const int lane = threadIdx.x & 63;
    const int job = __builtin_amdgcn_readfirstlane((int)((blockIdx.x * blockDim.x + threadIdx.x) >> 6));
    if (job >= p.n_jobs) return;
    int li = 0;
    if (p.table) {
        int lo = 0, hi = p.n_layers - 1;
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (load_desc(p.table + mid).job_start <= job) lo = mid; else hi = mid - 1;
        }
        li = lo;
    }
    const LayerDesc L = p.table ? load_desc(p.table + li) : p.single;
    const int local = job - L.job_start;
    const int c = local / L.G, g = local - c * L.G;
    switch (L.r) {
        case 2: xprep_job<2>(L, c, g, lane); break;
        case 3: xprep_job<3>(L, c, g, lane); break;
        case 4: xprep_job<4>(L, c, g, lane); break;
        case 6: xprep_job<6>(L, c, g, lane); break;
        default: xprep_job<8>(L, c, g, lane); break;
    }
}

// ------------------------------------------------------------------ main kernel
// D layout of a 32x32 accumulator: register v of lane l is D[8*(v/4) + 4*(l/32) + v%4][l%32];
// output column j = l%32 maps to batch column j%16 and tile-row half j/16.
struct LaneMap {
    int col;        // batch column inside the chunk
    int rowbase;    // tile row of v = 0: 32*(j/16) + 4*(l/32); row(v) = rowbase + 8*(v/4) + v%4
    bool b_live;    // as a B supplier the lane is k-half l/32 of output column j: non-zero only if l/32 == j/16
};
__device__ __forceinline__ LaneMap lane_map(int lane) {
    LaneMap m;
    const int j = lane & 31, hh = j >> 4, dh = lane >> 5;
    m.col = j & 15;
    m.rowbase = 32 * hh + 4 * dh;
    m.b_live = dh == hh;
    return m;
}

// Per-wave LDS: two stages of prepared activations (the B operands of one tile each) so
// that B is read just in time with ds_read instead of being held in 64..80 registers.
constexpr int kStageBytes = 6 * 1024;                 // >= (NMF + 1) * 256 for every width (NMF <= 20)
constexpr int kWaveLds = 2 * kStageBytes;
constexpr int kZeroOff = 4 * kWaveLds;                // 16 zero bytes after the four waves' stages
constexpr int kLdsBytes = kZeroOff + 16;

__device__ __forceinline__ float half_of(u32x2 v, int e) {
    const uint32_t w = e < 2 ? v.x : v.y;
    const uint16_t h = (uint16_t)(e & 1 ? w >> 16 : w & 0xFFFF);
    return (float)__builtin_bit_cast(_Float16, h);
}

template <int R> struct GemmCtx {
    using MF = Mfma<R>;
    static constexpr int NBLK = MF::NMF + 1;                // operand blocks per tile: the MFMAs' and the zero-offset's
    static constexpr int NXL = (NBLK * 256 + 1023) / 1024;  // 1 KiB wave-loads per tile of activations
    const LayerDesc &L;
    const LaneMap lm;
    const int lane, c;
    __amdgpu_buffer_rsrc_t xt;
    uint8_t *lds;   // this wave's two stages
    uint8_t *zero;  // 16 zero bytes

    __device__ __forceinline__ void load_w(uint32_t (&w)[4 * R], int u) const {
        const u32x4 MQ_GLOBAL *src = gl(reinterpret_cast<const u32x4 *>(L.Wp) + (size_t)u * (R * 64) + lane);
#pragma unroll
        for (int i = 0; i < R; ++i) {
            const u32x4 v = __builtin_nontemporal_load(src + i * 64);  // read once per call: streaming hint
            w[4 * i] = v.x; w[4 * i + 1] = v.y; w[4 * i + 2] = v.z; w[4 * i + 3] = v.w;
        }
    }
    // activations of group g of this chunk: NXL coalesced 16-byte loads (past the end of the buffer -> 0).
    // A lane copies the 16 bytes of batch column lane % 16 of four MFMA blocks; columns beyond M hold zeros,
    // so their lanes read out of range instead (0 comes back and no memory is touched: at M = 8 half the
    // activation traffic, which is as large as a 4-bit weight tile, is never requested).
    __device__ __forceinline__ void load_x(u32x4 (&xb)[NXL], int g) const {
        const bool live = c * kChunkCols + (lane & 15) < L.M;
        const uint32_t off = live ? (uint32_t)(c * L.G + g) * (NBLK * 256u) + (uint32_t)lane * 16u : 0x80000000u;
#pragma unroll
        for (int i = 0; i < NXL; ++i) xb[i] = __builtin_amdgcn_raw_buffer_load_b128(xt, off + i * 1024, 0, 0);
    }
    // (lanes that copy a batch column beyond M have nothing to store: nobody reads those bytes)
    __device__ __forceinline__ void store_x(const u32x4 (&xb)[NXL], int stage) const {
        if (c * kChunkCols + (lane & 15) >= L.M) return;
        u32x4 *dst = reinterpret_cast<u32x4 *>(lds + stage * kStageBytes) + lane;
#pragma unroll
        for (int i = 0; i < NXL; ++i) dst[i * 64] = xb[i];
    }
};

// One tile: NMF MFMAs on the masked fields, one on the zero-offset, then y += scale * (F * D).  B comes from LDS
// stage `stage`, read four MFMAs ahead of its use so that the LDS latency overlaps the previous MFMAs.
//   zl : zero-offset of the lane's OWN row (the lane is an A supplier of that row)
//   s4 : scales of the 16 rows the lane holds accumulator elements of
template <int R>
__device__ __forceinline__ void gemm_tile_math(const GemmCtx<R> &cx, const uint32_t (&w)[4 * R], int stage,
                                               const u32x2 (&s4)[4], _Float16 zl, float F, float (&yacc)[16]) {
    using T = Layout<R>;
    using MF = Mfma<R>;
    constexpr int kAhead = 4;
    constexpr int NBLK = MF::NMF + 1;
    // Lanes whose B operand is zero do not read at all (their registers are cleared once per tile): an LDS read
    // costs its bandwidth per active lane, and B operands are what the LDS pipe is busy with in this kernel.
    const u32x4 *bsrc = reinterpret_cast<const u32x4 *>(cx.lds + stage * kStageBytes) + cx.lm.col;
    constexpr int bstep = 16;  // u32x4 elements per operand block (256 bytes)
    u32x4 bq[kAhead];          // ring of B operands in flight
    static_for<kAhead>([&](auto i) { bq[i] = u32x4{0u, 0u, 0u, 0u}; });
    if (cx.lm.b_live) static_for<kAhead>([&](auto i) { bq[i] = bsrc[i * bstep]; });
    float16_t D;
#pragma unroll
    for (int v = 0; v < 16; ++v) D[v] = 0.f;
    static_for<MF::NMF>([&](auto mf) {
        constexpr int Q = mf / T::NOPS;
        constexpr Op o = T::op(mf % T::NOPS);
        uint32_t a[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint32_t v = w[(4 * Q + j) * T::UD + o.dw];
            if constexpr (o.sh != 0) v >>= o.sh;
            a[j] = v & ((uint32_t)o.mask * 0x10001u);
        }
        const u32x4 av = {a[0], a[1], a[2], a[3]};
        const u32x4 bv = bq[mf % kAhead];
        if constexpr (mf + kAhead < NBLK) {
            if (cx.lm.b_live) bq[mf % kAhead] = bsrc[(mf + kAhead) * bstep];
        }
        D = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8_t, av), __builtin_bit_cast(half8_t, bv), D,
                                                   0, 0, 0);
    });
    {   // zero-offset: A = (z', z', z', 0, ...) with z' = z * 2^(r-17), B = -X_g * 2^(e-15) in three pieces
        const _Float16 zs = zl * (_Float16)__builtin_ldexpf(1.f, R - 17);
        const half2_t zz = {zs, zs}, z0 = {zs, (_Float16)0.f};
        const u32x4 av = {__builtin_bit_cast(uint32_t, zz), __builtin_bit_cast(uint32_t, z0), 0u, 0u};
        D = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8_t, av),
                                                   __builtin_bit_cast(half8_t, bq[MF::NMF % kAhead]), D, 0, 0, 0);
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) yacc[v] = fmaf(half_of(s4[v >> 2], v & 3), D[v] * F, yacc[v]);
}

// Weight tiles a wave keeps in flight ahead of the one it is working on.  The ring has an even number of
// buffers (depth + 1) so that the two-deep ring of scales / zero / factor below keeps compile-time indices.
template <int R> struct GemmDepth {
    static constexpr int value = R <= 6 ? 3 : 1;
};

// Tiles [u_begin, u_end) of chunk c of one layer (tile index u = rb*G + g).
template <int R>
__device__ __forceinline__ void run_gemm_units(const LayerDesc &L, const StackParams &p, int c, int u_begin, int u_end,
                                               int wave, int lane, uint8_t *lds_wave, uint8_t *lds_zero) {
    using MF = Mfma<R>;
    using Ctx = GemmCtx<R>;
    constexpr int D = GemmDepth<R>::value, NB = D + 1;
    const uint32_t xt_bytes = (uint32_t)L.CB * L.G * (MF::NMF + 1) * 256u;
    LaneMap lmap = lane_map(lane);
    // a lane whose output column lies beyond M supplies zeros as B: it reads the 16 zero bytes instead of its stage
    lmap.b_live = lmap.b_live && c * kChunkCols + lmap.col < L.M;
    const Ctx cx{L, lmap, lane, c,
                 __builtin_amdgcn_make_buffer_rsrc(const_cast<uint4 *>(L.xt), 0, (int)xt_bytes, 0x00020000), lds_wave,
                 lds_zero};
    const LaneMap &lm = cx.lm;
    int rb = u_begin / L.G;
    int g = u_begin - rb * L.G;
    int ga = g;
    float yacc[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) yacc[v] = 0.f;
    const int col = c * kChunkCols + lm.col;
    const bool fast_store = (L.N & 3) == 0 && (reinterpret_cast<uintptr_t>(L.y) & 7) == 0;

    // ring of NB weight buffers with compile-time indices (no register copies); past the end
    // of the run the last tile is fetched again instead of branching around the loads
    uint32_t w[NB][4 * R];
    int u_pf = u_begin;
    auto prefetch_w = [&](uint32_t (&dst)[4 * R]) {
        cx.load_w(dst, u_pf);
        if (u_pf + 1 < u_end) ++u_pf;
    };
    // Scales, zero-offset and rescale factor of a tile are fetched one tile ahead, BEFORE that iteration's weight
    // prefetch: loads return in order, so waiting for anything issued after the prefetch would wait for the prefetch
    // itself (a full trip to HBM per tile).  Every wait of the loop is then for a load at least one tile old.
    static_assert(NB % 2 == 0, "the two-deep meta ring relies on an even unroll");
    struct TileMeta {
        u32x2 s4[4];
        _Float16 zl;
        float F;
    } meta[2];
    auto load_meta = [&](TileMeta &t, int ut, int gt) {
        const u32x2 MQ_GLOBAL *sp = gl(reinterpret_cast<const u32x2 *>(L.st + (size_t)ut * 64 + lm.rowbase));
#pragma unroll
        for (int q = 0; q < 4; ++q) t.s4[q] = __builtin_nontemporal_load(sp + 2 * q);
        // symmetric layer (no zero-offset array): every zero-offset is 2^(c-1)
        t.zl = L.zt ? __builtin_nontemporal_load(gl(L.zt) + (size_t)ut * 64 + lane) : (_Float16)(float)(1 << (kC - 1));
        t.F = gl(L.xsum)[(size_t)(c * L.G + gt) * kChunkCols + lm.col];
    };
    {
        u32x4 xb[Ctx::NXL];
        cx.load_x(xb, g);
        load_meta(meta[0], u_begin, g);
        static_for<D>([&](auto j) { prefetch_w(w[j]); });
        cx.store_x(xb, 0);
    }
    int u = u_begin;
    int st = 0;  // LDS stage holding the current tile's activations
    while (u < u_end) {
        static_for<NB>([&](auto j) {
            if (u >= u_end) return;
            const bool more = u + 1 < u_end;
            const int g_next = more ? (g + 1 == L.G ? 0 : g + 1) : g;
            u32x4 xb[Ctx::NXL];
            cx.load_x(xb, g_next);              // first: it is awaited first (loads return in order)
            load_meta(meta[(j + 1) % 2], more ? u + 1 : u, g_next);
            __builtin_amdgcn_sched_barrier(0);  // ... and these must really be issued ahead of the prefetch
            prefetch_w(w[(j + D) % NB]);
            __builtin_amdgcn_sched_barrier(0);  // keep the loads up here, ahead of the math
            gemm_tile_math<R>(cx, w[j], st, meta[j % 2].s4, meta[j % 2].zl, meta[j % 2].F, yacc);
            cx.store_x(xb, st ^ 1);
            st ^= 1;
            ++g;
            ++u;
            if (g == L.G || u == u_end) {
                const uint64_t a = L.cost_start + ((uint64_t)c * L.RB * L.G + (uint64_t)rb * L.G) * L.cost;
                const int row0 = rb * kRowBlock + lm.rowbase;
                finish_row_block<16>(L, p, p.cnt + L.cnt_off + c * L.RB + rb, a, ga, g, yacc, wave, lane,
                                     [&](const float(&tot)[16]) {
                                         if (col >= L.M) return;
                                         _Float16 MQ_GLOBAL *yrow = gl(L.y + (size_t)col * L.N);
#pragma unroll
                                         for (int q = 0; q < 4; ++q) {
                                             const int row = row0 + 8 * q;
                                             if (fast_store && row + 3 < L.N) {
                                                 const half2_t lo = {(_Float16)tot[4 * q], (_Float16)tot[4 * q + 1]};
                                                 const half2_t hi = {(_Float16)tot[4 * q + 2], (_Float16)tot[4 * q + 3]};
                                                 const u32x2 pk = {__builtin_bit_cast(uint32_t, lo),
                                                                   __builtin_bit_cast(uint32_t, hi)};
                                                 *(u32x2 MQ_GLOBAL *)(yrow + row) = pk;
                                             } else {
#pragma unroll
                                                 for (int e = 0; e < 4; ++e)
                                                     if (row + e < L.N) yrow[row + e] = (_Float16)tot[4 * q + e];
                                             }
                                         }
                                     });
                ++rb;
                g = 0;
                ga = 0;
#pragma unroll
                for (int v = 0; v < 16; ++v) yacc[v] = 0.f;
            }
        });
    }
}

__global__ __launch_bounds__(256, 2) void gemm_stack_kernel(const StackParams p) {
    __shared__ __attribute__((aligned(16))) uint8_t lds[kLdsBytes];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)((blockIdx.x * blockDim.x + threadIdx.x) >> 6));
    if (wave >= p.nwaves) return;
    uint8_t *lds_wave = lds + (threadIdx.x >> 6) * kWaveLds;
    uint8_t *lds_zero = lds + kZeroOff;
    if (lane < 4) reinterpret_cast<uint32_t *>(lds_zero)[lane] = 0u;  // every wave writes the same zeros before it reads them
    walk_tiles(p, wave, [&](const LayerDesc &L, int u_begin, int u_end) {
        const int per_chunk = L.RB * L.G;
        for (int c = u_begin / per_chunk; c < L.CB && c * per_chunk < u_end; ++c) {
            const int lo = (u_begin > c * per_chunk ? u_begin : c * per_chunk) - c * per_chunk;
            const int hi = (u_end < (c + 1) * per_chunk ? u_end : (c + 1) * per_chunk) - c * per_chunk;
            if (lo >= hi) continue;
            switch (L.r) {
                case 2: run_gemm_units<2>(L, p, c, lo, hi, wave, lane, lds_wave, lds_zero); break;
                case 3: run_gemm_units<3>(L, p, c, lo, hi, wave, lane, lds_wave, lds_zero); break;
                case 4: run_gemm_units<4>(L, p, c, lo, hi, wave, lane, lds_wave, lds_zero); break;
                case 6: run_gemm_units<6>(L, p, c, lo, hi, wave, lane, lds_wave, lds_zero); break;
                default: run_gemm_units<8>(L, p, c, lo, hi, wave, lane, lds_wave, lds_zero); break;
            }
        }
    });
}

static int gemm_resident_waves() {
    static int cached = 0;
    if (cached) return cached;
    int dev = 0, cus = 0, blocks = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&blocks, gemm_stack_kernel, 256, 0) != hipSuccess) return 0;
    if (blocks < 1) blocks = 1;
    int w = cus * blocks * 4;
    if (w > kMaxWavesMfma) w = kMaxWavesMfma;
    cached = w;
    return w;
}

hipError_t launch_stack_mfma(StackParams p, int max_cost, hipStream_t s) {
    int hw = gemm_resident_waves();
    if (hw <= 0) return hipErrorUnknown;
    if (p.worker_cap && hw > p.worker_cap) hw = p.worker_cap;
    // shares of at least four tiles: with one tile per wave a small layer (a 4096 x 4096 one has 2048 tiles) hands
    // every row block over between as many waves as it has groups, which costs more than the parallelism gains
    // (measured on the Llama-2-7B shapes at M = 8: 26 -> 19 us per call)
    uint64_t cap = p.cost_total / ((uint64_t)max_cost * 4);
    if (cap < 1) cap = 1;
    p.nwaves = (int)(cap < (uint64_t)hw ? cap : (uint64_t)hw);
    p.nworkers = p.nwaves;
    const hipError_t e = launch(xprep_kernel, dim3((unsigned)((p.n_jobs + 3) / 4)), dim3(256), 0, s, p);
    if (e != hipSuccess) return e;
    return launch(gemm_stack_kernel, dim3((unsigned)((p.nwaves + 3) / 4)), dim3(256), 0, s, p);
}

}  // namespace mq
