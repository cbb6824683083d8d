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
// Per tile, group-local sums stay in one 32x32 accumulator per field key; per
// group  y += scale * (2^(8-r) * D - zero * X_g)  in fp32, exactly as on the
// vector-ALU path (integer codes stay exact, scales are never rounded to fp16).
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
template <int R> __device__ __forceinline__ void xprep_job(const LayerDesc &L, int c, int g, int lane) {
    using T = Layout<R>;
    constexpr int NMF = Mfma<R>::NMF;
    const int m = lane >> 2, j = lane & 3;
    const int col = c * kChunkCols + m;
    const uint32_t live = col < L.M ? 0xFFFFFFFFu : 0u;
    const uint32_t MQ_GLOBAL *xrow =
        gl(reinterpret_cast<const uint32_t *>(L.x + (size_t)(live ? col : 0) * L.K) + (size_t)g * 64);
    uint32_t MQ_GLOBAL *out =
        gl(reinterpret_cast<uint32_t *>(const_cast<uint4 *>(L.xt)) + ((size_t)(c * L.G + g) * NMF) * 64 + lane);
    uint32_t v[NMF];
    static_for<NMF>([&](auto mf) {
        constexpr int Q = mf / T::NOPS;
        constexpr Op o = T::op(mf % T::NOPS);
        // dword j of the lane's operand = activation pair of unit 4Q+j, field o
        v[mf] = xrow[(4 * Q + j) * T::PPU + o.pair];
    });
    uint32_t q[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) q[i] = xrow[j * 16 + i];
    static_for<NMF>([&](auto mf) { out[mf * 64] = v[mf] & live; });
    // X_g for column m: lanes 4m..4m+3 each sum a quarter of the group
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s = dot2(q[i] & live, 0x3C003C00u, s);
    s = dpp_add<0xB1>(s);
    s = dpp_add<0x4E>(s);
    if (j == 0) gl(const_cast<float *>(L.xsum))[(size_t)(c * L.G + g) * kChunkCols + m] = s;
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
constexpr int kStageBytes = 5 * 1024;                 // >= NMF * 256 for every width (NMF <= 20)
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
    static constexpr int NXL = (MF::NMF * 256 + 1023) / 1024;  // 1 KiB wave-loads per tile of activations
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
        const uint32_t off = live ? (uint32_t)(c * L.G + g) * (MF::NMF * 256u) + (uint32_t)lane * 16u : 0x80000000u;
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

// MFMA order of a tile: key by key (so that one 32x32 accumulator is live at a time).
template <int R> struct MfmaOrder {
    using T = Layout<R>;
    static constexpr int NMF = Mfma<R>::NMF;
    // i-th MFMA in issue order -> index mf = Q * NOPS + oi
    static constexpr int at(int i) {
        int n = 0;
        for (int key = 0; key < T::NKEYS; ++key)
            for (int mf = 0; mf < NMF; ++mf)
                if (key_index<R>(mf % T::NOPS) == key) {
                    if (n == i) return mf;
                    ++n;
                }
        return -1;
    }
    static constexpr int key_of(int i) { return key_index<R>(at(i) % T::NOPS); }
    static constexpr bool last_of_key(int i) { return i + 1 == NMF || key_of(i + 1) != key_of(i); }
    static constexpr bool first_of_key(int i) { return i == 0 || key_of(i - 1) != key_of(i); }
};

// One tile: NMF MFMAs, then the per-group scale / zero step.  B comes from LDS stage `stage`,
// read four MFMAs ahead of its use so that the LDS latency overlaps the previous MFMAs.
template <int R>
__device__ __forceinline__ void gemm_tile_math(const GemmCtx<R> &cx, const uint32_t (&w)[4 * R], int stage,
                                               const u32x2 (&s4)[4], const u32x2 (&z4)[4], float xg,
                                               float (&yacc)[16]) {
    using T = Layout<R>;
    using MF = Mfma<R>;
    using Ord = MfmaOrder<R>;
    constexpr int kAhead = 4;
    const u32x4 *bsrc = cx.lm.b_live ? reinterpret_cast<const u32x4 *>(cx.lds + stage * kStageBytes) + cx.lm.col
                                     : reinterpret_cast<const u32x4 *>(cx.zero);
    const int bstep = cx.lm.b_live ? 16 : 0;  // u32x4 elements per MFMA block (256 bytes)
    u32x4 bq[kAhead];                          // ring of B operands in flight
    static_for<kAhead>([&](auto i) {
        if constexpr (i < MF::NMF) bq[i] = bsrc[Ord::at(i) * bstep];
    });
    // field value = digit * 2^(key-24): back to code units, then Eq. 1's rescale 2^(8-r)
    float dsum[16];
    float16_t D;
    static_for<MF::NMF>([&](auto i) {
        constexpr int mf = Ord::at(i);
        constexpr int Q = mf / T::NOPS;
        constexpr Op o = T::op(mf % T::NOPS);
        constexpr int key = Ord::key_of(i);
        if constexpr (Ord::first_of_key(i)) {
#pragma unroll
            for (int v = 0; v < 16; ++v) D[v] = 0.f;
        }
        uint32_t a[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint32_t v = w[(4 * Q + j) * T::UD + o.dw];
            if constexpr (o.sh != 0) v >>= o.sh;
            a[j] = v & ((uint32_t)o.mask * 0x10001u);
        }
        const u32x4 av = {a[0], a[1], a[2], a[3]};
        const u32x4 bv = bq[i % kAhead];
        if constexpr (i + kAhead < MF::NMF) bq[i % kAhead] = bsrc[Ord::at(i + kAhead) * bstep];
        D = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8_t, av), __builtin_bit_cast(half8_t, bv), D,
                                                   0, 0, 0);
        if constexpr (Ord::last_of_key(i)) {
            const float ck = __builtin_ldexpf(1.f, 24 - T::key(key) + kC - R);
#pragma unroll
            for (int v = 0; v < 16; ++v) dsum[v] = key == 0 ? D[v] * ck : fmaf(D[v], ck, dsum[v]);
        }
    });
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const float s = half_of(s4[v >> 2], v & 3), z = half_of(z4[v >> 2], v & 3);
        yacc[v] = fmaf(s, fmaf(-z, xg, dsum[v]), yacc[v]);
    }
}

// Weight tiles a wave keeps in flight ahead of the one it is working on (about 8 KB).
template <int R> struct GemmDepth {
    static constexpr int value = R <= 3 ? 4 : R == 4 ? 3 : 2;
};

// Tiles [u_begin, u_end) of chunk c of one layer (tile index u = rb*G + g).
template <int R>
__device__ __forceinline__ void run_gemm_units(const LayerDesc &L, const StackParams &p, int c, int u_begin, int u_end,
                                               int wave, int lane, uint8_t *lds_wave, uint8_t *lds_zero) {
    using MF = Mfma<R>;
    using Ctx = GemmCtx<R>;
    constexpr int D = GemmDepth<R>::value, NB = D + 1;
    const uint32_t xt_bytes = (uint32_t)L.CB * L.G * MF::NMF * 256u;
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
    {
        u32x4 xb[Ctx::NXL];
        cx.load_x(xb, g);
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
            __builtin_amdgcn_sched_barrier(0);  // ... and must really be issued first
            prefetch_w(w[(j + D) % NB]);
            u32x2 s4[4], z4[4];
            const u32x2 MQ_GLOBAL *sp = gl(reinterpret_cast<const u32x2 *>(L.st + (size_t)u * 64 + lm.rowbase));
            const u32x2 MQ_GLOBAL *zp = gl(reinterpret_cast<const u32x2 *>(L.zt + (size_t)u * 64 + lm.rowbase));
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                s4[q] = __builtin_nontemporal_load(sp + 2 * q);
                z4[q] = __builtin_nontemporal_load(zp + 2 * q);
            }
            const float xg = gl(L.xsum)[(size_t)(c * L.G + g) * kChunkCols + lm.col];
            __builtin_amdgcn_sched_barrier(0);  // keep the loads up here, ahead of the math
            gemm_tile_math<R>(cx, w[j], st, s4, z4, xg, yacc);
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
