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
// (16 columns x 8 halves each) and the per-column group sums X_g.
template <int R> __device__ __forceinline__ void xprep_job(const LayerDesc &L, int c, int g, int lane) {
    using T = Layout<R>;
    constexpr int NMF = Mfma<R>::NMF;
    const int m = lane >> 2, j = lane & 3;
    const int col = c * kChunkCols + m;
    const bool live = col < L.M;
    const uint32_t MQ_GLOBAL *xrow =
        gl(reinterpret_cast<const uint32_t *>(L.x + (size_t)(live ? col : 0) * L.K) + (size_t)g * 64);
    uint32_t MQ_GLOBAL *out =
        gl(reinterpret_cast<uint32_t *>(const_cast<uint4 *>(L.xt)) + ((size_t)(c * L.G + g) * NMF) * 64 + lane);
    static_for<NMF>([&](auto mf) {
        constexpr int Q = mf / T::NOPS;
        constexpr Op o = T::op(mf % T::NOPS);
        // dword j of the lane's operand = activation pair of unit 4Q+j, field o
        const uint32_t v = live ? xrow[(4 * Q + j) * T::PPU + o.pair] : 0u;
        out[mf * 64] = v;
    });
    // X_g for column m: lanes 4m..4m+3 each sum a quarter of the group
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s = dot2(live ? xrow[j * 16 + i] : 0u, 0x3C003C00u, s);
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
template <int R> struct GemmTile {
    uint32_t w[4 * R];
    u32x2 s4[4], z4[4];  // scale / zero of the 16 tile rows this lane holds in the D layout
    float xg;            // X_g of this lane's output column
};

// D layout of a 32x32 accumulator: register v of lane l is D[8*(v/4) + 4*(l/32) + v%4][l%32];
// output column j = l%32 maps to batch column j%16 and tile-row half j/16.
struct LaneMap {
    int col;      // batch column inside the chunk
    int rowbase;  // tile row of v = 0: 32*(j/16) + 4*(l/32); row(v) = rowbase + 8*(v/4) + v%4
    uint32_t boff;  // byte offset of this lane's B operand inside a 256-byte MFMA block, or out of range
};
__device__ __forceinline__ LaneMap lane_map(int lane) {
    LaneMap m;
    const int j = lane & 31, hh = j >> 4, dh = lane >> 5;
    m.col = j & 15;
    m.rowbase = 32 * hh + 4 * dh;
    // as a B supplier the lane is k-half dh of output column j: non-zero only if dh == hh
    m.boff = dh == hh ? (uint32_t)(m.col * 16) : 0xF0000000u;
    return m;
}

template <int R>
__device__ __forceinline__ void load_gemm_tile(GemmTile<R> &t, const LayerDesc &L, int c, int u, int g,
                                               const LaneMap &lm, int lane) {
    const u32x4 MQ_GLOBAL *src = gl(reinterpret_cast<const u32x4 *>(L.Wp) + (size_t)u * (R * 64) + lane);
#pragma unroll
    for (int i = 0; i < R; ++i) {
        const u32x4 v = src[i * 64];
        t.w[4 * i] = v.x; t.w[4 * i + 1] = v.y; t.w[4 * i + 2] = v.z; t.w[4 * i + 3] = v.w;
    }
    const u32x2 MQ_GLOBAL *s = gl(reinterpret_cast<const u32x2 *>(L.st + (size_t)u * 64 + lm.rowbase));
    const u32x2 MQ_GLOBAL *z = gl(reinterpret_cast<const u32x2 *>(L.zt + (size_t)u * 64 + lm.rowbase));
#pragma unroll
    for (int q = 0; q < 4; ++q) { t.s4[q] = s[2 * q]; t.z4[q] = z[2 * q]; }
    t.xg = gl(L.xsum)[(size_t)(c * L.G + g) * kChunkCols + lm.col];
}

__device__ __forceinline__ float half_of(u32x2 v, int e) {
    const uint32_t w = e < 2 ? v.x : v.y;
    const uint16_t h = (uint16_t)(e & 1 ? w >> 16 : w & 0xFFFF);
    return (float)__builtin_bit_cast(_Float16, h);
}

// B operands of one tile: NMF x 16 bytes per lane.  They are loaded one tile ahead, each
// register quad being refilled right after the MFMA that consumed it.
template <int R> struct BRegs {
    uint4_t b[Mfma<R>::NMF];
};
template <int R>
__device__ __forceinline__ void load_b_all(BRegs<R> &B, __amdgpu_buffer_rsrc_t xt, uint32_t voff) {
    static_for<Mfma<R>::NMF>([&](auto mf) { B.b[mf] = __builtin_amdgcn_raw_buffer_load_b128(xt, voff + mf * 256, 0, 0); });
}

// voff_next: this lane's B offset for the NEXT tile of the run (any valid tile if there is none).
template <int R>
__device__ __forceinline__ void gemm_tile_math(const GemmTile<R> &t, BRegs<R> &B, __amdgpu_buffer_rsrc_t xt,
                                               uint32_t voff_next, float (&yacc)[16]) {
    using T = Layout<R>;
    using MF = Mfma<R>;
    float16_t D[T::NKEYS];
#pragma unroll
    for (int k = 0; k < T::NKEYS; ++k)
#pragma unroll
        for (int v = 0; v < 16; ++v) D[k][v] = 0.f;
    static_for<MF::NMF>([&](auto mf) {
        constexpr int Q = mf / T::NOPS;
        constexpr int oi = mf % T::NOPS;
        constexpr Op o = T::op(oi);
        constexpr int key = key_index<R>(oi);
        uint32_t a[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint32_t v = t.w[(4 * Q + j) * T::UD + o.dw];
            if constexpr (o.sh != 0) v >>= o.sh;
            a[j] = v & ((uint32_t)o.mask * 0x10001u);
        }
        const uint4_t av = {a[0], a[1], a[2], a[3]};
        D[key] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8_t, av),
                                                        __builtin_bit_cast(half8_t, B.b[mf]), D[key], 0, 0, 0);
        B.b[mf] = __builtin_amdgcn_raw_buffer_load_b128(xt, voff_next + mf * 256, 0, 0);
    });
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const float s = half_of(t.s4[v >> 2], v & 3), z = half_of(t.z4[v >> 2], v & 3);
        float d = 0.f;
        static_for<T::NKEYS>([&](auto k) { d = fmaf(D[k][v], __builtin_ldexpf(1.f, 24 - T::key(k) + kC - R), d); });
        yacc[v] = fmaf(s, fmaf(-z, t.xg, d), yacc[v]);
    }
}

// Tiles [u_begin, u_end) of chunk c of one layer (tile index u = rb*G + g).
template <int R>
__device__ __forceinline__ void run_gemm_units(const LayerDesc &L, const StackParams &p, int c, int u_begin, int u_end,
                                               int wave, int lane) {
    using MF = Mfma<R>;
    const LaneMap lm = lane_map(lane);
    const uint32_t xt_bytes = (uint32_t)L.CB * L.G * MF::NMF * 256u;
    const __amdgpu_buffer_rsrc_t xt =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint4 *>(L.xt), 0, (int)xt_bytes, 0x00020000);
    int rb = u_begin / L.G;
    int g = u_begin - rb * L.G;
    int ga = g;
    float yacc[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) yacc[v] = 0.f;
    const int col = c * kChunkCols + lm.col;
    const bool fast_store = (L.N & 3) == 0 && (reinterpret_cast<uintptr_t>(L.y) & 7) == 0;

    GemmTile<R> cur, nxt;
    BRegs<R> B;
    load_gemm_tile<R>(cur, L, c, u_begin, g, lm, lane);
    load_b_all<R>(B, xt, lm.boff + (uint32_t)(c * L.G + g) * (MF::NMF * 256u));
    for (int u = u_begin; u < u_end; ++u) {
        const int g_next = (u + 1 < u_end) ? (g + 1 == L.G ? 0 : g + 1) : g;
        if (u + 1 < u_end) load_gemm_tile<R>(nxt, L, c, u + 1, g_next, lm, lane);
        gemm_tile_math<R>(cur, B, xt, lm.boff + (uint32_t)(c * L.G + g_next) * (MF::NMF * 256u), yacc);
        ++g;
        if (g == L.G || u + 1 == u_end) {
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
        cur = nxt;
    }
}

__global__ __launch_bounds__(256, 2) void gemm_stack_kernel(const StackParams p) {
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)((blockIdx.x * blockDim.x + threadIdx.x) >> 6));
    if (wave >= p.nwaves) return;
    walk_tiles(p, wave, [&](const LayerDesc &L, int u_begin, int u_end) {
        const int per_chunk = L.RB * L.G;
        for (int c = u_begin / per_chunk; c < L.CB && c * per_chunk < u_end; ++c) {
            const int lo = (u_begin > c * per_chunk ? u_begin : c * per_chunk) - c * per_chunk;
            const int hi = (u_end < (c + 1) * per_chunk ? u_end : (c + 1) * per_chunk) - c * per_chunk;
            if (lo >= hi) continue;
            switch (L.r) {
                case 2: run_gemm_units<2>(L, p, c, lo, hi, wave, lane); break;
                case 3: run_gemm_units<3>(L, p, c, lo, hi, wave, lane); break;
                case 4: run_gemm_units<4>(L, p, c, lo, hi, wave, lane); break;
                case 6: run_gemm_units<6>(L, p, c, lo, hi, wave, lane); break;
                default: run_gemm_units<8>(L, p, c, lo, hi, wave, lane); break;
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
    const int hw = gemm_resident_waves();
    if (hw <= 0) return hipErrorUnknown;
    uint64_t cap = p.cost_total / (uint64_t)max_cost;
    if (cap < 1) cap = 1;
    p.nwaves = (int)(cap < (uint64_t)hw ? cap : (uint64_t)hw);
    (void)hipGetLastError();  // drop stale errors of earlier, unrelated calls
    hipLaunchKernelGGL(xprep_kernel, dim3((unsigned)((p.n_jobs + 3) / 4)), dim3(256), 0, s, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(gemm_stack_kernel, dim3((unsigned)((p.nwaves + 3) / 4)), dim3(256), 0, s, p);
    return hipGetLastError();
}

}  // namespace mq
