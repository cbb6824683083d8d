// Small batch (4 < M <= 16): the same sliced linear layer on the matrix cores (Section 4 of the paper switches to
// TensorCores from batch 8; here the switch is at M = 5).  Same packed tiles, same persistent schedule and
// split-K hand-off (mq_device.h) as the vector-ALU kernel.
//
// MFMA mapping.  v_mfma_f32_32x32x16_f16 computes D[32x32] += A[32x16] * B[16x32]; lane l supplies
// A[l%32][8*(l/32) .. +7] and B[8*(l/32) .. +7][l%32].  In the tile layout lane l owns row l of the 64-row tile,
// and four masked dwords of a lane (the same bit-field of four units) are eight fp16 subnormals = eight columns
// k_0..k_7 of that row, i.e. already a valid A operand: lanes 0..31 feed tile rows 0..31 as the first k-half,
// lanes 32..63 feed tile rows 32..63 as the second k-half, both halves carrying the SAME eight columns.  B separates
// the two halves again: for output column j < 16 it holds x[j][k_e] in the first k-half and zero in the second, for
// j >= 16 the other way round.  Then
//   D[i][j] = sum_e W[row i][k_e] * x[j][k_e] (j < 16),   D[i][j] = sum_e W[row 32 + i][k_e] * x[j - 16][k_e] (j >= 16)
// so one MFMA handles 64 rows x 8 columns of W x 16 batch rows (half of B is zeros: the price of sharing one weight
// layout with the batch-1 kernel; the matrix pipe is not what bounds this kernel).
//
// One accumulation per tile.  A masked field is the fp16 subnormal digit * 2^(p-24) and stands for digit * 2^d of the
// code (p = position of the field in its half, d = first code bit it carries).  The B operand of each MFMA is the
// activations times 2^(e - (p - d)), prepared once per call by xprep_kernel: every MFMA of a tile then adds
// code-part * x * 2^(e-24) into the same accumulators and no vector instruction touches them before the group is
// complete.  e is a block exponent per (group, batch column) chosen so that the largest |x| of the group lands in
// [2^14, 2^15): the scaling is exact for every element within 2^-22 of the group's largest (smaller ones lose low
// bits worth less than 2^-38 of the largest product: far below the fp32 accumulation itself).
// The zero-offset rides on the matrix core as well: one more MFMA per tile multiplies the row's zero
// (A = z * 2^(r-17), exact for every zero >= 2) by -X_g * 2^(e-15) split into three fp16 pieces (relative error 2^-33),
// so that D = 2^(e+r-32) * sum_k x_k * (S_k - z).  Per group and accumulator element what is left for the vector ALUs
// is  y += scale * (F * D),  F = 2^(32-r-e)  from the prep kernel: integer codes stay exact and scales are never
// rounded to fp16, as on the vector-ALU path.
//
// Work split and memory pipeline.  A workgroup of eight waves walks a run of super-tiles (512 rows x one group);
// wave w owns row block 8*srb + w.  Everything travels global -> LDS without registers (mq_dma.h): the prepared
// activations of a group (6 KB, shared by the eight waves) into one of the stages, each wave's next weight tiles
// with their scales and zeros into a ring of its own.  Loads retire in order per wave, so whatever a tile needs must
// be as old as its weights when it is needed: with every transfer issued from assembly and every wait written out
// (how many LATER transfers may still be in flight), a tile's operands are always the oldest transfers of the wave
// and the prefetch distance is what the ring says.  (Left to the compiler, the activation and scale loads of the next
// tile, issued behind the weight prefetch of a tile three ahead, made every tile wait for that prefetch.)
#include "mq_device.h"
#include "mq_dma.h"

namespace mq {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float16_t __attribute__((ext_vector_type(16)));

template <int R> struct Mfma {
    using T = Layout<R>;
    static constexpr int NU = 4 * R / T::UD;       // units per lane and tile
    static constexpr int NQ = NU / 4;              // unit quads
    static constexpr int NMF = NQ * T::NOPS;       // MFMAs per tile on the masked fields
    static constexpr int NBLK = NMF + 1;           // operand blocks per tile: theirs and the zero-offset's
    static_assert(NU % 4 == 0, "units must come in quads");
};
// Activation block of a group: NBLK operand blocks of 272 bytes = 16 batch columns x 16 bytes (the eight halves a lane
// supplies as B) followed by 16 bytes that are always zero: a lane whose B operand is zero (the other k-half) reads
// those, so that no B read is masked.  The 16 factors F sit at the end.
constexpr int kOpBlockStride = 272;
constexpr int kFactorOff = kNarrowXtBlockBytes - 64;  // 16 floats F at the end of an activation block
static_assert(Mfma<2>::NBLK * kOpBlockStride <= kFactorOff && Mfma<3>::NBLK * kOpBlockStride <= kFactorOff &&
                  Mfma<4>::NBLK * kOpBlockStride <= kFactorOff && Mfma<6>::NBLK * kOpBlockStride <= kFactorOff &&
                  Mfma<8>::NBLK * kOpBlockStride <= kFactorOff,
              "operand blocks and factors must fit the activation block");

// ------------------------------------------------------------------ activation prep
// One wave per (layer, group): writes the activation block of the group: the B operands of the NMF MFMAs of a tile
// (16 columns x 8 halves each, scaled), the zero-offset block, and the factors F.  Branch-free: columns beyond M
// read column 0 and are masked to zero, all loads are issued before the stores.
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
template <int R> __device__ __forceinline__ void xprep_job(const LayerDesc &L, int g, int lane) {
    using T = Layout<R>;
    constexpr int NMF = Mfma<R>::NMF;
    const int m = lane >> 2, j = lane & 3;
    const uint32_t live = m < L.M ? 0xFFFFFFFFu : 0u;
    const uint32_t MQ_GLOBAL *xrow =
        gl(reinterpret_cast<const uint32_t *>(L.x + (size_t)(live ? m : 0) * L.K) + (size_t)g * 64);
    uint8_t *block = reinterpret_cast<uint8_t *>(const_cast<uint4 *>(L.xt)) + (size_t)g * kNarrowXtBlockBytes;
    uint32_t MQ_GLOBAL *out = gl(reinterpret_cast<uint32_t *>(block)) + lane;
    constexpr int kBlkDw = kOpBlockStride / 4;  // block stride in dwords
    uint32_t v[NMF];
    static_for<NMF>([&](auto mf) {
        constexpr int Q = mf / T::NOPS;
        constexpr Op o = T::op(mf % T::NOPS);
        // dword j of the lane's operand = activation pair of unit 4Q+j, field o
        v[mf] = x_pair(xrow[(4 * Q + j) * T::PPU + o.pair], L.flags) & live;
    });
    uint32_t q[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) q[i] = x_pair(xrow[j * 16 + i], L.flags) & live;
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
        out[mf * kBlkDw] = scale_pair(v[mf], base * __builtin_ldexpf(1.f, -key));
    });
    // the always-zero 16 bytes behind every operand block
    if (lane < 4) {
#pragma unroll
        for (int b = 0; b <= NMF; ++b) out[b * kBlkDw + 64] = 0u;
    }
    // the zero-offset block: -X_g * 2^(e-15) in three fp16 pieces (hi, mid, lo), then zeros
    const float xs = -s * base * 0x1p-15f;
    const _Float16 p0 = (_Float16)xs;
    const float r1 = xs - (float)p0;
    const _Float16 p1 = (_Float16)r1;
    const _Float16 p2 = (_Float16)(r1 - (float)p1);
    const half2_t d0 = {p0, p1}, d1 = {p2, (_Float16)0.f};
    out[NMF * kBlkDw] = j == 0 ? __builtin_bit_cast(uint32_t, d0) : j == 1 ? __builtin_bit_cast(uint32_t, d1) : 0u;
    // F = 2^(32 - r - e): what turns the accumulator back into code units times Eq. 1's rescale
    if (j == 0) gl(reinterpret_cast<float *>(block + kFactorOff))[m] = __builtin_ldexpf(1.f, 32 - R - e);
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
    const int g = job - L.job_start;
    switch (L.r) {
        case 2: xprep_job<2>(L, g, lane); break;
        case 3: xprep_job<3>(L, g, lane); break;
        case 4: xprep_job<4>(L, g, lane); break;
        case 6: xprep_job<6>(L, g, lane); break;
        default: xprep_job<8>(L, g, lane); break;
    }
}

// ------------------------------------------------------------------ main kernel
// D layout of a 32x32 accumulator: register v of lane l is D[8*(v/4) + 4*(l/32) + v%4][l%32];
// output column j = l%32 maps to batch column j%16 and tile-row half j/16.
struct LaneMap {
    int col;        // batch column
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

// LDS plan of a workgroup (one per compute unit): activation stages shared by the eight waves (one being read, the
// others landing) and per wave a ring of NBR weight tiles with their scale and zero lines.
constexpr int kNarrowWaves = kNarrowRowBlocks;  // waves per workgroup = row blocks per super-tile
constexpr int kStageBytes = kNarrowXtBlockBytes;
constexpr int narrow_slot_bytes(int R) { return R * 1024 + 256; }
constexpr int narrow_ring(int R) { return R <= 4 ? 3 : 2; }
constexpr int narrow_stages(int R) { return narrow_ring(R) + 1; }  // activations need the same lead as the weights
constexpr int narrow_lds_bytes(int R) {
    return narrow_stages(R) * kStageBytes + kNarrowWaves * narrow_ring(R) * narrow_slot_bytes(R);
}
constexpr int narrow_lds_bytes_max() {
    int m = 0;
    for (int r : {2, 3, 4, 6, 8}) m = narrow_lds_bytes(r) > m ? narrow_lds_bytes(r) : m;
    return m;
}
static_assert(narrow_lds_bytes_max() <= 160 * 1024, "LDS plan does not fit");

__device__ __forceinline__ float half_of(u32x2 v, int e) {
    const uint32_t w = e < 2 ? v.x : v.y;
    const uint16_t h = (uint16_t)(e & 1 ? w >> 16 : w & 0xFFFF);
    return (float)__builtin_bit_cast(_Float16, h);
}

// Super-tiles [u_begin, u_end) of one layer (u = srb * G + g), for the whole workgroup.
template <int R>
__device__ __forceinline__ void run_narrow_units(const LayerDesc &L, const StackParams &p, int u_begin, int u_end,
                                                 int worker, int wv, int lane, MQ_LDS uint8_t *lds) {
    using T = Layout<R>;
    using MF = Mfma<R>;
    constexpr int NBR = narrow_ring(R), NST = narrow_stages(R);
    constexpr int kSlot = narrow_slot_bytes(R);
    constexpr int kTileOps = R + 2;         // transfers per weight tile: R lines, scales, zeros
    constexpr int kBody = 1 + kTileOps;     // transfers a wave issues per tile body: one activation line first
    const int G = L.G;
    const int rb_real = (L.N + kRowBlock - 1) / kRowBlock;
    const uint8_t *xt = reinterpret_cast<const uint8_t *>(L.xt);
    MQ_LDS uint8_t *ring = lds + NST * kStageBytes + wv * (NBR * kSlot);
    const LaneMap lm = lane_map(lane);

    int srb = u_begin / G;
    int g = u_begin - srb * G;
    int ga = g;
    float yacc[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) yacc[v] = 0.f;

    // ---- weights: kTileOps transfers per tile into ring slot `slot`.  The number of transfers per tile body must
    // not depend on the data, so past the end of the run there are as many, but of one line of the last tile over and
    // over (cache hits: a run of a single call is short, and whole tiles fetched for nothing would be a fifth of its
    // traffic); nobody reads what they bring.
    int s_pf = srb, g_pf = g, n_pf = u_end - u_begin;  // tile to fetch next, tiles left to fetch
    bool past_end = false;
    constexpr int kWBlocks = (R + 3) / 4;  // pieces of a tile transfer: weight blocks of up to four lines, scales, zeros
    auto fetch_tile_piece = [&](auto piece, int slot) {
        int rb = kNarrowRowBlocks * s_pf + wv;
        if (rb >= rb_real) rb = rb_real - 1;  // a wave without rows of its own repeats the last block and discards the result
        const size_t tile = (size_t)rb * G + g_pf;
        MQ_LDS uint8_t *dst = ring + slot * kSlot;
        if constexpr (piece < kWBlocks) {
            const uint8_t *src = reinterpret_cast<const uint8_t *>(L.Wp) + tile * (R * 1024) + lane * 16;
            if (past_end) dma_same_line<(R - 4 * piece < 4 ? R - 4 * piece : 4), true>(src, dst);
            else dma_block<R, piece, true>(src, dst);
        } else if constexpr (piece == kWBlocks) {
            if (lane < 8) dma_lines<1, true>(reinterpret_cast<const uint8_t *>(L.st) + tile * 128 + lane * 16, dst + R * 1024);
        } else {
            // a symmetric layer reads constant lines of 2^(c-1) (tile & zmask picks one)
            const uint8_t *zsrc = reinterpret_cast<const uint8_t *>(L.zt);
            if (lane < 8) dma_lines<1, true>(zsrc + (tile & (size_t)(int64_t)L.zmask) * 128 + lane * 16, dst + R * 1024 + 128);
            if (n_pf > 1) {
                --n_pf;
                if (++g_pf == G) { g_pf = 0; ++s_pf; }
            } else {
                past_end = true;
            }
        }
    };
    auto fetch_tile = [&](int slot) { static_for<kWBlocks + 2>([&](auto piece) { fetch_tile_piece(piece, slot); }); };
    // ---- activations of the next group in line -> LDS stage; one 1 KB line per wave (the block has six lines:
    // waves 6 and 7 repeat lines 4 and 5, the same bytes to the same place); past the end the last group again
    int g_x = g, n_x = u_end - u_begin;
    const int xline = wv < 6 ? wv : wv - 2;
    auto fetch_x = [&](int stage) {
        dma_lines<1>(xt + (size_t)g_x * kNarrowXtBlockBytes + xline * 1024 + lane * 16, lds + stage * kStageBytes + xline * 1024);
        if (n_x > 1) {
            --n_x;
            if (++g_x == G) g_x = 0;
        }
    };
    // ---- ring slot -> registers: lane dwords, scales of the 16 rows the lane holds accumulator elements of, and the
    // zero-offset of the lane's own row (the lane is an A supplier of that row)
    uint32_t w[4 * R];
    u32x2 s4[4];
    _Float16 zl;
    auto open_tile = [&](int slot) {
        const MQ_LDS uint8_t *src = ring + slot * kSlot;
        const MQ_LDS u32x4 *wsrc = reinterpret_cast<const MQ_LDS u32x4 *>(src) + lane;
#pragma unroll
        for (int i = 0; i < R; ++i) {
            const u32x4 v = wsrc[i * 64];
            w[4 * i] = v.x; w[4 * i + 1] = v.y; w[4 * i + 2] = v.z; w[4 * i + 3] = v.w;
        }
        const MQ_LDS u32x2 *sp = reinterpret_cast<const MQ_LDS u32x2 *>(src + R * 1024 + 2 * lm.rowbase);
#pragma unroll
        for (int q = 0; q < 4; ++q) s4[q] = sp[2 * q];
        zl = reinterpret_cast<const MQ_LDS _Float16 *>(src + R * 1024 + 128)[lane];
    };

    {
        lds_barrier();  // the previous run's readers are done with all stages
#pragma unroll
        for (int k = 0; k < NST - 1; ++k) fetch_x(k);
#pragma unroll
        for (int k = 0; k < NBR; ++k) fetch_tile(k);
        wait_transfers<0>();
        open_tile(0);
        lds_barrier();
    }

    int st = 0;
    int slot_cur = 0;  // ring slot of tile u (already in registers)
    for (int u = u_begin; u < u_end; ++u) {
        const bool more = u + 1 < u_end;
        const int slot_next = slot_cur + 1 == NBR ? 0 : slot_cur + 1;
        const int st_next = st + 1 == NST ? 0 : st + 1;
        const int st_fill = st == 0 ? NST - 1 : st - 1;
        // This body's transfers, in this order: the stage read during the previous body takes the activations NST-1
        // tiles ahead, the ring slot of tile u (all of it is in registers) takes tile u + NBR.  They are issued piece by
        // piece between the MFMAs below: the eight waves of a compute unit share one path from the caches (64 bytes per
        // clock), and issued in one burst ahead of the math their transfers queue up behind each other while the matrix
        // pipe idles, and the waves reach the barrier as far apart as the queue is long.
        constexpr int kPieces = 1 + kWBlocks + 2;
        constexpr int kPieceStride = MF::NMF / kPieces;
        static_assert(kPieceStride >= 1, "more pieces than MFMAs");
        auto issue_piece = [&](auto pc) {
            if constexpr (pc == 0) fetch_x(st_fill);
            else fetch_tile_piece(IntC<pc - 1>{}, slot_cur);
        };

        // ---- one tile: NMF MFMAs on the masked fields, one on the zero-offset, into two accumulators taken
        // alternately (an MFMA that adds to the result of the one before it cannot issue until that result has left
        // the pipe), then y += scale * (F * D).  B operands come from the stage, read a few MFMAs ahead; lanes whose
        // operand is zero read the zeros behind the block.
        // (the activation block holds zeros for batch columns beyond M)
        const MQ_LDS u32x4 *bsrc =
            reinterpret_cast<const MQ_LDS u32x4 *>(lds + st * kStageBytes + (lm.b_live ? lm.col * 16 : 256));
        const float F = reinterpret_cast<const MQ_LDS float *>(lds + st * kStageBytes + kFactorOff)[lm.col];
        constexpr int kBlk = kOpBlockStride / 16;  // block stride in 16-byte units
        constexpr int kAhead = 4;
        u32x4 bq[kAhead];
        static_for<kAhead>([&](auto i) { bq[i] = bsrc[i * kBlk]; });
        float16_t D0, D1;
#pragma unroll
        for (int v = 0; v < 16; ++v) D0[v] = D1[v] = 0.f;
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
            if constexpr (mf + kAhead < MF::NBLK) bq[mf % kAhead] = bsrc[(mf + kAhead) * kBlk];
            if constexpr (mf % 2 == 0)
                D0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8_t, av), __builtin_bit_cast(half8_t, bv),
                                                            D0, 0, 0, 0);
            else
                D1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8_t, av), __builtin_bit_cast(half8_t, bv),
                                                            D1, 0, 0, 0);
            if constexpr (mf % kPieceStride == 0 && mf / kPieceStride < kPieces) {
                __builtin_amdgcn_sched_barrier(0);
                issue_piece(IntC<mf / kPieceStride>{});
                __builtin_amdgcn_sched_barrier(0);
            }
        });
        {   // zero-offset: A = (z', z', z', 0, ...) with z' = z * 2^(r-17), B = -X_g * 2^(e-15) in three pieces
            const _Float16 zs = zl * (_Float16)__builtin_ldexpf(1.f, R - 17);
            const half2_t zz = {zs, zs}, z0 = {zs, (_Float16)0.f};
            const u32x4 av = {__builtin_bit_cast(uint32_t, zz), __builtin_bit_cast(uint32_t, z0), 0u, 0u};
            const u32x4 bv = bq[MF::NMF % kAhead];
            if constexpr (MF::NMF % 2 == 0)
                D0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8_t, av), __builtin_bit_cast(half8_t, bv),
                                                            D0, 0, 0, 0);
            else
                D1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8_t, av), __builtin_bit_cast(half8_t, bv),
                                                            D1, 0, 0, 0);
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) yacc[v] = fmaf(half_of(s4[v >> 2], v & 3), (D0[v] + D1[v]) * F, yacc[v]);

        // tile u+1 has landed once at most the transfers of the NBR-1 bodies after its own are in flight
        wait_transfers<(NBR - 1) * kBody>();
        open_tile(slot_next);
        // the next tile's activations were issued NST-2 bodies ago, ahead of that body's weight tile
        wait_transfers<(NST - 2) * kBody + kTileOps>();
        lds_barrier();  // next stage complete for every wave, current stage free
        st = st_next;
        slot_cur = slot_next;
        ++g;
        if (g == G || !more) {
            const int rb = kNarrowRowBlocks * srb + wv;
            if (rb < rb_real) {
                const uint64_t a = L.cost_start + (uint64_t)srb * G * L.cost;
                StackParams pw = p;  // this wave's eighth of the workgroup's slots
                pw.part = p.part + (size_t)wv * (16 * 64);
                const int row0 = rb * kRowBlock + lm.rowbase;
                const int col = lm.col;
                const bool fast_store = (L.N & 3) == 0 && (reinterpret_cast<uintptr_t>(L.y) & 7) == 0;
                finish_row_block<16>(L, pw, p.cnt + L.cnt_off + rb, a, ga, g, yacc, worker, lane,
                                     [&](const float(&tot)[16]) {
                                         if (col >= L.M) return;
                                         uint16_t MQ_GLOBAL *yrow = gl(reinterpret_cast<uint16_t *>(L.y) + (size_t)col * L.N);
                                         const int fl = L.flags;
#pragma unroll
                                         for (int q = 0; q < 4; ++q) {
                                             const int row = row0 + 8 * q;
                                             if (fast_store && row + 3 < L.N) {
                                                 const u32x2 pk = {
                                                     (uint32_t)y_bits(tot[4 * q], fl) | ((uint32_t)y_bits(tot[4 * q + 1], fl) << 16),
                                                     (uint32_t)y_bits(tot[4 * q + 2], fl) | ((uint32_t)y_bits(tot[4 * q + 3], fl) << 16)};
                                                 *(u32x2 MQ_GLOBAL *)(yrow + row) = pk;
                                             } else {
#pragma unroll
                                                 for (int e = 0; e < 4; ++e)
                                                     if (row + e < L.N) yrow[row + e] = y_bits(tot[4 * q + e], fl);
                                             }
                                         }
                                     });
            }
            if (g == G) { ++srb; g = 0; }
            ga = g;
#pragma unroll
            for (int v = 0; v < 16; ++v) yacc[v] = 0.f;
            // Everything the hand-over loaded or stored has retired before the tile loop goes on: the compiler keeps
            // count of ITS memory instructions only and would otherwise protect their registers at the top of every
            // following tile with a wait that also drains the transfers in flight.
            __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0), other counters untouched
        }
    }
    wait_transfers<0>();  // nothing of this run may land in LDS after the next run has started
}

__global__ __launch_bounds__(64 * kNarrowWaves, 1) void gemm_stack_kernel(const StackParams p) {
    extern __shared__ __attribute__((aligned(16))) uint8_t lds_generic[];
    MQ_LDS uint8_t *lds = (MQ_LDS uint8_t *)lds_generic;
    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int worker = blockIdx.x;
    walk_tiles(p, worker, [&](const LayerDesc &L, int u_begin, int u_end) __attribute__((always_inline)) {
        switch (L.r) {
            case 2: run_narrow_units<2>(L, p, u_begin, u_end, worker, wv, lane, lds); break;
            case 3: run_narrow_units<3>(L, p, u_begin, u_end, worker, wv, lane, lds); break;
            case 4: run_narrow_units<4>(L, p, u_begin, u_end, worker, wv, lane, lds); break;
            case 6: run_narrow_units<6>(L, p, u_begin, u_end, worker, wv, lane, lds); break;
            default: run_narrow_units<8>(L, p, u_begin, u_end, worker, wv, lane, lds); break;
        }
    });
}

// workgroups the device keeps resident for a launch with lds_bytes of LDS per workgroup
static int narrow_resident_groups(int lds_bytes) {
    static int cached_bytes[2] = {0, 0}, cached[2] = {0, 0};
    for (int i = 0; i < 2; ++i)
        if (cached_bytes[i] == lds_bytes) return cached[i];
    int dev = 0, cus = 0, blocks = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_stack_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                            narrow_lds_bytes_max()) != hipSuccess)
        return 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&blocks, gemm_stack_kernel, 64 * kNarrowWaves, lds_bytes) != hipSuccess)
        return 0;
    if (blocks < 1) blocks = 1;
    int w = cus * blocks;
    if (w > kMaxGroupsNarrow) w = kMaxGroupsNarrow;
    const int slot = cached_bytes[0] == 0 ? 0 : 1;
    cached_bytes[slot] = lds_bytes;
    cached[slot] = w;
    return w;
}

hipError_t launch_stack_mfma(StackParams p, int max_cost, hipStream_t s) {
    // LDS per workgroup: a single layer takes the plan of its width, a stack the largest plan
    int lds_bytes = narrow_lds_bytes_max();
    if (!p.table) {
        switch (p.single.r) {
            case 2: lds_bytes = narrow_lds_bytes(2); break;
            case 3: lds_bytes = narrow_lds_bytes(3); break;
            case 4: lds_bytes = narrow_lds_bytes(4); break;
            case 6: lds_bytes = narrow_lds_bytes(6); break;
            default: lds_bytes = narrow_lds_bytes(8); break;
        }
    }
    int hw = narrow_resident_groups(lds_bytes);
    if (hw <= 0) return hipErrorUnknown;
    if (p.worker_cap && hw > p.worker_cap) hw = p.worker_cap;
    // every share at least one super-tile long (that makes a row block's contributor list exact); small layers are not
    // cut finer than four super-tiles per share, because every cut is a hand-over between workgroups and a workgroup's
    // start-up (first transfers, one full trip to memory) is worth several tiles (measured on the Llama-2-7B shapes
    // at M = 8 and 16: 23.0 -> 20.1, 24.4 -> 23.0, 33.6 -> 31.1 us per call against two)
    uint64_t cap = p.cost_total / ((uint64_t)max_cost * 4);
    if (cap < 1) cap = 1;
    p.nworkers = (int)(cap < (uint64_t)hw ? cap : (uint64_t)hw);
    p.nwaves = p.nworkers * kNarrowWaves;
    p.slot_floats = kNarrowWaves * 16 * 64;
    const hipError_t e = launch(xprep_kernel, dim3((unsigned)((p.n_jobs + 3) / 4)), dim3(256), 0, s, p);
    if (e != hipSuccess) return e;
    return launch(gemm_stack_kernel, dim3((unsigned)p.nworkers), dim3(64 * kNarrowWaves), (unsigned)lds_bytes, s, p);
}

}  // namespace mq
