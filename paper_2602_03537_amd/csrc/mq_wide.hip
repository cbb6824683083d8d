// Medium batch (16 < M <= 256): the sliced linear layer on the matrix cores with the
// weights of a tile unpacked ONCE and multiplied against up to 128 batch columns
// (Section 4 of the paper: the TensorCore kernel; the regime where the contraction is
// dense enough for the matrix pipe to matter).  Same packed tiles, same persistent
// schedule and split-K hand-over (mq_device.h) as the other kernels.
//
// Operand forming.  v_mfma_f32_32x32x16_f16 computes D[32x32] += A[32x16] * B[16x32];
// lane l supplies A[l%32][8*(l/32) .. +7] and B[8*(l/32) .. +7][l%32]: the two halves of
// a wave hold the two k-halves of the SAME 32 rows / columns.  In the tile layout lane l
// owns row l of a 64-row tile, so the halves of a wave hold different rows.  One
// v_permlane32_swap per pair of lane dwords (a, b) fixes that without touching LDS:
//     X = [lanes 0..31: dword a of rows 0..31  | lanes 32..63: dword b of rows 0..31 ]
//     Y = [lanes 0..31: dword a of rows 32..63 | lanes 32..63: dword b of rows 32..63]
// A bit-field of X, shifted down to bit 0 and masked, is a pair of fp16 subnormals
// code * 2^-24 of rows 0..31 for the columns of that field in dwords a and b; the same
// field of Y serves rows 32..63.  Three packed fp16 operations turn it into the weight
// operand  w = scale * (2^(8-r) * code - zero)  (the affine de-quantisation of Section 3.2;
// code * 2^-9 and 2^(8-r) * code - zero are exact for integer zeros, the product with the
// scale is rounded to fp16 once), so that the matrix core accumulates y itself over the
// whole row block in fp32 and no per-group vector work is left.  This is the one kernel of
// the library whose products are not exact: a weight carries a relative rounding error of
// at most 2^-11, like the fp16 output itself.
// The weights are the B operand (output column j = weight row), the activations the A
// operand (output row i = batch column).  The 16th code of a 3-bit unit and the two
// spare-bit codes of a 6-bit unit are assembled with a few vector-ALU operations before
// the swap, so every width needs exactly eight k-steps ("specs") of 16 columns per group
// and half-tile.
//
// Work split.  A workgroup of four waves walks a run of super-tiles (256 rows x one
// group); wave w owns row block 4*srb + w.  The activations of the group, re-ordered into
// A operands by xprep_wide_kernel (8 KB per 32 batch columns), are shared by the four
// waves through LDS (two stages: the next group's block is copied in while the current
// one is used).  Up to C = 4 chunks of 32 columns are multiplied against one unpacked
// tile; more columns take further passes over the weights (pass index slowest in the
// schedule); the chunk count is padded to passes * C with all-zero chunks.
#include "mq_device.h"
#include "mq_dma.h"

namespace mq {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float16_t __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kWideSpecs = 8;
constexpr int kWideBlockBytes = kWideSpecs * 1024;  // A operands of one (group, chunk)
static_assert(kWideBlockBytes == kWideXtBlockBytes, "host and device disagree on the activation block size");

struct WField {
    int sw;       // swap whose X / Y registers carry the field
    int bit;      // right shift before masking; < 0: the register already is the clean code pair
    int pair_lo;  // activation pair (column pair inside the group) met by lanes 0..31 ...
    int pair_hi;  // ... and by lanes 32..63
};

template <int R> struct Wide {
    using T = Layout<R>;
    static constexpr int NRAW = 4 * R;                            // lane dwords of a tile
    static constexpr int NASM = R == 3 ? 4 : R == 6 ? 16 : 0;     // assembled code pairs
    static constexpr int NE = NRAW + NASM;
    static constexpr int NSW = NE / 2;
    // swap k exchanges registers sa(k) and sb(k); afterwards e[sa] = X (rows 0..31), e[sb] = Y (rows 32..63)
    static constexpr int sa(int k) {
        if constexpr (T::UD == 1) return 8 * (k / 4) + k % 4;                        // unit quads 2q', 2q'+1
        else if constexpr (R == 6) return k < 12 ? (k % 4) * 3 + k / 4               // unit i <-> unit 4+i, dword k/4
                                                 : 24 + 2 * ((k - 12) % 4) + (k - 12) / 4;
        else return k < 4 ? 3 * k : k < 6 ? (k - 4) * 3 + 2 : 12 + (k - 6);        // r = 3
    }
    static constexpr int sb(int k) {
        if constexpr (T::UD == 1) return sa(k) + 4;
        else if constexpr (R == 6) return k < 12 ? sa(k) + 12 : sa(k) + 8;
        else return k < 4 ? 3 * k + 1 : k < 6 ? sa(k) + 6 : sa(k) + 2;              // dw0<->dw1; unit u <-> u+2
    }
    static constexpr WField fld(int spec, int i) {
        if constexpr (T::UD == 1) {
            const int q = spec / T::NOPS;
            const Op o = T::op(spec % T::NOPS);
            return {4 * q + i, o.sh + ctz16(o.mask), (8 * q + i) * T::PPU + o.pair, (8 * q + 4 + i) * T::PPU + o.pair};
        } else if constexpr (R == 6) {
            if (spec < 6) {
                const Op o = T::op(spec);  // the six whole codes of a unit
                return {o.dw * 4 + i, o.sh, i * 8 + o.pair, (4 + i) * 8 + o.pair};
            }
            const int t = spec - 6;        // assembled pairs 6 and 7
            return {12 + 4 * t + i, -1, 8 * i + 6 + t, 8 * (4 + i) + 6 + t};
        } else {
            if (spec < 5) return {i, 3 * spec, 16 * i + spec, 16 * i + 5 + spec};   // dwords 0 | 1 of unit i
            const int item = 2 * (spec - 5) + (i & 1), zi = i >> 1;                  // dword 2 of units zi | 2+zi
            if (item < 5) return {4 + zi, 3 * item, 16 * zi + 10 + item, 16 * (2 + zi) + 10 + item};
            return {6 + zi, -1, 16 * zi + 15, 16 * (2 + zi) + 15};
        }
    }
    // every activation pair of the group is met exactly once
    static constexpr bool ok() {
        bool seen[64] = {};
        for (int s = 0; s < kWideSpecs; ++s)
            for (int i = 0; i < 4; ++i) {
                const WField f = fld(s, i);
                if (f.sw < 0 || f.sw >= NSW || f.pair_lo < 0 || f.pair_lo > 63 || f.pair_hi < 0 || f.pair_hi > 63)
                    return false;
                if (seen[f.pair_lo] || seen[f.pair_hi] || f.pair_lo == f.pair_hi) return false;
                seen[f.pair_lo] = seen[f.pair_hi] = true;
            }
        bool used[NE] = {};
        for (int k = 0; k < NSW; ++k) {
            if (used[sa(k)] || used[sb(k)] || sa(k) == sb(k)) return false;
            used[sa(k)] = used[sb(k)] = true;
        }
        return true;
    }
};
static_assert(Wide<2>::ok() && Wide<3>::ok() && Wide<4>::ok() && Wide<6>::ok() && Wide<8>::ok(),
              "inconsistent operand plan");

// ------------------------------------------------------------------ activation prep
// One workgroup per (layer, group, chunk of 32 columns), wave q of it for specs 2q and 2q+1: lane l =
// (column l%32, k-half l/32) writes its A operand of those specs (16 bytes each).  Columns beyond M are zero.
template <int R>
__device__ __forceinline__ void xprep_wide_job(const LayerDesc &L, int g, int c, int nct, int sq, int lane) {
    const int j = lane & 31, h = lane >> 5;
    const int col = c * kWideCols + j;
    const uint32_t live = col < L.M ? 0xFFFFFFFFu : 0u;
    const uint32_t MQ_GLOBAL *xrow =
        gl(reinterpret_cast<const uint32_t *>(L.x + (size_t)(live ? col : 0) * L.K) + (size_t)g * 64);
    uint8_t *block = reinterpret_cast<uint8_t *>(const_cast<uint4 *>(L.xt)) + (size_t)(g * nct + c) * kWideBlockBytes;
    u32x4 MQ_GLOBAL *out = gl(reinterpret_cast<u32x4 *>(block)) + lane;
    static_for<kWideSpecs / 2>([&](auto q) {
        if (q != sq) return;
        uint32_t v[2][4];
        static_for<2>([&](auto ds) {
            static_for<4>([&](auto i) {
                constexpr WField f = Wide<R>::fld(2 * q + ds, i);
                v[ds][i] = x_pair(xrow[h ? f.pair_hi : f.pair_lo], L.flags) & live;
            });
        });
        static_for<2>([&](auto ds) {
            const u32x4 o = {v[ds][0], v[ds][1], v[ds][2], v[ds][3]};
            out[(2 * q + ds) * 64] = o;
        });
    });
}

__global__ __launch_bounds__(256) void xprep_wide_kernel(const StackParams p) {
    const int lane = threadIdx.x & 63;
    const int sq = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int job = blockIdx.x;
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
    // chunk count padded to whole passes; padding chunks are zero
    const int nct = L.CB * (((L.M + kWideCols - 1) / kWideCols + L.CB - 1) / L.CB);
    const int local = job - L.job_start;
    const int g = local / nct, c = local - g * nct;
    switch (L.r) {
        case 2: xprep_wide_job<2>(L, g, c, nct, sq, lane); break;
        case 3: xprep_wide_job<3>(L, g, c, nct, sq, lane); break;
        case 4: xprep_wide_job<4>(L, g, c, nct, sq, lane); break;
        case 6: xprep_wide_job<6>(L, g, c, nct, sq, lane); break;
        default: xprep_wide_job<8>(L, g, c, nct, sq, lane); break;
    }
}

// ------------------------------------------------------------------ main kernel
__device__ __forceinline__ void swap32(uint32_t &a, uint32_t &b) {
    const u32x2 r = __builtin_amdgcn_permlane32_swap(a, b, false, false);
    a = r.x;
    b = r.y;
}

// A tile in flight: lane dwords plus the lane's scale and zero
template <int R> struct WideTile {
    uint32_t w[4 * R];
    _Float16 s, z;
};

// Unpacking, first part: assembled codes and the lane swaps.  e[sa(k)] / e[sb(k)] become the X / Y
// registers of swap k; sz = packed fp16 pairs {scale, scale} and {-zero, -zero} of the rows a lane
// serves in the X registers (row l%32) and in the Y registers (row 32 + l%32).
template <int R>
__device__ __forceinline__ void wide_prework(const WideTile<R> &t, uint32_t (&e)[Wide<R>::NE], half2_t (&sc)[2],
                                             half2_t (&nz)[2]) {
    using W = Wide<R>;
#pragma unroll
    for (int i = 0; i < 4 * R; ++i) e[i] = t.w[i];
    if constexpr (R == 3) {
        // 16th code of a unit: bit 15 of the halves of its three dwords = code bits 0, 1, 2
#pragma unroll
        for (int u = 0; u < 4; ++u)
            e[12 + u] = ((t.w[3 * u] >> 15) & 0x00010001u) | ((t.w[3 * u + 1] >> 14) & 0x00020002u) |
                        ((t.w[3 * u + 2] >> 13) & 0x00040004u);
    }
    if constexpr (R == 6) {
        // pair 6 = B[12:13] + 4 * A[12:15], pair 7 = C[12:15] + 16 * B[14:15]  (A, B, C = dwords of the unit)
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const uint32_t A = t.w[3 * u], B = t.w[3 * u + 1], Cw = t.w[3 * u + 2];
            e[24 + 2 * u] = ((B >> 12) & 0x00030003u) | ((A >> 10) & 0x003C003Cu);
            e[24 + 2 * u + 1] = ((Cw >> 12) & 0x000F000Fu) | ((B >> 10) & 0x00300030u);
        }
    }
    static_for<W::NSW>([&](auto k) { swap32(e[W::sa(k)], e[W::sb(k)]); });
    const half2_t s2 = {t.s, t.s};
    const half2_t z2 = {(_Float16)(-t.z), (_Float16)(-t.z)};
    uint32_t sa = __builtin_bit_cast(uint32_t, s2), sb = sa, za = __builtin_bit_cast(uint32_t, z2), zb = za;
    swap32(sa, sb);
    swap32(za, zb);
    sc[0] = __builtin_bit_cast(half2_t, sa);
    sc[1] = __builtin_bit_cast(half2_t, sb);
    nz[0] = __builtin_bit_cast(half2_t, za);
    nz[1] = __builtin_bit_cast(half2_t, zb);
}

// Unpacking, second part: weight operand register q = (2 * spec + half) * 4 + i as de-quantised fp16 pair,
// in two stages of two vector instructions each (field * 2^k, then (.. * 2^k' - zero) * scale), so that
// stages of different registers can be interleaved and no instruction follows the one it depends on.
template <int R, int Q> __device__ __forceinline__ uint32_t wide_operand_s1(const uint32_t (&e)[Wide<R>::NE]) {
    using W = Wide<R>;
    constexpr int spec = Q / 8, h = (Q / 4) % 2, i = Q % 4;
    constexpr WField f = W::fld(spec, i);
    const uint32_t src = h == 0 ? e[W::sa(f.sw)] : e[W::sb(f.sw)];
    // A field that lies inside the fp16 mantissa (bits 0..9 of its half) is masked where it stands: the
    // pair of subnormals code * 2^(p-24) only changes the first multiplier.  Higher fields come down by
    // the one shift their width uses (shared by the fields of a register).
    constexpr int kShift = R == 2 ? 10 : R == 3 ? 9 : R == 4 ? 8 : R == 6 ? 6 : 8;
    constexpr int bit = f.bit < 0 ? 0 : f.bit;
    constexpr int sh = bit + R <= 10 ? 0 : kShift;
    constexpr int pos = bit - sh;
    static_assert(pos >= 0 && pos + R <= 10, "field outside the mantissa");
    constexpr uint32_t m = ((uint32_t)((1 << R) - 1) << pos) * 0x10001u;
    uint32_t field;
    if constexpr (f.bit < 0) field = src;
    else if constexpr (sh == 0) field = src & m;
    else field = (src >> sh) & m;
    // code * 2^(pos-24) (subnormal) -> code * 2^-9
    const _Float16 k1 = (_Float16)(float)(1 << (15 - pos));
    const half2_t k15 = {k1, k1};
    return __builtin_bit_cast(uint32_t, __builtin_bit_cast(half2_t, field) * k15);
}
template <int R, int Q>
__device__ __forceinline__ uint32_t wide_operand_s2(uint32_t c, const half2_t (&sc)[2], const half2_t (&nz)[2]) {
    constexpr int h = (Q / 4) % 2;
    // code * 2^-9 -> 2^(8-r) * code - zero -> times scale
    const _Float16 kr = (_Float16)(float)(1 << (9 + kC - R));
    const half2_t k2 = {kr, kr};
    const half2_t u = __builtin_elementwise_fma(__builtin_bit_cast(half2_t, c), k2, nz[h]);
    return __builtin_bit_cast(uint32_t, u * sc[h]);
}
template <int R, int Q>
__device__ __forceinline__ uint32_t wide_operand(const uint32_t (&e)[Wide<R>::NE], const half2_t (&sc)[2],
                                                 const half2_t (&nz)[2]) {
    return wide_operand_s2<R, Q>(wide_operand_s1<R, Q>(e), sc, nz);
}

// The eight operand registers of a spec are formed as four pairs in two stages each; the eight half-jobs
// in an order in which neighbours belong to different pairs.
constexpr int kJobStage[8] = {1, 1, 2, 1, 2, 1, 2, 2};
constexpr int kJobPair[8] = {0, 1, 0, 2, 1, 3, 2, 3};

// Split-K hand-over for many accumulators per lane: as finish_row_block, but the accumulators are
// fetched block by block (block(b) = 16 values) and the last contributor sums and delivers 16 values
// at a time (final(b, values)), so that only a block is ever held in vector registers.
template <int NBK, class Block, class Final>
__device__ __forceinline__ void finish_row_block_blocked(const LayerDesc &L, const StackParams &p, int32_t *cnt,
                                                         uint64_t a, int ga, int gb, Block &&block, int worker,
                                                         int lane, Final &&final) {
    constexpr int BLK = 16;
    if (ga == 0 && gb == L.G) {
        static_for<NBK>([&](auto b) {
            __builtin_amdgcn_sched_barrier(0);  // one block in vector registers at a time
            const float16_t v = block(b);
            float t[BLK];
#pragma unroll
            for (int i = 0; i < BLK; ++i) t[i] = v[i];
            final(b, t);
        });
        return;
    }
    const int slot = ga == 0 ? 1 : 0;
    const size_t slot_floats = (size_t)p.slot_floats;
    float MQ_GLOBAL *mine = gl(p.part + (size_t)(worker * 2 + slot) * slot_floats + lane);
    static_for<NBK>([&](auto b) {
        __builtin_amdgcn_sched_barrier(0);  // one block in vector registers at a time
        const float16_t v = block(b);
#pragma unroll
        for (int i = 0; i < BLK; ++i)
            __hip_atomic_store(mine + (b * BLK + i) * 64, v[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    });
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    int old = 0;
    if (lane == 0) old = __hip_atomic_fetch_add(gl(cnt), gb - ga, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    old = __builtin_amdgcn_readfirstlane(old);
    if (old + (gb - ga) != L.G) return;
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    const int w_lo = wave_of(a, p.nworkers, p.cost_total);
    const int w_hi = wave_of(a + (uint64_t)(L.G - 1) * L.cost, p.nworkers, p.cost_total);
    // Fixed summation order: slot 1 of share w_lo, then slot 0 of shares w_lo+1 .. w_hi.  A share spans many
    // tiles here, so there are two contributors as a rule: their values of block b+1 are on their way while
    // block b is summed and delivered; further contributors are fetched one after the other.
    const bool two = w_lo < w_hi;
    const float MQ_GLOBAL *first = gl(p.part + (size_t)(w_lo * 2 + 1) * slot_floats + lane);
    const float MQ_GLOBAL *second = gl(p.part + (size_t)((two ? w_lo + 1 : w_lo) * 2) * slot_floats + lane);
    float fv[2][BLK], sv[2][BLK];
    auto fetch = [&](auto b) {
#pragma unroll
        for (int v = 0; v < BLK; ++v) {
            fv[b % 2][v] = __hip_atomic_load(first + (b * BLK + v) * 64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            sv[b % 2][v] = __hip_atomic_load(second + (b * BLK + v) * 64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    };
    fetch(IntC<0>{});
    static_for<NBK>([&](auto b) {
        if constexpr (b + 1 < NBK) fetch(IntC<b + 1>{});
        float tot[BLK];
#pragma unroll
        for (int v = 0; v < BLK; ++v) tot[v] = two ? fv[b % 2][v] + sv[b % 2][v] : fv[b % 2][v];
        for (int w0 = w_lo + 2; w0 <= w_hi; w0 += 2) {  // two at a time, so that their round trips overlap
            float t[2][BLK];
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int w = w0 + j <= w_hi ? w0 + j : w_hi;
                const float MQ_GLOBAL *src = gl(p.part + (size_t)(w * 2) * slot_floats + lane) + b * BLK * 64;
#pragma unroll
                for (int v = 0; v < BLK; ++v)
                    t[j][v] = __hip_atomic_load(src + v * 64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
#pragma unroll
            for (int v = 0; v < BLK; ++v) tot[v] += t[0][v];
            if (w0 + 1 <= w_hi) {
#pragma unroll
                for (int v = 0; v < BLK; ++v) tot[v] += t[1][v];
            }
        }
        final(b, tot);
    });
    if (lane == 0) __hip_atomic_store(gl(cnt), 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// acc += A * B with the accumulator pinned to the accumulation registers: the C * 32 accumulators of a
// wave live there for a whole row block and no vector instruction touches them in between (left to
// itself the register allocator keeps shuttling them to vector registers and back).  Operands come from
// LDS reads and from operands finished a tile earlier, the result is read at the end of a row block only.
// (No wait states needed here: the A operand comes from LDS behind a counter wait, the B operand was
// formed by vector instructions at least one slot earlier.)
// AG = false (the variants that share a compute unit between two workgroups): the accumulators are pinned to ordinary
// vector registers instead -- a kernel that names accumulation registers anywhere is given only half of a wave's
// registers as vector registers, and with 256 in all that half does not hold the working set.
template <bool AG> __device__ __forceinline__ void mfma_acc(float16_t &acc, const u32x4 &a, const u32x4 &b) {
    if constexpr (AG)
        asm volatile("v_mfma_f32_32x32x16_f16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
    else
        asm volatile("v_mfma_f32_32x32x16_f16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b));
}
// acc = 0, also from the matrix core (0 * 0 + 0), so that the accumulators are never defined by a vector instruction
template <bool AG> __device__ __forceinline__ void mfma_zero(float16_t &acc) {
    const u32x4 z = {0u, 0u, 0u, 0u};
    // the wait states are for the vector writes that have just made z: inside inline assembly the
    // compiler does not see a matrix instruction and inserts none
    if constexpr (AG)
        asm volatile("s_nop 4\n\tv_mfma_f32_32x32x16_f16 %0, %1, %1, 0" : "=a"(acc) : "v"(z));
    else
        asm volatile("s_nop 4\n\tv_mfma_f32_32x32x16_f16 %0, %1, %1, 0" : "=&v"(acc) : "v"(z));
}
// One accumulator block out of the accumulation registers, at this point of the program and not earlier
// (the compiler would otherwise fetch all C * 64 accumulators into vector registers ahead of the hand-over).
template <bool AG> __device__ __forceinline__ float16_t read_acc(const float16_t &acc) {
    float16_t r;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        float x;
        if constexpr (AG)
            asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(x) : "a"(acc[v]) : "memory");
        else
            asm volatile("v_mov_b32 %0, %1" : "=v"(x) : "v"(acc[v]) : "memory");
        r[v] = x;
    }
    return r;
}
// LDS a workgroup may take.  Up to two chunks per pass the tile body is bound by the vector work of unpacking, which one
// wave per SIMD issues at about one instruction in five cycles: two workgroups share a compute unit there (two waves per
// SIMD, half the LDS each; the accumulators are 64 registers at most, so a wave fits 256 registers).
// (TWO = that variant of the kernel; it exists up to kWideTwoPerCuMaxC chunks and runs stacks.)
constexpr int kWideTwoPerCuMaxC = 2;
constexpr int wide_lds_budget(bool TWO) { return (TWO ? 80 : 160) * 1024; }
constexpr int wide_slot_bytes(int R) { return R * 1024 + 256; }  // lane dwords of a tile + its 64 scales + 64 zeros
// LDS plan of a workgroup: NST activation stages (one being read, the others landing) and per wave a
// ring of NBR weight tiles.  The activations of a group are re-read for every row block, long after the
// weight stream has pushed them out of the caches, so they need about as much lead as the weights.
struct WidePlan { int nst, nbr; };
constexpr int wide_plan_bytes(int R, int C, WidePlan q) { return q.nst * C * kWideBlockBytes + 4 * q.nbr * wide_slot_bytes(R); }
constexpr WidePlan wide_plan(int R, int C, bool TWO) {
    for (WidePlan q : {WidePlan{4, 3}, WidePlan{3, 3}, WidePlan{4, 2}, WidePlan{3, 2}, WidePlan{2, 2}, WidePlan{2, 1}})
        if (wide_plan_bytes(R, C, q) <= wide_lds_budget(TWO)) return q;
    return {2, 1};
}
constexpr int wide_lds_bytes(int R, int C, bool TWO) { return wide_plan_bytes(R, C, wide_plan(R, C, TWO)); }
constexpr int wide_lds_bytes_max(int C, bool TWO) {
    int m = 0;
    for (int r : {2, 3, 4, 6, 8}) m = wide_lds_bytes(r, C, TWO) > m ? wide_lds_bytes(r, C, TWO) : m;
    return m;
}
static_assert(wide_lds_bytes_max(4, false) <= wide_lds_budget(false) && wide_lds_bytes_max(kWideTwoPerCuMaxC, true) <= wide_lds_budget(true),
              "LDS plan does not fit");

// Super-tiles [u_begin, u_end) of pass `pass` of one layer (u = srb * G + g), for the whole workgroup.
// C = chunks of 32 batch columns per pass (the layer's chunk count is padded to passes * C; padding
// chunks hold zeros).
//
// TWO: the variant whose workgroups share a compute unit in pairs (two waves per SIMD, half the LDS, accumulators in
// vector registers); otherwise a wave is alone on its SIMD.  The schedule is written for the wave that is alone, where
// nothing but the instruction order hides latencies, and a second wave only adds to what it hides.  MFMAs run
// spec by spec: the two weight operands of spec s (rows 0..31 and 32..63 of the tile) meet the C chunks
// in 2C consecutive "slots"; each slot is one MFMA followed by a share of the vector work that forms
// the operands of the NEXT spec (the matrix core needs 32 cycles per MFMA, a vector instruction 4),
// fixed with scheduling barriers.  So only two specs' operands are ever held in registers, and the next
// tile is pulled out of the LDS ring while the last spec of the current one is multiplied.
template <int R, int C, bool TWO>
__device__ __forceinline__ void run_wide_units(const LayerDesc &L, const StackParams &p, int pass, int u_begin,
                                               int u_end, int worker, int wv, int lane, MQ_LDS uint8_t *lds) {
    using W = Wide<R>;
    constexpr int NBR = wide_plan(R, C, TWO).nbr, NST = wide_plan(R, C, TWO).nst;
    constexpr bool AG = !TWO;  // accumulators in the accumulation registers
    constexpr int kStage = C * kWideBlockBytes;
    constexpr int kSlot = wide_slot_bytes(R);
    constexpr int kSpecSlots = 2 * C;       // MFMAs per spec
    constexpr int kXLines = 2 * C;          // 1 KB lines of an activation block copied by each wave
    constexpr int kTileOps = R + 2;         // transfers per weight tile
    const int G = L.G;
    const int rb_real = (L.N + kRowBlock - 1) / kRowBlock;
    const int nct = L.CB * C;      // chunks of the layer, padded
    const int c0 = pass * C;
    const uint8_t *xt = reinterpret_cast<const uint8_t *>(L.xt);
    MQ_LDS uint8_t *ring = lds + NST * kStage + wv * (NBR * kSlot);

    int srb = u_begin / G;
    int g = u_begin - srb * G;
    int ga = g;
    float16_t acc[C][2];  // [chunk][row half]: y of the row block so far, accumulated by the matrix core
    auto clear_acc = [&]() {
#pragma unroll
        for (int c = 0; c < C; ++c)
#pragma unroll
            for (int h = 0; h < 2; ++h) mfma_zero<AG>(acc[c][h]);
    };
    clear_acc();

    // ---- weights: kTileOps transfers per tile into ring slot `slot`; past the end of the run the last
    // tile is fetched again (the number of transfers per tile body must not depend on the data)
    int s_pf = srb, g_pf = g, n_pf = u_end - u_begin;  // tile to fetch next, tiles left to fetch
    constexpr int kWBlocks = (R + 3) / 4;  // pieces of a tile transfer: weight blocks, scales, zeros
    auto fetch_tile_piece = [&](auto piece, int slot) {
        int rb = 4 * s_pf + wv;
        if (rb >= rb_real) rb = rb_real - 1;  // a wave without rows of its own repeats the last block and discards the result
        const size_t tile = (size_t)rb * G + g_pf;
        MQ_LDS uint8_t *dst = ring + slot * kSlot;
        if constexpr (piece < kWBlocks) {
            dma_block<R, piece, true>(reinterpret_cast<const uint8_t *>(L.Wp) + tile * (R * 1024) + lane * 16, dst);
        } else if constexpr (piece == kWBlocks) {
            if (lane < 8) dma_lines<1, true>(reinterpret_cast<const uint8_t *>(L.st) + tile * 128 + lane * 16, dst + R * 1024);
        } else {
            // A symmetric layer reads constant lines of 2^(c-1) (tile & zmask picks one).
            const uint8_t *zsrc = reinterpret_cast<const uint8_t *>(L.zt);
            if (lane < 8) dma_lines<1, true>(zsrc + (tile & (size_t)(int64_t)L.zmask) * 128 + lane * 16, dst + R * 1024 + 128);
            if (n_pf > 1) {
                --n_pf;
                if (++g_pf == G) { g_pf = 0; ++s_pf; }
            }
        }
    };
    auto fetch_tile = [&](int slot) { static_for<kWBlocks + 2>([&](auto piece) { fetch_tile_piece(piece, slot); }); };
    // ring slot -> swapped lane dwords e[], scales and zeros of the rows a lane serves
    uint32_t e[W::NE];
    half2_t sc[2], nz[2];
    auto open_tile = [&](int slot) {
        WideTile<R> t;
        const MQ_LDS uint8_t *src = ring + slot * kSlot;
        const MQ_LDS u32x4 *wsrc = reinterpret_cast<const MQ_LDS u32x4 *>(src) + lane;
#pragma unroll
        for (int i = 0; i < R; ++i) {
            const u32x4 v = wsrc[i * 64];
            t.w[4 * i] = v.x; t.w[4 * i + 1] = v.y; t.w[4 * i + 2] = v.z; t.w[4 * i + 3] = v.w;
        }
        t.s = reinterpret_cast<const MQ_LDS _Float16 *>(src + R * 1024)[lane];
        t.z = reinterpret_cast<const MQ_LDS _Float16 *>(src + R * 1024 + 128)[lane];
        wide_prework<R>(t, e, sc, nz);
    };
    // ---- activations of the next group in line (the C chunks of this pass) -> LDS stage; kXLines transfers
    // per wave; past the end of the run the last tile's group again
    int g_x = g, n_x = u_end - u_begin;
    constexpr int kXBlocks = (kXLines + 3) / 4;
    auto fetch_x_piece = [&](auto piece, int stage) {
        dma_block<kXLines, piece>(xt + (size_t)(g_x * nct + c0) * kWideBlockBytes + (wv * kXLines) * 1024 + lane * 16,
                                  lds + stage * kStage + (wv * kXLines) * 1024);
        if constexpr (piece == kXBlocks - 1) {
            if (n_x > 1) {
                --n_x;
                if (++g_x == G) g_x = 0;
            }
        }
    };
    auto fetch_x = [&](int stage) { static_for<kXBlocks>([&](auto piece) { fetch_x_piece(piece, stage); }); };
    constexpr int kPieces = kXBlocks + kWBlocks + 2;  // transfers of a tile body, in issue order: activations first

    uint32_t Wq[2][8];  // [spec parity][half * 4 + i]: weight operands of the spec being multiplied / being formed
    uint32_t half_done[4][2];  // operand pairs between their two stages
    {
        lds_barrier();  // the previous run's readers are done with all stages
#pragma unroll
        for (int k = 0; k < NST - 1; ++k) fetch_x(k);
#pragma unroll
        for (int k = 0; k < NBR; ++k) fetch_tile(k);
        wait_transfers<0>();
        open_tile(0);
        static_for<8>([&](auto q) { Wq[0][q] = wide_operand<R, q>(e, sc, nz); });  // spec 0 of the first tile
        lds_barrier();
    }

    int st = 0;
    int slot_cur = 0;  // ring slot of tile u
    for (int u = u_begin; u < u_end; ++u) {
        const bool more = u + 1 < u_end;
        const int slot_next = slot_cur + 1 == NBR ? 0 : slot_cur + 1;
        const int st_next = st + 1 == NST ? 0 : st + 1;
        const int st_fill = st == 0 ? NST - 1 : st - 1;

        const MQ_LDS u32x4 *abase = reinterpret_cast<const MQ_LDS u32x4 *>(lds + st * kStage) + lane;
        // A operands in the order of use: position i = s * C + c is chunk c of spec s
        auto a_at = [&](int i) { return abase[((i % C) * 8 + i / C) * 64]; };
        constexpr int kAhead = 3;
        u32x4 aq[kAhead];
        static_for<kAhead>([&](auto i) { aq[i] = a_at(i); });
        __builtin_amdgcn_sched_barrier(0);
        static_for<kWideSpecs>([&](auto s) {
            constexpr int SP = s & 1;
            if constexpr (s == kWideSpecs - 1) {
                // every field of tile u has been extracted: open tile u+1, which has landed once at most the
                // transfers of the NBR-1 tile bodies after its own are in flight
                wait_transfers<(NBR - 1) * (kXLines + kTileOps)>();
                open_tile(slot_next);
                __builtin_amdgcn_sched_barrier(0);
            }
            static_for<C>([&](auto c) {
                static_for<2>([&](auto h) {
                    constexpr int pos = s * C + c, slot = 2 * c + h;
                    const u32x4 bw = {Wq[SP][4 * h], Wq[SP][4 * h + 1], Wq[SP][4 * h + 2], Wq[SP][4 * h + 3]};
                    mfma_acc<AG>(acc[c][h], aq[pos % kAhead], bw);
                    __builtin_amdgcn_sched_barrier(0);
                    // this slot's share of the next spec's operands (after the last spec: spec 0 of tile u+1)
                    constexpr int j_lo = slot * 8 / kSpecSlots, j_hi = (slot + 1) * 8 / kSpecSlots;
                    static_for<j_hi - j_lo>([&](auto dj) {
                        constexpr int j = j_lo + dj, pr = kJobPair[j];
                        constexpr int q0 = ((s + 1) % kWideSpecs) * 8 + 2 * pr;
                        if constexpr (kJobStage[j] == 1) {
                            uint32_t a = wide_operand_s1<R, q0>(e), b = wide_operand_s1<R, q0 + 1>(e);
                            // Keeps the work in this slot.  Needed for correctness, not only for the schedule: the
                            // compiler places no wait states between these vector writes and an MFMA it cannot see
                            // inside inline assembly, so the operands must be formed a slot ahead of their use.
                            asm volatile("" : "+v"(a), "+v"(b));
                            half_done[pr][0] = a;
                            half_done[pr][1] = b;
                        } else {
                            uint32_t a = wide_operand_s2<R, q0>(half_done[pr][0], sc, nz);
                            uint32_t b = wide_operand_s2<R, q0 + 1>(half_done[pr][1], sc, nz);
                            asm volatile("" : "+v"(a), "+v"(b));
                            Wq[SP ^ 1][2 * pr] = a;
                            Wq[SP ^ 1][2 * pr + 1] = b;
                        }
                    });
                    if constexpr (h == 1 && pos + kAhead < C * 8) aq[pos % kAhead] = a_at(pos + kAhead);
                    // this body's transfers, one piece per slot: the stage read during the previous body takes
                    // the activations NST-1 tiles ahead, the ring slot of tile u (all of it is in registers)
                    // takes tile u + NBR
                    constexpr int piece = s * kSpecSlots + slot;
                    if constexpr (piece < kXBlocks) fetch_x_piece(IntC<piece>{}, st_fill);
                    else if constexpr (piece < kPieces) fetch_tile_piece(IntC<piece - kXBlocks>{}, slot_cur);
                    __builtin_amdgcn_sched_barrier(0);
                });
            });
        });
        // the next tile's activations were issued NST-2 bodies ago, before that body's weight tile
        wait_transfers<(NST - 2) * (kXLines + kTileOps) + kTileOps>();
        lds_barrier();  // next stage complete for every wave, current stage free
        st = st_next;
        slot_cur = slot_next;
        ++g;
        if (g == G || !more) {
            const int rb = 4 * srb + wv;
            if (rb < rb_real) {
                const uint64_t a = L.cost_start + ((uint64_t)pass * L.RB * G + (uint64_t)srb * G) * L.cost;
                StackParams pw = p;  // this wave's quarter of the workgroup's slots
                pw.part = p.part + (size_t)wv * (C * 32 * 64);
                const int row0 = rb * kRowBlock + (lane & 31);
                const int colq = 4 * (lane >> 5);
                asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");  // the last MFMA's result must have left the matrix pipe
                finish_row_block_blocked<2 * C>(
                    L, pw, p.cnt + L.cnt_off + pass * rb_real + rb, a, ga, g,
                    [&](auto b) { return read_acc<AG>(acc[b / 2][b % 2]); }, worker, lane,
                    [&](auto b, const float(&tot)[16]) {
                        // register v of lane l: batch column 8*(v/4) + 4*(l/32) + v%4 of the chunk, weight row l%32 of the half
                        constexpr int c = b / 2, hrow = b % 2;
                        const int row = row0 + 32 * hrow;
                        const int col0 = (c0 + c) * kWideCols + colq;
                        if (row >= L.N || col0 >= L.M) return;
                        uint16_t MQ_GLOBAL *dst = gl(reinterpret_cast<uint16_t *>(L.y)) + (size_t)col0 * L.N + row;
                        const int fl = L.flags;
                        if (col0 + 28 <= L.M) {  // all 16 columns of this lane are inside the batch
#pragma unroll
                            for (int v = 0; v < 16; ++v) dst[(size_t)(8 * (v >> 2) + (v & 3)) * L.N] = y_bits(tot[v], fl);
                        } else {
#pragma unroll
                            for (int v = 0; v < 16; ++v) {
                                const int dc = 8 * (v >> 2) + (v & 3);
                                if (col0 + dc < L.M) dst[(size_t)dc * L.N] = y_bits(tot[v], fl);
                            }
                        }
                    });
            }
            if (g == G) { ++srb; g = 0; }
            ga = g;
            clear_acc();
            // Everything the hand-over loaded or stored has retired before the tile loop goes on: otherwise
            // the compiler, which keeps count of ITS memory instructions only, protects their registers at
            // the top of every following tile with a wait that also drains the transfers in flight.
            __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0), other counters untouched
        }
    }
    wait_transfers<0>();  // nothing of this run may land in LDS after the next run has started
}

template <int C, bool TWO = false> __global__ __launch_bounds__(256, TWO ? 2 : 1) void wide_stack_kernel(const StackParams p) {
    extern __shared__ __attribute__((aligned(16))) uint8_t lds_generic[];
    MQ_LDS uint8_t *lds = (MQ_LDS uint8_t *)lds_generic;
    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int worker = blockIdx.x;
    walk_tiles(p, worker, [&](const LayerDesc &L, int u_begin, int u_end) __attribute__((always_inline)) {
        const int per_pass = L.RB * L.G;  // RB counts super row blocks on this path
        for (int pass = u_begin / per_pass; pass < L.CB && pass * per_pass < u_end; ++pass) {
            const int lo = (u_begin > pass * per_pass ? u_begin : pass * per_pass) - pass * per_pass;
            const int hi = (u_end < (pass + 1) * per_pass ? u_end : (pass + 1) * per_pass) - pass * per_pass;
            if (lo >= hi) continue;
            switch (L.r) {
                case 2: run_wide_units<2, C, TWO>(L, p, pass, lo, hi, worker, wv, lane, lds); break;
                case 3: run_wide_units<3, C, TWO>(L, p, pass, lo, hi, worker, wv, lane, lds); break;
                case 4: run_wide_units<4, C, TWO>(L, p, pass, lo, hi, worker, wv, lane, lds); break;
                case 6: run_wide_units<6, C, TWO>(L, p, pass, lo, hi, worker, wv, lane, lds); break;
                default: run_wide_units<8, C, TWO>(L, p, pass, lo, hi, worker, wv, lane, lds); break;
            }
        }
    });
}

// workgroups the device keeps resident for a launch with lds_bytes of LDS per workgroup
template <int C, bool TWO> static int wide_resident_groups(int lds_bytes) {
    static int cached_bytes[2] = {0, 0}, cached[2] = {0, 0};
    for (int i = 0; i < 2; ++i)
        if (cached_bytes[i] == lds_bytes) return cached[i];
    int dev = 0, cus = 0, blocks = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(&wide_stack_kernel<C, TWO>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, wide_lds_bytes_max(C, TWO)) != hipSuccess)
        return 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&blocks, wide_stack_kernel<C, TWO>, 256, lds_bytes) != hipSuccess)
        return 0;
    if (blocks < 1) blocks = 1;
    int w = cus * blocks;
    if (w > wide_max_groups(C)) w = wide_max_groups(C);
    if (!TWO && w > cus) w = cus;  // this variant is planned for a compute unit of its own
    const int slot = cached_bytes[0] == 0 ? 0 : 1;
    cached_bytes[slot] = lds_bytes;
    cached[slot] = w;
    return w;
}

template <int C, bool TWO> static hipError_t launch_wide_c(StackParams p, int max_cost, hipStream_t s) {
    // LDS per workgroup: a single layer takes the plan of its width, a stack the largest plan
    int lds_bytes = wide_lds_bytes_max(C, TWO);
    if (!p.table) {
        switch (p.single.r) {
            case 2: lds_bytes = wide_lds_bytes(2, C, TWO); break;
            case 3: lds_bytes = wide_lds_bytes(3, C, TWO); break;
            case 4: lds_bytes = wide_lds_bytes(4, C, TWO); break;
            case 6: lds_bytes = wide_lds_bytes(6, C, TWO); break;
            default: lds_bytes = wide_lds_bytes(8, C, TWO); break;
        }
    }
    const int hw = wide_resident_groups<C, TWO>(lds_bytes);
    if (hw <= 0) return hipErrorUnknown;
    // shares of at least eight super-tiles: a small layer cut into more shares spends more on handing its row blocks
    // over than it gains in parallelism (Llama-2-7B shapes at M = 128: 52 -> 40 us per call)
    uint64_t cap = p.cost_total / ((uint64_t)max_cost * 8);
    if (cap < 1) cap = 1;
    p.nworkers = (int)(cap < (uint64_t)hw ? cap : (uint64_t)hw);
    if (!p.table && p.nworkers == hw) {
        // Single layer: every workgroup re-reads the activations of a group for each of its row blocks, which
        // only stays cheap while the workgroups of a chip walk the SAME groups at the same time (then one
        // fetch serves them all from the L2).  Equal shares do that when a share is a whole number of row
        // blocks, or a whole fraction of one: give up a few compute units for such a share length.
        const int64_t G = p.single.G, T = (int64_t)p.single.CB * p.single.RB * G;
        for (int w = hw; w >= hw - hw / 4; --w) {
            if (T % w) continue;
            const int64_t len = T / w;
            if (len % G == 0 || G % len == 0) {
                p.nworkers = w;
                break;
            }
        }
    }
    p.nwaves = p.nworkers * 4;
    p.slot_floats = 4 * C * 32 * 64;
    const hipError_t e = launch(xprep_wide_kernel, dim3((unsigned)p.n_jobs), dim3(256), 0, s, p);
    if (e != hipSuccess) return e;
    return launch(wide_stack_kernel<C, TWO>, dim3((unsigned)p.nworkers), dim3(256), (unsigned)lds_bytes, s, p);
}

hipError_t launch_stack_wide(StackParams p, int max_cost, hipStream_t s) {
    switch (wide_chunks_per_pass(p.M)) {
        // Two workgroups per compute unit pay off where shares are long (a stack: 16 Llama-3-70B blocks at M = 64 take
        // 2.56 ms instead of 2.98).  A single layer cut into twice as many shares hands twice as many partial row
        // blocks over (64 KB each) and gains nothing: it keeps one workgroup per compute unit and the deeper rings.
        case 1: return p.table ? launch_wide_c<1, true>(p, max_cost, s) : launch_wide_c<1, false>(p, max_cost, s);
        case 2: return p.table ? launch_wide_c<2, true>(p, max_cost, s) : launch_wide_c<2, false>(p, max_cost, s);
        case 3: return launch_wide_c<3, false>(p, max_cost, s);
        default: return launch_wide_c<4, false>(p, max_cost, s);
    }
}

}  // namespace mq
