// The MatGPTQ column loop (Algorithm 2 of the paper's appendix), from the point where U, the
// upper-triangular Cholesky factor of the inverse Hessian, is given.  Rows of W are independent of
// each other; columns are strictly sequential (each column's code depends on every earlier
// column's error), so the work is cut as the listing cuts it:
//
//   gptq_block_kernel    : walks the B columns of a block for the rows of one wave: Algorithm 1
//                          on the current weight (mq_quant_core.h: the operations of the
//                          whole-matrix kernel, the 256 candidates spread over the 4, 16 or 64
//                          lanes that share a row), the error averaged over R and divided by
//                          U[j,j], rank-1 update of the block's remaining columns, which live in
//                          LDS;
//   gptq_trailing_kernel : W[:, i+B:] -= E @ U[i:i+B, i+B:], eight rows x four columns per lane.
//
// Every rounding decides later codes, so the arithmetic is fixed: binary32, each operation
// rounded on its own (no contraction), the error sum over r ascending as ((w - D_r1) + (w - D_r2))
// + ..., then / |R|, then / U[j,j]; an update is w = w - (E * U[j,k]); the update of the rest is
// applied as the same rank-1 terms in ascending j, so results do not depend on B.
#include "mq_quant_core.h"

namespace mq {

constexpr int kGptqMaxBlock = 128;
constexpr int kTrailRows = 8;

__device__ __forceinline__ float slice_value(uint32_t q, int r) {
    const int sh = kC - r;
    uint32_t t = sh ? (q + (1u << (sh - 1))) >> sh : q;
    const uint32_t top = (1u << r) - 1;
    t = t < top ? t : top;
    return (float)(t << sh);
}

// Lexicographic minimum of (E, q) over groups of LPR consecutive lanes, result in every lane of the
// group.  E >= 0, so the float order is the order of the bit patterns; equal E -> smaller q.
template <int CTRL> __device__ __forceinline__ void argmin_dpp(float &e, uint32_t &q) {
    const float oe = __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, e), CTRL, 0xf, 0xf, false));
    const uint32_t oq = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)q, CTRL, 0xf, 0xf, false);
    const bool take = oe < e || (oe == e && oq < q);
    e = take ? oe : e;
    q = take ? oq : q;
}
__device__ __forceinline__ void argmin_xor(float &e, uint32_t &q, int mask) {
    const float oe = __shfl_xor(e, mask);
    const uint32_t oq = (uint32_t)__shfl_xor((int)q, mask);
    const bool take = oe < e || (oe == e && oq < q);
    e = take ? oe : e;
    q = take ? oq : q;
}
template <int LPR> __device__ __forceinline__ void row_argmin(float &e, uint32_t &q) {
    static_assert(LPR == 4 || LPR == 16 || LPR == 64, "lanes per row");
    argmin_dpp<0xB1>(e, q);  // quad_perm [1,0,3,2]
    argmin_dpp<0x4E>(e, q);  // quad_perm [2,3,0,1]
    if constexpr (LPR >= 16) {
        argmin_dpp<0x141>(e, q);  // row_half_mirror: the two quads of each 8 lanes
        argmin_dpp<0x140>(e, q);  // row_mirror: the two halves of each 16 lanes
    }
    if constexpr (LPR == 64) {
        argmin_xor(e, q, 16);
        argmin_xor(e, q, 32);
    }
}

// One wave per workgroup; LPR lanes share a row: each evaluates 256 / LPR of the candidates, and
// they split the columns of the in-block update.  The block's current weights live in LDS as
// [column][row of the wave]; the values of U a lane needs for column j+1 are fetched into
// registers while column j is being decided.
template <uint32_t MASK, int LPR>
__global__ __launch_bounds__(64) void gptq_block_kernel(const float *__restrict__ W, int64_t ldw, int64_t N, int64_t i0,
                                                        int B, const float *__restrict__ U, int64_t ldu,
                                                        const _Float16 *__restrict__ scales,
                                                        const _Float16 *__restrict__ zeros, int64_t G,
                                                        const QuantLambda lam, float n_widths,
                                                        uint8_t *__restrict__ Q, int64_t ldq, float *__restrict__ E) {
#pragma clang fp contract(off)
    constexpr int RPW = 64 / LPR, CPL = 256 / LPR, CNT = kGptqMaxBlock / LPR;
    __shared__ float wl[kGptqMaxBlock * RPW];
    const int lane = threadIdx.x;
    const int rl = lane / LPR, part = lane % LPR;
    const int64_t n = (int64_t)blockIdx.x * RPW + rl;
    const bool valid = n < N;
    const int64_t nr = valid ? n : N - 1;  // idle lanes shadow the last row and store nothing
    for (int k = part; k < B; k += LPR) wl[k * RPW + rl] = W[nr * ldw + i0 + k];
    // a block never straddles a group (B divides the group size and blocks start at multiples of B)
    const int64_t g = i0 / kGroup;
    const float s = (float)scales[nr * G + g];
    const float z = (float)zeros[nr * G + g];
    // this lane's pieces of row j of U: the diagonal and columns j + 1 + part + c * LPR (clamped into the block)
    float un[CNT], ujj_n;
    auto fetch_u = [&](int j) {
        const float *urow = U + (i0 + j) * ldu + i0;
        ujj_n = urow[j];
#pragma unroll
        for (int c = 0; c < CNT; ++c) {
            const int k = j + 1 + part + c * LPR;
            un[c] = urow[k < B ? k : B - 1];
        }
    };
    fetch_u(0);
    __syncthreads();
    for (int j = 0; j < B; ++j) {
        float uc[CNT];
#pragma unroll
        for (int c = 0; c < CNT; ++c) uc[c] = un[c];
        const float ujj = ujj_n;
        if (j + 1 < B) fetch_u(j + 1);
        const float w = wl[j * RPW + rl];
        float best;
        uint32_t q;
        choose_codes_part<MASK, CPL>(w, s, z, lam, (uint32_t)(part * CPL), best, q);
        row_argmin<LPR>(best, q);
        float acc = 0.f;
        bool first = true;
#pragma unroll
        for (int r = 1; r <= kC; ++r) {
            if (lam.v[r - 1] != 0.f) {  // uniform: R is the set of widths with a non-zero lambda
                const float t = slice_value(q, r) - z;
                const float D = s * t;
                const float d = w - D;
                acc = first ? d : acc + d;
                first = false;
            }
        }
        const float err = (acc / n_widths) / ujj;
        if (valid && part == 0) {
            Q[n * ldq + i0 + j] = (uint8_t)q;
            E[n * B + j] = err;
        }
#pragma unroll
        for (int c = 0; c < CNT; ++c) {
            const int k = j + 1 + part + c * LPR;
            if (k < B) {
                const float p = err * uc[c];
                wl[k * RPW + rl] = wl[k * RPW + rl] - p;
            }
        }
    }
}

// W[n, c0 + k] -= sum_j E[n, j] * U[i0 + j, c0 + k], the terms subtracted one by one in ascending j.
// A wave owns kTrailRows rows x 256 columns (four consecutive columns per lane): per j one 16-byte
// load of U per lane, the E values are the same for the whole wave (scalar loads), and 2 x 4 x
// kTrailRows vector operations, so the kernel is bound by the vector ALUs, not by loads.
// VEC4 needs c0, ldw, ldu multiples of 4 and 16-byte aligned W and U; otherwise one column per lane.
template <bool VEC4>
__global__ __launch_bounds__(64) void gptq_trailing_kernel(float *__restrict__ W, int64_t ldw, int64_t N, int64_t c0,
                                                           int64_t ncols, const float *__restrict__ E, int B,
                                                           const float *__restrict__ U, int64_t ldu, int64_t i0,
                                                           int64_t kblocks) {
#pragma clang fp contract(off)
    constexpr int CPT = VEC4 ? 4 : 1;  // columns per lane
    const int64_t rb = blockIdx.x / kblocks;
    const int64_t k = ((blockIdx.x - rb * kblocks) * 64 + threadIdx.x) * CPT;
    const int64_t n0 = rb * kTrailRows;
    const bool in = k < ncols;  // ncols is a multiple of CPT on the VEC4 path
    const int64_t kc = in ? k : 0;
    float w[kTrailRows][CPT];
    int64_t row[kTrailRows];
#pragma unroll
    for (int i = 0; i < kTrailRows; ++i) {
        row[i] = n0 + i < N ? n0 + i : N - 1;  // uniform over the wave
        const float *src = W + row[i] * ldw + c0 + kc;
        if constexpr (VEC4) {
            const float4 v = *reinterpret_cast<const float4 *>(src);
            w[i][0] = v.x; w[i][1] = v.y; w[i][2] = v.z; w[i][3] = v.w;
        } else {
            w[i][0] = src[0];
        }
    }
    const float *u = U + i0 * ldu + c0 + kc;
    // eight terms at a time: their loads (one 16-byte piece of U per lane and term, eight consecutive E values
    // per row through the scalar unit) are all issued before the first of them is used
    constexpr int JC = 8;  // B is a multiple of 16
    for (int j0 = 0; j0 < B; j0 += JC) {
        float uv[JC][CPT];
#pragma unroll
        for (int jj = 0; jj < JC; ++jj) {
            if constexpr (VEC4) {
                const float4 v = *reinterpret_cast<const float4 *>(u + (int64_t)(j0 + jj) * ldu);
                uv[jj][0] = v.x; uv[jj][1] = v.y; uv[jj][2] = v.z; uv[jj][3] = v.w;
            } else {
                uv[jj][0] = u[(int64_t)(j0 + jj) * ldu];
            }
        }
        float ev[kTrailRows][JC];
#pragma unroll
        for (int i = 0; i < kTrailRows; ++i)
#pragma unroll
            for (int jj = 0; jj < JC; ++jj) ev[i][jj] = E[row[i] * B + j0 + jj];
#pragma unroll
        for (int jj = 0; jj < JC; ++jj)
#pragma unroll
            for (int i = 0; i < kTrailRows; ++i)
#pragma unroll
                for (int c = 0; c < CPT; ++c) {
                    const float p = ev[i][jj] * uv[jj][c];
                    w[i][c] = w[i][c] - p;
                }
    }
    if (!in) return;
#pragma unroll
    for (int i = 0; i < kTrailRows; ++i) {
        if (n0 + i < N) {
            float *dst = W + (n0 + i) * ldw + c0 + k;
            if constexpr (VEC4)
                *reinterpret_cast<float4 *>(dst) = make_float4(w[i][0], w[i][1], w[i][2], w[i][3]);
            else
                dst[0] = w[i][0];
        }
    }
}

template <uint32_t MASK, int LPR>
static hipError_t launch_gptq_block(const float *W, int64_t ldw, int64_t N, int64_t i0, int B, const float *U, int64_t ldu,
                              const _Float16 *scales, const _Float16 *zeros, int64_t G, const QuantLambda &lam,
                              float n_widths, uint8_t *Q, int64_t ldq, float *E, hipStream_t s) {
    constexpr int RPW = 64 / LPR;
    return launch((gptq_block_kernel<MASK, LPR>), dim3((unsigned)((N + RPW - 1) / RPW)), dim3(64), 0, s, W, ldw, N, i0, B, U,
                  ldu, scales, zeros, G, lam, n_widths, Q, ldq, E);
}

// Lanes per row: the column steps are a dependent chain, so the chip is filled by spreading each
// step's rows x candidates over the waves: the most lanes per row that keep the launch within about
// four waves per SIMD (measured on 4096 and 11008 rows: 64 lanes 7.0 / 14.2 ms, 16 lanes 8.1 / 11.5 ms,
// 4 lanes 15.6 / 17.9 ms for 4096 columns).
inline int gptq_lanes_per_row(int64_t N) { return N > 16384 ? 4 : N > 4096 ? 16 : 64; }

template <uint32_t MASK>
static hipError_t launch_gptq_mask(float *W, int64_t ldw, int64_t N, int64_t K, const float *U, int64_t ldu,
                                   const _Float16 *scales, const _Float16 *zeros, const QuantLambda &lam, float n_widths,
                                   int B, uint8_t *Q, int64_t ldq, float *E, hipStream_t s) {
    const int64_t G = K / kGroup;
    if (((K + 63) / 64) * ((N + kTrailRows - 1) / kTrailRows) > (int64_t)0x7fffffff) return hipErrorInvalidValue;
    const int lpr = gptq_lanes_per_row(N);
    // B, K and the block starts are multiples of 16, so only the strides and base addresses decide
    const bool vec4 = ldw % 4 == 0 && ldu % 4 == 0 && (reinterpret_cast<uintptr_t>(W) & 15) == 0 &&
                      (reinterpret_cast<uintptr_t>(U) & 15) == 0;
    for (int64_t i0 = 0; i0 < K; i0 += B) {
        hipError_t e;
        if (lpr == 4)
            e = launch_gptq_block<MASK, 4>(W, ldw, N, i0, B, U, ldu, scales, zeros, G, lam, n_widths, Q, ldq, E, s);
        else if (lpr == 16)
            e = launch_gptq_block<MASK, 16>(W, ldw, N, i0, B, U, ldu, scales, zeros, G, lam, n_widths, Q, ldq, E, s);
        else
            e = launch_gptq_block<MASK, 64>(W, ldw, N, i0, B, U, ldu, scales, zeros, G, lam, n_widths, Q, ldq, E, s);
        if (e != hipSuccess) return e;
        const int64_t c0 = i0 + B, ncols = K - c0;
        if (ncols > 0) {
            const int64_t rblocks = (N + kTrailRows - 1) / kTrailRows;
            if (vec4) {
                const int64_t kblocks = (ncols + 255) / 256;
                e = launch(gptq_trailing_kernel<true>, dim3((unsigned)(kblocks * rblocks)), dim3(64), 0, s, W, ldw, N, c0,
                           ncols, E, B, U, ldu, i0, kblocks);
            } else {
                const int64_t kblocks = (ncols + 63) / 64;
                e = launch(gptq_trailing_kernel<false>, dim3((unsigned)(kblocks * rblocks)), dim3(64), 0, s, W, ldw, N, c0,
                           ncols, E, B, U, ldu, i0, kblocks);
            }
            if (e != hipSuccess) return e;
        }
    }
    return hipSuccess;
}

hipError_t launch_gptq(float *W, int64_t ldw, int64_t N, int64_t K, const float *U, int64_t ldu, const _Float16 *scales,
                       const _Float16 *zeros, const float *lambda, int B, uint8_t *Q, int64_t ldq, float *E,
                       hipStream_t s) {
    QuantLambda lam;
    uint32_t need = 0;
    int nw = 0;
    for (int i = 0; i < kC; ++i) {
        lam.v[i] = lambda[i];
        if (lambda[i] != 0.f) {
            need |= 1u << i;
            ++nw;
        }
    }
    const float n_widths = (float)nw;
    switch (quant_variant_mask(need)) {
        case 0x80u: return launch_gptq_mask<0x80u>(W, ldw, N, K, U, ldu, scales, zeros, lam, n_widths, B, Q, ldq, E, s);
        case 0x8Cu: return launch_gptq_mask<0x8Cu>(W, ldw, N, K, U, ldu, scales, zeros, lam, n_widths, B, Q, ldq, E, s);
        case 0xAEu: return launch_gptq_mask<0xAEu>(W, ldw, N, K, U, ldu, scales, zeros, lam, n_widths, B, Q, ldq, E, s);
    }
    return launch_gptq_mask<0xFFu>(W, ldw, N, K, U, ldu, scales, zeros, lam, n_widths, B, Q, ldq, E, s);
}

}  // namespace mq
