// The MatGPTQ column loop (Algorithm 2 of the paper's appendix), from the point where U, the
// upper-triangular Cholesky factor of the inverse Hessian, is given.  Rows of W are independent of
// each other; columns are strictly sequential (each column's code depends on every earlier
// column's error), so the work is cut as the listing cuts it:
//
//   gptq_block_kernel    : one lane per row walks the B columns of a block: Algorithm 1 on the
//                          current weight (mq_quant_core.h, the same code as the whole-matrix
//                          kernel), the error averaged over R and divided by U[j,j], rank-1 update
//                          of the block's remaining columns, which live in LDS ([column][lane]:
//                          no bank conflicts, no dynamically indexed registers) next to the
//                          block's corner of U;
//   gptq_trailing_kernel : W[:, i+B:] -= E @ U[i:i+B, i+B:], four rows per lane.
//
// Every rounding decides later codes, so the arithmetic is fixed: binary32, each operation
// rounded on its own (no contraction), the error sum over r ascending as ((w - D_r1) + (w - D_r2))
// + ..., then / |R|, then / U[j,j]; an update is w = w - (E * U[j,k]); the update of the rest is
// applied as the same rank-1 terms in ascending j, so results do not depend on B.
#include "mq_quant_core.h"

namespace mq {

constexpr int kGptqMaxBlock = 128;
constexpr int kTrailRows = 4;

__device__ __forceinline__ float slice_value(uint32_t q, int r) {
    const int sh = kC - r;
    uint32_t t = sh ? (q + (1u << (sh - 1))) >> sh : q;
    const uint32_t top = (1u << r) - 1;
    t = t < top ? t : top;
    return (float)(t << sh);
}

// Dynamic LDS: [B][64] current weights of the block (column-major per wave), then the block's
// B x B corner of U (row-major), which every lane reads by broadcast.
template <uint32_t MASK>
__global__ __launch_bounds__(64) void gptq_block_kernel(const float *__restrict__ W, int64_t ldw, int64_t N, int64_t i0,
                                                        int B, const float *__restrict__ U, int64_t ldu,
                                                        const _Float16 *__restrict__ scales,
                                                        const _Float16 *__restrict__ zeros, int64_t G,
                                                        const QuantLambda lam, float n_widths,
                                                        uint8_t *__restrict__ Q, int64_t ldq, float *__restrict__ E) {
#pragma clang fp contract(off)
    extern __shared__ __attribute__((aligned(16))) float lds[];
    float *wl = lds;            // wl[k * 64 + lane]
    float *ul = lds + B * 64;   // ul[j * B + k] = U[i0 + j, i0 + k]
    const int lane = threadIdx.x;
    const int64_t n = (int64_t)blockIdx.x * 64 + lane;
    const bool valid = n < N;
    const int64_t nr = valid ? n : N - 1;  // idle lanes shadow the last row and store nothing
    for (int k = 0; k < B; ++k) wl[k * 64 + lane] = W[nr * ldw + i0 + k];
    for (int idx = lane; idx < B * B; idx += 64) {
        const int j = idx / B, k = idx - j * B;
        ul[idx] = U[(i0 + j) * ldu + i0 + k];
    }
    // a block never straddles a group (B divides the group size and blocks start at multiples of B)
    const int64_t g = i0 / kGroup;
    const float s = (float)scales[nr * G + g];
    const float z = (float)zeros[nr * G + g];
    __syncthreads();
    for (int j = 0; j < B; ++j) {
        float w[1] = {wl[j * 64 + lane]};
        uint32_t q[1];
        choose_codes<MASK, 1>(w, s, z, lam, q);
        float acc = 0.f;
        bool first = true;
#pragma unroll
        for (int r = 1; r <= kC; ++r) {
            if (lam.v[r - 1] != 0.f) {  // uniform: R is the set of widths with a non-zero lambda
                const float t = slice_value(q[0], r) - z;
                const float D = s * t;
                const float d = w[0] - D;
                acc = first ? d : acc + d;
                first = false;
            }
        }
        const float *urow = ul + j * B;
        const float err = (acc / n_widths) / urow[j];
        if (valid) {
            Q[n * ldq + i0 + j] = (uint8_t)q[0];
            E[n * B + j] = err;
        }
        for (int k = j + 1; k < B; ++k) {
            const float p = err * urow[k];
            wl[k * 64 + lane] = wl[k * 64 + lane] - p;
        }
    }
}

// W[n, c0 + k] -= sum_j E[n, j] * U[i0 + j, c0 + k], the terms subtracted one by one in ascending j.
__global__ __launch_bounds__(256) void gptq_trailing_kernel(float *__restrict__ W, int64_t ldw, int64_t N, int64_t c0,
                                                            int64_t ncols, const float *__restrict__ E, int B,
                                                            const float *__restrict__ U, int64_t ldu, int64_t i0,
                                                            int64_t kblocks) {
#pragma clang fp contract(off)
    const int64_t rb = blockIdx.x / kblocks;
    const int64_t k = (blockIdx.x - rb * kblocks) * 256 + threadIdx.x;
    if (k >= ncols) return;
    const int64_t n0 = rb * kTrailRows;
    float w[kTrailRows];
    int64_t row[kTrailRows];
#pragma unroll
    for (int i = 0; i < kTrailRows; ++i) {
        row[i] = n0 + i < N ? n0 + i : N - 1;
        w[i] = W[row[i] * ldw + c0 + k];
    }
    const float *u = U + i0 * ldu + c0 + k;
    for (int j = 0; j < B; ++j) {
        const float uv = u[(int64_t)j * ldu];
#pragma unroll
        for (int i = 0; i < kTrailRows; ++i) {
            const float p = E[row[i] * B + j] * uv;
            w[i] = w[i] - p;
        }
    }
#pragma unroll
    for (int i = 0; i < kTrailRows; ++i)
        if (n0 + i < N) W[(n0 + i) * ldw + c0 + k] = w[i];
}

template <uint32_t MASK>
static hipError_t launch_gptq_mask(float *W, int64_t ldw, int64_t N, int64_t K, const float *U, int64_t ldu,
                                   const _Float16 *scales, const _Float16 *zeros, const QuantLambda &lam, float n_widths,
                                   int B, uint8_t *Q, int64_t ldq, float *E, hipStream_t s) {
    const int64_t G = K / kGroup;
    if (((K + 255) / 256) * ((N + kTrailRows - 1) / kTrailRows) > (int64_t)0x7fffffff) return hipErrorInvalidValue;
    const size_t lds_bytes = ((size_t)B * 64 + (size_t)B * B) * sizeof(float);  // 96 KB at B = 128
    static bool attr_set = false;  // per variant; same value every time, so a race between threads is harmless
    if (!attr_set) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(gptq_block_kernel<MASK>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize,
                                                 (int)((kGptqMaxBlock * 64 + kGptqMaxBlock * kGptqMaxBlock) * sizeof(float)));
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    (void)hipGetLastError();  // drop stale errors of earlier, unrelated calls
    for (int64_t i0 = 0; i0 < K; i0 += B) {
        hipLaunchKernelGGL((gptq_block_kernel<MASK>), dim3((unsigned)((N + 63) / 64)), dim3(64), lds_bytes, s, W, ldw, N, i0,
                           B, U, ldu, scales, zeros, G, lam, n_widths, Q, ldq, E);
        const int64_t c0 = i0 + B, ncols = K - c0;
        if (ncols > 0) {
            const int64_t kblocks = (ncols + 255) / 256;
            const int64_t rblocks = (N + kTrailRows - 1) / kTrailRows;
            hipLaunchKernelGGL(gptq_trailing_kernel, dim3((unsigned)(kblocks * rblocks)), dim3(256), 0, s, W, ldw, N, c0,
                               ncols, E, B, U, ldu, i0, kblocks);
        }
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
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
