// Cross-bit-width choice of the parent code (Algorithm 1 of the paper): for every weight the code
// q in 0..255 that minimises
//     E(q) = sum_{r in R} lambda_r * (w - scale * (S(q, r) - zero))^2,      S = Eq. 1 (Section 2)
// by brute force over all 256 candidates, as the paper does (arithmetic: mq_quant_core.h).
// One lane owns VEC consecutive weights of a row (same group: same scale and zero).
#include "mq_quant_core.h"

namespace mq {

template <uint32_t MASK, int VEC>
__global__ __launch_bounds__(256) void quant_kernel(const float *__restrict__ W, int64_t ldw, int64_t N, int64_t ncols,
                                                    int64_t col0, const _Float16 *__restrict__ scales,
                                                    const _Float16 *__restrict__ zeros, int64_t G,
                                                    const QuantLambda lam, uint8_t *__restrict__ Q, int64_t ldq) {
    const int64_t cv = ncols / VEC;
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= N * cv) return;
    const int64_t n = idx / cv;
    const int64_t col = (idx - n * cv) * VEC;
    const int64_t g = (col0 + col) / kGroup;
    const float s = (float)scales[n * G + g];
    const float z = (float)zeros[n * G + g];
    float w[VEC];
    const float *src = W + n * ldw + col;
    if constexpr (VEC == 4) {
        const float4 v = *reinterpret_cast<const float4 *>(src);
        w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
    } else {
        w[0] = src[0];
    }
    uint32_t qb[VEC];
    choose_codes<MASK, VEC>(w, s, z, lam, qb);
    uint8_t *dst = Q + n * ldq + col;
    if constexpr (VEC == 4)
        *reinterpret_cast<uint32_t *>(dst) = qb[0] | (qb[1] << 8) | (qb[2] << 16) | (qb[3] << 24);
    else
        dst[0] = (uint8_t)qb[0];
}

template <uint32_t MASK>
static hipError_t launch_quant_mask(const float *W, int64_t ldw, int64_t N, int64_t ncols, int64_t col0,
                                    const _Float16 *scales, const _Float16 *zeros, int64_t G, const QuantLambda &lam,
                                    uint8_t *Q, int64_t ldq, bool vec4, hipStream_t s) {
    const int64_t threads = vec4 ? N * (ncols / 4) : N * ncols;
    const int64_t blocks = (threads + 255) / 256;
    if (blocks > (int64_t)0x7fffffff) return hipErrorInvalidValue;  // beyond one grid dimension
    if (vec4)
        return launch((quant_kernel<MASK, 4>), dim3((unsigned)blocks), dim3(256), 0, s, W, ldw, N, ncols, col0, scales, zeros,
                      G, lam, Q, ldq);
    return launch((quant_kernel<MASK, 1>), dim3((unsigned)blocks), dim3(256), 0, s, W, ldw, N, ncols, col0, scales, zeros, G,
                  lam, Q, ldq);
}

hipError_t launch_quant(const float *W, int64_t ldw, int64_t N, int64_t ncols, int64_t col0, const _Float16 *scales,
                        const _Float16 *zeros, int64_t G, const float *lambda, uint8_t *Q, int64_t ldq, bool vec4,
                        hipStream_t s) {
    QuantLambda lam;
    uint32_t need = 0;
    for (int i = 0; i < kC; ++i) {
        lam.v[i] = lambda[i];
        if (lambda[i] != 0.f) need |= 1u << i;
    }
    switch (quant_variant_mask(need)) {
        case 0x80u: return launch_quant_mask<0x80u>(W, ldw, N, ncols, col0, scales, zeros, G, lam, Q, ldq, vec4, s);
        case 0x8Cu: return launch_quant_mask<0x8Cu>(W, ldw, N, ncols, col0, scales, zeros, G, lam, Q, ldq, vec4, s);
        case 0xAEu: return launch_quant_mask<0xAEu>(W, ldw, N, ncols, col0, scales, zeros, G, lam, Q, ldq, vec4, s);
    }
    return launch_quant_mask<0xFFu>(W, ldw, N, ncols, col0, scales, zeros, G, lam, Q, ldq, vec4, s);
}

}  // namespace mq
