// Global memory -> LDS transfers without registers (global_load_lds), the waits that go with them, and the
// workgroup barrier for LDS traffic: shared by the matrix-core kernels (mq_gemm.hip, mq_wide.hip).
#pragma once
#include "mq_device.h"

namespace mq {

// Workgroup barrier that orders LDS traffic only: a wave's global loads stay in flight across it.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// ---- memory pipeline.  Weights and activations travel from global memory straight into LDS
// (global_load_lds: 16 bytes per lane, no registers), issued from inline assembly so that the waits are
// ours: loads retire in order, and a wait the compiler derives for one load of a deep software pipeline
// tends to retire the whole pipeline.  Every wait below names how many LATER transfers of this wave may
// still be in flight; transfers the wave issues elsewhere only make such a wait stricter, never wrong.
// N consecutive 1 KB lines (16 bytes per lane each): lane addresses src_lane + i * 1024 -> LDS dst_wave + i * 1024.
// The instruction offset of global_load_lds applies to the global and to the LDS address alike, so four
// lines share one address register pair and one setting of M0 (the LDS base of the wave's transfer).
// NT: non-temporal (streaming) transfers for data that is read once per call -- the weights, scales and zeros; the
// activations are shared by every workgroup and stay ordinary transfers.
template <int N, bool NT = false>
__device__ __forceinline__ void dma_lines(const uint8_t *src_lane, MQ_LDS uint8_t *dst_wave) {
    static_assert(N >= 1 && N <= 8, "one or two blocks of up to four lines");
    const uint32_t base = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)dst_wave);
    const uint8_t MQ_GLOBAL *src = gl(src_lane);
    constexpr int N0 = N < 4 ? N : 4;
#define MQ_DMA_LINES(POL)                                                                                              \
    if constexpr (N0 == 1)                                                                                             \
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" POL ::"s"(base), "v"(src)         \
                     : "memory");                                                                                      \
    else if constexpr (N0 == 2)                                                                                        \
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" POL "\n\t"                        \
                     "global_load_lds_dwordx4 %1, off offset:1024" POL ::"s"(base),                                    \
                     "v"(src)                                                                                          \
                     : "memory");                                                                                      \
    else if constexpr (N0 == 3)                                                                                        \
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" POL "\n\t"                        \
                     "global_load_lds_dwordx4 %1, off offset:1024" POL "\n\t"                                          \
                     "global_load_lds_dwordx4 %1, off offset:2048" POL ::"s"(base),                                    \
                     "v"(src)                                                                                          \
                     : "memory");                                                                                      \
    else                                                                                                               \
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" POL "\n\t"                        \
                     "global_load_lds_dwordx4 %1, off offset:1024" POL "\n\t"                                          \
                     "global_load_lds_dwordx4 %1, off offset:2048" POL "\n\t"                                          \
                     "global_load_lds_dwordx4 %1, off offset:3072" POL ::"s"(base),                                    \
                     "v"(src)                                                                                          \
                     : "memory");
    if constexpr (NT) {
        MQ_DMA_LINES(" nt")
    } else {
        MQ_DMA_LINES("")
    }
#undef MQ_DMA_LINES
    if constexpr (N > 4) dma_lines<N - 4, NT>(src_lane + 4096, dst_wave + 4096);
}
// N transfers (N <= 4) of ONE line to one place: for a wave that must issue as many transfers as the others but has
// nothing left to fetch (after the first they are cache hits)
template <int N, bool NT = false>
__device__ __forceinline__ void dma_same_line(const uint8_t *src_lane, MQ_LDS uint8_t *dst_wave) {
    static_assert(N >= 1 && N <= 4, "up to four transfers");
    const uint32_t base = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)dst_wave);
    const uint8_t MQ_GLOBAL *src = gl(src_lane);
#define MQ_DMA_SAME(POL)                                                                                               \
    if constexpr (N == 1)                                                                                              \
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" POL ::"s"(base), "v"(src)         \
                     : "memory");                                                                                      \
    else if constexpr (N == 2)                                                                                         \
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" POL "\n\t"                        \
                     "global_load_lds_dwordx4 %1, off" POL ::"s"(base),                                                \
                     "v"(src)                                                                                          \
                     : "memory");                                                                                      \
    else if constexpr (N == 3)                                                                                         \
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" POL "\n\t"                        \
                     "global_load_lds_dwordx4 %1, off" POL "\n\t"                                                      \
                     "global_load_lds_dwordx4 %1, off" POL ::"s"(base),                                                \
                     "v"(src)                                                                                          \
                     : "memory");                                                                                      \
    else                                                                                                               \
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" POL "\n\t"                        \
                     "global_load_lds_dwordx4 %1, off" POL "\n\t"                                                      \
                     "global_load_lds_dwordx4 %1, off" POL "\n\t"                                                      \
                     "global_load_lds_dwordx4 %1, off" POL ::"s"(base),                                                \
                     "v"(src)                                                                                          \
                     : "memory");
    if constexpr (NT) {
        MQ_DMA_SAME(" nt")
    } else {
        MQ_DMA_SAME("")
    }
#undef MQ_DMA_SAME
}
// block B (four lines each, the last one shorter) of an N-line transfer
template <int N, int B, bool NT = false>
__device__ __forceinline__ void dma_block(const uint8_t *src_lane, MQ_LDS uint8_t *dst_wave) {
    static_assert(4 * B < N, "no such block");
    dma_lines<(N - 4 * B < 4 ? N - 4 * B : 4), NT>(src_lane + 4096 * B, dst_wave + 4096 * B);
}
template <int N> __device__ __forceinline__ void wait_transfers() {
    static_assert(N >= 0 && N <= 63, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

}  // namespace mq
