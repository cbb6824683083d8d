// Internal declarations shared by the host API and the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <tuple>
#include <type_traits>
#include <utility>

#include "../../include/mq.h"
#include "mq_layout.h"

namespace mq {

// Caps on the wavefronts / workgroups of a persistent launch.  They size the partial-sum slots of a workspace, which
// must be plain host arithmetic (callable without a device); every launcher asks the device for its compute units
// and the kernel's occupancy and launches min(what is resident there, the cap), so a smaller or larger part stays
// correct and only loses the slots it cannot use.  (8192 = 256 compute units x 32 waves, the MI355X.)
constexpr int kMaxWaves = 8192;
// Narrow matrix-core path (kValuMaxM < M <= kNarrowMaxM): a workgroup of kNarrowRowBlocks waves owns a super-tile of
// kNarrowRowBlocks row blocks x one group; one workgroup per compute unit.
constexpr int kNarrowRowBlocks = 8;
constexpr int kMaxGroupsNarrow = 256;
constexpr int kNarrowXtBlockBytes = 6 * 1024;  // prepared activations of one group: operand blocks + 16 factors
// Vector-ALU stack kernel: each wave serves several interleaved shares of the schedule, so that
// layers of different widths (different speed per byte) even out over the waves.
constexpr int kSharesPerWave = 8;
constexpr size_t kMaxSlotBytes = (size_t)32 << 20;
inline int max_workers_valu(int64_t M) {
    const size_t by_mem = kMaxSlotBytes / (2 * (size_t)M * 64 * sizeof(float));
    const size_t want = (size_t)kMaxWaves * kSharesPerWave;
    return (int)(by_mem < want ? by_mem : want);
}
constexpr int kCounterBytesAlign = 256;

// Batches up to kValuMaxM run on the vector ALUs; up to kNarrowMaxM on MFMA with 16 columns per
// chunk and one wave per tile; larger ones on MFMA with 32 columns per chunk, four waves per
// super-tile of 256 rows and up to kWideMaxChunks chunks against one unpacked tile.
constexpr int kValuMaxM = 4;
constexpr int kChunkCols = 16;
constexpr int kNarrowMaxM = 16;
constexpr int kWideCols = 32;
constexpr int kWideMaxChunks = 4;
constexpr int kWideXtBlockBytes = 8 * 1024;  // prepared activations of one (group, chunk of 32 columns)
inline bool use_wide(int64_t M) { return M > kNarrowMaxM; }
inline int wide_chunks(int64_t M) { return (int)((M + kWideCols - 1) / kWideCols); }
inline int wide_passes(int64_t M) { return (wide_chunks(M) + kWideMaxChunks - 1) / kWideMaxChunks; }
// chunks per pass (the kernel variant, 1..4); the chunk count is padded to passes * chunks per pass
inline int wide_chunks_per_pass(int64_t M) { return (wide_chunks(M) + wide_passes(M) - 1) / wide_passes(M); }
inline int wide_chunks_padded(int64_t M) { return wide_passes(M) * wide_chunks_per_pass(M); }
// workgroups a wide launch may use (sizes the partial-sum slots): one per compute unit, two up to two chunks per pass
inline int wide_max_groups(int C) { return C <= 2 ? 512 : 256; }

// One layer as the persistent kernels see it.
struct LayerDesc {
    const uint4 *Wp;
    const _Float16 *st;
    const _Float16 *zt;
    const _Float16 *x;
    _Float16 *y;
    const uint4 *xt;        // MFMA paths: activations re-ordered (narrow path: and scaled) by the prep kernel
    const void *x_bf16;     // vector-ALU path with kFlagXBf16: the caller's bf16 activations (x then points to their fp16 copy)
    int32_t N, K, G, RB;    // RB = row blocks = ceil(N/64); super row blocks on the matrix-core paths: ceil(N/512) narrow, ceil(N/256) wide
    int32_t r;
    int32_t cost;           // schedule cost of one (row block, group) tile
    int32_t cnt_off;        // index of this layer's first row-block counter (CB*RB counters)
    int32_t M;              // batch rows of x
    int32_t CB;             // column chunks: 1 on the vector-ALU path, ceil(M/16) on the MFMA path; wide path: passes
    int32_t job_start;      // prep kernel: sum of CB*G over the preceding layers
    int32_t rs;             // 0, or: Wp is the 8-bit parent (r == 8) and Eq. 1 to rs bits is applied in registers
    int32_t flags;          // kFlagXBf16: x holds bf16 values; kFlagYBf16: y is written as bf16
    int32_t zmask;          // -1; a symmetric layer: zt is zmask + 1 lines of 64 x 128.0, tile u reads line u & zmask
    int32_t chain;          // chained small stack: bits 0..7 the layer's stage; kChainWaits: x is read only after every earlier stage is complete
    uint64_t cost_start;    // sum of CB*RB*G*cost over the preceding layers
};

// The descriptors of a small stack (at most kSmallStackLayers layers), passed to its low-latency kernel with the kernel
// arguments: a workgroup reads its descriptor from there in 0.3 us, where a first read from the table in device memory
// took 1.2 us of a launch that lasts 8.
constexpr int kSmallStackLayers = 16;
constexpr int kChainWaits = 0x100;
constexpr int kChainMaxM = 3;
constexpr int kChainCounters = kSmallStackLayers + 1;
struct SmallTable {
    LayerDesc d[kSmallStackLayers];
};
static_assert(sizeof(SmallTable) <= 2048, "kernel arguments are limited to 4 KiB");

struct StackParams {
    const LayerDesc *table;  // device table, or nullptr to use `single`
    int32_t n_layers;
    int32_t nwaves;          // wavefronts launched
    int32_t nworkers;        // schedule shares ("workers"); wave w serves workers w, w + nwaves, ...
    uint64_t cost_total;
    float *part;             // [nworkers][2][slot_floats] partial sums
    int32_t *cnt;            // row-block counters, zero between launches
    int32_t M;
    int32_t slot_floats;     // floats per partial-sum slot (64*M; a workgroup's 8 x 64*16 on the narrow matrix-core path)
    int32_t n_jobs;          // prep kernel jobs (MFMA path)
    int32_t worker_cap;      // 0, or: `part` holds slots for this many schedule shares only (a small workspace)
    int32_t ks_cap;          // low-latency launch of a small stack: most K slices per row block (0: as one layer would choose)
    int32_t ll_start[16];    // ... and the first workgroup of each layer (a workgroup finds its layer without reading the table)
    // Chained small stack (some layer reads what earlier layers of the same launch write): the layers form stages,
    // a new stage starting at every layer that waits.  Counter chain_off + s of `cnt` counts the finished row blocks
    // of stage s, counter chain_off + kSmallStackLayers all of them; the last row block of the launch zeroes them.
    int32_t chain_total;     // row blocks of all layers; 0: nothing is chained and nothing is counted
    int32_t chain_off;
    int32_t stage_rb[16];    // row blocks per stage
    LayerDesc single;
};

// Schedule cost of a tile on the vector-ALU path: measured times of uniform stacks (12 Llama-3-70B blocks, units of
// 10 us) per batch M = 1..4.  At M = 1 the kernel is HBM-bound and the cost close to a tile's bytes (4r + 2 lines of
// 256 bytes: 100 : 140 : 180 : 260 : 340), but the narrow widths run a little below the HBM rate of the wide ones, and
// mixed stacks are 1.6-1.8 % faster with the measured ratios than with the byte-proportional ones.  From M = 2 on the M
// accumulators per lane make the narrow widths ALU-bound and the cost much flatter than the bytes.
inline int valu_tile_cost(int r, int M) {
    static const int t[4][5] = {{100, 122, 155, 222, 290}, {89, 96, 98, 138, 176}, {109, 118, 117, 148, 178},
                                {134, 143, 138, 177, 187}};
    const int ri = r == 2 ? 0 : r == 3 ? 1 : r == 4 ? 2 : r == 6 ? 3 : 4;
    return t[(M < 1 ? 1 : M > 4 ? 4 : M) - 1][ri];
}

// Narrow MFMA path (kValuMaxM < M <= kNarrowMaxM): a tile's time there is set by instruction issue more than by its
// bytes, so the measured per-tile times of uniform stacks are the costs (M = 8, 12 Llama-3-70B blocks: 1.11, 1.24,
// 1.24, 1.61, 1.87 ms for r = 2, 3, 4, 6, 8).  With the byte-proportional costs a 2-bit share ran 1.6 times as long as
// an 8-bit share of a mixed stack.
inline int mfma_tile_cost(int r) {
    switch (r) {
        case 2: return 111;
        case 3: return 124;
        case 4: return 124;
        case 6: return 161;
        default: return 187;
    }
}

// Wide MFMA path: cost of a super-tile (256 rows x one group) per pass with C chunks of 32 columns, again the measured
// times of uniform stacks (12 Llama-3-70B blocks at M = 32, 64, 96, 128; units of 10 us; the first two rows with two
// workgroups per compute unit, as stacks run there).  The matrix-core work grows with C, the unpacking with r; bytes
// matter least.
inline int wide_tile_cost(int r, int C) {
    static const int t[4][5] = {{130, 141, 147, 178, 199}, {173, 186, 191, 222, 239},
                                {239, 252, 262, 306, 323}, {293, 308, 318, 358, 377}};
    const int ri = r == 2 ? 0 : r == 3 ? 1 : r == 4 ? 2 : r == 6 ? 3 : 4;
    return t[(C < 1 ? 1 : C > 4 ? 4 : C) - 1][ri];
}

// Enqueue a kernel and return the status of THIS launch.  The runtime's sticky "last error" is neither read nor
// cleared, so an error the caller's own earlier work left pending stays where the caller will find it.
template <class... KArgs, size_t... I>
inline hipError_t launch_impl(void (*kernel)(KArgs...), dim3 grid, dim3 block, unsigned lds_bytes, hipStream_t s,
                              std::tuple<std::decay_t<KArgs>...> &vals, std::index_sequence<I...>) {
    void *ptrs[sizeof...(KArgs) ? sizeof...(KArgs) : 1] = {static_cast<void *>(&std::get<I>(vals))...};
    return hipLaunchKernel(reinterpret_cast<const void *>(kernel), grid, block, ptrs, lds_bytes, s);
}
template <class... KArgs, class... Args>
inline hipError_t launch(void (*kernel)(KArgs...), dim3 grid, dim3 block, unsigned lds_bytes, hipStream_t s, Args &&...args) {
    static_assert(sizeof...(KArgs) == sizeof...(Args), "argument count differs from the kernel's");
    std::tuple<std::decay_t<KArgs>...> vals{static_cast<std::decay_t<KArgs>>(std::forward<Args>(args))...};
    return launch_impl(kernel, grid, block, lds_bytes, s, vals, std::index_sequence_for<KArgs...>{});
}

inline int64_t pad_rows(int64_t N) { return (N + kRowBlock - 1) / kRowBlock * kRowBlock; }

// launchers (mq_pack.hip / mq_linear.hip); each returns the hipError of the launch
hipError_t launch_slice(const uint8_t *parent, int64_t n, int c, int r, uint8_t *out, hipStream_t s);
hipError_t launch_pack(const uint8_t *S, int64_t N, int64_t K, int r, uint4 *packed, hipStream_t s);
hipError_t launch_unpack(const uint4 *packed, int64_t N, int64_t K, int r, uint8_t *S, hipStream_t s);
hipError_t launch_slice_pack(const uint8_t *parent, int64_t N, int64_t K, int r, uint4 *packed, hipStream_t s);
hipError_t launch_reslice(const uint4 *parent8, int64_t N, int64_t K, int r, uint4 *packed, hipStream_t s);
// n layers in ceil(n / kResliceBatch) launches; all arrays are host arrays of n entries
constexpr int kResliceBatch = 16;
hipError_t launch_reslice_many(const uint4 *const *src, uint4 *const *dst, const int64_t *N, const int64_t *K,
                               const int *r, int n, hipStream_t s);
hipError_t launch_pack_meta(const _Float16 *sc, const _Float16 *zr, int64_t N, int64_t G, _Float16 *st,
                            _Float16 *zt, hipStream_t s);
hipError_t launch_fill_zero(void *p, size_t bytes, hipStream_t s);
// xor of all 16-byte words of buf is xor-ed into *out (measurement aid); bytes is a multiple of 16
hipError_t launch_read_probe(const void *buf, size_t bytes, uint32_t *out, hipStream_t s);
// table: host, n descriptors -> dst: device.  ceil(n / 32) small launches; the host array is free again on return.
hipError_t launch_write_table(const LayerDesc *table, int n, LayerDesc *dst, hipStream_t s);
// Algorithm 1 (mq_quant.hip).  lambda: host, kC floats (width r at [r-1]); vec4: four columns per lane (alignment checked by the caller)
// Algorithm 2 column loop (mq_gptq.hip): 2 * K / B launches on s.  E: device, N * B floats of scratch.
hipError_t launch_gptq(float *W, int64_t ldw, int64_t N, int64_t K, const float *U, int64_t ldu, const _Float16 *scales,
                       const _Float16 *zeros, const float *lambda, int B, uint8_t *Q, int64_t ldq, float *E,
                       hipStream_t s);
hipError_t launch_quant(const float *W, int64_t ldw, int64_t N, int64_t ncols, int64_t col0, const _Float16 *scales,
                        const _Float16 *zeros, int64_t G, const float *lambda, uint8_t *Q, int64_t ldq, bool vec4,
                        hipStream_t s);
// bf16 activations of the layers that carry kFlagXBf16 -> fp16 in their LayerDesc::xt (ahead of a vector-ALU launch)
hipError_t launch_xcvt(const StackParams &p, hipStream_t s);
// Fills p.nwaves and launches (vector-ALU path, M <= kValuMaxM).  max_cost = largest tile cost in the stack.
// from_parent: every layer has rs != 0 (the kernel variant that slices in registers).
hipError_t launch_stack(StackParams p, int max_cost, bool from_parent, hipStream_t s);
// Single layer, M <= kValuMaxM: one workgroup per (row block, K slice); see mq_linear.hip.
bool linear_rb_fits(const LayerDesc &L, size_t part_bytes);
hipError_t launch_linear_rb(const LayerDesc &L, float *part, int32_t *cnt, hipStream_t s);
// The same shape for a small stack (M <= kValuMaxM): all layers' workgroups in one launch.  `table` is the host copy
// of the descriptors; false = the stack is too big for it.
// ks_cap: see StackParams.
// ll_start: see StackParams (16 entries).
// all_resident: the device holds every workgroup of that shape at one time (what a chained stack needs).
bool linear_rb_stack_shape(const LayerDesc *table, int n_layers, size_t part_bytes, bool from_parent, bool chained,
                           int *blocks, int *waves, int *ks_cap, int32_t *ll_start, bool *all_resident);
hipError_t launch_linear_rb_stack(const StackParams &p, const SmallTable &t, int blocks, int waves, bool from_parent,
                                  hipStream_t s);
// MFMA path (M > kValuMaxM): activation prep kernel + persistent MFMA kernel.
hipError_t launch_stack_mfma(StackParams p, int max_cost, hipStream_t s);
// Wide MFMA path (M > kNarrowMaxM): activation prep kernel + persistent kernel, one workgroup per share.
hipError_t launch_stack_wide(StackParams p, int max_cost, hipStream_t s);

}  // namespace mq
