// Internal declarations shared by the host API and the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/mq.h"
#include "mq_layout.h"

namespace mq {

// Upper bound on resident wavefronts of a persistent launch (256 CUs x 32);
// sizes the partial-sum slots of a workspace independently of the device.
constexpr int kMaxWaves = 8192;
constexpr int kCounterBytesAlign = 256;

// One layer as the persistent kernel sees it.
struct LayerDesc {
    const uint4 *Wp;
    const _Float16 *st;
    const _Float16 *zt;
    const _Float16 *x;
    _Float16 *y;
    int32_t N, K, G, RB;    // RB = row blocks = ceil(N/64)
    int32_t r;
    int32_t cost;           // schedule cost of one (row block, group) tile
    int32_t cnt_off;        // index of this layer's first row-block counter
    int32_t pad_;
    uint64_t cost_start;    // sum of RB*G*cost over the preceding layers
};

struct StackParams {
    const LayerDesc *table;  // device table, or nullptr to use `single`
    int32_t n_layers;
    int32_t nwaves;          // wavefronts taking part in the schedule
    uint64_t cost_total;
    float *part;             // [nwaves][2][M][64] partial sums
    int32_t *cnt;            // row-block counters, zero between launches
    int32_t M;
    int32_t pad_;
    LayerDesc single;
};

inline int tile_cost(int r) { return 4 * r + 2; }  // ~256-byte lines per tile: weights + meta/x

inline int64_t pad_rows(int64_t N) { return (N + kRowBlock - 1) / kRowBlock * kRowBlock; }

// launchers (mq_pack.hip / mq_linear.hip); each returns the hipError of the launch
hipError_t launch_slice(const uint8_t *parent, int64_t n, int c, int r, uint8_t *out, hipStream_t s);
hipError_t launch_pack(const uint8_t *S, int64_t N, int64_t K, int r, uint4 *packed, hipStream_t s);
hipError_t launch_unpack(const uint4 *packed, int64_t N, int64_t K, int r, uint8_t *S, hipStream_t s);
hipError_t launch_pack_meta(const _Float16 *sc, const _Float16 *zr, int64_t N, int64_t G, _Float16 *st,
                            _Float16 *zt, hipStream_t s);
hipError_t launch_fill_zero(void *p, size_t bytes, hipStream_t s);
// Fills p.nwaves and launches.  max_cost = largest tile cost in the stack.
hipError_t launch_stack(StackParams p, int max_cost, hipStream_t s);
// True if this build has a kernel for batch M.
bool linear_supports_m(int64_t M);

}  // namespace mq
