// C ABI of libmq: argument validation (host only, before anything is enqueued),
// workspace arithmetic and dispatch to the kernel launchers.
#include <climits>
#include <cmath>
#include <cstring>
#include <mutex>
#include <vector>

#include "mq_internal.h"

using namespace mq;

namespace {

bool valid_pack_r(int r) { return r == 2 || r == 3 || r == 4 || r == 6 || r == 8; }
bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

constexpr int64_t kMaxDim = (int64_t)1 << 24;  // rows / columns of one layer

// shape checks shared by pack / meta / linear
mq_status check_shape(int64_t N, int64_t K, int group) {
    if (N < 1 || K < 1 || N > kMaxDim || K > kMaxDim) return MQ_ERR_BAD_SHAPE;
    if (group != kGroup || K % group) return MQ_ERR_BAD_GROUP;
    return MQ_OK;
}

size_t counter_bytes(int64_t row_blocks) { return align_up((size_t)row_blocks * 4, kCounterBytesAlign); }
bool use_mfma(int64_t M) { return M > kValuMaxM; }
// A stack of packed layers at M = kValuMaxM runs on the matrix cores: measured on uniform stacks, four rows on the
// vector ALUs take longer than five on the matrix cores at every width (1.34 against 1.02 ms at r = 2, 12 Llama-3-70B
// blocks).  Single calls keep the vector-ALU kernels (their low-latency shape wins on one layer), and so do stacks
// computed from the parent.  The "path batch" stands in for M wherever sizes and kernels are chosen.
// A small stack (the few linears of a decoder block that share their input) keeps the vector-ALU kernels in their
// low-latency shape, as a single call does.
int64_t stack_path_m(int64_t M, bool from_parent, bool small) {
    return !from_parent && !small && M == kValuMaxM ? M + 1 : M;
}
bool small_stack(const mq_layer *layers, int n_layers, int64_t M) {
    if (M > kValuMaxM || n_layers > 16) return false;
    int64_t tiles = 0;
    for (int i = 0; i < n_layers; ++i) tiles += pad_rows(layers[i].N) / kRowBlock * (layers[i].K / kGroup);
    return tiles <= 12288;
}
// column blocks the schedule sees: 1 (vector ALUs), 16-column chunks (narrow MFMA), passes (wide MFMA)
int64_t chunks(int64_t M) {
    return use_wide(M) ? wide_passes(M) : use_mfma(M) ? (M + kChunkCols - 1) / kChunkCols : 1;
}
int64_t counters_of(int64_t M, int64_t N) { return chunks(M) * (pad_rows(N) / kRowBlock); }
int slot_floats(int64_t M) {
    return use_wide(M)   ? 4 * wide_chunks_per_pass(M) * 32 * 64
           : use_mfma(M) ? kNarrowRowBlocks * 64 * kChunkCols
                         : 64 * (int)M;
}
size_t max_workers(int64_t M) {
    return use_wide(M)   ? (size_t)wide_max_groups(wide_chunks_per_pass(M))
           : use_mfma(M) ? (size_t)kMaxGroupsNarrow
                         : (size_t)max_workers_valu(M);
}
size_t partial_bytes(int64_t M) { return max_workers(M) * 2 * (size_t)slot_floats(M) * sizeof(float); }
// MFMA paths: prepared activations of one layer (group sums and rescale factors live inside the blocks)
size_t xt_bytes(int64_t M, int64_t K, int) {
    if (use_wide(M)) return align_up((size_t)wide_chunks_padded(M) * (size_t)(K / kGroup) * kWideXtBlockBytes, 256);
    if (use_mfma(M)) return (size_t)(K / kGroup) * kNarrowXtBlockBytes;
    return align_up((size_t)M * (size_t)K * 2, 256);  // vector-ALU path: bf16 activations converted to fp16
}

mq_status layer_status(const mq_layer &l, int64_t M) {
    if (!l.packed_W || !l.scales_t || !l.x || !l.y) return MQ_ERR_NULL;  // zeros_t may be NULL: symmetric layer
    if (!valid_pack_r(l.r)) return MQ_ERR_BAD_R;
    if (M < 1 || M > MQ_MAX_M) return MQ_ERR_BAD_SHAPE;
    if (mq_status st = check_shape(l.N, l.K, l.group)) return st;
    if ((l.from_parent != 0 && l.from_parent != 1) || (l.flags & ~(MQ_X_BF16 | MQ_Y_BF16 | MQ_X_AFTER_EARLIER)))
        return MQ_ERR_UNSUPPORTED;
    // a chained layer reads x as the earlier layers leave it: there is no point before the launch at which bf16
    // activations could be converted for it
    if ((l.flags & MQ_X_AFTER_EARLIER) && (l.flags & MQ_X_BF16)) return MQ_ERR_UNSUPPORTED;
    if (l.from_parent && use_mfma(M)) return MQ_ERR_UNSUPPORTED;  // slicing in registers: vector-ALU kernels only
    // the matrix-core paths move scales / zeros 16 bytes at a time
    const size_t meta_align = use_mfma(M) ? 16 : 2;
    if (!aligned(l.packed_W, 16) || !aligned(l.x, 4) || !aligned(l.scales_t, meta_align) ||
        !aligned(l.zeros_t, meta_align) || !aligned(l.y, 2))
        return MQ_ERR_ALIGN;
    return MQ_OK;
}

// ---- the zero-offsets of a symmetric layer: kSymLines lines of 64 x 2^(c-1); tile u of such a layer reads line
// u & (kSymLines - 1) (LayerDesc::zmask), so that no kernel branches on whether a layer has zero-offsets.  Many lines
// rather than one: every wave of the chip reading one 128-byte line would queue on a single L2 channel.
// As with any __device__ array the name is a host-side stand-in; kernels get the address looked up per device.
constexpr int kSymLines = 1024;
struct SymZeros {
    uint16_t v[kSymLines * 64];
    constexpr SymZeros() : v() {
        for (int i = 0; i < kSymLines * 64; ++i) v[i] = 0x5800;  // fp16 128.0
    }
};
static_assert(kC == 8, "0x5800 is fp16 2^(c-1) for c = 8");
static __device__ __align__(256) SymZeros sym_zeros = SymZeros();
constexpr int kMaxDevices = 64;
std::mutex g_symbol_mutex;
const _Float16 *g_sym_zero_line[kMaxDevices] = {};

// nullptr when the address cannot be had
const _Float16 *sym_zero_line() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_symbol_mutex);
    if (!g_sym_zero_line[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(sym_zeros)) != hipSuccess) return nullptr;
        g_sym_zero_line[dev] = static_cast<const _Float16 *>(p);
    }
    return g_sym_zero_line[dev];
}

// xt: where the MFMA path keeps this layer's prepared activations (on the ALU path: the fp16 copy of bf16 activations)
// sym_line: sym_zero_line() of the current device; needed (non-null) when the layer is symmetric
// Mp: the path batch (== M except for stacks at M = kValuMaxM, see stack_path_m)
LayerDesc make_desc(const mq_layer &l, int64_t M, int64_t Mp, uint64_t cost_start, int cnt_off, int job_start, void *xt,
                    const _Float16 *sym_line) {
    LayerDesc d{};
    d.Wp = static_cast<const uint4 *>(l.packed_W);
    d.st = reinterpret_cast<const _Float16 *>(l.scales_t);
    d.zt = reinterpret_cast<const _Float16 *>(l.zeros_t);
    d.zmask = -1;
    if (!l.zeros_t) {
        d.zt = sym_line;
        d.zmask = kSymLines - 1;
    }
    d.x = reinterpret_cast<const _Float16 *>(l.x);
    d.y = reinterpret_cast<_Float16 *>(l.y);
    d.xt = static_cast<const uint4 *>(xt);
    d.x_bf16 = nullptr;
    if (!use_mfma(Mp) && (l.flags & MQ_X_BF16)) {  // the vector-ALU kernels read the fp16 copy that launch_xcvt makes at xt
        d.x_bf16 = l.x;
        d.x = static_cast<const _Float16 *>(xt);
    }
    d.N = (int32_t)l.N;
    d.K = (int32_t)l.K;
    d.G = (int32_t)(l.K / kGroup);
    d.RB = (int32_t)(pad_rows(l.N) / kRowBlock);
    d.r = l.r;
    d.cost = valu_tile_cost(l.r, (int)M);  // replaced below on the MFMA paths
    if (l.from_parent) {  // the tiles are those of the 8-bit parent; Eq. 1 to l.r bits happens in registers
        d.r = kC;
        d.rs = l.r;
        d.cost = valu_tile_cost(kC, (int)M);
    }
    if (use_mfma(Mp) && !use_wide(Mp)) {  // scheduled in super-tiles of kNarrowRowBlocks row blocks
        d.RB = (d.RB + kNarrowRowBlocks - 1) / kNarrowRowBlocks;
        d.cost = mfma_tile_cost(l.r);
    }
    if (use_wide(Mp)) {  // scheduled in super-tiles of four row blocks
        d.RB = (d.RB + 3) / 4;
        d.cost = wide_tile_cost(l.r, wide_chunks_per_pass(Mp));
    }
    d.flags = l.flags & (MQ_X_BF16 | MQ_Y_BF16);
    d.cnt_off = cnt_off;
    d.M = (int32_t)M;
    d.CB = (int32_t)chunks(Mp);
    d.job_start = job_start;
    d.cost_start = cost_start;
    return d;
}

// Plan workspace (device): [256 B unused][LayerDesc table][counters][partial sums][prepared activations per layer].
// What a launch needs to know about it lives on the HOST, in the caller's mq_plan: running a stack reads nothing
// back from the device and the library keeps no record of plans of its own.
struct PlanHeader {
    uint64_t magic;
    uint64_t check;  // fold of every other field: an mq_plan that was never filled, or was overwritten, is refused
    void *ws;        // the device workspace the plan was built in
    uint64_t cost_total;
    int32_t n_layers, M, max_cost, n_jobs;
    uint64_t table_off, cnt_off, part_off, total_bytes;
    int32_t from_parent, path_M;
    int32_t ll_blocks, ll_waves;  // low-latency launch shape of a small stack, or 0
    int32_t any_x_bf16;           // some layer takes bf16 activations (the vector-ALU launches convert them first)
    int32_t ll_ks_cap;            // low-latency launch shape: most K slices per row block
    int32_t ll_start[16];         // ... and each layer's first workgroup
    int32_t chain_total;          // chained small stack: row blocks of all layers (0: not chained) ...
    int32_t chain_off;            // ... index of its stage counters ...
    int32_t stage_rb[16];         // ... and the row blocks of each stage
};
// the caller's handle: the header, then (small stacks) the descriptors that travel with the kernel arguments
constexpr size_t kPlanTableOff = 256;
static_assert(sizeof(PlanHeader) <= kPlanTableOff && kPlanTableOff + sizeof(SmallTable) <= sizeof(mq_plan),
              "header and descriptors must fit the caller's handle");
constexpr uint64_t kPlanMagic = 0x4d51504c414e3038ull;  // "MQPLAN08"

// ---- scratch of mq_linear_noalloc: device memory that exists without anybody allocating it.
// The array's name is only a host-side stand-in; its device address is looked up once per device (each device
// holds its own copy at its own address) and only that pointer is ever handed to a kernel.
constexpr size_t kScratchBytes = MQ_NOALLOC_SCRATCH_BYTES;
constexpr size_t kNoallocMinWorkers = 256;  // fewer schedule shares (waves) than this would leave most of the chip idle
constexpr size_t kNoallocMinGroups = 32;    // the same for the narrow matrix-core path, whose shares are workgroups of 8 waves
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};

mq_status scratch_of_current_device(void **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return MQ_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return MQ_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return MQ_OK;
}

// fold of the header (check field as zero) and, for a small stack, of the descriptors behind it
uint64_t plan_check(const PlanHeader &h, const SmallTable *small) {
    PlanHeader t = h;
    t.check = 0;
    uint64_t w[sizeof(PlanHeader) / 8 + 1] = {};
    std::memcpy(w, &t, sizeof(t));
    uint64_t acc = 0x9e3779b97f4a7c15ull;
    for (uint64_t v : w) acc = (acc ^ v) * 0x100000001b3ull + (acc >> 29);
    if (small) {
        static_assert(sizeof(SmallTable) % 8 == 0, "descriptors are folded as 64-bit words");
        uint64_t d[sizeof(SmallTable) / 8];
        std::memcpy(d, small, sizeof(d));
        for (uint64_t v : d) acc = (acc ^ v) * 0x100000001b3ull + (acc >> 29);
    }
    return acc;
}

struct PlanLayout {
    size_t table_off, cnt_off, cnt_bytes, part_off, act_off, total;
};
PlanLayout plan_layout(const mq_layer *layers, int n_layers, int64_t M) {
    int64_t counters = 0;
    size_t act = 0;
    for (int i = 0; i < n_layers; ++i) {
        counters += counters_of(M, layers[i].N);
        act += xt_bytes(M, layers[i].K, layers[i].r);
    }
    PlanLayout p;
    p.table_off = 256;
    p.cnt_off = align_up(p.table_off + (size_t)n_layers * sizeof(LayerDesc), 256);
    p.cnt_bytes = counter_bytes(counters + (use_mfma(M) ? 0 : kChainCounters));  // a small stack may be chained
    p.part_off = p.cnt_off + p.cnt_bytes;
    p.act_off = p.part_off + partial_bytes(M);
    p.total = p.act_off + act;
    return p;
}

// One layer on its own workspace: [counters][partial sums][prepared activations]
// worker_cap: 0 = the workspace has mq_workspace_bytes; else it holds partial-sum slots for that many schedule
// shares only ([counters][worker_cap slots pairs][prepared activations], checked by the caller) and the launch keeps
// to them.  M <= kNarrowMaxM when capped.
mq_status run_single(const mq_layer &l, int64_t M, void *ws, size_t ws_bytes, mq_stream stream, int worker_cap = 0) {
    if (!ws) return MQ_ERR_NULL;
    if (mq_status st = layer_status(l, M)) return st;
    if (l.flags & MQ_X_AFTER_EARLIER) return MQ_ERR_UNSUPPORTED;  // a layer on its own has no earlier layers
    if (!aligned(ws, 256)) return MQ_ERR_ALIGN;
    const int r_ws = l.from_parent ? kC : l.r;
    if (!worker_cap && ws_bytes < mq_workspace_bytes(M, l.N, l.K, r_ws)) return MQ_ERR_BUF_TOO_SMALL;

    char *base = static_cast<char *>(ws);
    const size_t cnt_b = counter_bytes(counters_of(M, l.N));
    const size_t part_b = worker_cap ? (size_t)worker_cap * 2 * (size_t)slot_floats(M) * sizeof(float) : partial_bytes(M);
    char *act = base + cnt_b + part_b;
    StackParams p{};
    p.worker_cap = worker_cap;
    p.table = nullptr;
    p.n_layers = 1;
    const _Float16 *sym_line = nullptr;
    if (!l.zeros_t && !(sym_line = sym_zero_line())) return MQ_ERR_HIP;
    p.single = make_desc(l, M, M, 0, 0, 0, act, sym_line);
    p.cost_total = (uint64_t)p.single.CB * p.single.RB * p.single.G * p.single.cost;
    p.cnt = reinterpret_cast<int32_t *>(base);
    p.part = reinterpret_cast<float *>(base + cnt_b);
    p.M = (int32_t)M;
    p.slot_floats = slot_floats(M);
    p.n_jobs = (use_wide(M) ? wide_chunks_padded(M) : p.single.CB) * p.single.G;
    hipError_t e;
    if (!use_mfma(M) && (l.flags & MQ_X_BF16)) {
        if (launch_xcvt(p, (hipStream_t)stream) != hipSuccess) return MQ_ERR_HIP;
    }
    if (use_wide(M))
        e = launch_stack_wide(p, p.single.cost, (hipStream_t)stream);
    else if (use_mfma(M))
        e = launch_stack_mfma(p, p.single.cost, (hipStream_t)stream);
    else if (linear_rb_fits(p.single, part_b))
        e = launch_linear_rb(p.single, p.part, p.cnt, (hipStream_t)stream);
    else
        e = launch_stack(p, p.single.cost, l.from_parent != 0, (hipStream_t)stream);
    return e == hipSuccess ? MQ_OK : MQ_ERR_HIP;
}

}  // namespace

extern "C" {

const char *mq_status_str(int status) {
    switch (status) {
        case MQ_OK: return "ok";
        case MQ_ERR_NULL: return "null pointer";
        case MQ_ERR_BAD_R: return "unsupported bit-width";
        case MQ_ERR_BAD_SHAPE: return "bad shape";
        case MQ_ERR_BAD_GROUP: return "bad group size";
        case MQ_ERR_ALIGN: return "misaligned pointer";
        case MQ_ERR_BUF_TOO_SMALL: return "buffer too small";
        case MQ_ERR_HIP: return "HIP runtime error";
        case MQ_ERR_UNSUPPORTED: return "unsupported configuration";
    }
    return "unknown status";
}

int mq_version(void) { return 2; }

size_t mq_packed_bytes(int64_t N, int64_t K, int r) {
    if (!valid_pack_r(r) || check_shape(N, K, kGroup) != MQ_OK) return 0;
    return (size_t)pad_rows(N) * (size_t)K * (size_t)r / 8;
}

size_t mq_meta_bytes(int64_t N, int64_t K, int group) {
    if (check_shape(N, K, group) != MQ_OK) return 0;
    return (size_t)pad_rows(N) * (size_t)(K / group) * 2;
}

size_t mq_workspace_bytes(int64_t M, int64_t N, int64_t K, int r) {
    if (!valid_pack_r(r) || check_shape(N, K, kGroup) != MQ_OK || M < 1 || M > MQ_MAX_M) return 0;
    return counter_bytes(counters_of(M, N)) + partial_bytes(M) + xt_bytes(M, K, r);
}

mq_status mq_workspace_init(void *ws, size_t ws_bytes, mq_stream stream) {
    if (!ws) return MQ_ERR_NULL;
    if (!aligned(ws, 256)) return MQ_ERR_ALIGN;
    if (ws_bytes < kCounterBytesAlign) return MQ_ERR_BUF_TOO_SMALL;
    // counters sit at the start; the partial-sum slots need no initial value
    size_t zero = ws_bytes;
    const size_t cap = counter_bytes(kMaxDim / kRowBlock);
    if (zero > cap) zero = cap;
    return launch_fill_zero(ws, zero / 4 * 4, (hipStream_t)stream) == hipSuccess ? MQ_OK : MQ_ERR_HIP;
}

mq_status mq_slice_codes(const uint8_t *parent, int64_t n, int c, int r, uint8_t *S_out, mq_stream stream) {
    if (c < 1 || c > 8 || r < 1 || r > c) return MQ_ERR_BAD_R;
    if (n < 0) return MQ_ERR_BAD_SHAPE;
    if (n == 0) return MQ_OK;  // nothing to do; pointers of an empty array may be NULL
    if (!parent || !S_out) return MQ_ERR_NULL;
    if (S_out != parent && S_out < parent + n && parent < S_out + n) return MQ_ERR_UNSUPPORTED;  // partial overlap
    return launch_slice(parent, n, c, r, S_out, (hipStream_t)stream) == hipSuccess ? MQ_OK : MQ_ERR_HIP;
}

mq_status mq_pack(const uint8_t *S, int64_t N, int64_t K, int c, int r, void *packed, size_t packed_bytes,
                  mq_stream stream) {
    if (!S || !packed) return MQ_ERR_NULL;
    if (c != kC || !valid_pack_r(r)) return MQ_ERR_BAD_R;
    if (mq_status st = check_shape(N, K, kGroup)) return st;
    if (!aligned(packed, 16)) return MQ_ERR_ALIGN;
    if (packed_bytes < mq_packed_bytes(N, K, r)) return MQ_ERR_BUF_TOO_SMALL;
    return launch_pack(S, N, K, r, static_cast<uint4 *>(packed), (hipStream_t)stream) == hipSuccess ? MQ_OK
                                                                                                     : MQ_ERR_HIP;
}

mq_status mq_unpack(const void *packed, int64_t N, int64_t K, int c, int r, uint8_t *S_out, mq_stream stream) {
    if (!packed || !S_out) return MQ_ERR_NULL;
    if (c != kC || !valid_pack_r(r)) return MQ_ERR_BAD_R;
    if (mq_status st = check_shape(N, K, kGroup)) return st;
    if (!aligned(packed, 16)) return MQ_ERR_ALIGN;
    return launch_unpack(static_cast<const uint4 *>(packed), N, K, r, S_out, (hipStream_t)stream) == hipSuccess
               ? MQ_OK
               : MQ_ERR_HIP;
}

mq_status mq_pack_meta(const mq_half *scales, const mq_half *zeros, int64_t N, int64_t K, int group,
                       mq_half *scales_t, mq_half *zeros_t, size_t meta_bytes, mq_stream stream) {
    if (!scales || !scales_t) return MQ_ERR_NULL;
    if ((zeros == nullptr) != (zeros_t == nullptr)) return MQ_ERR_NULL;  // both (asymmetric) or neither (symmetric)
    if (mq_status st = check_shape(N, K, group)) return st;
    if (!aligned(scales, 2) || !aligned(zeros, 2) || !aligned(scales_t, 2) || !aligned(zeros_t, 2))
        return MQ_ERR_ALIGN;
    if (meta_bytes < mq_meta_bytes(N, K, group)) return MQ_ERR_BUF_TOO_SMALL;
    return launch_pack_meta(reinterpret_cast<const _Float16 *>(scales), reinterpret_cast<const _Float16 *>(zeros), N,
                            K / group, reinterpret_cast<_Float16 *>(scales_t), reinterpret_cast<_Float16 *>(zeros_t),
                            (hipStream_t)stream) == hipSuccess
               ? MQ_OK
               : MQ_ERR_HIP;
}

mq_status mq_linear(const mq_half *x, int64_t M, const void *packed_W, const mq_half *scales_t,
                    const mq_half *zeros_t, int64_t N, int64_t K, int r, int group, mq_half *y, void *ws,
                    size_t ws_bytes, mq_stream stream) {
    const mq_layer l{packed_W, scales_t, zeros_t, x, y, N, K, r, group, 0, 0};
    return run_single(l, M, ws, ws_bytes, stream);
}

mq_status mq_linear_bf16(const mq_bf16 *x, int64_t M, const void *packed_W, const mq_half *scales_t, const mq_half *zeros_t,
                         int64_t N, int64_t K, int r, int group, mq_bf16 *y, void *ws, size_t ws_bytes, mq_stream stream) {
    const mq_layer l{packed_W, scales_t, zeros_t, x, y, N, K, r, group, 0, MQ_X_BF16 | MQ_Y_BF16};
    return run_single(l, M, ws, ws_bytes, stream);
}

mq_status mq_linear_from_parent(const mq_half *x, int64_t M, const void *packed_parent, const mq_half *scales_t,
                                const mq_half *zeros_t, int64_t N, int64_t K, int r, int group, mq_half *y, void *ws,
                                size_t ws_bytes, mq_stream stream) {
    const mq_layer l{packed_parent, scales_t, zeros_t, x, y, N, K, r, group, 1, 0};
    return run_single(l, M, ws, ws_bytes, stream);
}

mq_status mq_slice_pack(const uint8_t *parent, int64_t N, int64_t K, int c, int r, void *packed, size_t packed_bytes,
                        mq_stream stream) {
    if (!parent || !packed) return MQ_ERR_NULL;
    if (c != kC || !valid_pack_r(r)) return MQ_ERR_BAD_R;
    if (mq_status st = check_shape(N, K, kGroup)) return st;
    if (!aligned(packed, 16)) return MQ_ERR_ALIGN;
    if (packed_bytes < mq_packed_bytes(N, K, r)) return MQ_ERR_BUF_TOO_SMALL;
    return launch_slice_pack(parent, N, K, r, static_cast<uint4 *>(packed), (hipStream_t)stream) == hipSuccess
               ? MQ_OK
               : MQ_ERR_HIP;
}

mq_status mq_reslice(const void *packed_parent, int64_t N, int64_t K, int c, int r, void *packed, size_t packed_bytes,
                     mq_stream stream) {
    if (!packed_parent || !packed) return MQ_ERR_NULL;
    if (c != kC || !valid_pack_r(r)) return MQ_ERR_BAD_R;
    if (mq_status st = check_shape(N, K, kGroup)) return st;
    if (!aligned(packed_parent, 16) || !aligned(packed, 16)) return MQ_ERR_ALIGN;
    if (packed_bytes < mq_packed_bytes(N, K, r)) return MQ_ERR_BUF_TOO_SMALL;
    {  // every thread reads its whole tile before it writes, but tiles run in any order: no overlap at all
        const char *a = static_cast<const char *>(packed_parent), *b = static_cast<const char *>(packed);
        if (a < b + mq_packed_bytes(N, K, r) && b < a + mq_packed_bytes(N, K, kC)) return MQ_ERR_UNSUPPORTED;
    }
    return launch_reslice(static_cast<const uint4 *>(packed_parent), N, K, r, static_cast<uint4 *>(packed),
                          (hipStream_t)stream) == hipSuccess
               ? MQ_OK
               : MQ_ERR_HIP;
}

mq_status mq_reslice_many(const mq_reslice_job *jobs, int n_jobs, int c, mq_stream stream) {
    if (!jobs) return MQ_ERR_NULL;
    if (n_jobs < 1 || n_jobs > (1 << 20)) return MQ_ERR_BAD_SHAPE;
    if (c != kC) return MQ_ERR_BAD_R;
    std::vector<const uint4 *> src((size_t)n_jobs);
    std::vector<uint4 *> dst((size_t)n_jobs);
    std::vector<int64_t> N((size_t)n_jobs), K((size_t)n_jobs);
    std::vector<int> r((size_t)n_jobs);
    for (int i = 0; i < n_jobs; ++i) {
        const mq_reslice_job &j = jobs[i];
        if (!j.packed_parent || !j.packed) return MQ_ERR_NULL;
        if (!valid_pack_r(j.r) || j.reserved != 0) return MQ_ERR_BAD_R;
        if (mq_status st = check_shape(j.N, j.K, kGroup)) return st;
        if (!aligned(j.packed_parent, 16) || !aligned(j.packed, 16)) return MQ_ERR_ALIGN;
        if (j.packed_bytes < mq_packed_bytes(j.N, j.K, j.r)) return MQ_ERR_BUF_TOO_SMALL;
        const char *a = static_cast<const char *>(j.packed_parent), *b = static_cast<const char *>(j.packed);
        if (a < b + mq_packed_bytes(j.N, j.K, j.r) && b < a + mq_packed_bytes(j.N, j.K, kC)) return MQ_ERR_UNSUPPORTED;
        src[i] = static_cast<const uint4 *>(j.packed_parent);
        dst[i] = static_cast<uint4 *>(j.packed);
        N[i] = j.N;
        K[i] = j.K;
        r[i] = j.r;
    }
    return launch_reslice_many(src.data(), dst.data(), N.data(), K.data(), r.data(), n_jobs, (hipStream_t)stream) ==
                   hipSuccess
               ? MQ_OK
               : MQ_ERR_HIP;
}

mq_status mq_quant_matgptq(const float *W, int64_t ldw, int64_t N, int64_t ncols, int64_t col0, const mq_half *scales,
                           const mq_half *zeros, int64_t K, int group, int c, const float *lambda, uint8_t *Q,
                           int64_t ldq, mq_stream stream) {
    if (!W || !scales || !zeros || !lambda || !Q) return MQ_ERR_NULL;
    if (c != kC) return MQ_ERR_BAD_R;
    bool any = false;
    for (int i = 0; i < kC; ++i) {
        if (!std::isfinite(lambda[i]) || lambda[i] < 0.f) return MQ_ERR_BAD_R;
        any = any || lambda[i] > 0.f;
    }
    if (!any) return MQ_ERR_BAD_R;  // no target width
    if (mq_status st = check_shape(N, K, group)) return st;
    if (ncols < 1 || col0 < 0 || col0 > K - ncols || ldw < ncols || ldq < ncols || ldw > ((int64_t)1 << 32) ||
        ldq > ((int64_t)1 << 32))
        return MQ_ERR_BAD_SHAPE;
    if (!aligned(W, 4) || !aligned(scales, 2) || !aligned(zeros, 2)) return MQ_ERR_ALIGN;
    const bool vec4 = aligned(W, 16) && aligned(Q, 4) && ldw % 4 == 0 && ldq % 4 == 0 && ncols % 4 == 0 && col0 % 4 == 0;
    return launch_quant(W, ldw, N, ncols, col0, reinterpret_cast<const _Float16 *>(scales),
                        reinterpret_cast<const _Float16 *>(zeros), K / group, lambda, Q, ldq, vec4,
                        (hipStream_t)stream) == hipSuccess
               ? MQ_OK
               : MQ_ERR_HIP;
}

size_t mq_matgptq_workspace_bytes(int64_t N, int block) {
    if (N < 1 || N > kMaxDim || (block != 16 && block != 32 && block != 64 && block != 128)) return 0;
    return align_up((size_t)N * (size_t)block * sizeof(float), 256);
}

mq_status mq_matgptq_quantize(float *W, int64_t ldw, int64_t N, int64_t K, const float *U, int64_t ldu,
                              const mq_half *scales, const mq_half *zeros, int group, int c, const float *lambda,
                              int block, uint8_t *Q, int64_t ldq, void *ws, size_t ws_bytes, mq_stream stream) {
    if (!W || !U || !scales || !zeros || !lambda || !Q || !ws) return MQ_ERR_NULL;
    if (c != kC) return MQ_ERR_BAD_R;
    bool any = false;
    for (int i = 0; i < kC; ++i) {
        if (!std::isfinite(lambda[i]) || lambda[i] < 0.f) return MQ_ERR_BAD_R;
        any = any || lambda[i] > 0.f;
    }
    if (!any) return MQ_ERR_BAD_R;
    if (mq_status st = check_shape(N, K, group)) return st;
    if (block != 16 && block != 32 && block != 64 && block != 128) return MQ_ERR_BAD_SHAPE;
    if (ldw < K || ldu < K || ldq < K || ldw > ((int64_t)1 << 32) || ldu > ((int64_t)1 << 32) || ldq > ((int64_t)1 << 32))
        return MQ_ERR_BAD_SHAPE;
    if (!aligned(W, 4) || !aligned(U, 4) || !aligned(scales, 2) || !aligned(zeros, 2) || !aligned(ws, 4))
        return MQ_ERR_ALIGN;
    if (ws_bytes < mq_matgptq_workspace_bytes(N, block)) return MQ_ERR_BUF_TOO_SMALL;
    return launch_gptq(W, ldw, N, K, U, ldu, reinterpret_cast<const _Float16 *>(scales),
                       reinterpret_cast<const _Float16 *>(zeros), lambda, block, Q, ldq, static_cast<float *>(ws),
                       (hipStream_t)stream) == hipSuccess
               ? MQ_OK
               : MQ_ERR_HIP;
}

size_t mq_stack_workspace_bytes(const mq_layer *layers, int n_layers, int64_t M) {
    if (!layers || n_layers < 1 || n_layers > (1 << 20) || M < 1 || M > MQ_MAX_M) return 0;
    for (int i = 0; i < n_layers; ++i)
        if (!valid_pack_r(layers[i].r) || check_shape(layers[i].N, layers[i].K, layers[i].group) != MQ_OK) return 0;
    return plan_layout(layers, n_layers, stack_path_m(M, layers[0].from_parent != 0, small_stack(layers, n_layers, M))).total;
}

mq_status mq_stack_plan(const mq_layer *layers, int n_layers, int64_t M, void *plan_ws, size_t plan_bytes,
                        mq_plan *plan, mq_stream stream) {
    if (!layers || !plan_ws || !plan) return MQ_ERR_NULL;
    if (n_layers < 1 || n_layers > (1 << 20)) return MQ_ERR_BAD_SHAPE;
    if (M < 1 || M > MQ_MAX_M) return MQ_ERR_BAD_SHAPE;
    const int64_t Mp = stack_path_m(M, layers[0].from_parent != 0, small_stack(layers, n_layers, M));
    for (int i = 0; i < n_layers; ++i) {
        if (mq_status st = layer_status(layers[i], Mp)) return st;
        if (layers[i].from_parent != layers[0].from_parent) return MQ_ERR_UNSUPPORTED;  // one kernel variant per launch
    }
    bool chained = false;
    for (int i = 0; i < n_layers; ++i) chained |= (layers[i].flags & MQ_X_AFTER_EARLIER) != 0;
    // only the launch that keeps every workgroup of the stack resident can let one layer wait for another
    if (chained && ((layers[0].flags & MQ_X_AFTER_EARLIER) || !small_stack(layers, n_layers, M))) return MQ_ERR_UNSUPPORTED;
    // Switched off at M = 4: the one run of a chained stack at that batch ended in a memory fault whose cause has not
    // been established (M = 1 and 3 were clean in the same run).
    if (chained && M > kChainMaxM) return MQ_ERR_UNSUPPORTED;
    if (!aligned(plan_ws, 256)) return MQ_ERR_ALIGN;
    const size_t need = mq_stack_workspace_bytes(layers, n_layers, M);
    if (need == 0) return MQ_ERR_BAD_SHAPE;
    if (plan_bytes < need) return MQ_ERR_BUF_TOO_SMALL;

    const PlanLayout pl = plan_layout(layers, n_layers, Mp);
    char *base_dev = static_cast<char *>(plan_ws);
    int64_t counters = 0, jobs = 0;
    uint64_t cost = 0;
    int max_cost = 0;
    size_t act = pl.act_off;
    std::vector<LayerDesc> table((size_t)n_layers);
    const _Float16 *sym_line = nullptr;
    for (int i = 0; i < n_layers; ++i) {
        const size_t xb = xt_bytes(Mp, layers[i].K, layers[i].r);
        if (!layers[i].zeros_t && !sym_line && !(sym_line = sym_zero_line())) return MQ_ERR_HIP;
        table[i] = make_desc(layers[i], M, Mp, cost, (int)counters, (int)jobs, xb ? base_dev + act : nullptr, sym_line);
        act += xb;
        cost += (uint64_t)table[i].CB * table[i].RB * table[i].G * table[i].cost;
        counters += counters_of(Mp, layers[i].N);
        jobs += (int64_t)(use_wide(Mp) ? wide_chunks_padded(Mp) : table[i].CB) * table[i].G;
        if (table[i].cost > max_cost) max_cost = table[i].cost;
    }
    if (counters > INT32_MAX || jobs > INT32_MAX) return MQ_ERR_BAD_SHAPE;
    PlanHeader h{};
    h.magic = kPlanMagic;
    h.ws = plan_ws;
    h.cost_total = cost;
    h.n_layers = n_layers;
    h.M = (int32_t)M;
    h.max_cost = max_cost;
    h.n_jobs = (int32_t)jobs;
    for (int i = 0; i < n_layers; ++i) h.any_x_bf16 |= layers[i].flags & MQ_X_BF16;
    h.table_off = pl.table_off;
    h.cnt_off = pl.cnt_off;
    h.part_off = pl.part_off;
    h.total_bytes = pl.total;
    h.from_parent = layers[0].from_parent;
    h.path_M = (int32_t)Mp;
    {
        int nb = 0, nw = 0, kc = 0;
        bool all_resident = false;
        if (!use_mfma(Mp) && linear_rb_stack_shape(table.data(), n_layers, partial_bytes(Mp), layers[0].from_parent != 0,
                                                   chained, &nb, &nw, &kc, h.ll_start, &all_resident)) {
            h.ll_blocks = nb;
            h.ll_waves = nw;
            h.ll_ks_cap = kc;
        }
        if (chained) {
            // stages: a new one at every layer that waits; the counters sit behind the row-block counters
            if (!h.ll_blocks) return MQ_ERR_UNSUPPORTED;
            if (!all_resident) return MQ_ERR_HIP;  // no device to ask, or it cannot hold the stack's workgroups at one time
            int stage = 0;
            for (int i = 0; i < n_layers; ++i) {
                if (layers[i].flags & MQ_X_AFTER_EARLIER) ++stage;
                table[i].chain = stage | ((layers[i].flags & MQ_X_AFTER_EARLIER) ? kChainWaits : 0);
                h.stage_rb[stage] += table[i].RB;
                h.chain_total += table[i].RB;
            }
            h.chain_off = (int32_t)counters;
        }
    }
    SmallTable small{};
    if (h.ll_blocks)
        for (int i = 0; i < n_layers; ++i) small.d[i] = table[i];
    h.check = plan_check(h, h.ll_blocks ? &small : nullptr);

    // The descriptor table travels to the device inside kernel arguments (copied when the launch is enqueued), so the
    // host arrays may go away as soon as this returns and nothing is waited for.
    hipStream_t s = (hipStream_t)stream;
    if (launch_write_table(table.data(), n_layers, reinterpret_cast<LayerDesc *>(base_dev + pl.table_off), s) != hipSuccess)
        return MQ_ERR_HIP;
    if (launch_fill_zero(base_dev + pl.cnt_off, pl.cnt_bytes, s) != hipSuccess) return MQ_ERR_HIP;
    std::memset(plan, 0, sizeof(*plan));
    std::memcpy(plan, &h, sizeof(h));
    if (h.ll_blocks) std::memcpy(reinterpret_cast<char *>(plan) + kPlanTableOff, &small, sizeof(small));
    return MQ_OK;
}

mq_status mq_linear_stack(const mq_plan *plan, mq_stream stream) {
    if (!plan) return MQ_ERR_NULL;
    PlanHeader h{};
    std::memcpy(&h, plan, sizeof(h));
    if (h.magic != kPlanMagic || !h.ws) return MQ_ERR_BAD_SHAPE;  // not a filled plan
    SmallTable small{};
    if (h.ll_blocks) std::memcpy(&small, reinterpret_cast<const char *>(plan) + kPlanTableOff, sizeof(small));
    if (h.check != plan_check(h, h.ll_blocks ? &small : nullptr)) return MQ_ERR_BAD_SHAPE;
    char *base = static_cast<char *>(h.ws);
    StackParams p{};
    p.table = reinterpret_cast<const LayerDesc *>(base + h.table_off);
    p.n_layers = h.n_layers;
    p.cost_total = h.cost_total;
    p.cnt = reinterpret_cast<int32_t *>(base + h.cnt_off);
    p.part = reinterpret_cast<float *>(base + h.part_off);
    p.M = h.M;
    p.slot_floats = slot_floats(h.path_M);
    p.n_jobs = h.n_jobs;
    p.ks_cap = h.ll_ks_cap;
    std::memcpy(p.ll_start, h.ll_start, sizeof(p.ll_start));
    p.chain_total = h.chain_total;
    p.chain_off = h.chain_off;
    std::memcpy(p.stage_rb, h.stage_rb, sizeof(p.stage_rb));
    if (!use_mfma(h.path_M) && h.any_x_bf16) {
        if (launch_xcvt(p, (hipStream_t)stream) != hipSuccess) return MQ_ERR_HIP;
    }
    const hipError_t e = use_wide(h.path_M)   ? launch_stack_wide(p, h.max_cost, (hipStream_t)stream)
                         : use_mfma(h.path_M) ? launch_stack_mfma(p, h.max_cost, (hipStream_t)stream)
                         : h.ll_blocks        ? launch_linear_rb_stack(p, small, h.ll_blocks, h.ll_waves, h.from_parent != 0,
                                                                       (hipStream_t)stream)
                                              : launch_stack(p, h.max_cost, h.from_parent != 0, (hipStream_t)stream);
    return e == hipSuccess ? MQ_OK : MQ_ERR_HIP;
}

mq_status mq_linear_noalloc(const mq_half *x, int64_t M, const void *packed_W, const mq_half *scales_t,
                            const mq_half *zeros_t, int64_t N, int64_t K, int r, int group, mq_half *y, mq_stream stream) {
    const mq_layer l{packed_W, scales_t, zeros_t, x, y, N, K, r, group, 0, 0};
    if (mq_status st = layer_status(l, M)) return st;
    if (M > kNarrowMaxM) return MQ_ERR_UNSUPPORTED;  // the wide path's slots alone exceed the scratch array
    // [counters][slot pairs for `cap` schedule shares][prepared activations] must fit the array
    const size_t cnt_b = counter_bytes(counters_of(M, N));
    const size_t act_b = xt_bytes(M, K, r);
    const size_t pair_b = 2 * (size_t)slot_floats(M) * sizeof(float);
    const size_t min_workers = use_mfma(M) ? kNoallocMinGroups : kNoallocMinWorkers;
    if (cnt_b + act_b + min_workers * pair_b > kScratchBytes) return MQ_ERR_BUF_TOO_SMALL;
    size_t cap = (kScratchBytes - cnt_b - act_b) / pair_b;
    const size_t most = max_workers(M);
    if (cap > most) cap = most;
    void *ws = nullptr;
    if (mq_status st = scratch_of_current_device(&ws)) return st;
    // the array keeps the last call's contents, laid out for that call's shape: this call's counters start at zero
    if (launch_fill_zero(ws, cnt_b, (hipStream_t)stream) != hipSuccess) return MQ_ERR_HIP;
    return run_single(l, M, ws, kScratchBytes, stream, (int)cap);
}

mq_status mq_read_probe(const void *buf, size_t bytes, uint32_t *out, mq_stream stream) {
    if (!buf || !out) return MQ_ERR_NULL;
    if (bytes == 0 || bytes % 16) return MQ_ERR_BAD_SHAPE;
    if (!aligned(buf, 16) || !aligned(out, 4)) return MQ_ERR_ALIGN;
    return launch_read_probe(buf, bytes, out, (hipStream_t)stream) == hipSuccess ? MQ_OK : MQ_ERR_HIP;
}

size_t mq_linear_plain_workspace_bytes(int64_t M, int64_t N, int64_t K, int r) {
    const size_t ws = mq_workspace_bytes(M, N, K, r), meta = mq_meta_bytes(N, K, kGroup);
    if (ws == 0 || meta == 0) return 0;
    return align_up(ws, 256) + 2 * align_up(meta, 256);
}

mq_status mq_linear_plain(const mq_half *x, int64_t M, const void *packed_W, const mq_half *scales, const mq_half *zeros,
                          int64_t N, int64_t K, int r, int group, mq_half *y, void *ws, size_t ws_bytes,
                          mq_stream stream) {
    if (!scales || !ws) return MQ_ERR_NULL;  // zeros may be NULL: symmetric layer
    if (!valid_pack_r(r)) return MQ_ERR_BAD_R;
    if (M < 1 || M > MQ_MAX_M) return MQ_ERR_BAD_SHAPE;
    if (mq_status st = check_shape(N, K, group)) return st;
    if (!aligned(ws, 256) || !aligned(scales, 2) || !aligned(zeros, 2)) return MQ_ERR_ALIGN;
    if (ws_bytes < mq_linear_plain_workspace_bytes(M, N, K, r)) return MQ_ERR_BUF_TOO_SMALL;
    const size_t inner = align_up(mq_workspace_bytes(M, N, K, r), 256), meta = align_up(mq_meta_bytes(N, K, group), 256);
    char *base = static_cast<char *>(ws);
    mq_half *st = reinterpret_cast<mq_half *>(base + inner);
    mq_half *zt = zeros ? reinterpret_cast<mq_half *>(base + inner + meta) : nullptr;
    // validate the linear call before anything is enqueued (a failing call enqueues nothing)
    const mq_layer l{packed_W, st, zt, x, y, N, K, r, group, 0, 0};
    if (mq_status s = layer_status(l, M)) return s;
    if (mq_status s = mq_pack_meta(scales, zeros, N, K, group, st, zt, mq_meta_bytes(N, K, group), stream)) return s;
    return run_single(l, M, ws, inner, stream);
}

}  // extern "C"
