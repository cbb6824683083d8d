/*
 * libmq -- Matryoshka-sliced, group-dequantised linear layers on AMD MI355X (gfx950).
 *
 * The library executes the inference path of MatGPTQ (arXiv 2602.03537):
 * a c = 8 bit "parent" integer checkpoint is sliced to r in {2,3,4,6,8} bits
 * (Eq. 1, Section 2), packed so that an r-bit layer streams r bits per weight,
 * and multiplied on the fly  y = x * W_D^T  with per-group scale / zero-offset
 * (Section 3.2 item 1; Section 4), each layer with its own r (Section 3.3).
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers owned by the caller unless the
 *     argument is marked "host".  The library never allocates or frees device
 *     memory, never copies between host and device, never synchronises and
 *     keeps no state of its own between calls (mq_linear_noalloc's static
 *     scratch array aside): every call enqueues kernels on
 *     `stream` (a hipStream_t passed as void*, NULL = the default stream) and
 *     returns.  Host arrays (layer tables, job lists, lambda) are consumed
 *     before the call returns.  Every call may be recorded into a HIP graph.
 *   - Arguments are validated on the host BEFORE anything is enqueued; a call
 *     that returns anything but MQ_OK because of its arguments has enqueued
 *     nothing.  No exceptions, no abort.  A launch the HIP runtime refuses maps
 *     to MQ_ERR_HIP (for the calls that enqueue several launches, the earlier
 *     ones stay enqueued).  The runtime's sticky "last error" is neither read
 *     nor cleared: an error the caller's own earlier work left pending is still
 *     there for the caller afterwards.
 *   - Launch shapes follow the device the calling thread has current (compute
 *     units, occupancy), queried once per process; sizes returned by the
 *     *_bytes functions do not depend on the device.
 *   - Matrices are row-major.  W is [N, K] (torch.nn.Linear convention:
 *     N output features, K input features), x is [M, K], y is [M, N].
 *   - fp16 values are IEEE binary16 (uint16_t storage on the C side).
 *   - c is fixed to 8 for packing and the linear kernels; mq_slice_codes
 *     accepts any 1 <= r <= c <= 8.
 *   - group must be 128 and must divide K.
 *   - Symmetric quantisation (the paper's own runs, appendix "Additional
 *     Hyperparameter Details": the zero-offset of every group is 2^(c-1) = 128):
 *     wherever a call takes the tiled zero-offsets `zeros_t` (or `zeros`), NULL
 *     means exactly that.  No zero-offset is read then, which takes 0.125 bit per
 *     weight off the stream; results are those of an array filled with 128,
 *     bit for bit.
 */
#ifndef MQ_H
#define MQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MQ_OK = 0,
    MQ_ERR_NULL = 1,          /* a required pointer is NULL */
    MQ_ERR_BAD_R = 2,         /* bit-width not supported by this entry point */
    MQ_ERR_BAD_SHAPE = 3,     /* M, N, K or a count is out of range */
    MQ_ERR_BAD_GROUP = 4,     /* group != 128 or group does not divide K */
    MQ_ERR_ALIGN = 5,         /* a pointer is not aligned as documented */
    MQ_ERR_BUF_TOO_SMALL = 6, /* packed / meta / workspace buffer too small */
    MQ_ERR_HIP = 7,           /* the HIP runtime refused a launch or a copy */
    MQ_ERR_UNSUPPORTED = 8    /* valid request this build has no kernel for */
} mq_status;

typedef void *mq_stream; /* hipStream_t */
typedef uint16_t mq_half; /* IEEE binary16 bits */
typedef uint16_t mq_bf16; /* bfloat16 bits (the upper half of an IEEE binary32) */

/* Rows of W are processed in blocks of MQ_ROW_BLOCK; packed buffers pad N up. */
#define MQ_ROW_BLOCK 64
#define MQ_GROUP 128
#define MQ_MAX_M 256
/* Bytes of device memory mq_linear_noalloc works in: a static array inside the library's code
 * object, held by every GPU the library runs on until the process ends. */
#define MQ_NOALLOC_SCRATCH_BYTES (8u << 20)

const char *mq_status_str(int status);
int mq_version(void);

/* ---------------------------------------------------------------- sizes
 * Pure host arithmetic, callable without a GPU.  All return 0 on invalid
 * arguments.  With Npad = N rounded up to MQ_ROW_BLOCK:
 *   mq_packed_bytes    = Npad * K * r / 8            (exactly r bits per weight)
 *   mq_meta_bytes      = Npad * (K/group) * 2        (bytes of EACH of the two
 *                                                     tiled arrays scales_t, zeros_t)
 *   mq_workspace_bytes = bytes mq_linear needs in `ws` for this problem.
 */
size_t mq_packed_bytes(int64_t N, int64_t K, int r);
size_t mq_meta_bytes(int64_t N, int64_t K, int group);
size_t mq_workspace_bytes(int64_t M, int64_t N, int64_t K, int r);

/* Zero the synchronisation counters at the start of a workspace.  Must be
 * enqueued once on a fresh workspace before its first use by mq_linear; the
 * kernels leave the counters zero when they finish, so it is not needed again.
 * A workspace must not be shared by calls that may run concurrently.
 * ws: device, 256-byte aligned. */
mq_status mq_workspace_init(void *ws, size_t ws_bytes, mq_stream stream);

/* ---------------------------------------------------------------- measurement aid
 * What a plain streaming read achieves on this device: every wavefront reads a contiguous share of
 * `buf` with non-temporal 16-byte loads (the access pattern of the linear kernels' weight stream,
 * with no arithmetic behind it) and the xor of all 32-bit words read is xor-ed into *out.  Timed by
 * the caller on a buffer well beyond the last-level cache, it gives the read bandwidth the kernels
 * are measured against, next to the published HBM peak.
 *   buf : device, 16-byte aligned, bytes > 0 and a multiple of 16;   out : device, one uint32
 * Errors: NULL, BAD_SHAPE, ALIGN, HIP. */
mq_status mq_read_probe(const void *buf, size_t bytes, uint32_t *out, mq_stream stream);

/* ---------------------------------------------------------------- slicing
 * Eq. 1 (Section 2): S = clamp(round(q / 2^(c-r)), 0, 2^r - 1) * 2^(c-r),
 * rounding half up (Section 3.1 "Slicing": the next lower bit alone decides),
 * r == c is the identity.  Elementwise over n codes.
 *   parent : device, n bytes, c-bit codes (values >= 2^c are masked to c bits)
 *   S_out  : device, n bytes, c-bit codes on the 2^(c-r) grid; either S_out == parent
 *            (in place) or the two do not overlap
 * Errors: BAD_R (r or c out of 1 <= r <= c <= 8), BAD_SHAPE (n < 0), NULL,
 * UNSUPPORTED (partial overlap).
 * n == 0 is a no-op that returns MQ_OK even for NULL pointers. */
mq_status mq_slice_codes(const uint8_t *parent, int64_t n, int c, int r, uint8_t *S_out,
                         mq_stream stream);

/* ---------------------------------------------------------------- packing
 * Section 4 ("offline pre-processing"): reorder and pack sliced codes for the
 * kernels.  The layout is this library's own (not the paper's three-buffer
 * split): W is cut into tiles of MQ_ROW_BLOCK rows x one group of 128 columns;
 * a tile is r consecutive 1 KiB lines, line i holding 16 bytes for each of the
 * 64 rows, so that one wavefront reads a tile with r fully coalesced 16-byte
 * loads and every lane owns one row's whole group.  Inside a lane's 4r dwords
 * each 16-bit half holds bit-fields at fixed positions that are valid fp16
 * subnormals after a mask (and at most one shift per dword).  Tiles are stored
 * row-block major, group minor.
 *
 *   S        : device, uint8 [N, K], codes on the 2^(8-r) grid as written by
 *              mq_slice_codes (the low 8-r bits are ignored)
 *   packed   : device, 16-byte aligned, packed_bytes >= mq_packed_bytes(N,K,r);
 *              rows N..Npad-1 are written as zero codes
 * mq_unpack is the exact inverse (writes S = t << (8-r) for the N real rows).
 * Errors: NULL, BAD_R (r not in {2,3,4,6,8} or c != 8), BAD_SHAPE (N < 1, K < 128),
 * BAD_GROUP (K % 128), ALIGN, BUF_TOO_SMALL. */
mq_status mq_pack(const uint8_t *S, int64_t N, int64_t K, int c, int r, void *packed,
                  size_t packed_bytes, mq_stream stream);
mq_status mq_unpack(const void *packed, int64_t N, int64_t K, int c, int r, uint8_t *S_out,
                    mq_stream stream);

/* ---------------------------------------------------------------- run-time re-slicing
 * Abstract / Section 1: ONE resident parent checkpoint serves every width; the
 * width of a layer is chosen when it is used, not when the file is written.
 * The resident form of the parent is its own 8-bit pack, `packed_parent` =
 * mq_pack(parent, c = 8, r = 8) (the unsliced codes in the tile layout above).
 *
 * mq_slice_pack : Eq. 1 + pack fused, from the row-major parent:
 *                 packed == mq_pack(mq_slice_codes(parent, 8, r), 8, r), bit for bit,
 *                 reading 1 byte and writing r/8 bytes per weight.
 * mq_reslice    : the same result from `packed_parent` (tile layout in, tile
 *                 layout out; both sides fully coalesced); this is the call that
 *                 switches a resident layer to another width.
 *   parent        : device, uint8 [N, K], 8-bit codes
 *   packed_parent : device, 16-byte aligned, mq_packed_bytes(N,K,8) bytes
 *   packed        : device, 16-byte aligned, packed_bytes >= mq_packed_bytes(N,K,r);
 *                   must not overlap packed_parent
 * Errors: NULL, BAD_R (r not in {2,3,4,6,8} or c != 8), BAD_SHAPE, BAD_GROUP, ALIGN,
 * BUF_TOO_SMALL. */
mq_status mq_slice_pack(const uint8_t *parent, int64_t N, int64_t K, int c, int r, void *packed,
                        size_t packed_bytes, mq_stream stream);
mq_status mq_reslice(const void *packed_parent, int64_t N, int64_t K, int c, int r, void *packed,
                     size_t packed_bytes, mq_stream stream);

/* mq_reslice for many layers at once (one launch per 16 layers; small layers are launch-bound one
 * by one): switches a whole resident model to another budget.  Each job as mq_reslice, with its
 * own r; outputs of different jobs must not overlap each other or any parent.
 *   jobs : HOST array of n_jobs entries; pointers inside are device pointers
 * Errors: as mq_reslice, for the first offending job; nothing is enqueued on error. */
typedef struct {
    const void *packed_parent; /* device, mq_pack(parent, 8, 8) of this layer */
    void *packed;              /* device, packed_bytes >= mq_packed_bytes(N, K, r) */
    size_t packed_bytes;
    int64_t N, K;
    int32_t r;        /* 2, 3, 4, 6 or 8 */
    int32_t reserved; /* 0 */
} mq_reslice_job;
mq_status mq_reslice_many(const mq_reslice_job *jobs, int n_jobs, int c, mq_stream stream);

/* Re-tile the per-group scale and zero-offset (Section 3.2 item 1: computed at
 * the master width c and shared by every r) to match the weight tiles:
 *   scales, zeros     : device, fp16 [N, K/group] row-major
 *   scales_t, zeros_t : device, fp16 [Npad/64][K/group][64], each of
 *                       meta_bytes >= mq_meta_bytes(N,K,group); pad rows get 0.
 *   zeros and zeros_t may both be NULL (symmetric layer: only the scales are tiled).
 * Errors: NULL (also: only one of zeros, zeros_t given), BAD_SHAPE, BAD_GROUP, BUF_TOO_SMALL. */
mq_status mq_pack_meta(const mq_half *scales, const mq_half *zeros, int64_t N, int64_t K,
                       int group, mq_half *scales_t, mq_half *zeros_t, size_t meta_bytes,
                       mq_stream stream);

/* ---------------------------------------------------------------- quantiser step
 * Algorithm 1 ("Generate Q^c given weight matrix W, target bit-widths R, and weights
 * lambda_R"; Section 3.2, item 2): for every weight the parent code q in 0 .. 2^c - 1 with the
 * smallest  E(q) = sum_{r in R} lambda_r * (w - scale * (S(q, r) - zero))^2,  S = Eq. 1, scale
 * and zero-offset those of the master width for every r.  All 256 candidates are evaluated (the
 * paper's brute force).  The argmin is taken in IEEE binary32 with every operation rounded on its
 * own, in the order  t = S - zero; D = scale * t; e = w - D; p = e * e; E = E + lambda_r * p,
 * r ascending; the smallest q wins a tie.  Inputs must be finite.
 *   W       : device, fp32, N rows of `ncols` weights, row stride ldw elements: columns
 *             col0 .. col0+ncols-1 of a layer with K input features (ncols = 1 is the
 *             column-at-a-time call of the GPTQ loop, ncols = K the whole matrix); 4-byte aligned
 *   scales, zeros : device, fp16 [N, K/group] row-major (NOT tiled)
 *   lambda  : HOST, 8 floats, lambda_r at [r-1] for r = 1..8; 0 = r is not a target width;
 *             all finite and >= 0, at least one > 0
 *   Q       : device, uint8, N rows of ncols codes, row stride ldq bytes
 * Four columns per lane when W is 16-byte and Q 4-byte aligned and ldw, ldq, ncols, col0 are
 * multiples of 4; one column per lane otherwise (same results).
 * Errors: NULL, BAD_R (c != 8, or lambda), BAD_SHAPE, BAD_GROUP, ALIGN, HIP. */
mq_status mq_quant_matgptq(const float *W, int64_t ldw, int64_t N, int64_t ncols, int64_t col0,
                           const mq_half *scales, const mq_half *zeros, int64_t K, int group, int c,
                           const float *lambda, uint8_t *Q, int64_t ldq, mq_stream stream);

/* The MatGPTQ column loop (Algorithm 2 of the appendix, "Quantize W given inverse Hessian ..."),
 * from the point where U, the upper-triangular Cholesky factor of H^-1 (the listing's
 * "H^-1 <- Cholesky(H^-1)^T"), is given.  In blocks of `block` columns, column by column j:
 *     Q[:, j] = Algorithm 1 on the current W[:, j]           (as mq_quant_matgptq, bit for bit)
 *     e       = mean over R of (W[:, j] - scale * (S(Q[:, j], r) - zero)),   E[:, j] = e / U[j, j]
 *     W[:, j+1 : end of block] -= E[:, j] * U[j, j+1 : end of block]
 * then W[:, after the block] -= E @ U[block rows, after the block].  lambda weighs Algorithm 1
 * only; the propagated error is the plain mean over R = {r : lambda_r != 0}.  Scale and
 * zero-offset are inputs fixed before the loop.  Arithmetic: binary32, every operation rounded on
 * its own, error terms added over r ascending, then / |R|, then / U[j,j]; each update is
 * w - (E * U[j,k]), applied in ascending j (the result does not depend on `block`).
 *   W       : device, fp32 [N, K], row stride ldw; OVERWRITTEN (working copy of the loop)
 *   U       : device, fp32 [K, K], row stride ldu; only the upper triangle is read
 *   scales, zeros : device, fp16 [N, K/group] row-major (NOT tiled)
 *   lambda  : HOST, 8 floats as for mq_quant_matgptq
 *   block   : 16, 32, 64 or 128 (the paper's B)
 *   Q       : device, uint8 [N, K], row stride ldq
 *   ws      : device, 4-byte aligned, ws_bytes >= mq_matgptq_workspace_bytes(N, block)
 * Enqueues 2 * K / block - 1 launches on `stream`; rows run in parallel, columns in sequence.
 * Errors: NULL, BAD_R, BAD_SHAPE, BAD_GROUP, ALIGN, BUF_TOO_SMALL, HIP. */
size_t mq_matgptq_workspace_bytes(int64_t N, int block);
mq_status mq_matgptq_quantize(float *W, int64_t ldw, int64_t N, int64_t K, const float *U, int64_t ldu,
                              const mq_half *scales, const mq_half *zeros, int group, int c,
                              const float *lambda, int block, uint8_t *Q, int64_t ldq, void *ws,
                              size_t ws_bytes, mq_stream stream);

/* ---------------------------------------------------------------- linear
 * Section 4:  y[m,n] = sum_k x[m,k] * scale[n,k/group] * (S[n,k] - zero[n,k/group])
 * with S the r-bit slice of Eq. 1 in c-bit units, fp16 inputs, fp32
 * accumulation, fp16 output (round to nearest even).
 *   x        : device, fp16 [M, K], 4-byte aligned
 *   packed_W : device, from mq_pack with the same N, K, r; 16-byte aligned
 *   scales_t, zeros_t : device, from mq_pack_meta; 16-byte aligned when M > 4;
 *                       zeros_t == NULL: symmetric layer
 *   y        : device, fp16 [M, N]; fully overwritten
 *   ws       : device, 256-byte aligned, ws_bytes >= mq_workspace_bytes(M,N,K,r),
 *              initialised once with mq_workspace_init
 * 1 <= M <= MQ_MAX_M.  Results do not depend on the launch shape run to run
 * (partial sums are combined in a fixed order).  Up to M = 16 every product
 * x * code is exact in fp32 and scale and zero are applied in fp32 once per
 * group; for M > 16 the weights are de-quantised to fp16 first (the fp16 operands
 * of the paper's TensorCore kernel): scale * (S - zero) carries one fp16 rounding,
 * relative 2^-11, before the fp32 accumulation.
 * Errors: NULL, BAD_R, BAD_SHAPE, BAD_GROUP, ALIGN, BUF_TOO_SMALL, UNSUPPORTED, HIP. */
mq_status mq_linear(const mq_half *x, int64_t M, const void *packed_W, const mq_half *scales_t,
                    const mq_half *zeros_t, int64_t N, int64_t K, int r, int group, mq_half *y,
                    void *ws, size_t ws_bytes, mq_stream stream);

/* mq_linear on bfloat16 activations with a bfloat16 result (flags MQ_X_BF16 | MQ_Y_BF16 of mq_layer;
 * a stack may also mix the two per layer).  Everything else as mq_linear. */
mq_status mq_linear_bf16(const mq_bf16 *x, int64_t M, const void *packed_W, const mq_half *scales_t,
                         const mq_half *zeros_t, int64_t N, int64_t K, int r, int group, mq_bf16 *y,
                         void *ws, size_t ws_bytes, mq_stream stream);

/* mq_linear for callers that cannot allocate and have no workspace to hand over: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels and results
 * as mq_linear (to rounding: the split-K shares may be cut differently), but the counters, the
 * split-K partial sums and, for M > 4, the prepared activations live in a static device array of
 * MQ_NOALLOC_SCRATCH_BYTES inside the library instead of a caller's `ws`.  The call allocates
 * nothing, frees nothing and initialises what it needs itself (one small fill kernel ahead of the
 * layer's launches, all on `stream`).
 *   1 <= M <= 16; larger batches return MQ_ERR_UNSUPPORTED (their partial sums alone exceed the array).
 *   Shapes whose counters + prepared activations + a minimum of partial-sum slot pairs (256 of
 *   64 x M floats up to M = 4, 32 of 8192 floats above) do not fit the array return
 *   MQ_ERR_BUF_TOO_SMALL (every Llama-2-7B and Llama-3-70B linear fits at M <= 16).
 * Every call on a GPU uses that GPU's one array: two calls that may overlap in time on the same
 * GPU (different streams, or graphs replayed concurrently) race; calls on one stream do not.  The
 * device current to the calling thread must be the stream's device.  The first call on a device
 * looks the array's address up (a host-side query): make it outside stream capture.
 * Other arguments, results and errors as mq_linear. */
mq_status mq_linear_noalloc(const mq_half *x, int64_t M, const void *packed_W, const mq_half *scales_t,
                            const mq_half *zeros_t, int64_t N, int64_t K, int r, int group, mq_half *y,
                            mq_stream stream);

/* The call shape of the paper's kernel interface (Section 4: activations, packed weights, scales,
 * zero-offsets in, y out) for callers that keep the quantiser's own [N, K/group] arrays: scales and
 * zeros are re-tiled into `ws` by one small extra launch (reads and writes 4 * N * K/group bytes)
 * and mq_linear runs on the result.  A hot loop tiles once with mq_pack_meta and calls mq_linear.
 *   scales, zeros : device, fp16 [N, K/group] row-major (NOT tiled)
 *   ws            : device, 256-byte aligned, ws_bytes >= mq_linear_plain_workspace_bytes(M,N,K,r),
 *                   initialised once with mq_workspace_init
 * Other arguments, results and errors as mq_linear. */
size_t mq_linear_plain_workspace_bytes(int64_t M, int64_t N, int64_t K, int r);
mq_status mq_linear_plain(const mq_half *x, int64_t M, const void *packed_W, const mq_half *scales,
                          const mq_half *zeros, int64_t N, int64_t K, int r, int group, mq_half *y,
                          void *ws, size_t ws_bytes, mq_stream stream);

/* The same layer computed straight from the resident 8-bit parent: Eq. 1 is
 * applied to the codes in registers, so any r is served without a packed copy of
 * its own (8 bits per weight are streamed whatever r is).  Same arithmetic as
 * mq_linear at M <= 4 (exact products, fp32 accumulation, scale and zero once per
 * group); the order of the fp32 additions differs from the r-bit layout's, so the
 * two agree to rounding, not bit for bit.
 *   packed_parent : device, 16-byte aligned, mq_pack(parent, 8, 8)
 *   ws            : as for mq_linear, ws_bytes >= mq_workspace_bytes(M,N,K,8)
 * 1 <= M <= 4 (the vector-ALU path); larger M returns MQ_ERR_UNSUPPORTED: re-slice
 * with mq_reslice and call mq_linear.  Other arguments and errors as mq_linear. */
mq_status mq_linear_from_parent(const mq_half *x, int64_t M, const void *packed_parent,
                                const mq_half *scales_t, const mq_half *zeros_t, int64_t N,
                                int64_t K, int r, int group, mq_half *y, void *ws,
                                size_t ws_bytes, mq_stream stream);

/* ---------------------------------------------------------------- stack
 * Sections 3.3 / 5.5: a model is the sliced layers stitched together, one r per
 * layer.  A stack is executed by ONE persistent launch that walks all layers.
 * Layers are independent: each has its own x and y (the attention / activation
 * code between Llama linears is outside this library). */
typedef struct {
    const void *packed_W;    /* device, mq_pack(N, K, r); the 8-bit pack of the parent if from_parent */
    const mq_half *scales_t; /* device, mq_pack_meta */
    const mq_half *zeros_t;  /* device, mq_pack_meta; NULL: symmetric layer (every zero-offset 128) */
    const mq_half *x;        /* device, fp16 [M, K] */
    mq_half *y;              /* device, fp16 [M, N] */
    int64_t N, K;
    int32_t r;     /* 2, 3, 4, 6 or 8 */
    int32_t group; /* 128 */
    int32_t from_parent; /* 0: packed_W holds r-bit codes.  1: packed_W is the resident 8-bit parent and
                            Eq. 1 is applied in registers (as mq_linear_from_parent; M <= 4, and all
                            layers of a stack must agree, else MQ_ERR_UNSUPPORTED) */
    int32_t flags;       /* 0, or MQ_X_BF16 | MQ_Y_BF16 | MQ_X_AFTER_EARLIER (below); other bits: MQ_ERR_UNSUPPORTED */
} mq_layer;

/* bf16 activations and outputs, per layer.
 *   MQ_X_BF16 : x points to bfloat16 values.  They are converted to fp16 before they are multiplied
 *               (M <= 4: by a small launch of its own ahead of the layer's, into the workspace; M > 4:
 *               inside the activation preparation), which is exact for every value whose magnitude is within the fp16 range
 *               (2^-14 <= |x| <= 65504, and 0): results are then those of the same values given as
 *               fp16, bit for bit.  Larger magnitudes become infinities, smaller ones keep what
 *               fp16 subnormals hold (absolute error <= 2^-25).
 *   MQ_Y_BF16 : y is written as bfloat16, the fp32 sums rounded to nearest even.  (An 8-bit
 *               significand rounds by up to 2^-9 relative: such outputs are within one bf16 rounding
 *               of the fp16-output result, not within its 1e-3 relative-L2 distance of the exact y.) */
#define MQ_X_BF16 1
#define MQ_Y_BF16 2

/* A chained stack (the decode-shaped fusion in which one launch carries layers that feed each other): per layer,
 *   MQ_X_AFTER_EARLIER : this layer's x is written by this very launch -- it is, or is assembled from, the y of
 *               EARLIER layers of the same stack (a chain x -> y0 -> y1, or two outputs side by side as one input).
 *               The layer's workgroups fetch their first weights, then wait inside the launch until every earlier
 *               layer's y is complete and visible to the whole device, and only then read x: a barrier across the
 *               launch in front of that layer.  Layers without the flag do not wait, whatever stands before them.
 * Only for a stack that is launched for latency with all its workgroups resident on the device at one time (at most
 * 16 layers and 12288 tiles in all, see below) and M <= 3: then every workgroup that is waited for is running, and it
 * waits, if at all, for strictly earlier layers, so every wait ends.  mq_stack_plan returns MQ_ERR_UNSUPPORTED for the
 * flag on the first layer, on a layer with MQ_X_BF16 (nothing could convert its activations ahead of the launch), in a
 * larger stack or at M > 3, and MQ_ERR_HIP if the device at hand cannot hold the stack's workgroups at one time.  (The
 * number of polls of a wait is bounded as well -- about a second; a wait that ran out would go on with whatever x
 * holds.)  Between the layers of a Llama block sits the caller's attention / activation code, which cannot run inside
 * this launch: the flag is for layers that really feed each other. */
#define MQ_X_AFTER_EARLIER 4

/* Kernels by batch: as mq_linear, except that a stack of packed layers already runs on the matrix
 * cores at M = 4 (scales_t / zeros_t 16-byte aligned from M = 4 on for a stack); stacks computed
 * from the parent stay on the vector ALUs (M <= 4).  A small stack (at most 16 layers and 12288
 * tiles of 64 rows x 128 columns in all, M <= 4: the q/k/v or gate/up linears of a decoder block,
 * which may share one x) is launched for latency, one workgroup per (layer, row block, K slice);
 * larger ones as one persistent stream-K launch.
 *
 * Bytes of plan workspace for a stack of these layers (host arithmetic; 0 on
 * invalid arguments).  layers: host. */
size_t mq_stack_workspace_bytes(const mq_layer *layers, int n_layers, int64_t M);

/* What mq_linear_stack needs to know about a planned stack.  HOST memory owned by the caller,
 * filled by mq_stack_plan, opaque (2176 bytes: a header and, for a stack of at most 16 layers that
 * is launched for latency, those layers' descriptors, which then travel with the kernel arguments).
 * It names the device workspace it was built in: it is valid for as long as that workspace and the
 * layers' buffers are, may be copied freely, and must be filled again if the workspace is reused for
 * anything else. */
typedef struct {
    uint64_t opaque[272];
} mq_plan;

/* Validate the layers and build the schedule of the stack: the descriptor table is written into
 * `plan_ws` (through kernel arguments, ceil(n_layers / 32) small launches on `stream`: `layers` may
 * be reused as soon as the call returns) and its counters are zeroed; `plan` receives the header.
 * Done once per stack, like packing.  Nothing is copied, read back or waited for.
 *   layers  : host, n_layers entries
 *   plan_ws : device, 256-byte aligned, plan_bytes >= mq_stack_workspace_bytes(layers, n_layers, M)
 *   plan    : host, out
 * Errors: NULL, BAD_SHAPE, BAD_R, BAD_GROUP, ALIGN, BUF_TOO_SMALL, UNSUPPORTED, HIP; `plan` is
 * written only on MQ_OK. */
mq_status mq_stack_plan(const mq_layer *layers, int n_layers, int64_t M, void *plan_ws,
                        size_t plan_bytes, mq_plan *plan, mq_stream stream);

/* Run every layer of a planned stack: one launch (two on the matrix-core paths), asynchronous on
 * `stream`, after the work mq_stack_plan enqueued (same stream, or ordered by the caller).
 * A plan must not be used by two calls that may run concurrently.
 * Errors: NULL; BAD_SHAPE if `plan` was not filled by mq_stack_plan (or was overwritten); HIP. */
mq_status mq_linear_stack(const mq_plan *plan, mq_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* MQ_H */
