/*
 * qail.h - C ABI of libqail: 4-bit quantised linear layers on AMD MI355X (gfx950).
 *
 * The operations are the deployed low-bit layers behind the efficiency results
 * of "Quantization-Aware Imitation-Learning for Resource-Efficient Robotic
 * Control" (Sec. 5.4 "Implementation" and the appendix "Analysis"):
 *
 *   W4A16  weight-only 4-bit linears of the Llama-2-7B backbone of the VLA
 *          policy.  Sec. 2.1: LLM linears are limited by weight loading, so only
 *          the weight operand of the GEMM is quantised; Sec. 5.1: 4-bit AWQ
 *          format (unsigned codes, scale, integer zero-point).  The appendix
 *          "Analysis" finds the decode stage memory-bound; that is the M = 1 case.
 *   W4A4   4-bit weights and 4-bit activations of the ResNet encoder of the
 *          driving policy.  Sec. 2.1: convolutional models are compute-bound, so
 *          both GEMM operands are quantised; Sec. 5.1: RTN / LSQ integer format.
 *
 * Conventions for every call
 *   - All data pointers are DEVICE pointers into memory owned by the caller,
 *     16-byte aligned.  Descriptors and size outputs are HOST pointers.  The
 *     library allocates nothing and frees nothing.  The only state it keeps is
 *     what it learns about the device at a call's first use (the number of
 *     compute units, the opt-in for large LDS blocks); those are set once,
 *     through atomics, so calls may come from several host threads.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     A call validates its arguments, enqueues its kernels and returns; it never
 *     synchronises.  Outputs are fully overwritten.
 *   - Argument errors (null pointer, bad shape, misalignment, short workspace)
 *     are detected before anything is launched and leave device memory untouched;
 *     they can be exercised on a host without a GPU.  A failed launch maps to
 *     QAIL_ERR_HIP.
 *   - Packed 4-bit data: 8 codes per uint32, code j of the packed axis in bits
 *     [4*(j%8), 4*(j%8)+3] of word j/8.  Signed codes are two's-complement nibbles.
 *   - bf16 and fp16 values cross the boundary as their 16-bit patterns (uint16_t).
 *   - Inputs are finite.  NaN or infinity in a tensor to be quantised gives
 *     unspecified codes (no fault).
 */
#ifndef QAIL_H
#define QAIL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    QAIL_OK = 0,
    QAIL_ERR_NULL = -1,        /* a required pointer is NULL */
    QAIL_ERR_SHAPE = -2,       /* a dimension is non-positive or violates a divisibility rule */
    QAIL_ERR_ALIGN = -3,       /* a device pointer is not 16-byte aligned */
    QAIL_ERR_WORKSPACE = -4,   /* workspace missing or smaller than the matching *_workspace query */
    QAIL_ERR_UNSUPPORTED = -5, /* valid request outside what the kernels cover */
    QAIL_ERR_HIP = -6          /* the HIP runtime refused a launch */
} qail_status;

typedef enum {
    /* Unsigned codes 0..15, one fp16 scale and one integer zero-point 0..15 per
     * group of `group_size` consecutive k of a row (Sec. 5.1, VLA policy;
     * group_size == K is the channel-wise case of the appendix). */
    QAIL_W4_ASYM_GROUP = 0,
    /* Signed codes -8..7, one fp32 scale per row (output channel); group_size is
     * ignored (Sec. 5.1, driving policy). */
    QAIL_W4_SYM_CHANNEL = 1,
    /* 8-bit variants (Sec. 5.4: W8A8 driving encoder, 8-bit weight-only backbone).  The paper
     * names no 8-bit quantiser; both are symmetric round-to-nearest with signed codes
     * -127..127, packed 4 per word (code i of a word in bits 8*(i%4)..8*(i%4)+7):
     * one fp32 scale max|w|/127 per row ... */
    QAIL_W8_SYM_CHANNEL = 2,
    /* ... or one fp16 scale per group of `group_size` consecutive k, rounded up, >= 2^-14. */
    QAIL_W8_SYM_GROUP = 3
} qail_scheme;

/* A quantised weight matrix W[N][K] (row n = output channel, K contiguous). */
typedef struct {
    int32_t N;          /* rows / output channels, >= 1 */
    int32_t K;          /* columns / input channels, multiple of 8 */
    int32_t group_size; /* ASYM_GROUP: multiple of 8 that divides K */
    int32_t scheme;     /* qail_scheme */
} qail_wdesc;

/* A 2-D convolution read as a GEMM with M = B*OH*OW, N = Cout, K = KH*KW*Cin,
 * OH = (H + 2*pad - KH)/stride + 1 (same for OW).  KH = KW = 1, stride = 1,
 * pad = 0 makes it a plain [B*H*W, Cin] x [Cout, Cin]^T GEMM. */
typedef struct {
    int32_t B, H, W;    /* batch, input height, input width */
    int32_t Cin, Cout;  /* Cin multiple of 8; Cout >= 1 */
    int32_t KH, KW;     /* filter taps */
    int32_t stride, pad;
} qail_conv_desc;

int qail_version(void);
const char* qail_status_string(int status);

/* ---------------------------------------------------------------- quantise --
 * Sec. 2.1 (round-to-nearest) and Sec. 5.1 (the two 4-bit formats). */

/* Byte sizes of the packed form of `d` (host computation only):
 *   qweight  N * K/8 uint32
 *   scales   ASYM_GROUP: N * K/group_size fp16     SYM_CHANNEL: N fp32
 *   zeros    ASYM_GROUP: N * ceil(K/group_size/8) uint32 (unused nibbles 0)
 *            SYM_CHANNEL: 0
 * Any output pointer may be NULL. */
int qail_packed_sizes(const qail_wdesc* d, size_t* qweight_bytes, size_t* scales_bytes,
                      size_t* zeros_bytes);

/* Round-to-nearest quantisation of w (fp32, [N][K] row-major) into the packed form.
 *
 * ASYM_GROUP, per row and group, in IEEE fp32 with correctly rounded division:
 *   lo = min(min w, 0); hi = max(max w, 0)
 *   s  = (hi - lo)/15 rounded UP to fp16, at least 2^-14; an all-zero group has s = 1
 *   z  = clamp(rint(-lo/s), 0, 15);  q = clamp(rint(w/s) + z, 0, 15)   (ties to even)
 * SYM_CHANNEL, per row:
 *   s  = max|w|/7 (fp32; 1 for an all-zero row);  q = clamp(rint(w/s), -8, 7)
 *   `zeros` is ignored and may be NULL.
 *
 * range_errors (device, one uint32, may be NULL): if given it is NOT cleared; it is
 * incremented once per ASYM group whose (hi-lo)/15 exceeds the largest fp16
 * (65504).  Such a group is stored with s = 65504 and clamped codes. */
int qail_quantize_weights(const qail_wdesc* d, const float* w, uint32_t* qweight, void* scales,
                          uint32_t* zeros, uint32_t* range_errors, void* stream);

/* Packed words -> one code per byte, [N][K]: uint8 0..15 (ASYM_GROUP) or int8 -8..7
 * (SYM_CHANNEL, sign-extended). */
int qail_unpack_weights(const qail_wdesc* d, const uint32_t* qweight, uint8_t* codes, void* stream);

/* One activation step size for a whole tensor (appendix: tensor-wise activation
 * quantisation): *s_a = max(a)/15 in fp32, or 1 if no element is positive.
 * a: fp32 [n]; s_a: device, one float. */
int qail_act_scale_u4(const float* a, size_t n, float* s_a, void* stream);

/* q = clamp(rint(a / *s_a), 0, 15), packed 8 per word along the flat index
 * (for an NHWC tensor that is along C).  n multiple of 8; s_a: device, one float. */
int qail_quantize_act_u4(const float* a, size_t n, const float* s_a, uint32_t* a_u4, void* stream);

/* ------------------------------------------------------------------ W4A16 --
 * y[m][n] = sum_k x[m][k] * (q[n][k] - z[n][k/g]) * s[n][k/g]
 * Sec. 2.1 (weight-only quantised GEMM operand); appendix "Analysis" (decode is
 * the memory-bound stage, prefill the compute-heavy one). */

/* Bytes of device scratch the call below needs for this (d, M).  0 for the streaming
 * kernels (M <= 16 on shapes they take, M <= 32 at group_size 128 with an even number of
 * groups per row); for the matrix-core GEMM it holds an fp16 copy
 * of x (rows padded to a multiple of 128, K to a multiple of 128), one float per padded
 * row and per output column, and two tile-shaped fp32 slots per block of the grid (one
 * block per compute unit) for output tiles whose K range is shared between blocks (tens
 * of MB at prefill sizes).  The workspace must be 256-byte aligned, is
 * overwritten by every call and carries nothing between calls; calls that share one
 * must be ordered on one stream. */
int qail_w4a16_workspace(const qail_wdesc* d, int32_t M, size_t* bytes);

/* d must be ASYM_GROUP.  x: bf16 [M][K]; y: bf16 [M][N].  Products are accumulated
 * in fp32 and rounded once to bf16 (nearest even).  M = 1 (decode) is served by a
 * bandwidth-bound streaming kernel, 2 <= M <= 4 by the same stream with four rows of x,
 * up to M = 16 (M = 32 at group_size 128 with an even number of groups per row) by a
 * weight-streaming MFMA kernel (x and codes exact in the products),
 * larger M (prefill) by an fp16 MFMA kernel that expands the codes in registers
 * ((q - z) * s rounded once to fp16, x rescaled per row by a power of two).
 * workspace may be NULL when the query returns 0; otherwise a missing or short one
 * is QAIL_ERR_WORKSPACE and a misaligned one QAIL_ERR_ALIGN. */
int qail_w4a16_linear(const qail_wdesc* d, const uint32_t* qweight, const uint16_t* scales,
                      const uint32_t* zeros, const uint16_t* x, uint16_t* y, int32_t M,
                      void* workspace, size_t workspace_bytes, void* stream);

/* One linear of a batch for qail_w4a16_linear_batch. */
typedef struct {
    qail_wdesc d;
    const uint32_t* qweight;
    const uint16_t* scales;
    const uint32_t* zeros;
    const uint16_t* x;   /* bf16 [M][K] */
    uint16_t* y;         /* bf16 [M][N] */
} qail_w4a16_item;

/* `count` linears with the same M, given as a HOST array, enqueued on one stream
 * (appendix "Analysis": a decode step is a fixed sequence of such linears, 4 per
 * layer).  The items must be independent: no item may read what another writes.
 * The library may run them in fewer launches, items side by side on shares of the
 * GPU.  The result is that of `count` calls of qail_w4a16_linear: bit for bit for
 * M <= 4; for larger M an item's sum over K may be divided between waves or blocks
 * at other places than in a call of its own, so the two can differ by the rounding
 * of fp32 partial sums (far inside the W4A16 tolerance); the same call on the same
 * GPU always gives the same bits.  count >= 0 (0 is a no-op). */
int qail_w4a16_linear_batch(const qail_w4a16_item* items, int32_t count, int32_t M,
                            void* workspace, size_t workspace_bytes, void* stream);
/* Workspace for the batch call.  Items that share a launch (M > 16: up to 8 at a time)
 * keep their prepared activations side by side in it, so the need can exceed that of
 * any single item; launches that follow each other on the stream reuse it. */
int qail_w4a16_batch_workspace(const qail_w4a16_item* items, int32_t count, int32_t M,
                               size_t* bytes);

/* Linears that depend on each other, M = 1, in one launch (appendix "Analysis": the decode stage
 * walks the backbone's linears one after the other, each a bandwidth-bound stream of weights).
 * Item i + 1 does not read its x before every element of item i's y has been written, so x of
 * item i + 1 may be, or overlap, y of item i; apart from that the results are those of
 * qail_w4a16_linear_batch at M = 1, bit for bit.  The whole grid is resident on the GPU and the
 * blocks meet between two items through counters in the workspace, while the first weights of the
 * next item are already on their way: the stream of weights does not stop between items as it
 * does between launches.  Up to 32 items share a launch; longer lists take several.
 *   items      HOST array; every item must be one the M = 1 streaming kernel takes
 *              (K % 32 == 0, group_size % 32 == 0, K <= 12288) with N <= 512 * CUs, else
 *              QAIL_ERR_UNSUPPORTED.
 *   workspace  qail_w4a16_chain_workspace() bytes, 256-byte aligned.  Its first uint32 is a status
 *              word, written by the call: 0 if every block saw the others arrive, 1 if some block
 *              gave up waiting (possible only when other work keeps part of the grid off the GPU;
 *              the outputs are then unspecified, and every kernel still ends). */
int qail_w4a16_chain_workspace(const qail_w4a16_item* items, int32_t count, size_t* bytes);
int qail_w4a16_linear_chain(const qail_w4a16_item* items, int32_t count, void* workspace,
                            size_t workspace_bytes, void* stream);

/* Low-rank adapter beside a 4-bit linear (Sec. 5.1: the 4-bit policy is fine-tuned with
 * rank-32 adapters on the quantised backbone; they stay separate from the packed weights):
 *     y[m][n] = sum_k x[m][k] w_hat[n][k]  +  scaling * sum_j (sum_k x[m][k] A[j][k]) B[n][j]
 * A: bf16 [r][K], B: bf16 [N][r], device memory, 16-byte aligned; 8 <= r <= 64, r % 8 == 0. */
typedef struct {
    const uint16_t* A;
    const uint16_t* B;
    int32_t r;
    float scaling;
} qail_lora;

/* Like qail_w4a16_linear_batch with one adapter per item (loras: HOST array of `count`).
 * At M = 1 on shapes the streaming kernel takes, the up-projection joins the linear before
 * the single bf16 rounding of y; otherwise it is added to the rounded y and rounded again
 * (inside the W4A16 tolerance).  The workspace (query below; 256-byte aligned) holds the
 * linear's own workspace and the down-projections x A^T in fp32.  Errors as for the batch
 * call, plus QAIL_ERR_SHAPE for a rank outside the range above. */
int qail_w4a16_lora_workspace(const qail_w4a16_item* items, const qail_lora* loras, int32_t count,
                              int32_t M, size_t* bytes);
int qail_w4a16_linear_lora_batch(const qail_w4a16_item* items, const qail_lora* loras, int32_t count,
                                 int32_t M, void* workspace, size_t workspace_bytes, void* stream);

/* qail_w4a16_linear_lora_batch for callers that cannot allocate device memory (code under
 * HIP graph capture, serving loops that must not call hipMalloc, harnesses that forbid it):
 * the same kernels and the same results, with the workspace taken from a scratch array that is
 * part of the library's device image (qail_static_scratch_bytes: 1 MiB, held on every GPU the
 * library runs on until the process ends).  The call allocates nothing and frees nothing.
 * A request whose qail_w4a16_lora_workspace figure exceeds the scratch returns
 * QAIL_ERR_WORKSPACE before anything is launched (a decode batch of M <= 16 on up to 16
 * linears that the streaming kernels take, e.g. the 7B shapes with groups of 128, needs
 * 64 KiB; anything routed to the matrix-core GEMM needs megabytes and does not fit).  All calls on one GPU share that GPU's array: calls that
 * overlap on one GPU (two streams, two host threads) race on it and must be serialised by the
 * caller; calls that follow each other on one stream are safe, since each call writes what it
 * reads.  The scratch address of a GPU is looked up at the first call made with that GPU
 * current; make that first call outside graph capture. */
int qail_static_scratch_bytes(size_t* bytes);
int qail_w4a16_linear_lora_batch_static(const qail_w4a16_item* items, const qail_lora* loras,
                                        int32_t count, int32_t M, void* stream);

/* ------------------------------------------------------------------- W4A4 --
 * acc[(b,oh,ow)][n] = sum_{kh,kw,c} a[b][oh*stride+kh-pad][ow*stride+kw-pad][c] * w[n][kh][kw][c]
 * with zero outside the image, exact in int32; then optionally
 * y = float(acc) * scale[n] + bias[n]   (one fp32 fused multiply-add).
 * Sec. 2.1 (both GEMM operands quantised for compute-bound convolutions);
 * Sec. 5.4 (W4A4 GPU kernels of the driving policy). */

int qail_w4a4_workspace(const qail_conv_desc* d, size_t* bytes);

/* a_u4: packed unsigned codes, NHWC [B][H][W][Cin/8] words.
 * w_s4: packed signed codes [Cout][KH][KW][Cin/8] words.
 * acc_out: int32 [M][Cout] or NULL.  y_out: fp32 [M][Cout] or NULL (then scale and
 * bias, fp32 [Cout], are required).  At least one output must be given.
 * |acc| <= 8*15*K must stay below 2^27 (K <= 1118480). */
int qail_w4a4_gemm(const qail_conv_desc* d, const uint32_t* a_u4, const uint32_t* w_s4,
                   int32_t* acc_out, const float* scale, const float* bias, float* y_out,
                   void* workspace, size_t workspace_bytes, void* stream);

/* The same convolution with the output written directly as the NEXT layer's packed
 * unsigned 4-bit activations (Sec. 5.1 and the appendix's implementation details for
 * autonomous driving: every activation tensor of the driving encoder is 4-bit with one
 * step per tensor, so the consumer's step s_out is a constant of the network).  Per
 * output element, each line one correctly rounded fp32 operation (no fused multiply-add):
 *     t = float(acc) * scale[n]
 *     t = t + bias[n]
 *     t = t + r                  only with a shortcut, see below
 *     t = max(t, 0)              ReLU
 *     q = clamp(rint(t / s_out), 0, 15)        rint: ties to even
 * out_u4: [M][Cout/8] words, i.e. NHWC [B][OH][OW][Cout/8], the a_u4 layout; Cout % 8 == 0.
 * Shortcut of a residual block, at most one of
 *     res_u4:  packed unsigned codes [M][Cout/8] (the block input), r = res_scale * code;
 *     res_f32: fp32 [M][Cout] (a projection shortcut's y_out), r = res_f32[m][n].
 * scale, bias: fp32 [Cout], required.  s_out > 0 and res_scale >= 0 are host values.
 * All buffers are device memory owned by the caller; nothing is allocated, the call is
 * enqueued on `stream` and returns.  Errors as for qail_w4a4_gemm, plus QAIL_ERR_SHAPE for
 * Cout % 8 != 0, s_out not positive and finite, or two shortcuts at once. */
int qail_w4a4_conv_u4(const qail_conv_desc* d, const uint32_t* a_u4, const uint32_t* w_s4,
                      const float* scale, const float* bias, float s_out,
                      const uint32_t* res_u4, float res_scale, const float* res_f32,
                      uint32_t* out_u4, void* workspace, size_t workspace_bytes, void* stream);

/* Several independent W4A4 convolutions in as few launches as possible (one, when every
 * item is a shape the tiled kernel runs and count <= 4).  Sec. 5.1 / appendix: the driving
 * encoder is a ResNet, whose down-sampling blocks start with two convolutions that read the same
 * input, the 3x3 stride-2 one and the 1x1 projection of the shortcut; at a small batch a launch
 * costs more than either of them.
 * An item is the argument list of qail_w4a4_gemm (out_u4 == NULL: acc_out and / or y_out) or
 * of qail_w4a4_conv_u4 (out_u4 != NULL: acc_out and y_out must be NULL); every rule of those
 * two calls holds per item, and each item's results equal the single call's bit for bit.
 * Items must be independent: no item may read a buffer another item writes, and no two may
 * write the same one.  1 <= count <= 64.  Errors are reported before anything is launched. */
typedef struct {
    qail_conv_desc d;
    const uint32_t* a_u4;    /* device */
    const uint32_t* w_s4;    /* device */
    const float* scale;      /* device, fp32 [Cout]; required with y_out or out_u4 */
    const float* bias;       /* device, fp32 [Cout]; required with y_out or out_u4 */
    int32_t* acc_out;        /* device, int32 [M][Cout] or NULL */
    float* y_out;            /* device, fp32 [M][Cout] or NULL */
    uint32_t* out_u4;        /* device, [M][Cout/8] words or NULL */
    float s_out;             /* fused output only */
    float res_scale;         /* fused output with res_u4 only */
    const uint32_t* res_u4;  /* device or NULL */
    const float* res_f32;    /* device or NULL */
} qail_conv_item;
int qail_w4a4_conv_batch(const qail_conv_item* items, int32_t count, void* stream);

/* ------------------------------------------------------------------ 8-bit --
 * Sec. 5.4 deploys the driving encoder also as W8A8 and the backbone also with 8-bit
 * weights only.  Weights: qail_quantize_weights / qail_packed_sizes with the W8 schemes
 * (zeros unused, may be NULL; qail_unpack_weights is not needed: the codes are bytes). */

/* One activation step for a whole tensor: *s_a = max|a| / 127 in fp32, 1 if all zero. */
int qail_act_scale_s8(const float* a, size_t n, float* s_a, void* stream);

/* q = clamp(rint(a / *s_a), -127, 127), 4 codes per word along the flat index; n % 4 == 0. */
int qail_quantize_act_s8(const float* a, size_t n, const float* s_a, uint32_t* a_s8, void* stream);

/* qail_w4a4_gemm with signed 8-bit codes on both sides: a_s8 NHWC [B][H][W][Cin/4] words,
 * w_s8 [Cout][KH][KW][Cin/4] words, Cin % 4 == 0, K = KH*KW*Cin <= 131071 (int32 exact for
 * all codes in [-128, 127]).  Outputs, errors and ownership as for qail_w4a4_gemm. */
int qail_w8a8_gemm(const qail_conv_desc* d, const uint32_t* a_s8, const uint32_t* w_s8,
                   int32_t* acc_out, const float* scale, const float* bias, float* y_out,
                   void* workspace, size_t workspace_bytes, void* stream);

/* y[m][n] = sum_k x[m][k] * q[n][k] * s[n][k/g], d of scheme QAIL_W8_SYM_GROUP, x and y bf16,
 * fp32 accumulation, one rounding.  M = 1 runs a bandwidth-bound streaming kernel (K % 16 == 0,
 * group_size % 16 == 0, K + K/g <= 16384).  2 <= M <= 32 at group_size 128 with an even number
 * of groups per row (N * K below 2 GB) runs the small-batch streaming kernel of
 * qail_w4a16_linear with byte weights (x and q exact in the products, fp32 accumulation, no
 * workspace).  Other M > 1 runs on the fp16 matrix cores (the kernel of
 * qail_w4a16_linear for M > 16 with byte codes: K % 64 == 0, group_size % 64 == 0, an even
 * number of scales; (q * s) is rounded once to fp16 before the fp32 accumulation) and needs the
 * workspace the query below reports, 256-byte aligned.  Shapes outside both go to a plain
 * one-thread-per-output kernel.  Errors as for qail_w4a16_linear. */
int qail_w8a16_workspace(const qail_wdesc* d, int32_t M, size_t* bytes);
int qail_w8a16_linear(const qail_wdesc* d, const uint32_t* qweight, const uint16_t* scales,
                      const uint16_t* x, uint16_t* y, int32_t M, void* workspace,
                      size_t workspace_bytes, void* stream);

/* One linear of a batch for qail_w8a16_linear_batch (device pointers, 16-byte aligned). */
typedef struct {
    qail_wdesc d;
    const uint32_t* qweight;
    const uint16_t* scales;
    const uint16_t* x;   /* bf16 [M][K] */
    uint16_t* y;         /* bf16 [M][N] */
} qail_w8a16_item;

/* `count` independent 8-bit weight-only linears with the same M, given as a HOST array
 * (Sec. 5.4 also deploys the backbone with 8-bit weights: a decode step is again four such
 * linears per layer, a prefill pass four such GEMMs).  At M = 1 the items the streaming kernel
 * takes share launches (up to 8 each), every item on a share of the blocks, with the single
 * calls' results bit for bit; at M > 1 up to 8 consecutive items of the matrix-core path share
 * launches the same way (a different division of K than in a call of its own, so equal within
 * the W4A16 tolerance rather than bit for bit).  count >= 0 (0 is a no-op); workspace as
 * reported by the batch query; errors as for the single call. */
int qail_w8a16_batch_workspace(const qail_w8a16_item* items, int32_t count, int32_t M, size_t* bytes);
int qail_w8a16_linear_batch(const qail_w8a16_item* items, int32_t count, int32_t M, void* workspace,
                            size_t workspace_bytes, void* stream);

/* ------------------------------------------------------- training-side operators --
 * Sec. 4.1 / Algorithm 1: the quantised policy is trained through its quantisers with the
 * straight-through estimator.  Sec. 4.2 / Eq. 3: the QBC term; the appendix instantiates its
 * discrepancy as the mean L2 distance between the two policies' final logits. */

/* Forward of quantisation-aware training for a 4-bit group-quantised weight: w_hat =
 * dequantise(quantise(w)) with the ASYM_GROUP quantiser above, fp32 [N][K] -> fp32 [N][K]
 * (exact: (q - z) * s has at most 16 significant bits).  Its straight-through backward is the
 * identity, so no call exists for it. */
int qail_fake_quant_w4(const qail_wdesc* d, const float* w, float* w_hat, void* stream);

/* Learned-step quantiser (named in Sec. 5.1 for the driving policy): v_hat = clamp(rint(v / *s),
 * qn, qp) * *s in fp32; s: device, one float; qn <= 0 <= qp. */
int qail_lsq_forward(const float* v, size_t n, const float* s, int32_t qn, int32_t qp, float* v_hat,
                     void* stream);

/* Straight-through backward: dv = dout where qn <= v / s <= qp, else 0;
 * *ds = grad_scale * sum dout * t, t = rint(v/s) - v/s inside, qn below, qp above (fp32 sums in
 * a fixed order).  workspace: qail_lsq_backward_workspace bytes, 16-byte aligned. */
int qail_lsq_backward_workspace(size_t* bytes);
int qail_lsq_backward(const float* v, const float* dout, size_t n, const float* s, int32_t qn, int32_t qp,
                      float grad_scale, float* dv, float* ds, void* workspace, size_t workspace_bytes,
                      void* stream);

/* *loss = mean_b || logits_q[b] - logits_fp[b] ||_2 over fp32 [B][D]; grad_q (optional, [B][D]) =
 * d loss / d logits_q = (diff / ||diff||) / B, zero for rows with zero distance.
 * workspace: B floats, 16-byte aligned. */
int qail_qbc_loss(const float* logits_q, const float* logits_fp, int32_t B, int32_t D, float* loss,
                  float* grad_q, void* workspace, size_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* QAIL_H */
