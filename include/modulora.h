/*
 * modulora.h -- C ABI of the MI355X (gfx950) ModuLoRA linear-layer library.
 *
 * The layer (ModuLoRA, arXiv 2309.16119, Section 3.1 eq. (3) and Figure 1) is a
 * frozen low-precision base weight plus a high-precision low-rank adapter:
 *
 *     forward          Y  = X What^T + s (X A) B
 *     backward, input  dX = dY What  + s (dY B^T) A^T
 *     backward, LoRA   dA = s X^T (dY B^T),   dB = s (X A)^T dY
 *
 * What [d_out][d_in] is never stored in high precision.  It is re-materialized
 * tile by tile inside the kernels, in the forward and again in the backward pass
 * (Section 3.1.2: recompute instead of save), from b-bit codes with a per-group
 * scale and zero point (Section 2.2 eq. (2), in integer-zero-point form):
 *
 *     What[n][k] = bf16_rne( (q[n][k] - zeros[k/g][n]) * scales[k/g][n] )
 *
 * Naming: K = d_in, N = d_out, M = tokens, r = LoRA rank, g = group_size,
 * s = lora_scale (alpha / r).  The paper's adapter factors B, A^T are called
 * A [K][r] and B [r][N] here.
 *
 * General rules for every entry point
 *   - Every data pointer is a DEVICE pointer (HIP global memory) unless it says
 *     "host".  The caller owns all buffers; the library never allocates, frees or
 *     keeps device memory and holds no per-layer state.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Work is
 *     only enqueued on that stream; no call synchronizes with the host.
 *   - Inputs are read-only.  Outputs are fully overwritten unless stated.
 *   - Arguments are validated on the host before any HIP call, so every
 *     MODULORA_ERR_* below except MODULORA_ERR_HIP can be produced without a GPU.
 *     Nothing aborts and nothing throws across this boundary.
 *   - 16-bit floats travel as uint16_t bit patterns: X, dY, Y, dX, What are
 *     bfloat16; scales are IEEE binary16.
 *   - `workspace` is scratch device memory of at least modulora_workspace_bytes()
 *     bytes, 256-byte aligned, contents irrelevant on entry and undefined on exit.
 *     Two calls that share a workspace must be ordered on one stream.
 */
#ifndef MODULORA_H
#define MODULORA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MODULORA_OK = 0,
    MODULORA_ERR_NULL = 1,      /* a required pointer is NULL                          */
    MODULORA_ERR_SHAPE = 2,     /* d_in / d_out / M out of range or not divisible      */
    MODULORA_ERR_BITS = 3,      /* bits not in {2, 3, 4}                               */
    MODULORA_ERR_GROUP = 4,     /* group_size not a multiple of 32 dividing d_in       */
    MODULORA_ERR_ALIGN = 5,     /* a pointer is not 16-byte aligned                    */
    MODULORA_ERR_RANK = 6,      /* r < 0, r > 64, or r > 0 with A or B NULL            */
    MODULORA_ERR_WORKSPACE = 7, /* workspace NULL, misaligned or too small             */
    MODULORA_ERR_HIP = 8,       /* a HIP call failed (launch error, wrong device, ...) */
    MODULORA_ERR_HYPER = 9      /* optimizer step or hyper-parameter out of range      */
} modulora_status;

/*
 * The frozen quantized base weight of one linear layer (Section 2.2 eq. (2): codes,
 * zeros and scales as produced by a black-box quantizer).  All pointers are device
 * pointers, borrowed for the duration of a call, never written.
 *
 *   qweight [d_in*bits/32][d_out] uint32, d_out contiguous.  The codes of output
 *           column n form one bitstream along d_in: code k occupies stream bits
 *           [k*bits, k*bits+bits); stream bit j is bit (j mod 32), LSB = bit 0, of
 *           word qweight[j / 32][n].  (3-bit: 32 codes per 3 words; codes 10 and 21
 *           of each 32 straddle a word boundary.)
 *   scales  [d_in/group_size][d_out] binary16 bit patterns (finite, normal).
 *   zeros   [d_in/group_size][d_out] uint8 integer zero points, used as stored.
 *
 * Requirements: bits in {2,3,4}; group_size a multiple of 32 that divides d_in
 * (group_size == d_in is the one-scale-per-row case of the paper); d_out a
 * multiple of 8; 32 <= d_in, 8 <= d_out, both <= 2^20.
 */
typedef struct {
    int32_t d_in;
    int32_t d_out;
    int32_t bits;
    int32_t group_size;
    const uint32_t *qweight;
    const uint16_t *scales;
    const uint8_t *zeros;
} modulora_qweight;

/* Human-readable name of a status code (static storage, host pointer). */
const char *modulora_status_string(int status);

/*
 * Bytes of workspace that modulora_fwd / modulora_bwd_input / modulora_bwd_lora need
 * for this layer at M tokens and rank r (the maximum over the three).  Returns 0 when
 * the arguments are invalid.  Never touches the GPU.
 */
size_t modulora_workspace_bytes(const modulora_qweight *w, int32_t M, int32_t r);

/*
 * Test-only: materialize the whole weight, What[n][k] as defined above, into
 * What_bf16 [d_out][d_in] (bfloat16 bits, d_in contiguous).  This is the weight
 * materialization step of Figure 1 (LPLinear.forward, before the product); the product
 * path never calls it -- it exists so that unpacking and dequantization can be
 * checked bit for bit.
 */
int modulora_dequant(const modulora_qweight *w, uint16_t *What_bf16, void *stream);

/*
 * Forward (Section 3.1 eq. (3), Figure 1 ModuLoRALinear.forward, without bias):
 *     Y[m][n] = sum_k X[m][k] What[n][k] + lora_scale * sum_j XA[m][j] B[j][n],
 *     XA = X A.
 *   X  [M][d_in] bfloat16          A [d_in][r] float32      B [r][d_out] float32
 *   Y  [M][d_out] bfloat16 (out)   XA [M][r] float32 (out, may be NULL)
 * r == 0 (A, B ignored) is the plain low-precision linear map LPLinear.forward.
 * fp32 accumulation; one round-to-nearest-even to bfloat16 at the end.
 * Arithmetic by token count.  Normally What is materialized tile by tile exactly as defined
 * above (rounded to bfloat16) and multiplied.  A handful of tokens -- M <= 16, or M <= 32 over a
 * weight of at least 4 MiB of codes (done as two passes of at most 16 rows) -- take, when the
 * shape allows (d_in a multiple of 128, group_size a multiple of 32 / 64 / 128 for 4 / 2 / 3
 * bits), the direct product with the quantized matrix of Section 3.1.2: the codes are multiplied
 * as they are and scale and zero point are applied to per-group sums, so What is NOT rounded to
 * bfloat16 first.  The result then differs from the materialized form by at most
 * 2^-8 sum_k |X[m][k]| |What[n][k]| (closer to the exact product); the same input row can
 * therefore give results that differ by this much on either side of that token count.
 */
int modulora_fwd(const modulora_qweight *w, const uint16_t *X, int32_t M,
                 const float *A, const float *B, int32_t r, float lora_scale,
                 uint16_t *Y, float *XA,
                 void *workspace, size_t workspace_bytes, void *stream);

/*
 * modulora_fwd for callers that cannot provide scratch memory or allocate any: code that runs
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, results (bit for bit) and error codes as modulora_fwd, minus the workspace: the
 * scratch is a static device array of MODULORA_STATIC_SCRATCH_BYTES inside the library (each GPU
 * the library runs on holds its own copy from the first call on that GPU until the process
 * ends).  The call allocates and frees nothing, on the host side of the GPU or through any
 * library.  A layer / M / r whose forward pass needs more scratch than that returns
 * MODULORA_ERR_WORKSPACE (the streaming passes for a handful of tokens need < 8 MiB at every benchmark layer; the
 * tile kernels need about 2 (M + d_out) (3 r + 16) bytes; partial tiles of a split last round of
 * 256 x 256 tiles are used only when they also fit, otherwise those tiles run whole).
 * All calls on one GPU share that GPU's array and it keeps the last call's contents (nothing in
 * it needs clearing: every region is written before it is read): two calls that overlap in
 * time on one GPU -- different streams, or different host threads -- race; order them on one
 * stream.  The first call on a GPU looks the array's address up (hipGetSymbolAddress) and must
 * not be made while a graph is being captured; later calls may be.
 */
#define MODULORA_STATIC_SCRATCH_BYTES (16u << 20)
int modulora_fwd_static(const modulora_qweight *w, const uint16_t *X, int32_t M,
                        const float *A, const float *B, int32_t r, float lora_scale,
                        uint16_t *Y, float *XA, void *stream);

/*
 * Backward with respect to the input (Figure 1 LPLinear.backward: the weight is
 * re-materialized, grad_input = grad_output What; plus the adapter path of
 * Section 3.1.1, d y~/d y = What^T + B A^T in the paper's naming):
 *     dX[m][k] = sum_n dY[m][n] What[n][k] + lora_scale * sum_j dYBt[m][j] A[k][j],
 *     dYBt = dY B^T.
 *   dY [M][d_out] bfloat16          dX [M][d_in] bfloat16 (out)
 *   dYBt [M][r] float32 (out, may be NULL)
 * No gradient flows to qweight, scales or zeros.
 * Arithmetic by token count, as for modulora_fwd: for the same handful of tokens (when d_out is
 * a multiple of 128, d_in a multiple of 128 and group_size 64 or a multiple of 128) the codes are
 * multiplied directly and the scaled
 * activation dY[m][n] * scales[g][n] is rounded to bfloat16 before the product; the result
 * differs from the materialized form by at most 2^-7 sum_n |dY[m][n]| |What[n][k]|.
 */
int modulora_bwd_input(const modulora_qweight *w, const uint16_t *dY, int32_t M,
                       const float *A, const float *B, int32_t r, float lora_scale,
                       uint16_t *dX, float *dYBt,
                       void *workspace, size_t workspace_bytes, void *stream);

/*
 * Adapter gradients (Section 3.1.1: they do not involve the quantized weight):
 *     dA[k][j] = lora_scale * sum_m X[m][k] dYBt[m][j]
 *     dB[j][n] = lora_scale * sum_m XA[m][j] dY[m][n]
 *   XA, dYBt [M][r] float32: the hand-offs written by modulora_fwd and
 *       modulora_bwd_input; either may be NULL and is then recomputed here from
 *       (X, A) or (dY, B).
 *   dA [d_in][r], dB [r][d_out] float32.  accumulate == 0 overwrites them,
 *       accumulate != 0 adds to their current contents (gradient accumulation over
 *       micro-batches).  The reduction over tokens adds per-chunk partial sums in a
 *       fixed order (no atomics): results are identical from run to run.
 * r must be >= 1.
 */
int modulora_bwd_lora(int32_t d_in, int32_t d_out, int32_t M, int32_t r, float lora_scale,
                      const uint16_t *X, const uint16_t *dY, const float *A, const float *B,
                      const float *XA, const float *dYBt,
                      float *dA, float *dB, int32_t accumulate,
                      void *workspace, size_t workspace_bytes, void *stream);

/*
 * Round-to-nearest group quantizer and packer (the quantizer Q of Section 2.2 in its
 * simplest form, the round-to-nearest baseline of the paper's quantizer ablation): turns a
 * float32 weight into the modulora_qweight storage format.
 *   W [d_out][d_in] float32 device pointer, d_in contiguous (finite values; per group,
 *     (max - min) / (2^bits - 1) must not exceed 65504, the largest binary16).
 *   qweight, scales, zeros: device output buffers of the shapes given at
 *     modulora_qweight, fully overwritten.
 * Per group of group_size inputs of an output column, all in IEEE float32 with round
 * half to even (so the result is defined bit for bit):
 *     lo = min(group, 0),  hi = max(group, 0)
 *     scale = the smallest binary16 >= max((hi - lo) / (2^bits - 1), 2^-14)
 *     zero  = clamp(rne(-lo / scale), 0, 2^bits - 1)
 *     q     = clamp(rne(w / scale) + zero, 0, 2^bits - 1)
 * which gives |w - (q - zero) scale| <= scale (1/2 + 2^-20).
 * Same shape requirements and error codes as a modulora_qweight; needs no workspace.
 */
int modulora_quantize_rtn(const float *W, int32_t d_in, int32_t d_out, int32_t bits, int32_t group_size,
                          uint32_t *qweight, uint16_t *scales, uint8_t *zeros, void *stream);

/*
 * One AdamW step on a flat float32 buffer, in place (the optimizer the paper trains the
 * adapter factors with, Appendix hyper-parameter tables; Adam with decoupled weight
 * decay, the decay scaled by the learning rate):
 *     m <- beta1 m + (1 - beta1) g            v <- beta2 v + (1 - beta2) g^2
 *     p <- p (1 - lr weight_decay) - lr (m / (1 - beta1^step)) / (sqrt(v / (1 - beta2^step)) + eps)
 * Meant for all adapter factors of a model (or of a layer) laid out back to back in
 * one allocation, so that one launch updates them all.
 *   param, exp_avg (m), exp_avg_sq (v)  [n] float32 device pointers, updated in place.
 *   grad                                [n] float32 device pointer, read only.
 *   step >= 1 is the number of this update (1 for the first).
 * fp32 arithmetic throughout; beta^step is evaluated on the host in double.
 * Errors: MODULORA_ERR_NULL, MODULORA_ERR_ALIGN (16-byte), MODULORA_ERR_SHAPE (n == 0),
 * MODULORA_ERR_HYPER (step < 1, lr < 0, beta outside [0, 1), eps <= 0, weight_decay < 0,
 * or a non-finite value).  Needs no workspace.
 */
int modulora_adamw(float *param, const float *grad, float *exp_avg, float *exp_avg_sq, size_t n,
                   float lr, float beta1, float beta2, float eps, float weight_decay, int32_t step,
                   void *stream);

/* ------------------------------------------------------------------------------------
 * The layer in the paper's own storage convention (Section 2.2 eq. (2): What = s (.) Wq + z
 * with a FLOATING zero point z; Section 3.2: z, s and the materialized What in a 16-bit
 * float; Figure 1 / eq. (3): a bias on the adapted layer):
 *
 *     What[n][k] = binary16( binary32( q[n][k] * scales[g][n] + zeros[g][n] ) ),  g = k / group_size
 *     Y  = X What^T + bias + lora_scale (X A) B
 *     dX = dY What + lora_scale (dY B^T) A^T         dA, dB as in modulora_bwd_lora
 *
 * q: the same LSB-first bitstream as modulora_qweight.qweight.  scales, zeros: IEEE binary16 bit
 * patterns, [d_in / group_size][d_out]; the zero point is ADDED (eq. (2)); group_size = d_in is
 * the paper's one (scale, zero) pair per output row.  The affine value is rounded once to binary32
 * (a fused multiply-add) and then to nearest even to binary16; finite, normal-or-zero scales and
 * zero points are the contract.  bias: binary16 [d_out] or NULL; it enters the forward pass only
 * (Figure 1: the frozen parts get no gradient).  X, dY, Y, dX: binary16 bit patterns, row-major.
 * A, B, XA, dYBt, dA, dB: float32 as in the calls above.  All pointers are DEVICE pointers,
 * borrowed, 16-byte aligned; the workspace is the caller's (256-byte aligned, at least
 * modulora_f16_workspace_bytes()).  Shape rules, rank rules, the stream argument, ownership and
 * error behaviour are those of the calls above: every argument error is found on the host
 * before any HIP call and returned as a modulora_status; nothing is allocated or synchronized.
 * Arithmetic by token count, as for modulora_fwd / modulora_bwd_input: for a handful of tokens
 * (same token counts, same shape conditions) the codes are multiplied directly (Section 3.1.2) and scale and zero point are
 * applied to per-group sums, so What is not rounded to binary16 first; forward results differ from
 * the materialized form by at most 2^-11 sum_k |X| |What|, input gradients (where dY * scale is
 * rounded to binary16) by at most 2^-10 sum_n |dY| |What|.
 * ------------------------------------------------------------------------------------ */
typedef struct {
    int32_t d_in;
    int32_t d_out;
    int32_t bits;              /* 2, 3 or 4 */
    int32_t group_size;        /* multiple of 32 that divides d_in */
    const uint32_t *qweight;   /* [d_in * bits / 32][d_out] */
    const uint16_t *scales;    /* binary16 [d_in / group_size][d_out] */
    const uint16_t *zeros;     /* binary16 [d_in / group_size][d_out], added */
    const uint16_t *bias;      /* binary16 [d_out], or NULL */
} modulora_qweight_f16;

/* Bytes of workspace the three calls below need for (w, M, r); 0 for invalid shapes. */
size_t modulora_f16_workspace_bytes(const modulora_qweight_f16 *w, int32_t M, int32_t r);

/* Testing only: What as binary16 bit patterns, [d_out][d_in] (eq. (2), rounding as above). */
int modulora_f16_dequant(const modulora_qweight_f16 *w, uint16_t *What_f16, void *stream);

/* Forward pass of Figure 1 (eq. (3)).  Y [M][d_out] binary16 is overwritten; XA [M][r] (may be
 * NULL) receives X A.  r == 0 is the plain low-precision linear layer (A, B ignored). */
int modulora_f16_fwd(const modulora_qweight_f16 *w, const uint16_t *X, int32_t M,
                     const float *A, const float *B, int32_t r, float lora_scale,
                     uint16_t *Y, float *XA,
                     void *workspace, size_t workspace_bytes, void *stream);

/* Input gradient (Figure 1, LPLinear.backward: What is re-materialized, Section 3.1.1).
 * dX [M][d_in] binary16 is overwritten; dYBt [M][r] (may be NULL) receives dY B^T. */
int modulora_f16_bwd_input(const modulora_qweight_f16 *w, const uint16_t *dY, int32_t M,
                           const float *A, const float *B, int32_t r, float lora_scale,
                           uint16_t *dX, float *dYBt,
                           void *workspace, size_t workspace_bytes, void *stream);

/* Adapter gradients (Section 3.1.1) from binary16 X and dY; arguments as modulora_bwd_lora. */
int modulora_f16_bwd_lora(int32_t d_in, int32_t d_out, int32_t M, int32_t r, float lora_scale,
                          const uint16_t *X, const uint16_t *dY, const float *A, const float *B,
                          const float *XA, const float *dYBt,
                          float *dA, float *dB, int32_t accumulate,
                          void *workspace, size_t workspace_bytes, void *stream);

/*
 * Per-kernel timing for benchmarks and tests (no operation of the paper).  Between
 * modulora_profile_begin() and modulora_profile_end() every kernel the library launches is
 * bracketed by a fresh pair of HIP events on the stream it is launched on.
 * modulora_profile_end() waits for those events (it synchronizes with the device -- the only
 * call that does), writes one record per distinct kernel name into `out` (host memory, at most
 * `capacity` records) and stores the number of records in *count.  While profiling is active
 * the launch path creates events, so calls made then must NOT be recorded into a HIP graph.
 * Not thread-safe; not for production use.
 */
typedef struct {
    char name[64];      /* kernel family and tile variant, NUL-terminated */
    int32_t launches;   /* launches seen since modulora_profile_begin()   */
    float total_ms;     /* sum of their durations in milliseconds         */
} modulora_kernel_time;

int modulora_profile_begin(void);
int modulora_profile_end(modulora_kernel_time *out, int32_t capacity, int32_t *count);

/*
 * Benchmark hook (no operation of the paper): one plain streaming read of `bytes` bytes of device
 * memory at `buf` (16-byte aligned, bytes a positive multiple of 16) by a hand-written kernel
 * with 16-byte non-temporal loads -- the measured read rate that the packed-weight GB/s of the
 * M <= 16 streaming kernels is reported beside.  `sink` is a device buffer of
 * MODULORA_BENCH_READ_SINK_WORDS uint32 that receives one checksum word per workgroup (so the
 * reads cannot be optimized away).  Enqueued on `stream`; timed by the caller or through
 * modulora_profile_begin/_end under the name "bench_read".
 * Errors: MODULORA_ERR_NULL, MODULORA_ERR_ALIGN, MODULORA_ERR_SHAPE, MODULORA_ERR_HIP.
 */
#define MODULORA_BENCH_READ_SINK_WORDS 2048
int modulora_bench_read(const void *buf, size_t bytes, uint32_t *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* MODULORA_H */
