/*
 * libunit -- mixed-precision conv2d / matmul on MI355X (gfx950) MFMA units.
 *
 * The operations are the ones the UNIT paper compiles tensorized instructions
 * for: dense tensor operations whose low-precision elementwise products are
 * reduced "horizontally" into one high-precision accumulator (Section I;
 * Section II-A).  int8 x int8 accumulates in int32, fp16 x fp16 accumulates in
 * fp32 (Section III-A).
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller.  The library
 *     never allocates, frees or keeps them.  Scratch comes from the caller's
 *     workspace `ws` (device memory, 256-byte aligned, at least as large as the
 *     matching *_workspace query).
 *   - `stream` is a hipStream_t passed as void* (NULL = default stream).  Calls
 *     enqueue work on it and return without synchronising.
 *   - fp16 tensors travel as uint16_t IEEE binary16 bit patterns.
 *   - Return value: UNIT_OK (0) or a negative unit_status.  Argument errors are
 *     detected on the host before anything is launched.
 *   - Concurrent calls are safe if their outputs and workspaces do not overlap.
 *   - Size limits, all reported as UNIT_ENOTSUP before anything is launched: every tensor of a
 *     conv call (activations, packed activations, weights, output) and every 256-row band of a
 *     matmul operand must be smaller than 2 GiB (the kernels address them through 32-bit buffer
 *     offsets), and the batch n of a conv or pack call must be at most 65535.
 */
#ifndef UNIT_H
#define UNIT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum unit_status {
    UNIT_OK         =  0,
    UNIT_EINVAL     = -1,   /* NULL pointer, non-positive dimension, empty output, misalignment */
    UNIT_ENOTSUP    = -2,   /* shape outside what the kernels cover                             */
    UNIT_EOVERFLOW  = -3,   /* byte reduction longer than UNIT_MAX_REDUCTION_*: int32 sum not
                               provably exact                                                   */
    UNIT_EWORKSPACE = -4,   /* workspace NULL or too small                                      */
    UNIT_EHIP       = -5,   /* a HIP runtime call or kernel launch failed                       */
    UNIT_ESCRATCH   = -6    /* *_static entry point: the problem needs more scratch than
                               UNIT_STATIC_SCRATCH_BYTES                                        */
};

/* Operand types: i8 x i8 -> i32, f16 x f16 -> f32, bf16 x bf16 -> f32, u8 x i8 -> i32
 * (unsigned activations / matmul A, signed weights / matmul B: the operand types of the
 * byte dot-product instruction of Section III-A), fp8 x fp8 -> f32 (OCP E4M3, finite-only). */
enum unit_dtype { UNIT_I8 = 0, UNIT_F16 = 1, UNIT_BF16 = 2, UNIT_U8I8 = 3, UNIT_FP8 = 4 };

/* Longest int8 reduction (c*r*s, or k for matmul) with |sum| <= len * 2^14 < 2^31. */
#define UNIT_MAX_REDUCTION_I8 131071
/* Same for u8 x i8: |sum| <= len * 255 * 128 < 2^31. */
#define UNIT_MAX_REDUCTION_U8I8 65793

/*
 * conv2d problem (Section III-C.2 index forms: c[x,y,k] += a[x+r,y+s,rc]*b[r,s,k,rc]):
 * cross-correlation with zero padding, dilation 1, groups 1.
 *   x: [n,c,h,w] (NCHW)    w: [k,c,r,s] (OIHW)    y: [n,k,p,q]
 *   p = floor((h + 2*pad_h - r)/stride_h) + 1,  q likewise.
 */
typedef struct unit_conv2d_desc {
    int32_t n, c, h, w;
    int32_t k, r, s;
    int32_t stride_h, stride_w, pad_h, pad_w;
} unit_conv2d_desc;

/*
 * Fused epilogue back to int8 (the quantised-inference use the paper targets,
 * Section II-A, Section V-C):
 *   t = acc + bias[k] + residual[n,k,p,q] + residual_mult * residual_packed[n,p,q,k]
 *                                                    (int32; caller keeps |t| < 2^31)
 *   g = (float)t * scale[k]                          (RNE conversion, one fp32 multiply)
 *   i = round-half-to-even(g); if relu: i = max(i,0); clamp to [-128,127]
 * The packed residual is the skip connection of a quantised residual block taken straight
 * from the int8 activations an earlier layer wrote (y_packed layout of this layer's output,
 * 16-byte aligned), rescaled by an integer; either residual form may be NULL, both may be given.
 */
typedef struct unit_requant {
    const float   *scale;            /* device [k]; finite                              */
    const int32_t *bias;             /* device [k] or NULL                              */
    const int32_t *residual;         /* device [n,k,p,q] int32 (NCHW) or NULL           */
    int32_t        relu;             /* 0 or 1                                          */
    int32_t        residual_mult;    /* multiplier of residual_packed                   */
    const void    *residual_packed;  /* device [n][p][q][kp] int8, kp = k rounded up to
                                        16, or NULL                                     */
} unit_requant;

/* Tile choice made by the selector for one problem (introspection / reports). */
typedef struct unit_tile_info {
    int32_t block_m, block_n;   /* workgroup tile: block_m output rows (out channels / matmul m),
                                   block_n output columns (pixels / matmul n)                      */
    int32_t block_k_bytes;      /* reduction bytes staged per main-loop step                       */
    int32_t waves_m, waves_n, waves_k;  /* wave grid inside the workgroup (waves_k = in-group split) */
    int32_t mfma;               /* 32 or 16: MFMA tile edge; 0: a matmul of at most 4 rows (int8, fp16)
                                   runs on the vector ALU's dot-product instructions instead, one
                                   wave per output column, block_n columns per workgroup            */
    int32_t split_k;            /* number of workgroups sharing one output tile (grid split)       */
    int32_t workgroups;         /* launched with this tile                                         */
    /* A large problem whose count of 256 x 256 tiles would leave the last round of workgroups partly
     * empty runs as two launches: whole rounds of the tile above over the first columns, then the
     * remaining columns with a narrower tile (256 x tail_block_n) that fits them into one round.   */
    int32_t tail_block_n;       /* 0: one launch                                                   */
    int32_t tail_workgroups;
    int32_t tail_first_col;     /* first output column (pixel index / matmul n) of the second launch */
} unit_tile_info;

int         unit_version(void);
const char *unit_status_str(int status);
/* Text of the last HIP error seen by this thread ("" if none). */
const char *unit_last_hip_error(void);

/* ------------------------------------------------------------------ queries (host only) */

/* Output extent; UNIT_EINVAL if any dimension is non-positive or the output is empty. */
int unit_conv2d_out_dims(const unit_conv2d_desc *d, int32_t *p, int32_t *q);

/* Bytes of the internal layouts (both multiples of 256):
 *   activations  [n][h][w][cp]       cp = c rounded up to 16 bytes of channels
 *   weights      [k][r][s][cp]       reduction-contiguous per output channel            */
size_t unit_packed_act_bytes(int32_t n, int32_t c, int32_t h, int32_t w, int dtype);
size_t unit_packed_weights_bytes(const unit_conv2d_desc *d, int dtype);

/* Workspace needed by unit_conv2d_{i8,f16} (packs both operands internally) and by
 * unit_conv2d_packed_* (split-K partial sums only; may be 0).  0 on invalid input. */
size_t unit_conv2d_workspace(const unit_conv2d_desc *d, int dtype);
size_t unit_conv2d_packed_workspace(const unit_conv2d_desc *d, int dtype);
size_t unit_matmul_workspace(int32_t m, int32_t n, int32_t k, int64_t lda, int64_t ldb, int dtype);

/* What the selector picks (the paper's tuner, Section III-C.3 and the GPU tuning paragraphs of
 * Section IV-C: register window, fused spatial dims, split reduction).  conv: rows = k, cols = n*p*q, kbytes = r*s*cp. */
int unit_select_conv2d(const unit_conv2d_desc *d, int dtype, unit_tile_info *out);
int unit_select_matmul(int32_t m, int32_t n, int32_t k, int dtype, unit_tile_info *out);
/* unit_select_conv2d reports the choice for packed activations (unit_conv2d_packed_*, or a wpacked
 * call that packs first).  The direct input modes may take another tile or grid split (their steps
 * cost differently): this variant reports the choice for the given unit_input_mode, whether or not
 * the problem qualifies for it (ask unit_conv2d_input_mode).  UNIT_EINVAL for an unknown mode. */
int unit_select_conv2d_input(const unit_conv2d_desc *d, int dtype, int input_mode, unit_tile_info *out);

/*
 * Measurement aid: the rate the matrix units sustain on register-resident operands.  The paper judges
 * its kernels by whether they keep the matrix units busy (Section VI-B); on this chip the clock of a
 * busy matrix pipe is set by power management and depends on the operands' switching activity, so the
 * nominal peak is not what a kernel on the benchmark's uniformly random operands can reach.  The call
 * launches 256 workgroups of eight waves that execute `steps` steps of the large tile's MFMA sequence
 * (32 MFMA 32x32 per wave and step = 256 x 256 x 128 bytes of reduction per workgroup and step, as in
 * the 4096^3 matmul: 32 steps for int8, 64 for fp16) on operands held in registers: no LDS, no memory
 * traffic.  random_operands != 0 fills them with uniformly random bytes (fp16 / bf16: random signs and
 * mantissas); 0 with constants.  The caller times the launch (events on `stream`); work per launch =
 * 256 * 8 * steps * 32 MFMAs * 32*32*K MACs each (K = 32 bytes of reduction: 32 for int8, 16 for
 * 2-byte types).  `counters` (device, 8-byte aligned, UNIT_MEASURE_COUNTERS_BYTES) receives per wave four
 * uint64: core clock cycles and 100 MHz real-time ticks from the wave's first to its last instruction,
 * and its start and end tick; cycles / ticks * 100 MHz is the shader clock the wave saw.  (The two waves
 * of a SIMD do not share the pipe evenly: the older one runs at nearly the full rate first.)
 * dtype: UNIT_I8, UNIT_F16 or UNIT_BF16.  Errors: UNIT_EINVAL, UNIT_EWORKSPACE, UNIT_EHIP.
 */
#define UNIT_MEASURE_COUNTERS_BYTES (256 * 8 * 4 * 8)
int unit_measure_mfma(int dtype, int32_t steps, int32_t random_operands, void *counters, size_t counters_bytes,
                      void *stream);

/*
 * Test and tuning-sweep hook (the "enumerate and profile" loop of Section IV-C drives it; Section
 * VI-B's ablation is measured with it): every later call of this process uses compiled tile `tile`
 * (0 .. 12, see unit_tile_info of a query for what it is) instead of the selector's choice, and
 * `split_k` workgroups per output tile (clipped to the reduction's steps).  A negative tile and a
 * split_k < 1 restore the rule for that half.  Process-wide and not synchronised with calls in
 * flight on other threads: not for production code.  A forced tile that has no kernel for a
 * call's input mode makes the call fall back to packed activations, or fail with UNIT_ENOTSUP.
 * Returns UNIT_EINVAL for a tile index that does not exist.
 */
int unit_debug_force_tile(int32_t tile, int32_t split_k);

/*
 * How unit_conv2d_wpacked_* (and unit_conv2d_*) will read the NCHW activations `x` of this
 * problem when no requantise epilogue is requested (introspection / reports; nothing is launched):
 *   UNIT_INPUT_PACKED          pack_act into the workspace, then the gather kernel
 *   UNIT_INPUT_DIRECT          1x1 stride-1 unpadded conv (any batch, any image size): the main
 *                              kernel reads NCHW itself (no pack_act launch)
 *   UNIT_INPUT_DIRECT_SHIFTED  stride 1, output grid equal to the input grid ("same" padding, any
 *                              window), whole reduction steps inside one tap, and a layer small
 *                              enough to be launch-bound (one image, or a few small ones): the main
 *                              kernel reads per-tap shifted windows of the NCHW channel rows, any
 *                              row alignment (no pack_act launch)
 * Returns the mode (>= 0) or a negative unit_status.
 */
enum unit_input_mode { UNIT_INPUT_PACKED = 0, UNIT_INPUT_DIRECT = 1, UNIT_INPUT_DIRECT_SHIFTED = 2 };
int unit_conv2d_input_mode(const unit_conv2d_desc *d, int dtype, const void *x);

/* ------------------------------------------------------------------ plain-layout calls */

/*
 * int8 conv2d.  x: NCHW int8, w: OIHW int8.
 *   rq == NULL : y_i32 (NKPQ int32) receives the raw accumulators; y_i8 must be NULL.
 *   rq != NULL : y_i8 (NKPQ int8) receives the requantised result; y_i32 may also be
 *                given to receive the raw accumulators (before bias/residual).
 * Errors: UNIT_EINVAL, UNIT_EOVERFLOW (c*r*s > UNIT_MAX_REDUCTION_I8), UNIT_EWORKSPACE, UNIT_EHIP.
 */
int unit_conv2d_i8(const unit_conv2d_desc *d, const int8_t *x, const int8_t *w,
                   int32_t *y_i32, const unit_requant *rq, int8_t *y_i8,
                   void *ws, size_t ws_bytes, void *stream);

/* fp16 conv2d with fp32 accumulation.  x: NCHW, w: OIHW (binary16 bits), y: NKPQ float. */
int unit_conv2d_f16(const unit_conv2d_desc *d, const uint16_t *x, const uint16_t *w,
                    float *y, void *ws, size_t ws_bytes, void *stream);

/*
 * C[m,n] = sum_k A[m,k] * B[k,n].   A row-major (A[m,k] at A[m*lda+k]), B column-major
 * (B[k,n] at B[n*ldb+k]), C row-major (C[m*ldc+n]); leading dimensions in elements,
 * lda,ldb >= k, ldc >= n.  An operand whose leading dimension or k (in bytes) is not a
 * multiple of 16 is first copied into the workspace with zero padding
 * (unit_matmul_workspace accounts for it); an operand used in place must start on a
 * 16-byte boundary (UNIT_EINVAL otherwise).  C must be 4-byte aligned.  A reduction split
 * across workgroups is only used when ldc == n.
 * Errors: UNIT_EINVAL, UNIT_EOVERFLOW (int8, k > UNIT_MAX_REDUCTION_I8), UNIT_EWORKSPACE, UNIT_EHIP.
 */
int unit_matmul_i8(int32_t m, int32_t n, int32_t k,
                   const int8_t *A, int64_t lda, const int8_t *B, int64_t ldb,
                   int32_t *C, int64_t ldc, void *ws, size_t ws_bytes, void *stream);
int unit_matmul_f16(int32_t m, int32_t n, int32_t k,
                    const uint16_t *A, int64_t lda, const uint16_t *B, int64_t ldb,
                    float *C, int64_t ldc, void *ws, size_t ws_bytes, void *stream);

/* ------------------------------------------------------------------ packed (steady-state) calls
 * The paper converts layouts once at graph level and keeps activations in the blocked
 * layout between layers (Section V-C; Section II-C.1 on tensor padding).  These calls
 * expose that: weights are packed once, activations stay packed from layer to layer.  */

int unit_pack_act_i8 (int32_t n, int32_t c, int32_t h, int32_t w, const int8_t *x_nchw,
                      void *x_packed, size_t packed_bytes, void *stream);
int unit_pack_act_f16(int32_t n, int32_t c, int32_t h, int32_t w, const uint16_t *x_nchw,
                      void *x_packed, size_t packed_bytes, void *stream);
int unit_pack_weights_i8 (const unit_conv2d_desc *d, const int8_t *w_oihw,
                          void *w_packed, size_t packed_bytes, void *stream);
int unit_pack_weights_f16(const unit_conv2d_desc *d, const uint16_t *w_oihw,
                          void *w_packed, size_t packed_bytes, void *stream);
/* Packed int8 activations [n][h][w][cp] back to NCHW (for inspection / tests). */
int unit_unpack_act_i8(int32_t n, int32_t c, int32_t h, int32_t w, const void *x_packed,
                       int8_t *x_nchw, void *stream);

/*
 * conv2d on packed operands.  Outputs (any subset, at least one):
 *   y_i32    NKPQ int32 raw accumulators
 *   y_i8     NKPQ int8 requantised            (needs rq)
 *   y_packed [n][p][q][kp] int8 requantised, kp = k rounded up to 16: the next layer's
 *            packed input; its padding channels are written as 0   (needs rq)
 * x_packed, w_packed and y_packed must be 16-byte aligned (UNIT_EINVAL otherwise): packed
 * operands are read in 16-byte chunks and y_packed is written four channels per store.
 */
int unit_conv2d_packed_i8(const unit_conv2d_desc *d, const void *x_packed, const void *w_packed,
                          int32_t *y_i32, const unit_requant *rq, int8_t *y_i8, void *y_packed,
                          void *ws, size_t ws_bytes, void *stream);
int unit_conv2d_packed_f16(const unit_conv2d_desc *d, const void *x_packed, const void *w_packed,
                           float *y, void *ws, size_t ws_bytes, void *stream);

/*
 * conv2d on plain NCHW activations with pre-packed weights: the per-layer call of an
 * inference loop whose weights were packed once.  Activations are packed into the workspace
 * first, except where the main kernel can read NCHW itself (16-byte aligned x, no requantise;
 * see unit_conv2d_input_mode): 1x1 / stride-1 / unpadded convs of any batch and image size, and
 * small stride-1 "same"-padded convs (one image, or a few small ones).  Outputs as in unit_conv2d_i8 /
 * unit_conv2d_f16.
 */
size_t unit_conv2d_wpacked_workspace(const unit_conv2d_desc *d, int dtype);
int unit_conv2d_wpacked_i8(const unit_conv2d_desc *d, const int8_t *x, const void *w_packed,
                           int32_t *y_i32, const unit_requant *rq, int8_t *y_i8,
                           void *ws, size_t ws_bytes, void *stream);
int unit_conv2d_wpacked_f16(const unit_conv2d_desc *d, const uint16_t *x, const void *w_packed,
                            float *y, void *ws, size_t ws_bytes, void *stream);

/*
 * unit_conv2d_wpacked_i8 for callers that cannot allocate device memory or carry a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments without `ws`: the scratch the call needs (packed activations of the layers that are
 * packed first, partial sums of a reduction split across workgroups; what
 * unit_conv2d_wpacked_workspace reports) lives in a buffer of UNIT_STATIC_SCRATCH_BYTES inside the
 * library's device code, one copy per GPU, held until the process ends.  The call makes no
 * allocating HIP call; its first use on a device looks up that device's copy of the buffer.
 * A problem that needs more scratch is refused with UNIT_ESCRATCH before anything is launched
 * (every layer of the ResNet-50- and ResNet-18-shaped sets fits up to batch 16).  All calls on one
 * GPU share the buffer: calls that overlap in time on one GPU (two streams, two threads) race and
 * must be serialised by the caller; consecutive calls on one stream are safe.  Results are
 * identical to unit_conv2d_wpacked_i8's.  Other errors as for that call.
 */
#define UNIT_STATIC_SCRATCH_BYTES (16u << 20)
int unit_conv2d_wpacked_i8_static(const unit_conv2d_desc *d, const int8_t *x, const void *w_packed,
                                  int32_t *y_i32, const unit_requant *rq, int8_t *y_i8, void *stream);

/* ------------------------------------------------------------------ conv3d
 * The paper's extensibility experiment (Section VI-C, "3D Convolution"): the same path with one
 * more spatial axis.  x: [n,c,d,h,w] (NCDHW), w: [k,c,t,r,s], y: [n,k,o,p,q];
 * o = floor((d + 2*pad_d - t)/stride_d) + 1, p and q likewise; zero padding, dilation 1.
 * Raw int32 / fp32 outputs only.  Errors as for the 2-D calls.                                  */
typedef struct unit_conv3d_desc {
    int32_t n, c, d, h, w;
    int32_t k, t, r, s;
    int32_t stride_d, stride_h, stride_w, pad_d, pad_h, pad_w;
} unit_conv3d_desc;

int    unit_conv3d_out_dims(const unit_conv3d_desc *d, int32_t *o, int32_t *p, int32_t *q);
size_t unit_conv3d_workspace(const unit_conv3d_desc *d, int dtype);
int unit_conv3d_i8 (const unit_conv3d_desc *d, const int8_t *x, const int8_t *w, int32_t *y,
                    void *ws, size_t ws_bytes, void *stream);
int unit_conv3d_f16(const unit_conv3d_desc *d, const uint16_t *x, const uint16_t *w, float *y,
                    void *ws, size_t ws_bytes, void *stream);

/* ------------------------------------------------------------------ int8 network glue
 * Operators the chained int8 inference needs around the convolutions.  They work on the
 * packed int8 layout [n][h][w][cp].                                                        */

/* Max over a window; padded positions never win.  Output packed [n][p][q][cp]. */
int unit_maxpool_packed_i8(int32_t n, int32_t c, int32_t h, int32_t w,
                           int32_t window, int32_t stride, int32_t pad,
                           const void *x_packed, void *y_packed, void *stream);
/* int32 sum over h*w per (n,c), then the requantise rule with scale[c] (no ReLU).
 * Output: [n][cp] int8 (row-major, padding channels 0): the A operand of the FC matmul. */
int unit_global_avgpool_packed_i8(int32_t n, int32_t c, int32_t h, int32_t w,
                                  const void *x_packed, const float *scale,
                                  int8_t *y, void *stream);
/* residual[n,k,p,q] (int32 NCHW) = (int32)x_packed[n,p,q,k] * mult. */
int unit_widen_residual_i8(int32_t n, int32_t c, int32_t h, int32_t w,
                           const void *x_packed, int32_t mult, int32_t *residual, void *stream);

/* ------------------------------------------------------------------------------------------
 * Further operand types through the same kernels (Section I and Section III-A: the method is
 * meant to extend to other mixed-precision operand types; Section III-A's byte instruction
 * multiplies unsigned by signed bytes).  Same tensor conventions, workspace rules (query with
 * UNIT_BF16 / UNIT_U8I8 / UNIT_FP8) and error behaviour as unit_conv2d_f16 / unit_matmul_f16 and
 * unit_conv2d_i8 / unit_matmul_i8 without the requantise epilogue.
 *   bf16: uint16_t bfloat16 bit patterns, fp32 accumulation and output.
 *   u8i8: x / A unsigned bytes, w / B signed bytes, exact int32 output; reduction length at
 *         most UNIT_MAX_REDUCTION_U8I8 (UNIT_EOVERFLOW beyond).  The matrix unit multiplies
 *         signed bytes: the unsigned operand is fed as u - 128 and 128 * (sum of the signed
 *         operand over the reduction) is added back in the epilogue, which is exact.
 *   fp8:  uint8_t OCP E4M3 bit patterns (1 sign, 4 exponent bits with bias 7, 3 fraction bits,
 *         no infinities, NaN = S.1111.111), fp32 accumulation and output, no block scaling.
 */
int unit_conv2d_bf16(const unit_conv2d_desc *d, const uint16_t *x, const uint16_t *w,
                     float *y, void *ws, size_t ws_bytes, void *stream);
int unit_matmul_bf16(int32_t m, int32_t n, int32_t k, const uint16_t *A, int64_t lda,
                     const uint16_t *B, int64_t ldb, float *C, int64_t ldc,
                     void *ws, size_t ws_bytes, void *stream);
int unit_conv2d_u8i8(const unit_conv2d_desc *d, const uint8_t *x, const int8_t *w,
                     int32_t *y, void *ws, size_t ws_bytes, void *stream);
int unit_conv2d_fp8(const unit_conv2d_desc *d, const uint8_t *x, const uint8_t *w,
                    float *y, void *ws, size_t ws_bytes, void *stream);
int unit_matmul_fp8(int32_t m, int32_t n, int32_t k, const uint8_t *A, int64_t lda,
                    const uint8_t *B, int64_t ldb, float *C, int64_t ldc,
                    void *ws, size_t ws_bytes, void *stream);
int unit_matmul_u8i8(int32_t m, int32_t n, int32_t k, const uint8_t *A, int64_t lda,
                     const int8_t *B, int64_t ldb, int32_t *C, int64_t ldc,
                     void *ws, size_t ws_bytes, void *stream);

/* ------------------------------------------------------------------------------------------
 * Applicability inspection (Section III-B; Algorithm 1; candidate order of Section IV-A).
 * Host-only: no device work, no stream.  Decides whether a tensorized instruction, written as
 * a small tensor program, can execute a tile of a tensor operation, and which loops of the
 * operation become the instruction's loops.
 *
 * Program text (NUL-terminated; statements separated by ';' or newlines):
 *     loop NAME EXTENT dp|red        data-parallel / reduction loop, outermost first (<= 32)
 *     out  NAME:DTYPE[INDEX,...]     element written
 *     acc  NAME:DTYPE[INDEX,...]     instruction only: separate addend register (d = c + sum);
 *                                    without it the instruction accumulates in place (+=)
 *     body EXPR                      value reduced into the output
 *     EXPR  := (OPCODE EXPR EXPR) | (cast DTYPE EXPR) | NAME:DTYPE[INDEX,...] | const:DTYPE:VALUE
 *     INDEX := terms [COEF*]VAR or integers joined by + or -
 *
 * Step 1 (Algorithm 1): both expression trees are walked together; node types must agree
 * (a binary node has its left child's type, a cast its destination type), leaves bind an
 * instruction register element to one operation operand, arithmetic nodes need equal opcodes
 * and matching children, left with left.  Step 2 (Section III-B.2): each instruction loop takes
 * one operation loop of the same annotation such that, for every bound operand pair and for the
 * outputs, the image of the operation's index variables lies inside the instruction's index
 * variables; instruction loops missing from the image are broadcast directions.  Candidates are
 * tried innermost (last declared) first, the instruction's first loop varying slowest, and the
 * first feasible assignment is reported; num_feasible counts them all (the tuning dimension).
 *
 * Returns UNIT_OK with *res filled (applicable 0 or 1), UNIT_EINVAL for NULL arguments or text
 * that does not parse, UNIT_ENOTSUP for an instruction with more than UNIT_INSPECT_MAX loops or
 * register operands.
 */
#define UNIT_INSPECT_MAX  8
#define UNIT_INSPECT_NAME 16
typedef struct unit_inspect_result {
    int32_t  applicable;     /* 1: both steps succeed                                          */
    int32_t  failed_step;    /* 0 none, 1 expression trees differ, 2 no feasible loop mapping  */
    int32_t  num_loops;      /* instruction loops, declaration order                           */
    char     instr_loop[UNIT_INSPECT_MAX][UNIT_INSPECT_NAME];
    char     op_loop[UNIT_INSPECT_MAX][UNIT_INSPECT_NAME];     /* operation loop tiled onto it  */
    int32_t  num_operands;   /* instruction registers: output, addend, then body operands      */
    char     instr_operand[UNIT_INSPECT_MAX][UNIT_INSPECT_NAME];
    char     op_operand[UNIT_INSPECT_MAX][UNIT_INSPECT_NAME];  /* array bound to it or "const"  */
    uint32_t broadcast[UNIT_INSPECT_MAX];  /* bit i: replicated along instr_loop[i]             */
    int32_t  num_feasible;
} unit_inspect_result;

int unit_inspect(const char *instruction, const char *operation, unit_inspect_result *res);

/* Program text of what this library executes, for unit_inspect.  Each writes at most `cap`
 * bytes (NUL-terminated, truncated if short; buf may be NULL) and returns the bytes needed
 * including the NUL, or UNIT_EINVAL.
 *   unit_describe_mfma    one MFMA tile, edge 32 or 16 (Section III-A form: the instruction as
 *                         a tensor program; accumulates in place like the paper's matrix unit)
 *   unit_describe_conv2d  the conv on the layouts the main kernel reads
 *                         (weights [k][r][s][c], activations [n][h][w][c])
 *   unit_describe_matmul  C[m,n] += A[m,k] * B[k,n], B addressed column-major            */
int unit_describe_mfma(int dtype, int32_t edge, char *buf, size_t cap);
int unit_describe_conv2d(const unit_conv2d_desc *d, int dtype, char *buf, size_t cap);
int unit_describe_matmul(int32_t m, int32_t n, int32_t k, int dtype, char *buf, size_t cap);

#ifdef __cplusplus
}
#endif
#endif /* UNIT_H */
