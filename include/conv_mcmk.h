/*
 * conv_mcmk.h -- C ABI of libconv_mcmk: multi-channel multi-kernel (MCMK) 2-D
 * convolution on one AMD MI355X (gfx950), computed the kn2row way.
 *
 * The operation (paper Eq. 1-3): for every image n, kernel m and output
 * position (q, p)
 *
 *     O[n][m][q][p] = sum_c sum_i sum_j  I[n][c][s q - pad + i][s p - pad + j] * K[m][c][i][j]
 *
 * with terms whose input coordinate falls outside the image dropped (zero
 * padding) and no kernel flip.  The paper treats stride s = 1 (section II-A),
 * where Q = H + 2 pad - k + 1 rows and P = W + 2 pad - k + 1 columns; as a
 * generalisation the library also takes s > 1, the unit-stride result kept at
 * every s-th row and column: Q = floor((H + 2 pad - k) / s) + 1, P likewise.
 *
 * Conventions common to every entry point
 *   - All tensors are dense, row-major, in DEVICE memory, 16-byte aligned, and
 *     owned by the caller: I[N][C][H][W], K[M][C][k][k] (row tap i, then column
 *     tap j), O[N][M][Q][P].  N = 1 is the paper's un-batched call.
 *   - The library allocates nothing, never synchronises and launches only on the
 *     stream handed in (`stream` is a hipStream_t passed as void*; NULL = the
 *     default stream).  Results are ready when that stream reaches the end of
 *     the call's work.
 *   - O is completely overwritten.  I, K / Kp, O and the workspace must not overlap.
 *   - Every argument is validated before anything is launched; errors are
 *     return codes (CONV_MCMK_OK = 0), nothing throws or aborts.
 *   - dtype CONV_MCMK_F32: I, packed kernel and O are float.
 *     dtype CONV_MCMK_BF16: I and the packed kernel are bfloat16 (the upper 16
 *     bits of a float, rounded to nearest even), accumulation and O are float.
 *     (The bf16 variants that read I[N][C][H][W] need H*W >= 2 -- IM2COL: Q*P >= 2 --
 *     and refuse a single-element plane with CONV_MCMK_ERR_UNSUPPORTED.)
 */
#ifndef CONV_MCMK_H
#define CONV_MCMK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct conv_mcmk_desc {
    int32_t n;       /* images in the batch, >= 1 */
    int32_t c;       /* input channels, >= 1 */
    int32_t h, w;    /* input rows, columns, >= 1 */
    int32_t m;       /* kernels (output channels), >= 1 */
    int32_t k;       /* kernel side, >= 1 (square kernels) */
    int32_t pad;     /* zero padding on every side, >= 0 */
    int32_t stride;  /* >= 1; 1 is the paper's case (section II-A).  The fused variants take 1 and 2 */
    int32_t dtype;   /* CONV_MCMK_F32 or CONV_MCMK_BF16 */
} conv_mcmk_desc;

enum { CONV_MCMK_F32 = 0, CONV_MCMK_BF16 = 1 };

/* How the convolution is computed.  All four give the same O up to rounding order. */
enum {
    CONV_MCMK_KN2ROW       = 0, /* k*k 1x1 GEMMs on the unreplicated input, shift-add fused into the
                                   accumulators (section III-A without the k*k-sized product matrix) */
    CONV_MCMK_KN2ROW_2PASS = 1, /* section III-A as written: one GEMM [k*k*M x C].[C x HW] into the
                                   workspace, then the shift-add post pass */
    CONV_MCMK_IM2COL       = 2, /* section II-B: build the column matrix in the workspace, then one GEMM */
    CONV_MCMK_DIRECT       = 3, /* the loop nest of Eq. 1-3, one output element per thread, no matrix cores */
    CONV_MCMK_KN2COL       = 4, /* section III-A, last paragraph: kn2row with the channel innermost in the input
                                   and in the output (I[N][H][W][C], O[N][Q][P][M]); shift-add fused as in KN2ROW */
    CONV_MCMK_IM2ROW       = 5  /* section II-B, last paragraph: patches unrolled into rows of the workspace
                                   (channels last), then one GEMM patches x kernels; layouts as KN2COL */
};

enum {
    CONV_MCMK_OK              = 0,
    CONV_MCMK_ERR_NULL        = 1, /* a required pointer is NULL */
    CONV_MCMK_ERR_SHAPE       = 2, /* a dimension or the stride < 1, pad < 0, empty output, or a tensor too large (one image of 2^29 or more input elements -- for IM2COL / IM2ROW: patch-matrix elements --, 2^31 or more output elements) */
    CONV_MCMK_ERR_UNSUPPORTED = 3, /* unknown dtype or variant, or a k / stride / dtype / channel count the variant does not implement */
    CONV_MCMK_ERR_WORKSPACE   = 4, /* workspace missing or smaller than conv_mcmk_workspace_bytes() */
    CONV_MCMK_ERR_DEVICE      = 5, /* the HIP runtime refused a launch */
    CONV_MCMK_ERR_ALIGN       = 6  /* a pointer is not 16-byte aligned */
};

/* Text for an error code; never NULL, static storage. */
const char *conv_mcmk_strerror(int code);

/* CONV_MCMK_OK if `variant` can run `desc`, else the error the compute call would return. */
int conv_mcmk_check(const conv_mcmk_desc *desc, int variant);

/*
 * Rows and columns of one output plane (section II-A's output height and width, generalised to any pad
 * and stride): *q = floor((H + 2 pad - k) / stride) + 1, *p likewise from W.  Host only.  Either
 * pointer may be NULL.  Returns CONV_MCMK_OK, or the shape error conv_mcmk_check gives (nothing is
 * written then); the variant plays no part.
 */
int conv_mcmk_output_dims(const conv_mcmk_desc *desc, int *q, int *p);

/*
 * Host-only introspection: writes one line of text saying how `variant` would run `desc` (for the
 * fused kernel: the tile shape, wave layout and channel split the cost estimate picks -- the
 * per-layer selection the paper's conclusion asks for -- and the number of workgroups) into buf,
 * NUL-terminated, at most n bytes.  Returns CONV_MCMK_OK or the error conv_mcmk_check would give.
 */
int conv_mcmk_describe_plan(const conv_mcmk_desc *desc, int variant, char *buf, size_t n);

/*
 * Bytes of caller-provided scratch a variant needs (0 for KN2ROW, KN2COL and DIRECT; 0 also for an invalid
 * desc -- use conv_mcmk_check for the reason).
 *   KN2ROW_2PASS: N * k*k*M * H*W floats -- the GEMM result of section III-A, per image
 *                 T[t*M + m][y*W + x], t = i*k + j (k*k times the output: the price section III names
 *                 for leaving the input unreplicated).
 *   IM2COL:       N * C*k*k * Q*P elements of the input's type -- the input-patch-matrix of
 *                 section II-B, per image Ihat[(c*k + i)*k + j][q*P + p] (k*k times the input).
 *   IM2ROW:       the same number of elements, per image rows[q*P + p][(i*k + j)*C + c].
 * After a 2PASS / IM2COL / IM2ROW call the workspace starts with exactly those matrices.
 * IM2COL and IM2ROW ask for more than their matrix when the matrix product that follows splits its contraction
 * C*k*k into 2, 4, 8 or 16 parts (deep contractions with small outputs, which would otherwise leave most of the chip
 * idle): behind the matrix, at the next multiple of 256 bytes, each part then stores a copy of the result (N*M*Q*P
 * floats rounded up to a multiple of 4), and a last pass adds the copies in a fixed order.  A workspace that holds
 * the matrix but not the copies is accepted: the parts then add into the zeroed output with atomics, which is slower
 * and, beyond two parts, not bit-reproducible from call to call.
 */
size_t conv_mcmk_workspace_bytes(const conv_mcmk_desc *desc, int variant);

/*
 * Bytes of the re-ordered kernel a variant consumes (0 for DIRECT, which reads K as is, and for an
 * invalid desc).  The re-ordering is the one-off, ahead-of-time step of section III-A: the
 * logical matrix is [k*k*M] x [C] for the kn2row variants (row t*M + m, channel innermost) and
 * [M] x [C*k*k] for im2col (section II-B's kernel-patch-matrix).  Physically it is stored in the order
 * the matrix-core instruction takes its operand, zero-padded to whole tiles:
 *   rows in blocks of 16 (MB = ceil(M/16) blocks per tap), contraction index in groups of G
 *   (G = 16 for F32, 32 for BF16; CG = ceil(Kc/G) groups; Kc = C for kn2row, C*k*k for im2col):
 *     F32 : float  Kp[t][mb][cg][lane 0..63][v 0..3]  = A_t[mb*16 + lane%16][cg*16 + 4*v + lane/16]
 *     BF16: bf16   Kp[t][mb][cg][lane 0..63][e 0..7]  = A_t[mb*16 + lane%16][cg*32 + 8*(lane/16) + e]
 *   where A_t[m][c] = K[m][c][i][j] for kn2row / kn2col (t = i*k + j); for im2col t = 0 and
 *   A_0[m][(c*k + i)*k + j] = K[m][c][i][j]; for im2row t = 0 and A_0[m][(i*k + j)*C + c] = K[m][c][i][j].
 *   Entries beyond M or Kc are zero.
 */
size_t conv_mcmk_packed_kernel_bytes(const conv_mcmk_desc *desc, int variant);

/*
 * Re-order K (device, float, [M][C][k][k]) into Kp (device, conv_mcmk_packed_kernel_bytes() bytes)
 * for `variant`; converts to bfloat16 when desc->dtype is CONV_MCMK_BF16.  Done once per layer and
 * not part of the timed convolution (section III-A).  The KN2ROW, KN2ROW_2PASS and KN2COL packings are identical.
 */
int conv_mcmk_prepack(const conv_mcmk_desc *desc, int variant, const void *K_dev, void *Kp_dev, void *stream);

/*
 * Per-layer choice of the algorithm (the paper's conclusion: no single method wins on every layer, so
 * a network should pick per layer).  Estimates the run time of every variant that can run `desc` in
 * the given layout (channels_last = 0: KN2ROW, KN2ROW_2PASS, IM2COL, DIRECT on I[N][C][H][W];
 * channels_last = 1: KN2COL, IM2ROW on I[N][H][W][C]) and whose workspace does not exceed
 * ws_limit_bytes, and returns the cheapest in *variant (and its estimate in microseconds in *est_us,
 * which may be NULL).  Host only.  Errors: CONV_MCMK_ERR_WORKSPACE when only the limit stands in the
 * way, otherwise the error conv_mcmk_check gives (e.g. bf16 with k > 7 and no workspace: the fused
 * kernel does not take the k, DIRECT does not take the type).
 */
int conv_mcmk_select(const conv_mcmk_desc *desc, int channels_last, size_t ws_limit_bytes, int *variant, double *est_us);

/* conv_mcmk_<variant>() chosen by number: the call to follow conv_mcmk_select + conv_mcmk_prepack. */
int conv_mcmk_run(const conv_mcmk_desc *desc, int variant, const void *I_dev, const void *K_dev, void *O_dev,
                  void *ws, size_t ws_bytes, void *stream);

/*
 * The convolution itself, one entry point per variant, same signature.
 *   I_dev   input, float or bfloat16 per desc->dtype
 *   Kp_dev  kernel: the packed form from conv_mcmk_prepack(desc, <this variant>) --
 *           except conv_mcmk_direct, which takes the plain float K[M][C][k][k]
 *   O_dev   output, float
 *   ws, ws_bytes  scratch of at least conv_mcmk_workspace_bytes() (at least the matrix named there: see the note
 *           on IM2COL / IM2ROW); may be NULL / 0 when that is 0
 * conv_mcmk_kn2row implements k = 1 .. 7 and stride 1 or 2 (otherwise CONV_MCMK_ERR_UNSUPPORTED; the
 * other variants take any k >= 1 and any stride >= 1).  conv_mcmk_direct implements CONV_MCMK_F32 only.
 * With a stride the two-pass variant still forms all k*k*M x H*W products (the GEMM of section III-A
 * has no notion of an output position) and subsamples in the post pass; im2col and im2row build
 * only the patches that are used.
 * Results are bit-reproducible from call to call: where conv_mcmk_kn2row splits the channels over two
 * workgroups it adds exactly two partial sums into a zeroed output, which is order-independent, and the deeper
 * splits of the im2col / im2row product add their parts' copies in a fixed order (given the workspace
 * conv_mcmk_workspace_bytes() asks for).
 */
int conv_mcmk_kn2row(const conv_mcmk_desc *desc, const void *I_dev, const void *Kp_dev, void *O_dev,
                     void *ws, size_t ws_bytes, void *stream);
int conv_mcmk_kn2row_2pass(const conv_mcmk_desc *desc, const void *I_dev, const void *Kp_dev, void *O_dev,
                           void *ws, size_t ws_bytes, void *stream);
int conv_mcmk_im2col(const conv_mcmk_desc *desc, const void *I_dev, const void *Kp_dev, void *O_dev,
                     void *ws, size_t ws_bytes, void *stream);
int conv_mcmk_direct(const conv_mcmk_desc *desc, const void *I_dev, const void *K_dev, void *O_dev,
                     void *ws, size_t ws_bytes, void *stream);

/*
 * conv_mcmk_kn2row_2pass for callers that cannot allocate device memory and have no workspace to hand in: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The k*k*M x H*W product of
 * pass 1 goes to a buffer inside the library's own device image instead of a caller-provided workspace; the
 * call allocates and frees nothing (no hipMalloc, no hipFree, no allocating library routine) and otherwise
 * behaves like conv_mcmk_kn2row_2pass: same kernels, same results, same validation and error codes.
 *   - The buffer holds CONV_MCMK_STATIC_SCRATCH_BYTES (32 MiB); a layer whose conv_mcmk_workspace_bytes(desc,
 *     CONV_MCMK_KN2ROW_2PASS) exceeds that gets CONV_MCMK_ERR_WORKSPACE and nothing is launched.
 *   - Every GPU the library is used on holds its own copy of the buffer from the first use until the process
 *     ends; its address on the current device is looked up once (CONV_MCMK_ERR_DEVICE if that fails).
 *   - All calls on one GPU share the buffer, and it keeps the previous call's contents; a call relies on
 *     none of them (pass 1 writes every element pass 2 reads).  Calls that overlap on one GPU -- two streams,
 *     two threads -- race on it: issue them on one stream, or one after the other.
 */
#define CONV_MCMK_STATIC_SCRATCH_BYTES ((size_t)32 << 20)
int conv_mcmk_kn2row_2pass_static(const conv_mcmk_desc *desc, const void *I_dev, const void *Kp_dev, void *O_dev,
                                  void *stream);

/*
 * kn2col (section III-A, last paragraph): the same sum of k*k 1x1 products with the layouts swapped so
 * that the channel is the innermost dimension -- the GEMM becomes [H*W x C] . [C x k*k*M].
 *   I_dev   input  I[N][H][W][C]  (float with C a multiple of 4, or bfloat16 with C a multiple of 8:
 *           the channel vectors are read 16 bytes at a time; other C: CONV_MCMK_ERR_UNSUPPORTED)
 *   Kp_dev  conv_mcmk_prepack(desc, CONV_MCMK_KN2COL): physically the KN2ROW packing (the matrix-core
 *           operand order does not care which of the two GEMM operands the kernel matrix is called)
 *   O_dev   output O[N][Q][P][M], float
 * No workspace; k = 1 .. 7, stride 1 or 2; otherwise as conv_mcmk_kn2row.
 */
int conv_mcmk_kn2col(const conv_mcmk_desc *desc, const void *I_dev, const void *Kp_dev, void *O_dev,
                     void *ws, size_t ws_bytes, void *stream);

/*
 * im2row (section II-B, last paragraph): the input-patch-matrix holds one ROW per output position,
 * rows[n][q*P+p][(i*k+j)*C + c] (the workspace: N * Q*P * k*k*C elements of the input's type, k*k times the
 * input), the kernel-patch-matrix one column per kernel, and O = rows x kernels.
 *   I_dev   input  I[N][H][W][C]  (float with C a multiple of 4, or bfloat16 with C a multiple of 8)
 *   Kp_dev  conv_mcmk_prepack(desc, CONV_MCMK_IM2ROW): A_0[m][(i*k+j)*C + c] = K[m][c][i][j] in the packed form
 *   O_dev   output O[N][Q][P][M], float
 * Any k >= 1.
 */
int conv_mcmk_im2row(const conv_mcmk_desc *desc, const void *I_dev, const void *Kp_dev, void *O_dev,
                     void *ws, size_t ws_bytes, void *stream);

/*
 * The fused variants followed by what a network layer usually applies next (neither is part of the
 * paper's method, which ends at Eq. 3; both act on the finished fp32 sums in registers, so O is still
 * written once):  O = O + bias[m], then O = max(O, 0) when relu != 0 (a NaN stays a NaN).
 *   bias_dev  float[M] in device memory, 4-byte aligned, or NULL for no bias
 *   relu      0 or 1
 * Layouts, packed kernel, supported k / stride and errors as conv_mcmk_kn2row / conv_mcmk_kn2col.
 * No workspace.  (The channel split over two workgroups is not used here: partial sums cannot be rectified.)
 */
int conv_mcmk_kn2row_bias_relu(const conv_mcmk_desc *desc, const void *I_dev, const void *Kp_dev,
                               const float *bias_dev, int relu, void *O_dev, void *stream);
int conv_mcmk_kn2col_bias_relu(const conv_mcmk_desc *desc, const void *I_dev, const void *Kp_dev,
                               const float *bias_dev, int relu, void *O_dev, void *stream);

/*
 * The 1 x 1 MCMK of section III-A on its own: O[n] = A[M x C] . I[n][C x HW], the building block kn2row
 * is made of.  desc->k must be 1 (else CONV_MCMK_ERR_UNSUPPORTED); I[N][C][H][W], O[N][M][Q][P];
 * Kp_dev = conv_mcmk_prepack(desc, CONV_MCMK_KN2ROW).  Without padding and stride the image is treated as
 * one row of H*W columns, so no tile is cut short at image edges; otherwise this is conv_mcmk_kn2row.
 */
int conv_mcmk_1x1(const conv_mcmk_desc *desc, const void *I_dev, const void *Kp_dev, void *O_dev, void *stream);

/* float -> bfloat16 (round to nearest even), `count` elements, device to device. */
int conv_mcmk_cvt_f32_bf16(const void *src_dev, void *dst_dev, size_t count, void *stream);

/*
 * Tuning aids (host only, process-wide, thread-safe; no part of the method).  The fused kernels and the
 * matrix product of the staged variants each pick a tile shape from a menu by a cost estimate;
 * conv_mcmk_force_tile / conv_mcmk_force_gemm_tile make every later call take menu entry `index` instead
 * (for an entry the layer's operand type, kernel side or stride does not have -- or an index beyond the menu -- the
 * estimate still chooses, among the menu's entries: while an index is set, a 1 x 1 layer is not run as a plain matrix
 * product on the flat tile shape); a negative index gives the choice back to the estimate.  The environment variables CONV_MCMK_TILE / CONV_MCMK_GEMM_TILE set
 * the initial value; they are read once, when the library is first used.
 */
void conv_mcmk_force_tile(int index);
void conv_mcmk_force_gemm_tile(int index);

/*
 * Measurement aids for the benchmark (no part of the method): the two machine rates the roofline
 * figures are compared with, measured on the device at hand.
 *   conv_mcmk_probe_mfma: launches `blocks` workgroups of 256 threads that each issue `iters` x 16
 *     independent matrix-core products from registers only (dtype CONV_MCMK_F32: v_mfma_f32_16x16x4_f32,
 *     2048 flop each; CONV_MCMK_BF16: v_mfma_f32_16x16x32_bf16, 16384 flop each) and store one value per
 *     lane to sink_dev (blocks * 256 floats, so that the products cannot be dropped).  Flop of a launch:
 *     blocks * 4 waves * iters * 16 * (2048 or 16384).
 *   conv_mcmk_probe_copy: copies `bytes` (a multiple of 16) from src_dev to dst_dev with 16-byte
 *     accesses, the plain streaming kernel of known traffic (bytes read + bytes written).
 * Both validate pointers and alignment like the other calls and launch on `stream`.
 */
int conv_mcmk_probe_mfma(int dtype, int blocks, int iters, float *sink_dev, void *stream);
int conv_mcmk_probe_copy(const void *src_dev, void *dst_dev, size_t bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* CONV_MCMK_H */
