/*
 * mdnn.h -- C ABI of the MI355X (gfx950) forward-propagation convolution.
 *
 * The operation is the minibatch convolution of Section 2 of the maxDNN paper
 * (arXiv 1501.06633), computed the way Sections 3 and 3.2 describe it: for
 * every output coordinate, an Nb x (Sk^2 Nc) patch gathered from the
 * batch-innermost input multiplies the (Sk^2 Nc) x No filter matrix, the
 * gather offsets of the patch columns being precomputed once per tile.
 *
 * All functions are extern "C", throw nothing, keep no mutable global state
 * that affects results, allocate no device memory and never synchronise the
 * device.  Pointers named "device" are HIP device pointers; everything else
 * is host memory.
 */
#ifndef MDNN_H_
#define MDNN_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum mdnn_status {
    MDNN_OK      = 0,
    MDNN_EINVAL  = 1,   /* a dimension < 1, stride < 1, pad < 0, filter larger than padded image,
                           non-finite alpha, unknown variant name */
    MDNN_ENULL   = 2,   /* a required pointer is NULL */
    MDNN_EALIGN  = 3,   /* a tensor pointer is not 16-byte aligned */
    MDNN_ETOOBIG = 4,   /* in or out is 2^32 bytes or larger, or filt 2^31 bytes or larger, or
                           (Nc Sk^2 + 64) No floats reach 2^32 bytes (32-bit byte offsets are used on
                           the device, the same kind of limit Section 3.1 notes for texture indices) */
    MDNN_ELAUNCH = 5    /* the HIP runtime refused the launch (hipGetLastError() != hipSuccess) */
} mdnn_status;

/*
 * FPROP convolution (Section 2; Section 3 for the layouts; Section 3.2 for the
 * per-output-coordinate tiling and the offset table).
 *
 *   in    device, fp32, [Nc][Hi][Wi][Nb]   batch innermost, NOT physically padded
 *   filt  device, fp32, [Nc][Sk][Sk][No]   = row-major (Nc*Sk*Sk) x No filter matrix
 *   out   device, fp32, [No][Ho][Wo][Nb]   fully overwritten (no accumulate)
 *
 *   out[o][y][x][n] = alpha * sum_{c,ky,kx} in[c][y*stride-pad+ky][x*stride-pad+kx][n]
 *                                         * filt[c][ky][kx][o]
 *   with taps outside the image reading zero (the zero apron), and
 *   Wo = floor((Wi + 2 pad - Sk)/stride) + 1, Ho likewise.
 *
 * Arithmetic is fp32 throughout (fp32 matrix-core FMAs, no reduced-precision
 * conversion); the summation order is unspecified.  Any Nb >= 1 and No >= 1
 * give correct results; the fastest kernels need Nb % 4 == 0 and No % 4 == 0,
 * other values take a variant of the same kernel that copies the operand
 * concerned (filters for No, input patches for Nb) 4 bytes at a time, 5 to 8
 * per cent slower.
 *
 * The caller owns all three buffers; out must not overlap in or filt.  The
 * call only enqueues work on `stream` (a hipStream_t; NULL = the default
 * stream) and returns; the result is valid once the stream has been
 * synchronised.  All argument checks happen before anything is enqueued:
 * on any status other than MDNN_OK nothing has been launched.  Nothing is
 * allocated, cleared with a memset or synchronised, so the call may be recorded
 * into a HIP graph; the first launch of a kernel on a device also raises that
 * kernel's LDS limit (a function attribute, not a stream operation), so make
 * one call outside the capture first.
 */
mdnn_status mdnn_conv_fprop(const float* in, const float* filt, float* out,
                            int Nb, int Wi, int Hi, int Nc, int No,
                            int Sk, int stride, int pad, float alpha,
                            void* stream);

/*
 * Same operation with the tile variant chosen by the caller instead of the
 * built-in heuristic (for tests and tuning).  `variant` is one of the names
 * mdnn_variant_name() enumerates, or NULL / "" / "auto" for the heuristic.
 * A name may be followed by ':' and one letter that pins how tiles are cut into
 * the smaller blocks of Section 3.4: w = no tile is cut; h, t, q, e = the tiles
 * of the last partial round in halves, thirds (48 + 48 + 32 filter rows),
 * quarters, eighths (16 rows); m, n = 128 of them in halves and the rest in
 * quarters (m, at most 64) or eighths (n, at most 32), p = 64 of them in quarters
 * and the rest (at most 32) in eighths, all launched in front of the whole tiles;
 * H, T, Q, E = every tile so.  A cut the kernel does not have, or that does not
 * fit the tile count, is MDNN_EINVAL.
 * Every variant and cut computes the same function for every valid argument set.
 */
mdnn_status mdnn_conv_fprop_variant(const float* in, const float* filt, float* out,
                                    int Nb, int Wi, int Hi, int Nc, int No,
                                    int Sk, int stride, int pad, float alpha,
                                    void* stream, const char* variant);

/* Output extents by the floor formula above (the paper gives none; this one
 * reproduces every input/output/kernel triple of Table 1).  Host only. */
mdnn_status mdnn_out_dims(int Wi, int Hi, int Sk, int stride, int pad, int* Wo, int* Ho);

/* Algorithmic complexity of Section 2: 2 Nb Wo Ho (Nc Sk^2 + 1) No FLOPs.
 * Returns 0 if any argument is < 1.  Host only. */
uint64_t mdnn_conv_flops(int Nb, int Wo, int Ho, int Nc, int No, int Sk);

/* Static, human-readable text for a status code.  Never NULL. */
const char* mdnn_status_string(mdnn_status s);

/* Name of tile variant number i (0 <= i < mdnn_variant_count()), else NULL. */
int         mdnn_variant_count(void);
const char* mdnn_variant_name(int i);

/* Name of the variant the heuristic picks for a problem, without launching
 * anything (host only).  Returns NULL if the geometry is invalid. */
const char* mdnn_choose_variant(int Nb, int Wi, int Hi, int Nc, int No,
                                int Sk, int stride, int pad);

/*
 * Data gradient (BPROP with respect to the input).  The paper builds FPROP only
 * and states the belief that the same techniques carry over (abstract, Section
 * 3.5); here they do, literally: the gradient is computed by the FPROP kernels
 * as a stride-1 convolution of the output gradient with the turned-over,
 * channel/filter-swapped filter bank.
 *
 *   dout  device, fp32, [No][Ho][Wo][Nb]   gradient w.r.t. the forward output
 *   filt  device, fp32, [Nc][Sk][Sk][No]   the forward filter bank, unchanged
 *   din   device, fp32, [Nc][Hi][Wi][Nb]   fully overwritten
 *
 *   din[c][iy][ix][n] = alpha * sum over every forward term in[c][iy][ix][n] took part in of
 *                       dout[o][y][x][n] * filt[c][ky][kx][o]
 *   (iy = y*stride - pad + ky, ix likewise); input pixels no window reaches get 0.
 *
 * The dimension arguments are those of the FORWARD call; any pad the forward
 * call accepts is accepted (a stride-1 layer with pad > Sk - 1 takes the same
 * route as a strided one).  `workspace` is device memory of at least the size
 * mdnn_conv_bprop_data_workspace() reports (16-byte aligned); it receives the
 * rearranged filter bank, nothing else: for stride > 1 the input pixels are
 * split by (iy + pad, ix + pad) modulo the stride, every class is a stride-1
 * problem with a ceil(Sk/stride)^2 sub-filter, all classes run as one
 * convolution, and that convolution stores each value straight to its
 * interleaved place in din.  The workspace may be reused or freed once the
 * stream has passed this call.  Same stream, ownership and error rules as
 * mdnn_conv_fprop, with one difference: the call enqueues two or three kernels,
 * and MDNN_ELAUNCH can be returned after the first of them was enqueued (din and
 * the workspace are then undefined).  MDNN_ETOOBIG also where the classes' common
 * grid, (Ho + T - 1)(Wo + T - 1) Nb s^2 Nc values with T = ceil(Sk/stride), reaches
 * 2^32 bytes (it is the kernel's index space, not memory).
 */
mdnn_status mdnn_conv_bprop_data_workspace(int Nb, int Wi, int Hi, int Nc, int No,
                                           int Sk, int stride, int pad, size_t* bytes);
mdnn_status mdnn_conv_bprop_data(const float* dout, const float* filt, float* din,
                                 void* workspace, size_t workspace_bytes,
                                 int Nb, int Wi, int Hi, int Nc, int No,
                                 int Sk, int stride, int pad, float alpha, void* stream);

/*
 * mdnn_conv_bprop_data for callers that cannot allocate device memory or hand
 * over a workspace: code that records a HIP graph, tight serving loops,
 * harnesses that forbid allocation.  Same operation, same kernels, same result
 * bit for bit; the workspace is a static device array of
 * MDNN_STATIC_SCRATCH_BYTES inside the library (every GPU the library runs on
 * holds its own copy until the process ends).  The call allocates and frees
 * nothing and uses no memset.  A problem whose workspace
 * (mdnn_conv_bprop_data_workspace()) exceeds MDNN_STATIC_SCRATCH_BYTES is
 * refused with MDNN_ETOOBIG before anything is enqueued: the limit covers the
 * rearranged bank of every layer up to 1024 x 1024 filters of 3 x 3.
 * All calls on one GPU share that GPU's array, which keeps whatever the last
 * call left in it (every call overwrites all it reads, nothing has to start
 * at zero): calls that overlap in time on one GPU -- different streams, or two
 * host threads -- race; calls on one stream are ordered and safe.  The first
 * call on a GPU looks up the array's address there (a runtime query, no
 * allocation); make that call outside a graph capture.  Other rules as for
 * mdnn_conv_bprop_data.
 */
#define MDNN_STATIC_SCRATCH_BYTES (40u << 20)
mdnn_status mdnn_conv_bprop_data_static(const float* dout, const float* filt, float* din,
                                        int Nb, int Wi, int Hi, int Nc, int No,
                                        int Sk, int stride, int pad, float alpha, void* stream);

/*
 * Filter gradient (BPROP with respect to the weights), the other half of what
 * the paper leaves as a conjecture (abstract, Section 3.5).  It is the
 * per-coordinate patch x filter-matrix product of Section 3 turned round: the
 * K x No gradient of the filter matrix is the sum, over all output coordinates
 * and images, of patch column times output-gradient row, computed as one
 * implicit GEMM on the matrix cores with the patch gathered as in Section 3.2.
 *
 *   in    device, fp32, [Nc][Hi][Wi][Nb]   the forward input
 *   dout  device, fp32, [No][Ho][Wo][Nb]   gradient w.r.t. the forward output
 *   dfilt device, fp32, [Nc][Sk][Sk][No]   fully overwritten
 *
 *   dfilt[c][ky][kx][o] = alpha * sum_{y,x,n} in[c][y*stride-pad+ky][x*stride-pad+kx][n] * dout[o][y][x][n]
 *   (apron reads are 0).
 *
 * The dimension arguments are those of the FORWARD call; any pad is accepted.
 * `workspace` is device memory of at least the size
 * mdnn_conv_bprop_filter_workspace() reports (16-byte aligned): the contraction
 * is cut into ranges so that the launch fills the chip, every range leaves a
 * partial gradient there, and a second kernel adds them in a fixed order (the
 * result is deterministic).  It may be reused or freed once the stream has
 * passed this call.  Same stream, ownership and error rules as mdnn_conv_fprop
 * (two kernels: MDNN_ELAUNCH can be returned after the first was enqueued);
 * in and dout must each be smaller than 2^32 bytes (MDNN_ETOOBIG).
 */
mdnn_status mdnn_conv_bprop_filter_workspace(int Nb, int Wi, int Hi, int Nc, int No,
                                             int Sk, int stride, int pad, size_t* bytes);
mdnn_status mdnn_conv_bprop_filter(const float* in, const float* dout, float* dfilt,
                                   void* workspace, size_t workspace_bytes,
                                   int Nb, int Wi, int Hi, int Nc, int No,
                                   int Sk, int stride, int pad, float alpha, void* stream);

/*
 * Plain SGEMM in the convolution's operand layout: the yardstick the paper's
 * conclusion (Section 3.5) holds its kernel against, and what Section 3's
 * patch-times-filter-matrix product becomes for a 1 x 1 filter, where the patch
 * is the input itself.  It runs the FPROP kernel on that degenerate geometry
 * (one pixel, M images), so the inner loop is the convolution's own.
 *
 *   a  device, fp32, [K][N]   row-major (the filter matrix: row k, column o)
 *   b  device, fp32, [K][M]   row-major (the input: row k, column m)
 *   c  device, fp32, [N][M]   row-major, fully overwritten
 *
 *   c[o][m] = alpha * sum_k a[k][o] * b[k][m]          (c = alpha * a^T b)
 *
 * Any N, M, K >= 1; the fast kernels need N % 4 == 0 and M % 4 == 0.  b and c
 * must each be smaller than 2^32 bytes and a smaller than 2^31 (MDNN_ETOOBIG).
 * Same stream, ownership, alignment and error rules as mdnn_conv_fprop.
 */
mdnn_status mdnn_sgemm_tn(const float* a, const float* b, float* c,
                          int N, int M, int K, float alpha, void* stream);

/*
 * Describe, as one line of text, how a problem would be launched: variant, tile
 * shape, number of tiles, how the last partial round of tiles is cut into
 * smaller pieces (the other block sizes Section 3.4 proposes), grid and LDS
 * size.  Host only, launches nothing.  `variant` as in mdnn_conv_fprop_variant.
 * `text` receives at most text_size bytes including the terminating 0.
 */
mdnn_status mdnn_describe_launch(int Nb, int Wi, int Hi, int Nc, int No,
                                 int Sk, int stride, int pad, const char* variant,
                                 char* text, size_t text_size);

/*
 * Measurement aid for the efficiency metric of Section 3.3 (actual over peak
 * throughput): enqueue a register-only loop of fp32 matrix-core FMAs on every
 * compute unit -- no memory traffic -- so that timing it gives the FP32 matrix
 * rate the chip sustains under its power cap.  `sink` is a device buffer of at
 * least 64 floats per launched wave (blocks * waves_per_block * 64 floats)
 * that keeps the compiler from deleting the loop.  *flops receives the FLOPs
 * one launch performs (host pointer, nullable).
 */
mdnn_status mdnn_mfma_peak_probe(float* sink, int blocks, int waves_per_block,
                                 int iters, uint64_t* flops, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MDNN_H_ */
