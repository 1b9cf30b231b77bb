/*
 * pcc.h -- C ABI of libpcc: per-pixel causal-context lossless image coding on
 * one MI355X (gfx950).
 *
 * The method is the learned pixel-by-pixel coder of arXiv 2212.01185: a small
 * network maps every pixel's causal neighbourhood of already coded pixels to
 * the parameters of a discretised Gaussian mixture per colour channel
 * (Sec. III-A, Eq. (1)-(4); network Sec. III-B), an entropy coder codes the
 * sub-pixels with those distributions, the encoder evaluates all pixels in
 * parallel and the decoder proceeds as a wavefront (Sec. III-C, Eq. (6)).
 *
 * Conventions
 *   - Images are uint8, layout [n][H][W][3] (rows, columns, RGB), contiguous,
 *     in DEVICE memory.  "d_" arguments are device pointers, "h_" host pointers.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the null stream).
 *     Kernels are launched on it; nothing else is synchronised.
 *   - Every buffer named in a call is owned by the caller; the library neither
 *     frees nor keeps it beyond the call.  A pcc_ctx owns its packed copy of
 *     the weights and a private device workspace that grows on demand
 *     (hipMalloc inside the first call that needs it, reused afterwards).
 *   - A pcc_ctx must not be used by two calls at the same time.
 *   - All functions returning int return PCC_OK (0) or a negative PCC_E_* code;
 *     no exceptions or aborts cross this boundary and damaged input cannot
 *     make a call hang (device waits are bounded).
 *
 * Weight blob (host memory): 16 little-endian uint32 header words {magic
 * "PCCW", version 1, n_layers, dims[8], K, neighbourhood size, wavefront delay
 * per row, activation id, distribution id}, then per layer W[out][in] and
 * b[out] as fp32.  Weights must be exactly representable in bf16 (biases are
 * fp32); components are Gaussian (distribution id 0, Eq. (1)) or logistic
 * (id 1, Eq. (8)).  This library accepts these models:
 *   - 30 -> 160 -> 160 -> 128 -> 60, ReLU (activation id 0), K = 5, the
 *     10-pixel neighbourhood {rows r-2, r-1 at columns c-2..c+1; row r at
 *     c-2, c-1}, delay 2 (the measured workloads);
 *   - 36 -> 128 -> 128 -> 128 -> 128 -> 36, LeakyReLU with slope 0.01 (id 1),
 *     K = 3, the 12-pixel neighbourhood {rows r-2, r-1 at columns c-2..c+2;
 *     row r at c-2, c-1}, delay 3 (the network of Sec. III-B with the
 *     hyper-parameters of Sec. IV-E);
 *   - the same shape with delay 1: the diagonal decoding order of Sec. III-C,
 *     Eq. (7).  A pass decodes the anti-diagonal r + c = t; the inputs of the
 *     three neighbours not yet decoded then, (r-2,c+2), (r-1,c+1), (r-1,c+2),
 *     carry copies of pixel (r-1,c) (zero in the first row), at the encoder too;
 *   - the six shapes of the ablations of Sec. IV-E, each the second model with
 *     one hyper-parameter changed: K = 5 (36 -> 128 x 4 -> 60), K = 7
 *     (36 -> 128 x 4 -> 84), 64 filters (36 -> 64 x 4 -> 36), 192 filters
 *     (36 -> 192 x 4 -> 36), four layers (36 -> 128 x 3 -> 36), six layers
 *     (36 -> 128 x 5 -> 36).
 * Head layout o[12 K]: for each of R,G,B: K mixture logits, K means, K
 * log-sigmas (units of 1/256 of the grey range); then K alphas, K betas,
 * K gammas of Eq. (3)-(4).
 *
 * Stream (device memory): 8 little-endian uint32 words {magic "PCC1", version
 * 2, n, H, W, K | nbhd<<8 | delay<<16 | 16<<24, distribution id, 0}, uint64 offsets[n*H+1]
 * (relative to the end of that table), then one rANS payload per image row:
 * the two initial decoder states (8 bytes each; sub-pixel i = 3 c + channel of
 * the row is coded on state i mod 2), then the 32-bit words, shared by both
 * states, in the order the decoder reads them.  Streams written by this library are read by this library; the
 * bytes depend on its floating-point evaluation order and are not portable to
 * another implementation of the same model.
 */
#ifndef PCC_H
#define PCC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PCC_OK 0
#define PCC_E_ARG (-1)      /* null pointer, non-positive or too large dimension */
#define PCC_E_BLOB (-2)     /* weight blob: bad magic, unsupported shape, size mismatch, non-bf16 weight */
#define PCC_E_CAP (-3)      /* output capacity too small */
#define PCC_E_STREAM (-4)   /* stream: bad header, dimensions differ, offsets out of range, payload over/under-read */
#define PCC_E_HIP (-5)      /* a HIP runtime call failed */
#define PCC_E_INTERNAL (-6) /* zero frequency or bounded device wait expired */
#define PCC_E_UNIMPL (-7)
#define PCC_E_SCRATCH (-8)  /* pcc_decode_static: the job needs more than PCC_STATIC_SCRATCH_BYTES of scratch memory */

#define PCC_HEAD_OUTPUTS 60 /* of the 30-160-160-128-60 network; in general pcc_model_info()[0] */

typedef struct pcc_ctx pcc_ctx;

/* Parse and pack the weight blob (host pointer) for device `hip_device`.
 * On success *out owns device memory until pcc_destroy.
 * Reads these environment variables, which exist for tests and measurements and
 * never change a result: PCC_ENCODE_VARIANT (0..3: tiles per work item and
 * workgroup size of the pixel kernel), PCC_ENCODE_OVERLAP (0: the row coder
 * always runs after the pixel kernel), PCC_RANS_PATIENCE (polls before a row
 * coder running beside the pixel kernel stands down), PCC_DECODE_VARIANT (1, 2:
 * decoder workgroups per compute unit; 0: chosen per job), PCC_DECODE_SPIN_LIMIT
 * (polls of a band for the band above before pcc_decode fails with
 * PCC_E_INTERNAL). */
int pcc_create(pcc_ctx **out, const void *h_blob, size_t blob_bytes, int hip_device);
void pcc_destroy(pcc_ctx *ctx);

/* Upper bound in bytes of the stream pcc_encode writes for n images of H x W. */
size_t pcc_stream_bound(int n, int H, int W);

/* Number of wavefront passes for an H x W image when each row trails the row
 * above by `delay` columns (right reach of the neighbourhood + 1): Eq. (6)
 * generalised, T = W + delay (H - 1).  0 for non-positive arguments. */
long pcc_wavefront_steps(int H, int W, int delay);

/* Shape of the network the ctx was created with, h_info[6] (host): head
 * outputs per pixel (12 K), K, neighbourhood size, delay, distribution id,
 * number of layers. */
int pcc_model_info(const pcc_ctx *ctx, int *h_info);

/* Network evaluation for every pixel (Sec. III-C first paragraph: at the
 * encoder all pixels are known and are processed in parallel).
 *   d_params [n][H][W][12 K] fp32: raw head outputs in the head layout above.
 *   d_bits   [n][H][W] fp32 or NULL: -log2 of the quantised joint probability
 *            of the pixel's true (r,g,b), i.e. its term of the loss Eq. (5).
 * Asynchronous: returns after the launch. */
int pcc_encode_probs(pcc_ctx *ctx, const uint8_t *d_img, int n, int H, int W,
                     float *d_params, float *d_bits, void *hip_stream);

/* Encoder (Sec. IV-C first paragraph): parameters for all pixels in parallel,
 * integer CDF values of the true sub-pixels, row-wise rANS, stream assembly.
 * Writes at most cap_bytes to d_stream and the byte count to *h_nbytes_out.
 * Synchronises hip_stream before returning (the size is read back).  When
 * hip_stream is idle at the call and the job has at most 3072 rows, the row
 * coder and the stream assembly run on a stream the ctx owns, beside the
 * pixel kernel; both streams have been waited for when the call returns, so
 * the caller's view is the same.  That mode needs the two kernels to run at
 * the same time.  Where something runs a process's kernels one after the other
 * (a profiler collecting counters does; so does a chip another job fills), the
 * row coder finds no symbols, gives up after PCC_RANS_PATIENCE polls (a few
 * milliseconds with the default) and is launched again behind the pixel kernel:
 * the result is the same, but such a call pays that wait first, i.e. ten times
 * a 768 x 512 encode.  PCC_ENCODE_OVERLAP=0 avoids the mode altogether.
 * One call at a time per ctx.  On an error return no kernel of the call is
 * still running on either stream. */
int pcc_encode(pcc_ctx *ctx, const uint8_t *d_img, int n, int H, int W,
               uint8_t *d_stream, size_t cap_bytes, size_t *h_nbytes_out, void *hip_stream);

/* Wavefront decoder (Sec. III-C): pass t decodes every pixel (r, c) with
 * delay * r + c = t.  d_img_out [n][H][W][3] is fully overwritten.  Synchronises
 * hip_stream before returning (the device status word is read back).  On
 * PCC_E_STREAM the image content is unspecified. */
int pcc_decode(pcc_ctx *ctx, const uint8_t *d_stream, size_t nbytes, int n, int H, int W,
               uint8_t *d_img_out, void *hip_stream);

/* pcc_decode for callers that cannot allocate device memory: code under HIP
 * graph capture restrictions, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, same result and same errors as pcc_decode, but the
 * decoder's only scratch buffer -- the mailbox through which a band of 16 rows
 * hands its last two rows to the band below, 8 bytes per pixel column and band:
 * pcc_decode_static_scratch_bytes(n, H, W) -- lives in an array of
 * PCC_STATIC_SCRATCH_BYTES that is part of the library's device code (every GPU
 * the library runs on holds it until the process ends) instead of the ctx's
 * workspace.  The call allocates and frees nothing, and clears what it uses of
 * the array with a kernel (no memset node).  A job that needs more returns
 * PCC_E_SCRATCH before anything is launched (8 MiB covers one 4096 x 2160 image
 * and 24 images of 768 x 512).  All ctxs on a GPU share that GPU's array: two
 * pcc_decode_static calls that overlap in time on one GPU race, whatever their
 * ctxs and streams.  Synchronises hip_stream before returning. */
#define PCC_STATIC_SCRATCH_BYTES (8u << 20)
size_t pcc_decode_static_scratch_bytes(int n, int H, int W);   /* 0 for invalid dimensions */
int pcc_decode_static(pcc_ctx *ctx, const uint8_t *d_stream, size_t nbytes, int n, int H, int W,
                      uint8_t *d_img_out, void *hip_stream);

/* Test hooks (not on the hot path). */

/* Eq. (1)-(4) + integer CDF rule alone: from given head outputs d_params
 * [count][12 K] and the conditioning sub-pixels d_rg [count][2] (r, g) write the
 * full tables d_cq [count][3][257] (uint32).  Asynchronous. */
int pcc_cdf_tables(pcc_ctx *ctx, const float *d_params, const uint8_t *d_rg, size_t count,
                   uint32_t *d_cq, void *hip_stream);

/* Copy the (start, freq) pairs the last pcc_encode on this ctx fed to the
 * coder: d_out [n][H][W][3] uint32, start | (freq - 1) << 16.  Asynchronous. */
int pcc_copy_intervals(pcc_ctx *ctx, uint32_t *d_out, size_t count, void *hip_stream);

/* Per-kernel timing.  With profiling enabled, pcc_encode and pcc_decode bracket
 * each kernel they launch with HIP events on the caller's stream; after the
 * call, pcc_last_timings copies the durations in milliseconds of the last such
 * call into h_ms[PCC_N_TIMINGS] (kernels that did not run: 0). */
#define PCC_T_ENCODE_PIXELS 0 /* gather + network + mixture -> (start,freq), all pixels */
#define PCC_T_ENCODE_RANS 1   /* row-wise rANS */
#define PCC_T_ENCODE_SCAN 2   /* offsets */
#define PCC_T_ENCODE_COMPACT 3
#define PCC_T_DECODE 4        /* wavefront decode kernel */
#define PCC_N_TIMINGS 5
int pcc_set_profiling(pcc_ctx *ctx, int enabled);
int pcc_last_timings(pcc_ctx *ctx, float *h_ms);

const char *pcc_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* PCC_H */
