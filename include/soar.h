/*
 * soar.h -- C-ABI of the MI355X (gfx950) SOAR NVFP4 weight-quantization library.
 *
 * The library implements the data-parallel hot path of SOAR (arXiv 2605.12245):
 * NVFP4 weight quantization (Sec. 3.1) with one Closed-form Joint Scale
 * Optimization step (Sec. 3.2, Eq. 5-6) followed by one Decoupled Scale Search
 * over E4M3 candidates for the stored block scale (Sec. 3.3, Eq. 7-8;
 * Algorithm 1 with T = 1 and beta = 1) -- the single-step path -- and, through
 * the same entry points, Algorithm 1 in full: T iterations, a grid of
 * quantization-scale factors beta, early stopping (the iterated path).
 *
 * Conventions common to all entry points
 *   - every pointer whose name starts with d_ is DEVICE memory owned by the
 *     caller; the library allocates no device memory and frees nothing.  What it
 *     owns, per GPU and until the process ends: the fixed array inside its device
 *     image that soar_quantize_static uses, four diagnostic counters, and -- created
 *     by the first batch call that is spread over two streams (see `streams`) -- one
 *     internal stream of default priority with two events;
 *   - work is enqueued on `hip_stream` (a hipStream_t passed as void*, NULL =
 *     the default stream) and the call returns without synchronising; results
 *     (global scale, error, data-dependent status) stay in device memory;
 *   - the quantize / dequantize / error entry points may be called from several
 *     host threads at once, each call with its own workspace and outputs; the
 *     timing and statistics switches are process-wide and not thread-safe;
 *   - inputs whose largest magnitude is below 2^-60 underflow inside the formulas
 *     (products w*q, alpha*Delta): both the library and its reference follow
 *     IEEE binary32 arithmetic there, but the results are not specified;
 *   - weights are row-major, `rows x cols`, leading dimension `ld_elems` >= cols
 *     (in elements); a block is 16 consecutive elements of a row, so
 *     cols % 16 == 0 is required; the weight base address must be 16-byte
 *     aligned and ld_elems * element size a multiple of 16 bytes;
 *   - packed codes: rows*cols/2 bytes, row-major and dense; element 2k of a row
 *     sits in bits 0-3 of byte k, element 2k+1 in bits 4-7; a nibble is
 *     sign<<3 | E2M1 magnitude code, magnitudes {0,.5,1,1.5,2,3,4,6};
 *   - block scales: rows*cols/16 bytes, row-major and dense, one positive OCP
 *     E4M3 ("fn": bias 7, max 448) byte in [0x01, 0x7E] per block;
 *   - host-checkable argument errors are returned before anything is enqueued
 *     and leave every output untouched; no exception crosses this boundary.
 */
#ifndef SOAR_H
#define SOAR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SOAR_OK = 0,
    SOAR_ERR_NULL = 1,       /* a required pointer is NULL                          */
    SOAR_ERR_SHAPE = 2,      /* rows/cols/ld out of range, cols % 16 != 0           */
    SOAR_ERR_DTYPE = 3,      /* unknown element type                                */
    SOAR_ERR_PARAM = 4,      /* bad soar_params field                               */
    SOAR_ERR_WORKSPACE = 5,  /* workspace missing, misaligned or too small          */
    SOAR_ERR_HIP = 6,        /* a HIP runtime call failed (launch error)            */
    SOAR_ERR_ALIGN = 7,      /* weight/output pointer or leading dimension misaligned */
    SOAR_ERR_TOO_LARGE = 8   /* soar_quantize_static: more blocks than its built-in workspace holds */
} soar_status;

typedef enum { SOAR_BF16 = 0, SOAR_FP32 = 1 } soar_dtype;

typedef enum {
    SOAR_METHOD_RTN = 0,     /* max-based NVFP4, Sec. 3.1 Eq. 1-2                   */
    SOAR_METHOD_SOAR = 1,    /* Eq. 1-2 init, Eq. 5-6 step, Eq. 8 search            */
    /* the arms of the component study (Sec. 4.3, first table), iterated path only: */
    SOAR_METHOD_CJSO_ONLY = 2, /* Sec. 3.2 alone: Eq. 5, Eq. 6, projection onto E4M3, ONE
                                block scale for assignment and storage; needs n_beta 1,
                                beta 1, SOAR_DD_WINDOW, dss_radius 0                 */
    SOAR_METHOD_DSS_ONLY = 3   /* Sec. 3.3 (i)-(ii) alone: the global scale keeps its
                                Eq. 1 value, the joint search is centred on the block's
                                current stored scale (window candidates)             */
} soar_method;

/* how the Eq. 8 search is carried out; every mode returns the same bytes */
typedef enum {
    SOAR_SEARCH_AUTO = 0,    /* the library's fastest exact strategy                */
    SOAR_SEARCH_FULL = 1     /* evaluate all 2K+1 candidates                        */
} soar_search_mode;

/* the one-launch kernel for a single tensor, see soar_params.resident */
typedef enum {
    SOAR_RESIDENT_AUTO = 0,  /* used when the tensor fits and the grid fits the GPU     */
    SOAR_RESIDENT_NEVER = 1  /* always the three-pass path                              */
} soar_resident_mode;

/* which E4M3 codes are candidates for the stored scale Delta^d (Sec. 3.3 (ii)) */
typedef enum {
    SOAR_DD_WINDOW = 0,      /* centre-K .. centre+K, centre = E4M3(Delta*) (App. D) */
    SOAR_DD_BRACKET = 1      /* the two codes that enclose Delta* (App. B.3)         */
} soar_dd_mode;

/* data-dependent status bits written to *d_status */
#define SOAR_STATUS_NONFINITE 1   /* NaN or Inf in the weights: outputs unspecified  */
#define SOAR_STATUS_ALLZERO   2   /* every weight is zero                            */
#define SOAR_STATUS_BAD_AMAX  4   /* supplied maximum not finite or not > 0: outputs
                                     unspecified                                     */
#define SOAR_STATUS_GAVE_UP   8   /* the one-launch kernel (see soar_params.resident) did not
                                     get all of its workgroups onto the GPU within
                                     resident_wait_us and left: outputs unspecified; run the
                                     call again, or with resident = SOAR_RESIDENT_NEVER    */

typedef struct {
    uint32_t struct_size;    /* sizeof(soar_params), for forward compatibility      */
    int32_t  method;         /* soar_method                                         */
    int32_t  block;          /* block size G of Algorithm 1; must be 16             */
    int32_t  iters;          /* iterations T of Algorithm 1, 1 .. 64                */
    int32_t  dss_radius;     /* K >= 0: stored-scale candidates are the E4M3 codes
                                centre-K .. centre+K (Sec. 3.3 (ii)); 0 = centre only */
    int32_t  n_beta;         /* size of the grid of quantization-scale factors,
                                1 .. 4096 (Sec. 3.3 (i); App. B.3 uses 101)          */
    float    beta_lo;        /* grid ends, 0 < beta_lo <= beta_hi; factor k is
                                (beta_lo (n-1-k) + beta_hi k) / (n-1) in binary32,   */
    float    beta_hi;        /* beta_lo alone when n_beta == 1                       */
    float    early_stop_rel; /* >= 0; the iterated path stops after an iteration that
                                lowers the error by less than this fraction of the
                                error before it (App. B.3: 1e-3); 0 = never         */
    int32_t  search_mode;    /* soar_search_mode                                    */
    int32_t  tiles_per_wg;   /* 0 = chosen by the library; a power of two <= 65536
                                forces how many 256-block tiles one workgroup walks
                                (for tests: outputs must not depend on it)          */
    int32_t  streams;        /* soar_quantize_batch: 0 = library default (launch
                                groups alternate between the caller's stream and one
                                internal stream, forked and joined by events);
                                1 = everything on the caller's stream.  Only calls
                                with streams = 1 (or that stay on one stream anyway:
                                one launch group) may be captured into a HIP graph:
                                the internal stream is shared by all callers, and a
                                capture that pulls it in would swallow their work  */
    int32_t  dd_mode;        /* soar_dd_mode; dss_radius is ignored for BRACKET     */
    int32_t  resident;       /* soar_resident_mode: may one tensor handed over alone (single-
                                step settings, tiles_per_wg 0, at most 4096 blocks per compute
                                unit: 2^20 blocks = 32 MiB of bf16 on an MI355X) take ONE
                                launch that keeps the tensor in registers and crosses its two
                                tensor-wide dependencies (Eq. 1 maximum, Eq. 5 sums) inside
                                the kernel?  Same bytes as the three-pass path, the weights
                                are read once.  It needs every workgroup of its grid (at most
                                one per compute unit) on the GPU at the same time and waits
                                for that at most resident_wait_us.  A call that arrives on
                                another stream while an earlier such kernel may still run
                                takes the three-pass path instead (two of them started at
                                once could each hold part of the GPU and wait for the rest) */
    int32_t  resident_wait_us; /* 0 = library default (2 s); > 0: the bound, in microseconds,
                                after which a workgroup of that kernel stops waiting, sets
                                SOAR_STATUS_GAVE_UP and leaves (every workgroup then does)   */
    int32_t  tiles_per_wg_absmax; /* single-step path: the maximum pass and the search pass   */
    int32_t  tiles_per_wg_search; /* have launch shapes of their own (the library picks them by
                                the schedule: kernels of two launch groups share the GPU in a
                                batch of several groups).  0 = as tiles_per_wg says, else the
                                library's choice; 1 .. 65536 forces that pass (any count:
                                these two deal their tiles round-robin; tests and tuning:
                                outputs must not depend on it)                              */
} soar_params;

/* Fills *p with the single-step defaults: SOAR, block 16, T = 1, K = 4, beta = {1},
 * window candidates. */
void soar_default_params(soar_params *p);

/* Fills *p with the full algorithm's settings of App. B.3: T = 15, 101 factors
 * beta in [0.5, 1.5], the two enclosing E4M3 codes, early stop at 1e-3. */
void soar_paper_params(soar_params *p);

/*
 * Bytes of device workspace soar_quantize needs for a rows x cols tensor
 * (control words, per-workgroup partial sums of the tensor-wide reductions of
 * Eq. 5, and 4 bytes per block for the block ratio a/b carried from the statistics
 * pass to the search pass).  The workspace must be 256-byte aligned; its
 * contents need no initialisation and are undefined afterwards.  Returns 0 on a
 * bad argument.
 */
size_t soar_workspace_bytes(int64_t rows, int64_t cols, const soar_params *params);

/*
 * soar_quantize -- the hot path.
 *
 * method RTN (Sec. 3.1): alpha = max|W| / (6*448); Delta_i = E4M3(max|W_i| /
 * (6 alpha)) (Eq. 1); codes = Q_FP4(W / (alpha Delta)) (Eq. 2).
 * method SOAR (Algorithm 1, T = 1): starts from the RTN state with
 * Delta^q = Delta^d; alpha <- Eq. 5; Delta*_i <- Eq. 6, kept unrounded as the
 * quantization scale Delta^q; codes <- Q_FP4(W / (alpha Delta^q)); the stored
 * scale Delta^d is the E4M3 code among centre-K..centre+K (centre = E4M3
 * projection of Delta*, Appendix D) that minimises the block error of Eq. 8,
 * candidates being tried in the order 0,-1,+1,-2,+2,... and a later one winning
 * only if strictly better in binary32.
 *
 *
 * The iterated path (taken when params differ from T = 1, beta = {1}, window
 * candidates, or when a descriptor of soar_quantize_batch asks for the trace)
 * runs Algorithm 1 as printed: in every iteration alpha <- Eq. 5 from the
 * current codes and stored scales, Delta* <- Eq. 6, then for each factor beta in
 * ascending order codes = Q_FP4(W / (alpha Delta* beta)) and, for each stored-
 * scale candidate (window order as above, or lower code then upper code), the
 * Eq. 8 error; the first pair with the smallest binary32 error is kept.  After
 * each iteration the tensor's error (binary64 adjacent-pair tree over the block
 * errors) is compared with the previous one for the early stop.  With T = 1,
 * beta = {1} and window candidates both paths return the same bytes.
 * search_mode on the iterated path: FULL evaluates the error of every pair; AUTO
 * (grids of 4 to 128 factors) first forms the codes of every factor and evaluates
 * errors only for the factors at which a block's codes change -- a pair whose codes
 * equal those of the factor before it has the same errors and can never be strictly
 * better.  Both return the same bytes.
 *
 * d_w            in   weights, bf16 or fp32 (see conventions)
 * d_codes        out  rows*cols/2 bytes
 * d_scales       out  rows*cols/16 bytes
 * d_global_scale out  1 float: alpha (1.0 for an all-zero tensor)
 * d_sse          out  1 double, may be NULL: sum over blocks of the Eq. 8 error
 *                     of the emitted codes and scales (= Eq. 4).  The order of the
 *                     binary64 additions follows the launch shape: bit-identical
 *                     from call to call for the same call (same tiles_per_wg*
 *                     settings, same path: one launch / three passes, same
 *                     tensors in a batch: the library picks the shapes by the
 *                     number of launch groups), equal to within 1e-12 otherwise
 * d_status       out  1 int32, may be NULL: SOAR_STATUS_* bits
 * d_workspace    tmp  >= soar_workspace_bytes(), 256-byte aligned; calls that
 *                     share a workspace must be ordered on one stream
 */
soar_status soar_quantize(const void *d_w, soar_dtype dtype, int64_t rows, int64_t cols,
                          int64_t ld_elems, const soar_params *params,
                          uint8_t *d_codes, uint8_t *d_scales, float *d_global_scale,
                          double *d_sse, int32_t *d_status,
                          void *d_workspace, size_t workspace_bytes, void *hip_stream);

/*
 * soar_quantize_static -- soar_quantize for callers that cannot allocate device memory or have
 * none to hand over as a workspace: code running under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, results and errors as soar_quantize minus
 * the workspace: the control words and the 4 bytes per block come from a fixed array inside the
 * library's device image (SOAR_STATIC_MAX_BLOCKS blocks, about 19 MiB on every GPU the library
 * runs on, held until the process ends).  The call allocates and frees nothing -- no device
 * memory, no stream, no event (per-kernel timing is not recorded for it).
 *   - rows * cols / 16 > SOAR_STATIC_MAX_BLOCKS returns SOAR_ERR_TOO_LARGE before anything is
 *     enqueued;
 *   - all calls on one GPU share that array, which keeps the previous call's contents (the
 *     library clears what must start at zero): calls must be ordered on one stream, or otherwise
 *     serialised by the caller -- two that overlap on one GPU race;
 *   - the device current at the call must own hip_stream and the buffers; the first call on a
 *     device looks the array's address up and must therefore come before any graph capture.
 */
#define SOAR_STATIC_MAX_BLOCKS 4194304   /* 2^22 blocks = 2^26 weights, e.g. 8192 x 8192 */
soar_status soar_quantize_static(const void *d_w, soar_dtype dtype, int64_t rows, int64_t cols,
                                 int64_t ld_elems, const soar_params *params,
                                 uint8_t *d_codes, uint8_t *d_scales, float *d_global_scale,
                                 double *d_sse, int32_t *d_status, void *hip_stream);

/* One tensor of a batch: the arguments of soar_quantize that differ per tensor. */
typedef struct {
    const void *d_w;
    int32_t     dtype;           /* soar_dtype */
    int64_t     rows, cols, ld_elems;
    uint8_t    *d_codes;
    uint8_t    *d_scales;
    float      *d_global_scale;
    double     *d_sse;           /* may be NULL */
    int32_t    *d_status;        /* may be NULL */
    int32_t    *d_iters_run;     /* may be NULL; 1 int32: iterations carried out (0 for an
                                    all-zero or non-finite tensor)                      */
    double     *d_sse_trace;     /* may be NULL; iters+1 doubles: [0] the error of the
                                    Eq. 1-2 state, [t] the error after iteration t;
                                    entries after an early stop are not written         */
    const float *d_amax_in;      /* may be NULL; method RTN only, and then for all tensors
                                    of a batch or for none: 1 float, the tensor's maximum
                                    magnitude SUPPLIED (activation quantization, Appendix
                                    B.2: calibrated, or from an earlier pass) instead of
                                    measured.  The tensor is then read once: alpha =
                                    amax/(6*448), block scales clipped to 448, values above
                                    amax saturate at +-6.  Not finite or not > 0:
                                    SOAR_STATUS_BAD_AMAX.  The weights are not scanned for
                                    non-finite values in this mode.                      */
} soar_tensor_desc;

/*
 * soar_quantize_batch -- soar_quantize for n tensors (the linear layers of a
 * model, Sec. 4.1) on one stream with one shared workspace of at least
 * soar_batch_workspace_bytes().  Consecutive tensors of one element type are
 * served by the same kernel launches (up to 8 tensors and 256 MiB of weights
 * per launch, 512 MiB where the maxima are supplied and one pass remains), each
 * tensor with its own tensor-wide reductions; results are those
 * of n separate soar_quantize calls.  `descs` is HOST memory and is not
 * referenced after the call returns.  All descriptors are validated before
 * anything is enqueued.
 */
soar_status soar_quantize_batch(int32_t n, const soar_tensor_desc *descs, const soar_params *params,
                                void *d_workspace, size_t workspace_bytes, void *hip_stream);

/* Workspace bytes soar_quantize_batch needs for these n tensors (0 on a bad
 * argument).  Only shapes and element types of the descriptors are read. */
size_t soar_batch_workspace_bytes(int32_t n, const soar_tensor_desc *descs, const soar_params *params);

/*
 * soar_dequantize -- Eq. 3: w^_ij = q_ij * (alpha * d_i), the product alpha*d_i
 * rounded to binary32 first; bf16 output rounds to nearest even.
 * d_out: rows x cols with leading dimension ld_elems, 16-byte aligned.
 */
soar_status soar_dequantize(const uint8_t *d_codes, const uint8_t *d_scales,
                            const float *d_global_scale, int64_t rows, int64_t cols,
                            soar_dtype out_dtype, void *d_out, int64_t ld_elems, void *hip_stream);

/*
 * soar_recon_error -- Eq. 4: sum_ij (w_ij - q_ij * alpha * d_i)^2 for stored
 * codes / scales / global scale, each block evaluated as in Eq. 8 (binary32),
 * blocks accumulated in binary64.  *d_sse is overwritten.
 */
soar_status soar_recon_error(const void *d_w, soar_dtype dtype, int64_t rows, int64_t cols,
                             int64_t ld_elems, const uint8_t *d_codes, const uint8_t *d_scales,
                             const float *d_global_scale, double *d_sse, void *hip_stream);

/*
 * Eq. 3 and Eq. 4 for the stored tensors of a whole model in a handful of launches:
 * up to 8 tensors of one element type share a launch, as in soar_quantize_batch.
 * All pointers are device pointers, owned by the caller; nothing is allocated;
 * everything is enqueued on hip_stream.
 *
 * soar_stored_desc: d_codes (rows*cols/2 bytes, 8-byte aligned), d_scales
 * (rows*cols/16 bytes), d_global_scale (1 float) as soar_quantize wrote them;
 * rows, cols, ld_elems and dtype describe the weight matrix -- d_w, read by
 * soar_recon_error_batch (Eq. 4; d_sse: 1 double, overwritten), or d_out, written
 * by soar_dequantize_batch (Eq. 3); both 16-byte aligned with ld_elems * element
 * size a multiple of 16.  The fields the other call uses may be null.
 * Eq. 3 gives the bytes of the one-tensor call; the Eq. 4 sums agree with it up to
 * the order of the binary64 additions (workgroup partials are added atomically,
 * in both forms).  Errors are those of the one-tensor calls, found before anything
 * is enqueued; n = 0 is a no-op.
 */
typedef struct soar_stored_desc {
    const uint8_t *d_codes;
    const uint8_t *d_scales;
    const float   *d_global_scale;
    int64_t  rows, cols, ld_elems;
    int32_t  dtype;            /* soar_dtype of d_w / d_out */
    int32_t  reserved;         /* 0 */
    const void *d_w;           /* Eq. 4 */
    void     *d_out;           /* Eq. 3 */
    double   *d_sse;           /* Eq. 4 */
} soar_stored_desc;

soar_status soar_dequantize_batch(int32_t n, const soar_stored_desc *descs, void *hip_stream);
soar_status soar_recon_error_batch(int32_t n, const soar_stored_desc *descs, void *hip_stream);

/*
 * Element-wise projections onto the two small formats, exposed so that the
 * hardware conversion paths can be checked exhaustively (Sec. 3.1 Eq. 2;
 * Appendix D last equation).  d_x: n floats.  d_out: n bytes -- an E2M1 nibble
 * (sign<<3 | magnitude code, saturating, round to nearest even) or a clipped
 * E4M3 code in [0x01, 0x7E].
 */
soar_status soar_e2m1_round_f32(const float *d_x, int64_t n, uint8_t *d_out, void *hip_stream);
soar_status soar_e4m3_project_f32(const float *d_x, int64_t n, uint8_t *d_out, void *hip_stream);

/*
 * ---- Decoupled Scale Search on MXFP4 (Sec. 4.3 of the paper, "DSS on MXFP4") ----
 *
 * The paper names the format without restating it; it is taken from the public OCP
 * Microscaling Formats specification v1.0: blocks of 32 consecutive elements of a
 * row (cols % 32 == 0) share one E8M0 scale byte e in [0, 254], X = 2^(e-127); the
 * elements are E2M1 nibbles packed as for NVFP4; there is no tensor-wide scale.
 * Plain conversion: e0 = clamp(floor(log2 max|W_i|) - 2, -127, 127) + 127 (127 for a
 * block of zeros), codes = Q_FP4(W_i / X0), saturating.  With dss = 1 the stored
 * code is searched over e0-K .. e0+K (order 0,-1,+1,...; codes outside [0, 254]
 * skipped) jointly with the assignment scale X0 * beta_k (beta grid as in
 * soar_params, ascending), the error of a pair being Eq. 8 with alpha = 1 over the
 * 32 elements; a later pair wins only if strictly better in binary32.
 */
typedef struct {
    uint32_t struct_size;    /* sizeof(soar_mx_params)                               */
    int32_t  dss;            /* 0: plain conversion; 1: decoupled scale search       */
    int32_t  n_beta;         /* 1 .. 4096                                            */
    float    beta_lo;        /* 0 < beta_lo <= beta_hi                               */
    float    beta_hi;
    int32_t  radius;         /* K, 0 .. 127                                          */
    int32_t  tiles_per_wg;   /* 0 = chosen by the library; a power of two <= 65536   */
    int32_t  single_pass;    /* 0: the library's fastest exact search (grids of 4-128
                                factors: codes of every factor first, errors only where a
                                block's codes change); 1: evaluate every pair.  Same bytes. */
    int32_t  streams;        /* soar_mxfp4_quantize_batch: 0 = launch groups alternate between
                                the caller's stream and one internal stream (forked and joined
                                by events); 1 = everything on the caller's stream            */
} soar_mx_params;

/* dss = 1, 101 factors in [0.5, 1.5], K = 1 */
void soar_mx_default_params(soar_mx_params *p);

/* Bytes of device workspace soar_mxfp4_quantize needs (256-byte aligned, no
 * initialisation needed); 0 on a bad argument. */
size_t soar_mxfp4_workspace_bytes(int64_t rows, int64_t cols, const soar_mx_params *params);

/*
 * d_w       in   rows x cols, bf16 or fp32, leading dimension ld_elems, 16-byte aligned
 * d_codes   out  rows*cols/2 bytes, 16-byte aligned
 * d_scales  out  rows*cols/32 E8M0 bytes
 * d_sse     out  1 double, may be NULL: sum over blocks of the block errors
 *                (binary32 per block, binary64 adjacent-pair tree over blocks)
 * d_status  out  1 int32, may be NULL: SOAR_STATUS_NONFINITE if a value is NaN or
 *                Inf (outputs then unspecified), else 0
 * One pass over the data; asynchronous on hip_stream.
 */
soar_status soar_mxfp4_quantize(const void *d_w, soar_dtype dtype, int64_t rows, int64_t cols,
                                int64_t ld_elems, const soar_mx_params *params,
                                uint8_t *d_codes, uint8_t *d_scales, double *d_sse, int32_t *d_status,
                                void *d_workspace, size_t workspace_bytes, void *hip_stream);

/* One tensor of an MXFP4 batch: the arguments of soar_mxfp4_quantize that differ per tensor. */
typedef struct {
    const void *d_w;
    int32_t     dtype;           /* soar_dtype */
    int64_t     rows, cols, ld_elems;
    uint8_t    *d_codes;
    uint8_t    *d_scales;
    double     *d_sse;           /* may be NULL */
    int32_t    *d_status;        /* may be NULL */
} soar_mx_tensor_desc;

/*
 * soar_mxfp4_quantize for n tensors on one stream with one workspace of at least
 * soar_mxfp4_batch_workspace_bytes(): up to 8 consecutive tensors of one element
 * type (and at most 512 MiB of input) share a kernel launch; results are those of n separate calls.  `descs` is
 * HOST memory, not referenced after the call returns; all descriptors are
 * validated before anything is enqueued.
 */
soar_status soar_mxfp4_quantize_batch(int32_t n, const soar_mx_tensor_desc *descs,
                                      const soar_mx_params *params, void *d_workspace,
                                      size_t workspace_bytes, void *hip_stream);
size_t soar_mxfp4_batch_workspace_bytes(int32_t n, const soar_mx_tensor_desc *descs,
                                        const soar_mx_params *params);

/* w^_ij = q_ij * X_i; bf16 output rounds to nearest even.  A scale byte 255 (NaN
 * in E8M0) leaves its block unwritten. */
soar_status soar_mxfp4_dequantize(const uint8_t *d_codes, const uint8_t *d_scales, int64_t rows,
                                  int64_t cols, soar_dtype out_dtype, void *d_out, int64_t ld_elems,
                                  void *hip_stream);

/* The same for n stored tensors in a handful of launches (up to 8 tensors of one element type
 * per launch): soar_stored_desc with d_codes (16-byte aligned), d_scales (E8M0 bytes), rows, cols
 * (a multiple of 32), ld_elems, dtype and d_out; the other fields are not read.  The bytes are
 * those of n one-tensor calls; errors are found before anything is enqueued. */
soar_status soar_mxfp4_dequantize_batch(int32_t n, const soar_stored_desc *descs, void *hip_stream);

/*
 * The reciprocal used inside the iterated path's search loop (hardware estimate
 * plus one fused Newton step), exposed so that the claim it rests on can be
 * checked exhaustively: for every positive binary32 x whose biased exponent lies
 * in [1, 252] the result is bit-identical to the correctly rounded 1/x.  (The
 * kernel falls back to the division outside that range.)  d_x, d_out: n floats.
 */
soar_status soar_rcp_midrange_f32(const float *d_x, int64_t n, float *d_out, void *hip_stream);

/*
 * Per-kernel timing for benchmarks.  While enabled, every kernel the library
 * launches is bracketed by HIP events on its stream (events without the
 * system-scope fence: they measure and order nothing).  soar_kernel_timing_read
 * synchronises, returns total milliseconds and launch count of one kernel
 * family since the last reset, and soar_kernel_timing_enable(…) resets.
 * (SOAR_KERNEL_ITER: one bracket round all iteration launches of a launch group,
 * counted as one.)
 * Not thread-safe; leave disabled in production.
 */
typedef enum {
    SOAR_KERNEL_INIT = 0, SOAR_KERNEL_ABSMAX = 1, SOAR_KERNEL_STATS = 2, SOAR_KERNEL_SEARCH = 3,
    SOAR_KERNEL_DEQUANT = 4, SOAR_KERNEL_RECON = 5, SOAR_KERNEL_ITER_INIT = 6, SOAR_KERNEL_ITER = 7,
    SOAR_KERNEL_MX = 8, SOAR_KERNEL_RESIDENT = 9, SOAR_KERNEL_COUNT = 10
} soar_kernel_id;
void        soar_kernel_timing_enable(int enable);
soar_status soar_kernel_timing_read(int kernel_id, double *total_ms, int64_t *launches);

/*
 * Diagnostics of the Eq. 8 search in SOAR_SEARCH_AUTO (single-step path): the library evaluates the two
 * candidates that enclose the block's least-squares scale and hands over to the exhaustive loop where it
 * cannot show that their winner is the exhaustive winner; since a wave walks one block per lane, one such
 * block makes its whole wave wait for the loop.  soar_search_stats_enable(1) zeroes the counters of the
 * current device (it synchronises the device) and makes every later launch count; (0) stops the counting.
 * soar_search_stats_read synchronises the device and returns counts[0] blocks searched, [1] blocks handed
 * over, [2] wave steps, [3] wave steps with at least one block handed over.  Counting costs atomics: leave
 * it off when timing.  Not thread-safe.
 */
soar_status soar_search_stats_enable(int enable);
soar_status soar_search_stats_read(int64_t counts[4]);

/*
 * For tests: the counting plan of the kernels' "last workgroup of a tensor finishes the reduction"
 * hand-off (host arithmetic only, no GPU needed).  Of a tensor's n_workgroups workgroups, workgroup w
 * counts itself in on first-level counter out[1] of out[0] counters in use, which out[2] workgroups
 * share; the workgroup that brings a first-level counter to its out[2] counts on the top counter, and
 * the one that brings that to out[0] is the last.  Leaves `out` untouched on a bad argument.
 */
void soar_debug_arrival_plan(uint32_t n_workgroups, uint32_t workgroup, uint32_t out[3]);

const char *soar_status_string(soar_status s);
uint32_t    soar_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SOAR_H */
