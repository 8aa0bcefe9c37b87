/*
 * demo.h -- C ABI of the MI355X (gfx950) implementation of DeMo's per-step
 * compression path (arXiv 2411.19870).
 *
 * The entry points follow the paper's algorithm statement: Algorithm 1 ("DeMo:
 * Decoupled Momentum") takes learning rate eta, momentum coefficient beta, weight
 * decay lambda, sparsity budget k and the DCT matrices (fixed by the chunk size
 * s); the appendix algorithm "Decoupled Momentum Optimization" lists the same
 * inputs plus the chunk sizes.  One call processes a whole list of tensors.
 *
 * Conventions
 *   - All tensor and payload pointers are DEVICE pointers owned by the caller; the
 *     library never frees or keeps them after the call returns.  `demo_tensor`
 *     arrays themselves are HOST memory and are copied during the call.
 *   - grad, mom and param must be 16-byte aligned (the kernels move rows with 16-byte accesses); idx and val
 *     need only 4-byte alignment (16-byte aligned payload arrays get the widest loads).  DEMO_ERR_ARG otherwise.
 *   - Tensors are dense row-major.  cols == 0 marks an order-1 tensor of `rows`
 *     elements, chunked into pieces of s; otherwise the tensor is rows x cols and
 *     is chunked into s x s blocks (appendix "Multilinear Transforms and
 *     Chunk-wise Tensor Blocking": block (k0,k1) holds X[k0*s+j0, k1*s+j1]).
 *     rows and cols must be multiples of s.  Chunks are numbered row-major over
 *     (k0, k1).
 *   - Payload of one worker for one tensor: idx[nchunks][k] (int32) and
 *     val[nchunks][k] (float32).  idx is the flat position u*s + v of a DCT
 *     coefficient inside its chunk, u being the frequency along dimension 0 (for
 *     order-1 tensors simply u).  Encode lists the k pairs of a chunk by
 *     descending magnitude, equal magnitudes by ascending index.  For decode the
 *     payloads of W workers are stacked worker-major: idx[W][nchunks][k],
 *     val[W][nchunks][k]; encode writes worker slot 0 of such a buffer.
 *   - Calls are asynchronous: work is enqueued on `hip_stream` (a hipStream_t
 *     passed as void*, NULL = default stream) and results are valid after that
 *     stream has been synchronised.  The context keeps the descriptor tables of the
 *     8 most recently used tensor lists (a list = the demo_tensor array's contents,
 *     buffer addresses included, and s); a call with one of them only launches
 *     kernels.  The first 8 distinct lists each cost one device allocation and one
 *     blocking copy; after that a new list reuses the memory of the least recently
 *     used one and its table is written by a small kernel on `hip_stream`, without
 *     allocation or host synchronisation (the device is synchronised first only if
 *     the evicted list was last used on another stream or its memory is too small).
 *     A list first used under stream capture must have been seen before the capture
 *     began; lists used under capture are never evicted.
 *   - Every function returns DEMO_OK (0) or a negative demo_status.  Arguments
 *     are validated on the host before anything is enqueued; on error nothing
 *     was launched.  No exceptions cross this boundary.
 *   - A context may be used from one host thread at a time.
 */
#ifndef DEMO_H_
#define DEMO_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct demo_ctx demo_ctx;

typedef enum demo_status {
  DEMO_OK = 0,
  DEMO_ERR_ARG = -1,         /* null pointer, n < 0, W < 1, k < 1, k > M (M = s or s*s)   */
  DEMO_ERR_SHAPE = -2,       /* rows or cols not a positive multiple of s                 */
  DEMO_ERR_UNSUPPORTED = -3, /* s not in {32,64,128}, unknown dtype, k > DEMO_MAX_K,
                                more than 2^31 - 1 chunks in a tensor or in a call,
                                cols >= DEMO_MAX_COLS                                      */
  DEMO_ERR_HIP = -4,         /* a HIP runtime call failed (see demo_last_hip_error)       */
  DEMO_ERR_NOMEM = -5,       /* host or device allocation for the context's tables failed */
  DEMO_ERR_LIMIT = -6        /* demo_encode_noalloc: the tensor list exceeds the static scratch array */
} demo_status;

typedef enum demo_dtype { DEMO_F32 = 0, DEMO_BF16 = 1 } demo_dtype;

/* Largest supported sparsity budget per chunk (the paper uses k <= 32). */
#define DEMO_MAX_K 256
/* Most workers demo_decode_ex / demo_step_ex accept with phi = DEMO_PHI_IDENTITY (see demo_hparams). */
#define DEMO_MAX_W_IDENTITY 1024
/* Order-2 tensors must have fewer columns than this: the kernels address the rows of a chunk with 32-bit byte
 * offsets from the chunk's origin (128 rows of 4-byte elements stay below 2^31). */
#define DEMO_MAX_COLS (1 << 22)

/* One tensor of the list.  64 bytes, no implicit padding. */
typedef struct demo_tensor {
  const void* grad;    /* device; gradient g, grad_dtype; read by encode/step; may be NULL for decode  */
  float*      mom;     /* device; momentum m (float32); updated in place by encode/step; NULL for decode */
  void*       param;   /* device; parameters x, param_dtype; updated in place by decode/step; NULL for encode */
  int32_t*    idx;     /* device; payload indices, see above                                           */
  float*      val;     /* device; payload values, see above                                            */
  int64_t     rows;    /* > 0                                                                           */
  int64_t     cols;    /* 0 for an order-1 tensor                                                       */
  int32_t     grad_dtype;   /* demo_dtype */
  int32_t     param_dtype;  /* demo_dtype */
} demo_tensor;

/* Create / destroy a context.  The context owns the DCT basis tables (built on
 * the host in double precision, rounded once to float32, one per chunk size) and
 * the cached device copies of tensor descriptor tables.  demo_create performs no
 * GPU call; device memory is allocated on first use.  */
int demo_create(demo_ctx** out);
int demo_destroy(demo_ctx* ctx);

/* Host-only helper: number of (idx, val) pairs one worker's payload has for a
 * tensor, nchunks * k (Sec. 2.1 "Top-k Sparsification": k coefficients per chunk,
 * a reduction of (prod s_i)/k).  Validates shape, s and k like the calls below. */
int demo_payload_elems(int64_t rows, int64_t cols, int s, int k, int64_t* out);

/* Worker side of Algorithm 1 for every tensor of the list (appendix algorithm
 * CompressChunks):   m <- beta*m + g;  per chunk Q = DCT(m), keep the k
 * largest-magnitude coefficients (exactly k), write them to idx/val (worker slot
 * 0), and m <- m - IDCT(kept).  Requires grad, mom, idx, val.
 * Arithmetic (all entry points): sums are accumulated in float32; the products of the
 * transforms are float32 multiplications or, in some kernels, multiplications of float32
 * operands carried as two float16 parts (22 significant bits, at a power-of-two scale
 * taken from the chunk).  Payload values and momentum come out within 1e-5 of the
 * chunk's largest magnitude of the exact result (measured below 1e-6), whatever the
 * absolute scale of the data between about 2^-100 and 2^100.  */
int demo_encode(demo_ctx* ctx, const demo_tensor* tensors, int n, float beta, int s, int k,
                void* hip_stream);

/* demo_encode for callers that cannot allocate device memory or synchronise: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and the same results as
 * demo_encode, but the tables the kernels read beside the tensors (DCT basis tables, tensor descriptors, the
 * queue of chunks handed to the exact top-k kernel) live in a static device array of DEMO_NOALLOC_SCRATCH_BYTES
 * that every GPU the library runs on holds until the process ends, and they are written there by small kernels
 * on `hip_stream`: the call performs no hipMalloc, hipFree, memory copy or synchronisation, whether or not the
 * list has been seen before.
 *   Limits: n <= DEMO_NOALLOC_MAX_TENSORS, at most DEMO_NOALLOC_MAX_CHUNKS order-2 chunks in the call, the DCT
 *   basis only (DEMO_ERR_UNSUPPORTED after demo_set_basis chose another matrix for s).  DEMO_ERR_LIMIT beyond
 *   them; nothing is launched then.
 *   All calls on one GPU share the one array (from any context or thread): calls of this entry point that
 *   overlap in time on one GPU race; issue them on one stream, or order the streams.  It is not used by any
 *   other entry point.  demo_set_timing does not cover it.  */
#define DEMO_NOALLOC_MAX_TENSORS 1024
#define DEMO_NOALLOC_MAX_CHUNKS (1 << 20)
#define DEMO_NOALLOC_SCRATCH_BYTES (128 * 1024 + 256 * 1024 + 4 * DEMO_NOALLOC_MAX_CHUNKS + 4096)
int demo_encode_noalloc(demo_ctx* ctx, const demo_tensor* tensors, int n, float beta, int s, int k,
                        void* hip_stream);

/* Server side of Algorithm 1 (appendix algorithm Decompress&Aggregate followed by
 * the update line):  per chunk sum the coefficients of the W payloads (workers
 * added in order 0..W-1, pairs whose index is outside [0, M) are skipped),
 * m_t = IDCT(sum), then x <- x - lr*(sgn(m_t) + weight_decay*x) with sgn(0) = 0,
 * evaluated in float32 as t = fma(weight_decay, x, sgn), x' = fma(-lr, t, x) and
 * rounded to param_dtype (nearest-even).  Requires param, idx, val.  */
int demo_decode(demo_ctx* ctx, const demo_tensor* tensors, int n, int W, float lr,
                float weight_decay, int s, int k, void* hip_stream);

/* One full single-worker step: demo_encode followed by demo_decode with W = 1 on
 * the payload just written.  Requires every pointer of demo_tensor.  */
int demo_step(demo_ctx* ctx, const demo_tensor* tensors, int n, float beta, float lr,
              float weight_decay, int s, int k, void* hip_stream);

/* The paper's other operating points (all scalar or per-element changes of the two
 * calls above).  demo_hparams_default fills in the algorithm boxes' values, with
 * which the _ex calls below are identical to demo_encode / demo_decode / demo_step.
 *   grad_scale    coefficient of g in the momentum update m <- beta*m + grad_scale*g; 1 in the
 *                 algorithm boxes, 1 - beta in the first display equation of Sec. 2.1.
 *   alpha         coefficient of the subtracted reconstruction, m <- m - alpha*IDCT(kept)
 *                 (display equation of "Momentum Subtraction as Error Feedback"; the ablation
 *                 "Impact of Momentum Subtraction" varies it in [0, 1], 0.2 being its best).  The
 *                 payload carries the kept coefficients themselves whatever alpha is.
 *   phi           DEMO_PHI_SIGN: x <- x - lr*(sgn(m_t) + weight_decay*x) (Signum);
 *                 DEMO_PHI_IDENTITY: x <- x - lr*(m_t + weight_decay*x) (SGD), same two float32
 *                 fused multiply-adds (update rule of "Momentum Reconstruction and Parameter
 *                 Update").  Muon's phi is not provided.  Accuracy of m_t under the identity: the
 *                 kernels sum a chunk's W payloads exactly, after rounding every value to a multiple
 *                 of 2^-(30 - ceil(log2 W)) of the chunk's largest payload magnitude (2^-24 of it at
 *                 W = 64, 2^-20 at W = 1024); the sign update is insensitive to that, the identity is
 *                 not, so it is limited to W <= DEMO_MAX_W_IDENTITY (DEMO_ERR_UNSUPPORTED beyond).
 *   aggregate     DEMO_AGG_SUM: plain sum over the W payloads (algorithm boxes);
 *                 DEMO_AGG_MEAN: sum / W (the AvgAllGather of "Top-k Sparsification");
 *                 DEMO_AGG_COUNT: each coefficient's sum divided by the number of workers that
 *                 sent it, 0/0 = 0 (appendix algorithm "Sparse Top-k Averaging"); needs W <= 255.
 * beta, lr, weight_decay as in the calls above.  DEMO_ERR_ARG for an unknown phi / aggregate, a
 * non-finite scalar, or DEMO_AGG_COUNT with W > 255.  32 bytes, no implicit padding.  */
typedef enum demo_phi { DEMO_PHI_SIGN = 0, DEMO_PHI_IDENTITY = 1 } demo_phi;
typedef enum demo_aggregate { DEMO_AGG_SUM = 0, DEMO_AGG_MEAN = 1, DEMO_AGG_COUNT = 2 } demo_aggregate;
typedef struct demo_hparams {
  float   beta;
  float   grad_scale;
  float   alpha;
  float   lr;
  float   weight_decay;
  int32_t phi;         /* demo_phi */
  int32_t aggregate;   /* demo_aggregate */
  int32_t reserved;    /* must be 0 */
} demo_hparams;
int demo_hparams_default(demo_hparams* hp, float beta, float lr, float weight_decay);
int demo_encode_ex(demo_ctx* ctx, const demo_tensor* tensors, int n, const demo_hparams* hp, int s, int k,
                   void* hip_stream);   /* uses beta, grad_scale, alpha */
int demo_decode_ex(demo_ctx* ctx, const demo_tensor* tensors, int n, int W, const demo_hparams* hp, int s,
                   int k, void* hip_stream);   /* uses lr, weight_decay, phi, aggregate */
int demo_step_ex(demo_ctx* ctx, const demo_tensor* tensors, int n, const demo_hparams* hp, int s, int k,
                 void* hip_stream);

/* Projection matrix used by later calls for chunk size s (ablation "Choice of Linear Projections"):
 *   DEMO_BASIS_DCT           the orthonormal DCT-II (default; a_host ignored);
 *   DEMO_BASIS_IDENTITY      P = I, no transformation (a_host ignored);
 *   DEMO_BASIS_GRAM_SCHMIDT  a_host points to s*s float32 values in HOST memory, row-major (the
 *                            paper draws them from N(0, 1) with the step number as seed, the same on
 *                            every worker; drawing them is the caller's business).  The rows are
 *                            orthonormalised in order by the Gram-Schmidt process in double precision
 *                            and rounded once to float32.  DEMO_ERR_ARG if they are linearly dependent.
 * The same matrix serves every dimension and both directions (inverse = transpose).  With a matrix
 * other than the DCT the calls run on the kernels that read the matrix from memory; the s = 64 / 32
 * wavefront kernels are specific to the DCT.  The call synchronises the device (kernels enqueued
 * earlier may still read the matrix it replaces) and copies s*s floats to it.  */
typedef enum demo_basis { DEMO_BASIS_DCT = 0, DEMO_BASIS_IDENTITY = 1, DEMO_BASIS_GRAM_SCHMIDT = 2 } demo_basis;
int demo_set_basis(demo_ctx* ctx, int s, int kind, const float* a_host);

/* Static text for a status code; hipGetErrorString of the last failing HIP call. */
const char* demo_strerror(int status);
const char* demo_last_hip_error(demo_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* DEMO_H_ */
