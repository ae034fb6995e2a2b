/*
 * mdbf.h -- C ABI of the MI355X (gfx950) forward product for Multi-Envelope
 * Double Binary Factorization (MDBF).
 *
 * The format (paper Sec. 4.2, Eq. "me-dbf-basis"): a weight matrix W (m x n) is
 * replaced by
 *        What = U V,   U = SA o (A Q^T)  (m x k),   V = SB o (G B^T)  (k x n)
 * with shared sign bases SA in {+-1}^{m x k}, SB in {+-1}^{k x n} (SB is the
 * paper's S_b transposed), rank-l real envelope factors A (m x l), Q (k x l),
 * G (k x l), B (n x l), and `o` the Hadamard product.  In the paper's symbols
 * m = N, n = M, k = R.
 *
 * The operation (paper Sec. 3.2 "Inference", generalised through the per-factor
 * expansion of Eq. "me-dbf-expand"): for every token b
 *        Y[b,:] = What X[b,:]
 * evaluated as two envelope-scaled binary products,
 *        z = sum_s g^(s) o ( SB (b^(s) o x) ),    y = sum_t a^(t) o ( SA (q^(t) o z) ).
 *
 * Conventions
 *  - Every pointer named *_dev is DEVICE memory owned by the caller; the library
 *    never allocates, frees or keeps device memory.  Everything else is host memory.
 *  - All launches are asynchronous on `stream` (a hipStream_t passed as void*;
 *    NULL is the default stream).  No call synchronises or reads device memory on
 *    the host, so the forward calls can be captured into a HIP graph.
 *  - Every function returns 0 (MDBF_OK) or a negative mdbf_status; arguments are
 *    validated before the first HIP call, so bad arguments are reported on hosts
 *    without a GPU as well.
 *  - Device pointers must be 16-byte aligned.
 */
#ifndef MDBF_H
#define MDBF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MDBF_VERSION 100
#define MDBF_MAX_L 16          /* envelope rank supported: 1..16 (the paper sweeps l in {1,2,3,8,16}) */

typedef enum {
  MDBF_OK = 0,
  MDBF_EINVAL = -1,        /* null pointer, non-positive shape, l out of range, T < 1, bad leading dimension */
  MDBF_EALIGN = -2,        /* a device pointer is not 16-byte aligned */
  MDBF_EDTYPE = -3,        /* unknown dtype code */
  MDBF_EWORKSPACE = -4,    /* workspace / output buffer too small */
  MDBF_EUNSUPPORTED = -5,  /* valid request this build cannot serve */
  MDBF_EHIP = -6           /* a HIP call failed; mdbf_last_hip_error() gives the text */
} mdbf_status;

typedef enum { MDBF_F16 = 0, MDBF_BF16 = 1, MDBF_F32 = 2 } mdbf_dtype;

/* flags of mdbf_desc_t */
#define MDBF_FLAG_PRECISE 1u   /* fp32 vector arithmetic throughout (no fp16 staging, no matrix cores); slow */
#define MDBF_FLAG_ACCUMULATE 4u /* Y += What x instead of Y = What x: the terms of a residual stack
                                   What = sum_p What^(p) with independent sign bases (paper Sec. 3.2,
                                   "Residual Compensation", Eq. "dbf-residual-comp") are applied by one call each
                                   on the same Y; the additions happen in the precision of Y.  Two terms of
                                   one Y must not sit in the same plan: a plan's layers run in no defined order */
#define MDBF_FLAG_BLOCK_SCALED 2u /* take the block-scaled matrix-core variant wherever it applies (l = 16, fp16
                                     envelopes, T <= 16), also for launches too small to fill the device with it;
                                     without the flag the library picks the variant by launch size */
#define MDBF_FLAG_FP16_STAGED 8u  /* never take the block-scaled variant: the scaled activations are staged in fp16
                                     (a plan takes the block-scaled variant only if none of its layers carries
                                     this flag); excludes MDBF_FLAG_BLOCK_SCALED (MDBF_EINVAL) */

typedef struct {
  int32_t m, n, k, l;      /* What is m x n, inner rank k, envelope rank l */
  int32_t x_dtype;         /* dtype of X            (mdbf_dtype) */
  int32_t env_dtype;       /* dtype of A, Q, G, B   (mdbf_dtype) */
  int32_t y_dtype;         /* dtype of Y            (mdbf_dtype) */
  uint32_t flags;
} mdbf_desc_t;

/* Envelope factors, row-major with the l modes of one row contiguous (the paper's
 * A = [a^(1) ... a^(l)] stored as m rows of l values). */
typedef struct {
  const void* A_dev;  /* m x l */
  const void* Q_dev;  /* k x l */
  const void* G_dev;  /* k x l */
  const void* B_dev;  /* n x l */
} mdbf_env_t;

/* ---- storage accounting (host only) ------------------------------------------------
 * Bits per weight: bit-packed signs plus the real envelope entries over the m*n entries
 * replaced (paper Sec. 3.2, last sentence of "Inference", applied to the factors listed
 * under Eq. "me-dbf-basis"):  [ (m+n)k + env_bits*l*(m+n+2k) ] / (mn).
 * merge_inner != 0 (only with l == 1) counts q o g as one vector, the plain DBF count.
 * Returns a negative value on invalid arguments. */
double mdbf_bpw(int m, int n, int k, int l, int env_bits, int merge_inner);

/* Inner rank for a bits-per-weight budget (paper Sec. 5.1, "largest inner rank that meets
 * the budget").  multiple <= 1: the largest k with mdbf_bpw <= bpw.  multiple > 1: the real
 * solution of mdbf_bpw(k) = bpw rounded to the nearest multiple (word-aligned ranks).
 * Returns k >= 0, or a negative mdbf_status. */
int mdbf_rank_for_budget(int m, int n, int l, double bpw, int env_bits, int multiple);

/* ---- sign bit-packing ("bit-packed sign matrices", paper Sec. 1 and Sec. 3.2) -------------
 * A sign matrix S (rows x cols) is contracted along `cols` in the forward product: for SA
 * rows = m, cols = k; for SB rows = k, cols = n.  One bit per entry, bit 1 <=> -1, in a
 * device tile layout private to this library (16-row tiles, 128-column blocks, padding bits 0).
 * mdbf_packed_bytes: size in bytes of the packed blob (host only). */
int mdbf_packed_bytes(int rows, int cols, size_t* bytes_out);

/* signs_dev: rows x cols int8, row-major with leading dimension ld >= cols; an entry < 0
 * packs as -1, an entry >= 0 as +1 (sign(0) = +1, paper Sec. 2).  packed_dev must hold
 * mdbf_packed_bytes(rows, cols) bytes (packed_bytes is checked) and is fully overwritten. */
int mdbf_pack(const int8_t* signs_dev, int rows, int cols, int64_t ld,
              void* packed_dev, size_t packed_bytes, void* stream);

/* Inverse of mdbf_pack: writes +1 / -1 into signs_dev (rows x cols int8, leading dim ld). */
int mdbf_unpack(const void* packed_dev, int rows, int cols,
                int8_t* signs_dev, int64_t ld, void* stream);

/* Envelope factor with zero modes appended (offline, like mdbf_pack): out_dev (rows x l_to, row-major)
 * receives env_dev (rows x l, row-major, elements of `dtype`) in its first l columns and zeros in the rest.
 * A layer whose four envelope factors are padded this way and whose descriptor says l_to denotes the same
 * What (paper Eq. "me-dbf-basis": the added modes are zero terms of the rank-l sums); ranks 8 and 16 with fp16
 * envelopes are the ones the matrix-core decode kernels serve, other ranks run the slower generic kernel.
 * l_to >= l, l_to <= MDBF_MAX_L; both pointers 16-byte aligned; the buffers must not overlap. */
int mdbf_pad_envelope(const void* env_dev, int rows, int l, int dtype, void* out_dev, int l_to, void* stream);

/* ---- forward product ------------------------------------------------------------------
 * Workspace bytes needed by mdbf_forward for T tokens (room for the inner vector z in fp32, for the
 * scaled activations of few-token calls, and for the partial sums of a one-token call).  Host arithmetic
 * only: the same value on every machine. */
int mdbf_workspace_bytes(const mdbf_desc_t* desc, int T, size_t* bytes_out);

/* Y[b,:] = What X[b,:] for b < T.
 *   SA_packed_dev  packed SA (m x k),  SB_packed_dev  packed SB (k x n)
 *   X_dev  T x n row-major, leading dimension ldx >= n (elements of x_dtype)
 *   Y_dev  T x m row-major, leading dimension ldy >= m (elements of y_dtype); overwritten
 *   workspace_dev / workspace_bytes  caller-owned scratch, >= mdbf_workspace_bytes()
 * Default arithmetic: fp32 accumulation on the matrix cores.  One token: z kept in fp32; the l-way
 * scaled activations (b^(s) o x and q^(t) o z) are quantised once -- to three fp6 limbs under a shared
 * power-of-two scale per 32 values (about 13 bits; the block-scaled variant, taken by single calls and large
 * plans of rank 8 or 16 with fp16 envelopes), or to fp16 (small plans, MDBF_FLAG_FP16_STAGED) -- and
 * contracted with the sign words.  A single one-token call of the block-scaled variant is two launches: each
 * factor's contraction is split across workgroups (a layer by itself cannot fill the device otherwise) and
 * the fp32 partial sums are added in a fixed order, so repeated calls return the same bits; they differ in
 * the last bits from what a plan returns for the same layer (another fixed order).  Two tokens or more: the factors
 * S_A o (A Q^T), S_B o (G B^T) are rebuilt piece by piece in fp16 and applied as dense products to the
 * fp16-rounded activations (x and z; z is stored in fp16 between the two products).  Magnitudes above
 * 65504 in those fp16 quantities overflow.
 * Range: the one-token variants carry their own power-of-two exponents (the block-scaled one per 32 values,
 * the fp16 one per 1024 columns of a scaled-activation vector) and keep z in fp32: they hold their accuracy
 * wherever the inputs and results are representable.  The general kernel (other ranks and envelope types) stages
 * b^(s) o x and q^(t) o z in plain fp16, divided by up to 8: magnitudes below about 5e-4 lose accuracy.  The
 * many-token variant needs the entries of A Q^T and
 * G B^T, the activations and z inside fp16's normal range (6e-5 .. 65504); What is unchanged when A is divided
 * and B multiplied by the same positive constant (likewise Q, G), so a layer can be rebalanced offline.
 * With MDBF_FLAG_PRECISE everything is fp32 vector arithmetic. */
int mdbf_forward(const mdbf_desc_t* desc,
                 const void* SA_packed_dev, const void* SB_packed_dev,
                 const mdbf_env_t* env,
                 const void* X_dev, int64_t ldx,
                 void* Y_dev, int64_t ldy, int T,
                 void* workspace_dev, size_t workspace_bytes, void* stream);

/* mdbf_forward without a workspace argument, for callers that cannot allocate device memory at all (code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc) and therefore have no
 * workspace to pass.  Same arguments, kernels, arithmetic and results as mdbf_forward; the scratch memory
 * (the inner vector z and the scaled activations) lives in a static device array of
 * MDBF_STATIC_SCRATCH_BYTES inside the library, which every GPU the library runs on holds until the process
 * ends.  The call allocates and frees nothing.  A request whose mdbf_workspace_bytes() exceeds
 * MDBF_STATIC_SCRATCH_BYTES returns MDBF_EWORKSPACE (checked on the host, before any HIP call): every layer
 * shape up to 11008 x 11008 with k <= 8192 fits with T <= 16; the 2048-token prefill does not.
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different streams,
 * or a captured graph replayed while another call runs) race on it; calls on one stream are ordered and safe.
 * The array keeps the last call's contents; no kernel depends on them.  The first call on a device looks up
 * the array's address (hipGetSymbolAddress): make it outside stream capture. */
#define MDBF_STATIC_SCRATCH_BYTES (16u << 20)
int mdbf_forward_static(const mdbf_desc_t* desc,
                        const void* SA_packed_dev, const void* SB_packed_dev,
                        const mdbf_env_t* env,
                        const void* X_dev, int64_t ldx,
                        void* Y_dev, int64_t ldy, int T, void* stream);

/* ---- many independent layers in one pair of launches -----------------------------------
 * One entry per layer; the same meaning as the arguments of mdbf_forward.  Serves sibling
 * projections and whole stacks of independent products with two kernel launches in total. */
typedef struct {
  mdbf_desc_t desc;
  const void* SA_packed_dev;
  const void* SB_packed_dev;
  mdbf_env_t env;
  const void* X_dev;
  int64_t ldx;
  void* Y_dev;
  int64_t ldy;
  int32_t T;
} mdbf_layer_t;

/* Sizes of the plan (a table the kernels read) and of the device workspace for `count` layers. */
int mdbf_batch_plan_bytes(int count, const mdbf_layer_t* layers, size_t* plan_bytes_out,
                          size_t* workspace_bytes_out);

/* Fills plan_host (plan_bytes from mdbf_batch_plan_bytes; any alignment) for the given layers and workspace
 * address.  The caller copies the plan verbatim to device memory (plan_dev, 16-byte aligned) before calling
 * mdbf_forward_batch and keeps plan_host alive: the host reads launch sizes from it. */
int mdbf_batch_plan_build(int count, const mdbf_layer_t* layers, void* workspace_dev,
                          size_t workspace_bytes, void* plan_host, size_t plan_bytes);

/* Runs all layers of a plan.  Asynchronous on `stream`, no allocation, no host-device copy. */
int mdbf_forward_batch(const void* plan_host, const void* plan_dev, size_t plan_bytes, void* stream);

/* Name of the product kernel a built plan runs for `stage` (1 = first factor, 2 = second factor): one of
 * "stage_mx_kernel" (block-scaled), "stage_fast_kernel" (fp16-staged), "stage_gemm_kernel" (many tokens),
 * "stage_generic_kernel", "stage_precise_kernel"; "" for an invalid plan or stage.  Host only; the string is
 * static.  For reports that must name the kernel they timed. */
const char* mdbf_batch_plan_kernel(const void* plan_host, size_t plan_bytes, int stage);

/* Kernel launches one mdbf_forward_batch of the plan issues (host only): 4 for the block-scaled and fp16-staged
 * kernels with a scale-in launch per factor, 3 when both factors run the block-scaled kernel (the first factor's
 * launch writes the second factor's activation records itself), 2 for the others; a negative status for an
 * invalid plan. */
int mdbf_batch_plan_launches(const void* plan_host, size_t plan_bytes);

/* Runs a part of a plan, for measuring its kernels one by one: `stages` and `kernels` are bit masks.
 * stages: 1 = first factor (x -> z), 2 = second factor (z -> y).  kernels: 1 = the scale-in kernel of the
 * stage (plans that have none skip it: also the second factor of a three-launch plan, whose records the first
 * factor's product kernel writes), 2 = the product kernel.  mdbf_forward_batch is (3, 3).  Results are
 * only meaningful if the caller preserves the order scale-in -> product, stage 1 -> stage 2. */
int mdbf_forward_batch_part(const void* plan_host, const void* plan_dev, size_t plan_bytes, int stages,
                            int kernels, void* stream);

/* Measurement aid: reads `bytes` bytes at src_dev once with plain 16-byte loads and folds them with XOR;
 * wave w of the launch stores the fold of the 32-bit words it read in sink_dev[w].  The launch has
 * sink_words waves (sink_words / 4 workgroups of 256 lanes; element i of the buffer, in 16-byte units, is
 * read by lane i mod (64 * sink_words)), so the XOR of sink_dev[0 .. sink_words) is the XOR of all 32-bit
 * words of the buffer.  Timed over a buffer far larger than the caches it gives the read bandwidth a kernel
 * can reach on this device, the yardstick next to the nominal HBM peak for the decode kernels (whose
 * work is streaming the packed signs of paper Sec. 3.2 once).
 * bytes: positive multiple of 16; sink_words: multiple of 4 in [4, 1 << 20]; pointers 16-byte aligned. */
int mdbf_stream_read(const void* src_dev, size_t bytes, uint32_t* sink_dev, int sink_words, void* stream);

/* ---- quantizer projection (offline) ----------------------------------------------------------
 * MSVID_l of a real matrix Z (paper Sec. 4.2, Eq. "msvid-def"): the sign mask S = sign(Z) (sign(0) = +1) and the
 * best rank-l approximation of |Z| in Frobenius norm, A Q^T = TSVD_l(|Z|), with the singular values split
 * evenly between A (rows x l) and Q (cols x l); S o (A Q^T) is the member of the format nearest to Z for the
 * mask S (Theorem 1, Eq. "Ustar"), at a distance of the tail of |Z|'s spectrum (Eq. "rankl-error").  This is
 * the projection the layer-wise optimisation applies to each factor (Eq. "admm-U-prox"); applied to a factor
 * U (N x R) it yields S_a, A, Q of the stored format, and to V (M x R) it yields S_b, B, G.
 * The truncated SVD is a block subspace iteration with b = mdbf_msvid_block(l) columns (l plus 8 to 15 of
 * oversampling) started from the caller's block X0 (cols x b, row-major, linearly independent columns: e.g.
 * seeded normal deviates; the library draws no random numbers) and ended by a Rayleigh-Ritz step; `iters`
 * (0 .. 64) is the number of passes (each is one product with |Z| and one with |Z|^T).  The result is the
 * exact TSVD_l once the iteration has converged: the error A Q^T leaves exceeds the optimum by a factor that
 * falls geometrically with iters at the rate of the gap between |Z|'s singular values l and b + 1.
 *   Z_dev      rows x cols, row-major fp32, leading dimension ld >= cols
 *   S_dev      rows x cols int8 (+1 / -1), row-major, ld = cols: the input mdbf_pack takes
 *   A_dev, Q_dev   rows x l and cols x l fp32, row-major;  sigma_dev  b Ritz values (fp32, descending; the first l
 *              are the singular values of A Q^T)
 *   workspace_dev  caller-owned, >= mdbf_msvid_workspace_bytes (a transposed copy of Z and the iteration's blocks)
 * Needs b <= min(rows, cols) (else MDBF_EUNSUPPORTED), 1 <= l <= MDBF_MAX_L, pointers 16-byte aligned.
 * Asynchronous on `stream`; no host synchronisation, no allocation; deterministic (fixed summation orders). */
int mdbf_msvid_block(int l);
int mdbf_msvid_workspace_bytes(int rows, int cols, int l, size_t* bytes_out);
int mdbf_msvid(const float* Z_dev, int rows, int cols, int64_t ld, int l, int iters, const float* X0_dev,
               int8_t* S_dev, float* A_dev, float* Q_dev, float* sigma_dev, void* workspace_dev,
               size_t workspace_bytes, void* stream);

/* ---- misc ----------------------------------------------------------------------------- */
const char* mdbf_strerror(int status);
const char* mdbf_last_hip_error(void);   /* text of the last failed HIP call on this thread, or "" */
int mdbf_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MDBF_H */
