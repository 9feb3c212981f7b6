/*
 * signmuon.h -- C ABI of the MI355X (gfx950) Sign-Muon optimizer hot path.
 *
 * One optimizer iteration of Sign-Muon ("SignMuon: Communication-Efficient
 * Distributed Muon Optimization"), with the paper's M data-parallel workers
 * laid out as a leading array dimension on one GPU:
 *
 *   momentum (Alg. 1 steps 5-6)  ->  PolarNS (Alg. PolarNS / PowerIter)
 *   ->  entrywise sign, packed to 1 bit or kept as int8 (Alg. 3 / Alg. 2)
 *   ->  integer majority vote over the M workers (eq. mv_def)
 *   ->  optional local polar step on the voted sign matrix
 *   ->  W <- W - eta * D (Alg. 2 last step, eq. signmuon_update).
 *
 * Conventions for every entry point
 *   - Pointers are DEVICE pointers unless the comment says HOST.  Matrices are
 *     row-major.  The caller owns every buffer; nothing is retained after the
 *     call except by the work already queued on the context's stream.
 *   - All work is queued asynchronously on the HIP stream given to
 *     signmuon_create; the caller synchronises.  Calls on one context must not
 *     overlap from several host threads.
 *   - Return value: SM_OK (0) or a negative SM_E* code.  Arguments are checked
 *     on the host before anything is launched; on error nothing has been
 *     queued.  signmuon_last_error gives the text of the last failure.
 *   - Alignment: signmuon_step needs 16-byte aligned blocks; the single-stage
 *     calls accept element-aligned matrices (4 bytes fp32, 2 bytes bf16) and run
 *     their vector paths when pointers and sizes allow 16-byte accesses; packed
 *     sign buffers are 8-byte aligned.
 *   - Results are deterministic: no floating-point atomics are used.
 */
#ifndef SIGNMUON_H
#define SIGNMUON_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct signmuon_ctx signmuon_ctx; /* opaque; owns only its own workspaces */

/* status codes */
#define SM_OK 0
#define SM_EINVAL (-1)       /* bad argument (NULL, size, alignment, enum) */
#define SM_EUNSUPPORTED (-2) /* valid request this build does not implement */
#define SM_ENOMEM (-3)       /* device workspace allocation failed */
#define SM_EHIP (-4)         /* a HIP runtime call failed; see signmuon_last_error */

/* element type of a matrix argument */
#define SM_F32 0
#define SM_BF16 1

/* sigma of Alg. PolarNS */
#define SM_SCALE_FRO 0      /* sigma = ||X||_F */
#define SM_SCALE_SPECTRAL 1 /* sigma = PowerIter(X, P, eps) from a caller-supplied start vector */
#define SM_SCALE_NONE 2     /* sigma = 1 (idealized Newton-Schulz algorithm, caller pre-scaled) */

/* transport format of the per-worker signs */
#define SM_SIGN_1BIT 0 /* Alg. 3: bit = (x >= 0); entry i -> bit (i mod 64) of little-endian
                          64-bit word (i div 64), i.e. bit (i mod 8) of byte (i div 8);
                          padding bits of the last word are 0 */
#define SM_SIGN_INT8 1 /* Alg. 2: +1 / -1 as int8 */

/* format of the voted sign written by signmuon_majority_vote */
#define SM_VOTE_BITS 0 /* packed like SM_SIGN_1BIT */
#define SM_VOTE_INT8 1 /* +1 / -1 int8 [n] */
#define SM_VOTE_BF16 2 /* +1 / -1 bfloat16 [n] */
#define SM_VOTE_F32 3  /* +1 / -1 float [n] */

/* ---- context ---------------------------------------------------------- */

/* Creates a context bound to the current HIP device and to `hip_stream`
 * (a hipStream_t; NULL = the default stream).  *out is set on success.
 * workspace_bytes_hint: device bytes to reserve for signmuon_step's workspace right
 * away (0 = none).  The workspace is otherwise sized by the first signmuon_step /
 * signmuon_polar_ns call for a new set of shapes, which allocates, clears it and
 * may wait for the stream: such a first call must not be captured into a HIP graph.
 * Later calls for the same shapes only queue kernels. */
int signmuon_create(signmuon_ctx** out, void* hip_stream, size_t workspace_bytes_hint);
/* Waits for the stream, frees the context's workspaces. */
int signmuon_destroy(signmuon_ctx* ctx);

/* Tuning switches of a context.  Every setting computes the same path within the
 * same tolerances; they exist for measurements and tests.  Values other than the
 * listed ones give SM_EINVAL. */
#define SM_OPT_GEMM_TILE 0 /* workgroup tile of the Newton-Schulz GEMMs: 0 = by launch size (default), 128, 256 */
#define SM_OPT_NS_PATH 1   /* how the K steps of the cubic iteration are grouped: */
#define SM_NS_PATH_PAIRS 0    /*   short-side recurrence, two steps per quartic (default) */
#define SM_NS_PATH_SINGLE 1   /*   short-side recurrence, one step at a time */
#define SM_NS_PATH_STEPWISE 2 /*   Alg. PolarNS as written: Gram and apply of Y per step */
#define SM_OPT_NS_STORE 2  /* storage of the symmetric s x s matrices of the recurrence: */
#define SM_NS_STORE_UPPER 0   /*   blocks on and above the diagonal only (default) */
#define SM_NS_STORE_FULL 1    /*   whole matrices */
#define SM_OPT_POWER_ITER 3 /* passes of Alg. PowerIter over X: */
#define SM_PI_AUTO 0          /*   fused where that is faster by a launch-cost estimate (default) */
#define SM_PI_FUSED 1         /*   u = X v and X^T u from one read of X wherever the matrix is narrow enough */
#define SM_PI_SEPARATE 2      /*   one pass per product */
#define SM_OPT_COUNT 4
int signmuon_set_option(signmuon_ctx* ctx, int option, int value);
int signmuon_get_option(const signmuon_ctx* ctx, int option, int* value);
/* Static text for a status code. */
const char* signmuon_strerror(int status);
/* Text of the last error on this context ("" if none).  HOST string owned by ctx. */
const char* signmuon_last_error(const signmuon_ctx* ctx);
/* Bytes of device workspace the context currently holds. */
size_t signmuon_workspace_bytes(const signmuon_ctx* ctx);


/* ---- a1: weight decay + momentum (Alg. 1 steps 5-6; Alg. 2 steps 6-7) --- */
/* For every worker p < M:  g = grad[p] + weight_decay * w ;
 *                          mom[p] <- beta * mom[p] + (1 - beta) * g     (in place)
 * in float32 with every product and sum rounded separately (no FMA) and
 * (1 - beta) formed in float32.
 *   mom  [M][rows][cols] f32, in/out      grad [M][rows][cols] f32
 *   w    [rows][cols] f32, read only; may be NULL iff weight_decay == 0
 * Optional fused outputs (either may be NULL):
 *   x_bf16 [M][rows][cols] bfloat16 copy of the new momentum (round to nearest even)
 *   sumsq  [M] f32, sum of squares of the new momentum of each worker
 *          (||M||_F^2 for the Frobenius scale of PolarNS). */
int signmuon_momentum(signmuon_ctx* ctx, float* mom, const float* grad, const float* w,
                      int M, int rows, int cols, float beta, float weight_decay,
                      void* x_bf16, float* sumsq);

/* The same operation for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Arguments, results and
 * rounding are those of signmuon_momentum, bit for bit.  The per-chunk partial sums behind
 * `sumsq` go to a static device array of SM_NOALLOC_SCRATCH_BYTES that the library holds on
 * every GPU it runs on (instead of context scratch grown on demand); the call allocates and
 * frees nothing, takes no timing taps, and only queues kernels on the context's stream.
 * Limit: M * ceil(rows * cols / 1024) * 4 <= SM_NOALLOC_SCRATCH_BYTES, beyond it SM_EUNSUPPORTED
 * and nothing is queued.  All contexts of one GPU share the array: calls whose kernels may
 * overlap on one GPU (different streams, no ordering between them) race on it; calls on one
 * stream are ordered and safe.  Nothing in it needs clearing: every partial sum a call reads
 * was written by that call. */
#define SM_NOALLOC_SCRATCH_BYTES (4u << 20)
int signmuon_momentum_noalloc(signmuon_ctx* ctx, float* mom, const float* grad, const float* w,
                              int M, int rows, int cols, float beta, float weight_decay,
                              void* x_bf16, float* sumsq);

/* ---- a2-a4: PolarNS (Alg. PolarNS; Alg. PowerIter; idealized NS algorithm) */
/* In place on x[batch][rows][cols] (dtype SM_F32 or SM_BF16):
 *   Y0 = X / max(sigma, eps);  `steps` times  Y <- Y (a I + b A + c A^2), A = Y^T Y,
 * evaluated through the Gram matrix of the short side (Y Y^T when rows < cols;
 * the same polynomial of the singular values).  coeffs = {a, b, c} (HOST array);
 * the paper's iteration is {1.5, -0.5, 0}.  Arithmetic: Y in bf16 with fp32
 * accumulation on the matrix cores, whatever the storage type of x.  For the cubic
 * with |a| <= 1.5 the steps are regrouped in segments of at most 5: one Gram of Y,
 * products of s x s matrices (s = the short side; kept in IEEE half precision), one
 * apply to Y -- the same iteration up to rounding order.
 *   v0 [batch][cols] f32: PowerIter start vector per matrix; required iff
 *   scale == SM_SCALE_SPECTRAL (the paper's random sample, made an input). */
int signmuon_polar_ns(signmuon_ctx* ctx, void* x, int dtype, int batch, int rows, int cols,
                      const float* coeffs, int steps, int scale, int power_iters, float eps,
                      const float* v0);

/* ---- a5: sign extraction + packing (Alg. 3 "Pack signs to bits" and its
 *          encoding note; appendix "Packed 1-bit representation") ---------- */
/* u[batch][n] (SM_F32 or SM_BF16) -> out + b * out_stride_bytes for each b.
 *   SM_SIGN_1BIT: out_stride_bytes >= 8 * ceil(n / 64), multiple of 8; the
 *                 8 * ceil(n / 64) bytes of each row are written, padding bits 0.
 *   SM_SIGN_INT8: out_stride_bytes >= n; n bytes written per row.
 * The decision is the IEEE comparison x >= 0: -0.0 -> +1, NaN -> -1. */
int signmuon_sign_pack(signmuon_ctx* ctx, const void* u, int dtype, int batch, int64_t n,
                       int fmt, void* out, int64_t out_stride_bytes);

/* ---- a6 (+ a8): majority vote (eq. mv_def; Lemma "majority vote equals sign
 *          of a sum-reduction"; appendix "Majority vote from gathered bits") */
/* signs: M rows of stride_bytes each, in format `fmt` (the gathered buffer of
 * Alg. 3, or the M int8 buffers that Alg. 2 all-reduces).
 *   1-bit: c_i = number of set bits, vote_i = +1 iff 2 c_i >= M.
 *   int8 : s_i = sum of the M int8 values in int32, vote_i = +1 iff s_i >= 0.
 * Ties give +1.  Outputs, each optional (NULL to skip):
 *   voted  in format vfmt (bits: 8*ceil(n/64) bytes, padding bits 0)
 *   counts int32[n]: c_i (1-bit) or s_i (int8)
 *   w      f32[n]:   w_i <- w_i - lr_scaled * vote_i  in the same pass. */
int signmuon_majority_vote(signmuon_ctx* ctx, const void* signs, int fmt, int M, int64_t n,
                           int64_t stride_bytes, void* voted, int vfmt, int32_t* counts,
                           float* w, float lr_scaled);

/* ---- whole path over a set of weight blocks (Alg. 2 / Alg. 3) ---------- */
/* The struct and the arrays it points to are HOST memory, read during the call
 * only; the pointers stored in those arrays are DEVICE pointers. */
typedef struct signmuon_step_args {
  int32_t n_mats;            /* number of weight blocks L */
  int32_t M;                 /* workers */
  const int32_t* rows;       /* [n_mats] */
  const int32_t* cols;       /* [n_mats] */
  float* const* w;           /* [n_mats] -> f32 [rows][cols], in/out */
  float* const* mom;         /* [n_mats] -> f32 [M][rows][cols], in/out */
  const float* const* grad;  /* [n_mats] -> f32 [M][rows][cols] */
  float beta, weight_decay, lr, eps;
  float coeffs[3];           /* Newton-Schulz polynomial {a, b, c} */
  int32_t ns_steps;          /* K, before the sign */
  int32_t scale;             /* SM_SCALE_* (also used by the local polar step) */
  int32_t power_iters;       /* P, spectral only */
  const float* const* v0;    /* [n_mats] -> f32 [M][cols]; spectral only, else NULL.
                                The local polar step uses worker 0's vector. */
  int32_t sign_fmt;          /* SM_SIGN_1BIT or SM_SIGN_INT8 */
  int32_t local_polar_steps; /* K' >= 0; 0: D = voted sign */
  int32_t update_rsqrt_mn;   /* scale kappa of the update W <- W - lr kappa D:
                                0: 1 (Alg. 2);  1: 1 / sqrt(rows*cols) (eq. signmuon_update);
                                2: 1 / max(sigma, eps), sigma = PowerIter(voted sign, power_iters, eps,
                                   worker 0's v0): the "normalized sign" D = S / ||S||_op of the
                                   appendix; needs v0 and local_polar_steps == 0 */
  int32_t reserved;
  /* optional taps, arrays may be NULL and so may single entries */
  void* const* signs_out;     /* [n_mats] -> per-worker signs, M rows of
                                 8*ceil(d/64) bytes (1-bit) or d bytes (int8) */
  int32_t* const* counts_out; /* [n_mats] -> int32 [d] */
  void* const* u_out;         /* [n_mats] -> bf16 [M][rows][cols]: PolarNS output before the sign */
  void* const* d_out;         /* [n_mats] -> bf16 [rows][cols]: update direction D (the voted sign itself
                                 when update_rsqrt_mn == 2: its scale is a scalar) */
} signmuon_step_args;

int signmuon_step(signmuon_ctx* ctx, const signmuon_step_args* args);

/* ---- timing taps for benchmarks ---------------------------------------- */
/* signmuon_profile_enable takes a bit mask of kernel classes (bit SM_K_x set:
 * every launch of that class is bracketed with HIP events on the context's
 * stream; 0 = off, the default).  signmuon_profile_read waits for the stream
 * and returns the launch count and summed duration (ms) of one class since the
 * last signmuon_profile_reset. */
#define SM_K_MOMENTUM 0
#define SM_K_NS_GRAM 1
#define SM_K_NS_APPLY 2
#define SM_K_SIGN_PACK 3
#define SM_K_VOTE 4
#define SM_K_UPDATE 5
#define SM_K_OTHER 6
#define SM_K_NS_SMALL 7
#define SM_K_POWER_ITER 8
#define SM_K_COUNT 9
int signmuon_profile_enable(signmuon_ctx* ctx, unsigned class_mask);
int signmuon_profile_reset(signmuon_ctx* ctx);
int signmuon_profile_read(signmuon_ctx* ctx, int kernel_class, int64_t* launches, double* total_ms);
/* Work booked by the timed launches of a GEMM class since the last reset:
 * flop_executed = 2 * rows * cols * K summed over the output tiles the launch really
 *   computes (for a symmetric product: the tiles on and above the diagonal), with rows,
 *   cols and K clipped to the logical (unpadded) sizes;
 * flop_dense = 2*M*N*K over the same products as written (what a kernel without the
 *   symmetry saving would execute);
 * bytes = their operands and results, each counted once (its stored share for a
 *   symmetric matrix kept in upper-block storage).
 * Zero for the other classes.  Any of the three pointers may be NULL. */
int signmuon_profile_work(signmuon_ctx* ctx, int kernel_class, double* flop_executed, double* flop_dense,
                          double* bytes);
const char* signmuon_kernel_name(int kernel_class);

#ifdef __cplusplus
}
#endif
#endif /* SIGNMUON_H */
