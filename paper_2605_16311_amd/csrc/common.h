// Internal declarations shared by the HIP sources of libsignmuon (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string>
#include <vector>

#include "../../include/signmuon.h"

typedef __bf16 bf16_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;
typedef __attribute__((ext_vector_type(4))) int i32x4;

// ---------------------------------------------------------------- context
struct sm_event_pair {
  hipEvent_t a, b;
};

struct signmuon_ctx {
  hipStream_t stream = nullptr;
  int device = 0;
  std::string last_error;

  // Workspaces: one growable device arena each, sub-allocated by a cached Newton-Schulz plan
  // (shape classes + offsets).  Slot SM_WS_STEP serves signmuon_step, SM_WS_NS signmuon_polar_ns,
  // so that calls of the two interleave without replanning.  `arena` is the arena of the slot
  // in use by the running call.
  struct workspace {
    void* arena = nullptr;
    size_t bytes = 0;
    struct ns_plan* plan = nullptr;
  } ws[2];
  void* arena = nullptr;
  // small scratch of the standalone entry points (partial sums of signmuon_momentum)
  void* aux = nullptr;
  size_t aux_bytes = 0;

  // device address of the library's static scratch array on this context's device
  // (signmuon_momentum_noalloc); fixed size SM_STATIC_SCRATCH_BYTES
  void* static_scratch = nullptr;

  // tuning switches (signmuon_set_option)
  int opt[SM_OPT_COUNT] = {};
  int n_cu = 256;  // compute units of the device
  int gemm_flip = 0;  // parity of the GEMM launches so far: every other launch walks its tile ranges backwards

  // timing taps
  unsigned profiling = 0;  // bit k set: launches of kernel class k are bracketed with events
  std::vector<sm_event_pair> ev_pool;        // every pair ever created
  size_t ev_used = 0;                        // pairs handed out since the last reset
  std::vector<std::pair<int, size_t>> ev_log;  // (kernel class, pool index)
  double work_flop[SM_K_COUNT] = {};         // flops of the output tiles that timed GEMM launches compute (logical sizes)
  double work_dense[SM_K_COUNT] = {};        // 2 M N K of the same products as written
  double work_bytes[SM_K_COUNT] = {};        // their operand + result bytes
};

int sm_fail(signmuon_ctx* ctx, int code, const std::string& msg);
int sm_hip_fail(signmuon_ctx* ctx, hipError_t e, const char* what);

#define SM_HIP(ctx, call)                                        \
  do {                                                           \
    hipError_t e__ = (call);                                     \
    if (e__ != hipSuccess) return sm_hip_fail(ctx, e__, #call);  \
  } while (0)

// Scoped launch bracket: records an event pair around a launch when profiling.
struct sm_launch_scope {
  signmuon_ctx* ctx;
  int klass;
  long idx = -1;
  sm_launch_scope(signmuon_ctx* c, int k);
  ~sm_launch_scope();
};

constexpr size_t SM_STATIC_SCRATCH_BYTES = SM_NOALLOC_SCRATCH_BYTES;
constexpr int SM_WS_STEP = 0, SM_WS_NS = 1;
// Ensures the arena of workspace `slot` holds at least `bytes` and makes it the current arena;
// contents (and the slot's plan) are lost when it grows.
int sm_arena_reserve(signmuon_ctx* ctx, int slot, size_t bytes);
// Ensures the auxiliary scratch holds at least `bytes`.
int sm_aux_reserve(signmuon_ctx* ctx, size_t bytes);

static inline int64_t sm_round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }
static inline bool sm_aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// ---------------------------------------------------------------- streaming kernels (stream.hip)
// Descriptor of one weight block for the grouped momentum launch.
struct sm_mom_desc {
  float* mom;          // [M][d]
  const float* grad;   // [M][d]
  const float* w;      // [d] or null
  bf16_t* x;           // [M][rows_p][ld] padded bf16 copy, or null
  float* partial;      // [M][chunks] per-chunk sums of squares, or null
  long long d;         // rows*cols
  long long x_stride;  // elements between workers in x
  int cols, ld;        // logical row length and padded row length of x
  int chunks;          // chunks per worker
  int block_begin;     // first workgroup of this block in the grouped launch
};
constexpr int SM_MOM_MAX_GROUP = 52;  // blocks per launch: the table rides in the kernel arguments (4 KB at most)
constexpr int SM_MOM_CHUNK = 1024;  // elements per workgroup: one 16-byte piece per thread (short-lived workgroups
                                    // keep the four streams of the momentum update close together in memory)

int sm_launch_momentum(signmuon_ctx* ctx, const sm_mom_desc* descs, int n, int M, float beta, float wd);
// sumsq[i] = sum_j partial[i*chunks + j], i < count (fixed order)
int sm_launch_reduce_partials(signmuon_ctx* ctx, const float* partial, int chunks, int count, float* sumsq);
// inv_sigma[i] = 1 / max(sqrt(sumsq[i]), eps)   (from_sq) or 1 / max(sumsq[i], eps)
int sm_launch_inv_sigma(signmuon_ctx* ctx, const float* sig, int count, float eps, bool from_sq, float* inv_sigma);
// Grouped form over a table of matrix classes, one launch: per class `count` items with
//   mode 0: sig = sum of the item's `chunks` partial sums of squares, inv = 1 / max(sqrt(sig), eps)
//   mode 1: inv = 1 / max(sig, eps)          mode 2: inv = value
struct sm_sigma_desc {
  const float* partial;
  float* sig;
  float* inv;
  int chunks, count, mode;
  float value;
  int block_begin;  // filled by the launcher
  int pad_;
};
constexpr int SM_SIGMA_MAX_GROUP = 64;
int sm_launch_sigma_group(signmuon_ctx* ctx, const sm_sigma_desc* descs, int n, float eps);

// Grouped sign pack: one launch over a table of matrices, `M` workers each.
struct sm_sp_desc {
  const void* u;            // [M][rows][ld]
  void* out;                // M rows of out_stride bytes
  long long n;              // rows * cols
  long long batch_stride;   // elements between workers in u
  long long out_stride;     // bytes
  long long bytes_per_row;  // filled by the launcher
  int cols, ld;
  int blocks_per_row, block_begin;  // filled by the launcher
};
constexpr int SM_SP_MAX_GROUP = 48;
int sm_launch_sign_pack_group(signmuon_ctx* ctx, const sm_sp_desc* descs, int n, int dtype, int fmt, int M);

// Grouped expanding vote (+ fused update): one launch over a table of matrices.
struct sm_vote_desc {
  const void* signs;
  long long n, stride_bytes;
  void* voted;       // non-bit formats only (SM_VOTE_INT8/BF16/F32), or null
  int32_t* counts;
  float* w;
  float lr;
  int M, vfmt, cols, ld;
  int block_begin;   // filled by the launcher
};
constexpr int SM_VOTE_MAX_GROUP = 48;
int sm_launch_vote_group(signmuon_ctx* ctx, const sm_vote_desc* descs, int n, int fmt);

// Grouped update after a local polar step: w[r][c] -= step * d[r][ld]
struct sm_upd_desc {
  float* w;
  const bf16_t* d;
  const float* kappa;  // optional device scalar multiplied into step
  int rows, cols, ld;
  float step;
  int block_begin;   // filled by the launcher
  int pad_;
};
constexpr int SM_UPD_MAX_GROUP = 64;
int sm_launch_update_group(signmuon_ctx* ctx, const sm_upd_desc* descs, int n);

// sign pack from a (possibly padded) 2-D source: u[batch][rows][ld] -> flat row-major bits
int sm_launch_sign_pack(signmuon_ctx* ctx, const void* u, int dtype, int batch, int rows, int cols,
                        int ld, long long batch_stride, int fmt, void* out, long long out_stride_bytes);

struct sm_vote_args {
  const void* signs;
  int fmt, M;
  long long n, stride_bytes;
  void* voted;
  int vfmt;          // SM_VOTE_*; for BF16/F32 the destination may be 2-D padded:
  int cols, ld;      // voted element i goes to (i / cols) * ld + (i % cols); ld == cols: flat
  int32_t* counts;
  float* w;
  float lr_scaled;
};
int sm_launch_vote(signmuon_ctx* ctx, const sm_vote_args& a);

// w[r][c] -= step * d[r][ld] (bf16 d)
int sm_launch_update(signmuon_ctx* ctx, float* w, const bf16_t* d, int rows, int cols, int ld, float step);

// ---------------------------------------------------------------- layout helpers (layout.hip)
// dst[b][rows_p][ld] (bf16, padding untouched) <- src[b][rows][cols] (f32 or bf16)
int sm_launch_copy_in(signmuon_ctx* ctx, const void* src, int dtype, int batch, int rows, int cols,
                      bf16_t* dst, int ld, long long dst_stride);
// dst[b][rows][cols] (f32 or bf16) <- scale[b] * src[b][rows][ld]; scale may be null
int sm_launch_copy_out(signmuon_ctx* ctx, const bf16_t* src, int ld, long long src_stride, int batch, int rows,
                       int cols, void* dst, int dtype, const float* scale);
// Writes zeros over the padding (columns cols..cp, rows rows..rp) of `items` matrices [rp][cp], `stride`
// elements apart: the working layout relies on padding that reads as zero, and a non-finite input would
// otherwise leave NaN there for every later call (0 * NaN in a product's padded rows).
struct sm_pad_desc {
  bf16_t* x;
  long long stride;
  int rows, cols, rp, cp;
  int items;
  int blocks_per_item, block_begin;  // filled by the launcher
  int pad_;
};
constexpr int SM_PAD_MAX_GROUP = 64;
int sm_launch_pad_clear(signmuon_ctx* ctx, const sm_pad_desc* descs, int n);
// sumsq[b] = sum of squares of x[b][0..n) (f32 or bf16; two stages, fixed order);
// scratch: batch * ceil(n / SM_MOM_CHUNK) floats
int sm_launch_sumsq(signmuon_ctx* ctx, const void* x, int dtype, long long n_per_batch, int batch, float* scratch,
                    float* sumsq);

// ---------------------------------------------------------------- GEMM (ns_gemm.hip)
// C[b] = rnd(rnd(alpha * scale[b]^scale_pow * (A' * B'^T) + diag * I) + gamma * R[b]),
//        A' = opA[b] + a_diag I,  B' = opB[b] + b_diag I
// opA is M x K, opB is N x K, C and R are [M][ldc]; M, N, K multiples of 64; fp32 accumulation.
// With a symmetric output R must be symmetric too.  The identity shifts need half-precision
// K-contiguous operands.
// Matrices hold 16-bit elements: bf16, or IEEE half where in_f16 (A, B) / out_f16 (C) say
// so (r_f16 for R); the pointer type is bf16_t either way.
struct sm_gemm_prob {
  const bf16_t* A;
  const bf16_t* B;
  bf16_t* C;
  const bf16_t* R;       // or null
  const float* scale;    // [batch] or null
  long long sA, sB, sC;  // batch strides in elements (C and R share sC)
  int M, N, K;
  int lda, ldb, ldc;
  int batch;
  int tiles_m, tiles_n;  // filled by the launcher
  int tile_begin;        // filled by the launcher
  int layout;            // bit 0: A stored [K][M] (lda = its row length), bit 1: B stored [K][N]
  // Optional sign output of a general (non-symmetric) bf16 product: the signs (x >= 0) of the
  // leading sign_rows x sign_cols part of C[b], packed row-major into
  // sign_out + b * sign_stride as in signmuon_sign_pack (sign_cols a multiple of 32).  C may
  // then be null.
  void* sign_out;
  long long sign_stride;
  int sign_rows, sign_cols;
  int sign_fmt;
  // Index (> own index) of a second problem of equal M, N, K and batch whose tiles are dealt item by
  // item right after this problem's (item b of this one, item b of the mate, item b + 1, ...), so
  // that operands the two share are read from HBM once; 0 = none.  The mate owns no tiles itself.
  int mate;
  // logical (unpadded) M, N, K for the work accounting of the timing taps; 0 = as M, N, K
  int mu, nu, ku;
};
constexpr int SM_GEMM_MAX_PROB = 24;
struct sm_gemm_args {
  int n_prob;
  int total_tiles;
  int xcd_begin[9];  // XCD x owns tiles [xcd_begin[x], xcd_begin[x + 1]) of the tile list
  int scale_pow;     // 0, 1 or 2
  float alpha, gamma, diag;
  float a_diag, b_diag;  // 0 = none
  int in_f16, out_f16, r_f16;
  int sym_store;     // bit 0: the operands hold valid data only in their 256 x 256 blocks on and above the diagonal
                     // (symmetric matrices; half precision, M == N == K); bit 1: write the output that way
  int reverse;       // an XCD walks its range of the tile list from the end (set by the launcher: every other launch)
  sm_gemm_prob p[SM_GEMM_MAX_PROB];
};
// One grouped launch over the problem table.  sym: every problem's output is symmetric (M == N;
// layout 0 or 3): only the upper triangle of tiles is computed and stored mirrored.  Otherwise
// layout 0 or 2.  Half-precision operands need sym and layout 0.  klass is the profiling class
// the launch is booked under.
int sm_launch_gemm(signmuon_ctx* ctx, sm_gemm_args& args, bool sym, int klass);

// ---------------------------------------------------------------- power iteration (poweriter.hip)
// sigma[item] = PowerIter(X[item], P, eps, v0[item]) for the `items` matrices of each table entry.
struct sm_pi_desc {
  const bf16_t* x;      // [items][rows][ld], zero beyond cols in every row
  long long stride;     // elements between matrices
  const float* v0;      // [items] start vectors of cols floats, v0_stride floats apart
  long long v0_stride;
  float* u;             // scratch [items][up]
  float* v;             // scratch [items][ld]
  float* part;          // scratch [items][chunks][ld]
  float* sigma;         // [items]
  int rows, cols, ld;   // ld a multiple of 64
  int up;               // rows rounded up to a multiple of 8
  int items;
  int chunks;           // ceil(rows / SM_PI_ROW_CHUNK)
  int block_begin;      // filled by the launcher
  int pad_;
};
constexpr int SM_PI_MAX_GROUP = 40;
constexpr int SM_PI_ROW_CHUNK = 128;
constexpr int SM_PI_FUSED_ROWS = 64;       // rows per workgroup of the fused pass
constexpr int SM_PI_FUSED_MAX_LD = 4096;   // widest matrix (padded columns) the fused pass holds in registers
int sm_launch_power_iter_group(signmuon_ctx* ctx, const sm_pi_desc* descs, int n, int P, float eps);
