// C-ABI entry points and the Newton-Schulz workspace plan.
//
// Working layout.  Weight blocks of equal shape form a class; a class keeps its
// matrices back to back as [block][worker][rows_p][cols_p] bf16 with both
// dimensions zero-padded to multiples of 64 (padding rows/columns stay zero
// through the iteration, so they change nothing).  One grouped GEMM launch then
// covers every class, block and worker of a Newton-Schulz half-step.
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>

#include "common.h"
#include "../../include/signmuon_debug.h"

struct ns_class {
  int rows = 0, cols = 0;  // logical shape
  int rp = 0, cp = 0;      // padded shape
  bool wide = true;        // rows <= cols: Gram over the rows (Y Y^T), else over the columns (Y^T Y)
  int s = 0, l = 0;        // padded short / long side
  int count = 0;           // blocks of this shape
  std::vector<int> members;
  long long mat = 0;       // rp * cp
  // arena offsets in bytes
  size_t off_x[2] = {0, 0}, off_sig = 0, off_inv = 0, off_partial = 0;
  // s x s matrices per item.  Step-by-step form: Bm in off_q[0], G in off_a.  Recurrence: A_0 in
  // off_q[0], later A_k in off_a / off_q[1], T in off_t, P_k in off_p[0/1].
  size_t off_q[2] = {0, 0}, off_a = 0, off_t = 0, off_p[2] = {0, 0};
  int chunks = 0;          // momentum chunks per worker
  // internal sign buffers of the class: [block][worker] rows of sign_stride bytes
  size_t off_signs = 0;
  long long sign_stride = 0;
  bool fuse_signs = false;  // the last apply of the pre-vote iteration can write the signs itself
};

struct ns_plan {
  std::vector<int> rows, cols;
  int M = 0;
  int sign_fmt = -1;
  std::vector<ns_class> classes;
  std::vector<int> class_of, index_in_class;  // per block
  std::vector<size_t> off_signs;              // per block, internal sign buffers (M rows)
  std::vector<long long> sign_stride;         // per block, bytes per worker
  size_t off_pi = 0;                          // power-iteration scratch
  size_t total = 0;
};

void sm_plan_free(signmuon_ctx* ctx, int slot) {
  delete ctx->ws[slot].plan;
  ctx->ws[slot].plan = nullptr;
}


namespace {

template <typename T>
T* at(signmuon_ctx* ctx, size_t off) {
  return reinterpret_cast<T*>(reinterpret_cast<unsigned char*>(ctx->arena) + off);
}

// The plan of workspace `slot` for this set of shapes; makes that workspace's arena the current
// one.  A new set of shapes replans: the arena is (re)allocated if it is too small and cleared.
int get_plan(signmuon_ctx* ctx, int slot, int n, const int* rows, const int* cols, int M, int sign_fmt,
             ns_plan** out) {
  ns_plan* pl = ctx->ws[slot].plan;
  if (pl && pl->M == M && pl->sign_fmt == sign_fmt && (int)pl->rows.size() == n &&
      std::equal(rows, rows + n, pl->rows.begin()) && std::equal(cols, cols + n, pl->cols.begin())) {
    ctx->arena = ctx->ws[slot].arena;
    *out = pl;
    return SM_OK;
  }
  sm_plan_free(ctx, slot);
  pl = new ns_plan();
  pl->rows.assign(rows, rows + n);
  pl->cols.assign(cols, cols + n);
  pl->M = M;
  pl->sign_fmt = sign_fmt;
  pl->class_of.resize(n);
  pl->index_in_class.resize(n);
  for (int i = 0; i < n; ++i) {
    int k = -1;
    for (size_t j = 0; j < pl->classes.size(); ++j)
      if (pl->classes[j].rows == rows[i] && pl->classes[j].cols == cols[i]) k = (int)j;
    if (k < 0) {
      ns_class c;
      c.rows = rows[i];
      c.cols = cols[i];
      c.rp = (int)sm_round_up(rows[i], 64);
      c.cp = (int)sm_round_up(cols[i], 64);
      c.wide = rows[i] <= cols[i];
      c.s = c.wide ? c.rp : c.cp;
      c.l = c.wide ? c.cp : c.rp;
      c.mat = (long long)c.rp * c.cp;
      c.chunks = (int)(((long long)rows[i] * cols[i] + SM_MOM_CHUNK - 1) / SM_MOM_CHUNK);
      pl->classes.push_back(c);
      k = (int)pl->classes.size() - 1;
    }
    pl->class_of[i] = k;
    pl->index_in_class[i] = pl->classes[k].count++;
    pl->classes[k].members.push_back(i);
  }
  size_t off = 0;
  auto take = [&](size_t bytes) {
    const size_t o = off;
    off += (bytes + 255) / 256 * 256;
    return o;
  };
  long long total_pi = 0;
  for (auto& c : pl->classes) {
    const long long batch = (long long)c.count * M;
    c.off_x[0] = take((size_t)batch * c.mat * 2);
    c.off_x[1] = take((size_t)batch * c.mat * 2);
    const size_t ssb = (size_t)batch * c.s * c.s * 2;
    c.off_q[0] = take(ssb);
    c.off_q[1] = take(ssb);
    c.off_a = take(ssb);
    c.off_t = take(ssb);
    c.off_p[0] = take(ssb);
    c.off_p[1] = take(ssb);
    c.off_sig = take((size_t)batch * 4);
    c.off_inv = take((size_t)batch * 4);
    c.off_partial = take((size_t)batch * c.chunks * 4);
    // per matrix: u, v and one partial X^T u per row chunk (the fused pass has the smaller chunks)
    total_pi += (long long)c.count * M * (sm_round_up(c.rows, 8) + c.cp * (1 + (c.rows + SM_PI_FUSED_ROWS - 1) / SM_PI_FUSED_ROWS));
  }
  pl->off_pi = take((size_t)total_pi * 4);
  pl->off_signs.resize(n);
  pl->sign_stride.resize(n);
  for (auto& c : pl->classes) {
    const long long d = (long long)c.rows * c.cols;
    c.sign_stride = (sign_fmt == SM_SIGN_INT8) ? sm_round_up(d, 16) : 8 * ((d + 63) / 64);
    c.off_signs = (sign_fmt < 0) ? 0 : take((size_t)c.sign_stride * M * c.count);
    // whole 32-bit words per 32 columns and no tail bits: the GEMM can emit the packed signs
    c.fuse_signs = sign_fmt >= 0 && c.cols % 32 == 0 && d % 64 == 0;
  }
  for (int i = 0; i < n; ++i) {
    const ns_class& c = pl->classes[pl->class_of[i]];
    pl->sign_stride[i] = c.sign_stride;
    pl->off_signs[i] = c.off_signs + (size_t)pl->index_in_class[i] * M * c.sign_stride;
  }
  pl->total = off;
  int rc = sm_arena_reserve(ctx, slot, pl->total);
  if (rc != SM_OK) {
    delete pl;
    return rc;
  }
  // padding must read as zero
  hipError_t e = hipMemsetAsync(ctx->arena, 0, pl->total, ctx->stream);
  if (e != hipSuccess) {
    delete pl;
    return sm_hip_fail(ctx, e, "hipMemsetAsync(workspace)");
  }
  ctx->ws[slot].plan = pl;
  *out = pl;
  return SM_OK;
}

// ---- grouped GEMM launches over the classes of a plan
struct gemm_params {
  float alpha = 1.f, gamma = 0.f, diag = 0.f, a_diag = 0.f, b_diag = 0.f;
  int scale_pow = 0;
  bool sym = true;
  bool in_f16 = false, out_f16 = false, r_f16 = false;
  int sym_store = 0;  // bit 0: operands valid in their upper blocks only; bit 1: write the output that way
  int klass = SM_K_NS_SMALL;
};

// fill(cl, P) sets up `per_class` consecutive problems for class cl (everything except the tile
// bookkeeping); classes are spread over as many launches as the problem table needs.
template <typename F>
int launch_over_classes(signmuon_ctx* ctx, ns_plan* pl, const gemm_params& gp, int per_class, F fill) {
  const size_t ncls = pl->classes.size();
  const size_t per_launch = SM_GEMM_MAX_PROB / per_class;
  for (size_t c0 = 0; c0 < ncls; c0 += per_launch) {
    const int g = (int)std::min(ncls - c0, per_launch);
    sm_gemm_args ga;
    ga.in_f16 = gp.in_f16;
    ga.out_f16 = gp.out_f16;
    ga.r_f16 = gp.r_f16;
    ga.sym_store = gp.sym_store;
    ga.alpha = gp.alpha;
    ga.gamma = gp.gamma;
    ga.diag = gp.diag;
    ga.a_diag = gp.a_diag;
    ga.b_diag = gp.b_diag;
    ga.scale_pow = gp.scale_pow;
    for (int i = 0; i < g; ++i) {
      sm_gemm_prob* P = &ga.p[i * per_class];
      for (int j = 0; j < per_class; ++j) {
        P[j].R = nullptr;
        P[j].scale = nullptr;
        P[j].layout = 0;
        P[j].sign_out = nullptr;
        P[j].sign_stride = 0;
        P[j].sign_rows = P[j].sign_cols = P[j].sign_fmt = P[j].mate = 0;
        P[j].mu = P[j].nu = P[j].ku = 0;
      }
      fill(pl->classes[c0 + i], P);
      // problems of one class given together share operands: deal their tiles item by item
      if (per_class == 2) P[0].mate = i * per_class + 1;
    }
    ga.n_prob = g * per_class;
    const int rc = sm_launch_gemm(ctx, ga, gp.sym, gp.klass);
    if (rc != SM_OK) return rc;
  }
  return SM_OK;
}

// C[s][s] from the short side of Y: Y Y^T (rows <= cols; Y's rows are K-contiguous) or Y^T Y.
void gram_of_y(ns_class& cl, sm_gemm_prob& P, const bf16_t* y, bf16_t* c, int batch) {
  P.A = P.B = y;
  P.C = c;
  P.sA = P.sB = cl.mat;
  P.sC = (long long)cl.s * cl.s;
  P.M = P.N = cl.s;
  P.K = cl.l;
  P.lda = P.ldb = cl.cp;
  P.ldc = cl.s;
  P.layout = cl.wide ? 0 : 3;
  P.batch = batch;
  P.mu = P.nu = std::min(cl.rows, cl.cols);
  P.ku = std::max(cl.rows, cl.cols);
}

// Y'[rp][cp] = S Y (rows <= cols; second operand stored [K][N]) or Y S, S symmetric s x s.
// signs: also (or, without write_y, only) emit the packed signs of the result into the class's
// sign buffers.
struct ns_sign_req {
  int fmt;
  bool write_y;
};

void apply_to_y(signmuon_ctx* ctx, ns_class& cl, sm_gemm_prob& P, const bf16_t* sm, const bf16_t* y, bf16_t* yout,
                int batch, const ns_sign_req* signs) {
  const long long ss = (long long)cl.s * cl.s;
  if (signs && cl.fuse_signs) {
    P.sign_out = at<void>(ctx, cl.off_signs);
    P.sign_stride = cl.sign_stride;
    P.sign_rows = cl.rows;
    P.sign_cols = cl.cols;
    P.sign_fmt = signs->fmt;
    if (!signs->write_y) yout = nullptr;
  }
  P.C = yout;
  P.sC = cl.mat;
  P.M = cl.rp;
  P.N = cl.cp;
  P.ldc = cl.cp;
  P.K = cl.s;
  P.batch = batch;
  P.mu = cl.rows;
  P.nu = cl.cols;
  P.ku = std::min(cl.rows, cl.cols);
  if (cl.wide) {
    P.A = sm;
    P.B = y;
    P.sA = ss;
    P.sB = cl.mat;
    P.lda = cl.s;
    P.ldb = cl.cp;
    P.layout = 2;
  } else {
    P.A = y;
    P.B = sm;
    P.sA = cl.mat;
    P.sB = ss;
    P.lda = cl.cp;
    P.ldb = cl.s;
    P.layout = 0;
  }
}

// C = A B^T over s x s symmetric matrices (all K-contiguous).
void small_product(ns_class& cl, sm_gemm_prob& P, const bf16_t* a, const bf16_t* b, bf16_t* c, int batch) {
  P.A = a;
  P.B = b;
  P.C = c;
  P.sA = P.sB = P.sC = (long long)cl.s * cl.s;
  P.M = P.N = P.K = cl.s;
  P.lda = P.ldb = P.ldc = cl.s;
  P.layout = 0;
  P.batch = batch;
  P.mu = P.nu = P.ku = std::min(cl.rows, cl.cols);
}

// Step-by-step form of Alg. PolarNS: per step one Gram launch (Bm = a I + b G [+ c G^2], G the
// Gram matrix of Y over its short side) and one apply launch (Y' = Bm Y or Y Bm) over all
// classes; batch = count * mult per class, starting from buffer `cur` (0/1) of each class.
// The first step carries the per-item 1 / sigma when use_scale.  Y is read in place.
int run_ns_stepwise(signmuon_ctx* ctx, ns_plan* pl, int mult, int steps, const float* coeffs, bool use_scale,
                    int* cur_io, const ns_sign_req* signs) {
  int cur = *cur_io;
  const float a = coeffs[0], b = coeffs[1], c = coeffs[2];
  for (int k = 0; k < steps; ++k) {
    const bool sc = use_scale && k == 0;
    gemm_params g;
    g.klass = SM_K_NS_GRAM;
    g.scale_pow = sc ? 2 : 0;
    g.alpha = (c != 0.f) ? 1.f : b;
    g.diag = (c != 0.f) ? 0.f : a;
    int rc = launch_over_classes(ctx, pl, g, 1, [&](ns_class& cl, sm_gemm_prob* P) {
      gram_of_y(cl, P[0], at<bf16_t>(ctx, cl.off_x[cur]), at<bf16_t>(ctx, (c != 0.f) ? cl.off_a : cl.off_q[0]),
                cl.count * mult);
      P[0].scale = sc ? at<float>(ctx, cl.off_inv) : nullptr;
    });
    if (rc != SM_OK) return rc;
    if (c != 0.f) {  // Bm = c G G^T + b G + a I   (G symmetric)
      gemm_params q;
      q.alpha = c;
      q.gamma = b;
      q.diag = a;
      rc = launch_over_classes(ctx, pl, q, 1, [&](ns_class& cl, sm_gemm_prob* P) {
        const bf16_t* gm = at<bf16_t>(ctx, cl.off_a);
        small_product(cl, P[0], gm, gm, at<bf16_t>(ctx, cl.off_q[0]), cl.count * mult);
        P[0].R = gm;
      });
      if (rc != SM_OK) return rc;
    }
    gemm_params ap;
    ap.klass = SM_K_NS_APPLY;
    ap.sym = false;
    ap.scale_pow = sc ? 1 : 0;
    rc = launch_over_classes(ctx, pl, ap, 1, [&](ns_class& cl, sm_gemm_prob* P) {
      apply_to_y(ctx, cl, P[0], at<bf16_t>(ctx, cl.off_q[0]), at<bf16_t>(ctx, cl.off_x[cur]),
                 at<bf16_t>(ctx, cl.off_x[cur ^ 1]), cl.count * mult, (k + 1 == steps) ? signs : nullptr);
      P[0].scale = sc ? at<float>(ctx, cl.off_inv) : nullptr;
    });
    if (rc != SM_OK) return rc;
    cur ^= 1;
  }
  *cur_io = cur;
  return SM_OK;
}

// Short-side recurrence for the cubic iteration (c == 0).  With A_k the Gram matrix of Y_k
// over its short side and Q_k = a I + b A_k, every Y_k is Y_0 times a polynomial in A_0, so
// all of these commute and
//     A_{k+1} = Q_k A_k Q_k,      Y_K = (Q_{K-1} ... Q_1 Q_0) Y_0
// hold exactly: K steps of Alg. PolarNS cost one Gram of Y, a chain of products of s x s
// matrices and one apply to Y, and Y is rounded to bf16 once instead of K times.  The s x s
// matrices are kept in IEEE half precision (all of their entries are bounded by a^K, and the
// half-precision MFMA runs at the bf16 rate): with three more mantissa bits than bf16 their
// rounding stays below that of Y itself, which bf16 storage of the products would not.  The
// last product is written in bf16, the type of the apply.  Q_k is never stored: a product
// Q_k X is b (A_k + (a / b) I) X, the GEMM shifting its operand by the identity on the fly.
// Rounding can leave A_k with small negative eigenvalues, which the recurrence grows by
// a^2 per step (the step-by-step form cannot have them), so a segment covers at most
// SM_NS_SEGMENT steps and longer iterations re-form the Gram matrix from Y between segments.
// Segments of three or more steps advance two steps at a time (see below: 5, 7, 10 products
// for 3, 4, 5 steps); a segment of two, or pairs == false, advances one step at a time with
// three products per step:
//   Gram     : A_0 = inv^2 Y Y^T
//   L1(k)    : T = Q_k A_k   and   P_{k+1} = Q_k P_k   (P_2 = Q_1 Q_0 from A_1 and A_0)
//   L2(k)    : A_{k+1} = Q_k T
//   last     : P_K = Q_{K-1} P_{K-1};      apply: Y' = inv P_K Y
constexpr int SM_NS_SEGMENT = 5;

// Coefficients of the two-steps-at-a-time form: with E = x (x + h),
//   (a + b x)(a + b x (a + b x)^2) = b4 E (E + u) + g x + a2.
struct pair_coeffs {
  float h, u, b4, g, a2;
};
pair_coeffs pair_coefficients(float a, float b) {
  pair_coeffs c;
  c.h = 1.5f * a / b;
  c.u = 0.75f * a * a / (b * b);
  c.b4 = b * b * b * b;
  c.g = a * b - a * a * a * b / 8.f;
  c.a2 = a * a;
  return c;
}

int run_ns_recurrence(signmuon_ctx* ctx, ns_plan* pl, int mult, int steps, const float* coeffs, bool use_scale,
                      int* cur_io, const ns_sign_req* signs, bool pairs) {
  int cur = *cur_io;
  const float a = coeffs[0], b = coeffs[1];
  if (b == 0.f) return SM_EINVAL;  // run_ns routes b == 0 to the step-by-step form
  // The s x s matrices between the Gram and the apply are symmetric: only their 256 x 256 blocks on and
  // above the diagonal are written, and a product reads the other blocks as transposes of those
  // (a third fewer bytes to and from memory).  SM_NS_STORE_FULL writes and reads whole matrices.
  const int ss = (ctx->opt[SM_OPT_NS_STORE] == SM_NS_STORE_FULL) ? 0 : 3;
  int done = 0;
  while (done < steps) {
    const int kk = std::min(SM_NS_SEGMENT, steps - done);
    const bool sc = use_scale && done == 0;
    // A_k alternates between off_a and off_q[1] (A_0 stays in off_q[0] until P_2 is formed);
    // P_k (k >= 2) alternates between off_p[0] and off_p[1]
    int ai = 0, pi = 0;
    auto a_ptr = [&](ns_class& cl, int which) { return at<bf16_t>(ctx, which == 0 ? cl.off_a : cl.off_q[1]); };
    gemm_params g;
    g.klass = SM_K_NS_GRAM;
    g.scale_pow = sc ? 2 : 0;
    g.out_f16 = (kk > 1);
    g.sym_store = (kk > 1) ? (ss & 2) : 0;  // A_0 is only read by the products below
    if (kk == 1) {  // only P_1 = Q_0 is needed, in bf16
      g.alpha = b;
      g.diag = a;
    }
    int rc = launch_over_classes(ctx, pl, g, 1, [&](ns_class& cl, sm_gemm_prob* P) {
      gram_of_y(cl, P[0], at<bf16_t>(ctx, cl.off_x[cur]), at<bf16_t>(ctx, cl.off_q[0]), cl.count * mult);
      P[0].scale = sc ? at<float>(ctx, cl.off_inv) : nullptr;
    });
    if (rc != SM_OK) return rc;
    // products  Q_k X = b (A_k + (a / b) I) X  over half-precision s x s matrices
    gemm_params qx;
    qx.alpha = b;
    qx.a_diag = a / b;
    qx.in_f16 = qx.out_f16 = true;
    qx.sym_store = ss;
    // first product of P: P_2 = Q_1 Q_0 = b^2 (A_1 + (a / b) I) (A_0 + (a / b) I)
    gemm_params qq = qx;
    qq.alpha = b * b;
    qq.b_diag = a / b;
    int p_final = -1;  // -1: P_1 = Q_0 (bf16, in off_q[0]); else index into off_p
    if (pairs && kk >= 3) {
      // Two steps at a time.  With x an eigenvalue of A_k, Q_{k+1} Q_k is the quartic
      //   q(x) = (a + b x)(a + b x (a + b x)^2) = b^4 E (E + u) + g x + a^2,
      //   E = x (x + h),  h = 3a / 2b,  u = 3a^2 / 4b^2,  g = a b - a^3 b / 8,
      // so q(A_k) takes two products (E, then q with A_k as the added term) and
      // A_{k+2} = q^2 A_k two more: four or five products per two steps instead of six, two of
      // them squares (one operand matrix to read).
      //   pair:   E = A (A + h I);  q = b^4 E (E + u I) + g A + a^2 I;
      //           S = q q  and  P' = q P  (the first pair's q is P_2 itself);  A' = S A
      //   single: P' = Q P  (an odd step count ends with one ordinary step)
      // A_k alternates between off_q[0] and off_a, E and S share off_t, q of a later pair sits in off_q[1].
      const pair_coeffs pc = pair_coefficients(a, b);
      gemm_params pe;  // E
      pe.in_f16 = pe.out_f16 = true;
      pe.sym_store = ss;
      pe.b_diag = pc.h;
      gemm_params pq = pe;  // q
      pq.alpha = pc.b4;
      pq.b_diag = pc.u;
      pq.diag = pc.a2;
      pq.gamma = pc.g;
      pq.r_f16 = true;
      gemm_params pm;  // plain product of stored matrices
      pm.in_f16 = pm.out_f16 = true;
      pm.sym_store = ss;
      auto ab = [&](ns_class& cl, int which) { return at<bf16_t>(ctx, which == 0 ? cl.off_q[0] : cl.off_a); };
      int left = kk, aw = 0, pw = -1;  // steps to go; where A_k is; which off_p holds P (-1: none yet)
      while (left >= 2) {
        const bool first = (pw < 0), fin = (left == 2);
        rc = launch_over_classes(ctx, pl, pe, 1, [&](ns_class& cl, sm_gemm_prob* P) {
          small_product(cl, P[0], ab(cl, aw), ab(cl, aw), at<bf16_t>(ctx, cl.off_t), cl.count * mult);
        });
        if (rc != SM_OK) return rc;
        auto qb = [&](ns_class& cl) { return at<bf16_t>(ctx, first ? cl.off_p[0] : cl.off_q[1]); };
        rc = launch_over_classes(ctx, pl, pq, 1, [&](ns_class& cl, sm_gemm_prob* P) {
          const bf16_t* e = at<bf16_t>(ctx, cl.off_t);
          small_product(cl, P[0], e, e, qb(cl), cl.count * mult);
          P[0].R = ab(cl, aw);
        });
        if (rc != SM_OK) return rc;
        if (!fin) {
          rc = launch_over_classes(ctx, pl, pm, first ? 1 : 2, [&](ns_class& cl, sm_gemm_prob* P) {
            small_product(cl, P[0], qb(cl), qb(cl), at<bf16_t>(ctx, cl.off_t), cl.count * mult);
            if (!first)
              small_product(cl, P[1], qb(cl), at<bf16_t>(ctx, cl.off_p[pw]), at<bf16_t>(ctx, cl.off_p[pw ^ 1]),
                            cl.count * mult);
          });
          if (rc != SM_OK) return rc;
          rc = launch_over_classes(ctx, pl, pm, 1, [&](ns_class& cl, sm_gemm_prob* P) {
            small_product(cl, P[0], at<bf16_t>(ctx, cl.off_t), ab(cl, aw), ab(cl, aw ^ 1), cl.count * mult);
          });
          if (rc != SM_OK) return rc;
          aw ^= 1;
          pw = first ? 0 : (pw ^ 1);
        } else {  // kk == 4: P_4 = q_2 P_2, in bf16 for the apply
          gemm_params lp = pm;
          lp.out_f16 = false;
        lp.sym_store = ss & 1;  // the apply reads P_K as a full matrix
          rc = launch_over_classes(ctx, pl, lp, 1, [&](ns_class& cl, sm_gemm_prob* P) {
            small_product(cl, P[0], qb(cl), at<bf16_t>(ctx, cl.off_p[pw]), at<bf16_t>(ctx, cl.off_p[pw ^ 1]),
                          cl.count * mult);
          });
          if (rc != SM_OK) return rc;
          pw ^= 1;
        }
        left -= 2;
      }
      if (left == 1) {  // P_K = Q_{K-1} P_{K-1}, in bf16 for the apply
        gemm_params lp = qx;
        lp.out_f16 = false;
        lp.sym_store = ss & 1;  // the apply reads P_K as a full matrix
        rc = launch_over_classes(ctx, pl, lp, 1, [&](ns_class& cl, sm_gemm_prob* P) {
          small_product(cl, P[0], ab(cl, aw), at<bf16_t>(ctx, cl.off_p[pw]), at<bf16_t>(ctx, cl.off_p[pw ^ 1]),
                        cl.count * mult);
        });
        if (rc != SM_OK) return rc;
        pw ^= 1;
      }
      p_final = pw;
    } else {
      for (int k = 0; k + 1 < kk; ++k) {
        // A_k: k == 0 in off_q[0], afterwards a_ptr(ai)
        auto ak = [&](ns_class& cl) { return k == 0 ? at<bf16_t>(ctx, cl.off_q[0]) : a_ptr(cl, ai); };
        const bool with_p = (k >= 2);
        rc = launch_over_classes(ctx, pl, qx, with_p ? 2 : 1, [&](ns_class& cl, sm_gemm_prob* P) {
          small_product(cl, P[0], ak(cl), ak(cl), at<bf16_t>(ctx, cl.off_t), cl.count * mult);
          if (with_p)
            small_product(cl, P[1], ak(cl), at<bf16_t>(ctx, cl.off_p[pi]), at<bf16_t>(ctx, cl.off_p[pi ^ 1]),
                          cl.count * mult);
        });
        if (rc != SM_OK) return rc;
        if (with_p) pi ^= 1;
        if (k == 1) {  // P_2 from A_1 and A_0
          rc = launch_over_classes(ctx, pl, qq, 1, [&](ns_class& cl, sm_gemm_prob* P) {
            small_product(cl, P[0], ak(cl), at<bf16_t>(ctx, cl.off_q[0]), at<bf16_t>(ctx, cl.off_p[pi]), cl.count * mult);
          });
          if (rc != SM_OK) return rc;
        }
        const int an = (k == 0) ? 0 : (ai ^ 1);
        rc = launch_over_classes(ctx, pl, qx, 1, [&](ns_class& cl, sm_gemm_prob* P) {
          small_product(cl, P[0], ak(cl), at<bf16_t>(ctx, cl.off_t), a_ptr(cl, an), cl.count * mult);
        });
        if (rc != SM_OK) return rc;
        ai = an;
      }
        if (kk == 2) {  // P_2 = Q_1 Q_0, written in bf16 for the apply
        gemm_params lp = qq;
        lp.out_f16 = false;
        lp.sym_store = ss & 1;  // the apply reads P_K as a full matrix
        rc = launch_over_classes(ctx, pl, lp, 1, [&](ns_class& cl, sm_gemm_prob* P) {
          small_product(cl, P[0], a_ptr(cl, ai), at<bf16_t>(ctx, cl.off_q[0]), at<bf16_t>(ctx, cl.off_p[0]), cl.count * mult);
        });
        if (rc != SM_OK) return rc;
        p_final = 0;
      } else if (kk > 2) {  // P_K = Q_{kk-1} P_{kk-1}
        gemm_params lp = qx;
        lp.out_f16 = false;
        lp.sym_store = ss & 1;  // the apply reads P_K as a full matrix
        rc = launch_over_classes(ctx, pl, lp, 1, [&](ns_class& cl, sm_gemm_prob* P) {
          small_product(cl, P[0], a_ptr(cl, ai), at<bf16_t>(ctx, cl.off_p[pi]), at<bf16_t>(ctx, cl.off_p[pi ^ 1]),
                        cl.count * mult);
        });
        if (rc != SM_OK) return rc;
        p_final = pi ^ 1;
      }
    }
    gemm_params ap;
    ap.klass = SM_K_NS_APPLY;
    ap.sym = false;
    ap.scale_pow = sc ? 1 : 0;
    rc = launch_over_classes(ctx, pl, ap, 1, [&](ns_class& cl, sm_gemm_prob* P) {
      apply_to_y(ctx, cl, P[0], at<bf16_t>(ctx, p_final < 0 ? cl.off_q[0] : cl.off_p[p_final]),
                 at<bf16_t>(ctx, cl.off_x[cur]), at<bf16_t>(ctx, cl.off_x[cur ^ 1]), cl.count * mult,
                 (done + kk == steps) ? signs : nullptr);
      P[0].scale = sc ? at<float>(ctx, cl.off_inv) : nullptr;
    });
    if (rc != SM_OK) return rc;
    cur ^= 1;
    done += kk;
  }
  *cur_io = cur;
  return SM_OK;
}

// Runs `steps` Newton-Schulz steps on every class and returns the buffer index of the result.
// The recurrence serves the cubic with |a| <= 1.5 (the paper's a = 3/2: growth of rounding noise
// bounded by a^(2 (SM_NS_SEGMENT - 1)) < 26); other coefficients take the step-by-step form.
// Option SM_OPT_NS_PATH forces the latter (SM_NS_PATH_STEPWISE) or the recurrence one step at a
// time (SM_NS_PATH_SINGLE: three products per step), for comparisons.
// signs (optional): the last apply also emits the packed signs of the classes marked fuse_signs.
int run_ns(signmuon_ctx* ctx, ns_plan* pl, int mult, int steps, const float* coeffs, bool use_scale, int* cur_io,
           const ns_sign_req* signs = nullptr) {
  const bool force_stepwise = ctx->opt[SM_OPT_NS_PATH] == SM_NS_PATH_STEPWISE;
  const bool force_single = ctx->opt[SM_OPT_NS_PATH] == SM_NS_PATH_SINGLE;
  if (!force_stepwise && coeffs[2] == 0.f && coeffs[1] != 0.f && fabsf(coeffs[0]) <= 1.5f && steps >= 2)
    return run_ns_recurrence(ctx, pl, mult, steps, coeffs, use_scale, cur_io, signs, !force_single);
  return run_ns_stepwise(ctx, pl, mult, steps, coeffs, use_scale, cur_io, signs);
}

// Spectral scale of Alg. PolarNS for every block of the plan: `items` matrices per block starting at
// matrix (index in class) * items_stride of buffer `buf` of its class; v0[i] is block i's start vectors.
int spectral_sigma(signmuon_ctx* ctx, ns_plan* pl, int buf, int items, int items_stride, const float* const* v0,
                   int P, float eps) {
  const int n = (int)pl->rows.size();
  std::vector<sm_pi_desc> d(n);
  float* scratch = at<float>(ctx, pl->off_pi);
  for (int i = 0; i < n; ++i) {
    ns_class& cl = pl->classes[pl->class_of[i]];
    const long long first = (long long)pl->index_in_class[i] * items_stride;
    const int up = (int)sm_round_up(cl.rows, 8);
    sm_pi_desc& D = d[i];
    D.x = at<bf16_t>(ctx, cl.off_x[buf]) + first * cl.mat;
    D.stride = cl.mat;
    D.v0 = v0[i];
    D.v0_stride = cl.cols;
    D.u = scratch;
    const int chunks = (cl.rows + SM_PI_ROW_CHUNK - 1) / SM_PI_ROW_CHUNK;
    D.v = scratch + (long long)items * up;
    D.part = D.v + (long long)items * cl.cp;
    D.chunks = chunks;
    D.pad_ = 0;
    scratch += (long long)items * (up + (long long)cl.cp * (1 + (cl.rows + SM_PI_FUSED_ROWS - 1) / SM_PI_FUSED_ROWS));
    D.sigma = at<float>(ctx, cl.off_sig) + first;
    D.rows = cl.rows;
    D.cols = cl.cols;
    D.ld = cl.cp;
    D.up = up;
    D.items = items;
    D.block_begin = 0;
  }
  return sm_launch_power_iter_group(ctx, d.data(), n, P, eps);
}

// inv = 1 / max(sigma, eps) for `items` matrices per block of every class, in one launch.
// mode 0: sigma from the momentum kernel's partial sums of squares; 1: sigma as left by PowerIter;
// 2: the Frobenius norm of a +-1 matrix, sqrt(rows * cols), known in closed form.
int class_inv_sigma(signmuon_ctx* ctx, ns_plan* pl, int items, int mode, float eps) {
  std::vector<sm_sigma_desc> d;
  for (auto& cl : pl->classes) {
    sm_sigma_desc D;
    D.partial = at<float>(ctx, cl.off_partial);
    D.sig = at<float>(ctx, cl.off_sig);
    D.inv = at<float>(ctx, cl.off_inv);
    D.chunks = cl.chunks;
    D.count = cl.count * items;
    D.mode = mode;
    D.value = 1.0f / fmaxf(sqrtf((float)cl.rows * (float)cl.cols), eps);
    D.block_begin = 0;
    D.pad_ = 0;
    d.push_back(D);
  }
  return sm_launch_sigma_group(ctx, d.data(), (int)d.size(), eps);
}

// Zeroes the padding of the first `items` matrices per block-count unit of buffer `buf` of every padded class:
// items_per_class(cl) matrices starting at the buffer's base.
template <typename F>
int clear_padding(signmuon_ctx* ctx, ns_plan* pl, int buf, F items_per_class) {
  std::vector<sm_pad_desc> d;
  for (auto& cl : pl->classes) {
    if (cl.rp == cl.rows && cl.cp == cl.cols) continue;
    sm_pad_desc D;
    D.x = at<bf16_t>(ctx, cl.off_x[buf]);
    D.stride = cl.mat;
    D.rows = cl.rows;
    D.cols = cl.cols;
    D.rp = cl.rp;
    D.cp = cl.cp;
    D.items = items_per_class(cl);
    D.blocks_per_item = D.block_begin = D.pad_ = 0;
    d.push_back(D);
  }
  if (d.empty()) return SM_OK;
  return sm_launch_pad_clear(ctx, d.data(), (int)d.size());
}

bool bad_coeffs(const float* c) { return !c || !isfinite(c[0]) || !isfinite(c[1]) || !isfinite(c[2]); }

}  // namespace

extern "C" {

// a1 for one block; partial sums of squares (when sumsq is asked for) go to `partial_buf`, which holds
// partial_cap bytes.
static int momentum_one(signmuon_ctx* ctx, float* mom, const float* grad, const float* w, int M, int rows, int cols,
                        float beta, float weight_decay, void* x_bf16, float* sumsq, float* partial_buf) {
  const long long d = (long long)rows * cols;
  const int chunks = (int)((d + SM_MOM_CHUNK - 1) / SM_MOM_CHUNK);
  sm_mom_desc D;
  D.mom = mom;
  D.grad = grad;
  D.w = (weight_decay != 0.f) ? w : nullptr;
  D.x = reinterpret_cast<bf16_t*>(x_bf16);
  D.partial = sumsq ? partial_buf : nullptr;
  D.d = d;
  D.x_stride = d;
  D.cols = cols;
  D.ld = cols;
  D.chunks = chunks;
  D.block_begin = 0;
  int rc = sm_launch_momentum(ctx, &D, 1, M, beta, weight_decay);
  if (rc != SM_OK) return rc;
  if (sumsq) return sm_launch_reduce_partials(ctx, partial_buf, chunks, M, sumsq);
  return SM_OK;
}

static int momentum_check(signmuon_ctx* ctx, float* mom, const float* grad, const float* w, int M, int rows, int cols,
                          float beta, float weight_decay, void* x_bf16, float* sumsq) {
  if (!mom || !grad || M < 1 || rows < 1 || cols < 1) return sm_fail(ctx, SM_EINVAL, "momentum: bad pointer or size");
  if (weight_decay != 0.f && !w) return sm_fail(ctx, SM_EINVAL, "momentum: weight_decay != 0 needs w");
  if (!(beta >= 0.f && beta < 1.f)) return sm_fail(ctx, SM_EINVAL, "momentum: beta must be in [0, 1)");
  if (!sm_aligned(mom, 4) || !sm_aligned(grad, 4) || (w && !sm_aligned(w, 4)) || (x_bf16 && !sm_aligned(x_bf16, 2)) ||
      (sumsq && !sm_aligned(sumsq, 4)))
    return sm_fail(ctx, SM_EINVAL, "momentum: misaligned pointer");
  const long long chunks = ((long long)rows * cols + SM_MOM_CHUNK - 1) / SM_MOM_CHUNK;
  if (chunks * M > 0x7FFFFFFFLL) return sm_fail(ctx, SM_EUNSUPPORTED, "momentum: too many entries for one launch");
  return SM_OK;
}

int signmuon_momentum(signmuon_ctx* ctx, float* mom, const float* grad, const float* w, int M, int rows, int cols,
                      float beta, float weight_decay, void* x_bf16, float* sumsq) {
  if (!ctx) return SM_EINVAL;
  int rc = momentum_check(ctx, mom, grad, w, M, rows, cols, beta, weight_decay, x_bf16, sumsq);
  if (rc != SM_OK) return rc;
  if (sumsq) {
    // per-chunk partial sums: the context's small scratch (not the step's workspace)
    const long long chunks = ((long long)rows * cols + SM_MOM_CHUNK - 1) / SM_MOM_CHUNK;
    rc = sm_aux_reserve(ctx, (size_t)M * chunks * 4);
    if (rc != SM_OK) return rc;
  }
  return momentum_one(ctx, mom, grad, w, M, rows, cols, beta, weight_decay, x_bf16, sumsq,
                      reinterpret_cast<float*>(ctx->aux));
}

int signmuon_momentum_noalloc(signmuon_ctx* ctx, float* mom, const float* grad, const float* w, int M, int rows,
                              int cols, float beta, float weight_decay, void* x_bf16, float* sumsq) {
  if (!ctx) return SM_EINVAL;
  int rc = momentum_check(ctx, mom, grad, w, M, rows, cols, beta, weight_decay, x_bf16, sumsq);
  if (rc != SM_OK) return rc;
  const long long chunks = ((long long)rows * cols + SM_MOM_CHUNK - 1) / SM_MOM_CHUNK;
  if ((unsigned long long)M * chunks * 4ull > SM_STATIC_SCRATCH_BYTES)
    return sm_fail(ctx, SM_EUNSUPPORTED,
                   "momentum_noalloc: M * ceil(rows*cols/1024) partial sums exceed the static scratch (" +
                       std::to_string(SM_STATIC_SCRATCH_BYTES) + " bytes)");
  if (!ctx->static_scratch) return sm_fail(ctx, SM_EHIP, "momentum_noalloc: no static scratch on this device");
  // timing taps create HIP events on demand: not on this path
  const unsigned taps = ctx->profiling;
  ctx->profiling = 0;
  rc = momentum_one(ctx, mom, grad, w, M, rows, cols, beta, weight_decay, x_bf16, sumsq,
                    reinterpret_cast<float*>(ctx->static_scratch));
  ctx->profiling = taps;
  return rc;
}

int signmuon_polar_ns(signmuon_ctx* ctx, void* x, int dtype, int batch, int rows, int cols, const float* coeffs,
                      int steps, int scale, int power_iters, float eps, const float* v0) {
  if (!ctx) return SM_EINVAL;
  if (!x || batch < 1 || rows < 1 || cols < 1 || steps < 0) return sm_fail(ctx, SM_EINVAL, "polar_ns: bad pointer or size");
  if (dtype != SM_F32 && dtype != SM_BF16) return sm_fail(ctx, SM_EINVAL, "polar_ns: bad dtype");
  if (bad_coeffs(coeffs)) return sm_fail(ctx, SM_EINVAL, "polar_ns: bad coeffs");
  if (scale != SM_SCALE_FRO && scale != SM_SCALE_SPECTRAL && scale != SM_SCALE_NONE)
    return sm_fail(ctx, SM_EINVAL, "polar_ns: bad scale");
  if (scale == SM_SCALE_SPECTRAL && (!v0 || power_iters < 0))
    return sm_fail(ctx, SM_EINVAL, "polar_ns: spectral scale needs v0 and power_iters >= 0");
  if (!(eps >= 0.f)) return sm_fail(ctx, SM_EINVAL, "polar_ns: eps must be >= 0");
  if (!sm_aligned(x, dtype == SM_F32 ? 4 : 2)) return sm_fail(ctx, SM_EINVAL, "polar_ns: misaligned x");
  if (batch > 65535) return sm_fail(ctx, SM_EUNSUPPORTED, "polar_ns: batch > 65535");
  ns_plan* pl = nullptr;
  int rc = get_plan(ctx, SM_WS_NS, 1, &rows, &cols, batch, -1, &pl);
  if (rc != SM_OK) return rc;
  ns_class& cl = pl->classes[0];
  rc = sm_launch_copy_in(ctx, x, dtype, batch, rows, cols, at<bf16_t>(ctx, cl.off_x[0]), cl.cp, cl.mat);
  if (rc != SM_OK) return rc;
  rc = clear_padding(ctx, pl, 0, [&](ns_class&) { return batch; });
  if (rc != SM_OK) return rc;
  bool use_scale = false;
  if (scale == SM_SCALE_FRO) {
    rc = sm_launch_sumsq(ctx, x, dtype, (long long)rows * cols, batch, at<float>(ctx, cl.off_partial),
                         at<float>(ctx, cl.off_sig));
    if (rc != SM_OK) return rc;
    rc = sm_launch_inv_sigma(ctx, at<float>(ctx, cl.off_sig), batch, eps, true, at<float>(ctx, cl.off_inv));
    if (rc != SM_OK) return rc;
    use_scale = true;
  } else if (scale == SM_SCALE_SPECTRAL) {
    rc = spectral_sigma(ctx, pl, 0, batch, batch, &v0, power_iters, eps);
    if (rc != SM_OK) return rc;
    rc = sm_launch_inv_sigma(ctx, at<float>(ctx, cl.off_sig), batch, eps, false, at<float>(ctx, cl.off_inv));
    if (rc != SM_OK) return rc;
    use_scale = true;
  }
  int cur = 0;
  rc = run_ns(ctx, pl, batch, steps, coeffs, use_scale, &cur);
  if (rc != SM_OK) return rc;
  return sm_launch_copy_out(ctx, at<bf16_t>(ctx, cl.off_x[cur]), cl.cp, cl.mat, batch, rows, cols, x, dtype,
                            (steps == 0 && use_scale) ? at<float>(ctx, cl.off_inv) : nullptr);
}

int signmuon_sign_pack(signmuon_ctx* ctx, const void* u, int dtype, int batch, int64_t n, int fmt, void* out,
                       int64_t out_stride_bytes) {
  if (!ctx) return SM_EINVAL;
  if (!out || batch < 0 || n < 0 || (!u && n > 0 && batch > 0)) return sm_fail(ctx, SM_EINVAL, "sign_pack: bad pointer or size");
  if (dtype != SM_F32 && dtype != SM_BF16) return sm_fail(ctx, SM_EINVAL, "sign_pack: bad dtype");
  if (fmt != SM_SIGN_1BIT && fmt != SM_SIGN_INT8) return sm_fail(ctx, SM_EINVAL, "sign_pack: bad fmt");
  if (n > 0x7FFFFFFFLL * 8) return sm_fail(ctx, SM_EINVAL, "sign_pack: n too large");
  if (fmt == SM_SIGN_1BIT) {
    if (out_stride_bytes % 8 || out_stride_bytes < 8 * ((n + 63) / 64) || !sm_aligned(out, 8))
      return sm_fail(ctx, SM_EINVAL, "sign_pack: 1-bit rows must be 8-byte aligned and hold ceil(n/64) words");
  } else if (out_stride_bytes < n) {
    return sm_fail(ctx, SM_EINVAL, "sign_pack: int8 stride shorter than n");
  }
  if (!sm_aligned(u, dtype == SM_F32 ? 4 : 2)) return sm_fail(ctx, SM_EINVAL, "sign_pack: misaligned u");
  if (batch == 0 || n == 0) return SM_OK;
  if (batch > 65535) return sm_fail(ctx, SM_EUNSUPPORTED, "sign_pack: batch > 65535");
  // treat each row as a 1 x n matrix; int counts are fine because cols is only used when ld != cols
  if (n > 0x7FFFFFFF) {
    // split long rows into 2-D with cols a multiple of 64 when possible
    return sm_fail(ctx, SM_EUNSUPPORTED, "sign_pack: n >= 2^31 per row");
  }
  return sm_launch_sign_pack(ctx, u, dtype, batch, 1, (int)n, (int)n, n, fmt, out, out_stride_bytes);
}

int signmuon_majority_vote(signmuon_ctx* ctx, const void* signs, int fmt, int M, int64_t n, int64_t stride_bytes,
                           void* voted, int vfmt, int32_t* counts, float* w, float lr_scaled) {
  if (!ctx) return SM_EINVAL;
  if (M < 1 || n < 0 || (!signs && n > 0)) return sm_fail(ctx, SM_EINVAL, "majority_vote: bad pointer or size");
  if (fmt != SM_SIGN_1BIT && fmt != SM_SIGN_INT8) return sm_fail(ctx, SM_EINVAL, "majority_vote: bad fmt");
  if (voted && (vfmt < SM_VOTE_BITS || vfmt > SM_VOTE_F32)) return sm_fail(ctx, SM_EINVAL, "majority_vote: bad vfmt");
  if (n >= (1LL << 40)) return sm_fail(ctx, SM_EINVAL, "majority_vote: n too large");
  if (fmt == SM_SIGN_1BIT) {
    if (stride_bytes % 8 || stride_bytes < 8 * ((n + 63) / 64) || !sm_aligned(signs, 8))
      return sm_fail(ctx, SM_EINVAL, "majority_vote: 1-bit rows must be 8-byte aligned and hold ceil(n/64) words");
  } else if (stride_bytes < n) {
    return sm_fail(ctx, SM_EINVAL, "majority_vote: int8 stride shorter than n");
  }
  if (voted && vfmt == SM_VOTE_BITS && !sm_aligned(voted, 8)) return sm_fail(ctx, SM_EINVAL, "majority_vote: misaligned voted bits");
  if (voted && vfmt == SM_VOTE_BF16 && !sm_aligned(voted, 8)) return sm_fail(ctx, SM_EINVAL, "majority_vote: voted bf16 needs 8-byte alignment");
  if (voted && vfmt == SM_VOTE_F32 && !sm_aligned(voted, 16)) return sm_fail(ctx, SM_EINVAL, "majority_vote: voted f32 needs 16-byte alignment");
  if (voted && vfmt == SM_VOTE_INT8 && !sm_aligned(voted, 4)) return sm_fail(ctx, SM_EINVAL, "majority_vote: voted int8 needs 4-byte alignment");
  if ((counts && !sm_aligned(counts, 16)) || (w && !sm_aligned(w, 16)))
    return sm_fail(ctx, SM_EINVAL, "majority_vote: counts and w need 16-byte alignment");
  if (n == 0) return SM_OK;
  sm_vote_args a;
  a.signs = signs;
  a.fmt = fmt;
  a.M = M;
  a.n = n;
  a.stride_bytes = stride_bytes;
  a.voted = voted;
  a.vfmt = vfmt;
  a.cols = 1;
  a.ld = 1;
  a.counts = counts;
  a.w = w;
  a.lr_scaled = lr_scaled;
  return sm_launch_vote(ctx, a);
}

int signmuon_step(signmuon_ctx* ctx, const signmuon_step_args* s) {
  if (!ctx) return SM_EINVAL;
  if (!s || s->n_mats < 1 || s->M < 1 || !s->rows || !s->cols || !s->w || !s->mom || !s->grad)
    return sm_fail(ctx, SM_EINVAL, "step: bad pointer or size");
  if (!(s->beta >= 0.f && s->beta < 1.f)) return sm_fail(ctx, SM_EINVAL, "step: beta must be in [0, 1)");
  if (s->ns_steps < 0 || s->local_polar_steps < 0) return sm_fail(ctx, SM_EINVAL, "step: negative step count");
  if (bad_coeffs(s->coeffs)) return sm_fail(ctx, SM_EINVAL, "step: bad coeffs");
  if (s->scale != SM_SCALE_FRO && s->scale != SM_SCALE_SPECTRAL && s->scale != SM_SCALE_NONE)
    return sm_fail(ctx, SM_EINVAL, "step: bad scale");
  if (s->sign_fmt != SM_SIGN_1BIT && s->sign_fmt != SM_SIGN_INT8) return sm_fail(ctx, SM_EINVAL, "step: bad sign_fmt");
  if (!(s->eps >= 0.f)) return sm_fail(ctx, SM_EINVAL, "step: eps must be >= 0");
  const bool spectral = (s->scale == SM_SCALE_SPECTRAL);
  if (spectral && (!s->v0 || s->power_iters < 0)) return sm_fail(ctx, SM_EINVAL, "step: spectral scale needs v0");
  if (s->update_rsqrt_mn < 0 || s->update_rsqrt_mn > 2) return sm_fail(ctx, SM_EINVAL, "step: bad update scale mode");
  const bool op_norm = (s->update_rsqrt_mn == 2);
  if (op_norm && (!s->v0 || s->power_iters < 0 || s->local_polar_steps != 0))
    return sm_fail(ctx, SM_EINVAL, "step: the normalized-sign update needs v0 and no local polar step");
  const int n = s->n_mats, M = s->M;
  for (int i = 0; i < n; ++i) {
    if (s->rows[i] < 1 || s->cols[i] < 1) return sm_fail(ctx, SM_EINVAL, "step: bad block shape");
    if (!s->w[i] || !s->mom[i] || !s->grad[i]) return sm_fail(ctx, SM_EINVAL, "step: NULL block pointer");
    if (!sm_aligned(s->w[i], 16) || !sm_aligned(s->mom[i], 16) || !sm_aligned(s->grad[i], 16))
      return sm_fail(ctx, SM_EINVAL, "step: block pointers need 16-byte alignment");
    if ((spectral || op_norm) && !s->v0[i]) return sm_fail(ctx, SM_EINVAL, "step: NULL v0 entry");
    if (s->signs_out && s->signs_out[i] && !sm_aligned(s->signs_out[i], 16))
      return sm_fail(ctx, SM_EINVAL, "step: signs_out needs 16-byte alignment");
    if (s->counts_out && s->counts_out[i] && !sm_aligned(s->counts_out[i], 16))
      return sm_fail(ctx, SM_EINVAL, "step: counts_out needs 16-byte alignment");
  }
  ns_plan* pl = nullptr;
  if (M > 65535) return sm_fail(ctx, SM_EUNSUPPORTED, "step: M > 65535");
  int rc = get_plan(ctx, SM_WS_STEP, n, s->rows, s->cols, M, s->sign_fmt, &pl);
  if (rc != SM_OK) return rc;

  // a1: momentum for every block and worker, with the bf16 working copy and the sums of squares
  std::vector<sm_mom_desc> descs(n);
  for (int i = 0; i < n; ++i) {
    ns_class& cl = pl->classes[pl->class_of[i]];
    const int idx = pl->index_in_class[i];
    sm_mom_desc& D = descs[i];
    D.mom = s->mom[i];
    D.grad = s->grad[i];
    D.w = (s->weight_decay != 0.f) ? s->w[i] : nullptr;
    D.x = at<bf16_t>(ctx, cl.off_x[0]) + (long long)idx * M * cl.mat;
    D.partial = at<float>(ctx, cl.off_partial) + (long long)idx * M * cl.chunks;
    D.d = (long long)cl.rows * cl.cols;
    D.x_stride = cl.mat;
    D.cols = cl.cols;
    D.ld = cl.cp;
    D.chunks = cl.chunks;
    D.block_begin = 0;
  }
  rc = sm_launch_momentum(ctx, descs.data(), n, M, s->beta, s->weight_decay);
  if (rc != SM_OK) return rc;
  // the first GEMM launch (the Gram of Y) walks its tile ranges backwards: it starts with the blocks whose
  // bf16 copies the momentum kernel wrote last
  ctx->gemm_flip = 1;
  // the momentum kernel writes the logical entries of X only: restore the zero padding, which an
  // earlier call with a non-finite matrix may have turned into NaN
  rc = clear_padding(ctx, pl, 0, [&](ns_class& cl) { return cl.count * M; });
  if (rc != SM_OK) return rc;

  // a2: sigma per (block, worker)
  bool use_scale = false;
  if (s->ns_steps > 0 || (s->u_out != nullptr)) {
    if (s->scale == SM_SCALE_FRO) {
      rc = class_inv_sigma(ctx, pl, M, 0, s->eps);
      if (rc != SM_OK) return rc;
      use_scale = true;
    } else if (spectral) {
      rc = spectral_sigma(ctx, pl, 0, M, M, s->v0, s->power_iters, s->eps);
      if (rc != SM_OK) return rc;
      rc = class_inv_sigma(ctx, pl, M, 1, s->eps);
      if (rc != SM_OK) return rc;
      use_scale = true;
    }
  }

  // a3 + a4: K Newton-Schulz steps on all (block, worker) matrices
  // When the iteration has at least one step, its last apply writes the packed signs (a5) of
  // every class whose rows pack into whole words; U itself is then only written if a tap asks.
  ns_sign_req sreq;
  sreq.fmt = s->sign_fmt;
  sreq.write_y = false;
  if (s->u_out)
    for (int i = 0; i < n; ++i) sreq.write_y = sreq.write_y || (s->u_out[i] != nullptr);
  const bool fused = s->ns_steps > 0;
  int cur = 0;
  rc = run_ns(ctx, pl, M, s->ns_steps, s->coeffs, use_scale, &cur, fused ? &sreq : nullptr);
  if (rc != SM_OK) return rc;

  const int Kp = s->local_polar_steps;
  // a5 + a6 (+ a8 when there is no local polar step): one sign-pack launch and one vote launch
  // over all blocks
  std::vector<sm_sp_desc> sp;
  sp.reserve(n);
  std::vector<sm_vote_desc> vd(n);
  for (int i = 0; i < n; ++i) {
    ns_class& cl = pl->classes[pl->class_of[i]];
    const int idx = pl->index_in_class[i];
    const long long d = (long long)cl.rows * cl.cols;
    const bf16_t* u = at<bf16_t>(ctx, cl.off_x[cur]) + (long long)idx * M * cl.mat;
    if (s->u_out && s->u_out[i]) {
      rc = sm_launch_copy_out(ctx, u, cl.cp, cl.mat, M, cl.rows, cl.cols, s->u_out[i], SM_BF16,
                              (s->ns_steps == 0 && use_scale) ? at<float>(ctx, cl.off_inv) + (long long)idx * M : nullptr);
      if (rc != SM_OK) return rc;
    }
    const bool tap = s->signs_out && s->signs_out[i];
    const bool in_gemm = fused && cl.fuse_signs;  // already in the internal buffer
    void* signs = (tap && !in_gemm) ? s->signs_out[i] : at<void>(ctx, pl->off_signs[i]);
    const long long stride =
        (tap && !in_gemm) ? ((s->sign_fmt == SM_SIGN_INT8) ? d : 8 * ((d + 63) / 64)) : pl->sign_stride[i];
    if (in_gemm) {
      // d is a multiple of 64 here, so the tap's rows have the internal stride
      if (tap) SM_HIP(ctx, hipMemcpyAsync(s->signs_out[i], signs, (size_t)stride * M, hipMemcpyDeviceToDevice, ctx->stream));
    } else {
      sm_sp_desc S;
      S.u = u;
      S.out = signs;
      S.n = d;
      S.batch_stride = cl.mat;
      S.out_stride = stride;
      S.bytes_per_row = 0;
      S.cols = cl.cols;
      S.ld = cl.cp;
      S.blocks_per_row = S.block_begin = 0;
      sp.push_back(S);
    }
    float step = s->lr;
    if (s->update_rsqrt_mn == 1) step = s->lr / sqrtf((float)cl.rows * (float)cl.cols);
    sm_vote_desc& V = vd[i];
    V.signs = signs;
    V.n = d;
    V.stride_bytes = stride;
    V.counts = (s->counts_out) ? s->counts_out[i] : nullptr;
    V.lr = step;
    V.M = M;
    V.block_begin = 0;
    if (Kp == 0 && !op_norm) {
      V.voted = nullptr;
      V.vfmt = SM_VOTE_BF16;
      V.cols = V.ld = 1;
      V.w = s->w[i];
    } else {
      // the voted +-1 matrix becomes item `idx` of the class's post-vote batch, in the
      // buffer that does not hold the workers' U
      V.voted = at<bf16_t>(ctx, cl.off_x[cur ^ 1]) + (long long)idx * cl.mat;
      V.vfmt = SM_VOTE_BF16;
      V.cols = cl.cols;
      V.ld = cl.cp;
      V.w = nullptr;
    }
  }
  if (!sp.empty()) {
    rc = sm_launch_sign_pack_group(ctx, sp.data(), (int)sp.size(), SM_BF16, s->sign_fmt, M);
    if (rc != SM_OK) return rc;
  }
  rc = sm_launch_vote_group(ctx, vd.data(), n, s->sign_fmt);
  if (rc != SM_OK) return rc;
  if (Kp == 0 && !op_norm && s->d_out) {  // W was already stepped; the tap only re-derives the vote
    for (int i = 0; i < n; ++i) {
      if (!s->d_out[i]) continue;
      sm_vote_desc t = vd[i];
      t.voted = s->d_out[i];
      t.vfmt = SM_VOTE_BF16;
      t.cols = t.ld = 1;
      t.counts = nullptr;
      t.w = nullptr;
      rc = sm_launch_vote_group(ctx, &t, 1, s->sign_fmt);
      if (rc != SM_OK) return rc;
    }
  }
  if (Kp == 0 && !op_norm) return SM_OK;
  // the voted matrices took over slots that held some workers' matrices before the vote: zero their padding
  rc = clear_padding(ctx, pl, cur ^ 1, [&](ns_class& cl) { return cl.count; });
  if (rc != SM_OK) return rc;

  // a7: local polar step on the voted sign matrices (one per block), or their operator norm for
  // the normalized-sign update (worker 0's start vector serves the voted matrix of each block)
  bool use_scale2 = false;
  if (op_norm) {
    rc = spectral_sigma(ctx, pl, cur ^ 1, 1, 1, s->v0, s->power_iters, s->eps);
    if (rc != SM_OK) return rc;
    rc = class_inv_sigma(ctx, pl, 1, 1, s->eps);
    if (rc != SM_OK) return rc;
  } else if (s->scale == SM_SCALE_FRO) {
    // every entry is +-1, so the Frobenius norm is exactly sqrt(rows*cols)
    rc = class_inv_sigma(ctx, pl, 1, 2, s->eps);
    if (rc != SM_OK) return rc;
    use_scale2 = true;
  } else if (spectral) {
    rc = spectral_sigma(ctx, pl, cur ^ 1, 1, 1, s->v0, s->power_iters, s->eps);
    if (rc != SM_OK) return rc;
    rc = class_inv_sigma(ctx, pl, 1, 1, s->eps);
    if (rc != SM_OK) return rc;
    use_scale2 = true;
  }
  cur ^= 1;
  rc = run_ns(ctx, pl, 1, Kp, s->coeffs, use_scale2, &cur);
  if (rc != SM_OK) return rc;

  // a8: W <- W - step * D, one launch over all blocks
  std::vector<sm_upd_desc> ud(n);
  for (int i = 0; i < n; ++i) {
    ns_class& cl = pl->classes[pl->class_of[i]];
    const int idx = pl->index_in_class[i];
    const bf16_t* dmat = at<bf16_t>(ctx, cl.off_x[cur]) + (long long)idx * cl.mat;
    float step = s->lr;
    if (s->update_rsqrt_mn == 1) step = s->lr / sqrtf((float)cl.rows * (float)cl.cols);
    ud[i].w = s->w[i];
    ud[i].d = dmat;
    ud[i].kappa = op_norm ? at<float>(ctx, cl.off_inv) + idx : nullptr;
    ud[i].rows = cl.rows;
    ud[i].cols = cl.cols;
    ud[i].ld = cl.cp;
    ud[i].step = step;
    ud[i].block_begin = 0;
    ud[i].pad_ = 0;
    if (s->d_out && s->d_out[i]) {
      rc = sm_launch_copy_out(ctx, dmat, cl.cp, cl.mat, 1, cl.rows, cl.cols, s->d_out[i], SM_BF16, nullptr);
      if (rc != SM_OK) return rc;
    }
  }
  rc = sm_launch_update_group(ctx, ud.data(), n);
  if (rc != SM_OK) return rc;
  return SM_OK;
}

}  // extern "C"

// Host-side check hook: the five coefficients {h, u, b^4, g, a^2} of the two-steps-at-a-time
// recurrence for the cubic with coefficients a, b.
extern "C" void signmuon_debug_pair_coefficients(float a, float b, float* out5) {
  const pair_coeffs c = pair_coefficients(a, b);
  out5[0] = c.h;
  out5[1] = c.u;
  out5[2] = c.b4;
  out5[3] = c.g;
  out5[4] = c.a2;
}
