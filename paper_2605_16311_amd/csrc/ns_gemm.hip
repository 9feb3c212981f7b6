// Newton-Schulz GEMMs of Alg. PolarNS on the gfx950 matrix cores: pipelined kernel, K slices of 64.
//
//   C = rnd(rnd(alpha * scale^pow * (A' * B'^T) + diag * I) + gamma * R),
//       A' = opA + a_diag I,  B' = opB + b_diag I         (16-bit operands, fp32 accumulate)
//
// opA is an M x K operand and opB an N x K operand; each may be stored K-contiguous
// ([rows][K], "KC") or MN-contiguous ([K][rows], "MN").  The products of the iteration are
//   Gram of Y,  rows <= cols : A = B = Y           (KC, KC)   symmetric output, bf16 in
//   Gram of Y,  rows >  cols : A = B = Y           (MN, MN)   symmetric output, bf16 in
//   s x s products           : A = A_k (+ shift), B = A_k | T | P   (KC, KC), symmetric, half precision
//   apply,      rows <= cols : A = S, B = Y        (KC, MN)   Y' = S Y      (S = Bm or P_K), bf16
//   apply,      rows >  cols : A = Y, B = S        (KC, KC)   Y' = Y S      (S symmetric), bf16
// so Y is only ever read in its own row-major layout and no transposed copy exists.  The
// layout is a per-problem flag: one launch covers every matrix of a phase.  The apply can emit
// the packed signs of its result (Alg. 3's encoding) besides or instead of the result itself.
//
// Structure.  A workgroup of 8 waves (2 per SIMD) owns a TS x TS tile of C (TS = 256, or 128
// for launches with little work); each wave a (TS/2) x (TS/4) sub-tile held as accumulators of
// v_mfma_f32_32x32x16_bf16 (or _f16).  K advances in slices of 64 (four MFMA k-steps), so that every
// global->LDS request covers a whole 128-byte line of a K-contiguous operand: the per-CU
// L2 -> LDS path is limited by the number of outstanding requests, not by bytes.
// Two LDS stages.  Timeline of slice j (stage j & 1):
//     barrier B(j-1)
//     issue slice j+1 -> other stage          (free: every wave finished reading slice j-1)
//     fetch k-step 0 of slice j               (visible since B(j-1))
//     MFMA  k-step 3 of slice j-1             (fragments were read before B(j-1))
//     fetch 1, MFMA 0; fetch 2, MFMA 1; fetch 3, MFMA 2
//     wait: own LDS reads done, own loads of slice j+1 landed;  barrier B(j)
// The barrier sits between two MFMA batches, so the matrix pipe keeps working while waves wait
// for each other, and there is one barrier per 64 of K.  Each stage is its own __shared__
// array so the compiler's tracking of pending global->LDS writes does not stall the LDS reads
// of the other stage; buffer loads (not flat/global) keep the lgkmcnt waits exact.
//
// LDS layouts (TS * 128 bytes per operand slice).  The LDS serves a 16-byte read sixteen lanes
// at a time, one 16-byte bank group per lane, and an 8-byte read thirty-two lanes at a time:
//   KC: TS rows of 128 bytes; chunk c of row r sits at slot c ^ ((r >> 1) & 7); fragments are
//       read with ds_read_b128.
//   MN: 64 k-rows of 2 TS bytes; 16-byte chunk c of k-row k sits at slot c ^ (4 (k & 3));
//       fragments are read with ds_read_b64_tr_b16, which hands lane i of a 16-lane group
//       column i of the 4 x 16 block whose rows the group's lanes address.
// The global->LDS load writes its 64 lanes in order, so each lane fetches the chunk that
// belongs in its slot.
//
// Symmetric outputs: only tiles with tile_m <= tile_n are computed; off-diagonal tiles are
// also stored mirrored (from the same staged copy, with transposing LDS reads).
// The s x s products can also keep their matrices in upper-block storage (sym_store): the
// mirrored store is skipped outside the diagonal 256 x 256 blocks, and a product reads block
// (r, c), r > c, of an operand as the transpose of block (c, r) -- the K walk then changes the
// operand form (MN for the transposed blocks, KC for the stored ones) at block boundaries.
// A third fewer bytes go to and come from memory, which is what bounds those products.
#include "common.h"
#include "../../include/signmuon_debug.h"
#include <type_traits>

namespace sm_gemm {

constexpr int BK = 64, NTH = 512;

typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
#define LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))

__device__ __forceinline__ const bf16_t* uniform_ptr(const bf16_t* p) {
  const unsigned long long v = reinterpret_cast<unsigned long long>(p);
  const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v);
  const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
  return reinterpret_cast<const bf16_t*>(((unsigned long long)hi << 32) | lo);
}

// Per-lane constants of one operand: where its global->LDS loads read, where its fragments sit.
template <bool MN, int TS>
struct operand_lane {
  static constexpr int NLOAD = TS / 64;  // wave-loads of this operand per wave and slice
  static constexpr int ROWB = TS * 2;    // MN: bytes per k-row
  int voff[NLOAD];  // byte offset of this lane's wave-loads inside the operand (slice offset is scalar)
  int frag_off;     // KC: LDS byte offset of this lane's row in fragment 0
  int frag_mn[4];   // MN: LDS byte offset of fragment f (k-step 0, first half) for this lane
  int ks_off[4];    // offset of k-step 0..3 inside the slice
  int kstep;        // scalar byte step per K slice

  // row0: first tile row of the workgroup; wrow: first row of this wave's sub-tile inside the tile
  __device__ __forceinline__ void init(int lane, int wv, int row0, int rows, int ld, int wrow) {
    if (!MN) {
#pragma unroll
      for (int q = 0; q < NLOAD; ++q) {
        const int row = 8 * (NLOAD * wv + q) + (lane >> 3);
        const int chunk = (lane & 7) ^ ((row >> 1) & 7);
        voff[q] = (min(row0 + row, rows - 1) * ld + chunk * 8) * 2;
      }
      const int fr = lane & 31, fg = lane >> 5, fsw = (fr >> 1) & 7;  // same swizzle for rows fr + 32 f
      frag_off = (wrow + fr) * (BK * 2);
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) ks_off[ks] = ((2 * ks + fg) ^ fsw) * 16;
      kstep = BK * 2;
    } else {
      constexpr int LPR = ROWB / 16;  // lanes (16-byte chunks) per k-row
      constexpr int KPL = 64 / LPR;   // k-rows per wave-load
#pragma unroll
      for (int q = 0; q < NLOAD; ++q) {
        const int k = KPL * (NLOAD * wv + q) + lane / LPR;
        const int chunk = (lane % LPR) ^ (4 * (k & 3));
        voff[q] = (k * ld + min(row0 + chunk * 8, rows - 8)) * 2;
      }
      // transposed read: 16-lane group g16, lane i in it; the group covers columns 16 (g16 & 1) ..+15
      // and k rows 8 (g16 >> 1) + 4 h + (i >> 2), h = 0, 1
      const int i = lane & 15, g16 = lane >> 4;
      const int col = wrow + 16 * (g16 & 1) + 4 * (i & 3);
      const int k = 8 * (g16 >> 1) + (i >> 2);
#pragma unroll
      for (int f = 0; f < 4; ++f)  // fragment f lies 32 columns further
        frag_mn[f] = k * ROWB + ((((col + 32 * f) >> 3) ^ (4 * (i >> 2))) << 4) + (col & 7) * 2;
      frag_off = 0;
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) ks_off[ks] = 16 * ks * ROWB;
      kstep = BK * ld * 2;
    }
  }
  // fragment f (32 rows further per f) of k-step ks from stage base s
  __device__ __forceinline__ bf16x8 fetch(const unsigned char* s, int f, int ks) const {
    if (!MN) {
      return *reinterpret_cast<const bf16x8*>(s + frag_off + f * 32 * (BK * 2) + ks_off[ks]);
    } else {
      const unsigned char* p = s + frag_mn[f] + ks_off[ks];
      const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p));
      const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p + 4 * ROWB));
      const s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
      return __builtin_bit_cast(bf16x8, v);
    }
  }
};

// 16-bit storage <-> fp32 for either element type
__device__ __forceinline__ unsigned pack2(float lo, float hi, bool f16) {
  if (f16) {
    const f16x2 v = {(_Float16)lo, (_Float16)hi};
    return __builtin_bit_cast(unsigned, v);
  }
  const bf16x2 v = {(bf16_t)lo, (bf16_t)hi};
  return __builtin_bit_cast(unsigned, v);
}
__device__ __forceinline__ void unpack2(unsigned w, bool f16, float& lo, float& hi) {
  if (f16) {
    const f16x2 v = __builtin_bit_cast(f16x2, w);
    lo = (float)v[0];
    hi = (float)v[1];
  } else {
    lo = __uint_as_float(w << 16);
    hi = __uint_as_float(w & 0xFFFF0000u);
  }
}

// x >= 0 for a bf16 bit pattern (IEEE comparison: -0 counts as >= 0, NaN does not)
__device__ __forceinline__ unsigned ge0_bf16(unsigned h) {
  const unsigned mag = h & 0x7FFFu;
  return (mag == 0u) | (((h >> 15) == 0u) & (mag <= 0x7F80u));
}

// One TS x TS tile of one problem.  The four stage arrays are the kernel's own __shared__
// variables, passed by reference so that every access keeps its identity after inlining.
template <int TS, bool A_MN, bool B_MN, bool SYM, bool F16, bool SYMSTORE = false>
__device__ __forceinline__ void gemm_tile(const sm_gemm_args& args, const sm_gemm_prob& P, int b, int tm, int tn,
                                          unsigned char (&sA0)[TS * 128], unsigned char (&sA1)[TS * 128],
                                          unsigned char (&sB0)[TS * 128], unsigned char (&sB1)[TS * 128]) {
  constexpr int WM = TS / 2, WN = TS / 4, FM = TS / 64, FN = TS / 128, NLOAD = TS / 64;
  const int m0 = tm * TS, n0 = tn * TS;
  const int M = P.M, N = P.N, K = P.K;
  // the operand bases depend on the workgroup only: pin them to scalar registers so that the
  // buffer descriptors are wave-uniform (no waterfall loop around the loads)
  const bf16_t* __restrict__ A = uniform_ptr(P.A + (long long)b * P.sA);
  const bf16_t* __restrict__ B = uniform_ptr(P.B + (long long)b * P.sB);

  // Opaque copy of the thread id: everything derived from it is recomputed per tile instead of
  // being hoisted out of the persistent tile loop for both operand layouts at once (which
  // would cost more registers than the kernel has).
  int tid = threadIdx.x;
  asm volatile("" : "+v"(tid));
  const int lane = tid & 63, wv = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform
  const int w_m = wv & 1, w_n = wv >> 1;

  // ---- global -> LDS: TS/8 wave-loads per operand slice; this wave issues NLOAD of A and of B.
  // Buffer loads: the per-lane byte offset is fixed for the whole K walk, the slice offset is scalar.
  const __amdgpu_buffer_rsrc_t ra = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(A), 0, 0x7FFFFFFF, 0x00020000);
  const __amdgpu_buffer_rsrc_t rb = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(B), 0, 0x7FFFFFFF, 0x00020000);
  operand_lane<A_MN, TS> oa;
  operand_lane<B_MN, TS> ob;
  oa.init(lane, wv, m0, M, P.lda, w_m * WM);
  ob.init(lane, wv, n0, N, P.ldb, w_n * WN);
  // plain locals: the buffer-load builtin is not instantiated on the host side when its
  // operands are member expressions of a dependent type
  int va[NLOAD], vb[NLOAD];
#pragma unroll
  for (int q = 0; q < NLOAD; ++q) {
    va[q] = oa.voff[q];
    vb[q] = ob.voff[q];
  }
  const int ksa = __builtin_amdgcn_readfirstlane(oa.kstep), ksb = __builtin_amdgcn_readfirstlane(ob.kstep);
#define ISSUE_V(sa, sb, slice, VA, KSA, VB, KSB)                                                                     \
  {                                                                                                                   \
    _Pragma("unroll") for (int q = 0; q < NLOAD; ++q) {                                                               \
      const int voa = VA[q], vob = VB[q];                                                                             \
      __builtin_amdgcn_raw_ptr_buffer_load_lds(ra, LDS_PTR((sa) + (NLOAD * wv + q) * 1024), 16, voa, (slice) * (KSA), \
                                               0, 0);                                                                 \
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rb, LDS_PTR((sb) + (NLOAD * wv + q) * 1024), 16, vob, (slice) * (KSB), \
                                               0, 0);                                                                 \
    }                                                                                                                 \
  }
#define ISSUE(sa, sb, slice) ISSUE_V(sa, sb, slice, va, ksa, vb, ksb)

  f32x16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // two fragment sets: while the matrix pipe works through one, the LDS reads of the other are in flight
  bf16x8 fa[2][FM], fb[2][FN];
#define FETCH_L(set, sa, sb, ks, LA, LB)                                                \
  {                                                                                     \
    _Pragma("unroll") for (int i = 0; i < FM; ++i) fa[set][i] = LA.fetch(sa, i, ks);    \
    _Pragma("unroll") for (int j = 0; j < FN; ++j) fb[set][j] = LB.fetch(sb, j, ks);    \
  }
#define FETCH(set, sa, sb, ks) FETCH_L(set, sa, sb, ks, oa, ob)
#define MMA(set)                                                                                                \
  {                                                                                                             \
    _Pragma("unroll") for (int i = 0; i < FM; ++i) _Pragma("unroll") for (int j = 0; j < FN; ++j) {             \
      if (F16)                                                                                                  \
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, fb[set][j]),               \
                                                           __builtin_bit_cast(f16x8, fa[set][i]), acc[i][j], 0, 0, 0); \
      else                                                                                                      \
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[set][j], fa[set][i], acc[i][j], 0, 0, 0);        \
    }                                                                                                           \
  }
#define SB() __builtin_amdgcn_sched_barrier(0)
  // wait for this wave's LDS reads and global->LDS loads, then meet the other waves
#define SYNC()                                    \
  {                                               \
    __builtin_amdgcn_s_waitcnt(0x0070);           \
    __builtin_amdgcn_s_barrier();                 \
    asm volatile("" ::: "memory");                \
  }
  // Slice j sits in (ca, cb); slice j + 1 goes to (na, nb).  On entry fragment set 1 holds k-step 3
  // of the previous slice (garbage-free zeros for the first slice: see below).
#define SLICE_STEP(ca, cb, na, nb, first)                                 \
  {                                                                       \
    ISSUE(na, nb, min(j + 1, nk - 1));                                    \
    FETCH(0, ca, cb, 0);                                                  \
    SB();                                                                 \
    if (!(first)) MMA(1);                                                 \
    SB();                                                                 \
    FETCH(1, ca, cb, 1);                                                  \
    SB();                                                                 \
    MMA(0);                                                               \
    SB();                                                                 \
    FETCH(0, ca, cb, 2);                                                  \
    SB();                                                                 \
    MMA(1);                                                               \
    SB();                                                                 \
    FETCH(1, ca, cb, 3);                                                  \
    SB();                                                                 \
    MMA(0);                                                               \
    SB();                                                                 \
    SYNC();                                                               \
    ++j;                                                                  \
    if (j < nk) SHIFT_DIAG(na, nb, j);                                    \
  }

  // Optional identity shift of the operands, opA + a_diag I and opB + b_diag I (half precision,
  // K-contiguous): the diagonal crosses a slice only inside the tile's own row (column) range, and
  // there one wave per operand adds the shift to the 64 diagonal elements of the slice in LDS,
  // after the slice has landed and before any fragment of it is read.
  const _Float16 dga = (_Float16)args.a_diag, dgb = (_Float16)args.b_diag;
  const bool dg_a = F16 && args.a_diag != 0.f, dg_b = F16 && args.b_diag != 0.f;
#define SHIFT_DIAG(sa, sb, slice)                                                                      \
  if (F16 && (dg_a || dg_b)) {                                                                         \
    const int ra = (slice) * BK - m0, rb = (slice) * BK - n0; /* tile row of the slice's first k */   \
    const bool ha = dg_a && ra >= 0 && ra < TS, hb = dg_b && rb >= 0 && rb < TS;                       \
    if (ha || hb) {                                                                                    \
      if (wv == 0 && ha) {                                                                             \
        const int r = ra + lane;                                                                       \
        _Float16* e = reinterpret_cast<_Float16*>((sa) + r * (BK * 2) + (((lane >> 3) ^ ((r >> 1) & 7)) << 4)) + (lane & 7); \
        *e = (_Float16)(*e + dga);                                                                     \
      }                                                                                                \
      if (wv == 1 && hb) {                                                                             \
        const int r = rb + lane;                                                                       \
        _Float16* e = reinterpret_cast<_Float16*>((sb) + r * (BK * 2) + (((lane >> 3) ^ ((r >> 1) & 7)) << 4)) + (lane & 7); \
        *e = (_Float16)(*e + dgb);                                                                     \
      }                                                                                                \
      __syncthreads();                                                                                 \
    }                                                                                                  \
  }
  const int nk = K / BK;
  int j = 0;
  if constexpr (!SYMSTORE) {
    ISSUE(sA0, sB0, 0);
    SYNC();
    SHIFT_DIAG(sA0, sB0, 0);
    // first slice: no pending k-step from a previous slice
    SLICE_STEP(sA0, sB0, sA1, sB1, true);
    // Past the end the issue re-reads the last slice (never consumed), so every step has the same shape.
    while (j + 1 < nk) {
      SLICE_STEP(sA1, sB1, sA0, sB0, false);
      SLICE_STEP(sA0, sB0, sA1, sB1, false);
    }
    if (j < nk) SLICE_STEP(sA1, sB1, sA0, sB0, false);
  } else {
    // Operands are symmetric matrices of which only the 256 x 256 blocks on and above the diagonal
    // hold valid data (M == N == K).  Block (r, c) with r > c is read as the transpose of block
    // (c, r): its K slices are fetched k-row by k-row (the MN form).  With J1 / J2 the first slice
    // of the tile's own row block / column block, the K walk has three phases,
    //   [0, J1): A and B transposed;   [J1, J2): A as stored, B transposed;   [J2, nk): both as stored,
    // each a multiple of four slices long, so every phase starts in stage 0; the last step of a
    // phase issues the first slice of the next in that phase's form.
    const int J1 = (m0 / 256) * 4, J2 = (n0 / 256) * 4;
    operand_lane<true, TS> ma, mb;
    ma.init(lane, wv, m0, M, P.lda, w_m * WM);
    mb.init(lane, wv, n0, N, P.ldb, w_n * WN);
    int vam[NLOAD], vbm[NLOAD];
#pragma unroll
    for (int q = 0; q < NLOAD; ++q) {
      vam[q] = ma.voff[q];
      vbm[q] = mb.voff[q];
    }
    const int ksam = __builtin_amdgcn_readfirstlane(ma.kstep), ksbm = __builtin_amdgcn_readfirstlane(mb.kstep);
    // fragment set 1 starts as zeros, so the first step can run its "previous k-step" like any other
#pragma unroll
    for (int i = 0; i < FM; ++i) fa[1][i] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < FN; ++i) fb[1][i] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
#define ISSUE_MM(sa, sb, slice) ISSUE_V(sa, sb, slice, vam, ksam, vbm, ksbm)
#define ISSUE_KM(sa, sb, slice) ISSUE_V(sa, sb, slice, va, ksa, vbm, ksbm)
#define ISSUE_KK(sa, sb, slice) ISSUE_V(sa, sb, slice, va, ksa, vb, ksb)
#define ISSUE_KKC(sa, sb, slice) ISSUE_KK(sa, sb, min((slice), nk - 1))
#define ISSUE_AT(sa, sb, slice)                  \
  {                                              \
    if ((slice) < J1) {                          \
      ISSUE_MM(sa, sb, slice);                   \
    } else if ((slice) < J2) {                   \
      ISSUE_KM(sa, sb, slice);                   \
    } else {                                     \
      ISSUE_KK(sa, sb, min((slice), nk - 1));    \
    }                                            \
  }
#define STEP3(ca, cb, na, nb, LA, LB, ISSUE_NEXT)                         \
  {                                                                       \
    ISSUE_NEXT(na, nb, j + 1);                                            \
    FETCH_L(0, ca, cb, 0, LA, LB);                                        \
    SB();                                                                 \
    MMA(1);                                                               \
    SB();                                                                 \
    FETCH_L(1, ca, cb, 1, LA, LB);                                        \
    SB();                                                                 \
    MMA(0);                                                               \
    SB();                                                                 \
    FETCH_L(0, ca, cb, 2, LA, LB);                                        \
    SB();                                                                 \
    MMA(1);                                                               \
    SB();                                                                 \
    FETCH_L(1, ca, cb, 3, LA, LB);                                        \
    SB();                                                                 \
    MMA(0);                                                               \
    SB();                                                                 \
    SYNC();                                                               \
    ++j;                                                                  \
    if (j < nk) SHIFT_DIAG(na, nb, j);                                    \
  }
#define PHASE3(LA, LB, ISSUE_SAME, jend)                                  \
  if (j < (jend)) {                                                       \
    while (j + 2 < (jend)) {                                              \
      STEP3(sA0, sB0, sA1, sB1, LA, LB, ISSUE_SAME);                      \
      STEP3(sA1, sB1, sA0, sB0, LA, LB, ISSUE_SAME);                      \
    }                                                                     \
    STEP3(sA0, sB0, sA1, sB1, LA, LB, ISSUE_SAME);                        \
    STEP3(sA1, sB1, sA0, sB0, LA, LB, ISSUE_AT);                          \
  }
    ISSUE_AT(sA0, sB0, 0);
    SYNC();
    SHIFT_DIAG(sA0, sB0, 0);
    PHASE3(ma, mb, ISSUE_MM, J1);
    PHASE3(oa, mb, ISSUE_KM, J2);
    // last phase: any number of slices; past the end the issue re-reads the last slice (never consumed)
    STEP3(sA0, sB0, sA1, sB1, oa, ob, ISSUE_KKC);
    while (j + 1 < nk) {
      STEP3(sA1, sB1, sA0, sB0, oa, ob, ISSUE_KKC);
      STEP3(sA0, sB0, sA1, sB1, oa, ob, ISSUE_KKC);
    }
    if (j < nk) STEP3(sA1, sB1, sA0, sB0, oa, ob, ISSUE_KKC);
#undef PHASE3
#undef STEP3
#undef ISSUE_AT
#undef ISSUE_KKC
#undef ISSUE_KK
#undef ISSUE_KM
#undef ISSUE_MM
  }
  MMA(1);  // k-step 3 of the last slice
#undef SLICE_STEP
#undef SHIFT_DIAG
#undef SYNC
#undef SB
#undef FETCH
#undef FETCH_L
#undef MMA
#undef ISSUE
#undef ISSUE_V

  // ---- epilogue straight from the accumulators: a lane holds row m and 4 consecutive columns
  float s = 1.f;
  if (P.scale && args.scale_pow) {
    s = P.scale[b];
    if (args.scale_pow == 2) s *= s;
  }
  const float alpha = args.alpha * s;
  const bool of16 = args.out_f16 != 0;
  bf16_t* __restrict__ C = P.C ? P.C + (long long)b * P.sC : nullptr;
  // a fresh opaque thread id: the store addresses are worked out here, after the K loop,
  // instead of being carried through it in registers
  int etid = threadIdx.x;
  asm volatile("" : "+v"(etid));
  const int elane = etid & 63, ewv = __builtin_amdgcn_readfirstlane(etid >> 6);  // wave-uniform
  const int e_m = ewv & 1, e_n = ewv >> 1;
  const int fr = elane & 31, fg = elane >> 5;
  if constexpr (!SYM) {
    // Only the packed 1-bit signs of the tile are wanted (the apply before the vote): they are taken
    // straight from the accumulators.  A lane holds, per 32 x 32 fragment, 16 entries of one row:
    // columns 8 vg + 4 fg + e of the fragment's 32.  For every value but -0, a negative denormal
    // and NaN, "the bf16 rounding of x is >= 0" is just "the sign bit of x is clear", which one
    // alignbit shifts into a word; a wave that meets one of those three recomputes its bits from
    // the rounded values, so the result is that of the staged path bit for bit.
    if (!C && P.sign_out && P.sign_fmt == SM_SIGN_1BIT && args.diag == 0.f && !of16) {
      unsigned words[FM][FN];
      bool rare = false;
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int jn = 0; jn < FN; ++jn) {
          unsigned neg = 0;
#pragma unroll
          for (int v = 15; v >= 0; --v) {
            const float o = alpha * acc[i][jn][v];
            rare |= __builtin_amdgcn_classf(o, 0x33);  // sNaN, qNaN, -denormal, -0
            neg = __builtin_amdgcn_alignbit(neg, __float_as_uint(o), 31);
          }
          words[i][jn] = ~neg & 0xFFFFu;  // bit 4 vg + e
        }
      if (__builtin_amdgcn_ballot_w64(rare) != 0) {
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
          for (int jn = 0; jn < FN; ++jn) {
            unsigned bits = 0;
#pragma unroll
            for (int v = 0; v < 16; v += 2) {
              const unsigned h = pack2(alpha * acc[i][jn][v], alpha * acc[i][jn][v + 1], false);
              bits |= (ge0_bf16(h & 0xFFFFu) << v) | (ge0_bf16(h >> 16) << (v + 1));
            }
            words[i][jn] = bits;
          }
      }
      unsigned char* so = reinterpret_cast<unsigned char*>(P.sign_out) + (long long)b * P.sign_stride;
#pragma unroll
      for (int i = 0; i < FM; ++i) {
        const int mg = m0 + e_m * WM + i * 32 + fr;
#pragma unroll
        for (int jn = 0; jn < FN; ++jn) {
          // nibble vg -> bits 8 vg + 4 fg .. + 3; the lane 32 further holds the other half of the word
          const unsigned x = words[i][jn];
          unsigned w = ((x & 0xFu) | ((x & 0xF0u) << 4) | ((x & 0xF00u) << 8) | ((x & 0xF000u) << 12)) << (4 * fg);
          w |= __shfl_xor(w, 32, 64);
          const int c0 = n0 + e_n * WN + jn * 32;
          if ((jn & 1) == fg && mg < P.sign_rows && c0 < P.sign_cols)  // sign_cols % 32 == 0: a word is live as a whole
            *reinterpret_cast<unsigned*>(so + (((long long)mg * P.sign_cols + c0) >> 3)) = w;
        }
      }
      return;
    }
  }
  // upper-only output (sym_store bit 1): the mirrored tile is written only inside a diagonal 256 x 256 block
  const bool mirror = SYM && (tm != tn) && (!(args.sym_store & 2) || (m0 / 256 == n0 / 256));
  // The tile leaves through LDS so that every global store is a 16-byte piece of a row.  The four
  // stage arrays hold 64 tile rows each (rows of TS * 2 bytes, 16-byte chunk c of row r at slot
  // c ^ (r & (CPR - 1))).  The tile is staged once; it is read out row by row for C and, for an
  // off-diagonal tile of a symmetric output, once more column by column (transposing LDS reads)
  // for the mirrored tile.  The R term (a symmetric matrix when the output is) is added at
  // read-out, on the rounded product, with loads shaped like the stores.
  constexpr int RB = TS * 2, CPR = TS / 8, RPP = NTH / CPR, PASSES = TS / RPP;
  const bf16_t* __restrict__ R = P.R ? P.R + (long long)b * P.sC : nullptr;
  const bool rf16 = args.r_f16 != 0;
  const float gamma = args.gamma;
  // 8 staged outputs + gamma times 8 elements of R, rounded again.  When both are half precision and
  // gamma is a half-precision number (the paper's coefficients give -0.5390625), packed
  // half-precision fmas do it with a single rounding and no conversions.
  const _Float16 gamma_h = (_Float16)gamma;
  const int r_mode = (of16 && rf16 && (float)gamma_h == gamma) ? 2 : (of16 ? 1 : 0) | (rf16 ? 4 : 0);
  auto add_r = [&](u32x4 v, u32x4 a) -> u32x4 {
    if (r_mode == 2) {
      const f16x8 g8 = {gamma_h, gamma_h, gamma_h, gamma_h, gamma_h, gamma_h, gamma_h, gamma_h};
      return __builtin_bit_cast(u32x4, __builtin_elementwise_fma(g8, __builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, v)));
    }
    const bool o16 = (r_mode & 1) != 0, r16 = (r_mode & 4) != 0;
    u32x4 w;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      float lo, hi, alo, ahi;
      unpack2(v[q], o16, lo, hi);
      unpack2(a[q], r16, alo, ahi);
      lo += gamma * alo;
      hi += gamma * ahi;
      w[q] = pack2(lo, hi, o16);
    }
    return w;
  };
  auto stage = [&](int idx) -> unsigned char* { return idx == 0 ? sA0 : idx == 1 ? sA1 : idx == 2 ? sB0 : sB1; };
  // the staging loop in four forms: with or without the check for diagonal entries (only tiles that
  // meet the diagonal of a product with a diag term need it) and for either output type, so that
  // neither costs vector instructions per entry where it does not apply
  auto stage_tile = [&](auto on_diag, auto half) {
    constexpr bool ON_DIAG = decltype(on_diag)::value, HALF = decltype(half)::value;
#pragma unroll
    for (int i = 0; i < FM; ++i) {
      const int ml = e_m * WM + i * 32 + fr;  // tile row of this lane
      const int mg = m0 + ml;
      // rows e_m*WM + i*32 .. +31 lie in one stage array (64 rows each): uniform choice
      unsigned char* sp = stage((e_m * WM + i * 32) >> 6);
#pragma unroll
      for (int jn = 0; jn < FN; ++jn) {
#pragma unroll
        for (int vg = 0; vg < 4; ++vg) {
          const int nl = e_n * WN + jn * 32 + 8 * vg + 4 * fg;  // first of 4 tile columns
          const int ng = n0 + nl;
          float o[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            o[e] = alpha * acc[i][jn][4 * vg + e];
            if (ON_DIAG && mg == ng + e) o[e] += args.diag;
          }
          const u32x2 h = {pack2(o[0], o[1], HALF), pack2(o[2], o[3], HALF)};
          *reinterpret_cast<u32x2*>(sp + (ml & 63) * RB + ((((nl >> 3) ^ (ml & (CPR - 1)))) << 4) + (nl & 7) * 2) = h;
        }
      }
    }
  };
  const bool diag_tile = args.diag != 0.f && m0 < n0 + TS && n0 < m0 + TS;
  if (diag_tile) {
    if (of16) stage_tile(std::true_type{}, std::true_type{}); else stage_tile(std::true_type{}, std::false_type{});
  } else {
    if (of16) stage_tile(std::false_type{}, std::true_type{}); else stage_tile(std::false_type{}, std::false_type{});
  }
  __syncthreads();
  if (SYM || C) {
    // rows: thread t handles chunk t % CPR of rows t / CPR + RPP * k
    const int rc = etid % CPR, rr = etid / CPR;
    const int gc = n0 + rc * 8;
    // with an R term: all of its pieces are requested before the first is used, so the read-out
    // pays one memory latency, not one per piece
    u32x4 rv[PASSES];
    if (R) {
#pragma unroll
      for (int k = 0; k < PASSES; ++k) {
        const int gr = m0 + rr + RPP * k;
        rv[k] = u32x4{0u, 0u, 0u, 0u};
        if (gr < M && gc < N) rv[k] = *reinterpret_cast<const u32x4*>(R + (long long)gr * P.ldc + gc);
      }
    }
#pragma unroll
    for (int k = 0; k < PASSES; ++k) {
      const int row = rr + RPP * k;  // tile row; (row >> 6) == (RPP * k) >> 6 is a constant
      const unsigned char* sp = stage((RPP * k) >> 6);
      const u32x4 v = *reinterpret_cast<const u32x4*>(sp + (row & 63) * RB + ((rc ^ (row & (CPR - 1))) << 4));
      const int gr = m0 + row;
      if (gr < M && gc < N) {
        const long long off = (long long)gr * P.ldc + gc;
        *reinterpret_cast<u32x4*>(C + off) = R ? add_r(v, rv[k]) : v;
      }
    }
  }
  if (!SYM && P.sign_out) {
    // packed signs of the tile: NTH / TS threads per tile row, each turning CPT consecutive columns
    // of the staged row into CPT / 8 bytes (1 bit) or CPT bytes (int8)
    constexpr int TPR = NTH / TS, CPT = TS / TPR, NCH = CPT / 8;
    const int row = etid / TPR, part = etid % TPR;
    const int gr = m0 + row, gc0 = n0 + part * CPT;
    const unsigned char* sp = stage(row >> 6) + (row & 63) * RB;
    unsigned char* so = reinterpret_cast<unsigned char*>(P.sign_out) + (long long)b * P.sign_stride;
    const long long e0 = (long long)gr * P.sign_cols + gc0;  // first entry; a multiple of 32
    unsigned word = 0;
#pragma unroll
    for (int q = 0; q < NCH; ++q) {
      const u32x4 w = *reinterpret_cast<const u32x4*>(sp + (((part * NCH + q) ^ (row & (CPR - 1))) << 4));
      unsigned bits = 0;
#pragma unroll
      for (int h = 0; h < 4; ++h)
        bits |= (ge0_bf16(w[h] & 0xFFFFu) << (2 * h)) | (ge0_bf16(w[h] >> 16) << (2 * h + 1));
      const bool live = gr < P.sign_rows && gc0 + 8 * q < P.sign_cols;
      if (P.sign_fmt == SM_SIGN_1BIT) {
        word |= bits << (8 * (q & 3));
        if ((q & 3) == 3) {
          // 32 columns per store; sign_cols is a multiple of 32, so a word is live as a whole
          if (live) *reinterpret_cast<unsigned*>(so + ((e0 + 8 * (q - 3)) >> 3)) = word;
          word = 0;
        }
      } else if (live) {
        u32x2 s8;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          unsigned v4 = 0;
#pragma unroll
          for (int k = 0; k < 4; ++k) v4 |= (((bits >> (4 * h + k)) & 1u) ? 0x01u : 0xFFu) << (8 * k);
          s8[h] = v4;
        }
        *reinterpret_cast<u32x2*>(so + e0 + 8 * q) = s8;
      }
    }
  }
  if (mirror) {
    // columns: a 16-lane group reads 8 tile rows x 16 tile columns with two transposing reads (lane i
    // addresses row i / 4, 8-byte segment i % 4 of a 4 x 16 block and receives column i), which
    // leaves lane i with 8 consecutive elements of row (column block + i) of the mirrored tile.
    // The four groups of a wave take neighbouring row chunks, i.e. 64 contiguous bytes per row.
    constexpr int NRC = TS / 8;         // 8-row chunks in the tile
    constexpr int CPI = 32 / NRC;       // 16-column blocks covered per iteration by the 32 groups
    const int G = etid >> 4, i16 = etid & 15;
    const int rchunk = G % NRC;
    const unsigned char* sp = stage((8 * (ewv * 4 % NRC)) >> 6);  // (8 * rchunk) >> 6 is wave-uniform
    const int r0 = 8 * rchunk + (i16 >> 2);
    constexpr int MIT = (TS / 16) / CPI;
    const int gc = m0 + 8 * rchunk;
    u32x4 rv[MIT];
    if (R) {
#pragma unroll
      for (int k = 0; k < MIT; ++k) {
        const int gr = n0 + 16 * (CPI * k + G / NRC) + i16;
        rv[k] = u32x4{0u, 0u, 0u, 0u};
        if (gr < N && gc < M) rv[k] = *reinterpret_cast<const u32x4*>(R + (long long)gr * P.ldc + gc);
      }
    }
#pragma unroll
    for (int k = 0; k < MIT; ++k) {
      const int cb = 16 * (CPI * k + G / NRC);
      const int col = cb + 4 * (i16 & 3);
      const unsigned char* p0 = sp + (r0 & 63) * RB + ((((col >> 3) ^ (r0 & (CPR - 1)))) << 4) + (col & 7) * 2;
      const unsigned char* p1 = sp + ((r0 + 4) & 63) * RB + ((((col >> 3) ^ ((r0 + 4) & (CPR - 1)))) << 4) + (col & 7) * 2;
      const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p0));
      const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p1));
      const s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
      const int gr = n0 + cb + i16;
      if (gr < N && gc < M) {
        const long long off = (long long)gr * P.ldc + gc;
        const u32x4 vv = __builtin_bit_cast(u32x4, v);
        *reinterpret_cast<u32x4*>(C + off) = R ? add_r(vv, rv[k]) : vv;
      }
    }
  }
}

// Tile t of a matrix's list.  The list goes through the tile grid in bands of BR tile rows and, inside a band,
// column by column with the rows running fastest (a symmetric output: only tiles with tile_m <= tile_n; a band
// starts with the upper triangle of its diagonal block, column by column).  The workgroups of an XCD work on
// about 32 (TS = 256) or 64 (TS = 128) neighbouring entries of the list at any one time: a run of that length
// covers BR rows and 8 columns, i.e. it needs BR + 8 operand panels instead of the 16 + 2 of a run down whole
// columns of a 16 x 16 grid, and every panel it needs is shared by tiles that run together, so it crosses HBM
// once per run.  A grid of up to BR rows (s <= 1024 at TS = 256) is a single band.
template <bool SYM, int BR>
__host__ __device__ __forceinline__ void tile_of(int t, int tiles_m, int tiles_n, int& tm, int& tn) {
  if (SYM) {
    const int T = tiles_m;
    int r0 = 0, h;
    for (;;) {
      h = (T - r0 < BR) ? T - r0 : BR;
      const int cnt = h * (h + 1) / 2 + (T - r0 - h) * h;
      if (t < cnt || r0 + h >= T) break;
      t -= cnt;
      r0 += h;
    }
    const int d = h * (h + 1) / 2;
    if (t < d) {  // diagonal block: (0,0) (0,1) (1,1) (0,2) ...
      int c = 0;
      while (t > c) {
        t -= c + 1;
        ++c;
      }
      tm = r0 + t;
      tn = r0 + c;
    } else {
      t -= d;
      const int c = t / h;
      tm = r0 + (t - c * h);
      tn = r0 + h + c;
    }
  } else {
    const int per_band = BR * tiles_n;
    const int b = t / per_band;
    t -= b * per_band;
    const int h = (tiles_m - b * BR < BR) ? tiles_m - b * BR : BR;
    tn = t / h;
    tm = b * BR + (t - tn * h);
  }
}

// KIND 0: symmetric output, bf16 operands both KC or both MN; the upper triangle of tiles is computed.
// KIND 1: general output, bf16 operands (A is KC; B is KC or MN).
// KIND 2: symmetric output, half-precision operands, both KC.
// KIND 3: as 2, with operands of which only the blocks on and above the diagonal are valid.
template <int KIND, int TS>
__global__ void __launch_bounds__(NTH) sm_ns_gemm_kernel(const sm_gemm_args args) {
  constexpr bool SYM = (KIND != 1);
  __shared__ __attribute__((aligned(1024))) unsigned char sA0[TS * 128], sA1[TS * 128];
  __shared__ __attribute__((aligned(1024))) unsigned char sB0[TS * 128], sB1[TS * 128];

  // Persistent workgroups: the grid is one (TS = 256) or two (TS = 128) workgroups per CU and each
  // walks a list of tiles, so the global stores of one tile drain while the next tile is loaded
  // and multiplied.  Workgroup ids are dealt round-robin to the 8 XCDs: XCD x owns a contiguous
  // range of the tile list (ranges of equal estimated cost) and its workgroups take neighbouring
  // tiles at any one time, so tiles that share operand panels share an L2.
  const int wg = blockIdx.x;
  const int per_xcd_wgs = gridDim.x >> 3;
  const int xcd_first = args.xcd_begin[wg & 7], xcd_end = args.xcd_begin[(wg & 7) + 1];
  bool first_tile = true;
  for (int Lf = xcd_first + (wg >> 3); Lf < xcd_end; Lf += per_xcd_wgs) {
    // every other launch goes through the range backwards: it starts with the matrices the launch before it
    // wrote last, which are the ones still in the caches
    const int L = args.reverse ? xcd_first + xcd_end - 1 - Lf : Lf;
    if (!first_tile) __syncthreads();  // the previous tile has been read out of the stage arrays
    first_tile = false;
    int pi = 0;
    while (pi + 1 < args.n_prob && L >= args.p[pi + 1].tile_begin) ++pi;
    int t = L - args.p[pi].tile_begin;
    const int per_batch = SYM ? args.p[pi].tiles_m * (args.p[pi].tiles_m + 1) / 2 : args.p[pi].tiles_m * args.p[pi].tiles_n;
    const int mate = args.p[pi].mate;
    const int per_item = mate ? 2 * per_batch : per_batch;
    const int b = t / per_item;
    t -= b * per_item;
    if (t >= per_batch) {  // the mate's tile of the same item
      t -= per_batch;
      pi = mate;
    }
    const sm_gemm_prob& P = args.p[pi];
    int tm, tn;
    tile_of<SYM, (TS == 256 ? 4 : 8)>(t, P.tiles_m, P.tiles_n, tm, tn);
    if (KIND == 0) {
      if (P.layout == 0)
        gemm_tile<TS, false, false, true, false>(args, P, b, tm, tn, sA0, sA1, sB0, sB1);
      else
        gemm_tile<TS, true, true, true, false>(args, P, b, tm, tn, sA0, sA1, sB0, sB1);
    } else if (KIND == 1) {
      if (P.layout == 0)
        gemm_tile<TS, false, false, false, false>(args, P, b, tm, tn, sA0, sA1, sB0, sB1);
      else
        gemm_tile<TS, false, true, false, false>(args, P, b, tm, tn, sA0, sA1, sB0, sB1);
    } else if (KIND == 2) {
      gemm_tile<TS, false, false, true, true>(args, P, b, tm, tn, sA0, sA1, sB0, sB1);
    } else {
      gemm_tile<TS, false, false, true, true, true>(args, P, b, tm, tn, sA0, sA1, sB0, sB1);
    }
  }
}

// Tile bookkeeping shared by every instantiation.  A tile costs its K slices plus a fixed part
// (prologue and write-out, about six slices' worth); the list is cut into eight ranges of equal
// cost, one per XCD.  Returns the largest number of tiles any XCD owns.
static int fill_tiles(sm_gemm_args& args, bool sym, int ts) {
  constexpr double FIXED = 6.0;
  int total = 0;
  double cost = 0.0;
  bool is_mate[SM_GEMM_MAX_PROB] = {};
  for (int i = 0; i < args.n_prob; ++i)
    if (args.p[i].mate) is_mate[args.p[i].mate] = true;
  for (int i = 0; i < args.n_prob; ++i) {
    sm_gemm_prob& P = args.p[i];
    P.tiles_m = (P.M + ts - 1) / ts;
    P.tiles_n = (P.N + ts - 1) / ts;
    P.tile_begin = total;  // for a mate: the end of its leader's range, which the tile lookup steps over
    if (is_mate[i]) continue;
    const int n = (sym ? P.tiles_m * (P.tiles_m + 1) / 2 : P.tiles_m * P.tiles_n) * P.batch * (P.mate ? 2 : 1);
    total += n;
    cost += n * (P.K / 64 + FIXED);
  }
  args.total_tiles = total;
  args.xcd_begin[0] = 0;
  int pi = 0, x = 1;
  double done = 0.0;  // cost of the problems before pi
  while (x < 8 && pi < args.n_prob) {
    const sm_gemm_prob& P = args.p[pi];
    const int end = (pi + 1 < args.n_prob) ? args.p[pi + 1].tile_begin : total;  // == tile_begin for a mate
    const double per_tile = P.K / 64 + FIXED, target = cost * x / 8;
    const double here = done + (double)(end - P.tile_begin) * per_tile;
    if (here < target) {
      done = here;
      ++pi;
      continue;
    }
    int cut = P.tile_begin + (int)((target - done) / per_tile + 0.5);
    cut = std::min(std::max(cut, args.xcd_begin[x - 1]), end);
    args.xcd_begin[x++] = cut;
  }
  for (; x <= 8; ++x) args.xcd_begin[x] = total;
  int most = 0;
  for (int k = 0; k < 8; ++k) most = std::max(most, args.xcd_begin[k + 1] - args.xcd_begin[k]);
  return most;
}

}  // namespace sm_gemm
using namespace sm_gemm;

// Host-side check hook: the tile bookkeeping of a launch, without launching.  Fills xcd_begin[9] and
// tile_begin[n_prob]; returns the total number of tiles, or -1 on bad arguments.
extern "C" int signmuon_debug_tile_ranges(int n_prob, const int* M, const int* N, const int* K, const int* batch,
                                          const int* mate, int sym, int ts, int* xcd_begin, int* tile_begin) {
  if (n_prob < 1 || n_prob > SM_GEMM_MAX_PROB || (ts != 128 && ts != 256)) return -1;
  sm_gemm_args a;
  a.n_prob = n_prob;
  for (int i = 0; i < n_prob; ++i) {
    a.p[i].M = M[i];
    a.p[i].N = N[i];
    a.p[i].K = K[i];
    a.p[i].batch = batch[i];
    a.p[i].mate = mate ? mate[i] : 0;
    a.p[i].mu = a.p[i].nu = a.p[i].ku = 0;
  }
  fill_tiles(a, sym != 0, ts);
  for (int x = 0; x < 9; ++x) xcd_begin[x] = a.xcd_begin[x];
  for (int i = 0; i < n_prob; ++i) tile_begin[i] = a.p[i].tile_begin;
  return a.total_tiles;
}

// Host-side check hook: entry t of the tile list of one matrix with a tiles_m x tiles_n grid of ts-wide tiles
// (sym: the upper triangle of a square grid), as the kernels decode it.  Returns 0, or -1 on bad arguments.
extern "C" int signmuon_debug_tile_of(int t, int tiles_m, int tiles_n, int sym, int ts, int* tile_m, int* tile_n) {
  if (!tile_m || !tile_n || tiles_m < 1 || tiles_n < 1 || (ts != 128 && ts != 256) || (sym && tiles_m != tiles_n)) return -1;
  const int total = sym ? tiles_m * (tiles_m + 1) / 2 : tiles_m * tiles_n;
  if (t < 0 || t >= total) return -1;
  if (sym) {
    if (ts == 256) tile_of<true, 4>(t, tiles_m, tiles_n, *tile_m, *tile_n);
    else tile_of<true, 8>(t, tiles_m, tiles_n, *tile_m, *tile_n);
  } else {
    if (ts == 256) tile_of<false, 4>(t, tiles_m, tiles_n, *tile_m, *tile_n);
    else tile_of<false, 8>(t, tiles_m, tiles_n, *tile_m, *tile_n);
  }
  return 0;
}

// Per problem, P.layout bit 0: A is MN-contiguous, bit 1: B is MN-contiguous.  sym: symmetric
// output, layout 0 or 3 (A and B may differ as long as the product is symmetric).  Otherwise
// layout 0 or 2.  K multiple of 64.
int sm_launch_gemm(signmuon_ctx* ctx, sm_gemm_args& args, bool sym, int klass) {
  const bool gram = sym;
  for (int i = 0; i < args.n_prob; ++i) {
    const sm_gemm_prob& P = args.p[i];
    if (P.M % 64 || P.N % 64 || P.K % 64 || P.lda % 8 || P.ldb % 8 || P.ldc % 8 || !sm_aligned(P.A, 16) ||
        !sm_aligned(P.B, 16) || !sm_aligned(P.C, 16) || P.sA % 8 || P.sB % 8 || P.sC % 8 || (gram && P.M != P.N))
      return sm_fail(ctx, SM_EINVAL, "internal: GEMM operand not padded/aligned");
    if (gram ? (P.layout != 0 && P.layout != 3) : (P.layout != 0 && P.layout != 2))
      return sm_fail(ctx, SM_EUNSUPPORTED, "internal: GEMM layout combination not built");
    if (!sm_aligned(P.R, 16)) return sm_fail(ctx, SM_EINVAL, "internal: GEMM R term misaligned");
    if (!P.C && (sym || !P.sign_out)) return sm_fail(ctx, SM_EINVAL, "internal: GEMM without an output");
    if (P.mate) {
      if (P.mate <= i || P.mate >= args.n_prob) return sm_fail(ctx, SM_EINVAL, "internal: GEMM mate index");
      const sm_gemm_prob& Q = args.p[P.mate];
      if (Q.mate || Q.M != P.M || Q.N != P.N || Q.K != P.K || Q.batch != P.batch)
        return sm_fail(ctx, SM_EINVAL, "internal: GEMM mate of a different shape");
    }
    if (P.sign_out && (sym || args.out_f16 || P.R || P.sign_cols % 32 || P.sign_stride % 8 || !sm_aligned(P.sign_out, 8) ||
                       (P.sign_fmt != SM_SIGN_1BIT && P.sign_fmt != SM_SIGN_INT8)))
      return sm_fail(ctx, SM_EUNSUPPORTED, "internal: GEMM sign output needs a general bf16 product and cols % 32 == 0");
    if ((args.a_diag != 0.f || args.b_diag != 0.f) && !args.in_f16)
      return sm_fail(ctx, SM_EUNSUPPORTED, "internal: operand identity shift needs half-precision operands");
    if (args.in_f16 && (!sym || P.layout != 0))
      return sm_fail(ctx, SM_EUNSUPPORTED, "internal: half-precision GEMM operands need a symmetric K-contiguous product");
    if ((args.sym_store & 1) && (!args.in_f16 || P.M != P.K || P.N != P.K))
      return sm_fail(ctx, SM_EUNSUPPORTED, "internal: upper-block operands need a square half-precision product");
    if ((args.sym_store & 2) && !sym)
      return sm_fail(ctx, SM_EUNSUPPORTED, "internal: upper-block output needs a symmetric product");
    // buffer offsets are 32-bit
    const long long a_ext = (P.layout & 1) ? (long long)P.K * P.lda : (long long)P.M * P.lda;
    const long long b_ext = (P.layout & 2) ? (long long)P.K * P.ldb : (long long)P.N * P.ldb;
    if (a_ext * 2 >= 0x7FFFFFFFLL || b_ext * 2 >= 0x7FFFFFFFLL)
      return sm_fail(ctx, SM_EUNSUPPORTED, "internal: GEMM operand larger than 2 GiB");
  }
  int ts = ctx->opt[SM_OPT_GEMM_TILE];
  if (ts != 128 && ts != 256) {
    // 256 x 256 tiles once there are enough of them to keep 256 CUs busy for several rounds, unless the
    // matrices fill them badly (a 384-wide matrix covers one and a half: the small tile then computes a
    // third less)
    auto tile_area = [&](int t) {
      double area = 0.0;
      for (int i = 0; i < args.n_prob; ++i) {
        const sm_gemm_prob& P = args.p[i];
        const double tm = (P.M + t - 1) / t, tn = (P.N + t - 1) / t;
        area += (gram ? tm * (tm + 1) / 2 : tm * tn) * (double)t * t * P.batch;
      }
      return area;
    };
    fill_tiles(args, gram, 256);
    ts = (args.total_tiles >= 1024 && tile_area(256) <= 1.15 * tile_area(128)) ? 256 : 128;
  }
  const int most = fill_tiles(args, gram, ts);
  if (args.total_tiles == 0) return SM_OK;
  args.reverse = ctx->gemm_flip;
  ctx->gemm_flip ^= 1;
  // persistent grid: one workgroup per CU (two for the small tile), a multiple of 8, never more than tiles
  int wgs = ctx->n_cu * (ts == 128 ? 2 : 1);
  wgs = std::max(1, std::min(wgs / 8, most)) * 8;
  const dim3 grid(wgs), block(NTH);
  if ((ctx->profiling >> klass) & 1u) {
    for (int i = 0; i < args.n_prob; ++i) {
      const sm_gemm_prob& P = args.p[i];
      const double mnk = (double)P.M * P.N * P.K * P.batch;
      ctx->work_dense[klass] += 2.0 * mnk;
      // executed: the tiles this launch computes, each clipped to the logical extent of the product
      const int mu = P.mu ? P.mu : P.M, nu = P.nu ? P.nu : P.N, ku = P.ku ? P.ku : P.K;
      double area = 0.0;
      for (int tn = 0; tn < P.tiles_n; ++tn)
        for (int tm = 0; tm < (gram ? tn + 1 : P.tiles_m); ++tm)
          area += (double)std::max(0, std::min(ts, mu - tm * ts)) * std::max(0, std::min(ts, nu - tn * ts));
      ctx->work_flop[klass] += 2.0 * area * ku * P.batch;
      const bool same = (P.A == P.B);
      // upper-block storage: the share of an s x s matrix that lies in its 256 x 256 blocks on and above the diagonal
      auto upper_share = [](int s) {
        double kept = 0.0;
        for (int r = 0; r < s; r += 256) kept += (double)std::min(256, s - r) * (s - r);
        return kept / ((double)s * s);
      };
      const double in_share = (args.sym_store & 1) ? upper_share(P.K) : 1.0;
      const double out_share = (args.sym_store & 2) ? upper_share(P.M) : 1.0;
      const double r_share = (args.sym_store & 2) ? out_share : 1.0;  // R is read where the output is written
      ctx->work_bytes[klass] +=
          2.0 * P.batch * (in_share * ((double)P.M * P.K + (same ? 0.0 : (double)P.N * P.K)) +
                           (double)P.M * P.N * (out_share * (P.C != nullptr) +
                                                r_share * (P.R != nullptr && P.R != P.A && P.R != P.B))) +
          (P.sign_out ? (double)P.batch * P.sign_stride : 0.0);
    }
  }
  {
    sm_launch_scope sc(ctx, klass);
    if (args.in_f16 && (args.sym_store & 1) && ts == 256)
      hipLaunchKernelGGL((sm_ns_gemm_kernel<3, 256>), grid, block, 0, ctx->stream, args);
    else if (args.in_f16 && (args.sym_store & 1))
      hipLaunchKernelGGL((sm_ns_gemm_kernel<3, 128>), grid, block, 0, ctx->stream, args);
    else if (args.in_f16 && ts == 256)
      hipLaunchKernelGGL((sm_ns_gemm_kernel<2, 256>), grid, block, 0, ctx->stream, args);
    else if (args.in_f16)
      hipLaunchKernelGGL((sm_ns_gemm_kernel<2, 128>), grid, block, 0, ctx->stream, args);
    else if (gram && ts == 256)
      hipLaunchKernelGGL((sm_ns_gemm_kernel<0, 256>), grid, block, 0, ctx->stream, args);
    else if (gram)
      hipLaunchKernelGGL((sm_ns_gemm_kernel<0, 128>), grid, block, 0, ctx->stream, args);
    else if (ts == 256)
      hipLaunchKernelGGL((sm_ns_gemm_kernel<1, 256>), grid, block, 0, ctx->stream, args);
    else
      hipLaunchKernelGGL((sm_ns_gemm_kernel<1, 128>), grid, block, 0, ctx->stream, args);
  }
  SM_HIP(ctx, hipGetLastError());
  return SM_OK;
}
