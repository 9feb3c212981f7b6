// Newton-Schulz GEMMs of Alg. PolarNS on the gfx950 matrix cores.
//
// One grouped launch computes, for every problem in a table and every batch
// item,   C = alpha * scale^pow * (A * B^T) + gamma * R + diag * I
// with A [M][K] and B [N][K] both K-contiguous bf16, fp32 accumulation in
// v_mfma_f32_32x32x16_bf16.  The Gram step of the iteration (A = B = Y, output
// a I + b Y Y^T) and the polynomial apply step are both of this form.
//
// Tiling: a workgroup of 4 waves owns a BM x BN tile of C; K is walked in
// slices of 64.  Slices are staged in LDS (double buffered) as rows of 128
// bytes = 8 chunks of 16 bytes; chunk c of row r sits at chunk position
// c ^ ((r >> 1) & 7), which makes the 16 rows that one ds_read_b128 phase
// touches fall in distinct banks.  Each wave owns a WM x WN sub-tile as
// (WM/32) x (WN/32) MFMA tiles.  The MFMA is issued with the B fragment as the
// first operand, so a lane ends up holding one row m and 4 consecutive columns
// n of C: the epilogue writes those 8-byte groups to LDS and the tile leaves
// with 16-byte coalesced row stores.
//
// Workgroup ids are dealt round-robin to the 8 XCDs by the hardware; the kernel
// renumbers them so that each XCD walks one contiguous eighth of the tile list
// and neighbouring tiles (sharing operand panels) hit the same L2.
#include "common.h"

namespace {

constexpr int BK = 64;
constexpr int NTHREADS = 256;

__device__ __forceinline__ int swz(int row, int chunk) { return chunk ^ ((row >> 1) & 7); }

template <int BM, int BN, int WM, int WN, int KIND>
__global__ void __launch_bounds__(NTHREADS) sm_ns_gemm_nt_kernel(const sm_gemm_args args) {
  constexpr int WGM = BM / WM;            // waves along m
  constexpr int FM = WM / 32, FN = WN / 32;
  constexpr int LA = BM / 32, LB = BN / 32;  // 16-byte chunks per thread per slice
  static_assert((BM / WM) * (BN / WN) == 4, "4 waves");
  constexpr int CS = BN + 4;              // epilogue row stride in elements (BN*2 + 8 bytes)

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16_t* As = reinterpret_cast<bf16_t*>(smem);                  // [2][BM][64]
  bf16_t* Bs = As + 2 * BM * BK;                                 // [2][BN][64]

  // ---- which tile
  const int wg = blockIdx.x;
  const int L = (wg & 7) * args.tiles_per_xcd + (wg >> 3);
  if (L >= args.total_tiles) return;
  int pi = 0;
  while (pi + 1 < args.n_prob && L >= args.p[pi + 1].tile_begin) ++pi;
  const sm_gemm_prob& P = args.p[pi];
  int t = L - P.tile_begin;
  const int per_batch = P.tiles_m * P.tiles_n;
  const int b = t / per_batch;
  t -= b * per_batch;
  const int tn = t / P.tiles_m, tm = t - tn * P.tiles_m;
  const int m0 = tm * BM, n0 = tn * BN;
  const int M = P.M, N = P.N, K = P.K;
  const bf16_t* __restrict__ A = P.A + (long long)b * P.sA;
  const bf16_t* __restrict__ B = P.B + (long long)b * P.sB;

  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int w_m = wv % WGM, w_n = wv / WGM;

  // ---- global -> register staging: thread covers chunk lp of rows lr + 32 j
  const int lp = tid & 7, lr = tid >> 3;
  const bf16_t* ga[LA];
  const bf16_t* gb[LB];
#pragma unroll
  for (int j = 0; j < LA; ++j) ga[j] = A + (long long)min(m0 + lr + 32 * j, M - 1) * P.lda + lp * 8;
#pragma unroll
  for (int j = 0; j < LB; ++j) gb[j] = B + (long long)min(n0 + lr + 32 * j, N - 1) * P.ldb + lp * 8;
  u32x4 ra[LA], rb[LB];
  auto load_slice = [&](int k0) {
#pragma unroll
    for (int j = 0; j < LA; ++j) ra[j] = *reinterpret_cast<const u32x4*>(ga[j] + k0);
#pragma unroll
    for (int j = 0; j < LB; ++j) rb[j] = *reinterpret_cast<const u32x4*>(gb[j] + k0);
  };
  auto store_slice = [&](int buf) {
#pragma unroll
    for (int j = 0; j < LA; ++j) {
      const int r = lr + 32 * j;
      *reinterpret_cast<u32x4*>(As + buf * BM * BK + r * BK + swz(r, lp) * 8) = ra[j];
    }
#pragma unroll
    for (int j = 0; j < LB; ++j) {
      const int r = lr + 32 * j;
      *reinterpret_cast<u32x4*>(Bs + buf * BN * BK + r * BK + swz(r, lp) * 8) = rb[j];
    }
  };

  f32x16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const int fr = lane & 31, fg = lane >> 5;
  const int nk = K / BK;
  load_slice(0);
  store_slice(0);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < nk) load_slice((kt + 1) * BK);
    const bf16_t* as = As + buf * BM * BK;
    const bf16_t* bs = Bs + buf * BN * BK;
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 fa[FM], fb[FN];
#pragma unroll
      for (int i = 0; i < FM; ++i) {
        const int r = w_m * WM + i * 32 + fr;
        fa[i] = *reinterpret_cast<const bf16x8*>(as + r * BK + swz(r, 2 * ks + fg) * 8);
      }
#pragma unroll
      for (int j = 0; j < FN; ++j) {
        const int r = w_n * WN + j * 32 + fr;
        fb[j] = *reinterpret_cast<const bf16x8*>(bs + r * BK + swz(r, 2 * ks + fg) * 8);
      }
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) store_slice(buf ^ 1);
    __syncthreads();
  }

  // ---- epilogue: scale, add diag / R, round to bf16, stage in LDS, coalesced stores
  float s = 1.f;
  if (P.scale && args.scale_pow) {
    s = P.scale[b];
    if (args.scale_pow == 2) s *= s;
  }
  const float alpha = args.alpha * s;
  const bf16_t* __restrict__ R = P.R ? P.R + (long long)b * P.sC : nullptr;
  bf16_t* Cs = reinterpret_cast<bf16_t*>(smem);  // [BM][CS]; the K loop ended with a barrier
#pragma unroll
  for (int i = 0; i < FM; ++i) {
    const int ml = w_m * WM + i * 32 + fr;
    const int mg = m0 + ml;
#pragma unroll
    for (int j = 0; j < FN; ++j) {
#pragma unroll
      for (int vg = 0; vg < 4; ++vg) {
        const int nl = w_n * WN + j * 32 + 8 * vg + 4 * fg;
        const int ng = n0 + nl;
        float o[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          o[e] = alpha * acc[i][j][4 * vg + e];
          if (mg == ng + e) o[e] += args.diag;
        }
        if (R && mg < M && ng < N) {
          const bf16x4 rv = *reinterpret_cast<const bf16x4*>(R + (long long)mg * P.ldc + ng);
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] += args.gamma * (float)rv[e];
        }
        const bf16x4 h = {(bf16_t)o[0], (bf16_t)o[1], (bf16_t)o[2], (bf16_t)o[3]};
        *reinterpret_cast<bf16x4*>(Cs + ml * CS + nl) = h;
      }
    }
  }
  __syncthreads();
  bf16_t* __restrict__ C = P.C + (long long)b * P.sC;
  constexpr int CPR = BN / 8;  // 16-byte chunks per tile row
#pragma unroll
  for (int it = 0; it < BM * CPR / NTHREADS; ++it) {
    const int q = it * NTHREADS + tid;
    const int r = q / CPR, cc = q % CPR;
    const int mg = m0 + r, ng = n0 + cc * 8;
    if (mg < M && ng < N) {
      const bf16x4 lo = *reinterpret_cast<const bf16x4*>(Cs + r * CS + cc * 8);
      const bf16x4 hi = *reinterpret_cast<const bf16x4*>(Cs + r * CS + cc * 8 + 4);
      bf16x8 v;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        v[e] = lo[e];
        v[e + 4] = hi[e];
      }
      *reinterpret_cast<bf16x8*>(C + (long long)mg * P.ldc + ng) = v;
    }
  }
}

template <int BM, int BN>
constexpr size_t gemm_lds_bytes() {
  const size_t loop = 2ull * (BM + BN) * BK * 2;
  const size_t epi = (size_t)BM * (BN + 4) * 2;
  return loop > epi ? loop : epi;
}

template <int BM, int BN, int WM, int WN, int KIND>
int launch_cfg(signmuon_ctx* ctx, sm_gemm_args& args, int klass) {
  int total = 0;
  for (int i = 0; i < args.n_prob; ++i) {
    sm_gemm_prob& P = args.p[i];
    P.tiles_m = (P.M + BM - 1) / BM;
    P.tiles_n = (P.N + BN - 1) / BN;
    P.tile_begin = total;
    total += P.tiles_m * P.tiles_n * P.batch;
  }
  args.total_tiles = total;
  args.tiles_per_xcd = (total + 7) / 8;
  if (total == 0) return SM_OK;
  auto kern = sm_ns_gemm_nt_kernel<BM, BN, WM, WN, KIND>;
  constexpr size_t lds = gemm_lds_bytes<BM, BN>();
  static bool attr_done = false;
  if (!attr_done) {
    SM_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)lds));
    attr_done = true;
  }
  {
    sm_launch_scope sc(ctx, klass);
    hipLaunchKernelGGL(kern, dim3(args.tiles_per_xcd * 8), dim3(NTHREADS), lds, ctx->stream, args);
  }
  SM_HIP(ctx, hipGetLastError());
  return SM_OK;
}

}  // namespace

int sm_gemm_tile_override = 0;  // 0: automatic; 128 or 256 forces a tile size (tuning aid)

int sm_launch_gemm_nt(signmuon_ctx* ctx, sm_gemm_args& args, int klass) {
  for (int i = 0; i < args.n_prob; ++i) {
    const sm_gemm_prob& P = args.p[i];
    if (P.M % 64 || P.N % 64 || P.K % 64 || P.lda % 8 || P.ldb % 8 || P.ldc % 8 || !sm_aligned(P.A, 16) ||
        !sm_aligned(P.B, 16) || !sm_aligned(P.C, 16) || P.sA % 8 || P.sB % 8 || P.sC % 8)
      return sm_fail(ctx, SM_EINVAL, "internal: GEMM operand not padded/aligned");
  }
  static const int env_tile = [] {
    const char* e = getenv("SIGNMUON_GEMM_TILE");
    return e ? atoi(e) : 0;
  }();
  int tile = sm_gemm_tile_override ? sm_gemm_tile_override : env_tile;
  if (tile == 0) {
    // large tiles once there is enough work to fill 256 CUs with them
    long long t256 = 0;
    for (int i = 0; i < args.n_prob; ++i) {
      const sm_gemm_prob& P = args.p[i];
      t256 += (long long)((P.M + 255) / 256) * ((P.N + 255) / 256) * P.batch;
    }
    tile = (t256 >= 512) ? 256 : 128;
  }
  const bool gram = (klass == SM_K_NS_GRAM);
  if (tile == 256) {
    return gram ? launch_cfg<256, 256, 128, 128, 0>(ctx, args, klass) : launch_cfg<256, 256, 128, 128, 1>(ctx, args, klass);
  }
  return gram ? launch_cfg<128, 128, 64, 64, 0>(ctx, args, klass) : launch_cfg<128, 128, 64, 64, 1>(ctx, args, klass);
}
