// Alg. PowerIter (spectral-norm estimate for the spectral scale of PolarNS):
//   v <- v0 / (|v0| + eps);  P times { u = X v, u /= |u| + eps;  v = X^T u, v /= |v| + eps };
//   sigma = |X v|.
// Grouped over a table of weight blocks, M matrices each: every pass over the X of ALL blocks and
// workers is one launch (two per table when the set has more blocks than a table holds).
// Matrices of up to SM_PI_FUSED_MAX_LD padded columns take the fused form: one pass over X yields both
// u = X v and w = X^T u, because row i's share of w, u_i X_i, needs only that row's own product u_i:
// a wave holds a row in registers, reduces u_i over its lanes and adds u_i X_i into per-lane sums.
// The two normalisations of a round are scalars, so they are applied afterwards
// (v' = (w / cu) / (|w / cu| + eps), cu = |u| + eps): P rounds and the final |X v| read X P + 1
// times instead of 2 P + 1.
// X is the bf16 working copy [rows][ld] with zero padding up to ld (a multiple of 64); vectors
// and sums are fp32, u padded to a multiple of 8 and v to ld with zeros.  Every reduction runs
// in a fixed order (no atomics), so sigma is reproducible.
#include "common.h"

#include <algorithm>

namespace {

constexpr int TPB = 256;

struct pi_args {
  int n;
  float eps;
  sm_pi_desc d[SM_PI_MAX_GROUP];
};

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
  return v;
}

__device__ __forceinline__ const sm_pi_desc& find_desc(const pi_args& a, int bx, int& local) {
  int di = 0;
  while (di + 1 < a.n && bx >= a.d[di + 1].block_begin) ++di;
  local = bx - a.d[di].block_begin;
  return a.d[di];
}

// 8 bf16 (one 16-byte load) times 8 floats
__device__ __forceinline__ float dot8(const u32x4 x, const float* __restrict__ v) {
  const f32x4 a = *reinterpret_cast<const f32x4*>(v), b = *reinterpret_cast<const f32x4*>(v + 4);
  float s = 0.f;
  s += __uint_as_float(x[0] << 16) * a[0];
  s += __uint_as_float(x[0] & 0xFFFF0000u) * a[1];
  s += __uint_as_float(x[1] << 16) * a[2];
  s += __uint_as_float(x[1] & 0xFFFF0000u) * a[3];
  s += __uint_as_float(x[2] << 16) * b[0];
  s += __uint_as_float(x[2] & 0xFFFF0000u) * b[1];
  s += __uint_as_float(x[3] << 16) * b[2];
  s += __uint_as_float(x[3] & 0xFFFF0000u) * b[3];
  return s;
}

// u[item][row] = sum_j X[item][row][j] v[item][j]: one wave per row, 16-byte loads, 4 rows per workgroup.
__global__ void __launch_bounds__(TPB) sm_pi_xv_kernel(const pi_args a) {
  int local;
  const sm_pi_desc& D = find_desc(a, blockIdx.x, local);
  const int rgroups = (D.rows + 3) / 4;
  const int item = local / rgroups;
  const int row = (local - item * rgroups) * 4 + (threadIdx.x >> 6);
  if (row >= D.rows) return;
  const int lane = threadIdx.x & 63;
  const bf16_t* xr = D.x + (long long)item * D.stride + (long long)row * D.ld;
  const float* v = D.v + (long long)item * D.ld;
  float s = 0.f;
  for (int j = lane * 8; j < D.ld; j += 512) s += dot8(__builtin_nontemporal_load(reinterpret_cast<const u32x4*>(xr + j)), v + j);
  s = wave_sum(s);
  if (lane == 0) D.u[(long long)item * D.up + row] = s;
}

// part[item][chunk][j] = sum over the chunk's rows of X[item][i][j] u[item][i]: a workgroup owns a strip of
// 512 columns and a chunk of SM_PI_ROW_CHUNK rows of one matrix; wave w takes rows w, w + 4, ... of the
// chunk, a lane 8 columns; the four partial strips are added in wave order.  The chunks are added (in
// order) by the normalisation that follows.
__global__ void __launch_bounds__(TPB) sm_pi_xtu_kernel(const pi_args a) {
  __shared__ float part[3][512];
  int local;
  const sm_pi_desc& D = find_desc(a, blockIdx.x, local);
  const int strips = (D.ld + 511) / 512;
  const int per_item = strips * D.chunks;
  const int item = local / per_item;
  const int rem = local - item * per_item;
  const int chunk = rem / strips;
  const int j0 = (rem - chunk * strips) * 512 + (threadIdx.x & 63) * 8;
  const int wv = threadIdx.x >> 6;
  const int r0 = chunk * SM_PI_ROW_CHUNK, r1 = min(D.rows, r0 + SM_PI_ROW_CHUNK);
  const bf16_t* xb = D.x + (long long)item * D.stride + j0;
  const float* u = D.u + (long long)item * D.up;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (j0 < D.ld) {
#pragma unroll 4
    for (int i = r0 + wv; i < r1; i += 4) {
      const u32x4 x = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(xb + (long long)i * D.ld));
      const float ui = u[i];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        acc[2 * q] += __uint_as_float(x[q] << 16) * ui;
        acc[2 * q + 1] += __uint_as_float(x[q] & 0xFFFF0000u) * ui;
      }
    }
  }
  const int c = (threadIdx.x & 63) * 8;
  if (wv > 0) {
#pragma unroll
    for (int k = 0; k < 8; ++k) part[wv - 1][c + k] = acc[k];
  }
  __syncthreads();
  if (wv == 0 && j0 < D.ld) {
    float* o = D.part + ((long long)item * D.chunks + chunk) * D.ld + j0;
#pragma unroll
    for (int k = 0; k < 8; ++k) o[k] = ((acc[k] + part[0][c + k]) + part[1][c + k]) + part[2][c + k];
  }
}

// Fused pass: u[item][row] = <X_row, v> for the rows of a chunk of SM_PI_FUSED_ROWS rows and, with AXPY,
// part[item][chunk][j] = sum over those rows of u_row X[row][j].  A workgroup owns one chunk of one matrix;
// wave w takes rows w, w + 4, ... of it, two at a time (both rows' loads are issued before either is
// used); a lane owns columns 512 t + 8 lane .. + 7 of strip t < NS and keeps its part of v and of the sums
// in registers.  The four waves' sums are added in wave order.
template <int NS, bool AXPY>
__global__ void __launch_bounds__(TPB) sm_pi_fused_kernel(const pi_args a) {
  __shared__ float part[AXPY ? 3 : 1][AXPY ? NS * 512 : 1];
  int local;
  const sm_pi_desc& D = find_desc(a, blockIdx.x, local);
  const int chunks = (D.rows + SM_PI_FUSED_ROWS - 1) / SM_PI_FUSED_ROWS;
  const int item = local / chunks, chunk = local - item * chunks;
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int r0 = chunk * SM_PI_FUSED_ROWS, r1 = min(D.rows, r0 + SM_PI_FUSED_ROWS);
  const bf16_t* xb = D.x + (long long)item * D.stride;
  const float* v = D.v + (long long)item * D.ld;
  float* u = D.u + (long long)item * D.up;
  float vr[NS][8], acc[NS][8];
#pragma unroll
  for (int t = 0; t < NS; ++t) {
    const int j = 512 * t + 8 * lane;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      vr[t][k] = (j < D.ld) ? v[j + k] : 0.f;
      acc[t][k] = 0.f;
    }
  }
  for (int i = r0 + wv; i < r1; i += 8) {
    const int i2 = i + 4;
    u32x4 x0[NS], x1[NS];
#pragma unroll
    for (int t = 0; t < NS; ++t) {
      const int j = 512 * t + 8 * lane;
      x0[t] = x1[t] = u32x4{0u, 0u, 0u, 0u};
      if (j < D.ld) {
        x0[t] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(xb + (long long)i * D.ld + j));
        if (i2 < r1) x1[t] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(xb + (long long)i2 * D.ld + j));
      }
    }
    float s0 = 0.f, s1 = 0.f;
#pragma unroll
    for (int t = 0; t < NS; ++t)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        s0 += __uint_as_float(x0[t][q] << 16) * vr[t][2 * q] + __uint_as_float(x0[t][q] & 0xFFFF0000u) * vr[t][2 * q + 1];
        s1 += __uint_as_float(x1[t][q] << 16) * vr[t][2 * q] + __uint_as_float(x1[t][q] & 0xFFFF0000u) * vr[t][2 * q + 1];
      }
    // every lane gets the row's product (butterfly: the same value in all lanes)
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
      s0 += __shfl_xor(s0, off, 64);
      s1 += __shfl_xor(s1, off, 64);
    }
    if (lane == 0) {
      u[i] = s0;
      if (i2 < r1) u[i2] = s1;
    }
    if (AXPY) {
#pragma unroll
      for (int t = 0; t < NS; ++t)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          acc[t][2 * q] += __uint_as_float(x0[t][q] << 16) * s0;
          acc[t][2 * q + 1] += __uint_as_float(x0[t][q] & 0xFFFF0000u) * s0;
          acc[t][2 * q] += __uint_as_float(x1[t][q] << 16) * s1;
          acc[t][2 * q + 1] += __uint_as_float(x1[t][q] & 0xFFFF0000u) * s1;
        }
    }
  }
  if (AXPY) {
    if (wv > 0) {
#pragma unroll
      for (int t = 0; t < NS; ++t)
#pragma unroll
        for (int k = 0; k < 8; ++k) part[wv - 1][512 * t + 8 * lane + k] = acc[t][k];
    }
    __syncthreads();
    if (wv == 0) {
      float* o = D.part + ((long long)item * chunks + chunk) * D.ld;
#pragma unroll
      for (int t = 0; t < NS; ++t) {
        const int j = 512 * t + 8 * lane;
        if (j < D.ld) {
#pragma unroll
          for (int k = 0; k < 8; ++k) o[j + k] = ((acc[t][k] + part[0][j + k]) + part[1][j + k]) + part[2][j + k];
        }
      }
    }
  }
}

// Sum over the row chunks' partial sums of one column, in chunk order, the loads of eight chunks issued
// before the first is added.
__device__ __forceinline__ float chunk_sum(const float* __restrict__ pp, int chunks, long long ld) {
  float t = 0.f;
  int ch = 0;
  for (; ch + 8 <= chunks; ch += 8) {
    float x[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) x[k] = pp[(ch + k) * ld];
#pragma unroll
    for (int k = 0; k < 8; ++k) t += x[k];
  }
  for (; ch < chunks; ++ch) t += pp[ch * ld];
  return t;
}

// One workgroup of TPN threads per matrix.  which = 0: v <- v0 / (|v0| + eps), zero-padded to ld.
// which = 1: u <- u / (|u| + eps).  which = 2: v <- s / (|s| + eps) with s the sum of the row chunks'
// partial X^T u.  which = 3: sigma = |u|.  which = 4 (after a fused pass, u and the partial sums not yet
// normalised): cu = |u| + eps, s = (sum of the chunks' partial X^T u) / cu, v <- s / (|s| + eps).
constexpr int TPN = 1024;
__global__ void __launch_bounds__(TPN) sm_pi_normalize_kernel(const pi_args a, int which) {
  __shared__ float red[TPN / 64];
  __shared__ float nrm;
  int local;
  const sm_pi_desc& D = find_desc(a, blockIdx.x, local);
  const int item = local;
  // sqrt of the workgroup's sum, the waves' sums added in wave order
  auto block_norm = [&](float ss) {
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    if (threadIdx.x == 0) {
      float t = 0.f;
      for (int w = 0; w < TPN / 64; ++w) t += red[w];
      nrm = sqrtf(t);
    }
    __syncthreads();
    const float r = nrm;
    __syncthreads();  // red and nrm may be written again
    return r;
  };
  const float* src;
  float* dst;
  int n, n_out;
  if (which == 4) {
    const float* uu = D.u + (long long)item * D.up;
    float su = 0.f;
    for (int i = threadIdx.x; i < D.rows; i += TPN) su += uu[i] * uu[i];
    const float inv_cu = 1.0f / (block_norm(su) + a.eps);
    const int chunks = (D.rows + SM_PI_FUSED_ROWS - 1) / SM_PI_FUSED_ROWS;
    dst = D.v + (long long)item * D.ld;
    const float* pp = D.part + (long long)item * chunks * D.ld;
    for (int i = threadIdx.x; i < D.cols; i += TPN) dst[i] = chunk_sum(pp + i, chunks, D.ld) * inv_cu;
    __syncthreads();
    src = dst;
    n = n_out = D.cols;
  } else if (which == 0) {
    src = D.v0 + (long long)item * D.v0_stride;
    dst = D.v + (long long)item * D.ld;
    n = D.cols;
    n_out = D.ld;
  } else if (which == 2) {
    dst = D.v + (long long)item * D.ld;
    const float* pp = D.part + (long long)item * D.chunks * D.ld;
    for (int i = threadIdx.x; i < D.cols; i += TPN) dst[i] = chunk_sum(pp + i, D.chunks, D.ld);
    __syncthreads();
    src = dst;
    n = n_out = D.cols;
  } else {
    src = dst = D.u + (long long)item * D.up;
    n = n_out = D.rows;
  }
  float ss = 0.f;
  for (int i = threadIdx.x; i < n; i += TPN) ss += src[i] * src[i];
  const float nr = block_norm(ss);
  if (which == 3) {
    if (threadIdx.x == 0) D.sigma[item] = nr;
    return;
  }
  const float inv = 1.0f / (nr + a.eps);
  for (int i = threadIdx.x; i < n_out; i += TPN) dst[i] = (i < n) ? src[i] * inv : 0.f;
}

}  // namespace

// strips of 512 columns the fused kernel is instantiated for (narrow matrices share the 3-strip kernel: a
// strip beyond the matrix issues no loads)
static int fused_strips(int ld) {
  const int need = (ld + 511) / 512;
  for (int ns : {3, 4, 6, 8})
    if (need <= ns) return ns;
  return 0;
}

template <bool AXPY>
static void launch_fused(int ns, unsigned blocks, hipStream_t st, const pi_args& a) {
  switch (ns) {
    case 3: hipLaunchKernelGGL((sm_pi_fused_kernel<3, AXPY>), dim3(blocks), dim3(TPB), 0, st, a); break;
    case 4: hipLaunchKernelGGL((sm_pi_fused_kernel<4, AXPY>), dim3(blocks), dim3(TPB), 0, st, a); break;
    case 6: hipLaunchKernelGGL((sm_pi_fused_kernel<6, AXPY>), dim3(blocks), dim3(TPB), 0, st, a); break;
    default: hipLaunchKernelGGL((sm_pi_fused_kernel<8, AXPY>), dim3(blocks), dim3(TPB), 0, st, a); break;
  }
}

// Fused form over a table whose matrices all take the same number of column strips `ns`.
static int power_iter_fused(signmuon_ctx* ctx, const sm_pi_desc* descs, int n, int P, float eps, int ns) {
  int done = 0;
  while (done < n) {
    const int g = std::min(n - done, SM_PI_MAX_GROUP);
    pi_args a_pass, a_nrm;
    long long b_pass = 0, b_nrm = 0;
    for (pi_args* a : {&a_pass, &a_nrm}) {
      a->n = g;
      a->eps = eps;
    }
    for (int i = 0; i < g; ++i) {
      const sm_pi_desc& d = descs[done + i];
      if (d.ld % 64 || d.up % 8 || d.up < d.rows || !sm_aligned(d.x, 16) || d.stride % 8 || !sm_aligned(d.v, 16))
        return sm_fail(ctx, SM_EINVAL, "internal: power iteration operands not padded/aligned");
      a_pass.d[i] = a_nrm.d[i] = d;
      a_pass.d[i].block_begin = (int)b_pass;
      a_nrm.d[i].block_begin = (int)b_nrm;
      b_pass += (long long)((d.rows + SM_PI_FUSED_ROWS - 1) / SM_PI_FUSED_ROWS) * d.items;
      b_nrm += d.items;
    }
    if (b_pass > 0x7FFFFFFFLL) return sm_fail(ctx, SM_EUNSUPPORTED, "power iteration: too many rows for one launch");
    if (b_nrm > 0) {
      sm_launch_scope sc(ctx, SM_K_POWER_ITER);
      auto normalize = [&](int which) {
        hipLaunchKernelGGL(sm_pi_normalize_kernel, dim3((unsigned)b_nrm), dim3(TPN), 0, ctx->stream, a_nrm, which);
      };
      normalize(0);
      for (int p = 0; p < P; ++p) {
        launch_fused<true>(ns, (unsigned)b_pass, ctx->stream, a_pass);
        normalize(4);
      }
      launch_fused<false>(ns, (unsigned)b_pass, ctx->stream, a_pass);
      normalize(3);
    }
    SM_HIP(ctx, hipGetLastError());
    done += g;
  }
  return SM_OK;
}

int sm_launch_power_iter_group(signmuon_ctx* ctx, const sm_pi_desc* descs, int n, int P, float eps) {
  // the fused form serves the matrices that fit its register budget; wider ones take a pass per product
  // One set of launches per strip count in use, so that narrow matrices do not run the wide kernel.  The
  // fused form saves two of five passes over X and costs more launches (7 per strip count in use instead
  // of 10 in all): it is taken when the bytes saved outweigh them at about 10 us a launch.
  std::vector<sm_pi_desc> wide;
  double bytes = 0.0;
  int buckets = 0;
  bool any_wide = false;
  for (int ns : {3, 4, 6, 8}) {
    bool used = false;
    for (int i = 0; i < n; ++i)
      if (descs[i].ld <= SM_PI_FUSED_MAX_LD && fused_strips(descs[i].ld) == ns) {
        used = true;
        bytes += 2.0 * descs[i].rows * descs[i].ld * descs[i].items;
      }
    buckets += used;
  }
  for (int i = 0; i < n; ++i) any_wide = any_wide || descs[i].ld > SM_PI_FUSED_MAX_LD;
  const double saved_us = 2.0 * bytes / 5e6;  // two passes at about 5 TB/s
  const double extra_us = 10.0 * (7.0 * buckets + (any_wide ? 10.0 : 0.0) - 10.0);
  const int mode = ctx->opt[SM_OPT_POWER_ITER];
  const bool fuse = P > 0 && buckets > 0 && mode != SM_PI_SEPARATE && (mode == SM_PI_FUSED || saved_us > extra_us);
  if (fuse) {
    for (int ns : {3, 4, 6, 8}) {
      std::vector<sm_pi_desc> bucket;
      for (int i = 0; i < n; ++i)
        if (descs[i].ld <= SM_PI_FUSED_MAX_LD && fused_strips(descs[i].ld) == ns) bucket.push_back(descs[i]);
      if (bucket.empty()) continue;
      const int rc = power_iter_fused(ctx, bucket.data(), (int)bucket.size(), P, eps, ns);
      if (rc != SM_OK) return rc;
    }
  }
  for (int i = 0; i < n; ++i)
    if (!fuse || descs[i].ld > SM_PI_FUSED_MAX_LD) wide.push_back(descs[i]);
  if (wide.empty()) return SM_OK;
  descs = wide.data();
  n = (int)wide.size();
  int done = 0;
  while (done < n) {
    const int g = std::min(n - done, SM_PI_MAX_GROUP);
    pi_args a_xv, a_xtu, a_nrm;
    long long b_xv = 0, b_xtu = 0, b_nrm = 0;
    for (pi_args* a : {&a_xv, &a_xtu, &a_nrm}) {
      a->n = g;
      a->eps = eps;
    }
    for (int i = 0; i < g; ++i) {
      const sm_pi_desc& d = descs[done + i];
      if (d.chunks != (d.rows + SM_PI_ROW_CHUNK - 1) / SM_PI_ROW_CHUNK) return sm_fail(ctx, SM_EINVAL, "internal: power iteration chunk count");
      if (d.ld % 64 || d.up % 8 || d.up < d.rows || !sm_aligned(d.x, 16) || d.stride % 8 || !sm_aligned(d.v, 16))
        return sm_fail(ctx, SM_EINVAL, "internal: power iteration operands not padded/aligned");
      a_xv.d[i] = a_xtu.d[i] = a_nrm.d[i] = d;
      a_xv.d[i].block_begin = (int)b_xv;
      a_xtu.d[i].block_begin = (int)b_xtu;
      a_nrm.d[i].block_begin = (int)b_nrm;
      b_xv += (long long)((d.rows + 3) / 4) * d.items;
      b_xtu += (long long)((d.ld + 511) / 512) * d.chunks * d.items;
      b_nrm += d.items;
    }
    if (b_xv > 0x7FFFFFFFLL || b_xtu > 0x7FFFFFFFLL)
      return sm_fail(ctx, SM_EUNSUPPORTED, "power iteration: too many rows for one launch");
    if (b_nrm > 0) {
      sm_launch_scope sc(ctx, SM_K_POWER_ITER);
      auto normalize = [&](int which) {
        hipLaunchKernelGGL(sm_pi_normalize_kernel, dim3((unsigned)b_nrm), dim3(TPN), 0, ctx->stream, a_nrm, which);
      };
      auto xv = [&]() { hipLaunchKernelGGL(sm_pi_xv_kernel, dim3((unsigned)b_xv), dim3(TPB), 0, ctx->stream, a_xv); };
      auto xtu = [&]() { hipLaunchKernelGGL(sm_pi_xtu_kernel, dim3((unsigned)b_xtu), dim3(TPB), 0, ctx->stream, a_xtu); };
      normalize(0);
      for (int p = 0; p < P; ++p) {
        xv();
        normalize(1);
        xtu();
        normalize(2);
      }
      xv();
      normalize(3);
    }
    SM_HIP(ctx, hipGetLastError());
    done += g;
  }
  return SM_OK;
}
