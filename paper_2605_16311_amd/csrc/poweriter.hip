// Alg. PowerIter (spectral-norm estimate for the spectral scale of PolarNS):
//   v <- v0 / (|v0| + eps);  P times { u = X v, u /= |u| + eps;  v = X^T u, v /= |v| + eps };
//   sigma = |X v|.
// X is the bf16 working copy [rows][ld]; vectors and sums are fp32.  Every
// reduction runs in a fixed order (no atomics), so sigma is reproducible.
#include "common.h"

namespace {

constexpr int TPB = 256;

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
  return v;
}

// u[b][i] = sum_j X[b][i][j] * v[b][j]; one wave per row.
__global__ void __launch_bounds__(TPB) sm_pi_xv_kernel(const bf16_t* __restrict__ x, int rows, int cols, int ld,
                                                       long long stride, const float* __restrict__ v,
                                                       long long vstride, float* __restrict__ u, long long ustride) {
  const int b = blockIdx.y;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const int lane = threadIdx.x & 63;
  const bf16_t* xr = x + (long long)b * stride + (long long)row * ld;
  const float* vb = v + (long long)b * vstride;
  float s = 0.f;
  for (int j = lane; j < cols; j += 64) s += (float)xr[j] * vb[j];
  s = wave_sum(s);
  if (lane == 0) u[(long long)b * ustride + row] = s;
}

// v[b][j] = sum_i X[b][i][j] * u[b][i]; one thread per column.
__global__ void __launch_bounds__(TPB) sm_pi_xtu_kernel(const bf16_t* __restrict__ x, int rows, int cols, int ld,
                                                        long long stride, const float* __restrict__ u,
                                                        long long ustride, float* __restrict__ v, long long vstride) {
  const int b = blockIdx.y;
  const int j = blockIdx.x * TPB + threadIdx.x;
  if (j >= cols) return;
  const bf16_t* xb = x + (long long)b * stride + j;
  const float* ub = u + (long long)b * ustride;
  float s = 0.f;
  for (int i = 0; i < rows; ++i) s += (float)xb[(long long)i * ld] * ub[i];
  v[(long long)b * vstride + j] = s;
}

// dst[b] = src[b] / (|src[b]| + eps) when dst != null; norm_out[b] = |src[b]| when non-null.
__global__ void __launch_bounds__(TPB) sm_pi_normalize_kernel(const float* src, long long sstride, int n,
                                                              float eps, float* dst, long long dstride,
                                                              float* __restrict__ norm_out) {
  __shared__ float red[4];
  __shared__ float nrm;
  const int b = blockIdx.x;
  const float* s = src + (long long)b * sstride;
  float ss = 0.f;
  for (int i = threadIdx.x; i < n; i += TPB) ss += s[i] * s[i];
  ss = wave_sum(ss);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  if (threadIdx.x == 0) {
    nrm = sqrtf((red[0] + red[1]) + (red[2] + red[3]));
    if (norm_out) norm_out[b] = nrm;
  }
  __syncthreads();
  if (dst) {
    const float inv = 1.0f / (nrm + eps);
    float* d = dst + (long long)b * dstride;
    for (int i = threadIdx.x; i < n; i += TPB) d[i] = s[i] * inv;
  }
}

}  // namespace

int sm_launch_power_iter(signmuon_ctx* ctx, const bf16_t* x, int rows, int cols, int ld, long long stride, int batch,
                         int P, float eps, const float* v0, long long v0_stride, float* scratch, float* sigma) {
  // scratch per batch item: u[rows], v[cols]
  const long long per = (long long)rows + cols;
  float* u = scratch;
  float* v = scratch + rows;
  sm_launch_scope sc(ctx, SM_K_OTHER);
  auto normalize = [&](const float* s, long long ss, int n, float* d, long long ds, float* nout) {
    hipLaunchKernelGGL(sm_pi_normalize_kernel, dim3(batch), dim3(TPB), 0, ctx->stream, s, ss, n, eps, d, ds, nout);
  };
  auto xv = [&]() {
    hipLaunchKernelGGL(sm_pi_xv_kernel, dim3((rows + 3) / 4, batch), dim3(TPB), 0, ctx->stream, x, rows, cols, ld,
                       stride, v, per, u, per);
  };
  auto xtu = [&]() {
    hipLaunchKernelGGL(sm_pi_xtu_kernel, dim3((cols + TPB - 1) / TPB, batch), dim3(TPB), 0, ctx->stream, x, rows, cols,
                       ld, stride, u, per, v, per);
  };
  normalize(v0, v0_stride, cols, v, per, nullptr);
  for (int p = 0; p < P; ++p) {
    xv();
    normalize(u, per, rows, u, per, nullptr);
    xtu();
    normalize(v, per, cols, v, per, nullptr);
  }
  xv();
  normalize(u, per, rows, nullptr, 0, sigma);
  SM_HIP(ctx, hipGetLastError());
  return SM_OK;
}
