// Layout helpers around the Newton-Schulz workspace: copies between caller
// matrices and the zero-padded bf16 working layout, and sums of squares for
// the Frobenius scale of Alg. PolarNS.
#include "common.h"

#include <algorithm>

namespace {

constexpr int TPB = 256;

template <int DT>
__global__ void __launch_bounds__(TPB) sm_copy_in_kernel(const void* __restrict__ src, int rows, int cols,
                                                         bf16_t* __restrict__ dst, int ld, long long dst_stride) {
  const int b = blockIdx.y;
  const long long n = (long long)rows * cols;
  const long long e = (long long)blockIdx.x * TPB + threadIdx.x;
  if (e >= n) return;
  const long long r = e / cols, c = e % cols;
  bf16_t v;
  if (DT == SM_F32)
    v = (bf16_t) reinterpret_cast<const float*>(src)[(long long)b * n + e];
  else
    v = reinterpret_cast<const bf16_t*>(src)[(long long)b * n + e];
  dst[(long long)b * dst_stride + r * ld + c] = v;
}

template <int DT>
__global__ void __launch_bounds__(TPB) sm_copy_out_kernel(const bf16_t* __restrict__ src, int ld, long long src_stride,
                                                          int rows, int cols, void* __restrict__ dst,
                                                          const float* __restrict__ scale) {
  const int b = blockIdx.y;
  const long long n = (long long)rows * cols;
  const long long e = (long long)blockIdx.x * TPB + threadIdx.x;
  if (e >= n) return;
  const long long r = e / cols, c = e % cols;
  float v = (float)src[(long long)b * src_stride + r * ld + c];
  if (scale) v *= scale[b];
  if (DT == SM_F32)
    reinterpret_cast<float*>(dst)[(long long)b * n + e] = v;
  else
    reinterpret_cast<bf16_t*>(dst)[(long long)b * n + e] = (bf16_t)v;
}

template <int DT>
__global__ void __launch_bounds__(TPB) sm_sumsq_kernel(const void* __restrict__ x, long long n, int chunks,
                                                       float* __restrict__ partial) {
  __shared__ float red[4];
  const int b = blockIdx.y, ch = blockIdx.x;
  const long long base = (long long)ch * SM_MOM_CHUNK;
  float ss = 0.f;
  for (int it = 0; it < SM_MOM_CHUNK / TPB; ++it) {
    const long long i = base + (long long)it * TPB + threadIdx.x;
    if (i >= n) break;
    float v;
    if (DT == SM_F32)
      v = reinterpret_cast<const float*>(x)[(long long)b * n + i];
    else
      v = (float) reinterpret_cast<const bf16_t*>(x)[(long long)b * n + i];
    ss += v * v;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) ss += __shfl_down(ss, off, 64);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  if (threadIdx.x == 0) partial[(long long)b * chunks + ch] = (red[0] + red[1]) + (red[2] + red[3]);
}

struct pad_args {
  int n;
  int pad_;
  sm_pad_desc d[SM_PAD_MAX_GROUP];
};

// Zero padding of the working layout: thread = one padding element of one matrix, first the strip to the
// right of the logical columns (row by row), then the rows below the logical ones.
__global__ void __launch_bounds__(TPB) sm_pad_clear_kernel(const pad_args a) {
  int di = 0;
  while (di + 1 < a.n && (int)blockIdx.x >= a.d[di + 1].block_begin) ++di;
  const sm_pad_desc& D = a.d[di];
  const int local = blockIdx.x - D.block_begin;
  const int item = local / D.blocks_per_item;
  const long long e = (long long)(local - item * D.blocks_per_item) * TPB + threadIdx.x;
  const int pc = D.cp - D.cols;
  const long long right = (long long)D.rows * pc, total = right + (long long)(D.rp - D.rows) * D.cp;
  if (e >= total) return;
  long long r, c;
  if (e < right) {
    r = e / pc;
    c = D.cols + e % pc;
  } else {
    r = D.rows + (e - right) / D.cp;
    c = (e - right) % D.cp;
  }
  D.x[(long long)item * D.stride + r * D.cp + c] = (bf16_t)0.0f;
}

}  // namespace

int sm_launch_pad_clear(signmuon_ctx* ctx, const sm_pad_desc* descs, int n) {
  int done = 0;
  while (done < n) {
    const int g = std::min(n - done, SM_PAD_MAX_GROUP);
    pad_args a;
    a.n = g;
    a.pad_ = 0;
    long long blocks = 0;
    for (int i = 0; i < g; ++i) {
      sm_pad_desc& D = a.d[i];
      D = descs[done + i];
      const long long total = (long long)D.rows * (D.cp - D.cols) + (long long)(D.rp - D.rows) * D.cp;
      D.blocks_per_item = (int)((total + TPB - 1) / TPB);
      D.block_begin = (int)blocks;
      blocks += (long long)D.blocks_per_item * D.items;
    }
    if (blocks > 0x7FFFFFFFLL) return sm_fail(ctx, SM_EUNSUPPORTED, "padding clear: too many elements for one launch");
    if (blocks > 0) {
      sm_launch_scope sc(ctx, SM_K_OTHER);
      hipLaunchKernelGGL(sm_pad_clear_kernel, dim3((unsigned)blocks), dim3(TPB), 0, ctx->stream, a);
    }
    SM_HIP(ctx, hipGetLastError());
    done += g;
  }
  return SM_OK;
}

int sm_launch_copy_in(signmuon_ctx* ctx, const void* src, int dtype, int batch, int rows, int cols, bf16_t* dst,
                      int ld, long long dst_stride) {
  const long long n = (long long)rows * cols;
  dim3 grid((unsigned)((n + TPB - 1) / TPB), batch);
  sm_launch_scope sc(ctx, SM_K_OTHER);
  if (dtype == SM_F32)
    hipLaunchKernelGGL(sm_copy_in_kernel<SM_F32>, grid, dim3(TPB), 0, ctx->stream, src, rows, cols, dst, ld, dst_stride);
  else
    hipLaunchKernelGGL(sm_copy_in_kernel<SM_BF16>, grid, dim3(TPB), 0, ctx->stream, src, rows, cols, dst, ld, dst_stride);
  SM_HIP(ctx, hipGetLastError());
  return SM_OK;
}

int sm_launch_copy_out(signmuon_ctx* ctx, const bf16_t* src, int ld, long long src_stride, int batch, int rows,
                       int cols, void* dst, int dtype, const float* scale) {
  const long long n = (long long)rows * cols;
  dim3 grid((unsigned)((n + TPB - 1) / TPB), batch);
  sm_launch_scope sc(ctx, SM_K_OTHER);
  if (dtype == SM_F32)
    hipLaunchKernelGGL(sm_copy_out_kernel<SM_F32>, grid, dim3(TPB), 0, ctx->stream, src, ld, src_stride, rows, cols, dst,
                       scale);
  else
    hipLaunchKernelGGL(sm_copy_out_kernel<SM_BF16>, grid, dim3(TPB), 0, ctx->stream, src, ld, src_stride, rows, cols,
                       dst, scale);
  SM_HIP(ctx, hipGetLastError());
  return SM_OK;
}

int sm_launch_sumsq(signmuon_ctx* ctx, const void* x, int dtype, long long n, int batch, float* scratch, float* sumsq) {
  const int chunks = (int)((n + SM_MOM_CHUNK - 1) / SM_MOM_CHUNK);
  {
    dim3 grid(chunks, batch);
    sm_launch_scope sc(ctx, SM_K_OTHER);
    if (dtype == SM_F32)
      hipLaunchKernelGGL(sm_sumsq_kernel<SM_F32>, grid, dim3(TPB), 0, ctx->stream, x, n, chunks, scratch);
    else
      hipLaunchKernelGGL(sm_sumsq_kernel<SM_BF16>, grid, dim3(TPB), 0, ctx->stream, x, n, chunks, scratch);
    SM_HIP(ctx, hipGetLastError());
  }
  return sm_launch_reduce_partials(ctx, scratch, chunks, batch, sumsq);
}
