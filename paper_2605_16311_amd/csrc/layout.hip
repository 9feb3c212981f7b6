// Layout helpers around the Newton-Schulz workspace: copies between caller
// matrices and the zero-padded bf16 working layout, bf16 transposes, and sums
// of squares for the Frobenius scale of Alg. PolarNS.
#include "common.h"

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

// 64 x 64 bf16 tile transpose through LDS.  grid = (C/64, R/64, batch).
__global__ void __launch_bounds__(TPB) sm_transpose_kernel(const bf16_t* __restrict__ src, int lds_, long long sstride,
                                                           bf16_t* __restrict__ dst, int ldd, long long dstride) {
  __shared__ unsigned short tile[64][66];
  const int b = blockIdx.z;
  const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  const unsigned short* s = reinterpret_cast<const unsigned short*>(src) + (long long)b * sstride;
  unsigned short* d = reinterpret_cast<unsigned short*>(dst) + (long long)b * dstride;
  const int t = threadIdx.x;
#pragma unroll
  for (int pass = 0; pass < 2; ++pass) {
    const int r = (t >> 3) + 32 * pass, ch = t & 7;
    const u32x4 v = *reinterpret_cast<const u32x4*>(s + (long long)(r0 + r) * lds_ + c0 + ch * 8);
    const unsigned wv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      tile[r][ch * 8 + 2 * k] = (unsigned short)(wv[k] & 0xFFFFu);
      tile[r][ch * 8 + 2 * k + 1] = (unsigned short)(wv[k] >> 16);
    }
  }
  __syncthreads();
#pragma unroll
  for (int pass = 0; pass < 2; ++pass) {
    const int c = (t >> 3) + 32 * pass, ch = t & 7;  // output row c, output cols ch*8..+7
    unsigned wv[4];
#pragma unroll
    for (int k = 0; k < 4; ++k)
      wv[k] = (unsigned)tile[ch * 8 + 2 * k][c] | ((unsigned)tile[ch * 8 + 2 * k + 1][c] << 16);
    u32x4 v = {wv[0], wv[1], wv[2], wv[3]};
    *reinterpret_cast<u32x4*>(d + (long long)(c0 + c) * ldd + r0 + ch * 8) = v;
  }
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

}  // namespace

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

int sm_launch_transpose(signmuon_ctx* ctx, const bf16_t* src, int R, int C, int lds, long long sstride, bf16_t* dst,
                        int ldd, long long dstride, int batch) {
  if (R % 64 || C % 64 || lds % 8 || ldd % 8 || !sm_aligned(src, 16) || !sm_aligned(dst, 16) || sstride % 8 ||
      dstride % 8)
    return sm_fail(ctx, SM_EINVAL, "internal: transpose operand not padded/aligned");
  int done = 0;
  while (done < batch) {  // grid.z is limited to 65535
    const int g = std::min(batch - done, 32768);
    dim3 grid(C / 64, R / 64, g);
    sm_launch_scope sc(ctx, SM_K_OTHER);
    hipLaunchKernelGGL(sm_transpose_kernel, grid, dim3(TPB), 0, ctx->stream, src + (long long)done * sstride, lds,
                       sstride, dst + (long long)done * dstride, ldd, dstride);
    SM_HIP(ctx, hipGetLastError());
    done += g;
  }
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
