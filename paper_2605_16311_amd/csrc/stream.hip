// HBM-bound kernels of the Sign-Muon step: momentum (a1), sign extraction and
// packing (a5), majority vote (a6) with the fused update (a8), and the update
// after a local polar step.  All are pure streaming passes: every byte is read
// once with 16-byte (or 4-byte broadcast) coalesced accesses and written once.
#include "common.h"

namespace {

constexpr int TPB = 256;

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
  return v;
}

// Sum over the 256 threads of a workgroup, fixed order; result valid in thread 0.
__device__ __forceinline__ float block_sum(float v, float* lds4) {
  v = wave_sum(v);
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  if (lane == 0) lds4[wv] = v;
  __syncthreads();
  float r = 0.f;
  if (threadIdx.x == 0) r = (lds4[0] + lds4[1]) + (lds4[2] + lds4[3]);
  return r;
}

// sign decision of Alg. 3's encoding note, x >= 0 by IEEE comparison, taken on
// the bit pattern so that it does not depend on the denormal mode:
// true for +0 .. +inf and for -0, false for negatives and every NaN.
__device__ __forceinline__ unsigned ge0_f32(unsigned u) { return (u <= 0x7F800000u) | (u == 0x80000000u); }
__device__ __forceinline__ unsigned ge0_bf16(unsigned h) { return (h <= 0x7F80u) | (h == 0x8000u); }

// ------------------------------------------------------------------ momentum
// start[k]: the block that holds workgroup (k << shift) of the launch, so that a workgroup finds its
// block in a step or two instead of walking the table (workgroups are short: the walk would show).
struct mom_args {
  int n, M;
  float beta, omb, wd;
  int shift;
  int start[64];
  sm_mom_desc d[SM_MOM_MAX_GROUP];
};
static_assert(sizeof(mom_args) <= 4096, "kernel arguments are limited to 4 KB");

__device__ __forceinline__ float mom_one(float m, float g, float w, const mom_args& a, bool has_wd) {
  if (has_wd) g = __fadd_rn(g, __fmul_rn(a.wd, w));
  return __fadd_rn(__fmul_rn(a.beta, m), __fmul_rn(a.omb, g));
}

template <bool VEC>
__global__ void __launch_bounds__(TPB) sm_momentum_kernel(const mom_args a) {
  __shared__ float red[4];
  int bi = a.start[blockIdx.x >> a.shift];
  while (bi + 1 < a.n && (int)blockIdx.x >= a.d[bi + 1].block_begin) ++bi;
  const sm_mom_desc& D = a.d[bi];
  const int local = blockIdx.x - D.block_begin;
  const int p = local / D.chunks, ch = local - p * D.chunks;
  const long long d = D.d;
  float* mom = D.mom + (long long)p * d;
  const float* grad = D.grad + (long long)p * d;
  const float* w = D.w;
  bf16_t* x = D.x ? D.x + (long long)p * D.x_stride : nullptr;
  const bool has_wd = (w != nullptr) && (a.wd != 0.f);
  const bool flat = (D.ld == D.cols);
  const long long base = (long long)ch * SM_MOM_CHUNK;
  float ss = 0.f;
  if (VEC) {
#pragma unroll
    for (int it = 0; it < SM_MOM_CHUNK / (TPB * 4); ++it) {
      const long long i = base + (long long)it * (TPB * 4) + threadIdx.x * 4;
      if (i >= d) break;  // d % 4 == 0 on this path
      f32x4 m = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(mom + i));
      const f32x4 g = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(grad + i));
      f32x4 ww = {0.f, 0.f, 0.f, 0.f};
      if (has_wd) ww = *reinterpret_cast<const f32x4*>(w + i);
      m.x = mom_one(m.x, g.x, ww.x, a, has_wd);
      m.y = mom_one(m.y, g.y, ww.y, a, has_wd);
      m.z = mom_one(m.z, g.z, ww.z, a, has_wd);
      m.w = mom_one(m.w, g.w, ww.w, a, has_wd);
      // neither the momentum nor its bf16 copy is read again before it has left the caches
      __builtin_nontemporal_store(m, reinterpret_cast<f32x4*>(mom + i));
      ss += (m.x * m.x + m.y * m.y) + (m.z * m.z + m.w * m.w);
      if (x) {
        if (flat || (D.cols & 3) == 0) {
          const long long xi = flat ? i : (i / D.cols) * D.ld + (i % D.cols);
          bf16x4 h = {(bf16_t)m.x, (bf16_t)m.y, (bf16_t)m.z, (bf16_t)m.w};
          __builtin_nontemporal_store(h, reinterpret_cast<bf16x4*>(x + xi));
        } else {
          const float mv[4] = {m.x, m.y, m.z, m.w};
          for (int k = 0; k < 4; ++k) {
            const long long e = i + k;
            x[(e / D.cols) * D.ld + (e % D.cols)] = (bf16_t)mv[k];
          }
        }
      }
    }
  } else {
    for (int it = 0; it < SM_MOM_CHUNK / TPB; ++it) {
      const long long i = base + (long long)it * TPB + threadIdx.x;
      if (i >= d) break;
      const float m = mom_one(mom[i], grad[i], has_wd ? w[i] : 0.f, a, has_wd);
      mom[i] = m;
      ss += m * m;
      if (x) x[flat ? i : (i / D.cols) * D.ld + (i % D.cols)] = (bf16_t)m;
    }
  }
  if (D.partial) {
    const float tot = block_sum(ss, red);
    if (threadIdx.x == 0) D.partial[(long long)p * D.chunks + ch] = tot;
  }
}

// sumsq[i] = sum of partial[i*chunks .. +chunks) in a fixed tree order; one workgroup per i.
__global__ void __launch_bounds__(TPB) sm_reduce_partials_kernel(const float* partial, int chunks, float* sumsq) {
  __shared__ float red[4];
  const float* src = partial + (long long)blockIdx.x * chunks;
  float s = 0.f;
  for (int j = threadIdx.x; j < chunks; j += TPB) s += src[j];
  const float tot = block_sum(s, red);
  if (threadIdx.x == 0) sumsq[blockIdx.x] = tot;
}

__global__ void sm_inv_sigma_kernel(const float* sig, int count, float eps, int from_sq, float* inv) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= count) return;
  float s = sig[i];
  if (from_sq) s = sqrtf(s);
  inv[i] = 1.0f / fmaxf(s, eps);
}

struct sigma_args {
  int n;
  float eps;
  sm_sigma_desc d[SM_SIGMA_MAX_GROUP];
};

// One workgroup per item of every class of the table.
__global__ void __launch_bounds__(TPB) sm_sigma_group_kernel(const sigma_args a) {
  __shared__ float red[4];
  int di = 0;
  while (di + 1 < a.n && (int)blockIdx.x >= a.d[di + 1].block_begin) ++di;
  const sm_sigma_desc& D = a.d[di];
  const int i = blockIdx.x - D.block_begin;
  if (D.mode == 0) {
    const float* src = D.partial + (long long)i * D.chunks;
    float s = 0.f;
    for (int j = threadIdx.x; j < D.chunks; j += TPB) s += src[j];
    const float tot = block_sum(s, red);
    if (threadIdx.x == 0) {
      D.sig[i] = tot;
      D.inv[i] = 1.0f / fmaxf(sqrtf(tot), a.eps);
    }
  } else if (threadIdx.x == 0) {
    D.inv[i] = (D.mode == 1) ? 1.0f / fmaxf(D.sig[i], a.eps) : D.value;
  }
}

// ------------------------------------------------------------------ sign pack
// One thread = one output byte = 8 consecutive entries of the flattened matrix.
// Source row index / padded leading dimension are resolved per byte (cols % 8 == 0
// on the fast path so a byte never straddles rows).
// One launch covers a table of matrices (all workers of each): workgroup -> (matrix, worker, chunk).
struct sp_args {
  int n;
  int pad_;
  sm_sp_desc d[SM_SP_MAX_GROUP];
};

template <int DT, int FMT, bool FAST>
__global__ void __launch_bounds__(TPB) sm_sign_pack_kernel(const sp_args a) {
  int di = 0;
  while (di + 1 < a.n && (int)blockIdx.x >= a.d[di + 1].block_begin) ++di;
  const sm_sp_desc& D = a.d[di];
  const int local = blockIdx.x - D.block_begin;
  const int b = local / D.blocks_per_row, bx = local - b * D.blocks_per_row;
  const long long n = D.n, bytes_per_row = D.bytes_per_row;
  const int cols = D.cols, ld = D.ld;
  const unsigned short* ub = reinterpret_cast<const unsigned short*>(D.u) + (DT == SM_BF16 ? (long long)b * D.batch_stride : 0);
  const unsigned* uf = reinterpret_cast<const unsigned*>(D.u) + (DT == SM_F32 ? (long long)b * D.batch_stride : 0);
  unsigned char* o = reinterpret_cast<unsigned char*>(D.out) + (long long)b * D.out_stride;
  constexpr int UNROLL = 4;
  const long long q0 = ((long long)bx * UNROLL) * TPB + threadIdx.x;
#pragma unroll
  for (int j = 0; j < UNROLL; ++j) {
    const long long q = q0 + (long long)j * TPB;  // byte index
    if (q >= bytes_per_row) break;
    const long long e0 = q * 8;
    unsigned bits = 0;
    if (FAST && e0 + 8 <= n) {
      const long long src = (ld == cols) ? e0 : (e0 / cols) * ld + (e0 % cols);
      if (DT == SM_BF16) {
        const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(ub + src));
        const unsigned wv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          bits |= ge0_bf16(wv[k] & 0xFFFFu) << (2 * k);
          bits |= ge0_bf16(wv[k] >> 16) << (2 * k + 1);
        }
      } else {
        const u32x4 v0 = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(uf + src));
        const u32x4 v1 = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(uf + src + 4));
        const unsigned wv[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
#pragma unroll
        for (int k = 0; k < 8; ++k) bits |= ge0_f32(wv[k]) << k;
      }
      if (FMT == SM_SIGN_INT8) {
        // +1 = 0x01, -1 = 0xFF
        unsigned lo = 0, hi = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          lo |= (((bits >> k) & 1u) ? 0x01u : 0xFFu) << (8 * k);
          hi |= (((bits >> (k + 4)) & 1u) ? 0x01u : 0xFFu) << (8 * k);
        }
        *reinterpret_cast<uint2*>(o + e0) = make_uint2(lo, hi);
        continue;
      }
    } else {
      for (int k = 0; k < 8; ++k) {
        const long long e = e0 + k;
        if (e >= n) break;
        const long long src = (ld == cols) ? e : (e / cols) * ld + (e % cols);
        const unsigned g = (DT == SM_BF16) ? ge0_bf16(ub[src]) : ge0_f32(uf[src]);
        bits |= g << k;
        if (FMT == SM_SIGN_INT8) o[e] = g ? 0x01 : 0xFF;
      }
      if (FMT == SM_SIGN_INT8) continue;
    }
    o[q] = (unsigned char)bits;
  }
}

// 1-bit output when every matrix of the launch can be read in whole 8-entry groups and its output is
// 4-byte aligned: SPB_UNROLL bytes per thread, all loads issued before the first use, and the
// bytes of four neighbouring lanes leave as one 32-bit store (byte stores cost a full store slot each).
constexpr int SPB_UNROLL = 2;

template <int DT>
__global__ void __launch_bounds__(TPB) sm_sign_pack_bits_kernel(const sp_args a) {
  int di = 0;
  while (di + 1 < a.n && (int)blockIdx.x >= a.d[di + 1].block_begin) ++di;
  const sm_sp_desc& D = a.d[di];
  const int local = blockIdx.x - D.block_begin;
  const int b = local / D.blocks_per_row, bx = local - b * D.blocks_per_row;
  const long long n = D.n, bytes_per_row = D.bytes_per_row;  // a multiple of 8: a 4-lane group is in range as a whole
  const int cols = D.cols, ld = D.ld;
  const unsigned short* ub = reinterpret_cast<const unsigned short*>(D.u) + (DT == SM_BF16 ? (long long)b * D.batch_stride : 0);
  const unsigned* uf = reinterpret_cast<const unsigned*>(D.u) + (DT == SM_F32 ? (long long)b * D.batch_stride : 0);
  unsigned char* o = reinterpret_cast<unsigned char*>(D.out) + (long long)b * D.out_stride;
  const long long q0 = ((long long)bx * SPB_UNROLL) * TPB + threadIdx.x;
  u32x4 v0[SPB_UNROLL], v1[SPB_UNROLL];
#pragma unroll
  for (int j = 0; j < SPB_UNROLL; ++j) {
    const long long e0 = (q0 + (long long)j * TPB) * 8;
    v0[j] = v1[j] = u32x4{0u, 0u, 0u, 0u};
    if (e0 + 8 <= n) {
      const long long src = (ld == cols) ? e0 : (e0 / cols) * ld + (e0 % cols);
      if (DT == SM_BF16) {
        v0[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(ub + src));
      } else {
        v0[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(uf + src));
        v1[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(uf + src + 4));
      }
    }
  }
#pragma unroll
  for (int j = 0; j < SPB_UNROLL; ++j) {
    const long long q = q0 + (long long)j * TPB;  // byte index
    const long long e0 = q * 8;
    unsigned bits = 0;
    if (e0 + 8 <= n) {
      if (DT == SM_BF16) {
        const unsigned wv[4] = {v0[j].x, v0[j].y, v0[j].z, v0[j].w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          bits |= ge0_bf16(wv[k] & 0xFFFFu) << (2 * k);
          bits |= ge0_bf16(wv[k] >> 16) << (2 * k + 1);
        }
      } else {
        const unsigned wv[8] = {v0[j].x, v0[j].y, v0[j].z, v0[j].w, v1[j].x, v1[j].y, v1[j].z, v1[j].w};
#pragma unroll
        for (int k = 0; k < 8; ++k) bits |= ge0_f32(wv[k]) << k;
      }
    } else {  // the group that holds entry n - 1, and the zero padding after it
      for (int k = 0; k < 8; ++k) {
        const long long e = e0 + k;
        if (e >= n) break;
        const long long src = (ld == cols) ? e : (e / cols) * ld + (e % cols);
        bits |= ((DT == SM_BF16) ? ge0_bf16(ub[src]) : ge0_f32(uf[src])) << k;
      }
    }
    bits |= __shfl_down(bits, 1, 64) << 8;
    bits |= __shfl_down(bits, 2, 64) << 16;
    if ((threadIdx.x & 3) == 0 && q < bytes_per_row) __builtin_nontemporal_store(bits, reinterpret_cast<unsigned*>(o + q));
  }
}

// ------------------------------------------------------------------ vote
// Voted bits only.  Bit-sliced counting: the M words of a position are added into
// PLANES binary counter planes with ripple carries (M < 2^PLANES), then the planes
// are compared with the threshold ceil(M/2) bit-serially from the top plane down.
// Adds the set bits of `x` into the bit-sliced counter `plane` (ripple carry).
template <int PLANES, typename W>
__device__ __forceinline__ void planes_add(W (&plane)[PLANES], W x) {
#pragma unroll
  for (int k = 0; k < PLANES; ++k) {
    const W t = plane[k] & x;
    plane[k] ^= x;
    x = t;
  }
}

// Bit mask of the positions whose count is >= T.
template <int PLANES, typename W>
__device__ __forceinline__ W planes_ge(const W (&plane)[PLANES], unsigned T) {
  W gt = 0, eq = ~(W)0;
#pragma unroll
  for (int k = PLANES - 1; k >= 0; --k) {
    const W tb = ((T >> k) & 1u) ? ~(W)0 : (W)0;
    gt |= eq & plane[k] & ~tb;
    eq &= ~(plane[k] ^ tb);
  }
  return gt | eq;
}

// Workers are read eight at a time: all eight loads of a group are issued before the first is
// added, so a thread keeps 8 x 16 bytes in flight (rows beyond M read as zero words, which
// count nothing).
constexpr int VOTE_GROUP = 8;

// A thread owns VB_PAIRS pairs of 64-bit words, TPB pairs apart (rows are 8-byte aligned with any stride: a
// pair is read with one 16-byte load only where row base and stride allow it).  Measured on 85 M entries, M = 8:
// one pair per thread 17.3 us, two 18.6 us, four 22.3 us.
constexpr int VB_PAIRS = 1;

template <int PLANES>
__global__ void __launch_bounds__(TPB) sm_vote_bits_kernel(const unsigned long long* __restrict__ signs, int M,
                                                           long long words, long long stride_words,
                                                           long long n, unsigned long long* __restrict__ voted) {
  typedef __attribute__((ext_vector_type(2))) unsigned long long u64x2;
  const bool vec_ok = ((stride_words & 1) == 0) && ((reinterpret_cast<uintptr_t>(signs) & 15) == 0);
  long long w0[VB_PAIRS];
  unsigned long long p0[VB_PAIRS][PLANES], p1[VB_PAIRS][PLANES];
#pragma unroll
  for (int r = 0; r < VB_PAIRS; ++r) {
    w0[r] = (((long long)blockIdx.x * VB_PAIRS + r) * TPB + threadIdx.x) * 2;
#pragma unroll
    for (int k = 0; k < PLANES; ++k) p0[r][k] = p1[r][k] = 0;
  }
  if (w0[0] >= words) return;
  for (int pb = 0; pb < M; pb += VOTE_GROUP) {
    unsigned long long a[VB_PAIRS][VOTE_GROUP], b[VB_PAIRS][VOTE_GROUP];
#pragma unroll
    for (int r = 0; r < VB_PAIRS; ++r) {
      const bool live = w0[r] < words, pair = w0[r] + 1 < words;
#pragma unroll
      for (int q = 0; q < VOTE_GROUP; ++q) {
        a[r][q] = b[r][q] = 0;
        if (live && pb + q < M) {
          const unsigned long long* src = signs + (long long)(pb + q) * stride_words + w0[r];
          if (vec_ok && pair) {
            const u64x2 v = __builtin_nontemporal_load(reinterpret_cast<const u64x2*>(src));
            a[r][q] = v[0];
            b[r][q] = v[1];
          } else {
            a[r][q] = __builtin_nontemporal_load(src);
            if (pair) b[r][q] = __builtin_nontemporal_load(src + 1);
          }
        }
      }
    }
#pragma unroll
    for (int r = 0; r < VB_PAIRS; ++r)
#pragma unroll
      for (int q = 0; q < VOTE_GROUP; ++q) {
        planes_add<PLANES>(p0[r], a[r][q]);
        planes_add<PLANES>(p1[r], b[r][q]);
      }
  }
  const unsigned T = (unsigned)((M + 1) / 2);  // vote = (count >= T)
  const bool out_vec = (reinterpret_cast<uintptr_t>(voted) & 15) == 0;
#pragma unroll
  for (int r = 0; r < VB_PAIRS; ++r) {
    if (w0[r] >= words) break;
    const bool pair = w0[r] + 1 < words;
    unsigned long long v[2] = {planes_ge<PLANES>(p0[r], T), planes_ge<PLANES>(p1[r], T)};
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const long long rem = n - (w0[r] + h) * 64;
      if (rem < 64) v[h] &= (rem <= 0) ? 0ull : ((1ull << rem) - 1ull);
    }
    if (pair && out_vec) {
      const u64x2 o = {v[0], v[1]};
      __builtin_nontemporal_store(o, reinterpret_cast<u64x2*>(voted + w0[r]));
    } else {
      voted[w0[r]] = v[0];
      if (pair) voted[w0[r] + 1] = v[1];
    }
  }
}

// Voted bits for any M (used beyond 255 workers): one thread = one byte.
__global__ void __launch_bounds__(TPB) sm_vote_bits_generic_kernel(const unsigned char* __restrict__ signs, int M,
                                                                   long long n, long long stride_bytes,
                                                                   unsigned char* __restrict__ voted,
                                                                   long long bytes_out) {
  const long long q = (long long)blockIdx.x * TPB + threadIdx.x;
  if (q >= bytes_out) return;
  int c[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int p = 0; p < M; ++p) {
    const unsigned b = signs[(long long)p * stride_bytes + q];
#pragma unroll
    for (int k = 0; k < 8; ++k) c[k] += (b >> k) & 1u;
  }
  unsigned bits = 0;
#pragma unroll
  for (int k = 0; k < 8; ++k)
    if (q * 8 + k < n && 2 * c[k] >= M) bits |= 1u << k;
  voted[q] = (unsigned char)bits;
}

typedef sm_vote_desc vote_x_args;
struct vote_g_args {
  int n;
  int pad_;
  sm_vote_desc d[SM_VOTE_MAX_GROUP];
};

// Expanding vote: one thread = 4 consecutive entries.  FMT selects the input
// transport; outputs (voted in a non-bit format, counts, fused W update) are all
// optional.  n4 = ceil(n/4) threads in total.
template <int FMT>
__global__ void __launch_bounds__(TPB) sm_vote_expand_kernel(const vote_g_args g) {
  int di = 0;
  while (di + 1 < g.n && (int)blockIdx.x >= g.d[di + 1].block_begin) ++di;
  const vote_x_args& a = g.d[di];
  const long long t = (long long)(blockIdx.x - a.block_begin) * TPB + threadIdx.x;
  const long long e0 = t * 4;
  if (e0 >= a.n) return;
  int c[4] = {0, 0, 0, 0};
  if (FMT == SM_SIGN_1BIT) {
    const unsigned* base = reinterpret_cast<const unsigned*>(a.signs) + (e0 >> 5);
    const int sh = (int)(e0 & 31);
    const long long stride_w = a.stride_bytes >> 2;
    int p = 0;
    while (p < a.M) {
      const int lim = min(a.M, p + 255);
      unsigned acc = 0;
      for (; p < lim; ++p) {
        const unsigned nib = (base[(long long)p * stride_w] >> sh) & 0xFu;
        acc += (nib * 0x00204081u) & 0x01010101u;
      }
#pragma unroll
      for (int k = 0; k < 4; ++k) c[k] += (acc >> (8 * k)) & 0xFF;
    }
  } else {
    const signed char* base = reinterpret_cast<const signed char*>(a.signs) + e0;
    if (e0 + 4 <= a.n && (a.stride_bytes & 3) == 0 && (reinterpret_cast<uintptr_t>(a.signs) & 3) == 0) {
      for (int p = 0; p < a.M; ++p) {
        const unsigned v = __builtin_nontemporal_load(reinterpret_cast<const unsigned*>(base + (long long)p * a.stride_bytes));
#pragma unroll
        for (int k = 0; k < 4; ++k) c[k] += (int)(signed char)(v >> (8 * k));
      }
    } else {
      for (int p = 0; p < a.M; ++p)
        for (int k = 0; k < 4; ++k)
          if (e0 + k < a.n) c[k] += base[(long long)p * a.stride_bytes + k];
    }
  }
  float s[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const bool plus = (FMT == SM_SIGN_1BIT) ? (2 * c[k] >= a.M) : (c[k] >= 0);
    s[k] = plus ? 1.0f : -1.0f;
  }
  const bool full = (e0 + 4 <= a.n);
  if (a.counts) {
    if (full) {
      *reinterpret_cast<int4*>(a.counts + e0) = make_int4(c[0], c[1], c[2], c[3]);
    } else {
      for (int k = 0; k < 4 && e0 + k < a.n; ++k) a.counts[e0 + k] = c[k];
    }
  }
  if (a.w) {
    if (full) {
      float4 wv = *reinterpret_cast<float4*>(a.w + e0);
      wv.x = __fsub_rn(wv.x, __fmul_rn(a.lr, s[0]));
      wv.y = __fsub_rn(wv.y, __fmul_rn(a.lr, s[1]));
      wv.z = __fsub_rn(wv.z, __fmul_rn(a.lr, s[2]));
      wv.w = __fsub_rn(wv.w, __fmul_rn(a.lr, s[3]));
      *reinterpret_cast<float4*>(a.w + e0) = wv;
    } else {
      for (int k = 0; k < 4 && e0 + k < a.n; ++k) a.w[e0 + k] = __fsub_rn(a.w[e0 + k], __fmul_rn(a.lr, s[k]));
    }
  }
  if (a.voted) {
    const bool flat = (a.ld == a.cols);
    if (a.vfmt == SM_VOTE_INT8) {
      signed char* o = reinterpret_cast<signed char*>(a.voted);
      if (full) {
        unsigned v = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) v |= (s[k] > 0.f ? 0x01u : 0xFFu) << (8 * k);
        *reinterpret_cast<unsigned*>(o + e0) = v;
      } else {
        for (int k = 0; k < 4 && e0 + k < a.n; ++k) o[e0 + k] = s[k] > 0.f ? 1 : -1;
      }
    } else if (a.vfmt == SM_VOTE_BF16) {
      bf16_t* o = reinterpret_cast<bf16_t*>(a.voted);
      if (full && (flat || (a.cols & 3) == 0)) {
        const long long di = flat ? e0 : (e0 / a.cols) * a.ld + (e0 % a.cols);
        bf16x4 h = {(bf16_t)s[0], (bf16_t)s[1], (bf16_t)s[2], (bf16_t)s[3]};
        *reinterpret_cast<bf16x4*>(o + di) = h;
      } else {
        for (int k = 0; k < 4 && e0 + k < a.n; ++k) {
          const long long e = e0 + k;
          o[flat ? e : (e / a.cols) * a.ld + (e % a.cols)] = (bf16_t)s[k];
        }
      }
    } else if (a.vfmt == SM_VOTE_F32) {
      float* o = reinterpret_cast<float*>(a.voted);
      if (full && (flat || (a.cols & 3) == 0)) {
        const long long di = flat ? e0 : (e0 / a.cols) * a.ld + (e0 % a.cols);
        *reinterpret_cast<float4*>(o + di) = make_float4(s[0], s[1], s[2], s[3]);
      } else {
        for (int k = 0; k < 4 && e0 + k < a.n; ++k) {
          const long long e = e0 + k;
          o[flat ? e : (e / a.cols) * a.ld + (e % a.cols)] = s[k];
        }
      }
    }
  }
}

// Packs +-1 int32 sums (int8 transport) into voted bits: one thread = one byte.
__global__ void __launch_bounds__(TPB) sm_vote_int8_bits_kernel(const signed char* __restrict__ signs, int M,
                                                                long long n, long long stride_bytes,
                                                                unsigned char* __restrict__ voted,
                                                                long long bytes_out) {
  const long long q = (long long)blockIdx.x * TPB + threadIdx.x;
  if (q >= bytes_out) return;
  unsigned bits = 0;
  for (int k = 0; k < 8; ++k) {
    const long long e = q * 8 + k;
    if (e >= n) break;
    int s = 0;
    for (int p = 0; p < M; ++p) s += signs[(long long)p * stride_bytes + e];
    bits |= (s >= 0 ? 1u : 0u) << k;
  }
  voted[q] = (unsigned char)bits;
}

// ------------------------------------------------------------------ update after a local polar step
struct upd_args {
  int n;
  int pad_;
  sm_upd_desc d[SM_UPD_MAX_GROUP];
};

// A workgroup owns UPD_ITERS * TPB * 4 consecutive entries of one block: UPD_ITERS rounds of 4 entries per
// thread, all loads of a round set issued before the first store.
constexpr int UPD_ITERS = 4;
constexpr int UPD_CHUNK = UPD_ITERS * TPB * 4;

__global__ void __launch_bounds__(TPB) sm_update_kernel(const upd_args g) {
  int di = 0;
  while (di + 1 < g.n && (int)blockIdx.x >= g.d[di + 1].block_begin) ++di;
  const sm_upd_desc& D = g.d[di];
  float* __restrict__ w = D.w;
  const bf16_t* __restrict__ d = D.d;
  const int cols = D.cols, ld = D.ld;
  const float step = D.kappa ? __fmul_rn(D.step, D.kappa[0]) : D.step;
  const long long n = (long long)D.rows * cols;
  const long long base = (long long)(blockIdx.x - D.block_begin) * UPD_CHUNK + threadIdx.x * 4;
  if ((cols & 3) == 0 && base - threadIdx.x * 4 + UPD_CHUNK <= n) {  // a full chunk of whole groups of 4
    bf16x4 h[UPD_ITERS];
    f32x4 wv[UPD_ITERS];
#pragma unroll
    for (int it = 0; it < UPD_ITERS; ++it) {
      const long long e0 = base + (long long)it * (TPB * 4);
      const long long di4 = (ld == cols) ? e0 : (e0 / cols) * ld + (e0 % cols);
      h[it] = __builtin_nontemporal_load(reinterpret_cast<const bf16x4*>(d + di4));
      wv[it] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(w + e0));
    }
#pragma unroll
    for (int it = 0; it < UPD_ITERS; ++it) {
      const long long e0 = base + (long long)it * (TPB * 4);
      wv[it].x = __fsub_rn(wv[it].x, __fmul_rn(step, (float)h[it][0]));
      wv[it].y = __fsub_rn(wv[it].y, __fmul_rn(step, (float)h[it][1]));
      wv[it].z = __fsub_rn(wv[it].z, __fmul_rn(step, (float)h[it][2]));
      wv[it].w = __fsub_rn(wv[it].w, __fmul_rn(step, (float)h[it][3]));
      __builtin_nontemporal_store(wv[it], reinterpret_cast<f32x4*>(w + e0));
    }
    return;
  }
  for (int it = 0; it < UPD_ITERS; ++it) {
    const long long e0 = base + (long long)it * (TPB * 4);
    if (e0 >= n) return;
    if (e0 + 4 <= n && (cols & 3) == 0) {
      const long long di4 = (ld == cols) ? e0 : (e0 / cols) * ld + (e0 % cols);
      const bf16x4 h = *reinterpret_cast<const bf16x4*>(d + di4);
      float4 wv = *reinterpret_cast<float4*>(w + e0);
      wv.x = __fsub_rn(wv.x, __fmul_rn(step, (float)h[0]));
      wv.y = __fsub_rn(wv.y, __fmul_rn(step, (float)h[1]));
      wv.z = __fsub_rn(wv.z, __fmul_rn(step, (float)h[2]));
      wv.w = __fsub_rn(wv.w, __fmul_rn(step, (float)h[3]));
      *reinterpret_cast<float4*>(w + e0) = wv;
    } else {
      for (int k = 0; k < 4 && e0 + k < n; ++k) {
        const long long e = e0 + k;
        const float dv = (float)d[(e / cols) * ld + (e % cols)];
        w[e] = __fsub_rn(w[e], __fmul_rn(step, dv));
      }
    }
  }
}

}  // namespace

// =================================================================== host side
int sm_launch_momentum(signmuon_ctx* ctx, const sm_mom_desc* descs, int n, int M, float beta, float wd) {
  int done = 0;
  while (done < n) {
    const int g = std::min(n - done, SM_MOM_MAX_GROUP);
    mom_args a;
    a.n = g;
    a.M = M;
    a.beta = beta;
    a.omb = 1.0f - beta;
    a.wd = wd;
    long long blocks = 0;
    bool vec = true;
    for (int i = 0; i < g; ++i) {
      a.d[i] = descs[done + i];
      a.d[i].block_begin = (int)blocks;
      blocks += (long long)M * a.d[i].chunks;
      const sm_mom_desc& D = a.d[i];
      vec = vec && (D.d % 4 == 0) && sm_aligned(D.mom, 16) && sm_aligned(D.grad, 16) &&
            (!D.w || sm_aligned(D.w, 16)) && (!D.x || (sm_aligned(D.x, 8) && D.ld % 4 == 0 && D.x_stride % 4 == 0));
    }
    if (blocks > 0x7FFFFFFFLL) return sm_fail(ctx, SM_EUNSUPPORTED, "momentum: too many entries for one launch");
    a.shift = 0;
    while ((blocks >> a.shift) >= 64) ++a.shift;
    for (int k = 0, bi = 0; k < 64; ++k) {
      while (bi + 1 < g && ((long long)k << a.shift) >= a.d[bi + 1].block_begin) ++bi;
      a.start[k] = bi;
    }
    if (blocks > 0) {
      sm_launch_scope sc(ctx, SM_K_MOMENTUM);
      if (vec)
        hipLaunchKernelGGL(sm_momentum_kernel<true>, dim3((unsigned)blocks), dim3(TPB), 0, ctx->stream, a);
      else
        hipLaunchKernelGGL(sm_momentum_kernel<false>, dim3((unsigned)blocks), dim3(TPB), 0, ctx->stream, a);
    }
    SM_HIP(ctx, hipGetLastError());
    done += g;
  }
  return SM_OK;
}

int sm_launch_reduce_partials(signmuon_ctx* ctx, const float* partial, int chunks, int count, float* sumsq) {
  sm_launch_scope sc(ctx, SM_K_OTHER);
  hipLaunchKernelGGL(sm_reduce_partials_kernel, dim3(count), dim3(TPB), 0, ctx->stream, partial, chunks, sumsq);
  SM_HIP(ctx, hipGetLastError());
  return SM_OK;
}

int sm_launch_inv_sigma(signmuon_ctx* ctx, const float* sig, int count, float eps, bool from_sq, float* inv_sigma) {
  sm_launch_scope sc(ctx, SM_K_OTHER);
  hipLaunchKernelGGL(sm_inv_sigma_kernel, dim3((count + 255) / 256), dim3(256), 0, ctx->stream, sig, count, eps,
                     from_sq ? 1 : 0, inv_sigma);
  SM_HIP(ctx, hipGetLastError());
  return SM_OK;
}

int sm_launch_sigma_group(signmuon_ctx* ctx, const sm_sigma_desc* descs, int n, float eps) {
  int done = 0;
  while (done < n) {
    const int g = std::min(n - done, SM_SIGMA_MAX_GROUP);
    sigma_args a;
    a.n = g;
    a.eps = eps;
    int blocks = 0;
    for (int i = 0; i < g; ++i) {
      a.d[i] = descs[done + i];
      a.d[i].block_begin = blocks;
      blocks += a.d[i].count;
    }
    if (blocks > 0) {
      sm_launch_scope sc(ctx, SM_K_OTHER);
      hipLaunchKernelGGL(sm_sigma_group_kernel, dim3(blocks), dim3(TPB), 0, ctx->stream, a);
    }
    SM_HIP(ctx, hipGetLastError());
    done += g;
  }
  return SM_OK;
}

int sm_launch_sign_pack_group(signmuon_ctx* ctx, const sm_sp_desc* descs, int n, int dtype, int fmt, int M) {
  int done = 0;
  while (done < n) {
    const int g = std::min(n - done, SM_SP_MAX_GROUP);
    sp_args a;
    a.n = g;
    a.pad_ = 0;
    int blocks = 0;
    bool fast_ok = true;
    for (int i = 0; i < g; ++i) {
      sm_sp_desc& D = a.d[i];
      D = descs[done + i];
      D.bytes_per_row = (fmt == SM_SIGN_1BIT) ? 8 * ((D.n + 63) / 64) : (D.n + 7) / 8;  // threads per row
      // the fast path reads whole 8-entry groups with 16-byte loads
      fast_ok = fast_ok && (D.ld == D.cols || (D.cols % 8 == 0 && D.ld % 8 == 0)) && sm_aligned(D.u, 16) &&
                (D.batch_stride % 8 == 0) &&
                (fmt == SM_SIGN_1BIT ? (sm_aligned(D.out, 4) && D.out_stride % 4 == 0)
                                     : (sm_aligned(D.out, 8) && D.out_stride % 8 == 0));
    }
    const int per_block = TPB * ((fmt == SM_SIGN_1BIT && fast_ok) ? SPB_UNROLL : 4);  // output bytes (threads' groups)
    for (int i = 0; i < g; ++i) {
      sm_sp_desc& D = a.d[i];
      D.blocks_per_row = (int)((D.bytes_per_row + per_block - 1) / per_block);
      D.block_begin = blocks;
      blocks += D.blocks_per_row * M;
    }
    if (blocks > 0) {
      const dim3 grid(blocks);
      sm_launch_scope sc(ctx, SM_K_SIGN_PACK);
#define SP_LAUNCH(DT, FMT, FAST) hipLaunchKernelGGL((sm_sign_pack_kernel<DT, FMT, FAST>), grid, dim3(TPB), 0, ctx->stream, a)
      if (dtype == SM_BF16) {
        if (fmt == SM_SIGN_1BIT) {
          if (fast_ok)
            hipLaunchKernelGGL((sm_sign_pack_bits_kernel<SM_BF16>), grid, dim3(TPB), 0, ctx->stream, a);
          else
            SP_LAUNCH(SM_BF16, SM_SIGN_1BIT, false);
        } else {
          if (fast_ok) SP_LAUNCH(SM_BF16, SM_SIGN_INT8, true); else SP_LAUNCH(SM_BF16, SM_SIGN_INT8, false);
        }
      } else {
        if (fmt == SM_SIGN_1BIT) {
          if (fast_ok)
            hipLaunchKernelGGL((sm_sign_pack_bits_kernel<SM_F32>), grid, dim3(TPB), 0, ctx->stream, a);
          else
            SP_LAUNCH(SM_F32, SM_SIGN_1BIT, false);
        } else {
          if (fast_ok) SP_LAUNCH(SM_F32, SM_SIGN_INT8, true); else SP_LAUNCH(SM_F32, SM_SIGN_INT8, false);
        }
      }
#undef SP_LAUNCH
    }
    SM_HIP(ctx, hipGetLastError());
    done += g;
  }
  return SM_OK;
}

int sm_launch_sign_pack(signmuon_ctx* ctx, const void* u, int dtype, int batch, int rows, int cols, int ld,
                        long long batch_stride, int fmt, void* out, long long out_stride_bytes) {
  sm_sp_desc D;
  D.u = u;
  D.out = out;
  D.n = (long long)rows * cols;
  D.batch_stride = batch_stride;
  D.out_stride = out_stride_bytes;
  D.bytes_per_row = 0;
  D.cols = cols;
  D.ld = ld;
  D.blocks_per_row = 0;
  D.block_begin = 0;
  return sm_launch_sign_pack_group(ctx, &D, 1, dtype, fmt, batch);
}

int sm_launch_vote(signmuon_ctx* ctx, const sm_vote_args& v) {
  const long long n = v.n;
  const bool want_bits = v.voted && v.vfmt == SM_VOTE_BITS;
  const bool want_expand = v.counts || v.w || (v.voted && v.vfmt != SM_VOTE_BITS);
  if (want_bits) {
    sm_launch_scope sc(ctx, SM_K_VOTE);
    if (v.fmt == SM_SIGN_1BIT) {
      const long long words = (n + 63) / 64;
      const dim3 grid((unsigned)(((words + 1) / 2 + TPB * VB_PAIRS - 1) / (TPB * VB_PAIRS)));  // VB_PAIRS word pairs per thread
      const unsigned long long* sp = reinterpret_cast<const unsigned long long*>(v.signs);
      unsigned long long* vp = reinterpret_cast<unsigned long long*>(v.voted);
      if (v.M < 8)
        hipLaunchKernelGGL(sm_vote_bits_kernel<3>, grid, dim3(TPB), 0, ctx->stream, sp, v.M, words, v.stride_bytes / 8, n, vp);
      else if (v.M < 32)
        hipLaunchKernelGGL(sm_vote_bits_kernel<5>, grid, dim3(TPB), 0, ctx->stream, sp, v.M, words, v.stride_bytes / 8, n, vp);
      else if (v.M < 256)
        hipLaunchKernelGGL(sm_vote_bits_kernel<8>, grid, dim3(TPB), 0, ctx->stream, sp, v.M, words, v.stride_bytes / 8, n, vp);
      else
        hipLaunchKernelGGL(sm_vote_bits_generic_kernel, dim3((unsigned)((words * 8 + TPB - 1) / TPB)), dim3(TPB), 0,
                           ctx->stream, reinterpret_cast<const unsigned char*>(v.signs), v.M, n, v.stride_bytes,
                           reinterpret_cast<unsigned char*>(v.voted), words * 8);
    } else {
      const long long bytes_out = 8 * ((n + 63) / 64);
      hipLaunchKernelGGL(sm_vote_int8_bits_kernel, dim3((unsigned)((bytes_out + TPB - 1) / TPB)), dim3(TPB), 0,
                         ctx->stream, reinterpret_cast<const signed char*>(v.signs), v.M, n, v.stride_bytes,
                         reinterpret_cast<unsigned char*>(v.voted), bytes_out);
    }
    SM_HIP(ctx, hipGetLastError());
  }
  if (want_expand) {
    sm_vote_desc a;
    a.signs = v.signs;
    a.n = n;
    a.stride_bytes = v.stride_bytes;
    a.voted = (v.voted && v.vfmt != SM_VOTE_BITS) ? v.voted : nullptr;
    a.counts = v.counts;
    a.w = v.w;
    a.lr = v.lr_scaled;
    a.M = v.M;
    a.vfmt = v.vfmt;
    a.cols = v.cols;
    a.ld = v.ld;
    a.block_begin = 0;
    return sm_launch_vote_group(ctx, &a, 1, v.fmt);
  }
  return SM_OK;
}

// Expanding vote over 1-bit signs, wide form: a lane takes one 32-bit word of every worker's
// buffer per run, counted bit-sliced (PLANES binary counter planes, M < 2^PLANES) and compared with
// ceil(M/2) as in sm_vote_bits_kernel.  The 2048 votes of a run are then spread over the wave's
// lanes so that every store (and every load of W) covers consecutive addresses: lane l
// writes 8 consecutive bf16 per store (4 stores), and steps 4 consecutive weights per load
// and store (8 of each).  For tables whose entries have n % 32 == 0, no counts output and, if
// a voted matrix is asked for, the flat bf16 form.
// A wave takes VW_GROUPS runs of 64 consecutive words; the loads of all runs (eight workers at a time) are
// issued before the first is counted.  Measured: one run per wave is fastest (fused W update on 85 M entries,
// M = 8: 125 us against 136 us with two or four runs); what matters is that the eight loads are in flight together.
constexpr int VW_GROUPS = 1;

template <int PLANES>
__global__ void __launch_bounds__(TPB) sm_vote_wide_kernel(const vote_g_args g) {
  int di = 0;
  while (di + 1 < g.n && (int)blockIdx.x >= g.d[di + 1].block_begin) ++di;
  const vote_x_args& a = g.d[di];
  const long long words = a.n >> 5;
  const int lane = threadIdx.x & 63;
  // the wave's first word: a workgroup covers TPB * VW_GROUPS words
  const long long wbase = ((long long)(blockIdx.x - a.block_begin) * TPB + (threadIdx.x & ~63)) * VW_GROUPS;
  const long long stride_w = a.stride_bytes >> 2;
  const unsigned* sbase = reinterpret_cast<const unsigned*>(a.signs);
  unsigned plane[VW_GROUPS][PLANES];
#pragma unroll
  for (int r = 0; r < VW_GROUPS; ++r)
#pragma unroll
    for (int k = 0; k < PLANES; ++k) plane[r][k] = 0;
  for (int pb = 0; pb < a.M; pb += VOTE_GROUP) {
    unsigned x[VW_GROUPS][VOTE_GROUP];
#pragma unroll
    for (int r = 0; r < VW_GROUPS; ++r) {
      const long long wi = wbase + 64 * r + lane;
#pragma unroll
      for (int q = 0; q < VOTE_GROUP; ++q) {
        x[r][q] = 0;
        if (wi < words && pb + q < a.M) x[r][q] = __builtin_nontemporal_load(sbase + (long long)(pb + q) * stride_w + wi);
      }
    }
#pragma unroll
    for (int r = 0; r < VW_GROUPS; ++r)
#pragma unroll
      for (int q = 0; q < VOTE_GROUP; ++q) planes_add<PLANES>(plane[r], x[r][q]);
  }
  const unsigned T = (unsigned)((a.M + 1) / 2);
#pragma unroll
  for (int r = 0; r < VW_GROUPS; ++r) {
    const long long w0 = wbase + 64 * r;  // the run's first word
    if (w0 >= words) break;               // wave-uniform
    const unsigned v = (w0 + lane < words) ? planes_ge<PLANES>(plane[r], T) : 0u;
    if (a.voted) {
      bf16_t* o = reinterpret_cast<bf16_t*>(a.voted) + w0 * 32;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        // chunk 64 k + lane of the run's 256 chunks of 8 entries: byte (lane & 3) of word 16 k + lane / 4
        const unsigned word = __shfl(v, 16 * k + (lane >> 2), 64);
        const unsigned bits = (word >> (8 * (lane & 3))) & 0xFFu;
        if (w0 + 16 * k + (lane >> 2) < words) {
          u32x4 h;
#pragma unroll
          for (int q = 0; q < 4; ++q)
            h[q] = (((bits >> (2 * q)) & 1u) ? 0x3F80u : 0xBF80u) | ((((bits >> (2 * q + 1)) & 1u) ? 0x3F80u : 0xBF80u) << 16);
          *reinterpret_cast<u32x4*>(o + (64 * k + lane) * 8) = h;
        }
      }
    }
    if (a.w) {
      float* wp = a.w + w0 * 32;
      // group 64 k + lane of the run's 512 groups of 4 entries: nibble (lane & 7) of word 8 k + lane / 8;
      // the eight loads are issued before the first store
      f32x4 wv[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        wv[k] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (w0 + 8 * k + (lane >> 3) < words)
          wv[k] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(wp + (64 * k + lane) * 4));
      }
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const unsigned word = __shfl(v, 8 * k + (lane >> 3), 64);
        const unsigned bits = (word >> (4 * (lane & 7))) & 0xFu;
        if (w0 + 8 * k + (lane >> 3) < words) {
          f32x4 o = wv[k];
          o.x = __fsub_rn(o.x, __fmul_rn(a.lr, (bits & 1u) ? 1.0f : -1.0f));
          o.y = __fsub_rn(o.y, __fmul_rn(a.lr, (bits & 2u) ? 1.0f : -1.0f));
          o.z = __fsub_rn(o.z, __fmul_rn(a.lr, (bits & 4u) ? 1.0f : -1.0f));
          o.w = __fsub_rn(o.w, __fmul_rn(a.lr, (bits & 8u) ? 1.0f : -1.0f));
          __builtin_nontemporal_store(o, reinterpret_cast<f32x4*>(wp + (64 * k + lane) * 4));
        }
      }
    }
  }
}

// Expanding vote over int8 signs, wide form: one thread = 16 consecutive entries (one 16-byte load per
// worker), int32 sums, then any of: counts, voted int8 / bf16 (flat), fused W update.  For tables whose
// entries have n % 16 == 0 and 16-byte aligned rows.
__global__ void __launch_bounds__(TPB) sm_vote_int8_wide_kernel(const vote_g_args g) {
  int di = 0;
  while (di + 1 < g.n && (int)blockIdx.x >= g.d[di + 1].block_begin) ++di;
  const vote_x_args& a = g.d[di];
  const long long t = (long long)(blockIdx.x - a.block_begin) * TPB + threadIdx.x;
  const long long e0 = t * 16;
  if (e0 >= a.n) return;
  int c[16];
#pragma unroll
  for (int k = 0; k < 16; ++k) c[k] = 0;
  const unsigned char* base = reinterpret_cast<const unsigned char*>(a.signs) + e0;
  for (int p = 0; p < a.M; ++p) {
    const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(base + (long long)p * a.stride_bytes));
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
      for (int k = 0; k < 4; ++k) c[4 * q + k] += (int)(signed char)(v[q] >> (8 * k));
  }
  if (a.counts) {
#pragma unroll
    for (int q = 0; q < 4; ++q)
      *reinterpret_cast<int4*>(a.counts + e0 + 4 * q) = make_int4(c[4 * q], c[4 * q + 1], c[4 * q + 2], c[4 * q + 3]);
  }
  if (a.w) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      float4 wv = *reinterpret_cast<float4*>(a.w + e0 + 4 * q);
      wv.x = __fsub_rn(wv.x, __fmul_rn(a.lr, c[4 * q] >= 0 ? 1.0f : -1.0f));
      wv.y = __fsub_rn(wv.y, __fmul_rn(a.lr, c[4 * q + 1] >= 0 ? 1.0f : -1.0f));
      wv.z = __fsub_rn(wv.z, __fmul_rn(a.lr, c[4 * q + 2] >= 0 ? 1.0f : -1.0f));
      wv.w = __fsub_rn(wv.w, __fmul_rn(a.lr, c[4 * q + 3] >= 0 ? 1.0f : -1.0f));
      *reinterpret_cast<float4*>(a.w + e0 + 4 * q) = wv;
    }
  }
  if (a.voted) {
    if (a.vfmt == SM_VOTE_INT8) {
      u32x4 o;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        unsigned v4 = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) v4 |= (c[4 * q + k] >= 0 ? 0x01u : 0xFFu) << (8 * k);
        o[q] = v4;
      }
      *reinterpret_cast<u32x4*>(reinterpret_cast<unsigned char*>(a.voted) + e0) = o;
    } else {  // bf16, flat
      bf16_t* ob = reinterpret_cast<bf16_t*>(a.voted) + e0;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        u32x4 o;
#pragma unroll
        for (int q = 0; q < 4; ++q)
          o[q] = (c[8 * h + 2 * q] >= 0 ? 0x3F80u : 0xBF80u) | ((c[8 * h + 2 * q + 1] >= 0 ? 0x3F80u : 0xBF80u) << 16);
        *reinterpret_cast<u32x4*>(ob + 8 * h) = o;
      }
    }
  }
}

int sm_launch_vote_group(signmuon_ctx* ctx, const sm_vote_desc* descs, int n, int fmt) {
  int done = 0;
  while (done < n) {
    const int g = std::min(n - done, SM_VOTE_MAX_GROUP);
    vote_g_args a;
    a.n = g;
    a.pad_ = 0;
    // the wide kernel serves tables made only of whole 32-entry words, bf16 flat outputs, no counts
    bool wide = (fmt == SM_SIGN_1BIT);
    int max_m = 0;
    for (int i = 0; i < g && wide; ++i) {
      const sm_vote_desc& d = descs[done + i];
      wide = d.n % 32 == 0 && !d.counts && d.M < 256 && d.stride_bytes % 4 == 0 && sm_aligned(d.signs, 4) &&
             (!d.voted || (d.vfmt == SM_VOTE_BF16 && d.ld == d.cols && sm_aligned(d.voted, 16))) &&
             (!d.w || sm_aligned(d.w, 16));
      max_m = std::max(max_m, d.M);
    }
    // the wide int8 kernel: whole 16-entry groups, 16-byte aligned rows and outputs, int8 or flat bf16 votes
    bool wide8 = (fmt == SM_SIGN_INT8);
    for (int i = 0; i < g && wide8; ++i) {
      const sm_vote_desc& d = descs[done + i];
      wide8 = d.n % 16 == 0 && d.stride_bytes % 16 == 0 && sm_aligned(d.signs, 16) &&
              (!d.voted || (d.vfmt == SM_VOTE_INT8 && sm_aligned(d.voted, 16)) ||
               (d.vfmt == SM_VOTE_BF16 && d.ld == d.cols && sm_aligned(d.voted, 16))) &&
              (!d.w || sm_aligned(d.w, 16)) && (!d.counts || sm_aligned(d.counts, 16));
    }
    long long blocks = 0;
    for (int i = 0; i < g; ++i) {
      a.d[i] = descs[done + i];
      a.d[i].block_begin = (int)blocks;
      const long long threads = wide ? (a.d[i].n / 32 + VW_GROUPS - 1) / VW_GROUPS : wide8 ? a.d[i].n / 16 : (a.d[i].n + 3) / 4;
      blocks += (threads + TPB - 1) / TPB;
    }
    if (blocks > 0x7FFFFFFFLL) return sm_fail(ctx, SM_EUNSUPPORTED, "vote: too many entries for one launch");
    if (blocks > 0) {
      sm_launch_scope sc(ctx, SM_K_VOTE);
      const dim3 grid((unsigned)blocks), block(TPB);
      if (wide && max_m < 8)
        hipLaunchKernelGGL(sm_vote_wide_kernel<3>, grid, block, 0, ctx->stream, a);
      else if (wide && max_m < 32)
        hipLaunchKernelGGL(sm_vote_wide_kernel<5>, grid, block, 0, ctx->stream, a);
      else if (wide)
        hipLaunchKernelGGL(sm_vote_wide_kernel<8>, grid, block, 0, ctx->stream, a);
      else if (wide8)
        hipLaunchKernelGGL(sm_vote_int8_wide_kernel, grid, block, 0, ctx->stream, a);
      else if (fmt == SM_SIGN_1BIT)
        hipLaunchKernelGGL(sm_vote_expand_kernel<SM_SIGN_1BIT>, grid, block, 0, ctx->stream, a);
      else
        hipLaunchKernelGGL(sm_vote_expand_kernel<SM_SIGN_INT8>, grid, block, 0, ctx->stream, a);
    }
    SM_HIP(ctx, hipGetLastError());
    done += g;
  }
  return SM_OK;
}

int sm_launch_update_group(signmuon_ctx* ctx, const sm_upd_desc* descs, int n) {
  int done = 0;
  while (done < n) {
    const int g = std::min(n - done, SM_UPD_MAX_GROUP);
    upd_args a;
    a.n = g;
    a.pad_ = 0;
    long long blocks = 0;
    for (int i = 0; i < g; ++i) {
      a.d[i] = descs[done + i];
      a.d[i].block_begin = (int)blocks;
      blocks += ((long long)a.d[i].rows * a.d[i].cols + UPD_CHUNK - 1) / UPD_CHUNK;
    }
    if (blocks > 0) {
      sm_launch_scope sc(ctx, SM_K_UPDATE);
      hipLaunchKernelGGL(sm_update_kernel, dim3((unsigned)blocks), dim3(TPB), 0, ctx->stream, a);
    }
    SM_HIP(ctx, hipGetLastError());
    done += g;
  }
  return SM_OK;
}

int sm_launch_update(signmuon_ctx* ctx, float* w, const bf16_t* d, int rows, int cols, int ld, float step) {
  sm_upd_desc D;
  D.w = w;
  D.d = d;
  D.rows = rows;
  D.cols = cols;
  D.ld = ld;
  D.kappa = nullptr;
  D.step = step;
  D.block_begin = 0;
  D.pad_ = 0;
  return sm_launch_update_group(ctx, &D, 1);
}
