// Training-mode batch normalisation for gfx950, forward and backward, with statistics per
// data-group (each group normalises over its own B*H*W values per channel). HBM-bound: every
// kernel streams [rows][ld] NHWC tensors once. Reductions run in fp64 registers inside a
// workgroup and are combined across workgroups in a fixed order, so results are reproducible.
//
//   forward : mu, var over the group's rows; xhat = (x - mu) * rstd; v = alpha * (gamma * xhat + beta) + res;
//             y = relu ? max(v, 0) : v   (+ sign plane of y)
//   backward: g = alpha * dy;  dbeta = sum g;  dgamma = sum g * xhat;
//             dx = gamma * rstd * (g - dbeta / m - xhat * dgamma / m),  m = rows per group
// The backward uses the mean, rstd and gamma that the forward of the same mini-batch stored.
#include "kernels.h"

namespace dds {
namespace {

struct bf16_t { uint16_t v; };

__device__ __forceinline__ float bf2f(uint16_t v) { return __uint_as_float(((uint32_t)v) << 16); }
__device__ __forceinline__ uint16_t f2bf(float f) {  // round to nearest even
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// Eight consecutive channels of one row. Channel strides are multiples of 8 (bf16) or 4 (fp32):
// `full` is false for the last group of an fp32 row whose stride is 4 mod 8 (upper half absent).
template <typename T>
__device__ __forceinline__ void load8(const void* base, size_t elem, bool full, float (&f)[8]) {
  if (sizeof(T) == 2) {
    const uint4 v = *(const uint4*)((const char*)base + elem * 2);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) { f[2 * i] = bf2f((uint16_t)(w[i] & 0xffffu)); f[2 * i + 1] = bf2f((uint16_t)(w[i] >> 16)); }
  } else {
    const float4 a = *(const float4*)((const char*)base + elem * 4);
    f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w;
    if (full) {
      const float4 b = *(const float4*)((const char*)base + elem * 4 + 16);
      f[4] = b.x; f[5] = b.y; f[6] = b.z; f[7] = b.w;
    } else {
      f[4] = f[5] = f[6] = f[7] = 0.f;
    }
  }
}

template <typename T>
__device__ __forceinline__ void store8(void* base, size_t elem, bool full, const float (&f)[8]) {
  if (sizeof(T) == 2) {
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = (uint32_t)f2bf(f[2 * i]) | ((uint32_t)f2bf(f[2 * i + 1]) << 16);
    *(uint4*)((char*)base + elem * 2) = make_uint4(w[0], w[1], w[2], w[3]);
  } else {
    *(float4*)((char*)base + elem * 4) = make_float4(f[0], f[1], f[2], f[3]);
    if (full) *(float4*)((char*)base + elem * 4 + 16) = make_float4(f[4], f[5], f[6], f[7]);
  }
}

// Thread layout shared by the four kernels: 256 threads = rpp rows x cg channel groups of 8.
struct Lane {
  int tg, tr, rpp, c0;
  bool active, full;
  long long row_lo, row_hi;  // this workgroup's rows (absolute)
};

__device__ __forceinline__ Lane make_lane(const BnParams& p) {
  Lane l;
  const int cg = (p.ld + 7) / 8;
  l.rpp = 256 / cg;
  l.tg = threadIdx.x % cg;
  l.tr = threadIdx.x / cg;
  l.active = l.tr < l.rpp;
  l.c0 = 8 * l.tg;
  l.full = l.c0 + 8 <= p.ld;
  const int split = blockIdx.x, rep = blockIdx.y;
  const long long lo = (long long)split * p.rows_per_split;
  const long long hi = lo + p.rows_per_split < p.rows_per_rep ? lo + p.rows_per_split : p.rows_per_rep;
  l.row_lo = (long long)rep * p.rows_per_rep + lo;
  l.row_hi = (long long)rep * p.rows_per_rep + hi;
  return l;
}

// ------------------------------------------------------------------ forward
// grid (nsplit, W). scratch[((rep * nsplit + split) * ld + c) * 2 + {0, 1}] = sum x, sum x^2 over the split's rows.
template <typename T>
__global__ __launch_bounds__(256) void bn_fwd_stats_kernel(BnParams p) {
  const Lane l = make_lane(p);
  const int cg = (p.ld + 7) / 8;
  double s[8], ss[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) s[i] = ss[i] = 0.0;
  if (l.active) {
    for (long long r = l.row_lo + l.tr; r < l.row_hi; r += l.rpp) {
      float f[8];
      load8<T>(p.x, (size_t)r * p.ld + l.c0, l.full, f);
#pragma unroll
      for (int i = 0; i < 8; ++i) { s[i] += (double)f[i]; ss[i] += (double)f[i] * (double)f[i]; }
    }
  }
  __shared__ double red[16 * 256];
#pragma unroll
  for (int i = 0; i < 8; ++i) { red[i * 256 + threadIdx.x] = s[i]; red[(8 + i) * 256 + threadIdx.x] = ss[i]; }
  __syncthreads();
  if (l.active && l.tr == 0) {
    double* out = p.scratch + (((size_t)blockIdx.y * gridDim.x + blockIdx.x) * p.ld + l.c0) * 2;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if (l.c0 + i >= p.ld) break;
      double a = 0.0, b = 0.0;
      for (int t = 0; t < l.rpp; ++t) { a += red[i * 256 + t * cg + l.tg]; b += red[(8 + i) * 256 + t * cg + l.tg]; }
      out[2 * i] = a;
      out[2 * i + 1] = b;
    }
  }
}

// grid (nsplit, W): same row partition as the statistics kernel. Every thread folds the nsplit
// partial sums of its 8 channels (in order) into scale / shift, then streams its rows.
template <typename T>
__global__ __launch_bounds__(256) void bn_fwd_apply_kernel(BnParams p) {
  const Lane l = make_lane(p);
  if (!l.active) return;
  const int rep = blockIdx.y, nsplit = gridDim.x;
  const float* gamma = p.gamma + (size_t)rep * p.rep_stride;
  const float* beta = p.beta + (size_t)rep * p.rep_stride;
  float scale[8], shift[8];
  const double m = (double)p.rows_per_rep;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    scale[i] = shift[i] = 0.f;
    const int c = l.c0 + i;
    if (c >= p.ld) continue;
    double a = 0.0, b = 0.0;
    for (int sp = 0; sp < nsplit; ++sp) {
      const double* in = p.scratch + (((size_t)rep * nsplit + sp) * p.ld + c) * 2;
      a += in[0];
      b += in[1];
    }
    const double mean = a / m;
    double var = b / m - mean * mean;
    var = var > 0.0 ? var : 0.0;
    const float rstd = (float)(1.0 / sqrt(var + (double)p.eps));
    const float g = c < p.C ? gamma[(size_t)c * p.gstride] : 0.f;
    const float bt = c < p.C ? beta[c] : 0.f;
    scale[i] = p.alpha * g * rstd;
    shift[i] = p.alpha * (bt - (float)mean * g * rstd);
    if (blockIdx.x == 0 && l.tr == 0) {  // what the backward of this mini-batch needs
      float* st = p.stats + (size_t)rep * 3 * p.ld;
      st[c] = (float)mean;
      st[p.ld + c] = rstd;
      st[2 * p.ld + c] = g;
    }
  }
  for (long long r = l.row_lo + l.tr; r < l.row_hi; r += l.rpp) {
    const size_t e = (size_t)r * p.ld + l.c0;
    float f[8], q[8];
    load8<T>(p.x, e, l.full, f);
    if (p.res) load8<T>(p.res, e, l.full, q);
    uint32_t bits = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      float v = fmaf(f[i], scale[i], shift[i]);
      if (p.res) v += q[i];
      if (p.relu) v = v > 0.f ? v : 0.f;
      f[i] = v;
    }
    store8<T>(p.y, e, l.full, f);
    if (p.bits_out) {
      // the sign of the stored (rounded) value, as the convolution epilogues define the plane
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float stored = sizeof(T) == 2 ? bf2f(f2bf(f[i])) : f[i];
        bits |= (stored > 0.f ? 1u : 0u) << i;
      }
      ((uint8_t*)p.bits_out)[(size_t)r * (p.ld / 8) + l.tg] = (uint8_t)bits;
    }
  }
}

// ------------------------------------------------------------------ backward
// grid (nsplit, W). Writes split row (rep * nsplit + split) of the parameter-gradient partials:
// dgamma[c] at c * gstride, dbeta[c] at C * gstride + c (the layout of a 1x1 "convolution" with one
// input channel, so that the update kernels treat gamma / beta like any other layer).
template <typename T>
__global__ __launch_bounds__(256) void bn_bwd_stats_kernel(BnParams p) {
  const Lane l = make_lane(p);
  const int cg = (p.ld + 7) / 8;
  const int rep = blockIdx.y;
  const float* st = p.stats + (size_t)rep * 3 * p.ld;
  float mean[8], rstd[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int c = l.c0 + i;
    mean[i] = l.active && c < p.ld ? st[c] : 0.f;
    rstd[i] = l.active && c < p.ld ? st[p.ld + c] : 0.f;
  }
  double s[8], ss[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) s[i] = ss[i] = 0.0;
  if (l.active) {
    for (long long r = l.row_lo + l.tr; r < l.row_hi; r += l.rpp) {
      const size_t e = (size_t)r * p.ld + l.c0;
      float f[8], g[8];
      load8<T>(p.x, e, l.full, f);
      load8<T>(p.dy, e, l.full, g);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float xh = (f[i] - mean[i]) * rstd[i];
        s[i] += (double)g[i];
        ss[i] += (double)g[i] * (double)xh;
      }
    }
  }
  __shared__ double red[16 * 256];
#pragma unroll
  for (int i = 0; i < 8; ++i) { red[i * 256 + threadIdx.x] = s[i]; red[(8 + i) * 256 + threadIdx.x] = ss[i]; }
  __syncthreads();
  if (l.active && l.tr == 0) {
    float* out = p.partial + ((size_t)rep * gridDim.x + blockIdx.x) * p.pstride;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int c = l.c0 + i;
      if (c >= p.C) break;
      double a = 0.0, b = 0.0;
      for (int t = 0; t < l.rpp; ++t) { a += red[i * 256 + t * cg + l.tg]; b += red[(8 + i) * 256 + t * cg + l.tg]; }
      out[(size_t)c * p.gstride] = p.alpha * (float)b;            // dgamma
      out[(size_t)p.C * p.gstride + c] = p.alpha * (float)a;      // dbeta
    }
  }
}

// grid (nsplit, W): folds the group's split rows (in order) into dbeta, dgamma and streams dx.
template <typename T>
__global__ __launch_bounds__(256) void bn_bwd_apply_kernel(BnParams p) {
  const Lane l = make_lane(p);
  if (!l.active) return;
  const int rep = blockIdx.y, nsplit = gridDim.x;
  const float* st = p.stats + (size_t)rep * 3 * p.ld;
  float mean[8], rstd[8], k0[8], k1[8], k2[8];
  const double m = (double)p.rows_per_rep;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int c = l.c0 + i;
    mean[i] = rstd[i] = k0[i] = k1[i] = k2[i] = 0.f;
    if (c >= p.C) continue;
    double db = 0.0, dg = 0.0;
    for (int sp = 0; sp < nsplit; ++sp) {
      const float* in = p.partial + ((size_t)rep * nsplit + sp) * p.pstride;
      dg += (double)in[(size_t)c * p.gstride];
      db += (double)in[(size_t)p.C * p.gstride + c];
    }
    mean[i] = st[c];
    rstd[i] = st[p.ld + c];
    const float gr = st[2 * p.ld + c] * rstd[i];  // gamma * rstd
    // dx = gr * (alpha*dy - db/m - xhat*dg/m), db and dg already carry alpha
    k0[i] = gr * p.alpha;
    k1[i] = gr * (float)(db / m);
    k2[i] = gr * (float)(dg / m);
  }
  for (long long r = l.row_lo + l.tr; r < l.row_hi; r += l.rpp) {
    const size_t e = (size_t)r * p.ld + l.c0;
    float f[8], g[8];
    load8<T>(p.x, e, l.full, f);
    load8<T>(p.dy, e, l.full, g);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float xh = (f[i] - mean[i]) * rstd[i];
      f[i] = k0[i] * g[i] - k1[i] - xh * k2[i];
    }
    store8<T>(p.dx, e, l.full, f);
  }
}

}  // namespace

#define DDS_BN_DISPATCH(dt, KERNEL, ...)               \
  do {                                                 \
    if ((dt) == DT_F32) KERNEL<float> __VA_ARGS__;     \
    else KERNEL<bf16_t> __VA_ARGS__;                   \
  } while (0)

void launch_bn_forward(int dt, const BnParams& p, hipStream_t s) {
  dim3 grid(p.nsplit, p.W);
  DDS_BN_DISPATCH(dt, bn_fwd_stats_kernel, <<<grid, 256, 0, s>>>(p));
  DDS_BN_DISPATCH(dt, bn_fwd_apply_kernel, <<<grid, 256, 0, s>>>(p));
}

void launch_bn_backward(int dt, const BnParams& p, hipStream_t s) {
  dim3 grid(p.nsplit, p.W);
  DDS_BN_DISPATCH(dt, bn_bwd_stats_kernel, <<<grid, 256, 0, s>>>(p));
  if (p.dx) DDS_BN_DISPATCH(dt, bn_bwd_apply_kernel, <<<grid, 256, 0, s>>>(p));
}

}  // namespace dds
