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

// Second half of the workgroup reduction. red[v * 256 + thread] holds quantity v (0-7: first sum of the
// thread's eight channels, 8-15: second sum) of every thread; thread = row-thread t * cg + channel group g.
// One thread per (v, g) adds the rpp row-threads in order and writes scale * total to
// out[channel * 2 + (v >> 3)], channel = 8 g + (v & 7).
__device__ __forceinline__ void fold_rows(const double* red, int cg, int rpp, int ld, double scale, double* out) {
  for (int o = threadIdx.x; o < 16 * cg; o += 256) {
    const int v = o / cg, g = o - v * cg;
    const int c = 8 * g + (v & 7);
    if (c >= ld) continue;
    double a = 0.0;
    for (int t = 0; t < rpp; ++t) a += red[v * 256 + t * cg + g];
    out[c * 2 + (v >> 3)] = scale * a;
  }
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
    // four rows per trip: four independent 16-byte loads in flight per thread
    long long r = l.row_lo + l.tr;
    for (; r + 3 * l.rpp < l.row_hi; r += 4 * l.rpp) {
      float f[4][8];
#pragma unroll
      for (int u = 0; u < 4; ++u) load8<T>(p.x, (size_t)(r + u * l.rpp) * p.ld + l.c0, l.full, f[u]);
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int i = 0; i < 8; ++i) { s[i] += (double)f[u][i]; ss[i] += (double)f[u][i] * (double)f[u][i]; }
    }
    for (; r < l.row_hi; r += l.rpp) {
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
  fold_rows(red, cg, l.rpp, p.ld, 1.0, p.scratch + ((size_t)blockIdx.y * gridDim.x + blockIdx.x) * p.ld * 2);
}

// grid (ceil(ld / 16), W), 256 threads = 16 split lanes x 16 channels: folds the nsplit partial sums of a
// channel (lane j takes splits j, j+16, ...; the sixteen lanes are combined in a fixed order) once per
// data-group, so that the streaming kernels read finished per-channel values.
// Forward (sum x, sum x^2): mean, rstd (and the gamma in use) into `stats`. Backward (sum g, sum g*xhat):
// dbeta, dgamma totals in fp64 into totals[(rep * ld + c) * 2 + {0, 1}] for the streaming kernel, and in fp32
// into row `rep` of the parameter-gradient partials (dgamma[c] at c * gstride, dbeta[c] at C * gstride + c: the
// layout of a 1x1 "convolution" with one input channel, so that the update kernels treat gamma / beta like
// any other layer with one split per data-group).
template <bool BWD>
__global__ __launch_bounds__(256) void bn_finalize_kernel(BnParams p) {
  const int rep = blockIdx.y, lane4 = threadIdx.x >> 4;
  const int c = blockIdx.x * 16 + (threadIdx.x & 15);
  const bool live = BWD ? c < p.C : c < p.ld;
  double a = 0.0, b = 0.0;
  if (live) {
#pragma unroll 8
    for (int sp = lane4; sp < p.nsplit; sp += 16) {
      const double* in = p.scratch + (((size_t)rep * p.nsplit + sp) * p.ld + c) * 2;
      a += in[0];
      b += in[1];
    }
  }
  __shared__ double red[2][16][16];
  red[0][lane4][threadIdx.x & 15] = a;
  red[1][lane4][threadIdx.x & 15] = b;
  __syncthreads();
  if (lane4 != 0 || !live) return;
  const int ch = threadIdx.x & 15;
  a = b = 0.0;
  for (int j = 0; j < 16; ++j) { a += red[0][j][ch]; b += red[1][j][ch]; }
  if (BWD) {
    double* out = p.totals + ((size_t)rep * p.ld + c) * 2;
    out[0] = a;  // dbeta
    out[1] = b;  // dgamma
    float* row = p.partial + (size_t)rep * p.pstride;
    row[(size_t)c * p.gstride] = (float)b;
    row[(size_t)p.C * p.gstride + c] = (float)a;
  } else {
    const double m = (double)p.rows_per_rep;
    const double mean = a / m;
    double var = b / m - mean * mean;
    var = var > 0.0 ? var : 0.0;
    float* st = p.stats + (size_t)rep * 3 * p.ld;
    st[c] = (float)mean;
    st[p.ld + c] = (float)(1.0 / sqrt(var + (double)p.eps));
    st[2 * p.ld + c] = c < p.C ? p.gamma[(size_t)rep * p.rep_stride + (size_t)c * p.gstride] : 0.f;
  }
}

// grid (nsplit, W): same row partition as the statistics kernel; streams its rows.
template <typename T>
__global__ __launch_bounds__(256) void bn_fwd_apply_kernel(BnParams p) {
  const Lane l = make_lane(p);
  if (!l.active) return;
  const int rep = blockIdx.y;
  const float* beta = p.beta + (size_t)rep * p.rep_stride;
  const float* st = p.stats + (size_t)rep * 3 * p.ld;
  float scale[8], shift[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    scale[i] = shift[i] = 0.f;
    const int c = l.c0 + i;
    if (c >= p.C) continue;
    const float mean = st[c], rstd = st[p.ld + c], g = st[2 * p.ld + c];
    scale[i] = p.alpha * g * rstd;
    shift[i] = p.alpha * (beta[c] - mean * g * rstd);
  }
  auto finish_row = [&](long long r, float (&f)[8], const float (&q)[8]) {
    const size_t e = (size_t)r * p.ld + l.c0;
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
      uint32_t bits = 0;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float stored = sizeof(T) == 2 ? bf2f(f2bf(f[i])) : f[i];
        bits |= (stored > 0.f ? 1u : 0u) << i;
      }
      ((uint8_t*)p.bits_out)[(size_t)r * (p.ld / 8) + l.tg] = (uint8_t)bits;
    }
  };
  // four rows per trip: all loads of the trip are issued before the first row is finished
  long long r = l.row_lo + l.tr;
  for (; r + 3 * l.rpp < l.row_hi; r += 4 * l.rpp) {
    float f[4][8], q[4][8];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const size_t e = (size_t)(r + u * l.rpp) * p.ld + l.c0;
      load8<T>(p.x, e, l.full, f[u]);
      if (p.res) load8<T>(p.res, e, l.full, q[u]);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) finish_row(r + u * l.rpp, f[u], q[u]);
  }
  for (; r < l.row_hi; r += l.rpp) {
    float f[8], q[8];
    const size_t e = (size_t)r * p.ld + l.c0;
    load8<T>(p.x, e, l.full, f);
    if (p.res) load8<T>(p.res, e, l.full, q);
    finish_row(r, f, q);
  }
}

// ------------------------------------------------------------------ backward
// grid (nsplit, W). scratch[((rep * nsplit + split) * ld + c) * 2 + {0, 1}] = sum g, sum g * xhat over the split's
// rows, g = alpha * dy.
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
    long long r = l.row_lo + l.tr;
    for (; r + 3 * l.rpp < l.row_hi; r += 4 * l.rpp) {
      float f[4][8], g[4][8];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const size_t e = (size_t)(r + u * l.rpp) * p.ld + l.c0;
        load8<T>(p.x, e, l.full, f[u]);
        load8<T>(p.dy, e, l.full, g[u]);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const float xh = (f[u][i] - mean[i]) * rstd[i];
          s[i] += (double)g[u][i];
          ss[i] += (double)g[u][i] * (double)xh;
        }
    }
    for (; r < l.row_hi; r += l.rpp) {
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
  fold_rows(red, cg, l.rpp, p.ld, (double)p.alpha, p.scratch + ((size_t)rep * gridDim.x + blockIdx.x) * p.ld * 2);
}

// grid (nsplit, W): streams dx from dy, x, the saved statistics and the finished dgamma / dbeta totals.
template <typename T>
__global__ __launch_bounds__(256) void bn_bwd_apply_kernel(BnParams p) {
  const Lane l = make_lane(p);
  if (!l.active) return;
  const int rep = blockIdx.y;
  const float* st = p.stats + (size_t)rep * 3 * p.ld;
  float mean[8], rstd[8], k0[8], k1[8], k2[8];
  const double m = (double)p.rows_per_rep;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int c = l.c0 + i;
    mean[i] = rstd[i] = k0[i] = k1[i] = k2[i] = 0.f;
    if (c >= p.C) continue;
    const double* tot = p.totals + ((size_t)rep * p.ld + c) * 2;
    const double db = tot[0], dg = tot[1];
    mean[i] = st[c];
    rstd[i] = st[p.ld + c];
    const float gr = st[2 * p.ld + c] * rstd[i];  // gamma * rstd
    // dx = gr * (alpha*dy - db/m - xhat*dg/m), db and dg already carry alpha
    k0[i] = gr * p.alpha;
    k1[i] = gr * (float)(db / m);
    k2[i] = gr * (float)(dg / m);
  }
  auto finish_row = [&](long long r, float (&f)[8], const float (&g)[8]) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float xh = (f[i] - mean[i]) * rstd[i];
      f[i] = k0[i] * g[i] - k1[i] - xh * k2[i];
    }
    store8<T>(p.dx, (size_t)r * p.ld + l.c0, l.full, f);
  };
  long long r = l.row_lo + l.tr;
  for (; r + 3 * l.rpp < l.row_hi; r += 4 * l.rpp) {
    float f[4][8], g[4][8];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const size_t e = (size_t)(r + u * l.rpp) * p.ld + l.c0;
      load8<T>(p.x, e, l.full, f[u]);
      load8<T>(p.dy, e, l.full, g[u]);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) finish_row(r + u * l.rpp, f[u], g[u]);
  }
  for (; r < l.row_hi; r += l.rpp) {
    float f[8], g[8];
    const size_t e = (size_t)r * p.ld + l.c0;
    load8<T>(p.x, e, l.full, f);
    load8<T>(p.dy, e, l.full, g);
    finish_row(r, f, g);
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
  dim3 fgrid((p.ld + 15) / 16, p.W);
  DDS_BN_DISPATCH(dt, bn_fwd_stats_kernel, <<<grid, 256, 0, s>>>(p));
  bn_finalize_kernel<false><<<fgrid, 256, 0, s>>>(p);
  DDS_BN_DISPATCH(dt, bn_fwd_apply_kernel, <<<grid, 256, 0, s>>>(p));
}

void launch_bn_backward(int dt, const BnParams& p, hipStream_t s) {
  dim3 grid(p.nsplit, p.W);
  dim3 fgrid((p.ld + 15) / 16, p.W);
  DDS_BN_DISPATCH(dt, bn_bwd_stats_kernel, <<<grid, 256, 0, s>>>(p));
  bn_finalize_kernel<true><<<fgrid, 256, 0, s>>>(p);
  DDS_BN_DISPATCH(dt, bn_bwd_apply_kernel, <<<grid, 256, 0, s>>>(p));
}

}  // namespace dds
