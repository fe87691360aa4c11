// Bandwidth-bound kernels for gfx950: batch ingest (layout + precision change),
// pooling, softmax cross-entropy, the fused replica-mean + SGD update, weight
// snapshots and parameter layout conversion. All tensors are NHWC with a channel
// stride that is a multiple of one 16-byte chunk.
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

// A 16-byte chunk viewed as CE floats.
template <typename T> struct Chunk;
template <> struct Chunk<float> {
  static constexpr int CE = 4;
  float f[4];
  __device__ __forceinline__ void load(const void* p) { uint4 v = *(const uint4*)p; f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y); f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w); }
  __device__ __forceinline__ void store(void* p) const { *(uint4*)p = make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3])); }
};
template <> struct Chunk<bf16_t> {
  static constexpr int CE = 8;
  float f[8];
  __device__ __forceinline__ void load(const void* p) {
    uint4 v = *(const uint4*)p;
    uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) { f[2 * i] = bf2f((uint16_t)(w[i] & 0xffffu)); f[2 * i + 1] = bf2f((uint16_t)(w[i] >> 16)); }
  }
  __device__ __forceinline__ void store(void* p) const {
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = (uint32_t)f2bf(f[2 * i]) | ((uint32_t)f2bf(f[2 * i + 1]) << 16);
    *(uint4*)p = make_uint4(w[0], w[1], w[2], w[3]);
  }
};

// ------------------------------------------------------------------ ingest
// caller batch [B][C][HW] fp32 (per replica) -> [W*B][HW][Cpad] T, zero channel padding
template <typename T>
__global__ void ingest_kernel(IngestParams p) {
  constexpr int CE = Chunk<T>::CE;
  const int chunks = p.Cpad / CE;
  const long long total = (long long)p.W * p.B * p.HW * chunks;
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < (long long)p.W * p.B) p.labels[i] = p.y[i / p.B][i % p.B];
  if (i >= total) return;
  // pixel index varies fastest across threads when the image has a spatial extent
  // (coalesced fp32 reads); chunk index fastest for flat inputs
  int n, hw, ch;
  if (p.HW > 1) {
    hw = (int)(i % p.HW);
    long long r = i / p.HW;
    ch = (int)(r % chunks);
    n = (int)(r / chunks);
  } else {
    hw = 0;
    ch = (int)(i % chunks);
    n = (int)(i / chunks);
  }
  const int s = n / p.B, b = n - s * p.B;
  const float* src = p.x[s] + (size_t)b * p.C * p.HW;
  Chunk<T> c;
#pragma unroll
  for (int e = 0; e < CE; ++e) {
    const int ci = ch * CE + e;
    c.f[e] = ci < p.C ? src[(size_t)ci * p.HW + hw] : 0.f;
  }
  c.store((char*)p.dst + (((size_t)n * p.HW + hw) * p.Cpad + (size_t)ch * CE) * sizeof(T));
}

// ------------------------------------------------------------------ pooling
template <typename T>
__global__ void maxpool_fwd_kernel(const char* x, char* y, int N, int H, int W, int C) {
  constexpr int CE = Chunk<T>::CE;
  const int chunks = C / CE, Ho = H / 2, Wo = W / 2;
  const long long total = (long long)N * Ho * Wo * chunks;
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const int ch = (int)(i % chunks);
  long long r = i / chunks;
  const int ow = (int)(r % Wo); r /= Wo;
  const int oh = (int)(r % Ho);
  const int n = (int)(r / Ho);
  Chunk<T> best, c;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const size_t off = ((((size_t)n * H + 2 * oh + (q >> 1)) * W + 2 * ow + (q & 1)) * C + (size_t)ch * CE) * sizeof(T);
    if (q == 0) best.load(x + off);
    else {
      c.load(x + off);
#pragma unroll
      for (int e = 0; e < CE; ++e) best.f[e] = c.f[e] > best.f[e] ? c.f[e] : best.f[e];
    }
  }
  best.store(y + ((((size_t)n * Ho + oh) * Wo + ow) * C + (size_t)ch * CE) * sizeof(T));
}

// gradient to the first maximum of each window (row-major order, strict comparisons);
// optionally times the ReLU derivative of the pre-pool tensor
template <typename T>
__global__ void maxpool_bwd_kernel(const char* dy, const char* x, char* dx, int N, int H, int W, int C, int relu_mask) {
  constexpr int CE = Chunk<T>::CE;
  const int chunks = C / CE, Ho = H / 2, Wo = W / 2;
  const long long total = (long long)N * Ho * Wo * chunks;
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const int ch = (int)(i % chunks);
  long long r = i / chunks;
  const int ow = (int)(r % Wo); r /= Wo;
  const int oh = (int)(r % Ho);
  const int n = (int)(r / Ho);
  Chunk<T> c[4], g;
  size_t off[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    off[q] = ((((size_t)n * H + 2 * oh + (q >> 1)) * W + 2 * ow + (q & 1)) * C + (size_t)ch * CE) * sizeof(T);
    c[q].load(x + off[q]);
  }
  g.load(dy + ((((size_t)n * Ho + oh) * Wo + ow) * C + (size_t)ch * CE) * sizeof(T));
  Chunk<T> o[4];
#pragma unroll
  for (int e = 0; e < CE; ++e) {
    int arg = 0;
    float best = c[0].f[e];
#pragma unroll
    for (int q = 1; q < 4; ++q)
      if (c[q].f[e] > best) { best = c[q].f[e]; arg = q; }
    const float gv = (relu_mask && !(best > 0.f)) ? 0.f : g.f[e];
#pragma unroll
    for (int q = 0; q < 4; ++q) o[q].f[e] = (q == arg) ? gv : 0.f;
  }
#pragma unroll
  for (int q = 0; q < 4; ++q) o[q].store(dx + off[q]);
}

template <typename T>
__global__ void gap_fwd_kernel(const char* x, char* y, int N, int HW, int C) {
  constexpr int CE = Chunk<T>::CE;
  const int chunks = C / CE;
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= N * chunks) return;
  const int ch = i % chunks, n = i / chunks;
  float acc[CE];
#pragma unroll
  for (int e = 0; e < CE; ++e) acc[e] = 0.f;
  Chunk<T> c;
  for (int q = 0; q < HW; ++q) {
    c.load(x + (((size_t)n * HW + q) * C + (size_t)ch * CE) * sizeof(T));
#pragma unroll
    for (int e = 0; e < CE; ++e) acc[e] += c.f[e];
  }
  const float inv = 1.f / (float)HW;
#pragma unroll
  for (int e = 0; e < CE; ++e) c.f[e] = acc[e] * inv;
  c.store(y + ((size_t)n * C + (size_t)ch * CE) * sizeof(T));
}

template <typename T>
__global__ void gap_bwd_kernel(const char* dy, const char* x, char* dx, int N, int HW, int C, int relu_mask) {
  constexpr int CE = Chunk<T>::CE;
  const int chunks = C / CE;
  const long long total = (long long)N * HW * chunks;
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const int ch = (int)(i % chunks);
  const long long r = i / chunks;
  const int n = (int)(r / HW);
  Chunk<T> g, c;
  g.load(dy + ((size_t)n * C + (size_t)ch * CE) * sizeof(T));
  const size_t off = ((size_t)r * C + (size_t)ch * CE) * sizeof(T);
  const float inv = 1.f / (float)HW;
  if (relu_mask) c.load(x + off);
#pragma unroll
  for (int e = 0; e < CE; ++e) {
    float v = g.f[e] * inv;
    if (relu_mask && !(c.f[e] > 0.f)) v = 0.f;
    g.f[e] = v;
  }
  g.store(dx + off);
}

// ------------------------------------------------------------------ softmax cross-entropy
// one workgroup per replica; thread per sample row; fixed-order tree for the loss sum
template <typename T>
__global__ __launch_bounds__(256) void softmax_ce_kernel(const float* logits, const int32_t* labels, char* dlogits,
                                                         float* loss, int B, int classes, int ldl, int ldg) {
  __shared__ float red[256];
  const int s = blockIdx.x;
  float lsum = 0.f;
  const float invB = 1.f / (float)B;
  for (int b = threadIdx.x; b < B; b += 256) {
    const size_t row = (size_t)s * B + b;
    const float* z = logits + row * ldl;
    const int y = labels[row];
    float mx = z[0];
    for (int c = 1; c < classes; ++c) mx = z[c] > mx ? z[c] : mx;
    float se = 0.f;
    for (int c = 0; c < classes; ++c) se += __expf(z[c] - mx);
    const float lse = __logf(se);
    lsum += -(z[y] - mx - lse);
    if (dlogits) {
      for (int c0 = 0; c0 < ldg; c0 += Chunk<T>::CE) {
        Chunk<T> g;
#pragma unroll
        for (int e = 0; e < Chunk<T>::CE; ++e) {
          const int c = c0 + e;
          float v = 0.f;
          if (c < classes) v = (__expf(z[c] - mx - lse) - (c == y ? 1.f : 0.f)) * invB;
          g.f[e] = v;
        }
        g.store(dlogits + (row * ldg + c0) * sizeof(T));
      }
    }
  }
  if (loss) {
    red[threadIdx.x] = lsum;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
      if (threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
      __syncthreads();
    }
    if (threadIdx.x == 0) loss[s] = red[0] * invB;
  }
}

// ------------------------------------------------------------------ update
// block_map[2*e] = descriptor index, block_map[2*e+1] = 1024-element block within the
// descriptor; four workgroups share an entry, 256 consecutive elements each. Lane l of every
// wave owns elements 4l..4l+3 of the workgroup's range; wave w sums the splits w, w+4, w+8, ...
// (eight row reads in flight, each a fully coalesced 1 KiB), in a fixed order: eight interleaved
// running sums, a fixed tree over them, then a fixed tree over the four waves through LDS. The
// result is bit-reproducible for a given split count. g = sum/W; v = mu*v + g; w -= lr*v (or lr*g).
template <typename T>
__global__ __launch_bounds__(256) void update_kernel(const UpdateDesc* descs, const int* block_map, float invW, float lr, float mu) {
  const UpdateDesc d = descs[block_map[2 * (blockIdx.x >> 2)]];
  const long long blk0 = (long long)block_map[2 * (blockIdx.x >> 2) + 1] * 1024 + (blockIdx.x & 3) * 256;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const long long base = blk0 + lane * 4;
  __shared__ float4 red[3][64];
  float4 a[8];
#pragma unroll
  for (int u = 0; u < 8; ++u) a[u] = make_float4(0.f, 0.f, 0.f, 0.f);
  if (base < d.n) {  // rows are pstride = n rounded up to 4 floats long: the vector read stays inside the row
    const float* src = d.partial + base;
    for (int j = wave; j < d.nsplit; j += 32) {
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int jj = j + 4 * u;
        if (jj < d.nsplit) {
          const float4 t = *(const float4*)(src + (size_t)jj * d.pstride);
          a[u].x += t.x; a[u].y += t.y; a[u].z += t.z; a[u].w += t.w;
        }
      }
    }
  }
#pragma unroll
  for (int w = 4; w > 0; w >>= 1)
#pragma unroll
    for (int u = 0; u < w; ++u) { a[u].x += a[u + w].x; a[u].y += a[u + w].y; a[u].z += a[u + w].z; a[u].w += a[u + w].w; }
  if (wave > 0) red[wave - 1][lane] = a[0];
  __syncthreads();
  if (wave > 0 || base >= d.n) return;
  {
    const float4 r1 = red[0][lane], r2 = red[1][lane], r3 = red[2][lane];
    a[0].x = (a[0].x + r1.x) + (r2.x + r3.x); a[0].y = (a[0].y + r1.y) + (r2.y + r3.y);
    a[0].z = (a[0].z + r1.z) + (r2.z + r3.z); a[0].w = (a[0].w + r1.w) + (r2.w + r3.w);
  }
  float g[4] = {a[0].x * invW, a[0].y * invW, a[0].z * invW, a[0].w * invW};
  if (base + 4 <= d.n) {
    float4 w = *(const float4*)(d.master + base);
    if (d.momentum) {
      float4 v = *(const float4*)(d.momentum + base);
      v.x = mu * v.x + g[0]; v.y = mu * v.y + g[1]; v.z = mu * v.z + g[2]; v.w = mu * v.w + g[3];
      *(float4*)(d.momentum + base) = v;
      g[0] = v.x; g[1] = v.y; g[2] = v.z; g[3] = v.w;
    }
    w.x -= lr * g[0]; w.y -= lr * g[1]; w.z -= lr * g[2]; w.w -= lr * g[3];
    *(float4*)(d.master + base) = w;
    if (d.work) {
      if (sizeof(T) == 2) {
        uint2 o;
        o.x = (uint32_t)f2bf(w.x) | ((uint32_t)f2bf(w.y) << 16);
        o.y = (uint32_t)f2bf(w.z) | ((uint32_t)f2bf(w.w) << 16);
        *(uint2*)((char*)d.work + base * 2) = o;
      } else {
        *(float4*)((char*)d.work + base * 4) = w;
      }
    }
  } else {
    for (long long i = base; i < d.n; ++i) {
      float w = d.master[i];
      float gg = g[i - base];
      if (d.momentum) { const float v = mu * d.momentum[i] + gg; d.momentum[i] = v; gg = v; }
      w -= lr * gg;
      d.master[i] = w;
      if (d.work) {
        if (sizeof(T) == 2) ((uint16_t*)d.work)[i] = f2bf(w);
        else ((float*)d.work)[i] = w;
      }
    }
  }
}

// work <- master (precision change only)
template <typename T>
__global__ __launch_bounds__(256) void recast_kernel(const UpdateDesc* descs, const int* block_map) {
  const UpdateDesc d = descs[block_map[2 * blockIdx.x]];
  const long long base = (long long)block_map[2 * blockIdx.x + 1] * 1024 + threadIdx.x * 4;
  if (!d.work) return;
  for (long long i = base; i < d.n && i < base + 4; ++i) {
    if (sizeof(T) == 2) ((uint16_t*)d.work)[i] = f2bf(d.master[i]);
    else ((float*)d.work)[i] = d.master[i];
  }
}

// Update (a)/(b) of Section 3.3 with a general mixing matrix P, for all W data-groups at once:
//   g_r = sum of data-group r's q splits (in order), v_r = mu*v_r + g_r, u_r = w_r - lr*v_r (or lr*g_r),
//   w_s = sum_r P[s][r] * u_r (r ascending, fp32), written to the fp32 master and the compute-precision copy.
// descs / block_map: data-group 0's entries (its `partial` points at split 0 of all W*q splits); data-group
// r's master / momentum / work lie r*rep_stride elements further. One thread owns four consecutive
// elements in all W copies, so the update is in place. Every layer's arrays are allocated in whole
// multiples of 64 elements and split rows in multiples of 4, so the four-wide accesses of the last
// thread of a layer stay inside that layer's padding.
template <typename T>
__global__ __launch_bounds__(256) void gossip_update_kernel(const UpdateDesc* descs, const int* block_map, const float* P,
                                                            int W, long long rep_stride, float lr, float mu) {
  const UpdateDesc d = descs[block_map[2 * blockIdx.x]];
  const long long base = (long long)block_map[2 * blockIdx.x + 1] * 1024 + threadIdx.x * 4;
  if (base >= d.n) return;
  const int q = d.nsplit;  // splits per data-group of this layer
  float4 u[32];
#pragma unroll
  for (int r = 0; r < 32; ++r) {
    if (r >= W) continue;
    const float* src = d.partial + (size_t)r * q * d.pstride + base;
    float4 g = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int j = 0; j < q; ++j) {
      const float4 t = *(const float4*)(src + (size_t)j * d.pstride);
      g.x += t.x; g.y += t.y; g.z += t.z; g.w += t.w;
    }
    if (d.momentum) {
      float4* vp = (float4*)(d.momentum + (long long)r * rep_stride + base);
      float4 v = *vp;
      v.x = mu * v.x + g.x; v.y = mu * v.y + g.y; v.z = mu * v.z + g.z; v.w = mu * v.w + g.w;
      *vp = v;
      g = v;
    }
    const float4 w = *(const float4*)(d.master + (long long)r * rep_stride + base);
    u[r] = make_float4(w.x - lr * g.x, w.y - lr * g.y, w.z - lr * g.z, w.w - lr * g.w);
  }
  for (int s = 0; s < W; ++s) {
    float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int r = 0; r < 32; ++r) {
      if (r >= W) continue;
      const float c = P[s * W + r];
      a.x = fmaf(c, u[r].x, a.x); a.y = fmaf(c, u[r].y, a.y); a.z = fmaf(c, u[r].z, a.z); a.w = fmaf(c, u[r].w, a.w);
    }
    *(float4*)(d.master + (long long)s * rep_stride + base) = a;
    if (d.work) {
      if (sizeof(T) == 2) {
        uint2 o;
        o.x = (uint32_t)f2bf(a.x) | ((uint32_t)f2bf(a.y) << 16);
        o.y = (uint32_t)f2bf(a.z) | ((uint32_t)f2bf(a.w) << 16);
        *(uint2*)((char*)d.work + ((long long)s * rep_stride + base) * 2) = o;
      } else {
        *(float4*)((char*)d.work + ((long long)s * rep_stride + base) * 4) = a;
      }
    }
  }
}

// Disagreement between data-groups (experiment section). Workgroup b owns 1024 elements of one
// layer (block_map entry b of data-group 0) and writes, for part 0 (weight) and 1 (bias) and every
// data-group s, sum_i (w_s[i] - mean_r w_r[i])^2 over its elements of that part, in fp64, to
// out[(2*b + part) * W + s]. The host adds the blocks of a tensor in order and takes the square
// root of the maximum.
__global__ __launch_bounds__(256) void consensus_kernel(const UpdateDesc* descs, const int* block_map, int W,
                                                        long long rep_stride, double* out) {
  const UpdateDesc d = descs[block_map[2 * blockIdx.x]];
  const long long blk0 = (long long)block_map[2 * blockIdx.x + 1] * 1024;
  const long long nw = d.n - d.Cout;
  double acc[2][32];
#pragma unroll
  for (int r = 0; r < 32; ++r) acc[0][r] = acc[1][r] = 0.0;
  for (int it = 0; it < 4; ++it) {
    const long long i = blk0 + it * 256 + threadIdx.x;
    if (i >= d.n) break;
    float w[32];
    double mean = 0.0;
#pragma unroll
    for (int r = 0; r < 32; ++r)
      if (r < W) { w[r] = d.master[(long long)r * rep_stride + i]; mean += (double)w[r]; }
    mean /= (double)W;
    const bool is_bias = i >= nw;
#pragma unroll
    for (int r = 0; r < 32; ++r)
      if (r < W) {
        const double e = (double)w[r] - mean;
        acc[0][r] += is_bias ? 0.0 : e * e;
        acc[1][r] += is_bias ? e * e : 0.0;
      }
  }
  __shared__ double red[256];
#pragma unroll
  for (int part = 0; part < 2; ++part)
#pragma unroll
    for (int r = 0; r < 32; ++r) {
      if (r >= W) continue;  // uniform
      red[threadIdx.x] = acc[part][r];
      __syncthreads();
      for (int h = 128; h > 0; h >>= 1) {
        if ((int)threadIdx.x < h) red[threadIdx.x] += red[threadIdx.x + h];
        __syncthreads();
      }
      if (threadIdx.x == 0) out[((size_t)2 * blockIdx.x + part) * W + r] = red[0];
      __syncthreads();
    }
}

// transposed snapshot: stash[slot][c][tap][kpad] <- master[k][tap][cpad], zero for k >= Cout.
// One workgroup moves a 64(k) x 64(c) tile of one tap through LDS so that both the reads
// (64 consecutive c) and the writes (64 consecutive k) are whole cache lines.
// block_map[2*blk+1] = tile index = (tap * cblocks + cb) * kblocks + kb.
template <typename T>
__global__ __launch_bounds__(256) void stash_kernel(const UpdateDesc* descs, const int* block_map, int slot) {
  const UpdateDesc d = descs[block_map[2 * blockIdx.x]];
  if (!d.stash) return;
  __shared__ float tile[64][65];
  const int kblocks = (d.Coutpad + 63) / 64, cblocks = (d.Cin + 63) / 64;
  int t = block_map[2 * blockIdx.x + 1];
  const int kb = t % kblocks; t /= kblocks;
  const int cb = t % cblocks;
  const int tap = t / cblocks;
  const int ty = threadIdx.x >> 6, tx = threadIdx.x & 63;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int k = kb * 64 + ty * 16 + i, c = cb * 64 + tx;
    tile[ty * 16 + i][tx] = (k < d.Cout && c < d.Cinpad) ? d.master[((size_t)k * d.RS + tap) * d.Cinpad + c] : 0.f;
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int c = cb * 64 + ty * 16 + i, k = kb * 64 + tx;
    if (c < d.Cin && k < d.Coutpad) {
      const size_t o = (size_t)slot * d.stash_slot_elems + ((size_t)c * d.RS + tap) * d.Coutpad + k;
      const float v = tile[tx][ty * 16 + i];
      if (sizeof(T) == 2) ((uint16_t*)d.stash)[o] = f2bf(v);
      else ((float*)d.stash)[o] = v;
    }
  }
}

__global__ void param_permute_kernel(const float* canon, float* internal, int Cout, int Cin, int RS, int Cinpad, int to_internal) {
  const long long total = (long long)Cout * RS * Cinpad + Cout;
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const long long nw = (long long)Cout * RS * Cinpad;
  const long long nwc = (long long)Cout * Cin * RS;
  if (i >= nw) {  // bias
    const long long k = i - nw;
    if (to_internal) internal[i] = canon[nwc + k];
    else ((float*)canon)[nwc + k] = internal[i];
    return;
  }
  const int c = (int)(i % Cinpad);
  const long long r = i / Cinpad;
  const int tap = (int)(r % RS);
  const int k = (int)(r / RS);
  if (c >= Cin) { if (to_internal) internal[i] = 0.f; return; }
  const size_t ci = ((size_t)k * Cin + c) * RS + tap;
  if (to_internal) internal[i] = canon[ci];
  else ((float*)canon)[ci] = internal[i];
}

__global__ void fill_zero_kernel(uint4* p, size_t n16) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) p[i] = make_uint4(0, 0, 0, 0);
}

inline unsigned blocks_for(long long n, int per) { return (unsigned)((n + per - 1) / per); }

}  // namespace

#define DDS_DISPATCH(dt, KERNEL, ...)                  \
  do {                                                 \
    if ((dt) == DT_F32) KERNEL<float> __VA_ARGS__;     \
    else KERNEL<bf16_t> __VA_ARGS__;                   \
  } while (0)

void launch_ingest(int dt, const IngestParams& p, hipStream_t s) {
  const long long total = (long long)p.W * p.B * p.HW * (p.Cpad / dtype_ce(dt));
  const long long n = total > (long long)p.W * p.B ? total : (long long)p.W * p.B;
  DDS_DISPATCH(dt, ingest_kernel, <<<blocks_for(n, 256), 256, 0, s>>>(p));
}

void launch_maxpool_fwd(int dt, const void* x, void* y, int N, int H, int W, int C, hipStream_t s) {
  const long long total = (long long)N * (H / 2) * (W / 2) * (C / dtype_ce(dt));
  DDS_DISPATCH(dt, maxpool_fwd_kernel, <<<blocks_for(total, 256), 256, 0, s>>>((const char*)x, (char*)y, N, H, W, C));
}

void launch_maxpool_bwd(int dt, const void* dy, const void* x, void* dx, int N, int H, int W, int C, int relu_mask,
                        hipStream_t s) {
  const long long total = (long long)N * (H / 2) * (W / 2) * (C / dtype_ce(dt));
  DDS_DISPATCH(dt, maxpool_bwd_kernel,
               <<<blocks_for(total, 256), 256, 0, s>>>((const char*)dy, (const char*)x, (char*)dx, N, H, W, C, relu_mask));
}

void launch_gap_fwd(int dt, const void* x, void* y, int N, int HW, int C, hipStream_t s) {
  const long long total = (long long)N * (C / dtype_ce(dt));
  DDS_DISPATCH(dt, gap_fwd_kernel, <<<blocks_for(total, 128), 128, 0, s>>>((const char*)x, (char*)y, N, HW, C));
}

void launch_gap_bwd(int dt, const void* dy, const void* x, void* dx, int N, int HW, int C, int relu_mask, hipStream_t s) {
  const long long total = (long long)N * HW * (C / dtype_ce(dt));
  DDS_DISPATCH(dt, gap_bwd_kernel,
               <<<blocks_for(total, 256), 256, 0, s>>>((const char*)dy, (const char*)x, (char*)dx, N, HW, C, relu_mask));
}

void launch_softmax_ce(int dt, const float* logits, const int32_t* labels, void* dlogits, float* loss, int W, int B,
                       int classes, int ldl, int ldg, hipStream_t s) {
  DDS_DISPATCH(dt, softmax_ce_kernel, <<<W, 256, 0, s>>>(logits, labels, (char*)dlogits, loss, B, classes, ldl, ldg));
}

void launch_update(int dt, const UpdateDesc* descs, const int* block_map, int total_blocks, int W, float lr, float mu,
                   hipStream_t s) {
  if (total_blocks <= 0) return;
  DDS_DISPATCH(dt, update_kernel, <<<4 * total_blocks, 256, 0, s>>>(descs, block_map, 1.f / (float)W, lr, mu));
}

void launch_recast(int dt, const UpdateDesc* descs, const int* block_map, int total_blocks, hipStream_t s) {
  if (total_blocks <= 0) return;
  DDS_DISPATCH(dt, recast_kernel, <<<total_blocks, 256, 0, s>>>(descs, block_map));
}

void launch_stash(int dt, const UpdateDesc* descs, const int* block_map, int total_blocks, int slot, hipStream_t s) {
  if (total_blocks <= 0) return;
  DDS_DISPATCH(dt, stash_kernel, <<<total_blocks, 256, 0, s>>>(descs, block_map, slot));
}

void launch_gossip_update(int dt, const UpdateDesc* descs, const int* block_map, int total_blocks, const float* P, int W,
                          long long rep_stride, float lr, float mu, hipStream_t s) {
  if (total_blocks <= 0) return;
  DDS_DISPATCH(dt, gossip_update_kernel, <<<total_blocks, 256, 0, s>>>(descs, block_map, P, W, rep_stride, lr, mu));
}

void launch_consensus(const UpdateDesc* descs, const int* block_map, int total_blocks, int W, long long rep_stride,
                      double* out, hipStream_t s) {
  if (total_blocks <= 0) return;
  consensus_kernel<<<total_blocks, 256, 0, s>>>(descs, block_map, W, rep_stride, out);
}

void launch_param_permute(const float* canon, float* internal, int Cout, int Cin, int RS, int Cinpad, int to_internal,
                          hipStream_t s) {
  const long long total = (long long)Cout * RS * Cinpad + Cout;
  param_permute_kernel<<<blocks_for(total, 256), 256, 0, s>>>(canon, internal, Cout, Cin, RS, Cinpad, to_internal);
}

void launch_fill_zero(void* p, size_t bytes, hipStream_t s) {
  const size_t n16 = bytes / 16;
  if (n16 == 0) return;
  size_t blocks = (n16 + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  fill_zero_kernel<<<(unsigned)blocks, 256, 0, s>>>((uint4*)p, n16);
}

}  // namespace dds
