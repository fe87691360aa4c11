// MFMA implicit-GEMM kernels for gfx950: convolution / linear forward and dgrad
// (one kernel, two gather modes) and wgrad with a split pixel reduction.
//
// Both kernels stage K-contiguous operand tiles in LDS ([row][k], 16-byte padded
// rows) and feed v_mfma_f32_32x32x16_bf16 (bf16) or v_mfma_f32_32x32x2_f32 (fp32)
// with one 16-byte LDS read per operand fragment. Lanes 0-31 read the first 16
// bytes of a 32-byte k-step and lanes 32-63 the second, for A and B alike, so the
// pairing of k indices inside an instruction is consistent by construction.
#include "kernels.h"

namespace dds {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;

struct bf16_t { uint16_t v; };

__device__ __forceinline__ float bf2f(uint16_t v) { return __uint_as_float(((uint32_t)v) << 16); }
__device__ __forceinline__ uint16_t f2bf(float f) {  // round to nearest even
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);  // NaN stays NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

template <typename T> __device__ __forceinline__ float load_elem(const void* p, size_t i);
template <> __device__ __forceinline__ float load_elem<float>(const void* p, size_t i) { return ((const float*)p)[i]; }
template <> __device__ __forceinline__ float load_elem<bf16_t>(const void* p, size_t i) { return bf2f(((const uint16_t*)p)[i]); }
template <typename T> __device__ __forceinline__ void store_elem(void* p, size_t i, float v);
template <> __device__ __forceinline__ void store_elem<float>(void* p, size_t i, float v) { ((float*)p)[i] = v; }
template <> __device__ __forceinline__ void store_elem<bf16_t>(void* p, size_t i, float v) { ((uint16_t*)p)[i] = f2bf(v); }

template <typename T> __device__ __forceinline__ void mfma16B(const uint4& a, const uint4& b, f32x16_t& c);
template <> __device__ __forceinline__ void mfma16B<bf16_t>(const uint4& a, const uint4& b, f32x16_t& c) {
  c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}
template <> __device__ __forceinline__ void mfma16B<float>(const uint4& a, const uint4& b, f32x16_t& c) {
  c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), c, 0, 0, 0);
}

// One BKB-byte-deep step of a WM x WN wave tile. As / Bs point at the wave's first row.
template <typename T, int WM, int WN, int BKB>
__device__ __forceinline__ void mma_step(const char* As, const char* Bs, int lane, f32x16_t (&acc)[WM / 32][WN / 32]) {
  constexpr int LDK = BKB + 16;
  const int row = lane & 31, half = lane >> 5;
#pragma unroll
  for (int ks = 0; ks < BKB / 32; ++ks) {
    uint4 a[WM / 32], b[WN / 32];
#pragma unroll
    for (int i = 0; i < WM / 32; ++i) a[i] = *(const uint4*)(As + (i * 32 + row) * LDK + ks * 32 + half * 16);
#pragma unroll
    for (int j = 0; j < WN / 32; ++j) b[j] = *(const uint4*)(Bs + (j * 32 + row) * LDK + ks * 32 + half * 16);
#pragma unroll
    for (int i = 0; i < WM / 32; ++i)
#pragma unroll
      for (int j = 0; j < WN / 32; ++j) mfma16B<T>(a[i], b[j], acc[i][j]);
  }
}

// ------------------------------------------------------------------ forward / dgrad
template <typename T, int BM, int BN, int WM, int WN, int BKB, bool DGRAD>
__global__ __launch_bounds__(256) void conv_gemm_kernel(ConvParams p) {
  constexpr int ES = sizeof(T);
  constexpr int CE = 16 / ES;     // elements per 16-byte chunk
  constexpr int BKE = BKB / ES;   // k elements per tile
  constexpr int CPR = BKB / 16;   // chunks per tile row
  constexpr int LDK = BKB + 16;
  constexpr int ROWS = 256 / CPR; // rows covered by one pass of all threads
  constexpr int AP = BM / ROWS, BP = BN / ROWS;
  static_assert((BM / WM) * (BN / WN) == 4, "four waves");
  static_assert(AP >= 1 && BP >= 1, "tile too small for the loader");
  __shared__ __align__(16) char smem[2 * (BM + BN) * LDK];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_m = wave % (BM / WM), wave_n = wave / (BM / WM);
  const int m0 = blockIdx.x * BM, n0 = blockIdx.y * BN;
  const int chunk = tid % CPR, rbase = tid / CPR;
  const int sh = p.stride - 1;  // stride is 1 or 2

  int a_h[AP], a_w[AP];
  const char* a_base[AP];
  bool a_ok[AP];
  const int HoWo = p.Ho * p.Wo;
#pragma unroll
  for (int i = 0; i < AP; ++i) {
    int m = m0 + rbase + i * ROWS;
    a_ok[i] = m < p.M;
    int mm = a_ok[i] ? m : 0;
    int img = mm / HoWo;
    int rem = mm - img * HoWo;
    int oh = rem / p.Wo, ow = rem - oh * p.Wo;
    if (DGRAD) { a_h[i] = oh + p.pad; a_w[i] = ow + p.pad; }
    else { a_h[i] = oh * p.stride - p.pad; a_w[i] = ow * p.stride - p.pad; }
    a_base[i] = (const char*)p.x + (size_t)img * p.H * p.W * p.Cx * ES;
  }
  const char* b_base[BP];
  bool b_ok[BP];
#pragma unroll
  for (int i = 0; i < BP; ++i) {
    int n = n0 + rbase + i * ROWS;
    b_ok[i] = n < p.Nout;
    b_base[i] = (const char*)p.w + (size_t)(b_ok[i] ? n : 0) * p.Ktot * ES;
  }
  // position of this thread's chunk in (tap, channel) space
  int kc = chunk * CE, kr = 0, ks = 0, kflat = chunk * CE;
  while (kc >= p.Cx) { kc -= p.Cx; if (++ks == p.S) { ks = 0; ++kr; } }

  uint4 ra[AP], rb[BP];
  auto load_global = [&]() {
#pragma unroll
    for (int i = 0; i < AP; ++i) {
      uint4 v = make_uint4(0, 0, 0, 0);
      if (a_ok[i] && kr < p.R) {
        int hi, wi;
        bool ok;
        if (DGRAD) {
          int nh = a_h[i] - kr, nw = a_w[i] - ks;
          ok = nh >= 0 && nw >= 0 && ((nh | nw) & sh) == 0;
          hi = nh >> sh; wi = nw >> sh;
          ok = ok && hi < p.H && wi < p.W;
        } else {
          hi = a_h[i] + kr; wi = a_w[i] + ks;
          ok = (unsigned)hi < (unsigned)p.H && (unsigned)wi < (unsigned)p.W;
        }
        if (ok) v = *(const uint4*)(a_base[i] + ((size_t)(hi * p.W + wi) * p.Cx + kc) * ES);
      }
      ra[i] = v;
    }
#pragma unroll
    for (int i = 0; i < BP; ++i) {
      uint4 v = make_uint4(0, 0, 0, 0);
      if (b_ok[i] && kflat < p.Ktot) v = *(const uint4*)(b_base[i] + (size_t)kflat * ES);
      rb[i] = v;
    }
    kflat += BKE;
    kc += BKE;
    while (kc >= p.Cx) { kc -= p.Cx; if (++ks == p.S) { ks = 0; ++kr; } }
  };
  auto store_lds = [&](int buf) {
    char* As = smem + buf * (BM + BN) * LDK;
    char* Bs = As + BM * LDK;
#pragma unroll
    for (int i = 0; i < AP; ++i) *(uint4*)(As + (rbase + i * ROWS) * LDK + chunk * 16) = ra[i];
#pragma unroll
    for (int i = 0; i < BP; ++i) *(uint4*)(Bs + (rbase + i * ROWS) * LDK + chunk * 16) = rb[i];
  };

  f32x16_t acc[WM / 32][WN / 32];
#pragma unroll
  for (int i = 0; i < WM / 32; ++i)
#pragma unroll
    for (int j = 0; j < WN / 32; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  const int nk = (p.Ktot + BKE - 1) / BKE;
  load_global();
  store_lds(0);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < nk) load_global();
    const char* As = smem + buf * (BM + BN) * LDK + wave_m * WM * LDK;
    const char* Bs = smem + buf * (BM + BN) * LDK + BM * LDK + wave_n * WN * LDK;
    mma_step<T, WM, WN, BKB>(As, Bs, lane, acc);
    if (kt + 1 < nk) store_lds(buf ^ 1);
    __syncthreads();
  }

  // epilogue: lane holds column n = lane%32 and rows 8*(e/4) + 4*(lane/32) + e%4 of each 32x32 tile
#pragma unroll
  for (int j = 0; j < WN / 32; ++j) {
    const int n = n0 + wave_n * WN + j * 32 + (lane & 31);
    if (n >= p.ldy) continue;
    const float bias = (p.bias != nullptr && n < p.Nout) ? p.bias[n] : 0.f;
#pragma unroll
    for (int i = 0; i < WM / 32; ++i) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int m = m0 + wave_m * WM + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
        if (m >= p.M) continue;
        const size_t o = (size_t)m * p.ldy + n;
        float v = p.alpha * (acc[i][j][e] + bias);
        if (p.res) v += load_elem<T>(p.res, o);
        if (p.relu) v = v > 0.f ? v : 0.f;
        if (p.mask) v = load_elem<T>(p.mask, o) > 0.f ? v : 0.f;
        if (p.out_f32) ((float*)p.y)[o] = v;
        else store_elem<T>(p.y, o, v);
      }
    }
  }
}

// ------------------------------------------------------------------ wgrad
// 16-byte chunks loaded along the channel axis for CE consecutive pixels are
// transposed in registers so that LDS rows run along the pixel (reduction) axis.
template <typename T> __device__ __forceinline__ void transpose_chunks(const uint4* in, uint4* out);
template <> __device__ __forceinline__ void transpose_chunks<float>(const uint4* in, uint4* out) {
  out[0] = make_uint4(in[0].x, in[1].x, in[2].x, in[3].x);
  out[1] = make_uint4(in[0].y, in[1].y, in[2].y, in[3].y);
  out[2] = make_uint4(in[0].z, in[1].z, in[2].z, in[3].z);
  out[3] = make_uint4(in[0].w, in[1].w, in[2].w, in[3].w);
}
__device__ __forceinline__ uint32_t pack_lo(uint32_t a, uint32_t b) { return (a & 0xffffu) | (b << 16); }
__device__ __forceinline__ uint32_t pack_hi(uint32_t a, uint32_t b) { return (a >> 16) | (b & 0xffff0000u); }
template <> __device__ __forceinline__ void transpose_chunks<bf16_t>(const uint4* in, uint4* out) {
  // out[e] = element e of in[0..7]
  out[0] = make_uint4(pack_lo(in[0].x, in[1].x), pack_lo(in[2].x, in[3].x), pack_lo(in[4].x, in[5].x), pack_lo(in[6].x, in[7].x));
  out[1] = make_uint4(pack_hi(in[0].x, in[1].x), pack_hi(in[2].x, in[3].x), pack_hi(in[4].x, in[5].x), pack_hi(in[6].x, in[7].x));
  out[2] = make_uint4(pack_lo(in[0].y, in[1].y), pack_lo(in[2].y, in[3].y), pack_lo(in[4].y, in[5].y), pack_lo(in[6].y, in[7].y));
  out[3] = make_uint4(pack_hi(in[0].y, in[1].y), pack_hi(in[2].y, in[3].y), pack_hi(in[4].y, in[5].y), pack_hi(in[6].y, in[7].y));
  out[4] = make_uint4(pack_lo(in[0].z, in[1].z), pack_lo(in[2].z, in[3].z), pack_lo(in[4].z, in[5].z), pack_lo(in[6].z, in[7].z));
  out[5] = make_uint4(pack_hi(in[0].z, in[1].z), pack_hi(in[2].z, in[3].z), pack_hi(in[4].z, in[5].z), pack_hi(in[6].z, in[7].z));
  out[6] = make_uint4(pack_lo(in[0].w, in[1].w), pack_lo(in[2].w, in[3].w), pack_lo(in[4].w, in[5].w), pack_lo(in[6].w, in[7].w));
  out[7] = make_uint4(pack_hi(in[0].w, in[1].w), pack_hi(in[2].w, in[3].w), pack_hi(in[4].w, in[5].w), pack_hi(in[6].w, in[7].w));
}
template <typename T> __device__ __forceinline__ uint4 one_chunk();
template <> __device__ __forceinline__ uint4 one_chunk<float>() { return make_uint4(0x3f800000u, 0, 0, 0); }
template <> __device__ __forceinline__ uint4 one_chunk<bf16_t>() { return make_uint4(0x3f80u, 0, 0, 0); }

template <typename T, int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(256) void wgrad_gemm_kernel(WgradParams p) {
  constexpr int ES = sizeof(T);
  constexpr int CE = 16 / ES;
  constexpr int BKB = 128;
  constexpr int BKE = BKB / ES;    // pixels per tile
  constexpr int KG = BKE / CE;     // pixel groups per tile (each CE pixels)
  constexpr int LDK = BKB + 16;
  constexpr int A_BLOCKS = (BM / CE) * KG, B_BLOCKS = (BN / CE) * KG;
  constexpr int NBLK = (A_BLOCKS + B_BLOCKS + 255) / 256;  // blocks per thread
  static_assert((BM / WM) * (BN / WN) == 4, "four waves");
  __shared__ __align__(16) char smem[2 * (BM + BN) * LDK];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_m = wave % (BM / WM), wave_n = wave / (BM / WM);
  const int m0 = blockIdx.x * BM, n0 = blockIdx.y * BN;
  const int z = blockIdx.z;
  const int pz0 = z * p.pix_per_split;
  const int pz1 = min(p.P, pz0 + p.pix_per_split);
  const int HoWo = p.Ho * p.Wo;

  // static description of this thread's blocks
  bool isA[NBLK], okc[NBLK], isBias[NBLK];
  int row0[NBLK], kg[NBLK], bh[NBLK], bw[NBLK], coff[NBLK];
#pragma unroll
  for (int b = 0; b < NBLK; ++b) {
    int id = tid + b * 256;
    isA[b] = id < A_BLOCKS;
    isBias[b] = false;
    if (id >= A_BLOCKS + B_BLOCKS) {  // spare loader slot: contributes nothing
      okc[b] = false;
      row0[b] = -1;
      kg[b] = bh[b] = bw[b] = coff[b] = 0;
    } else if (isA[b]) {
      int mc = id % (BM / CE);
      kg[b] = id / (BM / CE);
      row0[b] = mc * CE;
      int m = m0 + mc * CE;
      okc[b] = m < p.ldy;
      coff[b] = m;
      bh[b] = bw[b] = 0;
    } else {
      id -= A_BLOCKS;
      int nc = id % (BN / CE);
      kg[b] = id / (BN / CE);
      row0[b] = BM + nc * CE;
      int n = n0 + nc * CE;
      okc[b] = n < p.NK;
      isBias[b] = n == p.NK;
      int nn = okc[b] ? n : 0;
      int tap = nn / p.Cx;
      coff[b] = nn - tap * p.Cx;
      int r = tap / p.S;
      bh[b] = r - p.pad;
      bw[b] = (tap - r * p.S) - p.pad;
    }
  }

  uint4 regs[NBLK][CE];
  auto load_global = [&](int ptile) {
#pragma unroll
    for (int b = 0; b < NBLK; ++b) {
#pragma unroll
      for (int g = 0; g < CE; ++g) {
        const int pix = ptile + kg[b] * CE + g;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (pix < pz1) {
          if (isA[b]) {
            if (okc[b]) v = *(const uint4*)((const char*)p.dy + ((size_t)pix * p.ldy + coff[b]) * ES);
          } else if (okc[b]) {
            int img = pix / HoWo;
            int rem = pix - img * HoWo;
            int oh = rem / p.Wo, ow = rem - oh * p.Wo;
            int hi = oh * p.stride + bh[b], wi = ow * p.stride + bw[b];
            if ((unsigned)hi < (unsigned)p.H && (unsigned)wi < (unsigned)p.W)
              v = *(const uint4*)((const char*)p.x + (((size_t)img * p.H + hi) * p.W + wi) * p.Cx * ES + (size_t)coff[b] * ES);
          } else if (isBias[b]) {
            v = one_chunk<T>();
          }
        }
        regs[b][g] = v;
      }
    }
  };
  auto store_lds = [&](int buf) {
    char* base = smem + buf * (BM + BN) * LDK;
#pragma unroll
    for (int b = 0; b < NBLK; ++b) {
      if (row0[b] < 0) continue;
      uint4 t[CE];
      transpose_chunks<T>(regs[b], t);
#pragma unroll
      for (int e = 0; e < CE; ++e) *(uint4*)(base + (row0[b] + e) * LDK + kg[b] * 16) = t[e];
    }
  };

  f32x16_t acc[WM / 32][WN / 32];
#pragma unroll
  for (int i = 0; i < WM / 32; ++i)
#pragma unroll
    for (int j = 0; j < WN / 32; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  const int nk = (pz1 - pz0 + BKE - 1) / BKE;
  if (nk > 0) {
    load_global(pz0);
    store_lds(0);
  }
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < nk) load_global(pz0 + (kt + 1) * BKE);
    const char* As = smem + buf * (BM + BN) * LDK + wave_m * WM * LDK;
    const char* Bs = smem + buf * (BM + BN) * LDK + BM * LDK + wave_n * WN * LDK;
    mma_step<T, WM, WN, BKB>(As, Bs, lane, acc);
    if (kt + 1 < nk) store_lds(buf ^ 1);
    __syncthreads();
  }

  float* out = p.partial + (size_t)z * p.Pl;
#pragma unroll
  for (int j = 0; j < WN / 32; ++j) {
    const int n = n0 + wave_n * WN + j * 32 + (lane & 31);
    if (n > p.NK) continue;
#pragma unroll
    for (int i = 0; i < WM / 32; ++i) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int m = m0 + wave_m * WM + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
        if (m >= p.Mout) continue;
        const float v = p.alpha * acc[i][j][e];
        if (n < p.NK) out[(size_t)m * p.NK + n] = v;
        else out[(size_t)p.Mout * p.NK + m] = v;
      }
    }
  }
}

inline int cdiv(int a, int b) { return (a + b - 1) / b; }

template <typename T>
void launch_conv_t(const ConvParams& p, hipStream_t s) {
  constexpr int BKB = 64;
  if (p.ldy <= 64) {
    dim3 grid(cdiv(p.M, 256), cdiv(p.ldy, 64));
    if (p.dgrad) conv_gemm_kernel<T, 256, 64, 64, 64, BKB, true><<<grid, 256, 0, s>>>(p);
    else conv_gemm_kernel<T, 256, 64, 64, 64, BKB, false><<<grid, 256, 0, s>>>(p);
  } else {
    dim3 grid(cdiv(p.M, 128), cdiv(p.ldy, 128));
    if (p.dgrad) conv_gemm_kernel<T, 128, 128, 64, 64, BKB, true><<<grid, 256, 0, s>>>(p);
    else conv_gemm_kernel<T, 128, 128, 64, 64, BKB, false><<<grid, 256, 0, s>>>(p);
  }
}

template <typename T>
void launch_wgrad_t(const WgradParams& p, hipStream_t s) {
  constexpr int CE = 16 / sizeof(T);
  if (p.Mout <= 64) {
    dim3 grid(cdiv(p.Mout, 64), cdiv(p.NK + CE, 256), p.nsplit);
    wgrad_gemm_kernel<T, 64, 256, 64, 64><<<grid, 256, 0, s>>>(p);
  } else {
    dim3 grid(cdiv(p.Mout, 128), cdiv(p.NK + CE, 128), p.nsplit);
    wgrad_gemm_kernel<T, 128, 128, 64, 64><<<grid, 256, 0, s>>>(p);
  }
}

}  // namespace

void launch_conv(int dt, const ConvParams& p, hipStream_t s) {
  if (dt == DT_F32) launch_conv_t<float>(p, s);
  else launch_conv_t<bf16_t>(p, s);
}

void launch_wgrad(int dt, const WgradParams& p, hipStream_t s) {
  if (dt == DT_F32) launch_wgrad_t<float>(p, s);
  else launch_wgrad_t<bf16_t>(p, s);
}

int wgrad_choose_split(int dt, int Mout, int NK, int P, int W) {
  const int ce = dtype_ce(dt);
  const int bke = 128 / dtype_size(dt);
  int tiles = (Mout <= 64) ? cdiv(Mout, 64) * cdiv(NK + ce, 256) : cdiv(Mout, 128) * cdiv(NK + ce, 128);
  const int per_replica = P / W;  // pixels of one replica's mini-batch
  int q = cdiv(1024, tiles * W);  // aim at ~1024 workgroups
  int qmax = per_replica / (2 * bke);  // at least two k-tiles per split
  if (qmax < 1) qmax = 1;
  if (q > qmax) q = qmax;
  if (q < 1) q = 1;
  while (q > 1 && per_replica % q != 0) --q;  // splits never straddle replicas
  return W * q;
}

}  // namespace dds
