// MFMA implicit-GEMM kernels for gfx950: convolution / linear forward and dgrad
// (one kernel, two gather modes) and wgrad with a split pixel reduction.
//
// Both kernels stage K-contiguous operand tiles in LDS ([row][k], 16-byte padded
// rows) and feed v_mfma_f32_32x32x16_bf16 (bf16) or v_mfma_f32_32x32x2_f32 (fp32)
// with one 16-byte LDS read per operand fragment. Lanes 0-31 read the first 16
// bytes of a 32-byte k-step and lanes 32-63 the second, for A and B alike, so the
// pairing of k indices inside an instruction is consistent by construction.
#include <cstdlib>

#include "kernels.h"

namespace dds {
namespace {

#define DDS_LDS_AS __attribute__((address_space(3)))

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

__device__ __forceinline__ uint4 keep_if(bool ok, const uint4& v) {
  return make_uint4(ok ? v.x : 0u, ok ? v.y : 0u, ok ? v.z : 0u, ok ? v.w : 0u);
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

// LDS loads through an explicit address-space pointer (HIP's vector classes cannot be
// referenced through one, so native vector types carry the bits)
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
template <typename R> __device__ __forceinline__ R lds_load(const char DDS_LDS_AS* p);
template <> __device__ __forceinline__ uint4 lds_load<uint4>(const char DDS_LDS_AS* p) {
  const u32x4_t v = *(const u32x4_t DDS_LDS_AS*)p;
  return make_uint4(v.x, v.y, v.z, v.w);
}
template <> __device__ __forceinline__ uint2 lds_load<uint2>(const char DDS_LDS_AS* p) {
  const u32x2_t v = *(const u32x2_t DDS_LDS_AS*)p;
  return make_uint2(v.x, v.y);
}

// Four consecutive output channels of one pixel: v = alpha*(acc+bias) (+res) (relu) (mask),
// moved with one 8-byte (bf16) or 16-byte (fp32) access per operand. n is a multiple of 4.
template <typename T> __device__ __forceinline__ void load4(const void* p, size_t i, float* v);
template <> __device__ __forceinline__ void load4<float>(const void* p, size_t i, float* v) {
  const float4 t = *(const float4*)((const float*)p + i);
  v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
}
template <> __device__ __forceinline__ void load4<bf16_t>(const void* p, size_t i, float* v) {
  const uint2 t = *(const uint2*)((const uint16_t*)p + i);
  v[0] = __uint_as_float(t.x << 16); v[1] = __uint_as_float(t.x & 0xffff0000u);
  v[2] = __uint_as_float(t.y << 16); v[3] = __uint_as_float(t.y & 0xffff0000u);
}
template <typename T> __device__ __forceinline__ void store4(void* p, size_t i, const float* v);
template <> __device__ __forceinline__ void store4<float>(void* p, size_t i, const float* v) {
  *(float4*)((float*)p + i) = make_float4(v[0], v[1], v[2], v[3]);
}
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
// two floats -> packed bf16 pair, round to nearest even (v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
template <> __device__ __forceinline__ void store4<bf16_t>(void* p, size_t i, const float* v) {
  uint2 t;
  t.x = pack_bf16(v[0], v[1]);
  t.y = pack_bf16(v[2], v[3]);
  *(uint2*)((uint16_t*)p + i) = t;
}

// Epilogue of one 32-pixel tile column of a wave: this lane owns pixel `pix` and, for each
// of the NJ channel tiles, four groups of 4 consecutive channels starting at
// nb + 32*j + 8*g. All residual / mask reads are issued up front from clamped addresses
// (no branch around a load, so none of them is waited for one by one), then
// v = alpha*(acc+bias) (+res) (relu) (mask) is formed and stored with predicated vector stores.
template <typename T> struct Raw4;
template <> struct Raw4<float> { typedef uint4 type; };
template <> struct Raw4<bf16_t> { typedef uint2 type; };
__device__ __forceinline__ void unpack4(const uint4& t, float* v) {
  v[0] = __uint_as_float(t.x); v[1] = __uint_as_float(t.y); v[2] = __uint_as_float(t.z); v[3] = __uint_as_float(t.w);
}
__device__ __forceinline__ void unpack4(const uint2& t, float* v) {
  v[0] = __uint_as_float(t.x << 16); v[1] = __uint_as_float(t.x & 0xffff0000u);
  v[2] = __uint_as_float(t.y << 16); v[3] = __uint_as_float(t.y & 0xffff0000u);
}

// x > 0 decided on the stored bits (no conversion): fp32 as is; a packed bf16 pair w holds
// lo in bits 0-15 and hi in bits 16-31: hi > 0 <=> (int)w >= 0x10000, lo > 0 <=> (int)(w << 16) >= 0x10000
__device__ __forceinline__ void positive4(const uint4& t, bool* pos) {
  pos[0] = __uint_as_float(t.x) > 0.f; pos[1] = __uint_as_float(t.y) > 0.f;
  pos[2] = __uint_as_float(t.z) > 0.f; pos[3] = __uint_as_float(t.w) > 0.f;
}
__device__ __forceinline__ void positive4(const uint2& t, bool* pos) {
  pos[0] = (int)(t.x << 16) >= 0x10000; pos[1] = (int)t.x >= 0x10000;
  pos[2] = (int)(t.y << 16) >= 0x10000; pos[3] = (int)t.y >= 0x10000;
}

// Four bytes of a sign plane row: channels cbase .. cbase+31 of pixel pix (zero where the row ends earlier).
__device__ __forceinline__ uint32_t load_bits32(const void* bits, size_t pix, int ldy, int cbase, bool valid) {
  if (!valid || cbase >= ldy) return 0u;
  const uint8_t* row = (const uint8_t*)bits + pix * (size_t)(ldy >> 3) + (cbase >> 3);
  if ((ldy & 31) == 0) return *(const uint32_t*)row;
  uint32_t w = 0;
  for (int b = 0; b < 4 && cbase + 8 * b < ldy; ++b) w |= (uint32_t)row[b] << (8 * b);
  return w;
}
__device__ __forceinline__ void store_bits32(void* bits, size_t pix, int ldy, int cbase, uint32_t w) {
  if (cbase >= ldy) return;
  uint8_t* row = (uint8_t*)bits + pix * (size_t)(ldy >> 3) + (cbase >> 3);
  if ((ldy & 31) == 0) { *(uint32_t*)row = w; return; }
  for (int b = 0; b < 4 && cbase + 8 * b < ldy; ++b) row[b] = (uint8_t)(w >> (8 * b));
}
// nibble i of x -> bits [8i, 8i+4)
__device__ __forceinline__ uint32_t spread_nibbles(uint32_t x) {
  return (x & 0xfu) | ((x & 0xf0u) << 4) | ((x & 0xf00u) << 8) | ((x & 0xf000u) << 12);
}

// bias values of this lane's channel groups (zero past Nout), read once per kernel
template <int NJ>
__device__ __forceinline__ void load_bias_groups(const ConvParams& p, int nb, float (&bias)[NJ][4][4]) {
#pragma unroll
  for (int j = 0; j < NJ; ++j)
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int n = nb + 32 * j + 8 * g + q;
        float b = 0.f;
        if (p.bias) b = p.bias[n < p.Nout ? n : 0];
        bias[j][g][q] = n < p.Nout ? b : 0.f;
      }
}

// res_off / mask_off >= 0: the tile's residual / mask values were staged in LDS as
// [tile row][row_bytes] with 16-byte column c of row m stored at column c ^ (m & (ncol-1));
// tile_row is this lane's row, ncol = row_bytes / 16, nloc0 the lane's first channel inside the tile.
// The function is laid out in phases (gather operands, arithmetic, store, sign plane) with one
// uniform branch per phase at most: every option inside the arithmetic is a select, not a
// branch, because each branch costs the compiler's conservative waits at its join.
template <typename T, int NJ, int NI>
__device__ __forceinline__ void epilogue_tile(const ConvParams& p, const f32x16_t (&acc)[NJ][NI], int i, bool valid,
                                              size_t pix, int nb, const float (&bias)[NJ][4][4],
                                              const char DDS_LDS_AS* lds = nullptr, int res_off = -1, int mask_off = -1,
                                              int tile_row = 0, int row_bytes = 0, int nloc0 = 0, int ab_off = -1,
                                              const uint32_t* mbits = nullptr, int out_off = -1) {
  typedef typename Raw4<T>::type raw_t;
  static_assert(NJ <= 2, "the sign words hold 8 nibbles");
  const int half = (threadIdx.x >> 5) & 1;   // which 4 channels of every 8 this lane holds
  const int nwave0 = nb - 4 * half;           // first channel of the wave's span
  const int ncolm = (row_bytes >> 4) - 1;
  // explicit LDS address space: a generic pointer would turn these into flat loads, which
  // also count as vector-memory operations and would wait for every earlier global store
  auto lds_at = [&](int base_off, int j, int g) {
    const int bytecol = (nloc0 + 32 * j + 8 * g) * (int)sizeof(T);
    return (char DDS_LDS_AS*)lds + base_off + tile_row * row_bytes + ((((bytecol >> 4) ^ tile_row) & ncolm) << 4) + (bytecol & 15);
  };
  size_t o[NJ][4];
  bool ok[NJ][4];
#pragma unroll
  for (int j = 0; j < NJ; ++j)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int n = nb + 32 * j + 8 * g;
      ok[j][g] = valid && n < p.ldy;
      o[j][g] = ok[j][g] ? pix * p.ldy + n : 0;
    }

  uint32_t signs = 0;  // nibble 4 j + g: this lane's four outputs of group (j, g) that are > 0
  const float lower = p.relu ? 0.f : -__builtin_inff();
#pragma unroll
  for (int j = 0; j < NJ; ++j) {  // one 32-channel tile at a time keeps the temporaries at 16 registers each
    // ---- gather: alpha * bias, residual, mask (defaults: 0, 0, keep everything)
    float ab[4][4], rs[4][4];
    uint32_t keep = 0xffffffffu;  // bit 8 g + 4 half + q: output (g, q) survives the mask
    if (ab_off >= 0) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const uint4 t = lds_load<uint4>(lds + ab_off + (nloc0 + 32 * j + 8 * g) * 4);
        ab[g][0] = __uint_as_float(t.x); ab[g][1] = __uint_as_float(t.y);
        ab[g][2] = __uint_as_float(t.z); ab[g][3] = __uint_as_float(t.w);
      }
    } else {
#pragma unroll
      for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int q = 0; q < 4; ++q) ab[g][q] = p.alpha * bias[j][g][q];
    }
    if (res_off >= 0) {
#pragma unroll
      for (int g = 0; g < 4; ++g) unpack4(lds_load<raw_t>(lds_at(res_off, j, g)), rs[g]);
    } else if (p.res) {
      raw_t r[4];
#pragma unroll
      for (int g = 0; g < 4; ++g) r[g] = *(const raw_t*)((const T*)p.res + o[j][g]);
#pragma unroll
      for (int g = 0; g < 4; ++g) unpack4(r[g], rs[g]);
    } else {
#pragma unroll
      for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int q = 0; q < 4; ++q) rs[g][q] = 0.f;
    }
    if (p.maskbits) {
      keep = mbits ? mbits[j] : load_bits32(p.maskbits, pix, p.ldy, nwave0 + 32 * j, valid);
    } else if (p.mask) {
      raw_t mk[4];
#pragma unroll
      for (int g = 0; g < 4; ++g)
        mk[g] = mask_off >= 0 ? lds_load<raw_t>(lds_at(mask_off, j, g)) : *(const raw_t*)((const T*)p.mask + o[j][g]);
      keep = 0;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        bool pos[4];
        positive4(mk[g], pos);
#pragma unroll
        for (int q = 0; q < 4; ++q) keep |= (pos[q] ? 1u : 0u) << (8 * g + 4 * half + q);
      }
    }

    // ---- arithmetic: v = alpha * acc + alpha * bias + res, clamp below at 0 (ReLU) or -inf, apply the mask.
    // The optional parts (residual, mask, sign bits) sit behind wave-uniform branches that hold arithmetic only:
    // the epilogue's vector instructions compete with the MFMAs of the workgroup that shares the CU, and a
    // launch that needs none of them runs 5 instead of 12 instructions per output.
    float v[4][4];
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
      for (int q = 0; q < 4; ++q) v[g][q] = fmaf(p.alpha, acc[j][i][4 * g + q], ab[g][q]);
    if (res_off >= 0 || p.res) {
#pragma unroll
      for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int q = 0; q < 4; ++q) v[g][q] += rs[g][q];
    }
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
      for (int q = 0; q < 4; ++q) v[g][q] = __builtin_amdgcn_fmed3f(v[g][q], lower, __builtin_inff());  // one instruction; NaN -> lower
    if (p.maskbits || p.mask) {
#pragma unroll
      for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int q = 0; q < 4; ++q)  // bit -> 0 / all ones, then and
          v[g][q] = __uint_as_float(__float_as_uint(v[g][q]) & (uint32_t)__builtin_amdgcn_sbfe((int)keep, 8 * g + 4 * half + q, 1));
    }
    if (p.bits_out) {
#pragma unroll
      for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int q = 0; q < 4; ++q) signs |= (v[g][q] > 0.f ? 1u : 0u) << (4 * (4 * j + g) + q);
    }

    // ---- store: into the LDS output tile (same layout as the staged residual tile, possibly the very
    // same bytes: this lane has read its residual values from them already; the workgroup writes the
    // tile out afterwards in whole rows), or straight to global memory
    if (out_off >= 0) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        if (sizeof(T) == 2) {
          u32x2_t t = {pack_bf16(v[g][0], v[g][1]), pack_bf16(v[g][2], v[g][3])};
          *(u32x2_t DDS_LDS_AS*)(lds_at(out_off, j, g)) = t;
        } else {
          u32x4_t t = {__float_as_uint(v[g][0]), __float_as_uint(v[g][1]), __float_as_uint(v[g][2]), __float_as_uint(v[g][3])};
          *(u32x4_t DDS_LDS_AS*)(lds_at(out_off, j, g)) = t;
        }
      }
    } else if (p.out_f32) {
#pragma unroll
      for (int g = 0; g < 4; ++g)
        if (ok[j][g]) store4<float>(p.y, o[j][g], v[g]);
    } else {
#pragma unroll
      for (int g = 0; g < 4; ++g)
        if (ok[j][g]) store4<T>(p.y, o[j][g], v[g]);
    }
  }

  // ---- sign plane of the stored values
  if (p.bits_out) {
    // the other half of the wave holds the other four channels of every byte
    const uint32_t other = (uint32_t)__shfl_xor((int)signs, 32, 64);
    const uint32_t lo = half ? other : signs, hi = half ? signs : other;
    // half h writes word j = h (both halves hold all nibbles now); with NJ == 1 only half 0 writes
    const int jw = half;
    if (jw < NJ && valid) {
      const uint32_t w = spread_nibbles((lo >> (16 * jw)) & 0xffffu) | (spread_nibbles((hi >> (16 * jw)) & 0xffffu) << 4);
      store_bits32(p.bits_out, pix, p.ldy, nwave0 + 32 * jw, w);
    }
  }
}

// ------------------------------------------------------------------ forward / dgrad
// S2 (dgrad of a stride-2 convolution whose channel count is a multiple of the k-tile): the
// output pixels are dealt to workgroups by parity class (h % 2, w % 2), blockIdx.x =
// class * tiles_per_class + tile. A pixel of class (ch, cw) only receives taps r = ch + pad,
// s = cw + pad (mod 2), so a workgroup walks just those taps: on average 2.25 of the 9 taps
// of a 3x3 kernel, and 1 class in 4 has any tap at all for a 1x1 kernel.
template <typename T, int BM, int BN, int WM, int WN, int BKB, bool DGRAD, bool S2 = false>
__global__ __launch_bounds__(256, 2) void conv_gemm_kernel(ConvParams p_, int tiles_per_class) {
  ConvParams p = p_;
  constexpr int ES = sizeof(T);
  constexpr int CE = 16 / ES;     // elements per 16-byte chunk
  constexpr int BKE = BKB / ES;   // k elements per tile
  constexpr int CPR = BKB / 16;   // chunks per tile row
  constexpr int LDK = BKB + 16;
  constexpr int ROWS = 256 / CPR; // rows covered by one pass of all threads
  // loader passes over the A and B tiles; a B tile of fewer rows than one pass (BN < ROWS) leaves the
  // threads past its last row idle (their loads read row 0 and are not stored)
  constexpr int AP = BM / ROWS, BP = BN >= ROWS ? BN / ROWS : 1;
  static_assert((BM / WM) * (BN / WN) == 4, "four waves");
  static_assert(AP >= 1, "tile too small for the loader");
  __shared__ __align__(16) char smem[2 * (BM + BN) * LDK];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_m = wave % (BM / WM), wave_n = wave / (BM / WM);
  const int cls = S2 ? blockIdx.x / tiles_per_class : 0;
  const int ch = cls >> 1, cw = cls & 1;
  const int Hc = (p.Ho - ch + 1) >> 1, Wc = (p.Wo - cw + 1) >> 1;  // pixels of this class per image column / row
  const int Mc = S2 ? p.Nimg * Hc * Wc : p.M;
  const int m0 = (S2 ? blockIdx.x - cls * tiles_per_class : blockIdx.x) * BM, n0 = blockIdx.y * BN;
  if (p.nrep > 1) {  // the launcher made sure that a tile never straddles two data-groups
    const int rows_per_rep = Mc / p.nrep;
    const int r = min(m0 / rows_per_rep, p.nrep - 1);
    p.w = (const char*)p.w + (size_t)r * p.w_rep;
    if (p.bias) p.bias += (size_t)r * p.bias_rep;
    if (p.w2) p.w2 = (const char*)p.w2 + (size_t)r * p.w2_rep;
  }
  const int chunk = tid % CPR, rbase = tid / CPR;
  const int sh = p.stride - 1;  // stride is 1 or 2
  // row of the tile -> output pixel (image, oh, ow) and its flat index
  auto row_pixel = [&](int m, int& img, int& oh, int& ow) {
    if (S2) {
      const int HW = Hc * Wc;
      img = m / HW;
      const int rem = m - img * HW;
      const int h2 = rem / Wc;
      oh = 2 * h2 + ch;
      ow = 2 * (rem - h2 * Wc) + cw;
    } else {
      const int HoWo = p.Ho * p.Wo;
      img = m / HoWo;
      const int rem = m - img * HoWo;
      oh = rem / p.Wo;
      ow = rem - oh * p.Wo;
    }
  };

  int a_h[AP], a_w[AP], a_img[AP];
  const char* a_base[AP];
  bool a_ok[AP];
#pragma unroll
  for (int i = 0; i < AP; ++i) {
    int m = m0 + rbase + i * ROWS;
    a_ok[i] = m < Mc;
    int mm = a_ok[i] ? m : 0;
    int img, oh, ow;
    row_pixel(mm, img, oh, ow);
    a_img[i] = img;
    if (DGRAD) { a_h[i] = oh + p.pad; a_w[i] = ow + p.pad; }
    else { a_h[i] = oh * p.stride - p.pad; a_w[i] = ow * p.stride - p.pad; }
    a_base[i] = (const char*)p.x + (size_t)img * p.H * p.W * p.Cx * ES;
  }
  const char* b_base[BP];
  bool b_ok[BP];
  int b_n[BP];
#pragma unroll
  for (int i = 0; i < BP; ++i) {
    int n = n0 + rbase + i * ROWS;
    b_n[i] = n;
    b_ok[i] = n < p.Nout && rbase + i * ROWS < BN;
    b_base[i] = (const char*)p.w + (size_t)(b_ok[i] ? n : 0) * p.Ktot * ES;
  }
  // position of this thread's chunk in (tap, channel) space
  int kc = chunk * CE, kr = 0, ks = 0, kflat = chunk * CE;
  while (kc >= p.Cx) { kc -= p.Cx; if (++ks == p.S) { ks = 0; ++kr; } }

  // Loads are unconditional (out-of-range taps read the tensor base and are zeroed when
  // parked in LDS): a branch around a load would make the compiler drain every
  // outstanding load at each use.
  uint4 ra[AP], rb[BP];
  bool oka[AP], okb[BP];
  auto load_global = [&]() {
#pragma unroll
    for (int i = 0; i < AP; ++i) {
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
      ok = ok && a_ok[i] && kr < p.R;
      oka[i] = ok;
      const size_t off = ok ? ((size_t)(hi * p.W + wi) * p.Cx + kc) * ES : 0;
      ra[i] = *(const uint4*)(a_base[i] + off);
    }
#pragma unroll
    for (int i = 0; i < BP; ++i) {
      okb[i] = b_ok[i] && kflat < p.Ktot;
      rb[i] = *(const uint4*)(b_base[i] + (size_t)(okb[i] ? kflat : 0) * ES);
    }
    kflat += BKE;
    kc += BKE;
    while (kc >= p.Cx) { kc -= p.Cx; if (++ks == p.S) { ks = 0; ++kr; } }
  };
  // extra reduction steps of a folded 1x1 stride-2 shortcut (class (0, 0) only): same pixel as the
  // centre tap, other tensor and weights
  int k2 = chunk * CE;
  auto load_global2 = [&]() {
#pragma unroll
    for (int i = 0; i < AP; ++i) {
      const int hi = (a_h[i] - p.pad) >> 1, wi = (a_w[i] - p.pad) >> 1;
      oka[i] = a_ok[i];
      const size_t off = oka[i] ? ((size_t)(hi * p.W + wi) * p.Cx2 + k2) * ES : 0;
      ra[i] = *(const uint4*)((const char*)p.x2 + (size_t)a_img[i] * p.H * p.W * p.Cx2 * ES + off);
    }
#pragma unroll
    for (int i = 0; i < BP; ++i) {
      okb[i] = b_ok[i];
      rb[i] = *(const uint4*)((const char*)p.w2 + ((size_t)(b_ok[i] ? b_n[i] : 0) * p.Cx2 + k2) * ES);
    }
    k2 += BKE;
  };
  auto store_lds = [&](int buf) {
    char* As = smem + buf * (BM + BN) * LDK;
    char* Bs = As + BM * LDK;
#pragma unroll
    for (int i = 0; i < AP; ++i) *(uint4*)(As + (rbase + i * ROWS) * LDK + chunk * 16) = keep_if(oka[i], ra[i]);
#pragma unroll
    for (int i = 0; i < BP; ++i)
      if (BN >= ROWS || rbase + i * ROWS < BN) *(uint4*)(Bs + (rbase + i * ROWS) * LDK + chunk * 16) = keep_if(okb[i], rb[i]);
  };

  f32x16_t acc[WN / 32][WM / 32];
#pragma unroll
  for (int j = 0; j < WN / 32; ++j)
#pragma unroll
    for (int i = 0; i < WM / 32; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[j][i][e] = 0.f;

  // S2: taps of the wrong parity are stepped over whole (Cx / BKE k-tiles at a time; the
  // position is the same for every thread of the workgroup up to the chunk offset)
  const int tiles_per_tap = S2 ? p.Cx / BKE : 1;
  auto tap_live = [&]() { return ((ch + p.pad - kr) & 1) == 0 && ((cw + p.pad - ks) & 1) == 0; };
  auto skip_dead_taps = [&]() {
    if (S2) {
      while (kr < p.R && !tap_live()) {
        kflat += p.Cx;
        if (++ks == p.S) { ks = 0; ++kr; }
      }
    }
  };
  int nk = (p.Ktot + BKE - 1) / BKE;
  if (S2) {
    int nr = 0, ns = 0;
    for (int r = 0; r < p.R; ++r) nr += ((ch + p.pad - r) & 1) == 0;
    for (int q = 0; q < p.S; ++q) ns += ((cw + p.pad - q) & 1) == 0;
    nk = nr * ns * tiles_per_tap;
  }
  const int nk1 = nk;  // k-tiles of the layer itself; the folded shortcut follows
  if (S2 && p.x2 != nullptr && cls == 0) nk += p.Cx2 / BKE;
  auto load_tile = [&](int kt) {
    if (S2 && kt >= nk1) {
      load_global2();
    } else {
      skip_dead_taps();
      load_global();
    }
  };
  if (nk > 0) {
    load_tile(0);
    store_lds(0);
  }
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < nk) load_tile(kt + 1);
    const char* As = smem + buf * (BM + BN) * LDK + wave_m * WM * LDK;
    const char* Bs = smem + buf * (BM + BN) * LDK + BM * LDK + wave_n * WN * LDK;
    // weights are the MFMA A operand so that a lane ends up with 4 consecutive output
    // channels of one pixel (one vector access per operand in the epilogue)
    mma_step<T, WN, WM, BKB>(Bs, As, lane, acc);
    if (kt + 1 < nk) store_lds(buf ^ 1);
    __syncthreads();
  }

  // lane holds pixel m = lane%32 and channels 8*g + 4*(lane/32) + (0..3), g = 0..3, of each 32x32 tile
  const int nb = n0 + wave_n * WN + 4 * (lane >> 5);
  float bias[WN / 32][4][4];
  load_bias_groups<WN / 32>(p, nb, bias);
#pragma unroll
  for (int i = 0; i < WM / 32; ++i) {
    const int m = m0 + wave_m * WM + i * 32 + (lane & 31);
    size_t pix = (size_t)m;
    if (S2) {
      int img, oh, ow;
      row_pixel(m < Mc ? m : 0, img, oh, ow);
      pix = ((size_t)img * p.Ho + oh) * p.Wo + ow;
    }
    epilogue_tile<T, WN / 32, WM / 32>(p, acc, i, m < Mc, pix, nb, bias);
  }
}

// ------------------------------------------------------------------ tile geometry of the 3x3 stride-1 kernels
// A workgroup owns a TH x TW rectangle of one image (or IMGS whole small images) and stages the
// input patch of that rectangle including its one-pixel halo in LDS.
struct HaloGeom {
  int tw_log, th_log;      // log2 of the tile width / height in pixels
  int tiles_w, tiles_h;    // tiles per image
  int imgs;                // images per tile
  int PW, PP;              // patch row pitch (TW+2) and pixels per image patch ((TH+2)*(TW+2))
  int patch_pix;           // imgs * PP
  int patch_bytes;         // patch_pix * 144 rounded to 256
  int flip;                // dgrad: tap (r,s) reads the patch at (2-r, 2-s)
  int tpi_log, tilesw_log; // log2 of the tiles per image and per image row (both powers of two)
  uint32_t mPP, mPW;       // ceil(2^32 / PP), ceil(2^32 / PW): floor(i / d) == __umulhi(i, m) for i, d < 2^16
};

// ------------------------------------------------------------------ 3x3 stride-1 forward / dgrad, asynchronous LDS fills
// The workgroup owns BM output pixels and BN output channels. Per 64-byte channel chunk the
// input patch with its halo is staged in LDS ONCE and all nine taps read their MFMA operands
// from it at shifted rows, so activations cross the L2 about 1.3x instead of 9x; zero padding
// is materialised in the patch, not tested in the inner loop. Every operand byte travels global -> LDS
// with global_load_lds_dwordx4 (no staging registers, lane L of a wave fills bytes
// [16L, 16L+16) of a 1 KiB LDS block), issued two pipeline stages (tap, channel chunk)
// ahead of its use: weight tiles rotate through three LDS slots and the next channel
// chunk's patch is fetched in slices spread over taps 0..6 of the current one. The
// compiler does not model these copies, so their completion is counted by hand: loads
// retire in order, every stage issues a fixed number per lane, and each stage waits
// until only the younger ones are outstanding, then crosses one workgroup barrier.
// LDS rows are KB unpadded bytes; the 16-byte column c of a row lives at column c ^ f(row),
// applied by choosing which global column a lane fetches. A 16-byte-per-lane LDS read is
// served 16 lanes per cycle from 64 four-byte banks, and the 16 lanes of one cycle are the
// four-lane quads q = lane/4 of a 32-lane half whose index has even (or odd) bit parity:
// {0,3,5,6} and {1,2,4,7} (measured). f is chosen so that each such set reads 16 different
// 16-byte bank groups: weight rows (consecutive across lanes) use f = (row * KB / 256) mod
// (KB/16); patch rows use bits of the patch coordinates (see patch_swizzle), and the pixels
// of a 32-pixel fragment are dealt to lanes so that one cycle's lanes hold 16 consecutive ones.
__device__ __forceinline__ void dma16(const void* gsrc, uint32_t lds_base_uniform) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gsrc), "s"(lds_base_uniform) : "memory", "m0");
}
// Same copy with the address split into a wave-uniform 64-bit base (SGPR pair) and a per-lane
// unsigned 32-bit byte offset: the per-copy address arithmetic stays on the scalar unit.
__device__ __forceinline__ void dma16s(const void* gbase_uniform, uint32_t goff, uint32_t lds_base_uniform) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(goff), "s"(gbase_uniform), "s"(lds_base_uniform) : "memory", "m0");
}
template <int N> __device__ __forceinline__ void wait_vm() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }
__device__ __forceinline__ void wg_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

struct DmaGeom {
  HaloGeom h;
  int patch_rows;   // patch pixels rounded up to 8 (one wave fill = 8 rows)
  int tab_bytes;    // pixel-offset table, rounded to 1 KiB
  int smem_bytes;   // dynamic LDS of the launch
};

template <typename T, int BM, int BN, int WM, int WN, int PS, int KB>
__global__ __launch_bounds__(64 * (BM / WM) * (BN / WN), (BM / WM) * (BN / WN) == 4 ? 2 : 1) void conv3x3_dma_kernel(ConvParams p_, DmaGeom dg) {
  ConvParams p = p_;
  constexpr int ES = sizeof(T);
  constexpr int NW = (BM / WM) * (BN / WN);  // waves per workgroup (each owns a WM x WN sub-tile)
  constexpr int FROWS = 1024 / KB;     // LDS rows per wave fill (KB = bytes of channels per row: 64 or 128)
  constexpr int CPR = KB / 16;         // 16-byte columns per row
  constexpr int WL = BN / FROWS / NW;   // weight fills per lane per stage
  constexpr int NKS = KB / 32;         // MFMA k-steps per stage
  constexpr int FB = KB == 128 ? 3 : 2;   // swizzle bits = log2(CPR)
  constexpr int RPL = KB == 128 ? 1 : 2;  // log2(rows per 256 bytes of LDS)
  static_assert(KB == 64 || KB == 128, "row depth");
  static_assert(WL >= 1, "weight tile smaller than one fill per wave");
  constexpr int NI = WM / 32, NJ = WN / 32;
  static_assert(NW == 4 || NW == 8, "four or eight waves");
  extern __shared__ __align__(16) char smem[];
  const HaloGeom& g = dg.h;
  const int prow = dg.patch_rows;
  const int pbuf_bytes = prow * KB;
  int* tab = (int*)smem;
  char* pbuf = smem + dg.tab_bytes;
  char* wring = pbuf + (PS > 0 ? 2 : 1) * pbuf_bytes;
  const uint32_t lds0 = (uint32_t)(size_t)(DDS_LDS_AS char*)smem;
  const uint32_t lds_pbuf = lds0 + dg.tab_bytes;
  const uint32_t lds_wring = lds_pbuf + (PS > 0 ? 2 : 1) * pbuf_bytes;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // scalar: everything derived from it stays in SGPRs
  const int wave_m = wave % (BM / WM), wave_n = wave / (BM / WM);
  const int grp = blockIdx.x >> g.tpi_log, tin = blockIdx.x - (grp << g.tpi_log);
  const int th_idx = tin >> g.tilesw_log, tw_idx = tin - (th_idx << g.tilesw_log);
  const int img0 = grp * g.imgs, h0 = th_idx << g.th_log, w0 = tw_idx << g.tw_log;
  const int n0 = blockIdx.y * BN;
  if (p.nrep > 1) {  // the launcher made sure that the images of a tile belong to one data-group
    const int r = min(img0 / (p.Nimg / p.nrep), p.nrep - 1);
    p.w = (const char*)p.w + (size_t)r * p.w_rep;
    if (p.bias) p.bias += (size_t)r * p.bias_rep;
  }
  const int TWm = (1 << g.tw_log) - 1, THm = (1 << g.th_log) - 1;
  const int nchunks = (p.Cx * ES) / KB;
  const size_t pixbytes = (size_t)p.Cx * ES;
  // Swizzle of the patch row at patch coordinates (xx, yy). One LDS cycle reads a 16-pixel
  // run of the tile: 16 x 1, 8 x 2 or 4 x 4 pixels, shifted by the tap. The low RPL bits of x
  // already spread a run over the rows of one 256-byte bank line; f takes the next bits of x
  // that vary inside the run and fills up with low bits of y.
  const int sw_nx = min(FB, max(0, g.tw_log - RPL));
  const int sw_mx = (1 << sw_nx) - 1, sw_my = (1 << (FB - sw_nx)) - 1;
  auto patch_swizzle = [&](int xx, int yy) { return ((xx >> RPL) & sw_mx) | ((yy & sw_my) << sw_nx); };

  // pixel-offset table of the patch rows: pixel index in the gathered tensor, or -1 (zero row)
  for (int row = tid; row < prow; row += 64 * NW) {
    int v = -1;
    if (row < g.patch_pix) {
      const int im = (int)__umulhi((uint32_t)row, g.mPP), rem = row - im * g.PP;
      const int yy = (int)__umulhi((uint32_t)rem, g.mPW), xx = rem - yy * g.PW;
      const int gi = img0 + im, gh = h0 + yy - 1, gw = w0 + xx - 1;
      if (gi < p.Nimg && (unsigned)gh < (unsigned)p.H && (unsigned)gw < (unsigned)p.W)
        v = ((gi * p.H + gh) * p.W + gw) * CPR + patch_swizzle(xx, yy);
    }
    tab[row] = v;
  }
  __syncthreads();

  // column swizzle of a weight row (rows are consecutive across lanes, fills start at multiples of FROWS rows)
  auto swz = [](int r) { return (r >> RPL) & (CPR - 1); };
  const int l8 = lane / CPR;  // row inside a fill
  const int pcol = lane % CPR;
  const char* zsrc = (const char*)p.zeros + pcol * 16;  // the zero block is at least one pixel row long
  const int pw_total = prow / FROWS;  // wave fills in a patch
  const uint32_t lds_dump = lds_wring + 3 * (BN * KB);  // 1 KiB that absorbs surplus fills
  // Source of this lane's 16 bytes in the j-th patch fill of this wave, for channel chunk 0.
  // Rows outside the image and surplus fills read the zero block.
  // (table entries are read in one batch and turned into addresses with selects: a branch per
  // entry would serialise one LDS round trip per fill at the very start of the kernel)
  constexpr int NPRO = (KB == 128 && PS == 0) ? 11 : 7;  // fills per wave that cover the largest patch (4 waves x NPRO x FROWS rows)
  const char* pro_src[NPRO];
  {
    int offs[NPRO];
#pragma unroll
    for (int j = 0; j < NPRO; ++j) {
      const int wl = wave + NW * j;
      offs[j] = tab[(wl < pw_total ? wl * FROWS : 0) + l8];  // pixel * CPR + f, or -1
    }
#pragma unroll
    for (int j = 0; j < NPRO; ++j) {
      const bool ok = wave + NW * j < pw_total && offs[j] >= 0;
      const int o = ok ? offs[j] : 0;
      const char* a = (const char*)p.x + (size_t)(o >> FB) * pixbytes + ((pcol ^ (o & (CPR - 1))) << 4);
      pro_src[j] = ok ? a : zsrc;
    }
  }
  auto patch_src = [&](int j) -> const char* { return pro_src[j]; };
  auto patch_dst = [&](int j, int buf) {
    const int wl = wave + NW * j;
    return wl < pw_total ? lds_pbuf + buf * pbuf_bytes + wl * 1024 : lds_dump;
  };
  constexpr int NPF = 7 * PS;  // patch fills per wave and chunk issued inside the loop
  const char* psrc[NPF > 0 ? NPF : 1];
#pragma unroll
  for (int j = 0; j < NPF; ++j) psrc[j] = patch_src(j);
  // weight rows: byte offset of this lane's 16 bytes inside the weight tensor at tap 0, chunk 0.
  // Rows past Nout repeat the last one: their output columns lie past ldy == Nout and are never stored.
  uint32_t wvo[WL];
#pragma unroll
  for (int u = 0; u < WL; ++u) {
    const int gn = n0 + (wave + NW * u) * FROWS + l8;
    const int c16 = (pcol ^ swz(l8 + (wave & 1) * FROWS)) * 16;
    wvo[u] = (uint32_t)(gn < p.Nout ? gn : p.Nout - 1) * (uint32_t)(9 * pixbytes) + c16;
  }
  auto fill_w = [&](int chunk, int tap, int slot) {
    const char* base = (const char*)p.w + (size_t)tap * pixbytes + (size_t)chunk * KB;  // wave-uniform
#pragma unroll
    for (int u = 0; u < WL; ++u) dma16s(base, wvo[u], lds_wring + slot * (BN * KB) + (wave + NW * u) * 1024);
  };

  // pixel of the 32-pixel fragment held by this lane: quads {0,3,5,6} -> pixels 0..15, {1,2,4,7} -> 16..31
  const int lq = (lane >> 2) & 7;
  const int lpix = ((__builtin_popcount(lq) & 1) << 4) | ((lq >> 1) << 2) | (lane & 3);
  // dgrad through a ReLU: the sign bits of this lane's outputs are fetched now (a few bytes per
  // pixel, the oldest loads of the kernel) so that the epilogue reads nothing but the accumulators
  uint32_t mb[NI][NJ] = {};
  if (p.maskbits) {
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int m = wave_m * WM + i * 32 + lpix;
      const int x = m & TWm, y = (m >> g.tw_log) & THm, im = m >> (g.tw_log + g.th_log);
      const int gi = img0 + im;
      const size_t pix = ((size_t)gi * p.H + h0 + y) * p.W + w0 + x;
#pragma unroll
      for (int j = 0; j < NJ; ++j) mb[i][j] = load_bits32(p.maskbits, pix, p.ldy, n0 + wave_n * WN + 32 * j, gi < p.Nimg);
    }
  }

  // prologue: whole first patch, then the weight tiles of stages 0 and 1. Issued before the rest of
  // the set-up (fragment addresses, sign words, accumulators) so that it runs under the copies' latency.
#pragma unroll
  for (int j = 0; j < NPRO; ++j)
    if (wave + NW * j < pw_total) dma16(pro_src[j], patch_dst(j, 0));
  fill_w(0, 0, 0);
  fill_w(0, 1, 1);

  // fragment addressing
  const int half = lane >> 5;
  // Patch operand: LDS byte offset of a fragment row = row * KB + (((2 ks + half) ^ f) << 4) with
  // f = fx(x + tap_s) | fy(y + tap_r). Per lane and tap coordinate the swizzle bits are kept in
  // registers (sx also carries half), so a stage needs one add, one xor-add and one xor per k-step.
  int rowb[NI], sx[NI][3], sy[NI][3];
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const int m = wave_m * WM + i * 32 + lpix;
    const int x = m & TWm, y = (m >> g.tw_log) & THm, im = m >> (g.tw_log + g.th_log);
    rowb[i] = (im * g.PP + y * g.PW + x) * KB;
#pragma unroll
    for (int t = 0; t < 3; ++t) {
      const int tt = g.flip ? 2 - t : t;
      sx[i][t] = ((patch_swizzle(x + tt, 0)) ^ half) << 4;
      sy[i][t] = patch_swizzle(0, y + tt) << 4;
    }
  }
  int boff[NJ][NKS];
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int n = wave_n * WN + j * 32 + (lane & 31);
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) boff[j][ks] = n * KB + (((2 * ks + half) ^ swz(n)) << 4);
  }
  f32x16_t acc[NJ][NI];
#pragma unroll
  for (int j = 0; j < NJ; ++j)
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[j][i][e] = 0.f;

  const int pbuf_off = dg.tab_bytes;
  auto compute = [&](int chunk, int tap_r, int tap_s, int slot) {
    const int tapoff = (g.flip ? 2 - tap_r : tap_r) * g.PW + (g.flip ? 2 - tap_s : tap_s);
    const int sbase = pbuf_off + (PS > 0 ? (chunk & 1) * pbuf_bytes : 0) + tapoff * KB;  // wave-uniform
    const char* wb = wring + slot * (BN * KB);
    int a0[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      int rb = rowb[i];
      asm volatile("" : "+v"(rb));  // keeps the nine taps' addresses from being precomputed (and spilled)
      a0[i] = (sx[i][tap_s] ^ sy[i][tap_r]) + (rb + sbase);
    }
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
      uint4 a[NI], b[NJ];
#pragma unroll
      for (int i = 0; i < NI; ++i) a[i] = *(const uint4*)(smem + (a0[i] ^ (ks << 5)));
#pragma unroll
      for (int j = 0; j < NJ; ++j) b[j] = *(const uint4*)(wb + boff[j][ks]);
#pragma unroll
      for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int i = 0; i < NI; ++i) mfma16B<T>(b[j], a[i], acc[j][i]);
    }
  };

// One stage = one tap of one channel chunk. VM = fills per lane issued after the weight
// tile this stage consumes: one weight tile plus the patch slices of the two previous stages.
#define DDS_STAGE(TAP)                                                                              \
  {                                                                                                 \
    constexpr int VM = WL + PS * (((TAP) >= 2 && (TAP) <= 8 ? 1 : 0) + ((TAP) >= 1 && (TAP) <= 7 ? 1 : 0)); \
    wait_vm<VM>();                                                                                  \
    wg_barrier();                                                                                   \
    {                                                                                               \
      int ct = chunk + ((TAP) + 2 >= 9 ? 1 : 0), tt = ((TAP) + 2) % 9;                             \
      if (ct >= nchunks) { ct = nchunks - 1; tt = 8; }                                              \
      fill_w(ct, tt, ((TAP) + 2) % 3);                                                              \
    }                                                                                               \
    if (PS > 0 && (TAP) < 7) {                                                                      \
      const int cn = chunk + 1 < nchunks ? chunk + 1 : chunk;                                       \
      _Pragma("unroll") for (int u = 0; u < PS; ++u)                                                \
        dma16(psrc[((TAP) < 7 ? (TAP) : 0) * PS + u] + (size_t)cn * KB, patch_dst((TAP) * PS + u, (chunk + 1) & 1)); \
    }                                                                                               \
    compute(chunk, (TAP) / 3, (TAP) % 3, (TAP) % 3);                                                \
  }

  for (int chunk = 0; chunk < nchunks; ++chunk) {
    DDS_STAGE(0) DDS_STAGE(1) DDS_STAGE(2) DDS_STAGE(3) DDS_STAGE(4) DDS_STAGE(5) DDS_STAGE(6) DDS_STAGE(7) DDS_STAGE(8)
  }
#undef DDS_STAGE
  wait_vm<0>();

  // Stage the residual / mask tiles of this workgroup in LDS (the operand buffers are free
  // now) so the epilogue pays one global round trip instead of one per 32-pixel column.
  constexpr int ROWB = BN * ES;        // bytes per tile row
  constexpr int NCOL = ROWB / 16;      // 16-byte columns per row
  constexpr int RPF = 64 / NCOL;       // rows per wave fill
  constexpr int FPW = BM / RPF / NW;    // fills per wave
  int res_off = -1, mask_off = -1, nregions = 0;
  const int ab_off = (int)(lds_dump - lds0);  // the dump block now holds alpha * bias of this tile's channels
  float* ab_lds = (float*)(smem + ab_off);
  wg_barrier();
  if (tid < BN) {
    const int n = n0 + tid;
    ab_lds[tid] = (p.bias != nullptr && n < p.Nout) ? p.alpha * p.bias[n] : 0.f;
  }
  if (p.res || p.mask) {
    int region = 0;
    auto stage_tile = [&](const void* src_tensor) -> int {
      if ((region + 1) * BM * ROWB > dg.smem_bytes - 1024) return -1;
      const int rbase = region * BM * ROWB;
#pragma unroll
      for (int u = 0; u < FPW; ++u) {
        const int f = wave + NW * u;
        const int row = f * RPF + lane / NCOL, slot = lane % NCOL;
        const int gc = (slot ^ row) & (NCOL - 1);
        const int x = row & TWm, y = (row >> g.tw_log) & THm, im = row >> (g.tw_log + g.th_log);
        const int gi = img0 + im;
        const int n = n0 + gc * (16 / ES);
        const bool ok = gi < p.Nimg && n < p.ldy;
        const size_t pix = ((size_t)gi * p.H + h0 + y) * p.W + w0 + x;
        const char* src = ok ? (const char*)src_tensor + (pix * p.ldy + n) * ES : (const char*)p.zeros;
        dma16(src, lds0 + rbase + f * 1024);
      }
      ++region;
      return rbase;
    };
    if (p.mask) mask_off = stage_tile(p.mask);
    if (p.res) res_off = stage_tile(p.res);
    wait_vm<0>();
    nregions = region;
  }
  // Output tile in LDS: the residual tile's bytes if there is one, else the next free region.
  int out_off = res_off >= 0 ? res_off : ((nregions + 1) * BM * ROWB <= dg.smem_bytes - 1024 ? nregions * BM * ROWB : -1);
  if (p.out_f32) out_off = -1;
  __syncthreads();  // also orders the plain LDS stores of alpha * bias

  const int nb = n0 + wave_n * WN + 4 * (lane >> 5);
  float bias[NJ][4][4] = {};
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const int m = wave_m * WM + i * 32 + lpix;
    const int x = m & TWm, y = (m >> g.tw_log) & THm, im = m >> (g.tw_log + g.th_log);
    const int gi = img0 + im;
    const size_t pix = ((size_t)gi * p.H + h0 + y) * p.W + w0 + x;
    epilogue_tile<T, NJ, NI>(p, acc, i, gi < p.Nimg, pix, nb, bias, (const char DDS_LDS_AS*)smem, res_off, mask_off, m, ROWB,
                             wave_n * WN + 4 * (lane >> 5), ab_off, mb[i], out_off);
  }
  if (out_off >= 0) {
    // write the tile out: a wave stores RPF whole tile rows per instruction, 16 bytes per lane
    __syncthreads();
#pragma unroll
    for (int u = 0; u < FPW; ++u) {
      const int f = wave + NW * u;
      const int row = f * RPF + lane / NCOL, slot = lane % NCOL;
      const int gc = (slot ^ row) & (NCOL - 1);
      const int x = row & TWm, y = (row >> g.tw_log) & THm, im = row >> (g.tw_log + g.th_log);
      const int gi = img0 + im;
      const int n = n0 + gc * (16 / ES);
      const size_t pix = ((size_t)gi * p.H + h0 + y) * p.W + w0 + x;
      const u32x4_t v = *(const u32x4_t DDS_LDS_AS*)((const char DDS_LDS_AS*)smem + out_off + f * 1024 + lane * 16);
      if (gi < p.Nimg && n < p.ldy) *(u32x4_t*)((char*)p.y + (pix * p.ldy + n) * ES) = v;
    }
  }
}

inline int ilog2_exact(int v) {
  int l = 0;
  while ((1 << l) < v) ++l;
  return (1 << l) == v ? l : -1;
}

// Fills g and returns true when the 3x3 stride-1 tiling covers this problem.
template <typename T>
bool halo_geometry(const ConvParams& p, HaloGeom& g, int BM = 256, int chunk_bytes = 64) {
  const int CK = chunk_bytes / (int)sizeof(T);
  if (p.R != 3 || p.S != 3 || p.stride != 1 || p.pad != 1 || p.H != p.Ho || p.W != p.Wo) return false;
  if (p.Cx % CK != 0 || p.out_f32) return false;
  const int lw = ilog2_exact(p.W), lh = ilog2_exact(p.H);
  if (lw < 1 || lh < 1 || p.W > 32) return false;
  int TW = p.W, TH, imgs;
  if (p.H * p.W >= BM) {
    TH = BM / TW;
    imgs = 1;
    if (TH < 1 || TH > p.H || p.H % TH) return false;
  } else {
    TH = p.H;
    imgs = BM / (p.H * p.W);
  }
  g.tw_log = ilog2_exact(TW);
  g.th_log = ilog2_exact(TH);
  g.tiles_w = p.W / TW;
  g.tiles_h = p.H / TH;
  g.imgs = imgs;
  g.PW = TW + 2;
  g.PP = (TH + 2) * (TW + 2);
  g.patch_pix = imgs * g.PP;
  g.patch_bytes = (g.patch_pix * 144 + 255) / 256 * 256;
  g.flip = p.dgrad;
  g.tilesw_log = ilog2_exact(g.tiles_w);
  g.tpi_log = ilog2_exact(g.tiles_w * g.tiles_h);
  if (g.tilesw_log < 0 || g.tpi_log < 0 || g.PP >= 65536 || g.patch_pix >= 65536) return false;
  g.mPP = (uint32_t)(((1ull << 32) + g.PP - 1) / g.PP);
  g.mPW = (uint32_t)(((1ull << 32) + g.PW - 1) / g.PW);
  return true;
}

template <typename T, int BM, int BN, int WM, int WN, int PS, int KB>
bool launch_dma_inst(const ConvParams& p, const HaloGeom& h, hipStream_t s) {
  constexpr int FROWS = 1024 / KB;
  constexpr int NW = (BM / WM) * (BN / WN);
  DmaGeom dg;
  dg.h = h;
  dg.patch_rows = (h.patch_pix + FROWS - 1) / FROWS * FROWS;
  dg.tab_bytes = (dg.patch_rows * 4 + 1023) / 1024 * 1024;
  const int fills_per_wave = (dg.patch_rows / FROWS + NW - 1) / NW;
  if (p.Cx * (int)sizeof(T) % KB != 0) return false;
  const int nchunks = p.Cx * (int)sizeof(T) / KB;
  if (fills_per_wave > ((KB == 128 && PS == 0) ? 11 : 7)) return false;  // prologue sources kept per lane
  if (PS == 0 ? nchunks != 1 : (nchunks < 2 || 7 * PS < fills_per_wave)) return false;
  const int smem = dg.tab_bytes + (PS > 0 ? 2 : 1) * dg.patch_rows * KB + 3 * BN * KB + 1024;
  if (smem > 160 * 1024 || p.zeros == nullptr) return false;
  // pad rows come from the zero block; pad weight rows repeat row Nout-1 (columns past ldy are not stored);
  // per-lane weight offsets are 32-bit
  if (p.Cx * (int)sizeof(T) + 256 > kZeroBytes || p.ldy != p.Nout) return false;
  if ((long long)p.Nout * 9 * p.Cx * (long long)sizeof(T) >= (1ll << 31)) return false;
  dg.smem_bytes = smem;
  static bool attr_set = false;
  if (!attr_set) {
    (void)hipFuncSetAttribute((const void*)conv3x3_dma_kernel<T, BM, BN, WM, WN, PS, KB>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    attr_set = true;
  }
  const int groups = (p.Nimg + h.imgs - 1) / h.imgs;
  dim3 grid(groups * h.tiles_w * h.tiles_h, (p.ldy + BN - 1) / BN);
  conv3x3_dma_kernel<T, BM, BN, WM, WN, PS, KB><<<grid, 64 * NW, smem, s>>>(p, dg);
  return true;
}

// Picks the tile for the asynchronous kernel; false if the problem is outside its range.
// Channel chunks are 64 bytes deep: the LDS footprint lets two or three workgroups share a
// CU and hide each other's prologue and epilogue, and with 16 rows per wave fill a patch of
// up to 340 rows needs at most 6 fills per wave, so one slice per tap (PS = 1) is enough.
template <typename T>
bool launch_dma(const ConvParams& p, hipStream_t s) {
  HaloGeom h;
  constexpr int KB = 64;
  const int rowbytes = p.Cx * (int)sizeof(T);
  if (rowbytes % KB != 0) return false;
  const int nchunks = rowbytes / KB;
  // 64 bf16 (32 fp32) channels in and at most 64 out: one 128-byte chunk, i.e. whole cache lines per patch row,
  // nine stages instead of eighteen and the whole patch requested in the prologue (62.0 -> 59.4 us at 32 x 32 x 64)
  if (rowbytes == 128 && p.ldy <= 64 && halo_geometry<T>(p, h, 256, 128) &&
      launch_dma_inst<T, 256, 64, 64, 64, 0, 128>(p, h, s)) return true;
  if (nchunks == 1) {
    if (!halo_geometry<T>(p, h, 256, KB)) return false;
    if (p.ldy <= 64) return launch_dma_inst<T, 256, 64, 64, 64, 0, KB>(p, h, s);
    return launch_dma_inst<T, 256, 128, 128, 64, 0, KB>(p, h, s);
  }
  // small images: 128-pixel tiles give more workgroups. 256-pixel tiles from 256 workgroups up (one per CU: half the
  // weight copies per FLOP; with the other modules' kernels sharing the chip this beat two 128-pixel workgroups per
  // CU at 256 channels, 2.27 vs 2.31 ms per ResNet-18 step)
  const long long tiles256 = (long long)((p.M + 255) / 256) * ((p.ldy + 127) / 128);
  if (tiles256 >= 256 && halo_geometry<T>(p, h, 256, KB)) {
    if (p.ldy <= 64 && launch_dma_inst<T, 256, 64, 64, 64, 1, KB>(p, h, s)) return true;
    if (launch_dma_inst<T, 256, 128, 128, 64, 1, KB>(p, h, s)) return true;
  }
  if (halo_geometry<T>(p, h, 128, KB) && launch_dma_inst<T, 128, 128, 64, 64, 1, KB>(p, h, s)) return true;
  return false;
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
__global__ __launch_bounds__(256, 2) void wgrad_gemm_kernel(WgradParams p) {
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

  // unconditional loads from clamped addresses; validity is applied when the data is parked in LDS
  uint4 regs[NBLK][CE];
  uint32_t okmask[NBLK], onemask[NBLK];
  auto load_global = [&](int ptile) {
#pragma unroll
    for (int b = 0; b < NBLK; ++b) {
      okmask[b] = 0;
      onemask[b] = 0;
#pragma unroll
      for (int g = 0; g < CE; ++g) {
        const int pix = ptile + kg[b] * CE + g;
        const bool inr = pix < pz1;
        const char* src = (const char*)p.dy;
        bool ok = false;
        if (isA[b]) {
          ok = inr && okc[b];
          if (ok) src = (const char*)p.dy + ((size_t)pix * p.ldy + coff[b]) * ES;
        } else if (okc[b]) {
          const int pp = inr ? pix : 0;
          int img = pp / HoWo;
          int rem = pp - img * HoWo;
          int oh = rem / p.Wo, ow = rem - oh * p.Wo;
          int hi = oh * p.stride + bh[b], wi = ow * p.stride + bw[b];
          ok = inr && (unsigned)hi < (unsigned)p.H && (unsigned)wi < (unsigned)p.W;
          if (ok) src = (const char*)p.x + (((size_t)img * p.H + hi) * p.W + wi) * p.Cx * ES + (size_t)coff[b] * ES;
        } else if (isBias[b] && inr) {
          onemask[b] |= 1u << g;
        }
        okmask[b] |= (ok ? 1u : 0u) << g;
        regs[b][g] = *(const uint4*)src;
      }
    }
  };
  auto store_lds = [&](int buf) {
    char* base = smem + buf * (BM + BN) * LDK;
#pragma unroll
    for (int b = 0; b < NBLK; ++b) {
      if (row0[b] < 0) continue;
      uint4 sel[CE], t[CE];
#pragma unroll
      for (int g = 0; g < CE; ++g) {
        sel[g] = keep_if((okmask[b] >> g) & 1u, regs[b][g]);
        if ((onemask[b] >> g) & 1u) sel[g] = one_chunk<T>();
      }
      transpose_chunks<T>(sel, t);
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

// ------------------------------------------------------------------ 3x3 stride-1 wgrad, asynchronous LDS fills + LDS transpose reads (bf16)
// dW[k][tap][c] = sum over pixels p of dY[p][k] * X[p + tap][c]. The workgroup owns a
// 64(k) x 64(c) block for ALL nine taps and walks its split of the pixel axis in tiles of
// 128 pixels (rows of one image, or whole small images): per tile the dY rows and the X
// patch with halo are copied global -> LDS in their natural [pixel][channel] order (two
// slots: the next tile is copied while this one is multiplied) and the nine taps reuse them. The reduction
// index of this GEMM is the pixel, which is the slow axis of both operands in memory:
// ds_read_b64_tr_b16 hands each lane four pixels of one channel from a 4 x 16 block, so
// no register or LDS transposition is needed. 16-byte LDS columns are XOR-ed with
// 2*(row & 3) so that the four rows of such a block sit on different banks.
typedef short s16x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint2 lds_tr16(const char* p) {
  s16x4_t v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t DDS_LDS_AS*)p);
  return __builtin_bit_cast(uint2, v);
}

// Geometry the host passes along with WgradParams.
struct WgradGeom {
  int tiles_h;     // 128-pixel tiles per image (a power of two; 1 when a tile holds whole images)
  int cblocks;     // 64-channel blocks of the real input tensor
  int sub[4];      // S2: sub-pixel (dy * 2 + dx) served by blockIdx.y / cblocks
  int rmap[2][2];  // S2: real kernel row for (virtual row R', dy), -1 if none; the same table serves columns
  int xcd_remap;   // splits are a multiple of eight: workgroups of one split are dealt to one XCD (see the kernel)
};

// S2 = false: 3x3, stride 1, pad 1 (nine taps, TW x TH tiles of the image itself).
// S2 = true: a stride-2 convolution (3x3 pad 1, or 1x1 pad 0) seen as a stride-1 one on the
// input regrouped into 2x2 sub-pixels: output pixel (oy, ox) and real tap r read input row
// 2*oy + r - pad, i.e. sub-pixel row dy of super-pixel row oy - 1 or oy. A workgroup takes the
// 64 channels of ONE sub-pixel (dy, dx); its patch is that sub-grid (gathered at pixel stride
// 2 by the fills) and only the virtual taps R', S' in {0, 1} that a real tap maps to are
// accumulated: 1, 2, 2 and 4 of them for the four sub-pixels of a 3x3 kernel, none wasted.
__device__ __forceinline__ uint2 lds_tr16_at(uint32_t lds_byte_address) {
  s16x4_t v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t DDS_LDS_AS*)(size_t)lds_byte_address);
  return __builtin_bit_cast(uint2, v);
}

// Waves: four per tap group, each owning a 32(k) x 32(c) quarter of the block. Stride 1 runs
// three tap groups (one per kernel row, 12 waves, three per SIMD) so that the LDS reads of one wave
// hide behind the MFMAs of the others; a group's row shift is folded into its lanes' base addresses.
template <int TWLOG, int THLOG, bool S2>
__global__ __launch_bounds__(S2 ? 256 : 768) void wgrad_dma_kernel(WgradParams p, WgradGeom wg, const void* zeros) {
  constexpr int TW = 1 << TWLOG, TH = 1 << THLOG, PW = TW + 2, PP = (TH + 2) * PW;
  constexpr int IMGS = 128 / (TW * TH);
  static_assert(IMGS >= 1 && IMGS * TW * TH == 128, "a tile is 128 pixels");
  constexpr int NWV = S2 ? 4 : 12;                // waves per workgroup
  constexpr int PROW = (IMGS * PP + 7) / 8 * 8;   // patch rows, whole 8-row fills
  constexpr int FY = (16 + NWV - 1) / NWV;        // dY fills per wave (16 per tile)
  constexpr int PF = (PROW / 8 + NWV - 1) / NWV;  // patch fills per wave
  constexpr int NF = FY + PF;  // fills per lane per tile (surplus ones go to a dump block)
  constexpr int NT = S2 ? 4 : 3;                  // taps accumulated by one wave
  constexpr int SLOT = 16384 + PROW * 128;
  extern __shared__ __align__(16) char smem[];
  const uint32_t lds_ring = (uint32_t)(size_t)(DDS_LDS_AS char*)smem;
  // Tiles in flight in LDS. Two (the next tile is copied while this one is multiplied) keep a workgroup at 85 KB,
  // so that a conv workgroup of another module fits on the same CU; a third slot (copies two tiles ahead,
  // 127 KB) was 1-2 % slower per training step on every configuration although each launch alone was not.
  constexpr int RING = 2;
  const uint32_t lds_dump = lds_ring + RING * SLOT;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wave_m = wave & 1, wave_n = (wave >> 1) & 1;
  const int tg = wave >> 2;  // tap group: kernel row of this wave's three taps (stride 1)
  // Workgroup -> (k-block, sub-pixel / c-block, split). Every (k, c) block of one split reads the same dY rows and
  // X patches, so they should meet in one L2: workgroups are handed to the eight XCDs round-robin in launch order,
  // hence launch index i lands on XCD i % 8 as the (i / 8)-th workgroup of that XCD. With a split count that is
  // a multiple of eight, XCD x takes the splits z = x (mod 8) and runs all blocks of a split back to back, so
  // they are resident together and walk the pixel tiles at the same pace.
  int bx = blockIdx.x, by = blockIdx.y, z = blockIdx.z;
  if (wg.xcd_remap) {
    const int nblk = gridDim.x * gridDim.y;
    const int lin = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
    const int xcd = lin & 7, j = lin >> 3;
    const int blk = j % nblk;
    z = (j / nblk) * 8 + xcd;
    bx = blk % gridDim.x;
    by = blk / gridDim.x;
  }
  const int k0 = bx * 64;
  const int sub = S2 ? wg.sub[by / wg.cblocks] : 0;
  const int sdy = sub >> 1, sdx = sub & 1;
  const int c0 = (S2 ? by % wg.cblocks : by) * 64;
  // Split z = (data-group, j): the data-group's tiles are dealt to its q splits as evenly as whole
  // tiles allow (tile counts differ by at most one), so a split never mixes two data-groups.
  const int q = p.nsplit / p.nrep, rep_tiles = (p.P >> 7) / p.nrep;
  const int zr = z / q, zj = z - zr * q;
  const int tile0 = zr * rep_tiles + (zj * rep_tiles) / q;
  const int ntiles = zr * rep_tiles + ((zj + 1) * rep_tiles) / q - tile0;
  const size_t ybytes = (size_t)p.ldy * 2, xbytes = (size_t)p.Cx * 2;

  // A tile is 128 consecutive pixels of the flattened (image, row, column) index of the output
  // grid, so the source address of every fill advances by a constant from tile to tile; what is
  // kept per lane and fill is the byte offset of its patch row relative to the tile origin and
  // the row / column facts that decide whether that row is padding.
  const int l8 = lane >> 3;
  const int c16 = ((lane & 7) ^ ((l8 & 3) << 1)) * 16;  // global 16-byte column for LDS slot lane&7 of a row with row&3 == l8&3
  const char* zsrc = (const char*)zeros + c16;
  constexpr int pw_total = PROW >> 3;
  const bool ycol_ok = k0 + (c16 >> 1) < p.ldy;   // this lane's 8 output channels exist
  const bool xcol_ok = c0 + (c16 >> 1) < p.Cx;    // ... and its 8 input channels (tensors narrower than a 64-channel block)
  const size_t tile_ybytes = 128 * ybytes, tile_xbytes = (S2 ? 4 : 1) * 128 * xbytes;
  const char* ysrc0 = (const char*)p.dy + ((size_t)tile0 * 128 + (size_t)(wave * 8 + l8)) * ybytes + (size_t)k0 * 2 + c16;
  const char* xsrc0 = (const char*)p.x + (size_t)tile0 * tile_xbytes + (size_t)c0 * 2 + c16;
  int prel[PF], pflag[PF];  // byte offset from the tile origin; yy | column valid << 8
#pragma unroll
  for (int u = 0; u < PF; ++u) {
    const int row = (wave + NWV * u) * 8 + l8;
    int rel = 0, flag = 0;
    if (row < IMGS * PP) {
      const int im = row / PP, rem = row - im * PP;
      const int yy = rem / PW, xx = rem - yy * PW;
      if (S2) rel = (int)((((long long)im * p.H + 2 * (yy - 1) + sdy) * p.W + 2 * (xx - 1) + sdx) * (long long)xbytes);
      else rel = (int)((((long long)im * p.H + yy - 1) * p.W + (xx - 1)) * (long long)xbytes);
      flag = yy | (((unsigned)(xx - 1) < (unsigned)p.Wo ? 1 : 0) << 8);
    }
    prel[u] = rel;
    pflag[u] = flag;
  }
  const int tile_in_img_mask = wg.tiles_h - 1;
  auto fill_tile = [&](int t, int slot) {  // t: tile index inside this split (fills nothing real past the end)
    const bool live_t = t < ntiles;
    const int tt = live_t ? t : 0;
    const int h0 = ((tile0 + tt) & tile_in_img_mask) << THLOG;
    const uint32_t base = lds_ring + slot * SLOT;
    const char* ysrc = ysrc0 + (size_t)tt * tile_ybytes;
    const char* xsrc = xsrc0 + (size_t)tt * tile_xbytes;
    const bool yok = live_t && ycol_ok;
#pragma unroll
    for (int u = 0; u < FY; ++u) {  // dY rows: tile pixel 8*(wave + NWV u) + l8
      const bool live = live_t && wave + NWV * u < 16;  // wave-uniform
      if (RING == 2 && !live) continue;  // only a fixed count of fills per tile (wait_vm<NF>) needs the surplus ones
      dma16(yok && live ? ysrc + (size_t)u * (NWV * 8) * ybytes : zsrc, live ? base + (wave + NWV * u) * 1024 : lds_dump);
    }
#pragma unroll
    for (int u = 0; u < PF; ++u) {  // patch rows
      const int wl = wave + NWV * u;
      const bool live = live_t && wl < pw_total;  // wave-uniform
      if (RING == 2 && !live) continue;
      const int gh = h0 + (pflag[u] & 255) - 1;
      const bool ok = live && xcol_ok && (pflag[u] >> 8) && (unsigned)gh < (unsigned)p.Ho;
      dma16(ok ? xsrc + prel[u] : zsrc, live ? base + 16384 + wl * 1024 : lds_dump);
    }
  };

  // the first two tiles are requested before the rest of the set-up, which runs under their latency
  fill_tile(0, 0);
  if (RING == 3) fill_tile(1, 1);

  // fragment addressing (see lds_tr16): lane -> (16-lane group, row inside the 4-row block, 8-byte segment)
  const int lq = lane & 15, grp16 = (lane >> 4) & 1, khalf = lane >> 5;
  const int rsub = lq >> 2, seg = lq & 3;
  // A (dY): rows are tile pixels; row & 3 == rsub for every block this lane reads
  const int a_c = 4 * wave_m + 2 * grp16 + (seg >> 1);
  const int a_lane = (8 * khalf + rsub) * 128 + ((a_c ^ (rsub << 1)) << 4) + 8 * (seg & 1);
  // B (patch): k-step ks covers tile pixels 16 ks + ql, ql = 8 khalf + rsub + 4 hh for this
  // lane's two 4-pixel blocks hh. The patch row of such a pixel splits into a per-lane part
  // (kept in registers, one copy per value v of (row + tap offset) & 3 that the column
  // swizzle depends on) and a part that only depends on (ks, tap): a compile-time offset.
  const int b_c = 4 * wave_n + 2 * grp16 + (seg >> 1);
  int baddr[2][4];
#pragma unroll
  for (int hh = 0; hh < 2; ++hh) {
    const int ql = 8 * khalf + rsub + 4 * hh;
    const int rl = (ql >> TWLOG) * PW + (ql & (TW - 1)) + (S2 ? 0 : tg * PW);
#pragma unroll
    for (int v = 0; v < 4; ++v) baddr[hh][v] = rl * 128 + ((b_c ^ (((rl + v) & 3) << 1)) << 4) + 8 * (seg & 1);
  }
  bool live[NT];
  int tapreal[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    if (S2) {
      const int rr = wg.rmap[t >> 1][sdy], ss = wg.rmap[t & 1][sdx];
      live[t] = rr >= 0 && ss >= 0;
      tapreal[t] = rr * p.S + ss;
    } else {
      live[t] = true;
      tapreal[t] = tg * 3 + t;
    }
  }

  f32x16_t acc[NT], accb;
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;
#pragma unroll
  for (int e = 0; e < 16; ++e) accb[e] = 0.f;
  const uint4 ones = make_uint4(0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u);
  // narrow layers (at most 32 output or input channels): the waves of the empty half-blocks skip the arithmetic
  const bool idle_wave = k0 + wave_m * 32 >= p.Mout || c0 + wave_n * 32 >= p.Cx;

  for (int t = 0; t < ntiles; ++t) {
    if (RING == 3) wait_vm<NF>();  // everything but the youngest tile's fills has landed
    else wait_vm<0>();
    wg_barrier();
    fill_tile(t + RING - 1, (t + RING - 1) % RING);
    uint32_t ybuf = lds_ring + (t % RING) * SLOT + a_lane;
    uint32_t bp[2][4];
#pragma unroll
    for (int hh = 0; hh < 2; ++hh)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        bp[hh][v] = lds_ring + (t % RING) * SLOT + 16384 + baddr[hh][v];
        // opaque: otherwise every (lane part + compile-time part) sum is precomputed outside the
        // tile loop, one register each, instead of riding in the instruction's offset field
        asm volatile("" : "+v"(bp[hh][v]));
      }
    asm volatile("" : "+v"(ybuf));
    // Fragments of k-step ks + 1 (16 pixels each) are read into the other register set while the
    // MFMAs of k-step ks run, so only the first k-step of a tile waits for LDS.
    uint4 af[2], bf[2][NT];
    auto load_frags = [&](int ks, int set) {  // ks is a constant after unrolling
      const int q0 = ks * 16;
      const int rc = (q0 >> (TWLOG + THLOG)) * PP + ((q0 >> TWLOG) & (TH - 1)) * PW + (q0 & (TW - 1));
      const uint2 a0 = lds_tr16_at(ybuf + ks * 2048);
      const uint2 a1 = lds_tr16_at(ybuf + ks * 2048 + 512);
      af[set] = make_uint4(a0.x, a0.y, a1.x, a1.y);
#pragma unroll
      for (int tap = 0; tap < NT; ++tap) {
        const int toff = S2 ? (tap >> 1) * PW + (tap & 1) : tap;  // stride 1: the row shift sits in the base
        const int v = (rc + toff) & 3;
        const uint2 b0 = lds_tr16_at(bp[0][v] + (rc + toff) * 128);
        const uint2 b1 = lds_tr16_at(bp[1][v] + (rc + toff) * 128);
        bf[set][tap] = make_uint4(b0.x, b0.y, b1.x, b1.y);
      }
    };
    if (idle_wave) continue;  // its 32 x 32 block lies past the real channels: fills and barriers only
    load_frags(0, 0);
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      if (ks + 1 < 8) load_frags(ks + 1, (ks + 1) & 1);
#pragma unroll
      for (int tap = 0; tap < NT; ++tap)
        if (!S2 || live[tap]) mfma16B<bf16_t>(af[ks & 1], bf[ks & 1][tap], acc[tap]);
      if (wave_n == 0 && by == 0 && tg == (S2 ? 0 : 1)) mfma16B<bf16_t>(af[ks & 1], ones, accb);  // bias gradient: column sums of dY
    }
  }
  wait_vm<0>();

  float* out = p.partial + (size_t)z * p.Pl;
  const int cin = c0 + wave_n * 32 + (lane & 31);
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    const int k = k0 + wave_m * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
    if (k >= p.Mout) continue;
    if (cin < p.Cx) {
#pragma unroll
      for (int tap = 0; tap < NT; ++tap)
        if (live[tap]) out[(size_t)k * p.NK + tapreal[tap] * p.Cx + cin] = p.alpha * acc[tap][e];
    }
    if (wave_n == 0 && (lane & 31) == 0 && by == 0 && tg == (S2 ? 0 : 1)) out[(size_t)p.Mout * p.NK + k] = p.alpha * accb[e];
  }
}

inline int cdiv(int a, int b) { return (a + b - 1) / b; }

// Problem of data-group r alone (see ConvParams::nrep): its images, outputs and weights.
template <typename T>
ConvParams replica_slice(const ConvParams& p, int r) {
  constexpr size_t ES = sizeof(T);
  ConvParams q = p;
  const size_t Nr = (size_t)(p.Nimg / p.nrep);
  const size_t in_pix = r * Nr * p.H * p.W, out_el = r * Nr * p.Ho * p.Wo * p.ldy;
  q.x = (const char*)p.x + in_pix * p.Cx * ES;
  q.y = (char*)p.y + out_el * (p.out_f32 ? 4 : ES);
  if (p.res) q.res = (const char*)p.res + out_el * ES;
  if (p.mask) q.mask = (const char*)p.mask + out_el * ES;
  if (p.bits_out) q.bits_out = (char*)p.bits_out + out_el / 8;
  if (p.maskbits) q.maskbits = (const char*)p.maskbits + out_el / 8;
  if (p.x2) q.x2 = (const char*)p.x2 + in_pix * p.Cx2 * ES;
  q.w = (const char*)p.w + (size_t)r * p.w_rep;
  if (p.w2) q.w2 = (const char*)p.w2 + (size_t)r * p.w2_rep;
  if (p.bias) q.bias = p.bias + (size_t)r * p.bias_rep;
  q.Nimg = (int)Nr;
  q.M = p.M / p.nrep;
  q.nrep = 1;
  return q;
}

// True if no tile of any kernel variant (at most 256 rows) can hold pixels of two data-groups.
inline bool replicas_tile_aligned(const ConvParams& p) {
  const int Nr = p.Nimg / p.nrep;
  if (p.dgrad && p.stride == 2) {  // rows are enumerated per parity class of the output grid
    for (int cls = 0; cls < 4; ++cls) {
      const int Hc = (p.Ho - (cls >> 1) + 1) >> 1, Wc = (p.Wo - (cls & 1) + 1) >> 1;
      if ((Nr * Hc * Wc) % 256 != 0) return false;
    }
  }
  return (Nr * p.Ho * p.Wo) % 256 == 0;
}

template <typename T>
int launch_conv_one(const ConvParams& p, hipStream_t s);

template <typename T>
int launch_conv_t(const ConvParams& p, hipStream_t s) {
  if (p.nrep > 1 && (p.Nimg % p.nrep != 0 || !replicas_tile_aligned(p))) {
    int family = 1;  // one launch per data-group
    for (int r = 0; r < p.nrep; ++r) family &= launch_conv_one<T>(replica_slice<T>(p, r), s);
    return family;
  }
  return launch_conv_one<T>(p, s);
}

template <typename T>
int launch_conv_one(const ConvParams& p, hipStream_t s) {
  constexpr int BKB = 64;
  if (sizeof(T) == 2 && launch_conv_narrow(p, s)) return 1;
  if (launch_dma<T>(p, s)) return 1;
  // dgrad of a stride-2 convolution: workgroups per parity class (class (0,0) is the largest)
  const bool s2 = p.dgrad && p.stride == 2 && p.Cx % (BKB / (int)sizeof(T)) == 0 &&
                  (p.x2 == nullptr || p.Cx2 % (BKB / (int)sizeof(T)) == 0);
  const int mc = p.Nimg * ((p.Ho + 1) / 2) * ((p.Wo + 1) / 2);
  if (p.ldy <= 32 && !s2) {  // narrow layers (16 / 32 output channels): half the padded columns
    dim3 grid(cdiv(p.M, 256), 1);
    if (p.dgrad) conv_gemm_kernel<T, 256, 32, 64, 32, BKB, true><<<grid, 256, 0, s>>>(p, 0);
    else conv_gemm_kernel<T, 256, 32, 64, 32, BKB, false><<<grid, 256, 0, s>>>(p, 0);
  } else if (p.ldy <= 64) {
    const int tpc = cdiv(mc, 256);
    dim3 grid(s2 ? 4 * tpc : cdiv(p.M, 256), cdiv(p.ldy, 64));
    if (s2) conv_gemm_kernel<T, 256, 64, 64, 64, BKB, true, true><<<grid, 256, 0, s>>>(p, tpc);
    else if (p.dgrad) conv_gemm_kernel<T, 256, 64, 64, 64, BKB, true><<<grid, 256, 0, s>>>(p, 0);
    else conv_gemm_kernel<T, 256, 64, 64, 64, BKB, false><<<grid, 256, 0, s>>>(p, 0);
  } else {
    const int tpc = cdiv(mc, 128);
    dim3 grid(s2 ? 4 * tpc : cdiv(p.M, 128), cdiv(p.ldy, 128));
    if (s2) conv_gemm_kernel<T, 128, 128, 64, 64, BKB, true, true><<<grid, 256, 0, s>>>(p, tpc);
    else if (p.dgrad) conv_gemm_kernel<T, 128, 128, 64, 64, BKB, true><<<grid, 256, 0, s>>>(p, 0);
    else conv_gemm_kernel<T, 128, 128, 64, 64, BKB, false><<<grid, 256, 0, s>>>(p, 0);
  }
  return 0;
}

template <int TWLOG, int THLOG, bool S2>
void launch_wgrad_dma_inst(const WgradParams& p, const WgradGeom& wg, int nsub, hipStream_t s) {
  constexpr int TW = 1 << TWLOG, TH = 1 << THLOG;
  constexpr int PROW = ((128 / (TW * TH)) * (TH + 2) * (TW + 2) + 7) / 8 * 8;
  static bool attr_set = false;
  if (!attr_set) {
    (void)hipFuncSetAttribute((const void*)wgrad_dma_kernel<TWLOG, THLOG, S2>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    attr_set = true;
  }
  const int smem = 2 * (16384 + PROW * 128) + 1024;  // RING slots + dump block
  dim3 grid(cdiv(p.Mout, 64), nsub * wg.cblocks, p.nsplit);
  wgrad_dma_kernel<TWLOG, THLOG, S2><<<grid, S2 ? 256 : 768, smem, s>>>(p, wg, p.zeros);
}

// bf16 problems whose splits are whole 128-pixel tiles go to the asynchronous kernel: 3x3
// stride 1 pad 1, and the stride-2 layers (3x3 pad 1, 1x1 pad 0) on even-sized images.
// On success: sub-pixels served (1 for stride 1), 64-channel blocks, tile geometry.
bool wgrad_dma_eligible(const WgradParams& p, int* nsub_out, int* cblocks_out, int* lw_out = nullptr, int* th_log_out = nullptr,
                        int* tiles_h_out = nullptr) {
  const bool s1 = p.R == 3 && p.S == 3 && p.stride == 1 && p.pad == 1 && p.H == p.Ho && p.W == p.Wo;
  const bool s2 = p.stride == 2 && p.R == p.S && ((p.R == 3 && p.pad == 1) || (p.R == 1 && p.pad == 0)) &&
                  p.H == 2 * p.Ho && p.W == 2 * p.Wo;
  if (!s1 && !s2) return false;
  // every data-group's pixels are whole 128-pixel tiles, and no split is empty
  if (p.nrep < 1 || p.nsplit % p.nrep != 0 || p.P % (128 * p.nrep) != 0 || p.nsplit > p.P / 128) return false;
  if (p.Cx % 8 != 0 || (p.Cx > 64 && p.Cx % 64 != 0) || p.zeros == nullptr) return false;
  // byte offsets of patch rows relative to the tile origin are 32-bit
  if ((long long)(128 + 2 * p.W + 4) * 4 * p.Cx * 2 >= (1ll << 31) || p.Cx * 2 + 256 > kZeroBytes) return false;
  const int lw = ilog2_exact(p.Wo), lh = ilog2_exact(p.Ho);
  if (lw < 2 || lh < 0 || p.Wo > 32) return false;
  int th_log, tiles_h;
  if (p.Ho * p.Wo >= 128) { th_log = 7 - lw; tiles_h = p.Ho >> th_log; if (th_log > lh) return false; }
  else { th_log = lh; tiles_h = 1; }
  if (!((lw == 5 && th_log == 2) || (lw == 4 && th_log == 3) || (lw == 3 && th_log == 3) || (lw == 2 && th_log == 2))) return false;
  *nsub_out = s2 && p.R == 3 ? 4 : 1;
  *cblocks_out = cdiv(p.Cx, 64);
  if (lw_out) *lw_out = lw;
  if (th_log_out) *th_log_out = th_log;
  if (tiles_h_out) *tiles_h_out = tiles_h;
  return true;
}

bool launch_wgrad_dma(const WgradParams& p, hipStream_t s) {
  int nsub_e, cblocks, lw, th_log, tiles_h;
  if (!wgrad_dma_eligible(p, &nsub_e, &cblocks, &lw, &th_log, &tiles_h)) return false;
  const bool s2 = p.stride == 2;
  WgradGeom wg{};
  wg.tiles_h = tiles_h;
  wg.cblocks = cblocks;
  wg.xcd_remap = p.nsplit % 8 == 0 ? 1 : 0;
  int nsub = 1;
  if (s2) {
    // real tap for (virtual tap, sub-pixel offset): 3x3 pad 1: rows 2oy-1, 2oy, 2oy+1; 1x1 pad 0: row 2oy
    if (p.R == 3) { wg.rmap[0][0] = -1; wg.rmap[0][1] = 0; wg.rmap[1][0] = 1; wg.rmap[1][1] = 2; }
    else { wg.rmap[0][0] = -1; wg.rmap[0][1] = -1; wg.rmap[1][0] = 0; wg.rmap[1][1] = -1; }
    nsub = 0;
    // heaviest sub-pixels first: (1,1) accumulates four taps, (0,0) one
    for (int sub = 3; sub >= 0; --sub) {
      const int dy = sub >> 1, dx = sub & 1;
      const bool any_r = wg.rmap[0][dy] >= 0 || wg.rmap[1][dy] >= 0, any_s = wg.rmap[0][dx] >= 0 || wg.rmap[1][dx] >= 0;
      if (any_r && any_s) wg.sub[nsub++] = sub;
    }
  }
#define DDS_WG_CASE(TWL, THL)                                                        \
  if (lw == TWL && th_log == THL) {                                                  \
    if (s2) launch_wgrad_dma_inst<TWL, THL, true>(p, wg, nsub, s);                   \
    else launch_wgrad_dma_inst<TWL, THL, false>(p, wg, nsub, s);                     \
    return true;                                                                     \
  }
  DDS_WG_CASE(5, 2) DDS_WG_CASE(4, 3) DDS_WG_CASE(3, 3) DDS_WG_CASE(2, 2)
#undef DDS_WG_CASE
  return false;
}

template <typename T>
int launch_wgrad_t(const WgradParams& p, hipStream_t s) {
  constexpr int CE = 16 / sizeof(T);
  if (sizeof(T) == 2 && launch_wgrad_narrow(p, s)) return 1;
  if (sizeof(T) == 2 && launch_wgrad_dma(p, s)) return 1;
  if (p.Mout <= 64 && p.NK + CE <= 128) {  // e.g. the stem: 3 input channels, 9 taps
    dim3 grid(cdiv(p.Mout, 64), 1, p.nsplit);
    wgrad_gemm_kernel<T, 64, 128, 32, 64><<<grid, 256, 0, s>>>(p);
  } else if (p.Mout <= 64) {
    dim3 grid(cdiv(p.Mout, 64), cdiv(p.NK + CE, 256), p.nsplit);
    wgrad_gemm_kernel<T, 64, 256, 64, 64><<<grid, 256, 0, s>>>(p);
  } else {
    dim3 grid(cdiv(p.Mout, 128), cdiv(p.NK + CE, 128), p.nsplit);
    wgrad_gemm_kernel<T, 128, 128, 64, 64><<<grid, 256, 0, s>>>(p);
  }
  return 0;
}

}  // namespace

int launch_conv(int dt, const ConvParams& p, hipStream_t s) {
  return dt == DT_F32 ? launch_conv_t<float>(p, s) : launch_conv_t<bf16_t>(p, s);
}

int launch_wgrad(int dt, const WgradParams& p, hipStream_t s) {
  return dt == DT_F32 ? launch_wgrad_t<float>(p, s) : launch_wgrad_t<bf16_t>(p, s);
}

int wgrad_choose_split(int dt, const WgradParams& shape, int W, int target_wgs) {
  const int Mout = shape.Mout, NK = shape.NK, P = shape.P;
  const int per_replica = P / W;  // pixels of one replica's mini-batch
  if (dt != DT_F32) {
    if (const int n = wgrad_narrow_split(shape, W)) return n;
    // Asynchronous kernel: 64 x 64 output blocks per (sub-pixel, channel block); a data-group's 128-pixel
    // tiles are dealt to its splits. Take the fewest splits that give the launch target_wgs workgroups:
    // the partial sums cost HBM traffic (written here, read by the update) in proportion to the split
    // count. Measured on the ResNet-18 step (four modules on four hardware queues): 1024 / 512 workgroups cost
    // 3.45 / 3.13 ms against 2.64 at 256 under an earlier stream layout; now 64 / 128 / 192 / 256 -> 2.59 / 2.47 /
    // 2.46 / 2.48 ms. With two modules (ResNet-20 shapes) 256 beats 128 (1.47 vs 1.67 ms): the caller passes 128
    // when three or more modules share the chip (half the partial-sum traffic at equal speed), else 256.
    WgradParams probe = shape;
    probe.nsplit = W;
    probe.nrep = W;
    int nsub = 0, cblocks = 0;
    if (wgrad_dma_eligible(probe, &nsub, &cblocks)) {
      const int blocks = cdiv(Mout, 64) * nsub * cblocks;
      const int rep_tiles = per_replica / 128;
      // a stride-2 workgroup has four waves where a stride-1 one has twelve, and the four sub-pixels of a 3x3
      // kernel carry 4 : 2 : 2 : 1 taps: twice the workgroups (2.24 ms per ResNet-18 step; 2.26 with one or four times)
      if (shape.stride == 2) target_wgs *= 2;
      int q = cdiv(target_wgs, blocks * W);
      if (q > rep_tiles) q = rep_tiles;
      if (q * W > 256) q = 256 / W;
      if (q < 1) q = 1;
      probe.nsplit = W * q;
      if (wgrad_dma_eligible(probe, &nsub, &cblocks)) return W * q;  // the launch will take the same decision
    }
  }
  const int ce = dtype_ce(dt);
  const int bke = 128 / dtype_size(dt);
  int tiles = (Mout <= 64) ? cdiv(Mout, 64) * cdiv(NK + ce, 256) : cdiv(Mout, 128) * cdiv(NK + ce, 128);
  int q = cdiv(1024, tiles * W);  // aim at ~1024 workgroups (512 and 256 measured slower on the fp32 CNN: 2.33-2.35 vs 2.25 ms)
  int qmax = per_replica / (2 * bke);  // at least two k-tiles per split
  if (qmax < 1) qmax = 1;
  if (q > qmax) q = qmax;
  if (q * W > 256) q = 256 / W;
  if (q < 1) q = 1;
  while (q > 1 && per_replica % q != 0) --q;  // splits never straddle replicas
  return W * q;
}

}  // namespace dds
