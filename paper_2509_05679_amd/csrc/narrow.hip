// Kernels for the narrow layers (16 channels: the first stage of the ResNet-20 / ResNet-56 shapes), bf16.
//
// At 16 channels a 3x3 convolution does 4.6 kFLOP per pixel against 64-96 bytes of traffic: it is bound by
// memory, not by the matrix unit, and a tile sized for wide layers (64 or more output columns, operands staged
// in LDS) spends its time on padding. These kernels use v_mfma_f32_16x16x32_bf16 with the 16 output channels as
// the rows and 16 consecutive pixels as the columns of one accumulator tile, and keep everything else out of
// the way:
//   forward / dgrad: all nine taps of the weights (4.6 KB) live in registers as the A operand; the B operand of
//   a tap is read straight from global memory, 16 bytes per lane (eight channels of one pixel, shifted by the
//   tap) -- neighbouring taps re-read the same cache lines from the vector cache, so no LDS and no barrier;
//   weight gradient: see wgrad16_kernel below.
#include "kernels.h"

namespace dds {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;

__device__ __forceinline__ uint32_t pack_bf16_rne(float lo, float hi) {
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

__device__ __forceinline__ f32x4_t mfma16(const uint4& a, const uint4& b, f32x4_t c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}

// 3x3, stride 1, pad 1, 16 input channels (channel stride 16), at most 16 output channels (stride 16).
// One wave owns GROUPS runs of 16 consecutive pixels of the flattened (image, row, column) index; the image width
// is a multiple of 16, so a run lies inside one image row. Lane l = 16 g + j holds, as B operand of MFMA t,
// channels 8 (g & 1) .. +8 of pixel j shifted by tap 2 t + (g >> 1), and as A operand the same k-slice of weight
// row j; the accumulator gives it output channels 4 g .. 4 g + 3 of pixel j: one 8-byte store, and the four lane
// groups together write the 512 contiguous bytes of the run.
// DGRAD: x is the output gradient, w the transposed snapshot [cin][tap][cout], tap (r, s) gathers at
// (h + 1 - r, w + 1 - s); the epilogue options are the ones of ConvParams.
template <bool DGRAD, int GROUPS>
__global__ __launch_bounds__(256) void conv16_direct_kernel(ConvParams p) {
  const int lane = threadIdx.x & 63;
  const int wave = (blockIdx.x * 256 + threadIdx.x) >> 6;
  const int j = lane & 15, g = lane >> 4;
  const int half = g & 1;
  const int ngroups = p.M >> 4;
  const int grp0 = wave * GROUPS;
  if (grp0 >= ngroups) return;
  const int HW = p.H * p.W;

  const char* wbase = (const char*)p.w;
  const float* bias = p.bias;
  if (p.nrep > 1) {  // a run never leaves its image, a workgroup may: weights are picked per wave
    const int img = (grp0 << 4) / HW;
    const int r = min(img / (p.Nimg / p.nrep), p.nrep - 1);
    wbase += (size_t)r * p.w_rep;
    if (bias) bias += (size_t)r * p.bias_rep;
  }
  // weights: MFMA t, lane (j, g): row j, tap 2 t + (g >> 1), channels 8 half .. +8; zero past Nout and past tap 8
  uint4 wa[5];
  int dr[5], ds[5];
  bool tap_ok[5];
#pragma unroll
  for (int t = 0; t < 5; ++t) {
    const int tap = 2 * t + (g >> 1);
    tap_ok[t] = tap < 9;
    const int tt = tap_ok[t] ? tap : 0;
    const int r = tt / 3, s = tt - 3 * r;
    dr[t] = DGRAD ? 1 - r : r - 1;
    ds[t] = DGRAD ? 1 - s : s - 1;
    const bool ok = tap_ok[t] && j < p.Nout;
    const uint4 v = *(const uint4*)(wbase + ((size_t)((ok ? j : 0) * 9 + tt) * 16 + half * 8) * 2);
    wa[t] = ok ? v : make_uint4(0u, 0u, 0u, 0u);
  }
  float ab[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int n = 4 * g + e;
    ab[e] = (bias != nullptr && n < p.Nout) ? p.alpha * bias[n] : 0.f;
  }
  const float lower = p.relu ? 0.f : -__builtin_inff();

#pragma unroll
  for (int u = 0; u < GROUPS; ++u) {
    const int grp = grp0 + u;
    if (grp >= ngroups) break;  // wave-uniform
    const int pix = (grp << 4) + j;
    const int img = pix / HW, rem = pix - img * HW;
    const int h = rem / p.W, w = rem - h * p.W;
    const char* ximg = (const char*)p.x + (size_t)img * HW * 32 + half * 16;
    uint4 xb[5];
#pragma unroll
    for (int t = 0; t < 5; ++t) {
      const int hh = h + dr[t], ww = w + ds[t];
      const bool ok = tap_ok[t] && (unsigned)hh < (unsigned)p.H && (unsigned)ww < (unsigned)p.W;
      const uint4 v = *(const uint4*)(ximg + (size_t)(ok ? hh * p.W + ww : rem) * 32);  // unconditional, clamped
      xb[t] = ok ? v : make_uint4(0u, 0u, 0u, 0u);
    }
    // epilogue operands of this lane's four channels (8 bytes each), also unconditional
    const size_t o = (size_t)pix * 16 + 4 * g;
    uint2 rs = make_uint2(0u, 0u), mk = make_uint2(0u, 0u);
    uint32_t keep = 0xfu;
    if (p.res) rs = *(const uint2*)((const uint16_t*)p.res + o);
    if (p.maskbits) keep = ((uint32_t)((const uint16_t*)p.maskbits)[pix] >> (4 * g)) & 0xfu;
    else if (p.mask) {
      mk = *(const uint2*)((const uint16_t*)p.mask + o);
      keep = ((int)(mk.x << 16) >= 0x10000 ? 1u : 0u) | ((int)mk.x >= 0x10000 ? 2u : 0u) |
             ((int)(mk.y << 16) >= 0x10000 ? 4u : 0u) | ((int)mk.y >= 0x10000 ? 8u : 0u);
    }
    f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int t = 0; t < 5; ++t) acc = mfma16(wa[t], xb[t], acc);
    const float r4[4] = {__uint_as_float(rs.x << 16), __uint_as_float(rs.x & 0xffff0000u),
                         __uint_as_float(rs.y << 16), __uint_as_float(rs.y & 0xffff0000u)};
    float v[4];
    uint32_t signs = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float t = fmaf(p.alpha, acc[e], ab[e]) + r4[e];
      t = __builtin_amdgcn_fmed3f(t, lower, __builtin_inff());
      v[e] = ((keep >> e) & 1u) ? t : 0.f;
    }
    uint2 out;
    out.x = pack_bf16_rne(v[0], v[1]);
    out.y = pack_bf16_rne(v[2], v[3]);
    *(uint2*)((uint16_t*)p.y + o) = out;
    if (p.bits_out) {
      // the sign of the stored (rounded) value, as every other producer defines the plane
      signs = ((int)(out.x << 16) >= 0x10000 ? 1u : 0u) | ((int)out.x >= 0x10000 ? 2u : 0u) |
              ((int)(out.y << 16) >= 0x10000 ? 4u : 0u) | ((int)out.y >= 0x10000 ? 8u : 0u);
      uint32_t word = signs << (4 * g);
      word |= (uint32_t)__shfl_xor((int)word, 16, 64);
      word |= (uint32_t)__shfl_xor((int)word, 32, 64);
      if (g == 0) ((uint16_t*)p.bits_out)[pix] = (uint16_t)word;
    }
  }
}


// ------------------------------------------------------------------ weight gradient, 16-channel rows
// dW[k][tap][c] = sum over pixels p of dY[p][k] * X[p + tap][c] for a 3x3 stride-1 pad-1 layer whose dY and X
// rows are 16 channels (32 bytes) wide. The reduction index is the pixel: one v_mfma_f32_16x16x32_bf16 multiplies
// 32 pixels of dY^T (16 x 32) by the same 32 pixels of the tap-shifted X (32 x 16). Workgroup z owns one split of
// the flattened (image, row) index and walks it in chunks of 256 pixels (whole image rows, never across an image):
// the dY rows and the X patch with a one-pixel halo (zeros outside the image) are parked in LDS as plain
// [pixel][16 channels] rows, and ds_read_b64_tr_b16 hands a lane four pixels of one channel from a 4 x 16 block
// (128 contiguous bytes), so nothing is transposed in registers. The four waves share the nine taps (3 + 2 + 2 + 2,
// the bias gradient rides with a two-tap wave), each reads the dY fragments itself: no reduction across waves, every
// wave writes its taps of the split's partial row. Memory-bound: 64 bytes of dY and X per pixel against 4.6 kFLOP.
typedef short s16x4_t __attribute__((ext_vector_type(4)));
#define DDS_LDS_AS __attribute__((address_space(3)))
__device__ __forceinline__ uint2 lds_tr16_b64(uint32_t lds_byte_address) {
  s16x4_t v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t DDS_LDS_AS*)(size_t)lds_byte_address);
  return __builtin_bit_cast(uint2, v);
}

struct Wgrad16Geom {
  int CH;        // image rows per chunk (CH * W = 256 pixels)
  int PW;        // patch row pitch in pixels, W + 2
  int q;         // splits per data-group
  int rows_rep;  // flattened (image, row) rows per data-group
};

__global__ __launch_bounds__(256) void wgrad16_kernel(WgradParams p, Wgrad16Geom gm) {
  extern __shared__ __align__(16) char smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int W = p.W, H = p.H, PW = gm.PW, CH = gm.CH;
  const int ybytes = 256 * 32;                 // dY chunk
  const int prow = (CH + 2) * PW;              // patch pixels
  char* ybuf = smem;
  char* xbuf = smem + ybytes;
  const uint32_t lds_y = (uint32_t)(size_t)(DDS_LDS_AS char*)ybuf;
  const uint32_t lds_x = (uint32_t)(size_t)(DDS_LDS_AS char*)xbuf;

  // split z = (data-group, j): the data-group's rows are dealt to its q splits as evenly as whole rows allow
  const int z = blockIdx.x;
  const int zr = z / gm.q, zj = z - zr * gm.q;
  const int R0 = zr * gm.rows_rep + (int)(((long long)zj * gm.rows_rep) / gm.q);
  const int R1 = zr * gm.rows_rep + (int)(((long long)(zj + 1) * gm.rows_rep) / gm.q);

  // taps of this wave: wave 0: 0, 4, 8; wave w: w, w + 4. The bias gradient (column sums of dY) rides with wave 1.
  const int ntap = wave == 0 ? 3 : 2;
  f32x4_t acc[3], accb;
#pragma unroll
  for (int t = 0; t < 3; ++t) acc[t] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  accb = f32x4_t{0.f, 0.f, 0.f, 0.f};
  const uint4 ones = make_uint4(0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u);

  // fragment addressing: 16-lane group g covers pixels 8 g .. 8 g + 7 of a 32-pixel k-step as two 4-pixel blocks;
  // lane lq of the group supplies the address of row lq >> 2, 8-byte segment lq & 3 of the block
  const int lq = lane & 15, g = lane >> 4;
  const int blkrow = lq >> 2, seg = lq & 3;

  for (int R = R0; R < R1;) {
    const int img = R / H, h0 = R - img * H;
    int nr = CH;
    if (nr > H - h0) nr = H - h0;
    if (nr > R1 - R) nr = R1 - R;
    // ---- park the chunk: dY rows (zero past the chunk's last row) and the X patch (zero outside the image)
    for (int i = tid; i < 256 * 2; i += 256) {
      const int pix = i >> 1, hf = i & 1;
      const int y = pix / W;
      uint4 v = make_uint4(0u, 0u, 0u, 0u);
      if (y < nr) v = *(const uint4*)((const char*)p.dy + ((size_t)R * W + pix) * 32 + hf * 16);
      *(uint4*)(ybuf + pix * 32 + hf * 16) = v;
    }
    for (int i = tid; i < prow * 2; i += 256) {
      const int pp = i >> 1, hf = i & 1;
      const int yy = pp / PW, xx = pp - yy * PW;
      const int gh = h0 + yy - 1, gw = xx - 1;
      uint4 v = make_uint4(0u, 0u, 0u, 0u);
      if (yy <= nr + 1 && (unsigned)gh < (unsigned)H && (unsigned)gw < (unsigned)W)
        v = *(const uint4*)((const char*)p.x + (((size_t)img * H + gh) * W + gw) * 32 + hf * 16);
      *(uint4*)(xbuf + pp * 32 + hf * 16) = v;
    }
    __syncthreads();
    // ---- 8 k-steps of 32 pixels; pixel q of the chunk sits at tile row q / W, column q % W
#pragma unroll 2
    for (int ks = 0; ks < 8; ++ks) {
      uint4 a;
      int prow0[2];
#pragma unroll
      for (int hh = 0; hh < 2; ++hh) {
        const int q0 = ks * 32 + 8 * g + 4 * hh;            // first pixel of this lane group's block
        const uint2 t = lds_tr16_b64(lds_y + (q0 + blkrow) * 32 + seg * 8);
        if (hh == 0) { a.x = t.x; a.y = t.y; } else { a.z = t.x; a.w = t.y; }
        const int y = q0 / W, x = q0 - y * W;
        prow0[hh] = y * PW + x;                              // patch pixel of the block at tap (0, 0)
      }
#pragma unroll
      for (int t = 0; t < 3; ++t) {
        if (t < ntap) {  // wave-uniform
          const int tap = wave + 4 * t;
          const int toff = (tap / 3) * PW + (tap % 3);
          const uint2 b0 = lds_tr16_b64(lds_x + (prow0[0] + toff + blkrow) * 32 + seg * 8);
          const uint2 b1 = lds_tr16_b64(lds_x + (prow0[1] + toff + blkrow) * 32 + seg * 8);
          acc[t] = mfma16(a, make_uint4(b0.x, b0.y, b1.x, b1.y), acc[t]);
        }
      }
      if (wave == 1) accb = mfma16(a, ones, accb);
    }
    __syncthreads();
    R += nr;
  }

  // D[i][j]: lane holds rows i = 4 g + e (output channel k), column j = lane & 15 (input channel c)
  float* out = p.partial + (size_t)z * p.Pl;
  const int c = lane & 15;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int k = 4 * g + e;
    if (k >= p.Mout) continue;
#pragma unroll
    for (int t = 0; t < 3; ++t)
      if (t < ntap) out[(size_t)k * p.NK + (wave + 4 * t) * 16 + c] = p.alpha * acc[t][e];
    if (wave == 1 && c == 0) out[(size_t)p.Mout * p.NK + k] = p.alpha * accb[e];
  }
}

bool wgrad16_shape_ok(const WgradParams& p) {
  if (p.R != 3 || p.S != 3 || p.stride != 1 || p.pad != 1 || p.H != p.Ho || p.W != p.Wo) return false;
  if (p.Cx != 16 || p.ldy != 16 || p.Mout > 16 || p.NK != 144) return false;
  if (p.W % 16 != 0 || 256 % p.W != 0 || p.W > 128) return false;
  if (p.P != p.Nimg * p.H * p.W) return false;
  return true;
}

}  // namespace

// True if the launch was taken: bf16, 3x3 stride 1 pad 1, 16-channel input and output rows, image width a multiple of 16.
bool launch_conv_narrow(const ConvParams& p, hipStream_t s) {
  if (p.R != 3 || p.S != 3 || p.stride != 1 || p.pad != 1 || p.H != p.Ho || p.W != p.Wo) return false;
  if (p.Cx != 16 || p.ldy != 16 || p.Nout > 16 || p.out_f32 || p.x2 != nullptr) return false;
  if (p.W % 16 != 0 || p.M % 16 != 0 || p.M != p.Nimg * p.H * p.W) return false;
  // a wave's runs (64 pixels) must not straddle two data-groups
  if (p.nrep > 1 && (p.Nimg % p.nrep != 0 || (p.H * p.W) % 64 != 0)) return false;
  constexpr int GROUPS = 4;
  const int ngroups = p.M / 16;
  const int waves = (ngroups + GROUPS - 1) / GROUPS;
  const int blocks = (waves + 3) / 4;
  if (p.dgrad) conv16_direct_kernel<true, GROUPS><<<blocks, 256, 0, s>>>(p);
  else conv16_direct_kernel<false, GROUPS><<<blocks, 256, 0, s>>>(p);
  return true;
}

// Split count of the 16-channel weight-gradient kernel for this layer (a multiple of W), or 0 if the layer is not its.
int wgrad_narrow_split(const WgradParams& shape, int W) {
  if (!wgrad16_shape_ok(shape) || W < 1 || shape.Nimg % W != 0) return 0;
  const int rows_rep = (shape.Nimg / W) * shape.H;
  const int CH = 256 / shape.W;
  // about a thousand workgroups (four a CU), at least one chunk each
  // (measured on the ResNet-56 configuration: 256 / 512 / 1024 / 2048 workgroups -> 2.94 / 2.84 / 2.79 / 2.86 ms per
  // step; the update kernel reads one partial row per split, which is what more splits cost)
  int q = (1024 + W - 1) / W;
  const int qmax = rows_rep / CH > 0 ? rows_rep / CH : 1;
  if (q > qmax) q = qmax;
  if (q < 1) q = 1;
  return W * q;
}

bool launch_wgrad_narrow(const WgradParams& p, hipStream_t s) {
  if (!wgrad16_shape_ok(p) || p.nrep < 1 || p.nsplit % p.nrep != 0 || p.Nimg % p.nrep != 0) return false;
  Wgrad16Geom gm;
  gm.CH = 256 / p.W;
  gm.PW = p.W + 2;
  gm.q = p.nsplit / p.nrep;
  gm.rows_rep = (p.Nimg / p.nrep) * p.H;
  if (gm.q < 1 || gm.q > gm.rows_rep) return false;  // no empty split
  const int smem = 256 * 32 + (gm.CH + 2) * gm.PW * 32;
  wgrad16_kernel<<<p.nsplit, 256, smem, s>>>(p, gm);
  return true;
}

}  // namespace dds
