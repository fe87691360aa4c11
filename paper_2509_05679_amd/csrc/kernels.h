// Launch interface between the host engine and the HIP kernels (gfx950 only).
// Internal to the library: plain structs of device pointers and sizes.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dds {

enum DType : int { DT_F32 = 0, DT_BF16 = 1 };

inline int dtype_size(int dt) { return dt == DT_F32 ? 4 : 2; }
// channels per 16-byte chunk; every tensor's channel stride is a multiple of this
inline int dtype_ce(int dt) { return dt == DT_F32 ? 4 : 8; }

// Implicit-GEMM convolution / linear, forward or input-gradient (dgrad) form.
//   y[m, n] = epilogue( sum_{tap, c} gather(x; m, tap)[c] * w[n, tap, c] )
// forward : m = (img, ho, wo), gathers x at (ho*stride - pad + r, wo*stride - pad + s)
// dgrad   : m = (img, h, w) of the conv input, x is the output gradient, gathers at
//           ((h + pad - r)/stride, (w + pad - s)/stride) when divisible, w is the
//           transposed weight snapshot [cin][tap][cout_padded]
// epilogue: v = alpha * (acc + bias[n]); v += res[m, n]; relu; v = mask[m, n] > 0 ? v : 0
// Size of the block of zeros every launch may read padding from: at least one pixel row
// (all channels of one pixel) of any tensor the asynchronous kernels accept.
constexpr int kZeroBytes = 16384;

struct ConvParams {
  const void* x;
  const void* w;
  void* y;
  const float* bias;  // fp32 [Nout] or null
  const void* res;    // same layout as y (dtype T) or null
  const void* mask;   // same layout as y (dtype T) or null
  // Sign planes of ReLU outputs: [pixel][ldy / 8] bytes, bit c % 8 of byte c / 8 set iff channel c
  // of the stored tensor is > 0 (needs ldy % 8 == 0). bits_out: written with y by a forward launch
  // with relu. maskbits: what a dgrad launch multiplies by instead of reading `mask` (the full tensor).
  void* bits_out;
  const void* maskbits;
  // dgrad of a stride-2 layer only: gradient of a 1x1 stride-2 pad-0 shortcut that shares this
  // layer's input, folded in as extra reduction steps. x2: [Nimg][H][W][Cx2] (same pixel grid as x),
  // w2: [Nout][Cx2]; output pixel (oh, ow) with oh, ow even receives sum_k x2[oh/2, ow/2, k] * w2[n][k].
  const void* x2;
  const void* w2;
  int Cx2;
  const void* zeros;  // kZeroBytes zero bytes (source of padding rows for LDS fills)
  int Nimg, H, W, Cx; // gathered tensor: NHWC, channel stride Cx (= GEMM-K per tap)
  int Ho, Wo;         // pixel grid of y; M = Nimg*Ho*Wo
  int M;
  int Nout;           // valid rows of w
  int ldy;            // channel stride of y / res / mask
  int R, S, stride, pad;
  int Ktot;           // R*S*Cx
  float alpha;
  int relu;
  int out_f32;        // y is fp32 regardless of T (logits)
  int dgrad;
  // Data-groups with weights of their own (general mixing matrix): the Nimg images are nrep equal
  // groups of consecutive images and group r multiplies by w + r*w_rep bytes, adds bias + r*bias_rep
  // floats and (folded shortcut) uses w2 + r*w2_rep bytes. nrep <= 1: one weight set for all images.
  int nrep;
  long long w_rep, w2_rep, bias_rep;
};

// Weight-gradient GEMM with split reduction:
//   partial[z][m*NK + n] = alpha * sum_{p in split z} dy[p, m] * gather(x; p, n)
//   partial[z][Mout*NK + m] = alpha * sum_p dy[p, m]                (bias gradient)
// m = output channel, n = (tap, c), p = output pixel (img, ho, wo).
struct WgradParams {
  const void* dy;   // [P][ldy]
  const void* x;    // [Nimg][H][W][Cx]
  float* partial;   // [nsplit][Pl]
  const void* zeros; // kZeroBytes zero bytes
  int Nimg, H, W, Cx, Ho, Wo;
  int Mout;         // real output channels
  int ldy;
  int R, S, stride, pad;
  int NK;           // R*S*Cx
  int P;            // Nimg*Ho*Wo
  int pix_per_split; // generic kernel: pixels per split (P / nsplit, splits are equal)
  int nsplit;
  int nrep;          // data-groups: equal runs of consecutive images; nsplit is a multiple of it and no split
                     // holds pixels of two data-groups (the asynchronous kernel deals each group's 128-pixel
                     // tiles to its nsplit / nrep splits as evenly as whole tiles allow)
  long long Pl;     // floats between consecutive splits (>= Mout*NK + Mout)
  float alpha;
};

// Training-mode batch normalisation of a [W * rows_per_rep][ld] tensor, statistics per data-group.
//   forward : y = relu?( alpha * (gamma * (x - mean) * rstd + beta) + res ), stats <- mean, rstd, gamma
//   backward: dgamma / dbeta partial rows (one per (data-group, split)), dx from dy, x and the saved stats
struct BnParams {
  const void* x;      // input of the normalisation (the convolution output), dtype T
  void* y;            // forward output, dtype T
  const void* res;    // added after the normalisation (same layout as y) or null
  void* bits_out;     // sign plane of y ([row][ld / 8] bytes) or null
  const void* dy;     // backward: gradient with respect to y (already masked by y > 0 where relu)
  void* dx;           // backward: gradient with respect to x
  const float* gamma; // fp32 master: gamma[c * gstride]
  const float* beta;  // beta[c]
  long long rep_stride;  // floats between the parameters of consecutive data-groups (0: shared)
  int gstride;
  float* stats;       // [W][3][ld]: mean, rstd, gamma of this mini-batch
  double* scratch;    // [W][nsplit][ld][2] per-split sums (forward: x, x^2; backward: g, g * xhat)
  double* totals;     // backward: [W][ld][2] dbeta, dgamma per data-group
  float* partial;     // backward: [W][pstride] parameter-gradient rows, one per data-group
  long long pstride;
  int W, C, ld, nsplit;
  long long rows_per_rep, rows_per_split;
  float eps, alpha;
  int relu;
};

struct IngestParams {
  const float* x[32];
  const int32_t* y[32];
  void* dst;        // [W*B][H][W][Cpad] dtype T
  int32_t* labels;  // [W*B]
  int W, B, C, HW, Cpad;
};

// One entry per parameter tensor block of a module (weights followed by bias).
struct UpdateDesc {
  float* master;        // [n] fp32, internal layout
  float* momentum;      // [n] or null
  const float* partial; // [nsplit][n]
  void* work;           // compute-precision copy [n] or null (fp32 path uses master)
  void* stash;          // transposed snapshots [slot][Cin][RS][Coutpad] or null
  long long stash_slot_elems;
  long long n;          // Cout*RS*Cinpad + Cout
  long long pstride;    // floats between consecutive splits of `partial` (n rounded up to 4)
  int nsplit;
  int Cout, RS, Cinpad, Cin, Coutpad;
};

// Both return the kernel family that took the launch: 0 = generic implicit GEMM (register-staged),
// 1 = the asynchronous global->LDS kernels (conv3x3_dma_kernel / wgrad_dma_kernel).
int launch_conv(int dt, const ConvParams& p, hipStream_t s);
// bf16 3x3 stride-1 layers with 16-channel rows (narrow.hip); false: not taken, nothing launched
bool launch_conv_narrow(const ConvParams& p, hipStream_t s);
int launch_wgrad(int dt, const WgradParams& p, hipStream_t s);
// bf16 3x3 stride-1 layers with 16-channel rows (narrow.hip): the split count such a layer gets (0: not its), and
// the launch (false: not taken, nothing launched)
int wgrad_narrow_split(const WgradParams& shape, int W);
bool launch_wgrad_narrow(const WgradParams& p, hipStream_t s);
// Chooses the split count of the pixel reduction for a wgrad problem: a multiple of the replica
// count W, so that no split mixes two replicas. shape: every field that describes the layer
// (Nimg, H, W, Cx, Ho, Wo, Mout, ldy, R, S, stride, pad, NK, P, zeros non-null); nsplit,
// pix_per_split and the pointers are ignored.
// target_wgs: workgroups the asynchronous kernel's launch should reach (fewer splits = less partial-sum traffic).
int wgrad_choose_split(int dt, const WgradParams& shape, int W, int target_wgs);

void launch_ingest(int dt, const IngestParams& p, hipStream_t s);
void launch_maxpool_fwd(int dt, const void* x, void* y, int N, int H, int W, int C, hipStream_t s);
void launch_maxpool_bwd(int dt, const void* dy, const void* x, void* dx, int N, int H, int W, int C,
                        int relu_mask, hipStream_t s);
void launch_gap_fwd(int dt, const void* x, void* y, int N, int HW, int C, hipStream_t s);
void launch_gap_bwd(int dt, const void* dy, const void* x, void* dx, int N, int HW, int C, int relu_mask,
                    hipStream_t s);
// logits fp32 [W*B][ldl]; dlogits dtype T [W*B][ldg] (may be null); loss [W] (may be null)
void launch_softmax_ce(int dt, const float* logits, const int32_t* labels, void* dlogits, float* loss,
                       int W, int B, int classes, int ldl, int ldg, hipStream_t s);
// descs: device array of UpdateDesc; block_map: device array of (descriptor, block)
// pairs, one per workgroup of 1024 elements.
// update: g = (1/W) sum over splits, momentum, SGD on the fp32 master, recast into `work`.
void launch_update(int dt, const UpdateDesc* descs_dev, const int* block_map_dev, int total_blocks, int W,
                   float lr, float mu, hipStream_t s);
// General mixing matrix (W weight copies, rep_stride elements apart; a descriptor's nsplit = splits per data-group):
// u_r = w_r - lr*direction_r from data-group r's own splits, then w_s = sum_r P[s][r] u_r into master
// and `work`. descs / block_map / total_blocks: the entries of data-group 0. P: device, W x W row-major.
void launch_gossip_update(int dt, const UpdateDesc* descs_dev, const int* block_map_dev, int total_blocks,
                          const float* P_dev, int W, long long rep_stride, float lr, float mu, hipStream_t s);
// Squared distances to the data-group mean: out[(2*b + part) * W + s] for workgroup b of the
// update block map of data-group 0 (1024 elements of one layer each); part 0 = weight, 1 = bias; fp64.
void launch_consensus(const UpdateDesc* descs_dev, const int* block_map_dev, int total_blocks, int W,
                      long long rep_stride, double* out_dev, hipStream_t s);
// work <- master
void launch_recast(int dt, const UpdateDesc* descs_dev, const int* block_map_dev, int total_blocks,
                   hipStream_t s);
// stash[slot] <- transpose(master); block_map enumerates blocks of Cin*RS*Coutpad elements
void launch_stash(int dt, const UpdateDesc* descs_dev, const int* block_map_dev, int total_blocks, int slot,
                  hipStream_t s);
// three kernels each: per-split sums, their fold per data-group and channel, the streaming pass
void launch_bn_forward(int dt, const BnParams& p, hipStream_t s);
void launch_bn_backward(int dt, const BnParams& p, hipStream_t s);
// canonical [Cout][Cin][R][S] (+bias) <-> internal [Cout][RS][Cinpad] (+bias)
void launch_param_permute(const float* canon, float* internal, int Cout, int Cin, int RS, int Cinpad,
                          int to_internal, hipStream_t s);
void launch_fill_zero(void* p, size_t bytes, hipStream_t s);

}  // namespace dds
