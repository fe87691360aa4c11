// Host engine of libdds: validates the layer spec, fuses it into kernel nodes, lays
// the arena out (activation rings, weight snapshots, error mailboxes, gradient
// partials, master weights) and enqueues one training iteration per dds_step.
//
// Data flow (Section 3.2 / Algorithm 1 of the paper): at iteration t module k0
// forwards batch t-k0 into ring slot t mod R, back-propagates batch t-k0-2d from
// ring slot (t-2d) mod R with the transposed weight snapshot of the same slot and
// the error gradient module k0+1 left in the mailbox, then applies the replica-mean
// SGD update and snapshots the new weights into slot (t+1) mod R. A module reads its
// input activation directly from the ring of the module below (no copy): that slot
// stays live two iterations longer than the reader needs it.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdlib>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

#include "../../include/dds.h"
#include "kernels.h"

using namespace dds;

namespace {

thread_local std::string g_err;

int fail(int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_err = buf;
  return code;
}

#define HIP_TRY(expr)                                                                      \
  do {                                                                                     \
    hipError_t e_ = (expr);                                                                \
    if (e_ != hipSuccess) return fail(DDS_EHIP, "%s failed: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline int round_up(int x, int a) { return (x + a - 1) / a * a; }

constexpr int G_NONE = -1;     // no gradient wanted
constexpr int G_ERR_IN = -2;   // mailbox filled by module k0+1 (gradient of this module's output)
constexpr int G_ERR_OUT = -3;  // mailbox read by module k0-1 (gradient of this module's input)

enum TensorKind { T_RING, T_TEMP, T_EXTERNAL };
enum NodeKind { N_CONV, N_MAXPOOL, N_GAP, N_CE, N_BN };

struct Tensor {
  int C = 0, Cpad = 0, H = 0, W = 0;
  int dt = DT_F32;
  int kind = T_RING;
  bool relu_out = false;
  size_t bytes = 0;     // whole mini-batch of all replicas
  size_t ring_off = 0;  // offset inside a ring slot (T_RING), or inside the module's recompute area
  bool recomputed = false;  // T_RING tensor that is not kept per slot: one copy, rebuilt before the backward pass
  bool has_bits = false;  // a sign plane (one bit per element, > 0) is kept beside the tensor in its ring slot
  size_t bits_off = 0;
  char* temp = nullptr; // T_TEMP storage
  int grad = G_NONE;    // gradient buffer id
};

struct ParamLayer {
  int Cout, Cin, R, RS, Cinpad, Coutpad, stride, pad;
  long long n;        // Cout*RS*Cinpad + Cout
  long long pstride;  // n rounded up to 4
  long long off;      // element offset in the module's master array
  int nsplit = 0;
  bool need_stash = false;
  float* partial = nullptr;
  char* stash = nullptr;  // [copies][R_k][Cin*RS*Coutpad] compute dtype
  long long stash_elems = 0;
  size_t stash_slot_bytes = 0;  // one snapshot, rounded up to 256 bytes
};

struct Node {
  int kind;
  int in = -1, out = -1;
  int layer = -1;
  bool relu = false;
  int res = -1;       // tensor added in the forward epilogue
  float alpha = 1.f;
  int gout = G_NONE, gin = G_NONE, addend = G_NONE;
  bool mask_in = false;
  bool out_f32 = false;
  // batch normalisation (N_BN): layer = its gamma / beta block
  float eps = 0.f;
  size_t stats_off = 0;    // mean, rstd, gamma of the forwarded mini-batch, inside the ring slot
  int bn_nsplit = 0;       // row splits per data-group
  long long bn_rows_per_split = 0;
  int fold_sc = -1;        // first conv of a projection block: node of the 1x1 shortcut whose dgrad rides in this one's
  bool dgrad_folded = false;  // shortcut node: no dgrad launch of its own
};

struct GradBuf {
  size_t bytes = 0;
  char* ptr = nullptr;
};

struct Module {
  int k0 = 0, d = 0, R = 1;
  std::vector<Tensor> tensors;
  std::vector<Node> nodes;
  std::vector<ParamLayer> layers;  // canonical (spec) order
  std::vector<GradBuf> grads;
  size_t slot_bytes = 0;
  char* ring = nullptr;
  // Recompute policy (modules with d > 0): a ring slot keeps only what other iterations or modules read (the
  // module's output with its sign plane; module 0's ingested input); every other saved tensor and the batch-norm
  // statistics have one copy in `area`, which the forward pass fills for mini-batch f and a second forward pass,
  // run on the ring's input with the parameter snapshot of that slot, refills for mini-batch b before the backward.
  bool recompute = false;
  char* area = nullptr;
  float* snap_master = nullptr;  // [R][copies][n_master] fp32 parameters as the forward of that slot saw them
  char* snap_work = nullptr;     // the same for the compute-precision copy (bf16 path)
  double* bn_scratch = nullptr;  // per-split sums of the batch-normalisation kernels (largest node of the module)
  double* bn_totals = nullptr;   // dbeta / dgamma per data-group and channel of the node being back-propagated
  long long n_master = 0;  // floats per weight copy
  float* master = nullptr;    // [copies][n_master]
  float* momentum = nullptr;  // [copies][n_master]
  char* work = nullptr;       // compute-precision copy (bf16 path), [copies][n_master]
  double* cons_dev = nullptr; // [blocks_update][2][W] squared distances to the mean (general mixing matrix only)
  std::vector<int> map_update_host;  // (layer, block) pairs of weight copy 0
  // error mailbox written by module k0+1, read by this module
  int err_depth = 0;
  size_t err_bytes = 0;
  char* err = nullptr;
  UpdateDesc* descs_dev = nullptr;
  int* map_update_dev = nullptr;
  int* map_stash_dev = nullptr;
  int blocks_update = 0, blocks_stash = 0;
  int out_tensor = -1;
  long long canon_params = 0;
  hipStream_t stream = nullptr;
  hipEvent_t done[2] = {nullptr, nullptr};  // end of this module's program, by step parity
};

struct Arena {
  char* base = nullptr;
  size_t size = 0, used = 0;
  bool dry = true;
  char* take(size_t bytes) {
    size_t off = align_up(used, 256);
    used = off + bytes;
    if (dry) return nullptr;
    return base + off;
  }
};

}  // namespace

struct dds_ctx {
  int K = 0, W = 0, B = 0, N = 0;
  int dt = DT_F32;
  int classes = 0;
  int in_c = 0, in_h = 0, in_w = 0;
  float lr = 0.f, mu = 0.f;
  std::vector<int> d;
  std::vector<Module> mods;
  int label_depth = 0;
  int32_t* labels = nullptr;  // [label_depth][N]
  float* loss = nullptr;      // [W]
  char* zeros = nullptr;      // kZeroBytes zero bytes
  int64_t t = 0;
  bool have_loss = false;
  hipEvent_t fork = nullptr;
  // True while the done events of the previous iteration describe everything a module program depends on:
  // cleared by every call that touches module state from the caller's stream outside dds_step.
  bool chained = false;
  bool recompute = false;  // activation policy of the spec (applies to modules with d > 0)
  hipStream_t last_stream = nullptr;  // stream of the previous dds_step
  hipEvent_t step_end = nullptr;      // recorded on it after that step's joins
  std::vector<hipStream_t> pool;  // internal streams; module k0 runs on the caller's stream if k0 % (pool+1) == 0
  int64_t launches = 0;
  double gemm_flops = 0.0;
  size_t arena_used = 0;
  // general mixing matrix (Section 2.3): `copies` = W weight copies per module instead of one
  bool gossip = false;
  int copies = 1;
  std::vector<float> P;    // host, W x W
  float* P_dev = nullptr;
  bool serial = false;  // DDS_SERIAL=1 in the environment at dds_create: modules run one after another on the
                        // caller's stream (per-kernel timing without other modules sharing the chip)
  // optional per-launch timing of the MFMA kernels (events on the launching stream)
  bool profiling = false;
  bool profile_serial = false;  // dds_profile(ctx, 2): modules run one after another while profiling
  struct ProfRec { int cls; double flops; hipEvent_t a, b; };
  std::vector<ProfRec> prof_pending;
  std::vector<hipEvent_t> prof_pool;
  // classes: 0 forward, 1 dgrad, 2 wgrad on the generic kernels; 3, 4, 5 the same on the asynchronous kernels
  double prof_ms[6] = {}, prof_flops[6] = {};
  long long prof_count[6] = {};
};

namespace {

int check_delays(int K, const int* delays, std::vector<int>& d) {
  d.resize(K);
  for (int k = 0; k < K; ++k) d[k] = delays ? delays[k] : K - 1 - k;
  if (d[K - 1] < 0) return fail(DDS_EINVAL, "delay of the last module must be >= 0");
  for (int k = 0; k + 1 < K; ++k)
    if (d[k] < d[k + 1] + 1)
      return fail(DDS_EINVAL, "delays[%d]=%d must be >= delays[%d]+1=%d (the error gradient arrives one iteration later)",
                  k, d[k], k + 1, d[k + 1] + 1);
  return DDS_OK;
}

// --------------------------------------------------------------------------- schedule
// Every integer that drives module k0 at iteration t (Section 3.2 closed forms and the slot arithmetic that
// follows from them). dds_schedule reports exactly this record and dds_step executes from it: there is no
// second copy of these formulas in the library.
struct Sched {
  int64_t f, b;        // mini-batch forwarded / back-propagated (negative: idle)
  int R;               // ring depth 2d+1
  int fwd_slot;        // ring slot the forward writes: t mod R
  int bwd_slot;        // ring slot (activations and weight snapshot) the backward reads: (t-2d) mod R
  int err_read;        // error-mailbox slot holding the gradient module k0+1 sent for batch b; -1: last module
  int err_write;       // slot of module k0-1's mailbox this module's backward writes; -1: module 0
  int label_fwd;       // label-queue slot of batch f (last module, f >= 0), else -1
  int in_fwd_slot;     // slot of module k0-1's ring holding its output for batch f (forwarded there at f+k0-1); -1: none
  int in_bwd_slot;     // the same for batch b
  int label_bwd;       // label-queue slot of batch b (last module, b >= 0), else -1
  int snap_write;      // ring slot that receives the weights after this iteration's update: (t+1) mod R
  int label_write;     // label-queue slot the ingest writes (module 0): t mod depth, else -1
};

inline int wrap(int64_t x, int n) { return (int)((x % n + n) % n); }

Sched module_schedule(const std::vector<int>& d, int k0, int64_t t) {
  const int K = (int)d.size();
  Sched s;
  s.R = 2 * d[k0] + 1;
  s.f = t - k0;
  s.b = t - k0 - 2 * d[k0];
  s.fwd_slot = wrap(t, s.R);
  s.bwd_slot = wrap(t - 2 * d[k0], s.R);
  s.snap_write = wrap(t + 1, s.R);
  if (k0 < K - 1) {
    const int lag = 2 * (d[k0] - d[k0 + 1]) - 1;  // iterations between the producer's write and this module's read
    s.err_read = wrap(t - lag, lag + 1);
  } else {
    s.err_read = -1;
  }
  if (k0 > 0) {
    const int lag = 2 * (d[k0 - 1] - d[k0]) - 1;
    s.err_write = wrap(t, lag + 1);
    const int Rup = 2 * d[k0 - 1] + 1;
    s.in_fwd_slot = s.f >= 0 ? wrap(s.f + k0 - 1, Rup) : -1;
    s.in_bwd_slot = s.b >= 0 ? wrap(s.b + k0 - 1, Rup) : -1;
  } else {
    s.err_write = s.in_fwd_slot = s.in_bwd_slot = -1;
  }
  const int depth = K + 2 * d[K - 1];
  s.label_fwd = (k0 == K - 1 && s.f >= 0) ? wrap(s.f, depth) : -1;
  s.label_bwd = (k0 == K - 1 && s.b >= 0) ? wrap(s.b, depth) : -1;
  s.label_write = k0 == 0 ? wrap(t, depth) : -1;
  return s;
}

// --------------------------------------------------------------------------- planning
int new_tensor(Module& m, int N, int C, int H, int W, int dt, int kind) {
  Tensor t;
  t.C = C;
  t.Cpad = round_up(C, dtype_ce(dt));
  t.H = H;
  t.W = W;
  t.dt = dt;
  t.kind = kind;
  t.bytes = (size_t)N * H * W * t.Cpad * dtype_size(dt);
  m.tensors.push_back(t);
  return (int)m.tensors.size() - 1;
}

int add_layer(Module& m, int cin, int cout, int ksize, int stride, int pad, int dt) {
  ParamLayer L;
  L.Cout = cout;
  L.Cin = cin;
  L.R = ksize;
  L.RS = ksize * ksize;
  L.Cinpad = round_up(cin, dtype_ce(dt));
  L.Coutpad = round_up(cout, dtype_ce(dt));
  L.stride = stride;
  L.pad = pad;
  L.n = (long long)cout * L.RS * L.Cinpad + cout;
  L.pstride = (L.n + 3) / 4 * 4;
  L.off = m.n_master;
  m.n_master += (L.n + 63) / 64 * 64;
  m.canon_params += (long long)cout * cin * L.RS + cout;
  m.layers.push_back(L);
  return (int)m.layers.size() - 1;
}

int conv_out(int h, int k, int stride, int pad) { return (h + 2 * pad - k) / stride + 1; }

// Parses module k0's slice of the spec into fused nodes. in_* describe its input tensor.
int plan_module(const dds_spec& sp, int k0, int K, int N, int dt, const Tensor* input, Module& m) {
  const int lo = sp.bounds[k0], hi = sp.bounds[k0 + 1];
  // tensor 0 = module input
  {
    if (k0 == 0) {
      new_tensor(m, N, sp.in_c, sp.in_h, sp.in_w, dt, T_RING);
      m.tensors[0].grad = G_NONE;
    } else {
      Tensor t0 = *input;
      t0.kind = T_EXTERNAL;
      t0.grad = G_ERR_OUT;
      m.tensors.push_back(t0);
    }
  }
  int cur = 0;
  int res_in = -1;  // block input tensor while inside a residual block
  for (int i = lo; i < hi; ++i) {
    const dds_layer& L = sp.layers[i];
    switch (L.op) {
      case DDS_OP_CONV2D:
      case DDS_OP_LINEAR: {
        const bool lin = L.op == DDS_OP_LINEAR;
        const int ks = lin ? 1 : L.ksize, st = lin ? 1 : L.stride, pd = lin ? 0 : L.pad;
        const Tensor ti = m.tensors[cur];
        if (L.cin != ti.C) return fail(DDS_EINVAL, "layer %d: cin=%d but the incoming tensor has %d channels", i, L.cin, ti.C);
        if (lin && (ti.H != 1 || ti.W != 1)) return fail(DDS_EUNSUPPORTED, "layer %d: LINEAR needs a [N,C,1,1] input (insert GAP)", i);
        if (L.cout < 1 || ks < 1 || (st != 1 && st != 2) || pd < 0 || pd >= ks)
          return fail(DDS_EUNSUPPORTED, "layer %d: conv needs cout>=1, stride 1 or 2, 0<=pad<ksize", i);
        const int Ho = conv_out(ti.H, ks, st, pd), Wo = conv_out(ti.W, ks, st, pd);
        if (Ho < 1 || Wo < 1) return fail(DDS_EINVAL, "layer %d: empty output", i);
        Node nd;
        nd.kind = N_CONV;
        nd.in = cur;
        nd.layer = add_layer(m, L.cin, L.cout, ks, st, pd, dt);
        int nxt = i + 1;
        const bool to_ce = nxt < hi && sp.layers[nxt].op == DDS_OP_SOFTMAX_CE;
        const int odt = to_ce ? DT_F32 : dt;
        int out = new_tensor(m, N, L.cout, Ho, Wo, odt, T_RING);
        if (to_ce) {  // logits: fp32 values, padded like a compute-precision tensor so dlogits can mirror it
          Tensor& lt = m.tensors[out];
          lt.Cpad = round_up(L.cout, dtype_ce(dt));
          lt.bytes = (size_t)N * lt.Cpad * 4;
          nd.out_f32 = true;
        }
        nd.out = out;
        // A batch normalisation takes over what would otherwise be fused into the convolution's
        // epilogue: the residual addition (with its scale) and the ReLU.
        Node bn;
        const bool have_bn = nxt < hi && sp.layers[nxt].op == DDS_OP_BATCHNORM;
        if (have_bn) {
          const dds_layer& Bn = sp.layers[nxt];
          if (Bn.cout != L.cout) return fail(DDS_EINVAL, "layer %d: BATCHNORM over %d channels after %d", nxt, Bn.cout, L.cout);
          if (!(Bn.res_scale > 0.f)) return fail(DDS_EINVAL, "layer %d: BATCHNORM needs eps > 0 (in res_scale)", nxt);
          if (L.cout > 2048) return fail(DDS_EUNSUPPORTED, "layer %d: BATCHNORM over more than 2048 channels", nxt);
          bn.kind = N_BN;
          bn.in = out;
          bn.eps = Bn.res_scale;
          bn.layer = add_layer(m, 1, L.cout, 1, 1, 0, dt);  // gamma as a [cout][1] weight, beta as its bias
          bn.out = new_tensor(m, N, L.cout, Ho, Wo, dt, T_RING);
          ++nxt;
        }
        Node& tgt = have_bn ? bn : nd;  // the node whose output the block / the ReLU sees
        const int tgt_out = have_bn ? bn.out : out;
        const bool fuse_res = nxt < hi && sp.layers[nxt].op == DDS_OP_RES_ADD;
        const int res_add_at = nxt;
        Node sc_node;
        bool have_sc = false;
        if (fuse_res) {
          if (res_in < 0) return fail(DDS_EINVAL, "layer %d: RES_ADD without RES_BEGIN", nxt);
          const dds_layer& A = sp.layers[nxt];
          const Tensor tx = m.tensors[res_in];
          tgt.alpha = A.res_scale;
          if (A.cout > 0) {
            if (A.cin != tx.C || A.cout != L.cout) return fail(DDS_EINVAL, "layer %d: shortcut conv shape mismatch", nxt);
            if (A.ksize < 1 || (A.stride != 1 && A.stride != 2) || A.pad < 0 || A.pad >= A.ksize)
              return fail(DDS_EUNSUPPORTED, "layer %d: shortcut conv needs stride 1 or 2, 0<=pad<ksize", nxt);
            if (conv_out(tx.H, A.ksize, A.stride, A.pad) != Ho || conv_out(tx.W, A.ksize, A.stride, A.pad) != Wo)
              return fail(DDS_EINVAL, "layer %d: shortcut output size differs from the main path", nxt);
            sc_node.kind = N_CONV;
            sc_node.in = res_in;
            sc_node.out = new_tensor(m, N, A.cout, Ho, Wo, dt, T_TEMP);
            have_sc = true;
            tgt.res = sc_node.out;
          } else {
            if (tx.C != L.cout || tx.H != Ho || tx.W != Wo)
              return fail(DDS_EINVAL, "layer %d: identity shortcut needs equal shapes", nxt);
            tgt.res = res_in;
          }
          ++nxt;
        }
        if (nxt < hi && sp.layers[nxt].op == DDS_OP_RELU) {
          tgt.relu = true;
          m.tensors[tgt_out].relu_out = true;
          m.tensors[tgt_out].has_bits = !tgt.out_f32 && m.tensors[tgt_out].Cpad % 8 == 0;
          ++nxt;
        }
        if (have_sc) {
          // canonical order: main-path layers first, then the projection (it sits at RES_ADD)
          const dds_layer& A = sp.layers[res_add_at];
          sc_node.layer = add_layer(m, A.cin, A.cout, A.ksize, A.stride, A.pad, dt);
          m.nodes.push_back(sc_node);  // runs before the node whose epilogue adds it
        }
        m.nodes.push_back(nd);
        if (have_bn) m.nodes.push_back(bn);
        if (fuse_res) res_in = -1;
        cur = tgt_out;
        i = nxt - 1;
        break;
      }
      case DDS_OP_RELU:
        return fail(DDS_EUNSUPPORTED, "layer %d: RELU must directly follow CONV2D, LINEAR, BATCHNORM or RES_ADD", i);
      case DDS_OP_BATCHNORM:
        return fail(DDS_EUNSUPPORTED, "layer %d: BATCHNORM must directly follow CONV2D or LINEAR", i);
      case DDS_OP_MAXPOOL2: {
        const Tensor ti = m.tensors[cur];
        if (ti.H % 2 || ti.W % 2) return fail(DDS_EUNSUPPORTED, "layer %d: MAXPOOL2 needs even height and width", i);
        Node nd;
        nd.kind = N_MAXPOOL;
        nd.in = cur;
        nd.out = new_tensor(m, N, ti.C, ti.H / 2, ti.W / 2, dt, T_RING);
        m.nodes.push_back(nd);
        cur = nd.out;
        break;
      }
      case DDS_OP_GAP: {
        const Tensor ti = m.tensors[cur];
        Node nd;
        nd.kind = N_GAP;
        nd.in = cur;
        nd.out = new_tensor(m, N, ti.C, 1, 1, dt, T_RING);
        m.nodes.push_back(nd);
        cur = nd.out;
        break;
      }
      case DDS_OP_RES_BEGIN:
        if (res_in >= 0) return fail(DDS_EUNSUPPORTED, "layer %d: nested residual blocks", i);
        res_in = cur;
        break;
      case DDS_OP_RES_ADD:
        return fail(DDS_EUNSUPPORTED, "layer %d: RES_ADD must directly follow the block's last CONV2D (or its BATCHNORM)", i);
      case DDS_OP_SOFTMAX_CE: {
        if (k0 != K - 1 || i != sp.n_layers - 1) return fail(DDS_EINVAL, "layer %d: SOFTMAX_CE must be the last layer", i);
        const Tensor ti = m.tensors[cur];
        if (ti.dt != DT_F32 || ti.C != sp.classes || ti.H != 1 || ti.W != 1)
          return fail(DDS_EUNSUPPORTED, "layer %d: SOFTMAX_CE must follow a LINEAR/CONV2D producing [N,classes,1,1]", i);
        Node nd;
        nd.kind = N_CE;
        nd.in = cur;
        m.nodes.push_back(nd);
        break;
      }
      default:
        return fail(DDS_EINVAL, "layer %d: unknown op %d", i, L.op);
    }
  }
  if (res_in >= 0) return fail(DDS_EINVAL, "module %d ends inside a residual block", k0);
  if (k0 == K - 1) {
    if (m.nodes.empty() || m.nodes.back().kind != N_CE) return fail(DDS_EINVAL, "the last layer must be SOFTMAX_CE");
  } else if (m.tensors[cur].dt != dt) {
    return fail(DDS_EINVAL, "module %d: SOFTMAX_CE before the last module", k0);
  }
  m.out_tensor = cur;

  // gradient buffers: one per tensor that a backward kernel writes
  for (size_t ti = 1; ti < m.tensors.size(); ++ti) {
    Tensor& t = m.tensors[ti];
    if (t.kind == T_TEMP) continue;  // projection output: shares the block output's gradient
    if ((int)ti == m.out_tensor && k0 < K - 1) { t.grad = G_ERR_IN; continue; }
    GradBuf g;
    g.bytes = t.dt == dt ? t.bytes : (size_t)N * t.Cpad * dtype_size(dt);  // dlogits in compute precision
    m.grads.push_back(g);
    t.grad = (int)m.grads.size() - 1;
  }
  for (size_t ni = 0; ni < m.nodes.size(); ++ni) {
    Node& nd = m.nodes[ni];
    if (nd.kind == N_CE) { nd.gout = G_NONE; nd.gin = m.tensors[nd.in].grad; continue; }
    const Tensor& to = m.tensors[nd.out];
    nd.gin = m.tensors[nd.in].grad;
    nd.mask_in = m.tensors[nd.in].relu_out;
    if (to.kind == T_TEMP) {
      // projection shortcut: find the conv that consumes it
      for (size_t nj = ni + 1; nj < m.nodes.size(); ++nj)
        if ((m.nodes[nj].kind == N_CONV || m.nodes[nj].kind == N_BN) && m.nodes[nj].res == nd.out) { nd.gout = m.tensors[m.nodes[nj].out].grad; break; }
      if (nd.gin != G_NONE) {  // its input gradient goes to a scratch buffer the block's first conv adds
        GradBuf g;
        g.bytes = m.tensors[nd.in].bytes;
        m.grads.push_back(g);
        nd.gin = (int)m.grads.size() - 1;
        nd.mask_in = false;
      }
    } else {
      nd.gout = to.grad;
    }
  }
  // residual wiring: the first conv of a block adds the shortcut's gradient
  for (size_t ni = 0; ni < m.nodes.size(); ++ni) {
    Node& nd = m.nodes[ni];
    if ((nd.kind != N_CONV && nd.kind != N_BN) || nd.res < 0) continue;
    const Tensor& tr = m.tensors[nd.res];
    int block_in;
    int shortcut_grad;
    if (tr.kind == T_TEMP) {
      const Node* sc = nullptr;
      for (size_t nj = 0; nj < ni; ++nj)
        if (m.nodes[nj].out == nd.res) sc = &m.nodes[nj];
      block_in = sc->in;
      shortcut_grad = sc->gin;
    } else {
      block_in = nd.res;
      shortcut_grad = nd.gout;
    }
    // first node after the block input that consumes it on the main path
    Node* first = nullptr;
    for (size_t nj = 0; nj <= ni; ++nj)
      if (m.nodes[nj].in == block_in && m.tensors[m.nodes[nj].out].kind != T_TEMP) { first = &m.nodes[nj]; break; }
    if (!first || first->kind != N_CONV) return fail(DDS_EUNSUPPORTED, "a residual block must start with CONV2D");
    if (first == &nd) return fail(DDS_EUNSUPPORTED, "a residual block needs at least two convolutions");
    if (first->gin != G_NONE) {
      first->addend = shortcut_grad;
      // A 1x1 stride-2 pad-0 projection beside a stride-2 first conv: its input gradient only reaches
      // the even pixels and is accumulated inside the first conv's dgrad launch (the stride-2 dgrad
      // kernel takes it as extra reduction steps) instead of going through a scratch tensor.
      if (tr.kind == T_TEMP) {
        Node* sc = nullptr;
        for (size_t nj = 0; nj < ni; ++nj)
          if (m.nodes[nj].out == nd.res) sc = &m.nodes[nj];
        const ParamLayer& Ls = m.layers[sc->layer];
        const ParamLayer& Lf = m.layers[first->layer];
        const int bke = 64 / dtype_size(dt);  // k-tile of the generic kernels, in elements
        const Tensor& tf = m.tensors[first->out];
        const Tensor& ts = m.tensors[sc->out];
        if (Ls.R == 1 && Ls.stride == 2 && Ls.pad == 0 && Lf.stride == 2 && tf.H == ts.H && tf.W == ts.W &&
            tf.Cpad % bke == 0 && ts.Cpad % bke == 0 && sc->gin >= 0) {
          m.grads[sc->gin].bytes = 0;  // the scratch tensor is not needed
          sc->gin = G_NONE;
          sc->dgrad_folded = true;
          first->addend = G_NONE;
          first->fold_sc = (int)(sc - &m.nodes[0]);
        }
      }
    }
  }
  for (Node& nd : m.nodes)
    if (nd.kind == N_CONV && (nd.gin != G_NONE || nd.dgrad_folded)) m.layers[nd.layer].need_stash = true;
  return DDS_OK;
}

int layout(dds_ctx& c, Arena& A) {
  const int es = dtype_size(c.dt);
  for (int k0 = 0; k0 < c.K; ++k0) {
    Module& m = c.mods[k0];
    // ring: R slots of every saved tensor
    size_t off = 0, aoff = 0;
    m.recompute = c.recompute && m.d > 0;
    for (size_t ti = 0; ti < m.tensors.size(); ++ti) {
      Tensor& t = m.tensors[ti];
      if (t.kind != T_RING) continue;
      t.recomputed = m.recompute && (int)ti != m.out_tensor && !(k0 == 0 && ti == 0);
      size_t& o = t.recomputed ? aoff : off;
      t.ring_off = o;
      o = align_up(o + t.bytes, 256);
      if (t.has_bits) { t.bits_off = o; o = align_up(o + (size_t)c.N * t.H * t.W * t.Cpad / 8, 256); }
    }
    // batch normalisation: what the backward of a mini-batch needs from its forward (mean, rstd, gamma
    // per data-group and channel) lives in the ring slot too; the row splits are fixed here
    size_t bn_scratch_bytes = 0, bn_totals_bytes = 0;
    for (Node& nd : m.nodes) {
      if (nd.kind != N_BN) continue;
      const Tensor& tb = m.tensors[nd.out];
      {
        size_t& o = m.recompute ? aoff : off;
        nd.stats_off = o;
        o = align_up(o + (size_t)c.W * 3 * tb.Cpad * 4, 256);
      }
      const long long rows_per_rep = (long long)c.B * tb.H * tb.W;
      // about 32 KiB of the tensor per workgroup, at most 512 splits per data-group
      long long ns = rows_per_rep * tb.Cpad * es / 32768;
      ns = ns < 1 ? 1 : ns > 512 ? 512 : ns;
      nd.bn_rows_per_split = (rows_per_rep + ns - 1) / ns;
      nd.bn_nsplit = (int)((rows_per_rep + nd.bn_rows_per_split - 1) / nd.bn_rows_per_split);
      const size_t sb = (size_t)c.W * nd.bn_nsplit * tb.Cpad * 2 * sizeof(double);
      const size_t tb_bytes = (size_t)c.W * tb.Cpad * 2 * sizeof(double);
      bn_scratch_bytes = sb > bn_scratch_bytes ? sb : bn_scratch_bytes;
      bn_totals_bytes = tb_bytes > bn_totals_bytes ? tb_bytes : bn_totals_bytes;
    }
    m.slot_bytes = off;
    m.ring = A.take(m.slot_bytes * m.R);
    if (m.recompute) m.area = A.take(aoff);
    if (bn_scratch_bytes) { m.bn_scratch = (double*)A.take(bn_scratch_bytes); m.bn_totals = (double*)A.take(bn_totals_bytes); }
    for (Tensor& t : m.tensors)
      if (t.kind == T_TEMP) t.temp = A.take(t.bytes);
    for (GradBuf& g : m.grads) g.ptr = A.take(g.bytes);
    m.master = (float*)A.take((size_t)m.n_master * 4 * c.copies);
    if (c.mu != 0.f) m.momentum = (float*)A.take((size_t)m.n_master * 4 * c.copies);
    if (c.dt == DT_BF16) m.work = A.take((size_t)m.n_master * es * c.copies);
    if (m.recompute) {
      m.snap_master = (float*)A.take((size_t)m.n_master * 4 * c.copies * m.R);
      if (c.dt == DT_BF16) m.snap_work = A.take((size_t)m.n_master * es * c.copies * m.R);
    }
    for (Node& nd : m.nodes) {
      if (nd.kind == N_BN) {  // one parameter-gradient row per data-group
        ParamLayer& L = m.layers[nd.layer];
        L.nsplit = c.W;
        L.partial = (float*)A.take((size_t)L.nsplit * L.pstride * 4);
        continue;
      }
      if (nd.kind != N_CONV) continue;
      ParamLayer& L = m.layers[nd.layer];
      const Tensor& to = m.tensors[nd.out];
      const int P = c.N * to.H * to.W;
      {
        const Tensor& tin = m.tensors[nd.in];
        WgradParams w{};
        w.zeros = &w;  // non-null: only the shape matters here
        w.Nimg = c.N; w.H = tin.H; w.W = tin.W; w.Cx = tin.Cpad; w.Ho = to.H; w.Wo = to.W;
        w.Mout = L.Cout; w.ldy = to.Cpad;
        w.R = L.R; w.S = L.R; w.stride = L.stride; w.pad = L.pad;
        w.NK = L.RS * L.Cinpad;
        w.P = P;
        // with three or more module programs on concurrent streams a wgrad launch need not fill the chip alone
        L.nsplit = wgrad_choose_split(c.dt, w, c.W, c.K >= 3 ? 128 : 256);
      }
      L.partial = (float*)A.take((size_t)L.nsplit * L.pstride * 4);
      if (L.need_stash) {
        L.stash_elems = (long long)L.Cin * L.RS * L.Coutpad;
        L.stash_slot_bytes = align_up((size_t)L.stash_elems * es, 256);
        L.stash = A.take(L.stash_slot_bytes * m.R * c.copies);
      }
    }
    if (k0 < c.K - 1) {
      const int lag = 2 * (c.d[k0] - c.d[k0 + 1]) - 1;
      m.err_depth = lag + 1;
      m.err_bytes = align_up(m.tensors[m.out_tensor].bytes, 256);
      m.err = A.take(m.err_bytes * m.err_depth);
    }
    // descriptor tables
    int nb_u = 0, nb_s = 0;
    for (ParamLayer& L : m.layers) {
      nb_u += (int)((L.n + 1023) / 1024);
      if (L.need_stash) nb_s += L.RS * ((L.Cin + 63) / 64) * ((L.Coutpad + 63) / 64);  // 64 x 64 tiles per tap
    }
    if (c.gossip) m.cons_dev = (double*)A.take(sizeof(double) * 2 * (nb_u > 0 ? nb_u : 1) * c.W);
    m.blocks_update = nb_u;  // per weight copy; the tables list copy 0 first, then copy 1, ...
    m.blocks_stash = nb_s;
    m.descs_dev = (UpdateDesc*)A.take(sizeof(UpdateDesc) * m.layers.size() * c.copies);
    m.map_update_dev = (int*)A.take(sizeof(int) * 2 * (nb_u > 0 ? nb_u : 1) * c.copies);
    m.map_stash_dev = (int*)A.take(sizeof(int) * 2 * (nb_s > 0 ? nb_s : 1) * c.copies);
  }
  c.label_depth = c.K + 2 * c.d[c.K - 1];
  c.labels = (int32_t*)A.take(sizeof(int32_t) * c.N * c.label_depth);
  c.loss = (float*)A.take(sizeof(float) * c.W);
  c.zeros = A.take(kZeroBytes);
  if (c.gossip) c.P_dev = (float*)A.take(sizeof(float) * c.W * c.W);
  return DDS_OK;
}

int build(dds_ctx& c, const dds_spec* sp, int K, int W, const int* delays) {
  if (!sp || !sp->layers || !sp->bounds) return fail(DDS_EINVAL, "null spec");
  if (K < 1 || K > 64) return fail(DDS_EINVAL, "K=%d out of range [1,64]", K);
  if (W < 1 || W > 32) return fail(DDS_EINVAL, "W=%d out of range [1,32]", W);
  if (sp->batch < 1 || sp->n_layers < 1 || sp->classes < 2 || sp->in_c < 1 || sp->in_h < 1 || sp->in_w < 1)
    return fail(DDS_EINVAL, "bad batch / layer count / classes / input shape");
  if (sp->precision != DDS_F32 && sp->precision != DDS_BF16_F32MASTER) return fail(DDS_EINVAL, "unknown precision");
  if (!(sp->momentum >= 0.f && sp->momentum < 1.f)) return fail(DDS_EINVAL, "momentum must be in [0,1)");
  if (sp->bounds[0] != 0 || sp->bounds[K] != sp->n_layers) return fail(DDS_EINVAL, "bounds must start at 0 and end at n_layers");
  for (int k = 0; k < K; ++k)
    if (sp->bounds[k + 1] <= sp->bounds[k]) return fail(DDS_EINVAL, "module %d is empty", k);
  int rc = check_delays(K, delays, c.d);
  if (rc) return rc;
  if ((long long)W * sp->batch > (1 << 22)) return fail(DDS_EUNSUPPORTED, "W*B too large");
  c.K = K;
  c.W = W;
  c.B = sp->batch;
  c.N = W * sp->batch;
  c.dt = sp->precision == DDS_F32 ? DT_F32 : DT_BF16;
  c.classes = sp->classes;
  c.in_c = sp->in_c;
  c.in_h = sp->in_h;
  c.in_w = sp->in_w;
  c.lr = sp->lr;
  c.mu = sp->momentum;
  if (sp->activations != DDS_ACT_STORE && sp->activations != DDS_ACT_RECOMPUTE) return fail(DDS_EINVAL, "unknown activation policy");
  c.recompute = sp->activations == DDS_ACT_RECOMPUTE;
  if (sp->mixing) {
    // Section 2.3: P symmetric, doubly stochastic, entries in [0,1]
    for (int i = 0; i < W; ++i) {
      double row = 0.0;
      for (int j = 0; j < W; ++j) {
        const float v = sp->mixing[i * W + j];
        if (!(v >= 0.f && v <= 1.f)) return fail(DDS_EINVAL, "mixing[%d][%d]=%g is outside [0,1]", i, j, (double)v);
        if (std::fabs(v - sp->mixing[j * W + i]) > 1e-6f) return fail(DDS_EINVAL, "mixing matrix is not symmetric at (%d,%d)", i, j);
        row += v;
      }
      if (std::fabs(row - 1.0) > 1e-5) return fail(DDS_EINVAL, "row %d of the mixing matrix sums to %g, not 1", i, row);
    }
    c.gossip = true;
    c.copies = W;
    c.P.assign(sp->mixing, sp->mixing + (size_t)W * W);
  }
  c.mods.assign(K, Module());
  for (int k0 = 0; k0 < K; ++k0) {
    Module& m = c.mods[k0];
    m.k0 = k0;
    m.d = c.d[k0];
    m.R = 2 * m.d + 1;
    const Tensor* in = k0 ? &c.mods[k0 - 1].tensors[c.mods[k0 - 1].out_tensor] : nullptr;
    rc = plan_module(*sp, k0, K, c.N, c.dt, in, m);
    if (rc) return rc;
  }
  // sizes that index arithmetic in the kernels keeps in 32 bits
  for (Module& m : c.mods)
    for (Tensor& t : m.tensors)
      if ((long long)c.N * t.H * t.W > 0x7fffffffLL / 2 || t.bytes > ((size_t)1 << 40))
        return fail(DDS_EUNSUPPORTED, "tensor too large");
  return DDS_OK;
}

double count_flops(const dds_ctx& c) {
  double f = 0;
  for (const Module& m : c.mods)
    for (const Node& nd : m.nodes) {
      if (nd.kind != N_CONV) continue;
      const ParamLayer& L = m.layers[nd.layer];
      const Tensor& to = m.tensors[nd.out];
      const double macs = (double)c.N * to.H * to.W * L.Cout * L.Cin * L.RS;
      f += 2.0 * macs * (nd.gin != G_NONE ? 3 : 2);
    }
  return f;
}

// --------------------------------------------------------------------------- execution helpers
// Output of module k0-1 in slot `in_slot` of ITS ring (Sched::in_fwd_slot / in_bwd_slot): module k0's input.
char* input_ptr(dds_ctx& c, int k0, int in_slot) {
  Module& up = c.mods[k0 - 1];
  return up.ring + (size_t)in_slot * up.slot_bytes + up.tensors[up.out_tensor].ring_off;
}

// sign plane of a tensor in the given ring slot (null if it has none); in_slot: see input_ptr
char* bits_ptr(dds_ctx& c, Module& m, int ti, int slot, int in_slot) {
  const Tensor& t = m.tensors[ti];
  if (t.kind == T_RING) {
    if (!t.has_bits) return nullptr;
    return t.recomputed ? m.area + t.bits_off : m.ring + (size_t)slot * m.slot_bytes + t.bits_off;
  }
  if (t.kind == T_EXTERNAL) {
    Module& up = c.mods[m.k0 - 1];
    const Tensor& ut = up.tensors[up.out_tensor];
    return ut.has_bits ? up.ring + (size_t)in_slot * up.slot_bytes + ut.bits_off : nullptr;
  }
  return nullptr;
}

char* tptr(dds_ctx& c, Module& m, int ti, int slot, int in_slot) {
  const Tensor& t = m.tensors[ti];
  if (t.kind == T_TEMP) return t.temp;
  if (t.kind == T_RING) return t.recomputed ? m.area + t.ring_off : m.ring + (size_t)slot * m.slot_bytes + t.ring_off;
  return input_ptr(c, m.k0, in_slot);
}

char* gptr(dds_ctx& c, Module& m, int gid, const Sched& sc) {
  if (gid >= 0) return m.grads[gid].ptr;
  if (gid == G_ERR_IN) return m.err + (size_t)sc.err_read * m.err_bytes;
  if (gid == G_ERR_OUT) {
    Module& up = c.mods[m.k0 - 1];
    return up.err + (size_t)sc.err_write * up.err_bytes;
  }
  return nullptr;
}

hipEvent_t prof_event(dds_ctx& c) {
  if (!c.prof_pool.empty()) { hipEvent_t e = c.prof_pool.back(); c.prof_pool.pop_back(); return e; }
  hipEvent_t e = nullptr;
  (void)hipEventCreate(&e);
  return e;
}

// cls: 0 forward, 1 dgrad, 2 wgrad; + 3 once the launch reports the asynchronous kernel family
struct ProfScope {
  dds_ctx& c; hipStream_t s; int cls; double flops; hipEvent_t a = nullptr;
  bool on;
  ProfScope(dds_ctx& c_, hipStream_t s_, int cls_, double flops_, bool enabled = true)
      : c(c_), s(s_), cls(cls_), flops(flops_), on(c_.profiling && enabled) {
    if (on) { a = prof_event(c); (void)hipEventRecord(a, s); }
  }
  ~ProfScope() {
    if (on) { hipEvent_t b = prof_event(c); (void)hipEventRecord(b, s); c.prof_pending.push_back({cls, flops, a, b}); }
  }
};

// Fields of a batch-normalisation launch that forward and backward share; slot = ring slot of the mini-batch.
BnParams bn_params(dds_ctx& c, Module& m, const Node& nd, int slot, const float* master) {
  const ParamLayer& L = m.layers[nd.layer];
  const Tensor& to = m.tensors[nd.out];
  BnParams p{};
  p.gamma = (float*)master + L.off;
  p.beta = (float*)master + L.off + (long long)L.Cout * L.RS * L.Cinpad;
  p.rep_stride = c.gossip ? m.n_master : 0;
  p.gstride = L.Cinpad;
  p.stats = (float*)(m.recompute ? m.area + nd.stats_off : m.ring + (size_t)slot * m.slot_bytes + nd.stats_off);
  p.scratch = m.bn_scratch;
  p.totals = m.bn_totals;
  p.partial = L.partial;
  p.pstride = L.pstride;
  p.W = c.W;
  p.C = L.Cout;
  p.ld = to.Cpad;
  p.nsplit = nd.bn_nsplit;
  p.rows_per_rep = (long long)c.B * to.H * to.W;
  p.rows_per_split = nd.bn_rows_per_split;
  p.eps = nd.eps;
  p.alpha = nd.alpha;
  p.relu = nd.relu;
  return p;
}

// Forward pass of a mini-batch through the tensors of ring slot `slot`; its input (modules above the first) is in
// slot `in_slot` of the ring of the module below. snap < 0: with the current parameters (the pass of iteration
// t = f + k0). snap >= 0: the same pass again with the parameter snapshot of that slot, which rebuilds the tensors
// the recompute policy does not keep (the kernels are deterministic: identical bits).
void run_forward(dds_ctx& c, Module& m, int slot, int in_slot, hipStream_t s, int snap = -1) {
  const int es = dtype_size(c.dt);
  const size_t snap_off = snap >= 0 ? (size_t)snap * c.copies * m.n_master : 0;
  const float* master = snap >= 0 ? m.snap_master + snap_off : m.master;
  const char* work = snap >= 0 ? (m.snap_work ? m.snap_work + snap_off * es : nullptr) : m.work;
  for (const Node& nd : m.nodes) {
    if (nd.kind == N_CE) continue;
    const Tensor& ti = m.tensors[nd.in];
    const Tensor& to = m.tensors[nd.out];
    char* x = tptr(c, m, nd.in, slot, in_slot);
    char* y = tptr(c, m, nd.out, slot, in_slot);
    switch (nd.kind) {
      case N_CONV: {
        const ParamLayer& L = m.layers[nd.layer];
        ConvParams p{};
        p.x = x;
        p.w = c.dt == DT_BF16 ? (const void*)(work + (size_t)L.off * es) : (const void*)(master + L.off);
        p.y = y;
        p.bias = master + L.off + (long long)L.Cout * L.RS * L.Cinpad;
        p.res = nd.res >= 0 ? tptr(c, m, nd.res, slot, in_slot) : nullptr;
        p.mask = nullptr;
        p.bits_out = nd.relu ? bits_ptr(c, m, nd.out, slot, in_slot) : nullptr;
        p.zeros = c.zeros;
        p.Nimg = c.N; p.H = ti.H; p.W = ti.W; p.Cx = ti.Cpad;
        p.Ho = to.H; p.Wo = to.W;
        p.M = c.N * to.H * to.W;
        // general mixing matrix: data-group r's images meet data-group r's weights
        p.nrep = c.copies;
        p.w_rep = m.n_master * es;
        p.bias_rep = m.n_master;
        p.Nout = L.Cout;
        p.ldy = to.Cpad;
        p.R = L.R; p.S = L.R; p.stride = L.stride; p.pad = L.pad;
        p.Ktot = L.RS * L.Cinpad;
        p.alpha = nd.alpha;
        p.relu = nd.relu;
        p.out_f32 = nd.out_f32;
        p.dgrad = 0;
        {
          // the per-class launch timings cover each launch once: the repeated pass is the same launches again
          ProfScope ps(c, s, 0, 2.0 * p.M * L.Cout * L.Cin * L.RS, snap < 0);
          ps.cls += 3 * launch_conv(c.dt, p, s);
        }
        break;
      }
      case N_BN: {
        BnParams p = bn_params(c, m, nd, slot, master);
        p.x = x;
        p.y = y;
        p.res = nd.res >= 0 ? tptr(c, m, nd.res, slot, in_slot) : nullptr;
        p.bits_out = nd.relu ? bits_ptr(c, m, nd.out, slot, in_slot) : nullptr;
        launch_bn_forward(c.dt, p, s);
        ++c.launches;
        break;
      }
      case N_MAXPOOL:
        launch_maxpool_fwd(c.dt, x, y, c.N, ti.H, ti.W, ti.Cpad, s);
        break;
      case N_GAP:
        launch_gap_fwd(c.dt, x, y, c.N, ti.H * ti.W, ti.Cpad, s);
        break;
    }
    ++c.launches;
  }
}

void run_backward(dds_ctx& c, Module& m, const Sched& sc, hipStream_t s) {
  const int slot = sc.bwd_slot, in_slot = sc.in_bwd_slot;
  for (int ni = (int)m.nodes.size() - 1; ni >= 0; --ni) {
    const Node& nd = m.nodes[ni];
    if (nd.kind == N_CE) continue;  // dlogits were produced by the loss kernel
    const Tensor& ti = m.tensors[nd.in];
    const Tensor& to = m.tensors[nd.out];
    char* x = tptr(c, m, nd.in, slot, in_slot);
    char* gout = gptr(c, m, nd.gout, sc);
    char* gin = gptr(c, m, nd.gin, sc);
    switch (nd.kind) {
      case N_CONV: {
        const ParamLayer& L = m.layers[nd.layer];
        const int ldg = to.Cpad;
        // The weight gradient reads no weights: one launch serves every data-group, and since no
        // split mixes two of them, data-group r's gradient is the sum of its own nsplit / W splits.
        WgradParams w{};
        w.dy = gout;
        w.x = x;
        w.partial = L.partial;
        w.zeros = c.zeros;
        w.Nimg = c.N; w.H = ti.H; w.W = ti.W; w.Cx = ti.Cpad; w.Ho = to.H; w.Wo = to.W;
        w.Mout = L.Cout;
        w.ldy = ldg;
        w.R = L.R; w.S = L.R; w.stride = L.stride; w.pad = L.pad;
        w.NK = L.RS * L.Cinpad;
        w.P = c.N * to.H * to.W;
        w.nsplit = L.nsplit;
        w.nrep = c.W;
        w.pix_per_split = w.P / L.nsplit;
        w.Pl = L.pstride;
        w.alpha = nd.alpha;
        {
          ProfScope ps(c, s, 2, 2.0 * w.P * L.Cout * L.Cin * L.RS);
          ps.cls += 3 * launch_wgrad(c.dt, w, s);
        }
        ++c.launches;
        if (nd.gin != G_NONE) {
          ConvParams p{};
          p.x = gout;
          p.w = L.stash + (size_t)slot * L.stash_slot_bytes;
          p.y = gin;
          p.bias = nullptr;
          p.res = nd.addend != G_NONE ? gptr(c, m, nd.addend, sc) : nullptr;
          p.nrep = c.copies;  // data-group r back-propagates through its own snapshot
          p.w_rep = (long long)m.R * L.stash_slot_bytes;
          if (nd.fold_sc >= 0) {
            const Node& scn = m.nodes[nd.fold_sc];
            const ParamLayer& Ls = m.layers[scn.layer];
            p.x2 = gptr(c, m, scn.gout, sc);
            p.w2 = Ls.stash + (size_t)slot * Ls.stash_slot_bytes;
            p.Cx2 = m.tensors[scn.out].Cpad;
            p.w2_rep = (long long)m.R * Ls.stash_slot_bytes;
          }
          p.maskbits = nd.mask_in ? bits_ptr(c, m, nd.in, slot, in_slot) : nullptr;
          p.mask = nd.mask_in && !p.maskbits ? x : nullptr;
          p.zeros = c.zeros;
          p.Nimg = c.N; p.H = to.H; p.W = to.W; p.Cx = ldg;
          p.Ho = ti.H; p.Wo = ti.W;
          p.M = c.N * ti.H * ti.W;
          p.Nout = L.Cin;
          p.ldy = ti.Cpad;
          p.R = L.R; p.S = L.R; p.stride = L.stride; p.pad = L.pad;
          p.Ktot = L.RS * L.Coutpad;
          p.alpha = nd.alpha;
          p.relu = 0;
          p.out_f32 = 0;
          p.dgrad = 1;
          {
            ProfScope ps(c, s, 1, 2.0 * w.P * L.Cout * L.Cin * L.RS);
            ps.cls += 3 * launch_conv(c.dt, p, s);
          }
          ++c.launches;
        }
        break;
      }
      case N_BN: {
        BnParams p = bn_params(c, m, nd, slot, m.master);
        p.x = x;
        p.dy = gout;
        p.dx = gin;
        launch_bn_backward(c.dt, p, s);
        c.launches += 2;
        break;
      }
      case N_MAXPOOL:
        if (nd.gin != G_NONE) {
          launch_maxpool_bwd(c.dt, gout, x, gin, c.N, ti.H, ti.W, ti.Cpad, nd.mask_in, s);
          ++c.launches;
        }
        break;
      case N_GAP:
        if (nd.gin != G_NONE) {
          launch_gap_bwd(c.dt, gout, x, gin, c.N, ti.H * ti.W, ti.Cpad, nd.mask_in, s);
          ++c.launches;
        }
        break;
    }
  }
}

// Recompute policy: the parameters the next forward pass will use, copied into snapshot slot `slot`.
hipError_t snapshot_params(dds_ctx& c, Module& m, int slot, hipStream_t s) {
  const size_t n = (size_t)m.n_master * c.copies;
  hipError_t e = hipMemcpyAsync(m.snap_master + (size_t)slot * n, m.master, n * 4, hipMemcpyDeviceToDevice, s);
  if (e == hipSuccess && m.snap_work) {
    const size_t es = dtype_size(c.dt);
    e = hipMemcpyAsync(m.snap_work + (size_t)slot * n * es, m.work, n * es, hipMemcpyDeviceToDevice, s);
  }
  c.launches += m.snap_work ? 2 : 1;
  return e;
}

int upload_tables(dds_ctx& c) {
  const int es = dtype_size(c.dt);
  for (Module& m : c.mods) {
    // one descriptor per (weight copy, layer); copy r sums only its own data-group's splits
    const size_t nl = m.layers.size();
    std::vector<UpdateDesc> descs(nl * c.copies);
    std::vector<int> mu, ms;
    for (int r = 0; r < c.copies; ++r)
    for (size_t li = 0; li < nl; ++li) {
      const ParamLayer& L = m.layers[li];
      const int di = (int)(r * nl + li);
      const long long woff = (long long)r * m.n_master + L.off;
      const int q = L.nsplit / c.copies;
      UpdateDesc& d = descs[di];
      d.master = m.master + woff;
      d.momentum = m.momentum ? m.momentum + woff : nullptr;
      d.partial = L.partial + (size_t)r * q * L.pstride;
      d.work = m.work ? (void*)(m.work + (size_t)woff * es) : nullptr;
      d.stash = L.stash ? L.stash + (size_t)r * m.R * L.stash_slot_bytes : nullptr;
      d.stash_slot_elems = (long long)(L.stash_slot_bytes / es);
      d.n = L.n;
      d.pstride = L.pstride;
      d.nsplit = q;
      d.Cout = L.Cout; d.RS = L.RS; d.Cinpad = L.Cinpad; d.Cin = L.Cin; d.Coutpad = L.Coutpad;
      for (int b = 0; b < (int)((L.n + 1023) / 1024); ++b) { mu.push_back(di); mu.push_back(b); }
      if (L.need_stash)
        for (int b = 0; b < L.RS * ((L.Cin + 63) / 64) * ((L.Coutpad + 63) / 64); ++b) { ms.push_back(di); ms.push_back(b); }
    }
    if (!descs.empty()) HIP_TRY(hipMemcpy(m.descs_dev, descs.data(), sizeof(UpdateDesc) * descs.size(), hipMemcpyHostToDevice));
    if (!mu.empty()) HIP_TRY(hipMemcpy(m.map_update_dev, mu.data(), sizeof(int) * mu.size(), hipMemcpyHostToDevice));
    if (!ms.empty()) HIP_TRY(hipMemcpy(m.map_stash_dev, ms.data(), sizeof(int) * ms.size(), hipMemcpyHostToDevice));
    m.map_update_host.assign(mu.begin(), mu.begin() + 2 * m.blocks_update);
  }
  if (c.gossip) HIP_TRY(hipMemcpy(c.P_dev, c.P.data(), sizeof(float) * c.P.size(), hipMemcpyHostToDevice));
  return DDS_OK;
}

}  // namespace

// =========================================================================== C ABI
extern "C" {

const char* dds_last_error(void) { return g_err.c_str(); }

float dds_step_size(int rule, int64_t t, float eta0) {
  if (t < 0) return std::nanf("");
  switch (rule) {
    case DDS_ETA_CONSTANT: return eta0;
    case DDS_ETA_PIECEWISE: return t <= 15000 ? eta0 : t <= 30000 ? eta0 / 10.f : t <= 40000 ? eta0 / 100.f : eta0 / 1000.f;
    case DDS_ETA_DIMINISHING: return eta0 / (float)(t + 1);
    default: return std::nanf("");
  }
}

int dds_schedule(int K, const int* delays, int64_t t, int32_t* out) {
  if (K < 1 || !out || t < 0) return fail(DDS_EINVAL, "dds_schedule: bad arguments");
  std::vector<int> d;
  int rc = check_delays(K, delays, d);
  if (rc) return rc;
  for (int k0 = 0; k0 < K; ++k0) {
    const Sched sc = module_schedule(d, k0, t);
    int32_t* o = out + (size_t)k0 * DDS_SCHED_INTS;
    o[0] = (int32_t)sc.f;
    o[1] = (int32_t)sc.b;
    o[2] = sc.R;
    o[3] = sc.fwd_slot;
    o[4] = sc.bwd_slot;
    o[5] = sc.err_read;
    o[6] = sc.err_write;
    o[7] = sc.label_fwd;
    o[8] = sc.in_fwd_slot;
    o[9] = sc.in_bwd_slot;
    o[10] = sc.label_bwd;
    o[11] = sc.snap_write;
    o[12] = sc.label_write;
  }
  return DDS_OK;
}

int dds_arena_bytes(const dds_spec* spec, int K, int W, const int* delays, size_t* bytes) {
  if (!bytes) return fail(DDS_EINVAL, "null bytes");
  dds_ctx c;
  int rc = build(c, spec, K, W, delays);
  if (rc) return rc;
  Arena A;
  A.dry = true;
  rc = layout(c, A);
  if (rc) return rc;
  *bytes = align_up(A.used, 256);
  return DDS_OK;
}

int dds_create(const dds_spec* spec, int K, int W, const int* delays, void* arena, size_t arena_bytes, dds_ctx** out) {
  if (!out) return fail(DDS_EINVAL, "null out");
  *out = nullptr;
  if (!arena || ((uintptr_t)arena & 255)) return fail(DDS_EINVAL, "arena must be a 256-byte aligned device pointer");
  dds_ctx* c = new dds_ctx();
  int rc = build(*c, spec, K, W, delays);
  if (rc) { delete c; return rc; }
  Arena dry;
  layout(*c, dry);
  if (align_up(dry.used, 256) > arena_bytes) {
    size_t need = align_up(dry.used, 256);
    delete c;
    return fail(DDS_ENOMEM, "arena has %zu bytes, %zu needed", arena_bytes, need);
  }
  Arena A;
  A.dry = false;
  A.base = (char*)arena;
  A.size = arena_bytes;
  // re-plan on a fresh context so that layout() sees untouched modules
  delete c;
  c = new dds_ctx();
  rc = build(*c, spec, K, W, delays);
  if (rc) { delete c; return rc; }
  layout(*c, A);
  c->arena_used = align_up(A.used, 256);
  c->gemm_flops = count_flops(*c);
  hipError_t e = hipMemset(arena, 0, c->arena_used);
  if (e != hipSuccess) { delete c; return fail(DDS_EHIP, "hipMemset(arena) failed: %s", hipGetErrorString(e)); }
  rc = upload_tables(*c);
  if (rc) { delete c; return rc; }
  {
    const char* env = getenv("DDS_SERIAL");
    c->serial = env && env[0] == '1';
  }
  e = hipEventCreateWithFlags(&c->fork, hipEventDisableTiming);
  if (e == hipSuccess) e = hipEventCreateWithFlags(&c->step_end, hipEventDisableTiming);
  if (e != hipSuccess) { dds_destroy(c); return fail(DDS_EHIP, "hipEventCreate failed: %s", hipGetErrorString(e)); }
  if (K > 1) {
    // As many streams as the runtime has hardware queues (GPU_MAX_HW_QUEUES, 4 unless set), the caller's
    // included: a stream beyond that lands on a queue already in use and the two programs on it run one
    // after the other anyway -- better to choose which modules share. Module k0 -> stream k0 mod n.
    int nq = 4;
    if (const char* q = getenv("GPU_MAX_HW_QUEUES")) { const int v = atoi(q); if (v >= 1 && v <= 32) nq = v; }
    const int ns = K < nq ? K : nq;
    c->pool.resize(ns - 1, nullptr);
    for (hipStream_t& st : c->pool)
      if (hipStreamCreateWithFlags(&st, hipStreamNonBlocking) != hipSuccess) {
        dds_destroy(c);
        return fail(DDS_EHIP, "stream creation failed");
      }
    for (int k0 = 0; k0 < K; ++k0) {
      Module& m = c->mods[k0];
      if (k0 % ns != 0) m.stream = c->pool[k0 % ns - 1];  // else: on the caller's stream
      for (hipEvent_t& ev : m.done)
        if (hipEventCreateWithFlags(&ev, hipEventDisableTiming) != hipSuccess) {
          dds_destroy(c);
          return fail(DDS_EHIP, "event creation failed");
        }
    }
  }
  HIP_TRY(hipDeviceSynchronize());
  *out = c;
  return DDS_OK;
}

int dds_destroy(dds_ctx* c) {
  if (!c) return DDS_OK;
  (void)hipDeviceSynchronize();
  for (Module& m : c->mods) {
    for (hipEvent_t ev : m.done)
      if (ev) (void)hipEventDestroy(ev);
  }
  for (hipStream_t st : c->pool)
    if (st) (void)hipStreamDestroy(st);
  if (c->fork) (void)hipEventDestroy(c->fork);
  if (c->step_end) (void)hipEventDestroy(c->step_end);
  for (hipEvent_t e : c->prof_pool) (void)hipEventDestroy(e);
  delete c;
  return DDS_OK;
}

int64_t dds_param_count(const dds_ctx* c, int module) {
  if (!c || module < 0 || module >= c->K) return fail(DDS_EINVAL, "dds_param_count: bad module");
  return c->mods[module].canon_params;
}

int64_t dds_step_count(const dds_ctx* c) { return c ? c->t : (int64_t)fail(DDS_EINVAL, "null ctx"); }
int64_t dds_launches_last_step(const dds_ctx* c) { return c ? c->launches : (int64_t)fail(DDS_EINVAL, "null ctx"); }
double dds_gemm_flops_per_step(const dds_ctx* c) { return c ? c->gemm_flops : 0.0; }

// Calls that read or write module state from a stream other than the last iteration's are ordered after it.
static int order_after_last_step(dds_ctx* c, hipStream_t s) {
  if (c->t > 0 && s != c->last_stream) HIP_TRY(hipStreamWaitEvent(s, c->step_end, 0));
  return DDS_OK;
}

static int params_io(dds_ctx* c, int module, int replica, float* buf, size_t n_floats, void* stream, bool set) {
  if (!c || module < 0 || module >= c->K || !buf) return fail(DDS_EINVAL, "bad ctx / module / pointer");
  if (replica < 0 || replica >= c->W) return fail(DDS_EINVAL, "replica %d out of range [0,%d)", replica, c->W);
  Module& m = c->mods[module];
  c->chained = false;  // the next iteration must be ordered after this access from the caller's stream
  const long long roff = c->gossip ? (long long)replica * m.n_master : 0;
  if ((long long)n_floats != m.canon_params)
    return fail(DDS_EINVAL, "module %d has %lld parameters, caller passed %zu", module, m.canon_params, n_floats);
  hipStream_t s = (hipStream_t)stream;
  if (int rc = order_after_last_step(c, s)) return rc;
  size_t off = 0;
  for (ParamLayer& L : m.layers) {
    launch_param_permute(buf + off, m.master + roff + L.off, L.Cout, L.Cin, L.RS, L.Cinpad, set ? 1 : 0, s);
    off += (size_t)L.Cout * L.Cin * L.RS + L.Cout;
  }
  if (set) {  // always called with replica 0: every data-group starts from the same weights
    for (int r = 1; r < c->copies; ++r)
      HIP_TRY(hipMemcpyAsync(m.master + (size_t)r * m.n_master, m.master, (size_t)m.n_master * 4, hipMemcpyDeviceToDevice, s));
    if (m.momentum) launch_fill_zero(m.momentum, (size_t)m.n_master * 4 * c->copies, s);
    launch_recast(c->dt, m.descs_dev, m.map_update_dev, m.blocks_update * c->copies, s);
    for (int slot = 0; slot < m.R; ++slot) {
      launch_stash(c->dt, m.descs_dev, m.map_stash_dev, m.blocks_stash * c->copies, slot, s);
      if (m.recompute) HIP_TRY(snapshot_params(*c, m, slot, s));
    }
  }
  HIP_TRY(hipGetLastError());
  return DDS_OK;
}

int dds_get_params(dds_ctx* c, int module, float* dst, size_t n, void* stream) { return params_io(c, module, 0, dst, n, stream, false); }
int dds_get_params_replica(dds_ctx* c, int module, int replica, float* dst, size_t n, void* stream) {
  return params_io(c, module, replica, dst, n, stream, false);
}

// Disagreement measure with the per-block partial sums of every module in `shared` (device memory of at least
// 2 * blocks_update * W doubles for the largest module), or in the module's own arena block if shared is null. The
// kernel writes every entry the host reads, so stale contents do not matter.
static int consensus_error_impl(dds_ctx* c, double* host_out, hipStream_t s, double* shared) {
  *host_out = 0.0;
  if (!c->gossip) return DDS_OK;
  c->chained = false;
  if (int rc = order_after_last_step(c, s)) return rc;
  double worst = 0.0;
  std::vector<double> host, sums;
  for (Module& m : c->mods) {
    if (m.blocks_update == 0) continue;
    const size_t n = (size_t)2 * m.blocks_update * c->W;
    double* dev = shared ? shared : m.cons_dev;
    launch_consensus(m.descs_dev, m.map_update_dev, m.blocks_update, c->W, m.n_master, dev, s);
    HIP_TRY(hipGetLastError());
    host.resize(n);
    HIP_TRY(hipMemcpyAsync(host.data(), dev, n * sizeof(double), hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    // a layer's weight vector w_l (Section 2.1) is its weight and its bias together: [layer][s], both parts
    // of every block added in order
    sums.assign(m.layers.size() * c->W, 0.0);
    for (int b = 0; b < m.blocks_update; ++b) {
      const int layer = m.map_update_host[2 * b];
      for (int part = 0; part < 2; ++part)
        for (int r = 0; r < c->W; ++r) sums[(size_t)layer * c->W + r] += host[((size_t)2 * b + part) * c->W + r];
    }
    for (double v : sums) worst = v > worst ? v : worst;
  }
  *host_out = std::sqrt(worst);
  return DDS_OK;
}

int dds_consensus_error(dds_ctx* c, double* host_out, void* stream) {
  if (!c || !host_out) return fail(DDS_EINVAL, "dds_consensus_error: null argument");
  return consensus_error_impl(c, host_out, (hipStream_t)stream, nullptr);
}

// ---- the same measure for callers that must not trigger a device allocation: the per-block partial sums go to a
// file-scope device array instead of the arena block (so a context created in an arena sized without that block,
// or any caller that forbids allocations, can still ask). One array per GPU, shared by every call on that GPU.
constexpr size_t kStaticScratchDoubles = 65536;  // 512 KiB per GPU, held until the process ends
static __device__ __align__(256) double scratch[kStaticScratchDoubles];
constexpr int kMaxDevices = 64;
static double* g_scratch_ptr[kMaxDevices] = {};  // device address of `scratch` on each GPU (the array's name is only a host-side handle)

int dds_consensus_error_static(dds_ctx* c, double* host_out, void* stream) {
  if (!c || !host_out) return fail(DDS_EINVAL, "dds_consensus_error_static: null argument");
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(DDS_EUNSUPPORTED, "dds_consensus_error_static: device %d out of range", dev);
  if (!g_scratch_ptr[dev]) {  // once per device, with that device current: every GPU has its own copy at its own address
    void* ptr = nullptr;
    HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return fail(DDS_EHIP, "dds_consensus_error_static: no device address for the scratch array");
    g_scratch_ptr[dev] = (double*)ptr;
  }
  for (const Module& m : c->mods) {
    const size_t need = (size_t)2 * m.blocks_update * c->W;
    if (c->gossip && need > kStaticScratchDoubles)
      return fail(DDS_EUNSUPPORTED,
                  "dds_consensus_error_static: module %d needs %zu partial sums (2 per 1024 parameters and data-group), "
                  "the static scratch holds %zu; use dds_consensus_error",
                  m.k0, need, kStaticScratchDoubles);
  }
  return consensus_error_impl(c, host_out, (hipStream_t)stream, g_scratch_ptr[dev]);
}

int dds_set_params(dds_ctx* c, int module, const float* src, size_t n, void* stream) {
  if (c && c->t != 0) return fail(DDS_EINVAL, "dds_set_params is only valid before the first step");
  return params_io(c, module, 0, (float*)src, n, stream, true);
}

int dds_step(dds_ctx* c, const float* const* x, const int32_t* const* y, float lr, void* stream) {
  if (!c || !x || !y) return fail(DDS_EINVAL, "dds_step: null argument");
  for (int s = 0; s < c->W; ++s)
    if (!x[s] || !y[s]) return fail(DDS_EINVAL, "dds_step: null batch pointer for replica %d", s);
  hipStream_t us = (hipStream_t)stream;
  const int64_t t = c->t;
  const float step = std::isnan(lr) ? c->lr : lr;
  c->launches = 0;
  if (t > 0 && us != c->last_stream) {  // the caller switched streams: order this iteration after the previous one
    HIP_TRY(hipStreamWaitEvent(us, c->step_end, 0));
    c->chained = false;
  }

  // ingest: caller batches -> module 0's ring slot t mod R_0 (layout + precision), labels -> queue
  {
    Module& m0 = c->mods[0];
    const Sched sc0 = module_schedule(c->d, 0, t);
    IngestParams p{};
    for (int s = 0; s < c->W; ++s) { p.x[s] = x[s]; p.y[s] = y[s]; }
    p.dst = m0.ring + (size_t)sc0.fwd_slot * m0.slot_bytes + m0.tensors[0].ring_off;
    p.labels = c->labels + (size_t)sc0.label_write * c->N;
    p.W = c->W; p.B = c->B; p.C = c->in_c; p.HW = c->in_h * c->in_w; p.Cpad = m0.tensors[0].Cpad;
    launch_ingest(c->dt, p, us);
    ++c->launches;
  }
  const bool multi = c->K > 1 && !c->serial && !c->profile_serial;
  if (multi) HIP_TRY(hipEventRecord(c->fork, us));
  for (int k0 = 0; k0 < c->K; ++k0) {
    Module& m = c->mods[k0];
    // A module program on an internal stream starts as soon as what it reads is there and what it overwrites has
    // been read: its two neighbours' programs of the previous iteration (module k0-1 wrote its input and read the
    // error slot it now overwrites; module k0+1 wrote the error gradient it consumes and read the ring slot it now
    // overwrites). The first iteration, and any iteration after the caller touched module state from its own
    // stream, forks from the caller's stream instead. All programs are joined to the caller's stream after the loop.
    const bool own = multi && m.stream != nullptr;
    hipStream_t s = own ? m.stream : us;
    if (own) {
      if (c->chained) {
        if (k0 > 0) HIP_TRY(hipStreamWaitEvent(s, c->mods[k0 - 1].done[(t + 1) & 1], 0));
        if (k0 + 1 < c->K) HIP_TRY(hipStreamWaitEvent(s, c->mods[k0 + 1].done[(t + 1) & 1], 0));
      } else {
        HIP_TRY(hipStreamWaitEvent(s, c->fork, 0));
      }
    }
    const Sched sc = module_schedule(c->d, k0, t);
    const bool last = k0 == c->K - 1;
    if (sc.f >= 0) run_forward(*c, m, sc.fwd_slot, sc.in_fwd_slot, s);
    if (last && sc.f >= 0) {
      const Node& ce = m.nodes.back();
      const Tensor& lt = m.tensors[ce.in];
      const float* logits = (const float*)tptr(*c, m, ce.in, sc.fwd_slot, sc.in_fwd_slot);
      const int32_t* lab = c->labels + (size_t)sc.label_fwd * c->N;
      void* dl = (sc.b == sc.f) ? gptr(*c, m, ce.gin, sc) : nullptr;
      launch_softmax_ce(c->dt, logits, lab, dl, c->loss, c->W, c->B, c->classes, lt.Cpad, lt.Cpad, s);
      ++c->launches;
      c->have_loss = true;
    }
    if (m.recompute && sc.b >= 0) run_forward(*c, m, sc.bwd_slot, sc.in_bwd_slot, s, sc.bwd_slot);
    if (last && sc.b >= 0 && sc.b != sc.f) {  // a delayed last module: the loss gradient of the batch forwarded 2d iterations ago
      const Node& ce = m.nodes.back();
      const Tensor& lt = m.tensors[ce.in];
      const float* logits = (const float*)tptr(*c, m, ce.in, sc.bwd_slot, sc.in_bwd_slot);
      const int32_t* lab = c->labels + (size_t)sc.label_bwd * c->N;
      launch_softmax_ce(c->dt, logits, lab, gptr(*c, m, ce.gin, sc), nullptr, c->W, c->B, c->classes, lt.Cpad, lt.Cpad, s);
      ++c->launches;
    }
    if (sc.b >= 0) {
      run_backward(*c, m, sc, s);
      if (!c->gossip) {
        launch_update(c->dt, m.descs_dev, m.map_update_dev, m.blocks_update, c->W, step, c->mu, s);
      } else {
        // u_r = w_r - lr * direction_r from every data-group's own splits, then the mixing step, in one kernel
        launch_gossip_update(c->dt, m.descs_dev, m.map_update_dev, m.blocks_update, c->P_dev, c->W, m.n_master, step,
                             c->mu, s);
      }
      launch_stash(c->dt, m.descs_dev, m.map_stash_dev, m.blocks_stash * c->copies, sc.snap_write, s);
      c->launches += 2;
      if (m.recompute) HIP_TRY(snapshot_params(*c, m, sc.snap_write, s));
    }
    if (multi) HIP_TRY(hipEventRecord(m.done[t & 1], s));
  }
  if (multi)
    for (Module& m : c->mods)
      if (m.stream) HIP_TRY(hipStreamWaitEvent(us, m.done[t & 1], 0));
  // (with two modules the fork from the caller's stream measured 2.5 % faster than the chain)
  c->chained = multi && c->K >= 3;
  HIP_TRY(hipEventRecord(c->step_end, us));
  c->last_stream = us;
  HIP_TRY(hipGetLastError());
  c->t = t + 1;
  if (c->profiling) {  // harvest this step's event pairs (synchronises: profiling runs are not timed runs)
    HIP_TRY(hipStreamSynchronize(us));
    for (auto& r : c->prof_pending) {
      float ms = 0.f;
      if (hipEventElapsedTime(&ms, r.a, r.b) == hipSuccess) {
        c->prof_ms[r.cls] += ms;
        c->prof_flops[r.cls] += r.flops;
        c->prof_count[r.cls] += 1;
      }
      c->prof_pool.push_back(r.a);
      c->prof_pool.push_back(r.b);
    }
    c->prof_pending.clear();
  }
  return DDS_OK;
}

// Test-only raw view of the delay buffers.
static int debug_region(dds_ctx* c, int what, int module, int index, int slot, char** ptr, size_t* bytes) {
  if (!c || module < 0 || module >= c->K) return fail(DDS_EINVAL, "dds_debug: bad ctx / module");
  Module& m = c->mods[module];
  switch (what) {
    case DDS_DBG_INPUT: {
      if (module != 0) return fail(DDS_EINVAL, "dds_debug: only module 0 keeps its input in its own ring");
      if (slot < 0 || slot >= m.R) return fail(DDS_EINVAL, "dds_debug: ring slot %d out of [0,%d)", slot, m.R);
      const Tensor& t = m.tensors[0];
      *ptr = m.ring + (size_t)slot * m.slot_bytes + t.ring_off;
      *bytes = t.bytes;
      return DDS_OK;
    }
    case DDS_DBG_OUTPUT: {
      if (slot < 0 || slot >= m.R) return fail(DDS_EINVAL, "dds_debug: ring slot %d out of [0,%d)", slot, m.R);
      const Tensor& t = m.tensors[m.out_tensor];
      *ptr = m.ring + (size_t)slot * m.slot_bytes + t.ring_off;
      *bytes = t.bytes;
      return DDS_OK;
    }
    case DDS_DBG_ERROR: {
      if (module >= c->K - 1) return fail(DDS_EINVAL, "dds_debug: the last module has no error mailbox");
      if (slot < 0 || slot >= m.err_depth) return fail(DDS_EINVAL, "dds_debug: mailbox slot %d out of [0,%d)", slot, m.err_depth);
      *ptr = m.err + (size_t)slot * m.err_bytes;
      *bytes = m.tensors[m.out_tensor].bytes;
      return DDS_OK;
    }
    case DDS_DBG_LABELS: {
      if (slot < 0 || slot >= c->label_depth) return fail(DDS_EINVAL, "dds_debug: label slot %d out of [0,%d)", slot, c->label_depth);
      *ptr = (char*)(c->labels + (size_t)slot * c->N);
      *bytes = sizeof(int32_t) * c->N;
      return DDS_OK;
    }
    case DDS_DBG_SNAPSHOT: {
      if (index < 0 || index >= (int)m.layers.size()) return fail(DDS_EINVAL, "dds_debug: layer %d out of range", index);
      const ParamLayer& L = m.layers[index];
      if (!L.need_stash) return fail(DDS_EINVAL, "dds_debug: layer %d keeps no snapshots (nothing back-propagates through it)", index);
      if (slot < 0 || slot >= m.R) return fail(DDS_EINVAL, "dds_debug: ring slot %d out of [0,%d)", slot, m.R);
      *ptr = L.stash + (size_t)slot * L.stash_slot_bytes;
      *bytes = (size_t)L.stash_elems * dtype_size(c->dt);
      return DDS_OK;
    }
    default:
      return fail(DDS_EINVAL, "dds_debug: unknown region %d", what);
  }
}

int64_t dds_debug_bytes(dds_ctx* c, int what, int module, int index) {
  char* p = nullptr;
  size_t n = 0;
  const int rc = debug_region(c, what, module, index, 0, &p, &n);
  return rc ? (int64_t)rc : (int64_t)n;
}

int dds_debug_read(dds_ctx* c, int what, int module, int index, int slot, void* dst, size_t bytes, void* stream) {
  char* p = nullptr;
  size_t n = 0;
  if (int rc = debug_region(c, what, module, index, slot, &p, &n)) return rc;
  if (!dst || bytes != n) return fail(DDS_EINVAL, "dds_debug_read: the region has %zu bytes, caller passed %zu", n, bytes);
  hipStream_t s = (hipStream_t)stream;
  c->chained = false;
  if (int rc = order_after_last_step(c, s)) return rc;
  HIP_TRY(hipMemcpyAsync(dst, p, n, hipMemcpyDeviceToDevice, s));
  return DDS_OK;
}

int dds_profile(dds_ctx* c, int enable) {
  if (!c) return fail(DDS_EINVAL, "null ctx");
  c->chained = false;
  c->profiling = enable != 0;
  c->profile_serial = enable == 2;
  for (int i = 0; i < 6; ++i) { c->prof_ms[i] = 0; c->prof_flops[i] = 0; c->prof_count[i] = 0; }
  return DDS_OK;
}

int dds_profile_read(const dds_ctx* c, double* out18) {
  if (!c || !out18) return fail(DDS_EINVAL, "null argument");
  for (int i = 0; i < 6; ++i) {
    out18[3 * i + 0] = c->prof_ms[i];
    out18[3 * i + 1] = (double)c->prof_count[i];
    out18[3 * i + 2] = c->prof_flops[i];
  }
  return DDS_OK;
}

int dds_get_loss(dds_ctx* c, float* host_out, void* stream) {
  if (!c || !host_out) return fail(DDS_EINVAL, "dds_get_loss: null argument");
  if (!c->have_loss) return fail(DDS_EINVAL, "no loss yet: the last module has not forwarded a mini-batch");
  float tmp[32];
  if (int rc = order_after_last_step(c, (hipStream_t)stream)) return rc;
  HIP_TRY(hipMemcpyAsync(tmp, c->loss, sizeof(float) * c->W, hipMemcpyDeviceToHost, (hipStream_t)stream));
  HIP_TRY(hipStreamSynchronize((hipStream_t)stream));
  double acc = 0;
  for (int s = 0; s < c->W; ++s) acc += tmp[s];
  *host_out = (float)(acc / c->W);
  return DDS_OK;
}

}  // extern "C"
