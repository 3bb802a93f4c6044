// Device side of the library: context, weight upload, workspace, kernel sequencing.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <unordered_map>
#include <vector>

#include "heads.hip.h"
#include "mlp2.hip.h"
#include "mlp2_bwd.hip.h"
#include "mlp2_bwdz.hip.h"
#include "mlp2p.hip.h"
#include "resident.hip.h"
#include "mlp2r.hip.h"
#include "gat.hip.h"
#include "wgrad.hip.h"
#include "segsum.hip.h"
#include "xrl_internal.h"

using namespace xrl;

#define HIP_TRY(expr)                                                                       \
  do {                                                                                      \
    hipError_t e_ = (expr);                                                                 \
    if (e_ != hipSuccess)                                                                   \
      return fail(XRL_ERR_HIP, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, \
                  __LINE__);                                                                \
  } while (0)

namespace {

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

inline uint16_t bf16_bits(float x) {  // round to nearest even; inputs are finite
  uint32_t u;
  memcpy(&u, &x, 4);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

template <typename T> struct HostCvt;
template <> struct HostCvt<float> { static float cvt(float x) { return x; } };
template <> struct HostCvt<uint16_t> { static uint16_t cvt(float x) { return bf16_bits(x); } };

// Layer-1 weights W [K, H] -> fragment order [slab][feature block][lane][j]: lane l, element j
// of slab s holds W[s*2V + (l/32)*V + j][32*mb + l%32] (zero beyond K).
template <typename T>
void swizzle_l1(const float *W, int K, int H, int V, std::vector<T> &out) {
  const int SL = 2 * V, MB = H / 32, ns = (K + SL - 1) / SL;
  out.assign((size_t)ns * MB * 64 * V, HostCvt<T>::cvt(0.f));
  for (int s = 0; s < ns; ++s)
    for (int mb = 0; mb < MB; ++mb)
      for (int l = 0; l < 64; ++l)
        for (int j = 0; j < V; ++j) {
          const int k = s * SL + (l / 32) * V + j, f = 32 * mb + l % 32;
          if (k < K) out[(((size_t)s * MB + mb) * 64 + l) * V + j] = HostCvt<T>::cvt(W[(size_t)k * H + f]);
        }
}

// "Chain" order for a weight whose contraction index is fed from an accumulator tile:
// Wt [Kc, M] (row = contraction index, column = the index a lane addresses) ->
// [chunk][column block][lane][j]; element j of chunk c in lane group g is contraction index
// 2V*c + 8*(j/4) + 4*g + j%4 (the accumulator layout), lane l addresses column 32*b + l%32.
// Used for the forward's layer 2 (Wt = W2) and for the backward's W2^T and W1^T products.
template <typename T>
void swizzle_chain(const float *Wt, int Kc, int M, int ld, int V, std::vector<T> &out) {
  const int SL = 2 * V, MBk = M / 32, nc = Kc / SL;
  out.assign((size_t)nc * MBk * 64 * V, HostCvt<T>::cvt(0.f));
  for (int c = 0; c < nc; ++c)
    for (int b = 0; b < MBk; ++b)
      for (int l = 0; l < 64; ++l)
        for (int j = 0; j < V; ++j) {
          const int g = l / 32, k = SL * c + 8 * (j / 4) + 4 * g + j % 4, m = 32 * b + l % 32;
          out[(((size_t)c * MBk + b) * 64 + l) * V + j] = HostCvt<T>::cvt(Wt[(size_t)k * ld + m]);
        }
}

struct EncMlp {           // device pointers of one encoder MLP
  const void *W1s = nullptr, *W2s = nullptr;
  const void *W2bt = nullptr, *W1bt = nullptr;   // backward: contraction over the weight's columns
  const float *b1 = nullptr, *b2 = nullptr;
  int nslab1 = 0;
  // embed MLP, forward: W1's rows for [edge-attr sum | dense attrs] in fragment order (fp32), and
  // its rows for the one-hot op type as a plain [Tn, H] table
  const void *W1x = nullptr;
  const float *table = nullptr;
  int nslabx = 0;
};

}  // namespace

// kernels whose launches can be timed with HIP events (xrl_set_timing / xrl_read_timing)
enum { TK_EMBED = 0, TK_EDGE, TK_EDGE_FIXUP, TK_NODE, TK_POOL, TK_READOUT, TK_HEADS, TK_GAT_LINEAR,
       TK_GAT_AGGREGATE, TK_BWD_EDGE, TK_BWD_NODE, TK_BWD_EMBED, TK_WGRAD, TK_GRAD_GATHER, TK_GAT_BWD, TK_RESIDENT,
       TK_WGRAD_EDGE, TK_WGRAD_NODE, TK_WGRAD_EMBED, TK_COUNT };
static const char *const kTimedNames[TK_COUNT] = {"embed", "edge", "edge_fixup", "node", "pool", "readout",
                                                  "heads", "gat_linear", "gat_aggregate", "bwd_edge", "bwd_node",
                                                  "bwd_embed", "wgrad", "grad_gather", "gat_bwd", "resident",
                                                  "wgrad_edge", "wgrad_node", "wgrad_embed"};

constexpr int64_t kMaxFusedSlots = 4096;   // largest G the single-launch heads kernel takes
constexpr int64_t kClusterMaxGraphs = 256; // largest G of the one-launch encoder with several blocks per graph

// Scratch of xrl_policy_value_static, the entry point that allocates nothing: per-state counters,
// the logits when the caller does not ask for them, and the per-state mean embeddings. One copy
// per GPU, held until the process ends; host code never passes the array's name to a kernel, only
// the address hipGetSymbolAddress reports for the current device (static_scratch below).
constexpr int64_t kStaticMaxSlots = kMaxFusedSlots;          // G
constexpr int64_t kStaticMaxStateFloats = 65536;             // S * hidden
constexpr size_t kStaticCounterOff = 0;
constexpr size_t kStaticLogitOff = kStaticCounterOff + sizeof(int32_t) * kStaticMaxSlots;
constexpr size_t kStaticZmeanOff = kStaticLogitOff + sizeof(float) * kStaticMaxSlots;
constexpr size_t kStaticBytes = kStaticZmeanOff + sizeof(float) * kStaticMaxStateFloats;
static __device__ __align__(256) unsigned char scratch[kStaticBytes];

struct xrl_ctx {
  xrl_model_desc m;
  Layout L;
  hipStream_t stream = nullptr;
  int elem = 4;                 // bytes per stored activation / operand
  int n_cu = 256;               // compute units of the device
  int max_lds = 65536;          // LDS bytes one block may use
  int64_t p_min_rows = 8192;    // smallest row count for the persistent kernels (XRL_PERSISTENT_MIN_ROWS)
  int64_t wide_min_rows = 1 << 20;   // ... for the 256-column weight-gradient tiles (XRL_WGRAD_WIDE_MIN_ROWS)
  int64_t resident_max_graphs = 0;   // largest batch (graphs) for the one-launch encoder (XRL_RESIDENT_MAX_GRAPHS)
  int64_t resident_max_tiles = 0;    // ... and the most 32-row tiles (nodes, or edges) of one graph (XRL_RESIDENT_MAX_TILES)
  float *d_w = nullptr;         // flat fp32 weights
  int32_t *d_counter = nullptr; // kMaxFusedSlots per-state counters of policy_value_kernel, zero between launches
  unsigned *d_arrived = nullptr; // kClusterMaxGraphs per-graph counters of encode_cluster_kernel, zero between launches
  unsigned *h_fault = nullptr;   // pinned host word a kernel sets when one of its bounded waits gives up ...
  unsigned *d_fault = nullptr;   // ... and the address kernels write it through
  // mlp_layers = 1 (the layers of Section 3.4 exactly as printed: one learned matrix each) runs on the
  // two-layer kernels: the context's own model and layout (m, L) have a second layer whose matrix
  // is the identity and whose bias is zero -- relu(relu(z) I + 0) = relu(z) exactly, in both
  // precisions -- and the caller's one-layer vector is spread into that layout on upload. The
  // backward passes run on an internal gradient vector whose real tensors are then added to the
  // caller's (the identity layers' gradients are dropped).
  bool single_layer = false;
  Layout Lu;                      // the caller's layout (single_layer)
  float *d_dw_int = nullptr;      // [L.total] internal gradient vector (single_layer)
  int32_t *d_wmap = nullptr;      // [Lu.total] index in the internal vector of each of the caller's weights
  int64_t cluster_max_graphs = 0; // largest batch (graphs) for the one-launch encoder with several blocks per graph
  unsigned cluster_spin_limit = kClusterSpinLimit;   // polls after which one of its waits gives up (XRL_CLUSTER_SPIN_LIMIT)
  int device = 0;               // the device that was current at xrl_create
  char *static_ws = nullptr;    // this device's copy of `scratch` (its device address)
  void *zero_row = nullptr;     // 1 KB of zeros behind the weights
  bool agg_skip = false;        // last encode: the received-sum rows of nodes without in-edges were not written
                                // (their readers go by the batch's agg_src)
  char *d_swz = nullptr;        // fragment-ordered encoder weights
  size_t swz_bytes = 0;
  EncMlp embed;
  std::vector<EncMlp> edge, node;
  std::vector<const void *> gatW;   // XRL_ROUND_GAT: fragment-ordered W of each round
  std::vector<const void *> gatWt;  //   and of W^T (backward: dh = dz W^T)
  std::vector<float *> gat_ss, gat_sd;   // saved per-node scores of each round (inside ws)
  std::unordered_map<int64_t, const float *> row_w;   // readout / head matrices, 16-byte aligned copies
  // workspaces (grow-only): encoder activations, and a separate small one for the heads
  char *ws = nullptr;
  size_t ws_bytes = 0;
  char *hws = nullptr;
  size_t hws_bytes = 0;
  char *bws = nullptr;          // backward scratch
  size_t bws_bytes = 0;
  // buffers of the last encode (inside ws)
  uint64_t enc_batch = 0;
  bool enc_saved = false;
  float *pool = nullptr, *carry = nullptr, *ro_act[2] = {nullptr, nullptr};
  std::vector<void *> h, agg;   // h[0..R], agg[1..R] (index 0 unused)
  // what the forward kernels of large bf16 batches keep for the backward pass (inside ws): relu(z1)
  // of the embed MLP and of every round's edge and node MLP, and the mask bits of every round's
  // per-edge output (which is summed per receiver and never stored itself)
  bool fwd_kept = false;
  void *z1_embed = nullptr;
  std::vector<void *> z1_edge, z1_node;
  std::vector<uint16_t *> ym_edge, ym_node, zm_edge, zm_node;   // mask bits of y and of z1, per round
  uint16_t *ym_embed = nullptr, *zm_embed = nullptr;
  // optional per-kernel timing
  bool timing = false;
  struct Span { int kind; hipEvent_t a, b; };
  std::vector<Span> spans;
  std::vector<hipEvent_t> free_events;
};

namespace {
// Brackets the launches made during its lifetime with two events on the ctx stream.
struct Timed {
  xrl_ctx *c;
  int idx = -1;
  Timed(xrl_ctx *ctx, int kind) : c(ctx) {
    if (!c->timing) return;
    hipEvent_t ev[2];
    for (int i = 0; i < 2; ++i) {
      if (!c->free_events.empty()) { ev[i] = c->free_events.back(); c->free_events.pop_back(); }
      else if (hipEventCreate(&ev[i]) != hipSuccess) return;
    }
    c->spans.push_back({kind, ev[0], ev[1]});
    idx = (int)c->spans.size() - 1;
    (void)hipEventRecord(ev[0], c->stream);
  }
  ~Timed() { if (idx >= 0) (void)hipEventRecord(c->spans[idx].b, c->stream); }
};
}  // namespace

namespace {
// Device address of `scratch` on the current device, looked up once per device.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
char *g_scratch_ptr[kMaxDevices] = {};
int static_scratch(int dev, char **out) {
  if (dev < 0 || dev >= kMaxDevices) return fail(XRL_ERR_UNSUPPORTED, "device ordinal %d", dev);
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return fail(XRL_ERR_HIP, "hipGetSymbolAddress returned a null address");
    g_scratch_ptr[dev] = (char *)p;
  }
  *out = g_scratch_ptr[dev];
  return XRL_OK;
}
}  // namespace

extern "C" void xrl_batch_release_device(xrl_batch *b) {
  if (b && b->dev.block) {
    (void)hipFree(b->dev.block);
    b->dev = xrl_batch_device();
    b->uploaded = false;
  }
}

namespace {

// Internal index of the first element of the caller's tensor `t` (single-layer contexts): the tensor of
// the same name in the internal layout.
int64_t internal_offset(const xrl_ctx *c, const WeightTensor &t) {
  for (const WeightTensor &u : c->L.tensors)
    if (u.name == t.name) return u.offset;
  return -1;
}

int upload_weights(xrl_ctx *c, const float *w_user) {
  const xrl_model_desc &m = c->m;
  const int64_t n_user = c->single_layer ? c->Lu.total : c->L.total;
  for (int64_t i = 0; i < n_user; ++i)
    if (!std::isfinite(w_user[i])) return fail(XRL_ERR_VALUE, "weights[%lld] is not finite", (long long)i);
  std::vector<float> spread;
  if (c->single_layer) {
    spread.assign((size_t)c->L.total, 0.f);
    for (const WeightTensor &t : c->Lu.tensors) {
      const int64_t n = t.cols > 0 ? t.rows * t.cols : t.rows;
      memcpy(spread.data() + internal_offset(c, t), w_user + t.offset, sizeof(float) * (size_t)n);
    }
    const int H = m.hidden;
    auto identity = [&](const MlpRef &r) {
      for (int k = 0; k < H; ++k) spread[(size_t)r.w[1] + (size_t)k * H + k] = 1.f;
    };
    identity(c->L.embed);
    identity(c->L.readout);
    for (const MlpRef &r : c->L.edge) identity(r);
    for (const MlpRef &r : c->L.node) identity(r);
  }
  const float *w = c->single_layer ? spread.data() : w_user;
  const int V = c->elem == 2 ? 8 : 4, H = m.hidden;
  // build the fragment-ordered blob on the host
  std::vector<char> blob;
  struct Ref { size_t w1, w2, w2bt, w1bt, w1x = 0; int ns, nsx = 0; };
  std::vector<Ref> refs;
  auto add = [&](const MlpRef &r, bool l1_fp32) {
    Ref ref;
    const int V1 = l1_fp32 ? 4 : V;
    ref.ns = (r.d_in[0] + 2 * V1 - 1) / (2 * V1);
    auto put = [&](const void *p, size_t n) {
      size_t o = align_up(blob.size());
      blob.resize(o + n);
      memcpy(blob.data() + o, p, n);
      return o;
    };
    // transposed copies for the backward products: W2^T [H, H] and (W1^T)[:, :2H] [H, 2H]
    std::vector<float> w2t((size_t)H * H), w1t((size_t)H * 2 * H, 0.f);
    for (int f = 0; f < H; ++f)
      for (int f2 = 0; f2 < H; ++f2) w2t[(size_t)f2 * H + f] = w[r.w[1] + (size_t)f * H + f2];
    const bool has_dx = r.d_in[0] >= 2 * H;            // edge and node MLPs; not the embed MLP
    if (has_dx)
      for (int k = 0; k < 2 * H; ++k)
        for (int f = 0; f < H; ++f) w1t[(size_t)f * 2 * H + k] = w[r.w[0] + (size_t)k * H + f];
    if (l1_fp32) {                                     // the embed MLP (see EncMlp::W1x)
      const int De = m.d_edge, Tn = m.n_op_types, Dd = m.n_node_dense;
      std::vector<float> wc((size_t)(De + Dd) * H), tx;
      memcpy(wc.data(), w + r.w[0], sizeof(float) * (size_t)De * H);
      memcpy(wc.data() + (size_t)De * H, w + r.w[0] + (size_t)(De + Tn) * H, sizeof(float) * (size_t)Dd * H);
      swizzle_l1<float>(wc.data(), De + Dd, H, 4, tx);
      ref.w1x = put(tx.data(), tx.size() * 4);
      ref.nsx = (De + Dd + 7) / 8;
    }
    if (c->elem == 2) {
      std::vector<uint16_t> t;
      if (l1_fp32) {
        std::vector<float> t1;
        swizzle_l1<float>(w + r.w[0], r.d_in[0], H, 4, t1);
        ref.w1 = put(t1.data(), t1.size() * 4);
      } else {
        swizzle_l1<uint16_t>(w + r.w[0], r.d_in[0], H, V, t);
        ref.w1 = put(t.data(), t.size() * 2);
      }
      swizzle_chain<uint16_t>(w + r.w[1], H, H, H, V, t);
      ref.w2 = put(t.data(), t.size() * 2);
      swizzle_chain<uint16_t>(w2t.data(), H, H, H, V, t);
      ref.w2bt = put(t.data(), t.size() * 2);
      swizzle_chain<uint16_t>(w1t.data(), H, 2 * H, 2 * H, V, t);
      ref.w1bt = put(t.data(), t.size() * 2);
    } else {
      std::vector<float> t;
      swizzle_l1<float>(w + r.w[0], r.d_in[0], H, V, t);
      ref.w1 = put(t.data(), t.size() * 4);
      swizzle_chain<float>(w + r.w[1], H, H, H, V, t);
      ref.w2 = put(t.data(), t.size() * 4);
      swizzle_chain<float>(w2t.data(), H, H, H, V, t);
      ref.w2bt = put(t.data(), t.size() * 4);
      swizzle_chain<float>(w1t.data(), H, 2 * H, 2 * H, V, t);
      ref.w1bt = put(t.data(), t.size() * 4);
    }
    refs.push_back(ref);
  };
  add(c->L.embed, true);   // the embed MLP's first layer keeps fp32 operands in both modes
  const bool gat = m.round_kind == XRL_ROUND_GAT;
  std::vector<size_t> gat_off, gat_off_t;
  if (gat) {
    for (int r = 0; r < m.rounds; ++r) {               // one fragment-ordered [H, H] matrix per round
      size_t o = align_up(blob.size());
      if (c->elem == 2) {
        std::vector<uint16_t> t;
        swizzle_l1<uint16_t>(w + c->L.gat[r].W, H, H, V, t);
        blob.resize(o + t.size() * 2);
        memcpy(blob.data() + o, t.data(), t.size() * 2);
      } else {
        std::vector<float> t;
        swizzle_l1<float>(w + c->L.gat[r].W, H, H, V, t);
        blob.resize(o + t.size() * 4);
        memcpy(blob.data() + o, t.data(), t.size() * 4);
      }
      gat_off.push_back(o);
      std::vector<float> wt((size_t)H * H);
      for (int k = 0; k < H; ++k)
        for (int f = 0; f < H; ++f) wt[(size_t)f * H + k] = w[c->L.gat[r].W + (size_t)k * H + f];
      o = align_up(blob.size());
      if (c->elem == 2) {
        std::vector<uint16_t> t;
        swizzle_l1<uint16_t>(wt.data(), H, H, V, t);
        blob.resize(o + t.size() * 2);
        memcpy(blob.data() + o, t.data(), t.size() * 2);
      } else {
        std::vector<float> t;
        swizzle_l1<float>(wt.data(), H, H, V, t);
        blob.resize(o + t.size() * 4);
        memcpy(blob.data() + o, t.data(), t.size() * 4);
      }
      gat_off_t.push_back(o);
    }
  } else {
    for (int r = 0; r < m.rounds; ++r) { add(c->L.edge[r], false); add(c->L.node[r], false); }
  }
  // the row-MLPs read their matrices with 16-byte loads: aligned copies, keyed by flat offset
  std::vector<std::pair<int64_t, size_t>> row_off;
  for (const MlpRef *r : {&c->L.readout, &c->L.policy, &c->L.value})
    for (int l = 0; l < r->n_layers; ++l) {
      const size_t o = align_up(blob.size()), n = sizeof(float) * (size_t)r->d_in[l] * r->d_out[l];
      blob.resize(o + n);
      memcpy(blob.data() + o, w + r->w[l], n);
      row_off.push_back({r->w[l], o});
    }
  if (blob.size() > c->swz_bytes) {
    if (c->d_swz) HIP_TRY(hipFree(c->d_swz));
    c->d_swz = nullptr;
    HIP_TRY(hipMalloc((void **)&c->d_swz, blob.size()));
    c->swz_bytes = blob.size();
  }
  // synchronous copies: the host staging buffers die at return
  HIP_TRY(hipStreamSynchronize(c->stream));
  HIP_TRY(hipMemcpy(c->d_swz, blob.data(), blob.size(), hipMemcpyHostToDevice));
  HIP_TRY(hipMemcpy(c->d_w, w, sizeof(float) * c->L.total, hipMemcpyHostToDevice));
  auto bind = [&](EncMlp &e, const Ref &ref, const MlpRef &r) {
    e.W1s = c->d_swz + ref.w1;
    e.W2s = c->d_swz + ref.w2;
    e.W2bt = c->d_swz + ref.w2bt;
    e.W1bt = c->d_swz + ref.w1bt;
    e.b1 = c->d_w + r.b[0];
    e.b2 = c->d_w + r.b[1];
    e.nslab1 = ref.ns;
    e.W1x = c->d_swz + ref.w1x;
    e.nslabx = ref.nsx;
    e.table = c->d_w + r.w[0] + (size_t)m.d_edge * H;    // meaningful for the embed MLP only
  };
  c->row_w.clear();
  for (const auto &ro : row_off) c->row_w[ro.first] = (const float *)(c->d_swz + ro.second);
  size_t i = 0;
  bind(c->embed, refs[i++], c->L.embed);
  c->gatW.clear();
  if (gat) {
    c->gatWt.clear();
    for (int r = 0; r < m.rounds; ++r) {
      c->gatW.push_back(c->d_swz + gat_off[r]);
      c->gatWt.push_back(c->d_swz + gat_off_t[r]);
    }
    return XRL_OK;
  }
  c->edge.resize(m.rounds);
  c->node.resize(m.rounds);
  for (int r = 0; r < m.rounds; ++r) {
    bind(c->edge[r], refs[i++], c->L.edge[r]);
    bind(c->node[r], refs[i++], c->L.node[r]);
  }
  return XRL_OK;
}

int ensure_ws(xrl_ctx *c, size_t bytes) {
  if (bytes <= c->ws_bytes) return XRL_OK;
  HIP_TRY(hipStreamSynchronize(c->stream));
  if (c->ws) HIP_TRY(hipFree(c->ws));
  c->ws = nullptr;
  c->ws_bytes = 0;
  c->enc_batch = 0;
  c->enc_saved = false;
  hipError_t e = hipMalloc((void **)&c->ws, bytes);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return fail(XRL_ERR_OOM, "workspace of %zu bytes: %s", bytes, hipGetErrorString(e));
  }
  c->ws_bytes = bytes;
  return XRL_OK;
}

int ensure_buf(xrl_ctx *c, char **buf, size_t *have, size_t bytes, const char *what) {
  if (bytes <= *have) return XRL_OK;
  HIP_TRY(hipStreamSynchronize(c->stream));
  if (*buf) HIP_TRY(hipFree(*buf));
  *buf = nullptr;
  *have = 0;
  hipError_t e = hipMalloc((void **)buf, bytes);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return fail(XRL_ERR_OOM, "%s of %zu bytes: %s", what, bytes, hipGetErrorString(e));
  }
  *have = bytes;
  return XRL_OK;
}
int ensure_hws(xrl_ctx *c, size_t bytes) { return ensure_buf(c, &c->hws, &c->hws_bytes, bytes, "head workspace"); }
int ensure_bws(xrl_ctx *c, size_t bytes) { return ensure_buf(c, &c->bws, &c->bws_bytes, bytes, "backward workspace"); }

__global__ void fill_zero_kernel(float *p, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0.f;
}

struct Bump {
  char *base;
  size_t off = 0;
  template <typename T> T *take(size_t n) {
    T *p = (T *)(base + off);
    off += align_up(n * sizeof(T));
    return p;
  }
};

int check_batch(const xrl_ctx *c, const xrl_batch *b, const char *who) {
  if (!c || !b) return fail(XRL_ERR_NULL, "%s: ctx or batch is NULL", who);
  if (!b->uploaded) return fail(XRL_ERR_STATE, "%s: batch was not uploaded (xrl_batch_upload)", who);
  const xrl_model_desc &x = c->m, &y = b->model;
  if (x.n_op_types != y.n_op_types || x.n_node_dense != y.n_node_dense || x.d_edge != y.d_edge ||
      x.d_global != y.d_global)
    return fail(XRL_ERR_SHAPE, "%s: batch was packed for different feature widths", who);
  return XRL_OK;
}

// ---------------------------------------------------------------- launch helpers
template <typename TIn, typename TOut, int VEC, int RT>
int launch_segsum_rt(xrl_ctx *c, const void *vals, const int32_t *perm, const int32_t *ptr,
                     const int32_t *row_seg, int64_t n_rows, int64_t n_seg, int D, void *out,
                     float *carry, const int32_t *vals_seg = nullptr) {
  if (n_seg == 0) return XRL_OK;
  if (n_rows == 0) {
    static_assert(sizeof(TOut) == 4, "zero fill below writes fp32 words");
    const int64_t n = n_seg * D;
    fill_zero_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, c->stream>>>((float *)out, n);
    HIP_TRY(hipGetLastError());
    return XRL_OK;
  }
  SegsumArgs a;
  a.vals = vals; a.perm = perm; a.ptr = ptr; a.n_rows = n_rows; a.n_seg = n_seg;
  a.row_seg = vals_seg ? vals_seg : (perm ? nullptr : row_seg);
  a.D = D; a.RT = RT; a.out = out; a.carry = carry;
  const int64_t nsub = (n_rows + RT - 1) / RT;
  const int64_t threads = nsub * (D / VEC);
  const int64_t blocks = (threads + 255) / 256;
  segsum_kernel<TIn, TOut, VEC, RT><<<dim3((unsigned)blocks), dim3(256), 0, c->stream>>>(a);
  const int64_t fthreads = nsub * (D / 4);
  segsum_fixup<TOut><<<dim3((unsigned)((fthreads + 255) / 256)), dim3(256), 0, c->stream>>>(
      ptr, row_seg, n_rows, n_seg, D, RT, carry, (TOut *)out);
  HIP_TRY(hipGetLastError());
  return XRL_OK;
}

// Rows per sub-tile: 16 keeps sixteen 16-byte loads in flight per lane; tiny inputs (under 1 MB)
// use 4 so that they still produce a few waves per compute unit.
inline int segsum_rt(int64_t n_rows, int D, size_t elem) { return (size_t)n_rows * D * elem < ((size_t)1 << 20) ? 4 : 16; }

template <typename TIn, typename TOut, int VEC>
int launch_segsum(xrl_ctx *c, const void *vals, const int32_t *perm, const int32_t *ptr,
                  const int32_t *row_seg, int64_t n_rows, int64_t n_seg, int D, void *out,
                  float *carry) {
  if (segsum_rt(n_rows, D, sizeof(TIn)) == 4)
    return launch_segsum_rt<TIn, TOut, VEC, 4>(c, vals, perm, ptr, row_seg, n_rows, n_seg, D, out, carry);
  return launch_segsum_rt<TIn, TOut, VEC, 16>(c, vals, perm, ptr, row_seg, n_rows, n_seg, D, out, carry);
}

size_t segsum_carry_floats(int64_t n_rows, int D) { return (size_t)((n_rows + 3) / 4) * 2 * D; }

template <typename T, int H>
int launch_mlp2_h(xrl_ctx *c, int kind, const Mlp2Args &a) {
  if (a.n_rows <= 0) return XRL_OK;
  const unsigned grid = (unsigned)(((a.n_blocks + 7) / 8) * 8);
  if (kind == KIND_EMBED) mlp2_kernel<float, T, H, KIND_EMBED><<<dim3(grid), dim3(256), 0, c->stream>>>(a);
  else if (kind == KIND_EDGE) mlp2_kernel<T, T, H, KIND_EDGE><<<dim3(grid), dim3(256), 0, c->stream>>>(a);
  else mlp2_kernel<T, T, H, KIND_NODE><<<dim3(grid), dim3(256), 0, c->stream>>>(a);
  HIP_TRY(hipGetLastError());
  return XRL_OK;
}

// Persistent LDS-resident-weights variant (bf16, H <= 128, edge and node kinds).
constexpr int kPersistWaves = 8;
inline size_t mlp2p_lds_bytes(int H, int nslab1) {
  const int MB = H / 32, HS = H / 16;
  return ((size_t)nslab1 * MB + (size_t)HS * MB) * 1024 + (size_t)MB * 256 +
         (size_t)kPersistWaves * RowStage<bf16_t, 128>::BYTES;   // staging sized for the widest H served
}

template <int H, int KIND, bool SAVE>
int launch_mlp2p_ks(xrl_ctx *c, Mlp2Args &a, size_t lds) {
  constexpr int NW = kPersistWaves;
  auto kern = mlp2p_kernel<bf16_t, H, KIND, NW, SAVE>;
  static bool attr_set = false;          // one attribute per kernel instantiation
  if (!attr_set) {
    HIP_TRY(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    attr_set = true;
  }
  const int64_t n_wt = KIND == KIND_EDGE ? a.n_tiles : (a.n_rows + 31) / 32;
  a.n_blocks = n_wt;
  int64_t grid = ((n_wt + NW - 1) / NW + 7) / 8 * 8;
  const int64_t cap = (int64_t)c->n_cu / 8 * 8;
  if (grid > cap) grid = cap;
  kern<<<dim3((unsigned)grid), dim3(64 * NW), lds, c->stream>>>(a);
  HIP_TRY(hipGetLastError());
  return XRL_OK;
}

template <int H, int KIND>
int launch_mlp2p_k(xrl_ctx *c, Mlp2Args &a, size_t lds) {
  return a.z1 ? launch_mlp2p_ks<H, KIND, true>(c, a, lds) : launch_mlp2p_ks<H, KIND, false>(c, a, lds);
}

template <int H>
int launch_mlp2p(xrl_ctx *c, int kind, Mlp2Args &a) {
  const size_t lds = mlp2p_lds_bytes(H, a.nslab1);
  if (kind == KIND_EDGE) return launch_mlp2p_k<H, KIND_EDGE>(c, a, lds);
  return launch_mlp2p_k<H, KIND_NODE>(c, a, lds);
}

constexpr int embedp_waves(int H) { return H > 128 ? 4 : kPersistWaves; }
inline size_t embedp_lds_bytes(int H, int nslabx, int Tn) {
  const int MB = H / 32, HS = H / 16;
  const size_t w = ((size_t)nslabx * MB + (size_t)HS * MB) * 1024 + (size_t)MB * 256;
  if (H > 128) return w + (size_t)embedp_waves(H) * BlockStage<bf16_t>::BYTES;     // table stays in global memory
  return w + (size_t)Tn * H * 4 + (size_t)kPersistWaves * RowStage<bf16_t, 128>::BYTES;
}

template <int H, bool SAVE>
int launch_embedp_s(xrl_ctx *c, Mlp2Args &a) {
  constexpr int NW = embedp_waves(H);
  const size_t lds = embedp_lds_bytes(H, a.nslabx, a.Tn);
  auto kern = embedp_kernel<bf16_t, H, NW, SAVE>;
  static size_t attr_lds = 0;
  if (lds > attr_lds) {
    HIP_TRY(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    attr_lds = lds;
  }
  const int64_t n_wt = (a.n_rows + 31) / 32;
  a.n_blocks = n_wt;
  int64_t grid = ((n_wt + NW - 1) / NW + 7) / 8 * 8;
  const int per_cu = 2 * lds <= (size_t)c->max_lds ? 2 : 1;   // blocks that fit a CU's LDS
  const int64_t cap = (int64_t)c->n_cu / 8 * 8 * per_cu;
  if (grid > cap) grid = cap;
  kern<<<dim3((unsigned)grid), dim3(64 * NW), lds, c->stream>>>(a);
  HIP_TRY(hipGetLastError());
  return XRL_OK;
}

template <int H>
int launch_embedp(xrl_ctx *c, Mlp2Args &a) {
  return a.z1 ? launch_embedp_s<H, true>(c, a) : launch_embedp_s<H, false>(c, a);
}

inline bool mlp2p_applies(const xrl_ctx *c, int kind, const Mlp2Args &a) {
  const int H = c->m.hidden;
  if (c->elem != 2 || a.n_rows <= 0) return false;
  if (a.n_rows < c->p_min_rows) return false;
  if (kind == KIND_EMBED) {
    const int pieces = 4 * 64 * embedp_waves(H);             // see embedp_kernel
    return a.nslabx <= 2 && a.nslabx * (H / 32) * 64 <= pieces && (H > 128 || a.Tn * (H / 4) <= pieces) &&
           embedp_lds_bytes(H, a.nslabx, a.Tn) <= (size_t)c->max_lds;
  }
  if (H > 128) return false;
  if (kind == KIND_EDGE && a.nslab1 != 2 * (H / 16) + 1) return false;   // edge attrs must fit one slab
  return mlp2p_lds_bytes(H, a.nslab1) <= (size_t)c->max_lds;
}

// Register-stationary variant (bf16, edge and node kinds).
template <int H, int KIND, bool SAVE>
int launch_mlp2r_ks(xrl_ctx *c, Mlp2Args &a) {
  using R = RTile<H, KIND>;
  auto kern = mlp2r_kernel<H, KIND, SAVE>;
  static bool attr_set = false;
  if (!attr_set) {
    HIP_TRY(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, R::BYTES));
    attr_set = true;
  }
  const int64_t n_wt = KIND == KIND_EDGE ? a.n_tiles : (a.n_rows + 31) / 32;
  a.n_blocks = n_wt;
  const int by_lds = c->max_lds / R::BYTES, by_waves = 4 * R::WAVES_PER_SIMD / R::MB;
  const int per_cu = by_lds < by_waves ? by_lds : by_waves;      // blocks that can be resident on a CU
  int64_t grid = (n_wt + 7) / 8 * 8;
  const int64_t cap = (int64_t)c->n_cu / 8 * 8 * per_cu;
  if (grid > cap) grid = cap;
  kern<<<dim3((unsigned)grid), dim3(R::NT), R::BYTES, c->stream>>>(a);
  HIP_TRY(hipGetLastError());
  return XRL_OK;
}

template <int H, int KIND>
int launch_mlp2r_k(xrl_ctx *c, Mlp2Args &a) {
  return a.z1 ? launch_mlp2r_ks<H, KIND, true>(c, a) : launch_mlp2r_ks<H, KIND, false>(c, a);
}

template <int H>
int launch_mlp2r(xrl_ctx *c, int kind, Mlp2Args &a) {
  return kind == KIND_EDGE ? launch_mlp2r_k<H, KIND_EDGE>(c, a) : launch_mlp2r_k<H, KIND_NODE>(c, a);
}

inline bool mlp2r_applies(const xrl_ctx *c, int kind, const Mlp2Args &a) {
  // H = 256 only: at H <= 128 the weights fit LDS, a wave then runs its tile without block
  // barriers, and that kernel (mlp2p) measured faster (the template itself covers 64 and 128)
  const int H = c->m.hidden;
  if (c->elem != 2 || H != 256 || kind == KIND_EMBED || a.n_rows <= 0) return false;
  if (a.n_rows < c->p_min_rows) return false;
  if (kind == KIND_EDGE && (a.De > 8 || a.nslab1 != 2 * (H / 16) + 1)) return false;   // edge attrs: half a slab
  return RTile<256, KIND_EDGE>::BYTES <= c->max_lds;
}

template <typename T>
int launch_mlp2(xrl_ctx *c, int kind, Mlp2Args &a) {
  if (mlp2r_applies(c, kind, a))
    return launch_mlp2r<256>(c, kind, a);
  if (mlp2p_applies(c, kind, a)) {
    if (kind == KIND_EMBED)
      return c->m.hidden == 64 ? launch_embedp<64>(c, a) : c->m.hidden == 128 ? launch_embedp<128>(c, a) : launch_embedp<256>(c, a);
    return c->m.hidden == 64 ? launch_mlp2p<64>(c, kind, a) : launch_mlp2p<128>(c, kind, a);
  }
  a.n_blocks = kind == KIND_EDGE ? (a.n_tiles + 3) / 4 : (a.n_rows + 127) / 128;
  switch (c->m.hidden) {
    case 64: return launch_mlp2_h<T, 64>(c, kind, a);
    case 128: return launch_mlp2_h<T, 128>(c, kind, a);
    case 256: return launch_mlp2_h<T, 256>(c, kind, a);
  }
  return fail(XRL_ERR_UNSUPPORTED, "hidden = %d", c->m.hidden);
}

RowMlpArgs rowmlp_args(xrl_ctx *c, const MlpRef &r, bool relu_last, const float *in1, int w1, const float *in2,
                       int w2, int64_t n_rows, float *out, float *const *act, int *dmax_out = nullptr) {
  RowMlpArgs a;
  memset(&a, 0, sizeof(a));
  a.n_layers = r.n_layers;
  a.relu_last = relu_last ? 1 : 0;
  int dmax = r.d_in[0];
  for (int l = 0; l < r.n_layers; ++l) {
    const auto it = c->row_w.find(r.w[l]);
    a.W[l] = it != c->row_w.end() ? it->second : c->d_w + r.w[l];
    a.b[l] = c->d_w + r.b[l];
    a.d_in[l] = r.d_in[l];
    a.d_out[l] = r.d_out[l];
    a.act[l] = act ? act[l] : nullptr;
    if (r.d_out[l] > dmax) dmax = r.d_out[l];
  }
  a.in1 = in1; a.in2 = in2; a.w1 = w1; a.w2 = w2; a.n_rows = n_rows; a.out = out;
  if (dmax_out) *dmax_out = dmax;
  return a;
}

int launch_rowmlp(xrl_ctx *c, const MlpRef &r, bool relu_last, const float *in1, int w1,
                  const float *in2, int w2, int64_t n_rows, float *out, float *const *act) {
  if (n_rows <= 0) return XRL_OK;
  int dmax = 0;
  const RowMlpArgs a = rowmlp_args(c, r, relu_last, in1, w1, in2, w2, n_rows, out, act, &dmax);
  if (n_rows <= 4096) {
    rowmlp_kernel<1><<<dim3((unsigned)n_rows), dim3(256), (size_t)(1024 + 2 * dmax) * sizeof(float), c->stream>>>(a);
  } else {
    const unsigned blocks = (unsigned)((n_rows + 7) / 8);
    rowmlp_kernel<8><<<dim3(blocks), dim3(256), (size_t)2 * 8 * dmax * sizeof(float), c->stream>>>(a);
  }
  HIP_TRY(hipGetLastError());
  return XRL_OK;
}

// Policy MLP, per-state softmax statistics and value head (Section 3.3.2): one launch for batches
// of up to kMaxFusedSlots slots, otherwise the row-MLP kernel followed by the per-state kernel.
// pact / vact (nullable) receive every layer's output for the backward pass.
int launch_heads(xrl_ctx *c, const xrl_batch *b, const float *d_emb, float *logit, float *logp, float *entropy,
                 int32_t *action, float *zmean, float *value, float *const *pact, float *const *vact) {
  const int H = c->m.hidden;
  const xrl_batch_device &d = b->dev;
  const RowMlpArgs va = rowmlp_args(c, c->L.value, false, zmean, H, nullptr, 0, b->S, value, vact);
  if (b->G <= kMaxFusedSlots) {
    const RowMlpArgs pa = rowmlp_args(c, c->L.policy, false, d_emb, H, nullptr, 0, b->G, logit, pact);
    policy_value_kernel<<<dim3((unsigned)(b->G + b->S)), dim3(256), 0, c->stream>>>(
        pa, d.mask, d.state_graph_ptr, (int)b->G, (int)b->S, H, c->d_counter, logp, entropy, action, zmean, va);
    const hipError_t le = hipGetLastError();
    if (le != hipSuccess) {
      // (a launch that the runtime rejected has not run; one that failed later may have left
      // counters of unfinished states above zero: they go back to zero before the next use)
      (void)hipMemsetAsync(c->d_counter, 0, sizeof(int32_t) * kMaxFusedSlots, c->stream);
      return fail(XRL_ERR_HIP, "policy_value_kernel: %s", hipGetErrorString(le));
    }
    return XRL_OK;
  }
  int rc = launch_rowmlp(c, c->L.policy, false, d_emb, H, nullptr, 0, b->G, logit, pact);
  if (rc) return rc;
  state_policy_kernel<<<dim3((unsigned)b->S), dim3(256), 0, c->stream>>>(
      logit, d.mask, d.state_graph_ptr, d_emb, H, logp, entropy, action, zmean, va);
  HIP_TRY(hipGetLastError());
  return XRL_OK;
}

// row_src (or nullptr): the row of src to export for each row, -1 = a row of zeros
template <typename T>
__global__ void export_rows_kernel(const T *src, int64_t n_rows, int D, const int32_t *row_src, float *dst) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_rows * D) return;
  if (row_src) {
    const int64_t r = i / D;
    const int32_t s = row_src[r];
    dst[i] = s < 0 ? 0.f : (float)src[(int64_t)s * D + (i - r * D)];
    return;
  }
  dst[i] = (float)src[i];
}


template <typename T1, typename T, int H, int KIND>
int launch_mlp2_bwd_k(xrl_ctx *c, const Mlp2BwdArgs &a) {
  constexpr size_t lds = mlp2_bwd_lds_bytes<T, H>();
  auto kern = mlp2_bwd_kernel<T1, T, H, KIND>;
  static bool attr_set = false;          // one attribute per kernel instantiation
  if (!attr_set) {
    HIP_TRY(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    attr_set = true;
  }
  const unsigned grid = (unsigned)(((a.n_blocks + 7) / 8) * 8);
  kern<<<dim3(grid), dim3(256), lds, c->stream>>>(a);
  HIP_TRY(hipGetLastError());
  return XRL_OK;
}

template <typename T, int H>
int launch_mlp2_bwd_h(xrl_ctx *c, int kind, const Mlp2BwdArgs &a) {
  if (a.n_rows <= 0) return XRL_OK;
  if (kind == KIND_EMBED) return launch_mlp2_bwd_k<float, T, H, KIND_EMBED>(c, a);
  if (kind == KIND_EDGE) return launch_mlp2_bwd_k<T, T, H, KIND_EDGE>(c, a);
  return launch_mlp2_bwd_k<T, T, H, KIND_NODE>(c, a);
}

template <typename T>
int launch_mlp2_bwd(xrl_ctx *c, int kind, Mlp2BwdArgs &a) {
  a.n_blocks = (a.n_rows + 127) / 128;
  switch (c->m.hidden) {
    case 64: return launch_mlp2_bwd_h<T, 64>(c, kind, a);
    case 128: return launch_mlp2_bwd_h<T, 128>(c, kind, a);
    case 256: return launch_mlp2_bwd_h<T, 256>(c, kind, a);
  }
  return fail(XRL_ERR_UNSUPPORTED, "hidden = %d", c->m.hidden);
}

template <int H, int KIND, bool FOLD, bool GIVEN = false>
int launch_mlp2_bwdz_k(xrl_ctx *c, Mlp2BwdzArgs &a) {
  using S = BwdzShape<H>;
  auto kern = mlp2_bwdz_kernel<H, KIND, FOLD, GIVEN>;
  static bool attr_set = false;          // one attribute per kernel instantiation
  if (!attr_set) {
    HIP_TRY(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)S::LDS));
    attr_set = true;
  }
  const int64_t wave_tiles = KIND == KIND_EDGE ? a.n_tiles : (a.n_rows + 31) / 32;   // EDGE: the packer's edge tiles
  a.n_blocks = (wave_tiles + S::NW - 1) / S::NW;               // groups of NW tiles
  const unsigned grid = (unsigned)((a.n_blocks + 7) / 8 * 8);
  kern<<<dim3(grid), dim3(64 * S::NW), S::LDS, c->stream>>>(a);
  HIP_TRY(hipGetLastError());
  return XRL_OK;
}

template <int H>
int launch_mlp2_bwdz_h(xrl_ctx *c, int kind, Mlp2BwdzArgs &a, bool fold, bool given) {
  if (a.n_rows <= 0) return XRL_OK;
  if (kind == KIND_EMBED)
    return given ? launch_mlp2_bwdz_k<H, KIND_EMBED, false, true>(c, a) : launch_mlp2_bwdz_k<H, KIND_EMBED, false>(c, a);
  if (kind == KIND_EDGE) return fold ? launch_mlp2_bwdz_k<H, KIND_EDGE, true>(c, a) : launch_mlp2_bwdz_k<H, KIND_EDGE, false>(c, a);
  return given ? launch_mlp2_bwdz_k<H, KIND_NODE, false, true>(c, a) : launch_mlp2_bwdz_k<H, KIND_NODE, false>(c, a);
}

// fold (EDGE): dx_b receives the gradients w.r.t. h_receiver summed per receiver, [N, H].
// given (NODE, EMBED): a.dy is dz2 already (the gradient gather applied the layer's output mask)
int launch_mlp2_bwdz(xrl_ctx *c, int kind, Mlp2BwdzArgs &a, bool fold, bool given) {
  switch (c->m.hidden) {
    case 64: return launch_mlp2_bwdz_h<64>(c, kind, a, fold, given);
    case 128: return launch_mlp2_bwdz_h<128>(c, kind, a, fold, given);
    case 256: return launch_mlp2_bwdz_h<256>(c, kind, a, fold, given);
  }
  return fail(XRL_ERR_UNSUPPORTED, "hidden = %d", c->m.hidden);
}

// rows per chunk / number of chunks of the weight-gradient kernels
inline void wgrad_chunks(int64_t n_rows, int *rows_per_chunk, int *n_chunks) {
  int64_t nc = (n_rows + 127) / 128;        // (small batches: enough chunks to occupy the machine)
  if (nc > 512) nc = 512;
  if (nc < 1) nc = 1;
  int64_t rpc = (n_rows + nc - 1) / nc;
  rpc = (rpc + 63) / 64 * 64;
  *rows_per_chunk = (int)rpc;
  *n_chunks = (int)((n_rows + rpc - 1) / rpc);
  if (*n_chunks < 1) *n_chunks = 1;
}
inline size_t wgrad_partial_floats(int64_t n_rows, int Ka, int H, int n_cu) {
  int rpc, nc;
  wgrad_chunks(n_rows, &rpc, &nc);
  // transpose-read kernel: at most n_cu wide tiles of 256 columns plus 2 n_cu tiles of 128, or
  // 2 n_cu tiles of 128 columns alone (see launch_wgrad_h)
  const size_t wide = (size_t)n_cu * 256 * H + (size_t)2 * n_cu * 128 * H;
  return std::max((size_t)nc * ((Ka + 1 + 63) / 64 * 64) * H, wide);
}

template <int H, int KIND, int TA>
int launch_wgrad2(xrl_ctx *c, const WgradArgs &a, const Wgrad2Plan &p, int ka_base, int KaP, int bias_row) {
  constexpr int RS = TA == 256 ? 64 : 32;      // the wide tiles run one block per CU: 64 rows in flight per stage
  constexpr size_t lds = wgrad2_lds_bytes<H, TA, RS>();
  auto kern = wgrad2_kernel<H, KIND, TA, RS>;
  static bool attr_set = false;          // one attribute per kernel instantiation
  if (!attr_set) {
    HIP_TRY(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    attr_set = true;
  }
  WgradArgs b = a;
  b.rows_per_chunk = p.rows_per_slot;
  b.n_chunks = p.ny;
  kern<<<dim3((unsigned)(p.ny * p.kt)), dim3(2 * TA), lds, c->stream>>>(b, p.kt, p.ny, ka_base, KaP, bias_row);
  HIP_TRY(hipGetLastError());
  return XRL_OK;
}

template <int H, int TA>
int launch_wgrad2_kind(xrl_ctx *c, int kind, const WgradArgs &a, const Wgrad2Plan &p, int ka_base, int KaP,
                       int bias_row = -1) {
  if (kind == WG_PLAIN) return launch_wgrad2<H, WG_PLAIN, TA>(c, a, p, ka_base, KaP, bias_row);
  if (kind == WG_EDGE) return launch_wgrad2<H, WG_EDGE, TA>(c, a, p, ka_base, KaP, bias_row);
  return launch_wgrad2<H, WG_NODE, TA>(c, a, p, ka_base, KaP, bias_row);
}

template <typename T, int H>
int launch_wgrad_h(xrl_ctx *c, int kind, WgradArgs &a, float *dW, float *db) {
  if (a.n_rows <= 0) return XRL_OK;
  const int64_t n = (int64_t)(a.Ka + 1) * H;
  auto reduce = [&](const float *partial, int n_chunks, int KaP, int Ka, float *dw, float *dbias) {
    const int64_t cnt = (int64_t)(Ka + (dbias ? 1 : 0)) * H;
    if (cnt > 0)
      wgrad_reduce_kernel<<<dim3((unsigned)((cnt + 31) / 32)), dim3(256), 0, c->stream>>>(partial, n_chunks, KaP, Ka, H,
                                                                                         dw, dbias);
  };
  if constexpr (sizeof(T) == 2) {
    if (kind != WG_EMBED) {                                // transpose-read kernel
      int rc;
      const int k_main = kind == WG_PLAIN ? a.Ka : 2 * H;  // the H-wide column parts
      bool wide = false;
      if constexpr (H >= 128) wide = k_main % 256 == 0 && a.n_rows >= c->wide_min_rows;
      // PLAIN and NODE have one column past the H-wide parts, the all-ones bias column: its sums
      // come from the vector ALU of the first tile's blocks (EDGE also has the edge attributes
      // there and keeps them on the matrix cores)
      const bool only_bias = kind != WG_EDGE && a.Ka == k_main && k_main % 128 == 0;
      if (wide) {
        if constexpr (H >= 128) {
          const Wgrad2Plan pa = wgrad2_plan(a.n_rows, k_main / 256, c->n_cu, 1);
          const int KaP = k_main + (only_bias && db ? 1 : 0);
          if ((rc = launch_wgrad2_kind<H, 256>(c, kind, a, pa, 0, KaP, only_bias && db ? k_main : -1))) return rc;
          reduce(a.partial, pa.ny, KaP, k_main, dW, only_bias ? db : nullptr);
          if (!only_bias) {
            // one launch of narrow tiles for the columns past the H-wide parts
            WgradArgs t = a;
            t.partial = a.partial + (size_t)pa.ny * KaP * H;
            const Wgrad2Plan pb = wgrad2_plan(a.n_rows, 1, c->n_cu, 2);
            if ((rc = launch_wgrad2_kind<H, 128>(c, kind, t, pb, k_main, 128))) return rc;
            reduce(t.partial, pb.ny, 128, a.Ka - k_main, dW + (size_t)k_main * H, db);
          }
        }
      } else if (only_bias) {
        const Wgrad2Plan p = wgrad2_plan(a.n_rows, k_main / 128, c->n_cu, 2);
        const int KaP = k_main + (db ? 1 : 0);
        if ((rc = launch_wgrad2_kind<H, 128>(c, kind, a, p, 0, KaP, db ? k_main : -1))) return rc;
        reduce(a.partial, p.ny, KaP, a.Ka, dW, db);
      } else {
        const Wgrad2Plan p = wgrad2_plan(a.n_rows, (a.Ka + 1 + 127) / 128, c->n_cu, 2);
        if ((rc = launch_wgrad2_kind<H, 128>(c, kind, a, p, 0, p.kt * 128))) return rc;
        reduce(a.partial, p.ny, p.kt * 128, a.Ka, dW, db);
      }
      HIP_TRY(hipGetLastError());
      return XRL_OK;
    }
  }
  wgrad_chunks(a.n_rows, &a.rows_per_chunk, &a.n_chunks);
  const int kt = (a.Ka + 1 + 63) / 64;
  dim3 grid((unsigned)kt, (unsigned)a.n_chunks);
  if (kind == WG_PLAIN) wgrad_kernel<T, H, WG_PLAIN><<<grid, dim3(256), 0, c->stream>>>(a);
  else if (kind == WG_EDGE) wgrad_kernel<T, H, WG_EDGE><<<grid, dim3(256), 0, c->stream>>>(a);
  else if (kind == WG_NODE) wgrad_kernel<T, H, WG_NODE><<<grid, dim3(256), 0, c->stream>>>(a);
  else wgrad_kernel<T, H, WG_EMBED><<<grid, dim3(256), 0, c->stream>>>(a);
  wgrad_reduce_kernel<<<dim3((unsigned)((n + 31) / 32)), dim3(256), 0, c->stream>>>(
      a.partial, a.n_chunks, kt * 64, a.Ka, H, dW, db);
  HIP_TRY(hipGetLastError());
  return XRL_OK;
}

template <typename T>
int launch_wgrad(xrl_ctx *c, int kind, WgradArgs &a, float *dW, float *db) {
  switch (c->m.hidden) {
    case 64: return launch_wgrad_h<T, 64>(c, kind, a, dW, db);
    case 128: return launch_wgrad_h<T, 128>(c, kind, a, dW, db);
    case 256: return launch_wgrad_h<T, 256>(c, kind, a, dW, db);
  }
  return fail(XRL_ERR_UNSUPPORTED, "hidden = %d", c->m.hidden);
}

// dW[Kx, H] += X[:, :Kx]^T dZ and db += 1^T dZ for X = a.A [rows, a.Ka] (a.Ka = Kx rounded up to 8, the
// columns past Kx zero): the plain product, whose tile also holds the all-ones column at a.Ka
template <typename T>
int launch_wgrad_embed_rows(xrl_ctx *c, WgradArgs &a, int Kx, float *dW, float *db) {
  if constexpr (sizeof(T) == 2) {
    if (a.n_rows <= 0) return XRL_OK;
    auto run = [&](auto h) -> int {
      constexpr int H = decltype(h)::value;
      const Wgrad2Plan p = wgrad2_plan(a.n_rows, (a.Ka + 1 + 127) / 128, c->n_cu, 2);
      const int KaP = p.kt * 128;
      int rc = launch_wgrad2<H, WG_PLAIN, 128>(c, a, p, 0, KaP, -1);
      if (rc) return rc;
      const int64_t cnt_w = (int64_t)Kx * H;
      if (cnt_w > 0)
        wgrad_reduce_kernel<<<dim3((unsigned)((cnt_w + 31) / 32)), dim3(256), 0, c->stream>>>(a.partial, p.ny, KaP, Kx, H, dW, nullptr);
      wgrad_reduce_kernel<<<dim3((unsigned)((H + 31) / 32)), dim3(256), 0, c->stream>>>(a.partial + (size_t)a.Ka * H, p.ny, KaP, 0, H,
                                                                                     nullptr, db);
      HIP_TRY(hipGetLastError());
      return XRL_OK;
    };
    switch (c->m.hidden) {
      case 64: return run(std::integral_constant<int, 64>());
      case 128: return run(std::integral_constant<int, 128>());
      case 256: return run(std::integral_constant<int, 256>());
    }
  }
  return fail(XRL_ERR_UNSUPPORTED, "launch_wgrad_embed_rows: bf16 contexts only");
}

int launch_rowmlp_bwd(xrl_ctx *c, const MlpRef &r, bool relu_last, float *const *act, const float *dout,
                      int64_t n_rows, float *const *dz, float *dx) {
  if (n_rows <= 0) return XRL_OK;
  RowMlpBwdArgs a;
  memset(&a, 0, sizeof(a));
  a.n_layers = r.n_layers;
  a.relu_last = relu_last ? 1 : 0;
  int dmax = r.d_in[0];
  for (int l = 0; l < r.n_layers; ++l) {
    a.W[l] = c->d_w + r.w[l];
    a.d_in[l] = r.d_in[l];
    a.d_out[l] = r.d_out[l];
    a.act[l] = act[l];
    a.dz[l] = dz[l];
    if (r.d_out[l] > dmax) dmax = r.d_out[l];
  }
  a.dout = dout; a.n_rows = n_rows; a.dx = dx;
  if (n_rows <= 4096) {
    rowmlp_bwd_kernel<1><<<dim3((unsigned)n_rows), dim3(256), (size_t)2 * dmax * sizeof(float), c->stream>>>(a);
  } else {
    const unsigned blocks = (unsigned)((n_rows + 7) / 8);
    rowmlp_bwd_kernel<8><<<dim3(blocks), dim3(256), (size_t)2 * 8 * dmax * sizeof(float), c->stream>>>(a);
  }
  HIP_TRY(hipGetLastError());
  return XRL_OK;
}

// dW, db of every layer of a small row-MLP: x of layer 0 is [x1 | x2], of layer l > 0 act[l-1].
// Above kSmallWgradRows rows the rows are cut into chunks of that size (as many as `partial`,
// partial_floats long, has room for) whose partial sums are reduced in chunk order.
constexpr int kSmallWgradRows = 512;
inline size_t small_wgrad_partial_floats(const MlpRef &r, int64_t n_rows) {
  size_t big = 0;
  for (int l = 0; l < r.n_layers; ++l) big = std::max(big, (size_t)(r.d_in[l] + 1) * r.d_out[l]);
  const int64_t nc = (n_rows + kSmallWgradRows - 1) / kSmallWgradRows;
  return nc > 1 ? big * (size_t)nc : 0;
}
int launch_small_wgrads(xrl_ctx *c, const MlpRef &r, const float *x1, int w1, const float *x2, int w2,
                        float *const *act, float *const *dz, int64_t n_rows, float *dweights,
                        float *partial, size_t partial_floats) {
  if (n_rows <= 0) return XRL_OK;
  for (int l = 0; l < r.n_layers; ++l) {
    const int64_t n = (int64_t)(r.d_in[l] + 1) * r.d_out[l];
    const float *a1 = l == 0 ? x1 : act[l - 1];
    const int aw1 = l == 0 ? w1 : r.d_in[l];
    int64_t nc = (n_rows + kSmallWgradRows - 1) / kSmallWgradRows;
    if (partial && (size_t)nc * n > partial_floats) nc = (int64_t)(partial_floats / n);
    if (!partial || nc < 2) nc = 1;
    if (nc > 65535) nc = 65535;
    const int64_t rpc = (n_rows + nc - 1) / nc;
    nc = (n_rows + rpc - 1) / rpc;
    float *dW = dweights + r.w[l], *db = dweights + r.b[l];
    small_wgrad_kernel<<<dim3((unsigned)((n + 255) / 256), (unsigned)nc), dim3(256), 0, c->stream>>>(
        a1, aw1, l == 0 ? x2 : nullptr, l == 0 ? w2 : 0, dz[l], n_rows, (int)rpc, r.d_in[l], r.d_out[l], dW, db,
        nc > 1 ? partial : nullptr);
    if (nc > 1)
      wgrad_reduce_kernel<<<dim3((unsigned)((n + 31) / 32)), dim3(256), 0, c->stream>>>(
          partial, (int)nc, r.d_in[l] + 1, r.d_in[l], r.d_out[l], dW, db);
  }
  HIP_TRY(hipGetLastError());
  return XRL_OK;
}

// demb[j, :] = mask[j] ? demb[j, :] + dz[s, :] * inv_n[s] : 0 for the slots j of state s; one block
// per slot (a batch may be a single state of hundreds of slots), which finds its state by bisection
__global__ void demb_combine_kernel(float *demb, const float *dzs, const float *inv_n, const uint8_t *mask,
                                    const int32_t *state_graph_ptr, int S, int H) {
  const int j = blockIdx.x;
  int lo = 0, hi = S;                       // state_graph_ptr[lo] <= j < state_graph_ptr[hi]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (state_graph_ptr[mid] <= j) lo = mid; else hi = mid;
  }
  const float w = inv_n[lo];
  const bool on = mask[j] != 0;
  for (int f = threadIdx.x; f < H; f += blockDim.x) {
    const size_t o = (size_t)j * H + f;
    demb[o] = on ? demb[o] + dzs[(size_t)lo * H + f] * w : 0.f;
  }
}

// dh[n, :] = dx[graph(n), :H] (divided by the graph's node count for the mean readout), stored in
// the operand type like every later dh; one thread per four columns. node_graph null: one row per
// graph (n = the graph)
template <typename T>
__global__ void broadcast_dpool_kernel(const float *dx, int ldx, const int32_t *node_graph,
                                       const int32_t *graph_node_ptr, int mean, int64_t N, int H, T *dh) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int q = H / 4;
  if (i >= N * q) return;
  const int64_t n = i / q;
  const int f = (int)(i - n * q) * 4, gph = node_graph ? node_graph[n] : (int)n;
  float v[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) v[j] = dx[(size_t)gph * ldx + f + j];
  if (mean) {
    const int cnt = graph_node_ptr[gph + 1] - graph_node_ptr[gph];
    const float d = (float)(cnt > 1 ? cnt : 1);
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] /= d;
  }
  store4<T>(dh + (size_t)n * H + f, v);
}

// The node-update layer's input rows written out for its weight gradient (bf16 path):
// X[n, :] = [sum over node n's in-edges (receiver order: the node-update kernel's order) of their
// attribute rows | one-hot operator type | dense attributes | zeros up to Kp columns]; one thread per
// node and eight columns.
__global__ void embed_input_rows_kernel(const float *edge_feat, const int32_t *in_ptr, const int32_t *node_op,
                                        const float *node_dense, int64_t N, int De, int Tn, int Dd, int Kp, bf16_t *X) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int q = Kp / 8;
  if (i >= N * q) return;
  const int64_t n = i / q;
  const int k0 = (int)(i - n * q) * 8;
  float v[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) v[j] = 0.f;
  if (k0 < De) {
    // (De is a multiple of 4 and k0 of 8: columns k0 .. k0+3 are attributes, k0+4 .. k0+7 all or none)
    const bool two = k0 + 8 <= De;
    const int e1 = in_ptr[n + 1];
    for (int e = in_ptr[n]; e < e1; ++e) {
      const float *p = edge_feat + (size_t)e * De + k0;
      const f32x4 lo = *(const f32x4 *)p;
#pragma unroll
      for (int j = 0; j < 4; ++j) v[j] += lo[j];
      if (two) {
        const f32x4 hi = *(const f32x4 *)(p + 4);
#pragma unroll
        for (int j = 0; j < 4; ++j) v[4 + j] += hi[j];
      }
    }
  }
  const int op = node_op[n];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int k = k0 + j;
    if (k >= De && k < De + Tn) v[j] = k - De == op ? 1.f : 0.f;
    else if (k >= De + Tn && k < De + Tn + Dd) v[j] = node_dense[(size_t)n * Dd + (k - De - Tn)];
  }
  *(bf16x8 *)(X + (size_t)n * Kp + k0) = pack_bf16x8(v[0], v[1], v[2], v[3], v[4], v[5], v[6], v[7]);
}

template <typename T>
int encode_backward_impl(xrl_ctx *c, const xrl_batch *b, const float *d_demb, float *dweights) {
  const xrl_model_desc &m = c->m;
  const int H = m.hidden, R = m.rounds, De = m.d_edge, Dg = m.d_global;
  const int64_t N = b->N, E = b->E, G = b->G;
  const int64_t M = N > E ? N : E;
  const xrl_batch_device &d = b->dev;
  // ---- scratch plan
  size_t need = 0;
  auto acc = [&](size_t bytes) { need += align_up(bytes); };
  const bool kept = c->fwd_kept;                                   // the forward kept z1 and the ReLU masks
  // the per-edge gradients w.r.t. h_receiver leave the edge kernel already summed per receiver
  // (edge tiles end at receiver boundaries unless a receiver has more than 32 in-edges)
  const bool fold = kept && b->n_split_tiles == 0;
  for (int i = 0; i < (kept ? 2 : 3); ++i) acc((size_t)M * H * sizeof(T));      // (z1,) dz1, dz2
  acc((size_t)E * H * sizeof(T));                                  // per-edge d h_sender
  acc((size_t)M * H * sizeof(T));                                  // d h_receiver: per edge, or summed per receiver
  for (int i = 0; i < 3; ++i) acc((size_t)N * H * sizeof(T));      // dh (two buffers), dagg
  // bf16: the node-update layer's input rows are written out for its weight gradient, Kp columns
  const int Kx = De + m.n_op_types + m.n_node_dense, Kp = (Kx + 7) / 8 * 8;
  const bool embed_rows = sizeof(T) == 2 && N > 0;
  if (embed_rows) acc((size_t)N * Kp * 2);
  const size_t part = std::max(wgrad_partial_floats(M, 2 * H + De, H, c->n_cu), wgrad_partial_floats(M, H, H, c->n_cu));
  acc(part * 4);
  acc((size_t)G * H * 4); acc((size_t)G * H * 4); acc((size_t)G * (H + Dg) * 4);
  const bool gat = m.round_kind == XRL_ROUND_GAT;
  if (gat) {                                                       // softmax weights and score gradients
    for (int i = 0; i < 2; ++i) acc((size_t)E * 4);
    for (int i = 0; i < 4; ++i) acc((size_t)N * 4);
  }
  int rc = ensure_bws(c, need);
  if (rc) return rc;
  Bump bump{c->bws};
  T *z1 = kept ? nullptr : bump.take<T>((size_t)M * H);
  T *dz1 = bump.take<T>((size_t)M * H), *dz2 = bump.take<T>((size_t)M * H);
  T *dsrc = bump.take<T>((size_t)E * H), *ddst = bump.take<T>((size_t)M * H);
  T *dhA = bump.take<T>((size_t)N * H), *dhB = bump.take<T>((size_t)N * H);
  T *dagg = bump.take<T>((size_t)N * H);
  bf16_t *xrows = embed_rows ? bump.take<bf16_t>((size_t)N * Kp) : nullptr;
  float *partial = bump.take<float>(part);
  float *rdz[3] = {bump.take<float>((size_t)G * H), bump.take<float>((size_t)G * H), nullptr};
  float *rdx = bump.take<float>((size_t)G * (H + Dg));
  float *g_ale = nullptr, *g_due = nullptr, *g_als = nullptr, *g_dus = nullptr, *g_dss = nullptr, *g_dsd = nullptr;
  if (gat) {
    g_ale = bump.take<float>((size_t)E); g_due = bump.take<float>((size_t)E);
    g_als = bump.take<float>((size_t)N); g_dus = bump.take<float>((size_t)N);
    g_dss = bump.take<float>((size_t)N); g_dsd = bump.take<float>((size_t)N);
  }

  // ---- global-update layer backward
  float *ract[3] = {c->ro_act[0], c->ro_act[1], nullptr};
  if ((rc = launch_rowmlp_bwd(c, c->L.readout, true, ract, d_demb, G, rdz, rdx))) return rc;
  if ((rc = launch_small_wgrads(c, c->L.readout, c->pool, H, d.graph_global, Dg, ract, rdz, G, dweights, partial, part))) return rc;
  // The gradient w.r.t. the last node states is the pool's, the same row for every node of a graph.
  // From the kept forward, the first backward kernel reads it through the nodes' graph ids from a
  // [G, H] table (the kernel below with the graphs as its "nodes"); otherwise it is written out per node.
  const bool dpool_table = kept && !gat;
  if (N > 0) {
    if (dpool_table)
      broadcast_dpool_kernel<T><<<dim3((unsigned)((G * (H / 4) + 255) / 256)), dim3(256), 0, c->stream>>>(
          rdx, H + Dg, nullptr, d.graph_node_ptr, m.readout == XRL_READOUT_MEAN, G, H, dhA);
    else
      broadcast_dpool_kernel<T><<<dim3((unsigned)((N * (H / 4) + 255) / 256)), dim3(256), 0, c->stream>>>(
          rdx, H + Dg, d.node_graph, d.graph_node_ptr, m.readout == XRL_READOUT_MEAN, N, H, dhA);
  }
  bool dy_by_graph = dpool_table;          // until the first backward kernel has consumed the table

  Mlp2BwdArgs a;
  memset(&a, 0, sizeof(a));
  a.De = De; a.Tn = m.n_op_types; a.Dd = m.n_node_dense;
  a.in_ptr = d.in_ptr; a.in_src = d.in_src; a.in_dst = d.in_dst;
  a.edge_feat = d.edge_feat; a.node_op = d.node_op; a.node_dense = d.node_dense;
  a.z1 = z1; a.dz1 = dz1; a.dz2 = dz2;
  WgradArgs wa;
  memset(&wa, 0, sizeof(wa));
  wa.in_ptr = d.in_ptr; wa.in_src = d.in_src; wa.in_dst = d.in_dst; wa.edge_feat = d.edge_feat;
  // (after a forward of one launch per layer the received sums of nodes without in-edges were never written)
  a.zero_row = wa.zero_row = c->zero_row;
  wa.agg_src = d.agg_src;
  if (c->agg_skip) a.agg_src = d.agg_src;
  wa.node_op = d.node_op; wa.node_dense = d.node_dense; wa.De = De; wa.Tn = m.n_op_types; wa.Dd = m.n_node_dense;
  wa.partial = partial;
  auto set_w = [&](const EncMlp &e) {
    a.W1s = e.W1s; a.W2s = e.W2s; a.W2bt = e.W2bt; a.W1bt = e.W1bt; a.b1 = e.b1; a.b2 = e.b2; a.nslab1 = e.nslab1;
  };
  auto wgrads = [&](int kind, int64_t rows, int Ka, const MlpRef &r, const void *z1_kept) -> int {
    wa.n_rows = rows; wa.Ka = Ka; wa.dZ = dz1; wa.A = nullptr;
    // both layers' weight gradients of this MLP and their reductions
    Timed t(c, kind == WG_EDGE ? TK_WGRAD_EDGE : (kind == WG_NODE ? TK_WGRAD_NODE : TK_WGRAD_EMBED));
    int rc2 = launch_wgrad<T>(c, kind, wa, dweights + r.w[0], dweights + r.b[0]);
    if (rc2) return rc2;
    wa.Ka = H; wa.dZ = dz2; wa.A = kept ? z1_kept : z1;
    return launch_wgrad<T>(c, WG_PLAIN, wa, dweights + r.w[1], dweights + r.b[1]);
  };
  // gradients through one fused MLP: from what the forward kept, else with its first layer recomputed
  Mlp2BwdzArgs za;
  memset(&za, 0, sizeof(za));
  za.in_dst = d.in_dst; za.dz1 = dz1; za.dz2 = dz2;
  za.tile_ptr = d.tile_ptr; za.n_tiles = (int64_t)b->tile_ptr.size() - 1;
  bool dz2_given = false;
  auto mlp_bwd = [&](int kind, const EncMlp &e, const uint16_t *z1mask, const uint16_t *ymask) -> int {
    if constexpr (sizeof(T) == 2) {
      if (kept) {
        za.n_rows = a.n_rows; za.W2bt = e.W2bt; za.W1bt = e.W1bt; za.dy = a.dy;
        za.z1mask = z1mask; za.ymask = ymask; za.dx_a = a.dx_a; za.dx_b = a.dx_b; za.agg_src = d.agg_src;
        za.dy_index = (dy_by_graph && kind != KIND_EDGE) ? d.node_graph : nullptr;
        dy_by_graph = false;
        const bool given = dz2_given && kind != KIND_EDGE;   // (the gather of the round above left dz2 in place)
        if (given) za.dy = dz2;
        if (kind != KIND_EDGE) dz2_given = false;
        return launch_mlp2_bwdz(c, kind, za, fold, given);
      }
    }
    return launch_mlp2_bwd<T>(c, kind, a);
  };
  constexpr int PV = 16 / sizeof(T);
  for (int r = R - 1; r >= 0 && gat; --r) {
    // attention round r+1: input h[r], saved z (in the agg slot) and scores, output h[r+1]; upstream dhA
    if (N == 0) break;
    Timed t(c, TK_GAT_BWD);
    GatBwdArgs ga;
    memset(&ga, 0, sizeof(ga));
    ga.n_rows = N; ga.z = c->agg[r + 1]; ga.hout = c->h[r + 1]; ga.dout = dhA;
    ga.s_src = c->gat_ss[r]; ga.s_dst = c->gat_sd[r];
    ga.a_src = c->d_w + c->L.gat[r].a_src; ga.a_dst = c->d_w + c->L.gat[r].a_dst;
    ga.in_ptr = d.in_ptr; ga.in_src = d.in_src; ga.in_dst = d.in_dst; ga.out_ptr = d.out_ptr; ga.out_pos = d.out_pos;
    ga.alpha_e = g_ale; ga.du_e = g_due; ga.alpha_s = g_als; ga.du_s = g_dus; ga.d_ss = g_dss; ga.d_sd = g_dsd;
    ga.dpre = dz2; ga.dz = dz1;
    const int64_t threads = N * (H / PV);
    const dim3 grid_n((unsigned)((threads + 255) / 256));
    gat_bwd_scores_kernel<T, PV><<<grid_n, dim3(256), 0, c->stream>>>(ga, H);
    gat_bwd_dz_kernel<T, PV><<<grid_n, dim3(256), 0, c->stream>>>(ga, H);
    // d a_src, d a_dst: chunk partials (at most 512 chunks: they share the weight-gradient buffer)
    int64_t nc = (N + 1023) / 1024;
    if (nc > 512) nc = 512;
    const int rpc = (int)((N + nc - 1) / nc);
    nc = (N + rpc - 1) / rpc;
    gat_avec_grad_kernel<T, PV><<<dim3((unsigned)nc), dim3(256), (size_t)(256 / (H / PV)) * 2 * H * sizeof(float), c->stream>>>(
        (const T *)c->agg[r + 1], g_dss, g_dsd, N, rpc, H, partial);
    wgrad_reduce_kernel<<<dim3((unsigned)((H + 31) / 32)), dim3(256), 0, c->stream>>>(
        partial, (int)nc, 2, 1, H, dweights + c->L.gat[r].a_src, nullptr);
    wgrad_reduce_kernel<<<dim3((unsigned)((H + 31) / 32)), dim3(256), 0, c->stream>>>(
        partial + H, (int)nc, 2, 1, H, dweights + c->L.gat[r].a_dst, nullptr);
    // dW = h^T dz (no bias row), dh = dz W^T
    wa.n_rows = N; wa.Ka = H; wa.dZ = dz1; wa.A = c->h[r];
    if ((rc = launch_wgrad<T>(c, WG_PLAIN, wa, dweights + c->L.gat[r].W, nullptr))) return rc;
    GatArgs gl;
    memset(&gl, 0, sizeof(gl));
    gl.n_rows = N; gl.n_blocks = (N + 127) / 128;
    gl.h = dz1; gl.Ws = c->gatWt[r]; gl.a_src = ga.a_src; gl.a_dst = ga.a_dst; gl.z = dhB;
    const unsigned grid_l = (unsigned)((gl.n_blocks + 7) / 8 * 8);
    switch (H) {
      case 64: gat_linear_kernel<T, 64><<<dim3(grid_l), dim3(256), 0, c->stream>>>(gl); break;
      case 128: gat_linear_kernel<T, 128><<<dim3(grid_l), dim3(256), 0, c->stream>>>(gl); break;
      default: gat_linear_kernel<T, 256><<<dim3(grid_l), dim3(256), 0, c->stream>>>(gl); break;
    }
    HIP_TRY(hipGetLastError());
    std::swap(dhA, dhB);
  }
  for (int r = R - 1; r >= 0 && !gat; --r) {
    // node MLP of round r+1: inputs h[r], agg[r+1]; output h[r+1]; upstream dhA
    set_w(c->node[r]);
    a.n_rows = N; a.h = c->h[r]; a.agg = c->agg[r + 1]; a.y = c->h[r + 1]; a.dy = dhA;
    a.dx_a = dhB; a.dx_b = dagg;
    { Timed t(c, TK_BWD_NODE); rc = mlp_bwd(KIND_NODE, c->node[r], kept ? c->zm_node[r] : nullptr, kept ? c->ym_node[r] : nullptr); }
    if (rc) return rc;
    wa.h = c->h[r]; wa.agg = c->agg[r + 1];
    if ((rc = wgrads(WG_NODE, N, 2 * H, c->L.node[r], kept ? c->z1_node[r] : nullptr))) return rc;
    // edge MLP of round r+1: upstream = dagg gathered by receiver
    set_w(c->edge[r]);
    a.n_rows = E; a.h = c->h[r]; a.agg = nullptr; a.y = nullptr; a.dy = dagg;
    a.dx_a = dsrc; a.dx_b = ddst;
    { Timed t(c, TK_BWD_EDGE); rc = mlp_bwd(KIND_EDGE, c->edge[r], kept ? c->zm_edge[r] : nullptr, kept ? c->ym_edge[r] : nullptr); }
    if (rc) return rc;
    if ((rc = wgrads(WG_EDGE, E, 2 * H + De, c->L.edge[r], kept ? c->z1_edge[r] : nullptr))) return rc;
    // dh[r] = d(node MLP)/dh + sum over in-edges of d h_receiver + sum over out-edges of d h_sender
    if (E > 0) {
      Timed t(c, TK_GRAD_GATHER);
      const int64_t threads = N * (H / PV);
      // from the kept forward: the sum leaves multiplied by the output mask of the layer that
      // produced h[r] (the node MLP of the round below, or the node-update layer), as that layer's
      // dz2 -- its backward kernel then neither reads the mask nor stores dz2
      T *masked_out = nullptr;
      const uint16_t *mask = nullptr;
      if constexpr (sizeof(T) == 2) {
        if (kept) { masked_out = dz2; mask = r > 0 ? c->ym_node[r - 1] : c->ym_embed; }
      }
      node_grad_gather_kernel<T, PV><<<dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, c->stream>>>(
          ddst, dsrc, d.in_ptr, d.out_ptr, d.out_pos, N, H, dhB, fold ? 1 : 0, masked_out, mask);
      dz2_given = masked_out != nullptr;
    }
    std::swap(dhA, dhB);
  }
  // ---- node-update layer backward (weights only: its inputs are data)
  set_w(c->embed);
  a.n_rows = N; a.h = nullptr; a.agg = nullptr; a.y = c->h[0]; a.dy = dhA; a.dx_a = nullptr; a.dx_b = nullptr;
  { Timed t(c, TK_BWD_EMBED); rc = mlp_bwd(KIND_EMBED, c->embed, kept ? c->zm_embed : nullptr, kept ? c->ym_embed : nullptr); }
  if (rc) return rc;
  if constexpr (sizeof(T) == 2) {
    // first layer: dW1 = X^T dz1 on the transpose-read kernel, X written out once; its Kx real rows
    // and the bias row (row Kp of the slices' partial tiles) are reduced separately
    Timed t(c, TK_WGRAD_EMBED);
    const int64_t threads = N * (Kp / 8);
    embed_input_rows_kernel<<<dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, c->stream>>>(
        d.edge_feat, d.in_ptr, d.node_op, d.node_dense, N, De, m.n_op_types, m.n_node_dense, Kp, xrows);
    wa.n_rows = N; wa.Ka = Kp; wa.dZ = dz1; wa.A = xrows;
    if ((rc = launch_wgrad_embed_rows<T>(c, wa, Kx, dweights + c->L.embed.w[0], dweights + c->L.embed.b[0]))) return rc;
    wa.Ka = H; wa.dZ = dz2; wa.A = kept ? c->z1_embed : z1;
    if ((rc = launch_wgrad<T>(c, WG_PLAIN, wa, dweights + c->L.embed.w[1], dweights + c->L.embed.b[1]))) return rc;
  } else {
    if ((rc = wgrads(WG_EMBED, N, Kx, c->L.embed, nullptr))) return rc;
  }
  HIP_TRY(hipGetLastError());
  return XRL_OK;
}

template <typename T>
int encode_impl(xrl_ctx *c, const xrl_batch *b, float *d_emb, int save) {
  const xrl_model_desc &m = c->m;
  const int H = m.hidden, R = m.rounds, De = m.d_edge;
  const int64_t N = b->N, E = b->E, G = b->G;
  const int64_t n_tiles = (int64_t)b->tile_ptr.size() - 1;
  // ---- workspace plan
  const int nh = save ? R + 1 : (R > 0 ? 2 : 1), nagg = save ? R : (R > 0 ? 1 : 0);
  size_t need = 0;
  auto acc = [&](size_t bytes) { need += align_up(bytes); };
  constexpr int PV = 16 / sizeof(T);
  const bool gat = m.round_kind == XRL_ROUND_GAT;
  for (int i = 0; i < nh + nagg; ++i) acc((size_t)N * H * sizeof(T));   // (GAT: the agg slot holds z)
  const xrl_batch_device &d = b->dev;
  const bool resident_ok = !gat && H * sizeof(T) <= 256 && d.graph_tile_ptr && R <= kResidentMaxRounds;
  const int64_t graph_tiles = std::max<int64_t>((b->max_graph_nodes + 31) / 32, b->max_graph_tiles);
  // blocks per graph of the one-launch encoder: one while a graph's phase is a single pass of a
  // block's four waves; otherwise as many as give every tile of a phase a wave of its own, if
  // that many are resident at once (at most one block per CU; graphs padded to a multiple of 8)
  int cluster_k = 0;
  if (resident_ok && c->resident_max_graphs > 0 && G <= c->cluster_max_graphs && G > 0 &&
      graph_tiles > c->resident_max_tiles) {
    const int64_t slots = c->n_cu / (8 * ((G + 7) / 8));
    cluster_k = (int)((graph_tiles + 3) / 4);
    if (cluster_k > slots) cluster_k = 0;   // a phase would take a second pass: the launch-per-phase path is as fast
  }
  const bool resident_batch = resident_ok && ((G <= c->resident_max_graphs && graph_tiles <= c->resident_max_tiles) ||
                                              cluster_k > 0);
  // Large bf16 batches run on kernels that can keep z1 and the ReLU masks of every fused MLP for
  // the backward pass (a row of H elements and 2 H / 32 words per node or edge and MLP): kept when
  // every launch of this encode is one of them.
  bool keep = false;
  if constexpr (sizeof(T) == 2) {
    if (save && !gat && !resident_batch && N > 0) {
      Mlp2Args t;
      memset(&t, 0, sizeof(t));
      t.De = De; t.Tn = m.n_op_types; t.Dd = m.n_node_dense;
      t.n_rows = N; t.nslabx = c->embed.nslabx;
      keep = mlp2p_applies(c, KIND_EMBED, t);
      for (int r = 0; r < R && keep; ++r) {
        t.n_rows = E; t.nslab1 = c->edge[r].nslab1;
        keep = keep && (mlp2r_applies(c, KIND_EDGE, t) || mlp2p_applies(c, KIND_EDGE, t));
        t.n_rows = N; t.nslab1 = c->node[r].nslab1;
        keep = keep && (mlp2r_applies(c, KIND_NODE, t) || mlp2p_applies(c, KIND_NODE, t));
      }
    }
  }
  const size_t ym_words = (size_t)n_tiles * (H / 32) * 64;            // 16-bit words of one edge MLP's mask bits (z1 or y)
  const size_t nm_words = (size_t)((N + 31) / 32) * (H / 32) * 64;    // ... of a node-side MLP's
  if (keep) {
    for (int i = 0; i < R + 1; ++i) acc((size_t)N * H * sizeof(T));
    for (int i = 0; i < R; ++i) { acc((size_t)E * H * sizeof(T)); acc(ym_words * 2); acc(ym_words * 2); }
    for (int i = 0; i < 2 * (R + 1); ++i) acc(nm_words * 2);
  }
  const int n_gs = gat ? (save ? R : 1) : 0;                            // saved per round for the backward
  for (int i = 0; i < 2 * n_gs; ++i) acc((size_t)N * 4);
  const size_t carry_floats = std::max(std::max(segsum_carry_floats(E, De), segsum_carry_floats(N, H)),
                                       (size_t)n_tiles * 2 * H);
  acc(carry_floats * 4);
  acc((size_t)G * H * 4);
  acc((size_t)G * H * 4);
  acc((size_t)G * H * 4);
  int rc = ensure_ws(c, need);
  if (rc) return rc;
  Bump bump{c->ws};
  c->h.assign(R + 1, nullptr);
  c->agg.assign(R + 1, nullptr);
  std::vector<T *> hb(nh), ab(std::max(nagg, 1), nullptr);
  for (int i = 0; i < nh; ++i) hb[i] = bump.take<T>((size_t)N * H);
  for (int i = 0; i < nagg; ++i) ab[i] = bump.take<T>((size_t)N * H);
  c->gat_ss.assign(R, nullptr);
  c->gat_sd.assign(R, nullptr);
  for (int i = 0; i < n_gs; ++i) {
    c->gat_ss[i] = bump.take<float>((size_t)N);
    c->gat_sd[i] = bump.take<float>((size_t)N);
  }
  c->carry = bump.take<float>(carry_floats);
  c->pool = bump.take<float>((size_t)G * H);
  c->ro_act[0] = bump.take<float>((size_t)G * H);
  c->ro_act[1] = bump.take<float>((size_t)G * H);
  c->fwd_kept = keep;
  c->z1_edge.assign(R, nullptr); c->z1_node.assign(R, nullptr);
  c->ym_edge.assign(R, nullptr); c->zm_edge.assign(R, nullptr);
  c->ym_node.assign(R, nullptr); c->zm_node.assign(R, nullptr);
  c->z1_embed = nullptr; c->ym_embed = c->zm_embed = nullptr;
  if (keep) {
    c->z1_embed = bump.take<T>((size_t)N * H);
    c->zm_embed = bump.take<uint16_t>(nm_words);
    c->ym_embed = bump.take<uint16_t>(nm_words);
    for (int r = 0; r < R; ++r) {
      c->z1_node[r] = bump.take<T>((size_t)N * H);
      c->z1_edge[r] = bump.take<T>((size_t)E * H);
      c->zm_edge[r] = bump.take<uint16_t>(ym_words);
      c->ym_edge[r] = bump.take<uint16_t>(ym_words);
      c->zm_node[r] = bump.take<uint16_t>(nm_words);
      c->ym_node[r] = bump.take<uint16_t>(nm_words);
    }
  }
  c->enc_batch = b->id;
  c->enc_saved = save != 0;

  // ---- node-update layer: the embed MLP (it sums each node's incoming edge attrs itself)
  Mlp2Args a;
  memset(&a, 0, sizeof(a));
  a.De = De; a.Tn = m.n_op_types; a.Dd = m.n_node_dense;
  a.in_ptr = d.in_ptr; a.in_src = d.in_src; a.in_dst = d.in_dst;
  a.edge_feat = d.edge_feat; a.node_op = d.node_op; a.node_dense = d.node_dense;
  a.carry = c->carry; a.tile_ptr = d.tile_ptr; a.n_tiles = n_tiles; a.zero_row = c->zero_row;
  auto set_w = [&](const EncMlp &e) {
    a.W1s = e.W1s; a.W2s = e.W2s; a.b1 = e.b1; a.b2 = e.b2; a.nslab1 = e.nslab1;
    a.W1x = e.W1x; a.nslabx = e.nslabx; a.table = e.table;
  };
  set_w(c->embed);
  a.n_rows = N; a.out = hb[0];
  a.agg0 = ab[0]; a.n_agg = gat ? 0 : nagg; a.agg_stride = nagg > 1 ? (size_t)((char *)ab[1] - (char *)ab[0]) : 0;
  if (resident_batch) {
    // small batch: the whole encoder in one launch, one block per graph (rows of at most 256
    // bytes: the three inlined tile routines of wider ones do not fit the register file)
    ResidentArgs ra;
    memset(&ra, 0, sizeof(ra));
    c->agg_skip = false;               // (the node-update layer zeroes the rows nobody else writes)
    ra.base = a;
    ra.rounds = R; ra.E = E;
    ra.graph_node_ptr = d.graph_node_ptr; ra.graph_tile_ptr = d.graph_tile_ptr; ra.gtile_ptr = d.gtile_ptr;
    ra.h[0] = hb[0];
    c->h[0] = hb[0];
    for (int r = 0; r < R; ++r) {
      ra.edge[r] = ResidentMlp{c->edge[r].W1s, c->edge[r].W2s, c->edge[r].b1, c->edge[r].b2, c->edge[r].nslab1};
      ra.node[r] = ResidentMlp{c->node[r].W1s, c->node[r].W2s, c->node[r].b1, c->node[r].b2, c->node[r].nslab1};
      ra.agg[r] = save ? ab[r] : ab[0];
      ra.h[r + 1] = save ? hb[r + 1] : hb[(r + 1) & 1];
      c->h[r + 1] = ra.h[r + 1];
      c->agg[r + 1] = ra.agg[r];
    }
    ra.mean = m.readout == XRL_READOUT_MEAN ? 1 : 0;
    ra.pool = c->pool;
    int dmax = 0;
    ra.readout = rowmlp_args(c, c->L.readout, true, c->pool, H, d.graph_global, m.d_global, G, d_emb, c->ro_act, &dmax);
    const int MB = H / 32;
    int w1 = c->embed.nslabx;
    for (int r = 0; r < R; ++r) w1 = std::max(w1, std::max(c->edge[r].nslab1, c->node[r].nslab1));
    ra.w1_bytes_max = w1 * MB * 1024;
    const size_t w2_bytes = (size_t)MB * (32 / (2 * PV)) * MB * 1024;
    const size_t lds = std::max((size_t)4 * RowStage<T, 128>::BYTES + ra.w1_bytes_max + w2_bytes + (size_t)m.n_op_types * H * 4,
                                (size_t)(256 * PV + 2 * dmax) * sizeof(float));
    ra.K = cluster_k; ra.G = (int)G; ra.arrived = c->d_arrived; ra.fault = c->d_fault; ra.spin_limit = c->cluster_spin_limit;
    if (lds <= (size_t)c->max_lds) {
      Timed t(c, TK_RESIDENT);
      const unsigned grid = cluster_k > 0 ? (unsigned)(8 * ((G + 7) / 8) * cluster_k) : (unsigned)G;
      auto launch = [&](auto kern) -> int {
        if (lds > 65536) HIP_TRY(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        kern<<<dim3(grid), dim3(256), lds, c->stream>>>(ra);
        HIP_TRY(hipGetLastError());
        return XRL_OK;
      };
      if (cluster_k > 0) {   // (grid <= number of CUs and a block fits a CU: every block is resident)
        if (H == 64) return launch(encode_cluster_kernel<T, 64>);
        if constexpr (sizeof(T) == 2) return launch(encode_cluster_kernel<T, 128>);
      } else {
        if (H == 64) return launch(encode_resident_kernel<T, 64>);
        if constexpr (sizeof(T) == 2) return launch(encode_resident_kernel<T, 128>);
      }
    }
  }
  // one launch per layer: the node MLPs (and whatever reads the received sums afterwards) take
  // zeros for nodes without in-edges through agg_src, so nobody has to write those rows
  a.n_agg = 0; a.agg_src = d.agg_src;
  c->agg_skip = !gat;
  a.z1 = c->z1_embed; a.z1mask = c->zm_embed; a.ymask = c->ym_embed;
  { Timed t(c, TK_EMBED); rc = launch_mlp2<T>(c, KIND_EMBED, a); }
  if (rc) return rc;
  c->h[0] = hb[0];
  T *hcur = hb[0];
  // ---- message-passing rounds
  for (int r = 0; r < R; ++r) {
    T *aggb = save ? ab[r] : ab[0];
    T *hnext = save ? hb[r + 1] : hb[(r + 1) & 1];
    if (gat) {                         // graph-attention reading of the round
      if (N > 0) {
        GatArgs ga;
        ga.n_rows = N; ga.n_blocks = (N + 127) / 128;
        ga.h = hcur; ga.Ws = c->gatW[r];
        ga.a_src = c->d_w + c->L.gat[r].a_src; ga.a_dst = c->d_w + c->L.gat[r].a_dst;
        ga.z = aggb; ga.s_src = c->gat_ss[save ? r : 0]; ga.s_dst = c->gat_sd[save ? r : 0];
        ga.in_ptr = d.in_ptr; ga.in_src = d.in_src; ga.out = hnext;
        { Timed t(c, TK_GAT_LINEAR);
          const unsigned grid = (unsigned)((ga.n_blocks + 7) / 8 * 8);
          switch (H) {
            case 64: gat_linear_kernel<T, 64><<<dim3(grid), dim3(256), 0, c->stream>>>(ga); break;
            case 128: gat_linear_kernel<T, 128><<<dim3(grid), dim3(256), 0, c->stream>>>(ga); break;
            default: gat_linear_kernel<T, 256><<<dim3(grid), dim3(256), 0, c->stream>>>(ga); break;
          } }
        { Timed t(c, TK_GAT_AGGREGATE);
          const int64_t threads = N * (H / PV);
          gat_aggregate_kernel<T, PV><<<dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, c->stream>>>(ga, H); }
        HIP_TRY(hipGetLastError());
      }
      c->h[r + 1] = hnext;
      c->agg[r + 1] = aggb;            // (z of this round)
      hcur = hnext;
      continue;
    }
    set_w(c->edge[r]);
    a.n_rows = E; a.h = hcur; a.out = aggb;
    a.z1 = c->z1_edge[r]; a.z1mask = c->zm_edge[r]; a.ymask = c->ym_edge[r];
    { Timed t(c, TK_EDGE); rc = launch_mlp2<T>(c, KIND_EDGE, a); }
    if (rc) return rc;
    if (b->n_split_tiles > 0) {         // only a receiver with more than 32 in-edges spans tiles
      Timed t(c, TK_EDGE_FIXUP);
      const int64_t fthreads = n_tiles * (H / 4);
      edge_tile_fixup<T><<<dim3((unsigned)((fthreads + 255) / 256)), dim3(256), 0, c->stream>>>(
          d.tile_ptr, n_tiles, d.in_ptr, d.in_dst, H, c->carry, aggb);
    }
    set_w(c->node[r]);
    a.n_rows = N; a.h = hcur; a.agg = aggb; a.out = hnext;
    a.z1 = c->z1_node[r]; a.z1mask = c->zm_node[r]; a.ymask = c->ym_node[r];
    { Timed t(c, TK_NODE); rc = launch_mlp2<T>(c, KIND_NODE, a); }
    if (rc) return rc;
    c->h[r + 1] = hnext;
    c->agg[r + 1] = aggb;
    hcur = hnext;
  }
  // ---- global-update layer: per-graph sum (or mean), then the readout MLP
  if (N <= 4096 * G) {
    // many graphs of moderate size: one block per graph sums its nodes and runs the readout MLP
    Timed t(c, TK_POOL);
    int dmax = 0;
    const RowMlpArgs ra = rowmlp_args(c, c->L.readout, true, c->pool, H, d.graph_global, m.d_global, G, d_emb,
                                      c->ro_act, &dmax);
    const size_t lds = (size_t)(256 * PV + 2 * dmax) * sizeof(float);
    graph_readout_kernel<T, PV, 8><<<dim3((unsigned)G), dim3(256), lds, c->stream>>>(
        hcur, d.graph_node_ptr, H, m.readout == XRL_READOUT_MEAN ? 1 : 0, c->pool, ra);
    HIP_TRY(hipGetLastError());
    return XRL_OK;
  }
  { Timed t(c, TK_POOL);
    rc = launch_segsum<T, float, PV>(c, hcur, nullptr, d.graph_node_ptr, d.node_graph, N, G, H, c->pool, c->carry); }
  if (rc) return rc;
  if (m.readout == XRL_READOUT_MEAN && G > 0)
    mean_scale_kernel<<<dim3((unsigned)((G * H + 255) / 256)), dim3(256), 0, c->stream>>>(c->pool, d.graph_node_ptr, G, H, 0);
  { Timed t(c, TK_READOUT);
    rc = launch_rowmlp(c, c->L.readout, true, c->pool, H, d.graph_global, m.d_global, G, d_emb, c->ro_act); }
  if (rc) return rc;
  HIP_TRY(hipGetLastError());
  return XRL_OK;
}

}  // namespace

extern "C" {

int xrl_create(const xrl_model_desc *model, const float *weights_host, void *hip_stream,
               xrl_ctx **out) {
  if (!model || !weights_host || !out) return fail(XRL_ERR_NULL, "xrl_create: NULL argument");
  *out = nullptr;
  Layout L, Lu;
  int rc = build_layout(*model, Lu);
  if (rc) return rc;
  if (model->hidden != 64 && model->hidden != 128 && model->hidden != 256)
    return fail(XRL_ERR_UNSUPPORTED, "hidden = %d: the kernels cover 64, 128 and 256", model->hidden);
  if (model->mlp_layers != 1 && model->mlp_layers != 2)
    return fail(XRL_ERR_UNSUPPORTED, "mlp_layers = %d: the kernels cover 1 and 2", model->mlp_layers);
  xrl_model_desc model_int = *model;
  model_int.mlp_layers = 2;
  if ((rc = build_layout(model_int, L))) return rc;
  const bool single_layer = model->mlp_layers == 1;
  model = &model_int;
  if (model->d_edge % 4 != 0)
    return fail(XRL_ERR_UNSUPPORTED, "d_edge = %d: the kernels need a multiple of 4", model->d_edge);
  if (model->head_hidden[0] > 512 || model->head_hidden[1] > 512 || model->d_global > 256 ||
      model->d_edge > 256 || model->n_op_types + model->n_node_dense > 1024)
    return fail(XRL_ERR_UNSUPPORTED, "head/global/edge/node attribute width beyond the kernels' range");
  int ndev = 0;
  hipError_t e = hipGetDeviceCount(&ndev);
  if (e != hipSuccess || ndev < 1) {
    (void)hipGetLastError();
    return fail(XRL_ERR_HIP, "no usable GPU: %s", e != hipSuccess ? hipGetErrorString(e) : "0 devices");
  }
  xrl_ctx *c = new (std::nothrow) xrl_ctx();
  if (!c) return fail(XRL_ERR_OOM, "xrl_create: out of host memory");
  c->m = *model;
  c->L = L;
  c->single_layer = single_layer;
  if (single_layer) c->Lu = Lu;
  c->stream = (hipStream_t)hip_stream;
  c->elem = model->precision == XRL_PREC_BF16 ? 2 : 4;
  // Row count from which the persistent kernels replace the streaming one (tuning knob; the
  // default is where they start to win; 0 = always, a huge value = never)
  c->p_min_rows = 8192;
  if (const char *e = getenv("XRL_PERSISTENT_MIN_ROWS")) c->p_min_rows = atoll(e);
  // (measured: at H = 256 the 256-column tiles win from about 300 k rows on, at H = 128 from 1 M)
  c->wide_min_rows = model->hidden >= 256 ? (1 << 18) : (1 << 20);
  if (const char *e = getenv("XRL_WGRAD_WIDE_MIN_ROWS")) c->wide_min_rows = atoll(e);
  // Batches the one-launch encoder takes: one block of four waves per graph wins while every
  // phase of a graph is a single pass of its waves (measured: 51-node graphs, 9 to 144 of them,
  // 49 us against 66 us; 340-node graphs 190 us against 122 us). 0 graphs = never.
  c->resident_max_graphs = 256;
  c->resident_max_tiles = 4;
  if (const char *e = getenv("XRL_RESIDENT_MAX_GRAPHS")) c->resident_max_graphs = atoll(e);
  if (const char *e = getenv("XRL_RESIDENT_MAX_TILES")) c->resident_max_tiles = atoll(e);
  // ... and with several blocks per graph, for the few dozen larger graphs of one rewriting step
  // (measured, one state of 14 / 31 / 51 graphs: 338-node graphs 97 / 107 / 125 us against
  // 120 / 122 / 125 us for a launch per phase; 565-node graphs 105 / 128 us against 120 / 127 us)
  c->cluster_max_graphs = 48;
  if (const char *e = getenv("XRL_CLUSTER_MAX_GRAPHS")) c->cluster_max_graphs = std::min<int64_t>(atoll(e), kClusterMaxGraphs);
  if (const char *e = getenv("XRL_CLUSTER_SPIN_LIMIT")) c->cluster_spin_limit = (unsigned)std::max<long long>(0, std::min<long long>(atoll(e), kClusterSpinLimit));
  {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) == hipSuccess) {
      c->device = dev;
      if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0) c->n_cu = v;
      if (hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) == hipSuccess && v > 0) c->max_lds = v;
    }
  }
  // the weights, followed by 1 KB of zeros (16-byte aligned) that kernels read in place of absent rows
  const size_t w_bytes = align_up(sizeof(float) * L.total);
  // zero row, heads' counters, the one-launch encoder's counters
  const size_t tail_bytes = 1024 + sizeof(int32_t) * kMaxFusedSlots + sizeof(unsigned) * kClusterMaxGraphs;
  e = hipMalloc((void **)&c->d_w, w_bytes + tail_bytes);
  if (e != hipSuccess) {
    delete c;
    return fail(XRL_ERR_OOM, "device weights: %s", hipGetErrorString(e));
  }
  c->zero_row = (char *)c->d_w + w_bytes;
  c->d_counter = (int32_t *)((char *)c->zero_row + 1024);
  c->d_arrived = (unsigned *)(c->d_counter + kMaxFusedSlots);
  e = hipMemset(c->zero_row, 0, tail_bytes);
  if (e != hipSuccess) {
    xrl_destroy(c);
    return fail(XRL_ERR_HIP, "hipMemset: %s", hipGetErrorString(e));
  }
  e = hipHostMalloc((void **)&c->h_fault, sizeof(unsigned), hipHostMallocMapped);
  if (e == hipSuccess) {
    *c->h_fault = 0;
    e = hipHostGetDevicePointer((void **)&c->d_fault, c->h_fault, 0);
  }
  if (e != hipSuccess) {
    xrl_destroy(c);
    return fail(XRL_ERR_HIP, "pinned status word: %s", hipGetErrorString(e));
  }
  rc = upload_weights(c, weights_host);
  if (!rc && c->single_layer) {
    std::vector<int32_t> wmap((size_t)c->Lu.total);
    for (const WeightTensor &t : c->Lu.tensors) {
      const int64_t n = t.cols > 0 ? t.rows * t.cols : t.rows, o = internal_offset(c, t);
      for (int64_t i = 0; i < n; ++i) wmap[(size_t)(t.offset + i)] = (int32_t)(o + i);
    }
    e = hipMalloc((void **)&c->d_dw_int, sizeof(float) * (size_t)c->L.total);
    if (e == hipSuccess) e = hipMalloc((void **)&c->d_wmap, sizeof(int32_t) * wmap.size());
    if (e == hipSuccess) e = hipMemcpy(c->d_wmap, wmap.data(), sizeof(int32_t) * wmap.size(), hipMemcpyHostToDevice);
    if (e != hipSuccess) rc = fail(XRL_ERR_OOM, "internal gradient vector: %s", hipGetErrorString(e));
  }
  if (!rc) rc = static_scratch(c->device, &c->static_ws);
  if (rc) {
    xrl_destroy(c);
    return rc;
  }
  *out = c;
  return XRL_OK;
}

int xrl_set_weights(xrl_ctx *c, const float *weights_host) {
  if (!c || !weights_host) return fail(XRL_ERR_NULL, "xrl_set_weights: NULL argument");
  return upload_weights(c, weights_host);
}

int xrl_destroy(xrl_ctx *c) {
  if (!c) return XRL_OK;
  (void)hipStreamSynchronize(c->stream);
  if (c->d_w) (void)hipFree(c->d_w);
  if (c->h_fault) (void)hipHostFree(c->h_fault);
  if (c->d_dw_int) (void)hipFree(c->d_dw_int);
  if (c->d_wmap) (void)hipFree(c->d_wmap);
  if (c->d_swz) (void)hipFree(c->d_swz);
  if (c->ws) (void)hipFree(c->ws);
  if (c->hws) (void)hipFree(c->hws);
  if (c->bws) (void)hipFree(c->bws);
  for (auto &sp : c->spans) { (void)hipEventDestroy(sp.a); (void)hipEventDestroy(sp.b); }
  for (auto &e : c->free_events) (void)hipEventDestroy(e);
  delete c;
  return XRL_OK;
}

namespace {
// out[i, :] = from[i] >= 0 ? base[from[i], :] : added[-1 - from[i], :], rows of `width` 4-byte words:
// the per-node and per-edge attribute arrays of a batch packed from edits, filled on the device
// from the current graphs' attributes and the new items'.
__global__ void expand_rows_kernel(const int32_t *from, int64_t n, int width, const uint32_t *base, const uint32_t *added,
                                   uint32_t *out) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n * width) return;
  const int64_t r = i / width;
  const int j = (int)(i - r * width);
  const int32_t f = from[r];
  out[i] = f >= 0 ? base[(size_t)f * width + j] : added[(size_t)(-1 - f) * width + j];
}
// agg_src of a batch: n for a node with in-edges, -1 for one without
__global__ void agg_src_kernel(const int32_t *in_ptr, int64_t n, int32_t *agg_src) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) agg_src[i] = in_ptr[i + 1] > in_ptr[i] ? (int32_t)i : -1;
}
}  // namespace

int xrl_batch_upload(xrl_ctx *c, xrl_batch *b) {
  if (!c || !b) return fail(XRL_ERR_NULL, "xrl_batch_upload: NULL argument");
  if (b->uploaded) return XRL_OK;
  const int Dd = b->model.n_node_dense, De = b->model.d_edge, Dg = b->model.d_global;
  const int64_t S = b->S, G = b->G, N = b->N, E = b->E;
  size_t off = 0;
  auto plan = [&](size_t bytes) { size_t o = off; off += align_up(bytes + 16); return o; };
  const size_t o_sgp = plan((S + 1) * 4), o_gnp = plan((G + 1) * 4), o_op = plan(N * 4),
               o_inp = plan((N + 1) * 4), o_ins = plan(E * 4), o_ind = plan(E * 4),
               o_outp = plan((N + 1) * 4), o_outpos = plan(E * 4), o_ng = plan(N * 4),
               o_nd = plan((size_t)N * Dd * 4), o_ef = plan((size_t)E * De * 4),
               o_gg = plan((size_t)G * Dg * 4), o_mask = plan(G),
               o_tile = plan(b->tile_ptr.size() * 4), o_gtile = plan(b->gtile_ptr.size() * 4),
               o_gtp = plan(b->graph_tile_ptr.size() * 4), o_as = plan(N * 4);
  // packed from edits: the attribute arrays are filled on the device from these
  const bool ed = b->from_edits;
  const size_t o_nf = ed ? plan(N * 4) : 0, o_ef2 = ed ? plan(E * 4) : 0,
               o_bop = ed ? plan(b->base_node_op.size() * 4) : 0, o_nop = ed ? plan(b->new_node_op.size() * 4) : 0,
               o_bnd = ed ? plan(b->base_node_dense.size() * 4) : 0, o_nnd = ed ? plan(b->new_node_dense.size() * 4) : 0,
               o_bef = ed ? plan(b->base_edge_feat.size() * 4) : 0, o_nef = ed ? plan(b->new_edge_feat.size() * 4) : 0;
  char *blk = nullptr;
  hipError_t e = hipMalloc((void **)&blk, off);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return fail(XRL_ERR_OOM, "device copy of the batch (%zu bytes): %s", off, hipGetErrorString(e));
  }
  xrl_batch_device &d = b->dev;
  d.block = blk;
  d.bytes = off;
  // the host vectors live as long as the batch; wait for the copies anyway so that freeing the
  // batch right after this call is safe
  auto cp = [&](size_t o, const void *src, size_t bytes) -> hipError_t {
    return bytes ? hipMemcpyAsync(blk + o, src, bytes, hipMemcpyHostToDevice, c->stream) : hipSuccess;
  };
  HIP_TRY(cp(o_sgp, b->state_graph_ptr.data(), (S + 1) * 4));
  HIP_TRY(cp(o_gnp, b->graph_node_ptr.data(), (G + 1) * 4));
  if (!ed) HIP_TRY(cp(o_op, b->node_op.data(), N * 4));
  HIP_TRY(cp(o_inp, b->in_ptr.data(), (N + 1) * 4));
  if (N > 0) {
    agg_src_kernel<<<dim3((unsigned)((N + 255) / 256)), dim3(256), 0, c->stream>>>((const int32_t *)(blk + o_inp), N,
                                                                                  (int32_t *)(blk + o_as));
    HIP_TRY(hipGetLastError());
  }
  HIP_TRY(cp(o_ins, b->in_src.data(), E * 4));
  HIP_TRY(cp(o_ind, b->in_dst.data(), E * 4));
  HIP_TRY(cp(o_outp, b->out_ptr.data(), (N + 1) * 4));
  HIP_TRY(cp(o_outpos, b->out_pos.data(), E * 4));
  HIP_TRY(cp(o_ng, b->node_graph.data(), N * 4));
  if (!ed) {
    HIP_TRY(cp(o_nd, b->node_dense.data(), (size_t)N * Dd * 4));
    HIP_TRY(cp(o_ef, b->edge_feat.data(), (size_t)E * De * 4));
  } else {
    HIP_TRY(cp(o_nf, b->node_from.data(), N * 4));
    HIP_TRY(cp(o_ef2, b->edge_from.data(), E * 4));
    HIP_TRY(cp(o_bop, b->base_node_op.data(), b->base_node_op.size() * 4));
    HIP_TRY(cp(o_nop, b->new_node_op.data(), b->new_node_op.size() * 4));
    HIP_TRY(cp(o_bnd, b->base_node_dense.data(), b->base_node_dense.size() * 4));
    HIP_TRY(cp(o_nnd, b->new_node_dense.data(), b->new_node_dense.size() * 4));
    HIP_TRY(cp(o_bef, b->base_edge_feat.data(), b->base_edge_feat.size() * 4));
    HIP_TRY(cp(o_nef, b->new_edge_feat.data(), b->new_edge_feat.size() * 4));
    auto expand = [&](size_t o_from, int64_t n, int width, size_t o_base, size_t o_new, size_t o_out) {
      const int64_t total = n * width;
      if (total > 0)
        expand_rows_kernel<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, c->stream>>>(
            (const int32_t *)(blk + o_from), n, width, (const uint32_t *)(blk + o_base), (const uint32_t *)(blk + o_new),
            (uint32_t *)(blk + o_out));
    };
    expand(o_nf, N, 1, o_bop, o_nop, o_op);
    expand(o_nf, N, Dd, o_bnd, o_nnd, o_nd);
    expand(o_ef2, E, De, o_bef, o_nef, o_ef);
    HIP_TRY(hipGetLastError());
  }
  HIP_TRY(cp(o_gg, b->graph_global.data(), (size_t)G * Dg * 4));
  HIP_TRY(cp(o_mask, b->mask.data(), G));
  HIP_TRY(cp(o_tile, b->tile_ptr.data(), b->tile_ptr.size() * 4));
  HIP_TRY(cp(o_gtile, b->gtile_ptr.data(), b->gtile_ptr.size() * 4));
  HIP_TRY(cp(o_gtp, b->graph_tile_ptr.data(), b->graph_tile_ptr.size() * 4));
  HIP_TRY(hipStreamSynchronize(c->stream));
  d.state_graph_ptr = (int32_t *)(blk + o_sgp);
  d.graph_node_ptr = (int32_t *)(blk + o_gnp);
  d.node_op = (int32_t *)(blk + o_op);
  d.in_ptr = (int32_t *)(blk + o_inp);
  d.in_src = (int32_t *)(blk + o_ins);
  d.in_dst = (int32_t *)(blk + o_ind);
  d.out_ptr = (int32_t *)(blk + o_outp);
  d.out_pos = (int32_t *)(blk + o_outpos);
  d.node_graph = (int32_t *)(blk + o_ng);
  d.node_dense = (float *)(blk + o_nd);
  d.edge_feat = (float *)(blk + o_ef);
  d.graph_global = (float *)(blk + o_gg);
  d.mask = (uint8_t *)(blk + o_mask);
  d.tile_ptr = (int32_t *)(blk + o_tile);
  d.gtile_ptr = b->graph_tile_ptr.empty() ? nullptr : (int32_t *)(blk + o_gtile);
  d.graph_tile_ptr = b->graph_tile_ptr.empty() ? nullptr : (int32_t *)(blk + o_gtp);
  d.agg_src = (int32_t *)(blk + o_as);
  b->uploaded = true;
  return XRL_OK;
}

int xrl_encode(xrl_ctx *c, const xrl_batch *b, float *d_emb, int save_for_backward) {
  int rc = check_batch(c, b, "xrl_encode");
  if (rc) return rc;
  if (!d_emb && b->G > 0) return fail(XRL_ERR_NULL, "xrl_encode: d_emb is NULL");
  if (b->G == 0) return XRL_OK;
  if (*(volatile unsigned *)c->h_fault) {
    // an earlier one-launch encode gave up a wait between its blocks: its embeddings were wrong.
    // Its counters are put back to zero (after everything queued so far) before anything else runs.
    (void)hipStreamSynchronize(c->stream);
    (void)hipMemsetAsync(c->d_arrived, 0, sizeof(unsigned) * kClusterMaxGraphs, c->stream);
    *c->h_fault = 0;
    return fail(XRL_ERR_HIP, "xrl_encode: an earlier xrl_encode on this context did not complete (a wait between the "
                             "blocks of its one-launch form ran out); its embeddings are invalid");
  }
  return c->elem == 2 ? encode_impl<bf16_t>(c, b, d_emb, save_for_backward)
                      : encode_impl<float>(c, b, d_emb, save_for_backward);
}

int xrl_policy_value(xrl_ctx *c, const xrl_batch *b, const float *d_emb, float *d_logp,
                     float *d_value, float *d_entropy, int32_t *d_action, float *d_logit) {
  int rc = check_batch(c, b, "xrl_policy_value");
  if (rc) return rc;
  if (b->S == 0) return XRL_OK;
  if (!d_emb || !d_logp || !d_value || !d_entropy || !d_action)
    return fail(XRL_ERR_NULL, "xrl_policy_value: NULL device pointer");
  if ((uintptr_t)d_emb & 15) return fail(XRL_ERR_SHAPE, "xrl_policy_value: d_emb must be 16-byte aligned");
  const int H = c->m.hidden;
  rc = ensure_hws(c, align_up((size_t)b->G * 4) + align_up((size_t)b->S * H * 4));
  if (rc) return rc;
  float *logit = d_logit ? d_logit : (float *)c->hws;
  float *zmean = (float *)(c->hws + align_up((size_t)b->G * 4));
  Timed t(c, TK_HEADS);
  return launch_heads(c, b, d_emb, logit, d_logp, d_entropy, d_action, zmean, d_value, nullptr, nullptr);
}

int xrl_policy_value_static(xrl_ctx *c, const xrl_batch *b, const float *d_emb, float *d_logp,
                            float *d_value, float *d_entropy, int32_t *d_action, float *d_logit) {
  int rc = check_batch(c, b, "xrl_policy_value_static");
  if (rc) return rc;
  if (b->S == 0) return XRL_OK;
  if (!d_emb || !d_logp || !d_value || !d_entropy || !d_action)
    return fail(XRL_ERR_NULL, "xrl_policy_value_static: NULL device pointer");
  if ((uintptr_t)d_emb & 15) return fail(XRL_ERR_SHAPE, "xrl_policy_value_static: d_emb must be 16-byte aligned");
  const int H = c->m.hidden;
  if (b->G > kStaticMaxSlots || b->S * H > kStaticMaxStateFloats)
    return fail(XRL_ERR_UNSUPPORTED,
                "xrl_policy_value_static: %lld slots, %lld states x hidden %d exceed the fixed scratch "
                "(at most %lld slots and %lld state floats)",
                (long long)b->G, (long long)b->S, H, (long long)kStaticMaxSlots, (long long)kStaticMaxStateFloats);
  int32_t *counter = (int32_t *)(c->static_ws + kStaticCounterOff);
  float *logit = d_logit ? d_logit : (float *)(c->static_ws + kStaticLogitOff);
  float *zmean = (float *)(c->static_ws + kStaticZmeanOff);
  // the array keeps the last call's contents: the counters must start at zero
  fill_zero_kernel<<<dim3((unsigned)((b->S + 255) / 256)), dim3(256), 0, c->stream>>>((float *)counter, b->S);
  const RowMlpArgs va = rowmlp_args(c, c->L.value, false, zmean, H, nullptr, 0, b->S, d_value, nullptr);
  const RowMlpArgs pa = rowmlp_args(c, c->L.policy, false, d_emb, H, nullptr, 0, b->G, logit, nullptr);
  policy_value_kernel<<<dim3((unsigned)(b->G + b->S)), dim3(256), 0, c->stream>>>(
      pa, b->dev.mask, b->dev.state_graph_ptr, (int)b->G, (int)b->S, H, counter, d_logp, d_entropy, d_action, zmean, va);
  HIP_TRY(hipGetLastError());
  return XRL_OK;
}

int xrl_ppo_objective(xrl_ctx *c, const xrl_batch *b, const float *d_logp, const float *d_value,
                      const float *d_entropy, const int32_t *d_action, const float *d_old_logp,
                      const float *d_advantage, const float *d_v_target, float eps, float c1,
                      float c2, float *d_J, float *d_dlogp, float *d_dvalue, float *d_dentropy) {
  int rc = check_batch(c, b, "xrl_ppo_objective");
  if (rc) return rc;
  if (!d_J) return fail(XRL_ERR_NULL, "xrl_ppo_objective: d_J is NULL");
  if (b->S > 0 && (!d_logp || !d_value || !d_entropy || !d_action || !d_old_logp || !d_advantage ||
                   !d_v_target || !d_dlogp || !d_dvalue || !d_dentropy))
    return fail(XRL_ERR_NULL, "xrl_ppo_objective: NULL device pointer");
  if (b->G > 0)
    fill_zero_kernel<<<dim3((unsigned)((b->G + 255) / 256)), dim3(256), 0, c->stream>>>(d_dlogp, b->G);
  ppo_objective_kernel<<<dim3(1), dim3(256), 0, c->stream>>>(
      d_logp, d_value, d_entropy, b->dev.state_graph_ptr, b->dev.mask, d_action, d_old_logp, d_advantage, d_v_target,
      (int)b->S, eps, c1, c2, d_J, d_dlogp, d_dvalue, d_dentropy);
  HIP_TRY(hipGetLastError());
  return XRL_OK;
}

}  // extern "C"

namespace {
// user[i] += internal[map[i]]: the real tensors of a single-layer context's internal gradient vector,
// added to the caller's
__global__ void add_mapped_kernel(float *user, const float *internal, const int32_t *map, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) user[i] += internal[map[i]];
}

// Runs a backward pass that adds weight gradients into a vector of the context's own layout: the
// caller's vector itself, or (single-layer contexts) the internal one, zeroed first and folded
// into the caller's afterwards.
template <typename Run>
int with_weight_gradients(xrl_ctx *c, float *d_dweights, Run run) {
  if (!c->single_layer) return run(d_dweights);
  const int64_t n = c->L.total, nu = c->Lu.total;
  fill_zero_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, c->stream>>>(c->d_dw_int, n);
  HIP_TRY(hipGetLastError());
  const int rc = run(c->d_dw_int);
  if (rc) return rc;
  add_mapped_kernel<<<dim3((unsigned)((nu + 255) / 256)), dim3(256), 0, c->stream>>>(d_dweights, c->d_dw_int, c->d_wmap, nu);
  HIP_TRY(hipGetLastError());
  return XRL_OK;
}

int policy_value_backward_run(xrl_ctx *c, const xrl_batch *b, const float *d_emb, const float *d_dlogp,
                              const float *d_dvalue, const float *d_dentropy, float *d_demb, float *d_dweights);
}  // namespace

extern "C" {

int xrl_policy_value_backward(xrl_ctx *c, const xrl_batch *b, const float *d_emb,
                              const float *d_dlogp, const float *d_dvalue,
                              const float *d_dentropy, float *d_demb, float *d_dweights) {
  int rc = check_batch(c, b, "xrl_policy_value_backward");
  if (rc) return rc;
  if (b->S == 0) return XRL_OK;
  if (!d_emb || !d_dlogp || !d_dvalue || !d_dentropy || !d_demb || !d_dweights)
    return fail(XRL_ERR_NULL, "xrl_policy_value_backward: NULL device pointer");
  return with_weight_gradients(c, d_dweights, [&](float *dw) {
    return policy_value_backward_run(c, b, d_emb, d_dlogp, d_dvalue, d_dentropy, d_demb, dw);
  });
}

}  // extern "C"

namespace {
int policy_value_backward_run(xrl_ctx *c, const xrl_batch *b, const float *d_emb, const float *d_dlogp,
                              const float *d_dvalue, const float *d_dentropy, float *d_demb, float *d_dweights) {
  int rc = XRL_OK;
  if ((uintptr_t)d_emb & 15)
    return fail(XRL_ERR_SHAPE, "xrl_policy_value_backward: d_emb must be 16-byte aligned");
  const int H = c->m.hidden, h0 = c->m.head_hidden[0], h1 = c->m.head_hidden[1];
  const int64_t G = b->G, S = b->S;
  size_t need = 0;
  auto acc = [&](size_t n) { need += align_up(n * 4); };
  acc(G); acc(G); acc(S); acc(S * H); acc(S); acc(S);                 // logit logp ent zmean action value
  acc(G * h0); acc(G * h1); acc(G);                                   // policy activations
  acc(S * h0); acc(S * h1); acc(S);                                   // value activations
  acc(G); acc(S);                                                     // dlogit, 1/|valid|
  acc(G * h0); acc(G * h1); acc(G);                                   // policy dz
  acc(S * h0); acc(S * h1); acc(S); acc(S * H);                       // value dz, dz_mean
  const size_t spart_floats = std::max(small_wgrad_partial_floats(c->L.policy, G), small_wgrad_partial_floats(c->L.value, S));
  acc(spart_floats);                                                  // chunk partials of the heads' weight gradients
  if ((rc = ensure_hws(c, need))) return rc;
  Bump bump{c->hws};
  float *logit = bump.take<float>(G), *logp = bump.take<float>(G), *ent = bump.take<float>(S);
  float *zmean = bump.take<float>(S * H);
  int32_t *action = bump.take<int32_t>(S);
  float *value = bump.take<float>(S);
  float *pact[3] = {bump.take<float>(G * h0), bump.take<float>(G * h1), bump.take<float>(G)};
  float *vact[3] = {bump.take<float>(S * h0), bump.take<float>(S * h1), bump.take<float>(S)};
  float *dlogit = bump.take<float>(G), *inv_n = bump.take<float>(S);
  float *pdz[3] = {bump.take<float>(G * h0), bump.take<float>(G * h1), bump.take<float>(G)};
  float *vdz[3] = {bump.take<float>(S * h0), bump.take<float>(S * h1), bump.take<float>(S)};
  float *dzs = bump.take<float>(S * H);
  float *spart = spart_floats ? bump.take<float>(spart_floats) : nullptr;
  const xrl_batch_device &d = b->dev;
  // forward of the heads, keeping every layer's output
  if ((rc = launch_heads(c, b, d_emb, logit, logp, ent, action, zmean, value, pact, vact))) return rc;
  // backward
  state_policy_bwd_kernel<<<dim3((unsigned)S), dim3(256), 0, c->stream>>>(logp, ent, d.mask, d.state_graph_ptr,
                                                                        d_dlogp, d_dentropy, dlogit, inv_n);
  if ((rc = launch_rowmlp_bwd(c, c->L.policy, false, pact, dlogit, G, pdz, d_demb))) return rc;
  if ((rc = launch_rowmlp_bwd(c, c->L.value, false, vact, d_dvalue, S, vdz, dzs))) return rc;
  demb_combine_kernel<<<dim3((unsigned)G), dim3(H < 256 ? H : 256), 0, c->stream>>>(d_demb, dzs, inv_n, d.mask,
                                                                                 d.state_graph_ptr, (int)S, H);
  if ((rc = launch_small_wgrads(c, c->L.policy, d_emb, H, nullptr, 0, pact, pdz, G, d_dweights, spart, spart_floats))) return rc;
  if ((rc = launch_small_wgrads(c, c->L.value, zmean, H, nullptr, 0, vact, vdz, S, d_dweights, spart, spart_floats))) return rc;
  HIP_TRY(hipGetLastError());
  return XRL_OK;
}
}  // namespace

extern "C" {

int xrl_encode_backward(xrl_ctx *c, const xrl_batch *b, const float *d_demb, float *d_dweights) {
  int rc = check_batch(c, b, "xrl_encode_backward");
  if (rc) return rc;
  if (b->G == 0) return XRL_OK;
  if (!d_demb || !d_dweights) return fail(XRL_ERR_NULL, "xrl_encode_backward: NULL device pointer");
  if (!c->enc_saved || c->enc_batch != b->id)
    return fail(XRL_ERR_STATE, "xrl_encode_backward: the batch's last xrl_encode did not save for backward");
  return with_weight_gradients(c, d_dweights, [&](float *dw) {
    return c->elem == 2 ? encode_backward_impl<bf16_t>(c, b, d_demb, dw) : encode_backward_impl<float>(c, b, d_demb, dw);
  });
}

int xrl_set_timing(xrl_ctx *c, int enabled) {
  if (!c) return fail(XRL_ERR_NULL, "xrl_set_timing: ctx is NULL");
  c->timing = enabled != 0;
  return XRL_OK;
}

int xrl_read_timing(xrl_ctx *c, const char *kernel, double *total_ms, int64_t *launches) {
  if (!c || !kernel || !total_ms || !launches) return fail(XRL_ERR_NULL, "xrl_read_timing: NULL argument");
  int kind = -1;
  for (int k = 0; k < TK_COUNT; ++k)
    if (!strcmp(kernel, kTimedNames[k])) kind = k;
  if (kind < 0) return fail(XRL_ERR_INDEX, "xrl_read_timing: unknown kernel '%s'", kernel);
  HIP_TRY(hipStreamSynchronize(c->stream));
  double tot = 0.0;
  int64_t n = 0;
  std::vector<xrl_ctx::Span> keep;
  for (const auto &sp : c->spans) {
    if (sp.kind != kind) { keep.push_back(sp); continue; }
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, sp.a, sp.b));
    tot += ms;
    ++n;
    c->free_events.push_back(sp.a);
    c->free_events.push_back(sp.b);
  }
  c->spans.swap(keep);
  *total_ms = tot;
  *launches = n;
  return XRL_OK;
}

namespace {
// 4 independent accumulator tiles per wave, operands never change: nothing but the matrix pipe
__global__ __launch_bounds__(256) void mfma_peak_kernel(float *out, int iters) {
  bf16x8 a = Operand<bf16_t>::zero(), b = Operand<bf16_t>::zero();
  a[threadIdx.x & 7] = (bf16_t)1.0f;
  b[(threadIdx.x >> 3) & 7] = (bf16_t)0.5f;
  f32x16 acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[i][r];
  out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}
__global__ __launch_bounds__(256) void copy_peak_kernel(const f32x4 *src, f32x4 *dst, int64_t n) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}
}  // namespace

int xrl_measure_peaks(xrl_ctx *c, int64_t copy_bytes, double *mfma_tflops, double *copy_gbs) {
  if (!c || !mfma_tflops || !copy_gbs) return fail(XRL_ERR_NULL, "xrl_measure_peaks: NULL argument");
  if (copy_bytes < 16) return fail(XRL_ERR_SHAPE, "xrl_measure_peaks: copy_bytes = %lld", (long long)copy_bytes);
  const int64_t n16 = copy_bytes / 16;
  const int blocks = c->n_cu * 4;                              // 16 waves per CU
  char *buf = nullptr;
  hipError_t e = hipMalloc((void **)&buf, (size_t)n16 * 32 + (size_t)blocks * 256 * 4);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return fail(XRL_ERR_OOM, "xrl_measure_peaks: %s", hipGetErrorString(e));
  }
  f32x4 *src = (f32x4 *)buf, *dst = src + n16;
  float *out = (float *)(dst + n16);
  hipEvent_t e0 = nullptr, e1 = nullptr;
  int rc = XRL_OK;
  auto run = [&]() -> int {
    HIP_TRY(hipEventCreate(&e0));
    HIP_TRY(hipEventCreate(&e1));
    HIP_TRY(hipMemsetAsync(buf, 0, (size_t)n16 * 32, c->stream));
    const int iters = 20000;
    mfma_peak_kernel<<<dim3(blocks), dim3(256), 0, c->stream>>>(out, 100);          // warm-up
    HIP_TRY(hipEventRecord(e0, c->stream));
    mfma_peak_kernel<<<dim3(blocks), dim3(256), 0, c->stream>>>(out, iters);
    HIP_TRY(hipEventRecord(e1, c->stream));
    HIP_TRY(hipEventSynchronize(e1));
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, e0, e1));
    *mfma_tflops = (double)blocks * 4 * iters * 4 * (2.0 * 32 * 32 * 16) / (ms * 1e-3) / 1e12;
    copy_peak_kernel<<<dim3(c->n_cu * 8), dim3(256), 0, c->stream>>>(src, dst, n16);   // warm-up
    HIP_TRY(hipEventRecord(e0, c->stream));
    for (int i = 0; i < 5; ++i) copy_peak_kernel<<<dim3(c->n_cu * 8), dim3(256), 0, c->stream>>>(src, dst, n16);
    HIP_TRY(hipEventRecord(e1, c->stream));
    HIP_TRY(hipEventSynchronize(e1));
    HIP_TRY(hipEventElapsedTime(&ms, e0, e1));
    *copy_gbs = 5.0 * (double)n16 * 32 / (ms * 1e-3) / 1e9;
    return XRL_OK;
  };
  rc = run();
  (void)hipStreamSynchronize(c->stream);
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  (void)hipFree(buf);
  return rc;
}

int xrl_segment_sum(xrl_ctx *c, const float *d_values, const int32_t *d_ptr, int64_t n_rows,
                    int64_t n_seg, int32_t width, float *d_out) {
  if (!c || !d_ptr || !d_out || (n_rows > 0 && !d_values))
    return fail(XRL_ERR_NULL, "xrl_segment_sum: NULL argument");
  if (n_rows < 0 || n_seg < 0 || width < 4 || width > 256 || width % 4)
    return fail(XRL_ERR_SHAPE, "xrl_segment_sum: n_rows/n_seg negative or width not a multiple of 4 in [4, 256]");
  int rc = ensure_ws(c, align_up(segsum_carry_floats(n_rows, width) * 4));
  if (rc) return rc;
  c->enc_batch = 0;   // the workspace no longer holds an encode's activations
  c->enc_saved = false;
  return launch_segsum<float, float, 4>(c, d_values, nullptr, d_ptr, nullptr, n_rows, n_seg, width, d_out,
                                        (float *)c->ws);
}

int xrl_weight_gradient(xrl_ctx *c, const xrl_batch *b, int32_t kind, const void *d_x, const void *d_x2,
                        const void *d_dZ, int64_t n_rows, float *d_dW, float *d_db) {
  int rc = check_batch(c, b, "xrl_weight_gradient");
  if (rc) return rc;
  if (kind != XRL_WG_PLAIN && kind != XRL_WG_EDGE && kind != XRL_WG_NODE)
    return fail(XRL_ERR_INDEX, "xrl_weight_gradient: unknown kind %d", kind);
  const int H = c->m.hidden, De = c->m.d_edge;
  if (kind == XRL_WG_EDGE) n_rows = b->E;
  if (kind == XRL_WG_NODE) n_rows = b->N;
  if (n_rows < 0) return fail(XRL_ERR_SHAPE, "xrl_weight_gradient: n_rows is negative");
  if (n_rows == 0) return XRL_OK;
  if (!d_x || !d_dZ || !d_dW || !d_db || (kind == XRL_WG_NODE && !d_x2))
    return fail(XRL_ERR_NULL, "xrl_weight_gradient: NULL device pointer");
  const int Ka = kind == XRL_WG_PLAIN ? H : (kind == XRL_WG_EDGE ? 2 * H + De : 2 * H);
  const size_t part = wgrad_partial_floats(n_rows, Ka, H, c->n_cu);
  if ((rc = ensure_bws(c, align_up(part * 4)))) return rc;
  WgradArgs wa;
  memset(&wa, 0, sizeof(wa));
  const xrl_batch_device &d = b->dev;
  wa.in_ptr = d.in_ptr; wa.in_src = d.in_src; wa.in_dst = d.in_dst; wa.edge_feat = d.edge_feat;
  wa.agg_src = d.agg_src; wa.zero_row = c->zero_row;
  wa.node_op = d.node_op; wa.node_dense = d.node_dense; wa.De = De; wa.Tn = c->m.n_op_types; wa.Dd = c->m.n_node_dense;
  wa.partial = (float *)c->bws;
  wa.n_rows = n_rows; wa.Ka = Ka; wa.dZ = d_dZ;
  if (kind == XRL_WG_PLAIN) wa.A = d_x;
  else { wa.h = d_x; wa.agg = d_x2; }
  const int wk = kind == XRL_WG_PLAIN ? WG_PLAIN : (kind == XRL_WG_EDGE ? WG_EDGE : WG_NODE);
  Timed t(c, TK_WGRAD);
  return c->elem == 2 ? launch_wgrad<bf16_t>(c, wk, wa, d_dW, d_db) : launch_wgrad<float>(c, wk, wa, d_dW, d_db);
}

int xrl_mlp_backward(xrl_ctx *c, const xrl_batch *b, int32_t kind, int32_t round, const void *d_h,
                     const void *d_agg, const void *d_y, const void *d_dy, void *d_z1, void *d_dz1,
                     void *d_dz2, void *d_dxa, void *d_dxb) {
  int rc = check_batch(c, b, "xrl_mlp_backward");
  if (rc) return rc;
  if (c->m.round_kind != XRL_ROUND_MLP) return fail(XRL_ERR_UNSUPPORTED, "xrl_mlp_backward: MLP rounds only");
  if (kind != XRL_WG_EDGE && kind != XRL_WG_NODE) return fail(XRL_ERR_INDEX, "xrl_mlp_backward: unknown kind %d", kind);
  if (round < 0 || round >= c->m.rounds) return fail(XRL_ERR_INDEX, "xrl_mlp_backward: round %d outside [0, %d)", round, c->m.rounds);
  const int64_t rows = kind == XRL_WG_EDGE ? b->E : b->N;
  if (rows == 0) return XRL_OK;
  if (!d_h || !d_dy || !d_z1 || !d_dz1 || !d_dz2 || !d_dxa || !d_dxb || (kind == XRL_WG_NODE && (!d_agg || !d_y)))
    return fail(XRL_ERR_NULL, "xrl_mlp_backward: NULL device pointer");
  const xrl_batch_device &d = b->dev;
  Mlp2BwdArgs a;
  memset(&a, 0, sizeof(a));
  a.De = c->m.d_edge; a.Tn = c->m.n_op_types; a.Dd = c->m.n_node_dense;
  a.in_ptr = d.in_ptr; a.in_src = d.in_src; a.in_dst = d.in_dst;
  a.edge_feat = d.edge_feat; a.node_op = d.node_op; a.node_dense = d.node_dense;
  const EncMlp &e = kind == XRL_WG_EDGE ? c->edge[round] : c->node[round];
  a.W1s = e.W1s; a.W2s = e.W2s; a.W2bt = e.W2bt; a.W1bt = e.W1bt; a.b1 = e.b1; a.b2 = e.b2; a.nslab1 = e.nslab1;
  a.n_rows = rows; a.h = d_h; a.agg = d_agg; a.y = d_y; a.dy = d_dy;
  a.z1 = d_z1; a.dz1 = d_dz1; a.dz2 = d_dz2; a.dx_a = d_dxa; a.dx_b = d_dxb;
  const int k = kind == XRL_WG_EDGE ? KIND_EDGE : KIND_NODE;
  return c->elem == 2 ? launch_mlp2_bwd<bf16_t>(c, k, a) : launch_mlp2_bwd<float>(c, k, a);
}

int xrl_get_activation(xrl_ctx *c, const xrl_batch *b, const char *what, int32_t round, float *d_out) {
  int rc = check_batch(c, b, "xrl_get_activation");
  if (rc) return rc;
  if (!what || !d_out) return fail(XRL_ERR_NULL, "xrl_get_activation: NULL argument");
  if (!c->enc_saved || c->enc_batch != b->id)
    return fail(XRL_ERR_STATE, "xrl_get_activation: no saved forward of this batch");
  const int H = c->m.hidden, R = c->m.rounds;
  const int64_t N = b->N, G = b->G;
  const void *src = nullptr;
  int64_t rows = N;
  int D = H;
  bool typed = true;
  const int32_t *row_src = nullptr;
  if (!strcmp(what, "a0")) {   // not kept by the forward pass: recomputed with the segment-sum kernel
    return launch_segsum<float, float, 4>(c, b->dev.edge_feat, nullptr, b->dev.in_ptr, b->dev.in_dst, b->E, N,
                                          c->m.d_edge, d_out, c->carry);
  }
  else if (!strcmp(what, "pool")) { src = c->pool; rows = G; typed = false; }
  else if (!strcmp(what, "h")) {
    if (round < 0 || round > R) return fail(XRL_ERR_INDEX, "h: round %d outside [0, %d]", round, R);
    src = c->h[round];
  } else if (!strcmp(what, "agg")) {
    if (round < 1 || round > R) return fail(XRL_ERR_INDEX, "agg: round %d outside [1, %d]", round, R);
    if (c->m.round_kind == XRL_ROUND_GAT)
      return fail(XRL_ERR_UNSUPPORTED, "agg: the graph-attention rounds keep no received sums");
    src = c->agg[round];
    if (c->agg_skip) row_src = b->dev.agg_src;   // rows of nodes without in-edges were never written
  } else return fail(XRL_ERR_INDEX, "xrl_get_activation: unknown tensor '%s'", what);
  if (rows * D == 0) return XRL_OK;
  const unsigned blocks = (unsigned)((rows * D + 255) / 256);
  if (typed && c->elem == 2)
    export_rows_kernel<bf16_t><<<dim3(blocks), dim3(256), 0, c->stream>>>((const bf16_t *)src, rows, D, row_src, d_out);
  else
    export_rows_kernel<float><<<dim3(blocks), dim3(256), 0, c->stream>>>((const float *)src, rows, D, row_src, d_out);
  HIP_TRY(hipGetLastError());
  return XRL_OK;
}

}  // extern "C"
