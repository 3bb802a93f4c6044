// Device side of the library: context, weight upload, workspace, kernel sequencing.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>
#include <new>
#include <vector>

#include "heads.hip.h"
#include "mlp2.hip.h"
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

// Layer-2 weights W [H, H] -> [chunk][feature block][lane][j]: the contraction index follows the
// accumulator layout of layer 1: element j of chunk c in lane group g is input feature
// 2V*c + 8*(j/4) + 4*g + j%4; lane l addresses output feature 32*nb + l%32.
template <typename T>
void swizzle_l2(const float *W, int H, int V, std::vector<T> &out) {
  const int SL = 2 * V, MB = H / 32, nc = H / SL;
  out.assign((size_t)nc * MB * 64 * V, HostCvt<T>::cvt(0.f));
  for (int c = 0; c < nc; ++c)
    for (int nb = 0; nb < MB; ++nb)
      for (int l = 0; l < 64; ++l)
        for (int j = 0; j < V; ++j) {
          const int g = l / 32, f = SL * c + 8 * (j / 4) + 4 * g + j % 4, f2 = 32 * nb + l % 32;
          out[(((size_t)c * MB + nb) * 64 + l) * V + j] = HostCvt<T>::cvt(W[(size_t)f * H + f2]);
        }
}

struct EncMlp {           // device pointers of one encoder MLP
  const void *W1s = nullptr, *W2s = nullptr;
  const float *b1 = nullptr, *b2 = nullptr;
  int nslab1 = 0;
};

}  // namespace

struct xrl_ctx {
  xrl_model_desc m;
  Layout L;
  hipStream_t stream = nullptr;
  int elem = 4;                 // bytes per stored activation / operand
  float *d_w = nullptr;         // flat fp32 weights
  char *d_swz = nullptr;        // fragment-ordered encoder weights
  size_t swz_bytes = 0;
  EncMlp embed;
  std::vector<EncMlp> edge, node;
  // workspaces (grow-only): encoder activations, and a separate small one for the heads
  char *ws = nullptr;
  size_t ws_bytes = 0;
  char *hws = nullptr;
  size_t hws_bytes = 0;
  // buffers of the last encode (inside ws)
  uint64_t enc_batch = 0;
  bool enc_saved = false;
  float *a0 = nullptr, *pool = nullptr, *carry = nullptr, *ro_act[2] = {nullptr, nullptr};
  std::vector<void *> h, agg;   // h[0..R], agg[1..R] (index 0 unused)
};

extern "C" void xrl_batch_release_device(xrl_batch *b) {
  if (b && b->dev.block) {
    (void)hipFree(b->dev.block);
    b->dev = xrl_batch_device();
    b->uploaded = false;
  }
}

namespace {

int upload_weights(xrl_ctx *c, const float *w) {
  const xrl_model_desc &m = c->m;
  for (int64_t i = 0; i < c->L.total; ++i)
    if (!std::isfinite(w[i])) return fail(XRL_ERR_VALUE, "weights[%lld] is not finite", (long long)i);
  const int V = c->elem == 2 ? 8 : 4, H = m.hidden;
  // build the fragment-ordered blob on the host
  std::vector<char> blob;
  struct Ref { size_t w1, w2; int ns; };
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
      swizzle_l2<uint16_t>(w + r.w[1], H, V, t);
      ref.w2 = put(t.data(), t.size() * 2);
    } else {
      std::vector<float> t;
      swizzle_l1<float>(w + r.w[0], r.d_in[0], H, V, t);
      ref.w1 = put(t.data(), t.size() * 4);
      swizzle_l2<float>(w + r.w[1], H, V, t);
      ref.w2 = put(t.data(), t.size() * 4);
    }
    refs.push_back(ref);
  };
  add(c->L.embed, true);   // the embed MLP's first layer keeps fp32 operands in both modes
  for (int r = 0; r < m.rounds; ++r) { add(c->L.edge[r], false); add(c->L.node[r], false); }
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
    e.b1 = c->d_w + r.b[0];
    e.b2 = c->d_w + r.b[1];
    e.nslab1 = ref.ns;
  };
  size_t i = 0;
  bind(c->embed, refs[i++], c->L.embed);
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

int ensure_hws(xrl_ctx *c, size_t bytes) {
  if (bytes <= c->hws_bytes) return XRL_OK;
  HIP_TRY(hipStreamSynchronize(c->stream));
  if (c->hws) HIP_TRY(hipFree(c->hws));
  c->hws = nullptr;
  c->hws_bytes = 0;
  hipError_t e = hipMalloc((void **)&c->hws, bytes);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return fail(XRL_ERR_OOM, "head workspace of %zu bytes: %s", bytes, hipGetErrorString(e));
  }
  c->hws_bytes = bytes;
  return XRL_OK;
}

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
template <typename TIn, typename TOut, int VEC>
int launch_segsum(xrl_ctx *c, const void *vals, const int32_t *perm, const int32_t *ptr,
                  const int32_t *row_seg, int64_t n_rows, int64_t n_seg, int D, void *out,
                  float *carry) {
  constexpr int RT = 16;
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
  a.D = D; a.RT = RT; a.out = out; a.carry = carry;
  const int64_t nsub = (n_rows + RT - 1) / RT;
  const int64_t threads = nsub * (D / VEC);
  const int64_t blocks = (threads + 255) / 256;
  segsum_kernel<TIn, TOut, VEC, RT><<<dim3((unsigned)blocks), dim3(256), 0, c->stream>>>(a);
  segsum_fixup<TOut><<<dim3((unsigned)nsub), dim3(64), 0, c->stream>>>(ptr, row_seg, n_rows, n_seg, D,
                                                                      RT, carry, (TOut *)out);
  HIP_TRY(hipGetLastError());
  return XRL_OK;
}

size_t segsum_carry_floats(int64_t n_rows, int D) { return (size_t)((n_rows + 15) / 16) * 2 * D; }

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

template <typename T>
int launch_mlp2(xrl_ctx *c, int kind, Mlp2Args &a) {
  a.n_blocks = (a.n_rows + 127) / 128;
  switch (c->m.hidden) {
    case 64: return launch_mlp2_h<T, 64>(c, kind, a);
    case 128: return launch_mlp2_h<T, 128>(c, kind, a);
    case 256: return launch_mlp2_h<T, 256>(c, kind, a);
  }
  return fail(XRL_ERR_UNSUPPORTED, "hidden = %d", c->m.hidden);
}

int launch_rowmlp(xrl_ctx *c, const MlpRef &r, bool relu_last, const float *in1, int w1,
                  const float *in2, int w2, int64_t n_rows, float *out, float *const *act) {
  if (n_rows <= 0) return XRL_OK;
  RowMlpArgs a;
  memset(&a, 0, sizeof(a));
  a.n_layers = r.n_layers;
  a.relu_last = relu_last ? 1 : 0;
  int dmax = r.d_in[0];
  for (int l = 0; l < r.n_layers; ++l) {
    a.W[l] = c->d_w + r.w[l];
    a.b[l] = c->d_w + r.b[l];
    a.d_in[l] = r.d_in[l];
    a.d_out[l] = r.d_out[l];
    a.act[l] = act ? act[l] : nullptr;
    if (r.d_out[l] > dmax) dmax = r.d_out[l];
  }
  a.in1 = in1; a.in2 = in2; a.w1 = w1; a.w2 = w2; a.n_rows = n_rows; a.out = out;
  const size_t shm = (size_t)2 * ROWMLP_ROWS * dmax * sizeof(float);
  const unsigned blocks = (unsigned)((n_rows + ROWMLP_ROWS - 1) / ROWMLP_ROWS);
  rowmlp_kernel<<<dim3(blocks), dim3(256), shm, c->stream>>>(a);
  HIP_TRY(hipGetLastError());
  return XRL_OK;
}

template <typename T>
__global__ void export_rows_kernel(const T *src, const int32_t *in_ptr, int64_t n_rows, int D,
                                   float *dst) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_rows * D) return;
  const int64_t r = i / D;
  float v = (float)src[i];
  if (in_ptr && in_ptr[r + 1] == in_ptr[r]) v = 0.f;   // rows nobody wrote: receivers without in-edges
  dst[i] = v;
}

template <typename T>
int encode_impl(xrl_ctx *c, const xrl_batch *b, float *d_emb, int save) {
  const xrl_model_desc &m = c->m;
  const int H = m.hidden, R = m.rounds, De = m.d_edge;
  const int64_t N = b->N, E = b->E, G = b->G;
  // ---- workspace plan
  const int nh = save ? R + 1 : (R > 0 ? 2 : 1), nagg = save ? R : (R > 0 ? 1 : 0);
  size_t need = 0;
  auto acc = [&](size_t bytes) { need += align_up(bytes); };
  acc((size_t)N * De * 4);
  for (int i = 0; i < nh + nagg; ++i) acc((size_t)N * H * sizeof(T));
  const size_t carry_floats = std::max(std::max(segsum_carry_floats(E, De), segsum_carry_floats(N, H)),
                                       (size_t)((E + 31) / 32) * 2 * H);
  acc(carry_floats * 4);
  acc((size_t)G * H * 4);
  acc((size_t)G * H * 4);
  acc((size_t)G * H * 4);
  int rc = ensure_ws(c, need);
  if (rc) return rc;
  Bump bump{c->ws};
  c->a0 = bump.take<float>((size_t)N * De);
  c->h.assign(R + 1, nullptr);
  c->agg.assign(R + 1, nullptr);
  std::vector<T *> hb(nh), ab(std::max(nagg, 1), nullptr);
  for (int i = 0; i < nh; ++i) hb[i] = bump.take<T>((size_t)N * H);
  for (int i = 0; i < nagg; ++i) ab[i] = bump.take<T>((size_t)N * H);
  c->carry = bump.take<float>(carry_floats);
  c->pool = bump.take<float>((size_t)G * H);
  c->ro_act[0] = bump.take<float>((size_t)G * H);
  c->ro_act[1] = bump.take<float>((size_t)G * H);
  c->enc_batch = b->id;
  c->enc_saved = save != 0;
  const xrl_batch_device &d = b->dev;

  // ---- node-update layer: sum incoming edge attrs, then the embed MLP
  if (De % 4 == 0)
    rc = launch_segsum<float, float, 4>(c, d.edge_feat, nullptr, d.in_ptr, d.in_dst, E, N, De, c->a0, c->carry);
  else
    rc = launch_segsum<float, float, 1>(c, d.edge_feat, nullptr, d.in_ptr, d.in_dst, E, N, De, c->a0, c->carry);
  if (rc) return rc;
  Mlp2Args a;
  memset(&a, 0, sizeof(a));
  a.De = De; a.Tn = m.n_op_types; a.Dd = m.n_node_dense;
  a.in_ptr = d.in_ptr; a.in_src = d.in_src; a.in_dst = d.in_dst;
  a.edge_feat = d.edge_feat; a.a0 = c->a0; a.node_op = d.node_op; a.node_dense = d.node_dense;
  a.carry = c->carry;
  auto set_w = [&](const EncMlp &e) { a.W1s = e.W1s; a.W2s = e.W2s; a.b1 = e.b1; a.b2 = e.b2; a.nslab1 = e.nslab1; };
  set_w(c->embed);
  a.n_rows = N; a.out = hb[0];
  if ((rc = launch_mlp2<T>(c, KIND_EMBED, a))) return rc;
  c->h[0] = hb[0];
  T *hcur = hb[0];
  // ---- message-passing rounds
  for (int r = 0; r < R; ++r) {
    T *aggb = save ? ab[r] : ab[0];
    T *hnext = save ? hb[r + 1] : hb[(r + 1) & 1];
    set_w(c->edge[r]);
    a.n_rows = E; a.h = hcur; a.out = aggb;
    if ((rc = launch_mlp2<T>(c, KIND_EDGE, a))) return rc;
    if (E > 0) {
      const int64_t nwt = (E + 31) / 32;
      segsum_fixup<T><<<dim3((unsigned)nwt), dim3(64), 0, c->stream>>>(d.in_ptr, d.in_dst, E, N, H, 32,
                                                                    c->carry, aggb);
    }
    set_w(c->node[r]);
    a.n_rows = N; a.h = hcur; a.agg = aggb; a.out = hnext;
    if ((rc = launch_mlp2<T>(c, KIND_NODE, a))) return rc;
    c->h[r + 1] = hnext;
    c->agg[r + 1] = aggb;
    hcur = hnext;
  }
  // ---- global-update layer: per-graph sum (or mean), then the readout MLP
  constexpr int PV = 16 / sizeof(T);
  rc = launch_segsum<T, float, PV>(c, hcur, nullptr, d.graph_node_ptr, d.node_graph, N, G, H, c->pool, c->carry);
  if (rc) return rc;
  if (m.readout == XRL_READOUT_MEAN && G > 0)
    mean_scale_kernel<<<dim3((unsigned)((G * H + 255) / 256)), dim3(256), 0, c->stream>>>(c->pool, d.graph_node_ptr, G, H, 0);
  rc = launch_rowmlp(c, c->L.readout, true, c->pool, H, d.graph_global, m.d_global, G, d_emb, c->ro_act);
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
  Layout L;
  int rc = build_layout(*model, L);
  if (rc) return rc;
  if (model->hidden != 64 && model->hidden != 128 && model->hidden != 256)
    return fail(XRL_ERR_UNSUPPORTED, "hidden = %d: the kernels cover 64, 128 and 256", model->hidden);
  if (model->mlp_layers != 2)
    return fail(XRL_ERR_UNSUPPORTED, "mlp_layers = %d: the kernels cover 2", model->mlp_layers);
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
  c->stream = (hipStream_t)hip_stream;
  c->elem = model->precision == XRL_PREC_BF16 ? 2 : 4;
  e = hipMalloc((void **)&c->d_w, sizeof(float) * L.total);
  if (e != hipSuccess) {
    delete c;
    return fail(XRL_ERR_OOM, "device weights: %s", hipGetErrorString(e));
  }
  rc = upload_weights(c, weights_host);
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
  if (c->d_swz) (void)hipFree(c->d_swz);
  if (c->ws) (void)hipFree(c->ws);
  if (c->hws) (void)hipFree(c->hws);
  delete c;
  return XRL_OK;
}

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
               o_gg = plan((size_t)G * Dg * 4), o_mask = plan(G);
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
  HIP_TRY(cp(o_op, b->node_op.data(), N * 4));
  HIP_TRY(cp(o_inp, b->in_ptr.data(), (N + 1) * 4));
  HIP_TRY(cp(o_ins, b->in_src.data(), E * 4));
  HIP_TRY(cp(o_ind, b->in_dst.data(), E * 4));
  HIP_TRY(cp(o_outp, b->out_ptr.data(), (N + 1) * 4));
  HIP_TRY(cp(o_outpos, b->out_pos.data(), E * 4));
  HIP_TRY(cp(o_ng, b->node_graph.data(), N * 4));
  HIP_TRY(cp(o_nd, b->node_dense.data(), (size_t)N * Dd * 4));
  HIP_TRY(cp(o_ef, b->edge_feat.data(), (size_t)E * De * 4));
  HIP_TRY(cp(o_gg, b->graph_global.data(), (size_t)G * Dg * 4));
  HIP_TRY(cp(o_mask, b->mask.data(), G));
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
  b->uploaded = true;
  return XRL_OK;
}

int xrl_encode(xrl_ctx *c, const xrl_batch *b, float *d_emb, int save_for_backward) {
  int rc = check_batch(c, b, "xrl_encode");
  if (rc) return rc;
  if (!d_emb && b->G > 0) return fail(XRL_ERR_NULL, "xrl_encode: d_emb is NULL");
  if (b->G == 0) return XRL_OK;
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
  const int H = c->m.hidden;
  rc = ensure_hws(c, align_up((size_t)b->G * 4) + align_up((size_t)b->S * H * 4));
  if (rc) return rc;
  float *logit = d_logit ? d_logit : (float *)c->hws;
  float *zmean = (float *)(c->hws + align_up((size_t)b->G * 4));
  rc = launch_rowmlp(c, c->L.policy, false, d_emb, H, nullptr, 0, b->G, logit, nullptr);
  if (rc) return rc;
  state_policy_kernel<<<dim3((unsigned)b->S), dim3(256), 0, c->stream>>>(
      logit, b->dev.mask, b->dev.state_graph_ptr, d_emb, H, d_logp, d_entropy, d_action, zmean);
  rc = launch_rowmlp(c, c->L.value, false, zmean, H, nullptr, 0, b->S, d_value, nullptr);
  if (rc) return rc;
  HIP_TRY(hipGetLastError());
  return XRL_OK;
}

int xrl_policy_value_backward(xrl_ctx *c, const xrl_batch *b, const float *d_emb,
                              const float *d_dlogp, const float *d_dvalue,
                              const float *d_dentropy, float *d_demb, float *d_dweights) {
  (void)d_emb; (void)d_dlogp; (void)d_dvalue; (void)d_dentropy; (void)d_demb; (void)d_dweights;
  int rc = check_batch(c, b, "xrl_policy_value_backward");
  if (rc) return rc;
  return fail(XRL_ERR_UNSUPPORTED, "xrl_policy_value_backward: not built yet");
}

int xrl_encode_backward(xrl_ctx *c, const xrl_batch *b, const float *d_demb, float *d_dweights) {
  (void)d_demb; (void)d_dweights;
  int rc = check_batch(c, b, "xrl_encode_backward");
  if (rc) return rc;
  return fail(XRL_ERR_UNSUPPORTED, "xrl_encode_backward: not built yet");
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
  bool typed = true, mask_rows = false;
  if (!strcmp(what, "a0")) { src = c->a0; D = c->m.d_edge; typed = false; }
  else if (!strcmp(what, "pool")) { src = c->pool; rows = G; typed = false; }
  else if (!strcmp(what, "h")) {
    if (round < 0 || round > R) return fail(XRL_ERR_INDEX, "h: round %d outside [0, %d]", round, R);
    src = c->h[round];
  } else if (!strcmp(what, "agg")) {
    if (round < 1 || round > R) return fail(XRL_ERR_INDEX, "agg: round %d outside [1, %d]", round, R);
    src = c->agg[round];
    mask_rows = true;
  } else return fail(XRL_ERR_INDEX, "xrl_get_activation: unknown tensor '%s'", what);
  if (rows * D == 0) return XRL_OK;
  const unsigned blocks = (unsigned)((rows * D + 255) / 256);
  const int32_t *ip = mask_rows ? b->dev.in_ptr : nullptr;
  if (typed && c->elem == 2)
    export_rows_kernel<bf16_t><<<dim3(blocks), dim3(256), 0, c->stream>>>((const bf16_t *)src, ip, rows, D, d_out);
  else
    export_rows_kernel<float><<<dim3(blocks), dim3(256), 0, c->stream>>>((const float *)src, ip, rows, D, d_out);
  HIP_TRY(hipGetLastError());
  return XRL_OK;
}

}  // extern "C"
