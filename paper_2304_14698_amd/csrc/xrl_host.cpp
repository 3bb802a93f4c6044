// Host side of the library: weight layout, validation and packing of states into the
// receiver-sorted meta-batch. Nothing in this file calls the GPU runtime.
#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>
#include <system_error>
#include <thread>

#include "xrl_internal.h"

namespace xrl {

static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

int fail(int code, const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

static void add_mlp(Layout &L, MlpRef &ref, const std::string &prefix, int d_in,
                    const std::vector<int> &widths) {
  ref.n_layers = (int)widths.size();
  int d = d_in;
  for (size_t i = 0; i < widths.size(); ++i) {
    int w = widths[i];
    ref.d_in[i] = d;
    ref.d_out[i] = w;
    ref.w[i] = L.total;
    L.tensors.push_back({prefix + ".W" + std::to_string(i), L.total, d, w});
    L.total += (int64_t)d * w;
    ref.b[i] = L.total;
    L.tensors.push_back({prefix + ".b" + std::to_string(i), L.total, w, 0});
    L.total += w;
    d = w;
  }
}

int build_layout(const xrl_model_desc &m, Layout &L) {
  if (m.n_op_types < 1 || m.n_node_dense < 0 || m.d_edge < 1 || m.d_global < 0 || m.hidden < 1 ||
      m.rounds < 0 || m.mlp_layers < 1 || m.mlp_layers > 3 || m.head_hidden[0] < 1 ||
      m.head_hidden[1] < 1)
    return fail(XRL_ERR_SHAPE, "model: non-positive or out-of-range dimension");
  if (m.n_op_types > 4096 || m.n_node_dense > 4096 || m.d_edge > 4096 || m.d_global > 4096 ||
      m.hidden > 4096 || m.rounds > 1024 || m.head_hidden[0] > 4096 || m.head_hidden[1] > 4096)
    return fail(XRL_ERR_SHAPE, "model: dimension above 4096 (rounds above 1024)");
  if (m.readout != XRL_READOUT_SUM && m.readout != XRL_READOUT_MEAN)
    return fail(XRL_ERR_SHAPE, "model: readout must be XRL_READOUT_SUM or XRL_READOUT_MEAN");
  if (m.precision != XRL_PREC_FP32 && m.precision != XRL_PREC_BF16)
    return fail(XRL_ERR_SHAPE, "model: precision must be XRL_PREC_FP32 or XRL_PREC_BF16");
  if (m.round_kind != XRL_ROUND_MLP && m.round_kind != XRL_ROUND_GAT)
    return fail(XRL_ERR_SHAPE, "model: round_kind must be XRL_ROUND_MLP or XRL_ROUND_GAT");
  L = Layout();
  const int H = m.hidden;
  std::vector<int> enc(m.mlp_layers, H);
  add_mlp(L, L.embed, "embed", m.d_edge + m.n_op_types + m.n_node_dense, enc);
  if (m.round_kind == XRL_ROUND_GAT) {
    L.gat.resize(m.rounds);
    for (int r = 0; r < m.rounds; ++r) {
      const std::string p = "gat" + std::to_string(r);
      L.gat[r].W = L.total;
      L.tensors.push_back({p + ".W", L.total, H, H});
      L.total += (int64_t)H * H;
      L.gat[r].a_src = L.total;
      L.tensors.push_back({p + ".a_src", L.total, H, 0});
      L.total += H;
      L.gat[r].a_dst = L.total;
      L.tensors.push_back({p + ".a_dst", L.total, H, 0});
      L.total += H;
    }
  } else {
    L.edge.resize(m.rounds);
    L.node.resize(m.rounds);
    for (int r = 0; r < m.rounds; ++r) {
      add_mlp(L, L.edge[r], "edge" + std::to_string(r), 2 * H + m.d_edge, enc);
      add_mlp(L, L.node[r], "node" + std::to_string(r), 2 * H, enc);
    }
  }
  add_mlp(L, L.readout, "readout", H + m.d_global, enc);
  std::vector<int> head = {m.head_hidden[0], m.head_hidden[1], 1};
  add_mlp(L, L.policy, "policy", H, head);
  add_mlp(L, L.value, "value", H, head);
  return XRL_OK;
}

}  // namespace xrl

using namespace xrl;

namespace {
// Packing works graph by graph (a graph's nodes, and its edges in receiver order, occupy the same
// index ranges before and after), so large batches are cut into contiguous graph ranges of about
// equal nodes + edges, one per thread. XRL_PACK_THREADS overrides the thread count (1 = serial).
struct PackIssue {
  int code = 0;
  char msg[200] = "";
  void set(int c, const char *fmt, ...) {
    if (code) return;                                   // keep the first one of this range
    code = c;
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(msg, sizeof(msg), fmt, ap);
    va_end(ap);
  }
};

int pack_thread_count(int64_t work) {
  if (const char *e = getenv("XRL_PACK_THREADS")) {
    const int v = atoi(e);
    if (v >= 1) return v > 64 ? 64 : v;
  }
  int hw = (int)std::thread::hardware_concurrency();
  if (hw < 1) hw = 1;
  if (hw > 16) hw = 16;
  int64_t t = work / 65536;
  return (int)(t < 1 ? 1 : (t > hw ? hw : t));
}

// graph range boundaries [T + 1], balanced by nodes + edges
std::vector<int64_t> graph_ranges(const xrl_state_desc *st, int64_t G, int T) {
  std::vector<int64_t> cut(T + 1, G);
  cut[0] = 0;
  const int64_t total = (int64_t)st->graph_node_ptr[G] + st->graph_edge_ptr[G];
  int64_t g = 0;
  for (int t = 1; t < T; ++t) {
    const int64_t want = total * t / T;
    while (g < G && (int64_t)st->graph_node_ptr[g] + st->graph_edge_ptr[g] < want) ++g;
    cut[t] = g;
  }
  return cut;
}

// fn(t, g_begin, g_end) for every range; returns false if a range ran out of memory. Ranges whose
// thread cannot be started run on the calling thread.
template <typename F>
bool run_ranges(const std::vector<int64_t> &cut, F fn) {
  const int T = (int)cut.size() - 1;
  std::atomic<bool> ok{true};
  auto guarded = [&](int t) {
    try {
      fn(t, cut[t], cut[t + 1]);
    } catch (const std::bad_alloc &) {
      ok = false;
    }
  };
  std::vector<std::thread> th;
  th.reserve(T > 1 ? T - 1 : 0);
  int started = 1;
  for (; started < T; ++started) {
    try {
      th.emplace_back(guarded, started);
    } catch (const std::system_error &) {
      break;
    }
  }
  guarded(0);
  for (int t = started; t < T; ++t) guarded(t);
  for (auto &x : th) x.join();
  return ok;
}
}  // namespace

extern "C" {

const char *xrl_last_error(void) { return g_err; }
const char *xrl_version(void) { return "xrl 0.1 (gfx950)"; }

int64_t xrl_weight_count(const xrl_model_desc *model) {
  if (!model) return fail(XRL_ERR_NULL, "xrl_weight_count: model is NULL");
  Layout L;
  int rc = build_layout(*model, L);
  return rc ? rc : L.total;
}

int32_t xrl_weight_tensor_count(const xrl_model_desc *model) {
  if (!model) return fail(XRL_ERR_NULL, "xrl_weight_tensor_count: model is NULL");
  Layout L;
  int rc = build_layout(*model, L);
  return rc ? rc : (int32_t)L.tensors.size();
}

int xrl_weight_tensor(const xrl_model_desc *model, int32_t index, char *name, size_t name_cap,
                      int64_t *offset, int64_t *rows, int64_t *cols) {
  if (!model) return fail(XRL_ERR_NULL, "xrl_weight_tensor: model is NULL");
  Layout L;
  int rc = build_layout(*model, L);
  if (rc) return rc;
  if (index < 0 || index >= (int32_t)L.tensors.size())
    return fail(XRL_ERR_INDEX, "xrl_weight_tensor: index %d outside [0, %zu)", index,
                L.tensors.size());
  const WeightTensor &t = L.tensors[index];
  if (name && name_cap) {
    strncpy(name, t.name.c_str(), name_cap - 1);
    name[name_cap - 1] = 0;
  }
  if (offset) *offset = t.offset;
  if (rows) *rows = t.rows;
  if (cols) *cols = t.cols;
  return XRL_OK;
}

static int check_ptr(const int32_t *p, int64_t n, const char *what) {
  if (p[0] != 0) return fail(XRL_ERR_SHAPE, "%s[0] = %d, must be 0", what, p[0]);
  for (int64_t i = 0; i < n; ++i)
    if (p[i + 1] < p[i])
      return fail(XRL_ERR_SHAPE, "%s decreases at %lld (%d -> %d)", what, (long long)i, p[i],
                  p[i + 1]);
  return XRL_OK;
}

static bool all_finite(const float *p, int64_t n, int64_t *where) {
  for (int64_t i = 0; i < n; ++i)
    if (!std::isfinite(p[i])) {
      *where = i;
      return false;
    }
  return true;
}

int xrl_pack_state(const xrl_model_desc *model, const xrl_state_desc *st, xrl_batch **out) {
  if (!model || !st || !out) return fail(XRL_ERR_NULL, "xrl_pack_state: NULL argument");
  *out = nullptr;
  Layout L;
  int rc = build_layout(*model, L);
  if (rc) return rc;
  const int64_t S = st->n_states;
  if (S < 0) return fail(XRL_ERR_SHAPE, "n_states = %lld is negative", (long long)S);
  if (!st->state_graph_ptr || !st->graph_node_ptr || !st->graph_edge_ptr || !st->slot_mask)
    return fail(XRL_ERR_NULL, "xrl_pack_state: a ptr array or slot_mask is NULL");
  if ((rc = check_ptr(st->state_graph_ptr, S, "state_graph_ptr"))) return rc;
  const int64_t G = st->state_graph_ptr[S];
  for (int64_t s = 0; s < S; ++s)
    if (st->state_graph_ptr[s + 1] == st->state_graph_ptr[s])
      return fail(XRL_ERR_SHAPE, "state %lld has no graph (needs its current graph)", (long long)s);
  if ((rc = check_ptr(st->graph_node_ptr, G, "graph_node_ptr"))) return rc;
  if ((rc = check_ptr(st->graph_edge_ptr, G, "graph_edge_ptr"))) return rc;
  const int64_t N = st->graph_node_ptr[G], E = st->graph_edge_ptr[G];
  const int Dd = model->n_node_dense, De = model->d_edge, Dg = model->d_global;
  if (N > 0 && (!st->node_op || (Dd > 0 && !st->node_dense)))
    return fail(XRL_ERR_NULL, "node_op or node_dense is NULL");
  if (E > 0 && (!st->edge_src || !st->edge_dst || !st->edge_feat))
    return fail(XRL_ERR_NULL, "edge_src, edge_dst or edge_feat is NULL");
  for (int64_t s = 0; s < S; ++s)
    if (st->slot_mask[st->state_graph_ptr[s]] == 0)
      return fail(XRL_ERR_MASK, "state %lld masks its No-Op slot (its first graph)", (long long)s);
  // per-range checks, reported in the order a serial pass would find them: operator ids, edge
  // endpoints, node attributes, edge attributes; within a kind, the lowest range first
  const int T = pack_thread_count(N + E);
  const std::vector<int64_t> cut = graph_ranges(st, G, T);
  {
    std::vector<PackIssue> issue((size_t)4 * T);
    const bool ok = run_ranges(cut, [&](int t, int64_t g0, int64_t g1) {
      const int64_t n0 = st->graph_node_ptr[g0], n1 = st->graph_node_ptr[g1];
      const int64_t e0 = st->graph_edge_ptr[g0], e1 = st->graph_edge_ptr[g1];
      for (int64_t i = n0; i < n1; ++i)
        if (st->node_op[i] < 0 || st->node_op[i] >= model->n_op_types) {
          issue[0 * T + t].set(XRL_ERR_INDEX, "node %lld: op id %d outside [0, %d)", (long long)i,
                               st->node_op[i], model->n_op_types);
          break;
        }
      for (int64_t g = g0; g < g1 && !issue[1 * T + t].code; ++g) {
        const int32_t n = st->graph_node_ptr[g + 1] - st->graph_node_ptr[g];
        for (int64_t e = st->graph_edge_ptr[g]; e < st->graph_edge_ptr[g + 1]; ++e)
          if (st->edge_src[e] < 0 || st->edge_src[e] >= n || st->edge_dst[e] < 0 || st->edge_dst[e] >= n) {
            issue[1 * T + t].set(XRL_ERR_INDEX, "edge %lld of graph %lld: endpoint (%d -> %d) outside [0, %d)",
                                 (long long)e, (long long)g, st->edge_src[e], st->edge_dst[e], n);
            break;
          }
      }
      int64_t where = 0;
      if (Dd > 0 && !all_finite(st->node_dense + n0 * Dd, (n1 - n0) * Dd, &where))
        issue[2 * T + t].set(XRL_ERR_VALUE, "node_dense[%lld] is not finite", (long long)(n0 * Dd + where));
      if (!all_finite(st->edge_feat + e0 * De, (e1 - e0) * De, &where))
        issue[3 * T + t].set(XRL_ERR_VALUE, "edge_feat[%lld] is not finite", (long long)(e0 * De + where));
    });
    if (!ok) return fail(XRL_ERR_OOM, "xrl_pack_state: out of host memory");
    for (const PackIssue &is : issue)
      if (is.code) return fail(is.code, "%s", is.msg);
  }
  int64_t bad = 0;
  if (st->graph_global && !all_finite(st->graph_global, G * Dg, &bad))
    return fail(XRL_ERR_VALUE, "graph_global[%lld] is not finite", (long long)bad);

  xrl_batch *b = new (std::nothrow) xrl_batch();
  if (!b) return fail(XRL_ERR_OOM, "xrl_pack_state: out of host memory");
  try {
    static std::atomic<uint64_t> next_id{1};
    b->id = next_id++;
    b->model = *model;
    b->S = S; b->G = G; b->N = N; b->E = E;
    b->state_graph_ptr.assign(st->state_graph_ptr, st->state_graph_ptr + S + 1);
    b->graph_node_ptr.assign(st->graph_node_ptr, st->graph_node_ptr + G + 1);
    b->node_op.resize(N);                            // (copied by the packing threads below)
    b->node_dense.resize(Dd > 0 ? (size_t)N * Dd : 0);
    b->mask.resize(G);
    for (int64_t g = 0; g < G; ++g) b->mask[g] = st->slot_mask[g] ? 1 : 0;
    if (st->graph_global)
      b->graph_global.assign(st->graph_global, st->graph_global + G * Dg);
    else
      b->graph_global.assign((size_t)(G * Dg), 0.0f);
    for (int64_t s = 0; s < S; ++s) {
      int32_t c = st->state_graph_ptr[s + 1] - st->state_graph_ptr[s];
      if (c > b->max_slots) b->max_slots = c;
    }
    b->node_graph.resize(N);
    b->in_ptr.assign(N + 1, 0);
    b->out_ptr.assign(N + 1, 0);
    b->in_src.resize(E); b->in_dst.resize(E); b->in_eid.resize(E); b->out_pos.resize(E);
    b->edge_feat.resize((size_t)E * De);
    // Receiver order: stable counting sort of each graph's edges by receiver; then the sender-side
    // index (receiver-order positions grouped by sender, ascending position). A graph's edges
    // keep the index range they came with, so the graph ranges are independent.
    const bool sorted = run_ranges(cut, [&](int, int64_t g0, int64_t g1) {
      std::vector<int32_t> cur;
      for (int64_t g = g0; g < g1; ++g) {
        const int32_t base = st->graph_node_ptr[g], n = st->graph_node_ptr[g + 1] - base;
        const int64_t e0 = st->graph_edge_ptr[g], e1 = st->graph_edge_ptr[g + 1];
        for (int32_t i = 0; i < n; ++i) b->node_graph[base + i] = (int32_t)g;
        if (n > 0) {
          memcpy(&b->node_op[base], st->node_op + base, sizeof(int32_t) * n);
          if (Dd > 0) memcpy(&b->node_dense[(size_t)base * Dd], st->node_dense + (size_t)base * Dd, sizeof(float) * n * Dd);
        }
        int32_t *inp = b->in_ptr.data() + base + 1, *outp = b->out_ptr.data() + base + 1;   // counts, then ends
        for (int64_t e = e0; e < e1; ++e) {
          inp[st->edge_dst[e]]++;
          outp[st->edge_src[e]]++;
        }
        cur.assign((size_t)2 * n, 0);
        int32_t ri = (int32_t)e0, ro = (int32_t)e0;
        for (int32_t i = 0; i < n; ++i) {
          cur[i] = ri; cur[n + i] = ro;                   // first position of node i's in- / out-edges
          ri += inp[i]; ro += outp[i];
          inp[i] = ri; outp[i] = ro;
        }
        for (int64_t e = e0; e < e1; ++e) {
          const int32_t p = cur[st->edge_dst[e]]++;
          b->in_src[p] = base + st->edge_src[e];
          b->in_dst[p] = base + st->edge_dst[e];
          b->in_eid[p] = (int32_t)e;
          memcpy(&b->edge_feat[(size_t)p * De], &st->edge_feat[(size_t)e * De], sizeof(float) * De);
        }
        for (int64_t p = e0; p < e1; ++p) b->out_pos[cur[n + (b->in_src[p] - base)]++] = (int32_t)p;
      }
    });
    if (!sorted) throw std::bad_alloc();
    {  // Edge tiles of the message kernels: consecutive receiver-order edges, at most 32 per tile,
       // cut at receiver boundaries so that a receiver's in-edges share a tile. Only a receiver
       // with more than 32 in-edges is split (into full tiles plus a remainder that later
       // receivers may join); its pieces are recombined by the carry fix-up.
      b->tile_ptr.clear();
      b->tile_ptr.push_back(0);
      b->n_split_tiles = 0;
      int32_t fill = 0;                 // edges in the open tile
      for (int64_t n = 0; n < N; ++n) {
        int32_t d = b->in_ptr[n + 1] - b->in_ptr[n];
        if (d == 0) continue;
        if (fill + d > 32 && fill > 0) {
          b->tile_ptr.push_back(b->in_ptr[n]);
          fill = 0;
        }
        while (d > 32) {                // fill == 0 here
          b->tile_ptr.push_back(b->tile_ptr.back() + 32);
          b->n_split_tiles++;
          d -= 32;
        }
        fill += d;
      }
      if (fill > 0) b->tile_ptr.push_back((int32_t)E);
    }
    b->max_graph_nodes = 0;
    for (int64_t g = 0; g < G; ++g)
      b->max_graph_nodes = std::max(b->max_graph_nodes, b->graph_node_ptr[g + 1] - b->graph_node_ptr[g]);
    b->gtile_ptr.clear();
    b->graph_tile_ptr.clear();
    b->max_graph_tiles = 0;
    if (G <= kGraphTileMaxGraphs) {   // the same rule graph by graph (see xrl_batch)
      bool ok = true;
      b->graph_tile_ptr.push_back(0);
      for (int64_t g = 0; g < G && ok; ++g) {
        int32_t fill = 0;
        const int32_t n1 = b->graph_node_ptr[g + 1];
        for (int32_t n = b->graph_node_ptr[g]; n < n1; ++n) {
          const int32_t d = b->in_ptr[n + 1] - b->in_ptr[n];
          if (d == 0) continue;
          if (d > 32) { ok = false; break; }
          if (fill + d > 32 || fill == 0) {
            b->gtile_ptr.push_back(b->in_ptr[n]);
            fill = 0;
          }
          fill += d;
        }
        b->max_graph_tiles = std::max(b->max_graph_tiles, (int32_t)b->gtile_ptr.size() - b->graph_tile_ptr.back());
        b->graph_tile_ptr.push_back((int32_t)b->gtile_ptr.size());
      }
      if (ok) {
        b->gtile_ptr.push_back((int32_t)E);
      } else {
        b->gtile_ptr.clear();
        b->graph_tile_ptr.clear();
      }
    }
  } catch (const std::bad_alloc &) {
    delete b;
    return fail(XRL_ERR_OOM, "xrl_pack_state: out of host memory");
  }
  *out = b;
  return XRL_OK;
}

int xrl_edge_features_from_shapes(const int32_t *shape_ptr, const int64_t *dims, int64_t n_edges,
                                  double M, float *edge_feat) {
  if (n_edges < 0) return fail(XRL_ERR_SHAPE, "n_edges = %lld is negative", (long long)n_edges);
  if (!shape_ptr || (n_edges > 0 && !edge_feat))
    return fail(XRL_ERR_NULL, "xrl_edge_features_from_shapes: NULL argument");
  if (!(M > 0.0)) return fail(XRL_ERR_VALUE, "the normalisation constant M must be positive");
  if (shape_ptr[0] != 0) return fail(XRL_ERR_SHAPE, "shape_ptr[0] must be 0");
  for (int64_t e = 0; e < n_edges; ++e) {
    const int64_t r = (int64_t)shape_ptr[e + 1] - shape_ptr[e];
    if (r < 0 || r > 4)
      return fail(XRL_ERR_SHAPE, "edge %lld: rank %lld outside [0, 4]", (long long)e, (long long)r);
    if (r > 0 && !dims) return fail(XRL_ERR_NULL, "xrl_edge_features_from_shapes: dims is NULL");
    float *o = edge_feat + 4 * e;
    for (int k = 0; k < 4; ++k) o[k] = 0.0f;                  // leading dimensions padded with zeros
    for (int64_t k = 0; k < r; ++k) {
      const int64_t d = dims[shape_ptr[e] + k];
      if (d < 0) return fail(XRL_ERR_VALUE, "edge %lld: negative extent %lld", (long long)e, (long long)d);
      o[4 - r + k] = (float)((double)d / M);
    }
  }
  return XRL_OK;
}

int xrl_batch_dims(const xrl_batch *b, int64_t *S, int64_t *G, int64_t *N, int64_t *E) {
  if (!b) return fail(XRL_ERR_NULL, "xrl_batch_dims: batch is NULL");
  if (S) *S = b->S;
  if (G) *G = b->G;
  if (N) *N = b->N;
  if (E) *E = b->E;
  return XRL_OK;
}

int xrl_batch_host_view(const xrl_batch *b, xrl_packed_view *v) {
  if (!b || !v) return fail(XRL_ERR_NULL, "xrl_batch_host_view: NULL argument");
  v->S = b->S; v->G = b->G; v->N = b->N; v->E = b->E;
  v->state_graph_ptr = b->state_graph_ptr.data();
  v->graph_node_ptr = b->graph_node_ptr.data();
  v->in_ptr = b->in_ptr.data();
  v->in_src = b->in_src.data();
  v->in_dst = b->in_dst.data();
  v->in_eid = b->in_eid.data();
  v->out_ptr = b->out_ptr.data();
  v->out_pos = b->out_pos.data();
  v->node_graph = b->node_graph.data();
  v->edge_feat = b->edge_feat.data();
  v->n_tiles = (int64_t)b->tile_ptr.size() - 1;
  v->tile_ptr = b->tile_ptr.data();
  v->n_graph_tiles = b->gtile_ptr.empty() ? 0 : (int64_t)b->gtile_ptr.size() - 1;
  v->graph_tile_ptr = b->graph_tile_ptr.empty() ? nullptr : b->graph_tile_ptr.data();
  v->gtile_ptr = b->gtile_ptr.empty() ? nullptr : b->gtile_ptr.data();
  return XRL_OK;
}

int xrl_batch_free(xrl_batch *b) {
  if (!b) return XRL_OK;
  xrl_batch_release_device(b);
  delete b;
  return XRL_OK;
}

}  // extern "C"
