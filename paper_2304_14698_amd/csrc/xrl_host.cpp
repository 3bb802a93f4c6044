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

// Edge tiles of the message kernels and the per-graph tiles of the one-launch encoder, from the
// packed in_ptr / graph_node_ptr (serial: a tile boundary depends on the ones before it).
void build_tile_tables(xrl_batch *b) {
  const int64_t N = b->N, E = b->E, G = b->G;
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
    build_tile_tables(b);
  } catch (const std::bad_alloc &) {
    delete b;
    return fail(XRL_ERR_OOM, "xrl_pack_state: out of host memory");
  }
  *out = b;
  return XRL_OK;
}

int xrl_pack_state_edits(const xrl_model_desc *model, const xrl_edit_state_desc *st, xrl_batch **out) {
  if (!model || !st || !out) return fail(XRL_ERR_NULL, "xrl_pack_state_edits: NULL argument");
  *out = nullptr;
  Layout L;
  int rc = build_layout(*model, L);
  if (rc) return rc;
  const int64_t S = st->n_states;
  if (S < 0) return fail(XRL_ERR_SHAPE, "n_states = %lld is negative", (long long)S);
  if (!st->cur_node_ptr || !st->cur_edge_ptr || !st->state_cand_ptr || !st->del_node_ptr || !st->del_edge_ptr ||
      !st->add_node_ptr || !st->add_edge_ptr || !st->slot_mask)
    return fail(XRL_ERR_NULL, "xrl_pack_state_edits: a ptr array or slot_mask is NULL");
  if ((rc = check_ptr(st->cur_node_ptr, S, "cur_node_ptr"))) return rc;
  if ((rc = check_ptr(st->cur_edge_ptr, S, "cur_edge_ptr"))) return rc;
  if ((rc = check_ptr(st->state_cand_ptr, S, "state_cand_ptr"))) return rc;
  const int64_t C = st->state_cand_ptr[S], G = S + C;
  if ((rc = check_ptr(st->del_node_ptr, C, "del_node_ptr"))) return rc;
  if ((rc = check_ptr(st->del_edge_ptr, C, "del_edge_ptr"))) return rc;
  if ((rc = check_ptr(st->add_node_ptr, C, "add_node_ptr"))) return rc;
  if ((rc = check_ptr(st->add_edge_ptr, C, "add_edge_ptr"))) return rc;
  const int64_t Nc = st->cur_node_ptr[S], Ec = st->cur_edge_ptr[S];
  const int64_t n_dn = st->del_node_ptr[C], n_de = st->del_edge_ptr[C], n_an = st->add_node_ptr[C], n_ae = st->add_edge_ptr[C];
  const int Dd = model->n_node_dense, De = model->d_edge, Dg = model->d_global;
  if (Nc > 0 && (!st->node_op || (Dd > 0 && !st->node_dense))) return fail(XRL_ERR_NULL, "node_op or node_dense is NULL");
  if (Ec > 0 && (!st->edge_src || !st->edge_dst || !st->edge_feat))
    return fail(XRL_ERR_NULL, "edge_src, edge_dst or edge_feat is NULL");
  if ((n_dn > 0 && !st->del_node) || (n_de > 0 && !st->del_edge) || (n_an > 0 && (!st->add_node_op || (Dd > 0 && !st->add_node_dense))) ||
      (n_ae > 0 && (!st->add_edge_src || !st->add_edge_dst || !st->add_edge_feat)))
    return fail(XRL_ERR_NULL, "xrl_pack_state_edits: an edit array is NULL");
  // graph g of the batch: state s's current graph, or candidate c
  std::vector<int32_t> sgp(S + 1), g_state(G), g_cand(G);
  for (int64_t s = 0, g = 0; s < S; ++s) {
    sgp[s] = (int32_t)g;
    g_state[g] = (int32_t)s; g_cand[g] = -1; ++g;
    for (int32_t c = st->state_cand_ptr[s]; c < st->state_cand_ptr[s + 1]; ++c, ++g) { g_state[g] = (int32_t)s; g_cand[g] = c; }
    sgp[s + 1] = (int32_t)g;
  }
  for (int64_t s = 0; s < S; ++s)
    if (st->slot_mask[sgp[s]] == 0) return fail(XRL_ERR_MASK, "state %lld masks its No-Op slot (its first graph)", (long long)s);
  // ---- the current graphs and the new items (what is validated; everything else is copied from them)
  for (int64_t i = 0; i < Nc; ++i)
    if (st->node_op[i] < 0 || st->node_op[i] >= model->n_op_types)
      return fail(XRL_ERR_INDEX, "node %lld: op id %d outside [0, %d)", (long long)i, st->node_op[i], model->n_op_types);
  for (int64_t i = 0; i < n_an; ++i)
    if (st->add_node_op[i] < 0 || st->add_node_op[i] >= model->n_op_types)
      return fail(XRL_ERR_INDEX, "new node %lld: op id %d outside [0, %d)", (long long)i, st->add_node_op[i], model->n_op_types);
  for (int64_t s = 0; s < S; ++s) {
    const int32_t n = st->cur_node_ptr[s + 1] - st->cur_node_ptr[s];
    for (int64_t e = st->cur_edge_ptr[s]; e < st->cur_edge_ptr[s + 1]; ++e)
      if (st->edge_src[e] < 0 || st->edge_src[e] >= n || st->edge_dst[e] < 0 || st->edge_dst[e] >= n)
        return fail(XRL_ERR_INDEX, "edge %lld of state %lld's current graph: endpoint (%d -> %d) outside [0, %d)", (long long)e,
                    (long long)s, st->edge_src[e], st->edge_dst[e], n);
  }
  int64_t where = 0;
  if (Dd > 0 && !all_finite(st->node_dense, Nc * Dd, &where)) return fail(XRL_ERR_VALUE, "node_dense[%lld] is not finite", (long long)where);
  if (Dd > 0 && !all_finite(st->add_node_dense, n_an * Dd, &where)) return fail(XRL_ERR_VALUE, "add_node_dense[%lld] is not finite", (long long)where);
  if (!all_finite(st->edge_feat, Ec * De, &where)) return fail(XRL_ERR_VALUE, "edge_feat[%lld] is not finite", (long long)where);
  if (!all_finite(st->add_edge_feat, n_ae * De, &where)) return fail(XRL_ERR_VALUE, "add_edge_feat[%lld] is not finite", (long long)where);
  if (st->graph_global && !all_finite(st->graph_global, G * Dg, &where)) return fail(XRL_ERR_VALUE, "graph_global[%lld] is not finite", (long long)where);
  // ---- the edits, and the size of every graph
  std::vector<int32_t> gnp(G + 1, 0), gep(G + 1, 0);
  {
    std::vector<uint8_t> dead;                     // per node of the state's current graph
    for (int64_t g = 0; g < G; ++g) {
      const int64_t s = g_state[g];
      const int32_t n = st->cur_node_ptr[s + 1] - st->cur_node_ptr[s];
      const int64_t e0 = st->cur_edge_ptr[s], e1 = st->cur_edge_ptr[s + 1];
      if (g_cand[g] < 0) { gnp[g + 1] = n; gep[g + 1] = (int32_t)(e1 - e0); continue; }
      const int64_t c = g_cand[g];
      dead.assign(n, 0);
      for (int32_t k = st->del_node_ptr[c]; k < st->del_node_ptr[c + 1]; ++k) {
        const int32_t v = st->del_node[k];
        if (v < 0 || v >= n || (k > st->del_node_ptr[c] && v <= st->del_node[k - 1]))
          return fail(XRL_ERR_INDEX, "candidate %lld: del_node[%d] = %d out of range or not ascending", (long long)c, k, v);
        dead[v] = 1;
      }
      int32_t kept = 0;
      int32_t kd = st->del_edge_ptr[c];
      const int32_t kd1 = st->del_edge_ptr[c + 1];
      for (int32_t k = kd; k < kd1; ++k) {
        const int32_t v = st->del_edge[k];
        if (v < 0 || v >= e1 - e0 || (k > kd && v <= st->del_edge[k - 1]))
          return fail(XRL_ERR_INDEX, "candidate %lld: del_edge[%d] = %d out of range or not ascending", (long long)c, k, v);
      }
      for (int64_t e = e0; e < e1; ++e) {
        if (kd < kd1 && st->del_edge[kd] == e - e0) { ++kd; continue; }
        if (!dead[st->edge_src[e]] && !dead[st->edge_dst[e]]) ++kept;
      }
      const int32_t n_new = st->add_node_ptr[c + 1] - st->add_node_ptr[c];
      for (int32_t k = st->add_edge_ptr[c]; k < st->add_edge_ptr[c + 1]; ++k)
        for (const int32_t v : {st->add_edge_src[k], st->add_edge_dst[k]})
          if (v < 0 || v >= n + n_new || (v < n && dead[v]))
            return fail(XRL_ERR_INDEX, "candidate %lld: new edge %d has endpoint %d outside its graph or on a deleted node", (long long)c, k, v);
      gnp[g + 1] = n - (st->del_node_ptr[c + 1] - st->del_node_ptr[c]) + n_new;
      gep[g + 1] = kept + (st->add_edge_ptr[c + 1] - st->add_edge_ptr[c]);
    }
    int64_t nn = 0, ee = 0;
    for (int64_t g = 0; g < G; ++g) {
      nn += gnp[g + 1]; ee += gep[g + 1];
      if (nn > INT32_MAX || ee > INT32_MAX) return fail(XRL_ERR_SHAPE, "the batch has more than 2^31 - 1 nodes or edges");
      gnp[g + 1] = (int32_t)nn; gep[g + 1] = (int32_t)ee;
    }
  }
  const int64_t N = gnp[G], E = gep[G];

  xrl_batch *b = new (std::nothrow) xrl_batch();
  if (!b) return fail(XRL_ERR_OOM, "xrl_pack_state_edits: out of host memory");
  try {
    static std::atomic<uint64_t> next_id{(uint64_t)1 << 62};
    b->id = next_id++;
    b->model = *model;
    b->S = S; b->G = G; b->N = N; b->E = E;
    b->from_edits = true;
    b->state_graph_ptr = sgp;
    b->graph_node_ptr = gnp;
    b->mask.resize(G);
    for (int64_t g = 0; g < G; ++g) b->mask[g] = st->slot_mask[g] ? 1 : 0;
    if (st->graph_global) b->graph_global.assign(st->graph_global, st->graph_global + G * Dg);
    else b->graph_global.assign((size_t)(G * Dg), 0.0f);
    for (int64_t s = 0; s < S; ++s) b->max_slots = std::max(b->max_slots, sgp[s + 1] - sgp[s]);
    // (node_op, node_dense and edge_feat of the batch are not written here: the device fills its
    // copies from node_from / edge_from, and xrl_batch_host_view fills the host's on demand)
    b->node_graph.resize(N);
    b->in_ptr.assign(N + 1, 0); b->out_ptr.assign(N + 1, 0);
    b->in_src.resize(E); b->in_dst.resize(E); b->in_eid.resize(E); b->out_pos.resize(E);
    b->node_from.resize(N); b->edge_from.resize(E);
    b->base_node_op.assign(st->node_op, st->node_op + Nc);
    b->base_node_dense.assign(st->node_dense, st->node_dense + (Dd > 0 ? Nc * Dd : 0));
    b->base_edge_feat.assign(st->edge_feat, st->edge_feat + Ec * De);
    b->new_node_op.assign(st->add_node_op, st->add_node_op + n_an);
    b->new_node_dense.assign(st->add_node_dense, st->add_node_dense + (Dd > 0 ? n_an * Dd : 0));
    b->new_edge_feat.assign(st->add_edge_feat, st->add_edge_feat + n_ae * De);
    // ---- the current graph of every state in receiver order once: its in-edge lists (edge ids
    // ascending inside a receiver's list, i.e. the stable order)
    std::vector<int32_t> bin_ptr(Nc + S + 1, 0), bin_eid(Ec);
    for (int64_t s = 0; s < S; ++s) {
      const int32_t nb = st->cur_node_ptr[s], n = st->cur_node_ptr[s + 1] - nb;
      const int64_t e0 = st->cur_edge_ptr[s], e1 = st->cur_edge_ptr[s + 1];
      int32_t *ip = bin_ptr.data() + nb + s;          // [n + 1] of this state
      for (int64_t e = e0; e < e1; ++e) ip[st->edge_dst[e] + 1]++;
      for (int32_t i = 0; i < n; ++i) ip[i + 1] += ip[i];
      std::vector<int32_t> cur(ip, ip + n);
      for (int64_t e = e0; e < e1; ++e) bin_eid[e0 + cur[st->edge_dst[e]]++] = (int32_t)(e - e0);
    }
    // ---- every graph by merging; graph ranges on separate threads
    const int T = pack_thread_count(N + E);
    std::vector<int64_t> cut(T + 1, G);
    cut[0] = 0;
    for (int t = 1, g = 0; t < T; ++t) {
      const int64_t want = (N + E) * t / T;
      while (g < G && (int64_t)gnp[g] + gep[g] < want) ++g;
      cut[t] = g;
    }
    const bool merged = run_ranges(cut, [&](int, int64_t g0, int64_t g1) {
      std::vector<int32_t> newid, erank, cur, add_order;
      std::vector<uint8_t> dead;
      for (int64_t g = g0; g < g1; ++g) {
        const int64_t s = g_state[g], c = g_cand[g];
        const int32_t nb = st->cur_node_ptr[s], n = st->cur_node_ptr[s + 1] - nb;
        const int64_t e0 = st->cur_edge_ptr[s], e1 = st->cur_edge_ptr[s + 1];
        const int32_t *ip = bin_ptr.data() + nb + s;
        const int32_t base = gnp[g], ng = gnp[g + 1] - base, eb = gep[g];
        const int32_t an0 = c < 0 ? 0 : st->add_node_ptr[c], n_new = c < 0 ? 0 : st->add_node_ptr[c + 1] - an0;
        const int32_t ae0 = c < 0 ? 0 : st->add_edge_ptr[c], n_ae_c = c < 0 ? 0 : st->add_edge_ptr[c + 1] - ae0;
        // surviving nodes -> new ids; surviving edges -> rank in the candidate's edge list
        dead.assign(n, 0);
        if (c >= 0)
          for (int32_t k = st->del_node_ptr[c]; k < st->del_node_ptr[c + 1]; ++k) dead[st->del_node[k]] = 1;
        newid.assign(n + n_new, -1);
        int32_t nk = 0;
        for (int32_t i = 0; i < n; ++i)
          if (!dead[i]) newid[i] = nk++;
        for (int32_t k = 0; k < n_new; ++k) newid[n + k] = nk + k;
        erank.assign(e1 - e0, -1);
        int32_t ek = 0;
        {
          int32_t kd = c < 0 ? 0 : st->del_edge_ptr[c];
          const int32_t kd1 = c < 0 ? 0 : st->del_edge_ptr[c + 1];
          for (int64_t e = e0; e < e1; ++e) {
            if (kd < kd1 && st->del_edge[kd] == e - e0) { ++kd; continue; }
            if (!dead[st->edge_src[e]] && !dead[st->edge_dst[e]]) erank[e - e0] = ek++;
          }
        }
        // new edges grouped by receiver, in their own order inside a group
        add_order.resize(n_ae_c);
        for (int32_t k = 0; k < n_ae_c; ++k) add_order[k] = k;
        std::stable_sort(add_order.begin(), add_order.end(), [&](int32_t x, int32_t y) {
          return newid[st->add_edge_dst[ae0 + x]] < newid[st->add_edge_dst[ae0 + y]];
        });
        // nodes
        for (int32_t i = 0; i < n; ++i) {
          if (dead[i]) continue;
          const int32_t v = base + newid[i];
          b->node_graph[v] = (int32_t)g;
          b->node_from[v] = nb + i;
        }
        for (int32_t k = 0; k < n_new; ++k) {
          const int32_t v = base + nk + k;
          b->node_graph[v] = (int32_t)g;
          b->node_from[v] = -1 - (an0 + k);
        }
        // receiver order: per receiver its surviving in-edges (edge ids ascending), then its new ones
        int32_t p = eb, ka = 0;
        int32_t *inp = b->in_ptr.data() + base + 1, *outp = b->out_ptr.data() + base + 1;
        int32_t vcur = 0;
        for (int32_t i = 0; i < n + n_new; ++i) {
          if (i < n && dead[i]) continue;
          const int32_t v = vcur++;                  // == newid[i]
          if (i < n) {
            for (int32_t q = ip[i]; q < ip[i + 1]; ++q) {
              const int32_t el = bin_eid[e0 + q];
              if (erank[el] < 0) continue;
              const int64_t e = e0 + el;
              b->in_src[p] = base + newid[st->edge_src[e]];
              b->in_dst[p] = base + v;
              b->in_eid[p] = eb + erank[el];
              b->edge_from[p] = (int32_t)e;
              ++p;
            }
          }
          for (; ka < n_ae_c && newid[st->add_edge_dst[ae0 + add_order[ka]]] == v; ++ka) {
            const int32_t k = ae0 + add_order[ka];
            b->in_src[p] = base + newid[st->add_edge_src[k]];
            b->in_dst[p] = base + v;
            b->in_eid[p] = eb + ek + add_order[ka];
            b->edge_from[p] = -1 - k;
            ++p;
          }
          inp[v] = p;                                // end of v's in-edges
        }
        // sender-side index: receiver-order positions grouped by sender, ascending position
        for (int32_t v = 0; v < ng; ++v) outp[v] = 0;
        for (int32_t q = eb; q < p; ++q) outp[b->in_src[q] - base]++;
        cur.assign(ng, 0);
        int32_t ro = eb;
        for (int32_t v = 0; v < ng; ++v) { cur[v] = ro; ro += outp[v]; outp[v] = ro; }
        for (int32_t q = eb; q < p; ++q) b->out_pos[cur[b->in_src[q] - base]++] = q;
      }
    });
    if (!merged) throw std::bad_alloc();
    build_tile_tables(b);
  } catch (const std::bad_alloc &) {
    delete b;
    return fail(XRL_ERR_OOM, "xrl_pack_state_edits: out of host memory");
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

int xrl_batch_host_view(const xrl_batch *cb, xrl_packed_view *v) {
  if (!cb || !v) return fail(XRL_ERR_NULL, "xrl_batch_host_view: NULL argument");
  xrl_batch *b = const_cast<xrl_batch *>(cb);
  if (b->from_edits && b->edge_feat.size() != (size_t)b->E * b->model.d_edge) {
    // packed from edits: the per-edge attribute rows are written out on first request
    const int De = b->model.d_edge;
    try {
      b->edge_feat.resize((size_t)b->E * De);
    } catch (const std::bad_alloc &) {
      return fail(XRL_ERR_OOM, "xrl_batch_host_view: out of host memory");
    }
    for (int64_t p = 0; p < b->E; ++p) {
      const int32_t f = b->edge_from[p];
      const float *src = f >= 0 ? &b->base_edge_feat[(size_t)f * De] : &b->new_edge_feat[(size_t)(-1 - f) * De];
      memcpy(&b->edge_feat[(size_t)p * De], src, sizeof(float) * De);
    }
  }
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
