// Internal declarations shared by the host-side packer and the device-side runtime.
#pragma once
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <memory>
#include <string>
#include <vector>

#include "xrl.h"

namespace xrl {

void set_error(const char *fmt, ...);
int fail(int code, const char *fmt, ...);

// One tensor of the flat weight vector (order documented in xrl.h).
struct WeightTensor {
  std::string name;
  int64_t offset, rows, cols;  // cols == 0 for a bias vector of length rows
};

// Offsets of one MLP inside the flat vector: per layer (W offset, b offset, in, out).
struct MlpRef {
  int n_layers = 0;
  int64_t w[3] = {0, 0, 0}, b[3] = {0, 0, 0};
  int32_t d_in[3] = {0, 0, 0}, d_out[3] = {0, 0, 0};
};

struct Layout {
  std::vector<WeightTensor> tensors;
  int64_t total = 0;
  MlpRef embed, readout, policy, value;
  std::vector<MlpRef> edge, node;  // per round (XRL_ROUND_MLP)
  struct GatRef { int64_t W = 0, a_src = 0, a_dst = 0; };
  std::vector<GatRef> gat;         // per round (XRL_ROUND_GAT)
};

// Validates the dimensions that every part of the library relies on (positive widths, ...)
// and fills the layout. Returns XRL_OK or an error code (message set).
int build_layout(const xrl_model_desc &m, Layout &out);

}  // namespace xrl

// Allocator whose resize() leaves new trivially-constructible elements uninitialised: the packed
// arrays are written in full by the packing threads, which then also take their page faults.
template <typename T>
struct RawAlloc : std::allocator<T> {
  template <typename U> struct rebind { typedef RawAlloc<U> other; };
  RawAlloc() = default;
  template <typename U> RawAlloc(const RawAlloc<U> &) {}
  template <typename U> void construct(U *p) { ::new ((void *)p) U; }              // default-init: no write
  template <typename U, typename... A> void construct(U *p, A &&...a) { ::new ((void *)p) U(std::forward<A>(a)...); }
};
template <typename T> using RawVec = std::vector<T, RawAlloc<T>>;

// Device-side copies of a packed batch (all owned by one hipMalloc block).
struct xrl_batch_device {
  void *block = nullptr;
  size_t bytes = 0;
  int32_t *state_graph_ptr = nullptr, *graph_node_ptr = nullptr, *node_op = nullptr;
  int32_t *in_ptr = nullptr, *in_src = nullptr, *in_dst = nullptr;
  int32_t *out_ptr = nullptr, *out_pos = nullptr, *node_graph = nullptr, *tile_ptr = nullptr;
  int32_t *gtile_ptr = nullptr, *graph_tile_ptr = nullptr;   // null unless the batch has per-graph tiles
  int32_t *agg_src = nullptr;   // [N] n for a node with in-edges, -1 for one without (filled on the device)
  float *node_dense = nullptr, *edge_feat = nullptr, *graph_global = nullptr;
  uint8_t *mask = nullptr;
};

struct xrl_batch {
  xrl_model_desc model;
  int64_t S = 0, G = 0, N = 0, E = 0;
  int32_t max_slots = 0;  // largest number of slots in one state
  std::vector<int32_t> state_graph_ptr, graph_node_ptr, in_ptr, out_ptr;
  RawVec<int32_t> node_op, in_src, in_dst, in_eid, out_pos, node_graph;
  std::vector<int32_t> tile_ptr;  // [n_tiles + 1] edge tiles of the message kernels (see the packer)
  int64_t n_split_tiles = 0;      // tiles that end inside a receiver's in-edge range
  // Per-graph edge tiles for the one-launch encoder of small batches: the same cutting rule, but
  // a tile never spans two graphs; graph g owns tiles [graph_tile_ptr[g], graph_tile_ptr[g + 1])
  // of gtile_ptr. Both empty when the batch has more than kGraphTileMaxGraphs graphs or a node
  // with more than 32 in-edges.
  std::vector<int32_t> gtile_ptr, graph_tile_ptr;
  int32_t max_graph_nodes = 0;    // nodes of the largest graph
  int32_t max_graph_tiles = 0;    // most per-graph edge tiles of one graph
  RawVec<float> node_dense, edge_feat;
  std::vector<float> graph_global;
  std::vector<uint8_t> mask;
  // Batches packed from edits (xrl_pack_state_edits): where each node's and each receiver-order
  // edge's attributes come from -- an index into the current graphs' arrays (>= 0) or, as -1 - k,
  // into the new nodes' / edges' arrays -- and those compact attribute arrays. Empty otherwise.
  RawVec<int32_t> node_from, edge_from;
  RawVec<int32_t> base_node_op, new_node_op;
  RawVec<float> base_node_dense, new_node_dense, base_edge_feat, new_edge_feat;
  bool from_edits = false;
  xrl_batch_device dev;
  bool uploaded = false;
  uint64_t id = 0;  // unique per packed batch; ties saved activations to their batch
};

constexpr int64_t kGraphTileMaxGraphs = 4096;

// Implemented in the device translation unit; frees dev.block if any.
extern "C" void xrl_batch_release_device(xrl_batch *b);
