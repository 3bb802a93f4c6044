/*
 * xrl.h -- C ABI of the MI355X state encoder for graph-rewrite reinforcement learning
 * (X-RLflow, arXiv 2304.14698).
 *
 * A state is the current computation graph plus every candidate graph produced by an applicable
 * rewrite rule; the action picks one candidate or No-Op (Section 3.3.2). The library batches all
 * graphs of one or many states into one meta-graph, embeds every graph with the three-stage GNN
 * of Section 3.4 and evaluates the policy head (masked categorical over slots) and the value head
 * of Section 3.3.2, forward and backward (one back-propagation through heads and GNN, Section
 * 3.3.4).
 *
 * Conventions
 *   - "host" pointers are ordinary CPU memory, borrowed for the duration of the call only.
 *   - "device" pointers are GPU memory owned by the caller (any HIP allocation, e.g. a torch
 *     tensor's data_ptr); the library never frees or resizes them.
 *   - Every GPU call is enqueued on the HIP stream given to xrl_create and returns without
 *     synchronising; outputs are valid once that stream has reached the call.
 *   - Every function returns XRL_OK (0) or a negative xrl_status; it never aborts or throws. After
 *     an error no output may be trusted. xrl_last_error() gives a message for the calling thread.
 *   - All matrices are row-major; an affine layer is y = x W + b with W stored [in, out].
 */
#ifndef XRL_H
#define XRL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  XRL_OK = 0,
  XRL_ERR_NULL = -1,        /* a required pointer is NULL */
  XRL_ERR_SHAPE = -2,       /* negative count, non-monotone or inconsistent ptr array, misaligned buffer */
  XRL_ERR_INDEX = -3,       /* edge endpoint outside its graph, op id outside [0, n_op_types) */
  XRL_ERR_VALUE = -4,       /* NaN or Inf in a feature or weight */
  XRL_ERR_MASK = -5,        /* a state's No-Op slot (its first graph) is masked out */
  XRL_ERR_STATE = -6,       /* call order: batch not uploaded, backward without saved forward */
  XRL_ERR_UNSUPPORTED = -7, /* model dimensions the kernels do not cover */
  XRL_ERR_OOM = -8,         /* host or device allocation failed */
  XRL_ERR_HIP = -9          /* a HIP runtime call failed (no usable GPU, launch error) */
} xrl_status;

enum { XRL_READOUT_SUM = 0, XRL_READOUT_MEAN = 1 };
enum { XRL_ROUND_MLP = 0, XRL_ROUND_GAT = 1 };
enum { XRL_PREC_FP32 = 0,      /* fp32 operands, fp32 accumulate                              */
       XRL_PREC_BF16 = 1 };    /* bf16 MFMA operands (weights, stored activations), fp32
                                  accumulate, bias, ReLU, segment sums, readout and heads     */

/* Model dimensions. Encoder (Section 3.4): node-update layer, `rounds` message-passing layers
 * (k = 5 in the paper's appendix), global-update layer; every learned transform is an MLP of
 * `mlp_layers` affine layers, ReLU after each. Heads (Section 3.3.2): hidden sizes head_hidden
 * ([256, 64] in the appendix) with ReLU, then a linear output of width 1. */
typedef struct xrl_model_desc {
  int32_t n_op_types;     /* T: width of the one-hot operator attribute                       */
  int32_t n_node_dense;   /* extra dense node attributes after the one-hot (may be 0)         */
  int32_t d_edge;         /* edge attribute width (tensor-shape attributes)                    */
  int32_t d_global;       /* global attribute width (initialised to 0 by the paper)           */
  int32_t hidden;         /* H: 64, 128 or 256                                                */
  int32_t rounds;         /* number of message-passing layers, >= 0                           */
  int32_t mlp_layers;     /* affine layers per encoder transform; the GPU path supports 1, 2  */
  int32_t head_hidden[2];
  int32_t readout;        /* XRL_READOUT_SUM (the paper's sum) or XRL_READOUT_MEAN            */
  int32_t precision;      /* XRL_PREC_FP32 or XRL_PREC_BF16                                   */
  int32_t round_kind;     /* XRL_ROUND_MLP, or XRL_ROUND_GAT: the graph-attention reading of
                             the message-passing layers (Section 3.4, second equation): z = h W,
                             s = LeakyReLU_0.2(a_src.z_sender + a_dst.z_receiver), softmax over a
                             receiver's in-edges plus a self edge, h' = ReLU(sum alpha z)        */
} xrl_model_desc;

/* One or many states, all host memory. Graphs are listed state by state; the first graph of a
 * state is the current graph and doubles as the No-Op slot, the others are its candidates
 * (Section 3.3.2). Edge endpoints are node indices local to the edge's graph; edges may come in
 * any order; multi-edges and cycles are accepted. */
typedef struct xrl_state_desc {
  int32_t n_states;
  const int32_t *state_graph_ptr; /* [S+1] graph range of each state, starts at 0             */
  const int32_t *graph_node_ptr;  /* [G+1] node range of each graph, starts at 0              */
  const int32_t *graph_edge_ptr;  /* [G+1] edge range of each graph, starts at 0              */
  const int32_t *node_op;         /* [N] operator id                                          */
  const float *node_dense;        /* [N, n_node_dense] (NULL allowed if n_node_dense == 0)    */
  const int32_t *edge_src;        /* [E] sender, local index                                  */
  const int32_t *edge_dst;        /* [E] receiver, local index                                */
  const float *edge_feat;         /* [E, d_edge]                                              */
  const float *graph_global;      /* [G, d_global] or NULL for zeros                          */
  const uint8_t *slot_mask;       /* [G] 1 = slot may be chosen; each state's first must be 1 */
} xrl_state_desc;

/* The same states with every candidate given as an edit of its state's current graph (Section
 * 3.3.2: a candidate is the current graph with one rewrite rule applied, i.e. a local change of a
 * few nodes). All host memory. Per state: the current graph in full (node and edge arrays as in
 * xrl_state_desc, ranges cur_node_ptr / cur_edge_ptr) and its candidates [state_cand_ptr[s],
 * state_cand_ptr[s+1]); per candidate c:
 *   del_node[del_node_ptr[c] ..)  nodes of the current graph that disappear (local ids, strictly
 *                                 ascending); their edges disappear with them
 *   del_edge[del_edge_ptr[c] ..)  further edges of the current graph that disappear (indices into
 *                                 the current graph's own edge list, strictly ascending)
 *   add_node_*[add_node_ptr[c] ..) new nodes
 *   add_edge_*[add_edge_ptr[c] ..) new edges; an endpoint is a node id of the current graph (which
 *                                 must survive) or n_current + k for the candidate's k-th new node
 * The candidate graph this stands for: the surviving nodes of the current graph in their order,
 * then the new nodes; the surviving edges in their order, then the new edges. Graphs are listed
 * as in xrl_state_desc (per state: current graph, then its candidates), which is the order of
 * graph_global and slot_mask, G = n_states + number of candidates. */
typedef struct xrl_edit_state_desc {
  int32_t n_states;
  const int32_t *cur_node_ptr;    /* [S+1] node range of each state's current graph, starts at 0 */
  const int32_t *cur_edge_ptr;    /* [S+1] edge range of each state's current graph, starts at 0 */
  const int32_t *node_op;         /* current graphs: [Nc] operator id                            */
  const float *node_dense;        /* [Nc, n_node_dense]                                          */
  const int32_t *edge_src;        /* [Ec] sender, local to the current graph                     */
  const int32_t *edge_dst;        /* [Ec] receiver                                               */
  const float *edge_feat;         /* [Ec, d_edge]                                                */
  const int32_t *state_cand_ptr;  /* [S+1] candidate range of each state, starts at 0            */
  const int32_t *del_node_ptr;    /* [C+1] */
  const int32_t *del_node;
  const int32_t *del_edge_ptr;    /* [C+1] */
  const int32_t *del_edge;
  const int32_t *add_node_ptr;    /* [C+1] */
  const int32_t *add_node_op;
  const float *add_node_dense;    /* [total new nodes, n_node_dense]                             */
  const int32_t *add_edge_ptr;    /* [C+1] */
  const int32_t *add_edge_src;
  const int32_t *add_edge_dst;
  const float *add_edge_feat;     /* [total new edges, d_edge]                                   */
  const float *graph_global;      /* [S + C, d_global] or NULL for zeros                         */
  const uint8_t *slot_mask;       /* [S + C] 1 = slot may be chosen; each state's first must be 1 */
} xrl_edit_state_desc;

/* Read-only view of a packed batch's host arrays (valid until xrl_batch_free). Edges are stored
 * sorted by global receiver id, ties in input order ("receiver order"). */
typedef struct xrl_packed_view {
  int64_t S, G, N, E;
  const int32_t *state_graph_ptr; /* [S+1]                                                    */
  const int32_t *graph_node_ptr;  /* [G+1] global node offsets                                */
  const int32_t *in_ptr;          /* [N+1] receiver-order edge range of each receiver         */
  const int32_t *in_src;          /* [E] global sender id, receiver order                     */
  const int32_t *in_dst;          /* [E] global receiver id, receiver order (non-decreasing)  */
  const int32_t *in_eid;          /* [E] index of the edge in the caller's edge arrays        */
  const int32_t *out_ptr;         /* [N+1] out-edge range of each sender                      */
  const int32_t *out_pos;         /* [E] receiver-order position of each out-edge, by sender  */
  const int32_t *node_graph;      /* [N] graph id of each node                                */
  const float *edge_feat;         /* [E, d_edge] in receiver order                            */
  int64_t n_tiles;                /* edge tiles of the message kernels                        */
  const int32_t *tile_ptr;        /* [n_tiles+1] first receiver-order edge of each tile: 1..32
                                     edges per tile, cut at receiver boundaries except inside a
                                     receiver with more than 32 in-edges                      */
  int64_t n_graph_tiles;          /* per-graph tiles for the one-launch encoder of small
                                     batches, 0 when the batch has none (more than 4096 graphs,
                                     or a node with more than 32 in-edges)                     */
  const int32_t *graph_tile_ptr;  /* [G+1] graph g owns tiles [graph_tile_ptr[g], [g+1])      */
  const int32_t *gtile_ptr;       /* [n_graph_tiles+1] first edge of each: the same cutting
                                     rule, and no tile spans two graphs                        */
} xrl_packed_view;

typedef struct xrl_ctx xrl_ctx;     /* device weights + workspaces, bound to one HIP stream    */
typedef struct xrl_batch xrl_batch; /* one packed meta-batch (host copy + device copy)         */

/* ---- weights -------------------------------------------------------------------------------
 * One flat fp32 vector. Tensor order: embed MLP (input [sum of incoming edge attrs | one-hot op
 * | dense attrs], the node-update layer of Section 3.4); per round r: edge MLP (input [h_sender |
 * h_receiver | edge attrs]) then node MLP (input [h | received sum]) (message-passing layers of
 * Section 3.4); readout MLP (input [sum or mean of node states | global attrs], the global-update
 * layer); policy head; value head (Section 3.3.2). Each MLP lists, per layer, W [in, out] then
 * b [out]. With XRL_ROUND_GAT a round instead lists W [hidden, hidden], a_src [hidden], a_dst
 * [hidden] ("gat3.W", "gat3.a_src", "gat3.a_dst"). */
int64_t xrl_weight_count(const xrl_model_desc *model);        /* total floats, <0 on error     */
int32_t xrl_weight_tensor_count(const xrl_model_desc *model); /* number of tensors, <0 on error */
/* Tensor `index`: name (e.g. "edge3.W0") copied into name[name_cap]; vectors report cols = 0. */
int xrl_weight_tensor(const xrl_model_desc *model, int32_t index, char *name, size_t name_cap,
                      int64_t *offset, int64_t *rows, int64_t *cols);

/* ---- packing (host only; never touches the GPU) ---------------------------------------------
 * Batches current + candidate graphs into one meta-graph with its slot mask (Section 3.3.2):
 * validates, converts endpoints to global node ids, sorts edges by receiver (stable) and builds
 * the sender-side index. Errors: NULL, SHAPE, INDEX, VALUE (non-finite attribute), MASK. */
int xrl_pack_state(const xrl_model_desc *model, const xrl_state_desc *state, xrl_batch **out);
/* xrl_pack_state_edits: the same packed batch as xrl_pack_state on the candidate graphs the edits
 * stand for (every array of xrl_batch_host_view identical; in_eid counts edges in the order stated
 * above), built from the current graph's receiver-ordered edge lists by merging instead of
 * sorting every candidate from scratch; only the current graphs and the edits are validated.
 * xrl_batch_upload of such a batch sends the attributes of the current graphs and of the new
 * nodes and edges once, plus one index per node and edge, and a kernel fills the per-node and
 * per-edge attribute arrays on the device (about half the bytes of the plain upload).
 * Errors: NULL, SHAPE, INDEX (an id out of range, not ascending, an endpoint on a deleted node),
 * VALUE, MASK, OOM. */
int xrl_pack_state_edits(const xrl_model_desc *model, const xrl_edit_state_desc *state, xrl_batch **out);
int xrl_batch_dims(const xrl_batch *b, int64_t *S, int64_t *G, int64_t *N, int64_t *E);
int xrl_batch_host_view(const xrl_batch *b, xrl_packed_view *view);
int xrl_batch_free(xrl_batch *b);   /* frees host and device copies; NULL is accepted          */

/* ---- context --------------------------------------------------------------------------------
 * weights_host: xrl_weight_count floats. hip_stream: a hipStream_t (NULL = default stream).
 * Errors: NULL, UNSUPPORTED (hidden not in {64,128,256}, mlp_layers not 1 or 2, ...), VALUE, HIP, OOM.
 * mlp_layers = 1 (one learned matrix per layer, Section 3.4 as printed) runs on the two-layer kernels
 * with an identity second layer, which changes no result; weights and gradients keep the one-layer
 * layout of xrl_weight_tensor.
 * Environment, read here: XRL_PERSISTENT_MIN_ROWS = row count from which the persistent MLP
 * kernels replace the streaming one (default 8192; 0 = always; results agree within rounding);
 * XRL_WGRAD_WIDE_MIN_ROWS = row count from which the weight-gradient kernel uses 256-column
 * tiles (default 2^18 at hidden = 256, else 2^20; same sums in a different, equally fixed order);
 * XRL_RESIDENT_MAX_GRAPHS (default 256; 0 = never) and XRL_RESIDENT_MAX_TILES (default 4) =
 * largest batch, in graphs and in 32-row tiles of nodes or edges per graph, that xrl_encode runs
 * as one launch with a block per graph (message-passing rounds of the MLP kind, rows of at most
 * 256 bytes, no receiver of more than 32 in-edges; results identical to the other path's);
 * XRL_CLUSTER_MAX_GRAPHS (default 48; 0 = never) = largest batch of graphs of more tiles than
 * that which xrl_encode runs as one launch with several blocks per graph, used when a block per
 * four tiles of the largest graph fits the GPU at once (the few dozen candidates of one rewriting
 * step, Section 4.2; same results). Its blocks wait for each other; XRL_CLUSTER_SPIN_LIMIT =
 * polls after which such a wait gives up (default 2^21, about two seconds): the launch then
 * finishes with invalid embeddings, and the next xrl_encode on the context returns XRL_ERR_HIP
 * (once), after which the context works again. */
int xrl_create(const xrl_model_desc *model, const float *weights_host, void *hip_stream,
               xrl_ctx **out);
int xrl_set_weights(xrl_ctx *ctx, const float *weights_host);
int xrl_destroy(xrl_ctx *ctx);
/* Copies the packed arrays to the GPU (async on the ctx stream). Must precede the calls below. */
int xrl_batch_upload(xrl_ctx *ctx, xrl_batch *b);

/* ---- forward --------------------------------------------------------------------------------
 * xrl_encode: the GNN of Section 3.4 on every graph of the batch. d_emb: device [G, hidden]
 * fp32, the graph representations. save_for_backward != 0 keeps the per-round node states and
 * received sums inside ctx for xrl_encode_backward (overwritten by the next xrl_encode).
 * Errors: NULL, SHAPE, OOM, HIP (also: an earlier one-launch encode on this context did not
 * complete, see XRL_CLUSTER_SPIN_LIMIT). */
int xrl_encode(xrl_ctx *ctx, const xrl_batch *b, float *d_emb, int save_for_backward);

/* xrl_policy_value: heads of Section 3.3.2 on the embeddings. Per slot j: logit = policy MLP of
 * emb[j]; per state, over its valid slots only (invalid-action masking): d_logp [G] = log
 * softmax (-inf at masked slots), d_entropy [S], d_action [S] = slot index inside the state of
 * the largest valid logit, lowest index on ties (0 = No-Op), d_value [S] = value MLP of the mean
 * embedding of the valid slots. All device pointers (d_emb 16-byte aligned); d_logit [G] may be
 * NULL. Errors: NULL, SHAPE (alignment), STATE, HIP. */
int xrl_policy_value(xrl_ctx *ctx, const xrl_batch *b, const float *d_emb, float *d_logp,
                     float *d_value, float *d_entropy, int32_t *d_action, float *d_logit);

/* xrl_policy_value_static: xrl_policy_value for callers that cannot allocate (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc). Same arguments, same kernel and
 * bit-identical outputs, but it calls no allocation routine at all: its scratch (per-state
 * counters, the logits when d_logit is NULL, the per-state mean embeddings) is a fixed array in
 * device memory, 288 KiB per GPU, held until the process ends. Limits: at most 4096 slots (G) and
 * n_states * hidden <= 65536; beyond them XRL_ERR_UNSUPPORTED and nothing is launched. Every call
 * on a GPU shares that GPU's array: calls that overlap on one GPU (two streams, two contexts)
 * race; calls on one stream are safe. Other errors: NULL, SHAPE (alignment), STATE, HIP. */
int xrl_policy_value_static(xrl_ctx *ctx, const xrl_batch *b, const float *d_emb, float *d_logp,
                            float *d_value, float *d_entropy, int32_t *d_action, float *d_logit);

/* ---- backward (Section 3.3.4: one back-propagation through heads and GNN) -------------------
 * For a scalar J with dJ/dlogp = d_dlogp [G] (entries at masked slots are ignored), dJ/dvalue =
 * d_dvalue [S], dJ/dentropy = d_dentropy [S]:
 * xrl_policy_value_backward writes d_demb [G, hidden] = dJ/demb (exactly 0 at masked slots) and
 * ADDS the head weight gradients into d_dweights [xrl_weight_count] fp32 (flat layout above).
 * xrl_encode_backward ADDS the encoder weight gradients for upstream d_demb into d_dweights; it
 * needs the batch's last xrl_encode to have been called with save_for_backward != 0 (else STATE).
 * Results are run-to-run deterministic (no floating-point atomics). */
int xrl_policy_value_backward(xrl_ctx *ctx, const xrl_batch *b, const float *d_emb,
                              const float *d_dlogp, const float *d_dvalue,
                              const float *d_dentropy, float *d_demb, float *d_dweights);
int xrl_encode_backward(xrl_ctx *ctx, const xrl_batch *b, const float *d_demb, float *d_dweights);

/* ---- objective (Section 3.3.4: J = L_clip + c1 L_vf + c2 L_entropy, to be minimised) ----------
 * From the outputs of xrl_policy_value on a minibatch of S states and the rollout's records:
 * d_action [S] int32 = slot taken inside each state (0 = No-Op; must be a valid slot: an index outside
 * the state's slots or on a masked slot contributes nothing, leaves that state's derivatives zero and
 * turns all four entries of d_J into NaN, which is how the caller detects it), d_old_logp
 * [S] = its log-probability when sampled, d_advantage [S], d_v_target [S]; eps = clip range, c1,
 * c2 = weights of the value and entropy terms (0.5 and 0.01 in the paper's table; eps is not
 * printed there).  ratio_s = exp(logp[slot_s] - old_logp_s);
 *   L_clip = -mean_s min(ratio_s A_s, clip(ratio_s, 1-eps, 1+eps) A_s), L_vf = mean_s (value_s -
 *   v_target_s)^2, L_entropy = -mean_s entropy_s.
 * Writes d_J [4] = {J, L_clip, L_vf, L_entropy} and the derivatives d_dlogp [G] (zero except at
 * the taken slots; where both arguments of the min are equal the unclipped one is
 * differentiated), d_dvalue [S], d_dentropy [S]: the inputs of xrl_policy_value_backward. All
 * device pointers, fp32. Sums over states are taken in a fixed order. Errors: NULL, STATE, HIP. */
int xrl_ppo_objective(xrl_ctx *ctx, const xrl_batch *b, const float *d_logp, const float *d_value,
                      const float *d_entropy, const int32_t *d_action, const float *d_old_logp,
                      const float *d_advantage, const float *d_v_target, float eps, float c1,
                      float c2, float *d_J, float *d_dlogp, float *d_dvalue, float *d_dentropy);

/* ---- featurisation of Section 3.3.2 (the paragraph on building the graph input) --------------
 * Edge attributes from tensor shapes: an edge's attribute is its tensor's shape, zero-padded on
 * the leading side to rank 4 and divided by the constant M (4096 in the hyper-parameter table of
 * the appendix). All host memory. shape_ptr: [n_edges + 1], non-decreasing from 0, edge e's
 * shape is dims[shape_ptr[e] .. shape_ptr[e+1]) (rank 0 to 4, entries >= 0); edge_feat:
 * [n_edges, 4] fp32, written. With n_op_types ~ 40, n_node_dense = 0, d_edge = 4 and graph_global
 * NULL (zeros) this gives the state description the paper prints.
 * Errors: NULL, SHAPE (rank above 4, shape_ptr not monotone), VALUE (negative extent, M <= 0). */
int xrl_edge_features_from_shapes(const int32_t *shape_ptr, const int64_t *dims, int64_t n_edges,
                                  double M, float *edge_feat);

/* ---- building blocks exposed for measurement and per-step checks ----------------------------
 * xrl_segment_sum: out[i, :] = sum of values[r, :] over rows r in [d_ptr[i], d_ptr[i+1]) -- the
 * receiver-side aggregation of Section 3.4's first two equations on receiver-ordered rows, and
 * the per-graph sum of its third. d_values: device [n_rows, width] fp32; d_ptr: device [n_seg+1]
 * int32, non-decreasing, d_ptr[0] = 0, d_ptr[n_seg] = n_rows; d_out: device [n_seg, width] fp32.
 * width must be a multiple of 4 and at most 256. */
int xrl_segment_sum(xrl_ctx *ctx, const float *d_values, const int32_t *d_ptr, int64_t n_rows,
                    int64_t n_seg, int32_t width, float *d_out);

/* Copies one saved activation of the last xrl_encode(save_for_backward=1) into d_out as fp32:
 * what = "a0" [N, d_edge] (sum of incoming edge attrs), "h" [N, hidden] (node states after the
 * node-update layer for round = 0, after message-passing round r for round = r), "agg" [N,
 * hidden] (received sums of round r >= 1 as the node MLP reads them: zeros for nodes without
 * in-edges), "pool"
 * [G, hidden] (per-graph sum or mean). */
int xrl_get_activation(xrl_ctx *ctx, const xrl_batch *b, const char *what, int32_t round,
                       float *d_out);

/* xrl_weight_gradient: dW[k, f] += sum over rows of X[row, k] dZ[row, f] and db[f] += sum over
 * rows of dZ[row, f] -- the weight gradient of one affine layer of the encoder's MLPs as
 * xrl_encode_backward computes it (Section 3.3.4), exposed so that the product can be checked and
 * timed on its own. kind XRL_WG_PLAIN: X = d_x [n_rows, H]. XRL_WG_EDGE: X = [h[sender] |
 * h[receiver] | edge attributes] over the batch's E edges in receiver order, d_x = h [N, H].
 * XRL_WG_NODE: X = [h | received sums], d_x = h, d_x2 = the sums, both [N, H]; the sums' rows of
 * nodes without in-edges are not read and count as zero (n_rows is ignored for these two kinds).
 * d_x, d_x2 and d_dZ [rows, H] are device arrays in the ctx's operand type (fp32, or bf16 bit
 * patterns); d_dW [K, H] (K = columns of X) and d_db [H] are device fp32 and are accumulated
 * into. Deterministic. Uses the backward's scratch. Errors: NULL, STATE, INDEX, SHAPE, OOM, HIP. */
enum { XRL_WG_PLAIN = 0, XRL_WG_EDGE = 1, XRL_WG_NODE = 2 };
int xrl_weight_gradient(xrl_ctx *ctx, const xrl_batch *b, int32_t kind, const void *d_x, const void *d_x2,
                        const void *d_dZ, int64_t n_rows, float *d_dW, float *d_db);

/* xrl_mlp_backward: the gradients through one fused two-layer MLP of a message-passing round as
 * xrl_encode_backward computes them (Section 3.3.4), on caller-given inputs, for per-step checks.
 * For y = relu(relu(x W1 + b1) W2 + b2) of MLP (`kind`, `round`) and upstream dy:
 *   z1 = relu(x W1 + b1), dz2 = dy * [y > 0], dz1 = (dz2 W2^T) * [z1 > 0], dx = dz1 W1^T.
 * kind XRL_WG_EDGE: rows = the batch's E edges in receiver order, x = [h[sender] | h[receiver] |
 * edge attrs], d_dy [N, H] is indexed by receiver (y is recomputed), d_dxa / d_dxb [E, H] =
 * gradients w.r.t. h[sender] / h[receiver] per edge. XRL_WG_NODE: rows = N nodes, x = [d_h |
 * d_agg], d_y [N, H] = the forward's output, d_dy [N, H], d_dxa / d_dxb [N, H] = gradients w.r.t.
 * h / the received sums. Outputs d_z1, d_dz1, d_dz2 [rows, H]. All arrays are device memory in the
 * ctx's operand type. Errors: NULL, STATE, INDEX, UNSUPPORTED (attention rounds), HIP. */
int xrl_mlp_backward(xrl_ctx *ctx, const xrl_batch *b, int32_t kind, int32_t round, const void *d_h,
                     const void *d_agg, const void *d_y, const void *d_dy, void *d_z1, void *d_dz1,
                     void *d_dz2, void *d_dxa, void *d_dxb);

/* Per-kernel timing for roofline measurement. While enabled, every launch group of the forward
 * path and of the encoder's backward is bracketed by HIP events on the ctx stream.
 * xrl_read_timing synchronises the stream, returns the summed duration and launch count
 * recorded since the last read for `kernel` and forgets them. Forward: {"embed", "edge",
 * "edge_fixup", "node", "pool", "readout", "heads"} (the steps of Section 3.4 / 3.3.2 in
 * execution order; "gat_linear", "gat_aggregate" with XRL_ROUND_GAT; "resident" = the whole
 * encoder of a small batch in one launch). Backward (Section 3.3.4):
 * {"bwd_edge", "bwd_node", "bwd_embed"} = gradients through the fused MLPs, {"wgrad_edge",
 * "wgrad_node", "wgrad_embed"} = both layers' weight gradients of one such MLP with their
 * reductions ("wgrad": the same for a single product through xrl_weight_gradient), "grad_gather" =
 * per-node sum of the per-edge gradients; "gat_bwd" = one attention round's backward.
 * Errors: NULL, INDEX, HIP. */
int xrl_set_timing(xrl_ctx *ctx, int enabled);
int xrl_read_timing(xrl_ctx *ctx, const char *kernel, double *total_ms, int64_t *launches);

/* The machine's own ceilings, measured, to set beside the vendor figures the rooflines use:
 * *mfma_tflops = bf16 32x32x16 MFMA rate of a loop whose operands and accumulators stay in
 * registers (four independent accumulator tiles per wave, four waves per SIMD); *copy_gbs =
 * read + write rate of a plain 16-byte-per-lane device-to-device copy of copy_bytes (rounded down
 * to a multiple of 16; the library allocates and frees the two buffers). Synchronous.
 * Errors: NULL, SHAPE (copy_bytes < 16), OOM, HIP. */
int xrl_measure_peaks(xrl_ctx *ctx, int64_t copy_bytes, double *mfma_tflops, double *copy_gbs);

const char *xrl_last_error(void);
const char *xrl_version(void);

#ifdef __cplusplus
}
#endif
#endif /* XRL_H */
