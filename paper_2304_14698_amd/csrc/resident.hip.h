// One-launch encoder for small batches (the agent's own inference loop encodes one state of a few
// dozen candidate graphs per step, Section 4.2): one block per graph runs the node-update layer,
// every message-passing round and the global-update layer (Section 3.4) on its graph, with block
// barriers where the streaming path has kernel boundaries. A graph's node states and received
// sums live in the same global buffers as on the streaming path (a few hundred KB per graph: they
// stay in the CU's L1 and the XCD's L2), so both paths save the same activations for the
// backward pass; what the launch removes is a dozen launch latencies and pipeline drains.
//
// Tiles, arithmetic and the order of every sum are those of mlp2_wave_tile and
// graph_readout_block, so the embeddings equal the streaming path's bit for bit. Edge tiles
// come from the packer's per-graph table (no tile spans two graphs, no receiver spans two
// tiles), which is why no carry fix-up is needed here.
#pragma once
#include "heads.hip.h"
#include "mlp2.hip.h"

constexpr int kResidentMaxRounds = 8;

struct ResidentMlp {
  const void *W1s, *W2s;
  const float *b1, *b2;
  int nslab1;
};

struct ResidentArgs {
  Mlp2Args base;                         // batch arrays, embed weights, agg0 / n_agg / agg_stride, out = h[0]
  ResidentMlp edge[kResidentMaxRounds], node[kResidentMaxRounds];
  void *h[kResidentMaxRounds + 1];       // node states after the embed layer and after each round
  void *agg[kResidentMaxRounds];         // received sums of each round
  int rounds;
  int w1_bytes_max;                      // LDS reserved for a phase's first-layer weights
  int64_t E;
  const int32_t *graph_node_ptr, *graph_tile_ptr, *gtile_ptr;
  int mean;
  float *pool;
  RowMlpArgs readout;
  // several blocks per graph (encode_cluster_kernel)
  int K;                                 // blocks per graph
  int G;                                 // graphs
  unsigned *arrived;                     // [G] per-graph arrival counters, zero between launches
  unsigned *fault;                       // host-mapped word, set when a wait gives up
  unsigned spin_limit;                   // polls after which a wait gives up
};

// Copies `bytes` (a multiple of 16) from global memory into LDS with all 256 threads, eight
// 16-byte loads in flight per thread (a plain copy loop would pay one memory round trip per 4 KB).
__device__ __forceinline__ void fill_lds(char *dst, const void *src, int bytes) {
  const f32x4 *s = (const f32x4 *)src;
  f32x4 *d = (f32x4 *)dst;
  const int n = bytes / 16, tid = threadIdx.x;
  for (int base = 0; base < n; base += 256 * 8) {
    f32x4 t[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int k = base + i * 256 + tid;
      t[i] = s[k < n ? k : 0];
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int k = base + i * 256 + tid;
      if (k < n) d[k] = t[i];
    }
  }
}

// LDS: [four waves' row staging | W1 of the running phase | its W2 | the embed layer's table];
// the readout reuses it from the start. With a handful of tiles per graph a weight fragment
// requested from L2 one slab ahead of its MFMAs (as the streaming kernel does, where other waves
// hide the wait) would cost a memory round trip per slab, so every phase first copies its two
// matrices into LDS in one batch of loads.
template <typename T, int H>
__global__ __launch_bounds__(256) void encode_resident_kernel(const ResidentArgs ra) {
  extern __shared__ __align__(16) char smem[];
  constexpr int VEC = 16 / (int)sizeof(T), MB = H / 32;
  constexpr int W2_BYTES = MB * (32 / (2 * VEC)) * MB * 1024;   // fragment-ordered [H, H]
  const int gi = blockIdx.x, lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  char *stage = smem + wave * RowStage<T, H>::BYTES;
  char *w1l = smem + 4 * RowStage<T, H>::BYTES, *w2l = w1l + ra.w1_bytes_max, *tabl = w2l + W2_BYTES;
  const int n0 = ra.graph_node_ptr[gi], n1 = ra.graph_node_ptr[gi + 1];
  const int t0 = ra.graph_tile_ptr[gi], t1 = ra.graph_tile_ptr[gi + 1];
  const int n_node_tiles = (n1 - n0 + 31) / 32;

  Mlp2Args a = ra.base;
  fill_lds(w1l, a.W1x, a.nslabx * MB * 1024);
  fill_lds(w2l, a.W2s, W2_BYTES);
  fill_lds(tabl, a.table, a.Tn * H * 4);
  a.W1x = w1l; a.W2s = w2l; a.table = (const float *)tabl;
  __syncthreads();
  for (int k = wave; k < n_node_tiles; k += 4) {
    const int left = n1 - n0 - 32 * k;
    mlp2_wave_tile<float, T, H, KIND_EMBED>(a, n0 + 32 * k, left < 32 ? left : 32, 0, stage, lane);
  }
  __syncthreads();   // (a block's global stores are visible to its own waves after the barrier)
  a.W1s = w1l;
  for (int r = 0; r < ra.rounds; ++r) {
    fill_lds(w1l, ra.edge[r].W1s, ra.edge[r].nslab1 * MB * 1024);
    fill_lds(w2l, ra.edge[r].W2s, W2_BYTES);
    a.b1 = ra.edge[r].b1; a.b2 = ra.edge[r].b2; a.nslab1 = ra.edge[r].nslab1;
    a.n_rows = ra.E; a.h = ra.h[r]; a.out = ra.agg[r];
    __syncthreads();
    for (int wt = t0 + wave; wt < t1; wt += 4) {
      const int e0 = ra.gtile_ptr[wt];
      mlp2_wave_tile<T, T, H, KIND_EDGE>(a, e0, ra.gtile_ptr[wt + 1] - e0, wt, stage, lane);
    }
    __syncthreads();
    fill_lds(w1l, ra.node[r].W1s, ra.node[r].nslab1 * MB * 1024);
    fill_lds(w2l, ra.node[r].W2s, W2_BYTES);
    a.b1 = ra.node[r].b1; a.b2 = ra.node[r].b2; a.nslab1 = ra.node[r].nslab1;
    a.agg = ra.agg[r]; a.out = ra.h[r + 1];
    __syncthreads();
    for (int k = wave; k < n_node_tiles; k += 4) {
      const int left = n1 - n0 - 32 * k;
      mlp2_wave_tile<T, T, H, KIND_NODE>(a, n0 + 32 * k, left < 32 ? left : 32, 0, stage, lane);
    }
    __syncthreads();
  }
  graph_readout_block<T, VEC>((const T *)ra.h[ra.rounds], n0, n1, gi, H, ra.mean, ra.pool, ra.readout, (float *)smem);
}

// ---- several blocks per graph ------------------------------------------------------------------
// The same phases with a graph's tiles dealt over K blocks (K * G at most the number of CUs and
// one block per CU, so every block of the launch is resident while any of them waits): tile j of a
// phase goes to block j % K, wave (j / K) % 4. Where the one-block form has a block barrier, the
// blocks of a graph meet at a counter in global memory: a block's waves finish their stores
// (block barrier), one thread publishes them (release fence at device scope) and adds one to the
// graph's counter, the block copies the next phase's weights into LDS while the others arrive,
// the thread waits for the counter to reach K * (phases so far) and takes an acquire fence, and a
// second block barrier lets the other waves go on. The wait is bounded: a block that is not
// released within about two seconds reports through `fault` and goes on, so the grid always
// drains (the results are then wrong, and the next call on the context says so).
// Blocks b, b + 8, b + 16, ... hold one graph: the dispatcher deals consecutive blocks over the
// eight XCDs, so a graph's rows pass from block to block through one L2 (a placement that only
// matters for speed: the fences are device-wide).
constexpr unsigned kClusterSpinLimit = 1u << 21;   // default of ResidentArgs::spin_limit

__device__ __forceinline__ void cluster_arrive(unsigned *ctr) {
  __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void cluster_wait(unsigned *ctr, unsigned target, unsigned *fault, unsigned spin_limit) {
  // (spin_limit polls at most; with a limit of 0 the wait cannot see anything arrive and gives up at once)
  unsigned spins = 0;
  bool arrived = false;
  while (spins++ < spin_limit && !(arrived = __hip_atomic_load(ctr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= target))
    __builtin_amdgcn_s_sleep(2);
  if (!arrived) __hip_atomic_store(fault, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
}

template <typename T, int H>
__global__ __launch_bounds__(256) void encode_cluster_kernel(const ResidentArgs ra) {
  extern __shared__ __align__(16) char smem[];
  constexpr int VEC = 16 / (int)sizeof(T), MB = H / 32;
  constexpr int W2_BYTES = MB * (32 / (2 * VEC)) * MB * 1024;
  const int K = ra.K;
  const int q = blockIdx.x >> 3;
  const int gi = (q / K) * 8 + (blockIdx.x & 7), kb = q % K;
  if (gi >= ra.G) return;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  char *stage = smem + wave * RowStage<T, H>::BYTES;
  char *w1l = smem + 4 * RowStage<T, H>::BYTES, *w2l = w1l + ra.w1_bytes_max, *tabl = w2l + W2_BYTES;
  const int n0 = ra.graph_node_ptr[gi], n1 = ra.graph_node_ptr[gi + 1];
  const int t0 = ra.graph_tile_ptr[gi], t1 = ra.graph_tile_ptr[gi + 1];
  const int n_node_tiles = (n1 - n0 + 31) / 32;
  unsigned *ctr = ra.arrived + gi;
  unsigned met = 0;   // meetings so far

  // end of a phase: publish, copy the next phase's matrices, wait for the graph's other blocks
  auto meet = [&](const void *W1s, const void *W2s, int nslab1) {
    __syncthreads();
    if (threadIdx.x == 0) cluster_arrive(ctr);
    if (W1s) {
      fill_lds(w1l, W1s, nslab1 * MB * 1024);
      fill_lds(w2l, W2s, W2_BYTES);
    }
    ++met;
    if (threadIdx.x == 0) cluster_wait(ctr, met * (unsigned)K, ra.fault, ra.spin_limit);
    __syncthreads();
  };

  Mlp2Args a = ra.base;
  fill_lds(w1l, a.W1x, a.nslabx * MB * 1024);
  fill_lds(w2l, a.W2s, W2_BYTES);
  fill_lds(tabl, a.table, a.Tn * H * 4);
  a.W1x = w1l; a.W2s = w2l; a.table = (const float *)tabl;
  __syncthreads();
  for (int j = kb + K * wave; j < n_node_tiles; j += 4 * K) {
    const int left = n1 - n0 - 32 * j;
    mlp2_wave_tile<float, T, H, KIND_EMBED>(a, n0 + 32 * j, left < 32 ? left : 32, 0, stage, lane);
  }
  a.W1s = w1l;
  if (ra.rounds == 0 && kb != 0) {
    __syncthreads();
    if (threadIdx.x == 0) cluster_arrive(ctr);
    return;
  }
  if (ra.rounds > 0) meet(ra.edge[0].W1s, ra.edge[0].W2s, ra.edge[0].nslab1);
  else meet(nullptr, nullptr, 0);
  for (int r = 0; r < ra.rounds; ++r) {
    a.b1 = ra.edge[r].b1; a.b2 = ra.edge[r].b2; a.nslab1 = ra.edge[r].nslab1;
    a.n_rows = ra.E; a.h = ra.h[r]; a.out = ra.agg[r];
    for (int wt = t0 + kb + K * wave; wt < t1; wt += 4 * K) {
      const int e0 = ra.gtile_ptr[wt];
      mlp2_wave_tile<T, T, H, KIND_EDGE>(a, e0, ra.gtile_ptr[wt + 1] - e0, wt, stage, lane);
    }
    meet(ra.node[r].W1s, ra.node[r].W2s, ra.node[r].nslab1);
    a.b1 = ra.node[r].b1; a.b2 = ra.node[r].b2; a.nslab1 = ra.node[r].nslab1;
    a.agg = ra.agg[r]; a.out = ra.h[r + 1];
    for (int j = kb + K * wave; j < n_node_tiles; j += 4 * K) {
      const int left = n1 - n0 - 32 * j;
      mlp2_wave_tile<T, T, H, KIND_NODE>(a, n0 + 32 * j, left < 32 ? left : 32, 0, stage, lane);
    }
    if (r + 1 == ra.rounds && kb != 0) {
      // the graph's first block does the readout: the others only report that their rows are out
      __syncthreads();
      if (threadIdx.x == 0) cluster_arrive(ctr);
      return;
    }
    if (r + 1 < ra.rounds) meet(ra.edge[r + 1].W1s, ra.edge[r + 1].W2s, ra.edge[r + 1].nslab1);
    else meet(nullptr, nullptr, 0);
  }
  // (every block of the graph has arrived for the last time: the counter can go back to zero)
  if (threadIdx.x == 0) __hip_atomic_store(ctr, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  graph_readout_block<T, VEC>((const T *)ra.h[ra.rounds], n0, n1, gi, H, ra.mean, ra.pool, ra.readout, (float *)smem);
}
