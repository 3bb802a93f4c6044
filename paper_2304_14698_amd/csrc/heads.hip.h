// Small fp32 kernels on per-graph and per-state data: the readout MLP of the global-update layer
// (Section 3.4), the policy and value heads with invalid-action masking (Section 3.3.2), and
// their backward passes. G and S rows only -- latency-bound, plain vector ALU code.
#pragma once
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>
#include "segsum.hip.h"

// Rows per block of the row-MLP kernels: 8 reuses every weight read eight times (large batches);
// 1 gives one block per row so that small batches still spread over the chip.

// Up to three affine layers over rows of [in1 | in2]; ReLU after every layer except, when
// relu_last == 0, the last. Optionally stores every layer's output (post-activation) for the
// backward pass: act[l] is [n_rows, d_out[l]].
struct RowMlpArgs {
  int n_layers, relu_last;
  const float *W[3], *b[3];
  int d_in[3], d_out[3];
  const float *in1, *in2;  // in2 nullable
  int w1, w2;              // widths of in1 / in2; w1 + w2 == d_in[0]
  int64_t n_rows;
  float *out;              // [n_rows, d_out[last]]
  float *act[3];           // nullable each
};

// One row through the layers of `a`, all 256 threads of the block cooperating. These kernels are
// bound by memory latency, not bandwidth, so a layer's weights are requested in as few dependent
// rounds as possible: with d_out a multiple of 4 (and the matrix 16-byte aligned) a thread owns
// four adjacent outputs and one of 256 / (d_out / 4) slices of the contraction, loads its weights
// 16 bytes at a time, sixteen loads in flight, and the slices' partial sums are added in slice
// order; other layers (a single output, say) split the contraction the same way with scalar loads.
// cur holds the input row (d_in[0] floats) on entry; cur/nxt: >= widest layer; part: 1024 floats,
// 16-byte aligned. `row` indexes the stores to a.act[l] and a.out. COHERENT_OUT stores a.out with
// device scope, for a consumer in another block of the same launch.
template <bool COHERENT_OUT = false>
__device__ __forceinline__ void store_row_out(float *p, float y) {
  if constexpr (COHERENT_OUT) __hip_atomic_store(p, y, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  else *p = y;
}

template <bool COHERENT_OUT = false>
__device__ __forceinline__ void block_row_mlp(const RowMlpArgs &a, float *cur, float *nxt, float *part,
                                              int64_t row) {
  const int t = threadIdx.x;
  for (int l = 0; l < a.n_layers; ++l) {
    const int din = a.d_in[l], dout = a.d_out[l];
    const bool relu = a.relu_last || (l + 1 < a.n_layers);
    const float *W = a.W[l];
    if ((dout & 3) == 0 && dout <= 1024 && ((uintptr_t)W & 15) == 0) {
      const int fq = dout >> 2;                           // 16-byte columns
      int KQ = 256 / fq;                                  // slices of the contraction
      if (KQ > din) KQ = din;
      const int kc = (din + KQ - 1) / KQ;
      const int fl = t % fq, kq = t / fq;
      if (kq < KQ) {
        const int k0 = kq * kc, k1 = (k0 + kc) < din ? (k0 + kc) : din;
        const float4 *Wp = (const float4 *)W + fl;
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        int k = k0;
        for (; k + 16 <= k1; k += 16) {
          float4 w[16];
#pragma unroll
          for (int i = 0; i < 16; ++i) w[i] = Wp[(size_t)(k + i) * fq];
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const float x = cur[k + i];
            acc.x = fmaf(x, w[i].x, acc.x); acc.y = fmaf(x, w[i].y, acc.y);
            acc.z = fmaf(x, w[i].z, acc.z); acc.w = fmaf(x, w[i].w, acc.w);
          }
        }
        for (; k < k1; ++k) {
          const float4 w = Wp[(size_t)k * fq];
          const float x = cur[k];
          acc.x = fmaf(x, w.x, acc.x); acc.y = fmaf(x, w.y, acc.y);
          acc.z = fmaf(x, w.z, acc.z); acc.w = fmaf(x, w.w, acc.w);
        }
        ((float4 *)part)[kq * fq + fl] = acc;
      }
      __syncthreads();
      for (int f = t; f < dout; f += 256) {
        float v = part[f];
        for (int q = 1; q < KQ; ++q) v += part[q * dout + f];
        v += a.b[l][f];
        const float y = relu ? fmaxf(v, 0.f) : v;
        nxt[f] = y;
        if (a.act[l]) a.act[l][row * dout + f] = y;
        if (l + 1 == a.n_layers) store_row_out<COHERENT_OUT>(a.out + row * dout + f, y);
      }
      __syncthreads();
    } else {
      int fw = 256;                                       // outputs handled per pass
      while (fw / 2 >= dout && 256 / (fw / 2) <= din) fw /= 2;
      const int KQ = 256 / fw;                            // thread groups splitting the contraction
      const int kc = (din + KQ - 1) / KQ;
      const int fl = t % fw, kq = t / fw;
      const int k0 = kq * kc, k1 = (k0 + kc) < din ? (k0 + kc) : din;
      for (int f0 = 0; f0 < dout; f0 += fw) {
        const int f = f0 + fl;
        float acc = 0.f;
        if (f < dout) {
          int k = k0;
          for (; k + 16 <= k1; k += 16) {
            float w[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) w[i] = W[(size_t)(k + i) * dout + f];
#pragma unroll
            for (int i = 0; i < 16; ++i) acc = fmaf(cur[k + i], w[i], acc);
          }
          for (; k < k1; ++k) acc = fmaf(cur[k], W[(size_t)k * dout + f], acc);
        }
        if (KQ > 1) {
          part[t] = acc;
          __syncthreads();
          if (kq == 0) {
            acc = part[fl];
            for (int q = 1; q < KQ; ++q) acc += part[q * fw + fl];
          }
        }
        if (kq == 0 && f < dout) {
          acc += a.b[l][f];
          const float y = relu ? fmaxf(acc, 0.f) : acc;
          nxt[f] = y;
          if (a.act[l]) a.act[l][row * dout + f] = y;
          if (l + 1 == a.n_layers) store_row_out<COHERENT_OUT>(a.out + row * dout + f, y);
        }
        if (KQ > 1) __syncthreads();
      }
      __syncthreads();
    }
    float *tmp = cur; cur = nxt; nxt = tmp;
  }
}

template <int ROWMLP_ROWS>
__global__ __launch_bounds__(256) void rowmlp_kernel(const RowMlpArgs a) {
  // two buffers of ROWMLP_ROWS * dmax floats; with one row per block, 1024 floats of partial sums first
  extern __shared__ __align__(16) float sm[];
  int dmax = a.d_in[0];
  for (int l = 0; l < a.n_layers; ++l) dmax = a.d_out[l] > dmax ? a.d_out[l] : dmax;
  float *cur = sm + (ROWMLP_ROWS == 1 ? 1024 : 0), *nxt = cur + ROWMLP_ROWS * dmax;
  const int64_t row0 = (int64_t)blockIdx.x * ROWMLP_ROWS;
  for (int i = threadIdx.x; i < ROWMLP_ROWS * a.d_in[0]; i += blockDim.x) {
    const int r = i / a.d_in[0], k = i - r * a.d_in[0];
    const int64_t row = row0 + r;
    float v = 0.f;
    if (row < a.n_rows) v = k < a.w1 ? a.in1[row * a.w1 + k] : a.in2[row * a.w2 + (k - a.w1)];
    cur[r * dmax + k] = v;
  }
  __syncthreads();
  if constexpr (ROWMLP_ROWS == 1) {
    block_row_mlp(a, cur, nxt, sm, row0);
    return;
  }
  for (int l = 0; l < a.n_layers; ++l) {
    const int din = a.d_in[l], dout = a.d_out[l];
    const bool relu = a.relu_last || (l + 1 < a.n_layers);
    for (int f = threadIdx.x; f < dout; f += blockDim.x) {
      float acc[ROWMLP_ROWS];
      const float bv = a.b[l][f];
#pragma unroll
      for (int r = 0; r < ROWMLP_ROWS; ++r) acc[r] = bv;
#pragma unroll 16
      for (int k = 0; k < din; ++k) {
        const float w = a.W[l][(size_t)k * dout + f];
#pragma unroll
        for (int r = 0; r < ROWMLP_ROWS; ++r) acc[r] = fmaf(cur[r * dmax + k], w, acc[r]);
      }
#pragma unroll
      for (int r = 0; r < ROWMLP_ROWS; ++r) {
        const float y = relu ? fmaxf(acc[r], 0.f) : acc[r];
        nxt[r * dmax + f] = y;
        const int64_t row = row0 + r;
        if (row < a.n_rows) {
          if (a.act[l]) a.act[l][row * dout + f] = y;
          if (l + 1 == a.n_layers) a.out[row * dout + f] = y;
        }
      }
    }
    __syncthreads();
    float *t = cur; cur = nxt; nxt = t;
  }
}

// Global-update layer (Section 3.4) for one graph per block: the sum (or mean) of the graph's node
// states, then the readout MLP on [pool | global attrs], without leaving the block. The 256
// threads form 256 / (H / VEC) row groups, each lane owning a 16-byte column slice; a group
// takes every (number of groups)-th node with eight loads in flight, and the groups' partial
// sums are added in group order, so the result does not depend on timing. pool [G, H] is also
// stored (it is an input of the backward pass). Meant for batches of many graphs of moderate
// size; a few huge graphs go through the generic segment-sum kernels instead.
// (sm: (256 * VEC + 2 * widest layer) floats of LDS; all 256 threads of the block call it together.
// UF = loads a thread keeps in flight: a thread adds its rows in the same order whatever UF is.)
template <typename T, int VEC, int UF = 8>
__device__ __forceinline__ void graph_readout_block(const T *h, const int n0, const int n1, const int g, int H,
                                                    int mean, float *pool, const RowMlpArgs &mlp, float *sm) {
  const int t = threadIdx.x;
  const int tpr = H / VEC, ng = 256 / tpr, c0 = (t % tpr) * VEC, q = t / tpr;
  float acc[VEC];
#pragma unroll
  for (int j = 0; j < VEC; ++j) acc[j] = 0.f;
  int n = n0 + q;
  for (; n + (UF - 1) * ng < n1; n += UF * ng) {
    float v[UF][VEC];
#pragma unroll
    for (int i = 0; i < UF; ++i) RowVec<T, VEC>::load(h + (size_t)(n + i * ng) * H + c0, v[i]);
#pragma unroll
    for (int i = 0; i < UF; ++i)
#pragma unroll
      for (int j = 0; j < VEC; ++j) acc[j] += v[i][j];
  }
  if (n < n1) {
    // the last, partial round: the same loads in flight (rows past the end re-read the graph's
    // last row and are left out of the sum), not one dependent load after another
    float v[UF][VEC];
#pragma unroll
    for (int i = 0; i < UF; ++i) {
      const int r = n + i * ng;
      RowVec<T, VEC>::load(h + (size_t)(r < n1 ? r : n1 - 1) * H + c0, v[i]);
    }
#pragma unroll
    for (int i = 0; i < UF; ++i)
#pragma unroll
      for (int j = 0; j < VEC; ++j) acc[j] += n + i * ng < n1 ? v[i][j] : 0.f;
  }
#pragma unroll
  for (int j = 0; j < VEC; ++j) sm[(q * tpr + t % tpr) * VEC + j] = acc[j];
  __syncthreads();
  int dmax = mlp.d_in[0];
  for (int l = 0; l < mlp.n_layers; ++l) dmax = mlp.d_out[l] > dmax ? mlp.d_out[l] : dmax;
  float *cur = sm + 256 * VEC, *nxt = cur + dmax, *part = sm;   // (the partial sums are dead by then)
  const float scale = mean ? 1.f / (float)(n1 - n0 > 1 ? n1 - n0 : 1) : 1.f;
  for (int f = t; f < H; f += 256) {
    float a = sm[f];
    for (int k = 1; k < ng; ++k) a += sm[k * H + f];
    a *= scale;
    pool[(size_t)g * H + f] = a;
    cur[f] = a;
  }
  for (int k = t; k < mlp.w2; k += 256) cur[H + k] = mlp.in2[(size_t)g * mlp.w2 + k];
  __syncthreads();
  block_row_mlp(mlp, cur, nxt, part, g);
}

template <typename T, int VEC, int UF>
__global__ __launch_bounds__(256) void graph_readout_kernel(const T *h, const int32_t *graph_node_ptr, int H,
                                                            int mean, float *pool, const RowMlpArgs mlp) {
  extern __shared__ __align__(16) float sm[];   // [256 * VEC] partial sums, then the MLP's buffers
  const int g = blockIdx.x;
  graph_readout_block<T, VEC, UF>(h, graph_node_ptr[g], graph_node_ptr[g + 1], g, H, mean, pool, mlp, sm);
}

// pool[g, :] /= max(n_g, 1)  (mean readout)
__global__ void mean_scale_kernel(float *pool, const int32_t *graph_node_ptr, int64_t G, int H,
                                  int inverse_only_grad) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= G * H) return;
  const int64_t g = i / H;
  const int n = graph_node_ptr[g + 1] - graph_node_ptr[g];
  pool[i] = pool[i] / (float)(n > 1 ? n : 1);
}

// Block-wide reductions over 256 threads in a fixed tree order (deterministic).
__device__ __forceinline__ float block_sum(float v, float *red) {
  const int t = threadIdx.x;
  red[t] = v;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if (t < s) red[t] += red[t + s];
    __syncthreads();
  }
  const float r = red[0];
  __syncthreads();
  return r;
}

// One block per state: masked log-softmax over the state's slots, entropy, first-max action,
// the mean embedding of the valid slots and, on it, the value head (value.n_layers == 0 skips it).
__global__ __launch_bounds__(256) void state_policy_kernel(
    const float *logit, const uint8_t *mask, const int32_t *state_graph_ptr, const float *emb,
    int H, float *logp, float *entropy, int32_t *action, float *zmean, const RowMlpArgs value) {
  __shared__ float red[256];
  __shared__ int redi[256];
  __shared__ __align__(16) float zbuf[1024];                      // partial sums of the mean embedding
  __shared__ __align__(16) float vcur[512], vnxt[512];            // value head: layer input / output
  const int s = blockIdx.x, t = threadIdx.x;
  const int j0 = state_graph_ptr[s], j1 = state_graph_ptr[s + 1];
  // max valid logit and the lowest slot index attaining it
  float best = -INFINITY;
  int besti = 0x7fffffff;
  for (int j = j0 + t; j < j1; j += 256)
    if (mask[j]) {
      const float l = logit[j];
      if (l > best || (l == best && j < besti)) { best = l; besti = j; }
    }
  red[t] = best; redi[t] = besti;
  __syncthreads();
  for (int k = 128; k > 0; k >>= 1) {
    if (t < k) {
      const float o = red[t + k];
      const int oi = redi[t + k];
      if (o > red[t] || (o == red[t] && oi < redi[t])) { red[t] = o; redi[t] = oi; }
    }
    __syncthreads();
  }
  const float M = red[0];
  const int arg = redi[0];
  __syncthreads();
  float se = 0.f;
  int cnt = 0;
  for (int j = j0 + t; j < j1; j += 256)
    if (mask[j]) { se += expf(logit[j] - M); ++cnt; }
  const float lse = M + logf(block_sum(se, red));
  const float nvalid = block_sum((float)cnt, red);
  float ent = 0.f;
  for (int j = j0 + t; j < j1; j += 256) {
    if (mask[j]) {
      const float lp = logit[j] - lse;
      logp[j] = lp;
      ent -= expf(lp) * lp;
    } else {
      logp[j] = -INFINITY;
    }
  }
  ent = block_sum(ent, red);
  if (t == 0) { entropy[s] = ent; action[s] = arg - j0; }
  // mean embedding of the valid slots: H / 4 threads cover a row with 16-byte loads, the 1024 / H
  // thread groups take every (1024/H)-th slot, eight loads in flight each; the groups' partial
  // sums are combined in group order
  const int tpr = H / 4, ng = 256 / tpr, c4 = (t % tpr) * 4, q = t / tpr;     // H is 64, 128 or 256
  float4 p = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int j = j0 + q; j < j1; j += 8 * ng) {
    float4 v[8];
    bool on[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int ji = j + i * ng < j1 ? j + i * ng : j;
      v[i] = *(const float4 *)(emb + (size_t)ji * H + c4);
      on[i] = j + i * ng < j1 && mask[ji];
    }
#pragma unroll
    for (int i = 0; i < 8; ++i)
      if (on[i]) { p.x += v[i].x; p.y += v[i].y; p.z += v[i].z; p.w += v[i].w; }
  }
  float4 *zp = (float4 *)zbuf;                                   // [ng][H / 4]
  zp[t] = p;
  __syncthreads();
  if (t < tpr) {
    float4 acc = zp[t];
    for (int k = 1; k < ng; ++k) {
      const float4 o = zp[k * tpr + t];
      acc.x += o.x; acc.y += o.y; acc.z += o.z; acc.w += o.w;
    }
    acc.x /= nvalid; acc.y /= nvalid; acc.z /= nvalid; acc.w /= nvalid;
    *(float4 *)(zmean + (size_t)s * H + c4) = acc;
    *(float4 *)(vcur + c4) = acc;
  }
  __syncthreads();
  // value head on the mean embedding (Section 3.3.2), in the same block
  if (value.n_layers > 0) block_row_mlp(value, vcur, vnxt, zbuf, s);
}

// Both heads in one launch for batches of at most a few thousand slots. Blocks [0, G): the policy
// MLP of one slot, and the block that finishes a state's last slot (a per-state counter, which it
// also resets) does that state's masked log-softmax, entropy and first-max action. Blocks
// [G, G + S): the mean embedding of a state's valid slots and the value head on it, independent of
// the policy blocks. Results are the same as rowmlp_kernel<1> followed by state_policy_kernel.
// Logits cross blocks through device-scope stores and loads (each completed before the block's
// counter increment is issued), so no cache write-back or invalidation is needed.
__global__ __launch_bounds__(256) void policy_value_kernel(
    const RowMlpArgs policy, const uint8_t *mask, const int32_t *state_graph_ptr, int G, int S, int H,
    int32_t *counter, float *logp, float *entropy, int32_t *action, float *zmean, const RowMlpArgs value) {
  __shared__ __align__(16) float part[1024];
  __shared__ __align__(16) float bufa[512], bufb[512];
  __shared__ float red[256];
  __shared__ int redi[256];
  __shared__ int sh_state, sh_last;
  const int t = threadIdx.x;
  if ((int)blockIdx.x >= G) {
    // ---- value head of state s
    const int s = blockIdx.x - G;
    const int j0 = state_graph_ptr[s], j1 = state_graph_ptr[s + 1];
    const float *emb = policy.in1;
    const int tpr = H / 4, ng = 256 / tpr, c4 = (t % tpr) * 4, q = t / tpr;   // H is 64, 128 or 256
    float4 p = make_float4(0.f, 0.f, 0.f, 0.f);
    int cnt = 0;
    for (int j = j0 + q; j < j1; j += 8 * ng) {
      float4 v[8];
      bool on[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int ji = j + i * ng < j1 ? j + i * ng : j;
        v[i] = *(const float4 *)(emb + (size_t)ji * H + c4);
        on[i] = j + i * ng < j1 && mask[ji];
      }
#pragma unroll
      for (int i = 0; i < 8; ++i)
        if (on[i]) { p.x += v[i].x; p.y += v[i].y; p.z += v[i].z; p.w += v[i].w; ++cnt; }
    }
    ((float4 *)part)[t] = p;                                       // [ng][H / 4]
    redi[t] = cnt;
    __syncthreads();
    if (t < tpr) {
      float4 acc = ((float4 *)part)[t];
      int n = redi[0];
      for (int k = 1; k < ng; ++k) {
        const float4 o = ((float4 *)part)[k * tpr + t];
        acc.x += o.x; acc.y += o.y; acc.z += o.z; acc.w += o.w;
        n += redi[k * tpr];
      }
      const float nvalid = (float)n;
      acc.x /= nvalid; acc.y /= nvalid; acc.z /= nvalid; acc.w /= nvalid;
      *(float4 *)(zmean + (size_t)s * H + c4) = acc;
      *(float4 *)(bufa + c4) = acc;
    }
    __syncthreads();
    if (value.n_layers > 0) block_row_mlp(value, bufa, bufb, part, s);
    return;
  }
  // ---- policy MLP of slot j; meanwhile find the slot's state
  const int j = blockIdx.x;
  if (t == 0) sh_state = -1;
  for (int k = t; k < H; k += 256) bufa[k] = policy.in1[(size_t)j * H + k];
  __syncthreads();
  for (int s = t; s < S; s += 256)
    if (state_graph_ptr[s] <= j && j < state_graph_ptr[s + 1]) sh_state = s;
  block_row_mlp<true>(policy, bufa, bufb, part, j);
  __builtin_amdgcn_s_waitcnt(0x0F70);                              // vmcnt(0): this wave's logit store has completed
  __syncthreads();
  const int s = sh_state;
  if (s < 0) return;                                               // (a slot outside every state: not packed by this library)
  const int j0 = state_graph_ptr[s], j1 = state_graph_ptr[s + 1];
  if (t == 0) {
    const int done = atomicAdd(&counter[s], 1);
    sh_last = done == j1 - j0 - 1;
    if (sh_last) counter[s] = 0;                                   // ready for the next launch
  }
  __syncthreads();
  if (!sh_last) return;
  const float *logit = policy.out;
  auto ld = [&](int i) { return __hip_atomic_load(logit + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); };
  // max valid logit and the lowest slot index attaining it
  float best = -INFINITY;
  int besti = 0x7fffffff;
  for (int i = j0 + t; i < j1; i += 256)
    if (mask[i]) {
      const float l = ld(i);
      if (l > best || (l == best && i < besti)) { best = l; besti = i; }
    }
  red[t] = best; redi[t] = besti;
  __syncthreads();
  for (int k = 128; k > 0; k >>= 1) {
    if (t < k) {
      const float o = red[t + k];
      const int oi = redi[t + k];
      if (o > red[t] || (o == red[t] && oi < redi[t])) { red[t] = o; redi[t] = oi; }
    }
    __syncthreads();
  }
  const float M = red[0];
  const int arg = redi[0];
  __syncthreads();
  float se = 0.f;
  for (int i = j0 + t; i < j1; i += 256)
    if (mask[i]) se += expf(ld(i) - M);
  const float lse = M + logf(block_sum(se, red));
  float ent = 0.f;
  for (int i = j0 + t; i < j1; i += 256) {
    if (mask[i]) {
      const float lp = ld(i) - lse;
      logp[i] = lp;
      ent -= expf(lp) * lp;
    } else {
      logp[i] = -INFINITY;
    }
  }
  ent = block_sum(ent, red);
  if (t == 0) { entropy[s] = ent; action[s] = arg - j0; }
}

// dJ/dlogit per slot from (dlogp, dentropy) and the forward's logp/entropy; one block per state.
//   dlogit_k = c_k - p_k * sum_valid c  -  dent * p_k * (logp_k + entropy)      (0 when masked)
__global__ __launch_bounds__(256) void state_policy_bwd_kernel(
    const float *logp, const float *entropy, const uint8_t *mask, const int32_t *state_graph_ptr,
    const float *dlogp, const float *dentropy, float *dlogit, float *inv_nvalid) {
  __shared__ float red[256];
  const int s = blockIdx.x, t = threadIdx.x;
  const int j0 = state_graph_ptr[s], j1 = state_graph_ptr[s + 1];
  float cs = 0.f;
  int cnt = 0;
  for (int j = j0 + t; j < j1; j += 256)
    if (mask[j]) { cs += dlogp[j]; ++cnt; }
  cs = block_sum(cs, red);
  const float nvalid = block_sum((float)cnt, red);
  const float de = dentropy[s], ent = entropy[s];
  for (int j = j0 + t; j < j1; j += 256) {
    float d = 0.f;
    if (mask[j]) {
      const float lp = logp[j], p = expf(lp);
      d = dlogp[j] - p * cs - de * p * (lp + ent);
    }
    dlogit[j] = d;
  }
  if (t == 0) inv_nvalid[s] = 1.f / nvalid;
}

// Backward of rowmlp_kernel for up to three layers, one block per ROWMLP_ROWS rows:
// given dout [n_rows, d_out[last]] and the saved post-activation outputs act[l], computes the
// pre-activation gradients dz[l] (stored, for the weight-gradient pass) and dx [n_rows, d_in[0]].
struct RowMlpBwdArgs {
  int n_layers, relu_last;
  const float *W[3];
  int d_in[3], d_out[3];
  const float *act[3];   // saved outputs of each layer
  const float *dout;     // [n_rows, d_out[last]]
  int64_t n_rows;
  float *dz[3];          // [n_rows, d_out[l]]
  float *dx;             // [n_rows, d_in[0]] nullable
};

template <int ROWMLP_ROWS>
__global__ __launch_bounds__(256) void rowmlp_bwd_kernel(const RowMlpBwdArgs a) {
  extern __shared__ float sm[];
  int dmax = a.d_in[0];
  for (int l = 0; l < a.n_layers; ++l) dmax = a.d_out[l] > dmax ? a.d_out[l] : dmax;
  float *cur = sm, *nxt = sm + ROWMLP_ROWS * dmax;
  const int64_t row0 = (int64_t)blockIdx.x * ROWMLP_ROWS;
  const int L = a.n_layers;
  // dz of the last layer
  {
    const int dout = a.d_out[L - 1];
    for (int i = threadIdx.x; i < ROWMLP_ROWS * dout; i += blockDim.x) {
      const int r = i / dout, f = i - r * dout;
      const int64_t row = row0 + r;
      float v = 0.f;
      if (row < a.n_rows) {
        v = a.dout[row * dout + f];
        if (a.relu_last && !(a.act[L - 1][row * dout + f] > 0.f)) v = 0.f;
        a.dz[L - 1][row * dout + f] = v;
      }
      cur[r * dmax + f] = v;
    }
  }
  __syncthreads();
  for (int l = L - 1; l >= 0; --l) {
    // dy_in[k] = sum_f dz[l][f] W[l][k, f]; then mask by layer l-1's activation
    const int din = a.d_in[l], dout = a.d_out[l];
    if (l == 0 && !a.dx) break;
    for (int k = threadIdx.x; k < din; k += blockDim.x) {
      float acc[ROWMLP_ROWS];
#pragma unroll
      for (int r = 0; r < ROWMLP_ROWS; ++r) acc[r] = 0.f;
      const float *wrow = a.W[l] + (size_t)k * dout;
#pragma unroll 8
      for (int f = 0; f < dout; ++f) {
        const float w = wrow[f];
#pragma unroll
        for (int r = 0; r < ROWMLP_ROWS; ++r) acc[r] = fmaf(cur[r * dmax + f], w, acc[r]);
      }
#pragma unroll
      for (int r = 0; r < ROWMLP_ROWS; ++r) {
        const int64_t row = row0 + r;
        float v = acc[r];
        if (row < a.n_rows) {
          if (l > 0) {
            if (!(a.act[l - 1][row * din + k] > 0.f)) v = 0.f;
            a.dz[l - 1][row * din + k] = v;
          } else {
            a.dx[row * din + k] = v;
          }
        } else {
          v = 0.f;
        }
        nxt[r * dmax + k] = v;
      }
    }
    __syncthreads();
    float *t = cur; cur = nxt; nxt = t;
  }
}

// Weight gradient of one affine layer over a modest number of rows, deterministic:
//   dW[k, f] += sum_rows x[row, k] dz[row, f],  db[f] += sum_rows dz[row, f]
// x = [x1 | x2] (x2 nullable). One thread per (k, f) walks a chunk of rows in order (blockIdx.y =
// chunk). With one chunk the sums are added to dW / db directly; with several, chunk c writes
// partial[c][k][f] (k = din is the bias row) and the fixed-order reduction of the weight-gradient
// kernels adds them up.
__global__ void small_wgrad_kernel(const float *x1, int w1, const float *x2, int w2,
                                   const float *dz, int64_t n_rows, int rows_per_chunk, int din, int dout,
                                   float *dW, float *db, float *partial) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (int64_t)(din + 1) * dout) return;
  const int k = (int)(i / dout), f = (int)(i - (int64_t)k * dout);
  const int64_t r0 = (int64_t)blockIdx.y * rows_per_chunk;
  const int64_t r1 = r0 + rows_per_chunk < n_rows ? r0 + rows_per_chunk : n_rows;
  // rows are added in order, eight requested at a time (a plain loop waits for every row's loads)
  const float *xp = k < w1 ? x1 + k : (k < din ? x2 + (k - w1) : nullptr);
  const int xs = k < w1 ? w1 : w2;
  float acc = 0.f;
  for (int64_t r = r0; r < r1; r += 8) {
    float xv[8], dv[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int64_t ri = r + i < r1 ? r + i : r1 - 1;
      dv[i] = dz[ri * dout + f];
      xv[i] = xp ? xp[ri * xs] : 1.f;
    }
#pragma unroll
    for (int i = 0; i < 8; ++i)
      if (r + i < r1) acc = xp ? fmaf(xv[i], dv[i], acc) : acc + dv[i];
  }
  if (partial) partial[(size_t)blockIdx.y * (din + 1) * dout + i] = acc;
  else if (k == din) db[f] += acc;
  else dW[(size_t)k * dout + f] += acc;
}

// Clipped-surrogate objective of Section 3.3.4 and its derivatives w.r.t. the heads' outputs, one
// block for the whole minibatch (S is a few hundred at most; the means are block reductions in a
// fixed order). dlogp must be zero on entry: only the taken slots are written. A recorded action
// outside its state's slots, or on a masked slot, touches nothing of that state and turns all
// four entries of J into NaN.
__global__ __launch_bounds__(256) void ppo_objective_kernel(
    const float *logp, const float *value, const float *entropy, const int32_t *state_graph_ptr,
    const uint8_t *mask, const int32_t *action, const float *old_logp, const float *advantage, const float *v_target,
    int S, float eps, float c1, float c2, float *J, float *dlogp, float *dvalue, float *dentropy) {
  __shared__ float red[256];
  const int t = threadIdx.x;
  const float inv = 1.f / (float)(S > 0 ? S : 1);
  float clip = 0.f, vf = 0.f, ent = 0.f, bad = 0.f;
  for (int s = t; s < S; s += 256) {
    const int j0 = state_graph_ptr[s], n_slots = state_graph_ptr[s + 1] - j0, act = action[s];
    if (act < 0 || act >= n_slots || !mask[j0 + act]) {
      bad = 1.f;
      dvalue[s] = 0.f;
      dentropy[s] = 0.f;
      continue;
    }
    const int j = j0 + act;
    const float A = advantage[s];
    const float ratio = expf(logp[j] - old_logp[s]);
    const float s1 = ratio * A;
    const float s2 = fminf(fmaxf(ratio, 1.f - eps), 1.f + eps) * A;
    clip -= fminf(s1, s2);
    dlogp[j] = s1 <= s2 ? -s1 * inv : 0.f;
    const float dv = value[s] - v_target[s];
    vf += dv * dv;
    dvalue[s] = 2.f * c1 * dv * inv;
    ent -= entropy[s];
    dentropy[s] = -c2 * inv;
  }
  clip = block_sum(clip, red) * inv;
  vf = block_sum(vf, red) * inv;
  ent = block_sum(ent, red) * inv;
  bad = block_sum(bad, red);
  if (t == 0) {
    const float nan = __int_as_float(0x7fc00000);
    J[0] = bad > 0.f ? nan : clip + c1 * vf + c2 * ent;
    J[1] = bad > 0.f ? nan : clip;
    J[2] = bad > 0.f ? nan : vf;
    J[3] = bad > 0.f ? nan : ent;
  }
}
