// Small fp32 kernels on per-graph and per-state data: the readout MLP of the global-update layer
// (Section 3.4), the policy and value heads with invalid-action masking (Section 3.3.2), and
// their backward passes. G and S rows only -- latency-bound, plain vector ALU code.
#pragma once
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

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

template <int ROWMLP_ROWS>
__global__ __launch_bounds__(256) void rowmlp_kernel(const RowMlpArgs a) {
  extern __shared__ float sm[];          // two buffers of ROWMLP_ROWS * dmax floats
  int dmax = a.d_in[0];
  for (int l = 0; l < a.n_layers; ++l) dmax = a.d_out[l] > dmax ? a.d_out[l] : dmax;
  float *cur = sm, *nxt = sm + ROWMLP_ROWS * dmax;
  const int64_t row0 = (int64_t)blockIdx.x * ROWMLP_ROWS;
  for (int i = threadIdx.x; i < ROWMLP_ROWS * a.d_in[0]; i += blockDim.x) {
    const int r = i / a.d_in[0], k = i - r * a.d_in[0];
    const int64_t row = row0 + r;
    float v = 0.f;
    if (row < a.n_rows) v = k < a.w1 ? a.in1[row * a.w1 + k] : a.in2[row * a.w2 + (k - a.w1)];
    cur[r * dmax + k] = v;
  }
  __syncthreads();
  for (int l = 0; l < a.n_layers; ++l) {
    const int din = a.d_in[l], dout = a.d_out[l];
    const bool relu = a.relu_last || (l + 1 < a.n_layers);
    for (int f = threadIdx.x; f < dout; f += blockDim.x) {
      float acc[ROWMLP_ROWS];
      const float bv = a.b[l][f];
#pragma unroll
      for (int r = 0; r < ROWMLP_ROWS; ++r) acc[r] = bv;
#pragma unroll 8
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
// and the mean embedding of the valid slots (input of the value head).
__global__ __launch_bounds__(256) void state_policy_kernel(
    const float *logit, const uint8_t *mask, const int32_t *state_graph_ptr, const float *emb,
    int H, float *logp, float *entropy, int32_t *action, float *zmean) {
  __shared__ float red[256];
  __shared__ int redi[256];
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
  // mean embedding of the valid slots: 256 / H groups of threads take every (256/H)-th slot,
  // four independent partial sums each; partials are combined in a fixed order
  const int ng = 256 / H, f = t % H, q = t / H;     // H is 64, 128 or 256
  float p0 = 0.f, p1 = 0.f, p2 = 0.f, p3 = 0.f;
  int j = j0 + q;
  for (; j + 3 * ng < j1; j += 4 * ng) {
    const float v0 = emb[(size_t)j * H + f], v1 = emb[(size_t)(j + ng) * H + f];
    const float v2 = emb[(size_t)(j + 2 * ng) * H + f], v3 = emb[(size_t)(j + 3 * ng) * H + f];
    p0 += mask[j] ? v0 : 0.f;
    p1 += mask[j + ng] ? v1 : 0.f;
    p2 += mask[j + 2 * ng] ? v2 : 0.f;
    p3 += mask[j + 3 * ng] ? v3 : 0.f;
  }
  for (; j < j1; j += ng) p0 += mask[j] ? emb[(size_t)j * H + f] : 0.f;
  red[t] = (p0 + p1) + (p2 + p3);
  __syncthreads();
  if (q == 0) {
    float acc = red[f];
    for (int k = 1; k < ng; ++k) acc += red[k * H + f];
    zmean[(size_t)s * H + f] = acc / nvalid;
  }
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
// x = [x1 | x2] (x2 nullable). One thread per (k, f) walks the rows in order.
__global__ void small_wgrad_kernel(const float *x1, int w1, const float *x2, int w2,
                                   const float *dz, int64_t n_rows, int din, int dout, float *dW,
                                   float *db) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (int64_t)(din + 1) * dout) return;
  const int k = (int)(i / dout), f = (int)(i - (int64_t)k * dout);
  float acc = 0.f;
  if (k == din) {
    for (int64_t r = 0; r < n_rows; ++r) acc += dz[r * dout + f];
    db[f] += acc;
  } else {
    if (k < w1)
      for (int64_t r = 0; r < n_rows; ++r) acc = fmaf(x1[r * w1 + k], dz[r * dout + f], acc);
    else
      for (int64_t r = 0; r < n_rows; ++r) acc = fmaf(x2[r * w2 + (k - w1)], dz[r * dout + f], acc);
    dW[(size_t)k * dout + f] += acc;
  }
}
