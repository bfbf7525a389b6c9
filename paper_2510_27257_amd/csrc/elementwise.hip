// HBM-bound kernels of the units: normalisation forward/backward (Pre-Attn and
// Pre-MLP units, Eq. 1-2), GELU / SwiGLU, rotary embedding, bias-gradient
// column sums and the attention-backward row dot.  All math in fp32; storage
// type T is float or bf16.  Every global access is a 16-byte (bf16) or 32-byte
// (fp32) vector per lane, lanes contiguous.
#include "common.h"

// ======================================================================
// Norm forward: one 256-thread group per token row, the row in registers (chunk c of a thread covers
// elements (c*256 + tid)*8 .. +7), mean and variance (two passes over the registers) through cross-lane
// reductions and LDS.  Many short-lived groups keep several rows of loads in flight per compute unit
// and fill in wherever other streams' kernels leave room (one wave per row measured 4.5 TB/s at
// [6144, 4096] bf16, this shape 6 TB/s).
// ======================================================================
__device__ __forceinline__ float block_sum_256(float v, float *red) {
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  v = wave_sum(v);
  if (lane == 0) red[wv] = v;
  __syncthreads();
  return (red[0] + red[1]) + (red[2] + red[3]);
}

template <typename T, int NORM, int NCH>
__global__ __launch_bounds__(256) void norm_fwd_kernel(const T *__restrict__ x, const T *__restrict__ gamma,
                                                       const T *__restrict__ beta, T *__restrict__ y,
                                                       float *__restrict__ stats, int rows, int h, float eps) {
  __shared__ float red[8];
  const int tid = threadIdx.x;
  const int row = blockIdx.x;
  const T *xr = x + (size_t)row * h;
  float v[NCH][8];
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < NCH; c++) {
    const int col = (c * 256 + tid) * 8;
    if (col < h) {
      Vec8<T>::load(xr + col, v[c]);
#pragma unroll
      for (int i = 0; i < 8; i++) s += (NORM == STP_NORM_LN) ? v[c][i] : v[c][i] * v[c][i];
    }
  }
  s = block_sum_256(s, red);
  float mean = 0.f, rstd;
  if (NORM == STP_NORM_LN) {
    mean = s / (float)h;
    float q = 0.f;
#pragma unroll
    for (int c = 0; c < NCH; c++) {
      const int col = (c * 256 + tid) * 8;
      if (col < h) {
#pragma unroll
        for (int i = 0; i < 8; i++) { float d = v[c][i] - mean; q += d * d; }
      }
    }
    q = block_sum_256(q, red + 4);
    rstd = 1.0f / sqrtf(q / (float)h + eps);
  } else {
    rstd = 1.0f / sqrtf(s / (float)h + eps);
  }
  if (tid == 0) { stats[2 * (size_t)row] = mean; stats[2 * (size_t)row + 1] = rstd; }
  T *yr = y + (size_t)row * h;
#pragma unroll
  for (int c = 0; c < NCH; c++) {
    const int col = (c * 256 + tid) * 8;
    if (col < h) {
      float g[8], b[8], o[8];
      Vec8<T>::load(gamma + col, g);
      if (NORM == STP_NORM_LN && beta) Vec8<T>::load(beta + col, b);
      else {
#pragma unroll
        for (int i = 0; i < 8; i++) b[i] = 0.f;
      }
#pragma unroll
      for (int i = 0; i < 8; i++) o[i] = (v[c][i] - mean) * rstd * g[i] + b[i];
      Vec8<T>::store(yr + col, o);
    }
  }
}

// ======================================================================
// Norm backward (+ residual gradient, Eq. 2): one 256-thread group per row,
// groups stride over rows and keep the gain/bias gradient partials of their
// columns in registers; the partials go to the workspace and a second kernel
// adds them up in a fixed order (deterministic, no float atomics).
// With RSUM the column sums of the residual-path gradient are collected the same way: that gradient is read
// here anyway, and (1/t) of its column sum is the bias gradient of the row-parallel linear layer of the
// unit above (Eq. 1 adds b/t on every rank).  Partials of a group: [gain | bias | resid sum] (3h floats; 2h without RSUM).
// chunk c of a thread covers elements (c*256 + tid)*8 .. +7
// ======================================================================
// Eight elements as loaded, unconverted: what a thread keeps of the NEXT row while it works on the current one.
template <typename T> struct Raw8;
template <> struct Raw8<float> {
  float4 a, b;
  __device__ __forceinline__ void load(const float *p) {
    a = *reinterpret_cast<const float4 *>(p);
    b = *reinterpret_cast<const float4 *>(p + 4);
  }
  __device__ __forceinline__ void get(float (&v)[8]) const {
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  }
};
template <> struct Raw8<bf16_t> {
  uint4 u;
  __device__ __forceinline__ void load(const bf16_t *p) { u = *reinterpret_cast<const uint4 *>(p); }
  __device__ __forceinline__ void get(float (&v)[8]) const {
    const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int i = 0; i < 4; i++) {
      v[2 * i] = __uint_as_float(w[i] << 16);
      v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
};

template <typename T, int NORM, int NCH, bool RSUM>
__global__ __launch_bounds__(256) void norm_bwd_kernel(const T *__restrict__ x, const T *__restrict__ gamma,
                                                       const float *__restrict__ stats, const T *__restrict__ dy,
                                                       const T *__restrict__ dres, T *__restrict__ dx,
                                                       float *__restrict__ partial, int rows, int h) {
  __shared__ float red[2][4][2];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  float gam[NCH][8], acc_g[NCH][8], acc_b[NCH][8], acc_r[NCH][8];   // acc_r unused (and removed by the compiler) without RSUM
#pragma unroll
  for (int c = 0; c < NCH; c++) {
    int col = (c * 256 + tid) * 8;
#pragma unroll
    for (int i = 0; i < 8; i++) { gam[c][i] = 0.f; acc_g[c][i] = 0.f; acc_b[c][i] = 0.f; acc_r[c][i] = 0.f; }
    if (col < h) Vec8<T>::load(gamma + col, gam[c]);
  }
  // A row is one load latency, a reduction over the group and a store; a group works through its rows one
  // after the other, so the loads of the next row are issued before the current row is touched.
  Raw8<T> nx[NCH], nd[NCH], nr[NCH];
  float nmean = 0.f, nrstd = 0.f;
  auto fetch = [&](int row) {
    nmean = stats[2 * (size_t)row];
    nrstd = stats[2 * (size_t)row + 1];
    const size_t off = (size_t)row * h;
#pragma unroll
    for (int c = 0; c < NCH; c++) {
      int col = (c * 256 + tid) * 8;
      if (col < h) {
        nx[c].load(x + off + col);
        nd[c].load(dy + off + col);
        if (dres) nr[c].load(dres + off + col);
      }
    }
  };
  if ((int)blockIdx.x < rows) fetch(blockIdx.x);
  int it = 0;
  for (int row = blockIdx.x; row < rows; row += gridDim.x, it++) {
    const float mean = nmean, rstd = nrstd;
    const size_t off = (size_t)row * h;
    float xh[NCH][8], g[NCH][8], rs[NCH][8];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int c = 0; c < NCH; c++) {
      int col = (c * 256 + tid) * 8;
      if (col < h) {
        float xv[8], dv[8];
        nx[c].get(xv);
        nd[c].get(dv);
        if (dres) nr[c].get(rs[c]);
#pragma unroll
        for (int i = 0; i < 8; i++) {
          if (RSUM) acc_r[c][i] += rs[c][i];
          xh[c][i] = (xv[i] - mean) * rstd;
          acc_g[c][i] += dv[i] * xh[c][i];
          acc_b[c][i] += dv[i];
          g[c][i] = dv[i] * gam[c][i];
          s1 += g[c][i];
          s2 += g[c][i] * xh[c][i];
        }
      }
    }
    if (row + (int)gridDim.x < rows) fetch(row + gridDim.x);
    s1 = wave_sum(s1);
    s2 = wave_sum(s2);
    if (lane == 0) { red[it & 1][wv][0] = s1; red[it & 1][wv][1] = s2; }
    __syncthreads();
    float c1 = (red[it & 1][0][0] + red[it & 1][1][0]) + (red[it & 1][2][0] + red[it & 1][3][0]);
    float c2 = (red[it & 1][0][1] + red[it & 1][1][1]) + (red[it & 1][2][1] + red[it & 1][3][1]);
    c1 = (NORM == STP_NORM_LN) ? c1 / (float)h : 0.f;
    c2 = c2 / (float)h;
#pragma unroll
    for (int c = 0; c < NCH; c++) {
      int col = (c * 256 + tid) * 8;
      if (col < h) {
        float o[8];
#pragma unroll
        for (int i = 0; i < 8; i++) {
          o[i] = rstd * (g[c][i] - c1 - xh[c][i] * c2);
          if (dres) o[i] += rs[c][i];
        }
        Vec8<T>::store(dx + off + col, o);
      }
    }
  }
  if (partial) {
    float *pg = partial + (size_t)blockIdx.x * (RSUM ? 3 : 2) * h;
#pragma unroll
    for (int c = 0; c < NCH; c++) {
      int col = (c * 256 + tid) * 8;
      if (col < h) {
        Vec8<float>::store(pg + col, acc_g[c]);
        Vec8<float>::store(pg + h + col, acc_b[c]);
        if (RSUM) Vec8<float>::store(pg + 2 * h + col, acc_r[c]);
      }
    }
  }
}

// Column c of the partials belongs to segment c / seg_w, column c % seg_w of that segment's output:
//   out_k[c % seg_w] += scale_k * sum_{p < nparts} partial[p*stride + c]      (a NULL out_k skips the segment)
// in a fixed order: a 256-thread group owns 64 columns; thread (c, g) adds up rows g, g+4, g+8, ... (8 independent
// loads in flight), then the four row-group sums are combined 0+1+2+3 through LDS.  The gain, bias and
// residual-sum partials of a norm lie side by side (three segments of h columns) and are reduced by one launch;
// a plain column sum is one segment.
struct ReduceOut { float *out[3]; float scale[3]; };
__global__ __launch_bounds__(256) void partial_reduce_kernel(const float *__restrict__ partial, int nparts,
                                                            size_t stride, int n, int seg_w, ReduceOut ro) {
  __shared__ float red[4][64];
  const int cl = threadIdx.x & 63, g = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + cl;
  const int seg = c < n ? c / seg_w : 0;
  float *const dst = seg == 0 ? ro.out[0] : (seg == 1 ? ro.out[1] : ro.out[2]);
  const float scale = seg == 0 ? ro.scale[0] : (seg == 1 ? ro.scale[1] : ro.scale[2]);
  float s = 0.f;
  if (c < n && dst) {
    int p = g;
    for (; p + 28 < nparts; p += 32) {
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; u++) v[u] = partial[(size_t)(p + 4 * u) * stride + c];
#pragma unroll
      for (int u = 0; u < 8; u++) s += v[u];
    }
    for (; p < nparts; p += 4) s += partial[(size_t)p * stride + c];
  }
  red[g][cl] = s;
  __syncthreads();
  if (g == 0 && c < n && dst) dst[c - seg * seg_w] += scale * (((red[0][cl] + red[1][cl]) + red[2][cl]) + red[3][cl]);
}

// ======================================================================
// Column sums (bias gradients), stage 1: a 256-thread group owns a CS_ROWS-row x 256-column patch as
// 8 row-lanes x 32 column chunks; every thread adds CS_ROWS / 8 rows in batches of 8 independent 16-byte
// loads, the 8 row-lanes are combined through LDS in a fixed order, and the patch sum goes to the
// workspace; partial_reduce_kernel adds the patches of a column.  (Taller patches were no faster at
// [6144, 4096] and slower for narrower tensors, whose launch they leave with too few workgroups.)
// ======================================================================
constexpr int CS_ROWS = STP_COLSUM_ROWS;

// RL row-lanes x (256 / RL) column chunks of 8: RL = 8 gives 64-row x 256-column patches with one batch of 8
// loads per thread.  (RL = 2, patches of 1024 columns whose row pieces are 2 KB of contiguous memory, takes four
// batches per thread one after the other and measured half the rate.)
template <typename T, int RL>
__global__ __launch_bounds__(256) void colsum_kernel(const T *__restrict__ x, int rows, int n,
                                                     float *__restrict__ partial) {
  constexpr int CC = 256 / RL, PER = CS_ROWS / RL;      // column chunks per group, rows per thread
  __shared__ float red[RL][CC][9];
  const int cc = threadIdx.x % CC, rl = threadIdx.x / CC;
  const int col = (blockIdx.x * CC + cc) * 8;
  const int r0 = blockIdx.y * CS_ROWS;
  float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  if (col < n) {
#pragma unroll
    for (int b = 0; b < PER / 8; b++) {
      float v[8][8];
#pragma unroll
      for (int u = 0; u < 8; u++) {
        const int r = r0 + rl + RL * (8 * b + u);
        if (r < rows) Vec8<T>::load(x + (size_t)r * n + col, v[u]);
        else {
#pragma unroll
          for (int i = 0; i < 8; i++) v[u][i] = 0.f;
        }
      }
#pragma unroll
      for (int u = 0; u < 8; u++)
#pragma unroll
        for (int i = 0; i < 8; i++) acc[i] += v[u][i];
    }
  }
#pragma unroll
  for (int i = 0; i < 8; i++) red[rl][cc][i] = acc[i];
  __syncthreads();
  if (rl == 0 && col < n) {
    float s[8];
#pragma unroll
    for (int i = 0; i < 8; i++) {
      float t = 0.f;
#pragma unroll
      for (int k = 0; k < RL; k++) t += red[k][cc][i];
      s[i] = t;
    }
    Vec8<float>::store(partial + (size_t)blockIdx.y * n + col, s);
  }
}

// ======================================================================
// Activations
// ======================================================================
template <typename T>
__global__ __launch_bounds__(256) void gelu_fwd_kernel(const T *__restrict__ x, T *__restrict__ y, size_t n8) {
  for (size_t i = blockIdx.x * (size_t)256 + threadIdx.x; i < n8; i += (size_t)gridDim.x * 256) {
    float v[8];
    Vec8<T>::load(x + i * 8, v);
#pragma unroll
    for (int k = 0; k < 8; k++) v[k] = gelu_t<T>(v[k]);
    Vec8<T>::store(y + i * 8, v);
  }
}
template <typename T>
__global__ __launch_bounds__(256) void gelu_bwd_kernel(const T *__restrict__ x, const T *__restrict__ dy,
                                                       T *__restrict__ dx, size_t n8) {
  for (size_t i = blockIdx.x * (size_t)256 + threadIdx.x; i < n8; i += (size_t)gridDim.x * 256) {
    float v[8], d[8];
    Vec8<T>::load(x + i * 8, v);
    Vec8<T>::load(dy + i * 8, d);
#pragma unroll
    for (int k = 0; k < 8; k++) d[k] *= gelu_grad_t<T>(v[k]);
    Vec8<T>::store(dx + i * 8, d);
  }
}
template <typename T>
__global__ __launch_bounds__(256) void swiglu_fwd_kernel(const T *__restrict__ gate, const T *__restrict__ up,
                                                         T *__restrict__ y, size_t n8) {
  for (size_t i = blockIdx.x * (size_t)256 + threadIdx.x; i < n8; i += (size_t)gridDim.x * 256) {
    float g[8], u[8];
    Vec8<T>::load(gate + i * 8, g);
    Vec8<T>::load(up + i * 8, u);
#pragma unroll
    for (int k = 0; k < 8; k++) g[k] = g[k] * sigmoid_f(g[k]) * u[k];
    Vec8<T>::store(y + i * 8, g);
  }
}
template <typename T>
__global__ __launch_bounds__(256) void swiglu_bwd_kernel(const T *__restrict__ gate, const T *__restrict__ up,
                                                         const T *__restrict__ dy, T *__restrict__ dgate,
                                                         T *__restrict__ dup, size_t n8) {
  for (size_t i = blockIdx.x * (size_t)256 + threadIdx.x; i < n8; i += (size_t)gridDim.x * 256) {
    float g[8], u[8], d[8], dg[8], du[8];
    Vec8<T>::load(gate + i * 8, g);
    Vec8<T>::load(up + i * 8, u);
    Vec8<T>::load(dy + i * 8, d);
#pragma unroll
    for (int k = 0; k < 8; k++) {
      float sg = sigmoid_f(g[k]);
      du[k] = d[k] * g[k] * sg;
      dg[k] = d[k] * u[k] * sg * (1.0f + g[k] * (1.0f - sg));
    }
    Vec8<T>::store(dgate + i * 8, dg);
    Vec8<T>::store(dup + i * 8, du);
  }
}

// ======================================================================
// Row softmax on its own (the attention kernels fuse theirs; this pair exists so that the normalisation can be
// measured against the memory system by itself).  A 256-thread group per row, the row in registers
// (chunk c of a thread covers elements (c*256 + tid)*8 .. +7), row maximum and row sum through cross-lane
// reductions and LDS.  causal: the rows are stacked [n, n] squares; element j of row r is masked for j > r mod n.
//   forward : y = softmax(scale * x)
//   backward: dx = scale * y o (dy - rowsum(dy o y))
// ======================================================================
__device__ __forceinline__ float block_reduce_256(float v, bool is_max, float *red, int it) {
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  v = is_max ? wave_max(v) : wave_sum(v);
  if (lane == 0) red[(it & 1) * 4 + wv] = v;
  __syncthreads();
  const float *r = red + (it & 1) * 4;
  return is_max ? fmaxf(fmaxf(r[0], r[1]), fmaxf(r[2], r[3])) : (r[0] + r[1]) + (r[2] + r[3]);
}

template <typename T, int NCH>
__global__ __launch_bounds__(256) void softmax_fwd_kernel(const T *__restrict__ x, T *__restrict__ y, int rows, int n,
                                                          float scale_log2e, int causal) {
  __shared__ float red[16];
  const int tid = threadIdx.x;
  const int row = blockIdx.x;
  const int limit = causal ? (row % n) + 1 : n;      // keys 0 .. limit-1 take part
  const T *xr = x + (size_t)row * n;
  float v[NCH][8];
  float mx = -INFINITY;
#pragma unroll
  for (int c = 0; c < NCH; c++) {
    const int col = (c * 256 + tid) * 8;
    if (col < limit) {
      Vec8<T>::load(xr + col, v[c]);
#pragma unroll
      for (int i = 0; i < 8; i++) {
        v[c][i] = col + i < limit ? v[c][i] * scale_log2e : -INFINITY;
        mx = fmaxf(mx, v[c][i]);
      }
    } else {
#pragma unroll
      for (int i = 0; i < 8; i++) v[c][i] = -INFINITY;
    }
  }
  mx = block_reduce_256(mx, true, red, 0);
  float sum = 0.f;
#pragma unroll
  for (int c = 0; c < NCH; c++)
#pragma unroll
    for (int i = 0; i < 8; i++) {
      v[c][i] = __builtin_amdgcn_exp2f(v[c][i] - mx);      // exp2(-inf) = 0 for the masked keys
      sum += v[c][i];
    }
  sum = block_reduce_256(sum, false, red, 1);
  const float inv = 1.0f / sum;
  T *yr = y + (size_t)row * n;
#pragma unroll
  for (int c = 0; c < NCH; c++) {
    const int col = (c * 256 + tid) * 8;
    if (col < n) {
      float o[8];
#pragma unroll
      for (int i = 0; i < 8; i++) o[i] = v[c][i] * inv;
      Vec8<T>::store(yr + col, o);
    }
  }
}

template <typename T, int NCH>
__global__ __launch_bounds__(256) void softmax_bwd_kernel(const T *__restrict__ y, const T *__restrict__ dy, T *__restrict__ dx,
                                                          int rows, int n, float scale) {
  __shared__ float red[16];
  const int tid = threadIdx.x;
  const size_t off = (size_t)blockIdx.x * n;
  float p[NCH][8], g[NCH][8];
  float dot = 0.f;
#pragma unroll
  for (int c = 0; c < NCH; c++) {
    const int col = (c * 256 + tid) * 8;
    if (col < n) {
      Vec8<T>::load(y + off + col, p[c]);
      Vec8<T>::load(dy + off + col, g[c]);
#pragma unroll
      for (int i = 0; i < 8; i++) dot += p[c][i] * g[c][i];
    }
  }
  dot = block_reduce_256(dot, false, red, 0);
#pragma unroll
  for (int c = 0; c < NCH; c++) {
    const int col = (c * 256 + tid) * 8;
    if (col < n) {
      float o[8];
#pragma unroll
      for (int i = 0; i < 8; i++) o[i] = scale * p[c][i] * (g[c][i] - dot);
      Vec8<T>::store(dx + off + col, o);
    }
  }
}

// ======================================================================
// Rotary embedding, in place on the Q and K heads of qkv [T, (n + 2 n_kv) d] (the first nrot = n + n_kv heads
// of a row).  One thread rotates 8 pairs (i, i + d/2) of one head of one token.
// ======================================================================
template <typename T>
__global__ __launch_bounds__(256) void rope_kernel(T *__restrict__ qkv, int tokens, int seq, int nrot, int row_width, int d,
                                                   float log2_base, float sign) {
  const int half = d / 2, per_head = half / 8;
  size_t total = (size_t)tokens * nrot * per_head;
  size_t idx = blockIdx.x * (size_t)256 + threadIdx.x;
  if (idx >= total) return;
  int c = idx % per_head;
  size_t r = idx / per_head;
  int head = r % nrot;     // Q heads, then K heads (contiguous in a row)
  size_t tok = r / nrot;
  int pos = tok % seq;
  T *p = qkv + tok * (size_t)row_width + (size_t)head * d + c * 8;
  float a[8], b[8], oa[8], ob[8];
  Vec8<T>::load(p, a);
  Vec8<T>::load(p + half, b);
#pragma unroll
  for (int i = 0; i < 8; i++) {
    float inv_freq = exp2f(-2.0f * (float)(c * 8 + i) / (float)d * log2_base);
    float ang = (float)pos * inv_freq;
    float sn, cs;
    sincosf(ang, &sn, &cs);
    sn *= sign;
    oa[i] = a[i] * cs - b[i] * sn;
    ob[i] = b[i] * cs + a[i] * sn;
  }
  Vec8<T>::store(p, oa);
  Vec8<T>::store(p + half, ob);
}

// ======================================================================
// delta[b, head, i] = sum_c dctx[tok, head*d + c] * ctx[tok, head*d + c]
// (the rowsum(dP o P) term of the softmax backward).  A (token, head) pair is d contiguous elements at
// (tok*n + head)*d, so consecutive pairs are consecutive memory: a lane takes 8 elements, LPP = d/8 lanes a
// pair, a wave 64/LPP pairs (1 KB contiguous per operand), and the pair's lanes are summed by cross-lane
// operand modifiers.  LPP must be 2, 4, 8 or 16; other head dimensions take the one-pair-per-wave kernel below.
// ======================================================================
template <typename T, int LPP>
__global__ __launch_bounds__(256) void rowdot_packed_kernel(const T *__restrict__ a, const T *__restrict__ b,
                                                            float *__restrict__ delta, size_t pairs, int seq, int n) {
  const size_t v = blockIdx.x * (size_t)256 + threadIdx.x;     // 8-element vector index
  const size_t pair = v / LPP;
  float s = 0.f;
  if (pair < pairs) {
    float x[8], y[8];
    Vec8<T>::load(a + v * 8, x);
    Vec8<T>::load(b + v * 8, y);
#pragma unroll
    for (int i = 0; i < 8; i++) s += x[i] * y[i];
  }
  s += dpp_f32<0xB1>(s);                           // lanes 4k .. 4k+3
  if (LPP >= 4) s += dpp_f32<0x4E>(s);
  if (LPP >= 8) s += dpp_f32<0x141>(s);            // 8 lanes
  if (LPP >= 16) s += dpp_f32<0x140>(s);           // 16 lanes
  if (pair < pairs && v % LPP == 0) {
    const size_t tok = pair / n, head = pair % n;
    delta[((tok / seq) * n + head) * seq + tok % seq] = s;
  }
}
template <typename T>
__global__ __launch_bounds__(256) void rowdot_kernel(const T *__restrict__ a, const T *__restrict__ b,
                                                     float *__restrict__ delta, int tokens, int seq, int n, int d) {
  const int lane = threadIdx.x & 63;
  size_t w = blockIdx.x * (size_t)4 + (threadIdx.x >> 6);
  if (w >= (size_t)tokens * n) return;
  int head = w % n;
  size_t tok = w / n;
  float s = 0.f;
  int col = lane * 8;
  if (col < d) {
    float u[8], v[8];
    Vec8<T>::load(a + tok * (size_t)(n * d) + head * d + col, u);
    Vec8<T>::load(b + tok * (size_t)(n * d) + head * d + col, v);
#pragma unroll
    for (int i = 0; i < 8; i++) s += u[i] * v[i];
  }
  s = wave_sum(s);
  if (lane == 0) {
    size_t bidx = tok / seq, i = tok % seq;
    delta[(bidx * n + head) * seq + i] = s;
  }
}

// ======================================================================
// Host launchers
// ======================================================================
static inline int ew_grid(size_t n8) {
  size_t g = (n8 + 255) / 256;
  return (int)(g > 4096 ? 4096 : (g ? g : 1));
}

template <typename T>
static int norm_fwd_dispatch(stp_ctx *ctx, int norm, int rows, int h, float eps, const void *x, const void *gamma,
                             const void *beta, void *y, float *stats, hipStream_t s) {
  dim3 grid(rows), block(256);
  int nch = (h + 2047) / 2048;
#define LAUNCH(NORM, NCH)                                                                               \
  hipLaunchKernelGGL((norm_fwd_kernel<T, NORM, NCH>), grid, block, 0, s, (const T *)x, (const T *)gamma, \
                     (const T *)beta, (T *)y, stats, rows, h, eps)
#define BY_NCH(NORM)                                   \
  if (nch <= 1) LAUNCH(NORM, 1);                       \
  else if (nch <= 2) LAUNCH(NORM, 2);                  \
  else if (nch <= 3) LAUNCH(NORM, 3);                  \
  else LAUNCH(NORM, 4);
  if (norm == STP_NORM_LN) { BY_NCH(STP_NORM_LN) } else { BY_NCH(STP_NORM_RMS) }
#undef BY_NCH
#undef LAUNCH
  STP_LAUNCH_CHECK(ctx);
  return STP_OK;
}

extern "C" int stp_norm_forward(stp_ctx *ctx, int dtype, int norm, int32_t T, int32_t h, float eps, const void *x,
                                const void *gamma, const void *beta, void *y, float *stats, void *hip_stream) {
  if (!ctx) return STP_EINVAL;
  if (!x || !gamma || !y || !stats) return stp_fail(ctx, STP_EINVAL, "stp_norm_forward: null pointer%s");
  if (T < 0 || h <= 0 || h % 8 || h > 8192) return stp_fail(ctx, STP_ESHAPE, "stp_norm_forward: h must be a multiple of 8, <= 8192%s");
  if (!stp_aligned16(x) || !stp_aligned16(gamma) || !stp_aligned16(y) || (beta && !stp_aligned16(beta)))
    return stp_fail(ctx, STP_EALIGN, "stp_norm_forward: pointers must be 16-byte aligned%s");
  if (norm != STP_NORM_LN && norm != STP_NORM_RMS) return stp_fail(ctx, STP_EINVAL, "stp_norm_forward: bad norm%s");
  if (T == 0) return STP_OK;
  hipStream_t s = (hipStream_t)hip_stream;
  if (dtype == STP_BF16) return norm_fwd_dispatch<bf16_t>(ctx, norm, T, h, eps, x, gamma, beta, y, stats, s);
  if (dtype == STP_F32) return norm_fwd_dispatch<float>(ctx, norm, T, h, eps, x, gamma, beta, y, stats, s);
  return stp_fail(ctx, STP_EINVAL, "stp_norm_forward: bad dtype%s");
}

template <typename T>
static int norm_bwd_dispatch(stp_ctx *ctx, int norm, int rows, int h, const void *x, const void *gamma,
                             const float *stats, const void *dy, const void *dres, void *dx, float *partial,
                             bool rsum, hipStream_t s) {
  dim3 grid(stp_norm_bwd_blocks(rows, h)), block(256);
  int nch = (h + 2047) / 2048;
#define LAUNCH(NORM, NCH)                                                                                         \
  do {                                                                                                            \
    if (rsum) hipLaunchKernelGGL((norm_bwd_kernel<T, NORM, NCH, true>), grid, block, 0, s, (const T *)x,          \
                                 (const T *)gamma, stats, (const T *)dy, (const T *)dres, (T *)dx, partial, rows, h); \
    else hipLaunchKernelGGL((norm_bwd_kernel<T, NORM, NCH, false>), grid, block, 0, s, (const T *)x,              \
                            (const T *)gamma, stats, (const T *)dy, (const T *)dres, (T *)dx, partial, rows, h);  \
  } while (0)
#define BY_NCH(NORM)                                   \
  if (nch <= 1) LAUNCH(NORM, 1);                       \
  else if (nch <= 2) LAUNCH(NORM, 2);                  \
  else if (nch <= 3) LAUNCH(NORM, 3);                  \
  else LAUNCH(NORM, 4);
  if (norm == STP_NORM_LN) { BY_NCH(STP_NORM_LN) } else { BY_NCH(STP_NORM_RMS) }
#undef BY_NCH
#undef LAUNCH
  STP_LAUNCH_CHECK(ctx);
  return STP_OK;
}

extern "C" int stp_norm_backward(stp_ctx *ctx, int dtype, int norm, int32_t T, int32_t h, const void *x,
                                 const void *gamma, const float *stats, const void *dy, const void *d_resid,
                                 void *dx, float *dgamma, float *dbeta, float *d_resid_sum, float d_resid_sum_scale,
                                 int lane, void *hip_stream) {
  if (!ctx) return STP_EINVAL;
  if (!x || !gamma || !stats || !dy || !dx) return stp_fail(ctx, STP_EINVAL, "stp_norm_backward: null pointer%s");
  if (T < 0 || h <= 0 || h % 8 || h > 8192) return stp_fail(ctx, STP_ESHAPE, "stp_norm_backward: h must be a multiple of 8, <= 8192%s");
  if (!stp_aligned16(x) || !stp_aligned16(gamma) || !stp_aligned16(dy) || !stp_aligned16(dx) ||
      (d_resid && !stp_aligned16(d_resid)))
    return stp_fail(ctx, STP_EALIGN, "stp_norm_backward: pointers must be 16-byte aligned%s");
  if (norm != STP_NORM_LN && norm != STP_NORM_RMS) return stp_fail(ctx, STP_EINVAL, "stp_norm_backward: bad norm%s");
  if (lane < 0 || lane > 2) return stp_fail(ctx, STP_EINVAL, "stp_norm_backward: lane must be 0..2%s");
  if (dtype != STP_BF16 && dtype != STP_F32) return stp_fail(ctx, STP_EINVAL, "stp_norm_backward: bad dtype%s");
  if (d_resid_sum && !d_resid) return stp_fail(ctx, STP_EINVAL, "stp_norm_backward: d_resid_sum without d_resid%s");
  if (T == 0) return STP_OK;
  hipStream_t s = (hipStream_t)hip_stream;
  const int blocks = stp_norm_bwd_blocks(T, h);
  const bool rsum = d_resid_sum != nullptr;
  const bool want_beta = dbeta && norm == STP_NORM_LN;
  float *partial = nullptr;
  if (dgamma || want_beta || rsum) {
    size_t lane_bytes;
    char *ws = stp_ws_lane(ctx, lane, &lane_bytes);
    size_t need = (size_t)blocks * (rsum ? 3 : 2) * h * sizeof(float);
    if (!ws || lane_bytes < need) return stp_fail(ctx, STP_ENOSPACE, "stp_norm_backward: workspace lane too small%s (need %ld bytes)", "", (long)need);
    partial = (float *)ws;
  }
  int rc = dtype == STP_BF16 ? norm_bwd_dispatch<bf16_t>(ctx, norm, T, h, x, gamma, stats, dy, d_resid, dx, partial, rsum, s)
                             : norm_bwd_dispatch<float>(ctx, norm, T, h, x, gamma, stats, dy, d_resid, dx, partial, rsum, s);
  if (rc != STP_OK) return rc;
  if (partial) {   // the partials of a row group lie side by side: [gain | bias | residual sum]
    const int segs = rsum ? 3 : 2;
    ReduceOut ro = {{dgamma, want_beta ? dbeta : nullptr, d_resid_sum}, {1.0f, 1.0f, d_resid_sum_scale}};
    hipLaunchKernelGGL(partial_reduce_kernel, dim3((segs * h + 63) / 64), dim3(256), 0, s, partial, blocks, (size_t)segs * h, segs * h, h, ro);
    STP_LAUNCH_CHECK(ctx);
  }
  return STP_OK;
}

// the two stages of a column sum with the partial sums at `partial` (slabs x N floats)
static int colsum_launch(stp_ctx *ctx, int dtype, int T, int N, const void *x, float scale, float *out, float *partial, hipStream_t s) {
  const int slabs = stp_colsum_slabs(T);
  dim3 grid((N / 8 + 31) / 32, slabs), block(256);
  if (dtype == STP_BF16) hipLaunchKernelGGL((colsum_kernel<bf16_t, 8>), grid, block, 0, s, (const bf16_t *)x, T, N, partial);
  else hipLaunchKernelGGL((colsum_kernel<float, 8>), grid, block, 0, s, (const float *)x, T, N, partial);
  STP_LAUNCH_CHECK(ctx);
  ReduceOut ro = {{out, nullptr, nullptr}, {scale, 0.f, 0.f}};
  hipLaunchKernelGGL(partial_reduce_kernel, dim3((N + 63) / 64), dim3(256), 0, s, partial, slabs, (size_t)N, N, N, ro);
  STP_LAUNCH_CHECK(ctx);
  return STP_OK;
}

extern "C" int stp_colsum(stp_ctx *ctx, int dtype, int32_t T, int32_t N, const void *x, float scale, float *out,
                          int lane, void *hip_stream) {
  if (!ctx) return STP_EINVAL;
  if (!x || !out) return stp_fail(ctx, STP_EINVAL, "stp_colsum: null pointer%s");
  if (T < 0 || N <= 0 || N % 8) return stp_fail(ctx, STP_ESHAPE, "stp_colsum: N must be a multiple of 8%s");
  if (!stp_aligned16(x)) return stp_fail(ctx, STP_EALIGN, "stp_colsum: x must be 16-byte aligned%s");
  if (lane < 0 || lane > 2) return stp_fail(ctx, STP_EINVAL, "stp_colsum: lane must be 0..2%s");
  if (dtype != STP_BF16 && dtype != STP_F32) return stp_fail(ctx, STP_EINVAL, "stp_colsum: bad dtype%s");
  if (T == 0) return STP_OK;
  size_t lane_bytes;
  char *ws = stp_ws_lane(ctx, lane, &lane_bytes);
  size_t need = (size_t)stp_colsum_slabs(T) * N * sizeof(float);
  if (!ws || lane_bytes < need) return stp_fail(ctx, STP_ENOSPACE, "stp_colsum: workspace lane too small%s (need %ld bytes)", "", (long)need);
  return colsum_launch(ctx, dtype, T, N, x, scale, out, (float *)ws, (hipStream_t)hip_stream);
}

// ======================================================================
// Column sum without the caller's workspace, for callers that cannot allocate device memory or hand a
// workspace over (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc):
// the stage-1 partials live in a fixed array in the library's device image.  Each GPU the library runs on
// holds its own copy of the array at its own address; the address is looked up once per device.
// ======================================================================
#define STP_NOALLOC_SCRATCH_FLOATS (1u << 20)            // 4 MiB: ceil(T / 64) * N partial sums at most
#define STP_NOALLOC_MAX_DEVICES 16
static __device__ __align__(256) float scratch[STP_NOALLOC_SCRATCH_FLOATS];
static float *g_scratch_ptr[STP_NOALLOC_MAX_DEVICES];    // device address of `scratch` per device; the array's name is no address on the host

// Looks up the device address of the scratch array on `device` (which must be the current device).
int stp_noalloc_init(stp_ctx *ctx, int device) {
  if (device < 0 || device >= STP_NOALLOC_MAX_DEVICES) return stp_fail(ctx, STP_EINVAL, "stp_colsum_noalloc: device index out of range%s");
  if (g_scratch_ptr[device]) return STP_OK;
  float *p = nullptr;
  STP_HIP(ctx, hipGetSymbolAddress((void **)&p, HIP_SYMBOL(scratch)));
  if (!p) return stp_fail(ctx, STP_EHIP, "stp_colsum_noalloc: no device address for the scratch array%s");
  g_scratch_ptr[device] = p;
  return STP_OK;
}

extern "C" int stp_colsum_noalloc(stp_ctx *ctx, int dtype, int32_t T, int32_t N, const void *x, float scale, float *out,
                                  void *hip_stream) {
  if (!ctx) return STP_EINVAL;
  if (!x || !out) return stp_fail(ctx, STP_EINVAL, "stp_colsum_noalloc: null pointer%s");
  if (T < 0 || N <= 0 || N % 8) return stp_fail(ctx, STP_ESHAPE, "stp_colsum_noalloc: N must be a multiple of 8%s");
  if (!stp_aligned16(x)) return stp_fail(ctx, STP_EALIGN, "stp_colsum_noalloc: x must be 16-byte aligned%s");
  if (dtype != STP_BF16 && dtype != STP_F32) return stp_fail(ctx, STP_EINVAL, "stp_colsum_noalloc: bad dtype%s");
  if (T == 0) return STP_OK;
  const int slabs = stp_colsum_slabs(T);
  if ((size_t)slabs * N > (size_t)STP_NOALLOC_SCRATCH_FLOATS)
    return stp_fail(ctx, STP_ENOSPACE, "stp_colsum_noalloc: ceil(T / 64) * N%s = %ld exceeds the fixed scratch of %ld partial sums", "",
                    (long)slabs * N, (long)STP_NOALLOC_SCRATCH_FLOATS);
  int rc = stp_noalloc_init(ctx, ctx->device);   // a lookup; done at stp_create, repeated here only if that one failed
  if (rc != STP_OK) return rc;
  // stage 1 writes every partial that stage 2 reads (slabs x N), so what an earlier call left behind is never seen
  return colsum_launch(ctx, dtype, T, N, x, scale, out, g_scratch_ptr[ctx->device], (hipStream_t)hip_stream);
}

#define EW_CHECK(name, cond_null)                                                                          \
  if (!ctx) return STP_EINVAL;                                                                             \
  if (cond_null) return stp_fail(ctx, STP_EINVAL, name ": null pointer%s");                                \
  if (n % 8) return stp_fail(ctx, STP_ESHAPE, name ": element count must be a multiple of 8%s");           \
  if (dtype != STP_BF16 && dtype != STP_F32) return stp_fail(ctx, STP_EINVAL, name ": bad dtype%s");       \
  if (n == 0) return STP_OK;                                                                               \
  hipStream_t s = (hipStream_t)hip_stream;                                                                 \
  size_t n8 = n / 8;

extern "C" int stp_gelu_forward(stp_ctx *ctx, int dtype, size_t n, const void *x, void *y, void *hip_stream) {
  EW_CHECK("stp_gelu_forward", !x || !y)
  if (!stp_aligned16(x) || !stp_aligned16(y)) return stp_fail(ctx, STP_EALIGN, "stp_gelu_forward: alignment%s");
  if (dtype == STP_BF16) hipLaunchKernelGGL(gelu_fwd_kernel<bf16_t>, dim3(ew_grid(n8)), dim3(256), 0, s, (const bf16_t *)x, (bf16_t *)y, n8);
  else hipLaunchKernelGGL(gelu_fwd_kernel<float>, dim3(ew_grid(n8)), dim3(256), 0, s, (const float *)x, (float *)y, n8);
  STP_LAUNCH_CHECK(ctx);
  return STP_OK;
}
extern "C" int stp_gelu_backward(stp_ctx *ctx, int dtype, size_t n, const void *x, const void *dy, void *dx, void *hip_stream) {
  EW_CHECK("stp_gelu_backward", !x || !dy || !dx)
  if (!stp_aligned16(x) || !stp_aligned16(dy) || !stp_aligned16(dx)) return stp_fail(ctx, STP_EALIGN, "stp_gelu_backward: alignment%s");
  if (dtype == STP_BF16) hipLaunchKernelGGL(gelu_bwd_kernel<bf16_t>, dim3(ew_grid(n8)), dim3(256), 0, s, (const bf16_t *)x, (const bf16_t *)dy, (bf16_t *)dx, n8);
  else hipLaunchKernelGGL(gelu_bwd_kernel<float>, dim3(ew_grid(n8)), dim3(256), 0, s, (const float *)x, (const float *)dy, (float *)dx, n8);
  STP_LAUNCH_CHECK(ctx);
  return STP_OK;
}
extern "C" int stp_swiglu_forward(stp_ctx *ctx, int dtype, size_t n, const void *gate, const void *up, void *y, void *hip_stream) {
  EW_CHECK("stp_swiglu_forward", !gate || !up || !y)
  if (!stp_aligned16(gate) || !stp_aligned16(up) || !stp_aligned16(y)) return stp_fail(ctx, STP_EALIGN, "stp_swiglu_forward: alignment%s");
  if (dtype == STP_BF16) hipLaunchKernelGGL(swiglu_fwd_kernel<bf16_t>, dim3(ew_grid(n8)), dim3(256), 0, s, (const bf16_t *)gate, (const bf16_t *)up, (bf16_t *)y, n8);
  else hipLaunchKernelGGL(swiglu_fwd_kernel<float>, dim3(ew_grid(n8)), dim3(256), 0, s, (const float *)gate, (const float *)up, (float *)y, n8);
  STP_LAUNCH_CHECK(ctx);
  return STP_OK;
}
extern "C" int stp_swiglu_backward(stp_ctx *ctx, int dtype, size_t n, const void *gate, const void *up, const void *dy,
                                   void *dgate, void *dup, void *hip_stream) {
  EW_CHECK("stp_swiglu_backward", !gate || !up || !dy || !dgate || !dup)
  if (!stp_aligned16(gate) || !stp_aligned16(up) || !stp_aligned16(dy) || !stp_aligned16(dgate) || !stp_aligned16(dup))
    return stp_fail(ctx, STP_EALIGN, "stp_swiglu_backward: alignment%s");
  if (dtype == STP_BF16)
    hipLaunchKernelGGL(swiglu_bwd_kernel<bf16_t>, dim3(ew_grid(n8)), dim3(256), 0, s, (const bf16_t *)gate, (const bf16_t *)up,
                       (const bf16_t *)dy, (bf16_t *)dgate, (bf16_t *)dup, n8);
  else
    hipLaunchKernelGGL(swiglu_bwd_kernel<float>, dim3(ew_grid(n8)), dim3(256), 0, s, (const float *)gate, (const float *)up,
                       (const float *)dy, (float *)dgate, (float *)dup, n8);
  STP_LAUNCH_CHECK(ctx);
  return STP_OK;
}

extern "C" int stp_rope(stp_ctx *ctx, const stp_layer_desc *d, void *qkv, int inverse, void *hip_stream) {
  if (!ctx) return STP_EINVAL;
  if (!d || !qkv) return stp_fail(ctx, STP_EINVAL, "stp_rope: null pointer%s");
  int rc = stp_check_desc(d);
  if (rc != STP_OK) return stp_fail(ctx, rc, "stp_rope: bad layer description%s");
  if (d->head_dim % 16) return stp_fail(ctx, STP_ESHAPE, "stp_rope: head_dim must be a multiple of 16%s");
  if (!stp_aligned16(qkv)) return stp_fail(ctx, STP_EALIGN, "stp_rope: alignment%s");
  int tokens = d->seq * d->mbsz;
  if (tokens == 0) return STP_OK;
  const int nrot = d->heads_local + stp_kv_heads(d);
  size_t total = (size_t)tokens * nrot * (d->head_dim / 16);
  dim3 grid((total + 255) / 256), block(256);
  float log2_base = log2f(d->rope_base), sign = inverse ? -1.0f : 1.0f;
  hipStream_t s = (hipStream_t)hip_stream;
  if (d->dtype == STP_BF16)
    hipLaunchKernelGGL(rope_kernel<bf16_t>, grid, block, 0, s, (bf16_t *)qkv, tokens, d->seq, nrot, stp_qkv_width(d), d->head_dim, log2_base, sign);
  else
    hipLaunchKernelGGL(rope_kernel<float>, grid, block, 0, s, (float *)qkv, tokens, d->seq, nrot, stp_qkv_width(d), d->head_dim, log2_base, sign);
  STP_LAUNCH_CHECK(ctx);
  return STP_OK;
}

// used by the attention backward launchers
template <typename T>
static void rowdot_dispatch(const stp_layer_desc *d, const void *a, const void *b, float *delta, hipStream_t s) {
  const int tokens = d->seq * d->mbsz, n = d->heads_local, hd = d->head_dim;
  const size_t pairs = (size_t)tokens * n;
  const int lpp = hd / 8;
  if (lpp == 2 || lpp == 4 || lpp == 8 || lpp == 16) {
    dim3 grid((pairs * lpp + 255) / 256), block(256);
#define LAUNCH(L) hipLaunchKernelGGL((rowdot_packed_kernel<T, L>), grid, block, 0, s, (const T *)a, (const T *)b, delta, pairs, d->seq, n)
    if (lpp == 16) LAUNCH(16); else if (lpp == 8) LAUNCH(8); else if (lpp == 4) LAUNCH(4); else LAUNCH(2);
#undef LAUNCH
  } else {
    dim3 grid((pairs + 3) / 4), block(256);
    hipLaunchKernelGGL(rowdot_kernel<T>, grid, block, 0, s, (const T *)a, (const T *)b, delta, tokens, d->seq, n, hd);
  }
}
int stp_launch_rowdot(stp_ctx *ctx, const stp_layer_desc *d, const void *a, const void *b, float *delta, hipStream_t s) {
  if (d->dtype == STP_BF16) rowdot_dispatch<bf16_t>(d, a, b, delta, s);
  else rowdot_dispatch<float>(d, a, b, delta, s);
  STP_LAUNCH_CHECK(ctx);
  return STP_OK;
}

// ======================================================================
// Clock probe for the measurements: one wave spins for `wall_ticks` ticks of the constant-rate
// wall clock and reports how many shader-clock cycles passed meanwhile.  Launched on a side
// stream while the units run, it gives the sustained shader clock the rooflines should be read
// against (the chip lowers its clock under matrix-core load).
// ======================================================================
__global__ void clock_probe_kernel(long long *out, long long wall_ticks) {
  const long long w0 = wall_clock64(), c0 = clock64();
  long long w = w0;
  while (w - w0 < wall_ticks) w = wall_clock64();   // bounded: the wall clock always advances
  out[0] = clock64() - c0;
  out[1] = w - w0;
}

extern "C" int stp_clock_probe(stp_ctx *ctx, long long *device_out2, double milliseconds, void *hip_stream) {
  if (!ctx) return STP_EINVAL;
  if (!device_out2) return stp_fail(ctx, STP_EINVAL, "stp_clock_probe: null pointer%s");
  if (!(milliseconds > 0.0) || milliseconds > 1000.0) return stp_fail(ctx, STP_EINVAL, "stp_clock_probe: window must be in (0, 1000] ms%s");
  int rate_khz = 0;
  STP_HIP(ctx, hipDeviceGetAttribute(&rate_khz, hipDeviceAttributeWallClockRate, ctx->device));
  hipLaunchKernelGGL(clock_probe_kernel, dim3(1), dim3(64), 0, (hipStream_t)hip_stream, device_out2,
                     (long long)(milliseconds * rate_khz));
  STP_LAUNCH_CHECK(ctx);
  return STP_OK;
}

extern "C" int stp_wall_clock_khz(stp_ctx *ctx, int *khz) {
  if (!ctx) return STP_EINVAL;
  if (!khz) return stp_fail(ctx, STP_EINVAL, "stp_wall_clock_khz: null pointer%s");
  STP_HIP(ctx, hipDeviceGetAttribute(khz, hipDeviceAttributeWallClockRate, ctx->device));
  return STP_OK;
}

static int softmax_args_ok(stp_ctx *ctx, const char *who, int dtype, int32_t rows, int32_t n, const void *a, const void *b,
                           const void *c) {
  if (!a || !b || !c) return stp_fail(ctx, STP_EINVAL, "%s: null pointer", who);
  if (dtype != STP_BF16 && dtype != STP_F32) return stp_fail(ctx, STP_EINVAL, "%s: bad dtype", who);
  if (rows < 0 || n <= 0 || n % 8 || n > 16384) return stp_fail(ctx, STP_ESHAPE, "%s: n must be a multiple of 8, at most 16384", who);
  if (!stp_aligned16(a) || !stp_aligned16(b) || !stp_aligned16(c)) return stp_fail(ctx, STP_EALIGN, "%s: pointers must be 16-byte aligned", who);
  return STP_OK;
}

#define SOFTMAX_BY_NCH(KERN, T, ...)                                                              \
  do {                                                                                            \
    const int nch = (n + 2047) / 2048;                                                            \
    if (nch <= 1) hipLaunchKernelGGL((KERN<T, 1>), dim3(rows), dim3(256), 0, s, __VA_ARGS__);     \
    else if (nch <= 2) hipLaunchKernelGGL((KERN<T, 2>), dim3(rows), dim3(256), 0, s, __VA_ARGS__); \
    else if (nch <= 4) hipLaunchKernelGGL((KERN<T, 4>), dim3(rows), dim3(256), 0, s, __VA_ARGS__); \
    else hipLaunchKernelGGL((KERN<T, 8>), dim3(rows), dim3(256), 0, s, __VA_ARGS__);              \
  } while (0)

extern "C" int stp_softmax_forward(stp_ctx *ctx, int dtype, int32_t rows, int32_t n, float scale, int causal, const void *x,
                                   void *y, void *hip_stream) {
  if (!ctx) return STP_EINVAL;
  int rc = softmax_args_ok(ctx, "stp_softmax_forward", dtype, rows, n, x, y, y);
  if (rc != STP_OK) return rc;
  if (rows == 0) return STP_OK;
  hipStream_t s = (hipStream_t)hip_stream;
  const float sl = scale * 1.4426950408889634f;
  if (dtype == STP_BF16) SOFTMAX_BY_NCH(softmax_fwd_kernel, bf16_t, (const bf16_t *)x, (bf16_t *)y, rows, n, sl, causal);
  else SOFTMAX_BY_NCH(softmax_fwd_kernel, float, (const float *)x, (float *)y, rows, n, sl, causal);
  STP_LAUNCH_CHECK(ctx);
  return STP_OK;
}

extern "C" int stp_softmax_backward(stp_ctx *ctx, int dtype, int32_t rows, int32_t n, float scale, const void *y, const void *dy,
                                    void *dx, void *hip_stream) {
  if (!ctx) return STP_EINVAL;
  int rc = softmax_args_ok(ctx, "stp_softmax_backward", dtype, rows, n, y, dy, dx);
  if (rc != STP_OK) return rc;
  if (rows == 0) return STP_OK;
  hipStream_t s = (hipStream_t)hip_stream;
  if (dtype == STP_BF16) SOFTMAX_BY_NCH(softmax_bwd_kernel, bf16_t, (const bf16_t *)y, (const bf16_t *)dy, (bf16_t *)dx, rows, n, scale);
  else SOFTMAX_BY_NCH(softmax_bwd_kernel, float, (const float *)y, (const float *)dy, (float *)dx, rows, n, scale);
  STP_LAUNCH_CHECK(ctx);
  return STP_OK;
}
