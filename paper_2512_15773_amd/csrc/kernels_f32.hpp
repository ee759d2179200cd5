// fp32 operator kernels of the denoiser: one launch per operator, activations in global memory.
// This is the general path (any shape, both conditioning modes); bf16 networks run it on
// bf16-rounded weights until a fused MFMA kernel covers the shape.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tsdp {

// rows live on the device: every row-parallel kernel stops at *d_R
__device__ __forceinline__ int live_rows(const int32_t* d_R, int R_cap) {
  const int r = d_R ? *d_R : R_cap;
  return r < R_cap ? r : R_cap;
}

__device__ __forceinline__ float silu_f(float x) { return x / (1.0f + expf(-x)); }
__device__ __forceinline__ float gelu_tanh_f(float x) {
  const float k = 0.7978845608028654f;
  return 0.5f * x * (1.0f + tanhf(k * (x + 0.044715f * x * x * x)));
}

// h[row*H+tok, c] = x[row,tok,:] . tok_w[c,:] + tok_b[c] + pos[tok,c]
__global__ void k_embed(const float* __restrict__ x, const float* __restrict__ tok_w, const float* __restrict__ tok_b,
                        const float* __restrict__ pos, float* __restrict__ h, int H, int A, int d,
                        const int32_t* d_R, int R_cap) {
  const int R = live_rows(d_R, R_cap);
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (long long)R * H * d) return;
  const int c = (int)(i % d);
  const long long tokg = i / d;
  const int tok = (int)(tokg % H);
  const float* xr = x + tokg * A;
  float acc = tok_b[c] + pos[tok * d + c];
  for (int a = 0; a < A; ++a) acc = fmaf(xr[a], tok_w[c * A + a], acc);
  h[i] = acc;
}

// sg[row, c] = SiLU(temb[t_row, c] + cemb[env_row, c]);  t_row = clamp(t_arr[row] - t_sub, 0, T-1)
__global__ void k_gvec(const int32_t* __restrict__ t_arr, int t_sub, const int32_t* __restrict__ env_arr,
                       const float* __restrict__ temb, const float* __restrict__ cemb, float* __restrict__ sg,
                       int d, int T, const int32_t* d_R, int R_cap) {
  const int R = live_rows(d_R, R_cap);
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (long long)R * d) return;
  const int c = (int)(i % d);
  const int row = (int)(i / d);
  int t = t_arr[row] - t_sub;
  t = t < 0 ? 0 : (t >= T ? T - 1 : t);
  const int env = env_arr ? env_arr[row] : row;
  float g = temb[(long long)t * d + c];
  if (cemb) g += cemb[(long long)env * d + c];
  sg[i] = silu_f(g);
}

// out[M,N] (op)= act(in[M,K] . W[N,K]^T + bias[N]);  EPI 0 store, 1 GELU-tanh store, 2 add into out
template <int EPI>
__global__ __launch_bounds__(256) void k_linear(const float* __restrict__ in, const float* __restrict__ W,
                                                const float* __restrict__ bias, float* __restrict__ out,
                                                int rows_per_unit, int N, int K, const int32_t* d_R, int R_cap) {
  constexpr int BM = 64, BN = 64, BK = 16;
  const int M = live_rows(d_R, R_cap) * rows_per_unit;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  if (m0 >= M) return;
  __shared__ float Xs[BK][BM + 4];
  __shared__ float Ws[BK][BN + 4];
  const int tid = threadIdx.x;
  const int lr = tid >> 2, lk = (tid & 3) * 4;       // loader: row lr, k offset lk
  const int tm = (tid >> 4) * 4, tn = (tid & 15) * 4; // compute: 4x4 block
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += BK) {
    float4 xv = make_float4(0, 0, 0, 0), wv = make_float4(0, 0, 0, 0);
    if (m0 + lr < M && k0 + lk < K) xv = *reinterpret_cast<const float4*>(in + (long long)(m0 + lr) * K + k0 + lk);
    if (n0 + lr < N && k0 + lk < K) wv = *reinterpret_cast<const float4*>(W + (long long)(n0 + lr) * K + k0 + lk);
    Xs[lk + 0][lr] = xv.x; Xs[lk + 1][lr] = xv.y; Xs[lk + 2][lr] = xv.z; Xs[lk + 3][lr] = xv.w;
    Ws[lk + 0][lr] = wv.x; Ws[lk + 1][lr] = wv.y; Ws[lk + 2][lr] = wv.z; Ws[lk + 3][lr] = wv.w;
    __syncthreads();
#pragma unroll
    for (int k = 0; k < BK; ++k) {
      const float4 a = *reinterpret_cast<const float4*>(&Xs[k][tm]);
      const float4 b = *reinterpret_cast<const float4*>(&Ws[k][tn]);
      const float av[4] = {a.x, a.y, a.z, a.w}, bv[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + tm + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tn + j;
      if (n >= N) continue;
      float v = acc[i][j] + (bias ? bias[n] : 0.0f);
      float* o = out + (long long)m * N + n;
      if (EPI == 1) v = gelu_tanh_f(v);
      if (EPI == 2) v += *o;
      *o = v;
    }
  }
}

// a[tok, c] = LN(h[tok, :])[c] * (1 + gamma[row, c]) + beta[row, c]; one wave per token; d <= 1024
__global__ __launch_bounds__(256) void k_lnmod(const float* __restrict__ h, const float* __restrict__ gamma,
                                               const float* __restrict__ beta, int mod_stride, float* __restrict__ a,
                                               int H, int d, int rms, const int32_t* d_R, int R_cap) {
  const int R = live_rows(d_R, R_cap);
  const long long tok = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (tok >= (long long)R * H) return;
  const int lane = threadIdx.x & 63;
  const int row = (int)(tok / H);
  const float* hr = h + tok * d;
  float v[16];
  float s = 0.0f;
#pragma unroll
  for (int i = 0; i < 16; ++i) { const int c = lane + 64 * i; v[i] = c < d ? hr[c] : 0.0f; s += v[i]; }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
  const float mean = rms ? 0.0f : s / (float)d;        // RMSNorm: no centring
  float q = 0.0f;
#pragma unroll
  for (int i = 0; i < 16; ++i) { const int c = lane + 64 * i; const float e = c < d ? v[i] - mean : 0.0f; q += e * e; }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) q += __shfl_xor(q, o);
  const float rstd = 1.0f / sqrtf(q / (float)d + 1e-5f);
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int c = lane + 64 * i;
    if (c < d) {
      float y = (v[i] - mean) * rstd;
      if (gamma) y = y * (1.0f + gamma[(long long)row * mod_stride + c]) + beta[(long long)row * mod_stride + c];
      a[tok * d + c] = y;
    }
  }
}

// softmax(q k^T / sqrt(dh)) v for one (row, head).  q rows: Hq tokens of `row`; keys/values: Hk tokens of
// kv_row (= row for self-attention, = env for cross-attention).  Strides in floats between tokens.
__global__ __launch_bounds__(256) void k_attn(const float* __restrict__ q, int q_stride,
                                              const float* __restrict__ k, const float* __restrict__ v, int kv_stride,
                                              const int32_t* __restrict__ kv_row_of, float* __restrict__ out, int out_stride,
                                              int Hq, int Hk, int dh, const int32_t* d_R, int R_cap) {
  const int R = live_rows(d_R, R_cap);
  const int row = blockIdx.x, head = blockIdx.y;
  if (row >= R) return;
  const int kvr = kv_row_of ? kv_row_of[row] : row;
  extern __shared__ float sm[];
  float* S = sm;                      // [Hq][Hk]
  const float* qb = q + (long long)row * Hq * q_stride + head * dh;
  const float* kb = k + (long long)kvr * Hk * kv_stride + head * dh;
  const float* vb = v + (long long)kvr * Hk * kv_stride + head * dh;
  const float scale = 1.0f / sqrtf((float)dh);
  for (int p = threadIdx.x; p < Hq * Hk; p += blockDim.x) {
    const int i = p / Hk, j = p % Hk;
    float acc = 0.0f;
    for (int c = 0; c < dh; ++c) acc = fmaf(qb[i * q_stride + c], kb[j * kv_stride + c], acc);
    S[p] = acc * scale;
  }
  __syncthreads();
  for (int i = threadIdx.x; i < Hq; i += blockDim.x) {
    float mx = -INFINITY;
    for (int j = 0; j < Hk; ++j) mx = fmaxf(mx, S[i * Hk + j]);
    float sum = 0.0f;
    for (int j = 0; j < Hk; ++j) { const float e = expf(S[i * Hk + j] - mx); S[i * Hk + j] = e; sum += e; }
    const float inv = 1.0f / sum;
    for (int j = 0; j < Hk; ++j) S[i * Hk + j] *= inv;
  }
  __syncthreads();
  for (int p = threadIdx.x; p < Hq * dh; p += blockDim.x) {
    const int i = p / dh, c = p % dh;
    float acc = 0.0f;
    for (int j = 0; j < Hk; ++j) acc = fmaf(S[i * Hk + j], vb[j * kv_stride + c], acc);
    out[((long long)row * Hq + i) * out_stride + head * dh + c] = acc;
  }
}

}  // namespace tsdp
