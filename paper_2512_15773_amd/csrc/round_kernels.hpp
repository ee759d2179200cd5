// Row-table planning, the drafter's DDPM step and the acceptance kernel of the speculative round.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "philox.hpp"

namespace tsdp {

struct SchedTables {          // device pointers, fp32[T] each; posterior mean = c0 x0_hat + cx x + ce eps
  const float* sqrt_abar; const float* sqrt_1m; const float* c0; const float* cx; const float* sigma; const float* ce;
  int T;
};

// K_eff = min(clamp(K), t0), rows per env = live ? (bonus ? K_eff + 1 : max(K_eff,1)) : 0, exclusive scan into
// row_ptr[B+1].  K is clamped to 1..K_max (0..K_max with the bonus row, where K = 0 is a plain base step).
// n_draft[0] receives B if any environment has rows, else 0; n_draft[1] receives B if any environment drafts
// (K_eff > 0), else 0.  Single workgroup of 1024 threads, chunks of 1024 environments.
__global__ __launch_bounds__(1024) void k_plan(const int32_t* __restrict__ t0, const int32_t* __restrict__ K,
                                               const float* __restrict__ sigma_scale,
                                               int B, int K_max, int T, int bonus, int32_t* __restrict__ K_eff,
                                               int32_t* __restrict__ row_ptr, int32_t* __restrict__ status,
                                               int32_t* __restrict__ n_draft) {
  __shared__ int32_t part[1024];
  __shared__ int32_t carry;
  if (threadIdx.x == 0) carry = 0;
  __syncthreads();
  int any_draft = 0;
  for (int base = 0; base < B; base += 1024) {
    const int b = base + threadIdx.x;
    int n = 0, drafts = 0;
    if (b < B) {
      int k = K[b], t = t0[b];
      const int k_min = bonus ? 0 : 1;
      if (k < k_min || k > K_max) { atomicOr(status, 1); k = k < k_min ? k_min : K_max; }
      if (t >= T) { atomicOr(status, 2); t = T - 1; }
      if (t >= 0 && !(sigma_scale[b] > 0.0f)) atomicOr(status, 4);   // divides the mean difference: reported, not corrected
      const int ke = t < 0 ? 0 : (k < t ? k : t);
      K_eff[b] = ke;
      drafts = ke;
      n = t < 0 ? 0 : (bonus ? ke + 1 : (ke > 1 ? ke : 1));
    }
    part[threadIdx.x] = n;
    any_draft |= __syncthreads_or(drafts > 0);
    for (int o = 1; o < 1024; o <<= 1) {            // inclusive Hillis-Steele scan
      const int v = threadIdx.x >= o ? part[threadIdx.x - o] : 0;
      __syncthreads();
      part[threadIdx.x] += v;
      __syncthreads();
    }
    if (b < B) row_ptr[b] = carry + part[threadIdx.x] - n;
    __syncthreads();
    if (threadIdx.x == 1023) carry += part[1023];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    row_ptr[B] = carry;
    n_draft[0] = carry > 0 ? B : 0;                 // environments with rows: none once all have finished
    n_draft[1] = any_draft ? B : 0;                 // environments the drafter has to look at: none in a round of plain base steps
  }
}

// Range check of a caller-supplied row table (tsdp_verify): copies with the timestep clamped to 0..T-1 and the
// environment index to 0..n_env-1; status bit 1 / bit 3 report a clamp.
__global__ void k_check_rows(const int32_t* __restrict__ d_R, int R_cap, const int32_t* __restrict__ row_t,
                             const int32_t* __restrict__ row_env, int T, int n_env, int32_t* __restrict__ row_t_out,
                             int32_t* __restrict__ row_env_out, int32_t* __restrict__ status) {
  const int r = blockIdx.x * blockDim.x + threadIdx.x;
  const int R = min(*d_R, R_cap);
  if (r >= R) return;
  int t = row_t[r], e = row_env[r];
  if (t < 0 || t >= T) { atomicOr(status, 2); t = t < 0 ? 0 : T - 1; }
  if (e < 0 || e >= n_env) { atomicOr(status, 8); e = e < 0 ? 0 : n_env - 1; }
  row_t_out[r] = t;
  row_env_out[r] = e;
}

// Fills row_t / row_env, copies x into y (the rollout state), and for t0 = 0 environments writes the
// lone base-step row (state = x, eps_p = xi = 0).  One workgroup per environment.
__global__ void k_rows(const float* __restrict__ x, const int32_t* __restrict__ t0, const int32_t* __restrict__ row_ptr,
                       int T, int D, int32_t* __restrict__ row_t, int32_t* __restrict__ row_env,
                       float* __restrict__ y, float* __restrict__ states, float* __restrict__ eps_p,
                       float* __restrict__ xi, const int32_t* __restrict__ gate) {
  if (gate && *gate == 0) return;                   // chain driver: no environment is running any more
  const int b = blockIdx.x;
  const int r0 = row_ptr[b], n = row_ptr[b + 1] - r0;
  int t = t0[b];
  if (t >= T) t = T - 1;
  for (int j = threadIdx.x; j < n; j += blockDim.x) { row_t[r0 + j] = t - j; row_env[r0 + j] = b; }
  for (int e = threadIdx.x; e < D; e += blockDim.x) {
    const float v = x[(long long)b * D + e];
    y[(long long)b * D + e] = v;
    if (t == 0) {
      states[(long long)r0 * D + e] = v;
      eps_p[(long long)r0 * D + e] = 0.0f;
      if (xi) xi[(long long)r0 * D + e] = 0.0f;
    }
  }
}

// Drafted transition k for every environment with K_eff >= k:
//   states[row] = y;  eps_p[row] = eps;  xi[row] = xi_{env,t};  y <- mu_p(y, eps, t) + s sigma_t xi.
// One thread per 4 elements (one Philox block).
__global__ void k_draft_step(int k, const float* __restrict__ eps, const int32_t* __restrict__ t0,
                             const int32_t* __restrict__ K_eff, const int32_t* __restrict__ row_ptr,
                             const float* __restrict__ sigma_scale, const int32_t* __restrict__ env_id,
                             SchedTables tb, int clip, float clip_val, uint64_t seed, int B, int D,
                             float* __restrict__ y, float* __restrict__ states, float* __restrict__ eps_p,
                             float* __restrict__ xi) {
  const int nb = D >> 2;
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (long long)B * nb) return;
  const int b = (int)(i / nb), blk = (int)(i % nb);
  if (K_eff[b] < k) return;
  int t = t0[b];
  if (t >= tb.T) t = tb.T - 1;
  t = t - k + 1;
  const long long row = row_ptr[b] + k - 1;
  const float4 yv = *reinterpret_cast<const float4*>(y + (long long)b * D + 4 * blk);
  const float4 ev = *reinterpret_cast<const float4*>(eps + (long long)b * D + 4 * blk);
  const float4 z = xi_block(seed, env_id ? env_id[b] : b, t, blk);
  const float sa = tb.sqrt_abar[t], s1 = tb.sqrt_1m[t], c0 = tb.c0[t], cx = tb.cx[t], ce = tb.ce[t];
  const float sig = sigma_scale[b] * tb.sigma[t];
  const float yy[4] = {yv.x, yv.y, yv.z, yv.w}, ee[4] = {ev.x, ev.y, ev.z, ev.w}, zz[4] = {z.x, z.y, z.z, z.w};
  float o[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    float x0 = (yy[j] - s1 * ee[j]) / sa;
    if (clip) x0 = fminf(fmaxf(x0, -clip_val), clip_val);
    o[j] = c0 * x0 + cx * yy[j] + ce * ee[j] + sig * zz[j];
  }
  *reinterpret_cast<float4*>(states + row * D + 4 * blk) = yv;
  *reinterpret_cast<float4*>(eps_p + row * D + 4 * blk) = ev;
  if (xi) *reinterpret_cast<float4*>(xi + row * D + 4 * blk) = z;
  *reinterpret_cast<float4*>(y + (long long)b * D + 4 * blk) = make_float4(o[0], o[1], o[2], o[3]);
}

// Bonus row of every running environment: the state reached by the last draft, at timestep t0 - K_eff, with the
// noise a base step from it would use (none at timestep 0); there is no drafter prediction for it.
__global__ void k_bonus_rows(const int32_t* __restrict__ t0, const int32_t* __restrict__ K_eff,
                             const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ env_id, int T, int D,
                             uint64_t seed, const float* __restrict__ y, float* __restrict__ states,
                             float* __restrict__ eps_p, float* __restrict__ xi) {
  const int b = blockIdx.x;                          // (an environment without rows returns at once: no gate needed)
  const int r0 = row_ptr[b];
  if (row_ptr[b + 1] == r0) return;
  int t = t0[b];
  if (t >= T) t = T - 1;
  const int ke = K_eff[b];
  t -= ke;
  const long long row = r0 + ke;
  const int env = env_id ? env_id[b] : b;
  for (int blk = threadIdx.x; blk < (D >> 2); blk += blockDim.x) {
    const float4 z = t > 0 ? xi_block(seed, env, t, blk) : make_float4(0.f, 0.f, 0.f, 0.f);
    *reinterpret_cast<float4*>(states + row * D + 4 * blk) = *reinterpret_cast<const float4*>(y + (long long)b * D + 4 * blk);
    *reinterpret_cast<float4*>(eps_p + row * D + 4 * blk) = make_float4(0.f, 0.f, 0.f, 0.f);
    if (xi) *reinterpret_cast<float4*>(xi + row * D + 4 * blk) = z;
  }
}

// Stage tables of the chain driver: column 0 while t >= t_hi, 1 while t_lo <= t < t_hi, else 2.
__global__ void k_stage_select(int B, const int32_t* __restrict__ t, int t_hi, int t_lo, const int32_t* __restrict__ K3,
                               const float* __restrict__ s3, const float* __restrict__ l3, int32_t* __restrict__ K,
                               float* __restrict__ s, float* __restrict__ l) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  const int tt = t[b];
  const int st = tt >= t_hi ? 0 : (tt >= t_lo ? 1 : 2);
  K[b] = K3[3 * b + st];
  s[b] = s3[3 * b + st];
  if (l3) l[b] = l3[3 * b + st];
}

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// 16-byte load of data that is read once (streamed past the caches' replacement order)
__device__ __forceinline__ float4 load_once(const float4* a) {
  typedef float f4v __attribute__((ext_vector_type(4)));
  const f4v v = __builtin_nontemporal_load(reinterpret_cast<const f4v*>(a));
  return make_float4(v[0], v[1], v[2], v[3]);
}

// sums v over the G consecutive lanes of a lane group (G a power of two)
template <int G>
__device__ __forceinline__ double group_sum(double v) {
#pragma unroll
  for (int o = G / 2; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

__device__ __forceinline__ double group16_sum(double v) { return group_sum<16>(v); }

// Acceptance: one wavefront per environment, 64/G rows at a time (one row per group of G lanes; the host picks G so
// that the D/4 16-byte vectors of a row fill the lanes: 8 lanes x 5 vectors at D = 160, 16 x 7 at D = 448).  Each
// group streams eps_p, eps_q, xi (and the state when x0 is clamped) of its row with 16-byte loads, all of them
// issued before the first use, reduces |d|^2 and <d,xi> in fp64 and tests log U <= log alpha; the wave keeps the
// first rejection and finally writes the committed or the reflected latent.  Rows after the pass that holds the
// first rejection are not read (the method discards them) unless per-row diagnostics are requested.  xi may be
// null (REGEN): the noise of a row is then regenerated from its Philox counters (seed, environment, timestep).
// Every load is unconditional (a slot outside its row, or a group without a row, re-reads an address inside the
// environment's rows and its value is masked out of the sums): a load under a lane-dependent condition becomes a
// branch with its own wait, which serialises the stream.  The row data is read exactly once: non-temporal loads
// (2^20-row shape: 0.426 -> 0.391 ms).
template <bool CLIP, bool REGEN, int G, int MAXI>
__global__ __launch_bounds__(256) void k_accept(int B, int D, const int32_t* __restrict__ row_ptr,
                                                const int32_t* __restrict__ row_t, const int32_t* __restrict__ env_id,
                                                const float* __restrict__ sigma_scale, const float* __restrict__ states,
                                                const float* __restrict__ eps_p, const float* __restrict__ eps_q,
                                                const float* __restrict__ xi, const float* __restrict__ y_last,
                                                SchedTables tb, float clip_val, uint64_t seed,
                                                const float* __restrict__ lambda,   // per-env threshold rule, or null
                                                int bonus,                          // last row of an env is a base step
                                                float* __restrict__ x_out, int32_t* __restrict__ t_next,
                                                int32_t* __restrict__ n_accept, int32_t* __restrict__ n_adv,
                                                uint8_t* __restrict__ flags, float* __restrict__ logratio,
                                                float* __restrict__ logu_out, const int32_t* __restrict__ gate) {
  // chain driver: once no environment is running, latents, timesteps and counters stay as they are
  if (gate && *gate == 0) return;
  // MAXI = 16-byte vectors per lane and row: rows of up to G*MAXI*4 elements
  constexpr int RPP = 64 / G;                       // rows per pass
  const int lane = threadIdx.x & 63, grp = lane / G, gl = lane % G;
  const int b = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (b >= B) return;
  const int r0 = row_ptr[b], r1 = row_ptr[b + 1];
  const int nb = D >> 2;
  float4* xo = reinterpret_cast<float4*>(x_out + (long long)b * D);
  if (r1 == r0) {                                   // finished environment: latent passes through
    const float4* yl = reinterpret_cast<const float4*>(y_last + (long long)b * D);
    for (int i = lane; i < nb; i += 64) xo[i] = yl[i];
    if (lane == 0) { t_next[b] = -1; n_accept[b] = 0; if (n_adv) n_adv[b] = 0; }
    return;
  }
  const int t0 = row_t[r0];
  const double cv = (double)clip_val;
  // the last row is a step of the base model itself: always with the bonus row, else only at t0 = 0
  const bool base_row = bonus || t0 == 0;
  const int rd = base_row ? r1 - 1 : r1;            // drafted rows are r0 .. rd-1
  if (base_row && lane == 0) {
    if (flags) flags[rd] = 0;
    if (logratio) logratio[rd] = 0.0f;
    if (logu_out) logu_out[rd] = 0.0f;
  }
  const double s = (double)sigma_scale[b];
  const int env = env_id ? env_id[b] : b;
  const bool diag = flags || logratio || logu_out;  // diagnostics cover every row: no pass is skipped
  int jstar = 0;                                    // 0 = no rejection yet; else 1-based row index
  double rej_dd = 0.0, rej_dx = 0.0;
  for (int rb = r0; rb < rd && (jstar == 0 || diag); rb += RPP) {
    const int r = rb + grp;
    const bool live = r < rd;                       // a group without a row re-reads the last one; its result is unused
    const int rr = live ? r : rd - 1;
    const float4* ep = reinterpret_cast<const float4*>(eps_p + (long long)rr * D);
    const float4* eq = reinterpret_cast<const float4*>(eps_q + (long long)rr * D);
    const float4* zz = reinterpret_cast<const float4*>(xi + (long long)rr * D);
    const float4* st = reinterpret_cast<const float4*>(states + (long long)rr * D);
    float4 p[MAXI], q[MAXI], z[MAXI], y[MAXI];
#pragma unroll
    for (int it = 0; it < MAXI; ++it) {
      const int i = min(gl + G * it, nb - 1);
      p[it] = load_once(ep + i); q[it] = load_once(eq + i);
      if (!REGEN) z[it] = load_once(zz + i);
      if (CLIP) y[it] = load_once(st + i);
    }
    const int t = row_t[rr];
    if (REGEN) {                                    // no stored noise: the same Philox blocks the drafter drew
#pragma unroll
      for (int it = 0; it < MAXI; ++it) z[it] = xi_block(seed, env, t, min(gl + G * it, nb - 1));
    }
    const double sa = tb.sqrt_abar[t], s1 = tb.sqrt_1m[t], c0 = tb.c0[t], ce = tb.ce[t], sig = s * (double)tb.sigma[t];
    // stochastic test: log U;  threshold rule p = min(1, alpha) >= lambda  <=>  log alpha >= log lambda (lambda <= 1)
    const double lu = lambda ? log((double)lambda[b]) : log((double)accept_uniform(seed, env, t));
    // sums of delta^2 and delta*xi; clamped x0: delta = mu_p - mu_q, else delta = eps_p - eps_q (mu_p - mu_q is a
    // multiple of it)
    double dd = 0.0, dx = 0.0;
#pragma unroll
    for (int it = 0; it < MAXI; ++it) {
      const bool in = gl + G * it < nb;             // always true when the row fills the lanes exactly
      const float pp[4] = {p[it].x, p[it].y, p[it].z, p[it].w}, qq[4] = {q[it].x, q[it].y, q[it].z, q[it].w},
                  zv[4] = {z[it].x, z[it].y, z[it].z, z[it].w};
      if (CLIP) {
        const float yy[4] = {y[it].x, y[it].y, y[it].z, y[it].w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const double xp = fmin(fmax(((double)yy[j] - s1 * (double)pp[j]) / sa, -cv), cv);
          const double xq = fmin(fmax(((double)yy[j] - s1 * (double)qq[j]) / sa, -cv), cv);
          double de = c0 * (xp - xq) + ce * ((double)pp[j] - (double)qq[j]);
          de = in ? de : 0.0;
          dd = fma(de, de, dd); dx = fma(de, (double)zv[j], dx);
        }
      } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) {               // x0_p - x0_q = -(s1/sa)(eps_p - eps_q)
          double de = (double)pp[j] - (double)qq[j];
          de = in ? de : 0.0;
          dd = fma(de, de, dd); dx = fma(de, (double)zv[j], dx);
        }
      }
    }
    dd = group_sum<G>(dd); dx = group_sum<G>(dx);
    const double kap = CLIP ? 1.0 / sig : (ce - (c0 * s1) / sa) / sig;   // d = kap * delta
    const double n2 = kap * kap * dd, ip = kap * dx;                // |d|^2, <d,xi>
    const double l = -0.5 * n2 - ip;
    const bool acc = lu <= l;
    if (live && gl == 0) {
      if (flags) flags[r] = acc ? 1 : 0;
      if (logratio) logratio[r] = (float)l;
      if (logu_out) logu_out[r] = (float)lu;
    }
    // first rejected row among the rows of this pass
    const unsigned long long rejmask = __ballot(live && !acc);
    if (rejmask && jstar == 0) {
      const int g = (__ffsll((long long)rejmask) - 1) / G;
      jstar = rb + g - r0 + 1;
      rej_dd = __shfl(n2, g * G); rej_dx = __shfl(ip, g * G);
    }
  }
  const int K_eff = rd - r0;
  if (jstar == 0 && base_row) {                     // exact base transition from y_{K_eff} (no noise at timestep 0)
    const int t = t0 - K_eff;
    const double sa = tb.sqrt_abar[t], s1 = tb.sqrt_1m[t], c0 = tb.c0[t], cx = tb.cx[t], ce = tb.ce[t],
                 sig = t > 0 ? s * (double)tb.sigma[t] : 0.0;
    const float4* st = reinterpret_cast<const float4*>(states + (long long)rd * D);
    const float4* eq = reinterpret_cast<const float4*>(eps_q + (long long)rd * D);
    const float4* zz = reinterpret_cast<const float4*>(xi + (long long)rd * D);
    for (int i = lane; i < nb; i += 64) {
      const float4 y = st[i], e = eq[i];
      const float4 z = t > 0 ? (REGEN ? xi_block(seed, env, t, i) : zz[i]) : make_float4(0.f, 0.f, 0.f, 0.f);
      const float yy[4] = {y.x, y.y, y.z, y.w}, ee[4] = {e.x, e.y, e.z, e.w}, zv[4] = {z.x, z.y, z.z, z.w};
      float o[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        double x0 = ((double)yy[j] - s1 * (double)ee[j]) / sa;
        if (CLIP) x0 = fmin(fmax(x0, -cv), cv);
        o[j] = (float)(c0 * x0 + cx * (double)yy[j] + ce * (double)ee[j] + sig * (double)zv[j]);
      }
      xo[i] = make_float4(o[0], o[1], o[2], o[3]);
    }
    if (lane == 0) { t_next[b] = t - 1; n_accept[b] = K_eff; if (n_adv) n_adv[b] = K_eff + 1; }
    return;
  }
  if (jstar == 0) {                                 // every draft accepted: commit y_{K_eff}
    const float4* yl = reinterpret_cast<const float4*>(y_last + (long long)b * D);
    for (int i = lane; i < nb; i += 64) xo[i] = yl[i];
    if (lane == 0) { t_next[b] = t0 - K_eff; n_accept[b] = K_eff; if (n_adv) n_adv[b] = K_eff; }
    return;
  }
  {                                                 // reflect the first rejected draft about the target mean
    const int r = r0 + jstar - 1;
    const int t = row_t[r];
    const double sa = tb.sqrt_abar[t], s1 = tb.sqrt_1m[t], c0 = tb.c0[t], cx = tb.cx[t], ce = tb.ce[t],
                 sig = s * (double)tb.sigma[t];
    const double coef = rej_dd > 0.0 ? 2.0 * rej_dx / rej_dd : 0.0;   // 2 <d,xi>/|d|^2
    const float4* ep = reinterpret_cast<const float4*>(eps_p + (long long)r * D);
    const float4* eq = reinterpret_cast<const float4*>(eps_q + (long long)r * D);
    const float4* zz = reinterpret_cast<const float4*>(xi + (long long)r * D);
    const float4* st = reinterpret_cast<const float4*>(states + (long long)r * D);
    for (int i = lane; i < nb; i += 64) {
      const float4 p = ep[i], q = eq[i], z = REGEN ? xi_block(seed, env, t, i) : zz[i], y = st[i];
      const float pp[4] = {p.x, p.y, p.z, p.w}, qq[4] = {q.x, q.y, q.z, q.w}, zv[4] = {z.x, z.y, z.z, z.w},
                  yy[4] = {y.x, y.y, y.z, y.w};
      float o[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        double xp = ((double)yy[j] - s1 * (double)pp[j]) / sa;
        double xq = ((double)yy[j] - s1 * (double)qq[j]) / sa;
        if (CLIP) { xp = fmin(fmax(xp, -cv), cv); xq = fmin(fmax(xq, -cv), cv); }
        const double muq = c0 * xq + cx * (double)yy[j] + ce * (double)qq[j];
        const double dmu = c0 * (xp - xq) + ce * ((double)pp[j] - (double)qq[j]);   // mu_p - mu_q
        o[j] = (float)(muq + sig * (double)zv[j] - coef * dmu);
      }
      xo[i] = make_float4(o[0], o[1], o[2], o[3]);
    }
    if (lane == 0) { t_next[b] = t0 - jstar; n_accept[b] = jstar - 1; if (n_adv) n_adv[b] = jstar; }
  }
}

// Chain bookkeeping after a round: per-environment totals and the number of environments still running.
__global__ void k_chain_accum(int B, const int32_t* __restrict__ t, const int32_t* __restrict__ K_eff,
                              const int32_t* __restrict__ n_acc, const int32_t* __restrict__ n_adv,
                              const int32_t* __restrict__ row_ptr, int32_t* __restrict__ tot_accept,
                              int32_t* __restrict__ tot_drafts, int32_t* __restrict__ tot_rounds, int32_t* __restrict__ live,
                              int32_t* __restrict__ rounds_run) {
  if (rounds_run && blockIdx.x == 0 && threadIdx.x == 0 && row_ptr[B] > 0) *rounds_run += 1;   // a round that had rows
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  const bool ran = row_ptr[b + 1] > row_ptr[b];      // the environment had rows in this round
  if (ran) {
    if (tot_accept) tot_accept[b] += n_acc[b];
    if (tot_drafts) tot_drafts[b] += K_eff[b];
    if (tot_rounds) tot_rounds[b] += 1;
  }
  if (live && t[b] >= 0) atomicAdd(live, 1);
}

__global__ void k_fill_i32(int32_t* p, int n, int32_t v) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// Distillation-loss forward: per row the squared distance of the two noise predictions and of the two posterior
// means in units of sigma_t, reduced in fp64.  One row per group of 16 lanes; every workgroup writes one partial
// pair, a second single-workgroup kernel adds the partials in a fixed order (deterministic result).
template <bool CLIP>
__global__ __launch_bounds__(256) void k_distill_partial(int R, int D, const int32_t* __restrict__ row_t,
                                                         const float* __restrict__ states, const float* __restrict__ eps_p,
                                                         const float* __restrict__ eps_q, SchedTables tb, float clip_val,
                                                         double* __restrict__ partial) {
  __shared__ double sp[16], sn[16];
  const int lane = threadIdx.x & 63, grp = threadIdx.x >> 4, gl = threadIdx.x & 15;
  const int r = blockIdx.x * 16 + grp;
  const int nb = D >> 2;
  double pred = 0.0, nrm = 0.0;
  if (r < R) {
    const int t = row_t[r];
    const double sa = tb.sqrt_abar[t], s1 = tb.sqrt_1m[t], c0 = tb.c0[t], ce = tb.ce[t], sig = tb.sigma[t], cv = clip_val;
    const float4* ep = reinterpret_cast<const float4*>(eps_p + (long long)r * D);
    const float4* eq = reinterpret_cast<const float4*>(eps_q + (long long)r * D);
    const float4* st = reinterpret_cast<const float4*>(states + (long long)r * D);
    double dd = 0.0, dm = 0.0;
    for (int i = gl; i < nb; i += 16) {
      const float4 p = ep[i], q = eq[i];
      const float pp[4] = {p.x, p.y, p.z, p.w}, qq[4] = {q.x, q.y, q.z, q.w};
      float yy[4] = {0, 0, 0, 0};
      if (CLIP) { const float4 y = st[i]; yy[0] = y.x; yy[1] = y.y; yy[2] = y.z; yy[3] = y.w; }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const double de = (double)pp[j] - (double)qq[j];
        dd = fma(de, de, dd);
        if (CLIP) {
          const double xp = fmin(fmax(((double)yy[j] - s1 * (double)pp[j]) / sa, -cv), cv);
          const double xq = fmin(fmax(((double)yy[j] - s1 * (double)qq[j]) / sa, -cv), cv);
          const double dmu = c0 * (xp - xq) + ce * de;
          dm = fma(dmu, dmu, dm);
        }
      }
    }
    dd = group16_sum(dd); dm = group16_sum(dm);
    pred = dd;
    if (t > 0) {
      const double kap = CLIP ? 1.0 / sig : (ce - (c0 * s1) / sa) / sig;
      nrm = kap * kap * (CLIP ? dm : dd);
    }
  }
  (void)lane;
  if (gl == 0) { sp[grp] = pred; sn[grp] = nrm; }
  __syncthreads();
  if (threadIdx.x == 0) {
    double a = 0.0, b = 0.0;
    for (int i = 0; i < 16; ++i) { a += sp[i]; b += sn[i]; }
    partial[2 * blockIdx.x] = a; partial[2 * blockIdx.x + 1] = b;
  }
}

__global__ __launch_bounds__(256) void k_distill_final(int nparts, int R, const int32_t* __restrict__ row_t,
                                                       const double* __restrict__ partial, float lam1, float lam2,
                                                       double* __restrict__ loss) {
  __shared__ double sa[256], sb[256];
  __shared__ int sc[256];
  double a = 0.0, b = 0.0;
  int noisy = 0;
  for (int i = threadIdx.x; i < nparts; i += 256) { a += partial[2 * i]; b += partial[2 * i + 1]; }
  for (int i = threadIdx.x; i < R; i += 256) noisy += row_t[i] > 0;
  sa[threadIdx.x] = a; sb[threadIdx.x] = b; sc[threadIdx.x] = noisy;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) { sa[threadIdx.x] += sa[threadIdx.x + o]; sb[threadIdx.x] += sb[threadIdx.x + o]; sc[threadIdx.x] += sc[threadIdx.x + o]; }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const double lp = R > 0 ? sa[0] / R : 0.0, ln = sc[0] > 0 ? sb[0] / sc[0] : 0.0;
    loss[0] = lp; loss[1] = ln; loss[2] = (double)lam1 * lp + (double)lam2 * ln;
  }
}

}  // namespace tsdp
