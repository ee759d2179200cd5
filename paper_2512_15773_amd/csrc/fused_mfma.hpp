// Fused bf16 MFMA forward of the denoiser: one workgroup carries a tile of NT tokens (NT/H rows)
// through ALL layers without leaving the compute unit.  The fp32 residual stream lives in MFMA
// accumulator registers, bf16 activations are staged in LDS, and the weights stream from L2 straight
// into registers in a fragment order prepared at load time.  Every product is computed transposed
// (output features on the MFMA M axis, tokens on the N axis), so that an accumulator holds four
// consecutive features of one token and can be stored to LDS as one 8-byte bf16 vector.
//
// Two kernels share the body: k_fused_forward (batched verification, Section 3.2 "Verification of
// Speculative Drafts") and k_fused_draft (the drafter's K sequential steps with the DDPM step fused in,
// Section 3.2 "Draft Generation Procedure").
//
// mfma_f32_16x16x32_bf16 operand layout (checked on hardware): lane l supplies row (l%16) and the
// eight K entries (l/16)*8.. of A and of B^T; it receives column (l%16), rows (l/16)*4.. of C.
// mfma_f32_16x16x16_bf16: the same with four K entries (l/16)*4.. per lane.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>
#include "philox.hpp"

namespace tsdp {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;

struct FusedLayer {            // device pointers of one layer
  const bf16x8* qkv;           // [3D/16][D/32][64] fragments, rows grouped per head group as q|k|v per head
  const bf16x8* o;             // [D/16][D/32][64]
  const bf16x8* up;            // [M/16][D/32][64]
  const bf16x8* dn;            // [D/16][M/32][64]
  const bf16x8* cq;            // [D/16][D/32][64]   (cross-attention only)
  const bf16x8* co;            // [D/16][D/32][64]
  const float* qkv_b;          // [3D] in the same row order as qkv
  const float* o_b; const float* up_b; const float* dn_b; const float* cq_b; const float* co_b;
};

constexpr int FUSED_MAX_LAYERS = 16;

struct FusedNet {
  FusedLayer layer[FUSED_MAX_LAYERS];
  int L;
  const float* tok_w; const float* tok_b; const float* pos;   // fp32 [D,A], [D], [H,D]
  const bf16x8* head;          // [1][D/32][64] fragments of head_w padded to 16 rows
  const float* head_b;         // [A]
  const bf16x8* modw;          // [L*4D/16][D/32][64] FiLM projections of all layers (drafter kernel)
  const float* modb;           // [L*4D]
  const float* temb;           // [T, D]
  const float* cemb;           // [B, D] conditioning embedding (vector conditioning) or null
  // cross-attention operands of every (env, layer, head), prepared by tsdp_set_cond:
  const bf16x8* kc;            // [B][L][HEADS][S/16][DH/32][64]  keys as 16x16x32 A fragments
  const bf16x4* vct;           // [B][L][HEADS][DH/16][S/16][64]  values transposed as 16x16x16 A fragments
};

struct FusedIO {               // batched verification
  const float* x_rows;         // [R,H,A]
  const float* mod;            // [R, L*4*D] FiLM vectors (g1,b1,g2,b2 per layer)
  const int32_t* row_env;      // [R] or null (row index is the environment)
  const int32_t* d_R;          // live rows on the device, or null
  int R_cap;
  float* eps_out;              // [R,H,A]
};

struct SchedDev { const float* sqrt_abar; const float* sqrt_1m; const float* c0; const float* cx; const float* sigma; int T; };

struct DraftIO {               // drafter rollout
  int B;
  const int32_t* t0; const int32_t* K_eff; const int32_t* row_ptr; const float* sigma_scale; const int32_t* env_id;
  SchedDev tb; int clip; float clip_val; uint64_t seed;
  float* y;                    // [B,H,A]  in: the latents, out: the latents after the last drafted step
  float* states; float* eps_p; float* xi;   // [R,H,A] retained per drafted transition
};

__device__ __forceinline__ float gelu_fast(float x) {
  // x * sigmoid(2 sqrt(2/pi) (x + 0.044715 x^3)) == tanh form of GELU
  const float u = 1.5957691216057308f * (x + 0.044715f * x * x * x);
  return x / (1.0f + __expf(-u));
}

__device__ __forceinline__ bf16x4 to_bf16x4(f32x4 v) {
  bf16x4 r;
  r[0] = (__bf16)v[0]; r[1] = (__bf16)v[1]; r[2] = (__bf16)v[2]; r[3] = (__bf16)v[3];
  return r;
}

#ifndef TSDP_ABL
#define TSDP_ABL 0
#endif
#ifndef TSDP_INFLIGHT_CLK
#define TSDP_INFLIGHT_CLK 512
#endif
// acc[mb][nb] += W(frag rows mf0+mb, k-steps ks0..ks0+NKS) . act^T ; act is LDS bf16 [token][stride].
// Fully unrolled with compile-time trip counts.  The weight fragments of k-step k+PF are requested from L2
// before the MFMAs of k-step k issue, and the LDS operands of k-step k+1 are read while those of k-step k
// are multiplied; scheduling barriers keep the compiler from collapsing that software pipeline, and with no
// branch inside, the hardware wait counters stay exact.  PF is sized so that about TSDP_INFLIGHT_CLK cycles
// of MFMA work separate a request from its use (one L2 round trip) without flooding the 32 KB vector L1.
template <int MB, int NB, int NKS>
__device__ __forceinline__ void gemm_frag(const bf16x8* __restrict__ wp, int ks_total, int mf0, int ks0,
                                          const __bf16* act, int stride, f32x4 (&acc)[MB][NB], int lane) {
  constexpr int STEP_CLK = MB * NB * 16;              // MFMA cycles of one k-step
  constexpr int PFW = (TSDP_INFLIGHT_CLK + STEP_CLK - 1) / STEP_CLK;
  constexpr int PF0 = PFW < 1 ? 1 : (PFW > 4 ? 4 : PFW);
  constexpr int PF = PF0 > NKS ? NKS : PF0;
  const bf16x8* wl = wp + ((size_t)mf0 * ks_total + ks0) * 64 + lane;
  const __bf16* al = act + (lane & 15) * stride + (lane >> 4) * 8;
  bf16x8 a[PF + 1][MB];
  bf16x8 b[2][NB];
#pragma unroll
  for (int p = 0; p < PF; ++p)
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) a[p][mb] = wl[((size_t)mb * ks_total + p) * 64];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) b[0][nb] = *reinterpret_cast<const bf16x8*>(al + nb * 16 * stride);
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int k = 0; k < NKS; ++k) {
    if (k + PF < NKS) {
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
        a[(k + PF) % (PF + 1)][mb] = (TSDP_ABL & 1) ? a[0][mb] : wl[((size_t)mb * ks_total + k + PF) * 64];
    }
    if (k + 1 < NKS) {
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
        b[(k + 1) & 1][nb] = (TSDP_ABL & 2) ? b[0][nb] : *reinterpret_cast<const bf16x8*>(al + nb * 16 * stride + (k + 1) * 32);
    }
    __builtin_amdgcn_sched_barrier(0);
    if (!(TSDP_ABL & 4)) {
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
          acc[mb][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[k % (PF + 1)][mb], b[k & 1][nb], acc[mb][nb], 0, 0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
  }
}

// D model width, NT tokens per workgroup, H tokens per row, HEADS attention heads, CM conditioning mode,
// CH hidden-chunk width of the MLP, SX observation tokens (cross-attention).  256 threads = 4 wavefronts,
// each owning D/4 residual features of every token of the tile.
template <int D, int NT, int H, int HEADS, int CM, int CH, int SX>
struct FusedCfg {
  static constexpr int DH = D / HEADS;
  static constexpr int HP = DH >= 64 ? 1 : 64 / DH;     // heads per attention phase (64 features per phase)
  static constexpr int NB = NT / 16;                    // token fragments
  static constexpr int MBH = D / 64;                    // residual feature fragments per wave
  static constexpr int MBQ = HP * 3 * DH / 64;          // q|k|v feature fragments per wave and phase
  static constexpr int MBU = CH / 64;
  static constexpr int RPT = NT / H;                    // rows per tile
  static constexpr int NKF = H / 16;                    // key / query fragments of self-attention
  static constexpr int SF = SX / 16;                    // key fragments of cross-attention
  static constexpr int AS = D + 8;                      // LDS strides (bf16 elements), +8 against bank conflicts
  static constexpr int QS = DH + 8;
  static constexpr int VS = H + 4;
  static constexpr int US = CH + 8;
  static constexpr int ACT_B = NT * AS * 2;
  static constexpr int Q_B = HP * NT * QS * 2;
  static constexpr int VT_B = HP * RPT * DH * VS * 2;
  static constexpr int QKV_B = 2 * Q_B + VT_B;
  static constexpr int U_B = NT * US * 2;
  static constexpr int XT_B = NT * 64 * 4;              // fp32 latent staging of the verify kernel (A <= 64)
  static constexpr int SCR0_B = QKV_B > U_B ? QKV_B : U_B;
  static constexpr int SCR_B = SCR0_B > XT_B ? SCR0_B : XT_B;
  static constexpr int RED_B = 2 * 4 * NT * 4;
  static constexpr int LDS_B = ACT_B + SCR_B + RED_B;   // body; the drafter kernel appends its own regions
  static_assert(D % 64 == 0 && NT % 16 == 0 && H % 16 == 0 && NT % H == 0 && DH % 32 == 0, "shape");
  static_assert((HEADS % HP) == 0 && (HP * 3 * DH) % 64 == 0 && CH % 64 == 0 && (4 * D) % CH == 0, "shape");
  static_assert(CM == 0 || (SX % 16 == 0 && SX >= 16), "observation tokens must be a multiple of 16");
};

// One forward pass for the tile.  xt: LDS fp32 [NT][A] latent tokens (may alias the scratch region: it is
// consumed before the first barrier-protected write).  modp: FiLM vectors of local row r at
// modp + min(r, mod_rows-1)*mod_stride (global or LDS).  env_of_row: environment of local row r (cross-attention).
// eps is written to eo[t*A + a] for local tokens t < ntok_live.
template <int D, int NT, int H, int HEADS, int CM, int CH, int SX>
__device__ __forceinline__ void fused_body(const FusedNet& net, unsigned char* lds, const float* xt, int A,
                                           const float* modp, int mod_stride, int mod_rows,
                                           const int32_t* env_of_row, float* eo, int ntok_live) {
  using C = FusedCfg<D, NT, H, HEADS, CM, CH, SX>;
  constexpr int DH = C::DH, HP = C::HP, NB = C::NB, MBH = C::MBH, MBQ = C::MBQ, MBU = C::MBU, RPT = C::RPT,
                NKF = C::NKF, AS = C::AS, QS = C::QS, VS = C::VS, US = C::US, SF = C::SF;
  __bf16* act = reinterpret_cast<__bf16*>(lds);
  __bf16* qbuf = reinterpret_cast<__bf16*>(lds + C::ACT_B);
  __bf16* kbuf = qbuf + HP * NT * QS;
  __bf16* vtb = kbuf + HP * NT * QS;
  __bf16* ubuf = qbuf;
  float* red1 = reinterpret_cast<float*>(lds + C::ACT_B + C::SCR_B);
  float* red2 = red1 + 4 * NT;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l16 = lane & 15, lg = lane >> 4;

  // ---- token embedding in fp32: h = tok_w x + tok_b + pos -------------------------------------------------
  f32x4 h[MBH][NB];
#pragma unroll
  for (int mb = 0; mb < MBH; ++mb) {
    const int f0 = (wave * MBH + mb) * 16 + lg * 4;
    const f32x4 tb = *reinterpret_cast<const f32x4*>(net.tok_b + f0);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const int t = nb * 16 + l16;
      h[mb][nb] = tb + *reinterpret_cast<const f32x4*>(net.pos + (t % H) * D + f0);
    }
    for (int a = 0; a < A; ++a) {
      f32x4 wv;
#pragma unroll
      for (int i = 0; i < 4; ++i) wv[i] = net.tok_w[(f0 + i) * A + a];
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        const float xv = xt[(nb * 16 + l16) * A + a];
#pragma unroll
        for (int i = 0; i < 4; ++i) h[mb][nb][i] = fmaf(xv, wv[i], h[mb][nb][i]);
      }
    }
  }
  __syncthreads();

  // writes LN(h) (1 + g) + b as bf16 into act; which = 0 (attention) / 2 (MLP) selects the FiLM pair, -1 = none
  auto write_ln = [&](int layer, int which) {
    float mean[NB], rstd[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      float s = 0.0f;
#pragma unroll
      for (int mb = 0; mb < MBH; ++mb) s += h[mb][nb][0] + h[mb][nb][1] + h[mb][nb][2] + h[mb][nb][3];
      s += __shfl_xor(s, 16); s += __shfl_xor(s, 32);
      if (lane < 16) red1[wave * NT + nb * 16 + lane] = s;
    }
    __syncthreads();
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const int t = nb * 16 + l16;
      mean[nb] = (red1[t] + red1[NT + t] + red1[2 * NT + t] + red1[3 * NT + t]) * (1.0f / D);
      float q = 0.0f;
#pragma unroll
      for (int mb = 0; mb < MBH; ++mb)
#pragma unroll
        for (int i = 0; i < 4; ++i) { const float e = h[mb][nb][i] - mean[nb]; q += e * e; }
      q += __shfl_xor(q, 16); q += __shfl_xor(q, 32);
      if (lane < 16) red2[wave * NT + nb * 16 + lane] = q;
    }
    __syncthreads();
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const int t = nb * 16 + l16;
      rstd[nb] = rsqrtf((red2[t] + red2[NT + t] + red2[2 * NT + t] + red2[3 * NT + t]) * (1.0f / D) + 1e-5f);
    }
#pragma unroll
    for (int mb = 0; mb < MBH; ++mb) {
      const int f0 = (wave * MBH + mb) * 16 + lg * 4;
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        f32x4 v = (h[mb][nb] - mean[nb]) * rstd[nb];
        if (which >= 0) {
          const int row = min((nb * 16) / H, mod_rows - 1);
          const float* mp = modp + (size_t)row * mod_stride + layer * 4 * D + which * D + f0;
          const f32x4 g = *reinterpret_cast<const f32x4*>(mp);
          const f32x4 b = *reinterpret_cast<const f32x4*>(mp + D);
          v = v * (1.0f + g) + b;
        }
        *reinterpret_cast<bf16x4*>(act + (nb * 16 + l16) * AS + f0) = to_bf16x4(v);
      }
    }
    __syncthreads();
  };

  // softmax over keys for every query column of s (scores transposed: keys on rows), probabilities as bf16
  auto softmax_cols = [&](auto& s, auto& p, auto KF) {
    constexpr int NK = decltype(KF)::value;
    const float scale = rsqrtf((float)DH);
#pragma unroll
    for (int qf = 0; qf < NKF; ++qf) {
      float mx = -INFINITY;
#pragma unroll
      for (int kf = 0; kf < NK; ++kf)
#pragma unroll
        for (int i = 0; i < 4; ++i) { s[kf][qf][i] *= scale; mx = fmaxf(mx, s[kf][qf][i]); }
      mx = fmaxf(mx, __shfl_xor(mx, 16)); mx = fmaxf(mx, __shfl_xor(mx, 32));
      float sum = 0.0f;
#pragma unroll
      for (int kf = 0; kf < NK; ++kf)
#pragma unroll
        for (int i = 0; i < 4; ++i) { s[kf][qf][i] = __expf(s[kf][qf][i] - mx); sum += s[kf][qf][i]; }
      sum += __shfl_xor(sum, 16); sum += __shfl_xor(sum, 32);
      const float inv = 1.0f / sum;
#pragma unroll
      for (int kf = 0; kf < NK; ++kf) p[kf][qf] = to_bf16x4(s[kf][qf] * inv);
    }
  };

  // softmax(q k^T) v for one (row, head) held in LDS; the result overwrites the q rows of that (row, head)
  auto self_attention = [&](int r, int hh) {
    __bf16* qp = qbuf + (hh * NT + r * H) * QS;
    const __bf16* kp = kbuf + (hh * NT + r * H) * QS;
    f32x4 s[NKF][NKF];                                  // [key frag][query frag]; lane: query l16, keys lg*4..
#pragma unroll
    for (int kf = 0; kf < NKF; ++kf)
#pragma unroll
      for (int qf = 0; qf < NKF; ++qf) s[kf][qf] = f32x4{0, 0, 0, 0};
#pragma unroll
    for (int ks = 0; ks < DH / 32; ++ks) {
      bf16x8 ka[NKF], qb[NKF];
#pragma unroll
      for (int f = 0; f < NKF; ++f) {
        ka[f] = *reinterpret_cast<const bf16x8*>(kp + (f * 16 + l16) * QS + ks * 32 + lg * 8);
        qb[f] = *reinterpret_cast<const bf16x8*>(qp + (f * 16 + l16) * QS + ks * 32 + lg * 8);
      }
#pragma unroll
      for (int kf = 0; kf < NKF; ++kf)
#pragma unroll
        for (int qf = 0; qf < NKF; ++qf)
          s[kf][qf] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[kf], qb[qf], s[kf][qf], 0, 0, 0);
    }
    bf16x4 p[NKF][NKF];
    softmax_cols(s, p, std::integral_constant<int, NKF>{});
    const __bf16* vp = vtb + (size_t)(hh * RPT + r) * DH * VS;
#pragma unroll
    for (int cf = 0; cf < DH / 16; ++cf) {
      f32x4 o[NKF];
#pragma unroll
      for (int qf = 0; qf < NKF; ++qf) o[qf] = f32x4{0, 0, 0, 0};
#pragma unroll
      for (int kf = 0; kf < NKF; ++kf) {
        const s16x4 va = *reinterpret_cast<const s16x4*>(vp + (cf * 16 + l16) * VS + kf * 16 + lg * 4);
#pragma unroll
        for (int qf = 0; qf < NKF; ++qf)
          o[qf] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(va, __builtin_bit_cast(s16x4, p[kf][qf]), o[qf], 0, 0, 0);
      }
#pragma unroll
      for (int qf = 0; qf < NKF; ++qf)
        *reinterpret_cast<bf16x4*>(qp + (qf * 16 + l16) * QS + cf * 16 + lg * 4) = to_bf16x4(o[qf]);
    }
  };

  // attention of the H query tokens of (row, head) over the SX observation tokens of the row's environment;
  // keys and transposed values come from global memory already in MFMA fragment order
  auto cross_attention = [&](int r, int hh, int layer, int head) {
    if constexpr (CM == 1) {
      __bf16* qp = qbuf + (hh * NT + r * H) * QS;
      const size_t eh = ((size_t)env_of_row[r] * net.L + layer) * HEADS + head;
      const bf16x8* kcp = net.kc + eh * (SF * (DH / 32)) * 64 + lane;
      const bf16x4* vcp = net.vct + eh * ((DH / 16) * SF) * 64 + lane;
      f32x4 s[SF][NKF];
#pragma unroll
      for (int kf = 0; kf < SF; ++kf)
#pragma unroll
        for (int qf = 0; qf < NKF; ++qf) s[kf][qf] = f32x4{0, 0, 0, 0};
#pragma unroll
      for (int ks = 0; ks < DH / 32; ++ks) {
        bf16x8 qb[NKF];
#pragma unroll
        for (int f = 0; f < NKF; ++f) qb[f] = *reinterpret_cast<const bf16x8*>(qp + (f * 16 + l16) * QS + ks * 32 + lg * 8);
#pragma unroll
        for (int kf = 0; kf < SF; ++kf) {
          const bf16x8 ka = kcp[(kf * (DH / 32) + ks) * 64];
#pragma unroll
          for (int qf = 0; qf < NKF; ++qf)
            s[kf][qf] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka, qb[qf], s[kf][qf], 0, 0, 0);
        }
      }
      bf16x4 p[SF][NKF];
      softmax_cols(s, p, std::integral_constant<int, SF>{});
#pragma unroll
      for (int cf = 0; cf < DH / 16; ++cf) {
        f32x4 o[NKF];
#pragma unroll
        for (int qf = 0; qf < NKF; ++qf) o[qf] = f32x4{0, 0, 0, 0};
#pragma unroll
        for (int kf = 0; kf < SF; ++kf) {
          const s16x4 va = __builtin_bit_cast(s16x4, vcp[(cf * SF + kf) * 64]);
#pragma unroll
          for (int qf = 0; qf < NKF; ++qf)
            o[qf] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(va, __builtin_bit_cast(s16x4, p[kf][qf]), o[qf], 0, 0, 0);
        }
#pragma unroll
        for (int qf = 0; qf < NKF; ++qf)
          *reinterpret_cast<bf16x4*>(qp + (qf * 16 + l16) * QS + cf * 16 + lg * 4) = to_bf16x4(o[qf]);
      }
    }
  };

  auto add_bias_h = [&](const float* bias) {
#pragma unroll
    for (int mb = 0; mb < MBH; ++mb) {
      const f32x4 b = *reinterpret_cast<const f32x4*>(bias + (wave * MBH + mb) * 16 + lg * 4);
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) h[mb][nb] += b;
    }
  };

  for (int layer = 0; layer < net.L; ++layer) {
    const FusedLayer& W = net.layer[layer];
    // ================= self-attention block =================
    write_ln(layer, 0);
    for (int g = 0; g < HEADS / HP; ++g) {
      {
        f32x4 acc[MBQ][NB];
#pragma unroll
        for (int mb = 0; mb < MBQ; ++mb)
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) acc[mb][nb] = f32x4{0, 0, 0, 0};
        const int mf0 = g * (HP * 3 * DH / 16) + wave * MBQ;
        gemm_frag<MBQ, NB, D / 32>(W.qkv, D / 32, mf0, 0, act, AS, acc, lane);
        if (g > 0) __syncthreads();                     // previous group's O-projection has read qbuf
#pragma unroll
        for (int mb = 0; mb < MBQ; ++mb) {
          const int lr = (wave * MBQ + mb) * 16;        // first logical row of this fragment inside the group
          const int hh = lr / (3 * DH), cls = (lr / DH) % 3, c0 = lr % DH + lg * 4;
          const f32x4 bias = *reinterpret_cast<const f32x4*>(W.qkv_b + g * (HP * 3 * DH) + lr + lg * 4);
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) {
            const f32x4 v = acc[mb][nb] + bias;
            const int t = nb * 16 + l16;
            if (cls == 0) {
              *reinterpret_cast<bf16x4*>(qbuf + (hh * NT + t) * QS + c0) = to_bf16x4(v);
            } else if (cls == 1) {
              *reinterpret_cast<bf16x4*>(kbuf + (hh * NT + t) * QS + c0) = to_bf16x4(v);
            } else {
              __bf16* vp = vtb + ((size_t)(hh * RPT + t / H) * DH + c0) * VS + (t % H);
#pragma unroll
              for (int i = 0; i < 4; ++i) vp[i * VS] = (__bf16)v[i];
            }
          }
        }
      }
      __syncthreads();
      if (!(TSDP_ABL & 8)) for (int task = wave; task < RPT * HP; task += 4) self_attention(task % RPT, task / RPT);
      __syncthreads();
#pragma unroll
      for (int hh = 0; hh < HP; ++hh)
        gemm_frag<MBH, NB, DH / 32>(W.o, D / 32, wave * MBH, (g * HP + hh) * DH / 32, qbuf + hh * NT * QS, QS, h, lane);
    }
    add_bias_h(W.o_b);
    // ================= cross-attention block (observation tokens) =================
    if constexpr (CM == 1) {
      write_ln(layer, -1);                               // its barriers order the O-projection reads before qbuf writes
      for (int g = 0; g < HEADS / HP; ++g) {
        {
          f32x4 acc[1][NB];
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) acc[0][nb] = f32x4{0, 0, 0, 0};
          gemm_frag<1, NB, D / 32>(W.cq, D / 32, g * (HP * DH / 16) + wave, 0, act, AS, acc, lane);
          if (g > 0) __syncthreads();
          const int lr = wave * 16, hh = lr / DH, c0 = lr % DH + lg * 4;
          const f32x4 bias = *reinterpret_cast<const f32x4*>(W.cq_b + g * (HP * DH) + lr + lg * 4);
#pragma unroll
          for (int nb = 0; nb < NB; ++nb)
            *reinterpret_cast<bf16x4*>(qbuf + (hh * NT + nb * 16 + l16) * QS + c0) = to_bf16x4(acc[0][nb] + bias);
        }
        __syncthreads();
        if (!(TSDP_ABL & 8)) for (int task = wave; task < RPT * HP; task += 4) cross_attention(task % RPT, task / RPT, layer, g * HP + task / RPT);
        __syncthreads();
#pragma unroll
        for (int hh = 0; hh < HP; ++hh)
          gemm_frag<MBH, NB, DH / 32>(W.co, D / 32, wave * MBH, (g * HP + hh) * DH / 32, qbuf + hh * NT * QS, QS, h, lane);
      }
      add_bias_h(W.co_b);
    }
    // ================= MLP block =================
    write_ln(layer, 2);                                  // its barriers also order the projection reads before ubuf writes
    for (int c = 0; c < 4 * D / CH; ++c) {
      {
        f32x4 acc[MBU][NB];
#pragma unroll
        for (int mb = 0; mb < MBU; ++mb)
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) acc[mb][nb] = f32x4{0, 0, 0, 0};
        gemm_frag<MBU, NB, D / 32>(W.up, D / 32, c * (CH / 16) + wave * MBU, 0, act, AS, acc, lane);
        if (c > 0) __syncthreads();                     // previous chunk's down-projection has read ubuf
#pragma unroll
        for (int mb = 0; mb < MBU; ++mb) {
          const int f0 = (wave * MBU + mb) * 16 + lg * 4;
          const f32x4 bias = *reinterpret_cast<const f32x4*>(W.up_b + c * CH + f0);
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) {
            f32x4 v = acc[mb][nb] + bias;
#pragma unroll
            for (int i = 0; i < 4; ++i) v[i] = (TSDP_ABL & 16) ? v[i] : gelu_fast(v[i]);
            *reinterpret_cast<bf16x4*>(ubuf + (nb * 16 + l16) * US + f0) = to_bf16x4(v);
          }
        }
      }
      __syncthreads();
      gemm_frag<MBH, NB, CH / 32>(W.dn, 4 * D / 32, wave * MBH, c * (CH / 32), ubuf, US, h, lane);
    }
    add_bias_h(W.dn_b);
  }

  // ---- output head: eps = head_w LN(h) + head_b ---------------------------------------------------------
  write_ln(0, -1);
  {
    constexpr int NBW = (NB + 3) / 4;                   // token fragments per wave
    f32x4 e[1][NBW];
#pragma unroll
    for (int j = 0; j < NBW; ++j) e[0][j] = f32x4{0, 0, 0, 0};
    const int nb0 = wave * NBW;
    if (nb0 < NB) {
      gemm_frag<1, NBW, D / 32>(net.head, D / 32, 0, 0, act + nb0 * 16 * AS, AS, e, lane);
#pragma unroll
      for (int j = 0; j < NBW; ++j) {
        const int t = (nb0 + j) * 16 + l16;
        if (nb0 + j < NB && t < ntok_live) {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int a = lg * 4 + i;
            if (a < A) eo[t * A + a] = e[0][j][i] + net.head_b[a];
          }
        }
      }
    }
  }
}

// Batched verification: tile b of the grid takes rows b*RPT .. of the ragged batch.
template <int D, int NT, int H, int HEADS, int CM, int CH, int SX>
__global__ __launch_bounds__(256, (FusedCfg<D, NT, H, HEADS, CM, CH, SX>::LDS_B <= 80 * 1024 ? 2 : 1)) void k_fused_forward(FusedNet net, FusedIO io, int A) {
  using C = FusedCfg<D, NT, H, HEADS, CM, CH, SX>;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  __shared__ int32_t envs[C::RPT];
  const int R = io.d_R ? min(*io.d_R, io.R_cap) : io.R_cap;
  const int row0 = blockIdx.x * C::RPT;
  if (row0 >= R) return;
  const long long tok0 = (long long)row0 * H;
  const int ntok_live = min(NT, (R - row0) * H);
  float* xt = reinterpret_cast<float*>(lds + C::ACT_B);
  for (int i = threadIdx.x; i < NT * A; i += 256) xt[i] = i < ntok_live * A ? io.x_rows[tok0 * A + i] : 0.0f;
  if (threadIdx.x < C::RPT) {
    const int r = min(row0 + (int)threadIdx.x, R - 1);
    envs[threadIdx.x] = io.row_env ? io.row_env[r] : r;
  }
  __syncthreads();
  const int mod_stride = net.L * 4 * D;
  fused_body<D, NT, H, HEADS, CM, CH, SX>(net, lds, xt, A, io.mod + (size_t)row0 * mod_stride, mod_stride, R - row0, envs,
                                          io.eps_out + tok0 * A, ntok_live);
}

// Drafter rollout: the workgroup keeps the latents of RPT environments in LDS and runs their drafted
// transitions k = 1 .. max K_eff back to back; every step is one forward pass plus the DDPM step
//   y <- mu_p(y, eps, t_k) + s sigma_{t_k} xi_{env,t_k},   t_k = t0 - k + 1,
// and stores the input state, the drafter output and the noise of the transition in its ragged row.
template <int D, int NT, int H, int HEADS, int CM, int CH, int SX>
__global__ __launch_bounds__(256) void k_fused_draft(FusedNet net, DraftIO io, int A) {
  using C = FusedCfg<D, NT, H, HEADS, CM, CH, SX>;
  constexpr int RPT = C::RPT;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  __shared__ int32_t envs[RPT], s_t0[RPT], s_keff[RPT], s_rowp[RPT], s_kmax;
  const int DE = H * A;                                 // elements of one latent
  const int mod_stride = net.L * 4 * D;
  float* yt = reinterpret_cast<float*>(lds + C::LDS_B);              // [NT*A] latents
  float* et = yt + NT * A;                                           // [NT*A] drafter output
  float* modbuf = et + NT * A;                                       // [RPT][L*4D] FiLM vectors of this step
  __bf16* sgbuf = reinterpret_cast<__bf16*>(modbuf + RPT * mod_stride);   // [16][D+8] SiLU(g), rows >= RPT zero
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, l16 = lane & 15, lg = lane >> 4;
  const int env0 = blockIdx.x * RPT;
  if (threadIdx.x == 0) s_kmax = 0;
  __syncthreads();
  if (threadIdx.x < RPT) {
    const int b = env0 + threadIdx.x;
    const bool live = b < io.B;
    envs[threadIdx.x] = live ? b : io.B - 1;
    int t = live ? io.t0[b] : -1;
    if (t >= io.tb.T) t = io.tb.T - 1;
    s_t0[threadIdx.x] = t;
    const int ke = live ? io.K_eff[b] : 0;
    s_keff[threadIdx.x] = ke;
    s_rowp[threadIdx.x] = live ? io.row_ptr[b] : 0;
    atomicMax(&s_kmax, ke);
  }
  for (int i = threadIdx.x; i < 16 * (D + 8); i += 256) sgbuf[i] = (__bf16)0.0f;
  for (int i = threadIdx.x; i < NT * A; i += 256) {
    const int b = env0 + i / DE;
    yt[i] = b < io.B ? io.y[(size_t)env0 * DE + i] : 0.0f;
  }
  __syncthreads();
  const int kmax = s_kmax;
  for (int k = 1; k <= kmax; ++k) {
    // FiLM input of this step: SiLU(temb[t_k] + cemb[env]) as bf16 rows of the mod product's B operand
    for (int i = threadIdx.x; i < RPT * D; i += 256) {
      const int r = i / D, c = i % D;
      int t = s_t0[r] - k + 1;
      t = t < 0 ? 0 : t;
      float g = net.temb[(size_t)t * D + c];
      if (net.cemb) g += net.cemb[(size_t)envs[r] * D + c];
      sgbuf[r * (D + 8) + c] = (__bf16)(g / (1.0f + __expf(-g)));
    }
    __syncthreads();
    {
      constexpr int MBM = 4;
      const int fpw = net.L * 4 * D / 64;               // mod fragments per wave
      for (int f = 0; f < fpw; f += MBM) {
        f32x4 acc[MBM][1];
#pragma unroll
        for (int mb = 0; mb < MBM; ++mb) acc[mb][0] = f32x4{0, 0, 0, 0};
        gemm_frag<MBM, 1, D / 32>(net.modw, D / 32, wave * fpw + f, 0, sgbuf, D + 8, acc, lane);
        if (l16 < RPT) {
#pragma unroll
          for (int mb = 0; mb < MBM; ++mb) {
            const int f0 = (wave * fpw + f + mb) * 16 + lg * 4;
            const f32x4 b = *reinterpret_cast<const f32x4*>(net.modb + f0);
            *reinterpret_cast<f32x4*>(modbuf + l16 * mod_stride + f0) = acc[mb][0] + b;
          }
        }
      }
    }
    __syncthreads();
    fused_body<D, NT, H, HEADS, CM, CH, SX>(net, lds, yt, A, modbuf, mod_stride, RPT, envs, et, NT);
    __syncthreads();
    // DDPM step of transition k for the environments that still draft
    const int nblk = DE >> 2;
    for (int i = threadIdx.x; i < RPT * nblk; i += 256) {
      const int r = i / nblk, blk = i % nblk;
      if (k > s_keff[r]) continue;
      const int b = env0 + r;
      const int t = s_t0[r] - k + 1;
      const size_t row = (size_t)s_rowp[r] + k - 1;
      float* yp = yt + r * DE + 4 * blk;
      const float* ep = et + r * DE + 4 * blk;
      const f32x4 yv = *reinterpret_cast<const f32x4*>(yp);
      const f32x4 ev = *reinterpret_cast<const f32x4*>(ep);
      const float4 z4 = xi_block(io.seed, io.env_id ? io.env_id[b] : b, t, blk);
      const f32x4 z = {z4.x, z4.y, z4.z, z4.w};
      const float sa = io.tb.sqrt_abar[t], s1 = io.tb.sqrt_1m[t], c0 = io.tb.c0[t], cx = io.tb.cx[t];
      const float sig = io.sigma_scale[b] * io.tb.sigma[t];
      f32x4 o;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        float x0 = (yv[j] - s1 * ev[j]) / sa;
        if (io.clip) x0 = fminf(fmaxf(x0, -io.clip_val), io.clip_val);
        o[j] = c0 * x0 + cx * yv[j] + sig * z[j];
      }
      *reinterpret_cast<f32x4*>(io.states + row * DE + 4 * blk) = yv;
      *reinterpret_cast<f32x4*>(io.eps_p + row * DE + 4 * blk) = ev;
      *reinterpret_cast<f32x4*>(io.xi + row * DE + 4 * blk) = z;
      *reinterpret_cast<f32x4*>(yp) = o;
    }
    __syncthreads();
  }
  for (int i = threadIdx.x; i < NT * A; i += 256) {
    const int b = env0 + i / DE;
    if (b < io.B) io.y[(size_t)env0 * DE + i] = yt[i];
  }
}

// Cross-attention operands in MFMA fragment order (see FusedNet::kc / vct), from fp32 [B*S, d] projections.
__global__ void k_pack_kc(const float* __restrict__ Kp, __bf16* __restrict__ out, int B, int S, int d, int heads, int L,
                          int layer) {
  const int DH = d / heads, SF = S / 16, KS = DH / 32;
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (long long)B * heads * SF * KS * 64) return;
  const int lane = (int)(i % 64);
  long long r = i / 64;
  const int ks = (int)(r % KS); r /= KS;
  const int sf = (int)(r % SF); r /= SF;
  const int head = (int)(r % heads);
  const int env = (int)(r / heads);
  const float* src = Kp + ((long long)env * S + sf * 16 + (lane & 15)) * d + head * DH + ks * 32 + (lane >> 4) * 8;
  __bf16* dst = out + ((((((long long)env * L + layer) * heads + head) * SF + sf) * KS + ks) * 64 + lane) * 8;
  for (int j = 0; j < 8; ++j) dst[j] = (__bf16)src[j];
}

__global__ void k_pack_vct(const float* __restrict__ Vp, __bf16* __restrict__ out, int B, int S, int d, int heads, int L,
                           int layer) {
  const int DH = d / heads, SF = S / 16, CF = DH / 16;
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (long long)B * heads * CF * SF * 64) return;
  const int lane = (int)(i % 64);
  long long r = i / 64;
  const int sf = (int)(r % SF); r /= SF;
  const int cf = (int)(r % CF); r /= CF;
  const int head = (int)(r % heads);
  const int env = (int)(r / heads);
  const float* src = Vp + ((long long)env * S + sf * 16 + (lane >> 4) * 4) * d + head * DH + cf * 16 + (lane & 15);
  __bf16* dst = out + ((((((long long)env * L + layer) * heads + head) * CF + cf) * SF + sf) * 64 + lane) * 4;
  for (int j = 0; j < 4; ++j) dst[j] = (__bf16)src[(long long)j * d];
}

}  // namespace tsdp
