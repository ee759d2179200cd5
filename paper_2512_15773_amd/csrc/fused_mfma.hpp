// Fused MFMA forward of the denoiser (bf16 or fp32 operands, chosen by an element-type trait): one workgroup
// carries a tile of NT tokens (NT/H rows) through ALL layers without leaving the compute unit.  The fp32 residual
// stream lives in MFMA accumulator registers, activations are staged in LDS, and the weights stream from L2 straight
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
  const void* qkv;           // [3D/16][D/32][64] fragments, rows grouped per head group as q|k|v per head
  const void* o;             // [D/16][D/32][64]
  const void* up;            // [M/16][D/32][64]
  const void* dn;            // [D/16][M/32][64]
  const void* cq;            // [D/16][D/32][64]   (cross-attention only)
  const void* co;            // [D/16][D/32][64]
  const float* qkv_b;          // [3D] in the same row order as qkv
  const float* o_b; const float* up_b; const float* dn_b; const float* cq_b; const float* co_b;
};

constexpr int FUSED_MAX_LAYERS = 16;

struct FusedNet {
  FusedLayer layer[FUSED_MAX_LAYERS];
  int L;
  const float* tok_w; const float* tok_b; const float* pos;   // fp32 [D,A], [D], [H,D]
  const void* head;            // [ceil(A/16)][D/32][64] fragments of head_w, rows padded to a multiple of 16
  const float* head_b;         // [A]
  const void* modw;            // [L*4D/16][D/32][64] FiLM projections of all layers (drafter kernel)
  const float* modb;           // [L*4D]
  const float* modtab;         // [T][L*4D] FiLM vectors of every timestep when they depend on nothing else
                               // (token conditioning: no conditioning vector enters them), else null
  int rms;                     // 0 = LayerNorm, 1 = RMSNorm
  const float* temb;           // [T, D]
  const float* cemb;           // [B, D] conditioning embedding (vector conditioning) or null
  // cross-attention operands of every (env, layer, head), prepared by tsdp_set_cond:
  const bf16x8* kc;            // [B][L][HEADS][S/16][DH/32][64]  keys as 16x16x32 A fragments
  const bf16x4* vct;           // [B][L][HEADS][DH/16][S/16][64]  values transposed as 16x16x16 A fragments
};

struct FusedIO {               // batched verification
  const float* x_rows;         // [R,H,A]
  const float* mod;            // [R, L*4*D] FiLM vectors (g1,b1,g2,b2 per layer); unused when the network has modtab
  const int32_t* row_t;        // [R] timestep of the row minus t_sub (selects the modtab row)
  int t_sub, T;
  const int32_t* row_env;      // [R] or null (row index is the environment)
  const int32_t* d_R;          // live rows on the device, or null
  int R_cap;
  float* eps_out;              // [R,H,A]
};

struct SchedDev { const float* sqrt_abar; const float* sqrt_1m; const float* c0; const float* cx; const float* sigma; const float* ce; int T; };

struct DraftIO {               // drafter rollout
  int B;
  const int32_t* t0; const int32_t* K_eff; const int32_t* row_ptr; const float* sigma_scale; const int32_t* env_id;
  SchedDev tb; int clip; float clip_val; uint64_t seed;
  int mod_cols;                // columns of one in-kernel FiLM product: a multiple of RPT up to 16 (mod_cols/RPT steps at once)
  float* y;                    // [B,H,A]  in: the latents, out: the latents after the last drafted step
  float* states; float* eps_p; float* xi;   // [R,H,A] retained per drafted transition
  const int32_t* gate;         // chain driver: live row count of the round (0 = every environment finished), or null
};

__device__ __forceinline__ float gelu_fast(float x) {
  // x * sigmoid(2 sqrt(2/pi) (x + 0.044715 x^3)) == tanh form of GELU
  // exp(-u) as 2^(-u log2 e) and an approximate reciprocal: one v_exp_f32 and one v_rcp_f32 per element
  const float x2 = x * x;
  const float w = x * fmaf(x2, -0.044715f * 1.5957691216057308f * 1.4426950408889634f, -1.5957691216057308f * 1.4426950408889634f);
  return x * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(w));
}

// Element-type traits of the fused kernels.  A "fragment" is what one lane holds of a 16-row operand for one
// k-step: VW consecutive K entries (16 bytes), rows l%16, K offset (l/16)*VW.
//   TBF16: bf16 operands, k-step 32, one mfma_f32_16x16x32_bf16 per fragment pair.
//   TF32 : fp32 operands, k-step 16, four mfma_f32_16x16x4_f32 per fragment pair; MFMA j of the four contracts
//          the K entries {4g + j : g = 0..3}, which is just a permutation of the k-step's 16 entries.
struct TBF16 {
  typedef __bf16 elem;
  typedef bf16x8 frag;
  typedef bf16x4 vec4;
  static constexpr int VW = 8, KSTEP = 32, PAD = 8;
  static __device__ __forceinline__ void mma(const frag& a, const frag& b, f32x4& c) {
    c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
  }
  // 16-deep contraction with 4 entries per lane (keys (l/16)*4..): the P.V product of attention
  static __device__ __forceinline__ void mma16(const vec4& a, const vec4& b, f32x4& c) {
    c = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4, a), __builtin_bit_cast(s16x4, b), c, 0, 0, 0);
  }
  static __device__ __forceinline__ vec4 cvt(f32x4 v) {
    vec4 r;
    r[0] = (__bf16)v[0]; r[1] = (__bf16)v[1]; r[2] = (__bf16)v[2]; r[3] = (__bf16)v[3];
    return r;
  }
};

struct TF32 {
  typedef float elem;
  typedef f32x4 frag;
  typedef f32x4 vec4;
  static constexpr int VW = 4, KSTEP = 16, PAD = 4;
  static __device__ __forceinline__ void mma(const frag& a, const frag& b, f32x4& c) {
#pragma unroll
    for (int j = 0; j < 4; ++j) c = __builtin_amdgcn_mfma_f32_16x16x4f32(a[j], b[j], c, 0, 0, 0);
  }
  static __device__ __forceinline__ void mma16(const vec4& a, const vec4& b, f32x4& c) { mma(a, b, c); }
  static __device__ __forceinline__ vec4 cvt(f32x4 v) { return v; }
};

__device__ __forceinline__ float silu_fast(float g) { return g * __builtin_amdgcn_rcpf(1.0f + __expf(-g)); }

__device__ __forceinline__ bf16x4 to_bf16x4(f32x4 v) {
  bf16x4 r;
  r[0] = (__bf16)v[0]; r[1] = (__bf16)v[1]; r[2] = (__bf16)v[2]; r[3] = (__bf16)v[3];
  return r;
}

// Measured choices of the kernels below (each was timed against its alternative on the full-size workloads).
constexpr int INFLIGHT_CLK = 384;   // cycles of matrix work between the request of a weight fragment and its use
constexpr int PF_MAX = 4;           // upper limit of the weight ring's depth in k-steps

// Weight-streaming GEMM on fragments:  acc[mb][nb] += W(frag rows mf0+mb, k-steps ks0..ks0+NKS) . act^T,
// act = LDS bf16 [token][stride].  Fully unrolled with compile-time trip counts.  The weight fragments of
// k-step k+PF are requested from L2 before the MFMAs of k-step k issue and the LDS operands of k-step k+1
// are read while those of k-step k are multiplied; scheduling barriers keep the compiler from collapsing
// that software pipeline, and with no branch inside, the hardware wait counters stay exact.  PF is sized so
// that about INFLIGHT_CLK cycles of MFMA work separate a request from its use (one L2 round trip)
// without flooding the small vector L1.  issue() requests k-step 0 only and may be called a whole phase
// early (before an epilogue, a barrier or the attention of the previous phase); run() does the rest.
template <class TT, int MB, int NB, int NKS, int BD = 2>
struct FragGemm {
  typedef typename TT::frag frag;
  typedef typename TT::elem elem;
  static constexpr int STEP_CLK = MB * NB * 16;
  static constexpr int PFW = (INFLIGHT_CLK + STEP_CLK - 1) / STEP_CLK;
  static constexpr int PF0 = PFW < 1 ? 1 : (PFW > PF_MAX ? PF_MAX : PFW);
  static constexpr int PF = PF0 > NKS ? NKS : PF0;
  frag a[PF + 1][MB];
  const frag* wl;
  int kst;                     // elements between the fragment rows of consecutive mb (in k-steps)

  // fragment row of index mb is mf0 + mb*mfs
  __device__ __forceinline__ void issue(const void* __restrict__ wp, int ks_total, int mf0, int ks0, int lane, int mfs = 1) {
    wl = reinterpret_cast<const frag*>(wp) + ((size_t)mf0 * ks_total + ks0) * 64 + lane;
    kst = ks_total * mfs;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) a[0][mb] = wl[(size_t)mb * kst * 64];
  }

  // Priming: the first PF k-steps of this product requested stage by stage from inside the tail of the previous
  // product (whose own ring is draining then), so the weight stream does not stop at the phase boundary.
  // prime_begin sets the addresses, prime_stage(p) requests k-step p, run<PF>() then starts with a full ring.
  __device__ __forceinline__ void prime_begin(const void* __restrict__ wp, int ks_total, int mf0, int ks0, int lane, int mfs = 1) {
    wl = reinterpret_cast<const frag*>(wp) + ((size_t)mf0 * ks_total + ks0) * 64 + lane;
    kst = ks_total * mfs;
  }
  __device__ __forceinline__ void prime_stage(int p) {
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) a[p][mb] = wl[((size_t)mb * kst + p) * 64];
  }
  // to be called as side work of k-step k of a product of PREV k-steps: requests stage k - (PREV - PF)
  template <int PREV>
  __device__ __forceinline__ void prime_in_tail(int k) {
    static_assert(PREV >= PF, "the previous product is too short to hide the priming");
    if (k >= PREV - PF) prime_stage(k - (PREV - PF));
  }

  struct NoSide { __device__ __forceinline__ void operator()(int) const {} };

  __device__ __forceinline__ void run(const elem* act, int stride, f32x4 (&acc)[MB][NB], int lane) {
    run(act, stride, acc, lane, NoSide{});
  }

  // side(k) is called once per k-step after its MFMAs have been issued: independent vector work placed there
  // (an epilogue of the previous product) executes while the matrix pipeline is busy.  PRIMED = ring stages
  // already requested (1 after issue(), PF after priming).
  template <class Side, int PRIMED = 1>
  __device__ __forceinline__ void run(const elem* act, int stride, f32x4 (&acc)[MB][NB], int lane, Side&& side,
                                      std::integral_constant<int, PRIMED> = {}) {
    const elem* al = act + (lane & 15) * stride + (lane >> 4) * TT::VW;
    frag b[BD][NB];
#pragma unroll
    for (int p = PRIMED; p < PF; ++p)
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) a[p][mb] = wl[((size_t)mb * kst + p) * 64];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) b[0][nb] = *reinterpret_cast<const frag*>(al + nb * 16 * stride);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int k = 0; k < NKS; ++k) {
      if (k + PF < NKS) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
          a[(k + PF) % (PF + 1)][mb] = wl[((size_t)mb * kst + k + PF) * 64];
      }
      if (BD == 2 && k + 1 < NKS) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
          b[(k + 1) & 1][nb] = *reinterpret_cast<const frag*>(al + nb * 16 * stride + (k + 1) * TT::KSTEP);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
          TT::mma(a[k % (PF + 1)][mb], b[k % BD][nb], acc[mb][nb]);
      side(k);
      if (BD == 1 && k + 1 < NKS) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) b[0][nb] = *reinterpret_cast<const frag*>(al + nb * 16 * stride + (k + 1) * TT::KSTEP);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }
};

// D model width, NT tokens per workgroup, H tokens per row, HEADS attention heads, CM conditioning mode,
// CH hidden-chunk width of the MLP, SX observation tokens (cross-attention), HP heads per self-attention phase,
// HPX heads per cross-attention phase (it needs no key / value buffers in LDS, so it can take more heads at once),
// NW wavefronts per workgroup; every wavefront owns D/NW residual features of every token of the tile.
template <class TT_, int D_, int NT_, int H_, int HEADS_, int CM_, int CH_, int SX_, int HP_, int NW_, int HPX_ = HP_>
struct FusedCfg {
  typedef TT_ TT;
  static constexpr int ES = sizeof(typename TT_::elem), KSTEP = TT_::KSTEP;
  static constexpr int D = D_, NT = NT_, H = H_, HEADS = HEADS_, CM = CM_, CH = CH_, SX = SX_, HP = HP_, NW = NW_, HPX = HPX_;
  static constexpr int THREADS = NW * 64;
  static constexpr int DH = D / HEADS;
  static constexpr int NB = NT / 16;                    // token fragments
  static constexpr int MBH = D / 16 / NW;               // residual feature fragments per wave
  static constexpr int MBQ = HP * 3 * DH / 16 / NW;     // q|k|v feature fragments per wave and phase
  static constexpr int MBC = HPX * DH / 16 / NW;        // cross-attention query fragments per wave and phase
  static constexpr int MBU = CH / 16 / NW;
  static constexpr int RPT = NT / H;                    // rows per tile
  static constexpr int NKF = H / 16;                    // key / query fragments of self-attention
  static constexpr int SF = SX / 16;                    // key fragments of cross-attention
  static constexpr int AS = D + TT_::PAD;               // LDS strides (elements), +16 bytes against bank conflicts
  static constexpr int QS = DH + TT_::PAD;
  static constexpr int VS = H + 4;
  static constexpr int US = CH + TT_::PAD;
  static constexpr int ACT_B = NT * AS * ES;
  static constexpr int Q_B = HP * NT * QS * ES;
  static constexpr int VT_B = HP * RPT * DH * VS * ES;
  static constexpr int QKV0_B = 2 * Q_B + VT_B;
  static constexpr int QX_B = CM_ == 1 ? NT * (HPX * DH + TT_::PAD) * ES : 0;   // queries of one cross-attention phase
  static constexpr int QKV_B = QKV0_B > QX_B ? QKV0_B : QX_B;
  static constexpr int U_B = NT * US * ES;
  static constexpr int XT_B = NT * 64 * 4;              // fp32 latent staging of the verify kernel (A <= 64)
  // two hidden-chunk buffers (one barrier per chunk instead of two) when a single workgroup owns the CU's LDS
  static constexpr bool UDB = (NW == 8) && (ACT_B + 2 * U_B + 2 * NW * NT * 4 + 7 * D * 4 <= 160 * 1024) && (2 * U_B >= QKV_B);
  static constexpr int UU_B = UDB ? 2 * U_B : U_B;
  static constexpr int SCR0_B = QKV_B > UU_B ? QKV_B : UU_B;
  static constexpr int SCR_B = SCR0_B > XT_B ? SCR0_B : XT_B;
  static constexpr int RED_B = 2 * NW * NT * 4;
  static constexpr int UB_B = UDB ? 7 * D * 4 : 0;      // pipelined MLP: the layer's up-projection bias and the three residual biases (fp32)
  static constexpr int LDS_B = ACT_B + SCR_B + RED_B + UB_B;   // body; the drafter kernel appends its own regions
  static constexpr int WG_PER_CU = LDS_B <= 80 * 1024 && NW <= 4 ? 2 : 1;
  static constexpr bool LN_STAGE = true;                // FiLM vectors come from global memory: fetch them cooperatively
  static constexpr int WAVES_PER_SIMD = (WG_PER_CU * NW + 3) / 4;
  static constexpr int BD = WAVES_PER_SIMD >= 2 ? 1 : 2; // LDS operand buffers: a second wave on the SIMD hides LDS latency
  static constexpr bool XPF = WAVES_PER_SIMD == 1;      // request the first weight fragments of a phase one phase early
  static_assert(D % (16 * NW) == 0 && NT % 16 == 0 && H % 16 == 0 && NT % H == 0 && DH % KSTEP == 0, "shape");
  static_assert(D % KSTEP == 0 && CH % KSTEP == 0, "shape");
  static_assert((HEADS % HP) == 0 && (HP * 3 * DH) % (16 * NW) == 0 && (CM == 0 || (HPX * DH) % (16 * NW) == 0) &&
                (HEADS % HPX) == 0, "shape");
  static_assert(CH % (16 * NW) == 0 && (4 * D) % CH == 0, "shape");
  static_assert(CM == 0 || (SX % 16 == 0 && SX >= 16 && ES == 2), "cross-attention: bf16 only, tokens a multiple of 16");
};

// Configuration of the persistent drafter: a rollout has few workgroups in flight (one per environment tile), so no
// second wave hides latency; it therefore always prefetches across phases and double-buffers the LDS operands.
template <class Base>
struct DraftCfg : Base {
  static constexpr bool XPF = true;
  static constexpr bool LN_STAGE = false;               // the drafter's FiLM vectors are already in LDS (or a small table)
  static constexpr int BD = 2;
};

// One forward pass for the tile.  xt: LDS fp32 [NT][A] latent tokens (may alias the scratch region: it is
// consumed before the first barrier-protected write).  mrow[r]: FiLM vectors of local row r, all layers (global
// or LDS).  env_of_row: environment of local row r (cross-attention).
// eps is written to eo[t*A + a] for local tokens t < ntok_live.
template <class C>
__device__ __forceinline__ void fused_body(const FusedNet& net, unsigned char* lds, const float* xt, int A,
                                           const float* const* mrow,
                                           const int32_t* env_of_row, float* eo, int ntok_live,
                                           const float* lbias = nullptr) {
  constexpr int D = C::D, NT = C::NT, H = C::H, HEADS = C::HEADS, CM = C::CM, CH = C::CH, NW = C::NW;
  constexpr int DH = C::DH, HP = C::HP, NB = C::NB, MBH = C::MBH, MBQ = C::MBQ, MBU = C::MBU, MBC = C::MBC,
                RPT = C::RPT, NKF = C::NKF, AS = C::AS, QS = C::QS, VS = C::VS, US = C::US, SF = C::SF;
  constexpr int NG = HEADS / HP, NC = 4 * D / CH;
  // Self-attention queries (and, over them, the attention output) of a head group: token-major [NT][HP*DH + pad], so
  // the output projection contracts all heads of the group in one product; keys stay per head [HP][NT][DH + pad].
  constexpr int QTS = HP * DH + C::TT::PAD;
  static_assert(C::NT * QTS <= C::HP * C::NT * C::QS, "the token-major queries fit the per-head query region");
  typedef typename C::TT TT;
  typedef typename TT::elem elem;
  typedef typename TT::frag frag;
  typedef typename TT::vec4 vec4;
  constexpr int KSTEP = TT::KSTEP, VW = TT::VW;
  elem* act = reinterpret_cast<elem*>(lds);
  elem* qbuf = reinterpret_cast<elem*>(lds + C::ACT_B);
  elem* kbuf = qbuf + HP * NT * QS;                     // (the token-major queries need NT * QTS <= HP * NT * QS elements)
  elem* vtb = kbuf + HP * NT * QS;
  elem* ubuf = qbuf;
  float* red1 = reinterpret_cast<float*>(lds + C::ACT_B + C::SCR_B);
  float* red2 = red1 + NW * NT;
  float* upb = red2 + NW * NT;                          // pipelined MLP: biases of the current layer, [4D] up-projection,
  float* resb = upb + 4 * D;                            // then [3][D] self-attention output, cross-attention output, MLP down

  int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave index as a scalar
  __builtin_assume(wave >= 0 && wave < NW);
  int l16 = lane & 15, lg = lane >> 4;
  // Makes the lane coordinates opaque at phase boundaries: addresses derived from them are then recomputed
  // where they are used instead of being hoisted out of the layer loop and spilled to scratch.
#define FENCE_LANE_IDS() asm volatile("" : "+v"(lane), "+v"(l16), "+v"(lg))

  constexpr int BD = C::BD;
  constexpr bool XPF = C::XPF;
  constexpr int KD = D / KSTEP, KH = DH / KSTEP, KC = CH / KSTEP, KM = 4 * D / KSTEP;   // k-steps of D, DH, CH, 4D
  typedef FragGemm<TT, MBQ, NB, KD, BD> GQ;             // q|k|v projection of one head group
  typedef FragGemm<TT, MBH, NB, HP * KH, BD> GO;        // output projection, the slice of K of one head group
  typedef FragGemm<TT, MBU, NB, KD, BD> GU;             // MLP up, one hidden chunk
  typedef FragGemm<TT, MBH, NB, KC, BD> GD;             // MLP down, one hidden chunk of K
  typedef FragGemm<TT, (MBC > 0 ? MBC : 1), NB, KD, BD> GC;   // cross-attention query projection

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

  // writes LN(h) (1 + g) + b as bf16 into act; which = 0 (attention) / 2 (MLP) selects the FiLM pair, -1 = none.
  // Statistics: per-wave partial results (fp32) exchanged through LDS, one barrier.
  auto write_ln = [&](int layer, int which) {
    FENCE_LANE_IDS();
    // FiLM vectors of the tile's rows: requested first, so they arrive while the statistics are reduced
    // (only where they fit in 64 registers; otherwise they are read fragment row by fragment row)
    constexpr bool LNPF = MBH * RPT * 2 <= 16;
    constexpr int FR = LNPF ? RPT : 1;
    f32x4 fg[MBH][FR], fb[MBH][FR];
    if (LNPF && which >= 0) {
#pragma unroll
      for (int mb = 0; mb < MBH; ++mb)
#pragma unroll
        for (int r = 0; r < RPT; ++r) {
          const float* mp = mrow[r] + layer * 4 * D + which * D + (wave * MBH + mb) * 16 + lg * 4;
          fg[mb][r] = *reinterpret_cast<const f32x4*>(mp);
          fb[mb][r] = *reinterpret_cast<const f32x4*>(mp + D);
        }
    }
    // Otherwise the wave fetches its block [row][g|b][its features] cooperatively, 16 distinct bytes per lane and
    // request (read fragment by fragment every lane would re-read what 15 others read, in MBH dependent batches),
    // and passes it to its lanes through the scratch region, which is free between the two barriers below.
    constexpr bool LNST = !LNPF && C::LN_STAGE && (NW * RPT * 2 * MBH * 16 * 4 <= C::SCR_B);
    constexpr int CHK = RPT * 2 * MBH * 4, CPL = (CHK + 63) / 64;
    f32x4 st[LNST ? CPL : 1];
    if (LNST && which >= 0) {
#pragma unroll
      for (int i = 0; i < CPL; ++i) {
        const int c = lane + 64 * i;
        if (c < CHK) {
          const int r = c / (2 * MBH * 4), rem = c % (2 * MBH * 4);
          st[i] = *reinterpret_cast<const f32x4*>(mrow[r] + layer * 4 * D + which * D + (rem / (MBH * 4)) * D +
                                                  (wave * MBH + (rem / 4) % MBH) * 16 + (rem % 4) * 4);
        }
      }
    }
    // Statistics.  fp32 networks (results are held to 1e-5): without cancellation -- every wave reduces the sum of
    // its D/NW features of a token and then their squared deviations from its own mean (registers only); the NW
    // (sum, M2) pairs are combined after one barrier, M2 = sum_w M2_w + n_w (mean_w - mean)^2; the roundings are
    // pinned (no contraction), so every tile variant gives the same bits.  bf16 networks: one pass over x and x^2
    // (its fp32 cancellation error, 2^-24 mean^2 / var, is far below the bf16 rounding of the operands).
    // RMSNorm takes the plain second moment either way.
    constexpr bool CENTRED = std::is_same<TT, TF32>::value;
    constexpr float NWF = (float)(D / NW);              // features per wave
    float mean[NB], rstd[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      float s = 0.0f, q = 0.0f;
      if (CENTRED && !net.rms) {
#pragma unroll
        for (int mb = 0; mb < MBH; ++mb)
#pragma unroll
          for (int i = 0; i < 4; ++i) s += h[mb][nb][i];
        s += __shfl_xor(s, 16); s += __shfl_xor(s, 32);
        const float mw = __fmul_rn(s, 1.0f / NWF);
#pragma unroll
        for (int mb = 0; mb < MBH; ++mb)
#pragma unroll
          for (int i = 0; i < 4; ++i) { const float dv = __fsub_rn(h[mb][nb][i], mw); q = fmaf(dv, dv, q); }
      } else {
#pragma unroll
        for (int mb = 0; mb < MBH; ++mb)
#pragma unroll
          for (int i = 0; i < 4; ++i) { s += h[mb][nb][i]; q = fmaf(h[mb][nb][i], h[mb][nb][i], q); }
        s += __shfl_xor(s, 16); s += __shfl_xor(s, 32);
      }
      q += __shfl_xor(q, 16); q += __shfl_xor(q, 32);
      if (lane < 16) { red1[wave * NT + nb * 16 + lane] = s; red2[wave * NT + nb * 16 + lane] = q; }
    }
    __syncthreads();
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const int t = nb * 16 + l16;
      float sw[NW], s = 0.0f, q = 0.0f;
#pragma unroll
      for (int w = 0; w < NW; ++w) { sw[w] = red1[w * NT + t]; s += sw[w]; q += red2[w * NT + t]; }
      mean[nb] = net.rms ? 0.0f : s * (1.0f / D);     // RMSNorm: no centring, the second moment as it is
      if (CENTRED) {
        if (!net.rms) {
#pragma unroll
          for (int w = 0; w < NW; ++w) {
            const float dm = __fsub_rn(__fmul_rn(sw[w], 1.0f / NWF), mean[nb]);
            q = fmaf(__fmul_rn(NWF, dm), dm, q);
          }
        }
        rstd[nb] = rsqrtf(q * (1.0f / D) + 1e-5f);
      } else {
        rstd[nb] = rsqrtf(fmaxf(q * (1.0f / D) - mean[nb] * mean[nb], 0.0f) + 1e-5f);
      }
    }
    float* fs = reinterpret_cast<float*>(lds + C::ACT_B) + wave * (CHK * 4);   // this wave's staged FiLM block
    if (LNST && which >= 0) {
#pragma unroll
      for (int i = 0; i < CPL; ++i) {
        const int c = lane + 64 * i;
        if (c < CHK) *reinterpret_cast<f32x4*>(fs + c * 4) = st[i];
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();                  // written and read by the same wave: LDS keeps its order
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
#pragma unroll
    for (int mb = 0; mb < MBH; ++mb) {
      const int f0 = (wave * MBH + mb) * 16 + lg * 4;
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        f32x4 v = (h[mb][nb] - mean[nb]) * rstd[nb];
        if (which >= 0) {
          if (LNPF) {
            v = v * (1.0f + fg[mb][(nb * 16) / H]) + fb[mb][(nb * 16) / H];
          } else if (LNST) {
            const int r = (nb * 16) / H;
            const f32x4 g = *reinterpret_cast<const f32x4*>(fs + ((r * 2 + 0) * MBH + mb) * 16 + lg * 4);
            const f32x4 b = *reinterpret_cast<const f32x4*>(fs + ((r * 2 + 1) * MBH + mb) * 16 + lg * 4);
            v = v * (1.0f + g) + b;
          } else {
            const float* mp = mrow[(nb * 16) / H] + layer * 4 * D + which * D + f0;
            const f32x4 g = *reinterpret_cast<const f32x4*>(mp);
            const f32x4 b = *reinterpret_cast<const f32x4*>(mp + D);
            v = v * (1.0f + g) + b;
          }
        }
        *reinterpret_cast<vec4*>(act + (nb * 16 + l16) * AS + f0) = TT::cvt(v);
      }
      if (!LNPF && !LNST) __builtin_amdgcn_sched_barrier(0);   // keep the FiLM loads of one fragment row in flight, not all
    }
    __syncthreads();
  };

  // softmax over the keys (rows of s, NK key fragments) for the 16 queries of one fragment
  auto softmax_col = [&](auto& s, auto& p, auto KF) {
    constexpr int NK = decltype(KF)::value;
    const float scale = rsqrtf((float)DH);
    float mx = -INFINITY;
#pragma unroll
    for (int kf = 0; kf < NK; ++kf)
#pragma unroll
      for (int i = 0; i < 4; ++i) { s[kf][i] *= scale; mx = fmaxf(mx, s[kf][i]); }
    mx = fmaxf(mx, __shfl_xor(mx, 16)); mx = fmaxf(mx, __shfl_xor(mx, 32));
    float sum = 0.0f;
#pragma unroll
    for (int kf = 0; kf < NK; ++kf)
#pragma unroll
      for (int i = 0; i < 4; ++i) { s[kf][i] = __expf(s[kf][i] - mx); sum += s[kf][i]; }
    sum += __shfl_xor(sum, 16); sum += __shfl_xor(sum, 32);
    const float inv = __builtin_amdgcn_rcpf(sum);     // one approximate reciprocal (1 ulp) instead of an IEEE division
#pragma unroll
    for (int kf = 0; kf < NK; ++kf) p[kf] = TT::cvt(s[kf] * inv);
  };

  // softmax(q k^T) v for query fragment qf of (row, head) held in LDS; the result overwrites those q rows
  auto self_attention = [&](int r, int hh, int qf) {
    elem* qp = qbuf + (r * H + qf * 16) * QTS + hh * DH;
    const elem* kp = kbuf + (hh * NT + r * H) * QS;
    f32x4 s[NKF];                                       // [key frag]; lane: query l16, keys lg*4..
#pragma unroll
    for (int kf = 0; kf < NKF; ++kf) s[kf] = f32x4{0, 0, 0, 0};
#pragma unroll
    for (int ks = 0; ks < KH; ++ks) {
      const frag qb = *reinterpret_cast<const frag*>(qp + l16 * QTS + ks * KSTEP + lg * VW);
#pragma unroll
      for (int kf = 0; kf < NKF; ++kf) {
        const frag ka = *reinterpret_cast<const frag*>(kp + (kf * 16 + l16) * QS + ks * KSTEP + lg * VW);
        TT::mma(ka, qb, s[kf]);
      }
    }
    vec4 p[NKF];
    softmax_col(s, p, std::integral_constant<int, NKF>{});
    const elem* vp = vtb + (size_t)(hh * RPT + r) * DH * VS;
#pragma unroll
    for (int cf = 0; cf < DH / 16; ++cf) {
      f32x4 o = f32x4{0, 0, 0, 0};
#pragma unroll
      for (int kf = 0; kf < NKF; ++kf) {
        const vec4 va = *reinterpret_cast<const vec4*>(vp + (cf * 16 + l16) * VS + kf * 16 + lg * 4);
        TT::mma16(va, p[kf], o);
      }
      *reinterpret_cast<vec4*>(qp + l16 * QTS + cf * 16 + lg * 4) = TT::cvt(o);
    }
  };

  // Cross-attention of query fragment qf of (row, head) over the SX observation tokens of the row's environment.
  // Keys and transposed values come from global memory already in MFMA fragment order: cross_load_k / cross_load_v
  // request them, cross_scores and cross_pv consume them.
  constexpr int SFc = SF > 0 ? SF : 1;
  constexpr int KHc = KH > 0 ? KH : 1;
  // keys of (row r, head) as 16x16x32 A fragments, transposed values as 16x16x16 A fragments
  auto cross_load_k = [&](int r, int layer, int head, bf16x8 (&ka)[KHc][SFc]) {
    if constexpr (CM == 1) {
      const size_t eh = ((size_t)env_of_row[r] * net.L + layer) * HEADS + head;
      const bf16x8* kcp = net.kc + eh * (SF * (KH)) * 64 + lane;
#pragma unroll
      for (int ks = 0; ks < KH; ++ks)
#pragma unroll
        for (int kf = 0; kf < SF; ++kf) ka[ks][kf] = kcp[(kf * (KH) + ks) * 64];
    }
  };
  auto cross_load_v = [&](int r, int layer, int head, bf16x4 (&va)[DH / 16][SFc]) {
    if constexpr (CM == 1) {
      const size_t eh = ((size_t)env_of_row[r] * net.L + layer) * HEADS + head;
      const bf16x4* vcp = net.vct + eh * ((DH / 16) * SF) * 64 + lane;
#pragma unroll
      for (int cf = 0; cf < DH / 16; ++cf)
#pragma unroll
        for (int kf = 0; kf < SF; ++kf) va[cf][kf] = vcp[(cf * SF + kf) * 64];
    }
  };
  // qp: the 16 queries of the task, row stride qs.  scores: p = softmax over the keys of (k q^T)
  auto cross_scores = [&](const __bf16* qp, int qs, const bf16x8 (&ka)[KHc][SFc], bf16x4 (&p)[SFc]) {
    if constexpr (CM == 1) {
      f32x4 s[SF];
#pragma unroll
      for (int kf = 0; kf < SF; ++kf) s[kf] = f32x4{0, 0, 0, 0};
#pragma unroll
      for (int ks = 0; ks < KH; ++ks) {
        const bf16x8 qb = *reinterpret_cast<const bf16x8*>(qp + l16 * qs + ks * 32 + lg * 8);
#pragma unroll
        for (int kf = 0; kf < SF; ++kf) s[kf] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[ks][kf], qb, s[kf], 0, 0, 0);
      }
      vec4 pv[SF];
      softmax_col(s, pv, std::integral_constant<int, SF>{});
#pragma unroll
      for (int kf = 0; kf < SF; ++kf) p[kf] = __builtin_bit_cast(bf16x4, pv[kf]);
    }
  };
  // the attention output p v overwrites the task's queries
  auto cross_pv = [&](__bf16* qp, int qs, const bf16x4 (&p)[SFc], const bf16x4 (&va)[DH / 16][SFc]) {
    if constexpr (CM == 1) {
#pragma unroll
      for (int cf = 0; cf < DH / 16; ++cf) {
        f32x4 o = f32x4{0, 0, 0, 0};
#pragma unroll
        for (int kf = 0; kf < SF; ++kf)
          o = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4, va[cf][kf]),
                                                        __builtin_bit_cast(s16x4, p[kf]), o, 0, 0, 0);
        *reinterpret_cast<bf16x4*>(qp + l16 * qs + cf * 16 + lg * 4) = to_bf16x4(o);
      }
    }
  };

  // residual bias `which` (0 self-attention output, 1 cross-attention output, 2 MLP down): from LDS where the layer's
  // biases are staged (a global load here would be waited for with nothing to overlap it), else from global memory
  constexpr bool BSTAGE = C::UDB && !XPF && (NC % 2 == 0);
  auto add_bias_h = [&](const float* bias, int layer, int which) {
    if (BSTAGE) bias = resb + which * D;
    else if (lbias) bias = lbias + (layer * 3 + which) * D;
#pragma unroll
    for (int mb = 0; mb < MBH; ++mb) {
      const f32x4 b = *reinterpret_cast<const f32x4*>(bias + (wave * MBH + mb) * 16 + lg * 4);
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) h[mb][nb] += b;
    }
  };

  GQ gq;
  if (XPF) gq.issue(net.layer[0].qkv, KD, wave, 0, lane, NW);
  for (int layer = 0; layer < net.L; ++layer) {
    const FusedLayer& W = net.layer[layer];
    // ================= self-attention block =================
    write_ln(layer, 0);
    if constexpr (BSTAGE) {
      // The layer's biases that are added outside a product's own latency shadow go to LDS: the MLP's GELU runs inside
      // the products, where registers are scarce and a global load would queue behind the weight requests, and a
      // residual bias is needed right after a product with nothing to overlap a global load.  Written here, after
      // the barriers of the LayerNorm above: every wave has finished the previous layer, whose last act is to add
      // its down-projection bias; the first use of the new values is several barriers away.
      for (int i = threadIdx.x * 4; i < 4 * D; i += C::THREADS * 4)
        *reinterpret_cast<f32x4*>(upb + i) = *reinterpret_cast<const f32x4*>(W.up_b + i);
      for (int i = threadIdx.x * 4; i < D; i += C::THREADS * 4) {
        *reinterpret_cast<f32x4*>(resb + i) = *reinterpret_cast<const f32x4*>(W.o_b + i);
        if constexpr (CM == 1) *reinterpret_cast<f32x4*>(resb + D + i) = *reinterpret_cast<const f32x4*>(W.co_b + i);
        *reinterpret_cast<f32x4*>(resb + 2 * D + i) = *reinterpret_cast<const f32x4*>(W.dn_b + i);
      }
    }
    for (int g = 0; g < NG; ++g) {
      FENCE_LANE_IDS();
      GO go;
      {
        f32x4 acc[MBQ][NB];
        f32x4 bias[MBQ];
#pragma unroll
        for (int mb = 0; mb < MBQ; ++mb) {
          bias[mb] = *reinterpret_cast<const f32x4*>(W.qkv_b + g * (HP * 3 * DH) + (mb * NW + wave) * 16 + lg * 4);
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) acc[mb][nb] = f32x4{0, 0, 0, 0};
        }
        if (!XPF) gq.issue(W.qkv, KD, g * (HP * 3 * DH / 16) + wave, 0, lane, NW);
        gq.run(act, AS, acc, lane);
        if (XPF) go.issue(W.o, KD, wave * MBH, g * HP * KH, lane);      // needed only after the attention
        if (g > 0) __syncthreads();                     // previous group's O-projection has read qbuf
#pragma unroll
        for (int mb = 0; mb < MBQ; ++mb) {
          const int lr = (mb * NW + wave) * 16;         // first logical row of this fragment inside the group (rows are
                                                        // dealt round-robin so every wave gets q, k and v rows)
          const int hh = lr / (3 * DH), cls = (lr / DH) % 3, c0 = lr % DH + lg * 4;
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) {
            const f32x4 v = acc[mb][nb] + bias[mb];
            const int t = nb * 16 + l16;
            if (cls == 0) {
              *reinterpret_cast<vec4*>(qbuf + t * QTS + hh * DH + c0) = TT::cvt(v);
            } else if (cls == 1) {
              *reinterpret_cast<vec4*>(kbuf + (hh * NT + t) * QS + c0) = TT::cvt(v);
            } else {
              elem* vp = vtb + ((size_t)(hh * RPT + t / H) * DH + c0) * VS + (t % H);
#pragma unroll
              for (int i = 0; i < 4; ++i) vp[i * VS] = (elem)v[i];
            }
          }
        }
      }
      __syncthreads();
      for (int task = wave; task < RPT * HP * NKF; task += NW)
          self_attention((task / NKF) % RPT, task / (NKF * RPT), task % NKF);
      __syncthreads();
      if (XPF && g + 1 < NG) gq.issue(W.qkv, KD, (g + 1) * (HP * 3 * DH / 16) + wave, 0, lane, NW);
      if (!XPF) go.issue(W.o, KD, wave * MBH, g * HP * KH, lane);
      go.run(qbuf, QTS, h, lane);                        // one product over the heads of the group
    }
    add_bias_h(W.o_b, layer, 0);
    // ================= cross-attention block (observation tokens) =================
    if constexpr (CM == 1) {
      // HPX heads per phase; the queries of a phase are one token-major LDS matrix [NT][HPX*DH], so the output
      // projection contracts all its heads in one product.  Keys / values come from global memory in fragment
      // order; the keys of a wave's next task are requested once the scores of the current one are formed, its
      // values once the current values are consumed (one buffer each: double buffers would spill).
      constexpr int HPX = C::HPX, NGX = HEADS / HPX, QXS = HPX * DH + TT::PAD;
      constexpr int NTASK = RPT * HPX * NKF, TPW = (NTASK + NW - 1) / NW;
      typedef FragGemm<TT, MBH, NB, HPX * KH, BD> GOX;
      GC gc;
      if (XPF) gc.issue(W.cq, KD, wave * MBC, 0, lane);
      write_ln(layer, -1);                               // its barriers order the O-projection reads before qbuf writes
      for (int g = 0; g < NGX; ++g) {
        FENCE_LANE_IDS();
        GOX go;
        bf16x8 ka[KHc][SFc];
        bf16x4 va[DH / 16][SFc];
        // Task i of a wave -> (row, head of the phase, query fragment).  When the heads of a phase divide evenly over
        // the waves, a wave takes whole heads: the tasks of one head (its rows and query fragments) share the keys /
        // values as long as their rows belong to the same environment, so they are fetched once, not once per task.
        constexpr bool HEADMAJOR = HPX % NW == 0;
        constexpr int TPH = RPT * NKF;                  // tasks per head
        auto task_of = [&](int i) { return HEADMAJOR ? ((wave + (i / TPH) * NW) * TPH + i % TPH) : wave + i * NW; };
        auto task_row = [&](int task) { return (task / NKF) % RPT; };
        auto task_head = [&](int task) { return task / (NKF * RPT); };
        // does task i need operands other than those of task i-1?
        auto task_reload = [&](int i) {
          if (!HEADMAJOR || i % TPH == 0) return true;
          if (i % NKF != 0) return false;               // same row, next query fragment
          return env_of_row[task_row(task_of(i))] != env_of_row[task_row(task_of(i - 1))];
        };
        {
          f32x4 acc[MBC][NB];
          f32x4 bias[MBC];
#pragma unroll
          for (int mb = 0; mb < MBC; ++mb) {
            bias[mb] = *reinterpret_cast<const f32x4*>(W.cq_b + g * (HPX * DH) + (wave * MBC + mb) * 16 + lg * 4);
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) acc[mb][nb] = f32x4{0, 0, 0, 0};
          }
          if (!XPF) gc.issue(W.cq, KD, g * (HPX * DH / 16) + wave * MBC, 0, lane);
          gc.run(act, AS, acc, lane);
          if (XPF) go.issue(W.co, KD, wave * MBH, g * HPX * KH, lane);
          if (g > 0) __syncthreads();
#pragma unroll
          for (int mb = 0; mb < MBC; ++mb) {
            const int c0 = (wave * MBC + mb) * 16 + lg * 4;      // column = head-of-phase * DH + feature
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
              *reinterpret_cast<vec4*>(qbuf + (nb * 16 + l16) * QXS + c0) = TT::cvt(acc[mb][nb] + bias[mb]);
          }
        }
        // the first task's keys / values travel while the barrier is reached (requested only now: with the
        // projection's accumulators still live they would not fit in registers)
        __builtin_amdgcn_sched_barrier(0);
        if (task_of(0) < NTASK) {
          cross_load_k(task_row(task_of(0)), layer, g * HPX + task_head(task_of(0)), ka);
          cross_load_v(task_row(task_of(0)), layer, g * HPX + task_head(task_of(0)), va);
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < TPW; ++i) {
          const int task = task_of(i), nxt = task_of(i + 1);
          const bool more = i + 1 < TPW && nxt < NTASK && task_reload(i + 1);
          if (task < NTASK) {
            __bf16* qp = reinterpret_cast<__bf16*>(qbuf) + (task_row(task) * H + (task % NKF) * 16) * QXS + task_head(task) * DH;
            bf16x4 p[SFc];
            // scheduling fences: the requests must not be moved ahead of the products that free their registers
            cross_scores(qp, QXS, ka, p);
            __builtin_amdgcn_sched_barrier(0);
            if (more) cross_load_k(task_row(nxt), layer, g * HPX + task_head(nxt), ka);
            __builtin_amdgcn_sched_barrier(0);
            cross_pv(qp, QXS, p, va);
            __builtin_amdgcn_sched_barrier(0);
            if (more) cross_load_v(task_row(nxt), layer, g * HPX + task_head(nxt), va);
            __builtin_amdgcn_sched_barrier(0);
          }
        }
        __syncthreads();
        if (XPF && g + 1 < NGX) gc.issue(W.cq, KD, (g + 1) * (HPX * DH / 16) + wave * MBC, 0, lane);
        if (!XPF) go.issue(W.co, KD, wave * MBH, g * HPX * KH, lane);
        go.run(qbuf, QXS, h, lane);
      }
      add_bias_h(W.co_b, layer, 1);
    }
    // ================= MLP block =================
    if constexpr (C::UDB && !XPF && (NC % 2 == 0)) {
      // Two hidden-chunk buffers: the GELU epilogue of chunk c is vector work that runs in the issue slots the
      // matrix pipeline leaves free.  Its first half is spread over the k-steps of the down-projection of chunk
      // c-1, its second half over those of the up-projection of chunk c+1 (all of it in one product would need
      // more vector slots than that product leaves); one barrier per chunk.
      write_ln(layer, 2);
      f32x4 accA[MBU][NB], accB[MBU][NB];
      constexpr int PARTS = MBU * NB;
      constexpr int HALF = PARTS / 2;                         // parts done under the previous down-projection
      GU gu;
      GD gd;
      constexpr bool PRIME = KD >= GD::PF && KC >= GU::PF;
      typedef std::integral_constant<int, GU::PF> UFULL;
      typedef std::integral_constant<int, GD::PF> DFULL;
      typedef std::integral_constant<int, 1> ONE;
      auto zero = [&](f32x4 (&acc)[MBU][NB]) {
#pragma unroll
        for (int mb = 0; mb < MBU; ++mb)
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) acc[mb][nb] = f32x4{0, 0, 0, 0};
      };
      // GELU(acc + bias) of accumulator part idx of chunk c -> hidden buffer c & 1
      auto gelu_part = [&](int c, const f32x4 (&acc)[MBU][NB], int idx) {
        const int mb = idx / NB, nb = idx % NB;
        const int f0 = (wave * MBU + mb) * 16 + lg * 4;
        f32x4 v = acc[mb][nb] + *reinterpret_cast<const f32x4*>(upb + c * CH + f0);
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = gelu_fast(v[i]);
        *reinterpret_cast<vec4*>(ubuf + (c & 1) * NT * US + (nb * 16 + l16) * US + f0) = TT::cvt(v);
      };
      // chunk c: accumulator `cur` holds its pre-activations, parts [0, HALF) of its GELU are already in the hidden
      // buffer; `nxt` receives the pre-activations of chunk c+1.  UPRIMED: the weights of that up-projection were
      // requested in the tail of the previous down-projection.  Each product requests the first weights of the one
      // after it in its own tail (the down-projection those of the up-projection of chunk c+2; past the last chunk
      // it re-requests the last chunk's, which are simply not used).
      auto chunk = [&](int c, f32x4 (&cur)[MBU][NB], f32x4 (&nxt)[MBU][NB], auto HASNEXT, auto UPRIMED) {
        constexpr bool NEXT = decltype(HASNEXT)::value, UP = decltype(UPRIMED)::value && PRIME;
        FENCE_LANE_IDS();
        if (PRIME) gd.prime_begin(W.dn, KM, wave * MBH, c * (KC), lane);
        if constexpr (NEXT) {
          zero(nxt);
          if (!UP) gu.issue(W.up, KD, (c + 1) * (CH / 16) + wave * MBU, 0, lane);
          auto side = [&](int k) {
#pragma unroll
            for (int idx = HALF + k * (PARTS - HALF) / KD; idx < HALF + (k + 1) * (PARTS - HALF) / KD; ++idx)
              gelu_part(c, cur, idx);
            if (PRIME) gd.template prime_in_tail<KD>(k);
          };
          if constexpr (UP) gu.run(act, AS, nxt, lane, side, UFULL{});
          else gu.run(act, AS, nxt, lane, side, ONE{});
        } else {
          if (PRIME) {
#pragma unroll
            for (int p = 0; p < GD::PF; ++p) gd.prime_stage(p);
          }
#pragma unroll
          for (int idx = HALF; idx < PARTS; ++idx) gelu_part(c, cur, idx);
        }
        __syncthreads();
        if (!PRIME) gd.issue(W.dn, KM, wave * MBH, c * (KC), lane);
        if constexpr (NEXT) {
          const int c2 = c + 2 < NC ? c + 2 : NC - 1;
          if (PRIME) gu.prime_begin(W.up, KD, c2 * (CH / 16) + wave * MBU, 0, lane);
          // the buffer of chunk c+1 was last read by the down-projection of chunk c-1: every wave is past it
          auto side = [&](int k) {
#pragma unroll
            for (int idx = k * HALF / KC; idx < (k + 1) * HALF / KC; ++idx) gelu_part(c + 1, nxt, idx);
            if (PRIME) gu.template prime_in_tail<KC>(k);
          };
          if constexpr (PRIME) gd.run(ubuf + (c & 1) * NT * US, US, h, lane, side, DFULL{});
          else gd.run(ubuf + (c & 1) * NT * US, US, h, lane, side, ONE{});
        } else {
          if constexpr (PRIME) gd.run(ubuf + (c & 1) * NT * US, US, h, lane, typename GD::NoSide{}, DFULL{});
          else gd.run(ubuf + (c & 1) * NT * US, US, h, lane);
        }
      };
      zero(accA);
      gu.issue(W.up, KD, wave * MBU, 0, lane);
      gu.run(act, AS, accA, lane);
#pragma unroll
      for (int idx = 0; idx < HALF; ++idx) gelu_part(0, accA, idx);
      // one loop body: the pre-activations of the next chunk move into the registers of the current one
      auto rotate = [&]() {
#pragma unroll
        for (int mb = 0; mb < MBU; ++mb)
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) accA[mb][nb] = accB[mb][nb];
      };
      chunk(0, accA, accB, std::true_type{}, std::false_type{});
      rotate();
      for (int c = 1; c + 1 < NC; ++c) {
        chunk(c, accA, accB, std::true_type{}, std::true_type{});
        rotate();
      }
      chunk(NC - 1, accA, accB, std::false_type{}, std::false_type{});
    } else {
    GU gu;
    if (XPF) gu.issue(W.up, KD, wave * MBU, 0, lane);
    write_ln(layer, 2);                                  // its barriers also order the projection reads before ubuf writes
    for (int c = 0; c < NC; ++c) {
      FENCE_LANE_IDS();
      GD gd;
      {
        f32x4 acc[MBU][NB];
        f32x4 bias[MBU];
#pragma unroll
        for (int mb = 0; mb < MBU; ++mb) {
          bias[mb] = *reinterpret_cast<const f32x4*>(W.up_b + c * CH + (wave * MBU + mb) * 16 + lg * 4);
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) acc[mb][nb] = f32x4{0, 0, 0, 0};
        }
        if (!XPF) gu.issue(W.up, KD, c * (CH / 16) + wave * MBU, 0, lane);
        gu.run(act, AS, acc, lane);
        if (XPF) gd.issue(W.dn, KM, wave * MBH, c * (KC), lane);
        // single buffer: the previous chunk's down-projection has read ubuf; double buffer: the buffer written
        // now was last read two chunks ago, and every wave has passed a barrier since
        if (c > 0 && !C::UDB) __syncthreads();
        elem* ub = ubuf + (C::UDB ? (c & 1) * NT * US : 0);
#pragma unroll
        for (int mb = 0; mb < MBU; ++mb) {
          const int f0 = (wave * MBU + mb) * 16 + lg * 4;
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) {
            f32x4 v = acc[mb][nb] + bias[mb];
#pragma unroll
            for (int i = 0; i < 4; ++i) v[i] = gelu_fast(v[i]);
            *reinterpret_cast<vec4*>(ub + (nb * 16 + l16) * US + f0) = TT::cvt(v);
          }
        }
      }
      __syncthreads();
      if (XPF) {
        if (c + 1 < NC) gu.issue(W.up, KD, (c + 1) * (CH / 16) + wave * MBU, 0, lane);
        else if (layer + 1 < net.L) gq.issue(net.layer[layer + 1].qkv, KD, wave, 0, lane, NW);
      } else {
        gd.issue(W.dn, KM, wave * MBH, c * (KC), lane);
      }
      gd.run(ubuf + (C::UDB ? (c & 1) * NT * US : 0), US, h, lane);
    }
    }
    add_bias_h(W.dn_b, layer, 2);
  }

  // ---- output head: eps = head_w LN(h) + head_b ---------------------------------------------------------
  write_ln(0, -1);
  {
    constexpr int NBW = (NB + NW - 1) / NW;             // token fragments per wave
    const int nb0 = wave * NBW;
    if (nb0 < NB) {
      // the head's A output rows are packed as ceil(A/16) fragment rows (zero rows pad the last one)
      for (int hf = 0; hf * 16 < A; ++hf) {
        f32x4 e[1][NBW];
#pragma unroll
        for (int j = 0; j < NBW; ++j) e[0][j] = f32x4{0, 0, 0, 0};
        FragGemm<TT, 1, NBW, KD> gh;
        gh.issue(net.head, KD, hf, 0, lane);
        gh.run(act + nb0 * 16 * AS, AS, e, lane);
#pragma unroll
        for (int j = 0; j < NBW; ++j) {
          const int t = (nb0 + j) * 16 + l16;
          if (nb0 + j < NB && t < ntok_live) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const int a = hf * 16 + lg * 4 + i;
              if (a < A) eo[t * A + a] = e[0][j][i] + net.head_b[a];
            }
          }
        }
      }
    }
  }
}

// Batched verification: tile b of the grid takes rows b*RPT .. of the ragged batch.
template <class C>
__global__ __launch_bounds__(C::THREADS, C::WG_PER_CU) void k_fused_forward(FusedNet net, FusedIO io, int A) {
  constexpr int D = C::D, NT = C::NT, H = C::H;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  __shared__ int32_t envs[C::RPT];
  __shared__ const float* mrow[C::RPT];
  const int R = io.d_R ? min(*io.d_R, io.R_cap) : io.R_cap;
  const int row0 = blockIdx.x * C::RPT;
  if (row0 >= R) return;
  const long long tok0 = (long long)row0 * H;
  const int ntok_live = min(NT, (R - row0) * H);
  float* xt = reinterpret_cast<float*>(lds + C::ACT_B);
  for (int i = threadIdx.x; i < NT * A; i += C::THREADS) xt[i] = i < ntok_live * A ? io.x_rows[tok0 * A + i] : 0.0f;
  if (threadIdx.x < C::RPT) {
    const int r = min(row0 + (int)threadIdx.x, R - 1);
    envs[threadIdx.x] = io.row_env ? io.row_env[r] : r;
    const int mod_stride = net.L * 4 * D;
    if (net.modtab) {
      int t = io.row_t[r] - io.t_sub;
      t = t < 0 ? 0 : (t >= io.T ? io.T - 1 : t);
      mrow[threadIdx.x] = net.modtab + (size_t)t * mod_stride;
    } else {
      mrow[threadIdx.x] = io.mod + (size_t)r * mod_stride;
    }
  }
  __syncthreads();
  fused_body<C>(net, lds, xt, A, mrow, envs, io.eps_out + tok0 * A, ntok_live);
}

// Drafter rollout: the workgroup keeps the latents of RPT environments in LDS and runs their drafted
// transitions k = 1 .. max K_eff back to back; every step is one forward pass plus the DDPM step
//   y <- mu_p(y, eps, t_k) + s sigma_{t_k} xi_{env,t_k},   t_k = t0 - k + 1,
// and stores the input state, the drafter output and the noise of the transition in its ragged row.
template <class C>
__global__ __launch_bounds__(C::THREADS) void k_fused_draft(FusedNet net, DraftIO io, int A) {
  typedef typename C::TT TT;
  typedef typename TT::elem elem;
  constexpr int D = C::D, NT = C::NT, H = C::H, TH = C::THREADS, SGS = D + TT::PAD;
  constexpr int RPT = C::RPT;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  __shared__ int32_t envs[RPT], s_t0[RPT], s_keff[RPT], s_rowp[RPT], s_kmax;
  __shared__ const float* mrow[RPT];
  const int DE = H * A;                                 // elements of one latent
  const int mod_stride = net.L * 4 * D;
  float* yt = reinterpret_cast<float*>(lds + C::LDS_B);              // [NT*A] latents
  float* et = yt + NT * A;                                           // [NT*A] drafter output
  // The FiLM product has 16 columns (one MFMA tile): column j = environment j / SPE, step offset j % SPE.  With
  // mod_cols = 16 it yields the vectors of SPE = 16 / RPT consecutive steps at once, so the FiLM weights stream once
  // per SPE steps; with mod_cols = RPT (when LDS is short) one step at a time.
  const int mod_cols = io.mod_cols, SPE = mod_cols / RPT;
  float* modbuf = et + NT * A;                                       // [mod_cols][L*4D] FiLM vectors
  elem* sgbuf = reinterpret_cast<elem*>(modbuf + mod_cols * mod_stride);   // [16][D+pad] SiLU(g), unused rows zero
  // [L][3][D] residual biases (self-attention output, cross-attention output, MLP down) of all layers: they are added
  // right after a product, where a global load has nothing to overlap it, K times per rollout
  float* dbias = reinterpret_cast<float*>(sgbuf + 16 * SGS);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, l16 = lane & 15, lg = lane >> 4;
  const int env0 = blockIdx.x * RPT;
  if (io.gate && *io.gate == 0) return;
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
  for (int i = threadIdx.x; i < 16 * SGS; i += TH) sgbuf[i] = (elem)0.0f;
  for (int i = threadIdx.x; i < net.L * 3 * D; i += TH) {
    const int l = i / (3 * D), which = (i / D) % 3, c = i % D;
    const float* src = which == 0 ? net.layer[l].o_b : (which == 1 ? net.layer[l].co_b : net.layer[l].dn_b);
    dbias[i] = src ? src[c] : 0.0f;
  }
  for (int i = threadIdx.x; i < NT * A; i += TH) {
    const int b = env0 + i / DE;
    yt[i] = b < io.B ? io.y[(size_t)env0 * DE + i] : 0.0f;
  }
  __syncthreads();
  const int kmax = s_kmax;
  for (int k = 1; k <= kmax; ++k) {
    if (net.modtab) {                                   // FiLM vectors of timestep t_k straight from the table
      if (threadIdx.x < RPT) {
        int t = s_t0[threadIdx.x] - k + 1;
        t = t < 0 ? 0 : t;
        mrow[threadIdx.x] = net.modtab + (size_t)t * mod_stride;
      }
    } else {
    const int so = (k - 1) % SPE;                       // offset of this step in the current batch of SPE steps
    if (threadIdx.x < RPT) mrow[threadIdx.x] = modbuf + (threadIdx.x * SPE + so) * mod_stride;
    if (so == 0) {
    // FiLM inputs of steps k .. k+SPE-1: SiLU(temb[t] + cemb[env]) as rows of the mod product's B operand
    for (int i = threadIdx.x; i < mod_cols * D; i += TH) {
      const int j = i / D, c = i % D, r = j / SPE;
      int t = s_t0[r] - (k + j % SPE) + 1;
      t = t < 0 ? 0 : t;
      float g = net.temb[(size_t)t * D + c];
      if (net.cemb) g += net.cemb[(size_t)envs[r] * D + c];
      sgbuf[j * SGS + c] = (elem)silu_fast(g);
    }
    __syncthreads();
    {
      constexpr int MBM = 2;
      const int fpw = net.L * 4 * D / (16 * C::NW);     // mod fragments per wave
      for (int f = 0; f < fpw; f += MBM) {
        f32x4 acc[MBM][1];
#pragma unroll
        for (int mb = 0; mb < MBM; ++mb) acc[mb][0] = f32x4{0, 0, 0, 0};
        FragGemm<TT, MBM, 1, D / TT::KSTEP> gm;
        gm.issue(net.modw, D / TT::KSTEP, wave * fpw + f, 0, lane);
        gm.run(sgbuf, SGS, acc, lane);
        if (l16 < mod_cols) {
#pragma unroll
          for (int mb = 0; mb < MBM; ++mb) {
            const int f0 = (wave * fpw + f + mb) * 16 + lg * 4;
            const f32x4 b = *reinterpret_cast<const f32x4*>(net.modb + f0);
            *reinterpret_cast<f32x4*>(modbuf + l16 * mod_stride + f0) = acc[mb][0] + b;
          }
        }
      }
    }
    }
    }
    __syncthreads();
    fused_body<DraftCfg<C>>(net, lds, yt, A, mrow, envs, et, NT, dbias);
    __syncthreads();
    // DDPM step of transition k for the environments that still draft
    const int nblk = DE >> 2;
    for (int i = threadIdx.x; i < RPT * nblk; i += TH) {
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
      const float sa = io.tb.sqrt_abar[t], s1 = io.tb.sqrt_1m[t], c0 = io.tb.c0[t], cx = io.tb.cx[t], ce = io.tb.ce[t];
      const float sig = io.sigma_scale[b] * io.tb.sigma[t];
      f32x4 o;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        float x0 = (yv[j] - s1 * ev[j]) / sa;
        if (io.clip) x0 = fminf(fmaxf(x0, -io.clip_val), io.clip_val);
        o[j] = c0 * x0 + cx * yv[j] + ce * ev[j] + sig * z[j];
      }
      *reinterpret_cast<f32x4*>(io.states + row * DE + 4 * blk) = yv;
      *reinterpret_cast<f32x4*>(io.eps_p + row * DE + 4 * blk) = ev;
      if (io.xi) *reinterpret_cast<f32x4*>(io.xi + row * DE + 4 * blk) = z;
      *reinterpret_cast<f32x4*>(yp) = o;
    }
    __syncthreads();
  }
  for (int i = threadIdx.x; i < NT * A; i += TH) {
    const int b = env0 + i / DE;
    if (b < io.B) io.y[(size_t)env0 * DE + i] = yt[i];
  }
}

// FiLM vectors of a ragged batch with the matrix cores: mod[r, :] = W_mod SiLU(temb[t_r] + cemb[env_r]) + b_mod
// for all layers at once.  Tile: NR rows x 256 outputs per workgroup pass; the SiLU input rows are built in LDS as
// bf16 and the weights stream as fragments (FusedNet::modw).  NR = 64 keeps the tile under a third of the LDS at
// d <= 384, so three workgroups share a CU (the kernel is bound by its output stream, R x L*4D fp32).
template <int D, int NR>
__global__ __launch_bounds__(256) void k_mod_gemm(const void* __restrict__ modw, const float* __restrict__ modb,
                                                  const float* __restrict__ temb, const float* __restrict__ cemb,
                                                  const int32_t* __restrict__ t_arr, int t_sub,
                                                  const int32_t* __restrict__ env_arr, int T, int Nm,
                                                  const int32_t* d_R, int R_cap, float* __restrict__ mod) {
  constexpr int NB = NR / 16, MB = 4, AS = D + 8;
  __shared__ __attribute__((aligned(16))) __bf16 sg[NR * AS];
  const int R = d_R ? min(*d_R, R_cap) : R_cap;
  const int row0 = blockIdx.y * NR;
  if (row0 >= R) return;
  int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  // the SiLU rows: batches of independent gathers (row indices first, then the two embedding vectors of every slot of
  // the batch), so that a batch costs two memory round trips instead of two per slot
  constexpr int SLOTS = NR * (D / 4), BATCH = 8;
  for (int i0 = threadIdx.x; i0 < SLOTS; i0 += 256 * BATCH) {
    int tt[BATCH], ee[BATCH];
#pragma unroll
    for (int j = 0; j < BATCH; ++j) {
      const int i = min(i0 + 256 * j, SLOTS - 1);
      const int row = min(row0 + i / (D / 4), R - 1);
      tt[j] = t_arr[row] - t_sub;
      ee[j] = cemb ? (env_arr ? env_arr[row] : row) : 0;
    }
    f32x4 g[BATCH];
#pragma unroll
    for (int j = 0; j < BATCH; ++j) {
      const int i = min(i0 + 256 * j, SLOTS - 1);
      const int c = (i % (D / 4)) * 4;
      const int t = tt[j] < 0 ? 0 : (tt[j] >= T ? T - 1 : tt[j]);
      g[j] = *reinterpret_cast<const f32x4*>(temb + (size_t)t * D + c);
      if (cemb) g[j] += *reinterpret_cast<const f32x4*>(cemb + (size_t)ee[j] * D + c);
    }
#pragma unroll
    for (int j = 0; j < BATCH; ++j) {
      const int i = i0 + 256 * j;
      if (i < SLOTS) {
        f32x4 v = g[j];
#pragma unroll
        for (int q = 0; q < 4; ++q) v[q] = silu_fast(v[q]);
        *reinterpret_cast<bf16x4*>(sg + (i / (D / 4)) * AS + (i % (D / 4)) * 4) = TBF16::cvt(v);
      }
    }
  }
  __syncthreads();
  const int l16 = lane & 15, lg = lane >> 4;
  // output tiles of 256 features (16 fragment rows) are dealt to blockIdx.x round-robin
  for (int ft = blockIdx.x; ft * 256 < Nm; ft += gridDim.x) {
    const int mf0 = ft * 16 + wave * MB;
    f32x4 acc[MB][NB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) acc[mb][nb] = f32x4{0, 0, 0, 0};
    FragGemm<TBF16, MB, NB, D / 32> gm;
    gm.issue(modw, D / 32, mf0, 0, lane);
    gm.run(sg, AS, acc, lane);
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      const int f0 = (mf0 + mb) * 16 + lg * 4;
      const f32x4 b = *reinterpret_cast<const f32x4*>(modb + f0);
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        const int row = row0 + nb * 16 + l16;
        if (row < R) *reinterpret_cast<f32x4*>(mod + (size_t)row * Nm + f0) = acc[mb][nb] + b;
      }
    }
    asm volatile("" : "+v"(lane));
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
