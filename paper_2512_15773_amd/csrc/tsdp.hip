// C ABI of the speculative denoising round: context, weights, tables, workspace and launch sequences.
// Definitions of the operations: Section 3.1 (acceptance test, first rejection, reflection coupling)
// and Section 3.2 (drafter rollout, batched verification, log acceptance ratio) of the TS-DP paper.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

#include "../../include/tsdp.h"
#include "kernels_f32.hpp"
#include "fused_mfma.hpp"
#include "round_kernels.hpp"

using namespace tsdp;

namespace {

struct LayerOff {
  size_t mod_w, mod_b, qkv_w, qkv_b, o_w, o_b, cq_w, cq_b, ck_w, ck_b, cv_w, cv_b, co_w, co_b, up_w, up_b, dn_w, dn_b;
};

struct Net {
  int L = 0, d = 0, heads = 0, m = 0;
  size_t n_floats = 0;
  size_t tok_w, tok_b, pos, t_w1, t_b1, t_w2, t_b2, c_w, c_b, head_w, head_b;
  std::vector<LayerOff> lay;
  float* blob = nullptr;        // device copy of the (rounded) canonical blob
  float* temb = nullptr;        // [T, d] timestep embedding of every timestep
  float* modtab = nullptr;      // [T, L*4d] FiLM vectors of every timestep (token conditioning, fused bf16 path)
  int32_t* t_iota = nullptr;    // [T] 0..T-1, the row timesteps of the table build
  float* modw = nullptr;        // [L*4d, d] FiLM projections of all layers, concatenated
  float* modb = nullptr;        // [L*4d]
  float* cemb = nullptr;        // [B_max, d] conditioning embedding (mode 0)
  float* kc = nullptr;          // [L, B_max*S, d] cross-attention keys (mode 1)
  float* vc = nullptr;          // [L, B_max*S, d] cross-attention values (mode 1)
  bool loaded = false;
  const char* path = "f32-ops";
  // fused bf16 MFMA path (bf16 networks of supported shape)
  bool fused = false;
  FusedNet fnet;
  hipError_t (*fused_verify)(const FusedNet&, const FusedIO&, int A, int R_cap, hipStream_t) = nullptr;
  hipError_t (*fused_verify_few)(const FusedNet&, const FusedIO&, int A, int R_cap, hipStream_t) = nullptr;
  int verify_rpt = 1;
  void (*fused_mod)(const FusedNet&, const int32_t*, int, const int32_t*, int, const int32_t*, int, float*, hipStream_t) = nullptr;
  hipError_t (*fused_draft_small)(const FusedNet&, const DraftIO&, int A, hipStream_t) = nullptr;   // few environments per workgroup
  hipError_t (*fused_draft_big)(const FusedNet&, const DraftIO&, int A, hipStream_t) = nullptr;     // many environments per workgroup
  int draft_rpt_small = 0, draft_rpt_big = 0;
  uint16_t* kc_pk = nullptr;    // fragment-ordered bf16 keys / transposed values of every (env, layer, head)
  uint16_t* vct_pk = nullptr;
};

}  // namespace

// Scratch of tsdp_distill_loss_noalloc: the per-workgroup partial sums of the loss (one pair of doubles per 16
// rows) live in a file-scope device array instead of context memory, so that entry point allocates nothing.  Every
// GPU holds its own copy; host code uses the address hipGetSymbolAddress returns for the current device, looked up
// once per device in tsdp_create, never the symbol itself.
constexpr int NOALLOC_MAX_ROWS = 65536;
constexpr int NOALLOC_MAX_DEVICES = 64;
static __device__ __align__(256) double scratch[2 * (NOALLOC_MAX_ROWS / 16) + 2];
static double* g_scratch_ptr[NOALLOC_MAX_DEVICES];   // device address of `scratch` on each device, null until looked up

struct tsdp_ctx {
  tsdp_config cfg;
  int device = -1;              // the device that was current in tsdp_create
  int D = 0;
  std::string err;
  float* tables = nullptr;      // 6 x T fp32: sqrt_abar, sqrt_1m, c0, cx, sigma, ce
  SchedTables tb;
  Net net[2];
  bool cond_set = false;
  int cond_B = 0;
  int32_t* status = nullptr;
  int32_t* live = nullptr;      // environments still running (chain driver)
  int32_t* K_sel = nullptr;     // [B_max] per-round picks from the stage tables (staged chain driver)
  float* s_sel = nullptr;
  float* lam_sel = nullptr;
  double* loss_partial = nullptr;   // per-workgroup partial sums of the distillation loss
  int32_t* K_eff = nullptr;     // [B_max]
  int32_t* n_draft = nullptr;   // [0] B while some environment has rows in the current plan, [1] B while one drafts; else 0
  // network workspace (lazy)
  bool ws_ready = false;
  float *h = nullptr, *a = nullptr, *qkv = nullptr, *ao = nullptr, *u = nullptr, *sg = nullptr, *mod = nullptr;
  float* eps_tmp = nullptr;     // [B_max, D] drafter output of the current step
  int32_t *row_t_chk = nullptr, *row_env_chk = nullptr;   // [rows] range-checked copy of a caller's row table (tsdp_verify)
  int32_t* Bconst = nullptr;    // device ints holding B for row-count reads of dense (per-env) launches
  // round-owned ragged buffers (lazy)
  bool rb_ready = false;
  int32_t *row_ptr = nullptr, *row_t = nullptr, *row_env = nullptr, *t_next = nullptr, *n_acc = nullptr, *n_adv = nullptr;
  float *states = nullptr, *eps_p = nullptr, *eps_q = nullptr, *xi = nullptr, *y_last = nullptr;
  std::vector<void*> owned;
  // A round computes the base network's per-row FiLM vectors (k_mod_gemm, bound by its output stream) on a second
  // stream of the same priority while the drafter rolls out: forked after the row table, joined before the verify.
  hipStream_t aux = nullptr;
  hipEvent_t ev_fork = nullptr, ev_join = nullptr;
  // optional kernel timing: events recorded around the dominant kernel of each stage
  bool timing = false;
  int timing_mask = 15;         // stages whose kernels are bracketed by events while timing is on (bit = stage)
  hipEvent_t ev[4][2] = {{nullptr, nullptr}, {nullptr, nullptr}, {nullptr, nullptr}, {nullptr, nullptr}};   // draft, verify, accept, FiLM GEMM
  bool ev_used[4] = {false, false, false, false};
};

namespace {

int fail(tsdp_ctx* c, int code, const std::string& msg) {
  if (c) c->err = msg;
  return code;
}

inline void tick(tsdp_ctx* c, int stage, int edge, hipStream_t s) {
  if (c->timing && ((c->timing_mask >> stage) & 1)) {
    (void)hipEventRecord(c->ev[stage][edge], s);
    c->ev_used[stage] = true;
  }
}

#define HIPCHK(c, expr)                                                                         \
  do {                                                                                          \
    hipError_t e_ = (expr);                                                                     \
    if (e_ != hipSuccess)                                                                       \
      return fail(c, e_ == hipErrorOutOfMemory ? TSDP_E_NOMEM : TSDP_E_HIP,                     \
                  std::string(#expr) + ": " + hipGetErrorString(e_));                           \
  } while (0)

template <typename T>
int dev_alloc(tsdp_ctx* c, T** p, size_t count) {
  void* v = nullptr;
  HIPCHK(c, hipMalloc(&v, (count ? count : 1) * sizeof(T)));
  c->owned.push_back(v);
  *p = static_cast<T*>(v);
  return TSDP_OK;
}

float bf16_round(float f) {
  uint32_t b;
  std::memcpy(&b, &f, 4);
  if ((b & 0x7F800000u) == 0x7F800000u) return f;     // inf / nan unchanged
  b = (b + 0x7FFFu + ((b >> 16) & 1u)) & 0xFFFF0000u;
  std::memcpy(&f, &b, 4);
  return f;
}


uint16_t bf16_bits(float f) {
  uint32_t b;
  std::memcpy(&b, &f, 4);
  b = (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
  return (uint16_t)b;
}

// Fragment order of a logical [rows, K] matrix as MFMA A operands: [rows/16][Kpad/KSTEP][64 lanes][VW elements];
// lane l of fragment (mf, ks) holds row mf*16 + l%16, columns ks*KSTEP + (l/16)*VW .. +VW-1, with VW = 8 bf16
// (k-step 32) or VW = 4 fp32 (k-step 16).  src_row(lr) maps a logical row to a row of W (or -1 for a zero row).
// Offsets returned by the callers are in bytes of `out`.
template <typename RowMap>
void pack_frags(std::vector<uint8_t>& out, bool f32, const float* W, int K, int rows, RowMap src_row) {
  const int VW = f32 ? 4 : 8, KSTEP = 4 * VW, ES = f32 ? 4 : 2;
  const int mfs = (rows + 15) / 16, kss = (K + KSTEP - 1) / KSTEP;
  const size_t base = out.size();
  out.resize(base + (size_t)mfs * kss * 64 * VW * ES, 0);
  for (int mf = 0; mf < mfs; ++mf)
    for (int ks = 0; ks < kss; ++ks)
      for (int l = 0; l < 64; ++l) {
        const int lr = mf * 16 + (l & 15);
        const int sr = lr < rows ? src_row(lr) : -1;
        for (int i = 0; i < VW; ++i) {
          const int col = ks * KSTEP + (l >> 4) * VW + i;
          if (sr < 0 || col >= K) continue;
          const float v = W[(size_t)sr * K + col];
          uint8_t* dst = &out[base + ((((size_t)mf * kss + ks) * 64 + l) * VW + i) * ES];
          if (f32) {
            std::memcpy(dst, &v, 4);
          } else {
            const uint16_t b = bf16_bits(v);
            std::memcpy(dst, &b, 2);
          }
        }
      }
}

template <class C>
hipError_t launch_verify(const FusedNet& n, const FusedIO& io, int A, int R_cap, hipStream_t s) {
  auto kern = k_fused_forward<C>;
  static bool attr_set = false;
  if (!attr_set) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_B);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int tiles = (R_cap + C::RPT - 1) / C::RPT;
  if (tiles > 0) hipLaunchKernelGGL(kern, dim3(tiles), dim3(C::THREADS), C::LDS_B, s, n, io, A);
  return hipSuccess;
}

template <class C>
hipError_t launch_draft(const FusedNet& n, const DraftIO& io_in, int A, hipStream_t s) {
  auto kern = k_fused_draft<C>;
  DraftIO io = io_in;
  // FiLM vectors of up to 16 / RPT steps per in-kernel product, as many as LDS has room for
  const int fixed = C::LDS_B + 2 * C::NT * A * 4 + 16 * (C::D + C::TT::PAD) * C::ES + n.L * 3 * C::D * 4;
  const int per_col = n.L * 4 * C::D * 4;
  io.mod_cols = C::RPT;
  for (int cols = 16; cols > C::RPT; cols /= 2)
    if (cols % C::RPT == 0 && fixed + cols * per_col <= 160 * 1024) { io.mod_cols = cols; break; }
  const int lds = fixed + io.mod_cols * per_col;
  static int attr_lds = 0;
  if (lds > attr_lds) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    attr_lds = lds;
  }
  const int tiles = (io.B + C::RPT - 1) / C::RPT;
  if (tiles > 0) hipLaunchKernelGGL(kern, dim3(tiles), dim3(C::THREADS), lds, s, n, io, A);
  return hipSuccess;
}

template <int D>
void launch_mod(const FusedNet& n, const int32_t* t_arr, int t_sub, const int32_t* env_arr, int T, const int32_t* d_R,
                int R_cap, float* mod, hipStream_t s) {
  const int Nm = n.L * 4 * D;                           // a multiple of 256 because D is a multiple of 64
  constexpr int NR = 64;                                // rows per workgroup
  const int row_tiles = (R_cap + NR - 1) / NR;
  // output tiles of 256 features are dealt over blockIdx.x; enough workgroups for about twelve per CU at the row bound
  // (a ragged batch leaves the tiles beyond its live rows empty)
  const int fx = std::max(1, std::min(Nm / 256, (3072 + row_tiles - 1) / row_tiles));
  dim3 g(fx, row_tiles);
  hipLaunchKernelGGL((k_mod_gemm<D, NR>), g, dim3(256), 0, s, n.modw, n.modb, n.temb, n.cemb, t_arr, t_sub, env_arr, T, Nm, d_R,
                     R_cap, mod);
}

struct FusedKernels {
  // variant for batches of at most one tile per CU: one 8-wave workgroup per CU instead of two 4-wave ones
  hipError_t (*verify_few)(const FusedNet&, const FusedIO&, int, int, hipStream_t) = nullptr;
  int rpt_verify = 0;
  void (*mod)(const FusedNet&, const int32_t*, int, const int32_t*, int, const int32_t*, int, float*, hipStream_t) = nullptr;
  hipError_t (*verify)(const FusedNet&, const FusedIO&, int, int, hipStream_t) = nullptr;
  hipError_t (*draft_small)(const FusedNet&, const DraftIO&, int, hipStream_t) = nullptr;
  hipError_t (*draft_big)(const FusedNet&, const DraftIO&, int, hipStream_t) = nullptr;
  int rpt_small = 0, rpt_big = 0;
};

// Measured tile choices of the compiled shapes.
constexpr int NWS128 = 8;        // waves of the one-environment drafter tile, d = 128
constexpr int NWS256X = 8;       // waves and heads per phase of the one-environment drafter tile, d = 256 with cross-attention
constexpr int HPS256X = 8;
constexpr int F256_NW = 8;       // fp32 d = 256 verify kernel: waves, heads per phase, hidden chunk
constexpr int F256_HP = 2;
constexpr int F256_CH = 256;
constexpr int FEW_TILES = 288;   // up to this many tiles the 8-wave verify variant (one workgroup per CU) is used
constexpr int V512_HPX = 8;      // heads per cross-attention phase of the d = 512 verify kernel
constexpr int V512_CH = 256;     // hidden-chunk width of the d = 512 verify kernel
// shapes with compiled fused kernels
bool find_fused(int dtype, int D, int H, int heads, int cm, int S, int mlp_ratio, int L, FusedKernels& k) {
  if (mlp_ratio != 4 || L > FUSED_MAX_LAYERS) return false;
#define TSDP_SHAPE(TT_, DT_, D_, H_, HD_, CM_, SX_, NTV, CHV, HPV, NWV, HPXV, NTS, CHS, HPS, NWS, NTB, CHB, HPB, NWD)  \
  if (dtype == DT_ && D == D_ && H == H_ && heads == HD_ && cm == CM_ && (CM_ == 0 || S == SX_)) {             \
    k.verify = launch_verify<FusedCfg<TT_, D_, NTV, H_, HD_, CM_, CHV, SX_, HPV, NWV, HPXV>>;                  \
    k.rpt_verify = NTV / H_;                                                                                   \
    k.mod = DT_ == 1 ? launch_mod<D_> : nullptr;                                                               \
    k.draft_small = launch_draft<FusedCfg<TT_, D_, NTS, H_, HD_, CM_, CHS, SX_, HPS, NWS>>; k.rpt_small = NTS / H_; \
    k.draft_big = launch_draft<FusedCfg<TT_, D_, NTB, H_, HD_, CM_, CHB, SX_, HPB, NWD>>;   k.rpt_big = NTB / H_;   \
    return true;                                                                                               \
  }
  // The drafter's small tile (one environment per workgroup) is latency-bound: it takes all heads in one attention
  // phase and the whole MLP hidden layer in one chunk (d = 256 with cross-attention: half of it, 512; 1024 does not
  // fit the LDS), which minimises the number of barrier-separated phases; its four-environment tile at d = 192 takes
  // the hidden layer in two chunks of 384 (measured against 128 / 256: -15 % at d = 256, -3.5 % at d = 192).
  //         type dtype  D   H heads cm  S | verify: NT  CH  HP NW HPX | draft small: NT CH HP NW | big: NT CH HP | NW
  if (dtype == 1 && D == 256 && H == 16 && heads == 4 && cm == 0)
    k.verify_few = launch_verify<FusedCfg<TBF16, 256, 64, 16, 4, 0, 256, 0, 2, 8>>;
  if (dtype == 1 && D == 384 && H == 16 && heads == 6 && cm == 0)
    k.verify_few = launch_verify<FusedCfg<TBF16, 384, 64, 16, 6, 0, 256, 0, 2, 8>>;
  TSDP_SHAPE(TBF16, 1, 256, 16, 4, 0, 0, 64, 128, 1, 4, 1, 16, 128, 1, 4, 64, 128, 1, 4)
  TSDP_SHAPE(TBF16, 1, 384, 16, 6, 0, 0, 64, 192, 1, 4, 1, 16, 128, 1, 4, 64, 128, 1, 4)
  TSDP_SHAPE(TBF16, 1, 128, 16, 4, 0, 0, 128, 128, 2, 4, 2, 16, 512, 4, NWS128, 64, 128, 2, 4)
  TSDP_SHAPE(TBF16, 1, 192, 16, 6, 0, 0, 128, 128, 2, 4, 2, 16, 768, 6, 4, 64, 384, 2, 4)
  TSDP_SHAPE(TBF16, 1, 512, 32, 8, 1, 64, 64, V512_CH, 2, 8, V512_HPX, 32, 128, 1, 4, 64, 128, 1, 4)
  TSDP_SHAPE(TBF16, 1, 256, 32, 8, 1, 64, 64, 256, 2, 4, 2, 32, 512, HPS256X, NWS256X, 64, 128, 2, 4)
  // fp32 networks on the fp32 matrix cores: one row (16 tokens) per workgroup, weights streamed per workgroup
  TSDP_SHAPE(TF32, 0, 256, 16, 4, 0, 0, 16, F256_CH, F256_HP, F256_NW, F256_HP, 16, 128, 1, 4, 16, 128, 1, 4)
  TSDP_SHAPE(TF32, 0, 128, 16, 4, 0, 0, 16, 128, 2, 4, 2, 16, 512, 4, NWS128, 16, 512, 4, 4)
  TSDP_SHAPE(TF32, 0, 64, 16, 2, 0, 0, 16, 64, 2, 4, 2, 16, 64, 2, 4, 16, 64, 2, 4)
  TSDP_SHAPE(TF32, 0, 32, 16, 2, 0, 0, 16, 32, 2, 2, 2, 16, 128, 2, 2, 16, 128, 2, 2)
#undef TSDP_SHAPE
  return false;
}

size_t layout_net(const tsdp_config& cf, int which, Net& n) {
  n.L = which == 0 ? cf.base_layers : cf.draft_layers;
  n.d = which == 0 ? cf.base_d : cf.draft_d;
  n.heads = which == 0 ? cf.base_heads : cf.draft_heads;
  n.m = (which == 0 ? cf.base_mlp_ratio : cf.draft_mlp_ratio) * n.d;
  const size_t d = n.d, m = n.m, A = cf.A, H = cf.H, C = cf.cond_dim;
  size_t o = 0;
  auto take = [&](size_t cnt) { size_t r = o; o += cnt; return r; };
  n.tok_w = take(d * A); n.tok_b = take(d); n.pos = take(H * d);
  n.t_w1 = take(d * d); n.t_b1 = take(d); n.t_w2 = take(d * d); n.t_b2 = take(d);
  n.c_w = n.c_b = 0;
  if (cf.cond_mode == 0) { n.c_w = take(d * C); n.c_b = take(d); }
  n.lay.resize(n.L);
  for (auto& l : n.lay) {
    l.mod_w = take(4 * d * d); l.mod_b = take(4 * d);
    l.qkv_w = take(3 * d * d); l.qkv_b = take(3 * d);
    l.o_w = take(d * d); l.o_b = take(d);
    if (cf.cond_mode == 1) {
      l.cq_w = take(d * d); l.cq_b = take(d);
      l.ck_w = take(d * C); l.ck_b = take(d);
      l.cv_w = take(d * C); l.cv_b = take(d);
      l.co_w = take(d * d); l.co_b = take(d);
    }
    l.up_w = take(m * d); l.up_b = take(m);
    l.dn_w = take(d * m); l.dn_b = take(d);
  }
  n.head_w = take(A * d); n.head_b = take(A);
  n.n_floats = o;
  return o;
}


// Packs one network for the fused kernel (weights as bf16 MFMA fragments, q|k|v rows grouped per head
// group) and fills n.fnet.  `w` is the host copy of the bf16-rounded canonical blob.
int build_fused(tsdp_ctx* c, Net& n, const std::vector<float>& w, const std::vector<float>& modw_cat, const FusedKernels& fk) {
  const tsdp_config& cf = c->cfg;
  const int d = n.d, m = n.m, L = n.L, DH = d / n.heads, HP = DH >= 64 ? 1 : 64 / DH;
  const bool f32 = cf.dtype == 0;
  std::vector<uint8_t> pk;
  std::vector<float> qb((size_t)L * 3 * d);
  struct Off { size_t qkv, o, up, dn, cq, co; };
  std::vector<Off> off(L);
  auto ident = [](int r) { return r; };
  for (int l = 0; l < L; ++l) {
    const LayerOff& o = n.lay[l];
    // logical row lr of the q|k|v matrix: groups of HP heads, inside a group per head [q(DH) k(DH) v(DH)]
    auto qkv_row = [&](int lr) {
      const int g = lr / (HP * 3 * DH), r = lr % (HP * 3 * DH);
      const int head = g * HP + r / (3 * DH), cls = (r / DH) % 3, cdim = r % DH;
      return cls * d + head * DH + cdim;
    };
    off[l].qkv = pk.size(); pack_frags(pk, f32, &w[o.qkv_w], d, 3 * d, qkv_row);
    for (int lr = 0; lr < 3 * d; ++lr) qb[(size_t)l * 3 * d + lr] = w[o.qkv_b + qkv_row(lr)];
    off[l].o = pk.size(); pack_frags(pk, f32, &w[o.o_w], d, d, ident);
    off[l].up = pk.size(); pack_frags(pk, f32, &w[o.up_w], d, m, ident);
    off[l].dn = pk.size(); pack_frags(pk, f32, &w[o.dn_w], m, d, ident);
    if (cf.cond_mode == 1) {
      off[l].cq = pk.size(); pack_frags(pk, f32, &w[o.cq_w], d, d, ident);
      off[l].co = pk.size(); pack_frags(pk, f32, &w[o.co_w], d, d, ident);
    }
  }
  const size_t head_off = pk.size();
  pack_frags(pk, f32, &w[n.head_w], d, (cf.A + 15) / 16 * 16, [&](int r) { return r < cf.A ? r : -1; });
  const size_t mod_off = pk.size();
  pack_frags(pk, f32, modw_cat.data(), d, L * 4 * d, ident);
  uint8_t* dpk = nullptr;
  float* dqb = nullptr;
  int rc;
  if ((rc = dev_alloc(c, &dpk, pk.size()))) return rc;
  if ((rc = dev_alloc(c, &dqb, qb.size()))) return rc;
  HIPCHK(c, hipMemcpy(dpk, pk.data(), pk.size(), hipMemcpyHostToDevice));
  HIPCHK(c, hipMemcpy(dqb, qb.data(), qb.size() * sizeof(float), hipMemcpyHostToDevice));
  FusedNet& f = n.fnet;
  std::memset(&f, 0, sizeof(f));
  f.L = L;
  auto P = [&](size_t o) { return reinterpret_cast<const void*>(dpk + o); };
  for (int l = 0; l < L; ++l) {
    const LayerOff& o = n.lay[l];
    FusedLayer& fl = f.layer[l];
    fl.qkv = P(off[l].qkv); fl.o = P(off[l].o); fl.up = P(off[l].up); fl.dn = P(off[l].dn);
    fl.qkv_b = dqb + (size_t)l * 3 * d;
    fl.o_b = n.blob + o.o_b; fl.up_b = n.blob + o.up_b; fl.dn_b = n.blob + o.dn_b;
    if (cf.cond_mode == 1) {
      fl.cq = P(off[l].cq); fl.co = P(off[l].co);
      fl.cq_b = n.blob + o.cq_b; fl.co_b = n.blob + o.co_b;
    }
  }
  f.tok_w = n.blob + n.tok_w; f.tok_b = n.blob + n.tok_b; f.pos = n.blob + n.pos;
  f.head = P(head_off); f.head_b = n.blob + n.head_b;
  f.modtab = nullptr;
  f.rms = cf.norm;
  f.modw = P(mod_off); f.modb = n.modb; f.temb = n.temb; f.cemb = cf.cond_mode == 0 ? n.cemb : nullptr;
  if (cf.cond_mode == 1) {
    const size_t S = cf.cond_tokens, cnt = (size_t)cf.B_max * L * S * d;
    if ((rc = dev_alloc(c, &n.kc_pk, cnt))) return rc;
    if ((rc = dev_alloc(c, &n.vct_pk, cnt))) return rc;
    f.kc = reinterpret_cast<const bf16x8*>(n.kc_pk);
    f.vct = reinterpret_cast<const bf16x4*>(n.vct_pk);
  }
  n.fused = true;
  n.fused_verify = fk.verify;
  n.fused_verify_few = fk.verify_few;
  n.verify_rpt = fk.rpt_verify;
  n.fused_mod = fk.mod;
  n.fused_draft_small = fk.draft_small; n.fused_draft_big = fk.draft_big;
  n.draft_rpt_small = fk.rpt_small; n.draft_rpt_big = fk.rpt_big;
  n.path = f32 ? "f32-mfma-fused" : "bf16-mfma-fused";
  return TSDP_OK;
}

inline dim3 grid1(long long n, int bs) { return dim3((unsigned)((n + bs - 1) / bs)); }

template <int EPI>
void linear(hipStream_t s, const float* in, const float* W, const float* bias, float* out, int units_cap,
            int rows_per_unit, int N, int K, const int32_t* d_R) {
  const long long M = (long long)units_cap * rows_per_unit;
  dim3 g((N + 63) / 64, (unsigned)((M + 63) / 64));
  hipLaunchKernelGGL(k_linear<EPI>, g, dim3(256), 0, s, in, W, bias, out, rows_per_unit, N, K, d_R, units_cap);
}

// eps[R,H,A] = network(x_rows; t, cond) with the fp32 operator kernels.
void forward_f32(tsdp_ctx* c, Net& n, const float* x_rows, int R_cap, const int32_t* d_R, const int32_t* t_arr,
                 int t_sub, const int32_t* env_arr, float* eps_out, hipStream_t s) {
  const tsdp_config& cf = c->cfg;
  const int H = cf.H, A = cf.A, d = n.d, L = n.L, m = n.m, dh = n.d / n.heads;
  const long long M = (long long)R_cap * H;
  const float* w = n.blob;
  hipLaunchKernelGGL(k_embed, grid1(M * d, 256), dim3(256), 0, s, x_rows, w + n.tok_w, w + n.tok_b, w + n.pos, c->h,
                     H, A, d, d_R, R_cap);
  hipLaunchKernelGGL(k_gvec, grid1((long long)R_cap * d, 256), dim3(256), 0, s, t_arr, t_sub, env_arr, n.temb,
                     cf.cond_mode == 0 ? n.cemb : nullptr, c->sg, d, cf.T, d_R, R_cap);
  const int ms = L * 4 * d;                         // modulation row stride
  linear<0>(s, c->sg, n.modw, n.modb, c->mod, R_cap, 1, ms, d, d_R);
  const dim3 lng((unsigned)((M + 3) / 4));
  for (int l = 0; l < L; ++l) {
    const LayerOff& o = n.lay[l];
    const float* mod = c->mod + (size_t)l * 4 * d;
    hipLaunchKernelGGL(k_lnmod, lng, dim3(256), 0, s, c->h, mod, mod + d, ms, c->a, H, d, cf.norm, d_R, R_cap);
    linear<0>(s, c->a, w + o.qkv_w, w + o.qkv_b, c->qkv, R_cap, H, 3 * d, d, d_R);
    hipLaunchKernelGGL(k_attn, dim3(R_cap, n.heads), dim3(256), H * H * sizeof(float), s, c->qkv, 3 * d, c->qkv + d,
                       c->qkv + 2 * d, 3 * d, (const int32_t*)nullptr, c->ao, d, H, H, dh, d_R, R_cap);
    linear<2>(s, c->ao, w + o.o_w, w + o.o_b, c->h, R_cap, H, d, d, d_R);
    if (cf.cond_mode == 1) {
      const int S = cf.cond_tokens;
      const size_t per_layer = (size_t)cf.B_max * S * d;
      hipLaunchKernelGGL(k_lnmod, lng, dim3(256), 0, s, c->h, (const float*)nullptr, (const float*)nullptr, 0, c->a, H, d, cf.norm, d_R, R_cap);
      linear<0>(s, c->a, w + o.cq_w, w + o.cq_b, c->qkv, R_cap, H, d, d, d_R);
      hipLaunchKernelGGL(k_attn, dim3(R_cap, n.heads), dim3(256), H * S * sizeof(float), s, c->qkv, d,
                         n.kc + l * per_layer, n.vc + l * per_layer, d, env_arr, c->ao, d, H, S, dh, d_R, R_cap);
      linear<2>(s, c->ao, w + o.co_w, w + o.co_b, c->h, R_cap, H, d, d, d_R);
    }
    hipLaunchKernelGGL(k_lnmod, lng, dim3(256), 0, s, c->h, mod + 2 * d, mod + 3 * d, ms, c->a, H, d, cf.norm, d_R, R_cap);
    linear<1>(s, c->a, w + o.up_w, w + o.up_b, c->u, R_cap, H, m, d, d_R);
    linear<2>(s, c->u, w + o.dn_w, w + o.dn_b, c->h, R_cap, H, d, m, d_R);
  }
  hipLaunchKernelGGL(k_lnmod, lng, dim3(256), 0, s, c->h, (const float*)nullptr, (const float*)nullptr, 0, c->a, H, d, cf.norm, d_R, R_cap);
  linear<0>(s, c->a, w + n.head_w, w + n.head_b, eps_out, R_cap, H, A, d, d_R);
}

// eps[R,H,A] = network(x_rows; t, cond): fused bf16 MFMA kernel where the shape has one, fp32 operators otherwise.
// mod_ready: the FiLM vectors of these rows are already in c->mod (computed on the auxiliary stream; the caller has
// made `s` wait for them)
int forward(tsdp_ctx* c, Net& n, const float* x_rows, int R_cap, const int32_t* d_R, const int32_t* t_arr,
            int t_sub, const int32_t* env_arr, float* eps_out, hipStream_t s, bool mod_ready = false) {
  if (!n.fused) {
    forward_f32(c, n, x_rows, R_cap, d_R, t_arr, t_sub, env_arr, eps_out, s);
    return TSDP_OK;
  }
  const tsdp_config& cf = c->cfg;
  if (n.fnet.modtab || mod_ready) {
    // token conditioning: the FiLM vectors are a function of the timestep only and were tabulated at load time
  } else if (n.fused_mod) {
    const bool base = &n == &c->net[0];
    if (base) tick(c, 3, 0, s);
    n.fused_mod(n.fnet, t_arr, t_sub, env_arr, cf.T, d_R, R_cap, c->mod, s);
    if (base) tick(c, 3, 1, s);
  } else {                                            // fp32 networks: exact fp32 FiLM vectors from the operator kernels
    hipLaunchKernelGGL(k_gvec, grid1((long long)R_cap * n.d, 256), dim3(256), 0, s, t_arr, t_sub, env_arr, n.temb,
                       cf.cond_mode == 0 ? n.cemb : nullptr, c->sg, n.d, cf.T, d_R, R_cap);
    linear<0>(s, c->sg, n.modw, n.modb, c->mod, R_cap, 1, n.L * 4 * n.d, n.d, d_R);
  }
  FusedIO io;
  io.x_rows = x_rows; io.mod = c->mod; io.row_t = t_arr; io.t_sub = t_sub; io.T = cf.T; io.row_env = env_arr; io.d_R = d_R; io.R_cap = R_cap; io.eps_out = eps_out;
  const int stage = (&n == &c->net[0]) ? 1 : -1;          // only the base network's forward is the verify stage
  if (stage == 1) tick(c, 1, 0, s);
  const bool few = n.fused_verify_few && (R_cap + n.verify_rpt - 1) / n.verify_rpt <= FEW_TILES;
  HIPCHK(c, (few ? n.fused_verify_few : n.fused_verify)(n.fnet, io, cf.A, R_cap, s));
  if (stage == 1) tick(c, 1, 1, s);
  return TSDP_OK;
}

// dynamic LDS of the persistent drafter kernel for `rpt` environments per workgroup (mirrors launch_draft)
size_t fused_draft_lds(const Net& n, const tsdp_config& cf, int rpt) {
  const size_t ES = cf.dtype == 0 ? 4 : 2, PAD = cf.dtype == 0 ? 4 : 8;
  const size_t D = n.d, NT = (size_t)rpt * cf.H, DH = D / n.heads, HP = n.heads;      // upper bounds over the
  const size_t CH = 4 * D;                                                             // compiled tile variants
  const size_t act = NT * (D + PAD) * ES, q = HP * NT * (DH + PAD) * ES, vt = HP * rpt * DH * (cf.H + 4) * ES;
  const size_t scr = std::max(std::max(2 * q + vt, NT * (CH + PAD) * ES), NT * 64 * 4);
  return act + scr + 2 * 8 * NT * 4 + 2 * NT * cf.A * 4 + (size_t)rpt * n.L * 4 * D * 4 + 16 * (D + PAD) * ES;  // upper bound
}

// rows of the ragged batch a context must hold: K_max per environment, one more with the bonus row
inline size_t rows_max(const tsdp_config& cf) { return (size_t)cf.B_max * (cf.K_max + (cf.bonus_row ? 1 : 0)); }

int ensure_workspace(tsdp_ctx* c) {
  if (c->ws_ready) return TSDP_OK;
  const tsdp_config& cf = c->cfg;
  const size_t Rw = rows_max(cf), Mw = Rw * cf.H;
  const size_t dmax = std::max(cf.base_d, cf.draft_d);
  const size_t mmax = std::max(c->net[0].m, c->net[1].m);
  const size_t lmax = std::max(cf.base_layers, cf.draft_layers);
  int rc;
  if ((rc = dev_alloc(c, &c->h, Mw * dmax))) return rc;
  if ((rc = dev_alloc(c, &c->a, Mw * dmax))) return rc;
  if ((rc = dev_alloc(c, &c->qkv, Mw * 3 * dmax))) return rc;
  if ((rc = dev_alloc(c, &c->ao, Mw * dmax))) return rc;
  if ((rc = dev_alloc(c, &c->u, Mw * mmax))) return rc;
  if ((rc = dev_alloc(c, &c->sg, Rw * dmax))) return rc;
  if ((rc = dev_alloc(c, &c->mod, Rw * lmax * 4 * dmax))) return rc;
  if ((rc = dev_alloc(c, &c->eps_tmp, (size_t)cf.B_max * c->D))) return rc;
  if ((rc = dev_alloc(c, &c->row_t_chk, Rw))) return rc;
  if ((rc = dev_alloc(c, &c->row_env_chk, Rw))) return rc;
  c->ws_ready = true;
  return TSDP_OK;
}

int ensure_round_buffers(tsdp_ctx* c) {
  if (c->rb_ready) return TSDP_OK;
  const tsdp_config& cf = c->cfg;
  const size_t Rw = rows_max(cf), B = cf.B_max, D = c->D;
  int rc;
  if ((rc = dev_alloc(c, &c->row_ptr, B + 1))) return rc;
  if ((rc = dev_alloc(c, &c->row_t, Rw))) return rc;
  if ((rc = dev_alloc(c, &c->row_env, Rw))) return rc;
  if ((rc = dev_alloc(c, &c->t_next, B))) return rc;
  if ((rc = dev_alloc(c, &c->n_acc, B))) return rc;
  if ((rc = dev_alloc(c, &c->n_adv, B))) return rc;
  if ((rc = dev_alloc(c, &c->states, Rw * D))) return rc;
  if ((rc = dev_alloc(c, &c->eps_p, Rw * D))) return rc;
  if ((rc = dev_alloc(c, &c->eps_q, Rw * D))) return rc;
  if ((rc = dev_alloc(c, &c->xi, Rw * D))) return rc;
  if ((rc = dev_alloc(c, &c->y_last, B * D))) return rc;
  c->rb_ready = true;
  return TSDP_OK;
}

int check_ready(tsdp_ctx* c, int B, bool need_nets) {
  if (!c) return TSDP_E_INVAL;
  if (B < 0 || B > c->cfg.B_max) return fail(c, TSDP_E_SHAPE, "B outside 0..B_max");
  if (need_nets) {
    if (!c->net[0].loaded || !c->net[1].loaded) return fail(c, TSDP_E_STATE, "weights of both networks must be loaded");
    if (!c->cond_set) return fail(c, TSDP_E_STATE, "tsdp_set_cond has not been called");
    if (B > c->cond_B) return fail(c, TSDP_E_SHAPE, "B exceeds the batch given to tsdp_set_cond");
  }
  return TSDP_OK;
}

}  // namespace

extern "C" {

int tsdp_create(const tsdp_config* cfg, tsdp_ctx** out) {
  if (!cfg || !out) return TSDP_E_INVAL;
  *out = nullptr;
  const tsdp_config& f = *cfg;
  auto bad = [&](int d, int heads, int L, int mr) {
    return L < 1 || L > 64 || d < 8 || d > 1024 || d % 4 || heads < 1 || d % heads || (d / heads) > 128 || mr < 1 || mr > 8;
  };
  if (f.dtype < 0 || f.dtype > 1 || f.H < 1 || f.H > 64 || f.A < 1 || f.A > 64 || (f.H * f.A) % 4 || f.H * f.A > 512 || f.cond_mode < 0 ||
      f.cond_mode > 1 || f.cond_dim < 4 || f.cond_dim % 4 || (f.cond_mode == 1 && (f.cond_tokens < 1 || f.cond_tokens > 256)) ||
      bad(f.base_d, f.base_heads, f.base_layers, f.base_mlp_ratio) ||
      bad(f.draft_d, f.draft_heads, f.draft_layers, f.draft_mlp_ratio) || f.T < 1 || f.T > 4096 || f.schedule < 0 ||
      f.schedule > 1 || f.B_max < 1 || f.K_max < 1 || f.K_max > 64 || (f.clip_x0 && !(f.clip_val > 0.0f)))
    return TSDP_E_INVAL;
  if (f.sampler < 0 || f.sampler > 1 || (f.sampler == 1 && !(f.eta > 0.0f && f.eta <= 1.0f))) return TSDP_E_INVAL;
  if (f.schedule == 0 && !(f.beta0 > 0.0f && f.beta1 >= f.beta0 && f.beta1 < 1.0f)) return TSDP_E_INVAL;
  if (f.bonus_row < 0 || f.bonus_row > 1 || f.norm < 0 || f.norm > 1) return TSDP_E_INVAL;
  if ((long long)f.B_max * (f.K_max + 1) > (1ll << 24)) return TSDP_E_SHAPE;
  tsdp_ctx* c = new (std::nothrow) tsdp_ctx();
  if (!c) return TSDP_E_NOMEM;
  c->cfg = f;
  c->D = f.H * f.A;
  layout_net(f, 0, c->net[0]);
  layout_net(f, 1, c->net[1]);
  // DDPM tables: textbook epsilon-prediction posterior with the fixed-small variance, fp64 then fp32
  const int T = f.T;
  std::vector<double> beta(T), abar(T);
  const double PI = 3.14159265358979323846;
  for (int i = 0; i < T; ++i) {
    if (f.schedule == 0) {
      beta[i] = T == 1 ? (double)f.beta0 : (double)f.beta0 + ((double)f.beta1 - (double)f.beta0) * i / (T - 1);
    } else {
      auto fc = [&](double j) { double v = std::cos(((j / T) + 0.008) / 1.008 * PI / 2.0); return v * v; };
      beta[i] = std::min(1.0 - fc(i + 1.0) / fc((double)i), 0.999);
    }
    abar[i] = (i ? abar[i - 1] : 1.0) * (1.0 - beta[i]);
  }
  std::vector<float> tab(6 * (size_t)T);
  for (int t = 0; t < T; ++t) {
    const double ap = t ? abar[t - 1] : 1.0;
    tab[0 * T + t] = (float)std::sqrt(abar[t]);
    tab[1 * T + t] = (float)std::sqrt(1.0 - abar[t]);
    if (f.sampler == 0) {                             // DDPM posterior: mu = c0 x0_hat + cx x
      tab[2 * T + t] = (float)(std::sqrt(ap) * beta[t] / (1.0 - abar[t]));
      tab[3 * T + t] = (float)(std::sqrt(1.0 - beta[t]) * (1.0 - ap) / (1.0 - abar[t]));
      tab[4 * T + t] = (float)std::sqrt(beta[t] * (1.0 - ap) / (1.0 - abar[t]));
      tab[5 * T + t] = 0.0f;
    } else {                                          // DDIM(eta): mu = sqrt(abar') x0_hat + sqrt(1 - abar' - sigma^2) eps
      const double sig = (double)f.eta * std::sqrt((1.0 - ap) / (1.0 - abar[t])) * std::sqrt(1.0 - abar[t] / ap);
      tab[2 * T + t] = (float)std::sqrt(ap);
      tab[3 * T + t] = 0.0f;
      tab[4 * T + t] = (float)sig;
      tab[5 * T + t] = (float)std::sqrt(std::max(1.0 - ap - sig * sig, 0.0));
    }
  }
  auto cleanup = [&](int code) { tsdp_destroy(c); return code; };
  if (dev_alloc(c, &c->tables, tab.size())) return cleanup(TSDP_E_NOMEM);
  if (hipMemcpy(c->tables, tab.data(), tab.size() * sizeof(float), hipMemcpyHostToDevice) != hipSuccess)
    return cleanup(TSDP_E_HIP);
  c->tb = {c->tables, c->tables + T, c->tables + 2 * T, c->tables + 3 * T, c->tables + 4 * T, c->tables + 5 * T, T};
  if (dev_alloc(c, &c->status, 1) || dev_alloc(c, &c->K_eff, (size_t)f.B_max) || dev_alloc(c, &c->n_draft, 2))
    return cleanup(TSDP_E_NOMEM);
  if (hipGetDevice(&c->device) != hipSuccess || c->device < 0 || c->device >= NOALLOC_MAX_DEVICES) return cleanup(TSDP_E_HIP);
  if (!g_scratch_ptr[c->device]) {
    double* p = nullptr;
    if (hipGetSymbolAddress(reinterpret_cast<void**>(&p), HIP_SYMBOL(scratch)) != hipSuccess || !p) return cleanup(TSDP_E_HIP);
    g_scratch_ptr[c->device] = p;
  }
  if (hipMemset(c->status, 0, sizeof(int32_t)) != hipSuccess) return cleanup(TSDP_E_HIP);
  if (hipStreamCreateWithFlags(&c->aux, hipStreamNonBlocking) != hipSuccess ||
      hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming) != hipSuccess ||
      hipEventCreateWithFlags(&c->ev_join, hipEventDisableTiming) != hipSuccess)
    return cleanup(TSDP_E_HIP);
  *out = c;
  return TSDP_OK;
}

void tsdp_destroy(tsdp_ctx* c) {
  if (!c) return;
  (void)hipDeviceSynchronize();
  for (auto& st : c->ev)
    for (auto& e : st)
      if (e) (void)hipEventDestroy(e);
  if (c->ev_fork) (void)hipEventDestroy(c->ev_fork);
  if (c->ev_join) (void)hipEventDestroy(c->ev_join);
  if (c->aux) (void)hipStreamDestroy(c->aux);
  for (void* p : c->owned) (void)hipFree(p);
  delete c;
}

int tsdp_load_weights(tsdp_ctx* c, int which, const float* h_blob, size_t nbytes) {
  if (!c) return TSDP_E_INVAL;
  if (!h_blob || which < 0 || which > 1) return fail(c, TSDP_E_INVAL, "bad argument to tsdp_load_weights");
  Net& n = c->net[which];
  if (nbytes != n.n_floats * sizeof(float))
    return fail(c, TSDP_E_SHAPE, "weight blob has " + std::to_string(nbytes) + " bytes, expected " +
                                     std::to_string(n.n_floats * sizeof(float)));
  const tsdp_config& cf = c->cfg;
  std::vector<float> w(h_blob, h_blob + n.n_floats);
  if (cf.dtype == 1)
    for (auto& v : w) v = bf16_round(v);
  const int d = n.d, T = cf.T, L = n.L;
  // timestep embedding of every timestep (depends on the weights only): fp64 on the host
  std::vector<float> temb((size_t)T * d);
  {
    const int half = d / 2;
    std::vector<double> e(d), hdn(d);
    for (int t = 0; t < T; ++t) {
      for (int i = 0; i < half; ++i) {
        const double fr = std::exp(-std::log(10000.0) * i / half);
        e[i] = std::sin(t * fr);
        e[half + i] = std::cos(t * fr);
      }
      for (int i = 2 * half; i < d; ++i) e[i] = 0.0;
      for (int o = 0; o < d; ++o) {
        double acc = w[n.t_b1 + o];
        for (int i = 0; i < d; ++i) acc += (double)w[n.t_w1 + (size_t)o * d + i] * e[i];
        hdn[o] = acc / (1.0 + std::exp(-acc));
      }
      for (int o = 0; o < d; ++o) {
        double acc = w[n.t_b2 + o];
        for (int i = 0; i < d; ++i) acc += (double)w[n.t_w2 + (size_t)o * d + i] * hdn[i];
        temb[(size_t)t * d + o] = (float)acc;
      }
    }
  }
  std::vector<float> modw((size_t)L * 4 * d * d), modb((size_t)L * 4 * d);
  for (int l = 0; l < L; ++l) {
    std::memcpy(&modw[(size_t)l * 4 * d * d], &w[n.lay[l].mod_w], sizeof(float) * 4 * d * d);
    std::memcpy(&modb[(size_t)l * 4 * d], &w[n.lay[l].mod_b], sizeof(float) * 4 * d);
  }
  int rc;
  if (!n.blob) {
    if ((rc = dev_alloc(c, &n.blob, n.n_floats))) return rc;
    if ((rc = dev_alloc(c, &n.temb, temb.size()))) return rc;
    if ((rc = dev_alloc(c, &n.modw, modw.size()))) return rc;
    if ((rc = dev_alloc(c, &n.modb, modb.size()))) return rc;
    if (cf.cond_mode == 0) {
      if ((rc = dev_alloc(c, &n.cemb, (size_t)cf.B_max * d))) return rc;
    } else {
      const size_t cnt = (size_t)L * cf.B_max * cf.cond_tokens * d;
      if ((rc = dev_alloc(c, &n.kc, cnt))) return rc;
      if ((rc = dev_alloc(c, &n.vc, cnt))) return rc;
    }
  }
  HIPCHK(c, hipDeviceSynchronize());
  HIPCHK(c, hipMemcpy(n.blob, w.data(), w.size() * sizeof(float), hipMemcpyHostToDevice));
  HIPCHK(c, hipMemcpy(n.temb, temb.data(), temb.size() * sizeof(float), hipMemcpyHostToDevice));
  HIPCHK(c, hipMemcpy(n.modw, modw.data(), modw.size() * sizeof(float), hipMemcpyHostToDevice));
  HIPCHK(c, hipMemcpy(n.modb, modb.data(), modb.size() * sizeof(float), hipMemcpyHostToDevice));
  n.loaded = true;
  c->cond_set = false;
  n.fused = false;
  n.path = "f32-ops";
  if (!std::getenv("TSDP_DISABLE_FUSED")) {
    FusedKernels fk;
    if (find_fused(cf.dtype, n.d, cf.H, n.heads, cf.cond_mode, cf.cond_tokens, n.m / n.d, n.L, fk) &&
        (rc = build_fused(c, n, w, modw, fk)))
      return rc;
  }
  if (n.fused && n.fused_mod && cf.cond_mode == 1) {
    // With token conditioning no conditioning vector enters the FiLM projections: they depend on the timestep
    // alone, so the vectors of all T timesteps are computed once, by the kernel that otherwise computes them per row.
    const int T = cf.T;
    if (!n.modtab) {
      if ((rc = dev_alloc(c, &n.modtab, (size_t)T * L * 4 * d))) return rc;
      if ((rc = dev_alloc(c, &n.t_iota, (size_t)T))) return rc;
      std::vector<int32_t> iota(T);
      for (int t = 0; t < T; ++t) iota[t] = t;
      HIPCHK(c, hipMemcpy(n.t_iota, iota.data(), sizeof(int32_t) * T, hipMemcpyHostToDevice));
    }
    n.fused_mod(n.fnet, n.t_iota, 0, nullptr, T, nullptr, T, n.modtab, nullptr);
    HIPCHK(c, hipGetLastError());
    HIPCHK(c, hipDeviceSynchronize());
    n.fnet.modtab = n.modtab;
  }
  return TSDP_OK;
}

int tsdp_set_cond(tsdp_ctx* c, const float* d_cond, int B, void* stream) {
  if (!c) return TSDP_E_INVAL;
  if (!d_cond) return fail(c, TSDP_E_INVAL, "d_cond is null");
  if (B < 1 || B > c->cfg.B_max) return fail(c, TSDP_E_SHAPE, "B outside 1..B_max");
  if (!c->net[0].loaded || !c->net[1].loaded) return fail(c, TSDP_E_STATE, "weights of both networks must be loaded");
  hipStream_t s = (hipStream_t)stream;
  const tsdp_config& cf = c->cfg;
  for (int which = 0; which < 2; ++which) {
    Net& n = c->net[which];
    const float* w = n.blob;
    if (cf.cond_mode == 0) {
      linear<0>(s, d_cond, w + n.c_w, w + n.c_b, n.cemb, B, 1, n.d, cf.cond_dim, nullptr);
    } else {
      const int S = cf.cond_tokens;
      const size_t per_layer = (size_t)cf.B_max * S * n.d;
      for (int l = 0; l < n.L; ++l) {
        linear<0>(s, d_cond, w + n.lay[l].ck_w, w + n.lay[l].ck_b, n.kc + l * per_layer, B * S, 1, n.d, cf.cond_dim, nullptr);
        linear<0>(s, d_cond, w + n.lay[l].cv_w, w + n.lay[l].cv_b, n.vc + l * per_layer, B * S, 1, n.d, cf.cond_dim, nullptr);
        if (n.fused) {
          const long long cnt = (long long)B * S * n.d / 8;
          hipLaunchKernelGGL(k_pack_kc, grid1(cnt, 256), dim3(256), 0, s, (const float*)(n.kc + l * per_layer),
                             reinterpret_cast<__bf16*>(n.kc_pk), B, S, n.d, n.heads, n.L, l);
          hipLaunchKernelGGL(k_pack_vct, grid1(2 * cnt, 256), dim3(256), 0, s, (const float*)(n.vc + l * per_layer),
                             reinterpret_cast<__bf16*>(n.vct_pk), B, S, n.d, n.heads, n.L, l);
        }
      }
    }
  }
  HIPCHK(c, hipGetLastError());
  c->cond_set = true;
  c->cond_B = B;
  return TSDP_OK;
}

// gated: chain driver -- the row-table kernel also returns at once when no environment has rows (the drafter kernels
// always do: without rows there is nothing to draft)
static int draft_impl(tsdp_ctx* c, int B, const float* d_x, const int32_t* d_t0, const int32_t* d_K,
                      const float* d_sigma_scale, const int32_t* d_env_id, int32_t* d_row_ptr, int32_t* d_row_t,
                      int32_t* d_row_env, float* d_states, float* d_eps_p, float* d_xi, float* d_y_last, bool gated,
                      void* stream, int base_mod_rows = 0, bool* base_mod_started = nullptr) {
  // base_mod_rows > 0 (whole rounds): once the row table exists, the base network's per-row FiLM vectors of up to that
  // many rows are computed on the auxiliary stream, beside the rollout; *base_mod_started tells the caller to join
  int rc = check_ready(c, B, true);
  if (rc) return rc;
  if (B == 0) return TSDP_OK;                        // an empty batch is valid and touches nothing
  if (!d_x || !d_t0 || !d_K || !d_sigma_scale || !d_row_ptr || !d_row_t || !d_row_env || !d_states || !d_eps_p ||
      !d_y_last)
    return fail(c, TSDP_E_INVAL, "null pointer passed to tsdp_draft");
  if ((rc = ensure_workspace(c))) return rc;
  hipStream_t s = (hipStream_t)stream;
  const tsdp_config& cf = c->cfg;
  const int D = c->D;
  hipLaunchKernelGGL(k_plan, dim3(1), dim3(1024), 0, s, d_t0, d_K, d_sigma_scale, B, cf.K_max, cf.T, cf.bonus_row, c->K_eff,
                     d_row_ptr, c->status, c->n_draft);
  auto bonus_rows = [&]() {
    if (cf.bonus_row)
      hipLaunchKernelGGL(k_bonus_rows, dim3(B), dim3(128), 0, s, d_t0, (const int32_t*)c->K_eff, (const int32_t*)d_row_ptr,
                         d_env_id, cf.T, D, cf.seed, (const float*)d_y_last, d_states, d_eps_p, d_xi);
  };
  hipLaunchKernelGGL(k_rows, dim3(B), dim3(128), 0, s, d_x, d_t0, (const int32_t*)d_row_ptr, cf.T, D, d_row_t,
                     d_row_env, d_y_last, d_states, d_eps_p, d_xi, gated ? (const int32_t*)c->n_draft : nullptr);
  Net& dn = c->net[1];
  if (dn.fused) {
    // persistent drafter kernel: pick the tile (environments per workgroup) that fills the chip best
    const bool big = (B + dn.draft_rpt_big - 1) / dn.draft_rpt_big >= 192;
    const int rpt = big ? dn.draft_rpt_big : dn.draft_rpt_small;
    const size_t lds = fused_draft_lds(dn, cf, rpt);
    if (lds <= 160 * 1024) {
      Net& bn = c->net[0];
      if (base_mod_rows > 0 && bn.fused && bn.fused_mod && !bn.fnet.modtab) {
        // fork: the fused rollout keeps its FiLM vectors in LDS, so the shared buffer is free for the base network's
        HIPCHK(c, hipEventRecord(c->ev_fork, s));
        HIPCHK(c, hipStreamWaitEvent(c->aux, c->ev_fork, 0));
        bn.fused_mod(bn.fnet, d_row_t, 0, d_row_env, cf.T, d_row_ptr + B, base_mod_rows, c->mod, c->aux);
        HIPCHK(c, hipEventRecord(c->ev_join, c->aux));
        if (base_mod_started) *base_mod_started = true;
      }
      DraftIO io;
      io.B = B; io.t0 = d_t0; io.K_eff = c->K_eff; io.row_ptr = d_row_ptr; io.sigma_scale = d_sigma_scale;
      io.env_id = d_env_id;
      io.tb = {c->tb.sqrt_abar, c->tb.sqrt_1m, c->tb.c0, c->tb.cx, c->tb.sigma, c->tb.ce, c->tb.T};
      io.clip = cf.clip_x0; io.clip_val = cf.clip_val; io.seed = cf.seed;
      io.y = d_y_last; io.states = d_states; io.eps_p = d_eps_p; io.xi = d_xi;
      io.gate = c->n_draft + 1;
      tick(c, 0, 0, s);
      HIPCHK(c, (big ? dn.fused_draft_big : dn.fused_draft_small)(dn.fnet, io, cf.A, s));
      tick(c, 0, 1, s);
      bonus_rows();
      HIPCHK(c, hipGetLastError());
      return TSDP_OK;
    }
  }
  for (int k = 1; k <= cf.K_max; ++k) {
    // every environment runs the drafter at step k; the DDPM step masks those with K_eff < k
    if ((rc = forward(c, c->net[1], d_y_last, B, c->n_draft + 1, d_t0, k - 1, nullptr, c->eps_tmp, s))) return rc;
    hipLaunchKernelGGL(k_draft_step, grid1((long long)B * (D / 4), 256), dim3(256), 0, s, k, (const float*)c->eps_tmp,
                       d_t0, (const int32_t*)c->K_eff, (const int32_t*)d_row_ptr, d_sigma_scale, d_env_id, c->tb,
                       cf.clip_x0, cf.clip_val, cf.seed, B, D, d_y_last, d_states, d_eps_p, d_xi);
  }
  bonus_rows();
  HIPCHK(c, hipGetLastError());
  return TSDP_OK;
}

int tsdp_draft(tsdp_ctx* c, int B, const float* d_x, const int32_t* d_t0, const int32_t* d_K,
               const float* d_sigma_scale, const int32_t* d_env_id, int32_t* d_row_ptr, int32_t* d_row_t,
               int32_t* d_row_env, float* d_states, float* d_eps_p, float* d_xi, float* d_y_last, void* stream) {
  return draft_impl(c, B, d_x, d_t0, d_K, d_sigma_scale, d_env_id, d_row_ptr, d_row_t, d_row_env, d_states, d_eps_p, d_xi,
                    d_y_last, false, stream);
}

static int verify_impl(tsdp_ctx* c, int B, int R_cap, const int32_t* d_row_ptr, const int32_t* d_row_t,
                       const int32_t* d_row_env, const float* d_states, float* d_eps_q, bool own_table, void* stream,
                       bool mod_ready = false) {
  int rc = check_ready(c, B, true);
  if (rc) return rc;
  if (B == 0 || R_cap == 0) return TSDP_OK;
  if (!d_row_ptr || !d_row_t || !d_row_env || !d_states || !d_eps_q)
    return fail(c, TSDP_E_INVAL, "null pointer passed to tsdp_verify");
  if (R_cap < 0 || (size_t)R_cap > rows_max(c->cfg))
    return fail(c, TSDP_E_SHAPE, "R_cap outside 0..B_max*(K_max+bonus_row)");
  if ((rc = ensure_workspace(c))) return rc;
  hipStream_t s = (hipStream_t)stream;
  if (!own_table) {
    // a caller's row table: timesteps and environment indices are clamped into range (the kernels index tables
    // with them) and the status word reports it
    hipLaunchKernelGGL(k_check_rows, grid1(R_cap, 256), dim3(256), 0, s, d_row_ptr + B, R_cap, d_row_t, d_row_env, c->cfg.T,
                       c->cond_B, c->row_t_chk, c->row_env_chk, c->status);
    d_row_t = c->row_t_chk;
    d_row_env = c->row_env_chk;
  }
  if (mod_ready) HIPCHK(c, hipStreamWaitEvent(s, c->ev_join, 0));   // join: the FiLM vectors computed beside the rollout
  if ((rc = forward(c, c->net[0], d_states, R_cap, d_row_ptr + B, d_row_t, 0, d_row_env, d_eps_q, s, mod_ready))) return rc;
  HIPCHK(c, hipGetLastError());
  return TSDP_OK;
}

int tsdp_verify(tsdp_ctx* c, int B, int R_cap, const int32_t* d_row_ptr, const int32_t* d_row_t,
                const int32_t* d_row_env, const float* d_states, float* d_eps_q, void* stream) {
  return verify_impl(c, B, R_cap, d_row_ptr, d_row_t, d_row_env, d_states, d_eps_q, false, stream);
}

static int accept_impl(tsdp_ctx* c, int B, const int32_t* d_row_ptr, const int32_t* d_row_t, const int32_t* d_env_id,
                       const float* d_sigma_scale, const float* d_lambda, const float* d_states, const float* d_eps_p,
                       const float* d_eps_q, const float* d_xi, const float* d_y_last, float* d_x_out, int32_t* d_t_next,
                       int32_t* d_n_accept, int32_t* d_n_adv, uint8_t* d_flags, float* d_logratio, float* d_logu,
                       const int32_t* d_gate, void* stream) {
  int rc = check_ready(c, B, false);
  if (rc) return rc;
  if (B == 0) return TSDP_OK;
  if (!d_row_ptr || !d_row_t || !d_sigma_scale || !d_states || !d_eps_p || !d_eps_q || !d_y_last || !d_x_out ||
      !d_t_next || !d_n_accept)
    return fail(c, TSDP_E_INVAL, "null pointer passed to tsdp_accept");
  hipStream_t s = (hipStream_t)stream;
  const tsdp_config& cf = c->cfg;
  const int wpb = 4;                                // environments (wavefronts) per workgroup
  const dim3 g((B + wpb - 1) / wpb), blk(64 * wpb);
  tick(c, 2, 0, s);
  // lanes per row: the D/4 vectors of a row should fill them (8 lanes x 5 at D = 160, 16 x 7 at D = 448); at most 8 per lane
  const int nb = c->D / 4;
  const int maxi8 = (nb + 7) / 8, maxi16 = (nb + 15) / 16;
  const bool g8 = maxi8 <= 8 && nb * 16 * maxi16 > nb * 8 * maxi8;   // the 8-lane mapping fits and idles fewer lanes
  const int maxi = g8 ? maxi8 : maxi16;
#define TSDP_ACCEPT(CL, GG, MI)                                                                                 \
  if (d_xi) TSDP_ACCEPT_X(CL, false, GG, MI); else TSDP_ACCEPT_X(CL, true, GG, MI)
#define TSDP_ACCEPT_X(CL, RG, GG, MI)                                                                           \
  hipLaunchKernelGGL((k_accept<CL, RG, GG, MI>), g, blk, 0, s, B, c->D, d_row_ptr, d_row_t, d_env_id, d_sigma_scale, \
                     d_states, d_eps_p, d_eps_q, d_xi, d_y_last, c->tb, cf.clip_val, cf.seed, d_lambda, cf.bonus_row, d_x_out, d_t_next, \
                     d_n_accept, d_n_adv, d_flags, d_logratio, d_logu, d_gate)
#define TSDP_ACCEPT_MI(MI)                                                       \
  case MI:                                                                       \
    if (cf.clip_x0) { if (g8) TSDP_ACCEPT(true, 8, MI); else TSDP_ACCEPT(true, 16, MI); }    \
    else            { if (g8) TSDP_ACCEPT(false, 8, MI); else TSDP_ACCEPT(false, 16, MI); }  \
    break;
  switch (maxi) {
    TSDP_ACCEPT_MI(1) TSDP_ACCEPT_MI(2) TSDP_ACCEPT_MI(3) TSDP_ACCEPT_MI(4)
    TSDP_ACCEPT_MI(5) TSDP_ACCEPT_MI(6) TSDP_ACCEPT_MI(7) TSDP_ACCEPT_MI(8)
    default: return fail(c, TSDP_E_SHAPE, "H*A above 512 is not supported by the acceptance kernel");
  }
#undef TSDP_ACCEPT_MI
#undef TSDP_ACCEPT
#undef TSDP_ACCEPT_X
  tick(c, 2, 1, s);
  HIPCHK(c, hipGetLastError());
  return TSDP_OK;
}

int tsdp_accept(tsdp_ctx* c, int B, const int32_t* d_row_ptr, const int32_t* d_row_t, const int32_t* d_env_id,
                const float* d_sigma_scale, const float* d_states, const float* d_eps_p, const float* d_eps_q,
                const float* d_xi, const float* d_y_last, float* d_x_out, int32_t* d_t_next, int32_t* d_n_accept,
                int32_t* d_n_adv, uint8_t* d_flags, float* d_logratio, float* d_logu, void* stream) {
  return accept_impl(c, B, d_row_ptr, d_row_t, d_env_id, d_sigma_scale, nullptr, d_states, d_eps_p, d_eps_q, d_xi, d_y_last,
                     d_x_out, d_t_next, d_n_accept, d_n_adv, d_flags, d_logratio, d_logu, nullptr, stream);
}

int tsdp_accept_threshold(tsdp_ctx* c, int B, const int32_t* d_row_ptr, const int32_t* d_row_t,
                          const float* d_sigma_scale, const float* d_lambda, const float* d_states, const float* d_eps_p,
                          const float* d_eps_q, const float* d_xi, const float* d_y_last, float* d_x_out,
                          int32_t* d_t_next, int32_t* d_n_accept, int32_t* d_n_adv, uint8_t* d_flags, float* d_logratio,
                          void* stream) {
  if (c && B > 0 && !d_lambda) return fail(c, TSDP_E_INVAL, "d_lambda is null");
  if (c && B > 0 && !d_xi) return fail(c, TSDP_E_INVAL, "d_xi is null (no environment ids here to regenerate the noise from)");
  return accept_impl(c, B, d_row_ptr, d_row_t, nullptr, d_sigma_scale, d_lambda, d_states, d_eps_p, d_eps_q, d_xi, d_y_last,
                     d_x_out, d_t_next, d_n_accept, d_n_adv, d_flags, d_logratio, nullptr, nullptr, stream);
}

static int round_impl(tsdp_ctx* c, int B, float* d_x, int32_t* d_t, const int32_t* d_K, const float* d_sigma_scale,
                      const int32_t* d_env_id, const float* d_lambda, int32_t* d_n_accept, int32_t* d_n_advanced,
                      bool gated, void* stream) {
  int rc = check_ready(c, B, true);
  if (rc) return rc;
  if (B == 0) return TSDP_OK;
  if (!d_x || !d_t || !d_K || !d_sigma_scale) return fail(c, TSDP_E_INVAL, "null pointer passed to tsdp_round");
  if ((rc = ensure_round_buffers(c))) return rc;
  const int R_cap = B * (c->cfg.K_max + (c->cfg.bonus_row ? 1 : 0));
  bool mod_started = false;
  if ((rc = draft_impl(c, B, d_x, d_t, d_K, d_sigma_scale, d_env_id, c->row_ptr, c->row_t, c->row_env, c->states,
                       c->eps_p, c->xi, c->y_last, gated, stream, R_cap, &mod_started)))
    return rc;
  if ((rc = verify_impl(c, B, R_cap, c->row_ptr, c->row_t, c->row_env, c->states, c->eps_q, true, stream, mod_started)))
    return rc;
  // x and t are overwritten in place: the acceptance kernel reads only the round's own buffers
  return accept_impl(c, B, c->row_ptr, c->row_t, d_env_id, d_sigma_scale, d_lambda, c->states, c->eps_p, c->eps_q, c->xi,
                     c->y_last, d_x, d_t, d_n_accept ? d_n_accept : c->n_acc, d_n_advanced ? d_n_advanced : c->n_adv,
                     nullptr, nullptr, nullptr, gated ? (const int32_t*)c->n_draft : nullptr, stream);
}

int tsdp_round(tsdp_ctx* c, int B, float* d_x, int32_t* d_t, const int32_t* d_K, const float* d_sigma_scale,
               const int32_t* d_env_id, int32_t* d_n_accept, int32_t* d_n_advanced, void* stream) {
  return round_impl(c, B, d_x, d_t, d_K, d_sigma_scale, d_env_id, nullptr, d_n_accept, d_n_advanced, false, stream);
}

int tsdp_round_threshold(tsdp_ctx* c, int B, float* d_x, int32_t* d_t, const int32_t* d_K, const float* d_sigma_scale,
                         const int32_t* d_env_id, const float* d_lambda, int32_t* d_n_accept, int32_t* d_n_advanced,
                         void* stream) {
  if (c && B > 0 && !d_lambda) return fail(c, TSDP_E_INVAL, "d_lambda is null");
  return round_impl(c, B, d_x, d_t, d_K, d_sigma_scale, d_env_id, d_lambda, d_n_accept, d_n_advanced, false, stream);
}

static int ensure_chain_buffers(tsdp_ctx* c) {
  int rc;
  if ((rc = ensure_round_buffers(c))) return rc;
  if (!c->live && (rc = dev_alloc(c, &c->live, 1))) return rc;
  if (!c->K_sel) {
    if ((rc = dev_alloc(c, &c->K_sel, (size_t)c->cfg.B_max))) return rc;
    if ((rc = dev_alloc(c, &c->s_sel, (size_t)c->cfg.B_max))) return rc;
    if ((rc = dev_alloc(c, &c->lam_sel, (size_t)c->cfg.B_max))) return rc;
  }
  return TSDP_OK;
}

// host_checked: rounds are enqueued until the number of running environments, read back every check_every rounds,
// is zero (or max_rounds is reached).  Otherwise exactly max_rounds rounds are enqueued and nothing is read back:
// the kernels of a round return at once when the round's row table is empty (every environment has finished).
static int chain_impl(tsdp_ctx* c, int B, float* d_x, int32_t* d_t, const int32_t* d_K, const float* d_sigma_scale,
                      const int32_t* d_env_id, const float* d_lambda, bool staged, int t_hi, int t_lo, int max_rounds,
                      int check_every, bool host_checked, int32_t* d_tot_accept, int32_t* d_tot_drafts,
                      int32_t* d_tot_rounds, int32_t* h_rounds, int32_t* d_rounds_run, void* stream) {
  int rc = check_ready(c, B, true);
  if (rc) return rc;
  if (h_rounds) *h_rounds = 0;
  if (!host_checked && max_rounds < 0) return fail(c, TSDP_E_INVAL, "n_rounds must not be negative");
  hipStream_t s = (hipStream_t)stream;
  if (d_rounds_run) hipLaunchKernelGGL(k_fill_i32, dim3(1), dim3(1), 0, s, d_rounds_run, 1, 0);
  if (B == 0) return TSDP_OK;
  if (!d_x || !d_t || !d_K || !d_sigma_scale) return fail(c, TSDP_E_INVAL, "null pointer passed to tsdp_chain");
  if (host_checked && (max_rounds < 1 || check_every < 1))
    return fail(c, TSDP_E_INVAL, "max_rounds and check_every must be positive");
  if (staged && !(t_hi >= t_lo && t_lo >= 0)) return fail(c, TSDP_E_INVAL, "stage bounds must satisfy t_hi >= t_lo >= 0");
  if ((rc = ensure_chain_buffers(c))) return rc;
  const dim3 gb((B + 255) / 256), blk(256);
  for (int32_t* p : {d_tot_accept, d_tot_drafts, d_tot_rounds})
    if (p) hipLaunchKernelGGL(k_fill_i32, gb, blk, 0, s, p, B, 0);
  int rounds = 0;
  while (rounds < max_rounds) {
    if (staged) {
      // the round's K, sigma scale and threshold are those of the stage each environment is in now
      hipLaunchKernelGGL(k_stage_select, gb, blk, 0, s, B, (const int32_t*)d_t, t_hi, t_lo, d_K, d_sigma_scale, d_lambda,
                         c->K_sel, c->s_sel, c->lam_sel);
      rc = round_impl(c, B, d_x, d_t, c->K_sel, c->s_sel, d_env_id, d_lambda ? c->lam_sel : nullptr, c->n_acc, c->n_adv,
                      !host_checked, stream);
    } else {
      rc = round_impl(c, B, d_x, d_t, d_K, d_sigma_scale, d_env_id, d_lambda, c->n_acc, c->n_adv, !host_checked, stream);
    }
    if (rc) return rc;
    ++rounds;
    if (host_checked) hipLaunchKernelGGL(k_fill_i32, dim3(1), dim3(1), 0, s, c->live, 1, 0);
    hipLaunchKernelGGL(k_chain_accum, gb, blk, 0, s, B, (const int32_t*)d_t, (const int32_t*)c->K_eff,
                       (const int32_t*)c->n_acc, (const int32_t*)c->n_adv, (const int32_t*)c->row_ptr, d_tot_accept,
                       d_tot_drafts, d_tot_rounds, host_checked ? c->live : nullptr, d_rounds_run);
    if (host_checked && (rounds % check_every == 0 || rounds == max_rounds)) {
      int32_t live = 0;
      HIPCHK(c, hipMemcpyAsync(&live, c->live, sizeof(int32_t), hipMemcpyDeviceToHost, s));
      HIPCHK(c, hipStreamSynchronize(s));
      if (live == 0) break;
    }
  }
  if (h_rounds) *h_rounds = rounds;
  HIPCHK(c, hipGetLastError());
  return TSDP_OK;
}

int tsdp_chain(tsdp_ctx* c, int B, float* d_x, int32_t* d_t, const int32_t* d_K, const float* d_sigma_scale,
               const int32_t* d_env_id, const float* d_lambda, int max_rounds, int check_every, int32_t* d_tot_accept,
               int32_t* d_tot_drafts, int32_t* d_tot_rounds, int32_t* h_rounds, void* stream) {
  return chain_impl(c, B, d_x, d_t, d_K, d_sigma_scale, d_env_id, d_lambda, false, 0, 0, max_rounds, check_every, true,
                    d_tot_accept, d_tot_drafts, d_tot_rounds, h_rounds, nullptr, stream);
}

int tsdp_chain_staged(tsdp_ctx* c, int B, float* d_x, int32_t* d_t, const int32_t* d_K3, const float* d_sigma_scale3,
                      const float* d_lambda3, int t_hi, int t_lo, const int32_t* d_env_id, int max_rounds, int check_every,
                      int32_t* d_tot_accept, int32_t* d_tot_drafts, int32_t* d_tot_rounds, int32_t* h_rounds, void* stream) {
  return chain_impl(c, B, d_x, d_t, d_K3, d_sigma_scale3, d_env_id, d_lambda3, true, t_hi, t_lo, max_rounds, check_every,
                    true, d_tot_accept, d_tot_drafts, d_tot_rounds, h_rounds, nullptr, stream);
}

int tsdp_chain_enqueue(tsdp_ctx* c, int B, float* d_x, int32_t* d_t, const int32_t* d_K, const float* d_sigma_scale,
                       const float* d_lambda, int staged, int t_hi, int t_lo, const int32_t* d_env_id, int n_rounds,
                       int32_t* d_tot_accept, int32_t* d_tot_drafts, int32_t* d_tot_rounds, int32_t* d_rounds_run,
                       void* stream) {
  return chain_impl(c, B, d_x, d_t, d_K, d_sigma_scale, d_env_id, d_lambda, staged != 0, t_hi, t_lo, n_rounds, 0, false,
                    d_tot_accept, d_tot_drafts, d_tot_rounds, nullptr, d_rounds_run, stream);
}

int tsdp_prepare(tsdp_ctx* c) {
  if (!c) return TSDP_E_INVAL;
  if (!c->net[0].loaded || !c->net[1].loaded) return fail(c, TSDP_E_STATE, "weights of both networks must be loaded");
  int rc;
  if ((rc = ensure_workspace(c))) return rc;
  if ((rc = ensure_chain_buffers(c))) return rc;
  if (!c->loss_partial && (rc = dev_alloc(c, &c->loss_partial, 2 * ((rows_max(c->cfg) + 15) / 16) + 2))) return rc;
  // the launch attributes of the fused kernels (dynamic LDS size): a launch over zero rows sets them and enqueues nothing
  FusedIO io{};
  DraftIO dio{};
  Net& bn = c->net[0];
  if (bn.fused) {
    if (bn.fused_verify) HIPCHK(c, bn.fused_verify(bn.fnet, io, c->cfg.A, 0, nullptr));
    if (bn.fused_verify_few) HIPCHK(c, bn.fused_verify_few(bn.fnet, io, c->cfg.A, 0, nullptr));
  }
  Net& dn = c->net[1];
  if (dn.fused) {                                     // the tile variants tsdp_draft may pick (those that fit the LDS)
    if (fused_draft_lds(dn, c->cfg, dn.draft_rpt_small) <= 160 * 1024)
      HIPCHK(c, dn.fused_draft_small(dn.fnet, dio, c->cfg.A, nullptr));
    if (fused_draft_lds(dn, c->cfg, dn.draft_rpt_big) <= 160 * 1024)
      HIPCHK(c, dn.fused_draft_big(dn.fnet, dio, c->cfg.A, nullptr));
  }
  return TSDP_OK;
}

// partial: room for 2 * ceil(R / 16) doubles; every entry that is read is written first by the same call
static int distill_launch(tsdp_ctx* c, int R, const int32_t* d_row_t, const float* d_states, const float* d_eps_p,
                          const float* d_eps_q, float lambda1, float lambda2, double* partial, double* d_loss, hipStream_t s) {
  const int parts = (R + 15) / 16;
  if (parts > 0) {
    if (c->cfg.clip_x0)
      hipLaunchKernelGGL(k_distill_partial<true>, dim3(parts), dim3(256), 0, s, R, c->D, d_row_t, d_states, d_eps_p, d_eps_q,
                         c->tb, c->cfg.clip_val, partial);
    else
      hipLaunchKernelGGL(k_distill_partial<false>, dim3(parts), dim3(256), 0, s, R, c->D, d_row_t, d_states, d_eps_p, d_eps_q,
                         c->tb, c->cfg.clip_val, partial);
  }
  hipLaunchKernelGGL(k_distill_final, dim3(1), dim3(256), 0, s, parts, R, d_row_t, (const double*)partial, lambda1,
                     lambda2, d_loss);
  HIPCHK(c, hipGetLastError());
  return TSDP_OK;
}

int tsdp_distill_loss(tsdp_ctx* c, int R, const int32_t* d_row_t, const float* d_states, const float* d_eps_p,
                      const float* d_eps_q, float lambda1, float lambda2, double* d_loss, void* stream) {
  if (!c) return TSDP_E_INVAL;
  if (R < 0 || (size_t)R > rows_max(c->cfg)) return fail(c, TSDP_E_SHAPE, "R outside 0..B_max*(K_max+bonus_row)");
  if (!d_loss || (R > 0 && (!d_row_t || !d_states || !d_eps_p || !d_eps_q)))
    return fail(c, TSDP_E_INVAL, "null pointer passed to tsdp_distill_loss");
  if (!c->loss_partial) {
    int rc = dev_alloc(c, &c->loss_partial, 2 * ((rows_max(c->cfg) + 15) / 16) + 2);
    if (rc) return rc;
  }
  return distill_launch(c, R, d_row_t, d_states, d_eps_p, d_eps_q, lambda1, lambda2, c->loss_partial, d_loss,
                        (hipStream_t)stream);
}

int tsdp_distill_loss_noalloc(tsdp_ctx* c, int R, const int32_t* d_row_t, const float* d_states, const float* d_eps_p,
                              const float* d_eps_q, float lambda1, float lambda2, double* d_loss, void* stream) {
  if (!c) return TSDP_E_INVAL;
  if (R < 0 || R > NOALLOC_MAX_ROWS)
    return fail(c, TSDP_E_SHAPE, "tsdp_distill_loss_noalloc: R outside 0.." + std::to_string(NOALLOC_MAX_ROWS) +
                                     " (the size of the static scratch)");
  if (!d_loss || (R > 0 && (!d_row_t || !d_states || !d_eps_p || !d_eps_q)))
    return fail(c, TSDP_E_INVAL, "null pointer passed to tsdp_distill_loss_noalloc");
  int dev = -1;
  HIPCHK(c, hipGetDevice(&dev));
  if (dev != c->device || !g_scratch_ptr[dev])
    return fail(c, TSDP_E_STATE, "tsdp_distill_loss_noalloc must run with the context's device current");
  return distill_launch(c, R, d_row_t, d_states, d_eps_p, d_eps_q, lambda1, lambda2, g_scratch_ptr[dev], d_loss,
                        (hipStream_t)stream);
}

int tsdp_status(tsdp_ctx* c, void* stream, int32_t* h_status) {
  if (!c || !h_status) return TSDP_E_INVAL;
  hipStream_t s = (hipStream_t)stream;
  HIPCHK(c, hipMemcpyAsync(h_status, c->status, sizeof(int32_t), hipMemcpyDeviceToHost, s));
  HIPCHK(c, hipStreamSynchronize(s));
  // cleared with a tiny fill kernel-free path: a synchronous memset outside any capture
  HIPCHK(c, hipMemset(c->status, 0, sizeof(int32_t)));
  return TSDP_OK;
}

int tsdp_kernel_timing(tsdp_ctx* c, int enable) {
  if (!c) return TSDP_E_INVAL;
  if (enable && !c->ev[0][0]) {
    for (auto& st : c->ev)
      for (auto& e : st) HIPCHK(c, hipEventCreate(&e));
  }
  c->timing = enable != 0;
  c->timing_mask = enable <= 1 ? 15 : (enable >> 1) & 15;
  for (bool& u : c->ev_used) u = false;
  return TSDP_OK;
}

int tsdp_kernel_ms(tsdp_ctx* c, int stage, float* h_ms) {
  if (!c || !h_ms || stage < 0 || stage > 3) return TSDP_E_INVAL;
  if (!c->ev[0][0] || !c->ev_used[stage]) return fail(c, TSDP_E_STATE, "no timed launch of that stage since timing was enabled");
  HIPCHK(c, hipEventSynchronize(c->ev[stage][1]));
  HIPCHK(c, hipEventElapsedTime(h_ms, c->ev[stage][0], c->ev[stage][1]));
  return TSDP_OK;
}

const char* tsdp_path_name(const tsdp_ctx* c, int which) {
  if (!c || which < 0 || which > 1) return "";
  return c->net[which].path;
}

const char* tsdp_last_error(const tsdp_ctx* c) { return c ? c->err.c_str() : "null context"; }

}  // extern "C"
