// Gate of the failure-remapped MoE layer: router logits, failure-masked (group-limited) top-k,
// renormalised weights and the logical->physical replica remap.
//
// Paper: Sec. 2.1 (gating scores, top-k), Sec. 3.4 "Missing experts" and Sec. 4.2 (experts with
// no replica left are masked to -inf immediately before the top-k), Sec. 3.4 "Redundant experts"
// (the logical-to-physical map decides which replica serves a token).
#include "gemm_bf16.hpp"
#include "gemm_f32.hpp"

namespace revive {

namespace {

// Ordering of candidates: larger key first, equal keys by lower expert id.
__device__ __forceinline__ bool better(float ka, int ea, float kb, int eb) { return ka > kb || (ka == kb && ea < eb); }

struct RouteParams {
  const float* logits;
  const int32_t* l2p_count;
  const int32_t* l2p_table;
  int32_t* topk_logical;
  float* topk_weight;
  int32_t* topk_phys;
  int T, E, k, max_replicas, score_fn, n_group, topk_group;
  long long t_offset;  // index of token 0 within the whole batch
  float route_scale;
};

// One wavefront per token.  Lane l holds the logits of experts l, l+64, l+128, ... (VALS of them);
// a masked or excluded expert's key is -inf.  Expert order is decided on the fp32 logits
// themselves (softmax and sigmoid are increasing, so this is the order of the scores); group
// scores, which add two scores, and the output weights are evaluated in fp64.
// GROUPED variants hold the group scores in registers (n_group <= 8 or <= 32).
template <int VALS, int MAXG>
__global__ __launch_bounds__(256) void route_topk_kernel(RouteParams p) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= p.T) return;  // whole wavefront leaves together
  const float NEG = -__builtin_inff();

  float key[VALS];
  const float* row = p.logits + static_cast<int64_t>(t) * p.E;
  float vmax = NEG;  // largest live logit of the row: common shift of the exponentials (the best chosen score is exactly 1)
#pragma unroll
  for (int i = 0; i < VALS; ++i) {
    const int e = lane + 64 * i;
    float z = NEG;
    if (e < p.E) {
      z = row[e];
      if (p.l2p_count[e] <= 0) z = NEG;  // failure mask
      vmax = fmaxf(vmax, z);
    }
    key[i] = z;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) vmax = fmaxf(vmax, __shfl_xor(vmax, o));
  const double shift = static_cast<double>(vmax);

  auto score64 = [&](float z) -> double {  // unnormalised gating score of a live expert
    const double zd = static_cast<double>(z);
    return p.score_fn == REVIVE_SCORE_SIGMOID ? 1.0 / (1.0 + exp(-zd)) : exp(zd - shift);
  };

  if (MAXG > 1) {
    // Group score = sum of the two best live scores of the group (one if only one is live, -inf
    // if none).  A wave-wide top-2 per group finds the two logits; lane g then evaluates group
    // g's score in fp64 and every lane ranks it against the others through shuffles.
    const int gsz = p.E / p.n_group;
    float top1 = NEG, top2 = NEG;  // lane g keeps group g's two best keys
#pragma unroll 1
    for (int g = 0; g < p.n_group; ++g) {
      float m1 = NEG, m2 = NEG;
#pragma unroll
      for (int i = 0; i < VALS; ++i) {
        const int e = lane + 64 * i;
        const float z = (e < p.E && e / gsz == g) ? key[i] : NEG;
        if (z > m1) { m2 = m1; m1 = z; } else if (z > m2) { m2 = z; }
      }
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) {
        const float o1 = __shfl_xor(m1, o), o2 = __shfl_xor(m2, o);
        const float hi = fmaxf(m1, o1);
        const float lo = fmaxf(fminf(m1, o1), fmaxf(m2, o2));
        m1 = hi;
        m2 = lo;
      }
      if (lane == g) { top1 = m1; top2 = m2; }
    }
    double gs = -__builtin_inf();
    if (lane < p.n_group && top1 > NEG) {
      gs = score64(top1);
      if (top2 > NEG) gs += score64(top2);
    }
    // rank of my group among all groups (better score first, ties to the lower group id)
    int rank = 0;
#pragma unroll
    for (int h = 0; h < MAXG; ++h) {
      const double o = __shfl(gs, h);
      if (h < p.n_group) rank += (o > gs) || (o == gs && h < lane);
    }
    const unsigned long long kept = __ballot(lane < p.n_group && rank < p.topk_group);
#pragma unroll
    for (int i = 0; i < VALS; ++i) {
      const int e = lane + 64 * i;
      if (e < p.E && !((kept >> (e / gsz)) & 1ull)) key[i] = NEG;  // expert of a dropped group
    }
  }

  // k rounds of wave-wide arg-max; the winner of round j lands in lane j.
  int my_e = -1;
  float my_z = 0.f;
  for (int j = 0; j < p.k; ++j) {
    float bk = NEG;
    int be = 0x7fffffff;
#pragma unroll
    for (int i = 0; i < VALS; ++i) {
      const int e = lane + 64 * i;
      if (e < p.E && better(key[i], e, bk, be)) { bk = key[i]; be = e; }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      const float ok = __shfl_xor(bk, o);
      const int oe = __shfl_xor(be, o);
      if (better(ok, oe, bk, be)) { bk = ok; be = oe; }
    }
    if ((be & 63) == lane) {
#pragma unroll
      for (int i = 0; i < VALS; ++i)
        if (i == (be >> 6)) key[i] = NEG;
    }
    if (lane == j) { my_e = be; my_z = bk; }
  }

  // weights: score of the chosen expert over the sum of the chosen scores
  double s = (lane < p.k) ? score64(my_z) : 0.0;
  double sum = s;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
  if (lane < p.k) {
    const int64_t o = static_cast<int64_t>(t) * p.k + lane;
    const int c = p.l2p_count[my_e];
    p.topk_logical[o] = my_e;
    p.topk_weight[o] = static_cast<float>(s / sum * static_cast<double>(p.route_scale));
    // replica of this token: the (batch index of t mod count)-th surviving slot, ascending slot id
    p.topk_phys[o] = c > 0 ? p.l2p_table[my_e * p.max_replicas + static_cast<int>((p.t_offset + t) % c)] : -1;
  }
}

// Router logits for a small router (E <= 128) without LDS staging.  A workgroup of KS wavefronts
// owns 32 tokens and NTN tiles of 32 experts (blockIdx.y selects which); wavefront w multiplies the w-th slice of the hidden dimension
// with operands loaded straight from global memory in MFMA fragment order, and the KS partial
// sums are added in wavefront order through LDS (a fixed order: the result is deterministic).
// Per 64-wide K block a lane reads 64 contiguous bytes of its token row (lanes l and l+32 cover
// one 128-byte line), so x is streamed once in full lines; the router matrix stays in L2.
// Up to three K blocks are in flight per wavefront.
template <int NTN, int KS>
__global__ __launch_bounds__(64 * KS) void router_direct_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ w,
                                                                float* __restrict__ logits, int T, int E, int H) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  float* part = reinterpret_cast<float*>(smem);  // [KS-1][NTN][16][64]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane & 31, half = lane >> 5;
  const int row0 = blockIdx.x * 32;
  const int e0 = blockIdx.y * (NTN * 32);  // first expert of this workgroup
  const int kq = H / KS;  // K range of one wavefront, a multiple of 64
  const int64_t koff = static_cast<int64_t>(wave) * kq + half * 32;
  const unsigned char* a_ptr = reinterpret_cast<const unsigned char*>(x + static_cast<int64_t>(min(row0 + r, T - 1)) * H + koff);
  const unsigned char* b_ptr[NTN];
#pragma unroll
  for (int tn = 0; tn < NTN; ++tn)
    b_ptr[tn] = reinterpret_cast<const unsigned char*>(w + static_cast<int64_t>(min(e0 + tn * 32 + r, E - 1)) * H + koff);

  f32x16 acc[NTN];
#pragma unroll
  for (int tn = 0; tn < NTN; ++tn)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[tn][i] = 0.f;

  struct Frags { u32x4 a[4]; u32x4 b[NTN][4]; };
  auto load = [&](int blk, Frags& f) {
    const int64_t o = static_cast<int64_t>(blk) * 128;  // 64 bf16
#pragma unroll
    for (int j = 0; j < 4; ++j) f.a[j] = load_global_16B(a_ptr + o + j * 16);
#pragma unroll
    for (int tn = 0; tn < NTN; ++tn)
#pragma unroll
      for (int j = 0; j < 4; ++j) f.b[tn][j] = load_global_16B(b_ptr[tn] + o + j * 16);
  };
  auto mac = [&](const Frags& f) {
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int tn = 0; tn < NTN; ++tn)
        acc[tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f.b[tn][j]), __builtin_bit_cast(bf16x8, f.a[j]),
                                                          acc[tn], 0, 0, 0);
  };
  const int n = kq >> 6;
  Frags f0, f1, f2;
  load(0, f0);
  if (n > 1) load(1, f1);
  if (NTN <= 2 && n > 2) load(2, f2);
  if (NTN <= 2) {
    for (int blk = 0; blk < n; blk += 3) {
      mac(f0);
      if (blk + 3 < n) load(blk + 3, f0);
      if (blk + 1 < n) { mac(f1); if (blk + 4 < n) load(blk + 4, f1); }
      if (blk + 2 < n) { mac(f2); if (blk + 5 < n) load(blk + 5, f2); }
    }
  } else {
    for (int blk = 0; blk < n; blk += 2) {
      mac(f0);
      if (blk + 2 < n) load(blk + 2, f0);
      if (blk + 1 < n) { mac(f1); if (blk + 3 < n) load(blk + 3, f1); }
    }
  }

  if (wave > 0) {
#pragma unroll
    for (int tn = 0; tn < NTN; ++tn)
#pragma unroll
      for (int i = 0; i < 16; ++i) part[(((wave - 1) * NTN + tn) * 16 + i) * 64 + lane] = acc[tn][i];
  }
  __syncthreads();
  if (wave == 0) {
    const int row = row0 + r;
#pragma unroll
    for (int tn = 0; tn < NTN; ++tn) {
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        float v = acc[tn][i];
        for (int ws = 0; ws < KS - 1; ++ws) v += part[((ws * NTN + tn) * 16 + i) * 64 + lane];
        acc[tn][i] = v;
      }
      if (row < T) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int col = e0 + tn * 32 + q * 8 + half * 4;
#pragma unroll
          for (int rr = 0; rr < 4; ++rr)
            if (col + rr < E) logits[static_cast<int64_t>(row) * E + col + rr] = acc[tn][q * 4 + rr];
        }
      }
    }
  }
}

template <int NTN, int KS>
int launch_router_direct(revive_ctx* ctx, const void* x, const void* w, float* logits, int T, hipStream_t stream) {
  constexpr size_t lds = static_cast<size_t>(KS - 1) * NTN * 16 * 64 * sizeof(float);
  auto kern = router_direct_kernel<NTN, KS>;
  REVIVE_HIP(ctx, allow_dynamic_lds(reinterpret_cast<const void*>(kern), lds));
  hipLaunchKernelGGL(kern, dim3(ceil_div(T, 32), ceil_div(ctx->cfg.E, NTN * 32)), dim3(64 * KS), lds, stream, static_cast<const uint16_t*>(x),
                     static_cast<const uint16_t*>(w), logits, T, ctx->cfg.E, ctx->cfg.H);
  return check_hip(ctx, hipGetLastError(), "router_direct launch");
}

}  // namespace

int launch_router_gemm(revive_ctx* ctx, const void* x, const void* w, float* logits, int T, hipStream_t stream) {
  const revive_config& c = ctx->cfg;
  KernelTimer timer(ctx, REVIVE_K_ROUTER_GEMM, stream);
  if (c.dtype == REVIVE_DTYPE_BF16 && c.E <= 128 && c.H % 256 == 0 &&
      static_cast<int64_t>(ceil_div(T, 32)) * c.E * c.H * 2 <= (128ll << 20)) {
    // small router: every 32-token workgroup re-reads its part of the router matrix from L2.  With few
    // token blocks every 32-expert tile gets a workgroup of its own (more workgroups, and less
    // to pull through one CU's L1), otherwise one workgroup serves all experts of its tokens.
    const bool ks8 = c.H % 512 == 0;
    const bool split_experts = ceil_div(T, 32) < 512;
    switch (split_experts ? 1 : ceil_div(c.E, 32)) {
      case 1: return ks8 ? launch_router_direct<1, 8>(ctx, x, w, logits, T, stream) : launch_router_direct<1, 4>(ctx, x, w, logits, T, stream);
      case 2: return ks8 ? launch_router_direct<2, 8>(ctx, x, w, logits, T, stream) : launch_router_direct<2, 4>(ctx, x, w, logits, T, stream);
      case 3: return launch_router_direct<3, 4>(ctx, x, w, logits, T, stream);
      default: return launch_router_direct<4, 4>(ctx, x, w, logits, T, stream);
    }
  }
  if (c.dtype == REVIVE_DTYPE_BF16) {
    GemmArgs a{};
    a.A = x; a.lda = c.H;
    a.B_tab = nullptr; a.B_one = w; a.ldb = c.H;
    a.C = logits; a.ldc = c.E;
    a.n_out = c.E; a.K = c.H;
    a.tiles = nullptr; a.tile_count = nullptr; a.M = T;
    if (static_cast<int64_t>(ceil_div(T, 128)) * ceil_div(c.E, 128) >= 512) {
      // enough tiles to fill the chip twice over: wider tiles read x fewer times
      a.n_col_tiles = ceil_div(c.E, 128);
      return launch_gemm_bf16<128, 128, 2, 2, EPI_F32, REVIVE_K_ROUTER_GEMM>(ctx, a, ceil_div(T, 128), stream);
    }
    constexpr int BM = 128, BN = 64;
    a.n_col_tiles = ceil_div(c.E, BN);
    return launch_gemm_bf16<BM, BN, 4, 1, EPI_F32, REVIVE_K_ROUTER_GEMM>(ctx, a, ceil_div(T, BM), stream);
  }
  GemmF32Args a{};
  a.A = static_cast<const float*>(x); a.lda = c.H;
  a.B_tab = nullptr; a.B_one = static_cast<const float*>(w); a.ldb = c.H;
  a.C = logits; a.ldc = c.E;
  a.n_out = c.E; a.K = c.H;
  a.tiles = nullptr; a.tile_count = nullptr; a.M = T;
  a.n_col_tiles = ceil_div(c.E, 64);
  return launch_gemm_f32<false>(ctx, a, ceil_div(T, kTileM_f32), stream);
}

int launch_route_topk(revive_ctx* ctx, const float* logits, int T, int32_t* topk_logical, float* topk_weight,
                      int32_t* topk_phys, hipStream_t stream) {
  const revive_config& c = ctx->cfg;
  RouteParams p{};
  p.logits = logits;
  p.l2p_count = ctx->d_l2p_count();
  p.l2p_table = ctx->d_l2p_table();
  p.topk_logical = topk_logical;
  p.topk_weight = topk_weight;
  p.topk_phys = topk_phys;
  p.T = T; p.E = c.E; p.k = c.k; p.max_replicas = c.max_replicas;
  p.score_fn = c.score_fn; p.n_group = c.n_group; p.topk_group = c.topk_group;
  p.route_scale = c.route_scale;
  p.t_offset = ctx->token_offset;
  KernelTimer timer(ctx, REVIVE_K_ROUTE_TOPK, stream);
  const dim3 grid(ceil_div(T, 4)), block(256);
  const int vals = ceil_div(c.E, 64);
#define REVIVE_ROUTE_LAUNCH(V)                                                                               \
  do {                                                                                                       \
    if (c.n_group <= 1) hipLaunchKernelGGL((route_topk_kernel<V, 1>), grid, block, 0, stream, p);            \
    else if (c.n_group <= 8) hipLaunchKernelGGL((route_topk_kernel<V, 8>), grid, block, 0, stream, p);       \
    else hipLaunchKernelGGL((route_topk_kernel<V, 32>), grid, block, 0, stream, p);                          \
  } while (0)
  if (vals <= 1) REVIVE_ROUTE_LAUNCH(1);
  else if (vals <= 2) REVIVE_ROUTE_LAUNCH(2);
  else if (vals <= 4) REVIVE_ROUTE_LAUNCH(4);
  else if (vals <= 6) REVIVE_ROUTE_LAUNCH(6);
  else REVIVE_ROUTE_LAUNCH(8);
#undef REVIVE_ROUTE_LAUNCH
  return check_hip(ctx, hipGetLastError(), "route_topk launch");
}

}  // namespace revive
