// Combine (E2A) of the failure-remapped MoE layer.
//
// Paper: Sec. 2.3 (combine aggregates the expert outputs back to the tokens using the gating
// scores).  out[t] = sum_j w[t, j] * y_perm[dst_row[t*k + j]] (+ y_shared[t]); fp32 accumulation
// in ascending j, the shared expert last, one rounding to the working type.
#include "ctx.hpp"

namespace revive {

namespace {

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }
// Two fp32 -> one word of two bf16 (round-to-nearest-even), one v_cvt_pk_bf16_f32.
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// Every routed row is read exactly once and every output word written once: both bypass the caches' retention
// (non-temporal), which leaves the caches to the kernels before and after.
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
__device__ __forceinline__ uint4 load_once(const uint4* p) {
  const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void store_once(uint4* p, uint4 o) {
  const u32x4 v = {o.x, o.y, o.z, o.w};
  __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(p));
}

// One workgroup per token, 16-byte words (8 bf16 or 4 fp32 per thread and step).
template <bool BF16>
__global__ __launch_bounds__(256) void combine_kernel(const uint4* __restrict__ y_perm, const int32_t* __restrict__ dst_row,
                                                      const float* __restrict__ topk_weight, const uint4* __restrict__ y_shared,
                                                      int k, int row_words, uint4* __restrict__ out) {
  __shared__ int rows[kMaxK];
  __shared__ float wts[kMaxK];
  const int t = blockIdx.x;
  if (threadIdx.x < k) {
    rows[threadIdx.x] = dst_row[static_cast<int64_t>(t) * k + threadIdx.x];
    wts[threadIdx.x] = topk_weight[static_cast<int64_t>(t) * k + threadIdx.x];
  }
  __syncthreads();
  for (int c = threadIdx.x; c < row_words; c += 256) {
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    uint4 sh = make_uint4(0, 0, 0, 0);
    if (y_shared) sh = y_shared[static_cast<int64_t>(t) * row_words + c];
    // the gathers of up to eight routed rows are issued together, then added in ascending j
    for (int j0 = 0; j0 < k; j0 += 8) {
      uint4 v[8];
      bool on[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int r = j0 + u < k ? rows[j0 + u] : -1;
        on[u] = r >= 0;
        v[u] = on[u] ? load_once(y_perm + static_cast<int64_t>(r) * row_words + c) : make_uint4(0, 0, 0, 0);
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        if (!on[u]) continue;
        const float w = wts[j0 + u];
        if (BF16) {
          acc[0] = fmaf(w, bf16_lo(v[u].x), acc[0]); acc[1] = fmaf(w, bf16_hi(v[u].x), acc[1]);
          acc[2] = fmaf(w, bf16_lo(v[u].y), acc[2]); acc[3] = fmaf(w, bf16_hi(v[u].y), acc[3]);
          acc[4] = fmaf(w, bf16_lo(v[u].z), acc[4]); acc[5] = fmaf(w, bf16_hi(v[u].z), acc[5]);
          acc[6] = fmaf(w, bf16_lo(v[u].w), acc[6]); acc[7] = fmaf(w, bf16_hi(v[u].w), acc[7]);
        } else {
          acc[0] = fmaf(w, __uint_as_float(v[u].x), acc[0]); acc[1] = fmaf(w, __uint_as_float(v[u].y), acc[1]);
          acc[2] = fmaf(w, __uint_as_float(v[u].z), acc[2]); acc[3] = fmaf(w, __uint_as_float(v[u].w), acc[3]);
        }
      }
    }
    if (y_shared) {
      const uint4 v = sh;
      if (BF16) {
        acc[0] += bf16_lo(v.x); acc[1] += bf16_hi(v.x); acc[2] += bf16_lo(v.y); acc[3] += bf16_hi(v.y);
        acc[4] += bf16_lo(v.z); acc[5] += bf16_hi(v.z); acc[6] += bf16_lo(v.w); acc[7] += bf16_hi(v.w);
      } else {
        acc[0] += __uint_as_float(v.x); acc[1] += __uint_as_float(v.y);
        acc[2] += __uint_as_float(v.z); acc[3] += __uint_as_float(v.w);
      }
    }
    uint4 o;
    if (BF16) {
      o.x = pack_bf16(acc[0], acc[1]);
      o.y = pack_bf16(acc[2], acc[3]);
      o.z = pack_bf16(acc[4], acc[5]);
      o.w = pack_bf16(acc[6], acc[7]);
    } else {
      o.x = __float_as_uint(acc[0]); o.y = __float_as_uint(acc[1]);
      o.z = __float_as_uint(acc[2]); o.w = __float_as_uint(acc[3]);
    }
    store_once(out + static_cast<int64_t>(t) * row_words + c, o);
  }
}

}  // namespace

int launch_combine(revive_ctx* ctx, const void* y_perm, const int32_t* dst_row, const float* topk_weight, const void* y_shared,
                   int T, void* out, hipStream_t stream) {
  const revive_config& c = ctx->cfg;
  const int row_words = static_cast<int>(c.H * ctx->elem / 16);
  KernelTimer timer(ctx, REVIVE_K_COMBINE, stream);
  if (c.dtype == REVIVE_DTYPE_BF16)
    hipLaunchKernelGGL(combine_kernel<true>, dim3(T), dim3(256), 0, stream, static_cast<const uint4*>(y_perm), dst_row,
                       topk_weight, static_cast<const uint4*>(y_shared), c.k, row_words, static_cast<uint4*>(out));
  else
    hipLaunchKernelGGL(combine_kernel<false>, dim3(T), dim3(256), 0, stream, static_cast<const uint4*>(y_perm), dst_row,
                       topk_weight, static_cast<const uint4*>(y_shared), c.k, row_words, static_cast<uint4*>(out));
  return check_hip(ctx, hipGetLastError(), "combine launch");
}

}  // namespace revive
