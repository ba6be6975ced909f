// Un-permute and weighted top-k combine (paper Section 2.3: the Combine phase
// hands expert outputs back to their tokens; this is the part of it that runs
// on the computing rank): Y[t,:] = sum_j w[t,j] * Yp[inv[t,j],:] over the local
// slots of token t, fp32 sum in ascending j, one round-to-nearest-even to bf16.
// Pure HBM traffic: R*d*sizeof(Yp) bytes in, T*d*2 out.  One wavefront per
// token, 16 bytes of output per lane and step.
#include "common.h"

namespace {

constexpr int WAVES = 4;
constexpr int BLOCK = WAVES * 64;

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint32_t bf16_rne(float x) {
  uint32_t u = __float_as_uint(x);
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}

__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
  return bf16_rne(lo) | (bf16_rne(hi) << 16);
}

template <bool YP_BF16>
__global__ __launch_bounds__(BLOCK) void combine_kernel(const void* __restrict__ Yp,
                                                        const int* __restrict__ inv,
                                                        const float* __restrict__ w, int T, int k,
                                                        int nvec, u32x4* __restrict__ Y) {
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
  const long long t = (long long)blockIdx.x * WAVES + wave;
  if (t >= T) return;
  int my_row = -1;
  float my_w = 0.f;
  if (lane < k) {
    my_row = inv[t * k + lane];
    my_w = w[t * k + lane];
  }
  u32x4* out = Y + t * nvec;
  // the loop bound is uniform so that every lane takes part in the broadcasts
  for (int v0 = 0; v0 < nvec; v0 += 64) {
    const int v = v0 + lane;
    const bool live = v < nvec;
    float acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = 0.f;
    for (int j = 0; j < k; ++j) {
      const int r = __shfl(my_row, j, 64);
      if (r < 0) continue;  // uniform across the wave
      const float wj = __shfl(my_w, j, 64);
      if (!live) continue;
      if (YP_BF16) {
        const u32x4 p = ((const u32x4*)Yp)[(long long)r * nvec + v];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          acc[2 * i] = fmaf(wj, __uint_as_float(p[i] << 16), acc[2 * i]);
          acc[2 * i + 1] = fmaf(wj, __uint_as_float(p[i] & 0xffff0000u), acc[2 * i + 1]);
        }
      } else {
        const f32x4* row = (const f32x4*)Yp + ((long long)r * nvec + v) * 2;
        const f32x4 p0 = row[0], p1 = row[1];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          acc[i] = fmaf(wj, p0[i], acc[i]);
          acc[4 + i] = fmaf(wj, p1[i], acc[4 + i]);
        }
      }
    }
    u32x4 o;
    o[0] = pack2(acc[0], acc[1]);
    o[1] = pack2(acc[2], acc[3]);
    o[2] = pack2(acc[4], acc[5]);
    o[3] = pack2(acc[6], acc[7]);
    if (live) out[v] = o;
  }
}

}  // namespace

extern "C" int32_t feplb_unpermute_combine(const void* Yp, int32_t yp_dtype, const int32_t* inv,
                                           const float* topk_w, int32_t T, int32_t k, int32_t d,
                                           void* Y, void* stream) {
  FEPLB_REQUIRE(T >= 0 && k >= 1 && d >= 0, FEPLB_EINVAL, "combine: negative size");
  FEPLB_REQUIRE(k <= FEPLB_MAX_TOPK, FEPLB_ESHAPE, "combine: k=%d above %d", k, FEPLB_MAX_TOPK);
  FEPLB_REQUIRE(d % 8 == 0, FEPLB_ESHAPE, "combine: d=%d not a multiple of 8", d);
  FEPLB_REQUIRE(yp_dtype == FEPLB_F32 || yp_dtype == FEPLB_BF16, FEPLB_EINVAL,
                "combine: unknown yp_dtype %d", yp_dtype);
  if (T == 0 || d == 0) return FEPLB_OK;
  FEPLB_REQUIRE(inv && topk_w && Y, FEPLB_EINVAL, "combine: null buffer");
  FEPLB_REQUIRE(feplb::aligned16(Y) && feplb::aligned16(Yp), FEPLB_EALIGN,
                "combine: Y/Yp not 16-byte aligned");
  // Yp may be NULL only if no assignment is local; the kernel then never reads it.
  hipStream_t s = (hipStream_t)stream;
  const int blocks = (T + WAVES - 1) / WAVES;
  if (yp_dtype == FEPLB_BF16)
    hipLaunchKernelGGL(combine_kernel<true>, dim3(blocks), dim3(BLOCK), 0, s, Yp, inv, topk_w, T,
                       k, d / 8, (u32x4*)Y);
  else
    hipLaunchKernelGGL(combine_kernel<false>, dim3(blocks), dim3(BLOCK), 0, s, Yp, inv, topk_w, T,
                       k, d / 8, (u32x4*)Y);
  FEPLB_LAUNCH_CHECK("combine_kernel");
  return FEPLB_OK;
}
