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
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t bf16_rne(float x) {
  uint32_t u = __float_as_uint(x);
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}

__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
  return bf16_rne(lo) | (bf16_rne(hi) << 16);
}

// One wavefront per token.  The token's local slots are compacted into a wave-uniform bit mask,
// walked in ascending j (the summation order is fixed).  A lane owns 16 bytes of the SOURCE row
// per step (4 fp32 or 8 bf16 values), so every load instruction of the wavefront covers 1 KB of
// contiguous memory; per slot, UNROLL such loads are issued before the accumulators are touched,
// so that a token with a single local slot (the common case after top-k over many ranks) still
// has UNROLL independent loads in flight per lane.  The host picks UNROLL so that one pass covers
// the whole row when it can (up to 32 loads per lane): measured at d = 6144 with fp32 rows,
// 12 loads per lane and two passes give 5.49 TB/s, 24 loads and one pass 5.64 TB/s.  Rows are read once and Y is written once:
// both are marked non-temporal.
template <bool YP_BF16, int UNROLL>
__global__ __launch_bounds__(BLOCK) void combine_kernel(const void* __restrict__ Yp,
                                                        const int* __restrict__ inv,
                                                        const float* __restrict__ w, int T, int k,
                                                        int d, int R_cap, void* __restrict__ Y) {
  constexpr int PER = YP_BF16 ? 8 : 4;   // values per lane and load
  const int nchunk = d / PER;
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
  const long long t = (long long)blockIdx.x * WAVES + wave;
  if (t >= T) return;
  int my_row = -1;
  float my_w = 0.f;
  if (lane < k) {
    my_row = inv[t * k + lane];
    my_w = w[t * k + lane];
    if (my_row >= R_cap) my_row = -1;   // a row past the capacity was never computed: not local
  }
  const unsigned long long local = __ballot(my_row >= 0);
  if (local == 0) {
    // no local slot (most tokens of a rank's share): the row is +0, written with 16-byte stores
    const int n16 = d / 8;
    u32x4* row = (u32x4*)Y + t * n16;
    for (int c = lane; c < n16; c += 64) __builtin_nontemporal_store(u32x4{0u, 0u, 0u, 0u}, row + c);
    return;
  }
  for (int c0 = 0; c0 < nchunk; c0 += 64 * UNROLL) {
    float acc[UNROLL][PER];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u)
#pragma unroll
      for (int i = 0; i < PER; ++i) acc[u][i] = 0.f;
    for (unsigned long long m = local; m; m &= m - 1) {
      const int j = __builtin_ctzll(m);
      const int r = __builtin_amdgcn_readlane(my_row, j);
      const float wj = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(my_w), j));
      if (YP_BF16) {
        const u32x4* row = (const u32x4*)Yp + (long long)r * nchunk;
        u32x4 p[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
          const int c = c0 + u * 64 + lane;
          p[u] = c < nchunk ? __builtin_nontemporal_load(row + c) : u32x4{0, 0, 0, 0};
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            acc[u][2 * i] = fmaf(wj, __uint_as_float(p[u][i] << 16), acc[u][2 * i]);
            acc[u][2 * i + 1] = fmaf(wj, __uint_as_float(p[u][i] & 0xffff0000u), acc[u][2 * i + 1]);
          }
      } else {
        const f32x4* row = (const f32x4*)Yp + (long long)r * nchunk;
        f32x4 p[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
          const int c = c0 + u * 64 + lane;
          p[u] = c < nchunk ? __builtin_nontemporal_load(row + c) : f32x4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u)
#pragma unroll
          for (int i = 0; i < 4; ++i) acc[u][i] = fmaf(wj, p[u][i], acc[u][i]);
      }
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const int c = c0 + u * 64 + lane;
      if (c < nchunk) {
        if (YP_BF16) {
          u32x4 o;
#pragma unroll
          for (int i = 0; i < 4; ++i) o[i] = pack2(acc[u][2 * i], acc[u][2 * i + 1]);
          __builtin_nontemporal_store(o, (u32x4*)Y + t * nchunk + c);
        } else {
          u32x2 o;
          o[0] = pack2(acc[u][0], acc[u][1]);
          o[1] = pack2(acc[u][2], acc[u][3]);
          __builtin_nontemporal_store(o, (u32x2*)Y + t * nchunk + c);
        }
      }
    }
  }
}

}  // namespace

extern "C" int32_t feplb_unpermute_combine(const void* Yp, int32_t yp_dtype, int32_t R_cap, const int32_t* inv,
                                           const float* topk_w, int32_t T, int32_t k, int32_t d,
                                           void* Y, void* stream) {
  FEPLB_REQUIRE(T >= 0 && k >= 1 && d >= 0 && R_cap >= 0, FEPLB_EINVAL, "combine: negative size");
  FEPLB_REQUIRE(k <= FEPLB_MAX_TOPK, FEPLB_ESHAPE, "combine: k=%d above %d", k, FEPLB_MAX_TOPK);
  FEPLB_REQUIRE(d % 8 == 0, FEPLB_ESHAPE, "combine: d=%d not a multiple of 8", d);
  FEPLB_REQUIRE(yp_dtype == FEPLB_F32 || yp_dtype == FEPLB_BF16, FEPLB_EINVAL,
                "combine: unknown yp_dtype %d", yp_dtype);
  if (T == 0 || d == 0) return FEPLB_OK;
  FEPLB_REQUIRE(inv && topk_w && Y, FEPLB_EINVAL, "combine: null buffer");
  FEPLB_REQUIRE(feplb::aligned16(Y) && feplb::aligned16(Yp), FEPLB_EALIGN,
                "combine: Y/Yp not 16-byte aligned");
  FEPLB_REQUIRE(Yp || R_cap == 0, FEPLB_EINVAL, "combine: null Yp with R_cap=%d", R_cap);
  hipStream_t s = (hipStream_t)stream;
  const int blocks = (T + WAVES - 1) / WAVES;
  const int per_lane = (d / (yp_dtype == FEPLB_BF16 ? 8 : 4) + 63) / 64;   // 16-byte loads per lane and row
#define FEPLB_COMBINE(BF, U) \
  hipLaunchKernelGGL((combine_kernel<BF, U>), dim3(blocks), dim3(BLOCK), 0, s, Yp, inv, topk_w, T, k, d, R_cap, Y)
  if (yp_dtype == FEPLB_BF16) {
    if (per_lane <= 4) FEPLB_COMBINE(true, 4);
    else if (per_lane <= 8) FEPLB_COMBINE(true, 8);
    else if (per_lane <= 12) FEPLB_COMBINE(true, 12);
    else FEPLB_COMBINE(true, 16);
  } else {
    if (per_lane <= 8) FEPLB_COMBINE(false, 8);
    else if (per_lane <= 16) FEPLB_COMBINE(false, 16);
    else if (per_lane <= 24) FEPLB_COMBINE(false, 24);
    else FEPLB_COMBINE(false, 32);
  }
#undef FEPLB_COMBINE
  FEPLB_LAUNCH_CHECK("combine_kernel");
  return FEPLB_OK;
}
