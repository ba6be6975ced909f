// Backward of the layer's memory-bound steps (paper Section 3.2 times the MoE layer's backward
// pass; Section 2.3 names the steps): the combine, whose gradient feeds the grouped FFN's
// backward, and the routing weights.  The row gather's backward, dX[t,:] = sum of the gradients
// of token t's copies, is feplb_unpermute_combine with unit weights and needs no kernel here.
//
//   combine:  Y[t,:] = sum_j w[t,j] Yp[inv[t,j],:]  =>  dYp[inv[t,j],:] = w[t,j] dY[t,:]  (bf16),
//             dw[t,j] = <dY[t,:], Yp[inv[t,j],:]>, 0 for a slot that is not local
//   router:   w = softmax of the k kept logits      =>  dz[ids_j] = w_j (dw_j - sum_i w_i dw_i)
#include "common.h"
#include "gemm_device.h"

namespace {
using feplb::dev::pack_bf16;

constexpr int WAVES = 4;
constexpr int BLOCK = WAVES * 64;

using feplb::dev::u32x4;
typedef float f32x4 __attribute__((ext_vector_type(4)));

// One wavefront per token; its local slots are walked in ascending j.  A lane owns 16 bytes of
// the gradient row per step (8 bf16 values): it reads them from dY[t,:] (re-read per local slot,
// from cache after the first), scales them into the slot's dYp row, and multiplies them with the
// matching 8 values of the slot's Yp row for the weight's gradient, reduced over the wavefront
// at the end of the row.  Yp is read once and dYp written once: both non-temporal.
template <bool YP_BF16, int UNROLL>
__global__ __launch_bounds__(BLOCK) void combine_backward_kernel(
    const u32x4* __restrict__ dY, const void* __restrict__ Yp, const int* __restrict__ inv,
    const float* __restrict__ w, int T, int k, int d, int R_cap, u32x4* __restrict__ dYp,
    float* __restrict__ dw) {
  const int nchunk = d / 8;
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
  const long long t = (long long)blockIdx.x * WAVES + wave;
  if (t >= T) return;
  int my_row = -1;
  float my_w = 0.f;
  if (lane < k) {
    my_row = inv[t * k + lane];
    my_w = w[t * k + lane];
    if (my_row >= R_cap) my_row = -1;   // a row past the capacity does not exist in Yp / dYp
    if (my_row < 0) dw[t * k + lane] = 0.f;
  }
  const u32x4* g_row = dY + t * nchunk;
  for (unsigned long long m = __ballot(my_row >= 0); m; m &= m - 1) {
    const int j = __builtin_ctzll(m);
    const long long r = __builtin_amdgcn_readlane(my_row, j);
    const float wj = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(my_w), j));
    float dot = 0.f;
    for (int c0 = 0; c0 < nchunk; c0 += 64 * UNROLL) {
      u32x4 g[UNROLL];
      f32x4 y0[UNROLL], y1[UNROLL];
      u32x4 yb[UNROLL];
#pragma unroll
      for (int u = 0; u < UNROLL; ++u) {
        const int c = c0 + u * 64 + lane;
        g[u] = u32x4{0, 0, 0, 0};
        y0[u] = y1[u] = f32x4{0.f, 0.f, 0.f, 0.f};
        yb[u] = u32x4{0, 0, 0, 0};
        if (c < nchunk) {
          g[u] = g_row[c];
          if (YP_BF16) {
            yb[u] = __builtin_nontemporal_load((const u32x4*)Yp + r * nchunk + c);
          } else {
            const f32x4* yr = (const f32x4*)Yp + (r * nchunk + c) * 2;
            y0[u] = __builtin_nontemporal_load(yr);
            y1[u] = __builtin_nontemporal_load(yr + 1);
          }
        }
      }
#pragma unroll
      for (int u = 0; u < UNROLL; ++u) {
        const int c = c0 + u * 64 + lane;
        float gv[8], yv[8];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          gv[2 * i] = __uint_as_float(g[u][i] << 16);
          gv[2 * i + 1] = __uint_as_float(g[u][i] & 0xffff0000u);
          if (YP_BF16) {
            yv[2 * i] = __uint_as_float(yb[u][i] << 16);
            yv[2 * i + 1] = __uint_as_float(yb[u][i] & 0xffff0000u);
          } else {
            yv[2 * i] = i < 2 ? y0[u][2 * i] : y1[u][2 * i - 4];
            yv[2 * i + 1] = i < 2 ? y0[u][2 * i + 1] : y1[u][2 * i - 3];
          }
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) dot = fmaf(gv[i], yv[i], dot);
        if (c < nchunk) {
          u32x4 o;
#pragma unroll
          for (int i = 0; i < 4; ++i) o[i] = pack_bf16(wj * gv[2 * i], wj * gv[2 * i + 1]);
          __builtin_nontemporal_store(o, dYp + r * nchunk + c);
        }
      }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) dot += __shfl_xor(dot, off);
    if (lane == 0) dw[t * k + j] = dot;
  }
}

// one thread per (token, expert): the gradient of a kept expert's logit, zero for the others
__global__ __launch_bounds__(256) void route_backward_kernel(const int* __restrict__ ids, const float* __restrict__ w,
                                                             const float* __restrict__ dw, long long n, int E, int k,
                                                             float* __restrict__ dz) {
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= n) return;
  const long long t = idx / E;
  const int e = (int)(idx % E);
  float inner = 0.f, wj = 0.f, dwj = 0.f;
  bool kept = false;
  for (int j = 0; j < k; ++j) {
    const float wv = w[t * k + j], dv = dw[t * k + j];
    inner = fmaf(wv, dv, inner);
    if (ids[t * k + j] == e) {
      kept = true;
      wj = wv;
      dwj = dv;
    }
  }
  dz[idx] = kept ? wj * (dwj - inner) : 0.f;
}

}  // namespace

extern "C" int32_t feplb_combine_backward(const void* dY, const void* Yp, int32_t yp_dtype, int32_t R_cap,
                                          const int32_t* inv,
                                          const float* topk_w, int32_t T, int32_t k, int32_t d, void* dYp,
                                          float* dw, void* stream) {
  FEPLB_REQUIRE(T >= 0 && k >= 1 && d >= 0 && R_cap >= 0, FEPLB_EINVAL, "combine_backward: negative size");
  FEPLB_REQUIRE(k <= FEPLB_MAX_TOPK, FEPLB_ESHAPE, "combine_backward: k=%d above %d", k, FEPLB_MAX_TOPK);
  FEPLB_REQUIRE(d % 8 == 0, FEPLB_ESHAPE, "combine_backward: d=%d not a multiple of 8", d);
  FEPLB_REQUIRE(yp_dtype == FEPLB_F32 || yp_dtype == FEPLB_BF16, FEPLB_EINVAL,
                "combine_backward: unknown yp_dtype %d", yp_dtype);
  if (T == 0 || d == 0) return FEPLB_OK;
  FEPLB_REQUIRE(dY && inv && topk_w && dw, FEPLB_EINVAL, "combine_backward: null buffer");
  FEPLB_REQUIRE(feplb::aligned16(dY) && feplb::aligned16(Yp) && feplb::aligned16(dYp), FEPLB_EALIGN,
                "combine_backward: dY/Yp/dYp not 16-byte aligned");
  FEPLB_REQUIRE((Yp && dYp) || R_cap == 0, FEPLB_EINVAL, "combine_backward: null Yp/dYp with R_cap=%d", R_cap);
  hipStream_t s = (hipStream_t)stream;
  const int blocks = (T + WAVES - 1) / WAVES;
  // as many 16-byte pieces of the gradient row per lane as one pass over the row needs, up to 16
  const int per_lane = (d / 8 + 63) / 64;
#define FEPLB_COMBINE_BWD(BF, U)                                                                             \
  hipLaunchKernelGGL((combine_backward_kernel<BF, U>), dim3(blocks), dim3(BLOCK), 0, s, (const u32x4*)dY, Yp, \
                     inv, topk_w, T, k, d, R_cap, (u32x4*)dYp, dw)
  if (yp_dtype == FEPLB_BF16) {
    if (per_lane <= 4) FEPLB_COMBINE_BWD(true, 4);
    else if (per_lane <= 8) FEPLB_COMBINE_BWD(true, 8);
    else if (per_lane <= 12) FEPLB_COMBINE_BWD(true, 12);
    else FEPLB_COMBINE_BWD(true, 16);
  } else {
    if (per_lane <= 4) FEPLB_COMBINE_BWD(false, 4);
    else if (per_lane <= 8) FEPLB_COMBINE_BWD(false, 8);
    else if (per_lane <= 12) FEPLB_COMBINE_BWD(false, 12);
    else FEPLB_COMBINE_BWD(false, 16);
  }
#undef FEPLB_COMBINE_BWD
  FEPLB_LAUNCH_CHECK("combine_backward_kernel");
  return FEPLB_OK;
}

extern "C" int32_t feplb_route_topk_backward(const int32_t* topk_ids, const float* topk_w, const float* dw,
                                             int32_t T, int32_t E, int32_t k, float* dlogits, void* stream) {
  FEPLB_REQUIRE(T >= 0 && E >= 1 && k >= 1, FEPLB_EINVAL, "route_topk_backward: T=%d E=%d k=%d", T, E, k);
  FEPLB_REQUIRE(E <= FEPLB_MAX_EXPERTS && k <= E && k <= FEPLB_MAX_TOPK, FEPLB_ESHAPE,
                "route_topk_backward: E=%d k=%d out of range", E, k);
  if (T == 0) return FEPLB_OK;
  FEPLB_REQUIRE(topk_ids && topk_w && dw && dlogits, FEPLB_EINVAL, "route_topk_backward: null buffer");
  const long long n = (long long)T * E;
  FEPLB_REQUIRE(n < (1ll << 39), FEPLB_ESHAPE, "route_topk_backward: T*E too large");
  hipLaunchKernelGGL(route_backward_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream,
                     topk_ids, topk_w, dw, n, E, k, dlogits);
  FEPLB_LAUNCH_CHECK("route_backward_kernel");
  return FEPLB_OK;
}
