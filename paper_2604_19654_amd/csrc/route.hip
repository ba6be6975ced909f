// Top-k routing (paper Section 2.3: the router yields each token's expert
// choices; Section 3.1: top-k over 128 routed experts, no auxiliary loss).
// Score: softmax over all E logits, k largest kept and renormalised, which is
// the same as a softmax over the k kept logits.
//
// A token is handled by a sub-group of SG lanes of a wavefront, each lane
// holding VPL logits in registers, so a 64-wide wavefront routes 64/SG tokens
// at once.  Selection runs k rounds of "sub-group maximum of a 64-bit key";
// the key orders by logit descending, then expert id ascending, so ties need
// no extra pass.  HBM-bound in principle (T*E*4 bytes in, T*k*8 out).
#include "common.h"

namespace {

__device__ __forceinline__ uint32_t orderable(float x) {
  uint32_t u = __float_as_uint(x);
  if (u == 0x80000000u) u = 0u;  // -0.0 ties with +0.0
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ float from_orderable(uint32_t o) {
  uint32_t u = (o & 0x80000000u) ? (o & 0x7fffffffu) : ~o;
  return __uint_as_float(u);
}

template <int SG>
__device__ __forceinline__ unsigned long long group_max(unsigned long long v) {
#pragma unroll
  for (int m = SG / 2; m >= 1; m >>= 1) {
    unsigned long long o = __shfl_xor(v, m, SG);
    v = o > v ? o : v;
  }
  return v;
}

// Expert e of a token sits in lane (e % SG) of the token's sub-group, register e / SG.
template <int SG, int VPL>
__global__ __launch_bounds__(256) void route_topk_kernel(const float* __restrict__ logits, int T,
                                                         int E, int k, int* __restrict__ ids,
                                                         float* __restrict__ w,
                                                         int* __restrict__ counts) {
  extern __shared__ int hist[];
  const int tid = threadIdx.x;
  if (counts) {
    for (int e = tid; e < E; e += 256) hist[e] = 0;
    __syncthreads();
  }
  constexpr int TOK_PER_BLOCK = 256 / SG;
  const int sub = tid / SG;   // token slot inside the block
  const int li = tid % SG;    // lane inside the sub-group
  for (long long t0 = (long long)blockIdx.x * TOK_PER_BLOCK; t0 < T;
       t0 += (long long)gridDim.x * TOK_PER_BLOCK) {
    const long long t = t0 + sub;
    const bool live = t < T;
    unsigned long long key[VPL];
#pragma unroll
    for (int q = 0; q < VPL; ++q) {
      const int e = q * SG + li;
      key[q] = 0ull;
      if (live && e < E) {
        const float x = logits[t * E + e];
        key[q] = ((unsigned long long)orderable(x) << 32) | (unsigned long long)(0xffffffffu - (uint32_t)e);
      }
    }
    float top = 0.f, sum = 0.f, mine_x = 0.f;
    int mine_id = 0;
    for (int j = 0; j < k; ++j) {
      unsigned long long best = key[0];
#pragma unroll
      for (int q = 1; q < VPL; ++q) best = key[q] > best ? key[q] : best;
      best = group_max<SG>(best);
      const int e = (int)(0xffffffffu - (uint32_t)best);
      const float lv = from_orderable((uint32_t)(best >> 32));
      if (j == 0) top = lv;
      const float x = expf(lv - top);
      sum += x;
      if (li == j) {
        mine_id = e;
        mine_x = x;
      }
      if (li == e % SG) {
        const int q = e / SG;
#pragma unroll
        for (int qq = 0; qq < VPL; ++qq)
          if (qq == q) key[qq] = 0ull;
      }
    }
    if (live && li < k) {
      ids[t * k + li] = mine_id;
      w[t * k + li] = mine_x / sum;
      if (counts) atomicAdd(&hist[mine_id], 1);
    }
  }
  if (counts) {
    __syncthreads();
    for (int e = tid; e < E; e += 256)
      if (hist[e]) atomicAdd(&counts[e], hist[e]);
  }
}

__global__ void zero_i32_kernel(int* p, int n) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

template <int SG, int VPL>
void launch(const float* logits, int T, int E, int k, int* ids, float* w, int* counts,
            hipStream_t s) {
  const int per = 256 / SG;
  long long blocks = ((long long)T + per - 1) / per;
  if (blocks > 8192) blocks = 8192;
  hipLaunchKernelGGL((route_topk_kernel<SG, VPL>), dim3((unsigned)blocks), dim3(256),
                     counts ? (size_t)E * sizeof(int) : 0, s, logits, T, E, k, ids, w, counts);
}

template <int SG>
void pick_vpl(int vpl, const float* logits, int T, int E, int k, int* ids, float* w, int* counts,
              hipStream_t s) {
  if (vpl <= 1) launch<SG, 1>(logits, T, E, k, ids, w, counts, s);
  else if (vpl <= 2) launch<SG, 2>(logits, T, E, k, ids, w, counts, s);
  else if (vpl <= 4) launch<SG, 4>(logits, T, E, k, ids, w, counts, s);
  else if (vpl <= 8) launch<SG, 8>(logits, T, E, k, ids, w, counts, s);
  else launch<SG, 16>(logits, T, E, k, ids, w, counts, s);
}

int next_pow2(int v) {
  int p = 1;
  while (p < v) p <<= 1;
  return p;
}

}  // namespace

extern "C" int32_t feplb_route_topk(const float* logits, int32_t T, int32_t E, int32_t k,
                                    int32_t* topk_ids, float* topk_w, int32_t* counts,
                                    void* stream) {
  FEPLB_REQUIRE(T >= 0 && E >= 1 && k >= 1, FEPLB_EINVAL, "route_topk: T=%d E=%d k=%d", T, E, k);
  FEPLB_REQUIRE(E <= FEPLB_MAX_EXPERTS, FEPLB_ESHAPE, "route_topk: E=%d above %d", E,
                FEPLB_MAX_EXPERTS);
  FEPLB_REQUIRE(k <= E && k <= FEPLB_MAX_TOPK, FEPLB_ESHAPE, "route_topk: k=%d (E=%d, max %d)", k,
                E, FEPLB_MAX_TOPK);
  FEPLB_REQUIRE((long long)T * E < (1ll << 40), FEPLB_ESHAPE, "route_topk: T*E too large");
  hipStream_t s = (hipStream_t)stream;
  if (counts) {
    hipLaunchKernelGGL(zero_i32_kernel, dim3((E + 255) / 256), dim3(256), 0, s, counts, E);
    FEPLB_LAUNCH_CHECK("zero_i32_kernel");
  }
  if (T == 0) return FEPLB_OK;
  FEPLB_REQUIRE(logits && topk_ids && topk_w, FEPLB_EINVAL, "route_topk: null buffer");
  // sub-group width: at least k lanes (lane j keeps result j), and wide enough
  // that a lane holds at most 8 logits (16 for the largest E).
  int sg = next_pow2(k);
  const int by_e = next_pow2((E + 7) / 8);
  if (by_e > sg) sg = by_e;
  if (sg < 8) sg = 8;
  if (sg > 64) sg = 64;
  const int vpl = (E + sg - 1) / sg;
  switch (sg) {
    case 8: pick_vpl<8>(vpl, logits, T, E, k, topk_ids, topk_w, counts, s); break;
    case 16: pick_vpl<16>(vpl, logits, T, E, k, topk_ids, topk_w, counts, s); break;
    case 32: pick_vpl<32>(vpl, logits, T, E, k, topk_ids, topk_w, counts, s); break;
    default: pick_vpl<64>(vpl, logits, T, E, k, topk_ids, topk_w, counts, s); break;
  }
  FEPLB_LAUNCH_CHECK("route_topk_kernel");
  return FEPLB_OK;
}
