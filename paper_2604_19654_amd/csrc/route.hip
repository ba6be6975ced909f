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
//
// With many tokens (enough to give every SIMD a wavefront of them) a second kernel
// routes one token per LANE instead: the lane streams its token's logits with 16-byte
// loads in ascending expert order and keeps the k best so far as a sorted list in
// registers.  A logit enters the list only if it is strictly greater than an entry, so
// among equal logits the lower expert id stays ahead: the same total order, on plain
// float compares (-0.0 equals +0.0), with a third of the instructions per token and no
// cross-lane traffic.
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

// Sorted insertion without branches: x enters before the first entry it is strictly greater than,
// the entries from there on move down one place, the last one drops out.  above[i] = (x > v[i]) is
// monotone in i because the list is sorted descending.
template <int K>
__device__ __forceinline__ void insert_sorted(float (&v)[K], int (&id)[K], float x, int e) {
  float nv[K];
  int ni[K];
#pragma unroll
  for (int i = 0; i < K; ++i) {
    const bool above = x > v[i];
    const bool above_prev = i > 0 ? x > v[i > 0 ? i - 1 : 0] : false;
    const float shifted_v = above_prev ? v[i > 0 ? i - 1 : 0] : x;
    const int shifted_i = above_prev ? id[i > 0 ? i - 1 : 0] : e;
    nv[i] = above ? shifted_v : v[i];
    ni[i] = above ? shifted_i : id[i];
  }
#pragma unroll
  for (int i = 0; i < K; ++i) {
    v[i] = nv[i];
    id[i] = ni[i];
  }
}

// One token per lane.  K = k exactly; E a multiple of 32; logits 16-byte aligned.
// A wavefront owns 64 consecutive tokens.  Reading a token's row straight into its lane would
// touch 64 different memory lines per load instruction; instead the wavefront loads 32 logits of
// all its tokens at a time as whole lines (8 lanes per 128-byte line), parks them in 8 KB of LDS
// of its own and each lane reads its token's 32 values back.  16-byte slot p of token tk sits at
// slot p ^ (tk & 7), which spreads the 16-byte reads of 16 consecutive tokens over the banks.
constexpr int LANE_WAVES = 2;   // wavefronts per block
template <int K>
__global__ __launch_bounds__(LANE_WAVES * 64) void route_topk_lane_kernel(
    const float* __restrict__ logits, int T, int E, int* __restrict__ ids, float* __restrict__ w,
    int* __restrict__ counts) {
  extern __shared__ int hist[];
  __shared__ __attribute__((aligned(16))) float stage[LANE_WAVES][64 * 32];
  const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64;
  if (counts) {
    for (int e = tid; e < E; e += LANE_WAVES * 64) hist[e] = 0;
    __syncthreads();
  }
  const long long t_wave = ((long long)blockIdx.x * LANE_WAVES + wave) * 64;
  const long long t = t_wave + lane;
  float v[K];
  int id[K];
#pragma unroll
  for (int i = 0; i < K; ++i) {
    v[i] = -INFINITY;   // below every finite logit; E >= K fills all entries
    id[i] = 0;
  }
  auto insert = [&](float x, int e) { insert_sorted<K>(v, id, x, e); };
  // load i of a chunk: token t_wave + 8*i + lane/8 (clamped to the last token), 16-byte piece lane%8
  const int piece = lane % 8;
  typedef float f32x4 __attribute__((ext_vector_type(4)));   // a plain vector type stays in registers
  const f32x4* src[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    long long tk = t_wave + 8 * i + lane / 8;
    if (tk > T - 1) tk = T - 1;
    src[i] = (const f32x4*)(logits + tk * E) + piece;
  }
  f32x4* const st = (f32x4*)stage[wave];
  f32x4 buf[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) buf[i] = src[i][0];
  for (int c0 = 0; c0 < E; c0 += 32) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int tk = 8 * i + lane / 8;
      st[tk * 8 + (piece ^ (tk & 7))] = buf[i];
    }
    // next chunk (the last trip re-reads its own: no branch)
    const int next = min(c0 + 32, E - 32) / 4;
#pragma unroll
    for (int i = 0; i < 8; ++i) buf[i] = src[i][next];
    __builtin_amdgcn_wave_barrier();   // the LDS runs a wavefront's accesses in order; this keeps the compiler from reordering them
#pragma unroll
    for (int p = 0; p < 8; ++p) {
      const f32x4 x = st[lane * 8 + (p ^ (lane & 7))];
      insert(x.x, c0 + 4 * p);
      insert(x.y, c0 + 4 * p + 1);
      insert(x.z, c0 + 4 * p + 2);
      insert(x.w, c0 + 4 * p + 3);
    }
    __builtin_amdgcn_wave_barrier();
  }
  if (t < T) {
    float p[K], sum = 0.f;
#pragma unroll
    for (int j = 0; j < K; ++j) {
      p[j] = expf(v[j] - v[0]);
      sum += p[j];
    }
#pragma unroll
    for (int j = 0; j < K; ++j) {
      ids[t * K + j] = id[j];
      w[t * K + j] = p[j] / sum;
      if (counts) atomicAdd(&hist[id[j]], 1);
    }
  }
  if (counts) {
    __syncthreads();
    for (int e = tid; e < E; e += LANE_WAVES * 64)
      if (hist[e]) atomicAdd(&counts[e], hist[e]);
  }
}

template <int K>
void launch_lane(const float* logits, int T, int E, int* ids, float* w, int* counts, hipStream_t s) {
  const int per = LANE_WAVES * 64;
  hipLaunchKernelGGL((route_topk_lane_kernel<K>), dim3((unsigned)((T + per - 1) / per)), dim3(per),
                     counts ? (size_t)E * sizeof(int) : 0, s, logits, T, E, ids, w, counts);
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
  // enough tokens to occupy a good part of the chip with one token per lane (a wavefront = 64 tokens)
  if (T >= 16384 && E % 32 == 0 && ((uintptr_t)logits & 15) == 0 && (k == 2 || k == 4 || k == 8)) {
    if (k == 2) launch_lane<2>(logits, T, E, topk_ids, topk_w, counts, s);
    else if (k == 4) launch_lane<4>(logits, T, E, topk_ids, topk_w, counts, s);
    else launch_lane<8>(logits, T, E, topk_ids, topk_w, counts, s);
    FEPLB_LAUNCH_CHECK("route_topk_lane_kernel");
    return FEPLB_OK;
  }
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
