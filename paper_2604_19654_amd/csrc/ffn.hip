// Ragged grouped SwiGLU expert FFN on bf16 MFMA (paper Section 3.1: expert
// compute is a Grouped GEMM; Sections 1 and 2.3: its speed depends on each
// expert's batch size and it must not fragment into per-expert launches).
//
// Two GEMM kernels, each ONE launch for a whole range of groups:
//   gate_up : H[r,:]  = bf16( silu(Xp[r,:] Wg[g]) * (Xp[r,:] Wu[g]) )
//   down    : Yp[r,:] = H[r,:] Wd[g]
// A small schedule kernel turns offsets[] (device memory, ragged, possibly
// empty groups) into a table of 128-row tiles; the GEMM grid covers an upper
// bound of tiles and surplus blocks leave at once, so the host never needs R.
//
// Tile: 128 rows x 256 weight columns x 64 k per step, 4 wavefronts (2 x 2),
// each 64 x 128 as 2 x 4 MFMA 32x32x16 bf16 tiles with fp32 accumulators.  For
// gate_up the 256 weight columns are 128 gate + the matching 128 up columns, so
// the SwiGLU product happens in registers and only H is written.
// Weights are row-major [K,N] (N contiguous) as the caller stores them; an MFMA
// lane needs 8 consecutive k of one column, so each thread loads an 8(k) x 8(n)
// block and transposes it in registers on the way into LDS.
#include "common.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int BM = 128;    // rows per tile
constexpr int BNW = 256;   // weight columns per tile
constexpr int BK = 64;     // k per step
constexpr int LDK = BK + 8;  // LDS row pitch in bf16 (144 bytes: conflict-free 16-byte reads)
constexpr int THREADS = 256;

struct WeightTable {
  const void* w0[FEPLB_MAX_GROUPS];  // gate (gate_up) or down (down)
  const void* w1[FEPLB_MAX_GROUPS];  // up (gate_up only)
};

// ws layout: int4 header {n_tiles,0,0,0}, then int4 {group, row0, rows, 0} per tile
__global__ __launch_bounds__(FEPLB_MAX_GROUPS) void ffn_schedule_kernel(
    const int* __restrict__ offsets, int g_begin, int g_end, int R_cap, int max_tiles,
    int4* __restrict__ ws) {
  __shared__ int scan[FEPLB_MAX_GROUPS];
  const int i = threadIdx.x;
  const int g = g_begin + i;
  int lo = 0, hi = 0, mt = 0;
  if (g < g_end) {
    lo = min(offsets[g], R_cap);
    hi = min(offsets[g + 1], R_cap);
    mt = hi > lo ? (hi - lo + BM - 1) / BM : 0;
  }
  scan[i] = mt;
  __syncthreads();
  for (int d = 1; d < FEPLB_MAX_GROUPS; d <<= 1) {
    const int v = i >= d ? scan[i - d] : 0;
    __syncthreads();
    scan[i] += v;
    __syncthreads();
  }
  int first = scan[i] - mt;
  for (int m = 0; m < mt; ++m) {
    const int idx = first + m;
    if (idx < max_tiles) ws[1 + idx] = make_int4(g, lo + m * BM, min(BM, hi - lo - m * BM), 0);
  }
  if (i == FEPLB_MAX_GROUPS - 1) ws[0] = make_int4(min(scan[i], max_tiles), 0, 0, 0);
}

__device__ __forceinline__ uint32_t bf16_rne(float x) {
  uint32_t u = __float_as_uint(x);
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}

__device__ __forceinline__ float silu(float a) { return a / (1.0f + __expf(-a)); }

// MODE 0: gate_up (+SwiGLU, bf16 out); MODE 1: down (fp32 or bf16 out)
template <int MODE, bool OUT_BF16>
__global__ __launch_bounds__(THREADS) void grouped_gemm_kernel(
    const uint16_t* __restrict__ A, const int4* __restrict__ sched, int K, int N, int n_tiles_n,
    WeightTable wt, void* __restrict__ out) {
  __shared__ __attribute__((aligned(16))) uint16_t As[BM * LDK];
  __shared__ __attribute__((aligned(16))) uint16_t Bs[BNW * LDK];

  const int tid = threadIdx.x;
  const int nt = blockIdx.x % n_tiles_n;
  const int mt = blockIdx.x / n_tiles_n;
  if (mt >= sched[0].x) return;
  const int4 tile = sched[1 + mt];
  const int g = tile.x, row0 = tile.y, rows = tile.z;

  // ---- global -> register staging
  // A: 128 rows x 8 vectors of 8 bf16; thread handles vectors tid + 256*i
  const uint16_t* a_src[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int idx = tid + THREADS * i;
    const int r = min(idx / 8, rows - 1);
    a_src[i] = A + (size_t)(row0 + r) * K + (idx % 8) * 8;
  }
  // B: thread owns the 8(k) x 8(n) block (kb, nb)
  const int kb = tid % 8, nb = tid / 8;
  const uint16_t* b_src;
  if (MODE == 0) {
    const uint16_t* W = (const uint16_t*)(nb < 16 ? wt.w0[g] : wt.w1[g]);
    b_src = W + (size_t)(kb * 8) * N + (size_t)nt * 128 + (nb % 16) * 8;
  } else {
    b_src = (const uint16_t*)wt.w0[g] + (size_t)(kb * 8) * N + (size_t)nt * 256 + nb * 8;
  }

  u32x4 a_reg[4], b_reg[8];
  auto load_tiles = [&](int k0) {
#pragma unroll
    for (int i = 0; i < 4; ++i) a_reg[i] = *(const u32x4*)(a_src[i] + k0);
#pragma unroll
    for (int i = 0; i < 8; ++i) b_reg[i] = *(const u32x4*)(b_src + (size_t)(k0 + i) * N);
  };
  auto store_tiles = [&]() {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int idx = tid + THREADS * i;
      *(u32x4*)(As + (idx / 8) * LDK + (idx % 8) * 8) = a_reg[i];
    }
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      u32x4 o;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint32_t lo = b_reg[2 * j][c / 2], hi = b_reg[2 * j + 1][c / 2];
        o[j] = (c & 1) ? ((lo >> 16) | (hi & 0xffff0000u)) : ((lo & 0xffffu) | (hi << 16));
      }
      *(u32x4*)(Bs + (nb * 8 + c) * LDK + kb * 8) = o;
    }
  };

  // ---- wave tiling
  const int wave = tid / 64, lane = tid % 64;
  const int wm = wave / 2, wn = wave % 2;
  const int l32 = lane % 32, lk = (lane / 32) * 8;
  int b_row[4];
#pragma unroll
  for (int nj = 0; nj < 4; ++nj) {
    if (MODE == 0)
      b_row[nj] = (nj / 2) * 128 + wn * 64 + (nj % 2) * 32 + l32;
    else
      b_row[nj] = wn * 128 + nj * 32 + l32;
  }

  f32x16 acc[2][4];
#pragma unroll
  for (int mi = 0; mi < 2; ++mi)
#pragma unroll
    for (int nj = 0; nj < 4; ++nj)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[mi][nj][v] = 0.f;

  const int KT = K / BK;
  load_tiles(0);
  for (int kt = 0; kt < KT; ++kt) {
    __syncthreads();
    store_tiles();
    __syncthreads();
    if (kt + 1 < KT) load_tiles((kt + 1) * BK);
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 af[2], bfr[4];
#pragma unroll
      for (int mi = 0; mi < 2; ++mi)
        af[mi] = *(const bf16x8*)(As + (wm * 64 + mi * 32 + l32) * LDK + ks * 16 + lk);
#pragma unroll
      for (int nj = 0; nj < 4; ++nj)
        bfr[nj] = *(const bf16x8*)(Bs + b_row[nj] * LDK + ks * 16 + lk);
#pragma unroll
      for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int nj = 0; nj < 4; ++nj)
          acc[mi][nj] =
              __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[mi], bfr[nj], acc[mi][nj], 0, 0, 0);
    }
  }

  // ---- epilogue: lane holds column l32 of each 32x32 tile, rows 8*(v/4) + 4*(lane/32) + v%4
  const int rsub = (lane / 32) * 4;
  if (MODE == 0) {
    uint16_t* H = (uint16_t*)out;
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
      for (int nj = 0; nj < 2; ++nj) {
        const int col = nt * 128 + wn * 64 + nj * 32 + l32;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int r = wm * 64 + mi * 32 + 8 * (v / 4) + rsub + (v % 4);
          if (r < rows) {
            const float h = silu(acc[mi][nj][v]) * acc[mi][nj + 2][v];
            H[(size_t)(row0 + r) * N + col] = (uint16_t)bf16_rne(h);
          }
        }
      }
  } else {
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
      for (int nj = 0; nj < 4; ++nj) {
        const int col = nt * 256 + wn * 128 + nj * 32 + l32;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int r = wm * 64 + mi * 32 + 8 * (v / 4) + rsub + (v % 4);
          if (r < rows) {
            if (OUT_BF16)
              ((uint16_t*)out)[(size_t)(row0 + r) * N + col] = (uint16_t)bf16_rne(acc[mi][nj][v]);
            else
              ((float*)out)[(size_t)(row0 + r) * N + col] = acc[mi][nj][v];
          }
        }
      }
  }
}

int max_tiles_for(int R_cap, int ng) { return R_cap / BM + ng + 1; }

}  // namespace

extern "C" size_t feplb_grouped_ffn_workspace_bytes(int32_t R_cap, int32_t G) {
  if (R_cap < 0 || G < 0) return 0;
  return (size_t)(1 + max_tiles_for(R_cap, G)) * sizeof(int4);
}

extern "C" int32_t feplb_grouped_ffn(const void* Xp, const int32_t* offsets, int32_t g_begin,
                                     int32_t g_end, int32_t R_cap, int32_t d, int32_t f,
                                     const void* const* w_gate, const void* const* w_up,
                                     const void* const* w_down, void* H, void* Yp,
                                     int32_t yp_dtype, int32_t phases, void* ws, size_t ws_bytes,
                                     void* stream) {
  FEPLB_REQUIRE(g_begin >= 0 && g_end >= g_begin && R_cap >= 0 && d >= 0 && f >= 0, FEPLB_EINVAL,
                "grouped_ffn: negative size or empty range reversed");
  FEPLB_REQUIRE(g_end <= FEPLB_MAX_GROUPS, FEPLB_ESHAPE, "grouped_ffn: g_end=%d above %d", g_end,
                FEPLB_MAX_GROUPS);
  FEPLB_REQUIRE((phases & ~FEPLB_FFN_ALL) == 0 && phases != 0, FEPLB_EINVAL,
                "grouped_ffn: phases=%d", phases);
  FEPLB_REQUIRE(yp_dtype == FEPLB_F32 || yp_dtype == FEPLB_BF16, FEPLB_EINVAL,
                "grouped_ffn: unknown yp_dtype %d", yp_dtype);
  FEPLB_REQUIRE(d % 256 == 0 && f % 128 == 0 && d > 0 && f > 0, FEPLB_ESHAPE,
                "grouped_ffn: need d %% 256 == 0 and f %% 128 == 0 (d=%d f=%d)", d, f);
  const int ng = g_end - g_begin;
  if (ng == 0 || R_cap == 0) return FEPLB_OK;
  FEPLB_REQUIRE(offsets, FEPLB_EINVAL, "grouped_ffn: null offsets");
  const bool do_up = phases & FEPLB_FFN_GATE_UP, do_down = phases & FEPLB_FFN_DOWN;
  if (do_up) {
    FEPLB_REQUIRE(Xp && H && w_gate && w_up, FEPLB_EINVAL, "grouped_ffn: null Xp/H/w_gate/w_up");
    FEPLB_REQUIRE(feplb::aligned16(Xp) && feplb::aligned16(H), FEPLB_EALIGN,
                  "grouped_ffn: Xp/H not 16-byte aligned");
  }
  if (do_down) {
    FEPLB_REQUIRE(Yp && H && w_down, FEPLB_EINVAL, "grouped_ffn: null Yp/H/w_down");
    FEPLB_REQUIRE(feplb::aligned16(Yp) && feplb::aligned16(H), FEPLB_EALIGN,
                  "grouped_ffn: Yp/H not 16-byte aligned");
  }
  WeightTable up_tab{}, down_tab{};
  for (int g = g_begin; g < g_end; ++g) {
    if (do_up) {
      FEPLB_REQUIRE(w_gate[g] && w_up[g], FEPLB_EINVAL, "grouped_ffn: null weights of group %d", g);
      FEPLB_REQUIRE(feplb::aligned16(w_gate[g]) && feplb::aligned16(w_up[g]), FEPLB_EALIGN,
                    "grouped_ffn: weights of group %d not 16-byte aligned", g);
      up_tab.w0[g] = w_gate[g];
      up_tab.w1[g] = w_up[g];
    }
    if (do_down) {
      FEPLB_REQUIRE(w_down[g], FEPLB_EINVAL, "grouped_ffn: null w_down of group %d", g);
      FEPLB_REQUIRE(feplb::aligned16(w_down[g]), FEPLB_EALIGN,
                    "grouped_ffn: w_down of group %d not 16-byte aligned", g);
      down_tab.w0[g] = w_down[g];
      down_tab.w1[g] = nullptr;
    }
  }
  const int max_tiles = max_tiles_for(R_cap, ng);
  const size_t need = (size_t)(1 + max_tiles) * sizeof(int4);
  FEPLB_REQUIRE(ws && ws_bytes >= need, FEPLB_EWORKSPACE, "grouped_ffn: workspace %zu < %zu",
                ws_bytes, need);
  FEPLB_REQUIRE(feplb::aligned16(ws), FEPLB_EALIGN, "grouped_ffn: workspace not 16-byte aligned");
  hipStream_t s = (hipStream_t)stream;
  if (phases & FEPLB_FFN_SCHEDULE) {
    hipLaunchKernelGGL(ffn_schedule_kernel, dim3(1), dim3(FEPLB_MAX_GROUPS), 0, s, offsets,
                       g_begin, g_end, R_cap, max_tiles, (int4*)ws);
    FEPLB_LAUNCH_CHECK("ffn_schedule_kernel");
  }
  if (do_up) {
    const int ntn = f / 128;
    hipLaunchKernelGGL((grouped_gemm_kernel<0, true>), dim3((unsigned)max_tiles * ntn),
                       dim3(THREADS), 0, s, (const uint16_t*)Xp, (const int4*)ws, d, f, ntn, up_tab,
                       H);
    FEPLB_LAUNCH_CHECK("grouped_gemm_kernel<gate_up>");
  }
  if (do_down) {
    const int ntn = d / 256;
    if (yp_dtype == FEPLB_BF16)
      hipLaunchKernelGGL((grouped_gemm_kernel<1, true>), dim3((unsigned)max_tiles * ntn),
                         dim3(THREADS), 0, s, (const uint16_t*)H, (const int4*)ws, f, d, ntn,
                         down_tab, Yp);
    else
      hipLaunchKernelGGL((grouped_gemm_kernel<1, false>), dim3((unsigned)max_tiles * ntn),
                         dim3(THREADS), 0, s, (const uint16_t*)H, (const int4*)ws, f, d, ntn,
                         down_tab, Yp);
    FEPLB_LAUNCH_CHECK("grouped_gemm_kernel<down>");
  }
  return FEPLB_OK;
}
