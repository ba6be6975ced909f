// Ragged grouped SwiGLU expert FFN on bf16 MFMA (paper Section 3.1: expert
// compute is a Grouped GEMM; Sections 1 and 2.3: its speed depends on each
// expert's batch size and it must not fragment into per-expert launches).
//
// Two GEMM kernels, each ONE launch for a whole range of groups:
//   gate_up : H[r,:]  = bf16( silu(Xp[r,:] Wg[g]) * (Xp[r,:] Wu[g]) )
//   down    : Yp[r,:] = H[r,:] Wd[g]
// A small schedule kernel turns offsets[] (device memory, ragged, possibly
// empty groups) into a table of row tiles; the GEMM grid covers an upper bound
// of tiles and surplus blocks leave at once, so the host never needs R.
//
// Block tile: 256 rows x 256 weight columns x 64 k per step, 4 wavefronts
// (2 x 2), one per SIMD, each 128 x 128 as 4 x 4 MFMA 32x32x16 bf16 tiles
// (256 fp32 accumulators per lane).  For gate_up the 256 weight columns are
// 128 gate + the matching 128 up columns, so the SwiGLU product happens in
// registers and only H is written.  LDS holds two stages of (A 256 rows x 64 k,
// k-contiguous, 144-byte pitch; B 64 k x 256 columns, column-contiguous as in
// memory, 576-byte pitch); global loads for step kt+2 and the LDS fill of step
// kt+1 overlap the MFMAs of step kt, one barrier per step.
// Weights are row-major [K,N] (N contiguous) as the caller stores them, while
// an MFMA lane needs 8 consecutive k of one column: the B fragments are read
// with the transposing LDS load of gfx950 (ds_read_b64_tr_b16), which hands
// lane i of a 16-lane group the 4 k-values of column i from a 4(k) x 16(n)
// block, so no transpose is done in registers.
// Blocks are mapped to tiles in 8 x 4 patches per XCD (workgroups are dealt
// round-robin to the 8 XCDs, each with its own L2), so the 32 tiles an XCD
// runs at a time share 8 row panels and 4 weight panels.
#include "common.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef short i16x4 __attribute__((ext_vector_type(4)));

constexpr int BM = 256;      // rows per tile
constexpr int BNW = 256;     // weight columns per tile
constexpr int BK = 64;       // k per step
constexpr int LDK = BK + 8;    // A: LDS row pitch in bf16 (144 bytes: conflict-free 16-byte reads)
constexpr int LDN = BNW + 32;  // B: LDS row pitch in bf16 (576 bytes: 4 consecutive rows cover all banks)
constexpr int THREADS = 256;
constexpr int A_ELEMS = BM * LDK;
constexpr int STAGE_ELEMS = A_ELEMS + BK * LDN;             // bf16 elements per stage
constexpr size_t LDS_BYTES = 2 * (size_t)STAGE_ELEMS * 2;   // two stages
constexpr int XCDS = 8;

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
    int patch_n, WeightTable wt, void* __restrict__ out) {
  extern __shared__ __attribute__((aligned(16))) uint16_t lds[];

  // ---- block -> tile: patches of (32 / patch_n) row tiles x patch_n column tiles per XCD
  const int tid = threadIdx.x;
  const int xcd = blockIdx.x % XCDS;
  const int slot = blockIdx.x / XCDS;
  const int patch_m = 32 / patch_n;
  const int patch = (slot / 32) * XCDS + xcd;
  const int within = slot % 32;
  const int patches_n = n_tiles_n / patch_n;
  const int mt = (patch / patches_n) * patch_m + within % patch_m;
  const int nt = (patch % patches_n) * patch_n + within / patch_m;
  if (mt >= sched[0].x) return;
  const int4 tile = sched[1 + mt];
  const int g = tile.x, row0 = tile.y, rows = tile.z;

  // ---- global -> register staging
  // A: 256 rows x 8 vectors of 8 bf16; thread handles row tid/8 + 32*i, vector tid%8
  const int a_vec = tid % 8;
  uint32_t a_off[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int r = min(tid / 8 + 32 * i, rows - 1);
    a_off[i] = (uint32_t)r * (uint32_t)K + a_vec * 8;
  }
  const uint16_t* a_base = A + (size_t)row0 * K;
  // B: 64 k-rows x 32 vectors of 8 columns; thread handles k-row tid/32 + 8*i, vector tid%32
  // (a wavefront reads 2 rows x 512 contiguous bytes per load)
  const int b_vec = tid % 32, b_k = tid / 32;
  const uint16_t* b_src;
  if (MODE == 0) {
    const uint16_t* W = (const uint16_t*)(b_vec < 16 ? wt.w0[g] : wt.w1[g]);
    b_src = W + (size_t)b_k * N + (size_t)nt * 128 + (b_vec % 16) * 8;
  } else {
    b_src = (const uint16_t*)wt.w0[g] + (size_t)b_k * N + (size_t)nt * 256 + b_vec * 8;
  }

  u32x4 a_reg[8], b_reg[8];
  auto load_a = [&](int k0) {
#pragma unroll
    for (int i = 0; i < 8; ++i) a_reg[i] = *(const u32x4*)(a_base + a_off[i] + k0);
  };
  auto load_b = [&](int k0) {
#pragma unroll
    for (int i = 0; i < 8; ++i) b_reg[i] = *(const u32x4*)(b_src + (size_t)(k0 + 8 * i) * N);
  };
  auto store_a = [&](uint16_t* As) {
#pragma unroll
    for (int i = 0; i < 8; ++i)
      *(u32x4*)(As + (tid / 8 + 32 * i) * LDK + a_vec * 8) = a_reg[i];
  };
  // rows i0..i0+3 of the thread's share of the B tile, layout unchanged
  auto store_b_half = [&](uint16_t* Bs, int i0) {
#pragma unroll
    for (int i = i0; i < i0 + 4; ++i) *(u32x4*)(Bs + (b_k + 8 * i) * LDN + b_vec * 8) = b_reg[i];
  };

  // ---- wave tiling: 2 x 2 waves, each 128 rows x 128 weight columns
  const int wave = tid / 64, lane = tid % 64;
  const int wm = wave / 2, wn = wave % 2;
  const int l32 = lane % 32, lk = (lane / 32) * 8;
  int a_row[4], b_col[4];
#pragma unroll
  for (int mi = 0; mi < 4; ++mi) a_row[mi] = (wm * 128 + mi * 32 + l32) * LDK + lk;
  // transposing read: lane s of a 16-lane group addresses 4 columns of k-row s/4; the group
  // then holds column (lane % 16) of its 16-column block, k = 4 consecutive rows
  const int tr_row = (lane / 32) * 8 + (lane % 16) / 4;
  const int tr_col = ((lane / 16) % 2) * 16 + (lane % 4) * 4;
#pragma unroll
  for (int nj = 0; nj < 4; ++nj) {
    const int c = MODE == 0 ? (nj / 2) * 128 + wn * 64 + (nj % 2) * 32 : wn * 128 + nj * 32;
    b_col[nj] = A_ELEMS + tr_row * LDN + c + tr_col;
  }

  f32x16 acc[4][4];
#pragma unroll
  for (int mi = 0; mi < 4; ++mi)
#pragma unroll
    for (int nj = 0; nj < 4; ++nj)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[mi][nj][v] = 0.f;

  bf16x8 af[2][4], bfr[2][4];
  auto load_frags = [&](const uint16_t* S, int ks, int buf) {
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) af[buf][mi] = *(const bf16x8*)(S + a_row[mi] + ks * 16);
#pragma unroll
    for (int nj = 0; nj < 4; ++nj) {
      typedef __attribute__((address_space(3))) i16x4 lds_i16x4;
      const uint16_t* p = S + b_col[nj] + ks * 16 * LDN;
      const i16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4*)p);
      const i16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4*)(p + 4 * LDN));
      bfr[buf][nj] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    }
  };
  auto mfma16 = [&](int buf) {
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
      for (int nj = 0; nj < 4; ++nj)
        acc[mi][nj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[buf][mi], bfr[buf][nj],
                                                             acc[mi][nj], 0, 0, 0);
  };

  // Software pipeline.  Step kt computes from stage kt&1 while the registers
  // holding tile kt+1 are written to the other stage and tile kt+2 is fetched.
  // Loads past the end re-read the last tile (k clamped) and the matching LDS
  // fill goes to a stage nobody reads again, so the loop body has no branches
  // and the interleaving below applies to every step.
  const int KT = K / BK;
  const int k_last = K - BK;
  load_a(0);
  load_b(0);
  store_a(lds);
  store_b_half(lds + A_ELEMS, 0);
  store_b_half(lds + A_ELEMS, 4);
  load_a(min(BK, k_last));
  load_b(min(BK, k_last));
  __syncthreads();
  load_frags(lds, 0, 0);
  for (int kt = 0; kt < KT; ++kt) {
    const uint16_t* S = lds + (kt & 1) * STAGE_ELEMS;
    uint16_t* Sn = lds + ((kt + 1) & 1) * STAGE_ELEMS;
    const int k2 = min((kt + 2) * BK, k_last);
    // section 0: fragments of k-slice 1; first half of the B tile of step kt+1 -> LDS
    load_frags(S, 1, 1);
    store_b_half(Sn + A_ELEMS, 0);
    mfma16(0);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // 1 MFMA
      __builtin_amdgcn_sched_group_barrier(0x180, 1, 0);   // 1 LDS op
    }
    __builtin_amdgcn_sched_barrier(0);
    // section 1: fragments of k-slice 2; second half of the B tile -> LDS; its
    // registers are free again: fetch the B tile of step kt+2 (a full step ahead of its use)
    load_frags(S, 2, 0);
    store_b_half(Sn + A_ELEMS, 4);
    load_b(k2);
    mfma16(1);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x180, 1, 0);
      if (i >= 8) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);  // 1 global load
    }
    __builtin_amdgcn_sched_barrier(0);
    // section 2: fragments of k-slice 3; A tile of step kt+1 -> LDS, then fetch the A tile of step kt+2
    load_frags(S, 3, 1);
    store_a(Sn);
    load_a(k2);
    mfma16(0);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x180, 1, 0);
      if (i >= 8) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
    // every wave has finished reading stage kt&1 and writing the other one
    __syncthreads();
    // section 3: first fragments of step kt+1
    load_frags(Sn, 0, 0);
    mfma16(1);
#pragma unroll
    for (int i = 0; i < 12; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
  }

  // ---- epilogue: lane holds column l32 of each 32x32 tile, rows 8*(v/4) + 4*(lane/32) + v%4
  const int rsub = (lane / 32) * 4;
  if (MODE == 0) {
    uint16_t* H = (uint16_t*)out;
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
      for (int nj = 0; nj < 2; ++nj) {
        const int col = nt * 128 + wn * 64 + nj * 32 + l32;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int r = wm * 128 + mi * 32 + 8 * (v / 4) + rsub + (v % 4);
          if (r < rows) {
            const float h = silu(acc[mi][nj][v]) * acc[mi][nj + 2][v];
            H[(size_t)(row0 + r) * N + col] = (uint16_t)bf16_rne(h);
          }
        }
      }
  } else {
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
      for (int nj = 0; nj < 4; ++nj) {
        const int col = nt * 256 + wn * 128 + nj * 32 + l32;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int r = wm * 128 + mi * 32 + 8 * (v / 4) + rsub + (v % 4);
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

template <int MODE, bool OUT_BF16>
hipError_t launch_gemm(const void* A, const int4* sched, int K, int N, int n_tiles_n, int max_tiles,
                       const WeightTable& wt, void* out, hipStream_t s) {
  static hipError_t attr = hipFuncSetAttribute(
      reinterpret_cast<const void*>(&grouped_gemm_kernel<MODE, OUT_BF16>),
      hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS_BYTES);
  if (attr != hipSuccess) return attr;
  const int patch_n = n_tiles_n % 4 == 0 ? 4 : (n_tiles_n % 2 == 0 ? 2 : 1);
  const int patch_m = 32 / patch_n;
  const int patches_m = (max_tiles + patch_m - 1) / patch_m;
  const int patches = patches_m * (n_tiles_n / patch_n);
  const int patch_rounds = (patches + XCDS - 1) / XCDS;
  const unsigned blocks = (unsigned)patch_rounds * XCDS * 32;
  hipLaunchKernelGGL((grouped_gemm_kernel<MODE, OUT_BF16>), dim3(blocks), dim3(THREADS), LDS_BYTES,
                     s, (const uint16_t*)A, sched, K, N, n_tiles_n, patch_n, wt, out);
  return hipGetLastError();
}

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
    FEPLB_HIP((launch_gemm<0, true>(Xp, (const int4*)ws, d, f, f / 128, max_tiles, up_tab, H, s)));
  }
  if (do_down) {
    if (yp_dtype == FEPLB_BF16)
      FEPLB_HIP((launch_gemm<1, true>(H, (const int4*)ws, f, d, d / 256, max_tiles, down_tab, Yp, s)));
    else
      FEPLB_HIP((launch_gemm<1, false>(H, (const int4*)ws, f, d, d / 256, max_tiles, down_tab, Yp, s)));
  }
  return FEPLB_OK;
}
