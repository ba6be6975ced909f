// Backward-pass kernels of the grouped expert FFN that have no forward counterpart (paper
// Section 3.2 reports the layer's backward time beside the forward one):
//
//   weight gradients   C[g] = P_g^T Q_g, the sum over the rows of group g of outer products of a
//                      row of P with the same row of Q.  dW_down = H^T dYp, and
//                      [dW_gate | dW_up] = Xp^T [da | db].  The contraction runs over the ragged
//                      row range of the group, the output has the fixed shape of the weights.
//   transposes         W [r,c] -> W^T [c,r] (bf16), so that the input-gradient GEMMs
//                      (dH = dYp Wd^T, dXp = [da|db] [Wg^T; Wu^T]) can use the forward GEMM kernel,
//                      which wants its second operand row-major [K,N].
//
// The weight-gradient kernel has the forward kernel's shape: 256 x 256 output tile, 32 rows of
// the contraction per step, four wavefronts 2 x 2 of 128 x 128, MFMA 32x32x16 bf16, LDS-DMA
// loads with counted waits.  Both operands are row-major with the contraction index along the
// rows, which is how the forward kernel's weight operand lies, so both use that operand's LDS
// layout (two parts of 32 k-rows x 128 columns, XOR-swizzled) and its transposing LDS reads.
// Five stages of (P, Q) tiles, 32 KB each, fill the 160 KB of LDS.
#include <type_traits>
#include "common.h"
#include "gemm_device.h"

namespace {
using namespace feplb::dev;

constexpr int THREADS = 256;
constexpr int TILE = 256;             // output tile edge
constexpr int BK = 32;                // contraction rows per step
constexpr int NS = 5;                 // LDS stages
constexpr int PART_BYTES = BK * 128 * 2;      // one part: 32 k-rows x 128 columns
constexpr int STAGE_BYTES = 2 * PART_BYTES;   // 16 KB per operand and stage

struct OutTable {
  void* c0[FEPLB_MAX_GROUPS];   // output matrix for columns [0, n_split)
  void* c1[FEPLB_MAX_GROUPS];   // output matrix for columns [n_split, 2 n_split), or unused
};

// order[i] = the group (relative to g_begin) with the i-th most rows, ties by group index.  The
// weight-gradient grid walks the groups in this order: a tile's run time is proportional to its
// group's row count, and workgroups start in grid order, so the long tiles go first and the last
// compute units to finish are busy with short ones (empty groups, which only write zeros, last).
__global__ __launch_bounds__(FEPLB_MAX_GROUPS) void wgrad_order_kernel(const int* __restrict__ offsets, int g_begin,
                                                                       int n_groups, int R_cap, int* __restrict__ order) {
  __shared__ int rows[FEPLB_MAX_GROUPS];
  const int i = threadIdx.x;
  if (i < n_groups) {
    const int lo = min(offsets[g_begin + i], R_cap);
    rows[i] = max(min(offsets[g_begin + i + 1], R_cap), lo) - lo;
  }
  __syncthreads();
  if (i < n_groups) {
    int rank = 0;
    for (int j = 0; j < n_groups; ++j) rank += rows[j] > rows[i] || (rows[j] == rows[i] && j < i);
    order[rank] = i;
  }
}

__global__ __launch_bounds__(THREADS) void wgrad_gemm_kernel(
    const uint16_t* __restrict__ P, int ldp, const uint16_t* __restrict__ Q, int ldq,
    const int* __restrict__ offsets, const int* __restrict__ order, int g_begin, int n_groups, int R_cap,
    int m_tiles, int n_tiles, int patch_n, int n_split, OutTable out, int ldc, int accumulate) {
  __shared__ __attribute__((aligned(1024))) char lds_p0[STAGE_BYTES];
  __shared__ __attribute__((aligned(1024))) char lds_p1[STAGE_BYTES];
  __shared__ __attribute__((aligned(1024))) char lds_p2[STAGE_BYTES];
  __shared__ __attribute__((aligned(1024))) char lds_p3[STAGE_BYTES];
  __shared__ __attribute__((aligned(1024))) char lds_p4[STAGE_BYTES];
  __shared__ __attribute__((aligned(1024))) char lds_q0[STAGE_BYTES];
  __shared__ __attribute__((aligned(1024))) char lds_q1[STAGE_BYTES];
  __shared__ __attribute__((aligned(1024))) char lds_q2[STAGE_BYTES];
  __shared__ __attribute__((aligned(1024))) char lds_q3[STAGE_BYTES];
  __shared__ __attribute__((aligned(1024))) char lds_q4[STAGE_BYTES];
  auto stage_p = [&](auto st) -> char* {
    return st.value == 0 ? lds_p0 : st.value == 1 ? lds_p1 : st.value == 2 ? lds_p2 : st.value == 3 ? lds_p3 : lds_p4;
  };
  auto stage_q = [&](auto st) -> char* {
    return st.value == 0 ? lds_q0 : st.value == 1 ? lds_q1 : st.value == 2 ? lds_q2 : st.value == 3 ? lds_q3 : lds_q4;
  };

  // ---- block -> (group, tile): every group has the same tile grid; patches of (32 / patch_n) x
  // patch_n tiles go to one XCD, so the 32 tiles it runs at a time share few column panels
  const int tid = threadIdx.x;
  const int xcd = blockIdx.x % XCDS;
  const int slot = blockIdx.x / XCDS;
  const int patch_m = 32 / patch_n;
  const int patches_m = (m_tiles + patch_m - 1) / patch_m;
  const int patches_n = n_tiles / patch_n;
  const int per_group = patches_m * patches_n;
  const int patch_all = (slot / 32) * XCDS + xcd;
  const int slot_g = patch_all / per_group;
  if (slot_g >= n_groups) return;
  const int patch = patch_all % per_group;
  const int within = slot % 32;
  const int mt = (patch / patches_n) * patch_m + within % patch_m;
  const int nt = (patch % patches_n) * patch_n + within / patch_m;
  if (mt >= m_tiles) return;
  const int g = g_begin + order[slot_g];
  const int lo = __builtin_amdgcn_readfirstlane(min(offsets[g], R_cap));
  const int hi = __builtin_amdgcn_readfirstlane(max(min(offsets[g + 1], R_cap), lo));
  const int KT = (hi - lo + BK - 1) / BK;
  if (accumulate && KT == 0) return;   // nothing to add for an empty group
  // Row window of step kt: 32 rows from lo + 32 kt, except the last step, whose window ends at
  // the group's last row (moved back, never past the buffer) and is masked down to the rows the
  // earlier steps have not covered.
  const int w_last = min(max(hi - BK, 0), R_cap - BK);
  const int keep_lo = lo + (KT - 1) * BK;
  auto window = [&](int kt) { return kt < KT - 1 ? lo + kt * BK : w_last; };

  const int wave = __builtin_amdgcn_readfirstlane(tid / 64), lane = tid % 64;
  const int part = wave / 2;
  const int b_r = lane / 16;                       // k-row inside a load (= row & 3)
  const int b_slot = ((((lane % 16) >> 2) ^ b_r) << 2) | (lane & 3);   // 16-byte column slot read
  const uint32_t p_goff = ((uint32_t)((wave % 2) * 16 + b_r) * (uint32_t)ldp + b_slot * 8) * 2;
  const uint32_t q_goff = ((uint32_t)((wave % 2) * 16 + b_r) * (uint32_t)ldq + b_slot * 8) * 2;
  const char* p_gbase = wave_uniform(P + (size_t)mt * TILE + part * 128);
  const char* q_gbase = wave_uniform(Q + (size_t)nt * TILE + part * 128);
  const size_t p_row_bytes = (size_t)ldp * 2, q_row_bytes = (size_t)ldq * 2;
  auto issue_p = [&](auto stage, int row, int i) {
    load_to_lds_16(p_gbase + ((size_t)row + 4 * i) * p_row_bytes, p_goff,
                   lds_offset(stage_p(stage) + part * PART_BYTES + (wave % 2) * 4096 + i * 1024));
  };
  auto issue_q = [&](auto stage, int row, int i) {
    load_to_lds_16(q_gbase + ((size_t)row + 4 * i) * q_row_bytes, q_goff,
                   lds_offset(stage_q(stage) + part * PART_BYTES + (wave % 2) * 4096 + i * 1024));
  };

  // ---- wave tiling: 2 x 2 waves, each 128 columns of P (output rows) x 128 columns of Q
  const int wm = wave / 2, wn = wave % 2;
  const int l32 = lane % 32, h = lane / 32;
  // fragment (j, ks) of either operand: transposing read; lane s of a 16-lane group addresses 4
  // columns of k-row s/4 and ends up with 4 k-values of column (lane % 16) of the 16-column block
  uint32_t frag_off[4];
  {
    const int tr_r = h * 8 + (lane % 16) / 4;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int col = j * 32 + ((lane / 16) % 2) * 16 + (lane % 4) * 4;
      const int cs = col / 8;
      const int sw = ((((cs >> 2) ^ (tr_r & 3)) << 2) | (cs & 3));
      frag_off[j] = tr_r * 256 + sw * 16 + (col % 8) * 2;
    }
  }
  // A lane's fragment holds contraction rows window + 16 ks + 8 h + i, i = 0..7, two per
  // register.  tail[ks][v] keeps, in the last window, the rows in [keep_lo, hi).
  typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
  uint32_t tail[2][4];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks)
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int r0 = w_last + ks * 16 + h * 8 + 2 * v;
      tail[ks][v] = ((r0 >= keep_lo && r0 < hi) ? 0x0000ffffu : 0u) |
                    ((r0 + 1 >= keep_lo && r0 + 1 < hi) ? 0xffff0000u : 0u);
    }

  f32x16 acc[4][4];
#pragma unroll
  for (int mi = 0; mi < 4; ++mi)
#pragma unroll
    for (int nj = 0; nj < 4; ++nj)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[mi][nj][v] = 0.f;

  // fragment registers, double-buffered over the two 16-row slices of a step:
  // [buf][j] j < 4: P block j, else Q block j - 4; lo = rows 0..3 of the lane's eight, hi = 4..7
  u32x2 fl[2][8], fh[2][8];
  // read r of 16: fragment r / 2, half r % 2
  auto read_frag = [&](auto st, int ks, int buf, int r) {
    typedef __attribute__((address_space(3))) i16x4 lds_i16x4;
    const int j = r / 2;
    const char* base = j < 4 ? stage_p(st) + wm * PART_BYTES : stage_q(st) + wn * PART_BYTES;
    const char* p = base + ks * 16 * 256 + frag_off[j % 4] + (r % 2) * 4 * 256;
    const u32x2 v = __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4*)p));
    if (r % 2 == 0)
      fl[buf][j] = v;
    else
      fh[buf][j] = v;
  };
  // Row mask of the fragments in `buf` (slice ks = buf), all ones unless they belong to the
  // group's last window.  Applied in the half step that read them, behind its last reads and
  // between its later MFMAs, so that neither the LDS latency nor the 32 ANDs are exposed.
  auto mask_frags = [&](int buf, bool last) {
    uint32_t m[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) m[v] = last ? tail[buf][v] : 0xffffffffu;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      fl[buf][j] = u32x2{fl[buf][j].x & m[0], fl[buf][j].y & m[1]};
      fh[buf][j] = u32x2{fh[buf][j].x & m[2], fh[buf][j].y & m[3]};
    }
  };
  auto mfma16 = [&](int buf) {
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
      for (int nj = 0; nj < 4; ++nj) {
        const bf16x8 pf = __builtin_bit_cast(
            bf16x8, __builtin_shufflevector(fl[buf][mi], fh[buf][mi], 0, 1, 2, 3));
        const bf16x8 qf = __builtin_bit_cast(
            bf16x8, __builtin_shufflevector(fl[buf][4 + nj], fh[buf][4 + nj], 0, 1, 2, 3));
        // Q as the first operand: a lane ends up with one output row and runs of four columns
        acc[mi][nj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf, pf, acc[mi][nj], 0, 0, 0);
      }
  };

  // Software pipeline.  Step kt computes tile kt from stage kt % 5, in two halves of 16 MFMAs;
  // its barrier sits between the halves, when every wave holds the last fragments of tile kt.
  // Tile kt+4 is requested into the stage tile kt-1 has left: Q in the first half, P in the
  // second.  At the barrier of step kt tiles kt+2, kt+3 and the Q part of kt+4 (20 loads of
  // this wave) may still be in flight; everything older, tile kt+1 included, has landed.
  // Requests past the end re-read the last window into stages nobody reads again.
  auto step = [&](auto sc, int kt) {
    constexpr int s = decltype(sc)::value;                       // kt mod 5
    constexpr std::integral_constant<int, s % NS> cur{};
    constexpr std::integral_constant<int, (s + 1) % NS> nxt{};
    constexpr std::integral_constant<int, (s + 4) % NS> req{};
    const int row_req = window(min(kt + 4, KT - 1));
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      issue_q(req, row_req, q);
#pragma unroll
      for (int r = 4 * q; r < 4 * q + 4; ++r) read_frag(cur, 1, 1, r);
    }
    mask_frags(1, kt == KT - 1);
    mfma16(0);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);               // 1 MFMA
      if (i < 8)
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);             // 2 LDS reads
      else
        __builtin_amdgcn_sched_group_barrier(0x002, 5, 0);             // 5 VALU (the masking)
    }
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(0x4074);   // vmcnt(20) lgkmcnt(0)
    __syncthreads();
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      issue_p(req, row_req, q);
#pragma unroll
      for (int r = 4 * q; r < 4 * q + 4; ++r) read_frag(nxt, 0, 0, r);
    }
    mask_frags(0, kt + 1 == KT - 1);
    mfma16(1);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      if (i < 8)
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
      else
        __builtin_amdgcn_sched_group_barrier(0x002, 5, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
  };
  constexpr std::integral_constant<int, 0> c0{};
  constexpr std::integral_constant<int, 1> c1{};
  constexpr std::integral_constant<int, 2> c2{};
  constexpr std::integral_constant<int, 3> c3{};
  constexpr std::integral_constant<int, 4> c4{};
  if (KT > 0) {
    // prologue: tiles 0..3, Q then P each (32 loads of this wave); tile 0 is the first 8
#pragma unroll
    for (int q = 0; q < 4; ++q) issue_q(c0, window(0), q);
#pragma unroll
    for (int q = 0; q < 4; ++q) issue_p(c0, window(0), q);
#pragma unroll
    for (int q = 0; q < 4; ++q) issue_q(c1, window(min(1, KT - 1)), q);
#pragma unroll
    for (int q = 0; q < 4; ++q) issue_p(c1, window(min(1, KT - 1)), q);
#pragma unroll
    for (int q = 0; q < 4; ++q) issue_q(c2, window(min(2, KT - 1)), q);
#pragma unroll
    for (int q = 0; q < 4; ++q) issue_p(c2, window(min(2, KT - 1)), q);
#pragma unroll
    for (int q = 0; q < 4; ++q) issue_q(c3, window(min(3, KT - 1)), q);
#pragma unroll
    for (int q = 0; q < 4; ++q) issue_p(c3, window(min(3, KT - 1)), q);
    __builtin_amdgcn_s_waitcnt(0x4f78);   // vmcnt(24): tile 0 has landed
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 16; ++r) read_frag(c0, 0, 0, r);
    mask_frags(0, KT == 1);
    int kt = 0;
    for (; kt + 5 <= KT; kt += 5) {
      step(c0, kt);
      step(c1, kt + 1);
      step(c2, kt + 2);
      step(c3, kt + 3);
      step(c4, kt + 4);
    }
    // the remaining 0..4 steps (the stage phase is 0 again after whole trips of 5)
    if (kt < KT) {
      step(c0, kt);
      if (kt + 1 < KT) {
        step(c1, kt + 1);
        if (kt + 2 < KT) {
          step(c2, kt + 2);
          if (kt + 3 < KT) step(c3, kt + 3);
        }
      }
    }
    __builtin_amdgcn_s_waitcnt(0);   // the trailing re-reads must land before the stages are reused
    __syncthreads();
  }

  // ---- epilogue: fp32 tile.  A lane holds output row mi*32 + l32 of its wave's 128 and, in
  // accumulator registers 4c .. 4c+3, four consecutive columns 8c + 4 (lane / 32) .. +3 of block
  // nj.  Each wave passes 32 rows at a time through a 16 KB LDS region of its own and reads them
  // back with the lanes laid along the rows, so that every store writes whole lines.
  constexpr int ROW_BYTES = 128 * 4;
  constexpr int CH = ROW_BYTES / 16;   // 32 chunks per row
  constexpr int RPI = 64 / CH;         // 2 rows per store instruction
  char* ep = wave == 0 ? lds_p0 : wave == 1 ? lds_p1 : wave == 2 ? lds_p2 : lds_p3;
  const int csub = (lane / 32) * 4;
  int ncol0 = nt * TILE;
  char* cbase = (char*)out.c0[g];
  if (ncol0 >= n_split) {
    ncol0 -= n_split;
    cbase = (char*)out.c1[g];
  }
  char* out_wave = cbase + ((size_t)(mt * TILE + wm * 128) * ldc + ncol0 + wn * 128) * 4;
  const int rd_row = lane / CH, rd_chunk = lane % CH;
#pragma unroll
  for (int mi = 0; mi < 4; ++mi) {
#pragma unroll
    for (int nj = 0; nj < 4; ++nj)
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const int chunk = (nj * 32 + 8 * c + csub) / 4;
        *(float4*)(ep + l32 * ROW_BYTES + ((chunk ^ (l32 & (CH - 1))) << 4)) =
            make_float4(acc[mi][nj][4 * c], acc[mi][nj][4 * c + 1], acc[mi][nj][4 * c + 2], acc[mi][nj][4 * c + 3]);
      }
#pragma unroll
    for (int j = 0; j < 32 / RPI; ++j) {
      const int r = j * RPI + rd_row;
      typedef float f32x4 __attribute__((ext_vector_type(4)));
      f32x4 v = *(const f32x4*)(ep + r * ROW_BYTES + ((rd_chunk ^ (r & (CH - 1))) << 4));
      f32x4* dst = (f32x4*)(out_wave + (size_t)(mi * 32 + r) * ldc * 4 + rd_chunk * 16);
      if (accumulate) v += __builtin_nontemporal_load(dst);
      __builtin_nontemporal_store(v, dst);
    }
  }
}

// W [rows, cols] -> W^T [cols, rows], bf16, one 64 x 64 tile per block; z picks the group
constexpr int TT = 64;
__global__ __launch_bounds__(256) void transpose_bf16_kernel(WeightTable src, int g_begin, int rows, int cols,
                                                              uint16_t* __restrict__ dst0, size_t dst_group_stride) {
  __shared__ uint16_t tile[TT][TT + 2];
  const int g = g_begin + blockIdx.z;
  const uint16_t* __restrict__ W = (const uint16_t*)src.w0[g];
  uint16_t* __restrict__ WT = dst0 + (size_t)blockIdx.z * dst_group_stride;
  const int r0 = blockIdx.y * TT, c0 = blockIdx.x * TT;
  const int t = threadIdx.x;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int idx = t + i * 256;           // 512 pieces of 8 elements
    const int r = idx / 8, c8 = (idx % 8) * 8;
    const u32x4 v = __builtin_nontemporal_load((const u32x4*)(W + (size_t)(r0 + r) * cols + c0 + c8));
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      tile[r][c8 + 2 * e] = (uint16_t)(w[e] & 0xffffu);
      tile[r][c8 + 2 * e + 1] = (uint16_t)(w[e] >> 16);
    }
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int idx = t + i * 256;
    const int c = idx / 8, r8 = (idx % 8) * 8;   // output row c (a column of W), 8 consecutive rows of W
    uint32_t w[4];
#pragma unroll
    for (int e = 0; e < 4; ++e)
      w[e] = (uint32_t)tile[r8 + 2 * e][c] | ((uint32_t)tile[r8 + 2 * e + 1][c] << 16);
    const u32x4 o = {w[0], w[1], w[2], w[3]};
    __builtin_nontemporal_store(o, (u32x4*)(WT + (size_t)(c0 + c) * rows + r0 + r8));
  }
}

}  // namespace

namespace feplb {

// C[g] = P_g^T Q_g for g in [g_begin, g_begin + n_groups): P [R_cap, ldp] columns [0, M),
// Q [R_cap, ldq] columns [0, N); output fp32 row-major with row stride ldc; columns of the
// product at or past n_split go to c1[g] (shifted by n_split).  M, N, n_split multiples of 256.
// accumulate: the product is added to what the output matrices hold (an empty group's are left
// alone) instead of replacing it.
hipError_t launch_wgrad(const void* P, int ldp, int M, const void* Q, int ldq, int N, const int* offsets,
                        const int* order, int g_begin, int n_groups, int R_cap, void* const* c0, void* const* c1,
                        int n_split, int ldc, bool accumulate, hipStream_t s) {
  OutTable tab{};
  for (int i = 0; i < n_groups; ++i) {
    tab.c0[g_begin + i] = c0[g_begin + i];
    tab.c1[g_begin + i] = c1 ? c1[g_begin + i] : nullptr;
  }
  const int m_tiles = M / TILE, n_tiles = N / TILE;
  const int patch_n = n_tiles % 4 == 0 ? 4 : (n_tiles % 2 == 0 ? 2 : 1);
  const int patch_m = 32 / patch_n;
  const int per_group = ((m_tiles + patch_m - 1) / patch_m) * (n_tiles / patch_n);
  const long patches = (long)per_group * n_groups;
  const unsigned blocks = (unsigned)((patches + XCDS - 1) / XCDS) * XCDS * 32;
  hipLaunchKernelGGL(wgrad_gemm_kernel, dim3(blocks), dim3(THREADS), 0, s, (const uint16_t*)P, ldp,
                     (const uint16_t*)Q, ldq, offsets, order, g_begin, n_groups, R_cap, m_tiles, n_tiles, patch_n,
                     n_split, tab, ldc, accumulate ? 1 : 0);
  return hipGetLastError();
}

// order[0 .. n_groups) = the groups of [g_begin, g_begin + n_groups) by descending row count
hipError_t launch_wgrad_order(const int* offsets, int g_begin, int n_groups, int R_cap, int* order, hipStream_t s) {
  hipLaunchKernelGGL(wgrad_order_kernel, dim3(1), dim3(FEPLB_MAX_GROUPS), 0, s, offsets, g_begin, n_groups, R_cap, order);
  return hipGetLastError();
}

// dst + i * group_stride (elements) receives the transpose of src[g_begin + i] ([rows, cols] bf16)
hipError_t launch_transpose(const void* const* src, int g_begin, int n_groups, int rows, int cols, void* dst,
                            size_t group_stride, hipStream_t s) {
  WeightTable tab{};
  for (int i = 0; i < n_groups; ++i) tab.w0[g_begin + i] = src[g_begin + i];
  hipLaunchKernelGGL(transpose_bf16_kernel, dim3(cols / TT, rows / TT, n_groups), dim3(256), 0, s, tab, g_begin,
                     rows, cols, (uint16_t*)dst, group_stride);
  return hipGetLastError();
}

}  // namespace feplb
