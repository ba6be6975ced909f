// Ragged grouped SwiGLU expert FFN on bf16 MFMA (paper Section 3.1: expert
// compute is a Grouped GEMM; Sections 1 and 2.3: its speed depends on each
// expert's batch size and it must not fragment into per-expert launches).
//
// Two GEMM kernels, each ONE launch for a whole range of groups:
//   gate_up : H[r,:]  = bf16( silu(x_r Wg[g]) * (x_r Wu[g]) ),  x_r = Xp[r,:] or, with row_src,
//             the token row X[row_src[r] / k, :] gathered while it is loaded
//   down    : Yp[r,:] = H[r,:] Wd[g]
// The same kernel serves training (Section 3.2 times the backward pass as well): the gate_up
// form can also keep, for the backward pass, the two partial derivatives of its output with
// respect to the products a = x Wg and b = x Wu,
//   p = dH/da = b s (1 + a (1 - s)),   q = dH/db = a s,   s = sigmoid(a)        (bf16),
// and two more forms give the input gradients,
//   dswiglu : dH = dYp Wd^T, then [da | db] = [dH p | dH q], written over [p | q]
//   plain   : dXp = [da | db] [Wg^T; Wu^T]   (the down form with another K)
// with the transposed weights made by a small kernel of ffn_backward.hip, which also holds the
// ragged weight-gradient GEMM.
// A small schedule kernel turns offsets[] (device memory, ragged, possibly
// empty groups) into a table of row tiles; the GEMM grid covers an upper bound
// of tiles and surplus blocks leave at once, so the host never needs R.
//
// Block tile: 256 rows x 256 weight columns x 32 k per step, 4 wavefronts
// (2 x 2), one per SIMD, each 128 x 128 as 4 x 4 MFMA 32x32x16 bf16 tiles
// (256 fp32 accumulators per lane).  For gate_up the 256 weight columns are
// 128 gate + the matching 128 up columns, so the SwiGLU product happens in
// registers and only H is written.  LDS (all 160 KB of a CU) holds six stages of A
// (256 rows x 32 k, k-contiguous) and four of B (32 k x 256 columns, column-contiguous as
// in memory), filled by LDS-DMA loads (global_load_lds_dwordx4: HBM/L2 -> LDS without
// passing through registers) with XOR-swizzled layouts instead of padding; one barrier
// per step; A tiles are requested in pairs that share 128-byte memory lines.
// Weights are row-major [K,N] (N contiguous) as the caller stores them, while
// an MFMA lane needs 8 consecutive k of one column: the B fragments are read
// with the transposing LDS load of gfx950 (ds_read_b64_tr_b16), which hands
// lane i of a 16-lane group the 4 k-values of column i from a 4(k) x 16(n)
// block, so no transpose is done in registers.
// The MFMAs take the weights as their first operand, so a lane ends up with one token row and
// runs of four consecutive output columns; the epilogue passes them through LDS once more so
// that every store instruction writes whole 128-byte lines.
// Blocks are mapped to tiles in 8 x 4 patches per XCD (workgroups are dealt
// round-robin to the 8 XCDs, each with its own L2), so the 32 tiles an XCD
// runs at a time share 8 row panels and 4 weight panels.
#include <mutex>
#include <type_traits>
#include "common.h"
#include "gemm_device.h"

namespace {
using namespace feplb::dev;

constexpr int BM = 256;      // rows per tile
constexpr int BNW = 256;     // weight columns per tile
constexpr int BK = 32;       // k per step
constexpr int NSA = 6;       // LDS stages of the A operand
constexpr int NSB = 4;       // LDS stages of the B operand
constexpr int THREADS = 256;
// LDS: NSA A stages and NSB B stages of 16 KB each (160 KB, all of a CU's LDS); a B stage is two
// parts of 32 k-rows x 256 bytes.
constexpr int A_STAGE_BYTES = BM * BK * 2;
constexpr int B_PART_BYTES = BK * 128 * 2;
constexpr int B_STAGE_BYTES = 2 * B_PART_BYTES;

// ws layout: int4 header {n_tiles,0,0,0}, then int4 {group, row0, rows, 0} per tile
constexpr int SCHED_THREADS = 256;
__global__ __launch_bounds__(SCHED_THREADS) void ffn_schedule_kernel(
    const int* __restrict__ offsets, int g_begin, int g_end, int R_cap, int max_tiles,
    int4* __restrict__ ws) {
  // inclusive scan of the groups' tile counts, then every thread places tiles by binary search
  __shared__ int scan[FEPLB_MAX_GROUPS], lo_s[FEPLB_MAX_GROUPS], hi_s[FEPLB_MAX_GROUPS];
  const int i = threadIdx.x;
  if (i < FEPLB_MAX_GROUPS) {
    const int g = g_begin + i;
    int lo = 0, hi = 0, mt = 0;
    if (g < g_end) {
      lo = min(offsets[g], R_cap);
      hi = min(offsets[g + 1], R_cap);
      mt = hi > lo ? (hi - lo + BM - 1) / BM : 0;
    }
    scan[i] = mt;
    lo_s[i] = lo;
    hi_s[i] = hi;
  }
  __syncthreads();
  for (int d = 1; d < FEPLB_MAX_GROUPS; d <<= 1) {
    int v = 0;
    if (i < FEPLB_MAX_GROUPS && i >= d) v = scan[i - d];
    __syncthreads();
    if (i < FEPLB_MAX_GROUPS) scan[i] += v;
    __syncthreads();
  }
  const int total = min(scan[FEPLB_MAX_GROUPS - 1], max_tiles);
  for (int t = i; t < total; t += SCHED_THREADS) {
    int a = 0, b = FEPLB_MAX_GROUPS - 1;   // first group whose inclusive count exceeds t
    while (a < b) {
      const int m = (a + b) / 2;
      if (scan[m] > t) b = m; else a = m + 1;
    }
    const int first = a ? scan[a - 1] : 0;
    const int row0 = lo_s[a] + (t - first) * BM;
    ws[1 + t] = make_int4(g_begin + a, row0, min(BM, hi_s[a] - row0), 0);
  }
  if (i == 0) ws[0] = make_int4(total, 0, 0, 0);
}

// MODE 0: gate_up (+SwiGLU, bf16 out; with SAVE the derivatives p, q of the SwiGLU product with
//         respect to the gate and up products are also stored, as bf16, in columns [0,N) and
//         [N,2N) of `aux`, for the backward pass);
// MODE 1: plain GEMM (down, or the input gradient), fp32 or bf16 out;
// MODE 2: backward of the SwiGLU product: the GEMM result is dH; `aux` holds the saved
//         derivatives p | q on entry and the gradients da = dH p | db = dH q on exit; `out` is
//         not used.
template <int MODE, bool OUT_BF16, bool SAVE>
__global__ __launch_bounds__(THREADS) void grouped_gemm_kernel(
    const uint16_t* __restrict__ A, int lda, const int* __restrict__ row_src, int n_src_rows, int src_k,
    const int4* __restrict__ sched, int K, int N, int n_tiles_n, int patch_n, WeightTable wt,
    void* __restrict__ out, int ldo, void* aux, int ld_aux) {
  // Separate LDS arrays per stage (not one block with run-time offsets): the compiler can then
  // prove that an LDS-DMA load into one stage and the fragment reads of another stage do not
  // alias, and does not make the reads wait for the loads just issued.
  __shared__ __attribute__((aligned(1024))) char lds_a0[A_STAGE_BYTES];
  __shared__ __attribute__((aligned(1024))) char lds_a1[A_STAGE_BYTES];
  __shared__ __attribute__((aligned(1024))) char lds_a2[A_STAGE_BYTES];
  __shared__ __attribute__((aligned(1024))) char lds_a3[A_STAGE_BYTES];
  __shared__ __attribute__((aligned(1024))) char lds_a4[A_STAGE_BYTES];
  __shared__ __attribute__((aligned(1024))) char lds_a5[A_STAGE_BYTES];
  __shared__ __attribute__((aligned(1024))) char lds_b0[B_STAGE_BYTES];
  __shared__ __attribute__((aligned(1024))) char lds_b1[B_STAGE_BYTES];
  __shared__ __attribute__((aligned(1024))) char lds_b2[B_STAGE_BYTES];
  __shared__ __attribute__((aligned(1024))) char lds_b3[B_STAGE_BYTES];
  auto stage_a = [&](auto st) -> char* {
    return st.value == 0 ? lds_a0 : st.value == 1 ? lds_a1 : st.value == 2 ? lds_a2
         : st.value == 3 ? lds_a3 : st.value == 4 ? lds_a4 : lds_a5;
  };
  auto stage_b = [&](auto st) -> char* {
    return st.value == 0 ? lds_b0 : st.value == 1 ? lds_b1 : st.value == 2 ? lds_b2 : lds_b3;
  };

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

  // ---- global -> LDS, directly (LDS-DMA loads: no register staging, no LDS store instructions)
  // A wavefront-wide 16-byte load writes 1 KB of contiguous LDS, lane l at byte 16*l, so the
  // LDS layouts are swizzled through the choice of the global address each lane reads.
  const int wave = __builtin_amdgcn_readfirstlane(tid / 64), lane = tid % 64;
  // A stage: 256 rows x 64 bytes (32 k).  Load i of wave w fills rows 64w + 16i .. +15; the lane
  // at 16-byte slot p of row r holds k-chunk p ^ ((r >> 2) & 3), which makes the 16-byte
  // fragment reads of 16 consecutive rows hit 16 different bank groups.
  // With row_src the tile's rows are gathered from the unpermuted matrix as they are loaded:
  // row r of the tile is A[row_src[row0 + r] / src_k, :] -- row_src holds flat (token, slot)
  // assignment indices -- and the permute step never has to write a permuted copy.  Rows past the tile's end repeat its last row either way.
  uint32_t a_goff[4];
  const bool gather = MODE == 0 && row_src != nullptr;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = wave * 64 + i * 16 + lane / 4;
    const int chunk = (lane % 4) ^ ((r >> 2) & 3);
    int row = min(r, rows - 1);
    if (gather) row = min(max(row_src[row0 + row] / src_k, 0), n_src_rows - 1);
    a_goff[i] = ((uint32_t)row * (uint32_t)lda + chunk * 8) * 2;
  }
  const char* a_gbase = wave_uniform(gather ? A : A + (size_t)row0 * lda);
  // B stage: two parts (gate | up, or the two column halves) of 32 k-rows x 256 bytes (128
  // columns).  Waves 0,1 fill part 0, waves 2,3 part 1; load i fills k-rows 4q .. 4q+3,
  // q = 4*(w%2) + i.  Inside a row the four 64-byte groups are XOR-ed with (row & 3) so that
  // the transposing reads of 4 consecutive k-rows cover all banks.
  const int part = wave / 2;
  const int b_r = lane / 16;                       // k-row inside the load (= row & 3)
  const int b_slot = ((((lane % 16) >> 2) ^ b_r) << 2) | (lane & 3);   // 16-byte column slot read
  const uint32_t b_goff = ((uint32_t)((wave % 2) * 16 + b_r) * (uint32_t)N + b_slot * 8) * 2;
  const char* b_gbase;
  if (MODE == 0)
    b_gbase = wave_uniform((const uint16_t*)(part ? wt.w1[g] : wt.w0[g]) + (size_t)nt * 128);
  else
    b_gbase = wave_uniform((const uint16_t*)wt.w0[g] + (size_t)nt * 256 + part * 128);
  const size_t b_row_bytes = (size_t)N * 2;

  // one wavefront-wide load (1 KB) of the A / B tile at k0 into `stage`, i = 0..3
  auto issue_a = [&](auto stage, int k0, int i) {
    load_to_lds_16(a_gbase + (size_t)k0 * 2, a_goff[i], lds_offset(stage_a(stage) + wave * 4096 + i * 1024));
  };
  auto issue_b = [&](auto stage, int k0, int i) {
    load_to_lds_16(b_gbase + ((size_t)k0 + 4 * i) * b_row_bytes, b_goff,
                   lds_offset(stage_b(stage) + part * B_PART_BYTES + (wave % 2) * 4096 + i * 1024));
  };

  // ---- wave tiling: 2 x 2 waves, each 128 rows x 128 weight columns
  const int wm = wave / 2, wn = wave % 2;
  const int l32 = lane % 32, h = lane / 32;
  // A fragment (mi, ks): row wm*128 + mi*32 + l32, k-chunk 2*ks + h, at its swizzled slot
  uint32_t a_addr[4][2];
#pragma unroll
  for (int mi = 0; mi < 4; ++mi) {
    const int r = wm * 128 + mi * 32 + l32;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) a_addr[mi][ks] = r * 64 + (((2 * ks + h) ^ ((r >> 2) & 3)) * 16);
  }
  // B fragment (nj, ks): transposing read; lane s of a 16-lane group addresses 4 columns of
  // k-row s/4 and ends up with the 4 k-values of column (lane % 16) of the 16-column block
  uint32_t b_addr[4];
  {
    const int tr_r = h * 8 + (lane % 16) / 4;      // k-row inside the 16-row slice (ks adds 16, the second read 4)
#pragma unroll
    for (int nj = 0; nj < 4; ++nj) {
      const int prt = MODE == 0 ? nj / 2 : wn;
      const int col = (MODE == 0 ? wn * 64 + (nj % 2) * 32 : nj * 32) + ((lane / 16) % 2) * 16 + (lane % 4) * 4;
      const int slot = col / 8;
      const int sw = ((((slot >> 2) ^ (tr_r & 3)) << 2) | (slot & 3));
      b_addr[nj] = prt * B_PART_BYTES + tr_r * 256 + sw * 16 + (col % 8) * 2;
    }
  }

  f32x16 acc[4][4];
#pragma unroll
  for (int mi = 0; mi < 4; ++mi)
#pragma unroll
    for (int nj = 0; nj < 4; ++nj)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[mi][nj][v] = 0.f;

  // fragment registers, double-buffered over the two 16-wide k-slices of a step
  bf16x8 af[2][4];
  i16x4 bl[2][4], bh[2][4];
  // fragment read j of 12: j < 4: A rows block j; else B column block (j-4)/2, k-half (j-4)%2
  auto read_frag = [&](auto sa, auto sb, int ks, int buf, int j) {
    typedef __attribute__((address_space(3))) i16x4 lds_i16x4;
    if (j < 4) {
      af[buf][j] = *(const bf16x8*)(stage_a(sa) + a_addr[j][ks]);
    } else {
      const int nj = (j - 4) / 2;
      const char* p = stage_b(sb) + ks * 16 * 256 + b_addr[nj];
      if ((j - 4) % 2 == 0)
        bl[buf][nj] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4*)p);
      else
        bh[buf][nj] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4*)(p + 4 * 256));
    }
  };
  auto load_frags = [&](auto sa, auto sb, int ks, int buf) {
#pragma unroll
    for (int j = 0; j < 12; ++j) read_frag(sa, sb, ks, buf, j);
  };
  auto mfma16 = [&](int buf) {
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
      for (int nj = 0; nj < 4; ++nj) {
        const bf16x8 b = __builtin_bit_cast(
            bf16x8, __builtin_shufflevector(bl[buf][nj], bh[buf][nj], 0, 1, 2, 3, 4, 5, 6, 7));
        // weights as the first operand: the product comes out transposed, see the epilogue
        acc[mi][nj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, af[buf][mi], acc[mi][nj], 0, 0, 0);
      }
  };

  // Software pipeline over 32-wide k tiles.  Step kt computes tile kt in two halves of 16 MFMAs
  // per wave, from A stage kt % 6 and B stage kt % 4.  Its single barrier sits between the
  // halves: by then every wave holds the last fragments of tile kt in registers and its stages
  // are free.
  //   B: tile kt+3 is requested in the first half of step kt (into the stage freed by step kt-1).
  //   A: a row of a 32-wide tile is 64 bytes, half a 128-byte memory line, and a line fetched
  //      for one tile would be evicted from the vector cache before the next tile asks for its
  //      other half.  So A tiles are requested in pairs (t, t+1), t even, by back-to-back loads
  //      of the two halves of the same lines, which the cache merges into one fetch: row
  //      blocks 0,1 of tiles (kt+5, kt+6) in the second half of an odd step kt, row blocks 2,3
  //      of the same pair in the second half of the next (even) step.  Six A stages hold the
  //      four tiles ahead of the one being computed plus the pair in flight.
  // Every half step thus issues four wavefront-wide loads per 16 MFMAs, an even stream for the
  // address unit.  At the barrier of step kt the 16 most recent loads may still be in flight;
  // the older ones include all of tile kt+1.
  // Loads past the end re-read the last tile (k clamped) into stages nobody reads again, so
  // the loop body has no branches except the exits after every fourth step.
  const int KT = K / BK;   // a multiple of 4: K is a multiple of 128
  const int k_last = K - BK;
  auto kclamp = [&](int kt) { return min(kt * BK, k_last); };
  auto step = [&](auto sc, int kt) {
    constexpr int s = decltype(sc)::value;                       // kt mod 12
    constexpr std::integral_constant<int, s % NSA> a_cur{};
    constexpr std::integral_constant<int, (s + 1) % NSA> a_nxt{};
    constexpr std::integral_constant<int, s % NSB> b_cur{};
    constexpr std::integral_constant<int, (s + 1) % NSB> b_nxt{};
    constexpr std::integral_constant<int, (s + 3) % NSB> b_req{};
    constexpr int pair = (s % 2) ? 5 : 4;                        // first tile of the A pair, relative to kt
    constexpr int q0 = (s % 2) ? 0 : 2;                          // its row blocks requested in this step
    constexpr std::integral_constant<int, (s + pair) % NSA> a_req0{};
    constexpr std::integral_constant<int, (s + pair + 1) % NSA> a_req1{};
    const int kb = kclamp(kt + 3), ka0 = kclamp(kt + pair), ka1 = kclamp(kt + pair + 1);
    // first half: B part of tile kt+3, fragments of k-slice 1, MFMAs of k-slice 0
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      issue_b(b_req, kb, q);
#pragma unroll
      for (int j = 3 * q; j < 3 * q + 3; ++j) read_frag(a_cur, b_cur, 1, 1, j);
    }
    mfma16(0);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // 1 MFMA
      if (i < 12) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);       // 1 LDS read
    }
    __builtin_amdgcn_sched_barrier(0);
    // tile kt+1 has landed (this wave's share; the 16 newer loads may be in flight) and all
    // fragment reads of tile kt are complete
    __builtin_amdgcn_s_waitcnt(0x4070);   // vmcnt(16) lgkmcnt(0)
    __syncthreads();
    // second half: two row blocks of an A pair, first fragments of step kt+1
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      if (q % 2 == 0)
        issue_a(a_req0, ka0, q0 + q / 2);
      else
        issue_a(a_req1, ka1, q0 + q / 2);
#pragma unroll
      for (int j = 3 * q; j < 3 * q + 3; ++j) read_frag(a_nxt, b_nxt, 0, 0, j);
    }
    mfma16(1);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      if (i < 12) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
  };
  constexpr std::integral_constant<int, 0> c0{};
  constexpr std::integral_constant<int, 1> c1{};
  constexpr std::integral_constant<int, 2> c2{};
  constexpr std::integral_constant<int, 3> c3{};
  constexpr std::integral_constant<int, 4> c4{};
  constexpr std::integral_constant<int, 5> c5{};
  constexpr std::integral_constant<int, 6> c6{};
  constexpr std::integral_constant<int, 7> c7{};
  constexpr std::integral_constant<int, 8> c8{};
  constexpr std::integral_constant<int, 9> c9{};
  constexpr std::integral_constant<int, 10> c10{};
  constexpr std::integral_constant<int, 11> c11{};
  // prologue: A pairs (0,1) and (2,3), B tiles 0..2, row blocks 0,1 of the A pair (4,5) -- 32
  // loads.  Their order matters for the counted waits: tile 0 is the first 12 loads, and B
  // tile 1 must have at least 16 loads behind it by the barrier of step 0 (it has 20 with the
  // B loads of that step), as every later tile has in the steady state.
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    issue_a(c0, kclamp(0), q);
    issue_a(c1, kclamp(1), q);
  }
#pragma unroll
  for (int q = 0; q < 4; ++q) issue_b(c0, kclamp(0), q);
#pragma unroll
  for (int q = 0; q < 4; ++q) issue_b(c1, kclamp(1), q);
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    issue_a(c2, kclamp(2), q);
    issue_a(c3, kclamp(3), q);
  }
#pragma unroll
  for (int q = 0; q < 4; ++q) issue_b(c2, kclamp(2), q);
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    issue_a(c4, kclamp(4), q);
    issue_a(c5, kclamp(5), q);
  }
  __builtin_amdgcn_s_waitcnt(0x4f74);   // vmcnt(20): the first 12 loads, tile 0, have landed
  __syncthreads();
  load_frags(c0, c0, 0, 0);
  int kt = 0;
  for (; kt + 12 <= KT; kt += 12) {
    step(c0, kt);
    step(c1, kt + 1);
    step(c2, kt + 2);
    step(c3, kt + 3);
    step(c4, kt + 4);
    step(c5, kt + 5);
    step(c6, kt + 6);
    step(c7, kt + 7);
    step(c8, kt + 8);
    step(c9, kt + 9);
    step(c10, kt + 10);
    step(c11, kt + 11);
  }
  // the remaining 0, 4 or 8 steps (the stage phase is 0 again after whole trips of 12)
  if (kt < KT) {
    step(c0, kt);
    step(c1, kt + 1);
    step(c2, kt + 2);
    step(c3, kt + 3);
    if (kt + 4 < KT) {
      step(c4, kt + 4);
      step(c5, kt + 5);
      step(c6, kt + 6);
      step(c7, kt + 7);
    }
  }
  __builtin_amdgcn_s_waitcnt(0);   // the clamped trailing loads must land before the block ends
  __syncthreads();

  // ---- epilogue.  The MFMAs computed (X W)^T per 32 x 32 block, so a lane holds ONE token row
  // (mi*32 + l32 of the wave's 128) and, in accumulator registers 4c .. 4c+3, FOUR consecutive
  // weight columns 8c + 4*(lane/32) .. +3 of block nj.  Stored straight from there a row's
  // bytes would leave in 8- or 16-byte pieces from different instructions; partial-line writes
  // are slow in the L2.  Instead each wave passes its outputs, 32 rows at a time, through a
  // 16 KB LDS region of its own (the A stages are free now) and reads them back with the lanes
  // laid along the rows, so that every store instruction writes whole 128-byte lines.
  // No barrier: the region is private to the wave and the LDS executes one wave's
  // instructions in order.
  constexpr int COLS = MODE == 0 ? 64 : 128;                    // output columns of this wave
  constexpr int ESZ = (MODE == 0 || MODE == 2 || OUT_BF16) ? 2 : 4;
  constexpr int ROW_BYTES = COLS * ESZ;                         // 128, 256 or 512
  constexpr int CH = ROW_BYTES / 16;                            // 16-byte chunks per row
  constexpr int RPI = 64 / CH;                                  // rows per store instruction
  constexpr int SWZ_DIV = ROW_BYTES >= 256 ? 1 : 256 / ROW_BYTES;
  // chunk q of row r sits at slot q ^ swz(r): spreads a column of pieces over all banks
  auto swz = [&](int r) { return (r / SWZ_DIV) & (CH - 1); };
  char* ep = wave == 0 ? lds_a0 : wave == 1 ? lds_a1 : wave == 2 ? lds_a2 : lds_a3;
  const int csub = (lane / 32) * 4;
  const int col0 = MODE == 0 ? nt * 128 + wn * 64 : nt * 256 + wn * 128;
  const int rd_row = lane / CH, rd_chunk = lane % CH;
  // position of the 8- or 16-byte piece (nj, c) of this lane's row in the staging region
  auto piece = [&](int nj, int c) -> char* {
    const int boff = (nj * 32 + 8 * c + csub) * ESZ;            // byte offset of the piece in its row
    return ep + l32 * ROW_BYTES + ((((boff >> 4) ^ swz(l32))) << 4) + (boff & 15);
  };
  // the 32 staged rows leave as whole lines: lanes laid along the rows
  auto store_lines = [&](int mi, char* dst_wave, int ld_bytes, bool streaming) {
#pragma unroll
    for (int j = 0; j < 32 / RPI; ++j) {
      const int r = j * RPI + rd_row;                            // row inside this pass
      const uint4 v = *(const uint4*)(ep + r * ROW_BYTES + ((rd_chunk ^ swz(r)) << 4));
      if (wm * 128 + mi * 32 + r < rows) {
        u32x4* dst = (u32x4*)(dst_wave + (size_t)(mi * 32 + r) * ld_bytes + rd_chunk * 16);
        const u32x4 vv = {v.x, v.y, v.z, v.w};
        if (streaming) __builtin_nontemporal_store(vv, dst); else *dst = vv;
      }
    }
  };
  if constexpr (MODE == 2) {
    // p | q come in as whole lines, pass through the staging region (p in its first 8 KB, q in
    // the second) to reach the lanes that hold the matching dH values, and leave the same way
    char* aux_wave = (char*)aux + ((size_t)(row0 + wm * 128) * ld_aux + col0) * 2;
    const size_t b_shift = (size_t)N * 2;                        // b sits N columns to the right of a
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) {
      u32x4 la[32 / RPI], lb[32 / RPI];
#pragma unroll
      for (int j = 0; j < 32 / RPI; ++j) {
        const int r = j * RPI + rd_row;
        la[j] = lb[j] = u32x4{0u, 0u, 0u, 0u};
        if (wm * 128 + mi * 32 + r < rows) {
          const char* src = aux_wave + (size_t)(mi * 32 + r) * ld_aux * 2 + rd_chunk * 16;
          la[j] = *(const u32x4*)src;
          lb[j] = *(const u32x4*)(src + b_shift);
        }
      }
#pragma unroll
      for (int j = 0; j < 32 / RPI; ++j) {
        const int r = j * RPI + rd_row;
        char* q = ep + r * ROW_BYTES + ((rd_chunk ^ swz(r)) << 4);
        *(u32x4*)q = la[j];
        *(u32x4*)(q + 8192) = lb[j];
      }
#pragma unroll
      for (int nj = 0; nj < 4; ++nj)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          char* q = piece(nj, c);
          const uint2 pv = *(const uint2*)q, qv = *(const uint2*)(q + 8192);
          const float dp[4] = {bf16_lo(pv.x), bf16_hi(pv.x), bf16_lo(pv.y), bf16_hi(pv.y)};
          const float dq[4] = {bf16_lo(qv.x), bf16_hi(qv.x), bf16_lo(qv.y), bf16_hi(qv.y)};
          float da[4], db[4];
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float dh = acc[mi][nj][4 * c + i];
            da[i] = dh * dp[i];
            db[i] = dh * dq[i];
          }
          *(uint2*)q = make_uint2(pack_bf16(da[0], da[1]), pack_bf16(da[2], da[3]));
          *(uint2*)(q + 8192) = make_uint2(pack_bf16(db[0], db[1]), pack_bf16(db[2], db[3]));
        }
      store_lines(mi, aux_wave, ld_aux * 2, false);
      ep += 8192;
      store_lines(mi, aux_wave + b_shift, ld_aux * 2, false);
      ep -= 8192;
    }
  } else {
    char* out_wave = (char*)out + ((size_t)(row0 + wm * 128) * ldo + col0) * ESZ;
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) {
      if constexpr (MODE == 0 && SAVE) {
        // H and the two derivatives share the sigmoid; the three 4 KB pieces of the pass sit
        // behind each other in the staging region
#pragma unroll
        for (int nj = 0; nj < 2; ++nj)
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            char* dst = piece(nj, c);
            float hv[4], pv[4], qv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const float a = acc[mi][nj][4 * c + i], b = acc[mi][nj + 2][4 * c + i];
              const float sg = __builtin_amdgcn_rcpf(1.0f + __expf(-a));
              qv[i] = a * sg;                              // silu(a) = dH/db
              hv[i] = qv[i] * b;
              pv[i] = b * sg * (1.0f + a - qv[i]);         // dH/da; a (1 - s) = a - a s
            }
            *(uint2*)dst = make_uint2(pack_bf16(hv[0], hv[1]), pack_bf16(hv[2], hv[3]));
            *(uint2*)(dst + 4096) = make_uint2(pack_bf16(pv[0], pv[1]), pack_bf16(pv[2], pv[3]));
            *(uint2*)(dst + 8192) = make_uint2(pack_bf16(qv[0], qv[1]), pack_bf16(qv[2], qv[3]));
          }
        char* aux_wave = (char*)aux + ((size_t)(row0 + wm * 128) * ld_aux + col0) * 2;
        store_lines(mi, out_wave, ldo * ESZ, false);
        ep += 4096;
        store_lines(mi, aux_wave, ld_aux * 2, false);
        ep += 4096;
        store_lines(mi, aux_wave + (size_t)N * 2, ld_aux * 2, false);
        ep -= 8192;
      } else {
#pragma unroll
        for (int nj = 0; nj < (MODE == 0 ? 2 : 4); ++nj)
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            char* dst = piece(nj, c);
            float v[4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
              v[i] = MODE == 0 ? silu(acc[mi][nj][4 * c + i]) * acc[mi][nj + 2][4 * c + i] : acc[mi][nj][4 * c + i];
            if (ESZ == 2)
              *(uint2*)dst = make_uint2(pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]));
            else
              *(float4*)dst = make_float4(v[0], v[1], v[2], v[3]);
          }
        store_lines(mi, out_wave, ldo * ESZ, MODE == 1 && !OUT_BF16);
      }
    }
  }
}

int max_tiles_for(int R_cap, int ng) { return R_cap / BM + ng + 1; }

template <int MODE, bool OUT_BF16, bool SAVE = false>
hipError_t launch_gemm(const void* A, int lda, const int* row_src, int n_src_rows, int src_k, const int4* sched,
                       int K, int N, int n_tiles_n, int max_tiles, const WeightTable& wt, void* out,
                       int ldo, hipStream_t s, void* aux = nullptr, int ld_aux = 0) {
  const int patch_n = n_tiles_n % 4 == 0 ? 4 : (n_tiles_n % 2 == 0 ? 2 : 1);
  const int patch_m = 32 / patch_n;
  const int patches_m = (max_tiles + patch_m - 1) / patch_m;
  const int patches = patches_m * (n_tiles_n / patch_n);
  const int patch_rounds = (patches + XCDS - 1) / XCDS;
  const unsigned blocks = (unsigned)patch_rounds * XCDS * 32;
  hipLaunchKernelGGL((grouped_gemm_kernel<MODE, OUT_BF16, SAVE>), dim3(blocks), dim3(THREADS), 0,
                     s, (const uint16_t*)A, lda, row_src, n_src_rows, src_k, sched, K, N, n_tiles_n, patch_n, wt,
                     out, ldo, aux, ld_aux);
  return hipGetLastError();
}

// workspace: the tile table, then (backward pass only) the groups ordered by row count
size_t table_bytes(int R_cap, int ng) { return (size_t)(1 + max_tiles_for(R_cap, ng)) * sizeof(int4); }

}  // namespace

extern "C" size_t feplb_grouped_ffn_workspace_bytes(int32_t R_cap, int32_t G) {
  if (R_cap < 0 || G < 0) return 0;
  return table_bytes(R_cap, G) + FEPLB_MAX_GROUPS * sizeof(int);
}

namespace {
int32_t forward_impl(const void* Xp, const int32_t* row_src, int32_t T, int32_t k,
                     const int32_t* offsets, int32_t g_begin,
                     int32_t g_end, int32_t R_cap, int32_t d, int32_t f,
                     const void* const* w_gate, const void* const* w_up,
                     const void* const* w_down, void* H, void* AB, void* Yp,
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
  // (both k extents, d and f, are then multiples of 128: the k loop runs two 64-wide steps per trip)
  FEPLB_REQUIRE(d % 256 == 0 && f % 128 == 0 && d > 0 && f > 0, FEPLB_ESHAPE,
                "grouped_ffn: need d %% 256 == 0 and f %% 128 == 0 (d=%d f=%d)", d, f);
  const int ng = g_end - g_begin;
  if (ng == 0 || R_cap == 0) return FEPLB_OK;
  FEPLB_REQUIRE(offsets, FEPLB_EINVAL, "grouped_ffn: null offsets");
  const bool do_up = phases & FEPLB_FFN_GATE_UP, do_down = phases & FEPLB_FFN_DOWN;
  if (do_up) {
    FEPLB_REQUIRE(Xp && H && w_gate && w_up, FEPLB_EINVAL, "grouped_ffn: null Xp/H/w_gate/w_up");
    if (row_src) {
      // the kernel addresses a gathered row as a 32-bit byte offset from X
      FEPLB_REQUIRE(T > 0 && k > 0 && (uint64_t)T * (uint64_t)d * 2 <= 0xffffffffull, FEPLB_ESHAPE,
                    "grouped_ffn: gathering needs T > 0, k > 0 and T*d*2 < 4 GiB (T=%d k=%d d=%d)", T, k, d);
    }
    FEPLB_REQUIRE(feplb::aligned16(Xp) && feplb::aligned16(H) && feplb::aligned16(AB), FEPLB_EALIGN,
                  "grouped_ffn: Xp/H/AB not 16-byte aligned");
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
    hipLaunchKernelGGL(ffn_schedule_kernel, dim3(1), dim3(SCHED_THREADS), 0, s, offsets,
                       g_begin, g_end, R_cap, max_tiles, (int4*)ws);
    FEPLB_LAUNCH_CHECK("ffn_schedule_kernel");
  }
  if (do_up) {
    if (AB)
      FEPLB_HIP((launch_gemm<0, true, true>(Xp, d, row_src, T, k, (const int4*)ws, d, f, f / 128, max_tiles, up_tab, H, f, s, AB, 2 * f)));
    else
      FEPLB_HIP((launch_gemm<0, true>(Xp, d, row_src, T, k, (const int4*)ws, d, f, f / 128, max_tiles, up_tab, H, f, s)));
  }
  if (do_down) {
    if (yp_dtype == FEPLB_BF16)
      FEPLB_HIP((launch_gemm<1, true>(H, f, nullptr, 0, 1, (const int4*)ws, f, d, d / 256, max_tiles, down_tab, Yp, d, s)));
    else
      FEPLB_HIP((launch_gemm<1, false>(H, f, nullptr, 0, 1, (const int4*)ws, f, d, d / 256, max_tiles, down_tab, Yp, d, s)));
  }
  return FEPLB_OK;
}
}  // namespace

extern "C" int32_t feplb_grouped_ffn(const void* Xp, const int32_t* row_src, int32_t T, int32_t k,
                                     const int32_t* offsets, int32_t g_begin,
                                     int32_t g_end, int32_t R_cap, int32_t d, int32_t f,
                                     const void* const* w_gate, const void* const* w_up,
                                     const void* const* w_down, void* H, void* Yp,
                                     int32_t yp_dtype, int32_t phases, void* ws, size_t ws_bytes,
                                     void* stream) {
  return forward_impl(Xp, row_src, T, k, offsets, g_begin, g_end, R_cap, d, f, w_gate, w_up, w_down, H,
                      nullptr, Yp, yp_dtype, phases, ws, ws_bytes, stream);
}

// ---- the forward call for callers that cannot allocate: its tile table lives in device memory
// that belongs to the library's code object instead of a caller's workspace
namespace {
static __device__ __align__(256) unsigned char scratch[FEPLB_STATIC_WS_BYTES];

constexpr int MAX_DEVICES = 64;
void* g_scratch_ptr[MAX_DEVICES];   // this process's address of `scratch` on each device, once known
std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device.  In host code the array's name is only a
// handle for the runtime, not a device address: every use below goes through this pointer.
int32_t static_scratch(void** out) {
  int dev = -1;
  FEPLB_HIP(hipGetDevice(&dev));
  FEPLB_REQUIRE(dev >= 0 && dev < MAX_DEVICES, FEPLB_ESHAPE, "grouped_ffn_static: device %d above %d", dev, MAX_DEVICES);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    FEPLB_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    FEPLB_REQUIRE(p && feplb::aligned16(p), FEPLB_EHIP, "grouped_ffn_static: no device address for the scratch array");
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return FEPLB_OK;
}
}  // namespace

extern "C" int32_t feplb_grouped_ffn_static(const void* Xp, const int32_t* row_src, int32_t T, int32_t k,
                                            const int32_t* offsets, int32_t g_begin, int32_t g_end,
                                            int32_t R_cap, int32_t d, int32_t f, const void* const* w_gate,
                                            const void* const* w_up, const void* const* w_down, void* H,
                                            void* Yp, int32_t yp_dtype, int32_t phases, void* stream) {
  FEPLB_REQUIRE(g_begin >= 0 && g_end >= g_begin && R_cap >= 0, FEPLB_EINVAL,
                "grouped_ffn_static: negative size or empty range reversed");
  const size_t need = feplb_grouped_ffn_workspace_bytes(R_cap, g_end - g_begin);
  FEPLB_REQUIRE(need <= (size_t)FEPLB_STATIC_WS_BYTES, FEPLB_ESHAPE,
                "grouped_ffn_static: R_cap=%d rows in %d groups need %zu bytes of tile table, the built-in scratch "
                "holds %d; use feplb_grouped_ffn with a workspace", R_cap, g_end - g_begin, need, FEPLB_STATIC_WS_BYTES);
  void* ws = nullptr;
  const int32_t rc = static_scratch(&ws);
  if (rc != FEPLB_OK) return rc;
  return forward_impl(Xp, row_src, T, k, offsets, g_begin, g_end, R_cap, d, f, w_gate, w_up, w_down, H,
                      nullptr, Yp, yp_dtype, phases, ws, FEPLB_STATIC_WS_BYTES, stream);
}

extern "C" int32_t feplb_grouped_ffn_train(const void* Xp, const int32_t* row_src, int32_t T, int32_t k,
                                           const int32_t* offsets, int32_t g_begin,
                                           int32_t g_end, int32_t R_cap, int32_t d, int32_t f,
                                           const void* const* w_gate, const void* const* w_up,
                                           const void* const* w_down, void* H, void* AB, void* Yp,
                                           int32_t yp_dtype, int32_t phases, void* ws, size_t ws_bytes,
                                           void* stream) {
  FEPLB_REQUIRE(AB || !(phases & FEPLB_FFN_GATE_UP), FEPLB_EINVAL, "grouped_ffn_train: null AB");
  return forward_impl(Xp, row_src, T, k, offsets, g_begin, g_end, R_cap, d, f, w_gate, w_up, w_down, H,
                      AB, Yp, yp_dtype, phases, ws, ws_bytes, stream);
}

extern "C" size_t feplb_grouped_ffn_backward_wt_bytes(int32_t n_groups, int32_t d, int32_t f) {
  if (n_groups < 0 || d < 0 || f < 0) return 0;
  return (size_t)n_groups * 3 * (size_t)d * (size_t)f * 2;
}

extern "C" int32_t feplb_grouped_ffn_backward(const void* Xp, const int32_t* offsets, int32_t g_begin,
                                              int32_t g_end, int32_t R_cap, int32_t d, int32_t f,
                                              const void* const* w_gate, const void* const* w_up,
                                              const void* const* w_down, const void* H, void* AB,
                                              const void* dYp, void* dXp, int32_t dxp_dtype,
                                              void* const* dw_gate, void* const* dw_up,
                                              void* const* dw_down, void* WT, size_t wt_bytes,
                                              int32_t phases, void* ws, size_t ws_bytes, void* stream) {
  FEPLB_REQUIRE(g_begin >= 0 && g_end >= g_begin && R_cap >= 0 && d >= 0 && f >= 0, FEPLB_EINVAL,
                "grouped_ffn_backward: negative size or empty range reversed");
  FEPLB_REQUIRE(g_end <= FEPLB_MAX_GROUPS, FEPLB_ESHAPE, "grouped_ffn_backward: g_end=%d above %d", g_end,
                FEPLB_MAX_GROUPS);
  FEPLB_REQUIRE((phases & ~(FEPLB_BWD_ALL | FEPLB_BWD_ACCUMULATE)) == 0 && (phases & FEPLB_BWD_ALL) != 0, FEPLB_EINVAL,
                "grouped_ffn_backward: phases=%d", phases);
  FEPLB_REQUIRE(dxp_dtype == FEPLB_F32 || dxp_dtype == FEPLB_BF16, FEPLB_EINVAL,
                "grouped_ffn_backward: unknown dxp_dtype %d", dxp_dtype);
  FEPLB_REQUIRE(d % 256 == 0 && f % 256 == 0 && d > 0 && f > 0, FEPLB_ESHAPE,
                "grouped_ffn_backward: need d %% 256 == 0 and f %% 256 == 0 (d=%d f=%d)", d, f);
  const int ng = g_end - g_begin;
  if (ng == 0) return FEPLB_OK;
  const bool do_t = phases & FEPLB_BWD_TRANSPOSE, do_d = phases & FEPLB_BWD_DGRAD, do_w = phases & FEPLB_BWD_WGRAD;
  // the weight-gradient kernel reads whole windows of 32 rows and runs for empty inputs too
  // (it writes the zero gradients), so the row buffers must hold at least one window
  FEPLB_REQUIRE(!do_w || R_cap >= 32, FEPLB_ESHAPE, "grouped_ffn_backward: WGRAD needs R_cap >= 32 (R_cap=%d)", R_cap);
  FEPLB_REQUIRE(offsets, FEPLB_EINVAL, "grouped_ffn_backward: null offsets");
  // column offsets inside a row travel as 32-bit byte offsets
  FEPLB_REQUIRE((uint64_t)(2 * (size_t)f + d) * 64 * 2 <= 0xffffffffull, FEPLB_ESHAPE, "grouped_ffn_backward: d, f too large");
  if (do_t) {
    FEPLB_REQUIRE(w_gate && w_up && w_down, FEPLB_EINVAL, "grouped_ffn_backward: null weight tables");
    for (int g = g_begin; g < g_end; ++g) {
      FEPLB_REQUIRE(w_gate[g] && w_up[g] && w_down[g], FEPLB_EINVAL, "grouped_ffn_backward: null weights of group %d", g);
      FEPLB_REQUIRE(feplb::aligned16(w_gate[g]) && feplb::aligned16(w_up[g]) && feplb::aligned16(w_down[g]),
                    FEPLB_EALIGN, "grouped_ffn_backward: weights of group %d not 16-byte aligned", g);
    }
  }
  if (do_t || do_d) {
    const size_t need_wt = feplb_grouped_ffn_backward_wt_bytes(ng, d, f);
    FEPLB_REQUIRE(WT && wt_bytes >= need_wt, FEPLB_EWORKSPACE, "grouped_ffn_backward: WT %zu < %zu", wt_bytes, need_wt);
    FEPLB_REQUIRE(feplb::aligned16(WT), FEPLB_EALIGN, "grouped_ffn_backward: WT not 16-byte aligned");
  }
  if (do_d) {
    FEPLB_REQUIRE(AB && dYp && dXp, FEPLB_EINVAL, "grouped_ffn_backward: null AB/dYp/dXp");
    FEPLB_REQUIRE(feplb::aligned16(AB) && feplb::aligned16(dYp) && feplb::aligned16(dXp), FEPLB_EALIGN,
                  "grouped_ffn_backward: AB/dYp/dXp not 16-byte aligned");
  }
  if (do_w) {
    FEPLB_REQUIRE(Xp && H && AB && dYp && dw_gate && dw_up && dw_down, FEPLB_EINVAL,
                  "grouped_ffn_backward: null Xp/H/AB/dYp or gradient tables");
    FEPLB_REQUIRE(feplb::aligned16(Xp) && feplb::aligned16(H) && feplb::aligned16(AB) && feplb::aligned16(dYp),
                  FEPLB_EALIGN, "grouped_ffn_backward: Xp/H/AB/dYp not 16-byte aligned");
    for (int g = g_begin; g < g_end; ++g) {
      FEPLB_REQUIRE(dw_gate[g] && dw_up[g] && dw_down[g], FEPLB_EINVAL, "grouped_ffn_backward: null gradient of group %d", g);
      FEPLB_REQUIRE(feplb::aligned16(dw_gate[g]) && feplb::aligned16(dw_up[g]) && feplb::aligned16(dw_down[g]),
                    FEPLB_EALIGN, "grouped_ffn_backward: gradient of group %d not 16-byte aligned", g);
    }
  }
  const int max_tiles = max_tiles_for(R_cap, ng);
  const size_t order_at = table_bytes(R_cap, ng);
  {
    const size_t need = order_at + FEPLB_MAX_GROUPS * sizeof(int);
    FEPLB_REQUIRE(ws && ws_bytes >= need, FEPLB_EWORKSPACE, "grouped_ffn_backward: workspace %zu < %zu", ws_bytes, need);
    FEPLB_REQUIRE(feplb::aligned16(ws), FEPLB_EALIGN, "grouped_ffn_backward: workspace not 16-byte aligned");
  }
  hipStream_t s = (hipStream_t)stream;
  const size_t df = (size_t)d * f;
  if ((phases & FEPLB_BWD_SCHEDULE) && R_cap > 0) {
    hipLaunchKernelGGL(ffn_schedule_kernel, dim3(1), dim3(SCHED_THREADS), 0, s, offsets, g_begin, g_end, R_cap,
                       max_tiles, (int4*)ws);
    FEPLB_LAUNCH_CHECK("ffn_schedule_kernel");
  }
  // the order in which the weight-gradient grid walks the groups is rebuilt by every WGRAD call
  if (do_w && R_cap > 0)
    FEPLB_HIP(feplb::launch_wgrad_order(offsets, g_begin, ng, R_cap, (int*)((char*)ws + order_at), s));
  const int* order = (const int*)((const char*)ws + order_at);
  if (do_t) {
    // per group: Wd^T [d,f], then Wg^T [f,d] and Wu^T [f,d], the last two forming [2f,d]
    uint16_t* wt0 = (uint16_t*)WT;
    FEPLB_HIP(feplb::launch_transpose(w_down, g_begin, ng, f, d, wt0, 3 * df, s));
    FEPLB_HIP(feplb::launch_transpose(w_gate, g_begin, ng, d, f, wt0 + df, 3 * df, s));
    FEPLB_HIP(feplb::launch_transpose(w_up, g_begin, ng, d, f, wt0 + 2 * df, 3 * df, s));
  }
  WeightTable dT{}, guT{};
  for (int g = g_begin; g < g_end; ++g) {
    const uint16_t* base = (const uint16_t*)WT + (size_t)(g - g_begin) * 3 * df;
    dT.w0[g] = base;
    guT.w0[g] = base + df;
  }
  if (do_w && R_cap > 0)   // dW_down = H^T dYp: before DGRAD, which does not touch H or dYp
    FEPLB_HIP(feplb::launch_wgrad(H, f, f, dYp, d, d, offsets, order, g_begin, ng, R_cap, dw_down, nullptr, d, d, phases & FEPLB_BWD_ACCUMULATE, s));
  if (do_d && R_cap > 0)   // dH = dYp Wd^T, turned into [da | db] in place over the saved [a | b]
    FEPLB_HIP((launch_gemm<2, true>(dYp, d, nullptr, 0, 1, (const int4*)ws, d, f, f / 256, max_tiles, dT, nullptr, 0, s, AB, 2 * f)));
  if (do_w && R_cap > 0)   // [dW_gate | dW_up] = Xp^T [da | db]
    FEPLB_HIP(feplb::launch_wgrad(Xp, d, d, AB, 2 * f, 2 * f, offsets, order, g_begin, ng, R_cap, dw_gate, dw_up, f, f, phases & FEPLB_BWD_ACCUMULATE, s));
  if (do_d && R_cap > 0) {   // dXp = [da | db] [Wg^T; Wu^T]
    if (dxp_dtype == FEPLB_BF16)
      FEPLB_HIP((launch_gemm<1, true>(AB, 2 * f, nullptr, 0, 1, (const int4*)ws, 2 * f, d, d / 256, max_tiles, guT, dXp, d, s)));
    else
      FEPLB_HIP((launch_gemm<1, false>(AB, 2 * f, nullptr, 0, 1, (const int4*)ws, 2 * f, d, d / 256, max_tiles, guT, dXp, d, s)));
  }
  return FEPLB_OK;
}
