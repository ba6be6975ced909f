// Permute: group the rank's token rows by static / dynamic expert group
// (paper Section 2.2 Phase 1: tokens are permuted by expert where they will be
// computed; Section 2.3: static vs dynamic experts).
//
// The row order is fully determined (groups in table order, ascending flat
// assignment inside a group), so no atomics may decide a row position.  It is a
// stable counting sort over the flat assignments a = t*k + j, split in chunks
// of 256 or 1024 assignments (by batch size), one wavefront per chunk:
//   1. chunk_hist : per-chunk, per-expert counts (LDS histogram per wave)
//   2. chunk_scan : per expert, exclusive prefix over chunks -> the ordinal of
//                   the first occurrence in each chunk, and the expert's total
//   3. group_offsets : sizes of the ordinal windows -> offsets[G+1]; per-expert
//                   chains of groups for the lookup in step 4
//   4. assign_rows: per chunk, walk 64 assignments at a time; the ordinal inside
//                   the slice comes from a ballot-based match of equal experts,
//                   the running ordinal per expert lives in LDS; the window
//                   that contains the ordinal gives the row
//   5. gather_rows: Xp[r,:] = X[row_src[r] / k, :], one wavefront per row,
//                   16-byte lanes (pure HBM traffic: 2*R*d*2 bytes)
#include "common.h"

namespace {

// assignments per wavefront: small batches get shorter chunks, i.e. more wavefronts for the
// serial walk of assign_rows (a multiple of 64 either way)
int chunk_for(long long A) { return A <= (1ll << 18) ? 256 : 1024; }
constexpr int WAVES = 4;             // wavefronts per block
constexpr int BLOCK = WAVES * 64;

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

struct GroupTable {
  feplb_group g[FEPLB_MAX_GROUPS];
};

__global__ __launch_bounds__(BLOCK) void chunk_hist_kernel(const int* __restrict__ ids,
                                                           long long A, int E, int nchunks, int chunk,
                                                           int* __restrict__ chunk_hist) {
  extern __shared__ int lds[];
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
  int* h = lds + wave * E;
  const int c = blockIdx.x * WAVES + wave;
  for (int e = lane; e < E; e += 64) h[e] = 0;
  __builtin_amdgcn_wave_barrier();
  if (c < nchunks) {
    const long long a0 = (long long)c * chunk;
    for (int i = lane; i < chunk; i += 64) {
      const long long a = a0 + i;
      if (a < A) {
        const int e = ids[a];
        if ((unsigned)e < (unsigned)E) atomicAdd(&h[e], 1);
      }
    }
  }
  __syncthreads();
  if (c < nchunks)
    for (int e = lane; e < E; e += 64) chunk_hist[(long long)c * E + e] = h[e];
}

// One wavefront per expert; lane l owns a contiguous run of chunks.
__global__ __launch_bounds__(BLOCK) void chunk_scan_kernel(int* __restrict__ chunk_hist, int E,
                                                           int nchunks, int* __restrict__ total) {
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
  const int e = blockIdx.x * WAVES + wave;
  if (e >= E) return;
  const int per = (nchunks + 63) / 64;
  const int c0 = lane * per;
  const int c1 = min(c0 + per, nchunks);
  int sum = 0;
  for (int c = c0; c < c1; ++c) sum += chunk_hist[(long long)c * E + e];
  int incl = sum;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const int o = __shfl_up(incl, d, 64);
    if (lane >= d) incl += o;
  }
  int run = incl - sum;
  for (int c = c0; c < c1; ++c) {
    const int v = chunk_hist[(long long)c * E + e];
    chunk_hist[(long long)c * E + e] = run;
    run += v;
  }
  if (lane == 63) total[e] = incl;
}

// meta layout (ints): head[E] | next[G] | lo[G] | hi[G] | start[G]
__global__ __launch_bounds__(FEPLB_MAX_GROUPS) void group_offsets_kernel(
    GroupTable tab, int G, int E, const int* __restrict__ total, int* offsets,
    int* __restrict__ meta, int append) {
  __shared__ int scan[FEPLB_MAX_GROUPS];
  const int g = threadIdx.x;
  // appending: the rows of these groups follow those of an earlier call, whose end is offsets[0]
  const int base = append ? offsets[0] : 0;
  __syncthreads();   // every thread has read the base before offsets[0] is written again
  int size = 0, lo = 0, hi = 0, e = -1;
  if (g < G) {
    e = tab.g[g].expert;
    lo = tab.g[g].ord_lo;
    hi = tab.g[g].ord_hi;
    const int n = ((unsigned)e < (unsigned)E) ? total[e] : 0;
    size = max(0, min(hi, n) - min(lo, n));
  }
  scan[g] = size;
  __syncthreads();
  for (int d = 1; d < FEPLB_MAX_GROUPS; d <<= 1) {
    const int v = g >= d ? scan[g - d] : 0;
    __syncthreads();
    scan[g] += v;
    __syncthreads();
  }
  int* head = meta;
  int* next = meta + E;
  int* glo = next + G;
  int* ghi = glo + G;
  int* gstart = ghi + G;
  if (g < G) {
    const int off = base + scan[g] - size;
    offsets[g] = off;
    glo[g] = lo;
    ghi[g] = hi;
    gstart[g] = off - lo;  // row = start + ordinal
    if (g == G - 1) offsets[G] = base + scan[g];
  }
  if (G == 0 && g == 0) offsets[0] = base;
  for (int i = g; i < E; i += FEPLB_MAX_GROUPS) head[i] = -1;
  __syncthreads();
  if (g == 0) {
    for (int i = G - 1; i >= 0; --i) {
      const int ei = tab.g[i].expert;
      if ((unsigned)ei < (unsigned)E) {
        next[i] = head[ei];
        head[ei] = i;
      } else {
        next[i] = -1;
      }
    }
  }
}

__global__ __launch_bounds__(BLOCK) void assign_rows_kernel(
    const int* __restrict__ ids, long long A, int E, int G, int nchunks, int chunk,
    const int* __restrict__ chunk_base, const int* __restrict__ meta, int R_cap,
    int* __restrict__ row_src, int* __restrict__ inv, int append) {
  extern __shared__ int lds[];
  // LDS: run[WAVES][E] | head[E] | next[G] lo[G] hi[G] start[G]
  volatile int* run_all = lds;
  int* head = lds + WAVES * E;
  int* next = head + E;
  int* glo = next + G;
  int* ghi = glo + G;
  int* gstart = ghi + G;
  for (int i = threadIdx.x; i < E + 4 * G; i += BLOCK) head[i] = meta[i];
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
  const int c = blockIdx.x * WAVES + wave;
  volatile int* run = run_all + wave * E;
  if (c < nchunks)
    for (int e = lane; e < E; e += 64) run[e] = chunk_base[(long long)c * E + e];
  __syncthreads();
  if (c >= nchunks) return;
  int nbits = 0;
  while ((1 << nbits) < E) ++nbits;
  const long long a0 = (long long)c * chunk;
  const unsigned long long below = (1ull << lane) - 1ull;
  for (int i = 0; i < chunk; i += 64) {
    const long long a = a0 + i + lane;
    if (a0 + i >= A) break;  // uniform across the wave
    int e = -1;
    if (a < A) {
      e = ids[a];
      if ((unsigned)e >= (unsigned)E) e = -1;
    }
    const bool valid = e >= 0;
    unsigned long long same = __ballot(valid);
    for (int b = 0; b < nbits; ++b) {
      const bool bit = (e >> b) & 1;
      const unsigned long long m = __ballot(bit);
      same &= bit ? m : ~m;
    }
    int row = -1;
    if (valid) {
      const int base = run[e];
      const int o = base + __popcll(same & below);
      if ((same >> lane) == 1ull) run[e] = base + __popcll(same);  // highest lane of the set
      for (int g = head[e]; g >= 0; g = next[g])
        if (o >= glo[g] && o < ghi[g]) {
          row = gstart[g] + o;
          break;
        }
    }
    __builtin_amdgcn_wave_barrier();
    if (a < A) {
      if (!append || row >= 0) inv[a] = row;   // appending leaves the other calls' entries alone
      if (row >= 0 && row < R_cap) row_src[row] = (int)a;
    }
  }
}

// One wavefront per row and per workgroup: measured against 2, 4 and 8 rows per workgroup at
// d = 6144, single-wave workgroups copy 2 % faster (5.60 against 5.48 TB/s).
template <int UNROLL>
__global__ __launch_bounds__(64) void gather_rows_kernel(const u32x4* __restrict__ X,
                                                            const int* __restrict__ row_src,
                                                            const int* __restrict__ offsets, int G,
                                                            int k, int nvec, int R_cap,
                                                            u32x4* __restrict__ Xp) {
  const int lane = threadIdx.x;
  const long long r = blockIdx.x;
  const int R = min(offsets[G], R_cap);
  if (r < offsets[0] || r >= R) return;   // offsets[0] > 0 only for an appending call
  const long long t = row_src[r] / k;
  const u32x4* src = X + t * nvec;
  u32x4* dst = Xp + r * nvec;
  for (int v0 = 0; v0 < nvec; v0 += 64 * UNROLL) {
    u32x4 p[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const int v = v0 + u * 64 + lane;
      if (v < nvec) p[u] = __builtin_nontemporal_load(src + v);
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const int v = v0 + u * 64 + lane;
      if (v < nvec) {
        __builtin_nontemporal_store(p[u], dst + v);   // written once, read by a later kernel
      }
    }
  }
}

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct Layout {
  int nchunks, chunk;
  size_t hist_off, total_off, meta_off, bytes;
};

Layout layout(long long A, int E, int G) {
  Layout L;
  L.chunk = chunk_for(A);
  L.nchunks = (int)((A + L.chunk - 1) / L.chunk);
  size_t off = 0;
  L.hist_off = off;
  off = align_up(off + (size_t)(L.nchunks > 0 ? L.nchunks : 1) * E * sizeof(int), 256);
  L.total_off = off;
  off = align_up(off + (size_t)E * sizeof(int), 256);
  L.meta_off = off;
  off = align_up(off + ((size_t)E + 4 * (size_t)(G > 0 ? G : 1)) * sizeof(int), 256);
  L.bytes = off;
  return L;
}

}  // namespace

extern "C" size_t feplb_permute_workspace_bytes(int32_t T, int32_t k, int32_t E, int32_t G) {
  if (T < 0 || k < 1 || E < 1 || G < 0) return 0;
  return layout((long long)T * k, E, G).bytes;
}

namespace {
int32_t permute_impl(const int32_t* topk_ids, int32_t T, int32_t k, int32_t E,
                     const feplb_group* groups, int32_t G, const void* X, int32_t d,
                     void* Xp, int32_t R_cap, int32_t* offsets, int32_t* row_src,
                     int32_t* inv, void* ws, size_t ws_bytes, void* stream, int append) {
  FEPLB_REQUIRE(T >= 0 && k >= 1 && E >= 1 && G >= 0 && R_cap >= 0 && d >= 0, FEPLB_EINVAL,
                "permute: negative size");
  FEPLB_REQUIRE(E <= FEPLB_MAX_EXPERTS && G <= FEPLB_MAX_GROUPS && k <= FEPLB_MAX_TOPK,
                FEPLB_ESHAPE, "permute: E=%d G=%d k=%d above the limits", E, G, k);
  const long long A = (long long)T * k;
  FEPLB_REQUIRE(A < (1ll << 31), FEPLB_ESHAPE, "permute: T*k does not fit int32");
  FEPLB_REQUIRE(offsets, FEPLB_EINVAL, "permute: null offsets");
  FEPLB_REQUIRE(groups || G == 0, FEPLB_EINVAL, "permute: null groups");
  FEPLB_REQUIRE((topk_ids && inv) || A == 0, FEPLB_EINVAL, "permute: null ids/inv");
  FEPLB_REQUIRE(row_src || R_cap == 0, FEPLB_EINVAL, "permute: null row_src");
  FEPLB_REQUIRE(X || !Xp || A == 0 || d == 0, FEPLB_EINVAL, "permute: Xp given without X");
  if (X && Xp) {
    FEPLB_REQUIRE(d % 8 == 0, FEPLB_ESHAPE, "permute: d=%d not a multiple of 8", d);
    FEPLB_REQUIRE(feplb::aligned16(X) && feplb::aligned16(Xp), FEPLB_EALIGN,
                  "permute: X/Xp not 16-byte aligned");
  }
  GroupTable tab;
  for (int g = 0; g < G; ++g) {
    FEPLB_REQUIRE(groups[g].ord_lo >= 0 && groups[g].ord_hi >= groups[g].ord_lo, FEPLB_EINVAL,
                  "permute: group %d has window [%d,%d)", g, groups[g].ord_lo, groups[g].ord_hi);
    FEPLB_REQUIRE(groups[g].expert >= 0 && groups[g].expert < E, FEPLB_EINVAL,
                  "permute: group %d names expert %d", g, groups[g].expert);
    for (int h = 0; h < g; ++h)
      if (groups[h].expert == groups[g].expert) {
        const bool apart =
            groups[h].ord_hi <= groups[g].ord_lo || groups[g].ord_hi <= groups[h].ord_lo;
        FEPLB_REQUIRE(apart, FEPLB_EINVAL, "permute: groups %d and %d overlap on expert %d", h, g,
                      groups[g].expert);
      }
    tab.g[g] = groups[g];
  }
  const Layout L = layout(A, E, G);
  FEPLB_REQUIRE(ws && ws_bytes >= L.bytes, FEPLB_EWORKSPACE, "permute: workspace %zu < %zu",
                ws_bytes, L.bytes);
  FEPLB_REQUIRE(feplb::aligned16(ws), FEPLB_EALIGN, "permute: workspace not 16-byte aligned");
  hipStream_t s = (hipStream_t)stream;
  char* base = (char*)ws;
  int* hist = (int*)(base + L.hist_off);
  int* total = (int*)(base + L.total_off);
  int* meta = (int*)(base + L.meta_off);
  const int cblocks = (L.nchunks + WAVES - 1) / WAVES;
  if (L.nchunks > 0) {
    hipLaunchKernelGGL(chunk_hist_kernel, dim3(cblocks), dim3(BLOCK),
                       (size_t)WAVES * E * sizeof(int), s, topk_ids, A, E, L.nchunks, L.chunk, hist);
    FEPLB_LAUNCH_CHECK("chunk_hist_kernel");
  }
  hipLaunchKernelGGL(chunk_scan_kernel, dim3((E + WAVES - 1) / WAVES), dim3(BLOCK), 0, s, hist, E,
                     L.nchunks, total);
  FEPLB_LAUNCH_CHECK("chunk_scan_kernel");
  hipLaunchKernelGGL(group_offsets_kernel, dim3(1), dim3(FEPLB_MAX_GROUPS), 0, s, tab, G, E, total,
                     offsets, meta, append);
  FEPLB_LAUNCH_CHECK("group_offsets_kernel");
  if (L.nchunks > 0) {
    const size_t lds = ((size_t)WAVES * E + E + 4 * (size_t)G) * sizeof(int);
    hipLaunchKernelGGL(assign_rows_kernel, dim3(cblocks), dim3(BLOCK), lds, s, topk_ids, A, E, G,
                       L.nchunks, L.chunk, hist, meta, R_cap, row_src, inv, append);
    FEPLB_LAUNCH_CHECK("assign_rows_kernel");
  }
  if (X && Xp && R_cap > 0 && d > 0) {
    hipLaunchKernelGGL((gather_rows_kernel<4>), dim3(R_cap), dim3(64), 0, s, (const u32x4*)X,
                       row_src, offsets, G, k, d / 8, R_cap, (u32x4*)Xp);
    FEPLB_LAUNCH_CHECK("gather_rows_kernel");
  }
  return FEPLB_OK;
}
}  // namespace

extern "C" int32_t feplb_permute(const int32_t* topk_ids, int32_t T, int32_t k, int32_t E,
                                 const feplb_group* groups, int32_t G, const void* X, int32_t d,
                                 void* Xp, int32_t R_cap, int32_t* offsets, int32_t* row_src,
                                 int32_t* inv, void* ws, size_t ws_bytes, void* stream) {
  return permute_impl(topk_ids, T, k, E, groups, G, X, d, Xp, R_cap, offsets, row_src, inv, ws,
                      ws_bytes, stream, 0);
}

extern "C" int32_t feplb_permute_append(const int32_t* topk_ids, int32_t T, int32_t k, int32_t E,
                                        const feplb_group* groups, int32_t G, const void* X,
                                        int32_t d, void* Xp, int32_t R_cap, int32_t* offsets,
                                        int32_t* row_src, int32_t* inv, void* ws, size_t ws_bytes,
                                        void* stream) {
  return permute_impl(topk_ids, T, k, E, groups, G, X, d, Xp, R_cap, offsets, row_src, inv, ws,
                      ws_bytes, stream, 1);
}

