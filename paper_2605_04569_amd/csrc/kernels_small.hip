// The small stages of ISA: block table, block means (Alg. 1 Stage 1), pooled attention scores with
// context saliency (Sec. 3, Eq. 1) and sharpness (Alg. 1 Stage 3), and the integer selection work
// (Eq. 2, Alg. 1 Stage 3 split, Alg. 2 Stage 2).  All reductions run in a fixed order, so results
// are reproducible from run to run.
#include <hip/hip_bf16.h>

#include "isa_internal.h"

namespace isa {

// ------------------------------------------------------------------------------------------
// helpers
// ------------------------------------------------------------------------------------------
__device__ inline float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
  return x;
}
__device__ inline double wave_sum(double x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
  return x;
}
__device__ inline float wave_max(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
  return x;
}

// Block-wide reductions for 256 threads (4 waves); every thread gets the result.
template <typename T>
__device__ inline T block_sum(T x, T* red /* >= 4 elements of LDS */) {
  x = wave_sum(x);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = x;
  __syncthreads();
  return ((red[0] + red[1]) + red[2]) + red[3];
}
__device__ inline float block_max(float x, float* red) {
  x = wave_max(x);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = x;
  __syncthreads();
  return fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}

__device__ inline float bf16_bits_to_float(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// ------------------------------------------------------------------------------------------
// Block table: token offset and real token count of every block of every batch item.
// ------------------------------------------------------------------------------------------
__global__ void k_layout(SegDesc seg, int block, int T_max, int* blk_start, int* blk_n, int4* btab) {
  const int b = blockIdx.x;
  for (int j = threadIdx.x; j < T_max; j += blockDim.x) {
    int start = 0, n = 0, first = 0, off = 0;
    for (int s = seg.seg_ptr[b]; s < seg.seg_ptr[b + 1]; ++s) {
      const int len = seg.seg_len[s];
      const int nb = (len + block - 1) / block;
      if (j >= first && j < first + nb) {
        const int local = j - first;
        start = off + local * block;
        n = min(block, len - local * block);
      }
      first += nb;
      off += len;
    }
    blk_start[b * T_max + j] = start;   // blocks past the batch item's T get n = 0
    blk_n[b * T_max + j] = n;
    btab[b * T_max + j] = make_int4(start, n, j, 0);
  }
}

hipError_t launch_layout(const Problem& pr, const Workspace& ws, hipStream_t st) {
  hipLaunchKernelGGL(k_layout, dim3(pr.p.B), dim3(256), 0, st, pr.seg, pr.p.block, pr.cnt.T_max, ws.blk_start, ws.blk_n, ws.btab);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Block means.  One workgroup per (block, head, batch); q, k and v in turn.
// A thread owns VEC consecutive channels (one 16-byte load) of every RP-th row.
// ------------------------------------------------------------------------------------------
template <typename T> struct Vec16;
template <> struct Vec16<float> {
  static constexpr int N = 4;
  __device__ static void load(const float* p, float* o) {
    const float4 v = *reinterpret_cast<const float4*>(p);
    o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
  }
};
template <> struct Vec16<uint16_t> {   // bf16 storage
  static constexpr int N = 8;
  __device__ static void load(const uint16_t* p, float* o) {
    const uint4 v = *reinterpret_cast<const uint4*>(p);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      o[2 * i] = __uint_as_float(w[i] << 16);
      o[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
};

template <typename T, int D>
__global__ __launch_bounds__(256) void k_block_means(const T* __restrict__ q, const T* __restrict__ k,
                                                     const T* __restrict__ v, float* __restrict__ qc,
                                                     float* __restrict__ kc, float* __restrict__ vc,
                                                     const int* __restrict__ blk_start, const int* __restrict__ blk_n,
                                                     Geometry g) {
  constexpr int VEC = Vec16<T>::N;
  constexpr int CH = D / VEC;          // 16-byte chunks per row
  constexpr int RP = 256 / CH;         // rows covered per pass
  __shared__ float red[RP][D];
  const int j = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int n = blk_n[b * g.T_max + j];
  if (n == 0) return;
  const int start = blk_start[b * g.T_max + j];
  const int c = threadIdx.x % CH, rg = threadIdx.x / CH;
  const long long base = (long long)b * g.stride_b + (long long)h * g.stride_h + (long long)start * g.stride_t + c * VEC;
  const long long obase = (((long long)b * g.H + h) * g.T_max + j) * D;
  const T* src[3] = {q, k, v};
  float* dst[3] = {qc, kc, vc};
  const int n_tensors = v ? 3 : 2;        // without v: its means come from the kernel that packs V^T
  for (int t = 0; t < n_tensors; ++t) {
    float acc[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] = 0.f;
    for (int r = rg; r < n; r += RP) {
      float x[VEC];
      Vec16<T>::load(src[t] + base + (long long)r * g.stride_t, x);
#pragma unroll
      for (int i = 0; i < VEC; ++i) acc[i] += x[i];
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < VEC; ++i) red[rg][c * VEC + i] = acc[i];
    __syncthreads();
    if (threadIdx.x < D) {
      float s = 0.f;
#pragma unroll
      for (int r = 0; r < RP; ++r) s += red[r][threadIdx.x];
      dst[t][obase + threadIdx.x] = s / (float)n;
    }
  }
}

hipError_t launch_block_means(const Problem& pr, const Workspace& ws, const void* q, const void* k, const void* v,
                              float* qc, float* kc, float* vc, hipStream_t st) {
  const dim3 grid(pr.cnt.T_max, pr.p.H, pr.p.B), blk(256);
#define ISA_MEANS(T, D)                                                                                        \
  hipLaunchKernelGGL((k_block_means<T, D>), grid, blk, 0, st, (const T*)q, (const T*)k, (const T*)v, qc, kc, vc, \
                     ws.blk_start, ws.blk_n, pr.geo)
  if (pr.p.dtype == ISA_BF16) {
    if (pr.p.D == 128) ISA_MEANS(uint16_t, 128); else ISA_MEANS(uint16_t, 64);
  } else {
    if (pr.p.D == 128) ISA_MEANS(float, 128); else ISA_MEANS(float, 64);
  }
#undef ISA_MEANS
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Pooled attention: rows of S_coarse = softmax_j(qc_i . kc_j / sqrt(D)) (Alg. 1 Stage 1).
// One workgroup computes ROWS rows; it writes the context columns of the source rows to pctx (for
// the column means of Eq. 1) and the sharpness of every row (Alg. 1 Stage 3).
//
// Logits: fp32 matrix instructions (v_mfma_f32_16x16x4_f32), transposed: the 16 rows of the A operand are 16 mean
// keys, the 16 columns of the B operand the workgroup's mean queries, so that a lane ends up with four consecutive
// columns of one row of S_coarse (one 16-byte LDS store).  With l = lane % 16 and g = lane / 16, lane (l, g) feeds
// channel 16 t + 4 g + i of key / query l into step (t, i): one 16-byte load per lane covers four steps.  The mean
// queries stay in registers for the whole workgroup; the four waves take pairs of 16-column tiles in turn.
// Workgroup ids go round-robin over the XCDs, so XCD x sees ids x, x + 8, ...; each XCD owns every 8th
// (batch, head) and works through its heads one after the other: the workgroups that run together read the same
// head's mean keys out of that XCD's L2.
// ------------------------------------------------------------------------------------------
typedef float f32x4_t __attribute__((ext_vector_type(4)));

template <int D, int ROWS>
__global__ __launch_bounds__(256) void k_coarse(const float* __restrict__ qc, const float* __restrict__ kc,
                                                float* __restrict__ pctx, float* __restrict__ sharp,
                                                float* __restrict__ z_out, const float* __restrict__ vc,
                                                float* __restrict__ ocoarse, Counts cnt, int B, int H, int Tsrc_max,
                                                int Tctx_max, int zs_stride, int row_tiles) {
  static_assert(ROWS == 8 || ROWS == 16, "a row tile is half or all of the matrix instruction's 16 columns");
  extern __shared__ __attribute__((aligned(16))) float zs[];      // [ROWS][zs_stride]
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int bhid = (slot / row_tiles) * 8 + xcd;
  if (bhid >= B * H) return;
  const int b = bhid / H, i0 = (slot % row_tiles) * ROWS;
  const int T = cnt.b[b].T, T_src = cnt.b[b].T_src, T_max = cnt.T_max;
  if (i0 >= T) return;
  const long long bh = bhid;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int l16 = lane & 15, g = lane >> 4;
  const float scale = 1.0f / sqrtf((float)D);
  constexpr int NT = D / 16;                                       // 16-byte loads per lane and row
  __shared__ float rowmax[4][16];
  {
    // mean queries: rows past the batch item's last block repeat it (their logits are never read)
    float4 bq[NT];
    const float* qrow = qc + (bh * T_max + min(i0 + l16, T - 1)) * D + 4 * g;
#pragma unroll
    for (int t = 0; t < NT; ++t)
      bq[t] = (ROWS == 16 || l16 < ROWS) ? *reinterpret_cast<const float4*>(qrow + 16 * t) : make_float4(0.f, 0.f, 0.f, 0.f);
    const int n_ct = (T + 15) / 16;
    // mean keys of the column tiles jt, jt + 1; columns past the last block repeat it, so they change no maximum
    auto load_pair = [&](int jt, float4 (&ak)[2][NT]) {
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const float* krow = kc + (bh * T_max + min((jt + u) * 16 + l16, T - 1)) * D + 4 * g;
#pragma unroll
        for (int t = 0; t < NT; ++t) ak[u][t] = *reinterpret_cast<const float4*>(krow + 16 * t);
      }
    };
    float rmax = -INFINITY;                                         // over this lane's columns of row l16
    float4 ak[2][NT], ak_next[2][NT];
    load_pair(2 * wave, ak);
    for (int jt = 2 * wave; jt < n_ct; jt += 8) {
      load_pair(jt + 8, ak_next);                                   // the next pair's loads fly under this pair's products
      f32x4_t acc[2] = {f32x4_t{0.f, 0.f, 0.f, 0.f}, f32x4_t{0.f, 0.f, 0.f, 0.f}};
#pragma unroll
      for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          acc[u] = __builtin_amdgcn_mfma_f32_16x16x4f32(ak[u][t].x, bq[t].x, acc[u], 0, 0, 0);
          acc[u] = __builtin_amdgcn_mfma_f32_16x16x4f32(ak[u][t].y, bq[t].y, acc[u], 0, 0, 0);
          acc[u] = __builtin_amdgcn_mfma_f32_16x16x4f32(ak[u][t].z, bq[t].z, acc[u], 0, 0, 0);
          acc[u] = __builtin_amdgcn_mfma_f32_16x16x4f32(ak[u][t].w, bq[t].w, acc[u], 0, 0, 0);
        }
      // lane (l16, g) holds columns 16 jt + 4 g .. + 3 of row l16; zs_stride covers whole column tiles
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const float4 zv = make_float4(acc[u][0] * scale, acc[u][1] * scale, acc[u][2] * scale, acc[u][3] * scale);
        rmax = fmaxf(fmaxf(rmax, fmaxf(zv.x, zv.y)), fmaxf(zv.z, zv.w));
        if ((ROWS == 16 || l16 < ROWS) && jt + u < n_ct) *reinterpret_cast<float4*>(zs + l16 * zs_stride + (jt + u) * 16 + 4 * g) = zv;
      }
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int t = 0; t < NT; ++t) ak[u][t] = ak_next[u][t];
    }
    rmax = fmaxf(rmax, __shfl_xor(rmax, 16, 64));
    rmax = fmaxf(rmax, __shfl_xor(rmax, 32, 64));
    if (g == 0) rowmax[wave][l16] = rmax;
  }
  __syncthreads();
  // softmax, context columns and sharpness of a row: one wave per row (waves take rows wave, wave + 4, ...), a lane
  // owns the columns lane, lane + 64, ... from here on, so that nothing has to be synchronised between the passes
  // over a row.  Sums in double precision: the variance of a softmax row over hundreds of columns cancels badly in
  // single precision.
  for (int r = wave; r < ROWS; r += 4) {
    const int i = i0 + r;
    if (i >= T) break;                                  // uniform over the wave
    float* zr = zs + r * zs_stride;
    if (z_out)
      for (int j = lane; j < T; j += 64) z_out[(bh * T_max + i) * T_max + j] = zr[j];
    const float m = fmaxf(fmaxf(rowmax[0][r], rowmax[1][r]), fmaxf(rowmax[2][r], rowmax[3][r]));
    // one pass: e = exp(z - m) with the sums of e over all columns, and of e and e^2 over the source columns
    double l = 0.0, l_src = 0.0, q_src = 0.0;
#pragma unroll 4
    for (int j = lane; j < T; j += 64) {
      const float e = expf(zr[j] - m);
      zr[j] = e;
      const double ed = (double)e;
      l += ed;
      if (j < T_src) {
        l_src += ed;
        q_src = fma(ed, ed, q_src);
      }
    }
    l = wave_sum(l);
    l_src = wave_sum(l_src);
    q_src = wave_sum(q_src);
    // sharpness: variance of the row's softmax weights p = e / l over the source columns, E[p^2] - E[p]^2
    const double mu = l_src / l / (double)T_src;
    const double var = q_src / (l * l) / (double)T_src - mu * mu;
    if (lane == 0) sharp[bh * T_max + i] = (float)fmax(var, 0.0);
    const float inv = (float)(1.0 / l);
    // the weights themselves: the context columns of a source row go to pctx (Eq. 1); all of them stay in LDS for
    // the coarse output
    const int j_lo = ocoarse ? 0 : T_src;
    if (ocoarse || i < T_src) {
#pragma unroll 4
      for (int j = j_lo + lane; j < T; j += 64) {
        const float pw = zr[j] * inv;
        zr[j] = pw;
        if (j >= T_src && i < T_src) pctx[(bh * Tsrc_max + i) * Tctx_max + (j - T_src)] = pw;
      }
    }
  }
  // O_coarse = S_coarse V^c (Alg. 1 Stage 1), only when the caller wants the coarse residual: the rows of
  // S_coarse of this workgroup's query blocks are in LDS; one thread per (row, channel), channels fastest
  if (ocoarse) {
    __syncthreads();
    for (int x = threadIdx.x; x < ROWS * D; x += 256) {
      const int r = x / D, ch = x % D;
      if (i0 + r >= T) continue;
      const float* pr = zs + r * zs_stride;
      const float* vcol = vc + bh * T_max * D + ch;
      double acc = 0.0;
      for (int j = 0; j < T; ++j) acc += (double)pr[j] * (double)vcol[(long long)j * D];
      ocoarse[(bh * T_max + i0 + r) * D + ch] = (float)acc;
    }
  }
}

// Eq. 1: mean over the source query blocks of each context column.  64 columns per workgroup; the four waves each add a
// quarter of the rows, and the quarters are added in a fixed order.
__global__ __launch_bounds__(256) void k_colmean(const float* __restrict__ pctx, float* __restrict__ s_ctx, Counts cnt,
                                                 int H, int Tsrc_max, int Tctx_max) {
  __shared__ double part[4][64];
  const int b = blockIdx.z, h = blockIdx.y, lane = threadIdx.x & 63, quarter = threadIdx.x >> 6;
  const int j = blockIdx.x * 64 + lane;
  const int T_src = cnt.b[b].T_src, T_ctx = cnt.b[b].T_ctx;
  const long long bh = (long long)b * H + h;
  const int per = (T_src + 3) / 4, i_lo = quarter * per, i_hi = min(T_src, i_lo + per);
  double acc = 0.0;
  if (j < T_ctx)
    for (int i = i_lo; i < i_hi; ++i) acc += (double)pctx[(bh * Tsrc_max + i) * Tctx_max + j];
  part[quarter][lane] = acc;
  __syncthreads();
  if (quarter == 0 && j < T_ctx)
    s_ctx[bh * cnt.T_max + j] = (float)((((part[0][lane] + part[1][lane]) + part[2][lane]) + part[3][lane]) / (double)T_src);
}

template <int D, int ROWS>
static hipError_t launch_coarse_rows(const Problem& pr, const Workspace& ws, const float* qc, const float* kc, float* sharp,
                                     float* z, const float* vc, float* ocoarse, hipStream_t st) {
  const int T_max = pr.cnt.T_max;
  const int zs_stride = ((T_max + 15) / 16) * 16 + 4;          // whole column tiles; + 4 spreads the rows over the banks
  const int row_tiles = (T_max + ROWS - 1) / ROWS;
  const size_t lds = (size_t)ROWS * zs_stride * sizeof(float);
  if (lds > 64 * 1024) {                                        // beyond the default limit of dynamic LDS: ask for it
    hipError_t ea = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_coarse<D, ROWS>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (ea != hipSuccess) return ea;
  }
  const int bh = pr.p.B * pr.p.H;
  const unsigned grid = (unsigned)(N_XCD * ((bh + N_XCD - 1) / N_XCD) * row_tiles);
  hipLaunchKernelGGL((k_coarse<D, ROWS>), dim3(grid), dim3(256), lds, st, qc, kc, ws.pctx, sharp, z, vc, ocoarse, pr.cnt,
                     pr.p.B, pr.p.H, pr.Tsrc_max, pr.Tctx_max, zs_stride, row_tiles);
  return hipGetLastError();
}

hipError_t launch_coarse(const Problem& pr, const Workspace& ws, const float* qc, const float* kc, float* s_ctx,
                         float* sharp, float* z, const float* vc, float* ocoarse, hipStream_t st) {
  // 16 rows per workgroup (every column of the matrix instruction's B operand in use) while two such workgroups fit
  // a compute unit's LDS; 8 rows for longer rows (up to ISA_MAX_BLOCKS columns: 131 KB)
  const bool wide = (size_t)16 * (((pr.cnt.T_max + 15) / 16) * 16 + 4) * sizeof(float) <= 80 * 1024;
  hipError_t e;
  if (pr.p.D == 128) e = wide ? launch_coarse_rows<128, 16>(pr, ws, qc, kc, sharp, z, vc, ocoarse, st)
                              : launch_coarse_rows<128, 8>(pr, ws, qc, kc, sharp, z, vc, ocoarse, st);
  else e = wide ? launch_coarse_rows<64, 16>(pr, ws, qc, kc, sharp, z, vc, ocoarse, st)
                : launch_coarse_rows<64, 8>(pr, ws, qc, kc, sharp, z, vc, ocoarse, st);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(k_colmean, dim3((pr.Tctx_max + 63) / 64, pr.p.H, pr.p.B), dim3(256), 0, st, ws.pctx, s_ctx, pr.cnt,
                     pr.p.H, pr.Tsrc_max, pr.Tctx_max);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Selection.  One workgroup of 1024 threads per (head, batch, list kind): the kept context blocks (Eq. 2), or the
// split of the query blocks by sharpness (Alg. 1 Stage 3).  Rank of an entry = number of entries that beat it
// (larger score, or equal score and lower index); entries of rank < k are chosen.  Chosen and unchosen indices are
// compacted in ascending order with a block-wide scan.
// ------------------------------------------------------------------------------------------
__device__ inline bool beats(float sa, int ia, float sb, int ib) { return sa > sb || (sa == sb && ia < ib); }

constexpr int SEL_THREADS = 1024;
constexpr int SEL_PARTS = 16;        // lanes that share the count of one entry's rank (each counts 1/16 of the peers)

// flags[j] = 1 for the entries of sc[0..n) that fewer than k others beat.  Integer counts: the result does not depend
// on how the peers are divided among the lanes.
__device__ void rank_flags(const float* sc, int n, int k, int* flags) {
  const int part = threadIdx.x % SEL_PARTS;
  const int per = (n + SEL_PARTS - 1) / SEL_PARTS, lo = min(n, part * per), hi = min(n, lo + per);
  for (int j0 = 0; j0 < n; j0 += SEL_THREADS / SEL_PARTS) {          // the same trip count for every thread
    const int j = j0 + threadIdx.x / SEL_PARTS;
    int rank = 0;
    if (j < n) {
      const float s = sc[j];
      for (int x = lo; x < hi; ++x) rank += beats(sc[x], x, s, j) ? 1 : 0;
    }
#pragma unroll
    for (int o = SEL_PARTS / 2; o > 0; o >>= 1) rank += __shfl_xor(rank, o, 64);
    if (j < n && part == 0) flags[j] = rank < k ? 1 : 0;
  }
}

// flags[0..n) -> ascending indices of flagged entries to out_yes (offset add), of the others to out_no.
__device__ void compact(const int* flags, int n, int add, int* out_yes, int* out_no, int* wsum /* [SEL_THREADS / 64] LDS */) {
  const int chunk = (n + SEL_THREADS - 1) / SEL_THREADS;
  const int lo = min(n, (int)threadIdx.x * chunk), hi = min(n, lo + chunk);
  int c = 0;
  for (int x = lo; x < hi; ++x) c += flags[x];
  // exclusive scan of c over the workgroup: inside a wave with shuffles, then the sums of the waves before this one
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int inc = c;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int t = __shfl_up(inc, o, 64);
    if (lane >= o) inc += t;
  }
  __syncthreads();
  if (lane == 63) wsum[wave] = inc;
  __syncthreads();
  int yes = inc - c;
  for (int w = 0; w < wave; ++w) yes += wsum[w];
  int no = lo - yes;
  for (int x = lo; x < hi; ++x) {
    if (flags[x]) out_yes[yes++] = x + add;
    else if (out_no) out_no[no++] = x + add;
  }
  __syncthreads();
}

__global__ __launch_bounds__(SEL_THREADS) void k_select(const float* __restrict__ s_ctx, const float* __restrict__ sharp,
                                                        int* __restrict__ kv_list, int* __restrict__ full_list,
                                                        int* __restrict__ flat_list, Counts cnt, int H) {
  extern __shared__ float sm[];
  float* sc = sm;                                   // [T_max]
  int* flags = reinterpret_cast<int*>(sm + cnt.T_max);   // [T_max]
  __shared__ int wsum[SEL_THREADS / 64];
  const int h = blockIdx.x, b = blockIdx.y;
  const BatchCounts c = cnt.b[b];
  const long long off = ((long long)b * H + h) * cnt.T_max;

  if (blockIdx.z == 0) {       // context blocks by saliency: kv_list = all source blocks, then the kept context blocks
    for (int j = threadIdx.x; j < c.T_ctx; j += SEL_THREADS) sc[j] = s_ctx[off + j];
    for (int j = threadIdx.x; j < cnt.T_max; j += SEL_THREADS) kv_list[off + j] = j < c.T_src ? j : -1;
    __syncthreads();
    rank_flags(sc, c.T_ctx, c.k_keep, flags);
    __syncthreads();
    compact(flags, c.T_ctx, c.T_src, kv_list + off + c.T_src, nullptr, wsum);
  } else {                     // query blocks by sharpness
    for (int i = threadIdx.x; i < c.T; i += SEL_THREADS) sc[i] = sharp[off + i];
    for (int i = threadIdx.x; i < cnt.T_max; i += SEL_THREADS) {
      full_list[off + i] = -1;
      flat_list[off + i] = -1;
    }
    __syncthreads();
    rank_flags(sc, c.T, c.n_full, flags);
    __syncthreads();
    compact(flags, c.T, 0, full_list + off, flat_list + off, wsum);
  }
}

// Alg. 2 Stage 2: for the Taylor query block at position r of flat_list, mark the k_exact positions of
// kv_list with the largest coarse logit.
__global__ __launch_bounds__(256) void k_exact_sets(const float* __restrict__ z, const int* __restrict__ kv_list,
                                                    const int* __restrict__ flat_list, uint32_t* __restrict__ mask,
                                                    Counts cnt, int H) {
  extern __shared__ float sm[];                      // [T_max]
  const int r = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const BatchCounts c = cnt.b[b];
  if (r >= c.n_flat) return;
  const long long bh = (long long)b * H + h;
  const int i = block_in_range(flat_list[bh * cnt.T_max + r], c.T);
  const float* zr = z + (bh * cnt.T_max + i) * cnt.T_max;
  for (int t = threadIdx.x; t < c.T_new; t += 256) sm[t] = zr[block_in_range(kv_list[bh * cnt.T_max + t], c.T)];
  __syncthreads();
  uint32_t* mrow = mask + (bh * cnt.T_max + r) * cnt.mask_words;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int base = wave * 64; base < cnt.mask_words * 32; base += 256) {
    const int t = base + lane;
    bool bit = false;
    if (t < c.T_new) {
      const float s = sm[t];
      int rank = 0;
      for (int x = 0; x < c.T_new; ++x) rank += beats(sm[x], x, s, t) ? 1 : 0;
      bit = rank < c.k_exact;
    }
    const unsigned long long bal = __ballot(bit);
    if (lane == 0) {
      mrow[base / 32] = (uint32_t)bal;
      if (base / 32 + 1 < cnt.mask_words) mrow[base / 32 + 1] = (uint32_t)(bal >> 32);
    }
  }
}

hipError_t launch_select(const Problem& pr, const Workspace& ws, const float* s_ctx, const float* sharp, const float* z,
                         int* kv_list, int* full_list, int* flat_list, uint32_t* exact_mask, hipStream_t st) {
  const size_t lds = (size_t)pr.cnt.T_max * 8;
  hipLaunchKernelGGL(k_select, dim3(pr.p.H, pr.p.B, 2), dim3(SEL_THREADS), lds, st, s_ctx, sharp, kv_list, full_list,
                     flat_list, pr.cnt, pr.p.H);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || !(pr.p.exact_frac > 0.0)) return e;
  int nflat_max = 0;
  for (int b = 0; b < pr.p.B; ++b) nflat_max = pr.cnt.b[b].n_flat > nflat_max ? pr.cnt.b[b].n_flat : nflat_max;
  if (nflat_max == 0) return hipSuccess;
  hipLaunchKernelGGL(k_exact_sets, dim3(nflat_max, pr.p.H, pr.p.B), dim3(256), (size_t)pr.cnt.T_max * 4, st, z, kv_list,
                     flat_list, exact_mask, pr.cnt, pr.p.H);
  return hipGetLastError();
}

}  // namespace isa
