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
// Pooled attention: rows of S_coarse = softmax_j(qc_i . kc_j / sqrt(D)).
// One workgroup computes ROWS rows; it writes the context columns of the source rows to pctx (for
// the column means of Eq. 1) and the sharpness of every row.
// ------------------------------------------------------------------------------------------
constexpr int CROWS = 8;

template <int D>
__global__ __launch_bounds__(256) void k_coarse(const float* __restrict__ qc, const float* __restrict__ kc,
                                                float* __restrict__ pctx, float* __restrict__ sharp,
                                                float* __restrict__ z_out, const float* __restrict__ vc,
                                                float* __restrict__ ocoarse, Counts cnt, int H, int Tsrc_max, int Tctx_max) {
  extern __shared__ float sm[];
  float* qs = sm;                       // [CROWS][D]
  float* zs = sm + CROWS * D;           // [CROWS][T_max]
  const int b = blockIdx.z, h = blockIdx.y, i0 = blockIdx.x * CROWS;
  const int T = cnt.b[b].T, T_src = cnt.b[b].T_src, T_max = cnt.T_max;
  if (i0 >= T) return;
  const long long bh = (long long)b * H + h;
  const float* qrow = qc + (bh * T_max + i0) * D;
  for (int x = threadIdx.x; x < CROWS * D; x += 256) qs[x] = (i0 + x / D < T) ? qrow[x] : 0.f;
  __syncthreads();
  const float scale = 1.0f / sqrtf((float)D);
  for (int j = threadIdx.x; j < T; j += 256) {
    const float4* kr = reinterpret_cast<const float4*>(kc + (bh * T_max + j) * D);
    float acc[CROWS];
#pragma unroll
    for (int r = 0; r < CROWS; ++r) acc[r] = 0.f;
#pragma unroll 4
    for (int d4 = 0; d4 < D / 4; ++d4) {
      const float4 kv = kr[d4];
#pragma unroll
      for (int r = 0; r < CROWS; ++r) {
        const float* qq = qs + r * D + d4 * 4;
        acc[r] = fmaf(qq[0], kv.x, acc[r]);
        acc[r] = fmaf(qq[1], kv.y, acc[r]);
        acc[r] = fmaf(qq[2], kv.z, acc[r]);
        acc[r] = fmaf(qq[3], kv.w, acc[r]);
      }
    }
#pragma unroll
    for (int r = 0; r < CROWS; ++r) zs[r * T_max + j] = acc[r] * scale;
  }
  __syncthreads();
  // softmax, context columns and sharpness of a row: one wave per row (waves take rows wave, wave + 4), a lane owns the
  // columns lane, lane + 64, ... from here on, so that nothing has to be synchronised between the passes over a row
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  for (int r = wave; r < CROWS; r += 4) {
    const int i = i0 + r;
    if (i >= T) break;                                  // uniform over the wave
    float* zr = zs + r * T_max;
    if (z_out)
      for (int j = lane; j < T; j += 64) z_out[(bh * T_max + i) * T_max + j] = zr[j];
    float m = -INFINITY;
    for (int j = lane; j < T; j += 64) m = fmaxf(m, zr[j]);
    m = wave_max(m);
    double l = 0.0;
    for (int j = lane; j < T; j += 64) {
      const float e = expf(zr[j] - m);
      zr[j] = e;
      l += (double)e;
    }
    l = wave_sum(l);
    const float inv = (float)(1.0 / l);
    double mu = 0.0;
    for (int j = lane; j < T; j += 64) {
      const float p = zr[j] * inv;
      zr[j] = p;
      if (j < T_src) mu += (double)p;
      else if (i < T_src) pctx[(bh * Tsrc_max + i) * Tctx_max + (j - T_src)] = p;
    }
    mu = wave_sum(mu) / (double)T_src;
    double var = 0.0;
    for (int j = lane; j < T_src; j += 64) {
      const double d = (double)zr[j] - mu;
      var += d * d;
    }
    var = wave_sum(var) / (double)T_src;
    if (lane == 0) sharp[bh * T_max + i] = (float)var;
  }
  // O_coarse = S_coarse V^c (Alg. 1 Stage 1), only when the caller wants the coarse residual: the rows of
  // S_coarse of this workgroup's query blocks are in LDS; one thread per (row, channel), channels fastest
  if (ocoarse) {
    __syncthreads();
    for (int x = threadIdx.x; x < CROWS * D; x += 256) {
      const int r = x / D, ch = x % D;
      if (i0 + r >= T) continue;
      const float* pr = zs + r * T_max;
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

hipError_t launch_coarse(const Problem& pr, const Workspace& ws, const float* qc, const float* kc, float* s_ctx,
                         float* sharp, float* z, const float* vc, float* ocoarse, hipStream_t st) {
  const int T_max = pr.cnt.T_max;
  const dim3 grid((T_max + CROWS - 1) / CROWS, pr.p.H, pr.p.B);
  const size_t lds = (size_t)CROWS * (pr.p.D + T_max) * sizeof(float);
  if (lds > 64 * 1024) {                                // beyond the default limit of dynamic LDS (about 1900 blocks): ask for it
    hipError_t ea = pr.p.D == 128
        ? hipFuncSetAttribute(reinterpret_cast<const void*>(&k_coarse<128>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)
        : hipFuncSetAttribute(reinterpret_cast<const void*>(&k_coarse<64>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (ea != hipSuccess) return ea;
  }
  if (pr.p.D == 128)
    hipLaunchKernelGGL((k_coarse<128>), grid, dim3(256), lds, st, qc, kc, ws.pctx, sharp, z, vc, ocoarse, pr.cnt, pr.p.H, pr.Tsrc_max,
                       pr.Tctx_max);
  else
    hipLaunchKernelGGL((k_coarse<64>), grid, dim3(256), lds, st, qc, kc, ws.pctx, sharp, z, vc, ocoarse, pr.cnt, pr.p.H, pr.Tsrc_max,
                       pr.Tctx_max);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(k_colmean, dim3((pr.Tctx_max + 63) / 64, pr.p.H, pr.p.B), dim3(256), 0, st, ws.pctx, s_ctx, pr.cnt,
                     pr.p.H, pr.Tsrc_max, pr.Tctx_max);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Selection.  One workgroup per (head, batch).  Rank of an entry = number of entries that beat it
// (larger score, or equal score and lower index); entries of rank < k are chosen.  Chosen and
// unchosen indices are compacted in ascending order with a block-wide scan.
// ------------------------------------------------------------------------------------------
__device__ inline bool beats(float sa, int ia, float sb, int ib) { return sa > sb || (sa == sb && ia < ib); }

// flags[0..n) -> ascending indices of flagged entries to out_yes (offset add), of the others to out_no.
__device__ void compact(const int* flags, int n, int add, int* out_yes, int* out_no, int* cnts /* [257] LDS */) {
  const int chunk = (n + 255) / 256;
  const int lo = min(n, (int)threadIdx.x * chunk), hi = min(n, lo + chunk);
  int c = 0;
  for (int x = lo; x < hi; ++x) c += flags[x];
  __syncthreads();
  cnts[threadIdx.x + 1] = c;
  __syncthreads();
  if (threadIdx.x == 0) {
    cnts[0] = 0;
    for (int t = 1; t <= 256; ++t) cnts[t] += cnts[t - 1];
  }
  __syncthreads();
  int yes = cnts[threadIdx.x], no = lo - yes;
  for (int x = lo; x < hi; ++x) {
    if (flags[x]) out_yes[yes++] = x + add;
    else if (out_no) out_no[no++] = x + add;
  }
  __syncthreads();
}

__global__ __launch_bounds__(256) void k_select(const float* __restrict__ s_ctx, const float* __restrict__ sharp,
                                                int* __restrict__ kv_list, int* __restrict__ full_list,
                                                int* __restrict__ flat_list, Counts cnt, int H) {
  extern __shared__ float sm[];
  float* sc = sm;                                   // [T_max]
  int* flags = reinterpret_cast<int*>(sm + cnt.T_max);   // [T_max]
  __shared__ int cnts[257];
  const int h = blockIdx.x, b = blockIdx.y;
  const BatchCounts c = cnt.b[b];
  const long long off = ((long long)b * H + h) * cnt.T_max;

  // context blocks by saliency
  for (int j = threadIdx.x; j < c.T_ctx; j += 256) sc[j] = s_ctx[off + j];
  __syncthreads();
  for (int j = threadIdx.x; j < c.T_ctx; j += 256) {
    const float s = sc[j];
    int rank = 0;
    for (int x = 0; x < c.T_ctx; ++x) rank += beats(sc[x], x, s, j) ? 1 : 0;
    flags[j] = rank < c.k_keep ? 1 : 0;
  }
  for (int j = threadIdx.x; j < cnt.T_max; j += 256) kv_list[off + j] = j < c.T_src ? j : -1;
  __syncthreads();
  compact(flags, c.T_ctx, c.T_src, kv_list + off + c.T_src, nullptr, cnts);

  // query blocks by sharpness
  for (int i = threadIdx.x; i < c.T; i += 256) sc[i] = sharp[off + i];
  for (int i = threadIdx.x; i < cnt.T_max; i += 256) {
    full_list[off + i] = -1;
    flat_list[off + i] = -1;
  }
  __syncthreads();
  for (int i = threadIdx.x; i < c.T; i += 256) {
    const float s = sc[i];
    int rank = 0;
    for (int x = 0; x < c.T; ++x) rank += beats(sc[x], x, s, i) ? 1 : 0;
    flags[i] = rank < c.n_full ? 1 : 0;
  }
  __syncthreads();
  compact(flags, c.T, 0, full_list + off, flat_list + off, cnts);
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
  hipLaunchKernelGGL(k_select, dim3(pr.p.H, pr.p.B), dim3(256), lds, st, s_ctx, sharp, kv_list, full_list, flat_list,
                     pr.cnt, pr.p.H);
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
