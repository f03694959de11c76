// Prologue of the operator: tile-order flattening (Sec. 2 "Block Sparse Attention": spatiotemporal tiles are formed
// first and flattened in tile order, then the sequence is cut into blocks) and the decoupled rotary embedding (Sec. 4:
// applied to the source and to every context reference independently, coordinates counted from zero in each), fused
// with the block means of Alg. 1 Stage 1 into one streaming pass over Q, K and V.
//
// Input tokens of a segment arrive row-major over its (t, h, w) grid, w fastest.  Output position p of a segment holds
// the p-th token in tile order: tiles row-major over tile coordinates, tokens row-major inside a tile, tiles clipped at
// the far edges of the grid.  Q and K are rotated on interleaved channel pairs (2i, 2i+1): the first rope_dims[0]
// channels by the frame coordinate, the next rope_dims[1] by the row, the next rope_dims[2] by the column; pair j of an
// axis with d channels turns by coordinate * theta^(-2j/d) radians.  V is only reordered.
//
// HBM-bound: one workgroup owns one output block (<= 128 tokens) of HPW heads, reads every token row once with 16-byte
// loads (a row is D contiguous elements wherever it comes from, so the gather costs nothing in coalescing), rotates in
// registers (the sines and cosines of a thread's pairs are computed once and reused for every head and for Q and K),
// writes the row once and keeps the running sums for the block means.
#include <math.h>
#include <string.h>

#include "isa_internal.h"

namespace isa {

constexpr int HPW = 4;        // heads per workgroup
constexpr int PBLOCK = 128;   // largest block

struct GridDesc {             // passed to kernels by value
  int grid[ISA_MAX_SEGMENTS][3];
  int tile[3];
  int rope_dims[3];
  double log2_theta;
};

struct BlockPos { int n, start, seg_start, p0, t, h, w; };

// Block j of batch item b: its real tokens n (0 if there is no such block), first token `start` inside the batch item,
// the first token of its segment, its offset p0 inside the segment and the segment's grid.  Static indices only.
__device__ inline BlockPos locate_block(const SegDesc& seg, const GridDesc& gd, int b, int j, int block) {
  int s0 = 0, s1 = 0;
#pragma unroll
  for (int i = 0; i < ISA_MAX_BATCH; ++i)
    if (i == b) { s0 = seg.seg_ptr[i]; s1 = seg.seg_ptr[i + 1]; }
  BlockPos r = {0, 0, 0, 0, 1, 1, 1};
  int blocks = 0, tok = 0;
  bool found = false;
#pragma unroll
  for (int s = 0; s < ISA_MAX_SEGMENTS; ++s) {
    if (s >= s0 && s < s1) {
      const int len = seg.seg_len[s];
      const int nb = (len + block - 1) / block;
      if (!found && j < blocks + nb) {
        found = true;
        r.p0 = (j - blocks) * block;
        r.n = min(block, len - r.p0);
        r.seg_start = tok;
        r.start = tok + r.p0;
        r.t = gd.grid[s][0]; r.h = gd.grid[s][1]; r.w = gd.grid[s][2];
      }
      blocks += nb;
      tok += len;
    }
  }
  return r;
}

// Coordinates of the token at position p of a segment's tile order.
__device__ inline void tile_coords(int p, int t, int h, int w, int tt, int th, int tw, int* ct, int* ch, int* cw) {
  tt = min(tt, t); th = min(th, h); tw = min(tw, w);
  const int a = p / (tt * h * w);                  // all tiles before tile plane a cover tt whole frames each
  p -= a * tt * h * w;
  const int st = min(tt, t - a * tt);
  const int bq = p / (st * th * w);                // inside the plane: tile rows cover th whole rows of st frames
  p -= bq * st * th * w;
  const int sh = min(th, h - bq * th);
  const int c = p / (st * sh * tw);
  p -= c * st * sh * tw;
  const int sw = min(tw, w - c * tw);
  const int lt = p / (sh * sw);
  p -= lt * sh * sw;
  const int lh = p / sw;
  *ct = a * tt + lt;
  *ch = bq * th + lh;
  *cw = c * tw + (p - lh * sw);
}

template <typename T> struct Row16;
template <> struct Row16<float> {
  static constexpr int N = 4;
  __device__ static void load(const float* p, float* o) {
    const float4 v = *reinterpret_cast<const float4*>(p);
    o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
  }
  __device__ static void store(float* p, float* o) {       // o is left holding the stored values
    *reinterpret_cast<float4*>(p) = make_float4(o[0], o[1], o[2], o[3]);
  }
};
template <> struct Row16<uint16_t> {   // bf16 storage
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
  __device__ static uint32_t round_bf16(float f) {         // round to nearest even, NaN kept quiet
    const uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
  }
  __device__ static void store(uint16_t* p, float* o) {    // o is left holding the rounded values
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t lo = round_bf16(o[2 * i]), hi = round_bf16(o[2 * i + 1]);
      w[i] = lo | (hi << 16);
      o[2 * i] = __uint_as_float(lo << 16);
      o[2 * i + 1] = __uint_as_float(hi << 16);
    }
    *reinterpret_cast<uint4*>(p) = make_uint4(w[0], w[1], w[2], w[3]);
  }
};

template <typename T, int D>
__global__ __launch_bounds__(256) void k_prologue(const T* __restrict__ q_in, const T* __restrict__ k_in,
                                                  const T* __restrict__ v_in, T* __restrict__ q_out,
                                                  T* __restrict__ k_out, T* __restrict__ v_out,
                                                  float* __restrict__ qc, float* __restrict__ kc,
                                                  float* __restrict__ vc, SegDesc seg, GridDesc gd, Geometry g) {
  constexpr int VEC = Row16<T>::N;
  constexpr int CH = D / VEC;            // 16-byte chunks per row
  constexpr int RP = 256 / CH;           // rows covered per pass
  constexpr int TPT = PBLOCK / RP;       // rows per thread
  constexpr int NP = VEC / 2;            // channel pairs per thread
  __shared__ int s_src[PBLOCK];
  __shared__ int s_pos[PBLOCK][3];
  __shared__ float red[RP][D];
  const int j = blockIdx.x, b = blockIdx.z, h0 = blockIdx.y * HPW;
  const BlockPos bp = locate_block(seg, gd, b, j, g.block);
  if (bp.n == 0) return;
  if (threadIdx.x < bp.n) {
    int ct, ch, cw;
    tile_coords(bp.p0 + threadIdx.x, bp.t, bp.h, bp.w, gd.tile[0], gd.tile[1], gd.tile[2], &ct, &ch, &cw);
    s_src[threadIdx.x] = bp.seg_start + (ct * bp.h + ch) * bp.w + cw;
    s_pos[threadIdx.x][0] = ct; s_pos[threadIdx.x][1] = ch; s_pos[threadIdx.x][2] = cw;
  }
  __syncthreads();

  const int c = threadIdx.x % CH, rg = threadIdx.x / CH;
  // the thread's channel pairs: which coordinate turns them, and how fast
  int axis[NP];
  double freq[NP];
#pragma unroll
  for (int i = 0; i < NP; ++i) {
    int pr = c * NP + i, d_a = 0;
    axis[i] = -1;
    if (pr < gd.rope_dims[0] / 2) { axis[i] = 0; d_a = gd.rope_dims[0]; }
    else if ((pr -= gd.rope_dims[0] / 2) < gd.rope_dims[1] / 2) { axis[i] = 1; d_a = gd.rope_dims[1]; }
    else if ((pr -= gd.rope_dims[1] / 2) < gd.rope_dims[2] / 2) { axis[i] = 2; d_a = gd.rope_dims[2]; }
    freq[i] = axis[i] < 0 ? 0.0 : exp2(-2.0 * (double)pr / (double)d_a * gd.log2_theta);
  }
  int src[TPT];
  float cs[TPT][NP], sn[TPT][NP];
#pragma unroll
  for (int tk = 0; tk < TPT; ++tk) {
    const int r = rg + tk * RP;
    src[tk] = r < bp.n ? s_src[r] : -1;
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      cs[tk][i] = 1.f; sn[tk][i] = 0.f;
      if (r < bp.n && axis[i] >= 0) {
        const int pos = axis[i] == 0 ? s_pos[r][0] : axis[i] == 1 ? s_pos[r][1] : s_pos[r][2];
        double ang = (double)pos * freq[i];
        ang -= 6.283185307179586476925 * rint(ang * 0.1591549430918953357689);     // into [-pi, pi]
        sincosf((float)ang, &sn[tk][i], &cs[tk][i]);
      }
    }
  }

  const T* in[3] = {q_in, k_in, v_in};
  T* out[3] = {q_out, k_out, v_out};
  float* mean[3] = {qc, kc, vc};
  const float inv_n = 1.0f / (float)bp.n;
  for (int hh = 0; hh < HPW; ++hh) {
    const int h = h0 + hh;
    if (h >= g.H) break;
    const long long base = (long long)b * g.stride_b + (long long)h * g.stride_h + c * VEC;
    const long long mbase = (((long long)b * g.H + h) * g.T_max + j) * D;
#pragma unroll
    for (int t = 0; t < 3; ++t) {
      float x[TPT][VEC];
#pragma unroll
      for (int tk = 0; tk < TPT; ++tk)
        if (src[tk] >= 0) Row16<T>::load(in[t] + base + (long long)src[tk] * g.stride_t, x[tk]);
      float acc[VEC];
#pragma unroll
      for (int i = 0; i < VEC; ++i) acc[i] = 0.f;
#pragma unroll
      for (int tk = 0; tk < TPT; ++tk) {
        if (src[tk] < 0) continue;
        if (t < 2) {
#pragma unroll
          for (int i = 0; i < NP; ++i) {
            const float a0 = x[tk][2 * i], a1 = x[tk][2 * i + 1];
            x[tk][2 * i] = a0 * cs[tk][i] - a1 * sn[tk][i];
            x[tk][2 * i + 1] = a0 * sn[tk][i] + a1 * cs[tk][i];
          }
        }
        Row16<T>::store(out[t] + base + (long long)(bp.start + rg + tk * RP) * g.stride_t, x[tk]);
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[i] += x[tk][i];
      }
      if (mean[t]) {        // uniform
        __syncthreads();
#pragma unroll
        for (int i = 0; i < VEC; ++i) red[rg][c * VEC + i] = acc[i];
        __syncthreads();
        if (threadIdx.x < D) {
          float s = 0.f;
#pragma unroll
          for (int r = 0; r < RP; ++r) s += red[r][threadIdx.x];
          mean[t][mbase + threadIdx.x] = s * inv_n;
        }
      }
    }
  }
}

// Inverse reordering of one tensor: token p of the tile order goes back to its row-major place.
template <typename T, int D>
__global__ __launch_bounds__(256) void k_untile(const T* __restrict__ x_tiled, T* __restrict__ x_raster, SegDesc seg,
                                                GridDesc gd, Geometry g) {
  constexpr int VEC = Row16<T>::N;
  constexpr int CH = D / VEC;
  constexpr int RP = 256 / CH;
  constexpr int TPT = PBLOCK / RP;
  __shared__ int s_src[PBLOCK];
  const int j = blockIdx.x, b = blockIdx.z, h0 = blockIdx.y * HPW;
  const BlockPos bp = locate_block(seg, gd, b, j, g.block);
  if (bp.n == 0) return;
  if (threadIdx.x < bp.n) {
    int ct, ch, cw;
    tile_coords(bp.p0 + threadIdx.x, bp.t, bp.h, bp.w, gd.tile[0], gd.tile[1], gd.tile[2], &ct, &ch, &cw);
    s_src[threadIdx.x] = bp.seg_start + (ct * bp.h + ch) * bp.w + cw;
  }
  __syncthreads();
  const int c = threadIdx.x % CH, rg = threadIdx.x / CH;
  int src[TPT];
#pragma unroll
  for (int tk = 0; tk < TPT; ++tk) src[tk] = rg + tk * RP < bp.n ? s_src[rg + tk * RP] : -1;
  for (int hh = 0; hh < HPW; ++hh) {
    const int h = h0 + hh;
    if (h >= g.H) break;
    const long long base = (long long)b * g.stride_b + (long long)h * g.stride_h + c * VEC;
    uint4 x[TPT];
#pragma unroll
    for (int tk = 0; tk < TPT; ++tk) {      // rows past the block's end re-read its first row and are not stored
      const int row = src[tk] >= 0 ? bp.start + rg + tk * RP : bp.start;
      x[tk] = *reinterpret_cast<const uint4*>(x_tiled + base + (long long)row * g.stride_t);
    }
#pragma unroll
    for (int tk = 0; tk < TPT; ++tk)
      if (src[tk] >= 0) *reinterpret_cast<uint4*>(x_raster + base + (long long)src[tk] * g.stride_t) = x[tk];
  }
}

static GridDesc make_desc(const Problem& pr, const isa_grid* gr) {
  GridDesc gd;
  memset(&gd, 0, sizeof(gd));
  const int n_seg = pr.seg.seg_ptr[pr.p.B];
  for (int s = 0; s < n_seg; ++s)
    for (int a = 0; a < 3; ++a) gd.grid[s][a] = gr->seg_grid[3 * s + a];
  for (int a = 0; a < 3; ++a) { gd.tile[a] = gr->tile[a]; gd.rope_dims[a] = gr->rope_dims[a]; }
  gd.log2_theta = log2(gr->rope_theta);
  return gd;
}

hipError_t launch_prologue(const Problem& pr, const isa_grid* gr, const void* q_in, const void* k_in, const void* v_in,
                           void* q_out, void* k_out, void* v_out, float* qc, float* kc, float* vc, hipStream_t st) {
  const GridDesc gd = make_desc(pr, gr);
  const dim3 grid(pr.cnt.T_max, (pr.p.H + HPW - 1) / HPW, pr.p.B), blk(256);
#define ISA_PRO(T, D)                                                                                                \
  hipLaunchKernelGGL((k_prologue<T, D>), grid, blk, 0, st, (const T*)q_in, (const T*)k_in, (const T*)v_in, (T*)q_out, \
                     (T*)k_out, (T*)v_out, qc, kc, vc, pr.seg, gd, pr.geo)
  if (pr.p.dtype == ISA_BF16) {
    if (pr.p.D == 128) ISA_PRO(uint16_t, 128); else ISA_PRO(uint16_t, 64);
  } else {
    if (pr.p.D == 128) ISA_PRO(float, 128); else ISA_PRO(float, 64);
  }
#undef ISA_PRO
  return hipGetLastError();
}

hipError_t launch_untile(const Problem& pr, const isa_grid* gr, const void* x_tiled, void* x_raster, hipStream_t st) {
  const GridDesc gd = make_desc(pr, gr);
  const dim3 grid(pr.cnt.T_max, (pr.p.H + HPW - 1) / HPW, pr.p.B), blk(256);
#define ISA_UNT(T, D) \
  hipLaunchKernelGGL((k_untile<T, D>), grid, blk, 0, st, (const T*)x_tiled, (T*)x_raster, pr.seg, gd, pr.geo)
  if (pr.p.dtype == ISA_BF16) {
    if (pr.p.D == 128) ISA_UNT(uint16_t, 128); else ISA_UNT(uint16_t, 64);
  } else {
    if (pr.p.D == 128) ISA_UNT(float, 128); else ISA_UNT(float, 64);
  }
#undef ISA_UNT
  return hipGetLastError();
}

}  // namespace isa
