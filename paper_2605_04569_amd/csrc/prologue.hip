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
// HBM-bound: one workgroup owns one output block (<= 128 tokens) of a few heads, reads every token row once with 16-byte
// loads (a row is D contiguous elements wherever it comes from, so the gather costs nothing in coalescing), rotates in
// registers (the sines and cosines of a thread's pairs are computed once and reused for every head and for Q and K),
// writes the row once and keeps the running sums for the block means.  The rows of the next (head, tensor) pass are
// loaded into a second set of registers while the current pass is rotated and stored.
#include <math.h>
#include <string.h>

#include "isa_internal.h"

namespace isa {

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

template <typename T> struct Row16;      // 16 bytes of a token row
template <> struct Row16<float> {
  static constexpr int N = 4;
  __device__ static void unpack(const uint4& v, float* o) {
    o[0] = __uint_as_float(v.x); o[1] = __uint_as_float(v.y); o[2] = __uint_as_float(v.z); o[3] = __uint_as_float(v.w);
  }
  __device__ static void store(float* p, float* o) {       // o is left holding the stored values
    *reinterpret_cast<float4*>(p) = make_float4(o[0], o[1], o[2], o[3]);
  }
};
template <> struct Row16<uint16_t> {   // bf16 storage
  static constexpr int N = 8;
  __device__ static void unpack(const uint4& v, float* o) {
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

// Loads the thread's 16-byte piece of TPT token rows (all in flight together).
template <typename T, int TPT>
__device__ __forceinline__ void load_rows(uint4 (&raw)[TPT], const T* ip, const int (&src)[TPT], long long stride_t) {
#pragma unroll
  for (int tk = 0; tk < TPT; ++tk) raw[tk] = *reinterpret_cast<const uint4*>(ip + (long long)src[tk] * stride_t);
}

// Rotates (if asked), stores and sums the rows that load_rows brought in; acc receives the column sums of what was stored.
template <typename T, int TPT, int NP>
__device__ __forceinline__ void finish_rows(const uint4 (&raw)[TPT], const float (&cs)[TPT][NP], const float (&sn)[TPT][NP],
                                            bool rotate, unsigned valid, T* op, const int (&dst)[TPT], long long stride_t,
                                            float (&acc)[2 * NP]) {
#pragma unroll
  for (int i = 0; i < 2 * NP; ++i) acc[i] = 0.f;
#pragma unroll
  for (int tk = 0; tk < TPT; ++tk) {
    float x[2 * NP];
    Row16<T>::unpack(raw[tk], x);
    if (rotate) {      // uniform
#pragma unroll
      for (int i = 0; i < NP; ++i) {
        const float a0 = x[2 * i], a1 = x[2 * i + 1];
        x[2 * i] = a0 * cs[tk][i] - a1 * sn[tk][i];
        x[2 * i + 1] = a0 * sn[tk][i] + a1 * cs[tk][i];
      }
    }
    if (valid >> tk & 1) {
      Row16<T>::store(op + (long long)dst[tk] * stride_t, x);
#pragma unroll
      for (int i = 0; i < 2 * NP; ++i) acc[i] += x[i];
    }
  }
}

template <typename T, int D>
__global__ __launch_bounds__(256) void k_prologue(const T* __restrict__ q_in, const T* __restrict__ k_in,
                                                  const T* __restrict__ v_in, T* __restrict__ q_out,
                                                  T* __restrict__ k_out, T* __restrict__ v_out,
                                                  float* __restrict__ qc, float* __restrict__ kc,
                                                  float* __restrict__ vc, SegDesc seg, GridDesc gd, Geometry g, int hpw,
                                                  int inverse) {
  constexpr int VEC = Row16<T>::N;
  constexpr int CH = D / VEC;            // 16-byte chunks per row
  constexpr int RP = 256 / CH;           // rows covered per pass
  constexpr int TPT = PBLOCK / RP;       // rows per thread
  constexpr int NP = VEC / 2;            // channel pairs per thread
  __shared__ int s_src[PBLOCK];
  __shared__ int s_pos[PBLOCK][3];
  __shared__ float red[2][RP][D];
  const int j = blockIdx.x, b = blockIdx.z, h0 = blockIdx.y * hpw;
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
  // the thread's rows: where each is read and where it is written (rows past the block's end re-read the block's first
  // row and are dropped).  Forward: gathered from the row-major place, written at the tile-order place; the inverse
  // direction (the transpose, used for gradients) swaps the two.
  int src[TPT], dst[TPT];
  unsigned valid = 0;
#pragma unroll
  for (int tk = 0; tk < TPT; ++tk) {
    const int r = rg + tk * RP, rc = r < bp.n ? r : 0;
    const int raster = s_src[rc], tiled = bp.start + rc;
    src[tk] = inverse ? tiled : raster;
    dst[tk] = inverse ? raster : tiled;
    valid |= (r < bp.n ? 1u : 0u) << tk;
  }
  const int n_it = 3 * min(hpw, g.H - h0);        // (head, tensor) passes of this workgroup, q, k, v of a head in turn
  const long long base0 = (long long)b * g.stride_b + (long long)h0 * g.stride_h + c * VEC;

  // Two sets of landing registers: the rows of pass it + 1 are in flight while pass it is rotated and stored.
  uint4 raw0[TPT], raw1[TPT];
#define ISA_IN_PTR(it) ((((it) % 3) == 0 ? q_in : ((it) % 3) == 1 ? k_in : v_in) + base0 + (long long)((it) / 3) * g.stride_h)
  load_rows<T, TPT>(raw0, ISA_IN_PTR(0), src, g.stride_t);

  // the thread's channel pairs: which coordinate turns them, and how fast; then the sines and cosines of its rows
  // (computed while the first rows are on their way)
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
  float cs[TPT][NP], sn[TPT][NP];
#pragma unroll
  for (int tk = 0; tk < TPT; ++tk) {
    const int r = rg + tk * RP;
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      cs[tk][i] = 1.f; sn[tk][i] = 0.f;
      if (r < bp.n && axis[i] >= 0) {
        const int pos = axis[i] == 0 ? s_pos[r][0] : axis[i] == 1 ? s_pos[r][1] : s_pos[r][2];
        double turns = (double)pos * freq[i] * 0.1591549430918953357689;          // angle / 2 pi
        turns -= rint(turns);                                                        // into [-1/2, 1/2]
        sincospif((float)(2.0 * turns), &sn[tk][i], &cs[tk][i]);
        if (inverse) sn[tk][i] = -sn[tk][i];                                         // turn back
      }
    }
  }

  const float inv_n = 1.0f / (float)bp.n;
  const bool means = qc != nullptr;
  // the second half of a pass: the block means of what was just stored.  red[B] is next written two passes later,
  // behind the barrier of the pass in between.
#define ISA_PASS(RAW, B, it)                                                                                          \
  {                                                                                                                   \
    const int t_ = (it) % 3, hh_ = (it) / 3;                                                                          \
    float acc_[VEC];                                                                                                  \
    finish_rows<T, TPT, NP>(RAW, cs, sn, t_ < 2, valid,                                                               \
                            (t_ == 0 ? q_out : t_ == 1 ? k_out : v_out) + base0 + (long long)hh_ * g.stride_h,         \
                            dst, g.stride_t, acc_);                                                                    \
    if (means) {                                                                                                      \
      _Pragma("unroll") for (int i = 0; i < VEC; ++i) red[B][rg][c * VEC + i] = acc_[i];                              \
      __syncthreads();                                                                                                \
      if (threadIdx.x < D) {                                                                                          \
        float sum_ = 0.f;                                                                                             \
        _Pragma("unroll") for (int r = 0; r < RP; ++r) sum_ += red[B][r][threadIdx.x];                                \
        float* mp_ = t_ == 0 ? qc : t_ == 1 ? kc : vc;                                                                \
        mp_[(((long long)b * g.H + h0 + hh_) * g.T_max + j) * D + threadIdx.x] = sum_ * inv_n;                        \
      }                                                                                                               \
    }                                                                                                                 \
  }
  for (int it = 0; it < n_it; it += 2) {
    if (it + 1 < n_it) load_rows<T, TPT>(raw1, ISA_IN_PTR(it + 1), src, g.stride_t);
    ISA_PASS(raw0, 0, it)
    if (it + 1 < n_it) {
      if (it + 2 < n_it) load_rows<T, TPT>(raw0, ISA_IN_PTR(it + 2), src, g.stride_t);
      ISA_PASS(raw1, 1, it + 1)
    }
  }
#undef ISA_PASS
#undef ISA_IN_PTR
}

// Inverse reordering of one tensor: token p of the tile order goes back to its row-major place.
template <typename T, int D>
__global__ __launch_bounds__(256) void k_untile(const T* __restrict__ x_tiled, T* __restrict__ x_raster, SegDesc seg,
                                                GridDesc gd, Geometry g, int hpw) {
  constexpr int VEC = Row16<T>::N;
  constexpr int CH = D / VEC;
  constexpr int RP = 256 / CH;
  constexpr int TPT = PBLOCK / RP;
  __shared__ int s_src[PBLOCK];
  const int j = blockIdx.x, b = blockIdx.z, h0 = blockIdx.y * hpw;
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
  for (int hh = 0; hh < hpw; ++hh) {
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

// Heads per workgroup: as many as still leave about eight workgroups per compute unit (the per-block set-up, the sines
// and cosines above all, is paid once per workgroup).
static int heads_per_wg(const Problem& pr) {
  const long long blocks = (long long)pr.cnt.T_max * pr.p.B;
  long long hpw = blocks * pr.p.H / 2048;
  if (hpw < 1) hpw = 1;
  if (hpw > pr.p.H) hpw = pr.p.H;
  return (int)hpw;
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
                           void* q_out, void* k_out, void* v_out, float* qc, float* kc, float* vc, bool inverse,
                           hipStream_t st) {
  const GridDesc gd = make_desc(pr, gr);
  const int hpw = heads_per_wg(pr);
  const dim3 grid(pr.cnt.T_max, (pr.p.H + hpw - 1) / hpw, pr.p.B), blk(256);
#define ISA_PRO(T, D)                                                                                                \
  hipLaunchKernelGGL((k_prologue<T, D>), grid, blk, 0, st, (const T*)q_in, (const T*)k_in, (const T*)v_in, (T*)q_out, \
                     (T*)k_out, (T*)v_out, qc, kc, vc, pr.seg, gd, pr.geo, hpw, inverse ? 1 : 0)
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
  const int hpw = heads_per_wg(pr);
  const dim3 grid(pr.cnt.T_max, (pr.p.H + hpw - 1) / hpw, pr.p.B), blk(256);
#define ISA_UNT(T, D) \
  hipLaunchKernelGGL((k_untile<T, D>), grid, blk, 0, st, (const T*)x_tiled, (T*)x_raster, pr.seg, gd, pr.geo, hpw)
  if (pr.p.dtype == ISA_BF16) {
    if (pr.p.D == 128) ISA_UNT(uint16_t, 128); else ISA_UNT(uint16_t, 64);
  } else {
    if (pr.p.D == 128) ISA_UNT(float, 128); else ISA_UNT(float, 64);
  }
#undef ISA_UNT
  return hipGetLastError();
}

}  // namespace isa
