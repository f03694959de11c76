// Backward pass of In-Context Sparse Attention for bf16, D = 128, block = 128 on gfx950 (the paper states that the
// operator is trainable, Sec. 4 "Implementation Detail and Analysis", and gives no formulas: these are the analytic
// gradients of Alg. 1 Stage 4 with the index decisions of Stages 2 and 3 held fixed, exact sets empty, gamma = 0).
//
// With P = softmax weights of a query row (exact branch: over the tokens of the kept blocks; Taylor branch, Eq. 4: over
// the kept blocks' mean keys, each weighted with its token count n_j), delta = rowsum(dO * O) and dP = dO V^T:
//     dS = P * (dP - delta),   dQ = dS K / sqrt(D),   dK = dS^T Q / sqrt(D),   dV = P^T dO,
// and the gradient of a block mean is spread evenly over the block's tokens (dK[t] += dKc[j] / n_j, same for V).
//
// One kernel does all six products.  A workgroup (8 waves) keeps 2 x 128 "stationary" rows in registers and streams
// 64-row tiles of the other side through LDS; per tile it forms T1 = Y1 X1^T (the scores) and, where dS is needed,
// T2 = Y2 X2^T (dP), turns them into W = P or dS in registers and accumulates acc^T += Yt W^T, where Yt is a packed,
// transposed copy of the streamed rows in the key order of the 16x16x32 accumulators (the same copy kernel and
// the same operand layouts as the forward kernel).  The six launches:
//     dQ, exact branch : stationary (Q, dO) of the full-attention blocks,  streamed K, V, K^T of the kept tokens
//     dQ, Taylor branch: stationary (Q, dO) of the Taylor blocks,          streamed Kc, Vc, Kc^T (block means)
//     dKc, dVc         : stationary (Kc, Vc) / Kc rows,                    streamed Q, dO, Q^T / dO^T of the Taylor blocks
//     dK, dV           : stationary (K, V) / K of the kept blocks,         streamed Q, dO, Q^T / dO^T of the full-attention
//                        blocks; the epilogue adds the block's dKc / n_j (dVc / n_j) and writes bf16
// Every output element is written by exactly one workgroup: no atomics, results are reproducible.
#include "attn_mfma.h"

namespace isa {

namespace {

constexpr int STAGE = 2 * K_TILE + V_TILE;           // bf16 elements of one LDS stage: Y1, Y2 and Yt tiles
constexpr int SIDE_BYTES = 1024;                      // per stage: {bias, delta} of the 64 streamed rows (512 B used)

// 16 bytes per lane from global memory straight into LDS (lane i -> LDS bytes lds_addr + 16 i); inline assembly so
// that the only wait for these loads is the explicit one at the top of the loop.
__device__ __forceinline__ void dma16(const void* sbase, uint32_t voff_bytes, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :: "s"(lds_addr), "v"(voff_bytes), "s"(sbase) : "memory");
}
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
  return (uint32_t)(size_t)(__attribute__((address_space(3))) const void*)p;
}
__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

}  // namespace

struct BwdArgs {
  // stationary rows: token tensors (strides of `geo`, blocks taken from `stat_list`) or gathered mean rows [bh][Tn_pad][128]
  const uint16_t* x1; const uint16_t* x2;
  const int* stat_list;                       // [bh][T_max] block ids; unused for mean rows
  const float* bx; const float* dx;           // per stationary row: additive exponent term / delta ([bh][S_max] or [bh][Tn_pad]); null = 0
  // streamed tiles: token tensors (tiles from `ytab`) or gathered mean rows
  const uint16_t* y1; const uint16_t* y2; const uint16_t* yt;
  const int4* ytab;                           // [bh][T_max] {token offset, tokens, block id} per list entry; unused for mean rows
  const float2* ybd;                          // {additive exponent term (-inf: masked), delta} per streamed position
  // outputs
  uint16_t* out_bf; float* out_f32;           // token rows (bf16, strides of `geo`) or mean rows (fp32 [bh][Tn_pad][128])
  const float* add_rows;                      // [bh][Tn_pad][128] or null: row `entry`, divided by the block's tokens, is added to every row
  float oscale;
  const int* blk_start; const int* blk_n;
  Geometry geo; Counts cnt;
  int Tn_pad, S_max;
  int stat_kind;                              // token rows: 0 full-attention blocks, 1 Taylor blocks, 2 kept blocks
  int stream_kind;                            // token tiles: 0 kept blocks, 1 full-attention blocks, 2 Taylor blocks
  int items;                                  // work items (pairs of stationary blocks) per (batch, head) in this launch
};

// SM: stationary rows are block means; YM: streamed rows are block means; T2: W = P * (T2 - delta), else W = P.
template <bool SM, bool YM, bool T2>
__global__ __launch_bounds__(512, 1) void k_attn_bwd(BwdArgs a) {
  __shared__ __attribute__((aligned(1024))) uint16_t lds[2 * STAGE + 2 * SIDE_BYTES / 2];
  // Workgroup ids go round-robin over the 8 XCDs: XCD x gets every 8th (batch, head) and works through its items one
  // head after the other, so that the workgroups that run together on an XCD (and share its L2) stream the same rows.
  const int xcd = blockIdx.x & 7, jj = blockIdx.x >> 3;
  const int item = jj % a.items, bhid = (jj / a.items) * 8 + xcd;
  if (bhid >= a.geo.B * a.geo.H) return;
  const int h = bhid % a.geo.H, b = bhid / a.geo.H;
  const int T_new = a.cnt.b[b].T_new, n_full = a.cnt.b[b].n_full, n_flat = a.cnt.b[b].n_flat;
  const int T_max = a.geo.T_max;
  const long long bh = bhid;
  const int n_stat = SM ? (T_new + 127) / 128 : (a.stat_kind == 0 ? n_full : a.stat_kind == 1 ? n_flat : T_new);
  if (2 * item >= n_stat) return;
  const int n_ent = YM ? 0 : (a.stream_kind == 0 ? T_new : a.stream_kind == 1 ? n_full : n_flat);
  const int n_tiles = YM ? (T_new + KT - 1) / KT : 2 * n_ent;
  const long long tbase = (long long)b * a.geo.stride_b + (long long)h * a.geo.stride_h;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int grp = wave >> 2, wq = wave & 3;
  const int r16 = lane & 15, q = lane >> 4;

  // ---- stationary rows of this wave: 32 rows of block `entry` (the second group idles on block 0 in the last pair of
  // an odd list: computes, stores nothing)
  const int entry = 2 * item + grp;
  const bool active = entry < n_stat;
  const int e_use = active ? entry : 0;
  int n_x, x_start = 0;
  const uint16_t *xb1, *xb2;
  long long xstride;
  long long bx_base;
  if (SM) {
    n_x = active ? min(128, T_new - entry * 128) : 0;
    xb1 = a.x1 + (bh * a.Tn_pad + (long long)e_use * 128) * MD;
    xb2 = T2 ? a.x2 + (bh * a.Tn_pad + (long long)e_use * 128) * MD : nullptr;
    xstride = MD;
    bx_base = bh * a.Tn_pad + (long long)e_use * 128;
  } else {
    const int blk = a.stat_list[bh * T_max + e_use];
    n_x = active ? a.blk_n[b * T_max + blk] : 0;
    x_start = a.blk_start[b * T_max + blk];
    xb1 = a.x1 + tbase + (long long)x_start * a.geo.stride_t;
    xb2 = T2 ? a.x2 + tbase + (long long)x_start * a.geo.stride_t : nullptr;
    xstride = a.geo.stride_t;
    bx_base = bh * a.S_max + x_start;
  }
  int rowq[2];
  bool row_ok[2];
  bf16x8 x1f[2][4], x2f[2][4];
  float bxv[2], dxv[2];
#pragma unroll
  for (int qt = 0; qt < 2; ++qt) {
    rowq[qt] = wq * 32 + 16 * qt + r16;
    row_ok[qt] = rowq[qt] < n_x;
    const long long ro = (long long)(row_ok[qt] ? rowq[qt] : 0) * xstride + 8 * q;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      x1f[qt][ks] = *reinterpret_cast<const bf16x8*>(xb1 + ro + 32 * ks);
      if (T2) x2f[qt][ks] = *reinterpret_cast<const bf16x8*>(xb2 + ro + 32 * ks);
    }
    bxv[qt] = (a.bx && row_ok[qt]) ? a.bx[bx_base + rowq[qt]] : 0.f;
    dxv[qt] = (a.dx && row_ok[qt]) ? a.dx[bx_base + rowq[qt]] : 0.f;
  }
  // consume the prologue loads here: the waits the compiler places inside the loop must not cover them
#pragma unroll
  for (int qt = 0; qt < 2; ++qt) {
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      asm volatile("" : "+v"(x1f[qt][ks]));
      if (T2) asm volatile("" : "+v"(x2f[qt][ks]));
    }
    asm volatile("" : "+v"(bxv[qt]), "+v"(dxv[qt]));
  }

  // ---- tile loads: global -> LDS, 16 bytes per lane, rows XOR-swizzled on the source side (the layouts of the forward
  // kernel: natural tiles 64 rows x 256 B, chunk c of row r at c ^ (r & 15); packed tiles as two units of 128 rows x
  // 64 B, chunk c of row r at c ^ ((r >> 2) & 3))
  const int l16 = lane >> 4;
  uint32_t nchunk_b[2];
  int nrow_l[2];
  uint32_t tlane_b[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    nrow_l[i] = 8 * wave + 4 * i + l16;
    nchunk_b[i] = (uint32_t)((((lane & 15) ^ (nrow_l[i] & 15)) * 8) * 2);
    tlane_b[i] = (uint32_t)(((wave < 4 ? 0 : 32) + (((wave * 2 + i) & 7) * 16 + (lane >> 2)) * KT + (((lane & 3) ^ (l16 & 3)) * 8)) * 2);
  }
  const uint32_t ystride_b = (uint32_t)(YM ? MD : (int)a.geo.stride_t) * 2u;
  const char* const y1_head = reinterpret_cast<const char*>(YM ? a.y1 + bh * a.Tn_pad * MD : a.y1 + tbase);
  const char* const y2_head = T2 ? reinterpret_cast<const char*>(YM ? a.y2 + bh * a.Tn_pad * MD : a.y2 + tbase) : nullptr;
  const char* const yt_head = reinterpret_cast<const char*>(
      YM ? a.yt + bh * (a.Tn_pad / KT) * (long long)(MD * KT) : a.yt + bh * T_max * 2 * (long long)(MD * KT));
  const char* const ybd_head = reinterpret_cast<const char*>(YM ? a.ybd + bh * a.Tn_pad : a.ybd + bh * T_max * 128);
  // The table row of a tile is fetched one iteration before the tile's loads are issued, so that its latency is not
  // waited for inside the loop.
  auto row_of = [&](int T) -> int4 {
    if (YM || n_ent == 0) return make_int4(0, 0, 0, 0);
    return a.ytab[bh * T_max + min(T >> 1, n_ent - 1)];
  };
  auto issue_tile = [&](int T, int stage, const int4 ent) {
    uint32_t y_off, t_off, bd_off;
    int nk;
    if (YM) {
      y_off = (uint32_t)T * (uint32_t)(KT * MD * 2);
      t_off = (uint32_t)T * (uint32_t)(MD * KT * 2);
      bd_off = (uint32_t)T * (uint32_t)(KT * 8);
      nk = KT;                                            // the gathered mean arrays are padded to whole tiles
    } else {
      const int sub = T & 1;
      const bool empty = ent.y <= sub * KT;               // second tile of a short block: masked, reads the block's first rows
      y_off = (uint32_t)(ent.x + (empty ? 0 : sub * KT)) * ystride_b;
      t_off = ((uint32_t)ent.z * 2u + (uint32_t)sub) * (uint32_t)(MD * KT * 2);
      bd_off = (uint32_t)((T >> 1) * 128 + sub * KT) * 8u;
      nk = empty ? 1 : min(KT, ent.y - sub * KT);
    }
    // wave-uniform by construction; made scalar explicitly so that the bases of the loads live in scalar registers
    y_off = __builtin_amdgcn_readfirstlane(y_off);
    t_off = __builtin_amdgcn_readfirstlane(t_off);
    bd_off = __builtin_amdgcn_readfirstlane(bd_off);
    nk = __builtin_amdgcn_readfirstlane(nk);
    uint16_t* sb = lds + stage * STAGE;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const uint32_t ro = (uint32_t)min(nrow_l[i], nk - 1) * ystride_b + nchunk_b[i];     // rows past the end re-read the last one
      dma16(y1_head + y_off, ro, lds_addr(sb + (wave * 2 + i) * 512));
      if (T2) dma16(y2_head + y_off, ro, lds_addr(sb + K_TILE + (wave * 2 + i) * 512));
      dma16(yt_head + t_off, tlane_b[i], lds_addr(sb + 2 * K_TILE + (wave * 2 + i) * 512));
    }
    if (wave == 0)                                         // {bias, delta} of the 64 rows: 512 B, lanes 32..63 repeat lanes 0..31
      dma16(ybd_head + bd_off, (uint32_t)(lane & 31) * 16u, lds_addr(lds + 2 * STAGE + stage * (SIDE_BYTES / 2)));
  };

  // per-lane fragment offsets (bf16 elements), as in the forward kernel
  int koff[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) koff[ks] = r16 * MD + (((4 * ks + q) ^ r16) * 8);
  const int voff = r16 * 32 + ((q ^ ((r16 >> 2) & 3)) * 8);

  f32x4 acc[8][2];
#pragma unroll
  for (int ct = 0; ct < 8; ++ct)
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) acc[ct][qt] = f32x4{0.f, 0.f, 0.f, 0.f};
  const float cscale = 1.4426950408889634f / sqrtf((float)MD);       // log2(e) / sqrt(D)

  int4 ent_next = row_of(0);
  if (n_tiles > 0) issue_tile(0, 0, ent_next);
  ent_next = row_of(1);
  for (int T = 0; T < n_tiles; ++T) {
    // this wave's loads of tile T have landed; after the barrier everybody's have, and everybody has finished reading
    // the other stage (tile T - 1), which the loads of tile T + 1 now overwrite
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (T + 1 < n_tiles) issue_tile(T + 1, (T + 1) & 1, ent_next);
    ent_next = row_of(T + 2);
    const uint16_t* sb = lds + (T & 1) * STAGE;
    const float2* side = reinterpret_cast<const float2*>(lds + 2 * STAGE + (T & 1) * (SIDE_BYTES / 2));
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {
      f32x4 t1[2][2], t2[2][2];
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int qt = 0; qt < 2; ++qt) { t1[kt][qt] = f32x4{0.f, 0.f, 0.f, 0.f}; t2[kt][qt] = f32x4{0.f, 0.f, 0.f, 0.f}; }
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
          const bf16x8 f1 = *reinterpret_cast<const bf16x8*>(sb + (32 * hh + 16 * kt) * MD + koff[ks]);
          t1[kt][0] = mfma16(f1, x1f[0][ks], t1[kt][0]);
          t1[kt][1] = mfma16(f1, x1f[1][ks], t1[kt][1]);
          if (T2) {
            const bf16x8 f2 = *reinterpret_cast<const bf16x8*>(sb + K_TILE + (32 * hh + 16 * kt) * MD + koff[ks]);
            t2[kt][0] = mfma16(f2, x2f[0][ks], t2[kt][0]);
            t2[kt][1] = mfma16(f2, x2f[1][ks], t2[kt][1]);
          }
        }
      // W: element 4 kt + i of a lane's fragment is streamed row 32 hh + 16 kt + 4 q + i
      bf16x8 w[2];
#pragma unroll
      for (int kt = 0; kt < 2; ++kt) {
        float2 bd[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) bd[i] = side[32 * hh + 16 * kt + 4 * q + i];
#pragma unroll
        for (int qt = 0; qt < 2; ++qt)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float p = __builtin_amdgcn_exp2f(fmaf(t1[kt][qt][i], cscale, bd[i].x + bxv[qt]));
            const float val = T2 ? p * (t2[kt][qt][i] - dxv[qt] - bd[i].y) : p;
            w[qt][4 * kt + i] = (__bf16)val;
          }
      }
#pragma unroll
      for (int ct = 0; ct < 8; ++ct) {
        const bf16x8 ft = *reinterpret_cast<const bf16x8*>(sb + 2 * K_TILE + hh * (V_TILE / 2) + ct * 16 * 32 + voff);
        acc[ct][0] = mfma16(ft, w[0], acc[ct][0]);
        acc[ct][1] = mfma16(ft, w[1], acc[ct][1]);
      }
    }
  }

  // ---- store: element i of acc[ct][qt] is channel 16 ct + 4 q + i of stationary row 16 qt + r
  const float inv_n = n_x > 0 ? 1.0f / (float)n_x : 0.f;
  const float* addp = a.add_rows ? a.add_rows + (bh * a.Tn_pad + e_use) * MD + 4 * q : nullptr;
#pragma unroll
  for (int qt = 0; qt < 2; ++qt) {
    if (!row_ok[qt]) continue;
    const int row = rowq[qt];
#pragma unroll
    for (int ct = 0; ct < 8; ++ct) {
      float4 r = make_float4(acc[ct][qt][0] * a.oscale, acc[ct][qt][1] * a.oscale, acc[ct][qt][2] * a.oscale,
                             acc[ct][qt][3] * a.oscale);
      if (addp) {
        const float4 m4 = *reinterpret_cast<const float4*>(addp + 16 * ct);
        r.x = fmaf(m4.x, inv_n, r.x); r.y = fmaf(m4.y, inv_n, r.y);
        r.z = fmaf(m4.z, inv_n, r.z); r.w = fmaf(m4.w, inv_n, r.w);
      }
      if (SM) {
        *reinterpret_cast<float4*>(a.out_f32 + (bh * a.Tn_pad + (long long)entry * 128 + row) * MD + 16 * ct + 4 * q) = r;
      } else {
        bf16x2 lo = {(__bf16)r.x, (__bf16)r.y};
        bf16x2 hi = {(__bf16)r.z, (__bf16)r.w};
        uint2 o;
        o.x = *reinterpret_cast<uint32_t*>(&lo);
        o.y = *reinterpret_cast<uint32_t*>(&hi);
        *reinterpret_cast<uint2*>(a.out_bf + tbase + (long long)(x_start + row) * a.geo.stride_t + 16 * ct + 4 * q) = o;
      }
    }
  }
}

// delta[bh][token] = sum_d dO * O (fp32); 16 lanes per token row, 16 bytes per lane and tensor.
__global__ __launch_bounds__(256) void k_bwd_delta(const uint16_t* __restrict__ o, const uint16_t* __restrict__ d_o,
                                                   float* __restrict__ delta, Geometry g, Counts cnt, int S_max) {
  const int h = blockIdx.y, b = blockIdx.z;
  const int t = blockIdx.x * 16 + (threadIdx.x >> 4), c16 = threadIdx.x & 15;
  const bool ok = t < cnt.b[b].S;
  float s = 0.f;
  if (ok) {
    const long long off = (long long)b * g.stride_b + (long long)h * g.stride_h + (long long)t * g.stride_t + 8 * c16;
    const uint4 uo = *reinterpret_cast<const uint4*>(o + off), ud = *reinterpret_cast<const uint4*>(d_o + off);
    const uint32_t wo[4] = {uo.x, uo.y, uo.z, uo.w}, wd[4] = {ud.x, ud.y, ud.z, ud.w};
#pragma unroll
    for (int i = 0; i < 4; ++i)
      s += __uint_as_float(wo[i] << 16) * __uint_as_float(wd[i] << 16) +
           __uint_as_float(wo[i] & 0xffff0000u) * __uint_as_float(wd[i] & 0xffff0000u);
  }
#pragma unroll
  for (int m = 8; m >= 1; m >>= 1) s += __shfl_xor(s, m, 64);
  if (ok && c16 == 0) delta[((long long)b * g.H + h) * S_max + t] = s;
}

// Per list entry: the table row of its block and the {exponent term, delta} pair of each of its 128 row positions
// (masked positions: -inf, 0).  kind 0: kept blocks as streamed keys (term 0), plus the per-mean arrays of the Taylor
// branch (log2 n_j per gathered mean, -inf for the padding); kinds 1, 2: full-attention / Taylor blocks as streamed
// queries (term = minus the row's log-sum-exp in the log2 domain, delta of the row).
__global__ __launch_bounds__(128) void k_bwd_rows(const int* __restrict__ list, int kind, const int4* __restrict__ btab,
                                                  const float* __restrict__ nlse, const float* __restrict__ delta,
                                                  int4* __restrict__ tab, float2* __restrict__ ybd,
                                                  float2* __restrict__ ybd_mean, float* __restrict__ bx_mean, Counts cnt,
                                                  int H, int Tn_pad, int S_max) {
  const int e = blockIdx.x, h = blockIdx.y, b = blockIdx.z, r = threadIdx.x;
  const int T_max = cnt.T_max;
  const long long bh = (long long)b * H + h;
  const int n_list = kind == 0 ? cnt.b[b].T_new : kind == 1 ? cnt.b[b].n_full : cnt.b[b].n_flat;
  if (kind == 0 && e < Tn_pad && r == 0) {
    float l2 = -INFINITY;
    if (e < n_list) l2 = log2f((float)btab[b * T_max + list[bh * T_max + e]].y);
    ybd_mean[bh * Tn_pad + e] = make_float2(l2, 0.f);
    bx_mean[bh * Tn_pad + e] = e < n_list ? l2 : 0.f;
  }
  if (e >= n_list || e >= T_max) return;
  const int4 ent = btab[b * T_max + list[bh * T_max + e]];
  if (r == 0) tab[bh * T_max + e] = ent;
  float2 v = make_float2(-INFINITY, 0.f);
  if (r < ent.y) {
    if (kind == 0) v = make_float2(0.f, 0.f);
    else v = make_float2(nlse[bh * S_max + ent.x + r], delta[bh * S_max + ent.x + r]);
  }
  ybd[(bh * T_max + e) * 128 + r] = v;
}

// Zeroes the rows of a token tensor (gradients of keys and values of context blocks that were not kept).
__global__ __launch_bounds__(256) void k_bwd_zero(uint16_t* __restrict__ x, Geometry g, Counts cnt) {
  const int h = blockIdx.y, b = blockIdx.z;
  const int t = blockIdx.x * 16 + (threadIdx.x >> 4), c16 = threadIdx.x & 15;
  if (t >= cnt.b[b].S) return;
  *reinterpret_cast<uint4*>(x + (long long)b * g.stride_b + (long long)h * g.stride_h + (long long)t * g.stride_t + 8 * c16) =
      make_uint4(0, 0, 0, 0);
}

hipError_t launch_attn_bwd(const Problem& pr, const Workspace& ws, const void* q, const void* k, const void* v,
                           const void* out, const void* d_out, const int* kv_list, const int* full_list,
                           const int* flat_list, void* dq, void* dk, void* dv, hipStream_t st) {
  const int B = pr.p.B, H = pr.p.H, T_max = pr.cnt.T_max;
  int S_max = pr.S_max, sf = 0, sl = 0, sk = 0;
  for (int b = 0; b < B; ++b) {
    const BatchCounts& c = pr.cnt.b[b];
    sf = c.n_full > sf ? c.n_full : sf;
    sl = c.n_flat > sl ? c.n_flat : sl;
    sk = c.T_new > sk ? c.T_new : sk;
  }
  const dim3 bhg(1, H, B);
#define ISA_BWD_CHECK()                           \
  do {                                            \
    hipError_t e__ = hipGetLastError();           \
    if (e__ != hipSuccess) return e__;            \
  } while (0)
  // delta, zero fill, per-list tables and row terms
  hipLaunchKernelGGL(k_bwd_delta, dim3((S_max + 15) / 16, H, B), dim3(256), 0, st, (const uint16_t*)out,
                     (const uint16_t*)d_out, ws.delta, pr.geo, pr.cnt, S_max);
  ISA_BWD_CHECK();
  hipLaunchKernelGGL(k_bwd_zero, dim3((S_max + 15) / 16, H, B), dim3(256), 0, st, (uint16_t*)dk, pr.geo, pr.cnt);
  hipLaunchKernelGGL(k_bwd_zero, dim3((S_max + 15) / 16, H, B), dim3(256), 0, st, (uint16_t*)dv, pr.geo, pr.cnt);
  ISA_BWD_CHECK();
  const int gx = T_max > pr.Tn_pad ? T_max : pr.Tn_pad;
  hipLaunchKernelGGL(k_bwd_rows, dim3(gx, H, B), dim3(128), 0, st, kv_list, 0, ws.btab, ws.nlse, ws.delta, ws.ktab,
                     ws.ybd_kv, ws.ybd_mean, ws.bx_mean, pr.cnt, H, pr.Tn_pad, S_max);
  hipLaunchKernelGGL(k_bwd_rows, dim3(gx, H, B), dim3(128), 0, st, full_list, 1, ws.btab, ws.nlse, ws.delta, ws.ftab,
                     ws.ybd_full, ws.ybd_mean, ws.bx_mean, pr.cnt, H, pr.Tn_pad, S_max);
  hipLaunchKernelGGL(k_bwd_rows, dim3(gx, H, B), dim3(128), 0, st, flat_list, 2, ws.btab, ws.nlse, ws.delta, ws.ltab,
                     ws.ybd_flat, ws.ybd_mean, ws.bx_mean, pr.cnt, H, pr.Tn_pad, S_max);
  ISA_BWD_CHECK();

  BwdArgs a;
  a.blk_start = ws.blk_start; a.blk_n = ws.blk_n;
  a.geo = pr.geo; a.cnt = pr.cnt; a.Tn_pad = pr.Tn_pad; a.S_max = S_max;
  const float scale = 1.0f / sqrtf((float)MD);
  const uint16_t *Q = (const uint16_t*)q, *K = (const uint16_t*)k, *V = (const uint16_t*)v, *DO = (const uint16_t*)d_out;
  hipError_t e;

  // ---- dQ: exact branch over the kept tokens (needs K^T packed), Taylor branch over the kept blocks' means
  if ((e = launch_pack_t(pr, ws, K, ws.vt, st)) != hipSuccess) return e;
  a.x1 = Q; a.x2 = DO; a.bx = ws.nlse; a.dx = ws.delta;
  a.out_bf = (uint16_t*)dq; a.out_f32 = nullptr; a.add_rows = nullptr; a.oscale = scale;
  if (sf > 0) {
    a.stat_list = full_list; a.stat_kind = 0;
    a.y1 = K; a.y2 = V; a.yt = ws.vt; a.ytab = ws.ktab; a.ybd = ws.ybd_kv; a.stream_kind = 0;
    a.items = (sf + 1) / 2;
    hipLaunchKernelGGL((k_attn_bwd<false, false, true>), dim3((unsigned)(a.items * 8 * ((B * H + 7) / 8))), dim3(512), 0, st, a);
    ISA_BWD_CHECK();
  }
  if (sl > 0) {
    a.stat_list = flat_list; a.stat_kind = 1;
    a.y1 = ws.kcn; a.y2 = ws.vcn; a.yt = ws.kcnt; a.ytab = nullptr; a.ybd = ws.ybd_mean; a.stream_kind = 0;
    a.items = (sl + 1) / 2;
    hipLaunchKernelGGL((k_attn_bwd<false, true, true>), dim3((unsigned)(a.items * 8 * ((B * H + 7) / 8))), dim3(512), 0, st, a);
    ISA_BWD_CHECK();
  }

  // ---- dKc and dK (streamed Q, dO, Q^T packed)
  if ((e = launch_pack_t(pr, ws, Q, ws.vt, st)) != hipSuccess) return e;
  a.y1 = Q; a.y2 = DO; a.yt = ws.vt; a.dx = nullptr;
  const int n_mean_pairs = ((sk + 127) / 128 + 1) / 2;
  if (sl > 0) {
    a.x1 = ws.kcn; a.x2 = ws.vcn; a.stat_list = nullptr; a.stat_kind = 2; a.bx = ws.bx_mean;
    a.ytab = ws.ltab; a.ybd = ws.ybd_flat; a.stream_kind = 2;
    a.out_bf = nullptr; a.out_f32 = ws.dkc; a.add_rows = nullptr; a.oscale = scale;
    a.items = n_mean_pairs;
    hipLaunchKernelGGL((k_attn_bwd<true, false, true>), dim3((unsigned)(a.items * 8 * ((B * H + 7) / 8))), dim3(512), 0, st, a);
    ISA_BWD_CHECK();
  }
  a.x1 = K; a.x2 = V; a.stat_list = kv_list; a.stat_kind = 2; a.bx = nullptr;
  a.ytab = ws.ftab; a.ybd = ws.ybd_full; a.stream_kind = 1;
  a.out_bf = (uint16_t*)dk; a.out_f32 = nullptr; a.add_rows = sl > 0 ? ws.dkc : nullptr; a.oscale = scale;
  a.items = (sk + 1) / 2;
  if (a.items > 0)
    hipLaunchKernelGGL((k_attn_bwd<false, false, true>), dim3((unsigned)(a.items * 8 * ((B * H + 7) / 8))), dim3(512), 0, st, a);
  ISA_BWD_CHECK();

  // ---- dVc and dV (streamed Q, dO^T packed)
  if ((e = launch_pack_t(pr, ws, DO, ws.vt, st)) != hipSuccess) return e;
  a.y1 = Q; a.y2 = nullptr; a.yt = ws.vt;
  if (sl > 0) {
    a.x1 = ws.kcn; a.x2 = nullptr; a.stat_list = nullptr; a.stat_kind = 2; a.bx = ws.bx_mean;
    a.ytab = ws.ltab; a.ybd = ws.ybd_flat; a.stream_kind = 2;
    a.out_bf = nullptr; a.out_f32 = ws.dvc; a.add_rows = nullptr; a.oscale = 1.0f;
    a.items = n_mean_pairs;
    hipLaunchKernelGGL((k_attn_bwd<true, false, false>), dim3((unsigned)(a.items * 8 * ((B * H + 7) / 8))), dim3(512), 0, st, a);
    ISA_BWD_CHECK();
  }
  a.x1 = K; a.x2 = nullptr; a.stat_list = kv_list; a.stat_kind = 2; a.bx = nullptr;
  a.ytab = ws.ftab; a.ybd = ws.ybd_full; a.stream_kind = 1;
  a.out_bf = (uint16_t*)dv; a.out_f32 = nullptr; a.add_rows = sl > 0 ? ws.dvc : nullptr; a.oscale = 1.0f;
  a.items = (sk + 1) / 2;
  if (a.items > 0)
    hipLaunchKernelGGL((k_attn_bwd<false, false, false>), dim3((unsigned)(a.items * 8 * ((B * H + 7) / 8))), dim3(512), 0, st, a);
  ISA_BWD_CHECK();
#undef ISA_BWD_CHECK
  return hipSuccess;
}

}  // namespace isa
