// Ping-pong MFMA attention kernel for bf16, D = 128, block = 128 on gfx950: dense attention, the exact
// branch of ISA (Alg. 1 Stage 4 / Alg. 2 Part A) and the Taylor branch without exact sets (Eq. 4, Alg. 2
// Part B).
//
// One workgroup of 8 waves owns two query blocks (256 rows): waves 0-3 (group A) the first, waves 4-7
// (group B) the second; wave w of a group owns rows 32w .. 32w+31 of its block.  Both groups walk the same
// sequence of 64-key tiles, which all 8 waves load cooperatively into LDS, so each K / V^T tile is fetched
// once per 256 query rows.
//
// A SIMD holds one wave of each group.  The work per tile splits into a matrix phase X(j) = { O += V P of
// tile j-1, S = K Q of tile j } (32 MFMAs, no vector ALU work) and a softmax phase Y(j) (exp2 and friends,
// no MFMA).  Left alone, two waves that run the same X/Y cycle on one SIMD fall into step -- both in X,
// then both in Y -- and the matrix pipe idles through every Y.  Here group B is started one phase late and
// a workgroup barrier closes every phase, so that while one group's wave keeps the SIMD's matrix pipe busy
// the other group's wave uses its vector ALU, and vice versa.
//
// Scores are computed transposed (S^T = K Q^T) and V is read from the packed, key-permuted V^T copy, as in
// the 4-wave kernel: P stays in registers in the layout the second product needs.
#include "attn_mfma.h"

namespace isa {

struct PTile {                              // wave-uniform description of one 64-key tile
  const uint16_t* krows;                    // row 0 of the block (token tiles) or of the tile (mean tiles)
  const uint16_t* vt;                       // 128 x 64 packed V^T
  const float* bias;                        // per-key additive term on the raw score, or null
  int row0, kstride, nk, last_row;
};

__global__ __launch_bounds__(512, 1) void k_attn_pp(MfmaArgs a) {
  __shared__ __attribute__((aligned(1024))) uint16_t lds[2 * K_TILE + 2 * V_TILE];
  uint16_t* ldsK = lds;                     // K of tile j lives in buffer j & 1
  uint16_t* ldsV = lds + 2 * K_TILE;        // V^T of tile j lives in buffer j & 1

  // ---- which work item: consecutive logical ids go to the same XCD, so that the workgroups that run
  // together on one XCD (and share its L2) read the same head's keys and values
  const int per_xcd = gridDim.x >> 3;       // grid is a multiple of 8
  const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (logical >= a.total) return;
  const int slot = logical % a.slots;
  const int bhid = logical / a.slots;
  const int h = bhid % a.geo.H, b = bhid / a.geo.H;
  const BatchCounts c = a.cnt.b[b];
  const int T_max = a.geo.T_max;
  const long long bh = bhid;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // 0..7, scalar
  const int grp = wave >> 2, wq = wave & 3;
  const int col = lane & 31, g = lane >> 5;

  // slots of a (batch, head): pairs of exact-branch blocks first (the long ones), then pairs of Taylor blocks
  const int full_pairs = a.dense ? (c.T + 1) >> 1 : (c.n_full + 1) >> 1;
  const int flat_pairs = (a.dense || !a.taylor_here) ? 0 : (c.n_flat + 1) >> 1;
  if (slot >= full_pairs + flat_pairs) return;
  const bool taylor = slot >= full_pairs;
  const int* kvl = a.dense ? nullptr : a.kv_list + bh * T_max;
  const int n_list = a.dense ? c.T : c.T_new;
  int entry, n_entries;
  const int* qlist;
  if (a.dense) { entry = 2 * slot + grp; n_entries = c.T; qlist = nullptr; }
  else if (!taylor) { entry = 2 * slot + grp; n_entries = c.n_full; qlist = a.full_list + bh * T_max; }
  else { entry = 2 * (slot - full_pairs) + grp; n_entries = c.n_flat; qlist = a.flat_list + bh * T_max; }
  const bool active = entry < n_entries;                          // group B idles in the last pair of an odd list
  const int* bn = a.blk_n + b * T_max;
  const int* bs = a.blk_start + b * T_max;
  const int qi = active ? (qlist ? qlist[entry] : entry) : 0;
  const int n_q = active ? bn[qi] : 0;
  const int q_start = bs[qi];
  const long long tbase = (long long)b * a.geo.stride_b + (long long)h * a.geo.stride_h;
  const int n_tiles = taylor ? (n_list + KT - 1) / KT : 2 * n_list;

  auto tile_at = [&](int idx, PTile& t) {                          // idx < n_tiles
    if (!taylor) {
      const int e = idx >> 1, sub = idx & 1;
      const int j = a.dense ? e : kvl[e];
      const int n_j = bn[j];
      t.krows = a.k + tbase + (long long)bs[j] * a.geo.stride_t;
      t.row0 = sub * KT;
      t.kstride = (int)a.geo.stride_t;
      t.vt = a.vt + ((bh * T_max + j) * 2 + sub) * (long long)(MD * KT);
      t.bias = nullptr;
      t.nk = max(0, min(KT, n_j - sub * KT));
      t.last_row = max(n_j - 1, 0);
    } else {
      const long long row0 = bh * a.Tn_pad + (long long)idx * KT;
      t.krows = a.kcn + row0 * MD;
      t.row0 = 0;
      t.kstride = MD;
      t.vt = a.vcnt + (bh * (a.Tn_pad / KT) + idx) * (long long)(MD * KT);
      t.bias = a.biasn + row0;
      t.nk = min(KT, n_list - idx * KT);
      t.last_row = KT - 1;                                          // the gathered arrays are padded to whole tiles
    }
  };

  // ---- Q fragments: B operand of S^T = K Q^T; lane holds channels 16s + 8g .. +7 of its query row
  const int row = wq * 32 + col;
  const bool row_ok = row < n_q;
  const uint16_t* qp = a.q + tbase + (long long)(q_start + (row_ok ? row : 0)) * a.geo.stride_t + 8 * g;
  bf16x8 qf[8];
#pragma unroll
  for (int s = 0; s < 8; ++s) qf[s] = *reinterpret_cast<const bf16x8*>(qp + 16 * s);

  // ---- global -> LDS, 16 bytes per lane, no staging registers.  One wave instruction fills 1024 contiguous
  // LDS bytes (lane i -> bytes 16i..16i+15), so rows cannot be padded; instead the 16-byte chunk c of a row is
  // stored at chunk position c ^ f(row), applied on the source side: the lane that fills position pc of row r
  // fetches chunk pc ^ f(r).  K rows are 256 B (f = r & 15), V^T rows are 128 B (f = (r >> 1) & 7); with these
  // the 16-lane groups of a b128 fragment read hit 16 different bank groups.  A wave issues two such
  // instructions per tile and tensor; instruction i of wave w fills chunks (2w+i)*64 .. +63, i.e. K rows
  // 8w+4i .. +3 and V^T rows 16w+8i .. +7.
  const int l16 = lane >> 4;
  uint32_t kchunk_b[2], vsrc_b;
#pragma unroll
  for (int i = 0; i < 2; ++i) kchunk_b[i] = (uint32_t)((((lane & 15) ^ ((8 * wave + 4 * i + l16) & 15)) * 8) * 2);
  vsrc_b = (uint32_t)((((lane >> 3) * KT) + (((lane & 7) ^ (l16 & 7)) * 8)) * 2);   // (row >> 1) & 7 = lane >> 4 for rows 16w+8i+lane/8
  auto load_k = [&](const PTile& t, int buf) {
    const char* kb = reinterpret_cast<const char*>(t.krows);
    const uint32_t kstride_b = (uint32_t)t.kstride * 2u;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      // rows past the block's end re-read its last row; the row index is never negative
      const int r = max(min(t.row0 + wave * 8 + 4 * i + l16, t.last_row), 0);
      const uint32_t koff_b = (uint32_t)r * kstride_b + kchunk_b[i];
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(kb + koff_b),
                                       (__attribute__((address_space(3))) void*)(ldsK + buf * K_TILE + (wave * 2 + i) * 512), 16, 0, 0);
    }
  };
  auto load_v = [&](const PTile& t, int buf) {
    const char* vb = reinterpret_cast<const char*>(t.vt) + wave * 2048;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      // rows 16w+8i+lane/8: (row >> 1) & 7 = ((8w + 4i) + lane/16) & 7 = (4i + lane/16) & 7
      const uint32_t off = (uint32_t)((((lane >> 3) * KT) + (((lane & 7) ^ ((4 * i + l16) & 7)) * 8)) * 2);
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(vb + i * 1024 + off),
                                       (__attribute__((address_space(3))) void*)(ldsV + buf * V_TILE + (wave * 2 + i) * 512), 16, 0, 0);
    }
  };
  (void)vsrc_b;

  // per-lane fragment offsets (bf16 elements): K row = col, chunk (2s+g) ^ (col & 15); V^T row = col, chunk (2ks+g) ^ ((col>>1)&7)
  int koff[8], voff[4];
#pragma unroll
  for (int s = 0; s < 8; ++s) koff[s] = col * MD + (((2 * s + g) ^ (col & 15)) * 8);
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) voff[ks] = col * KT + (((2 * ks + g) ^ ((col >> 1) & 7)) * 8);

  f32x16 oacc[4], sacc[2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) oacc[i][e] = 0.f;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) sacc[i][e] = 0.f;
  bf16x8 pf[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 8; ++e) pf[i][e] = (__bf16)0.0f;
  float m_run = M_INIT, l_run = 0.f;
  const float cscale = 1.4426950408889634f / sqrtf((float)MD);       // log2(e) / sqrt(D)
  const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};

  // ---- prologue: K of tile 0; V^T buffer 1 is cleared because the first matrix phase multiplies it by P = 0
  PTile lt;
  tile_at(0, lt);
  load_k(lt, 0);
  for (int x = tid; x < V_TILE / 8; x += 512) reinterpret_cast<uint4*>(ldsV + V_TILE)[x] = make_uint4(0, 0, 0, 0);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();

  // ---- phases.  Global phase ph = 0, 1, 2, ...; every phase ends with a workgroup barrier.  Group A runs X(j)
  // in phase 2j and Y(j) in phase 2j+1; group B runs one phase later.  In every even phase 2j the whole
  // workgroup requests K of tile j+1 and V^T of tile j from global memory (for group A that is the start of
  // X(j), for group B the start of Y(j-1)); the requests are awaited at the end of the following odd phase.
  auto issue_loads = [&](int j) {
    if (j + 1 < n_tiles) { tile_at(j + 1, lt); load_k(lt, (j + 1) & 1); }
    if (j < n_tiles) { tile_at(j, lt); load_v(lt, j & 1); }
  };
  if (grp == 1) {                          // phase 0 of group B: only the loads
    issue_loads(0);
    asm volatile("s_barrier" ::: "memory");
  }
  for (int j = 0; j <= n_tiles; ++j) {
    // ---- X(j): O^T += V_{j-1}^T P_{j-1}^T, then S_j^T = K_j Q^T
    if (grp == 0) issue_loads(j);
    // All 16 V^T fragments are requested from LDS first; while the 16 MFMAs of the second product consume
    // them, the 16 K fragments of the score product are requested, so that the matrix pipe does not wait for
    // LDS between MFMAs.  The fences pin that order.
    {
      const uint16_t* vbase = ldsV + ((j + 1) & 1) * V_TILE;
      const uint16_t* kbase = ldsK + (j & 1) * K_TILE;
      bf16x8 vf[4][4], kf[8][2];
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
#pragma unroll
        for (int db = 0; db < 4; ++db) vf[ks][db] = *reinterpret_cast<const bf16x8*>(vbase + db * 32 * KT + voff[ks]);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
        for (int db = 0; db < 4; ++db)
          oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[ks][db], pf[ks], oacc[db], 0, 0, 0);
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
          for (int kb = 0; kb < 2; ++kb)
            kf[2 * ks + s2][kb] = *reinterpret_cast<const bf16x8*>(kbase + kb * 32 * MD + koff[2 * ks + s2]);
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int e = 0; e < 16; ++e) sacc[kb][e] = 0.f;
#pragma unroll
      for (int s = 0; s < 8; ++s)
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
          sacc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s][kb], qf[s], sacc[kb], 0, 0, 0);
    }
    if (grp == 1) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    asm volatile("s_barrier" ::: "memory");
    if (grp == 1 && j == n_tiles) break;

    // ---- Y(j): online softmax in the log2 domain on S_j -> P_j (Alg. 2 Part A / Part B)
    if (grp == 1) issue_loads(j + 1);
    if (j < n_tiles) {
      PTile ct;
      tile_at(j, ct);
      if (ct.bias != nullptr || ct.nk < KT) {
        // accumulator element e of group kb is key 32kb + 8(e/4) + 4g + e%4
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
          float addv[16];
#pragma unroll
          for (int e = 0; e < 16; ++e) addv[e] = 0.f;
          if (ct.bias) {
#pragma unroll
            for (int e4 = 0; e4 < 4; ++e4) {                              // keys 8*e4 + 4g + 0..3: one 16-byte load
              const float4 bv = *reinterpret_cast<const float4*>(ct.bias + 32 * kb + 8 * e4 + 4 * g);
              addv[4 * e4] = bv.x; addv[4 * e4 + 1] = bv.y; addv[4 * e4 + 2] = bv.z; addv[4 * e4 + 3] = bv.w;
            }
          }
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int key = 32 * kb + 8 * (e >> 2) + 4 * g + (e & 3);
            sacc[kb][e] = key >= ct.nk ? -INFINITY : sacc[kb][e] + addv[e];
          }
        }
      }
      float mx = fmaxf(sacc[0][0], sacc[1][0]);
#pragma unroll
      for (int e = 1; e < 16; ++e) mx = fmaxf(mx, fmaxf(sacc[0][e], sacc[1][e]));
      float tmax = mx * cscale;
      tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
      const bool raise = tmax > m_run + RESCALE_TAU;
      if (__ballot(raise) != 0ull) {                   // rare after the first tiles: rescale the accumulators
        const float m_new = raise ? tmax : m_run;
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        m_run = m_new;
        l_run *= alpha;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int e = 0; e < 16; ++e) oacc[i][e] *= alpha;
      }
      const float neg_m = -m_run;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int e = 0; e < 16; e += 2) {
          const float p0 = __builtin_amdgcn_exp2f(fmaf(sacc[kb][e], cscale, neg_m));
          const float p1 = __builtin_amdgcn_exp2f(fmaf(sacc[kb][e + 1], cscale, neg_m));
          const bf16x2 pp = {(__bf16)p0, (__bf16)p1};
          l_run = __builtin_amdgcn_fdot2_f32_bf16(pp, ones, l_run, false);   // sum of the rounded weights
          pf[kb * 2 + (e >> 3)][e & 7] = pp[0];
          pf[kb * 2 + (e >> 3)][(e & 7) + 1] = pp[1];
        }
    }
    if (grp == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    asm volatile("s_barrier" ::: "memory");
  }

  // ---- normalise and store: element e of channel group db is channel 32db + 8(e/4) + 4g + e%4
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  if (row_ok) {
    const float inv = 1.0f / l_tot;
    uint16_t* op = a.out + tbase + (long long)(q_start + row) * a.geo.stride_t + 4 * g;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int e4 = 0; e4 < 4; ++e4) {
        bf16x2 lo = {(__bf16)(oacc[db][4 * e4] * inv), (__bf16)(oacc[db][4 * e4 + 1] * inv)};
        bf16x2 hi = {(__bf16)(oacc[db][4 * e4 + 2] * inv), (__bf16)(oacc[db][4 * e4 + 3] * inv)};
        uint2 o;
        o.x = *reinterpret_cast<uint32_t*>(&lo);
        o.y = *reinterpret_cast<uint32_t*>(&hi);
        *reinterpret_cast<uint2*>(op + 32 * db + 8 * e4) = o;
      }
  }
}

// Launches the attention kernels of the MFMA path: the ping-pong kernel for dense attention, the exact
// branch and the Taylor branch without exact sets; the 4-wave kernel for Taylor blocks with exact sets.
hipError_t launch_attn_mfma(const Problem& pr, const Workspace& ws, const AttnArgs& a, hipStream_t st) {
  MfmaArgs m;
  m.q = (const uint16_t*)a.q; m.k = (const uint16_t*)a.k; m.out = (uint16_t*)a.out;
  m.vt = ws.vt; m.kcn = ws.kcn; m.vcnt = ws.vcnt; m.biasn = ws.biasn;
  m.blk_start = a.blk_start; m.blk_n = a.blk_n;
  m.kv_list = a.kv_list; m.full_list = a.full_list; m.flat_list = a.flat_list;
  m.exact_mask = a.exact_mask;
  m.geo = a.geo; m.cnt = a.cnt; m.dense = a.dense;
  m.Tn_pad = pr.Tn_pad;
  const bool exact_sets = !a.dense && pr.p.exact_frac > 0.0 && a.exact_mask != nullptr;
  m.taylor_here = exact_sets ? 0 : 1;
  m.taylor_only = 1;
  // slots per (batch, head) of the ping-pong kernel: the largest pair count over the batch
  int slots = 0;
  for (int b = 0; b < pr.p.B; ++b) {
    const BatchCounts& c = pr.cnt.b[b];
    const int s = a.dense ? (c.T + 1) / 2 : (c.n_full + 1) / 2 + (m.taylor_here ? (c.n_flat + 1) / 2 : 0);
    slots = s > slots ? s : slots;
  }
  const bool prof = g_prof_on && g_prof_start && g_prof_stop;
  if (prof) (void)hipEventRecord(g_prof_start, st);
  hipError_t e = hipSuccess;
  if (slots > 0) {
    m.slots = slots;
    m.total = pr.p.B * pr.p.H * slots;
    const int grid = (m.total + 7) / 8 * 8;
    hipLaunchKernelGGL(k_attn_pp, dim3(grid), dim3(512), 0, st, m);
    e = hipGetLastError();
  }
  if (e == hipSuccess && exact_sets) e = launch_attn_mfma4(pr, m, st);
  if (prof) {
    (void)hipEventRecord(g_prof_stop, st);
    g_prof_recorded = 1;
  }
  return e;
}

}  // namespace isa
