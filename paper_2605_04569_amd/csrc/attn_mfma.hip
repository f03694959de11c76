// Pack kernels of the MFMA path, and the 4-wave MFMA attention kernel that runs the Taylor branch when its query
// blocks carry exact sets (exact_frac > 0; Eq. 3 + Eq. 4, Alg. 2 Parts A and B): bf16, D = 128, block = 128 on gfx950
// (wave64, v_mfma_f32_32x32x16_bf16).  Dense attention, the exact branch and the Taylor branch without exact sets
// run in the 8-wave kernel of attn_sp.hip.
//
// One workgroup (4 waves) owns one query block of 128 rows; wave w owns rows 32w .. 32w+31.  Two
// workgroups fit a compute unit (<= 256 VGPRs, 64 KB LDS each).
//
// Scores are computed transposed, S^T = K Q^T (M = keys, N = queries), so that the accumulator layout of
// the MFMA (a lane holds one query column and 16 key rows per 32-key group) is already the B-operand
// layout of the second product O^T = V^T P^T: P never leaves registers, and the row maximum / row sum of
// the online softmax (Alg. 2 Part A) need one cross-lane exchange only.  The A operand of the second
// product wants, per lane, 8 consecutive keys of one channel; V is therefore read from a copy that the
// pack kernel stores transposed per 64-key half block, with key positions permuted to the accumulator's
// key order (bits 2 and 3 of the key index swapped).
//
// The Taylor branch (Sec. 3, Eq. 4; Alg. 2 Part B) runs through the same tile code: its "keys" are the
// block means gathered in kv_list order, its "values" the gathered mean values, and the token count n_j
// enters as an additive ln(n_j) on the scaled logit, which is the same as weighting exp() by n_j.
#include "attn_mfma.h"

namespace isa {

// ------------------------------------------------------------------------------------------
// Pack kernels
// ------------------------------------------------------------------------------------------
// V^T copies: vt[((bh*T_max + j)*2 + half)][d][pos]; keys past n_j are zero.  `vt` is in the key order of the
// 16x16x32 kernel (position p holds key key_of_pos16(p)); `vt4`, written only when given, in that of the 4-wave
// 32x32x16 kernel (position p holds key swap23(p)).  With `vc` the block's mean value (fp32, Alg. 1 Stage 1) is written
// as well: the tile is in LDS anyway, and the block-mean kernel then need not read V a second time.
__global__ __launch_bounds__(256) void k_pack_vt(const uint16_t* __restrict__ v, uint16_t* __restrict__ vt,
                                                 uint16_t* __restrict__ vt4, const int* __restrict__ blk_start,
                                                 const int* __restrict__ blk_n, uint16_t* __restrict__ zero_tile,
                                                 float* __restrict__ vc, int* __restrict__ long_ctr, Geometry g) {
  __shared__ uint16_t tile[128][MD + 2];
  __shared__ float colsum[MD];
  const int j = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  if (j == 0 && h == 0 && b == 0) {                               // the all-zero V^T tile the attention kernel pads with
    for (int x = threadIdx.x; x < MD * KT / 8; x += 256) reinterpret_cast<uint4*>(zero_tile)[x] = make_uint4(0, 0, 0, 0);
    if (threadIdx.x == 0) *long_ctr = 0;                          // the counter a dense launch may take its items from
  }
  const int n = blk_n[b * g.T_max + j];
  if (n == 0) return;
  const int start = blk_start[b * g.T_max + j];
  const long long base = (long long)b * g.stride_b + (long long)h * g.stride_h + (long long)start * g.stride_t;
  for (int x = threadIdx.x; x < 128 * 16; x += 256) {          // 16-byte chunks
    const int r = x >> 4, c = x & 15;
    uint4 val = make_uint4(0, 0, 0, 0);
    if (r < n) val = *reinterpret_cast<const uint4*>(v + base + (long long)r * g.stride_t + c * 8);
    uint32_t* dst = reinterpret_cast<uint32_t*>(&tile[r][c * 8]);
    dst[0] = val.x; dst[1] = val.y; dst[2] = val.z; dst[3] = val.w;
  }
  __syncthreads();
  if (vc) {                                 // rows past n are zero: both halves of the threads add 64 rows of a channel
    const int d = threadIdx.x & (MD - 1), r0 = (threadIdx.x >> 7) * 64;
    float s = 0.f;
#pragma unroll 8
    for (int r = 0; r < 64; ++r) s += __uint_as_float((uint32_t)tile[r0 + r][d] << 16);
    if (r0) colsum[d] = s;
    __syncthreads();
    if (!r0) vc[(((long long)b * g.H + h) * g.T_max + j) * MD + d] = (s + colsum[d]) / (float)n;
  }
  const long long tile_off = (((long long)b * g.H + h) * g.T_max + j) * (2 * MD * KT);
  for (int x = threadIdx.x; x < 2 * MD * 8; x += 256) {         // one 16-byte chunk = 8 key positions of one channel
    const int half = x / (MD * 8), rem = x % (MD * 8);
    const int d = rem >> 3, pc = rem & 7;
    uint16_t e[8];
    uint4 o;
#pragma unroll
    for (int i = 0; i < 8; ++i) e[i] = tile[half * 64 + key_of_pos16(pc * 8 + i)][d];
    o.x = e[0] | ((uint32_t)e[1] << 16); o.y = e[2] | ((uint32_t)e[3] << 16);
    o.z = e[4] | ((uint32_t)e[5] << 16); o.w = e[6] | ((uint32_t)e[7] << 16);
    *reinterpret_cast<uint4*>(vt + tile_off + (half * MD + d) * KT + pc * 8) = o;
    if (vt4) {
#pragma unroll
      for (int i = 0; i < 8; ++i) e[i] = tile[half * 64 + swap23(pc * 8 + i)][d];    // swap23 is an involution
      o.x = e[0] | ((uint32_t)e[1] << 16); o.y = e[2] | ((uint32_t)e[3] << 16);
      o.z = e[4] | ((uint32_t)e[5] << 16); o.w = e[6] | ((uint32_t)e[7] << 16);
      *reinterpret_cast<uint4*>(vt4 + tile_off + (half * MD + d) * KT + pc * 8) = o;
    }
  }
}

hipError_t launch_pack_vt(const Problem& pr, const Workspace& ws, const void* v, float* vc, hipStream_t st) {
  hipLaunchKernelGGL(k_pack_vt, dim3(pr.cnt.T_max, pr.p.H, pr.p.B), dim3(256), 0, st, (const uint16_t*)v, ws.vt,
                     ws.vt4, ws.blk_start, ws.blk_n, ws.zero_tile, vc, ws.taylor_ctr + 1, pr.geo);
  return hipGetLastError();
}

// Mean keys (without exact sets: minus the mean key of block 0) / values gathered in kv_list order, rounded to bf16, in the
// layouts the attention kernel reads:
// kcn[bh][t][d], vcn[bh][t][d]; vcnt[bh][t/64][d][pos] with the list position t%64 = key_of_pos16(pos) (and vcnt4, when given, with
// t%64 = swap23(pos), for the 4-wave kernel); biasn[bh][t] = ln(n_j) sqrt(D), -inf past T_new.
__global__ __launch_bounds__(256) void k_gather_means(const float* __restrict__ kc, const float* __restrict__ vc,
                                                      const int* __restrict__ kv_list, const int* __restrict__ blk_n,
                                                      const int4* __restrict__ btab, uint16_t* __restrict__ kcn,
                                                      uint16_t* __restrict__ kcnb, uint16_t* __restrict__ vcn, uint16_t* __restrict__ vcnt,
                                                      uint16_t* __restrict__ vcnt4,
                                                      float* __restrict__ biasn, int* __restrict__ tflag,
                                                      int4* __restrict__ ktab, int* __restrict__ taylor_ctr, Counts cnt, int H,
                                                      int Tn_pad, int block) {
  __shared__ uint16_t vtile[KT][MD + 2];
  __shared__ int ids[KT];
  __shared__ int plain;                       // every mean key of the tile exists and stands for a full block
  if (threadIdx.x == 0) plain = 1;
  // the attention launch that follows hands out its Taylor groups by counting this up from zero
  if (threadIdx.x == 0 && blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0) *taylor_ctr = 0;
  __syncthreads();
  const int tile = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int T_new = cnt.b[b].T_new, T_max = cnt.T_max;
  const long long bh = (long long)b * H + h;
  const int t0 = tile * KT;
  if (threadIdx.x < KT) {
    const int t = t0 + threadIdx.x;
    const int j = t < T_new ? block_in_range(kv_list[bh * T_max + t], cnt.b[b].T) : -1;
    ids[threadIdx.x] = j;
    if (j >= 0) ktab[bh * T_max + t] = btab[b * T_max + j];
    // ln(n_j) * sqrt(D): added to the raw score q.k, it becomes ln(n_j) after the 1/sqrt(D) scaling.  Without exact sets
    // (no token keys beside the mean keys) a common factor of the weights cancels in the softmax: ln(n_j / block) is
    // stored instead, which is exactly 0 for full blocks, and tiles of nothing but full blocks take the kernel's plain path
    // (the log-sum-exp the forward hands to the backward is then short of ln(block); the backward uses the same terms).
    const int n_j = j >= 0 ? blk_n[b * T_max + j] : 0;
    const float shift = vcnt4 ? 0.f : logf((float)block);
    biasn[bh * Tn_pad + t] = j >= 0 ? (n_j == block && !vcnt4 ? 0.f : (logf((float)n_j) - shift) * sqrtf((float)MD)) : -INFINITY;
    if (j < 0 || n_j != block || vcnt4) plain = 0;          // benign race: every writer stores 0
  }
  __syncthreads();
  for (int x = threadIdx.x; x < KT * MD; x += 256) {
    const int r = x / MD, d = x % MD;
    const int j = ids[r];
    float kval = 0.f, vval = 0.f;
    if (j >= 0) {
      // A vector common to all keys of a softmax changes nothing, so the mean key of block 0 (a source block, always
      // kept) is subtracted before the rounding to bf16: a component common to all keys (an offset of many standard
      // deviations costs 2^-9 of itself per channel otherwise) then does not eat the precision of what distinguishes
      // them.  Without exact sets the mean keys are the only keys of a Taylor row and nothing else is needed.  With exact
      // sets they share a softmax with token keys: the 4-wave kernel and the backward kernels add each query's product
      // with the subtracted vector (q . Kc_0, kept per query row) back onto its mean-key scores; kcnb is the copy without
      // the subtraction, which the backward's dQ multiplies dS with.
      const float kraw = kc[(bh * T_max + j) * MD + d];
      kval = kraw - kc[bh * T_max * MD + d];
      if (kcnb) kcnb[(bh * Tn_pad + t0 + r) * MD + d] = f2bf(kraw);
      vval = vc[(bh * T_max + j) * MD + d];
    }
    kcn[(bh * Tn_pad + t0 + r) * MD + d] = f2bf(kval);
    if (kcnb && j < 0) kcnb[(bh * Tn_pad + t0 + r) * MD + d] = 0;
    if (vcn) vcn[(bh * Tn_pad + t0 + r) * MD + d] = f2bf(vval);       // row-major mean values: the backward pass streams them
    vtile[r][d] = f2bf(vval);
  }
  __syncthreads();
  if (threadIdx.x == 0) tflag[bh * (Tn_pad / KT) + tile] = plain ? 0 : 1;
  const long long out_off = (bh * (Tn_pad / KT) + tile) * (MD * KT);
  for (int x = threadIdx.x; x < MD * KT; x += 256) {
    const int d = x / KT, pos = x % KT;
    vcnt[out_off + d * KT + pos] = vtile[key_of_pos16(pos)][d];
    if (vcnt4) vcnt4[out_off + d * KT + pos] = vtile[swap23(pos)][d];
  }
}

hipError_t launch_gather_means(const Problem& pr, const Workspace& ws, const float* kc, const float* vc,
                               const int* kv_list, hipStream_t st) {
  hipLaunchKernelGGL(k_gather_means, dim3(pr.Tn_pad / KT, pr.p.H, pr.p.B), dim3(256), 0, st, kc, vc, kv_list, ws.blk_n,
                     ws.btab, ws.kcn, ws.kcnb, ws.vcn, ws.vcnt, ws.vcnt4, ws.biasn, ws.tflag, ws.ktab, ws.taylor_ctr, pr.cnt, pr.p.H,
                     pr.Tn_pad, pr.p.block);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Attention kernel
// ------------------------------------------------------------------------------------------
struct Tile {                               // wave-uniform description of one 64-key tile
  const uint16_t* krows;                    // row 0 of the block (token tiles) or of the tile (mean tiles)
  int row0;                                 // first row of the tile relative to krows
  int kstride;                              // elements between key rows
  const uint16_t* vt;                       // 128 x 64 packed V^T
  const float* bias;                        // per-key additive terms on the raw scores (global memory; staged in LDS with the tile), or null
  int nk;                                   // valid keys (0..64); rows past it are masked
  int last_row;                             // last row relative to krows that may be read (>= 0)
  uint32_t mw0, mw1;                        // mean tiles: the exact-mask bits of the tile's 64 list entries (masked out)
};

// One 64-key tile for the 32 query columns of a wave: S^T = K Q^T, online softmax in the log2 domain
// (Alg. 2 Part A / Part B), O^T += V^T P^T.  When `general` (wave-uniform) the per-key bias, the lane's `shift` (its
// query's product with the vector the mean keys are stored short of; 0 for token tiles) and the masks are applied to
// the raw scores first; bias and shift are in units of the raw score, so that both cases share the rest of the code.
__device__ __forceinline__ void tile_body(const uint16_t* __restrict__ kbase, const uint16_t* __restrict__ vbase,
                                          const bf16x8 (&qf)[8], f32x16 (&oacc)[4], float& m_run, float& l_run,
                                          const int (&koff)[8], const int (&voff)[4], float cscale, int g, bool general,
                                          int nk, const float* __restrict__ bias, float shift, uint32_t mw0, uint32_t mw1) {
  f32x16 sacc[2];
#pragma unroll
  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
    for (int e = 0; e < 16; ++e) sacc[kb][e] = 0.f;
  // All 16 K fragments of the tile are requested from LDS up front (64 VGPRs that are free in this phase); the
  // MFMAs then start as the fragments arrive.  The sched_group_barrier sequence pins that order.
  bf16x8 kf[8][2];
#pragma unroll
  for (int s = 0; s < 8; ++s)
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) kf[s][kb] = *reinterpret_cast<const bf16x8*>(kbase + kb * 32 * MD + koff[s]);
#pragma unroll
  for (int s = 0; s < 8; ++s)
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
      sacc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s][kb], qf[s], sacc[kb], 0, 0, 0);
  __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);     // 8 DS reads
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);   // 2 MFMA
    __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);   // 2 DS reads
  }
  __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);     // the remaining MFMAs
  // accumulator element e of group kb is key 32kb + 8(e/4) + 4g + e%4
  if (general) {
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      const uint32_t mw = kb ? mw1 : mw0;
      float addv[16];
#pragma unroll
      for (int e = 0; e < 16; ++e) addv[e] = 0.f;
      if (bias) {
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) {                                  // keys 8*e4 + 4g + 0..3: one 16-byte load
          const float4 bv = *reinterpret_cast<const float4*>(bias + 32 * kb + 8 * e4 + 4 * g);
          addv[4 * e4] = bv.x; addv[4 * e4 + 1] = bv.y; addv[4 * e4 + 2] = bv.z; addv[4 * e4 + 3] = bv.w;
        }
      }
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int key = 32 * kb + 8 * (e >> 2) + 4 * g + (e & 3);
        const bool off = (key >= nk) || ((mw >> (key & 31)) & 1u);
        sacc[kb][e] = off ? -INFINITY : sacc[kb][e] + (addv[e] + shift);
      }
    }
  }
  float mx = fmaxf(sacc[0][0], sacc[1][0]);
#pragma unroll
  for (int e = 1; e < 16; ++e) mx = fmaxf(mx, fmaxf(sacc[0][e], sacc[1][e]));
  float tmax = mx * cscale;
  tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
  const bool raise = tmax > m_run + RESCALE_TAU;
  if (__ballot(raise) != 0ull) {                     // rare after the first tiles: rescale the accumulators
    const float m_new = raise ? tmax : m_run;
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
    m_run = m_new;
    l_run *= alpha;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) oacc[i][e] *= alpha;
  }
  bf16x8 pf[4];
  const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
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
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
    for (int db = 0; db < 4; ++db) {
      const bf16x8 af = *reinterpret_cast<const bf16x8*>(vbase + db * 32 * KT + voff[ks]);
      oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, pf[ks], oacc[db], 0, 0, 0);
    }
  }
}

// `a`, `b`: the 8-byte pieces a lane holds of two neighbouring 8-channel groups of its row (lane g = lane / 32 of the row:
// channels 4 g .. + 3 of each group).  The upper half of `a` changes places with the lower half of `b`; afterwards lane g
// holds the 16 bytes of group g.
__device__ __forceinline__ uint4 halves_of_two_groups(uint2 a, uint2 b) {
  const auto x = __builtin_amdgcn_permlane32_swap(a.x, b.x, false, false);
  const auto y = __builtin_amdgcn_permlane32_swap(a.y, b.y, false, false);
  return make_uint4(x[0], y[0], x[1], y[1]);
}

__global__ __launch_bounds__(256, 2) void k_attn_mfma(MfmaArgs a) {
  __shared__ __attribute__((aligned(1024))) uint16_t lds[2 * K_TILE + 2 * V_TILE + 2 * 512];
  uint16_t* ldsK = lds;                     // [2][K_TILE]
  uint16_t* ldsV = lds + 2 * K_TILE;        // [2][V_TILE]
  float* ldsB = reinterpret_cast<float*>(lds + 2 * K_TILE + 2 * V_TILE);      // [2][256]: per-key additive terms of a mean tile

  // ---- which work item: consecutive logical ids go to the same XCD, so that the workgroups that run
  // together on one XCD (and share its L2) read the same head's keys and values
  const int nwg = gridDim.x;
  const int per_xcd = nwg >> 3;             // grid is a multiple of 8
  const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (logical >= a.total) return;
  const int slot = logical % a.slots;
  const int bhid = logical / a.slots;
  const int h = bhid % a.geo.H, b = bhid / a.geo.H;
  const BatchCounts c = a.cnt.b[b];
  if (slot >= c.T) return;
  const int T_max = a.geo.T_max;
  const long long bh = bhid;

  // only the Taylor slots of the (batch, head): its exact-branch blocks are handled by the 8-wave kernel
  if (slot < c.n_full) return;
  const int n_list = c.T_new;
  const int qi = block_in_range(a.flat_list[bh * T_max + slot - c.n_full], c.T);
  const uint32_t* mrow = (a.exact_mask && c.k_exact > 0)
                             ? a.exact_mask + (bh * T_max + (slot - c.n_full)) * a.cnt.mask_words : nullptr;
  const int* bn = a.blk_n + b * T_max;
  const int* bs = a.blk_start + b * T_max;
  const int n_q = bn[qi];
  const int q_start = bs[qi];
  const long long tbase = (long long)b * a.geo.stride_b + (long long)h * a.geo.stride_h;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // wave-uniform, kept in a scalar register
  const int col = lane & 31, g = lane >> 5;

  // ---- Q fragments: B operand of S^T = K Q^T; lane holds channels 16s + 8g .. +7 of its query row
  const int row = wave * 32 + col;
  const bool row_ok = row < n_q;
  const uint16_t* qp = a.q + tbase + (long long)(q_start + (row_ok ? row : 0)) * a.geo.stride_t + 8 * g;
  bf16x8 qf[8];
#pragma unroll
  for (int s = 0; s < 8; ++s) qf[s] = *reinterpret_cast<const bf16x8*>(qp + 16 * s);

  // The gathered mean keys are stored minus the mean key of block 0 (see k_gather_means): q . Kc_0, in fp32, goes back
  // onto this query's raw scores against mean keys, which share the softmax with the token keys of the exact set.
  float q_ref = 0.f;
  {
    const float* ref = a.kc + bh * T_max * MD + 8 * g;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      const float4 r0 = *reinterpret_cast<const float4*>(ref + 16 * s), r1 = *reinterpret_cast<const float4*>(ref + 16 * s + 4);
      const float rr[8] = {r0.x, r0.y, r0.z, r0.w, r1.x, r1.y, r1.z, r1.w};
#pragma unroll
      for (int e = 0; e < 8; ++e) q_ref = fmaf((float)qf[s][e], rr[e], q_ref);
    }
    q_ref += __shfl_xor(q_ref, 32, 64);
    if (a.rq && row_ok && g == 0) a.rq[bh * a.S_max + q_start + row] = q_ref;      // the backward pass adds it back the same way
  }

  f32x16 oacc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) oacc[i][e] = 0.f;
  float m_run = M_INIT, l_run = 0.f;
  const float cscale = 1.4426950408889634f / sqrtf((float)MD);       // log2(e) / sqrt(D)

  // ---- tile sequence.  Phase A: the token tiles (two 64-key halves) of the list entries in the block's exact set.
  // Phase B: tiles of 64 gathered block means (the entries of the exact set masked out).
  // Nothing in the loop below may wait on a global load: the counter such a wait uses also counts the next tile's loads
  // in flight.  So the block's row of exact-set bits lives in two registers (lane L: words L and 64 + L, handed out with
  // readlane), and the table rows {token offset, tokens, block} of 64 entries of the exact set at a time live in three
  // registers (lane L: entry ebase + L), fetched before the loop and, for exact sets of more than 64 entries, in a
  // branch that consumes its own loads.
  const int4* const tab = a.ktab + bh * T_max;
  uint32_t bits_lo = 0u, bits_hi = 0u;
  if (mrow) {
    if (lane < a.cnt.mask_words) bits_lo = mrow[lane];
    if (lane + 64 < a.cnt.mask_words) bits_hi = mrow[lane + 64];
  }
  auto word_of = [&](int w) __attribute__((always_inline)) -> uint32_t {      // word w of the row, bits past the list cleared
    w = __builtin_amdgcn_readfirstlane(w);
    const uint32_t x = w < 64 ? (uint32_t)__builtin_amdgcn_readlane((int)bits_lo, w)
                              : (uint32_t)__builtin_amdgcn_readlane((int)bits_hi, min(w - 64, 63));
    const int left = n_list - 32 * w;
    return left >= 32 ? x : (left <= 0 ? 0u : x & ((1u << left) - 1u));
  };
  asm volatile("" : "+v"(bits_lo), "+v"(bits_hi));
  const int n_words = (n_list + 31) >> 5;
  int n_exact = 0;                          // entries of the exact set
  if (mrow)
    for (int w = 0; w < n_words; ++w) n_exact += __builtin_popcount(word_of(w));
  int ent_off = 0, ent_n = 0, ent_blk = 0, ebase = 0;
  auto refill = [&](int e0) {               // lane L <- table row of entry e0 + L of the exact set
    int my_e = 0, cnt = 0;
    for (int w = 0; w < n_words && cnt < e0 + 64; ++w) {
      uint32_t x = word_of(w);
      while (x != 0u && cnt < e0 + 64) {
        const int e = 32 * w + __builtin_ctz(x);
        x &= x - 1u;
        if (cnt - e0 == lane) my_e = e;
        ++cnt;
      }
    }
    const int4 r = tab[my_e];
    ent_off = r.x; ent_n = r.y; ent_blk = r.z;
    asm volatile("" : "+v"(ent_off), "+v"(ent_n), "+v"(ent_blk));      // the wait for this load stays here
    ebase = e0;
  };
  if (n_exact > 0) refill(0);
  int ei = 0, it_sub = 0, it_mean = 0;      // next token tile: half it_sub of entry ei; next mean tile
  const int n_mean_tiles = (n_list + KT - 1) / KT;
  auto next_tile = [&](Tile& t) -> bool {
    if (ei < n_exact) {
      if (__builtin_expect(ei - ebase >= 64, 0)) refill(ebase + 64);
      const int l = ei - ebase;
      const int off = __builtin_amdgcn_readlane(ent_off, l), n_j = __builtin_amdgcn_readlane(ent_n, l);
      const int blk = __builtin_amdgcn_readlane(ent_blk, l);
      const int k0 = it_sub * KT;
      t.krows = a.k + tbase + (long long)off * a.geo.stride_t;
      t.row0 = k0;
      t.kstride = (int)a.geo.stride_t;
      t.vt = a.vt + ((bh * T_max + blk) * 2 + it_sub) * (long long)(MD * KT);
      t.bias = nullptr;
      t.nk = max(0, min(KT, n_j - k0));
      t.last_row = max(n_j - 1, 0);
      t.mw0 = t.mw1 = 0u;
      ei += it_sub;
      it_sub ^= 1;
      return true;
    }
    if (it_mean < n_mean_tiles) {
      const long long row0 = bh * a.Tn_pad + (long long)it_mean * KT;
      t.krows = a.kcn + row0 * MD;
      t.row0 = 0;
      t.kstride = MD;
      t.vt = a.vcnt + (bh * (a.Tn_pad / KT) + it_mean) * (long long)(MD * KT);
      t.bias = a.biasn + row0;
      t.nk = min(KT, n_list - it_mean * KT);
      t.last_row = KT - 1;                                          // the gathered arrays are padded to whole tiles
      const int w = 2 * it_mean;
      t.mw0 = mrow ? word_of(w) : 0u;
      t.mw1 = mrow ? word_of(w + 1) : 0u;
      ++it_mean;
      return true;
    }
    return false;
  };

  // ---- global -> LDS, 16 bytes per lane, no staging registers.  One wave instruction fills 1024 contiguous
  // LDS bytes (lane i -> bytes 16i..16i+15), so rows cannot be padded; instead the 16-byte chunk c of a row is
  // stored at chunk position c ^ f(row), applied here on the source side: the lane that fills position pc of
  // row r fetches chunk pc ^ f(r).  K rows are 256 B (f = r & 15), V^T rows are 128 B (f = (r >> 1) & 7); with
  // these the 16-lane groups of a b128 fragment read hit 16 different bank groups.
  // Per-lane constants of the four wave instructions a wave issues per tile and tensor: K row / swizzled chunk
  // offset, and the V^T source offset (bytes).
  int krow[4];
  uint32_t kchunk_b[4], vsrc_b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int ch = (wave * 4 + i) * 64 + lane;
    krow[i] = ch >> 4;
    kchunk_b[i] = (uint32_t)((((ch & 15) ^ ((ch >> 4) & 15)) * 8) * 2);
    const int r = ch >> 3;
    vsrc_b[i] = (uint32_t)((r * KT + (((ch & 7) ^ ((r >> 1) & 7)) * 8)) * 2);
  }
  // The loads are written as inline assembly (16 bytes per lane straight into LDS, wave-uniform base in scalar
  // registers, M0 = LDS address): issued through the compiler's builtin, every later LDS read is preceded by a wait for
  // all such loads in flight (the compiler cannot tell that they fill the other buffer), so that the loads of the next
  // tile would be waited for before the arithmetic of the current one.  Here the only wait is the explicit one at the
  // end of an iteration; the compiler's own waits for its own loads can only wait longer than needed, never shorter.
  auto dma16 = [](const char* sbase, uint32_t voff_bytes, uint32_t lds_addr) __attribute__((always_inline)) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_addr), "v"(voff_bytes), "s"(sbase) : "memory", "m0");
  };
  auto uniform = [](const void* ptr) __attribute__((always_inline)) -> const char* {       // wave-uniform by construction
    const uint64_t u = (uint64_t)(uintptr_t)ptr;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)u), hi = __builtin_amdgcn_readfirstlane((uint32_t)(u >> 32));
    return reinterpret_cast<const char*>((uintptr_t)(((uint64_t)hi << 32) | lo));
  };
  auto lds_addr_of = [](const void* ptr) __attribute__((always_inline)) -> uint32_t {
    return (uint32_t)(size_t)(__attribute__((address_space(3))) const void*)ptr;
  };
  auto load_tile = [&](const Tile& t, int buf) {
    const char* kb = uniform(t.krows);
    const char* vb = uniform(t.vt);
    const uint32_t kstride_b = (uint32_t)__builtin_amdgcn_readfirstlane(t.kstride) * 2u;
    const int row0 = __builtin_amdgcn_readfirstlane(t.row0), last_row = __builtin_amdgcn_readfirstlane(t.last_row);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int wchunk = (wave * 4 + i) * 64;                       // first chunk this wave instruction fills
      // rows past the block's end re-read its last row; the row index is never negative
      const uint32_t koff_b = (uint32_t)max(min(row0 + krow[i], last_row), 0) * kstride_b + kchunk_b[i];
      dma16(kb, koff_b, lds_addr_of(ldsK + buf * K_TILE + wchunk * 8));
      dma16(vb, vsrc_b[i], lds_addr_of(ldsV + buf * V_TILE + wchunk * 8));
    }
    // the 64 additive terms of a tile of gathered means come along into LDS (256 B; lanes 16..63 repeat lanes 0..15)
    if (t.bias != nullptr && wave == 0) dma16(uniform(t.bias), (uint32_t)(lane & 15) * 16u, lds_addr_of(ldsB + buf * 256));
  };

  // per-lane fragment offsets (bf16 elements): K row = col, chunk (2s+g) ^ (col & 15); V^T row = col, chunk (2ks+g) ^ ((col>>1)&7)
  int koff[8], voff[4];
#pragma unroll
  for (int s = 0; s < 8; ++s) koff[s] = col * MD + (((2 * s + g) ^ (col & 15)) * 8);
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) voff[ks] = col * KT + (((2 * ks + g) ^ ((col >> 1) & 7)) * 8);

  Tile cur, nxt, nn;
  bool have = next_tile(cur);
  bool have_next = next_tile(nxt);          // (returns false again once the sequence has ended)
  if (have) load_tile(cur, 0);
  // The Q fragments are consumed here, so that the compiler's waits for them stay out of the loop (inside it they would
  // also wait for the tile loads in flight, which the compiler does not know about).
#pragma unroll
  for (int s = 0; s < 8; ++s) asm volatile("" : "+v"(qf[s]));
  asm volatile("" : "+v"(q_ref));
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  int buf = 0;
  while (have) {
    // the description of the tile after next (register work only, see above), then the loads of the next tile
    const bool have_nn = next_tile(nn);
    if (have_next) load_tile(nxt, buf ^ 1);
    const uint16_t* kbase = ldsK + buf * K_TILE;
    const uint16_t* vbase = ldsV + buf * V_TILE;
    const bool general = cur.bias != nullptr || cur.nk < KT;
    tile_body(kbase, vbase, qf, oacc, m_run, l_run, koff, voff, cscale, g, general, cur.nk,
              cur.bias != nullptr ? ldsB + buf * 256 : nullptr, cur.bias != nullptr ? q_ref : 0.f, cur.mw0, cur.mw1);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    buf ^= 1;
    cur = nxt;
    nxt = nn;
    have = have_next;
    have_next = have_nn;
  }

  // ---- normalise and store: element e of channel group db is channel 32db + 8(e/4) + 4g + e%4
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  if (row_ok) {
    const float inv = 1.0f / l_tot;
    if (a.nlse && g == 0) a.nlse[bh * a.S_max + q_start + row] = -m_run - __log2f(l_tot);
    // coarse residual (Alg. 1 Stage 5): the block's row of O_coarse, the same for all of its tokens
    const float* oc = a.ocoarse ? a.ocoarse + (bh * T_max + qi) * MD + 4 * g : nullptr;
    // The two lanes of a row (g = 0, 1) hold channels 4 g .. + 3 of every group of 8: 8 bytes of bf16 each.  Two groups
    // at a time they exchange halves (the upper half of the wave with the lower half, one swap instruction per
    // register), after which lane g holds all 8 channels of group e4 + g: one 16-byte store per lane, 32 contiguous
    // bytes per row and instruction, half the store instructions.
    uint16_t* op = a.out + tbase + (long long)(q_start + row) * a.geo.stride_t + 8 * g;
    uint16_t* lp = a.olo ? a.olo + (bh * a.S_max + q_start + row) * MD + 8 * g : nullptr;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int e4 = 0; e4 < 4; e4 += 2) {
        uint2 o[2], cut[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const int e = e4 + u;
          float4 r = make_float4(oacc[db][4 * e] * inv, oacc[db][4 * e + 1] * inv, oacc[db][4 * e + 2] * inv, oacc[db][4 * e + 3] * inv);
          if (oc) {
            const float4 c4 = *reinterpret_cast<const float4*>(oc + 32 * db + 8 * e);
            r.x = fmaf(a.gamma, c4.x, r.x); r.y = fmaf(a.gamma, c4.y, r.y);
            r.z = fmaf(a.gamma, c4.z, r.z); r.w = fmaf(a.gamma, c4.w, r.w);
          }
          split_bf16x4(r, o[u], cut[u]);
        }
        *reinterpret_cast<uint4*>(op + 32 * db + 8 * e4) = halves_of_two_groups(o[0], o[1]);
        if (lp) *reinterpret_cast<uint4*>(lp + 32 * db + 8 * e4) = halves_of_two_groups(cut[0], cut[1]);
      }
  }
}

// The 4-wave kernel on the Taylor slots only (used when Taylor blocks carry exact sets).
hipError_t launch_attn_mfma4(const Problem& pr, MfmaArgs m, hipStream_t st) {
  m.slots = pr.cnt.T_max;
  m.total = pr.p.B * pr.p.H * pr.cnt.T_max;
  const int grid = (m.total + 7) / 8 * 8;
  hipLaunchKernelGGL(k_attn_mfma, dim3(grid), dim3(256), 0, st, m);
  return hipGetLastError();
}

}  // namespace isa
