// Software-pipelined MFMA attention kernel for bf16, D = 128, block = 128 on gfx950: dense attention, the
// exact branch of ISA (Alg. 1 Stage 4 / Alg. 2 Part A) and the Taylor branch without exact sets (Eq. 4,
// Alg. 2 Part B).
//
// Shape.  One workgroup of 8 waves owns two query blocks (2 x 128 rows) that walk the same tile sequence, so every
// K / V^T tile is fetched once per 256 query rows; a SIMD holds two waves.  Scores are computed transposed
// (S^T = K Q^T) with v_mfma_f32_16x16x32_bf16 and V is read from a packed, key-permuted V^T copy, so the softmax
// weights go from the score accumulators to the second product (O^T = V^T P^T) without leaving their registers.
//
// Pipeline.  Keys are handled in halves of 32.  Each wave runs one instruction stream of "steps" of two MFMAs (one
// LDS fragment against both 16-query tiles of the wave), each followed by one softmax weight (fma + exp2), and every
// second one by a bf16 conversion; scheduling fences and value pins hold that order.  Three halves are in flight:
// while the score MFMAs of half g run, the weights of half g-1 are computed, and the value MFMAs add half g-2.  The
// value product is therefore a whole 64-key tile behind the score product, and the V^T tile staged in LDS lags the
// K tile by one loop iteration.  One barrier per iteration; three LDS buffers per tensor; tiles arrive by direct
// global->LDS loads issued inside the MFMA stream two (K) and one (V^T) iterations ahead.
//
// What bounds it (measured).  With real operands the 32x32x16 MFMA is limited by power: a stream of nothing but such
// MFMAs runs at 2.4 PFLOP/s on constant operands and 1.8 on random ones, and a kernel built on it held 1.9 GHz; the
// 16x16x32 shape moves fewer accumulator bytes per flop (2.0 PFLOP/s on random operands).  In this kernel the matrix
// pipe of a SIMD is busy two thirds of the cycles and the vector issue port a little over half; the two waves of a
// SIMD wait for each other the rest of the time, and every vector instruction taken out of the loop has shown up in
// the run time, while scalar instructions, waits and barrier latency have not.
#include <type_traits>

#include "attn_mfma.h"

namespace isa {

// Wave-uniform description of one 64-key tile.  Offsets are 32-bit byte offsets from per-head base pointers that do
// not change inside the loop, and the description is computed without branches: it is built once per iteration by
// every wave, in scalar instructions that the wave cannot overlap with its own MFMAs.
struct STile {
  uint32_t k_off;                           // bytes from the head's key base to the first row of the tile
  uint32_t v_off;                           // bytes from the head's V^T base to the 128 x 64 packed V^T of the tile
  int bias_off;                             // elements from the head's bias base (mean tiles only)
  int nk, last_row;                         // real keys; last row that may be read (rows count from k_off)
  bool zero_v;                              // a tile past the end: V^T comes from the all-zero tile
};

typedef short short4v __attribute__((ext_vector_type(4)));
#define ISA_FENCE() __builtin_amdgcn_sched_barrier(0)
constexpr int NBUF = 3;                     // LDS tile buffers: the loads of two tiles are in flight while one is consumed

// 16 bytes per lane from global memory straight into LDS: lane i of the wave writes LDS bytes lds_addr + 16 i.
// Written as inline assembly on purpose.  Issued through the compiler's builtin, every later LDS read is
// preceded by a wait for all such loads in flight (the compiler cannot tell that they fill the *other*
// buffer), which puts the whole memory latency in front of the first MFMA of each iteration.  Here the only
// wait is the explicit one at the top of the loop.  M0 is declared clobbered, so the compiler keeps nothing of its own there.
__device__ __forceinline__ void lds_dma16(const void* sbase, uint32_t voff_bytes, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :: "s"(lds_addr), "v"(voff_bytes), "s"(sbase) : "memory", "m0");
}
__device__ __forceinline__ uint32_t lds_addr_of(const void* p) {
  return (uint32_t)(size_t)(__attribute__((address_space(3))) const void*)p;
}

// Keeps a value (and everything it depends on) on this side of the next scheduling fence: without it the
// compiler sinks work whose result is needed only later (row sums, maxima) out of the MFMA shadow it was placed in.
__device__ __forceinline__ void pin(float& x) { asm volatile("" : "+v"(x)); }
__device__ __forceinline__ void pin(bf16x2& x) {
  uint32_t w = __builtin_bit_cast(uint32_t, x);
  asm volatile("" : "+v"(w));
  x = __builtin_bit_cast(bf16x2, w);
}
__device__ __forceinline__ float max_raw(float a, float b) {        // v_max_f32 without the NaN-quieting prologue
  float r;
  asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}

// Register layout (v_mfma_f32_16x16x32_bf16, S^T = K Q^T and O^T = V^T P^T).  With r = lane % 16 and q = lane / 16:
//   a wave owns 32 query rows = two 16-query tiles qt; lane (r, q) works for queries 16 qt + r;
//   the scores of a 32-key half are four 16x16 tiles t[kt][qt] of 4 registers: element i is key 16 kt + 4 q + i;
//   the weights of query tile qt are one B fragment of 8 bf16: position 4 kt + i of the lane, i.e. k index
//   8 q + 4 kt + i -- the packed V^T copy stores key 16 kt + 4 q + i of a 32-key group at that position, so the
//   weights go from the score accumulators to the second product without moving;
//   the output is sixteen 16x16 tiles oacc[ct][qt]: element i is channel 16 ct + 4 q + i.
struct Scores { f32x4 t[2][2]; };            // [kt][qt]

__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}
// maximum over the four lanes (r, 0..3) that share query r: rows of 16 lanes are exchanged with the two swap
// instructions, which (unlike a shuffle through the LDS crossbar) do not queue behind the LDS fragment reads
__device__ __forceinline__ float max_over_q(float x) {
  const uint32_t u = __float_as_uint(x);
  const auto s16 = __builtin_amdgcn_permlane16_swap(u, u, false, false);   // rows 1,3 of the first <-> rows 0,2 of the second
  const float y = max_raw(__uint_as_float(s16[0]), __uint_as_float(s16[1]));
  const uint32_t v = __float_as_uint(y);
  const auto s32 = __builtin_amdgcn_permlane32_swap(v, v, false, false);   // upper half of the first <-> lower half of the second
  return max_raw(__uint_as_float(s32[0]), __uint_as_float(s32[1]));
}

// `a` and `b` are the 8-byte pieces a lane holds of two neighbouring 16-channel tiles of its row (lane (r, q): channels
// 4 q .. 4 q + 3 of each).  Rows 1, 3 of `a` change places with rows 0, 2 of `b`; afterwards lane q holds, as 16
// consecutive bytes, channels 8 (q / 2) .. + 7 of tile q % 2.
__device__ __forceinline__ uint4 pair_halves(uint2 a, uint2 b) {
  const auto x = __builtin_amdgcn_permlane16_swap(a.x, b.x, false, false);
  const auto y = __builtin_amdgcn_permlane16_swap(a.y, b.y, false, false);
  return make_uint4(x[0], y[0], x[1], y[1]);
}

// One half step g: sixteen steps of two MFMAs each.  Three halves are in flight:
//   score MFMAs (steps 0..7) produce the raw scores of half g in `sout` from the 8 K fragments in `kf` (fragment f =
//   key tile f % 2, channels 32 (f / 2) .., fetched from LDS during the previous half step);
//   the softmax weights of half g-1 are computed from `sin` (raw scores, bias and masks already applied, running maxima
//   already raised): one weight (fma, exp2) per step, one bf16 pair converted every second step, into `pnew`;
//   value MFMAs (steps 8..15) add V^T P^T of half g-2 (`pacc`, finished in the previous half step; V^T unit VU of the
//   staged tile) to the output, and the 4x4x4 MFMAs its row sums.
// exp2 runs at half the vector rate on this chip, so the 16 weights of a half have to be spread over all 16
// steps: bunched behind the score MFMAs they made those steps vector-ALU bound while the value steps had nothing to do.
// `tmax_out[qt]` is the scaled maximum of `sout` over the lane's own 8 keys of its query of tile qt, and `raise_out`
// the ballot of the lanes in which it exceeds the running maximum by more than 2^tau (both valid when `sout` needs no
// bias or mask).  LDS fragments are requested a phase before the MFMAs that consume them: the V^T fragments
// during the score steps, the K fragments of the following half step (32 rows at `kpre`) during the value steps;
// every fragment feeds two MFMAs (both query tiles).  `hook(f)` adds tile set-up and tile loads of a later iteration
// in score step f.
template <int VU, typename Hook>
__device__ __forceinline__ void half_step(const uint16_t* __restrict__ kpre, const uint16_t* __restrict__ vbase,
                                          const bf16x8 (&qf)[2][4], bf16x8 (&kf)[8], const Scores& sin, Scores& sout,
                                          f32x4 (&oacc)[8][2], const float (&neg_m)[2], const float (&thr)[2], f32x4 (&l_run)[2],
                                          float (&tmax_out)[2], unsigned long long& raise_out, const bf16x8 (&pacc)[2],
                                          bf16x8 (&pnew)[2],
                                          const int (&koff)[4], int voff, float cscale, Hook hook
                                          ) {
  const bf16x4 ones4 = {(__bf16)1.0f, (__bf16)1.0f, (__bf16)1.0f, (__bf16)1.0f};
  const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};
  bf16x8 vf[8];
  float pe = 0.f;                            // the even weight of the pair in progress
  float mx[2] = {-INFINITY, -INFINITY};
  // weight t of the half: query tile t / 8, position t % 8 of its fragment = element (t / 4) % 2, t % 4 of `sin`
  auto weight = [&](int t) {
    const int qt = t >> 3, kt = (t >> 2) & 1, i = t & 3;
    const float p = __builtin_amdgcn_exp2f(fmaf(sin.t[kt][qt][i], cscale, neg_m[qt]));
    if (t & 1) {
      bf16x2 pw = {(__bf16)pe, (__bf16)p};
      pin(pw);
      pnew[qt][t & 6] = pw[0];
      pnew[qt][(t & 6) + 1] = pw[1];
    } else {
      pe = p;
      pin(pe);
    }
  };
#pragma unroll
  for (int f = 0; f < 8; ++f) {
    const int kt = f & 1, ks = f >> 1;
    ISA_FENCE();
    vf[f] = *reinterpret_cast<const bf16x8*>(vbase + VU * (V_TILE / 2) + f * 16 * 32 + voff);      // channels 16 f ..
    sout.t[kt][0] = mfma16(kf[f], qf[0][ks], ks == 0 ? zero4 : sout.t[kt][0]);
    sout.t[kt][1] = mfma16(kf[f], qf[1][ks], ks == 0 ? zero4 : sout.t[kt][1]);
    weight(f);
    hook(f);
  }
#pragma unroll
  for (int c = 0; c < 8; ++c) {
    ISA_FENCE();
    kf[c] = *reinterpret_cast<const bf16x8*>(kpre + (c & 1) * 16 * MD + koff[c >> 1]);
    oacc[c][0] = mfma16(vf[c], pacc[0], oacc[c][0]);
    oacc[c][1] = mfma16(vf[c], pacc[1], oacc[c][1]);
    weight(8 + c);
    if (c < 2) {
      // Row sums over the weights as rounded to bf16 (what the value product multiplies), so that the rounding of a
      // dominant weight cancels between numerator and denominator.  A 4x4x4 MFMA with an all-ones A operand adds up
      // the four bf16 values each lane holds in its B operand (D[i][j] = sum_k B[k][j], column j = the lane itself):
      // two of them per weight fragment, 8 matrix-pipe cycles each, instead of 16 unpack-and-add vector instructions.
      const bf16x4 lo = {pacc[c][0], pacc[c][1], pacc[c][2], pacc[c][3]};
      const bf16x4 hi = {pacc[c][4], pacc[c][5], pacc[c][6], pacc[c][7]};
      l_run[c] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(__builtin_bit_cast(short4v, ones4), __builtin_bit_cast(short4v, lo), l_run[c], 0, 0, 0);
      l_run[c] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(__builtin_bit_cast(short4v, ones4), __builtin_bit_cast(short4v, hi), l_run[c], 0, 0, 0);
    }
    if (c < 4) {                               // raw maxima of the new scores (their MFMAs have retired by now)
      const int qt = c >> 1, kt = c & 1;
      mx[qt] = fmaxf(fmaxf(mx[qt], sout.t[kt][qt][0]), sout.t[kt][qt][1]);
      mx[qt] = fmaxf(fmaxf(mx[qt], sout.t[kt][qt][2]), sout.t[kt][qt][3]);
      pin(mx[qt]);
    }
    if (c == 4 || c == 5) {
      mx[c - 4] *= cscale;
      pin(mx[c - 4]);
    }
  }
  // Does any lane see a score that is more than 2^tau above its running maximum?  The lanes that share a query keep
  // identical running maxima, so "some lane of the query exceeds it" is the condition for raising it; the exchange of
  // the maxima between those lanes is left to the (rare) case that the answer is yes.
  raise_out = __ballot(mx[0] > thr[0]) | __ballot(mx[1] > thr[1]);
  ISA_FENCE();
  tmax_out[0] = mx[0];
  tmax_out[1] = mx[1];
}

// Bias / masks of a special half (block means, ragged tails), then the running maxima of the online softmax
// (Alg. 2 Part A).  `tmax` comes in as the lane's scaled maxima of a plain half and `raise` as the ballot of the lanes
// that exceed their running maximum by more than 2^tau; a special half recomputes both here.  Returns whether any
// maximum was raised; `alpha[qt]` is then the factor the accumulators have to be multiplied with -- after the half
// step that follows, because that half step still adds weights that were computed against the old maximum.
__device__ __forceinline__ bool prepare_half(Scores& sc, float (&tmax)[2], unsigned long long raise, bool general,
                                             int nk_half, const float* __restrict__ bias, int q, float cscale,
                                             float (&neg_m)[2], float (&thr)[2], float (&alpha)[2]) {
  if (__builtin_expect(general, 0)) {
    float m2[2] = {-INFINITY, -INFINITY};
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
      float4 bv = make_float4(0.f, 0.f, 0.f, 0.f);
      if (bias) bv = *reinterpret_cast<const float4*>(bias + 16 * kt + 4 * q);      // keys 16 kt + 4 q + 0..3
      const float add[4] = {bv.x, bv.y, bv.z, bv.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const bool past = 16 * kt + 4 * q + i >= nk_half;
#pragma unroll
        for (int qt = 0; qt < 2; ++qt) {
          sc.t[kt][qt][i] = past ? -INFINITY : sc.t[kt][qt][i] + add[i];
          m2[qt] = fmaxf(m2[qt], sc.t[kt][qt][i]);
        }
      }
    }
    tmax[0] = m2[0] * cscale;
    tmax[1] = m2[1] * cscale;
    raise = __ballot(tmax[0] > thr[0]) | __ballot(tmax[1] > thr[1]);
  }
  if (__builtin_expect(raise == 0ull, 1)) return false;                      // the common case after the first tiles
#pragma unroll
  for (int qt = 0; qt < 2; ++qt) {
    const float t = max_over_q(tmax[qt]);               // the query's maximum over all 32 keys of the half
    const float m_new = t > thr[qt] ? t : -neg_m[qt];
    alpha[qt] = __builtin_amdgcn_exp2f(-neg_m[qt] - m_new);
    neg_m[qt] = -m_new;
    thr[qt] = m_new + RESCALE_TAU;
  }
  return true;
}

// The deferred rescale of the accumulators after a half step whose prepare_half raised a maximum.
__device__ __forceinline__ void rescale(const float (&alpha)[2], f32x4 (&l_run)[2], f32x4 (&oacc)[8][2]) {
#pragma unroll
  for (int qt = 0; qt < 2; ++qt) {
    l_run[qt] *= alpha[qt];                               // all four elements hold the same sum
#pragma unroll
    for (int c = 0; c < 8; ++c) oacc[c][qt] *= alpha[qt];
  }
}

// One work item.  `taylor` is a template parameter so that the tile set-up inside the loop carries no selects or
// branches between the two kinds of key sequence (token tiles of kept blocks / tiles of gathered block means).
template <bool taylor>
__device__ __forceinline__ void attn_sp_item(const MfmaArgs& a, uint16_t* lds, const int taken) {
  uint16_t* ldsK = lds;                     // K tile T lives in buffer T % NBUF
  uint16_t* ldsV = lds + NBUF * K_TILE;     // V^T tile T lives in buffer T % NBUF
  uint16_t* ldsQ = lds + NBUF * K_TILE + NBUF * V_TILE;       // 2 x 128 query rows of a Taylor group's next pair

  // ---- which work item.  Workgroup ids go round-robin over the 8 XCDs, so XCD x sees ids x, x + 8, ... in
  // order.  Each XCD owns every 8th (batch, head) (`hpx` of them: batch items of different lengths are spread
  // evenly over the XCDs), and works through their exact-branch pairs (the long items) one head after the other, so
  // that the workgroups that run together on it (and share its L2) read the same head's keys and values.  The Taylor
  // groups (short items) belong to no XCD: the workgroups that come after an XCD's long items take them from one
  // counter (`taken`), so they fill the compute units that the last, incomplete round of long items leaves
  // idle, and the XCDs that get through their long items sooner take more of them.  A launch of nothing but very many
  // long items (dense attention over a long sequence) hands those out from a counter as well (`taken` >= 0, numbered
  // over all (batch, head)s, head after head: the whole chip then works on one head at a time and every XCD streams that
  // head's tiles through its L2 once per round of its workgroups, as before).
  const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
  // The last n_split long items of the XCD (those of its last, incomplete round) run as `parts` sub-items, each over
  // 1/parts of the key sequence, so that the round fills all compute units; a merge kernel combines their partial
  // results afterwards.
  const int n_whole = a.n_long - a.n_split;
  const bool counted = taylor || taken >= 0;                    // the item's number comes from a counter
  const bool split = !counted && j >= n_whole;
  const int item = counted ? taken : split ? n_whole + (j - n_whole) / a.parts : j;
  const int part = split ? (j - n_whole) % a.parts : 0;
  // A Taylor work item is a group of up to `tgroup` consecutive pairs of one head, handled one after the other (all of
  // them read the same sequence of mean tiles); an exact-branch item is one pair.
  const int hl = taylor ? item / a.groups_second : item / a.slots_first;
  int slot = taylor ? (item % a.groups_second) * a.tgroup : item % a.slots_first;   // (first) pair index inside its branch
  const int bhid = counted ? hl : hl * 8 + xcd;                // counted items are numbered over all (batch, head)s
  if ((!counted && hl >= a.hpx) || bhid >= a.geo.B * a.geo.H) return;
  const int h = bhid % a.geo.H, b = bhid / a.geo.H;
  const BatchCounts c = a.cnt.b[b];
  const int T_max = a.geo.T_max;
  const long long bh = bhid;

  // waves 0-3 take the first block of the pair, waves 4-7 the second
  const int n_first_blocks = a.dense ? c.T : c.n_full;
  const int n_second_blocks = (a.dense || !a.taylor_here) ? 0 : c.n_flat;
  if (slot >= (((taylor ? n_second_blocks : n_first_blocks) + 1) >> 1)) return;
  const int n_list = a.dense ? c.T : c.T_new;
  const int* bn = a.blk_n + b * T_max;
  const int* bs = a.blk_start + b * T_max;
  const long long tbase = (long long)b * a.geo.stride_b + (long long)h * a.geo.stride_h;
  const int n_tiles = taylor ? (n_list + KT - 1) / KT : 2 * n_list;
  // tiles [t_begin, t_end) of the sequence are this item's; sub-items cut the list at block boundaries
  const int t_begin = split ? 2 * (int)(((long long)n_list * part) / a.parts) : 0;
  const int t_end = split ? 2 * (int)(((long long)n_list * (part + 1)) / a.parts) : n_tiles;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // 0..7, scalar
  const int grp = wave >> 2, wq = wave & 3;
  const int r16 = lane & 15, q = lane >> 4;
  // this wave's query block; the second group idles (computes on block 0, stores nothing) in the last pair of
  // an odd list
  const int entry = 2 * slot + grp;
  const bool active = entry < (taylor ? n_second_blocks : n_first_blocks);
  int qi = !active ? 0 : a.dense ? entry : block_in_range(taylor ? a.flat_list[bh * T_max + entry] : a.full_list[bh * T_max + entry], c.T);
  int n_q = active ? bn[qi] : 0;
  int q_start = bs[qi];
  // Taylor group: the pairs that follow the first one, and what lane L knows about list entry 2 (slot + 1) + L (block
  // index, rows, first row), handed out with readlane when the group moves on
  const int n_here = taylor ? min(a.tgroup, ((n_second_blocks + 1) >> 1) - slot) : 1;
  int nx_qi = 0, nx_n = 0, nx_start = 0;
  if constexpr (taylor) {
    const int e = 2 * (slot + 1) + lane;
    if (lane < 2 * (n_here - 1) && e < n_second_blocks) {
      nx_qi = block_in_range(a.flat_list[bh * T_max + e], c.T);
      nx_n = bn[nx_qi];
    }
    nx_start = bs[nx_qi];
  }

  // Tile idx of the sequence.  Token tiles come from the table row {token offset, real tokens, block index} of their
  // list entry; idx >= t_end (past the end) gives a fully masked tile over valid memory.
  const int4* tab = a.dense ? a.btab + (long long)b * T_max : a.ktab + bh * T_max;
  // Every workgroup of a head walks the tile sequence from its start: the workgroups that run together on an XCD
  // then stream the same tiles at about the same time and share them in that XCD's L2 (measured: starting them at
  // spread-out points of the sequence multiplies the traffic behind the L2 and is slower).
  // per-head bases of everything a tile description points into (mean tiles read the gathered bf16 means)
  const char* const k_head = taylor ? reinterpret_cast<const char*>(a.kcn + bh * a.Tn_pad * MD)
                                    : reinterpret_cast<const char*>(a.k + tbase);
  const char* const v_head = taylor ? reinterpret_cast<const char*>(a.vcnt + bh * (a.Tn_pad / KT) * (long long)(MD * KT))
                                    : reinterpret_cast<const char*>(a.vt + bh * T_max * 2 * (long long)(MD * KT));
  const float* const bias_head = taylor ? a.biasn + bh * a.Tn_pad : nullptr;
  const uint32_t kstride_b = (uint32_t)(taylor ? MD : (int)a.geo.stride_t) * 2u;
  // The descriptions of 64 token tiles at a time are worked out by the 64 lanes in parallel (lane L: tile cbase + L)
  // from one vector load of table rows, and handed out with readlane: no load other than the tile loads is in
  // flight inside the loop, and the per-iteration scalar work is three readlanes and the clamps at the end.
  uint32_t c_koff = 0, c_voff = 0;
  int c_nk = 0, cbase = 0;
  auto refill = [&](int t0) {
    if constexpr (!taylor) {
      const int idx = min(t0 + lane, n_tiles - 1), sub = idx & 1;
      const int4 ent = tab[idx >> 1];
      const int n_j = ent.y;
      const bool empty = n_j <= sub * KT;                 // second tile of a short block: masked, reads the block's first rows
      c_koff = (uint32_t)(ent.x + (empty ? 0 : sub * KT)) * kstride_b;
      c_voff = ((uint32_t)ent.z * 2u + (uint32_t)sub) * (uint32_t)(MD * KT * 2);
      c_nk = empty ? 0 : min(KT, n_j - sub * KT);
      // consume the values here, so that the wait for this (rare) load sits inside this branch and not at the
      // loop-wide join, where it would also wait for the tile loads that were just issued
      asm volatile("" : "+v"(c_koff), "+v"(c_voff), "+v"(c_nk));
    }
    cbase = t0;
  };
  auto make_tile = [&](int idx, STile& t) {
    const bool past = idx >= t_end;
    idx = past ? t_end - 1 : idx;
    if constexpr (taylor) {
      t.k_off = (uint32_t)idx * (uint32_t)(KT * MD * 2);
      t.v_off = (uint32_t)idx * (uint32_t)(MD * KT * 2);
      t.bias_off = idx * KT;
      t.nk = past ? 0 : min(KT, n_list - idx * KT);
      t.last_row = KT - 1;                                // the gathered mean arrays are padded to whole tiles
    } else {
      const int l = idx - cbase;                          // 0..63 by construction of the refills
      t.k_off = __builtin_amdgcn_readlane(c_koff, l);
      t.v_off = __builtin_amdgcn_readlane(c_voff, l);
      const int nk = __builtin_amdgcn_readlane(c_nk, l);
      t.bias_off = 0;
      t.nk = past ? 0 : nk;
      t.last_row = max(nk - 1, 0);                        // rows are counted from the tile's first row
    }
    t.zero_v = past;
  };
  auto bias_of = [&](const STile& t) -> const float* { return bias_head ? bias_head + t.bias_off : nullptr; };
  auto vt_of = [&](const STile& t) -> const uint16_t* {
    return t.zero_v ? a.zero_tile : reinterpret_cast<const uint16_t*>(v_head + t.v_off);
  };

  // ---- Q fragments: B operand of S^T = K Q^T; lane (r, q) holds channels 32 ks + 8 q .. +7 of query 16 qt + r
  int rowq[2];
  bool row_ok[2];
  bf16x8 qf[2][4];
  // mean tiles only: lane L fetches whether tile L needs its bias and masks (tiles past the 64th are taken to)
  int tile_flag = 1;
  if constexpr (taylor) tile_flag = a.tflag[bh * (a.Tn_pad / KT) + max(min(lane, n_tiles - 1), 0)];
#pragma unroll
  for (int qt = 0; qt < 2; ++qt) {
    rowq[qt] = wq * 32 + 16 * qt + r16;
    row_ok[qt] = rowq[qt] < n_q;
    const uint16_t* qp = a.q + tbase + (long long)(q_start + (row_ok[qt] ? rowq[qt] : 0)) * a.geo.stride_t + 8 * q;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) qf[qt][ks] = *reinterpret_cast<const bf16x8*>(qp + 32 * ks);
  }

  // ---- global -> LDS, 16 bytes per lane, no staging registers.  One wave instruction fills 1024 contiguous
  // LDS bytes (lane i -> bytes 16i..16i+15), so rows cannot be padded; instead the 16-byte chunk c of a row is
  // stored at chunk position c ^ f(row), applied on the source side: the lane that fills position pc of row r
  // fetches chunk pc ^ f(r).  K rows are 256 B (f = r & 15), V^T rows are 128 B (f = (r >> 1) & 7); with these
  // the 16-lane groups of a b128 fragment read hit 16 different bank groups.  A wave issues two such
  // instructions per tile and tensor; instruction i of wave w fills chunks (2w+i)*64 .. +63, i.e. K rows
  // 8w+4i .. +3.
  const int l16 = lane >> 4;
  // Rows past the block's end re-read its last row (they are masked); the row index is never negative.  The row
  // is clamped per lane (three vector instructions per load) rather than per wave, which would need a branch.
  uint32_t kchunk_b[2];
  int krow_l[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    krow_l[i] = 8 * wave + 4 * i + l16;
    kchunk_b[i] = (uint32_t)((((lane & 15) ^ (krow_l[i] & 15)) * 8) * 2);
  }
  auto load_k1 = [&](const STile& t, int buf, int i) {
    const int r = min(krow_l[i], t.last_row);
    lds_dma16(k_head + t.k_off, (uint32_t)r * kstride_b + kchunk_b[i],
              lds_addr_of(ldsK + buf * K_TILE + (wave * 2 + i) * 512));
  };
  auto load_k = [&](const STile& t, int buf) { load_k1(t, buf, 0); load_k1(t, buf, 1); };
  // V^T tile in LDS, unit-major: unit u = key positions 32 u .. 32 u + 31 of the tile; a unit is 128 rows (channels) of
  // 64 B, 16-byte chunk c of row r stored at chunk c ^ ((r >> 1) & 3): with that swizzle the fragment reads of the value
  // product are free of bank conflicts (measured with a probe kernel and the LDS bank-conflict counter; the more
  // obvious c ^ ((r >> 2) & 3) conflicts two-way).  Waves 0-3 fill unit 0 and waves 4-7 unit 1, so the source tile of
  // an instruction is wave-uniform and the per-lane part of the address is one constant: rows 16(2w+i mod 8) +
  // lane/4, chunk (lane & 3) ^ ((lane >> 3) & 3).
  const uint32_t vlane_b = (uint32_t)(((lane >> 2) * KT + (((lane & 3) ^ ((lane >> 3) & 3)) * 8)) * 2);
  auto load_v1 = [&](const uint16_t* vt, int buf, int i) {
    const uint16_t* srcu = vt + (wave < 4 ? 0 : 32);
    const char* sw = reinterpret_cast<const char*>(srcu + (((wave * 2 + i) & 7) * 16) * KT);
    lds_dma16(sw, vlane_b, lds_addr_of(ldsV + buf * V_TILE + (wave * 2 + i) * 512));
  };
  auto load_v = [&](const uint16_t* vt, int buf) { load_v1(vt, buf, 0); load_v1(vt, buf, 1); };
  int pair_in_group = 0;                    // Taylor group: which of its pairs is being worked on
  // Query rows of the group's next pair, global -> LDS: wave w fetches rows 32 w .. 32 w + 31 of the pair's 256 (its own
  // rows; waves 0-3 hold the first block), four rows per instruction, chunk c of row r stored at chunk c ^ (r & 15) like
  // the K tiles.  Rows past the block's end repeat its first row, as in the direct loads above.  `i0`: first of the four
  // instructions issued by this call (eight per wave and pair).
  auto stage_q_rows = [&](int i0) {
    if constexpr (taylor) {
      const int nn = __builtin_amdgcn_readlane(nx_n, 2 * pair_in_group + grp);
      const int ns = __builtin_amdgcn_readlane(nx_start, 2 * pair_in_group + grp);
      const char* src = reinterpret_cast<const char*>(a.q + tbase + (long long)ns * a.geo.stride_t);
      // the per-lane address arithmetic is redone at every call: hoisted out of the loop, its results would have to live
      // in registers the loop does not have (the opaque copy of the lane id is what keeps it here)
      int ln = lane;
      asm volatile("" : "+v"(ln));
#pragma unroll
      for (int i = i0; i < i0 + 4; ++i) {
        const int r = wq * 32 + 4 * i + (ln >> 4);                     // row of the block; its LDS row has the same low bits
        lds_dma16(src, (uint32_t)(r < nn ? r : 0) * (uint32_t)(a.geo.stride_t * 2) + (uint32_t)(((ln & 15) ^ (r & 15)) * 16),
                  lds_addr_of(ldsQ + (wave * 32 + 4 * i) * MD));
      }
    }
  };

  // per-lane fragment offsets (bf16 elements): K row r of a 16-key tile, chunk (4 ks + q) ^ r; V^T unit row r of a
  // 16-channel tile, chunk q ^ ((r >> 1) & 3)
  int koff[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) koff[ks] = r16 * MD + (((4 * ks + q) ^ r16) * 8);
  const int voff = r16 * 32 + ((q ^ ((r16 >> 1) & 3)) * 8);

  f32x4 oacc[8][2];
  Scores s0, s1;
#pragma unroll
  for (int c = 0; c < 8; ++c)
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) oacc[c][qt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int kt = 0; kt < 2; ++kt)
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
      s0.t[kt][qt] = f32x4{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
      s1.t[kt][qt] = f32x4{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
    }
  // running maxima of the online softmax, kept as the two values the loop uses: their negative (the addend of the
  // weights' exponent) and the threshold above which a new score raises them
  float neg_m[2] = {-M_INIT, -M_INIT}, thr[2] = {M_INIT + RESCALE_TAU, M_INIT + RESCALE_TAU};
  float mx0[2] = {-INFINITY, -INFINITY}, mx1[2] = {-INFINITY, -INFINITY};     // scaled row maxima of s0 / s1
  f32x4 l_run[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
  const float cscale = 1.4426950408889634f / sqrtf((float)MD);       // log2(e) / sqrt(D)

  // ---- loop over T = t_begin .. t_end (one extra, fully masked iteration drains the pipeline).  Iteration T:
  //   wait for this wave's loads of K tile T+1 and V^T tile T; barrier (both complete for every wave);
  //   half step 2T:   score MFMAs of half (T,0), weights of half (T-1,1), value MFMAs of half (T-1,0), with the
  //                   set-up and the loads of K tile T+2 and V^T tile T+1 in the shadows of the score MFMAs;
  //   half step 2T+1: score MFMAs of half (T,1), weights of half (T,0), value MFMAs of half (T-1,1); in the shadows of
  //                   its value MFMAs the K fragments of half (T+1,0) are fetched, so that no LDS latency is exposed
  //                   after the next barrier.
  // Three buffers each: K tile T is consumed, T+1 complete and read ahead, T+2 in flight; V^T tile T-1 is consumed, T
  // complete, T+1 in flight.  The buffers that are being filled were last read in iteration T-1, which every wave
  // has left once it is past this iteration's barrier.
  STile tprev, tcur, tnext, tnn;
  refill(t_begin);
  make_tile(t_begin, tcur);
  make_tile(t_begin + 1, tnext);
  tprev = tcur; tprev.nk = 0;
  load_k(tcur, 0);
  load_k(tnext, 1);
  load_v(a.zero_tile, 2);                   // stands in for V^T tile t_begin - 1: multiplied with zero weights, must be finite
  load_v(vt_of(tcur), 0);
  // The Q fragments are consumed here, behind the first tile loads, so that the two latencies overlap: the compiler's
  // own wait for them must not land inside the loop, where it would also wait for the tile loads in flight (which it
  // does not know about).
#pragma unroll
  for (int qt = 0; qt < 2; ++qt)
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) asm volatile("" : "+v"(qf[qt][ks]));
  if constexpr (taylor) asm volatile("" : "+v"(nx_qi), "+v"(nx_n), "+v"(nx_start));      // likewise
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  const unsigned long long gen_mask = taylor ? __ballot(tile_flag != 0) : 0ull;
  auto needs_general = [&](const STile& t) -> bool {
    const int idx = t.bias_off / KT;
    return idx >= 64 || ((gen_mask >> idx) & 1ull) != 0ull;
  };
  __syncthreads();
  bf16x8 kf[8];                           // K fragments of the next 32 rows to be multiplied
#pragma unroll
  for (int f = 0; f < 8; ++f) kf[f] = *reinterpret_cast<const bf16x8*>(ldsK + (f & 1) * 16 * MD + koff[f >> 1]);
  bf16x8 pa[2], pb[2];                    // weight fragments: one is being filled while the other is multiplied
#pragma unroll
  for (int qt = 0; qt < 2; ++qt)
#pragma unroll
    for (int e = 0; e < 8; ++e) { pa[qt][e] = (__bf16)0.f; pb[qt][e] = (__bf16)0.f; }
  float alpha[2] = {1.f, 1.f};
  unsigned long long raise0 = 0ull, raise1 = 0ull;     // ballots that go with mx0 / mx1
  // One iteration; `bcur` = (T - t_begin) % NBUF is the buffer of K tile T, either a compile-time constant (the loop
  // is then unrolled three times and every LDS address is a per-lane constant plus an immediate) or a run-time value.
  // `pending`: what this wave still has in flight that the iteration needs -- 0 nothing, 1 tile loads (wait for
  // everything), 2 tile loads followed by the eight loads that stage the next pair's query rows (loads complete in the
  // order of their issue, so "all but the last eight" is enough: the staged rows are not needed before the pair ends).
  auto iteration = [&](const int T, const auto bcur_c, const int pending, const bool stage_q) {
    const int bcur = bcur_c;
    if (pending == 2) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
    else if (pending == 1) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    const int bnext = bcur == 2 ? 0 : bcur + 1;                     // buffer of tiles T + 1
    const int bnn = bcur == 0 ? 2 : bcur - 1;                       // buffer of tiles T + 2 and T - 1
    const uint16_t* kbase = ldsK + bcur * K_TILE;
    const uint16_t* vbase = ldsV + bnn * V_TILE;                    // V^T tile T - 1
    {   // scores of half (T,0) into s0; weights of half (T-1,1) from s1 into pb; value product of pa = half (T-1,0)
      const int nkh = min(32, max(0, tprev.nk - 32));
      const bool general = (taylor && needs_general(tprev)) || nkh < 32;
      const bool raised = prepare_half(s1, mx1, raise1, general, nkh, taylor ? bias_of(tprev) + 32 : nullptr, q, cscale, neg_m, thr, alpha);
      half_step<0>(kbase + 32 * MD, vbase, qf, kf, s1, s0, oacc, neg_m, thr, l_run, mx0, raise0, pa, pb, koff, voff, cscale, [&](int f) {
        if (f == 0) {
          if constexpr (taylor) {
            // the pairs of a group follow each other without a gap: behind a pair's last tile and its drain tile come
            // the first tiles of the next pair, which are the same mean tiles again
            make_tile(T + 2 > t_end ? T + 1 - t_end : T + 2, tnn);
          } else {
            if (__builtin_expect(min(T + 2, t_end - 1) >= cbase + 64, 0)) refill(cbase + 64);
            make_tile(T + 2, tnn);
          }
        }
        if (f == 2) load_k1(tnn, bnn, 0);
        if (f == 3) load_k1(tnn, bnn, 1);
        if (f == 4) load_v1(vt_of(tnext), bnext, 0);
        if (f == 5) load_v1(vt_of(tnext), bnext, 1);
        if constexpr (taylor) {
          if (f >= 6 && stage_q) {
            stage_q_rows(4 * (f - 6));
          }
        }
      }
      );
      if (__builtin_expect(raised, 0)) rescale(alpha, l_run, oacc);
    }
    {   // scores of half (T,1) into s1; weights of half (T,0) from s0 into pa; value product of pb = half (T-1,1)
      const int nkh = min(32, tcur.nk);
      const bool general = (taylor && needs_general(tcur)) || nkh < 32;
      const bool raised = prepare_half(s0, mx0, raise0, general, nkh, bias_of(tcur), q, cscale, neg_m, thr, alpha);
      half_step<1>(ldsK + bnext * K_TILE, vbase, qf, kf, s0, s1, oacc, neg_m, thr, l_run, mx1, raise1, pb, pa, koff, voff, cscale, [](int) {}
      );
      if (__builtin_expect(raised, 0)) rescale(alpha, l_run, oacc);
    }
    tprev = tcur;
    tcur = tnext;
    tnext = tnn;
  };
  // ---- normalise and store: element i of oacc[ct][qt] is channel 16 ct + 4 q + i of query 16 qt + r
  auto store_rows = [&]() {
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
      float l_tot = l_run[qt][0];
      l_tot += __shfl_xor(l_tot, 16, 64);
      l_tot += __shfl_xor(l_tot, 32, 64);
      if (!row_ok[qt]) continue;
      const int row = rowq[qt];
      if (split) {
        // partial result of a sub-item: unnormalised fp32 outputs and the {maximum, sum} they refer to
        const long long sid = (((long long)xcd * a.n_split + (item - n_whole)) * a.parts + part) * 2 + grp;
        float* op = a.split_o + (sid * 128 + row) * MD + 4 * q;
#pragma unroll
        for (int c = 0; c < 8; ++c)
          *reinterpret_cast<float4*>(op + 16 * c) = make_float4(oacc[c][qt][0], oacc[c][qt][1], oacc[c][qt][2], oacc[c][qt][3]);
        if (q == 0) *reinterpret_cast<float2*>(a.split_ml + (sid * 128 + row) * 2) = make_float2(-neg_m[qt], l_tot);
      } else {
        const float inv = 1.0f / l_tot;
        // the mean keys' biases may be stored short of a common term (see k_gather_means): the log-sum-exp gets it back
        if (a.nlse && q == 0) a.nlse[bh * a.S_max + q_start + row] = neg_m[qt] - __log2f(l_tot) - (taylor ? a.lse_shift : 0.f);
        // coarse residual (Alg. 1 Stage 5): the block's row of O_coarse, the same for all of its tokens
        const float* oc = a.ocoarse ? a.ocoarse + (bh * T_max + qi) * MD + 4 * q : nullptr;
        // A lane holds channels 16 c + 4 q .. + 3 of its row: 8 bytes of bf16.  Two channel tiles at a time, the lanes
        // q = 0, 1 and q = 2, 3 of a row exchange halves (one row-swap instruction per register), after which lane q
        // holds 8 consecutive channels, 16 (c + q % 2) + 8 (q / 2) .. + 7: one 16-byte store per lane, 64 contiguous
        // bytes per row and instruction, half the store instructions.
        const int ch = 16 * (q & 1) + 8 * (q >> 1);
        uint16_t* op = a.out + tbase + (long long)(q_start + row) * a.geo.stride_t + ch;
        uint16_t* lp = a.olo ? a.olo + (bh * a.S_max + q_start + row) * MD + ch : nullptr;
#pragma unroll
        for (int c = 0; c < 8; c += 2) {
          uint2 o[2], cut[2];
#pragma unroll
          for (int u = 0; u < 2; ++u) {
            float4 r = make_float4(oacc[c + u][qt][0] * inv, oacc[c + u][qt][1] * inv, oacc[c + u][qt][2] * inv, oacc[c + u][qt][3] * inv);
            if (oc) {
              const float4 c4 = *reinterpret_cast<const float4*>(oc + 16 * (c + u));
              r.x = fmaf(a.gamma, c4.x, r.x); r.y = fmaf(a.gamma, c4.y, r.y);
              r.z = fmaf(a.gamma, c4.z, r.z); r.w = fmaf(a.gamma, c4.w, r.w);
            }
            split_bf16x4(r, o[u], cut[u]);
          }
          *reinterpret_cast<uint4*>(op + 16 * c) = pair_halves(o[0], o[1]);
          if (lp) *reinterpret_cast<uint4*>(lp + 16 * c) = pair_halves(cut[0], cut[1]);
        }
      }
    }
  };

  if constexpr (taylor) {
    // A handful of iterations per pair: not worth three copies of the loop.  The pairs of the group run through one
    // continuous tile pipeline: pair p takes positions p (t_end + 1) .. p (t_end + 1) + t_end of it, its mean tiles and
    // one drain position whose (masked) tile is consumed while the last real tile's value product is added.  In the drain
    // position the pipeline already holds the next pair's first tiles, so only the accumulators, the running maxima
    // and the Q fragments change between pairs: the next pair's 2 x 128 query rows are fetched into LDS during the
    // current pair's first iteration (each wave fetches, and later reads, exactly its own 32 rows).
    int bcur = 0;
    int pending = 1;
    for (int p = 0;; ++p) {
      const bool more = p + 1 < n_here;
      pair_in_group = p;
      for (int T = 0; T <= t_end; ++T) {
        iteration(T, bcur, pending, more && T == 0);
        pending = (more && T == 0) ? 2 : 1;
        bcur = bcur == 2 ? 0 : bcur + 1;
      }
      // the tile loads of the drain iteration have had that iteration to land: after this wait nothing but the stores
      // below is in flight, and the next iteration does not wait for them
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      store_rows();
      if (!more) break;
      // ---- the next pair of the group
      qi = __builtin_amdgcn_readlane(nx_qi, 2 * p + grp);
      n_q = __builtin_amdgcn_readlane(nx_n, 2 * p + grp);
      q_start = __builtin_amdgcn_readlane(nx_start, 2 * p + grp);
#pragma unroll
      for (int qt = 0; qt < 2; ++qt) {
        row_ok[qt] = rowq[qt] < n_q;
        const uint16_t* qrow = ldsQ + (wave * 32 + 16 * qt + r16) * MD;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          qf[qt][ks] = *reinterpret_cast<const bf16x8*>(qrow + (((4 * ks + q) ^ r16) * 8));
          asm volatile("" : "+v"(qf[qt][ks]));
        }
      }
#pragma unroll
      for (int c = 0; c < 8; ++c)
#pragma unroll
        for (int qt = 0; qt < 2; ++qt) oacc[c][qt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int qt = 0; qt < 2; ++qt) {
        l_run[qt] = f32x4{0.f, 0.f, 0.f, 0.f};
        neg_m[qt] = -M_INIT;
        thr[qt] = M_INIT + RESCALE_TAU;
        alpha[qt] = 1.f;
      }
      pending = 0;
    }
  } else {
    for (int T = t_begin;;) {
      iteration(T, std::integral_constant<int, 0>{}, 1, false);
      if (++T > t_end) break;
      iteration(T, std::integral_constant<int, 1>{}, 1, false);
      if (++T > t_end) break;
      iteration(T, std::integral_constant<int, 2>{}, 1, false);
      if (++T > t_end) break;
    }
    // the loads of the two tiles past the end still target this workgroup's LDS: let them land before the waves end
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    store_rows();
  }
}

__global__ __launch_bounds__(512, 1) void k_attn_sp(MfmaArgs a) {
  // three K tiles, three V^T tiles, and the staged query rows of a Taylor group's next pair: all 160 KB of a compute unit
  __shared__ __attribute__((aligned(1024))) uint16_t lds[NBUF * K_TILE + NBUF * V_TILE + 256 * MD];
  // the workgroups that take the Taylor groups come after all exact-branch items (whole and split) of their XCD
  if ((int)(blockIdx.x >> 3) >= a.n_long - a.n_split + a.n_split * a.parts) {
    // Each of them takes the next group from the counter until none is left: the counter only grows, so every
    // workgroup gets there.  The taken number reaches the other waves through LDS (the staging area of the query rows,
    // which is idle between groups); the second barrier keeps it from being overwritten before everyone has read it,
    // and both together keep the first tile loads of a group behind the last LDS reads of the group before it.
    int* taken = reinterpret_cast<int*>(lds + NBUF * K_TILE + NBUF * V_TILE);
    const int n_groups = a.geo.B * a.geo.H * a.groups_second;
    for (;;) {
      if (threadIdx.x == 0) *taken = atomicAdd(a.taylor_ctr, 1);
      __syncthreads();
      const int g = __builtin_amdgcn_readfirstlane(*taken);
      __syncthreads();
      if (g >= n_groups) break;
      attn_sp_item<true>(a, lds, g);
    }
  } else if (a.long_ctr) {
    // long items from a counter: one per workgroup; the launch has more workgroups than items, the surplus leaves here
    int* slot = reinterpret_cast<int*>(lds + NBUF * K_TILE + NBUF * V_TILE);
    if (threadIdx.x == 0) *slot = atomicAdd(a.long_ctr, 1);
    __syncthreads();
    const int g = __builtin_amdgcn_readfirstlane(*slot);
    if (g >= a.n_long_all) return;
    attn_sp_item<false>(a, lds, g);
  } else {
    attn_sp_item<false>(a, lds, -1);
  }
}

// Combines the partial results of the split work items: out = sum_p O_p 2^(m_p - m) / sum_p l_p 2^(m_p - m) with
// m = max_p m_p (the merge step of the online softmax, Alg. 2 Part A).  One workgroup per (XCD, split item, block of the
// pair, 8 query rows); 32 threads per row, 4 channels each.
__global__ __launch_bounds__(256) void k_split_merge(MfmaArgs a) {
  const int rows8 = blockIdx.x & 15, grp = (blockIdx.x >> 4) & 1;
  const int r = (blockIdx.x >> 5) % a.n_split, xcd = (blockIdx.x >> 5) / a.n_split;
  const int item = a.n_long - a.n_split + r;
  const int hl = item / a.slots_first, slot = item % a.slots_first;
  const int bhid = hl * 8 + xcd;
  if (hl >= a.hpx || bhid >= a.geo.B * a.geo.H) return;
  const int h = bhid % a.geo.H, b = bhid / a.geo.H;
  const BatchCounts c = a.cnt.b[b];
  const int T_max = a.geo.T_max;
  const int n_blocks = a.dense ? c.T : c.n_full;
  const int entry = 2 * slot + grp;
  if (entry >= n_blocks) return;
  const int qi = a.dense ? entry : block_in_range(a.full_list[(long long)bhid * T_max + entry], c.T);
  const int n_q = a.blk_n[b * T_max + qi], q_start = a.blk_start[b * T_max + qi];
  const int row = rows8 * 8 + (threadIdx.x >> 5), ch = (threadIdx.x & 31) * 4;
  if (row >= n_q) return;
  const long long sid0 = (((long long)xcd * a.n_split + r) * a.parts) * 2 + grp;       // part p is at sid0 + 2p
  float m = M_INIT;
  for (int p = 0; p < a.parts; ++p) m = fmaxf(m, a.split_ml[((sid0 + 2 * p) * 128 + row) * 2]);
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  float l = 0.f;
  for (int p = 0; p < a.parts; ++p) {
    const float2 ml = *reinterpret_cast<const float2*>(a.split_ml + ((sid0 + 2 * p) * 128 + row) * 2);
    const float w = __builtin_amdgcn_exp2f(ml.x - m);
    const float4 o = *reinterpret_cast<const float4*>(a.split_o + ((sid0 + 2 * p) * 128 + row) * MD + ch);
    acc.x += w * o.x; acc.y += w * o.y; acc.z += w * o.z; acc.w += w * o.w;
    l += w * ml.y;
  }
  const float inv = 1.0f / l;
  const long long tbase = (long long)b * a.geo.stride_b + (long long)h * a.geo.stride_h;
  if (a.nlse && ch == 0) a.nlse[(long long)bhid * a.S_max + q_start + row] = -m - __log2f(l);
  acc.x *= inv; acc.y *= inv; acc.z *= inv; acc.w *= inv;
  if (a.ocoarse) {                                           // coarse residual, as in the attention kernel's own store
    const float4 c4 = *reinterpret_cast<const float4*>(a.ocoarse + ((long long)bhid * T_max + qi) * MD + ch);
    acc.x = fmaf(a.gamma, c4.x, acc.x); acc.y = fmaf(a.gamma, c4.y, acc.y);
    acc.z = fmaf(a.gamma, c4.z, acc.z); acc.w = fmaf(a.gamma, c4.w, acc.w);
  }
  uint2 o, cut;
  split_bf16x4(acc, o, cut);
  *reinterpret_cast<uint2*>(a.out + tbase + (long long)(q_start + row) * a.geo.stride_t + ch) = o;
  if (a.olo) *reinterpret_cast<uint2*>(a.olo + ((long long)bhid * a.S_max + q_start + row) * MD + ch) = cut;
}

// Pairs of Taylor query blocks per group, the unit a workgroup takes from the counter.  A pair costs its mean tiles plus
// one drain iteration; the set-up of a group (taking its number; list entry -> block table -> query rows -> first tiles,
// three dependent memory latencies), about as long as half the mean tiles of a 480p pair together, is paid once per group.
// Four keeps the groups short enough for the workgroups to run out of them at about the same time.
constexpr int TAYLOR_GROUP = 4;

// Launches the attention kernels of the MFMA path: the software-pipelined kernel for dense attention, the
// exact branch and the Taylor branch without exact sets; the 4-wave kernel for Taylor blocks with exact sets.
hipError_t launch_attn_mfma(const Problem& pr, const Workspace& ws, const AttnArgs& a, hipStream_t st) {
  MfmaArgs m;
  m.q = (const uint16_t*)a.q; m.k = (const uint16_t*)a.k; m.out = (uint16_t*)a.out;
  m.vt = ws.vt; m.kcn = ws.kcn; m.vcnt = ws.vcnt; m.biasn = ws.biasn; m.tflag = ws.tflag;
  m.kc = a.kc;
  m.lse_shift = ws.vcnt4 ? 0.f : log2f((float)pr.p.block);
  m.zero_tile = ws.zero_tile;
  m.blk_start = a.blk_start; m.blk_n = a.blk_n;
  m.btab = ws.btab; m.ktab = ws.ktab;
  m.kv_list = a.kv_list; m.full_list = a.full_list; m.flat_list = a.flat_list;
  m.exact_mask = a.exact_mask;
  m.ocoarse = a.dense ? nullptr : a.ocoarse; m.gamma = a.gamma;
  m.geo = a.geo; m.cnt = a.cnt; m.dense = a.dense;
  m.Tn_pad = pr.Tn_pad;
  m.nlse = a.dense ? nullptr : ws.nlse; m.S_max = pr.S_max;
  m.olo = a.dense ? nullptr : ws.olo;
  m.rq = a.dense ? nullptr : ws.rq;
  const bool exact_sets = !a.dense && pr.p.exact_frac > 0.0 && a.exact_mask != nullptr;
  m.taylor_here = exact_sets ? 0 : 1;
  // pair slots per (batch, head): the largest counts over the batch
  int sf = 0, ss = 0;
  for (int b = 0; b < pr.p.B; ++b) {
    const BatchCounts& c = pr.cnt.b[b];
    const int f = a.dense ? (c.T + 1) / 2 : (c.n_full + 1) / 2;
    const int s2 = (a.dense || !m.taylor_here) ? 0 : (c.n_flat + 1) / 2;
    sf = f > sf ? f : sf;
    ss = s2 > ss ? s2 : ss;
  }
  const bool prof = g_prof_on && g_prof_start && g_prof_stop;
  if (prof) (void)hipEventRecord(g_prof_start, st);
  hipError_t e = hipSuccess;
  if (sf + ss > 0) {
    m.slots_first = sf > 0 ? sf : 1;        // divisors in the kernel; a branch with no work gets no workgroups
    m.slots_second = ss > 0 ? ss : 1;
    m.hpx = (pr.p.B * pr.p.H + 7) / 8;
    m.n_long = m.hpx * sf;
    // An XCD runs one workgroup per compute unit, so its long items go in rounds of `cus`; when the last round is at
    // most half full, its items are cut into as many key ranges as fill it (each at least 8 key blocks long).
    m.n_split = 0; m.parts = 1;
    m.split_o = ws.split_o; m.split_ml = ws.split_ml;
    const int cus = cus_per_xcd(), rem = m.n_long % cus;
    if (rem > 0 && rem <= cus / 2 && rem <= sf && ws.split_o) {
      int min_list = 1 << 30;
      for (int b = 0; b < pr.p.B; ++b) {
        const int nl = a.dense ? pr.cnt.b[b].T : pr.cnt.b[b].T_new;
        min_list = nl < min_list ? nl : min_list;
      }
      int parts = cus / rem;
      if (parts > min_list / 8) parts = min_list / 8;
      while (parts >= 2 && N_XCD * rem * parts > SPLIT_MAX_SUB) --parts;      // the partial-result area holds SPLIT_MAX_SUB sub-items
      if (parts >= 2) { m.n_split = rem; m.parts = parts; }
    }
    // Taylor pairs go in groups of up to TAYLOR_GROUP consecutive pairs of a head per workgroup
    m.tgroup = TAYLOR_GROUP;
    m.groups_second = ss > 0 ? (ss + TAYLOR_GROUP - 1) / TAYLOR_GROUP : 1;
    // one such workgroup per compute unit (they stay until the groups run out), fewer if there are fewer groups
    const long long n_groups = ss > 0 ? (long long)pr.p.B * pr.p.H * m.groups_second : 0;
    m.n_taylor_wg = (int)((n_groups + N_XCD - 1) / N_XCD < cus_per_xcd() ? (n_groups + N_XCD - 1) / N_XCD : cus_per_xcd());
    m.taylor_ctr = ws.taylor_ctr;
    // Dense attention over a long sequence: nothing but long items, 64 rounds of them or more.  The XCDs of a chip differ
    // in speed by several per cent, and with equal shares the launch ends with the slowest; there are no short items to
    // level with, so the long items themselves are taken from a counter (zeroed by the V^T pack, which precedes every
    // such launch), one per workgroup, with an eighth more workgroups than items and one round of the chip to spare.  With
    // fewer rounds the last, ragged round of such a launch would cost what the levelling gains.
    m.long_ctr = nullptr; m.n_long_all = 0;
    if (a.dense && ss == 0 && m.n_long >= 64 * cus) {
      const long long all = (long long)pr.p.B * pr.p.H * sf;
      m.long_ctr = ws.taylor_ctr + 1;
      m.n_long_all = (int)all;
      m.n_split = 0; m.parts = 1;
      m.n_long = (int)((all + all / 8) / N_XCD + cus + 1);      // workgroups per XCD
    }
    const long long per_xcd = (long long)m.n_long - m.n_split + (long long)m.n_split * m.parts + m.n_taylor_wg;
    m.slots = 0; m.total = 0;
    hipLaunchKernelGGL(k_attn_sp, dim3((unsigned)(per_xcd * 8)), dim3(512), 0, st, m);
    e = hipGetLastError();
    if (e == hipSuccess && m.n_split > 0) {
      hipLaunchKernelGGL(k_split_merge, dim3((unsigned)(8 * m.n_split * 32)), dim3(256), 0, st, m);
      e = hipGetLastError();
    }
  }
  if (e == hipSuccess && exact_sets) {
    m.vt = ws.vt4; m.vcnt = ws.vcnt4;               // the 4-wave kernel reads its own key order
    e = launch_attn_mfma4(pr, m, st);
  }
  if (prof) {
    (void)hipEventRecord(g_prof_stop, st);
    g_prof_recorded = 1;
  }
  return e;
}

}  // namespace isa
