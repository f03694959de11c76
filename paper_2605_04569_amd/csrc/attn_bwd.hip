// Backward pass of In-Context Sparse Attention for bf16, D = 128, block = 128 on gfx950 (the paper states that the
// operator is trainable, Sec. 4 "Implementation Detail and Analysis", and gives no formulas: these are the analytic
// gradients of Alg. 1 Stages 4-5 with the index decisions of Stages 2 and 3 held fixed).
//
// With P = softmax weights of a query row (exact branch: over the tokens of the kept blocks; Taylor branch, Eq. 4: over
// the kept blocks' mean keys, each weighted with its token count n_j, and, with exact sets, Alg. 2 Part A, over the
// tokens of the block's exact set instead of their means), delta = rowsum(dO * O) and dP = dO V^T:
//     dS = P * (dP - delta),   dQ = dS K / sqrt(D),   dK = dS^T Q / sqrt(D),   dV = P^T dO,
// and the gradient of a block mean is spread evenly over the block's tokens (dK[t] += dKc[j] / n_j, same for V).
// The coarse residual gamma * O_coarse (Stages 1 and 5) adds the gradient of a small T x T attention over the block
// means (kernels at the end of this file), which enters the big launches through their epilogues.
//
// One kernel does all six products.  A workgroup (8 waves) keeps 2 x 128 "stationary" rows in registers and streams
// 64-row tiles of the other side through LDS; per tile it forms T1 = Y1 X1^T (the scores) and, where dS is needed,
// T2 = Y2 X2^T (dP), turns them into W = P or dS in registers and accumulates acc^T += Yt W^T, where Yt is the
// transpose of a streamed tile: its fragments are read out of the row-major tile in LDS with ds_read_b64_tr_b16, in the
// key order of the 16x16x32 accumulators, so no transposed copy of any tensor exists.  The six launches:
//     dQ, exact branch : stationary (Q, dO) of the full-attention blocks,  streamed K, V of the kept tokens (Yt = K^T)
//     dQ, Taylor branch: stationary (Q, dO) of the Taylor blocks,          streamed Kc, Vc (block means), after the
//                        K, V tiles of the blocks' exact sets
//     dKc, dVc         : stationary (Kc, Vc) / Kc rows,                    streamed Q, dO of the Taylor blocks (Yt = Q^T / dO^T)
//     dK, dV           : stationary (K, V) / K of the kept blocks,         streamed Q, dO of the full-attention
//                        blocks and of the Taylor blocks whose exact set holds the block; the epilogue adds the block's
//                        dKc / n_j (dVc / n_j) and writes bf16
// Every output element is written by exactly one workgroup: no atomics, results are reproducible.
//
// The additive terms of a weight ride in the MFMA accumulators: T1 starts at b_x / c (minus the log-sum-exp of a
// stationary query row, log2 n_j of a stationary mean), T2 at minus delta: of the stationary rows when those are queries,
// of the streamed rows when these are (read from the tile's side array as the C operand of the first T2 MFMA), so that
// a weight costs an fma, an exp2, a multiplication and half a packed conversion.  Matrix and vector instructions issue
// through one port on this chip and a sub-tile's weights take about as long as its MFMAs, so the weights are issued in
// slices between the MFMAs of the following sub-tile, with the LDS fragments requested a step ahead.
#include "attn_mfma.h"

namespace isa {

#define ISA_BWD_FENCE() __builtin_amdgcn_sched_barrier(0)

namespace {

constexpr int STAGE = 2 * K_TILE;                    // bf16 elements of one LDS stage: the Y1 and Y2 tiles
constexpr int SIDE_BYTES = 1024;                      // per stage: 64 exponent terms, then 64 minus-deltas, of the streamed rows (512 B used)

// 16 bytes per lane from global memory straight into LDS (lane i -> LDS bytes lds_addr + 16 i); inline assembly so
// that the only wait for these loads is the explicit one at the top of the loop.
__device__ __forceinline__ void dma16(const void* sbase, uint32_t voff_bytes, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :: "s"(lds_addr), "v"(voff_bytes), "s"(sbase) : "memory", "m0");
}
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
  return (uint32_t)(size_t)(__attribute__((address_space(3))) const void*)p;
}
// A pointer that is wave-uniform by construction, moved to scalar registers explicitly.
__device__ __forceinline__ const char* uniform_ptr(const void* p) {
  const uint64_t u = (uint64_t)(uintptr_t)p;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)u), hi = __builtin_amdgcn_readfirstlane((uint32_t)(u >> 32));
  return reinterpret_cast<const char*>((uintptr_t)(((uint64_t)hi << 32) | lo));
}
typedef short short4v __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) short4v* lds_s4_ptr;
__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

}  // namespace

// One phase of the streamed side of a launch: token tiles of the blocks of a list, or tiles of gathered block means.
struct BwdStream {
  const uint16_t* y1; const uint16_t* y2;     // row-major rows for the scores / for dP; the accumulation product reads
                                              // the transpose of y1 (launches that need dS) or of y2 (the others: dO)
  const uint16_t* y3;                         // EX == 2, mean tiles: rows whose transpose the accumulation product reads instead of
                                              // y1's (the mean keys without the subtraction of Kc_0); null otherwise
  const int4* tab;                            // token tiles: [bh][T_max] {token offset, tokens, block id} per list entry; null: mean tiles
  const float2* ybd;                          // per tile of 64 streamed positions: 64 additive exponent terms (-inf: masked), then 64 minus-deltas
  int kind;                                   // token tiles: list entries = 0 kept blocks, 1 full-attention blocks, 2 Taylor blocks
  int masked;                                 // exact sets (Alg. 2 Part A): 0 none; 1 token tiles of the entries whose bit is set for the
                                              // stationary entry, others skipped; 2 mean tiles, positions whose bit is set are masked;
                                              // 3 (mean rows stationary) entries whose bit is set for the lane's row are masked
};

struct BwdArgs {
  // stationary rows: token tensors (strides of `geo`, blocks taken from `stat_list`) or gathered mean rows [bh][Tn_pad][128]
  const uint16_t* x1; const uint16_t* x2;
  const int* stat_list;                       // [bh][T_max] block ids; unused for mean rows
  const float* bx; const float* dx;           // per stationary row: additive exponent term / delta ([bh][S_max] or [bh][Tn_pad]); null = 0
  // EX == 2 only (stationary Taylor queries; the streamed gathered mean keys are stored minus the mean key of block 0):
  // rx [bh][S_max] = q . Kc_0 of every stationary row in raw score units, added to its scores against mean tiles
  const float* rx;
  BwdStream s[2];
  int n_phases;
  // exact sets: bit matrix [bh][T_max][mask_words] whose row is a stationary entry (token blocks) or a stationary mean row,
  // and whose bit index is a streamed list entry / mean position
  const uint32_t* bits; int mask_words;
  // outputs
  uint16_t* out_bf; float* out_f32;           // token rows (bf16, strides of `geo`) or mean rows (fp32 [bh][Tn_pad][128])
  const float* add_rows;                      // null, or fp32 rows of 128 of which one, divided by the block's tokens, is added to every row:
  int add_by_block;                           //   0: [bh][Tn_pad] indexed by the stationary entry; 1: [bh][T_max] indexed by its block id
  float oscale;
  const int* blk_start; const int* blk_n;
  Geometry geo; Counts cnt;
  int Tn_pad, S_max;
  int stat_kind;                              // token rows: 0 full-attention blocks, 1 Taylor blocks, 2 kept blocks
  int items;                                  // work items (pairs of stationary blocks) per (batch, head) in this launch
  // mean rows only: every item runs as `parts` workgroups, each over its share of the streamed entries, and writes its
  // partial sums to out_f32 + part * part_stride (k_bwd_sum_parts adds them up)
  int parts; long long part_stride;
  // token rows, one phase only: the last tail_items items of every XCD (its last, incomplete round over the compute
  // units) run as tail_parts workgroups each, every one over its share of the streamed entries; they leave their
  // unscaled fp32 sums in tail_scratch [XCD][tail item][part][256 rows][128] and k_bwd_tail_merge writes the rows
  int items_xcd, tail_items, tail_parts;
  float* tail_scratch;
  // token rows: null, or a counter (0 when the launch starts) from which every workgroup takes the number of its item,
  // numbered over all (batch, head)s: the launch then has more workgroups than items, and an XCD that gets through its
  // workgroups sooner takes more of the items (the XCDs of a chip are not equally fast)
  int* dyn_ctr;
};

// SM: stationary rows are block means; T2: W = P * (T2 - delta), else W = P; EX: exact-set bits are in play (1: whole
// tiles are masked or not; 2: also single positions of a tile of gathered means).
// YD: the streamed rows carry deltas of their own (they are queries) and the stationary rows none; otherwise the other
// way round.
template <bool SM, bool T2, int EX, bool YD>
__global__ __launch_bounds__(512, 1) void k_attn_bwd(BwdArgs a) {
  constexpr int STG = EX == 2 ? STAGE + K_TILE : STAGE;      // EX == 2: a third tile per stage (see BwdStream::y3)
  __shared__ __attribute__((aligned(1024))) uint16_t lds[2 * STG + 2 * SIDE_BYTES / 2];
  // Workgroup ids go round-robin over the 8 XCDs: XCD x gets every 8th (batch, head) and works through its items one
  // head after the other, so that the workgroups that run together on an XCD (and share its L2) stream the same rows.
  const int xcd = blockIdx.x & 7, jj = blockIdx.x >> 3;
  int parts = 1, part = 0, item, bhid, tail_slot = -1;
  if (SM) {
    parts = a.parts;
    const int item_all = jj % (a.items * parts);
    bhid = (jj / (a.items * parts)) * 8 + xcd;
    item = item_all / parts;
    part = item_all - item * parts;
  } else {
    if (a.dyn_ctr) {
      __shared__ int taken;
      if (threadIdx.x == 0) taken = atomicAdd(a.dyn_ctr, 1);
      __syncthreads();
      const int idx = __builtin_amdgcn_readfirstlane(taken);
      if (idx >= a.items * a.geo.B * a.geo.H) return;     // the launch has more workgroups than items
      item = idx % a.items;
      bhid = idx / a.items;
    } else {
      const int n_reg = a.items_xcd - a.tail_items;       // items_xcd = items x heads of an XCD; no tail: jj itself
      int idx = jj;
      if (jj >= n_reg) {
        const int u = jj - n_reg;
        tail_slot = u / a.tail_parts;
        part = u - tail_slot * a.tail_parts;
        parts = a.tail_parts;
        idx = n_reg + tail_slot;
      }
      item = idx % a.items;
      bhid = (idx / a.items) * 8 + xcd;
    }
  }
  if (bhid >= a.geo.B * a.geo.H) return;
  const int h = bhid % a.geo.H, b = bhid / a.geo.H;
  const int T_new = a.cnt.b[b].T_new, n_full = a.cnt.b[b].n_full, n_flat = a.cnt.b[b].n_flat;
  const int T_max = a.geo.T_max;
  const long long bh = bhid;
  const int n_stat = SM ? (T_new + 127) / 128 : (a.stat_kind == 0 ? n_full : a.stat_kind == 1 ? n_flat : T_new);
  if (2 * item >= n_stat) return;
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
  int n_x, x_start = 0, x_blk = 0;
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
    const int blk = block_in_range(a.stat_list[bh * T_max + e_use], a.cnt.b[b].T);
    x_blk = blk;
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
  float bxv[2], dxv[2], rxv[2] = {0.f, 0.f};
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
    if (EX == 2) rxv[qt] = (a.rx && row_ok[qt]) ? a.rx[bx_base + rowq[qt]] : 0.f;
  }
  // Exact-set bits of the stationary token blocks: lane L holds word L of the row of this wave's own entry and of the
  // pair's other entry (zeros for an entry that does not exist); handed out with readlane.
  uint32_t bits_own = 0u, bits_other = 0u, bits_own_hi = 0u, bits_other_hi = 0u;     // words L and 64 + L
  if (EX && !SM) {
    const int e_other = 2 * item + (1 - grp);
    if (active && lane < a.mask_words) bits_own = a.bits[(bh * T_max + entry) * a.mask_words + lane];
    if (active && lane + 64 < a.mask_words) bits_own_hi = a.bits[(bh * T_max + entry) * a.mask_words + lane + 64];
    if (e_other < n_stat && lane < a.mask_words) bits_other = a.bits[(bh * T_max + e_other) * a.mask_words + lane];
    if (e_other < n_stat && lane + 64 < a.mask_words) bits_other_hi = a.bits[(bh * T_max + e_other) * a.mask_words + lane + 64];
  }
  const uint32_t bits_any = bits_own | bits_other, bits_any_hi = bits_own_hi | bits_other_hi;
  // word w (0..127) of a bit row held as (lo, hi)
  auto word_of = [&](uint32_t lo, uint32_t hi, int w) __attribute__((always_inline)) -> uint32_t {
    return w < 64 ? (uint32_t)__builtin_amdgcn_readlane((int)lo, w) : (uint32_t)__builtin_amdgcn_readlane((int)hi, min(w - 64, 63));
  };
  // consume the prologue loads here: the waits the compiler places inside the loop must not cover them
#pragma unroll
  for (int qt = 0; qt < 2; ++qt) {
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      asm volatile("" : "+v"(x1f[qt][ks]));
      if (T2) asm volatile("" : "+v"(x2f[qt][ks]));
    }
    asm volatile("" : "+v"(bxv[qt]), "+v"(dxv[qt]));
    if (EX == 2) asm volatile("" : "+v"(rxv[qt]));
  }
  if (EX) asm volatile("" : "+v"(bits_own), "+v"(bits_other), "+v"(bits_own_hi), "+v"(bits_other_hi));

  // ---- tile loads: global -> LDS, 16 bytes per lane, rows XOR-swizzled on the source side (the row-major layout of
  // the forward kernel: tiles of 64 rows x 256 B, chunk c of row r at c ^ (r & 15))
  const int l16 = lane >> 4;
  uint32_t nchunk_b[2];
  int nrow_l[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    nrow_l[i] = 8 * wave + 4 * i + l16;
    nchunk_b[i] = (uint32_t)((((lane & 15) ^ (nrow_l[i] & 15)) * 8) * 2);
  }

  // ---- the sequence of streamed tiles: phase p, tile T of the phase (token tiles: entry T / 2, half T % 2).
  // Everything the loop needs to know about the two phases is copied into plain variables here and selected by value:
  // indexing the kernel argument (or a closure) with a run-time phase number would move it to scratch memory.
  struct Cursor { int p, T; };
  const int n_phases = a.n_phases;
  const int ph_ent0 = a.s[0].kind == 0 ? T_new : a.s[0].kind == 1 ? n_full : n_flat;
  const int ph_ent1 = a.s[1].kind == 0 ? T_new : a.s[1].kind == 1 ? n_full : n_flat;
  const int4* const ph_tab0 = a.s[0].tab;
  const int4* const ph_tab1 = a.s[1].tab;
  const int ent_lo = parts > 1 ? (int)((long long)part * ph_ent0 / parts) : 0;        // this part's share of the entries
  const int ent_hi = parts > 1 ? (int)((long long)(part + 1) * ph_ent0 / parts) : ph_ent0;
  const int ph_tiles0 = ph_tab0 ? 2 * ent_hi : (T_new + KT - 1) / KT;
  const int ph_tiles1 = ph_tab1 ? 2 * ph_ent1 : (T_new + KT - 1) / KT;
  const int ph_masked0 = a.s[0].masked, ph_masked1 = a.s[1].masked;
  const uint16_t* const ph_y1_0 = a.s[0].y1; const uint16_t* const ph_y1_1 = a.s[1].y1;
  const uint16_t* const ph_y2_0 = a.s[0].y2; const uint16_t* const ph_y2_1 = a.s[1].y2;
  const uint16_t* const ph_y3_0 = a.s[0].y3; const uint16_t* const ph_y3_1 = a.s[1].y3;
  const float2* const ph_ybd_0 = a.s[0].ybd; const float2* const ph_ybd_1 = a.s[1].ybd;
#define PH(p, x0, x1) ((p) == 0 ? (x0) : (x1))
  auto tiles_of = [&](int p) __attribute__((always_inline)) -> int { return PH(p, ph_tiles0, ph_tiles1); };
  // first entry >= e0 of the phase whose bit is set for either stationary entry of the pair (n_ent if none)
  auto next_linked = [&](int e0, int n_ent) __attribute__((always_inline)) -> int {
    int w = e0 >> 5;
    if (e0 >= n_ent) return n_ent;
    uint32_t word = word_of(bits_any, bits_any_hi, w) & (~0u << (e0 & 31));
    const int nw = (n_ent + 31) >> 5;
    while (word == 0u && ++w < nw) word = word_of(bits_any, bits_any_hi, w);
    if (word == 0u) return n_ent;
    return min(n_ent, w * 32 + __builtin_ctz(word));
  };
  // normalises a cursor: skips unlinked entries of a masked token phase and moves on to the next phase at the end
  auto settle = [&](Cursor c) __attribute__((always_inline)) -> Cursor {
    while (c.p < n_phases) {
      const int nt = tiles_of(c.p);
      if (EX && !SM && PH(c.p, ph_masked0, ph_masked1) == 1 && (c.T & 1) == 0 && c.T < nt) c.T = 2 * next_linked(c.T >> 1, nt >> 1);
      if (c.T < nt) break;
      c.p += 1;
      c.T = 0;
    }
    return c;
  };
  auto advance = [&](Cursor c) __attribute__((always_inline)) -> Cursor { c.T += 1; return settle(c); };
  // The table row of a tile is fetched one iteration before the tile's loads are issued, so that its latency is not
  // waited for inside the loop.
  auto row_of = [&](Cursor c) __attribute__((always_inline)) -> int4 {
    const int4* const tab = PH(c.p, ph_tab0, ph_tab1);
    if (c.p >= n_phases || !tab) return make_int4(0, 0, 0, 0);
    return tab[bh * T_max + (c.T >> 1)];
  };
  auto issue_tile = [&](Cursor c, int stage, const int4 ent) __attribute__((always_inline)) {
    const bool means = PH(c.p, ph_tab0, ph_tab1) == nullptr;
    const uint16_t* const ph_y1 = PH(c.p, ph_y1_0, ph_y1_1);
    const uint16_t* const ph_y2 = PH(c.p, ph_y2_0, ph_y2_1);
    const float2* const ph_ybd = PH(c.p, ph_ybd_0, ph_ybd_1);
    const int T = c.T;
    uint32_t y_off, bd_off, ystride_b;
    int nk;
    const char *y1_head, *y2_head, *ybd_head;
    if (means) {
      ystride_b = (uint32_t)MD * 2u;
      y1_head = reinterpret_cast<const char*>(ph_y1 + bh * a.Tn_pad * MD);
      y2_head = reinterpret_cast<const char*>(ph_y2 + bh * a.Tn_pad * MD);
      ybd_head = reinterpret_cast<const char*>(ph_ybd + bh * a.Tn_pad);
      y_off = (uint32_t)T * (uint32_t)(KT * MD * 2);
      bd_off = (uint32_t)T * (uint32_t)(KT * 8);
      nk = KT;                                            // the gathered mean arrays are padded to whole tiles
    } else {
      ystride_b = (uint32_t)a.geo.stride_t * 2u;
      y1_head = reinterpret_cast<const char*>(ph_y1 + tbase);
      y2_head = reinterpret_cast<const char*>(ph_y2 + tbase);
      ybd_head = reinterpret_cast<const char*>(ph_ybd + bh * T_max * 128);
      const int sub = T & 1;
      const bool empty = ent.y <= sub * KT;               // second tile of a short block: masked, reads the block's first rows
      y_off = (uint32_t)(ent.x + (empty ? 0 : sub * KT)) * ystride_b;
      bd_off = (uint32_t)((T >> 1) * 128 + sub * KT) * 8u;
      nk = empty ? 1 : min(KT, ent.y - sub * KT);
    }
    // wave-uniform by construction; made scalar explicitly so that the bases of the loads live in scalar registers
    y_off = __builtin_amdgcn_readfirstlane(y_off);
    bd_off = __builtin_amdgcn_readfirstlane(bd_off);
    nk = __builtin_amdgcn_readfirstlane(nk);
    ystride_b = __builtin_amdgcn_readfirstlane(ystride_b);
    const char* const y1_tile = uniform_ptr(y1_head + y_off);
    const char* const y2_tile = uniform_ptr(y2_head + y_off);
    const char* const ybd_tile = uniform_ptr(ybd_head + bd_off);
    uint16_t* sb = lds + stage * STG;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const uint32_t ro = (uint32_t)min(nrow_l[i], nk - 1) * ystride_b + nchunk_b[i];     // rows past the end re-read the last one
      dma16(y1_tile, ro, lds_addr(sb + (wave * 2 + i) * 512));
      dma16(y2_tile, ro, lds_addr(sb + K_TILE + (wave * 2 + i) * 512));
    }
    if (EX == 2 && means) {                                // the mean keys as they are, for the transposed read
      const char* const y3_tile = uniform_ptr(reinterpret_cast<const char*>(PH(c.p, ph_y3_0, ph_y3_1) + bh * a.Tn_pad * MD) + y_off);
#pragma unroll
      for (int i = 0; i < 2; ++i)
        dma16(y3_tile, (uint32_t)nrow_l[i] * ystride_b + nchunk_b[i], lds_addr(sb + 2 * K_TILE + (wave * 2 + i) * 512));
    }
    if (wave == 0)                                         // {bias, delta} of the 64 rows: 512 B, lanes 32..63 repeat lanes 0..31
      dma16(ybd_tile, (uint32_t)(lane & 31) * 16u, lds_addr(lds + 2 * STG + stage * (SIDE_BYTES / 2)));
  };

  // per-lane fragment offsets (bf16 elements), as in the forward kernel
  int koff[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) koff[ks] = r16 * MD + (((4 * ks + q) ^ r16) * 8);
  // Transposed fragments of the accumulation product (A operand: 16 channels x 32 streamed rows) come straight out of
  // a row-major tile with ds_read_b64_tr_b16: in every group of 16 lanes, lane s points at 4 consecutive channels
  // 16 ct + 4 (s & 3) .. of row 4 q + (s >> 2) of a 16-row sub-tile, and lane l receives, for i = 0..3, channel 16 ct + l
  // of row 4 q + i -- the four rows whose weights the lane group holds in elements 4 kt + i of its W fragment.
  const int tr_row = 4 * q + (r16 >> 2);
  int tr_base[2];                              // sub-tile kt: row offset plus the lane's half of a 16-byte chunk
#pragma unroll
  for (int kt = 0; kt < 2; ++kt) tr_base[kt] = (16 * kt + tr_row) * MD + 4 * (r16 & 1);
  int tr_pos[8];                               // channel tile ct: swizzled position of the lane's chunk in its row
#pragma unroll
  for (int ct = 0; ct < 8; ++ct) tr_pos[ct] = ((2 * ct + ((r16 & 3) >> 1)) ^ (tr_row & 15)) * 8;

  f32x4 acc[8][2];
#pragma unroll
  for (int ct = 0; ct < 8; ++ct)
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) acc[ct][qt] = f32x4{0.f, 0.f, 0.f, 0.f};
  const float cscale = 1.4426950408889634f / sqrtf((float)MD);       // log2(e) / sqrt(D)
  f32x4 t1_init[2], t2_init[2];
#pragma unroll
  for (int qt = 0; qt < 2; ++qt) {
    const float b0 = bxv[qt] / cscale;
    t1_init[qt] = f32x4{b0, b0, b0, b0};
    t2_init[qt] = f32x4{-dxv[qt], -dxv[qt], -dxv[qt], -dxv[qt]};
  }

  // cur: tile being multiplied; nxt: tile whose loads are in flight; nn: tile whose table row is being fetched
  Cursor cur = settle(Cursor{0, 2 * ent_lo});
  Cursor nxt = cur.p < n_phases ? advance(cur) : cur;
  int4 ent_nxt = row_of(cur);
  if (cur.p < n_phases) issue_tile(cur, 0, ent_nxt);
  ent_nxt = row_of(nxt);
  uint32_t sm_word[2] = {0u, 0u};             // masked == 3: word (entry / 32) of the bit rows of the lane's two mean rows
  int sm_word_of = -1;
  for (int it = 0; cur.p < n_phases; ++it) {
    // this wave's loads of the current tile have landed; after the barrier everybody's have, and everybody has finished
    // reading the other stage (the previous tile), which the loads of the next tile now overwrite
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    const uint16_t* sb = lds + (it & 1) * STG;
    const float* side = reinterpret_cast<const float*>(lds + 2 * STG + (it & 1) * (SIDE_BYTES / 2));   // 64 terms, 64 minus-deltas
    const bool mean_tile = EX == 2 && PH(cur.p, ph_tab0, ph_tab1) == nullptr;     // wave-uniform
    f32x4 nd[2];                              // YD: minus delta of the streamed rows of the sub-tile whose T steps are next
    auto load_delta = [&](int hh, int kt) {
      if (T2 && YD) nd[kt] = *reinterpret_cast<const f32x4*>(side + 64 + 32 * hh + 16 * kt + 4 * q);
    };
    // LDS fragments are requested PF steps before the MFMAs that read them (a step is 64 or 32 cycles of matrix pipe,
    // an LDS read takes longer than one of them), in PF + 1 rotating register sets
    constexpr int PF = EX == 2 ? 1 : 2, NB = PF + 1;        // (EX == 2: one step ahead, its registers are all spoken for)
    bf16x8 fa[NB], fb[NB];                    // Y1 / Y2 fragments of T steps n .. n + PF
    bf16x8 fc[NB];                            // Yt fragments of C steps
    auto t_load = [&](int n) {                // fragments of T step n (sub-tile n / 4, k-slice n % 4)
      const int s2 = n >> 2, ks2 = n & 3;
      const uint16_t* rowp = sb + (32 * (s2 >> 1) + 16 * (s2 & 1)) * MD + koff[ks2];
      fa[n % NB] = *reinterpret_cast<const bf16x8*>(rowp);
      if (T2) fb[n % NB] = *reinterpret_cast<const bf16x8*>(rowp + K_TILE);
    };
    auto c_load = [&](int n) {                // fragment of C step n (half n / 8, channel tile n % 8)
      // the tile whose transpose is Yt
      const uint16_t* src = sb + (T2 ? ((EX == 2 && mean_tile) ? 2 * K_TILE : 0) : K_TILE) + (n >> 3) * 32 * MD + tr_pos[n & 7];
      const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4_ptr)(src + tr_base[0]));
      const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4_ptr)(src + tr_base[1]));
      fc[n % NB] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };
#pragma unroll
    for (int n = 0; n < PF; ++n) t_load(n);
    load_delta(0, 0);
    // the first fragments are on their way from LDS while the next tile's loads are set up and issued
    if (nxt.p < n_phases) issue_tile(nxt, (it + 1) & 1, ent_nxt);
    const Cursor nn = nxt.p < n_phases ? advance(nxt) : nxt;
    ent_nxt = row_of(nn);
    // exact sets: what of this tile is masked for this wave's stationary rows
    float gm_tile[2] = {0.f, 0.f};            // per stationary 16-row tile of the wave
    uint32_t pos_w0 = 0u, pos_w1 = 0u;        // masked == 2: bits of the tile's 64 positions (set = masked)
    bool dead = false;                        // the whole tile is masked for all stationary rows of this wave
    if (EX) {
      const int masked = PH(cur.p, ph_masked0, ph_masked1);
      if (!SM && masked == 1) {
        const int e = cur.T >> 1;
        const bool linked = (word_of(bits_own, bits_own_hi, e >> 5) >> (e & 31)) & 1u;
        gm_tile[0] = gm_tile[1] = linked ? 0.f : -INFINITY;
        dead = !linked;                       // streamed for the other block of the pair only: every weight would be 0
      } else if (EX == 2 && !SM && masked == 2) {
        pos_w0 = word_of(bits_own, bits_own_hi, 2 * cur.T);
        pos_w1 = word_of(bits_own, bits_own_hi, 2 * cur.T + 1);
      } else if (SM && masked == 3) {
        const int e = cur.T >> 1;
        if ((e >> 5) != sm_word_of) {
          sm_word_of = e >> 5;
#pragma unroll
          for (int qt = 0; qt < 2; ++qt)
            sm_word[qt] = row_ok[qt] ? a.bits[(bh * T_max + entry * 128 + rowq[qt]) * a.mask_words + sm_word_of] : 0u;
        }
#pragma unroll
        for (int qt = 0; qt < 2; ++qt) gm_tile[qt] = ((sm_word[qt] >> (e & 31)) & 1u) ? -INFINITY : 0.f;
      }
    }
    // One tile = two halves (hh) of 32 streamed rows, each of two 16-row sub-tiles (kt).  Per sub-tile: the T products
    // (4 steps of 4 MFMAs, 2 without T2) and then 8 weights per lane on the vector ALU (exp2 runs at half the
    // vector rate, so a sub-tile's weights cost about as much as its MFMAs); per half: the C product (8 steps of 2 MFMAs)
    // once all 16 weights exist.  Back to back these would take turns on the two pipes; instead the weights of a
    // sub-tile are issued in slices between the MFMAs of the next sub-tile's T steps, and those of the last sub-tile
    // between the MFMAs of the first half's C steps:
    //   T(0,0) | T(0,1) + W(0,0) | T(1,0) + W(0,1) | T(1,1) + W(1,0) | C(0) + W(1,1) | C(1)
    if (!(EX && dead)) {                      // wave-uniform
    f32x4 t1[2][2], t2[2][2];                 // [kt][qt]
    bf16x8 w[2][2];                           // [hh][qt]; element 4 kt + i = streamed row 32 hh + 16 kt + 4 q + i
    f32x4 c1[2];
#pragma unroll
    for (int qt = 0; qt < 2; ++qt)
      c1[qt] = EX ? t1_init[qt] + f32x4{gm_tile[qt], gm_tile[qt], gm_tile[qt], gm_tile[qt]} : t1_init[qt];
    if (EX == 2 && mean_tile) {               // the gathered mean keys are stored minus Kc_0: q . Kc_0 goes back onto the scores
#pragma unroll
      for (int qt = 0; qt < 2; ++qt) c1[qt] += f32x4{rxv[qt], rxv[qt], rxv[qt], rxv[qt]};
    }
    f32x4 bt[2];                              // exponent terms of the sub-tile whose weights are in progress, [kt]
    auto load_side = [&](int hh, int kt) {
      const uint32_t pos_w = hh ? pos_w1 : pos_w0;
      bt[kt] = *reinterpret_cast<const f32x4*>(side + 32 * hh + 16 * kt + 4 * q);
      if (EX == 2) {                          // only the launch that streams gathered means under exact sets has such bits
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if ((pos_w >> (16 * kt + 4 * q + i)) & 1u) bt[kt][i] = -INFINITY;
      }
    };
    auto weight2 = [&](int hh, int kt, int tp) {          // weights 2 tp and 2 tp + 1 of sub-tile (hh, kt): tile qt = tp / 2
      const int qt = tp >> 1, i0 = (2 * tp) & 3;
      float val[2];
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const float pw = __builtin_amdgcn_exp2f(fmaf(t1[kt][qt][i0 + j], cscale, bt[kt][i0 + j]));
        val[j] = T2 ? pw * t2[kt][qt][i0 + j] : pw;       // T2 started at minus the deltas: it already is dP - delta
      }
      w[hh][qt][4 * kt + i0] = (__bf16)val[0];
      w[hh][qt][4 * kt + i0 + 1] = (__bf16)val[1];
    };
#pragma unroll
    for (int s = 0; s < 4; ++s) {             // sub-tile (hh, kt) = (s / 2, s % 2)
      const int kt = s & 1;
      if (s > 0) load_side((s - 1) >> 1, (s - 1) & 1);
      if (s < 3) load_delta((s + 1) >> 1, (s + 1) & 1);   // read by the first MFMAs of the next sub-tile
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const int n = 4 * s + ks, cb = n % NB;
        ISA_BWD_FENCE();
        if (n + PF < 16) t_load(n + PF);
        else c_load(n + PF - 16);
        t1[kt][0] = mfma16(fa[cb], x1f[0][ks], ks == 0 ? c1[0] : t1[kt][0]);
        t1[kt][1] = mfma16(fa[cb], x1f[1][ks], ks == 0 ? c1[1] : t1[kt][1]);
        if (T2) {
          t2[kt][0] = mfma16(fb[cb], x2f[0][ks], ks == 0 ? (YD ? nd[kt] : t2_init[0]) : t2[kt][0]);
          t2[kt][1] = mfma16(fb[cb], x2f[1][ks], ks == 0 ? (YD ? nd[kt] : t2_init[1]) : t2[kt][1]);
        }
        if (s > 0) weight2((s - 1) >> 1, (s - 1) & 1, ks);
      }
    }
    load_side(1, 1);
#pragma unroll
    for (int hh = 0; hh < 2; ++hh)
#pragma unroll
      for (int ct = 0; ct < 8; ++ct) {
        const int n = 8 * hh + ct, cb = n % NB;
        ISA_BWD_FENCE();
        if (n + PF < 16) c_load(n + PF);
        acc[ct][0] = mfma16(fc[cb], w[hh][0], acc[ct][0]);
        acc[ct][1] = mfma16(fc[cb], w[hh][1], acc[ct][1]);
        if (hh == 0 && (ct & 1)) weight2(1, 1, ct >> 1);
      }
    }
    ISA_BWD_FENCE();
    cur = nxt;
    nxt = nn;
  }

#undef PH
  if (!SM && tail_slot >= 0) {                // a part of a tail item: unscaled sums to scratch, the merge kernel does the rest
    float* dst = a.tail_scratch + ((((long long)xcd * a.tail_items + tail_slot) * parts + part) * 256 + grp * 128) * MD;
#pragma unroll
    for (int qt = 0; qt < 2; ++qt)
#pragma unroll
      for (int ct = 0; ct < 8; ++ct)
        *reinterpret_cast<f32x4*>(dst + rowq[qt] * MD + 16 * ct + 4 * q) = acc[ct][qt];
    return;
  }
  // ---- store: element i of acc[ct][qt] is channel 16 ct + 4 q + i of stationary row 16 qt + r
  const float inv_n = n_x > 0 ? 1.0f / (float)n_x : 0.f;
  const float* addp = !a.add_rows ? nullptr
                      : a.add_by_block ? a.add_rows + (bh * T_max + x_blk) * MD + 4 * q
                                       : a.add_rows + (bh * a.Tn_pad + e_use) * MD + 4 * q;
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
        *reinterpret_cast<float4*>(a.out_f32 + part * a.part_stride + (bh * a.Tn_pad + (long long)entry * 128 + row) * MD + 16 * ct + 4 * q) = r;
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

// delta[bh][token] = sum_d dO * O (fp32); 16 lanes per token row, 16 bytes per lane and tensor.  O is taken as out + olo:
// the bf16 output plus what its rounding cut off, which the forward kernels keep for this purpose.  With the bf16 output
// alone, delta carries that rounding (2^-9 |dO||O|) into dS = P (dP - delta), which for a query that attends almost
// one-hot is a difference of nearly equal numbers.
__global__ __launch_bounds__(256) void k_bwd_delta(const uint16_t* __restrict__ o, const uint16_t* __restrict__ olo,
                                                   const uint16_t* __restrict__ d_o, float* __restrict__ delta, int* __restrict__ ctr,
                                                   Geometry g, Counts cnt, int S_max) {
  const int h = blockIdx.y, b = blockIdx.z;
  // the item counters of the launches that follow start at zero (ordinary stores: the call can be captured in a graph)
  if (blockIdx.x == 0 && h == 0 && b == 0 && threadIdx.x < 8) ctr[threadIdx.x] = 0;
  const int t = blockIdx.x * 16 + (threadIdx.x >> 4), c16 = threadIdx.x & 15;
  const bool ok = t < cnt.b[b].S;
  float s = 0.f;
  if (ok) {
    const long long off = (long long)b * g.stride_b + (long long)h * g.stride_h + (long long)t * g.stride_t + 8 * c16;
    const uint4 uo = *reinterpret_cast<const uint4*>(o + off), ud = *reinterpret_cast<const uint4*>(d_o + off);
    uint4 ul = make_uint4(0u, 0u, 0u, 0u);
    if (olo) ul = *reinterpret_cast<const uint4*>(olo + (((long long)b * g.H + h) * S_max + t) * MD + 8 * c16);
    const uint32_t wo[4] = {uo.x, uo.y, uo.z, uo.w}, wd[4] = {ud.x, ud.y, ud.z, ud.w}, wl[4] = {ul.x, ul.y, ul.z, ul.w};
#pragma unroll
    for (int i = 0; i < 4; ++i)
      s += (__uint_as_float(wo[i] << 16) + __uint_as_float(wl[i] << 16)) * __uint_as_float(wd[i] << 16) +
           (__uint_as_float(wo[i] & 0xffff0000u) + __uint_as_float(wl[i] & 0xffff0000u)) * __uint_as_float(wd[i] & 0xffff0000u);
  }
#pragma unroll
  for (int m = 8; m >= 1; m >>= 1) s += __shfl_xor(s, m, 64);
  if (ok && c16 == 0) delta[((long long)b * g.H + h) * S_max + t] = s;
}

// Per list entry: the table row of its block and the {exponent term, minus delta} pair of each of its 128 row positions
// (masked positions: -inf, 0), stored per tile of 64 positions as 64 terms followed by 64 minus-deltas.  kind 0: kept blocks as streamed keys (term 0), plus the per-mean arrays of the Taylor
// branch (log2 n_j per gathered mean, -inf for the padding); kinds 1, 2: full-attention / Taylor blocks as streamed
// queries (term = minus the row's log-sum-exp in the log2 domain, delta of the row); with `rq` (Taylor blocks under exact
// sets, for scores against the gathered means, which are stored minus Kc_0) the row's q . Kc_0, scaled to the log2
// domain, is added to the term.
__global__ __launch_bounds__(128) void k_bwd_rows(const int* __restrict__ list, int kind, const int4* __restrict__ btab,
                                                  const float* __restrict__ nlse, const float* __restrict__ rq, float rq_scale,
                                                  const float* __restrict__ delta,
                                                  int4* __restrict__ tab, float2* __restrict__ ybd,
                                                  float2* __restrict__ ybd_mean, float* __restrict__ bx_mean, Counts cnt,
                                                  int H, int Tn_pad, int S_max) {
  const int e = blockIdx.x, h = blockIdx.y, b = blockIdx.z, r = threadIdx.x;
  const int T_max = cnt.T_max;
  const long long bh = (long long)b * H + h;
  const int n_list = kind == 0 ? cnt.b[b].T_new : kind == 1 ? cnt.b[b].n_full : cnt.b[b].n_flat;      // kinds 2, 3: Taylor blocks
  if (kind == 0 && e < Tn_pad && r == 0) {
    float l2 = -INFINITY;
    if (e < n_list) l2 = log2f((float)btab[b * T_max + block_in_range(list[bh * T_max + e], cnt.b[b].T)].y);
    const long long m = bh * Tn_pad + e;                      // planar per 64 positions: 64 terms, then 64 deltas
    float* ym = reinterpret_cast<float*>(ybd_mean);
    ym[(m >> 6) * 128 + (m & 63)] = l2;
    ym[(m >> 6) * 128 + 64 + (m & 63)] = 0.f;
    bx_mean[bh * Tn_pad + e] = e < n_list ? l2 : 0.f;
  }
  if (e >= n_list || e >= T_max) return;
  const int4 ent = btab[b * T_max + block_in_range(list[bh * T_max + e], cnt.b[b].T)];
  if (r == 0) tab[bh * T_max + e] = ent;
  float2 v = make_float2(-INFINITY, 0.f);
  if (r < ent.y) {
    if (kind == 0) v = make_float2(0.f, 0.f);
    else v = make_float2(nlse[bh * S_max + ent.x + r] + (rq ? rq_scale * rq[bh * S_max + ent.x + r] : 0.f),
                         -delta[bh * S_max + ent.x + r]);
  }
  const long long pos = (bh * T_max + e) * 128 + r;
  float* yf = reinterpret_cast<float*>(ybd);
  yf[(pos >> 6) * 128 + (pos & 63)] = v.x;
  yf[(pos >> 6) * 128 + 64 + (pos & 63)] = v.y;
}

// Rows of a token tensor that no later launch writes (keys and values of context blocks that were not kept): zero, or,
// with the coarse residual, the block's share `rows[block] / n` of the gradient of its mean.  Written for every block;
// the launches over the kept blocks overwrite theirs.
__global__ __launch_bounds__(256) void k_bwd_fill(uint16_t* __restrict__ x, const float* __restrict__ rows,
                                                  const int4* __restrict__ btab, Geometry g, Counts cnt) {
  const int blk = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  if (blk >= cnt.b[b].T) return;
  const int4 ent = btab[b * cnt.T_max + blk];
  const int c16 = threadIdx.x & 15;
  uint4 val = make_uint4(0, 0, 0, 0);
  if (rows) {
    const float inv = 1.0f / (float)ent.y;
    const float* rp = rows + (((long long)b * g.H + h) * cnt.T_max + blk) * MD + 8 * c16;
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = f2bf(rp[2 * i] * inv) | ((uint32_t)f2bf(rp[2 * i + 1] * inv) << 16);
    val = make_uint4(w[0], w[1], w[2], w[3]);
  }
  for (int r = threadIdx.x >> 4; r < ent.y; r += 16)
    *reinterpret_cast<uint4*>(x + (long long)b * g.stride_b + (long long)h * g.stride_h + (long long)(ent.x + r) * g.stride_t + 8 * c16) = val;
}

// ---- coarse residual (Alg. 1 Stage 1 and Stage 5): out += gamma * O_coarse[block], O_coarse = softmax(Qc Kc^T / sqrt D) Vc.
// Its gradient: dOc[i] = gamma * (sum of dO over block i); dVc = S^T dOc; dS = dOc Vc^T; dZ = S * (dS - rowsum(dS * S));
// dQc = dZ Kc / sqrt D; dKc = dZ^T Qc / sqrt D; each mean's gradient is spread evenly over its block's tokens.

// One workgroup per (block, head): doc[block] = gamma * column sums of the block's dO rows, and the residual's share is
// taken out of delta (the attention branches' delta is rowsum(dO * (out - gamma * O_coarse[block]))).
__global__ __launch_bounds__(128) void k_bwd_docoarse(const uint16_t* __restrict__ d_o, const float* __restrict__ ocoarse,
                                                      float gamma, float* __restrict__ delta, float* __restrict__ doc,
                                                      const int4* __restrict__ btab, Geometry g, Counts cnt, int S_max) {
  __shared__ uint16_t tile[128][MD + 2];
  __shared__ float oc[MD];
  const int blk = blockIdx.x, h = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
  if (blk >= cnt.b[b].T) return;
  const int4 ent = btab[b * cnt.T_max + blk];
  const long long bh = (long long)b * g.H + h;
  const long long base = (long long)b * g.stride_b + (long long)h * g.stride_h + (long long)ent.x * g.stride_t;
  oc[tid] = ocoarse[(bh * cnt.T_max + blk) * MD + tid];
  for (int x = tid; x < 128 * 16; x += 128) {
    const int r = x >> 4, c = x & 15;
    uint4 val = make_uint4(0, 0, 0, 0);
    if (r < ent.y) val = *reinterpret_cast<const uint4*>(d_o + base + (long long)r * g.stride_t + c * 8);
    uint32_t* dst = reinterpret_cast<uint32_t*>(&tile[r][c * 8]);
    dst[0] = val.x; dst[1] = val.y; dst[2] = val.z; dst[3] = val.w;
  }
  __syncthreads();
  float sum = 0.f;
  for (int r = 0; r < ent.y; ++r) sum += __uint_as_float((uint32_t)tile[r][tid] << 16);
  doc[(bh * cnt.T_max + blk) * MD + tid] = gamma * sum;
  if (tid < ent.y) {
    float dot = 0.f;
    for (int d = 0; d < MD; ++d) dot += __uint_as_float((uint32_t)tile[tid][d] << 16) * oc[d];
    delta[bh * S_max + ent.x + tid] -= gamma * dot;
  }
}

// Row i of the pooled map: softmax statistics {max, sum, rowsum(dS * S)} and dQc[i].  LDS: qc_i, doc_i, T values.
__global__ __launch_bounds__(256) void k_bwd_coarse_rows(const float* __restrict__ qc, const float* __restrict__ kc,
                                                         const float* __restrict__ vc, const float* __restrict__ doc,
                                                         float4* __restrict__ stats, float* __restrict__ dqc, Counts cnt,
                                                         int H) {
  extern __shared__ float sm[];
  float* qi = sm; float* di = sm + MD; float* val = sm + 2 * MD;        // val[T]
  __shared__ float red[256];
  const int i = blockIdx.x, h = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
  const int T = cnt.b[b].T, T_max = cnt.T_max;
  if (i >= T) return;
  const long long row0 = ((long long)b * H + h) * T_max;
  const float scale = 1.0f / sqrtf((float)MD);
  if (tid < MD) { qi[tid] = qc[(row0 + i) * MD + tid]; di[tid] = doc[(row0 + i) * MD + tid]; }
  __syncthreads();
  auto reduce = [&](float x, bool take_max) -> float {
    red[tid] = x;
    __syncthreads();
    for (int s2 = 128; s2 > 0; s2 >>= 1) {
      if (tid < s2) red[tid] = take_max ? fmaxf(red[tid], red[tid + s2]) : red[tid] + red[tid + s2];
      __syncthreads();
    }
    const float r = red[0];
    __syncthreads();
    return r;
  };
  float mloc = -INFINITY;
  for (int j = tid; j < T; j += 256) {
    const float4* kp = reinterpret_cast<const float4*>(kc + (row0 + j) * MD);
    float z = 0.f;
    for (int d4 = 0; d4 < MD / 4; ++d4) {
      const float4 k4 = kp[d4];
      z += qi[4 * d4] * k4.x + qi[4 * d4 + 1] * k4.y + qi[4 * d4 + 2] * k4.z + qi[4 * d4 + 3] * k4.w;
    }
    val[j] = z * scale;
    mloc = fmaxf(mloc, z * scale);
  }
  const float m = reduce(mloc, true);
  float lloc = 0.f;
  for (int j = tid; j < T; j += 256) lloc += __expf(val[j] - m);
  const float l = reduce(lloc, false);
  float rloc = 0.f;
  for (int j = tid; j < T; j += 256) {                  // val[j] <- dZ_ij needs rowdot first: keep S in val, dS in registers twice
    const float4* vp = reinterpret_cast<const float4*>(vc + (row0 + j) * MD);
    float ds = 0.f;
    for (int d4 = 0; d4 < MD / 4; ++d4) {
      const float4 v4 = vp[d4];
      ds += di[4 * d4] * v4.x + di[4 * d4 + 1] * v4.y + di[4 * d4 + 2] * v4.z + di[4 * d4 + 3] * v4.w;
    }
    const float sj = __expf(val[j] - m) / l;
    rloc += sj * ds;
    val[j] = sj * ds;                                   // S * dS for now; turned into dZ below
  }
  const float rowdot = reduce(rloc, false);
  if (tid == 0) stats[row0 + i] = make_float4(m, l, rowdot, 0.f);
  // dZ_ij = S_ij dS_ij - S_ij rowdot; S_ij is recomputed from the logit, which val no longer holds: recompute it
  for (int j = tid; j < T; j += 256) {
    const float4* kp = reinterpret_cast<const float4*>(kc + (row0 + j) * MD);
    float z = 0.f;
    for (int d4 = 0; d4 < MD / 4; ++d4) {
      const float4 k4 = kp[d4];
      z += qi[4 * d4] * k4.x + qi[4 * d4 + 1] * k4.y + qi[4 * d4 + 2] * k4.z + qi[4 * d4 + 3] * k4.w;
    }
    val[j] -= __expf(z * scale - m) / l * rowdot;
  }
  __syncthreads();
  if (tid < MD) {
    float acc = 0.f;
    for (int j = 0; j < T; ++j) acc += val[j] * kc[(row0 + j) * MD + tid];
    dqc[(row0 + i) * MD + tid] = acc * scale;
  }
}

// Column j of the pooled map: dKc[j] = sum_i dZ_ij Qc_i / sqrt D, dVc[j] = sum_i S_ij dOc_i, with S and dZ recomputed from the
// row statistics.  LDS: kc_j, vc_j, 2 T values.
__global__ __launch_bounds__(256) void k_bwd_coarse_cols(const float* __restrict__ qc, const float* __restrict__ kc,
                                                         const float* __restrict__ vc, const float* __restrict__ doc,
                                                         const float4* __restrict__ stats, float* __restrict__ dkc,
                                                         float* __restrict__ dvc, Counts cnt, int H) {
  extern __shared__ float sm[];
  float* kj = sm; float* vj = sm + MD; float* sv = sm + 2 * MD; float* dz = sv + cnt.T_max;
  const int j = blockIdx.x, h = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
  const int T = cnt.b[b].T, T_max = cnt.T_max;
  if (j >= T) return;
  const long long row0 = ((long long)b * H + h) * T_max;
  const float scale = 1.0f / sqrtf((float)MD);
  if (tid < MD) { kj[tid] = kc[(row0 + j) * MD + tid]; vj[tid] = vc[(row0 + j) * MD + tid]; }
  __syncthreads();
  for (int i = tid; i < T; i += 256) {
    const float4* qp = reinterpret_cast<const float4*>(qc + (row0 + i) * MD);
    const float4* dp = reinterpret_cast<const float4*>(doc + (row0 + i) * MD);
    float z = 0.f, ds = 0.f;
    for (int d4 = 0; d4 < MD / 4; ++d4) {
      const float4 q4 = qp[d4], o4 = dp[d4];
      z += q4.x * kj[4 * d4] + q4.y * kj[4 * d4 + 1] + q4.z * kj[4 * d4 + 2] + q4.w * kj[4 * d4 + 3];
      ds += o4.x * vj[4 * d4] + o4.y * vj[4 * d4 + 1] + o4.z * vj[4 * d4 + 2] + o4.w * vj[4 * d4 + 3];
    }
    const float4 st = stats[row0 + i];
    const float sij = __expf(z * scale - st.x) / st.y;
    sv[i] = sij;
    dz[i] = sij * (ds - st.z);
  }
  __syncthreads();
  if (tid < MD) {
    float ak = 0.f, av = 0.f;
    for (int i = 0; i < T; ++i) {
      ak += dz[i] * qc[(row0 + i) * MD + tid];
      av += sv[i] * doc[(row0 + i) * MD + tid];
    }
    dkc[(row0 + j) * MD + tid] = ak * scale;
    dvc[(row0 + j) * MD + tid] = av;
  }
}

// mean_grad[bh][e] (gradient of the gathered mean of kv_list[e], or nothing yet if `fresh`) += coarse[bh][kv_list[e]]
__global__ __launch_bounds__(128) void k_bwd_add_coarse(float* __restrict__ mean_grad, const float* __restrict__ coarse,
                                                        const int* __restrict__ kv_list, int fresh, Counts cnt, int H,
                                                        int Tn_pad) {
  const int e = blockIdx.x, h = blockIdx.y, b = blockIdx.z, d = threadIdx.x;
  if (e >= cnt.b[b].T_new) return;
  const long long bh = (long long)b * H + h;
  const int blk = block_in_range(kv_list[bh * cnt.T_max + e], cnt.b[b].T);
  const float prev = fresh ? 0.f : mean_grad[(bh * Tn_pad + e) * MD + d];
  mean_grad[(bh * Tn_pad + e) * MD + d] = prev + coarse[(bh * cnt.T_max + blk) * MD + d];
}

// Transposed exact-set bits: bit r of word r / 32 of row t is bit t of row r of `mask` (r: position in the Taylor list,
// t: position in the kept list), so that a kept block finds the Taylor blocks that attend to its tokens.
__global__ __launch_bounds__(128) void k_bwd_tmask(const uint32_t* __restrict__ mask, uint32_t* __restrict__ mask_t,
                                                  Counts cnt, int H) {
  const int t = blockIdx.x, h = blockIdx.y, b = blockIdx.z, w = threadIdx.x;
  const int T_max = cnt.T_max, mw = cnt.mask_words;
  if (w >= mw) return;
  const long long bh = (long long)b * H + h;
  uint32_t out = 0u;
  if (t < cnt.b[b].T_new)
    for (int i = 0; i < 32; ++i) {
      const int r = 32 * w + i;
      if (r < cnt.b[b].n_flat) out |= ((mask[(bh * T_max + r) * mw + (t >> 5)] >> (t & 31)) & 1u) << i;
    }
  mask_t[(bh * T_max + t) * mw + w] = out;
}

// Adds the partial sums of the parts of a mean-row launch into part 0: one workgroup per gathered mean row.
__global__ __launch_bounds__(128) void k_bwd_sum_parts(float* __restrict__ g, int parts, long long part_stride, Counts cnt,
                                                       int H, int Tn_pad) {
  const int e = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  if (e >= cnt.b[b].T_new) return;
  const long long i = (((long long)b * H + h) * Tn_pad + e) * MD + threadIdx.x;
  float sum = g[i];
  for (int p = 1; p < parts; ++p) sum += g[p * part_stride + i];
  g[i] = sum;
}

// Adds up the parts of the tail items of a token-row launch and writes their rows: what the attention kernel's own store
// does for whole items.  One workgroup per (XCD, tail item, block of the pair, 8 rows); 32 threads per row, 4 channels each.
__global__ __launch_bounds__(256) void k_bwd_tail_merge(BwdArgs a) {
  const int rows8 = blockIdx.x & 15, grp = (blockIdx.x >> 4) & 1;
  const int r = (blockIdx.x >> 5) % a.tail_items, xcd = (blockIdx.x >> 5) / a.tail_items;
  const int idx = a.items_xcd - a.tail_items + r;
  const int item = idx % a.items, bhid = (idx / a.items) * 8 + xcd;
  if (bhid >= a.geo.B * a.geo.H) return;
  const int h = bhid % a.geo.H, b = bhid / a.geo.H;
  const long long bh = bhid;
  const int T_max = a.geo.T_max;
  const int n_stat = a.stat_kind == 0 ? a.cnt.b[b].n_full : a.stat_kind == 1 ? a.cnt.b[b].n_flat : a.cnt.b[b].T_new;
  const int entry = 2 * item + grp;
  if (entry >= n_stat) return;
  const int blk = block_in_range(a.stat_list[bh * T_max + entry], a.cnt.b[b].T);
  const int n_x = a.blk_n[b * T_max + blk], x_start = a.blk_start[b * T_max + blk];
  const int row = rows8 * 8 + (threadIdx.x >> 5), ch = (threadIdx.x & 31) * 4;
  if (row >= n_x) return;
  const float* src = a.tail_scratch + ((((long long)xcd * a.tail_items + r) * a.tail_parts) * 256 + grp * 128 + row) * MD + ch;
  float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int p = 0; p < a.tail_parts; ++p) {
    const float4 o = *reinterpret_cast<const float4*>(src + (long long)p * 256 * MD);
    sum.x += o.x; sum.y += o.y; sum.z += o.z; sum.w += o.w;
  }
  sum.x *= a.oscale; sum.y *= a.oscale; sum.z *= a.oscale; sum.w *= a.oscale;
  if (a.add_rows) {
    const float inv_n = 1.0f / (float)n_x;
    const float4 m4 = *reinterpret_cast<const float4*>(a.add_by_block ? a.add_rows + (bh * T_max + blk) * MD + ch
                                                                      : a.add_rows + (bh * a.Tn_pad + entry) * MD + ch);
    sum.x = fmaf(m4.x, inv_n, sum.x); sum.y = fmaf(m4.y, inv_n, sum.y);
    sum.z = fmaf(m4.z, inv_n, sum.z); sum.w = fmaf(m4.w, inv_n, sum.w);
  }
  bf16x2 lo = {(__bf16)sum.x, (__bf16)sum.y};
  bf16x2 hi = {(__bf16)sum.z, (__bf16)sum.w};
  uint2 o;
  o.x = *reinterpret_cast<uint32_t*>(&lo);
  o.y = *reinterpret_cast<uint32_t*>(&hi);
  const long long tbase = (long long)b * a.geo.stride_b + (long long)h * a.geo.stride_h;
  *reinterpret_cast<uint2*>(a.out_bf + tbase + (long long)(x_start + row) * a.geo.stride_t + ch) = o;
}

// YD (the streamed rows are queries, which carry deltas; the stationary rows then must not: a.dx == nullptr) is implied
// by what the launch streams.
template <bool SM, bool T2, bool YD>
static hipError_t launch_one(BwdArgs a, int ex, int B, int H, hipStream_t st, bool split_tail = false, int* dyn_ctr = nullptr) {
  if (a.items <= 0) return hipSuccess;
  if (YD && a.dx != nullptr) return hipErrorInvalidValue;
  const int hpx = (B * H + 7) / 8;                // (batch, head)s per XCD
  a.items_xcd = a.items * hpx;
  a.tail_items = 0; a.tail_parts = 1;
  a.dyn_ctr = SM ? nullptr : dyn_ctr;
  if (!SM && !a.dyn_ctr && split_tail && a.n_phases == 1 && ex == 0 && a.tail_scratch) {
    // the last round of an XCD's 32 compute units: if at most half of them would have an item, cut those items
    const int cus = cus_per_xcd(), t = a.items_xcd % cus;
    if (t > 0 && t <= cus / 2) {
      int parts = cus / t > 8 ? 8 : cus / t;
      while (parts > 1 && N_XCD * t * parts > SPLIT_MAX_SUB) --parts;       // the partial-result area holds SPLIT_MAX_SUB sub-items
      if (parts > 1) { a.tail_items = t; a.tail_parts = parts; }
    }
  }
  // dynamic items: an eighth more workgroups than items and one round of the chip, so that the faster XCDs do not run out
  // of workgroups before the items run out
  const long long n_dyn = (long long)a.items * B * H;
  const long long dyn_wgs = ((n_dyn + n_dyn / 8) / N_XCD + cus_per_xcd() + 1) * N_XCD;
  const dim3 grid((unsigned)(SM ? a.items * a.parts * hpx * 8
                                : a.dyn_ctr ? dyn_wgs : (a.items_xcd - a.tail_items + a.tail_items * a.tail_parts) * 8));
  if (ex == 2) {                                // position bits only occur with token rows as stationary rows and dS
    if (SM || !T2 || YD) return hipErrorInvalidValue;
    hipLaunchKernelGGL((k_attn_bwd<false, true, 2, false>), grid, dim3(512), 0, st, a);
  } else if (ex == 1) {
    hipLaunchKernelGGL((k_attn_bwd<SM, T2, 1, YD>), grid, dim3(512), 0, st, a);
  } else {
    hipLaunchKernelGGL((k_attn_bwd<SM, T2, 0, YD>), grid, dim3(512), 0, st, a);
  }
  if (a.tail_items > 0)
    hipLaunchKernelGGL(k_bwd_tail_merge, dim3((unsigned)(8 * a.tail_items * 32)), dim3(256), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_attn_bwd(const Problem& pr, const Workspace& ws, const void* q, const void* k, const void* v,
                           const void* out, const void* d_out, const int* kv_list, const int* full_list,
                           const int* flat_list, const uint32_t* exact_mask, void* dq, void* dk, void* dv,
                           hipStream_t st) {
  const float gamma = (float)pr.p.gamma;
  const bool resid = pr.p.gamma != 0.0;               // ws.ocoarse holds O_coarse (recomputed by the caller of this function)
  const int B = pr.p.B, H = pr.p.H, T_max = pr.cnt.T_max;
  int S_max = pr.S_max, sf = 0, sl = 0, sk = 0, kx = 0;
  for (int b = 0; b < B; ++b) {
    const BatchCounts& c = pr.cnt.b[b];
    sf = c.n_full > sf ? c.n_full : sf;
    sl = c.n_flat > sl ? c.n_flat : sl;
    sk = c.T_new > sk ? c.T_new : sk;
    kx = c.k_exact > kx ? c.k_exact : kx;
  }
  // The forward ran its 4-wave kernel (exact sets, possibly empty ones when exact_frac is too small for the list): token
  // keys and mean keys in one softmax, the mean keys stored minus Kc_0 and q . Kc_0 kept per Taylor row (ws.rq).
  const bool ex = pr.p.exact_frac > 0.0 && sl > 0 && exact_mask != nullptr;
  (void)kx;
#define ISA_BWD_CHECK()                           \
  do {                                            \
    hipError_t e__ = hipGetLastError();           \
    if (e__ != hipSuccess) return e__;            \
  } while (0)
  // delta, zero fill, per-list tables and row terms
  hipLaunchKernelGGL(k_bwd_delta, dim3((S_max + 15) / 16, H, B), dim3(256), 0, st, (const uint16_t*)out,
                     ws.olo, (const uint16_t*)d_out, ws.delta, ws.bwd_ctr, pr.geo, pr.cnt, S_max);
  ISA_BWD_CHECK();
  if (resid) {
    // gradient of the coarse residual with respect to the block means (all blocks, by block id), and delta without
    // the residual's share
    hipLaunchKernelGGL(k_bwd_docoarse, dim3(T_max, H, B), dim3(128), 0, st, (const uint16_t*)d_out, ws.ocoarse, gamma,
                       ws.delta, ws.doc, ws.btab, pr.geo, pr.cnt, S_max);
    ISA_BWD_CHECK();
    hipLaunchKernelGGL(k_bwd_coarse_rows, dim3(T_max, H, B), dim3(256), (size_t)(2 * MD + T_max) * 4, st, ws.qc, ws.kc,
                       ws.vc, ws.doc, ws.cstats, ws.cdq, pr.cnt, H);
    hipLaunchKernelGGL(k_bwd_coarse_cols, dim3(T_max, H, B), dim3(256), (size_t)(2 * MD + 2 * T_max) * 4, st, ws.qc,
                       ws.kc, ws.vc, ws.doc, ws.cstats, ws.cdk, ws.cdv, pr.cnt, H);
    ISA_BWD_CHECK();
  }
  hipLaunchKernelGGL(k_bwd_fill, dim3(T_max, H, B), dim3(256), 0, st, (uint16_t*)dk, resid ? ws.cdk : nullptr, ws.btab,
                     pr.geo, pr.cnt);
  hipLaunchKernelGGL(k_bwd_fill, dim3(T_max, H, B), dim3(256), 0, st, (uint16_t*)dv, resid ? ws.cdv : nullptr, ws.btab,
                     pr.geo, pr.cnt);
  ISA_BWD_CHECK();
  const int gx = T_max > pr.Tn_pad ? T_max : pr.Tn_pad;
  const float* no_rq = nullptr;
  const float cs = 1.4426950408889634f / sqrtf((float)MD);      // raw score -> log2 domain
  hipLaunchKernelGGL(k_bwd_rows, dim3(gx, H, B), dim3(128), 0, st, kv_list, 0, ws.btab, ws.nlse, no_rq, 0.f, ws.delta, ws.ktab,
                     ws.ybd_kv, ws.ybd_mean, ws.bx_mean, pr.cnt, H, pr.Tn_pad, S_max);
  hipLaunchKernelGGL(k_bwd_rows, dim3(gx, H, B), dim3(128), 0, st, full_list, 1, ws.btab, ws.nlse, no_rq, 0.f, ws.delta, ws.ftab,
                     ws.ybd_full, ws.ybd_mean, ws.bx_mean, pr.cnt, H, pr.Tn_pad, S_max);
  hipLaunchKernelGGL(k_bwd_rows, dim3(gx, H, B), dim3(128), 0, st, flat_list, 2, ws.btab, ws.nlse, no_rq, 0.f, ws.delta, ws.ltab,
                     ws.ybd_flat, ws.ybd_mean, ws.bx_mean, pr.cnt, H, pr.Tn_pad, S_max);
  if (ex)             // the same rows with q . Kc_0 in their exponent terms, for the launches that score them against gathered means
    hipLaunchKernelGGL(k_bwd_rows, dim3(gx, H, B), dim3(128), 0, st, flat_list, 2, ws.btab, ws.nlse, (const float*)ws.rq, cs, ws.delta,
                       ws.ltab, ws.ybd_flatm, ws.ybd_mean, ws.bx_mean, pr.cnt, H, pr.Tn_pad, S_max);
  ISA_BWD_CHECK();
  if (ex) {
    hipLaunchKernelGGL(k_bwd_tmask, dim3(T_max, H, B), dim3(128), 0, st, exact_mask, ws.mask_t, pr.cnt, H);
    ISA_BWD_CHECK();
  }

  BwdArgs a;
  a.blk_start = ws.blk_start; a.blk_n = ws.blk_n;
  a.geo = pr.geo; a.cnt = pr.cnt; a.Tn_pad = pr.Tn_pad; a.S_max = S_max;
  a.mask_words = pr.cnt.mask_words;
  a.parts = 1; a.part_stride = 0;
  a.items_xcd = 0; a.tail_items = 0; a.tail_parts = 1; a.tail_scratch = ws.split_o;   // the forward's partial-result area: 256 x 256 x 128 floats
  const float scale = 1.0f / sqrtf((float)MD);
  const uint16_t *Q = (const uint16_t*)q, *K = (const uint16_t*)k, *V = (const uint16_t*)v, *DO = (const uint16_t*)d_out;
  const BwdStream none = {nullptr, nullptr, nullptr, nullptr, nullptr, 0, 0};
  hipError_t e;

  // ---- dQ: exact branch over the kept tokens; Taylor branch over the tokens of each block's exact
  // set and the means of the other kept blocks
  const BwdStream kept_tokens = {K, V, nullptr, ws.ktab, ws.ybd_kv, 0, 0};
  const uint16_t* mean_keys = ws.kcn;             // stored minus the mean key of block 0
  const BwdStream kept_means = {mean_keys, ws.vcn, ex ? ws.kcnb : nullptr, nullptr, ws.ybd_mean, 0, 0};
  a.x1 = Q; a.x2 = DO; a.bx = ws.nlse; a.dx = ws.delta; a.rx = nullptr;
  a.out_bf = (uint16_t*)dq; a.out_f32 = nullptr; a.oscale = scale;
  a.add_rows = resid ? ws.cdq : nullptr; a.add_by_block = 1;       // every query block's share of dQc
  a.stat_list = full_list; a.stat_kind = 0; a.items = (sf + 1) / 2;
  a.s[0] = kept_tokens; a.s[1] = none; a.n_phases = 1; a.bits = nullptr;
  if ((e = launch_one<false, true, false>(a, 0, B, H, st, true)) != hipSuccess) return e;
  a.stat_list = flat_list; a.stat_kind = 1; a.items = (sl + 1) / 2;
  if (ex) {
    a.s[0] = kept_tokens; a.s[0].masked = 1;
    a.s[1] = kept_means; a.s[1].masked = 2;
    a.n_phases = 2; a.bits = exact_mask;
    a.rx = ws.rq;
  } else {
    a.s[0] = kept_means; a.n_phases = 1;
  }
  if ((e = launch_one<false, true, false>(a, ex ? 2 : 0, B, H, st, false, ws.bwd_ctr + 0)) != hipSuccess) return e;

  // ---- dKc and dK (streamed Q, dO)
  const int n_mean_pairs = ((sk + 127) / 128 + 1) / 2;
  // The mean-row launches have few items (one per 256 gathered means and head): each is cut into up to BWD_MEAN_PARTS
  // parts along the streamed entries, as many as make the launch's rounds over the 256 compute units shortest.
  int mean_parts = 1;
  {
    const long long wgs = (long long)n_mean_pairs * B * H;
    double best = 1e30;
    for (int p = 1; p <= BWD_MEAN_PARTS; ++p) {
      const long long chip = (long long)cus_per_xcd() * N_XCD;
      const double rounds = (double)((wgs * p + chip - 1) / chip) / p;
      if (rounds < best - 1e-9) { best = rounds; mean_parts = p; }
    }
  }
  const BwdStream full_q = {Q, DO, nullptr, ws.ftab, ws.ybd_full, 1, 0};
  const BwdStream flat_q = {Q, DO, nullptr, ws.ltab, ws.ybd_flat, 2, 0};
  const BwdStream flat_q_means = {Q, DO, nullptr, ws.ltab, ex ? ws.ybd_flatm : ws.ybd_flat, 2, 0};     // scored against gathered means
  a.dx = nullptr; a.rx = nullptr;
  for (int pass = 0; pass < 2; ++pass) {          // pass 0: dKc, dK (W = dS, read Q transposed); pass 1: dVc, dV (W = P, dO transposed)
    float* mean_grad = pass == 0 ? ws.dkc : ws.dvc;
    const float osc = pass == 0 ? scale : 1.0f;
    if (sl > 0) {                                 // gradients of the gathered means: every Taylor block, minus its exact set
      a.x1 = mean_keys; a.x2 = pass == 0 ? ws.vcn : nullptr; a.stat_list = nullptr; a.stat_kind = 2; a.bx = ws.bx_mean;
      a.s[0] = flat_q_means; a.s[0].masked = ex ? 3 : 0; a.s[1] = none; a.n_phases = 1; a.bits = ws.mask_t;
      a.out_bf = nullptr; a.out_f32 = mean_grad; a.add_rows = nullptr; a.add_by_block = 0; a.oscale = osc; a.items = n_mean_pairs;
      a.parts = mean_parts; a.part_stride = (long long)B * H * pr.Tn_pad * MD;
      e = pass == 0 ? launch_one<true, true, true>(a, ex ? 1 : 0, B, H, st) : launch_one<true, false, false>(a, ex ? 1 : 0, B, H, st);
      if (e != hipSuccess) return e;
      if (mean_parts > 1) {
        hipLaunchKernelGGL(k_bwd_sum_parts, dim3(sk, H, B), dim3(128), 0, st, mean_grad, mean_parts, a.part_stride, pr.cnt, H,
                           pr.Tn_pad);
        ISA_BWD_CHECK();
      }
      a.parts = 1;
    }
    if (resid) {                                  // the coarse residual's gradient of the same means joins the Taylor branch's
      hipLaunchKernelGGL(k_bwd_add_coarse, dim3(sk, H, B), dim3(128), 0, st, mean_grad, pass == 0 ? ws.cdk : ws.cdv,
                         kv_list, sl > 0 ? 0 : 1, pr.cnt, H, pr.Tn_pad);
      ISA_BWD_CHECK();
    }
    // gradients of the kept tokens: every full-attention block, the Taylor blocks whose exact set holds the block, and
    // the block's share of its mean's gradient
    a.x1 = K; a.x2 = pass == 0 ? V : nullptr; a.stat_list = kv_list; a.stat_kind = 2; a.bx = nullptr;
    a.s[0] = full_q; a.s[1] = none; a.n_phases = 1; a.bits = nullptr;
    if (ex) { a.s[1] = flat_q; a.s[1].masked = 1; a.n_phases = 2; a.bits = ws.mask_t; }
    a.out_bf = (uint16_t*)(pass == 0 ? dk : dv); a.out_f32 = nullptr;
    a.add_rows = (sl > 0 || resid) ? mean_grad : nullptr; a.add_by_block = 0;
    a.oscale = osc; a.items = (sk + 1) / 2;
    e = pass == 0 ? launch_one<false, true, true>(a, ex ? 1 : 0, B, H, st, true, ws.bwd_ctr + 1)
                  : launch_one<false, false, false>(a, ex ? 1 : 0, B, H, st, true, ws.bwd_ctr + 2);
    if (e != hipSuccess) return e;
  }
#undef ISA_BWD_CHECK
  return hipSuccess;
}

}  // namespace isa
