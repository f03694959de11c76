// Declarations shared by the MFMA attention kernels (bf16, D = 128, block = 128).
#pragma once

#include "isa_internal.h"

namespace isa {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int MD = 128;           // head dim
constexpr int KT = 64;            // keys per LDS tile
constexpr int K_TILE = KT * MD;   // bf16 elements of one K tile in LDS: 64 rows x 256 B, 16-byte chunks XOR-swizzled
constexpr int V_TILE = MD * KT;   // bf16 elements of one V^T tile in LDS: 128 rows x 128 B, 16-byte chunks XOR-swizzled
constexpr float RESCALE_TAU = 8.0f;    // the running max is only raised when a tile exceeds it by 2^tau
constexpr float M_INIT = -1.0e30f;

__device__ inline uint16_t f2bf(float f) {     // round to nearest even
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
  return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}
// Four fp32 results as stored: `hi` the bf16 roundings that go to `out`, `lo` the bf16 roundings of what those cut off.
__device__ __forceinline__ void split_bf16x4(const float4 r, uint2& hi, uint2& lo) {
  const float x[4] = {r.x, r.y, r.z, r.w};
  uint16_t h[4], l[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const __bf16 hb = (__bf16)x[i];
    h[i] = __builtin_bit_cast(uint16_t, hb);
    l[i] = __builtin_bit_cast(uint16_t, (__bf16)(x[i] - (float)hb));
  }
  hi = make_uint2(h[0] | ((uint32_t)h[1] << 16), h[2] | ((uint32_t)h[3] << 16));
  lo = make_uint2(l[0] | ((uint32_t)l[1] << 16), l[2] | ((uint32_t)l[3] << 16));
}
__device__ inline int swap23(int k) { return (k & ~12) | ((k & 4) << 1) | ((k & 8) >> 1); }
// Key stored at position p of a 64-key V^T row in the layout of the 16x16x32 kernel: inside each 32-key group,
// position 8 q + 4 kt + i holds key 16 kt + 4 q + i (the order in which a lane's score registers list its keys).
__device__ inline int key_of_pos16(int p) { return (p & 32) | ((p & 4) << 2) | ((p >> 1) & 12) | (p & 3); }

struct MfmaArgs {
  const uint16_t* q; const uint16_t* k; uint16_t* out;
  const uint16_t* vt;                       // packed V^T
  const uint16_t* kcn; const uint16_t* vcnt; const float* biasn;
  const float* kc;                          // fp32 block means of K, [bh][T_max][128]: row 0 is what kcn is stored short of
  const int* tflag;                         // per tile of gathered means: 1 = needs the bias / mask path (k_attn_sp)
  float lse_shift;                          // log2 of the factor the mean keys' weights are stored short of (0 with exact sets)
  const uint16_t* zero_tile;                // 16 KB of zeros (a V^T tile that contributes nothing)
  const int* blk_start; const int* blk_n;
  const int4* btab; const int4* ktab;        // {token offset, real tokens, block index} per block / per kv_list entry
  const int* kv_list; const int* full_list; const int* flat_list;
  const uint32_t* exact_mask;
  const float* ocoarse; float gamma;        // coarse residual: out += gamma * ocoarse[bh, block] (never in dense mode)
  Geometry geo;
  Counts cnt;
  int dense;
  int Tn_pad;
  int slots;                                // work slots per (batch, head) = T_max
  int total;                                // B * H * slots
  int slots_first, slots_second;            // k_attn_sp: exact / Taylor pair slots per (batch, head), each at least 1
  int tgroup, groups_second;                // k_attn_sp: Taylor pairs per group; such groups per (batch, head), at least 1
  int n_taylor_wg;                          // k_attn_sp: workgroups per XCD that work through the Taylor groups
  int* taylor_ctr;                          // k_attn_sp: the next Taylor group to be taken (device memory, 0 when the launch starts)
  int* long_ctr; int n_long_all;            // k_attn_sp: null, or the next long item to be taken, numbered over all (batch, head)s, and their number
  int hpx, n_long;                          // k_attn_sp: (batch, head)s per XCD; exact-branch items per XCD (0 if none)
  int n_split, parts;                       // k_attn_sp: the last n_split exact-branch items of an XCD run as `parts` sub-items over key ranges
  float* split_o; float* split_ml;          // their partial results: unnormalised outputs [sub-item][2][128][128], {max, sum} [sub-item][2][128][2]
  float* nlse; int S_max;                   // minus the log-sum-exp (log2 domain) of every query row, [bh][S_max]; may be null
  float* rq;                                // [bh][S_max], may be null: q . Kc_0 (raw score units) of every Taylor row with exact sets
  uint16_t* olo;                            // [bh][S_max][128] bf16, may be null: what the rounding of `out` to bf16 cut off
                                            // (out + olo is the fp32 result to about 2^-17), for the backward's delta
  int taylor_here;                          // k_attn_sp: 1 = also process the Taylor slots (no exact sets), 0 = exact branch only
};

hipError_t launch_attn_mfma4(const Problem& pr, MfmaArgs m, hipStream_t st);

}  // namespace isa
