// Internal declarations shared by the host API and the kernel files of libisa_hip.
// Nothing here is exported; the C ABI lives in include/isa.h.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "isa.h"

namespace isa {

// Segment lengths of every batch item, passed to kernels by value.
struct SegDesc {
  int B;
  int seg_ptr[ISA_MAX_BATCH + 1];
  int seg_len[ISA_MAX_SEGMENTS];
};

// Per-batch counts derived on the host (see isa_counts), passed to kernels by value.
struct BatchCounts {
  int S, T, T_src, T_ctx, k_keep, T_new, n_flat, n_full, k_exact;
};
struct Counts {
  BatchCounts b[ISA_MAX_BATCH];
  int T_max;
  int mask_words;   // uint32 words per exact_mask row = ceil(T_max / 32)
};

// Shapes and strides common to all kernels.
struct Geometry {
  int B, H, D, block, T_max;
  long long stride_b, stride_h, stride_t;   // element strides of q, k, v, out
};

// Workspace carve-up (device pointers into the caller's workspace).
constexpr int BWD_MEAN_PARTS = 4;    // backward: parts a mean-row work item may be cut into (partial sums in dkc / dvc)
constexpr int SPLIT_MAX_SUB = 256;   // sub-items of split work items per launch: at most one per compute unit

struct Workspace {
  int* blk_start;        // [B][T_max] token offset of each block inside its batch item
  int* blk_n;            // [B][T_max] real tokens of each block
  int4* btab;            // [B][T_max] {token offset, real tokens, block index, 0} of each block
  float* qc;             // [B,H,T_max,D]
  float* kc;
  float* vc;
  float* s_ctx;          // [B,H,T_max]
  float* sharp;          // [B,H,T_max]
  float* pctx;           // [B,H,Tsrc_max,Tctx_max] context part of the source rows of S_coarse
  int* kv_list;          // [B,H,T_max]
  int* full_list;
  int* flat_list;
  float* z;              // [B,H,T_max,T_max], only when exact_frac > 0
  uint32_t* exact_mask;  // [B,H,T_max,mask_words], only when exact_frac > 0
  // operand copies of the MFMA path (bf16, D = 128, block = 128)
  uint16_t* vt;          // [B,H,T_max][D][128]: V of each block, transposed and key-permuted
  uint16_t* kcn;         // [B,H,Tn_pad][D]: mean keys gathered in kv_list order, minus the mean key of block 0
  uint16_t* vcnt;        // [B,H,Tn_pad/128][D][128]: mean values gathered, transposed, key-permuted
  float* biasn;          // [B,H,Tn_pad]: ln(n_j) sqrt(D) per gathered mean key (without exact sets: ln(n_j / block) sqrt(D)), -inf for padding
  int* tflag;            // [B,H,Tn_pad/64]: 1 if a tile of mean keys needs its bias or masks (padding, a short block, exact sets)
  uint16_t* vt4; uint16_t* vcnt4;   // the same two arrays in the key order of the 4-wave kernel (only with exact sets)
  uint16_t* zero_tile;   // 16 KB of zeros, written by the V^T pack kernel
  int* taylor_ctr;       // the next Taylor group of the attention launch (zeroed by the mean gather, counted up by the launch)
  int* bwd_ctr;          // backward: the next work item of each launch that hands its items out dynamically (8 counters, zeroed by k_bwd_delta)
  int4* ktab;            // [B,H,T_max] the btab rows of the blocks of kv_list, in list order
  float* ocoarse;        // [B,H,T_max,D] pooled attention output (only carved when gamma != 0)
  float* split_o;        // partial outputs of work items split along the key sequence (at most 256 sub-items)
  float* split_ml;       // their running maxima and sums
  // backward pass (MFMA path): what the forward leaves for it, and its own scratch
  float* nlse;           // [B,H,S_max] minus the log-sum-exp of every query row, log2 domain (written by the forward)
  uint16_t* olo;         // [B,H,S_max,D] bf16: what the rounding of the output to bf16 cut off (written by the forward)
  float* delta;          // [B,H,S_max] rowsum(dO * O)
  uint16_t* vcn;         // [B,H,Tn_pad][D]: mean values gathered in kv_list order (row-major, bf16)
  float* dkc; float* dvc;             // [BWD_MEAN_PARTS][B,H,Tn_pad][D] gradients of the gathered mean keys / values (part 0: the sum)
  int4* ftab; int4* ltab;             // [B,H,T_max] table rows of the full-attention / Taylor blocks, in list order
  float2* ybd_kv; float2* ybd_full; float2* ybd_flat;   // [B,H,T_max*128 pairs] per tile of 64 row positions of the list entries: 64 exponent terms, then 64 minus-deltas
  float2* ybd_mean;      // [B,H,Tn_pad] the same per gathered mean key
  uint16_t* kcnb;        // [B,H,Tn_pad][D]: the gathered mean keys without the subtraction of Kc_0 (only with exact sets: what the
                         // backward's dQ of a Taylor row multiplies dS with)
  float2* ybd_flatm;     // as ybd_flat, the exponent terms with the rows' q . Kc_0 added (only with exact sets: for scores against
                         // the gathered mean keys, which are stored minus Kc_0)
  float* rq;             // [B,H,S_max] q . Kc_0 in raw score units, written by the forward's 4-wave kernel (only with exact sets)
  float* bx_mean;        // [B,H,Tn_pad] log2(n_j) per gathered mean key
  uint32_t* mask_t;      // [B,H,T_max,mask_words] exact_mask transposed (only when exact_frac > 0)
  float* doc; float* cdq; float* cdk; float* cdv;   // [B,H,T_max,D] coarse residual: gamma * block sums of dO, gradients of the means (only when gamma != 0)
  float4* cstats;        // [B,H,T_max] {max, sum, rowsum(dS * S)} of every row of the pooled map (only when gamma != 0)
  size_t bytes;          // total size
};

struct Problem {          // validated problem + everything derived from it
  isa_problem p;
  SegDesc seg;
  Counts cnt;
  Geometry geo;
  int Tsrc_max, Tctx_max, Tn_pad, S_max;
  bool mfma_shape;        // bf16, D = 128, block = 128
};

// A block index read from a caller-provided list, forced into the batch item's range: the lists of the staged entry
// points are not validated, and an entry out of range must give a wrong result, not an access outside the tensors.
__device__ __forceinline__ int block_in_range(int j, int T) { return j < 0 ? 0 : (j >= T ? T - 1 : j); }

extern hipEvent_t g_prof_start, g_prof_stop;   // events recorded around the MFMA attention kernel when g_prof_on
extern int g_prof_on, g_prof_recorded;

// Compute units per XCD of the current device (the launch heuristics that cut the items of a last, half-empty round into
// parts count rounds over them): a device's compute units / 8, as the workgroup ids of a launch go round-robin over the 8
// XCDs of an MI355X; 32 there, and 32 if the device cannot be asked.  Only work distribution depends on it, no result.
int cus_per_xcd();
constexpr int N_XCD = 8;

int validate(const isa_problem* p, Problem* out);
// forward_only: without the arrays that the forward pass leaves for, and that are scratch of, the backward pass
void carve(const Problem& pr, void* base, Workspace* ws, bool forward_only = false);

// ---- kernel launchers (each returns hipError_t of the launch) -------------------------------
struct AttnArgs {
  const void* q; const void* k; const void* v; void* out;
  const float* kc; const float* vc;             // block means, fp32 [B,H,T_max,D]
  const int* blk_start; const int* blk_n;       // [B][T_max]
  const int* kv_list; const int* full_list; const int* flat_list;   // [B,H,T_max]; null in dense mode
  const uint32_t* exact_mask;                   // may be null
  const float* ocoarse; float gamma;            // coarse residual: out += gamma * ocoarse[block] (ocoarse null when gamma == 0)
  Geometry geo;
  Counts cnt;
  int dense;                                    // 1: every query block attends to every block
};

hipError_t launch_layout(const Problem& pr, const Workspace& ws, hipStream_t st);
hipError_t launch_block_means(const Problem& pr, const Workspace& ws, const void* q, const void* k, const void* v,
                              float* qc, float* kc, float* vc, hipStream_t st);
hipError_t launch_coarse(const Problem& pr, const Workspace& ws, const float* qc, const float* kc,
                         float* s_ctx, float* sharp, float* z, const float* vc, float* ocoarse, hipStream_t st);
hipError_t launch_select(const Problem& pr, const Workspace& ws, const float* s_ctx, const float* sharp, const float* z,
                         int* kv_list, int* full_list, int* flat_list, uint32_t* exact_mask, hipStream_t st);
hipError_t launch_attn_simt(const Problem& pr, const AttnArgs& a, hipStream_t st);

// MFMA path (bf16, D = 128, block = 128)
// vc (may be null): also writes the fp32 block means of V, [B,H,T_max,D]
hipError_t launch_pack_vt(const Problem& pr, const Workspace& ws, const void* v, float* vc, hipStream_t st);
hipError_t launch_gather_means(const Problem& pr, const Workspace& ws, const float* kc, const float* vc,
                               const int* kv_list, hipStream_t st);
hipError_t launch_attn_mfma(const Problem& pr, const Workspace& ws, const AttnArgs& a, hipStream_t st);
hipError_t launch_attn_bwd(const Problem& pr, const Workspace& ws, const void* q, const void* k, const void* v,
                           const void* out, const void* d_out, const int* kv_list, const int* full_list,
                           const int* flat_list, const uint32_t* exact_mask, void* dq, void* dk, void* dv,
                           hipStream_t st);

// prologue (prologue.hip): tile order, rotary embedding and block means in one pass (inverse: its transpose, no means);
// the inverse reordering of one tensor
hipError_t launch_prologue(const Problem& pr, const isa_grid* gr, const void* q_in, const void* k_in, const void* v_in,
                           void* q_out, void* k_out, void* v_out, float* qc, float* kc, float* vc, bool inverse,
                           hipStream_t st);
hipError_t launch_untile(const Problem& pr, const isa_grid* gr, const void* x_tiled, void* x_raster, hipStream_t st);

}  // namespace isa
