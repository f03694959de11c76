// Host side of libisa_hip: argument validation, count derivation, workspace carve-up and the
// sequence of kernel launches behind each C-ABI entry point declared in include/isa.h.
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <atomic>
#include <mutex>

#include "isa_internal.h"

namespace isa {

static thread_local int g_last_hip = 0;
hipEvent_t g_prof_start = nullptr, g_prof_stop = nullptr;
int g_prof_on = 0, g_prof_recorded = 0;
static std::atomic<int> g_use_mfma{1};

int cus_per_xcd() {
  static const int cus = [] {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 32;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 32;
    return (n >= N_XCD && n % N_XCD == 0) ? n / N_XCD : 32;
  }();
  return cus;
}

static inline bool ratio_ok(double r) { return r >= 0.0 && r <= 1.0; }   // false for NaN
// token tensors are read and written 16 bytes at a time
static inline bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }
template <typename... P> static inline bool all_aligned16(P... ptrs) { return (aligned16(ptrs) && ...); }

int validate(const isa_problem* p, Problem* out) {
  if (!p || !out) return ISA_ERR_NULL;
  if (!p->seg_ptr || !p->seg_len) return ISA_ERR_NULL;
  if (p->dtype != ISA_BF16 && p->dtype != ISA_F32) return ISA_ERR_DTYPE;
  if (p->B < 1 || p->B > ISA_MAX_BATCH || p->H < 1 || p->H > 65535) return ISA_ERR_SHAPE;
  if (p->D != 64 && p->D != 128) return ISA_ERR_SHAPE;
  if (p->block != 64 && p->block != 128) return ISA_ERR_SHAPE;
  if (!ratio_ok(p->keep_ratio) || !ratio_ok(p->full_frac) || !ratio_ok(p->exact_frac)) return ISA_ERR_RATIO;
  if (!isfinite(p->gamma)) return ISA_ERR_UNSUPPORTED;
  if (p->stride_t < p->D || p->stride_t % 8 || p->stride_h % 8 || p->stride_b % 8) return ISA_ERR_SHAPE;
  if (p->stride_h < 0 || p->stride_b < 0) return ISA_ERR_SHAPE;

  Problem& pr = *out;
  memset(&pr, 0, sizeof(pr));
  pr.p = *p;
  pr.seg.B = p->B;
  if (p->seg_ptr[0] != 0) return ISA_ERR_SHAPE;
  int T_max = 0, Tsrc_max = 0, Tctx_max = 0, Tnew_max = 0;
  for (int b = 0; b < p->B; ++b) {
    const int s0 = p->seg_ptr[b], s1 = p->seg_ptr[b + 1];
    if (s1 <= s0 || s1 > ISA_MAX_SEGMENTS) return ISA_ERR_SHAPE;      // at least the source segment
    pr.seg.seg_ptr[b] = s0;
    pr.seg.seg_ptr[b + 1] = s1;
    long long S = 0, T = 0;
    for (int s = s0; s < s1; ++s) {
      const int len = p->seg_len[s];
      if (len < 0 || (s == s0 && len < 1)) return ISA_ERR_SHAPE;     // empty source segment
      pr.seg.seg_len[s] = len;
      S += len;
      T += (len + p->block - 1) / p->block;
      if (S > 0x7fffffffLL / 2) return ISA_ERR_SHAPE;
    }
    if (T > ISA_MAX_BLOCKS) return ISA_ERR_SHAPE;
    BatchCounts& c = pr.cnt.b[b];
    c.S = (int)S;
    c.T = (int)T;
    c.T_src = (p->seg_len[s0] + p->block - 1) / p->block;
    c.T_ctx = c.T - c.T_src;
    c.k_keep = (int)floor(p->keep_ratio * (double)c.T_ctx);
    c.T_new = c.T_src + c.k_keep;
    c.n_flat = (int)floor((1.0 - p->full_frac) * (double)c.T);
    c.n_full = c.T - c.n_flat;
    c.k_exact = (int)floor(p->exact_frac * (double)c.T_new);
    T_max = c.T > T_max ? c.T : T_max;
    Tsrc_max = c.T_src > Tsrc_max ? c.T_src : Tsrc_max;
    Tctx_max = c.T_ctx > Tctx_max ? c.T_ctx : Tctx_max;
    Tnew_max = c.T_new > Tnew_max ? c.T_new : Tnew_max;
  }
  pr.cnt.T_max = T_max;
  pr.cnt.mask_words = (T_max + 31) / 32;
  pr.Tsrc_max = Tsrc_max;
  pr.Tctx_max = Tctx_max > 0 ? Tctx_max : 1;
  pr.Tn_pad = (Tnew_max + 127) / 128 * 128;
  pr.geo = Geometry{p->B, p->H, p->D, p->block, T_max, p->stride_b, p->stride_h, p->stride_t};
  // the MFMA kernels address a head's keys with 32-bit byte offsets: the tokens of one (batch, head) must span < 4 GiB
  long long S_max = 0;
  for (int b = 0; b < p->B; ++b) S_max = pr.cnt.b[b].S > S_max ? pr.cnt.b[b].S : S_max;
  pr.S_max = (int)S_max;
  pr.mfma_shape = p->dtype == ISA_BF16 && p->D == 128 && p->block == 128;
  if (pr.mfma_shape && (unsigned long long)S_max * (unsigned long long)p->stride_t * 2ull >= (1ull << 32)) {
    // Not a silent drop to the portable kernels (50 times slower, and no backward pass): the caller is told, and can
    // still ask for those kernels explicitly with isa_set_mfma(0).
    if (g_use_mfma.load()) return ISA_ERR_UNSUPPORTED;
    pr.mfma_shape = false;
  }
  return ISA_OK;
}

static inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

void carve(const Problem& pr, void* base, Workspace* ws, bool forward_only) {
  const size_t B = pr.p.B, H = pr.p.H, D = pr.p.D, T = pr.cnt.T_max;
  size_t off = 0;
  // integer arithmetic: `base` may be null (size and layout queries), and offsetting a null pointer is undefined
  const uintptr_t b0 = (uintptr_t)base;
  auto take = [&](size_t bytes) { const uintptr_t r = b0 + off; off += align256(bytes); return (void*)r; };
  ws->blk_start = (int*)take(B * T * 4);
  ws->blk_n = (int*)take(B * T * 4);
  ws->btab = (int4*)take(B * T * 16);
  ws->qc = (float*)take(B * H * T * D * 4);
  ws->kc = (float*)take(B * H * T * D * 4);
  ws->vc = (float*)take(B * H * T * D * 4);
  ws->s_ctx = (float*)take(B * H * T * 4);
  ws->sharp = (float*)take(B * H * T * 4);
  ws->pctx = (float*)take(B * H * (size_t)pr.Tsrc_max * (size_t)pr.Tctx_max * 4);
  ws->kv_list = (int*)take(B * H * T * 4);
  ws->full_list = (int*)take(B * H * T * 4);
  ws->flat_list = (int*)take(B * H * T * 4);
  ws->ocoarse = pr.p.gamma != 0.0 ? (float*)take(B * H * T * D * 4) : nullptr;
  if (pr.p.exact_frac > 0.0) {
    ws->z = (float*)take(B * H * T * T * 4);
    ws->exact_mask = (uint32_t*)take(B * H * T * (size_t)pr.cnt.mask_words * 4);
  } else {
    ws->z = nullptr;
    ws->exact_mask = nullptr;
  }
  if (pr.mfma_shape) {
    ws->vt = (uint16_t*)take(B * H * T * D * 128 * 2);
    ws->kcn = (uint16_t*)take(B * H * (size_t)pr.Tn_pad * D * 2);
    ws->vcnt = (uint16_t*)take(B * H * (size_t)pr.Tn_pad * D * 2);
    ws->biasn = (float*)take(B * H * (size_t)pr.Tn_pad * 4);
    ws->tflag = (int*)take(B * H * (size_t)(pr.Tn_pad / 64) * 4);
    ws->vt4 = pr.p.exact_frac > 0.0 ? (uint16_t*)take(B * H * T * D * 128 * 2) : nullptr;
    ws->vcnt4 = pr.p.exact_frac > 0.0 ? (uint16_t*)take(B * H * (size_t)pr.Tn_pad * D * 2) : nullptr;
    ws->zero_tile = (uint16_t*)take(128 * 64 * 2);
    ws->taylor_ctr = (int*)take(256);
    ws->ktab = (int4*)take(B * H * T * 16);
    ws->split_o = (float*)take((size_t)SPLIT_MAX_SUB * 2 * 128 * 128 * 4);
    ws->split_ml = (float*)take((size_t)SPLIT_MAX_SUB * 2 * 128 * 2 * 4);
  }
  if (pr.mfma_shape && !forward_only) {       // what the forward leaves for the backward pass, and the backward's own scratch
    const size_t S = (size_t)pr.S_max, Tn = (size_t)pr.Tn_pad;
    ws->nlse = (float*)take(B * H * S * 4);
    ws->olo = (uint16_t*)take(B * H * S * D * 2);
    ws->delta = (float*)take(B * H * S * 4);
    ws->bwd_ctr = (int*)take(256);
    ws->vcn = (uint16_t*)take(B * H * Tn * D * 2);
    ws->rq = pr.p.exact_frac > 0.0 ? (float*)take(B * H * S * 4) : nullptr;
    ws->kcnb = pr.p.exact_frac > 0.0 ? (uint16_t*)take(B * H * Tn * D * 2) : nullptr;
    ws->ybd_flatm = pr.p.exact_frac > 0.0 ? (float2*)take(B * H * T * 128 * 8) : nullptr;
    ws->dkc = (float*)take(BWD_MEAN_PARTS * B * H * Tn * D * 4);
    ws->dvc = (float*)take(BWD_MEAN_PARTS * B * H * Tn * D * 4);
    ws->ftab = (int4*)take(B * H * T * 16);
    ws->ltab = (int4*)take(B * H * T * 16);
    ws->ybd_kv = (float2*)take(B * H * T * 128 * 8);
    ws->ybd_full = (float2*)take(B * H * T * 128 * 8);
    ws->ybd_flat = (float2*)take(B * H * T * 128 * 8);
    ws->ybd_mean = (float2*)take(B * H * Tn * 8);
    ws->bx_mean = (float*)take(B * H * Tn * 4);
    ws->mask_t = pr.p.exact_frac > 0.0 ? (uint32_t*)take(B * H * T * (size_t)pr.cnt.mask_words * 4) : nullptr;
    if (pr.p.gamma != 0.0) {
      ws->doc = (float*)take(B * H * T * D * 4);
      ws->cdq = (float*)take(B * H * T * D * 4);
      ws->cdk = (float*)take(B * H * T * D * 4);
      ws->cdv = (float*)take(B * H * T * D * 4);
      ws->cstats = (float4*)take(B * H * T * 16);
    } else {
      ws->doc = ws->cdq = ws->cdk = ws->cdv = nullptr;
      ws->cstats = nullptr;
    }
  } else {
    ws->nlse = ws->delta = ws->dkc = ws->dvc = ws->bx_mean = nullptr;
    ws->vcn = ws->olo = nullptr;
    ws->bwd_ctr = nullptr;
    ws->rq = nullptr;
    ws->kcnb = nullptr;
    ws->ybd_flatm = nullptr;
    ws->ftab = ws->ltab = nullptr;
    ws->ybd_kv = ws->ybd_full = ws->ybd_flat = ws->ybd_mean = nullptr;
    ws->mask_t = nullptr;
    ws->doc = ws->cdq = ws->cdk = ws->cdv = nullptr;
    ws->cstats = nullptr;
  }
  if (!pr.mfma_shape) {
    ws->vt = ws->kcn = ws->vcnt = ws->vt4 = ws->vcnt4 = nullptr;
    ws->biasn = nullptr;
    ws->tflag = nullptr;
    ws->zero_tile = nullptr;
    ws->taylor_ctr = nullptr;
    ws->ktab = nullptr;
    ws->split_o = ws->split_ml = nullptr;
  }
  ws->bytes = off;
}

static int check_ws(const Problem& pr, void* workspace, size_t bytes, Workspace* ws) {
  if (!workspace || ((uintptr_t)workspace & 255)) return ISA_ERR_WORKSPACE;
  carve(pr, workspace, ws);
  if (bytes < ws->bytes) return ISA_ERR_WORKSPACE;
  return ISA_OK;
}

static int hip_fail(hipError_t e) {
  g_last_hip = (int)e;
  return ISA_ERR_HIP;
}

#define ISA_TRY(expr)                         \
  do {                                        \
    hipError_t e__ = (expr);                  \
    if (e__ != hipSuccess) return hip_fail(e__); \
  } while (0)

// Debug mode (environment variable ISA_DEBUG=1, read once): every stage of an entry point is followed by a wait for the
// stream and a check of the error state, so that a failing kernel is reported by the call that launched it (ISA_ERR_HIP
// right after the stage, isa_last_hip_error() for the code) instead of by some later, unrelated HIP call.  Entry points
// then block the host, and must not be called on a stream that is being captured.
static bool debug_mode() {
  static const bool on = [] {
    const char* v = getenv("ISA_DEBUG");
    return v && v[0] && !(v[0] == '0' && !v[1]);
  }();
  return on;
}
// A stage: one launcher call on the stream `st` of the enclosing function.
#define ISA_STAGE(expr)                                                  \
  do {                                                                   \
    hipError_t e__ = (expr);                                             \
    if (e__ == hipSuccess && debug_mode()) {                             \
      e__ = hipStreamSynchronize(st);                                    \
      if (e__ == hipSuccess) e__ = hipGetLastError();                    \
    }                                                                    \
    if (e__ != hipSuccess) return hip_fail(e__);                         \
  } while (0)

static AttnArgs attn_args(const Problem& pr, const Workspace& ws, const void* q, const void* k, const void* v, void* out,
                          const float* kc, const float* vc, const int* kv, const int* full, const int* flat,
                          const uint32_t* mask, const float* ocoarse, int dense) {
  AttnArgs a;
  a.q = q; a.k = k; a.v = v; a.out = out;
  a.kc = kc; a.vc = vc;
  a.blk_start = ws.blk_start; a.blk_n = ws.blk_n;
  a.kv_list = kv; a.full_list = full; a.flat_list = flat;
  a.exact_mask = mask;
  a.ocoarse = (!dense && pr.p.gamma != 0.0) ? ocoarse : nullptr;
  a.gamma = (float)pr.p.gamma;
  a.geo = pr.geo;
  a.cnt = pr.cnt;
  a.dense = dense;
  return a;
}

static int run_attend(const Problem& pr, const Workspace& ws, const AttnArgs& a, const void* v, bool vt_ready,
                      hipStream_t st) {
  const bool mfma = pr.mfma_shape && g_use_mfma.load();
  if (!mfma) {
    ISA_STAGE(launch_attn_simt(pr, a, st));
    return ISA_OK;
  }
  if (!vt_ready) ISA_STAGE(launch_pack_vt(pr, ws, v, nullptr, st));
  if (!a.dense) ISA_STAGE(launch_gather_means(pr, ws, a.kc, a.vc, a.kv_list, st));
  ISA_STAGE(launch_attn_mfma(pr, ws, a, st));
  return ISA_OK;
}

}  // namespace isa

using namespace isa;

extern "C" {

int isa_get_counts(const isa_problem* p, int b, isa_counts* out) {
  if (!out) return ISA_ERR_NULL;
  Problem pr;
  int rc = validate(p, &pr);
  if (rc != ISA_OK) return rc;
  if (b < 0 || b >= p->B) return ISA_ERR_SHAPE;
  const BatchCounts& c = pr.cnt.b[b];
  *out = isa_counts{c.S, c.T, c.T_src, c.T_ctx, c.k_keep, c.T_new, c.n_flat, c.n_full, c.k_exact, pr.cnt.T_max};
  return ISA_OK;
}

size_t isa_workspace_bytes(const isa_problem* p) {
  Problem pr;
  if (validate(p, &pr) != ISA_OK) return 0;
  Workspace ws;
  carve(pr, nullptr, &ws);
  return ws.bytes;
}

int isa_workspace_layout(const isa_problem* p, isa_ws_layout* out) {
  if (!out) return ISA_ERR_NULL;
  Problem pr;
  int rc = validate(p, &pr);
  if (rc != ISA_OK) return rc;
  Workspace ws;
  carve(pr, nullptr, &ws);                              // base 0: every pointer is its own offset
  auto off = [](const void* ptr) { return ptr ? (size_t)(uintptr_t)ptr : ISA_NO_ARRAY; };
  out->bytes = ws.bytes;
  // the first array sits at offset 0, which a null check would take for "absent"
  out->qc = (size_t)(uintptr_t)ws.qc; out->kc = (size_t)(uintptr_t)ws.kc; out->vc = (size_t)(uintptr_t)ws.vc;
  out->s_ctx = (size_t)(uintptr_t)ws.s_ctx; out->sharp = (size_t)(uintptr_t)ws.sharp;
  out->kv_list = (size_t)(uintptr_t)ws.kv_list; out->full_list = (size_t)(uintptr_t)ws.full_list;
  out->flat_list = (size_t)(uintptr_t)ws.flat_list;
  out->exact_mask = off(ws.exact_mask);
  out->o_coarse = off(ws.ocoarse);
  out->nlse = off(ws.nlse);
  return ISA_OK;
}

int isa_block_means(const isa_problem* p, const void* q, const void* k, const void* v, float* qc, float* kc, float* vc,
                    void* workspace, size_t workspace_bytes, void* hip_stream) {
  Problem pr;
  int rc = validate(p, &pr);
  if (rc != ISA_OK) return rc;
  if (!q || !k || !v || !qc || !kc || !vc) return ISA_ERR_NULL;
  if (!all_aligned16(q, k, v, qc, kc, vc)) return ISA_ERR_SHAPE;
  Workspace ws;
  if ((rc = check_ws(pr, workspace, workspace_bytes, &ws)) != ISA_OK) return rc;
  hipStream_t st = (hipStream_t)hip_stream;
  ISA_STAGE(launch_layout(pr, ws, st));
  ISA_STAGE(launch_block_means(pr, ws, q, k, v, qc, kc, vc, st));
  return ISA_OK;
}

int isa_coarse_scores(const isa_problem* p, const float* qc, const float* kc, float* s_ctx, float* sharp, float* z,
                      void* workspace, size_t workspace_bytes, void* hip_stream) {
  Problem pr;
  int rc = validate(p, &pr);
  if (rc != ISA_OK) return rc;
  if (!qc || !kc || !s_ctx || !sharp) return ISA_ERR_NULL;
  Workspace ws;
  if ((rc = check_ws(pr, workspace, workspace_bytes, &ws)) != ISA_OK) return rc;
  hipStream_t st = (hipStream_t)hip_stream;
  ISA_STAGE(launch_coarse(pr, ws, qc, kc, s_ctx, sharp, z, nullptr, nullptr, st));
  return ISA_OK;
}

int isa_coarse_output(const isa_problem* p, const float* qc, const float* kc, const float* vc, float* o_coarse,
                      void* workspace, size_t workspace_bytes, void* hip_stream) {
  Problem pr;
  int rc = validate(p, &pr);
  if (rc != ISA_OK) return rc;
  if (!qc || !kc || !vc || !o_coarse) return ISA_ERR_NULL;
  Workspace ws;
  if ((rc = check_ws(pr, workspace, workspace_bytes, &ws)) != ISA_OK) return rc;
  hipStream_t st = (hipStream_t)hip_stream;
  // the same kernel as isa_coarse_scores; its scores land in the workspace's own arrays
  ISA_STAGE(launch_coarse(pr, ws, qc, kc, ws.s_ctx, ws.sharp, nullptr, vc, o_coarse, st));
  return ISA_OK;
}

int isa_select(const isa_problem* p, const float* s_ctx, const float* sharp, const float* z, int32_t* kv_list,
               int32_t* full_list, int32_t* flat_list, uint32_t* exact_mask, void* workspace, size_t workspace_bytes,
               void* hip_stream) {
  Problem pr;
  int rc = validate(p, &pr);
  if (rc != ISA_OK) return rc;
  if (!s_ctx || !sharp || !kv_list || !full_list || !flat_list) return ISA_ERR_NULL;
  if (p->exact_frac > 0.0 && (!z || !exact_mask)) return ISA_ERR_NULL;
  Workspace ws;
  if ((rc = check_ws(pr, workspace, workspace_bytes, &ws)) != ISA_OK) return rc;
  hipStream_t st = (hipStream_t)hip_stream;
  ISA_STAGE(launch_select(pr, ws, s_ctx, sharp, z, kv_list, full_list, flat_list, exact_mask, st));
  return ISA_OK;
}

int isa_attend(const isa_problem* p, const void* q, const void* k, const void* v, const float* kc, const float* vc,
               const int32_t* kv_list, const int32_t* full_list, const int32_t* flat_list, const uint32_t* exact_mask,
               const float* o_coarse, void* out, void* workspace, size_t workspace_bytes, void* hip_stream) {
  Problem pr;
  int rc = validate(p, &pr);
  if (rc != ISA_OK) return rc;
  if (!q || !k || !v || !kc || !vc || !kv_list || !full_list || !flat_list || !out) return ISA_ERR_NULL;
  if (p->exact_frac > 0.0 && !exact_mask) return ISA_ERR_NULL;
  if (p->gamma != 0.0 && !o_coarse) return ISA_ERR_NULL;
  if (!all_aligned16(q, k, v, out, kc, vc)) return ISA_ERR_SHAPE;
  Workspace ws;
  if ((rc = check_ws(pr, workspace, workspace_bytes, &ws)) != ISA_OK) return rc;
  hipStream_t st = (hipStream_t)hip_stream;
  ISA_STAGE(launch_layout(pr, ws, st));
  AttnArgs a = attn_args(pr, ws, q, k, v, out, kc, vc, kv_list, full_list, flat_list,
                         p->exact_frac > 0.0 ? exact_mask : nullptr, o_coarse, 0);
  return run_attend(pr, ws, a, v, false, st);
}

// Alg. 1, all stages, on a carved workspace (the body of isa_attention and of its allocation-free twin).
static int run_attention(const Problem& pr, const Workspace& ws, const void* q, const void* k, const void* v, void* out,
                         hipStream_t st) {
  ISA_STAGE(launch_layout(pr, ws, st));
  // the matrix-core kernels want a packed V^T copy: the kernel that writes it has every block of V in LDS and writes the
  // block's mean value too, so the block-mean kernel reads Q and K only
  const bool pack_first = pr.mfma_shape && g_use_mfma.load();
  if (pack_first) ISA_STAGE(launch_pack_vt(pr, ws, v, ws.vc, st));
  ISA_STAGE(launch_block_means(pr, ws, q, k, pack_first ? nullptr : v, ws.qc, ws.kc, ws.vc, st));
  ISA_STAGE(launch_coarse(pr, ws, ws.qc, ws.kc, ws.s_ctx, ws.sharp, ws.z, ws.vc, ws.ocoarse, st));
  ISA_STAGE(launch_select(pr, ws, ws.s_ctx, ws.sharp, ws.z, ws.kv_list, ws.full_list, ws.flat_list, ws.exact_mask, st));
  AttnArgs a = attn_args(pr, ws, q, k, v, out, ws.kc, ws.vc, ws.kv_list, ws.full_list, ws.flat_list, ws.exact_mask, ws.ocoarse, 0);
  return run_attend(pr, ws, a, v, pack_first, st);
}

int isa_attention(const isa_problem* p, const void* q, const void* k, const void* v, void* out, void* workspace,
                  size_t workspace_bytes, void* hip_stream) {
  Problem pr;
  int rc = validate(p, &pr);
  if (rc != ISA_OK) return rc;
  if (!q || !k || !v || !out) return ISA_ERR_NULL;
  if (!all_aligned16(q, k, v, out)) return ISA_ERR_SHAPE;
  Workspace ws;
  if ((rc = check_ws(pr, workspace, workspace_bytes, &ws)) != ISA_OK) return rc;
  return run_attention(pr, ws, q, k, v, out, (hipStream_t)hip_stream);
}

// ---- the entry point that allocates nothing and takes no workspace -------------------------------------------------------
// Its scratch is this file-scope device array: every GPU the library's code object is loaded on holds one copy, at its own
// address, until the process ends.  In host code the array's name is only a handle for hipGetSymbolAddress; the device
// address obtained from it (once per device, kept in g_static_ptr) is what kernels and carve() are given.
static __device__ __align__(256) unsigned char scratch[ISA_STATIC_SCRATCH_BYTES];
constexpr int STATIC_MAX_DEVICES = 64;
static void* g_static_ptr[STATIC_MAX_DEVICES];          // device address of `scratch` on each device; null = not asked yet
static std::mutex g_static_mu;

static int static_scratch(void** ptr) {
  int dev = -1;
  ISA_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= STATIC_MAX_DEVICES) return ISA_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_static_mu);
  if (!g_static_ptr[dev]) {
    void* d = nullptr;
    size_t bytes = 0;
    ISA_TRY(hipGetSymbolAddress(&d, HIP_SYMBOL(scratch)));      // of the current device's copy
    ISA_TRY(hipGetSymbolSize(&bytes, HIP_SYMBOL(scratch)));
    if (!d || bytes < (size_t)ISA_STATIC_SCRATCH_BYTES || ((uintptr_t)d & 255)) return ISA_ERR_WORKSPACE;
    g_static_ptr[dev] = d;
  }
  *ptr = g_static_ptr[dev];
  return ISA_OK;
}

int isa_attention_static(const isa_problem* p, const void* q, const void* k, const void* v, void* out, void* hip_stream) {
  Problem pr;
  int rc = validate(p, &pr);
  if (rc != ISA_OK) return rc;
  if (!q || !k || !v || !out) return ISA_ERR_NULL;
  if (!all_aligned16(q, k, v, out)) return ISA_ERR_SHAPE;
  Workspace ws;
  carve(pr, nullptr, &ws, true);                       // the forward pass only: nothing is kept for a backward call
  if (ws.bytes > (size_t)ISA_STATIC_SCRATCH_BYTES) return ISA_ERR_WORKSPACE;
  void* base = nullptr;
  if ((rc = static_scratch(&base)) != ISA_OK) return rc;
  carve(pr, base, &ws, true);
  // every array of the carve-up is written by a kernel of this call before any kernel reads it, so what the previous
  // call left in the scratch does not matter and nothing has to be cleared
  return run_attention(pr, ws, q, k, v, out, (hipStream_t)hip_stream);
}

int isa_dense_attention(const isa_problem* p, const void* q, const void* k, const void* v, void* out, void* workspace,
                        size_t workspace_bytes, void* hip_stream) {
  Problem pr;
  int rc = validate(p, &pr);
  if (rc != ISA_OK) return rc;
  if (!q || !k || !v || !out) return ISA_ERR_NULL;
  if (!all_aligned16(q, k, v, out)) return ISA_ERR_SHAPE;
  Workspace ws;
  if ((rc = check_ws(pr, workspace, workspace_bytes, &ws)) != ISA_OK) return rc;
  hipStream_t st = (hipStream_t)hip_stream;
  ISA_STAGE(launch_layout(pr, ws, st));
  AttnArgs a = attn_args(pr, ws, q, k, v, out, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 1);
  return run_attend(pr, ws, a, v, false, st);
}

int isa_attention_backward(const isa_problem* p, const void* q, const void* k, const void* v, const void* out,
                           const void* d_out, const int32_t* kv_list, const int32_t* full_list,
                           const int32_t* flat_list, const uint32_t* exact_mask, void* dq, void* dk, void* dv,
                           void* workspace, size_t workspace_bytes, void* hip_stream) {
  Problem pr;
  int rc = validate(p, &pr);
  if (rc != ISA_OK) return rc;
  if (!q || !k || !v || !out || !d_out || !dq || !dk || !dv) return ISA_ERR_NULL;
  if (!all_aligned16(q, k, v, out, d_out, dq, dk, dv)) return ISA_ERR_SHAPE;
  const int n_lists = (kv_list != nullptr) + (full_list != nullptr) + (flat_list != nullptr);
  if (n_lists != 0 && n_lists != 3) return ISA_ERR_NULL;
  if (n_lists == 3 && p->exact_frac > 0.0 && !exact_mask) return ISA_ERR_NULL;
  if (!pr.mfma_shape || !g_use_mfma.load()) return ISA_ERR_UNSUPPORTED;
  Workspace ws;
  if ((rc = check_ws(pr, workspace, workspace_bytes, &ws)) != ISA_OK) return rc;
  hipStream_t st = (hipStream_t)hip_stream;
  if (n_lists == 0) {
    kv_list = ws.kv_list; full_list = ws.full_list; flat_list = ws.flat_list;
    exact_mask = ws.exact_mask;
  }
  if (p->exact_frac <= 0.0) exact_mask = nullptr;
  // The log-sum-exp of every query row is what the forward call left in the workspace.  After isa_attention (lists taken
  // from the workspace) the block table, the block means, the gathered mean keys and O_coarse are still there as well;
  // the staged forward takes its means and O_coarse from the caller, so after it they are computed again here.
  if (n_lists != 0) {
    ISA_STAGE(launch_layout(pr, ws, st));
    ISA_STAGE(launch_block_means(pr, ws, q, k, v, ws.qc, ws.kc, ws.vc, st));
    ISA_STAGE(launch_gather_means(pr, ws, ws.kc, ws.vc, kv_list, st));
    if (p->gamma != 0.0)                            // O_coarse of Alg. 1 Stage 1
      ISA_STAGE(launch_coarse(pr, ws, ws.qc, ws.kc, ws.s_ctx, ws.sharp, nullptr, ws.vc, ws.ocoarse, st));
  }
  ISA_STAGE(launch_attn_bwd(pr, ws, q, k, v, out, d_out, kv_list, full_list, flat_list, exact_mask, dq, dk, dv, st));
  return ISA_OK;
}

int isa_attention_simple(const void* q, const void* k, const void* v, int H, int D, int n_src, int n_ctx,
                         double keep_ratio, double full_frac, int block, void* out, void* hip_stream) {
  int32_t seg_ptr[2] = {0, n_ctx > 0 ? 2 : 1};
  int32_t seg_len[2] = {n_src, n_ctx};
  if (n_src < 1 || n_ctx < 0) return ISA_ERR_SHAPE;
  isa_problem p;
  memset(&p, 0, sizeof(p));
  p.B = 1; p.H = H; p.D = D; p.dtype = ISA_BF16; p.block = block;
  p.seg_ptr = seg_ptr; p.seg_len = seg_len;
  p.stride_t = D;
  p.stride_h = (int64_t)D * ((int64_t)n_src + n_ctx);
  p.stride_b = p.stride_h * H;
  p.keep_ratio = keep_ratio; p.full_frac = full_frac; p.exact_frac = 0.0; p.gamma = 0.0;
  Problem pr;
  int rc = validate(&p, &pr);
  if (rc != ISA_OK) return rc;
  if (!q || !k || !v || !out) return ISA_ERR_NULL;
  if (!all_aligned16(q, k, v, out)) return ISA_ERR_SHAPE;
  const size_t bytes = isa_workspace_bytes(&p);
  hipStream_t st = (hipStream_t)hip_stream;
  // it allocates: not for a stream that is being captured into a graph (isa_attention and isa_attention_static are)
  hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
  ISA_TRY(hipStreamIsCapturing(st, &cap));
  if (cap != hipStreamCaptureStatusNone) return ISA_ERR_UNSUPPORTED;
  void* ws = nullptr;
  ISA_TRY(hipMallocAsync(&ws, bytes, st));
  rc = isa_attention(&p, q, k, v, out, ws, bytes, hip_stream);
  hipError_t e = hipFreeAsync(ws, st);
  if (rc == ISA_OK && e != hipSuccess) return hip_fail(e);
  return rc;
}

// Checks an isa_grid against the validated problem.
static int check_grid(const Problem& pr, const isa_grid* g, bool rope) {
  if (!g || !g->seg_grid) return ISA_ERR_NULL;
  const int n_seg = pr.seg.seg_ptr[pr.p.B];
  for (int s = 0; s < n_seg; ++s) {
    const long long t = g->seg_grid[3 * s], h = g->seg_grid[3 * s + 1], w = g->seg_grid[3 * s + 2];
    if (t < 0 || h < 0 || w < 0 || t > 0x7fffffffLL || h > 0x7fffffffLL || w > 0x7fffffffLL) return ISA_ERR_SHAPE;
    if (t * h > 0x7fffffffLL || t * h * w != (long long)pr.seg.seg_len[s]) return ISA_ERR_SHAPE;
  }
  for (int a = 0; a < 3; ++a)
    if (g->tile[a] < 1) return ISA_ERR_SHAPE;
  if (rope) {
    long long sum = 0;
    for (int a = 0; a < 3; ++a) {
      if (g->rope_dims[a] < 0 || g->rope_dims[a] % 2) return ISA_ERR_SHAPE;
      sum += g->rope_dims[a];
    }
    if (sum > pr.p.D) return ISA_ERR_SHAPE;
    if (!(g->rope_theta > 0.0) || !isfinite(g->rope_theta)) return ISA_ERR_UNSUPPORTED;
  }
  return ISA_OK;
}

static int run_prologue(const isa_problem* p, const isa_grid* grid, const void* q_in, const void* k_in, const void* v_in,
                        void* q_out, void* k_out, void* v_out, float* qc, float* kc, float* vc, bool inverse,
                        void* hip_stream) {
  Problem pr;
  int rc = validate(p, &pr);
  if (rc != ISA_OK) return rc;
  if (!q_in || !k_in || !v_in || !q_out || !k_out || !v_out) return ISA_ERR_NULL;
  if ((qc || kc || vc) && !(qc && kc && vc)) return ISA_ERR_NULL;
  if ((rc = check_grid(pr, grid, true)) != ISA_OK) return rc;
  const void* ins[3] = {q_in, k_in, v_in};
  const void* outs[3] = {q_out, k_out, v_out};
  for (int i = 0; i < 3; ++i) {
    if (!aligned16(ins[i]) || !aligned16(outs[i])) return ISA_ERR_SHAPE;
    for (int j = 0; j < 3; ++j)
      if (outs[i] == ins[j] || (i != j && outs[i] == outs[j])) return ISA_ERR_SHAPE;
  }
  hipStream_t st = (hipStream_t)hip_stream;
  ISA_STAGE(launch_prologue(pr, grid, q_in, k_in, v_in, q_out, k_out, v_out, qc, kc, vc, inverse, st));
  return ISA_OK;
}

int isa_prologue(const isa_problem* p, const isa_grid* grid, const void* q_in, const void* k_in, const void* v_in,
                 void* q_out, void* k_out, void* v_out, float* qc, float* kc, float* vc, void* hip_stream) {
  return run_prologue(p, grid, q_in, k_in, v_in, q_out, k_out, v_out, qc, kc, vc, false, hip_stream);
}

int isa_prologue_backward(const isa_problem* p, const isa_grid* grid, const void* dq_out, const void* dk_out,
                          const void* dv_out, void* dq_in, void* dk_in, void* dv_in, void* hip_stream) {
  return run_prologue(p, grid, dq_out, dk_out, dv_out, dq_in, dk_in, dv_in, nullptr, nullptr, nullptr, true, hip_stream);
}

int isa_untile(const isa_problem* p, const isa_grid* grid, const void* x_tiled, void* x_raster, void* hip_stream) {
  Problem pr;
  int rc = validate(p, &pr);
  if (rc != ISA_OK) return rc;
  if (!x_tiled || !x_raster) return ISA_ERR_NULL;
  if ((rc = check_grid(pr, grid, false)) != ISA_OK) return rc;
  if (!aligned16(x_tiled) || !aligned16(x_raster) || x_tiled == x_raster) return ISA_ERR_SHAPE;
  hipStream_t st = (hipStream_t)hip_stream;
  ISA_STAGE(launch_untile(pr, grid, x_tiled, x_raster, st));
  return ISA_OK;
}

const char* isa_strerror(int status) {
  switch (status) {
    case ISA_OK: return "ISA_OK";
    case ISA_ERR_NULL: return "ISA_ERR_NULL: a required pointer is NULL";
    case ISA_ERR_SHAPE: return "ISA_ERR_SHAPE: unsupported shape, segments or strides";
    case ISA_ERR_RATIO: return "ISA_ERR_RATIO: ratio outside [0, 1]";
    case ISA_ERR_DTYPE: return "ISA_ERR_DTYPE: unknown dtype";
    case ISA_ERR_UNSUPPORTED: return "ISA_ERR_UNSUPPORTED: not available for this problem or in this state (see isa.h)";
    case ISA_ERR_WORKSPACE: return "ISA_ERR_WORKSPACE: workspace missing, misaligned or too small";
    case ISA_ERR_HIP: return "ISA_ERR_HIP: a HIP call failed (see isa_last_hip_error)";
    default: return "unknown isa_status";
  }
}

int isa_last_hip_error(void) { return g_last_hip; }

int isa_set_mfma(int enabled) { return g_use_mfma.exchange(enabled ? 1 : 0); }

int isa_time_attention_kernel(int enabled) {
  if (enabled && !isa::g_prof_start) {
    ISA_TRY(hipEventCreate(&isa::g_prof_start));
    ISA_TRY(hipEventCreate(&isa::g_prof_stop));
  }
  isa::g_prof_on = enabled ? 1 : 0;
  return ISA_OK;
}

int isa_last_attention_kernel_ms(float* ms) {
  if (!ms) return ISA_ERR_NULL;
  if (!isa::g_prof_recorded) return ISA_ERR_UNSUPPORTED;
  ISA_TRY(hipEventSynchronize(isa::g_prof_stop));
  ISA_TRY(hipEventElapsedTime(ms, isa::g_prof_start, isa::g_prof_stop));
  return ISA_OK;
}

}  // extern "C"
