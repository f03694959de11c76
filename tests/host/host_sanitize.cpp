// Host-side checks of the C ABI, meant to be built with -fsanitize=address,undefined on the host code of isa_api.hip
// (tests/test_host_sanitized.py does that).  Every call here ends in the library's own argument checks or in host-only
// arithmetic: no kernel is launched and no GPU is needed.
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

#include "isa.h"

static int failures = 0;
#define EXPECT(cond)                                                     \
  do {                                                                   \
    if (!(cond)) { printf("FAILED %s:%d: %s\n", __FILE__, __LINE__, #cond); ++failures; } \
  } while (0)

static isa_problem make(int B, int H, int D, int dtype, int block, const int32_t* seg_ptr, const int32_t* seg_len, long S_max) {
  isa_problem p;
  memset(&p, 0, sizeof(p));
  p.B = B; p.H = H; p.D = D; p.dtype = dtype; p.block = block;
  p.seg_ptr = seg_ptr; p.seg_len = seg_len;
  p.stride_t = D; p.stride_h = (int64_t)D * S_max; p.stride_b = p.stride_h * H;
  p.keep_ratio = 0.5; p.full_frac = 0.25; p.exact_frac = 0.0; p.gamma = 0.0;
  return p;
}

int main() {
  // ---- counts, workspace size and layout over a spread of shapes, up to the limits of the header
  {
    std::vector<int32_t> seg_len(ISA_MAX_SEGMENTS), seg_ptr(ISA_MAX_BATCH + 1);
    for (int trial = 0; trial < 200; ++trial) {
      srand(trial);
      const int B = 1 + rand() % ISA_MAX_BATCH;
      int used = 0;
      long S_max = 0;
      seg_ptr[0] = 0;
      for (int b = 0; b < B; ++b) {
        const int room = ISA_MAX_SEGMENTS - used - (B - 1 - b);
        const int n = 1 + rand() % (room < 4 ? room : 4);
        long S = 0;
        for (int s = 0; s < n; ++s) {
          seg_len[used + s] = (s == 0 ? 1 : 0) + rand() % 5000;
          S += seg_len[used + s];
        }
        used += n;
        seg_ptr[b + 1] = used;
        S_max = S > S_max ? S : S_max;
      }
      const int D = (rand() & 1) ? 64 : 128, block = (rand() & 1) ? 64 : 128, dtype = rand() & 1;
      isa_problem p = make(B, 1 + rand() % 48, D, dtype, block, seg_ptr.data(), seg_len.data(), S_max);
      p.keep_ratio = (rand() % 101) / 100.0; p.full_frac = (rand() % 101) / 100.0;
      p.exact_frac = (rand() % 3 == 0) ? (rand() % 101) / 100.0 : 0.0;
      p.gamma = (rand() % 3 == 0) ? 0.5 : 0.0;
      isa_ws_layout lay;
      const int rc = isa_workspace_layout(&p, &lay);
      EXPECT(rc == ISA_OK);
      EXPECT(isa_workspace_bytes(&p) == lay.bytes && lay.bytes > 0);
      EXPECT(lay.kv_list < lay.bytes && lay.full_list < lay.bytes && lay.flat_list < lay.bytes && lay.vc < lay.bytes);
      EXPECT((lay.exact_mask == ISA_NO_ARRAY) == (p.exact_frac == 0.0));
      EXPECT((lay.o_coarse == ISA_NO_ARRAY) == (p.gamma == 0.0));
      for (int b = 0; b < B; ++b) {
        isa_counts c;
        EXPECT(isa_get_counts(&p, b, &c) == ISA_OK);
        EXPECT(c.T == c.T_src + c.T_ctx && c.T_new == c.T_src + c.k_keep && c.n_full + c.n_flat == c.T);
        EXPECT(c.k_keep >= 0 && c.k_keep <= c.T_ctx && c.k_exact >= 0 && c.k_exact <= c.T_new && c.T <= c.T_max);
      }
      isa_counts c;
      EXPECT(isa_get_counts(&p, B, &c) == ISA_ERR_SHAPE && isa_get_counts(&p, -1, &c) == ISA_ERR_SHAPE);
    }
  }
  // ---- the limits themselves
  {
    int32_t seg_ptr[2] = {0, 1}, seg_len[1] = {ISA_MAX_BLOCKS * 128};
    isa_problem p = make(1, 1, 128, ISA_BF16, 128, seg_ptr, seg_len, seg_len[0]);
    p.exact_frac = 0.01;
    isa_counts c;
    EXPECT(isa_get_counts(&p, 0, &c) == ISA_OK && c.T == ISA_MAX_BLOCKS);
    EXPECT(isa_workspace_bytes(&p) > 0);
    seg_len[0] += 1;
    EXPECT(isa_get_counts(&p, 0, &c) == ISA_ERR_SHAPE && isa_workspace_bytes(&p) == 0);
    std::vector<int32_t> many(ISA_MAX_SEGMENTS + 1, 64);
    int32_t ptr2[2] = {0, ISA_MAX_SEGMENTS + 1};
    isa_problem p2 = make(1, 1, 64, ISA_F32, 64, ptr2, many.data(), 64 * (ISA_MAX_SEGMENTS + 1));
    EXPECT(isa_get_counts(&p2, 0, &c) == ISA_ERR_SHAPE);
    ptr2[1] = ISA_MAX_SEGMENTS;
    EXPECT(isa_get_counts(&p2, 0, &c) == ISA_OK && c.T == ISA_MAX_SEGMENTS);
    int32_t bad_ptr[3] = {0, 2, 1};                       // not ascending
    isa_problem p3 = make(2, 1, 64, ISA_F32, 64, bad_ptr, many.data(), 128);
    EXPECT(isa_get_counts(&p3, 0, &c) == ISA_ERR_SHAPE);
    int32_t off_ptr[2] = {1, 2};                          // does not start at 0
    isa_problem p4 = make(1, 1, 64, ISA_F32, 64, off_ptr, many.data(), 64);
    EXPECT(isa_get_counts(&p4, 0, &c) == ISA_ERR_SHAPE);
  }
  // ---- every entry point refuses bad arguments before it touches the GPU
  {
    int32_t seg_ptr[2] = {0, 2}, seg_len[2] = {512, 512};
    isa_problem p = make(1, 2, 128, ISA_BF16, 128, seg_ptr, seg_len, 1024);
    void* a = (void*)(uintptr_t)4096;                     // aligned, never dereferenced
    void* odd = (void*)(uintptr_t)4104;
    const size_t big = (size_t)1 << 40;
    EXPECT(isa_attention(nullptr, a, a, a, a, a, big, nullptr) == ISA_ERR_NULL);
    EXPECT(isa_attention(&p, a, a, a, nullptr, a, big, nullptr) == ISA_ERR_NULL);
    EXPECT(isa_attention(&p, a, a, a, a, nullptr, big, nullptr) == ISA_ERR_WORKSPACE);
    EXPECT(isa_attention(&p, a, a, a, a, a, 1024, nullptr) == ISA_ERR_WORKSPACE);
    EXPECT(isa_attention(&p, a, odd, a, a, a, big, nullptr) == ISA_ERR_SHAPE);
    EXPECT(isa_attention_static(&p, a, a, nullptr, a, nullptr) == ISA_ERR_NULL);
    EXPECT(isa_dense_attention(&p, a, a, a, a, odd, big, nullptr) == ISA_ERR_WORKSPACE);
    EXPECT(isa_block_means(&p, a, a, a, nullptr, (float*)a, (float*)a, a, big, nullptr) == ISA_ERR_NULL);
    EXPECT(isa_coarse_scores(&p, (float*)a, nullptr, (float*)a, (float*)a, nullptr, a, big, nullptr) == ISA_ERR_NULL);
    EXPECT(isa_select(&p, (float*)a, (float*)a, nullptr, nullptr, (int32_t*)a, (int32_t*)a, nullptr, a, big, nullptr) == ISA_ERR_NULL);
    isa_problem px = p;
    px.exact_frac = 0.25;
    EXPECT(isa_select(&px, (float*)a, (float*)a, nullptr, (int32_t*)a, (int32_t*)a, (int32_t*)a, nullptr, a, big, nullptr) == ISA_ERR_NULL);
    EXPECT(isa_attend(&px, a, a, a, (float*)a, (float*)a, (int32_t*)a, (int32_t*)a, (int32_t*)a, nullptr, nullptr, a, a, big, nullptr) == ISA_ERR_NULL);
    EXPECT(isa_attention_backward(&p, a, a, a, a, a, (int32_t*)a, nullptr, nullptr, nullptr, a, a, a, a, big, nullptr) == ISA_ERR_NULL);
    EXPECT(isa_attention_backward(&p, a, a, a, a, a, nullptr, nullptr, nullptr, nullptr, a, a, a, a, 16, nullptr) == ISA_ERR_WORKSPACE);
    EXPECT(isa_attention_simple(a, a, a, 2, 128, 0, 10, 0.5, 0.5, 128, a, nullptr) == ISA_ERR_SHAPE);
    EXPECT(isa_attention_simple(a, a, a, 2, 128, 10, -1, 0.5, 0.5, 128, a, nullptr) == ISA_ERR_SHAPE);
    EXPECT(isa_attention_simple(a, a, a, 2, 96, 10, 10, 0.5, 0.5, 128, a, nullptr) == ISA_ERR_SHAPE);
    isa_problem pr = p;
    pr.keep_ratio = nan("");
    EXPECT(isa_attention(&pr, a, a, a, a, a, big, nullptr) == ISA_ERR_RATIO);
    pr = p; pr.gamma = INFINITY;
    EXPECT(isa_attention(&pr, a, a, a, a, a, big, nullptr) == ISA_ERR_UNSUPPORTED);
    pr = p; pr.dtype = 7;
    EXPECT(isa_attention(&pr, a, a, a, a, a, big, nullptr) == ISA_ERR_DTYPE);
    // prologue: grids
    int32_t grid_ok[6] = {4, 8, 16, 4, 8, 16}, grid_bad[6] = {4, 8, 16, 4, 8, 15};
    isa_grid g;
    memset(&g, 0, sizeof(g));
    g.seg_grid = grid_ok; g.tile[0] = 2; g.tile[1] = 4; g.tile[2] = 8;
    g.rope_dims[0] = 44; g.rope_dims[1] = 42; g.rope_dims[2] = 42; g.rope_theta = 10000.0;
    void* b2 = (void*)(uintptr_t)8192; void* c2 = (void*)(uintptr_t)12288;
    void* d2 = (void*)(uintptr_t)16384; void* e2 = (void*)(uintptr_t)20480; void* f2 = (void*)(uintptr_t)24576;
    EXPECT(isa_prologue(&p, &g, a, b2, c2, d2, e2, nullptr, nullptr, nullptr, nullptr, nullptr) == ISA_ERR_NULL);
    EXPECT(isa_prologue(&p, &g, a, b2, c2, a, e2, f2, nullptr, nullptr, nullptr, nullptr) == ISA_ERR_SHAPE);
    g.seg_grid = grid_bad;
    EXPECT(isa_prologue(&p, &g, a, b2, c2, d2, e2, f2, nullptr, nullptr, nullptr, nullptr) == ISA_ERR_SHAPE);
    g.seg_grid = grid_ok; g.rope_dims[0] = 46;
    EXPECT(isa_prologue(&p, &g, a, b2, c2, d2, e2, f2, nullptr, nullptr, nullptr, nullptr) == ISA_ERR_SHAPE);
    g.rope_dims[0] = 44; g.rope_theta = -1.0;
    EXPECT(isa_prologue_backward(&p, &g, a, b2, c2, d2, e2, f2, nullptr) == ISA_ERR_UNSUPPORTED);
    EXPECT(isa_untile(&p, &g, a, a, nullptr) == ISA_ERR_SHAPE);
    EXPECT(isa_untile(&p, nullptr, a, b2, nullptr) == ISA_ERR_NULL);
  }
  for (int s = 1; s >= -9; --s) EXPECT(isa_strerror(s) != nullptr && strlen(isa_strerror(s)) > 0);
  float ms = 0.f;
  EXPECT(isa_last_attention_kernel_ms(nullptr) == ISA_ERR_NULL);
  (void)ms;
  printf("%s (%d failures)\n", failures ? "FAILED" : "host checks ok", failures);
  return failures ? 1 : 0;
}
