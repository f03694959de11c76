// Portable attention kernels in fp32 arithmetic: exact online-softmax attention (Alg. 2 Part A) and
// block-wise 0-th order Taylor attention (Sec. 3, Eq. 3-4; Alg. 2 Parts A+B).  They serve the fp32
// checking mode and every shape the MFMA kernels do not cover.  One workgroup handles 64 query rows
// of one query block; four lanes share a query, each owning every fourth group of 4 channels.
#include "isa_internal.h"

namespace isa {

constexpr int QB = 64;    // query rows per workgroup
constexpr int KT = 32;    // key slots per LDS tile

template <typename T> __device__ inline float4 load4(const T* p);
template <> __device__ inline float4 load4<float>(const float* p) { return *reinterpret_cast<const float4*>(p); }
template <> __device__ inline float4 load4<uint16_t>(const uint16_t* p) {
  const uint2 v = *reinterpret_cast<const uint2*>(p);
  return make_float4(__uint_as_float(v.x << 16), __uint_as_float(v.x & 0xffff0000u), __uint_as_float(v.y << 16),
                     __uint_as_float(v.y & 0xffff0000u));
}
__device__ inline void store4(float* p, float4 v) { *reinterpret_cast<float4*>(p) = v; }
__device__ inline void store4(uint16_t* p, float4 v) {
  auto rne = [](float f) -> uint32_t {          // fp32 -> bf16, round to nearest even
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
  };
  uint2 o;
  o.x = rne(v.x) | (rne(v.y) << 16);
  o.y = rne(v.z) | (rne(v.w) << 16);
  *reinterpret_cast<uint2*>(p) = o;
}

template <typename T, int D>
__global__ __launch_bounds__(256) void k_attn_simt(AttnArgs a) {
  constexpr int G = D / 16;                 // float4 groups owned by a lane
  __shared__ float Ks[KT][D];
  __shared__ float Vs[KT][D];
  __shared__ float Ws[KT];                  // weight of each slot: 1 token, n_j block mean, 0 unused

  const int h = blockIdx.y, b = blockIdx.z;
  const int subs = a.geo.block / QB;
  const int slot = blockIdx.x / subs, sub = blockIdx.x % subs;
  const BatchCounts c = a.cnt.b[b];
  const int T_max = a.geo.T_max;
  if (slot >= c.T) return;
  const long long bh = (long long)b * a.geo.H + h;

  // which query block, and how it is evaluated
  int qi, n_kv;
  bool taylor = false;
  const int* kvl = nullptr;
  if (a.dense) {
    qi = slot;
    n_kv = c.T;
  } else {
    kvl = a.kv_list + bh * T_max;
    n_kv = c.T_new;
    if (slot < c.n_full) qi = block_in_range(a.full_list[bh * T_max + slot], c.T);
    else { qi = block_in_range(a.flat_list[bh * T_max + slot - c.n_full], c.T); taylor = true; }
  }
  const uint32_t* mrow = (taylor && a.exact_mask && c.k_exact > 0)
                             ? a.exact_mask + (bh * T_max + (slot - c.n_full)) * a.cnt.mask_words : nullptr;
  const int n_q = a.blk_n[b * T_max + qi];
  if (sub * QB >= n_q) return;
  const int q_start = a.blk_start[b * T_max + qi];

  const int ql = threadIdx.x >> 2, part = threadIdx.x & 3;
  const int row = sub * QB + ql;
  const bool row_ok = row < n_q;
  const long long tbase = (long long)b * a.geo.stride_b + (long long)h * a.geo.stride_h;
  const T* qp = (const T*)a.q + tbase + (long long)(q_start + (row_ok ? row : 0)) * a.geo.stride_t;

  float4 qr[G], o[G];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    qr[g] = load4<T>(qp + (g * 4 + part) * 4);
    o[g] = make_float4(0.f, 0.f, 0.f, 0.f);
  }
  float m = -INFINITY, l = 0.f;
  const float scale = 1.0f / sqrtf((float)D);

  // consume the nk slots currently staged in LDS
  auto consume = [&](int nk) {
    float s[KT];
    float tmax = -INFINITY;
#pragma unroll
    for (int kk = 0; kk < KT; ++kk) {
      float acc = 0.f;
      if (kk < nk) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
          const float4 kv = *reinterpret_cast<const float4*>(&Ks[kk][(g * 4 + part) * 4]);
          acc = fmaf(qr[g].x, kv.x, acc);
          acc = fmaf(qr[g].y, kv.y, acc);
          acc = fmaf(qr[g].z, kv.z, acc);
          acc = fmaf(qr[g].w, kv.w, acc);
        }
      }
      acc += __shfl_xor(acc, 1, 64);
      acc += __shfl_xor(acc, 2, 64);
      s[kk] = acc * scale;
      if (kk < nk && Ws[kk] > 0.f) tmax = fmaxf(tmax, s[kk]);
    }
    if (tmax == -INFINITY) return;             // nothing live in this tile (uniform per 4-lane group)
    const float m_new = fmaxf(m, tmax);
    const float alpha = expf(m - m_new);       // m = -inf -> 0
    l *= alpha;
#pragma unroll
    for (int g = 0; g < G; ++g) { o[g].x *= alpha; o[g].y *= alpha; o[g].z *= alpha; o[g].w *= alpha; }
    m = m_new;
#pragma unroll
    for (int kk = 0; kk < KT; ++kk) {
      if (kk < nk) {
        const float w = Ws[kk];
        if (w > 0.f) {
          const float p = w * expf(s[kk] - m);
          l += p;
#pragma unroll
          for (int g = 0; g < G; ++g) {
            const float4 vv = *reinterpret_cast<const float4*>(&Vs[kk][(g * 4 + part) * 4]);
            o[g].x = fmaf(p, vv.x, o[g].x);
            o[g].y = fmaf(p, vv.y, o[g].y);
            o[g].z = fmaf(p, vv.z, o[g].z);
            o[g].w = fmaf(p, vv.w, o[g].w);
          }
        }
      }
    }
  };

  // Part A: blocks evaluated token by token
  for (int t = 0; t < n_kv; ++t) {
    if (taylor && !(mrow && ((mrow[t >> 5] >> (t & 31)) & 1u))) continue;
    const int j = a.dense ? t : block_in_range(kvl[t], c.T);
    const int n_j = a.blk_n[b * T_max + j];
    const int k_start = a.blk_start[b * T_max + j];
    for (int k0 = 0; k0 < n_j; k0 += KT) {
      const int nk = min(KT, n_j - k0);
      __syncthreads();
      for (int x = threadIdx.x; x < nk * (D / 4); x += 256) {
        const int r = x / (D / 4), c4 = x % (D / 4);
        const long long off = tbase + (long long)(k_start + k0 + r) * a.geo.stride_t + c4 * 4;
        store4(&Ks[r][c4 * 4], load4<T>((const T*)a.k + off));
        store4(&Vs[r][c4 * 4], load4<T>((const T*)a.v + off));
      }
      if (threadIdx.x < KT) Ws[threadIdx.x] = threadIdx.x < nk ? 1.f : 0.f;
      __syncthreads();
      consume(nk);
    }
  }
  // Part B: every other block of kv_list through its mean key, mean value and token count
  if (taylor) {
    for (int t0 = 0; t0 < n_kv; t0 += KT) {
      const int nk = min(KT, n_kv - t0);
      __syncthreads();
      for (int x = threadIdx.x; x < nk * (D / 4); x += 256) {
        const int r = x / (D / 4), c4 = x % (D / 4);
        const long long off = (bh * T_max + block_in_range(kvl[t0 + r], c.T)) * D + c4 * 4;
        store4(&Ks[r][c4 * 4], *reinterpret_cast<const float4*>(a.kc + off));
        store4(&Vs[r][c4 * 4], *reinterpret_cast<const float4*>(a.vc + off));
      }
      if (threadIdx.x < KT) {
        float w = 0.f;
        if (threadIdx.x < nk) {
          const int t = t0 + threadIdx.x;
          const bool exact = mrow && ((mrow[t >> 5] >> (t & 31)) & 1u);
          w = exact ? 0.f : (float)a.blk_n[b * T_max + block_in_range(kvl[t], c.T)];
        }
        Ws[threadIdx.x] = w;
      }
      __syncthreads();
      consume(nk);
    }
  }

  if (row_ok) {
    const float inv = 1.0f / l;
    T* op = (T*)a.out + tbase + (long long)(q_start + row) * a.geo.stride_t;
    // coarse residual (Alg. 1 Stage 5): the block's row of O_coarse, the same for all of its tokens
    const float* oc = (a.ocoarse && !a.dense) ? a.ocoarse + (bh * T_max + qi) * D : nullptr;
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float4 r = make_float4(o[g].x * inv, o[g].y * inv, o[g].z * inv, o[g].w * inv);
      if (oc) {
        const float4 c4 = *reinterpret_cast<const float4*>(oc + (g * 4 + part) * 4);
        r.x = fmaf(a.gamma, c4.x, r.x); r.y = fmaf(a.gamma, c4.y, r.y);
        r.z = fmaf(a.gamma, c4.z, r.z); r.w = fmaf(a.gamma, c4.w, r.w);
      }
      store4(op + (g * 4 + part) * 4, r);
    }
  }
}

hipError_t launch_attn_simt(const Problem& pr, const AttnArgs& a, hipStream_t st) {
  const dim3 grid(pr.cnt.T_max * (pr.p.block / QB), pr.p.H, pr.p.B), blk(256);
  if (pr.p.dtype == ISA_BF16) {
    if (pr.p.D == 128) hipLaunchKernelGGL((k_attn_simt<uint16_t, 128>), grid, blk, 0, st, a);
    else hipLaunchKernelGGL((k_attn_simt<uint16_t, 64>), grid, blk, 0, st, a);
  } else {
    if (pr.p.D == 128) hipLaunchKernelGGL((k_attn_simt<float, 128>), grid, blk, 0, st, a);
    else hipLaunchKernelGGL((k_attn_simt<float, 64>), grid, blk, 0, st, a);
  }
  return hipGetLastError();
}

}  // namespace isa
