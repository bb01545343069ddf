// gfx950 kernel: rotary position embedding of a pass's query rows and new key rows,
// in place, at their absolute positions (the step of the scorer's attention layer
// that precedes the append into the cache and the attention itself).
//
//   theta_i = base^(-2 i / D), i = 0 .. D/2 - 1;  a row at position p turns every pair
//   (x_i, x_{i + D/2}) by the angle p * theta_i   (RoFormer, Sec. 3.2 / 3.4.2, in the
//   half-split pairing of the Llama / Qwen model families).
//
// Bound by HBM: every row is read and written once (bf16).  Angles are formed and
// reduced in double precision (positions reach tens of thousands of radians for the
// fastest pair), the rotation itself is fp32 on bf16 inputs with one rounding to bf16.
#include <hip/hip_runtime.h>

#include "oppo_internal.h"

namespace oppo {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

constexpr int kRopeTok = 8;          // tokens per workgroup
constexpr int kMaxRopeItems = 1000;  // 1000 * 12 B + header in the kernel arguments
constexpr int kMaxQkvItems = 1000;   // 1000 * 24 B + header

struct RopeParams {
  uint16_t* q;      // [rows][Hq][D], may be null
  uint16_t* k;      // [rows][Hkv][D], may be null
  double log2_base;
  int32_t Hq, Hkv;
  int32_t n_items;
  RopeItem items[kMaxRopeItems];
};
static_assert(sizeof(RopeParams) <= 32768, "kernel arguments are kept within 32 KiB");

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  bf16x2 p;
  p[0] = (__bf16)a;   // round to nearest even
  p[1] = (__bf16)b;
  return *(uint32_t*)&p;
}

// grid = (items, pieces of kRopeTok tokens); 256 threads.
template <int D>
__global__ __launch_bounds__(256) void rope_kernel(const RopeParams P) {
  constexpr int HALF = D / 2;
  constexpr int UPH = HALF / 8;   // 16-byte units per half head
  __shared__ float cs[kRopeTok][HALF][2];
  const RopeItem it = P.items[blockIdx.x];
  const int tok0 = blockIdx.y * kRopeTok;
  if (tok0 >= it.n_tok) return;
  const int ntok = min(kRopeTok, it.n_tok - tok0);
  for (int e = threadIdx.x; e < ntok * HALF; e += 256) {
    const int t = e / HALF, i = e % HALF;
    const double theta = exp2(-(2.0 * i / D) * P.log2_base);
    double s, c;
    sincos((double)(it.pos0 + tok0 + t) * theta, &s, &c);
    cs[t][i][0] = (float)c;
    cs[t][i][1] = (float)s;
  }
  __syncthreads();
  // a unit = 8 pairs of one head: 16 bytes from each half of the head's row
  const int heads = (P.q ? P.Hq : 0) + (P.k ? P.Hkv : 0);
  const int units = ntok * heads * UPH;
  for (int u = threadIdx.x; u < units; u += 256) {
    const int g = u % UPH;
    const int h = (u / UPH) % heads;
    const int t = u / (UPH * heads);
    const int64_t row = (int64_t)it.row0 + tok0 + t;
    const int hq = P.q ? P.Hq : 0;
    uint16_t* base = h < hq ? P.q + (row * P.Hq + h) * D : P.k + (row * P.Hkv + (h - hq)) * D;
    u32x4* pa = (u32x4*)(base + g * 8);
    u32x4* pb = (u32x4*)(base + HALF + g * 8);
    const u32x4 a = *pa, b = *pb;
    u32x4 ra, rb;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float c0 = cs[t][g * 8 + 2 * w][0], s0 = cs[t][g * 8 + 2 * w][1];
      const float c1 = cs[t][g * 8 + 2 * w + 1][0], s1 = cs[t][g * 8 + 2 * w + 1][1];
      const float a0 = bf16_lo(a[w]), a1 = bf16_hi(a[w]), b0 = bf16_lo(b[w]), b1 = bf16_hi(b[w]);
      ra[w] = pack_bf16(a0 * c0 - b0 * s0, a1 * c1 - b1 * s1);
      rb[w] = pack_bf16(b0 * c0 + a0 * s0, b1 * c1 + a1 * s1);
    }
    *pa = ra;
    *pb = rb;
  }
}

// ---------------------------------------------------------------------------------
// The same rotation as the epilogue of the layer's fused QKV projection: one pass over
// the projection's output rows [q heads | k heads | v heads] writes the rotated queries
// to their own array and the rotated keys and the values straight into the cache slabs.
struct QkvParams {
  const uint16_t* qkv;   // [rows][Hq + 2 Hkv][D]
  uint16_t* q_out;       // [rows][Hq][D]
  uint16_t* cache_k;     // [slots][Hkv][D]
  uint16_t* cache_v;
  double log2_base;
  int32_t Hq, Hkv;
  int32_t n_items;
  QkvItem items[kMaxQkvItems];
};
static_assert(sizeof(QkvParams) <= 32768, "kernel arguments are kept within 32 KiB");

template <int D>
__global__ __launch_bounds__(256) void qkv_rope_append_kernel(const QkvParams P) {
  constexpr int HALF = D / 2;
  constexpr int UPH = HALF / 8;
  __shared__ float cs[kRopeTok][HALF][2];
  const QkvItem it = P.items[blockIdx.x];
  const int tok0 = blockIdx.y * kRopeTok;
  if (tok0 >= it.n_tok) return;
  const int ntok = min(kRopeTok, it.n_tok - tok0);
  for (int e = threadIdx.x; e < ntok * HALF; e += 256) {
    const int t = e / HALF, i = e % HALF;
    const double theta = exp2(-(2.0 * i / D) * P.log2_base);
    double s, c;
    sincos((double)(it.pos0 + tok0 + t) * theta, &s, &c);
    cs[t][i][0] = (float)c;
    cs[t][i][1] = (float)s;
  }
  __syncthreads();
  const int heads = P.Hq + 2 * P.Hkv;
  const int units = ntok * heads * UPH;
  for (int u = threadIdx.x; u < units; u += 256) {
    const int g = u % UPH;
    const int h = (u / UPH) % heads;
    const int t = u / (UPH * heads);
    const int64_t src_row = (int64_t)it.src_row + tok0 + t;
    const int64_t dst_row = it.dst_row + tok0 + t;
    const uint16_t* src = P.qkv + (src_row * heads + h) * D;
    const u32x4 a = *(const u32x4*)(src + g * 8), b = *(const u32x4*)(src + HALF + g * 8);
    uint16_t* dst;
    if (h < P.Hq) {
      dst = P.q_out + (src_row * P.Hq + h) * D;
    } else if (h < P.Hq + P.Hkv) {
      dst = P.cache_k + (dst_row * P.Hkv + (h - P.Hq)) * D;
    } else {
      dst = P.cache_v + (dst_row * P.Hkv + (h - P.Hq - P.Hkv)) * D;
      *(u32x4*)(dst + g * 8) = a;            // values are copied as they are
      *(u32x4*)(dst + HALF + g * 8) = b;
      continue;
    }
    u32x4 ra, rb;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float c0 = cs[t][g * 8 + 2 * w][0], s0 = cs[t][g * 8 + 2 * w][1];
      const float c1 = cs[t][g * 8 + 2 * w + 1][0], s1 = cs[t][g * 8 + 2 * w + 1][1];
      const float a0 = bf16_lo(a[w]), a1 = bf16_hi(a[w]), b0 = bf16_lo(b[w]), b1 = bf16_hi(b[w]);
      ra[w] = pack_bf16(a0 * c0 - b0 * s0, a1 * c1 - b1 * s1);
      rb[w] = pack_bf16(b0 * c0 + a0 * s0, b1 * c1 + a1 * s1);
    }
    *(u32x4*)(dst + g * 8) = ra;
    *(u32x4*)(dst + HALF + g * 8) = rb;
  }
}

int launch_qkv_rope_append(const LayerShape& ls, const void* qkv, void* q_out, void* cache_k, void* cache_v,
                           const QkvItem* items, int n_items, double theta_base, void* stream) {
  hipStream_t st = (hipStream_t)stream;
  for (int base = 0; base < n_items; base += kMaxQkvItems) {
    QkvParams P;
    P.qkv = (const uint16_t*)qkv;
    P.q_out = (uint16_t*)q_out;
    P.cache_k = (uint16_t*)cache_k;
    P.cache_v = (uint16_t*)cache_v;
    P.log2_base = log2(theta_base);
    P.Hq = ls.Hq;
    P.Hkv = ls.Hkv;
    const int n = n_items - base < kMaxQkvItems ? n_items - base : kMaxQkvItems;
    P.n_items = n;
    int mt = 0;
    for (int i = 0; i < n; ++i) {
      P.items[i] = items[base + i];
      if (items[base + i].n_tok > mt) mt = items[base + i].n_tok;
    }
    dim3 grid((unsigned)n, (unsigned)((mt + kRopeTok - 1) / kRopeTok)), block(256);
    if (ls.D == 128)
      hipLaunchKernelGGL(qkv_rope_append_kernel<128>, grid, block, 0, st, P);
    else
      hipLaunchKernelGGL(qkv_rope_append_kernel<64>, grid, block, 0, st, P);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return (int)e;
  }
  return 0;
}

int launch_rope(const LayerShape& ls, void* q, void* k, const RopeItem* items, int n_items, double theta_base,
                void* stream) {
  hipStream_t st = (hipStream_t)stream;
  for (int base = 0; base < n_items; base += kMaxRopeItems) {
    RopeParams P;
    P.q = (uint16_t*)q;
    P.k = (uint16_t*)k;
    P.log2_base = log2(theta_base);
    P.Hq = ls.Hq;
    P.Hkv = ls.Hkv;
    const int n = n_items - base < kMaxRopeItems ? n_items - base : kMaxRopeItems;
    P.n_items = n;
    int mt = 0;
    for (int i = 0; i < n; ++i) {
      P.items[i] = items[base + i];
      if (items[base + i].n_tok > mt) mt = items[base + i].n_tok;
    }
    dim3 grid((unsigned)n, (unsigned)((mt + kRopeTok - 1) / kRopeTok)), block(256);
    if (ls.D == 128)
      hipLaunchKernelGGL(rope_kernel<128>, grid, block, 0, st, P);
    else
      hipLaunchKernelGGL(rope_kernel<64>, grid, block, 0, st, P);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return (int)e;
  }
  return 0;
}

}  // namespace oppo
