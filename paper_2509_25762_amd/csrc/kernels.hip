// gfx950 kernels: ragged chunked-prefill attention, split-KV merge, KV append.
//
// Attention (per workgroup = one AttnItem x one kv-head), 4 waves of 64 lanes:
//   * the query tile packs TM tokens x G q-heads of the kv-head into 256 rows;
//     wave w owns rows [64w, 64w+64).  The transposed product S^T = K Q^T is
//     computed with v_mfma_f32_32x32x16_bf16 (K as the A operand from LDS, Q^T
//     as the B operand held in registers), so one lane owns one query column:
//     the softmax statistics are per-lane scalars and the probabilities land
//     in the B-operand layout of the second product O^T = V^T P^T without any
//     cross-lane movement.  V^T fragments come from the token-major V tile in
//     LDS through the transposing LDS read (ds_read_b64_tr_b16).
//   * keys are streamed in tiles of 64 with an online softmax (running max and
//     sum in fp32, exp2 domain with the scale folded in).
//   * causal mask aligned to the end of the cache: the tile's token t at
//     absolute position pos0+t sees keys <= pos0+t.
#include <hip/hip_runtime.h>

#include "oppo_internal.h"

namespace oppo {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

struct AttnParams {
  const uint16_t* q;
  const uint16_t* k;
  const uint16_t* v;
  uint16_t* out;
  float* part_o;
  float* part_ml;
  int32_t Hq, Hkv, G, TM;
  float c;
  int32_t n_items;
  AttnItem items[kMaxAttnItems];
};
static_assert(sizeof(AttnParams) <= 4096, "kernel arguments must fit 4 KiB");

struct CombineParams {
  uint16_t* out;
  const float* part_o;
  const float* part_ml;
  int32_t Hq, Hkv, G, TM;
  float c;
  int32_t n_items;
  CombineItem items[kMaxCombineItems];
};
static_assert(sizeof(CombineParams) <= 4096, "kernel arguments must fit 4 KiB");

struct AppendParams {
  uint16_t* cache_k;
  uint16_t* cache_v;
  const uint16_t* k_new;
  const uint16_t* v_new;
  int32_t row_granules;  // 16-byte granules per token row = Hkv*D/8
  int32_t n_items;
  AppendItem items[kMaxAppendItems];
};
static_assert(sizeof(AppendParams) <= 4096, "kernel arguments must fit 4 KiB");

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Transposing LDS read: within each group of 16 lanes, lane j supplies the
// address of 4 consecutive bf16; lane i receives element (i & 3) of the
// pieces supplied by lanes (i >> 2), 4 + (i >> 2), 8 + (i >> 2), 12 + (i >> 2).
__device__ __forceinline__ s16x4 lds_read_tr16(const unsigned char* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (s16x4 __attribute__((address_space(3)))*)(const_cast<unsigned char*>(p)));
}

template <int D>
__global__ __launch_bounds__(256) void attn_fwd_kernel(const AttnParams P) {
  constexpr int NG = D / 8;    // 16-byte granules per K/V row
  constexpr int KK = D / 16;   // k-steps of S^T = K Q^T
  constexpr int DB = D / 32;   // 32-row blocks of O^T
  constexpr int BN = kKeyTile;
  constexpr int ROWB = D * 2;  // bytes per K/V row in LDS
  constexpr int TILE_BYTES = BN * ROWB;
  constexpr int LD_PER_THREAD = BN * NG / 256;
  constexpr int VSWZ_MASK = NG / 4 - 1;

  __shared__ __attribute__((aligned(16))) unsigned char lds[2][2][TILE_BYTES];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int l32 = lane & 31;
  const int hi = lane >> 5;
  const int kvh = blockIdx.x % P.Hkv;
  const AttnItem it = P.items[blockIdx.x / P.Hkv];
  const int Hq = P.Hq, Hkv = P.Hkv, G = P.G, TM = P.TM;
  const float c = P.c;

  // ---- per-lane query columns -------------------------------------------------
  int lim[2];          // last visible key of the column
  bool valid[2];
  int64_t qoff[2];     // element offset of the column's row in q / out
  bf16x8 qf[2][KK];
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
    const int r = wave * 64 + qb * 32 + l32;
    const int hh = r / TM;
    const int tok = r - hh * TM;
    valid[qb] = (hh < G) && (tok < it.n_tok);
    const int tokc = min(tok, it.n_tok - 1);
    const int hhc = min(hh, G - 1);
    lim[qb] = min(it.pos0 + tokc, it.k_end - 1);
    qoff[qb] = ((int64_t)(it.q_row0 + tokc) * Hq + kvh * G + hhc) * D;
    const uint16_t* qp = P.q + qoff[qb] + hi * 8;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) qf[qb][kk] = *(const bf16x8*)(qp + kk * 16);
  }
  // smallest limit of the workgroup's rows: tiles entirely below it need no mask
  const int min_lim = min(it.pos0, it.k_end - 1);

  f32x16 o[DB][2];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[db][qb][r] = 0.f;
  float m_run[2] = {-1e30f, -1e30f};
  float l_run[2] = {0.f, 0.f};

  // ---- cooperative K/V tile loads ------------------------------------------------
  const int k_hi = it.k_end;
  const int nt = (k_hi - it.k_begin + BN - 1) / BN;
  const uint16_t* kbase = P.k + ((int64_t)it.kv_row0 * Hkv + kvh) * D;
  const uint16_t* vbase = P.v + ((int64_t)it.kv_row0 * Hkv + kvh) * D;
  const int64_t row_stride = (int64_t)Hkv * D;

  u32x4 kreg[LD_PER_THREAD], vreg[LD_PER_THREAD];
  auto load_tile = [&](int key0) {
#pragma unroll
    for (int i = 0; i < LD_PER_THREAD; ++i) {
      const int gid = tid + 256 * i;
      const int row = gid / NG;
      const int lg = gid % NG;
      const int src = min(key0 + row, k_hi - 1);  // rows past the range repeat the last key
      const int64_t off = (int64_t)src * row_stride + lg * 8;
      kreg[i] = *(const u32x4*)(kbase + off);
      vreg[i] = *(const u32x4*)(vbase + off);
    }
  };
  auto store_tile = [&](int buf) {
#pragma unroll
    for (int i = 0; i < LD_PER_THREAD; ++i) {
      const int gid = tid + 256 * i;
      const int row = gid / NG;
      const int lg = gid % NG;
      *(u32x4*)(&lds[buf][0][row * ROWB + ((lg ^ (row % NG)) * 16)]) = kreg[i];
      *(u32x4*)(&lds[buf][1][row * ROWB + ((lg ^ ((row & VSWZ_MASK) << 2)) * 16)]) = vreg[i];
    }
  };

  load_tile(it.k_begin);
  store_tile(0);
  __syncthreads();

  for (int t = 0; t < nt; ++t) {
    const int buf = t & 1;
    const int key0 = it.k_begin + t * BN;
    if (t + 1 < nt) load_tile(key0 + BN);

    const unsigned char* Kt = lds[buf][0];
    const unsigned char* Vt = lds[buf][1];

    // ---- S^T = K Q^T : s[kb][qb] holds keys kb*32.. x query columns qb*32.. -------
    f32x16 s[2][2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int r = 0; r < 16; ++r) s[kb][qb][r] = 0.f;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        const int row = kb * 32 + l32;
        const int lg = kk * 2 + hi;
        const bf16x8 a = *(const bf16x8*)(Kt + row * ROWB + ((lg ^ (row % NG)) * 16));
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
          s[kb][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[qb][kk], s[kb][qb], 0, 0, 0);
      }
    }

    // ---- causal / range mask on tiles that cross a limit -----------------------
    if (key0 + BN - 1 > min_lim) {
#pragma unroll
      for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = key0 + kb * 32 + 8 * (r >> 2) + 4 * hi + (r & 3);
            if (key > lim[qb]) s[kb][qb][r] = -INFINITY;
          }
    }

    // ---- online softmax, one query column per lane (two halves in lanes l, l^32)
    bf16x8 pf[2][2][2];  // [kb][u][qb] : B operands of O^T += V^T P^T
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      float mx = s[0][qb][0];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kb][qb][r]);
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float m_new = fmaxf(m_run[qb], mx);
      const float alpha = fast_exp2((m_run[qb] - m_new) * c);
      const float mc = m_new * c;
      m_run[qb] = m_new;
      float rs = 0.f;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float p = fast_exp2(fmaf(s[kb][qb][r], c, -mc));
          s[kb][qb][r] = p;
          rs += p;
        }
      l_run[qb] = l_run[qb] * alpha + rs;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[db][qb][r] *= alpha;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          bf16x8 b;
#pragma unroll
          for (int j = 0; j < 8; ++j) b[j] = (__bf16)s[kb][qb][8 * u + j];
          pf[kb][u][qb] = b;
        }
    }

    // ---- O^T += V^T P^T ------------------------------------------------------------
    {
      const int j = lane & 15;
      const int half16 = (lane >> 4) & 1;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const int row0 = kb * 32 + 16 * u + 4 * hi + (j >> 2);
          const int row1 = row0 + 8;
#pragma unroll
          for (int db = 0; db < DB; ++db) {
            const int lg = db * 4 + 2 * half16 + ((j & 3) >> 1);
            const int sub = (j & 1) * 8;
            const s16x4 v0 = lds_read_tr16(Vt + row0 * ROWB + ((lg ^ ((row0 & VSWZ_MASK) << 2)) * 16) + sub);
            const s16x4 v1 = lds_read_tr16(Vt + row1 * ROWB + ((lg ^ ((row1 & VSWZ_MASK) << 2)) * 16) + sub);
            union { struct { s16x4 a, b; } h; bf16x8 v; } cat;
            cat.h.a = v0;
            cat.h.b = v1;
#pragma unroll
            for (int qb = 0; qb < 2; ++qb)
              o[db][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cat.v, pf[kb][u][qb], o[db][qb], 0, 0, 0);
          }
        }
    }

    if (t + 1 < nt) store_tile(buf ^ 1);
    __syncthreads();
  }

  // ---- epilogue ---------------------------------------------------------------------
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
    const float l_tot = l_run[qb] + __shfl_xor(l_run[qb], 32);
    if (it.part < 0) {
      if (valid[qb]) {
        const float inv = 1.0f / l_tot;
        uint16_t* op = P.out + qoff[qb];
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int b = 0; b < 4; ++b) {
            bf16x4 w;
#pragma unroll
            for (int e = 0; e < 4; ++e) w[e] = (__bf16)(o[db][qb][4 * b + e] * inv);
            *(bf16x4*)(op + db * 32 + 8 * b + 4 * hi) = w;
          }
      }
    } else {
      const int r = wave * 64 + qb * 32 + l32;
      const int64_t slot = ((int64_t)it.part * Hkv + kvh) * kTileRows + r;
      float* po = P.part_o + slot * D;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
          float4 w;
          w.x = o[db][qb][4 * b + 0];
          w.y = o[db][qb][4 * b + 1];
          w.z = o[db][qb][4 * b + 2];
          w.w = o[db][qb][4 * b + 3];
          *(float4*)(po + db * 32 + 8 * b + 4 * hi) = w;
        }
      if (hi == 0) {
        P.part_ml[slot * 2 + 0] = m_run[qb];
        P.part_ml[slot * 2 + 1] = l_tot;
      }
    }
  }
}

// Merge the partial (max, sum, unnormalised O) of the pieces of a split tile:
// out = sum_s w_s O_s / sum_s w_s l_s with w_s = exp2((m_s - max_s m_s) * c).
template <int D>
__global__ __launch_bounds__(256) void combine_kernel(const CombineParams P) {
  constexpr int TPR = D / 4;          // threads per row (float4 each)
  constexpr int RPB = 256 / TPR;      // rows per block
  const CombineItem it = P.items[blockIdx.x / P.Hkv];
  const int kvh = blockIdx.x % P.Hkv;
  const int r = blockIdx.y * RPB + threadIdx.x / TPR;
  const int d4 = (threadIdx.x % TPR) * 4;
  const int hh = r / P.TM;
  const int tok = r - hh * P.TM;
  if (hh >= P.G || tok >= it.n_tok) return;
  float m_max = -INFINITY;
  for (int s = 0; s < it.nsplit; ++s) {
    const int64_t slot = ((int64_t)(it.part0 + s) * P.Hkv + kvh) * kTileRows + r;
    m_max = fmaxf(m_max, P.part_ml[slot * 2]);
  }
  float4 acc = {0.f, 0.f, 0.f, 0.f};
  float l = 0.f;
  for (int s = 0; s < it.nsplit; ++s) {
    const int64_t slot = ((int64_t)(it.part0 + s) * P.Hkv + kvh) * kTileRows + r;
    const float w = fast_exp2((P.part_ml[slot * 2] - m_max) * P.c);
    l += w * P.part_ml[slot * 2 + 1];
    const float4 x = *(const float4*)(P.part_o + slot * D + d4);
    acc.x += w * x.x;
    acc.y += w * x.y;
    acc.z += w * x.z;
    acc.w += w * x.w;
  }
  const float inv = 1.0f / l;
  bf16x4 w4;
  w4[0] = (__bf16)(acc.x * inv);
  w4[1] = (__bf16)(acc.y * inv);
  w4[2] = (__bf16)(acc.z * inv);
  w4[3] = (__bf16)(acc.w * inv);
  uint16_t* op = P.out + ((int64_t)(it.q_row0 + tok) * P.Hq + kvh * P.G + hh) * D + d4;
  *(bf16x4*)op = w4;
}

// KV append: each item is one contiguous run of token rows (token-major layout
// makes a sequence's chunk contiguous in both source and destination).
// grid = (items, pieces of kAppendTok tokens, 2 = K/V); 16-byte copies.
constexpr int kAppendTok = 16;
__global__ __launch_bounds__(256) void kv_append_kernel(const AppendParams P) {
  const AppendItem it = P.items[blockIdx.x];
  const int tok0 = blockIdx.y * kAppendTok;
  if (tok0 >= it.n_tok) return;
  const int ntok = min(kAppendTok, it.n_tok - tok0);
  const uint16_t* src = (blockIdx.z == 0 ? P.k_new : P.v_new);
  uint16_t* dst = (blockIdx.z == 0 ? P.cache_k : P.cache_v);
  const int64_t rg = P.row_granules;
  const u32x4* s = (const u32x4*)src + ((int64_t)it.src_row + tok0) * rg;
  u32x4* d = (u32x4*)dst + (it.dst_row + tok0) * rg;
  const int64_t n = (int64_t)ntok * rg;
  for (int64_t i = threadIdx.x; i < n; i += 256) d[i] = s[i];
}

// ---------------------------------------------------------------------------------
// Launchers
// ---------------------------------------------------------------------------------

int launch_attention(const LayerShape& ls, const void* q, const void* k, const void* v, void* out,
                     float* part_o, float* part_ml, const AttnItem* items, int n_items, void* stream) {
  hipStream_t st = (hipStream_t)stream;
  for (int base = 0; base < n_items; base += kMaxAttnItems) {
    AttnParams P;
    P.q = (const uint16_t*)q;
    P.k = (const uint16_t*)k;
    P.v = (const uint16_t*)v;
    P.out = (uint16_t*)out;
    P.part_o = part_o;
    P.part_ml = part_ml;
    P.Hq = ls.Hq;
    P.Hkv = ls.Hkv;
    P.G = ls.G;
    P.TM = ls.TM;
    P.c = ls.c;
    const int n = n_items - base < kMaxAttnItems ? n_items - base : kMaxAttnItems;
    P.n_items = n;
    for (int i = 0; i < n; ++i) P.items[i] = items[base + i];
    dim3 grid((unsigned)(n * ls.Hkv)), block(256);
    if (ls.D == 128)
      hipLaunchKernelGGL(attn_fwd_kernel<128>, grid, block, 0, st, P);
    else
      hipLaunchKernelGGL(attn_fwd_kernel<64>, grid, block, 0, st, P);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return (int)e;
  }
  return 0;
}

int launch_combine(const LayerShape& ls, void* out, const float* part_o, const float* part_ml,
                   const CombineItem* items, int n_items, void* stream) {
  hipStream_t st = (hipStream_t)stream;
  for (int base = 0; base < n_items; base += kMaxCombineItems) {
    CombineParams P;
    P.out = (uint16_t*)out;
    P.part_o = part_o;
    P.part_ml = part_ml;
    P.Hq = ls.Hq;
    P.Hkv = ls.Hkv;
    P.G = ls.G;
    P.TM = ls.TM;
    P.c = ls.c;
    const int n = n_items - base < kMaxCombineItems ? n_items - base : kMaxCombineItems;
    P.n_items = n;
    for (int i = 0; i < n; ++i) P.items[i] = items[base + i];
    const int rpb = 256 / (ls.D / 4);
    dim3 grid((unsigned)(n * ls.Hkv), (unsigned)(kTileRows / rpb)), block(256);
    if (ls.D == 128)
      hipLaunchKernelGGL(combine_kernel<128>, grid, block, 0, st, P);
    else
      hipLaunchKernelGGL(combine_kernel<64>, grid, block, 0, st, P);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return (int)e;
  }
  return 0;
}

int launch_append(const LayerShape& ls, void* cache_k, void* cache_v, const void* k_new,
                  const void* v_new, const AppendItem* items, int n_items, int max_tok, void* stream) {
  hipStream_t st = (hipStream_t)stream;
  for (int base = 0; base < n_items; base += kMaxAppendItems) {
    AppendParams P;
    P.cache_k = (uint16_t*)cache_k;
    P.cache_v = (uint16_t*)cache_v;
    P.k_new = (const uint16_t*)k_new;
    P.v_new = (const uint16_t*)v_new;
    P.row_granules = ls.Hkv * ls.D / 8;
    const int n = n_items - base < kMaxAppendItems ? n_items - base : kMaxAppendItems;
    P.n_items = n;
    int mt = 0;
    for (int i = 0; i < n; ++i) {
      P.items[i] = items[base + i];
      if (items[base + i].n_tok > mt) mt = items[base + i].n_tok;
    }
    (void)max_tok;
    dim3 grid((unsigned)n, (unsigned)((mt + kAppendTok - 1) / kAppendTok), 2), block(256);
    hipLaunchKernelGGL(kv_append_kernel, grid, block, 0, st, P);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return (int)e;
  }
  return 0;
}

const char* hip_error_string(int err) { return hipGetErrorString((hipError_t)err); }

}  // namespace oppo
