// gfx950 kernels: the layer's fused QKV projection with the rotary embedding and the
// cache write as its epilogue.
//
//   y[m, n] = sum_k x[m, k] * w[n, k]     x: bf16 [rows][hidden], w: bf16 [(Hq + 2 Hkv) D][hidden]
//
// (both operands contiguous along k, fp32 accumulation), and then, per output row m at
// absolute position p and per head: query and key heads are rotated pair by pair
// ((t, t + D/2), angle p * base^(-2t/D): RoFormer Sec. 3.2 / 3.4.2 in the half-split pairing),
// rounded once to bf16 and written to q_out / to the sequence's cache slab; value heads go
// to the cache as they are.  The projection's output never exists in memory.
//
// Workgroup = 256 x 256 tile of y, 8 waves in a 4 x 2 arrangement of 64 x 128 (2 x 4 blocks of
// v_mfma_f32_32x32x16_bf16: six fragment reads feed eight MFMAs).  Passes too thin to give every
// compute unit such a tile take tiles of 128 or 64 rows instead (2 x 4 waves of 64 x 64 or 32 x 64).
// k advances in tiles of 64
// through two LDS stages per operand (128 KiB in all, one workgroup per compute unit, two
// waves per SIMD); tiles travel global -> LDS directly, the
// XOR swizzle of the LDS rows applied by choosing which 16-byte granule each lane fetches, so
// the fragment reads (ds_read_b128, one row per lane) spread over the banks.  The epilogue
// parks the fp32 tile in the same LDS, 64 rows at a time, from where threads take 8-column pieces of a row and
// their partners D/2 columns further on, rotate them with the (cos, sin) table a small kernel
// made beforehand for the pass's rows, and store 16 bytes at a time.
#include <hip/hip_runtime.h>

#include "oppo_internal.h"

namespace oppo {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kGemmBN = 256, kGemmBK = 64;   // the tile's rows BM (256, 128 or 64) are chosen per launch
constexpr int kProjCUs = 256;         // compute units of the chip: what a pass's tile count is weighed against
constexpr int kMaxProjItems = 1000;   // 1000 * 24 B + header in the kernel arguments

// Per-row data of a pass, made by proj_rows_kernel in the caller's workspace:
//   dst[rows]            int64  cache row (token slot) the row's keys and values go to
//   cs[rows][D/2]        float2 (cos, sin) of position * base^(-2t/D)
struct ProjRowsParams {
  int64_t* dst;
  float2* cs;
  double log2_base;
  int32_t half;      // D / 2
  int32_t n_items;
  QkvItem items[kMaxProjItems];
};
static_assert(sizeof(ProjRowsParams) <= 32768, "kernel arguments are kept within 32 KiB");

// grid = (items, pieces of 8 tokens); 256 threads.  Angles in double precision (they reach
// tens of thousands of radians for the fastest pair), kept as fp32.
__global__ __launch_bounds__(256) void proj_rows_kernel(const ProjRowsParams P) {
  const QkvItem it = P.items[blockIdx.x];
  const int tok0 = blockIdx.y * 8;
  if (tok0 >= it.n_tok) return;
  const int ntok = min(8, it.n_tok - tok0);
  const int D = 2 * P.half;
  for (int e = threadIdx.x; e < ntok * P.half; e += 256) {
    const int t = e / P.half, i = e % P.half;
    const int64_t row = (int64_t)it.src_row + tok0 + t;
    const double theta = exp2(-(2.0 * i / D) * P.log2_base);
    double s, c;
    sincos((double)(it.pos0 + tok0 + t) * theta, &s, &c);
    P.cs[row * P.half + i] = make_float2((float)c, (float)s);
    if (i == 0) P.dst[row] = it.dst_row + tok0 + t;
  }
}

struct ProjParams {
  const uint16_t* x;     // [rows][hidden]
  const uint16_t* w;     // [n_out][hidden]
  uint16_t* q_out;       // [rows][Hq][D]
  uint16_t* cache_k;     // [slots][Hkv][D]
  uint16_t* cache_v;
  const int64_t* dst;    // [rows]
  const float2* cs;      // [rows][D/2]
  int32_t rows, hidden, n_out;
  int32_t Hq, Hkv;
};

// 16 bytes per lane, global -> LDS: lane l reads gbase[voff_bytes .. +16), the data lands at
// lds_addr + 16 * l (gbase and lds_addr wave-uniform).  See the same helper of the attention
// kernel for why it is written as assembly and why M0 is not on a clobber list.
__device__ __forceinline__ void gemm_async_copy16(const void* gbase, uint32_t voff_bytes, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :: "s"(lds_addr), "v"(voff_bytes), "s"(gbase) : "memory");
}

__device__ __forceinline__ uint32_t gemm_pack_bf16(float a, float b) {
  bf16x2 p;
  p[0] = (__bf16)a;   // round to nearest even
  p[1] = (__bf16)b;
  return *(uint32_t*)&p;
}

template <int D, int BM>
__global__ __launch_bounds__(512) void qkv_proj_kernel(const ProjParams P) {
  constexpr int BN = kGemmBN, BK = kGemmBK;
  constexpr int ROWB = BK * 2;            // bytes of a tile row in LDS (128)
  constexpr int NGR = ROWB / 16;          // 16-byte granules per row (8)
  constexpr int RPL = 1024 / ROWB;        // rows one wave-wide copy covers (8)
  constexpr int TILE_A = BM * ROWB;       // bytes of an x tile (32, 16 or 8 KiB)
  constexpr int TILE_B = BN * ROWB;       // bytes of a w tile (32 KiB)
  constexpr int STAGE = TILE_A + TILE_B;
  constexpr int WR = BM == 256 ? 4 : 2, WC = 8 / WR;   // waves down and across the tile
  constexpr int MI = BM / WR / 32, NJ = BN / WC / 32;  // 32 x 32 blocks of a wave: 2 x 4, 2 x 2 or 1 x 2
  constexpr int CA = BM / RPL / 8, CB = BN / RPL / 8;  // copies per wave and tile: x (4, 2 or 1), w (4)
  static_assert(BN == 256 && BK == 64 && (BM == 256 || BM == 128 || BM == 64), "8 waves, k tiles of 64");
  // stages of the tile ring: two tiles of 256 rows fill the LDS; the smaller tiles run on passes
  // whose k loop is bound by the tiles' latency, and keep two tiles in flight instead of one
  constexpr int NST = BM == 256 ? 2 : 3;   // (four stages of the 64-row tile: measured, no faster)
  static_assert(NST * STAGE >= 64 * BN * 4 && NST * STAGE <= 160 * 1024, "ring and the epilogue's 64 x 256 fp32 strip fit the LDS");
  // [stage][x tile | w tile]; the epilogue reuses it as a 64 x 256 fp32 strip at a time
  __shared__ __attribute__((aligned(1024))) unsigned char smem[NST * STAGE];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, hi = lane >> 5;
  const int wm = wave / WC, wn = wave % WC;    // the wave's (32 MI) x (32 NJ) part of the tile
  // Workgroups are dealt round-robin to the chip's 8 XCDs, each with a level-2 cache of its own.
  // The 32 workgroups an XCD runs at a time take one block of 8 x 4 tiles: they stream through k
  // together, so every slice of the block's 8 row tiles and 4 column tiles is fetched into that
  // cache once and serves 4 resp. 8 workgroups.
  const int m_tiles = (P.rows + BM - 1) / BM, n_tiles = (P.n_out + BN - 1) / BN;
  const int gm_count = (m_tiles + 7) / 8;
  const int xcd = blockIdx.x % 8, slot = blockIdx.x / 8;
  const int group = (slot / 32) * 8 + xcd, within = slot % 32;
  const int tile_m = (group % gm_count) * 8 + within % 8, tile_n = (group / gm_count) * 4 + within / 8;
  if (tile_m >= m_tiles || tile_n >= n_tiles) return;
  const int64_t m0 = (int64_t)tile_m * BM, n0 = (int64_t)tile_n * BN;

  // ---- loads: a wave-wide copy moves 8 rows (8 x 128 B); wave w moves rows 8 (w + 8 i) .. of
  // x (i < CA) and of w (i < CB).  A row's eight granules are swizzled by (row / 2) % 8, so that
  // sixteen consecutive rows cover all sixteen 16-byte bank groups.  Rows past the end of x / w
  // repeat the last valid row (their products are never stored).
  const int lrow = lane / NGR, pg = lane % NGR;
  uint32_t offa[CA], offb[CB];
#pragma unroll
  for (int i = 0; i < CB; ++i) {
    const int r = RPL * (wave + 8 * i) + lrow;
    const int64_t ra = min(m0 + r, (int64_t)P.rows - 1) - m0, rb = min(n0 + r, (int64_t)P.n_out - 1) - n0;
    if (i < CA) offa[i] = (uint32_t)(ra * P.hidden + ((pg ^ ((r >> 1) % NGR)) * 8)) * 2u;
    offb[i] = (uint32_t)(rb * P.hidden + ((pg ^ ((r >> 1) % NGR)) * 8)) * 2u;
  }
  const uint16_t* xa = P.x + m0 * P.hidden;
  const uint16_t* wb = P.w + n0 * P.hidden;
  const uint32_t smem0 = (uint32_t)(uintptr_t)((const __attribute__((address_space(3))) unsigned char*)smem);
  const uint32_t wave_u = (uint32_t)__builtin_amdgcn_readfirstlane(wave);
  auto issue = [&](int kt, int stage) __attribute__((always_inline)) {
    const uint16_t* ga = xa + (int64_t)kt * BK;
    const uint16_t* gb = wb + (int64_t)kt * BK;
#pragma unroll
    for (int i = 0; i < CB; ++i) {
      const uint32_t dst = smem0 + (uint32_t)stage * (uint32_t)STAGE + (wave_u + 8u * i) * 1024u;
      if (i < CA) gemm_async_copy16(ga, offa[i], dst);
      gemm_async_copy16(gb, offb[i], dst + TILE_A);
    }
  };
  auto barrier = [&]() __attribute__((always_inline)) {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  };

  // ---- fragments: lane (l32, hi) reads row (block * 32 + l32), elements k = 16 kk + 8 hi ..;
  // per-lane base addresses (the swizzle (row / 2) % 8 is (l32 / 2) % 8 for every block), stage
  // and k-step folded in as immediates / XORs
  typedef const __attribute__((address_space(3))) unsigned char* lds_cptr;
  const uint32_t a_base = smem0 + (uint32_t)((wm * 32 * MI + l32) * ROWB);
  const uint32_t b_base = smem0 + TILE_A + (uint32_t)((wn * 32 * NJ + l32) * ROWB);
  const uint32_t swz = (uint32_t)((l32 >> 1) % NGR);
  auto frag = [&](uint32_t base, int stage, int block, int kk) __attribute__((always_inline)) -> bf16x8 {
    const uint32_t a = base + (uint32_t)stage * (uint32_t)STAGE + (uint32_t)(block * 32 * ROWB) + ((((uint32_t)(kk * 2 + hi)) ^ swz) * 16u);
    return *(const __attribute__((address_space(3))) bf16x8*)(lds_cptr)(uintptr_t)a;
  };

  f32x16 acc[MI][NJ];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int KT = P.hidden / BK;
  // one tile's 4 k-steps out of ring stage st
  auto compute = [&](int st) __attribute__((always_inline)) {
    bf16x8 a[2][MI], b[2][NJ];   // fragments of k-step kk in [kk & 1]: read one step ahead of their MFMAs
#pragma unroll
    for (int i = 0; i < MI; ++i) a[0][i] = frag(a_base, st, i, 0);
#pragma unroll
    for (int j = 0; j < NJ; ++j) b[0][j] = frag(b_base, st, j, 0);
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      const int c = kk & 1;
      if (kk + 1 < BK / 16) {
#pragma unroll
        for (int i = 0; i < MI; ++i) a[c ^ 1][i] = frag(a_base, st, i, kk + 1);
#pragma unroll
        for (int j = 0; j < NJ; ++j) b[c ^ 1][j] = frag(b_base, st, j, kk + 1);
      }
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[c][i], b[c][j], acc[i][j], 0, 0, 0);
    }
  };
  if constexpr (NST == 2) {
    issue(0, 0);
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
    barrier();
    for (int kt = 0; kt < KT; ++kt) {
      const int st = kt & 1;
      if (kt + 1 < KT) issue(kt + 1, st ^ 1);
      compute(st);
      __builtin_amdgcn_s_waitcnt(0x0F70);   // this wave's share of the next tile is in LDS
      barrier();
    }
  } else {
    // tile t lives in stage t % NST; tiles kt + 1 .. kt + NST - 2 stay in flight while tile kt is
    // waited for, and tile kt + NST - 1 is requested into the stage of tile kt - 1 once every wave
    // has passed the barrier behind that tile's MFMAs
    static_assert(NST == 3 || NST == 4, "the waits below are written for one or two later tiles in flight");
    constexpr int CPT = CA + CB;   // copies per wave and tile
#pragma unroll
    for (int t = 0; t < NST - 1; ++t)
      if (t < KT) issue(t, t);
    int st = 0, st_in = NST - 1;
    for (int kt = 0; kt < KT; ++kt) {
      // this wave's copies of tile kt have landed: only those of the later tiles may be outstanding
      if (NST == 4 && kt + 2 < KT)
        __builtin_amdgcn_s_waitcnt(0x0F70 | (2 * CPT));   // vmcnt(2 CPT)
      else if (kt + 1 < KT)
        __builtin_amdgcn_s_waitcnt(0x0F70 | CPT);         // vmcnt(CPT)
      else
        __builtin_amdgcn_s_waitcnt(0x0F70);               // vmcnt(0)
      barrier();
      if (kt + NST - 1 < KT) issue(kt + NST - 1, st_in);
      compute(st);
      st_in = st;
      st = st + 1 == NST ? 0 : st + 1;
    }
    barrier();   // every wave is through with the ring before the epilogue reuses it
  }

  // ---- epilogue, one strip of 64 rows at a time (the waves whose blocks lie in it: one wm, or
  // both for tiles of 64 rows): the fp32 strip into LDS (row-major, 256 floats per row), then out
  // again as row pieces - an item is (row, head of the tile, group of 8 pairs)
  float* ct = (float*)smem;
  constexpr int HALF = D / 2, GPH = HALF / 8, HPT = BN / D;   // groups per head, heads per tile
  const int heads = P.Hq + 2 * P.Hkv;
  for (int strip = 0; strip < (BM + 63) / 64; ++strip) {
#pragma unroll
    for (int i = 0; i < MI; ++i) {
      const int row0 = (wm * MI + i) * 32;   // the block's first row in the tile
      if (row0 / 64 != strip) continue;
#pragma unroll
      for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          // register r of lane (l32, hi): row 8 (r / 4) + 4 hi + r % 4, column l32 of the 32 x 32 block
          const int m = row0 % 64 + 8 * (r >> 2) + 4 * hi + (r & 3);
          const int n = (wn * NJ + j) * 32 + l32;
          ct[m * BN + n] = acc[i][j][r];
        }
    }
    __syncthreads();
    for (int item = tid; item < 64 * HPT * GPH; item += 512) {
      const int g = item % GPH, hl = (item / GPH) % HPT, m = item / (GPH * HPT);
      const int64_t row = m0 + strip * 64 + m;
      const int head = (int)(n0 / D) + hl;
      if (row >= P.rows || head >= heads) continue;
      const float* src = ct + m * BN + hl * D + g * 8;
      const f32x4 a0 = *(const f32x4*)(src), a1 = *(const f32x4*)(src + 4);
      const f32x4 b0 = *(const f32x4*)(src + HALF), b1 = *(const f32x4*)(src + HALF + 4);
      const float av[8] = {a0[0], a0[1], a0[2], a0[3], a1[0], a1[1], a1[2], a1[3]};
      const float bv[8] = {b0[0], b0[1], b0[2], b0[3], b1[0], b1[1], b1[2], b1[3]};
      uint16_t* dst;
      u32x4 ra, rb;
      if (head >= P.Hq + P.Hkv) {   // a value head: as it is
        dst = P.cache_v + (P.dst[row] * P.Hkv + (head - P.Hq - P.Hkv)) * D;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          ra[w] = gemm_pack_bf16(av[2 * w], av[2 * w + 1]);
          rb[w] = gemm_pack_bf16(bv[2 * w], bv[2 * w + 1]);
        }
      } else {
        dst = head < P.Hq ? P.q_out + (row * P.Hq + head) * D : P.cache_k + (P.dst[row] * P.Hkv + (head - P.Hq)) * D;
        const float2* cs = P.cs + row * HALF + g * 8;
        float ca[8], sa[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float2 v = cs[e];
          ca[e] = v.x;
          sa[e] = v.y;
        }
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          const int e = 2 * w;
          ra[w] = gemm_pack_bf16(av[e] * ca[e] - bv[e] * sa[e], av[e + 1] * ca[e + 1] - bv[e + 1] * sa[e + 1]);
          rb[w] = gemm_pack_bf16(bv[e] * ca[e] + av[e] * sa[e], bv[e + 1] * ca[e + 1] + av[e + 1] * sa[e + 1]);
        }
      }
      *(u32x4*)(dst + g * 8) = ra;
      *(u32x4*)(dst + HALF + g * 8) = rb;
    }
    __syncthreads();
  }
}

size_t proj_workspace_bytes(int D, int64_t rows) {
  return (size_t)rows * (sizeof(int64_t) + (size_t)(D / 2) * sizeof(float2));
}

int launch_qkv_proj(const LayerShape& ls, const void* x, const void* w, int32_t hidden, int32_t rows, void* q_out,
                    void* cache_k, void* cache_v, const QkvItem* items, int n_items, double theta_base, void* workspace,
                    void* stream) {
  hipStream_t st = (hipStream_t)stream;
  int64_t* dst = (int64_t*)workspace;
  float2* cs = (float2*)((unsigned char*)workspace + (size_t)rows * sizeof(int64_t));
  for (int base = 0; base < n_items; base += kMaxProjItems) {
    ProjRowsParams R;
    R.dst = dst;
    R.cs = cs;
    R.log2_base = log2(theta_base);
    R.half = ls.D / 2;
    const int n = n_items - base < kMaxProjItems ? n_items - base : kMaxProjItems;
    R.n_items = n;
    int mt = 0;
    for (int i = 0; i < n; ++i) {
      R.items[i] = items[base + i];
      if (items[base + i].n_tok > mt) mt = items[base + i].n_tok;
    }
    hipLaunchKernelGGL(proj_rows_kernel, dim3((unsigned)n, (unsigned)((mt + 7) / 8)), dim3(256), 0, st, R);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return (int)e;
  }
  ProjParams P;
  P.x = (const uint16_t*)x;
  P.w = (const uint16_t*)w;
  P.q_out = (uint16_t*)q_out;
  P.cache_k = (uint16_t*)cache_k;
  P.cache_v = (uint16_t*)cache_v;
  P.dst = dst;
  P.cs = cs;
  P.rows = rows;
  P.hidden = hidden;
  P.n_out = (ls.Hq + 2 * ls.Hkv) * ls.D;
  P.Hq = ls.Hq;
  P.Hkv = ls.Hkv;
  // Tile rows: one workgroup per compute unit at a time, so a launch takes ceil(tiles / 256) rounds of one
  // tile's duration; per k tile that duration was measured as 1.8 / 1.0 / 0.67 us for tiles of 256 / 128 /
  // 64 rows.  The cheapest estimate wins, the larger tile on a tie: thin passes spread over more compute
  // units, mid-sized ones avoid a mostly empty last round.
  const int n_tiles = (P.n_out + kGemmBN - 1) / kGemmBN;
  auto rounds_at = [&](int bm) { return (((int64_t)(rows + bm - 1) / bm) * n_tiles + kProjCUs - 1) / kProjCUs; };
  const double cost256 = 1.8 * (double)rounds_at(256), cost128 = 1.0 * (double)rounds_at(128), cost64 = 0.67 * (double)rounds_at(64);
  const int bm = (cost256 <= cost128 && cost256 <= cost64) ? 256 : cost128 <= cost64 ? 128 : 64;
  // blocks of 8 x 4 tiles, one block per XCD at a time (see the kernel); a launch has whole rounds of 8 blocks
  const int m_tiles = (rows + bm - 1) / bm;
  const int groups = ((m_tiles + 7) / 8) * ((n_tiles + 3) / 4);
  dim3 grid((unsigned)(((groups + 7) / 8) * 8 * 32));
  if (ls.D == 128) {
    if (bm == 256) hipLaunchKernelGGL((qkv_proj_kernel<128, 256>), grid, dim3(512), 0, st, P);
    else if (bm == 128) hipLaunchKernelGGL((qkv_proj_kernel<128, 128>), grid, dim3(512), 0, st, P);
    else hipLaunchKernelGGL((qkv_proj_kernel<128, 64>), grid, dim3(512), 0, st, P);
  } else {
    if (bm == 256) hipLaunchKernelGGL((qkv_proj_kernel<64, 256>), grid, dim3(512), 0, st, P);
    else if (bm == 128) hipLaunchKernelGGL((qkv_proj_kernel<64, 128>), grid, dim3(512), 0, st, P);
    else hipLaunchKernelGGL((qkv_proj_kernel<64, 64>), grid, dim3(512), 0, st, P);
  }
  return (int)hipGetLastError();
}

}  // namespace oppo
