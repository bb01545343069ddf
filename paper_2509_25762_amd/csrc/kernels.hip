// gfx950 kernels: ragged chunked-prefill attention, split-KV merge, KV append.
//
// Attention (per workgroup = one AttnItem x one kv-head), 8 waves of 64 lanes:
//   * the query tile packs TM tokens x G q-heads of the kv-head into 256 rows;
//     wave w owns rows [32w, 32w+32).  The transposed product S^T = K Q^T is
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

#include <type_traits>

#include "oppo_internal.h"

namespace oppo {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
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
static_assert(sizeof(AttnParams) <= 32768, "kernel arguments are kept within 32 KiB");

struct CombineParams {
  uint16_t* out;
  const float* part_o;
  const float* part_ml;
  int32_t Hq, Hkv, G, TM;
  float c;
  int32_t n_items;
  CombineItem items[kMaxCombineItems];
};
static_assert(sizeof(CombineParams) <= 32768, "kernel arguments are kept within 32 KiB");

struct AppendParams {
  uint16_t* cache_k;
  uint16_t* cache_v;
  const uint16_t* k_new;
  const uint16_t* v_new;
  int32_t row_granules;  // 16-byte granules per token row = Hkv*D/8
  int32_t n_items;
  AppendItem items[kMaxAppendItems];
};
static_assert(sizeof(AppendParams) <= 32768, "kernel arguments are kept within 32 KiB");

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Exchange of the two 32-lane halves of a wave: every lane receives the value
// held by the lane 32 away (v_permlane32_swap; the compiler's builtin for it
// mis-assigns the second result, so the instruction is written out).
__device__ __forceinline__ float swap_halves(float x) {
  float a = x, b = x;
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
  // a = {x[0:31], x[0:31]}, b = {x[32:63], x[32:63]}: pick the other half
  return (threadIdx.x & 32) ? a : b;
}

// LDS byte address of a __shared__ object.
__device__ __forceinline__ uint32_t lds_addr_of(const void* p) {
  return (uint32_t)(uintptr_t)((const __attribute__((address_space(3))) unsigned char*)p);
}

// Direct global -> LDS copy of 16 bytes per lane: lane l of the wave reads
// gbase[voff_bytes .. +16) and the data lands at LDS address lds_addr + 16 * l
// (gbase and lds_addr are wave-uniform).  Completion is tracked by vmcnt.
// Written as inline assembly on purpose: for the intrinsic form the compiler
// cannot tell the ring stages apart and waits for the copy before every later
// LDS read, which would serialise the prefetch; the waits are placed by hand.
// M0 is a reserved register that the compiler sets before each of its own uses.
__device__ __forceinline__ void async_copy16(const void* gbase, uint32_t voff_bytes, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :: "s"(lds_addr), "v"(voff_bytes), "s"(gbase) : "memory");
}

// Transposing LDS read: within each group of 16 lanes, lane j supplies the
// address of 4 consecutive bf16; lane i receives element (i & 3) of the
// pieces supplied by lanes (i >> 2), 4 + (i >> 2), 8 + (i >> 2), 12 + (i >> 2).
__device__ __forceinline__ s16x4 lds_read_tr16(const unsigned char* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (s16x4 __attribute__((address_space(3)))*)(const_cast<unsigned char*>(p)));
}

// Eight waves, each owning 32 query columns of the 256-row tile; two waves share
// a SIMD, so one wave's MFMAs fill the matrix pipe while the other waits for an
// operand or runs vector ALU work.  Within a wave the instruction stream is laid
// out by hand (fenced with sched_barrier so the compiler keeps it):
//   * operand fragments are read from LDS several steps before the MFMA that
//     consumes them (rolling register buffers ka / vf), the first K fragments of
//     the next tile already during the current tile's second product;
//   * the two MFMA chains (S^T, then O^T) are kept dense; the softmax in between
//     is pure vector ALU work that the other wave of the SIMD overlaps with its
//     own MFMAs.
// K/V tiles go straight from global memory into a ring of four LDS stages, three
// tiles ahead: the loads of tile t+3 are issued after barrier t into the stage
// last read before that barrier, and each wave waits for its own loads of tile
// t+2 before barrier t+1, after which that tile may be read.
template <int D>
__global__ __launch_bounds__(512) void attn_fwd_kernel(const AttnParams P) {
  constexpr int NT = 512;            // threads
  constexpr int NG = D / 8;          // 16-byte granules per K/V row
  constexpr int KK = D / 16;         // k-steps of S^T = K Q^T
  constexpr int DB = D / 32;         // 32-row blocks of O^T
  constexpr int BN = kKeyTile;
  constexpr int ROWB = D * 2;        // bytes per K/V row in LDS
  constexpr int TILE_BYTES = BN * ROWB;
  constexpr int VSWZ_MASK = NG / 4 - 1;
  constexpr int NSTAGE = 4;
  constexpr int RPI = 1024 / ROWB;     // tile rows one wave-wide 16-byte load covers
  constexpr int IPW = BN / RPI / 8;    // such loads per wave, per tile, for K and again for V
  constexpr int KDEPTH = 3;          // k-steps of K fragments kept in flight
  constexpr int VDEPTH = 4;          // V^T fragments kept in flight
  constexpr int PV_STEPS = 4 * DB;   // MFMAs of the second product per tile
  static_assert(IPW >= 1 && NT == 512, "tile smaller than the workgroup");
  static_assert(KK >= KDEPTH && KK >= VDEPTH && PV_STEPS >= VDEPTH, "pipeline deeper than the tile");

  // one array per stage and operand, so that the compiler can tell a pending
  // direct-to-LDS load of one stage from the fragment reads of another
  __shared__ __attribute__((aligned(1024))) unsigned char sk0[TILE_BYTES], sk1[TILE_BYTES], sk2[TILE_BYTES], sk3[TILE_BYTES];
  __shared__ __attribute__((aligned(1024))) unsigned char sv0[TILE_BYTES], sv1[TILE_BYTES], sv2[TILE_BYTES], sv3[TILE_BYTES];
  auto SK = [&](int b) __attribute__((always_inline)) { return b == 0 ? sk0 : b == 1 ? sk1 : b == 2 ? sk2 : sk3; };
  auto SV = [&](int b) __attribute__((always_inline)) { return b == 0 ? sv0 : b == 1 ? sv1 : b == 2 ? sv2 : sv3; };

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int l32 = lane & 31;
  const int hi = lane >> 5;
  const int kvh = blockIdx.x % P.Hkv;
  const AttnItem it = P.items[blockIdx.x / P.Hkv];
  const int Hq = P.Hq, Hkv = P.Hkv, G = P.G, TM = P.TM;
  const float c = P.c;

  // ---- this lane's query column ---------------------------------------------------
  const int r_tile = wave * 32 + l32;   // row of the packed (head, token) tile
  const int hh = r_tile / TM;
  const int tok = r_tile - hh * TM;
  const bool valid = (hh < G) && (tok < it.n_tok);
  const int tokc = min(tok, it.n_tok - 1);
  const int hhc = min(hh, G - 1);
  const int lim = min(it.pos0 + tokc, it.k_end - 1);   // last visible key of the column
  const int64_t qoff = ((int64_t)(it.q_row0 + tokc) * Hq + kvh * G + hhc) * D;
  bf16x8 qf[KK];
  {
    const uint16_t* qp = P.q + qoff + hi * 8;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) qf[kk] = *(const bf16x8*)(qp + kk * 16);
  }
  // smallest limit of the workgroup's rows: tiles entirely below it need no mask
  const int min_lim = min(it.pos0, it.k_end - 1);

  f32x16 o[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[db][r] = 0.f;
  float m_run = -1e30f, l_run = 0.f;

  // ---- cooperative K/V tile loads ------------------------------------------------
  const int k_hi = it.k_end;
  const int nt = (k_hi - it.k_begin + BN - 1) / BN;
  const int row_stride = Hkv * D;  // elements between consecutive tokens
  const uint16_t* kbase = P.k + ((int64_t)it.kv_row0 * Hkv + kvh) * D;
  const uint16_t* vbase = P.v + ((int64_t)it.kv_row0 * Hkv + kvh) * D;

  // Tiles travel global -> LDS directly (global_load_lds_dwordx4): a wave-wide
  // load drops 64 x 16 bytes at consecutive LDS addresses, i.e. RPI whole rows;
  // the LDS swizzle is applied by choosing which 16-byte granule of the row each
  // lane fetches.  Wave w moves rows (w + 8i) * RPI .. of the tile.
  const int lrow = lane / NG;
  const int pg = lane % NG;
  uint32_t goffk[IPW], goffv[IPW];   // byte offsets of this lane's granules in a full tile
#pragma unroll
  for (int i = 0; i < IPW; ++i) {
    const int r = (wave + 8 * i) * RPI + lrow;
    goffk[i] = (uint32_t)(r * row_stride + ((pg ^ (r % NG)) * 8)) * 2u;
    goffv[i] = (uint32_t)(r * row_stride + ((pg ^ ((r & VSWZ_MASK) << 2)) * 8)) * 2u;
  }
  const uint32_t wave_rows = (uint32_t)__builtin_amdgcn_readfirstlane(wave) * 1024u;
  auto issue_tile = [&](int stage, int t) __attribute__((always_inline)) {
    const int key0 = it.k_begin + t * BN;
    const int last = k_hi - 1 - key0;
    const uint16_t* kt = kbase + (int64_t)key0 * row_stride;
    const uint16_t* vt = vbase + (int64_t)key0 * row_stride;
#pragma unroll
    for (int i = 0; i < IPW; ++i) {
      uint32_t ok = goffk[i], ov = goffv[i];
      if (last < BN - 1) {  // ragged last tile: rows past the range repeat the last key
        const int r = (wave + 8 * i) * RPI + lrow;
        const int rc = min(r, last);
        ok = (uint32_t)(rc * row_stride + ((pg ^ (r % NG)) * 8)) * 2u;
        ov = (uint32_t)(rc * row_stride + ((pg ^ ((r & VSWZ_MASK) << 2)) * 8)) * 2u;
      }
      async_copy16(kt, ok, lds_addr_of(SK(stage)) + wave_rows + i * 8192u);
      async_copy16(vt, ov, lds_addr_of(SV(stage)) + wave_rows + i * 8192u);
    }
  };
  // workgroup barrier without the implied wait for this wave's LDS reads: the only
  // reads still in flight at a barrier are the K fragments of the next tile, whose
  // stage is not overwritten before they have been consumed
  auto wg_barrier = [&]() __attribute__((always_inline)) {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  };

  // per-lane LDS offsets of the operand fragments (the swizzles are XORs, so they
  // are folded here once instead of per read)
  int koff[KK];  // K fragment of k-step kk, key block 0 (block 1 is +32 rows)
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) koff[kk] = l32 * ROWB + (((kk * 2 + hi) ^ (l32 % NG)) * 16);
  int voff[DB];  // V^T fragment of d-block db, keys 4*hi.. of a 16-key group
  {
    const int j = lane & 15;
    const int half16 = (lane >> 4) & 1;
    const int vrow = 4 * hi + (j >> 2);
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      const int lg = db * 4 + 2 * half16 + ((j & 3) >> 1);
      voff[db] = vrow * ROWB + ((lg ^ ((vrow & VSWZ_MASK) << 2)) * 16) + (j & 1) * 8;
    }
  }
  // K fragment (A operand of S^T = K Q^T): keys kb*32 + l32, elements kk*16 + 8*hi..
  auto ldk = [&](int buf, int kk, int kb) __attribute__((always_inline)) -> bf16x8 {
    return *(const bf16x8*)(SK(buf) + kb * 32 * ROWB + koff[kk]);
  };
  // V^T fragment (A operand of O^T += V^T P^T) of PV step `step` = (16-key group g, d-block db)
  auto ldv = [&](int buf, int step) __attribute__((always_inline)) -> bf16x8 {
    const int g = step / DB, db = step % DB;
    const unsigned char* vp = SV(buf) + g * 16 * ROWB + voff[db];
    union { struct { s16x4 a, b; } h; bf16x8 v; } cat;
    cat.h.a = lds_read_tr16(vp);
    cat.h.b = lds_read_tr16(vp + 8 * ROWB);
    return cat.v;
  };

  // the running max is refreshed only when a score exceeds it by more than 2^8
  // in the exp2 domain; until then probabilities stay below 256, which fp32
  // sums and bf16 operands hold without loss
  const float tau = 8.0f / c;
  const bf16x2 ones2 = {(__bf16)1.0f, (__bf16)1.0f};

  f32x16 s[2];            // S^T of the current tile: keys kb*32.. x this wave's 32 columns
  bf16x8 ka[KDEPTH][2];   // K fragments in flight
  bf16x8 vf[VDEPTH];      // V^T fragments in flight
  union { bf16x2 h[4]; bf16x8 v; } pf[4];  // probabilities of 16-key group g, B operand layout
  float mc = 0.f, rs0 = 0.f, rs1 = 0.f;

  // probabilities 2j, 2j+1 of group g: exp2, round to bf16, add to the row sum
  // (the sum uses the rounded values, like the numerator does)
  auto exp_pair = [&](int g, int j) __attribute__((always_inline)) {
    const int kb = g >> 1, u = g & 1;
    const float p0 = fast_exp2(fmaf(s[kb][8 * u + 2 * j], c, -mc));
    const float p1 = fast_exp2(fmaf(s[kb][8 * u + 2 * j + 1], c, -mc));
    bf16x2 pk;
    pk[0] = (__bf16)p0;
    pk[1] = (__bf16)p1;
    pf[g].h[j] = pk;
    if (j & 1)
      rs1 = __builtin_amdgcn_fdot2_f32_bf16(pk, ones2, rs1, false);
    else
      rs0 = __builtin_amdgcn_fdot2_f32_bf16(pk, ones2, rs0, false);
  };

  // S^T = K Q^T of the tile in stage kbuf (its first K fragments are already in ka);
  // the first V^T fragments are fetched under the last MFMAs
  auto qk_phase = [&](int kbuf) __attribute__((always_inline)) {
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) s[kb][r] = 0.f;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[kk % KDEPTH][0], qf[kk], s[0], 0, 0, 0);
      s[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[kk % KDEPTH][1], qf[kk], s[1], 0, 0, 0);
      if (kk + KDEPTH < KK) {
        ka[kk % KDEPTH][0] = ldk(kbuf, kk + KDEPTH, 0);
        ka[kk % KDEPTH][1] = ldk(kbuf, kk + KDEPTH, 1);
      }
      if (kk >= KK - VDEPTH) vf[kk - (KK - VDEPTH)] = ldv(kbuf, kk - (KK - VDEPTH));
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  auto tile_step = [&](auto BUFC, int t) __attribute__((always_inline)) {
    constexpr int buf = decltype(BUFC)::value;
    constexpr int nbuf = (buf + 1) % NSTAGE;
    const bool pre = t + 3 < nt;
    const bool next = t + 1 < nt;
    if (pre) issue_tile((buf + 3) % NSTAGE, t + 3);
    qk_phase(buf);

    // ---- causal / range mask on tiles that cross a limit -----------------------
    const int key0 = it.k_begin + t * BN;
    if (key0 + BN - 1 > min_lim) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = key0 + kb * 32 + 8 * (r >> 2) + 4 * hi + (r & 3);
          if (key > lim) s[kb][r] = -INFINITY;
        }
    }

    // ---- running max: one query column per lane, key halves in lanes l and l^32 -----
    {
      float mx4[4];
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {  // four independent chains
        mx4[q4] = fmaxf(s[0][q4], s[1][q4]);
#pragma unroll
        for (int r = 4; r < 16; r += 4) mx4[q4] = fmaxf(mx4[q4], fmaxf(s[0][r + q4], s[1][r + q4]));
      }
      float mx = fmaxf(fmaxf(mx4[0], mx4[1]), fmaxf(mx4[2], mx4[3]));
      mx = fmaxf(mx, swap_halves(mx));
      if (__any(mx > m_run + tau)) {
        const float m_new = fmaxf(m_run, mx);
        const float alpha = fast_exp2((m_run - m_new) * c);
        m_run = m_new;
        l_run *= alpha;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[db][r] *= alpha;
      }
      mc = m_run * c;
    }
    rs0 = 0.f;
    rs1 = 0.f;
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
      for (int j = 0; j < 4; ++j) exp_pair(g, j);
    __builtin_amdgcn_sched_barrier(0);

    // ---- O^T += V^T P^T -----------------------------------------------------------------
#pragma unroll
    for (int step = 0; step < PV_STEPS; ++step) {
      const int g = step / DB, db = step % DB;
      o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[step % VDEPTH], pf[g].v, o[db], 0, 0, 0);
      if (step + VDEPTH < PV_STEPS) vf[step % VDEPTH] = ldv(buf, step + VDEPTH);
      if (step >= PV_STEPS - KDEPTH && next) {
        ka[step - (PV_STEPS - KDEPTH)][0] = ldk(nbuf, step - (PV_STEPS - KDEPTH), 0);
        ka[step - (PV_STEPS - KDEPTH)][1] = ldk(nbuf, step - (PV_STEPS - KDEPTH), 1);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    l_run += rs0 + rs1;
    // tile t+2 must have landed (in every wave) before the next iteration reads its
    // K fragments ahead; the loads of tile t+3, issued above, may stay in flight
    if (pre)
      __builtin_amdgcn_s_waitcnt(0x0F70 | (2 * IPW));
    else
      __builtin_amdgcn_s_waitcnt(0x0F70);
    wg_barrier();
  };

  // ---- prologue: tiles 0..2 into stages 0..2 ---------------------------------------
  issue_tile(0, 0);
  if (nt > 1) issue_tile(1, 1);
  if (nt > 2) issue_tile(2, 2);
  // Everything issued so far (the Q fragments included) must have landed before the
  // loop; a wait left to the compiler would sit inside the loop, where it would
  // also cover the loads of later tiles.
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
  wg_barrier();
#pragma unroll
  for (int kk = 0; kk < KDEPTH; ++kk) {
    ka[kk][0] = ldk(0, kk, 0);
    ka[kk][1] = ldk(0, kk, 1);
  }

  for (int t = 0; t < nt; t += 4) {
    tile_step(std::integral_constant<int, 0>{}, t);
    if (t + 1 < nt) tile_step(std::integral_constant<int, 1>{}, t + 1);
    if (t + 2 < nt) tile_step(std::integral_constant<int, 2>{}, t + 2);
    if (t + 3 < nt) tile_step(std::integral_constant<int, 3>{}, t + 3);
  }

  // ---- epilogue ---------------------------------------------------------------------
  const float l_tot = l_run + __shfl_xor(l_run, 32);
  if (it.part < 0) {
    if (valid) {
      const float inv = 1.0f / l_tot;
      uint16_t* op = P.out + qoff;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
          bf16x4 w;
#pragma unroll
          for (int e = 0; e < 4; ++e) w[e] = (__bf16)(o[db][4 * b + e] * inv);
          *(bf16x4*)(op + db * 32 + 8 * b + 4 * hi) = w;
        }
    }
  } else {
    const int64_t slot = ((int64_t)it.part * Hkv + kvh) * kTileRows + r_tile;
    float* po = P.part_o + slot * D;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        float4 w;
        w.x = o[db][4 * b + 0];
        w.y = o[db][4 * b + 1];
        w.z = o[db][4 * b + 2];
        w.w = o[db][4 * b + 3];
        *(float4*)(po + db * 32 + 8 * b + 4 * hi) = w;
      }
    if (hi == 0) {
      P.part_ml[slot * 2 + 0] = m_run;
      P.part_ml[slot * 2 + 1] = l_tot;
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
    dim3 grid((unsigned)(n * ls.Hkv));
    if (ls.D == 128)
      hipLaunchKernelGGL(attn_fwd_kernel<128>, grid, dim3(512), 0, st, P);
    else
      hipLaunchKernelGGL(attn_fwd_kernel<64>, grid, dim3(512), 0, st, P);
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
