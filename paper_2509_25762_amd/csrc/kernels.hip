// gfx950 kernels: ragged chunked-prefill attention, split-KV merge, KV append.
//
// Attention (per workgroup = one AttnItem x one kv-head), 8 waves of 64 lanes:
//   * the query tile packs TM tokens x G q-heads of the kv-head into 256 rows
//     (row r = head r % G of token r / G);
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

#include <mutex>
#include <type_traits>
#include <vector>

#include "oppo_internal.h"

namespace oppo {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(2))) int i32x2;
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(8))) int i32x8;

struct AttnParams {
  const uint16_t* q;
  uint16_t* k;             // keys / values: the cache, or the packed sequences of a one-shot prefill
  uint16_t* v;
  const uint16_t* k_new;   // appending variant only: the chunk's keys / values, rows indexed like q
  const uint16_t* v_new;
  uint16_t* out;
  float* part_o;
  float* part_ml;
  int32_t Hq, Hkv, G, TM;
  float c;
  float out_scale;     // 8-bit cache: the value tensor's scale (the output is the weighted mean of codes times it)
  float q_mult;        // 8-bit cache: c * 2^k, what the queries are multiplied by before they are rounded to E4M3
  int32_t q_scale_byte;   // ... and the E8M0 code of 2^-k (127 - k), the query operand's scale in the MFMA
  int32_t n_queues;
  uint32_t g_magic;    // ceil(2^16 / G): r / G == (r * g_magic) >> 16 for the rows r < 256 of a packed tile
  uint16_t first[kMaxQueues + 1];   // queue j runs pieces first[j] .. first[j+1]-1, in that order
  AttnItem items[kMaxAttnItems];
};
static_assert(sizeof(AttnParams) <= 32768, "kernel arguments are kept within 32 KiB");

struct CombineParams {
  uint16_t* out;
  const float* part_o;
  const float* part_ml;
  int32_t Hq, Hkv, G, TM;
  float c;
  float out_scale;     // 1, or the value tensor's scale of an 8-bit cache
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

__device__ __forceinline__ s16x4 lds_read_tr16_l(const __attribute__((address_space(3))) unsigned char* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p));
}

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
// M0 is written here.  It is a reserved register: the compiler sets it before each of its
// own uses (LDS-DMA and GWS instructions, of which this kernel has none besides these), and
// it refuses M0 on a clobber list ("reserved register ... may lead to undefined behaviour"),
// so none is given.  The LDS addresses this produces are pinned by every GPU parity test.
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

// Eight bf16 values times `mult` -> eight E4M3 codes (round to nearest even; products beyond the
// format's largest finite value, 448, are clamped to it first), element i in byte i.
__device__ __forceinline__ long bf16x8_to_fp8x8(bf16x8 x, float mult) {
  union { bf16x8 v; uint32_t w[4]; } u;
  u.v = x;
  int lo = 0, hi = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float a = __builtin_amdgcn_fmed3f(__uint_as_float(u.w[i] << 16) * mult, -448.0f, 448.0f);
    const float b = __builtin_amdgcn_fmed3f(__uint_as_float(u.w[i] & 0xffff0000u) * mult, -448.0f, 448.0f);
    // (the half of the word that is written has to be a literal)
    if (i == 0) lo = __builtin_amdgcn_cvt_pk_fp8_f32(a, b, lo, false);
    else if (i == 1) lo = __builtin_amdgcn_cvt_pk_fp8_f32(a, b, lo, true);
    else if (i == 2) hi = __builtin_amdgcn_cvt_pk_fp8_f32(a, b, hi, false);
    else hi = __builtin_amdgcn_cvt_pk_fp8_f32(a, b, hi, true);
  }
  return (long)(((unsigned long)(uint32_t)hi << 32) | (unsigned long)(uint32_t)lo);
}

// Persistent workgroups: the launch has one workgroup per (queue, kv-head), about
// one per compute unit, and workgroup (queue j, kv-head g) runs the pieces
// first[j] .. first[j+1]-1 of the work list one after the other.
// Eight waves, each owning 32 query columns of the 256-row tile; two waves share
// a SIMD.  On this hardware vector ALU instructions hide under MFMAs only when
// the two are mixed finely (a handful of vector instructions per MFMA), so the
// instruction stream is laid out by hand and fenced with sched_barrier: see the
// main loop.  Operand fragments are read from LDS several steps before the MFMA
// that consumes them (rolling register buffers ka / vf).
// K/V tiles go straight from global memory into a ring of four LDS stages, two
// tiles ahead: the loads of the tile two places further down the workgroup's
// tile stream are issued after the barrier that opens an iteration, into the
// stage whose last reader finished before that barrier, and each wave waits for
// its own loads before the barrier that closes it.  The stream runs across piece
// boundaries: the first two tiles of the next piece are requested during the last
// two iterations of the current one, and the next piece's Q fragments are
// requested as soon as the current piece's last S^T MFMA has been issued.
// APPEND: the chunk's own keys and values are not in the cache yet.  The key loop
// takes them from k_new / v_new, and the piece that starts a query tile's key
// range also copies the tile's token rows into the cache (nothing in this launch
// reads those cache rows).
template <int D, bool APPEND>
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
  constexpr int KDEPTH = KK / 2;     // K fragments kept in flight (half a unit ahead: four MFMA steps cover the
                                     // LDS latency several times over, and a whole unit costs 16 more registers)
  constexpr int VDEPTH = DB;         // V^T fragments kept in flight
  static_assert(IPW >= 1 && NT == 512, "tile smaller than the workgroup");

  // K stages and V stages are two arrays of at most 64 KiB each, so that every
  // fragment read is "per-lane base register + immediate offset" (the LDS
  // instructions take 16-bit offsets)
  __shared__ __attribute__((aligned(1024))) unsigned char sk[NSTAGE][TILE_BYTES];
  __shared__ __attribute__((aligned(1024))) unsigned char sv[NSTAGE][TILE_BYTES];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int l32 = lane & 31;
  const int hi = lane >> 5;
  const int Hq = P.Hq, Hkv = P.Hkv, G = P.G, TM = P.TM;
  const int kvh = blockIdx.x % Hkv;
  const int queue = blockIdx.x / Hkv;
  const int p_first = P.first[queue];
  const int p_last = P.first[queue + 1];
  if (p_first >= p_last) return;
  const float c = P.c;

  // The queue's piece descriptors are copied from the kernel-argument segment into
  // LDS once: a read of that segment costs microseconds, far too much to pay at
  // every piece boundary.
  __shared__ __attribute__((aligned(16))) AttnItem spiece[kMaxAttnItems];
  {
    const u32x4* src = (const u32x4*)(P.items + p_first);
    const int n16 = (p_last - p_first) * (int)(sizeof(AttnItem) / 16);
    for (int i = tid; i < n16; i += NT) ((u32x4*)spiece)[i] = src[i];
    __syncthreads();
  }
  // descriptor of piece p (a wave-uniform value, moved to scalar registers)
  auto piece = [&](int p) __attribute__((always_inline)) -> AttnItem {
    const u32x4* w = (const u32x4*)&spiece[p - p_first];
    const u32x4 a = w[0], b = w[1];
    AttnItem r;
    r.kv_row0 = (int64_t)(((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)a[1]) << 32) |
                          (uint32_t)__builtin_amdgcn_readfirstlane((int)a[0]));
    r.q_row0 = __builtin_amdgcn_readfirstlane((int)a[2]);
    r.n_tok = __builtin_amdgcn_readfirstlane((int)a[3]);
    r.pos0 = __builtin_amdgcn_readfirstlane((int)b[0]);
    r.k_begin = __builtin_amdgcn_readfirstlane((int)b[1]);
    r.k_end = __builtin_amdgcn_readfirstlane((int)b[2]);
    r.part = __builtin_amdgcn_readfirstlane((int)b[3]);
    return r;
  };

  // ---- this lane's query column (row of the packed (token, head) tile) --------------
  bf16x8 qf[KK];

  // ---- cooperative K/V tile loads ------------------------------------------------
  // Tiles travel global -> LDS directly (global_load_lds_dwordx4): a wave-wide
  // load drops 64 x 16 bytes at consecutive LDS addresses, i.e. RPI whole rows;
  // the LDS swizzle is applied by choosing which 16-byte granule of the row each
  // lane fetches.  Wave w moves rows (w + 8i) * RPI .. of the tile.
  const int row_stride = Hkv * D;  // elements between consecutive tokens
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

  // ---- the wave's staging area: turning 32 x D blocks around ----------------------
  // A lane owns one query column, so its share of Q (a B operand) and of the output
  // is 16-byte / 8-byte pieces of one row: moved to and from global memory like
  // that, every instruction would touch 32 or 64 different rows.  Q and O blocks
  // therefore travel as whole row pieces (16 bytes per lane, consecutive lanes on
  // consecutive addresses) and are turned around in LDS, half of D at a time.  The
  // staging area is the part of a ring stage that this very wave fills with its
  // next tile request (2*IPW chunks of 1 KiB), used at a time when the stage's last
  // readers have passed a barrier: no other wave is involved, no barrier needed.
  constexpr int RB = D;             // bytes of a row per round (half a row)
  constexpr int NS = RB / 16;       // 16-byte slots of a row per round
  constexpr int RPC = 1024 / RB;    // rows per 1 KiB chunk
  typedef __attribute__((address_space(3))) unsigned char* lds_ptr;
  // The lane-dependent offsets below are needed at piece boundaries only.  They are
  // derived from a copy of the lane number that the optimiser cannot see through,
  // so that it recomputes them there instead of keeping them in registers (which
  // the key loop has none to spare) for the whole kernel.
  auto lane_now = [&]() __attribute__((always_inline)) -> int {
    int x = lane;
    asm volatile("" : "+v"(x));
    return x;
  };
  // row-piece side: lane ln handles slot ln % NS of row ln / NS of each chunk
  auto roff_of = [&](int ln) __attribute__((always_inline)) -> uint32_t {
    return (uint32_t)((ln / NS) * RB + (((ln % NS) ^ ((ln / NS) & (NS - 1))) * 16));
  };
  // column side: the row of lane ln, (ln & 31), lies in chunk (ln & 31) / RPC; cx_of = its swizzle
  auto cx_of = [&](int ln) __attribute__((always_inline)) -> uint32_t { return (uint32_t)(ln & (NS - 1)) * 16u; };
  auto area_of = [&](int stage, int k) __attribute__((always_inline)) -> uint32_t {   // chunk k of the area in `stage`
    return ((k / IPW) ? lds_addr_of(&sv[0][0]) : lds_addr_of(&sk[0][0])) + (uint32_t)stage * TILE_BYTES + wave_rows +
           (uint32_t)((k % IPW) * 8192);
  };
  auto carea_of = [&](int stage, int ln) __attribute__((always_inline)) -> uint32_t {   // the row of lane ln in its chunk
    const int row = ln & 31;
    return (((row / RPC) / IPW) ? lds_addr_of(&sv[0][0]) : lds_addr_of(&sk[0][0])) + (uint32_t)stage * TILE_BYTES + wave_rows +
           (uint32_t)(((row / RPC) % IPW) * 8192 + (row % RPC) * RB);
  };
  // rows wave*32 + k*RPC + ln/NS of the packed tile -> (q-head of the group, token):
  // row R is head R % G of token R / G, so the rows of a tile of n tokens are the
  // first n * G ones (and rows from TM * G on, if G does not divide 256, are never used)
  auto row_of = [&](int ln, int k, int* hk, int* tk) __attribute__((always_inline)) {
    const int R = (int)(wave_rows >> 10) * 32 + ln / NS + k * RPC;   // (wave number as a scalar)
    const int t = (int)(((uint32_t)R * P.g_magic) >> 16);            // R / G
    *tk = t;
    *hk = R - t * G;
  };
  u32x4 qraw[2][2 * IPW];   // Q row pieces on their way: [half of D][chunk]
  auto q_request = [&](const AttnItem& a) __attribute__((always_inline)) {
    const int ln = lane_now();
#pragma unroll
    for (int k = 0; k < 2 * IPW; ++k) {
      int hk, tk;
      row_of(ln, k, &hk, &tk);
      // rows beyond the tile repeat a valid row; their columns are never stored
      const uint16_t* qp = P.q + ((int64_t)(a.q_row0 + min(tk, tokens_of(a) - 1)) * Hq + kvh * G + hk) * D + (ln % NS) * 8;
#pragma unroll
      for (int h = 0; h < 2; ++h) qraw[h][k] = *(const u32x4*)(qp + h * (D / 2));
    }
  };
  auto q_collect = [&](int stage) __attribute__((always_inline)) {
    const int ln = lane_now();
    const uint32_t roff = roff_of(ln);
    const uint32_t cbase = carea_of(stage, ln);
    const uint32_t cxh = cx_of(ln) ^ ((uint32_t)(ln >> 5) * 16u);   // the lane's slots are 2*kl + hi, swizzled
#pragma unroll
    for (int h = 0; h < 2; ++h) {
#pragma unroll
      for (int k = 0; k < 2 * IPW; ++k)
        *(__attribute__((address_space(3))) u32x4*)(lds_ptr)(uintptr_t)(area_of(stage, k) + roff) = qraw[h][k];
#pragma unroll
      for (int kl = 0; kl < KK / 2; ++kl)
        qf[h * (KK / 2) + kl] = *(const __attribute__((address_space(3))) bf16x8*)(lds_ptr)(uintptr_t)(
            cbase + ((uint32_t)(kl * 32) ^ cxh));
    }
  };
  // The request cursor walks the workgroup's tile stream (all tiles of piece
  // p_first, then of the next piece, ...): all of it is wave-uniform.
  int c_piece = p_first;        // piece of the next tile to request
  int c_left = 0;               // keys of that piece not requested yet
  int c_cached = 0;             // APPEND: how many of them (counted from the next tile on) are in the cache
  // first row of the next tile, this kv-head, as a byte address in k, and (APPEND) where
  // that row would be in k_new; the v addresses are a fixed distance away
  uintptr_t c_k = 0, c_kn = 0;
  const uintptr_t k_to_v = (uintptr_t)P.v - (uintptr_t)P.k;
  const uintptr_t kn_to_vn = APPEND ? (uintptr_t)P.v_new - (uintptr_t)P.k_new : 0;
  const uintptr_t tile_step = (uintptr_t)BN * row_stride * 2u;
  auto cursor_open = [&]() __attribute__((always_inline)) {
    const AttnItem a = piece(c_piece);
    c_k = (uintptr_t)(P.k + (((int64_t)a.kv_row0 + a.k_begin) * Hkv + kvh) * D);
    c_left = a.k_end - a.k_begin;
    if (APPEND) {
      const int j0 = tile_of(a) * TM;          // the tile's first token within its chunk
      c_cached = (a.pos0 - j0) - a.k_begin;    // keys before the chunk are cached
      c_kn = (uintptr_t)(P.k_new + (((int64_t)(a.q_row0 - j0) - c_cached) * Hkv + kvh) * D);
    }
  };
  cursor_open();
  auto issue_next = [&](int stage) __attribute__((always_inline)) {
    if (c_piece >= p_last) return;
    const int last = c_left - 1;
    // (LDS addresses are formed here from a copy of the wave's offset that the optimiser
    // cannot see through: otherwise it keeps one precomputed address per stage, array and
    // load in scalar registers for the whole kernel, and those run out)
    uint32_t wave_rows_now = wave_rows;
    asm volatile("" : "+s"(wave_rows_now));
    if (APPEND && c_cached > 0 && c_cached < BN && c_cached <= last) {
      // cache rows, then chunk rows: each lane's 16 bytes land at the LDS address of its
      // lane number, so the two sources fill one tile with complementary lane masks
#pragma unroll
      for (int i = 0; i < IPW; ++i) {
        const int r = (wave + 8 * i) * RPI + lrow;
        const int rc = min(r, last);   // rows past the range repeat the last key
        const uint32_t ok = (uint32_t)(rc * row_stride + ((pg ^ (r % NG)) * 8)) * 2u;
        const uint32_t ov = (uint32_t)(rc * row_stride + ((pg ^ ((r & VSWZ_MASK) << 2)) * 8)) * 2u;
        const uint32_t lk = lds_addr_of(&sk[stage][0]) + wave_rows_now + i * 8192u;
        const uint32_t lv = lds_addr_of(&sv[stage][0]) + wave_rows_now + i * 8192u;
        if (rc < c_cached) {
          async_copy16((const void*)c_k, ok, lk);
          async_copy16((const void*)(c_k + k_to_v), ov, lv);
        } else {
          async_copy16((const void*)c_kn, ok, lk);
          async_copy16((const void*)(c_kn + kn_to_vn), ov, lv);
        }
      }
    } else {
      const bool all_new = APPEND && c_cached <= 0;
      const uintptr_t bk = all_new ? c_kn : c_k;
      const uintptr_t bv = bk + (all_new ? kn_to_vn : k_to_v);
#pragma unroll
      for (int i = 0; i < IPW; ++i) {
        uint32_t ok = goffk[i], ov = goffv[i];
        if (last < BN - 1) {  // ragged last tile: rows past the range repeat the last key
          const int r = (wave + 8 * i) * RPI + lrow;
          const int rc = min(r, last);
          ok = (uint32_t)(rc * row_stride + ((pg ^ (r % NG)) * 8)) * 2u;
          ov = (uint32_t)(rc * row_stride + ((pg ^ ((r & VSWZ_MASK) << 2)) * 8)) * 2u;
        }
        async_copy16((const void*)bk, ok, lds_addr_of(&sk[stage][0]) + wave_rows_now + i * 8192u);
        async_copy16((const void*)bv, ov, lds_addr_of(&sv[stage][0]) + wave_rows_now + i * 8192u);
      }
    }
    c_k += tile_step;
    if (APPEND) {
      c_kn += tile_step;
      c_cached -= BN;
    }
    c_left -= BN;
    if (c_left <= 0) {
      ++c_piece;
      if (c_piece < p_last) cursor_open();
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
  // per-lane base pointers; stage, key half and group then are immediate offsets
  // (made opaque to the optimiser, which would otherwise fold the array address
  // into each read and rebuild the sum with a vector instruction every time)
  typedef const __attribute__((address_space(3))) unsigned char* lds_cptr;
  lds_cptr kptr[KK];   // K fragment of k-step kk, key block 0 (block 1 is +32 rows)
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) {
    uint32_t a = lds_addr_of(&sk[0][0]) + (uint32_t)(l32 * ROWB + (((kk * 2 + hi) ^ (l32 % NG)) * 16));
    asm volatile("" : "+v"(a));
    kptr[kk] = (lds_cptr)(uintptr_t)a;
  }
  lds_cptr vptr[DB];   // V^T fragment of d-block db, keys 4*hi.. of a 16-key group
  {
    const int j = lane & 15;
    const int half16 = (lane >> 4) & 1;
    const int vrow = 4 * hi + (j >> 2);
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      const int lg = db * 4 + 2 * half16 + ((j & 3) >> 1);
      uint32_t a = lds_addr_of(&sv[0][0]) + (uint32_t)(vrow * ROWB + ((lg ^ ((vrow & VSWZ_MASK) << 2)) * 16) + (j & 1) * 8);
      asm volatile("" : "+v"(a));
      vptr[db] = (lds_cptr)(uintptr_t)a;
    }
  }
  // K fragment (A operand of S^T = K Q^T): keys kb*32 + l32, elements kk*16 + 8*hi..;
  // `off` = stage * TILE_BYTES (an immediate in the main loop)
  auto ldk = [&](int off, int kb, int kk) __attribute__((always_inline)) -> bf16x8 {
    return *(const __attribute__((address_space(3))) bf16x8*)(kptr[kk] + off + kb * 32 * ROWB);
  };
  // V^T fragment (A operand of O^T += V^T P^T) of step j = (16-key group, d-block)
  // of the 32-key unit (stage, kb)
  auto ldv = [&](int off, int kb, int j) __attribute__((always_inline)) -> bf16x8 {
    lds_cptr vp = vptr[j % DB] + off + (2 * kb + j / DB) * 16 * ROWB;
    union { struct { s16x4 a, b; } h; bf16x8 v; } cat;
    cat.h.a = lds_read_tr16_l(vp);
    cat.h.b = lds_read_tr16_l(vp + 8 * ROWB);
    return cat.v;
  };

  // A column's reference value m_run (the "running max" of the online softmax) is
  // only moved when the partial row sum of a 32-key unit exceeds 2^24: the weights
  // stay far inside the fp32 / bf16 range, relative precision does not depend on
  // the reference, and the maximum is not needed on the common path.
  constexpr float kRowSumLimit = 16777216.0f;
  const bf16x2 ones2 = {(__bf16)1.0f, (__bf16)1.0f};

  // ------------------------------------------------------------------------------
  // Main loop, software-pipelined over 32-key units (two per 64-key tile).  The
  // body of unit u issues, interleaved instruction by instruction,
  //   * the MFMAs of S^T for unit u+1            (one dependent chain),
  //   * the MFMAs of O^T += V^T P^T for unit u-1 (DB independent chains),
  //   * the exp2 / bf16 rounding / row-sum vector work of unit u,
  // so the matrix pipe always has an independent MFMA to run and the vector ALU
  // work (about three instructions per MFMA) is spread evenly under it.
  constexpr int QS = KK;          // S^T MFMAs per unit
  constexpr int PS = 2 * DB;      // O^T MFMAs per unit
  constexpr int PPS = 8 / QS;     // probability pairs handled per step
  static_assert(QS == PS && QS % KDEPTH == 0 && PS % VDEPTH == 0, "pipeline shape");

  f32x16 o[DB];
  f32x16 s[2];                                   // s[u & 1] = S^T of unit u
  bf16x8 ka[KDEPTH];                             // K fragments in flight: step j of a unit sits in ka[j % KDEPTH]
  bf16x8 vf[VDEPTH];                             // V^T fragments in flight, likewise
  union { bf16x2 h[8]; bf16x8 v[2]; } pf[2];     // pf[u & 1] = probabilities of unit u, B-operand layout
  float m_run, l_run, mc, rs0 = 0.f, rs1 = 0.f;

  // state of the piece being computed
  AttnItem it = piece(p_first);
  int lim = 0;       // last key this lane's column may see, minus 4 * (lane / 32): compared with the key
                     // of the lane's register r of the other 32-lane half, see the mask in unit_body
  int min_lim = 0;   // smallest such limit in the workgroup: units entirely below it need no mask

  // probabilities 2p, 2p+1 of the unit in s[cur]: exp2, round to bf16, add to the
  // row sum (the sum uses the rounded values, like the numerator does)
  // The empty asm statement pins the work to its place in the instruction stream: the
  // results are "used" by it, and such statements keep their order.  (The inputs are read
  // from the score registers as they are: a statement that "defines" them as well costs a
  // register copy per score, because the scores have to survive for a possible redo.)
  auto exp_pair = [&](int cur, int pr) __attribute__((always_inline)) {
    const float x0 = s[cur][2 * pr], x1 = s[cur][2 * pr + 1];
    const float p0 = fast_exp2(fmaf(x0, c, -mc));
    const float p1 = fast_exp2(fmaf(x1, c, -mc));
    bf16x2 pk;
    pk[0] = (__bf16)p0;
    pk[1] = (__bf16)p1;
    if (pr & 1) {
      rs1 = __builtin_amdgcn_fdot2_f32_bf16(pk, ones2, rs1, false);
      asm volatile("" : "+v"(pk), "+v"(rs1));
    } else {
      rs0 = __builtin_amdgcn_fdot2_f32_bf16(pk, ones2, rs0, false);
      asm volatile("" : "+v"(pk), "+v"(rs0));
    }
    pf[cur].h[pr] = pk;
  };

  // Body of unit u.  BC = position of the unit in the LDS ring (stage, key half),
  // a compile-time value, so that every fragment read has an immediate offset.
  auto unit_body = [&](auto BC, int u) __attribute__((always_inline)) {
    constexpr int b = decltype(BC)::value;
    constexpr int st_c = b / 2, kb_c = b % 2;                   // unit u
    constexpr int st_n = ((b + 1) % 8) / 2, kb_n = (b + 1) % 2; // unit u+1
    constexpr int st_nn = ((b + 2) % 8) / 2, kb_nn = b % 2;     // unit u+2
    constexpr int st_p = ((b + 7) % 8) / 2, kb_p = (b + 7) % 2; // unit u-1
    constexpr int cur = b % 2, nxt = cur ^ 1;

    // ---- causal / range mask on units that cross a limit -------------------------
    const int key0 = it.k_begin + 32 * u;
    if (key0 + 31 > min_lim) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        // register r holds key key0 + 8 * (r / 4) + 4 * (lane / 32) + r % 4
        if (key0 + 8 * (r >> 2) + (r & 3) > lim) s[cur][r] = -INFINITY;
      }
    }
    // The probabilities of this unit are formed against the reference value m_run
    // the column already has (no maximum is taken first); only if a row sum comes
    // out too large - always for a column's first visible keys, otherwise almost
    // never - the unit is redone against its true maximum, see below.
    rs0 = 0.f;
    rs1 = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) s[nxt][r] = 0.f;

#pragma unroll
    for (int i = 0; i < QS; ++i) {
      s[nxt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[i % KDEPTH], qf[i], s[nxt], 0, 0, 0);
      ka[i % KDEPTH] = (i + KDEPTH < QS) ? ldk(st_n * TILE_BYTES, kb_n, i + KDEPTH)
                                         : ldk(st_nn * TILE_BYTES, kb_nn, i + KDEPTH - QS);
      o[i % DB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[i % VDEPTH], pf[nxt].v[i / DB], o[i % DB], 0, 0, 0);
      vf[i % VDEPTH] = (i + VDEPTH < PS) ? ldv(st_p * TILE_BYTES, kb_p, i + VDEPTH)
                                         : ldv(st_c * TILE_BYTES, kb_c, i + VDEPTH - PS);
#pragma unroll
      for (int jj = 0; jj < PPS; ++jj) exp_pair(cur, i * PPS + jj);
      // within the step: an MFMA, the K fragment read, half of the vector work, the
      // other MFMA, the two transposed V reads, the rest of the vector work
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x402, 3 * PPS, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
      __builtin_amdgcn_sched_group_barrier(0x402, 3 * PPS, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    float rs = rs0 + rs1;
    // pin the vector work above to this block: without a use here the compiler
    // sinks it below the branch that follows, away from the MFMAs it should hide under
    asm volatile("" : "+v"(pf[cur].v[0]), "+v"(pf[cur].v[1]), "+v"(rs));
    __builtin_amdgcn_sched_barrier(0);
    if (u == 0) {
      // the O^T MFMAs of a piece's first body belong to no unit (zero probabilities
      // times whatever the ring stage held): the accumulation starts here
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[db][r] = 0.f;
    }
    if (__any(rs > kRowSumLimit)) {
      // Some column saw a score far above its reference (or has no reference yet):
      // take the unit's true maximum (one query column per lane, its key halves in
      // lanes l and l^32), move every column's reference up to it, redo the unit's
      // probabilities, and rescale what has been accumulated so far - unit u-1
      // included, whose MFMAs above still used the old reference.
      float mx4[4];
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4)
        mx4[q4] = fmaxf(fmaxf(fmaxf(s[cur][q4], s[cur][4 + q4]), s[cur][8 + q4]), s[cur][12 + q4]);
      float mx = fmaxf(fmaxf(fmaxf(mx4[0], mx4[1]), mx4[2]), mx4[3]);
      mx = fmaxf(mx, swap_halves(mx));
      const float m_new = fmaxf(m_run, mx);
      const float alpha = fast_exp2((m_run - m_new) * c);
      m_run = m_new;
      mc = m_run * c;
      l_run *= alpha;
      rs0 = 0.f;
      rs1 = 0.f;
#pragma unroll
      for (int pr = 0; pr < 8; ++pr) exp_pair(cur, pr);
      rs = rs0 + rs1;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[db][r] *= alpha;
    }
    l_run += rs;
  };

  // iteration = one tile = units 2t and 2t+1 of the piece (U units in all); TC is
  // the tile's ring stage.  The tile two places down the stream is requested at
  // its start and awaited at its end, before the barrier after which the next
  // iteration starts reading the tile in between.
  int U = 0;
  // A wave whose 32 rows all lie beyond the tile's tokens (a short tile fills the
  // first n_tok * G rows only) does none of the arithmetic of the piece: it still
  // requests its share of every key tile and joins the barriers, and leaves the
  // matrix and vector units of its SIMD to the waves that have rows.
  auto has_rows = [&](const AttnItem& a) __attribute__((always_inline)) -> bool {
    return (int)(wave_rows >> 10) * 32 < tokens_of(a) * G;
  };
  bool act = true;
  auto iteration = [&](auto TC, int t) __attribute__((always_inline)) {
    constexpr int ts = decltype(TC)::value;
    issue_next((ts + 2) % NSTAGE);
    unit_body(std::integral_constant<int, 2 * ts>{}, 2 * t);
    if (2 * t + 1 < U) unit_body(std::integral_constant<int, 2 * ts + 1>{}, 2 * t + 1);
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wave's share of the requested tile is in LDS
    wg_barrier();
  };

  // ---- start-up: Q of the first piece, the first two tiles of the stream ------------
  act = has_rows(it);
  q_request(it);
  issue_next(0);
  issue_next(1);
  q_collect(2);
  // Everything issued so far must have landed before the loop; a wait left to the
  // compiler would sit inside the loop, where it would also cover later tiles.
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
  wg_barrier();

  int ph = 0;   // ring stage of the current piece's first tile
  for (int p = p_first;;) {
    // (per-lane values that only matter here are recomputed from an opaque copy of the
    // lane number, see lane_now)
    const int ln_top = lane_now();
    const int r_tile = (int)(wave_rows >> 10) * 32 + (ln_top & 31);   // the lane's row of the packed tile
    const int tok = (int)(((uint32_t)r_tile * P.g_magic) >> 16);     // its token within the tile (r_tile / G)
    const int tokc = min(tok, tokens_of(it) - 1);
    lim = min(it.pos0 + tokc, it.k_end - 1) - 4 * (ln_top >> 5);
    min_lim = min(it.pos0, it.k_end - 1);
    const int nkeys = it.k_end - it.k_begin;
    const int nt = (nkeys + BN - 1) / BN;
    U = (nkeys + 31) / 32;
    m_run = -1e30f;
    l_run = 0.f;
    {
      float c_now = c;
      asm volatile("" : "+s"(c_now));
      mc = m_run * c_now;
    }
    // the accumulators start undefined (they are cleared after the first body, see
    // unit_body); saying so ends their live range at the previous piece's epilogue
#pragma unroll
    for (int db = 0; db < DB; ++db) asm volatile("" : "=v"(o[db]));

    // Whatever this wave still has in flight (the previous piece's stores, the tiles
    // requested ahead) is awaited here, on the path of every wave: left to the compiler,
    // the wait for the stores ends up inside the key loop, where it would cover each
    // newly requested tile as well.
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    // S^T of unit 0 on its own, then the operand buffers as the first body expects
    // them.  The ring stage is a run-time value here (and only here and in the drain).
    if (act) {
      const int off0 = ph * TILE_BYTES;
      const int offm = ((ph + 3) & 3) * TILE_BYTES;   // "unit -1": any stage, see unit_body
#pragma unroll
      for (int j = 0; j < KDEPTH; ++j) ka[j] = ldk(off0, 0, j);
#pragma unroll
      for (int r = 0; r < 16; ++r) s[0][r] = 0.f;
      // ring position of unit 0 is 2*ph: s[] and pf[] are indexed by its parity, 0
#pragma unroll
      for (int i = 0; i < QS; ++i) {
        s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[i % KDEPTH], qf[i], s[0], 0, 0, 0);
        ka[i % KDEPTH] = (i + KDEPTH < QS) ? ldk(off0, 0, i + KDEPTH) : ldk(off0, 1, i + KDEPTH - QS);
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int j = 0; j < VDEPTH; ++j) vf[j] = ldv(offm, 1, j);
      const bf16x2 z2 = {(__bf16)0.0f, (__bf16)0.0f};
#pragma unroll
      for (int j = 0; j < 8; ++j) pf[1].h[j] = z2;
    }

    // tiles of the piece, the loop unrolled over the four ring stages
    const int tau1 = ph + nt;
    if (act) {
      for (int tb = 0; tb < tau1; tb += 4) {
        if (tb >= ph) iteration(std::integral_constant<int, 0>{}, tb - ph);
        if (tb + 1 >= ph && tb + 1 < tau1) iteration(std::integral_constant<int, 1>{}, tb + 1 - ph);
        if (tb + 2 >= ph && tb + 2 < tau1) iteration(std::integral_constant<int, 2>{}, tb + 2 - ph);
        if (tb + 3 >= ph && tb + 3 < tau1) iteration(std::integral_constant<int, 3>{}, tb + 3 - ph);
      }
    } else {
      // (the same requests, waits and barriers as `iteration`, nothing else)
      for (int t = 0; t < nt; ++t) {
        issue_next((ph + t + 2) & 3);
        __builtin_amdgcn_s_waitcnt(0x0F70);
        wg_barrier();
      }
    }

    // request the next piece's Q rows; they are collected after the epilogue
    const AttnItem done = it;
    const bool more = p + 1 < p_last;
    if (more) {
      it = piece(p + 1);
      act = has_rows(it);
      q_request(it);
    } else {
      // (defined on every path, so that the values are not kept alive across the key loop)
#pragma unroll
      for (int k = 0; k < 2 * IPW; ++k) qraw[0][k] = qraw[1][k] = u32x4{0u, 0u, 0u, 0u};
    }
    const int st_area = (ph + nt + 2) & 3;   // the stage the next tile request goes to

    // APPEND: the piece that starts the tile's key range moves the tile's token rows
    // (this kv-head's D elements of each) from k_new / v_new into the cache, 16 bytes
    // per thread and pass of CP_ROWS rows.  The first two passes are requested here
    // and stored after the epilogue; query tiles of more than 2 * CP_ROWS tokens
    // finish in a plain loop.  The data waits in the registers of s[1], which the
    // key loop no longer needs and the next piece's first body clears.
    constexpr int CP_ROWS = NT / NG;   // token rows per pass
    const bool cp_on = APPEND && done.k_begin == 0;
    const int cp_tid = (int)(wave_rows >> 4) + lane_now();   // thread number, recomputed here
    const int cp_row = cp_tid / NG, cp_g = cp_tid % NG;
    auto cp_src = [&](int row) __attribute__((always_inline)) -> int64_t {
      return (((int64_t)done.q_row0 + row) * Hkv + kvh) * D + cp_g * 8;
    };
    auto cp_dst = [&](int row) __attribute__((always_inline)) -> int64_t {
      return (((int64_t)done.kv_row0 + done.pos0 + row) * Hkv + kvh) * D + cp_g * 8;
    };
    auto park = [&](int slot, const u32x4& x) __attribute__((always_inline)) {
#pragma unroll
      for (int e = 0; e < 4; ++e) s[1][4 * slot + e] = __uint_as_float(x[e]);
    };
    auto unpark = [&](int slot) __attribute__((always_inline)) -> u32x4 {
      u32x4 x;
#pragma unroll
      for (int e = 0; e < 4; ++e) x[e] = __float_as_uint(s[1][4 * slot + e]);
      return x;
    };
    if (cp_on) {
#pragma unroll
      for (int ps = 0; ps < 2; ++ps) {
        const int row = ps * CP_ROWS + cp_row;
        if (row < tokens_of(done)) {
          park(2 * ps, *(const u32x4*)(P.k_new + cp_src(row)));
          park(2 * ps + 1, *(const u32x4*)(P.v_new + cp_src(row)));
        }
      }
    }

    // ---- drain: O^T += V^T P^T of the last unit ----------------------------------------
    {
      const int ul = U - 1;
      const int off = (((ul >> 1) + ph) & 3) * TILE_BYTES;
      const int kb = ul & 1;
      // the fragments preloaded by the last body belong to this unit already; its
      // probabilities are pf[ul & 1] (picked as values: an array indexed at run time
      // would be put into scratch memory)
      bf16x8 e0 = pf[0].v[0], e1 = pf[0].v[1], d0 = pf[1].v[0], d1 = pf[1].v[1];
      asm volatile("" : "+v"(e0), "+v"(e1), "+v"(d0), "+v"(d1));
      const bool odd = (ul & 1) != 0;
      const bf16x8 pl[2] = {odd ? d0 : e0, odd ? d1 : e1};
#pragma unroll
      for (int i = 0; i < PS; ++i) {
        o[i % DB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[i % VDEPTH], pl[i / DB], o[i % DB], 0, 0, 0);
        if (i + VDEPTH < PS) vf[i % VDEPTH] = ldv(off, kb, i + VDEPTH);
      }
    }

    // ---- epilogue ---------------------------------------------------------------------
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    if (done.part < 0) {
      // final rows, turned around in the wave's staging area.  They (and the appended cache
      // rows further down) are stored with the non-temporal hint: nothing in this launch reads
      // them again, and lines that do not linger dirty in the level-2 cache need no write-back
      // when the kernel ends.
      const float inv = 1.0f / l_tot;
      const int ln = lane_now();
      const uint32_t roff = roff_of(ln), cx = cx_of(ln);
      const uint32_t wbase = carea_of(st_area, ln) + (uint32_t)(ln >> 5) * 8u;
      int grow[2 * IPW];                // head-row (token * Hq + head) of the row in out, -1: not a row of this tile
#pragma unroll
      for (int k = 0; k < 2 * IPW; ++k) {
        int hk, tk;
        row_of(ln, k, &hk, &tk);
        grow[k] = tk < tokens_of(done) ? (done.q_row0 + tk) * Hq + kvh * G + hk : -1;
      }
#pragma unroll
      for (int h = 0; h < 2; ++h) {
#pragma unroll
        for (int dbl = 0; dbl < DB / 2; ++dbl)
#pragma unroll
          for (int b = 0; b < 4; ++b) {
            bf16x4 w;
#pragma unroll
            for (int e = 0; e < 4; ++e) w[e] = (__bf16)(o[h * (DB / 2) + dbl][4 * b + e] * inv);
            *(__attribute__((address_space(3))) bf16x4*)(lds_ptr)(uintptr_t)(wbase + ((uint32_t)((dbl * 4 + b) * 16) ^ cx)) = w;
          }
#pragma unroll
        for (int k = 0; k < 2 * IPW; ++k) {
          const u32x4 val = *(const __attribute__((address_space(3))) u32x4*)(lds_ptr)(uintptr_t)(
              area_of(st_area, k) + roff);
          if (grow[k] >= 0) __builtin_nontemporal_store(val, (u32x4*)(P.out + (int64_t)grow[k] * D + (ln % NS) * 8 + h * (D / 2)));
        }
      }
    } else {
      const int lnp = lane_now();
      const int hip = lnp >> 5;
      const int64_t slot = ((int64_t)done.part * Hkv + kvh) * kTileRows + (int)(wave_rows >> 10) * 32 + (lnp & 31);
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
          *(float4*)(po + db * 32 + 8 * b + 4 * hip) = w;
        }
      if (hip == 0) {
        P.part_ml[slot * 2 + 0] = m_run;
        P.part_ml[slot * 2 + 1] = l_tot;
      }
    }
    if (cp_on) {
#pragma unroll
      for (int ps = 0; ps < 2; ++ps) {
        const int row = ps * CP_ROWS + cp_row;
        if (row < tokens_of(done)) {
          __builtin_nontemporal_store(unpark(2 * ps), (u32x4*)(P.k + cp_dst(row)));
          __builtin_nontemporal_store(unpark(2 * ps + 1), (u32x4*)(P.v + cp_dst(row)));
        }
      }
      for (int row = 2 * CP_ROWS + cp_row; row < tokens_of(done); row += CP_ROWS) {
        const u32x4 a = *(const u32x4*)(P.k_new + cp_src(row));
        const u32x4 b = *(const u32x4*)(P.v_new + cp_src(row));
        __builtin_nontemporal_store(a, (u32x4*)(P.k + cp_dst(row)));
        __builtin_nontemporal_store(b, (u32x4*)(P.v + cp_dst(row)));
      }
    }
    if (more) q_collect(st_area);
    if (!more) break;
    ++p;
    ph = (ph + nt) & 3;
  }
}

#include "attn_fp8_kernel.h"

// Merge the partial (max, sum, unnormalised O) of the pieces of a split tile
// (at most kMaxSplit pieces):
// out = sum_s w_s O_s / sum_s w_s l_s with w_s = exp2((m_s - max_s m_s) * c).
// MAXS: upper bound on the pieces of any tile of the launch (4, 8 or MAXS); the per-piece
// arrays live in registers, and fewer of them means more waves in flight to hide the loads.
template <int D, int MAXS>
__global__ __launch_bounds__(256) void combine_kernel(const CombineParams P) {
  constexpr int TPR = D / 4;          // threads per row (float4 each)
  constexpr int RPB = 256 / TPR;      // rows per block
  const CombineItem it = P.items[blockIdx.x / P.Hkv];
  const int kvh = blockIdx.x % P.Hkv;
  const int r = blockIdx.y * RPB + threadIdx.x / TPR;
  const int d4 = (threadIdx.x % TPR) * 4;
  const int tok = r / P.G;    // row r of the packed tile is head r % G of token r / G
  const int hh = r - tok * P.G;
  if (tok >= it.n_tok) return;
  // all loads of a batch are issued before the first use, so the merge is bound
  // by bandwidth and not by a chain of dependent memory latencies
  const int64_t slot0 = ((int64_t)it.part0 * P.Hkv + kvh) * kTileRows + r;
  const int64_t sstride = (int64_t)P.Hkv * kTileRows;   // slots between consecutive pieces
  float ms[MAXS], ls[MAXS];
#pragma unroll
  for (int s = 0; s < MAXS; ++s) {
    const bool on = s < it.nsplit;
    const float2 ml = on ? *(const float2*)(P.part_ml + (slot0 + s * sstride) * 2) : float2{-INFINITY, 0.f};
    ms[s] = ml.x;
    ls[s] = ml.y;
  }
  float m_max = -INFINITY;
#pragma unroll
  for (int s = 0; s < MAXS; ++s) m_max = fmaxf(m_max, ms[s]);
  float l = 0.f;
#pragma unroll
  for (int s = 0; s < MAXS; ++s) {
    ms[s] = (s < it.nsplit) ? fast_exp2((ms[s] - m_max) * P.c) : 0.f;   // now the weight of piece s
    l += ms[s] * ls[s];
  }
  float4 acc = {0.f, 0.f, 0.f, 0.f};
  constexpr int BATCH = MAXS < 8 ? MAXS : 8;
#pragma unroll
  for (int s0 = 0; s0 < MAXS; s0 += BATCH) {
    if (s0 >= it.nsplit) break;
    float4 x[BATCH];
#pragma unroll
    for (int j = 0; j < BATCH; ++j) {
      const int sj = min(s0 + j, it.nsplit - 1);   // clamped pieces carry weight 0 ... see below
      x[j] = *(const float4*)(P.part_o + (slot0 + sj * sstride) * D + d4);
    }
#pragma unroll
    for (int j = 0; j < BATCH; ++j) {
      const float w = (s0 + j < it.nsplit) ? ms[s0 + j] : 0.f;
      acc.x += w * x[j].x;
      acc.y += w * x[j].y;
      acc.z += w * x[j].z;
      acc.w += w * x[j].w;
    }
  }
  const float inv = P.out_scale / l;
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

// KV append into the 8-bit cache.  A bf16 value x becomes the E4M3 code nearest (ties to even)
// to clamp(fl32(x * inv_scale), -448, 448).  Keys keep the token-major order, one byte per
// element; values go into blocks of 64 tokens, [block][kv-head][element][token % 64], and what is
// left of the last block a run touches is filled with zero bytes.
// grid = (items, 64-token blocks the longest run touches, kv-heads); 2 * D threads.
struct Append8Params {
  uint8_t* cache_k;
  uint8_t* cache_v;
  const uint16_t* k_new;
  const uint16_t* v_new;
  float k_inv, v_inv;    // fl32(1 / scale) of the two tensors
  int32_t Hkv;
  int32_t n_items;
  AppendItem items[kMaxAppendItems];
};
static_assert(sizeof(Append8Params) <= 32768, "kernel arguments are kept within 32 KiB");

__device__ __forceinline__ float code_range(uint32_t bf16_bits, float inv) {
  return __builtin_amdgcn_fmed3f(__uint_as_float(bf16_bits << 16) * inv, -448.0f, 448.0f);
}

template <int D>
__global__ __launch_bounds__(2 * D) void kv_append_fp8_kernel(const Append8Params P) {
  constexpr int NT = 2 * D;       // one thread per (4 tokens, 8 elements) of a 64-token block
  constexpr int BLK = kKeyTile;   // tokens per value block
  constexpr int NG = D / 8;       // 16-byte granules of a bf16 row of one kv-head
  constexpr int LROW = BLK + 4;   // bytes per element row of the transposed block in LDS (padded: 17 dwords)
  __shared__ __attribute__((aligned(16))) uint32_t vt[D * LROW / 4];
  const AppendItem it = P.items[blockIdx.x];
  const int64_t first = it.dst_row, end = it.dst_row + it.n_tok;   // the run's slots
  const int64_t blk = first / BLK + blockIdx.y;
  if (blk * BLK >= end) return;
  const int kvh = blockIdx.z;
  const int64_t lo = first > blk * BLK ? first : blk * BLK;             // the run's slots inside this block
  const int64_t hi = end < (blk + 1) * BLK ? end : (blk + 1) * BLK;
  const int64_t row_stride = (int64_t)P.Hkv * D;
  // keys: 8 elements (16 bytes in, 8 bytes out) per thread and step
  const int n8 = (int)(hi - lo) * NG;
  for (int idx = threadIdx.x; idx < n8; idx += NT) {
    const int64_t slot = lo + idx / NG;
    const int g = idx % NG;
    const u32x4 raw = *(const u32x4*)(P.k_new + (it.src_row + (slot - first)) * row_stride + kvh * D + g * 8);
    int w0 = 0, w1 = 0;
    w0 = __builtin_amdgcn_cvt_pk_fp8_f32(code_range(raw[0] & 0xffffu, P.k_inv), code_range(raw[0] >> 16, P.k_inv), w0, false);
    w0 = __builtin_amdgcn_cvt_pk_fp8_f32(code_range(raw[1] & 0xffffu, P.k_inv), code_range(raw[1] >> 16, P.k_inv), w0, true);
    w1 = __builtin_amdgcn_cvt_pk_fp8_f32(code_range(raw[2] & 0xffffu, P.k_inv), code_range(raw[2] >> 16, P.k_inv), w1, false);
    w1 = __builtin_amdgcn_cvt_pk_fp8_f32(code_range(raw[3] & 0xffffu, P.k_inv), code_range(raw[3] >> 16, P.k_inv), w1, true);
    *(u32x2*)(P.cache_k + slot * row_stride + kvh * D + g * 8) = u32x2{(uint32_t)w0, (uint32_t)w1};
  }
  // values, step 1: thread (quad, granule) reads 8 elements of the block's tokens 4 * quad .. + 3
  // (whole 16-byte pieces of the token rows), turns each element's four tokens into one 32-bit word
  // of codes (tokens outside the run: zero) and puts it into the transposed block in LDS
  {
    const int quad = threadIdx.x / NG, g = threadIdx.x % NG;
    const int64_t s0 = blk * BLK + 4 * quad;
    u32x4 raw[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int64_t slot = s0 + e;
      raw[e] = u32x4{0u, 0u, 0u, 0u};
      if (slot >= lo && slot < hi)
        raw[e] = *(const u32x4*)(P.v_new + (it.src_row + (slot - first)) * row_stride + kvh * D + g * 8);
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      float x[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) x[e] = code_range((j & 1) ? raw[e][j / 2] >> 16 : raw[e][j / 2] & 0xffffu, P.v_inv);
      int w = 0;
      w = __builtin_amdgcn_cvt_pk_fp8_f32(x[0], x[1], w, false);
      w = __builtin_amdgcn_cvt_pk_fp8_f32(x[2], x[3], w, true);
      vt[((8 * g + j) * LROW) / 4 + quad] = (uint32_t)w;
    }
  }
  __syncthreads();
  // step 2: 16-byte pieces (element d, tokens 16 * tq ..) go out, a wave writing 1 KiB in one piece.
  // Bytes of tokens before the run are kept, bytes of tokens behind it are zero.
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int piece = threadIdx.x + i * NT;
    const int d = piece / 4, tq = piece % 4;
    const int64_t s0 = blk * BLK + tq * 16;
    if (s0 + 16 <= lo) continue;   // all of it was there before
    uint8_t* dst = P.cache_v + ((blk * P.Hkv + kvh) * D + d) * BLK + tq * 16;
    u32x4 res;
#pragma unroll
    for (int j = 0; j < 4; ++j) res[j] = vt[(d * LROW) / 4 + tq * 4 + j];
    if (s0 < lo) {
      const u32x4 old = *(const u32x4*)dst;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        uint32_t keep = 0u;   // bytes of tokens before the run
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (s0 + 4 * j + e < lo) keep |= 0xffu << (8 * e);
        res[j] = (old[j] & keep) | (res[j] & ~keep);
      }
    }
    *(u32x4*)dst = res;
  }
}

// ---------------------------------------------------------------------------------
// Launchers
// ---------------------------------------------------------------------------------

// Optional per-kernel timing: HIP events recorded on the launch stream right
// before and after each kernel launch while enabled.  The list of pairs is shared by
// all host threads and guarded by a lock.
struct EventPair { hipEvent_t a, b; int kind; bool closed; };
static std::mutex g_prof_mu;
static bool g_prof_on = false;
static std::vector<EventPair> g_prof_events;

// Returns the index of the pair that was opened, or -1 (profiling off, or no event to be had:
// then the launch is simply not timed).
static int prof_begin(int kind, hipStream_t st) {
  std::lock_guard<std::mutex> lock(g_prof_mu);
  if (!g_prof_on) return -1;
  EventPair p;
  p.kind = kind;
  p.closed = false;
  if (hipEventCreate(&p.a) != hipSuccess) return -1;
  if (hipEventCreate(&p.b) != hipSuccess) {
    (void)hipEventDestroy(p.a);
    return -1;
  }
  (void)hipEventRecord(p.a, st);
  g_prof_events.push_back(p);
  return (int)g_prof_events.size() - 1;
}
static void prof_end(int pair, hipStream_t st) {
  if (pair < 0) return;
  std::lock_guard<std::mutex> lock(g_prof_mu);
  if ((size_t)pair >= g_prof_events.size()) return;   // read (and cleared) by another thread meanwhile
  (void)hipEventRecord(g_prof_events[(size_t)pair].b, st);
  g_prof_events[(size_t)pair].closed = true;
}
int profile_enable(int on) {
  std::lock_guard<std::mutex> lock(g_prof_mu);
  g_prof_on = on != 0;
  return 0;
}
bool profile_is_on() {
  std::lock_guard<std::mutex> lock(g_prof_mu);
  return g_prof_on;
}
// Waits for the recorded pairs and forgets them.  Sums per kind go to ms / launches; if
// `each_ms` is given, the first max_each launches' own durations and kinds as well, in
// launch order (n_each = how many were written).
int profile_read(double ms[3], int32_t launches[3], double* each_ms, int32_t* each_kind, int32_t max_each,
                 int32_t* n_each) {
  for (int k = 0; k < 3; ++k) ms[k] = 0.0, launches[k] = 0;
  std::vector<EventPair> pairs;
  {
    std::lock_guard<std::mutex> lock(g_prof_mu);
    pairs.swap(g_prof_events);
  }
  int rc = 0;
  int32_t written = 0;
  for (EventPair& p : pairs) {
    if (p.closed) {
      float t = 0.f;
      hipError_t e = hipEventSynchronize(p.b);
      if (e == hipSuccess) e = hipEventElapsedTime(&t, p.a, p.b);
      if (e != hipSuccess) rc = (int)e;
      else if (p.kind >= 0 && p.kind < 3) {
        ms[p.kind] += t, launches[p.kind] += 1;
        if (each_ms && written < max_each) {
          each_ms[written] = t;
          if (each_kind) each_kind[written] = p.kind;
          ++written;
        }
      }
    }
    (void)hipEventDestroy(p.a);
    (void)hipEventDestroy(p.b);
  }
  if (n_each) *n_each = written;
  return rc;
}

// Scratch buffer of the entry point that allocates nothing (partial results of split key
// ranges).  The array's name is a host-side stand-in for the symbol: kernels are given the
// address hipGetSymbolAddress reports for the current device, looked up once per device.
// Nothing in it has to start at zero: every partial row is written before it is read.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mu;
static void* g_scratch_ptr[kMaxDevices] = {};

int static_scratch(void** ptr) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return (int)e;
  if (dev < 0 || dev >= kMaxDevices) return (int)hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return (int)e;
    if (!p) return (int)hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
  }
  *ptr = g_scratch_ptr[dev];
  return 0;
}

int launch_attention(const LayerShape& ls, const void* q, void* k, void* v, const void* k_new, const void* v_new,
                     void* out, float* part_o, float* part_ml, const AttnItem* items, int n_items,
                     const uint16_t* first, int n_queues, void* stream, bool timed) {
  hipStream_t st = (hipStream_t)stream;
  if (n_items <= 0 || n_queues <= 0) return 0;
  if (n_items > kMaxAttnItems || n_queues > kMaxQueues) return (int)hipErrorInvalidValue;
  AttnParams P;
  P.q = (const uint16_t*)q;
  P.k = (uint16_t*)k;
  P.v = (uint16_t*)v;
  P.k_new = (const uint16_t*)k_new;
  P.v_new = (const uint16_t*)v_new;
  P.out = (uint16_t*)out;
  P.part_o = part_o;
  P.part_ml = part_ml;
  P.Hq = ls.Hq;
  P.Hkv = ls.Hkv;
  P.G = ls.G;
  P.TM = ls.TM;
  P.c = ls.c;
  P.out_scale = ls.out_scale;
  P.q_mult = 1.0f;
  P.q_scale_byte = 127;
  if (ls.fp8) {
    // k with 4 <= c * 2^k < 8: queries of magnitude 2^-8 .. 56 stay inside E4M3's normal range
    int e = 0;
    (void)frexpf(ls.c, &e);                  // c = f * 2^e, 0.5 <= f < 1
    const int k = 3 - e;                     // c * 2^k = 8 f, in [4, 8)
    if (k < -120 || k > 120) return (int)hipErrorInvalidValue;
    P.q_mult = ldexpf(ls.c, k);
    P.q_scale_byte = 127 - k;
  }
  P.n_queues = n_queues;
  P.g_magic = (65536u + (uint32_t)ls.G - 1u) / (uint32_t)ls.G;
  for (int j = 0; j <= n_queues; ++j) P.first[j] = first[j];
  for (int i = 0; i < n_items; ++i) P.items[i] = items[i];
  dim3 grid((unsigned)(n_queues * ls.Hkv));
  const bool append = k_new != nullptr;
  const int pair = timed ? prof_begin(0, st) : -1;
  if (ls.fp8) {
    // (the 8-bit cache is filled by its own append kernel)
    if (append) return (int)hipErrorInvalidValue;
    if (ls.D == 128) hipLaunchKernelGGL(attn_fwd_fp8_kernel<128>, grid, dim3(512), 0, st, P);
    else hipLaunchKernelGGL(attn_fwd_fp8_kernel<64>, grid, dim3(512), 0, st, P);
  } else if (ls.D == 128) {
    if (append) hipLaunchKernelGGL((attn_fwd_kernel<128, true>), grid, dim3(512), 0, st, P);
    else hipLaunchKernelGGL((attn_fwd_kernel<128, false>), grid, dim3(512), 0, st, P);
  } else {
    if (append) hipLaunchKernelGGL((attn_fwd_kernel<64, true>), grid, dim3(512), 0, st, P);
    else hipLaunchKernelGGL((attn_fwd_kernel<64, false>), grid, dim3(512), 0, st, P);
  }
  prof_end(pair, st);
  return (int)hipGetLastError();
}

int launch_combine(const LayerShape& ls, void* out, const float* part_o, const float* part_ml,
                   const CombineItem* items, int n_items, void* stream, bool timed) {
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
    P.c = ls.fp8 ? 1.0f : ls.c;   // (the 8-bit kernel stores its references in log2 units)
    P.out_scale = ls.out_scale;
    const int n = n_items - base < kMaxCombineItems ? n_items - base : kMaxCombineItems;
    P.n_items = n;
    for (int i = 0; i < n; ++i) P.items[i] = items[base + i];
    const int rpb = 256 / (ls.D / 4);
    dim3 grid((unsigned)(n * ls.Hkv), (unsigned)(kTileRows / rpb)), block(256);
    int max_split = 0;
    for (int i = 0; i < n; ++i) max_split = items[base + i].nsplit > max_split ? items[base + i].nsplit : max_split;
    const int pair = timed ? prof_begin(1, st) : -1;
    if (ls.D == 128) {
      if (max_split <= 4) hipLaunchKernelGGL((combine_kernel<128, 4>), grid, block, 0, st, P);
      else if (max_split <= 8) hipLaunchKernelGGL((combine_kernel<128, 8>), grid, block, 0, st, P);
      else hipLaunchKernelGGL((combine_kernel<128, kMaxSplit>), grid, block, 0, st, P);
    } else {
      if (max_split <= 4) hipLaunchKernelGGL((combine_kernel<64, 4>), grid, block, 0, st, P);
      else if (max_split <= 8) hipLaunchKernelGGL((combine_kernel<64, 8>), grid, block, 0, st, P);
      else hipLaunchKernelGGL((combine_kernel<64, kMaxSplit>), grid, block, 0, st, P);
    }
    prof_end(pair, st);
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
    const int pair = prof_begin(2, st);
    hipLaunchKernelGGL(kv_append_kernel, grid, block, 0, st, P);
    prof_end(pair, st);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return (int)e;
  }
  return 0;
}

int launch_append_fp8(const LayerShape& ls, void* cache_k, void* cache_v, const void* k_new, const void* v_new,
                      float k_inv, float v_inv, const AppendItem* items, int n_items, void* stream) {
  hipStream_t st = (hipStream_t)stream;
  if (ls.D != 128 && ls.D != 64) return (int)hipErrorInvalidValue;
  for (int base = 0; base < n_items; base += kMaxAppendItems) {
    Append8Params P;
    P.cache_k = (uint8_t*)cache_k;
    P.cache_v = (uint8_t*)cache_v;
    P.k_new = (const uint16_t*)k_new;
    P.v_new = (const uint16_t*)v_new;
    P.k_inv = k_inv;
    P.v_inv = v_inv;
    P.Hkv = ls.Hkv;
    const int n = n_items - base < kMaxAppendItems ? n_items - base : kMaxAppendItems;
    P.n_items = n;
    int64_t blocks = 0;   // 64-token blocks the longest run of this launch touches
    for (int i = 0; i < n; ++i) {
      const AppendItem& a = items[base + i];
      P.items[i] = a;
      const int64_t nb = (a.dst_row + a.n_tok - 1) / kKeyTile - a.dst_row / kKeyTile + 1;
      if (nb > blocks) blocks = nb;
    }
    if (blocks > 65535) return (int)hipErrorInvalidValue;
    dim3 grid((unsigned)n, (unsigned)blocks, (unsigned)ls.Hkv);
    const int pair = prof_begin(2, st);
    if (ls.D == 128) hipLaunchKernelGGL(kv_append_fp8_kernel<128>, grid, dim3(256), 0, st, P);
    else hipLaunchKernelGGL(kv_append_fp8_kernel<64>, grid, dim3(128), 0, st, P);
    prof_end(pair, st);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return (int)e;
  }
  return 0;
}

const char* hip_error_string(int err) { return hipGetErrorString((hipError_t)err); }

}  // namespace oppo
