// Chunked-prefill attention over the cache of 8-bit codes: the kernel (device code only; this
// file is included by kernels.hip inside namespace oppo, after the shared helpers and AttnParams).
//
// Same work decomposition as attn_fwd_kernel - persistent workgroups of eight waves, each wave
// owning 32 query columns of the packed 256-row tile, pieces = (tile, key range), K/V tiles of 64
// keys travelling global -> LDS through a four-stage ring - but both products run on the 8-bit
// MFMA with 64-deep contraction (v_mfma_scale_f32_32x32x64_f8f6f4 with unit scales), which on
// this chip issues at twice the rate of the 16-bit MFMA per multiply-add (the older 16-deep 8-bit
// MFMA only matches the 16-bit rate).  Operand layout of that instruction: lane l holds row (A)
// or column (B) l % 32 and the 32 consecutive contraction indices 32 * (l / 32) ..; the result
// sits as for the other 32x32 MFMAs (register i of lane l = row 8 (i / 4) + 4 (l / 32) + i % 4,
// column l % 32).
//
//   S^T = K Q^T, per 32-key unit: two MFMAs (contraction over the 128 elements of a head).
//         A = 32 key rows of the tile in LDS (row = key, 128 bytes), B = the wave's query
//         columns, rounded to E4M3 once per piece.
//   O^T += V^T P^T, per 64-key tile: four MFMAs (one per 32 output elements; contraction over
//         the tile's 64 keys).  A = rows of the value tile, which is stored transposed (row =
//         element, 64 key bytes); B = the tile's softmax weights, rounded to E4M3.
//
// A lane's weights of a tile must be 32 consecutive keys of it for the second product, but an
// S^T result register holds rows 8a + 4h + b (h = lane / 32).  The keys are therefore assigned to
// MFMA rows in a permuted order: row 8a + 4h + b of unit ub (0, 1) of a tile is the tile's key
// 32h + 16ub + 4a + b, i.e. register i of half h of unit ub is key 32h + 16ub + i, and the two
// units of a tile fill the lane's 32 weight bytes in order.  The permutation costs nothing: it is
// the LDS row a lane reads its K fragment from.  (Unit 0 of a tile thus covers its keys 0-15 and
// 32-47, unit 1 the keys 16-31 and 48-63; both units of every tile are run, a unit without
// visible keys contributes zeros.)
//
// Scores and references.  The instruction multiplies each operand by a power of two of its own
// (the block scales of the scaled formats), which is used here to keep the vector unit out of the
// score arithmetic: the queries are multiplied by the whole score factor c (softmax scale x log2 e
// x the keys' scale) times 2^k before they are rounded to E4M3 - k chosen by the launcher so that
// they land in the format's normal range, and one rounding either way - and the B operand's scale
// 2^-k takes the power of two out again, so S^T comes out of the MFMA in log2 units.  A column's
// reference enters as the accumulator input of a unit's first MFMA (sixteen registers holding
// kBias minus the reference), so a weight is exp2 of an accumulator register as it stands.
// As in attn_fwd_kernel the reference is held and only moved (with an exact redo of the unit) when
// a unit's row sum exceeds the limit.  The weights are rounded to E4M3 (largest finite value
// 448): the limit is 448 and kBias = 4, i.e. a key at the reference weighs 16, sixteen of them
// stay below the limit, and weights keep full precision down to 2^-10 of the reference; sum and
// numerator carry the same factor, which cancels.  The row sum adds the weights before rounding
// (rounding to nearest is unbiased; turning codes back into numbers would cost more than two
// additions).  A column's first reference is the maximum of the first unit in which it sees a
// key; until then it is the arbitrary 0 and the column has accumulated nothing.
// The values' scale is folded into the final normalisation.
// Head size 64: the contraction of S^T is one MFMA deep, O^T has two 32-row blocks; a tile of
// either array is 4 KiB, so waves 0-3 move the keys and waves 4-7 the values.
template <int D>
__global__ __launch_bounds__(512) void attn_fwd_fp8_kernel(const AttnParams P) {
  static_assert(D == 128 || D == 64, "head sizes 64 and 128");
  constexpr int NT = 512;
  constexpr int BN = kKeyTile;
  constexpr int ROWB = D;                  // bytes per key row
  constexpr int TILE_BYTES = BN * ROWB;    // (a value tile is D rows of BN bytes: the same size)
  constexpr int NSTAGE = 4;
  constexpr int NCH = D / 32;              // 1 KiB chunks of a wave's staging area
  constexpr int DB = D / 32;               // 32-row blocks of O^T
  constexpr int KS = D / 64;               // MFMAs of S^T per unit = O^T MFMAs per unit body
  constexpr int NGK = ROWB / 16;           // 16-byte granules per key row
  constexpr int UM = D / 32 - 1;           // a key row's 32-byte units are swizzled by (row >> KSH) & UM
  constexpr int KSH = D == 128 ? 1 : 2;
  static_assert(BN == 64, "64-key tiles");

  __shared__ __attribute__((aligned(1024))) unsigned char sk[NSTAGE][TILE_BYTES];
  __shared__ __attribute__((aligned(1024))) unsigned char sv[NSTAGE][TILE_BYTES];
  // staging areas for turning 32 x D bf16 blocks around (queries in, outputs out): 4 KiB per wave
  __shared__ __attribute__((aligned(1024))) unsigned char sq[8 * NCH * 1024];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int l32 = lane & 31;
  const int hi = lane >> 5;
  const int Hq = P.Hq, Hkv = P.Hkv, G = P.G;
  const int kvh = blockIdx.x % Hkv;
  const int queue = blockIdx.x / Hkv;
  const int p_first = P.first[queue];
  const int p_last = P.first[queue + 1];
  if (p_first >= p_last) return;
  const float q_mult = P.q_mult;           // c * 2^k, applied to the queries before rounding
  const int q_scale = P.q_scale_byte;      // E8M0 code of 2^-k, the B operand's scale in S^T

  // the queue's piece descriptors, copied from the kernel-argument segment into LDS once
  __shared__ __attribute__((aligned(16))) AttnItem spiece[kMaxAttnItems];
  {
    const u32x4* src = (const u32x4*)(P.items + p_first);
    const int n16 = (p_last - p_first) * (int)(sizeof(AttnItem) / 16);
    for (int i = tid; i < n16; i += NT) ((u32x4*)spiece)[i] = src[i];
    // The first piece's first tile multiplies zero weights with "the tile before it", whatever ring
    // stage 3 holds: make that zero bytes (valid codes; afterwards the ring only ever holds codes).
    if (tid < TILE_BYTES / 16) ((u32x4*)&sv[NSTAGE - 1][0])[tid] = u32x4{0u, 0u, 0u, 0u};
    __syncthreads();
  }
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

  // ---- cooperative K/V tile loads (global -> LDS directly, 16 bytes per lane) ----------------
  // K: a wave-wide load covers 1 KiB of key rows (8 rows of D = 128, 16 of D = 64).  A row's
  // 32-byte units (the piece of a row one lane reads as an MFMA operand) are swizzled by
  // (row / 2) % 4 resp. (row / 4) % 2.  V: a tile is one contiguous block of D rows of 64 key
  // bytes, 16 rows per wave-wide load; a row's two 32-byte units are swizzled by (row / 4) % 2.
  // D = 128: every wave moves 1 KiB of each; D = 64: waves 0-3 the keys, waves 4-7 the values.
  const int row_stride = Hkv * D;   // bytes between consecutive tokens' keys
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);
  const bool moves_k = D == 128 || wave_s < 4, moves_v = D == 128 || wave_s >= 4;
  const int kwave = wave_s, vwave = D == 128 ? wave_s : (wave_s & 3);
  const int kr = (kwave & (TILE_BYTES / 1024 - 1)) * (64 / NGK) + lane / NGK;
  const int kg = lane % NGK;
  const uint32_t goffk = (uint32_t)(kr * row_stride + ((kg ^ (((kr >> KSH) & UM) << 1)) * 16));
  const int vr = vwave * 16 + lane / 4;
  const uint32_t goffv = (uint32_t)(vr * BN + (((lane % 4) ^ (((vr >> 2) & 1) << 1)) * 16));
  const uint32_t wave_rows = (uint32_t)wave_s * 1024u;
  const uint32_t kdst = (uint32_t)(kwave & (TILE_BYTES / 1024 - 1)) * 1024u, vdst = (uint32_t)vwave * 1024u;

  // ---- the wave's staging area -----------------------------------------------------------------
  // Q and O blocks travel to and from global memory as whole row pieces (16 bytes per lane,
  // consecutive lanes on consecutive addresses) and are turned around in LDS, half of D at a
  // time: a lane owns one query column, i.e. pieces of one row.
  constexpr int RB = D;             // bytes of a bf16 row per round (half a row)
  constexpr int NS = RB / 16;       // 16-byte slots of a row per round
  constexpr int RPC = 1024 / RB;    // rows per 1 KiB chunk
  typedef __attribute__((address_space(3))) unsigned char* lds_ptr;
  typedef const __attribute__((address_space(3))) unsigned char* lds_cptr;
  // (lane-dependent offsets needed at piece boundaries only are recomputed there from a copy of the
  // lane number the optimiser cannot see through, instead of living in registers through the key loop)
  auto lane_now = [&]() __attribute__((always_inline)) -> int {
    int x = lane;
    asm volatile("" : "+v"(x));
    return x;
  };
  auto roff_of = [&](int ln) __attribute__((always_inline)) -> uint32_t {
    return (uint32_t)((ln / NS) * RB + (((ln % NS) ^ ((ln / NS) & (NS - 1))) * 16));
  };
  auto cx_of = [&](int ln) __attribute__((always_inline)) -> uint32_t { return (uint32_t)(ln & (NS - 1)) * 16u; };
  auto area_of = [&](int k) __attribute__((always_inline)) -> uint32_t {
    return lds_addr_of(&sq[0]) + wave_rows * NCH + (uint32_t)(k * 1024);
  };
  auto carea_of = [&](int ln) __attribute__((always_inline)) -> uint32_t {   // the row of lane ln in its chunk
    const int row = ln & 31;
    return lds_addr_of(&sq[0]) + wave_rows * NCH + (uint32_t)((row / RPC) * 1024 + (row % RPC) * RB);
  };
  // rows wave*32 + k*RPC + ln/NS of the packed tile -> (q-head of the group, token)
  auto row_of = [&](int ln, int k, int* hk, int* tk) __attribute__((always_inline)) {
    const int R = (int)(wave_rows >> 10) * 32 + ln / NS + k * RPC;
    const int t = (int)(((uint32_t)R * P.g_magic) >> 16);            // R / G
    *tk = t;
    *hk = R - t * G;
  };
  i32x8 qf[KS];           // the lane's query column as E4M3 codes: elements 64 kk + 32 hi .. of it in qf[kk]
  u32x4 qraw[2][NCH];     // Q row pieces on their way: [half of D][chunk]
  auto q_request = [&](const AttnItem& a) __attribute__((always_inline)) {
    const int ln = lane_now();
#pragma unroll
    for (int k = 0; k < NCH; ++k) {
      int hk, tk;
      row_of(ln, k, &hk, &tk);
      // rows beyond the tile repeat a valid row; their columns are never stored
      const uint16_t* qp = P.q + ((int64_t)(a.q_row0 + min(tk, tokens_of(a) - 1)) * Hq + kvh * G + hk) * D + (ln % NS) * 8;
#pragma unroll
      for (int h = 0; h < 2; ++h) qraw[h][k] = *(const u32x4*)(qp + h * (D / 2));
    }
  };
  auto q_collect = [&]() __attribute__((always_inline)) {
    const int ln = lane_now();
    const uint32_t roff = roff_of(ln);
    const uint32_t cbase = carea_of(ln);
    const uint32_t cx = cx_of(ln);
    const int hl = ln >> 5;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
#pragma unroll
      for (int k = 0; k < NCH; ++k)
        *(__attribute__((address_space(3))) u32x4*)(lds_ptr)(uintptr_t)(area_of(k) + roff) = qraw[h][k];
      // round h holds elements (D / 2) h .. of every row.  D = 128: the lane wants 32 hl .. of them (slots
      // 4 hl + j) for its operand of contraction half h; D = 64: round hl as a whole is the lane's operand
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int sl = D == 128 ? 4 * hl + j : j;
        const bf16x8 f = *(const __attribute__((address_space(3))) bf16x8*)(lds_ptr)(uintptr_t)(
            cbase + ((uint32_t)(sl * 16) ^ cx));
        const long w = bf16x8_to_fp8x8(f, q_mult);
        const int w0 = (int)(uint32_t)((unsigned long)w & 0xffffffffu), w1 = (int)(uint32_t)((unsigned long)w >> 32);
        if constexpr (D == 128) {
          qf[h][2 * j] = w0;
          qf[h][2 * j + 1] = w1;
        } else {
          if (h == 0 || hl == 1) {   // (round 0 for the lower lanes, overwritten by round 1 for the upper ones)
            qf[0][2 * j] = w0;
            qf[0][2 * j + 1] = w1;
          }
        }
      }
    }
  };

  // ---- the request cursor over the workgroup's tile stream (wave-uniform) ---------------------
  int c_piece = p_first;        // piece of the next tile to request
  int c_left = 0;               // keys of that piece not requested yet
  uintptr_t c_k = 0, c_v = 0;   // the next tile of this kv-head: its first key row, its value block
  const uintptr_t k_step = (uintptr_t)BN * row_stride;
  const uintptr_t v_step = (uintptr_t)row_stride * BN;   // one 64-token block of all kv-heads
  auto cursor_open = [&]() __attribute__((always_inline)) {
    const AttnItem a = piece(c_piece);
    c_k = (uintptr_t)P.k + (uintptr_t)((((int64_t)a.kv_row0 + a.k_begin) * Hkv + kvh) * D);
    c_v = (uintptr_t)P.v + (uintptr_t)(((((int64_t)a.kv_row0 + a.k_begin) / BN) * Hkv + kvh) * D) * BN;
    c_left = a.k_end - a.k_begin;
  };
  cursor_open();
  auto issue_next = [&](int stage) __attribute__((always_inline)) {
    if (c_piece >= p_last) return;
    const int last = c_left - 1;
    uint32_t wave_rows_now = wave_rows;
    asm volatile("" : "+s"(wave_rows_now));
    (void)wave_rows_now;
    uint32_t ok = goffk;
    if (last < BN - 1) {  // ragged last tile: rows past the range repeat the last key
      const int rc = min(kr, last);
      ok = (uint32_t)(rc * row_stride + ((kg ^ (((kr >> KSH) & UM) << 1)) * 16));
    }
    uint32_t kd = kdst, vd = vdst;
    asm volatile("" : "+s"(kd), "+s"(vd));
    // (a value block is read whole: what lies beyond the last token in it is later tokens' codes or zeros)
    if (moves_k) async_copy16((const void*)c_k, ok, lds_addr_of(&sk[stage][0]) + kd);
    if (moves_v) async_copy16((const void*)c_v, goffv, lds_addr_of(&sv[stage][0]) + vd);
    c_k += k_step;
    c_v += v_step;
    c_left -= BN;
    if (c_left <= 0) {
      ++c_piece;
      if (c_piece < p_last) cursor_open();
    }
  };
  auto wg_barrier = [&]() __attribute__((always_inline)) {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  };

  // ---- per-lane LDS addresses of the operand fragments ----------------------------------------
  // K: MFMA row l32 = 8a + 4h' + b of unit 0 is the tile's key row 32h' + 4a + b (unit 1: 16 rows further)
  lds_cptr kptr[KS];   // elements 64 kk + 32 hi .. of that row
  {
    const int krow = 32 * ((l32 >> 2) & 1) + 4 * (l32 >> 3) + (l32 & 3);
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
      uint32_t a = lds_addr_of(&sk[0][0]) + (uint32_t)(krow * ROWB + (((2 * kk + hi) ^ ((krow >> KSH) & UM)) * 32));
      asm volatile("" : "+v"(a));
      kptr[kk] = (lds_cptr)(uintptr_t)a;
    }
  }
  lds_cptr vptr;      // keys 32 hi .. of value row l32 (element l32 of d-block 0; d-block db: 32 rows further)
  {
    uint32_t a = lds_addr_of(&sv[0][0]) + (uint32_t)(l32 * BN + ((hi ^ ((l32 >> 2) & 1)) * 32));
    asm volatile("" : "+v"(a));
    vptr = (lds_cptr)(uintptr_t)a;
  }
  auto ld32 = [&](lds_cptr p) __attribute__((always_inline)) -> i32x8 {
    const i32x4 a = *(const __attribute__((address_space(3))) i32x4*)(p);
    const i32x4 b = *(const __attribute__((address_space(3))) i32x4*)(p + 16);
    return __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
  };
  // K fragment of unit (stage offset `off`, ub), contraction half kk
  auto ldk = [&](int off, int ub, int kk) __attribute__((always_inline)) -> i32x8 {
    return ld32(kptr[kk] + off + ub * 16 * ROWB);
  };
  // V^T fragment of the tile at stage offset `off`, d-block db
  auto ldv = [&](int off, int db) __attribute__((always_inline)) -> i32x8 {
    return ld32(vptr + off + db * 32 * BN);
  };
  // S^T: the query operand carries the scale 2^-k; O^T: unit scales (127 = 2^0)
  auto mma_s = [&](const i32x8& a, const i32x8& b, const f32x16& acc) __attribute__((always_inline)) -> f32x16 {
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, acc, 0, 0, 0, 127, 0, q_scale);
  };
  auto mma = [&](const i32x8& a, const i32x8& b, const f32x16& acc) __attribute__((always_inline)) -> f32x16 {
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, acc, 0, 0, 0, 127, 0, 127);
  };

  constexpr float kRowSumLimit = 448.0f;
  constexpr float kBias = 4.0f;

  // ------------------------------------------------------------------------------------------
  // Main loop, software-pipelined over 32-key units (two per tile).  The body of unit u issues,
  // interleaved, the two S^T MFMAs of unit u+1, two of the four O^T MFMAs of the PREVIOUS tile
  // (its weights are complete once both of its units are done), and the exp2 / rounding /
  // row-sum vector work of unit u: per MFMA (16 passes) two pairs of weights, 14 vector
  // instructions.
  // ------------------------------------------------------------------------------------------
  f32x16 o[DB];
  f32x16 s[2];          // s[u & 1] = S^T of unit u
  i32x8 ka[KS];         // K fragments in flight (the contraction halves of a unit)
  i32x8 vf[KS];         // V^T fragments in flight
  i32x8 pw[2];          // pw[tile's ring stage & 1] = the tile's weights, B-operand layout (byte j = key 32 hi + j)
  f32x16 negm;          // kBias minus the column's reference (log2 units), in all sixteen registers
  float mref = 0.f;     // the reference
  bool noref = true;    // the column has seen no key of the piece yet
  bool noref_any = true;
  float l_run, rs0 = 0.f, rs1 = 0.f;

  AttnItem it = piece(p_first);
  int lim = 0;       // last key this lane's column may see, minus 32 * (lane / 32)
  int min_lim = 0;   // smallest last visible key in the workgroup: units entirely below it need no mask

  // weights 2p, 2p+1 of the unit in s[cur] -> half (p & 1) of the word w, which is returned
  // (`shift`: what the redo path has just moved the reference by, 0 on the common path)
  auto exp_pair = [&](int cur, int pr, int w, float shift) __attribute__((always_inline)) -> int {
    const float x0 = s[cur][2 * pr], x1 = s[cur][2 * pr + 1];
    const float p0 = fast_exp2(x0 - shift);
    const float p1 = fast_exp2(x1 - shift);
    if (pr & 1) {
      w = __builtin_amdgcn_cvt_pk_fp8_f32(p0, p1, w, true);
      rs1 += p0 + p1;
      asm volatile("" : "+v"(w), "+v"(rs1));
    } else {
      w = __builtin_amdgcn_cvt_pk_fp8_f32(p0, p1, w, false);
      rs0 += p0 + p1;
      asm volatile("" : "+v"(w), "+v"(rs0));
    }
    return w;
  };

  // Body of unit u.  BC = position of the unit in the LDS ring (stage, unit of the tile), a
  // compile-time value, so that every fragment read has an immediate offset.
  auto unit_body = [&](auto BC, int u) __attribute__((always_inline)) {
    constexpr int b = decltype(BC)::value;
    constexpr int st_c = b / 2, ub = b % 2;                      // unit u
    constexpr int st_n = ((b + 1) % 8) / 2, ub_n = (b + 1) % 2;  // unit u+1
    constexpr int st_nn = ((b + 2) % 8) / 2;                     // unit u+2 (same unit of the next tile)
    constexpr int st_p = (st_c + 3) % 4;                         // the previous tile
    constexpr int cur = ub, nxt = cur ^ 1;
    constexpr int tp = st_c & 1, tq = tp ^ 1;                    // weight buffers of this tile / the previous one

    // ---- causal / range mask: register i is the tile's key 16 ub + i (+ 32 for the upper lanes) ----
    const int key0 = it.k_begin + BN * (u >> 1) + 16 * ub;
    if (key0 + 47 > min_lim) {
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (key0 + r > lim) s[cur][r] = -INFINITY;
    }
    rs0 = 0.f;
    rs1 = 0.f;

    constexpr int PPSN = 8 / KS;   // pairs of weights per step
#pragma unroll
    for (int i = 0; i < KS; ++i) {
      s[nxt] = mma_s(ka[i], qf[i], i == 0 ? negm : s[nxt]);
      ka[i] = ldk(st_nn * TILE_BYTES, ub, i);
      o[KS * ub + i] = mma(vf[i], pw[tq], o[KS * ub + i]);
      // the O^T MFMA after this one in program order: d-block KS + i of the same tile (ub = 0), or
      // d-block i of the tile that is current now (ub = 1)
      vf[i] = ub == 0 ? ldv(st_p * TILE_BYTES, KS + i) : ldv(st_c * TILE_BYTES, i);
#pragma unroll
      for (int jj = 0; jj < PPSN; ++jj) {
        const int pr = PPSN * i + jj;
        pw[tp][4 * ub + pr / 2] = exp_pair(cur, pr, pw[tp][4 * ub + pr / 2], 0.f);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
      __builtin_amdgcn_sched_group_barrier(0x402, 5 * PPSN / 2, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
      __builtin_amdgcn_sched_group_barrier(0x402, 5 * PPSN / 2, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    (void)st_n;
    (void)ub_n;
    float rs = rs0 + rs1;
    // pin the work above to this block: without a use here the compiler sinks it - the MFMAs
    // included - below the branch that follows
    if constexpr (KS == 2) asm volatile("" : "+v"(pw[tp]), "+v"(rs), "+v"(s[nxt]), "+v"(o[2 * ub]), "+v"(o[2 * ub + 1]));
    else asm volatile("" : "+v"(pw[tp]), "+v"(rs), "+v"(s[nxt]), "+v"(o[ub]));
    __builtin_amdgcn_sched_barrier(0);
    // (the O^T MFMAs of a piece's first tile multiply zero weights with a tile of valid codes: nothing)
    const bool over = __any(rs > kRowSumLimit);
    if (noref_any | over) {   // (noref_any: always at a piece's first unit; no short-circuit: one branch)
      // A column without a reference yet, or one that saw a score far above its reference: take the
      // unit's true maximum (one query column per lane, its key halves in lanes l and l^32; the
      // registers hold score - reference + kBias), move the references to it - up only, except for a
      // column's first -, redo the unit's weights and rescale what was formed against the old
      // references: the accumulators, and S^T of unit u+1.
      float mx4[4];
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4)
        mx4[q4] = fmaxf(fmaxf(fmaxf(s[cur][q4], s[cur][4 + q4]), s[cur][8 + q4]), s[cur][12 + q4]);
      float mx = fmaxf(fmaxf(fmaxf(mx4[0], mx4[1]), mx4[2]), mx4[3]);
      mx = fmaxf(mx, swap_halves(mx));
      const bool seen = mx > -INFINITY;
      const float delta = noref ? (seen ? mx - kBias : 0.f) : fmaxf(mx - kBias, 0.f);
      const float alpha = noref ? 1.0f : fast_exp2(-delta);   // (a column without a reference has accumulated nothing)
      noref = noref && !seen;
      noref_any = __any(noref);
      mref += delta;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        negm[r] -= delta;
        s[nxt][r] -= delta;
      }
      l_run *= alpha;
      rs0 = 0.f;
      rs1 = 0.f;
#pragma unroll
      for (int pr = 0; pr < 8; ++pr) pw[tp][4 * ub + pr / 2] = exp_pair(cur, pr, pw[tp][4 * ub + pr / 2], delta);
      rs = rs0 + rs1;
      // Weights that were formed against the old reference and have not been through their MFMAs
      // yet follow (codes -> numbers -> times alpha -> codes): those of this tile's first unit if this
      // is its second, and the previous tile's if this is the first - half of that tile's O^T
      // MFMAs come in the next body.
      auto rescale = [&](int w_old) __attribute__((always_inline)) -> int {
        const auto lo2 = __builtin_amdgcn_cvt_pk_f32_fp8(w_old, false);
        const auto hi2 = __builtin_amdgcn_cvt_pk_f32_fp8(w_old, true);
        int w = 0;
        w = __builtin_amdgcn_cvt_pk_fp8_f32(lo2[0] * alpha, lo2[1] * alpha, w, false);
        w = __builtin_amdgcn_cvt_pk_fp8_f32(hi2[0] * alpha, hi2[1] * alpha, w, true);
        return w;
      };
      if (ub == 1) {
#pragma unroll
        for (int wd = 0; wd < 4; ++wd) pw[tp][wd] = rescale(pw[tp][wd]);
      } else {
#pragma unroll
        for (int wd = 0; wd < 8; ++wd) pw[tq][wd] = rescale(pw[tq][wd]);
      }
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[db][r] *= alpha;
    }
    l_run += rs;
  };

  // A wave whose 32 rows all lie beyond the tile's tokens does none of the arithmetic of the piece:
  // it still requests its share of every key tile and joins the barriers.
  auto has_rows = [&](const AttnItem& a) __attribute__((always_inline)) -> bool {
    return (int)(wave_rows >> 10) * 32 < tokens_of(a) * G;
  };
  bool act = true;
  auto iteration = [&](auto TC, int t) __attribute__((always_inline)) {
    constexpr int ts = decltype(TC)::value;
    issue_next((ts + 2) % NSTAGE);
    unit_body(std::integral_constant<int, 2 * ts>{}, 2 * t);
    unit_body(std::integral_constant<int, 2 * ts + 1>{}, 2 * t + 1);
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wave's share of the requested tile is in LDS
    wg_barrier();
  };

  // ---- start-up: Q of the first piece, the first two tiles of the stream ------------------------
  act = has_rows(it);
  q_request(it);
  issue_next(0);
  issue_next(1);
  q_collect();
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
  wg_barrier();

  int ph = 0;   // ring stage of the current piece's first tile
  for (int p = p_first;;) {
    const int ln_top = lane_now();
    const int r_tile = (int)(wave_rows >> 10) * 32 + (ln_top & 31);   // the lane's row of the packed tile
    const int tok = (int)(((uint32_t)r_tile * P.g_magic) >> 16);     // its token within the tile (r_tile / G)
    const int tokc = min(tok, tokens_of(it) - 1);
    lim = min(it.pos0 + tokc, it.k_end - 1) - 32 * (ln_top >> 5);
    min_lim = min(it.pos0, it.k_end - 1);
    const int nkeys = it.k_end - it.k_begin;
    const int nt = (nkeys + BN - 1) / BN;
    l_run = 0.f;
    mref = 0.f;
    noref = true;
    noref_any = true;
#pragma unroll
    for (int r = 0; r < 16; ++r) negm[r] = kBias;
    // the first tile's bodies run the O^T MFMAs "of the tile before it": with zero weights
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[db][r] = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) pw[0][j] = pw[1][j] = 0;

    // whatever this wave still has in flight (the previous piece's stores, the tiles requested
    // ahead) is awaited here, on the path of every wave
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    // S^T of unit 0 on its own, then the operand buffers as the first body expects them
    if (act) {
      const int off0 = ph * TILE_BYTES;
      const int offm = ((ph + 3) & 3) * TILE_BYTES;   // "the previous tile": any stage
#pragma unroll
      for (int i = 0; i < KS; ++i) ka[i] = ldk(off0, 0, i);
#pragma unroll
      for (int i = 0; i < KS; ++i) {
        s[0] = mma_s(ka[i], qf[i], i == 0 ? negm : s[0]);
        ka[i] = ldk(off0, 1, i);
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int i = 0; i < KS; ++i) vf[i] = ldv(offm, i);
    }

    const int tau1 = ph + nt;
    if (act) {
      for (int tb = 0; tb < tau1; tb += 4) {
        if (tb >= ph) iteration(std::integral_constant<int, 0>{}, tb - ph);
        if (tb + 1 >= ph && tb + 1 < tau1) iteration(std::integral_constant<int, 1>{}, tb + 1 - ph);
        if (tb + 2 >= ph && tb + 2 < tau1) iteration(std::integral_constant<int, 2>{}, tb + 2 - ph);
        if (tb + 3 >= ph && tb + 3 < tau1) iteration(std::integral_constant<int, 3>{}, tb + 3 - ph);
      }
    } else {
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
#pragma unroll
      for (int k = 0; k < NCH; ++k) qraw[0][k] = qraw[1][k] = u32x4{0u, 0u, 0u, 0u};
    }

    // ---- drain: O^T += V^T P^T of the last tile ------------------------------------------------
    {
      const int sl = (ph + nt - 1) & 3;
      const int off = sl * TILE_BYTES;
      // its weights are pw[sl & 1] (picked as values: an array indexed at run time would be put
      // into scratch memory); the fragments of the first KS d-blocks were preloaded by the last body
      i32x8 e = pw[0], d = pw[1];
      asm volatile("" : "+v"(e), "+v"(d));
      const i32x8 pl = (sl & 1) ? d : e;
#pragma unroll
      for (int i = 0; i < DB; ++i) {
        o[i] = mma(vf[i % KS], pl, o[i]);
        if (i + KS < DB) vf[i % KS] = ldv(off, i + KS);
      }
    }

    // ---- epilogue ---------------------------------------------------------------------------------
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    if (done.part < 0) {
      // final rows, turned around in the wave's staging area and stored with the non-temporal hint
      const float inv = P.out_scale / l_tot;
      const int ln = lane_now();
      const uint32_t roff = roff_of(ln), cx = cx_of(ln);
      const uint32_t wbase = carea_of(ln) + (uint32_t)(ln >> 5) * 8u;
      int grow[NCH];                    // head-row (token * Hq + head) of the row in out, -1: not a row of this tile
#pragma unroll
      for (int k = 0; k < NCH; ++k) {
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
        for (int k = 0; k < NCH; ++k) {
          const u32x4 val = *(const __attribute__((address_space(3))) u32x4*)(lds_ptr)(uintptr_t)(area_of(k) + roff);
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
        // the reference in log2 units (the merge is launched with a factor of 1); a column that saw
        // no key of the piece must not set the maximum there
        P.part_ml[slot * 2 + 0] = l_tot > 0.f ? mref : -1e30f;
        P.part_ml[slot * 2 + 1] = l_tot;
      }
    }
    if (more) q_collect();
    if (!more) break;
    ++p;
    ph = (ph + nt) & 3;
  }
}
