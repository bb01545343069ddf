// Internal types shared by the host planner and the gfx950 kernels.
// Not part of the public ABI (see include/oppo_attn.h for that).
#pragma once
#include <stddef.h>
#include <stdint.h>

namespace oppo {

// Rows of the packed (token x q-head-of-group) query tile one workgroup owns:
// 8 waves x 32 query columns.
constexpr int kTileRows = 256;
// Keys per iteration of the key loop.
constexpr int kKeyTile = 64;
// Most pieces a query tile's key range is ever cut into.
constexpr int kMaxSplit = 32;
// Work descriptors travel by value in the kernel-argument segment, so the
// host arrays are snapshotted at launch time without any staging copy.
constexpr int kMaxAttnItems = 960;      // 960 * 32 B + queue table + header < 32 KiB
constexpr int kMaxQueues = 256;         // persistent workgroups per kv-head
constexpr int kMaxCombineItems = 1000;  // 1000 * 16 B + header
constexpr int kMaxAppendItems = 1000;   // 1000 * 16 B + header

// One piece of attention work: a tile of up to TM tokens of one sequence (all G
// q-heads of one kv-head; the kv-head comes from the block index) against the
// key range [k_begin, k_end) of that sequence.  A workgroup runs a queue of
// pieces one after the other.
struct AttnItem {
  int64_t kv_row0;  // row of the sequence's token 0 in the k/v arrays
  int32_t q_row0;   // row of the tile's first token in q/out
  int32_t n_tok;    // tokens in the tile (1..TM) | index of the tile within its chunk << 9
  int32_t pos0;     // absolute position of the tile's first token
  int32_t k_begin;  // first key of the range (multiple of kKeyTile)
  int32_t k_end;    // one past the last key, <= pos0 + n_tok
  int32_t part;     // -1: write final bf16 rows; >= 0: partial slot to fill
};
static_assert(sizeof(AttnItem) == 32, "AttnItem layout");
#if defined(__HIPCC__)
#define OPPO_HD __host__ __device__
#else
#define OPPO_HD
#endif
OPPO_HD inline int32_t pack_tokens(int n_tok, int tile) { return n_tok | (tile << 9); }
OPPO_HD inline int tokens_of(const AttnItem& a) { return a.n_tok & 511; }
OPPO_HD inline int tile_of(const AttnItem& a) { return a.n_tok >> 9; }

// Merge of the partial results of one split tile.
struct CombineItem {
  int32_t q_row0;
  int32_t n_tok;
  int32_t part0;   // first partial slot; the pieces are consecutive
  int32_t nsplit;
};

// One contiguous run of chunk rows going into a cache slab.
struct AppendItem {
  int64_t dst_row;  // first slot (token row) in the cache
  int32_t src_row;  // first row in k_new / v_new
  int32_t n_tok;
};

// One contiguous run of a pass's rows to rotate: rows [row0, row0 + n_tok) of q / k_new
// sit at absolute positions pos0, pos0 + 1, ...
struct RopeItem {
  int32_t row0;
  int32_t n_tok;
  int32_t pos0;
};

// One sequence's rows of a fused QKV projection output: rows [src_row, src_row + n_tok)
// at positions pos0, pos0 + 1, ...; keys and values go to cache rows dst_row, dst_row + 1, ...
struct QkvItem {
  int64_t dst_row;
  int32_t src_row;
  int32_t n_tok;
  int32_t pos0;
  int32_t pad_;
};

struct LayerShape {
  int32_t Hq, Hkv, G, D;
  int32_t TM;       // tokens per query tile = kTileRows / G
  float c;          // softmax_scale * log2(e) (8-bit cache: times the key tensor's scale)
  float out_scale = 1.0f;   // 8-bit cache: the value tensor's scale
  int32_t fp8 = 0;          // keys and values are E4M3 codes (values in blocks of 64 tokens)
};

// Launchers (kernels.hip).  Return a hipError_t as int (0 = success).
// k_new / v_new null: keys and values come from k / v alone.  Otherwise the
// kernel also appends: a sequence's keys from position pos0 - tile * TM on are
// read from k_new / v_new (rows indexed like q) and copied into k / v.
// timed: bracket the launch with an event pair while profiling is enabled.
int launch_attention(const LayerShape& ls, const void* q, void* k, void* v, const void* k_new, const void* v_new,
                     void* out, float* part_o, float* part_ml, const AttnItem* items, int n_items,
                     const uint16_t* first, int n_queues, void* stream, bool timed);
int launch_combine(const LayerShape& ls, void* out, const float* part_o, const float* part_ml,
                   const CombineItem* items, int n_items, void* stream, bool timed);
int launch_append(const LayerShape& ls, void* cache_k, void* cache_v, const void* k_new,
                  const void* v_new, const AppendItem* items, int n_items, int max_tok, void* stream);
// Append into a cache of E4M3 codes (keys token-major, values in blocks of 64 tokens, every
// dst_row's slab starting on a block boundary); k_inv / v_inv = fl32(1 / scale).
int launch_append_fp8(const LayerShape& ls, void* cache_k, void* cache_v, const void* k_new, const void* v_new,
                      float k_inv, float v_inv, const AppendItem* items, int n_items, void* stream);
// q / k null: that array is left alone.  (rope.hip)
int launch_rope(const LayerShape& ls, void* q, void* k, const RopeItem* items, int n_items, double theta_base,
                void* stream);
int launch_qkv_rope_append(const LayerShape& ls, const void* qkv, void* q_out, void* cache_k, void* cache_v,
                           const QkvItem* items, int n_items, double theta_base, void* stream);
// The fused QKV projection with the rotary / cache epilogue (gemm.hip).  workspace holds
// proj_workspace_bytes(D, rows) bytes of per-row data made by a small kernel of the same call.
size_t proj_workspace_bytes(int D, int64_t rows);
int launch_qkv_proj(const LayerShape& ls, const void* x, const void* w, int32_t hidden, int32_t rows, void* q_out,
                    void* cache_k, void* cache_v, const QkvItem* items, int n_items, double theta_base, void* workspace,
                    void* stream);
const char* hip_error_string(int err);

// The built-in scratch buffer of the entry point that allocates nothing: a device array
// of this many bytes that lives in the library's code object, one copy per GPU.
// static_scratch gives its address on the current device (looked up once per device).
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
int static_scratch(void** ptr);

// Records the reason of a failing call (thread-local, read by oppo_last_error) and
// returns `code`.
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
int profile_enable(int on);
bool profile_is_on();
// kinds: 0 attention, 1 merge, 2 append
int profile_read(double ms[3], int32_t launches[3], double* each_ms, int32_t* each_kind, int32_t max_each,
                 int32_t* n_each);

// Bytes of one partial slot (all kv-heads): kTileRows rows x (D + 2) floats each.
inline size_t part_slot_bytes(int Hkv, int D) {
  return (size_t)Hkv * kTileRows * (size_t)(D + 2) * sizeof(float);
}

}  // namespace oppo
