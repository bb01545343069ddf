// Stand-ins for the kernel launchers, for the CPU-only build of the host sources that the
// test suite runs under AddressSanitizer / UndefinedBehaviorSanitizer: every launcher checks
// what the kernels assume of a work list (bounds of the fixed-size argument arrays, key
// ranges on tile boundaries, slots inside the workspace) and launches nothing.
#include <stdint.h>
#include <stdlib.h>

#include "oppo_internal.h"

namespace oppo {

namespace {
int g_profile_on = 0;
}

int launch_attention(const LayerShape& ls, const void*, void*, void*, const void*, const void*, void*, float* part_o,
                     float*, const AttnItem* items, int n_items, const uint16_t* first, int n_queues, void*, bool) {
  if (n_items <= 0 || n_queues <= 0) return 0;
  if (n_items > kMaxAttnItems || n_queues > kMaxQueues) return 1;
  if (first[0] != 0 || first[n_queues] != n_items) return 1;
  for (int j = 0; j < n_queues; ++j)
    if (first[j] >= first[j + 1]) return 1;   // empty queues never reach the kernel
  for (int i = 0; i < n_items; ++i) {
    const AttnItem& a = items[i];
    const int n = tokens_of(a);
    if (n < 1 || n > ls.TM) return 1;
    if (a.k_begin < 0 || a.k_begin % kKeyTile != 0 || a.k_end <= a.k_begin || a.k_end > a.pos0 + n) return 1;
    if (a.part >= 0 && !part_o) return 1;
    if (ls.fp8 && a.kv_row0 % kKeyTile != 0) return 1;
  }
  return 0;
}

int launch_combine(const LayerShape&, void*, const float* part_o, const float*, const CombineItem* items, int n_items,
                   void*, bool) {
  for (int i = 0; i < n_items; ++i)
    if (items[i].nsplit < 2 || items[i].nsplit > kMaxSplit || items[i].part0 < 0 || !part_o) return 1;
  return 0;
}

int launch_append(const LayerShape&, void*, void*, const void*, const void*, const AppendItem* items, int n_items, int,
                  void*) {
  for (int i = 0; i < n_items; ++i)
    if (items[i].n_tok < 1 || items[i].dst_row < 0 || items[i].src_row < 0) return 1;
  return 0;
}

int launch_append_fp8(const LayerShape& ls, void*, void*, const void*, const void*, float k_inv, float v_inv,
                      const AppendItem* items, int n_items, void*) {
  if (!(k_inv > 0.0f) || !(v_inv > 0.0f) || (ls.D != 64 && ls.D != 128)) return 1;
  for (int i = 0; i < n_items; ++i)
    if (items[i].n_tok < 1 || items[i].dst_row < 0 || items[i].src_row < 0) return 1;
  return 0;
}

int launch_rope(const LayerShape&, void*, void*, const RopeItem*, int, double, void*) { return 0; }

int launch_qkv_rope_append(const LayerShape&, const void*, void*, void*, void*, const QkvItem*, int, double, void*) {
  return 0;
}

size_t proj_workspace_bytes(int D, int64_t rows) { return (size_t)rows * (8 + (size_t)(D / 2) * 8); }

int launch_qkv_proj(const LayerShape&, const void*, const void*, int32_t hidden, int32_t rows, void*, void*, void*,
                    const QkvItem* items, int n_items, double, void* workspace, void*) {
  if (hidden % 64 != 0 || rows <= 0 || !workspace) return 1;
  int64_t total = 0;
  for (int i = 0; i < n_items; ++i) total += items[i].n_tok;
  return total == rows ? 0 : 1;
}

const char* hip_error_string(int) { return "launcher stub refused the work list"; }

int static_scratch(void** ptr) {
  static void* block = malloc(256);   // an address only: nothing dereferences it on the host
  *ptr = block;
  return 0;
}

int profile_enable(int on) {
  g_profile_on = on;
  return 0;
}
bool profile_is_on() { return g_profile_on != 0; }
int profile_read(double ms[3], int32_t launches[3], double*, int32_t*, int32_t, int32_t* n_each) {
  for (int k = 0; k < 3; ++k) ms[k] = 0.0, launches[k] = 0;
  if (n_each) *n_each = 0;
  return 0;
}

}  // namespace oppo
