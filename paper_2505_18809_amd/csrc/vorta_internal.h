// Internal declarations shared by the translation units of libvorta.
#pragma once

#include <cstdint>
#include <mutex>
#include <vector>

#include "vorta.h"

struct vorta_plan {
  vorta_layer_desc d;
  int64_t L = 0, N = 0;          // video tokens, all tokens
  int nt[3] = {0, 0, 0};         // tile grid
  int n_tiles = 0, tile_tokens = 0;
  int nb[3] = {0, 0, 0};         // bucket grid (ceil)
  int n_buckets = 0;
  int64_t Lc = 0;                // core-set slots
  int max_runs = 0;
  int window_key_tiles = 0;
  int elem_bytes = 0;
  float scale = 0.f;
  // first row of every tile in tile order, [n_tiles + 1]: a tile that the grid clips (the tile
  // does not divide the axis) holds fewer rows than tile_tokens
  std::vector<int32_t> tile_row0;
  std::vector<int32_t> boxes;    // [n_tiles][6]
  std::vector<int32_t> runs;     // [n_tiles][max_runs][2]
  std::vector<int32_t> n_runs;   // [n_tiles]
  std::vector<int32_t> slot_base;  // [n_buckets + 1]
  // window work items (tiles of at most 128 tokens): tiles with identical key sets grouped, up to
  // three tiles and 256 rows per item; {tile, tile, tile, count} each, the n_win_big items of more
  // than 128 rows first, then the n_win_small others.  Empty when a tile holds more than 128 tokens.
  std::vector<int32_t> win_items;
  int n_win_big = 0, n_win_small = 0;
  // rotary embedding: (cos, sin) of position * rate for every position of every axis,
  // [F][pairs_F] then [H][pairs_H] then [W][pairs_W]; empty without rope_dims
  bool rope = false;
  std::vector<float> rope_cs;

  // device copies of runs / n_runs / slot_base and the tile-order -> sequence-order token table
  // (identity for the text rows), uploaded on first device use
  std::mutex mu;
  bool on_device = false;
  int device = -1;
  int n_cus = 256;               // compute units of that device
  int32_t* d_runs = nullptr;
  int32_t* d_n_runs = nullptr;
  int32_t* d_slot_base = nullptr;
  int32_t* d_tok_of = nullptr;   // [N]
  int32_t* d_tile_row0 = nullptr;   // [n_tiles + 1]
  float* d_rope_cs = nullptr;
  int32_t* d_win_items = nullptr;
};

namespace vorta {

int fail(int code, const char* fmt, ...);        // records the thread-local message, returns code
void clear_error();

struct RouteLists {
  int count[3] = {0, 0, 0};
  int heads[3][VORTA_MAX_HEADS];                 // head ids per route, ascending
};
int split_routes(const vorta_plan* p, const uint8_t* routes, RouteLists* out);

int ensure_device_tables(vorta_plan* p);         // vorta_passes.hip
// set by the device side when it is linked in: frees the device tables of a plan
extern void (*g_release_device_tables)(vorta_plan* p);

// Launchers (each returns VORTA_OK / VORTA_EHIP).  Pointers are device memory.
struct UserTensor {                               // a tensor in the caller's layout
  const void* base;
  int64_t head_stride;                            // elements
  int64_t row_stride;                             // elements
};
UserTensor user_tensor(const vorta_plan* p, const void* base);

int launch_reorder(vorta_plan* p, const RouteLists& rl, const void* user, void* tiled, bool to_tiles,
                   void* stream);
// feat.head_stride == 0: one feature tensor shared by every head
int launch_bcs_index(vorta_plan* p, const RouteLists& rl, const UserTensor& feat, int32_t* keep_idx,
                     int32_t* assign, void* stream);
int launch_bcs_pool(vorta_plan* p, const RouteLists& rl, const void* src, const int32_t* keep_idx,
                    const int32_t* assign, bool rotate, void* dst, void* stream);
bool bcs_fused_applies(const vorta_plan* p);
int launch_bcs_select_pool(vorta_plan* p, const RouteLists& rl, const void* q, const void* k, const void* v,
                           int32_t* keep_idx, int32_t* assign, void* qc, void* kc, void* vc, void* stream);
int launch_rope_rows(vorta_plan* p, const RouteLists& rl, const void* src, void* dst, void* stream);
int launch_unpool(vorta_plan* p, const RouteLists& rl, const void* o_c, const int32_t* assign, void* out,
                  void* stream);
int launch_attention_f32(vorta_plan* p, const RouteLists& rl, const vorta_attn_io* io, void* stream);
int launch_router(const float* t_emb, const float* w_r, int n_steps, int d_t, int heads, float* alpha,
                  uint8_t* routes, void* stream);
int launch_blend3(vorta_plan* p, const void* o0, const void* o1, const void* o2, const float* alpha_host,
                  void* out, void* stream);

}  // namespace vorta
