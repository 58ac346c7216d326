// Work decomposition shared by the attention kernels.
//
// A launch covers some or all heads of the layer.  Its grid is up to four consecutive segments
// of work items, longest items first so the short ones fill the tail of the launch:
//   [ route 1: (slot, q-block over the text rows)         | keys: rows [0, N)                  ]
//   [ route 0: (head, q-block) over all N rows            | keys: rows [0, N) of the head      ]
//   [ route 2: (slot, q-block) over L_c + n_text rows     | keys: all rows of the core-set     ]
//   [ route 1: (slot, tile, q-block inside the tile)      | keys: the tile's run list          ]
// A work item is BM query rows; its keys are a short list of runs of consecutive rows.  The
// text rows of a window head attend to every row, so their items cost as much as those of a
// full-attention head and sit with them at the front.
#pragma once

#include <cstdint>

#include "vorta_internal.h"

namespace vorta {

struct AttnArgs {
  // route 0: caller's tensors
  const void *q0, *k0, *v0;
  void* o0;
  long head_stride0, row_stride0;   // elements
  // route 2: [n_lr][Nc][d]
  const void *qc, *kc, *vc;
  void* oc;
  // route 1: [n_win][N][d] in tile order
  const void *qt, *kt, *vt;
  void* ot;
  // route 1 without tile-ordered copies (qt == null): rows of the caller's tensors are gathered
  // through tok_of (tile-order index -> token index); win_heads = head id of each window slot
  const int* tok_of;                // [N]
  const int* tile_row0;             // [n_tiles + 1]: first tile-order row of each tile (edge tiles may be clipped)
  int win_gather;
  const int* runs;                  // [n_tiles][max_runs][2]
  const int* n_runs;                // [n_tiles]
  int max_runs;
  int N, Nc, L, n_text;
  int n_tiles, tile_tokens;
  // Route 1, gathered form, tiles of at most 128 tokens: window tiles whose key sets are identical
  // (under the clamped centre rule the first floor(w/2) + 1 tiles of every axis end, under the
  // block rule all tiles of a block) are computed together, up to three tiles and 256 rows per
  // work item -- one key stream serves them all.  win_items[i] = {tile, tile, tile, count};
  // a launch covers entries [win_first, win_first + win_count) for every window head.
  // Null: one item per (tile, q-block), by arithmetic.
  const int* win_items;
  int win_first, win_count;
  // The last work items of a launch leave most CUs idle while a few finish them.  Items with
  // index >= split_from are therefore issued as two items of BM / 2 rows each (grid index
  // split_from + 2 j + h -> rows [h BM / 2, (h + 1) BM / 2) of item split_from + j); a workgroup
  // whose upper wavefronts have no rows runs them as helpers (staging only), which takes about
  // half the time of a full item.  split_from = INT_MAX: no split.
  int split_from;
  int qb_dense, qb_core, qb_tile, qb_text;   // q-blocks per head / core-set / tile / text part
  int end_text, end_dense, end_core, end_tile;   // cumulative item counts, in grid order; end_tile = all
  float scale;
  uint8_t dense_heads[VORTA_MAX_HEADS];
  uint8_t win_heads[VORTA_MAX_HEADS];
};

// Eq. 5 epilogue of a dense launch over all heads: the rows it writes are
//   a1 (its own result) + a2 (the sliding-tile result, already in `out`) + a3 (core-set result of
//   the slot the row is assigned to),
// the first still in registers / LDS, the other two read as bf16 rows.  Text rows see every key
// under the sliding-tile branch too, so for them the second term equals the first.
struct MixArgs {
  const void* oc;              // [heads][Nc][d]: core-set outputs of every head
  const int* assign;           // [heads][L]
  int Lc;
  float alpha[VORTA_MAX_HEADS][3];
};
struct NoMix {};

struct WorkItem {
  long q_off, kv_off, o_off;   // element offsets of the head's row 0 in q / k,v / o
  long row_stride;             // elements
  int head;                    // head id (dense segment only)
  int seg;                     // 0 dense, 1 core-set, 2 window
  int row0, n_rows;            // query rows: n_rows of them; row i is row(i) below
  // an item made of several tiles: its rows are up to three ranges of tile-order rows, range 0
  // from row0, the others from rb1, rb2; rc0, rc1 = rows before range 1, range 2; first = the
  // workgroup's first row within the item.  Single range: rc0 = INT_MAX, first = 0.
  int rb1, rb2, rc0, rc1, first;
  __device__ __forceinline__ int row(int i) const {
    const int r = first + i;
    return r < rc0 ? row0 + r : r < rc1 ? rb1 + (r - rc0) : rb2 + (r - rc1);
  }
  int n_runs;
  const int* runs;             // null: the single run {0, single_len}
  int single_len;
};

template <int BM, int D>
__device__ __forceinline__ WorkItem decode_item(const AttnArgs& a, int item) {
  WorkItem w;
  w.runs = nullptr;
  w.n_runs = 1;
  w.head = 0;
  w.rb1 = w.rb2 = w.first = 0;
  w.rc0 = w.rc1 = 0x7fffffff;
  int half = -1;
  if (item >= a.split_from) {
    half = (item - a.split_from) & 1;
    item = a.split_from + ((item - a.split_from) >> 1);
  }
  if (item < a.end_text) {
    const int slot = item / a.qb_text, qb = item - slot * a.qb_text;
    w.seg = a.win_gather ? 0 : 2;   // gathered: rows of the caller's tensors, like a dense head
    w.q_off = w.kv_off = w.o_off = a.win_gather ? a.win_heads[slot] * a.head_stride0 : (long)slot * a.N * D;
    w.row_stride = a.win_gather ? a.row_stride0 : D;
    w.row0 = a.L + qb * BM;
    w.n_rows = min(BM, a.n_text - qb * BM);
    w.single_len = a.N;
  } else if (item < a.end_dense) {
    item -= a.end_text;
    const int slot = item / a.qb_dense, qb = item - slot * a.qb_dense;
    w.seg = 0;
    w.head = a.dense_heads[slot];
    w.q_off = w.kv_off = w.o_off = a.dense_heads[slot] * a.head_stride0;
    w.row_stride = a.row_stride0;
    w.row0 = qb * BM;
    w.n_rows = min(BM, a.N - w.row0);
    w.single_len = a.N;
  } else if (item < a.end_core) {
    item -= a.end_dense;
    const int slot = item / a.qb_core, qb = item - slot * a.qb_core;
    w.seg = 1;
    w.q_off = w.kv_off = w.o_off = (long)slot * a.Nc * D;
    w.row_stride = D;
    w.row0 = qb * BM;
    w.n_rows = min(BM, a.Nc - w.row0);
    w.single_len = a.Nc;
  } else if (a.win_items) {
    item -= a.end_core;
    const int slot = item / a.win_count, i = item - slot * a.win_count;
    const int* it = a.win_items + 4 * (a.win_first + i);
    const int t0 = it[0], count = it[3];
    w.seg = 2;
    w.q_off = w.kv_off = w.o_off = a.win_heads[slot] * a.head_stride0;    // gathered form only
    w.row_stride = a.row_stride0;
    w.row0 = a.tile_row0[t0];
    w.n_rows = a.tile_row0[t0 + 1] - w.row0;
    if (count > 1) {
      const int t1 = it[1];
      w.rb1 = a.tile_row0[t1];
      w.rc0 = w.n_rows;
      w.n_rows += a.tile_row0[t1 + 1] - w.rb1;
    }
    if (count > 2) {
      const int t2 = it[2];
      w.rb2 = a.tile_row0[t2];
      w.rc1 = w.n_rows;
      w.n_rows += a.tile_row0[t2 + 1] - w.rb2;
    }
    w.runs = a.runs + (long)t0 * a.max_runs * 2;      // the same for every tile of the item
    w.n_runs = a.n_runs[t0];
    w.single_len = 0;
    if (half >= 0) {
      w.first = half * (BM / 2);
      w.n_rows = min(BM / 2, w.n_rows - w.first);
    }
    return w;
  } else {
    item -= a.end_core;
    const int per_head = a.n_tiles * a.qb_tile;
    const int slot = item / per_head, r = item - slot * per_head;
    const int tile = r / a.qb_tile, qb = r - tile * a.qb_tile;
    w.seg = 2;
    w.q_off = w.kv_off = w.o_off = a.win_gather ? a.win_heads[slot] * a.head_stride0 : (long)slot * a.N * D;
    w.row_stride = a.win_gather ? a.row_stride0 : D;
    const int first = a.tile_row0[tile];
    w.row0 = first + qb * BM;
    w.n_rows = min(BM, a.tile_row0[tile + 1] - first - qb * BM);   // <= 0 for a clipped tile with fewer q-blocks
    w.runs = a.runs + (long)tile * a.max_runs * 2;
    w.n_runs = a.n_runs[tile];
    w.single_len = 0;
  }
  if (half >= 0) {          // n_rows may come out <= 0 here too: the workgroup then has nothing to do
    w.row0 += half * (BM / 2);
    w.n_rows = min(BM / 2, w.n_rows - half * (BM / 2));
  }
  return w;
}

// Work item of a workgroup.  Consecutive workgroup ids are dealt round-robin to the 8 XCDs
// (each with its own L2); with chunked = true the ids are re-dealt so that every XCD gets one
// contiguous range of the n items instead -- neighbouring window tiles, whose key sets
// overlap, then run on the same XCD at about the same time and share its L2.  Only for
// launches whose items all cost the same (a contiguous deal of unequal items would leave
// some XCDs with all the long ones).
__device__ __forceinline__ int xcd_item(int block, int n, bool chunked) {
  if (!chunked) return block;
  const int xcd = block & 7, loc = block >> 3, q = n >> 3, r = n & 7;
  return xcd * q + min(xcd, r) + loc;
}

// Work of the window heads (route 1) that a launch includes.
enum WindowPart { WIN_NONE = 0, WIN_TEXT = 1, WIN_TILES = 2, WIN_ALL = 3 };

// Fills AttnArgs for a launch over the heads of rl with BM-row work items; win_part selects
// which items of the window heads it carries.  win_list: -1 = one item per (tile, q-block);
// 0 / 1 = the plan's grouped items of more than 128 rows / of at most 128 rows.
int fill_attn_args(vorta_plan* p, const RouteLists& rl, const vorta_attn_io* io, int BM, int win_part, AttnArgs* a,
                   int win_list = -1);

int launch_attention_bf16(vorta_plan* p, const RouteLists& rl, const vorta_attn_io* io, void* stream,
                          const MixArgs* mix = nullptr, bool win_text = true);

}  // namespace vorta
