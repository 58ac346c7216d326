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
  int row0, n_rows;            // query rows [row0, row0 + n_rows)
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
// which items of the window heads it carries.
int fill_attn_args(vorta_plan* p, const RouteLists& rl, const vorta_attn_io* io, int BM, int win_part, AttnArgs* a);

int launch_attention_bf16(vorta_plan* p, const RouteLists& rl, const vorta_attn_io* io, void* stream,
                          const MixArgs* mix = nullptr, bool win_text = true);

}  // namespace vorta
