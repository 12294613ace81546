// Internal: host-side layout handle shared by the layout builder and the launch code.
#pragma once
#include <cstdint>
#include <vector>

#include "../../include/s2attn.h"

namespace s2 {

// Merged tile list: groups of `group` block rows (or block columns) share one list of partner
// blocks; each entry packs (partner_index << 16) | membership_bits, bit r set when member r of
// the group keeps that partner.  With 16-token blocks a partner is a UNIT of two adjacent blocks
// (the kernels step through partners 32 tokens at a time at least) and bit 2r + c says that
// member r keeps block c of the unit.  This is the Merge-Q idea of section 3.2 (one large tile serves
// several fine-grained mask rows) and its mirror image for key tiles.  Row groups are
// consecutive rows.  Column groups are formed from columns with similar partner sets (a stripe
// column is attended by every later row, its neighbours only by the local window), so members
// of a column group need not be adjacent: `members` names them (they are adjacent for 16-token
// blocks, where a wavefront's 32 key rows span two members).
constexpr int kMaxListUnits = 1 << 15;  // partner indices take the 15 bits above the membership bits

struct TileList {
  int group = 0;                 // members per tile (1..8; members x blocks per unit <= 16 bits)
  int tiles_per_head = 0;        // ceil(B / group)
  std::vector<int32_t> ptr;      // [H*tiles_per_head + 1]
  std::vector<int32_t> ent;      // packed entries; partner ascending inside a row tile,
                                 // descending inside a column tile
  std::vector<int32_t> order;    // [H*tiles_per_head]: per head, tile ids by descending length
  std::vector<int32_t> members;  // [H*tiles_per_head*group]: block index of each member, -1 = none
  int32_t* d_ptr = nullptr;      // device copies (owned by the layout)
  int32_t* d_ent = nullptr;
  int32_t* d_order = nullptr;
  int32_t* d_members = nullptr;
  int max_len = 0;
};

}  // namespace s2

struct s2_layout {
  s2_layout_params p{};
  std::vector<int32_t> row_ptr, col_idx, col_ptr, row_idx;
  int64_t nnz = 0;
  int max_row_blocks = 0;
  int covers_all = 0;
  bool on_device = false;
  int device = -1;
  int32_t* d_row_ptr = nullptr;  // device copies of the compressed rows (decode reads one row of them)
  int32_t* d_col_idx = nullptr;
  s2::TileList fwd_tiles; // row groups  -> kept KV blocks   (forward)
  s2::TileList q_tiles;   // row groups  -> kept KV blocks   (dQ pass)
  s2::TileList kv_tiles;  // column groups -> attending Q blocks (dK/dV pass)
  // Backward that keeps dS (64- and 128-token blocks): the dK/dV pass leaves dS in units of 64
  // queries x 64 keys, unit (2 * step + wavefront pair) of its walk over kv_tiles; dq_units names, for
  // every 64-key chunk of the q_tiles lists and either 64-row half of the query tile, the unit that
  // holds it (-1: the mask row drops the block, or no pair of the piece is causal).
  std::vector<int32_t> dq_units;
  int32_t* d_dq_units = nullptr;
  int64_t ds_units = 0;   // units per batch element (0: this layout does not support the path)
};

namespace s2 {
// Host-only construction (no HIP calls).  Returns an S2_* status.
int build_host(const s2_layout_params& p, s2_layout& L);
// The same from caller-supplied compressed rows (validated: ascending, causal, diagonal kept).
int build_from_csr(int num_heads, int num_blocks, int block_size, const int32_t* row_ptr,
                   const int32_t* col_idx, s2_layout& L);
// Kept block columns of block row i of local head `head`, ascending, in closed form (no layout
// needed, any i >= 0): writes at most `capacity` of them to out and returns how many there are.
int64_t row_blocks(const s2_layout_params& p, int head, int i, int32_t* out, int64_t capacity);
// Merge `group` consecutive rows (transpose=false) or columns (transpose=true).
void build_tiles(const s2_layout& L, int group, bool transpose, TileList& out);
// Fills dq_units / ds_units from q_tiles and kv_tiles (built before, with 128-row and 128-key tiles).
void build_ds_units(s2_layout& L);
}  // namespace s2
