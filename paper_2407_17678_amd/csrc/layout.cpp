// Host-side layout builder: the per-head block mask of section 4.2 written out in closed form
// as compressed lists (section 3.2 stores the mask in compressed-sparse-row form), plus the
// merged tile lists the kernels iterate over.  Integer work only; no HIP calls in this file.
#include "layout.h"

#include <algorithm>
#include <limits>
#include <numeric>

namespace s2 {

namespace {

inline int head_offset(const s2_layout_params& p, int h) {
  return p.stride > 0 ? (p.head_index_base + h) % p.stride : 0;
}

// Kept columns of block row i, ascending: the stripe columns o, o+s, ... that lie at least B_l
// rows back (and inside the window), then the local run ending at the diagonal.
template <class F>
inline void for_row(const s2_layout_params& p, int o, int i, F&& emit) {
  if (p.dense) {
    for (int j = 0; j <= i; ++j) emit(j);
    return;
  }
  const int local_lo = std::max(0, i - p.local_blocks + 1);
  if (p.stride > 0) {
    int lo = 0;  // smallest admissible column
    if (p.window_blocks > 0) lo = std::max(0, i - p.window_blocks + 1);
    // first stripe column >= lo
    int j = o;
    if (lo > o) j = o + ((lo - o + p.stride - 1) / p.stride) * p.stride;
    for (; j < local_lo; j += p.stride) emit(j);
  }
  for (int j = local_lo; j <= i; ++j) emit(j);
}

// Rows keeping block column j, ascending: the local run starting at the diagonal, then (when j
// lies on one of the head's stripes) every later row inside the window.
template <class F>
inline void for_col(const s2_layout_params& p, int o, int j, F&& emit) {
  const int B = p.num_blocks;
  if (p.dense) {
    for (int i = j; i < B; ++i) emit(i);
    return;
  }
  const int local_hi = std::min(B - 1, j + p.local_blocks - 1);
  for (int i = j; i <= local_hi; ++i) emit(i);
  if (p.stride > 0 && j >= o && (j - o) % p.stride == 0) {
    int hi = B - 1;
    if (p.window_blocks > 0) hi = std::min(hi, j + p.window_blocks - 1);
    for (int i = local_hi + 1; i <= hi; ++i) emit(i);
  }
}

}  // namespace

namespace {
// union over heads covers every causal block?
int covers_all_blocks(const s2_layout& L) {
  const int H = L.p.num_heads, B = L.p.num_blocks;
  std::vector<uint8_t> seen((size_t)B);
  for (int i = 0; i < B; ++i) {
    std::fill(seen.begin(), seen.begin() + i + 1, 0);
    for (int h = 0; h < H; ++h) {
      const int32_t* c = L.col_idx.data() + L.row_ptr[(size_t)h * B + i];
      const int32_t* e = L.col_idx.data() + L.row_ptr[(size_t)h * B + i + 1];
      for (; c != e; ++c) seen[*c] = 1;
    }
    for (int j = 0; j <= i; ++j)
      if (!seen[j]) return 0;
  }
  return 1;
}
}  // namespace

int64_t row_blocks(const s2_layout_params& p, int head, int i, int32_t* out, int64_t capacity) {
  int64_t n = 0;
  for_row(p, head_offset(p, head), i, [&](int j) {
    if (n < capacity) out[n] = j;
    ++n;
  });
  return n;
}

int build_host(const s2_layout_params& p, s2_layout& L) {
  if (p.num_heads < 1 || p.num_blocks < 1 || p.head_index_base < 0) return S2_ERR_BAD_PARAM;
  if (p.block_size != 16 && p.block_size != 32 && p.block_size != 64 && p.block_size != 128)
    return S2_ERR_BAD_PARAM;
  if (p.block_size == 16 && (p.num_blocks & 1)) return S2_ERR_BAD_PARAM;  // whole 32-token units
  if (!p.dense && (p.local_blocks < 1 || p.stride < 0 || p.window_blocks < 0)) return S2_ERR_BAD_PARAM;
  if (p.dense != 0 && p.dense != 1) return S2_ERR_BAD_PARAM;
  const int H = p.num_heads, B = p.num_blocks;
  if ((int64_t)H * B + 1 > std::numeric_limits<int32_t>::max()) return S2_ERR_OVERFLOW;
  if ((int64_t)B * p.block_size > std::numeric_limits<int32_t>::max()) return S2_ERR_OVERFLOW;
  if (B / (p.block_size < 32 ? 2 : 1) > kMaxListUnits) return S2_ERR_OVERFLOW;

  L.p = p;
  // pass 1: count
  int64_t nnz = 0;
  int max_row = 0;
  L.row_ptr.assign((size_t)H * B + 1, 0);
  for (int h = 0; h < H; ++h) {
    const int o = head_offset(p, h);
    for (int i = 0; i < B; ++i) {
      int c = 0;
      for_row(p, o, i, [&](int) { ++c; });
      nnz += c;
      if (nnz > std::numeric_limits<int32_t>::max()) return S2_ERR_OVERFLOW;
      max_row = std::max(max_row, c);
      L.row_ptr[(size_t)h * B + i + 1] = (int32_t)nnz;
    }
  }
  L.nnz = nnz;
  L.max_row_blocks = max_row;
  // pass 2: fill rows
  L.col_idx.resize((size_t)nnz);
  for (int h = 0; h < H; ++h) {
    const int o = head_offset(p, h);
    for (int i = 0; i < B; ++i) {
      int32_t* dst = L.col_idx.data() + L.row_ptr[(size_t)h * B + i];
      for_row(p, o, i, [&](int j) { *dst++ = j; });
    }
  }
  // transpose, also in closed form
  L.col_ptr.assign((size_t)H * B + 1, 0);
  L.row_idx.resize((size_t)nnz);
  int64_t n = 0;
  for (int h = 0; h < H; ++h) {
    const int o = head_offset(p, h);
    for (int j = 0; j < B; ++j) {
      for_col(p, o, j, [&](int i) { L.row_idx[(size_t)n++] = i; });
      L.col_ptr[(size_t)h * B + j + 1] = (int32_t)n;
    }
  }
  if (n != nnz) return S2_ERR_BAD_PARAM;  // the two closed forms disagree: a bug, never silent

  L.covers_all = covers_all_blocks(L);
  return S2_OK;
}

int build_from_csr(int num_heads, int num_blocks, int block_size, const int32_t* row_ptr,
                   const int32_t* col_idx, s2_layout& L) {
  if (num_heads < 1 || num_blocks < 1) return S2_ERR_BAD_PARAM;
  if (block_size != 16 && block_size != 32 && block_size != 64 && block_size != 128) return S2_ERR_BAD_PARAM;
  if (block_size == 16 && (num_blocks & 1)) return S2_ERR_BAD_PARAM;  // whole 32-token units
  const int H = num_heads, B = num_blocks;
  if ((int64_t)H * B + 1 > std::numeric_limits<int32_t>::max()) return S2_ERR_OVERFLOW;
  if ((int64_t)B * block_size > std::numeric_limits<int32_t>::max()) return S2_ERR_OVERFLOW;
  if (B / (block_size < 32 ? 2 : 1) > kMaxListUnits) return S2_ERR_OVERFLOW;
  const size_t rows = (size_t)H * B;
  if (row_ptr[0] != 0) return S2_ERR_BAD_PARAM;
  int max_row = 0;
  for (size_t r = 0; r < rows; ++r) {
    const int64_t lo = row_ptr[r], hi = row_ptr[r + 1];
    if (hi <= lo) return S2_ERR_BAD_PARAM;  // every row keeps at least its diagonal block
    const int i = (int)(r % B);
    // strictly ascending, none above the diagonal, the diagonal itself last
    for (int64_t n = lo; n < hi; ++n) {
      const int j = col_idx[n];
      if (j < 0 || j > i) return S2_ERR_BAD_PARAM;
      if (n > lo && j <= col_idx[n - 1]) return S2_ERR_BAD_PARAM;
    }
    if (col_idx[hi - 1] != i) return S2_ERR_BAD_PARAM;
    max_row = std::max(max_row, (int)(hi - lo));
  }
  const int64_t nnz = row_ptr[rows];
  L.p = s2_layout_params{};
  L.p.num_heads = H;
  L.p.num_blocks = B;
  L.p.block_size = block_size;
  L.nnz = nnz;
  L.max_row_blocks = max_row;
  L.row_ptr.assign(row_ptr, row_ptr + rows + 1);
  L.col_idx.assign(col_idx, col_idx + nnz);
  // transpose by counting; rows come out ascending inside each column because rows are visited
  // in ascending order
  L.col_ptr.assign(rows + 1, 0);
  for (int h = 0; h < H; ++h)
    for (int i = 0; i < B; ++i)
      for (int32_t n = row_ptr[(size_t)h * B + i]; n < row_ptr[(size_t)h * B + i + 1]; ++n)
        ++L.col_ptr[(size_t)h * B + col_idx[n] + 1];
  for (size_t r = 0; r < rows; ++r) L.col_ptr[r + 1] += L.col_ptr[r];
  L.row_idx.resize((size_t)nnz);
  std::vector<int32_t> fill(L.col_ptr.begin(), L.col_ptr.end() - 1);
  for (int h = 0; h < H; ++h)
    for (int i = 0; i < B; ++i)
      for (int32_t n = row_ptr[(size_t)h * B + i]; n < row_ptr[(size_t)h * B + i + 1]; ++n)
        L.row_idx[(size_t)fill[(size_t)h * B + col_idx[n]]++] = i;
  L.covers_all = covers_all_blocks(L);
  return S2_OK;
}

// column tiles of one length that a head must have before they walk their rows in step (see below)
constexpr int kRotateMinTiles = 8;

void build_tiles(const s2_layout& L, int group, bool transpose, TileList& out) {
  // partner blocks per entry: the kernels walk partners in units of at least 32 tokens, so with
  // 16-token blocks an entry covers two of them
  const int sub = L.p.block_size < 32 ? 32 / L.p.block_size : 1;
  const int H = L.p.num_heads, B = L.p.num_blocks;
  const std::vector<int32_t>& ptr = transpose ? L.col_ptr : L.row_ptr;
  const std::vector<int32_t>& idx = transpose ? L.row_idx : L.col_idx;
  const int T = (B + group - 1) / group;
  out.group = group;
  out.tiles_per_head = T;
  out.ptr.assign((size_t)H * T + 1, 0);
  out.ent.clear();
  out.order.resize((size_t)H * T);
  out.members.assign((size_t)H * T * group, -1);
  out.max_len = 0;
  std::vector<int> cur(group), end(group);
  std::vector<int32_t> seq(B);
  for (int h = 0; h < H; ++h) {
    const int32_t* hp0 = ptr.data() + (size_t)h * B;
    // which blocks go together: rows stay in order; columns are sorted by how many rows keep
    // them (longest first, ties by index) so that stripe columns pair up with stripe columns
    std::iota(seq.begin(), seq.end(), 0);
    // (with 16-token blocks members stay adjacent, which the kernel relies on for its key rows)
    if (transpose && group > 1 && sub == 1)
      std::stable_sort(seq.begin(), seq.end(),
                       [&](int a, int b) { return hp0[a + 1] - hp0[a] > hp0[b + 1] - hp0[b]; });
    for (int t = 0; t < T; ++t) {
      const int n_members = std::min(group, B - t * group);
      int32_t* mem = out.members.data() + ((size_t)h * T + t) * group;
      for (int r = 0; r < n_members; ++r) mem[r] = seq[t * group + r];
      std::sort(mem, mem + n_members);
      for (int r = 0; r < n_members; ++r) {
        cur[r] = hp0[mem[r]];
        end[r] = hp0[mem[r] + 1];
      }
      const size_t start = out.ent.size();
      for (;;) {  // k-way merge of ascending lists
        int best = std::numeric_limits<int>::max();
        for (int r = 0; r < n_members; ++r)
          if (cur[r] < end[r]) best = std::min(best, (int)idx[cur[r]] / sub);
        if (best == std::numeric_limits<int>::max()) break;
        int bits = 0;
        for (int r = 0; r < n_members; ++r)
          while (cur[r] < end[r] && idx[cur[r]] / sub == best) {
            bits |= 1 << (r * sub + idx[cur[r]] % sub);
            ++cur[r];
          }
        out.ent.push_back((int32_t)((best << 16) | bits));
      }
      // Column tiles are walked from the last query block down.  Every stripe tile of a head ends
      // at the last row, so tiles started together then read the same Q / dO blocks at the same
      // time and share them in L2 instead of each streaming them from HBM.
      if (transpose) std::reverse(out.ent.begin() + start, out.ent.end());
      const int len = (int)(out.ent.size() - start);
      out.max_len = std::max(out.max_len, len);
      out.ptr[(size_t)h * T + t + 1] = (int32_t)out.ent.size();
    }
    // ... except where many column tiles have the same length and each attends one unbroken run of
    // rows: the local-window tiles, whose runs are shifted against each other by a tile's width.
    // They are dispatched one after the other (equal lengths keep their index order below) and run
    // side by side, and walking every run from its own end would have neighbours read the same Q / dO
    // block several steps apart - by then it has left the L2.  Such a tile of n entries instead starts
    // at its row that is a multiple of n and goes down from there, wrapping round to its last row: at
    // any step, tiles of one length are at rows congruent modulo n, which for overlapping runs is the
    // same row.
    if (transpose) {
      const int32_t* hp = out.ptr.data() + (size_t)h * T;
      std::vector<int> same((size_t)out.max_len + 2, 0);
      for (int t = 0; t < T; ++t) ++same[hp[t + 1] - hp[t]];
      for (int t = 0; t < T; ++t) {
        const int n = hp[t + 1] - hp[t];
        if (n < 2 || same[n] < kRotateMinTiles) continue;
        int32_t* e = out.ent.data() + hp[t];
        const int top = e[0] >> 16, bottom = e[n - 1] >> 16;
        if (top - bottom != n - 1) continue;  // not one unbroken run
        std::rotate(e, e + (top - (top / n) * n), e + n);
      }
    }
    // heaviest tiles first inside the head, so the tail of a launch is made of short tiles
    int32_t* ord = out.order.data() + (size_t)h * T;
    std::iota(ord, ord + T, 0);
    const int32_t* hp = out.ptr.data() + (size_t)h * T;
    std::stable_sort(ord, ord + T, [&](int a, int b) { return hp[a + 1] - hp[a] > hp[b + 1] - hp[b]; });
  }
}

void build_ds_units(s2_layout& L) {
  L.dq_units.clear();
  L.ds_units = 0;
  const int S = L.p.block_size;
  if (S != 64 && S != 128) return;
  const int sub = S / 64;  // 64-token pieces per block side = 64-row chunks per list entry
  const int H = L.p.num_heads, B = L.p.num_blocks;
  const TileList& kt = L.kv_tiles;
  const TileList& qt = L.q_tiles;
  if (kt.group != 128 / S || qt.group != 128 / S) return;
  if ((int64_t)kt.ent.size() * sub * 2 > std::numeric_limits<int32_t>::max()) return;
  // position of block (i, j) of head h in the compressed rows (it is there: both lists come from them)
  auto csr_pos = [&](int h, int i, int j) -> int64_t {
    const int32_t* lo = L.col_idx.data() + L.row_ptr[(size_t)h * B + i];
    const int32_t* hi = L.col_idx.data() + L.row_ptr[(size_t)h * B + i + 1];
    const int32_t* it = std::lower_bound(lo, hi, j);
    return (it != hi && *it == j) ? (int64_t)(it - L.col_idx.data()) : -1;
  };
  // the dK/dV pass: which unit each 64 x 64 piece of a kept block goes to
  std::vector<int32_t> unit_of((size_t)L.nnz * sub * sub, -1);
  const int Tk = kt.tiles_per_head;
  for (int h = 0; h < H; ++h)
    for (int t = 0; t < Tk; ++t) {
      const int32_t* mem = kt.members.data() + ((size_t)h * Tk + t) * kt.group;
      for (int32_t eg = kt.ptr[(size_t)h * Tk + t]; eg < kt.ptr[(size_t)h * Tk + t + 1]; ++eg) {
        const int e = kt.ent[(size_t)eg], partner = e >> 16;
        for (int c = 0; c < sub; ++c) {
          const int q64 = partner * sub + (sub - 1 - c);  // the pass walks an entry's chunks last first
          for (int pair = 0; pair < 2; ++pair) {
            const int member = sub == 1 ? pair : 0;
            if (mem[member] < 0 || !((e >> member) & 1)) continue;
            const int k64 = sub == 1 ? mem[member] : mem[0] * 2 + pair;
            if (k64 > q64) continue;  // every key of the piece lies after every query: never computed
            const int64_t n = csr_pos(h, q64 / sub, k64 / sub);
            if (n < 0) continue;
            unit_of[(size_t)n * sub * sub + (q64 % sub) * sub + k64 % sub] = (int32_t)(((int64_t)eg * sub + c) * 2 + pair);
          }
        }
      }
    }
  // the dQ pass: where each chunk of its lists finds its two pieces
  const int Tq = qt.tiles_per_head;
  L.dq_units.assign(qt.ent.size() * sub * 2, -1);
  for (int h = 0; h < H; ++h)
    for (int t = 0; t < Tq; ++t)
      for (int32_t eg = qt.ptr[(size_t)h * Tq + t]; eg < qt.ptr[(size_t)h * Tq + t + 1]; ++eg) {
        const int e = qt.ent[(size_t)eg], j = e >> 16;
        for (int c = 0; c < sub; ++c) {
          const int k64 = j * sub + c;
          for (int m = 0; m < 2; ++m) {
            const int q64 = t * 2 + m, member = (m * 64) / S;
            if (q64 / sub >= B || !((e >> member) & 1) || k64 > q64) continue;
            const int64_t n = csr_pos(h, q64 / sub, j);
            if (n < 0) continue;
            L.dq_units[((size_t)eg * sub + c) * 2 + m] = unit_of[(size_t)n * sub * sub + (q64 % sub) * sub + k64 % sub];
          }
        }
      }
  L.ds_units = (int64_t)kt.ent.size() * sub * 2;
}

}  // namespace s2
