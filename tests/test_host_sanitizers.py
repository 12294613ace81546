"""The host side of the library (the closed-form layout builder, the builder from caller-supplied
rows, the merged tile lists and the unit table of the backward that keeps dS; integer code, no HIP) compiled with g++ under AddressSanitizer and
UndefinedBehaviorSanitizer and driven over the training workloads, a random parameter sweep and
the inputs the builders reject."""

import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2407_17678_amd", "csrc")

DRIVER = r"""
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>
#include "layout.h"
#include "config.h"

static int fails = 0;
#define CHECK(c) do { if (!(c)) { std::printf("FAILED %s line %d\n", #c, __LINE__); ++fails; } } while (0)

static void exercise(const s2_layout_params& p) {
  s2_layout L;
  const int st = s2::build_host(p, L);
  CHECK(st == S2_OK);
  if (st != S2_OK) return;
  const int H = p.num_heads, B = p.num_blocks;
  CHECK((int)L.row_ptr.size() == H * B + 1 && (int)L.col_ptr.size() == H * B + 1);
  CHECK(L.row_ptr.back() == L.nnz && L.col_ptr.back() == L.nnz);
  // the closed-form row enumeration agrees with the stored rows
  std::vector<int32_t> row(B + 1);
  for (int h = 0; h < H; ++h)
    for (int i = 0; i < B; i += (B > 64 ? 37 : 1)) {
      const int64_t n = s2::row_blocks(p, h, i, row.data(), (int64_t)row.size());
      const int32_t lo = L.row_ptr[(size_t)h * B + i], hi = L.row_ptr[(size_t)h * B + i + 1];
      CHECK(n == hi - lo);
      for (int64_t k = 0; k < n && k < hi - lo; ++k) CHECK(row[k] == L.col_idx[lo + k]);
    }
  // merged tile lists of the three passes
  const int S = p.block_size;
  s2::TileList t;
  s2::build_tiles(L, s2::kFwdBM / S > 0 ? s2::kFwdBM / S : 1, false, t);
  CHECK((int)t.ptr.size() == H * t.tiles_per_head + 1 && t.ptr.back() == (int32_t)t.ent.size());
  s2::build_tiles(L, s2::kBwdBN / S > 0 ? s2::kBwdBN / S : 1, true, t);
  CHECK((int)t.members.size() == H * t.tiles_per_head * t.group);
  // the unit table of the backward that keeps dS (64- and 128-token blocks)
  if (S >= 64) {
    s2::build_tiles(L, s2::kBwdBM / S, false, L.q_tiles);
    s2::build_tiles(L, s2::kBwdBN / S, true, L.kv_tiles);
    s2::build_ds_units(L);
    const size_t cpb = (size_t)S / 64;
    CHECK(L.ds_units == (int64_t)(L.kv_tiles.ent.size() * cpb * 2));
    CHECK(L.dq_units.size() == L.q_tiles.ent.size() * cpb * 2);
    int64_t named = 0;
    for (int32_t u : L.dq_units) {
      CHECK(u >= -1 && u < L.ds_units);
      named += u >= 0;
    }
    CHECK(named >= L.nnz);  // every kept block has at least one piece with a causal pair
  }
  // the same pattern handed back as caller-supplied rows
  s2_layout L2;
  CHECK(s2::build_from_csr(H, B, S, L.row_ptr.data(), L.col_idx.data(), L2) == S2_OK);
  CHECK(L2.nnz == L.nnz && L2.col_ptr == L.col_ptr && L2.row_idx == L.row_idx);
}

int main() {
  const int wl[4][6] = {{4, 8, 64, 2, 4, 0}, {16, 128, 64, 4, 8, 0}, {32, 512, 64, 16, 16, 0}, {32, 1024, 128, 8, 32, 0}};
  for (auto& w : wl) {
    s2_layout_params p{};
    p.num_heads = w[0]; p.num_blocks = w[1]; p.block_size = w[2]; p.local_blocks = w[3]; p.stride = w[4]; p.window_blocks = w[5];
    exercise(p);
  }
  std::mt19937 rng(7);
  const int sizes[4] = {16, 32, 64, 128};
  for (int n = 0; n < 150; ++n) {
    s2_layout_params p{};
    p.num_heads = 1 + rng() % 9;
    p.head_index_base = rng() % 5;
    p.block_size = sizes[rng() % 4];
    p.num_blocks = 1 + rng() % 70;
    if (p.block_size == 16) p.num_blocks += p.num_blocks & 1;   // 16-token blocks come in pairs
    p.local_blocks = 1 + rng() % 9;
    p.stride = rng() % 12;
    p.window_blocks = (rng() % 3 == 0) ? 1 + rng() % 40 : 0;
    p.dense = (rng() % 10 == 0);
    exercise(p);
  }
  // rejected inputs: a status, never a crash or an out-of-bounds access
  {
    s2_layout L;
    s2_layout_params p{};
    p.num_heads = 2; p.num_blocks = 8; p.block_size = 64; p.local_blocks = 0; p.stride = 4;
    CHECK(s2::build_host(p, L) != S2_OK);
    p.local_blocks = 2; p.block_size = 48;
    CHECK(s2::build_host(p, L) != S2_OK);
    p.block_size = 64; p.stride = -1;
    CHECK(s2::build_host(p, L) != S2_OK);
    p.stride = 4; p.num_heads = 0;
    CHECK(s2::build_host(p, L) != S2_OK);
    const int32_t rp_bad[3] = {0, 2, 1};           // not ascending
    const int32_t ci[2] = {0, 0};
    CHECK(s2::build_from_csr(1, 2, 64, rp_bad, ci, L) != S2_OK);
    const int32_t rp[3] = {0, 1, 2};
    const int32_t above[2] = {0, 5};               // column beyond the diagonal / the layout
    CHECK(s2::build_from_csr(1, 2, 64, rp, above, L) != S2_OK);
    const int32_t nodiag[2] = {0, 0};              // second row lacks its diagonal block
    CHECK(s2::build_from_csr(1, 2, 64, rp, nodiag, L) != S2_OK);
  }
  std::printf(fails ? "sanitizer driver: %d check(s) failed\n" : "sanitizer driver: ok\n", fails);
  return fails ? 1 : 0;
}
"""


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_layout_builder_under_asan_and_ubsan(tmp_path):
    drv = tmp_path / "driver.cpp"
    drv.write_text(DRIVER)
    exe = tmp_path / "driver"
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-I", CSRC, str(drv), os.path.join(CSRC, "layout.cpp"), "-o", str(exe)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0")
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, (r.stdout[-2000:], r.stderr[-3000:])
    assert "sanitizer driver: ok" in r.stdout
