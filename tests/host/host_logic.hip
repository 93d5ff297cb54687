// Host-side checks of the launch arithmetic that the kernels rely on (no GPU is touched: the
// program is compiled by hipcc and runs on the CPU).  Prints "ok" and exits 0, or prints the
// first failures and exits 1.  Built and run by tests/test_host_logic.py.
#include <cstdint>
#include <cstdio>
#include <set>
#include <vector>

#include "dispatch_util.h"
#include "launch_util.h"
#include "vec_io.h"

static int failures = 0;
#define CHECK(cond, ...)                                   \
  do {                                                     \
    if (!(cond)) {                                         \
      if (failures < 20) {                                 \
        std::printf("FAIL %s:%d %s : ", __FILE__, __LINE__, #cond); \
        std::printf(__VA_ARGS__);                          \
        std::printf("\n");                                 \
      }                                                    \
      ++failures;                                          \
    }                                                      \
  } while (0)

// xcd_block_row: a permutation of every run of 64 workgroups that hands the workgroups of one
// XCD (equal index mod 8) eight consecutive rows, and keeps rows 64 apart in one class.
static void check_xcd_block_row() {
  for (unsigned base = 0; base < 4096; base += 64) {
    std::set<int64_t> seen;
    for (unsigned b = base; b < base + 64; ++b) {
      const int64_t r = rms::xcd_block_row(b);
      CHECK(r >= base && r < base + 64, "block %u row %lld", b, (long long)r);
      seen.insert(r);
      CHECK((r % 64) / 8 == b % 8, "block %u (XCD %u) got row %lld", b, b % 8, (long long)r);
      CHECK(rms::xcd_block_row(b + 64) == r + 64, "block %u", b);
    }
    CHECK(seen.size() == 64, "run at %u is not a permutation", base);
  }
}

// row_cut and the slot assignment of the element-addressed kernels: for every offset of a row
// from a line and a range of lengths, head + whole slots + tail make up the row, and with
// CHUNKS = ceil(floor(row bytes / 16) / G) the lanes' slots (lane t of chunk c holds slot
// c * G + t, the lanes of chunk 0 before `first` hold slot CHUNKS * G + t) cover [first, end)
// exactly once; the chunks between the first and the last hold whole slots only.
template <int EB>
static void check_row_cut() {
  alignas(128) static char buffer[256];
  const int lengths[] = {1, 2, 3, 7, 8, 9, 15, 16, 17, 63, 64, 65, 511, 512, 513, 1023, 1025, 1537, 2047, 2049,
                         4095, 4096, 4097, 8191, 8192, 8193, 12289, 16383, 20481, 57343};
  for (int off = 0; off < 128; off += EB) {
    for (int n : lengths) {
      const rms::RowCut c = rms::row_cut<EB>(buffer + off, n);
      CHECK(c.off == off, "off %d n %d", off, n);
      CHECK(c.first * 16 >= off && c.first * 16 - off < 16, "first: off %d n %d", off, n);
      CHECK(c.end >= c.first && (c.end == c.first || c.end * 16 <= off + n * EB), "end: off %d n %d", off, n);
      CHECK(c.head >= 0 && c.tail >= 0, "off %d n %d", off, n);
      CHECK(c.head * EB + 16 * (c.end - c.first) + c.tail * EB == n * EB, "pieces: off %d n %d: %d %d %d %d", off, n,
            c.head, c.first, c.end, c.tail);
      CHECK(c.head * EB < 16 || c.head == n, "head: off %d n %d", off, n);
      if (c.end > c.first) CHECK(c.tail * EB < 16, "tail: off %d n %d", off, n);
      CHECK(c.head <= 16 && c.tail <= 16, "edge threads: off %d n %d", off, n);   // threads 0.. and 16..
      const int pieces = n * EB / 16;
      for (int G : {64, 256, 512, 1024}) {
        const int chunks = pieces == 0 ? 1 : (pieces + G - 1) / G;
        std::vector<int> hits(chunks * G + G, 0);
        for (int ch = 0; ch < chunks; ++ch) {
          for (int t = 0; t < G; ++t) {
            const int slot = (ch == 0 && t < c.first) ? chunks * G + t : ch * G + t;
            const bool between = ch > 0 && ch < chunks - 1;
            if (between) CHECK(slot >= c.first && slot < c.end, "middle chunk: off %d n %d G %d slot %d", off, n, G, slot);
            if (between || slot < c.end) {
              CHECK(slot >= c.first && slot < c.end, "slot outside the row: off %d n %d G %d slot %d", off, n, G, slot);
              if (slot < (int)hits.size()) ++hits[slot];
            }
          }
        }
        for (int slot = c.first; slot < c.end; ++slot)
          CHECK(hits[slot] == 1, "off %d n %d G %d: slot %d held %d times", off, n, G, slot, hits[slot]);
      }
    }
  }
}

// with_chunks / with_shape: the callback gets the run-time numbers as constants, and only
// inside the bounds.
static void check_shapes() {
  for (int chunks = -1; chunks <= 10; ++chunks) {
    int got = 0;
    const bool ok = rms::host::with_chunks<2, 8>(chunks, [&](auto c) { got = decltype(c)::value; });
    CHECK(ok == (chunks >= 2 && chunks <= 8) && got == (ok ? chunks : 0), "with_chunks %d", chunks);
  }
  for (int threads : {8, 64, 100, 256, 512}) {
    for (int chunks = 0; chunks <= 9; ++chunks) {
      int g = 0, ch = 0;
      auto f = [&](auto gg, auto cc) { g = decltype(gg)::value; ch = decltype(cc)::value; };
      const bool ok = rms::host::with_shape<64, 4>(threads, chunks, f) || rms::host::with_shape<256, 8>(threads, chunks, f);
      const bool want = (threads == 64 && chunks >= 1 && chunks <= 4) || (threads == 256 && chunks >= 1 && chunks <= 8);
      CHECK(ok == want && (!ok || (g == threads && ch == chunks)), "with_shape %d %d", threads, chunks);
    }
  }
  CHECK(rms::host::whole_pieces(4097, 2) == 512 && rms::host::whole_pieces(8191, 2) == 1023 &&
            rms::host::whole_pieces(4097, 4) == 1024 && rms::host::whole_pieces(7, 2) == 0, "whole_pieces");
}

// with_packed_shape: L a power of two up to 64, (E - 1) * L < N <= E * L, E <= kPackElems; rows of
// a multiple of the bank period get at least 8 lanes.
static void check_packed_lanes() {
  for (int elem : {2, 4}) {
    for (int64_t N = 1; N <= 64 * rms::kPackElems; ++N) {
      int L = 0, E = 0, calls = 0;
      rms::host::with_packed_shape(N, elem, 64, [&](auto l, auto e) { L = decltype(l)::value; E = decltype(e)::value; ++calls; });
      CHECK(calls == 1, "N %lld elem %d: %d calls", (long long)N, elem, calls);
      CHECK(L >= 1 && L <= 64 && (L & (L - 1)) == 0 && E >= 1 && E <= rms::kPackElems, "N %lld: L %d E %d", (long long)N, L, E);
      CHECK((int64_t)(E - 1) * L < N && N <= (int64_t)E * L, "N %lld elem %d: L %d E %d", (long long)N, elem, L, E);
      if ((N * elem) % 64 == 0) CHECK(L >= 8, "N %lld elem %d: L %d on a multiple of 64 bytes", (long long)N, elem, L);
      else CHECK(L == 1 || (int64_t)(L / 2) * rms::kPackElems < N, "N %lld elem %d: L %d wider than needed", (long long)N, elem, L);
    }
  }
}

// packed_shape: tiles fit, are whole passes where more than one pass fits, the grid respects its
// cap, and the tiles are shared out in as few rounds as the cap allows.
static void check_packed_shape() {
  for (int64_t row_bytes : {2, 16, 154, 394, 514, 1002, 2044, 4096}) {
    for (int lanes : {1, 8, 16, 64}) {
      for (int64_t M : {1, 5, 37, 1000, 170320, 1 << 20}) {
        for (int64_t target : {rms::host::kPackedTargetReadWrite, rms::host::kPackedTargetReadOnly}) {
          for (int64_t cap : {64, 4096, 1 << 15}) {
            const rms::host::PackedShape s = rms::host::packed_shape(M, row_bytes, lanes, 256, 16384, target, cap);
            const int groups = 256 / lanes;
            CHECK(s.tile_rows >= 1 && s.tile_rows * row_bytes <= 16384, "tile: %lld %d %lld", (long long)row_bytes, lanes, (long long)M);
            if (16384 / row_bytes > groups && s.tile_rows < M)
              CHECK(s.tile_rows % groups == 0, "passes: %lld %d %lld: %d rows", (long long)row_bytes, lanes, (long long)M, s.tile_rows);
            const int64_t tiles = (M + s.tile_rows - 1) / s.tile_rows;
            CHECK(s.blocks >= 1 && s.blocks <= cap && s.blocks <= tiles, "grid: %lld blocks", (long long)s.blocks);
            CHECK((tiles + s.blocks - 1) / s.blocks == (tiles + cap - 1) / cap, "rounds: %lld tiles on %lld blocks, cap %lld",
                  (long long)tiles, (long long)s.blocks, (long long)cap);
          }
        }
      }
    }
  }
}

// Grids: flat grids are multiples of 64 that cover M (up to the cap); walking grids are multiples
// of the compute units (256 without a device, itself a multiple of 64) with at least two rows each.
static void check_grids() {
  for (int64_t M : {1, 63, 64, 65, 1000, 8192, 1 << 20, (1 << 20) + 77}) {
    const int64_t g = rms::host::flat_grid(M, 1 << 20);
    CHECK(g % 64 == 0 && g >= (M < (1 << 20) ? M : (1 << 20)) && g < M + 64 && g <= (1 << 20), "flat_grid %lld -> %lld", (long long)M, (long long)g);
  }
  // flat_rows: XCD blocks (and then a grid of a multiple of 64) for workgroups of 256 threads and
  // more on rows of 8 to 64 KiB only; everything else keeps one row per workgroup index.
  for (int threads : {64, 128, 256, 512, 1024}) {
    for (int64_t row_bytes : {16, 4096, 8176, 8192, 16384, 64000, 65536, 65552, 131072}) {
      for (int64_t M : {1, 63, 64, 65, 8192, (1 << 20) + 77}) {
        const rms::host::FlatRows r = rms::host::flat_rows(M, 1 << 20, threads, row_bytes);
        const bool want = threads >= 256 && row_bytes >= 8192 && row_bytes <= 65536;
        const int64_t capped = M < (1 << 20) ? M : (1 << 20);
        CHECK(r.xcd_blocks == (want ? 1 : 0), "flat_rows %d threads, %lld bytes", threads, (long long)row_bytes);
        CHECK(want ? (r.blocks % 64 == 0 && r.blocks >= capped && r.blocks < capped + 64) : r.blocks == capped,
              "flat_rows grid %lld for %lld rows", (long long)r.blocks, (long long)M);
      }
    }
  }
  for (int64_t row_bytes : {2050, 8194, 16382, 40962, 114686}) {
    for (int threads : {64, 256, 512, 1024}) {
      for (int64_t M : {1, 100, 511, 512, 1024, 1500, 3000, 8192, 16384, 100000}) {
        const int64_t g = rms::host::walk_grid(M, row_bytes, threads, 26 * 1024);
        CHECK(g >= 0 && g % 256 == 0, "walk_grid %lld", (long long)g);
        if (g > 0) CHECK(M >= 2 * g && g * threads <= 256 * 2048, "walk_grid: %lld rows on %lld workgroups of %d", (long long)M, (long long)g, threads);
      }
    }
  }
  CHECK(rms::host::walk_grid(16384, 16382, 256, 26 * 1024) == 512, "the 8191-element bf16 shape");
}

int main() {
  check_xcd_block_row();
  check_row_cut<2>();
  check_row_cut<4>();
  check_shapes();
  check_packed_lanes();
  check_packed_shape();
  check_grids();
  if (failures) {
    std::printf("%d checks failed\n", failures);
    return 1;
  }
  std::printf("ok\n");
  return 0;
}
