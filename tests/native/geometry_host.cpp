// Host-only checks of the launch geometry the library derives from a tensor's scale group: which class of kernel
// steps it, how many rows a workgroup of the wide-group kernel takes, and what one helper launch can hold.
#include <cstdio>
#include <cstdlib>

#include "eco_internal.hpp"

#define CHECK(c)                                                   \
  do {                                                             \
    if (!(c)) { std::printf("FAILED line %d: %s\n", __LINE__, #c); return 1; } \
  } while (0)

int main() {
  using namespace eco;
  // classes
  CHECK(classify_group(128, 1 << 20) == GROUP_BLOCK && classify_group(32, 100) == GROUP_BLOCK && classify_group(512, 7) == GROUP_BLOCK);
  CHECK(classify_group(1024, 1 << 20) == GROUP_WIDE && classify_group(8192, 1 << 20) == GROUP_WIDE && classify_group(24, 1 << 20) == GROUP_WIDE);
  CHECK(classify_group(1000, 1 << 20) == GROUP_WIDE && classify_group(1 << 20, 4096) == GROUP_WIDE);       // one scale, small tensor
  CHECK(classify_group(1 << 20, 1 << 20) == GROUP_TENSOR && classify_group(8200, 8200) == GROUP_TENSOR && classify_group(1 << 30, 100) == GROUP_TENSOR);
  CHECK(classify_group(8200, 1 << 20) == GROUP_UNSUPPORTED && classify_group(20, 1 << 20) == GROUP_UNSUPPORTED && classify_group(16, 1 << 20) == GROUP_WIDE);

  // rows to a workgroup: known cases
  struct { uint64_t rows_in_tensor, g; uint32_t rows, waves; } known[] = {
      {2304, 576, 8, 9}, {576, 2304, 2, 9}, {2048, 1408, 4, 11}, {64, 640, 4, 5}, {6, 768, 2, 3}, {8, 1152, 4, 9},
      {5, 1408, 1, 3},          // not a whole number of bundles
      {4, 1024, 1, 2}, {4, 2048, 1, 4}, {3, 8192, 1, 16}, {16, 1000, 1, 2}, {8, 520, 1, 2}, {2, 6912, 1, 14}, {64, 96, 1, 1},
      {2, 7936, 1, 16},         // two rows would need 31 waves
  };
  for (const auto &k : known) {
    const WideGeometry w = wide_geometry(k.rows_in_tensor * k.g, k.g);
    if (w.rows != k.rows || w.waves != k.waves || w.units != k.rows_in_tensor / k.rows) {
      std::printf("FAILED: %llu rows of %llu: got %u rows, %u waves, %llu units\n", (unsigned long long)k.rows_in_tensor,
                  (unsigned long long)k.g, w.rows, w.waves, (unsigned long long)w.units);
      return 1;
    }
  }
  // a ragged last row never bundles
  CHECK(wide_geometry(8 * 1408 + 8, 1408).rows == 1 && wide_geometry(8 * 1408 + 8, 1408).units == 9);
  // every group length and a few row counts: what the kernel relies on
  for (uint64_t g = 8; g <= MAX_WIDE_GROUP; g += 8) {
    for (uint64_t n : {1ull, 2ull, 3ull, 4ull, 7ull, 8ull, 16ull, 24ull, 1000ull}) {
      const WideGeometry w = wide_geometry(n * g, g);
      CHECK(w.waves >= 1 && w.waves <= (uint32_t)MAX_WIDE_WAVES && w.rows >= 1 && w.rows <= 8);
      CHECK(w.units * w.rows == n);
      if (w.rows == 1) {
        CHECK(w.waves == (g + TILE_ELEMS - 1) / TILE_ELEMS);
      } else {
        CHECK(g > (uint64_t)TILE_ELEMS && (uint64_t)w.rows * g == (uint64_t)w.waves * TILE_ELEMS);   // every lane busy, whole rows
        CHECK(2 * g > (uint64_t)TILE_ELEMS);                                                          // a wave meets at most two rows
      }
    }
  }
  // what one helper launch holds
  CHECK(flat_call_fits((1ull << 35) - 512, 128) && !flat_call_fits(1ull << 35, 128) && !flat_call_fits((1ull << 40) + 1, 128));
  CHECK(flat_call_fits(1ull << 34, 520) && !flat_call_fits(1ull << 35, 520) && flat_call_fits(1ull << 30, 1ull << 31));
  std::printf("geometry ok\n");
  return 0;
}
