// Host-only driver for the sanitizer build of the attention planner (tests/test_attention_plan.py compiles
// the planner's source files with AddressSanitizer and UndefinedBehaviorSanitizer on the host side and links
// this file against them): a few thousand random batches through hs_tree_attention_plan, which reads the
// host arrays, validates them and plans the launch exactly as the real call does, without touching a GPU.
#include <cstdio>
#include <cstdlib>
#include <vector>
#include "heterospec.h"
int main() {
  unsigned long long x = 88172645463325252ull;
  auto rnd = [&]() { x ^= x << 13; x ^= x >> 7; x ^= x << 17; return (unsigned)(x >> 11); };
  long checked = 0;
  for (int it = 0; it < 3000; ++it) {
    const int B = 1 + rnd() % (it % 50 == 0 ? 130 : 20);
    static const int heads[][2] = {{32, 8}, {8, 8}, {64, 8}, {4, 1}, {12, 6}, {3, 3}};
    const int* h = heads[rnd() % 6];
    const int D = rnd() % 3 ? 128 : 64;
    std::vector<int32_t> no(B + 1, 0);
    std::vector<int64_t> po(B + 1, 0), lens(B);
    for (int s = 0; s < B; ++s) {
      static const int ms[] = {0, 1, 9, 61, 64, 129, 257, 1024};
      static const int ls[] = {0, 1, 63, 64, 500, 2048, 4100, 16384, 70000};
      no[s + 1] = no[s] + ms[rnd() % 8];
      const int64_t L = ls[rnd() % 9];
      po[s + 1] = po[s] + L;
      lens[s] = L ? rnd() % (L + 1) : 0;
    }
    int64_t totals[6];
    std::vector<int32_t> per(4 * B);
    const int mode = rnd() % 3;  // dense, spare capacity, paged
    hs_status st = hs_tree_attention_plan(no.data(), po.data(), mode ? lens.data() : nullptr, mode == 2, mode == 2 ? 1100 : 0, B,
                                          h[0], h[1], D, rnd() % 4 ? HS_BF16 : HS_F32, totals, per.data());
    if (st != HS_OK) { std::printf("status %d: %s\n", (int)st, hs_last_error()); return 1; }
    checked += totals[1];
  }
  std::printf("ok %ld\n", checked);
  return 0;
}
