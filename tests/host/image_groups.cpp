// Host check of the work-group dealing of the input transform (image_on_one_xcd with the
// parameters with_image_groups sets, csrc/wino_kernels.hpp).  Launch slot b runs on XCD b % 8.
// For a sweep of layer shapes, in row and fragment order:
//   * the map from launch slots to work groups is one-to-one onto 0 .. groups - 1 (no tile is
//     transformed twice or left out);
//   * inside the dealt range, all work groups of one image have launch slots on one XCD;
//   * outside it (and when the dealing is off) the order is the plain one.
// Prints "ok <shapes> <dealt shapes>" and exits 0, or the first failure and exits 1.
#include <cstdint>
#include <cstdio>
#include <vector>

#include "wino_kernels.hpp"

int main() {
  long shapes = 0, dealt = 0;
  const int ms[3] = {2, 4, 6};
  const int Ns[9] = {1, 7, 8, 9, 15, 16, 33, 64, 250};
  const int HWs[7][2] = {{4, 4}, {8, 8}, {7, 9}, {16, 16}, {14, 14}, {32, 32}, {5, 23}};
  const int Cs[7] = {16, 64, 80, 128, 256, 272, 512};
  for (int frag = 0; frag < 2; ++frag)
    for (int m : ms)
      for (int N : Ns)
        for (const auto& hw : HWs)
          for (int C : Cs) {
            wino::Geometry g0{};
            g0.N = N, g0.H = hw[0], g0.W = hw[1], g0.C = C, g0.K = 64, g0.m = m;
            g0.TH = (hw[0] + m - 1) / m, g0.TW = (hw[1] + m - 1) / m;
            g0.T = N * g0.TH * g0.TW, g0.frag = frag;
            const bool whole = !frag && wino::whole_tiles(C, hw[0], hw[1]);
            const wino::Geometry g = wino::with_image_groups(g0, whole);
            const unsigned nb = wino::input_blocks(g);
            ++shapes;
            if (g.img_blocks) ++dealt;
            if (g.img_blocks && ((unsigned)g.img_blocks_end > nb || g.img_blocks_end % (8 * g.img_blocks))) {
              std::printf("frag %d m %d N %d %dx%d C %d: dealt range %d of %u groups, %d per image\n",
                          frag, m, N, hw[0], hw[1], C, g.img_blocks_end, nb, g.img_blocks);
              return 1;
            }
            std::vector<int> slot_of(nb, -1);
            for (unsigned b = 0; b < nb; ++b) {
              const unsigned grp = wino::image_on_one_xcd(g, b);
              if (grp >= nb || slot_of[grp] >= 0) {
                std::printf("frag %d m %d N %d %dx%d C %d: slot %u -> group %u (of %u) %s\n", frag, m,
                            N, hw[0], hw[1], C, b, grp, nb, grp >= nb ? "out of range" : "taken twice");
                return 1;
              }
              slot_of[grp] = (int)b;
              if ((!g.img_blocks || b >= (unsigned)g.img_blocks_end) && grp != b) {
                std::printf("frag %d m %d N %d %dx%d C %d: slot %u outside the dealt range moved to %u\n",
                            frag, m, N, hw[0], hw[1], C, b, grp);
                return 1;
              }
            }
            if (g.img_blocks)
              for (unsigned grp = 0; grp < (unsigned)g.img_blocks_end; ++grp) {
                const unsigned first = grp / g.img_blocks * g.img_blocks;   // first group of the image
                if ((slot_of[grp] & 7) != (slot_of[first] & 7)) {
                  std::printf("frag %d m %d N %d %dx%d C %d: groups %u and %u of one image on XCDs %d and %d\n",
                              frag, m, N, hw[0], hw[1], C, first, grp, slot_of[first] & 7, slot_of[grp] & 7);
                  return 1;
                }
              }
          }
  std::printf("ok %ld %ld\n", shapes, dealt);
  return 0;
}
