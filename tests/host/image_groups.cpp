// Host check of the work-group dealing of the transforms (image_on_one_xcd with the parameters
// that with_image_groups / with_output_groups set, csrc/wino_kernels.hpp).  Launch slot b runs
// on XCD b % 8.  For a sweep of layer shapes, in row and fragment order:
//   * the map from launch slots to work groups is one-to-one onto 0 .. groups - 1 (no tile is
//     transformed twice or left out), for the input and for the output transform;
//   * inside the dealt range, all work groups of one unit (an image, a run of tiles) have launch
//     slots on one XCD; outside it (and when the dealing is off) the order is the plain one;
//   * fragment order: the unit is 32 tiles, and tile block j of the contraction + output kernel
//     (XCD j % 8) holds the tiles whose input work groups ran on that XCD;
//   * rows, where xcd_chunk_tiles says the stage kernels are aligned: input transform,
//     contraction (8 tile groups, group j on XCD j) and output transform give every tile to
//     the same XCD.
// Prints "ok <shapes> <dealt shapes> <aligned shapes>" and exits 0, or the first failure and exits 1.
#include <cstdint>
#include <cstdio>
#include <vector>

#include "wino_kernels.hpp"

int main() {
  long shapes = 0, dealt = 0, aligned = 0;
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
            // which XCD transforms tile t (first channel group)?
            const long gpt_in = frag ? 0 : C / 256;
            auto input_xcd = [&](long t) -> int {
              const long grp = frag ? (t / 4) * ((C + 63) / 64) : t * gpt_in;
              return slot_of[grp] & 7;
            };
            if (frag && g.img_blocks) {
              for (long t = 0; t < (long)g.img_blocks_end / g.img_blocks * 32; ++t)
                if (input_xcd(t) != (int)((t / 32) % 8)) {
                  std::printf("frag m %d N %d %dx%d C %d: tile %ld transformed on XCD %d, contracted on %ld\n",
                              m, N, hw[0], hw[1], C, t, input_xcd(t), (t / 32) % 8);
                  return 1;
                }
            }
            for (int K : {256, 512}) {
              wino::Geometry gk = g0;
              gk.K = K;
              const long chunk = wino::xcd_chunk_tiles(gk);
              const wino::Geometry go = wino::with_output_groups(gk);
              const unsigned nbo = wino::blocks_for((long)gk.T * K);
              std::vector<int> oslot(nbo, -1);
              for (unsigned b = 0; b < nbo; ++b) {
                const unsigned grp = wino::image_on_one_xcd(go, b);
                if (grp >= nbo || oslot[grp] >= 0) {
                  std::printf("output m %d N %d %dx%d K %d: slot %u -> group %u (of %u)\n", m, N, hw[0],
                              hw[1], K, b, grp, nbo);
                  return 1;
                }
                oslot[grp] = (int)b;
              }
              if ((chunk > 0) != (go.img_blocks > 0)) return 1;
              if (chunk == 0 || !whole || C != K) continue;
              ++aligned;
              const wino::Geometry gi = wino::with_image_groups(gk, true);
              const int tt = wino::contract_tile_rows(gk);
              if (wino::contract_tile_groups(gk, tt) != 8 || chunk % tt != 0 || chunk * 8 != gk.T) {
                std::printf("aligned m %d N %d %dx%d C %d: chunk %ld, block %d\n", m, N, hw[0], hw[1], C,
                            chunk, tt);
                return 1;
              }
              for (long t = 0; t < gk.T; ++t) {
                // inverse of the dealing for the tile's first work group of each transform
                int xi = -1, xo = -1;
                for (unsigned b = 0; b < wino::input_blocks(gi) && xi < 0; ++b)
                  if (wino::image_on_one_xcd(gi, b) == (unsigned)(t * (C / 256))) xi = (int)(b & 7);
                xo = oslot[t * (K / 256)] & 7;
                const int xc = (int)(t / chunk);     // contraction: tile group j on XCD j
                if (xi != xc || xo != xc) {
                  std::printf("aligned m %d N %d %dx%d C %d: tile %ld on XCDs %d / %d / %d\n", m, N, hw[0],
                              hw[1], C, t, xi, xc, xo);
                  return 1;
                }
              }
            }
          }
  std::printf("ok %ld %ld %ld\n", shapes, dealt, aligned);
  return 0;
}
