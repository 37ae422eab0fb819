// The one-column-per-lane streaming kernel with fp32 factors, its launch plan and its entry
// point (the variant for 16-bit factors is compiled in a file of its own).
#include "smallt4_impl.hpp"

namespace qalora {

// Launch shape: slabs x parts with parts chosen to fill the compute units (at least one chunk
// per part).  Of the slab widths, the one with the fewest parts to add among those that keep at
// least kEnoughBlocks compute units streaming -- HBM is saturated from about four fifths of the
// chip on, and every further part costs a hand-over (measured at 8192 x 22016, one token:
// 242 blocks x 11 parts 27.1 us, 215 x 5 26.2 us, 172 x 2 26.2 us; but the vector-bound 2- and
// 3-bit forms lose on 172) -- otherwise the one that occupies most compute units.  (A third
// width, 1024 columns with no split inside the block, never won once the hand-over had become
// cheap, and is no longer built.)
SmallTPlan smallt4_plan(int d_in, int d_out, int tokens) {
  constexpr int kEnoughBlocks = 200;
  const int chunks = d_in / 128;
  const int tg = tokens <= 4 ? 1 : (tokens <= 8 ? 2 : 4);
  SmallTPlan best{};
  bool have = false;
  for (int halves = 4; halves >= 2; halves /= 2) {
    SmallTPlan pl;
    pl.halves = halves;
    pl.slab_cols = (S4_WAVES / halves) * S4_WCOLS;
    if (pl.slab_cols * 4 * tg > ST_PARTIAL_FLOATS) continue;
    pl.slabs = ceil_div(d_out, pl.slab_cols);
    int m = ST_MAX_BLOCKS / pl.slabs;
    if (m > chunks) m = chunks;
    if (m < 1) m = 1;
    pl.parts = m;
    pl.blocks = pl.slabs * m;
    const int busy = pl.blocks < ST_MAX_BLOCKS ? pl.blocks : ST_MAX_BLOCKS;
    const int best_busy = best.blocks < ST_MAX_BLOCKS ? best.blocks : ST_MAX_BLOCKS;
    bool better;
    if (!have) better = true;
    else if (busy >= kEnoughBlocks && best_busy >= kEnoughBlocks)
      better = pl.parts < best.parts || (pl.parts == best.parts && busy > best_busy);
    else
      better = busy > best_busy;
    if (better) {
      best = pl;
      have = true;
    }
  }
  return best;
}

// `args.nonce` is set by the caller (launch_smallt), which also owns the measurement hook.
hipError_t launch_smallt4(const SmallTArgs& a, hipStream_t st) {
  return a.fac16 ? launch_smallt4_f16(a, st) : launch_smallt4_impl<false>(a, st);
}

}  // namespace qalora
