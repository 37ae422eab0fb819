// The one-column-per-lane streaming kernel with fp32 factors, its launch plan and its entry
// point (the variant for 16-bit factors is compiled in a file of its own).
#include "smallt4_impl.hpp"

namespace qalora {

// Launch shape: slabs x parts with parts chosen to fill the compute units (at least one chunk
// per part); of the slab widths, the one that occupies most compute units (ties: the narrower
// slab, which has fewer partials to add).  A partial holds at most ST_PARTIAL_FLOATS values, so
// more than eight tokens rule out the 1024-column slab.
SmallTPlan smallt4_plan(int d_in, int d_out, int tokens) {
  const int chunks = d_in / 128;
  const int tg = tokens <= 4 ? 1 : (tokens <= 8 ? 2 : 4);
  SmallTPlan best{};
  for (int halves = 4; halves >= 1; halves /= 2) {
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
    if (halves == 4 || busy > best_busy) best = pl;
  }
  return best;
}

// `args.nonce` is set by the caller (launch_smallt), which also owns the measurement hook.
hipError_t launch_smallt4(const SmallTArgs& a, hipStream_t st) {
  return a.fac16 ? launch_smallt4_f16(a, st) : launch_smallt4_impl<false>(a, st);
}

}  // namespace qalora
