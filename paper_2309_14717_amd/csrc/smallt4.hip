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

// Repack for deployment: thread = (column, chunk) writes its record units.
__global__ __launch_bounds__(256) void deploy_kernel(const uint32_t* __restrict__ plane0,
                                                     const float* __restrict__ alpha,
                                                     const float* __restrict__ beta, int d_in, int d_out,
                                                     int group, uint32_t* __restrict__ out) {
  const int C = d_in / 128, sub = group / 32, units = s4_dep_units(sub);
  const int cols64 = ceil_div(d_out, 64) * 64;
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (size_t)cols64 * C) return;
  const int j = (int)(idx % cols64), c = (int)(idx / cols64);
  const int lane = j & 63, cg = j >> 6;
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  u32x4* rec = reinterpret_cast<u32x4*>(out) + ((size_t)c * (cols64 / 64) + cg) * (size_t)(units * 64) + lane;
  const bool ok = j < d_out;
  for (int u = 0; u < 4; ++u) {
    u32x4 v = {0, 0, 0, 0};
    if (ok)
      for (int q = 0; q < 4; ++q) v[q] = plane0[(size_t)(16 * c + 4 * u + q) * d_out + j];
    rec[u * 64] = v;
  }
  const int ng = 4 / sub;  // groups per chunk
  auto fa = [&](int g) { return ok ? __float_as_uint(alpha[(size_t)(ng * c + g) * d_out + j]) : 0u; };
  auto fb = [&](int g) { return ok ? __float_as_uint(beta[(size_t)(ng * c + g) * d_out + j]) : 0u; };
  if (sub == 1) {
    rec[4 * 64] = u32x4{fa(0), fa(1), fa(2), fa(3)};
    rec[5 * 64] = u32x4{fb(0), fb(1), fb(2), fb(3)};
  } else if (sub == 2) {
    rec[4 * 64] = u32x4{fa(0), fa(1), fb(0), fb(1)};
  } else {
    rec[4 * 64] = u32x4{fa(0), fb(0), 0u, 0u};
  }
}

hipError_t launch_deploy(const uint32_t* plane0, const float* alpha, const float* beta, int d_in, int d_out,
                         int group, void* stream_out, hipStream_t st) {
  const size_t n = (size_t)ceil_div(d_out, 64) * 64 * (d_in / 128);
  deploy_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(plane0, alpha, beta, d_in, d_out, group,
                                                            static_cast<uint32_t*>(stream_out));
  return hipGetLastError();
}

hipError_t launch_smallt4_deployed(const SmallTArgs& args, hipStream_t st) {
  SmallTArgs a = args;
  if (a.T < 1 || a.T > 4 || a.bits != 4 || a.d_in % 128 != 0 || !a.stream) return hipErrorInvalidValue;
  a.nonce = smallt_next_nonce();
  const SmallTPlan pl = smallt4_plan(a.d_in, a.d_out, a.T);
  ProfileHook hook = g_profile_hook[0];
  g_profile_hook[0] = ProfileHook{nullptr, nullptr, nullptr};
  if (hook.start) (void)hipEventRecord(hook.start, st);
  hipError_t e = hipErrorInvalidValue;
  const int sub = a.group / 32;
  if (sub == 1) e = launch_dep4<1>(a, pl, st);
  else if (sub == 2) e = launch_dep4<2>(a, pl, st);
  else if (sub == 4) e = launch_dep4<4>(a, pl, st);
  if (hook.stop) (void)hipEventRecord(hook.stop, st);
  return e;
}

// `args.nonce` is set by the caller (launch_smallt), which also owns the measurement hook.
hipError_t launch_smallt4(const SmallTArgs& a, hipStream_t st) {
  return a.fac16 ? launch_smallt4_f16(a, st) : launch_smallt4_impl<false>(a, st);
}

}  // namespace qalora
