// Geometry of one call, derived on the host from the descriptor.  Plain C++ (no HIP), so that
// host-only builds of the set-up logic can include it.
#pragma once

namespace cs {

struct Geo {
  int N, Np, NB;                    // batch, padded batch, Np/32
  int C, H, W, K, R, S, P, Q;
  int sh, sw, ph, pw;
  int k0, Ks;
  int HW, PQ, RS, CRS;
};

}  // namespace cs
