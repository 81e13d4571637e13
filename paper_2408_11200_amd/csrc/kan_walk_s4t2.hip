// backward_walk_kernel with 4 streams per wave and 2 outputs per lane (see kan_walk.hip).
#include "kan_walk_kernel.hpp"

namespace kan {

void walk_launch_s4t2(bool dx, unsigned blocks, hipStream_t st, const SplineGeom &g, const WalkRecords &rec,
                      const float *gy, const float *cf, const float *w_b, float *part_c, float *part_b, float *gx,
                      int64_t B, const WalkPlan &p, int bpc, int m, int prezeroed, float *carry, int chunk0,
                      int n_chunks)
{
    walk_launch<4, 2>(dx, blocks, st, g, rec, gy, cf, w_b, part_c, part_b, gx, B, p, bpc, m, prezeroed, carry, chunk0,
                      n_chunks);
}

}  // namespace kan
