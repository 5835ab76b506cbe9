// Aggregation kernels for fp32 tables (16-, 8- and 4-byte vectors per lane).
#include "aggregate_kernels.h"

namespace mgg {

hipError_t launch_aggregate_f32(const AggArgs &a, bool gcn, int vec, dim3 grid, int wpb, hipStream_t stream, int lpr, int ch, bool lds)
{
    if (vec == 4) return dispatch_shape<false, 4>(a, gcn, grid, wpb, stream, lpr, ch, lds);
    if (vec == 2) return dispatch_shape<false, 2>(a, gcn, grid, wpb, stream, lpr, ch, lds);
    return dispatch_shape<false, 1>(a, gcn, grid, wpb, stream, lpr, ch, lds);
}

}  // namespace mgg
