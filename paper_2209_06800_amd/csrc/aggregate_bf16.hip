// Aggregation kernels for bf16 tables (16-, 4- and 2-byte vectors per lane), fp32 accumulation.
#include "aggregate_kernels.h"

namespace mgg {

hipError_t launch_aggregate_bf16(const AggArgs &a, bool gcn, int vec, dim3 grid, int wpb, hipStream_t stream, int lpr, int ch, bool lds)
{
    if (vec == 8) return dispatch_shape<true, 8>(a, gcn, grid, wpb, stream, lpr, ch, lds);
    if (vec == 2) return dispatch_shape<true, 2>(a, gcn, grid, wpb, stream, lpr, ch, lds);
    return dispatch_shape<true, 1>(a, gcn, grid, wpb, stream, lpr, ch, lds);
}

}  // namespace mgg
