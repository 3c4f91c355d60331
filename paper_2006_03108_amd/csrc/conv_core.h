// The partitioned convolution layer with the halo exchange switchable, shared by the public calls and by the
// channel-partitioned layer.
#pragma once
#include <cstddef>

#include "common.h"

namespace distdl {

int conv_fwd_core(distdl_plan* plan, void* const x_bufs_dev[], const void* w_dev, const void* bias_dev,
                  void* const y_dev[], hipStream_t st, bool halo);
int conv_bwd_core(distdl_plan* plan, const void* const x_bufs_dev[], const void* w_dev, const void* const dy_dev[],
                  void* const dx_bufs_dev[], void* dw_dev, void* dbias_dev, void* workspace_dev, size_t workspace_bytes,
                  hipStream_t st, bool halo);
int run_halo(distdl_plan* p, bool adjoint, PtrTable& tab, void* const* bufs_host, hipStream_t st);

}  // namespace distdl
