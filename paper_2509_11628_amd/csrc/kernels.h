// Host-callable launchers of the gfx950 kernels.  Every launcher validates what the kernel
// and its grid assume and enqueues on the given stream without synchronising.
#pragma once

#include "common.h"

namespace speca {

// ---- cache (HBM-bound) -----------------------------------------------------------------
// out[slot][i][E] = sum_o rt.w[i][o] * D^o[slot][rt.row[i]]      (Eq. 2)
Error launch_forecast(const CacheGeom& g, const RowTable& rt, void* out, hipStream_t st);
// D0 <- feat[slot][i]; D^o <- (D^{o-1}_new - D^{o-1}_old) * rt.w[i][o-1], o <= rt.order[i]   (Eq. 3 recursion)
Error launch_refresh(const CacheGeom& g, const RowTable& rt, const void* feat, hipStream_t st);
// Read D^0 .. D^{order-1} of (slot, rt.row[i]) and drop the values: a cache hint ahead of a fused refresh.
// The old differences were written a whole step ago and are cold; read from inside the GEMM epilogue
// they cost four dependent HBM round trips with the matrix cores idle (measured 21 us per launch for
// 19 MB), read here they stream at full rate and the epilogue then finds them in the memory-side cache.
Error launch_cache_warm(const CacheGeom& g, const RowTable& rt, int slot, hipStream_t st);
// Eq. 4 (or another metric) per row.  g == nullptr: pred is a tensor [n_rows][E];
// otherwise the prediction is formed from slot `slot` of the cache with rt's weights.
// partial: device scratch of n_rows * verify_chunks(E) * 3 floats.
int verify_chunks(int64_t E);
constexpr int kMaxVerifyRows = 1024;   // rows of one launch when prediction and truth are both tensors
Error launch_verify(int metric, const void* pred, int pred_dtype, const void* truth, int truth_dtype, int64_t E,
                    const CacheGeom* g, const RowTable* rt, int slot, int n_rows, float eps, const float* tau_dev,
                    float* partial, float* err_dev, uint8_t* accept_dev, hipStream_t st);

}  // namespace speca
