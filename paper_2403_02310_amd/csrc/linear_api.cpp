// C ABI of the linear layer (declared and documented in include/sarathi.h): argument checks, the
// split-K decision, the launch.  Stateless: no handle, nothing allocated.
#include <hip/hip_runtime_api.h>

#include <cstdint>

#include "internal.h"
#include "sarathi.h"

using namespace sarathi;

namespace {

bool shape_ok(int32_t T, int32_t N, int32_t K) {
    if (T < 0 || N <= 0 || K <= 0) return false;
    if (N % 128 != 0 || K % 64 != 0 || K > (1 << 20)) return false;
    return (int64_t)T * N < ((int64_t)1 << 40);
}

}  // namespace

extern "C" size_t sarathi_linear_workspace_bytes(int32_t num_tokens, int32_t out_features, int32_t in_features) {
    if (!shape_ok(num_tokens, out_features, in_features) || num_tokens == 0) return 0;
    const LinearPlan pl = plan_linear(num_tokens, out_features, in_features, SIZE_MAX);
    return pl.splits > 1 ? sizeof(float) * (size_t)pl.splits * (size_t)num_tokens * (size_t)out_features : 0;
}

extern "C" sarathi_status sarathi_linear(const void *x, const void *w, void *y, int32_t num_tokens,
                                         int32_t out_features, int32_t in_features, void *workspace,
                                         size_t workspace_bytes, void *stream) {
    if (!shape_ok(num_tokens, out_features, in_features)) return SARATHI_ESHAPE;
    if (num_tokens == 0) return SARATHI_OK;
    if (!x || !w || !y) return SARATHI_EINVAL;
    const LinearPlan pl = plan_linear(num_tokens, out_features, in_features, workspace ? workspace_bytes : 0);
    const hipError_t e = (hipError_t)launch_linear(pl, x, w, y, num_tokens, out_features, in_features, workspace, stream);
    return e == hipSuccess ? SARATHI_OK : SARATHI_EHIP;
}
