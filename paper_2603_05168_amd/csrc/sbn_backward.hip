// placeholder until the backward kernels land
#include "sbn_internal.hpp"
namespace sbn {
size_t backward_workspace_bytes(int64_t, int64_t, int64_t) { return 256; }
sbn_status launch_backward(const void *, int64_t, int64_t, int64_t, const Pattern &, const void *, const float *,
                           const int8_t *, const float *, void *, void *, int, void *, size_t, hipStream_t)
{
    return SBN_EUNSUPPORTED;
}
}
