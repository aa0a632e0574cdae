// placeholder until the MFMA GEMM kernels land
#include "sbn_internal.hpp"
namespace sbn {
sbn_status launch_gemm_smfmac(const LinearItem &, hipStream_t) { return SBN_EUNSUPPORTED; }
sbn_status launch_gemm_dense(const LinearItem &, int8_t *, hipStream_t) { return SBN_EUNSUPPORTED; }
}
