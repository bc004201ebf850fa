#include "internal.hpp"
namespace csd {
hipError_t launch_gemm_bf16(const GemmArgs&, hipStream_t) { return hipErrorNotSupported; }
}
