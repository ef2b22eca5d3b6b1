// bf16 matrix-core (MFMA) kernels: placeholder until the fast paths land.
#include "dev.h"
#include "kernels.h"

namespace ssdt {
namespace k {

size_t gemm_scratch_bytes(int, int, int, bool, bool, int) { return 0; }
hipError_t gemm_mfma_bf16(const Gemm &, hipStream_t) { return hipErrorNotSupported; }
hipError_t attn_fwd_mfma_bf16(const Attn &, hipStream_t) { return hipErrorNotSupported; }
hipError_t attn_bwd_mfma_bf16(const Attn &, hipStream_t) { return hipErrorNotSupported; }

}  // namespace k
}  // namespace ssdt
