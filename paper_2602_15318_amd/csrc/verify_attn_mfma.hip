#include "verify_attn.hpp"
namespace sparrow {
bool verify_partial_mfma_supported(int, int) { return false; }
hipError_t launch_verify_partial_mfma(const VerifyArgs &, const SeqTable &, hipStream_t) { return hipErrorNotSupported; }
}
