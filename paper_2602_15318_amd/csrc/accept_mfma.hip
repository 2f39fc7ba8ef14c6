#include "accept.hpp"
namespace sparrow {
bool lm_head_mfma_supported(int, int, int, int) { return false; }
int accept_num_candidates(int, int, int, int) { return 0; }
hipError_t launch_lm_head_mfma(const AcceptArgs &, hipStream_t) { return hipErrorNotSupported; }
}
