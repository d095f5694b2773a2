// MFMA attention over the latent cache (placeholder until the kernel lands).
#include "kvcar_internal.hpp"
namespace kvcar {
bool attend_mfma_available() { return false; }
hipError_t launch_attend_mfma(const AttendParams&, int, hipStream_t) { return hipErrorNotSupported; }
}
