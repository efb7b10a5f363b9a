// Compact engine (placeholder until the kernel lands): reports that no state fits.
#include "p2_device.h"
namespace p2 {
size_t compact_lds_bytes(int, int) { return 0; }
hipError_t launch_eval_compact(const DevQuery*, int, int, unsigned long long, unsigned long long, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_cost_compact(const DevQuery*, int, int, const unsigned long long*, uint32_t, p2_program*, double*, hipStream_t) { return hipErrorNotSupported; }
}
