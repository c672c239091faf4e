// Instantiates the scan kernel for one (element type, draft layout) pair, race times drawn min-first.
#include "scan.hpp"

namespace llc {
hipError_t launch_scan_bf16_perk_minf(int kt, bool probs, bool finish, unsigned grid, hipStream_t s, const ScanParams &p) {
  return launch_scan<BF16In, false, true>(kt, probs, finish, grid, s, p);
}
}  // namespace llc
