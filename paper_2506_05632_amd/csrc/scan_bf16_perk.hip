// Instantiates the scan kernel for one (element type, draft layout) pair.
#include "scan.hpp"

namespace llc {
hipError_t launch_scan_bf16_perk(int kt, bool probs, unsigned grid, hipStream_t s, const ScanParams &p) {
  return launch_scan<BF16In, false>(kt, probs, grid, s, p);
}
}  // namespace llc
