// Instantiates the scan kernel for one (element type, draft layout) pair, one word per (index, draft).
#include "scan.hpp"

namespace llc {
hipError_t launch_scan_f32_perk(int kt, bool probs, bool finish, unsigned grid, hipStream_t s, const ScanParams &p) {
  return launch_scan<F32In, false, false>(kt, probs, finish, grid, s, p);
}
}  // namespace llc
