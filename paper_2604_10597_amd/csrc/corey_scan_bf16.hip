// selective_scan_fwd kernels instantiated for bf16 storage (uint16_t).
#include "corey_scan_impl.h"

namespace corey_scan {
void launch_scan_bf16(const ScanArgs& a, const LaunchPlan& p) { launch_scan<uint16_t>(a, p); }
}  // namespace corey_scan
