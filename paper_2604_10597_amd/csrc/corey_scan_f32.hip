// selective_scan_fwd kernels instantiated for f32 storage (float).
#include "corey_scan_impl.h"

namespace corey_scan {
void launch_scan_f32(const ScanArgs& a, const LaunchPlan& p) { launch_scan<float>(a, p); }
}  // namespace corey_scan
