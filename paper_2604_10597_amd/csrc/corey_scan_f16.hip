// selective_scan_fwd kernels instantiated for f16 storage (_Float16).
#include "corey_scan_impl.h"

namespace corey_scan {
void launch_scan_f16(const ScanArgs& a, const LaunchPlan& p) { launch_scan<_Float16>(a, p); }
}  // namespace corey_scan
