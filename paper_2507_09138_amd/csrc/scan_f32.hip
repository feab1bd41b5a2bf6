// List-scan kernel instantiations for HR_F32 storage (all supported dimensions).
#include "scan_kernel.h"

namespace hr {
hipError_t launch_scan_f32(int d, const ScanArgs& a, int shape, int grid, size_t lds, hipStream_t s)
{
    return launch_scan_dtype<HR_F32>(d, a, shape, grid, lds, s);
}
hipError_t launch_scan_f16x2(int d, const ScanArgs& a, int shape, int grid, size_t lds, hipStream_t s)
{
    return launch_scan_dtype<HR_F16X2>(d, a, shape, grid, lds, s);
}
hipError_t launch_seed_f32(int d, const SeedArgs& a, hipStream_t s) { return launch_seed_dtype<HR_F32>(d, a, s); }
}  // namespace hr
