// placeholder until the table-tile kernels land
#include "ax_internal.h"
namespace ax {
bool tab_supported(const Geom&) { return false; }
TabPlan tab_plan(const Geom&, const Options&) { TabPlan p{}; p.total = 256; return p; }
hipError_t launch_tab(const Geom&, const QParams&, const TabPlan&, const uint8_t*, const uint8_t*, const uint16_t*,
                      int32_t*, float*, void*, hipStream_t) { return hipErrorNotSupported; }
}
