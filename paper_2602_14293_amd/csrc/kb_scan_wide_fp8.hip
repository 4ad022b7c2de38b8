// Full-line scan kernel instantiations for fp8 keys with fp8 queries.
#include "kb_configs.hpp"
#include "kb_scan_wide.hpp"

namespace kbi {

hipError_t launch_scan_wide_fp8(int config, bool sample, int grid, const ScanArgs &a, hipStream_t s)
{
    switch (config) {
#define XW(ID, KT, TQ) \
    case ID: return launch_scan_wide_cfg<WideCfg<KT, TQ, true>>(sample, grid, a, s);
        KB_SCAN_WIDE_CONFIGS_FP8_Q8(XW)
#undef XW
    default: return hipErrorInvalidValue;
    }
}

}  // namespace kbi
