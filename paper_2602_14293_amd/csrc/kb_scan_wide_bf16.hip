// Full-line scan kernel instantiations for bf16 keys.
#include "kb_configs.hpp"
#include "kb_scan_wide.hpp"

namespace kbi {

hipError_t launch_scan_wide_bf16(int config, bool sample, int grid, const ScanArgs &a, hipStream_t s)
{
    switch (config) {
#define XW(ID, KT, TQ) \
    case ID: return launch_scan_wide_cfg<WideCfg<KT, TQ>>(sample, grid, a, s);
        KB_SCAN_WIDE_CONFIGS_BF16(XW)
#undef XW
    default: return hipErrorInvalidValue;
    }
}

}  // namespace kbi
