// Register-tile scan kernel instantiations for bf16 keys.
#include "kb_configs.hpp"
#include "kb_scan_big.hpp"

namespace kbi {

hipError_t launch_scan_big_bf16(int config, bool sample, int grid, const ScanArgs &a, hipStream_t s)
{
    switch (config) {
#define XB(ID, KT, NSA, NSB) \
    case ID: return launch_scan_big_cfg<BigCfg<KT, NSA, NSB>>(sample, grid, a, s);
        KB_SCAN_BIG_CONFIGS_BF16(XB)
#undef XB
    default: return hipErrorInvalidValue;
    }
}

}  // namespace kbi
