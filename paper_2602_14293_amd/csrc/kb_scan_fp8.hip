// Scan kernel instantiations for fp8 keys.
#include "kb_configs.hpp"
#include "kb_scan.hpp"

namespace kbi {

hipError_t launch_scan_fp8(int config, bool sample, int grid, const ScanArgs &a, hipStream_t s)
{
    switch (config) {
#define X(ID, KT, TK, TQ, WM, WN, RBA, NSTAGE, WGPC) \
    case ID: return launch_scan_cfg<ScanCfg<KT, TK, TQ, WM, WN, RBA, NSTAGE, WGPC>>(sample, grid, a, s);
        KB_SCAN_CONFIGS_FP8(X)
        KB_SCAN_CONFIGS_FP8_Q8(X)
#undef X
    default: return hipErrorInvalidValue;
    }
}

}  // namespace kbi
