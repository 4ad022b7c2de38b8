// Software-pipelined scan kernel instantiations for bf16 keys.
#include "kb_configs.hpp"
#include "kb_scan_sp.hpp"

namespace kbi {

hipError_t launch_scan_sp_bf16(int config, bool sample, int grid, const ScanArgs &a, hipStream_t s)
{
    switch (config) {
#define XI(ID, KT, TQ, NSA, NSB) \
    case ID: return launch_scan_sp_cfg<SPCfg<KT, TQ, NSA, NSB, false, true>>(sample, grid, a, s);
        KB_SCAN_SP_CONFIGS_BF16_IL(XI)
#undef XI
    default: return hipErrorInvalidValue;
    }
}

}  // namespace kbi
