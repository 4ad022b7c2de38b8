// Ping-pong scan kernel instantiations for bf16 keys.
#include "kb_configs.hpp"
#include "kb_scan_pp.hpp"

namespace kbi {

hipError_t launch_scan_pp_bf16(int config, bool sample, int grid, const ScanArgs &a, hipStream_t s)
{
    switch (config) {
#define XP(ID, KT, TQ, NSA, NSB) \
    case ID: return launch_scan_pp_cfg<PPCfg<KT, TQ, NSA, NSB>>(sample, grid, a, s);
        KB_SCAN_PP_CONFIGS_BF16(XP)
#undef XP
    default: return hipErrorInvalidValue;
    }
}

}  // namespace kbi
