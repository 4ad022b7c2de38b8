// Software-pipelined scan kernel instantiations for fp8 (e4m3) keys with bf16 queries.
#include "kb_configs.hpp"
#include "kb_scan_sp.hpp"

namespace kbi {

hipError_t launch_scan_sp_fp8(int config, bool sample, int grid, const ScanArgs &a, hipStream_t s)
{
    switch (config) {
#define XS(ID, KT, TQ, NSA, NSB) \
    case ID: return launch_scan_sp_cfg<SPCfg<KT, TQ, NSA, NSB>>(sample, grid, a, s);
        KB_SCAN_SP_CONFIGS_FP8(XS)
#undef XS
#define XQ(ID, KT, TQ, NSA, NSB) \
    case ID: return launch_scan_sp_cfg<SPCfg<KT, TQ, NSA, NSB, true, true>>(sample, grid, a, s);
        KB_SCAN_SP_CONFIGS_FP8_Q8(XQ)
#undef XQ
    default: return hipErrorInvalidValue;
    }
}

}  // namespace kbi
