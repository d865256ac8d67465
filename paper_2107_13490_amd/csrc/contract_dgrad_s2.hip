// Kernel instances of the stride-2 data gradient that visits its rows in parity-class order (see ContractArgs::dg_classes);
// a translation unit of its own keeps the build parallel
#include "contract_kernel.hpp"

namespace adapt {

hipError_t launch_planned_dgrad_s2(adapt_ctx *ctx, const ContractPlan &p)
{
    if (p.empty) return hipSuccess;
    return p.limbs == 1 ? launch_modes<OP_DGRAD_S2, 1>(ctx, p.kern, p.splits, p.tile) : launch_modes<OP_DGRAD_S2, 2>(ctx, p.kern, p.splits, p.tile);
}

}  // namespace adapt
