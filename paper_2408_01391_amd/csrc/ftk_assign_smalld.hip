// Small-D assignment kernel (fp32, D <= 32): placeholder dispatch hooks.
#include "ftk_internal.h"

namespace ftk {

bool smalld_supported(ftk_dtype, int, int) { return false; }

void plan_smalld(int64_t, int, int, ftk_ft_mode, AssignPlan &) {}

ftk_status launch_assign_smalld(const AssignCall &, const AssignPlan &, const Workspace &, hipStream_t)
{
    set_error("small-D variant not built");
    return FTK_EINVAL;
}

}  // namespace ftk
