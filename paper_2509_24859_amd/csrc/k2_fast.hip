// placeholder until the 32-bit kernel lands: routes to the generic kernel
#include "harp_internal.h"
namespace harp {
size_t plan_fast_ws_per_group(int L, int S_max) { return plan_generic_ws_per_group(L, S_max); }
int plan_fast_groups(int L, int n_cu) { (void)L; return n_cu * 8; }
void launch_plan_fast(const TablesDev &tb, const CandDev &cd, const PlansDev &out, void *ws,
                      int n_groups, hipStream_t st) { launch_plan_generic(tb, cd, out, ws, n_groups, st); }
}
