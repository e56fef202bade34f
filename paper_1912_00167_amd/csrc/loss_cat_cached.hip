// Specialised loss kernels for categorical policies on cached log pi_worker(a), log pi_target(a).
#include "policy_cat.h"

namespace impact {

template <int MODE>
static bool launch_mode(int dtype, bool slot_major, LossArgs &a, hipStream_t s)
{
    switch (a.A) {
    case 4: launch_loss_static<CatPolicy<4, 1, MODE>>(dtype, slot_major, a, s); return true;
    case 6: launch_loss_static<CatPolicy<6, 1, MODE>>(dtype, slot_major, a, s); return true;
    case 9: launch_loss_static<CatPolicy<9, 1, MODE>>(dtype, slot_major, a, s); return true;
    case 18: launch_loss_static<CatPolicy<18, 2, MODE>>(dtype, slot_major, a, s); return true;
    default: return false;
    }
}

bool launch_loss_cat_cached(int dtype, bool slot_major, LossArgs &a, hipStream_t s)
{
    if (a.act_bytes == 1) return launch_loss_cat_u8(dtype, slot_major, a, s);
    return a.target ? launch_mode<POLICY_CACHED_TARGET>(dtype, slot_major, a, s)
                    : launch_mode<POLICY_CACHED>(dtype, slot_major, a, s);
}

}  // namespace impact
