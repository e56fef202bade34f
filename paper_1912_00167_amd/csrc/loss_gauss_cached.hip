// Specialised loss kernels for diagonal-Gaussian policies on cached log pi_worker(a), log pi_target(a).
#include "policy_gauss.h"

namespace impact {

template <int MODE>
static bool launch_mode(int dtype, bool slot_major, LossArgs &a, hipStream_t s)
{
    switch (a.A) {
    case 3: launch_loss_static<GaussPolicy<3, 1, MODE>>(dtype, slot_major, a, s); return true;
    case 6: launch_loss_static<GaussPolicy<6, 1, MODE>>(dtype, slot_major, a, s); return true;
    case 17: launch_loss_static<GaussPolicy<17, 2, MODE>>(dtype, slot_major, a, s); return true;
    default: return false;
    }
}

bool launch_loss_gauss_cached(int dtype, bool slot_major, LossArgs &a, hipStream_t s)
{
    return a.target ? launch_mode<POLICY_CACHED_TARGET>(dtype, slot_major, a, s)
                    : launch_mode<POLICY_CACHED>(dtype, slot_major, a, s);
}

}  // namespace impact
