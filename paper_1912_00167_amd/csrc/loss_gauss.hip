// Specialised loss kernels for diagonal-Gaussian policies: both distributions read from the batch.
#include "policy_gauss.h"

namespace impact {

// Action dimensions of the MuJoCo tasks the paper trains on (Hopper 3, HalfCheetah 6, Humanoid 17).
bool launch_loss_gauss_static(int dtype, bool slot_major, LossArgs &a, hipStream_t s)
{
    switch (a.A) {
    case 3: launch_loss_static<GaussPolicy<3, 1>>(dtype, slot_major, a, s); return true;
    case 6: launch_loss_static<GaussPolicy<6, 1>>(dtype, slot_major, a, s); return true;
    case 17: launch_loss_static<GaussPolicy<17, 2>>(dtype, slot_major, a, s); return true;
    default: return false;
    }
}

}  // namespace impact
