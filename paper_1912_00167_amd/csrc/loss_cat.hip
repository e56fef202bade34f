// Specialised loss kernels for categorical policies: both distributions read from the batch.
#include "policy_cat.h"

namespace impact {

// Action-set sizes of the Atari games the paper trains on (minimal action sets: 4, 6, 9, 18).
bool launch_loss_cat_static(int dtype, bool slot_major, LossArgs &a, hipStream_t s)
{
    if (a.act_bytes == 1) return launch_loss_cat_u8(dtype, slot_major, a, s);
    switch (a.A) {
    case 4: launch_loss_static<CatPolicy<4, 1>>(dtype, slot_major, a, s); return true;
    case 6: launch_loss_static<CatPolicy<6, 1>>(dtype, slot_major, a, s); return true;
    case 9: launch_loss_static<CatPolicy<9, 1>>(dtype, slot_major, a, s); return true;
    case 18: launch_loss_static<CatPolicy<18, 2>>(dtype, slot_major, a, s); return true;
    default: return false;
    }
}

}  // namespace impact
