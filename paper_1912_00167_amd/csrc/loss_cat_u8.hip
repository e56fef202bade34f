// Specialised loss kernels for categorical policies whose batches store the action index as one byte
// (a storage variant of the buffer): the full action set of 18, on both distributions or on cached
// log-probabilities.  Other action-set sizes with one-byte indices run on the shape-generic kernel.
#include "policy_cat.h"

namespace impact {

bool launch_loss_cat_u8(int dtype, bool slot_major, LossArgs &a, hipStream_t s)
{
    if (a.A != 18) return false;
    if (!a.logp) launch_loss_static<CatPolicy<18, 2, POLICY_FULL, uint8_t>>(dtype, slot_major, a, s);
    else if (a.target) launch_loss_static<CatPolicy<18, 2, POLICY_CACHED_TARGET, uint8_t>>(dtype, slot_major, a, s);
    else launch_loss_static<CatPolicy<18, 2, POLICY_CACHED, uint8_t>>(dtype, slot_major, a, s);
    return true;
}

}  // namespace impact
