// Specialised convolution kernels (none yet: every shape takes the general kernel).
#include "q8t_common.h"
#include "q8t_internal.h"

bool q8t_fast_conv_supported(int, const q8t_conv_desc *, const void *, const void *, const void *, const void *)
{
    return false;
}
size_t q8t_fast_conv_ws(int, const q8t_conv_desc *) { return 0; }
int q8t_fast_conv(int, const q8t_conv_desc *, const void *, const q8t_qparams *, const void *, const q8t_qparams *,
                  float *, void *, void *, hipStream_t)
{
    return Q8T_ERR_SHAPE;
}
