#include <stdio.h>
#include "bagel_internal.h"

int bagel_prepare_impl(bagel_ctx *c, const float *, const float *, const float *, const float *, const float *,
                       const float *, const float *, const float *, const float *, float *)
{
    BAGEL_FAIL(c, BAGEL_EHIP, "bagel_prepare_samples: not implemented yet");
}
