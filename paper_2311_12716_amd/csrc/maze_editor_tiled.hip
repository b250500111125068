// Tiled store-layout kernel of the teacher editor env (placeholder: no shape is
// covered yet, the per-cell kernel runs).
#include "maze_internal.h"

int editor_tiled_launch(const editor_ctx *, const int32_t *, int, int8_t *, int32_t *, uint8_t *,
                        hipStream_t)
{
    return 0;
}
