#include "common.h"
int32_t pa_decode_splits(const powattn_pattern* pat, int64_t capacity) { (void)pat; (void)capacity; return 1; }
int pa_launch_decode_bf16(const pa_decode_args& a) { (void)a; return POWATTN_UNSUPPORTED; }
