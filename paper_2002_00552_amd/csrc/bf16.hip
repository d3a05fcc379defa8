// bfloat16 instance of the 16-bit forward path: the dwm_bf16_* calls (see half_impl.inc).
#define DWM16_BF16 1
#define DWM16_ELEM dwm_bf16_t
#include "half_impl.inc"
