// IEEE binary16 instance of the 16-bit forward path: the dwm_f16_* calls (see half_impl.inc).
#define DWM16_BF16 0
#define DWM16_ELEM dwm_half_t
#include "half_impl.inc"
