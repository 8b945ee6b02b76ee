// Decode kernels for float models with head_dim 128 (see ls_kernels.inc).
#include <stdint.h>
typedef uint16_t bf16_t;
#define LS_VARIANT_T float
#define LS_VARIANT_HD 128
#define LS_VARIANT_NAME f32_hd128
#include "ls_kernels.inc"
