// Decode kernels for bf16 models with head_dim 64 (see ls_kernels.inc).
#include <stdint.h>
typedef uint16_t bf16_t;
#define LS_VARIANT_T bf16_t
#define LS_VARIANT_HD 64
#define LS_VARIANT_NAME bf16_hd64
#include "ls_kernels.inc"
