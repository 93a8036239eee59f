// Implicit-GEMM instantiations that read weights in the caller's [M][C/G][k][k] layout.
#define HGC_IGEMM_PACKED 0
#define HGC_IGEMM_ACCESSOR igemm_variants_raw
#include "igemm_kernel.h"
