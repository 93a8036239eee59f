// Implicit-GEMM instantiations that read weights in the caller's [M][C/G][k][k] layout: part 1 of the table.
#define HGC_IGEMM_PACKED 0
#define HGC_IGEMM_PART 1
#define HGC_IGEMM_ACCESSOR igemm_variants_raw_1
#include "igemm_kernel.h"
