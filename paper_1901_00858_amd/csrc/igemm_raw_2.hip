// Implicit-GEMM instantiations that read weights in the caller's [M][C/G][k][k] layout: part 2 of the table.
#define HGC_IGEMM_PACKED 0
#define HGC_IGEMM_PART 2
#define HGC_IGEMM_ACCESSOR igemm_variants_raw_2
#include "igemm_kernel.h"
