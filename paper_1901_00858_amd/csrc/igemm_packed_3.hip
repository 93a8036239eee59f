// Implicit-GEMM instantiations that read weights pre-packed by hgc_conv2d_pack_weights: part 3 of the table.
#define HGC_IGEMM_PACKED 1
#define HGC_IGEMM_PART 3
#define HGC_IGEMM_ACCESSOR igemm_variants_packed_3
#include "igemm_kernel.h"
