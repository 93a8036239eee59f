// The implicit-GEMM instantiation tables, joined from the parts that are compiled separately
// (igemm_packed_<part>.hip, igemm_raw_<part>.hip).  The order of the parts fixes the variant numbers
// that plans, forced launch shapes and measured launch shapes refer to.
#include <vector>

#include "hgc_internal.h"

namespace hgc {

typedef const IgemmVariant *(*PartFn)(int *);

const IgemmVariant *igemm_variants_packed_0(int *);
const IgemmVariant *igemm_variants_packed_1(int *);
const IgemmVariant *igemm_variants_packed_2(int *);
const IgemmVariant *igemm_variants_packed_3(int *);
const IgemmVariant *igemm_variants_raw_0(int *);
const IgemmVariant *igemm_variants_raw_1(int *);
const IgemmVariant *igemm_variants_raw_2(int *);
const IgemmVariant *igemm_variants_raw_3(int *);

static std::vector<IgemmVariant> join(std::initializer_list<PartFn> parts)
{
    std::vector<IgemmVariant> all;
    for (PartFn f : parts) {
        int n = 0;
        const IgemmVariant *v = f(&n);
        all.insert(all.end(), v, v + n);
    }
    return all;
}

const IgemmVariant *igemm_variants_packed(int *count)
{
    static const std::vector<IgemmVariant> all =
        join({igemm_variants_packed_0, igemm_variants_packed_1, igemm_variants_packed_2, igemm_variants_packed_3});
    *count = (int)all.size();
    return all.data();
}

const IgemmVariant *igemm_variants_raw(int *count)
{
    static const std::vector<IgemmVariant> all =
        join({igemm_variants_raw_0, igemm_variants_raw_1, igemm_variants_raw_2, igemm_variants_raw_3});
    *count = (int)all.size();
    return all.data();
}

}  // namespace hgc
