// Instantiations of the specialised kernels (kvc_fast.h), one group of page shapes per compilation:
// the build compiles this file once for every KVC_FAST_GROUP in 0 .. kFastGroups - 1, so that the groups
// compile side by side.  A group is one channel count D with its page lengths NP (passes of 512
// elements; tokens = NP * 512 / D):
//   N = 16 (the paper's block of 16 tokens): every D from 32 to 256; N = 8: D = 64, 128, 192, 256;
//   N = 32: D = 32, 64, 96, 128.
#include "kvc_fast.h"

#ifndef KVC_FAST_GROUP
#error "compile with -DKVC_FAST_GROUP=<0..7>"
#endif

namespace kvc {

#if KVC_FAST_GROUP == 0
#define KVC_GROUP_SHAPES(X) X(32, 1) X(32, 2)
#elif KVC_FAST_GROUP == 1
#define KVC_GROUP_SHAPES(X) X(64, 1) X(64, 2) X(64, 4)
#elif KVC_FAST_GROUP == 2
#define KVC_GROUP_SHAPES(X) X(96, 3) X(96, 6)
#elif KVC_FAST_GROUP == 3
#define KVC_GROUP_SHAPES(X) X(128, 2) X(128, 4) X(128, 8)
#elif KVC_FAST_GROUP == 4
#define KVC_GROUP_SHAPES(X) X(160, 5)
#elif KVC_FAST_GROUP == 5
#define KVC_GROUP_SHAPES(X) X(192, 3) X(192, 6)
#elif KVC_FAST_GROUP == 6
#define KVC_GROUP_SHAPES(X) X(224, 7)
#elif KVC_FAST_GROUP == 7
#define KVC_GROUP_SHAPES(X) X(256, 4) X(256, 8)
#else
#error "KVC_FAST_GROUP out of range"
#endif

#define KVC_TABLE_ENTRY(D, NP) &FastOps<D, NP>::kTable,
static const FastKernels* const kGroupTable[] = {KVC_GROUP_SHAPES(KVC_TABLE_ENTRY)};

#define KVC_CAT2(a, b) a##b
#define KVC_CAT(a, b) KVC_CAT2(a, b)
const FastKernels* KVC_CAT(fast_kernels_group, KVC_FAST_GROUP)(int N, int d) {
    for (const FastKernels* k : kGroupTable)
        if (k->N == N && k->d == d) return k;
    return nullptr;
}

}  // namespace kvc
