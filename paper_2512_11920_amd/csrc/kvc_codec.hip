// Instantiations of the codec kernels (kvc_codec.h), one group of page shapes per compilation: the build
// compiles this file once for every KVC_SHAPE_GROUP in 0 .. kShapeGroups - 1, so that the groups compile side
// by side.  Group 2 i + h holds channel count D = 32 (i + 1) with page lengths NP = 4 h + 1 .. 4 h + 4
// (passes of 512 elements): for every NP the shape with a short last pass (any token count N with
// 512 (NP - 1) < N D < 512 NP), and, where 512 NP is a multiple of D, the exact shape N = 512 NP / D.  Exact
// shapes are built for N = 16 (the paper's block of 16 tokens) at every D, for N = 8 at D = 64, 128, 192, 256
// and for N = 32 at D = 32, 64, 96, 128; other whole-pass pages run as "partial" pages with a full last pass.
#include "kvc_codec.h"

#ifndef KVC_SHAPE_GROUP
#error "compile with -DKVC_SHAPE_GROUP=<0..15>"
#endif

namespace kvc {

#define KVC_D (32 * (KVC_SHAPE_GROUP / 2 + 1))
#define KVC_NP0 (4 * (KVC_SHAPE_GROUP % 2))

// exact shapes of this group's D and half
#if KVC_SHAPE_GROUP == 0
#define KVC_EXACT(X) X(32, 1) X(32, 2)
#elif KVC_SHAPE_GROUP == 2
#define KVC_EXACT(X) X(64, 1) X(64, 2) X(64, 4)
#elif KVC_SHAPE_GROUP == 4
#define KVC_EXACT(X) X(96, 3)
#elif KVC_SHAPE_GROUP == 5
#define KVC_EXACT(X) X(96, 6)
#elif KVC_SHAPE_GROUP == 6
#define KVC_EXACT(X) X(128, 2) X(128, 4)
#elif KVC_SHAPE_GROUP == 7
#define KVC_EXACT(X) X(128, 8)
#elif KVC_SHAPE_GROUP == 9
#define KVC_EXACT(X) X(160, 5)
#elif KVC_SHAPE_GROUP == 10
#define KVC_EXACT(X) X(192, 3)
#elif KVC_SHAPE_GROUP == 11
#define KVC_EXACT(X) X(192, 6)
#elif KVC_SHAPE_GROUP == 13
#define KVC_EXACT(X) X(224, 7)
#elif KVC_SHAPE_GROUP == 14
#define KVC_EXACT(X) X(256, 4)
#elif KVC_SHAPE_GROUP == 15
#define KVC_EXACT(X) X(256, 8)
#elif KVC_SHAPE_GROUP >= 0 && KVC_SHAPE_GROUP < 16
#define KVC_EXACT(X)
#else
#error "KVC_SHAPE_GROUP out of range"
#endif

#define KVC_EXACT_ENTRY(D, NP) &ShapeOps<D, NP, false>::kTable,
static const ShapeKernels* const kGroupTable[] = {
    KVC_EXACT(KVC_EXACT_ENTRY)
    &ShapeOps<KVC_D, KVC_NP0 + 1, true>::kTable, &ShapeOps<KVC_D, KVC_NP0 + 2, true>::kTable,
    &ShapeOps<KVC_D, KVC_NP0 + 3, true>::kTable, &ShapeOps<KVC_D, KVC_NP0 + 4, true>::kTable};

#define KVC_CAT2(a, b) a##b
#define KVC_CAT(a, b) KVC_CAT2(a, b)
const ShapeKernels* KVC_CAT(shape_kernels_group, KVC_SHAPE_GROUP)(int d, int np, bool partial) {
    for (const ShapeKernels* k : kGroupTable)
        if (k->d == d && k->np == np && k->partial == partial) return k;
    return nullptr;
}

}  // namespace kvc
