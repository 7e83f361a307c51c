// Direct-to-LDS kernels with paired sub-steps (DlTile::PAIR): the variant tables.
#include "xp_mfma_dl.hpp"

namespace xp {
namespace {

#define XP_DL_PAIR_VARIANT(NAME, TYPESTR, INT8, BM, BN, WM, WN, PAIR, PAIRSTR, EFF)                                       \
    typedef DlTile<BM, BN, WM, WN, 2, 128, false, 1, 16, false, 3, PAIR> NAME##_tile;                                     \
    bool NAME##_can(const Problem &q) { return !q.conv && dl_can_run_common<INT8>(q, BM, BN, 128, 16); }                  \
    hipError_t NAME##_launch(const Problem &q) { return dl_pair_launch<INT8, NAME##_tile>(q); }                           \
    double NAME##_cost(const Problem &q) { return dl_cost<NAME##_tile>(q, EFF); }                                         \
    const Variant NAME = {TYPESTR " " #BM "x" #BN "x128B waves " #WM "x" #WN " ring 3(A)+2(B) direct-to-lds, reads as assembly, sub-steps paired" PAIRSTR ", mfma16", \
                          NAME##_can, NAME##_launch, NAME##_cost};

#define XP_DL_PAIR_OUTER_VARIANT(NAME, MODE, WHAT, EFF)                                                                    \
    typedef DlTile<256, 256, 2, 2, 2, 128, false, 1, 16, false, 3, 1> NAME##_tile;                                        \
    bool NAME##_can(const Problem &q) { return dl_outer_can_run(q, 256, 256, MODE == 4 || MODE == 5, MODE == 3 || MODE == 5); } \
    hipError_t NAME##_launch(const Problem &q) { return dl_outer_launch<NAME##_tile, MODE>(q); }                          \
    double NAME##_cost(const Problem &q) { return dl_cost<NAME##_tile>(q, EFF); }                                         \
    const Variant NAME = {"bf16 256x256x128B waves 2x2 ring 3(A)+2(B) direct-to-lds, " WHAT " by transposing reads, sub-steps paired, mfma16", \
                          NAME##_can, NAME##_launch, NAME##_cost};

XP_DL_PAIR_OUTER_VARIANT(kBfPairBnm, 3, "B along N", 0.54)
XP_DL_PAIR_OUTER_VARIANT(kBfPairAmm, 4, "A along M", 0.52)
XP_DL_PAIR_OUTER_VARIANT(kBfPairAmmBnm, 5, "A along M and B along N", 0.52)
XP_DL_PAIR_VARIANT(kBfPair256x256, "bf16", false, 256, 256, 2, 4, 1, "", 0.56)
XP_DL_PAIR_VARIANT(kI8Pair256x256, "i8", true, 256, 256, 2, 4, 1, "", 0.56)
XP_DL_PAIR_VARIANT(kI8PairW4, "i8", true, 256, 256, 2, 2, 1, "", 0.58)
// the two tile heights of the convolution (and of tall GEMMs) with paired sub-steps: 7 and 6 block rows per wave
typedef DlTile<224, 256, 2, 2, 2, 128, false, 1, 16, false, 3, 1> TwoHiP;
typedef DlTile<192, 256, 2, 2, 2, 128, false, 1, 16, false, 3, 1> TwoLoP;
// (a planar output is left to the eight-wave kernels: its column-by-column stores want more waves to issue them;
// the stage 32x56x56x256 -> 256 from NCHW tensors: 847 against 906 TFLOP/s)
bool kBfPairTwoHeights_can(const Problem &q) { return !q.c_plane && dl_can_run_common<false>(q, 224, 256, 128, 16); }
hipError_t kBfPairTwoHeights_launch(const Problem &q) { return dl_launch_two_heights<false, TwoHiP, TwoLoP, true>(q); }
double kBfPairTwoHeights_cost(const Problem &q) { return dl_cost<TwoHiP>(q, 0.51); }
const Variant kBfPairTwoHeights = {"bf16 224x256x128B then 192x256 in the last round, waves 2x2 ring 3(A)+2(B) direct-to-lds, reads as assembly, sub-steps paired, mfma16",
                                   kBfPairTwoHeights_can, kBfPairTwoHeights_launch, kBfPairTwoHeights_cost};
XP_DL_PAIR_VARIANT(kBfPairW4, "bf16", false, 256, 256, 2, 2, 1, "", 0.58)
}  // namespace

// Registered after the small ones.
int dl_pair_variants(xp_dtype in_type, const Variant **out)
{
    if (in_type == XP_BF16) { out[0] = &kBfPair256x256; out[1] = &kBfPairW4; out[2] = &kBfPairBnm; out[3] = &kBfPairAmm; out[4] = &kBfPairAmmBnm; out[5] = &kBfPairTwoHeights; return 6; }
    if (in_type == XP_I8) { out[0] = &kI8Pair256x256; out[1] = &kI8PairW4; return 2; }
    return 0;
}

}  // namespace xp
