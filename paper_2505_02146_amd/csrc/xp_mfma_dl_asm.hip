// Direct-to-LDS kernels with assembly fragment reads (modes 3-8 of dl_body): the variant tables.
#include "xp_mfma_dl.hpp"

namespace xp {
namespace {

#define XP_DL_OUTER_VARIANT(NAME, MODE, WHAT, BM, BN, WM, WN, NSA, NSB, OCC, EFF)                                          \
    typedef DlTile<BM, BN, WM, WN, NSB, 128, false, OCC, 16, false, NSA> NAME##_tile;                                     \
    bool NAME##_can(const Problem &q) { return dl_outer_can_run(q, BM, BN, MODE == 4 || MODE == 5, MODE == 3 || MODE == 5); } \
    hipError_t NAME##_launch(const Problem &q) { return dl_outer_launch<NAME##_tile, MODE>(q); }                          \
    double NAME##_cost(const Problem &q) { return dl_cost<NAME##_tile>(q, EFF); }                                         \
    const Variant NAME = {"bf16 " #BM "x" #BN "x128B waves " #WM "x" #WN " ring " #NSA "(A)+" #NSB "(B) direct-to-lds, " WHAT " by transposing reads, mfma16", \
                          NAME##_can, NAME##_launch, NAME##_cost};

XP_DL_OUTER_VARIANT(kBfBnm256x256a3, 3, "B along N", 256, 256, 2, 4, 3, 2, 1, 0.50)
XP_DL_OUTER_VARIANT(kBfBnm256x256, 3, "B along N", 256, 256, 2, 4, 2, 2, 1, 0.48)
XP_DL_OUTER_VARIANT(kBfBnm256x256b3, 3, "B along N", 256, 256, 2, 4, 2, 3, 1, 0.50)
XP_DL_OUTER_VARIANT(kBfBnm128x128, 3, "B along N", 128, 128, 2, 2, 2, 2, 2, 0.32)
XP_DL_OUTER_VARIANT(kBfAmm256x256, 4, "A along M", 256, 256, 2, 4, 2, 2, 1, 0.48)
XP_DL_OUTER_VARIANT(kBfAmm128x128, 4, "A along M", 128, 128, 2, 2, 2, 2, 2, 0.32)
XP_DL_OUTER_VARIANT(kBfAmmBnm256x256, 5, "A along M and B along N", 256, 256, 2, 4, 2, 2, 1, 0.48)
XP_DL_OUTER_VARIANT(kBfAmmBnm128x128, 5, "A along M and B along N", 128, 128, 2, 2, 2, 2, 2, 0.32)
// small tiles with deep rings for batched problems that are bound by memory, not by the matrix cores: 48 KB of LDS
// (three workgroups a compute unit, each with two K steps of loads in flight) or 64 KB (two, with three)
XP_DL_OUTER_VARIANT(kBfBnm64x64n3, 3, "B along N", 64, 64, 2, 2, 3, 3, 3, 0.20)
XP_DL_OUTER_VARIANT(kBfBnm64x64n4, 3, "B along N", 64, 64, 2, 2, 4, 4, 2, 0.20)
XP_DL_OUTER_VARIANT(kBfBnm128x64n3, 3, "B along N", 128, 64, 4, 1, 3, 3, 2, 0.25)
// half-size tiles with three buffers per ring, for shapes that 256x256 tiles cut into too few pieces
XP_DL_OUTER_VARIANT(kBfBnm256x128, 3, "B along N", 256, 128, 4, 2, 3, 3, 1, 0.44)
XP_DL_OUTER_VARIANT(kBfBnm128x256, 3, "B along N", 128, 256, 2, 4, 3, 3, 1, 0.44)
XP_DL_OUTER_VARIANT(kBfAmm256x128, 4, "A along M", 256, 128, 4, 2, 3, 3, 1, 0.44)
XP_DL_OUTER_VARIANT(kBfAmm128x256, 4, "A along M", 128, 256, 2, 4, 3, 3, 1, 0.44)
XP_DL_OUTER_VARIANT(kBfAmmBnm256x128, 5, "A along M and B along N", 256, 128, 4, 2, 3, 3, 1, 0.44)
XP_DL_OUTER_VARIANT(kBfAmmBnm128x256, 5, "A along M and B along N", 128, 256, 2, 4, 3, 3, 1, 0.44)

#define XP_DL_ASM_VARIANT(NAME, TYPESTR, INT8, BM, BN, WM, WN, NSA, NSB, OCC, EFF)                                          \
    typedef DlTile<BM, BN, WM, WN, NSB, 128, false, OCC, 16, false, NSA> NAME##_tile;                                     \
    bool NAME##_can(const Problem &q) { return dl_can_run_common<INT8>(q, BM, BN, 128, 16); }                             \
    hipError_t NAME##_launch(const Problem &q) { return dl_asm_launch<INT8, NAME##_tile>(q); }                            \
    double NAME##_cost(const Problem &q) { return dl_cost<NAME##_tile>(q, EFF); }                                         \
    const Variant NAME = {TYPESTR " " #BM "x" #BN "x128B waves " #WM "x" #WN " ring " #NSA "(A)+" #NSB "(B) direct-to-lds, reads as assembly, mfma16", \
                          NAME##_can, NAME##_launch, NAME##_cost};

XP_DL_ASM_VARIANT(kBfAsm256x256a3, "bf16", false, 256, 256, 2, 4, 3, 2, 1, 0.55)
XP_DL_ASM_VARIANT(kBfAsm256x256, "bf16", false, 256, 256, 2, 4, 2, 2, 1, 0.54)
XP_DL_ASM_VARIANT(kBfAsm224x256a3, "bf16", false, 224, 256, 2, 4, 3, 2, 1, 0.50)
XP_DL_ASM_VARIANT(kBfAsm128x128, "bf16", false, 128, 128, 2, 2, 2, 2, 2, 0.36)
XP_DL_ASM_VARIANT(kBfAsm256x128, "bf16", false, 256, 128, 4, 2, 3, 3, 1, 0.46)
XP_DL_ASM_VARIANT(kBfAsm128x256, "bf16", false, 128, 256, 2, 4, 3, 3, 1, 0.46)
XP_DL_ASM_VARIANT(kBfAsm224x256, "bf16", false, 224, 256, 2, 4, 2, 2, 1, 0.50)
typedef DlTile<224, 256, 2, 4, 2, 128, false, 1, 16, false, 2> TwoHi2;
typedef DlTile<192, 256, 2, 4, 2, 128, false, 1, 16, false, 2> TwoLo2;
bool kBfAsmTwoHeights2_can(const Problem &q) { return dl_can_run_common<false>(q, 224, 256, 128, 16); }
hipError_t kBfAsmTwoHeights2_launch(const Problem &q) { return dl_launch_two_heights<false, TwoHi2, TwoLo2, true>(q); }
double kBfAsmTwoHeights2_cost(const Problem &q) { return dl_cost<TwoHi2>(q, 0.50); }
const Variant kBfAsmTwoHeights2 = {"bf16 224x256x128B then 192x256 in the last round, waves 2x4 ring 2(A)+2(B) direct-to-lds, reads as assembly, mfma16",
                                   kBfAsmTwoHeights2_can, kBfAsmTwoHeights2_launch, kBfAsmTwoHeights2_cost};
bool kBfAsmTwoHeights_can(const Problem &q) { return dl_can_run_common<false>(q, 224, 256, 128, 16); }
hipError_t kBfAsmTwoHeights_launch(const Problem &q) { return dl_launch_two_heights<false, TwoHi, TwoLo, true>(q); }
double kBfAsmTwoHeights_cost(const Problem &q) { return dl_cost<TwoHi>(q, 0.50); }
const Variant kBfAsmTwoHeights = {"bf16 224x256x128B then 192x256 in the last round, waves 2x4 ring 3(A)+2(B) direct-to-lds, reads as assembly, mfma16",
                                  kBfAsmTwoHeights_can, kBfAsmTwoHeights_launch, kBfAsmTwoHeights_cost};
XP_DL_ASM_VARIANT(kI8Asm256x256a3, "i8", true, 256, 256, 2, 4, 3, 2, 1, 0.55)
XP_DL_ASM_VARIANT(kI8Asm128x128, "i8", true, 128, 128, 2, 2, 2, 2, 2, 0.36)
XP_DL_ASM_VARIANT(kI8Asm256x128, "i8", true, 256, 128, 4, 2, 3, 3, 1, 0.46)
XP_DL_ASM_VARIANT(kI8Asm128x256, "i8", true, 128, 256, 2, 4, 3, 3, 1, 0.46)
XP_DL_ASM_VARIANT(kI8Asm256x256, "i8", true, 256, 256, 2, 4, 2, 2, 1, 0.54)

}  // namespace

int dl_asm_variants(xp_dtype in_type, const Variant **out)
{
    if (in_type == XP_BF16) {
        const Variant *v[] = {&kBfAsm256x256a3, &kBfAsm256x256, &kBfAsm224x256a3, &kBfAsmTwoHeights, &kBfAsm128x128, &kBfAsm256x128, &kBfAsm128x256,
                              &kBfAsm224x256, &kBfAsmTwoHeights2};
        for (size_t i = 0; i < sizeof v / sizeof *v; ++i) out[i] = v[i];
        return (int)(sizeof v / sizeof *v);
    }
    if (in_type == XP_I8) {
        const Variant *v[] = {&kI8Asm256x256a3, &kI8Asm256x256, &kI8Asm128x128, &kI8Asm256x128, &kI8Asm128x256};
        for (size_t i = 0; i < sizeof v / sizeof *v; ++i) out[i] = v[i];
        return (int)(sizeof v / sizeof *v);
    }
    return 0;
}

int dl_bnm_variants(xp_dtype in_type, const Variant **out)
{
    if (in_type != XP_BF16) return 0;
    const Variant *v[] = {&kBfBnm256x256a3, &kBfBnm256x256, &kBfBnm256x256b3, &kBfBnm128x128,
                          &kBfAmm256x256, &kBfAmm128x128, &kBfAmmBnm256x256, &kBfAmmBnm128x128,
                          &kBfBnm256x128, &kBfBnm128x256, &kBfAmm256x128, &kBfAmm128x256, &kBfAmmBnm256x128, &kBfAmmBnm128x256};
    for (size_t i = 0; i < sizeof v / sizeof *v; ++i) out[i] = v[i];
    return (int)(sizeof v / sizeof *v);
}

// Registered last of all: the variants before them keep their indices.
int dl_small_variants(xp_dtype in_type, const Variant **out)
{
    if (in_type != XP_BF16) return 0;
    out[0] = &kBfBnm64x64n3; out[1] = &kBfBnm64x64n4; out[2] = &kBfBnm128x64n3;
    return 3;
}

}  // namespace xp
