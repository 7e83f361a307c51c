// Direct-to-LDS kernels, fragment reads left to the compiler (modes 0-2 of dl_body): the variant tables.
#include "xp_mfma_dl.hpp"

namespace xp {
namespace {

#define XP_DL_VARIANT(NAME, TYPESTR, INT8, BM, BN, WM, WN, NS, RB, SPREAD, SPREADSTR, OCC, MF, NT, NTSTR, EFF)                                        \
    bool NAME##_can(const Problem &q) { return dl_can_run_common<INT8>(q, BM, BN, RB, MF); }                       \
    hipError_t NAME##_launch(const Problem &q) { return dl_launch<INT8, DlTile<BM, BN, WM, WN, NS, RB, SPREAD, OCC, MF, NT>>(q); }  \
    double NAME##_cost(const Problem &q) { return dl_cost<DlTile<BM, BN, WM, WN, NS, RB, SPREAD, OCC, MF, NT>>(q, EFF); }           \
    const Variant NAME = {TYPESTR " " #BM "x" #BN "x" #RB "B waves " #WM "x" #WN " ring " #NS SPREADSTR " direct-to-lds" NTSTR " mfma" #MF, \
                          NAME##_can, NAME##_launch, NAME##_cost};

XP_DL_VARIANT(kBfDl256x256r128n2, "bf16", false, 256, 256, 2, 4, 2, 128, false, "", 1, 32, false, "", 0.52)
XP_DL_VARIANT(kBfDl256x256r128n2m16, "bf16", false, 256, 256, 2, 4, 2, 128, false, "", 1, 16, false, "", 0.55)
XP_DL_VARIANT(kBfDl208x256w1x8m16, "bf16", false, 208, 256, 1, 8, 2, 128, false, "", 1, 16, false, "", 0.50)
XP_DL_VARIANT(kBfDl224x256w2x4m16, "bf16", false, 224, 256, 2, 4, 2, 128, false, "", 1, 16, false, "", 0.50)
XP_DL_VARIANT(kBfDl256x256r128n2w4m16, "bf16", false, 256, 256, 2, 2, 2, 128, false, "", 1, 16, false, "", 0.5)
XP_DL_VARIANT(kBfDl256x256r64n4m16, "bf16", false, 256, 256, 2, 4, 4, 64, false, "", 1, 16, false, "", 0.5)
XP_DL_VARIANT(kBfDl128x128r128n2m16, "bf16", false, 128, 128, 2, 2, 2, 128, false, "", 2, 16, false, "", 0.34)
XP_DL_VARIANT(kBfDl256x256r64n4, "bf16", false, 256, 256, 2, 4, 4, 64, false, "", 1, 32, false, "", 0.5)
XP_DL_VARIANT(kBfDl256x256r64n4s, "bf16", false, 256, 256, 2, 4, 4, 64, true, " spread", 1, 32, false, "", 0.5)
XP_DL_VARIANT(kBfDl256x256r64n3s, "bf16", false, 256, 256, 2, 4, 3, 64, true, " spread", 1, 32, false, "", 0.5)
XP_DL_VARIANT(kBfDl256x256r128n2w4, "bf16", false, 256, 256, 2, 2, 2, 128, false, "", 1, 32, false, "", 0.48)
XP_DL_VARIANT(kBfDl256x128r64n3, "bf16", false, 256, 128, 2, 2, 3, 64, false, "", 2, 32, false, "", 0.45)
XP_DL_VARIANT(kBfDl256x128r64n3s, "bf16", false, 256, 128, 2, 2, 3, 64, true, " spread", 2, 32, false, "", 0.45)
XP_DL_VARIANT(kBfDl128x256r64n3s, "bf16", false, 128, 256, 2, 2, 3, 64, true, " spread", 2, 32, false, "", 0.45)
XP_DL_VARIANT(kBfDl128x128r128n2, "bf16", false, 128, 128, 2, 2, 2, 128, false, "", 2, 32, false, "", 0.32)
XP_DL_VARIANT(kBfDl128x128r64n4s, "bf16", false, 128, 128, 2, 2, 4, 64, true, " spread", 2, 32, false, "", 0.40)

XP_DL_VARIANT(kI8Dl256x256r128n2, "i8", true, 256, 256, 2, 4, 2, 128, false, "", 1, 32, false, "", 0.52)
XP_DL_VARIANT(kI8Dl256x256r128n2m16, "i8", true, 256, 256, 2, 4, 2, 128, false, "", 1, 16, false, "", 0.55)
XP_DL_VARIANT(kI8Dl256x256r128n2w4m16, "i8", true, 256, 256, 2, 2, 2, 128, false, "", 1, 16, false, "", 0.5)
XP_DL_VARIANT(kI8Dl256x256r64n4m16, "i8", true, 256, 256, 2, 4, 4, 64, false, "", 1, 16, false, "", 0.5)
XP_DL_VARIANT(kI8Dl128x128r128n2m16, "i8", true, 128, 128, 2, 2, 2, 128, false, "", 2, 16, false, "", 0.34)
XP_DL_VARIANT(kI8Dl256x256r64n4, "i8", true, 256, 256, 2, 4, 4, 64, false, "", 1, 32, false, "", 0.5)
XP_DL_VARIANT(kI8Dl256x256r64n4s, "i8", true, 256, 256, 2, 4, 4, 64, true, " spread", 1, 32, false, "", 0.5)
XP_DL_VARIANT(kI8Dl256x256r64n3s, "i8", true, 256, 256, 2, 4, 3, 64, true, " spread", 1, 32, false, "", 0.5)
XP_DL_VARIANT(kI8Dl256x256r128n2w4, "i8", true, 256, 256, 2, 2, 2, 128, false, "", 1, 32, false, "", 0.48)
XP_DL_VARIANT(kI8Dl256x128r64n3, "i8", true, 256, 128, 2, 2, 3, 64, false, "", 2, 32, false, "", 0.45)
XP_DL_VARIANT(kI8Dl256x128r64n3s, "i8", true, 256, 128, 2, 2, 3, 64, true, " spread", 2, 32, false, "", 0.45)
XP_DL_VARIANT(kI8Dl128x256r64n3s, "i8", true, 128, 256, 2, 2, 3, 64, true, " spread", 2, 32, false, "", 0.45)
XP_DL_VARIANT(kI8Dl128x128r128n2, "i8", true, 128, 128, 2, 2, 2, 128, false, "", 2, 32, false, "", 0.32)
XP_DL_VARIANT(kI8Dl128x128r64n4s, "i8", true, 128, 128, 2, 2, 4, 64, true, " spread", 2, 32, false, "", 0.40)

// one more A buffer than B buffers: three A + two B buffers of 32 KB fill the 160 KB of LDS exactly
#define XP_DL_ASYM_VARIANT(NAME, TYPESTR, INT8, BM, BN, WM, WN, MF, EFF)                                                              \
    bool NAME##_can(const Problem &q) { return dl_can_run_common<INT8>(q, BM, BN, 128, 16); }                                            \
    hipError_t NAME##_launch(const Problem &q) { return dl_launch<INT8, DlTile<BM, BN, WM, WN, 2, 128, false, 1, MF, false, 3>>(q); } \
    double NAME##_cost(const Problem &q) { return dl_cost<DlTile<BM, BN, WM, WN, 2, 128, false, 1, MF, false, 3>>(q, EFF); }          \
    const Variant NAME = {TYPESTR " " #BM "x" #BN "x128B waves " #WM "x" #WN " ring 3(A)+2(B) direct-to-lds mfma" #MF, NAME##_can, \
                          NAME##_launch, NAME##_cost};

XP_DL_ASYM_VARIANT(kBfDl256x256a3m16, "bf16", false, 256, 256, 2, 4, 16, 0.54)
XP_DL_ASYM_VARIANT(kBfDl224x256a3m16, "bf16", false, 224, 256, 2, 4, 16, 0.49)
XP_DL_ASYM_VARIANT(kI8Dl256x256a3m16, "i8", true, 256, 256, 2, 4, 16, 0.54)

bool kBfDlTwoHeights_can(const Problem &q) { return dl_can_run_common<false>(q, 224, 256, 128, 16); }
hipError_t kBfDlTwoHeights_launch(const Problem &q) { return dl_launch_two_heights<false, TwoHi, TwoLo>(q); }
double kBfDlTwoHeights_cost(const Problem &q) { return dl_cost<TwoHi>(q, 0.49); }
const Variant kBfDlTwoHeights = {"bf16 224x256x128B then 192x256 in the last round, waves 2x4 ring 3(A)+2(B) direct-to-lds mfma16",
                                 kBfDlTwoHeights_can, kBfDlTwoHeights_launch, kBfDlTwoHeights_cost};

}  // namespace

#ifdef XP_TRACE
long long *g_dl_trace = nullptr;
void set_dl_trace(long long *p) { g_dl_trace = p; }
#endif

// Registered after every other family so that the older variants keep their indices.
int dl_asym_variants(xp_dtype in_type, const Variant **out)
{
    if (in_type == XP_BF16) { out[0] = &kBfDl256x256a3m16; out[1] = &kBfDl224x256a3m16; out[2] = &kBfDlTwoHeights; return 3; }
    if (in_type == XP_I8) { out[0] = &kI8Dl256x256a3m16; return 1; }
    return 0;
}

int dl_variants(xp_dtype in_type, const Variant **out)
{
    if (in_type == XP_BF16) {
        const Variant *v[] = {&kBfDl256x256r128n2, &kBfDl256x256r128n2m16, &kBfDl208x256w1x8m16, &kBfDl224x256w2x4m16, &kBfDl256x256r128n2w4m16, &kBfDl256x256r64n4m16, &kBfDl128x128r128n2m16, &kBfDl256x256r64n4, &kBfDl256x256r64n4s, &kBfDl256x256r64n3s, &kBfDl256x256r128n2w4, &kBfDl256x128r64n3, &kBfDl256x128r64n3s, &kBfDl128x256r64n3s, &kBfDl128x128r128n2, &kBfDl128x128r64n4s};
        for (size_t i = 0; i < sizeof v / sizeof *v; ++i) out[i] = v[i];
        return (int)(sizeof v / sizeof *v);
    }
    if (in_type == XP_I8) {
        const Variant *v[] = {&kI8Dl256x256r128n2, &kI8Dl256x256r128n2m16, &kI8Dl256x256r128n2w4m16, &kI8Dl256x256r64n4m16, &kI8Dl128x128r128n2m16, &kI8Dl256x256r64n4, &kI8Dl256x256r64n4s, &kI8Dl256x256r64n3s, &kI8Dl256x256r128n2w4, &kI8Dl256x128r64n3, &kI8Dl256x128r64n3s, &kI8Dl128x256r64n3s, &kI8Dl128x128r128n2, &kI8Dl128x128r64n4s};
        for (size_t i = 0; i < sizeof v / sizeof *v; ++i) out[i] = v[i];
        return (int)(sizeof v / sizeof *v);
    }
    return 0;
}

}  // namespace xp

#ifdef XP_TRACE
// Diagnostic build only (not declared in include/xp.h): device buffer of 16 x 64-bit words per workgroup that every
// direct-to-LDS kernel launched afterwards fills with its time stamps; nullptr switches it off.
extern "C" void xp_debug_set_dl_trace(void *device_buffer) { xp::set_dl_trace((long long *)device_buffer); }
#endif
