// Explicit instantiations of the tiled kernel family.  Compiled once per WPK_PART (0..7) so the
// build can run the parts in parallel; each part emits the variants tagged with its number.
#include "wpk_wsplit.h"

#ifndef WPK_PART
#error "compile with -DWPK_PART=<0..7>"
#endif

namespace wpk {
#define WPK_EMIT(BM, BN, BK, WM, WN, PD) \
    template hipError_t launch_igemm<BM, BN, BK, WM, WN, PD>(const IgemmArgs &, hipStream_t);
#define WPK_SKIP(BM, BN, BK, WM, WN, PD)
#define WPK_SEL_0 WPK_SKIP
#define WPK_SEL_1 WPK_SKIP
#define WPK_SEL_2 WPK_SKIP
#define WPK_SEL_3 WPK_SKIP
#define WPK_SEL_4 WPK_SKIP
#define WPK_SEL_5 WPK_SKIP
#define WPK_SEL_6 WPK_SKIP
#define WPK_SEL_7 WPK_SKIP
#if WPK_PART == 0
#undef WPK_SEL_0
#define WPK_SEL_0 WPK_EMIT
#elif WPK_PART == 1
#undef WPK_SEL_1
#define WPK_SEL_1 WPK_EMIT
#elif WPK_PART == 2
#undef WPK_SEL_2
#define WPK_SEL_2 WPK_EMIT
#elif WPK_PART == 3
#undef WPK_SEL_3
#define WPK_SEL_3 WPK_EMIT
#elif WPK_PART == 4
#undef WPK_SEL_4
#define WPK_SEL_4 WPK_EMIT
#elif WPK_PART == 5
#undef WPK_SEL_5
#define WPK_SEL_5 WPK_EMIT
#elif WPK_PART == 6
#undef WPK_SEL_6
#define WPK_SEL_6 WPK_EMIT
#elif WPK_PART == 7
#undef WPK_SEL_7
#define WPK_SEL_7 WPK_EMIT
#endif
#define WPK_VARIANT(PART, BM, BN, BK, WM, WN, PD) WPK_SEL_##PART(BM, BN, BK, WM, WN, PD)
#include WPK_VARIANTS_FILE
#undef WPK_VARIANT
}  // namespace wpk
