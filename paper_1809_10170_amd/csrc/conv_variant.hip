// One compiled kernel variant per translation unit, so that the variants build in
// parallel.  The build passes V_NAME (the variant's name), V_FAMILY (DMA, ROWS, TAPS, PW or PWK) and
// V_PARAMS (the geometry's template arguments) from the matching row of variants.def.
#if !defined(V_NAME) || !defined(V_PARAMS) || !defined(V_FAMILY)
#error "compile with -DV_NAME=<name> -DV_FAMILY=<DMA|ROWS|TAPS|PW|PWK> -DV_PARAMS=<geometry template arguments>"
#endif

#define CONVD_FAMILY_DMA 2
#define CONVD_FAMILY_ROWS 3
#define CONVD_FAMILY_PW 4
#define CONVD_FAMILY_TAPS 5
#define CONVD_FAMILY_PWK 6
#define CONVD_CAT_(a, b) a##b
#define CONVD_CAT(a, b) CONVD_CAT_(a, b)
#define CONVD_STR_(a) #a
#define CONVD_STR(a) CONVD_STR_(a)

#if CONVD_CAT(CONVD_FAMILY_, V_FAMILY) == CONVD_FAMILY_DMA
#include "conv_dma_kernel.h"
#define CONVD_MAKE make_dma_variant<DmaGeom<V_PARAMS>>
#elif CONVD_CAT(CONVD_FAMILY_, V_FAMILY) == CONVD_FAMILY_ROWS
#include "conv_rows_kernel.h"
#define CONVD_MAKE make_rows_variant<RowGeom<V_PARAMS>>
#elif CONVD_CAT(CONVD_FAMILY_, V_FAMILY) == CONVD_FAMILY_PW
#include "conv_pw_kernel.h"
#define CONVD_MAKE make_pw_variant<PwGeom<V_PARAMS>>
#elif CONVD_CAT(CONVD_FAMILY_, V_FAMILY) == CONVD_FAMILY_PWK
#include "conv_pwk_kernel.h"
#define CONVD_MAKE make_pwk_variant<PwkGeom<V_PARAMS>>
#elif CONVD_CAT(CONVD_FAMILY_, V_FAMILY) == CONVD_FAMILY_TAPS
#include "conv_taps_kernel.h"
#define CONVD_MAKE make_taps_variant<TapGeom<V_PARAMS>>
#else
#error "unknown V_FAMILY"
#endif

namespace convd {
// Not const on purpose: a const object with a constant initialiser would also be
// emitted into the device code object, where the host launcher it points at is unknown.
extern Variant CONVD_CAT(variant_, V_NAME);
Variant CONVD_CAT(variant_, V_NAME) = CONVD_MAKE(CONVD_STR(V_NAME));
}  // namespace convd
