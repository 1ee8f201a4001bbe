// One compiled tile variant per translation unit, so that the variants build in
// parallel.  The build passes V_NAME (the variant's name) and V_PARAMS (the Geom
// template arguments) from the matching row of variants.def.
#include "conv_tile_kernel.h"

#if !defined(V_NAME) || !defined(V_PARAMS)
#error "compile with -DV_NAME=<name> -DV_PARAMS=<R,S,ST,TP,TQ,KBW,PBW,WK,WP,CB,PAIR,OCC,PREF>"
#endif

#define CONVD_CAT_(a, b) a##b
#define CONVD_CAT(a, b) CONVD_CAT_(a, b)
#define CONVD_STR_(a) #a
#define CONVD_STR(a) CONVD_STR_(a)

namespace convd {
// Not const on purpose: a const object with a constant initialiser would also be
// emitted into the device code object, where the host launcher it points at is unknown.
extern Variant CONVD_CAT(variant_, V_NAME);
Variant CONVD_CAT(variant_, V_NAME) = make_variant<Geom<V_PARAMS>>(CONVD_STR(V_NAME));
}  // namespace convd
