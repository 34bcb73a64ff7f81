// Analytic cost model (Sec. 5.1): t_c, t_s, t_x tables.
#include "lwp.h"

extern "C" lwp_status lwp_build_cost_tables(lwp_ctx*, const lwp_layer*, int32_t, const int32_t*, int32_t,
                                            const lwp_config*, int32_t, const lwp_machine*, int32_t*, int32_t*,
                                            int32_t*) {
    return LWP_E_INVAL;   // filled in by the table-builder kernels
}
