// One translation unit per launcher and (element type, head dimension, with / without the distance-bias code):
//   -DENTMAX_INST_FWD or -DENTMAX_INST_BWD, -DENTMAX_INST_T=<bf16_t|float>, -DENTMAX_INST_D=<64|128>,
//   -DENTMAX_INST_BIAS=<0|1>
#if defined(ENTMAX_INST_FWD)
#include "run_fwd.hip.h"
namespace entmax {
template int run_fwd<ENTMAX_INST_T, ENTMAX_INST_D, ENTMAX_INST_BIAS != 0>(const entmax_attn_params*, const Layout&, const void*,
                                                                         const void*, const void*, const float*,
                                                                         const float*, const float*, void*, float*, char*,
                                                                         size_t, uint64_t*, char*, hipStream_t, void* const*);
}
#elif defined(ENTMAX_INST_BWD)
#include "run_bwd.hip.h"
namespace entmax {
template int run_bwd<ENTMAX_INST_T, ENTMAX_INST_D, ENTMAX_INST_BIAS != 0>(const entmax_attn_params*, const Layout&, const void*,
                                                                         const void*, const void*, const void*,
                                                                         const float*, const char*, size_t, const float*,
                                                                         const float*, const float*, void*, void*, void*,
                                                                         float*, float*, uint64_t*, char*, hipStream_t,
                                                                         void* const*);
}
#else
#error "define ENTMAX_INST_FWD or ENTMAX_INST_BWD"
#endif
