// The selective unit with the first layers' weights of CNN_2 and CNN_3 as instruction literals: the workgroup routine
// of select_body.h compiled for the device only into a code object whose placeholder constants the host replaces.
#define CNNC_LITERAL_DEVICE_ONLY
#include "literal_weights.h"
#include "select_body.h"

using namespace cnnc;
using namespace cnnc::selbody;

static_assert(kFirstLayers <= kMaxLiteralWeights, "placeholder range");

#define CNNC_SELECT_LIT(NAME, ACT)                                                                                          \
    extern "C" __global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(4, 4))) void NAME(                  \
        const uint8_t *__restrict__ frame, int fw, int fh, int pitch, const LevelDev *__restrict__ levels,                   \
        const ScanLevel *__restrict__ slev, int n_levels, const uint32_t *__restrict__ idx, const float *__restrict__ resp,  \
        const int32_t *__restrict__ d_n, int n_max, const float *__restrict__ w2, const float *__restrict__ w3,              \
        const float *__restrict__ f2, const float *__restrict__ f3, float t2, float t3, int t_nn, int rule,                  \
        cnnc_region *__restrict__ rec, float *__restrict__ maps2, float *__restrict__ maps3)                                 \
    {                                                                                                                        \
        select_regions<ACT>(frame, fw, fh, pitch, levels, slev, n_levels, idx, resp, d_n, n_max, w2, w3, LiteralWeightsAt<0>{}, \
                            LiteralWeightsAt<kFirst2>{}, f2, f3, t2, t3, t_nn, rule, rec, maps2, maps3);                     \
    }

CNNC_SELECT_LIT(cnnc_select_lit_act1, CNNC_ACT_RATIONAL)
CNNC_SELECT_LIT(cnnc_select_lit_act2, CNNC_ACT_SCALED_TANH)
CNNC_SELECT_LIT(cnnc_select_lit_act3, CNNC_ACT_TANH)
