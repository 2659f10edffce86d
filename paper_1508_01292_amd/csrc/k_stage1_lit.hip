// Stage 1 with its weights as instruction literals: the same workgroup routine as stage1_kernel, compiled for the
// gfx950 device only into a code object of its own whose placeholder constants the host replaces by a weight set
// (paper, Section 3.4: one fused routine per network).  No host code here.
#define CNNC_LITERAL_DEVICE_ONLY
#include "literal_weights.h"
#include "stage1_body.h"

using namespace cnnc;

static_assert(kS1Prepared <= kMaxLiteralWeights, "placeholder range");

#define CNNC_S1_LIT(NAME, ACT, EMIT)                                                                                  \
    extern "C" __global__ __launch_bounds__(s1body::kThreads) void NAME(                                               \
        const uint8_t *__restrict__ pyr, const LevelDev *__restrict__ levels, const uint32_t *__restrict__ tiles,      \
        float *__restrict__ score, float thr, uint32_t *__restrict__ mask)                                             \
    {                                                                                                                  \
        s1body::stage1_tile<ACT, EMIT>(pyr, levels, tiles, LiteralWeights{}, score, thr, mask);                         \
    }

CNNC_S1_LIT(cnnc_s1_lit_act1, CNNC_ACT_RATIONAL, false)
CNNC_S1_LIT(cnnc_s1_lit_act2, CNNC_ACT_SCALED_TANH, false)
CNNC_S1_LIT(cnnc_s1_lit_act3, CNNC_ACT_TANH, false)
CNNC_S1_LIT(cnnc_s1_lit_act1_emit, CNNC_ACT_RATIONAL, true)
CNNC_S1_LIT(cnnc_s1_lit_act2_emit, CNNC_ACT_SCALED_TANH, true)
CNNC_S1_LIT(cnnc_s1_lit_act3_emit, CNNC_ACT_TANH, true)
