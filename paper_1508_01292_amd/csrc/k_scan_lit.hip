// The first stage in the paper's geometry with its weights as instruction literals: the workgroup routine of scan_body.h
// compiled for the device only into a code object whose placeholder constants the host replaces by a weight set.
#define CNNC_LITERAL_DEVICE_ONLY
#include "literal_weights.h"
#include "scan_body.h"

using namespace cnnc;

static_assert(scanbody::kScanParams <= kMaxLiteralWeights, "placeholder range");

#define CNNC_SCAN_LIT(NAME, ACT)                                                                                       \
    extern "C" __global__ __launch_bounds__(scanbody::kThreads) void NAME(                                             \
        const uint8_t *__restrict__ pyr, const ScanLevel *__restrict__ levels, const uint32_t *__restrict__ tiles,     \
        float *__restrict__ out)                                                                                       \
    {                                                                                                                  \
        scanbody::scan_tile<ACT>(pyr, levels, tiles, LiteralWeights{}, out);                                           \
    }

CNNC_SCAN_LIT(cnnc_scan_lit_act1, CNNC_ACT_RATIONAL)
CNNC_SCAN_LIT(cnnc_scan_lit_act2, CNNC_ACT_SCALED_TANH)
CNNC_SCAN_LIT(cnnc_scan_lit_act3, CNNC_ACT_TANH)
