// The first stage in the paper's geometry with its weights as instruction literals: the workgroup routine of scan_body.h
// compiled for the device only into a code object whose placeholder constants the host replaces by a weight set.
#define CNNC_LITERAL_DEVICE_ONLY
#include "literal_weights.h"
#include "scan_body.h"

using namespace cnnc;

static_assert(scanbody::kScanParams <= kMaxLiteralWeights, "placeholder range");

#define CNNC_SCAN_LIT(NAME, ACT, SHAPE)                                                                                \
    extern "C" __global__ __launch_bounds__(scanbody::SHAPE::kThreads) void NAME(                                      \
        const uint8_t *__restrict__ pyr, const ScanLevel *__restrict__ levels, const uint32_t *__restrict__ tiles,     \
        float *__restrict__ out)                                                                                       \
    {                                                                                                                  \
        scanbody::scan_tile<ACT, scanbody::SHAPE>(pyr, levels, tiles, LiteralWeights{}, out);                          \
    }

CNNC_SCAN_LIT(cnnc_scan_lit_act1_t8, CNNC_ACT_RATIONAL, Shape8)
CNNC_SCAN_LIT(cnnc_scan_lit_act2_t8, CNNC_ACT_SCALED_TANH, Shape8)
CNNC_SCAN_LIT(cnnc_scan_lit_act3_t8, CNNC_ACT_TANH, Shape8)
CNNC_SCAN_LIT(cnnc_scan_lit_act1_t16, CNNC_ACT_RATIONAL, Shape16)
CNNC_SCAN_LIT(cnnc_scan_lit_act2_t16, CNNC_ACT_SCALED_TANH, Shape16)
CNNC_SCAN_LIT(cnnc_scan_lit_act3_t16, CNNC_ACT_TANH, Shape16)
