// Stage 1 (paper, Section 3.3: the first CNN densely scans every pyramid image; Section 3.4: the
// network is coded as one fused routine instead of a stack of layers).
//
// One launch covers every level through a (level, tile) table; the work of a workgroup is in stage1_body.h.
// Two builds of it exist: stage1_kernel reads its weights from memory (wave-uniform scalar loads), and the code
// object of k_stage1_lit.hip carries them as instruction literals, written in by the host for the context's weight
// set (literal_weights.h).  The second issues its multiply-adds at up to twice the rate and gives the same bits; it
// is used whenever its module loads.
#include "literal_weights.h"
#include "stage1_body.h"

#include "stage1_lit_image.inc"      // written by the build: kStage1LitImage, kStage1LitPatch

namespace cnnc {

using s1body::kThreads;

template <int ACT, bool EMIT>
__global__ __launch_bounds__(kThreads)
void stage1_kernel(const uint8_t *__restrict__ pyr, const LevelDev *__restrict__ levels,
                   const uint32_t *__restrict__ tiles, const float *__restrict__ wt,
                   float *__restrict__ score, float thr, uint32_t *__restrict__ mask)
{
    s1body::stage1_tile<ACT, EMIT>(pyr, levels, tiles, wt, score, thr, mask);
}

// ---- the build with literal weights ---------------------------------------------------------------------------
struct Stage1Literal {
    LiteralModule *mod = nullptr;
    hipFunction_t fn[3][2] = {{nullptr, nullptr}, {nullptr, nullptr}, {nullptr, nullptr}};   // [activation - 1][emit]
};

// Second convolution in the Winograd domain: F(3,3) along the kernel rows, interpolation points 0, 1, -1, 2 and infinity,
//   U = G w,  G = [1/2 0 0; -1/2 -1/2 -1/2; -1/6 1/6 -1/6; 1/6 1/3 2/3; 0 0 1]   (in fp64, then rounded)
void stage1_prepare_weights(const float *blob, float *prepared)
{
    static const double G[5][3] = {{0.5, 0, 0}, {-0.5, -0.5, -0.5}, {-1.0 / 6, 1.0 / 6, -1.0 / 6}, {1.0 / 6, 1.0 / 3, 2.0 / 3}, {0, 0, 1}};
    for (int i = 0; i < 40; ++i) prepared[s1p::W1 + i] = blob[s1::W1 + i];                  // first convolution and its biases
    for (int row = 0; row < 8 * 4 * 3; ++row)                                                // (k, c, a): one kernel row each
        for (int pt = 0; pt < 5; ++pt) {
            const float *w = blob + s1::W2 + row * 3;
            prepared[s1p::U2 + row * 5 + pt] = (float)(G[pt][0] * (double)w[0] + G[pt][1] * (double)w[1] + G[pt][2] * (double)w[2]);
        }
    for (int i = 0; i < 8; ++i) prepared[s1p::B2 + i] = blob[s1::B2 + i];
    for (int i = 0; i < 73; ++i) prepared[s1p::W3 + i] = blob[s1::W3 + i];                  // fc weights and bias
}

Stage1Literal *stage1_literal_create(const float *weights)
{
    static const LiteralImage img = {kStage1LitImage, sizeof(kStage1LitImage), kStage1LitPatch,
                                     sizeof(kStage1LitPatch) / sizeof(kStage1LitPatch[0]), kS1Prepared};
    LiteralModule *m = literal_acquire(img, weights);
    if (!m) return nullptr;
    Stage1Literal *s = new Stage1Literal();
    s->mod = m;
    static const char *const names[3][2] = {{"cnnc_s1_lit_act1", "cnnc_s1_lit_act1_emit"},
                                            {"cnnc_s1_lit_act2", "cnnc_s1_lit_act2_emit"},
                                            {"cnnc_s1_lit_act3", "cnnc_s1_lit_act3_emit"}};
    for (int a = 0; a < 3; ++a)
        for (int e = 0; e < 2; ++e)
            if (!(s->fn[a][e] = literal_function(m, names[a][e]))) {
                stage1_literal_destroy(s);
                return nullptr;
            }
    return s;
}

void stage1_literal_destroy(Stage1Literal *s)
{
    if (!s) return;
    literal_release(s->mod);
    delete s;
}

namespace {
hipError_t launch_literal(const cnnc_ctx *c, bool emit, int tile_begin, int n_tiles, float thr, uint32_t *mask, hipStream_t st)
{
    const uint8_t *pyr = c->d_pyr;
    const LevelDev *levels = c->d_levels;
    const uint32_t *tiles = c->d_tiles_s1 + tile_begin;
    float *score = c->d_score1;
    void *args[] = {&pyr, &levels, &tiles, &score, &thr, &mask};
    return hipModuleLaunchKernel(c->s1_literal->fn[c->act - 1][emit ? 1 : 0], (unsigned)n_tiles, 1, 1, kThreads, 1, 1, 0, st, args, nullptr);
}
}  // namespace

#define CNNC_S1(ACT, EMIT, THR, MASK)                                                                        \
    hipLaunchKernelGGL((stage1_kernel<ACT, EMIT>), grid, block, 0, st, c->d_pyr, c->d_levels, c->d_tiles_s1 + tile_begin, \
                       c->d_wt[0], c->d_score1, THR, MASK)

hipError_t launch_stage1(const cnnc_ctx *c, int tile_begin, int tile_end, hipStream_t st)
{
    if (tile_end <= tile_begin) return hipSuccess;
    if (c->s1_literal && c->use_literals) return launch_literal(c, false, tile_begin, tile_end - tile_begin, 0.0f, nullptr, st);
    dim3 grid(tile_end - tile_begin), block(kThreads);
    switch (c->act) {
    case CNNC_ACT_RATIONAL: CNNC_S1(CNNC_ACT_RATIONAL, false, 0.0f, (uint32_t *)nullptr); break;
    case CNNC_ACT_SCALED_TANH: CNNC_S1(CNNC_ACT_SCALED_TANH, false, 0.0f, (uint32_t *)nullptr); break;
    default: CNNC_S1(CNNC_ACT_TANH, false, 0.0f, (uint32_t *)nullptr); break;
    }
    return hipGetLastError();
}

hipError_t launch_stage1_emit(const cnnc_ctx *c, float thr, hipStream_t st)
{
    const int tile_begin = 0;
    if (c->s1_literal && c->use_literals) return launch_literal(c, true, 0, c->n_tiles_s1, thr, c->d_mask1, st);
    dim3 grid(c->n_tiles_s1), block(kThreads);
    switch (c->act) {
    case CNNC_ACT_RATIONAL: CNNC_S1(CNNC_ACT_RATIONAL, true, thr, c->d_mask1); break;
    case CNNC_ACT_SCALED_TANH: CNNC_S1(CNNC_ACT_SCALED_TANH, true, thr, c->d_mask1); break;
    default: CNNC_S1(CNNC_ACT_TANH, true, thr, c->d_mask1); break;
    }
    return hipGetLastError();
}
#undef CNNC_S1

}  // namespace cnnc
