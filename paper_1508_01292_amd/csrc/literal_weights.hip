// Modules whose weights are instruction literals: patch, load, share (see literal_weights.h).
#include "literal_weights.h"

#include <string.h>

#include <mutex>
#include <vector>

namespace cnnc {

struct LiteralModule {
    const unsigned char *image;      // which code object
    int device;
    std::vector<float> weights;
    hipModule_t mod;
    int refs;
};

namespace {
std::mutex g_mu;
std::vector<LiteralModule *> g_modules;
}  // namespace

LiteralModule *literal_acquire(const LiteralImage &img, const float *weights)
{
    if (!img.image || img.size == 0 || img.n_patch == 0 || img.n_weights <= 0 || !weights) return nullptr;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return nullptr;
    std::lock_guard<std::mutex> lock(g_mu);
    for (LiteralModule *m : g_modules)
        if (m->image == img.image && m->device == dev &&
            memcmp(m->weights.data(), weights, sizeof(float) * (size_t)img.n_weights) == 0) {
            ++m->refs;
            return m;
        }
    std::vector<unsigned char> code(img.image, img.image + img.size);
    for (size_t k = 0; k < img.n_patch; ++k) {
        const uint32_t off = img.patch[k][0], idx = img.patch[k][1];
        if ((size_t)off + 4 > img.size || idx >= (uint32_t)img.n_weights) return nullptr;   // a table that does not fit its image
        memcpy(code.data() + off, weights + idx, 4);
    }
    hipModule_t mod = nullptr;
    if (hipModuleLoadData(&mod, code.data()) != hipSuccess) {
        (void)hipGetLastError();
        return nullptr;
    }
    LiteralModule *m = new LiteralModule{img.image, dev, std::vector<float>(weights, weights + img.n_weights), mod, 1};
    g_modules.push_back(m);
    return m;
}

void literal_release(LiteralModule *m)
{
    if (!m) return;
    std::lock_guard<std::mutex> lock(g_mu);
    if (--m->refs > 0) return;
    for (size_t k = 0; k < g_modules.size(); ++k)
        if (g_modules[k] == m) { g_modules.erase(g_modules.begin() + (long)k); break; }
    (void)hipModuleUnload(m->mod);
    delete m;
}

hipFunction_t literal_function(LiteralModule *m, const char *name)
{
    hipFunction_t f = nullptr;
    if (!m || hipModuleGetFunction(&f, m->mod, name) != hipSuccess) {
        (void)hipGetLastError();
        return nullptr;
    }
    return f;
}

}  // namespace cnnc
