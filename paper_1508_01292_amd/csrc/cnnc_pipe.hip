// Frame ingest: a ring of slots, each with its own context, stream, pinned host frame and device frame, so that
// the host-to-device copy of one frame, the kernels of others and the read-back of finished ones overlap
// (paper, Section 3.4: asynchronous mode, frames processed in constant time; Section 4.2: video throughput).
// With graphs on, the per-frame sequence (copy in, every kernel of the path, results out) is captured once per
// slot and replayed with one launch per frame.
#include <string.h>

#include <new>
#include <string>
#include <vector>

#include "cnnc_internal.h"

namespace {

struct Slot {
    cnnc_ctx *ctx = nullptr;
    hipStream_t st = nullptr;
    uint8_t *h_frame = nullptr;   // pinned, w * h bytes, row pitch w
    uint8_t *d_frame = nullptr;
    hipGraph_t graph = nullptr;
    hipGraphExec_t exec = nullptr;
    int runs = 0;                 // frames this slot has processed since its parameters last changed
    bool busy = false;
    int64_t ticket = -1;
};

}  // namespace

struct cnnc_pipe {
    std::vector<Slot> slots;
    int w = 0, h = 0;
    bool use_graph = false;
    bool paper = false;            // submit runs the path in the paper's geometry (cnnc_pipe_set_paper)
    cnnc_paper_params pp{};
    int64_t next_ticket = 0;
    std::string err;
};

namespace {

int pfail(cnnc_pipe *p, int code, const std::string &msg)
{
    if (p) p->err = msg;
    return code;
}

#define PIPE_HIP(p, expr)                                                                         \
    do {                                                                                          \
        hipError_t e_ = (expr);                                                                   \
        if (e_ != hipSuccess) return pfail((p), e_ == hipErrorOutOfMemory ? CNNC_E_NOMEM : CNNC_E_HIP, \
                                           std::string(#expr) + ": " + hipGetErrorString(e_));    \
    } while (0)

// The slot the next submit uses: the free slot that has waited longest (slots are fetched in any order).
Slot *free_slot(cnnc_pipe *p)
{
    Slot *best = nullptr;
    for (Slot &s : p->slots)
        if (!s.busy && (!best || s.ticket < best->ticket)) best = &s;
    return best;
}

void drop_graph(Slot &s)
{
    if (s.exec) { (void)hipGraphExecDestroy(s.exec); s.exec = nullptr; }
    if (s.graph) { (void)hipGraphDestroy(s.graph); s.graph = nullptr; }
}

// Copy in + the whole path + results out, on the slot's stream.
int enqueue_frame(cnnc_pipe *p, Slot &s)
{
    PIPE_HIP(p, hipMemcpyAsync(s.d_frame, s.h_frame, (size_t)p->w * p->h, hipMemcpyHostToDevice, s.st));
    const int rc = p->paper ? cnnc_detect_paper_async(s.ctx, s.d_frame, p->w, p->h, p->w, &p->pp, s.st)
                            : cnnc_detect_async(s.ctx, s.d_frame, p->w, p->h, p->w, s.st);
    if (rc) return pfail(p, rc, std::string("detect: ") + cnnc_last_error(s.ctx));
    return CNNC_OK;
}

}  // namespace

extern "C" {

int cnnc_pipe_destroy(cnnc_pipe *p)
{
    if (!p) return CNNC_OK;
    for (Slot &s : p->slots) {
        if (s.st) (void)hipStreamSynchronize(s.st);
        drop_graph(s);
        if (s.ctx) (void)cnnc_destroy(s.ctx);
        if (s.h_frame) (void)hipHostFree(s.h_frame);
        if (s.d_frame) (void)hipFree(s.d_frame);
        if (s.st) (void)hipStreamDestroy(s.st);
    }
    delete p;
    return CNNC_OK;
}

int cnnc_pipe_create(cnnc_pipe **out, const cnnc_stage_desc stages[3], int w, int h, int max_survivors, int depth,
                     int use_graph)
{
    if (!out) return CNNC_E_INVAL;
    *out = nullptr;
    if (!stages || depth < 1 || depth > 16 || w < CNNC_WINDOW || h < CNNC_WINDOW) return CNNC_E_INVAL;
    cnnc_pipe *p = new (std::nothrow) cnnc_pipe();
    if (!p) return CNNC_E_NOMEM;
    p->w = w; p->h = h; p->use_graph = use_graph != 0;
    p->slots.resize((size_t)depth);
    int rc = CNNC_OK;
    for (Slot &s : p->slots) {
        if ((rc = cnnc_create(&s.ctx, stages, w, h, max_survivors))) break;
        if (hipStreamCreateWithFlags(&s.st, hipStreamNonBlocking) != hipSuccess) { rc = CNNC_E_HIP; break; }
        if (hipHostMalloc((void **)&s.h_frame, (size_t)w * h, hipHostMallocDefault) != hipSuccess) { rc = CNNC_E_NOMEM; break; }
        if (hipMalloc((void **)&s.d_frame, (size_t)w * h) != hipSuccess) { rc = CNNC_E_NOMEM; break; }
    }
    if (rc) { cnnc_pipe_destroy(p); return rc; }
    *out = p;
    return CNNC_OK;
}

int cnnc_pipe_set_params(cnnc_pipe *p, const cnnc_params *prm)
{
    if (!p || !prm) return CNNC_E_INVAL;
    for (Slot &s : p->slots)
        if (s.busy) return pfail(p, CNNC_E_STATE, "frames are still in flight: fetch them before changing parameters");
    for (Slot &s : p->slots) {
        const int rc = cnnc_set_params(s.ctx, prm);
        if (rc) return pfail(p, rc, cnnc_last_error(s.ctx));
        drop_graph(s);             // thresholds and geometry are baked into the captured launches
        s.runs = 0;
    }
    return CNNC_OK;
}

int cnnc_pipe_set_paper(cnnc_pipe *p, const float *scan_w, int n_scan, int scan_act, const float *w2, int n2, const float *w3,
                        int n3, int sel_act, int rule, const cnnc_paper_params *pp)
{
    if (!p || !pp) return CNNC_E_INVAL;
    for (Slot &s : p->slots)
        if (s.busy) return pfail(p, CNNC_E_STATE, "frames are still in flight: fetch them before changing the path");
    for (Slot &s : p->slots) {
        int rc = cnnc_scan_set_weights(s.ctx, scan_w, n_scan, scan_act);
        if (!rc) rc = cnnc_select_set_weights(s.ctx, w2, n2, w3, n3, sel_act);
        if (!rc) rc = cnnc_select_set_rule(s.ctx, rule);
        if (rc) return pfail(p, rc, cnnc_last_error(s.ctx));
        drop_graph(s);             // another sequence of launches; thresholds are baked into a captured one
        s.runs = 0;
    }
    p->pp = *pp;
    p->paper = true;
    return CNNC_OK;
}

int cnnc_pipe_frame_buffer(cnnc_pipe *p, uint8_t **h_frame)
{
    if (!p || !h_frame) return CNNC_E_INVAL;
    Slot *fs = free_slot(p);
    if (!fs) return pfail(p, CNNC_E_STATE, "every slot is in flight: fetch a frame first");
    *h_frame = fs->h_frame;
    return CNNC_OK;
}

int cnnc_pipe_submit(cnnc_pipe *p, const uint8_t *h_frame, int pitch, int64_t *ticket)
{
    if (!p || !ticket) return CNNC_E_INVAL;
    Slot *fs = free_slot(p);
    if (!fs) return pfail(p, CNNC_E_STATE, "every slot is in flight: fetch a frame first");
    Slot &s = *fs;
    if (h_frame && h_frame != s.h_frame) {
        if (pitch < p->w) return pfail(p, CNNC_E_INVAL, "pitch < width");
        for (int y = 0; y < p->h; ++y) memcpy(s.h_frame + (size_t)y * p->w, h_frame + (size_t)y * pitch, (size_t)p->w);
    }
    int rc = CNNC_OK;
    if (!p->use_graph || s.runs == 0) {
        // eager; a slot's first frame always is, so that every table and buffer exists before a capture
        rc = enqueue_frame(p, s);
    } else {
        if (!s.exec) {
            PIPE_HIP(p, hipStreamBeginCapture(s.st, hipStreamCaptureModeThreadLocal));
            rc = enqueue_frame(p, s);
            hipGraph_t g = nullptr;
            const hipError_t e = hipStreamEndCapture(s.st, &g);
            if (rc == CNNC_OK && e != hipSuccess) rc = pfail(p, CNNC_E_HIP, std::string("hipStreamEndCapture: ") + hipGetErrorString(e));
            if (rc) { if (g) (void)hipGraphDestroy(g); return rc; }
            const hipError_t ei = hipGraphInstantiate(&s.exec, g, nullptr, nullptr, 0);
            if (ei != hipSuccess) {
                (void)hipGraphDestroy(g);
                s.exec = nullptr;
                return pfail(p, CNNC_E_HIP, std::string("hipGraphInstantiate: ") + hipGetErrorString(ei));
            }
            s.graph = g;
        }
        PIPE_HIP(p, hipGraphLaunch(s.exec, s.st));
    }
    if (rc) return rc;
    ++s.runs;
    s.busy = true;
    s.ticket = p->next_ticket++;
    *ticket = s.ticket;
    return CNNC_OK;
}

int cnnc_pipe_fetch(cnnc_pipe *p, int64_t ticket, cnnc_det *out, int cap, int *n_out)
{
    if (!p || !n_out || (!out && cap > 0) || cap < 0) return CNNC_E_INVAL;
    if (p->paper) return pfail(p, CNNC_E_STATE, "this pipe runs the paper-geometry path: use cnnc_pipe_fetch_paper");
    for (Slot &s : p->slots) {
        if (!s.busy || s.ticket != ticket) continue;
        const int rc = cnnc_fetch_detections(s.ctx, out, cap, n_out);
        s.busy = false;
        if (rc) return pfail(p, rc, cnnc_last_error(s.ctx));
        return CNNC_OK;
    }
    return pfail(p, CNNC_E_INVAL, "no frame in flight has this ticket");
}

int cnnc_pipe_fetch_paper(cnnc_pipe *p, int64_t ticket, cnnc_rdet *out, int cap, int *n_out)
{
    if (!p || !n_out || (!out && cap > 0) || cap < 0) return CNNC_E_INVAL;
    if (!p->paper) return pfail(p, CNNC_E_STATE, "cnnc_pipe_set_paper has not been called");
    for (Slot &s : p->slots) {
        if (!s.busy || s.ticket != ticket) continue;
        const int rc = cnnc_fetch_paper(s.ctx, out, cap, n_out);
        s.busy = false;
        if (rc) return pfail(p, rc, cnnc_last_error(s.ctx));
        return CNNC_OK;
    }
    return pfail(p, CNNC_E_INVAL, "no frame in flight has this ticket");
}

const char *cnnc_pipe_last_error(const cnnc_pipe *p) { return p ? p->err.c_str() : "null pipe"; }

}  // extern "C"
