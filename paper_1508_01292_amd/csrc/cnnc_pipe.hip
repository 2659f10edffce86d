// Frame ingest: a ring of slots (pinned host frame + device frame) fed to a few lanes (context + stream), so that the
// host-to-device copy of one frame, the kernels of others and the read-back of finished ones overlap
// (paper, Section 3.4: asynchronous mode, frames processed in constant time; Section 4.2: video throughput).
//
// Copies are carried out by the DMA engine; a lane's stream waits for the copy of the frame it is about to process.
// A process has four hardware queues here, each taking its packets in order: one serves the default stream, the
// streams a process creates share the other three.  Hence at most three lanes however many slots the ring has (a
// fourth compute stream shares a queue with another lane and costs a sixth of the throughput), and hence the copies are
// enqueued on the default stream: on a stream of the ring's own they share a queue with one of the lanes, whose kernels
// then wait behind the marker of a copy that they do not depend on (measured on 4K frames in the paper's geometry:
// 6,180 frames/s with the copies on the default stream whatever else the process had created, 3,100 to 6,180 on a
// stream of the ring's own, depending on which queue it was given).  The lanes' streams do not synchronise with the
// default stream.  With three lanes and four slots the next frame has arrived on the device by the time a lane
// becomes free.  A lane's
// results live in its context until they are fetched, so a frame waits (copied in) until a fetch frees a lane; if the
// caller asks for a waiting frame first, results of running ones are set aside in host memory to make room.
// With graphs on, the per-frame sequence (every kernel of the path, results out) is captured once per slot and lane and
// replayed with one launch per frame; the copy in front of it is never captured: as a graph node it would be carried out
// by a copy kernel on the compute units (250 us for a 4K frame next to the other lanes' kernels instead of 150 us of DMA).
#include <string.h>

#include <algorithm>
#include <new>
#include <string>
#include <vector>

#include "cnnc_internal.h"

namespace {

constexpr int kMaxDepth = 16;
constexpr int kLanes = 3;          // compute streams that do not share a hardware queue
const hipStream_t kCopyStream = nullptr;       // the default stream: a hardware queue that no lane shares

enum SlotState { FREE, WAITING, RUNNING, SET_ASIDE };

struct Slot {
    uint8_t *h_frame = nullptr;   // pinned, w * h bytes, row pitch w
    uint8_t *d_frame = nullptr;
    hipEvent_t copied = nullptr;  // the frame has arrived in d_frame
    hipGraph_t graph[kLanes] = {};         // the path on this slot's device frame, captured on each lane's stream
    hipGraphExec_t exec[kLanes] = {};
    const uint8_t *ext_frame = nullptr;    // a frame of the caller's that is on the device already (cnnc_pipe_submit_device)
    int ext_pitch = 0;
    SlotState state = FREE;
    int lane = -1;                // while RUNNING
    int64_t ticket = -1;
    // results taken out of a lane's context before the caller asked for them (SET_ASIDE)
    std::vector<unsigned char> held;
    int held_n = 0, held_rc = CNNC_OK;
    std::string held_err;
};

// The path on a device frame of the caller's, captured per frame address and lane.
struct FrameGraph {
    const uint8_t *d_frame = nullptr;
    int pitch = 0, lane = 0;
    hipGraph_t graph = nullptr;
    hipGraphExec_t exec = nullptr;
};
constexpr size_t kMaxFrameGraphs = 48;       // (address, lane) pairs beyond that many run without a graph

struct Lane {
    cnnc_ctx *ctx = nullptr;
    hipStream_t st = nullptr;
    int running = -1;             // slot whose frame the context is processing or holds the results of
    int runs = 0;                 // frames this lane has processed since its parameters last changed
};

}  // namespace

struct cnnc_pipe {
    std::vector<Slot> slots;
    std::vector<Lane> lanes;
    std::vector<int> waiting;      // slots whose frames are copied in (or on their way) and wait for a lane, in submit order
    std::vector<FrameGraph> frame_graphs;
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
        if (s.state == FREE && (!best || s.ticket < best->ticket)) best = &s;
    return best;
}

bool in_flight(const cnnc_pipe *p)
{
    for (const Slot &s : p->slots)
        if (s.state != FREE) return true;
    return false;
}

void drop_frame_graphs(cnnc_pipe *p)
{
    for (FrameGraph &g : p->frame_graphs) {
        if (g.exec) (void)hipGraphExecDestroy(g.exec);
        if (g.graph) (void)hipGraphDestroy(g.graph);
    }
    p->frame_graphs.clear();
}

void drop_graphs(Slot &s)
{
    for (int l = 0; l < kLanes; ++l) {
        if (s.exec[l]) { (void)hipGraphExecDestroy(s.exec[l]); s.exec[l] = nullptr; }
        if (s.graph[l]) { (void)hipGraphDestroy(s.graph[l]); s.graph[l] = nullptr; }
    }
}

// The whole path + results out for the frame in slot s, on the lane's stream.
int enqueue_path(cnnc_pipe *p, Lane &l, Slot &s)
{
    const uint8_t *frame = s.ext_frame ? s.ext_frame : s.d_frame;
    const int pitch = s.ext_frame ? s.ext_pitch : p->w;
    const int rc = p->paper ? cnnc_detect_paper_async(l.ctx, frame, p->w, p->h, pitch, &p->pp, l.st)
                            : cnnc_detect_async(l.ctx, frame, p->w, p->h, pitch, l.st);
    if (rc) return pfail(p, rc, std::string("detect: ") + cnnc_last_error(l.ctx));
    return CNNC_OK;
}

// Give the frames that wait to the lanes that are free, oldest first.
int dispatch(cnnc_pipe *p)
{
    for (size_t li = 0; li < p->lanes.size() && !p->waiting.empty(); ++li) {
        Lane &l = p->lanes[li];
        if (l.running >= 0) continue;
        const int si = p->waiting.front();
        Slot &s = p->slots[(size_t)si];
        if (!s.ext_frame) PIPE_HIP(p, hipStreamWaitEvent(l.st, s.copied, 0));
        int rc = CNNC_OK;
        hipGraphExec_t *exec = &s.exec[li];
        hipGraph_t *graph = &s.graph[li];
        bool eager = !p->use_graph || l.runs == 0;               // a lane's first frame always is, so that every table and
                                                                 // buffer exists before a capture
        if (!eager && s.ext_frame) {                             // graphs of the caller's frames: by address and lane
            FrameGraph *fg = nullptr;
            for (FrameGraph &g : p->frame_graphs)
                if (g.d_frame == s.ext_frame && g.pitch == s.ext_pitch && g.lane == (int)li) fg = &g;
            if (!fg && p->frame_graphs.size() < kMaxFrameGraphs) {
                FrameGraph g;
                g.d_frame = s.ext_frame; g.pitch = s.ext_pitch; g.lane = (int)li;
                p->frame_graphs.push_back(g);
                fg = &p->frame_graphs.back();
            }
            if (fg) { exec = &fg->exec; graph = &fg->graph; }
            else eager = true;                                   // more frame addresses than graphs are kept for
        }
        if (eager) {
            rc = enqueue_path(p, l, s);
        } else {
            if (!*exec) {
                PIPE_HIP(p, hipStreamBeginCapture(l.st, hipStreamCaptureModeThreadLocal));
                rc = enqueue_path(p, l, s);
                hipGraph_t g = nullptr;
                const hipError_t e = hipStreamEndCapture(l.st, &g);
                if (rc == CNNC_OK && e != hipSuccess) rc = pfail(p, CNNC_E_HIP, std::string("hipStreamEndCapture: ") + hipGetErrorString(e));
                if (rc) { if (g) (void)hipGraphDestroy(g); return rc; }
                const hipError_t ei = hipGraphInstantiate(exec, g, nullptr, nullptr, 0);
                if (ei != hipSuccess) {
                    (void)hipGraphDestroy(g);
                    *exec = nullptr;
                    return pfail(p, CNNC_E_HIP, std::string("hipGraphInstantiate: ") + hipGetErrorString(ei));
                }
                *graph = g;
            }
            PIPE_HIP(p, hipGraphLaunch(*exec, l.st));
            l.ctx->last_stream = l.st;                           // what the captured calls would have noted: the fetch waits for it
        }
        if (rc) return rc;
        p->waiting.erase(p->waiting.begin());
        l.running = si;
        ++l.runs;
        s.lane = (int)li;
        s.state = RUNNING;
    }
    return CNNC_OK;
}

// Results of the lane's running frame into `out` (cnnc_det or cnnc_rdet records, by the pipe's path); the context is
// free afterwards whatever the outcome.
int take_results(cnnc_pipe *p, Lane &l, void *out, int cap, int *n_out)
{
    const int rc = p->paper ? cnnc_fetch_paper(l.ctx, static_cast<cnnc_rdet *>(out), cap, n_out)
                            : cnnc_fetch_detections(l.ctx, static_cast<cnnc_det *>(out), cap, n_out);
    l.running = -1;
    return rc;
}

int fetch_ticket(cnnc_pipe *p, int64_t ticket, void *out, int cap, int *n_out)
{
    const size_t rec = p->paper ? sizeof(cnnc_rdet) : sizeof(cnnc_det);
    for (Slot &s : p->slots) {
        if (s.state == FREE || s.ticket != ticket) continue;
        int rc = CNNC_OK;
        if (s.state == SET_ASIDE) {
            *n_out = s.held_n;
            rc = s.held_rc;
            if (rc) p->err = s.held_err;
            else {
                const size_t n = (size_t)std::min(s.held_n, cap);
                if (n) memcpy(out, s.held.data(), rec * n);
                if (s.held_n > cap) rc = pfail(p, CNNC_E_OVERFLOW, "output array too small");
            }
            s.held.clear();
            s.state = FREE;
            return rc;
        }
        // asked for while it waits for a lane: make room by setting aside the results of the oldest running frame
        while (s.state == WAITING) {
            if ((rc = dispatch(p))) return rc;
            if (s.state != WAITING) break;
            Lane *old = nullptr;
            for (Lane &l : p->lanes)
                if (l.running >= 0 && (!old || p->slots[(size_t)l.running].ticket < p->slots[(size_t)old->running].ticket)) old = &l;
            if (!old) return pfail(p, CNNC_E_STATE, "a frame waits although no lane is busy");
            Slot &e = p->slots[(size_t)old->running];
            const int cap_all = old->ctx->merge_cap;
            e.held.resize(rec * (size_t)cap_all);
            e.held_n = 0;
            e.held_rc = take_results(p, *old, e.held.data(), cap_all, &e.held_n);
            e.held_err = e.held_rc ? cnnc_last_error(old->ctx) : "";
            e.held.resize(rec * (size_t)(e.held_rc ? 0 : e.held_n));
            e.state = SET_ASIDE;
        }
        Lane &l = p->lanes[(size_t)s.lane];
        rc = take_results(p, l, out, cap, n_out);
        if (rc) pfail(p, rc, cnnc_last_error(l.ctx));
        s.state = FREE;
        const int rd = dispatch(p);                              // a waiting frame has been copied in meanwhile
        return rc ? rc : rd;
    }
    return pfail(p, CNNC_E_INVAL, "no frame in flight has this ticket");
}

}  // namespace

extern "C" {

int cnnc_pipe_destroy(cnnc_pipe *p)
{
    if (!p) return CNNC_OK;
    for (Slot &s : p->slots)
        if (s.copied && s.state != FREE) (void)hipEventSynchronize(s.copied);      // a copy may still be reading the pinned frame
    for (Lane &l : p->lanes)
        if (l.st) (void)hipStreamSynchronize(l.st);
    drop_frame_graphs(p);
    for (Slot &s : p->slots) {
        drop_graphs(s);
        if (s.copied) (void)hipEventDestroy(s.copied);
        if (s.h_frame) (void)hipHostFree(s.h_frame);
        if (s.d_frame) (void)hipFree(s.d_frame);
    }
    for (Lane &l : p->lanes) {
        if (l.ctx) (void)cnnc_destroy(l.ctx);
        if (l.st) (void)hipStreamDestroy(l.st);
    }
    delete p;
    return CNNC_OK;
}

int cnnc_pipe_create(cnnc_pipe **out, const cnnc_stage_desc stages[3], int w, int h, int max_survivors, int depth,
                     int use_graph)
{
    if (!out) return CNNC_E_INVAL;
    *out = nullptr;
    if (!stages || depth < 1 || depth > kMaxDepth || w < CNNC_WINDOW || h < CNNC_WINDOW) return CNNC_E_INVAL;
    cnnc_pipe *p = new (std::nothrow) cnnc_pipe();
    if (!p) return CNNC_E_NOMEM;
    p->w = w; p->h = h; p->use_graph = use_graph != 0;
    p->slots.resize((size_t)depth);
    p->lanes.resize((size_t)std::min(depth, kLanes));
    int rc = CNNC_OK;
    for (size_t i = 0; !rc && i < p->lanes.size(); ++i) {
        Lane &l = p->lanes[i];
        if ((rc = cnnc_create(&l.ctx, stages, w, h, max_survivors))) break;
        if (hipStreamCreateWithFlags(&l.st, hipStreamNonBlocking) != hipSuccess) rc = CNNC_E_HIP;
    }
    for (size_t i = 0; !rc && i < p->slots.size(); ++i) {
        Slot &s = p->slots[i];
        if (hipEventCreateWithFlags(&s.copied, hipEventDisableTiming) != hipSuccess) { rc = CNNC_E_HIP; break; }
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
    if (in_flight(p)) return pfail(p, CNNC_E_STATE, "frames are still in flight: fetch them before changing parameters");
    for (Lane &l : p->lanes) {
        const int rc = cnnc_set_params(l.ctx, prm);
        if (rc) return pfail(p, rc, cnnc_last_error(l.ctx));
        l.runs = 0;
    }
    for (Slot &s : p->slots) drop_graphs(s);       // thresholds and geometry are baked into the captured launches
    drop_frame_graphs(p);
    return CNNC_OK;
}

int cnnc_pipe_set_paper(cnnc_pipe *p, const float *scan_w, int n_scan, int scan_act, const float *w2, int n2, const float *w3,
                        int n3, int sel_act, int rule, const cnnc_paper_params *pp)
{
    if (!p || !pp) return CNNC_E_INVAL;
    if (in_flight(p)) return pfail(p, CNNC_E_STATE, "frames are still in flight: fetch them before changing the path");
    for (Lane &l : p->lanes) {
        int rc = cnnc_scan_set_weights(l.ctx, scan_w, n_scan, scan_act);
        if (!rc) rc = cnnc_select_set_weights(l.ctx, w2, n2, w3, n3, sel_act);
        if (!rc) rc = cnnc_select_set_rule(l.ctx, rule);
        if (rc) return pfail(p, rc, cnnc_last_error(l.ctx));
        l.runs = 0;
    }
    for (Slot &s : p->slots) drop_graphs(s);       // another sequence of launches; thresholds are baked into a captured one
    drop_frame_graphs(p);
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

// The slot joins the frames that wait for a lane and gets its ticket; a free lane takes it at once.
static int enter_ring(cnnc_pipe *p, Slot &s, int64_t *ticket)
{
    const int si = (int)(&s - p->slots.data());
    p->waiting.push_back(si);
    s.state = WAITING;
    s.ticket = p->next_ticket++;
    *ticket = s.ticket;
    const int rc = dispatch(p);
    if (rc && s.state == WAITING) {                              // could not be started: the slot is free again
        p->waiting.erase(std::find(p->waiting.begin(), p->waiting.end(), si));
        s.state = FREE;
    }
    return rc;
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
    PIPE_HIP(p, hipMemcpyAsync(s.d_frame, s.h_frame, (size_t)p->w * p->h, hipMemcpyHostToDevice, kCopyStream));
    PIPE_HIP(p, hipEventRecord(s.copied, kCopyStream));
    s.ext_frame = nullptr;
    return enter_ring(p, s, ticket);
}

int cnnc_pipe_submit_device(cnnc_pipe *p, const uint8_t *d_frame, int pitch, int64_t *ticket)
{
    if (!p || !ticket) return CNNC_E_INVAL;
    if (!d_frame || pitch < p->w) return pfail(p, CNNC_E_INVAL, "null frame or pitch < width");
    Slot *fs = free_slot(p);
    if (!fs) return pfail(p, CNNC_E_STATE, "every slot is in flight: fetch a frame first");
    fs->ext_frame = d_frame;
    fs->ext_pitch = pitch;
    return enter_ring(p, *fs, ticket);
}

int cnnc_pipe_fetch(cnnc_pipe *p, int64_t ticket, cnnc_det *out, int cap, int *n_out)
{
    if (!p || !n_out || (!out && cap > 0) || cap < 0) return CNNC_E_INVAL;
    if (p->paper) return pfail(p, CNNC_E_STATE, "this pipe runs the paper-geometry path: use cnnc_pipe_fetch_paper");
    return fetch_ticket(p, ticket, out, cap, n_out);
}

int cnnc_pipe_fetch_paper(cnnc_pipe *p, int64_t ticket, cnnc_rdet *out, int cap, int *n_out)
{
    if (!p || !n_out || (!out && cap > 0) || cap < 0) return CNNC_E_INVAL;
    if (!p->paper) return pfail(p, CNNC_E_STATE, "cnnc_pipe_set_paper has not been called");
    return fetch_ticket(p, ticket, out, cap, n_out);
}

const char *cnnc_pipe_last_error(const cnnc_pipe *p) { return p ? p->err.c_str() : "null pipe"; }

}  // extern "C"
