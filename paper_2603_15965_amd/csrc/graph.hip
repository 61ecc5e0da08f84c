// Replayable launch sequences (the paper's serving loop replays one captured graph per batch
// shape; Sec. "CUDA Graph Compatibility"): a thin layer over HIP stream capture, so that a
// caller without HIP bindings can record any sequence of molora_* calls once and replay it
// with a single launch.  All molora_* launches are capturable: they allocate nothing, never
// synchronise, read no device memory on the host and clear memory with kernels only; the one
// thing that is not a launch, the once-per-device set-up, is done before the capture begins.
#include "../../include/molora.h"

#include "common.h"

#include <new>

struct molora_graph {
    hipGraph_t graph;
    hipGraphExec_t exec;
};

extern "C" {

molora_status molora_graph_begin(void *stream) {
    if (stream == nullptr) return MOLORA_EINVAL;  // the null stream cannot be captured
    // the once-per-device set-up (function attributes) must not fall inside the capture
    if (molora::ensure_device_ready() != hipSuccess) return MOLORA_EHIP;
    const hipError_t e =
        hipStreamBeginCapture(static_cast<hipStream_t>(stream), hipStreamCaptureModeThreadLocal);
    return e == hipSuccess ? MOLORA_OK : MOLORA_EHIP;
}

molora_status molora_graph_end(void *stream, molora_graph **out) {
    if (stream == nullptr || out == nullptr) return MOLORA_EINVAL;
    *out = nullptr;
    hipGraph_t g = nullptr;
    if (hipStreamEndCapture(static_cast<hipStream_t>(stream), &g) != hipSuccess || g == nullptr) {
        (void)hipGetLastError();
        return MOLORA_EHIP;
    }
    hipGraphExec_t ex = nullptr;
    if (hipGraphInstantiate(&ex, g, nullptr, nullptr, 0) != hipSuccess) {
        (void)hipGetLastError();
        (void)hipGraphDestroy(g);
        return MOLORA_EHIP;
    }
    molora_graph *mg = new (std::nothrow) molora_graph{g, ex};
    if (mg == nullptr) {
        (void)hipGraphExecDestroy(ex);
        (void)hipGraphDestroy(g);
        return MOLORA_EHIP;
    }
    *out = mg;
    return MOLORA_OK;
}

molora_status molora_graph_launch(molora_graph *g, void *stream) {
    if (g == nullptr) return MOLORA_EINVAL;
    return hipGraphLaunch(g->exec, static_cast<hipStream_t>(stream)) == hipSuccess ? MOLORA_OK
                                                                                 : MOLORA_EHIP;
}

void molora_graph_destroy(molora_graph *g) {
    if (g == nullptr) return;
    (void)hipGraphExecDestroy(g->exec);
    (void)hipGraphDestroy(g->graph);
    delete g;
}

}  // extern "C"
