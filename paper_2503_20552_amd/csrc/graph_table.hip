// Table of pre-recorded decode steps (Sec. 3.2.2, "Kernel Pre-launching"): launching the executor's
// kernels one by one costs more CPU time than they take on the GPU, so a step -- every layer's
// append, attention and merge -- is recorded once per batch capacity on an interval grid and a
// batch of n rows replays the smallest capacity that holds it, its surplus rows being padded rows
// (seq_len 0: no append, no cache read, a zero output row).
//
// Host code only.  The recorded work is the public adr_decode_step, captured from the given
// stream; what is replayed is therefore exactly what an eager call enqueues.
#include "../../include/adr.h"

#include <hip/hip_runtime.h>

#include <new>
#include <vector>

struct adr_graph_table {
    int interval = 0;
    int max_capacity = 0;
    std::vector<hipGraph_t> graphs;         // index c: capacity (c + 1) * interval
    std::vector<hipGraphExec_t> executables;
};

namespace {
void release(adr_graph_table *t)
{
    for (hipGraphExec_t e : t->executables)
        if (e)
            (void)hipGraphExecDestroy(e);
    for (hipGraph_t g : t->graphs)
        if (g)
            (void)hipGraphDestroy(g);
    delete t;
}
} // namespace

extern "C" {

int adr_graph_table_create(adr_graph_table **table, const adr_step_buffers *b, int interval, int max_capacity,
                           void *capture_stream)
{
    if (!table || !b || !b->caches || !capture_stream)
        return ADR_ERR_NULL; // (a recording needs a stream of its own: the default stream cannot record)
    *table = nullptr;
    if (interval <= 0 || max_capacity < interval || max_capacity % interval != 0 || b->n_layers <= 0)
        return ADR_ERR_SHAPE;
    adr_graph_table *t = new (std::nothrow) adr_graph_table;
    if (!t)
        return ADR_ERR_LAUNCH;
    t->interval = interval;
    t->max_capacity = max_capacity;
    hipStream_t stream = (hipStream_t)capture_stream;
    for (int capacity = interval; capacity <= max_capacity; capacity += interval) {
        // Arguments are checked by the first eager-style call below; a rejected call records nothing.
        if (hipStreamBeginCapture(stream, hipStreamCaptureModeThreadLocal) != hipSuccess) {
            release(t);
            return ADR_ERR_LAUNCH;
        }
        int rc = ADR_OK;
        for (int layer = 0; layer < b->n_layers && rc == ADR_OK; ++layer)
            rc = adr_decode_step(b->out, b->out_dtype, b->lse, b->q, b->q_row_stride, b->k_new, b->v_new,
                                 b->new_row_stride, &b->caches[layer], b->block_table, b->max_pages_per_req,
                                 b->seq_lens, capacity, b->Hq, b->scale, b->max_seq_len, b->partition_tokens,
                                 b->workspace, b->workspace_bytes, b->flags, capture_stream);
        hipGraph_t graph = nullptr;
        const hipError_t ended = hipStreamEndCapture(stream, &graph); // always, so that the stream leaves recording
        if (rc != ADR_OK || ended != hipSuccess || !graph) {
            if (graph)
                (void)hipGraphDestroy(graph);
            (void)hipGetLastError();
            release(t);
            return rc != ADR_OK ? rc : ADR_ERR_LAUNCH;
        }
        hipGraphExec_t exec = nullptr;
        if (hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0) != hipSuccess || !exec) {
            (void)hipGraphDestroy(graph);
            release(t);
            return ADR_ERR_LAUNCH;
        }
        t->graphs.push_back(graph);
        t->executables.push_back(exec);
    }
    *table = t;
    return ADR_OK;
}

int adr_graph_table_capacity(const adr_graph_table *table, int n_rows)
{
    if (!table)
        return -1;
    return adr_graph_capacity(n_rows, table->interval, table->max_capacity);
}

int adr_graph_table_launch(adr_graph_table *table, int n_rows, void *stream)
{
    if (!table)
        return ADR_ERR_NULL;
    const int capacity = adr_graph_capacity(n_rows, table->interval, table->max_capacity);
    if (capacity < 0)
        return ADR_ERR_SHAPE;
    const hipGraphExec_t exec = table->executables[(size_t)(capacity / table->interval - 1)];
    return hipGraphLaunch(exec, (hipStream_t)stream) == hipSuccess ? ADR_OK : ADR_ERR_LAUNCH;
}

int adr_graph_table_destroy(adr_graph_table *table)
{
    if (!table)
        return ADR_ERR_NULL;
    release(table);
    return ADR_OK;
}

} // extern "C"
