// Weight paging over a stack of MoE layers: the I/O side of the paper's pipeline
// (section 4.1, its paragraph on paging the weights and scheduling the transfers, and Algorithm 1; the
// double-buffered weight region of appendix A.1; the resident fraction r_w of
// section 4.2).  Host code only: it orders copies and layer calls on two streams.
//
// For layer l and its n micro-batches j = 0 .. n-1
//   copy stream   : hidden states of (l, j) host -> device      (the paper's transfer D2)
//                   chunk j of the non-resident pages of layer l+1  (transfer D3)
//   compute stream: the MoE layer l on micro-batch j, once its hidden states have arrived
// so the weights of the next layer arrive while the current layer computes, cut into as
// many chunks as there are micro-batches, and a small hidden-state copy never queues
// behind more than one chunk.  The chunks go into the half of a double buffer that the
// previous layer has finished with.  Layers are taken cyclically: during the last layer the
// first layer's pages are fetched for the next call (the next decode step).
#include <vector>

#include "moe_internal.h"

using namespace moe;

struct moe_pipeline {
    moe_shape shape;
    Geom geom;
    int32_t n_layers, max_micro, n_res, n_str;      // n_str = streamed pages per expert
    std::vector<const char*> host_pages;           // [L]
    std::vector<std::vector<int32_t>> host_tables;  // [L][E * ppe]
    char* pool;
    int64_t pool_pages;
    int32_t* device_tables;                         // device [L][2][E][ppe]
    int64_t stream_base[2];                         // first pool slot of each half of the double buffer
    int64_t seq;                                    // layers processed so far: layer number `seq` uses half seq & 1
    bool prefetched;                                // the half of layer `seq` already holds that layer's pages
    std::vector<hipEvent_t> x_ready, x_free;        // per micro-batch
    hipEvent_t w_ready[2], w_free[2];
};

namespace {

int64_t pipeline_pool_pages(const Geom& g, int E, int L, int n_res) {
    return (int64_t)L * E * n_res + 2 * (int64_t)E * (g.ppe - n_res);
}

// Copies streamed pages [first, last) of layer `layer` (in the order expert-major, page-minor) into
// buffer half `half`.  Runs that are consecutive on both sides go out as one copy.
int enqueue_chunk(moe_pipeline* p, int layer, int half, int64_t first, int64_t last, hipStream_t copy) {
    const int64_t pb = p->shape.page_bytes;
    const int32_t* table = p->host_tables[(size_t)layer].data();
    auto host_slot = [&](int64_t i) { return (int64_t)table[(i / p->n_str) * p->geom.ppe + p->n_res + i % p->n_str]; };
    int64_t i = first;
    while (i < last) {
        int64_t j = i + 1;
        while (j < last && host_slot(j) == host_slot(j - 1) + 1) ++j;      // device slots are consecutive in i
        MOE_HIP_TRY(hipMemcpyAsync(p->pool + (p->stream_base[half] + i) * pb, p->host_pages[(size_t)layer] + host_slot(i) * pb,
                                   (size_t)((j - i) * pb), hipMemcpyHostToDevice, copy));
        i = j;
    }
    return MOE_OK;
}

}  // namespace

extern "C" {

int moe_pipeline_pool_pages(const moe_shape* s, int32_t n_layers, int32_t resident_pages_per_expert, int64_t* pool_pages) {
    int rc = validate_shape(s);
    if (rc != MOE_OK) return rc;
    const Geom g = geometry(*s);
    if (!pool_pages || n_layers < 1 || resident_pages_per_expert < 0 || resident_pages_per_expert > g.ppe)
        return MOE_ERR_INVALID_ARG;
    *pool_pages = pipeline_pool_pages(g, s->E, n_layers, resident_pages_per_expert);
    return MOE_OK;
}

int moe_pipeline_create(const moe_shape* s, int32_t n_layers, int32_t max_micro_batches,
                        const void* const* host_pages, const int64_t* host_pool_pages,
                        const int32_t* const* host_page_tables, int32_t resident_pages_per_expert,
                        void* device_pool, int64_t device_pool_pages, int32_t* device_tables,
                        moe_pipeline** out) {
    int rc = validate_shape(s);
    if (rc != MOE_OK) return rc;
    const Geom g = geometry(*s);
    if (n_layers < 1 || max_micro_batches < 1 || !host_pages || !host_pool_pages || !host_page_tables || !device_pool ||
        !device_tables || !out || resident_pages_per_expert < 0 || resident_pages_per_expert > g.ppe)
        return MOE_ERR_INVALID_ARG;
    const int n_res = resident_pages_per_expert, n_str = (int)g.ppe - n_res, E = s->E;
    if (device_pool_pages < pipeline_pool_pages(g, E, n_layers, n_res)) return MOE_ERR_INVALID_ARG;
    for (int l = 0; l < n_layers; ++l) {
        if (!host_pages[l] || !host_page_tables[l] || host_pool_pages[l] <= 0) return MOE_ERR_INVALID_ARG;
        rc = check_table_host(*s, g, host_page_tables[l], host_pool_pages[l], false);
        if (rc != MOE_OK) return rc;
    }
    moe_pipeline* p = new moe_pipeline();
    p->shape = *s;
    p->geom = g;
    p->n_layers = n_layers;
    p->max_micro = max_micro_batches;
    p->n_res = n_res;
    p->n_str = n_str;
    p->pool = (char*)device_pool;
    p->pool_pages = device_pool_pages;
    p->device_tables = device_tables;
    p->stream_base[0] = (int64_t)n_layers * E * n_res;
    p->stream_base[1] = p->stream_base[0] + (int64_t)E * n_str;
    p->seq = 0;
    p->prefetched = false;
    // device tables: [layer][half][expert][page]; resident pages have a slot of their own
    std::vector<int32_t> tables((size_t)n_layers * 2 * E * g.ppe);
    const int64_t pb = s->page_bytes;
    for (int l = 0; l < n_layers; ++l) {
        p->host_pages.push_back((const char*)host_pages[l]);
        p->host_tables.emplace_back(host_page_tables[l], host_page_tables[l] + (int64_t)E * g.ppe);
        for (int half = 0; half < 2; ++half)
            for (int e = 0; e < E; ++e)
                for (int64_t pg = 0; pg < g.ppe; ++pg) {
                    const int64_t slot = pg < n_res ? ((int64_t)l * E + e) * n_res + pg
                                                    : p->stream_base[half] + (int64_t)e * n_str + (pg - n_res);
                    tables[(((size_t)l * 2 + half) * E + e) * g.ppe + pg] = (int32_t)slot;
                }
        // resident pages are placed once, here (not a hot call)
        for (int e = 0; e < E; ++e)
            for (int64_t pg = 0; pg < n_res; ++pg) {
                const int64_t hs = host_page_tables[l][(int64_t)e * g.ppe + pg];
                const hipError_t err = hipMemcpy(p->pool + (((int64_t)l * E + e) * n_res + pg) * pb,
                                                 p->host_pages[(size_t)l] + hs * pb, (size_t)pb, hipMemcpyHostToDevice);
                if (err != hipSuccess) {
                    set_hip_error(err);
                    delete p;
                    return MOE_ERR_HIP;
                }
            }
    }
    hipError_t err = hipMemcpy(device_tables, tables.data(), tables.size() * 4, hipMemcpyHostToDevice);
    p->x_ready.assign((size_t)max_micro_batches, nullptr);
    p->x_free.assign((size_t)max_micro_batches, nullptr);
    for (int j = 0; j < max_micro_batches && err == hipSuccess; ++j) {
        err = hipEventCreateWithFlags(&p->x_ready[(size_t)j], hipEventDisableTiming);
        if (err == hipSuccess) err = hipEventCreateWithFlags(&p->x_free[(size_t)j], hipEventDisableTiming);
    }
    for (int i = 0; i < 2; ++i) {
        p->w_ready[i] = p->w_free[i] = nullptr;
        if (err == hipSuccess) err = hipEventCreateWithFlags(&p->w_ready[i], hipEventDisableTiming);
        if (err == hipSuccess) err = hipEventCreateWithFlags(&p->w_free[i], hipEventDisableTiming);
    }
    if (err != hipSuccess) {
        set_hip_error(err);
        moe_pipeline_destroy(p);
        return MOE_ERR_HIP;
    }
    *out = p;
    return MOE_OK;
}

int moe_pipeline_destroy(moe_pipeline* p) {
    if (!p) return MOE_ERR_INVALID_ARG;
    for (hipEvent_t e : p->x_ready)
        if (e) (void)hipEventDestroy(e);
    for (hipEvent_t e : p->x_free)
        if (e) (void)hipEventDestroy(e);
    for (int i = 0; i < 2; ++i) {
        if (p->w_ready[i]) (void)hipEventDestroy(p->w_ready[i]);
        if (p->w_free[i]) (void)hipEventDestroy(p->w_free[i]);
    }
    delete p;
    return MOE_OK;
}

int moe_pipeline_run(moe_pipeline* p, int32_t n_micro, const void* const* x_host, void* x_dev,
                     const void* const* Wr, const float* const* bias, float* const* y,
                     void* workspace, size_t workspace_bytes, void* stream, void* copy_stream) {
    if (!p) return MOE_ERR_INVALID_ARG;
    const moe_shape& s = p->shape;
    if (n_micro < 1 || n_micro > p->max_micro || !x_host || !x_dev || !Wr || !y || !workspace || stream == copy_stream)
        return MOE_ERR_INVALID_ARG;
    if (s.T == 0) return MOE_OK;
    if (workspace_bytes < layer_workspace_bytes(s)) return MOE_ERR_WORKSPACE_TOO_SMALL;
    if (((uintptr_t)workspace & 255) != 0) return MOE_ERR_INVALID_ARG;
    const int L = p->n_layers, E = s.E;
    for (int i = 0; i < L * n_micro; ++i)
        if (!x_host[i] || !y[i]) return MOE_ERR_INVALID_ARG;
    for (int l = 0; l < L; ++l)
        if (!Wr[l]) return MOE_ERR_INVALID_ARG;
    hipStream_t comp = (hipStream_t)stream, copy = (hipStream_t)copy_stream;
    const int64_t x_bytes = (int64_t)s.T * s.H * p->geom.esize;
    const int64_t n_stream_pages = (int64_t)E * p->n_str;       // per layer
    const size_t table_stride = (size_t)E * p->geom.ppe;
    int rc;
    if (!p->prefetched && n_stream_pages > 0) {
        // cold start: nothing overlaps the first layer's pages
        const int half = (int)(p->seq & 1);
        MOE_HIP_TRY(hipStreamWaitEvent(copy, p->w_free[half], 0));
        rc = enqueue_chunk(p, 0, half, 0, n_stream_pages, copy);
        if (rc != MOE_OK) return rc;
        MOE_HIP_TRY(hipEventRecord(p->w_ready[half], copy));
    }
    for (int l = 0; l < L; ++l) {
        const int half = (int)((p->seq + l) & 1), other = half ^ 1;
        const int next_layer = (l + 1) % L;
        if (n_stream_pages > 0) {
            MOE_HIP_TRY(hipStreamWaitEvent(comp, p->w_ready[half], 0));   // this layer's pages have arrived
            MOE_HIP_TRY(hipStreamWaitEvent(copy, p->w_free[other], 0));   // the layer before has left the other half
        }
        const int32_t* table = p->device_tables + ((size_t)l * 2 + half) * table_stride;
        for (int j = 0; j < n_micro; ++j) {
            // D2: hidden states of (l, j); the staging row is free once the layer call that read it is done
            MOE_HIP_TRY(hipStreamWaitEvent(copy, p->x_free[(size_t)j], 0));
            char* xj = (char*)x_dev + (int64_t)j * x_bytes;
            MOE_HIP_TRY(hipMemcpyAsync(xj, x_host[(size_t)l * n_micro + j], (size_t)x_bytes, hipMemcpyHostToDevice, copy));
            MOE_HIP_TRY(hipEventRecord(p->x_ready[(size_t)j], copy));
            // D3: chunk j of the next layer's pages
            if (n_stream_pages > 0) {
                rc = enqueue_chunk(p, next_layer, other, n_stream_pages * j / n_micro, n_stream_pages * (j + 1) / n_micro, copy);
                if (rc != MOE_OK) return rc;
            }
            MOE_HIP_TRY(hipStreamWaitEvent(comp, p->x_ready[(size_t)j], 0));
            rc = layer_resident(s, xj, Wr[l], bias ? bias[l] : nullptr, table, p->pool, p->pool_pages,
                                y[(size_t)l * n_micro + j], (char*)workspace, comp);
            if (rc != MOE_OK) return rc;
            MOE_HIP_TRY(hipEventRecord(p->x_free[(size_t)j], comp));
        }
        if (n_stream_pages > 0) {
            MOE_HIP_TRY(hipEventRecord(p->w_ready[other], copy));
            MOE_HIP_TRY(hipEventRecord(p->w_free[half], comp));
        }
    }
    p->seq += L;
    p->prefetched = true;
    return MOE_OK;
}

}  // extern "C"
