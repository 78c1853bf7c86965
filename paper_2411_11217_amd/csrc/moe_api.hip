// Host side of the C ABI: argument checks, page geometry, the weight packer,
// workspace layout, and the entry points that enqueue the kernels.
#include <algorithm>
#include <cstring>
#include <thread>
#include <vector>

#include "moe_internal.h"

namespace moe {

static thread_local int g_last_hip_error = 0;
void set_hip_error(hipError_t e) { g_last_hip_error = (int)e; }

// ---- options ----------------------------------------------------------------
static int g_opts[OPT_COUNT] = {
    /*OPT_XCD_REMAP*/ 1,     // 1: the column tiles of the expert GEMMs are dealt round robin to the 8 XCDs
    /*OPT_PROFILE*/ 0,       // 1: moe_layer records stage events (see moe_profile_read)
    /*OPT_DOWN_COLS*/ 0,     // column tiles of the bf16 down GEMM: 0 = by grid size, 1 = 128 wide, 2 = 256 wide
    /*OPT_HALF_TILES*/ 1,    // 1: bf16 row tiles with at most 128 rows run the half-height loop
    /*OPT_FUSE_GATHER*/ 1,   // 1: the bf16 gate/up GEMM of moe_layer reads the rows of x through row_src (no x_perm copy)
    /*OPT_TALL_TILES*/ 1,    // 1: bf16: row tiles may be up to 32 rows higher than 256 (a small remainder needs no tile of its own)
    /*OPT_TALL_FIRST*/ 1,    // 1: bf16 tile numbering: inside a chunk of column-tile groups the tall row tiles come first
    /*OPT_CHUNKED*/ 32,      // tile numbering: the column-tile groups of an expert go to the XCDs in chunks of about this many tiles (at most 32; 0: single groups)
    /*OPT_BALANCE*/ 1,       // 1: an XCD with more than an eighth of a launch's tiles gives the rest to XCDs with fewer
    /*OPT_GATE_COLS*/ 0,     // column tiles of the bf16 gate/up GEMM: 0 = by grid size, 1 = 64 features wide, 2 = 128 features wide
};
static const char* g_opt_names[OPT_COUNT] = {"xcd_remap", "profile", "down_cols", "half_tiles", "fuse_gather", "tall_tiles", "tall_first", "chunked", "balance", "gate_cols"};
int get_opt(int id) { return g_opts[id]; }

static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

static int layout(const moe_shape& s, moe_workspace_layout* L) {
    const Geom g = geometry(s);
    const size_t R = (size_t)s.T * s.k, A = 256;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + std::max<size_t>(bytes, 4), A); return o; };
    L->status = take(16);
    L->topk_ids = take(R * 4);
    L->topk_w = take(R * 4);
    L->counts = take((size_t)s.E * 4);
    L->offsets = take((size_t)(s.E + 1) * 4);
    L->row_src = take(R * 4);
    L->row_of = take(R * 4);
    L->row_w = take(R * 4);
    L->permute_bytes = permute_workspace_bytes(s);
    L->scan = take(L->permute_bytes);
    L->x_perm = take(R * s.H * g.esize);
    L->h = take(R * s.F * g.esize);
    L->out = take(R * s.H * 4);
    L->total = off;
    return MOE_OK;
}

// ---- stage timing ---------------------------------------------------------------
struct Profiler {
    bool ready = false;
    hipEvent_t ev[MOE_PROFILE_RING][MOE_PROFILE_STAGES + 1];
    int next = 0, count = 0;
};
static Profiler g_prof;

// Creates the ring of stage events once (called from moe_set_option("profile", 1): the hot calls never create any).
static int prof_prepare() {
    if (g_prof.ready) return MOE_OK;
    for (int i = 0; i < MOE_PROFILE_RING; ++i)
        for (int j = 0; j <= MOE_PROFILE_STAGES; ++j) {
            const hipError_t e = hipEventCreate(&g_prof.ev[i][j]);
            if (e != hipSuccess) {                  // give back what was created
                for (int q = 0; q < i * (MOE_PROFILE_STAGES + 1) + j; ++q)
                    (void)hipEventDestroy(g_prof.ev[q / (MOE_PROFILE_STAGES + 1)][q % (MOE_PROFILE_STAGES + 1)]);
                set_hip_error(e);
                return MOE_ERR_HIP;
            }
        }
    g_prof.ready = true;
    return MOE_OK;
}

static int prof_slot() {
    if (!g_opts[OPT_PROFILE] || !g_prof.ready) return -1;
    const int slot = g_prof.next;
    g_prof.next = (g_prof.next + 1) % MOE_PROFILE_RING;
    if (g_prof.count < MOE_PROFILE_RING) ++g_prof.count;
    return slot;
}
static void prof_mark(int slot, int j, hipStream_t st) {
    if (slot >= 0) (void)hipEventRecord(g_prof.ev[slot][j], st);
}
static hipEvent_t prof_event(int slot, int j) { return slot >= 0 ? g_prof.ev[slot][j] : nullptr; }

// The body of the layer on one stream; `ffn` runs the expert FFN stage.
template <class FfnFn>
static int layer_body(const moe_shape& s, const void* x, const void* Wr, const float* bias, float* y,
                      char* ws, hipStream_t st, FfnFn ffn) {
    moe_workspace_layout L;
    layout(s, &L);
    int32_t* status = (int32_t*)(ws + L.status);
    int32_t* ids = (int32_t*)(ws + L.topk_ids);
    float* w = (float*)(ws + L.topk_w);
    int32_t* counts = (int32_t*)(ws + L.counts);
    int32_t* offsets = (int32_t*)(ws + L.offsets);
    int32_t* row_src = (int32_t*)(ws + L.row_src);
    int32_t* row_of = (int32_t*)(ws + L.row_of);
    float* row_w = (float*)(ws + L.row_w);
    const int ps = prof_slot();
    prof_mark(ps, 0, st);
    int rc = launch_route(s, x, Wr, bias, ids, w, nullptr, st);
    if (rc != MOE_OK) return rc;
    prof_mark(ps, 1, st);
    // bf16: the gate/up GEMM gathers the rows of x by itself (32-bit byte offsets into x), and x_perm stays unwritten
    const bool fuse = s.dtype == MOE_DTYPE_BF16 && get_opt(OPT_FUSE_GATHER) && (int64_t)s.T * s.H * 2 < ((int64_t)1 << 32);
    rc = launch_permute(s, ids, w, fuse ? nullptr : x, counts, offsets, row_src, row_of, row_w,
                        fuse ? nullptr : ws + L.x_perm, ws + L.scan, status, st);   // also clears the status words (in a kernel: the call can be graph-captured)
    if (rc != MOE_OK) return rc;
    prof_mark(ps, 2, st);
    rc = ffn(fuse ? x : ws + L.x_perm, fuse ? row_src : nullptr, offsets, row_w, ws + L.h, (float*)(ws + L.out), status,
             prof_event(ps, 3));
    if (rc != MOE_OK) return rc;
    prof_mark(ps, 4, st);
    // the gate weight was applied in the down-projection epilogue: plain sum here
    rc = launch_combine(s, (const float*)(ws + L.out), row_of, nullptr, y, st);
    prof_mark(ps, 5, st);
    return rc;
}

size_t layer_workspace_bytes(const moe_shape& s) {
    moe_workspace_layout L;
    layout(s, &L);
    return L.total;
}

int layer_resident(const moe_shape& sh, const void* x, const void* Wr, const float* bias, const int32_t* page_table,
                   const char* page_pool, int64_t pool_pages, float* y, char* workspace, hipStream_t st) {
    return layer_body(sh, x, Wr, bias, y, workspace, st,
                      [&](const void* xp, const int32_t* gather_src, const int32_t* offsets, const float* row_w, void* h,
                          float* out, int32_t* status, hipEvent_t mid) {
                          FfnArgs a{xp, offsets, page_table, page_pool, pool_pages, row_w, h, out,
                                    status, 0, sh.E, 0, mid, gather_src};
                          return launch_expert_ffn(sh, a, st);
                      });
}

}  // namespace moe

using namespace moe;

extern "C" {

int moe_last_hip_error(void) { return g_last_hip_error; }

int moe_workspace_layout_get(const moe_shape* s, moe_workspace_layout* out) {
    int rc = validate_shape(s);
    if (rc != MOE_OK) return rc;
    if (!out) return MOE_ERR_INVALID_ARG;
    return layout(*s, out);
}

int moe_route(const moe_shape* s, const void* x, const void* Wr, const float* bias,
              int32_t* topk_ids, float* topk_w, float* logits, void* stream) {
    int rc = validate_shape(s);
    if (rc != MOE_OK) return rc;
    if (s->T == 0) return MOE_OK;
    if (!x || !Wr || !topk_ids || !topk_w) return MOE_ERR_INVALID_ARG;
    return launch_route(*s, x, Wr, bias, topk_ids, topk_w, logits, (hipStream_t)stream);
}

int moe_permute(const moe_shape* s, const int32_t* topk_ids, const float* topk_w, const void* x,
                int32_t* counts, int32_t* offsets, int32_t* row_src, int32_t* row_of,
                float* row_w, void* x_perm, void* workspace, size_t workspace_bytes, void* stream) {
    int rc = validate_shape(s);
    if (rc != MOE_OK) return rc;
    if (!counts || !offsets) return MOE_ERR_INVALID_ARG;
    if (s->T > 0 && (!topk_ids || !row_src || !row_of)) return MOE_ERR_INVALID_ARG;
    if ((x == nullptr) != (x_perm == nullptr)) return MOE_ERR_INVALID_ARG;
    if (row_w && !topk_w) return MOE_ERR_INVALID_ARG;
    if (!workspace) return MOE_ERR_INVALID_ARG;
    if (workspace_bytes < permute_workspace_bytes(*s)) return MOE_ERR_WORKSPACE_TOO_SMALL;
    return launch_permute(*s, topk_ids, topk_w, x, counts, offsets, row_src, row_of, row_w, x_perm,
                          workspace, nullptr, (hipStream_t)stream);
}

int moe_expert_ffn(const moe_shape* s, const void* x_perm, const int32_t* offsets,
                   const int32_t* page_table, const void* page_pool, int64_t pool_pages,
                   const float* row_w, void* h_ws, float* out, int32_t* status, void* stream) {
    int rc = validate_shape(s);
    if (rc != MOE_OK) return rc;
    if (s->T == 0) return MOE_OK;
    if (!x_perm || !offsets || !page_table || !page_pool || !h_ws || !out || pool_pages <= 0)
        return MOE_ERR_INVALID_ARG;
    FfnArgs a{x_perm, offsets, page_table, (const char*)page_pool, pool_pages, row_w, h_ws, out, status,
              0, s->E, 0, nullptr};
    return launch_expert_ffn(*s, a, (hipStream_t)stream);
}

int moe_combine(const moe_shape* s, const float* out, const int32_t* row_of,
                const float* topk_w, float* y, void* stream) {
    int rc = validate_shape(s);
    if (rc != MOE_OK) return rc;
    if (s->T == 0) return MOE_OK;
    if (!out || !row_of || !y) return MOE_ERR_INVALID_ARG;
    return launch_combine(*s, out, row_of, topk_w, y, (hipStream_t)stream);
}

int moe_layer(const moe_shape* s, const void* x, const void* Wr, const float* bias,
              const int32_t* page_table, const void* page_pool, int64_t pool_pages,
              float* y, void* workspace, size_t workspace_bytes, void* stream) {
    int rc = validate_shape(s);
    if (rc != MOE_OK) return rc;
    if (s->T == 0) return MOE_OK;
    if (!x || !Wr || !page_table || !page_pool || !y || !workspace || pool_pages <= 0)
        return MOE_ERR_INVALID_ARG;
    if (workspace_bytes < layer_workspace_bytes(*s)) return MOE_ERR_WORKSPACE_TOO_SMALL;
    if (((uintptr_t)workspace & 255) != 0) return MOE_ERR_INVALID_ARG;
    return layer_resident(*s, x, Wr, bias, page_table, (const char*)page_pool, pool_pages, y, (char*)workspace,
                          (hipStream_t)stream);
}

}  // extern "C"

// ---- the layer on the library's own scratch ----------------------------------------------
// The workspace of moe_layer_static: a file-scope device array, one copy per GPU the library runs on, held until
// the process ends.  In host code the array's name is only a stand-in; its device address is asked for once
// per device and kept in g_static_scratch[].
static __device__ __align__(256) char g_scratch_array[MOE_STATIC_SCRATCH_BYTES];
static constexpr int kMaxDevices = 64;
static char* g_static_scratch[kMaxDevices] = {};

// -> MOE_OK and *ptr = the device address of the current device's copy of the array
static int static_scratch(char** ptr) {
    int dev = -1;
    MOE_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return MOE_ERR_INVALID_ARG;
    if (!g_static_scratch[dev]) {
        void* p = nullptr;
        MOE_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(g_scratch_array)));
        if (!p || ((uintptr_t)p & 255) != 0) return MOE_ERR_INVALID_ARG;
        g_static_scratch[dev] = (char*)p;
    }
    *ptr = g_static_scratch[dev];
    return MOE_OK;
}

extern "C" {

int moe_layer_static(const moe_shape* s, const void* x, const void* Wr, const float* bias,
                     const int32_t* page_table, const void* page_pool, int64_t pool_pages,
                     float* y, void* stream) {
    int rc = validate_shape(s);
    if (rc != MOE_OK) return rc;
    if (s->T == 0) return MOE_OK;
    if (!x || !Wr || !page_table || !page_pool || !y || pool_pages <= 0) return MOE_ERR_INVALID_ARG;
    if (layer_workspace_bytes(*s) > (size_t)MOE_STATIC_SCRATCH_BYTES) return MOE_ERR_WORKSPACE_TOO_SMALL;
    char* ws = nullptr;
    rc = static_scratch(&ws);
    if (rc != MOE_OK) return rc;
    // everything that must start at zero (the status words) is cleared by the layer's own kernels
    return layer_resident(*s, x, Wr, bias, page_table, (const char*)page_pool, pool_pages, y, ws, (hipStream_t)stream);
}

int moe_set_option(const char* name, int value) {
    if (!name) return MOE_ERR_INVALID_ARG;
    for (int i = 0; i < OPT_COUNT; ++i)
        if (std::strcmp(name, g_opt_names[i]) == 0) {
            if (i == OPT_PROFILE && value) {        // the stage events are created here, not inside a layer call
                const int rc = prof_prepare();
                if (rc != MOE_OK) return rc;
            }
            g_opts[i] = value;
            return MOE_OK;
        }
    return MOE_ERR_INVALID_ARG;
}

int moe_profile_read(double* avg_ms, int* n_calls) {
    if (!avg_ms || !n_calls) return MOE_ERR_INVALID_ARG;
    for (int j = 0; j < MOE_PROFILE_STAGES; ++j) avg_ms[j] = 0.0;
    *n_calls = 0;
    if (!g_prof.ready || g_prof.count == 0) return MOE_OK;
    const int n = g_prof.count;
    for (int i = 0; i < n; ++i) {
        const int slot = ((g_prof.next - 1 - i) % MOE_PROFILE_RING + MOE_PROFILE_RING) % MOE_PROFILE_RING;
        for (int j = 0; j < MOE_PROFILE_STAGES; ++j) {
            float ms = 0.f;
            MOE_HIP_TRY(hipEventElapsedTime(&ms, g_prof.ev[slot][j], g_prof.ev[slot][j + 1]));
            avg_ms[j] += ms;
        }
    }
    for (int j = 0; j < MOE_PROFILE_STAGES; ++j) avg_ms[j] /= n;
    *n_calls = n;
    g_prof.count = 0;
    return MOE_OK;
}

int moe_get_option(const char* name, int* value) {
    if (!name || !value) return MOE_ERR_INVALID_ARG;
    for (int i = 0; i < OPT_COUNT; ++i)
        if (std::strcmp(name, g_opt_names[i]) == 0) {
            *value = g_opts[i];
            return MOE_OK;
        }
    return MOE_ERR_INVALID_ARG;
}

}  // extern "C"

// ---- streamed pages -------------------------------------------------------------
// One expert's pages are copied into slot (e & 1) on the copy stream while the
// GEMMs of expert e-1 read the other slot on the compute stream.
struct moe_streamer {
    moe_shape shape;
    Geom geom;
    const char* host_pages;
    std::vector<int32_t> host_table;   // [E][ppe]
    char* slots;
    int32_t* slot_table;               // device [2][ppe]
    hipEvent_t loaded[2];              // slot s holds the pages of its current expert
    hipEvent_t released[2];            // the GEMMs reading slot s have been enqueued and finished
    bool slot_used[2] = {false, false};   // released[s] has been recorded at least once (by this or an earlier call)
};

extern "C" {

int moe_stream_create(const moe_shape* s, const void* host_pages, int64_t host_pool_pages,
                      const int32_t* host_page_table, void* slots, int32_t* slot_table,
                      moe_streamer** out) {
    int rc = validate_shape(s);
    if (rc != MOE_OK) return rc;
    if (!host_pages || !host_page_table || !slots || !slot_table || !out || host_pool_pages <= 0)
        return MOE_ERR_INVALID_ARG;
    const Geom g = geometry(*s);
    rc = check_table_host(*s, g, host_page_table, host_pool_pages, false);
    if (rc != MOE_OK) return rc;
    std::vector<int32_t> st_host((size_t)2 * g.ppe);
    for (int sl = 0; sl < 2; ++sl)
        for (int64_t p = 0; p < g.ppe; ++p) st_host[(size_t)sl * g.ppe + p] = (int32_t)(sl * g.ppe + p);
    MOE_HIP_TRY(hipMemcpy(slot_table, st_host.data(), st_host.size() * 4, hipMemcpyHostToDevice));
    moe_streamer* st = new moe_streamer();
    st->shape = *s;
    st->geom = g;
    st->host_pages = (const char*)host_pages;
    st->host_table.assign(host_page_table, host_page_table + (int64_t)s->E * g.ppe);
    st->slots = (char*)slots;
    st->slot_table = slot_table;
    // the four events; on a failure those already created are destroyed and the record is freed
    hipEvent_t* evs[4] = {&st->loaded[0], &st->loaded[1], &st->released[0], &st->released[1]};
    for (int i = 0; i < 4; ++i) {
        const hipError_t e = hipEventCreateWithFlags(evs[i], hipEventDisableTiming);
        if (e != hipSuccess) {
            for (int q = 0; q < i; ++q) (void)hipEventDestroy(*evs[q]);
            delete st;
            set_hip_error(e);
            return MOE_ERR_HIP;
        }
    }
    *out = st;
    return MOE_OK;
}

int moe_stream_destroy(moe_streamer* st) {
    if (!st) return MOE_ERR_INVALID_ARG;
    for (int i = 0; i < 2; ++i) {
        (void)hipEventDestroy(st->loaded[i]);
        (void)hipEventDestroy(st->released[i]);
    }
    delete st;
    return MOE_OK;
}

}  // extern "C"

namespace moe {

// Enqueue the copies of expert e's pages into slot e&1.  Runs of pages that are
// consecutive in the host pool go out as one copy.
static int enqueue_expert_copy(moe_streamer* st, int e, hipStream_t copy) {
    const Geom& g = st->geom;
    const int64_t pb = st->shape.page_bytes;
    const int32_t* row = st->host_table.data() + (int64_t)e * g.ppe;
    char* dst = st->slots + (int64_t)(e & 1) * g.ppe * pb;
    int64_t p = 0;
    while (p < g.ppe) {
        int64_t q = p + 1;
        while (q < g.ppe && row[q] == row[q - 1] + 1) ++q;
        MOE_HIP_TRY(hipMemcpyAsync(dst + p * pb, st->host_pages + (int64_t)row[p] * pb, (size_t)((q - p) * pb),
                                   hipMemcpyHostToDevice, copy));
        p = q;
    }
    return MOE_OK;
}

static int ffn_streamed(moe_streamer* st, const void* x_perm, const int32_t* gather_src, const int32_t* offsets,
                        const float* row_w, void* h_ws, float* out, int32_t* status, hipStream_t comp, hipStream_t copy) {
    const moe_shape& s = st->shape;
    const Geom& g = st->geom;
    // A copy into a slot waits for the GEMMs that last read that slot and for nothing else - also across calls: the first
    // two copies of a call wait for the last users of their slots in the call before (not for that call's end), so in a
    // sequence of calls the first expert's pages travel while the last expert's GEMMs, the combine step and the next
    // call's routing run (the paper's double buffer, appendix A.1, carried over the call boundary).
    for (int e = 0; e < s.E; ++e) {
        const int sl = e & 1;
        if (st->slot_used[sl]) MOE_HIP_TRY(hipStreamWaitEvent(copy, st->released[sl], 0));
        int rc = enqueue_expert_copy(st, e, copy);
        if (rc != MOE_OK) return rc;
        MOE_HIP_TRY(hipEventRecord(st->loaded[sl], copy));
        MOE_HIP_TRY(hipStreamWaitEvent(comp, st->loaded[sl], 0));
        FfnArgs a{x_perm, offsets, st->slot_table, st->slots, 2 * g.ppe, row_w, h_ws, out, status, e, e + 1, 2, nullptr,
                  gather_src};
        rc = launch_expert_ffn(s, a, comp);
        if (rc != MOE_OK) return rc;
        MOE_HIP_TRY(hipEventRecord(st->released[sl], comp));
        st->slot_used[sl] = true;
    }
    return MOE_OK;
}

}  // namespace moe

extern "C" {

int moe_expert_ffn_streamed(moe_streamer* st, const void* x_perm, const int32_t* offsets,
                            const float* row_w, void* h_ws, float* out, int32_t* status,
                            void* stream, void* copy_stream) {
    if (!st) return MOE_ERR_INVALID_ARG;
    if (st->shape.T == 0) return MOE_OK;
    if (!x_perm || !offsets || !h_ws || !out || stream == copy_stream) return MOE_ERR_INVALID_ARG;
    return ffn_streamed(st, x_perm, nullptr, offsets, row_w, h_ws, out, status, (hipStream_t)stream, (hipStream_t)copy_stream);
}

int moe_layer_streamed(moe_streamer* st, const void* x, const void* Wr, const float* bias,
                       float* y, void* workspace, size_t workspace_bytes,
                       void* stream, void* copy_stream) {
    if (!st) return MOE_ERR_INVALID_ARG;
    const moe_shape sh = st->shape;
    if (sh.T == 0) return MOE_OK;
    if (!x || !Wr || !y || !workspace || stream == copy_stream) return MOE_ERR_INVALID_ARG;
    moe_workspace_layout L;
    layout(sh, &L);
    if (workspace_bytes < L.total) return MOE_ERR_WORKSPACE_TOO_SMALL;
    if (((uintptr_t)workspace & 255) != 0) return MOE_ERR_INVALID_ARG;
    hipStream_t comp = (hipStream_t)stream, copy = (hipStream_t)copy_stream;
    return layer_body(sh, x, Wr, bias, y, (char*)workspace, comp,
                      [&](const void* xp, const int32_t* gather_src, const int32_t* offsets, const float* row_w, void* h,
                          float* out, int32_t* status, hipEvent_t) {
                          return ffn_streamed(st, xp, gather_src, offsets, row_w, h, out, status, comp, copy);
                      });
}

}  // extern "C"
