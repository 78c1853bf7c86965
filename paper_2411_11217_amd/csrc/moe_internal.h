// Internal declarations shared by the translation units of the MoE library.
// Nothing here is part of the C ABI (that is include/moe.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "moe.h"
#include "moe_host.h"

namespace moe {

// The layer with all pages resident, enqueued on st (arguments already validated).
size_t layer_workspace_bytes(const moe_shape& s);
int layer_resident(const moe_shape& s, const void* x, const void* Wr, const float* bias, const int32_t* page_table,
                   const char* page_pool, int64_t pool_pages, float* y, char* workspace, hipStream_t st);

// thread-local record of the last failing HIP call
void set_hip_error(hipError_t e);
#define MOE_HIP_TRY(expr)                               \
    do {                                                \
        hipError_t _e = (expr);                         \
        if (_e != hipSuccess) {                         \
            ::moe::set_hip_error(_e);                   \
            return MOE_ERR_HIP;                         \
        }                                               \
    } while (0)

int get_opt(int id);
enum Opt { OPT_XCD_REMAP = 0, OPT_PROFILE, OPT_DOWN_COLS, OPT_HALF_TILES, OPT_FUSE_GATHER, OPT_TALL_TILES, OPT_TALL_FIRST, OPT_CHUNKED, OPT_BALANCE, OPT_GATE_COLS, OPT_COUNT };

// ---- kernel launchers (each returns MOE_OK or MOE_ERR_HIP) -----------------
int launch_route(const moe_shape& s, const void* x, const void* Wr, const float* bias,
                 int32_t* ids, float* w, float* logits, hipStream_t st);

size_t permute_workspace_bytes(const moe_shape& s);
int launch_permute(const moe_shape& s, const int32_t* ids, const float* topk_w, const void* x,
                   int32_t* counts, int32_t* offsets, int32_t* row_src, int32_t* row_of,
                   float* row_w, void* x_perm, void* ws, int32_t* status_to_clear, hipStream_t st);   // status_to_clear: int32[4] zeroed by the index kernels, or null

struct FfnArgs {
    const void* x_perm;        // dtype [R][H]
    const int32_t* offsets;    // [E+1]
    const int32_t* page_table; // [table_experts][ppe]; row used for expert e is (e & table_mask_or_all)
    const char* pool;
    int64_t pool_pages;
    const float* row_w;        // [R] or null
    void* h;                   // dtype [R][F]
    float* out;                // [R][H]
    int32_t* status;           // [4] or null
    int e_begin, e_end;        // experts processed by this launch
    int table_row_mod;         // 0: table row = e; n>0: table row = e % n (streamed slots)
    hipEvent_t mid_event;      // recorded between the gate/up and the down launch when not null
    const int32_t* gather_src = nullptr;   // bf16 only.  Not null: x_perm is x [T][H], and row r reads x[gather_src[r] / k]
};
int launch_expert_ffn(const moe_shape& s, const FfnArgs& a, hipStream_t st);
int launch_expert_ffn_bf16(const moe_shape& s, const Geom& g, const FfnArgs& a, hipStream_t st);
int launch_expert_ffn_f32(const moe_shape& s, const Geom& g, const FfnArgs& a, hipStream_t st);

// Dense y = x W^T over paged weights (bf16 in, f32 out); offsets: device int32[2] = {0, T}.
struct LinearArgs {
    const void* x;             // bf16 [T][K]
    int T, K, N;
    const int32_t* offsets;
    const int32_t* page_table; // device [pages]
    const char* pool;
    int64_t pool_pages, page_bytes, pages;
    float* out;                // [T][N]
    int32_t* status;           // [4] or null
};
int launch_linear_bf16(const LinearArgs& a, hipStream_t st);

int launch_combine(const moe_shape& s, const float* out, const int32_t* row_of, const float* topk_w,
                   float* y, hipStream_t st);

}  // namespace moe
