// a2. Permutation of routed rows by expert: a stable counting sort of the flat
// indices i = t*k + slot by expert id, in two small kernels plus a row copy.
//
//   count   : every block owns kChunk consecutive flat indices; per wavefront
//             and per expert the population count of a ballot gives how many
//             of its 64 entries go to that expert; the counts are staged in LDS
//             and the block's totals go to block_counts[block][E].  Skipped when
//             one block holds all indices.
//   place   : same chunking.  Thread e first adds up block_counts[.][e]: the sum over
//             the blocks before its own is the block's base inside expert e, the sum
//             over all blocks is counts[e], whose exclusive scan is offsets[] (block 0
//             writes both).  With more than kScanInPlace blocks a one-block scan kernel
//             does these sums once instead (block_base, counts, offsets).  The rank of an
//             entry inside its expert is offsets[e] + base + (entries of earlier wavefront
//             passes of the block, from LDS) + popcount(ballot & lanes below).
//             No atomics: the placement is a pure function of the input, hence
//             stable (ascending flat index inside an expert) and reproducible.
//   gather  : x_perm[row] = x[row_src[row] / k], 16 bytes per lane, one block per row.
#include "moe_internal.h"

namespace moe {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kPasses = 4;
constexpr int kChunk = kThreads * kPasses;   // flat indices per block
constexpr int kScanInPlace = 256;            // up to this many blocks every placing block sums the block counts itself

__device__ __forceinline__ int lanes_below(uint64_t mask, int lane) {
    return __popcll(mask & ((1ull << lane) - 1ull));
}

__global__ __launch_bounds__(kThreads) void count_kernel(const int32_t* __restrict__ ids, int R, int E,
                                                         int32_t* __restrict__ block_counts) {
    __shared__ int32_t cnt[kPasses * kWaves][MOE_MAX_EXPERTS];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int base = blockIdx.x * kChunk;
    int my_id[kPasses];
#pragma unroll
    for (int p = 0; p < kPasses; ++p) {               // all loads under way at once
        const int i = base + p * kThreads + threadIdx.x;
        my_id[p] = i < R ? ids[i] : -1;
    }
#pragma unroll
    for (int p = 0; p < kPasses; ++p) {
        for (int e = 0; e < E; ++e) {
            const uint64_t m = __ballot(my_id[p] == e);
            if (lane == 0) cnt[p * kWaves + wave][e] = __popcll(m);
        }
    }
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += kThreads) {
        int sum = 0;
        for (int j = 0; j < kPasses * kWaves; ++j) sum += cnt[j][e];
        block_counts[(size_t)blockIdx.x * E + e] = sum;
    }
}

__global__ __launch_bounds__(64) void scan_kernel(const int32_t* __restrict__ block_counts, int nblocks, int E,
                                                  int32_t* __restrict__ block_base, int32_t* __restrict__ counts,
                                                  int32_t* __restrict__ offsets, int32_t* __restrict__ status) {
    __shared__ int32_t total[MOE_MAX_EXPERTS];
    const int e = threadIdx.x;
    if (status && threadIdx.x < 4) status[threadIdx.x] = 0;
    if (e < E) {
        int run = 0;
        for (int b = 0; b < nblocks; ++b) {
            const int c = block_counts[(size_t)b * E + e];
            block_base[(size_t)b * E + e] = run;
            run += c;
        }
        total[e] = run;
        counts[e] = run;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int run = 0;
        for (int j = 0; j < E; ++j) {
            offsets[j] = run;
            run += total[j];
        }
        offsets[E] = run;
    }
}

// block_base != null: the scan kernel has run (block_base, counts, offsets are inputs).  Else they are
// formed here from block_counts[nblocks][E] (nblocks == 1: from this block's own counts), and block 0
// writes counts[], offsets[] and clears status[0..3] when status is not null.
__global__ __launch_bounds__(kThreads) void place_kernel(const int32_t* __restrict__ ids,
                                                         const float* __restrict__ topk_w, int R, int E,
                                                         const int32_t* __restrict__ block_counts, int nblocks,
                                                         const int32_t* __restrict__ block_base,
                                                         int32_t* __restrict__ counts, int32_t* __restrict__ offsets,
                                                         int32_t* __restrict__ row_src, int32_t* __restrict__ row_of,
                                                         float* __restrict__ row_w, int32_t* __restrict__ status) {
    __shared__ int32_t cnt[kPasses * kWaves][MOE_MAX_EXPERTS];
    __shared__ int32_t start[MOE_MAX_EXPERTS];
    __shared__ int32_t total[MOE_MAX_EXPERTS];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int base = blockIdx.x * kChunk;
    // sums over the other blocks' counts (loads under way during the ballots below)
    int before = 0, all = 0;
    if (threadIdx.x < E) {
        const int e = threadIdx.x;
        if (block_base) {
            before = offsets[e] + block_base[(size_t)blockIdx.x * E + e];
        } else if (nblocks > 1) {
            for (int b = 0; b < nblocks; ++b) {
                const int c = block_counts[(size_t)b * E + e];
                all += c;
                if (b < (int)blockIdx.x) before += c;
            }
        }
    }
    if (!block_base && status && blockIdx.x == 0 && threadIdx.x < 4) status[threadIdx.x] = 0;
    int my_id[kPasses], my_rank[kPasses];
    float my_w[kPasses];
#pragma unroll
    for (int p = 0; p < kPasses; ++p) {               // all loads under way at once
        const int i = base + p * kThreads + threadIdx.x;
        my_id[p] = i < R ? ids[i] : -1;
        my_w[p] = (row_w && i < R) ? topk_w[i] : 0.f;
    }
#pragma unroll
    for (int p = 0; p < kPasses; ++p) {
        const int id = my_id[p];
        my_rank[p] = 0;
        for (int e = 0; e < E; ++e) {
            const uint64_t m = __ballot(id == e);
            if (lane == 0) cnt[p * kWaves + wave][e] = __popcll(m);
            if (id == e) my_rank[p] = lanes_below(m, lane);
        }
    }
    __syncthreads();
    // exclusive running sum over the (pass, wavefront) order in which flat indices grow
    for (int e = threadIdx.x; e < E; e += kThreads) {
        int run = 0;
        for (int j = 0; j < kPasses * kWaves; ++j) {
            const int c = cnt[j][e];
            cnt[j][e] = run;
            run += c;
        }
        total[e] = nblocks > 1 ? all : run;
        start[e] = before;
    }
    if (!block_base) {
        __syncthreads();
        if (threadIdx.x == 0) {
            int run = 0;
            for (int e = 0; e < E; ++e) {
                start[e] += run;
                if (blockIdx.x == 0) {
                    offsets[e] = run;
                    counts[e] = total[e];
                }
                run += total[e];
            }
            if (blockIdx.x == 0) offsets[E] = run;
        }
    }
    __syncthreads();
#pragma unroll
    for (int p = 0; p < kPasses; ++p) {
        const int i = base + p * kThreads + threadIdx.x;
        const int e = my_id[p];
        if (i < R && e >= 0 && e < E) {                      // ids outside [0,E) are left unplaced
            const int r = start[e] + cnt[p * kWaves + wave][e] + my_rank[p];
            row_of[i] = r;
            row_src[r] = i;
            if (row_w) row_w[r] = my_w[p];
        }
    }
}

__global__ __launch_bounds__(256) void gather_rows_kernel(const uint4* __restrict__ x, const int32_t* __restrict__ row_src,
                                                          int k, int T, int row_vec, uint4* __restrict__ x_perm) {
    const int r = blockIdx.x;
    const int t = min(max(row_src[r] / k, 0), T - 1);   // stays in bounds even if ids were invalid
    const uint4* src = x + (size_t)t * row_vec;
    uint4* dst = x_perm + (size_t)r * row_vec;
    for (int c = threadIdx.x; c < row_vec; c += 256) dst[c] = src[c];
}

}  // namespace

size_t permute_workspace_bytes(const moe_shape& s) {
    const size_t R = (size_t)s.T * s.k;
    const size_t nblocks = (R + kChunk - 1) / kChunk;
    return 2 * std::max<size_t>(nblocks, 1) * s.E * sizeof(int32_t);
}

int launch_permute(const moe_shape& s, const int32_t* ids, const float* topk_w, const void* x, int32_t* counts,
                   int32_t* offsets, int32_t* row_src, int32_t* row_of, float* row_w, void* x_perm, void* ws,
                   int32_t* status_to_clear, hipStream_t st) {
    const int R = s.T * s.k;
    const int nblocks = std::max((R + kChunk - 1) / kChunk, 1);      // R == 0: one block writes the zero counts
    int32_t* block_counts = (int32_t*)ws;
    int32_t* block_base = nullptr;
    if (nblocks > 1) {
        hipLaunchKernelGGL(count_kernel, dim3(nblocks), dim3(kThreads), 0, st, ids, R, s.E, block_counts);
        MOE_HIP_TRY(hipGetLastError());
    }
    if (nblocks > kScanInPlace) {
        block_base = block_counts + (size_t)nblocks * s.E;
        hipLaunchKernelGGL(scan_kernel, dim3(1), dim3(64), 0, st, block_counts, nblocks, s.E, block_base, counts, offsets,
                           status_to_clear);
        MOE_HIP_TRY(hipGetLastError());
    }
    hipLaunchKernelGGL(place_kernel, dim3(nblocks), dim3(kThreads), 0, st, ids, topk_w, R, s.E, block_counts, nblocks,
                       block_base, counts, offsets, row_src, row_of, row_w, status_to_clear);
    MOE_HIP_TRY(hipGetLastError());
    if (R > 0) {
        if (x && x_perm) {
            const int row_vec = s.H * (s.dtype == MOE_DTYPE_BF16 ? 2 : 4) / 16;
            hipLaunchKernelGGL(gather_rows_kernel, dim3(R), dim3(256), 0, st, (const uint4*)x, row_src, s.k, s.T, row_vec,
                               (uint4*)x_perm);
            MOE_HIP_TRY(hipGetLastError());
        }
    }
    return MOE_OK;
}

}  // namespace moe
