// Gather of ragged row chunks: what one GPU of an expert-parallel group does
// between the All-to-All-V and its local experts (Section 3.3, forward
// workflow).  The received rows lie source rank by source rank, each source's
// rows by local expert; the expert GEMMs need them expert by expert, and the
// way back needs the source order again.  Both are the same operation: dst is
// the sequence of src chunks order[0], order[1], ...
//
//   1. sort_chunks_plan_kernel  one workgroup: start rows of every source chunk
//                               (scan of the chunk sizes), then start row in dst
//                               and in src of every destination chunk (scan of
//                               the gathered sizes); also the per-group offsets
//                               the grouped GEMM takes.
//   2. sort_chunks_copy_kernel  one wave per destination row: chunk found by a
//                               binary search of the plan held in LDS, row moved
//                               with 16-byte lanes.
#include "common.h"

namespace moe {

namespace {

constexpr int kMaxChunks = 4096;
constexpr int kPlanThreads = 1024;
constexpr int kPerThread = kMaxChunks / kPlanThreads;

// Exclusive prefix of one value per thread over the 1024-thread workgroup.
__device__ __forceinline__ int block_prefix(int v, int* wave_sums) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int inc = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int o = __shfl_up(inc, d, 64);
        if (lane >= d) inc += o;
    }
    __syncthreads();  // the previous use of wave_sums is over
    if (lane == 63) wave_sums[wave] = inc;
    __syncthreads();
    int base = 0;
    for (int w = 0; w < wave; ++w) base += wave_sums[w];
    return base + inc - v;
}

// plan [2 * n_dst + 1]: dst start row of every destination chunk, the total, then
// the src start row of every destination chunk.
__global__ __launch_bounds__(kPlanThreads) void sort_chunks_plan_kernel(
    const int32_t* __restrict__ chunk_rows, int n_src, const int32_t* __restrict__ order, int n_dst,
    int group, int32_t* __restrict__ plan, int32_t* __restrict__ chunk_rows_out,
    int32_t* __restrict__ group_offsets) {
    __shared__ int rows_src[kMaxChunks];
    __shared__ int start_src[kMaxChunks];
    __shared__ int wave_sums[kPlanThreads / 64];
    const int t = threadIdx.x;
    int v[kPerThread], sum = 0;
#pragma unroll
    for (int j = 0; j < kPerThread; ++j) {
        const int c = t * kPerThread + j;
        int r = (c < n_src) ? chunk_rows[c] : 0;
        if (r < 0) r = 0;
        v[j] = r;
        sum += r;
    }
    int run = block_prefix(sum, wave_sums);
#pragma unroll
    for (int j = 0; j < kPerThread; ++j) {
        const int c = t * kPerThread + j;
        rows_src[c] = v[j];
        start_src[c] = run;
        run += v[j];
    }
    __syncthreads();
    int from[kPerThread];
    sum = 0;
#pragma unroll
    for (int j = 0; j < kPerThread; ++j) {
        const int p = t * kPerThread + j;
        const int c = (p < n_dst) ? order[p] : -1;
        const bool ok = (unsigned)c < (unsigned)n_src;
        v[j] = ok ? rows_src[c] : 0;
        from[j] = ok ? start_src[c] : 0;
        sum += v[j];
    }
    run = block_prefix(sum, wave_sums);
#pragma unroll
    for (int j = 0; j < kPerThread; ++j) {
        const int p = t * kPerThread + j;
        if (p < n_dst) {
            plan[p] = run;
            plan[n_dst + 1 + p] = from[j];
            if (chunk_rows_out) chunk_rows_out[p] = v[j];
            if (group_offsets && p % group == 0) group_offsets[p / group] = run;
        }
        run += v[j];
        if (p == n_dst - 1 || (n_dst == 0 && p == 0)) {
            const int total = (n_dst == 0) ? 0 : run;
            plan[n_dst] = total;
            if (group_offsets) group_offsets[(n_dst + group - 1) / group] = total;
        }
    }
}

// One wave per destination row.  row_bytes is a multiple of 16.
__global__ __launch_bounds__(256) void sort_chunks_copy_kernel(const uint8_t* __restrict__ src, int r_src,
                                                               const int32_t* __restrict__ plan, int n_dst,
                                                               uint8_t* __restrict__ dst, int r_dst,
                                                               int row_bytes) {
    __shared__ int start_dst[kMaxChunks + 1];
    __shared__ int start_src[kMaxChunks];
    for (int i = threadIdx.x; i <= n_dst; i += 256) start_dst[i] = plan[i];
    for (int i = threadIdx.x; i < n_dst; i += 256) start_src[i] = plan[n_dst + 1 + i];
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int total = min(start_dst[n_dst], r_dst);
    for (int row = blockIdx.x * 4 + wave; row < total; row += gridDim.x * 4) {
        // first chunk boundary above the row; the chunk in front of it holds the row
        int lo = 0, hi = n_dst;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (start_dst[mid + 1] > row) hi = mid; else lo = mid + 1;
        }
        if (lo >= n_dst) continue;  // cannot happen for row < total; never an address
        const int from = start_src[lo] + (row - start_dst[lo]);
        if ((unsigned)from >= (unsigned)r_src) continue;
        const uint8_t* s = src + (size_t)from * row_bytes;
        uint8_t* d = dst + (size_t)row * row_bytes;
        for (int o = lane * 16; o < row_bytes; o += 4096) {
            u32x4 v[4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (o + i * 1024 < row_bytes) v[i] = *reinterpret_cast<const u32x4*>(s + o + i * 1024);
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (o + i * 1024 < row_bytes) *reinterpret_cast<u32x4*>(d + o + i * 1024) = v[i];
        }
    }
}

}  // namespace

int sort_chunks_max_chunks() { return kMaxChunks; }

size_t sort_chunks_workspace_bytes(int n_dst) { return up256((size_t)(2 * n_dst + 1) * sizeof(int32_t)); }

void launch_sort_chunks(const void* src, int r_src, const int32_t* chunk_rows, int n_src, const int32_t* order,
                        int n_dst, int group, int row_bytes, void* dst, int r_dst, int32_t* chunk_rows_out,
                        int32_t* group_offsets, void* ws, hipStream_t s) {
    int32_t* plan = static_cast<int32_t*>(ws);
    hipLaunchKernelGGL(sort_chunks_plan_kernel, dim3(1), dim3(kPlanThreads), 0, s, chunk_rows, n_src, order, n_dst,
                       group > 0 ? group : 1, plan, chunk_rows_out, group_offsets);
    if (src == nullptr || dst == nullptr || r_dst == 0 || r_src == 0 || n_dst == 0) return;
    int grid = (r_dst + 3) / 4;
    if (grid > 4096) grid = 4096;
    hipLaunchKernelGGL(sort_chunks_copy_kernel, dim3(grid), dim3(256), 0, s, static_cast<const uint8_t*>(src), r_src,
                       plan, n_dst, static_cast<uint8_t*>(dst), r_dst, row_bytes);
}

}  // namespace moe
