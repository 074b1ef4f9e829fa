// a2. Permute: the local part of the paper's token dispatching (Section 3.1.2:
// rows of one expert contiguous in memory) with the capacity rule of Eq. 4 and
// sub-sequence dropping (Section 3.3).
//
// The permutation is a stable counting sort of the T*K assignments by expert,
// built without any slot-claiming atomics so the maps are bit-reproducible:
//   1. permute_hist_kernel  per chunk of 1024 assignments, a per-expert
//                           histogram (integer LDS atomics: only counts).
//   2. permute_map_kernel   every workgroup sums the chunk histograms (totals
//                           and its own exclusive base), scans the clamped
//                           counts into offsets, ranks its chunk's assignments
//                           with wave ballots and writes both maps.
//   3. permute_copy_kernel  one wave per token: the row is read once with
//                           16-byte lanes and stored to each kept destination.
// Layers with few experts and a small index array (the Mixtral shapes) take
// permute_fused_kernel instead: the same maps from ONE launch, the counting
// hidden under the latency of the row loads.
#include <mutex>

#include "fp8_convert.h"

namespace moe {

namespace {

constexpr int kChunk = 1024;  // assignments per workgroup
constexpr int kUnits = kChunk / 64;

// Scratch of moe_permute_noalloc: the chunk histograms of one call (the role `workspace` plays in
// moe_permute).  One copy per GPU, held from the library's load to the end of the process; every call on a
// GPU shares it.  In host code the array's name is only a handle for hipGetSymbolAddress, never an address.
constexpr size_t kScratchInts = 256 * 1024;   // 1 MiB
static __device__ __align__(256) int32_t scratch[kScratchInts];
constexpr int kMaxDevices = 64;
static int32_t* g_scratch_ptr[kMaxDevices] = {};   // device address of `scratch`, per device ordinal
static std::mutex g_scratch_mutex;

__global__ __launch_bounds__(256) void permute_hist_kernel(const int32_t* __restrict__ idx, int A,
                                                           int E, int32_t* __restrict__ chunk_hist) {
    __shared__ int hist[kMaxExperts];
    for (int e = threadIdx.x; e < E; e += 256) hist[e] = 0;
    __syncthreads();
    const int a0 = blockIdx.x * kChunk;
#pragma unroll
    for (int j = 0; j < kChunk / 256; ++j) {
        const int a = a0 + j * 256 + threadIdx.x;
        if (a < A) {
            const int e = idx[a];
            if ((unsigned)e < (unsigned)E) atomicAdd(&hist[e], 1);
        }
    }
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += 256) chunk_hist[(size_t)blockIdx.x * E + e] = hist[e];
}

__global__ __launch_bounds__(256) void permute_map_kernel(
    const int32_t* __restrict__ idx, const int32_t* __restrict__ chunk_hist, int A, int E,
    int capacity, int pad, int r_max, int nchunks, int32_t* __restrict__ counts,
    int32_t* __restrict__ offsets, int32_t* __restrict__ row_of_assign,
    int32_t* __restrict__ assign_of_row) {
    __shared__ int tot[kMaxExperts];
    __shared__ int base[kMaxExperts];
    __shared__ int scan[2][kMaxExperts];
    __shared__ int off[kMaxExperts + 1];
    __shared__ int unit_cnt[kUnits][kMaxExperts];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int chunk = blockIdx.x;

    tot[tid] = 0;
    base[tid] = 0;
    for (int i = tid; i < kUnits * kMaxExperts; i += 256) (&unit_cnt[0][0])[i] = 0;
    __syncthreads();
    {
        // per-expert totals over all chunks and over the chunks before this one.  Thread
        // (cs, e) sums every `groups`-th chunk privately (independent loads, so many are in
        // flight), then adds its two partial sums to the shared cells once.
        int ep = 1;
        while (ep < E) ep <<= 1;
        const int groups = 256 / ep, cs = tid / ep, e = tid % ep;
        if (e < E) {
            int t_sum = 0, b_sum = 0;
#pragma unroll 8
            for (int c = cs; c < nchunks; c += groups) {
                const int v = chunk_hist[(size_t)c * E + e];
                t_sum += v;
                b_sum += (c < chunk) ? v : 0;
            }
            if (t_sum) atomicAdd(&tot[e], t_sum);
            if (b_sum) atomicAdd(&base[e], b_sum);
        }
    }
    __syncthreads();
    // counts = min(total, capacity); offsets = exclusive scan (256-wide Hillis-Steele)
    const int cnt = (tid < E) ? ((capacity > 0 && tot[tid] > capacity) ? capacity : tot[tid]) : 0;
    scan[0][tid] = cnt;
    __syncthreads();
    int cur = 0;
    for (int d = 1; d < kMaxExperts; d <<= 1) {
        const int v = scan[cur][tid] + ((tid >= d) ? scan[cur][tid - d] : 0);
        scan[cur ^ 1][tid] = v;
        cur ^= 1;
        __syncthreads();
    }
    // padded layout: every expert owns a block of `capacity` rows, whatever it keeps
    const int incl = pad ? (tid + 1) * capacity : scan[cur][tid];
    if (tid < E) off[tid + 1] = incl;
    if (tid == 0) off[0] = 0;
    if (pad) tot[tid] = cnt;   // kept rows per expert, for the marking of the unused rows below
    if (chunk == 0) {
        if (tid < E) {
            counts[tid] = cnt;
            offsets[tid + 1] = incl;
        }
        if (tid == 0) offsets[0] = 0;
    }

    // rank of every assignment of this chunk inside its (expert, 64-assignment unit)
    int nbits = 0;
    while ((1 << nbits) < E) ++nbits;
    int my_e[kChunk / 256], my_r[kChunk / 256];
    const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
#pragma unroll
    for (int j = 0; j < kChunk / 256; ++j) {
        const int u = j * 4 + wave;
        const int a = chunk * kChunk + u * 64 + lane;
        int e = (a < A) ? idx[a] : -1;
        const bool valid = (unsigned)e < (unsigned)E;
        if (!valid) e = -1;
        // lanes of this unit that name the same expert: one ballot per bit of the expert index
        uint64_t peers = __ballot(valid);
        for (int b = 0; b < nbits; ++b) {   // uniform trip count
            const bool bit = (e >> b) & 1;
            const uint64_t m = __ballot(valid && bit);
            peers &= bit ? m : ~m;
        }
        int r = 0;
        if (valid) {
            r = __popcll(peers & lt_mask);
            if (r == 0) unit_cnt[u][e] = __popcll(peers);   // the first lane of the group records its size
        }
        my_e[j] = e;
        my_r[j] = r;
    }
    __syncthreads();
    if (tid < E) {
        int run = 0;
#pragma unroll
        for (int u = 0; u < kUnits; ++u) {
            const int c = unit_cnt[u][tid];
            unit_cnt[u][tid] = run;
            run += c;
        }
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < kChunk / 256; ++j) {
        const int u = j * 4 + wave;
        const int a = chunk * kChunk + u * 64 + lane;
        if (a < A) {
            const int e = my_e[j];
            int row = -1;
            if (e >= 0) {
                const int rank = base[e] + unit_cnt[u][e] + my_r[j];
                if (capacity <= 0 || rank < capacity) row = off[e] + rank;
            }
            if (row >= r_max) row = -1;  // cannot happen for a consistent r_max; never an address
            row_of_assign[a] = row;
            if (row >= 0) assign_of_row[row] = a;
        }
    }
    // rows past the kept total are marked unused; in the padded layout also the tail of every block
    if (pad) {
        __syncthreads();   // tot[] now holds the kept counts
        for (int r = chunk * 256 + tid; r < r_max; r += nchunks * 256) {
            const int e = r / capacity;
            if (e >= E || r - e * capacity >= tot[e]) assign_of_row[r] = -1;
        }
    } else {
        const int R = off[E];
        for (int r = R + chunk * 256 + tid; r < r_max; r += nchunks * 256) assign_of_row[r] = -1;
    }
}

// ---- drop by score ----
// Order-preserving 32-bit key of a finite float (larger float <=> larger key; -0 = +0).
__device__ __forceinline__ uint32_t score_key(float s) {
    uint32_t b = __float_as_uint(s);
    if (s == 0.f) b = 0u;
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

constexpr int kSelThreads = 1024;   // threads of permute_select_kernel

// exclusive prefix of a flag over the threads of the workgroup and its total; `wsum` is LDS scratch, one int per wave
__device__ __forceinline__ int block_rank(bool flag, int* wsum, int& total) {
    constexpr int NWAVE = kSelThreads / 64;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint64_t m = __ballot(flag);
    const uint64_t lt = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
    __syncthreads();   // the previous use of wsum is over
    if (lane == 0) wsum[wave] = __popcll(m);
    __syncthreads();
    int before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < NWAVE; ++w) {
        const int c = wsum[w];
        before += (w < wave) ? c : 0;
        all += c;
    }
    total = all;
    return before + __popcll(m & lt);
}

// One workgroup per expert.  seg_off / seg_aor: the dropless grouping (expert e's assignments in
// ascending index at seg_aor[seg_off[e] .. seg_off[e+1])).  An expert with more than `capacity`
// assignments keeps those with the largest scores (ties: lower assignment index): the capacity-th
// largest 32-bit key is found by a 4-pass radix selection over the expert's keys, then one ordered
// pass assigns rows to the kept assignments in ascending assignment index.  row_of_assign holds -1
// for assignments without a valid expert on entry (written by the dropless grouping).
__global__ __launch_bounds__(kSelThreads) void permute_select_kernel(
    const float* __restrict__ scores, const int32_t* __restrict__ seg_off, const int32_t* __restrict__ seg_aor,
    uint32_t* __restrict__ keys, int E, int capacity, int pad, int r_max, int32_t* __restrict__ counts,
    int32_t* __restrict__ offsets, int32_t* __restrict__ row_of_assign, int32_t* __restrict__ assign_of_row) {
    __shared__ int scan[2][kMaxExperts];
    __shared__ int hist[256];
    __shared__ int wsum[kSelThreads / 64];
    __shared__ uint32_t sel[2];   // decided key prefix, keys still to take at this prefix
    const int tid = threadIdx.x, e = blockIdx.x;
    // rows kept by every expert, and this expert's first row (scan by the first kMaxExperts threads)
    const bool scanner = tid < kMaxExperts;
    const int n_mine = (tid < E) ? seg_off[tid + 1] - seg_off[tid] : 0;
    const int cnt = n_mine > capacity ? capacity : n_mine;
    if (scanner) scan[0][tid] = cnt;
    __syncthreads();
    int cur = 0;
    for (int d = 1; d < kMaxExperts; d <<= 1) {
        if (scanner) scan[cur ^ 1][tid] = scan[cur][tid] + ((tid >= d) ? scan[cur][tid - d] : 0);
        cur ^= 1;
        __syncthreads();
    }
    const int lo = seg_off[e], n = seg_off[e + 1] - lo;
    const int kept = n > capacity ? capacity : n;
    const int base = pad ? e * capacity : (e ? scan[cur][e - 1] : 0);
    const int R = pad ? E * capacity : scan[cur][E - 1];
    if (tid == 0) {
        counts[e] = kept;
        offsets[e] = base;
        if (e == E - 1) offsets[E] = R;
    }
    const bool all = n <= capacity;
    uint32_t thr = 0;
    int need_eq = 0;
    if (!all) {   // uniform over the workgroup
        if (tid == 0) {
            sel[0] = 0u;
            sel[1] = (uint32_t)capacity;
        }
        for (int pass = 0; pass < 4; ++pass) {
            const int shift = 24 - 8 * pass;
            if (tid < 256) hist[tid] = 0;
            __syncthreads();
            const uint32_t prefix = sel[0];
#pragma unroll 4
            for (int i = tid; i < n; i += kSelThreads) {
                uint32_t key;
                if (pass == 0) {
                    key = score_key(scores[seg_aor[lo + i]]);
                    keys[lo + i] = key;
                } else {
                    key = keys[lo + i];
                }
                // 64-bit shift: the first pass compares nothing
                if (((uint64_t)(key ^ prefix) >> (shift + 8)) == 0) atomicAdd(&hist[(key >> shift) & 255u], 1);
            }
            __syncthreads();
            if (tid == 0) {
                int remaining = (int)sel[1], d = 255;
                while (d > 0 && hist[d] < remaining) {   // the digit that holds the `remaining`-th largest key
                    remaining -= hist[d];
                    --d;
                }
                sel[0] = prefix | ((uint32_t)d << shift);
                sel[1] = (uint32_t)remaining;
            }
            __syncthreads();
        }
        thr = sel[0];
        need_eq = (int)sel[1];   // keys equal to thr that are still kept: the first need_eq in index order
    }
    int run_eq = 0, run_kept = 0;
    for (int c0 = 0; c0 < n; c0 += kSelThreads) {
        const int i = c0 + tid;
        const bool valid = i < n;
        const int a = valid ? seg_aor[lo + i] : -1;
        const uint32_t key = (valid && !all) ? keys[lo + i] : 0u;
        const bool gt = valid && (all || key > thr);
        const bool eq = valid && !all && key == thr;
        int tot_eq, tot_keep;
        const int eq_rank = run_eq + block_rank(eq, wsum, tot_eq);
        const bool keep = gt || (eq && eq_rank < need_eq);
        const int k_rank = run_kept + block_rank(keep, wsum, tot_keep);
        if (valid) {
            int row = keep ? base + k_rank : -1;
            if (row >= r_max) row = -1;   // cannot happen for a consistent r_max; never an address
            row_of_assign[a] = row;
            if (row >= 0) assign_of_row[row] = a;
        }
        run_eq += tot_eq;
        run_kept += tot_keep;
    }
    // unused rows
    if (pad) {
        for (int r = base + kept + tid; r < base + capacity && r < r_max; r += kSelThreads) assign_of_row[r] = -1;
    }
    for (int r = R + e * kSelThreads + tid; r < r_max; r += E * kSelThreads) assign_of_row[r] = -1;
}

// Zero the rows that no assignment owns (padded layout).  One wave per row.
__global__ __launch_bounds__(256) void permute_zero_rows_kernel(const int32_t* __restrict__ assign_of_row,
                                                                uint8_t* __restrict__ x_perm, int rows,
                                                                int row_bytes) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int r = blockIdx.x * 4 + wave; r < rows; r += gridDim.x * 4) {
        if (assign_of_row[r] >= 0) continue;
        uint8_t* dst = x_perm + (size_t)r * row_bytes;
        for (int o = lane * 16; o < row_bytes; o += 1024) *reinterpret_cast<u32x4*>(dst + o) = u32x4{0u, 0u, 0u, 0u};
    }
}

// One wave per token.  row_bytes is a multiple of 16.
__global__ __launch_bounds__(256) void permute_copy_kernel(const uint8_t* __restrict__ x,
                                                           const int32_t* __restrict__ row_of_assign,
                                                           uint8_t* __restrict__ x_perm, int T, int K,
                                                           int row_bytes, int r_max) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int t = blockIdx.x * 4 + wave; t < T; t += gridDim.x * 4) {
        int my_row = (lane < K) ? row_of_assign[(size_t)t * K + lane] : -1;
        if ((unsigned)my_row >= (unsigned)r_max) my_row = -1;
        const uint64_t kept = __ballot(my_row >= 0);
        if (!kept) continue;
        const uint8_t* src = x + (size_t)t * row_bytes;
        for (int o0 = 0; o0 < row_bytes; o0 += 4096) {  // uniform trip count: shuffles inside
            const int o = o0 + lane * 16;
            u32x4 v[4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (o + i * 1024 < row_bytes)
                    v[i] = *reinterpret_cast<const u32x4*>(src + o + i * 1024);
            uint64_t m = kept;
            while (m) {
                const int k = __ffsll((unsigned long long)m) - 1;
                m &= m - 1;
                const int row = __shfl(my_row, k, 64);
                uint8_t* dst = x_perm + (size_t)row * row_bytes + o;
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (o + i * 1024 < row_bytes) *reinterpret_cast<u32x4*>(dst + i * 1024) = v[i];
            }
        }
    }
}

// Copy fused with FP8 quantisation (Section 4.5 recipe): bf16 rows are read
// once, scaled, rounded to E4M3 and stored as H bytes to each kept destination;
// max |x| over the rows that were read is folded into *amax.
__global__ __launch_bounds__(256) void permute_copy_fp8_kernel(const uint8_t* __restrict__ x,
                                                               const int32_t* __restrict__ row_of_assign,
                                                               uint8_t* __restrict__ x_perm, int T, int K, int H,
                                                               int r_max, float scale, float* __restrict__ amax) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int row_bytes = H * 2;
    float m = 0.f;
    for (int t = blockIdx.x * 4 + wave; t < T; t += gridDim.x * 4) {
        int my_row = (lane < K) ? row_of_assign[(size_t)t * K + lane] : -1;
        if ((unsigned)my_row >= (unsigned)r_max) my_row = -1;
        const uint64_t kept = __ballot(my_row >= 0);
        if (!kept) continue;
        const uint8_t* src = x + (size_t)t * row_bytes;
        for (int o0 = 0; o0 < row_bytes; o0 += 4096) {  // uniform trip count: shuffles inside
            const int o = o0 + lane * 16;
            u32x2 q[4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (o + i * 1024 < row_bytes) {
                    const u32x4 v = *reinterpret_cast<const u32x4*>(src + o + i * 1024);
                    float f[8];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        f[2 * j] = __uint_as_float(v[j] << 16);
                        f[2 * j + 1] = __uint_as_float(v[j] & 0xffff0000u);
                    }
#pragma unroll
                    for (int j = 0; j < 8; ++j) m = fmaxf(m, fabsf(f[j]));
                    q[i][0] = f32x4_to_e4m3(f[0] * scale, f[1] * scale, f[2] * scale, f[3] * scale);
                    q[i][1] = f32x4_to_e4m3(f[4] * scale, f[5] * scale, f[6] * scale, f[7] * scale);
                }
            uint64_t mk = kept;
            while (mk) {
                const int k = __ffsll((unsigned long long)mk) - 1;
                mk &= mk - 1;
                const int row = __shfl(my_row, k, 64);
                uint8_t* dst = x_perm + (size_t)row * H + (o >> 1);
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (o + i * 1024 < row_bytes) *reinterpret_cast<u32x2*>(dst + i * 512) = q[i];
            }
        }
    }
    if (amax) {
        // one atomic per workgroup at most, and none if the value read is already as large
        // (*amax only grows): atomics on one address serialise
        __shared__ float wave_max[4];
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
        if (lane == 0) wave_max[wave] = m;
        __syncthreads();
        if (threadIdx.x == 0) {
            m = fmaxf(fmaxf(wave_max[0], wave_max[1]), fmaxf(wave_max[2], wave_max[3]));
            if (m > __builtin_nontemporal_load(amax)) atomicMax(reinterpret_cast<int*>(amax), __float_as_int(m));
        }
    }
}

// ---- all of a2 in one launch, for layers with few experts and an index array small enough that every workgroup can
// count it itself (E <= 8, T*K <= 32768: the Mixtral shapes) ----
// A workgroup of 16 waves owns TB = 16 * tpw consecutive tokens (wave w the tokens t0 + w, t0 + w + 16, ...; one
// workgroup per compute unit at the benchmark shapes).  Every wave first requests
// the row of its first token (rows do not depend on the maps), then, while that load is in flight, the workgroup counts the WHOLE
// index array: every thread keeps eight 8-bit counters in one 64-bit register (it sees at most 64 assignments),
// one for the whole array and one for the assignments before the workgroup's own; the threads' registers are
// widened to 16-bit fields and added across the workgroup (integer sums: no order dependence).  Totals clamp to
// the capacity and scan to the offsets; the workgroup's own few assignments are ranked in ascending order with
// wave ballots; the maps are written and the rows stored.  Same maps, bit for bit, as the three-kernel path: rank = assignments of the same expert
// with a lower index.  No workgroup waits for another.
constexpr int kFusedMaxRowVecs = 16;       // row of at most 16 KiB: 16 x 16 bytes per lane
constexpr int kFusedMaxAssign = 65532;     // <= 64 assignments per thread (8-bit counters), totals below 2^16
constexpr int kFusedMaxExperts = 8;
constexpr int kFusedWaves = 16;

// NV: 16-byte pieces per lane of a row (row of at most NV KiB); TPW: tokens per wave, all requested up front
template <int NV, int TPW>
__global__ __launch_bounds__(kFusedWaves * 64) void permute_fused_kernel(
    const uint8_t* __restrict__ x, const int32_t* __restrict__ idx, int T, int K, int E, int capacity, int row_bytes,
    int r_max, uint8_t* __restrict__ x_perm, int32_t* __restrict__ counts, int32_t* __restrict__ offsets,
    int32_t* __restrict__ row_of_assign, int32_t* __restrict__ assign_of_row) {
    constexpr int NWV = kFusedWaves, NTH = NWV * 64;
    __shared__ unsigned long long red[NWV][4];
    __shared__ int base[kFusedMaxExperts];
    __shared__ int run[kFusedMaxExperts];
    __shared__ int off[kFusedMaxExperts + 1];
    __shared__ int rows[NWV * TPW * kFusedMaxExperts];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int A = T * K;
    constexpr int TB = NWV * TPW;
    const int t0 = blockIdx.x * TB;
    const int a0 = t0 * K;                                   // first assignment of this workgroup (a multiple of 4)
    const int na = min(TB, T - t0) * K;                      // its assignments

    // The index array first, then the rows: loads return in order, so the counting below can start as soon as the
    // (cached) indices are back while the rows are still on their way from memory.
    constexpr int NPRE = 4;                                  // index groups per thread requested up front
    const int ngroups = A >> 2;
    const int4* idx4 = reinterpret_cast<const int4*>(idx);
    int4 pre[NPRE];
#pragma unroll
    for (int q = 0; q < NPRE; ++q) {
        const int g = tid + q * NTH;
        pre[q] = (g < ngroups) ? idx4[g] : int4{-1, -1, -1, -1};
    }
    // phase 0: the row of this wave's first token (rows do not depend on the maps)
    const bool copy = x != nullptr;
    u32x4 v[TPW][NV];
    if (copy) {
#pragma unroll
        for (int j = 0; j < TPW; ++j) {
            const int t = t0 + j * NWV + wave;
#pragma unroll
            for (int i = 0; i < NV; ++i)
                if (t < T && i * 1024 + lane * 16 < row_bytes)
                    v[j][i] = *reinterpret_cast<const u32x4*>(x + (size_t)t * row_bytes + i * 1024 + lane * 16);
        }
    }
    if (tid < kFusedMaxExperts) run[tid] = 0;

    // phase 1: per-expert totals over all assignments and over those before a0, eight 8-bit counters per register
    unsigned long long tot8 = 0, base8 = 0;
    auto field = [&](int e) -> unsigned long long { return ((unsigned)e < (unsigned)E) ? 1ull << (8 * e) : 0ull; };
    {
#pragma unroll
        for (int q = 0; q < NPRE; ++q) {
            const int g = tid + q * NTH;
            const unsigned long long inc = field(pre[q].x) + field(pre[q].y) + field(pre[q].z) + field(pre[q].w);
            tot8 += inc;
            if (4 * g < a0) base8 += inc;                    // a0 is a multiple of 4: a group never straddles it
        }
        for (int g = tid + NPRE * NTH; g < ngroups; g += NTH) {
            const int4 e4 = idx4[g];
            const unsigned long long inc = field(e4.x) + field(e4.y) + field(e4.z) + field(e4.w);
            tot8 += inc;
            if (4 * g < a0) base8 += inc;
        }
        const int a = (ngroups << 2) + tid;                  // the last A mod 4 assignments
        if (tid < 4 && a < A) {
            const unsigned long long inc = field(idx[a]);
            tot8 += inc;
            if (a < a0) base8 += inc;
        }
    }
    // 16-bit fields (even experts, odd experts), added over the wave, then over the waves
    const unsigned long long M = 0x00FF00FF00FF00FFull;
    unsigned long long s4[4] = {tot8 & M, (tot8 >> 8) & M, base8 & M, (base8 >> 8) & M};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
#pragma unroll
        for (int d = 32; d > 0; d >>= 1) {
            const uint32_t lo = __shfl_xor((uint32_t)s4[q], d, 64);
            const uint32_t hi = __shfl_xor((uint32_t)(s4[q] >> 32), d, 64);
            s4[q] += ((unsigned long long)hi << 32) | lo;
        }
        if (lane == 0) red[wave][q] = s4[q];
    }
    __syncthreads();
    // phase 2: every thread holds all totals; thread 0 scans them
    if (tid < kFusedMaxExperts) {
        const int e = tid;
        const int q = e & 1, sh = 16 * (e >> 1);
        unsigned long long tsum = 0, bsum = 0;
#pragma unroll
        for (int w = 0; w < NWV; ++w) {
            tsum += red[w][q];
            bsum += red[w][2 + q];
        }
        const int tot_e = (e < E) ? (int)((tsum >> sh) & 0xFFFFu) : 0;
        base[e] = (int)((bsum >> sh) & 0xFFFFu);
        const int cnt = (capacity > 0 && tot_e > capacity) ? capacity : tot_e;
        // inclusive prefix over the eight lanes
        int incl = cnt;
#pragma unroll
        for (int d = 1; d < kFusedMaxExperts; d <<= 1) {
            const int o = __shfl_up(incl, d, 64);
            if (lane >= d) incl += o;
        }
        off[e + 1] = incl;
        if (e == 0) off[0] = 0;
        if (blockIdx.x == 0 && e < E) {
            counts[e] = cnt;
            offsets[e + 1] = incl;
            if (e == 0) offsets[0] = 0;
        }
    }
    __syncthreads();

    // phase 3: this workgroup's own assignments, unit by unit in ascending order (wave 0; at most 512)
    int nbits = 0;
    while ((1 << nbits) < E) ++nbits;
    const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
    if (wave == 0) {
        for (int u0 = 0; u0 < na; u0 += 64) {
            const int a = a0 + u0 + lane;
            int e = (u0 + lane < na) ? idx[a] : -1;
            const bool valid = (unsigned)e < (unsigned)E;
            // lanes of this unit that name the same expert: one ballot per bit of the expert index
            uint64_t peers = __ballot(valid);
            for (int b = 0; b < nbits; ++b) {   // uniform trip count
                const bool bit = (e >> b) & 1;
                const uint64_t m = __ballot(valid && bit);
                peers &= bit ? m : ~m;
            }
            int row = -1;
            if (valid) {
                const int before_unit = run[e];                                  // earlier units of this workgroup
                const int rank = base[e] + before_unit + __popcll(peers & lt_mask);
                if (capacity <= 0 || rank < capacity) row = off[e] + rank;
                if (row >= r_max) row = -1;  // cannot happen for a consistent r_max; never an address
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");           // every lane has read run[e]
                if ((peers & lt_mask) == 0) run[e] = before_unit + __popcll(peers);
            }
            if (u0 + lane < na) {
                rows[u0 + lane] = row;
                row_of_assign[a] = row;
                if (row >= 0) assign_of_row[row] = a;
            }
        }
    }
    // rows past the kept total are marked unused
    {
        const int R = off[E];
        for (int r = R + blockIdx.x * NTH + tid; r < r_max; r += gridDim.x * NTH) assign_of_row[r] = -1;
    }
    __syncthreads();

    // phase 4: every row to each of its kept destinations 
    if (copy) {
#pragma unroll
        for (int j = 0; j < TPW; ++j) {
            const int lt = j * NWV + wave;
            if (t0 + lt >= T) continue;
            for (int k = 0; k < K; ++k) {
                const int row = rows[lt * K + k];                                  // wave-uniform
                if (row < 0) continue;
                uint8_t* dst = x_perm + (size_t)row * row_bytes + lane * 16;
#pragma unroll
                for (int i = 0; i < NV; ++i)
                    if (i * 1024 + lane * 16 < row_bytes) *reinterpret_cast<u32x4*>(dst + i * 1024) = v[j][i];
            }
        }
    }
}

__global__ void fill_i32_kernel(int32_t* p, int n, int32_t v0, int32_t step) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v0 + i * step;
}

}  // namespace

static int g_permute_fused = 1;   // 0: always the three-kernel path
void set_permute_fused(int v) { g_permute_fused = v; }   // 2 / 3: force one / two tokens per wave (experiments)

size_t permute_workspace_bytes(int T, int K, int E) {
    const long long A = (long long)T * K;
    const long long nchunks = (A + kChunk - 1) / kChunk;
    return (size_t)((nchunks > 0 ? nchunks : 1) * E) * sizeof(int32_t);
}

void launch_permute(const void* x, const int32_t* idx, int T, int H, int E, int K, int capacity,
                    int r_max, moe_dtype_t dt, void* x_perm, int32_t* counts, int32_t* offsets,
                    int32_t* row_of_assign, int32_t* assign_of_row, void* ws, hipStream_t s) {
    const int A = T * K;
    const int row_bytes_all = H * (dt == MOE_BF16 ? 2 : 4);
    if (g_permute_fused && E <= kFusedMaxExperts && A <= kFusedMaxAssign && row_bytes_all <= kFusedMaxRowVecs * 1024 &&
        row_bytes_all % 16 == 0) {
        // few experts, small index array: one launch (the workspace is not used)
        const uint8_t* xs = (x != nullptr && x_perm != nullptr) ? static_cast<const uint8_t*>(x) : nullptr;
        // two tokens per wave (one round of workgroups at T = 8192) where both rows fit into the registers of a
        // 16-wave workgroup, else one
        const int nv = (row_bytes_all + 1023) / 1024;
        const bool two = (g_permute_fused == 1 && nv <= 12 && T > kFusedWaves * 256) || g_permute_fused == 3;
#define FUSED_CASE(NVV, TPWW)                                                                                           \
    hipLaunchKernelGGL((permute_fused_kernel<NVV, TPWW>), dim3((T + kFusedWaves * TPWW - 1) / (kFusedWaves * TPWW)),     \
                       dim3(kFusedWaves * 64), 0, s, xs, idx, T, K, E, capacity, row_bytes_all, r_max,                   \
                       static_cast<uint8_t*>(x_perm), counts, offsets, row_of_assign, assign_of_row)
        if (two && nv <= 12) {
            if (nv <= 4) FUSED_CASE(4, 2); else if (nv <= 8) FUSED_CASE(8, 2); else FUSED_CASE(12, 2);
        } else {
            if (nv <= 4) FUSED_CASE(4, 1); else if (nv <= 8) FUSED_CASE(8, 1); else if (nv <= 12) FUSED_CASE(12, 1); else FUSED_CASE(16, 1);
        }
#undef FUSED_CASE
        return;
    }
    const int nchunks = (A + kChunk - 1) / kChunk;
    int32_t* chunk_hist = static_cast<int32_t*>(ws);
    hipLaunchKernelGGL(permute_hist_kernel, dim3(nchunks), dim3(256), 0, s, idx, A, E, chunk_hist);
    hipLaunchKernelGGL(permute_map_kernel, dim3(nchunks), dim3(256), 0, s, idx, chunk_hist, A, E,
                       capacity, 0, r_max, nchunks, counts, offsets, row_of_assign, assign_of_row);
    if (x != nullptr && x_perm != nullptr) {
        const int row_bytes = H * (dt == MOE_BF16 ? 2 : 4);
        int grid = (T + 3) / 4;
        if (grid > 256 * 16) grid = 256 * 16;
        hipLaunchKernelGGL(permute_copy_kernel, dim3(grid), dim3(256), 0, s,
                           static_cast<const uint8_t*>(x), row_of_assign,
                           static_cast<uint8_t*>(x_perm), T, K, row_bytes, r_max);
    }
}

// Layout of the variant's workspace: chunk histograms, then the dropless grouping (offsets, rows) and the keys
size_t permute_variant_workspace_bytes(int T, int K, int E) {
    const size_t A = (size_t)T * K;
    return up256(permute_workspace_bytes(T, K, E)) + up256((size_t)(E + 1) * 4) + up256((size_t)E * 4) +
           up256((A + 1) * 4) + up256((A + 1) * 4);
}

// Dispatch with the drop rule (by position / by score) and the layout (packed / padded to capacity) chosen.
// capacity > 0 whenever by_score or pad is set.
void launch_permute_variant(const void* x, const int32_t* idx, const float* scores, int T, int H, int E, int K,
                            int capacity, int by_score, int pad, int r_max, moe_dtype_t dt, void* x_perm,
                            int32_t* counts, int32_t* offsets, int32_t* row_of_assign, int32_t* assign_of_row,
                            void* ws, hipStream_t s) {
    const int A = T * K;
    const int nchunks = (A + kChunk - 1) / kChunk;
    uint8_t* w = static_cast<uint8_t*>(ws);
    int32_t* chunk_hist = reinterpret_cast<int32_t*>(w);
    w += up256(permute_workspace_bytes(T, K, E));
    int32_t* seg_off = reinterpret_cast<int32_t*>(w);
    w += up256((size_t)(E + 1) * 4);
    int32_t* seg_cnt = reinterpret_cast<int32_t*>(w);
    w += up256((size_t)E * 4);
    int32_t* seg_aor = reinterpret_cast<int32_t*>(w);
    w += up256(((size_t)A + 1) * 4);
    uint32_t* keys = reinterpret_cast<uint32_t*>(w);
    hipLaunchKernelGGL(permute_hist_kernel, dim3(nchunks), dim3(256), 0, s, idx, A, E, chunk_hist);
    if (by_score) {
        // dropless grouping first (row_of_assign serves as its scratch map), then the selection per expert
        hipLaunchKernelGGL(permute_map_kernel, dim3(nchunks), dim3(256), 0, s, idx, chunk_hist, A, E, 0, 0, A,
                           nchunks, seg_cnt, seg_off, row_of_assign, seg_aor);
        hipLaunchKernelGGL(permute_select_kernel, dim3(E), dim3(kSelThreads), 0, s, scores, seg_off, seg_aor, keys, E,
                           capacity, pad, r_max, counts, offsets, row_of_assign, assign_of_row);
    } else {
        hipLaunchKernelGGL(permute_map_kernel, dim3(nchunks), dim3(256), 0, s, idx, chunk_hist, A, E, capacity,
                           pad, r_max, nchunks, counts, offsets, row_of_assign, assign_of_row);
    }
    if (x != nullptr && x_perm != nullptr) {
        const int row_bytes = H * (dt == MOE_BF16 ? 2 : 4);
        int grid = (T + 3) / 4;
        if (grid > 256 * 16) grid = 256 * 16;
        hipLaunchKernelGGL(permute_copy_kernel, dim3(grid), dim3(256), 0, s, static_cast<const uint8_t*>(x),
                           row_of_assign, static_cast<uint8_t*>(x_perm), T, K, row_bytes, r_max);
        if (pad) launch_permute_zero_rows(assign_of_row, x_perm, r_max, row_bytes, s);
    }
}

size_t permute_scratch_bytes() { return kScratchInts * sizeof(int32_t); }

// Device address of this GPU's copy of `scratch` (looked up once per device, with that device current).
// Returns nullptr and fills `err` if the runtime refuses.
int32_t* permute_scratch(hipError_t* err) {
    int dev = -1;
    *err = hipGetDevice(&dev);
    if (*err != hipSuccess) return nullptr;
    if (dev < 0 || dev >= kMaxDevices) {
        *err = hipErrorInvalidDevice;
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        *err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (*err != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = static_cast<int32_t*>(p);
    }
    return g_scratch_ptr[dev];
}

void launch_permute_zero_rows(const int32_t* assign_of_row, void* x_perm, int rows, int row_bytes, hipStream_t s) {
    if (rows <= 0) return;
    int grid = (rows + 3) / 4;
    if (grid > 256 * 16) grid = 256 * 16;
    hipLaunchKernelGGL(permute_zero_rows_kernel, dim3(grid), dim3(256), 0, s, assign_of_row,
                       static_cast<uint8_t*>(x_perm), rows, row_bytes);
}

void launch_permute_fp8(const void* x, const int32_t* idx, int T, int H, int E, int K, int capacity, int r_max,
                        float scale, void* x_perm_fp8, int32_t* counts, int32_t* offsets, int32_t* row_of_assign,
                        int32_t* assign_of_row, float* amax, void* ws, hipStream_t s) {
    // maps as in launch_permute, then the quantising copy
    launch_permute(nullptr, idx, T, H, E, K, capacity, r_max, MOE_BF16, nullptr, counts, offsets, row_of_assign,
                   assign_of_row, ws, s);
    int grid = (T + 3) / 4;
    if (grid > 256 * 4) grid = 256 * 4;   // few, longer-lived workgroups: fewer amax atomics
    hipLaunchKernelGGL(permute_copy_fp8_kernel, dim3(grid), dim3(256), 0, s, static_cast<const uint8_t*>(x),
                       row_of_assign, static_cast<uint8_t*>(x_perm_fp8), T, K, H, r_max, scale, amax);
}

void launch_fill_i32(int32_t* p, int n, int32_t v0, int32_t step, hipStream_t s) {
    hipLaunchKernelGGL(fill_i32_kernel, dim3((n + 63) / 64), dim3(64), 0, s, p, n, v0, step);
}

}  // namespace moe
