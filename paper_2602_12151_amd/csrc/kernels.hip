// gfx950 kernels of a decode step: expansion of the plan's records into work-item descriptors, the
// split kernel (one wavefront per work item; the work itself is in decode_body.h, shared with the
// mixed prefill + decode kernel) and the log-sum-exp merge of the splits.
#include "decode_body.h"
#include "launch_util.h"

namespace oserve {
namespace {

using decode_detail::wave_xor_f32;

// Reads the plan's run records and request info from pinned host memory, copies the request info
// into the workspace (for the merge kernel) and expands every run into its work-item descriptors.
// One workgroup; a kernel rather than a memcpy so that the split kernel follows it in the same
// queue without a copy-engine hand-over, and so that only the compact records cross PCIe.
constexpr int kExpandThreads = 1024;
constexpr int kExpandChunk = 1024;  // run records held in LDS per pass (32 KB)
constexpr int kExpandLanes = 16;    // lanes that expand one run together
__global__ __launch_bounds__(kExpandThreads) void expand_plan_kernel(const ExpandParams p) {
    __shared__ uint4 staged[kExpandChunk * 2];
    const int tid = threadIdx.x;
    {
        const uint4* src = reinterpret_cast<const uint4*>(p.req_info_host);
        uint4* dst = reinterpret_cast<uint4*>(p.req_info);
        const int n16 = (p.batch * static_cast<int>(sizeof(RequestInfo)) + 15) / 16;
        for (int i = tid; i < n16; i += kExpandThreads) dst[i] = src[i];
    }
    for (int i = tid; i < p.zero_words; i += kExpandThreads) p.zero[i] = 0;
    {
        const uint4* src = reinterpret_cast<const uint4*>(p.blob_host);
        uint4* dst = reinterpret_cast<uint4*>(p.blob);
        for (int i = tid; i < p.blob_words; i += kExpandThreads) dst[i] = src[i];
    }
    const uint4* src = reinterpret_cast<const uint4*>(p.records_host);
    for (int r0 = 0; r0 < p.num_runs; r0 += kExpandChunk) {
        const int n = min(kExpandChunk, p.num_runs - r0);
        for (int i = tid; i < 2 * n; i += kExpandThreads) staged[i] = src[2 * r0 + i];
        __syncthreads();
        // a group of kExpandLanes lanes per run, one lane per item of the run
        for (int r = tid / kExpandLanes; r < n; r += kExpandThreads / kExpandLanes) {
            const RunRecord rec = reinterpret_cast<const RunRecord*>(staged)[r];
            const int n_items = rec.num_splits * p.num_kv_heads;
            for (int k = tid % kExpandLanes; k < n_items; k += kExpandLanes) {
                const int split = p.num_kv_heads == 1 ? k : static_cast<int>(__umulhi(static_cast<uint32_t>(k), p.kv_heads_magic));
                const int kvh = k - split * p.num_kv_heads;
                const int pbeg = rec.page_begin + split * rec.pages_per_split;
                ItemDesc d;
                d.request_kvh = rec.request | (kvh << kKvHeadShift);
                d.page_begin = pbeg;
                d.page_end = min(rec.page_end, pbeg + rec.pages_per_split);
                d.row = rec.total_splits == 1 ? -1 : rec.row_base + split;
                p.items[rec.first_item + k] = d;
            }
        }
        __syncthreads();
    }
}

template <int D, int NBUF, int WPE>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(WPE, WPE)))
void paged_decode_split_kernel(const SplitParams p) {
    decode_detail::decode_item_body<D, NBUF, false>(p, blockIdx.x, threadIdx.x);
}

// One wavefront per (request, query head) with more than one split:
//   m* = max_s m_s ; w_s = 2^(m_s - m*) ; out = sum_s w_s o_s / sum_s w_s l_s
// Splits are combined in index order, so the result is bit-reproducible.
template <int D>
__global__ __launch_bounds__(64) void paged_decode_merge_kernel(const MergeParams p) {
    constexpr int DPL = D / 64;  // dims per lane
    const int lane = threadIdx.x;
    const int b = blockIdx.x / p.num_q_heads;
    const int h = blockIdx.x - b * p.num_q_heads;
    const RequestInfo info = p.req_info[b];
    const int S = info.num_splits;
    if (S <= 1) return;  // the split kernel already wrote `out` (1), or not a decode request of this launch (0)
    // row of split s: (split_base + s) * Hq + h
    const int64_t row0 = static_cast<int64_t>(info.split_base) * p.num_q_heads + h;
    const int64_t row_step = p.num_q_heads;

    float mmax = -INFINITY;
    for (int s = lane; s < S; s += 64) mmax = fmaxf(mmax, p.partial_ml[(row0 + s * row_step) * 2]);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) mmax = fmaxf(mmax, wave_xor_f32(mmax, off));

    float num[DPL];
#pragma unroll
    for (int d = 0; d < DPL; ++d) num[d] = 0.f;
    float den = 0.f;
#pragma unroll 4
    for (int s = 0; s < S; ++s) {
        const int64_t row = row0 + s * row_step;
        const float w = __builtin_amdgcn_exp2f(p.partial_ml[row * 2] - mmax);
        den += w * p.partial_ml[row * 2 + 1];
        const float* o = p.partial_o + row * D + lane * DPL;
        if constexpr (DPL == 2) {
            const float2 v = *reinterpret_cast<const float2*>(o);
            num[0] += w * v.x;
            num[1] += w * v.y;
        } else {
            num[0] += w * o[0];
        }
    }
    float* dst = p.out + (static_cast<int64_t>(info.q_row) * p.num_q_heads + h) * D + lane * DPL;
    const float inv = 1.f / den;
#pragma unroll
    for (int d = 0; d < DPL; ++d) dst[d] = num[d] * inv;
}

}  // namespace

// The split kernel runs with two pages in flight per wavefront and registers budgeted for one
// wavefront per SIMD: the measured best of the (pages in flight, wavefronts per SIMD) variants.
constexpr int kPagesInFlight = 2;
constexpr int kWavesPerSimd = 1;

hipError_t launch_split(const SplitParams& p, int head_dim, int num_items, hipStream_t stream,
                        hipEvent_t start, hipEvent_t stop) {
    if (num_items <= 0) return hipSuccess;
    if (head_dim == 128)
        return launch_kernel(paged_decode_split_kernel<128, kPagesInFlight, kWavesPerSimd>, dim3(num_items), dim3(64),
                             stream, start, stop, p);
    if (head_dim == 64)
        return launch_kernel(paged_decode_split_kernel<64, kPagesInFlight, kWavesPerSimd>, dim3(num_items), dim3(64),
                             stream, start, stop, p);
    return hipErrorInvalidValue;
}

hipError_t launch_expand(const ExpandParams& p, hipStream_t stream, hipEvent_t done) {
    return launch_kernel(expand_plan_kernel, dim3(1), dim3(kExpandThreads), stream, nullptr, done, p);
}

hipError_t launch_merge(const MergeParams& p, int head_dim, int batch, hipStream_t stream) {
    const int grid = batch * p.num_q_heads;
    if (grid <= 0) return hipSuccess;
    if (head_dim == 128) return launch_kernel(paged_decode_merge_kernel<128>, dim3(grid), dim3(64), stream, nullptr, nullptr, p);
    if (head_dim == 64) return launch_kernel(paged_decode_merge_kernel<64>, dim3(grid), dim3(64), stream, nullptr, nullptr, p);
    return hipErrorInvalidValue;
}

}  // namespace oserve
