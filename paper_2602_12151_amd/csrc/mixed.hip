// gfx950 kernel: one launch for a batch that holds both decode requests (one query token, HBM-bound)
// and prefill chunks (many query tokens, MFMA-bound) - the spatially heterogeneous batch of paper
// section 1 (i) and section 2 ("Workload heterogeneity": short compute-bound requests next to long
// memory-bound ones).
//
// What was measured on the part about running the two kinds together:
//   * Giving the two kinds separate compute units gains nothing (it loses 13-25 %).  The decode
//     side's K/V stream is limited by the memory requests each compute unit can keep in flight, so
//     it needs all of the units to keep HBM busy; whatever units the prefill side takes, the decode
//     side loses in proportion.
//   * A compute unit that holds prefill wavefronts and decode wavefronts at the same time, one of
//     each per SIMD, does both in less time than one after the other (9 % less on uniform work).
//     Left to itself the hardware dispatcher does not produce that pairing: workgroups of one
//     launch go wherever room is, and compute units fill up with one kind.
// So the launch is built to make the pairing happen.  It has two workgroups of four wavefronts (one
// per SIMD) per compute unit, and each lasts for the whole launch and takes its work from queues.
// Registers and LDS are budgeted so that a compute unit holds exactly two of them, and the
// dispatcher places the first workgroup of every compute unit of an XCD before the second; the
// workgroups that come first are "prefill workgroups", the ones that come second "decode
// workgroups".  A prefill workgroup works through prefill items (prefill_body.h), all four
// wavefronts on one item; each wavefront of a decode workgroup works through decode items
// (decode_body.h) on its own.  Every SIMD thus runs a prefill wavefront's MFMAs
// next to a decode wavefront's K/V stream for as long as both queues last.  A workgroup whose queue
// has run dry turns to the other queue, so the tail of the launch is all decode (eight wavefronts per
// compute unit) or all prefill (two items per compute unit).  Should the dispatcher place workgroups
// differently, the result is the same and only the pairing is lost.
//
// Queues: counters in device memory (cleared by the kernel that precedes this one on the stream);
// decode items are taken in launch order (largest first) from one queue; prefill items from one
// queue per XCD (the blocks of one (request, kv head) are in one XCD's queue so that they share its
// L2), the other XCDs' queues when its own is empty.  Which wavefront computes an item does not
// change the item's result, so the output is the same bit for bit from run to run.
#include "decode_body.h"
#include "prefill_body.h"
#include "launch_util.h"

namespace oserve {
namespace {

constexpr int kMixedWaves = kPrefillWaves;         // wavefronts of a workgroup
constexpr int kMixedThreads = 64 * kMixedWaves;

// The two kinds of work as functions of their own (not inlined), each with its queue loop inside.
// Compiled into one function, each kind's register pressure spoils the other's instruction schedule
// (the prefill code loses its software pipelining: every LDS read waits for the one before); as
// functions each is compiled like the kernel it also exists as.  The loop over a queue's items is
// inside the function because a function saves the registers it must preserve to scratch memory on
// entry and reloads them on exit (30 KB per wavefront for the prefill function): called per item
// that was 3 % of the launch's time; called once per phase it is 80 MB of scratch traffic per launch.
// The functions read their parameters from the kernel-argument segment, in the constant address
// space: scalar loads into scalar registers, as in a kernel.  (Handed over by reference the
// parameters would be vector-memory loads where they are used, and waiting for one of those also
// waits for every tile or page load in flight.)
typedef const __attribute__((address_space(4))) MixedParams* KernelArgs;
typedef __attribute__((address_space(3))) int* LdsInts;

// Next prefill item for the workgroup (the same value in all of its wavefronts), or -1 when every queue is
// empty.  Its own XCD's queue first, then the others in turn.
__device__ inline int take_prefill(KernelArgs a, int xcd, LdsInts picked, int& turn) {
    if (threadIdx.x == 0) {
        int item = -1;
        const int nx = a->num_xcds;
        for (int k = 0; k < nx && item < 0; ++k) {
            const int x = (xcd + k) % nx;
            const int n = a->prefill_queue_size[x];
            if (n == 0) continue;
            const int i = atomicAdd(a->queue_next + x, 1);
            if (i < n) item = a->prefill_queue_first[x] + i;
        }
        picked[turn] = item;
    }
    __syncthreads();
    const int item = picked[turn];
    turn ^= 1;                        // the slot is written again only after another barrier
    return __builtin_amdgcn_readfirstlane(item);
}

// All four wavefronts of the workgroup on one prefill item after the other, until the queues are empty.
template <int D>
__device__ __attribute__((noinline)) void run_prefill_items(KernelArgs a, int xcd, prefill_detail::lds_byte* lds, LdsInts picked) {
    PrefillParams u;
    u.items = a->prefill.items; u.q = a->prefill.q; u.k_pages = a->prefill.k_pages; u.v_pages = a->prefill.v_pages;
    u.block_table = a->prefill.block_table; u.out = a->prefill.out; u.scale_log2e = a->prefill.scale_log2e;
    u.num_q_heads = a->prefill.num_q_heads; u.num_kv_heads = a->prefill.num_kv_heads; u.group = a->prefill.group;
    u.group_shift = a->prefill.group_shift; u.max_pages_per_seq = a->prefill.max_pages_per_seq;
    u.tile_shift = a->prefill.tile_shift;
    int turn = 0;
#pragma nounroll
    for (int item = take_prefill(a, xcd, picked, turn); item >= 0; item = take_prefill(a, xcd, picked, turn))
        prefill_detail::prefill_item_body<D>(u, u.items + item, lds, prefill_detail::WorkgroupBarrier{},
                                             static_cast<int>(threadIdx.x) >> 6);
}

// Each wavefront on its own, one decode item after the other, until the queue is empty.
template <int D>
__device__ __attribute__((noinline)) void run_decode_items(KernelArgs a) {
    SplitParams u;
    u.items = a->decode.items; u.req_info = a->decode.req_info; u.q = a->decode.q; u.k_pages = a->decode.k_pages;
    u.v_pages = a->decode.v_pages; u.block_table = a->decode.block_table; u.context_lens = a->decode.context_lens;
    u.out = a->decode.out; u.partial_o = a->decode.partial_o; u.partial_ml = a->decode.partial_ml;
    u.scale_log2e = a->decode.scale_log2e; u.num_q_heads = a->decode.num_q_heads; u.num_kv_heads = a->decode.num_kv_heads;
    u.group = a->decode.group; u.max_pages_per_seq = a->decode.max_pages_per_seq; u.tile_shift = a->decode.tile_shift;
    const int lane = threadIdx.x & 63;
    const int n = a->num_decode_items;
    int32_t* next = a->queue_next + kMaxQueueXcds;
#pragma nounroll
    for (;;) {
        int item = 0;
        if (lane == 0) item = atomicAdd(next, 1);
        item = __builtin_amdgcn_readfirstlane(item);
        if (item >= n) break;
        decode_detail::decode_item_body<D, 2, true>(u, item, lane);
    }
}

template <int D>
__global__ __launch_bounds__(kMixedThreads) __attribute__((amdgpu_waves_per_eu(2, 2)))
void paged_mixed_kernel(const MixedParams p) {
    __shared__ __align__(16) unsigned char lds[prefill_detail::prefill_lds_bytes<D>()];
    __shared__ int picked[2];             // the prefill item the workgroup takes next (two slots, used in turn)

    // MixedParams is the kernel's only argument, so it sits at the start of the kernel-argument segment
    const KernelArgs args = (KernelArgs)__builtin_amdgcn_kernarg_segment_ptr();
    // Workgroups go to the XCDs in turn; inside an XCD the first units_per_xcd of them are the first
    // workgroups of its compute units, the following ones the second.
    const int xcd = blockIdx.x % p.num_xcds;
    const int units_per_xcd = max(1, static_cast<int>(gridDim.x) / (2 * p.num_xcds));
    const bool prefill_first = ((blockIdx.x / p.num_xcds) / units_per_xcd) % 2 == 0;
    // a prefill workgroup: prefill queues first, then the decode queue; a decode workgroup the other way
    // round (the first barrier of its prefill phase waits until all four wavefronts have left the decode queue)
#pragma nounroll
    for (int phase = 0; phase < 2; ++phase) {
        if ((phase == 0) == prefill_first) {
            __builtin_amdgcn_s_setprio(0);
            run_prefill_items<D>(args, xcd, (prefill_detail::lds_byte*)lds, (LdsInts)picked);
        } else {
            // Decode wavefronts issue few instructions and every delay of theirs is a gap in the K/V
            // stream, so they get the higher issue priority.
            __builtin_amdgcn_s_setprio(2);
            run_decode_items<D>(args);
        }
    }
}

}  // namespace

hipError_t launch_mixed(const MixedParams& p, int head_dim, int num_workgroups, hipStream_t stream,
                        hipEvent_t start, hipEvent_t stop) {
    if (num_workgroups <= 0) return hipSuccess;
    if (head_dim == 128) return launch_kernel(paged_mixed_kernel<128>, dim3(num_workgroups), dim3(kMixedThreads), stream, start, stop, p);
    if (head_dim == 64) return launch_kernel(paged_mixed_kernel<64>, dim3(num_workgroups), dim3(kMixedThreads), stream, start, stop, p);
    return hipErrorInvalidValue;
}

}  // namespace oserve
