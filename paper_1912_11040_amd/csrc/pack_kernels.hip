// Work-item tables of a packed batch, built on the device from the device copy of the offsets.
//
// The example queue of Sec. 2.2 hands over a new padded batch, with new utterance lengths, at every step,
// so the tables that cut a batch into convolution blocks and frame groups are rebuilt per call; doing it
// here keeps the call asynchronous (no host loop over blocks, no blocking copy, no stream wait).
//   first[u]  = number of items of utterances 0..u-1 (exclusive prefix sum of per-utterance item counts)
//   items[i]  = (u, index of item i within utterance u, times `step`)
// Per-utterance item counts: ceil(len_u / conv_block) convolution blocks, ceil(rows_u / frames_per_group)
// frame groups (rows_u = output rows the utterance owns).

#include "aug_internal.h"

namespace aug {
namespace {

constexpr int kScanThreads = 1024;

// One work group: exclusive prefix sums of both item counts over the utterances.  Thread t owns a
// contiguous run of utterances; the runs' totals are scanned across the group through LDS.
__global__ __launch_bounds__(kScanThreads) void pack_prefix_kernel(
    int n_utt, const int64_t* __restrict__ offsets, const int64_t* __restrict__ frame_offsets, int conv_block,
    int frames_per_group, int* __restrict__ conv_first, int* __restrict__ frame_first) {
    __shared__ int part[2][kScanThreads];
    const int tid = threadIdx.x;
    const int per = (n_utt + kScanThreads - 1) / kScanThreads;
    const int u0 = min(tid * per, n_utt), u1 = min(u0 + per, n_utt);
    int sc = 0, sf = 0;
    for (int u = u0; u < u1; ++u) {
        if (conv_first) sc += (int)((offsets[u + 1] - offsets[u] + conv_block - 1) / conv_block);
        if (frame_first) sf += (int)((frame_offsets[u + 1] - frame_offsets[u] + frames_per_group - 1) / frames_per_group);
    }
    part[0][tid] = sc;
    part[1][tid] = sf;
    __syncthreads();
    for (int off = 1; off < kScanThreads; off <<= 1) {          // inclusive scan of the runs' totals
        const int a = tid >= off ? part[0][tid - off] : 0;
        const int b = tid >= off ? part[1][tid - off] : 0;
        __syncthreads();
        part[0][tid] += a;
        part[1][tid] += b;
        __syncthreads();
    }
    int ac = part[0][tid] - sc, af = part[1][tid] - sf;          // exclusive prefix at the run's first utterance
    for (int u = u0; u < u1; ++u) {
        if (conv_first) {
            conv_first[u] = ac;
            ac += (int)((offsets[u + 1] - offsets[u] + conv_block - 1) / conv_block);
        }
        if (frame_first) {
            frame_first[u] = af;
            af += (int)((frame_offsets[u + 1] - frame_offsets[u] + frames_per_group - 1) / frames_per_group);
        }
    }
    if (tid == kScanThreads - 1) {
        if (conv_first) conv_first[n_utt] = part[0][tid];
        if (frame_first) frame_first[n_utt] = part[1][tid];
    }
}

// One thread per item: the utterance that holds it (last u with first[u] <= i; empty utterances share
// their successor's value and are skipped by taking the last) and its index within the utterance.
__global__ void pack_items_kernel(int n_utt, const int* __restrict__ first, int n_items, int step, int2* __restrict__ items) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_items || i >= first[n_utt]) return;
    int lo = 0, hi = n_utt - 1;                                  // invariant: first[lo] <= i
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (first[mid] <= i) lo = mid; else hi = mid - 1;
    }
    items[i] = make_int2(lo, (i - first[lo]) * step);
}

}  // namespace

hipError_t launch_pack(hipStream_t s, int n_utt, const int64_t* d_offsets, const int64_t* d_frame_offsets,
                       int conv_block, int frames_per_group, int* conv_first, int2* conv_items, int64_t n_conv_items,
                       int* frame_first, int2* frame_items, int64_t n_frame_items) {
    if (n_utt <= 0 || (!conv_first && !frame_first)) return hipSuccess;
    pack_prefix_kernel<<<dim3(1), dim3(kScanThreads), 0, s>>>(n_utt, d_offsets, d_frame_offsets, conv_block,
                                                              frames_per_group, conv_first, frame_first);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (conv_first && n_conv_items > 0) {
        pack_items_kernel<<<dim3((unsigned)((n_conv_items + 255) / 256)), dim3(256), 0, s>>>(
            n_utt, conv_first, (int)n_conv_items, 1, conv_items);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (frame_first && n_frame_items > 0) {
        pack_items_kernel<<<dim3((unsigned)((n_frame_items + 255) / 256)), dim3(256), 0, s>>>(
            n_utt, frame_first, (int)n_frame_items, frames_per_group, frame_items);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace aug
