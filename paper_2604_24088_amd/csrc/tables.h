// Kernel-argument tables: which tensors a launch works on.
//
// Every kernel takes its tensors as one table passed BY VALUE in the kernel-argument segment (no
// device-side pointer table, nothing to allocate or copy).  The ordinary entry points fill in one
// tensor; the batched entry points up to kMaxBatch, so that many small tensors (the shards of one
// exchange, the tensors of several layers) share the ramp-up and the drain of a single launch.  A
// workgroup finds its tensor with locate(): a binary search over the prefix sums of the tensors'
// workgroup counts, uniform over the workgroup (scalar loads and compares; none for one tensor).
// Only the entries a kernel reads are ever fetched from the argument segment.
//
// Tables are indexed directly (tab.item[i]), never through a pointer to a member, so that the
// compiler reads them with scalar loads from the argument segment and makes no private copy.
#pragma once

#include <stdint.h>

namespace taco {

constexpr int kMaxK = 16;             // payloads one decode can add (TACO_MAX_K)
constexpr int kMaxBatch = 32;         // tensors per batched launch (TACO_MAX_BATCH)
constexpr int kMaxBatchSources = 128; // payloads of all tensors of a batched decode together

// Largest i < count with first[i] <= wg (first[0] = 0): binary search, five dependent scalar loads at most
// (a linear scan over 32 entries costs a one-shot workgroup a fifth of its life).
__device__ __forceinline__ int last_not_above(const int64_t (&first)[kMaxBatch + 1], int count, int64_t wg) {
    int lo = 0;
    if (count > 1) {
#pragma unroll
        for (int step = kMaxBatch / 2; step >= 1; step >>= 1) {
            const int mid = lo + step;
            if (mid < count && wg >= first[mid]) lo = mid;
        }
    }
    return lo;
}

// ---- compress: x -> payload, scales -------------------------------------------------------------

struct CompressItem {
    const void* x;      // n bf16 values
    void* payload;      // codes (split layout) or records (interleaved)
    void* scales;       // {alpha, s} records; unused in the interleaved layout
    int64_t n;          // elements
};

struct CompressTable {
    CompressItem item[kMaxBatch];
    int64_t first[kMaxBatch + 1];       // first workgroup of tensor i; first[count] = workgroups of the launch
    __device__ __forceinline__ void locate(int64_t wg, int count, int& idx, int64_t& local) const {
        idx = last_not_above(first, count, wg);
        local = wg - first[idx];
    }
    __device__ __forceinline__ const void* x(int i) const { return item[i].x; }
    __device__ __forceinline__ void* payload(int i) const { return item[i].payload; }
    __device__ __forceinline__ void* scales(int i) const { return item[i].scales; }
    __device__ __forceinline__ int64_t n(int i) const { return item[i].n; }
};

// ---- decode: k payloads (+ scales) -> bf16 sum, or -> re-compressed payload -----------------------

struct DecodeTable {
    const void* src_payload[kMaxBatchSources];      // payload i of tensor t at [t * k + i]
    const void* src_scales[kMaxBatchSources];
    void* out[kMaxBatch];
    void* payload_out[kMaxBatch];
    void* scales_out[kMaxBatch];
    int64_t n_elems[kMaxBatch];
    int64_t first[kMaxBatch + 1];
    __device__ __forceinline__ void locate(int64_t wg, int count, int& idx, int64_t& local) const {
        idx = last_not_above(first, count, wg);
        local = wg - first[idx];
    }
    __device__ __forceinline__ const void* payload(int t, int k, int i) const { return src_payload[t * k + i]; }
    __device__ __forceinline__ const void* scales(int t, int k, int i) const { return src_scales[t * k + i]; }
    __device__ __forceinline__ void* output(int t) const { return out[t]; }
    __device__ __forceinline__ void* payload_output(int t) const { return payload_out[t]; }
    __device__ __forceinline__ void* scales_output(int t) const { return scales_out[t]; }
    __device__ __forceinline__ int64_t n(int t) const { return n_elems[t]; }
};

}  // namespace taco
