// Launch interfaces between the C-ABI layer (api.cpp) and the kernel
// translation units.  Every launcher only enqueues on `stream`.
#pragma once

#include <atomic>
#include <hip/hip_runtime.h>

#include "common.h"

namespace va {

struct AttnParams {
    const void* q;        // [T, Hq, D]
    const void* k;        // [T, Hkv, D]
    const void* v;        // [T, Hkv, D]
    void* out;            // [T, Hq, D]
    float* lse;           // [Hq, T]
    const void* dout;     // [T, Hq, D]
    void* dq;             // [T, Hq, D]
    void* dk;             // [T, Hkv, D]
    void* dv;             // [T, Hkv, D]
    float* delta;         // [Hq, T]  -rowsum(dO * O): negated, the dK/dV kernel starts its dP sums from it
    float* lse2;          // [Hq, T]  LSE * log2(e), written by the delta kernel
    const float* q_descale;  // fp8 only
    const float* k_descale;
    const float* v_descale;
    const WorkItem* items;     // device: item records of the work list
    const int32_t* wg_table;   // device: 16 words per persistent workgroup (first descriptor, ids, range)
    const int32_t* work_ids;   // device: item * works_per_item + head chunk
    const WorkItem* merges;    // device: merge records of a dK/dV list (split key tiles)
    float* partials;           // partial-sum slots of split key tiles, in the backward workspace
    int32_t num_merges;
    int32_t dkdv_by_ids;       // dK/dV list: workgroup b runs the work at position b of the id array
    int32_t num_items;
    int32_t num_workgroups;
    int32_t works_per_item;
    int32_t T, Hq, Hkv, D;
    int32_t mask_mode;
    float scale;
};

// Kernels that need more than the default 64 KiB of dynamic LDS must say so once per device (a process
// may drive several).  One DynamicLds object per launch site remembers the devices it has served.
struct DynamicLds {
    std::atomic<unsigned long long> served{0};  // bit d: device d has the attribute
    hipError_t allow(const void* kernel, size_t bytes) {
        if (bytes <= 64 * 1024) return hipSuccess;
        int dev = -1;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        const bool tracked = dev >= 0 && dev < 64;
        if (tracked && (served.load(std::memory_order_acquire) >> dev & 1ull)) return hipSuccess;
        e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
        if (e == hipSuccess && tracked) served.fetch_or(1ull << dev, std::memory_order_release);
        return e;
    }
};
// expands to an expression of type hipError_t; the lambda gives every launch site (and every template
// instantiation of it) a DynamicLds of its own
#define VA_ALLOW_DYNAMIC_LDS(kernel, bytes)                                   \
    ([&]() -> hipError_t {                                                    \
        static ::va::DynamicLds site;                                         \
        return site.allow(reinterpret_cast<const void*>(kernel), (bytes));    \
    }())

hipError_t launch_fwd_bf16(const AttnParams& p, hipStream_t stream);
// blockwise: the three descale arrays are per token row and head instead of per head
hipError_t launch_fwd_fp8(const AttnParams& p, bool blockwise, hipStream_t stream);
hipError_t launch_bwd_delta(const AttnParams& p, hipStream_t stream);
hipError_t launch_bwd_dkdv(const AttnParams& p, hipStream_t stream);
hipError_t launch_bwd_dq(const AttnParams& p, hipStream_t stream);
hipError_t launch_quantize_e4m3(const void* x, int32_t T, int32_t H, int32_t D, void* codes, float* descale,
                                hipStream_t stream);
hipError_t launch_quantize_e4m3_blockwise(const void* x, const int32_t* cu_device, int32_t num_seqs, int32_t T,
                                          int32_t num_blocks, int32_t H, int32_t D, void* codes, float* descale_tok,
                                          hipStream_t stream);

}  // namespace va
