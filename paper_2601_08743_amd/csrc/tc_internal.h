// Internal declarations shared by the host side of libtablecache and its kernel files.
// Nothing here is part of the public ABI (see include/tablecache.h).
#pragma once
#include <hip/hip_runtime.h>
#include <atomic>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "tc_types.h"

namespace tc {

// Where a kernel goes: the stream, and optionally two events that receive the dispatch's own begin
// and end timestamps (per-kernel timing without bracketing packets on the stream).
struct Launch {
    hipStream_t stream;
    hipEvent_t start, stop;
};
#define TC_LAUNCH(kernel, grid, lds_bytes, L, ...) \
    hipExtLaunchKernelGGL(kernel, dim3(grid), dim3(256), (lds_bytes), (L).stream, (L).start, (L).stop, 0, __VA_ARGS__)

// A kernel's dynamic-LDS limit (hipFuncSetAttribute) is a property of the kernel on one device: each
// launcher keeps one of these per kernel and raises the limit the first time it launches on a device.
// (Two threads that race on a device's first launch both set the same value.)
struct PerDeviceOnce {
    static constexpr int kDevices = 64;
    std::atomic<unsigned char> done[kDevices];
    template <typename F>
    hipError_t run(F &&set_attributes)
    {
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        if (dev < 0 || dev >= kDevices) return hipErrorInvalidDevice;
        if (done[dev].load(std::memory_order_acquire)) return hipSuccess;
        e = set_attributes();
        if (e == hipSuccess) done[dev].store(1, std::memory_order_release);
        return e;
    }
};

// kv_stitch.hip
hipError_t launch_stitch(const Geom &g, const BatchDev &b, int l0, int l1, bool rope, const Launch &L);
hipError_t launch_format(const Geom &g, const void *raw, int64_t v_part, int n_tokens, int first_block, int l0,
                         int l1, const Launch &L);
hipError_t launch_append(const Geom &g, const BatchDev &b, int layer, const void *k_new,
                         const void *v_new, const Launch &L);
hipError_t launch_readback(const Geom &g, int layer, const int32_t *blocks_dev, int n_tokens,
                           void *k_out_dev, void *v_out_dev, hipStream_t s);
// prefill_attn_bf16.hip / prefill_attn_f32.hip
hipError_t launch_attn_bf16(const Geom &g, const BatchDev &b, const AttnArgs &a, int row_blocks, bool pipelined,
                            const Launch &L);
// decode_attn_bf16.hip
hipError_t launch_append_blocks(const Geom &g, const BatchDev &b, int layer, const void *k_new, const void *v_new,
                                int n_blocks, const Launch &L);
hipError_t launch_attn_pp_bf16(const Geom &g, const BatchDev &b, const AttnArgs &a, const Launch &L);
hipError_t launch_decode_bf16(const Geom &g, const BatchDev &b, const AttnArgs &a, const Launch &L);
hipError_t launch_decode_finish(const Geom &g, const BatchDev &b, const AttnArgs &a, int max_splits, const Launch &L);
hipError_t launch_attn_f32(const Geom &g, const BatchDev &b, const AttnArgs &a, const Launch &L);
hipError_t launch_merge(const Geom &g, const BatchDev &b, const AttnArgs &a, const Launch &L);
hipError_t launch_merge_bf16(const Geom &g, const AttnArgs &a, const MergeGroup *groups, int n_groups,
                             int row_blocks, const Launch &L);

}  // namespace tc
