// Host-side helpers shared by the stand-alone entry points (index, quality measures, initialisation).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>
#include <vector>

#include "nomad.h"

namespace {

struct Buffers {   // device allocations of one call, released on every path
    std::vector<void*> ptrs;
    ~Buffers() { for (void* p : ptrs) (void)hipFree(p); }
    template <typename T>
    hipError_t alloc(T** p, size_t count) {
        *p = nullptr;
        hipError_t e = hipMalloc((void**)p, std::max<size_t>(count, 1) * sizeof(T));
        if (e == hipSuccess) ptrs.push_back(*p);
        return e;
    }
};

#define KTRY(call)                                                          \
    do {                                                                    \
        hipError_t e_ = (call);                                             \
        if (e_ != hipSuccess) return e_ == hipErrorOutOfMemory ? NOMAD_E_OOM : NOMAD_E_HIP; \
    } while (0)

inline uint32_t blocks_of(int64_t items, int per) { return (uint32_t)((items + per - 1) / per); }

}  // namespace
