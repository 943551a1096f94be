// libnomad: memory-system probes.  They follow no passage of the paper: they measure the machine (streaming copy,
// random 8-byte gathers, random atomics, scattered record appends), so that the ceilings quoted for the epoch
// kernels can be recomputed from known request counts.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "nomad.h"

namespace {

constexpr int kProbeBlock = 256;
constexpr int kProbeGrid = 8192;       // 32 workgroups per compute unit
constexpr int kInFlight = 8;           // independent requests a lane has outstanding

// cheap integer mixer (the probes must not be bound by their index arithmetic)
__device__ __forceinline__ uint32_t mix32(uint32_t x) {
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return x;
}

// Plain streaming copy (16 bytes per lane, grid-stride).
__global__ void __launch_bounds__(kProbeBlock) k_copy_probe(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t count) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += stride) dst[i] = src[i];
}

// Every lane loads `rounds` x kInFlight 8-byte slots at uniformly random positions of the table.
__global__ void __launch_bounds__(kProbeBlock) k_gather_probe(const float2* __restrict__ table, uint32_t slots, uint32_t rounds,
                                                              float* __restrict__ sink) {
    const uint32_t tid = blockIdx.x * kProbeBlock + threadIdx.x;
    float acc = 0.f;
    for (uint32_t r = 0; r < rounds; ++r) {
        const uint32_t h = mix32((tid * rounds + r) * kInFlight);
        float2 v[kInFlight];
#pragma unroll
        for (int g = 0; g < kInFlight; ++g) v[g] = table[__umulhi(mix32(h + (uint32_t)g * 0x9E3779B9u), slots)];
#pragma unroll
        for (int g = 0; g < kInFlight; ++g) acc += v[g].x + v[g].y;
    }
    if (acc == 12345.678f) *sink = acc;   // keeps the loads alive; a table of zeros never writes
}

// KIND 0: two fp32 atomic adds to a random slot; KIND 1: one 64-bit integer atomic add to a random slot
template <int KIND>
__global__ void __launch_bounds__(kProbeBlock) k_atomic_probe(float2* __restrict__ table, uint32_t slots, uint32_t rounds) {
    const uint32_t tid = blockIdx.x * kProbeBlock + threadIdx.x;
    for (uint32_t r = 0; r < rounds; ++r) {
        const uint32_t h = mix32((tid * rounds + r) * kInFlight);
#pragma unroll
        for (int g = 0; g < kInFlight; ++g) {
            const uint32_t idx = __umulhi(mix32(h + (uint32_t)g * 0x9E3779B9u), slots);
            if (KIND == 0) { unsafeAtomicAdd(&table[idx].x, 1.0f); unsafeAtomicAdd(&table[idx].y, 2.0f); }
            else atomicAdd((unsigned long long*)&table[idx], 1ull);
        }
    }
}

// One persistent workgroup of 1,024 lanes per compute unit, each with `chains` private append regions of `cap`
// 12-byte records; every lane appends `per_lane` records, each to a uniformly random chain of its workgroup at the
// position an LDS counter hands out.  GROUP = 1: every record is written by its own lane (a 12-byte partial line
// write per lane); GROUP = 8: eight adjacent lanes write to one chain at consecutive positions (96 contiguous bytes).
template <int GROUP>
__global__ void __launch_bounds__(1024) k_append_probe(uint32_t* __restrict__ table, uint32_t chains, uint32_t cap, uint32_t per_lane) {
    extern __shared__ uint32_t cursor[];
    for (uint32_t c = threadIdx.x; c < chains; c += 1024) cursor[c] = 0;
    __syncthreads();
    uint32_t* mine = table + (size_t)blockIdx.x * chains * cap * 3;
    uint32_t h = mix32(blockIdx.x * 1024u + (threadIdx.x / GROUP) + 12345u);
    for (uint32_t k = 0; k < per_lane; ++k) {
        h = mix32(h + k);
        const uint32_t c = __umulhi(h, chains);
        uint32_t pos = 0;
        if (threadIdx.x % GROUP == 0) pos = atomicAdd(&cursor[c], (uint32_t)GROUP);
        if (GROUP > 1) pos = __shfl(pos, (threadIdx.x & 63) / GROUP * GROUP, 64) + threadIdx.x % GROUP;
        if (pos < cap) {
            uint32_t* dst = mine + ((size_t)c * cap + pos) * 3;
            dst[0] = h; dst[1] = h + 1u; dst[2] = h + 2u;
        }
    }
}

}  // namespace

#pragma GCC visibility push(default)
extern "C" {

int nomad_copy_probe(void* dst, const void* src, uint64_t bytes, void* stream) {
    if (!dst || !src || (bytes & 15u) || (((uintptr_t)dst | (uintptr_t)src) & 15u)) return NOMAD_E_INVALID_ARG;
    if (bytes == 0) return NOMAD_OK;
    hipLaunchKernelGGL(k_copy_probe, dim3(65536), dim3(kProbeBlock), 0, (hipStream_t)stream, (const uint4*)src, (uint4*)dst, (size_t)(bytes / 16));
    return hipGetLastError() == hipSuccess ? NOMAD_OK : NOMAD_E_HIP;
}

int nomad_gather_probe(const void* table, uint64_t table_bytes, uint64_t n_requests, uint64_t* issued_out, void* sink, void* stream) {
    if (!table || !sink || !issued_out || ((uintptr_t)table & 7u) || table_bytes < 8 || (table_bytes >> 3) > 0xFFFFFFFFull) return NOMAD_E_INVALID_ARG;
    const uint64_t per_round = (uint64_t)kProbeGrid * kProbeBlock * kInFlight;
    const uint64_t rounds = (n_requests + per_round - 1) / per_round;
    if (rounds == 0 || rounds > 4096) return NOMAD_E_INVALID_ARG;
    hipLaunchKernelGGL(k_gather_probe, dim3(kProbeGrid), dim3(kProbeBlock), 0, (hipStream_t)stream, (const float2*)table,
                       (uint32_t)(table_bytes >> 3), (uint32_t)rounds, (float*)sink);
    *issued_out = rounds * per_round;
    return hipGetLastError() == hipSuccess ? NOMAD_OK : NOMAD_E_HIP;
}

int nomad_scatter_probe(int kind, void* table, uint64_t table_bytes, uint64_t n_requests, uint32_t chains, uint64_t* issued_out, void* stream) {
    if (!table || !issued_out || ((uintptr_t)table & 7u) || table_bytes < 8) return NOMAD_E_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    if (kind == NOMAD_PROBE_ATOMIC_F32X2 || kind == NOMAD_PROBE_ATOMIC_U64) {
        if ((table_bytes >> 3) > 0xFFFFFFFFull) return NOMAD_E_INVALID_ARG;
        const uint64_t per_round = (uint64_t)kProbeGrid * kProbeBlock * kInFlight;
        const uint64_t rounds = (n_requests + per_round - 1) / per_round;
        if (rounds == 0 || rounds > 4096) return NOMAD_E_INVALID_ARG;
        if (kind == NOMAD_PROBE_ATOMIC_F32X2)
            hipLaunchKernelGGL(k_atomic_probe<0>, dim3(kProbeGrid), dim3(kProbeBlock), 0, st, (float2*)table, (uint32_t)(table_bytes >> 3), (uint32_t)rounds);
        else
            hipLaunchKernelGGL(k_atomic_probe<1>, dim3(kProbeGrid), dim3(kProbeBlock), 0, st, (float2*)table, (uint32_t)(table_bytes >> 3), (uint32_t)rounds);
        *issued_out = rounds * per_round;
    } else if (kind == NOMAD_PROBE_APPEND12 || kind == NOMAD_PROBE_APPEND12_GROUPED) {
        constexpr uint64_t kWorkgroups = 256;
        if (chains < 1 || chains > 16384) return NOMAD_E_INVALID_ARG;
        const uint64_t per_lane = (n_requests + kWorkgroups * 1024 - 1) / (kWorkgroups * 1024);
        if (per_lane == 0 || per_lane > (1u << 20)) return NOMAD_E_INVALID_ARG;
        const uint64_t cap = table_bytes / (kWorkgroups * chains * 12);
        // every chain must be able to take its share with a wide margin, so that no append is dropped in practice
        if (cap > 0xFFFFFFFFull || cap * chains < per_lane * 1024 * 5 / 4 + 64ull * chains) return NOMAD_E_INVALID_ARG;
        if (kind == NOMAD_PROBE_APPEND12)
            hipLaunchKernelGGL(k_append_probe<1>, dim3(kWorkgroups), dim3(1024), chains * sizeof(uint32_t), st, (uint32_t*)table, chains, (uint32_t)cap, (uint32_t)per_lane);
        else
            hipLaunchKernelGGL(k_append_probe<8>, dim3(kWorkgroups), dim3(1024), chains * sizeof(uint32_t), st, (uint32_t*)table, chains, (uint32_t)cap, (uint32_t)per_lane);
        *issued_out = per_lane * kWorkgroups * 1024;
    } else {
        return NOMAD_E_INVALID_ARG;
    }
    return hipGetLastError() == hipSuccess ? NOMAD_OK : NOMAD_E_HIP;
}

}  // extern "C"
#pragma GCC visibility pop
