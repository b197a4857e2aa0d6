// Wavefront-level helpers for gfx950 (64-lane wavefronts).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace distsim {

constexpr int kWave = 64;

// DPP controls of the GCN3/CDNA ISA ("wavefront shift by one lane").
constexpr int kDppWaveShl1 = 0x130;   // lane i reads lane i+1
constexpr int kDppWaveShr1 = 0x138;   // lane i reads lane i-1

// Value held by the previous lane (lane 0 receives 0).  Two v_mov_b32 with a DPP modifier.
__device__ __forceinline__ double from_prev_lane(double x) {
    int lo = __double2loint(x), hi = __double2hiint(x);
    lo = __builtin_amdgcn_update_dpp(0, lo, kDppWaveShr1, 0xf, 0xf, true);
    hi = __builtin_amdgcn_update_dpp(0, hi, kDppWaveShr1, 0xf, 0xf, true);
    return __hiloint2double(hi, lo);
}

// Value held by the next lane (lane 63 receives 0).
__device__ __forceinline__ double from_next_lane(double x) {
    int lo = __double2loint(x), hi = __double2hiint(x);
    lo = __builtin_amdgcn_update_dpp(0, lo, kDppWaveShl1, 0xf, 0xf, true);
    hi = __builtin_amdgcn_update_dpp(0, hi, kDppWaveShl1, 0xf, 0xf, true);
    return __hiloint2double(hi, lo);
}

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }

// max / sum over aligned groups of `width` lanes (width a power of two <= 64); every lane of
// the group gets the result.
__device__ __forceinline__ int64_t group_max(int64_t v, int width) {
    for (int d = 1; d < width; d <<= 1) {
        int64_t o = __shfl_xor(v, d, kWave);
        v = o > v ? o : v;
    }
    return v;
}
__device__ __forceinline__ int64_t group_sum(int64_t v, int width) {
    for (int d = 1; d < width; d <<= 1)
        v += __shfl_xor(v, d, kWave);
    return v;
}
__device__ __forceinline__ int wave_max_i32(int v) {
    for (int d = 1; d < kWave; d <<= 1) {
        int o = __shfl_xor(v, d, kWave);
        v = o > v ? o : v;
    }
    return v;
}

// Inclusive prefix sum over the 64 lanes of a wavefront.
__device__ __forceinline__ int64_t wave_inclusive_sum(int64_t v) {
    const int lane = lane_id();
    for (int d = 1; d < kWave; d <<= 1) {
        int64_t o = __shfl_up(v, d, kWave);
        if (lane >= d) v += o;
    }
    return v;
}

// Truncating unsigned division.  Operands below 2^53 (the usual case) go through one
// correctly rounded fp64 division and an exact integer fix-up of the quotient; anything
// larger takes the generic 64-bit path.
__device__ __forceinline__ uint64_t udiv64(uint64_t num, uint64_t den) {
    if (((num | den) >> 53) == 0) {
        uint64_t q = (uint64_t)((double)num / (double)den);
        int64_t r = (int64_t)(num - q * den);
        while (r < 0) { q--; r += (int64_t)den; }
        while (r >= (int64_t)den) { q++; r -= (int64_t)den; }
        return q;
    }
    return num / den;
}

// ---- collective cost events (Sec. 4.2 ring volume; integer, truncating) ---------------

struct ClusterDev {
    int32_t num_devices, gpus_per_node;
    int64_t alpha[2], beta[2];
    int64_t bucket;
    int32_t blocking;          // p2p events occupy the sender
};

__device__ __forceinline__ int64_t p2p_ns(const ClusterDev& cl, int64_t bytes, int k) {
    return cl.alpha[k] + (int64_t)udiv64((uint64_t)bytes, (uint64_t)cl.beta[k]);
}
__device__ __forceinline__ int64_t allreduce_ns(const ClusterDev& cl, int64_t n, int64_t bytes) {
    if (n <= 1 || bytes <= 0) return 0;
    const int k = n <= cl.gpus_per_node ? 0 : 1;
    return cl.alpha[k] + (int64_t)udiv64(2ull * (uint64_t)(n - 1) * (uint64_t)bytes, (uint64_t)n * (uint64_t)cl.beta[k]);
}
__device__ __forceinline__ int64_t alltoall_ns(const ClusterDev& cl, int64_t n, int64_t bytes) {
    if (n <= 1 || bytes <= 0) return 0;
    const int k = n <= cl.gpus_per_node ? 0 : 1;
    return cl.alpha[k] + (int64_t)udiv64((uint64_t)(n - 1) * (uint64_t)bytes, (uint64_t)n * (uint64_t)cl.beta[k]);
}

}  // namespace distsim
