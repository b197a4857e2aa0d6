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

// DPP controls that pair every lane with the lane holding the other half of a 2-, 4-, 8- and
// 16-lane block: two quad permutations, then the mirrored half-row and the mirrored row.
constexpr int kDppXor1 = 0xB1;          // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;          // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141;   // row_half_mirror
constexpr int kDppMirror = 0x140;       // row_mirror

template <int CTRL>
__device__ __forceinline__ int dpp_i32(int v) { return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, true); }
template <int CTRL>
__device__ __forceinline__ int64_t dpp_i64(int64_t v) {
    const int lo = dpp_i32<CTRL>((int)(uint32_t)v), hi = dpp_i32<CTRL>((int)(uint32_t)((uint64_t)v >> 32));
    return (int64_t)(((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo);
}
__device__ __forceinline__ int64_t readlane_i64(int64_t v, int l) {
    const int lo = __builtin_amdgcn_readlane((int)(uint32_t)v, l);
    const int hi = __builtin_amdgcn_readlane((int)(uint32_t)((uint64_t)v >> 32), l);
    return (int64_t)(((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo);
}

// Reduction over aligned groups of `width` lanes (a wave-uniform power of two <= 64); every lane
// of the group gets the result.  DPP inside a row of 16 lanes, scalar row totals above.
template <typename Op>
__device__ __forceinline__ int64_t group_reduce(int64_t v, int width, Op op) {
    if (width >= 2) v = op(v, dpp_i64<kDppXor1>(v));
    if (width >= 4) v = op(v, dpp_i64<kDppXor2>(v));
    if (width >= 8) v = op(v, dpp_i64<kDppHalfMirror>(v));
    if (width >= 16) v = op(v, dpp_i64<kDppMirror>(v));
    if (width >= 32) {
        const int64_t a = op(readlane_i64(v, 0), readlane_i64(v, 16));
        const int64_t b = op(readlane_i64(v, 32), readlane_i64(v, 48));
        v = width == 64 ? op(a, b) : ((threadIdx.x & 32) ? b : a);
    }
    return v;
}
__device__ __forceinline__ int64_t group_max(int64_t v, int width) {
    return group_reduce(v, width, [](int64_t x, int64_t y) { return x > y ? x : y; });
}
__device__ __forceinline__ int64_t group_sum(int64_t v, int width) {
    return group_reduce(v, width, [](int64_t x, int64_t y) { return x + y; });
}
// true in every lane of a group in which some lane has `b` set
__device__ __forceinline__ bool group_any(bool b, int width) {
    const uint64_t m = __builtin_amdgcn_ballot_w64(b);
    if (width == 64) return m != 0;
    const int base = (threadIdx.x & 63) & ~(width - 1);
    return ((m >> base) & ((1ull << width) - 1)) != 0;
}
// number of lanes of the group that have `b` set
__device__ __forceinline__ int group_count(bool b, int width) {
    const uint64_t m = __builtin_amdgcn_ballot_w64(b);
    if (width == 64) return __popcll(m);
    const int base = (threadIdx.x & 63) & ~(width - 1);
    return __popcll((m >> base) & ((1ull << width) - 1));
}
// max over the wavefront, wave-uniform
__device__ __forceinline__ int wave_max_i32(int v) {
    auto mx = [](int x, int y) { return x > y ? x : y; };
    v = mx(v, dpp_i32<kDppXor1>(v));
    v = mx(v, dpp_i32<kDppXor2>(v));
    v = mx(v, dpp_i32<kDppHalfMirror>(v));
    v = mx(v, dpp_i32<kDppMirror>(v));
    return mx(mx(__builtin_amdgcn_readlane(v, 0), __builtin_amdgcn_readlane(v, 16)),
              mx(__builtin_amdgcn_readlane(v, 32), __builtin_amdgcn_readlane(v, 48)));
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

// max of two doubles that are known not to be NaN: one instruction (the builtin first rewrites
// each operand that it cannot prove canonical)
__device__ __forceinline__ double max_f64(double a, double b) {
    double r;
    asm("v_max_f64 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}

// Sum / maximum of doubles over aligned groups of `width` lanes, as group_reduce does for integers.
template <int CTRL>
__device__ __forceinline__ double dpp_f64(double v) {
    return __longlong_as_double(dpp_i64<CTRL>(__double_as_longlong(v)));
}
__device__ __forceinline__ double readlane_f64(double v, int l) {
    return __longlong_as_double(readlane_i64(__double_as_longlong(v), l));
}
template <typename Op>
__device__ __forceinline__ double group_reduce_f64(double v, int width, Op op) {
    if (width >= 2) v = op(v, dpp_f64<kDppXor1>(v));
    if (width >= 4) v = op(v, dpp_f64<kDppXor2>(v));
    if (width >= 8) v = op(v, dpp_f64<kDppHalfMirror>(v));
    if (width >= 16) v = op(v, dpp_f64<kDppMirror>(v));
    if (width >= 32) {
        const double a = op(readlane_f64(v, 0), readlane_f64(v, 16));
        const double b = op(readlane_f64(v, 32), readlane_f64(v, 48));
        v = width == 64 ? op(a, b) : ((threadIdx.x & 32) ? b : a);
    }
    return v;
}
__device__ __forceinline__ double group_sum_f64(double v, int width) {
    return group_reduce_f64(v, width, [](double x, double y) { return x + y; });
}
__device__ __forceinline__ double group_max_f64(double v, int width) {
    return group_reduce_f64(v, width, [](double x, double y) { return max_f64(x, y); });
}

// Exact conversion of a double that holds an integer of [0, 2^53) (five instructions).
__device__ __forceinline__ int64_t double_to_i64(double d) {
    const uint32_t hi = (uint32_t)(d * (1.0 / 4294967296.0));              // truncates
    const uint32_t lo = (uint32_t)__fma_rn(-(double)hi, 4294967296.0, d);
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

// The same for an integer of [0, 2^52): adding 2^52 puts the integer into the low mantissa bits.
__device__ __forceinline__ int64_t small_double_to_i64(double d) {
    return __double_as_longlong(d + 4503599627370496.0) & 0xfffffffffffffll;
}

// Boundary s of the uniform partition of L layers into `parts` parts: floor(s L / parts) for
// 0 <= s <= parts <= 64 and L <= 255.  The product is below 2^15, so the fp32 quotient (reciprocal
// and product, a few units in the last place) is off by at most one; the remainder corrects it.
__device__ __forceinline__ int uniform_bound(int s, int L, int parts) {
    const int x = s * L;
    int q = (int)__fdividef((float)x, (float)parts);
    const int r = x - q * parts;
    if (r < 0) q--;
    else if (r >= parts) q++;
    return q;
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

// The same with the reciprocal of the divisor at hand (a divisor used many times): one
// multiplication instead of the division; the fix-up makes the quotient exact whatever the
// rounding of the product (its error is a few units for quotients below 2^53).
__device__ __forceinline__ uint64_t udiv64_by(uint64_t num, uint64_t den, double inv_den) {
    if (((num | den) >> 53) == 0) {
        uint64_t q = (uint64_t)((double)num * inv_den);
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
    int32_t blocking;          // 1: p2p events occupy the sender; 2: sends queue on their link
    double inv_gpus_per_node;  // 1 / gpus_per_node (set on the host)
    double gpus_per_node_f;    // gpus_per_node as a double (set on the host: a kernel argument stays in scalar registers)
    double inv_bucket;         // 1 / bucket, 0 when there are no buckets (set on the host)
};

// Node of the first rank of pipeline position s when a position spans tpdp < gpus_per_node
// ranks: floor(s * tpdp / gpus_per_node) for s < 64.  The product is exact in fp64 and the
// quotient is below 64, so one multiplication by the reciprocal and an exact remainder give it.
__device__ __forceinline__ int node_of_position(const ClusterDev& cl, int s, int tpdp) {
    const double x = (double)s * (double)tpdp, g = cl.gpus_per_node_f;
    int q = (int)(x * cl.inv_gpus_per_node);
    const double r = __fma_rn(-(double)q, g, x);
    if (r < 0.0) q--;
    else if (r >= g) q++;
    return q;
}

__device__ __forceinline__ int64_t p2p_ns(const ClusterDev& cl, int64_t bytes, int k) {
    return cl.alpha[k] + (int64_t)udiv64((uint64_t)bytes, (uint64_t)cl.beta[k]);
}
__device__ __forceinline__ int64_t allreduce_ns(const ClusterDev& cl, int64_t n, int64_t bytes) {
    if (n <= 1 || bytes <= 0) return 0;
    const int k = n <= cl.gpus_per_node ? 0 : 1;
    return cl.alpha[k] + (int64_t)udiv64(2ull * (uint64_t)(n - 1) * (uint64_t)bytes, (uint64_t)n * (uint64_t)cl.beta[k]);
}
// The same with the reciprocal of n * beta at hand (k_layer_tables keeps it per (variant, pp) row).
__device__ __forceinline__ int64_t allreduce_ns_by(const ClusterDev& cl, int64_t n, int64_t bytes, double inv_den) {
    if (n <= 1 || bytes <= 0) return 0;
    const int k = n <= cl.gpus_per_node ? 0 : 1;
    return cl.alpha[k] + (int64_t)udiv64_by(2ull * (uint64_t)(n - 1) * (uint64_t)bytes, (uint64_t)n * (uint64_t)cl.beta[k], inv_den);
}
__device__ __forceinline__ int64_t alltoall_ns(const ClusterDev& cl, int64_t n, int64_t bytes) {
    if (n <= 1 || bytes <= 0) return 0;
    const int k = n <= cl.gpus_per_node ? 0 : 1;
    return cl.alpha[k] + (int64_t)udiv64((uint64_t)(n - 1) * (uint64_t)bytes, (uint64_t)n * (uint64_t)cl.beta[k]);
}

}  // namespace distsim
