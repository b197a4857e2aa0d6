// Strategy search (Sec. 6): argmin over candidates, ties to the lowest index.
#pragma once
#include "device_utils.hpp"

namespace distsim {

struct Best {
    int64_t idx;     // -1 = none
    int64_t val;     // batch_ns
    int64_t wgt;     // weight (objective 1), else 1
};

// true iff a is strictly better than b
template <int OBJ>
__device__ __forceinline__ bool better(const Best& a, const Best& b) {
    if (a.idx < 0) return false;
    if (b.idx < 0) return true;
    if (OBJ == 0) {
        if (a.val != b.val) return a.val < b.val;
    } else {
        // a.val / a.wgt < b.val / b.wgt  <=>  a.val * b.wgt < b.val * a.wgt   (128-bit exact)
        const uint64_t lh = __umul64hi((uint64_t)a.val, (uint64_t)b.wgt), ll = (uint64_t)a.val * (uint64_t)b.wgt;
        const uint64_t rh = __umul64hi((uint64_t)b.val, (uint64_t)a.wgt), rl = (uint64_t)b.val * (uint64_t)a.wgt;
        if (lh != rh) return lh < rh;
        if (ll != rl) return ll < rl;
    }
    return a.idx < b.idx;
}

template <int OBJ>
__device__ __forceinline__ Best wave_best(Best a) {
    for (int d = 1; d < kWave; d <<= 1) {
        Best o;
        o.idx = __shfl_xor(a.idx, d, kWave);
        o.val = __shfl_xor(a.val, d, kWave);
        o.wgt = __shfl_xor(a.wgt, d, kWave);
        if (better<OBJ>(o, a)) a = o;
    }
    return a;
}

constexpr int kSearchBlock = 256;
// Eight workgroups per CU, i.e. every wavefront slot of the chip once: a list long enough for HBM
// to matter (2^27 candidates) streams at 5.0 TB/s that way with one 8-byte load per candidate,
// against 3.3 TB/s with half as many workgroups and 4.4 to 4.8 TB/s with two or four times as many;
// several loads per thread and turn (strided) were slower than one (4.7 TB/s); two neighbouring
// candidates per 16-byte non-temporal load: 6.4 TB/s.
constexpr int kSearchMaxBlocks = 2048;

template <int OBJ>
__device__ __forceinline__ Best block_best(Best a) {
    __shared__ Best sh[kSearchBlock / kWave];
    a = wave_best<OBJ>(a);
    if (lane_id() == 0) sh[threadIdx.x / kWave] = a;
    __syncthreads();
    Best r = sh[0];
    for (int i = 1; i < kSearchBlock / kWave; i++) if (better<OBJ>(sh[i], r)) r = sh[i];
    __syncthreads();
    return r;
}

template <int OBJ>
__global__ __launch_bounds__(kSearchBlock) void k_search_partial(const int64_t* __restrict__ batch_ns,
                                                                  const int64_t* __restrict__ weight, int64_t C,
                                                                  Best* __restrict__ partial) {
    // one streaming pass over 8 (16 with weights) bytes per candidate; the order in which
    // candidates meet does not matter (ties go to the lowest index inside better())
    Best a{-1, INT64_MAX, 1};
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    auto take = [&](int64_t c, int64_t val, int64_t wgt) {
        Best b{c, val, wgt};
        if (b.val == INT64_MAX) return;
        if (OBJ == 1 && b.wgt <= 0) return;
        if (better<OBJ>(b, a)) a = b;
    };
    typedef long long i64x2 __attribute__((ext_vector_type(2)));
    const bool wide = (((uintptr_t)batch_ns | (OBJ == 1 ? (uintptr_t)weight : 0)) & 15) == 0;
    if (wide) {
        // two candidates per load, read once and never again: 16-byte streaming loads
        const int64_t pairs = C / 2;
        for (int64_t q = t; q < pairs; q += stride) {
            const i64x2 v = __builtin_nontemporal_load(reinterpret_cast<const i64x2*>(batch_ns) + q);
            i64x2 g{1, 1};
            if (OBJ == 1) g = __builtin_nontemporal_load(reinterpret_cast<const i64x2*>(weight) + q);
            take(2 * q, v.x, g.x);
            take(2 * q + 1, v.y, g.y);
        }
        if ((C & 1) && t == 0) take(C - 1, batch_ns[C - 1], OBJ == 1 ? weight[C - 1] : 1);
    } else {
        for (int64_t c = t; c < C; c += stride) take(c, batch_ns[c], OBJ == 1 ? weight[c] : 1);
    }
    a = block_best<OBJ>(a);
    if (threadIdx.x == 0) partial[blockIdx.x] = a;
}

template <int OBJ>
__global__ __launch_bounds__(kSearchBlock) void k_search_final(const Best* __restrict__ partial, int n,
                                                                int64_t* __restrict__ best) {
    Best a{-1, INT64_MAX, 1};
    for (int i = threadIdx.x; i < n; i += blockDim.x) if (better<OBJ>(partial[i], a)) a = partial[i];
    a = block_best<OBJ>(a);
    if (threadIdx.x == 0) { best[0] = a.idx; best[1] = a.idx < 0 ? INT64_MAX : a.val; }
}

}  // namespace distsim
