// Steps in front of event-flow generation: identical operators share one event (Sec. 4.1,
// event generator), and the elapsed time of a communication event follows from its profile
// (Sec. 4.2: point-to-point = min(SEND, RECV); all-reduce over more than 8 devices = the 8-device
// profile rescaled by the ring volume 2(N-1)/N).
#pragma once
#include "device_utils.hpp"

namespace distsim {

constexpr int kMaxRecordWords = 16;
constexpr int kScanBlock = 1024;

// finalizer of the SplitMix64 generator (Steele, Lea, Flood 2014), used as a bit mixer
__device__ __forceinline__ uint64_t mix64(uint64_t x) {
    x += 0x9e3779b97f4a7c15ull;
    x = (x ^ (x >> 30)) * 0xbf58476d1ce4e5b9ull;
    x = (x ^ (x >> 27)) * 0x94d049bb133111ebull;
    return x ^ (x >> 31);
}

__global__ __launch_bounds__(256) void k_dedup_clear(int32_t* __restrict__ table, int64_t size) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < size) table[i] = -1;
}

// Open addressing with linear probing over record indices.  A slot is claimed by the first
// record that finds it empty; records with equal words join the slot and lower its entry to the
// smallest index among them, records with other words probe on.  The table has at least 2n
// slots, so every probe sequence meets an empty slot within `size` steps.
// Equal records are merged inside the workgroup first (a small table in LDS over the workgroup's
// own records, same probing): only one record per distinct operator of the workgroup, carrying the
// smallest index among its equals, goes to the table in memory, and the others take its slot.  A
// popular operator is in nearly every wavefront; without the merge all of them would read the same
// slot and the same representative record, one L2 channel serving them one after the other.
constexpr int kDedupBlock = 512, kDedupLocal = 2 * kDedupBlock;
constexpr int kDedupStagedWords = 12;        // records of up to that many words are staged in LDS (48 KB)
__global__ __launch_bounds__(kDedupBlock) void k_dedup_insert(const int64_t* __restrict__ rec, int64_t n, int K,
                                                              int32_t* table, int64_t size, int32_t* __restrict__ slot_of) {
    const bool in_lds = K <= kDedupStagedWords;     // the launch brings K * kDedupBlock * 8 bytes of dynamic LDS then
    __shared__ int32_t local[kDedupLocal];      // thread that claimed the local slot | bits of its hash << 9, -1 = empty
    __shared__ int32_t lowest[kDedupBlock];     // by claiming thread: smallest record index among its equals
    __shared__ int32_t global_slot[kDedupBlock];
    // the workgroup's records, word k of thread t at staged[k * kDedupBlock + t]: a record that meets
    // an equal one in the workgroup's table is compared with it here, not through memory
    extern __shared__ int64_t staged[];
    const int tid = threadIdx.x;
    const int64_t base = (int64_t)blockIdx.x * kDedupBlock, i = base + tid;
    for (int q = tid; q < kDedupLocal; q += kDedupBlock) local[q] = -1;
    lowest[tid] = INT32_MAX;
    __syncthreads();
    int64_t w[kMaxRecordWords];
    uint64_t h = 0;
    int leader = -1;
    if (i < n) {
#pragma unroll
        for (int k = 0; k < kMaxRecordWords; k++) {
            if (k < K) { w[k] = rec[i * K + k]; h = mix64(h ^ (uint64_t)w[k]); if (in_lds) staged[k * kDedupBlock + tid] = w[k]; }
        }
    }
    __syncthreads();
    if (i < n) {
        // the workgroup's own table: other bits of the hash than the table in memory uses
        // an entry is the claiming thread and 22 more bits of its hash, so that records are compared
        // word for word only when those agree
        static_assert(kDedupBlock == 512, "nine bits for the thread");
        int pos = (int)(h >> 40) & (kDedupLocal - 1);
        const int32_t mine = (int32_t)((h >> 8 & 0x3fffff) << 9) | tid;
        for (int probe = 0; probe < kDedupLocal && leader < 0; probe++) {
            int32_t cur = local[pos];
            if (cur == -1) {
                cur = atomicCAS(&local[pos], -1, mine);
                if (cur == -1) { leader = tid; break; }
            }
            bool same = (cur >> 9) == (mine >> 9);
            if (same) {
#pragma unroll
                for (int k = 0; k < kMaxRecordWords; k++)
                    if (k < K && (in_lds ? staged[k * kDedupBlock + (cur & 511)] : rec[(base + (cur & 511)) * K + k]) != w[k]) same = false;
            }
            if (same) leader = cur & 511;
            else pos = (pos + 1) & (kDedupLocal - 1);
        }
        if (leader >= 0) atomicMin(&lowest[leader], (int32_t)i);
    }
    __syncthreads();
    if (i < n && leader == tid) {
        const int32_t first = lowest[tid];          // stands for all its equals in the workgroup
        int64_t slot = (int64_t)(h & (uint64_t)(size - 1));
        int32_t found = -1;
        for (int64_t probe = 0; probe < size && found < 0; probe++) {
            // look before locking (an ordinary load: a stale value only costs an atomic that changes
            // nothing, because a slot goes from empty to an index and then only to lower indices of
            // equal records)
            int32_t cur = table[slot];
            if (cur == -1) {
                cur = atomicCAS(&table[slot], -1, first);
                if (cur == -1) { found = (int32_t)slot; break; }
            }
            bool same = true;
#pragma unroll
            for (int k = 0; k < kMaxRecordWords; k++)
                if (k < K && rec[(int64_t)cur * K + k] != w[k]) same = false;
            if (same) {
                if (cur > first) atomicMin(&table[slot], first);
                found = (int32_t)slot;
            } else {
                slot = (slot + 1) & (size - 1);
            }
        }
        global_slot[tid] = found;
    }
    __syncthreads();
    if (i < n) slot_of[i] = leader >= 0 ? global_slot[leader] : -1;
}

// Exclusive prefix count of the first occurrences (records that are their slot's entry), per
// block of kScanBlock records, and the block's total.
__global__ __launch_bounds__(kScanBlock) void k_dedup_scan_blocks(const int32_t* __restrict__ table,
                                                                  const int32_t* __restrict__ slot_of, int64_t n,
                                                                  int32_t* __restrict__ excl, int32_t* __restrict__ block_tot) {
    __shared__ int32_t wave_tot[kScanBlock / kWave];
    const int64_t i = (int64_t)blockIdx.x * kScanBlock + threadIdx.x;
    const int lane = lane_id(), wv = threadIdx.x / kWave;
    const bool first = i < n && slot_of[i] >= 0 && table[slot_of[i]] == (int32_t)i;
    const uint64_t b = __builtin_amdgcn_ballot_w64(first);
    const int before = __popcll(b & ((1ull << lane) - 1));
    if (lane == 0) wave_tot[wv] = __popcll(b);
    __syncthreads();
    int base = 0, tot = 0;
    for (int k = 0; k < kScanBlock / kWave; k++) { if (k < wv) base += wave_tot[k]; tot += wave_tot[k]; }
    if (i < n) excl[i] = base + before;
    if (threadIdx.x == 0) block_tot[blockIdx.x] = tot;
}

// Exclusive scan of the block totals in place (one workgroup); the grand total goes to
// num_events.
__global__ __launch_bounds__(kScanBlock) void k_dedup_scan_totals(int32_t* block_tot, int64_t nb, int64_t* num_events) {
    __shared__ int32_t wave_tot[kScanBlock / kWave];
    __shared__ int32_t carry_s;
    const int lane = lane_id(), wv = threadIdx.x / kWave;
    if (threadIdx.x == 0) carry_s = 0;
    __syncthreads();
    for (int64_t b0 = 0; b0 < nb; b0 += kScanBlock) {
        const int64_t i = b0 + threadIdx.x;
        const int32_t v = i < nb ? block_tot[i] : 0;
        int32_t inc = v;
        for (int d = 1; d < kWave; d <<= 1) { const int32_t o = __shfl_up(inc, d, kWave); if (lane >= d) inc += o; }
        if (lane == kWave - 1) wave_tot[wv] = inc;
        __syncthreads();
        int32_t base = carry_s;
        for (int k = 0; k < wv; k++) base += wave_tot[k];
        if (i < nb) block_tot[i] = base + inc - v;
        __syncthreads();
        if (threadIdx.x == kScanBlock - 1) carry_s = base + inc;
        __syncthreads();
    }
    if (threadIdx.x == 0) *num_events = carry_s;
}

// Event ids in order of first occurrence, and each event's representative record.
__global__ __launch_bounds__(256) void k_dedup_assign(const int32_t* __restrict__ table, const int32_t* __restrict__ slot_of,
                                                      const int32_t* __restrict__ excl, const int32_t* __restrict__ block_tot,
                                                      int64_t n, int32_t* __restrict__ event_id, int32_t* __restrict__ rep) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int32_t s = slot_of[i];
    if (s < 0) { event_id[i] = -1; return; }
    const int32_t r = table[s];
    const int32_t id = excl[r] + block_tot[r / kScanBlock];
    event_id[i] = id;
    if (r == (int32_t)i) rep[id] = r;
}

// Elapsed time of communication events from their profiles.
//   kind 0, point-to-point: the transmission lasts min(SEND call, RECV call).
//   kind 1, all-reduce over `ranks` devices: the profile itself up to 8 devices; above, the
//   8-device profile times [2(N-1)/N] / [2*7/8] = 8(N-1) / (7N), truncated.
// Anything else, a rank count below 1 or a negative time gives -1.
__global__ __launch_bounds__(256) void k_comm_event_times(int64_t n, const int32_t* __restrict__ kind,
                                                          const int32_t* __restrict__ ranks, const int64_t* __restrict__ t_a,
                                                          const int64_t* __restrict__ t_b, int64_t* __restrict__ elapsed) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int kd = kind[i];
    const int64_t N = ranks[i], a = t_a[i];
    int64_t e = -1;
    if (kd == 0) {
        const int64_t b = t_b[i];
        if (a >= 0 && b >= 0) e = a < b ? a : b;
    } else if (kd == 1 && N >= 1 && a >= 0) {
        if (N <= 8) e = a;
        else {
            // floor(a * 8(N-1) / (7N)) without leaving 64 bits.  With a = q * 7N + r the result is
            // q * 8(N-1) + floor(x (N-1) / (7N)), x = 8r < 56N; and with x = 7c + b that last term
            // is c + floor((b N - x) / (7N)), whose numerator lies in (-8 * 7N, 7N).
            const int64_t den = 7 * N;
            const int64_t q = a / den, r = a % den;
            const int64_t x = 8 * r, c = x / 7, b = x % 7;
            const int64_t s = b * N - x;
            const int64_t fl = s >= 0 ? s / den : -((-s + den - 1) / den);
            e = q * (8 * (N - 1)) + c + fl;
        }
    }
    elapsed[i] = e;
}

}  // namespace distsim
