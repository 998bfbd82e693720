// Device-wide building blocks used by the grant path: an exclusive scan and a
// stable least-significant-digit radix pass (8-bit digits).  Plain, three
// kernels each; sizes here are tens of millions of items at most.
#pragma once

#include "sja_internal.h"

namespace sja {

// --------------------------------------------------------------------------
// Exclusive scan of int32, in place, any length: per-block scan of 2048
// items, one block scans the block sums, a third kernel adds them back.
// --------------------------------------------------------------------------
constexpr int kScanTile = 2048;

__global__ __launch_bounds__(256) void k_scan_tiles(int32_t *data, int64_t n, int32_t *tile_sums)
{
    __shared__ int s_part[256];
    const int64_t base = int64_t(blockIdx.x) * kScanTile + threadIdx.x * 8;
    int v[8];
    int sum = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        v[i] = (base + i < n) ? data[base + i] : 0;
        sum += v[i];
    }
    s_part[threadIdx.x] = sum;
    __syncthreads();
    for (int d = 1; d < 256; d <<= 1) {
        const int add = threadIdx.x >= d ? s_part[threadIdx.x - d] : 0;
        __syncthreads();
        s_part[threadIdx.x] += add;
        __syncthreads();
    }
    int run = s_part[threadIdx.x] - sum;           // exclusive prefix of this thread
    if (threadIdx.x == 255) tile_sums[blockIdx.x] = s_part[255];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        if (base + i < n) data[base + i] = run;
        run += v[i];
    }
}

__global__ __launch_bounds__(1024) void k_scan_sums(int32_t *sums, int n_tiles, int32_t *total)
{
    __shared__ int s_part[1024];
    __shared__ int s_carry;
    if (threadIdx.x == 0) s_carry = 0;
    __syncthreads();
    for (int b0 = 0; b0 < n_tiles; b0 += 1024) {
        const int i = b0 + threadIdx.x;
        const int mine = i < n_tiles ? sums[i] : 0;
        s_part[threadIdx.x] = mine;
        __syncthreads();
        for (int d = 1; d < 1024; d <<= 1) {
            const int add = threadIdx.x >= d ? s_part[threadIdx.x - d] : 0;
            __syncthreads();
            s_part[threadIdx.x] += add;
            __syncthreads();
        }
        const int carry = s_carry;
        if (i < n_tiles) sums[i] = carry + s_part[threadIdx.x] - mine;
        __syncthreads();
        if (threadIdx.x == 1023) s_carry = carry + s_part[1023];
        __syncthreads();
    }
    if (threadIdx.x == 0 && total) *total = s_carry;
}

__global__ __launch_bounds__(256) void k_scan_add(int32_t *data, int64_t n, const int32_t *tile_sums)
{
    const int add = tile_sums[blockIdx.x];
    const int64_t base = int64_t(blockIdx.x) * kScanTile + threadIdx.x * 8;
#pragma unroll
    for (int i = 0; i < 8; ++i)
        if (base + i < n) data[base + i] += add;
}

// Enqueues an in-place exclusive scan; tile_sums needs ceil(n/2048) ints.
// total (device, may be null) receives the sum of all items.
inline hipError_t enqueue_scan(hipStream_t st, int32_t *data, int64_t n, int32_t *tile_sums, int32_t *total)
{
    if (n <= 0) return hipSuccess;
    const int n_tiles = int((n + kScanTile - 1) / kScanTile);
    hipLaunchKernelGGL(k_scan_tiles, dim3(n_tiles), dim3(256), 0, st, data, n, tile_sums);
    hipLaunchKernelGGL(k_scan_sums, dim3(1), dim3(1024), 0, st, tile_sums, n_tiles, total);
    hipLaunchKernelGGL(k_scan_add, dim3(n_tiles), dim3(256), 0, st, data, n, tile_sums);
    return hipGetLastError();
}

// --------------------------------------------------------------------------
// Stable radix pass over bare 64-bit keys (the grant-list entries), tiles of
// kKeyTile items.  A tile is ranked per wave (each wave owns a contiguous
// quarter, walked in order so the pass stays stable), put in digit order in
// LDS and written out from there, so that items of one digit leave as one
// contiguous run.  hist is digit-major ([256][n_tiles]) so that one exclusive
// scan over it yields every (digit, tile) output offset.  n lives in device
// memory (it is produced by earlier kernels).
// --------------------------------------------------------------------------
constexpr int kKeyTile = 4096;
constexpr int kKeyPerWave = kKeyTile / 4;
constexpr int kKeyChunks = kKeyPerWave / kWave;

// Lanes of the wave (among `valid`) holding the same 8-bit digit as this lane.
__device__ __forceinline__ unsigned long long digit_peers(unsigned d, bool valid)
{
    unsigned long long peers = __ballot(valid);
#pragma unroll
    for (int b = 0; b < 8; ++b) {
        const unsigned long long m = __ballot((d >> b) & 1u);
        peers &= ((d >> b) & 1u) ? m : ~m;
    }
    return peers;
}

__global__ __launch_bounds__(256) void k_keys_hist(const unsigned long long *__restrict__ keys,
                                                   const int32_t *n_ptr, int shift, unsigned digit_mask, int32_t *hist,
                                                   int n_tiles)
{
    __shared__ int s_h[256];
    const int64_t n = *n_ptr;
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    s_h[tid] = 0;
    __syncthreads();
    const int64_t base = int64_t(blockIdx.x) * kKeyTile;
#pragma unroll 4
    for (int r = 0; r < kKeyTile / 256; ++r) {
        const int64_t i = base + r * 256 + tid;
        const bool valid = i < n;
        const unsigned d = valid ? unsigned(keys[i] >> shift) & digit_mask : 0u;
        // counting needs no order: a wave whose keys all carry one digit (the block digits, and
        // any digit of keys that the earlier passes have brought together) adds its count once,
        // any other wave lets every lane add its own one (finding each lane's peers first, as
        // the scatter has to, made this kernel bound by the instructions of that search)
        const unsigned long long live = __ballot(valid);
        if (live == 0) continue;
        const unsigned d0 = unsigned(__builtin_amdgcn_readlane(int(d), __ffsll((long long)live) - 1));
        if (__ballot(valid && d != d0) == 0) {
            if (lane == 0) atomicAdd(&s_h[d0], __popcll(live));
        } else if (valid) {
            atomicAdd(&s_h[d], 1);
        }
    }
    __syncthreads();
    hist[int64_t(tid) * n_tiles + blockIdx.x] = s_h[tid];
}

// What the last pass over list entries writes instead of the keys themselves: 16-byte records
// (job, rank, lo | hi << 8, 0); rank is the key's rank field, lo (6 bits) and hi (7 bits) its
// lowest lane_bits bits, and the job either rides in the key above job_shift (no pass sorts by
// those bits) or, with job_shift < 0, is looked up through the rank (one gather per key).
struct KeyRecords {
    const int2 *ranked;
    uint4 *rec;
    int lane_bits, rank_bits, job_shift;
};

__device__ __forceinline__ uint4 key_record(const KeyRecords &out, unsigned long long v)
{
    const uint32_t rank = uint32_t((v >> out.lane_bits) & ((1ull << out.rank_bits) - 1ull));
    const uint32_t job = out.job_shift >= 0 ? uint32_t(v >> out.job_shift) : uint32_t(out.ranked[rank].x);
    const unsigned int lo = unsigned(v) & 63u, hi = unsigned(v >> 6) & 127u;
    return make_uint4(job, rank, lo | (hi << 8), 0u);
}

// PAY: every key carries a 32-bit payload that moves with it.  REC: the sorted keys are not
// written at all, their records are (the pass that finishes the order of the list entries).
template <bool PAY, bool REC = false>
__global__ __launch_bounds__(256) void k_keys_scatter(const unsigned long long *__restrict__ src,
                                                      unsigned long long *__restrict__ dst,
                                                      const uint32_t *__restrict__ pay_src,
                                                      uint32_t *__restrict__ pay_dst, const int32_t *n_ptr,
                                                      int shift, unsigned digit_mask, const int32_t *__restrict__ hist,
                                                      int n_tiles, KeyRecords out = KeyRecords{})
{
    __shared__ unsigned long long s_key[kKeyTile];
    __shared__ uint32_t s_pay[PAY ? kKeyTile : 1];
    __shared__ int s_cnt[4][256];       // per wave and digit: running count, later the offset inside the digit
    __shared__ int s_start[256];        // first tile-local slot of a digit
    __shared__ int s_goff[256];         // where the tile's items of a digit go
    __shared__ int s_wsum[4];
    const int64_t n = *n_ptr;
    const int64_t base = int64_t(blockIdx.x) * kKeyTile;
    if (base >= n) return;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
#pragma unroll
    for (int w = 0; w < 4; ++w) s_cnt[w][tid] = 0;
    s_goff[tid] = hist[int64_t(tid) * n_tiles + blockIdx.x];
    __syncthreads();

    unsigned long long key[kKeyChunks];
    uint32_t pay[PAY ? kKeyChunks : 1];
    int pos[kKeyChunks];
    const int64_t wbase = base + wave * kKeyPerWave + lane;
#pragma unroll
    for (int c = 0; c < kKeyChunks; ++c) {
        key[c] = wbase + c * kWave < n ? src[wbase + c * kWave] : ~0ull;
        if (PAY) pay[c] = wbase + c * kWave < n ? pay_src[wbase + c * kWave] : 0u;
    }
    volatile int *cnt = &s_cnt[wave][0];
#pragma unroll
    for (int c = 0; c < kKeyChunks; ++c) {
        const bool valid = wbase + c * kWave < n;
        const unsigned d = unsigned(key[c] >> shift) & digit_mask;
        const unsigned long long peers = digit_peers(d, valid);
        const int before = __popcll(peers & ((1ull << lane) - 1ull));
        const int prev = cnt[d];
        pos[c] = prev + before;
        __builtin_amdgcn_wave_barrier();
        if (valid && before == 0) cnt[d] = prev + __popcll(peers);
        __builtin_amdgcn_wave_barrier();
    }
    __syncthreads();

    {   // digit tid: offsets of the four waves inside the digit, then the digits' starts
        const int c0 = s_cnt[0][tid], c1 = s_cnt[1][tid], c2 = s_cnt[2][tid], c3 = s_cnt[3][tid];
        s_cnt[0][tid] = 0; s_cnt[1][tid] = c0; s_cnt[2][tid] = c0 + c1; s_cnt[3][tid] = c0 + c1 + c2;
        const int total = c0 + c1 + c2 + c3;
        int incl = total;
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) {
            const int t = __shfl_up(incl, d, kWave);
            if (lane >= d) incl += t;
        }
        if (lane == kWave - 1) s_wsum[wave] = incl;
        __syncthreads();
        int off = 0;
        for (int w = 0; w < wave; ++w) off += s_wsum[w];
        s_start[tid] = off + incl - total;
    }
    __syncthreads();
#pragma unroll
    for (int c = 0; c < kKeyChunks; ++c) {
        if (wbase + c * kWave < n) {
            const unsigned d = unsigned(key[c] >> shift) & digit_mask;
            const int slot = s_start[d] + s_cnt[wave][d] + pos[c];
            s_key[slot] = key[c];
            if (PAY) s_pay[slot] = pay[c];
        }
    }
    __syncthreads();
    const int count = int(n - base < kKeyTile ? n - base : kKeyTile);
    for (int k = tid; k < count; k += 256) {
        const unsigned long long v = s_key[k];
        const unsigned d = unsigned(v >> shift) & digit_mask;
        const int64_t o = int64_t(s_goff[d]) + (k - s_start[d]);
        if (REC) {
            out.rec[o] = key_record(out, v);
        } else {
            dst[o] = v;
        }
        if (PAY) pay_dst[o] = s_pay[k];
    }
}

// out[i] = keys[idx[i]]: the keys of a permutation, laid out in its order.
__global__ void k_gather_keys(const int32_t *n_ptr, const unsigned long long *__restrict__ keys,
                              const uint32_t *__restrict__ idx, unsigned long long *__restrict__ out)
{
    const int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < *n_ptr) out[i] = keys[idx[i]];
}

// bits[0] |= ~a[i], bits[1] |= ~b[i] over all items: the bytes in which inverted keys differ from "all ones".
__global__ __launch_bounds__(256) void k_key_bits(const int32_t *n_ptr, const unsigned long long *__restrict__ a,
                                                  const unsigned long long *__restrict__ b,
                                                  unsigned long long *bits)
{
    __shared__ unsigned long long s_a[4], s_b[4];
    const int64_t n = *n_ptr;
    unsigned long long oa = 0, ob = 0;
    for (int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; i < n; i += int64_t(gridDim.x) * blockDim.x) {
        oa |= ~a[i];
        ob |= ~b[i];
    }
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        oa |= (unsigned long long)__shfl_xor((long long)oa, d, kWave);
        ob |= (unsigned long long)__shfl_xor((long long)ob, d, kWave);
    }
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    if (lane == 0) { s_a[wave] = oa; s_b[wave] = ob; }
    __syncthreads();
    if (threadIdx.x == 0) {
        atomicOr(&bits[0], s_a[0] | s_a[1] | s_a[2] | s_a[3]);
        atomicOr(&bits[1], s_b[0] | s_b[1] | s_b[2] | s_b[3]);
    }
}

}  // namespace sja
