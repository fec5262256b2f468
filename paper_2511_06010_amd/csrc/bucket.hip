// moska_bucket: query aggregation (paper Sec. III-A) as a deterministic counting sort without
// atomics, and the work-tile list the shared-attention kernels consume.
//
// One workgroup per KV head (buckets of different heads never mix, and head h owns exactly
// B*k items, so its output range starts at h*B*k).  The NW waves of the group take contiguous
// slices of the head's items in index order.  Inside a wave, lanes that hold the same chunk id
// find each other with ballots over the id's bits; the lowest such lane bumps the wave's private
// LDS histogram, and every lane derives its rank inside (wave, chunk).  After a barrier the
// histograms are prefix-summed over waves and over chunks, giving each item its final position:
// ascending item index inside every bucket, bit-identical from run to run.
#include "moska_internal.h"

namespace moska {
namespace {

// Exclusive scan of v over the block's threads (blockDim.x a multiple of 64, <= 1024); every
// thread gets its prefix, *total the grand sum.  Wave-level shuffles, then the (at most 16) wave
// totals through LDS.  tmp: 16 ints of LDS.  Two barriers.
__device__ int block_exclusive_scan(int v, int *tmp, int *total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    int incl = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int up = __shfl_up(incl, d);
        if (lane >= d) incl += up;
    }
    if (lane == 63) tmp[wave] = incl;
    __syncthreads();
    int base = 0, sum = 0;
    for (int w = 0; w < nw; ++w) {
        const int t = tmp[w];
        if (w < wave) base += t;
        sum += t;
    }
    *total = sum;
    __syncthreads();
    return base + incl - v;
}

__global__ __launch_bounds__(1024) void bucket_kernel(const int32_t *__restrict__ ids, int32_t *__restrict__ off,
                                                       int32_t *__restrict__ items, int32_t *__restrict__ rank,
                                                       int B, int Hkv, int C, int k, int nbits) {
    extern __shared__ int lds[];
    const int NW = blockDim.x / kWave, wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int h = blockIdx.x;
    const int n = B * k;                          // items of this head
    int *hist = lds;                              // [NW][C]
    int *coff = lds + NW * C;                     // [C] exclusive chunk offsets
    int *tmp = coff + C;                          // [blockDim.x]

    for (int i = threadIdx.x; i < NW * C; i += blockDim.x) hist[i] = 0;
    __syncthreads();

    const int slice = ((n + NW - 1) / NW + kWave - 1) / kWave * kWave;
    const int lo = wave * slice, hi = min(n, lo + slice);
    int *myhist = hist + wave * C;
    const uint64_t below = (1ull << lane) - 1ull;
    // chunk id of item i of this head (0 past the slice); the next batch's ids are requested before the
    // current batch is worked on, so that a batch does not start with a global-memory round trip
    auto id_of = [&](int i) {
        if (i >= hi) return 0;
        const int b = i / k, j = i - b * k;
        return ids[((int64_t)b * Hkv + h) * k + j];
    };
    int cnext = id_of(lo + lane);
    for (int i0 = lo; i0 < hi; i0 += kWave) {
        const int i = i0 + lane;
        const bool valid = i < hi;
        const int c = cnext;
        cnext = id_of(i + kWave);
        uint64_t peers = __ballot(valid);
        for (int bit = 0; bit < nbits; ++bit) {
            const bool one = (c >> bit) & 1;
            const uint64_t m = __ballot(one);
            peers &= one ? m : ~m;
        }
        if (valid) {
            const int r = __popcll(peers & below);
            const int base = myhist[c];           // same-wave LDS accesses execute in order
            rank[(int64_t)h * n + i] = base + r;
            if (r == 0) myhist[c] = base + __popcll(peers);
        }
    }
    __syncthreads();

    // prefix over waves per chunk, chunk totals, then prefix over chunks
    const int per = (C + blockDim.x - 1) / blockDim.x;
    const int c0 = threadIdx.x * per, c1 = min(C, c0 + per);
    int mine = 0;
    for (int c = c0; c < c1; ++c) {
        int run = 0;
        for (int w = 0; w < NW; ++w) {
            const int t = hist[w * C + c];
            hist[w * C + c] = run;
            run += t;
        }
        coff[c] = run;
        mine += run;
    }
    int total;
    int pre = block_exclusive_scan(mine, tmp, &total);
    for (int c = c0; c < c1; ++c) {
        const int t = coff[c];
        coff[c] = pre;
        off[h * C + c] = h * n + pre;
        pre += t;
    }
    if (threadIdx.x == 0 && h == Hkv - 1) off[Hkv * C] = Hkv * n;
    __syncthreads();

    cnext = id_of(lo + lane);
    int rnext = lo + lane < hi ? rank[(int64_t)h * n + lo + lane] : 0;
    for (int i0 = lo; i0 < hi; i0 += kWave) {
        const int i = i0 + lane;
        const int c = cnext, r = rnext;
        cnext = id_of(i + kWave);
        rnext = i + kWave < hi ? rank[(int64_t)h * n + i + kWave] : 0;
        if (i < hi) items[(int64_t)h * n + coff[c] + myhist[c] + r] = i;
    }
}

// ---- the same counting sort over several workgroups per KV head, for heads with very many items
// (B*k in the hundreds of thousands: the single workgroup above would run them one after another) ----
//
//   count    block (h, blk) takes a contiguous slice of the head's items: rank of every item among the
//            slice's items of the same chunk (ballots and wave-private histograms as above), and the
//            slice's histogram hist[h][blk][c]
//   scan     per head: exclusive prefix over the slices for every chunk, then over the chunks; off[]
//            comes out, and hist[h][blk][c] becomes the position of the slice's first item of chunk c
//   scatter  block (h, blk): items[hist[h][blk][c] + rank] = item
// Deterministic and free of atomics like the single-workgroup form, and the same result.

__global__ __launch_bounds__(1024) void bucket_count_kernel(const int32_t *__restrict__ ids, int32_t *__restrict__ rank,
                                                             int32_t *__restrict__ bhist, int B, int Hkv, int C, int k,
                                                             int nbits, int nblk, int per_blk) {
    extern __shared__ int lds[];
    const int NW = blockDim.x / kWave, wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int h = blockIdx.x / nblk, blk = blockIdx.x - h * nblk;
    const int n = B * k;
    int *hist = lds;                              // [NW][C]
    for (int i = threadIdx.x; i < NW * C; i += blockDim.x) hist[i] = 0;
    __syncthreads();
    const int b0 = min(n, blk * per_blk), b1 = min(n, b0 + per_blk);
    const int slice = ((per_blk + NW - 1) / NW + kWave - 1) / kWave * kWave;
    const int lo = min(b1, b0 + wave * slice), hi = min(b1, lo + slice);
    int *myhist = hist + wave * C;
    const uint64_t below = (1ull << lane) - 1ull;
    auto id_of = [&](int i) {
        if (i >= hi) return 0;
        const int b = i / k, j = i - b * k;
        return ids[((int64_t)b * Hkv + h) * k + j];
    };
    int cnext = id_of(lo + lane);
    for (int i0 = lo; i0 < hi; i0 += kWave) {
        const int i = i0 + lane;
        const bool valid = i < hi;
        const int c = cnext;
        cnext = id_of(i + kWave);
        uint64_t peers = __ballot(valid);
        for (int bit = 0; bit < nbits; ++bit) {
            const bool one = (c >> bit) & 1;
            const uint64_t m = __ballot(one);
            peers &= one ? m : ~m;
        }
        if (valid) {
            const int r = __popcll(peers & below);
            const int base = myhist[c];           // same-wave LDS accesses execute in order
            rank[(int64_t)h * n + i] = base + r;
            if (r == 0) myhist[c] = base + __popcll(peers);
        }
    }
    __syncthreads();
    // prefix over the waves per chunk; the slice's totals go to global memory
    int32_t *out = bhist + ((int64_t)h * nblk + blk) * C;
    for (int c = threadIdx.x; c < C; c += blockDim.x) {
        int run = 0;
        for (int w = 0; w < NW; ++w) {
            const int t = hist[w * C + c];
            hist[w * C + c] = run;
            run += t;
        }
        out[c] = run;
    }
    __syncthreads();
    // ranks inside the slice: add the wave's start (each lane re-reads the ranks it wrote itself)
    cnext = id_of(lo + lane);
    for (int i0 = lo; i0 < hi; i0 += kWave) {
        const int i = i0 + lane;
        const int c = cnext;
        cnext = id_of(i + kWave);
        if (i < hi) rank[(int64_t)h * n + i] += myhist[c];
    }
}

constexpr int kScanPer = 16;                      // chunks per thread of the scan kernel: C <= 16384

__global__ __launch_bounds__(1024) void bucket_scan_kernel(int32_t *__restrict__ bhist, int32_t *__restrict__ off, int B,
                                                            int Hkv, int C, int k, int nblk) {
    __shared__ int tmp[16];
    const int h = blockIdx.x, n = B * k;
    int32_t *hh = bhist + (int64_t)h * nblk * C;
    const int per = (C + blockDim.x - 1) / blockDim.x;      // <= kScanPer
    const int c0 = min(C, (int)threadIdx.x * per);
    int tot[kScanPer];
    int mine = 0;
#pragma unroll
    for (int ci = 0; ci < kScanPer; ++ci) {
        const int c = c0 + ci;
        int run = 0;
        if (ci < per && c < C) {
            for (int b = 0; b < nblk; ++b) {
                const int t = hh[(int64_t)b * C + c];
                hh[(int64_t)b * C + c] = run;
                run += t;
            }
        }
        tot[ci] = run;
        mine += run;
    }
    int total;
    int pre = h * n + block_exclusive_scan(mine, tmp, &total);
#pragma unroll
    for (int ci = 0; ci < kScanPer; ++ci) {
        const int c = c0 + ci;
        if (ci < per && c < C) {
            off[h * C + c] = pre;
            for (int b = 0; b < nblk; ++b) hh[(int64_t)b * C + c] += pre;
        }
        pre += tot[ci];
    }
    if (threadIdx.x == 0 && h == Hkv - 1) off[Hkv * C] = Hkv * n;
}

__global__ __launch_bounds__(1024) void bucket_scatter_kernel(const int32_t *__restrict__ ids,
                                                               const int32_t *__restrict__ rank,
                                                               const int32_t *__restrict__ bhist,
                                                               int32_t *__restrict__ items, int B, int Hkv, int C, int k,
                                                               int nblk, int per_blk) {
    const int h = blockIdx.x / nblk, blk = blockIdx.x - h * nblk;
    const int n = B * k;
    const int b0 = min(n, blk * per_blk), b1 = min(n, b0 + per_blk);
    const int32_t *start = bhist + ((int64_t)h * nblk + blk) * C;
    for (int i = b0 + threadIdx.x; i < b1; i += blockDim.x) {
        const int b = i / k, j = i - b * k;
        const int c = ids[((int64_t)b * Hkv + h) * k + j];
        items[start[c] + rank[(int64_t)h * n + i]] = i;
    }
}

// class of the tile that takes `rem` remaining rows of a bucket
__device__ __forceinline__ int tile_class(int rem, int cmin, int cmax) {
    int c = cmin;
    while (c < cmax && class_rows(c) < rem) ++c;
    return c;
}

// Tile list grouped by size class: hdr[c] = first entry of class c, hdr[kNumClasses] = total;
// entry t = (bucket, first row).  A bucket of r rows gives (r-1)/R full tiles of the largest class
// in use (R rows) and one tile of the smallest class that holds the rest.  Thread t owns buckets
// t, t+T, t+2T, ... (coalesced reads of the offsets); inside a class the entries are ordered by
// owner thread, then bucket, so the tiles of one bucket are neighbours.
constexpr int kTileListLds = 15360;     // bucket row counts kept in LDS up to this many buckets

__global__ __launch_bounds__(1024) void tile_list_kernel(const int32_t *__restrict__ off, int NB, int G, int cmin,
                                                          int cmax, int32_t *__restrict__ hdr,
                                                          int32_t *__restrict__ tiles) {
    __shared__ int tmp[16 * kNumClasses];
    __shared__ int cstart[kNumClasses + 1];
    __shared__ int rows_lds[kTileListLds];
    const int T = blockDim.x, tid = threadIdx.x;
    const bool staged = NB <= kTileListLds;
    if (staged) {
        for (int b = tid; b < NB; b += T) rows_lds[b] = (off[b + 1] - off[b]) * G;
        __syncthreads();
    }
    auto rows_of = [&](int b) { return staged ? rows_lds[b] : (off[b + 1] - off[b]) * G; };
    const int R = class_rows(cmax);
    int mine[kNumClasses] = {0, 0, 0, 0, 0};
    for (int b = tid; b < NB; b += T) {
        const int r = rows_of(b);
        if (r <= 0) continue;
        const int nfull = (r - 1) / R, c = tile_class(r - nfull * R, cmin, cmax);
#pragma unroll
        for (int cc = 0; cc < kNumClasses; ++cc) mine[cc] += (cc == c) + (cc == cmax ? nfull : 0);
    }
    // exclusive scan of the five counters over the block's threads in one go: wave-level shuffles,
    // then the (at most 16) wave totals through LDS
    int pre[kNumClasses];
    const int lane = tid & 63, wave = tid >> 6, nw = T >> 6;
#pragma unroll
    for (int cc = 0; cc < kNumClasses; ++cc) {
        int incl = mine[cc];
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int up = __shfl_up(incl, d);
            if (lane >= d) incl += up;
        }
        if (lane == 63) tmp[wave * kNumClasses + cc] = incl;
        pre[cc] = incl - mine[cc];
    }
    __syncthreads();
    int first = 0;                                          // first entry of the class
#pragma unroll
    for (int cc = 0; cc < kNumClasses; ++cc) {
        int before = 0, total = 0;
        for (int w = 0; w < nw; ++w) {
            const int t = tmp[w * kNumClasses + cc];
            if (w < wave) before += t;
            total += t;
        }
        pre[cc] += first + before;
        if (tid == 0) cstart[cc] = first;
        first += total;
    }
    if (tid == 0) cstart[kNumClasses] = first;
    for (int b = tid; b < NB; b += T) {
        const int r = rows_of(b);
        if (r <= 0) continue;
        const int nfull = (r - 1) / R, c = tile_class(r - nfull * R, cmin, cmax);
        int pfull = 0, prem = 0;
#pragma unroll
        for (int cc = 0; cc < kNumClasses; ++cc) {
            if (cc == cmax) { pfull = pre[cc]; pre[cc] += nfull; }
            if (cc == c) prem = pre[cc]++;
        }
        for (int i = 0; i < nfull; ++i) {
            tiles[2 * (pfull + i)] = b;
            tiles[2 * (pfull + i) + 1] = i * R;
        }
        tiles[2 * prem] = b;
        tiles[2 * prem + 1] = nfull * R;
    }
    __syncthreads();
    if (tid <= kNumClasses) hdr[tid] = cstart[tid];
}

}  // namespace

int bucket_slices(const moska_problem_t &p) {
    const int64_t n = (int64_t)p.B * q_len(p) * p.k;        // items per KV head
    if (n < 32768 || p.C > 1024 * kScanPer) return 1;
    const int64_t nblk = (n + 8191) / 8192;                 // slices of about 8192 items
    return (int)(nblk > 64 ? 64 : nblk);
}

int launch_bucket(const moska_problem_t &p, const int32_t *ids, int32_t *off, int32_t *items, int32_t *rank,
                  int32_t *bhist, hipStream_t s) {
    int nbits = 0;
    while ((1 << nbits) < p.C) ++nbits;
    const int nblk = bucket_slices(p);
    if (nblk > 1) {
        int NW = 16;
        while (NW > 1 && (size_t)NW * p.C * sizeof(int) > 144u * 1024u) NW >>= 1;
        const size_t lds = (size_t)NW * p.C * sizeof(int);
        if (lds > 144u * 1024u) return MOSKA_ERR_UNSUPPORTED;
        if (lds > 48 * 1024 &&
            hipFuncSetAttribute((const void *)bucket_count_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) !=
                hipSuccess)
            return MOSKA_ERR_HIP;
        const int64_t n = (int64_t)p.B * p.k;
        const int per_blk = (int)(((n + nblk - 1) / nblk + kWave - 1) / kWave * kWave);
        const dim3 grid((unsigned)(p.Hkv * nblk));
        hipLaunchKernelGGL(bucket_count_kernel, grid, dim3(NW * kWave), lds, s, ids, rank, bhist, p.B, p.Hkv, p.C, p.k,
                           nbits, nblk, per_blk);
        hipLaunchKernelGGL(bucket_scan_kernel, dim3(p.Hkv), dim3(1024), 0, s, bhist, off, p.B, p.Hkv, p.C, p.k, nblk);
        hipLaunchKernelGGL(bucket_scatter_kernel, grid, dim3(1024), 0, s, ids, (const int32_t *)rank,
                           (const int32_t *)bhist, items, p.B, p.Hkv, p.C, p.k, nblk, per_blk);
        return hip_status(hipGetLastError());
    }
    // LDS: NW*C (histograms) + C (offsets) + threads (scan) ints; take as many waves as fit in 144 KiB
    int NW = 16;
    auto need = [&](int nw) { return ((size_t)nw * p.C + p.C + (size_t)nw * kWave) * sizeof(int); };
    while (NW > 1 && need(NW) > 144u * 1024u) NW >>= 1;
    if (need(NW) > 144u * 1024u) return MOSKA_ERR_UNSUPPORTED;
    const int64_t per_head = (int64_t)p.B * p.k;
    while (NW > 1 && (int64_t)(NW / 2) * kWave >= per_head) NW >>= 1;   // no point in idle waves
    const size_t lds = need(NW);
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void *)bucket_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)lds);
        if (e != hipSuccess) return MOSKA_ERR_HIP;
    }
    hipLaunchKernelGGL(bucket_kernel, dim3(p.Hkv), dim3(NW * kWave), lds, s, ids, off, items, rank, p.B, p.Hkv, p.C,
                       p.k, nbits);
    return hip_status(hipGetLastError());
}

int launch_tile_list(const moska_problem_t &p, const int32_t *off, const SharedPlan &pl, int32_t *hdr,
                     int32_t *tiles, hipStream_t s) {
    hipLaunchKernelGGL(tile_list_kernel, dim3(1), dim3(1024), 0, s, off, p.Hkv * p.C, p.Hq / p.Hkv, pl.cmin, pl.cmax,
                       hdr, tiles);
    return hip_status(hipGetLastError());
}

}  // namespace moska
