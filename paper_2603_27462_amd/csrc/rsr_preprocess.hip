// One-time preprocessing kernels of librsr (paper, System Overview, "Algorithm
// overview", and Kernels Implementation):
//   encode       pattern code of every (block, column)
//   sort         per block, stable counting sort of the columns by code, done
//                digit group by digit group (each pass is a counting sort over
//                4 or 9 buckets: count, scan, stable placement), then the group
//                boundaries over all P codes
//   stream_len / pack_stream / finalize_stream
//                the compact stream the multiply kernel reads: 16-bit entries,
//                zero-contribution group dropped, one tail flag per group,
//                laid out for coalesced per-lane strips
#include <cstdlib>

#include "rsr_internal.h"

namespace rsr {

namespace {

constexpr int kThreads = 256;  // workgroup size of every preprocessing kernel
constexpr int kWaves = kThreads / 64;

__device__ __forceinline__ int digit_of(int m, int mode) {
    switch (mode) {
        case MODE_BINARY: return (m == 0) ? 0 : (m == 1) ? 1 : -1;
        case MODE_POS: return (m == 1) ? 1 : (m == 0 || m == -1) ? 0 : -1;
        case MODE_NEG: return (m == -1) ? 1 : (m == 0 || m == 1) ? 0 : -1;
        default: return (m == 0) ? 0 : (m == 1) ? 1 : (m == -1) ? 2 : -1;
    }
}

// code[b][j] = sum_r digit(M[b*k+r][j]) * base^r; rows past the end are zero.
__global__ __launch_bounds__(kThreads) void k_encode(const int8_t *__restrict__ M, int64_t rows,
                                                     int64_t cols, int k, int mode, int64_t nb,
                                                     uint16_t *__restrict__ code,
                                                     int *__restrict__ err_flag) {
    const int64_t cols_pad = (cols + kThreads - 1) / kThreads * kThreads;
    const int64_t gid = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int64_t b = gid / cols_pad;
    const int64_t j = gid % cols_pad;
    if (b >= nb || j >= cols) return;
    const uint32_t base = (mode == MODE_FUSED3) ? 3u : 2u;
    uint32_t c = 0, weight = 1;
    bool bad = false;
    for (int r = 0; r < k; ++r) {
        const int64_t i = b * k + r;
        if (i < rows) {
            int d = digit_of(M[i * cols + j], mode);
            if (d < 0) { bad = true; d = 0; }
            c += (uint32_t)d * weight;
        }
        weight *= base;
    }
    if (bad) atomicOr(err_flag, 1);
    code[b * cols + j] = (uint16_t)c;
}

__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t x) {
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        uint32_t y = __shfl_up(x, d, 64);
        if (lane >= d) x += y;
    }
    return x;
}

// Exclusive scan of one value per thread over the workgroup; *total gets the sum.
// wsum: kWaves words of LDS.  Contains two barriers.
__device__ __forceinline__ uint32_t wg_exclusive_scan(uint32_t x, uint32_t *wsum, uint32_t *total) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const uint32_t incl = wave_inclusive_scan(x);
    if (lane == 63) wsum[w] = incl;
    __syncthreads();
    uint32_t before = 0, all = 0;
#pragma unroll
    for (int i = 0; i < kWaves; ++i) {
        const uint32_t t = wsum[i];
        if (i < w) before += t;
        all += t;
    }
    __syncthreads();
    *total = all;
    return before + incl - x;
}

// Stable sort of the columns of each block by pattern code.  R = buckets per
// digit pass (4 = two binary digits, 9 = two ternary digits).  Each thread
// owns a contiguous strip of positions, so placing strip after strip in
// thread order keeps equal keys in their previous order.
template <int R>
__global__ __launch_bounds__(kThreads) void k_sort(const uint16_t *__restrict__ code, int64_t nb,
                                                   int n, int passes, int64_t P,
                                                   uint16_t *__restrict__ pi,
                                                   uint32_t *__restrict__ off) {
    extern __shared__ unsigned char smem[];
    const int npad = (n + 7) & ~7;
    uint16_t *A = reinterpret_cast<uint16_t *>(smem);
    uint16_t *B = A + npad;
    uint32_t *cnt = reinterpret_cast<uint32_t *>(B + npad);  // [R][kThreads]
    uint32_t *wsum = cnt + R * kThreads;                      // [kWaves]
    const int tid = threadIdx.x;
    const int L = (n + kThreads - 1) / kThreads;
    const int lo = min(n, tid * L), hi = min(n, lo + L);

    for (int64_t b = blockIdx.x; b < nb; b += gridDim.x) {
        const uint16_t *cb = code + b * n;
        for (int t = tid; t < n; t += kThreads) A[t] = (uint16_t)t;
        __syncthreads();
        uint32_t div = 1;
        for (int pass = 0; pass < passes; ++pass) {
#pragma unroll
            for (int d = 0; d < R; ++d) cnt[d * kThreads + tid] = 0;
            for (int t = lo; t < hi; ++t) {                      // count
                const uint32_t d = ((uint32_t)cb[A[t]] / div) % R;
                cnt[d * kThreads + tid] += 1;
            }
            __syncthreads();
            // exclusive scan over the bucket-major array cnt[R*kThreads]
            uint32_t local[R], sum = 0;
#pragma unroll
            for (int i = 0; i < R; ++i) { local[i] = cnt[tid * R + i]; sum += local[i]; }
            uint32_t total;
            uint32_t run = wg_exclusive_scan(sum, wsum, &total);
#pragma unroll
            for (int i = 0; i < R; ++i) { cnt[tid * R + i] = run; run += local[i]; }
            __syncthreads();
            for (int t = lo; t < hi; ++t) {                      // stable placement
                const uint16_t j = A[t];
                const uint32_t d = ((uint32_t)cb[j] / div) % R;
                const uint32_t dst = cnt[d * kThreads + tid]++;
                B[dst] = j;
            }
            __syncthreads();
            uint16_t *tmp = A; A = B; B = tmp;
            div *= R;
        }
        // A is pi_b.  Group boundaries: off[c] = first position whose code >= c.
        uint16_t *pib = pi + b * n;
        uint32_t *ob = off + b * (P + 1);
        for (int t = tid; t < n; t += kThreads) {
            const uint16_t j = A[t];
            pib[t] = j;
            const int64_t ccur = cb[j];
            const int64_t cprev = t ? (int64_t)cb[A[t - 1]] : -1;
            for (int64_t c = cprev + 1; c <= ccur; ++c) ob[c] = (uint32_t)t;
            if (t == n - 1)
                for (int64_t c = ccur + 1; c <= P; ++c) ob[c] = (uint32_t)n;
        }
        __syncthreads();
    }
}

// lens[b] = stream entries of block b: columns outside group 0 plus one
// placeholder for every empty group among codes 1..P-1; *longest = max over blocks
// (the caller zeroes it).
__global__ __launch_bounds__(kThreads) void k_stream_len(const uint32_t *__restrict__ off,
                                                         int64_t nb, int64_t n, int64_t P,
                                                         uint32_t *__restrict__ lens,
                                                         uint32_t *__restrict__ longest) {
    __shared__ uint32_t empties;
    for (int64_t b = blockIdx.x; b < nb; b += gridDim.x) {
        const uint32_t *ob = off + b * (P + 1);
        if (threadIdx.x == 0) empties = 0;
        __syncthreads();
        uint32_t mine = 0;
        for (int64_t c = 1 + threadIdx.x; c < P; c += kThreads) mine += (ob[c + 1] == ob[c]);
        if (mine) atomicAdd(&empties, mine);
        __syncthreads();
        if (threadIdx.x == 0) {
            const uint32_t len = (uint32_t)(n - ob[1]) + empties;
            lens[b] = len;
            atomicMax(longest, len);
        }
        __syncthreads();
    }
}

// Stream of block b: for code c = 1..P-1 in order, the columns of group c in
// ascending order (entry = column<<1, last one |1), or one placeholder entry
// (zero slot = index n, tail bit set) when the group is empty; then filler
// entries (zero slot, no tail) up to S.  Hence every code 1..P-1 owns exactly
// one tail entry, and a reader can recover codes by counting tails.
__global__ __launch_bounds__(kThreads) void k_pack_stream(const uint16_t *__restrict__ pi,
                                                          const uint32_t *__restrict__ off,
                                                          int64_t nb, int n, int64_t P, int64_t S,
                                                          uint16_t *__restrict__ stream) {
    __shared__ uint32_t wsum[kWaves];
    const uint16_t zero_entry = (uint16_t)(n << 1);
    for (int64_t b = blockIdx.x; b < nb; b += gridDim.x) {
        const uint16_t *pib = pi + b * n;
        const uint32_t *ob = off + b * (P + 1);
        uint16_t *sb = stream + b * S;
        const uint32_t off1 = ob[1];
        uint32_t carry = 0;
        for (int64_t c0 = 1; c0 < P; c0 += kThreads) {
            const int64_t c = c0 + threadIdx.x;
            const bool valid = c < P;
            const uint32_t s = valid ? ob[c] : 0, e = valid ? ob[c + 1] : 0;
            const uint32_t empty = (valid && s == e) ? 1u : 0u;
            uint32_t total;
            const uint32_t eb = carry + wg_exclusive_scan(empty, wsum, &total);
            if (valid) {
                const uint32_t dst = s - off1 + eb;
                if (empty) {
                    sb[dst] = zero_entry | 1;
                } else {
                    for (uint32_t t = s; t < e; ++t)
                        sb[dst + (t - s)] = (uint16_t)((pib[t] << 1) | (t + 1 == e ? 1 : 0));
                }
            }
            carry += total;
        }
        const int64_t len = (int64_t)(n - off1) + carry;
        for (int64_t t = len + threadIdx.x; t < S; t += kThreads) sb[t] = zero_entry;
    }
}

// Reorders the logical stream inside its groups so that the LDS gathers of the multiply
// kernel collide less.  Gather instruction i of a wave reads entry i of all 64 strips of a
// chunk; the LDS serves the two half-waves side by side and needs one cycle per distinct
// dword that falls on the same of its 32 banks.  The order of the columns inside a group
// is free for the kernel (sums commute up to rounding; the canonical pi is not touched),
// so for every run of entries of one group inside a strip, each slot takes the remaining
// column whose bank (for a bf16 vector: (col / 2) mod 32) is least loaded so far in that
// slot of the half-wave; two more sweeps re-place every strip against all the others.
// One wave per (block, chunk): thread = (half-wave, slot), strips in order; the first slot
// of a run places the run.
constexpr int kSpreadSweeps = 3;
constexpr int kSpreadMaxRun = 8;

__global__ __launch_bounds__(64) void k_spread_banks(uint16_t *__restrict__ logical, int64_t nb,
                                                     int64_t C, int H) {
    __shared__ uint8_t load[2][32][33];   // [half][slot][bank], padded
    __shared__ uint16_t strip[64][33];    // the chunk: [strip][slot], padded
    const int epl = 8 * H;
    const int half = threadIdx.x >> 5, slot = threadIdx.x & 31;
    const bool live = slot < epl;
    for (int64_t chunk = blockIdx.x; chunk < nb * C; chunk += gridDim.x) {
        uint16_t *cb = logical + chunk * 64 * epl;
        for (int i = threadIdx.x; i < 64 * epl; i += 64) strip[i / epl][i % epl] = cb[i];
        for (int k = 0; k < 33; ++k) load[half][slot][k] = 0;
        __syncthreads();
        for (int sweep = 0; sweep < kSpreadSweeps; ++sweep) {
            for (int l = 0; l < 32; ++l) {
                uint16_t *st = strip[32 * half + l];
                // slots past the strip count as tails, so that no run reaches into them
                const uint32_t entry = live ? st[slot] : 1u;
                const uint32_t tail = entry & 1u;
                const uint64_t ball = __ballot(tail != 0);
                const uint32_t tails = (uint32_t)(ball >> (32 * half));
                if (live) {
                    st[slot] = (uint16_t)(entry >> 1);  // columns only while the strip is placed
                    if (sweep > 0) --load[half][slot][(entry >> 2) & 31];
                }
                __syncthreads();
                const bool start = live && (slot == 0 || ((tails >> (slot - 1)) & 1u));
                if (start) {
                    const uint32_t rest = tails >> slot;
                    int e = rest ? slot + __builtin_ctz(rest) : epl - 1;
                    if (e > epl - 1) e = epl - 1;
                    // (long runs -- filler behind the last group, or one very common pattern --
                    // are counted as they stand: placing them would cost run^2 steps)
                    const bool place = e - slot < kSpreadMaxRun;
                    for (int sl = slot; sl <= e; ++sl) {
                        int best = sl;
                        uint8_t bl = load[half][sl][(st[sl] >> 1) & 31];
                        for (int t = sl + 1; place && t <= e; ++t) {
                            const uint8_t x = load[half][sl][(st[t] >> 1) & 31];
                            if (x < bl) { bl = x; best = t; }
                        }
                        const uint16_t c = st[best];
                        st[best] = st[sl];
                        st[sl] = c;
                        ++load[half][sl][(c >> 1) & 31];
                    }
                }
                __syncthreads();
                if (live) st[slot] = (uint16_t)((st[slot] << 1) | tail);
            }
        }
        __syncthreads();
        for (int i = threadIdx.x; i < 64 * epl; i += 64) cb[i] = strip[i / epl][i % epl];
        __syncthreads();
    }
}

// Final layout of the stream (see PassData): re-encodes the entries, moves
// them to the lane-major slabs, and records for every lane strip the group
// code of the first tail at or after its start (1 + tails before it).  Also
// checks that the block holds exactly P-1 tails.
__global__ __launch_bounds__(kThreads) void k_finalize_stream(
    const uint16_t *__restrict__ logical, int64_t nb, int64_t P, int64_t C, int H, int enc,
    uint16_t *__restrict__ entries, uint16_t *__restrict__ codes, int *__restrict__ err_flag) {
    __shared__ uint32_t wsum[kWaves];
    const int epl = 8 * H;
    const int64_t S = C * 64 * epl;
    const int64_t strips = C * 64;
    for (int64_t b = blockIdx.x; b < nb; b += gridDim.x) {
        const uint16_t *lb = logical + b * S;
        uint32_t carry = 1;
        for (int64_t g0 = 0; g0 < strips; g0 += kThreads) {
            const int64_t g = g0 + threadIdx.x;
            uint32_t cnt = 0;
            if (g < strips)
                for (int i = 0; i < epl; ++i) cnt += lb[g * epl + i] & 1u;
            uint32_t total;
            const uint32_t ex = wg_exclusive_scan(cnt, wsum, &total);
            if (g < strips) {
                const int64_t chunk = g >> 6;
                const int lane = (int)(g & 63);
                codes[(b * C + chunk) * 64 + lane] = (uint16_t)(carry + ex);
                for (int i = 0; i < epl; ++i) {
                    const uint32_t e = lb[g * epl + i];
                    const uint32_t out = (enc == kEncSmall) ? (((e & 1u) << 15) | (e & 0xfffeu)) : e;
                    entries[(((b * C + chunk) * H + (i >> 3)) * 64 + lane) * 8 + (i & 7)] =
                        (uint16_t)out;
                }
            }
            carry += total;
        }
        if (threadIdx.x == 0 && (int64_t)carry != P) atomicOr(err_flag, 2);
    }
}

// Plain fill (used instead of a memset node so that callers may capture the sequence).
__global__ __launch_bounds__(kThreads) void k_fill_u32(uint32_t *__restrict__ p, uint32_t value,
                                                       int64_t count) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i < count) p[i] = value;
}

int grid_for_blocks(int64_t nb) { return (int)(nb < 4096 ? nb : 4096); }

// T[j][i] = M[i][j] through 64 x 64 tiles in LDS (coalesced on both sides).
__global__ __launch_bounds__(256) void k_transpose_i8(const int8_t *__restrict__ M, int64_t rows,
                                                      int64_t cols, int8_t *__restrict__ T) {
    __shared__ int8_t tile[64][65];
    const int64_t tiles_x = (cols + 63) / 64;
    const int64_t ti = blockIdx.x / tiles_x, tj = blockIdx.x % tiles_x;
    const int x = threadIdx.x & 63, y0 = threadIdx.x >> 6;
    for (int y = y0; y < 64; y += 4) {
        const int64_t i = ti * 64 + y, j = tj * 64 + x;
        tile[y][x] = (i < rows && j < cols) ? M[i * cols + j] : (int8_t)0;
    }
    __syncthreads();
    for (int y = y0; y < 64; y += 4) {
        const int64_t j = tj * 64 + y, i = ti * 64 + x;
        if (i < rows && j < cols) T[j * rows + i] = tile[x][y];
    }
}

}  // namespace

hipError_t launch_encode(const int8_t *M, int64_t rows, int64_t cols, int k, int mode,
                         uint16_t *code, int *err_flag) {
    const int64_t nb = (rows + k - 1) / k;
    const int64_t cols_pad = (cols + kThreads - 1) / kThreads * kThreads;
    const int64_t groups = nb * cols_pad / kThreads;
    hipLaunchKernelGGL(k_encode, dim3((unsigned)groups), dim3(kThreads), 0, 0, M, rows, cols, k,
                       mode, nb, code, err_flag);
    return hipGetLastError();
}

hipError_t launch_sort(const uint16_t *code, int64_t nb, int64_t cols, int k, int base, int64_t P,
                       uint16_t *pi, uint32_t *off) {
    const int n = (int)cols;
    const int npad = (n + 7) & ~7;
    const int passes = (k + 1) / 2;
    const int R = (base == 2) ? 4 : 9;
    const size_t lds = (size_t)npad * 4 + (size_t)(R * kThreads + kWaves) * 4;
    hipError_t e;
    if (base == 2) {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_sort<4>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(k_sort<4>, dim3(grid_for_blocks(nb)), dim3(kThreads), lds, 0, code, nb,
                           n, passes, P, pi, off);
    } else {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_sort<9>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(k_sort<9>, dim3(grid_for_blocks(nb)), dim3(kThreads), lds, 0, code, nb,
                           n, passes, P, pi, off);
    }
    return hipGetLastError();
}

hipError_t launch_transpose(const int8_t *M, int64_t rows, int64_t cols, int8_t *T) {
    const int64_t tiles = ((rows + 63) / 64) * ((cols + 63) / 64);
    hipLaunchKernelGGL(k_transpose_i8, dim3((unsigned)tiles), dim3(256), 0, 0, M, rows, cols, T);
    return hipGetLastError();
}

hipError_t launch_stream_len(const uint32_t *off, int64_t nb, int64_t cols, int64_t P,
                             uint32_t *lens, uint32_t *longest) {
    hipLaunchKernelGGL(k_stream_len, dim3(grid_for_blocks(nb)), dim3(kThreads), 0, 0, off, nb,
                       cols, P, lens, longest);
    return hipGetLastError();
}

hipError_t launch_fill_u32(uint32_t *p, uint32_t value, int64_t count) {
    hipLaunchKernelGGL(k_fill_u32, dim3((unsigned)((count + kThreads - 1) / kThreads)), dim3(kThreads),
                       0, 0, p, value, count);
    return hipGetLastError();
}

hipError_t launch_pack_stream(const uint16_t *pi, const uint32_t *off, int64_t nb, int64_t cols,
                              int64_t P, int64_t C, int H, int enc, uint16_t *scratch,
                              uint16_t *entries, uint16_t *codes, int *err_flag) {
    const int64_t S = C * 64 * 8 * H;
    hipLaunchKernelGGL(k_pack_stream, dim3(grid_for_blocks(nb)), dim3(kThreads), 0, 0, pi, off, nb,
                       (int)cols, P, S, scratch);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    {
        static const bool off = std::getenv("RSR_NO_SPREAD") != nullptr;  // tuning only
        const int64_t units = nb * C;
        if (!off)
            hipLaunchKernelGGL(k_spread_banks, dim3((unsigned)(units < 65536 ? units : 65536)), dim3(64),
                               0, 0, scratch, nb, C, H);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(k_finalize_stream, dim3(grid_for_blocks(nb)), dim3(kThreads), 0, 0, scratch,
                       nb, P, C, H, enc, entries, codes, err_flag);
    return hipGetLastError();
}

}  // namespace rsr
