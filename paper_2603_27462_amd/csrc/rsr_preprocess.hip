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

// Slabs wave w owns when S slabs are dealt to W waves, the longer shares first.
__device__ __forceinline__ void wave_share(int S, int W, int w, int *first, int *count) {
    const int per = S / W, rem = S - per * W;
    *first = w * per + min(w, rem);
    *count = per + (w < rem ? 1 : 0);
}

// stats[0] = max over blocks of the columns outside group 0; stats[1] = the same plus one
// placeholder per empty group among codes 1..P-1; stats[2] = most non-empty groups among
// codes 1..P-1.  The caller zeroes stats.
__global__ __launch_bounds__(kThreads) void k_stream_stats(const uint32_t *__restrict__ off,
                                                           int64_t nb, int64_t n, int64_t P,
                                                           uint32_t *__restrict__ stats) {
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
            const uint32_t real = (uint32_t)(n - ob[1]);
            atomicMax(&stats[0], real);
            atomicMax(&stats[1], real + empties);
            atomicMax(&stats[2], (uint32_t)(P - 1) - empties);
        }
        __syncthreads();
    }
}

// Logical stream of block b (L entries): for code c = 1..P-1 in order, the columns of
// group c in ascending order (entry = column<<1, last one |1).  Indexed by code: an empty
// group contributes one placeholder entry (zero slot = index n, tail bit set), so that
// every code owns exactly one tail.  Indexed by rank: empty groups contribute nothing and
// gcode[b][rank] records the code of every non-empty group (rank 1.., gcode[b][0] = 0,
// zeros behind the last one), gcount[b] their number.  Filler entries (zero slot, no tail)
// up to L.
__global__ __launch_bounds__(kThreads) void k_pack_stream(const uint16_t *__restrict__ pi,
                                                          const uint32_t *__restrict__ off,
                                                          int64_t nb, int n, int64_t P, int64_t L,
                                                          int by_rank, int64_t slots,
                                                          uint16_t *__restrict__ stream,
                                                          uint16_t *__restrict__ gcode,
                                                          uint32_t *__restrict__ gcount) {
    __shared__ uint32_t wsum[kWaves];
    const uint16_t zero_entry = (uint16_t)(n << 1);
    for (int64_t b = blockIdx.x; b < nb; b += gridDim.x) {
        const uint16_t *pib = pi + b * n;
        const uint32_t *ob = off + b * (P + 1);
        uint16_t *sb = stream + b * L;
        uint16_t *gb = by_rank ? gcode + b * slots : nullptr;
        const uint32_t off1 = ob[1];
        uint32_t carry = 0;  // empty groups among the codes before the current batch
        for (int64_t c0 = 1; c0 < P; c0 += kThreads) {
            const int64_t c = c0 + threadIdx.x;
            const bool valid = c < P;
            const uint32_t s = valid ? ob[c] : 0, e = valid ? ob[c + 1] : 0;
            const uint32_t empty = (valid && s == e) ? 1u : 0u;
            uint32_t total;
            const uint32_t eb = carry + wg_exclusive_scan(empty, wsum, &total);
            if (valid) {
                if (empty) {
                    if (!by_rank) sb[s - off1 + eb] = zero_entry | 1;
                } else {
                    const uint32_t dst = s - off1 + (by_rank ? 0u : eb);
                    for (uint32_t t = s; t < e; ++t)
                        sb[dst + (t - s)] = (uint16_t)((pib[t] << 1) | (t + 1 == e ? 1 : 0));
                    if (by_rank) gb[c - eb] = (uint16_t)c;
                }
            }
            carry += total;
        }
        const int64_t len = (int64_t)(n - off1) + (by_rank ? 0 : carry);
        for (int64_t t = len + threadIdx.x; t < L; t += kThreads) sb[t] = zero_entry;
        if (by_rank) {
            const int64_t count = P - 1 - carry;
            if (threadIdx.x == 0) { gcount[b] = (uint32_t)count; gb[0] = 0; }
            for (int64_t r = count + 1 + threadIdx.x; r < slots; r += kThreads) gb[r] = 0;
        }
        __syncthreads();
    }
}

// Reorders the logical stream inside its groups so that the LDS gathers of the multiply
// kernel collide less.  Gather instruction i of a wave reads entry i of all 64 strips of
// the wave; the LDS serves the two half-waves side by side and needs one cycle per
// distinct dword that falls on the same of its 32 banks.  The order of the columns inside
// a group is free for the kernel (sums commute up to rounding; the canonical pi is not
// touched), so for every run of entries of one group inside a strip, each slot takes the
// remaining column whose banks are least loaded so far in that slot of the half-wave --
// counted for both vector types the kernel serves: bank (col / 2) mod 32 for 2-byte
// elements and col mod 32 for 4-byte elements; two more sweeps re-place every strip
// against all the others.  One wave per (block, wave of the multiply kernel): thread =
// (half-wave, slot), strips in order; the first slot of a run places the run.  Strips of
// more than 32 entries are left as they are.
constexpr int kSpreadSweeps = 3;
constexpr int kSpreadMaxRun = 8;

__global__ __launch_bounds__(64) void k_spread_banks(uint16_t *__restrict__ logical, int64_t nb,
                                                     int S, int W) {
    __shared__ uint8_t load2[2][32][33];  // [half][slot][bank of a 2-byte element], padded
    __shared__ uint8_t load4[2][32][33];  // [half][slot][bank of a 4-byte element]
    __shared__ uint16_t strip[64][33];    // the wave's part: [strip][slot], padded
    const int half = threadIdx.x >> 5, slot = threadIdx.x & 31;
    for (int64_t unit = blockIdx.x; unit < nb * W; unit += gridDim.x) {
        const int64_t b = unit / W;
        int first, count;
        wave_share(S, W, (int)(unit - b * W), &first, &count);
        const int epl = 8 * count;
        if (epl == 0 || epl > 32) continue;
        const bool live = slot < epl;
        uint16_t *cb = logical + (b * S + first) * kSlab;
        for (int i = threadIdx.x; i < 64 * epl; i += 64) strip[i / epl][i % epl] = cb[i];
        for (int k = 0; k < 33; ++k) { load2[half][slot][k] = 0; load4[half][slot][k] = 0; }
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
                    if (sweep > 0) {
                        --load2[half][slot][(entry >> 2) & 31];
                        --load4[half][slot][(entry >> 1) & 31];
                    }
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
                        int bl = load2[half][sl][(st[sl] >> 1) & 31] + load4[half][sl][st[sl] & 31];
                        for (int t = sl + 1; place && t <= e; ++t) {
                            const int x = load2[half][sl][(st[t] >> 1) & 31] + load4[half][sl][st[t] & 31];
                            if (x < bl) { bl = x; best = t; }
                        }
                        const uint16_t c = st[best];
                        st[best] = st[sl];
                        st[sl] = c;
                        ++load2[half][sl][(c >> 1) & 31];
                        ++load4[half][sl][c & 31];
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

// Final layout of the stream (see PassData): re-encodes the entries, moves them to the
// slabs, and records for every strip the slot of the first tail at or after its start
// (1 + tails before it).  Also checks that the block holds the expected number of tails:
// P - 1 (indexed by code) or gcount[b] (indexed by rank).
__global__ __launch_bounds__(kThreads) void k_finalize_stream(
    const uint16_t *__restrict__ logical, int64_t nb, int64_t P, int S, int W, int enc,
    const uint32_t *__restrict__ gcount, uint16_t *__restrict__ entries,
    uint16_t *__restrict__ start, int *__restrict__ err_flag) {
    __shared__ uint32_t wsum[kWaves];
    const int strips = W * 64;
    for (int64_t b = blockIdx.x; b < nb; b += gridDim.x) {
        const uint16_t *lb = logical + b * S * kSlab;
        uint32_t carry = 1;
        for (int g0 = 0; g0 < strips; g0 += kThreads) {
            const int g = g0 + threadIdx.x;
            const int w = g >> 6, lane = g & 63;
            int first = 0, count = 0;
            if (g < strips) wave_share(S, W, w, &first, &count);
            const int epl = 8 * count;
            const uint16_t *sp = lb + (int64_t)first * kSlab + (int64_t)lane * epl;
            uint32_t cnt = 0;
            for (int i = 0; i < epl; ++i) cnt += sp[i] & 1u;
            uint32_t total;
            const uint32_t ex = wg_exclusive_scan(cnt, wsum, &total);
            if (g < strips) {
                start[(b * W + w) * 64 + lane] = (uint16_t)(carry + ex);
                for (int i = 0; i < epl; ++i) {
                    const uint32_t e = sp[i];
                    const uint32_t out = (enc == kEncSmall) ? (((e & 1u) << 15) | (e & 0xfffeu)) : e;
                    entries[(((b * S + first + (i >> 3)) * 64) + lane) * 8 + (i & 7)] = (uint16_t)out;
                }
            }
            carry += total;
        }
        const int64_t expect = gcount ? (int64_t)gcount[b] : P - 1;
        if (threadIdx.x == 0 && (int64_t)carry != expect + 1) atomicOr(err_flag, 2);
        __syncthreads();
    }
}

// Sign of digit r of code c as a 2-bit two's complement field (00: 0, 01: +1, 11: -1).
__device__ __forceinline__ uint32_t sign2_of(uint32_t c, int r, int base) {
    for (int i = 0; i < r; ++i) c /= (uint32_t)base;
    const uint32_t d = c % (uint32_t)base;
    return d == 0 ? 0u : d == 1 ? 1u : 3u;
}
__device__ __forceinline__ int sign_of(uint32_t c, int r, int base) {
    const uint32_t s = sign2_of(c, r, base);
    return s == 3u ? -1 : (int)s;
}

// Code of the first group closed at or after the start of the strip that follows strip g of
// block b; false when there is none (last strip, or no tail from there on).
__device__ __forceinline__ bool next_strip_code(const uint16_t *__restrict__ start, int64_t b, int g,
                                                int strips, int64_t P,
                                                const uint16_t *__restrict__ gcode,
                                                const uint32_t *__restrict__ gcount, int64_t slots,
                                                uint32_t *code) {
    if (g + 1 >= strips) return false;
    const uint32_t slot = start[b * strips + g + 1];
    if (gcode) {
        if (slot > gcount[b]) return false;
        *code = gcode[b * slots + slot];
        return true;
    }
    if ((int64_t)slot >= P) return false;
    *code = slot;
    return true;
}

// Strip signs, indexed by code: word (b, r, l) holds, at bits 2w, the sign of digit r of the
// code that follows strip (w, l).  16-bit words when W <= 8.
__global__ __launch_bounds__(kThreads) void k_strip_signs_rows(const uint16_t *__restrict__ start,
                                                               int64_t nb, int W, int k, int base,
                                                               int64_t P, void *__restrict__ sgn) {
    const int64_t gid = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (gid >= nb * k * 64) return;
    const int lane = (int)(gid & 63);
    const int r = (int)((gid >> 6) % k);
    const int64_t b = (gid >> 6) / k;
    uint32_t word = 0;
    for (int w = 0; w < W; ++w) {
        uint32_t c;
        if (next_strip_code(start, b, w * 64 + lane, W * 64, P, nullptr, nullptr, 0, &c))
            word |= sign2_of(c, r, base) << (2 * w);
    }
    if (W <= 8)
        static_cast<uint16_t *>(sgn)[gid] = (uint16_t)word;
    else
        static_cast<uint32_t *>(sgn)[gid] = word;
}

// Strip signs, indexed by rank: word (b, w, l) holds, at bits 2r, the sign of digit r of
// the code that follows strip (w, l).
__global__ __launch_bounds__(kThreads) void k_strip_signs_strips(
    const uint16_t *__restrict__ start, int64_t nb, int W, int k, int base, int64_t P,
    const uint16_t *__restrict__ gcode, const uint32_t *__restrict__ gcount, int64_t slots,
    uint32_t *__restrict__ sgn) {
    const int64_t gid = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (gid >= nb * W * 64) return;
    const int g = (int)(gid % (W * 64));
    const int64_t b = gid / (W * 64);
    uint32_t word = 0, c;
    if (next_strip_code(start, b, g, W * 64, P, gcode, gcount, slots, &c))
        for (int r = 0; r < k; ++r) word |= sign2_of(c, r, base) << (2 * r);
    sgn[gid] = word;
}

// Weights of the slots of a rank-indexed E: field r of gword[b][s] (fw bits, two's
// complement) = sgn_r(code of rank s) - sgn_r(code of rank s+1), the second term 0 behind
// the last group; 0 for s = 0 and behind the last group.
__global__ __launch_bounds__(kThreads) void k_group_words(const uint16_t *__restrict__ gcode,
                                                          const uint32_t *__restrict__ gcount,
                                                          int64_t nb, int64_t slots, int k, int base,
                                                          int fw, uint32_t *__restrict__ gword) {
    const int64_t gid = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (gid >= nb * slots) return;
    const int64_t b = gid / slots, s = gid - b * slots;
    const int64_t count = gcount[b];
    uint32_t word = 0;
    if (s >= 1 && s <= count) {
        const uint32_t c = gcode[gid];
        const bool has_next = s < count;
        const uint32_t cn = has_next ? gcode[gid + 1] : 0u;
        for (int r = 0; r < k; ++r) {
            const int wgt = sign_of(c, r, base) - (has_next ? sign_of(cn, r, base) : 0);
            word |= ((uint32_t)wgt & ((1u << fw) - 1u)) << (fw * r);
        }
    }
    gword[gid] = word;
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

hipError_t launch_stream_stats(const uint32_t *off, int64_t nb, int64_t cols, int64_t P,
                               uint32_t *stats) {
    hipLaunchKernelGGL(k_stream_stats, dim3(grid_for_blocks(nb)), dim3(kThreads), 0, 0, off, nb,
                       cols, P, stats);
    return hipGetLastError();
}

hipError_t launch_fill_u32(uint32_t *p, uint32_t value, int64_t count) {
    hipLaunchKernelGGL(k_fill_u32, dim3((unsigned)((count + kThreads - 1) / kThreads)), dim3(kThreads),
                       0, 0, p, value, count);
    return hipGetLastError();
}

hipError_t launch_pack_pass(const rsr_handle_s *h, int pass, uint16_t *logical, uint16_t *gcode,
                            int *err_flag) {
    const PassData &pd = h->pass[pass];
    const int64_t nb = h->nb, P = h->P;
    const int S = (int)pd.S, W = h->W;
    const int by_rank = h->by_rank;
    auto blocks_for = [](int64_t threads) { return dim3((unsigned)((threads + kThreads - 1) / kThreads)); };
    hipLaunchKernelGGL(k_pack_stream, dim3(grid_for_blocks(nb)), dim3(kThreads), 0, 0, pd.pi, pd.off,
                       nb, (int)h->cols, P, (int64_t)S * kSlab, by_rank, h->slots, logical, gcode,
                       pd.gcount);
    if (hipError_t e = hipGetLastError()) return e;
    const int64_t units = nb * W;
    hipLaunchKernelGGL(k_spread_banks, dim3((unsigned)(units < 65536 ? units : 65536)), dim3(64), 0, 0,
                       logical, nb, S, W);
    if (hipError_t e = hipGetLastError()) return e;
    hipLaunchKernelGGL(k_finalize_stream, dim3(grid_for_blocks(nb)), dim3(kThreads), 0, 0, logical, nb,
                       P, S, W, h->enc, by_rank ? pd.gcount : nullptr, pd.entries, pd.start, err_flag);
    if (hipError_t e = hipGetLastError()) return e;
    if (by_rank) {
        hipLaunchKernelGGL(k_strip_signs_strips, blocks_for(nb * W * 64), dim3(kThreads), 0, 0, pd.start,
                           nb, W, h->k, h->base, P, gcode, pd.gcount, h->slots,
                           static_cast<uint32_t *>(pd.sgn));
        if (hipError_t e = hipGetLastError()) return e;
        hipLaunchKernelGGL(k_group_words, blocks_for(nb * h->slots), dim3(kThreads), 0, 0, gcode,
                           pd.gcount, nb, h->slots, h->k, h->base, gword_field_bits(h->base), pd.gword);
    } else {
        hipLaunchKernelGGL(k_strip_signs_rows, blocks_for(nb * h->k * 64), dim3(kThreads), 0, 0, pd.start,
                           nb, W, h->k, h->base, P, pd.sgn);
    }
    return hipGetLastError();
}

}  // namespace rsr
