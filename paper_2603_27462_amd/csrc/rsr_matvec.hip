// RSR multiply kernel for gfx950 (paper, System Overview: aggregate the entries
// of v of each group of identical column patterns, then distribute every group
// sum once; Kernels Implementation: gather, aggregate and scatter phases; one
// metadata word per existing group, zero-contribution groups dropped).
//
// One workgroup of W waves handles one block of k output rows:
//   gather     the block's stream of 16-bit column entries arrives in slabs of
//              512 entries (one coalesced 16-byte load per lane); a lane owns a
//              strip of consecutive entries, eight per slab of its wave; v sits
//              in LDS and is gathered through the entries.  Every slab is
//              processed as soon as it has arrived: nothing in this phase
//              crosses lanes, so the work overlaps the rest of the stream.
//   aggregate  instead of one sum per group the kernel keeps running prefix
//              sums: the entry that closes a group (tail flag) stores the
//              prefix of its strip into the group's slot of the LDS array E.
//              Each slot is written once with a plain store: no atomics, no
//              zero fill, deterministic.  Group sums are never materialised.
//   scatter    out[r] = sum_c sgn_r(c) u[c] = sum_s E*[s] (sgn_r(c_s) - sgn_r(c_s+1))
//              over the slots s in code order, E* the prefix over the whole
//              stream.  The stored prefixes are local to a strip; the weighted
//              sum is linear in E, so the total T of a strip is folded in
//              afterwards: it is missing from every prefix stored by later
//              strips, whose weights telescope to sgn_r(first code closed
//              after the strip), a sign precomputed per (strip, row).
// Two indexings of E (chosen at preprocessing time):
//   by code    slot = pattern code; empty groups own a placeholder entry.  Digit
//              r only matters where it changes, so the weighted sum is taken in
//              two levels (all P entries for the lowest digits, every Tc-th for
//              the others) with weights from a small table.
//   by rank    slot = rank among the non-empty groups (for pattern spaces much
//              larger than the column count); one weight word per slot is read
//              from the stream side.
//
// LDS addresses are raw integers: this kernel owns the whole LDS allocation
// (it declares no static __shared__), so dynamic LDS starts at address 0.
#include <cstdio>
#ifdef RSR_TUNING
#include <cstdlib>
#endif

#include "rsr_device.h"
#include "rsr_internal.h"

namespace rsr {

namespace {

// What the kernel reads of one pass.
struct PassArgs {
    const uint16_t *entries;
    const uint16_t *start;
    const void *sgn;
    const uint32_t *gword;
    const uint32_t *gcount;
    int S;           // slabs per block
    int per, rem;    // wave w owns per + (w < rem) slabs, the longer shares first
    float sign;
};

struct FoldArgs {
    const uint32_t *fpack;
    const uint32_t *fshare;
    int k, slots, m, Tc, Q, G, parts, cnt1, fw;
};

struct OutArgs {
    float *out;
    long long ldo;
    int n_out;
    float scale;
    LayerTable layers;  // stacked handles: per-layer outputs, scales and row counts
};

// Output rows, rows left and scale of block b: of the matrix, or of the layer the block
// belongs to.
__device__ __forceinline__ void block_output(const OutArgs &o, long long b, int k, int vec,
                                             float **out_rows, long long *rows_left, float *scale) {
    if (o.layers.n == 0) {
        *out_rows = o.out + (long long)vec * o.ldo + b * k;
        *rows_left = (long long)o.n_out - b * k;
        *scale = o.scale;
        return;
    }
    int s = 0;
#pragma unroll
    for (int i = 1; i < kMaxLayers; ++i)
        if (i < o.layers.n && b >= o.layers.first[i]) s = i;
    const long long local = (b - o.layers.first[s]) * k;
    *out_rows = o.layers.out[s] + local;
    *rows_left = (long long)o.layers.rows[s] - local;
    *scale = o.layers.scale[s];
}

// Slabs of the first group a wave requests before v is staged; the others follow the first
// barrier.  With all four up front the requests for v queue behind 32 KiB of stream per
// block and the first barrier comes later (measured: 7.4 -> 7.05 us cold, 6.0 -> 5.85 warm).
constexpr int kEarlySlabs = 2;

template <typename T>
__device__ __forceinline__ void pin(T &x) {
    asm volatile("" : "+v"(x));
}

// ---- scatter phase, E indexed by code ---------------------------------------------------
// out[r] = sum_c E[c] (sgn_r(c) - sgn_r(c+1)) + strip-total terms.
// Level 1: thread (part, class t) adds up its share of E[t], E[t + Tc], E[t + 2 Tc], ...
// (the entries that agree with t in the m lowest digits) and leaves the sum in
// C1[part][t]; a class is shared by at most two threads.  Every thread adds the same
// number of entries (cnt1): E is followed by one row of Tc zeros, which the second part
// reads when Q is odd.  With Q == 1 (all P codes fit the workgroup) the class sums are E
// itself and level 1 and its barrier are left out.
// Level 2: one wave per output row.  Rows r < m weigh the class sums with the weight of
// (t, r); rows r >= m weigh E[Tc i + Tc - 1], the only entries where their digit
// changes, with the weight of (i, r).  Lane l adds the totals of the strips (w, l), each
// times the sign of the row's digit in the code that follows the strip; one scan over
// the wave adds everything up and lane 63 writes the row.
// fpack[r][g][lane] packs, one byte each, the weights of j = lane + 64 (4g + u), u < 4:
// r < m: sgn_r(j) - sgn_r((j+1) mod Tc); m <= r < k: sgn_{r-m}(j) - sgn_{r-m}(j+1).
// share: first E index of the thread's level-1 share (0xffffffff: no share).
//
// A wave64 vector instruction occupies its SIMD for four cycles, so the vector
// instruction count is what the phases behind the last slab cost.  Everything below that
// does not depend on E -- LDS addresses, unpacked weights, predicates -- is therefore
// computed by prepare_scatter() while the global loads of the pass are still in flight,
// and pinned in registers until it is used.
constexpr int kL1Regs = 16;  // level-1 entries per thread read in one batch

struct ScatterPrep {
    uint32_t first;     // level 1: LDS address of the thread's first entry (E[0] without a share)
    uint32_t c1_store;  // level 1: where the thread's sum goes
    uint32_t la[8];     // level 2 (one row per wave): class sums / entries of the row
    uint32_t t_lane;    // level 2: total of strip (0, lane); strip (w, lane) is w * 256 bytes on
    float wf[4];        // level 2: weights of the four elements
    bool has_share;
};

// TC: the class count as a compile-time constant (0: only known at run time), which turns
// the strides of level 1 into instruction offsets.
template <int TC>
__device__ __forceinline__ uint32_t class_step(const FoldArgs &f) {
    return TC > 0 ? (uint32_t)TC * 4u : (uint32_t)f.Tc * 4u;
}

template <int TC>
__device__ __forceinline__ void prepare_scatter(ScatterPrep &sp, const FoldArgs &f, uint32_t share,
                                                uint32_t wpre, uint32_t t_at, uint32_t e_at,
                                                uint32_t c1_at, int W, int w, int lane, int tid) {
    const uint32_t step = class_step<TC>(f);
    const int Tc = TC > 0 ? TC : f.Tc;
    sp.has_share = share != 0xffffffffu;
    sp.first = e_at + (sp.has_share ? share : 0u) * 4u;
    pin(sp.first);
    sp.c1_store = c1_at + (uint32_t)tid * 4u;  // C1[part][class]: tid = part * Tc + class
    pin(sp.c1_store);
    // level 2, one row per wave (used when G == 1 and k <= W)
    const int r = min(w, f.k - 1);
    const bool low = r < f.m;
    const int n = low ? Tc : f.Q;
    // with one entry per class (Q == 1) the class sums are E itself: no level 1
    const uint32_t base = low ? (f.Q == 1 ? e_at : c1_at) : e_at + (uint32_t)(Tc - 1) * 4u;
    const uint32_t stride = low ? 4u : step;
    const uint32_t last = base + stride * (uint32_t)(n - 1);
    sp.la[0] = min(base + stride * (uint32_t)lane, last);
    sp.la[1] = min(sp.la[0] + 64 * stride, last);
    sp.la[2] = min(sp.la[0] + 128 * stride, last);
    sp.la[3] = min(sp.la[0] + 192 * stride, last);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        sp.la[4 + j] = sp.la[j] + step;  // the second part's class sums
        pin(sp.la[j]);
        pin(sp.la[4 + j]);
    }
    sp.t_lane = t_at + (uint32_t)lane * 4u;
    pin(sp.t_lane);
    sp.wf[0] = (float)(int)(signed char)(wpre & 0xffu);
    sp.wf[1] = (float)(int)(signed char)((wpre >> 8) & 0xffu);
    sp.wf[2] = (float)(int)(signed char)((wpre >> 16) & 0xffu);
    sp.wf[3] = (float)(int)(signed char)(wpre >> 24);
#pragma unroll
    for (int j = 0; j < 4; ++j) pin(sp.wf[j]);
}

// Sum over the strips (w, lane) of total * sign; sw holds the signs at bits 2w.  The totals
// of at least eight waves exist in LDS (rows of waves that do not exist are zero).
__device__ __forceinline__ float strip_terms(const ScatterPrep &sp, uint32_t sw, int W) {
    float t[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) t[j] = *lds_float(sp.t_lane + (uint32_t)j * 256u);
    float x = 0.0f;
#pragma unroll
    for (int j = 0; j < 8; ++j) x += t[j] * field_as_float(sw, 2 * j, 2);
    if (W > 8) {
        for (int j = 8; j < W; ++j)
            x += *lds_float(sp.t_lane + (uint32_t)j * 256u) * field_as_float(sw, 2 * j, 2);
    }
    return x;
}

__device__ __forceinline__ uint32_t load_sign_word(const void *sgn, long long index, int W) {
    return W <= 8 ? (uint32_t) static_cast<const uint16_t *>(sgn)[index]
                  : static_cast<const uint32_t *>(sgn)[index];
}

constexpr int kMoreRows = 3;  // further rows of a wave (w + W, w + 2W, ...) whose tables are requested up front

template <bool FIRST, int TC>
__device__ __forceinline__ void scatter_by_code(const FoldArgs &f, const ScatterPrep &sp,
                                                uint32_t wpre, uint32_t sw,
                                                const uint32_t (&pk_more)[kMoreRows],
                                                const uint32_t (&sw_more)[kMoreRows], const void *sgn,
                                                long long b, uint32_t t_at, uint32_t e_at,
                                                uint32_t c1_at, int W, int w, int lane,
                                                float sign_scale, float *out_rows,
                                                long long rows_left) {
    if (f.Q > 1 && sp.has_share) {
        // the thread's cnt1 entries, E[first + i Tc]: whole batches of four, then the rest one
        // by one (wave-uniform branches; the loads of a batch are in flight together)
        const uint32_t step = class_step<TC>(f);
        float x[kL1Regs];
        float rest = 0.0f;
        if (f.cnt1 <= 4) {
            // short shares: entries past the share read E[0], which is zero (no branches)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                x[i] = *lds_float(i < f.cnt1 ? sp.first + (uint32_t)i * step : e_at);
            x[0] = (x[0] + x[1]) + (x[2] + x[3]);
        } else {
#pragma unroll
            for (int i = 0; i < kL1Regs; ++i) x[i] = 0.0f;
            const int n1 = f.cnt1 < kL1Regs ? f.cnt1 : kL1Regs;
#pragma unroll
            for (int i0 = 0; i0 < kL1Regs; i0 += 4) {
                if (i0 + 4 <= n1) {
#pragma unroll
                    for (int i = i0; i < i0 + 4; ++i) x[i] = *lds_float(sp.first + (uint32_t)i * step);
                } else {
#pragma unroll
                    for (int i = i0; i < i0 + 3; ++i)
                        if (i < n1) x[i] = *lds_float(sp.first + (uint32_t)i * step);
                }
            }
            if (f.cnt1 > kL1Regs) {
                uint32_t at = sp.first + (uint32_t)kL1Regs * step;
                for (int i = kL1Regs; i < f.cnt1; ++i) {
                    rest += *lds_float(at);
                    at += step;
                }
            }
#pragma unroll
            for (int d = 1; d < kL1Regs; d *= 2)
#pragma unroll
                for (int i = 0; i + d < kL1Regs; i += 2 * d) x[i] += x[i + d];
        }
        const float col = x[0] + rest;
        *lds_float(sp.c1_store) = col;
    }
    if (f.Q > 1) __syncthreads();
    if (f.G == 1 && f.k <= W) {
        // common shape: at most one row per wave, at most 256 table entries per row
        if (w < f.k) {
            const int r = w;
            float v0 = *lds_float(sp.la[0]), v1 = *lds_float(sp.la[1]);
            float v2 = *lds_float(sp.la[2]), v3 = *lds_float(sp.la[3]);
            float x = strip_terms(sp, sw, W);
            if (r < f.m && f.parts == 2) {
                const float u0 = *lds_float(sp.la[4]), u1 = *lds_float(sp.la[5]);
                const float u2 = *lds_float(sp.la[6]), u3 = *lds_float(sp.la[7]);
                v0 += u0; v1 += u1; v2 += u2; v3 += u3;
            }
            // entries past the end of the row carry weight 0 in the table
            x += sp.wf[0] * v0;
            x += sp.wf[1] * v1;
            x += sp.wf[2] * v2;
            x += sp.wf[3] * v3;
            const float tot = wave_inclusive_scan(x);
            if (lane == 63 && r < rows_left) {
                const float term = sign_scale * tot;
                __builtin_nontemporal_store(FIRST ? term : out_rows[r] + term, &out_rows[r]);
            }
        }
        return;
    }
    int turn = 0;
    for (int r = w; r < f.k; r += W, ++turn) {
        const bool low = r < f.m;
        const int n = low ? f.Tc : f.Q;
        // element j of the row: class sum C1[0][j] (+ C1[1][j]), or E[Tc j + Tc - 1]
        const uint32_t base = low ? (f.Q == 1 ? e_at : c1_at) : e_at + (uint32_t)(f.Tc - 1) * 4u;
        const uint32_t stride = low ? 4u : class_step<TC>(f);
        const bool two = low && f.parts == 2;
        const uint32_t second = class_step<TC>(f);
        uint32_t swr = sw, pk0 = wpre;
        if (turn == 1) { swr = sw_more[0]; pk0 = pk_more[0]; }
        if (turn == 2) { swr = sw_more[1]; pk0 = pk_more[1]; }
        if (turn == 3) { swr = sw_more[2]; pk0 = pk_more[2]; }
        if (turn > kMoreRows) {
            swr = load_sign_word(sgn, (b * f.k + r) * 64 + lane, W);
            pk0 = f.fpack[(r * f.G) * 64 + lane];
        }
        float x = strip_terms(sp, swr, W);
        for (int g = 0; g * 256 < n; ++g) {
            const uint32_t pk = (g == 0) ? pk0 : f.fpack[(r * f.G + g) * 64 + lane];
            const int j0 = lane + 256 * g;
            // the four loads first, then the arithmetic (entries past n have weight 0)
            const uint32_t a0 = base + stride * (uint32_t)min(j0, n - 1);
            const uint32_t a1 = base + stride * (uint32_t)min(j0 + 64, n - 1);
            const uint32_t a2 = base + stride * (uint32_t)min(j0 + 128, n - 1);
            const uint32_t a3 = base + stride * (uint32_t)min(j0 + 192, n - 1);
            float v0 = *lds_float(a0), v1 = *lds_float(a1), v2 = *lds_float(a2), v3 = *lds_float(a3);
            if (two) {
                const float u0 = *lds_float(a0 + second), u1 = *lds_float(a1 + second);
                const float u2 = *lds_float(a2 + second), u3 = *lds_float(a3 + second);
                v0 += u0; v1 += u1; v2 += u2; v3 += u3;
            }
            x += (float)(int)(signed char)(pk & 0xffu) * v0;
            x += (float)(int)(signed char)((pk >> 8) & 0xffu) * v1;
            x += (float)(int)(signed char)((pk >> 16) & 0xffu) * v2;
            x += (float)(int)(signed char)(pk >> 24) * v3;
        }
        const float tot = wave_inclusive_scan(x);
        if (lane == 63 && r < rows_left) {
            const float term = sign_scale * tot;
            // pass 2 adds to what pass 1 wrote
            __builtin_nontemporal_store(FIRST ? term : out_rows[r] + term, &out_rows[r]);
        }
    }
}

// ---- scatter phase, E indexed by rank ---------------------------------------------------
// out[r] = sum_s E[s] w_r(s) + sum over strips of total * sign, with w_r(s) the field r of
// gword[s].  Thread t takes the slots t, t + threads, ...; every thread adds its own
// strip's term; the k sums are reduced over the wave by a scan and over the waves through
// LDS.
constexpr int kMaxRows = 16;

template <bool FIRST>
__device__ __forceinline__ void scatter_by_rank(const FoldArgs &f, const uint32_t *__restrict__ gword,
                                                uint32_t count, uint32_t sword, float total,
                                                uint32_t e_at, uint32_t red_at, int W, int w, int lane,
                                                int tid, float sign_scale, float *out_rows,
                                                long long rows_left) {
    const int nthreads = W * 64;
    float acc[kMaxRows];
#pragma unroll
    for (int r = 0; r < kMaxRows; ++r)
        acc[r] = (r < f.k) ? total * field_as_float(sword, 2 * r, 2) : 0.0f;
    for (uint32_t s0 = 1; s0 <= count; s0 += 2 * nthreads) {
        // two slots per round, loads first
        const uint32_t sa = s0 + tid, sb = sa + nthreads;
        const uint32_t wa = sa <= count ? gword[sa] : 0u;
        const uint32_t wb = sb <= count ? gword[sb] : 0u;
        const float ea = sa <= count ? *lds_float(e_at + sa * 4u) : 0.0f;
        const float eb = sb <= count ? *lds_float(e_at + sb * 4u) : 0.0f;
#pragma unroll
        for (int r = 0; r < kMaxRows; ++r)
            if (r < f.k) {
                acc[r] += ea * field_as_float(wa, f.fw * r, f.fw);
                acc[r] += eb * field_as_float(wb, f.fw * r, f.fw);
            }
    }
#pragma unroll
    for (int r = 0; r < kMaxRows; ++r)
        if (r < f.k) {
            const float tot = wave_inclusive_scan(acc[r]);
            if (lane == 63) *lds_float(red_at + (uint32_t)(w * kMaxRows + r) * 4u) = tot;
        }
    __syncthreads();
    if (tid < f.k && tid < rows_left) {
        float sum = 0.0f;
        for (int i = 0; i < W; ++i) sum += *lds_float(red_at + (uint32_t)(i * kMaxRows + tid) * 4u);
        const float term = sign_scale * sum;
        out_rows[tid] = FIRST ? term : out_rows[tid] + term;
    }
}

// ---- gather + aggregate: one slab of a wave -----------------------------------------------
// Eight entries per lane: gather the eight elements of v, extend the strip's running sum,
// and let every tail store its prefix.
template <typename VT, int ENC>
__device__ __forceinline__ void slab_step(const u32x4 &q, uint32_t (&g)[8], float &prev,
                                          uint32_t &ptr) {
    const uint32_t d[4] = {q.x, q.y, q.z, q.w};
    uint32_t a[8];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        a[2 * j] = entry_addr<VT, ENC, 0>(d[j]);
        a[2 * j + 1] = entry_addr<VT, ENC, 1>(d[j]);
    }
    gather8<VT>(g, a);
    float s[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        prev += __uint_as_float(g[i]);
        s[i] = prev;
    }
    if (ENC == kEncSmall) {
        tail_store8_small(d[0], d[1], d[2], d[3], s, ptr);
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) tail_store2_big(d[j], s[2 * j], s[2 * j + 1], ptr);
    }
}

// One pass (binary, M+, M- or fused) of one block.  FIRST: v still has to be staged into
// LDS and the output rows are overwritten; otherwise the pass adds to them.
template <typename VT, int ENC, bool BYRANK, bool FIRST, int TC>
__device__ __forceinline__ void run_pass(const uint16_t *__restrict__ entries,
                                         const uint16_t *__restrict__ start, int S, int per, int rem,
                                         const PassArgs &a, const void *__restrict__ v, long long ldv,
                                         int n_in, int W, const FoldArgs &f, const OutArgs &o,
                                         int vec) {
    // LDS (byte addresses): v (n_in + zero slot) | T[max(W, 8)][64] | E[slots] | by code: Tc
    // zeros, C1[threads]; by rank: partial sums [W][16]
    const uint32_t vbytes = ((n_in + 1) * (uint32_t)sizeof(VT) + 15u) & ~15u;
    const uint32_t t_at = vbytes;
    const uint32_t e_at = t_at + (uint32_t)max(W, 8) * 256u;
    const uint32_t z_at = e_at + (uint32_t)f.slots * 4u;
    const uint32_t c1_at = z_at + class_step<TC>(f);
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nthreads = W * 64;
    const long long b = blockIdx.x;

    // the wave's slabs, in groups of four; the first group may be short (n0 slabs)
    const int n_w = per + (w < rem ? 1 : 0);
    const int first = w * per + min(w, rem);
    const int ngroups = (n_w + kGroupSlabs - 1) / kGroupSlabs;
    const int n0 = n_w - (ngroups - 1) * kGroupSlabs;

    // ---- the global loads of the pass, in the order of use: v (the first barrier waits for
    // it), the strip's first slot, the first slabs and the small tables of the scatter phase;
    // behind the first barrier the remaining slabs ------------------------------------------
    const long long vstride = ldv * (long long)sizeof(VT);
    const unsigned char *vg = reinterpret_cast<const unsigned char *>(v) + (long long)vec * vstride;
    const int nbytes = n_in * (int)sizeof(VT);
    const int n16 = nbytes >> 4;
    const bool v_aligned = (reinterpret_cast<uintptr_t>(vg) & 15) == 0;
    const u32x4 *v16 = reinterpret_cast<const u32x4 *>(vg);
    lds_u128 *l16 = reinterpret_cast<lds_u128 *>(static_cast<uintptr_t>(0));
    u32x4 s0, s1, s2, s3;
    const int j_0 = tid, j_1 = j_0 + nthreads, j_2 = j_1 + nthreads, j_3 = j_2 + nthreads;
    if (FIRST && v_aligned && n16 > 0) {
        // loads past the end are redirected to the last valid 16 bytes
        s0 = v16[min(j_0, n16 - 1)];
        s1 = v16[min(j_1, n16 - 1)];
        s2 = v16[min(j_2, n16 - 1)];
        s3 = v16[min(j_3, n16 - 1)];
    }
    const uint32_t slot0 = __builtin_nontemporal_load(&start[(b * W + w) * 64 + lane]);
    // The stream is read once: non-temporal loads keep it out of the way of v and the
    // tables.  Slots without a slab (the end of a short first group, waves without slabs)
    // repeat a neighbouring slab and are ignored: no branch, so nothing delays the requests
    // and the number of loads in flight is the same in every wave.
    const u32x4 *ep = reinterpret_cast<const u32x4 *>(entries) + (b * S) * 64 + lane;
    u32x4 q[kGroupSlabs];
#pragma unroll
    for (int j = 0; j < kEarlySlabs; ++j)
        q[j] = __builtin_nontemporal_load(&ep[(long long)min(first + min(j, n0 - 1), S - 1) * 64]);
    uint32_t share = 0, wpre = 0, sw = 0, count = 0;
    uint32_t pk_more[kMoreRows] = {0, 0, 0}, sw_more[kMoreRows] = {0, 0, 0};
    auto load_tables = [&]() {
        if (BYRANK) {
            sw = static_cast<const uint32_t *>(a.sgn)[(b * W + w) * 64 + lane];
            count = a.gcount[b];
        } else {
            share = f.fshare[tid];
            wpre = f.fpack[(min(w, f.k - 1) * f.G) * 64 + lane];
            sw = load_sign_word(a.sgn, (b * f.k + min(w, f.k - 1)) * 64 + lane, W);
            if (f.k > W) {  // fewer waves than rows: the tables of the wave's further rows
#pragma unroll
                for (int i = 0; i < kMoreRows; ++i) {
                    const int r = min(w + (i + 1) * W, f.k - 1);
                    pk_more[i] = f.fpack[(r * f.G) * 64 + lane];
                    sw_more[i] = load_sign_word(a.sgn, (b * f.k + r) * 64 + lane, W);
                }
            }
        }
    };
    load_tables();

    // ---- stage v -----------------------------------------------------------------------------
    if (FIRST) {
        if (v_aligned) {
            if (n16 > 0) {
                if (j_0 < n16) l16[j_0] = s0;
                if (j_1 < n16) l16[j_1] = s1;
                if (j_2 < n16) l16[j_2] = s2;
                if (j_3 < n16) l16[j_3] = s3;
                for (int j = j_3 + nthreads; j < n16; j += nthreads) l16[j] = v16[j];
            }
            for (int j = (n16 << 4) + tid * (int)sizeof(VT); j < nbytes;
                 j += nthreads * (int)sizeof(VT))
                lds_store_v<VT>(j, *reinterpret_cast<const VT *>(vg + j));
        } else {
            for (int j = tid * (int)sizeof(VT); j < nbytes; j += nthreads * (int)sizeof(VT))
                lds_store_v<VT>(j, *reinterpret_cast<const VT *>(vg + j));
        }
        if (tid == 0) lds_store_v<VT>(nbytes, VT(0));
    }
    // ---- work that needs no stream data, done while the loads are in flight ----------------
    ScatterPrep sp;
    if (kEarlySlabs == kGroupSlabs && !BYRANK)
        prepare_scatter<TC>(sp, f, share, wpre, t_at, e_at, c1_at, W, w, lane, tid);
    uint32_t g[8];  // gather targets: for bf16 the low halves must be zero
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        g[i] = 0u;
        pin(g[i]);
    }
    if (!BYRANK) {
        if (tid < (TC > 0 ? TC : f.Tc)) *lds_float(z_at + (uint32_t)tid * 4u) = 0.0f;
        // totals of waves that do not exist (the scatter phase reads eight rows)
        for (int i = nthreads + tid; i < 8 * 64; i += nthreads) *lds_float(t_at + (uint32_t)i * 4u) = 0.0f;
    }
    if (tid == 0) *lds_float(e_at) = 0.0f;
    __syncthreads();
    if (kEarlySlabs < kGroupSlabs) {
#pragma unroll
        for (int j = kEarlySlabs; j < kGroupSlabs; ++j)
            q[j] = __builtin_nontemporal_load(&ep[(long long)min(first + min(j, n0 - 1), S - 1) * 64]);
    }

    // ---- gather + aggregate, slab by slab as the loads return ------------------------------
    float prev = 0.0f;
    uint32_t ptr = e_at + slot0 * 4u;
    if (ngroups > 0) {
#pragma unroll
        for (int j = 0; j < kGroupSlabs; ++j)
            if (j < n0) slab_step<VT, ENC>(q[j], g, prev, ptr);
        for (int grp = 1; grp < ngroups; ++grp) {
            const u32x4 *gp = ep + (long long)(first + n0 + (grp - 1) * kGroupSlabs) * 64;
#pragma unroll
            for (int j = 0; j < kGroupSlabs; ++j) q[j] = __builtin_nontemporal_load(&gp[j * 64]);
#pragma unroll
            for (int j = 0; j < kGroupSlabs; ++j) slab_step<VT, ENC>(q[j], g, prev, ptr);
        }
    }
    if (kEarlySlabs < kGroupSlabs && !BYRANK)
        prepare_scatter<TC>(sp, f, share, wpre, t_at, e_at, c1_at, W, w, lane, tid);
    if (!BYRANK) *lds_float(t_at + (uint32_t)tid * 4u) = prev;
    lds_drain();
    __syncthreads();

    // ---- scatter ----------------------------------------------------------------------------
    float *out_rows;
    long long rows_left;
    float scale;
    block_output(o, b, f.k, vec, &out_rows, &rows_left, &scale);
    if (BYRANK)
        scatter_by_rank<FIRST>(f, a.gword + b * f.slots, count, sw, prev, e_at, z_at, W, w, lane, tid,
                               scale * a.sign, out_rows, rows_left);
    else
        scatter_by_code<FIRST, TC>(f, sp, wpre, sw, pk_more, sw_more, a.sgn, b, t_at, e_at, c1_at, W, w, lane,
                                   scale * a.sign, out_rows, rows_left);
}

// TC: 0, or the class count of the code-indexed scatter phase when it is the common one
// (243 = 3^5: fused ternary blocks of five or more rows with 4 to 11 waves).
// The arguments every early address depends on come first and as plain values (they can be
// handed to the wave in registers); the rest is grouped.
template <typename VT, int ENC, int NPASS, bool BYRANK, int TC>
__global__ __launch_bounds__(1024, 4) void k_rsr_matvec(
    const uint16_t *__restrict__ entries0, const uint16_t *__restrict__ start0,
    const void *__restrict__ v, int S0, int per0, int rem0, int n_in, int W, long long ldv,
    const PassArgs a0, const FoldArgs f, const PassArgs a1, const OutArgs o) {
    run_pass<VT, ENC, BYRANK, true, TC>(entries0, start0, S0, per0, rem0, a0, v, ldv, n_in, W, f, o,
                                        (int)blockIdx.y);
    if (NPASS == 2) {
        __syncthreads();  // the second pass reuses E and the totals
        run_pass<VT, ENC, BYRANK, false, TC>(a1.entries, a1.start, a1.S, a1.per, a1.rem, a1, v, ldv, n_in,
                                             W, f, o, (int)blockIdx.y);
    }
}

struct LaunchArgs {
    PassArgs a0, a1;
    const void *v;
    long long ldv;
    int n_in, W, nblocks, batch, device;
    FoldArgs f;
    OutArgs o;
    size_t lds;
    hipStream_t stream;
};

constexpr int kCommonClasses = 243;

template <typename VT, int ENC, int NPASS, bool BYRANK, int TC>
hipError_t launch(const LaunchArgs &x) {
    static std::atomic<size_t> enabled[kMaxDevices];
    auto kern = k_rsr_matvec<VT, ENC, NPASS, BYRANK, TC>;
    if (hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(kern), x.lds, x.device, enabled))
        return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)x.nblocks, (unsigned)x.batch), dim3(x.W * 64), x.lds,
                       x.stream, x.a0.entries, x.a0.start, x.v, x.a0.S, x.a0.per, x.a0.rem, x.n_in, x.W, x.ldv,
                       x.a0, x.f, x.a1, x.o);
    return hipGetLastError();
}

template <typename VT, int ENC>
hipError_t launch_nr(const LaunchArgs &x, int npass, bool by_rank) {
    if (by_rank) return npass == 1 ? launch<VT, ENC, 1, true, 0>(x) : launch<VT, ENC, 2, true, 0>(x);
    if (npass == 1 && x.f.Tc == kCommonClasses) return launch<VT, ENC, 1, false, kCommonClasses>(x);
    return npass == 1 ? launch<VT, ENC, 1, false, 0>(x) : launch<VT, ENC, 2, false, 0>(x);
}

// ---- preprocessing-time tables of the code-indexed scatter phase --------------------------
template <int BASE>
__device__ __forceinline__ int sgn_digit(uint32_t c, int r) {
    for (int i = 0; i < r; ++i) c /= BASE;
    const uint32_t d = c % BASE;
    if (BASE == 2) return (int)d;
    return d == 1u ? 1 : d == 2u ? -1 : 0;
}

// fpack[r][g][lane], r < k: byte u holds the weight of j = lane + 64 (4g + u) in row r:
// r < m: sgn_r(j) - sgn_r((j+1) mod Tc) for j < Tc (class j); m <= r < k:
// sgn_{r-m}(j) - sgn_{r-m}(j+1) for j < Q (entry E[Tc*j + Tc-1]); 0 past the end.
// fshare[t] for every thread t of the workgroup: first E index of its level-1 share,
// (class) + Tc * cnt1 * (part), or 0xffffffff for threads without a share.
template <int BASE>
__global__ void k_fold_tables(int k, FoldShape fs, int threads, uint32_t *__restrict__ fpack,
                              uint32_t *__restrict__ fshare) {
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t < k * fs.G * 64) {
        const int lane = t & 63, g = (t >> 6) % fs.G, r = (t >> 6) / fs.G;
        uint32_t pk = 0;
        for (int u = 0; u < 4; ++u) {
            const int j = lane + 64 * (4 * g + u);
            int wgt = 0;
            if (r < fs.m) {
                if (j < fs.Tc)
                    wgt = sgn_digit<BASE>(j, r) - sgn_digit<BASE>((j + 1 == fs.Tc) ? 0 : j + 1, r);
            } else if (j < fs.Q) {
                wgt = sgn_digit<BASE>(j, r - fs.m) - sgn_digit<BASE>(j + 1, r - fs.m);
            }
            pk |= ((uint32_t)wgt & 0xffu) << (8 * u);
        }
        fpack[t] = pk;
    }
    if (t < threads) {
        uint32_t share = 0xffffffffu;
        if (t < fs.Tc * fs.parts) {
            const int part = t / fs.Tc, cls = t - part * fs.Tc;
            share = (uint32_t)(cls + fs.Tc * fs.cnt1 * part);
        }
        fshare[t] = share;
    }
}

}  // namespace

int choose_waves(int64_t slabs, int64_t nb, int k, bool by_rank) {
    // A wave should own at most four slabs (one group: every load of the wave is requested
    // up front).
    const int64_t need = (slabs + kGroupSlabs - 1) / kGroupSlabs;
    int w;
    if (!by_rank && k <= 8) {
        // E by code, up to eight rows: one wave per output row.  The second level of the
        // scatter phase then is one straight pass per wave; fewer waves make some of them
        // loop over rows (measured 15 to 30 % slower), more waves only add the fixed cost a
        // wave has (4096 x 4096: fused k = 4, 6, 8 best at 4, 6, 8 waves; binary 1024 x 1024,
        // k = 8, three slabs: 4.5 us with three waves, 3.4 us with eight, five of them
        // without a slab).  Longer streams take more waves, beyond 16 eight waves that work
        // through several groups.
        w = (int)(need > k ? need : k);
        if (w > kMaxWaves) w = 8;
    } else {
        // Otherwise 1, 2 or 4 slabs per wave as the stream grows and at most 8 waves, so that
        // two workgroups share a CU; with three or more rounds of 8-wave workgroups (1536
        // blocks) half the waves per block keep twice as many blocks in flight.  E by code
        // with more than eight rows: at most two rows per wave.
        const int cap = nb >= 1536 ? 4 : 8;
        int per = kGroupSlabs;
        for (int cand = 1; cand <= kGroupSlabs; cand *= 2)
            if ((slabs + cand - 1) / cand <= cap) { per = cand; break; }
        const int64_t waves = (slabs + per - 1) / per;
        w = (int)(waves < 1 ? 1 : waves <= kMaxWaves ? waves : 8);
        if (!by_rank && w < 8 && 2 * w < k) w = (k + 1) / 2 < 8 ? (k + 1) / 2 : 8;
    }
#ifdef RSR_TUNING
    if (const char *s = std::getenv("RSR_W")) {
        const int x = std::atoi(s);
        if (x >= 1 && x <= kMaxWaves) w = x;
    }
#endif
    return w;
}

bool choose_by_rank(int64_t P, int64_t cols, int64_t longest_by_code, int64_t longest_by_rank,
                    int64_t most_groups) {
    if (matvec_lds_bytes(P, cols, 4, kMaxWaves, false) > kLdsBytes) return true;
#ifdef RSR_TUNING
    if (const char *s = std::getenv("RSR_BY_RANK")) return std::atoi(s) != 0;
#endif
    // bytes per block beside the real entries: 2 per placeholder against 4 per group; the
    // rank-indexed scatter phase costs about k multiply-adds per group more, so it has to
    // win clearly
    return 2 * (longest_by_code - longest_by_rank) > 3 * 4 * most_groups;
}

void make_fold_shape(int base, int k, int64_t P, int W, FoldShape *fs) {
    const int threads = W * 64;
    int m = 0;
    long long Tc = 1;
    while (m < k && Tc * base <= threads) { Tc *= base; ++m; }
    fs->m = m;
    fs->Tc = (int)Tc;
    fs->Q = (int)(P / Tc);
    int parts = 1;
    if (fs->Q <= fs->Tc) {
        parts = threads / fs->Tc;
        if (parts > 2) parts = 2;  // two additions into one class sum commute; three would not
        if (parts > fs->Q) parts = fs->Q;
        if (parts < 1) parts = 1;
    }
    fs->parts = parts;
    fs->cnt1 = (fs->Q + parts - 1) / parts;
    fs->nrows = fs->Tc > fs->Q ? fs->Tc : fs->Q;
    fs->G = (fs->nrows + 255) / 256;
}

hipError_t launch_fold_tables(int base, int k, const FoldShape &fs, int W, uint32_t *fpack,
                              uint32_t *fshare) {
    const int nthreads = W * 64;
    const int rows = k * fs.G * 64;
    const int span = rows > nthreads ? rows : nthreads;
    const int threads = 256, groups = (span + threads - 1) / threads;
    if (base == 2)
        hipLaunchKernelGGL(k_fold_tables<2>, dim3(groups), dim3(threads), 0, 0, k, fs, nthreads, fpack,
                           fshare);
    else
        hipLaunchKernelGGL(k_fold_tables<3>, dim3(groups), dim3(threads), 0, 0, k, fs, nthreads, fpack,
                           fshare);
    return hipGetLastError();
}

hipError_t launch_rsr_matvec(const rsr_handle_s *h, const void *v, int v_dtype, float scale,
                             float *out, int batch, int64_t ldv, int64_t ldo, hipStream_t stream,
                             const LayerTable *layers) {
    LaunchArgs x;
    const FoldShape &fs = h->fold;
    PassArgs *pa[2] = {&x.a0, &x.a1};
    for (int i = 0; i < 2; ++i) {
        const PassData &pd = h->pass[i < h->npass ? i : 0];
        pa[i]->entries = pd.entries;
        pa[i]->start = pd.start;
        pa[i]->sgn = pd.sgn;
        pa[i]->gword = pd.gword;
        pa[i]->gcount = pd.gcount;
        pa[i]->S = (int)pd.S;
        pa[i]->per = (int)(pd.S / h->W);
        pa[i]->rem = (int)(pd.S % h->W);
        pa[i]->sign = pd.sign;
    }
    x.v = v;
    x.ldv = ldv;
    x.n_in = (int)h->cols;
    x.W = h->W;
    x.nblocks = (int)h->nb;
    x.device = h->device;
    x.batch = batch;
    x.f.fpack = h->fpack;
    x.f.fshare = h->fshare;
    x.f.k = h->k;
    x.f.slots = (int)h->slots;
    x.f.m = fs.m;
    x.f.Tc = fs.Tc;
    x.f.Q = fs.Q;
    x.f.G = fs.G;
    x.f.parts = fs.parts;
    x.f.cnt1 = fs.cnt1;
    x.f.fw = gword_field_bits(h->base);
    x.o.out = out;
    x.o.ldo = ldo;
    x.o.n_out = (int)h->rows;
    x.o.scale = scale;
    if (layers)
        x.o.layers = *layers;
    else
        x.o.layers.n = 0;
    x.lds = (size_t)matvec_lds_bytes(h->slots, h->cols, (v_dtype == RSR_BF16) ? 2 : 4, h->W,
                                     h->by_rank != 0);
    x.stream = stream;
    const bool r = h->by_rank != 0;
    if (v_dtype == RSR_BF16)
        return h->enc == kEncSmall ? launch_nr<uint16_t, kEncSmall>(x, h->npass, r)
                                   : launch_nr<uint16_t, kEncBig>(x, h->npass, r);
    return h->enc == kEncSmall ? launch_nr<float, kEncSmall>(x, h->npass, r)
                               : launch_nr<float, kEncBig>(x, h->npass, r);
}

void rsr_matvec_kernel_name(const rsr_handle_s *h, int v_dtype, char *buf, size_t len) {
    // as a profiler prints the instantiation
    const bool common = !h->by_rank && h->npass == 1 && h->fold.Tc == kCommonClasses;
    std::snprintf(buf, len, "k_rsr_matvec<%s, %d, %d, %s, %d>",
                  v_dtype == RSR_BF16 ? "unsigned short" : "float", h->enc, h->npass,
                  h->by_rank ? "true" : "false", common ? kCommonClasses : 0);
}

}  // namespace rsr
