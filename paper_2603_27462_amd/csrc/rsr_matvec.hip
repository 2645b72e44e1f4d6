// RSR multiply kernel for gfx950 (paper, System Overview: aggregate the entries
// of v of each group of identical column patterns, then distribute every group
// sum once; Kernels Implementation: gather, aggregate and scatter phases).
//
// One workgroup of W waves handles one block of k output rows:
//   gather     the block's stream of 16-bit column entries is read with H
//              coalesced 16-byte loads per lane (a strip of 8H consecutive
//              entries); v sits in LDS and is gathered through the entries
//   aggregate  instead of one sum per group the kernel keeps running prefix
//              sums: the entry that closes group c (tail flag) stores the
//              prefix E[c] = sum of everything up to and including group c.
//              Every code 1..P-1 owns exactly one tail (empty groups have a
//              placeholder entry pointing at a zero slot), so each E[c] is
//              written once with a plain store: no atomics, no zero fill,
//              deterministic.  u[c] = E[c] - E[c-1] is never materialised.
//   scatter    out[r] = sum_c sgn_r(c) u[c] = sum_c E[c] (sgn_r(c) - sgn_r(c+1)),
//              a weighted sum over E in which digit r only matters where it
//              changes: all P entries for the lowest digit, every base-th for
//              the next, and so on (1.5 P or 2 P terms in total).  The weights
//              come from a small table built at preprocessing time.
// Prefixes are local to a wave.  Because the weighted sum is linear in E, the
// total T_w of wave w is folded in afterwards: it is missing from every
// prefix stored by later waves, whose weights telescope to sgn_r(first code
// closed by wave w+1); that sign is precomputed per (block, wave, row).
//
// LDS addresses are raw integers: this kernel owns the whole LDS allocation
// (it declares no static __shared__), so dynamic LDS starts at address 0.
#include <cstdio>
#include <cstdlib>

#include "rsr_device.h"
#include "rsr_internal.h"

namespace rsr {

namespace {

// Kernel arguments.  The ones every address depends on come first and as plain
// scalars; the rest is grouped.
struct PassArgs {
    const uint16_t *entries;
    const uint16_t *codes;
    const int8_t *wsign;
    int C;             // chunks per block
    int cbase, crem;   // wave w owns cbase + (w < crem) chunks, the longer shares first
    float sign;
};

struct FoldArgs {
    const uint32_t *fpack;
    const uint32_t *fshare;
    int k, P, m, Tc, Q, G, parts, cnt1;
};

struct OutArgs {
    float *out;
    long long ldo;
    int n_out;
    float scale;
    int batch;          // number of vectors
    int vper;           // vectors one workgroup handles, one after the other
    long long *stamps;  // [blocks][8] shader-clock stamps of thread 0 (profiling builds only)
    int stop_after;     // profiling builds only: leave the kernel after this phase (0 = never)
};

#ifdef RSR_PHASE_TIMING
#define RSR_STAMP(i)                                                          \
    do {                                                                      \
        if (o.stamps && threadIdx.x == 0 && blockIdx.y == 0)                  \
            o.stamps[blockIdx.x * 16 + (i)] = (long long)__builtin_readcyclecounter(); \
    } while (0)
#else
#define RSR_STAMP(i) do { } while (0)
#endif
#ifdef RSR_PHASE_TIMING
#define RSR_STOP(i) do { if (o.stop_after == (i)) return; } while (0)
#else
#define RSR_STOP(i) do { } while (0)
#endif

// ---- scatter phase: out[r] = sum_c E[c] (sgn_r(c) - sgn_r(c+1)) + wave-total terms -------
// Level 1: thread (part, class t) adds up its share of E[t], E[t + Tc], E[t + 2 Tc], ...
// (the entries that agree with t in the m lowest digits) and leaves the sum in
// C1[part][t]; a class is shared by at most two threads.  Every thread adds the same
// number of entries (cnt1): E is followed by one row of Tc zeros, which the second part
// reads when Q is odd.
// Level 2: one wave per output row.  Rows r < m weigh the class sums with the weight of
// (t, r); rows r >= m weigh E[Tc i + Tc - 1], the only entries where their digit
// changes, with the weight of (i, r).  The wave-total terms join, one scan over the
// wave adds everything up and lane 63 writes the row.
// fpack[r][g][lane] packs, one byte each, the weights of j = lane + 64 (4g + u), u < 4:
// r < m: sgn_r(j) - sgn_r((j+1) mod Tc); m <= r < k: sgn_{r-m}(j) - sgn_{r-m}(j+1).
// share: x = first E index of the thread's level-1 share (0xffffffff: no share).
//
// A wave64 vector instruction occupies its SIMD for four cycles, and with four waves per
// SIMD the vector instruction count is what the phases after the first barrier cost.
// Everything below that does not depend on E -- LDS addresses, unpacked weights,
// predicates -- is therefore computed by prepare_scatter() while the global loads of
// the pass are still in flight, and pinned in registers until it is used.
struct ScatterArgs {
    const uint32_t *fpack;
    int k, m, Tc, Q, G, parts, cnt1;  // G = groups of 256 table entries per row
};

constexpr int kL1Regs = 16;  // level-1 entries per thread covered by prepared addresses

struct ScatterPrep {
    uint32_t a1[kL1Regs];  // level 1: LDS addresses of the thread's first entries
    uint32_t c1_store;     // level 1: where the thread's sum goes
    uint32_t la[8];        // level 2 (one row per wave): class sums / entries of the row
    uint32_t corr_a;       // level 2: wave-total term of lane's wave for this row
    float wf[4];           // level 2: weights of the four elements
    bool has_share;
};

template <typename T>
__device__ __forceinline__ void pin(T &x) {
    asm volatile("" : "+v"(x));
}

__device__ __forceinline__ void prepare_scatter(ScatterPrep &sp, const ScatterArgs &f,
                                                uint2 share2, uint32_t wpre, uint32_t corr_at,
                                                uint32_t e_at, uint32_t c1_at, int W, int w,
                                                int lane, int tid) {
    const uint32_t step = (uint32_t)f.Tc * 4u;
    sp.has_share = share2.x != 0xffffffffu;
    const uint32_t first = e_at + (sp.has_share ? share2.x : 0u) * 4u;
#pragma unroll
    for (int i = 0; i < kL1Regs; ++i) {
        // entries past the share read E[0], which is zero
        sp.a1[i] = (i < f.cnt1) ? first + (uint32_t)i * step : e_at;
        pin(sp.a1[i]);
    }
    sp.c1_store = c1_at + (uint32_t)tid * 4u;  // C1[part][class]: tid = part * Tc + class
    pin(sp.c1_store);
    // level 2, one row per wave (used when G == 1 and k <= W)
    const int r = min(w, f.k - 1);
    const bool low = r < f.m;
    const int n = low ? f.Tc : f.Q;
    const uint32_t base = low ? c1_at : e_at + (uint32_t)(f.Tc - 1) * 4u;
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
    sp.corr_a = (lane < W) ? corr_at + (uint32_t)(lane * 16 + r) * 4u : e_at;
    pin(sp.corr_a);
    sp.wf[0] = (float)(int)(signed char)(wpre & 0xffu);
    sp.wf[1] = (float)(int)(signed char)((wpre >> 8) & 0xffu);
    sp.wf[2] = (float)(int)(signed char)((wpre >> 16) & 0xffu);
    sp.wf[3] = (float)(int)(signed char)(wpre >> 24);
#pragma unroll
    for (int j = 0; j < 4; ++j) pin(sp.wf[j]);
}

template <bool FIRST>
__device__ __forceinline__ void scatter_phase(const ScatterArgs &f, const ScatterPrep &sp,
                                              uint32_t wpre, uint32_t corr_at, uint32_t e_at,
                                              uint32_t c1_at, int W, int w, int lane, int tid,
                                              float sign_scale, float *out_rows,
                                              long long rows_left, const OutArgs &o) {
    if (sp.has_share) {
        float col;
        if (f.cnt1 <= 4) {
            const float x0 = *lds_float(sp.a1[0]), x1 = *lds_float(sp.a1[1]);
            const float x2 = *lds_float(sp.a1[2]), x3 = *lds_float(sp.a1[3]);
            col = (x0 + x1) + (x2 + x3);
        } else {
            float x[kL1Regs];
#pragma unroll
            for (int i = 0; i < kL1Regs; ++i) x[i] = *lds_float(sp.a1[i]);
            float rest = 0.0f;
            if (f.cnt1 > kL1Regs) {
                const uint32_t step = (uint32_t)f.Tc * 4u;
                uint32_t at = sp.a1[kL1Regs - 1] + step;
                for (int i = kL1Regs; i < f.cnt1; ++i) {
                    rest += *lds_float(at);
                    at += step;
                }
            }
#pragma unroll
            for (int d = 1; d < kL1Regs; d *= 2)
#pragma unroll
                for (int i = 0; i + d < kL1Regs; i += 2 * d) x[i] += x[i + d];
            col = x[0] + rest;
        }
        *lds_float(sp.c1_store) = col;
    }
    RSR_STAMP(5);
    __syncthreads();
    RSR_STAMP(6);
    RSR_STOP(3);
    if (f.G == 1 && f.k <= W) {
        // common shape: at most one row per wave, at most 256 table entries per row
        if (w < f.k) {
            const int r = w;
            float v0 = *lds_float(sp.la[0]), v1 = *lds_float(sp.la[1]);
            float v2 = *lds_float(sp.la[2]), v3 = *lds_float(sp.la[3]);
            const float cr = *lds_float(sp.corr_a);
            if (r < f.m && f.parts == 2) {
                const float u0 = *lds_float(sp.la[4]), u1 = *lds_float(sp.la[5]);
                const float u2 = *lds_float(sp.la[6]), u3 = *lds_float(sp.la[7]);
                v0 += u0; v1 += u1; v2 += u2; v3 += u3;
            }
            // entries past the end of the row carry weight 0 in the table
            float x = cr + sp.wf[0] * v0;
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
    for (int r = w; r < f.k; r += W) {
        const bool low = r < f.m;
        const int n = low ? f.Tc : f.Q;
        // element j of the row: class sum C1[0][j] (+ C1[1][j]), or E[Tc j + Tc - 1]
        const uint32_t base = low ? c1_at : e_at + (uint32_t)(f.Tc - 1) * 4u;
        const uint32_t stride = low ? 4u : (uint32_t)f.Tc * 4u;
        const bool two = low && f.parts == 2;
        const uint32_t second = (uint32_t)f.Tc * 4u;
        float x = 0.0f;
        for (int g = 0; g * 256 < n; ++g) {
            const uint32_t pk = (r == w && g == 0) ? wpre : f.fpack[(r * f.G + g) * 64 + lane];
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
        if (lane < W) x += *lds_float(corr_at + (lane * 16 + r) * 4);
        const float tot = wave_inclusive_scan(x);
        if (lane == 63 && r < rows_left) {
            const float term = sign_scale * tot;
            // pass 2 adds to what pass 1 wrote
            __builtin_nontemporal_store(FIRST ? term : out_rows[r] + term, &out_rows[r]);
        }
    }
}

// Requests chunks first..first+PF-1 of a wave (those below `end`): H 16-byte loads and
// one start code per lane and chunk.  ep / cp already point at this lane.
template <int H, int PF>
__device__ __forceinline__ void load_group(const uint4 *ep, const uint16_t *cp, int first, int end,
                                           uint4 (&q)[PF][H], uint32_t (&code)[PF]) {
#pragma unroll
    for (int f = 0; f < PF; ++f) {
#pragma unroll
        for (int h = 0; h < H; ++h) q[f][h] = make_uint4(0u, 0u, 0u, 0u);
        code[f] = 0;
        if (first + f < end) {
#pragma unroll
            for (int h = 0; h < H; ++h) q[f][h] = ep[((first + f) * H + h) * 64];
            code[f] = cp[(first + f) * 64];
        }
    }
}

// One pass (binary, M+, M- or fused) of one block.  FIRST: v still has to be staged into
// LDS and the output rows are overwritten; otherwise the pass adds to them.
template <typename VT, int H, int ENC, bool FIRST>
__device__ __forceinline__ void run_pass(const PassArgs &a, const void *v, long long ldv, int n_in,
                                         int W, const FoldArgs &f, const OutArgs &o, int vec) {
    constexpr int PF = 4 / H;  // chunks requested together (16 dwords per lane)
    // LDS (byte addresses): v (n_in + zero slot) | wave-total terms | E[P] | Tc zeros | C1[threads]
    const uint32_t vbytes = ((n_in + 1) * (uint32_t)sizeof(VT) + 15u) & ~15u;
    const uint32_t corr_at = vbytes;          // float [16 waves][16 rows]
    const uint32_t e_at = vbytes + kLdsMisc;  // float [P]

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nthreads = W * 64;
    const long long b = blockIdx.x;

    const int C = a.C;
    const int c0 = w * a.cbase + min(w, a.crem);
    const int c1 = c0 + a.cbase + (w < a.crem ? 1 : 0);
    const uint4 *ep = reinterpret_cast<const uint4 *>(a.entries) + (b * C * H) * 64 + lane;
    const uint16_t *cp = a.codes + (b * C) * 64 + lane;

    // chunks are consumed in groups of PF; a group's loads (PF*H 16-byte loads per
    // lane) are all in flight before its first entry is used, and the next group is
    // requested before the current one is processed
    uint4 q[PF][H];
    uint32_t code[PF];
    // requested now, used after the gather phase:
    // per (wave, row): sign of row r's digit in the first code closed by wave w+1
    const int8_t wsg8 = a.wsign[(b * W + w) * 16 + (lane & 15)];
    // scatter phase: this thread's level-1 share and the weights of the wave's first row
    const ScatterArgs sa = {f.fpack, f.k, f.m, f.Tc, f.Q, f.G, f.parts, f.cnt1};
    const uint2 share = make_uint2(f.fshare[tid], 0u);
    const uint32_t wpre = f.fpack[(min(w, f.k - 1) * f.G) * 64 + lane];
    const uint32_t z_at = e_at + (uint32_t)f.P * 4u;    // float [Tc]: zeros behind E
    const uint32_t c1_at = z_at + (uint32_t)f.Tc * 4u;  // float [threads]: level-1 sums
    if (FIRST) {
        // stage v into LDS (16-byte copies when the source allows it); requested
        // before the stream so that it arrives first
        const unsigned char *vg = reinterpret_cast<const unsigned char *>(v) +
                                  (long long)vec * ldv * (long long)sizeof(VT);
        const int nbytes = n_in * (int)sizeof(VT);
        if ((reinterpret_cast<uintptr_t>(vg) & 15) == 0) {
            const int n16 = nbytes >> 4;
            const u32x4 *v16 = reinterpret_cast<const u32x4 *>(vg);
            lds_u128 *l16 = reinterpret_cast<lds_u128 *>(static_cast<uintptr_t>(0));
            for (int j0 = 0; j0 < n16; j0 += 4 * nthreads) {
                // loads past the end are redirected to the last valid 16 bytes
                const int j_0 = j0 + tid, j_1 = j_0 + nthreads, j_2 = j_1 + nthreads,
                          j_3 = j_2 + nthreads;
                const u32x4 s0 = v16[min(j_0, n16 - 1)];
                const u32x4 s1 = v16[min(j_1, n16 - 1)];
                const u32x4 s2 = v16[min(j_2, n16 - 1)];
                const u32x4 s3 = v16[min(j_3, n16 - 1)];
                if (j0 == 0) load_group<H, PF>(ep, cp, c0, c1, q, code);
                if (j_0 < n16) l16[j_0] = s0;
                if (j_1 < n16) l16[j_1] = s1;
                if (j_2 < n16) l16[j_2] = s2;
                if (j_3 < n16) l16[j_3] = s3;
            }
            if (n16 == 0) load_group<H, PF>(ep, cp, c0, c1, q, code);
            for (int j = (n16 << 4) + tid * (int)sizeof(VT); j < nbytes;
                 j += nthreads * (int)sizeof(VT))
                lds_store_v<VT>(j, *reinterpret_cast<const VT *>(vg + j));
        } else {
            load_group<H, PF>(ep, cp, c0, c1, q, code);
            for (int j = tid * (int)sizeof(VT); j < nbytes; j += nthreads * (int)sizeof(VT))
                lds_store_v<VT>(j, *reinterpret_cast<const VT *>(vg + j));
        }
        if (tid == 0) lds_store_v<VT>(nbytes, VT(0));
    } else {
        load_group<H, PF>(ep, cp, c0, c1, q, code);
    }
    if (tid == 0) *lds_float(e_at) = 0.0f;
    if (tid < f.Tc) *lds_float(z_at + (uint32_t)tid * 4u) = 0.0f;
    __syncthreads();
    RSR_STAMP(1);

    // ---- gather + aggregate ------------------------------------------------
    float run = 0.0f;
    uint32_t g[H][8];
#pragma unroll
    for (int h = 0; h < H; ++h)
#pragma unroll
        for (int i = 0; i < 8; ++i) g[h][i] = 0u;
    for (int it = c0; it < c1; it += PF) {
        uint4 qn[PF][H];
        uint32_t coden[PF];
        load_group<H, PF>(ep, cp, it + PF, c1, qn, coden);
#pragma unroll
        for (int f = 0; f < PF; ++f) {
            if (it + f < c1) {
                uint32_t d[H][4];
#pragma unroll
                for (int h = 0; h < H; ++h) {
                    d[h][0] = q[f][h].x; d[h][1] = q[f][h].y;
                    d[h][2] = q[f][h].z; d[h][3] = q[f][h].w;
                }
                // gathers of 16-byte load h+1 are issued before those of load h are used
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    gather<VT>(g[0][2 * j], entry_addr<VT, ENC, 0>(d[0][j]));
                    gather<VT>(g[0][2 * j + 1], entry_addr<VT, ENC, 1>(d[0][j]));
                }
                float s[H][8];
                float prev = 0.0f;
#pragma unroll
                for (int h = 0; h < H; ++h) {
                    if (h + 1 < H) {
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            gather<VT>(g[h + 1][2 * j], entry_addr<VT, ENC, 0>(d[h + 1][j]));
                            gather<VT>(g[h + 1][2 * j + 1], entry_addr<VT, ENC, 1>(d[h + 1][j]));
                        }
                        lds_wait<8>(g[h]);
                    } else {
                        lds_wait<0>(g[h]);
                    }
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        prev += __uint_as_float(g[h][i]);
                        s[h][i] = prev;
                    }
                }
                const float incl = wave_inclusive_scan(prev);
                const float base = run + wave_shift_right(incl);
                uint32_t ptr = e_at + code[f] * 4u;
#pragma unroll
                for (int h = 0; h < H; ++h) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        tail_store2<ENC>(d[h][j], base, s[h][2 * j], s[h][2 * j + 1], ptr);
                    }
                }
                run += lane63(incl);
            }
        }
#pragma unroll
        for (int f = 0; f < PF; ++f) {
#pragma unroll
            for (int h = 0; h < H; ++h) q[f][h] = qn[f][h];
            code[f] = coden[f];
        }
    }
    RSR_STAMP(2);
    if (lane < 16) *lds_float(corr_at + (w * 16 + lane) * 4) = run * (float)wsg8;
    // (this kernel keeps its registers for the chunk loop: the scatter constants are made here)
    ScatterPrep sp;
    prepare_scatter(sp, sa, share, wpre, corr_at, e_at, c1_at, W, w, lane, tid);
    lds_drain();
    __syncthreads();
    RSR_STAMP(3);

    // ---- scatter ----------------------------------------------------------------
    scatter_phase<FIRST>(sa, sp, wpre, corr_at, e_at, c1_at, W, w, lane, tid,
                         o.scale * a.sign, o.out + (long long)vec * o.ldo + b * f.k,
                         (long long)o.n_out - b * f.k, o);
}

template <typename VT, int H, int ENC, int NPASS>
__global__ __launch_bounds__(1024) void k_rsr_matvec(const PassArgs a0, const void *v,
                                                     long long ldv, int n_in, int W,
                                                     const FoldArgs f, const PassArgs a1,
                                                     const OutArgs o) {
    RSR_STAMP(0);
    run_pass<VT, H, ENC, true>(a0, v, ldv, n_in, W, f, o, (int)blockIdx.y);
    if (NPASS == 2) {
        __syncthreads();
        run_pass<VT, H, ENC, false>(a1, v, ldv, n_in, W, f, o, (int)blockIdx.y);
    }
    RSR_STAMP(7);
}

// ---- one chunk per wave ---------------------------------------------------------------
// The common shape: the block's stream has at most W chunks, wave w owns chunk w, and
// nothing loops.  Same phases as run_pass, with every load of the pass requested up front
// and the scatter-phase constants prepared while they are in flight.  MULTI: the workgroup
// multiplies several vectors in turn with the stream kept in registers.

// What a wave loads of its chunk: H 16-byte pieces of stream per lane and the strip's start
// code.
template <int H>
struct StreamRegs {
    uint4 q[H];
    uint32_t code;
};

// The stream is read once: non-temporal loads keep it out of the way of v and the tables.
// Waves without a chunk (w >= C) load the last chunk and ignore it: no branch, so nothing
// delays the requests.
template <int H>
__device__ __forceinline__ void load_stream(StreamRegs<H> &r, const uint16_t *__restrict__ entries,
                                            const uint16_t *__restrict__ codes, int C, long long b,
                                            int w, int lane) {
    const int wc = min(w, C - 1);
    const u32x4 *ep = reinterpret_cast<const u32x4 *>(entries) + ((b * C + wc) * H) * 64 + lane;
#pragma unroll
    for (int h = 0; h < H; ++h) {
        const u32x4 t = __builtin_nontemporal_load(&ep[h * 64]);
        r.q[h] = make_uint4(t.x, t.y, t.z, t.w);
    }
    r.code = __builtin_nontemporal_load(&codes[(b * C + wc) * 64 + lane]);
}

struct SecondPass {
    const uint16_t *entries;
    const uint16_t *codes;
    const int8_t *wsign;
    int C;
    float sign;
};

// NEXT: the pass also requests the stream of the pass that follows it (two-pass kinds),
// after its first barrier, into `next`; PRE: the pass finds its own stream in `pre`.
template <typename VT, int H, int ENC, bool FIRST, bool MULTI, bool NEXT, bool PRE>
__device__ __forceinline__ void single_pass(const uint16_t *__restrict__ entries,
                                            const uint16_t *__restrict__ codes,
                                            const int8_t *__restrict__ wsign, int C, float sign,
                                            const void *__restrict__ v, long long ldv, int n_in,
                                            int W, const FoldArgs &f, float *out, long long ldo,
                                            int n_out, float scale, const OutArgs &o, int vec0,
                                            int nvec_arg, const SecondPass *nextp,
                                            StreamRegs<H> *next, const StreamRegs<H> *pre) {
    const int nvec = MULTI ? nvec_arg : 1;
    const uint32_t vbytes = ((n_in + 1) * (uint32_t)sizeof(VT) + 15u) & ~15u;
    const uint32_t corr_at = vbytes;                    // float [16 waves][16 rows]
    const uint32_t e_at = vbytes + kLdsMisc;            // float [P]
    const uint32_t z_at = e_at + (uint32_t)f.P * 4u;    // float [Tc]: zeros behind E
    const uint32_t c1_at = z_at + (uint32_t)f.Tc * 4u;  // float [threads]: level-1 sums
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nthreads = W * 64;
    const long long b = blockIdx.x;
    const ScatterArgs sa = {f.fpack, f.k, f.m, f.Tc, f.Q, f.G, f.parts, f.cnt1};
    const bool active = w < C;  // this wave owns a chunk

    // ---- every global load of the pass is requested here: the small tables first (they
    // are turned into scatter-phase constants while the rest is in flight), then v, then
    // the stream ------------------------------------------------------------------------------
    const uint2 share = make_uint2(f.fshare[tid], 0u);
    const uint32_t wpre = f.fpack[(min(w, f.k - 1) * f.G) * 64 + lane];
    // (requested before the stream: it is converted while the stream is still in flight)
    const int8_t wsg8 = wsign[(b * W + w) * 16 + (lane & 15)];
    // vectors vec0 .. vec0+nvec-1 are multiplied one after the other with the same stream
    // registers (nvec > 1 only in the first pass of one-pass kinds)
    const long long vstride = ldv * (long long)sizeof(VT);
    const unsigned char *vg = reinterpret_cast<const unsigned char *>(v) + (long long)vec0 * vstride;
    const int nbytes = n_in * (int)sizeof(VT);
    const int n16 = nbytes >> 4;
    const bool v_aligned = (reinterpret_cast<uintptr_t>(vg) & 15) == 0 && (nvec == 1 || (vstride & 15) == 0);
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
    StreamRegs<H> own;
    if (PRE)
        own = *pre;
    else
        load_stream<H>(own, entries, codes, C, b, w, lane);
    uint4 q[H];
#pragma unroll
    for (int h = 0; h < H; ++h) q[h] = own.q[h];
    uint32_t code = own.code;

    // ---- work that needs no stream data, done while the loads are in flight ----------------
    ScatterPrep sp;
    if (!MULTI) prepare_scatter(sp, sa, share, wpre, corr_at, e_at, c1_at, W, w, lane, tid);
    float wsg = (float)wsg8;
    pin(wsg);
    uint32_t g[H][8];  // gather targets: for bf16 the low halves must be zero
#pragma unroll
    for (int h = 0; h < H; ++h)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            g[h][i] = 0u;
            pin(g[h][i]);
        }
    if (tid < f.Tc) *lds_float(z_at + (uint32_t)tid * 4u) = 0.0f;

    // ---- stage v (the first vector comes from the registers requested above) --------------
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
    for (int vi = 0; vi < nvec; ++vi) {
    if (MULTI && FIRST && vi > 0) {
        // later vectors: every wave is past the gather phase of the previous one
        if (v_aligned) {
            for (int j = tid; j < n16; j += nthreads) l16[j] = v16[j];
            for (int j = (n16 << 4) + tid * (int)sizeof(VT); j < nbytes;
                 j += nthreads * (int)sizeof(VT))
                lds_store_v<VT>(j, *reinterpret_cast<const VT *>(vg + j));
        } else {
            for (int j = tid * (int)sizeof(VT); j < nbytes; j += nthreads * (int)sizeof(VT))
                lds_store_v<VT>(j, *reinterpret_cast<const VT *>(vg + j));
        }
    }
    if (tid == 0) *lds_float(e_at) = 0.0f;
    __syncthreads();
    RSR_STAMP(1);
    RSR_STOP(1);
    // the following pass's stream is requested once this pass's own data is here, so that
    // the two do not compete for HBM, and arrives while this pass computes
    if (NEXT && vi == 0) load_stream_second<H>(*next, nextp, b, w, lane);
    if (MULTI && FIRST) {  // from here on vg is the next vector
        vg += vstride;
        v16 = reinterpret_cast<const u32x4 *>(vg);
    }

    // ---- gather + aggregate -------------------------------------------------------------
    float total = 0.0f;
    asm volatile("" : "+v"(code));  // first use of the stream: nothing above waits for it
    if (active) {
        uint32_t d[H][4];
#pragma unroll
        for (int h = 0; h < H; ++h) {
            d[h][0] = q[h].x; d[h][1] = q[h].y; d[h][2] = q[h].z; d[h][3] = q[h].w;
        }
        // gathers of 16-byte load h+1 are issued before those of load h are used
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            gather<VT>(g[0][2 * j], entry_addr<VT, ENC, 0>(d[0][j]));
            gather<VT>(g[0][2 * j + 1], entry_addr<VT, ENC, 1>(d[0][j]));
        }
        float s[H][8];
        float prev = 0.0f;
#pragma unroll
        for (int h = 0; h < H; ++h) {
            if (h + 1 < H) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    gather<VT>(g[h + 1][2 * j], entry_addr<VT, ENC, 0>(d[h + 1][j]));
                    gather<VT>(g[h + 1][2 * j + 1], entry_addr<VT, ENC, 1>(d[h + 1][j]));
                }
                lds_wait<8>(g[h]);
            } else {
                RSR_STAMP(8);
                lds_wait<0>(g[h]);
                RSR_STAMP(9);
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                prev = (h == 0 && i == 0) ? __uint_as_float(g[0][0]) : prev + __uint_as_float(g[h][i]);
                s[h][i] = prev;
            }
        }
        RSR_STAMP(10);
        const float incl = wave_inclusive_scan(prev);
        const float base = wave_shift_right(incl);
        RSR_STAMP(11);
        uint32_t ptr = e_at + code * 4u;
#pragma unroll
        for (int h = 0; h < H; ++h) {
            if (ENC == kEncSmall) {
                tail_store8_small(d[h][0], d[h][1], d[h][2], d[h][3], base, s[h], ptr);
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    tail_store2<ENC>(d[h][j], base, s[h][2 * j], s[h][2 * j + 1], ptr);
            }
        }
        total = lane63(incl);
    }
    RSR_STAMP(2);
    if (lane < 16) *lds_float(corr_at + (w * 16 + lane) * 4) = total * wsg;
    lds_drain();
    __syncthreads();
    RSR_STAMP(3);
    RSR_STOP(2);

    // ---- scatter ----------------------------------------------------------------------
    // (with several vectors the registers are needed for the stream: constants are made here)
    if (MULTI) {
        // opaque copies, so that the constants are recomputed here rather than kept alive
        int tid_i = tid;
        uint2 share_i = share;
        uint32_t wpre_i = wpre;
        pin(tid_i);
        pin(share_i.x);
        pin(wpre_i);
        prepare_scatter(sp, sa, share_i, wpre_i, corr_at, e_at, c1_at, W, w, tid_i & 63, tid_i);
    }
    scatter_phase<FIRST>(sa, sp, wpre, corr_at, e_at, c1_at, W, w, lane, tid, scale * sign,
                         out + (long long)(vec0 + vi) * ldo + b * f.k, (long long)n_out - b * f.k, o);
    }
}

template <int H>
__device__ __forceinline__ void load_stream_second(StreamRegs<H> &r, const SecondPass *p, long long b,
                                                   int w, int lane) {
    load_stream<H>(r, p->entries, p->codes, p->C, b, w, lane);
}

template <typename VT, int H, int ENC, int NPASS, bool MULTI>
__global__ __launch_bounds__(1024, 4) void k_rsr_matvec1(
    const uint16_t *__restrict__ entries0, const uint16_t *__restrict__ codes0,
    const void *__restrict__ v, int C0, int n_in, int W, long long ldv,
    const int8_t *__restrict__ wsign0, const FoldArgs f, float sign0, const SecondPass a1,
    const OutArgs o) {
    RSR_STAMP(0);
#ifdef RSR_PHASE_TIMING
    if (o.stamps && threadIdx.x == 0 && blockIdx.y == 0) {  // where the workgroup runs
        o.stamps[blockIdx.x * 16 + 12] = __builtin_amdgcn_s_getreg((4) | (0 << 6) | (31 << 11));   // HW_ID
        o.stamps[blockIdx.x * 16 + 13] = __builtin_amdgcn_s_getreg((20) | (0 << 6) | (31 << 11));  // XCC_ID
    }
#endif
    // MULTI (one-pass kinds only): the workgroup multiplies o.vper vectors one after the
    // other, keeping the stream in registers; otherwise one vector per workgroup
    const int vec0 = MULTI ? blockIdx.y * o.vper : blockIdx.y;
    const int nvec = MULTI ? min(o.vper, o.batch - vec0) : 1;
    // two passes: the second pass's stream is requested while the first pass computes (kept in
    // registers meanwhile; not for the largest chunk size, which has none to spare)
    constexpr bool kAhead = NPASS == 2 && H <= 2;
    StreamRegs<H> second;
    single_pass<VT, H, ENC, true, MULTI, kAhead, false>(entries0, codes0, wsign0, C0, sign0, v, ldv,
                                                        n_in, W, f, o.out, o.ldo, o.n_out, o.scale, o,
                                                        vec0, nvec, &a1, &second, nullptr);
    if (NPASS == 2) {
        __syncthreads();
        single_pass<VT, H, ENC, false, false, false, kAhead>(a1.entries, a1.codes, a1.wsign, a1.C,
                                                             a1.sign, v, ldv, n_in, W, f, o.out, o.ldo,
                                                             o.n_out, o.scale, o, vec0, 1, nullptr,
                                                             nullptr, &second);
    }
    RSR_STAMP(7);
}

struct LaunchArgs {
    PassArgs a0, a1;
    const void *v;
    long long ldv;
    int n_in, W, npass, nblocks, batch, device;
    FoldArgs f;
    OutArgs o;
    size_t lds;
    hipStream_t stream;
    bool single;  // every pass has at most W chunks: one chunk per wave, no loops
};

template <typename VT, int H, int ENC, int NPASS, bool MULTI>
hipError_t launch_single(const LaunchArgs &x) {
    static std::atomic<size_t> enabled[kMaxDevices];
    auto kern = k_rsr_matvec1<VT, H, ENC, NPASS, MULTI>;
    if (hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(kern), x.lds, x.device, enabled))
        return e;
    SecondPass a1;
    a1.entries = x.a1.entries;
    a1.codes = x.a1.codes;
    a1.wsign = x.a1.wsign;
    a1.C = x.a1.C;
    a1.sign = x.a1.sign;
    const int groups = MULTI ? (x.batch + x.o.vper - 1) / x.o.vper : x.batch;
    hipLaunchKernelGGL(kern, dim3((unsigned)x.nblocks, (unsigned)groups),
                       dim3(x.W * 64), x.lds, x.stream, x.a0.entries, x.a0.codes, x.v, x.a0.C, x.n_in, x.W, x.ldv,
                       x.a0.wsign, x.f, x.a0.sign, a1, x.o);
    return hipGetLastError();
}

template <typename VT, int H, int ENC, int NPASS>
hipError_t launch(const LaunchArgs &x) {
    if (x.single) {
        if (NPASS == 1 && x.o.vper > 1) return launch_single<VT, H, ENC, 1, true>(x);
        return launch_single<VT, H, ENC, NPASS, false>(x);
    }
    static std::atomic<size_t> enabled[kMaxDevices];
    auto kern = k_rsr_matvec<VT, H, ENC, NPASS>;
    if (hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(kern), x.lds, x.device, enabled))
        return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)x.nblocks, (unsigned)x.batch),
                       dim3(x.W * 64), x.lds, x.stream, x.a0, x.v, x.ldv, x.n_in, x.W, x.f, x.a1, x.o);
    return hipGetLastError();
}

template <typename VT, int H, int ENC>
hipError_t launch_n(const LaunchArgs &x) {
    return x.npass == 1 ? launch<VT, H, ENC, 1>(x) : launch<VT, H, ENC, 2>(x);
}

template <typename VT>
hipError_t launch_he(const LaunchArgs &x, int H, int enc) {
    if (enc == kEncSmall) {
        if (H == 1) return launch_n<VT, 1, kEncSmall>(x);
        if (H == 2) return launch_n<VT, 2, kEncSmall>(x);
        return launch_n<VT, 4, kEncSmall>(x);
    }
    if (H == 1) return launch_n<VT, 1, kEncBig>(x);
    if (H == 2) return launch_n<VT, 2, kEncBig>(x);
    return launch_n<VT, 4, kEncBig>(x);
}

// ---- preprocessing-time tables of the scatter phase ------------------------------------
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

// wsign[b][w][r] = sgn_r(first code closed by wave w+1) (0 for the last wave): the
// weight with which the total of wave w enters output row r.
template <int BASE>
__global__ void k_wave_signs(const uint16_t *__restrict__ codes, long long nb, int C, int W, int k,
                             FoldShape fs, int pass, int8_t *__restrict__ wsign) {
    const long long gid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= nb * W * 16) return;
    const int r = (int)(gid & 15);
    const int w = (int)((gid >> 4) % W);
    const long long b = (gid >> 4) / W;
    int s = 0;
    if (w + 1 < W && r < k && fs.cb[pass][w + 1] < C) {  // waves past the last chunk close nothing
        const uint32_t c = codes[(b * C + fs.cb[pass][w + 1]) * 64];
        s = sgn_digit<BASE>(c, r);
    }
    wsign[gid] = (int8_t)s;
}

}  // namespace

void choose_launch_shape(int64_t longest, int64_t nb, int *H, int *W) {
    // Preferred: one chunk per wave and at most 8 waves, so that two workgroups share a CU
    // without register pressure; the chunk grows with the stream (H = 1, 2, 4).  Longer
    // streams take up to 16 waves, and beyond that 8 waves that loop over their chunks.
    // A CU runs 16 of these waves: with three or more rounds of 8-wave workgroups (1536
    // blocks) it pays to halve the waves per block and keep twice as many blocks in flight
    // (measured: 14336 x 4096, k = 8: 12.1 -> 10.5 us; 13824 x 2560, k = 6: 10.7 -> 9.0 us).
    const int kWaves = nb >= 1536 ? 4 : 8;
    int h = 4;
    for (int cand = 1; cand <= 4; cand *= 2)
        if ((longest + kLoad * cand - 1) / (kLoad * cand) <= kWaves) { h = cand; break; }
    if (const char *s = std::getenv("RSR_H")) {
        const int x = std::atoi(s);
        if (x == 1 || x == 2 || x == 4) h = x;
    }
    const int64_t chunks = (longest + kLoad * h - 1) / (kLoad * h);
    int w = (int)(chunks < 1 ? 1 : chunks <= kMaxWaves ? chunks : 8);
    if (const char *s = std::getenv("RSR_W")) {
        const int x = std::atoi(s);
        if (x >= 1 && x <= kMaxWaves) w = x;
    }
    *H = h;
    *W = w;
}

void make_fold_shape(int base, int k, int64_t P, int W, const int64_t C[2], int npass,
                     FoldShape *fs) {
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
    const int span1 = fs->Tc * parts;
    const int span2 = fs->Q < threads ? fs->Q : threads;
    fs->nact = ((span1 > span2 ? span1 : span2) + 63) / 64;
    fs->nrows = fs->Tc > fs->Q ? fs->Tc : fs->Q;
    fs->G = (fs->nrows + 255) / 256;
    for (int ps = 0; ps < 2; ++ps)
        for (int w = 0; w <= kMaxWaves; ++w)
            fs->cb[ps][w] = (unsigned short)((ps < npass && w <= W)
                                                 ? w * (C[ps] / W) + (w < C[ps] % W ? w : C[ps] % W)
                                                 : 0);
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

bool matvec_is_single(const rsr_handle_s *h) {
    for (int ps = 0; ps < h->npass; ++ps)
        if (h->pass[ps].C > h->W) return false;
    return true;
}

hipError_t launch_wave_signs(int base, int k, const uint16_t *codes, int64_t nb, int64_t C, int W,
                             const FoldShape &fs, int pass, int8_t *wsign) {
    const long long total = nb * W * 16;
    const int threads = 256;
    const unsigned groups = (unsigned)((total + threads - 1) / threads);
    if (base == 2)
        hipLaunchKernelGGL(k_wave_signs<2>, dim3(groups), dim3(threads), 0, 0, codes, (long long)nb,
                           (int)C, W, k, fs, pass, wsign);
    else
        hipLaunchKernelGGL(k_wave_signs<3>, dim3(groups), dim3(threads), 0, 0, codes, (long long)nb,
                           (int)C, W, k, fs, pass, wsign);
    return hipGetLastError();
}

hipError_t launch_rsr_matvec(const rsr_handle_s *h, const void *v, int v_dtype, float scale,
                             float *out, int batch, int64_t ldv, int64_t ldo, hipStream_t stream) {
    LaunchArgs x;
    const FoldShape &fs = h->fold;
    PassArgs *pa[2] = {&x.a0, &x.a1};
    for (int i = 0; i < 2; ++i) {
        const PassData &pd = h->pass[i < h->npass ? i : 0];
        pa[i]->entries = pd.entries;
        pa[i]->codes = pd.codes;
        pa[i]->wsign = pd.wsign;
        pa[i]->C = (int)pd.C;
        pa[i]->cbase = (int)(pd.C / h->W);
        pa[i]->crem = (int)(pd.C % h->W);
        pa[i]->sign = pd.sign;
    }
    x.v = v;
    x.ldv = ldv;
    x.n_in = (int)h->cols;
    x.W = h->W;
    x.npass = h->npass;
    x.nblocks = (int)h->nb;
    x.device = h->device;
    x.batch = batch;
    x.f.fpack = h->fpack;
    x.f.fshare = h->fshare;
    x.f.k = h->k;
    x.f.P = (int)h->P;
    x.f.m = fs.m;
    x.f.Tc = fs.Tc;
    x.f.Q = fs.Q;
    x.f.G = fs.G;
    x.f.parts = fs.parts;
    x.f.cnt1 = fs.cnt1;
    x.o.out = out;
    x.o.ldo = ldo;
    x.o.n_out = (int)h->rows;
    x.o.scale = scale;
    x.o.batch = batch;
    // enough workgroups to fill the chip twice over first, then several vectors per workgroup
    // (measured: keeping the stream in registers pays once there are that many workgroups)
    {
        static const int forced = [] {  // RSR_VPER overrides the choice (tuning only)
            const char *e = std::getenv("RSR_VPER");
            return e ? std::atoi(e) : 0;
        }();
        const long long per = forced > 0 ? forced : (long long)h->nb * batch / 1024;
        x.o.vper = (int)(per < 1 ? 1 : per > batch ? batch : per);
    }
    x.o.stamps = nullptr;
    x.o.stop_after = 0;
#ifdef RSR_PHASE_TIMING
    if (const char *sp = std::getenv("RSR_STOP_AFTER")) x.o.stop_after = std::atoi(sp);
    if (const char *sp = std::getenv("RSR_STAMPS"))
        x.o.stamps = reinterpret_cast<long long *>(std::strtoull(sp, nullptr, 0));
#endif
    x.lds = (size_t)matvec_lds_bytes(h->P, h->cols, (v_dtype == RSR_BF16) ? 2 : 4, h->W);
    x.stream = stream;
    x.single = matvec_is_single(h);
    return (v_dtype == RSR_BF16) ? launch_he<uint16_t>(x, h->H, h->enc)
                                 : launch_he<float>(x, h->H, h->enc);
}

const char *rsr_matvec_kernel_name(int v_dtype, int H, int enc, int npass, bool single) {
    // one static string per instantiation, as a profiler prints the template arguments
    static char names[2][2][3][2][2][64];
    const int hi = (H == 1) ? 0 : (H == 2) ? 1 : 2;
    char *n = names[single][v_dtype == RSR_BF16][hi][enc == kEncBig][npass == 2];
    if (!n[0])
        std::snprintf(n, sizeof(names[0][0][0][0][0]), "k_rsr_matvec%s<%s, %d, %d, %d%s>",
                      single ? "1" : "", v_dtype == RSR_BF16 ? "unsigned short" : "float", H, enc,
                      npass, single ? ", false" : "");  // one vector per workgroup
    return n;
}

}  // namespace rsr
