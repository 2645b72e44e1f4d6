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
    const int8_t *ftab;
    int ib[5];  // stage-1 share of part j: [ib[j], ib[j+1])
    int k, P, m, Tc, Q, parts, nact, nrows;
};

struct OutArgs {
    float *out;
    long long ldo;
    int n_out;
    float scale;
    long long *stamps;  // [blocks][8] shader-clock stamps of thread 0 (profiling builds only)
};

#ifdef RSR_PHASE_TIMING
#define RSR_STAMP(i)                                                          \
    do {                                                                      \
        if (o.stamps && threadIdx.x == 0 && blockIdx.y == 0)                  \
            o.stamps[blockIdx.x * 8 + (i)] = (long long)__builtin_readcyclecounter(); \
    } while (0)
#else
#define RSR_STAMP(i) do { } while (0)
#endif

typedef __attribute__((address_space(3))) float lds_f32;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) u32x4 lds_u128;

__device__ __forceinline__ lds_f32 *lds_float(uint32_t addr) {
    return reinterpret_cast<lds_f32 *>(static_cast<uintptr_t>(addr));
}

// ---- cross-lane primitives (DPP; wave64) -------------------------------------------
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_add(float x) {
    // x + (x moved by the DPP pattern); lanes without a source add 0
    const int moved = __builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, ROW_MASK, 0xf, false);
    return x + __int_as_float(moved);
}

// Inclusive prefix sum over each row of 16 lanes.
__device__ __forceinline__ float row_inclusive_scan(float x) {
    x = dpp_add<0x111, 0xf>(x);  // row_shr:1
    x = dpp_add<0x112, 0xf>(x);  // row_shr:2
    x = dpp_add<0x114, 0xf>(x);  // row_shr:4
    x = dpp_add<0x118, 0xf>(x);  // row_shr:8
    return x;
}

// Inclusive prefix sum over the 64 lanes, in lane order.
__device__ __forceinline__ float wave_inclusive_scan(float x) {
    x = row_inclusive_scan(x);
    x = dpp_add<0x142, 0xa>(x);  // row_bcast:15 into rows 1 and 3
    x = dpp_add<0x143, 0xc>(x);  // row_bcast:31 into rows 2 and 3
    return x;
}

// Value of lane l-1 (0 in lane 0).
__device__ __forceinline__ float wave_shift_right(float x) {
    return __int_as_float(
        __builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x138 /* wave_shr:1 */, 0xf, 0xf, false));
}

__device__ __forceinline__ float lane63(float x) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 63));
}

// ---- the per-entry steps, written out as instructions --------------------------------
// The compiler does not see the LDS operations below, so every consumer is tied
// to them through register operands and the waits are explicit.

// LDS byte address of the element of v an entry names.  HALF = 0: low 16 bits of d.
template <typename VT, int ENC, int HALF>
__device__ __forceinline__ uint32_t entry_addr(uint32_t d) {
    constexpr bool wide = sizeof(VT) == 4;
    if (ENC == kEncSmall) {  // tail<<15 | idx<<1
        if (!wide) return HALF ? ((d >> 16) & 0x7ffeu) : (d & 0x7ffeu);
        return HALF ? ((d >> 15) & 0xfffcu) : ((d & 0x7ffeu) << 1);
    }
    // idx<<1 | tail
    if (!wide) return HALF ? ((d >> 16) & 0xfffeu) : (d & 0xfffeu);
    return HALF ? ((d >> 15) & 0x1fffcu) : ((d & 0xfffeu) << 1);
}

// Gather one element of v as float bits.  For bf16 the 16 bits land in the high
// half of g, whose low half is zero and stays zero (g is only ever written here).
template <typename VT>
__device__ __forceinline__ void gather(uint32_t &g, uint32_t addr) {
    if (sizeof(VT) == 4)
        asm volatile("ds_read_b32 %0, %1" : "=v"(g) : "v"(addr));
    else
        asm volatile("ds_read_u16_d16_hi %0, %1" : "+v"(g) : "v"(addr));
}

// Wait until at most N of the LDS operations issued so far are outstanding; the
// eight registers are the results the caller is about to read.
template <int N>
__device__ __forceinline__ void lds_wait(uint32_t (&g)[8]) {
    asm volatile("s_waitcnt lgkmcnt(%8)"
                 : "+v"(g[0]), "+v"(g[1]), "+v"(g[2]), "+v"(g[3]), "+v"(g[4]), "+v"(g[5]),
                   "+v"(g[6]), "+v"(g[7])
                 : "n"(N));
}

// If the entry is a tail: E[ptr] = base + s, ptr += 4.  Small encoding: the tail
// flag is the sign of the 16-bit entry (low half: 16-bit compare on d; high
// half: sign of the dword).
template <int ENC, int HALF>
__device__ __forceinline__ void tail_store(uint32_t d, float base, float s, uint32_t &ptr) {
    float t;
    uint64_t saved;
    if (ENC == kEncSmall) {
        if (HALF)
            asm volatile(
                "v_cmp_gt_i32 vcc, 0, %[d]\n\t"
                "s_and_saveexec_b64 %[sv], vcc\n\t"
                "v_add_f32 %[t], %[b], %[s]\n\t"
                "ds_write_b32 %[p], %[t]\n\t"
                "v_add_u32 %[p], 4, %[p]\n\t"
                "s_mov_b64 exec, %[sv]"
                : [p] "+v"(ptr), [t] "=&v"(t), [sv] "=&s"(saved)
                : [d] "v"(d), [b] "v"(base), [s] "v"(s)
                : "vcc", "scc", "memory");
        else
            asm volatile(
                "v_cmp_gt_i16 vcc, 0, %[d]\n\t"
                "s_and_saveexec_b64 %[sv], vcc\n\t"
                "v_add_f32 %[t], %[b], %[s]\n\t"
                "ds_write_b32 %[p], %[t]\n\t"
                "v_add_u32 %[p], 4, %[p]\n\t"
                "s_mov_b64 exec, %[sv]"
                : [p] "+v"(ptr), [t] "=&v"(t), [sv] "=&s"(saved)
                : [d] "v"(d), [b] "v"(base), [s] "v"(s)
                : "vcc", "scc", "memory");
    } else {
        // idx<<1 | tail: bit 0 (low half) or bit 16 (high half)
        asm volatile(
            "v_bfe_i32 %[t], %[d], %[bit], 1\n\t"
            "v_cmp_gt_i32 vcc, 0, %[t]\n\t"
            "s_and_saveexec_b64 %[sv], vcc\n\t"
            "v_add_f32 %[t], %[b], %[s]\n\t"
            "ds_write_b32 %[p], %[t]\n\t"
            "v_add_u32 %[p], 4, %[p]\n\t"
            "s_mov_b64 exec, %[sv]"
            : [p] "+v"(ptr), [t] "=&v"(t), [sv] "=&s"(saved)
            : [d] "v"(d), [b] "v"(base), [s] "v"(s), [bit] "n"(HALF ? 16 : 0)
            : "vcc", "scc", "memory");
    }
}

__device__ __forceinline__ void lds_drain() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

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

template <typename VT>
__device__ __forceinline__ void lds_store_v(int byte_addr, VT x) {
    *reinterpret_cast<__attribute__((address_space(3))) VT *>(static_cast<uintptr_t>(byte_addr)) = x;
}

// One pass (binary, M+, M- or fused) of one block.  FIRST: v still has to be staged into
// LDS and the output rows are overwritten; otherwise the pass adds to them.
template <typename VT, int H, int ENC, bool FIRST>
__device__ __forceinline__ void run_pass(const PassArgs &a, const void *v, long long ldv, int n_in,
                                         int W, const FoldArgs &f, const OutArgs &o) {
    constexpr int PF = 4 / H;  // chunks requested together (16 dwords per lane)
    // LDS (byte addresses): v (n_in + zero slot) | wave-total terms | E[P] | red[k][fold threads]
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
    // fold weights of this thread: one 16-byte row of the table
    const int part = (tid >= f.Tc) + (tid >= 2 * f.Tc) + (tid >= 3 * f.Tc);
    const int cls = tid - part * f.Tc;
    const bool in_stage1 = part < f.parts;
    const uint4 wrow =
        reinterpret_cast<const uint4 *>(f.ftab)[min(in_stage1 ? cls : tid, f.nrows - 1)];
    if (FIRST) {
        // stage v into LDS (16-byte copies when the source allows it); requested
        // before the stream so that it arrives first
        const unsigned char *vg = reinterpret_cast<const unsigned char *>(v) +
                                  (long long)blockIdx.y * ldv * (long long)sizeof(VT);
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
                        tail_store<ENC, 0>(d[h][j], base, s[h][2 * j], ptr);
                        tail_store<ENC, 1>(d[h][j], base, s[h][2 * j + 1], ptr);
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
    lds_drain();
    __syncthreads();
    RSR_STAMP(3);

    // ---- scatter: weighted sum over E ---------------------------------------
    const int nfold = f.nact * 64;                     // threads of the fold waves
    const uint32_t red_at = e_at + (uint32_t)f.P * 4u;  // float [k][nfold]
    if (w < f.nact) {  // only the waves that hold fold threads
        float col = 0.0f;
        if (in_stage1) {
            // digits below m: the class c mod Tc decides the weight
            const int i0 = part == 0 ? f.ib[0] : part == 1 ? f.ib[1] : part == 2 ? f.ib[2] : f.ib[3];
            const int i1 = part == 0 ? f.ib[1] : part == 1 ? f.ib[2] : part == 2 ? f.ib[3] : f.ib[4];
            const uint32_t step = (uint32_t)f.Tc * 4u;
            uint32_t at = e_at + (uint32_t)cls * 4u + step * (uint32_t)i0;
            const uint32_t last = e_at + (uint32_t)cls * 4u + step * (uint32_t)(i1 - 1);
            float c0s = 0.0f, c1s = 0.0f;
            for (int i = i0; i < i1; i += 8) {
                float x[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    x[u] = *lds_float(min(at, last));  // reads past the share repeat its last entry
                    at += step;
                }
#pragma unroll
                for (int u = 0; u < 8; u += 2) {
                    if (i + u < i1) c0s += x[u];
                    if (i + u + 1 < i1) c1s += x[u + 1];
                }
            }
            col = c0s + c1s;
        }
        // digits m..k-1 change only between c = Tc*i + Tc-1 and c+1
        float gq = 0.0f;
        if (tid < f.Q) gq = *lds_float(e_at + (uint32_t)(f.Tc * tid + f.Tc - 1) * 4u);
        const uint32_t ww[4] = {wrow.x, wrow.y, wrow.z, wrow.w};
        float acc[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            if (r < f.k) {
                const float wt = (float)(int)(signed char)((ww[r >> 2] >> (8 * (r & 3))) & 0xffu);
                acc[r] = wt * (r < f.m ? col : gq);
            }
        }
        for (int i = tid + nthreads; i < f.Q; i += nthreads) {  // only when Q > threads
            const uint4 xr = reinterpret_cast<const uint4 *>(f.ftab)[i];
            const uint32_t xw[4] = {xr.x, xr.y, xr.z, xr.w};
            const float gx = *lds_float(e_at + (uint32_t)(f.Tc * i + f.Tc - 1) * 4u);
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (r >= f.m && r < f.k)
                    acc[r] += (float)(int)(signed char)((xw[r >> 2] >> (8 * (r & 3))) & 0xffu) * gx;
        }
        RSR_STAMP(4);
        // every fold thread leaves its term of every row in LDS: red[r][tid]
        uint32_t rp = red_at + (uint32_t)tid * 4u;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            if (r < f.k) {
                *lds_float(rp) = acc[r];
                rp += (uint32_t)nfold * 4u;
            }
        }
    }
    RSR_STAMP(5);
    __syncthreads();
    RSR_STAMP(6);
    // wave w sums rows w, w+W, ...: lane j takes red[r][j], red[r][j+64], ... and, for
    // j < W, the wave-total term of wave j; one scan over the wave finishes the row
#pragma unroll
    for (int rr = 0; rr < 16; ++rr) {
        const int r = w + rr * W;
        if (r < f.k) {
            const uint32_t at = red_at + (uint32_t)(r * nfold + lane) * 4u;
            float x0 = 0.0f, x1 = 0.0f;
            for (int i = 0; i < f.nact; i += 2) {
                x0 += *lds_float(at + (uint32_t)i * 256u);
                if (i + 1 < f.nact) x1 += *lds_float(at + (uint32_t)(i + 1) * 256u);
            }
            if (lane < W) x0 += *lds_float(corr_at + (lane * 16 + r) * 4);
            const float tot = wave_inclusive_scan(x0 + x1);
            if (lane == 63) {
                const long long row = b * f.k + r;
                if (row < o.n_out) {
                    float *dst = o.out + (long long)blockIdx.y * o.ldo + row;
                    const float term = o.scale * a.sign * tot;
                    *dst = FIRST ? term : *dst + term;  // pass 2 adds to what pass 1 wrote
                }
            }
        }
    }
}

template <typename VT, int H, int ENC, int NPASS>
__global__ __launch_bounds__(1024) void k_rsr_matvec(const PassArgs a0, const void *v,
                                                     long long ldv, int n_in, int W,
                                                     const FoldArgs f, const PassArgs a1,
                                                     const OutArgs o) {
    RSR_STAMP(0);
    run_pass<VT, H, ENC, true>(a0, v, ldv, n_in, W, f, o);
    if (NPASS == 2) {
        __syncthreads();
        run_pass<VT, H, ENC, false>(a1, v, ldv, n_in, W, f, o);
    }
    RSR_STAMP(7);
}

struct LaunchArgs {
    PassArgs a0, a1;
    const void *v;
    long long ldv;
    int n_in, W, npass, nblocks, batch;
    FoldArgs f;
    OutArgs o;
    size_t lds;
    hipStream_t stream;
};

template <typename VT, int H, int ENC, int NPASS>
hipError_t launch(const LaunchArgs &x) {
    static size_t attr_bytes = 0;  // largest dynamic LDS size enabled for this kernel so far
    auto kern = k_rsr_matvec<VT, H, ENC, NPASS>;
    if (x.lds > attr_bytes) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)x.lds);
        if (e != hipSuccess) return e;
        attr_bytes = x.lds;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)x.nblocks, (unsigned)x.batch), dim3(x.W * 64), x.lds,
                       x.stream, x.a0, x.v, x.ldv, x.n_in, x.W, x.f, x.a1, x.o);
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

// tab[t][r], r < m : sgn_r(t) - sgn_r((t+1) mod Tc) for t < Tc   (weight of class t)
// tab[t][r], m <= r < k : sgn_{r-m}(t) - sgn_{r-m}(t+1) for t < Q  (weight of E[Tc*t + Tc-1])
template <int BASE>
__global__ void k_fold_table(int k, int m, int Tc, int Q, int nrows, int8_t *__restrict__ tab) {
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= nrows) return;
    for (int r = 0; r < 16; ++r) {
        int wgt = 0;
        if (r < m) {
            if (t < Tc) wgt = sgn_digit<BASE>(t, r) - sgn_digit<BASE>((t + 1 == Tc) ? 0 : t + 1, r);
        } else if (r < k) {
            if (t < Q) wgt = sgn_digit<BASE>(t, r - m) - sgn_digit<BASE>(t + 1, r - m);
        }
        tab[t * 16 + r] = (int8_t)wgt;
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

void choose_launch_shape(int64_t longest, int *H, int *W) {
    // Two workgroups of up to 8 waves share a CU without register pressure; each wave
    // should own at most two chunks, so the chunk grows with the stream (H = 1, 2, 4).
    constexpr int kWaves = 8;
    int h = 4;
    for (int cand = 1; cand <= 4; cand *= 2)
        if ((longest + kLoad * cand - 1) / (kLoad * cand) <= 2 * kWaves) { h = cand; break; }
    if (const char *s = std::getenv("RSR_H")) {
        const int x = std::atoi(s);
        if (x == 1 || x == 2 || x == 4) h = x;
    }
    const int64_t chunks = (longest + kLoad * h - 1) / (kLoad * h);
    int w = (int)(chunks < 1 ? 1 : chunks > kWaves ? kWaves : chunks);
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
        if (parts > 4) parts = 4;
        if (parts > fs->Q) parts = fs->Q;
        if (parts < 1) parts = 1;
    }
    fs->parts = parts;
    for (int j = 0; j <= 4; ++j)
        fs->ib[j] = (j <= parts) ? (int)((long long)j * fs->Q / parts) : fs->Q;
    const int span1 = fs->Tc * parts;
    const int span2 = fs->Q < threads ? fs->Q : threads;
    fs->nact = ((span1 > span2 ? span1 : span2) + 63) / 64;
    fs->nrows = fs->Tc > fs->Q ? fs->Tc : fs->Q;
    for (int ps = 0; ps < 2; ++ps)
        for (int w = 0; w <= kMaxWaves; ++w)
            fs->cb[ps][w] = (unsigned short)((ps < npass && w <= W)
                                                 ? w * (C[ps] / W) + (w < C[ps] % W ? w : C[ps] % W)
                                                 : 0);
}

hipError_t launch_fold_tables(int base, int k, const FoldShape &fs, int8_t *ftab) {
    const int threads = 256, groups = (fs.nrows + threads - 1) / threads;
    if (base == 2)
        hipLaunchKernelGGL(k_fold_table<2>, dim3(groups), dim3(threads), 0, 0, k, fs.m, fs.Tc, fs.Q,
                           fs.nrows, ftab);
    else
        hipLaunchKernelGGL(k_fold_table<3>, dim3(groups), dim3(threads), 0, 0, k, fs.m, fs.Tc, fs.Q,
                           fs.nrows, ftab);
    return hipGetLastError();
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
    x.batch = batch;
    x.f.ftab = h->ftab;
    for (int j = 0; j < 5; ++j) x.f.ib[j] = fs.ib[j];
    x.f.k = h->k;
    x.f.P = (int)h->P;
    x.f.m = fs.m;
    x.f.Tc = fs.Tc;
    x.f.Q = fs.Q;
    x.f.parts = fs.parts;
    x.f.nact = fs.nact;
    x.f.nrows = fs.nrows;
    x.o.out = out;
    x.o.ldo = ldo;
    x.o.n_out = (int)h->rows;
    x.o.scale = scale;
    x.o.stamps = nullptr;
#ifdef RSR_PHASE_TIMING
    if (const char *sp = std::getenv("RSR_STAMPS"))
        x.o.stamps = reinterpret_cast<long long *>(std::strtoull(sp, nullptr, 0));
#endif
    x.lds = (size_t)matvec_lds_bytes(h->P, h->cols, (v_dtype == RSR_BF16) ? 2 : 4, h->k, fs.nact);
    x.stream = stream;
    return (v_dtype == RSR_BF16) ? launch_he<uint16_t>(x, h->H, h->enc)
                                 : launch_he<float>(x, h->H, h->enc);
}

const char *rsr_matvec_kernel_name(int v_dtype, int H, int enc, int npass) {
    // one static string per instantiation, as a profiler prints the template arguments
    static char names[2][3][2][2][48];
    const int hi = (H == 1) ? 0 : (H == 2) ? 1 : 2;
    char *n = names[v_dtype == RSR_BF16][hi][enc == kEncBig][npass == 2];
    if (!n[0])
        std::snprintf(n, sizeof(names[0][0][0][0]), "k_rsr_matvec<%s, %d, %d, %d>",
                      v_dtype == RSR_BF16 ? "unsigned short" : "float", H, enc, npass);
    return n;
}

}  // namespace rsr
