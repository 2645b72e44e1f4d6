// RSR multiply kernel for gfx950 (paper, System Overview: aggregate the entries
// of v of each group of identical column patterns, then distribute every group
// sum once; Kernels Implementation: gather, aggregate and scatter phases).
//
// One workgroup of W waves handles one block of k output rows:
//   gather     the block's stream of 16-bit column entries is read with one
//              coalesced 16-byte load per lane (8 consecutive entries); v sits
//              in LDS and is gathered through the entries
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
//              the next, and so on (1.5 P or 2 P terms in total).
// Prefixes are local to a wave; the waves' totals are folded in afterwards with
// the same weights (the weighted sum is linear in E).
#include "rsr_internal.h"

namespace rsr {

namespace {

struct MatvecParams {
    const uint16_t *stream[2];
    const uint32_t *hdr[2];
    long long S[2];
    float sign[2];
    int npass, n_in, n_out, k, P, W;
    int m, Tc, Q;  // fold split: Tc = base^m column classes, Q = P / Tc
    const void *v;
    long long ldv;
    float *out;
    long long ldo;
    float scale;
};

template <typename VT>
__device__ __forceinline__ float widen(VT x);
template <>
__device__ __forceinline__ float widen<float>(float x) { return x; }
template <>
__device__ __forceinline__ float widen<uint16_t>(uint16_t x) {
    return __uint_as_float((uint32_t)x << 16);  // bf16 -> f32 is exact
}

// Contribution sign of a digit: binary {0,1}; ternary digit 1 -> +1, 2 -> -1.
template <int BASE>
__device__ __forceinline__ float sgn(uint32_t d) {
    if (BASE == 2) return (float)d;
    return (d == 1u) ? 1.0f : (d == 2u) ? -1.0f : 0.0f;
}

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) x += __shfl_xor(x, d, 64);
    return x;
}

template <typename VT, int BASE>
__global__ __launch_bounds__(1024) void k_rsr_matvec(const MatvecParams p) {
    extern __shared__ __align__(16) unsigned char smem[];
    // LDS: v (n_in + zero slot) | wave totals | partial outputs | wave codes | E[P]
    const int vbytes = ((p.n_in + 1) * (int)sizeof(VT) + 15) & ~15;
    VT *vbuf = reinterpret_cast<VT *>(smem);
    float *wtot = reinterpret_cast<float *>(smem + vbytes);  // [16]
    float *part = wtot + 16;                                 // [16][16]
    uint32_t *cs = reinterpret_cast<uint32_t *>(part + 256); // [17]
    float *E = reinterpret_cast<float *>(smem + vbytes + kLdsMisc);

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int nthreads = blockDim.x;
    const long long b = blockIdx.x;
    const VT *vg = reinterpret_cast<const VT *>(p.v) + (long long)blockIdx.y * p.ldv;

    for (int j = tid; j < p.n_in; j += nthreads) vbuf[j] = vg[j];
    if (tid == 0) vbuf[p.n_in] = VT(0);

    float final_r = 0.0f;  // thread r < k accumulates output row b*k + r

    for (int pass = 0; pass < p.npass; ++pass) {
        const long long S = p.S[pass];
        const int share = (int)(S / p.W);
        const int n_iter = share / kChunk;
        const uint16_t *sp = p.stream[pass] + b * S + (long long)w * share;
        const uint32_t *hb = p.hdr[pass] + b * p.W;
        if (tid == 0) { E[0] = 0.0f; cs[p.W] = (uint32_t)p.P; }
        if (tid < p.W) cs[tid] = hb[tid];
        float run_sum = 0.0f;
        uint32_t run_code = hb[w];
        __syncthreads();

        // ---- gather + aggregate ------------------------------------------------
        for (int it = 0; it < n_iter; ++it) {
            const uint4 q = *reinterpret_cast<const uint4 *>(sp + it * kChunk + lane * 8);
            const uint32_t ew[4] = {q.x, q.y, q.z, q.w};
            float s[8];
            uint32_t tl[8];
            uint32_t ntails = 0;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const uint32_t e = (ew[i >> 1] >> ((i & 1) * 16)) & 0xffffu;
                const float g = widen<VT>(vbuf[e >> 1]);
                s[i] = i ? s[i - 1] + g : g;
                tl[i] = e & 1u;
                ntails += tl[i];
            }
            // exclusive scans over the lanes of (strip total, tail count)
            float incl_s = s[7];
            uint32_t incl_c = ntails;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const float ys = __shfl_up(incl_s, d, 64);
                const uint32_t yc = __shfl_up(incl_c, d, 64);
                if (lane >= d) { incl_s += ys; incl_c += yc; }
            }
            float excl_s = __shfl_up(incl_s, 1, 64);
            if (lane == 0) excl_s = 0.0f;
            const float base = run_sum + excl_s;
            uint32_t code = run_code + incl_c - ntails;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                if (tl[i]) { E[code] = base + s[i]; code += 1; }
            }
            run_sum += __shfl(incl_s, 63, 64);
            run_code += __shfl(incl_c, 63, 64);
        }
        if (lane == 0) wtot[w] = run_sum;
        __syncthreads();

        // ---- scatter: weighted sum over E ---------------------------------------
        float acc[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
        if (tid < p.Tc) {
            // digits below m: class t = c mod Tc decides the weight
            float col = 0.0f;
            for (int i = 0; i < p.Q; ++i) col += E[tid + p.Tc * i];
            uint32_t qa = tid, qb = (tid + 1 == p.Tc) ? 0 : tid + 1;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                if (r < p.m) {
                    const uint32_t da = qa % BASE, db = qb % BASE;
                    qa /= BASE; qb /= BASE;
                    acc[r] += (sgn<BASE>(da) - sgn<BASE>(db)) * col;
                }
            }
        }
        for (int i = tid; i < p.Q; i += nthreads) {
            // digits m..k-1 change only between c = Tc*i + Tc-1 and c+1
            const float g = E[p.Tc * i + p.Tc - 1];
            uint32_t qa = i, qb = i + 1;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                if (r >= p.m && r < p.k) {
                    const uint32_t da = qa % BASE, db = qb % BASE;
                    qa /= BASE; qb /= BASE;
                    acc[r] += (sgn<BASE>(da) - sgn<BASE>(db)) * g;
                }
            }
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            if (r < p.k) {
                const float t = wave_sum(acc[r]);
                if (lane == 0) part[w * 16 + r] = t;
            }
        }
        __syncthreads();
        if (tid < p.k) {
            const int r = tid;
            uint32_t pw = 1;
            for (int i = 0; i < r; ++i) pw *= BASE;
            float tot = 0.0f, wbase = 0.0f;
            for (int ww = 0; ww < p.W; ++ww) {
                tot += part[ww * 16 + r];
                // codes whose tail lies in wave ww are [cs[ww], cs[ww+1]); their
                // stored prefixes all miss the totals of the waves before ww
                const uint32_t d0 = (cs[ww] / pw) % BASE, d1 = (cs[ww + 1] / pw) % BASE;
                tot += wbase * (sgn<BASE>(d0) - sgn<BASE>(d1));
                wbase += wtot[ww];
            }
            final_r += p.sign[pass] * tot;
        }
        if (pass + 1 < p.npass) __syncthreads();
    }
    if (tid < p.k) {
        const long long row = b * p.k + tid;
        if (row < p.n_out) p.out[(long long)blockIdx.y * p.ldo + row] = p.scale * final_r;
    }
}

template <typename VT, int BASE>
hipError_t launch(const MatvecParams &p, int batch, size_t lds, hipStream_t stream) {
    static size_t attr_bytes = 0;  // largest dynamic LDS size enabled for this kernel so far
    auto kern = k_rsr_matvec<VT, BASE>;
    if (lds > attr_bytes) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_bytes = lds;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)(p.n_out + p.k - 1) / p.k, (unsigned)batch),
                       dim3(p.W * 64), lds, stream, p);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_rsr_matvec(const rsr_handle_s *h, const void *v, int v_dtype, float scale,
                             float *out, int batch, int64_t ldv, int64_t ldo, hipStream_t stream) {
    MatvecParams p;
    for (int i = 0; i < 2; ++i) {
        p.stream[i] = h->pass[i].stream;
        p.hdr[i] = h->pass[i].hdr;
        p.S[i] = h->pass[i].S;
        p.sign[i] = h->pass[i].sign;
    }
    p.npass = h->npass;
    p.n_in = (int)h->cols;
    p.n_out = (int)h->rows;
    p.k = h->k;
    p.P = (int)h->P;
    p.W = h->W;
    // fold split: the largest power of the base that fits the workgroup
    int m = 0;
    long long Tc = 1;
    while (m < h->k && Tc * h->base <= (long long)h->W * 64) { Tc *= h->base; ++m; }
    p.m = m;
    p.Tc = (int)Tc;
    p.Q = (int)(h->P / Tc);
    p.v = v;
    p.ldv = ldv;
    p.out = out;
    p.ldo = ldo;
    p.scale = scale;
    const int vb = (v_dtype == RSR_BF16) ? 2 : 4;
    const size_t lds = (size_t)matvec_lds_bytes(h->P, h->cols, vb);
    if (h->base == 2)
        return (v_dtype == RSR_BF16) ? launch<uint16_t, 2>(p, batch, lds, stream)
                                     : launch<float, 2>(p, batch, lds, stream);
    return (v_dtype == RSR_BF16) ? launch<uint16_t, 3>(p, batch, lds, stream)
                                 : launch<float, 3>(p, batch, lds, stream);
}

const char *rsr_matvec_kernel_name(int base, int v_dtype) {
    if (base == 2) return v_dtype == RSR_BF16 ? "k_rsr_matvec<unsigned short, 2>" : "k_rsr_matvec<float, 2>";
    return v_dtype == RSR_BF16 ? "k_rsr_matvec<unsigned short, 3>" : "k_rsr_matvec<float, 3>";
}

}  // namespace rsr
