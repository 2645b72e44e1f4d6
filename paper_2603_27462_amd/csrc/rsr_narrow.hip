// RSR multiply for narrow matrices (cols <= 256; paper, Kernels Implementation: metadata
// shrunk to compact types to cut bandwidth in the inference hot path): one wave per block
// of k rows, 8-bit column indices, one tail bit per entry, one sign word per non-empty
// group, nothing for empty groups.  With at most 256 entries per block the workgroup-wide
// machinery of the wide kernel (barriers, start slots, strip signs, two-level weighted
// sum) would cost more than the block itself; here a block is four entries per lane:
//   gather     lane l owns entries 4l..4l+3 of the block's stream (one dword), gathers
//              the four elements of v from LDS
//   aggregate  running sums inside the lane, one DPP scan over the wave for the true
//              prefix; the lane's tails store their prefix into E[rank] (rank from a DPP
//              scan of the lanes' tail counts), E private to the wave in LDS
//   scatter    u[g] = E[g] - E[g-1] is the sum of group g; lane l takes groups 4l..4l+3,
//              multiplies each by the sign of every row (fields of the group's sign word)
//              and the k sums are reduced over the wave
// No barrier after v is staged: the waves of a workgroup work through their blocks on
// their own.
#include "rsr_device.h"
#include "rsr_internal.h"

namespace rsr {
namespace {

constexpr int kNarrowWaves = 4;       // waves (blocks in flight) per workgroup
constexpr int kNarrowThreads = kNarrowWaves * 64;
constexpr int kNarrowTurns = 4;       // blocks a wave handles one after the other
constexpr int kNarrowRows = 16;

struct NarrowPass {
    const uint32_t *ent;   // [nb][64]: entries 4l..4l+3 of the block, one byte each
    const uint8_t *meta;   // [nb][64]: bits 0-3 tail flags, bits 4-7 valid flags of those entries
    const void *sw;        // [nb][gs]: sign word of every group in rank order (fw bits per row)
    float sign;
};

// Sign words of the lane's four groups, whatever the word size.
__device__ __forceinline__ void load_sign_words(const void *sw, long long index, int bytes,
                                                uint32_t (&w)[4]) {
    if (bytes == 1) {
        const uint32_t x = *reinterpret_cast<const uint32_t *>(static_cast<const uint8_t *>(sw) + index);
        w[0] = x & 0xffu; w[1] = (x >> 8) & 0xffu; w[2] = (x >> 16) & 0xffu; w[3] = x >> 24;
    } else if (bytes == 2) {
        const uint2 x = *reinterpret_cast<const uint2 *>(static_cast<const uint16_t *>(sw) + index);
        w[0] = x.x & 0xffffu; w[1] = x.x >> 16; w[2] = x.y & 0xffffu; w[3] = x.y >> 16;
    } else {
        const uint4 x = *reinterpret_cast<const uint4 *>(static_cast<const uint32_t *>(sw) + index);
        w[0] = x.x; w[1] = x.y; w[2] = x.z; w[3] = x.w;
    }
}

__device__ __forceinline__ uint32_t wave_inclusive_scan_u32(uint32_t x) {
    // integer twin of wave_inclusive_scan (DPP row shifts, then the two row broadcasts)
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x111, 0xf, 0xf, false);
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x112, 0xf, 0xf, false);
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x114, 0xf, 0xf, false);
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x118, 0xf, 0xf, false);
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x142, 0xa, 0xf, false);
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x143, 0xc, 0xf, false);
    return x;
}

__device__ __forceinline__ float wave_shift_right1(float x) {  // value of lane l-1, 0 in lane 0
    return __int_as_float(
        __builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x138 /* wave_shr:1 */, 0xf, 0xf, false));
}

template <typename VT>
__global__ __launch_bounds__(kNarrowThreads) void k_rsr_narrow(
    const NarrowPass p0, const NarrowPass p1, int npass, const void *__restrict__ v, long long ldv,
    int n_in, long long nb, int k, int fw, int sw_bytes, long long gs, float *__restrict__ out,
    long long ldo, long long n_out, float scale) {
    // LDS: v as float [256] | E[waves][256]
    __shared__ float vl[256];
    __shared__ __attribute__((aligned(16))) float El[kNarrowWaves][256];
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = tid >> 6;
    const int vec = blockIdx.y;
    const VT *vg = static_cast<const VT *>(v) + (long long)vec * ldv;
    if (tid < n_in) {
        if (sizeof(VT) == 4)
            vl[tid] = reinterpret_cast<const float *>(vg)[tid];
        else
            vl[tid] = __uint_as_float((uint32_t) reinterpret_cast<const uint16_t *>(vg)[tid] << 16);
    } else {
        vl[tid] = 0.0f;
    }
    __syncthreads();
    float *E = El[w];
    const long long wave0 = ((long long)blockIdx.x * kNarrowWaves + w) * kNarrowTurns;
    for (int turn = 0; turn < kNarrowTurns; ++turn) {
        const long long b = wave0 + turn;
        if (b >= nb) break;
        float acc[kNarrowRows];
#pragma unroll
        for (int r = 0; r < kNarrowRows; ++r) acc[r] = 0.0f;
        for (int ps = 0; ps < npass; ++ps) {
            const NarrowPass &p = ps ? p1 : p0;
            const uint32_t d = __builtin_nontemporal_load(&p.ent[b * 64 + lane]);
            const uint32_t meta = __builtin_nontemporal_load(&p.meta[b * 64 + lane]);
            uint32_t sw[4] = {0u, 0u, 0u, 0u};
            if (4 * lane < gs) load_sign_words(p.sw, b * gs + 4 * lane, sw_bytes, sw);
            // gather + running sums (entries past the end of the block count as zero)
            float g0 = vl[d & 0xffu], g1 = vl[(d >> 8) & 0xffu], g2 = vl[(d >> 16) & 0xffu], g3 = vl[d >> 24];
            g0 = (meta & 0x10u) ? g0 : 0.0f;
            g1 = (meta & 0x20u) ? g1 : 0.0f;
            g2 = (meta & 0x40u) ? g2 : 0.0f;
            g3 = (meta & 0x80u) ? g3 : 0.0f;
            const float s0 = g0, s1 = s0 + g1, s2 = s1 + g2, s3 = s2 + g3;
            const float incl = wave_inclusive_scan(s3);
            const float base = wave_shift_right1(incl);
            // ranks of the lane's tails: tails before the lane, then tails before the entry
            const uint32_t t0 = meta & 1u, t1 = (meta >> 1) & 1u, t2 = (meta >> 2) & 1u, t3 = (meta >> 3) & 1u;
            const uint32_t cnt = t0 + t1 + t2 + t3;
            const uint32_t rbase = wave_inclusive_scan_u32(cnt) - cnt;
            // E[rank] = prefix through the group; slots that no group owns stay zero
            reinterpret_cast<float4 *>(E)[lane] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            if (t0) E[rbase] = base + s0;
            if (t1) E[rbase + t0] = base + s1;
            if (t2) E[rbase + t0 + t1] = base + s2;
            if (t3) E[rbase + t0 + t1 + t2] = base + s3;
            // (the wave's LDS operations execute in order: no barrier inside a wave)
            const float4 e = reinterpret_cast<const float4 *>(E)[lane];
            // group sums of ranks 4l..4l+3; ranks past the last group have sign word 0 and an
            // E of zero, so whatever their difference is it is multiplied by zero
            const float before = wave_shift_right1(e.w);
            const float u0 = e.x - before, u1 = e.y - e.x, u2 = e.z - e.y, u3 = e.w - e.z;
            const float sg = p.sign;
#pragma unroll
            for (int r = 0; r < kNarrowRows; ++r)
                if (r < k) {
                    float x = u0 * field_as_float(sw[0], fw * r, fw);
                    x += u1 * field_as_float(sw[1], fw * r, fw);
                    x += u2 * field_as_float(sw[2], fw * r, fw);
                    x += u3 * field_as_float(sw[3], fw * r, fw);
                    acc[r] += sg * x;
                }
        }
        // one-bit fields read as 0 / -1: binary kinds come out negated
        const float fix = (fw == 1) ? -scale : scale;
        float *out_rows = out + (long long)vec * ldo + b * k;
        const long long rows_left = n_out - b * k;
#pragma unroll
        for (int r = 0; r < kNarrowRows; ++r)
            if (r < k) {
                const float tot = wave_inclusive_scan(acc[r]);
                if (lane == 63 && r < rows_left) __builtin_nontemporal_store(fix * tot, &out_rows[r]);
            }
    }
}

// ---- preprocessing ------------------------------------------------------------------------
constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;

__device__ __forceinline__ uint32_t wave_scan_u32_shfl(uint32_t x) {
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        uint32_t y = __shfl_up(x, d, 64);
        if (lane >= d) x += y;
    }
    return x;
}

__device__ __forceinline__ uint32_t wg_exclusive_scan(uint32_t x, uint32_t *wsum, uint32_t *total) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const uint32_t incl = wave_scan_u32_shfl(x);
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

// Sign word of code c: field r (fw bits) = sign of digit r; fw = 1: the binary digit itself,
// fw = 2: two's complement (00: 0, 01: +1, 11: -1).
__device__ __forceinline__ uint32_t sign_word(uint32_t c, int k, int base, int fw) {
    uint32_t word = 0;
    for (int r = 0; r < k; ++r) {
        const uint32_t d = c % (uint32_t)base;
        c /= (uint32_t)base;
        const uint32_t f = (fw == 1) ? d : (d == 0 ? 0u : d == 1 ? 1u : 3u);
        word |= f << (fw * r);
    }
    return word;
}

// The narrow stream of every block from the canonical pi / off: entries in code order
// (group 0 left out, empty groups contribute nothing), four per lane; tail and valid flags;
// the sign word of every non-empty group in rank order, zeros behind the last one.
__global__ __launch_bounds__(kThreads) void k_pack_narrow(
    const uint16_t *__restrict__ pi, const uint32_t *__restrict__ off, int64_t nb, int n, int64_t P,
    int k, int base, int fw, int sw_bytes, int64_t gs, uint32_t *__restrict__ ent,
    uint8_t *__restrict__ meta, void *__restrict__ sw, int *__restrict__ err_flag) {
    __shared__ uint32_t wsum[kWaves];
    __shared__ uint8_t e8[256], tl[256];
    __shared__ uint32_t swl[256];
    const int tid = threadIdx.x;
    for (int64_t b = blockIdx.x; b < nb; b += gridDim.x) {
        const uint16_t *pib = pi + b * n;
        const uint32_t *ob = off + b * (P + 1);
        const uint32_t off1 = ob[1];
        const uint32_t len = (uint32_t)n - off1;
        e8[tid] = 0;
        tl[tid] = 0;
        swl[tid] = 0;
        __syncthreads();
        uint32_t carry = 0;  // empty groups among the codes before the current batch
        for (int64_t c0 = 1; c0 < P; c0 += kThreads) {
            const int64_t c = c0 + tid;
            const bool valid = c < P;
            const uint32_t s = valid ? ob[c] : 0, e = valid ? ob[c + 1] : 0;
            const uint32_t empty = (valid && s == e) ? 1u : 0u;
            uint32_t total;
            const uint32_t eb = carry + wg_exclusive_scan(empty, wsum, &total);
            if (valid && !empty) {
                for (uint32_t t = s; t < e; ++t) e8[t - off1] = (uint8_t)pib[t];
                tl[e - 1 - off1] = 1;
                swl[c - eb - 1] = sign_word((uint32_t)c, k, base, fw);  // rank c - eb, 1-based
            }
            carry += total;
        }
        __syncthreads();
        const int64_t groups = P - 1 - carry;
        if (tid == 0 && (groups > gs || len > 256)) atomicOr(err_flag, 2);
        if (tid < 64) {
            uint32_t d = 0, m = 0;
            for (int i = 0; i < 4; ++i) {
                const uint32_t t = 4 * tid + i;
                d |= (uint32_t)e8[t] << (8 * i);
                m |= (uint32_t)tl[t] << i;
                if (t < len) m |= 16u << i;
            }
            ent[b * 64 + tid] = d;
            meta[b * 64 + tid] = (uint8_t)m;
        }
        for (int64_t g = tid; g < gs; g += kThreads) {
            const uint32_t x = g < 256 ? swl[g] : 0u;
            if (sw_bytes == 1)
                static_cast<uint8_t *>(sw)[b * gs + g] = (uint8_t)x;
            else if (sw_bytes == 2)
                static_cast<uint16_t *>(sw)[b * gs + g] = (uint16_t)x;
            else
                static_cast<uint32_t *>(sw)[b * gs + g] = x;
        }
        __syncthreads();
    }
}

}  // namespace

hipError_t launch_pack_narrow(const rsr_handle_s *h, int pass, int *err_flag) {
    const PassData &pd = h->pass[pass];
    const int64_t nb = h->nb;
    hipLaunchKernelGGL(k_pack_narrow, dim3((unsigned)(nb < 8192 ? nb : 8192)), dim3(kThreads), 0, 0, pd.pi,
                       pd.off, nb, (int)h->cols, h->P, h->k, h->base, h->narrow_fw, h->narrow_sw_bytes,
                       h->slots, pd.nent, pd.nmeta, pd.nsw, err_flag);
    return hipGetLastError();
}

hipError_t launch_narrow_matvec(const rsr_handle_s *h, const void *v, int v_dtype, float scale, float *out,
                                int batch, int64_t ldv, int64_t ldo, hipStream_t stream) {
    NarrowPass p[2];
    for (int i = 0; i < 2; ++i) {
        const PassData &pd = h->pass[i < h->npass ? i : 0];
        p[i].ent = pd.nent;
        p[i].meta = pd.nmeta;
        p[i].sw = pd.nsw;
        p[i].sign = pd.sign;
    }
    const long long per_wg = (long long)kNarrowWaves * kNarrowTurns;
    const dim3 grid((unsigned)((h->nb + per_wg - 1) / per_wg), (unsigned)batch);
    if (v_dtype == RSR_BF16)
        hipLaunchKernelGGL(k_rsr_narrow<uint16_t>, grid, dim3(kNarrowThreads), 0, stream, p[0], p[1], h->npass, v,
                           (long long)ldv, (int)h->cols, (long long)h->nb, h->k, h->narrow_fw,
                           h->narrow_sw_bytes, (long long)h->slots, out, (long long)ldo, (long long)h->rows,
                           scale);
    else
        hipLaunchKernelGGL(k_rsr_narrow<float>, grid, dim3(kNarrowThreads), 0, stream, p[0], p[1], h->npass, v,
                           (long long)ldv, (int)h->cols, (long long)h->nb, h->k, h->narrow_fw,
                           h->narrow_sw_bytes, (long long)h->slots, out, (long long)ldo, (long long)h->rows,
                           scale);
    return hipGetLastError();
}

}  // namespace rsr
