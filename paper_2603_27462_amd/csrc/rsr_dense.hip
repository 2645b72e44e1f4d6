// Dense 2-bit packed ternary matvec: the on-GPU comparison point for the RSR
// kernel (the role the paper gives its low-bit "BitNet" multiplier baseline in
// Benchmarking Results).  No preprocessing beyond packing; every matrix entry
// is decoded and multiplied.
//
// Kernel layout (tiled so that both the weight loads and the LDS reads of v
// are contiguous across a wave): rows are taken in groups of 4, columns in
// tiles of 1024.  For group G, tile t, lane l, one uint4 holds the dwords of
// rows 4G..4G+3; bit field f (2 bits, two's complement: 00 = 0, 01 = +1,
// 11 = -1) of each dword is column t*1024 + 256*(f/4) + 4*l + f%4.
#include "rsr_internal.h"

namespace rsr {

namespace {

constexpr int kTile = 1024;

__global__ __launch_bounds__(256) void k_pack2_tiled(const int8_t *__restrict__ M, int64_t rows,
                                                     int64_t cols, int ntiles,
                                                     uint32_t *__restrict__ tiled,
                                                     int *__restrict__ err_flag) {
    const int64_t ngroups = (rows + 3) / 4;
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (gid >= ngroups * ntiles * 256) return;
    const int rr = (int)(gid & 3);
    const int lane = (int)((gid >> 2) & 63);
    const int64_t gt = gid >> 8;
    const int64_t G = gt / ntiles, t = gt % ntiles;
    const int64_t i = G * 4 + rr;
    uint32_t word = 0;
    bool bad = false;
    if (i < rows) {
        for (int f = 0; f < 16; ++f) {
            const int64_t j = t * kTile + 256 * (f >> 2) + 4 * lane + (f & 3);
            if (j < cols) {
                const int m = M[i * cols + j];
                if (m < -1 || m > 1) bad = true;
                word |= ((uint32_t)m & 3u) << (2 * f);
            }
        }
    }
    if (bad) atomicOr(err_flag, 1);
    tiled[gid] = word;
}

template <typename VT>
__device__ __forceinline__ float widen(VT x);
template <>
__device__ __forceinline__ float widen<float>(float x) { return x; }
template <>
__device__ __forceinline__ float widen<uint16_t>(uint16_t x) {
    return __uint_as_float((uint32_t)x << 16);
}

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) x += __shfl_xor(x, d, 64);
    return x;
}

// sign-extended 2-bit field f of w, as float (-1, 0 or +1)
__device__ __forceinline__ float field(uint32_t w, int f) {
    return (float)(((int)(w << (30 - 2 * f))) >> 30);
}

// Workgroup = 4 waves = 2 row groups x 2 halves of the tile range.
template <typename VT>
__global__ __launch_bounds__(256) void k_dense_matvec(const uint4 *__restrict__ tiled, int ntiles,
                                                      int n_in, int n_out, int ngroups,
                                                      const void *__restrict__ v, long long ldv,
                                                      float *__restrict__ out, long long ldo,
                                                      float scale) {
    extern __shared__ __align__(16) unsigned char smem[];
    float *vf = reinterpret_cast<float *>(smem);       // [ntiles*1024], zero padded
    float *red = vf + ntiles * kTile;                  // [4 waves][4 rows]
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const VT *vg = reinterpret_cast<const VT *>(v) + (long long)blockIdx.y * ldv;
    for (int j = tid; j < ntiles * kTile; j += 256) vf[j] = (j < n_in) ? widen<VT>(vg[j]) : 0.0f;
    __syncthreads();

    const int rgl = w & 1, half = w >> 1;
    const int G = blockIdx.x * 2 + rgl;
    const int tmid = (ntiles + 1) / 2;
    const int t0 = half ? tmid : 0, t1 = half ? ntiles : tmid;
    float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    if (G < ngroups) {
        for (int t = t0; t < t1; ++t) {
            const uint4 q = tiled[((long long)G * ntiles + t) * 64 + lane];
            const uint32_t wq[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                const float4 vv =
                    *reinterpret_cast<const float4 *>(&vf[t * kTile + 256 * i4 + 4 * lane]);
                const float vs[4] = {vv.x, vv.y, vv.z, vv.w};
#pragma unroll
                for (int s = 0; s < 4; ++s) {
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr)
                        acc[rr] = fmaf(field(wq[rr], i4 * 4 + s), vs[s], acc[rr]);
                }
            }
        }
    }
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
        const float t = wave_sum(acc[rr]);
        if (lane == 0) red[w * 4 + rr] = t;
    }
    __syncthreads();
    if (tid < 8) {
        const int g = tid >> 2, rr = tid & 3;
        const long long row = ((long long)blockIdx.x * 2 + g) * 4 + rr;
        if (row < n_out)
            out[(long long)blockIdx.y * ldo + row] = scale * (red[g * 4 + rr] + red[(g + 2) * 4 + rr]);
    }
}

template <typename VT>
hipError_t launch(const rsr_handle_s *h, const void *v, float scale, float *out, int batch,
                  int64_t ldv, int64_t ldo, hipStream_t stream) {
    static size_t attr_bytes = 0;  // largest dynamic LDS size enabled for this kernel so far
    auto kern = k_dense_matvec<VT>;
    const int ntiles = (int)(h->row_bytes / 256);
    const int ngroups = (int)((h->rows + 3) / 4);
    const size_t lds = (size_t)ntiles * kTile * 4 + 64;
    if (lds > attr_bytes) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_bytes = lds;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)((ngroups + 1) / 2), (unsigned)batch), dim3(256), lds,
                       stream, reinterpret_cast<const uint4 *>(h->packed), ntiles, (int)h->cols,
                       (int)h->rows, ngroups, v, (long long)ldv, out, (long long)ldo, scale);
    return hipGetLastError();
}

}  // namespace

// packed: [ceil(rows/4)][row_bytes/256 tiles][64 lanes][4 rows] dwords; row_bytes = tiles*256.
hipError_t launch_pack2(const int8_t *M, int64_t rows, int64_t cols, int64_t row_bytes,
                        uint8_t *packed, int *err_flag) {
    const int ntiles = (int)(row_bytes / 256);
    const int64_t total = (rows + 3) / 4 * ntiles * 256;
    hipLaunchKernelGGL(k_pack2_tiled, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, 0, M,
                       rows, cols, ntiles, reinterpret_cast<uint32_t *>(packed), err_flag);
    return hipGetLastError();
}

hipError_t launch_dense_matvec(const rsr_handle_s *h, const void *v, int v_dtype, float scale,
                               float *out, int batch, int64_t ldv, int64_t ldo,
                               hipStream_t stream) {
    return (v_dtype == RSR_BF16) ? launch<uint16_t>(h, v, scale, out, batch, ldv, ldo, stream)
                                 : launch<float>(h, v, scale, out, batch, ldv, ldo, stream);
}

const char *dense_matvec_kernel_name(int v_dtype) {
    return v_dtype == RSR_BF16 ? "k_dense_matvec<unsigned short>" : "k_dense_matvec<float>";
}

}  // namespace rsr
