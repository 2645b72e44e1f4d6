// Dense 2-bit packed ternary matvec: the on-GPU comparison point for the RSR
// kernel (the role the paper gives its low-bit "BitNet" multiplier baseline in
// Benchmarking Results).  No preprocessing beyond packing; every matrix entry
// is decoded and multiplied.
//
// The product is a dense contraction, so it runs on the matrix cores:
// v_mfma_f32_16x16x32_bf16 with A = 16 rows x 32 columns of weights and B = the
// matching 32 entries of v (the same in all 16 B columns; column 0 of the
// result is read).  A 2-bit code (00 = 0, 01 = +1, 11 = -1) placed in the two
// top bits of a bf16 is 0, +2.0 or -2.0, so one shift and one AND turn a dword
// of 16 codes into a pair of A elements; the factor 2 is taken out of the
// output scale.  float32 vectors are split exactly into three bf16 planes
// (top, middle and bottom 8 mantissa bits) and take three MFMAs per step.  A batch
// of vectors fills the B columns: up to 16 vectors cost one pass over the weights.
//
// Layout: [row group of 16][tile of 256 columns][lane][4 dwords], one 16-byte
// load per lane and tile (1 KiB per wave).  Lane l holds row l%16 and the
// column slices 8*(l/16).. of the tile's eight 32-column steps: dword d feeds
// steps 2d and 2d+1; inside a dword, pair slot p (0..7) has its even column in
// bits 14-2p.. and its odd column in bits 30-2p...
#include "rsr_device.h"
#include "rsr_internal.h"

namespace rsr {

namespace {

constexpr int kSlabTiles = 64;  // tiles of v staged in LDS at a time (16384 columns)
constexpr int kDenseWaves = 8;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void k_pack2_tiled(const int8_t *__restrict__ M, int64_t rows,
                                                     int64_t cols, int64_t ntiles,
                                                     uint32_t *__restrict__ tiled,
                                                     int *__restrict__ err_flag) {
    const int64_t ngroups = (rows + kDenseRows - 1) / kDenseRows;
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (gid >= ngroups * ntiles * 256) return;
    const int d = (int)(gid & 3);
    const int lane = (int)((gid >> 2) & 63);
    const int64_t gt = gid >> 8;
    const int64_t G = gt / ntiles, t = gt % ntiles;
    const int64_t i = G * kDenseRows + (lane & 15);
    const int kq = lane >> 4;
    uint32_t word = 0;
    bool bad = false;
    if (i < rows) {
        for (int p = 0; p < 8; ++p) {
            for (int hi = 0; hi < 2; ++hi) {
                const int64_t j = t * kDenseTileCols + (2 * d + (p >> 2)) * 32 + 8 * kq + 2 * (p & 3) + hi;
                if (j < cols) {
                    const int m = M[i * cols + j];
                    if (m < -1 || m > 1) bad = true;
                    word |= ((uint32_t)m & 3u) << ((hi ? 30 : 14) - 2 * p);
                }
            }
        }
    }
    if (bad) atomicOr(err_flag, 1);
    tiled[gid] = word;
}

// Stages columns [c0, c0 + ncols) of one vector (zero past n_in) into LDS at byte address
// `at` as bf16 planes of `plane` bytes each: one plane for bf16 input, three for float32.
template <typename VT>
__device__ __forceinline__ void stage_v(const VT *__restrict__ vg, int n_in, int c0, int ncols,
                                        uint32_t at, uint32_t plane, int tid, int nthreads);

template <>
__device__ __forceinline__ void stage_v<uint16_t>(const uint16_t *__restrict__ vg, int n_in, int c0,
                                                  int ncols, uint32_t at, uint32_t plane, int tid,
                                                  int nthreads) {
    (void)plane;
    lds_u128 *l16 = reinterpret_cast<lds_u128 *>(static_cast<uintptr_t>(at));
    const bool aligned = (reinterpret_cast<uintptr_t>(vg + c0) & 15) == 0;
    const int full = aligned ? max(0, min(ncols, n_in - c0)) >> 3 : 0;  // whole 16-byte pieces
    const u32x4 *v16 = reinterpret_cast<const u32x4 *>(vg + c0);
    for (int j = tid; j < full; j += nthreads) l16[j] = v16[j];
    for (int j = full * 8 + tid; j < ncols; j += nthreads)
        lds_store_v<uint16_t>((int)at + j * 2, (c0 + j < n_in) ? vg[c0 + j] : (uint16_t)0);
}

template <>
__device__ __forceinline__ void stage_v<float>(const float *__restrict__ vg, int n_in, int c0,
                                               int ncols, uint32_t at, uint32_t plane, int tid,
                                               int nthreads) {
    for (int j = tid; j < ncols; j += nthreads) {
        const float x = (c0 + j < n_in) ? vg[c0 + j] : 0.0f;
        // x = top + mid + bot exactly: each piece keeps 8 of the 24 significant bits
        const uint32_t top = __float_as_uint(x) & 0xffff0000u;
        const float r1 = x - __uint_as_float(top);
        const uint32_t mid = __float_as_uint(r1) & 0xffff0000u;
        const float r2 = r1 - __uint_as_float(mid);
        lds_store_v<uint16_t>((int)at + j * 2, (uint16_t)(top >> 16));
        lds_store_v<uint16_t>((int)(at + plane) + j * 2, (uint16_t)(mid >> 16));
        lds_store_v<uint16_t>((int)(at + 2 * plane) + j * 2, (uint16_t)(__float_as_uint(r2) >> 16));
    }
}

// One tile (16 rows x 256 columns) of one wave: eight MFMA steps (three MFMAs each for
// float32 input).  vb: LDS byte address of this lane's slice of the tile's first step.
template <int PLANES>
__device__ __forceinline__ void tile_mfma(const u32x4 q, uint32_t vb, uint32_t plane, f32x4 &acc) {
    const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
    for (int d = 0; d < 4; ++d) {
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            u32x4 a;
            a.x = (w[d] << (8 * half)) & 0xc000c000u;
            a.y = (w[d] << (8 * half + 2)) & 0xc000c000u;
            a.z = (w[d] << (8 * half + 4)) & 0xc000c000u;
            a.w = (w[d] << (8 * half + 6)) & 0xc000c000u;
            const uint32_t at = vb + (uint32_t)(2 * d + half) * 64u;
#pragma unroll
            for (int pl = 0; pl < PLANES; ++pl) {
                const u32x4 b = *reinterpret_cast<lds_u128 *>(static_cast<uintptr_t>(at + pl * plane));
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                              __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
            }
        }
    }
}

// Workgroup = 8 waves = 8/wpg groups of 16 rows, times up to 16 vectors (the B columns of
// the MFMA); the wpg waves of a row group split the tiles of every slab (wpg = 8 unless
// the matrix has fewer than 8 column tiles).  LDS: vector n at n * vstride (planes
// back to back; the stride is padded by 64 bytes so that the 16-byte reads of the 64
// lanes -- 16 vectors x 4 column slices -- fall on distinct banks), then the partial
// results, float [8 waves][16 vectors][16 rows].
template <typename VT, int wpg>
__global__ __launch_bounds__(kDenseWaves * 64) void k_dense_matvec(
    const u32x4 *__restrict__ tiled, int ntiles, int slab_tiles, int ngroups, int n_in,
    int n_out, const void *__restrict__ v, long long ldv, int batch, int nv, float *__restrict__ out,
    long long ldo, float scale, const LayerTable layers) {
    constexpr int PLANES = sizeof(VT) == 4 ? 3 : 1;
    constexpr int nthreads = kDenseWaves * 64;
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int vec0 = blockIdx.y * nv, nvh = min(nv, batch - vec0);  // this workgroup's vectors
    const VT *vg = reinterpret_cast<const VT *>(v) + (long long)vec0 * ldv;
    const uint32_t plane = (uint32_t)slab_tiles * kDenseTileCols * 2u;
    const uint32_t vstride = plane * PLANES + 64u;
    const uint32_t red_at = vstride * (uint32_t)nv;
    constexpr int gpw = kDenseWaves / wpg;              // row groups of this workgroup
    const int wg = w / wpg, ws = w - wg * wpg;          // the wave's row group and share
    const long long G = (long long)blockIdx.x * gpw + wg;
    const bool live = G < ngroups;
    const u32x4 *wp = tiled + ((live ? G : 0) * ntiles) * 64 + lane;
    // B column lane%16 is vector lane%16 (columns without a vector repeat vector 0)
    const int col = lane & 15;
    const uint32_t lane_vb = (uint32_t)(col < nvh ? col : 0) * vstride + (uint32_t)(lane >> 4) * 16u;
    f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};

    for (int s0 = 0; s0 < ntiles; s0 += slab_tiles) {
        const int st = min(slab_tiles, ntiles - s0);  // tiles in this slab
        // this wave's tiles of the slab: [t0, t1)
        const int t0 = s0 + (st * ws) / wpg, t1 = live ? s0 + (st * (ws + 1)) / wpg : t0;
        // the first eight weight loads leave before v is staged
        u32x4 q[8];
        if (t1 > t0) {
#pragma unroll
            for (int i = 0; i < 8; ++i)
                q[i] = __builtin_nontemporal_load(&wp[(long long)min(t0 + i, t1 - 1) * 64]);
        }
        if (s0 > 0) __syncthreads();  // the previous slab is no longer read
        for (int n = 0; n < nvh; ++n)
            stage_v<VT>(vg + (long long)n * ldv, n_in, s0 * kDenseTileCols, st * kDenseTileCols,
                        (uint32_t)n * vstride, plane, tid, nthreads);
        __syncthreads();
        for (int tb = t0; tb < t1; tb += 8) {
            if (tb > t0) {
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    q[i] = __builtin_nontemporal_load(&wp[(long long)min(tb + i, t1 - 1) * 64]);
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                if (tb + i < t1)
                    tile_mfma<PLANES>(q[i], (uint32_t)(tb + i - s0) * (kDenseTileCols * 2) + lane_vb,
                                      plane, acc);
            }
        }
    }
    // the 16x16 result: lane holds column lane%16, rows 4*(lane/16) .. +3
    {
        const uint32_t at = red_at + (uint32_t)((w * 16 + col) * 16 + (lane >> 4) * 4) * 4u;
        *lds_float(at) = acc.x;
        *lds_float(at + 4) = acc.y;
        *lds_float(at + 8) = acc.z;
        *lds_float(at + 12) = acc.w;
    }
    __syncthreads();
    for (int e = tid; e < gpw * 256; e += nthreads) {  // (row group, vector, row)
        const int g = e >> 8, n = (e >> 4) & 15, r = e & 15;
        float sum = 0.0f;
#pragma unroll
        for (int i = 0; i < wpg; ++i)
            sum += *lds_float(red_at + (uint32_t)(((g * wpg + i) * 16 + n) * 16 + r) * 4u);
        const long long group = (long long)blockIdx.x * gpw + g;
        const long long row = group * kDenseRows + r;
        // the weights were +-2
        if (layers.n == 0) {
            if (n < nvh && row < n_out) out[(long long)(vec0 + n) * ldo + row] = (0.5f * scale) * sum;
        } else if (n == 0 && row < n_out) {
            // stacked handle: the group belongs to one layer (layers start on group boundaries)
            int s_ = 0;
#pragma unroll
            for (int i = 1; i < kMaxLayers; ++i)
                if (i < layers.n && group >= layers.first[i]) s_ = i;
            const long long local = (group - layers.first[s_]) * kDenseRows + r;
            if (local < layers.rows[s_]) layers.out[s_][local] = (0.5f * layers.scale[s_]) * sum;
        }
    }
}


template <typename VT, int WPG>
hipError_t launch_w(const rsr_handle_s *h, const void *v, float scale, float *out, int batch,
                    int64_t ldv, int64_t ldo, hipStream_t stream, int nv, int slab_tiles, size_t lds,
                    const LayerTable &layers) {
    static std::atomic<size_t> enabled[kMaxDevices];
    auto kern = k_dense_matvec<VT, WPG>;
    const int ntiles = (int)(h->row_bytes / (kDenseTileCols / 4));
    const int ngroups = (int)((h->rows + kDenseRows - 1) / kDenseRows);
    if (hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(kern), lds, h->device, enabled))
        return e;
    constexpr int gpw = kDenseWaves / WPG;
    hipLaunchKernelGGL(kern, dim3((unsigned)((ngroups + gpw - 1) / gpw), (unsigned)((batch + nv - 1) / nv)),
                       dim3(kDenseWaves * 64), lds, stream,
                       reinterpret_cast<const u32x4 *>(h->packed), ntiles, slab_tiles, ngroups,
                       (int)h->cols, (int)h->rows, v, (long long)ldv, batch, nv, out, (long long)ldo,
                       scale, layers);
    return hipGetLastError();
}

constexpr size_t kDenseLdsBudget = 150 * 1024;

template <typename VT>
hipError_t launch(const rsr_handle_s *h, const void *v, float scale, float *out, int batch,
                  int64_t ldv, int64_t ldo, hipStream_t stream, const LayerTable &layers) {
    const int ntiles = (int)(h->row_bytes / (kDenseTileCols / 4));
    const int planes = sizeof(VT) == 4 ? 3 : 1;
    // vectors per workgroup (the weights are read once for all of them) and the slab of
    // columns staged at a time: as many vectors as keep a slab of at least 8 tiles in LDS
    auto slab_for = [&](int nv) {
        const size_t per_tile = (size_t)nv * planes * kDenseTileCols * 2;
        const size_t fit = (kDenseLdsBudget - (size_t)nv * 64) / per_tile;
        return (int)(fit < (size_t)kSlabTiles ? fit : (size_t)kSlabTiles);
    };
    int nv = batch < 16 ? batch : 16;
    while (nv > 1 && slab_for(nv) < 8 && slab_for(nv) < ntiles) nv = (nv + 1) / 2;
    int slab_tiles = slab_for(nv);
    if (slab_tiles > ntiles) slab_tiles = ntiles;
    if (slab_tiles < 1) slab_tiles = 1;
    const size_t lds = (size_t)nv * ((size_t)slab_tiles * kDenseTileCols * 2 * planes + 64) +
                       (size_t)kDenseWaves * 16 * 16 * 4;
    // waves per row group: a power of two, at most one per tile of a slab
    if (slab_tiles >= 8) return launch_w<VT, 8>(h, v, scale, out, batch, ldv, ldo, stream, nv, slab_tiles, lds, layers);
    if (slab_tiles >= 4) return launch_w<VT, 4>(h, v, scale, out, batch, ldv, ldo, stream, nv, slab_tiles, lds, layers);
    if (slab_tiles >= 2) return launch_w<VT, 2>(h, v, scale, out, batch, ldv, ldo, stream, nv, slab_tiles, lds, layers);
    return launch_w<VT, 1>(h, v, scale, out, batch, ldv, ldo, stream, nv, slab_tiles, lds, layers);
}

}  // namespace

// packed: [ceil(rows/16)][row_bytes/64 tiles][64 lanes][4] dwords; row_bytes = tiles*64.
hipError_t launch_pack2(const int8_t *M, int64_t rows, int64_t cols, int64_t row_bytes,
                        uint8_t *packed, int *err_flag) {
    const int64_t ntiles = row_bytes / (kDenseTileCols / 4);
    const int64_t total = (rows + kDenseRows - 1) / kDenseRows * ntiles * 256;
    hipLaunchKernelGGL(k_pack2_tiled, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, 0, M,
                       rows, cols, ntiles, reinterpret_cast<uint32_t *>(packed), err_flag);
    return hipGetLastError();
}

hipError_t launch_dense_matvec(const rsr_handle_s *h, const void *v, int v_dtype, float scale,
                               float *out, int batch, int64_t ldv, int64_t ldo,
                               hipStream_t stream, const LayerTable *layers) {
    LayerTable none;
    none.n = 0;
    const LayerTable &lt = layers ? *layers : none;
    return (v_dtype == RSR_BF16) ? launch<uint16_t>(h, v, scale, out, batch, ldv, ldo, stream, lt)
                                 : launch<float>(h, v, scale, out, batch, ldv, ldo, stream, lt);
}

const char *dense_matvec_kernel_name(const rsr_handle_s *h, int v_dtype) {
    // the instantiation a single vector launches
    const int64_t ntiles = h->row_bytes / (kDenseTileCols / 4);
    const bool bf = v_dtype == RSR_BF16;
    if (ntiles >= 8) return bf ? "k_dense_matvec<unsigned short, 8>" : "k_dense_matvec<float, 8>";
    if (ntiles >= 4) return bf ? "k_dense_matvec<unsigned short, 4>" : "k_dense_matvec<float, 4>";
    if (ntiles >= 2) return bf ? "k_dense_matvec<unsigned short, 2>" : "k_dense_matvec<float, 2>";
    return bf ? "k_dense_matvec<unsigned short, 1>" : "k_dense_matvec<float, 1>";
}

}  // namespace rsr
