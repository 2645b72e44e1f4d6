// Internal declarations shared by the librsr translation units (not installed).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "rsr.h"

namespace rsr {

constexpr int kMaxWaves = 16;          // waves per workgroup in the multiply kernel
constexpr int kChunk = 512;            // stream entries one wave consumes per iteration
constexpr int kMaxCols = 32766;        // index 'cols' is the zero slot; entry = idx<<1|tail
constexpr int kLdsBytes = 160 * 1024;  // LDS per workgroup on gfx950
constexpr int kLdsMisc = 2048;         // wave totals, partial outputs, wave start codes

// One pass of an RSR handle (binary, M+, M- or fused).
struct PassData {
    uint16_t *pi = nullptr;      // canonical column permutation  [nb][cols]
    uint32_t *off = nullptr;     // canonical group boundaries    [nb][P+1]
    uint16_t *stream = nullptr;  // multiply-kernel stream        [nb][S]
    uint32_t *hdr = nullptr;     // first group code of each wave [nb][W]
    int64_t S = 0;               // stream entries per block (multiple of W*kChunk)
    float sign = 1.0f;
};

}  // namespace rsr

struct rsr_handle_s {
    uint32_t magic = 0;
    int kind = 0, k = 0, base = 0, npass = 0, W = 0, device = 0;
    int64_t rows = 0, cols = 0, nb = 0, P = 0;
    rsr::PassData pass[2];
    uint8_t *packed = nullptr;   // dense kind: [rows][row_bytes], row_bytes % 16 == 0
    int64_t row_bytes = 0;
};

namespace rsr {

constexpr uint32_t kMagic = 0x52535231u;

// mode of an encode pass
enum { MODE_BINARY = 0, MODE_POS = 1, MODE_NEG = 2, MODE_FUSED3 = 3 };

// --- preprocessing launches (null stream) ------------------------------------
hipError_t launch_encode(const int8_t *M, int64_t rows, int64_t cols, int k, int mode,
                         uint16_t *code, int *err_flag);
hipError_t launch_sort(const uint16_t *code, int64_t nb, int64_t cols, int k, int base, int64_t P,
                       uint16_t *pi, uint32_t *off);
hipError_t launch_stream_len(const uint32_t *off, int64_t nb, int64_t cols, int64_t P,
                             uint32_t *lens);
hipError_t launch_pack_stream(const uint16_t *pi, const uint32_t *off, int64_t nb, int64_t cols,
                              int64_t P, int64_t S, int W, uint16_t *stream, uint32_t *hdr,
                              int *err_flag);
hipError_t launch_pack2(const int8_t *M, int64_t rows, int64_t cols, int64_t row_bytes,
                        uint8_t *packed, int *err_flag);

// --- multiply launches ---------------------------------------------------------
hipError_t launch_rsr_matvec(const rsr_handle_s *h, const void *v, int v_dtype, float scale,
                             float *out, int batch, int64_t ldv, int64_t ldo, hipStream_t stream);
hipError_t launch_dense_matvec(const rsr_handle_s *h, const void *v, int v_dtype, float scale,
                               float *out, int batch, int64_t ldv, int64_t ldo, hipStream_t stream);
const char *rsr_matvec_kernel_name(int base, int v_dtype);
const char *dense_matvec_kernel_name(int v_dtype);

// LDS bytes the RSR multiply kernel needs for a pass layout and vector type.
inline int64_t matvec_lds_bytes(int64_t P, int64_t cols, int v_elem_bytes) {
    int64_t vbytes = ((cols + 1) * v_elem_bytes + 15) / 16 * 16;
    return P * 4 + kLdsMisc + vbytes;
}

}  // namespace rsr
