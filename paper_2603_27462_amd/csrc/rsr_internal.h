// Internal declarations shared by the librsr translation units (not installed).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "rsr.h"

namespace rsr {

constexpr int kMaxWaves = 16;          // waves per workgroup in the multiply kernel
constexpr int kLoad = 512;             // stream entries one 16-byte-per-lane wave load covers
constexpr int kMaxCols = 32766;        // index 'cols' is the zero slot and must fit 15 bits
constexpr int kSmallCols = 16383;      // up to here an entry is tail<<15 | idx<<1
constexpr int kLdsBytes = 160 * 1024;  // LDS per workgroup on gfx950
constexpr int kLdsMisc = 1024;         // wave-total terms of the scatter phase
constexpr int kDenseRows = 16;         // dense comparison kernel: rows per workgroup
constexpr int kDenseTileCols = 256;    // and columns per 16-byte-per-lane tile

// One pass of an RSR handle (binary, M+, M- or fused).
//
// Multiply-kernel stream of a block: C chunks of 64*8*H entries.  In stream
// order a chunk is 64 strips of 8*H consecutive entries, strip l belonging to
// lane l; in memory it is H slabs of 512 entries, slab h holding entries
// 8h..8h+7 of every strip, lane after lane, so that each of the H loads of a
// wave is one contiguous 1 KiB read.  codes[chunk][l] is the group code of the
// first tail entry at or after the start of strip l.
struct PassData {
    uint16_t *pi = nullptr;       // canonical column permutation  [nb][cols]
    uint32_t *off = nullptr;      // canonical group boundaries    [nb][P+1]
    uint16_t *entries = nullptr;  // [nb][C][H][64][8]
    uint16_t *codes = nullptr;    // [nb][C][64]
    int8_t *wsign = nullptr;      // [nb][W][16]: weight of wave w's total in output row r
    int64_t C = 0;                // chunks per block
    float sign = 1.0f;
};

// Launch-time constants of the scatter phase and the split of chunks over waves.
struct FoldShape {
    int m = 0, Tc = 0, Q = 0;   // Tc = base^m classes handled by stage 1, Q = P / Tc
    int parts = 1;              // threads sharing one class in level 1 (1 or 2)
    int cnt1 = 0;               // entries every level-1 thread adds: ceil(Q / parts)
    int nact = 0;               // waves that hold fold threads
    int nrows = 0;              // entries per row of the weight table: max(Tc, Q)
    int G = 0;                  // groups of 256 entries per row
    unsigned short cb[2][kMaxWaves + 1] = {};  // per pass: wave w owns chunks [cb[w], cb[w+1])
};

}  // namespace rsr

struct rsr_handle_s {
    uint32_t magic = 0;
    int kind = 0, k = 0, base = 0, npass = 0, device = 0;
    int W = 0;    // waves per workgroup of the multiply kernel
    int H = 0;    // 16-byte loads per lane per chunk (1, 2 or 4)
    int enc = 0;  // entry encoding: kEncSmall or kEncBig
    int64_t rows = 0, cols = 0, nb = 0, P = 0;
    rsr::PassData pass[2];
    rsr::FoldShape fold;
    uint32_t *fpack = nullptr;   // scatter-phase weights, four per dword: [k][fold.G][64]
    uint32_t *fshare = nullptr;  // first entry of the level-1 share of every thread [W*64]
    bool stale = false;          // a failed rsr_preprocess_into left the buffers half-written
    uint8_t *packed = nullptr;   // dense kind: [rows/16][tiles][64 lanes][16 bytes], row_bytes = 64 tiles
    int64_t row_bytes = 0;
};

namespace rsr {

constexpr uint32_t kMagic = 0x52535231u;

// Entry encodings.  Small (cols <= kSmallCols): tail<<15 | idx<<1, so the LDS
// byte address of a bf16 element is one AND away and the tail flag is the sign
// of the 16-bit entry.  Big: idx<<1 | tail.
enum { kEncSmall = 0, kEncBig = 1 };

// mode of an encode pass
enum { MODE_BINARY = 0, MODE_POS = 1, MODE_NEG = 2, MODE_FUSED3 = 3 };

// --- preprocessing launches (null stream) ------------------------------------
hipError_t launch_encode(const int8_t *M, int64_t rows, int64_t cols, int k, int mode,
                         uint16_t *code, int *err_flag);
hipError_t launch_sort(const uint16_t *code, int64_t nb, int64_t cols, int k, int base, int64_t P,
                       uint16_t *pi, uint32_t *off);
hipError_t launch_stream_len(const uint32_t *off, int64_t nb, int64_t cols, int64_t P,
                             uint32_t *lens, uint32_t *longest);
hipError_t launch_fill_u32(uint32_t *p, uint32_t value, int64_t count);
hipError_t launch_pack_stream(const uint16_t *pi, const uint32_t *off, int64_t nb, int64_t cols,
                              int64_t P, int64_t C, int H, int enc, uint16_t *scratch,
                              uint16_t *entries, uint16_t *codes, int *err_flag);
hipError_t launch_transpose(const int8_t *M, int64_t rows, int64_t cols, int8_t *T);
hipError_t launch_pack2(const int8_t *M, int64_t rows, int64_t cols, int64_t row_bytes,
                        uint8_t *packed, int *err_flag);

// --- multiply launches ---------------------------------------------------------
hipError_t launch_rsr_matvec(const rsr_handle_s *h, const void *v, int v_dtype, float scale,
                             float *out, int batch, int64_t ldv, int64_t ldo, hipStream_t stream);
hipError_t launch_dense_matvec(const rsr_handle_s *h, const void *v, int v_dtype, float scale,
                               float *out, int batch, int64_t ldv, int64_t ldo, hipStream_t stream);
const char *rsr_matvec_kernel_name(int v_dtype, int H, int enc, int npass, bool single);
// True when every pass has at most W chunks per block (one chunk per wave, no loops).
bool matvec_is_single(const rsr_handle_s *h);
const char *dense_matvec_kernel_name(const rsr_handle_s *h, int v_dtype);

// Picks the chunk size (H loads of 512 entries per wave) and the number of
// waves per workgroup for nb blocks whose longest stream has `longest` entries.
// The environment variables RSR_H and RSR_W override the choice (tuning only).
void choose_launch_shape(int64_t longest, int64_t nb, int *H, int *W);


void make_fold_shape(int base, int k, int64_t P, int W, const int64_t C[2], int npass,
                     FoldShape *fs);
hipError_t launch_fold_tables(int base, int k, const FoldShape &fs, int W, uint32_t *fpack,
                              uint32_t *fshare);
hipError_t launch_wave_signs(int base, int k, const uint16_t *codes, int64_t nb, int64_t C, int W,
                             const FoldShape &fs, int pass, int8_t *wsign);

// Dynamic LDS beyond 64 KiB has to be enabled per kernel and device.  `enabled` is the
// kernel's table of the largest size enabled so far on each device (zero-initialised
// static storage).  Concurrent callers may both set the attribute: harmless.
constexpr int kMaxDevices = 64;
inline hipError_t ensure_dynamic_lds(const void *kernel, size_t bytes, int device,
                                     std::atomic<size_t> (&enabled)[kMaxDevices]) {
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    if (bytes <= enabled[device].load(std::memory_order_relaxed)) return hipSuccess;
    const hipError_t e =
        hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess) enabled[device].store(bytes, std::memory_order_relaxed);
    return e;
}

// LDS bytes the RSR multiply kernel needs: v and its zero slot, the wave-total terms,
// E[P] followed by a row of zeros (at most one per thread), and one level-1 sum per thread.
inline int64_t matvec_lds_bytes(int64_t P, int64_t cols, int v_elem_bytes, int W) {
    const int64_t vbytes = ((cols + 1) * v_elem_bytes + 15) / 16 * 16;
    return vbytes + kLdsMisc + P * 4 + 2 * (int64_t)W * 64 * 4;
}

}  // namespace rsr
