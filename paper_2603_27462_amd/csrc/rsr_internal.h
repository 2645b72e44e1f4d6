// Internal declarations shared by the librsr translation units (not installed).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "rsr.h"

namespace rsr {

constexpr int kMaxWaves = 16;          // waves per workgroup in the multiply kernel
constexpr int kSlab = 512;             // stream entries of one slab: 64 lanes x 8 entries (16 bytes per lane)
constexpr int kGroupSlabs = 4;         // slabs a wave requests together
constexpr int kMaxCols = 32766;        // index 'cols' is the zero slot and must fit 15 bits
constexpr int kSmallCols = 16383;      // up to here an entry is tail<<15 | idx<<1
constexpr int kLdsBytes = 160 * 1024;  // LDS per workgroup on gfx950
constexpr int kDenseRows = 16;         // dense comparison kernel: rows per workgroup
constexpr int kDenseTileCols = 256;    // and columns per 16-byte-per-lane tile

constexpr int kMaxLayers = 8;          // sibling layers one stacked handle can hold

// Kernel argument of a stacked handle: where the rows of every layer go.  A unit is a
// block of k rows (RSR kinds) or a group of 16 rows (dense kind); layers start on unit
// boundaries.  n = 0: not stacked.
struct LayerTable {
    float *out[kMaxLayers];
    float scale[kMaxLayers];
    int first[kMaxLayers + 1];  // first unit of layer i; first[n] = all units
    int rows[kMaxLayers];
    int n;
};

// One pass of an RSR handle (binary, M+, M- or fused).
//
// Multiply-kernel stream of a block: in stream order, for every group of identical
// columns in ascending pattern code (group 0, which contributes nothing, left out), the
// columns of the group, the last one flagged as tail.  The stream is cut into S slabs of
// 512 entries; wave w of the block's workgroup owns n_w = S/W + (w < S%W) consecutive
// slabs, lane l of the wave owns the strip of 8*n_w consecutive entries starting at
// entry l*8*n_w of the wave's part, and in memory slab h of a wave holds entries
// 8h..8h+7 of each of its 64 strips, lane after lane, so that every load of a wave is
// one contiguous KiB.  Each tail stores one prefix sum into a slot of the LDS array E:
//   indexed by code  slot = pattern code; an empty group has a placeholder entry (tail
//                    flag, zero slot of v), so every code 1..P-1 owns exactly one tail
//   indexed by rank  slot = rank of the group among the non-empty ones (1-based);
//                    no placeholders; the weights of every slot come from gword
// start[w][l] is the slot of the first tail at or after the start of strip (w, l).
struct PassData {
    uint16_t *pi = nullptr;       // canonical column permutation  [nb][cols]
    uint32_t *off = nullptr;      // canonical group boundaries    [nb][P+1]
    uint16_t *entries = nullptr;  // [nb][S][64][8]
    uint16_t *start = nullptr;    // [nb][W][64]
    // sign (2 bits, two's complement) of digit r of the code of the first group closed at or
    // after the start of the strip that follows strip (w, l); 0 when there is none.
    //   by code: [nb][k][64] words, (r, l) holds the W strips (w, l) at bits 2w (16-bit words
    //            when W <= 8, else 32-bit)
    //   by rank: [nb][W][64] 32-bit words, (w, l) holds the k rows at bits 2r
    void *sgn = nullptr;
    // narrow handles (cols <= 256, see rsr_narrow.hip): entries of a block four per lane, one
    // byte each; tail and valid flags per lane; sign words of the groups in rank order
    uint32_t *nent = nullptr;     // [nb][64]
    uint8_t *nmeta = nullptr;     // [nb][64]
    void *nsw = nullptr;          // [nb][slots], narrow_sw_bytes each
    uint32_t *gword = nullptr;    // by rank: [nb][slots] difference weights of every slot, fw bits per row
    uint32_t *gcount = nullptr;   // by rank: [nb] non-empty groups of the block
    int64_t S = 0;                // slabs per block
    float sign = 1.0f;
};

// Launch-time constants of the code-indexed scatter phase.
struct FoldShape {
    int m = 0, Tc = 0, Q = 0;   // Tc = base^m classes handled by stage 1, Q = P / Tc
    int parts = 1;              // threads sharing one class in level 1 (1 or 2)
    int cnt1 = 0;               // entries every level-1 thread adds: ceil(Q / parts)
    int nrows = 0;              // entries per row of the weight table: max(Tc, Q)
    int G = 0;                  // groups of 256 entries per row
};

}  // namespace rsr

struct rsr_handle_s {
    uint32_t magic = 0;
    int kind = 0, k = 0, base = 0, npass = 0, device = 0;
    int W = 0;        // waves per workgroup of the multiply kernel
    int enc = 0;      // entry encoding: kEncSmall or kEncBig
    int narrow = 0;   // cols <= 256: one wave per block, 8-bit entries (slots = sign words per block)
    int narrow_fw = 0, narrow_sw_bytes = 0;  // bits per row in a sign word, bytes per sign word
    int by_rank = 0;  // E indexed by group rank (no placeholders) instead of by pattern code
    int64_t rows = 0, cols = 0, nb = 0, P = 0;
    int64_t slots = 0;  // entries of E: P (by code) or 1 + the most non-empty groups of a block
    rsr::PassData pass[2];
    rsr::FoldShape fold;
    uint32_t *fpack = nullptr;   // by code: scatter-phase weights, four per dword: [k][fold.G][64]
    uint32_t *fshare = nullptr;  // by code: first entry of the level-1 share of every thread [W*64]
    int nlayers = 0;             // > 0: stacked handle (rows = the layers' rows padded to whole units)
    int64_t layer_rows[rsr::kMaxLayers] = {};
    int64_t layer_first[rsr::kMaxLayers + 1] = {};  // first unit (block / group of 16 rows) of a layer
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
hipError_t launch_fill_u32(uint32_t *p, uint32_t value, int64_t count);
hipError_t launch_encode(const int8_t *M, int64_t rows, int64_t cols, int k, int mode,
                         uint16_t *code, int *err_flag);
hipError_t launch_sort(const uint16_t *code, int64_t nb, int64_t cols, int k, int base, int64_t P,
                       uint16_t *pi, uint32_t *off);
// stats[0..2] = max over blocks of: columns outside group 0; the same plus the empty groups
// among codes 1..P-1; the non-empty groups among codes 1..P-1 (the caller zeroes them)
hipError_t launch_stream_stats(const uint32_t *off, int64_t nb, int64_t cols, int64_t P,
                               uint32_t *stats);
// Everything the multiply kernel reads of one pass, from the canonical pi / off:
// `logical` is scratch of nb * S * kSlab entries, `gcode` scratch of nb * slots entries
// (by rank only).  *err_flag |= 2 when a block does not hold the expected number of tails.
hipError_t launch_pack_pass(const rsr_handle_s *h, int pass, uint16_t *logical, uint16_t *gcode,
                            int *err_flag);
hipError_t launch_transpose(const int8_t *M, int64_t rows, int64_t cols, int8_t *T);
hipError_t launch_pack2(const int8_t *M, int64_t rows, int64_t cols, int64_t row_bytes,
                        uint8_t *packed, int *err_flag);

// --- multiply launches ---------------------------------------------------------
// `layers` (may be null): per-layer outputs and scales of a stacked handle; then out, scale
// and ldo are not used and batch is 1.
hipError_t launch_rsr_matvec(const rsr_handle_s *h, const void *v, int v_dtype, float scale,
                             float *out, int batch, int64_t ldv, int64_t ldo, hipStream_t stream,
                             const LayerTable *layers = nullptr);
hipError_t launch_dense_matvec(const rsr_handle_s *h, const void *v, int v_dtype, float scale,
                               float *out, int batch, int64_t ldv, int64_t ldo, hipStream_t stream,
                               const LayerTable *layers = nullptr);
// Writes the name of the multiply kernel h launches for (v_dtype, batch) into buf.
void rsr_matvec_kernel_name(const rsr_handle_s *h, int v_dtype, char *buf, size_t len);
const char *dense_matvec_kernel_name(const rsr_handle_s *h, int v_dtype);

// --- narrow matrices (cols <= kNarrowCols) ---------------------------------------------
constexpr int kNarrowCols = 256;
hipError_t launch_pack_narrow(const rsr_handle_s *h, int pass, int *err_flag);
hipError_t launch_narrow_matvec(const rsr_handle_s *h, const void *v, int v_dtype, float scale, float *out,
                                int batch, int64_t ldv, int64_t ldo, hipStream_t stream);

// --- reference launches of the benchmark ---------------------------------------------
hipError_t launch_probe_empty(int workgroups, int threads, int lds_bytes, hipStream_t stream);
hipError_t launch_probe_read(const void *src, int64_t bytes, int workgroups, int threads, void *sink,
                             hipStream_t stream);

// Waves per workgroup for nb blocks of k rows whose longest stream has `slabs` slabs.
int choose_waves(int64_t slabs, int64_t nb, int k, bool by_rank);
// True when E is better indexed by group rank: P floats do not fit LDS, or the placeholders
// of a code-indexed stream would outweigh the per-group weight words.
bool choose_by_rank(int64_t P, int64_t cols, int64_t longest_by_code, int64_t longest_by_rank,
                    int64_t most_groups);

void make_fold_shape(int base, int k, int64_t P, int W, FoldShape *fs);
hipError_t launch_fold_tables(int base, int k, const FoldShape &fs, int W, uint32_t *fpack,
                              uint32_t *fshare);

// bits per row in a gword: differences of two signs
inline int gword_field_bits(int base) { return base == 2 ? 2 : 3; }

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

// LDS bytes the RSR multiply kernel needs: v and its zero slot, one total per strip (at
// least eight waves' worth), E, and
// behind E either a row of zeros and one level-1 sum per thread (by code) or one partial
// per (wave, row) (by rank).
inline int64_t matvec_lds_bytes(int64_t slots, int64_t cols, int v_elem_bytes, int W, bool by_rank) {
    const int64_t vbytes = ((cols + 1) * v_elem_bytes + 15) / 16 * 16;
    const int64_t tail = by_rank ? (int64_t)W * 16 * 4 : 2 * (int64_t)W * 64 * 4;
    return vbytes + (int64_t)(W < 8 ? 8 : W) * 64 * 4 + slots * 4 + tail;
}

}  // namespace rsr
