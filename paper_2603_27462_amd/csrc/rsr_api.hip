// C ABI of librsr: argument checks, device-memory ownership, and the order of
// the preprocessing launches.  All arithmetic of the method is in the kernels
// (rsr_preprocess.hip, rsr_matvec.hip, rsr_dense.hip).
#include <cstring>
#include <new>
#include <vector>

#include "rsr_internal.h"

namespace {

thread_local int g_last_error = RSR_OK;

int fail(int code) {
    g_last_error = code;
    return code;
}

bool good(const rsr_handle_s *h) { return h && h->magic == rsr::kMagic; }
bool is_rsr_kind(int kind) {
    return kind == RSR_BINARY || kind == RSR_TERNARY_2PASS || kind == RSR_TERNARY_FUSED;
}

template <typename T>
hipError_t dev_alloc(T **p, size_t count) {
    *p = nullptr;
    return hipMalloc(reinterpret_cast<void **>(p), count ? count * sizeof(T) : sizeof(T));
}

void free_handle(rsr_handle_s *h) {
    if (!h) return;
    for (auto &ps : h->pass) {
        if (ps.pi) (void)hipFree(ps.pi);
        if (ps.off) (void)hipFree(ps.off);
        if (ps.entries) (void)hipFree(ps.entries);
        if (ps.start) (void)hipFree(ps.start);
        if (ps.sgn) (void)hipFree(ps.sgn);
        if (ps.gword) (void)hipFree(ps.gword);
        if (ps.nent) (void)hipFree(ps.nent);
        if (ps.nmeta) (void)hipFree(ps.nmeta);
        if (ps.nsw) (void)hipFree(ps.nsw);
        if (ps.gcount) (void)hipFree(ps.gcount);
    }
    if (h->fpack) (void)hipFree(h->fpack);
    if (h->fshare) (void)hipFree(h->fshare);
    if (h->packed) (void)hipFree(h->packed);
    h->magic = 0;
    delete h;
}

int64_t ipow(int64_t b, int e) {
    int64_t p = 1;
    for (int i = 0; i < e; ++i) p *= b;
    return p;
}

// Translate a HIP failure: out-of-memory is reported as such.
int hip_code(hipError_t e) { return e == hipErrorOutOfMemory ? RSR_ENOMEM : RSR_EHIP; }

#define RSR_TRY(expr)                                   \
    do {                                                \
        hipError_t e_ = (expr);                         \
        if (e_ != hipSuccess) { rc = hip_code(e_); goto done; } \
    } while (0)

// Device memory a preprocessing run needs besides the handle's own buffers: the pattern
// codes of every (block, column), the stream in logical order, the codes of the non-empty
// groups (rank-indexed handles), and a few words of flags (kFlagErr: entry outside the
// alphabet / self-check; kFlagStats + 3 * pass: the three maxima of launch_stream_stats).
struct Temps {
    uint16_t *code = nullptr;     // [nb][cols]
    uint16_t *logical = nullptr;  // [nb][max over passes of S * 512]
    uint16_t *gcode = nullptr;    // [nb][slots], rank-indexed handles only
    int *flags = nullptr;         // [kFlagWords]
};
constexpr int kFlagErr = 0, kFlagStats = 1, kFlagWords = 64;

// What the streams of a matrix need, per pass: longest stream of a block without and with
// placeholders for empty groups, and the most non-empty groups of a block.
struct StreamStats {
    int64_t real[2] = {0, 0}, with_empty[2] = {0, 0}, groups[2] = {0, 0};
};

int read_flags(const Temps &t, int (&host)[kFlagWords]) {
    return hipMemcpy(host, t.flags, sizeof(host), hipMemcpyDeviceToHost) == hipSuccess ? RSR_OK
                                                                                       : RSR_EHIP;
}

int run_dense(rsr_handle_s *h, const int8_t *M, const Temps &t) {
    int host[kFlagWords];
    if (rsr::launch_fill_u32(reinterpret_cast<uint32_t *>(t.flags), 0u, kFlagWords) != hipSuccess ||
        rsr::launch_pack2(M, h->rows, h->cols, h->row_bytes, h->packed, t.flags + kFlagErr) != hipSuccess)
        return RSR_EHIP;
    if (int rc = read_flags(t, host)) return rc;
    return host[kFlagErr] ? RSR_EVALUE : RSR_OK;
}

// encode -> counting sort -> stream statistics, per pass
int run_sort_passes(rsr_handle_s *h, const int8_t *M, const Temps &t, StreamStats *st) {
    static const int modes[3][2] = {{rsr::MODE_BINARY, 0}, {rsr::MODE_POS, rsr::MODE_NEG},
                                    {rsr::MODE_FUSED3, 0}};
    int host[kFlagWords];
    if (rsr::launch_fill_u32(reinterpret_cast<uint32_t *>(t.flags), 0u, kFlagWords) != hipSuccess)
        return RSR_EHIP;
    for (int ps = 0; ps < h->npass; ++ps) {
        rsr::PassData &pd = h->pass[ps];
        pd.sign = (ps == 0) ? 1.0f : -1.0f;
        if (rsr::launch_encode(M, h->rows, h->cols, h->k, modes[h->kind][ps], t.code,
                               t.flags + kFlagErr) != hipSuccess ||
            rsr::launch_sort(t.code, h->nb, h->cols, h->k, h->base, h->P, pd.pi, pd.off) != hipSuccess ||
            rsr::launch_stream_stats(pd.off, h->nb, h->cols, h->P,
                                     reinterpret_cast<uint32_t *>(t.flags + kFlagStats + 3 * ps)) !=
                hipSuccess)
            return RSR_EHIP;
    }
    if (int rc = read_flags(t, host)) return rc;
    if (host[kFlagErr]) return RSR_EVALUE;
    for (int ps = 0; ps < h->npass; ++ps) {
        st->real[ps] = (uint32_t)host[kFlagStats + 3 * ps];
        st->with_empty[ps] = (uint32_t)host[kFlagStats + 3 * ps + 1];
        st->groups[ps] = (uint32_t)host[kFlagStats + 3 * ps + 2];
    }
    return RSR_OK;
}

int64_t slabs_for(int64_t entries) {
    const int64_t s = (entries + rsr::kSlab - 1) / rsr::kSlab;
    return s < 1 ? 1 : s;
}

// the stream and the small tables of the multiply kernel, in the layout the handle records
int run_pack_passes(rsr_handle_s *h, const Temps &t) {
    int host[kFlagWords];
    if (h->narrow) {
        for (int ps = 0; ps < h->npass; ++ps)
            if (rsr::launch_pack_narrow(h, ps, t.flags + kFlagErr) != hipSuccess) return RSR_EHIP;
        if (int rc = read_flags(t, host)) return rc;
        return host[kFlagErr] ? RSR_EINTERNAL : RSR_OK;
    }
    if (!h->by_rank &&
        rsr::launch_fold_tables(h->base, h->k, h->fold, h->W, h->fpack, h->fshare) != hipSuccess)
        return RSR_EHIP;
    for (int ps = 0; ps < h->npass; ++ps)
        if (rsr::launch_pack_pass(h, ps, t.logical, t.gcode, t.flags + kFlagErr) != hipSuccess)
            return RSR_EHIP;
    if (int rc = read_flags(t, host)) return rc;
    return host[kFlagErr] ? RSR_EINTERNAL : RSR_OK;
}

// Bytes of the strip-sign table of one pass.
size_t sign_table_bytes(const rsr_handle_s *h) {
    if (h->by_rank) return (size_t)h->nb * h->W * 64 * 4;
    return (size_t)h->nb * h->k * 64 * (h->W <= 8 ? 2 : 4);
}

int preprocess_dense(rsr_handle_s *h, const int8_t *M) {
    int rc = RSR_OK;
    Temps t;
    const int64_t ntiles = (h->cols + rsr::kDenseTileCols - 1) / rsr::kDenseTileCols;
    h->row_bytes = ntiles * (rsr::kDenseTileCols / 4);
    const size_t bytes =
        (size_t)((h->rows + rsr::kDenseRows - 1) / rsr::kDenseRows) * rsr::kDenseRows * h->row_bytes;
    RSR_TRY(dev_alloc(&h->packed, bytes));
    RSR_TRY(dev_alloc(&t.flags, kFlagWords));
    rc = run_dense(h, M, t);
done:
    if (t.flags) (void)hipFree(t.flags);
    return rc;
}

int preprocess_rsr(rsr_handle_s *h, const int8_t *M, bool allow_narrow) {
    int rc = RSR_OK;
    Temps t;
    const int64_t nb = h->nb, cols = h->cols, P = h->P;
    StreamStats st;

    RSR_TRY(dev_alloc(&t.code, (size_t)(nb * cols)));
    RSR_TRY(dev_alloc(&t.flags, kFlagWords));
    for (int ps = 0; ps < h->npass; ++ps) {
        RSR_TRY(dev_alloc(&h->pass[ps].pi, (size_t)(nb * cols)));
        RSR_TRY(dev_alloc(&h->pass[ps].off, (size_t)(nb * (P + 1))));
    }
    if ((rc = run_sort_passes(h, M, t, &st)) != RSR_OK) goto done;
    {
        // narrow matrices: 8-bit entries, one wave per block
        const int fw = h->base == 2 ? 1 : 2;
        if (allow_narrow && cols <= rsr::kNarrowCols && h->k * fw <= 32) {
            int64_t most = st.groups[0] > st.groups[1] ? st.groups[0] : st.groups[1];
            h->narrow = 1;
            h->narrow_fw = fw;
            h->narrow_sw_bytes = h->k * fw <= 8 ? 1 : h->k * fw <= 16 ? 2 : 4;
            h->slots = most < 4 ? 4 : (most + 3) / 4 * 4;
            for (int ps = 0; ps < h->npass; ++ps) {
                rsr::PassData &pd = h->pass[ps];
                RSR_TRY(dev_alloc(&pd.nent, (size_t)nb * 64));
                RSR_TRY(dev_alloc(&pd.nmeta, (size_t)nb * 64));
                RSR_TRY(dev_alloc(reinterpret_cast<unsigned char **>(&pd.nsw),
                                  (size_t)(nb * h->slots) * h->narrow_sw_bytes));
            }
            rc = run_pack_passes(h, t);
            goto done;
        }
    }
    {
        const int ph = (h->npass == 2 && st.with_empty[1] > st.with_empty[0]) ? 1 : 0;  // the heavier pass
        h->by_rank = rsr::choose_by_rank(P, cols, st.with_empty[ph], st.real[ph], st.groups[ph]) ? 1 : 0;
        int64_t maxS = 0, most = 0;
        for (int ps = 0; ps < h->npass; ++ps) {
            rsr::PassData &pd = h->pass[ps];
            pd.S = slabs_for(h->by_rank ? st.real[ps] : st.with_empty[ps]);
            if (pd.S > maxS) maxS = pd.S;
            if (st.groups[ps] > most) most = st.groups[ps];
        }
        h->slots = h->by_rank ? most + 1 : P;
        h->W = rsr::choose_waves(maxS, nb, h->k, h->by_rank != 0);
        h->enc = (cols <= rsr::kSmallCols) ? rsr::kEncSmall : rsr::kEncBig;
        if (rsr::matvec_lds_bytes(h->slots, cols, 4, h->W, h->by_rank != 0) > rsr::kLdsBytes) {
            rc = RSR_EUNSUPPORTED;
            goto done;
        }
        if (h->by_rank) {
            RSR_TRY(dev_alloc(&t.gcode, (size_t)(nb * h->slots)));
        } else {
            rsr::make_fold_shape(h->base, h->k, P, h->W, &h->fold);
            RSR_TRY(dev_alloc(&h->fpack, (size_t)h->k * h->fold.G * 64));
            RSR_TRY(dev_alloc(&h->fshare, (size_t)h->W * 64));
        }
        RSR_TRY(dev_alloc(&t.logical, (size_t)(nb * maxS * rsr::kSlab)));
        for (int ps = 0; ps < h->npass; ++ps) {
            rsr::PassData &pd = h->pass[ps];
            RSR_TRY(dev_alloc(&pd.entries, (size_t)(nb * pd.S * rsr::kSlab)));
            RSR_TRY(dev_alloc(&pd.start, (size_t)(nb * h->W * 64)));
            RSR_TRY(dev_alloc(reinterpret_cast<unsigned char **>(&pd.sgn), sign_table_bytes(h)));
            if (h->by_rank) {
                RSR_TRY(dev_alloc(&pd.gword, (size_t)(nb * h->slots)));
                RSR_TRY(dev_alloc(&pd.gcount, (size_t)nb));
            }
        }
    }
    rc = run_pack_passes(h, t);
done:
    if (t.code) (void)hipFree(t.code);
    if (t.logical) (void)hipFree(t.logical);
    if (t.gcode) (void)hipFree(t.gcode);
    if (t.flags) (void)hipFree(t.flags);
    return rc;
}

}  // namespace

namespace {

// Preprocessing with a given block height (k is ignored for the dense kind).
rsr_handle_s *preprocess_with_k(const int8_t *M, int64_t rows, int64_t cols, int k, int kind,
                                bool allow_narrow = true) {
    rsr_handle_s *h = new (std::nothrow) rsr_handle_s();
    if (!h) { fail(RSR_ENOMEM); return nullptr; }
    h->magic = rsr::kMagic;
    h->kind = kind;
    h->rows = rows;
    h->cols = cols;
    if (hipGetDevice(&h->device) != hipSuccess) { free_handle(h); fail(RSR_EHIP); return nullptr; }

    int rc;
    if (kind == RSR_DENSE_TERNARY_P2) {
        rc = preprocess_dense(h, M);
    } else {
        const bool fused = (kind == RSR_TERNARY_FUSED);
        const int kmax = fused ? 10 : 15;
        h->k = k;
        h->base = fused ? 3 : 2;
        h->npass = (kind == RSR_TERNARY_2PASS) ? 2 : 1;
        if (k > kmax) { free_handle(h); fail(RSR_EUNSUPPORTED); return nullptr; }
        h->P = ipow(h->base, k);
        h->nb = (rows + k - 1) / k;
        rc = preprocess_rsr(h, M, allow_narrow);
    }
    if (rc == RSR_OK && hipDeviceSynchronize() != hipSuccess) rc = RSR_EHIP;
    if (rc != RSR_OK) {
        (void)hipGetLastError();
        free_handle(h);
        fail(rc);
        return nullptr;
    }
    g_last_error = RSR_OK;
    return h;
}

hipError_t launch_any(rsr_handle_s *h, const void *v, int v_dtype, float *out) {
    return h->narrow ? rsr::launch_narrow_matvec(h, v, v_dtype, 1.0f, out, 1, h->cols, h->rows, 0)
                     : rsr::launch_rsr_matvec(h, v, v_dtype, 1.0f, out, 1, h->cols, h->rows, 0);
}

// Average duration in microseconds of the multiply kernel of h on zero vectors (null stream,
// device buffers supplied by the caller): both vector types, kTimed launches each; negative
// on failure.
float time_matvec(rsr_handle_s *h, const void *v, float *out) {
    hipEvent_t e0 = nullptr, e1 = nullptr;
    float ms = -1.0f;
    constexpr int kWarm = 5, kTimed = 60;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) goto done;
    for (int i = 0; i < kWarm; ++i)
        if (launch_any(h, v, i & 1 ? RSR_F32 : RSR_BF16, out) != hipSuccess) goto done;
    if (hipEventRecord(e0, 0) != hipSuccess) goto done;
    for (int i = 0; i < 2 * kTimed; ++i)
        if (launch_any(h, v, i & 1 ? RSR_F32 : RSR_BF16, out) != hipSuccess) goto done;
    if (hipEventRecord(e1, 0) != hipSuccess || hipEventSynchronize(e1) != hipSuccess) goto done;
    if (hipEventElapsedTime(&ms, e0, e1) != hipSuccess) ms = -1.0f;
done:
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    return ms < 0.0f ? -1.0f : ms * 1e3f / (2 * kTimed);
}

// k = 0: the block height is a tuning knob whose best value moves with the shape and the
// device (paper, Demonstration Scenarios: the best-k comparison across shapes and devices,
// and the k sweep of its interface), so it is chosen by measurement: preprocess with each
// candidate height (make(k) returns the handle or null), time the multiply kernel, keep the
// fastest handle.  padded_rows: an upper bound of the rows of any candidate handle.
template <typename Make>
rsr_handle_s *preprocess_auto_k(int kind, int64_t padded_rows, int64_t cols, Make make) {
    static const int fused_k[] = {4, 5, 6, 7, 8};
    static const int binary_k[] = {4, 6, 8, 10, 12};
    const int *cand = (kind == RSR_TERNARY_FUSED) ? fused_k : binary_k;
    float *v = nullptr;
    float *out = nullptr;
    rsr_handle_s *best = nullptr;
    float best_us = 0.0f;
    int last_err = RSR_EUNSUPPORTED;
    if (dev_alloc(&v, (size_t)cols) != hipSuccess || dev_alloc(&out, (size_t)padded_rows) != hipSuccess ||
        hipMemset(v, 0, (size_t)cols * 4) != hipSuccess) {
        (void)hipGetLastError();
        last_err = RSR_ENOMEM;
    } else {
        for (int i = 0; i < 5; ++i) {
            rsr_handle_s *h = make(cand[i]);
            if (!h) {
                if (g_last_error != RSR_EUNSUPPORTED) { last_err = g_last_error; break; }
                continue;
            }
            const float us = time_matvec(h, v, out);
            if (us >= 0.0f && (!best || us < best_us)) {
                if (best) free_handle(best);
                best = h;
                best_us = us;
            } else {
                free_handle(h);
            }
        }
        (void)hipDeviceSynchronize();
    }
    if (v) (void)hipFree(v);
    if (out) (void)hipFree(out);
    if (!best) { fail(last_err); return nullptr; }
    g_last_error = RSR_OK;
    return best;
}

// Sibling layers stacked row-wise, every layer completed with zero rows to a whole number
// of units (blocks of k rows / groups of 16 rows), so that no unit mixes two layers.
rsr_handle_s *preprocess_stacked_with_k(const int8_t *const *Ms, const int64_t *rows, int n, int64_t cols,
                                        int k, int kind) {
    const int64_t unit = (kind == RSR_DENSE_TERNARY_P2) ? rsr::kDenseRows : k;
    int64_t first[rsr::kMaxLayers + 1];
    first[0] = 0;
    for (int i = 0; i < n; ++i) first[i + 1] = first[i] + (rows[i] + unit - 1) / unit;
    const int64_t padded = first[n] * unit;
    int8_t *T = nullptr;
    if (dev_alloc(&T, (size_t)(padded * cols)) != hipSuccess) {
        (void)hipGetLastError();
        fail(RSR_ENOMEM);
        return nullptr;
    }
    hipError_t e = hipMemsetAsync(T, 0, (size_t)(padded * cols), 0);
    for (int i = 0; e == hipSuccess && i < n; ++i)
        e = hipMemcpyAsync(T + first[i] * unit * cols, Ms[i], (size_t)(rows[i] * cols),
                           hipMemcpyDeviceToDevice, 0);
    rsr_handle_s *h = nullptr;
    if (e != hipSuccess) {
        (void)hipGetLastError();
        fail(RSR_EHIP);
    } else {
        // (the narrow kernel writes one output vector: stacked handles take the general one)
        h = preprocess_with_k(T, padded, cols, k, kind, false);  // synchronises before returning
    }
    (void)hipFree(T);
    if (h) {
        h->nlayers = n;
        for (int i = 0; i < n; ++i) h->layer_rows[i] = rows[i];
        for (int i = 0; i <= n; ++i) h->layer_first[i] = first[i];
    }
    return h;
}

}  // namespace

extern "C" {

rsr_handle_t rsr_preprocess(const int8_t *M, int64_t rows, int64_t cols, int k, int kind) {
    if (!M || rows < 1 || cols < 1 || (!is_rsr_kind(kind) && kind != RSR_DENSE_TERNARY_P2)) {
        fail(RSR_EINVAL);
        return nullptr;
    }
    if (is_rsr_kind(kind) && k < 0) { fail(RSR_EINVAL); return nullptr; }
    if (cols > rsr::kMaxCols || rows > (int64_t)1 << 30) { fail(RSR_EUNSUPPORTED); return nullptr; }
    if (is_rsr_kind(kind) && k == 0)
        return preprocess_auto_k(kind, rows, cols,
                                 [&](int kk) { return preprocess_with_k(M, rows, cols, kk, kind); });
    return preprocess_with_k(M, rows, cols, k, kind);
}

rsr_handle_t rsr_preprocess_stacked(const int8_t *const *Ms, const int64_t *rows, int n, int64_t cols, int k,
                                    int kind) {
    if (!Ms || !rows || n < 1 || cols < 1 || (!is_rsr_kind(kind) && kind != RSR_DENSE_TERNARY_P2) ||
        (is_rsr_kind(kind) && k < 0)) {
        fail(RSR_EINVAL);
        return nullptr;
    }
    if (n > rsr::kMaxLayers || cols > rsr::kMaxCols) { fail(RSR_EUNSUPPORTED); return nullptr; }
    int64_t total = 0;
    for (int i = 0; i < n; ++i) {
        if (!Ms[i] || rows[i] < 1) { fail(RSR_EINVAL); return nullptr; }
        total += rows[i] + 16;
    }
    if (total > (int64_t)1 << 30) { fail(RSR_EUNSUPPORTED); return nullptr; }
    if (is_rsr_kind(kind) && k == 0)
        return preprocess_auto_k(kind, total, cols, [&](int kk) {
            return preprocess_stacked_with_k(Ms, rows, n, cols, kk, kind);
        });
    return preprocess_stacked_with_k(Ms, rows, n, cols, k, kind);
}

int rsr_num_layers(rsr_handle_t h) { return good(h) ? h->nlayers : 0; }

int rsr_matvec_stacked(rsr_handle_t h, const void *v, int v_dtype, const float *scales, void *const *outs,
                       void *stream) {
    if (!good(h) || h->nlayers < 1 || !v || !outs || (v_dtype != RSR_F32 && v_dtype != RSR_BF16))
        return fail(RSR_EINVAL);
    if (h->stale) return fail(RSR_EINVAL);
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess) return fail(RSR_EHIP);
    if (device != h->device) return fail(RSR_EINVAL);
    rsr::LayerTable lt;
    lt.n = h->nlayers;
    for (int i = 0; i < rsr::kMaxLayers; ++i) {
        const bool live = i < h->nlayers;
        if (live && !outs[i]) return fail(RSR_EINVAL);
        lt.out[i] = live ? static_cast<float *>(outs[i]) : nullptr;
        lt.scale[i] = live ? (scales ? scales[i] : 1.0f) : 0.0f;
        lt.rows[i] = live ? (int)h->layer_rows[i] : 0;
    }
    for (int i = 0; i <= rsr::kMaxLayers; ++i)
        lt.first[i] = (int)h->layer_first[i <= h->nlayers ? i : h->nlayers];
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    const hipError_t e = (h->kind == RSR_DENSE_TERNARY_P2)
                             ? rsr::launch_dense_matvec(h, v, v_dtype, 1.0f, nullptr, 1, h->cols, h->rows, s, &lt)
                             : rsr::launch_rsr_matvec(h, v, v_dtype, 1.0f, nullptr, 1, h->cols, h->rows, s, &lt);
    if (e != hipSuccess) return fail(hip_code(e));
    return RSR_OK;
}

rsr_handle_t rsr_preprocess_transposed(const int8_t *M, int64_t rows, int64_t cols, int k, int kind) {
    if (!M || rows < 1 || cols < 1) { fail(RSR_EINVAL); return nullptr; }
    if (rows > rsr::kMaxCols || cols > (int64_t)1 << 30) { fail(RSR_EUNSUPPORTED); return nullptr; }
    int8_t *T = nullptr;
    if (dev_alloc(&T, (size_t)(rows * cols)) != hipSuccess) {
        (void)hipGetLastError();
        fail(RSR_ENOMEM);
        return nullptr;
    }
    rsr_handle_t h = nullptr;
    if (rsr::launch_transpose(M, rows, cols, T) != hipSuccess) {
        (void)hipGetLastError();
        fail(RSR_EHIP);
    } else {
        h = rsr_preprocess(T, cols, rows, k, kind);  // synchronises before returning
    }
    (void)hipFree(T);
    return h;
}

int rsr_block_height(rsr_handle_t h) { return good(h) ? h->k : 0; }

}  // extern "C"

// ---- preprocessing without allocation ---------------------------------------------------
// The temporaries of rsr_preprocess_into live in this fixed array.  Each GPU holds its own
// copy at its own address; host code must go through the address hipGetSymbolAddress
// returns for the current device (kept per device below), never through the array's name.
namespace {

constexpr size_t kStaticScratchBytes = (size_t)RSR_INTO_SCRATCH_BYTES;
static __device__ __attribute__((used)) __align__(256) unsigned char scratch[kStaticScratchBytes];

std::atomic<unsigned char *> g_scratch_ptr[rsr::kMaxDevices];

// Address of the current device's copy of the scratch array (device must be current).
int static_scratch(int device, unsigned char **out) {
    if (device < 0 || device >= rsr::kMaxDevices) return RSR_EHIP;
    unsigned char *p = g_scratch_ptr[device].load(std::memory_order_acquire);
    if (!p) {
        void *sym = nullptr;
        if (hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)) != hipSuccess || !sym) {
            (void)hipGetLastError();
            return RSR_EHIP;
        }
        p = static_cast<unsigned char *>(sym);
        g_scratch_ptr[device].store(p, std::memory_order_release);  // same value from any thread
    }
    *out = p;
    return RSR_OK;
}

size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }

}  // namespace

extern "C" {

int rsr_preprocess_into(rsr_handle_t h, const int8_t *M) {
    if (!good(h) || !M) return fail(RSR_EINVAL);
    if (h->nlayers > 0) return fail(RSR_EUNSUPPORTED);
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess) return fail(RSR_EHIP);
    if (device != h->device) return fail(RSR_EINVAL);
    unsigned char *base = nullptr;
    if (int rc = static_scratch(device, &base)) return fail(rc);

    // carve the temporaries out of the fixed array; refuse what does not fit
    Temps t;
    size_t at = 0;
    t.flags = reinterpret_cast<int *>(base + at);
    at += align256(kFlagWords * sizeof(int));
    int rc;
    if (h->kind == RSR_DENSE_TERNARY_P2) {
        h->stale = true;
        rc = run_dense(h, M, t);
    } else {
        int64_t maxS = 0;
        for (int ps = 0; ps < h->npass; ++ps)
            if (h->pass[ps].S > maxS) maxS = h->pass[ps].S;
        t.code = reinterpret_cast<uint16_t *>(base + at);
        at += align256((size_t)(h->nb * h->cols) * sizeof(uint16_t));
        if (!h->narrow) {
            t.logical = reinterpret_cast<uint16_t *>(base + at);
            at += align256((size_t)(h->nb * maxS * rsr::kSlab) * sizeof(uint16_t));
        }
        if (h->by_rank) {
            t.gcode = reinterpret_cast<uint16_t *>(base + at);
            at += align256((size_t)(h->nb * h->slots) * sizeof(uint16_t));
        }
        if (at > kStaticScratchBytes) return fail(RSR_ESCRATCH);
        h->stale = true;  // from here on the handle's buffers are being rewritten
        StreamStats st;
        rc = run_sort_passes(h, M, t, &st);
        for (int ps = 0; rc == RSR_OK && ps < h->npass; ++ps) {
            // the new matrix has to fit the layout the handle was allocated for
            const int64_t need = h->by_rank ? st.real[ps] : st.with_empty[ps];
            if (h->narrow ? st.groups[ps] > h->slots
                          : (need > h->pass[ps].S * rsr::kSlab || (h->by_rank && st.groups[ps] + 1 > h->slots)))
                rc = RSR_EUNSUPPORTED;
        }
        if (rc == RSR_OK) rc = run_pack_passes(h, t);
    }
    if (rc == RSR_OK && hipDeviceSynchronize() != hipSuccess) rc = RSR_EHIP;
    if (rc != RSR_OK) {
        (void)hipGetLastError();
        return fail(rc);
    }
    h->stale = false;
    g_last_error = RSR_OK;
    return RSR_OK;
}


// ---- a handle as bytes --------------------------------------------------------------------
}  // extern "C"

namespace {

constexpr uint32_t kSerialMagic = 0x53525352u;  // "RSRS"
constexpr uint32_t kSerialVersion = 2;

struct SerialHeader {
    uint32_t magic, version;
    int32_t kind, k, base, npass, W, by_rank, enc, narrow;
    int64_t rows, cols, nb, P, row_bytes;
    int64_t S[2];
    int64_t slots;
    float sign[2];
    int64_t total_bytes;  // header + buffers
};

struct Piece {
    void **dev;      // the handle's device pointer
    size_t bytes;
};

// The device buffers of a handle in file order, with the sizes its geometry dictates.
std::vector<Piece> pieces_of(rsr_handle_s *h) {
    std::vector<Piece> p;
    if (h->kind == RSR_DENSE_TERNARY_P2) {
        const size_t groups = (size_t)((h->rows + rsr::kDenseRows - 1) / rsr::kDenseRows);
        p.push_back({reinterpret_cast<void **>(&h->packed), groups * rsr::kDenseRows * (size_t)h->row_bytes});
        return p;
    }
    for (int ps = 0; ps < h->npass; ++ps) {
        rsr::PassData &pd = h->pass[ps];
        p.push_back({reinterpret_cast<void **>(&pd.pi), (size_t)(h->nb * h->cols) * 2});
        p.push_back({reinterpret_cast<void **>(&pd.off), (size_t)(h->nb * (h->P + 1)) * 4});
        if (h->narrow) {
            p.push_back({reinterpret_cast<void **>(&pd.nent), (size_t)h->nb * 64 * 4});
            p.push_back({reinterpret_cast<void **>(&pd.nmeta), (size_t)h->nb * 64});
            p.push_back({&pd.nsw, (size_t)(h->nb * h->slots) * h->narrow_sw_bytes});
            continue;
        }
        p.push_back({reinterpret_cast<void **>(&pd.entries), (size_t)(h->nb * pd.S * rsr::kSlab) * 2});
        p.push_back({reinterpret_cast<void **>(&pd.start), (size_t)(h->nb * h->W * 64) * 2});
        p.push_back({&pd.sgn, sign_table_bytes(h)});
        if (h->by_rank) {
            p.push_back({reinterpret_cast<void **>(&pd.gword), (size_t)(h->nb * h->slots) * 4});
            p.push_back({reinterpret_cast<void **>(&pd.gcount), (size_t)h->nb * 4});
        }
    }
    if (!h->by_rank && !h->narrow) {
        p.push_back({reinterpret_cast<void **>(&h->fpack), (size_t)h->k * h->fold.G * 64 * 4});
        p.push_back({reinterpret_cast<void **>(&h->fshare), (size_t)h->W * 64 * 4});
    }
    return p;
}

}  // namespace

extern "C" {

int64_t rsr_serialized_size(rsr_handle_t h) {
    if (!good(h)) { fail(RSR_EINVAL); return -1; }
    if (h->nlayers > 0) { fail(RSR_EUNSUPPORTED); return -1; }
    int64_t total = (int64_t)sizeof(SerialHeader);
    for (const Piece &pc : pieces_of(h)) total += (int64_t)pc.bytes;
    return total;
}

int rsr_serialize(rsr_handle_t h, void *host_buf, int64_t capacity) {
    if (!good(h) || !host_buf) return fail(RSR_EINVAL);
    if (h->nlayers > 0) return fail(RSR_EUNSUPPORTED);
    const int64_t total = rsr_serialized_size(h);
    if (capacity < total) return fail(RSR_EINVAL);
    SerialHeader hd;
    std::memset(&hd, 0, sizeof(hd));
    hd.magic = kSerialMagic;
    hd.version = kSerialVersion;
    hd.kind = h->kind; hd.k = h->k; hd.base = h->base; hd.npass = h->npass;
    hd.W = h->W; hd.by_rank = h->by_rank; hd.enc = h->enc; hd.slots = h->slots; hd.narrow = h->narrow;
    hd.rows = h->rows; hd.cols = h->cols; hd.nb = h->nb; hd.P = h->P; hd.row_bytes = h->row_bytes;
    for (int ps = 0; ps < 2; ++ps) { hd.S[ps] = h->pass[ps].S; hd.sign[ps] = h->pass[ps].sign; }
    hd.total_bytes = total;
    unsigned char *out = static_cast<unsigned char *>(host_buf);
    std::memcpy(out, &hd, sizeof(hd));
    size_t at = sizeof(hd);
    for (const Piece &pc : pieces_of(h)) {
        if (hipMemcpy(out + at, *pc.dev, pc.bytes, hipMemcpyDeviceToHost) != hipSuccess) {
            (void)hipGetLastError();
            return fail(RSR_EHIP);
        }
        at += pc.bytes;
    }
    g_last_error = RSR_OK;
    return RSR_OK;
}

rsr_handle_t rsr_deserialize(const void *host_buf, int64_t size) {
    if (!host_buf || size < (int64_t)sizeof(SerialHeader)) { fail(RSR_EINVAL); return nullptr; }
    SerialHeader hd;
    std::memcpy(&hd, host_buf, sizeof(hd));
    if (hd.magic != kSerialMagic || hd.version != kSerialVersion || hd.total_bytes != size) {
        fail(RSR_EINVAL);
        return nullptr;
    }
    // the geometry has to be one rsr_preprocess could have produced
    const bool dense = hd.kind == RSR_DENSE_TERNARY_P2;
    bool ok = (dense || is_rsr_kind(hd.kind)) && hd.rows >= 1 && hd.rows <= (int64_t)1 << 30 &&
              hd.cols >= 1 && hd.cols <= rsr::kMaxCols;
    if (ok && dense) {
        const int64_t ntiles = (hd.cols + rsr::kDenseTileCols - 1) / rsr::kDenseTileCols;
        ok = hd.row_bytes == ntiles * (rsr::kDenseTileCols / 4);
    } else if (ok) {
        const bool fused = hd.kind == RSR_TERNARY_FUSED;
        ok = hd.k >= 1 && hd.k <= (fused ? 10 : 15) && hd.base == (fused ? 3 : 2) &&
             hd.npass == (hd.kind == RSR_TERNARY_2PASS ? 2 : 1) && (hd.narrow == 0 || hd.narrow == 1) &&
             hd.P == ipow(hd.base, hd.k) && hd.nb == (hd.rows + hd.k - 1) / hd.k;
        if (ok && hd.narrow) {
            // at most one group per column; the kernel reads sign words 4 at a time
            ok = hd.cols <= rsr::kNarrowCols && hd.k * (fused ? 2 : 1) <= 32 && hd.slots >= 4 &&
                 hd.slots <= 256 && hd.slots % 4 == 0;
        } else if (ok) {
            ok = hd.W >= 1 && hd.W <= rsr::kMaxWaves && (hd.by_rank == 0 || hd.by_rank == 1) &&
                 hd.enc == (hd.cols <= rsr::kSmallCols ? rsr::kEncSmall : rsr::kEncBig) &&
                 // slots: P by code; by rank at most one per column (every slot owns a tail
                 // entry), and the kernel addresses LDS with it, so it has to fit
                 (hd.by_rank ? (hd.slots >= 1 && hd.slots <= hd.cols + 1) : hd.slots == hd.P) &&
                 rsr::matvec_lds_bytes(hd.slots, hd.cols, 4, hd.W, hd.by_rank != 0) <= rsr::kLdsBytes;
            for (int ps = 0; ok && ps < hd.npass; ++ps)
                ok = hd.S[ps] >= 1 && hd.S[ps] * rsr::kSlab <= hd.cols + hd.P + rsr::kSlab;
        }
    }
    if (!ok) { fail(RSR_EINVAL); return nullptr; }

    rsr_handle_s *h = new (std::nothrow) rsr_handle_s();
    if (!h) { fail(RSR_ENOMEM); return nullptr; }
    h->magic = rsr::kMagic;
    h->kind = hd.kind; h->k = hd.k; h->base = hd.base; h->npass = hd.npass;
    h->W = hd.W; h->by_rank = hd.by_rank; h->enc = hd.enc; h->slots = hd.slots; h->narrow = hd.narrow;
    if (h->narrow) {
        h->narrow_fw = h->base == 2 ? 1 : 2;
        h->narrow_sw_bytes = h->k * h->narrow_fw <= 8 ? 1 : h->k * h->narrow_fw <= 16 ? 2 : 4;
    }
    h->rows = hd.rows; h->cols = hd.cols; h->nb = hd.nb; h->P = hd.P; h->row_bytes = hd.row_bytes;
    for (int ps = 0; ps < 2; ++ps) { h->pass[ps].S = hd.S[ps]; h->pass[ps].sign = hd.sign[ps]; }
    if (!dense && !h->by_rank && !h->narrow) rsr::make_fold_shape(h->base, h->k, h->P, h->W, &h->fold);
    int rc = RSR_OK;
    if (hipGetDevice(&h->device) != hipSuccess) rc = RSR_EHIP;
    const std::vector<Piece> pieces = pieces_of(h);
    int64_t need = (int64_t)sizeof(SerialHeader);
    for (const Piece &pc : pieces) need += (int64_t)pc.bytes;
    if (rc == RSR_OK && need != size) rc = RSR_EINVAL;
    const unsigned char *in = static_cast<const unsigned char *>(host_buf);
    size_t at = sizeof(SerialHeader);
    for (size_t i = 0; rc == RSR_OK && i < pieces.size(); ++i) {
        hipError_t e = hipMalloc(pieces[i].dev, pieces[i].bytes ? pieces[i].bytes : 1);
        if (e == hipSuccess) e = hipMemcpy(*pieces[i].dev, in + at, pieces[i].bytes, hipMemcpyHostToDevice);
        if (e != hipSuccess) rc = hip_code(e);
        at += pieces[i].bytes;
    }
    if (rc != RSR_OK) {
        (void)hipGetLastError();
        free_handle(h);
        fail(rc);
        return nullptr;
    }
    g_last_error = RSR_OK;
    return h;
}

int rsr_matvec_ex(rsr_handle_t h, const void *v, int v_dtype, float scale, void *out, int batch,
                  int64_t ldv, int64_t ldo, void *stream) {
    if (!good(h) || !v || !out || batch < 1 || (v_dtype != RSR_F32 && v_dtype != RSR_BF16))
        return fail(RSR_EINVAL);
    if (h->stale) return fail(RSR_EINVAL);  // a failed rsr_preprocess_into left it half-written
    if (h->nlayers > 0) return fail(RSR_EINVAL);  // stacked handles multiply through rsr_matvec_stacked
    if (batch > 65535) return fail(RSR_EUNSUPPORTED);
    if (batch > 1 && (ldv < h->cols || ldo < h->rows)) return fail(RSR_EINVAL);
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess) return fail(RSR_EHIP);
    if (device != h->device) return fail(RSR_EINVAL);  // the handle's buffers live on another GPU
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    hipError_t e = (h->kind == RSR_DENSE_TERNARY_P2)
                       ? rsr::launch_dense_matvec(h, v, v_dtype, scale, static_cast<float *>(out),
                                                  batch, ldv, ldo, s)
                   : h->narrow
                       ? rsr::launch_narrow_matvec(h, v, v_dtype, scale, static_cast<float *>(out), batch, ldv,
                                                   ldo, s)
                       : rsr::launch_rsr_matvec(h, v, v_dtype, scale, static_cast<float *>(out),
                                                batch, ldv, ldo, s);
    if (e != hipSuccess) return fail(hip_code(e));
    return RSR_OK;
}

int rsr_probe_empty(int workgroups, int threads, int lds_bytes, void *stream) {
    if (workgroups < 1 || threads < 64 || threads > 1024 || threads % 64 || lds_bytes < 0 ||
        lds_bytes > rsr::kLdsBytes)
        return fail(RSR_EINVAL);
    const hipError_t e = rsr::launch_probe_empty(workgroups, threads, lds_bytes,
                                                 reinterpret_cast<hipStream_t>(stream));
    return e == hipSuccess ? RSR_OK : fail(hip_code(e));
}

int rsr_probe_read(const void *src, int64_t bytes, int workgroups, int threads, void *sink, void *stream) {
    if (!src || bytes < 1024 || workgroups < 1 || threads < 64 || threads > 1024 || threads % 64)
        return fail(RSR_EINVAL);
    const hipError_t e = rsr::launch_probe_read(src, bytes, workgroups, threads, sink,
                                                reinterpret_cast<hipStream_t>(stream));
    return e == hipSuccess ? RSR_OK : fail(hip_code(e));
}

int rsr_launch_shape(rsr_handle_t h, int v_dtype, int *workgroups, int *threads, int *lds_bytes) {
    if (!good(h) || !is_rsr_kind(h->kind) || (v_dtype != RSR_F32 && v_dtype != RSR_BF16))
        return fail(RSR_EINVAL);
    if (h->narrow) return fail(RSR_EUNSUPPORTED);
    if (workgroups) *workgroups = (int)h->nb;
    if (threads) *threads = h->W * 64;
    if (lds_bytes)
        *lds_bytes = (int)rsr::matvec_lds_bytes(h->slots, h->cols, v_dtype == RSR_BF16 ? 2 : 4, h->W,
                                                h->by_rank != 0);
    return RSR_OK;
}

int rsr_matvec(rsr_handle_t h, const void *v, void *out, void *stream) {
    if (!good(h)) return fail(RSR_EINVAL);
    return rsr_matvec_ex(h, v, RSR_F32, 1.0f, out, 1, h->cols, h->rows, stream);
}

void rsr_destroy(rsr_handle_t h) {
    if (good(h)) free_handle(h);
}

int rsr_last_error(void) { return g_last_error; }

const char *rsr_error_string(int code) {
    switch (code) {
        case RSR_OK: return "ok";
        case RSR_EINVAL: return "invalid argument";
        case RSR_EVALUE: return "matrix entry outside the alphabet of the kind";
        case RSR_EUNSUPPORTED: return "request outside the supported limits";
        case RSR_ENOMEM: return "out of memory";
        case RSR_EHIP: return "HIP runtime error";
        case RSR_EINTERNAL: return "preprocessing self-check failed";
        case RSR_ESCRATCH: return "input needs more temporary memory than the fixed scratch of rsr_preprocess_into";
        default: return "unknown error";
    }
}

int rsr_get_perm(rsr_handle_t h, int pass, uint32_t *host_pi) {
    if (!good(h) || !host_pi || !is_rsr_kind(h->kind) || pass < 0 || pass >= h->npass)
        return fail(RSR_EINVAL);
    const size_t n = (size_t)(h->nb * h->cols);
    std::vector<uint16_t> tmp(n);
    if (hipMemcpy(tmp.data(), h->pass[pass].pi, n * sizeof(uint16_t), hipMemcpyDeviceToHost) !=
        hipSuccess)
        return fail(RSR_EHIP);
    for (size_t i = 0; i < n; ++i) host_pi[i] = tmp[i];
    return RSR_OK;
}

int rsr_get_offsets(rsr_handle_t h, int pass, uint32_t *host_off) {
    if (!good(h) || !host_off || !is_rsr_kind(h->kind) || pass < 0 || pass >= h->npass)
        return fail(RSR_EINVAL);
    const size_t n = (size_t)(h->nb * (h->P + 1));
    if (hipMemcpy(host_off, h->pass[pass].off, n * sizeof(uint32_t), hipMemcpyDeviceToHost) !=
        hipSuccess)
        return fail(RSR_EHIP);
    return RSR_OK;
}

int rsr_get_packed(rsr_handle_t h, uint8_t *host_packed) {
    if (!good(h) || !host_packed || h->kind != RSR_DENSE_TERNARY_P2) return fail(RSR_EINVAL);
    const int64_t ntiles = h->row_bytes / (rsr::kDenseTileCols / 4);
    const int64_t ngroups = (h->rows + rsr::kDenseRows - 1) / rsr::kDenseRows;
    const size_t words = (size_t)(ngroups * ntiles * 256);
    std::vector<uint32_t> tiled(words);
    if (hipMemcpy(tiled.data(), h->packed, words * 4, hipMemcpyDeviceToHost) != hipSuccess)
        return fail(RSR_EHIP);
    // undo the kernel tiling: pure data movement of 2-bit fields
    const int64_t rb = (h->cols + 3) / 4;
    for (int64_t i = 0; i < h->rows * rb; ++i) host_packed[i] = 0;
    for (int64_t i = 0; i < h->rows; ++i) {
        const int64_t G = i / rsr::kDenseRows, rr = i % rsr::kDenseRows;
        for (int64_t j = 0; j < h->cols; ++j) {
            const int64_t t = j / rsr::kDenseTileCols, jj = j % rsr::kDenseTileCols;
            const int64_t step = jj / 32, kq = (jj % 32) / 8, e = jj % 8;
            const int64_t d = step / 2, p = (step % 2) * 4 + e / 2;
            const int shift = (int)(((e & 1) ? 30 : 14) - 2 * p);
            const uint32_t word = tiled[(size_t)(((G * ntiles + t) * 64 + (rr + 16 * kq)) * 4 + d)];
            const uint32_t two = (word >> shift) & 3u;
            host_packed[i * rb + j / 4] |= (uint8_t)(two << (2 * (j % 4)));
        }
    }
    return RSR_OK;
}

int64_t rsr_num_blocks(rsr_handle_t h) { return good(h) ? h->nb : 0; }
int64_t rsr_num_patterns(rsr_handle_t h) { return good(h) ? h->P : 0; }
int rsr_num_passes(rsr_handle_t h) { return good(h) ? h->npass : 0; }

int64_t rsr_algorithmic_bytes(rsr_handle_t h, int v_dtype, int batch) {
    if (!good(h) || batch < 1 || (v_dtype != RSR_F32 && v_dtype != RSR_BF16)) {
        fail(RSR_EINVAL);
        return -1;
    }
    const int64_t vb = (v_dtype == RSR_BF16) ? 2 : 4;
    int64_t weight_side;
    if (h->kind == RSR_DENSE_TERNARY_P2) {
        weight_side = (h->rows + rsr::kDenseRows - 1) / rsr::kDenseRows * rsr::kDenseRows * h->row_bytes;
    } else {
        weight_side = 0;
        for (int ps = 0; h->narrow && ps < h->npass; ++ps)
            weight_side += h->nb * (64 * 4 + 64 + h->slots * h->narrow_sw_bytes);
        for (int ps = 0; !h->narrow && ps < h->npass; ++ps)
            weight_side += h->nb * (h->pass[ps].S * (int64_t)rsr::kSlab * 2 + (int64_t)h->W * 64 * 2 +
                                    (h->by_rank ? h->slots * 4 + 4 : 0)) +
                           (int64_t)sign_table_bytes(h);
        if (!h->by_rank && !h->narrow) weight_side += (int64_t)h->k * h->fold.G * 256 + (int64_t)h->W * 64 * 4;
    }
    return weight_side + (int64_t)batch * (h->cols * vb + h->rows * 4);
}

const char *rsr_kernel_name(rsr_handle_t h, int v_dtype) {
    if (!good(h) || (v_dtype != RSR_F32 && v_dtype != RSR_BF16)) {
        fail(RSR_EINVAL);
        return nullptr;
    }
    if (h->kind == RSR_DENSE_TERNARY_P2) return rsr::dense_matvec_kernel_name(h, v_dtype);
    if (h->narrow) return v_dtype == RSR_BF16 ? "k_rsr_narrow<unsigned short>" : "k_rsr_narrow<float>";
    static thread_local char name[96];
    rsr::rsr_matvec_kernel_name(h, v_dtype, name, sizeof(name));
    return name;
}

}  // extern "C"
