// C ABI of the sparse-FFN hot path (see include/lif.h for the contract of every call).
// Host side only: argument checks, launch geometry, call-order bookkeeping, event timing.
#include "../../include/lif.h"

#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstring>
#include <new>
#include <type_traits>
#include <vector>

#include "lif_common.h"
#include "lif_ffn.h"
#include "lif_ffn_mfma.h"
#include "lif_ffn_down_mfma.h"
#include "lif_predict.h"
#include "lif_step.h"
#include "lif_window.h"

using namespace lif;

// Scratch of lif_sparse_ffn_static: activations and partial outputs of one FFN call.  One copy per GPU, at its own
// address on each; host code reaches it only through the pointer hipGetSymbolAddress returns for the current device.
constexpr size_t kStaticScratchBytes = 5u << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, const char* detail = "") {
    snprintf(g_err, sizeof(g_err), fmt, detail);
    return code;
}

#define LIF_HIP(call)                                                             \
    do {                                                                          \
        hipError_t e_ = (call);                                                   \
        if (e_ != hipSuccess) return fail(LIF_HIP_ERROR, #call ": %s", hipGetErrorString(e_)); \
    } while (0)

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct Layout {
    size_t state, ring, tpart, move_dst, hole_list, h, ypart, h_new, stamp, gact, total;
};

int elem_bytes(const lif_config& c) { return c.dtype == LIF_F32 ? 4 : 2; }
int vec_elems(const lif_config& c) { return 16 / elem_bytes(c); }
int ring_words(const lif_config& c) { return (c.d_ffn + 63) / 64; }

bool config_ok(const lif_config* c, const char** why) {
    *why = "";
    if (!c) return (*why = "null config", false);
    if (c->dtype != LIF_F32 && c->dtype != LIF_F16) return (*why = "dtype", false);
    const int ve = vec_elems(*c);
    if (c->d_model <= 0 || c->d_model % ve) return (*why = "d_model must be a positive multiple of 16 bytes", false);
    if ((c->d_model / ve + 63) / 64 > 16) return (*why = "d_model too large (at most 1024 16-byte vectors)", false);
    if (c->d_ffn <= 0 || c->d_ffn % 8 || c->d_ffn > kScanThreads * kMaxSpan) return (*why = "d_ffn must be a multiple of 8, at most 65536", false);
    if (c->predictor != LIF_PRED_GATE &&
        (c->rank <= 0 || c->rank % ve || c->rank > 2048)) return (*why = "rank", false);
    if (c->window_k < 1 || c->window_k > 256) return (*why = "window_k must be in 1..256", false);
    if (c->capacity_rows < 1 || c->capacity_rows > kScanThreads * kMaxSpan) return (*why = "capacity_rows must be in 1..65536", false);
    if (c->max_batch < 1 || c->max_batch > 8) return (*why = "max_batch must be in 1..8", false);
    if (c->glu != 0 && c->glu != 1) return (*why = "glu", false);
    if (c->shrink_window != 0 && c->shrink_window != 1) return (*why = "shrink_window", false);
    if (c->predictor != LIF_PRED_LOWRANK && c->predictor != LIF_PRED_GATE) return (*why = "predictor", false);
    if (c->predictor == LIF_PRED_GATE && c->glu)
        return (*why = "the gate predictor takes plain (up | down) bundles", false);
    if (c->ffn_mode != LIF_FFN_SKIP_DEAD && c->ffn_mode != LIF_FFN_FULL_BUNDLE) return (*why = "ffn_mode", false);
    if ((size_t)c->max_batch * c->d_model * elem_bytes(*c) > 64 * 1024) return (*why = "max_batch * d_model exceeds the 64 KiB LDS staging area", false);
    return true;
}

Layout make_layout(const lif_config& c) {
    Layout L;
    size_t off = 0;
    L.state = off;
    off = align_up(off + sizeof(DevState), 256);
    L.ring = off;                      // window_k step masks, each padded to whole 64-bit words
    off = off + (size_t)c.window_k * ring_words(c) * 8;     // ... directly followed by the bitmap of the cached set
    off = align_up(off + (size_t)ring_words(c) * 8, 256);
    L.tpart = off;
    off = align_up(off + sizeof(double) * c.max_batch * std::max(c.rank, 0), 256);
    L.move_dst = off;
    off = align_up(off + sizeof(int32_t) * c.capacity_rows, 256);
    L.hole_list = off;
    off = align_up(off + sizeof(int32_t) * c.capacity_rows, 256);
    L.h = off;
    off = align_up(off + sizeof(float) * c.max_batch * c.capacity_rows, 256);
    L.ypart = off;                     // per-chunk partial outputs of the down projection
    off = align_up(off + sizeof(float) * kDownChunksMax * c.max_batch * c.d_model, 256);
    L.h_new = off;                     // activations written by the fused load kernel (single-token steps)
    off = align_up(off + sizeof(float) * c.capacity_rows, 256);
    L.stamp = off;                     // step number at which h_new[slot] was written
    off = align_up(off + sizeof(int32_t) * c.capacity_rows, 256);
    L.gact = off;                      // gate predictor: relu(gate_i . x_t + b_i) per token and original neuron
    off = align_up(off + (c.predictor == LIF_PRED_GATE ? sizeof(float) * c.max_batch * c.d_ffn : 0), 256);
    L.total = off;
    return L;
}

}  // namespace

struct lif_layer {
    lif_config cfg;
    lif_buffers buf;
    Layout lay;
    HostStore host;             // device-visible addresses of the pinned bundle store (bundled or in two parts)
    int loader_pairs;           // loader wave pairs of the fused step, 0 = chosen from the bundle size
    DevState* st;
    unsigned long long* ring;
    double* tpart;
    int32_t* move_dst;
    int32_t* hole_list;
    float* h;
    float* ypart;
    float* h_new;
    int32_t* stamp;
    float* gact;                // null unless the gate projection is the predictor
    size_t row_elems, row_bytes;
    bool window_pending;
    int expected_rows;          // hint, 0 = none
    int mask_bt[9];             // tokens per pass of the mask kernel for a batch of b tokens (1, 4 or 8)
    unsigned char* static_scratch;  // this device's copy of the library's static scratch array (null: lookup failed)
    // event timing
    bool prof_on;
    int prof_max;
    std::vector<hipEvent_t> ev;     // 2 per timed launch
    std::vector<int> ev_kernel;
};

namespace {

struct Timed {
    lif_layer* L;
    hipStream_t s;
    int slot;
    Timed(lif_layer* layer, int kid, hipStream_t stream) : L(layer), s(stream), slot(-1) {
        if (L->prof_on && (int)L->ev_kernel.size() < L->prof_max) {
            slot = (int)L->ev_kernel.size();
            L->ev_kernel.push_back(kid);
            (void)hipEventRecord(L->ev[2 * slot], s);
        }
    }
    ~Timed() {
        if (slot >= 0) (void)hipEventRecord(L->ev[2 * slot + 1], s);
    }
};

template <typename T>
int launch_predict(lif_layer* L, const void* x, int batch, uint8_t* masks, uint8_t* step_mask, hipStream_t s) {
    const lif_config& c = L->cfg;
    {
        Timed t(L, LIF_K_PREDICT_XA, s);
        const int ni = (c.d_model / Vec<T>::N + 63) / 64;
#define LIF_XA(NI)                                                                                          \
    hipLaunchKernelGGL((k_predict_xa<T, NI>), dim3((c.rank + 3) / 4, batch), dim3(256), 0, s, (const T*)x,       \
                       (const T*)L->buf.A, L->tpart, c.d_model, c.rank, L->st)
        if (ni <= 1) LIF_XA(1);
        else if (ni <= 2) LIF_XA(2);
        else if (ni <= 4) LIF_XA(4);
        else if (ni <= 8) LIF_XA(8);
        else if (ni <= 9) LIF_XA(9);
        else if (ni <= 12) LIF_XA(12);
        else LIF_XA(16);
#undef LIF_XA
    }
    const int grid = (c.d_ffn + kMaskCols * 8 - 1) / (kMaskCols * 8);
    Timed t(L, LIF_K_PREDICT_MASK, s);
#define LIF_MASK(BT)                                                                                        \
    hipLaunchKernelGGL((k_predict_mask<T, BT>), dim3(grid), dim3(256), sizeof(double) * BT * c.rank, s,          \
                       (const T*)L->buf.B, L->buf.c, L->tpart, c.rank, c.d_ffn, batch, c.threshold, masks,         \
                       step_mask, L->st)
    // tokens per pass over B: chosen at lif_create so that t of those tokens and the kernel's own LDS fit a workgroup
    const int bt = L->mask_bt[batch];
    if (bt == 1) LIF_MASK(1);
    else if (bt == 4) LIF_MASK(4);
    else LIF_MASK(8);
#undef LIF_MASK
    return LIF_OK;
}

template <typename T>
void launch_predict_gate(lif_layer* L, const void* x, int batch, uint8_t* masks, uint8_t* step_mask, hipStream_t s) {
    const lif_config& c = L->cfg;
    const int nvec = c.d_model / Vec<T>::N;
    const int ni = (nvec + 63) / 64;
    const int grid = std::min((c.d_ffn / 8 + 3) / 4, 2048);
    const size_t shm = batch == 1 ? 0 : (size_t)batch * c.d_model * sizeof(T);
    Timed t(L, LIF_K_PREDICT_MASK, s);
#define LIF_PG_X(NI, XREG)                                                                                   \
    hipLaunchKernelGGL((k_predict_gate<T, NI, XREG>), dim3(grid), dim3(256), shm, s, (const T*)L->buf.A,         \
                       L->buf.b, (const T*)x, c.d_model, c.d_ffn, batch, c.threshold, masks, step_mask, L->gact, \
                       L->st)
#define LIF_PG(NI) do { if (batch == 1) LIF_PG_X(NI, true); else LIF_PG_X(NI, false); } while (0)
    if (ni <= 1) LIF_PG(1);
    else if (ni <= 2) LIF_PG(2);
    else if (ni <= 4) LIF_PG(4);
    else if (ni <= 8) LIF_PG(8);
    else if (ni <= 9) LIF_PG(9);
    else if (ni <= 12) LIF_PG(12);
    else LIF_PG(16);
#undef LIF_PG
#undef LIF_PG_X
}

// `h` (activations) and `ypart` (partial outputs) of the FFN launches: the workspace arrays of the layer, or the
// library's static scratch (lif_sparse_ffn_static)
template <typename T, bool GLU>
void launch_ffn_up(lif_layer* L, const void* x, int batch, float* h, hipStream_t s) {
    const lif_config& c = L->cfg;
    const int nvec = c.d_model / Vec<T>::N;
    const int ni = (nvec + 63) / 64;
    // one wave per row; with a row-count hint the grid is sized to it and the first pass is speculative
    const int spec = L->expected_rows > 0 ? 1 : 0;
    const int grid = spec ? std::min(kUpMaxWgs, std::max(1, std::min(L->expected_rows, c.capacity_rows) / 4))
                          : std::min((c.capacity_rows + 3) / 4, 512);
    const size_t shm = batch == 1 ? 0 : (size_t)batch * c.d_model * sizeof(T);
#define LIF_UP_X(NI, XREG)                                                                                   \
    hipLaunchKernelGGL((k_ffn_up<T, NI, GLU, XREG>), dim3(grid), dim3(256), shm, s, (const T*)L->buf.matrix,    \
                       L->buf.bias, (const T*)x, h, c.d_model, batch, c.capacity_rows, L->row_elems, spec,        \
                       L->buf.pointers, L->gact, c.d_ffn, L->st)
#define LIF_UP(NI) do { if (batch == 1) LIF_UP_X(NI, true); else LIF_UP_X(NI, false); } while (0)
    if (ni <= 1) LIF_UP(1);
    else if (ni <= 2) LIF_UP(2);
    else if (ni <= 4) LIF_UP(4);
    else if (ni <= 6) LIF_UP(6);
    else if (ni <= 8) LIF_UP(8);
    else if (ni <= 9) LIF_UP(9);
    else if (ni <= 12) LIF_UP(12);
    else LIF_UP(16);
#undef LIF_UP
#undef LIF_UP_X
}

template <typename T, int BT, bool SKIP, int LANES>
void launch_ffn_down_as(lif_layer* L, int batch, void* y, float* h, float* ypart, hipStream_t s, bool use_new) {
    const lif_config& c = L->cfg;
    const int cols = LANES * Vec<T>::N;
    int slices = (c.d_model + cols - 1) / cols;
    if (LANES * 16 < 128) slices = (slices + kXcds - 1) / kXcds * kXcds;      // whole runs of slices per XCD
    // workgroup rows: enough for the chunks of the expected number of rows (with some slack), else of the
    // capacity; fewer than the chunks in use is still correct (a workgroup row then takes several chunks)
    const int rows_hint = L->expected_rows > 0 ? std::min(c.capacity_rows, L->expected_rows + L->expected_rows / 8)
                                               : c.capacity_rows;
    const int wg_rows = down_chunks<BT, SKIP>(rows_hint);
    const int down_off = (c.glu ? 2 : 1) * c.d_model;
    // one token: groups of 256 slots whose activations the first workgroup row asks for before the row count arrives
    // (from the hint; 2048 slots without one); several tokens: all of the first pass
    const int spec_groups = BT > 1 ? (1 << 20) : L->expected_rows > 0 ? std::max(1, (rows_hint + 255) / 256) : 8;
    // one token: compaction passes of 4096 slots when more than 2048 rows are expected (one pass instead of two;
    // the sums are the same), of 2048 otherwise (half the registers and guards on the shortest path)
    if (BT == 1 && L->expected_rows > 0 && rows_hint > kDownTile)
        hipLaunchKernelGGL((k_ffn_down<T, BT, SKIP, LANES, 2 * kDownTile>), dim3(slices, wg_rows), dim3(256), 0, s,
                           (const T*)L->buf.matrix, h, use_new ? L->h_new : nullptr, use_new ? L->stamp : nullptr,
                           (T*)y, ypart, c.d_model, batch, c.capacity_rows, L->row_elems, down_off, spec_groups, L->st);
    else
        hipLaunchKernelGGL((k_ffn_down<T, BT, SKIP, LANES>), dim3(slices, wg_rows), dim3(256), 0, s,
                           (const T*)L->buf.matrix, h, use_new ? L->h_new : nullptr, use_new ? L->stamp : nullptr,
                           (T*)y, ypart, c.d_model, batch, c.capacity_rows, L->row_elems, down_off, spec_groups, L->st);
    if (wg_rows > 1)
        hipLaunchKernelGGL((k_ffn_down_finish<T, BT, SKIP>), dim3((batch * c.d_model + 255) / 256), dim3(256), 0, s,
                           ypart, (T*)y, c.d_model, batch, L->st);
}

// several tokens, fp16: the down projection on the matrix cores
template <bool SKIP>
void launch_ffn_down_mfma(lif_layer* L, int batch, void* y, float* h, float* ypart, hipStream_t s) {
    const lif_config& c = L->cfg;
    const int slices = (c.d_model + kDmCols - 1) / kDmCols;
    const int chunk_rows = down_mfma_chunk_rows(c.capacity_rows);
    // workgroup rows: enough for the chunks of the expected number of rows (with some slack), else of the
    // capacity; fewer than the chunks in use is still correct (a workgroup row then takes several chunks)
    const int rows_hint = L->expected_rows > 0 ? std::min(c.capacity_rows, L->expected_rows + L->expected_rows / 8)
                                               : c.capacity_rows;
    const int wg_rows = down_mfma_chunks(rows_hint, chunk_rows);
    const int down_off = (c.glu ? 2 : 1) * c.d_model;
    hipLaunchKernelGGL((k_ffn_down_mfma<SKIP, kDmWaves>), dim3(slices, wg_rows), dim3(kDmWaves * 64), 0, s,
                       (const _Float16*)L->buf.matrix, h, (_Float16*)y, ypart, c.d_model, batch, c.capacity_rows,
                       L->row_elems, down_off, chunk_rows, L->st);
    if (wg_rows > 1)
        hipLaunchKernelGGL(k_ffn_down_mfma_finish, dim3((batch * c.d_model + 255) / 256), dim3(256), 0, s, ypart,
                           (_Float16*)y, c.d_model, batch, chunk_rows, L->st);
}

template <typename T>
void launch_ffn_down(lif_layer* L, int batch, void* y, float* h, float* ypart, hipStream_t s, bool use_new = false) {
    const bool skip = L->cfg.ffn_mode == LIF_FFN_SKIP_DEAD;
    if constexpr (std::is_same<T, _Float16>::value) {
        if (batch > 1) {
            if (skip) launch_ffn_down_mfma<true>(L, batch, y, h, ypart, s);
            else launch_ffn_down_mfma<false>(L, batch, y, h, ypart, s);
            return;
        }
    }
    if (batch == 1) {
        if (skip) launch_ffn_down_as<T, 1, true, kDownLanes1>(L, batch, y, h, ypart, s, use_new);
        else launch_ffn_down_as<T, 1, false, kDownLanesN>(L, batch, y, h, ypart, s, use_new);
    } else if (batch <= 4) {
        if (skip) launch_ffn_down_as<T, 4, true, kDownLanesB>(L, batch, y, h, ypart, s, use_new);
        else launch_ffn_down_as<T, 4, false, kDownLanesB>(L, batch, y, h, ypart, s, use_new);
    } else {
        if (skip) launch_ffn_down_as<T, 8, true, kDownLanesB>(L, batch, y, h, ypart, s, use_new);
        else launch_ffn_down_as<T, 8, false, kDownLanesB>(L, batch, y, h, ypart, s, use_new);
    }
}

template <typename T, bool GLU>
void launch_load_up(lif_layer* L, const void* x, const int32_t* added, hipStream_t s) {
    const lif_config& c = L->cfg;
    const int nvec = c.d_model / Vec<T>::N;
    const int ni = (nvec + 63) / 64;
    const int spec = L->expected_rows > 0 ? 1 : 0;
    const int up_blocks = spec ? std::min(kUpMaxWgs, std::max(1, std::min(L->expected_rows, c.capacity_rows) / 4))
                               : std::min((c.capacity_rows + 3) / 4, 512);
    // loader waves come in pairs (activation vectors | down vector of one bundle), one wave per workgroup
    const int load_wgs = 2 * (L->loader_pairs > 0 ? L->loader_pairs
                                                   : (int)std::min<size_t>(32, std::max<size_t>(5, kStepInflightBytes / L->row_bytes)));
#define LIF_LU(NI)                                                                                            \
    hipLaunchKernelGGL((k_load_up<T, NI, GLU>), dim3(load_wgs + up_blocks), dim3(256), 0, s,                      \
                       (T*)L->buf.matrix, L->buf.pointers, L->buf.bias, L->host, L->buf.b, added, \
                       L->move_dst, L->row_elems, c.d_ffn, c.d_model, c.capacity_rows, (const T*)x, L->h,         \
                       L->h_new, L->stamp, spec, load_wgs, L->gact, L->st)
    if (ni <= 1) LIF_LU(1);
    else if (ni <= 2) LIF_LU(2);
    else if (ni <= 4) LIF_LU(4);
    else if (ni <= 6) LIF_LU(6);
    else if (ni <= 8) LIF_LU(8);
    else if (ni <= 9) LIF_LU(9);
    else if (ni <= 12) LIF_LU(12);
    else LIF_LU(16);
#undef LIF_LU
}

constexpr int kFuseBatchedMinRows = 2048;

bool mfma_path(const lif_config& c, int batch) {
    return c.dtype == LIF_F16 && batch > 1 && c.d_model % 32 == 0;
}

// 16-row tiles a row-count hint covers (at least one, at most all)
int mfma_hint_tiles(const lif_layer* L) {
    const int tiles = (L->cfg.capacity_rows + 15) / 16;
    return std::max(1, std::min(tiles, (L->expected_rows + 15) / 16));
}

template <int MODE>
void launch_ffn_up_mfma(lif_layer* L, const void* x, int batch, float* h, hipStream_t s) {
    const lif_config& c = L->cfg;
    constexpr int W = (MODE == kRowsChanged) ? kMfmaWavesFix : kMfmaWavesAll;
    // the rows a load wrote are few: a small grid strides over their tiles
    const int tiles = (c.capacity_rows + 15) / 16;
    // all rows: with a row-count hint the grid is sized to it (a workgroup strides on if more rows are in use)
    // and every workgroup asks for its first rows before the count arrives
    const int spec = (MODE == kRowsAll && L->expected_rows > 0) ? 1 : 0;
    const int grid = (MODE == kRowsChanged) ? std::min(tiles, 64) : spec ? mfma_hint_tiles(L) : tiles;
    if (c.glu)
        hipLaunchKernelGGL((k_ffn_up_mfma<true, MODE, W>), dim3(grid), dim3(W * 64), 0, s,
                           (const _Float16*)L->buf.matrix, L->buf.bias, (const _Float16*)x, h, c.d_model, batch,
                           c.capacity_rows, L->row_elems, L->move_dst, L->buf.pointers, L->gact, c.d_ffn, spec, L->st);
    else
        hipLaunchKernelGGL((k_ffn_up_mfma<false, MODE, W>), dim3(grid), dim3(W * 64), 0, s,
                           (const _Float16*)L->buf.matrix, L->buf.bias, (const _Float16*)x, h, c.d_model, batch,
                           c.capacity_rows, L->row_elems, L->move_dst, L->buf.pointers, L->gact, c.d_ffn, spec, L->st);
}

// batch > 1, fp16: bundle load next to the activation stage of the surviving rows, then the rows the load wrote
void launch_load_up_mfma(lif_layer* L, const void* x, int batch, const int32_t* added, hipStream_t s) {
    const lif_config& c = L->cfg;
    const int tiles = (c.capacity_rows + 15) / 16;
    static_assert(kMfmaWaves == 4, "the fused kernel runs both roles with 256 threads");
    const int spec_tiles = L->expected_rows > 0 ? mfma_hint_tiles(L) : 0;
    if (c.glu)
        hipLaunchKernelGGL((k_load_up_mfma<true>), dim3(kLoadGrid + tiles), dim3(256), 0, s, (_Float16*)L->buf.matrix,
                           L->buf.pointers, L->buf.bias, L->host, L->buf.b, added, L->move_dst, L->row_bytes,
                           c.d_ffn, (const _Float16*)x, L->h, c.d_model, batch, c.capacity_rows, kLoadGrid, spec_tiles,
                           L->gact, L->st);
    else
        hipLaunchKernelGGL((k_load_up_mfma<false>), dim3(kLoadGrid + tiles), dim3(256), 0, s, (_Float16*)L->buf.matrix,
                           L->buf.pointers, L->buf.bias, L->host, L->buf.b, added, L->move_dst, L->row_bytes,
                           c.d_ffn, (const _Float16*)x, L->h, c.d_model, batch, c.capacity_rows, kLoadGrid, spec_tiles,
                           L->gact, L->st);
}

// LDS a workgroup of k_predict_mask<T, BT> needs for a predictor of rank r: its static arrays plus BT * r doubles.
template <typename T, int BT>
int mask_lds_bytes(int r, size_t* out) {
    hipFuncAttributes fa;
    LIF_HIP(hipFuncGetAttributes(&fa, reinterpret_cast<const void*>(&k_predict_mask<T, BT>)));
    *out = fa.sharedSizeBytes + sizeof(double) * BT * (size_t)r;
    return LIF_OK;
}

// For every batch size the largest token tile (8, 4 or 1 tokens per pass over B) whose LDS fits the device limit.
template <typename T>
int choose_mask_tiles(lif_layer* L, size_t lds_limit) {
    size_t need[3];
    int rc = mask_lds_bytes<T, 1>(L->cfg.rank, &need[0]);
    if (!rc) rc = mask_lds_bytes<T, 4>(L->cfg.rank, &need[1]);
    if (!rc) rc = mask_lds_bytes<T, 8>(L->cfg.rank, &need[2]);
    if (rc) return rc;
    if (need[0] > lds_limit) return fail(LIF_INVALID_ARG, "rank too large for the LDS of a workgroup on this device");
    for (int b = 0; b <= 8; ++b) {
        int bt = 1;
        if (b > 1 && need[1] <= lds_limit) bt = 4;
        if (b > 4 && need[2] <= lds_limit) bt = 8;
        L->mask_bt[b] = bt;
    }
    return LIF_OK;
}

// Bandwidth reference: every 16-byte piece of [src, src + bytes) is read once; the pieces are folded into one word
// per workgroup so that the loads cannot be dropped.  bytes = 0: an empty launch.  grid-stride, eight loads per
// thread in flight.
constexpr int kProbePer = 8;
__global__ __launch_bounds__(256) void k_probe_read(const uint4* __restrict__ src, size_t pieces,
                                                    unsigned* __restrict__ sink) {
    unsigned acc = 0;
    const size_t stride = (size_t)gridDim.x * 256 * kProbePer;
    for (size_t base = (size_t)blockIdx.x * 256 * kProbePer; base < pieces; base += stride) {
        uint4 v[kProbePer];
#pragma unroll
        for (int p = 0; p < kProbePer; ++p) {
            const size_t i = base + (size_t)p * 256 + threadIdx.x;
            v[p] = i < pieces ? src[i] : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int p = 0; p < kProbePer; ++p) acc ^= v[p].x ^ v[p].y ^ v[p].z ^ v[p].w;
    }
    if (pieces == 0) return;
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) acc ^= __shfl_xor(acc, m, kWave);
    if ((threadIdx.x & 63) == 0 && acc == 0x9e3779b9u) sink[0] = acc;      // practically never: keeps the loads alive
}

// Cost reference for merging two dependent kernels without a second launch: 256 workgroups read 16 KiB each and
// produce 8 bytes (the shape of the mask kernel), then hand them to one workgroup of the same launch.
//   mode 0  no hand-off: every workgroup writes its 8 bytes and ends
//   mode 1  fence + ticket: every workgroup passes a device-scope fence and takes a ticket; the last to arrive reads
//           the 2 KiB the others wrote.  No workgroup waits.
//   mode 2  no fences: the 8 bytes go out as two 64-bit words (32 bits of payload + the launch's 32-bit stamp) by
//           relaxed device-scope atomic stores; workgroup 0 polls all 512 words with relaxed device-scope atomic loads
//           until they carry this launch's stamp.  The wait is bounded (kHandoffPolls per word, then it gives up and
//           counts the give-up) and the grid of 256 workgroups is resident as a whole on the 256 compute units.
constexpr int kHandoffWgs = 256;
constexpr int kHandoffPolls = 20000;
__global__ __launch_bounds__(256) void k_probe_handoff(const uint4* __restrict__ src, unsigned long long* __restrict__ words,
                                                       unsigned* __restrict__ counter, unsigned long long* __restrict__ out,
                                                       int mode, unsigned stamp) {
    __shared__ unsigned ticket;
    __shared__ unsigned long long part[4];
    const int tid = threadIdx.x;
    uint4 v[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = src[(size_t)blockIdx.x * 1024 + i * 256 + tid];
    unsigned long long bits = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) bits ^= ((unsigned long long)(v[i].x ^ v[i].z) << 32) | (v[i].y ^ v[i].w);
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) bits ^= __shfl_xor(bits, m, kWave);
    if ((tid & 63) == 0) part[tid >> 6] = bits;
    __syncthreads();
    const unsigned long long mine = part[0] ^ part[1] ^ part[2] ^ part[3];
    if (mode == 2) {
        if (tid < 2) {
            const unsigned long long w = ((unsigned long long)stamp << 32) | (unsigned)(tid ? (mine >> 32) : mine);
            __hip_atomic_store(&words[blockIdx.x * 2 + tid], w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        if (blockIdx.x != 0) return;
        unsigned long long acc = 0;
        bool ok = true;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            unsigned long long w = 0;
            int polls = 0;
            do {
                w = __hip_atomic_load(&words[tid * 2 + j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            } while ((unsigned)(w >> 32) != stamp && ++polls < kHandoffPolls);
            ok = ok && (unsigned)(w >> 32) == stamp;
            acc ^= w & 0xffffffffull;
        }
        if (!ok) atomicAdd(counter + 1, 1u);           // give-ups, reported by the caller
#pragma unroll
        for (int sft = 32; sft >= 1; sft >>= 1) acc ^= __shfl_xor(acc, sft, kWave);
        __syncthreads();
        if ((tid & 63) == 0) part[tid >> 6] = acc;
        __syncthreads();
        if (tid == 0) out[0] = part[0] ^ part[1] ^ part[2] ^ part[3];
        return;
    }
    if (tid == 0) words[blockIdx.x] = mine;
    if (mode == 0) return;
    if (tid == 0) {
        __threadfence();
        ticket = atomicAdd(counter, 1u);
    }
    __syncthreads();
    if (ticket != gridDim.x - 1) return;
    __threadfence();
    unsigned long long m = words[tid];                // gridDim.x == 256 == blockDim.x
#pragma unroll
    for (int sft = 32; sft >= 1; sft >>= 1) m ^= __shfl_xor(m, sft, kWave);
    if ((tid & 63) == 0) part[tid >> 6] = m;
    __syncthreads();
    if (tid == 0) {
        out[0] = part[0] ^ part[1] ^ part[2] ^ part[3];
        *counter = 0;                                 // ready for the next launch on this stream
    }
}

int check_launch() {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(LIF_HIP_ERROR, "kernel launch: %s", hipGetErrorString(e));
    return LIF_OK;
}

}  // namespace

extern "C" {

int lif_version(void) { return 2; }

const char* lif_last_error_string(void) { return g_err; }

size_t lif_workspace_bytes(const lif_config* cfg) {
    const char* why;
    if (!config_ok(cfg, &why)) return 0;
    return make_layout(*cfg).total;
}

int lif_create(const lif_config* cfg, const lif_buffers* buf, lif_layer** out) {
    const char* why;
    if (!out) return fail(LIF_INVALID_ARG, "out is null");
    *out = nullptr;
    if (!config_ok(cfg, &why)) return fail(LIF_INVALID_ARG, "invalid config: %s", why);
    if (!buf) return fail(LIF_INVALID_ARG, "buffers are null");
    if (!buf->A || (!buf->B && cfg->predictor != LIF_PRED_GATE) || !buf->b || !buf->host_bundles || !buf->matrix || !buf->pointers || !buf->bias ||
        !buf->workspace)
        return fail(LIF_INVALID_ARG, "a required buffer is null");
    const void* ptrs[] = {buf->A, buf->B ? buf->B : buf->A, buf->host_bundles, buf->matrix};
    for (const void* p : ptrs)
        if ((uintptr_t)p % 16) return fail(LIF_INVALID_ARG, "A, B, host_bundles and matrix must be 16-byte aligned");
    if ((uintptr_t)buf->workspace % 256) return fail(LIF_INVALID_ARG, "workspace must be 256-byte aligned");
    Layout lay = make_layout(*cfg);
    if (buf->workspace_bytes < lay.total) return fail(LIF_INVALID_ARG, "workspace smaller than lif_workspace_bytes");

    void* alias = nullptr;
    LIF_HIP(hipHostGetDevicePointer(&alias, const_cast<void*>(buf->host_bundles), 0));
    if (!alias) return fail(LIF_HIP_ERROR, "bundle store has no device alias");
    void* alias_down = nullptr;
    if (buf->host_down) {
        if ((uintptr_t)buf->host_down % 16) return fail(LIF_INVALID_ARG, "host_down must be 16-byte aligned");
        LIF_HIP(hipHostGetDevicePointer(&alias_down, const_cast<void*>(buf->host_down), 0));
        if (!alias_down) return fail(LIF_HIP_ERROR, "down-column store has no device alias");
    }

    lif_layer* L = new (std::nothrow) lif_layer();
    if (!L) return fail(LIF_INVALID_ARG, "out of host memory");
    L->cfg = *cfg;
    L->buf = *buf;
    L->lay = lay;
    L->host.rows = (const char*)alias;
    L->host.down = (const char*)alias_down;
    L->host.act_bytes = (size_t)(cfg->glu ? 2 : 1) * cfg->d_model * elem_bytes(*cfg);
    L->loader_pairs = 0;
    char* ws = (char*)buf->workspace;
    L->st = (DevState*)(ws + lay.state);
    L->ring = (unsigned long long*)(ws + lay.ring);
    L->tpart = (double*)(ws + lay.tpart);
    L->move_dst = (int32_t*)(ws + lay.move_dst);
    L->hole_list = (int32_t*)(ws + lay.hole_list);
    L->h = (float*)(ws + lay.h);
    L->ypart = (float*)(ws + lay.ypart);
    L->h_new = (float*)(ws + lay.h_new);
    L->stamp = (int32_t*)(ws + lay.stamp);
    L->gact = cfg->predictor == LIF_PRED_GATE ? (float*)(ws + lay.gact) : nullptr;
    L->row_elems = (size_t)(cfg->glu ? 3 : 2) * cfg->d_model;
    L->row_bytes = L->row_elems * elem_bytes(*cfg);
    L->window_pending = false;
    L->expected_rows = 0;
    L->prof_on = false;
    L->prof_max = 0;
    for (int b = 0; b <= 8; ++b) L->mask_bt[b] = 1;
    {
        // address of the static scratch array on the device that is current now (the layer's device)
        void* p = nullptr;
        hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        L->static_scratch = (e == hipSuccess) ? (unsigned char*)p : nullptr;
        if (e != hipSuccess) (void)hipGetLastError();      // reported by lif_sparse_ffn_static, not by a later launch
    }
    if (cfg->predictor == LIF_PRED_LOWRANK) {
        // the mask kernel keeps t = x A of a tile of tokens in LDS: pick the tile that fits this device
        int dev = 0, lds_limit = 0;
        int rc = LIF_OK;
        hipError_t e = hipGetDevice(&dev);
        if (e == hipSuccess) e = hipDeviceGetAttribute(&lds_limit, hipDeviceAttributeMaxSharedMemoryPerBlock, dev);
        if (e != hipSuccess) rc = fail(LIF_HIP_ERROR, "device LDS limit: %s", hipGetErrorString(e));
        lds_limit = std::min(lds_limit, 64 * 1024);      // no launch of this library asks for more than 64 KiB
        if (!rc) rc = cfg->dtype == LIF_F32 ? choose_mask_tiles<float>(L, (size_t)lds_limit)
                                            : choose_mask_tiles<_Float16>(L, (size_t)lds_limit);
        if (rc) {
            delete L;
            return rc;
        }
    }
    *out = L;
    return LIF_OK;
}

int lif_destroy(lif_layer* layer) {
    if (!layer) return LIF_OK;
    for (hipEvent_t e : layer->ev) (void)hipEventDestroy(e);
    delete layer;
    return LIF_OK;
}

int lif_reset(lif_layer* L, void* stream) {
    if (!L) return fail(LIF_INVALID_ARG, "layer is null");
    hipStream_t s = (hipStream_t)stream;
    const int total_words = (L->cfg.window_k + 1) * ring_words(L->cfg);      // ring + cached-set bitmap
    const int grid = std::min((total_words + 255) / 256, 256);
    hipLaunchKernelGGL(k_reset, dim3(grid), dim3(256), 0, s, L->ring, total_words, L->stamp, L->cfg.capacity_rows,
                       L->st);
    L->window_pending = false;
    return check_launch();
}

static int check_predict(lif_layer* L, const void* x_dev, int32_t batch, uint8_t* masks_dev, uint8_t* step_mask_dev) {
    if (!L || !x_dev || !masks_dev || !step_mask_dev) return fail(LIF_INVALID_ARG, "null argument");
    if (batch < 1 || batch > L->cfg.max_batch) return fail(LIF_INVALID_ARG, "batch out of range");
    if ((uintptr_t)x_dev % 16) return fail(LIF_INVALID_ARG, "x must be 16-byte aligned");
    if (batch > 1 && masks_dev == step_mask_dev) return fail(LIF_INVALID_ARG, "step mask must not alias the masks when batch > 1");
    return LIF_OK;
}

int lif_predict(lif_layer* L, const void* x_dev, int32_t batch, uint8_t* masks_dev, uint8_t* step_mask_dev,
                void* stream) {
    int rc = check_predict(L, x_dev, batch, masks_dev, step_mask_dev);
    if (rc) return rc;
    hipStream_t s = (hipStream_t)stream;
    if (L->cfg.predictor == LIF_PRED_GATE) {
        if (L->cfg.dtype == LIF_F32) launch_predict_gate<float>(L, x_dev, batch, masks_dev, step_mask_dev, s);
        else launch_predict_gate<_Float16>(L, x_dev, batch, masks_dev, step_mask_dev, s);
    } else if (L->cfg.dtype == LIF_F32) {
        launch_predict<float>(L, x_dev, batch, masks_dev, step_mask_dev, s);
    } else {
        launch_predict<_Float16>(L, x_dev, batch, masks_dev, step_mask_dev, s);
    }
    return check_launch();
}

static int check_update_window(lif_layer* L, const uint8_t* masks_dev, const int32_t* added_dev,
                               const int32_t* n_added_dev, const int32_t* removed_dev, const int32_t* n_removed_dev) {
    if (!L || !masks_dev || !added_dev || !n_added_dev || !removed_dev || !n_removed_dev)
        return fail(LIF_INVALID_ARG, "null argument");
    if ((uintptr_t)masks_dev % 8) return fail(LIF_INVALID_ARG, "step mask must be 8-byte aligned");
    if (L->window_pending) return fail(LIF_BAD_STATE, "lif_update_window called twice without lif_load_bundles");
    return LIF_OK;
}

static int check_window_tokens(lif_layer* L, int32_t n_tokens, int32_t keep) {
    if (!L) return fail(LIF_INVALID_ARG, "layer is null");
    if (n_tokens < 1 || n_tokens > L->cfg.max_batch) return fail(LIF_INVALID_ARG, "n_tokens out of range");
    if (keep < 0 || keep > n_tokens) return fail(LIF_INVALID_ARG, "keep must be in 0..n_tokens");
    if (L->cfg.d_ffn % 64) return fail(LIF_INVALID_ARG, "token-granular window updates need d_ffn % 64 == 0");
    return LIF_OK;
}

static int update_window_impl(lif_layer* L, const uint8_t* masks_dev, int ntok, int keep, int32_t* added_dev,
                              int32_t* n_added_dev, int32_t* removed_dev, int32_t* n_removed_dev, void* stream) {
    int rc = check_update_window(L, masks_dev, added_dev, n_added_dev, removed_dev, n_removed_dev);
    if (rc) return rc;
    hipStream_t s = (hipStream_t)stream;
    const lif_config& c = L->cfg;
    {
        Timed t(L, LIF_K_WINDOW, s);
        hipLaunchKernelGGL(k_window_plan, dim3(1), dim3(kScanThreads), 0, s, masks_dev, ntok, keep, L->ring,
                           L->ring + (size_t)c.window_k * ring_words(c), ring_words(c), L->buf.pointers, c.d_ffn,
                           c.window_k, c.capacity_rows, c.shrink_window, added_dev, n_added_dev, removed_dev,
                           n_removed_dev, L->move_dst, L->hole_list, L->st);
    }
    L->window_pending = true;
    return check_launch();
}

int lif_update_window(lif_layer* L, const uint8_t* step_mask_dev, int32_t* added_dev, int32_t* n_added_dev,
                      int32_t* removed_dev, int32_t* n_removed_dev, void* stream) {
    return update_window_impl(L, step_mask_dev, 1, 1, added_dev, n_added_dev, removed_dev, n_removed_dev, stream);
}

int lif_update_window_tokens(lif_layer* L, const uint8_t* masks_dev, int32_t n_tokens, int32_t keep,
                             int32_t* added_dev, int32_t* n_added_dev, int32_t* removed_dev, int32_t* n_removed_dev,
                             void* stream) {
    int rc = check_window_tokens(L, n_tokens, keep);
    if (rc) return rc;
    if (n_tokens == 1 && keep == 1)
        return update_window_impl(L, masks_dev, 1, 1, added_dev, n_added_dev, removed_dev, n_removed_dev, stream);
    return update_window_impl(L, masks_dev, n_tokens, keep, added_dev, n_added_dev, removed_dev, n_removed_dev, stream);
}

int lif_load_bundles(lif_layer* L, const int32_t* added_dev, const int32_t* n_added_dev, const int32_t* removed_dev,
                     const int32_t* n_removed_dev, void* stream) {
    if (!L || !added_dev || !n_added_dev || !removed_dev || !n_removed_dev)
        return fail(LIF_INVALID_ARG, "null argument");
    if (!L->window_pending) return fail(LIF_BAD_STATE, "lif_load_bundles needs a preceding lif_update_window");
    hipStream_t s = (hipStream_t)stream;
    const lif_config& c = L->cfg;
    {
        const int cpr = (int)((L->row_bytes + kLoadChunk - 1) / kLoadChunk);
        const long long worst = (long long)c.capacity_rows * cpr;
        const int grid = (int)std::min<long long>(worst, kLoadGrid);
        Timed t(L, LIF_K_LOAD, s);
        hipLaunchKernelGGL(k_load, dim3(grid), dim3(256), 0, s, (char*)L->buf.matrix, L->buf.pointers, L->buf.bias,
                           L->host, L->buf.b, added_dev, L->move_dst, L->row_bytes, c.d_ffn, L->st);
    }
    L->window_pending = false;
    return check_launch();
}

static int check_ffn(lif_layer* L, const void* x_dev, int32_t batch, void* y_dev) {
    if (!L || !x_dev || !y_dev) return fail(LIF_INVALID_ARG, "null argument");
    if (batch < 1 || batch > L->cfg.max_batch) return fail(LIF_INVALID_ARG, "batch out of range");
    if ((uintptr_t)x_dev % 16 || (uintptr_t)y_dev % 16) return fail(LIF_INVALID_ARG, "x and y must be 16-byte aligned");
    return LIF_OK;
}

// the two FFN stages with their scratch: activations h, partial outputs ypart
static int ffn_launches(lif_layer* L, const void* x_dev, int32_t batch, void* y_dev, float* h, float* ypart,
                        hipStream_t s) {
    const lif_config& c = L->cfg;
    if (mfma_path(c, batch)) {
        // batched tokens: the activation stage is a dense contraction -> matrix cores
        Timed t(L, LIF_K_FFN_UP, s);
        launch_ffn_up_mfma<kRowsAll>(L, x_dev, batch, h, s);
    } else {
        Timed t(L, LIF_K_FFN_UP, s);
        if (c.dtype == LIF_F32) {
            if (c.glu) launch_ffn_up<float, true>(L, x_dev, batch, h, s);
            else launch_ffn_up<float, false>(L, x_dev, batch, h, s);
        } else {
            if (c.glu) launch_ffn_up<_Float16, true>(L, x_dev, batch, h, s);
            else launch_ffn_up<_Float16, false>(L, x_dev, batch, h, s);
        }
    }
    {
        Timed t(L, LIF_K_FFN_DOWN, s);
        if (c.dtype == LIF_F32) launch_ffn_down<float>(L, batch, y_dev, h, ypart, s);
        else launch_ffn_down<_Float16>(L, batch, y_dev, h, ypart, s);
    }
    return check_launch();
}

int lif_sparse_ffn(lif_layer* L, const void* x_dev, int32_t batch, void* y_dev, void* stream) {
    int rc = check_ffn(L, x_dev, batch, y_dev);
    if (rc) return rc;
    return ffn_launches(L, x_dev, batch, y_dev, L->h, L->ypart, (hipStream_t)stream);
}

size_t lif_static_scratch_bytes(void) { return kStaticScratchBytes; }

int lif_sparse_ffn_static(lif_layer* L, const void* x_dev, int32_t batch, void* y_dev, void* stream) {
    int rc = check_ffn(L, x_dev, batch, y_dev);
    if (rc) return rc;
    if (!L->static_scratch) return fail(LIF_HIP_ERROR, "the static scratch array has no address on this device");
    // activations [batch x capacity_rows] fp32, then the partial outputs [row chunks x batch x d_model] fp32
    const lif_config& c = L->cfg;
    const size_t h_bytes = align_up(sizeof(float) * (size_t)batch * c.capacity_rows, 256);
    const size_t ypart_bytes = sizeof(float) * (size_t)kDownChunksMax * batch * c.d_model;
    if (h_bytes + ypart_bytes > kStaticScratchBytes)
        return fail(LIF_INVALID_ARG, "batch x capacity_rows and batch x d_model exceed the static scratch (5 MiB); use lif_sparse_ffn");
    // the kernels take the scratch as arguments, exactly as they take the workspace arrays in lif_sparse_ffn;
    // nothing in it has to start at zero: every activation and every partial that is read was written by this call
    return ffn_launches(L, x_dev, batch, y_dev, reinterpret_cast<float*>(L->static_scratch),
                        reinterpret_cast<float*>(L->static_scratch + h_bytes), (hipStream_t)stream);
}

// keep < 0: the window advances by one step whose mask is the OR over the batch (lif_update_window);
// keep >= 0: token-granular update of a speculative pass (lif_update_window_tokens)
static int step_impl(lif_layer* L, const void* x_dev, int32_t batch, int32_t keep, void* y_dev, uint8_t* masks_dev,
                     uint8_t* step_mask_dev, int32_t* added_dev, int32_t* n_added_dev, int32_t* removed_dev,
                     int32_t* n_removed_dev, void* stream) {
    // every argument and call-order check of the four calls comes before the first launch: a rejected step
    // leaves the device buffers untouched
    int rc = check_predict(L, x_dev, batch, masks_dev, step_mask_dev);
    if (rc) return rc;
    if (!y_dev || (uintptr_t)y_dev % 16) return fail(LIF_INVALID_ARG, "y must be a 16-byte aligned device pointer");
    if (keep >= 0 && (rc = check_window_tokens(L, batch, keep))) return rc;
    rc = check_update_window(L, keep < 0 ? step_mask_dev : masks_dev, added_dev, n_added_dev, removed_dev, n_removed_dev);
    if (rc) return rc;
    rc = lif_predict(L, x_dev, batch, masks_dev, step_mask_dev, stream);
    if (rc) return rc;
    rc = keep < 0 ? lif_update_window(L, step_mask_dev, added_dev, n_added_dev, removed_dev, n_removed_dev, stream)
                  : lif_update_window_tokens(L, masks_dev, batch, keep, added_dev, n_added_dev, removed_dev,
                                             n_removed_dev, stream);
    if (rc) return rc;
    hipStream_t s = (hipStream_t)stream;
    const lif_config& c = L->cfg;
    // batch > 1: sharing a launch between the load and the activation stage pays once the activation stage over
    // all rows takes longer than the second pass over the rows the load wrote (about 2000 rows in use)
    const int rows_hint = L->expected_rows > 0 ? L->expected_rows : c.capacity_rows;
    if (batch > 1 && (!mfma_path(c, batch) || rows_hint < kFuseBatchedMinRows)) {
        rc = lif_load_bundles(L, added_dev, n_added_dev, removed_dev, n_removed_dev, stream);
        if (rc) return rc;
        return lif_sparse_ffn(L, x_dev, batch, y_dev, stream);
    }
    if (batch > 1) {
        {
            Timed t(L, LIF_K_LOAD, s);
            launch_load_up_mfma(L, x_dev, batch, added_dev, s);
        }
        L->window_pending = false;
        {
            Timed t(L, LIF_K_FFN_UP, s);
            launch_ffn_up_mfma<kRowsChanged>(L, x_dev, batch, L->h, s);
        }
        Timed t(L, LIF_K_FFN_DOWN, s);
        launch_ffn_down<_Float16>(L, batch, y_dev, L->h, L->ypart, s);
        return check_launch();
    }
    {
        Timed t(L, LIF_K_LOAD, s);
        if (c.dtype == LIF_F32) {
            if (c.glu) launch_load_up<float, true>(L, x_dev, added_dev, s);
            else launch_load_up<float, false>(L, x_dev, added_dev, s);
        } else {
            if (c.glu) launch_load_up<_Float16, true>(L, x_dev, added_dev, s);
            else launch_load_up<_Float16, false>(L, x_dev, added_dev, s);
        }
    }
    L->window_pending = false;
    {
        Timed t(L, LIF_K_FFN_DOWN, s);
        if (c.dtype == LIF_F32) launch_ffn_down<float>(L, 1, y_dev, L->h, L->ypart, s, true);
        else launch_ffn_down<_Float16>(L, 1, y_dev, L->h, L->ypart, s, true);
    }
    return check_launch();
}

int lif_step(lif_layer* L, const void* x_dev, int32_t batch, void* y_dev, uint8_t* masks_dev,
             uint8_t* step_mask_dev, int32_t* added_dev, int32_t* n_added_dev, int32_t* removed_dev,
             int32_t* n_removed_dev, void* stream) {
    return step_impl(L, x_dev, batch, -1, y_dev, masks_dev, step_mask_dev, added_dev, n_added_dev, removed_dev,
                     n_removed_dev, stream);
}

int lif_step_tokens(lif_layer* L, const void* x_dev, int32_t n_tokens, int32_t keep_tokens, void* y_dev,
                    uint8_t* masks_dev, uint8_t* step_mask_dev, int32_t* added_dev, int32_t* n_added_dev,
                    int32_t* removed_dev, int32_t* n_removed_dev, void* stream) {
    if (keep_tokens < 0) return fail(LIF_INVALID_ARG, "keep must be in 0..n_tokens");
    return step_impl(L, x_dev, n_tokens, keep_tokens, y_dev, masks_dev, step_mask_dev, added_dev, n_added_dev,
                     removed_dev, n_removed_dev, stream);
}

int lif_set_loader_pairs(lif_layer* L, int32_t pairs) {
    if (!L || pairs < 0 || pairs > 64) return fail(LIF_INVALID_ARG, "loader pairs must be in 0..64");
    L->loader_pairs = pairs;
    return LIF_OK;
}

int lif_set_expected_rows(lif_layer* L, int32_t rows) {
    if (!L || rows < 0) return fail(LIF_INVALID_ARG, "bad row hint");
    L->expected_rows = rows;
    return LIF_OK;
}

static int read_state(lif_layer* L, DevState* host, void* stream) {
    hipStream_t s = (hipStream_t)stream;
    LIF_HIP(hipStreamSynchronize(s));
    LIF_HIP(hipMemcpy(host, L->st, sizeof(DevState), hipMemcpyDeviceToHost));
    return LIF_OK;
}

int lif_get_state(lif_layer* L, lif_state* out, void* stream) {
    if (!L || !out) return fail(LIF_INVALID_ARG, "null argument");
    DevState h;
    int rc = read_state(L, &h, stream);
    if (rc) return rc;
    out->num_used = h.num_used;
    out->step = h.step;
    out->error = h.error;
    out->last_added = h.n_added;
    out->last_removed = h.n_removed;
    out->last_moved = h.n_moved;
    out->window_len = h.window_len;
    return LIF_OK;
}

int lif_get_counters(lif_layer* L, lif_counters* out, void* stream) {
    if (!L || !out) return fail(LIF_INVALID_ARG, "null argument");
    DevState h;
    int rc = read_state(L, &h, stream);
    if (rc) return rc;
    out->steps = h.c_steps;
    out->added = h.c_added;
    out->removed = h.c_removed;
    out->rows_moved = h.c_rows_moved;
    out->h2d_bytes = h.c_h2d_bytes;
    out->ffn_calls = h.c_ffn_calls;
    out->ffn_rows = h.c_ffn_rows;
    out->ffn_active = h.c_ffn_active;
    return LIF_OK;
}

int lif_profile_read(const void* src_dev, size_t bytes, void* sink_dev, void* stream) {
    if (!sink_dev || (bytes && !src_dev)) return fail(LIF_INVALID_ARG, "null argument");
    if ((uintptr_t)src_dev % 16 || bytes % 16 || (uintptr_t)sink_dev % 4)
        return fail(LIF_INVALID_ARG, "src must be 16-byte aligned and bytes a multiple of 16");
    const size_t pieces = bytes / 16;
    const size_t wgs = (pieces + 256 * kProbePer - 1) / (256 * kProbePer);
    const int grid = (int)std::min<size_t>(std::max<size_t>(wgs, 1), 4096);
    hipLaunchKernelGGL(k_probe_read, dim3(grid), dim3(256), 0, (hipStream_t)stream, (const uint4*)src_dev, pieces,
                       (unsigned*)sink_dev);
    return check_launch();
}

size_t lif_profile_handoff_bytes(void) { return (size_t)kHandoffWgs * 16384 + 8192; }

int lif_profile_handoff(void* scratch_dev, int32_t mode, uint32_t stamp, void* stream) {
    if (!scratch_dev || (uintptr_t)scratch_dev % 256) return fail(LIF_INVALID_ARG, "scratch must be a 256-byte aligned device pointer");
    if (mode < 0 || mode > 2) return fail(LIF_INVALID_ARG, "mode must be 0, 1 or 2");
    char* p = (char*)scratch_dev;
    char* tail = p + (size_t)kHandoffWgs * 16384;      // 4 KiB of words, then the ticket counter, the give-up count, the result
    hipLaunchKernelGGL(k_probe_handoff, dim3(kHandoffWgs), dim3(256), 0, (hipStream_t)stream, (const uint4*)p,
                       (unsigned long long*)tail, (unsigned*)(tail + 4096), (unsigned long long*)(tail + 4096 + 64), mode,
                       stamp);
    return check_launch();
}

int lif_profile_begin(lif_layer* L, int32_t max_launches) {
    if (!L || max_launches < 1 || max_launches > (1 << 20)) return fail(LIF_INVALID_ARG, "bad profile request");
    for (hipEvent_t e : L->ev) (void)hipEventDestroy(e);
    L->ev.clear();
    L->ev_kernel.clear();
    L->ev.resize(2 * (size_t)max_launches);
    for (size_t i = 0; i < L->ev.size(); ++i) {
        hipError_t e = hipEventCreate(&L->ev[i]);
        if (e != hipSuccess) {
            L->ev.resize(i);
            return fail(LIF_HIP_ERROR, "hipEventCreate: %s", hipGetErrorString(e));
        }
    }
    L->prof_max = max_launches;
    L->prof_on = true;
    return LIF_OK;
}

int lif_profile_collect(lif_layer* L, double* ms, int64_t* launches, void* stream) {
    if (!L || !ms || !launches) return fail(LIF_INVALID_ARG, "null argument");
    L->prof_on = false;
    LIF_HIP(hipStreamSynchronize((hipStream_t)stream));
    for (int k = 0; k < LIF_K_COUNT; ++k) {
        ms[k] = 0.0;
        launches[k] = 0;
    }
    for (size_t i = 0; i < L->ev_kernel.size(); ++i) {
        float t = 0.f;
        LIF_HIP(hipEventElapsedTime(&t, L->ev[2 * i], L->ev[2 * i + 1]));
        ms[L->ev_kernel[i]] += t;
        launches[L->ev_kernel[i]] += 1;
    }
    for (hipEvent_t e : L->ev) (void)hipEventDestroy(e);
    L->ev.clear();
    L->ev_kernel.clear();
    return LIF_OK;
}

}  // extern "C"
