// Step 4 for a batch of tokens (2..8), fp16: the activation stage becomes a dense contraction
//   H[s][t] = sum_i U[s][i] * X[t][i]        (16 cached rows x 16 token slots per tile)
// and runs on the matrix cores (v_mfma_f32_16x16x32_f16, fp32 accumulation).  It is still bound
// by streaming the up (and gate) vectors once - 8 flop per byte - so the layout is chosen for
// the loads, not for the MFMA: a lane's A fragment is 16 contiguous bytes of its row, which is
// exactly one global load.  Any assignment of k indices to fragment positions is valid as long
// as the A and the B fragment of a lane use the same one, because the contraction sums over k.
#pragma once

#include "lif_common.h"

namespace lif {

constexpr int kMfmaUnroll = 8;     // k-steps (32 elements each) a wave keeps in flight

// A workgroup owns the 16 rows of a tile and exits at once if they are not in use; its waves take contiguous
// parts of the k range.  Two forms of the tile follow: ffn_up_mfma_tile loads the fragments directly (a wave
// instruction reads 64 bytes of 16 rows; used with 16 waves for the few tiles a load wrote), and
// ffn_up_mfma_tile_staged reads row-contiguous pieces and passes them through LDS (the pass over all rows and the
// one next to the loaders).  Both give the same bits.
// Fragment layout of the 16x16x32 MFMA: lane l supplies row (l mod 16) of A and column (l mod 16)
// of B for the k sub-block (l div 16); it receives D[4 * (l div 16) + r][l mod 16], r = 0..3.
// Here A = rows of the cache, B = tokens (columns >= batch are zero).
// Requires d % 32 == 0.
constexpr int kMfmaParts = 16;      // parts of the k range, each summed from zero, added as a tree (below)
constexpr int kMfmaWaves = 4;       // waves per tile in the launch shared with the loaders (256 threads per workgroup)
constexpr int kMfmaWavesFix = 16;   // ... for the short pass over the rows a load wrote: few tiles, so a
                                    // tile is spread over 16 waves (one round of loads each)

// How the 16 partial tiles of a row tile are added: as a balanced binary tree in part order,
//   ((p0 + p1) + (p2 + p3)) + ((p4 + p5) + (p6 + p7)) + ...
// so a wave that owns 1, 2 or 4 consecutive parts adds its own subtree in registers and the subtrees of the waves are
// added the same way: the result does not depend on how many waves share a tile.
// tree_push: part number pp (0, 1, 2, ... in order) of a wave arrives; lvl[b] holds a finished subtree of 2^b parts.
template <int PP>
__device__ __forceinline__ void tree_push(f32x4 (&lvl)[3], f32x4 v) {
    static_assert(PP >= 0 && PP < 4, "at most four parts per wave");
    if constexpr ((PP & 1) == 0) lvl[0] = v;                       // p0, p2
    else if constexpr ((PP & 2) == 0) lvl[1] = lvl[0] + v;         // p0 + p1
    else lvl[2] = lvl[1] + (lvl[0] + v);                           // (p0 + p1) + (p2 + p3)
}
// tree over the WAVES subtrees of one output, in wave order
template <int WAVES>
__device__ __forceinline__ float tree_sum(float (&v)[WAVES]) {
#pragma unroll
    for (int stride = 1; stride < WAVES; stride *= 2)
#pragma unroll
        for (int k = 0; k < WAVES; k += 2 * stride) v[k] = v[k] + v[k + stride];
    return v[0];
}

// Which rows a launch of the MFMA activation stage covers.
enum MfmaRows {
    kRowsAll = 0,     // slots [0, num_used)
    kRowsKept = 1,    // slots [0, n_base): the rows that survive a pending deletion, while the loader role of the
                      // same launch moves rows into holes and appends new ones (values of holes are recomputed later)
    kRowsChanged = 2  // the slots the last load wrote: holes filled by a move, then the appended rows
};

// One 16-row tile.  `tile` indexes the list of rows of the given mode; entry e of the list is slot e for
// kRowsAll / kRowsKept; for kRowsChanged it is move_dst[e] for e < n_removed (-1 = tail slot that was not
// moved: skipped) and slot n_base + (e - n_removed) for the n_added entries after that.
// Returns false (for the whole workgroup) when the tile lies past the end of the list.
// `gact` (may be null; plain bundles only): gate activations relu(gate_i . x_t + b_i) per token and neuron,
// [batch x gact_n], written by the gate predictor; the activation of a row is then gact[t][pointers[row]] * (up . x_t).
template <bool GLU, int MODE, int WAVES>
__device__ __forceinline__ bool ffn_up_mfma_tile(const _Float16* __restrict__ matrix, const float* __restrict__ bias,
                                                 const _Float16* __restrict__ x, float* __restrict__ h, int d,
                                                 int batch, int capacity, size_t row_elems,
                                                 const int32_t* __restrict__ move_dst, int tile,
                                                 const int32_t* __restrict__ pointers, const float* __restrict__ gact,
                                                 int gact_n, const DevState* __restrict__ st) {
    __shared__ float red[GLU ? 2 : 1][WAVES][64][4];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int i = lane & 15, q = lane >> 4;
    const int s0 = tile * 16;
    // requested together with the state (the list spans the capacity, so the address is valid; masked below)
    int moved_to = -1;
    if (MODE == kRowsChanged && s0 + i < capacity) moved_to = move_dst[s0 + i];
    const int err = st->error;
    const int n_removed = st->n_removed, n_base = st->n_base;
    const int n = (MODE == kRowsAll) ? st->num_used : (MODE == kRowsKept) ? n_base : n_removed + st->n_added;
    if (err || s0 >= n) return false;                             // uniform

    int srow = s0 + i;                                            // slot of list entry s0 + i (-1: none)
    if (MODE == kRowsChanged) {
        const int e = s0 + i;
        srow = (e >= n) ? -1 : (e < n_removed ? moved_to : n_base + (e - n_removed));
    } else if (srow >= n) {
        srow = -1;
    }
    // the lane that finishes D rows 4q .. 4q + 3 for token i asks for their biases now, ahead of the row loads
    int orow[4];
    float obias[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        orow[r] = __shfl(srow, 4 * q + r, kWave);                 // lane j < 16 holds the slot of tile row j
        obias[r] = 0.f;
        if (w == 0 && orow[r] >= 0) {
            if (GLU || !gact) obias[r] = bias[orow[r]];
            else if (i < batch) obias[r] = gact[(size_t)i * gact_n + min(max(pointers[orow[r]], 0), gact_n - 1)];
        }
    }
    const _Float16* grow = matrix + (size_t)min(max(srow, 0), capacity - 1) * row_elems;   // masked rows read slot 0
    const _Float16* urow = grow + (GLU ? d : 0);
    const bool xok = i < batch;
    const _Float16* xrow = x + (size_t)(xok ? i : 0) * d;
    const int nks = d >> 5;

    // The k-steps are cut into kMfmaParts contiguous parts, each accumulated from zero; wave w takes the parts
    // w * PPW .. w * PPW + PPW - 1 and adds them as its subtree (tree_push).
    constexpr int PPW = kMfmaParts / WAVES;
    constexpr int kTop = PPW == 1 ? 0 : PPW == 2 ? 1 : 2;
    static_assert(PPW == 1 || PPW == 2 || PPW == 4, "a wave owns a subtree of the parts");
    const int per = (nks + kMfmaParts - 1) / kMfmaParts;
    f32x4 lu[3], lg[3];
#pragma unroll
    for (int pp = 0; pp < PPW; ++pp) {
        const int part = w * PPW + pp;
        const int ks_begin = part * per, ks_end = min(nks, ks_begin + per);
        f32x4 cu = {0.f, 0.f, 0.f, 0.f}, cg = {0.f, 0.f, 0.f, 0.f};
        for (int ks0 = ks_begin; ks0 < ks_end; ks0 += kMfmaUnroll) {
            f16x8 uf[kMfmaUnroll], gf[GLU ? kMfmaUnroll : 1], xf[kMfmaUnroll];
#pragma unroll
            for (int u = 0; u < kMfmaUnroll; ++u) {
                const int ks = ks0 + u;
                const int off = (ks << 5) + (q << 3);
                const bool in = ks < ks_end;
                uf[u] = in ? *reinterpret_cast<const f16x8*>(urow + off) : f16x8(0);
                if (GLU) gf[u] = in ? *reinterpret_cast<const f16x8*>(grow + off) : f16x8(0);
                xf[u] = (in && xok) ? *reinterpret_cast<const f16x8*>(xrow + off) : f16x8(0);
            }
#pragma unroll
            for (int u = 0; u < kMfmaUnroll; ++u) {
                cu = __builtin_amdgcn_mfma_f32_16x16x32_f16(uf[u], xf[u], cu, 0, 0, 0);
                if (GLU) cg = __builtin_amdgcn_mfma_f32_16x16x32_f16(gf[u], xf[u], cg, 0, 0, 0);
            }
        }
        if (pp == 0) { tree_push<0>(lu, cu); if (GLU) tree_push<0>(lg, cg); }
        if (pp == 1) { tree_push<1>(lu, cu); if (GLU) tree_push<1>(lg, cg); }
        if (pp == 2) { tree_push<2>(lu, cu); if (GLU) tree_push<2>(lg, cg); }
        if (pp == 3) { tree_push<3>(lu, cu); if (GLU) tree_push<3>(lg, cg); }
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        red[0][w][lane][r] = lu[kTop][r];
        if (GLU) red[GLU ? 1 : 0][w][lane][r] = lg[kTop][r];
    }
    __syncthreads();
    if (w == 0 && xok) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = orow[r];
            if (row >= 0) {
                float v[WAVES];
#pragma unroll
                for (int ww = 0; ww < WAVES; ++ww) v[ww] = red[0][ww][lane][r];
                const float su = tree_sum<WAVES>(v);
                const float bs = obias[r];
                float act;
                if (GLU) {
#pragma unroll
                    for (int ww = 0; ww < WAVES; ++ww) v[ww] = red[GLU ? 1 : 0][ww][lane][r];
                    const float sg = tree_sum<WAVES>(v);
                    act = fmaxf(sg + bs, 0.f) * su;
                } else if (gact) {
                    act = bs * su;                    // bs = this token's gate activation of the row's neuron
                } else {
                    act = fmaxf(su + bs, 0.f);
                }
                h[(size_t)i * capacity + row] = act;
            }
        }
    }
    return true;
}

// The same tile with the rows read row-contiguously and staged in LDS (kRowsAll and kRowsKept only).
// The fragment pattern above asks for 64 bytes of 16 different rows per wave instruction; measured at the
// Llama-2 shape with 8700 rows in use that pattern streams at 4.2 TB/s where whole 256-byte pieces of a row
// (4 rows per wave instruction) reach 5.4 TB/s.  Here a wave reads a stage of kStageSteps k-steps of its 16 rows
// that way, passes the up rows and then the gate rows through its own LDS area (rows padded by 16 bytes: the
// b128 reads of 16 lanes then fall on 16 distinct bank groups) and reads the fragments back from there; the
// registers are refilled with the next stage as soon as they are written out, across part boundaries too.
// The MFMA operands, the k order inside a part and the order in which the parts are added are those of
// ffn_up_mfma_tile, so every number of waves and both functions give the same bits.  With 8 waves a tile takes
// half the dependent stages per wave: 7.7 us against 10 us at 1400 rows, 26 us against 27 us at 8700.
// `spec`: the first stage is requested before the row count arrives (the addresses of slots [0, capacity) are
// always valid); the host sets it for the tiles a row-count hint covers.
constexpr int kStageSteps = 4;                           // k-steps per stage: 256 bytes of a row
constexpr int kStagePitch = kStageSteps * 64 + 16;       // bytes between the staged rows of a wave
constexpr int kMfmaWavesAll = 8;                         // waves per tile of the stand-alone pass over all rows

template <bool GLU>
struct StageRegs {
    f16x8 u[4], g[GLU ? 4 : 1];
};

template <bool GLU, int MODE, int WAVES>
__device__ __forceinline__ bool ffn_up_mfma_tile_staged(const _Float16* __restrict__ matrix,
                                                        const float* __restrict__ bias,
                                                        const _Float16* __restrict__ x, float* __restrict__ h, int d,
                                                        int batch, int capacity, size_t row_elems, int tile,
                                                        bool spec, const int32_t* __restrict__ pointers,
                                                        const float* __restrict__ gact, int gact_n,
                                                        const DevState* __restrict__ st) {
    static_assert(MODE == kRowsAll || MODE == kRowsKept, "list entry e must be slot e");
    static_assert(kStageSteps == 4, "a wave instruction covers 4 rows x 16 units of 16 bytes");
    static_assert(kMfmaParts % WAVES == 0, "whole parts per wave");
    constexpr int NG = GLU ? 2 : 1;
    constexpr int PPW = kMfmaParts / WAVES;
    constexpr int kTop = PPW == 1 ? 0 : PPW == 2 ? 1 : 2;
    static_assert(PPW == 1 || PPW == 2 || PPW == 4, "a wave owns a subtree of the parts");
    __shared__ __align__(16) unsigned char lds[WAVES * 16 * kStagePitch];      // one staging area per wave
    __shared__ float red[NG][WAVES][64][4];                                    // the waves' subtrees
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int i = lane & 15, q = lane >> 4;
    const int s0 = tile * 16;
    // loader view of a lane: instruction j reads unit i (16 bytes) of tile row 4 j + q
    // (kept as 32-bit offsets in units of 16 bytes: row_elems is a multiple of 8 when d is a multiple of 32)
    const f16x8* mat8 = reinterpret_cast<const f16x8*>(matrix);
    const unsigned row8 = (unsigned)(row_elems >> 3), d8 = (unsigned)(d >> 3);
    unsigned lrow[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) lrow[j] = (unsigned)min(s0 + 4 * j + q, capacity - 1) * row8;
    const int nks = d >> 5;
    const int per = (nks + kMfmaParts - 1) / kMfmaParts;
    const int S = (per + kStageSteps - 1) / kStageSteps;      // stages per part
    StageRegs<GLU> R;
    // stage s of a part: k-steps [part * per + s * kStageSteps, + kStageSteps), cut at the end of the part
    auto issue = [&](int part, int s) {
        const int ks0 = part * per + s * kStageSteps, ks_end = min(nks, part * per + per);
        const bool in = ks0 + (i >> 2) < ks_end;
        const unsigned off = (unsigned)(ks0 << 2) + (unsigned)i;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            R.u[j] = in ? mat8[(size_t)(lrow[j] + (GLU ? d8 : 0u) + off)] : f16x8(0);
            if (GLU) R.g[j] = in ? mat8[(size_t)(lrow[j] + off)] : f16x8(0);
        }
    };
    if (spec) issue(w * PPW, 0);
    const int err = st->error;
    const int n = (MODE == kRowsAll) ? st->num_used : st->n_base;
    if (err || s0 >= n) return false;                             // uniform
    if (!spec) issue(w * PPW, 0);

    // the lane that finishes D rows 4q .. 4q + 3 for token i asks for their biases now, ahead of the row loads
    float obias[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int row = s0 + 4 * q + r;
        obias[r] = 0.f;
        if (w == 0 && row < n) {
            if (GLU || !gact) obias[r] = bias[row];
            else if (i < batch) obias[r] = gact[(size_t)i * gact_n + min(max(pointers[row], 0), gact_n - 1)];
        }
    }
    const bool xok = i < batch;
    const _Float16* xrow = x + (size_t)(xok ? i : 0) * d;
    // The area is this wave's alone and a wave's LDS operations complete in order, so the steps below need no
    // barrier instruction (wave_barrier only keeps the compiler from moving LDS accesses across it).
    unsigned char* wr = lds + w * (16 * kStagePitch) + q * kStagePitch + i * 16;      // + 4 j rows for instruction j
    const unsigned char* rd = lds + w * (16 * kStagePitch) + i * kStagePitch + q * 16; // + 64 bytes per k-step

    f32x4 lu[3], lg[3];
#pragma unroll
    for (int pp = 0; pp < PPW; ++pp) {
        const int part = w * PPW + pp;
        const int ks_end = min(nks, part * per + per);
        f32x4 au = {0.f, 0.f, 0.f, 0.f}, ag = {0.f, 0.f, 0.f, 0.f};
        for (int s = 0; s < S; ++s) {
            const int ks0 = part * per + s * kStageSteps;
            f16x8 xf[kStageSteps];
#pragma unroll
            for (int u = 0; u < kStageSteps; ++u)
                xf[u] = (ks0 + u < ks_end && xok)
                            ? *reinterpret_cast<const f16x8*>(xrow + ((ks0 + u) << 5) + (q << 3)) : f16x8(0);
#pragma unroll
            for (int j = 0; j < 4; ++j) *reinterpret_cast<f16x8*>(wr + j * 4 * kStagePitch) = R.u[j];
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int u = 0; u < kStageSteps; ++u) {
                const f16x8 uf = *reinterpret_cast<const f16x8*>(rd + u * 64);
                au = __builtin_amdgcn_mfma_f32_16x16x32_f16(uf, xf[u], au, 0, 0, 0);
            }
            __builtin_amdgcn_wave_barrier();
            if (GLU) {
#pragma unroll
                for (int j = 0; j < 4; ++j) *reinterpret_cast<f16x8*>(wr + j * 4 * kStagePitch) = R.g[j];
            }
            if (s + 1 < S) issue(part, s + 1);
            else if (pp + 1 < PPW) issue(part + 1, 0);
            __builtin_amdgcn_wave_barrier();
            if (GLU) {
#pragma unroll
                for (int u = 0; u < kStageSteps; ++u) {
                    const f16x8 gf = *reinterpret_cast<const f16x8*>(rd + u * 64);
                    ag = __builtin_amdgcn_mfma_f32_16x16x32_f16(gf, xf[u], ag, 0, 0, 0);
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
        if (pp == 0) { tree_push<0>(lu, au); if (GLU) tree_push<0>(lg, ag); }
        if (pp == 1) { tree_push<1>(lu, au); if (GLU) tree_push<1>(lg, ag); }
        if (pp == 2) { tree_push<2>(lu, au); if (GLU) tree_push<2>(lg, ag); }
        if (pp == 3) { tree_push<3>(lu, au); if (GLU) tree_push<3>(lg, ag); }
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        red[0][w][lane][r] = lu[kTop][r];
        if (GLU) red[NG - 1][w][lane][r] = lg[kTop][r];
    }
    __syncthreads();
    if (w == 0 && xok) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = s0 + 4 * q + r;
            if (row < n) {
                float v[WAVES];
#pragma unroll
                for (int ww = 0; ww < WAVES; ++ww) v[ww] = red[0][ww][lane][r];
                const float su = tree_sum<WAVES>(v);
                const float bs = obias[r];
                float act;
                if (GLU) {
#pragma unroll
                    for (int ww = 0; ww < WAVES; ++ww) v[ww] = red[NG - 1][ww][lane][r];
                    const float sg = tree_sum<WAVES>(v);
                    act = fmaxf(sg + bs, 0.f) * su;
                } else if (gact) {
                    act = bs * su;
                } else {
                    act = fmaxf(su + bs, 0.f);
                }
                h[(size_t)i * capacity + row] = act;
            }
        }
    }
    return true;
}

template <bool GLU, int MODE, int WAVES>
__global__ __launch_bounds__(WAVES * 64, WAVES == kMfmaWavesAll ? 4 : 1) void k_ffn_up_mfma(const _Float16* __restrict__ matrix,
                                                                 const float* __restrict__ bias,
                                                                 const _Float16* __restrict__ x, float* __restrict__ h,
                                                                 int d, int batch, int capacity, size_t row_elems,
                                                                 const int32_t* __restrict__ move_dst,
                                                                 const int32_t* __restrict__ pointers,
                                                                 const float* __restrict__ gact, int gact_n,
                                                                 int spec, const DevState* __restrict__ st) {
    // `spec`: the grid was sized from a row-count hint, the first tile of a workgroup is requested ahead of the state
    // grid-stride over tiles (the grid may be smaller than the tile count; LDS is reused between tiles)
    for (int tile = blockIdx.x;; tile += gridDim.x) {
        bool more;
        if constexpr (MODE == kRowsChanged)
            more = ffn_up_mfma_tile<GLU, MODE, WAVES>(matrix, bias, x, h, d, batch, capacity, row_elems, move_dst, tile,
                                                      pointers, gact, gact_n, st);
        else
            more = ffn_up_mfma_tile_staged<GLU, MODE, WAVES>(matrix, bias, x, h, d, batch, capacity, row_elems, tile,
                                                      spec != 0 && tile == (int)blockIdx.x, pointers, gact, gact_n, st);
        if (!more) break;
        __syncthreads();
    }
}

}  // namespace lif
