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

// grid = ceil(capacity / 16) workgroups of 256 threads; workgroup b owns cached rows 16b .. 16b+15
// and exits at once if they are not in use.  Its four waves take the k-steps w, w+4, w+8, ...
// (so the workgroup reads 256 contiguous bytes of every row per round) and their partial tiles
// are added in wave order through LDS.
// Fragment layout of the 16x16x32 MFMA: lane l supplies row (l mod 16) of A and column (l mod 16)
// of B for the k sub-block (l div 16); it receives D[4 * (l div 16) + r][l mod 16], r = 0..3.
// Here A = rows of the cache, B = tokens (columns >= batch are zero).
// Requires d % 32 == 0.
template <bool GLU>
__global__ __launch_bounds__(256) void k_ffn_up_mfma(const _Float16* __restrict__ matrix,
                                                     const float* __restrict__ bias,
                                                     const _Float16* __restrict__ x, float* __restrict__ h, int d,
                                                     int batch, int capacity, size_t row_elems,
                                                     const DevState* __restrict__ st) {
    __shared__ float red[GLU ? 2 : 1][4][64][4];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int i = lane & 15, q = lane >> 4;
    const int err = st->error;
    const int n = st->num_used;
    const int s0 = blockIdx.x * 16;
    if (err || s0 >= n) return;                                   // uniform

    const int srow = min(s0 + i, capacity - 1);                   // rows past the cache end repeat the last one; masked below
    const _Float16* grow = matrix + (size_t)srow * row_elems;
    const _Float16* urow = grow + (GLU ? d : 0);
    const bool xok = i < batch;
    const _Float16* xrow = x + (size_t)(xok ? i : 0) * d;
    const int nks = d >> 5;

    f32x4 cu = {0.f, 0.f, 0.f, 0.f}, cg = {0.f, 0.f, 0.f, 0.f};
    for (int ks0 = w; ks0 < nks; ks0 += 4 * kMfmaUnroll) {
        f16x8 uf[kMfmaUnroll], gf[GLU ? kMfmaUnroll : 1], xf[kMfmaUnroll];
#pragma unroll
        for (int u = 0; u < kMfmaUnroll; ++u) {
            const int ks = ks0 + 4 * u;
            const int off = (ks << 5) + (q << 3);
            const bool in = ks < nks;
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
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        red[0][w][lane][r] = cu[r];
        if (GLU) red[GLU ? 1 : 0][w][lane][r] = cg[r];
    }
    __syncthreads();
    if (w == 0 && xok) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = s0 + 4 * q + r;
            if (row < n) {
                const float su = ((red[0][0][lane][r] + red[0][1][lane][r]) + red[0][2][lane][r]) + red[0][3][lane][r];
                const float bs = bias[row];
                float act;
                if (GLU) {
                    const float sg = ((red[GLU ? 1 : 0][0][lane][r] + red[GLU ? 1 : 0][1][lane][r]) +
                                      red[GLU ? 1 : 0][2][lane][r]) + red[GLU ? 1 : 0][3][lane][r];
                    act = fmaxf(sg + bs, 0.f) * su;
                } else {
                    act = fmaxf(su + bs, 0.f);
                }
                h[(size_t)i * capacity + row] = act;
            }
        }
    }
}

}  // namespace lif

namespace lif {

#ifndef LIF_DOWNB_LANES
#define LIF_DOWNB_LANES 16
#endif
#ifndef LIF_DOWNB_UNROLL
#define LIF_DOWNB_UNROLL 4
#endif
#ifndef LIF_DOWNB_CHUNKS
#define LIF_DOWNB_CHUNKS 32
#endif
constexpr int kDownBLanes = LIF_DOWNB_LANES;     // lanes per row piece: 16 x 16 B = 256 contiguous bytes of a down column
constexpr int kDownChunks = LIF_DOWNB_CHUNKS;    // row chunks of the batched down projection (partial outputs per chunk)
constexpr int kDownBTile = 512;                  // cached rows whose activations sit in LDS per pass

// Row chunks actually used for n rows in use: about 256 rows per chunk, at most kDownChunks (the finish
// kernel applies the same rule, so unused chunks are neither written nor read).
__device__ __forceinline__ int down_chunks_in_use(int n) { return min(kDownChunks, max(1, (n + 255) / 256)); }

// Down projection for a batch of tokens: Y[t][j] = sum_s H[t][s] * D[s][j] over the rows in use.
// grid = (ceil(d / (kDownBLanes * VE)), kDownChunks), block = 256 = row groups x kDownBLanes lanes.
// Workgroup (slice, chunk) owns 256 contiguous bytes of every down column of the rows of its
// chunk (wide pieces keep HBM efficient when the rows come from memory): it compacts the rows
// that contribute (SKIP: some token's activation is non-zero), streams their 16-byte pieces
// once and updates all tokens from registers (8 FMAs per element: the VALU stays far below
// the memory time, so the matrix cores would only add a transpose here).  Partial outputs go
// to ypart[chunk][token][d] in fp32; k_ffn_down_finish adds the chunks in order.
template <typename T, int BT, bool SKIP>
__global__ __launch_bounds__(256) void k_ffn_down_batched(const T* __restrict__ matrix, const float* __restrict__ h,
                                                          float* __restrict__ ypart, int d, int batch, int capacity,
                                                          size_t row_elems, int down_off, DevState* __restrict__ st) {
    using V = typename Vec<T>::type;
    constexpr int VE = Vec<T>::N;
    constexpr int PER = kDownBTile / 256;
    constexpr int RG = 256 / kDownBLanes;            // row groups per workgroup
    __shared__ int list[kDownBTile];
    __shared__ float hv[BT][kDownBTile];
    __shared__ int wave_tot[4];
    __shared__ float red[4][kDownBLanes][BT][VE];
    __shared__ int n_active;

    const int tid = threadIdx.x, l = tid & (kDownBLanes - 1), rg = tid / kDownBLanes;
    const int col = blockIdx.x * (kDownBLanes * VE) + l * VE;
    const bool col_ok = col < d;
    const T* base = matrix + down_off + (col_ok ? col : 0);
    const int err = st->error;
    const int n = st->num_used;
    if (err) return;
    const int eff = down_chunks_in_use(n);
    if ((int)blockIdx.y >= eff) return;              // uniform: fewer, fatter chunks when few rows are in use
    const int per_chunk = (n + eff - 1) / eff;
    const int r0 = blockIdx.y * per_chunk, r1 = min(n, r0 + per_chunk);

    float acc[BT][VE];
#pragma unroll
    for (int b = 0; b < BT; ++b)
#pragma unroll
        for (int e = 0; e < VE; ++e) acc[b][e] = 0.f;
    if (tid == 0) n_active = 0;
    __syncthreads();

    for (int s_base = r0; s_base < r1; s_base += kDownBTile) {
        float hloc[PER][BT];
        unsigned flags = 0, nonzero = 0;
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            const int s = s_base + q * 256 + tid;
            bool any = false;
#pragma unroll
            for (int b = 0; b < BT; ++b) {
                const float v = (s < r1 && b < batch) ? h[(size_t)b * capacity + s] : 0.f;
                hloc[q][b] = v;
                any |= (v != 0.f);
            }
            if (any) nonzero |= 1u << q;
            if (!SKIP) any = s < r1;
            if (any) flags |= 1u << q;
        }
        if (blockIdx.x == 0 && nonzero) atomicAdd(&n_active, __popc(nonzero));   // statistics only
        int cnt;
        int off = block_exclusive_scan(__popc(flags), wave_tot, &cnt);
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            if (flags & (1u << q)) {
                list[off] = s_base + q * 256 + tid;
#pragma unroll
                for (int b = 0; b < BT; ++b) hv[b][off] = hloc[q][b];
                ++off;
            }
        }
        __syncthreads();
        if (col_ok) {
#pragma unroll LIF_DOWNB_UNROLL
            for (int i = rg; i < cnt; i += RG) {
                const V v = *reinterpret_cast<const V*>(base + (size_t)list[i] * row_elems);
#pragma unroll
                for (int b = 0; b < BT; ++b) {
                    const float hb = hv[b][i];
#pragma unroll
                    for (int e = 0; e < VE; ++e) acc[b][e] = __builtin_fmaf(hb, (float)v[e], acc[b][e]);
                }
            }
        }
        __syncthreads();
    }
    // the row groups of a wave sit kDownBLanes lanes apart: butterfly over the upper lane bits, then LDS over waves
#pragma unroll
    for (int b = 0; b < BT; ++b)
#pragma unroll
        for (int e = 0; e < VE; ++e) {
            float v = acc[b][e];
#pragma unroll
            for (int m = kDownBLanes; m < kWave; m <<= 1) v += __shfl_xor(v, m, kWave);
            if ((tid & 63) < kDownBLanes) red[tid >> 6][l][b][e] = v;
        }
    __syncthreads();
    if (blockIdx.x == 0 && tid == 0 && n_active) atomicAdd(&st->c_ffn_active, (unsigned long long)n_active);
    for (int idx = tid; idx < kDownBLanes * BT; idx += 256) {
        const int b = idx / kDownBLanes, l2 = idx - b * kDownBLanes;
        const int col2 = blockIdx.x * (kDownBLanes * VE) + l2 * VE;
        if (col2 < d && b < batch) {
            float* out = ypart + ((size_t)blockIdx.y * batch + b) * d + col2;
#pragma unroll
            for (int e = 0; e < VE; ++e)
                out[e] = ((red[0][l2][b][e] + red[1][l2][b][e]) + red[2][l2][b][e]) + red[3][l2][b][e];
        }
    }
}

// y[t][j] = sum over the chunks, in chunk order, rounded once to the element type.
template <typename T>
__global__ __launch_bounds__(256) void k_ffn_down_finish(const float* __restrict__ ypart, T* __restrict__ y, int d,
                                                         int batch, DevState* __restrict__ st) {
    if (st->error) return;
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < batch * d) {
        const int eff = down_chunks_in_use(st->num_used);
        float s = 0.f;
        for (int c = 0; c < eff; ++c) s += ypart[(size_t)c * batch * d + i];
        y[i] = (T)s;
    }
    if (i == 0) {
        st->c_ffn_calls += 1;
        st->c_ffn_rows += (unsigned long long)st->num_used;
    }
}

}  // namespace lif
