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

#ifndef LIF_MFMA_UNROLL
#define LIF_MFMA_UNROLL 8
#endif
constexpr int kMfmaUnroll = LIF_MFMA_UNROLL;     // k-steps (32 elements each) a wave keeps in flight

// grid = ceil(capacity / 16) workgroups of 256 threads; workgroup b owns cached rows 16b .. 16b+15
// and exits at once if they are not in use.  Each of its four waves takes a contiguous quarter of the
// k-steps (a wave instruction reads 64 bytes of 16 rows; consecutive instructions of one wave then
// complete whole 128-byte lines: measured 6.5 TB/s against 4.6 TB/s when the waves interleave
// k-steps) and the partial tiles are added in wave order through LDS.
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
    const int per = (nks + 3) >> 2;                               // k-steps per wave: a contiguous quarter of the row
    const int ks_begin = w * per, ks_end = min(nks, ks_begin + per);
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
