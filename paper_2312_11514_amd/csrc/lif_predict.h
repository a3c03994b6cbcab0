// Step 1: low-rank predictor  mask_i = [ ((x A) B)_i + c_i > theta ]
// (Section 3.1 "Anticipating ReLU Sparsity", Fig. 3b; active = strictly positive output).
//
// Both contractions accumulate in fp64: every product of two fp16 or two fp32 values is
// exact in fp64, so the result depends on the summation order only at the 1e-16 level
// and the thresholded bits can be compared bit for bit with a CPU evaluation.  The path
// stays bandwidth bound (one fp64 FMA per 2 or 4 bytes read).
//
// Both kernels are a few microseconds long, i.e. latency bound: each issues all of its
// global loads (weights, partial sums, offsets, state) before the first dependent use.
#pragma once

#include "lif_common.h"

namespace lif {

constexpr int kXaRows = 256;       // rows of A per workgroup of predict_xa
constexpr int kXaBatch = 16;       // rows of A a thread keeps in flight
constexpr int kMaskCols = 8;       // mask bytes (groups of 8 neurons) per workgroup of predict_mask
constexpr int kMaskJg = 32;        // rank groups per workgroup of predict_mask
constexpr int kMaskRows = 8;       // rows of B a thread keeps in flight

// t_partial[b][chunk][j] = sum_{i in chunk} x[b][i] * A[i][j]
// grid = (ceil(d / kXaRows), batch), block = 256.
// Thread (rl, cl): column lanes cl cover a row of A with 16-byte loads, rl strides rows.
template <typename T>
__global__ __launch_bounds__(256) void k_predict_xa(const T* __restrict__ x, const T* __restrict__ A,
                                                    double* __restrict__ tpart, int d, int r,
                                                    const DevState* __restrict__ st) {
    using V = typename Vec<T>::type;
    constexpr int VE = Vec<T>::N;
    __shared__ float xs[kXaRows];
    __shared__ double red[256 * VE];

    const int tid = threadIdx.x;
    const int lpr = r / VE;                 // lanes per row (host guarantees 1 <= lpr <= 256)
    const int rp = 256 / lpr;               // rows per pass
    const int rl = tid / lpr, cl = tid - rl * lpr;
    const int chunk = blockIdx.x, b = blockIdx.y, nchunks = gridDim.x;
    const int row0 = chunk * kXaRows;
    const int nrows = min(kXaRows, d - row0);
    const bool lane_ok = rl < rp;
    const V* __restrict__ Av = reinterpret_cast<const V*>(A) + (size_t)row0 * lpr + cl;

    // loads first: x, the first batch of A rows, the error flag
    const float xreg = (tid < nrows) ? (float)x[(size_t)b * d + row0 + tid] : 0.f;
    V a[kXaBatch];
#pragma unroll
    for (int u = 0; u < kXaBatch; ++u) {
        const int i = rl + u * rp;
        a[u] = (lane_ok && i < nrows) ? Av[(size_t)i * lpr] : V(0);
    }
    const int err = st->error;
    xs[tid] = xreg;
    __syncthreads();

    double acc[VE];
#pragma unroll
    for (int e = 0; e < VE; ++e) acc[e] = 0.0;
#pragma unroll
    for (int u = 0; u < kXaBatch; ++u) {
        const int i = rl + u * rp;
        const double xv = (double)xs[min(i, kXaRows - 1)];
#pragma unroll
        for (int e = 0; e < VE; ++e) acc[e] = __builtin_fma(xv, (double)a[u][e], acc[e]);   // a[u] is 0 past the end
    }
    if (lane_ok) {
        for (int i = rl + kXaBatch * rp; i < nrows; i += rp) {     // only when rank / VE > 16
            const V av = Av[(size_t)i * lpr];
            const double xv = (double)xs[i];
#pragma unroll
            for (int e = 0; e < VE; ++e) acc[e] = __builtin_fma(xv, (double)av[e], acc[e]);
        }
    }
#pragma unroll
    for (int e = 0; e < VE; ++e) red[tid * VE + e] = acc[e];
    __syncthreads();
    if (err) return;
    // column j lives in lane cl = j / VE, element e = j % VE; rows-in-pass summed ascending
    for (int j = tid; j < r; j += 256) {
        const int jc = j / VE, je = j - jc * VE;
        double s = 0.0;
        for (int q = 0; q < rp; ++q) s += red[(q * lpr + jc) * VE + je];
        tpart[((size_t)b * nchunks + chunk) * r + j] = s;
    }
}

// logits = t B + c, threshold, pack 8 neurons per byte; step mask = OR over the batch.
// grid = ceil(F / 64), block = 256 = 32 rank groups x 8 column lanes; each column lane owns
// 8 consecutive neurons = one mask byte.  t = sum of the chunk partials, reduced redundantly
// by every workgroup in a fixed order.  dynamic LDS: BT * r doubles.
template <typename T, int BT>
__global__ __launch_bounds__(256) void k_predict_mask(const T* __restrict__ B, const float* __restrict__ c,
                                                      const double* __restrict__ tpart, int nchunks, int r,
                                                      int F, int batch, float theta,
                                                      uint8_t* __restrict__ masks, uint8_t* __restrict__ step_mask,
                                                      const DevState* __restrict__ st) {
    using V = typename Vec<T>::type;
    constexpr int VE = Vec<T>::N;
    constexpr int LPB = 8 / VE;             // 16-byte loads per group of 8 neurons
    extern __shared__ double tl[];          // [BT][r]
    __shared__ double red[4][kMaskCols][BT][8];
    __shared__ uint8_t bytes[BT][kMaskCols];

    const int tid = threadIdx.x, wave = tid >> 6;
    const int cl = tid & (kMaskCols - 1), jg = tid >> 3;
    const int n0 = (blockIdx.x * kMaskCols + cl) * 8;
    const bool col_ok = n0 < F;
    const int mask_stride = F >> 3;
    const double th = (double)theta;
    uint8_t or_byte = 0;

    // loads that do not depend on t: the first kMaskRows rows of B of this thread, the offsets, the flag
    V bv[kMaskRows][LPB];
#pragma unroll
    for (int u = 0; u < kMaskRows; ++u) {
        const int j = jg + u * kMaskJg;
#pragma unroll
        for (int q = 0; q < LPB; ++q)
            bv[u][q] = (col_ok && j < r) ? reinterpret_cast<const V*>(B + (size_t)j * F + n0)[q] : V(0);
    }
    float cv[8];
    {
        const int c2 = tid & (kMaskCols - 1);
        const int n2 = (blockIdx.x * kMaskCols + c2) * 8;
#pragma unroll
        for (int e = 0; e < 8; ++e) cv[e] = (c && tid < kMaskCols * BT && n2 < F) ? c[n2 + e] : 0.f;
    }
    const int err = st->error;

    for (int b0 = 0; b0 < batch; b0 += BT) {
        __syncthreads();
        for (int idx = tid; idx < BT * r; idx += 256) {
            const int bt = idx / r, j = idx - bt * r;
            double s = 0.0;
            if (b0 + bt < batch) {
                const double* p = tpart + ((size_t)(b0 + bt) * nchunks) * r + j;
#pragma unroll 8
                for (int ch = 0; ch < nchunks; ++ch) s += p[(size_t)ch * r];
            }
            tl[idx] = s;
        }
        __syncthreads();

        double acc[BT][8];
#pragma unroll
        for (int bt = 0; bt < BT; ++bt)
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[bt][e] = 0.0;
#pragma unroll
        for (int u = 0; u < kMaskRows; ++u) {
            const int j = min(jg + u * kMaskJg, r - 1);           // bv[u] is 0 past the end
#pragma unroll
            for (int bt = 0; bt < BT; ++bt) {
                const double tj = tl[bt * r + j];
#pragma unroll
                for (int q = 0; q < LPB; ++q)
#pragma unroll
                    for (int e = 0; e < VE; ++e)
                        acc[bt][q * VE + e] = __builtin_fma(tj, (double)bv[u][q][e], acc[bt][q * VE + e]);
            }
        }
        if (col_ok) {
            for (int j = jg + kMaskRows * kMaskJg; j < r; j += kMaskJg) {      // only when rank > 256
                const V* bp = reinterpret_cast<const V*>(B + (size_t)j * F + n0);
                V bw[LPB];
#pragma unroll
                for (int q = 0; q < LPB; ++q) bw[q] = bp[q];
#pragma unroll
                for (int bt = 0; bt < BT; ++bt) {
                    const double tj = tl[bt * r + j];
#pragma unroll
                    for (int q = 0; q < LPB; ++q)
#pragma unroll
                        for (int e = 0; e < VE; ++e)
                            acc[bt][q * VE + e] = __builtin_fma(tj, (double)bw[q][e], acc[bt][q * VE + e]);
                }
            }
        }
        // the eight rank groups of a wave sit 8 lanes apart: butterfly, then LDS across the 4 waves
#pragma unroll
        for (int bt = 0; bt < BT; ++bt)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                double v = acc[bt][e];
                v += __shfl_xor(v, 8, kWave);
                v += __shfl_xor(v, 16, kWave);
                v += __shfl_xor(v, 32, kWave);
                if ((tid & 63) < kMaskCols) red[wave][cl][bt][e] = v;
            }
        __syncthreads();
        if (tid < kMaskCols * BT) {
            const int bt = tid / kMaskCols, c2 = tid - bt * kMaskCols;
            const int n2 = (blockIdx.x * kMaskCols + c2) * 8;
            uint8_t byte = 0;
            if (n2 < F && b0 + bt < batch) {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    double z = ((red[0][c2][bt][e] + red[1][c2][bt][e]) + red[2][c2][bt][e]) + red[3][c2][bt][e];
                    z += (double)cv[e];
                    if (z > th) byte |= (uint8_t)(1u << e);
                }
                if (!err) masks[(size_t)(b0 + bt) * mask_stride + (n2 >> 3)] = byte;
            }
            bytes[bt][c2] = byte;
        }
        __syncthreads();
        if (tid < kMaskCols) {
#pragma unroll
            for (int bt = 0; bt < BT; ++bt) or_byte |= bytes[bt][tid];
        }
    }
    if (tid < kMaskCols && n0 < F && !err) step_mask[n0 >> 3] = or_byte;
}

// Gate projection as the predictor (Appendix, Llama 2, "Alternative approaches"): the gate matrix stays
// resident and  a_i = gate_i . x + b_i  decides exactly which neurons fire (mask bit = a_i > theta); the same
// pass leaves relu(a_i) per neuron for the FFN, so bundles hold only up row | down column.
// One wave per group of 8 neurons (one mask byte): 16-byte loads along the row, fp64 accumulation (bit-exact
// decision), wave reduction.  grid-stride over F / 8 groups, block = 256.  NI as in the FFN kernels.
template <typename T, int NI>
__global__ __launch_bounds__(256) void k_predict_gate(const T* __restrict__ Wg, const float* __restrict__ b,
                                                      const T* __restrict__ x, int d, int F, float theta,
                                                      uint8_t* __restrict__ mask, float* __restrict__ gact,
                                                      const DevState* __restrict__ st) {
    using V = typename Vec<T>::type;
    constexpr int VE = Vec<T>::N;
    const int tid = threadIdx.x, lane = tid & 63;
    const int nvec = d / VE;
    const int gw = blockIdx.x * 4 + (tid >> 6), nw = gridDim.x * 4;
    const V* xv = reinterpret_cast<const V*>(x);
    V xr[NI];
#pragma unroll
    for (int it = 0; it < NI; ++it) {
        const int idx = it * 64 + lane;
        xr[it] = (idx < nvec) ? xv[idx] : V(0);
    }
    if (st->error) return;
    const double th = (double)theta;
    for (int grp = gw; grp * 8 < F; grp += nw) {
        unsigned byte = 0;
        float keep_act = 0.f;
#pragma unroll 2
        for (int e = 0; e < 8; ++e) {
            const int i = grp * 8 + e;
            const V* row = reinterpret_cast<const V*>(Wg + (size_t)i * d);
            V g[NI];
#pragma unroll
            for (int it = 0; it < NI; ++it) {
                const int idx = it * 64 + lane;
                g[it] = (idx < nvec) ? row[idx] : V(0);
            }
            double acc = 0.0;
#pragma unroll
            for (int it = 0; it < NI; ++it)
#pragma unroll
                for (int q = 0; q < VE; ++q) acc = __builtin_fma((double)g[it][q], (double)xr[it][q], acc);
#pragma unroll
            for (int msk = 32; msk >= 1; msk >>= 1) acc += __shfl_xor(acc, msk, kWave);
            const double a = acc + (double)b[i];
            if (a > th) byte |= 1u << e;
            if (lane == e) keep_act = (float)(a > 0.0 ? a : 0.0);
        }
        if (lane == 0) mask[grp] = (uint8_t)byte;
        if (lane < 8) gact[grp * 8 + lane] = keep_act;
    }
}

}  // namespace lif
