// Step 1: low-rank predictor  mask_i = [ ((x A) B)_i + c_i > theta ]
// (Section 3.1 "Anticipating ReLU Sparsity", Fig. 3b; active = strictly positive output).
//
// Both contractions accumulate in fp64: every product of two fp16 or two fp32 values is
// exact in fp64, so the result depends on the summation order only at the 1e-16 level
// and the thresholded bits can be compared bit for bit with a CPU evaluation.  The path
// stays bandwidth bound (one fp64 FMA per 2 or 4 bytes read).
//
// Both kernels are a few microseconds long, i.e. latency bound: each issues all of its
// global loads (weights, offsets, state) before the first dependent use.
#pragma once

#include <type_traits>

#include "lif_common.h"

namespace lif {

// acc + sum_q a[q] * b[q] with every product and sum in fp64.  A product of two fp16 values is exact in fp32
// (22 significant bits, exponents far inside the fp32 range), so for fp16 it is formed there and widened once:
// the same bits as widening both factors, at half the conversions.
__device__ __forceinline__ double dot_f64(f16x8 a, f16x8 b, double acc) {
#pragma unroll
    for (int q = 0; q < 8; ++q) acc += (double)((float)a[q] * (float)b[q]);
    return acc;
}
__device__ __forceinline__ double dot_f64(f32x4 a, f32x4 b, double acc) {
#pragma unroll
    for (int q = 0; q < 4; ++q) acc = __builtin_fma((double)a[q], (double)b[q], acc);
    return acc;
}

constexpr int kMaskCols = 8;       // mask bytes (groups of 8 neurons) per workgroup of predict_mask
constexpr int kMaskJg = 32;        // rank groups per workgroup of predict_mask
constexpr int kMaskRows = 8;       // rows of B a thread keeps in flight

// t[b][j] = sum_i x[b][i] * At[j][i]   (At = the first predictor matrix with the contraction dimension
// contiguous, [r x d]).  One wave per (j, b): 16-byte loads along the row, fp64 accumulation, wave
// reduction - every t[b][j] is complete after this kernel, so the mask kernel needs no partial sums.
// grid = (ceil(r / 4), batch), block = 256.  NI = ceil(d / (64 * VE)) loads per lane.
template <typename T, int NI>
__global__ __launch_bounds__(256) void k_predict_xa(const T* __restrict__ x, const T* __restrict__ At,
                                                    double* __restrict__ t, int d, int r,
                                                    const DevState* __restrict__ st) {
    using V = typename Vec<T>::type;
    constexpr int VE = Vec<T>::N;
    const int lane = threadIdx.x & 63;
    const int j = blockIdx.x * 4 + (threadIdx.x >> 6), b = blockIdx.y;
    if (j >= r) return;                              // wave-uniform; the kernel has no barrier
    const int nvec = d / VE;
    const V* xv = reinterpret_cast<const V*>(x + (size_t)b * d);
    const V* row = reinterpret_cast<const V*>(At + (size_t)j * d);
    V a[NI], xr[NI];
#pragma unroll
    for (int it = 0; it < NI; ++it) {
        const int idx = it * 64 + lane;
        a[it] = (idx < nvec) ? row[idx] : V(0);
        xr[it] = (idx < nvec) ? xv[idx] : V(0);
    }
    const int err = st->error;
    double acc = 0.0;
#pragma unroll
    for (int it = 0; it < NI; ++it) acc = dot_f64(a[it], xr[it], acc);
    acc = wave_sum(acc);
    if (lane == 0 && !err) t[(size_t)b * r + j] = acc;
}

// logits = t B + c, threshold, pack 8 neurons per byte; step mask = OR over the batch.
// grid = ceil(F / 64), block = 256 = 32 rank groups x 8 column lanes; each column lane owns
// 8 consecutive neurons = one mask byte.  dynamic LDS: BT * r doubles (t of the tokens of a pass).
template <typename T, int BT>
__global__ __launch_bounds__(256) void k_predict_mask(const T* __restrict__ B, const float* __restrict__ c,
                                                      const double* __restrict__ t, int r, int F, int batch,
                                                      float theta,
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
    // one token per pass: the kMaskRows values of t this thread multiplies with come straight from global memory,
    // requested with the rows (no staging in LDS, no barriers in front of the multiply-adds)
    double tr[BT == 1 ? kMaskRows : 1];
    if (BT == 1) {
#pragma unroll
        for (int u = 0; u < kMaskRows; ++u) tr[u] = t[min(jg + u * kMaskJg, r - 1)];
    }
    const int err = st->error;

    for (int b0 = 0; b0 < batch; b0 += BT) {
        if (BT == 1 && r <= kMaskRows * kMaskJg && b0 > 0) __syncthreads();   // red is still read from the pass before
        if (BT > 1 || r > kMaskRows * kMaskJg) {
            __syncthreads();
            for (int idx = tid; idx < BT * r; idx += 256) {
                const int bt = idx / r, j = idx - bt * r;
                tl[idx] = (b0 + bt < batch) ? t[(size_t)(b0 + bt) * r + j] : 0.0;
            }
            __syncthreads();
        }
        if (BT == 1 && b0 > 0) {                     // batches served token by token (large ranks)
#pragma unroll
            for (int u = 0; u < kMaskRows; ++u) tr[u] = t[(size_t)b0 * r + min(jg + u * kMaskJg, r - 1)];
        }

        double v[BT * 8];                    // v[bt * 8 + e]: logit sums of token bt, neuron e of this lane's byte
#pragma unroll
        for (int i = 0; i < BT * 8; ++i) v[i] = 0.0;
#pragma unroll
        for (int u = 0; u < kMaskRows; ++u) {
            const int j = min(jg + u * kMaskJg, r - 1);           // bv[u] is 0 past the end
#pragma unroll
            for (int bt = 0; bt < BT; ++bt) {
                const double tj = (BT == 1) ? tr[u] : tl[bt * r + j];
#pragma unroll
                for (int q = 0; q < LPB; ++q)
#pragma unroll
                    for (int e = 0; e < VE; ++e)
                        v[bt * 8 + q * VE + e] = __builtin_fma(tj, (double)bv[u][q][e], v[bt * 8 + q * VE + e]);
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
                            v[bt * 8 + q * VE + e] = __builtin_fma(tj, (double)bw[q][e], v[bt * 8 + q * VE + e]);
                }
            }
        }
        // The eight rank groups of a wave sit 8 lanes apart (lane bits 3..5): butterfly over those bits, then LDS
        // across the 4 waves.  While a lane still holds the sums of more than one token, a step halves them: the
        // lane keeps the tokens selected by its own bit and hands the other half to its partner (56 exchanges
        // instead of 192 for 8 tokens).  Afterwards lane (g, cl), g = lane bits 3..5, holds the 8 sums of token
        // `owner` (all lanes for BT = 8; even g / g = 0 only for fewer tokens).
        int owner = 0;
        auto halve = [&](auto half_c, int m) {       // keep the half selected by this lane's bit m, add the partner's
            constexpr int half = decltype(half_c)::value;
            const bool up = (tid & m) != 0;
#pragma unroll
            for (int i = 0; i < half; ++i) {
                const double send = up ? v[i] : v[i + half], keep = up ? v[i + half] : v[i];
                // lanes 8 apart sit in one row of 16: a rotation by 8 (DPP) instead of a shuffle through LDS
                v[i] = keep + (m == 8 ? dpp_from<0x128, 0xf>(send) : __shfl_xor(send, m, kWave));
            }
            owner = owner * 2 + (up ? 1 : 0);
        };
        auto full = [&](int m) {
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] += (m == 8 ? dpp_from<0x128, 0xf>(v[i]) : __shfl_xor(v[i], m, kWave));
        };
        if constexpr (BT == 8) {
            halve(std::integral_constant<int, 32>{}, 32);
            halve(std::integral_constant<int, 16>{}, 16);
            halve(std::integral_constant<int, 8>{}, 8);
        } else if constexpr (BT == 4) {
            halve(std::integral_constant<int, 16>{}, 32);
            halve(std::integral_constant<int, 8>{}, 16);
            full(8);
        } else {
            // one token: the 8 neurons of the byte are halved the same way (7 exchanges instead of 24), the step over
            // lanes 8 apart first, while a lane still holds all 8: lane (g, cl) ends with neuron `owner`
            halve(std::integral_constant<int, 4>{}, 8);
            halve(std::integral_constant<int, 2>{}, 16);
            halve(std::integral_constant<int, 1>{}, 32);
        }
        // which lanes hold a finished token: those whose bits of the non-halving steps are zero
        constexpr int kHalvings = (BT == 8) ? 3 : (BT == 4) ? 2 : 0;
        const bool holder = ((tid & 63) & ((64 >> kHalvings) - 8)) == 0;
        if (BT == 1) {
            red[wave][cl][0][owner] = v[0];
        } else if (holder) {
#pragma unroll
            for (int e = 0; e < 8; ++e) red[wave][cl][owner][e] = v[e];
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
            if (BT == 1) or_byte |= byte;            // one token per pass: this thread owns column tid of the step mask
            else bytes[bt][c2] = byte;
        }
        if (BT > 1) {
            __syncthreads();
            if (tid < kMaskCols) {
#pragma unroll
                for (int bt = 0; bt < BT; ++bt) or_byte |= bytes[bt][tid];
            }
        }
    }
    if (tid < kMaskCols && n0 < F && !err) step_mask[n0 >> 3] = or_byte;
}

// Gate projection as the predictor (Appendix, Llama 2, "Alternative approaches"): the gate matrix stays
// resident and  a_i = gate_i . x + b_i  decides exactly which neurons fire (mask bit = a_i > theta); the same
// pass leaves relu(a_i) per token and neuron for the FFN, so bundles hold only up row | down column.
// One wave per group of 8 neurons (one mask byte per token): 16-byte loads along the row, fp64 accumulation
// (bit-exact decision), wave reduction.  grid-stride over F / 8 groups, block = 256.  NI as in the FFN kernels.
// XREG (one token): x stays in registers.  Otherwise the tokens' x are staged in LDS (dynamic LDS: batch * d
// elements) and every gate row, loaded once, is applied to each token in turn; masks [batch x F/8], step mask = OR
// over the tokens, gact [batch x F].
template <typename T, int NI, bool XREG>
__global__ __launch_bounds__(256) void k_predict_gate(const T* __restrict__ Wg, const float* __restrict__ b,
                                                      const T* __restrict__ x, int d, int F, int batch, float theta,
                                                      uint8_t* __restrict__ mask, uint8_t* __restrict__ step_mask,
                                                      float* __restrict__ gact, const DevState* __restrict__ st) {
    using V = typename Vec<T>::type;
    constexpr int VE = Vec<T>::N;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_gate[];
    V* xs = reinterpret_cast<V*>(smem_gate);
    const int tid = threadIdx.x, lane = tid & 63;
    const int nvec = d / VE;
    const int gw = blockIdx.x * 4 + (tid >> 6), nw = gridDim.x * 4;
    const V* xv = reinterpret_cast<const V*>(x);
    V xr[XREG ? NI : 1];
    if (XREG) {
#pragma unroll
        for (int it = 0; it < NI; ++it) {
            const int idx = it * 64 + lane;
            xr[it] = (idx < nvec) ? xv[idx] : V(0);
        }
    } else {
        for (int i = tid; i < batch * nvec; i += 256) xs[i] = xv[i];
        __syncthreads();
    }
    if (st->error) return;
    const double th = (double)theta;
    const int mask_stride = F >> 3;
    for (int grp = gw; grp * 8 < F; grp += nw) {
        unsigned long long bits = 0;                 // bit 8 * token + e: neuron grp * 8 + e fires for that token
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
            const double bi = (double)b[i];
            for (int t = 0; t < (XREG ? 1 : batch); ++t) {
                double acc = 0.0;
#pragma unroll
                for (int it = 0; it < NI; ++it) {
                    const int idx = it * 64 + lane;
                    if (XREG) acc = dot_f64(g[it], xr[it], acc);          // both are 0 past the end of the vector
                    else if (idx < nvec) acc = dot_f64(g[it], xs[t * nvec + idx], acc);
                }
                acc = wave_sum(acc);
                const double a = acc + bi;
                if (a > th) bits |= 1ull << (8 * t + e);
                if (lane == 0) gact[(size_t)t * F + i] = (float)(a > 0.0 ? a : 0.0);
            }
        }
        if (XREG) {
            if (lane == 0) {
                mask[grp] = (uint8_t)bits;
                if (step_mask != mask) step_mask[grp] = (uint8_t)bits;   // one token: the step mask is the mask
            }
        } else {
            if (lane < batch) mask[(size_t)lane * mask_stride + grp] = (uint8_t)(bits >> (8 * lane));
            if (lane == 0) {
                unsigned long long o = bits | (bits >> 32);
                o |= o >> 16;
                o |= o >> 8;
                step_mask[grp] = (uint8_t)o;
            }
        }
    }
}

}  // namespace lif
