// Step 4: FFN over the cached rows (Section 3.3 item 3):
//   y = sum_{s < num_used} relu(up_s . x + bias_s) * down_s        (gated: relu(gate_s . x + bias_s) * (up_s . x))
//
// Two kernels, both pure streaming of bundle bytes (1 flop per byte at fp16).  At the sizes of
// one decode token (10-60 MB) they run a few microseconds, so what counts is the number of
// dependent memory round trips; each kernel has two (state + first loads, then the rest).
//   ffn_up    one wave per cached row: all 16-byte loads of the row's up (and gate) vector are
//             issued before the first use; the wave reduces the dot product and writes the
//             activation h[s].
//   ffn_down  one workgroup per slice of output columns: it owns those columns of y, so no
//             cross-workgroup reduction or atomics are needed and the summation order is
//             fixed.  It compacts the rows with a non-zero activation (prefix sum in LDS) and
//             streams only their down columns.  (A variant without compaction - predicated
//             loads over all rows - measured 1.6 us slower at the OPT-6.7B shape.)
#pragma once

#include "lif_common.h"

namespace lif {

// grid-stride over rows, block = 256 (4 waves, one row per wave at a time).
// NI = 16-byte loads per lane and vector (ceil(d / (64 * VE))).
// XREG (batch 1): every lane keeps its fragments of x in registers, loaded straight from
// global memory.  Otherwise x is staged once per workgroup in LDS (dynamic LDS: batch * d
// elements) and re-read per token.
// spec != 0: the first row of every wave is requested before the row count is known (slot <
// capacity is always valid memory; the result is dropped if the slot is not in use), so the
// state, x and the first rows travel in one round trip.  The host only asks for this when it
// was told how many rows to expect and has sized the grid to that many waves.
// `block` / `nblocks`: index and count of the workgroups that share this role; `n_ptr`: device
// address of the number of rows to cover (num_used, or the rows kept by a pending deletion).
// `gact` (may be null, plain bundles only): per-neuron gate activations relu(gate_i . x + b_i) written by the
// gate predictor (Appendix, Llama 2, "Alternative approaches": the resident gate projection is the predictor);
// the activation of slot s is then gact[pointers[s]] * (up_s . x).  gact_n = d_ffn bounds the lookup.
template <typename T, int NI, bool GLU, bool XREG>
__device__ __forceinline__ void ffn_up_role(const T* __restrict__ matrix, const float* __restrict__ bias,
                                            const T* __restrict__ x, float* __restrict__ h, int d, int batch,
                                            int capacity, size_t row_elems, int spec, int block, int nblocks,
                                            const int32_t* __restrict__ n_ptr, const int32_t* __restrict__ pointers,
                                            const float* __restrict__ gact, int gact_n,
                                            const DevState* __restrict__ st) {
    using V = typename Vec<T>::type;
    constexpr int VE = Vec<T>::N;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    V* xs = reinterpret_cast<V*>(smem_raw);
    const int tid = threadIdx.x, lane = tid & 63;
    const int nvec = d / VE;
    const int gw = block * 4 + (tid >> 6), nw = nblocks * 4;
    const V* xv = reinterpret_cast<const V*>(x);

    V xr[XREG ? NI : 1];
    if (XREG) {
#pragma unroll
        for (int it = 0; it < NI; ++it) {
            const int idx = it * 64 + lane;
            xr[it] = (idx < nvec) ? xv[idx] : V(0);
        }
    }
    // speculative first row
    V u[NI], g[GLU ? NI : 1];
    float bs = 0.f;
    if (spec) {
        const bool ok = gw < capacity;
        const V* row = reinterpret_cast<const V*>(matrix + (size_t)(ok ? gw : 0) * row_elems);
#pragma unroll
        for (int it = 0; it < NI; ++it) {
            const int idx = it * 64 + lane;
            const bool in = ok && idx < nvec;
            if (GLU) {
                g[it] = in ? row[idx] : V(0);
                u[it] = in ? row[nvec + idx] : V(0);
            } else {
                u[it] = in ? row[idx] : V(0);
            }
        }
        if (ok) bs = gact ? gact[min(max(pointers[gw], 0), gact_n - 1)] : bias[gw];
    }
    const int err = st->error;
    const int n = *n_ptr;
    if (err || block * 4 >= n) return;               // whole workgroup has no row (uniform)

    if (!XREG) {
        for (int i = tid; i < batch * nvec; i += 256) xs[i] = xv[i];
        __syncthreads();
    }

    for (int s = gw; s < n; s += nw) {
        if (s != gw || !spec) {                       // not requested yet: load now that the count is known
            const V* row = reinterpret_cast<const V*>(matrix + (size_t)s * row_elems);
#pragma unroll
            for (int it = 0; it < NI; ++it) {
                const int idx = it * 64 + lane;
                const bool in = idx < nvec;
                if (GLU) {
                    g[it] = in ? row[idx] : V(0);
                    u[it] = in ? row[nvec + idx] : V(0);
                } else {
                    u[it] = in ? row[idx] : V(0);
                }
            }
            bs = gact ? gact[min(max(pointers[s], 0), gact_n - 1)] : bias[s];
        }
        for (int b = 0; b < (XREG ? 1 : batch); ++b) {
            float du = 0.f, dg = 0.f;
#pragma unroll
            for (int it = 0; it < NI; ++it) {
                const int idx = it * 64 + lane;
                if (XREG) {
                    du = dot_acc(u[it], xr[it], du);              // both are 0 past the end of the vector
                    if (GLU) dg = dot_acc(g[it], xr[it], dg);
                } else if (idx < nvec) {
                    const V xb = xs[b * nvec + idx];
                    du = dot_acc(u[it], xb, du);
                    if (GLU) dg = dot_acc(g[it], xb, dg);
                }
            }
            du = wave_sum(du);
            float act;
            if (GLU) {
                dg = wave_sum(dg);
                act = fmaxf(dg + bs, 0.f) * du;
            } else if (gact) {
                act = bs * du;                        // resident gate: bs = relu(gate . x + bias) from the predictor
            } else {
                act = fmaxf(du + bs, 0.f);
            }
            if (lane == 0) h[(size_t)b * capacity + s] = act;
        }
    }
}

template <typename T, int NI, bool GLU, bool XREG>
__global__ __launch_bounds__(256) void k_ffn_up(const T* __restrict__ matrix, const float* __restrict__ bias,
                                                const T* __restrict__ x, float* __restrict__ h, int d, int batch,
                                                int capacity, size_t row_elems, int spec,
                                                const int32_t* __restrict__ pointers, const float* __restrict__ gact,
                                                int gact_n, const DevState* __restrict__ st) {
    ffn_up_role<T, NI, GLU, XREG>(matrix, bias, x, h, d, batch, capacity, row_elems, spec, blockIdx.x, gridDim.x,
                                  &st->num_used, pointers, gact, gact_n, st);
}

constexpr int kXcds = 8;            // accelerator complex dies of an MI355X, each with a private L2
constexpr int kDownLanes = 4;       // lanes per column slice (4 x 16 B = 64 B of every down column)
constexpr int kDownRg = 64;         // row groups per workgroup
constexpr int kDownTile = 2048;     // cached rows compacted per pass

// grid = ceil(d / (4 * VE)), block = 256 = 64 row groups x 4 lanes.
// SKIP: rows whose activation is zero for every token of the batch are not read.
// h_new / stamp (may be null): activations of the rows that the fused load kernel wrote during the
// step whose number equals stamp[s]; they override h for those rows.
template <typename T, int BT, bool SKIP>
__global__ __launch_bounds__(256) void k_ffn_down(const T* __restrict__ matrix, const float* __restrict__ h,
                                                  const float* __restrict__ h_new, const int32_t* __restrict__ stamp,
                                                  T* __restrict__ y, int d, int batch, int capacity,
                                                  size_t row_elems, int down_off, DevState* __restrict__ st) {
    using V = typename Vec<T>::type;
    constexpr int VE = Vec<T>::N;
    constexpr int TS = kDownTile / BT;
    constexpr int PER = TS / 256;                    // slots per thread in the compaction
    __shared__ int list[TS];
    __shared__ float hv[BT][TS];
    __shared__ int wave_tot[4];
    __shared__ float red[4][kDownLanes][BT][VE];
    __shared__ int n_active;

    const int tid = threadIdx.x, l = tid & (kDownLanes - 1), rg = tid >> 2;
    // XCD-aware slice order: workgroups are dealt round-robin to the 8 XCDs, each with its own L2.
    // A slice is 64 bytes wide, an L2 line 128: giving every XCD a contiguous run of slices makes
    // the two halves of a line meet in one L2 instead of being fetched by two.
    const int per_xcd = gridDim.x / kXcds;                   // the host rounds the grid up to a multiple of 8
    const int slice = (blockIdx.x % kXcds) * per_xcd + blockIdx.x / kXcds;
    const int col = slice * (kDownLanes * VE) + l * VE;
    const bool col_ok = col < d;
    const T* base = matrix + down_off + col;

    float acc[BT][VE];
#pragma unroll
    for (int b = 0; b < BT; ++b)
#pragma unroll
        for (int e = 0; e < VE; ++e) acc[b][e] = 0.f;

    if (tid == 0) n_active = 0;
    // the activations of the first tile are requested before the row count is known (the
    // activation array spans the whole capacity, so the addresses are valid; values past
    // num_used are masked below): one memory round trip less on the critical path
    float hfirst[PER][BT];
#pragma unroll
    for (int q = 0; q < PER; ++q)
#pragma unroll
        for (int b = 0; b < BT; ++b) {
            const int s = q * 256 + tid;
            hfirst[q][b] = (s < capacity && b < batch) ? h[(size_t)b * capacity + s] : 0.f;
        }
    int sfirst[PER];
#pragma unroll
    for (int q = 0; q < PER; ++q) {
        const int s = q * 256 + tid;
        sfirst[q] = (stamp && s < capacity) ? stamp[s] : -1;
    }
    const int err = st->error;
    const int n = err ? 0 : st->num_used;
    const int cur_step = st->step;
    if (stamp) {
#pragma unroll
        for (int q = 0; q < PER; ++q)
            if (sfirst[q] == cur_step) {
#pragma unroll
                for (int b = 0; b < BT; ++b)
                    if (b < batch) hfirst[q][b] = h_new[(size_t)b * capacity + q * 256 + tid];
            }
    }
    __syncthreads();
    if (err) return;
    for (int s_base = 0; s_base < n; s_base += TS) {
        // compaction of the rows that contribute, in a fixed order (thread-major over slots q * 256 + tid)
        float hloc[PER][BT];
        unsigned flags = 0, nonzero = 0;
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            const int s = s_base + q * 256 + tid;
            bool any = false;
#pragma unroll
            for (int b = 0; b < BT; ++b) {
                float v = 0.f;
                if (s < n && b < batch) {
                    if (s_base == 0) v = hfirst[q][b];
                    else v = (stamp && stamp[s] == cur_step) ? h_new[(size_t)b * capacity + s]
                                                             : h[(size_t)b * capacity + s];
                }
                hloc[q][b] = v;
                any |= (v != 0.f);
            }
            if (any) nonzero |= 1u << q;
            if (!SKIP) any = s < n;
            if (any) flags |= 1u << q;
        }
        if (slice == 0 && nonzero) atomicAdd(&n_active, __popc(nonzero));   // statistics only
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
#pragma unroll 4
            for (int i = rg; i < cnt; i += kDownRg) {
                const int s = list[i];
                const V v = *reinterpret_cast<const V*>(base + (size_t)s * row_elems);
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
    // row groups of one wave sit 4 lanes apart: butterfly over lane bits 2..5, then LDS over waves
#pragma unroll
    for (int b = 0; b < BT; ++b)
#pragma unroll
        for (int e = 0; e < VE; ++e) {
            float v = acc[b][e];
            v += __shfl_xor(v, 4, kWave);
            v += __shfl_xor(v, 8, kWave);
            v += __shfl_xor(v, 16, kWave);
            v += __shfl_xor(v, 32, kWave);
            if ((tid & 63) < kDownLanes) red[tid >> 6][l][b][e] = v;
        }
    __syncthreads();
    if (slice == 0 && tid == 0) {
        st->c_ffn_calls += 1;
        st->c_ffn_rows += (unsigned long long)n;
        st->c_ffn_active += (unsigned long long)n_active;
    }
    if (tid < kDownLanes * BT) {
        const int b = tid / kDownLanes, l2 = tid - b * kDownLanes;
        const int col2 = slice * (kDownLanes * VE) + l2 * VE;
        if (col2 < d && b < batch) {
            V out;
#pragma unroll
            for (int e = 0; e < VE; ++e)
                out[e] = (T)(((red[0][l2][b][e] + red[1][l2][b][e]) + red[2][l2][b][e]) + red[3][l2][b][e]);
            *reinterpret_cast<V*>(y + (size_t)b * d + col2) = out;
        }
    }
}

}  // namespace lif
