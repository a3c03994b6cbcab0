// Step 4: FFN over the cached rows (Section 3.3 item 3):
//   y = sum_{s < num_used} relu(up_s . x + bias_s) * down_s        (gated: relu(gate_s . x + bias_s) * (up_s . x))
//
// Two kernels, both pure streaming of bundle bytes (1 flop per byte at fp16).  At the sizes of
// one decode token (10-60 MB) they run a few microseconds, so what counts is the number of
// dependent memory round trips; each kernel has two (state + first loads, then the rest).
//   ffn_up    one wave per cached row: all 16-byte loads of the row's up (and gate) vector are
//             issued before the first use; the wave reduces the dot product and writes the
//             activation h[s].
//   ffn_down  workgroups per slice of output columns (and per chunk of rows once the cache is large): no
//             atomics, fixed summation order.  It compacts the rows with a non-zero activation
//             (prefix sum in LDS) and streams only their down columns.  (A variant without
//             compaction - predicated loads over all rows - measured 1.6 us slower at the
//             OPT-6.7B shape.)
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
// the activation of slot s for token t is then gact[t][pointers[s]] * (up_s . x_t), gact [batch x gact_n];
// gact_n = d_ffn bounds the lookup.
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
        if (ok) bs = gact ? gact[min(max(pointers[gw], 0), gact_n - 1)] : bias[gw];     // token 0 (the only one if XREG)
    }
    const int err = st->error;
    const int n = *n_ptr;
    if (err || block * 4 >= n) return;               // whole workgroup has no row (uniform)

    if (!XREG) {
        for (int i = tid; i < batch * nvec; i += 256) xs[i] = xv[i];
        __syncthreads();
    }

    if (!spec && gw < n) {                            // not requested yet: load now that the count is known
        const V* row = reinterpret_cast<const V*>(matrix + (size_t)gw * row_elems);
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
        bs = gact ? gact[min(max(pointers[gw], 0), gact_n - 1)] : bias[gw];
    }
    for (int s = gw; s < n; s += nw) {
        // the next row of this wave is requested before the current one is reduced (when the grid is
        // smaller than the row count, every wave keeps two rows in flight)
        const int sn = s + nw;
        V un[NI], gn[GLU ? NI : 1];
        float bsn = 0.f;
        if (sn < n) {
            const V* row = reinterpret_cast<const V*>(matrix + (size_t)sn * row_elems);
#pragma unroll
            for (int it = 0; it < NI; ++it) {
                const int idx = it * 64 + lane;
                const bool in = idx < nvec;
                if (GLU) {
                    gn[it] = in ? row[idx] : V(0);
                    un[it] = in ? row[nvec + idx] : V(0);
                } else {
                    un[it] = in ? row[idx] : V(0);
                }
            }
            bsn = gact ? gact[min(max(pointers[sn], 0), gact_n - 1)] : bias[sn];
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
                // resident gate: relu(gate . x_b + bias) from the predictor (bs holds token 0's)
                const float gb = (XREG || b == 0) ? bs
                                                  : gact[(size_t)b * gact_n + min(max(pointers[s], 0), gact_n - 1)];
                act = gb * du;
            } else {
                act = fmaxf(du + bs, 0.f);
            }
            if (lane == 0) h[(size_t)b * capacity + s] = act;
        }
        if (sn < n) {
#pragma unroll
            for (int it = 0; it < NI; ++it) {
                u[it] = un[it];
                if (GLU) g[it] = gn[it];
            }
            bs = bsn;
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

constexpr int kUpMaxWgs = 1024;   // workgroups of the activation stage: beyond this, waves loop over rows (x stays in registers)

constexpr int kXcds = 8;            // accelerator complex dies of an MI355X, each with a private L2
constexpr int kDownTile = 2048;     // activations (rows x tokens) compacted per pass (at least 512 rows)
constexpr int kDownChunksMax = 32;  // row chunks of the down projection (partial outputs per chunk)
constexpr int kDownLanesB = 16;       // lanes per column slice for several tokens
constexpr int kDownLanes1 = 4;        // ... single token skipping dead rows (latency bound)
constexpr int kDownLanesN = 8;        // ... when most rows are read: 8 x 16 B = one 128-byte line per row
constexpr int kDownRowsSparse = 4096; // rows per chunk: single token, rows without activation skipped
constexpr int kDownRowsDense = 512;   // ... single token, every row read
constexpr int kDownRowsBatch = 512;   // ... several tokens

// Row chunks in use for n cached rows.  For a single token and up to 4096 rows (1024 in full-bundle mode), one
// chunk (one workgroup per column slice, no partial sums) is the shortest path: the kernel is latency bound
// there.  Beyond that, the single-token
// case that skips rows without activation keeps chunks of 4096 rows (one compaction pass each; few rows
// contribute); when most rows are read (full-bundle mode, or several tokens whose active sets add up) a
// chunk is 512 rows so that several hundred workgroups stream at once: column slices alone (d / 64
// workgroups) reach only about 3 TB/s.  The host sizes the grid with the same rule.
template <int BT, bool SKIP>
__host__ __device__ __forceinline__ int down_chunks(int n) {
    constexpr int per = (BT == 1 && SKIP) ? kDownRowsSparse : (BT == 1 ? kDownRowsDense : kDownRowsBatch);
    if (BT == 1 && n <= (SKIP ? kDownRowsSparse : 2 * kDownRowsDense)) return 1;
    const int c = (n + per - 1) / per;
    return c < 1 ? 1 : (c > kDownChunksMax ? kDownChunksMax : c);
}

// Down projection  y[t][j] = sum_s H[t][s] * D[s][j]  over the rows in use, for 1..BT tokens.
// grid = (column slices, row-chunk workgroups), block = 256 = (256 / LANES) row groups x LANES lanes; a
// lane owns 16 bytes of every down column it reads, a workgroup LANES * 16 contiguous bytes.
// SKIP: rows whose activation is zero for every token of the batch are not read (they are compacted
// away with a prefix sum in LDS, in a fixed order).
// h_new / stamp (may be null): activations of the rows that the fused load kernel wrote during the
// step whose number equals stamp[s]; they override h for those rows.
// The rows are cut into down_chunks(n) chunks - a function of n alone, so the arithmetic does not
// depend on the launch geometry - and workgroup row y takes the chunks y, y + gridDim.y, ...  Every
// chunk is summed from zero.  With one chunk in use the workgroup writes its columns of y.  With more,
// a grid of one workgroup row adds its chunk sums in chunk order and writes y; a taller grid writes
// them to ypart[chunk][token][d] (fp32) and k_ffn_down_finish adds them in the same order.  No atomics.
template <typename T, int BT, bool SKIP, int LANES, int TS1 = kDownTile>
__global__ __launch_bounds__(256) void k_ffn_down(const T* __restrict__ matrix, const float* __restrict__ h,
                                                  const float* __restrict__ h_new, const int32_t* __restrict__ stamp,
                                                  T* __restrict__ y, float* __restrict__ ypart, int d, int batch,
                                                  int capacity, size_t row_elems, int down_off, int spec_groups,
                                                  DevState* __restrict__ st) {
    using V = typename Vec<T>::type;
    constexpr int VE = Vec<T>::N;
    constexpr int RG = 256 / LANES;                  // row groups per workgroup
    // rows per compaction pass (one token: TS1, 2048 or 4096 - the host picks by the row-count hint; both give the
    // same bits, see below)
    constexpr int TS = (BT == 1) ? TS1 : (kDownTile / BT < 512) ? 512 : kDownTile / BT;
    constexpr int PER = TS / 256;                    // slots per thread in the compaction
    __shared__ int list[TS];
    __shared__ float hv[BT][TS];
    __shared__ int wave_tot[4];
    __shared__ float red[4][LANES][BT * VE];
    __shared__ int n_active;

    const int tid = threadIdx.x, l = tid & (LANES - 1), rg = tid / LANES;
    // XCD-aware slice order when a slice is narrower than a 128-byte L2 line: workgroups are dealt
    // round-robin to the 8 XCDs, each with its own L2; giving every XCD a contiguous run of slices makes
    // the parts of a line meet in one L2 instead of being fetched by several (the host rounds the
    // grid up to a multiple of 8 in that case).
    int slice = blockIdx.x;
    if (LANES * 16 < 128) {
        const int per_xcd = gridDim.x / kXcds;
        slice = (blockIdx.x % kXcds) * per_xcd + blockIdx.x / kXcds;
    }
    const int col = slice * (LANES * VE) + l * VE;
    const bool col_ok = col < d;
    const T* base = matrix + down_off + (col_ok ? col : 0);

    if (tid == 0) n_active = 0;
    // the first workgroup row requests the activations of its first pass before the row count is known
    // (the activation array spans the whole capacity, so the addresses are valid; values past
    // num_used are masked below): one memory round trip less on the critical path
    const bool first_row = blockIdx.y == 0;
    // (uniform branches around unconditional loads from clamped slots: a predicate per load would cost a branch each;
    // spec_groups = how many groups of 256 slots to ask for now when a pass has more than 8: the host derives it from
    // the row-count hint, the rest is read once the count is known)
    float hfirst[PER][BT], hnfirst[PER][BT];
    int sfirst[PER];
#pragma unroll
    for (int q = 0; q < PER; ++q) {
        sfirst[q] = -1;
#pragma unroll
        for (int b = 0; b < BT; ++b) hfirst[q][b] = hnfirst[q][b] = 0.f;
    }
    if (first_row) {
#pragma unroll
        for (int b = 0; b < BT; ++b) {
            if (b < batch) {
#pragma unroll
                for (int q = 0; q < PER; ++q)
                    if (PER <= 8 || q < spec_groups) hfirst[q][b] = h[(size_t)b * capacity + min(q * 256 + tid, capacity - 1)];
            }
        }
        if (stamp) {
            // the loader-written activations travel in the same round trip as h and the stamps
#pragma unroll
            for (int q = 0; q < PER; ++q)
                if (PER <= 8 || q < spec_groups) sfirst[q] = stamp[min(q * 256 + tid, capacity - 1)];
#pragma unroll
            for (int b = 0; b < BT; ++b) {
                if (b < batch) {
#pragma unroll
                    for (int q = 0; q < PER; ++q)
                        if (PER <= 8 || q < spec_groups) hnfirst[q][b] = h_new[(size_t)b * capacity + min(q * 256 + tid, capacity - 1)];
                }
            }
        }
    }
    const int err = st->error;
    const int n = err ? 0 : st->num_used;
    const int cur_step = st->step;
    if (err) return;
    const int chunks = down_chunks<BT, SKIP>(n);
    if ((int)blockIdx.y >= chunks) return;           // uniform
    const int per_chunk = (n + chunks - 1) / chunks;
    if (first_row && stamp) {
#pragma unroll
        for (int q = 0; q < PER; ++q)
            if (sfirst[q] == cur_step) {
#pragma unroll
                for (int b = 0; b < BT; ++b) hfirst[q][b] = hnfirst[q][b];
            }
    }
    const int ob = tid / LANES, ol = tid - ob * LANES;            // (token, lane) whose 16-byte piece this thread writes
    const int ocol = slice * (LANES * VE) + ol * VE;
    const bool writer = tid < LANES * BT && ocol < d && ob < batch;
    float total[VE];
#pragma unroll
    for (int e = 0; e < VE; ++e) total[e] = 0.f;

    for (int chunk = blockIdx.y; chunk < chunks; chunk += gridDim.y) {
        const int r0 = chunk * per_chunk, r1 = min(n, r0 + per_chunk);
        float acc[BT * VE];                          // acc[b * VE + e]: token b, element e of this lane's 16 bytes
#pragma unroll
        for (int i = 0; i < BT * VE; ++i) acc[i] = 0.f;
        __syncthreads();
        if constexpr (BT == 1) {
            // One token: every wave compacts the slots of its own lanes with ballots into its own quarter of the
            // list and then reads the rows of that quarter, so a pass needs no workgroup barrier and no scan through
            // LDS (a wave's LDS operations complete in order).  Slots are dealt to threads round-robin, so the waves
            // get even shares.  Order inside a wave: slot-major (q, then lane); the adds stay in list order.
            constexpr int WL = TS / 4;                   // list entries per wave (PER slots x 64 lanes)
            constexpr int RGW = 64 / LANES;              // row groups per wave
            const int lane = tid & 63, wv = tid >> 6, rgw = lane / LANES;
            int* wlist = list + wv * WL;
            float* whv = hv[0] + wv * WL;
            // A thread takes the list positions i with i mod RGW = its row group, counted over the whole chunk and
            // not per pass, and adds them in ascending order: passes of 2048 or of 4096 slots give the same sums.
            int cnt = 0;                                 // entries of this wave's list so far (uniform over the wave)
            for (int s_base = r0; s_base < r1; s_base += TS) {
                const int start = cnt;                   // list position of the first entry of this pass
                int nz = 0;
                float hval[PER];
                const int need = min(PER, (r1 - s_base + 255) >> 8);      // groups of 256 slots with rows in them
                const int have = (s_base == 0) ? (PER <= 8 ? PER : min(spec_groups, PER)) : 0;   // ... of which requested at the start
#pragma unroll
                for (int q = 0; q < PER; ++q) hval[q] = hfirst[q][0];       // (only chunk 0 starts at row 0)
                if (need > have) {
#pragma unroll
                    for (int q = 0; q < PER; ++q)
                        if (q >= have && q < need) hval[q] = h[min(s_base + q * 256 + tid, capacity - 1)];
                    if (stamp) {
#pragma unroll
                        for (int q = 0; q < PER; ++q) {
                            if (q >= have && q < need) {
                                const int sc = min(s_base + q * 256 + tid, capacity - 1);
                                const float hn = h_new[sc];
                                if (stamp[sc] == cur_step) hval[q] = hn;
                            }
                        }
                    }
                }
#pragma unroll
                for (int q = 0; q < PER; ++q) {
                    if (PER <= 8 || q < need) {           // uniform (short passes: all groups, empty ones cost little)
                        const int s = s_base + q * 256 + tid;
                        const float v = (s < r1) ? hval[q] : 0.f;
                        const bool nonzero = v != 0.f;
                        const bool take = SKIP ? nonzero : s < r1;
                        const unsigned long long m = __ballot(take);
                        if (take) {
                            const int pos = cnt + (int)__builtin_amdgcn_mbcnt_hi((unsigned)(m >> 32),
                                                                                  __builtin_amdgcn_mbcnt_lo((unsigned)m, 0u));
                            wlist[pos - start] = s;
                            whv[pos - start] = v;
                        }
                        cnt += __popcll(m);
                        nz += SKIP ? __popcll(m) : __popcll(__ballot(nonzero));
                    }
                }
                if (slice == 0 && lane == 0 && nz) atomicAdd(&n_active, nz);      // statistics only
                __builtin_amdgcn_wave_barrier();
                if (col_ok) {
                    // all row loads of a pass over kInFlight rows per thread are issued before the first use
                    constexpr int kInFlight = 8;
                    const int first = start + ((rgw - start) & (RGW - 1));   // first position >= start of this row group
                    for (int i0 = first; i0 < cnt; i0 += RGW * kInFlight) {
                        V v[kInFlight];
#pragma unroll
                        for (int u = 0; u < kInFlight; ++u) {
                            const int i = i0 + u * RGW;
                            const int sr = wlist[(i < cnt ? i : i0) - start];
                            v[u] = (i < cnt) ? *reinterpret_cast<const V*>(base + (size_t)sr * row_elems) : V(0);
                        }
#pragma unroll
                        for (int u = 0; u < kInFlight; ++u) {
                            const int i = i0 + u * RGW;
                            if (i < cnt) {
                                const float hb = whv[i - start];
#pragma unroll
                                for (int e = 0; e < VE; ++e) acc[e] = __builtin_fmaf(hb, (float)v[u][e], acc[e]);
                            }
                        }
                    }
                }
                __builtin_amdgcn_wave_barrier();
            }
        } else {
            for (int s_base = r0; s_base < r1; s_base += TS) {
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
                        if (s < r1 && b < batch) {
                            if (s_base == 0) v = hfirst[q][b];       // only chunk 0 (first workgroup row) starts at row 0
                            else v = (stamp && stamp[s] == cur_step) ? h_new[(size_t)b * capacity + s]
                                                                     : h[(size_t)b * capacity + s];
                        }
                        hloc[q][b] = v;
                        any |= (v != 0.f);
                    }
                    if (any) nonzero |= 1u << q;
                    if (!SKIP) any = s < r1;
                    if (any) flags |= 1u << q;
                }
                if (slice == 0 && nonzero) atomicAdd(&n_active, __popc(nonzero));   // statistics only
                int cnt;
                int off = block_exclusive_scan<4>(__popc(flags), wave_tot, &cnt);
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
                    // all row loads of a pass over kInFlight rows per thread are issued before the first use (a loop with a
                    // run-time trip count would wait for every load in turn); the adds stay in ascending row order
                    constexpr int kInFlight = (BT == 1) ? 8 : 4;
                    for (int i0 = rg; i0 < cnt; i0 += RG * kInFlight) {
                        V v[kInFlight];
#pragma unroll
                        for (int u = 0; u < kInFlight; ++u) {
                            const int i = i0 + u * RG;
                            const int s = list[i < cnt ? i : i0];
                            v[u] = (i < cnt) ? *reinterpret_cast<const V*>(base + (size_t)s * row_elems) : V(0);
                        }
#pragma unroll
                        for (int u = 0; u < kInFlight; ++u) {
                            const int i = i0 + u * RG;
                            if (i < cnt) {
#pragma unroll
                                for (int b = 0; b < BT; ++b) {
                                    const float hb = hv[b][i];
#pragma unroll
                                    for (int e = 0; e < VE; ++e)
                                        acc[b * VE + e] = __builtin_fmaf(hb, (float)v[u][e], acc[b * VE + e]);
                                }
                            }
                        }
                    }
                }
                __syncthreads();
            }
        }
        // the row groups of one wave sit LANES lanes apart: halving butterfly over the upper lane bits (a lane
        // ends with a few finished sums), then LDS over waves
        {
            constexpr int held = wave_fold_held<BT * VE, LANES>();
            constexpr int dup = wave_fold_dup_mask<BT * VE, LANES>();
            const int first = wave_fold<BT * VE, LANES>(acc, tid & 63);
            if (((tid & 63) & dup) == 0) {
#pragma unroll
                for (int i = 0; i < held; ++i) red[tid >> 6][l][first + i] = acc[i];
            }
        }
        __syncthreads();
        if (writer) {
            float sum[VE];
#pragma unroll
            for (int e = 0; e < VE; ++e)
                sum[e] = ((red[0][ol][ob * VE + e] + red[1][ol][ob * VE + e]) + red[2][ol][ob * VE + e]) +
                         red[3][ol][ob * VE + e];
            if (chunks > 1 && gridDim.y > 1) {
                float* out = ypart + ((size_t)chunk * batch + ob) * d + ocol;
#pragma unroll
                for (int e = 0; e < VE; ++e) out[e] = sum[e];
            } else {
#pragma unroll
                for (int e = 0; e < VE; ++e) total[e] += sum[e];      // chunk order; 0 + first sum is exact
            }
        }
    }
    if (slice == 0 && tid == 0) {
        if (first_row) {
            atomicAdd(&st->c_ffn_calls, 1ull);
            atomicAdd(&st->c_ffn_rows, (unsigned long long)n);
        }
        if (n_active) atomicAdd(&st->c_ffn_active, (unsigned long long)n_active);
    }
    if (writer && (chunks == 1 || gridDim.y == 1)) {
        V out;
#pragma unroll
        for (int e = 0; e < VE; ++e) out[e] = (T)total[e];
        *reinterpret_cast<V*>(y + (size_t)ob * d + ocol) = out;
    }
}

// y = sum of the chunk partials in chunk order, rounded once to the element type.  Launched after a
// k_ffn_down grid of more than one workgroup row; does nothing when a single chunk was in use (y is
// written already).  grid = ceil(batch * d / 256), block = 256.
template <typename T, int BT, bool SKIP>
__global__ __launch_bounds__(256) void k_ffn_down_finish(const float* __restrict__ ypart, T* __restrict__ y, int d,
                                                         int batch, const DevState* __restrict__ st) {
    if (st->error) return;
    const int chunks = down_chunks<BT, SKIP>(st->num_used);
    if (chunks == 1) return;
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= batch * d) return;
    // all partials are requested before the first add (a loop with a run-time trip count would wait for
    // every load in turn)
    float v[kDownChunksMax];
#pragma unroll
    for (int c = 0; c < kDownChunksMax; ++c) v[c] = (c < chunks) ? ypart[(size_t)c * batch * d + i] : 0.f;
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < kDownChunksMax; ++c)
        if (c < chunks) s += v[c];
    y[i] = (T)s;
}

}  // namespace lif
