// Step 4, down projection for a batch of 2..8 tokens (fp16) on the matrix cores:
//   Y[t][j] = sum_s H[t][s] * D[s][j]      over the cached rows s that contribute (Section 3.3 item 3).
// With several tokens the vector units are the limit of the streaming form (k_ffn_down: 64 multiply-adds and 8 LDS
// reads per 16 bytes of a down column; measured at the Llama-2 shape, 8 tokens, 8700 rows: 9 us in the row loop,
// 5.6 us with the arithmetic taken out).  Here one v_mfma_f32_16x16x32_f16 covers K = 32 rows x N = 16 groups of
// columns x M = 16 token slots.  Memory is contiguous along the columns and the matrix instruction wants K (rows)
// packed per lane, so a lane loads 16 bytes (its 8 columns) of 8 rows and transposes the 8 x 8 block in its own
// registers (32 v_perm_b32); column j of the block feeds the j-th of eight accumulator tiles.
// The activations are fp32.  They enter as fp16 pairs: scaled by a power of two so that the largest of a pass is
// below 2^15 (exact), then split into a high and a low part (h * scale = hi + lo up to 2^-22 relative); token
// slots 0..7 of M carry the high parts of tokens 0..7, slots 8..15 their low parts, and the two halves of the
// result are added at the end of a pass.  Products are exact, accumulation is fp32.
#pragma once

#include "lif_ffn.h"

namespace lif {

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

constexpr int kDmRows = 512;             // rows compacted per pass
constexpr int kDmPitch = kDmRows + 8;    // fp16 values per token slot in LDS (16 bytes of padding: lanes of one
                                         // row block read 16 different slots at the same offset)
constexpr int kDmCols = 128;             // columns per workgroup: 16 lanes x 16 bytes
constexpr int kDmWaves = 4;              // waves per workgroup: 8 are faster below 4000 rows (9 against 12 us) but their
                                         // registers leave one workgroup per compute unit (27 against 16 us at 8700 rows)

// Rows per chunk (one partial output per chunk): a multiple of kDmRows that depends on the capacity alone, so a
// workgroup row knows where its first chunk starts before the row count arrives, and at most kDownChunksMax
// chunks are ever in use.
__host__ __device__ __forceinline__ int down_mfma_chunk_rows(int capacity) {
    const int per = kDmRows * kDownChunksMax;
    const int passes = (capacity + per - 1) / per;
    return kDmRows * (passes < 1 ? 1 : passes);
}
__host__ __device__ __forceinline__ int down_mfma_chunks(int n, int chunk_rows) {
    const int c = (n + chunk_rows - 1) / chunk_rows;
    return c < 1 ? 1 : c;
}

// Two fp16 values (one from each source register) packed into one: the low halves or the high halves.
// v_perm_b32 picks bytes out of {s0 = bytes 7..4, s1 = bytes 3..0}.
__device__ __forceinline__ unsigned pack_halves(unsigned second, unsigned first, bool high) {
    return high ? __builtin_amdgcn_perm(second, first, 0x07060302u) : __builtin_amdgcn_perm(second, first, 0x05040100u);
}

// grid = (ceil(d / 128) column slices, row-chunk workgroups), block = WAVES waves; lane l of a wave: column
// group n16 = l mod 16 (8 columns) and token slot n16, row block q = l div 16 (8 of the 32 rows of an instruction).
// A pass compacts the contributing rows of 512 slots (SKIP: rows with some activation; else all rows in use) in a
// fixed order (thread-major over slots p * threads + tid); the waves take groups of 32 compacted rows in turn.
// A chunk's passes are added in order, the waves in wave order, the chunks in chunk order (by this kernel when
// one workgroup row is launched, else by k_ffn_down_mfma_finish from ypart[chunk][token][d]).  Nothing depends on
// the launch geometry.
template <bool SKIP, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void k_ffn_down_mfma(const _Float16* __restrict__ matrix,
                                                              const float* __restrict__ h, _Float16* __restrict__ y,
                                                              float* __restrict__ ypart, int d, int batch, int capacity,
                                                              size_t row_elems, int down_off, int chunk_rows,
                                                              DevState* __restrict__ st) {
    constexpr int BT = 8, T = WAVES * 64;
    constexpr int PER = kDmRows / T;                 // slots per thread in the compaction
    constexpr int OUTS = BT * kDmCols / T;           // outputs per thread
    static_assert(kDmRows % T == 0 && (BT * kDmCols) % T == 0, "whole slots and outputs per thread");
    __shared__ int list[kDmRows];
    __shared__ __attribute__((aligned(16))) _Float16 hv[16][kDmPitch];
    __shared__ int wave_tot[WAVES];
    __shared__ float wave_max[WAVES];
    __shared__ float red[WAVES][32][33];             // per wave and lane with q < 2: 32 sums, padded
    __shared__ int n_active;

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int n16 = lane & 15, q = lane >> 4;
    const int col = blockIdx.x * kDmCols + n16 * 8;
    const bool col_ok = col < d;
    const _Float16* base = matrix + down_off + (col_ok ? col : 0);

    if (tid == 0) n_active = 0;
    // the activations of the first pass are requested before the row count is known (the array spans the capacity)
    float hfirst[PER][BT];
#pragma unroll
    for (int p = 0; p < PER; ++p) {
        const int s = blockIdx.y * chunk_rows + p * T + tid;
#pragma unroll
        for (int b = 0; b < BT; ++b) hfirst[p][b] = (s < capacity && b < batch) ? h[(size_t)b * capacity + s] : 0.f;
    }
    const int err = st->error;
    const int n = err ? 0 : st->num_used;
    if (err) return;
    const int chunks = down_mfma_chunks(n, chunk_rows);
    if ((int)blockIdx.y >= chunks) return;           // uniform

    float total[OUTS];                               // thread tid finishes outputs tid + k * T of the 8 tokens x 128 columns
#pragma unroll
    for (int k = 0; k < OUTS; ++k) total[k] = 0.f;

    for (int chunk = blockIdx.y; chunk < chunks; chunk += gridDim.y) {
        const int r0 = chunk * chunk_rows, r1 = min(n, r0 + chunk_rows);
        // red[w][lane with q < 2][j * 4 + r]: this wave's sum for tokens 4q + r, column j of the lane's 8
        if (q < 2) {
#pragma unroll
            for (int i = 0; i < 32; ++i) red[w][lane][i] = 0.f;
        }
        for (int s_base = r0; s_base < r1; s_base += kDmRows) {
            // compaction of the rows that contribute and the largest |activation| of the pass
            const bool spec = chunk == (int)blockIdx.y && s_base == r0;
            float hloc[PER][BT];
            unsigned flags = 0, nonzero = 0;
            float amax = 0.f;
#pragma unroll
            for (int p = 0; p < PER; ++p) {
                const int s = s_base + p * T + tid;
                bool any = false;
#pragma unroll
                for (int b = 0; b < BT; ++b) {
                    float v = 0.f;
                    if (s < r1 && b < batch) v = spec ? hfirst[p][b] : h[(size_t)b * capacity + s];
                    hloc[p][b] = v;
                    any |= (v != 0.f);
                    amax = fmaxf(amax, fabsf(v));
                }
                if (any) nonzero |= 1u << p;
                if (SKIP ? any : s < r1) flags |= 1u << p;
            }
            if (blockIdx.x == 0 && nonzero) atomicAdd(&n_active, __popc(nonzero));   // statistics only
#pragma unroll
            for (int m = 32; m >= 1; m >>= 1) amax = fmaxf(amax, __shfl_xor(amax, m, kWave));
            if (lane == 0) wave_max[w] = amax;       // (the barriers of the scan order this write and the reads below,
                                                     //  and keep the previous pass's readers of list / hv ahead of the writes)
            int cnt;
            int off = block_exclusive_scan<WAVES>(__popc(flags), wave_tot, &cnt);
            float smax = wave_max[0];
#pragma unroll
            for (int i = 1; i < WAVES; ++i) smax = fmaxf(smax, wave_max[i]);
            // power-of-two scale: the largest scaled activation lies in [2^14, 2^15)
            const bool scalable = smax > 0.f && smax < 3.0e38f;
            const int ex = scalable ? ilogbf(smax) : 14;
            const float scale = ldexpf(1.f, 14 - ex), inv_scale = ldexpf(1.f, ex - 14);
#pragma unroll
            for (int p = 0; p < PER; ++p) {
                if (flags & (1u << p)) {
                    list[off] = s_base + p * T + tid;
#pragma unroll
                    for (int b = 0; b < BT; ++b) {
                        const float hs = hloc[p][b] * scale;
                        const _Float16 hi = (_Float16)hs;
                        hv[b][off] = hi;
                        hv[BT + b][off] = (_Float16)(hs - (float)hi);
                    }
                    ++off;
                }
            }
            // the matrix instruction reads whole groups of 32 rows: zero activations behind the last row
            if (tid < 32 && cnt + tid < ((cnt + 31) & ~31)) {
#pragma unroll
                for (int m = 0; m < 16; ++m) hv[m][cnt + tid] = (_Float16)0.f;
            }
            __syncthreads();
            if (smax > 0.f) {                        // uniform over the workgroup
                f32x4 acc[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
                // the rows of a group: 8 loads of 16 bytes per lane
                auto load = [&](f16x8 (&v)[8], int g) {
#pragma unroll
                    for (int r = 0; r < 8; ++r) {
                        const int i = g * 32 + q * 8 + r;
                        const int sr = list[i < cnt ? i : 0];
                        v[r] = (i < cnt && col_ok) ? *reinterpret_cast<const f16x8*>(base + (size_t)sr * row_elems) : f16x8(0);
                    }
                };
                auto compute = [&](const f16x8 (&v)[8], int g) {
                    // this lane's token slot: activations of rows i0 .. i0 + 7
                    const f16x8 a = *reinterpret_cast<const f16x8*>(&hv[n16][g * 32 + q * 8]);
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        // column j of the 8 x 8 block: rows 2 r2 and 2 r2 + 1 packed into dword r2
                        u32x4 bj;
#pragma unroll
                        for (int r2 = 0; r2 < 4; ++r2) {
                            const u32x4 lo = __builtin_bit_cast(u32x4, v[2 * r2]), hi = __builtin_bit_cast(u32x4, v[2 * r2 + 1]);
                            bj[r2] = pack_halves(hi[j >> 1], lo[j >> 1], (j & 1) != 0);
                        }
                        acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, __builtin_bit_cast(f16x8, bj), acc[j], 0, 0, 0);
                    }
                };
                // (a second register set that requests the wave's next group ahead of the arithmetic was measured:
                // no faster at 1400 rows, and the registers cost a third of the resident waves at 8700)
                for (int g = w; g * 32 < cnt; g += WAVES) {
                    f16x8 v[8];
                    load(v, g);
                    compute(v, g);
                }
                // token slots 8..15 (lanes with q >= 2) hold the low-part products of tokens 0..7: add them; the
                // passes of a chunk add up in the wave's own LDS entries (0 + first pass is exact)
#pragma unroll
                for (int j = 0; j < 8; ++j)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const float lo = __shfl_down(acc[j][r], 32, kWave);
                        if (q < 2) red[w][lane][j * 4 + r] += (acc[j][r] + lo) * inv_scale;
                    }
            }
        }
        // the waves took different rows: add in wave order
        __syncthreads();
#pragma unroll
        for (int k = 0; k < OUTS; ++k) {
            const int o = tid + k * T;               // token o / 128, column o % 128 of the slice
            const int t = o >> 7, c = o & 127;
            const int src_lane = (t >> 2) * 16 + (c >> 3), src = (c & 7) * 4 + (t & 3);
            float sum = red[0][src_lane][src];
#pragma unroll
            for (int ww = 1; ww < WAVES; ++ww) sum += red[ww][src_lane][src];
            const int ocol = blockIdx.x * kDmCols + c;
            if (chunks > 1 && gridDim.y > 1) {
                if (t < batch && ocol < d) ypart[((size_t)chunk * batch + t) * d + ocol] = sum;
            } else {
                total[k] += sum;                     // chunk order; 0 + first sum is exact
            }
        }
        __syncthreads();                             // red is written again by the next chunk
    }
    if (blockIdx.x == 0 && tid == 0) {
        if (blockIdx.y == 0) {
            atomicAdd(&st->c_ffn_calls, 1ull);
            atomicAdd(&st->c_ffn_rows, (unsigned long long)n);
        }
        if (n_active) atomicAdd(&st->c_ffn_active, (unsigned long long)n_active);
    }
    if (chunks == 1 || gridDim.y == 1) {
#pragma unroll
        for (int k = 0; k < OUTS; ++k) {
            const int o = tid + k * T;
            const int t = o >> 7, ocol = blockIdx.x * kDmCols + (o & 127);
            if (t < batch && ocol < d) y[(size_t)t * d + ocol] = (_Float16)total[k];
        }
    }
}

// y = sum of the chunk partials in chunk order, rounded once to fp16.  Launched after a k_ffn_down_mfma grid of
// more than one workgroup row; does nothing when a single chunk was in use (y is written already).
// grid = ceil(batch * d / 256), block = 256.
__global__ __launch_bounds__(256) void k_ffn_down_mfma_finish(const float* __restrict__ ypart, _Float16* __restrict__ y,
                                                              int d, int batch, int chunk_rows,
                                                              const DevState* __restrict__ st) {
    if (st->error) return;
    const int chunks = down_mfma_chunks(st->num_used, chunk_rows);
    if (chunks == 1) return;
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= batch * d) return;
    // all partials are requested before the first add
    float v[kDownChunksMax];
#pragma unroll
    for (int c = 0; c < kDownChunksMax; ++c) v[c] = (c < chunks) ? ypart[(size_t)c * batch * d + i] : 0.f;
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < kDownChunksMax; ++c)
        if (c < chunks) s += v[c];
    y[i] = (_Float16)s;
}

}  // namespace lif
