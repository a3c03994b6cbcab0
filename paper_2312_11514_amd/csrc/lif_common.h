// Shared device-side definitions of the sparse-FFN hot path (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lif {

constexpr int kWave = 64;

// Device-resident state of one layer.  Lives at the start of the caller's workspace so
// that the hot calls chain on a stream without the host ever knowing a count.
struct DevState {
    int32_t num_used;     // rows of the cache in use (Section 3.3 "num_used")
    int32_t n_base;       // rows kept after the pending deletion (n' = num_used - c)
    int32_t step;         // completed window updates
    int32_t error;        // sticky lif_status (0 or LIF_CAPACITY)
    int32_t n_added;      // |added| of the pending / last update
    int32_t n_removed;    // |removed| of the pending / last update
    int32_t n_moved;      // rows moved by the last deletion
    int32_t window_len;   // step masks currently in the window (<= k; smaller after a dynamic shrink)
    int32_t ring_pos;     // ring entry the next mask goes to
    int32_t pad;
    // counters: only ever updated with atomic adds whose result is not used (a load-add-store at the end of a kernel
    // would keep its last wave waiting for a memory round trip)
    unsigned long long c_steps, c_added, c_removed, c_rows_moved, c_h2d_bytes;
    unsigned long long c_ffn_calls, c_ffn_rows, c_ffn_active;   // FFN calls, rows in use, rows with a non-zero activation
};

// Where the bundle of neuron i lives in pinned host memory (Section 3.2, Fig. 5).  Bundled (down == null): one
// contiguous chunk of row_bytes at rows + i * row_bytes.  Not bundled: the activation vectors ((gate |) up row,
// act_bytes) at rows + i * act_bytes and the down column at down + i * (row_bytes - act_bytes): two reads per
// neuron, the layout that bundling replaces.  All sizes are multiples of 16 bytes.
struct HostStore {
    const char* rows;
    const char* down;
    size_t act_bytes;
};
// address of byte `off` (a multiple of 16, < row_bytes) of the bundle of neuron i
__device__ __forceinline__ const char* host_piece(const HostStore& hs, int i, size_t off, size_t row_bytes) {
    if (hs.down && off >= hs.act_bytes) return hs.down + (size_t)i * (row_bytes - hs.act_bytes) + (off - hs.act_bytes);
    return hs.rows + (size_t)i * (hs.down ? hs.act_bytes : row_bytes) + off;
}

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// 16-byte vector view of the element type.
template <typename T> struct Vec;
template <> struct Vec<_Float16> {
    using type = f16x8;
    static constexpr int N = 8;
};
template <> struct Vec<float> {
    using type = f32x4;
    static constexpr int N = 4;
};

// acc + sum_e a[e] * b[e], products of E-typed values, fp32 accumulation.
#if defined(__HIP_DEVICE_COMPILE__)     // (the host pass only parses device functions)
static_assert(__has_builtin(__builtin_amdgcn_fdot2), "built for gfx950: the packed fp16 dot product is required");
#endif
__device__ __forceinline__ float dot_acc(f16x8 a, f16x8 b, float acc) {
    acc = __builtin_amdgcn_fdot2(__builtin_shufflevector(a, a, 0, 1), __builtin_shufflevector(b, b, 0, 1), acc, false);
    acc = __builtin_amdgcn_fdot2(__builtin_shufflevector(a, a, 2, 3), __builtin_shufflevector(b, b, 2, 3), acc, false);
    acc = __builtin_amdgcn_fdot2(__builtin_shufflevector(a, a, 4, 5), __builtin_shufflevector(b, b, 4, 5), acc, false);
    acc = __builtin_amdgcn_fdot2(__builtin_shufflevector(a, a, 6, 7), __builtin_shufflevector(b, b, 6, 7), acc, false);
    return acc;
}
__device__ __forceinline__ float dot_acc(f32x4 a, f32x4 b, float acc) {
#pragma unroll
    for (int e = 0; e < 4; ++e) acc = __builtin_fmaf(a[e], b[e], acc);
    return acc;
}

// Sum over the 64 lanes of a wave; every lane receives the result.  Data-parallel-primitive moves instead of
// shuffles through the LDS crossbar: an inclusive prefix sum (shifts by 1, 2, 4, 8 inside the rows of 16 lanes,
// lane 15 of a row into the next row, lane 31 into the upper half) leaves the total in lane 63, which is then
// broadcast.  Lanes without a source add 0.
template <int CTRL, int ROWS>
__device__ __forceinline__ float dpp_from(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROWS, 0xf, false));
}
template <int CTRL, int ROWS>
__device__ __forceinline__ double dpp_from(double v) {
    const unsigned long long u = __builtin_bit_cast(unsigned long long, v);
    const unsigned lo = (unsigned)__builtin_amdgcn_update_dpp(0, (int)(unsigned)u, CTRL, ROWS, 0xf, false);
    const unsigned hi = (unsigned)__builtin_amdgcn_update_dpp(0, (int)(unsigned)(u >> 32), CTRL, ROWS, 0xf, false);
    return __builtin_bit_cast(double, ((unsigned long long)hi << 32) | lo);
}
__device__ __forceinline__ float wave_sum(float v) {
    v += dpp_from<0x111, 0xf>(v);   // row_shr:1
    v += dpp_from<0x112, 0xf>(v);   // row_shr:2
    v += dpp_from<0x114, 0xf>(v);   // row_shr:4
    v += dpp_from<0x118, 0xf>(v);   // row_shr:8
    v += dpp_from<0x142, 0xa>(v);   // row_bcast:15 into rows 1 and 3
    v += dpp_from<0x143, 0xc>(v);   // row_bcast:31 into rows 2 and 3
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}
__device__ __forceinline__ double wave_sum(double v) {
    v += dpp_from<0x111, 0xf>(v);
    v += dpp_from<0x112, 0xf>(v);
    v += dpp_from<0x114, 0xf>(v);
    v += dpp_from<0x118, 0xf>(v);
    v += dpp_from<0x142, 0xa>(v);
    v += dpp_from<0x143, 0xc>(v);
    const unsigned long long u = __builtin_bit_cast(unsigned long long, v);
    const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)u, 63);
    const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(u >> 32), 63);
    return __builtin_bit_cast(double, ((unsigned long long)hi << 32) | lo);
}

// Workgroup barrier that orders LDS accesses only: unlike __syncthreads() it does not wait for the global
// stores a wave has in flight (their acknowledgement from the L2 costs several hundred nanoseconds).  Use it
// where the data handed over lives in LDS and no thread reads global memory that another one has just written.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Inclusive prefix sum over the lanes of a wave.
__device__ __forceinline__ int wave_inclusive_scan(int v, int /*lane*/) {
    // data-parallel-primitive moves instead of six shuffles through the LDS crossbar: shifts by 1, 2, 4, 8 inside
    // the rows of 16 lanes (lanes without a source add 0), then lane 15 of a row into the next row (rows 1 and 3)
    // and lane 31 into rows 2 and 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, false);   // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, false);   // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, false);   // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, false);   // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);   // row_bcast:15
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);   // row_bcast:31
    return v;
}

// Exclusive prefix sum of one int per thread over a workgroup of NW waves (thread order).
// `wave_tot` is LDS scratch of at least NW ints.  Returns the exclusive prefix; *total receives the
// workgroup sum.  Contains two barriers (the first keeps a previous scan's readers of wave_tot ahead of the writes).
template <int NW>
__device__ __forceinline__ int block_exclusive_scan(int v, int* wave_tot, int* total) {
    const int tid = threadIdx.x, lane = tid & (kWave - 1), w = tid >> 6;
    const int inc = wave_inclusive_scan(v, lane);
    __syncthreads();
    if (lane == kWave - 1) wave_tot[w] = inc;
    __syncthreads();
    int before = 0, all = 0;
#pragma unroll
    for (int i = 0; i < NW; ++i) {
        const int t = wave_tot[i];
        if (i < w) before += t;
        all += t;
    }
    *total = all;
    return before + inc - v;
}


// Sum of v[0..N) over the lanes that differ in the lane bits M, 2M, ..., 32 (groups of lanes M apart).
// While a lane holds more than one value, a step halves them: the lane keeps the half selected by its own
// bit and hands the other half to its partner, so N - N / 2^steps (+ the remaining full steps) exchanges
// replace steps * N.  Returns through `first` the index of the first value this lane ends up with; it then
// holds wave_fold_held<N, M>() finished sums in v[0..held).  Lanes whose bits of the steps taken after a
// single value was left are not all zero hold a duplicate (wave_fold_dup_mask gives those bits).
template <int N, int M>
constexpr int wave_fold_held() {
    int held = N;
    for (int m = M; m < kWave; m <<= 1)
        if (held > 1) held >>= 1;
    return held;
}
template <int N, int M>
constexpr int wave_fold_dup_mask() {
    int held = N, mask = 0;
    for (int m = M; m < kWave; m <<= 1) {
        if (held > 1) held >>= 1;
        else mask |= m;
    }
    return mask;
}
template <int HELD, int M, int N>
__device__ __forceinline__ void wave_fold_step(float (&v)[N], int& first, int lane) {
    if constexpr (M < kWave) {
        if constexpr (HELD > 1) {
            constexpr int half = HELD / 2;
            const bool up = (lane & M) != 0;
#pragma unroll
            for (int i = 0; i < half; ++i) {
                const float send = up ? v[i] : v[i + half], keep = up ? v[i + half] : v[i];
                v[i] = keep + __shfl_xor(send, M, kWave);
            }
            first += up ? half : 0;
            wave_fold_step<half, M * 2, N>(v, first, lane);
        } else {
            v[0] += __shfl_xor(v[0], M, kWave);
            wave_fold_step<1, M * 2, N>(v, first, lane);
        }
    }
}
template <int N, int M>
__device__ __forceinline__ int wave_fold(float (&v)[N], int lane) {
    static_assert((N & (N - 1)) == 0, "power of two");
    int first = 0;
    wave_fold_step<N, M, N>(v, first, lane);
    return first;
}

}  // namespace lif
