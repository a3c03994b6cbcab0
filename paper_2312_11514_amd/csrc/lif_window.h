// Step 2: sliding window over the last k step masks (Section 3.1 "The Sliding Window
// Technique", Fig. 4b) and Step 3: neuron-cache update (Section 3.3 items 1-2, Fig. 6).
//
// Window state is one int32 per original neuron: the last step at which it was predicted
// active ("last_k_active").  A neuron is in the window after step t iff
// last_active >= t - k + 1.  Everything is integer work: results are exact.
#pragma once

#include "lif_common.h"

namespace lif {

constexpr int kScanThreads = 1024;   // single-workgroup kernels: 16 waves
constexpr int kMaxSpan = 64;         // neurons / slots per thread (bitmaps are 64-bit)
constexpr int kHoleLds = 4096;       // holes kept in LDS; longer lists spill to the global scratch list

// Exclusive prefix sums of two counts per thread in one pass (both < 2^31 in total, packed
// into one 64-bit lane value).  Same contract as block_exclusive_scan.
__device__ __forceinline__ void block_exclusive_scan2(int va, int vb, unsigned long long* wave_tot, int* off_a,
                                                      int* off_b, int* tot_a, int* tot_b) {
    const int tid = threadIdx.x, lane = tid & (kWave - 1), w = tid >> 6;
    const int nw = (blockDim.x + kWave - 1) >> 6;
    const unsigned long long v = ((unsigned long long)(unsigned)vb << 32) | (unsigned)va;
    unsigned long long inc = v;
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        unsigned long long u = __shfl_up(inc, o, kWave);
        if (lane >= o) inc += u;
    }
    __syncthreads();
    if (lane == kWave - 1) wave_tot[w] = inc;
    __syncthreads();
    unsigned long long before = 0, all = 0;
    for (int i = 0; i < nw; ++i) {
        const unsigned long long t = wave_tot[i];
        if (i < w) before += t;
        all += t;
    }
    const unsigned long long ex = before + inc - v;
    *off_a = (int)(unsigned)(ex & 0xffffffffull);
    *off_b = (int)(unsigned)(ex >> 32);
    *tot_a = (int)(unsigned)(all & 0xffffffffull);
    *tot_b = (int)(unsigned)(all >> 32);
}

// One workgroup does the window update and the deletion plan back to back.
//
// Window: the workgroup walks all F neurons in thread-contiguous spans, so that a
// workgroup-wide prefix sum over per-thread popcounts yields ids in ascending order.
//
// Deletion plan (Section 3.3 item 1): a slot is dead iff its neuron was just removed (looked
// up in an LDS bitmap of the removed ids).  With n' = n - c, the dead slots below n'
// ("holes", ascending) are filled by the live slots at or above n' ("fillers"): hole j takes
// the (H-1-j)-th filler - the lowest hole receives the last row, exactly what the
// sequential swap-with-last loop does.  Sources (>= n') and destinations (< n') are
// disjoint, so the moves can later run in any order.
// Output of the plan: move_dst[q] for tail slot n' + q = destination slot, or -1 if dead.
//
// Every global load (state, mask bytes, last_active, pointers) is issued before the first
// use, so the kernel pays one memory round trip, not one per phase.
// SPAN_F = neurons per thread (multiple of 8, <= 64); SPAN_C = cache slots per thread (<= 64).
template <int SPAN_F, int SPAN_C>
__global__ __launch_bounds__(kScanThreads) void k_window_plan(
    const uint8_t* __restrict__ step_mask, int32_t* __restrict__ last_active, const int32_t* __restrict__ pointers,
    int F, int k, int capacity, int32_t* __restrict__ added, int32_t* __restrict__ n_added,
    int32_t* __restrict__ removed, int32_t* __restrict__ n_removed, int32_t* __restrict__ move_dst,
    int32_t* __restrict__ hole_list, DevState* st) {
    __shared__ unsigned long long wave_tot[kScanThreads / kWave];
    __shared__ unsigned rem_bm[kScanThreads * kMaxSpan / 32];
    __shared__ int hole_lds[kHoleLds];
    const int tid = threadIdx.x;

    // ---- issue all loads ----
    const int i0 = tid * SPAN_F, s0 = tid * SPAN_C;
    int4 la[SPAN_F / 4];
    unsigned mbyte[SPAN_F / 8];
    int ptr[SPAN_C];
#pragma unroll
    for (int g = 0; g < SPAN_F / 8; ++g) {
        const int i = i0 + g * 8;
        const bool ok = i < F;
        mbyte[g] = ok ? step_mask[i >> 3] : 0u;
        la[2 * g] = ok ? *reinterpret_cast<const int4*>(last_active + i) : make_int4(kNever, kNever, kNever, kNever);
        la[2 * g + 1] = ok ? *reinterpret_cast<const int4*>(last_active + i + 4) : make_int4(kNever, kNever, kNever, kNever);
    }
#pragma unroll
    for (int q = 0; q < SPAN_C; ++q) ptr[q] = (s0 + q < capacity) ? pointers[s0 + q] : -1;
    const int err = st->error;
    const int t = st->step;
    const int n = st->num_used;
    for (int wd = tid; wd < (F + 31) / 32; wd += kScanThreads) rem_bm[wd] = 0u;

    if (err) {
        if (tid == 0) {
            *n_added = 0;
            *n_removed = 0;
            st->n_added = 0;
            st->n_removed = 0;
        }
        return;
    }

    // ---- window ----
    unsigned long long abits = 0, rbits = 0, mbits = 0;
#pragma unroll
    for (int g = 0; g < SPAN_F / 8; ++g) {
        const int v[8] = {la[2 * g].x, la[2 * g].y, la[2 * g].z, la[2 * g].w,
                          la[2 * g + 1].x, la[2 * g + 1].y, la[2 * g + 1].z, la[2 * g + 1].w};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const bool in_prev = v[e] >= t - k;                 // in S_{t-1}
            const bool hit = (mbyte[g] >> e) & 1u;
            const bool in_now = hit || v[e] >= t - k + 1;       // in S_t
            const unsigned long long bit = 1ull << (g * 8 + e);
            if (hit) mbits |= bit;
            if (in_now && !in_prev) abits |= bit;
            if (in_prev && !in_now) rbits |= bit;
        }
    }
    int off_a, off_r, tot_a, tot_r;
    block_exclusive_scan2(__popcll(abits), __popcll(rbits), wave_tot, &off_a, &off_r, &tot_a, &tot_r);

    const int n2 = n - tot_r;
    if (n2 < 0 || n2 + tot_a > capacity) {          // uniform: leave the window untouched
        if (tid == 0) {
            st->error = 3;                           // LIF_CAPACITY
            *n_added = 0;
            *n_removed = 0;
            st->n_added = 0;
            st->n_removed = 0;
        }
        return;
    }
    while (abits) {
        const int bpos = __ffsll((long long)abits) - 1;
        added[off_a++] = i0 + bpos;
        abits &= abits - 1;
    }
    while (rbits) {
        const int bpos = __ffsll((long long)rbits) - 1;
        const int id = i0 + bpos;
        removed[off_r++] = id;
        atomicOr(&rem_bm[id >> 5], 1u << (id & 31));
        rbits &= rbits - 1;
    }
    while (mbits) {
        const int bpos = __ffsll((long long)mbits) - 1;
        last_active[i0 + bpos] = t;
        mbits &= mbits - 1;
    }
    __syncthreads();

    // ---- deletion plan ----
    unsigned long long holebits = 0, fillbits = 0;
#pragma unroll
    for (int q = 0; q < SPAN_C; ++q) {
        const int s = s0 + q;
        if (s < n) {
            const int id = ptr[q];
            const bool dead = (id < 0 || id >= F) ? true : ((rem_bm[id >> 5] >> (id & 31)) & 1u);
            if (s < n2 && dead) holebits |= 1ull << q;
            if (s >= n2 && !dead) fillbits |= 1ull << q;
        }
    }
    int off_h, off_f, H, Fc;
    block_exclusive_scan2(__popcll(holebits), __popcll(fillbits), wave_tot, &off_h, &off_f, &H, &Fc);
    const bool in_lds = H <= kHoleLds;
    {
        unsigned long long hb = holebits;
        while (hb) {
            const int q = __ffsll((long long)hb) - 1;
            if (in_lds) hole_lds[off_h] = s0 + q;
            else hole_list[off_h] = s0 + q;
            ++off_h;
            hb &= hb - 1;
        }
    }
    __syncthreads();   // the hole list (LDS, or global scratch when long) is read by other threads below
#pragma unroll
    for (int q = 0; q < SPAN_C; ++q) {
        const int s = s0 + q;
        if (s >= n2 && s < n) {
            int dst = -1;
            if ((fillbits >> q) & 1ull) {
                const int j = H - 1 - off_f;
                if (j >= 0 && j < H) dst = in_lds ? hole_lds[j] : hole_list[j];
                ++off_f;
            }
            move_dst[s - n2] = dst;
        }
    }
    if (tid == 0) {
        *n_added = tot_a;
        *n_removed = tot_r;
        st->n_added = tot_a;
        st->n_removed = tot_r;
        st->n_base = n2;
        st->n_moved = H;
        st->step = t + 1;
        st->c_steps += 1;
        st->c_added += (unsigned long long)tot_a;
        st->c_removed += (unsigned long long)tot_r;
        st->c_rows_moved += (unsigned long long)H;
    }
}

// Row moves of the deletion plan fused with the host-to-device append (Section 3.3 item 2;
// one contiguous bundle per neuron, Section 3.2).  Work item q covers tail slot s = n' + q:
//   (1) if slot s is a live tail row, copy it to its hole;  (2) if q < |added|, read the
//   bundle of added[q] from pinned host memory and write it to slot s.
// Every 16-byte piece of slot s is read (1) and overwritten (2) by the same thread in
// program order, holes lie below n' and appends at or above it, so no two work items
// touch the same bytes.  grid-stride over (item, 16 KiB chunk); block = 256, four 16-byte
// loads per thread in flight.
// The host link wants FEW requests in flight: measured on MI355X / PCIe Gen5, 146 bundles of
// 16 KiB take 45 us with 32-64 workgroups (128-256 KiB in flight) and 58 us with 146 or more.
constexpr int kLoadPer = 4;
constexpr size_t kLoadChunk = 256 * 16 * kLoadPer;
constexpr int kLoadGrid = 32;

__global__ __launch_bounds__(256) void k_load(char* __restrict__ matrix, int32_t* __restrict__ pointers,
                                              float* __restrict__ bias, const char* __restrict__ host,
                                              const float* __restrict__ b, const int32_t* __restrict__ added,
                                              const int32_t* __restrict__ move_dst, size_t row_bytes, int F,
                                              DevState* st) {
    if (st->error) return;
    const int n2 = st->n_base, c = st->n_removed, a = st->n_added;
    const int items = max(c, a);
    const int cpr = (int)((row_bytes + kLoadChunk - 1) / kLoadChunk);
    const long long total = (long long)items * cpr;
    const int tid = threadIdx.x;
    for (long long it = blockIdx.x; it < total; it += gridDim.x) {
        const int q = (int)(it / cpr), ch = (int)(it - (long long)q * cpr);
        const int s = n2 + q;
        const int dst = (q < c) ? move_dst[q] : -1;
        int nid = (q < a) ? added[q] : -1;
        if (nid >= F) nid = -1;
        const size_t off0 = (size_t)ch * kLoadChunk + (size_t)tid * 16;
        const char* hsrc = host + (size_t)max(nid, 0) * row_bytes + off0;
        const char* msrc = matrix + (size_t)s * row_bytes + off0;
        char* mdst = matrix + (size_t)max(dst, 0) * row_bytes + off0;
        char* adst = matrix + (size_t)s * row_bytes + off0;
        uint4 hv[kLoadPer], mv[kLoadPer];
        bool ok[kLoadPer];
#pragma unroll
        for (int p = 0; p < kLoadPer; ++p) {
            ok[p] = off0 + (size_t)p * 4096 < row_bytes;
            hv[p] = make_uint4(0, 0, 0, 0);
            mv[p] = make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int p = 0; p < kLoadPer; ++p)
            if (ok[p] && nid >= 0) hv[p] = *reinterpret_cast<const uint4*>(hsrc + (size_t)p * 4096);
#pragma unroll
        for (int p = 0; p < kLoadPer; ++p)
            if (ok[p] && dst >= 0) mv[p] = *reinterpret_cast<const uint4*>(msrc + (size_t)p * 4096);
#pragma unroll
        for (int p = 0; p < kLoadPer; ++p)
            if (ok[p] && dst >= 0) *reinterpret_cast<uint4*>(mdst + (size_t)p * 4096) = mv[p];
#pragma unroll
        for (int p = 0; p < kLoadPer; ++p)
            if (ok[p] && nid >= 0) *reinterpret_cast<uint4*>(adst + (size_t)p * 4096) = hv[p];
        if (ch == 0 && tid == 0) {
            const int32_t old_ptr = pointers[s];
            const float old_bias = bias[s];
            if (dst >= 0) {
                pointers[dst] = old_ptr;
                bias[dst] = old_bias;
            }
            if (nid >= 0) {
                pointers[s] = nid;
                bias[s] = b[nid];
            }
        }
    }
    if (blockIdx.x == 0 && tid == 0) {
        st->num_used = n2 + a;
        st->c_h2d_bytes += (unsigned long long)a * row_bytes;
    }
}

// Empty cache: every neuron "never active", state and counters zero.
__global__ void k_reset(int32_t* __restrict__ last_active, int F, DevState* st) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    for (int j = i; j < F; j += gridDim.x * blockDim.x) last_active[j] = kNever;
    if (i == 0) {
        DevState z = {};
        *st = z;
    }
}

}  // namespace lif
