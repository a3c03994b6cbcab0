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

// One workgroup walks all F neurons in thread-contiguous spans, so that a workgroup-wide
// prefix sum over per-thread popcounts yields ids in ascending order.
// span = neurons per thread, multiple of 8, <= 64.
__global__ __launch_bounds__(kScanThreads) void k_window(const uint8_t* __restrict__ step_mask,
                                                         int32_t* __restrict__ last_active, int F, int k,
                                                         int capacity, int span, int32_t* __restrict__ added,
                                                         int32_t* __restrict__ n_added,
                                                         int32_t* __restrict__ removed,
                                                         int32_t* __restrict__ n_removed, DevState* st) {
    __shared__ int wave_tot[kScanThreads / kWave];
    const int tid = threadIdx.x;
    if (st->error) {
        if (tid == 0) {
            *n_added = 0;
            *n_removed = 0;
            st->n_added = 0;
            st->n_removed = 0;
        }
        return;
    }
    const int t = st->step;
    const int n_prev = st->num_used;
    const int i0 = tid * span;
    unsigned long long abits = 0, rbits = 0, mbits = 0;
    for (int g = 0; g < span; g += 8) {
        const int i = i0 + g;
        if (i < F) {
            const unsigned m = step_mask[i >> 3];
            const int4 la0 = *reinterpret_cast<const int4*>(last_active + i);
            const int4 la1 = *reinterpret_cast<const int4*>(last_active + i + 4);
            const int la[8] = {la0.x, la0.y, la0.z, la0.w, la1.x, la1.y, la1.z, la1.w};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const bool in_prev = la[e] >= t - k;               // in S_{t-1}
                const bool hit = (m >> e) & 1u;
                const bool in_now = hit || la[e] >= t - k + 1;     // in S_t
                const unsigned long long bit = 1ull << (g + e);
                if (hit) mbits |= bit;
                if (in_now && !in_prev) abits |= bit;
                if (in_prev && !in_now) rbits |= bit;
            }
        }
    }
    int tot_a, tot_r;
    int off_a = block_exclusive_scan(__popcll(abits), wave_tot, &tot_a);
    int off_r = block_exclusive_scan(__popcll(rbits), wave_tot, &tot_r);

    if (n_prev + tot_a - tot_r > capacity) {       // uniform: leave the window untouched
        if (tid == 0) {
            st->error = 3;                          // LIF_CAPACITY
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
        removed[off_r++] = i0 + bpos;
        rbits &= rbits - 1;
    }
    while (mbits) {
        const int bpos = __ffsll((long long)mbits) - 1;
        last_active[i0 + bpos] = t;
        mbits &= mbits - 1;
    }
    if (tid == 0) {
        *n_added = tot_a;
        *n_removed = tot_r;
        st->n_added = tot_a;
        st->n_removed = tot_r;
        st->step = t + 1;
        st->c_steps += 1;
        st->c_added += (unsigned long long)tot_a;
        st->c_removed += (unsigned long long)tot_r;
    }
}

// Deletion plan.  A slot is dead iff its neuron left the window.  With n' = n - #dead, the
// dead slots below n' ("holes", ascending) are filled by the live slots at or above n'
// ("fillers"): hole j takes the (H-1-j)-th filler - the lowest hole receives the last row,
// exactly what the sequential swap-with-last loop does.  Sources (>= n') and destinations
// (< n') are disjoint, so the moves can run in any order.
// Output: move_dst[q] for tail slot n' + q: destination slot, or -1 if that slot is dead.
// span = slots per thread (<= 64), capacity <= 1024 * span.
__global__ __launch_bounds__(kScanThreads) void k_plan(const int32_t* __restrict__ pointers,
                                                       const int32_t* __restrict__ last_active,
                                                       const int32_t* __restrict__ n_added_p, int F, int k,
                                                       int capacity, int span, int32_t* __restrict__ move_dst,
                                                       int32_t* __restrict__ hole_list, DevState* st) {
    __shared__ int wave_tot[kScanThreads / kWave];
    const int tid = threadIdx.x;
    if (st->error) return;
    const int n = st->num_used;
    const int horizon = st->step - k;      // dead iff last_active < step - k (step already advanced)
    const int s0 = tid * span;
    unsigned long long deadbits = 0;
    for (int q = 0; q < span; ++q) {
        const int s = s0 + q;
        if (s < n) {
            const int id = pointers[s];
            const bool dead = (id < 0 || id >= F) ? true : (last_active[id] < horizon);
            if (dead) deadbits |= 1ull << q;
        }
    }
    int c;
    block_exclusive_scan(__popcll(deadbits), wave_tot, &c);
    const int n2 = n - c;
    unsigned long long holebits = 0, fillbits = 0;
    for (int q = 0; q < span; ++q) {
        const int s = s0 + q;
        if (s < n) {
            const bool dead = (deadbits >> q) & 1ull;
            if (s < n2 && dead) holebits |= 1ull << q;
            if (s >= n2 && !dead) fillbits |= 1ull << q;
        }
    }
    int H, Fc;
    int off_h = block_exclusive_scan(__popcll(holebits), wave_tot, &H);
    int off_f = block_exclusive_scan(__popcll(fillbits), wave_tot, &Fc);
    {
        unsigned long long hb = holebits;
        while (hb) {
            const int q = __ffsll((long long)hb) - 1;
            hole_list[off_h++] = s0 + q;
            hb &= hb - 1;
        }
    }
    __syncthreads();   // hole_list (global) is read by other threads of this workgroup below
    for (int q = 0; q < span; ++q) {
        const int s = s0 + q;
        if (s >= n2 && s < n) {
            int dst = -1;
            if ((fillbits >> q) & 1ull) {
                dst = hole_list[H - 1 - off_f];
                ++off_f;
            }
            move_dst[s - n2] = dst;
        }
    }
    if (tid == 0) {
        int a = *n_added_p;
        a = max(0, min(a, capacity - n2));
        st->n_base = n2;
        st->n_removed = c;
        st->n_added = a;
        st->n_moved = H;
        st->c_rows_moved += (unsigned long long)H;
    }
}

// Row moves of the deletion plan fused with the host-to-device append (Section 3.3 item 2;
// one contiguous bundle per neuron, Section 3.2).  Work item q covers tail slot s = n' + q:
//   (1) if slot s is a live tail row, copy it to its hole;  (2) if q < |added|, read the
//   bundle of added[q] from pinned host memory and write it to slot s.
// Every 16-byte piece of slot s is read (1) and overwritten (2) by the same thread in
// program order, holes lie below n' and appends at or above it, so no two work items
// touch the same bytes.  grid-stride over (item, 4 KiB chunk); block = 256.
__global__ __launch_bounds__(256) void k_load(char* __restrict__ matrix, int32_t* __restrict__ pointers,
                                              float* __restrict__ bias, const char* __restrict__ host,
                                              const float* __restrict__ b, const int32_t* __restrict__ added,
                                              const int32_t* __restrict__ move_dst, size_t row_bytes, int F,
                                              DevState* st) {
    if (st->error) return;
    const int n2 = st->n_base, c = st->n_removed, a = st->n_added;
    const int items = max(c, a);
    const int cpr = (int)((row_bytes + 4095) / 4096);
    const long long total = (long long)items * cpr;
    const int tid = threadIdx.x;
    for (long long it = blockIdx.x; it < total; it += gridDim.x) {
        const int q = (int)(it / cpr), ch = (int)(it - (long long)q * cpr);
        const size_t off = (size_t)ch * 4096 + (size_t)tid * 16;
        const bool inb = off < row_bytes;
        const int s = n2 + q;
        const int dst = (q < c) ? move_dst[q] : -1;
        int nid = (q < a) ? added[q] : -1;
        if (nid >= F) nid = -1;
        uint4 mv = {0, 0, 0, 0}, hv = {0, 0, 0, 0};
        if (inb && dst >= 0) mv = *reinterpret_cast<const uint4*>(matrix + (size_t)s * row_bytes + off);
        if (inb && nid >= 0) hv = *reinterpret_cast<const uint4*>(host + (size_t)nid * row_bytes + off);
        if (inb && dst >= 0) *reinterpret_cast<uint4*>(matrix + (size_t)dst * row_bytes + off) = mv;
        if (inb && nid >= 0) *reinterpret_cast<uint4*>(matrix + (size_t)s * row_bytes + off) = hv;
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
