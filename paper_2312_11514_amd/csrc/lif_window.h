// Step 2: sliding window over the last k step masks (Section 3.1 "The Sliding Window
// Technique", Fig. 4b) and Step 3: neuron-cache update (Section 3.3 items 1-2, Fig. 6).
//
// Window state ("last_k_active") is a ring of the last k step masks, one bit per neuron:
// the active set is their bitwise OR, so a 64-bit word settles 64 neurons at once.
// Everything is integer work: results are exact.
#pragma once

#include "lif_common.h"

namespace lif {

constexpr int kScanThreads = 1024;   // single-workgroup kernels: 16 waves; one 64-neuron word or one 64-slot block per lane
constexpr int kMaxSpan = 64;         // d_ffn <= 1024 * 64; capacity <= 1024 * 64
constexpr int kHoleLds = 4096;       // holes kept in LDS; longer lists spill to the global scratch list
constexpr int kRingRegs = 8;         // window masks a lane keeps in registers (larger k takes a second pass)

// 64 mask bits starting at neuron 64 * w; the mask has nbytes bytes (a multiple of 8 bits, maybe not of 64)
__device__ __forceinline__ unsigned long long load_mask_word(const uint8_t* __restrict__ m, int w, int nbytes) {
    const int b0 = w * 8;
    if (b0 + 8 <= nbytes) return *reinterpret_cast<const unsigned long long*>(m + b0);
    unsigned long long v = 0;
    for (int i = 0; i < 8; ++i)
        if (b0 + i < nbytes) v |= (unsigned long long)m[b0 + i] << (8 * i);
    return v;
}

// Exclusive prefix sums of two counts per thread (each at most 64) in one pass over a workgroup of NW waves.
// Inside a wave both counts travel in one 32-bit value (a wave sums to at most 4096 per count); the totals of
// the waves are kept as two 32-bit halves of a 64-bit LDS word.  One barrier, two with GUARD (needed when
// wave_tot may still be read from an earlier scan that no barrier separates from this one).
template <int NW, bool GUARD>
__device__ __forceinline__ void block_exclusive_scan2(int va, int vb, unsigned long long* wave_tot, int* off_a,
                                                      int* off_b, int* tot_a, int* tot_b) {
    const int tid = threadIdx.x, lane = tid & (kWave - 1), w = tid >> 6;
    const int v = (vb << 16) | va;
    const int inc = wave_inclusive_scan(v, lane);
    if (GUARD) lds_barrier();
    if (lane == kWave - 1) wave_tot[w] = ((unsigned long long)(unsigned)(inc >> 16) << 32) | (unsigned)(inc & 0xffff);
    lds_barrier();
    unsigned long long before = 0, all = 0;
#pragma unroll
    for (int i = 0; i < NW; ++i) {
        const unsigned long long t = wave_tot[i];
        if (i < w) before += t;
        all += t;
    }
    const int ex = inc - v;                                  // exclusive inside the wave, both halves at once
    *off_a = (int)(unsigned)(before & 0xffffffffull) + (ex & 0xffff);
    *off_b = (int)(unsigned)(before >> 32) + (ex >> 16);
    *tot_a = (int)(unsigned)(all & 0xffffffffull);
    *tot_b = (int)(unsigned)(all >> 32);
}

// One workgroup does the window update and the deletion plan back to back.
//
// Window (Section 3.1): ring[j] holds the step masks of the last k steps; step t overwrites
// ring[t mod k].  Lane w owns the 64 neurons of word w:
//   prev = OR of all ring words (S_{t-1});  keep = OR of all but ring[t mod k];  S_t = keep | m
//   added = m & ~prev;  removed = prev & ~(keep | m)
// A workgroup-wide prefix sum over the popcounts puts the ids out in ascending order.
//
// Deletion plan (Section 3.3 item 1): a slot is dead iff its neuron was just removed (looked
// up in the removed words, kept in LDS).  With n' = n - c, the dead slots below n' ("holes",
// ascending) are filled by the live slots at or above n' ("fillers"): hole j takes the
// (H-1-j)-th filler - the lowest hole receives the last row, exactly what the sequential
// swap-with-last loop does.  Sources (>= n') and destinations (< n') are disjoint, so the
// moves can later run in any order.  Slots are walked in blocks of 64 (one per lane), block b
// by wave b mod 16; ballots rank the slots inside a block, a prefix over the per-block counts
// ranks the blocks.  Only the blocks below num_used are visited.
// Output of the plan: move_dst[q] for tail slot n' + q = destination slot, or -1 if dead.
//
// The loads that do not depend on the state (mask word, ring words, first block of pointers)
// are issued together with the state itself.
__global__ __launch_bounds__(kScanThreads) void k_window_plan(
    const uint8_t* __restrict__ step_mask, int ntok, int keep_tok, unsigned long long* __restrict__ ring,
    unsigned long long* __restrict__ cur_set, int ring_words, const int32_t* __restrict__ pointers, int F, int k,
    int capacity, int shrink, int32_t* __restrict__ added,
    int32_t* __restrict__ n_added, int32_t* __restrict__ removed, int32_t* __restrict__ n_removed,
    int32_t* __restrict__ move_dst, int32_t* __restrict__ hole_list, DevState* st) {
    constexpr int THREADS = kScanThreads;
    constexpr int NW = THREADS / kWave;
    __shared__ unsigned long long wave_tot[NW];
    __shared__ unsigned long long rem64[THREADS];
    __shared__ int hole_lds[kHoleLds];
    __shared__ int blk_h[THREADS], blk_f[THREADS];                // per 64-slot block: counts, then exclusive prefixes
    __shared__ int cnt_age[264];                                  // dynamic window: |union of the newest a masks| (a <= 256)
    const int tid = threadIdx.x, lane = tid & (kWave - 1), w = tid >> 6;
    const unsigned long long lt = (1ull << lane) - 1ull;
    const int nwords = (F + 63) >> 6, nbytes = F >> 3;
    const bool have = tid < nwords;

    // ---- issue the state-independent loads ----
    unsigned long long m = have ? load_mask_word(step_mask, tid, nbytes) : 0ull;   // first (or only) mask of the step
    const unsigned long long cur = have ? cur_set[tid] : 0ull;                       // what the cache holds now
    unsigned long long rv[kRingRegs];
#pragma unroll
    for (int j = 0; j < kRingRegs; ++j) rv[j] = (have && j < k) ? ring[(size_t)j * ring_words + tid] : 0ull;
    // slot owners of the first blocks of this wave (4096 slots over the workgroup), for the deletion plan below; the
    // array spans the capacity, entries past num_used are masked when used
    constexpr int kPtrPre = 64 / NW;
    int idpre[kPtrPre];
#pragma unroll
    for (int it = 0; it < kPtrPre; ++it) {
        const int s = (w + it * NW) * kWave + lane;
        idpre[it] = (s < capacity) ? pointers[s] : -1;
    }
    const int err = st->error;
    const int t = st->step;
    const int n = st->num_used;
    const int wl_prev = st->window_len;
    const int pos = st->ring_pos;

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
    const int slot = pos % k;                            // ring entry that this step's (first) mask replaces
    const unsigned long long prev = cur;
    unsigned long long keep = 0;
#pragma unroll
    for (int j = 0; j < kRingRegs; ++j)
        if (j != slot) keep |= rv[j];
    if (have) {
        for (int j = kRingRegs; j < k; ++j) {                 // only for windows longer than kRingRegs steps
            const unsigned long long v = ring[(size_t)j * ring_words + tid];
            if (j != slot) keep |= v;
        }
    }
    unsigned long long now = keep | m;                   // S_t with the full window
    int k_eff = k;
    const bool multi = ntok != 1 || keep_tok != 1;
    if (multi) {
        // Several tokens in one step (speculative verification, Section 4.3 "Speculative Decoding" and the
        // related-work note that the window is then updated with several tokens at once): all ntok masks
        // are needed for this step's FFN, but only the first keep_tok of them enter the window (one ring
        // entry per token, as if pushed one after the other); the others are transient.
        const size_t row_bytes = (size_t)nbytes;           // the host checks F % 64 == 0 for this path
        now = 0ull;
        if (have) {
            for (int i = 0; i < ntok; ++i) now |= load_mask_word(step_mask + (size_t)i * row_bytes, tid, nbytes);
            for (int j = 0; j < k; ++j) {
                const int since = j - pos + (j < pos ? k : 0);   // (j - pos) mod k: this entry is overwritten by kept token `since`
                if (since >= keep_tok) now |= ring[(size_t)j * ring_words + tid];
            }
        }
    }
    if (shrink && multi) {
        // Dynamic window for a pass of several tokens (Section 4.3 with the Appendix's dynamic window): T = all
        // masks of the pass is held in any case; the window after the pass - its masks by age a = 1 (newest)
        // .. k: the kept tokens, newest first, then the ring entries the pass does not overwrite - keeps the
        // newest k_eff masks, k_eff the largest count for which |T u U_a| fits the capacity (cnt_age[a], a = 0
        // .. k; the counts grow with a).  The kept tokens are subsets of T, so they always stay.
        auto age_mask = [&](int a) -> unsigned long long {        // mask of age a (1 <= a <= k), word of this lane
            if (a <= keep_tok) return load_mask_word(step_mask + (size_t)(keep_tok - a) * nbytes, tid, nbytes);
            const int m_old = a - keep_tok;                        // m_old-th most recent entry written before this pass
            return ring[(size_t)(((pos - m_old) % k + k) % k) * ring_words + tid];
        };
        for (int a = tid; a <= k; a += THREADS) cnt_age[a] = 0;
        __syncthreads();
        unsigned long long u = 0ull;
        if (have)
            for (int i = 0; i < ntok; ++i) u |= load_mask_word(step_mask + (size_t)i * nbytes, tid, nbytes);
        const unsigned long long pass_all = u;
        if (u) atomicAdd(&cnt_age[0], __popcll(u));
        for (int a = 1; a <= k; ++a) {
            if (have) u |= age_mask(a);
            if (u) atomicAdd(&cnt_age[a], __popcll(u));
        }
        __syncthreads();
        k_eff = -1;
        for (int a = 0; a <= k; ++a)
            if (cnt_age[a] <= capacity) k_eff = a;
        if (k_eff < 0) {                                     // uniform: the masks of the pass alone do not fit
            if (tid == 0) {
                st->error = 3;                               // LIF_CAPACITY
                *n_added = 0;
                *n_removed = 0;
                st->n_added = 0;
                st->n_removed = 0;
            }
            return;
        }
        now = pass_all;
        if (have)
            for (int a = 1; a <= k_eff; ++a) now |= age_mask(a);
    }
    if (shrink && !multi) {
        // Dynamic window (Appendix, Persimmon / Phi-2: the window is reduced whenever the cache would
        // pass its memory limit): keep the newest k_eff <= k masks, k_eff the largest count whose
        // union fits the capacity.  U_a = union of the newest a masks (a = 1: this step's mask).
        for (int a = tid; a < k; a += THREADS) cnt_age[a] = 0;
        __syncthreads();
        unsigned long long ua[kRingRegs];                // ua[a - 1] = U_a, a = 1 .. min(k, kRingRegs)
        if (k <= kRingRegs && tid >= ((nwords + kWave - 1) & ~(kWave - 1))) {
            // this wave holds no mask word: nothing to count (all 16 waves share one compute unit, so the
            // idle ones would only slow the few that hold the masks)
#pragma unroll
            for (int a = 0; a < kRingRegs; ++a) ua[a] = 0ull;
        } else if (k <= kRingRegs) {
            // The ring entries in order of age (entry slot - a holds the mask pushed a steps ago) are picked out of the
            // register copy with selects on the wave-uniform index: some hundred instructions, but no second trip
            // to memory (measured: this phase 3.0 us with the reload).  Per-wave sums (two 16-bit counts per word) by
            // a prefix sum of DPP moves whose last lane holds the total, then one LDS atomic per wave and age.
            unsigned long long e[kRingRegs];
#pragma unroll
            for (int a = 1; a < kRingRegs; ++a) {
                const int idx = slot - a + (slot < a ? k : 0);
                unsigned long long v = 0ull;
#pragma unroll
                for (int j = 0; j < kRingRegs; ++j)
                    if (j == idx) v = rv[j];
                e[a] = (a < k) ? v : 0ull;
            }
            unsigned long long u = m;
            ua[0] = u;
#pragma unroll
            for (int a = 1; a < kRingRegs; ++a) {
                u |= e[a];
                ua[a] = u;
            }
#pragma unroll
            for (int i = 0; i < kRingRegs / 2; ++i) {
                const int pk = __popcll(ua[2 * i]) | (__popcll(ua[2 * i + 1]) << 16);       // 64 lanes x 64 bits < 2^16
                const int v = __builtin_amdgcn_readlane(wave_inclusive_scan(pk, lane), kWave - 1);
                if (lane == 0 && v) {
                    if (2 * i < k) atomicAdd(&cnt_age[2 * i], v & 0xffff);
                    if (2 * i + 1 < k) atomicAdd(&cnt_age[2 * i + 1], (int)((unsigned)v >> 16));
                }
            }
        } else {
            unsigned long long u = m;
            for (int a = 1; a <= k; ++a) {
                if (a > 1 && have) u |= ring[(size_t)((slot - (a - 1) + k) % k) * ring_words + tid];
                const int pc = __popcll(u);
                if (pc) atomicAdd(&cnt_age[a - 1], pc);
            }
        }
        __syncthreads();
        k_eff = 0;
        if (k <= kRingRegs) {
#pragma unroll
            for (int a = 1; a <= kRingRegs; ++a)
                if (a <= k && cnt_age[a - 1] <= capacity) k_eff = a;   // the counts grow with a
        } else {
            for (int a = 1; a <= k; ++a)
                if (cnt_age[a - 1] <= capacity) k_eff = a;
        }
        if (k_eff == 0) {                                    // uniform: this step's mask alone does not fit
            if (tid == 0) {
                st->error = 3;                               // LIF_CAPACITY
                *n_added = 0;
                *n_removed = 0;
                st->n_added = 0;
                st->n_removed = 0;
            }
            return;
        }
        now = m;
        if (k <= kRingRegs) {
#pragma unroll
            for (int a = 1; a < kRingRegs; ++a)
                if (a < k_eff) now = ua[a];                  // U_a grows with a: the last one taken is U_{k_eff}
        } else if (have) {
            for (int a = 2; a <= k_eff; ++a) now |= ring[(size_t)((slot - (a - 1) + k) % k) * ring_words + tid];
        }
    }
    unsigned long long abits = now & ~prev;
    unsigned long long rbits = prev & ~now;
    int off_a, off_r, tot_a, tot_r;
    block_exclusive_scan2<NW, false>(__popcll(abits), __popcll(rbits), wave_tot, &off_a, &off_r, &tot_a, &tot_r);

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
    rem64[tid] = rbits;
    lds_barrier();                                   // rem64 is read below

    // ---- deletion plan: classify the slots below n, block by block ----
    const int nblk = (n + kWave - 1) >> 6;           // <= 1024
    unsigned long long holebits = 0, fillbits = 0;   // bit it = flag of this lane in its it-th block
    for (int b = w, it = 0; b < nblk; b += NW, ++it) {
        const int s = b * kWave + lane;
        int id;
        if (it < kPtrPre) {                          // requested with the state
            id = idpre[0];
#pragma unroll
            for (int q = 1; q < kPtrPre; ++q)
                if (it == q) id = idpre[q];
            if (s >= n) id = -1;
        } else {
            id = (s < n) ? pointers[s] : -1;
        }
        bool hole = false, fill = false;
        if (s < n) {
            const bool dead = (id < 0 || id >= F) ? true : ((rem64[id >> 6] >> (id & 63)) & 1ull);
            hole = s < n2 && dead;
            fill = s >= n2 && !dead;
        }
        if (hole) holebits |= 1ull << it;
        if (fill) fillbits |= 1ull << it;
        const int ch = __popcll(__ballot(hole)), cf = __popcll(__ballot(fill));
        if (lane == 0) {
            blk_h[b] = ch;
            blk_f[b] = cf;
        }
    }
    lds_barrier();
    int H, Fc;
    // At most 64 blocks in use (4096 rows): every wave scans the block counts itself (one DPP prefix sum over
    // the lanes, both counts in one value) and picks the prefixes of its own blocks out of the lanes: no scan
    // across waves, no write-back, two barriers fewer.
    const bool few = nblk <= kWave;                  // uniform
    int ex_few = 0;
    if (few) {
        const int v = (lane < nblk) ? (blk_h[lane] | (blk_f[lane] << 16)) : 0;
        const int inc = wave_inclusive_scan(v, lane);
        ex_few = inc - v;
        const int tot = __builtin_amdgcn_readlane(inc, kWave - 1);
        H = tot & 0xffff;
        Fc = tot >> 16;
    } else {
        int pre_h, pre_f;
        const int vh = (tid < nblk) ? blk_h[tid] : 0, vf = (tid < nblk) ? blk_f[tid] : 0;
        block_exclusive_scan2<NW, false>(vh, vf, wave_tot, &pre_h, &pre_f, &H, &Fc);
        // the scan's barrier separates the reads of the counts above from these writes
        blk_h[tid] = pre_h;
        blk_f[tid] = pre_f;
        lds_barrier();
    }
    const bool in_lds = H <= kHoleLds;
    for (int b = w, it = 0; b < nblk; b += NW, ++it) {
        const bool hole = (holebits >> it) & 1ull;
        const unsigned long long bh = __ballot(hole);
        const int ph = few ? (__builtin_amdgcn_readlane(ex_few, b) & 0xffff) : blk_h[b];
        if (hole) {
            const int pos = ph + __popcll(bh & lt);
            if (in_lds) hole_lds[pos] = b * kWave + lane;
            else hole_list[pos] = b * kWave + lane;
        }
    }
    // the hole list (LDS, or global scratch when long) is read by other threads below
    if (in_lds) lds_barrier();
    else __syncthreads();
    for (int b = w, it = 0; b < nblk; b += NW, ++it) {
        const int s = b * kWave + lane;
        const bool fill = (fillbits >> it) & 1ull;
        const unsigned long long bf = __ballot(fill);
        const int pf = few ? (int)((unsigned)__builtin_amdgcn_readlane(ex_few, b) >> 16) : blk_f[b];
        if (s >= n2 && s < n) {
            int dst = -1;
            if (fill) {
                const int q = H - 1 - (pf + __popcll(bf & lt));
                if (q >= 0 && q < H) dst = in_lds ? hole_lds[q] : hole_list[q];
            }
            move_dst[s - n2] = dst;
        }
    }
    // ---- the new window and the id lists go out last: nothing in this kernel reads them back, and the plan above
    // does not wait for them ----
    if (have) {
        cur_set[tid] = now;
        if (!multi) {
            ring[(size_t)slot * ring_words + tid] = m;
            for (int a = k_eff + 1; a <= k; ++a)             // masks dropped by the dynamic window leave it for good
                ring[(size_t)((slot - (a - 1) + k) % k) * ring_words + tid] = 0ull;
        } else {
            for (int i = max(0, keep_tok - k); i < keep_tok; ++i)
                ring[(size_t)((pos + i) % k) * ring_words + tid] =
                    load_mask_word(step_mask + (size_t)i * nbytes, tid, nbytes);
            // entries written before this pass that the dynamic window dropped (ages above k_eff) leave for good
            for (int m_old = max(k_eff - keep_tok, 0) + 1; m_old <= k - keep_tok; ++m_old)
                ring[(size_t)(((pos - m_old) % k + k) % k) * ring_words + tid] = 0ull;
        }
    }
    while (abits) {
        added[off_a++] = tid * 64 + __ffsll((long long)abits) - 1;
        abits &= abits - 1;
    }
    while (rbits) {
        removed[off_r++] = tid * 64 + __ffsll((long long)rbits) - 1;
        rbits &= rbits - 1;
    }
    if (tid == 0) {
        *n_added = tot_a;
        *n_removed = tot_r;
        st->n_added = tot_a;
        st->n_removed = tot_r;
        st->n_base = n2;
        st->n_moved = H;
        st->window_len = multi ? min(min(wl_prev + keep_tok, k), k_eff) : min(min(wl_prev + 1, k), k_eff);
        st->ring_pos = (pos + (multi ? keep_tok : 1)) % k;
        st->step = t + 1;
        atomicAdd(&st->c_steps, 1ull);
        atomicAdd(&st->c_added, (unsigned long long)tot_a);
        atomicAdd(&st->c_removed, (unsigned long long)tot_r);
        atomicAdd(&st->c_rows_moved, (unsigned long long)H);
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

// `block` / `nblocks`: index and count of the workgroups that share this role.
__device__ __forceinline__ void load_rows_role(char* __restrict__ matrix, int32_t* __restrict__ pointers,
                                               float* __restrict__ bias, const HostStore host,
                                               const float* __restrict__ b, const int32_t* __restrict__ added,
                                               const int32_t* __restrict__ move_dst, size_t row_bytes, int F,
                                               int block, int nblocks, DevState* st) {
    if (st->error) return;
    const int n2 = st->n_base, c = st->n_removed, a = st->n_added;
    const int items = max(c, a);
    const int cpr = (int)((row_bytes + kLoadChunk - 1) / kLoadChunk);
    const long long total = (long long)items * cpr;
    const int tid = threadIdx.x;
    for (long long it = block; it < total; it += nblocks) {
        const int q = (int)(it / cpr), ch = (int)(it - (long long)q * cpr);
        const int s = n2 + q;
        const int dst = (q < c) ? move_dst[q] : -1;
        int nid = (q < a) ? added[q] : -1;
        if (nid >= F) nid = -1;
        const size_t off0 = (size_t)ch * kLoadChunk + (size_t)tid * 16;
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
            if (ok[p] && nid >= 0)
                hv[p] = *reinterpret_cast<const uint4*>(host_piece(host, nid, off0 + (size_t)p * 4096, row_bytes));
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
    if (block == 0 && tid == 0) {
        st->num_used = n2 + a;
        atomicAdd(&st->c_h2d_bytes, (unsigned long long)a * row_bytes);
    }
}

__global__ __launch_bounds__(256) void k_load(char* __restrict__ matrix, int32_t* __restrict__ pointers,
                                              float* __restrict__ bias, const HostStore host,
                                              const float* __restrict__ b, const int32_t* __restrict__ added,
                                              const int32_t* __restrict__ move_dst, size_t row_bytes, int F,
                                              DevState* st) {
    load_rows_role(matrix, pointers, bias, host, b, added, move_dst, row_bytes, F, blockIdx.x, gridDim.x, st);
}

// Empty cache: no mask in the window, state and counters zero.
// (ring_total_words covers the ring and the current-set bitmap that follows it)
__global__ void k_reset(unsigned long long* __restrict__ ring, int ring_total_words, int32_t* __restrict__ stamp,
                        int capacity, DevState* st) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    for (int j = i; j < ring_total_words; j += gridDim.x * blockDim.x) ring[j] = 0ull;
    for (int j = i; j < capacity; j += gridDim.x * blockDim.x) stamp[j] = -1;   // no activation from a fused step
    if (i == 0) {
        DevState z = {};
        *st = z;
    }
}

}  // namespace lif
