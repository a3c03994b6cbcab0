// Fused cache update + activation stage (lif_step, lif_step_tokens).
//
// The host-to-device gather of new bundles is bound by the host link and keeps only ~32
// workgroups busy for tens of microseconds (Section 3.3 item 2), while the activation stage of
// the FFN (Section 3.3 item 3) streams the rows that are already resident.  Both only need the
// token's x and the deletion plan, so one launch runs them side by side:
//   workgroups [0, load_wgs)       loader role: row moves + pinned-host appends with the layout of
//                                  k_load, and - since every bundle passes through their registers -
//                                  the activation of each row they write (h_new, stamped with the step);
//   workgroups [load_wgs, ...)     activation role over the rows kept by the deletion (slots < n').
// The activation role may read a hole while a loader overwrites it; that value is never used,
// because the loader's stamped activation takes precedence in the down-projection kernel.
#pragma once

#include "lif_ffn.h"
#include "lif_ffn_mfma.h"
#include "lif_window.h"

namespace lif {

// The host link runs best with a few hundred KiB of reads outstanding: a read-only gather of 146 bundles of
// 16 KiB measured 52 GB/s with 256 KiB in flight in pieces of 1 to 8 KiB per wave, 50 GB/s with 384 KiB,
// 42 GB/s with 16 KiB pieces.
// The number of loader wave pairs (one bundle in flight per pair, one wave per workgroup so that they spread
// over compute units) is therefore chosen from the bundle size: kStepInflightBytes / bundle bytes, within 5..32.
constexpr int kStepInflightBytes = 256 * 1024;
constexpr int kStepLoadWaves = 1;                     // waves of a loader workgroup that load (the others exit at once)

// Loader role.  Work item q covers tail slot s = n' + q (see k_load) and is shared by a PAIR of waves:
// wave 2p takes the vectors the activation needs (gate | up), wave 2p + 1 the down vector, so a bundle
// crosses the host link as two request streams of d * E bytes (measured: 8 KiB pieces with 32 waves move
// 4 % more than 16 KiB pieces with 16 waves at the same bytes in flight, and the tail - the last items,
// when most waves have run out of work - is half as long).  Each wave requests its part of the host bundle of
// added[q] first (the long latency), moves its part of the live tail row to its hole meanwhile, then writes
// the bundle part to slot s.  In the activation wave, lane l holds the same 16-byte pieces of every vector as
// in the activation role (piece it * 64 + l), keeps x in registers the same way and sums in the same order, so
// the activations it writes are bit for bit those the activation kernel would compute; it also does the
// bookkeeping of the slot (pointers, bias).  nwaves must be even.  Rows of at most 2 KiB per vector (NI <= 2)
// are not split: one wave takes the whole bundle.
template <typename T, int NI, bool GLU>
__device__ __forceinline__ void load_role(T* __restrict__ matrix, int32_t* __restrict__ pointers,
                                          float* __restrict__ bias, const HostStore host,
                                          const float* __restrict__ b, const int32_t* __restrict__ added,
                                          const int32_t* __restrict__ move_dst, size_t row_elems, int F, int d,
                                          int capacity, const T* __restrict__ x, float* __restrict__ h_new,
                                          int32_t* __restrict__ stamp, const float* __restrict__ gact, int wave_id,
                                          int nwaves, DevState* st) {
    using V = typename Vec<T>::type;
    constexpr int VE = Vec<T>::N;
    constexpr bool PAIRED = NI > 2;                      // vectors of up to 2 KiB: one wave per bundle (halves of
                                                         // small bundles cross the host link badly)
    constexpr int GA = PAIRED ? (GLU ? 2 : 1) : (GLU ? 3 : 2);   // vectors a wave handles at most
    const int lane = threadIdx.x & 63;
    const int nvec = d / VE;
    const int part = PAIRED ? (wave_id & 1) : 0;         // 0: activation vectors and bookkeeping, 1: down vector
    const int pair_id = PAIRED ? (wave_id >> 1) : wave_id, pairs = PAIRED ? (nwaves >> 1) : nwaves;
    const int g0 = part ? GA : 0;                        // first vector of this wave's part
    const int gn = part ? 1 : GA;                        // number of vectors in it
    const bool act_wave = part == 0;
    const size_t row_bytes = row_elems * sizeof(T);
    const V* xv = reinterpret_cast<const V*>(x);
    V xr[NI];
#pragma unroll
    for (int it = 0; it < NI; ++it) {
        const int idx = it * 64 + lane;
        xr[it] = (act_wave && idx < nvec) ? xv[idx] : V(0);
    }
    // The bookkeeping of the first 64 work items of this wave (one per lane) is requested together
    // with the state, before the counts are known (the arrays span the whole capacity; entries past
    // the counts are masked afterwards): one device-memory round trip in front of the host reads.
    int dst_l = -1, nid_l = -1;
    {
        const int ql = pair_id + lane * pairs;
        if (ql < capacity) dst_l = move_dst[ql];
        if (ql < F) nid_l = added[ql];
    }
    if (st->error) return;
    const int n2 = st->n_base, c = st->n_removed, a = st->n_added, step = st->step;
    const int items = max(c, a);
    for (int q0 = pair_id; q0 < items; q0 += pairs * kWave) {
      const int ql = q0 + lane * pairs;                  // work item of this lane
      if (q0 != pair_id) {                               // later batches (more than 64 items per wave)
          dst_l = (ql < c) ? move_dst[ql] : -1;
          nid_l = (ql < a) ? added[ql] : -1;
      }
      if (ql >= c) dst_l = -1;
      if (ql >= a || nid_l >= F) nid_l = -1;
      int optr_l = -1;
      float obias_l = 0.f, nbias_l = 0.f;
      float ogate_l = 0.f, ngate_l = 0.f;                // resident-gate activations of the moved / new neuron
      if (act_wave && ql < items) {
          optr_l = pointers[n2 + ql];
          obias_l = bias[n2 + ql];
          if (nid_l >= 0) nbias_l = b[nid_l];
          if (gact) {
              if (nid_l >= 0) ngate_l = gact[nid_l];
              if (optr_l >= 0 && optr_l < F) ogate_l = gact[optr_l];
          }
      }
      const int nitems = min(kWave, (items - q0 + pairs - 1) / pairs);
      // Software pipeline over the items of this wave: the reads of item j+1 are requested as soon
      // as the registers of item j are free (after its stores and per-lane dot products) and fly
      // while item j's wave reductions and bookkeeping writes complete.  Device rows (the move) are
      // requested before host rows so that waiting for them does not wait for the host link.
      int dst = __shfl(dst_l, 0, kWave), nid = __shfl(nid_l, 0, kWave);
      V hv[GA][NI], mv[GA][NI];
      {
          const V* srow = reinterpret_cast<const V*>(matrix + (size_t)(n2 + q0) * row_elems) + (size_t)g0 * nvec;
#pragma unroll
          for (int g = 0; g < GA; ++g)
#pragma unroll
              for (int it = 0; it < NI; ++it) {
                  const int idx = it * 64 + lane;
                  mv[g][it] = (dst >= 0 && g < gn && idx < nvec) ? srow[g * nvec + idx] : V(0);
              }
#pragma unroll
          for (int g = 0; g < GA; ++g)
#pragma unroll
              for (int it = 0; it < NI; ++it) {
                  const int idx = it * 64 + lane;
                  hv[g][it] = (nid >= 0 && g < gn && idx < nvec)
                                  ? *reinterpret_cast<const V*>(host_piece(host, nid, ((size_t)(g0 + g) * nvec + idx) * 16, row_bytes))
                                  : V(0);
              }
      }
      for (int j = 0; j < nitems; ++j) {
        const int s = n2 + q0 + j * pairs;
        V* srow = reinterpret_cast<V*>(matrix + (size_t)s * row_elems) + (size_t)g0 * nvec;
        V* drow = reinterpret_cast<V*>(matrix + (size_t)max(dst, 0) * row_elems) + (size_t)g0 * nvec;
        const int32_t old_ptr = __shfl(optr_l, j, kWave);
        const float old_bias = __shfl(obias_l, j, kWave);
        const float new_bias = __shfl(nbias_l, j, kWave);
        const float old_gate = __shfl(ogate_l, j, kWave), new_gate = __shfl(ngate_l, j, kWave);
        float mdu = 0.f, mdg = 0.f, hdu = 0.f, hdg = 0.f;
        if (dst >= 0) {                                   // wave-uniform
#pragma unroll
            for (int g = 0; g < GA; ++g)
#pragma unroll
                for (int it = 0; it < NI; ++it) {
                    const int idx = it * 64 + lane;
                    if (g < gn && idx < nvec) drow[g * nvec + idx] = mv[g][it];
                }
            if (act_wave) {
#pragma unroll
                for (int it = 0; it < NI; ++it) {
                    mdu = dot_acc(mv[GLU ? 1 : 0][it], xr[it], mdu);
                    if (GLU) mdg = dot_acc(mv[0][it], xr[it], mdg);
                }
            }
        }
        if (nid >= 0) {                                   // wave-uniform
#pragma unroll
            for (int g = 0; g < GA; ++g)
#pragma unroll
                for (int it = 0; it < NI; ++it) {
                    const int idx = it * 64 + lane;
                    if (g < gn && idx < nvec) srow[g * nvec + idx] = hv[g][it];
                }
            if (act_wave) {
#pragma unroll
                for (int it = 0; it < NI; ++it) {
                    hdu = dot_acc(hv[GLU ? 1 : 0][it], xr[it], hdu);
                    if (GLU) hdg = dot_acc(hv[0][it], xr[it], hdg);
                }
            }
        }
        // request item j + 1
        const int dst_n = (j + 1 < nitems) ? __shfl(dst_l, j + 1, kWave) : -1;
        const int nid_n = (j + 1 < nitems) ? __shfl(nid_l, j + 1, kWave) : -1;
        if (j + 1 < nitems) {
            const V* nrow = reinterpret_cast<const V*>(matrix + (size_t)(s + pairs) * row_elems) + (size_t)g0 * nvec;
#pragma unroll
            for (int g = 0; g < GA; ++g)
#pragma unroll
                for (int it = 0; it < NI; ++it) {
                    const int idx = it * 64 + lane;
                    mv[g][it] = (dst_n >= 0 && g < gn && idx < nvec) ? nrow[g * nvec + idx] : V(0);
                }
#pragma unroll
            for (int g = 0; g < GA; ++g)
#pragma unroll
                for (int it = 0; it < NI; ++it) {
                    const int idx = it * 64 + lane;
                    hv[g][it] = (nid_n >= 0 && g < gn && idx < nvec)
                                    ? *reinterpret_cast<const V*>(host_piece(host, nid_n, ((size_t)(g0 + g) * nvec + idx) * 16, row_bytes))
                                    : V(0);
                }
        }
        // finish item j: same order of operations as the activation kernel
        if (act_wave && dst >= 0) {
            const float du = wave_sum(mdu);
            float act;
            if (GLU) {
                const float dg = wave_sum(mdg);
                act = fmaxf(dg + old_bias, 0.f) * du;
            } else if (gact) {
                act = old_gate * du;
            } else {
                act = fmaxf(du + old_bias, 0.f);
            }
            if (lane == 0) {
                pointers[dst] = old_ptr;
                bias[dst] = old_bias;
                h_new[dst] = act;
                stamp[dst] = step;
            }
        }
        if (act_wave && nid >= 0) {
            const float du = wave_sum(hdu);
            float act;
            if (GLU) {
                const float dg = wave_sum(hdg);
                act = fmaxf(dg + new_bias, 0.f) * du;
            } else if (gact) {
                act = new_gate * du;
            } else {
                act = fmaxf(du + new_bias, 0.f);
            }
            if (lane == 0) {
                pointers[s] = nid;
                bias[s] = new_bias;
                h_new[s] = act;
                stamp[s] = step;
            }
        }
        dst = dst_n;
        nid = nid_n;
      }
    }
    if (wave_id == 0 && lane == 0) {
        st->num_used = n2 + a;
        atomicAdd(&st->c_h2d_bytes, (unsigned long long)a * row_elems * sizeof(T));
    }
}

// grid = load_wgs + up_blocks, block = 256.  Batch 1 only.
template <typename T, int NI, bool GLU>
__global__ __launch_bounds__(256) void k_load_up(T* __restrict__ matrix, int32_t* __restrict__ pointers,
                                                 float* __restrict__ bias, const HostStore host,
                                                 const float* __restrict__ b, const int32_t* __restrict__ added,
                                                 const int32_t* __restrict__ move_dst, size_t row_elems, int F, int d,
                                                 int capacity, const T* __restrict__ x, float* __restrict__ h,
                                                 float* __restrict__ h_new, int32_t* __restrict__ stamp, int spec,
                                                 int load_wgs, const float* __restrict__ gact, DevState* st) {
    if ((int)blockIdx.x < load_wgs) {
        const int w = threadIdx.x >> 6;
        if (w >= kStepLoadWaves) return;
        load_role<T, NI, GLU>(matrix, pointers, bias, host, b, added, move_dst, row_elems, F, d, capacity, x, h_new, stamp,
                              gact, blockIdx.x * kStepLoadWaves + w, load_wgs * kStepLoadWaves, st);
    } else {
        ffn_up_role<T, NI, GLU, true>(matrix, bias, x, h, d, 1, capacity, row_elems, spec, blockIdx.x - load_wgs,
                                      gridDim.x - load_wgs, &st->n_base, pointers, gact, F, st);
    }
}

// The same overlap for a batch of tokens (fp16): loader workgroups (layout of k_load) next to the MFMA activation
// stage over the rows that survive the deletion.  The slots the loaders write (filled holes, appended rows) get
// their activations from a second, short launch of k_ffn_up_mfma<GLU, kRowsChanged> once the load is complete.
// grid = load_wgs + ceil(capacity / 16), block = 256.
template <bool GLU>
__global__ __launch_bounds__(256) void k_load_up_mfma(_Float16* __restrict__ matrix, int32_t* __restrict__ pointers,
                                                      float* __restrict__ bias, const HostStore host,
                                                      const float* __restrict__ b, const int32_t* __restrict__ added,
                                                      const int32_t* __restrict__ move_dst, size_t row_bytes, int F,
                                                      const _Float16* __restrict__ x, float* __restrict__ h, int d,
                                                      int batch, int capacity, int load_wgs, int spec_tiles,
                                                      const float* __restrict__ gact, DevState* st) {
    if ((int)blockIdx.x < load_wgs)
        load_rows_role(reinterpret_cast<char*>(matrix), pointers, bias, host, b, added, move_dst, row_bytes, F,
                       blockIdx.x, load_wgs, st);
    else
        // (with the gate predictor a hole's pointer may change under this role: the lookup is clamped and the
        // slot's activation is recomputed by the pass over the written slots)
        // (tiles below spec_tiles - those a row-count hint covers - ask for their first rows ahead of the state)
        ffn_up_mfma_tile_staged<GLU, kRowsKept, kMfmaWaves>(matrix, bias, x, h, d, batch, capacity, row_bytes / sizeof(_Float16),
                                                blockIdx.x - load_wgs, (int)blockIdx.x - load_wgs < spec_tiles, pointers,
                                                gact, F, st);
}

}  // namespace lif
