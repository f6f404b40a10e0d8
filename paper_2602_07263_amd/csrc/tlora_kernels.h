// Launch wrappers of the gfx950 kernels.  Every pointer is a device pointer; every launch is
// asynchronous on the given stream.  The wrappers check nothing: the planner has already
// validated shapes and sized every table.
#pragma once
#include <hip/hip_runtime.h>

#include "tlora_internal.h"

namespace tlora {

// bf16 copies of the adapters in the layouts the MFMA kernels read (zero padded to rpad).
void launch_pack_adapters(const JobDev* jobs, int num_jobs, int d_in, int d_out, int max_rpad,
                          uint16_t* atp, uint16_t* ap, uint16_t* bp, hipStream_t st);

// out_j[t, p] = sum_k act[t, k] * P_j[p, k]   (P_j = A_j^T packed, or B_j packed)
// writes fp32 `S` and bf16 `Sb = scale_j * S` in the packed ragged layout.
void launch_shrink(const JobDev* jobs, const ShrinkUnit* units, int num_units, int shrink_rows,
                   const uint16_t* act, int K, const uint16_t* packed, bool packed_is_atp,
                   float* S, uint16_t* Sb, hipStream_t st);

// out[t, n] = sum_k act[t, k] * Wop[k, n] + sum_p Sb_j[t, p] * Eop_j[p, n]
//   w_is_kn = true : W is [K, N] row-major (forward,  Eop_j = B_j packed [rpad, N])
//   w_is_kn = false: W is [N, K] row-major (backward, Eop_j = A_j packed [N, rpad])
void launch_seg_gemm(bool w_is_kn, const JobDev* jobs, const TileJobs* tile_jobs, const uint16_t* act,
                     const uint16_t* W, const uint16_t* Sb, const uint16_t* packed, uint16_t* out, int T, int K,
                     int N, hipStream_t st);

// partial[u] = sum_{t in unit u} U_j[t, p] * V[t, c]   then   G_j = scale_j * sum_u partial[u]
void launch_rank_grad(int mb, const JobDev* jobs, const GradUnit* units, int num_units, const float* U,
                      const uint16_t* V, int D, float* partial, hipStream_t st);
void launch_grad_reduce(int mb, const JobDev* jobs, const GradGroup* groups, int num_groups, const float* partial,
                        int D, bool out_is_dA, hipStream_t st);

// fp32 configuration: strided products on plain FMA units.
void launch_f32_units(const F32Unit* units, const F32Tile* tiles, int num_tiles, hipStream_t st);

}  // namespace tlora
