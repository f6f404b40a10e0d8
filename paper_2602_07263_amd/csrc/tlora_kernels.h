// Launch wrappers of the gfx950 kernels.  Every pointer is a device pointer; every launch is
// asynchronous on the given stream.  The wrappers check nothing: the planner has already
// validated shapes and sized every table.
#pragma once
#include <hip/hip_runtime.h>

#include "tlora_internal.h"

namespace tlora {

// bf16 copies of the adapters in the layouts the MFMA kernels read (zero padded to rpad).
// atp: per job A_j^T [rpad, d_in], stacked in job order ([R + 32, d_in], trailing rows zero);  a_all: [d_in, R + 32] with job j in columns roff_j ..;  b_all: [R + 32, d_out]
// with job j in rows roff_j ..  (R = r_total; the 32 trailing columns / rows are zero).
void launch_pack_adapters(const JobDev* jobs, int num_jobs, int d_in, int d_out, int max_rpad, int r_total,
                          uint16_t* atp, uint16_t* a_all, uint16_t* b_all, hipStream_t st);

// out[c, r] = in[r, c]; bf16 [rows, cols] row-major, rows and cols multiples of 8, 16-byte aligned.
void launch_transpose_bf16(const uint16_t* in, uint16_t* out, int rows, int cols, hipStream_t st);

// Zero `bytes` (multiple of 16) of device memory with a plain store kernel.
void launch_zero_fill(void* ptr, size_t bytes, hipStream_t st);

// Copy `bytes` of HOST memory to device memory `dst` (4-byte aligned, room for bytes rounded up to 4) by value,
// through the arguments of small store kernels: no staging buffer, no copy node, nothing allocated.
void launch_table_write(const void* host_src, size_t bytes, void* dst, hipStream_t st);
// Copy `bytes` (a multiple of 16) from pinned host memory, given by its device address, to device memory.
void launch_table_copy(const void* src_device_view, void* dst, size_t bytes, hipStream_t st);

// out_j[t, p] = sum_k act[t, k] * P_j[p, k]   (P_j = A_j^T packed, or B_j packed)
// row_index (null = identity): the row of `act` that holds token row t of the job-sorted order (token-indexed calls).
// writes the result as bf16 hi + lo planes (packed ragged layout, each job's rows zero padded to a multiple of
// 32) and bf16 `scale_j * S` into the per-tile K-extension matrices `Sx`.
// packed_is_atp: P_j = atp + atp_off_j (row stride K);  otherwise P_j = b_all + roff_j * K.
void launch_shrink(const JobDev* jobs, const TileDev* tiles, const ShrinkUnit* units, int num_units,
                   int shrink_rows, const uint16_t* act, int K, const uint16_t* packed, bool packed_is_atp,
                   uint16_t* S_hi, uint16_t* S_lo, uint16_t* Sx, const int32_t* row_index, hipStream_t st);
// Same result for K % 32 == 0 with streaming units (shrink_rows = 64 | 128 token rows x 128 rank columns).
void launch_shrink_stream(const JobDev* jobs, const TileDev* tiles, const ShrinkUnit* units, int num_units,
                          int shrink_rows, int stages, const uint16_t* act, int K, const uint16_t* packed,
                          bool packed_is_atp, uint16_t* S_hi, uint16_t* S_lo, uint16_t* Sx, const int32_t* row_index,
                          hipStream_t st);

// out[t, n] = sum_k act[t, k] * Wop[k, n] + sum_p Sx_tile[t, p] * Eop[roff_first + p, n]
//   w_is_kn = true : W is [K, N] row-major (forward,  Eop = b_all [R + 32, N])
//   w_is_kn = false: W is [N, K] row-major (backward, Eop = a_all^T, stored [N, R + 32])
void launch_seg_gemm(bool w_is_kn, const TileDev* tiles, const uint16_t* act, const uint16_t* W,
                     const uint16_t* Sx, const uint16_t* packed, int r_total, uint16_t* out,
                     const int32_t* out_index /* null, or the output row of every row (scatter) */,
                     const int32_t* in_index /* null, or the row of `act` behind every row (gather; needs T * K * 2 < 4 GiB) */,
                     int T, int K, int N,
                     unsigned long long* clk /* null, or 2 zeroed words: every 64th workgroup adds the shader
                                                cycles and 100 MHz ticks of its K-loop */,
                     hipStream_t st);

// partial[u] = sum_{t in unit u} U_j[t, p] * V[t, c]   then   G_j = scale_j * sum_u partial[u]
void launch_rank_grad(const JobDev* jobs, const GradUnit* units, int num_units, const uint16_t* U_hi,
                      const uint16_t* U_lo, const uint16_t* V, int D, float* partial,
                      const int32_t* row_index /* null, or the row of V behind every token row */, hipStream_t st);
// accumulate: G_j += ... instead of G_j = ...
void launch_grad_reduce(const JobDev* jobs, const GradGroup* groups, int num_groups, const float* partial, int D,
                        bool out_is_dA, bool accumulate, hipStream_t st);

// fp32 configuration: strided products on plain FMA units.
void launch_f32_units(const F32Unit* units, const F32Tile* tiles, int num_tiles, hipStream_t st);

// AdamW step over a device table of `count` tensors (max_n = the largest element count).
void launch_adamw(const AdamwDev* tensors, int count, int64_t max_n, hipStream_t st);

// Glue of the MLP block (bf16 = tensors are bf16, else fp32; d and n multiples of 8; rstd fp32 [T]).
void launch_rmsnorm_fwd(bool bf16, const void* X, const void* gamma, float eps, int T, int d, void* Xn, float* rstd,
                        hipStream_t st);
// dX = dOut + d/dX [RMSNorm(X) gamma] applied to (dXa + dXb [+ dXc]); dXc may be null
void launch_rmsnorm_bwd(bool bf16, const void* X, const void* gamma, const float* rstd, const void* dXa,
                        const void* dXb, const void* dXc, const void* dOut, int T, int d, void* dX, hipStream_t st);
void launch_swiglu_fwd(bool bf16, const void* G, const void* U, void* Z, int64_t n, hipStream_t st);
void launch_swiglu_bwd(bool bf16, const void* G, const void* U, const void* dZ, void* dG, void* dU, int64_t n,
                       hipStream_t st);
void launch_residual_add(bool bf16, const void* X, const void* D, void* Out, int64_t n, hipStream_t st);

// Row gather (dst[i] = src[index[i]]) / scatter (dst[index[i]] = src[i]); row_bytes a multiple of 16.
void launch_permute_rows(const void* src, void* dst, const int32_t* index, int64_t rows, int64_t row_bytes, bool scatter,
                         hipStream_t st);
// Copy of a row list with every entry forced into [0, rows)  (rows < 2^31).
void launch_clamp_index(const int32_t* src, int32_t* dst, int64_t rows, hipStream_t st);

// ---- attention half (bf16, head size 128) -----------------------------------------------------------------
constexpr int kAttnHeadDim = 128;
// 128 consecutive tokens [t0, t0 + 128) of the sequence that starts at token seq_start and has seq_len tokens
struct AttnTile {
  int32_t seq_start, seq_len, t0, pad;
};
// Causal grouped-query attention over [T, heads * 128] tensors (Q, O, dO, dQ: Hq heads; K, V, dK, dV: Hkv heads,
// Hq % Hkv == 0).  lse [T, Hq] fp32 = log2 of the softmax denominator (base-2 domain, including the maximum);
// D [T, Hq] fp32 is scratch of the backward.  The backward is deterministic (no atomics).
void launch_attn_fwd(const AttnTile* tiles, int n_tiles, const uint16_t* Q, const uint16_t* K, const uint16_t* V,
                     uint16_t* O, float* lse, int Hq, int Hkv, hipStream_t st);
void launch_attn_bwd(const AttnTile* tiles, int n_tiles, const uint16_t* Q, const uint16_t* K, const uint16_t* V,
                     const uint16_t* O, const uint16_t* dO, const float* lse, float* D, uint16_t* dQ, uint16_t* dK,
                     uint16_t* dV, int64_t T, int Hq, int Hkv, hipStream_t st);
// table [positions, 64, 2] fp32 = (cos, sin) of position * base^(-i / 64)
void launch_rope_table(float* table, int positions, float base, hipStream_t st);
// In-place rotary embedding of x [T, heads * 128] at positions pos [T] (all < the table's positions);
// inverse = the transposed rotation.
void launch_rope(uint16_t* x, const int32_t* pos, const float* table, int64_t T, int heads, bool inverse, hipStream_t st);

}  // namespace tlora
