// gfx950 kernels of the attention half of a decoder layer: rotary position embedding and causal grouped-query
// attention (forward, and the backward as two deterministic kernels), bf16 with fp32 accumulation, head size 128.
// (Sec. 3.2 runs the fused jobs on one frozen backbone; Sec. 4.1's backbones are 8B-class decoders with exactly this
// attention.  The paper gives no kernel for it: these are the standard definitions.)
//
// All three attention kernels work on "transposed" score blocks S^T[kv, q] (or S[q, kv] in the dK/dV kernel) so
// that the 32 x 32 x 16 MFMA leaves every lane with 16 scores of ONE query (key) column: softmax statistics are
// per lane (plus one exchange with lane ^ 32), and the probabilities a lane holds are, in accumulator order,
// exactly the 8 k-values the next MFMA wants from it as an operand -- provided the other operand enumerates the
// keys in the same order, which the transposing LDS read does by fetching rows {4h .. 4h+3, 8 + 4h .. 8 + 4h + 3}
// of every 16-row slice (h = lane / 32).  So P never leaves the registers.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tlora_kernels.h"

namespace tlora {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))

namespace {

constexpr int HD = kAttnHeadDim;          // 128
constexpr int ROWB = HD * 2;              // bytes per tile row
constexpr float kNegInf = -__builtin_huge_valf();

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  bf16x2 v = {(__bf16)lo, (__bf16)hi};
  return __builtin_bit_cast(uint32_t, v);
}
__device__ __forceinline__ bf16x8 pack8(const f32x16& a, int first) {
  u32x4 r = {pack2(a[first], a[first + 1]), pack2(a[first + 2], a[first + 3]), pack2(a[first + 4], a[first + 5]),
             pack2(a[first + 6], a[first + 7])};
  return __builtin_bit_cast(bf16x8, r);
}
// LDS tile [rows][128] bf16 (256 B per row): the 16-byte chunk c of row r sits at slot c ^ sw(r),
// sw(r) = ((r & 3) << 2) | ((r >> 2) & 3).  16 consecutive rows read at one logical chunk hit 16 distinct bank
// groups, and the 4 rows x 64 bytes of a transposing read hit 4 distinct 64-byte groups.
__device__ __forceinline__ int tile_off(int r, int c) { return r * ROWB + ((c ^ (((r & 3) << 2) | ((r >> 2) & 3))) << 4); }
// Per-lane byte offsets of the operand fragments inside a tile, computed once per kernel: everything that changes
// afterwards (tile buffer, 32-row block, 16-row slice) is a compile-time multiple of the row pitch on top, which the
// LDS instructions carry in their immediate offset -- the loops spend no vector instructions on addresses.
struct FragPat {
  int row[8];       // "rows of the tile" fragment, k-slice s: row lane % 32, chunk 2 s + lane / 32
  int col_lo[4];    // "columns of the tile" fragment, column block db: rows 4 h + j / 4 (h = lane / 32, j = lane % 16)
  int col_hi[4];    //                                                  ... and those rows + 8
};
__device__ __forceinline__ FragPat make_frag_pat(int lane) {
  FragPat P;
  const int lr = lane & 31, hl = lane >> 5, j = lane & 15;
#pragma unroll
  for (int s = 0; s < 8; ++s) P.row[s] = tile_off(lr, 2 * s + hl);
  const int half16 = (lane >> 4) & 1;
#pragma unroll
  for (int db = 0; db < 4; ++db) {
    const int col = db * 32 + half16 * 16 + (j & 3) * 4;
    const int r0 = 4 * hl + (j >> 2);
    P.col_lo[db] = tile_off(r0, col >> 3) + (col & 7) * 2;
    P.col_hi[db] = tile_off(r0 + 8, col >> 3) + (col & 7) * 2;
  }
  // opaque to the optimiser from here on: kept in registers instead of being recomputed inside the loops
#pragma unroll
  for (int s = 0; s < 8; ++s) asm volatile("" : "+v"(P.row[s]));
#pragma unroll
  for (int db = 0; db < 4; ++db) { asm volatile("" : "+v"(P.col_lo[db]));  asm volatile("" : "+v"(P.col_hi[db])); }
  return P;
}
// operand fragment "rows of the tile": rows rb .. rb + 31 (rb a multiple of 32), k-slice s (head-dim values 16 s ..).
// The swizzle of row rb + r equals that of row r for rb a multiple of 16, so rb only adds rb row pitches.
__device__ __forceinline__ bf16x8 frag_rows(const uint8_t* tile, int rb, int s, const FragPat& P) {
  return __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(tile + rb * ROWB + P.row[s]));
}
// operand fragment "columns of the tile": columns 32 db .. 32 db + 31 as operand rows, k = tile rows
// r16 + {4h .. 4h+3, 8 + 4h .. 8 + 4h + 3} (h = lane / 32, r16 a multiple of 16), through the transposing LDS read
__device__ __forceinline__ bf16x8 frag_cols(const uint8_t* tile, int db, int r16, const FragPat& P) {
  s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, tile + r16 * ROWB + P.col_lo[db]));
  s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, tile + r16 * ROWB + P.col_hi[db]));
  return __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}
template <int N>
struct IntC {
  static constexpr int value = N;
};
// Asynchronous 16-byte-per-lane global->LDS load issued as raw instructions: lane l's 16 bytes land at LDS byte
// address lds_base + 16 l (lds_base wave-uniform, carried in M0); the global address is a wave-uniform 64-bit base
// plus an unsigned 32-bit byte offset per lane.  The compiler does not track these loads: the kernels wait
// (s_waitcnt vmcnt(0)) and synchronise by hand before reading what they wrote, and drain before they end.
__device__ __forceinline__ void dma16s(uint32_t voff, const void* sbase, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(sbase), "s"(lds_base)
               : "memory");
}
// 4 bytes per lane: lane l's word lands at lds_base + 4 l
__device__ __forceinline__ void dma4s(uint32_t voff, const void* sbase, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1" ::"v"(voff), "s"(sbase), "s"(lds_base)
               : "memory");
}
__device__ __forceinline__ const char* uniform_ptr(const void* p) {
  const uint64_t v = reinterpret_cast<uint64_t>(p);
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return reinterpret_cast<const char*>(((uint64_t)hi << 32) | lo);
}
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
  return __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)LDS_PTR(const uint8_t, p));
}
// every load of this wave has landed (vmcnt = expcnt = lgkmcnt = 0), then the workgroup meets
__device__ __forceinline__ void wait_all_and_sync() {
  __builtin_amdgcn_s_waitcnt(0);
  __builtin_amdgcn_s_barrier();
}
// One wave's share (LOADS x 4 rows) of an asynchronous tile copy: rows row0 + 4 i + lane / 16 of a [.., row_bytes]
// global matrix whose rows past `last_row` repeat row `last_row` (finite stand-ins that a zero probability
// multiplies), into the swizzled tile.  Rows row0 + 4 i are multiples of 4, so the swizzle of a lane's chunk
// depends on i and the lane only.
template <int LOADS>
__device__ __forceinline__ void tile_dma(const char* sbase, uint32_t row_bytes, int row0, int last_row, uint32_t tile_lds,
                                         int lane, int grow0 = 0 /* tile row r holds global row grow0 + r */) {
  const int lr = lane >> 4, slot = lane & 15;
#pragma unroll
  for (int i = 0; i < LOADS; ++i) {
    const int r = row0 + 4 * i + lr;
    const int c = slot ^ ((lr << 2) | (((row0 >> 2) + i) & 3));
    dma16s((uint32_t)min(grow0 + r, last_row) * row_bytes + (uint32_t)c * 16u, sbase, tile_lds + (uint32_t)(row0 + 4 * i) * ROWB);
  }
}
// the 8 k-slices of one token row as a "column" operand: lane l -> row (given), head-dim values 16 s + 8 (l / 32) ..
__device__ __forceinline__ void load_row_frags(const uint16_t* row, int lane, bf16x8 (&f)[8]) {
#pragma unroll
  for (int s = 0; s < 8; ++s)
    f[s] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(row + 16 * s + 8 * (lane >> 5)));
}
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
// x of this lane and x of lane ^ 32, in unspecified order: one v_permlane32_swap (the upper half of the first operand
// trades places with the lower half of the second) instead of a round trip through the LDS crossbar.  Both callers
// combine the two symmetrically (max, sum).
__device__ __forceinline__ void with_partner32(float x, float& a, float& b) {
  const unsigned u = __builtin_bit_cast(unsigned, x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  a = __builtin_bit_cast(float, (unsigned)r[0]);
  b = __builtin_bit_cast(float, (unsigned)r[1]);
}
// key (query) index inside a 32-block that accumulator element i of lanes with lane / 32 = hl stands for
__device__ __forceinline__ int acc_row(int i, int hl) { return 8 * (i >> 2) + 4 * hl + (i & 3); }

}  // namespace

// ---------------------------------------------------------------------------------------------------
// Forward.  One workgroup = 128 queries of one sequence and head (4 waves x 32); keys / values stream through
// LDS in tiles of 64 (double buffered, asynchronous loads).  Scores stay unscaled in the accumulators; with
// c = log2(e) / sqrt(128) the probabilities are exp2(c s - c m), one multiply-add and one exponential per score.
// The running maximum only rescales the output accumulators when it moved in some lane of the wave, and only
// tiles on the diagonal are masked.  lse = c m + log2(sum)  (base-2 domain).  Two workgroups share a CU so that
// one's softmax overlaps the other's matrix products.
// ---------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
attn_fwd_kernel(const AttnTile* __restrict__ tiles, const uint16_t* __restrict__ Q, const uint16_t* __restrict__ K,
                const uint16_t* __restrict__ V, uint16_t* __restrict__ O, float* __restrict__ lse, int Hq, int Hkv, float c) {
  __shared__ __attribute__((aligned(1024))) uint8_t kt[2][64 * ROWB];
  __shared__ __attribute__((aligned(1024))) uint8_t vt[2][64 * ROWB];
  const AttnTile t = tiles[blockIdx.x];
  const int h = blockIdx.y, hk = h / (Hq / Hkv);
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), hl = lane >> 5;
  const int q0w = t.t0 + wave * 32;
  const bool active = q0w < t.seq_len;                               // a wave of padding rows only computes nothing
  const int qmin = min(q0w, t.seq_len - 1), qmax = min(q0w + 31, t.seq_len - 1);
  const int qpos = min(q0w + (lane & 31), t.seq_len - 1);          // padded rows act like the last row; not stored
  const bool qvalid = q0w + (lane & 31) < t.seq_len;
  const int64_t qs = (int64_t)Hq * HD, ks = (int64_t)Hkv * HD;
  bf16x8 qf[8];
  const uint16_t* Kh = K + (int64_t)t.seq_start * ks + hk * HD;
  const uint16_t* Vh = V + (int64_t)t.seq_start * ks + hk * HD;
  const uint32_t kv_row_bytes = (uint32_t)ks * 2u;
  const uint32_t kt_lds = lds_addr(kt), vt_lds = lds_addr(vt);
  f32x16 oacc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) oacc[i][e] = 0.f;
  float m = kNegInf, lsum = 0.f;                                     // lsum: this lane's half of the row sum
  const int nkv = min(t.seq_len, t.t0 + 128);                     // keys this workgroup can see
  const int ntiles = (nkv + 63) / 64;
  auto issue = [&](int it) {
    const int kvbase = it * 64;
    const uint32_t buf = (uint32_t)(it & 1) * 64 * ROWB;
    tile_dma<4>(uniform_ptr(Kh + (int64_t)kvbase * ks), kv_row_bytes, 16 * wave, nkv - 1 - kvbase, kt_lds + buf, lane);
    tile_dma<4>(uniform_ptr(Vh + (int64_t)kvbase * ks), kv_row_bytes, 16 * wave, nkv - 1 - kvbase, vt_lds + buf, lane);
  };
  const FragPat P = make_frag_pat(lane);
  {
    // The 128 query rows come in like a key tile, through the second buffers (rows 0-63 in the key buffer, 64-127
    // in the value buffer), together with the first key / value tile; each wave then takes its 32 rows' fragments
    // into registers and the buffers are free again before the second key / value tile is requested.
    const char* const qbase = uniform_ptr(Q + (int64_t)(t.seq_start + t.t0) * qs + h * HD);
    const uint32_t q_row_bytes = (uint32_t)qs * 2u;
    const int last_q = t.seq_len - 1 - t.t0;
    tile_dma<4>(qbase, q_row_bytes, 16 * wave, last_q, kt_lds + 64 * ROWB, lane);
    tile_dma<4>(qbase, q_row_bytes, 16 * wave, last_q, vt_lds + 64 * ROWB, lane, 64);
    issue(0);
    wait_all_and_sync();
    const uint8_t* const qtile = wave < 2 ? kt[1] : vt[1];
#pragma unroll
    for (int s = 0; s < 8; ++s) qf[s] = frag_rows(qtile, 32 * (wave & 1), s, P);
  }
  auto tile_step = [&](auto bufc, int it) {
    constexpr int buf = decltype(bufc)::value;
    wait_all_and_sync();                                              // tile `it` is in LDS; the other buffer is free
    if (it + 1 < ntiles) issue(it + 1);
    const int kvbase = it * 64;
    if (active && kvbase <= qmax) {                                   // wave-uniform: something at or below the diagonal
      const uint8_t* kb = kt[buf];
      const uint8_t* vb = vt[buf];
      f32x16 sacc[2];
#pragma unroll
      for (int j = 0; j < 2; ++j) {
#pragma unroll
        for (int e = 0; e < 16; ++e) sacc[j][e] = 0.f;
#pragma unroll
        for (int s = 0; s < 8; ++s) sacc[j] = mfma32(frag_rows(kb, 32 * j, s, P), qf[s], sacc[j]);
      }
      if (kvbase + 63 > qmin) {                                       // the tile reaches past some query of the wave
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int i = 0; i < 16; ++i)
            if (kvbase + 32 * j + acc_row(i, hl) > qpos) sacc[j][i] = kNegInf;
      }
      float mx = sacc[0][0];
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) mx = fmaxf(mx, sacc[j][i]);
      {
        float a, b;
        with_partner32(mx, a, b);
        mx = fmaxf(a, b);
      }
      const float mnew = fmaxf(m, mx);                                // finite: key 0 is visible to every query
      if (__any(mnew != m)) {
        const float alpha = fast_exp2((m - mnew) * c);                // 0 for m = -inf
        lsum *= alpha;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int e = 0; e < 16; ++e) oacc[i][e] *= alpha;
        m = mnew;
      }
      const float mc = m * c;
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const float p = fast_exp2(fmaf(sacc[j][i], c, -mc));      // exp2(-inf) = 0 for masked scores
          sacc[j][i] = p;
          lsum += p;
        }
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          const bf16x8 pf = pack8(sacc[j], 8 * s2);
#pragma unroll
          for (int db = 0; db < 4; ++db) oacc[db] = mfma32(frag_cols(vb, db, 32 * j + 16 * s2, P), pf, oacc[db]);
        }
    }
  };
  for (int it = 0; it < ntiles; it += 2) {                           // two steps per trip: the buffer is a constant
    tile_step(IntC<0>{}, it);
    if (it + 1 < ntiles) tile_step(IntC<1>{}, it + 1);
  }
  if (qvalid) {
    float la, lb;
    with_partner32(lsum, la, lb);
    const float l = la + lb;
    const float inv = 1.f / l;
    uint16_t* orow = O + (int64_t)(t.seq_start + qpos) * qs + h * HD;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int g = 0; g < 4; ++g)
        *reinterpret_cast<u32x2*>(orow + db * 32 + 8 * g + 4 * hl) =
            u32x2{pack2(oacc[db][4 * g] * inv, oacc[db][4 * g + 1] * inv),
                  pack2(oacc[db][4 * g + 2] * inv, oacc[db][4 * g + 3] * inv)};
    if (hl == 0) lse[(int64_t)(t.seq_start + qpos) * Hq + h] = m * c + log2f(l);
  }
}

// D[t, h] = sum_d dO[t, h, d] * O[t, h, d]   (16 lanes x 16 bytes per (token, head) row, 16 rows per workgroup)
__global__ void __launch_bounds__(256) attn_rowdot_kernel(const uint16_t* __restrict__ dO, const uint16_t* __restrict__ O,
                                                          float* __restrict__ D, int64_t n_rows) {
  const int64_t r = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);
  const int sub = threadIdx.x & 15;
  float s = 0.f;
  if (r < n_rows) {
    const u32x4 a = *reinterpret_cast<const u32x4*>(dO + r * HD + sub * 8);
    const u32x4 b = *reinterpret_cast<const u32x4*>(O + r * HD + sub * 8);
#pragma unroll
    for (int e = 0; e < 4; ++e)
      s += __builtin_bit_cast(float, a[e] << 16) * __builtin_bit_cast(float, b[e] << 16) +
           __builtin_bit_cast(float, a[e] & 0xffff0000u) * __builtin_bit_cast(float, b[e] & 0xffff0000u);
  }
#pragma unroll
  for (int o = 8; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
  if (sub == 0 && r < n_rows) D[r] = s;
}

// ---------------------------------------------------------------------------------------------------
// Backward, dQ.  Same decomposition as the forward: per 32 keys
//   S^T = K Q^T,  P^T = exp2(c S^T - lse),  dP^T = V dO^T,  dS^T = P^T (dP^T - D),  dQ^T += K^T dS^T,  dQ = dQ / sqrt(128).
// ---------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
attn_bwd_dq_kernel(const AttnTile* __restrict__ tiles, const uint16_t* __restrict__ Q, const uint16_t* __restrict__ K,
                   const uint16_t* __restrict__ V, const uint16_t* __restrict__ dO, const float* __restrict__ lse,
                   const float* __restrict__ D, uint16_t* __restrict__ dQ, int Hq, int Hkv, float c, float scale) {
  __shared__ __attribute__((aligned(1024))) uint8_t kt[2][64 * ROWB];
  __shared__ __attribute__((aligned(1024))) uint8_t vt[2][64 * ROWB];
  const AttnTile t = tiles[blockIdx.x];
  const int h = blockIdx.y, hk = h / (Hq / Hkv);
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), hl = lane >> 5;
  const int q0w = t.t0 + wave * 32;
  const bool active = q0w < t.seq_len;
  const int qmin = min(q0w, t.seq_len - 1), qmax = min(q0w + 31, t.seq_len - 1);
  const int qpos = min(q0w + (lane & 31), t.seq_len - 1);
  const bool qvalid = q0w + (lane & 31) < t.seq_len;
  const int64_t qs = (int64_t)Hq * HD, ks = (int64_t)Hkv * HD;
  const int64_t qrow = t.seq_start + qpos;
  bf16x8 qf[8], dof[8];
  load_row_frags(Q + qrow * qs + h * HD, lane, qf);
  load_row_frags(dO + qrow * qs + h * HD, lane, dof);
  const float L = lse[qrow * Hq + h], Dq = D[qrow * Hq + h];
  const uint16_t* Kh = K + (int64_t)t.seq_start * ks + hk * HD;
  const uint16_t* Vh = V + (int64_t)t.seq_start * ks + hk * HD;
  const uint32_t kv_row_bytes = (uint32_t)ks * 2u;
  const uint32_t kt_lds = lds_addr(kt), vt_lds = lds_addr(vt);
  f32x16 dq[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) dq[i][e] = 0.f;
  const int nkv = min(t.seq_len, t.t0 + 128);
  const int ntiles = (nkv + 63) / 64;
  auto issue = [&](int it) {
    const int kvbase = it * 64;
    const uint32_t buf = (uint32_t)(it & 1) * 64 * ROWB;
    tile_dma<4>(uniform_ptr(Kh + (int64_t)kvbase * ks), kv_row_bytes, 16 * wave, nkv - 1 - kvbase, kt_lds + buf, lane);
    tile_dma<4>(uniform_ptr(Vh + (int64_t)kvbase * ks), kv_row_bytes, 16 * wave, nkv - 1 - kvbase, vt_lds + buf, lane);
  };
  const FragPat P = make_frag_pat(lane);
  issue(0);
  auto tile_step = [&](auto bufc, int it) {
    constexpr int buf = decltype(bufc)::value;
    wait_all_and_sync();
    if (it + 1 < ntiles) issue(it + 1);
    const int kvbase = it * 64;
    if (active && kvbase <= qmax) {
      const uint8_t* kb = kt[buf];
      const uint8_t* vb = vt[buf];
      const bool diag = kvbase + 63 > qmin;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        f32x16 sacc, dp;
#pragma unroll
        for (int e = 0; e < 16; ++e) { sacc[e] = 0.f;  dp[e] = 0.f; }
#pragma unroll
        for (int s = 0; s < 8; ++s) {
          sacc = mfma32(frag_rows(kb, 32 * j, s, P), qf[s], sacc);
          dp = mfma32(frag_rows(vb, 32 * j, s, P), dof[s], dp);
        }
        if (diag) {
#pragma unroll
          for (int i = 0; i < 16; ++i)
            if (kvbase + 32 * j + acc_row(i, hl) > qpos) sacc[i] = kNegInf;
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) sacc[i] = fast_exp2(fmaf(sacc[i], c, -L)) * (dp[i] - Dq);   // dS^T
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          const bf16x8 dsf = pack8(sacc, 8 * s2);
#pragma unroll
          for (int db = 0; db < 4; ++db) dq[db] = mfma32(frag_cols(kb, db, 32 * j + 16 * s2, P), dsf, dq[db]);
        }
      }
    }
  };
  for (int it = 0; it < ntiles; it += 2) {
    tile_step(IntC<0>{}, it);
    if (it + 1 < ntiles) tile_step(IntC<1>{}, it + 1);
  }
  if (qvalid) {
    uint16_t* orow = dQ + qrow * qs + h * HD;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int g = 0; g < 4; ++g)
        *reinterpret_cast<u32x2*>(orow + db * 32 + 8 * g + 4 * hl) =
            u32x2{pack2(dq[db][4 * g] * scale, dq[db][4 * g + 1] * scale),
                  pack2(dq[db][4 * g + 2] * scale, dq[db][4 * g + 3] * scale)};
  }
}

// ---------------------------------------------------------------------------------------------------
// Backward, dK and dV.  One workgroup = 128 keys of one sequence and key/value head (4 waves x 32 keys); it walks
// the query heads of the group and, for each, the queries at or after its keys in steps of 64 (two blocks of 32):
//   S = Q K^T,  P = exp2(c S - lse_q),  dV^T += dO^T P,  dP = dO V^T,  dS = P (dP - D_q),  dK^T += Q^T dS.
// A lane owns one key column; Q, dO, lse and D of a step arrive in LDS through asynchronous loads issued two
// steps ahead (three stages; every wave issues the same 10 loads per step so that one counter value means
// "everything but the newest step has landed").  Sums run in a fixed order.  Tiles are taken from the end of the
// table: there the first keys of the long sequences come first, which have the most queries to walk.
// ---------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) attn_bwd_dkv_kernel(const AttnTile* __restrict__ tiles, int n_tiles,
                                                           const uint16_t* __restrict__ Q, const uint16_t* __restrict__ K,
                                                           const uint16_t* __restrict__ V, const uint16_t* __restrict__ dO,
                                                           const float* __restrict__ lse, const float* __restrict__ D,
                                                           uint16_t* __restrict__ dK, uint16_t* __restrict__ dV, int Hq,
                                                           int Hkv, float c, float scale) {
  constexpr int NS = 3, QS = 64;                                     // stages, queries per step
  constexpr int kLoads = 10;                                         // asynchronous loads per wave and step
  __shared__ __attribute__((aligned(1024))) uint8_t qt[NS][QS * ROWB];
  __shared__ __attribute__((aligned(1024))) uint8_t dot[NS][QS * ROWB];
  __shared__ __attribute__((aligned(256))) float ls[NS][QS], ds[NS][QS];
  const AttnTile t = tiles[n_tiles - 1 - (int)blockIdx.x];
  const int hk = blockIdx.y, G = Hq / Hkv;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), hl = lane >> 5;
  const int k0w = t.t0 + wave * 32;
  const bool active = k0w < t.seq_len;
  const int kpos = min(k0w + (lane & 31), t.seq_len - 1);
  const int kmax = min(k0w + 31, t.seq_len - 1);
  const bool kvalid = k0w + (lane & 31) < t.seq_len;
  const int64_t qs = (int64_t)Hq * HD, ks = (int64_t)Hkv * HD;
  const int64_t krow = t.seq_start + kpos;
  bf16x8 kf[8], vf[8];
  load_row_frags(K + krow * ks + hk * HD, lane, kf);
  load_row_frags(V + krow * ks + hk * HD, lane, vf);
  const uint32_t q_row_bytes = (uint32_t)qs * 2u;
  const uint32_t qt_lds = lds_addr(qt), dot_lds = lds_addr(dot), ls_lds = lds_addr(ls), ds_lds = lds_addr(ds);
  f32x16 dk[4], dv[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) { dk[i][e] = 0.f;  dv[i][e] = 0.f; }
  const int q_first = t.t0;                                          // queries before the first key see none of them
  const int nq = (t.seq_len - q_first + QS - 1) / QS;                // query steps per head
  const int nsteps = nq * G;
  auto issue = [&](int st) {
    const int hq = hk * G + st / nq, q0 = q_first + (st % nq) * QS;
    const int stage = st % NS, last = t.seq_len - 1 - q0;
    const int64_t base = (int64_t)(t.seq_start + q0) * qs + hq * HD;
    tile_dma<4>(uniform_ptr(Q + base), q_row_bytes, 16 * wave, last, qt_lds + (uint32_t)stage * QS * ROWB, lane);
    tile_dma<4>(uniform_ptr(dO + base), q_row_bytes, 16 * wave, last, dot_lds + (uint32_t)stage * QS * ROWB, lane);
    // per-query statistics, one word per lane (rows past the sequence repeat its last row); all waves write the
    // same words
    const uint32_t off = (uint32_t)min(lane, last) * (uint32_t)Hq * 4u;
    const int64_t sbase = (int64_t)(t.seq_start + q0) * Hq + hq;
    dma4s(off, uniform_ptr(lse + sbase), ls_lds + (uint32_t)stage * QS * 4);
    dma4s(off, uniform_ptr(D + sbase), ds_lds + (uint32_t)stage * QS * 4);
  };
  const FragPat P = make_frag_pat(lane);
  if (nsteps > 0) issue(0);
  if (nsteps > 1) issue(1);
  auto q_step = [&](auto stagec, int st) {
    constexpr int stage = decltype(stagec)::value;                   // = st % NS
    // everything but the loads of step st + 1 has landed (vmcnt in bits 3:0 and 15:14, the other counters 0)
    if (st + 1 < nsteps) __builtin_amdgcn_s_waitcnt(kLoads & 15);
    else                 __builtin_amdgcn_s_waitcnt(0);
    __builtin_amdgcn_s_barrier();
    if (st + 2 < nsteps) issue(st + 2);
    const int q0s = q_first + (st % nq) * QS;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const int q0 = q0s + 32 * half;
      if (active && q0 + 31 >= k0w && q0 < t.seq_len) {              // wave-uniform: some query at or after a key
        const uint8_t* qb = qt[stage];
        const uint8_t* dob = dot[stage];
        f32x16 sacc, dp;
#pragma unroll
        for (int e = 0; e < 16; ++e) { sacc[e] = 0.f;  dp[e] = 0.f; }
#pragma unroll
        for (int s = 0; s < 8; ++s) {
          sacc = mfma32(frag_rows(qb, 32 * half, s, P), kf[s], sacc);
          dp = mfma32(frag_rows(dob, 32 * half, s, P), vf[s], dp);
        }
        if (q0 < kmax || q0 + 31 >= t.seq_len) {                     // some query before a key of the wave, or padding
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int q = q0 + acc_row(i, hl);
            if (q < kpos || q >= t.seq_len) sacc[i] = kNegInf;
          }
        }
        f32x16 pm;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const f32x4 l4 = *reinterpret_cast<const f32x4*>(&ls[stage][32 * half + 8 * g + 4 * hl]);
          const f32x4 d4 = *reinterpret_cast<const f32x4*>(&ds[stage][32 * half + 8 * g + 4 * hl]);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float p = fast_exp2(fmaf(sacc[4 * g + e], c, -l4[e]));
            pm[4 * g + e] = p;
            sacc[4 * g + e] = p * (dp[4 * g + e] - d4[e]);             // dS
          }
        }
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          const bf16x8 pf = pack8(pm, 8 * s2), dsf = pack8(sacc, 8 * s2);
#pragma unroll
          for (int db = 0; db < 4; ++db) {
            dv[db] = mfma32(frag_cols(dob, db, 32 * half + 16 * s2, P), pf, dv[db]);
            dk[db] = mfma32(frag_cols(qb, db, 32 * half + 16 * s2, P), dsf, dk[db]);
          }
        }
      }
    }
  };
  for (int st = 0; st < nsteps; st += NS) {                          // NS steps per trip: the stage is a constant
    q_step(IntC<0>{}, st);
    if (st + 1 < nsteps) q_step(IntC<1>{}, st + 1);
    if (st + 2 < nsteps) q_step(IntC<2>{}, st + 2);
  }
  if (kvalid) {
    uint16_t* krow_o = dK + krow * ks + hk * HD;
    uint16_t* vrow_o = dV + krow * ks + hk * HD;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int d = db * 32 + 8 * g + 4 * hl;
        *reinterpret_cast<u32x2*>(krow_o + d) = u32x2{pack2(dk[db][4 * g] * scale, dk[db][4 * g + 1] * scale),
                                                      pack2(dk[db][4 * g + 2] * scale, dk[db][4 * g + 3] * scale)};
        *reinterpret_cast<u32x2*>(vrow_o + d) = u32x2{pack2(dv[db][4 * g], dv[db][4 * g + 1]),
                                                      pack2(dv[db][4 * g + 2], dv[db][4 * g + 3])};
      }
  }
}

// ---------------------------------------------------------------------------------------------------
// Rotary position embedding, in place, on [T, heads * 128] bf16.  A table kernel first writes (cos, sin) of
// position * base^(-i / 64) for every position up to the longest sequence and i < 64 (fp32); the rotation kernel
// then only streams: 8 lanes per (token, head) row, each rotating the pairs (i, i + 64) for 8 consecutive i.
// inverse = the transposed rotation (the backward of the forward one).
// ---------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) rope_table_kernel(float2* __restrict__ tab, int n /* positions * 64 */,
                                                         float log2_base) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx >= n) return;
  const float ang = (float)(idx >> 6) * exp2f(-log2_base * (float)(idx & 63) / 64.f);
  float sn, cs;
  sincosf(ang, &sn, &cs);
  tab[idx] = float2{cs, sn};
}
__global__ void __launch_bounds__(256) rope_kernel(uint16_t* __restrict__ x, const int32_t* __restrict__ pos,
                                                   const float2* __restrict__ tab, int heads,
                                                   int64_t n_rows /* tokens * heads */, int inverse) {
  const int64_t r = (int64_t)blockIdx.x * 32 + (threadIdx.x >> 3);
  if (r >= n_rows) return;
  const int i0 = (threadIdx.x & 7) * 8;
  const float2* tr = tab + (int64_t)pos[r / heads] * 64 + i0;
  uint16_t* row = x + r * HD + i0;
  const u32x4 lo = *reinterpret_cast<const u32x4*>(row), hi = *reinterpret_cast<const u32x4*>(row + 64);
  f32x4 cs[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) cs[e] = *reinterpret_cast<const f32x4*>(tr + 2 * e);     // (cos, sin) of two pairs
  u32x4 olo, ohi;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    float a[2] = {__builtin_bit_cast(float, lo[e] << 16), __builtin_bit_cast(float, lo[e] & 0xffff0000u)};
    float b[2] = {__builtin_bit_cast(float, hi[e] << 16), __builtin_bit_cast(float, hi[e] & 0xffff0000u)};
    float ra[2], rb[2];
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      const float c = cs[e][2 * k], sn = inverse ? -cs[e][2 * k + 1] : cs[e][2 * k + 1];
      ra[k] = a[k] * c - b[k] * sn;
      rb[k] = b[k] * c + a[k] * sn;
    }
    olo[e] = pack2(ra[0], ra[1]);
    ohi[e] = pack2(rb[0], rb[1]);
  }
  *reinterpret_cast<u32x4*>(row) = olo;
  *reinterpret_cast<u32x4*>(row + 64) = ohi;
}

void launch_attn_fwd(const AttnTile* tiles, int n_tiles, const uint16_t* Q, const uint16_t* K, const uint16_t* V,
                     uint16_t* O, float* lse, int Hq, int Hkv, hipStream_t st) {
  if (n_tiles == 0) return;
  const float c = 1.4426950408889634f / sqrtf((float)HD);
  hipLaunchKernelGGL(attn_fwd_kernel, dim3(n_tiles, Hq), dim3(256), 0, st, tiles, Q, K, V, O, lse, Hq, Hkv, c);
}
void launch_attn_bwd(const AttnTile* tiles, int n_tiles, const uint16_t* Q, const uint16_t* K, const uint16_t* V,
                     const uint16_t* O, const uint16_t* dO, const float* lse, float* D, uint16_t* dQ, uint16_t* dK,
                     uint16_t* dV, int64_t T, int Hq, int Hkv, hipStream_t st) {
  if (n_tiles == 0) return;
  const float scale = 1.f / sqrtf((float)HD), c = 1.4426950408889634f * scale;
  const int64_t rows = T * Hq;
  hipLaunchKernelGGL(attn_rowdot_kernel, dim3((unsigned)((rows + 15) / 16)), dim3(256), 0, st, dO, O, D, rows);
  hipLaunchKernelGGL(attn_bwd_dq_kernel, dim3(n_tiles, Hq), dim3(256), 0, st, tiles, Q, K, V, dO, lse, D, dQ, Hq, Hkv, c,
                     scale);
  hipLaunchKernelGGL(attn_bwd_dkv_kernel, dim3(n_tiles, Hkv), dim3(256), 0, st, tiles, n_tiles, Q, K, V, dO, lse, D, dK, dV,
                     Hq, Hkv, c, scale);
}
void launch_rope_table(float* table, int positions, float base, hipStream_t st) {
  const int n = positions * 64;
  if (n == 0) return;
  hipLaunchKernelGGL(rope_table_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, reinterpret_cast<float2*>(table), n,
                     log2f(base));
}
void launch_rope(uint16_t* x, const int32_t* pos, const float* table, int64_t T, int heads, bool inverse, hipStream_t st) {
  const int64_t rows = T * heads;
  if (rows == 0) return;
  hipLaunchKernelGGL(rope_kernel, dim3((unsigned)((rows + 31) / 32)), dim3(256), 0, st, x, pos,
                     reinterpret_cast<const float2*>(table), heads, rows, inverse ? 1 : 0);
}

}  // namespace tlora
