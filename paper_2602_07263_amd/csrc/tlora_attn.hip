// gfx950 kernels of the attention half of a decoder layer: rotary position embedding and causal grouped-query
// attention (forward, and the backward as two deterministic kernels), bf16 with fp32 accumulation, head size 128.
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
// operand fragment "rows of the tile": rows rb .. rb+31, k-slice s (head-dim values 16 s .. 16 s + 15)
__device__ __forceinline__ bf16x8 frag_rows(const uint8_t* tile, int rb, int s, int lane) {
  return __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(tile + tile_off(rb + (lane & 31), 2 * s + (lane >> 5))));
}
// operand fragment "columns of the tile": columns 32 cb .. 32 cb + 31 as operand rows, k = tile rows
// r16 + {4h .. 4h+3, 8 + 4h .. 8 + 4h + 3} (h = lane / 32), through the transposing LDS read
__device__ __forceinline__ bf16x8 frag_cols(const uint8_t* tile, int cb, int r16, int lane) {
  const int j = lane & 15, h = lane >> 5;
  const int col = cb * 32 + ((lane >> 4) & 1) * 16 + (j & 3) * 4;
  const int c = col >> 3, inner = (col & 7) * 2;
  const int r0 = r16 + 4 * h + (j >> 2);
  s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, tile + tile_off(r0, c) + inner));
  s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, tile + tile_off(r0 + 8, c) + inner));
  return __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}
// copy `nrows` rows (zero beyond `valid`) of one head from global memory ([token][heads * 128]) into a tile
template <int NROWS>
__device__ __forceinline__ void load_tile_regs(const uint16_t* base, int64_t row_stride, int valid, u32x4 (&regs)[NROWS / 16]) {
#pragma unroll
  for (int i = 0; i < NROWS / 16; ++i) {
    const int id = threadIdx.x + i * 256, r = id >> 4, c = id & 15;
    regs[i] = r < valid ? *reinterpret_cast<const u32x4*>(base + (int64_t)r * row_stride + c * 8) : u32x4{0, 0, 0, 0};
  }
}
template <int NROWS>
__device__ __forceinline__ void store_tile_regs(uint8_t* tile, const u32x4 (&regs)[NROWS / 16]) {
#pragma unroll
  for (int i = 0; i < NROWS / 16; ++i) {
    const int id = threadIdx.x + i * 256;
    *reinterpret_cast<u32x4*>(tile + tile_off(id >> 4, id & 15)) = regs[i];
  }
}
// the 8 k-slices of one token row as a "column" operand: lane l -> row (given), head-dim values 16 s + 8 (l / 32) ..
__device__ __forceinline__ void load_row_frags(const uint16_t* row, int lane, bf16x8 (&f)[8]) {
#pragma unroll
  for (int s = 0; s < 8; ++s)
    f[s] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(row + 16 * s + 8 * (lane >> 5)));
}

}  // namespace

// ---------------------------------------------------------------------------------------------------
// Forward.  One workgroup = 128 queries of one sequence and head (4 waves x 32); keys / values stream through
// LDS in tiles of 64, double buffered through registers.  c = log2(e) / sqrt(128); lse is kept in the base-2
// domain: lse = max + log2(sum).
// ---------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) attn_fwd_kernel(const AttnTile* __restrict__ tiles, const uint16_t* __restrict__ Q,
                                                       const uint16_t* __restrict__ K, const uint16_t* __restrict__ V,
                                                       uint16_t* __restrict__ O, float* __restrict__ lse, int Hq, int Hkv,
                                                       float c) {
  __shared__ __attribute__((aligned(1024))) uint8_t kt[2][64 * ROWB];
  __shared__ __attribute__((aligned(1024))) uint8_t vt[2][64 * ROWB];
  const AttnTile t = tiles[blockIdx.x];
  const int h = blockIdx.y, hk = h / (Hq / Hkv);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, hl = lane >> 5;
  const int q0w = t.t0 + wave * 32;
  const int qpos = min(q0w + (lane & 31), t.seq_len - 1);          // padded rows act like the last row; not stored
  const bool qvalid = q0w + (lane & 31) < t.seq_len;
  const int64_t qs = (int64_t)Hq * HD, ks = (int64_t)Hkv * HD;
  bf16x8 qf[8];
  load_row_frags(Q + (int64_t)(t.seq_start + qpos) * qs + h * HD, lane, qf);
  const uint16_t* Kh = K + (int64_t)t.seq_start * ks + hk * HD;
  const uint16_t* Vh = V + (int64_t)t.seq_start * ks + hk * HD;
  f32x16 oacc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) oacc[i][e] = 0.f;
  float m = kNegInf, lsum = 0.f;
  const int nkv = min(t.seq_len, t.t0 + 128);                     // keys this workgroup can see
  const int ntiles = (nkv + 63) / 64;
  u32x4 kr[4], vr[4];
  load_tile_regs<64>(Kh, ks, nkv, kr);
  load_tile_regs<64>(Vh, ks, nkv, vr);
  store_tile_regs<64>(kt[0], kr);
  store_tile_regs<64>(vt[0], vr);
  for (int it = 0; it < ntiles; ++it) {
    __syncthreads();
    const int kvbase = it * 64;
    if (it + 1 < ntiles) {
      load_tile_regs<64>(Kh + (int64_t)(kvbase + 64) * ks, ks, nkv - kvbase - 64, kr);
      load_tile_regs<64>(Vh + (int64_t)(kvbase + 64) * ks, ks, nkv - kvbase - 64, vr);
    }
    if (kvbase <= q0w + 31) {                                       // wave-uniform: something below the diagonal
      const uint8_t* kb = kt[it & 1];
      const uint8_t* vb = vt[it & 1];
      f32x16 sacc[2];
#pragma unroll
      for (int j = 0; j < 2; ++j) {
#pragma unroll
        for (int e = 0; e < 16; ++e) sacc[j][e] = 0.f;
#pragma unroll
        for (int s = 0; s < 8; ++s) sacc[j] = mfma32(frag_rows(kb, 32 * j, s, lane), qf[s], sacc[j]);
      }
      float mx = kNegInf;
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int kv = kvbase + 32 * j + 8 * (i >> 2) + 4 * hl + (i & 3);
          const float v = kv <= qpos ? sacc[j][i] * c : kNegInf;     // kv <= qpos < seq_len
          sacc[j][i] = v;
          mx = fmaxf(mx, v);
        }
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float mnew = fmaxf(m, mx);                               // finite: key 0 is visible to every query
      const float alpha = m == kNegInf ? 0.f : exp2f(m - mnew);
      float rs = 0.f;
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const float p = sacc[j][i] == kNegInf ? 0.f : exp2f(sacc[j][i] - mnew);
          sacc[j][i] = p;
          rs += p;
        }
      rs += __shfl_xor(rs, 32, 64);
      lsum = lsum * alpha + rs;
      m = mnew;
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) oacc[i][e] *= alpha;
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          const bf16x8 pf = pack8(sacc[j], 8 * s2);
#pragma unroll
          for (int db = 0; db < 4; ++db) oacc[db] = mfma32(frag_cols(vb, db, 32 * j + 16 * s2, lane), pf, oacc[db]);
        }
    }
    if (it + 1 < ntiles) {
      store_tile_regs<64>(kt[(it + 1) & 1], kr);
      store_tile_regs<64>(vt[(it + 1) & 1], vr);
    }
  }
  if (qvalid) {
    const float inv = 1.f / lsum;
    uint16_t* orow = O + (int64_t)(t.seq_start + qpos) * qs + h * HD;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int g = 0; g < 4; ++g)
        *reinterpret_cast<u32x2*>(orow + db * 32 + 8 * g + 4 * hl) =
            u32x2{pack2(oacc[db][4 * g] * inv, oacc[db][4 * g + 1] * inv),
                  pack2(oacc[db][4 * g + 2] * inv, oacc[db][4 * g + 3] * inv)};
    if (hl == 0) lse[(int64_t)(t.seq_start + qpos) * Hq + h] = m + log2f(lsum);
  }
}

// D[t, h] = sum_d dO[t, h, d] * O[t, h, d]   (one wave per (token, head))
__global__ void __launch_bounds__(256) attn_rowdot_kernel(const uint16_t* __restrict__ dO, const uint16_t* __restrict__ O,
                                                          float* __restrict__ D, int64_t n_rows) {
  const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= n_rows) return;
  const int lane = threadIdx.x & 63;
  const uint32_t a = *reinterpret_cast<const uint32_t*>(dO + r * HD + lane * 2);
  const uint32_t b = *reinterpret_cast<const uint32_t*>(O + r * HD + lane * 2);
  float s = __builtin_bit_cast(float, a << 16) * __builtin_bit_cast(float, b << 16) +
            __builtin_bit_cast(float, a & 0xffff0000u) * __builtin_bit_cast(float, b & 0xffff0000u);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
  if (lane == 0) D[r] = s;
}

// ---------------------------------------------------------------------------------------------------
// Backward, dQ.  Same decomposition as the forward: per 32 keys
//   S^T = K Q^T,  P^T = exp2(c S^T - lse),  dP^T = V dO^T,  dS^T = P^T (dP^T - D),  dQ^T += K^T dS^T,  dQ = dQ / sqrt(128).
// ---------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) attn_bwd_dq_kernel(const AttnTile* __restrict__ tiles, const uint16_t* __restrict__ Q,
                                                          const uint16_t* __restrict__ K, const uint16_t* __restrict__ V,
                                                          const uint16_t* __restrict__ dO, const float* __restrict__ lse,
                                                          const float* __restrict__ D, uint16_t* __restrict__ dQ, int Hq,
                                                          int Hkv, float c, float scale) {
  __shared__ __attribute__((aligned(1024))) uint8_t kt[2][64 * ROWB];
  __shared__ __attribute__((aligned(1024))) uint8_t vt[2][64 * ROWB];
  const AttnTile t = tiles[blockIdx.x];
  const int h = blockIdx.y, hk = h / (Hq / Hkv);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, hl = lane >> 5;
  const int q0w = t.t0 + wave * 32;
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
  f32x16 dq[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) dq[i][e] = 0.f;
  const int nkv = min(t.seq_len, t.t0 + 128);
  const int ntiles = (nkv + 63) / 64;
  u32x4 kr[4], vr[4];
  load_tile_regs<64>(Kh, ks, nkv, kr);
  load_tile_regs<64>(Vh, ks, nkv, vr);
  store_tile_regs<64>(kt[0], kr);
  store_tile_regs<64>(vt[0], vr);
  for (int it = 0; it < ntiles; ++it) {
    __syncthreads();
    const int kvbase = it * 64;
    if (it + 1 < ntiles) {
      load_tile_regs<64>(Kh + (int64_t)(kvbase + 64) * ks, ks, nkv - kvbase - 64, kr);
      load_tile_regs<64>(Vh + (int64_t)(kvbase + 64) * ks, ks, nkv - kvbase - 64, vr);
    }
    if (kvbase <= q0w + 31) {
      const uint8_t* kb = kt[it & 1];
      const uint8_t* vb = vt[it & 1];
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        f32x16 sacc, dp;
#pragma unroll
        for (int e = 0; e < 16; ++e) { sacc[e] = 0.f;  dp[e] = 0.f; }
#pragma unroll
        for (int s = 0; s < 8; ++s) {
          sacc = mfma32(frag_rows(kb, 32 * j, s, lane), qf[s], sacc);
          dp = mfma32(frag_rows(vb, 32 * j, s, lane), dof[s], dp);
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int kv = kvbase + 32 * j + 8 * (i >> 2) + 4 * hl + (i & 3);
          const float p = kv <= qpos ? exp2f(sacc[i] * c - L) : 0.f;
          sacc[i] = p * (dp[i] - Dq);                                 // dS^T
        }
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          const bf16x8 dsf = pack8(sacc, 8 * s2);
#pragma unroll
          for (int db = 0; db < 4; ++db) dq[db] = mfma32(frag_cols(kb, db, 32 * j + 16 * s2, lane), dsf, dq[db]);
        }
      }
    }
    if (it + 1 < ntiles) {
      store_tile_regs<64>(kt[(it + 1) & 1], kr);
      store_tile_regs<64>(vt[(it + 1) & 1], vr);
    }
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
// the query heads of the group and, for each, the query tiles at or after its keys.  Per 32 queries:
//   S = Q K^T,  P = exp2(c S - lse_q),  dV^T += dO^T P,  dP = dO V^T,  dS = P (dP - D_q),  dK^T += Q^T dS.
// A lane owns one key column; lse and D of the 16 queries it sees come from LDS.  Sums run in a fixed order.
// ---------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) attn_bwd_dkv_kernel(const AttnTile* __restrict__ tiles, const uint16_t* __restrict__ Q,
                                                           const uint16_t* __restrict__ K, const uint16_t* __restrict__ V,
                                                           const uint16_t* __restrict__ dO, const float* __restrict__ lse,
                                                           const float* __restrict__ D, uint16_t* __restrict__ dK,
                                                           uint16_t* __restrict__ dV, int Hq, int Hkv, float c, float scale) {
  __shared__ __attribute__((aligned(1024))) uint8_t qt[2][32 * ROWB];      // 32 queries per step
  __shared__ __attribute__((aligned(1024))) uint8_t dot[2][32 * ROWB];
  __shared__ float ls[2][32], ds[2][32];
  const AttnTile t = tiles[blockIdx.x];
  const int hk = blockIdx.y, G = Hq / Hkv;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, hl = lane >> 5;
  const int k0w = t.t0 + wave * 32;
  const int kpos = min(k0w + (lane & 31), t.seq_len - 1);
  const bool kvalid = k0w + (lane & 31) < t.seq_len;
  const int64_t qs = (int64_t)Hq * HD, ks = (int64_t)Hkv * HD;
  const int64_t krow = t.seq_start + kpos;
  bf16x8 kf[8], vf[8];
  load_row_frags(K + krow * ks + hk * HD, lane, kf);
  load_row_frags(V + krow * ks + hk * HD, lane, vf);
  f32x16 dk[4], dv[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) { dk[i][e] = 0.f;  dv[i][e] = 0.f; }
  const int q_first = t.t0 & ~31;                                   // queries before the first key see none of them
  const int nq = (t.seq_len - q_first + 31) / 32;                   // query steps per head
  const int nsteps = nq * G;
  auto step_src = [&](int st, const uint16_t*& qp, const uint16_t*& dop, int& q0, int& hq) {
    hq = hk * G + st / nq;
    q0 = q_first + (st % nq) * 32;
    qp = Q + (int64_t)(t.seq_start + q0) * qs + hq * HD;
    dop = dO + (int64_t)(t.seq_start + q0) * qs + hq * HD;
  };
  u32x4 qr[2], dr[2];
  float lr = 0.f, dd = 0.f;
  auto fetch = [&](int st) {
    const uint16_t* qp;  const uint16_t* dop;  int q0, hq;
    step_src(st, qp, dop, q0, hq);
    load_tile_regs<32>(qp, qs, t.seq_len - q0, qr);
    load_tile_regs<32>(dop, qs, t.seq_len - q0, dr);
    if (threadIdx.x < 32) {
      const int qq = min(q0 + (int)threadIdx.x, t.seq_len - 1);
      lr = lse[(int64_t)(t.seq_start + qq) * Hq + hq];
      dd = D[(int64_t)(t.seq_start + qq) * Hq + hq];
    }
  };
  auto stash = [&](int buf) {
    store_tile_regs<32>(qt[buf], qr);
    store_tile_regs<32>(dot[buf], dr);
    if (threadIdx.x < 32) { ls[buf][threadIdx.x] = lr;  ds[buf][threadIdx.x] = dd; }
  };
  if (nsteps > 0) { fetch(0);  stash(0); }
  for (int st = 0; st < nsteps; ++st) {
    __syncthreads();
    if (st + 1 < nsteps) fetch(st + 1);
    const int q0 = q_first + (st % nq) * 32;
    if (q0 + 31 >= k0w) {                                            // wave-uniform: some query at or after a key
      const uint8_t* qb = qt[st & 1];
      const uint8_t* dob = dot[st & 1];
      f32x16 sacc, dp;
#pragma unroll
      for (int e = 0; e < 16; ++e) { sacc[e] = 0.f;  dp[e] = 0.f; }
#pragma unroll
      for (int s = 0; s < 8; ++s) {
        sacc = mfma32(frag_rows(qb, 0, s, lane), kf[s], sacc);
        dp = mfma32(frag_rows(dob, 0, s, lane), vf[s], dp);
      }
      f32x16 pm;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int ql = 8 * (i >> 2) + 4 * hl + (i & 3), q = q0 + ql;
        const float p = (q >= kpos && q < t.seq_len) ? exp2f(sacc[i] * c - ls[st & 1][ql]) : 0.f;
        pm[i] = p;
        sacc[i] = p * (dp[i] - ds[st & 1][ql]);                      // dS
      }
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        const bf16x8 pf = pack8(pm, 8 * s2), dsf = pack8(sacc, 8 * s2);
#pragma unroll
        for (int db = 0; db < 4; ++db) {
          dv[db] = mfma32(frag_cols(dob, db, 16 * s2, lane), pf, dv[db]);
          dk[db] = mfma32(frag_cols(qb, db, 16 * s2, lane), dsf, dk[db]);
        }
      }
    }
    if (st + 1 < nsteps) stash((st + 1) & 1);
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
// Rotary position embedding, in place, on [T, heads * 128] bf16: one wave per (token, head); lane i rotates the
// pair (i, i + 64) by pos * base^(-i / 64).  inverse = the transposed rotation (the backward of the forward one).
// ---------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) rope_kernel(uint16_t* __restrict__ x, const int32_t* __restrict__ pos, int heads,
                                                   int64_t n_rows /* tokens * heads */, float log2_base, int inverse) {
  const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= n_rows) return;
  const int lane = threadIdx.x & 63;
  const int p = pos[r / heads];
  const float ang = (float)p * exp2f(-log2_base * (float)lane / 64.f);
  float sn, cs;
  sincosf(ang, &sn, &cs);
  if (inverse) sn = -sn;
  uint16_t* row = x + r * HD;
  const float a = __builtin_bit_cast(float, (uint32_t)row[lane] << 16);
  const float b = __builtin_bit_cast(float, (uint32_t)row[lane + 64] << 16);
  row[lane] = (uint16_t)(pack2(a * cs - b * sn, 0.f) & 0xffffu);
  row[lane + 64] = (uint16_t)(pack2(b * cs + a * sn, 0.f) & 0xffffu);
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
  hipLaunchKernelGGL(attn_rowdot_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, st, dO, O, D, rows);
  hipLaunchKernelGGL(attn_bwd_dq_kernel, dim3(n_tiles, Hq), dim3(256), 0, st, tiles, Q, K, V, dO, lse, D, dQ, Hq, Hkv, c,
                     scale);
  hipLaunchKernelGGL(attn_bwd_dkv_kernel, dim3(n_tiles, Hkv), dim3(256), 0, st, tiles, Q, K, V, dO, lse, D, dK, dV, Hq, Hkv,
                     c, scale);
}
void launch_rope(uint16_t* x, const int32_t* pos, int64_t T, int heads, float base, bool inverse, hipStream_t st) {
  const int64_t rows = T * heads;
  if (rows == 0) return;
  hipLaunchKernelGGL(rope_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, st, x, pos, heads, rows, log2f(base),
                     inverse ? 1 : 0);
}

}  // namespace tlora
