// gfx950 (CDNA4) kernels of the fused multi-LoRA linear layer.
//
// Wavefront = 64 lanes.  The rank-bound kernels contract on v_mfma_f32_32x32x16_bf16: lane l feeds row/column
// (l % 32) of its operand with the 8 consecutive k-values 8*(l/32) .. +7, and owns, of the 32x32 fp32
// result, column (l % 32) and rows 8*(i/4) + 4*(l/32) + (i%4) for accumulator register i.  The segmented GEMM
// uses v_mfma_f32_16x16x32_bf16 (row/column l % 16, k-values 8*(l/16) .. +7; result column l % 16, rows
// 4*(l/16) + i).  All kernels put the weight-side operand first, so a lane ends up with 4 consecutive output
// features of one token and stores them with one 8- or 16-byte access.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include <algorithm>

#include "tlora_kernels.h"

namespace tlora {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
// 16 x 16 x 32: lane l supplies row (column) l % 16 of its operand, k-values 8 (l / 16) .. + 7, and receives
// D[4 (l / 16) + i][l % 16], i = 0..3.
__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }
__device__ __forceinline__ u32x4 ldg16(const void* p) { return *reinterpret_cast<const u32x4*>(p); }
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  bf16x2 v = {(__bf16)lo, (__bf16)hi};   // round-to-nearest-even
  return __builtin_bit_cast(uint32_t, v);
}

// Asynchronous 16-byte-per-lane global->LDS load issued as raw instructions: lane l's 16 bytes land at LDS
// byte address `lds_base` + 16 l (lds_base wave-uniform; it travels in M0).  Unlike the compiler builtin this
// is invisible to the compiler's bookkeeping of outstanding loads, so it never adds a wait of its own: the
// kernel that uses it orders everything by hand (s_waitcnt vmcnt + barrier before the data is read, and a
// full drain before the LDS is reused or the kernel ends).  A kernel must not mix it with the builtin, which
// also keeps its LDS base in M0.
__device__ __forceinline__ void dma16(const void* gptr, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gptr), "s"(lds_base) : "memory");
}
// Same load with the address given as a wave-uniform 64-bit base plus a 32-bit unsigned byte offset per lane.
__device__ __forceinline__ void dma16s(uint32_t voff, const void* sbase, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(sbase), "s"(lds_base)
               : "memory");
}
// A pointer the program knows to be wave-uniform, moved into scalar registers (64-bit products are computed on the
// vector ALU, and the "s" operand of the load above must really be a scalar register pair).
__device__ __forceinline__ const char* uniform_ptr(const char* p) {
  const uint64_t v = reinterpret_cast<uint64_t>(p);
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return reinterpret_cast<const char*>(((uint64_t)hi << 32) | lo);
}
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
  return __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)LDS_PTR(const uint8_t, p));
}

// ---------------------------------------------------------------------------------------------------
// LDS tile layouts.
//  "row tile": R rows x 64 bf16 (128 B per row), k contiguous.  The 16-byte chunk c of row r sits at
//  chunk slot c ^ ((r >> 1) & 7): 16 consecutive rows read at one logical chunk hit 16 distinct
//  16-byte bank groups.
//  "kn tile": 64 k-rows x 256 bf16 (512 B per row), n contiguous (W as stored for the forward).  The
//  16-byte chunk c of k-row k sits at slot c ^ ((k & 3) << 2): the four k-rows one transposing read
//  touches land in four distinct 64-byte bank groups.
// ---------------------------------------------------------------------------------------------------
__device__ __forceinline__ int row_tile_off(int r, int c) { return r * 128 + ((c ^ ((r >> 1) & 7)) << 4); }
__device__ __forceinline__ int kn_tile_off(int k, int c) { return k * 512 + ((c ^ ((k & 3) << 2)) << 4); }

// MFMA operand fragment of a row tile: rows rb .. rb+31, k-step kk (16 k-values).
__device__ __forceinline__ bf16x8 frag_row_tile(const uint8_t* tile, int rb, int kk, int lane) {
  const int r = rb + (lane & 31);
  const int c = kk * 2 + (lane >> 5);
  return as_bf16x8(*reinterpret_cast<const u32x4*>(tile + row_tile_off(r, c)));
}
// "row tile" with 32 k-values per row (64 B rows): 16-byte chunk c of row r sits at slot c ^ ((r >> 2) & 3),
// so 16 consecutive rows read at one logical chunk cover all 64 banks once.
__device__ __forceinline__ int row32_off(int r, int c) { return r * 64 + ((c ^ ((r >> 2) & 3)) << 4); }
__device__ __forceinline__ bf16x8 frag_row32(const uint8_t* tile, int rb, int kk, int lane) {
  const int r = rb + (lane & 31);
  return as_bf16x8(*reinterpret_cast<const u32x4*>(tile + row32_off(r, kk * 2 + (lane >> 5))));
}

// MFMA operand fragment of a kn tile: columns nb .. nb+31, k-step kk, through the transposing LDS read
// (ds_read_b64_tr_b16: inside each group of 16 lanes, lane i receives element (i % 4) of the 8-byte
// rows addressed by lanes 4e + i/4, e = 0..3 -- i.e. 4 consecutive k for column i of a 4 x 16 block).
__device__ __forceinline__ bf16x8 frag_kn_tile(const uint8_t* tile, int nb, int kk, int lane) {
  const int s = lane & 15;
  const int n = nb + ((lane >> 4) & 1) * 16 + (s & 3) * 4;     // column this lane addresses
  const int kbase = kk * 16 + (lane >> 5) * 8 + (s >> 2);
  const int c = n >> 3;
  const int inner = (n & 7) * 2;
  s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, tile + kn_tile_off(kbase, c) + inner));
  s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, tile + kn_tile_off(kbase + 4, c) + inner));
  typedef short s16x8 __attribute__((ext_vector_type(8)));
  s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, v);
}

// Operand fragments of the 16 x 16 x 32 MFMA (the segmented GEMM): 16 rows x 32 k-values.
//  k-contiguous tiles (64-byte rows when BK = 32, 128-byte rows when BK = 64): one 16-byte read per lane.
template <int BK>
__device__ __forceinline__ bf16x8 frag16_rows(const uint8_t* tile, int rb, int ks, int lane) {
  const int r = rb + (lane & 15), g = lane >> 4;
  return as_bf16x8(*reinterpret_cast<const u32x4*>(tile + (BK == 32 ? row32_off(r, g) : row_tile_off(r, ks * 4 + g))));
}
//  "kn16 tile": k-rows x 256 bf16 (512 B per row) as W lies in memory for the forward.  Chunk c of k-row k sits at
//  slot c ^ ((k & 3) << 2) ^ (((k >> 3) & 1) << 1): the 4 k-rows x 32 bytes that one 16-lane group of a transposing
//  read touches, and those of the neighbouring group (k + 8), fall into 16 distinct 16-byte bank groups.
__device__ __forceinline__ int kn16_off(int k, int c) {
  return k * 512 + ((c ^ ((k & 3) << 2) ^ (((k >> 3) & 1) << 1)) << 4);
}
__device__ __forceinline__ bf16x8 frag16_kn(const uint8_t* tile, int nb, int ks, int lane) {
  const int s = lane & 15;
  const int n = nb + (s & 3) * 4;                              // column this lane addresses
  const int kbase = ks * 32 + (lane >> 4) * 8 + (s >> 2);
  const int c = n >> 3;
  const int inner = (n & 7) * 2;
  s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, tile + kn16_off(kbase, c) + inner));
  s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, tile + kn16_off(kbase + 4, c) + inner));
  typedef short s16x8 __attribute__((ext_vector_type(8)));
  s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, v);
}

// ---------------------------------------------------------------------------------------------------
// Adapter packing: bf16 copies, zero padded to rpad, in the three layouts the kernels read.
//   atp   : per job, A_j^T [rpad, d_in], stacked: [R + 32, d_in] with job j in rows roff_j ..
//                                                             (shrink operand; dX K-extension operand when dX runs
//                                                              against the transposed weight)
//   a_all : [d_in, R + 32], job j in columns roff_j ..        (dX K-extension operand, k contiguous)
//   b_all : [R + 32, d_out], job j in rows roff_j ..          (forward K-extension operand; dS shrink operand)
// blockIdx.y == num_jobs zero-fills the 32 trailing columns / rows, which the last tile's K-extension
// may read (against zero activations) when its rank range is rounded up to the K-step.
// ---------------------------------------------------------------------------------------------------
// Every thread assembles 8 consecutive output elements and stores them as one 16-byte chunk (d_in, d_out, rpad,
// roff and R are multiples of 8, so every chunk is aligned); A_j is read element by element (its rows are r_j
// elements long, any alignment), B_j in 16-byte chunks when its base is aligned.
__global__ void __launch_bounds__(256) pack_adapters_kernel(const JobDev* __restrict__ jobs, int num_jobs, int d_in,
                                                            int d_out, int r_total, uint16_t* __restrict__ atp,
                                                            uint16_t* __restrict__ a_all,
                                                            uint16_t* __restrict__ b_all) {
  const int stride = (int)(gridDim.x * blockDim.x);
  const int first = (int)(blockIdx.x * blockDim.x + threadIdx.x);
  const int ra = r_total + 32;
  const int kout8 = d_out / 8;
  const u32x4 zero = {0, 0, 0, 0};
  if ((int)blockIdx.y == num_jobs) {
    for (int i = first; i < 4 * d_in; i += stride)
      *reinterpret_cast<u32x4*>(a_all + (int64_t)(i >> 2) * ra + r_total + (i & 3) * 8) = zero;
    for (int i = first; i < 4 * d_in; i += stride) *reinterpret_cast<u32x4*>(atp + (int64_t)r_total * d_in + (int64_t)i * 8) = zero;
    for (int i = first; i < 4 * d_out; i += stride) *reinterpret_cast<u32x4*>(b_all + (int64_t)r_total * d_out + (int64_t)i * 8) = zero;
    return;
  }
  const JobDev jb = jobs[blockIdx.y];
  if (jb.rpad == 0) return;
  const uint16_t* A = static_cast<const uint16_t*>(jb.A);
  const uint16_t* B = static_cast<const uint16_t*>(jb.B);
  const int rank = jb.rank;
  // A_j is read once, in tiles of 64 k-rows x 64 rank columns, row by row (contiguous elements), into LDS; both
  // packed layouts are written from there: a_all chunks along the rank, A_j^T chunks along k.
  __shared__ uint16_t tile[64][66];
  const int tk = (d_in + 63) / 64, tp = (jb.rpad + 63) / 64;
  for (int t = blockIdx.x; t < tk * tp; t += gridDim.x) {
    const int k_base = (t / tp) * 64, p_base = (t % tp) * 64;
#pragma unroll
    for (int h = 0; h < 16; ++h) {
      const int kk = (threadIdx.x >> 6) + h * 4, pp = threadIdx.x & 63;
      const int k = k_base + kk, pcol = p_base + pp;
      tile[kk][pp] = (k < d_in && pcol < rank) ? A[(int64_t)k * rank + pcol] : (uint16_t)0;
    }
    __syncthreads();
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int c = threadIdx.x + h * 256;                       // 512 chunks of 8 per layout
      {   // a_all: row k, rank columns p0 .. p0 + 7
        const int kk = c >> 3, p0 = (c & 7) * 8;
        if (k_base + kk < d_in && p_base + p0 < jb.rpad) {
          uint32_t v[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] = tile[kk][p0 + e];
          *reinterpret_cast<u32x4*>(a_all + (int64_t)(k_base + kk) * ra + jb.roff + p_base + p0) =
              u32x4{v[0] | (v[1] << 16), v[2] | (v[3] << 16), v[4] | (v[5] << 16), v[6] | (v[7] << 16)};
        }
      }
      {   // A_j^T: rank row p, k0 .. k0 + 7
        const int pp = c >> 3, k0 = (c & 7) * 8;
        if (p_base + pp < jb.rpad && k_base + k0 < d_in) {
          uint32_t v[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] = tile[k0 + e][pp];
          *reinterpret_cast<u32x4*>(atp + jb.atp_off + (int64_t)(p_base + pp) * d_in + k_base + k0) =
              u32x4{v[0] | (v[1] << 16), v[2] | (v[3] << 16), v[4] | (v[5] << 16), v[6] | (v[7] << 16)};
        }
      }
    }
    __syncthreads();
  }
  // B_j into its rows of b_all
  uint16_t* bdst = b_all + (int64_t)jb.roff * d_out;
  const bool b_aligned = (reinterpret_cast<uintptr_t>(B) & 15) == 0;
  for (int i = first; i < jb.rpad * kout8; i += stride) {
    const int p = i / kout8, c0 = (i - p * kout8) * 8;
    u32x4 v = zero;
    if (p < rank) {
      const uint16_t* src = B + (int64_t)p * d_out + c0;
      if (b_aligned) {
        v = *reinterpret_cast<const u32x4*>(src);
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = (uint32_t)src[2 * e] | ((uint32_t)src[2 * e + 1] << 16);
      }
    }
    *reinterpret_cast<u32x4*>(bdst + (int64_t)p * d_out + c0) = v;
  }
}

void launch_pack_adapters(const JobDev* jobs, int num_jobs, int d_in, int d_out, int max_rpad, int r_total,
                          uint16_t* atp, uint16_t* a_all, uint16_t* b_all, hipStream_t st) {
  if (max_rpad == 0) return;
  const int64_t n = (int64_t)max_rpad * (d_in > d_out ? d_in : d_out) / 8;     // 16-byte chunks of the largest layout
  int bx = (int)((n + 256 * 4 - 1) / (256 * 4));
  if (bx > 512) bx = 512;
  if (bx < 1) bx = 1;
  hipLaunchKernelGGL(pack_adapters_kernel, dim3(bx, num_jobs + 1), dim3(256), 0, st, jobs, num_jobs, d_in, d_out,
                     r_total, atp, a_all, b_all);
}

// out[c, r] = in[r, c] for a row-major bf16 matrix [rows, cols] (both multiples of 8): 64 x 64 tiles through LDS,
// 16-byte global accesses on both sides.
__global__ void __launch_bounds__(256) transpose_bf16_kernel(const uint16_t* __restrict__ in, uint16_t* __restrict__ out,
                                                             int rows, int cols) {
  __shared__ uint16_t tile[64][72];        // [c][r]; 144-byte pitch keeps the 16-byte row reads aligned
  const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  const int tid = threadIdx.x;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int r = (tid >> 3) + h * 32, cc = (tid & 7) * 8;
    u32x4 v = {0, 0, 0, 0};
    if (r0 + r < rows && c0 + cc < cols) v = ldg16(in + (int64_t)(r0 + r) * cols + c0 + cc);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      tile[cc + 2 * e][r] = (uint16_t)(v[e] & 0xffffu);
      tile[cc + 2 * e + 1][r] = (uint16_t)(v[e] >> 16);
    }
  }
  __syncthreads();
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int c = (tid >> 3) + h * 32, rr = (tid & 7) * 8;
    if (c0 + c < cols && r0 + rr < rows)
      *reinterpret_cast<u32x4*>(out + (int64_t)(c0 + c) * rows + r0 + rr) = *reinterpret_cast<const u32x4*>(&tile[c][rr]);
  }
}

void launch_transpose_bf16(const uint16_t* in, uint16_t* out, int rows, int cols, hipStream_t st) {
  if (rows == 0 || cols == 0) return;
  hipLaunchKernelGGL(transpose_bf16_kernel, dim3((cols + 63) / 64, (rows + 63) / 64), dim3(256), 0, st, in, out, rows,
                     cols);
}

__global__ void __launch_bounds__(256) zero_fill_kernel(u32x4* __restrict__ dst, size_t n16) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = u32x4{0, 0, 0, 0};
}

void launch_zero_fill(void* ptr, size_t bytes, hipStream_t st) {
  const size_t n16 = bytes / 16;
  if (n16 == 0) return;
  size_t blocks = (n16 + 255) / 256;
  if (blocks > 2048) blocks = 2048;
  hipLaunchKernelGGL(zero_fill_kernel, dim3((unsigned)blocks), dim3(256), 0, st, static_cast<u32x4*>(ptr), n16);
}

// Host tables -> device memory through kernel arguments: a launch carries up to kArgChunkWords 32-bit words by
// value and its threads store them.  No staging buffer and no copy: usable where nothing may be allocated, and
// under stream capture (the words are part of the recorded launch).
constexpr int kArgChunkWords = 896;            // 3584 bytes: below the 4 KB of a launch's argument block
struct ArgChunk {
  uint32_t w[kArgChunkWords];
};
__global__ void __launch_bounds__(256) table_write_kernel(uint32_t* __restrict__ dst, const ArgChunk c, int n) {
  for (int i = threadIdx.x; i < n; i += 256) dst[i] = c.w[i];
}

void launch_table_write(const void* host_src, size_t bytes, void* dst, hipStream_t st) {
  const size_t words = (bytes + 3) / 4;        // the destination is padded to 256 bytes by the planner
  const uint8_t* src = static_cast<const uint8_t*>(host_src);
  for (size_t w0 = 0; w0 < words; w0 += kArgChunkWords) {
    ArgChunk c;
    const size_t n = std::min<size_t>(kArgChunkWords, words - w0);
    const size_t nbytes = std::min<size_t>(n * 4, bytes - w0 * 4);
    memset(&c, 0, sizeof(c));
    memcpy(c.w, src + w0 * 4, nbytes);
    hipLaunchKernelGGL(table_write_kernel, dim3(1), dim3(256), 0, st, static_cast<uint32_t*>(dst) + w0, c, (int)n);
  }
}

// Plan tables from a pinned staging buffer (host memory, read through its device address) into the workspace, as an
// ordinary kernel on the caller's stream: a host-to-device copy command makes the stream's next kernel wait for the
// copy engine's signal (~20 us of idle stream per call), a kernel in the same queue does not.
__global__ void __launch_bounds__(256) table_copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst,
                                                         size_t n16) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}
void launch_table_copy(const void* src_device_view, void* dst, size_t bytes, hipStream_t st) {
  const size_t n16 = bytes / 16;                 // the caller passes a multiple of 16 bytes
  if (n16 == 0) return;
  const unsigned blocks = (unsigned)std::min<size_t>((n16 + 255) / 256, 256);
  hipLaunchKernelGGL(table_copy_kernel, dim3(blocks), dim3(256), 0, st, static_cast<const u32x4*>(src_device_view),
                     static_cast<u32x4*>(dst), n16);
}

// ---------------------------------------------------------------------------------------------------
// Shrink:  out_j[t, p] = sum_k act[t, k] * P_j[p, k]      (Sec. 3.3: the compact |X_j| x r_j intermediate)
// One workgroup = ROWS token rows of one job x 64 padded rank columns; 4 waves.
// ---------------------------------------------------------------------------------------------------
template <int ROWS>
__global__ void __launch_bounds__(256) shrink_kernel(const JobDev* __restrict__ jobs,
                                                     const TileDev* __restrict__ tiles,
                                                     const ShrinkUnit* __restrict__ units,
                                                     const uint16_t* __restrict__ act, int K,
                                                     const uint16_t* __restrict__ packed, int packed_is_atp,
                                                     uint16_t* __restrict__ Shi, uint16_t* __restrict__ Slo,
                                                     uint16_t* __restrict__ Sx, const int32_t* __restrict__ row_index) {
  constexpr int WM = ROWS / 32;          // waves along token rows
  constexpr int WN = 4 / WM;             // waves along rank columns
  constexpr int PW = kShrinkCols / WN;   // rank columns per wave
  constexpr int NPB = PW / 32;           // 32-wide rank blocks per wave
  constexpr int A_CH = ROWS * 8 / 256;   // 16-byte chunks per thread, activation tile
  constexpr int P_CH = kShrinkCols * 8 / 256;
  static_assert(kGemmBM == 256, "the row -> GEMM tile lookup below shifts by 8");

  __shared__ __attribute__((aligned(16))) uint8_t lds[2 * (ROWS + kShrinkCols) * 128];
  auto a_tile = [&](int buf) { return lds + buf * ((ROWS + kShrinkCols) * 128); };
  auto p_tile = [&](int buf) { return lds + buf * ((ROWS + kShrinkCols) * 128) + ROWS * 128; };

  const ShrinkUnit u = units[blockIdx.x];
  const JobDev jb = jobs[u.job];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave % WM, wn = wave / WM;
  const int p0 = u.pb * kShrinkCols;                     // first padded rank column of this unit
  const int pvalid = min(kShrinkCols, jb.rpad - p0);     // > 0 by construction
  const uint16_t* P = packed + (packed_is_atp ? jb.atp_off : (int64_t)jb.roff * K) + (int64_t)p0 * K;

  f32x16 acc[NPB];
#pragma unroll
  for (int i = 0; i < NPB; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;

  // the activation rows this thread fetches (row_index: the batch row that holds token row t of the job-sorted order)
  const uint16_t* arow[A_CH];
#pragma unroll
  for (int i = 0; i < A_CH; ++i) {
    const int t = u.t0 + min((tid + i * 256) >> 3, u.nrows - 1);
    arow[i] = act + (int64_t)(row_index ? row_index[t] : t) * K;
  }
  u32x4 areg[A_CH], preg[P_CH];
  auto load_tiles = [&](int k0) {
#pragma unroll
    for (int i = 0; i < A_CH; ++i) {
      const int id = tid + i * 256, r = id >> 3, c = id & 7;
      const bool ok = r < u.nrows && k0 + c * 8 < K;
      areg[i] = ok ? ldg16(arow[i] + k0 + c * 8) : u32x4{0, 0, 0, 0};
    }
#pragma unroll
    for (int i = 0; i < P_CH; ++i) {
      const int id = tid + i * 256, r = id >> 3, c = id & 7;
      const bool ok = r < pvalid && k0 + c * 8 < K;
      preg[i] = ok ? ldg16(P + (int64_t)r * K + k0 + c * 8) : u32x4{0, 0, 0, 0};
    }
  };
  auto store_tiles = [&](int buf) {
#pragma unroll
    for (int i = 0; i < A_CH; ++i) {
      const int id = tid + i * 256, r = id >> 3, c = id & 7;
      *reinterpret_cast<u32x4*>(a_tile(buf) + row_tile_off(r, c)) = areg[i];
    }
#pragma unroll
    for (int i = 0; i < P_CH; ++i) {
      const int id = tid + i * 256, r = id >> 3, c = id & 7;
      *reinterpret_cast<u32x4*>(p_tile(buf) + row_tile_off(r, c)) = preg[i];
    }
  };

  const int nkt = (K + 63) / 64;
  load_tiles(0);
  store_tiles(0);
  __syncthreads();
  for (int kt = 0; kt < nkt; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < nkt) load_tiles((kt + 1) * 64);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      const bf16x8 xf = frag_row_tile(a_tile(buf), wm * 32, kk, lane);
#pragma unroll
      for (int i = 0; i < NPB; ++i) {
        const bf16x8 pf = frag_row_tile(p_tile(buf), wn * PW + i * 32, kk, lane);
        acc[i] = mfma32(pf, xf, acc[i]);
      }
    }
    if (kt + 1 < nkt) store_tiles(buf ^ 1);
    __syncthreads();
  }

  // lane: token row (lane % 32); registers: 4 consecutive rank columns per group g.
  // Outputs: the intermediate as bf16 hi + lo planes (hi = bf16(x), lo = bf16(x - hi): ~16 mantissa bits for
  // the dA / dB contractions) in the packed ragged layout, whose rows are padded with zeros to a multiple of
  // kGradStep per job (the job's last unit writes them: its accumulators there are zero); and bf16
  // scale_j * x in the row's slot of its GEMM tile's K-extension operand.
  const int r = wm * 32 + (lane & 31);
  const int jrow = u.t0 - jb.row0 + r;                                        // row inside the job
  const bool last_unit = u.t0 + u.nrows == jb.row1;
  const int jrows_padded = (jb.row1 - jb.row0 + kGradStep - 1) / kGradStep * kGradStep;
  if (r < u.nrows || (last_unit && jrow < jrows_padded)) {
    const bool live = r < u.nrows;
    const int t = u.t0 + r;
    const int64_t rowbase = jb.soff + (int64_t)jrow * jb.rpad;
    const TileDev td = tiles[min(t, jb.row1 - 1) >> 8];
    uint16_t* const xrow = Sx + td.aoff + (int64_t)(t & 255) * td.kext + (jb.roff - td.roff_first);
#pragma unroll
    for (int i = 0; i < NPB; ++i)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int p = p0 + wn * PW + i * 32 + g * 8 + (lane >> 5) * 4;
        if (p < jb.rpad) {
          const float v[4] = {acc[i][g * 4 + 0], acc[i][g * 4 + 1], acc[i][g * 4 + 2], acc[i][g * 4 + 3]};
          float lo[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) lo[e] = v[e] - (float)(__bf16)v[e];
          *reinterpret_cast<u32x2*>(Shi + rowbase + p) = u32x2{pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])};
          *reinterpret_cast<u32x2*>(Slo + rowbase + p) = u32x2{pack_bf16x2(lo[0], lo[1]), pack_bf16x2(lo[2], lo[3])};
          if (live) {
            u32x2 b = {pack_bf16x2(jb.scale * v[0], jb.scale * v[1]), pack_bf16x2(jb.scale * v[2], jb.scale * v[3])};
            *reinterpret_cast<u32x2*>(xrow + p) = b;
          }
        }
      }
  }
}

// s_waitcnt immediate: vmcnt(vm) lgkmcnt(0), export counter untouched (vmcnt is 6 bits, split 4 + 2)
constexpr int waitcnt_vm_lgkm0(int vm) { return (vm & 15) | ((vm >> 4) << 14) | 0x0070; }

// ---------------------------------------------------------------------------------------------------
// Shrink, streaming version (needs K % KS == 0, KS = 32 or 64 k-values per step): one workgroup = ROWS token rows of one job x up to 128 padded
// rank columns.  K-steps of 32; a stage holds the activation tile (ROWS x 32) and the adapter tile
// (128 x 32); NS stages are filled NS - 1 steps ahead by raw asynchronous global->LDS loads, so several KB
// per wave stay in flight without holding registers -- the kernel is bound by how fast X (or dY) streams in.
// ---------------------------------------------------------------------------------------------------
// PCOLS: rank columns staged per step.  A unit whose job has at most 32 padded rank columns stages a 32-column
// adapter tile and spends the LDS it saves on more stages: the kernel is bound by the bytes of X in flight.
// WAVES: 4, or 8 for the 128-row units.  A CU runs one workgroup (the stages fill its LDS), so with four waves every
// SIMD has a single wave whose LDS reads, MFMAs and waits follow one another; for a 128-column unit that serial
// chain (20 KB of fragment reads and 16 MFMAs per wave and step) is as long as the step's share of the memory
// stream, and since a launch is one round of units its slowest units set its duration.  Eight waves (4 row blocks
// x 2 column halves) put two waves on every SIMD, so one's fragment reads overlap the other's MFMAs, and halve the
// loads each wave issues.  For a 32-column unit waves 4-7 only help to load.
template <int ROWS, int NS, int KS, int PCOLS, int WAVES>
__device__ __forceinline__ void shrink_stream_body(uint8_t* lds, const ShrinkUnit u, const JobDev jb,
                                                   const TileDev* __restrict__ tiles,
                                                   const uint16_t* __restrict__ act, int K,
                                                   const uint16_t* __restrict__ packed, int packed_is_atp,
                                                   uint16_t* __restrict__ Shi, uint16_t* __restrict__ Slo,
                                                   uint16_t* __restrict__ Sx, const int32_t* __restrict__ row_index) {
  constexpr int CW = PCOLS == 32 ? 4 : WAVES;      // waves that multiply
  constexpr int WM = PCOLS == 32 ? 4 : ROWS / 32;  // waves along token rows
  constexpr int WN = CW / WM;                      // waves along rank columns
  static_assert(WM * 32 == ROWS || PCOLS != 32, "a 32-column unit needs 128 token rows for its four waves");
  constexpr int PW = PCOLS / WN, NPB = PW / 32;    // rank columns (and 32-wide blocks) per wave
  static_assert(WN >= 1 && PW % 32 == 0 && NPB >= 1, "wave layout");
  constexpr int RB = KS * 2;                       // bytes per tile row: 64 (K-steps of 32) or 128 (of 64)
  constexpr int CPR = RB / 16;                     // 16-byte chunks per tile row
  constexpr int A_BYTES = ROWS * RB, P_BYTES = PCOLS * RB, STAGE = A_BYTES + P_BYTES;
  constexpr int A_TOT = A_BYTES / 1024, P_TOT = P_BYTES / 1024;            // 1 KB wave-loads per tile
  constexpr int A_LD = A_TOT / WAVES, P_LD = (P_TOT + WAVES - 1) / WAVES;   // loads per wave per step
  static_assert(kGemmBM == 256, "the row -> GEMM tile lookup below shifts by 8");
  static_assert(NS * STAGE <= 160 * 1024, "LDS of a CU");
  static_assert(A_LD >= 1 && A_LD * WAVES == A_TOT && P_LD >= 1, "every wave issues the same number of loads per step");

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, so LDS bases stay in SGPRs
  const bool multiplies = wave < CW;
  const int wm = wave % WM, wn = (wave / WM) % WN;
  const int p0 = u.pb * PCOLS;
  const int pvalid = min(PCOLS, jb.rpad - p0);     // > 0 by construction
  const uint16_t* P = packed + (packed_is_atp ? jb.atp_off : (int64_t)jb.roff * K) + (int64_t)p0 * K;
  const int nsteps = K / KS;

  f32x16 acc[NPB];
#pragma unroll
  for (int i = 0; i < NPB; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;

  // lane -> (row, 16-byte chunk) of the 64-byte-row tiles; rows beyond the unit / beyond rpad are clamped
  // (they only feed outputs that are not stored, or that are stored as zeros)
  const uint16_t* asrc[A_LD];
  const uint16_t* psrc[P_LD];
  int pslot[P_LD];         // which 1 KB piece of the adapter tile this wave's load i fills (when the tile has fewer
                           // pieces than there are waves, the upper waves repeat the lower waves' loads: same bytes
                           // to the same place, and every wave keeps the same number of loads in flight)
  bool plive[P_LD];        // adapter-tile lanes beyond rpad fetch nothing (the stale slots only feed unused rank
                           // columns); lane 0 always fetches so every wave issues the same number of loads
#pragma unroll
  for (int i = 0; i < A_LD; ++i) {
    const int q = (wave * A_LD + i) * 64 + lane, r = q / CPR;
    const int c = KS == 32 ? (q & 3) ^ ((r >> 2) & 3) : (q & 7) ^ ((r >> 1) & 7);
    const int t = u.t0 + min(r, u.nrows - 1);      // token row of the job-sorted order; row_index: where it lies
    asrc[i] = act + (int64_t)(row_index ? row_index[t] : t) * K + c * 8;
  }
#pragma unroll
  for (int i = 0; i < P_LD; ++i) {
    pslot[i] = (wave * P_LD + i) % P_TOT;
    const int q = pslot[i] * 64 + lane, r = q / CPR;
    const int c = KS == 32 ? (q & 3) ^ ((r >> 2) & 3) : (q & 7) ^ ((r >> 1) & 7);
    psrc[i] = P + (int64_t)min(r, pvalid - 1) * K + c * 8;
    plive[i] = r < pvalid || lane == 0;
  }
  const uint32_t lds0 = lds_addr(lds);
  int f_step = 0;
  auto issue = [&]() {
    const int st = min(f_step, nsteps - 1);        // trailing issues re-load the last step (uniform load count)
    const uint32_t base = lds0 + (f_step % NS) * STAGE;
#pragma unroll
    for (int i = 0; i < A_LD; ++i) dma16(asrc[i] + st * KS, base + (wave * A_LD + i) * 1024);
#pragma unroll
    for (int i = 0; i < P_LD; ++i)
      if (plive[i]) dma16(psrc[i] + st * KS, base + A_BYTES + __builtin_amdgcn_readfirstlane(pslot[i]) * 1024);
    ++f_step;
  };
  for (int i = 0; i < NS - 1; ++i) issue();
  for (int kt = 0; kt < nsteps; ++kt) {
    // loads complete in order: all but those of the NS - 2 youngest steps have landed
    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0((NS - 2) * (A_LD + P_LD)));
    __builtin_amdgcn_s_barrier();
    issue();                                       // into the stage read in step kt - 1
    if (multiplies) {
      const uint8_t* S = lds + (kt % NS) * STAGE;
      // all fragments of the step first, then the MFMAs: a read -> wait -> MFMA chain per k-slice would pay the LDS
      // latency KS / 16 times per step
      bf16x8 xf[KS / 16], pf[KS / 16][NPB];
#pragma unroll
      for (int kk = 0; kk < KS / 16; ++kk) {
        xf[kk] = KS == 32 ? frag_row32(S, wm * 32, kk, lane) : frag_row_tile(S, wm * 32, kk, lane);
#pragma unroll
        for (int i = 0; i < NPB; ++i)
          pf[kk][i] = KS == 32 ? frag_row32(S + A_BYTES, wn * PW + i * 32, kk, lane)
                               : frag_row_tile(S + A_BYTES, wn * PW + i * 32, kk, lane);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int kk = 0; kk < KS / 16; ++kk)
#pragma unroll
        for (int i = 0; i < NPB; ++i) acc[i] = mfma32(pf[kk][i], xf[kk], acc[i]);
    }
  }
  __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(0));   // drain: the stages are reused below
  __syncthreads();

  // Outputs: bf16 hi + lo planes (hi = bf16(x), lo = bf16(x - hi); pad rows of the job's last unit written as zeros)
  // and bf16 scale_j * x into the row's slot of its GEMM tile's K-extension operand.  A lane holds 4 rank columns of
  // one token row per accumulator group, so storing from the registers would be 8-byte pieces 2 * rpad bytes apart;
  // instead each of the three tensors goes through LDS ([ROWS][PCOLS] bf16, row pitch padded by 8 bytes so the 32 rows
  // a store instruction touches fall into distinct banks) and leaves as 16 bytes per lane along the rows -- in the
  // packed layout the unit's rows follow one another, so a 128-column unit writes one contiguous 32 KB block per plane.
  constexpr int OPITCH = PCOLS * 2 + 8;
  static_assert(ROWS * OPITCH <= NS * STAGE, "the output tile fits in the stages");
  const int jrows_padded = (jb.row1 - jb.row0 + kGradStep - 1) / kGradStep * kGradStep;
  const bool last_unit = u.t0 + u.nrows == jb.row1;
#pragma unroll
  for (int which = 0; which < 3; ++which) {            // 0: hi plane, 1: lo plane, 2: scaled operand of the GEMM
    if (multiplies) {
      const int r = wm * 32 + (lane & 31);
      const bool live = r < u.nrows;
#pragma unroll
      for (int i = 0; i < NPB; ++i)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int pl = wn * PW + i * 32 + g * 8 + (lane >> 5) * 4;
          float v[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float x = live ? acc[i][g * 4 + e] : 0.f;
            v[e] = which == 0 ? x : which == 1 ? x - (float)(__bf16)x : jb.scale * x;
          }
          *reinterpret_cast<u32x2*>(lds + r * OPITCH + pl * 2) = u32x2{pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])};
        }
    }
    __syncthreads();
    constexpr int CPT = PCOLS / 8;                      // 16-byte chunks per tile row
    for (int q = tid; q < ROWS * CPT; q += WAVES * 64) {
      const int r = q / CPT, c = q % CPT;
      const int p = p0 + c * 8;
      const int jrow = u.t0 - jb.row0 + r;
      const bool live = r < u.nrows;
      if (p < jb.rpad && (live || (which < 2 && last_unit && jrow < jrows_padded))) {
        const u32x2 a = *reinterpret_cast<const u32x2*>(lds + r * OPITCH + c * 16);
        const u32x2 b = *reinterpret_cast<const u32x2*>(lds + r * OPITCH + c * 16 + 8);
        const u32x4 v = {a[0], a[1], b[0], b[1]};
        if (which < 2) {
          *reinterpret_cast<u32x4*>((which == 0 ? Shi : Slo) + jb.soff + (int64_t)jrow * jb.rpad + p) = v;
        } else {
          const int t = u.t0 + r;
          const TileDev td = tiles[t >> 8];
          *reinterpret_cast<u32x4*>(Sx + td.aoff + (int64_t)(t & 255) * td.kext + (jb.roff - td.roff_first) + p) = v;
        }
      }
    }
    if (which < 2) __syncthreads();
  }
}

template <int ROWS, int NS, int KS, int WAVES>
__global__ void __launch_bounds__(WAVES * 64) shrink_stream_kernel(const JobDev* __restrict__ jobs,
                                                                   const TileDev* __restrict__ tiles,
                                                                   const ShrinkUnit* __restrict__ units,
                                                                   const uint16_t* __restrict__ act, int K,
                                                                   const uint16_t* __restrict__ packed, int packed_is_atp,
                                                                   uint16_t* __restrict__ Shi, uint16_t* __restrict__ Slo,
                                                                   uint16_t* __restrict__ Sx,
                                                                   const int32_t* __restrict__ row_index) {
  // NS stages of (ROWS + 128) rows, or -- 128-row units of low-rank jobs, K-steps of 64 -- 8 stages of 128 + 32 rows
  constexpr int LOW = ROWS == 128 && KS == 64;
  constexpr int BYTES = LOW ? 8 * (128 + 32) * 128 : NS * (ROWS + 128) * KS * 2;
  constexpr int NS_HIGH = LOW ? 5 : NS;          // the LDS is there anyway: a fifth stage for the 128-column units
  __shared__ __attribute__((aligned(1024))) uint8_t lds[BYTES];
  const ShrinkUnit u = units[blockIdx.x];
  const JobDev jb = jobs[u.job];
  if (LOW && jb.rpad <= 32)
    shrink_stream_body<128, 8, 64, 32, WAVES>(lds, u, jb, tiles, act, K, packed, packed_is_atp, Shi, Slo, Sx, row_index);
  else
    shrink_stream_body<ROWS, NS_HIGH, KS, 128, WAVES>(lds, u, jb, tiles, act, K, packed, packed_is_atp, Shi, Slo, Sx,
                                                      row_index);
}

void launch_shrink(const JobDev* jobs, const TileDev* tiles, const ShrinkUnit* units, int num_units, int shrink_rows,
                   const uint16_t* act, int K, const uint16_t* packed, bool packed_is_atp, uint16_t* S_hi,
                   uint16_t* S_lo, uint16_t* Sx, const int32_t* row_index, hipStream_t st) {
  if (num_units == 0) return;
  // generic kernel: units of 64 rows x 64 rank columns
  hipLaunchKernelGGL(shrink_kernel<64>, dim3(num_units), dim3(256), 0, st, jobs, tiles, units, act, K, packed,
                     packed_is_atp ? 1 : 0, S_hi, S_lo, Sx, row_index);
  (void)shrink_rows;
}

void launch_shrink_stream(const JobDev* jobs, const TileDev* tiles, const ShrinkUnit* units, int num_units,
                          int shrink_rows, int stages, const uint16_t* act, int K, const uint16_t* packed,
                          bool packed_is_atp, uint16_t* S_hi, uint16_t* S_lo, uint16_t* Sx, const int32_t* row_index,
                          hipStream_t st) {
  if (num_units == 0) return;
  const int atp = packed_is_atp ? 1 : 0;
#define TLORA_SHRINK_LAUNCH(R, N, KS, WV)                                                                              \
  hipLaunchKernelGGL((shrink_stream_kernel<R, N, KS, WV>), dim3(num_units), dim3(WV * 64), 0, st, jobs, tiles, units,  \
                     act, K, packed, atp, S_hi, S_lo, Sx, row_index)
  const bool wide = K % 64 == 0 && stages < 8;      // K-steps of 64: half as many barriers per byte
  if (shrink_rows == 128) {
    if (wide)             TLORA_SHRINK_LAUNCH(128, 4, 64, 8);
    else if (stages >= 8) TLORA_SHRINK_LAUNCH(128, 8, 32, 8);
    else                  TLORA_SHRINK_LAUNCH(128, 4, 32, 8);
  } else if (shrink_rows == 32 && K % 64 == 0) {      // the planner asks for 32 rows only when K % 64 == 0
    TLORA_SHRINK_LAUNCH(32, 4, 64, 4);
  } else {
    if (wide)             TLORA_SHRINK_LAUNCH(64, 4, 64, 4);
    else if (stages >= 8) TLORA_SHRINK_LAUNCH(64, 8, 32, 4);
    else                  TLORA_SHRINK_LAUNCH(64, 4, 32, 4);
  }
#undef TLORA_SHRINK_LAUNCH
}

// ---------------------------------------------------------------------------------------------------
// Segmented backbone GEMM with the adapter expand fused as extra K-steps:
//   out[t, :] = act[t, :] . Wop  +  Sb_j[t, :] . Eop_j          (job j = owner of row t)
// 256 x 256 output tile per workgroup of 8 waves (2 along tokens x 4 along features, 128 x 64 each).
// Row tiles are uniform over the concatenated batch and may hold rows of several jobs: the backbone
// K-loop is job-blind, and each job present in the tile then adds ceil(rpad_j / 32) K-steps in which only
// its own rows are non-zero.
//
// K-loop: steps of 32 k-values (one 16 x 16 x 32 MFMA slice).  The operands stream through a ring of five
// 32 KB LDS slots as an alternating sequence of tiles L_0, L_1, ...: L_q with q odd is an activation tile,
// q even a weight tile, and L_q holds the k-values of steps q - 1 and q (256 rows x 64 k-values, 128 B per row
// for a k-contiguous operand; 64 k-rows x 256 columns for the forward weight).  Step s reads the second half of
// L_s and the first half of L_s+1, then L_s is free; L_s+4 is issued at step s, so three tiles (96 KB) are in
// flight per CU.  Compared with loading both operands 32 k-values at a time, every row of a k-contiguous
// operand is fetched as a whole 128-byte line: the same bytes in half as many L2 requests (a load-only
// replica of the two streams sustains ~15.4 TB/s this way against ~11.5 TB/s).
// ---------------------------------------------------------------------------------------------------
struct GemmParams {
  const TileDev* tiles;
  const uint16_t* act;      // [T, K]
  const uint16_t* W;        // KN: [K, N]   else [N, K]
  const uint16_t* Sx;       // per-tile K-extension operands [256, kext] (bf16, scaled, zero padded)
  const uint16_t* packed;   // KN: b_all [R + 32, N];  else a_all [N, R + 32]
  uint16_t* out;            // [T, N]
  int T, K, N;
  int ra;                   // R + 32: row stride of a_all
  int tiles_m, tiles_n;
  unsigned long long* clk;  // optional: every 64th workgroup adds {cycles, 100 MHz ticks} of its K-loop (pre-zeroed)
  const int32_t* out_index; // optional: output row of tile row t (scatter); null = t itself
  const int32_t* in_index;  // INDEXED instantiations: batch row that holds activation row t (gather inside the loads)
};

// KTAIL: the instantiation for K % 32 != 0 carries the extra predicated step; keeping it out of the common one
// keeps its register pressure away from every tile.
// INDEXED: the activation rows are fetched through P.in_index (token-indexed calls: the batch stays in its own order).
// A lane then keeps one byte offset per row it loads (four) instead of two offsets plus scalar row strides; offsets are
// 32 bits, so the launcher takes this instantiation only while T * K * 2 stays below 4 GiB.
template <bool KN, bool KTAIL, bool INDEXED>
__global__ void __launch_bounds__(512) seg_gemm_kernel(GemmParams P) {
  constexpr int NT = 512;                            // threads: 8 waves
  constexpr int NFB = 4;                             // 16-wide feature blocks per wave (64 columns)
  constexpr int BM = kGemmBM, BN = kGemmBN;
  static_assert(BM == 256 && BN == 256 && kGemmBK == 32, "tile shape is baked into the index arithmetic below");
  constexpr int SLOT = 32768;
  // 5 x 32 KB: the whole LDS of a CU.  The loads are raw instructions the compiler does not track; every wait on
  // them is written out below.  (A spilled register in this loop would be fatal for the pipeline: its reload is a
  // vector-memory load, and waiting for it means waiting for every tile in flight.)
  __shared__ __attribute__((aligned(1024))) uint8_t lds[5 * SLOT];
  uint8_t* const sl0 = lds;
  uint8_t* const sl1 = lds + SLOT;
  uint8_t* const sl2 = lds + 2 * SLOT;
  uint8_t* const sl3 = lds + 3 * SLOT;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave & 1, wn = wave >> 1;

  // Workgroup ids are dealt round-robin to the 8 XCDs; hand each XCD a contiguous run of logical tile
  // ids, and walk tiles in groups of 4 row tiles so the 32 workgroups an XCD runs together share
  // 4 activation panels and 8 weight panels in its L2 (the weight tiles are the cheaper stream: whole 512-byte
  // rows; groups of 4 measured 1-4 % faster than 8, and 16 or 32 slower).
  int tm, tn;
  {
    const int nb = P.tiles_m * P.tiles_n, b = blockIdx.x;
    const int q = nb >> 3, rem = nb & 7, x = b & 7;
    const int L = x * q + min(x, rem) + (b >> 3);
    constexpr int GM = 4;
    const int per_group = GM * P.tiles_n;
    const int grp = L / per_group, first_m = grp * GM;
    const int gsize = min(GM, P.tiles_m - first_m);
    const int Lg = L - grp * per_group;
    // (the divisions run on the vector ALU; everything derived from the tile id is wave-uniform and belongs in
    // scalar registers)
    tm = __builtin_amdgcn_readfirstlane(first_m + Lg % gsize);
    tn = __builtin_amdgcn_readfirstlane(Lg / gsize);
  }
  const int row0 = tm * BM, col0 = tn * BN;
  const int rows_valid = min(BM, P.T - row0);
  const TileDev td = P.tiles[tm];

  // 16 x 16 x 32 MFMAs: with dense random operands the chip sustains ~15 % more of them per second than of the
  // 32 x 32 x 16 shape under its power limit (half the accumulator traffic per flop).
  f32x4 acc[NFB][8];                                 // [feature block][token block of 16]
#pragma unroll
  for (int j = 0; j < NFB; ++j)
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[j][i] = f32x4{0.f, 0.f, 0.f, 0.f};

  auto mma_slice = [&](const bf16x8 (&xf)[8], const bf16x8 (&wf)[NFB]) {
#pragma unroll
    for (int j = 0; j < NFB; ++j)
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[j][i] = mfma16(wf[j], xf[i], acc[j][i]);
  };

  // ---- the K-loop: K / 32 backbone steps, then kext / 32 adapter steps, one software pipeline ----------------
  const int nfull = P.K / 32;
  const int ntot = nfull + td.kext / 32;
  const bool clocked = P.clk != nullptr && (blockIdx.x & 63) == 0;   // a sample of workgroups across the grid
  unsigned long long cyc0 = 0, tick0 = 0;
  if (clocked) { cyc0 = __builtin_readcyclecounter();  tick0 = __builtin_amdgcn_s_memrealtime(); }
  if (ntot > 0) {
    // Loads.  A tile is 2048 16-byte slots; wave w issues four 1 KB loads per tile, lane l's 16 bytes landing at
    // slot (4 w + i) 64 + l.  Which k-values and which row / column that slot holds follows from the tile
    // layout, so the source address is recomputed per load from the step index t of the lane's half of the
    // tile: t < K / 32 reads the backbone operands, later steps the tile's dense [256, kext] adapter operand
    // (rows of other jobs are stored zeros) against rows roff_first.. of b_all (forward) or columns roff_first..
    // of a_all (backward).  Steps outside 0 .. ntot - 1 (first half of L_0, tiles past the end) and rows /
    // columns beyond the problem edge are clamped to valid ones: they only fill LDS that is never read or feed
    // outputs that are never stored.  Selects, not branches: a branch around a load would make the compiler
    // wait for every outstanding load where the paths merge.
    //  k-contiguous tile ("row tile", 128 B rows): slot p -> row p / 8, 16-byte chunk (p % 8) ^ ((row / 2) % 8).
    // A tile whose two steps lie on the same side of the backbone / adapter boundary (all but one or two per
    // operand) is loaded as wave-uniform base + per-lane 32-bit offset; the offsets are loop constants.  The
    // others take the general path, which derives each lane's address from scratch.
    const int lr = wave * 32 + (lane >> 3);                   // row / column of the tile for i = 0 (i adds 8)
    const int coff = ((lane & 3) ^ (lane >> 4)) * 16;         // byte offset of the lane's chunk inside its 32-k half
    const int h0 = (lane >> 2) & 1;                           // which half, for even i (odd i: the other one)
    const char* const a_base = uniform_ptr(reinterpret_cast<const char*>(INDEXED ? P.act : P.act + (int64_t)row0 * P.K));
    const char* const x_base = uniform_ptr(reinterpret_cast<const char*>(P.Sx + td.aoff) - (int64_t)nfull * 64);
    const char* const w_base = uniform_ptr(reinterpret_cast<const char*>(KN ? P.W + col0 : P.W + (int64_t)col0 * P.K));
    const char* const e_base = uniform_ptr(
        KN ? reinterpret_cast<const char*>(P.packed + (int64_t)td.roff_first * P.N + col0) - (int64_t)nfull * 64 * P.N
           : reinterpret_cast<const char*>(P.packed + (int64_t)col0 * P.ra + td.roff_first) - (int64_t)nfull * 64);
    const uint32_t lds0 = lds_addr(lds);
    // Interior tiles (no row / column clamping) need two offsets per operand: the lane's row and chunk for even
    // and for odd i; the 8 i rows between consecutive loads go into the uniform base.
    const bool interior_m = rows_valid == BM, interior_n = col0 + BN <= P.N;
    uint32_t k_off[2], x_off[2], kn_off[2];
#pragma unroll
    for (int par = 0; par < 2; ++par) {
      k_off[par] = (uint32_t)lr * (uint32_t)(P.K * 2) + coff + (h0 ^ par) * 64;       // rows of K elements: act, NT weight
      x_off[par] = INDEXED ? 0u : (uint32_t)lr * (uint32_t)(td.kext * 2) + coff + (h0 ^ par) * 64;   // rows of the adapter operand
      const int kl = wave * 8 + par * 2 + (lane >> 5);                                // forward weight: k-row of i = par
      const int c = (lane & 31) ^ ((kl & 3) << 2) ^ (((kl >> 3) & 1) << 1);
      kn_off[par] = KN ? (uint32_t)(kl & 31) * (uint32_t)(P.N * 2) + c * 16 : 0u;
    }
    // INDEXED: byte offset (from P.act) of the batch row behind each of the lane's four tile rows, chunk and half
    // included; rows beyond the problem edge repeat the last valid one
    uint32_t g_off[INDEXED ? 4 : 1];
    if (INDEXED) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
        g_off[i] = (uint32_t)P.in_index[row0 + min(lr + i * 8, rows_valid - 1)] * (uint32_t)(P.K * 2) + coff + (h0 ^ (i & 1)) * 64;
    }
    auto issue_act = [&](int slot, int tq) {                  // activation tile holding steps tq, tq + 1 (tq >= 0)
      const uint32_t dst = lds0 + slot * SLOT + wave * 4096;
      if (INDEXED && tq + 1 < nfull) {
        const char* const sb = a_base + (int64_t)tq * 64;
#pragma unroll
        for (int i = 0; i < 4; ++i) dma16s(g_off[i], sb, dst + i * 1024);
      } else if (!INDEXED && interior_m && tq + 1 < nfull) {
        const char* const sb = a_base + (int64_t)tq * 64;
#pragma unroll
        for (int i = 0; i < 4; ++i) dma16s(k_off[i & 1], uniform_ptr(sb + (int64_t)i * 16 * P.K), dst + i * 1024);
      } else if (!INDEXED && tq >= nfull && tq + 1 < ntot) {   // (INDEXED keeps no offsets for these few steps: general path)
        const char* const sb = x_base + (int64_t)tq * 64;
#pragma unroll
        for (int i = 0; i < 4; ++i) dma16s(x_off[i & 1], uniform_ptr(sb + (int64_t)i * 16 * td.kext), dst + i * 1024);
      } else {
        int r0 = lr;
        asm volatile("" : "+v"(r0));         // keep what this rare path derives out of the loop's live registers
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int r = r0 + i * 8;
          const int t = min(max(tq + (h0 ^ (i & 1)), 0), ntot - 1);
          const bool ext = t >= nfull;
          const uint32_t off = (ext ? (uint32_t)r * (uint32_t)(td.kext * 2)
                                : INDEXED ? g_off[i] - coff - (h0 ^ (i & 1)) * 64
                                          : (uint32_t)min(r, rows_valid - 1) * (uint32_t)(P.K * 2)) + t * 64 + coff;
          dma16((ext ? x_base : a_base) + off, dst + i * 1024);
        }
      }
    };
    auto issue_wgt = [&](int slot, int tq) {                  // weight tile holding steps tq, tq + 1
      const uint32_t dst = lds0 + slot * SLOT + wave * 4096;
      if (KN) {
        //  "kn16 tile": slot p -> k-row p / 32 (0..63), chunk (p % 32) ^ swizzle(k-row); a wave's rows all belong
        //  to one step, so base and step clamping are wave-uniform
        const int t = min(max(tq + (wave >> 2), 0), ntot - 1);
        const char* const sb = (t >= nfull ? e_base : w_base) + (int64_t)t * 64 * P.N;
        if (interior_n) {
#pragma unroll
          for (int i = 0; i < 4; ++i)
            dma16s(kn_off[i & 1], uniform_ptr(sb + (int64_t)(i >> 1) * 8 * P.N), dst + i * 1024);   // i / 2: 4 k-rows on
        } else {
          int ln = lane;
          asm volatile("" : "+v"(ln));
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int kl = wave * 8 + i * 2 + (ln >> 5);
            const int c = (ln & 31) ^ ((kl & 3) << 2) ^ (((kl >> 3) & 1) << 1);
            dma16(sb + (int64_t)(kl & 31) * (P.N * 2) + min(c * 16, (P.N - 8 - col0) * 2), dst + i * 1024);
          }
        }
      } else if (interior_n && tq >= 0 && tq + 1 < nfull) {
        const char* const sb = w_base + (int64_t)tq * 64;
#pragma unroll
        for (int i = 0; i < 4; ++i) dma16s(k_off[i & 1], uniform_ptr(sb + (int64_t)i * 16 * P.K), dst + i * 1024);
      } else {                                // the few adapter steps of the backward weight operand included
        int r0 = lr;
        asm volatile("" : "+v"(r0));
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int n = min(r0 + i * 8, P.N - 1 - col0);
          const int t = min(max(tq + (h0 ^ (i & 1)), 0), ntot - 1);
          const bool ext = t >= nfull;
          const uint32_t off = (uint32_t)n * (uint32_t)((ext ? P.ra : P.K) * 2) + t * 64 + coff;
          dma16((ext ? e_base : w_base) + off, dst + i * 1024);
        }
      }
    };
    // The two groups of four waves (one wave of each group per SIMD: waves w and w + 4 share a SIMD) run half a
    // step apart: while one group issues its 32 MFMAs of a step, the other reads its fragments of the next step
    // from LDS and issues its loads, so the MFMA pipe does not idle behind the burst of LDS reads that follows a
    // common barrier.  Every half step ends in a workgroup barrier; the late group passes one extra barrier
    // first, the early group one extra at the end.  Loads complete in order: with the 2 x 4 loads of the two
    // youngest tiles allowed in flight, everything older has landed, and after the barrier so has everyone
    // else's share.
    const bool late = (wave >> 2) != 0;
    auto gate = [&]() {
      __builtin_amdgcn_sched_barrier(0);
      __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(8));
      __builtin_amdgcn_s_barrier();
      __builtin_amdgcn_sched_barrier(0);
    };
    // step s (s % 10 == U): second half of L_s, first half of L_s+1; then L_s+4 goes into the slot L_s-1 left
    // Fragment addresses: one lane pattern for every k-contiguous tile (row l % 16 of a 16-row block, chunk
    // l / 16 under the row swizzle; the second 32-k half is the same address with bit 6 flipped, block i adds
    // 2048 bytes, the weight rows add a uniform constant) and four for the forward weight tile (one per feature
    // block: its chunk swizzle mixes with the block index).  The empty asm in each step makes the compiler
    // re-derive the per-slot addresses from these few registers instead of keeping all of them live.
    uint32_t pa0 = (wm * 128 + (lane & 15)) * 128 + (((lane >> 4) ^ ((lane & 15) >> 1)) << 4);
    const int wdelta = (wn * 64 - wm * 128) * 128;
    uint32_t pk[NFB];
#pragma unroll
    for (int j = 0; j < NFB; ++j) {
      const int sl = lane & 15, n = wn * 64 + j * 16 + (sl & 3) * 4;
      const int kb = (lane >> 4) * 8 + (sl >> 2);
      pk[j] = KN ? kn16_off(kb, n >> 3) + (n & 7) * 2 : 0;
    }
#define TLORA_GEMM_STEP(U, s)                                                                                \
  {                                                                                                          \
    constexpr int slA = ((U) & 1) ? (U) % 5 : ((U) + 1) % 5, slB = ((U) & 1) ? ((U) + 1) % 5 : (U) % 5;      \
    constexpr int hA = ((U) & 1) ? 1 : 0, hB = 1 - hA;                                                       \
    bf16x8 xf[8], wf[NFB];                                                                                   \
    asm volatile("" : "+v"(pa0));                                                                            \
    gate();                                  /* L_s, L_s+1 have landed for everyone; L_s-1 is no longer read */ \
    {                                                                                                        \
      const uint8_t* const fa = lds + slA * SLOT + (pa0 ^ (hA * 64));                                        \
      _Pragma("unroll") for (int i = 0; i < 8; ++i)                                                          \
        xf[i] = as_bf16x8(*reinterpret_cast<const u32x4*>(fa + i * 2048));                                   \
    }                                                                                                        \
    if (KN) {                                                                                                \
      _Pragma("unroll") for (int j = 0; j < NFB; ++j) {                                                      \
        asm volatile("" : "+v"(pk[j]));                                                                      \
        const uint8_t* const fw = lds + slB * SLOT + hB * 16384 + pk[j];                                     \
        s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, fw));                              \
        s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, fw + 2048));                       \
        typedef short s16x8_ __attribute__((ext_vector_type(8)));                                            \
        wf[j] = __builtin_bit_cast(bf16x8, (s16x8_)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7)); \
      }                                                                                                      \
    } else {                                                                                                 \
      const uint8_t* const fw = lds + slB * SLOT + ((pa0 + wdelta) ^ (hB * 64));                             \
      _Pragma("unroll") for (int j = 0; j < NFB; ++j)                                                        \
        wf[j] = as_bf16x8(*reinterpret_cast<const u32x4*>(fw + j * 2048));                                   \
    }                                                                                                        \
    if (((U) & 1)) issue_act(((U) + 4) % 5, (s) + 3); else issue_wgt(((U) + 4) % 5, (s) + 3);                \
    gate();                                  /* fragments are in registers */                              \
    mma_slice(xf, wf);                                                                                       \
  }
    issue_wgt(0, -1);
    issue_act(1, 0);
    issue_wgt(2, 1);
    issue_act(3, 2);
    if (late) gate();              // its share of L_0, L_1 must have landed before the early group reads them
    int s = 0;
    for (; s + 10 <= ntot; s += 10) {
      TLORA_GEMM_STEP(0, s)      TLORA_GEMM_STEP(1, s + 1)  TLORA_GEMM_STEP(2, s + 2)  TLORA_GEMM_STEP(3, s + 3)
      TLORA_GEMM_STEP(4, s + 4)  TLORA_GEMM_STEP(5, s + 5)  TLORA_GEMM_STEP(6, s + 6)  TLORA_GEMM_STEP(7, s + 7)
      TLORA_GEMM_STEP(8, s + 8)  TLORA_GEMM_STEP(9, s + 9)
    }
    if (s + 0 < ntot) TLORA_GEMM_STEP(0, s)
    if (s + 1 < ntot) TLORA_GEMM_STEP(1, s + 1)
    if (s + 2 < ntot) TLORA_GEMM_STEP(2, s + 2)
    if (s + 3 < ntot) TLORA_GEMM_STEP(3, s + 3)
    if (s + 4 < ntot) TLORA_GEMM_STEP(4, s + 4)
    if (s + 5 < ntot) TLORA_GEMM_STEP(5, s + 5)
    if (s + 6 < ntot) TLORA_GEMM_STEP(6, s + 6)
    if (s + 7 < ntot) TLORA_GEMM_STEP(7, s + 7)
    if (s + 8 < ntot) TLORA_GEMM_STEP(8, s + 8)
#undef TLORA_GEMM_STEP
    __builtin_amdgcn_sched_barrier(0);
    if (!late) __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_s_waitcnt(0x0070);     // vmcnt(0): the trailing loads must not land in reused LDS
  }
  if (clocked && tid == 0) {
    atomicAdd(&P.clk[0], __builtin_readcyclecounter() - cyc0);        // integer sums: order does not matter
    atomicAdd(&P.clk[1], __builtin_amdgcn_s_memrealtime() - tick0);
  }

  // ---- K tail (K % 32 != 0): one register-staged, zero-padded step through slot 0 (activation rows as 64-byte
  // rows in its first 16 KB, the weight slice behind them) --------------------------------------------------
  if (KTAIL) {
    const int k0 = nfull * 32, kvalid = P.K - k0;
    constexpr int TCH = 1024 / NT;          // 16-byte chunks per thread and tile
    u32x4 areg[TCH], breg[TCH];
#pragma unroll
    for (int i = 0; i < TCH; ++i) {
      const int id = tid + i * NT, r = id >> 2, c = id & 3;
      const bool ok = r < rows_valid && c * 8 < kvalid;
      const int64_t arow = INDEXED ? (int64_t)P.in_index[row0 + min(r, rows_valid - 1)] : (int64_t)(row0 + r);
      areg[i] = ok ? ldg16(P.act + arow * P.K + k0 + c * 8) : u32x4{0, 0, 0, 0};
      if (KN) {
        const int k = id >> 5, cc = id & 31;
        const bool okb = k < kvalid && col0 + cc * 8 < P.N;
        breg[i] = okb ? ldg16(P.W + (int64_t)(k0 + k) * P.N + col0 + cc * 8) : u32x4{0, 0, 0, 0};
      } else {
        const bool okb = col0 + r < P.N && c * 8 < kvalid;
        breg[i] = okb ? ldg16(P.W + (int64_t)(col0 + r) * P.K + k0 + c * 8) : u32x4{0, 0, 0, 0};
      }
    }
    __syncthreads();                       // every wave is done reading the slots
#pragma unroll
    for (int i = 0; i < TCH; ++i) {
      const int id = tid + i * NT;
      *reinterpret_cast<u32x4*>(sl0 + row32_off(id >> 2, id & 3)) = areg[i];
      if (KN) *reinterpret_cast<u32x4*>(sl0 + 16384 + kn16_off(id >> 5, id & 31)) = breg[i];
      else    *reinterpret_cast<u32x4*>(sl0 + 16384 + row32_off(id >> 2, id & 3)) = breg[i];
    }
    __syncthreads();
    {                                       // chunks and k-rows beyond kvalid were stored as zeros
      bf16x8 xf[8], wf[NFB];
#pragma unroll
      for (int i = 0; i < 8; ++i) xf[i] = frag16_rows<32>(sl0, wm * 128 + i * 16, 0, lane);
#pragma unroll
      for (int j = 0; j < NFB; ++j)
        wf[j] = KN ? frag16_kn(sl0 + 16384, wn * 64 + j * 16, 0, lane)
                   : frag16_rows<32>(sl0 + 16384, wn * 64 + j * 16, 0, lane);
      mma_slice(xf, wf);
    }
  }

  // ---- epilogue: accumulators -> bf16 -> LDS (slots 0-3 hold 64 output rows each, 512 B per row, 16-byte
  // chunk c of row R at slot c ^ (R & 31)) -> full 512-byte rows to global memory. -----------------------------
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    // lane l holds token (l % 16) of block i, features 4 (l / 16) .. + 3 of each feature block
    uint8_t* const obuf = wm ? (i < 4 ? sl2 : sl3) : (i < 4 ? sl0 : sl1);
    const int R = wm * 128 + i * 16 + (lane & 15);
    uint8_t* const orow = obuf + (R & 63) * 512 + ((lane >> 4) & 1) * 8;
#pragma unroll
    for (int j = 0; j < NFB; ++j) {
      const int c = wn * 8 + j * 2 + (lane >> 5);
      u32x2 v = {pack_bf16x2(acc[j][i][0], acc[j][i][1]), pack_bf16x2(acc[j][i][2], acc[j][i][3])};
      *reinterpret_cast<u32x2*>(orow + ((c ^ (R & 31)) << 4)) = v;
    }
  }
  __syncthreads();
  constexpr int RPI = NT / 32;              // output rows per iteration
#pragma unroll
  for (int it = 0; it < 256 / RPI; ++it) {
    const uint8_t* const obuf = it * RPI < 64 ? sl0 : it * RPI < 128 ? sl1 : it * RPI < 192 ? sl2 : sl3;
    const int R = (tid >> 5) + it * RPI, c = tid & 31;
    const u32x4 v = *reinterpret_cast<const u32x4*>(obuf + (R & 63) * 512 + ((c ^ (R & 31)) << 4));
    if (R < rows_valid && col0 + c * 8 < P.N) {
      const int64_t orow = P.out_index ? P.out_index[row0 + R] : row0 + R;
      *reinterpret_cast<u32x4*>(P.out + orow * P.N + col0 + c * 8) = v;
    }
  }
}

void launch_seg_gemm(bool w_is_kn, const TileDev* tiles, const uint16_t* act, const uint16_t* W, const uint16_t* Sx,
                     const uint16_t* packed, int r_total, uint16_t* out, const int32_t* out_index,
                     const int32_t* in_index, int T, int K, int N, unsigned long long* clk, hipStream_t st) {
  GemmParams P;
  P.clk = clk;
  P.out_index = out_index;
  P.in_index = in_index;
  P.tiles = tiles;  P.act = act;  P.W = W;  P.Sx = Sx;  P.packed = packed;  P.out = out;
  P.T = T;  P.K = K;  P.N = N;  P.ra = r_total + 32;
  P.tiles_m = (T + kGemmBM - 1) / kGemmBM;
  P.tiles_n = (N + kGemmBN - 1) / kGemmBN;
  const int nb = P.tiles_m * P.tiles_n;
  if (nb == 0) return;
  const bool tail = K % kGemmBK != 0;
#define TLORA_GEMM_LAUNCH(KN, TAIL, IDX) \
  hipLaunchKernelGGL((seg_gemm_kernel<KN, TAIL, IDX>), dim3(nb), dim3(512), 0, st, P)
  if (in_index) {
    if (w_is_kn) { if (tail) TLORA_GEMM_LAUNCH(true, true, true);  else TLORA_GEMM_LAUNCH(true, false, true); }
    else         { if (tail) TLORA_GEMM_LAUNCH(false, true, true); else TLORA_GEMM_LAUNCH(false, false, true); }
  } else {
    if (w_is_kn) { if (tail) TLORA_GEMM_LAUNCH(true, true, false);  else TLORA_GEMM_LAUNCH(true, false, false); }
    else         { if (tail) TLORA_GEMM_LAUNCH(false, true, false); else TLORA_GEMM_LAUNCH(false, false, false); }
  }
#undef TLORA_GEMM_LAUNCH
}

// ---------------------------------------------------------------------------------------------------
// dA / dB:  G_j[p, c] = scale_j * sum_{t in seg j} U_j[t, p] * V[t, c]
//   dB_j: U = S_j, V = dY;   dA_j^T: U = dS_j, V = X.   U comes as two bf16 planes hi + lo (two MFMAs keep ~16
//   mantissa bits of the fp32 intermediate), packed [T_j padded to 32, rpad_j] with zero pad rows.
// The contraction runs over tokens, the row index of both operands, so both are staged in LDS as they lie
// in memory (token-major) and read through the transposing LDS read.  One workgroup (8 waves) owns
// kGradCols = 256 feature columns x 32*MB rank rows for a chunk of tokens, so V is read from memory once for all
// rank rows; a wave takes 64 columns and every other rank block.  Per step of 32 tokens a stage holds the V tile (32 x 256, 16 KB) and
// the two U tiles (32 x 32*MB); four stages are filled by asynchronous global->LDS loads three steps
// ahead.  V rows beyond the chunk are clamped to its last row: they meet the zero pad rows of U.
// ---------------------------------------------------------------------------------------------------
__device__ __forceinline__ bf16x8 frag_tr_u(const uint8_t* plane, int pitch, int sw_shift, int sw_mask, int nb, int kk,
                                            int lane) {
  const int s = lane & 15;
  const int n = nb + ((lane >> 4) & 1) * 16 + (s & 3) * 4;     // rank column this lane addresses
  const int k = kk * 16 + (lane >> 5) * 8 + (s >> 2);          // k and k + 4 share the swizzle term
  const int c = (n >> 3) ^ (((k >> sw_shift) & sw_mask) << 2);
  const uint8_t* a = plane + k * pitch + (c << 4) + (n & 7) * 2;
  s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, a));
  s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, a + 4 * pitch));
  typedef short s16x8 __attribute__((ext_vector_type(8)));
  s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, v);
}

// Eight waves: wave w owns the 64 feature columns of group (w % 4) and the rank blocks (w / 4), (w / 4) + 2 of the
// unit's up to four.  A CU runs one workgroup (the stages fill most of its LDS); with two waves per SIMD the fragment
// reads of one overlap the MFMAs of the other, and a 128-rank unit's 32 MFMAs and 20 KB of reads per step are split
// over two waves (with four waves such a unit took about twice as long per byte as a low-rank one, and the slowest
// units of the one-round launch set its duration).
// INDEXED: the rows of V are fetched through row_index (token-indexed calls).  A separate instantiation, so that the
// plain one carries no trace of it: even a branch around a memory load inside the load loop would make the compiler
// wait, where the paths merge, for every asynchronous load in flight.
template <bool INDEXED>
__global__ void __launch_bounds__(512) rank_grad_kernel(const JobDev* __restrict__ jobs,
                                                        const GradUnit* __restrict__ units,
                                                        const uint16_t* __restrict__ Uhi,
                                                        const uint16_t* __restrict__ Ulo,
                                                        const uint16_t* __restrict__ V, int D,
                                                        float* __restrict__ partial,
                                                        const int32_t* __restrict__ row_index) {
  constexpr int MB = kGradMaxBlocks;                        // the U tile always has room for 4 blocks of 32 ranks;
  constexpr int RP = kGradRanks * MB;                       // a unit multiplies only its u.mb live ones
  constexpr int UPITCH = 2 * RP;                            // 256 bytes per token row of a U tile
  // 16-byte chunk c of token row k sits at slot c ^ ((k & 3) << 2) so that the four rows one transposing read
  // touches start in four distinct 64-byte bank groups
  constexpr int SW_SHIFT = 0;
  constexpr int SW_MASK = 3;
  constexpr int UPLANE = kGradStep * UPITCH;                // 2 KB * MB
  constexpr int VTILE = kGradStep * kGradCols * 2;          // 16 KB
  constexpr int WAVES = 8;
  constexpr int V_LD = VTILE / 1024 / WAVES;                // 2 loads per wave: V tile
  constexpr int U_LD = 2 * UPLANE / 1024 / WAVES;           // 2 loads per wave: hi and lo planes of U
  constexpr int LOADS = V_LD + U_LD;                        // asynchronous loads per wave per step
  constexpr int MW = MB / 2;                                // rank blocks per wave
  static_assert(V_LD * WAVES * 1024 == VTILE && U_LD * WAVES * 1024 == 2 * UPLANE && MB == 4, "load split over the waves");
  __shared__ __attribute__((aligned(1024))) uint8_t g0[VTILE];
  __shared__ __attribute__((aligned(1024))) uint8_t g1[VTILE];
  __shared__ __attribute__((aligned(1024))) uint8_t g2[VTILE];
  __shared__ __attribute__((aligned(1024))) uint8_t g3[VTILE];
  __shared__ __attribute__((aligned(1024))) uint8_t h0[2 * UPLANE];
  __shared__ __attribute__((aligned(1024))) uint8_t h1[2 * UPLANE];
  __shared__ __attribute__((aligned(1024))) uint8_t h2[2 * UPLANE];
  __shared__ __attribute__((aligned(1024))) uint8_t h3[2 * UPLANE];
  // token-indexed calls: where in the batch each token row of the unit lies (row_index of the unit's chunk, staged
  // once so that the load loop never waits for an index from memory; a unit has at most kGradMaxTokens tokens)
  __shared__ int32_t srow[INDEXED ? kGradMaxTokens : 1];

  const GradUnit u = units[blockIdx.x];
  const JobDev jb = jobs[u.job];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int cg = wave & 3, rh = wave >> 2;                  // column group, rank half
  const int col0 = u.cb * kGradCols;
  const int pbase = u.pb * RP;
  const int nsteps = (u.t1 - u.t0 + kGradStep - 1) / kGradStep;

  f32x16 acc[MW][2];
#pragma unroll
  for (int m = 0; m < MW; ++m)
#pragma unroll
    for (int n = 0; n < 2; ++n)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[m][n][e] = 0.f;

  // V tile [32 tokens][512 B], same swizzle as the GEMM's weight tile: lane -> (token k, chunk c)
  int vk[V_LD], vcol[V_LD];
#pragma unroll
  for (int i = 0; i < V_LD; ++i) {
    const int p = (wave * V_LD + i) * 64 + lane;
    vk[i] = p >> 5;
    const int c = (p & 31) ^ ((vk[i] & 3) << 2);
    vcol[i] = min(col0 + c * 8, D - 8);               // columns beyond D are clamped; their results are not stored
  }
  // U tiles: hi plane then lo plane, 2 * MB KB each = 2 * MB wave-loads; wave w issues loads q = w * U_LD + i of the
  // 4 * MB.  Lanes whose rank chunk lies beyond rpad fetch nothing: the stale slots only feed rank rows >= rpad
  // of the tile, which are never stored.
  const uint16_t* usrc[U_LD];
  int udst[U_LD];
  bool ulive[U_LD];
#pragma unroll
  for (int i = 0; i < U_LD; ++i) {
    const int q = wave * U_LD + i;                    // 0 .. 4 MB - 1
    const int plane = q / (2 * MB), within = q % (2 * MB);
    const int slot = within * 64 + lane;              // 16-byte slot inside the plane
    const int k = slot / (RP / 8), cphys = slot % (RP / 8);
    const int c = cphys ^ (((k >> SW_SHIFT) & SW_MASK) << 2);
    ulive[i] = pbase + c * 8 < jb.rpad || lane == 0;    // lane 0 keeps every wave's load count the same
    const int p = min(pbase + c * 8, jb.rpad - 8);
    usrc[i] = (plane ? Ulo : Uhi) + jb.soff + (int64_t)(u.t0 - jb.row0 + k) * jb.rpad + p;
    udst[i] = plane * UPLANE + within * 1024;
  }
  if (INDEXED) {
    for (int i = tid; i < min(u.t1 - u.t0, kGradMaxTokens); i += WAVES * 64) srow[i] = row_index[u.t0 + i];
    __syncthreads();
  }
  int f_step = 0;                                     // next step to fetch
  auto issue = [&](uint8_t* S, uint8_t* H) {
    const int st = min(f_step, nsteps - 1);           // trailing issues re-load the last step (uniform load count)
    const uint32_t sbase = lds_addr(S + wave * (V_LD * 1024)), hbase = lds_addr(H);
#pragma unroll
    for (int i = 0; i < V_LD; ++i) {
      int t = min(u.t0 + st * kGradStep + vk[i], u.t1 - 1);
      if (INDEXED) t = srow[min(t - u.t0, kGradMaxTokens - 1)];
      dma16(V + (int64_t)t * D + vcol[i], sbase + i * 1024);
    }
#pragma unroll
    for (int i = 0; i < U_LD; ++i)
      if (ulive[i]) dma16(usrc[i] + (int64_t)st * kGradStep * jb.rpad, hbase + __builtin_amdgcn_readfirstlane(udst[i]));
    ++f_step;
  };
  auto compute = [&](const uint8_t* S, const uint8_t* H) {
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
      bf16x8 vf[2];
#pragma unroll
      for (int n = 0; n < 2; ++n) vf[n] = frag_kn_tile(S, cg * 64 + n * 32, kk, lane);
#pragma unroll
      for (int i = 0; i < MW; ++i) {
        const int m = rh + 2 * i;
        if (m < u.mb) {
          const bf16x8 hi = frag_tr_u(H, UPITCH, SW_SHIFT, SW_MASK, m * 32, kk, lane);
          const bf16x8 lo = frag_tr_u(H + UPLANE, UPITCH, SW_SHIFT, SW_MASK, m * 32, kk, lane);
#pragma unroll
          for (int n = 0; n < 2; ++n) {
            acc[i][n] = mfma32(hi, vf[n], acc[i][n]);
            acc[i][n] = mfma32(lo, vf[n], acc[i][n]);
          }
        }
      }
    }
  };
  auto landed = [&]() {
    // loads complete in order: all but those of the two youngest steps have landed
    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(2 * LOADS));
    __builtin_amdgcn_s_barrier();
  };
  if (nsteps > 0) {
    issue(g0, h0);
    issue(g1, h1);
    issue(g2, h2);
    int kt = 0;
    for (; kt + 4 <= nsteps; kt += 4) {
      landed();  issue(g3, h3);  compute(g0, h0);
      landed();  issue(g0, h0);  compute(g1, h1);
      landed();  issue(g1, h1);  compute(g2, h2);
      landed();  issue(g2, h2);  compute(g3, h3);
    }
    if (kt < nsteps)     { landed();  issue(g3, h3);  compute(g0, h0); }
    if (kt + 1 < nsteps) { landed();  issue(g0, h0);  compute(g1, h1); }
    if (kt + 2 < nsteps) { landed();  issue(g1, h1);  compute(g2, h2); }
    __builtin_amdgcn_s_waitcnt(0x0070);   // drain the trailing loads before the workgroup's LDS is released
  }

  // partial tile [32 * u.mb][256]: lane holds column (lane % 32) of its n-block and 16 rank rows per m-block
  float* out = partial + u.part_off;
#pragma unroll
  for (int i = 0; i < MW; ++i) {
    const int m = rh + 2 * i;
    if (m < u.mb) {
#pragma unroll
      for (int n = 0; n < 2; ++n)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int pl = m * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
          out[pl * kGradCols + cg * 64 + n * 32 + (lane & 31)] = acc[i][n][e];
        }
    }
  }
}

void launch_rank_grad(const JobDev* jobs, const GradUnit* units, int num_units, const uint16_t* U_hi,
                      const uint16_t* U_lo, const uint16_t* V, int D, float* partial, const int32_t* row_index,
                      hipStream_t st) {
  if (num_units == 0) return;
  if (row_index)
    hipLaunchKernelGGL(rank_grad_kernel<true>, dim3(num_units), dim3(512), 0, st, jobs, units, U_hi, U_lo, V, D, partial,
                       row_index);
  else
    hipLaunchKernelGGL(rank_grad_kernel<false>, dim3(num_units), dim3(512), 0, st, jobs, units, U_hi, U_lo, V, D,
                       partial, row_index);
}

// Sum the partial tiles of one output tile in unit order, scale, and store (dB_j row-major [r, D];
// dA_j is the transpose of the computed tile: [D, r]).  One thread per column; a workgroup takes the slabs of 4 rank
// rows blockIdx.y, blockIdx.y + kReduceSplit, ... of its group's 256 columns (a grid over all 32 possible slabs
// would consist mostly of workgroups that find their slab beyond the job's rank).  The partial tiles are read row
// by row (coalesced across the threads); dB rows are stored the same way, dA as 16 bytes per thread and slab.
constexpr int kReduceSplit = 8;
__global__ void __launch_bounds__(256) grad_reduce_kernel(const JobDev* __restrict__ jobs,
                                                          const GradGroup* __restrict__ groups,
                                                          const float* __restrict__ partial, int D, int out_is_dA,
                                                          int accumulate) {
  const GradGroup g = groups[blockIdx.x];
  const JobDev jb = jobs[g.job];
  const int c = g.cb * kGradCols + threadIdx.x;
  const int tile_rows = g.mb * kGradRanks;                 // live rows of this tile
  const int pb_rows = kGradMaxBlocks * kGradRanks;         // rank rows per rank block
  const int live = min(tile_rows, jb.rank - g.pb * pb_rows);   // rows of the tile that exist in the job
  if (c >= D) return;
  const int64_t tile_elems = (int64_t)tile_rows * kGradCols;
  float* dst = static_cast<float*>(out_is_dA ? jb.dA : jb.dB);
  const bool vec = out_is_dA && (jb.rank & 3) == 0 && (reinterpret_cast<uintptr_t>(dst) & 15) == 0;
  for (int pl0 = blockIdx.y * 4; pl0 < live; pl0 += 4 * kReduceSplit) {
    const float* src = partial + g.part_off + (int64_t)pl0 * kGradCols + threadIdx.x;
    float s[4] = {0.f, 0.f, 0.f, 0.f};
    for (int k = 0; k < g.nunits; ++k) {          // fixed order: bit-reproducible
#pragma unroll
      for (int i = 0; i < 4; ++i) s[i] += src[k * tile_elems + i * kGradCols];
    }
    const int p0 = g.pb * pb_rows + pl0;
    if (vec) {                                    // rank % 4 == 0: the slab's 4 rows all exist
      f32x4 v = {s[0] * jb.scale, s[1] * jb.scale, s[2] * jb.scale, s[3] * jb.scale};
      f32x4* const q = reinterpret_cast<f32x4*>(dst + (int64_t)c * jb.rank + p0);
      if (accumulate) { const f32x4 o = *q;  v = f32x4{o[0] + v[0], o[1] + v[1], o[2] + v[2], o[3] + v[3]}; }
      *q = v;
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int p = p0 + i;
        if (p < jb.rank) {
          float* const d = out_is_dA ? dst + (int64_t)c * jb.rank + p : dst + (int64_t)p * D + c;
          const float v = s[i] * jb.scale;
          *d = accumulate ? *d + v : v;
        }
      }
    }
  }
}

void launch_grad_reduce(const JobDev* jobs, const GradGroup* groups, int num_groups, const float* partial, int D,
                        bool out_is_dA, bool accumulate, hipStream_t st) {
  if (num_groups == 0) return;
  hipLaunchKernelGGL(grad_reduce_kernel, dim3(num_groups, kReduceSplit), dim3(256), 0, st, jobs, groups, partial, D,
                     out_is_dA ? 1 : 0, accumulate ? 1 : 0);
}

// ---------------------------------------------------------------------------------------------------
// fp32 configuration: strided products C (+)= alpha * A.B, 64 x 64 tile per workgroup.  Operands and
// results are fp32; the running sums are kept in fp64 so that long token reductions (dA, dB) stay
// within 1e-5 of the exact value even where the result is close to zero.
// ---------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) f32_units_kernel(const F32Unit* __restrict__ units,
                                                        const F32Tile* __restrict__ tiles) {
  __shared__ float As[16][65];
  __shared__ float Bs[16][65];
  const F32Tile t = tiles[blockIdx.x];
  const F32Unit u = units[t.unit];
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int m0 = t.tm * 64, n0 = t.tn * 64;
  double acc[4][4] = {};
  for (int k0 = 0; k0 < u.K; k0 += 16) {
    for (int i = threadIdx.x; i < 16 * 64; i += 256) {
      const int kk = i & 15, mm = i >> 4;             // A tile: 64 rows x 16 k
      const int m = m0 + mm, k = k0 + kk;
      As[kk][mm] = (m < u.M && k < u.K) ? u.A[(int64_t)m * u.a_rs + (int64_t)k * u.a_cs] : 0.f;
      const int nn = i & 63, kb = i >> 6;             // B tile: 16 k x 64 cols
      const int n = n0 + nn, k2 = k0 + kb;
      Bs[kb][nn] = (n < u.N && k2 < u.K) ? u.B[(int64_t)k2 * u.b_rs + (int64_t)n * u.b_cs] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_fma((double)a[i], (double)b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
      if (m < u.M && n < u.N) {
        float* c = u.C + (int64_t)m * u.c_rs + n;
        const double v = (double)u.alpha * acc[i][j];
        *c = (float)(u.accumulate ? (double)*c + v : v);
      }
    }
}

void launch_f32_units(const F32Unit* units, const F32Tile* tiles, int num_tiles, hipStream_t st) {
  if (num_tiles == 0) return;
  hipLaunchKernelGGL(f32_units_kernel, dim3(num_tiles), dim3(256), 0, st, units, tiles);
}

// ---------------------------------------------------------------------------------------------------
// Per-job optimizer step (AdamW with decoupled weight decay) over a table of tensors: blockIdx.y = tensor,
// blockIdx.x = chunk of 4096 elements.  fp32 arithmetic on the fp32 master copy; the tensor the layer reads is
// rewritten from it (round-to-nearest-even for bf16).  Reads 16 and writes 14 (bf16) bytes per element.
// ---------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) adamw_kernel(const AdamwDev* __restrict__ tensors) {
  const AdamwDev t = tensors[blockIdx.y];
  const int64_t base = (int64_t)blockIdx.x * 4096;
  if (base >= t.n) return;
  float* const wsrc = t.master ? t.master : static_cast<float*>(t.param);
#pragma unroll 4
  for (int k = 0; k < 16; ++k) {
    const int64_t i = base + k * 256 + threadIdx.x;
    if (i >= t.n) break;
    const float g = t.grad[i];
    const float m = t.beta1 * t.m[i] + (1.f - t.beta1) * g;
    const float v = t.beta2 * t.v[i] + (1.f - t.beta2) * g * g;
    const float w0 = wsrc[i];
    const float w = w0 - t.lr * ((m * t.c1) / (sqrtf(v * t.c2) + t.eps) + t.weight_decay * w0);
    t.m[i] = m;
    t.v[i] = v;
    wsrc[i] = w;
    if (t.param_is_bf16) {
      static_cast<uint16_t*>(t.param)[i] = (uint16_t)(pack_bf16x2(w, 0.f) & 0xffffu);
    } else if (t.master) {
      static_cast<float*>(t.param)[i] = w;
    }
  }
}

void launch_adamw(const AdamwDev* tensors, int count, int64_t max_n, hipStream_t st) {
  if (count == 0 || max_n == 0) return;
  hipLaunchKernelGGL(adamw_kernel, dim3((unsigned)((max_n + 4095) / 4096), count), dim3(256), 0, st, tensors);
}

// ---------------------------------------------------------------------------------------------------
// Glue of the MLP block around the three fused projections: RMSNorm, gated SiLU, residual.  All HBM-bound,
// 16-byte accesses, fp32 arithmetic; BF = tensors are bf16 (else fp32).  8 elements per lane and access.
// ---------------------------------------------------------------------------------------------------
template <bool BF>
__device__ __forceinline__ void load8(const void* p, int64_t i, float (&v)[8]) {
  if (BF) {
    const u32x4 r = *reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(p) + i);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      v[2 * e] = __builtin_bit_cast(float, r[e] << 16);
      v[2 * e + 1] = __builtin_bit_cast(float, r[e] & 0xffff0000u);
    }
  } else {
    const f32x4* f = reinterpret_cast<const f32x4*>(static_cast<const float*>(p) + i);
    const f32x4 a = f[0], b = f[1];
#pragma unroll
    for (int e = 0; e < 4; ++e) { v[e] = a[e];  v[4 + e] = b[e]; }
  }
}
template <bool BF>
__device__ __forceinline__ void store8(void* p, int64_t i, const float (&v)[8]) {
  if (BF) {
    *reinterpret_cast<u32x4*>(static_cast<uint16_t*>(p) + i) =
        u32x4{pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7])};
  } else {
    f32x4* f = reinterpret_cast<f32x4*>(static_cast<float*>(p) + i);
    f[0] = f32x4{v[0], v[1], v[2], v[3]};
    f[1] = f32x4{v[4], v[5], v[6], v[7]};
  }
}
// sum over the 256 threads of a workgroup (every thread gets the total)
__device__ __forceinline__ float block_sum(float x, float* red) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = x;
  __syncthreads();
  const float t = red[0] + red[1] + red[2] + red[3];
  __syncthreads();
  return t;
}

// Xn[t, :] = X[t, :] * rstd_t * gamma,  rstd_t = 1 / sqrt(mean(X[t, :]^2) + eps).  One workgroup per row.
template <bool BF>
__global__ void __launch_bounds__(256) rmsnorm_fwd_kernel(const void* __restrict__ X, const void* __restrict__ gamma,
                                                          float eps, int d, void* __restrict__ Xn,
                                                          float* __restrict__ rstd) {
  __shared__ float red[4];
  const int64_t row = (int64_t)blockIdx.x * d;
  float ss = 0.f;
  for (int c = threadIdx.x * 8; c < d; c += 2048) {
    float v[8];
    load8<BF>(X, row + c, v);
#pragma unroll
    for (int e = 0; e < 8; ++e) ss += v[e] * v[e];
  }
  const float r = 1.0f / sqrtf(block_sum(ss, red) / (float)d + eps);
  if (threadIdx.x == 0) rstd[blockIdx.x] = r;
  for (int c = threadIdx.x * 8; c < d; c += 2048) {
    float v[8], g[8];
    load8<BF>(X, row + c, v);
    load8<BF>(gamma, c, g);
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = v[e] * r * g[e];
    store8<BF>(Xn, row + c, v);
  }
}

// dX[t, :] = dOut[t, :] + rstd_t * gd - X[t, :] * rstd_t^3 * sum(gd * X[t, :]) / d,   gd = (dXa + dXb) * gamma
template <bool BF>
__global__ void __launch_bounds__(256) rmsnorm_bwd_kernel(const void* __restrict__ X, const void* __restrict__ gamma,
                                                          const float* __restrict__ rstd, const void* __restrict__ dXa,
                                                          const void* __restrict__ dXb, const void* __restrict__ dXc,
                                                          const void* __restrict__ dOut, int d, void* __restrict__ dX) {
  __shared__ float red[4];
  const int64_t row = (int64_t)blockIdx.x * d;
  float dot = 0.f;
  for (int c = threadIdx.x * 8; c < d; c += 2048) {
    float x[8], a[8], b[8], g[8];
    load8<BF>(X, row + c, x);  load8<BF>(dXa, row + c, a);  load8<BF>(dXb, row + c, b);  load8<BF>(gamma, c, g);
    if (dXc) {
      float cc[8];
      load8<BF>(dXc, row + c, cc);
#pragma unroll
      for (int e = 0; e < 8; ++e) a[e] = a[e] + b[e] + cc[e], b[e] = 0.f;
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) dot += (a[e] + b[e]) * g[e] * x[e];
  }
  const float r = rstd[blockIdx.x];
  const float k = block_sum(dot, red) * r * r * r / (float)d;
  for (int c = threadIdx.x * 8; c < d; c += 2048) {
    float x[8], a[8], b[8], g[8], o[8];
    load8<BF>(X, row + c, x);  load8<BF>(dXa, row + c, a);  load8<BF>(dXb, row + c, b);  load8<BF>(gamma, c, g);
    load8<BF>(dOut, row + c, o);
    if (dXc) {
      float cc[8];
      load8<BF>(dXc, row + c, cc);
#pragma unroll
      for (int e = 0; e < 8; ++e) a[e] = a[e] + b[e] + cc[e], b[e] = 0.f;
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = o[e] + r * (a[e] + b[e]) * g[e] - x[e] * k;
    store8<BF>(dX, row + c, o);
  }
}

// Z = silu(G) * U            (n8 = number of 8-element chunks)
template <bool BF>
__global__ void __launch_bounds__(256) swiglu_fwd_kernel(const void* __restrict__ G, const void* __restrict__ U,
                                                         void* __restrict__ Z, int64_t n8) {
  const int64_t stride = (int64_t)gridDim.x * 256;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n8; i += stride) {
    float g[8], u[8];
    load8<BF>(G, i * 8, g);  load8<BF>(U, i * 8, u);
#pragma unroll
    for (int e = 0; e < 8; ++e) g[e] = g[e] / (1.0f + expf(-g[e])) * u[e];
    store8<BF>(Z, i * 8, g);
  }
}
// dU = dZ * silu(G),  dG = dZ * U * sig (1 + G (1 - sig)),  sig = 1 / (1 + exp(-G))
template <bool BF>
__global__ void __launch_bounds__(256) swiglu_bwd_kernel(const void* __restrict__ G, const void* __restrict__ U,
                                                         const void* __restrict__ dZ, void* __restrict__ dG,
                                                         void* __restrict__ dU, int64_t n8) {
  const int64_t stride = (int64_t)gridDim.x * 256;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n8; i += stride) {
    float g[8], u[8], z[8], dg[8], du[8];
    load8<BF>(G, i * 8, g);  load8<BF>(U, i * 8, u);  load8<BF>(dZ, i * 8, z);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float sig = 1.0f / (1.0f + expf(-g[e]));
      du[e] = z[e] * g[e] * sig;
      dg[e] = z[e] * u[e] * sig * (1.0f + g[e] * (1.0f - sig));
    }
    store8<BF>(dG, i * 8, dg);  store8<BF>(dU, i * 8, du);
  }
}
// Out = X + D
template <bool BF>
__global__ void __launch_bounds__(256) residual_add_kernel(const void* __restrict__ X, const void* __restrict__ D,
                                                           void* __restrict__ Out, int64_t n8) {
  const int64_t stride = (int64_t)gridDim.x * 256;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n8; i += stride) {
    float x[8], y[8];
    load8<BF>(X, i * 8, x);  load8<BF>(D, i * 8, y);
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] += y[e];
    store8<BF>(Out, i * 8, x);
  }
}

static unsigned ew_blocks(int64_t n8) { return (unsigned)std::min<int64_t>((n8 + 255) / 256, 256 * 32); }

void launch_rmsnorm_fwd(bool bf16, const void* X, const void* gamma, float eps, int T, int d, void* Xn, float* rstd,
                        hipStream_t st) {
  if (T == 0) return;
  if (bf16) hipLaunchKernelGGL(rmsnorm_fwd_kernel<true>, dim3(T), dim3(256), 0, st, X, gamma, eps, d, Xn, rstd);
  else      hipLaunchKernelGGL(rmsnorm_fwd_kernel<false>, dim3(T), dim3(256), 0, st, X, gamma, eps, d, Xn, rstd);
}
void launch_rmsnorm_bwd(bool bf16, const void* X, const void* gamma, const float* rstd, const void* dXa,
                        const void* dXb, const void* dXc, const void* dOut, int T, int d, void* dX, hipStream_t st) {
  if (T == 0) return;
  if (bf16) hipLaunchKernelGGL(rmsnorm_bwd_kernel<true>, dim3(T), dim3(256), 0, st, X, gamma, rstd, dXa, dXb, dXc, dOut, d, dX);
  else      hipLaunchKernelGGL(rmsnorm_bwd_kernel<false>, dim3(T), dim3(256), 0, st, X, gamma, rstd, dXa, dXb, dXc, dOut, d, dX);
}
void launch_swiglu_fwd(bool bf16, const void* G, const void* U, void* Z, int64_t n, hipStream_t st) {
  if (n == 0) return;
  if (bf16) hipLaunchKernelGGL(swiglu_fwd_kernel<true>, dim3(ew_blocks(n / 8)), dim3(256), 0, st, G, U, Z, n / 8);
  else      hipLaunchKernelGGL(swiglu_fwd_kernel<false>, dim3(ew_blocks(n / 8)), dim3(256), 0, st, G, U, Z, n / 8);
}
void launch_swiglu_bwd(bool bf16, const void* G, const void* U, const void* dZ, void* dG, void* dU, int64_t n,
                       hipStream_t st) {
  if (n == 0) return;
  if (bf16) hipLaunchKernelGGL(swiglu_bwd_kernel<true>, dim3(ew_blocks(n / 8)), dim3(256), 0, st, G, U, dZ, dG, dU, n / 8);
  else      hipLaunchKernelGGL(swiglu_bwd_kernel<false>, dim3(ew_blocks(n / 8)), dim3(256), 0, st, G, U, dZ, dG, dU, n / 8);
}
void launch_residual_add(bool bf16, const void* X, const void* D, void* Out, int64_t n, hipStream_t st) {
  if (n == 0) return;
  if (bf16) hipLaunchKernelGGL(residual_add_kernel<true>, dim3(ew_blocks(n / 8)), dim3(256), 0, st, X, D, Out, n / 8);
  else      hipLaunchKernelGGL(residual_add_kernel<false>, dim3(ew_blocks(n / 8)), dim3(256), 0, st, X, D, Out, n / 8);
}

// dst[i, :] = src[index[i], :] (gather) or dst[index[i], :] = src[i, :] (scatter); rows of `row_bytes` bytes
// (a multiple of 16), one workgroup per 4 rows.
__global__ void __launch_bounds__(256) permute_rows_kernel(const uint8_t* __restrict__ src, uint8_t* __restrict__ dst,
                                                           const int32_t* __restrict__ index, int64_t rows,
                                                           int64_t row_bytes, int scatter) {
  const int64_t i = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (i >= rows) return;
  const int64_t other = index[i];
  const u32x4* s = reinterpret_cast<const u32x4*>(src + (scatter ? i : other) * row_bytes);
  u32x4* d = reinterpret_cast<u32x4*>(dst + (scatter ? other : i) * row_bytes);
  for (int64_t c = threadIdx.x & 63; c < row_bytes / 16; c += 64) d[c] = s[c];
}
void launch_permute_rows(const void* src, void* dst, const int32_t* index, int64_t rows, int64_t row_bytes, bool scatter,
                         hipStream_t st) {
  if (rows == 0 || row_bytes == 0) return;
  hipLaunchKernelGGL(permute_rows_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, st,
                     static_cast<const uint8_t*>(src), static_cast<uint8_t*>(dst), index, rows, row_bytes, scatter ? 1 : 0);
}

// dst[i] = src[i] forced into [0, rows): whatever list the caller passed, the kernels that fetch and scatter rows through
// the copy stay inside the tensors (a bad list then gives wrong rows, never an access outside them).
__global__ void __launch_bounds__(256) clamp_index_kernel(const int32_t* __restrict__ src, int32_t* __restrict__ dst,
                                                          int rows) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < rows) dst[i] = min(max(src[i], 0), rows - 1);
}
void launch_clamp_index(const int32_t* src, int32_t* dst, int64_t rows, hipStream_t st) {
  if (rows <= 0) return;
  hipLaunchKernelGGL(clamp_index_kernel, dim3((unsigned)((rows + 255) / 256)), dim3(256), 0, st, src, dst, (int)rows);
}

}  // namespace tlora
