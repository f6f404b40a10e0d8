// Internal tables shared by the host planner and the gfx950 kernels (plain PODs, copied to the
// head of the caller's workspace once per call).
#pragma once
#include <stddef.h>
#include <stdint.h>

namespace tlora {

constexpr int kRankGranule = 8;     // ranks are padded to 8 elements = one 16-byte bf16 chunk
constexpr int kGemmBM = 256;        // backbone GEMM macro tile (token rows x output columns)
constexpr int kGemmBN = 256;
constexpr int kGemmBK = 32;
constexpr int kShrinkCols = 64;     // rank columns per shrink work unit
constexpr int kGradCols = 256;      // feature columns per dA/dB work unit (4 waves x 64)
constexpr int kGradRanks = 32;      // rank rows per MFMA block of the dA/dB kernel
constexpr int kGradMaxBlocks = 4;   // rank blocks of 32 per dA/dB work unit (128 rank rows)
constexpr int kGradStep = 32;       // tokens per pipeline step of the dA/dB kernel
constexpr int kGradMaxTokens = 4096;  // most tokens of one dA/dB work unit (32 per live rank row of a full 128-row block)

// One job's view of the problem (Sec. 3.2: one adapter branch per job on the shared backbone).
struct JobDev {
  int32_t row0, row1;      // token segment [row0, row1) of the concatenated batch
  int32_t rank, rpad;      // r_j and r_j rounded up to kRankGranule
  float scale;
  int32_t pad_;
  int64_t soff;            // element offset of the job's [T_j, rpad] block in the fp32 S / dS buffers
  int64_t atp_off;         // element offset of A_j^T packed [rpad, d_in]  (bf16)
  int32_t roff;            // sum of rpad_i over i < j: the job's row in B-all [R + 32, d_out] and its
  int32_t pad2_;           //   column in A-all [d_in, R + 32]  (R = sum of all rpad_i)
  const void* A;           // caller's A_j [d_in, r_j]
  const void* B;           // caller's B_j [r_j, d_out]
  void* dA;                // caller's dA_j (fp32) or null
  void* dB;                // caller's dB_j (fp32) or null
};

// Row tile of the backbone GEMM (256 token rows of the concatenated batch).  Its adapter K-extension is
// the padded-rank range [roff_first, roff_first + kext) of the jobs first..last that have a row inside
// the tile; the bf16 operand s_j * S_j (resp. s_j * dS_j) of the tile is a dense zero-padded
// [256, kext] matrix at element offset aoff, non-zero only where a row meets its own job's columns.
struct TileDev {
  int32_t first, last;
  int32_t kext;            // multiple of 32 (0: no adapter work in this tile)
  int32_t roff_first;
  int64_t aoff;
};

// Work unit of the shrink kernels (S_j = X_j.A_j and dS_j = dY_j.B_j^T): a block of token rows of
// one job times a block of kShrinkCols padded rank columns.
struct ShrinkUnit {
  int32_t job;
  int32_t t0;              // first global token row
  int32_t nrows;           // rows in this unit (<= shrink_rows)
  int32_t pb;              // rank-column block
};

// Work unit of the dA/dB kernels: tokens [t0, t1) of one job x kGradCols feature columns x rank block pb
// (128 rank rows, of which the first 32 * mb hold ranks below rpad); writes one partial tile
// [32 * mb, kGradCols] (fp32) at float offset part_off, which the reduce pass sums in unit order.
struct GradUnit {
  int32_t job;
  int32_t t0, t1;
  int32_t cb;              // feature-column block
  int32_t pb;              // rank block (of 128 rows)
  int32_t mb;              // live 32-row blocks in it: 1 .. 4
  int64_t part_off;
};

// One output tile of dA_j / dB_j: the run of nunits consecutive partial tiles that sum to it.
struct GradGroup {
  int32_t job;
  int32_t cb, pb;
  int32_t mb;
  int32_t nunits;          // number of partial tiles (token chunks); 0 for an empty segment
  int32_t pad_;
  int64_t part_off;        // float offset of the first partial tile
};

// fp32 path: one strided matrix product  C (+)= alpha * A.B  (used for the fp32 configuration).
struct F32Unit {
  const float* A;
  const float* B;
  float* C;
  int32_t M, N, K;
  int32_t accumulate;
  int64_t a_rs, a_cs, b_rs, b_cs, c_rs;
  float alpha;
  int32_t pad_;
};
struct F32Tile {
  int32_t unit, tm, tn, pad_;
};

// one tensor of the optimizer step (device table entry)
struct AdamwDev {
  void* param;          // bf16 or fp32
  float* master;        // may be null (fp32 param updated in place)
  const float* grad;
  float* m;
  float* v;
  int64_t n;
  float lr, beta1, beta2, eps, weight_decay;
  float c1, c2;         // 1 / (1 - beta1^t), 1 / (1 - beta2^t)
  int32_t param_is_bf16;
};

}  // namespace tlora
