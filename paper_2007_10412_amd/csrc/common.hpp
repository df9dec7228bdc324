// Shared device-side definitions for the RAD kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rad {

constexpr int kBucket = 256;      // columns per offset-table bucket of a store
constexpr int kWave = 64;

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

enum Scheme : int { kExact = 0, kBernoulli = 1, kFixedKShared = 2, kFixedKPerExample = 3, kReplaceShared = 4,
                    kReplacePerExample = 5, kProjectShared = 6, kProjectPerExample = 7 };
enum DType : int { kF32 = 0, kBF16 = 1 };

// fp32 -> bf16 bits, round to nearest even (NaN payload is not preserved; the
// library never produces NaN from finite inputs).
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) {
  return __uint_as_float(((uint32_t)b) << 16);
}

// lanes of this wave with a lower lane id that have `pred` set
__device__ __forceinline__ int lanes_below(uint64_t ballot) {
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(ballot >> 32),
                                   __builtin_amdgcn_mbcnt_lo((uint32_t)ballot, 0));
}

// View of a compressed store as kernels see it.  All pointers are device memory.
struct StoreView {
  void* values;              // capacity entries, storage dtype
  uint16_t* indices;         // capacity entries, column of each value
  uint32_t* row_ptr;         // rows + 1, first entry of every row
  uint16_t* bucket_off;      // [plan_rows][nb + 1]: entries of the row before column 256*t
  uint32_t* bitmap;          // transient keep bitmap [plan_rows][bm_pitch] words
  int64_t capacity;
  int rows;                  // rows of one step block
  int cols;
  int nb;                    // ceil(cols / 256)
  int bm_pitch;              // words per bitmap row
  int plan_row_stride;       // 1, or 0 when every row shares one plan row (shared scheme)
  int idx_shared;            // shared scheme: `indices` holds the k columns once (written by row 0)
  const uint16_t* mult;      // with-replacement draws: how often each entry's column was drawn, [plan_rows][mult_pitch]
  int mult_pitch;            //   in entry order of the row; null otherwise (every weight is 1)
  int shared_k;              // shared scheme: entries per row (rows are k rounded up to 8 apart); else 0
  int may_overflow;          // Bernoulli draws: an entry position may lie beyond `capacity` and must be checked
  int paired;                // bf16 per-entry draws: `values` holds 32-bit (value, column) entries, no `indices`
  float scale;
};

// LDS layout of a 32-deep bf16 operand tile (64-byte rows of four 16-byte units): row r is kept at row
// tile_row(r) and its unit kc at position kc ^ tile_swz(r).  The row permutation moves rows that are 8
// apart (what the lanes of the transposing loader write in one instruction) into different 64-byte bank
// windows, and the unit swizzle spreads the rest, so that the MFMA fragment reads (consecutive rows, one
// unit), the 16-byte writes of the K-contiguous loader (4 rows x 4 units) and the 8-byte writes of the
// transposing loader (rows 8 apart) all touch every LDS bank once per pass.
__host__ __device__ __forceinline__ constexpr int tile_row(int r) { return r ^ ((r >> 3) & 3); }   // an involution
__host__ __device__ __forceinline__ constexpr int tile_swz(int r) {
  return (((r >> 2) & 1) | (((r >> 3) & 1) << 1)) ^ ((r >> 5) & 3);
}

// Entry of a paired bf16 store: the bf16 value bits in the high half; in the low half the column inside
// its 256-column bucket, written as the byte offset of that column's row in the LDS tile the dW kernel
// scatters into (tile_row(column) << 6, swizzle term of the row in bits 4..5).  The kernel gets the LDS
// address of an entry with one XOR; everything else decodes the column back.
constexpr int kPairPad = 64;     // entries allocated past the capacity, so a lane may read beyond a segment
__host__ __device__ __forceinline__ constexpr uint32_t pair_code(int col_in_bucket) {
  return ((uint32_t)tile_row(col_in_bucket) << 6) | ((uint32_t)tile_swz(col_in_bucket) << 4);
}
__host__ __device__ __forceinline__ constexpr uint32_t pair_make(uint32_t bf16_bits, int col) {
  return (bf16_bits << 16) | pair_code(col & (kBucket - 1));
}
__host__ __device__ __forceinline__ constexpr int pair_col(uint32_t entry, int bucket) {
  return bucket * kBucket + tile_row((int)((entry >> 6) & (uint32_t)(kBucket - 1)));
}

}  // namespace rad
