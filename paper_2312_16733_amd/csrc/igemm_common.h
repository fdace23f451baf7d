// Pieces shared by the implicit-GEMM kernels: LDS row format, tile geometry, the inline LDS read.
#pragma once
#include "common.h"

#include <type_traits>

namespace sna {
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((address_space(3))) char lds_char;

constexpr int BK = 64;             // reduction elements per LDS stage
static_assert(BK == 64, "one LDS row holds one K step");
constexpr int ROW_B = 128;         // bytes per LDS row (one K step of one tile row)

// s_waitcnt immediate that waits until at most n vector-memory operations are outstanding
// (vmcnt is split over bits [3:0] and [15:14]; expcnt and lgkmcnt fields left at "no wait").
constexpr int vmcnt_imm(int n) { return 0x0F70 | (n & 15) | ((n >> 4) << 14); }

template <int BM, int BN, int WARPS_M, int WARPS_N, int NS>
struct IgemmCfg {
  static constexpr int NWAVES = WARPS_M * WARPS_N, NTHREADS = 64 * NWAVES;
  static constexpr int WTM = BM / WARPS_M, WTN = BN / WARPS_N;
  static constexpr int TM = WTM / 32, TN = WTN / 32;
  static constexpr int PASS_ROWS = NTHREADS / 8;                 // tile rows fetched per pass of the block
  static constexpr int A_IT = (BM + PASS_ROWS - 1) / PASS_ROWS, B_IT = (BN + PASS_ROWS - 1) / PASS_ROWS;
  static constexpr int STAGE_B = (BM + BN) * ROW_B;
  static constexpr int EPI_STRIDE = WTN + 4;                     // floats per staged row
  static constexpr int TILE_BYTES = NS * STAGE_B;
  static constexpr int EPI_BYTES = NWAVES * 32 * EPI_STRIDE * 4;
  static constexpr int SMEM = TILE_BYTES > EPI_BYTES ? TILE_BYTES : EPI_BYTES;
};

__device__ __forceinline__ unsigned long long low_bits(int n) { return n >= 64 ? ~0ull : (1ull << n) - 1ull; }   // n >= 0

__device__ __forceinline__ u32x4 lds_read_b128(unsigned addr, int imm) {
  u32x4 v;
#if defined(__HIP_DEVICE_COMPILE__)
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(imm));
#else
  v = u32x4{addr, (unsigned)imm, 0u, 0u};      // host pass only parses this file
#endif
  return v;
}


}  // namespace sna
