// WeightSlice convolution / linear as an implicit GEMM on bf16 MFMA (gfx950).
//
//   Y[m, k] = sum_{r,s,c} X[n, p*st + r - pad, q*st + s - pad, c] * W[k, r0 + r, s0 + s, c]
//   m = (n, p, q) over the requests of one subnet cfg, k < K_active, c < C_active.
//
// The weight operand is the resident max-size tensor: a block reads the leading K_active rows,
// and inside each (k, r, s) the leading C_active channels, through the tensor's own strides.
// The reduction index is flattened over the ACTIVE extent only, in units of 8 channels
// (16 bytes): unit u -> (tap rs, c8) = (u / C8, u % C8), so a narrow subnet pays for its own K,
// not for the SuperNet's.  Active channel counts are multiples of 8, so a unit never straddles a
// tap and every 16-byte load is aligned.
//
// Tiling: 256 threads = 4 waves; block tile BM x BN, K step 64, double-buffered LDS (one barrier
// per step) with the next step's global loads in flight during the MFMAs;
// v_mfma_f32_32x32x16_bf16, fp32 accumulators.  Per-thread addressing is set up once: a base
// offset and a tap-validity bitmask per fetched row, tap offsets in a small LDS table; the K loop
// only adds.  The epilogue (fused SubnetNorm scale/shift, residual, activation) goes through a
// per-wave fp32 LDS tile so that residual loads and output stores are 16 bytes per lane and
// contiguous along channels.  Blocks are renumbered so that consecutive tiles (which share
// activation rows) run on the same XCD and meet in its L2.
// A launch is grouped: each block finds its problem (one per subnet cfg) from its tile number.
#include "common.h"

namespace sna {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

constexpr int BK = 64;             // reduction elements per LDS stage
constexpr int LDS_STRIDE = 64;     // bf16 per LDS row: 128-byte rows, 16-byte chunks XOR-swizzled by (row >> 1) & 7
constexpr int NTHREADS = 256;
constexpr int TAP_TABLE = 40;      // entries per tap table (taps <= 32, rest zero)
constexpr int SMEM_HEAD = 512;     // bytes reserved for the two tap tables

template <int BM, int BN, int WARPS_M, int WARPS_N>
struct IgemmCfg {
  static constexpr int WTM = BM / WARPS_M, WTN = BN / WARPS_N;
  static constexpr int TM = WTM / 32, TN = WTN / 32;
  static constexpr int EPI_STRIDE = WTN + 4;                                 // floats per staged row
  static constexpr int TILE_BYTES = 2 * (BM + BN) * LDS_STRIDE * 2;
  static constexpr int EPI_BYTES = 4 * 32 * EPI_STRIDE * 4;
  static constexpr int SMEM = SMEM_HEAD + (TILE_BYTES > EPI_BYTES ? TILE_BYTES : EPI_BYTES);
};

template <int BM, int BN, int WARPS_M, int WARPS_N>
__global__ __launch_bounds__(NTHREADS) __attribute__((amdgpu_waves_per_eu(2))) void igemm_kernel(const ConvGroupArgs args) {
  using Cfg = IgemmCfg<BM, BN, WARPS_M, WARPS_N>;
  static_assert(WARPS_M * WARPS_N == 4, "4 waves");
  constexpr int WTM = Cfg::WTM, WTN = Cfg::WTN, TM = Cfg::TM, TN = Cfg::TN;
  static_assert(TM >= 1 && TN >= 1 && WTM % 32 == 0 && WTN % 32 == 0, "wave tile");
  constexpr int A_IT = BM / 32, B_IT = BN / 32;      // rows fetched per thread (32 rows per pass)

  extern __shared__ __attribute__((aligned(16))) char smem[];
  int* tap_x = (int*)smem;
  int* tap_w = tap_x + TAP_TABLE;
  bf16_t* tiles = (bf16_t*)(smem + SMEM_HEAD);

  // XCD-aware renumbering: hardware block b runs on XCD b % 8; give each XCD a contiguous tile range
  const int per_xcd = gridDim.x >> 3;
  const int tile_id = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (tile_id >= args.total_tiles) return;

  const int g = find_problem(args, tile_id);
  const ConvProblem& p = args.p[g];
  const int local = tile_id - p.tile_start;
  const int tn = local % p.tiles_n, tm = local / p.tiles_n;
  const int m0 = tm * BM, n0 = tn * BN;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WARPS_N, wn = wave % WARPS_N;
  const int kc = tid & 7;                 // this thread's 16-byte unit inside a K step
  const int lrow = tid >> 3;              // 0..31

  const bf16_t* __restrict__ X = (const bf16_t*)p.x;
  const bf16_t* __restrict__ Wt = (const bf16_t*)p.w;
  const int C = p.C, H = p.H, Wd = p.W, S = p.S, RS = p.R * p.S;

  if (tid < TAP_TABLE) {
    int tx = 0, tw = 0;
    if (tid < RS) {
      const int r = tid / S, s = tid - r * S;
      tx = (r * Wd + s) * C;
      tw = r * p.wr + s * p.ws;
    }
    tap_x[tid] = tx;
    tap_w[tid] = tw;
  }

  // rows this thread fetches: base offset of the window's first tap and which taps are in range
  int a_base[A_IT];
  unsigned a_mask[A_IT];
#pragma unroll
  for (int i = 0; i < A_IT; ++i) {
    const int m = m0 + lrow + 32 * i;
    a_base[i] = 0;
    a_mask[i] = 0;
    if (m < p.M) {
      const int q = m % p.Wo, t = m / p.Wo;
      const int pp = t % p.Ho, n = t / p.Ho;
      const int ih0 = pp * p.stride - p.pad, iw0 = q * p.stride - p.pad;
      a_base[i] = ((n * H + ih0) * Wd + iw0) * C * 2;       // bytes
      unsigned mk = 0;
      for (int r = 0; r < p.R; ++r)
        for (int s = 0; s < S; ++s)
          if (ih0 + r >= 0 && ih0 + r < H && iw0 + s >= 0 && iw0 + s < Wd) mk |= 1u << (r * S + s);
      a_mask[i] = mk;
    }
  }
  int b_base[B_IT];
  unsigned b_ok = 0;
#pragma unroll
  for (int j = 0; j < B_IT; ++j) {
    const int k = n0 + lrow + 32 * j;
    if (k < p.K) b_ok |= 1u << j;
    b_base[j] = k * p.wk * 2;                             // bytes
  }

  // reduction position of this thread's unit: tap rs and channel octet c8
  int rs = kc / p.C8;
  int c8 = kc - rs * p.C8;

  uint4 a_reg[2][A_IT], b_reg[2][B_IT];  // two K steps of operands in flight in registers
  const int KT = (p.K8 + 7) >> 3;         // K steps of 64 elements
  __syncthreads();                        // tap tables visible

  // Operand loads go through buffer descriptors: an offset at or beyond the tensor's size returns
  // zeros without touching memory, which is how padding taps, ragged rows and the K tail are fed.
  const __amdgpu_buffer_rsrc_t rsrc_x = __builtin_amdgcn_make_buffer_rsrc((void*)X, 0, (int)p.x_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_w = __builtin_amdgcn_make_buffer_rsrc((void*)Wt, 0, (int)p.w_bytes, 0x00020000);
  constexpr unsigned OOB = 0x80000000u;
  auto fetch = [&](uint4 (&ar)[A_IT], uint4 (&br)[B_IT]) {
    const bool u_ok = rs < RS;
    const int rsc = u_ok ? rs : RS;       // entry RS of the tables is zero
    const int tx = (tap_x[rsc] + c8 * 8) * 2, tw = (tap_w[rsc] + c8 * 8) * 2;
#pragma unroll
    for (int i = 0; i < A_IT; ++i) {
      const bool ok = u_ok && ((a_mask[i] >> rsc) & 1u);
      const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rsrc_x, ok ? (unsigned)(a_base[i] + tx) : OOB, 0, 0);
      ar[i] = make_uint4(v.x, v.y, v.z, v.w);
    }
#pragma unroll
    for (int j = 0; j < B_IT; ++j) {
      const bool ok = u_ok && ((b_ok >> j) & 1u);
      const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rsrc_w, ok ? (unsigned)(b_base[j] + tw) : OOB, 0, 0);
      br[j] = make_uint4(v.x, v.y, v.z, v.w);
    }
    c8 += 8;                              // advance one K step
    while (c8 >= p.C8) { c8 -= p.C8; ++rs; }
  };
  // LDS rows are 128 bytes (one K step); the 16-byte chunk c of row r lives in slot c ^ ((r >> 1) & 7),
  // which keeps both the row-wise stores and the column-wise fragment loads free of bank conflicts.
  const int kc_sw = kc ^ ((lrow >> 1) & 7);
  auto stage = [&](int buf, const uint4 (&ar)[A_IT], const uint4 (&br)[B_IT]) {
    bf16_t* As = tiles + buf * (BM + BN) * LDS_STRIDE;
    bf16_t* Bs = As + BM * LDS_STRIDE;
#pragma unroll
    for (int i = 0; i < A_IT; ++i) *(uint4*)(As + (lrow + 32 * i) * LDS_STRIDE + kc_sw * 8) = ar[i];
#pragma unroll
    for (int j = 0; j < B_IT; ++j) *(uint4*)(Bs + (lrow + 32 * j) * LDS_STRIDE + kc_sw * 8) = br[j];
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const int frag_row = lane & 31, frag_hi = lane >> 5, frag_sw = (frag_row >> 1) & 7;
  int frag_off[BK / 16];                   // swizzled element offset of this lane's chunk in each 16-wide slice
#pragma unroll
  for (int ks = 0; ks < BK / 16; ++ks) frag_off[ks] = ((ks * 2 + frag_hi) ^ frag_sw) * 8;
  auto compute = [&](int buf) {
    const bf16_t* As = tiles + buf * (BM + BN) * LDS_STRIDE + (wm * WTM + frag_row) * LDS_STRIDE;
    const bf16_t* Bs = tiles + buf * (BM + BN) * LDS_STRIDE + (BM + wn * WTN + frag_row) * LDS_STRIDE;
    bf16x8 af[2][TM], bfr[2][TN];        // fragments of the next 16-wide slice load while this one multiplies
#pragma unroll
    for (int i = 0; i < TM; ++i) af[0][i] = *(const bf16x8*)(As + i * 32 * LDS_STRIDE + frag_off[0]);
#pragma unroll
    for (int j = 0; j < TN; ++j) bfr[0][j] = *(const bf16x8*)(Bs + j * 32 * LDS_STRIDE + frag_off[0]);
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      const int cur = ks & 1, nxt = cur ^ 1;
      if (ks + 1 < BK / 16) {
#pragma unroll
        for (int i = 0; i < TM; ++i) af[nxt][i] = *(const bf16x8*)(As + i * 32 * LDS_STRIDE + frag_off[ks + 1]);
#pragma unroll
        for (int j = 0; j < TN; ++j) bfr[nxt][j] = *(const bf16x8*)(Bs + j * 32 * LDS_STRIDE + frag_off[ks + 1]);
      }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[cur][i], bfr[cur][j], acc[i][j], 0, 0, 0);
    }
  };

  // Software pipeline.  At the top of step kt the register sets hold the operands of steps kt+1
  // and kt+2 (loads in flight); set (kt+1)&1 goes to the idle LDS buffer and is refilled with
  // step kt+3 before the MFMAs of step kt start, so LDS stores and global loads run under them.
  fetch(a_reg[0], b_reg[0]);                        // step 0
  stage(0, a_reg[0], b_reg[0]);
  if (KT > 1) fetch(a_reg[1], b_reg[1]);            // step 1
  if (KT > 2) fetch(a_reg[0], b_reg[0]);            // step 2
  for (int kt = 0; kt < KT; kt += 2) {
    __syncthreads();
    if (kt + 1 < KT) stage(1, a_reg[1], b_reg[1]);
    if (kt + 3 < KT) fetch(a_reg[1], b_reg[1]);
    compute(0);
    if (kt + 1 >= KT) break;
    __syncthreads();
    if (kt + 2 < KT) stage(0, a_reg[0], b_reg[0]);
    if (kt + 4 < KT) fetch(a_reg[0], b_reg[0]);
    compute(1);
  }
  __syncthreads();

  // ---- epilogue -----------------------------------------------------------------------------
  // accumulator element v of lane l is row 8*(v/4) + 4*(l/32) + v%4, column l%32 of a 32x32 tile.
  // Per 32-row strip: SubnetNorm scale/shift on the accumulators, fp32 strip into this wave's LDS
  // region, then each lane takes (row, 8 consecutive channels): residual, activation, store.
  float* epi = (float*)(smem + SMEM_HEAD) + wave * 32 * Cfg::EPI_STRIDE;
  const int col_l = lane & 31, row_l = (lane >> 5) * 4;
  float sc[TN], sh[TN];
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int k = n0 + wn * WTN + j * 32 + col_l;
    sc[j] = (p.scale && k < p.K) ? p.scale[k] : 1.f;
    sh[j] = (p.shift && k < p.K) ? p.shift[k] : 0.f;
  }
  constexpr int OCT = WTN / 8;                 // channel octets per staged row
  constexpr int PAIRS = 32 * OCT / 64;         // (row, octet) pairs per lane
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v)
        epi[(8 * (v >> 2) + row_l + (v & 3)) * Cfg::EPI_STRIDE + j * 32 + col_l] = fmaf(acc[i][j][v], sc[j], sh[j]);
    // wave-private region: the wave's own LDS writes are visible to its later reads
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_s_waitcnt(0xc07f);        // lgkmcnt(0)
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int t = 0; t < PAIRS; ++t) {
      const int id = t * 64 + lane;
      const int row = id / OCT, oct = id - row * OCT;
      const int m = m0 + wm * WTM + i * 32 + row;
      const int k = n0 + wn * WTN + oct * 8;
      if (m < p.M && k < p.K) {
        const float4 v0 = *(const float4*)(epi + row * Cfg::EPI_STRIDE + oct * 8);
        const float4 v1 = *(const float4*)(epi + row * Cfg::EPI_STRIDE + oct * 8 + 4);
        float val[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
        float rv[8];
        if (p.res) {
          const uint4 r4 = *(const uint4*)((const bf16_t*)p.res + (long)m * p.res_stride + k);
          const unsigned ru[4] = {r4.x, r4.y, r4.z, r4.w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            rv[2 * e] = __uint_as_float(ru[e] << 16);
            rv[2 * e + 1] = __uint_as_float(ru[e] & 0xffff0000u);
          }
          if (!p.res_after_act) {
#pragma unroll
            for (int e = 0; e < 8; ++e) val[e] += rv[e];
          }
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) val[e] = apply_act(val[e], p.act);
        if (p.res && p.res_after_act) {
#pragma unroll
          for (int e = 0; e < 8; ++e) val[e] += rv[e];
        }
        if (p.out_fp32) {
          float* yo = (float*)p.y + (long)m * p.y_stride + k;
          *(float4*)yo = make_float4(val[0], val[1], val[2], val[3]);
          *(float4*)(yo + 4) = make_float4(val[4], val[5], val[6], val[7]);
        } else {
          uint4 o;
          o.x = (unsigned)f32_to_bf16(val[0]) | ((unsigned)f32_to_bf16(val[1]) << 16);
          o.y = (unsigned)f32_to_bf16(val[2]) | ((unsigned)f32_to_bf16(val[3]) << 16);
          o.z = (unsigned)f32_to_bf16(val[4]) | ((unsigned)f32_to_bf16(val[5]) << 16);
          o.w = (unsigned)f32_to_bf16(val[6]) | ((unsigned)f32_to_bf16(val[7]) << 16);
          *(uint4*)((bf16_t*)p.y + (long)m * p.y_stride + k) = o;
        }
      }
    }
  }
}

struct Variant { int bm, bn, smem; void (*fn)(const ConvGroupArgs); };
#define SNA_VARIANT(BM, BN, WM, WN) \
  { BM, BN, IgemmCfg<BM, BN, WM, WN>::SMEM, igemm_kernel<BM, BN, WM, WN> }
static const Variant kVariants[] = {
    SNA_VARIANT(128, 128, 2, 2), SNA_VARIANT(128, 64, 2, 2), SNA_VARIANT(128, 96, 4, 1),
    SNA_VARIANT(128, 32, 4, 1),  SNA_VARIANT(64, 64, 2, 2),  SNA_VARIANT(64, 128, 1, 4),
    SNA_VARIANT(32, 128, 1, 4),
};
constexpr int kNumVariants = sizeof(kVariants) / sizeof(kVariants[0]);

int igemm_num_variants() { return kNumVariants; }
void igemm_tile_shape(int variant, int* bm, int* bn) {
  *bm = kVariants[variant].bm;
  *bn = kVariants[variant].bn;
}

hipError_t launch_igemm(const ConvGroupArgs& a, int variant, hipStream_t s) {
  if (a.n == 0) return hipSuccess;
  if (variant < 0 || variant >= kNumVariants) return hipErrorInvalidValue;
  static bool attr_done[kNumVariants] = {false};
  const Variant& v = kVariants[variant];
  if (!attr_done[variant]) {
    hipError_t e = hipFuncSetAttribute((const void*)v.fn, hipFuncAttributeMaxDynamicSharedMemorySize, v.smem);
    if (e != hipSuccess) return e;
    attr_done[variant] = true;
  }
  const int blocks = (a.total_tiles + 7) / 8 * 8;
  hipLaunchKernelGGL(v.fn, dim3(blocks), dim3(NTHREADS), v.smem, s, a);
  return hipGetLastError();
}

}  // namespace sna
