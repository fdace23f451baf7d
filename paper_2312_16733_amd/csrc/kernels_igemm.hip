// WeightSlice convolution / linear as an implicit GEMM on bf16 MFMA (gfx950).
//
//   Y[m, k] = sum_{r,s,c} X[n, p*st + r - pad, q*st + s - pad, c] * W[k, r0 + r, s0 + s, c]
//   m = (n, p, q) over the requests of one subnet cfg, k < K_active, c < C_active.
//
// The weight operand is the resident max-size tensor: a block reads the leading K_active rows,
// and inside each (k, r, s) the leading C_active channels, through the tensor's own strides.
// The reduction index is flattened over the ACTIVE extent only, in units of 8 channels
// (16 bytes): unit u -> (r, s, c8) = (u / C8 / S, u / C8 % S, u % C8), so a narrow subnet pays
// for its own K, not for the SuperNet's.  Active channel counts are multiples of 8, so a unit
// never straddles a tap and every 16-byte load is aligned.
//
// Tiling: 256 threads = 4 waves; block tile BM x BN, K step 32, double-buffered LDS with the next
// tile's global loads in flight during the MFMAs; v_mfma_f32_32x32x16_bf16, fp32 accumulators.
// Epilogue (fused SubnetNorm scale/shift, residual, activation) runs on the accumulators.
// A launch is grouped: each block finds its problem (one per subnet cfg) from the block index.
#include "common.h"

namespace sna {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int BK = 32;            // reduction elements per LDS stage
constexpr int LDS_STRIDE = 40;    // bf16 per LDS row: 32 + 8 pad -> 80-byte rows, conflict-free b128 reads
constexpr int NTHREADS = 256;

template <int BM, int BN, int WARPS_M, int WARPS_N>
__global__ __launch_bounds__(NTHREADS) void igemm_kernel(const ConvGroupArgs args) {
  static_assert(WARPS_M * WARPS_N == 4, "4 waves");
  constexpr int WTM = BM / WARPS_M, WTN = BN / WARPS_N;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  static_assert(TM >= 1 && TN >= 1 && WTM % 32 == 0 && WTN % 32 == 0, "wave tile");
  constexpr int A_IT = (BM * 4 + NTHREADS - 1) / NTHREADS;
  constexpr int B_IT = (BN * 4 + NTHREADS - 1) / NTHREADS;

  __shared__ __attribute__((aligned(16))) bf16_t lds[2 * (BM + BN) * LDS_STRIDE];

  const int g = find_problem(args, blockIdx.x);
  const ConvProblem& p = args.p[g];
  const int local = blockIdx.x - p.tile_start;
  const int tn = local % p.tiles_n, tm = local / p.tiles_n;
  const int m0 = tm * BM, n0 = tn * BN;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WARPS_N, wn = wave % WARPS_N;
  const int kc = tid & 3;                 // this thread's 16-byte unit inside a K step
  const int lrow = tid >> 2;              // 0..63

  const bf16_t* __restrict__ X = (const bf16_t*)p.x;
  const bf16_t* __restrict__ Wt = (const bf16_t*)p.w;
  const int C = p.C, H = p.H, Wd = p.W, S = p.S;

  // per-thread A rows: pixel coordinates of the rows this thread fetches
  long a_base[A_IT];
  int a_ih0[A_IT], a_iw0[A_IT];
#pragma unroll
  for (int i = 0; i < A_IT; ++i) {
    const int row = lrow + 64 * i;
    const int m = m0 + row;
    if (row < BM && m < p.M) {
      const int q = m % p.Wo, t = m / p.Wo;
      const int pp = t % p.Ho, n = t / p.Ho;
      a_base[i] = (long)n * H * Wd * C;
      a_ih0[i] = pp * p.stride - p.pad;
      a_iw0[i] = q * p.stride - p.pad;
    } else {
      a_base[i] = 0;
      a_ih0[i] = -100000;               // never in range -> zero fill
      a_iw0[i] = 0;
    }
  }
  long b_base[B_IT];
  bool b_ok[B_IT];
#pragma unroll
  for (int j = 0; j < B_IT; ++j) {
    const int row = lrow + 64 * j;
    const int k = n0 + row;
    b_ok[j] = (row < BN) && (k < p.K);
    b_base[j] = (long)k * p.wk;
  }

  uint4 a_reg[A_IT], b_reg[B_IT];
  const int KT = (p.K8 + 3) >> 2;         // K steps of 32 elements

  auto fetch = [&](int kt) {
    const int u = kt * 4 + kc;
    const bool u_ok = u < p.K8;
    const int rs = (int)(((unsigned long long)(unsigned)u * p.magic_c8) >> 24);
    const int c8 = u - rs * p.C8;
    const int r = rs / S, s = rs - r * S;
#pragma unroll
    for (int i = 0; i < A_IT; ++i) {
      const int ih = a_ih0[i] + r, iw = a_iw0[i] + s;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (u_ok && ih >= 0 && ih < H && iw >= 0 && iw < Wd)
        v = *(const uint4*)(X + a_base[i] + ((long)ih * Wd + iw) * C + c8 * 8);
      a_reg[i] = v;
    }
    const long woff = (long)r * p.wr + (long)s * p.ws + c8 * 8;
#pragma unroll
    for (int j = 0; j < B_IT; ++j) {
      uint4 v = make_uint4(0, 0, 0, 0);
      if (u_ok && b_ok[j]) v = *(const uint4*)(Wt + b_base[j] + woff);
      b_reg[j] = v;
    }
  };
  auto stage = [&](int buf) {
    bf16_t* As = lds + buf * (BM + BN) * LDS_STRIDE;
    bf16_t* Bs = As + BM * LDS_STRIDE;
#pragma unroll
    for (int i = 0; i < A_IT; ++i) {
      const int row = lrow + 64 * i;
      if (row < BM) *(uint4*)(As + row * LDS_STRIDE + kc * 8) = a_reg[i];
    }
#pragma unroll
    for (int j = 0; j < B_IT; ++j) {
      const int row = lrow + 64 * j;
      if (row < BN) *(uint4*)(Bs + row * LDS_STRIDE + kc * 8) = b_reg[j];
    }
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  fetch(0);
  stage(0);
  __syncthreads();
  const int frag_row = lane & 31, frag_k = (lane >> 5) * 8;
  for (int kt = 0; kt < KT; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < KT) fetch(kt + 1);
    const bf16_t* As = lds + buf * (BM + BN) * LDS_STRIDE;
    const bf16_t* Bs = As + BM * LDS_STRIDE;
#pragma unroll
    for (int kk = 0; kk < BK; kk += 16) {
      bf16x8 af[TM], bfr[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i)
        af[i] = *(const bf16x8*)(As + (wm * WTM + i * 32 + frag_row) * LDS_STRIDE + kk + frag_k);
#pragma unroll
      for (int j = 0; j < TN; ++j)
        bfr[j] = *(const bf16x8*)(Bs + (wn * WTN + j * 32 + frag_row) * LDS_STRIDE + kk + frag_k);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < KT) stage(buf ^ 1);
    __syncthreads();
  }

  // epilogue: accumulator element v of lane l is row 8*(v/4) + 4*(l/32) + v%4, column l%32
  const int col_l = lane & 31, row_l = (lane >> 5) * 4;
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int k = n0 + wn * WTN + j * 32 + col_l;
    if (k >= p.K) continue;
    const float sc = p.scale ? p.scale[k] : 1.f;
    const float sh = p.shift ? p.shift[k] : 0.f;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int m = m0 + wm * WTM + i * 32 + 8 * (v >> 2) + row_l + (v & 3);
        if (m >= p.M) continue;
        float val = fmaf(acc[i][j][v], sc, sh);
        if (p.res && !p.res_after_act) val += bf16_to_f32(((const bf16_t*)p.res)[(long)m * p.res_stride + k]);
        val = apply_act(val, p.act);
        if (p.res && p.res_after_act) val += bf16_to_f32(((const bf16_t*)p.res)[(long)m * p.res_stride + k]);
        if (p.out_fp32) ((float*)p.y)[(long)m * p.y_stride + k] = val;
        else ((bf16_t*)p.y)[(long)m * p.y_stride + k] = f32_to_bf16(val);
      }
    }
  }
}

struct Variant { int bm, bn; void (*fn)(const ConvGroupArgs); };
static const Variant kVariants[] = {
    {128, 128, igemm_kernel<128, 128, 2, 2>},
    {128, 64, igemm_kernel<128, 64, 2, 2>},
    {128, 96, igemm_kernel<128, 96, 4, 1>},
    {128, 32, igemm_kernel<128, 32, 4, 1>},
    {64, 64, igemm_kernel<64, 64, 2, 2>},
    {64, 128, igemm_kernel<64, 128, 1, 4>},
    {32, 128, igemm_kernel<32, 128, 1, 4>},
};

int igemm_num_variants() { return (int)(sizeof(kVariants) / sizeof(kVariants[0])); }
void igemm_tile_shape(int variant, int* bm, int* bn) {
  *bm = kVariants[variant].bm;
  *bn = kVariants[variant].bn;
}

hipError_t launch_igemm(const ConvGroupArgs& a, int variant, hipStream_t s) {
  if (a.n == 0) return hipSuccess;
  if (variant < 0 || variant >= igemm_num_variants()) return hipErrorInvalidValue;
  const int blocks = a.p[a.n - 1].tile_start + a.p[a.n - 1].tiles;
  hipLaunchKernelGGL(kVariants[variant].fn, dim3(blocks), dim3(NTHREADS), 0, s, a);
  return hipGetLastError();
}

}  // namespace sna
