// Transformer pieces that are not plain linear layers: softmax attention over the leading heads
// of a layer (head_dim 64, up to 128 tokens per request) on bf16 MFMA, and LayerNorm.
#include "common.h"

namespace sna {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

constexpr int AT_S = 128;          // max tokens per request
constexpr int AT_D = 64;           // head dim
constexpr int AT_LD = AT_S + 8;    // LDS row stride (bf16) for V^T and P

// One block = one (request, head); wave w owns queries [32w, 32w + 32).
//   scores = Q K^T / 8 (fp32) -> softmax over keys (fp32) -> P rounded to bf16 -> ctx = P V -> bf16.
// The scores are computed transposed (K as the row operand, Q as the column operand), so that a lane
// of the accumulator holds one query (column lane % 32) and 16 of the 32 keys of each key block:
// the softmax reduction over keys runs inside a lane plus one exchange with lane ^ 32, and the
// probabilities are already laid out as the row operand of the second product (row = query, 8
// values per K slice) without a trip through LDS.  The slice's 8 values are keys
// {base + 4 hi + 0..3, base + 8 + 4 hi + 0..3} (hi = lane / 32) instead of 8 consecutive keys; a
// sum over keys may take them in any order as long as the V operand uses the same one, and V^T in
// LDS gives each lane its two runs of 4 keys as two 8-byte reads.
// Q and K fragments come straight from global memory (a lane's 8 consecutive head-dim values are
// contiguous); V is transposed through LDS.
__global__ __launch_bounds__(256) void attention_kernel(const AttnGroupArgs args) {
  __shared__ __attribute__((aligned(16))) bf16_t Vt[AT_D * AT_LD];
  const int g = find_problem(args, blockIdx.x);
  const AttnProblem& p = args.p[g];
  const int local = blockIdx.x - p.tile_start;
  const int h = local % p.heads, b = local / p.heads;
  const int S = p.S, ld = p.ld;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const bf16_t* Q = (const bf16_t*)p.q + (long)b * S * ld + h * AT_D;
  const bf16_t* Kp = (const bf16_t*)p.k + (long)b * S * ld + h * AT_D;
  const bf16_t* V = (const bf16_t*)p.v + (long)b * S * ld + h * AT_D;

  // V^T into LDS: Vt[d][key], zero for keys >= S
  for (int idx = tid; idx < AT_S * (AT_D / 8); idx += 256) {
    const int key = idx >> 3, d8 = idx & 7;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (key < S) v = *(const uint4*)(V + (long)key * ld + d8 * 8);
    const unsigned u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      Vt[(d8 * 8 + 2 * e) * AT_LD + key] = (bf16_t)(u[e] & 0xffffu);
      Vt[(d8 * 8 + 2 * e + 1) * AT_LD + key] = (bf16_t)(u[e] >> 16);
    }
  }

  const int r32 = lane & 31, hi = lane >> 5;
  const int qrow = wave * 32 + r32;
  bf16x8 qf[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    uint4 v = make_uint4(0, 0, 0, 0);
    if (qrow < S) v = *(const uint4*)(Q + (long)qrow * ld + ks * 16 + hi * 8);
    qf[ks] = __builtin_bit_cast(bf16x8, v);
  }
  // sc[j][v]: query qrow, key 32 j + 8 (v / 4) + 4 hi + v % 4
  f32x16 sc[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
#pragma unroll
    for (int v = 0; v < 16; ++v) sc[j][v] = 0.f;
    const int key = j * 32 + r32;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      uint4 v = make_uint4(0, 0, 0, 0);
      if (key < S) v = *(const uint4*)(Kp + (long)key * ld + ks * 16 + hi * 8);
      sc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, v), qf[ks], sc[j], 0, 0, 0);
    }
  }
  // softmax over the keys of this lane's query, in base 2: exp(x / 8 - max) = exp2((x - max') * log2(e) / 8)
  const float kScale = 0.125f * 1.44269504088896340736f;
  float m = -3.0e38f;
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int key = 32 * j + 8 * (v >> 2) + 4 * hi + (v & 3);
      sc[j][v] = key < S ? sc[j][v] * kScale : -3.0e38f;
      m = fmaxf(m, sc[j][v]);
    }
  m = fmaxf(m, __shfl_xor(m, 32, 64));
  float sum = 0.f;
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int key = 32 * j + 8 * (v >> 2) + 4 * hi + (v & 3);
      sc[j][v] = key < S ? __builtin_amdgcn_exp2f(sc[j][v] - m) : 0.f;
      sum += sc[j][v];
    }
  sum += __shfl_xor(sum, 32, 64);
  const float inv = 1.f / sum;
  __syncthreads();                     // V^T complete (all waves)
  f32x16 oc[2];
#pragma unroll
  for (int jd = 0; jd < 2; ++jd)
#pragma unroll
    for (int v = 0; v < 16; ++v) oc[jd][v] = 0.f;
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int ap = 0; ap < 2; ++ap) {
      // probabilities rounded to bf16: elements 8 ap .. 8 ap + 7 of the key block
      u32x4 pw;
      pw.x = pack_bf16x2(sc[j][8 * ap + 0] * inv, sc[j][8 * ap + 1] * inv);
      pw.y = pack_bf16x2(sc[j][8 * ap + 2] * inv, sc[j][8 * ap + 3] * inv);
      pw.z = pack_bf16x2(sc[j][8 * ap + 4] * inv, sc[j][8 * ap + 5] * inv);
      pw.w = pack_bf16x2(sc[j][8 * ap + 6] * inv, sc[j][8 * ap + 7] * inv);
      const int key0 = 32 * j + 16 * ap + 4 * hi;
#pragma unroll
      for (int jd = 0; jd < 2; ++jd) {
        const bf16_t* vrow = Vt + (jd * 32 + r32) * AT_LD + key0;
        const uint2 v0 = *(const uint2*)vrow, v1 = *(const uint2*)(vrow + 8);
        const u32x4 vw = {v0.x, v0.y, v1.x, v1.y};
        oc[jd] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, pw), __builtin_bit_cast(bf16x8, vw), oc[jd], 0, 0, 0);
      }
    }
  bf16_t* O = (bf16_t*)p.o + (long)b * S * ld + h * AT_D;
#pragma unroll
  for (int jd = 0; jd < 2; ++jd)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int row = wave * 32 + 8 * (v >> 2) + 4 * hi + (v & 3);
      if (row < S) O[(long)row * ld + jd * 32 + r32] = f32_to_bf16(oc[jd][v]);
    }
}

hipError_t launch_attention(const AttnGroupArgs& a, hipStream_t s) {
  if (a.n == 0) return hipSuccess;
  AttnGroupArgs b = a;
  int start = 0;
  for (int i = 0; i < b.n; ++i) {
    if (b.p[i].S > AT_S || b.p[i].S < 1 || b.p[i].ld % 8) return hipErrorInvalidValue;
    b.p[i].tile_start = start;
    b.p[i].tiles = b.p[i].B * b.p[i].heads;
    start += b.p[i].tiles;
  }
  hipLaunchKernelGGL(attention_kernel, dim3(start), dim3(256), 0, s, b);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// LayerNorm over the last dimension, one wave per row; the row stays in registers between the
// mean, variance and normalise passes.  cols is a multiple of 8 and at most 2048.
// ---------------------------------------------------------------------------------------------
constexpr int LN_MAX_OCT = 4;      // octets per lane -> cols <= 2048

__global__ __launch_bounds__(256) void layernorm_kernel(const LnGroupArgs args) {
  const int g = find_problem(args, blockIdx.x);
  const LnProblem& p = args.p[g];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const long row = (long)(blockIdx.x - p.tile_start) * 4 + wave;
  if (row >= p.rows) return;
  const int octs = p.cols >> 3;
  const bf16_t* x = (const bf16_t*)p.x + row * p.cols;
  float v[LN_MAX_OCT][8];
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < LN_MAX_OCT; ++i) {
    const int o = lane + 64 * i;
    if (o < octs) {
      const uint4 u = *(const uint4*)(x + o * 8);
      const unsigned w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        v[i][2 * e] = __uint_as_float(w[e] << 16);
        v[i][2 * e + 1] = __uint_as_float(w[e] & 0xffff0000u);
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) sum += v[i][e];
    }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off, 64);
  const float mean = sum / (float)p.cols;
  float sq = 0.f;
#pragma unroll
  for (int i = 0; i < LN_MAX_OCT; ++i)
    if (lane + 64 * i < octs) {
#pragma unroll
      for (int e = 0; e < 8; ++e) { const float d = v[i][e] - mean; sq = fmaf(d, d, sq); }
    }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) sq += __shfl_xor(sq, off, 64);
  const float rstd = 1.f / sqrtf(sq / (float)p.cols + 1e-5f);
  bf16_t* y = (bf16_t*)p.y + row * p.cols;
#pragma unroll
  for (int i = 0; i < LN_MAX_OCT; ++i) {
    const int o = lane + 64 * i;
    if (o < octs) {
      float r[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) r[e] = fmaf((v[i][e] - mean) * rstd, p.gamma[o * 8 + e], p.beta[o * 8 + e]);
      uint4 out;
      out.x = pack_bf16x2(r[0], r[1]);
      out.y = pack_bf16x2(r[2], r[3]);
      out.z = pack_bf16x2(r[4], r[5]);
      out.w = pack_bf16x2(r[6], r[7]);
      *(uint4*)(y + o * 8) = out;
    }
  }
}

hipError_t launch_layernorm(const LnGroupArgs& a, hipStream_t s) {
  if (a.n == 0) return hipSuccess;
  LnGroupArgs b = a;
  int start = 0;
  for (int i = 0; i < b.n; ++i) {
    if (b.p[i].cols % 8 || b.p[i].cols > 8 * 64 * LN_MAX_OCT) return hipErrorInvalidValue;
    b.p[i].tile_start = start;
    b.p[i].tiles = (b.p[i].rows + 3) / 4;
    start += b.p[i].tiles;
  }
  hipLaunchKernelGGL(layernorm_kernel, dim3(start), dim3(256), 0, s, b);
  return hipGetLastError();
}

}  // namespace sna
