// Depthwise WeightSlice convolution (centre k x k window of a stored 7x7, leading channels) with
// fused SubnetNorm + activation, and the squeeze-excite gate.  All of it is HBM-bound streaming:
// threads own 8 consecutive channels (16-byte loads / stores, channel-fastest across lanes).
#include "common.h"

namespace sna {

__device__ __forceinline__ void unpack8(const uint4 v, float* f) {
  const unsigned u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    f[2 * e] = __uint_as_float(u[e] << 16);
    f[2 * e + 1] = __uint_as_float(u[e] & 0xffff0000u);
  }
}
__device__ __forceinline__ uint4 pack8(const float* f) {
  uint4 o;
  o.x = pack_bf16x2(f[0], f[1]);
  o.y = pack_bf16x2(f[2], f[3]);
  o.z = pack_bf16x2(f[4], f[5]);
  o.w = pack_bf16x2(f[6], f[7]);
  return o;
}

// ---------------------------------------------------------------------------------------------
// One thread = TW adjacent output pixels of one row x 8 channels.  For every kernel row the
// thread loads the (TW-1)*STRIDE + K input columns it needs once and reuses them across its TW
// outputs, so an input element is fetched K (not K*K) times per output row from L1/L2 and once
// from HBM.  y = act(scale[c] * sum_{r,s} x * w[r0+r][s0+s][c] + shift[c]).
// ---------------------------------------------------------------------------------------------
constexpr int DW_TW = 4;

template <int K, int STRIDE>
__global__ __launch_bounds__(256) void depthwise_kernel(const DwGroupArgs args) {
  const int g = find_problem(args, blockIdx.x);
  const DwProblem& p = args.p[g];
  const int c8n = p.C >> 3;
  const int strips = (p.Wo + DW_TW - 1) / DW_TW;
  const long idx = (long)(blockIdx.x - p.tile_start) * 256 + threadIdx.x;
  const long total = (long)p.N * p.Ho * strips * c8n;
  if (idx >= total) return;
  const int c8 = idx % c8n;
  long t = idx / c8n;
  const int qs = t % strips; t /= strips;
  const int pp = t % p.Ho;
  const int n = t / p.Ho;
  const int q0 = qs * DW_TW;
  constexpr int COLS = (DW_TW - 1) * STRIDE + K;
  constexpr int PAD = K / 2;
  const bf16_t* x = (const bf16_t*)p.x + (long)n * p.H * p.W * p.C + c8 * 8;
  const bf16_t* w = (const bf16_t*)p.w + c8 * 8;           // already at the centre window's first tap
  // The taps of a kernel row are taken two at a time with v_dot2_f32_bf16: per channel one register
  // holds (x[col], x[col + 1]) and one (w[s], w[s + 1]), built from the channel-pair words of memory with
  // byte permutes; no bf16 -> fp32 unpacking and half the multiply-add instructions.  An odd last tap
  // is paired with a zero weight.
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  constexpr int WP = (K + 1) / 2;                          // tap pairs per kernel row
  constexpr int CSTEP = STRIDE == 2 ? 2 : 1;                 // stride 2 only ever pairs (even, odd) columns
  float acc[DW_TW][8];
#pragma unroll
  for (int o = 0; o < DW_TW; ++o)
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[o][e] = 0.f;
  const int iw0 = q0 * STRIDE - PAD;
#pragma unroll
  for (int r = 0; r < K; ++r) {
    const int ih = pp * STRIDE + r - PAD;
    if (ih < 0 || ih >= p.H) continue;
    uint4 raw[COLS + 1];
#pragma unroll
    for (int cidx = 0; cidx < COLS; ++cidx) {
      const int iw = iw0 + cidx;
      raw[cidx] = (iw >= 0 && iw < p.W) ? *(const uint4*)(x + ((long)ih * p.W + iw) * p.C) : make_uint4(0, 0, 0, 0);
    }
    raw[COLS] = make_uint4(0, 0, 0, 0);
    unsigned wp[WP][8];                    // [tap pair][channel]: (w[2t], w[2t + 1])
#pragma unroll
    for (int t = 0; t < WP; ++t) {
      const uint4 w0 = *(const uint4*)(w + (long)r * p.wr + (long)(2 * t) * p.ws);
      const uint4 w1 = 2 * t + 1 < K ? *(const uint4*)(w + (long)r * p.wr + (long)(2 * t + 1) * p.ws) : make_uint4(0, 0, 0, 0);
      const unsigned a0[4] = {w0.x, w0.y, w0.z, w0.w}, a1[4] = {w1.x, w1.y, w1.z, w1.w};
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        wp[t][2 * d] = __builtin_amdgcn_perm(a1[d], a0[d], 0x05040100u);
        wp[t][2 * d + 1] = __builtin_amdgcn_perm(a1[d], a0[d], 0x07060302u);
      }
    }
#pragma unroll
    for (int c = 0; c < COLS; c += CSTEP) {
      // is this column pair the start of a tap pair of some output?  (c = o * STRIDE + 2 t)
      bool used = false;
#pragma unroll
      for (int o = 0; o < DW_TW; ++o)
#pragma unroll
        for (int t = 0; t < WP; ++t) used = used || (c == o * STRIDE + 2 * t);
      if (!used) continue;
      const unsigned x0[4] = {raw[c].x, raw[c].y, raw[c].z, raw[c].w};
      const unsigned x1[4] = {raw[c + 1].x, raw[c + 1].y, raw[c + 1].z, raw[c + 1].w};
      unsigned xp[8];                      // [channel]: (x[col c], x[col c + 1])
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        xp[2 * d] = __builtin_amdgcn_perm(x1[d], x0[d], 0x05040100u);
        xp[2 * d + 1] = __builtin_amdgcn_perm(x1[d], x0[d], 0x07060302u);
      }
#pragma unroll
      for (int o = 0; o < DW_TW; ++o)
#pragma unroll
        for (int t = 0; t < WP; ++t)
          if (c == o * STRIDE + 2 * t) {
#pragma unroll
            for (int e = 0; e < 8; ++e)
              acc[o][e] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, xp[e]),
                                                          __builtin_bit_cast(bf16x2_t, wp[t][e]), acc[o][e], false);
          }
    }
  }
  float sc[8], sh[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) { sc[e] = p.scale[c8 * 8 + e]; sh[e] = p.shift[c8 * 8 + e]; }
  bf16_t* y = (bf16_t*)p.y + (((long)n * p.Ho + pp) * p.Wo) * p.C + c8 * 8;
#pragma unroll
  for (int o = 0; o < DW_TW; ++o) {
    if (q0 + o >= p.Wo) break;
    float v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = apply_act(fmaf(acc[o][e], sc[e], sh[e]), p.act);
    *(uint4*)(y + (long)(q0 + o) * p.C) = pack8(v);
  }
}

hipError_t launch_depthwise(const DwGroupArgs& a, hipStream_t s) {
  // one launch per (kernel size, stride) present among the problems
  for (int k = 3; k <= 7; k += 2)
    for (int st = 1; st <= 2; ++st) {
      DwGroupArgs b;
      b.n = 0;
      int start = 0;
      for (int i = 0; i < a.n; ++i) {
        if (a.p[i].k != k || a.p[i].stride != st) continue;
        DwProblem p = a.p[i];
        const long strips = (p.Wo + DW_TW - 1) / DW_TW;
        p.tiles = (int)(((long)p.N * p.Ho * strips * (p.C / 8) + 255) / 256);
        p.tile_start = start;
        start += p.tiles;
        b.p[b.n++] = p;
      }
      if (!b.n) continue;
#define SNA_DW(KK, SS) if (k == KK && st == SS) hipLaunchKernelGGL((depthwise_kernel<KK, SS>), dim3(start), dim3(256), 0, s, b)
      SNA_DW(3, 1); SNA_DW(3, 2); SNA_DW(5, 1); SNA_DW(5, 2); SNA_DW(7, 1); SNA_DW(7, 2);
#undef SNA_DW
      hipError_t e = hipGetLastError();
      if (e != hipSuccess) return e;
    }
  return hipSuccess;
}

// ---------------------------------------------------------------------------------------------
// Squeeze-excite gate:
//   z = pooled[n][:C] (fp32 mean over pixels, computed by the pooling kernel)
//   h = relu(W1[:Q,:C] z + b1[:Q]);  gate = hardsigmoid(W2[:C,:Q] h + b2[:C])
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// One fully-connected layer of the gate: out[n][o] = f(W[o, :I] . in[n][:I] + b[o]) for o < O.
// A block owns one request and 32 outputs; each of its 4 waves computes 8 of them, one at a
// time: lanes read 8 consecutive bf16 weights (16 bytes) and the matching fp32 inputs, then the
// wave reduces in a fixed butterfly order.  HSIG selects hard-sigmoid (second layer) or ReLU.
template <bool HSIG>
__global__ __launch_bounds__(256) void se_fc_kernel(const SeGroupArgs args) {
  const int g = find_problem(args, blockIdx.x);
  const SeProblem& p = args.p[g];
  const int I = HSIG ? p.Q : p.C, O = HSIG ? p.C : p.Q;
  const int oblocks = (O + 31) / 32;
  const int local = blockIdx.x - p.tile_start;
  const int n = local / oblocks, ob = local % oblocks;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const bf16_t* w = (const bf16_t*)(HSIG ? p.w2 : p.w1);
  const int ws = HSIG ? p.w2_stride : p.w1_stride;
  const float* bias = HSIG ? p.b2 : p.b1;
  const float* in = (HSIG ? p.hidden : p.pooled) + (long)n * I;
  float* out = (HSIG ? p.gate : p.hidden) + (long)n * O;
#pragma unroll 1
  for (int t = 0; t < 8; ++t) {
    const int o = ob * 32 + wave * 8 + t;
    if (o >= O) break;
    float a = 0.f;
    for (int i8 = lane; i8 < (I >> 3); i8 += 64) {
      float wv[8];
      unpack8(*(const uint4*)(w + (long)o * ws + i8 * 8), wv);
      float4 x0 = *(const float4*)(in + i8 * 8), x1 = *(const float4*)(in + i8 * 8 + 4);
      if (!HSIG && p.pool_segs > 1) {           // the pool left segment sums: add them in order, then scale
        for (int sgm = 1; sgm < p.pool_segs; ++sgm) {
          const float* ins = in + (long)sgm * p.N * I;
          const float4 y0 = *(const float4*)(ins + i8 * 8), y1 = *(const float4*)(ins + i8 * 8 + 4);
          x0.x += y0.x; x0.y += y0.y; x0.z += y0.z; x0.w += y0.w;
          x1.x += y1.x; x1.y += y1.y; x1.z += y1.z; x1.w += y1.w;
        }
        x0.x *= p.inv_hw; x0.y *= p.inv_hw; x0.z *= p.inv_hw; x0.w *= p.inv_hw;
        x1.x *= p.inv_hw; x1.y *= p.inv_hw; x1.z *= p.inv_hw; x1.w *= p.inv_hw;
      }
      a = fmaf(wv[0], x0.x, a); a = fmaf(wv[1], x0.y, a); a = fmaf(wv[2], x0.z, a); a = fmaf(wv[3], x0.w, a);
      a = fmaf(wv[4], x1.x, a); a = fmaf(wv[5], x1.y, a); a = fmaf(wv[6], x1.z, a); a = fmaf(wv[7], x1.w, a);
    }
    a = wave_sum(a);
    if (lane == 0) {
      a += bias[o];
      out[o] = HSIG ? fminf(fmaxf(a + 3.f, 0.f), 6.f) * (1.f / 6.f) : fmaxf(a, 0.f);
    }
  }
}

// y[n, hw, c] = bf16(x[n, hw, c] * gate[n, c])
__global__ __launch_bounds__(256) void se_scale_kernel(const SeGroupArgs args) {
  const int g = find_problem(args, blockIdx.x);
  const SeProblem& p = args.p[g];
  const int c8n = p.C >> 3;
  const long idx = (long)(blockIdx.x - p.tile_start) * 256 + threadIdx.x;
  const long total = (long)p.N * p.HW * c8n;
  if (idx >= total) return;
  const int c8 = idx % c8n;
  const long pix = idx / c8n;
  const int n = pix / p.HW;
  float v[8];
  unpack8(*(const uint4*)((const bf16_t*)p.x + pix * p.C + c8 * 8), v);
  const float* gt = p.gate + (long)n * p.C + c8 * 8;
#pragma unroll
  for (int e = 0; e < 8; ++e) v[e] *= gt[e];
  *(uint4*)((bf16_t*)p.y + pix * p.C + c8 * 8) = pack8(v);
}

hipError_t launch_se(const SeGroupArgs& a, hipStream_t s) {
  if (a.n == 0) return hipSuccess;
  SeGroupArgs b = a;
  int start = 0;
  for (int i = 0; i < b.n; ++i) {
    if (b.p[i].C % 8 || b.p[i].Q % 8 || b.p[i].w1_stride % 8 || b.p[i].w2_stride % 8) return hipErrorInvalidValue;
    b.p[i].tiles = b.p[i].N * ((b.p[i].Q + 31) / 32);
    b.p[i].tile_start = start; start += b.p[i].tiles;
  }
  hipLaunchKernelGGL(se_fc_kernel<false>, dim3(start), dim3(256), 0, s, b);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  start = 0;
  for (int i = 0; i < b.n; ++i) {
    b.p[i].tiles = b.p[i].N * ((b.p[i].C + 31) / 32);
    b.p[i].tile_start = start; start += b.p[i].tiles;
  }
  hipLaunchKernelGGL(se_fc_kernel<true>, dim3(start), dim3(256), 0, s, b);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  start = 0;
  for (int i = 0; i < b.n; ++i) {
    const long total = (long)b.p[i].N * b.p[i].HW * (b.p[i].C / 8);
    b.p[i].tiles = (int)((total + 255) / 256);
    b.p[i].tile_start = start; start += b.p[i].tiles;
  }
  hipLaunchKernelGGL(se_scale_kernel, dim3(start), dim3(256), 0, s, b);
  return hipGetLastError();
}

}  // namespace sna
