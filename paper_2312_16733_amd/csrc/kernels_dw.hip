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
//
// POOL (the layer feeds a squeeze-excite gate): blocks are laid out per request, and each block
// also leaves the per-channel sum of the outputs it stored (the rounded values, which is what the
// gate's average pool is defined on), added in a fixed order: per thread over its outputs, then over
// the block's threads of one channel group in thread order.  The gate adds the blocks' sums in order.
// ---------------------------------------------------------------------------------------------
constexpr int DW_TW = 4;

template <int K, int STRIDE, bool POOL>
__global__ __launch_bounds__(256) void depthwise_kernel(const DwGroupArgs args) {
  const int g = find_problem(args, blockIdx.x);
  const DwProblem& p = args.p[g];
  const int c8n = p.C >> 3;
  const int strips = (p.Wo + DW_TW - 1) / DW_TW;
  const long per_req = (long)p.Ho * strips * c8n;
  const int block = blockIdx.x - p.tile_start;
  long idx;
  bool valid;
  if (POOL) {
    const long in_req = (long)(block % p.bpr) * 256 + threadIdx.x;
    valid = in_req < per_req;
    idx = (long)(block / p.bpr) * per_req + in_req;
  } else {
    idx = (long)block * 256 + threadIdx.x;
    valid = idx < per_req * p.N;
    if (!valid) return;
  }
  float psum[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) psum[e] = 0.f;
  if (valid) {
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
  if (p.raw_out) {
    float* yr = (float*)p.y + (((long)n * p.Ho + pp) * p.Wo) * p.C + c8 * 8;
#pragma unroll
    for (int o = 0; o < DW_TW; ++o) {
      if (q0 + o >= p.Wo) break;
      *(float4*)(yr + (long)(q0 + o) * p.C) = make_float4(acc[o][0], acc[o][1], acc[o][2], acc[o][3]);
      *(float4*)(yr + (long)(q0 + o) * p.C + 4) = make_float4(acc[o][4], acc[o][5], acc[o][6], acc[o][7]);
    }
    return;
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
    const uint4 packed = pack8(v);
    *(uint4*)(y + (long)(q0 + o) * p.C) = packed;
    if (POOL) {
      unpack8(packed, v);
#pragma unroll
      for (int e = 0; e < 8; ++e) psum[e] += v[e];
    }
  }
  }
  if (POOL) {
    __shared__ float red[8][256];
#pragma unroll
    for (int e = 0; e < 8; ++e) red[e][threadIdx.x] = psum[e];
    __syncthreads();
    // thread t < c8n owns the channel group of the block's t-th element; its other elements sit c8n apart
    if ((int)threadIdx.x < c8n) {
      const int in_block = block % p.bpr;
      const int c8 = (int)(((long)in_block * 256 + threadIdx.x) % c8n);
      float s8[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) s8[e] = 0.f;
      for (int t = threadIdx.x; t < 256; t += c8n)
#pragma unroll
        for (int e = 0; e < 8; ++e) s8[e] += red[e][t];
      float* out = p.pool_part + ((long)block * p.C) + c8 * 8;     // block = n * bpr + in_block
      *(float4*)out = make_float4(s8[0], s8[1], s8[2], s8[3]);
      *(float4*)(out + 4) = make_float4(s8[4], s8[5], s8[6], s8[7]);
    }
  }
}

hipError_t launch_depthwise(const DwGroupArgs& a, hipStream_t s) {
  // one launch per (kernel size, stride, with / without pool) present among the problems
  for (int pool = 0; pool < 2; ++pool)
    for (int k = 3; k <= 7; k += 2)
      for (int st = 1; st <= 2; ++st) {
        DwGroupArgs b;
        b.n = 0;
        int start = 0;
        for (int i = 0; i < a.n; ++i) {
          if (a.p[i].k != k || a.p[i].stride != st || (a.p[i].pool_part != nullptr) != (pool == 1)) continue;
          DwProblem p = a.p[i];
          const long strips = (p.Wo + DW_TW - 1) / DW_TW;
          const long per_req = (long)p.Ho * strips * (p.C / 8);
          if (pool) {
            // every block must meet every channel group, or some sums would never be written
            if (p.C / 8 > 256 || p.bpr != (int)((per_req + 255) / 256)) return hipErrorInvalidValue;
            p.tiles = p.N * p.bpr;
          } else {
            p.tiles = (int)((per_req * p.N + 255) / 256);
          }
          p.tile_start = start;
          start += p.tiles;
          b.p[b.n++] = p;
        }
        if (!b.n) continue;
#define SNA_DW(KK, SS)                                                                                              \
  if (k == KK && st == SS) {                                                                                        \
    if (pool) hipLaunchKernelGGL((depthwise_kernel<KK, SS, true>), dim3(start), dim3(256), 0, s, b);               \
    else hipLaunchKernelGGL((depthwise_kernel<KK, SS, false>), dim3(start), dim3(256), 0, s, b);                   \
  }
        SNA_DW(3, 1); SNA_DW(3, 2); SNA_DW(5, 1); SNA_DW(5, 2); SNA_DW(7, 1); SNA_DW(7, 2);
#undef SNA_DW
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
      }
  return hipSuccess;
}

int depthwise_pool_blocks(int Ho, int Wo, int C) {
  const long strips = (Wo + DW_TW - 1) / DW_TW;
  return (int)(((long)Ho * strips * (C / 8) + 255) / 256);
}

// ---------------------------------------------------------------------------------------------
// Squeeze-excite gate:
//   z = mean over pixels of the depthwise output (from the depthwise blocks' partial sums)
//   h = relu(W1[:Q,:C] z + b1[:Q]);  gate = hardsigmoid(W2[:C,:Q] h + b2[:C]);  y = x * gate
// Two launches: h per request, then gate and scaling together.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// h[n][o] = relu(W1[o, :C] . z[n] + b1[o]).  A block owns one request and 32 outputs.  It first
// builds z in LDS (partial sums added in block order, then scaled by 1 / HW); each of its 4 waves
// then computes 8 outputs together: lanes read 8 consecutive bf16 weights (16 bytes) of each row and
// the matching z, and the wave reduces each output in a fixed butterfly order.
__global__ __launch_bounds__(256) void se_hidden_kernel(const SeGroupArgs args) {
  extern __shared__ __attribute__((aligned(16))) float z[];
  const int g = find_problem(args, blockIdx.x);
  const SeProblem& p = args.p[g];
  const int oblocks = (p.Q + 31) / 32;
  const int local = blockIdx.x - p.tile_start;
  const int n = local / oblocks, ob = local % oblocks;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const float* part = p.pooled + (long)n * p.pool_segs * p.C;
  for (int c4 = threadIdx.x; c4 < (p.C >> 2); c4 += 256) {
    float4 a = *(const float4*)(part + c4 * 4);
#pragma unroll 8                                    // loads in batches of 8, the additions still in block order
    for (int sgm = 1; sgm < p.pool_segs; ++sgm) {
      const float4 b = *(const float4*)(part + (long)sgm * p.C + c4 * 4);
      a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
    }
    a.x *= p.inv_hw; a.y *= p.inv_hw; a.z *= p.inv_hw; a.w *= p.inv_hw;
    *(float4*)(z + c4 * 4) = a;
  }
  __syncthreads();
  // the wave's 8 rows are independent: all their weight loads are issued before the first sum is needed
  // (one row at a time paid the L2 latency 8 times over)
  const bf16_t* w = (const bf16_t*)p.w1;
  const int o0 = ob * 32 + wave * 8;
  float a[8];
#pragma unroll
  for (int t = 0; t < 8; ++t) a[t] = 0.f;
  for (int i8 = lane; i8 < (p.C >> 3); i8 += 64) {
    const float4 x0 = *(const float4*)(z + i8 * 8), x1 = *(const float4*)(z + i8 * 8 + 4);
    uint4 wq[8];
#pragma unroll
    for (int t = 0; t < 8; ++t)
      wq[t] = o0 + t < p.Q ? *(const uint4*)(w + (long)(o0 + t) * p.w1_stride + i8 * 8) : make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      float wv[8];
      unpack8(wq[t], wv);
      a[t] = fmaf(wv[0], x0.x, a[t]); a[t] = fmaf(wv[1], x0.y, a[t]); a[t] = fmaf(wv[2], x0.z, a[t]); a[t] = fmaf(wv[3], x0.w, a[t]);
      a[t] = fmaf(wv[4], x1.x, a[t]); a[t] = fmaf(wv[5], x1.y, a[t]); a[t] = fmaf(wv[6], x1.z, a[t]); a[t] = fmaf(wv[7], x1.w, a[t]);
    }
  }
#pragma unroll
  for (int t = 0; t < 8; ++t) {
    const float sum = wave_sum(a[t]);
    if (lane == 0 && o0 + t < p.Q) p.hidden[(long)n * p.Q + o0 + t] = fmaxf(sum + p.b1[o0 + t], 0.f);
  }
}

// gate[n][c] = hardsigmoid(W2[c, :Q] . h[n] + b2[c]);  y[n, hw, c] = bf16(x[n, hw, c] * gate[n][c]).
// A block owns one request, 64 channels and SE_PIX pixels: its threads first compute the 64 gate
// values (4 threads per channel, each a quarter of Q in order, the quarters added in order), then
// stream the pixels, 8 lanes per pixel row of 128 bytes.  The gate is recomputed by every pixel
// segment of a request: 64 x Q multiply-adds against one more launch and a round trip through memory.
constexpr int SE_PIX = 256;
constexpr int SE_MAX_Q = 512;       // squeeze channels per gate (host-checked)
__global__ __launch_bounds__(256) void se_gate_scale_kernel(const SeGroupArgs args) {
  __shared__ float gate_s[64];
  __shared__ __attribute__((aligned(16))) float h_s[SE_MAX_Q];
  const int g = find_problem(args, blockIdx.x);
  const SeProblem& p = args.p[g];
  const int cgroups = (p.C + 63) / 64, psegs = (p.HW + SE_PIX - 1) / SE_PIX;
  int local = blockIdx.x - p.tile_start;
  const int pseg = local % psegs; local /= psegs;
  const int cg = local % cgroups;
  const int n = local / cgroups;
  // the thread's pixels do not depend on the gate: request them first, so that their latency runs
  // under the gate computation
  const int c8 = cg * 8 + (threadIdx.x & 7);
  const bool live = c8 * 8 < p.C;
  const int h_end = (pseg + 1) * SE_PIX < p.HW ? (pseg + 1) * SE_PIX : p.HW;
  const int h0 = pseg * SE_PIX + (threadIdx.x >> 3);
  const bf16_t* x = (const bf16_t*)p.x + (long)n * p.HW * p.C + c8 * 8;
  uint4 px[SE_PIX / 32];
#pragma unroll
  for (int j = 0; j < SE_PIX / 32; ++j)
    px[j] = (live && h0 + 32 * j < h_end) ? *(const uint4*)(x + (long)(h0 + 32 * j) * p.C) : make_uint4(0, 0, 0, 0);
  for (int i = threadIdx.x; i < p.Q; i += 256) h_s[i] = p.hidden[(long)n * p.Q + i];
  __syncthreads();
  {
    const int c = cg * 64 + (threadIdx.x >> 2), quarter = threadIdx.x & 3;
    const int q8n = p.Q >> 3, per = (q8n + 3) >> 2;          // per <= SE_MAX_Q / 32
    float a = 0.f;
    if (c < p.C) {
      const bf16_t* w = (const bf16_t*)p.w2 + (long)c * p.w2_stride;
      const int end = (quarter + 1) * per < q8n ? (quarter + 1) * per : q8n;
      // fixed trip count, loads first: a loop over [begin, end) paid the L2 latency once per 8 weights
      uint4 wq[SE_MAX_Q / 32];
#pragma unroll
      for (int j = 0; j < SE_MAX_Q / 32; ++j) {
        const int i8 = quarter * per + j;
        wq[j] = (j < per && i8 < end) ? *(const uint4*)(w + i8 * 8) : make_uint4(0, 0, 0, 0);
      }
#pragma unroll
      for (int j = 0; j < SE_MAX_Q / 32; ++j) {
        const int i8 = quarter * per + j;
        if (j < per && i8 < end) {
          float wv[8];
          unpack8(wq[j], wv);
          const float4 x0 = *(const float4*)(h_s + i8 * 8), x1 = *(const float4*)(h_s + i8 * 8 + 4);
          a = fmaf(wv[0], x0.x, a); a = fmaf(wv[1], x0.y, a); a = fmaf(wv[2], x0.z, a); a = fmaf(wv[3], x0.w, a);
          a = fmaf(wv[4], x1.x, a); a = fmaf(wv[5], x1.y, a); a = fmaf(wv[6], x1.z, a); a = fmaf(wv[7], x1.w, a);
        }
      }
    }
    // quarters 0..3 of a channel sit in adjacent lanes: ((q0 + q1) + (q2 + q3))
    a += __shfl_xor(a, 1, 64);
    a += __shfl_xor(a, 2, 64);
    if (quarter == 0 && c < p.C) gate_s[threadIdx.x >> 2] = fminf(fmaxf(a + p.b2[c] + 3.f, 0.f), 6.f) * (1.f / 6.f);
  }
  __syncthreads();
  if (!live) return;
  float gt[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) gt[e] = gate_s[(threadIdx.x & 7) * 8 + e];
  bf16_t* y = (bf16_t*)p.y + (long)n * p.HW * p.C + c8 * 8;
#pragma unroll
  for (int j = 0; j < SE_PIX / 32; ++j) {
    const int h = h0 + 32 * j;
    if (h >= h_end) break;
    float v[8];
    unpack8(px[j], v);
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] *= gt[e];
    *(uint4*)(y + (long)h * p.C) = pack8(v);
  }
}

hipError_t launch_se(const SeGroupArgs& a, hipStream_t s) {
  if (a.n == 0) return hipSuccess;
  SeGroupArgs b = a;
  int start = 0, c_max = 0;
  for (int i = 0; i < b.n; ++i) {
    if (b.p[i].C % 8 || b.p[i].Q % 8 || b.p[i].Q > SE_MAX_Q || b.p[i].w1_stride % 8 || b.p[i].w2_stride % 8 || b.p[i].pool_segs < 1)
      return hipErrorInvalidValue;
    b.p[i].tiles = b.p[i].N * ((b.p[i].Q + 31) / 32);
    b.p[i].tile_start = start; start += b.p[i].tiles;
    if (b.p[i].C > c_max) c_max = b.p[i].C;
  }
  if (c_max * 4 > 64 * 1024) return hipErrorInvalidValue;
  hipLaunchKernelGGL(se_hidden_kernel, dim3(start), dim3(256), c_max * 4, s, b);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  start = 0;
  for (int i = 0; i < b.n; ++i) {
    b.p[i].tiles = b.p[i].N * ((b.p[i].C + 63) / 64) * ((b.p[i].HW + SE_PIX - 1) / SE_PIX);
    b.p[i].tile_start = start; start += b.p[i].tiles;
  }
  hipLaunchKernelGGL(se_gate_scale_kernel, dim3(start), dim3(256), 0, s, b);
  return hipGetLastError();
}

}  // namespace sna
