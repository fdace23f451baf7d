// Direct convolution (stems, fp32 tiny net), pooling, request gather / scatter and the
// load-time folding of SubnetNorm statistics.  All forward kernels are grouped launches.
#include "common.h"

namespace sna {

// ---------------------------------------------------------------------------------------------
// Direct WeightSlice convolution: one thread = one output pixel x KT consecutive output channels.
// The block's KT-channel slab of the ACTIVE weight slice (leading C input channels, centre RxS
// window) is staged once in LDS as fp32 [R*S*C][KT]; every lane then reads the same LDS address
// (a broadcast) while walking its own input patch.  Used where the input has too few channels
// for the MFMA path (3-channel stems) and for the fp32 family.
// ---------------------------------------------------------------------------------------------
constexpr int DIRECT_KT = 16;
constexpr int DIRECT_THREADS = 256;

template <typename T> __device__ __forceinline__ float ld_f32(const T* p);
template <> __device__ __forceinline__ float ld_f32<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float ld_f32<bf16_t>(const bf16_t* p) { return bf16_to_f32(*p); }
template <typename T> __device__ __forceinline__ void st_f32(T* p, float v);
template <> __device__ __forceinline__ void st_f32<float>(float* p, float v) { *p = v; }
template <> __device__ __forceinline__ void st_f32<bf16_t>(bf16_t* p, float v) { *p = f32_to_bf16(v); }

template <typename T>
__global__ __launch_bounds__(DIRECT_THREADS) void direct_conv_kernel(const ConvGroupArgs args) {
  extern __shared__ float wlds[];                       // [R*S*C][KT]
  const int g = find_problem(args, blockIdx.x);
  const ConvProblem& p = args.p[g];
  const int local = blockIdx.x - p.tile_start;
  const int kt = local % p.tiles_n;                     // channel tile
  const int mt = local / p.tiles_n;                     // pixel tile
  const int k0 = kt * DIRECT_KT;
  const int RSC = p.R * p.S * p.C;
  const T* w = (const T*)p.w;
  for (int i = threadIdx.x; i < RSC * DIRECT_KT; i += DIRECT_THREADS) {
    const int kk = i % DIRECT_KT, e = i / DIRECT_KT;    // e = (r*S + s)*C + c
    const int c = e % p.C, rs = e / p.C;
    const int s = rs % p.S, r = rs / p.S;
    float v = 0.f;
    if (k0 + kk < p.K) v = ld_f32<T>(w + (long)(k0 + kk) * p.wk + (long)r * p.wr + (long)s * p.ws + c);
    wlds[e * DIRECT_KT + kk] = v;
  }
  __syncthreads();
  const int m = mt * DIRECT_THREADS + threadIdx.x;
  if (m >= p.M) return;
  const int q = m % p.Wo, t = m / p.Wo;
  const int pp = t % p.Ho, n = t / p.Ho;
  float acc[DIRECT_KT];
#pragma unroll
  for (int i = 0; i < DIRECT_KT; ++i) acc[i] = 0.f;
  const T* x = (const T*)p.x;
  for (int r = 0; r < p.R; ++r) {
    const int ih = pp * p.stride + r - p.pad;
    if (ih < 0 || ih >= p.H) continue;
    for (int s = 0; s < p.S; ++s) {
      const int iw = q * p.stride + s - p.pad;
      if (iw < 0 || iw >= p.W) continue;
      const T* xp = x + (((long)n * p.H + ih) * p.W + iw) * p.C;
      const float* wp = wlds + (long)((r * p.S + s) * p.C) * DIRECT_KT;
      for (int c = 0; c < p.C; ++c) {
        const float xv = ld_f32<T>(xp + c);
        const float4* w4 = (const float4*)(wp + c * DIRECT_KT);
#pragma unroll
        for (int i = 0; i < DIRECT_KT / 4; ++i) {
          const float4 wv = w4[i];
          acc[4 * i + 0] = fmaf(xv, wv.x, acc[4 * i + 0]);
          acc[4 * i + 1] = fmaf(xv, wv.y, acc[4 * i + 1]);
          acc[4 * i + 2] = fmaf(xv, wv.z, acc[4 * i + 2]);
          acc[4 * i + 3] = fmaf(xv, wv.w, acc[4 * i + 3]);
        }
      }
    }
  }
#pragma unroll
  for (int i = 0; i < DIRECT_KT; ++i) {
    const int k = k0 + i;
    if (k < p.K) {
      float v = acc[i];
      v = fmaf(v, p.scale ? p.scale[k] : 1.f, p.shift ? p.shift[k] : 0.f);
      if (p.res && !p.res_after_act) v += ld_f32<T>((const T*)p.res + (long)m * p.res_stride + k);
      v = apply_act(v, p.act);
      if (p.res && p.res_after_act) v += ld_f32<T>((const T*)p.res + (long)m * p.res_stride + k);
      if (p.out_fp32) ((float*)p.y)[(long)m * p.y_stride + k] = v;
      else st_f32<T>((T*)p.y + (long)m * p.y_stride + k, v);
    }
  }
}

size_t direct_lds_bytes(const ConvGroupArgs& a) {
  size_t mx = 0;
  for (int i = 0; i < a.n; ++i) {
    size_t b = (size_t)a.p[i].R * a.p[i].S * a.p[i].C * DIRECT_KT * sizeof(float);
    mx = b > mx ? b : mx;
  }
  return mx;
}

hipError_t launch_direct_conv(const ConvGroupArgs& a, int dtype, hipStream_t s) {
  if (a.n == 0) return hipSuccess;
  const int blocks = a.p[a.n - 1].tile_start + a.p[a.n - 1].tiles;
  const size_t lds = direct_lds_bytes(a);
  if (lds > 150 * 1024) return hipErrorInvalidValue;
  if (dtype == SNA_DTYPE_FP32) {
    static bool attr32 = false;
    if (!attr32) {
      hipError_t e = hipFuncSetAttribute((const void*)direct_conv_kernel<float>,
                                         hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
      if (e != hipSuccess) return e;
      attr32 = true;
    }
    hipLaunchKernelGGL(direct_conv_kernel<float>, dim3(blocks), dim3(DIRECT_THREADS), lds, s, a);
  } else {
    static bool attr16 = false;
    if (!attr16) {
      hipError_t e = hipFuncSetAttribute((const void*)direct_conv_kernel<bf16_t>,
                                         hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
      if (e != hipSuccess) return e;
      attr16 = true;
    }
    hipLaunchKernelGGL(direct_conv_kernel<bf16_t>, dim3(blocks), dim3(DIRECT_THREADS), lds, s, a);
  }
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// 3x3 / stride 2 / pad 1 max pooling, NHWC.  bf16: one thread = one output pixel x 8 channels
// (16-byte loads and stores); fp32: 4 channels.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void maxpool_bf16_kernel(const PoolGroupArgs args) {
  const int g = find_problem(args, blockIdx.x);
  const PoolProblem& p = args.p[g];
  const int c8n = p.C >> 3;
  const long idx = (long)(blockIdx.x - p.tile_start) * 256 + threadIdx.x;
  const long total = (long)p.N * p.Ho * p.Wo * c8n;
  if (idx >= total) return;
  const int c8 = idx % c8n;
  long t = idx / c8n;
  const int q = t % p.Wo; t /= p.Wo;
  const int pp = t % p.Ho;
  const int n = t / p.Ho;
  float best[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) best[i] = -3.0e38f;
  const bf16_t* x = (const bf16_t*)p.x;
  for (int r = 0; r < 3; ++r) {
    const int ih = 2 * pp + r - 1;
    if (ih < 0 || ih >= p.H) continue;
    for (int s = 0; s < 3; ++s) {
      const int iw = 2 * q + s - 1;
      if (iw < 0 || iw >= p.W) continue;
      const uint4 v = *(const uint4*)(x + (((long)n * p.H + ih) * p.W + iw) * p.C + c8 * 8);
      const unsigned u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        best[2 * i] = fmaxf(best[2 * i], __uint_as_float(u[i] << 16));
        best[2 * i + 1] = fmaxf(best[2 * i + 1], __uint_as_float(u[i] & 0xffff0000u));
      }
    }
  }
  uint4 o;
  unsigned* ou = (unsigned*)&o;
#pragma unroll
  for (int i = 0; i < 4; ++i)   // inputs are bf16 values: the max needs no rounding
    ou[i] = (__float_as_uint(best[2 * i]) >> 16) | (__float_as_uint(best[2 * i + 1]) & 0xffff0000u);
  *(uint4*)((bf16_t*)p.y + (((long)n * p.Ho + pp) * p.Wo + q) * p.C + c8 * 8) = o;
}

hipError_t launch_maxpool(const PoolGroupArgs& a, int dtype, hipStream_t s) {
  if (a.n == 0) return hipSuccess;
  if (dtype != SNA_DTYPE_BF16) return hipErrorInvalidValue;
  const int blocks = a.p[a.n - 1].tile_start + a.p[a.n - 1].tiles;
  hipLaunchKernelGGL(maxpool_bf16_kernel, dim3(blocks), dim3(256), 0, s, a);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Global average pool [N][HW][C] -> [N][C] in the storage dtype.  A block covers one request and
// 32 channel groups; 8 lanes per group walk HW with stride 8 and are reduced through LDS in a
// fixed order.
// ---------------------------------------------------------------------------------------------
template <typename T, int VEC>
__global__ __launch_bounds__(256) void gap_kernel(const PoolGroupArgs args) {
  __shared__ float red[8][32][VEC];
  const int g = find_problem(args, blockIdx.x);
  const PoolProblem& p = args.p[g];
  const int cvn = p.C / VEC;
  const int cblocks = (cvn + 31) / 32;
  const int local = blockIdx.x - p.tile_start;
  const int n = local / cblocks;
  const int cv = (local % cblocks) * 32 + (threadIdx.x & 31);
  const int hl = threadIdx.x >> 5;
  const int HW = p.H * p.W;
  float acc[VEC];
#pragma unroll
  for (int i = 0; i < VEC; ++i) acc[i] = 0.f;
  if (cv < cvn) {
    const T* x = (const T*)p.x + (long)n * HW * p.C + cv * VEC;
#pragma unroll 4
    for (int h = hl; h < HW; h += 8) {
#pragma unroll
      for (int i = 0; i < VEC; ++i) acc[i] += ld_f32<T>(x + (long)h * p.C + i);
    }
  }
#pragma unroll
  for (int i = 0; i < VEC; ++i) red[hl][threadIdx.x & 31][i] = acc[i];
  __syncthreads();
  if (hl == 0 && cv < cvn) {
    const float inv = 1.f / (float)HW;
    const long yo = (long)n * p.C + cv * VEC;
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
      float sum = 0.f;
#pragma unroll
      for (int j = 0; j < 8; ++j) sum += red[j][threadIdx.x & 31][i];
      if (p.out_fp32) ((float*)p.y)[yo + i] = sum * inv;
      else st_f32<T>((T*)p.y + yo + i, sum * inv);
    }
  }
}

hipError_t launch_gap(const PoolGroupArgs& a, int dtype, hipStream_t s) {
  if (a.n == 0) return hipSuccess;
  const int blocks = a.p[a.n - 1].tile_start + a.p[a.n - 1].tiles;
  if (dtype == SNA_DTYPE_FP32) hipLaunchKernelGGL((gap_kernel<float, 8>), dim3(blocks), dim3(256), 0, s, a);
  else hipLaunchKernelGGL((gap_kernel<bf16_t, 8>), dim3(blocks), dim3(256), 0, s, a);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Gather / scatter of whole requests: block (b, y) copies a share of item b.  16-byte vectors when
// source, destination and length allow it, 2-byte elements otherwise (odd resolutions).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void copy_items_kernel(const CopyArgs args) {
  const CopyItem it = args.it[blockIdx.x];
  const char* s = (const char*)args.src + it.src;
  char* d = (char*)args.dst + it.dst;
  const unsigned long step = (unsigned long)gridDim.y * 256;
  if ((((unsigned long)s | (unsigned long)d | it.n) & 15) == 0) {
    const unsigned long n16 = it.n >> 4;
    for (unsigned long i = blockIdx.y * 256 + threadIdx.x; i < n16; i += step)
      ((uint4*)d)[i] = ((const uint4*)s)[i];
  } else {
    const unsigned long n2 = it.n >> 1;
    for (unsigned long i = blockIdx.y * 256 + threadIdx.x; i < n2; i += step)
      ((unsigned short*)d)[i] = ((const unsigned short*)s)[i];
  }
}

hipError_t launch_copy(const CopyArgs& a, hipStream_t s) {
  if (a.n == 0) return hipSuccess;
  unsigned long mx = 0;
  for (int i = 0; i < a.n; ++i) mx = a.it[i].n > mx ? a.it[i].n : mx;
  long gy = (long)((mx / 16 + 256 * 8 - 1) / (256 * 8));
  gy = gy < 1 ? 1 : (gy > 64 ? 64 : gy);
  hipLaunchKernelGGL(copy_items_kernel, dim3(a.n, (unsigned)gy), dim3(256), 0, s, a);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Channel padding of request inputs: [pixels][c_in] bf16 -> [pixels][8] bf16 with zeros in the
// added channels, so that a narrow-input stem conv can use 16-byte operand loads on the MFMA
// path.  Block (b, y) handles a share of item b; one thread = one pixel (16-byte store).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void pad_input_kernel(const PadArgs args) {
  const PadItem it = args.it[blockIdx.x];
  const bf16_t* s = (const bf16_t*)((const char*)args.src + it.src);
  uint4* d = (uint4*)((char*)args.dst + it.dst);
  const int c = args.c_in;
  for (unsigned long i = blockIdx.y * 256 + threadIdx.x; i < it.pixels; i += (unsigned long)gridDim.y * 256) {
    unsigned v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = e < c ? (unsigned)s[i * c + e] : 0u;
    d[i] = make_uint4(v[0] | (v[1] << 16), v[2] | (v[3] << 16), v[4] | (v[5] << 16), v[6] | (v[7] << 16));
  }
}

hipError_t launch_pad_input(const PadArgs& a, hipStream_t s) {
  if (a.n == 0) return hipSuccess;
  unsigned long mx = 0;
  for (int i = 0; i < a.n; ++i) mx = a.it[i].pixels > mx ? a.it[i].pixels : mx;
  long gy = (long)((mx + 256 * 4 - 1) / (256 * 4));
  gy = gy < 1 ? 1 : (gy > 2048 ? 2048 : gy);
  hipLaunchKernelGGL(pad_input_kernel, dim3(a.n, (unsigned)gy), dim3(256), 0, s, a);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// SubnetNorm calibration (the paper computes every subnet's statistics by forward passes before
// serving).  Per channel, mean and sum of squared deviations are carried as (n, mean, M2) and merged
// pairwise with Chan's formula, always in the same order: a thread takes its rows in groups of 8
// (group mean, then squared deviations from it, all 8 values in registers), merges group after
// group, the 4 row lanes of a block merge in lane order, the row blocks in lane-strided order by 16
// lanes that merge in lane order.  The variance stored is the population one (M2 / n).
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void chan_merge(float& n, float& mean, float& m2, float nb, float meanb, float m2b) {
  if (nb == 0.f) return;
  const float nt = n + nb, d = meanb - mean;
  mean += d * (nb / nt);
  m2 += m2b + d * d * (n * nb / nt);
  n = nt;
}

__global__ __launch_bounds__(256) void channel_stats_partial_kernel(const NormCalArgs a) {
  __shared__ float red[3][4][64];
  const int ch = blockIdx.y * 64 + (threadIdx.x & 63), rl = threadIdx.x >> 6;
  const int r0 = blockIdx.x * SNA_CAL_ROWS;
  const int r1 = r0 + SNA_CAL_ROWS < a.M ? r0 + SNA_CAL_ROWS : a.M;
  float n = 0.f, mean = 0.f, m2 = 0.f;
  if (ch < a.K) {
    const float* src = a.raw + ch;
    for (int r = r0 + rl; r < r1; r += 32) {      // 8 rows of this lane: r, r+4, ..., r+28
      float v[8];
      int cnt = 0;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int rr = r + 4 * j;
        const bool in = rr < r1;
        v[j] = in ? src[(long)rr * a.K] : 0.f;
        cnt += in;
      }
      float sum = 0.f;
#pragma unroll
      for (int j = 0; j < 8; ++j) sum += v[j];
      const float nb = (float)cnt, gm = sum / nb;
      float g2 = 0.f;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float d = (r + 4 * j < r1) ? v[j] - gm : 0.f;
        g2 = fmaf(d, d, g2);
      }
      chan_merge(n, mean, m2, nb, gm, g2);
    }
  }
  red[0][rl][threadIdx.x & 63] = n; red[1][rl][threadIdx.x & 63] = mean; red[2][rl][threadIdx.x & 63] = m2;
  __syncthreads();
  if (rl == 0 && ch < a.K) {
#pragma unroll
    for (int j = 1; j < 4; ++j) chan_merge(n, mean, m2, red[0][j][threadIdx.x], red[1][j][threadIdx.x], red[2][j][threadIdx.x]);
    float* o = a.part + ((long)blockIdx.x * a.K + ch) * 3;
    o[0] = n; o[1] = mean; o[2] = m2;
  }
}

__device__ __forceinline__ void chan_merge_d(double& n, double& mean, double& m2, double nb, double meanb, double m2b) {
  if (nb == 0) return;
  const double nt = n + nb, d = meanb - mean;
  mean += d * (nb / nt);
  m2 += m2b + d * d * (n * nb / nt);
  n = nt;
}

// 16 channels per block, 16 lanes per channel over the row blocks; double precision from here on.
__global__ __launch_bounds__(256) void channel_stats_final_kernel(const NormCalArgs a) {
  __shared__ double red[3][16][16];
  const int cl = threadIdx.x & 15, lane = threadIdx.x >> 4;
  const int ch = blockIdx.x * 16 + cl;
  double n = 0, mean = 0, m2 = 0;
  if (ch < a.K)
    for (int b = lane; b < a.nrb; b += 16) {
      const float* q = a.part + ((long)b * a.K + ch) * 3;
      chan_merge_d(n, mean, m2, q[0], q[1], q[2]);
    }
  red[0][lane][cl] = n; red[1][lane][cl] = mean; red[2][lane][cl] = m2;
  __syncthreads();
  if (lane != 0 || ch >= a.K) return;
  for (int j = 1; j < 16; ++j) chan_merge_d(n, mean, m2, red[0][j][cl], red[1][j][cl], red[2][j][cl]);
  const float mean_f = (float)mean, var_f = (float)(m2 / n);
  a.mean[ch] = mean_f;
  a.var[ch] = var_f;
  // folded from the values as stored, exactly like the load-time fold
  const double sc = (double)a.gamma[ch] / sqrt((double)var_f + 1e-5);
  a.scale[ch] = (float)sc;
  a.shift[ch] = (float)((double)a.beta[ch] - (double)mean_f * sc);
}

hipError_t launch_norm_calibrate(const NormCalArgs& a, hipStream_t s) {
  if (a.M < 1 || a.K < 1 || a.nrb != (a.M + SNA_CAL_ROWS - 1) / SNA_CAL_ROWS) return hipErrorInvalidValue;
  hipLaunchKernelGGL(channel_stats_partial_kernel, dim3(a.nrb, (a.K + 63) / 64), dim3(256), 0, s, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(channel_stats_final_kernel, dim3((a.K + 15) / 16), dim3(256), 0, s, a);
  return hipGetLastError();
}

// One element per thread (any K and strides), or, where K and both row strides are multiples of 4
// and the pointers aligned for it, four consecutive channels per thread with 16-byte loads.
template <typename T, int V>
__global__ __launch_bounds__(256) void norm_apply_kernel(const NormApplyArgs a) {
  const unsigned idx = blockIdx.x * 256u + threadIdx.x;     // in units of V elements; the launcher bounds it
  const unsigned kv = (unsigned)a.K / V;
  const unsigned m = idx / kv;
  if (m >= (unsigned)a.M) return;
  const int k = (int)(idx - m * kv) * V;
  float v[V], sc[V], sh[V], r[V];
  const float* raw = a.raw + (long)m * a.K + k;
  if constexpr (V == 4) {
    const float4 q = *(const float4*)raw, s4 = *(const float4*)(a.scale + k), h4 = *(const float4*)(a.shift + k);
    v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
    sc[0] = s4.x; sc[1] = s4.y; sc[2] = s4.z; sc[3] = s4.w;
    sh[0] = h4.x; sh[1] = h4.y; sh[2] = h4.z; sh[3] = h4.w;
  } else {
    v[0] = raw[0]; sc[0] = a.scale[k]; sh[0] = a.shift[k];
  }
  if (a.res) {
    const T* rp = (const T*)a.res + (long)m * a.res_stride + k;
    if constexpr (V == 4 && sizeof(T) == 2) {
      const uint2 u = *(const uint2*)rp;
      r[0] = __uint_as_float(u.x << 16); r[1] = __uint_as_float(u.x & 0xffff0000u);
      r[2] = __uint_as_float(u.y << 16); r[3] = __uint_as_float(u.y & 0xffff0000u);
    } else {
#pragma unroll
      for (int j = 0; j < V; ++j) r[j] = ld_f32<T>(rp + j);
    }
  }
  T* yp = (T*)a.y + (long)m * a.y_stride + k;
  float w[V];
#pragma unroll
  for (int j = 0; j < V; ++j) {
    w[j] = fmaf(v[j], sc[j], sh[j]);
    if (a.res && !a.res_after_act) w[j] += r[j];
    w[j] = apply_act(w[j], a.act);
    if (a.res && a.res_after_act) w[j] += r[j];
  }
  if constexpr (V == 4 && sizeof(T) == 2) {
    *(uint2*)yp = make_uint2(pack_bf16x2(w[0], w[1]), pack_bf16x2(w[2], w[3]));
  } else if constexpr (V == 4) {
    *(float4*)yp = make_float4(w[0], w[1], w[2], w[3]);
  } else {
    st_f32<T>(yp, w[0]);
  }
}

hipError_t launch_norm_apply(const NormApplyArgs& a, int dtype, hipStream_t s) {
  const long total = (long)a.M * a.K;
  if (total < 1 || total >= (1l << 32) - 256) return hipErrorInvalidValue;
  const size_t esz = dtype == SNA_DTYPE_FP32 ? 4 : 2;
  const bool vec = a.K % 4 == 0 && a.res_stride % 4 == 0 && a.y_stride % 4 == 0 && (uintptr_t)a.raw % 16 == 0 &&
                   (uintptr_t)a.scale % 16 == 0 && (uintptr_t)a.shift % 16 == 0 && (uintptr_t)a.y % (4 * esz) == 0 &&
                   (uintptr_t)a.res % (4 * esz) == 0;
  const unsigned blocks = (unsigned)(((vec ? total / 4 : total) + 255) / 256);
  if (dtype == SNA_DTYPE_FP32) {
    if (vec) hipLaunchKernelGGL((norm_apply_kernel<float, 4>), dim3(blocks), dim3(256), 0, s, a);
    else hipLaunchKernelGGL((norm_apply_kernel<float, 1>), dim3(blocks), dim3(256), 0, s, a);
  } else {
    if (vec) hipLaunchKernelGGL((norm_apply_kernel<bf16_t, 4>), dim3(blocks), dim3(256), 0, s, a);
    else hipLaunchKernelGGL((norm_apply_kernel<bf16_t, 1>), dim3(blocks), dim3(256), 0, s, a);
  }
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// SubnetNorm folding at load time: stats [n_subnets][4][row_len] (mean, var, gamma, beta) ->
// folded [n_subnets][2][row_len] with scale = gamma / sqrt(var + eps), shift = beta - mean*scale.
// ---------------------------------------------------------------------------------------------
__global__ void fold_stats_kernel(const float* stats, float* folded, int n_subnets, long row_len) {
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (long)n_subnets * row_len) return;
  const long i = idx / row_len, c = idx % row_len;
  const float* s = stats + i * 4 * row_len;
  const double mean = s[c], var = s[row_len + c], gamma = s[2 * row_len + c], beta = s[3 * row_len + c];
  const double sc = gamma / sqrt(var + 1e-5);
  folded[i * 2 * row_len + c] = (float)sc;
  folded[i * 2 * row_len + row_len + c] = (float)(beta - mean * sc);
}

hipError_t launch_fold_stats(const float* stats, float* folded, int n_subnets, long row_len, hipStream_t s) {
  const long total = (long)n_subnets * row_len;
  if (total == 0) return hipSuccess;
  hipLaunchKernelGGL(fold_stats_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s,
                     stats, folded, n_subnets, row_len);
  return hipGetLastError();
}

}  // namespace sna
