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
// Data path: operands go from global memory straight into LDS (buffer loads with the LDS
// destination, 16 bytes per lane; an out-of-range offset writes zeros, which feeds padding taps,
// ragged rows and the K tail).  LDS holds a ring of NS stages of one K step (64 elements) each;
// rows are 128 bytes with the 16-byte chunks XOR-swizzled by (row >> 1) & 7 so that both the
// linear DMA writes and the column-wise fragment reads are bank-conflict free.  Loads for step
// kt + NS - 1 are issued before the MFMAs of step kt; waits are explicit (s_waitcnt vmcnt with
// the number of newer loads still allowed in flight, then s_barrier).  Fragment reads are
// software-pipelined one 16-wide slice ahead of the v_mfma_f32_32x32x16_bf16 that use them.
// The epilogue (fused SubnetNorm scale/shift, residual, activation) goes through a per-wave
// fp32 LDS tile so that residual loads and output stores are 16 bytes per lane.  Blocks are
// renumbered so that consecutive tiles (which share activation rows) run on the same XCD.
// A launch is grouped: each block finds its problem (one per subnet cfg) from its tile number.
#include "igemm_common.h"

#include <atomic>

namespace sna {

// Waves per SIMD the register allocation must leave room for: tiles with short reductions are
// launched with a small LDS request and then run that many blocks per CU.
constexpr int igemm_min_waves(int bm, int bn) {
  return bm * bn > 128 * 128 ? 2 : (bm * bn >= 128 * 128 ? 3 : (bm * bn >= 128 * 96 ? 4 : 5));
}

// Accesses that are coherent across the chip without cache-wide flushes: relaxed atomics at agent
// scope.  Such a store is written through to memory and such a load is not served from the CU's own
// cache.  The chunk sums that blocks on different XCDs hand to each other go through these; fences
// instead would write back and invalidate the whole L2 of an XCD under the feet of its other blocks
// (measured: forwards at batch 16 lost 15-25 %).  8 bytes per access is the widest atomic there is.
__device__ __forceinline__ void store_f8_agent(float* ptr, const float* v) {      // 8 floats, 32-byte aligned
  unsigned long long* q = (unsigned long long*)ptr;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const unsigned long long w = (unsigned long long)__float_as_uint(v[2 * i]) |
                                 ((unsigned long long)__float_as_uint(v[2 * i + 1]) << 32);
    __hip_atomic_store(q + i, w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}
__device__ __forceinline__ void load_f8_agent(const float* ptr, float4& lo, float4& hi) {
  const unsigned long long* q = (const unsigned long long*)ptr;
  unsigned long long w[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) w[i] = __hip_atomic_load(q + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  lo = make_float4(__uint_as_float((unsigned)w[0]), __uint_as_float((unsigned)(w[0] >> 32)),
                   __uint_as_float((unsigned)w[1]), __uint_as_float((unsigned)(w[1] >> 32)));
  hi = make_float4(__uint_as_float((unsigned)w[2]), __uint_as_float((unsigned)(w[2] >> 32)),
                   __uint_as_float((unsigned)w[3]), __uint_as_float((unsigned)(w[3] >> 32)));
}

// Sum of the fp32 chunk sums of output row m, channels k .. k+7, in chunk order, then SubnetNorm scale /
// shift, residual and activation exactly as the fused epilogue does: the same bits as one block walking
// all chunks.  `src` points at part 0's row-major [M][K] sums.  Used by the reduction kernel and by the
// matrix kernel's own last-arriving block.
// AGENT: `src0` already points at this octet inside part 0 (the matrix kernel's tile-major layout).
template <bool AGENT>
__device__ __forceinline__ void reduce_octet(const ConvProblem& p, const float* src0, int m, int k) {
  // all loads first (at most 4 chunks), then the sums in chunk order
  const float* src = AGENT ? src0 : src0 + (long)m * p.K + k;
  float4 pa[4], pb[4];
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    if (c < p.parts) {
      const float* sp = (const float*)((const char*)src + (size_t)c * p.part_stride);
      if (AGENT) {
        load_f8_agent(sp, pa[c], pb[c]);      // written by other blocks of this launch
      } else {
        pa[c] = *(const float4*)sp;
        pb[c] = *(const float4*)(sp + 4);
      }
    }
  }
  float4 sc0 = make_float4(1.f, 1.f, 1.f, 1.f), sc1 = sc0, sh0 = make_float4(0.f, 0.f, 0.f, 0.f), sh1 = sh0;
  // the per-channel vectors are only guaranteed 4-byte alignment
  auto load8 = [&](const float* v, float4& lo, float4& hi) {
    if (((size_t)v & 15) == 0) {
      lo = *(const float4*)(v + k);
      hi = *(const float4*)(v + k + 4);
    } else {
      lo = make_float4(v[k], v[k + 1], v[k + 2], v[k + 3]);
      hi = make_float4(v[k + 4], v[k + 5], v[k + 6], v[k + 7]);
    }
  };
  if (p.scale) load8(p.scale, sc0, sc1);
  if (p.shift) load8(p.shift, sh0, sh1);
  uint4 r4 = make_uint4(0, 0, 0, 0);
  if (p.res) r4 = *(const uint4*)((const bf16_t*)p.res + (long)m * p.res_stride + k);
  float val[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) val[e] = 0.f;
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    if (c < p.parts) {
      val[0] = val[0] + pa[c].x; val[1] = val[1] + pa[c].y; val[2] = val[2] + pa[c].z; val[3] = val[3] + pa[c].w;
      val[4] = val[4] + pb[c].x; val[5] = val[5] + pb[c].y; val[6] = val[6] + pb[c].z; val[7] = val[7] + pb[c].w;
    }
  }
  const float scv[8] = {sc0.x, sc0.y, sc0.z, sc0.w, sc1.x, sc1.y, sc1.z, sc1.w};
  const float shv[8] = {sh0.x, sh0.y, sh0.z, sh0.w, sh1.x, sh1.y, sh1.z, sh1.w};
#pragma unroll
  for (int e = 0; e < 8; ++e) val[e] = fmaf(val[e], scv[e], shv[e]);
  float rv[8];
  if (p.res) {
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
    o.x = pack_bf16x2(val[0], val[1]);
    o.y = pack_bf16x2(val[2], val[3]);
    o.z = pack_bf16x2(val[4], val[5]);
    o.w = pack_bf16x2(val[6], val[7]);
    *(uint4*)((bf16_t*)p.y + (long)m * p.y_stride + k) = o;
  }
}

// WS (wave-specialised): the block has twice the waves; the second half only fetches (address
// arithmetic, global->LDS loads, the wait for them), the first half only computes, and the two
// meet at the one barrier per K step.  A fetching wave stalled on the texture path no longer
// holds up MFMA issue, which matters when a CU has a single block to overlap with itself.
template <int BM, int BN, int WARPS_M, int WARPS_N, int NS, bool CHUNKED, bool WS>
__global__ __launch_bounds__(64 * WARPS_M * WARPS_N * (WS ? 2 : 1),
                             WS ? (BM * BN >= 128 * 128 ? 2 : 4)
                                : (CHUNKED ? (BM * BN == 128 * 64 ? 3 : (BM * BN > 128 * 128 ? 1 : 2)) : igemm_min_waves(BM, BN)))
void igemm_kernel(const ConvGroupArgs args) {
#if defined(__HIP_DEVICE_COMPILE__)        // the host pass needs the symbol only, not the body
  using Cfg = IgemmCfg<BM, BN, WARPS_M, WARPS_N, NS>;
  constexpr int WTM = Cfg::WTM, WTN = Cfg::WTN, TM = Cfg::TM, TN = Cfg::TN;
  static_assert(TM >= 1 && TN >= 1 && WTM % 32 == 0 && WTN % 32 == 0, "wave tile");
  static_assert(BM % 8 == 0 && BN % 8 == 0 && Cfg::PASS_ROWS % 8 == 0, "DMA rows come in groups of 8");
  constexpr int A_IT = Cfg::A_IT, B_IT = Cfg::B_IT, L = A_IT + B_IT;   // DMA loads per thread per stage
  static_assert(NS >= 1 && (NS - 2) * L < 64, "vmcnt range");
  static_assert(NS > 1 || !WS, "a fetching wave needs a second stage to run ahead");
  static_assert(BM % Cfg::PASS_ROWS == 0 && BN % Cfg::PASS_ROWS == 0, "every wave issues the same number of loads");

  extern __shared__ __attribute__((aligned(16))) char smem[];
  const unsigned lds0 = (unsigned)(size_t)(lds_char*)smem;              // LDS byte address of the tiles

  // XCD-aware renumbering: hardware block b runs on XCD b % 8; give each XCD a contiguous tile range
  const int per_xcd = gridDim.x >> 3;
  const int tile_id = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (tile_id >= args.total_tiles) return;

  // by value: uniform fields live in SGPRs across the asm blocks.  The first problem's descriptor sits at
  // a fixed kernarg offset, so its load does not wait for the problem search (most launches carry one).
  ConvProblem p = args.p[0];
  if (args.n > 1) {
    const int g = find_problem(args, tile_id);
    if (g > 0) p = args.p[g];
  }
  int local = tile_id - p.tile_start;
  int part = 0;                            // which K range of the problem this block reduces over
  if (p.parts > 1) {
    part = local / p.tiles_base;
    local -= part * p.tiles_base;
  }
  const int tn = local % p.tiles_n, tm = local / p.tiles_n;
  const int m0 = tm * BM, n0 = tn * BN;

  constexpr int NW = WARPS_M * WARPS_N;
  const int lane = threadIdx.x & 63;
  const bool fetcher = WS && (int)(threadIdx.x >> 6) >= NW;
  const bool do_load = !WS || fetcher, do_math = !WS || !fetcher;
  const int wave = WS ? (int)(threadIdx.x >> 6) % NW : (int)(threadIdx.x >> 6);   // index within its role
  const int tid = wave * 64 + lane;
  const int wm = wave / WARPS_N, wn = wave % WARPS_N;
  const int lrow = tid >> 3;                               // row inside a pass
  const int kc = (tid & 7) ^ ((lrow >> 1) & 7);            // global 16-byte unit this lane's LDS slot holds

  const int C = p.C, H = p.H, Wd = p.W, S = p.S, RS = p.R * p.S;

  // rows this thread fetches: byte offset of the window's first tap and which taps are in range
  int a_base[A_IT];
  unsigned long long a_mask[A_IT];      // bit rs set: tap rs of this row's window is inside the image
  unsigned long long tap_rows = 0;      // bit r * S for every window row r (uniform)
  for (int r = 0; r < p.R; ++r) tap_rows |= 1ull << (r * S);
  const bool pointwise = RS == 1 && p.stride == 1 && p.pad == 0;   // output pixel m reads input pixel m
#pragma unroll
  for (int i = 0; i < A_IT; ++i) {
    const int row = lrow + Cfg::PASS_ROWS * i;
    const int m = m0 + row;
    a_base[i] = 0;
    a_mask[i] = 0;
    if (row < BM && m < p.M) {
      if (pointwise) {
        a_base[i] = m * C * 2;
        a_mask[i] = 1;
      } else {
        // m -> (n, pp, q) with multiply-high by the host's reciprocals (exact for m * divisor < 2^32)
        const int t = p.Wo == 1 ? m : (int)__umulhi((unsigned)m, p.magic_wo);
        const int q = m - t * p.Wo;
        const int n = p.Ho == 1 ? t : (int)__umulhi((unsigned)t, p.magic_ho);
        const int pp = t - n * p.Ho;
        const int ih0 = pp * p.stride - p.pad, iw0 = q * p.stride - p.pad;
        a_base[i] = ((n * H + ih0) * Wd + iw0) * C * 2;
        // taps inside the image: columns [s_lo, s_hi) of window rows [r_lo, r_hi), without loops
        const int s_lo = iw0 < 0 ? -iw0 : 0, s_hi = Wd - iw0 < S ? Wd - iw0 : S;
        const int r_lo = ih0 < 0 ? -ih0 : 0, r_hi = H - ih0 < p.R ? H - ih0 : p.R;
        unsigned long long mk = 0;
        if (s_hi > s_lo && r_hi > r_lo) {
          const unsigned long long colm = low_bits(s_hi) & ~low_bits(s_lo);
          mk = colm * (tap_rows & low_bits(r_hi * S) & ~low_bits(r_lo * S));      // one copy of colm per window row
        }
        a_mask[i] = mk;
      }
    }
  }
  int b_base[B_IT];
  unsigned b_ok = 0;
#pragma unroll
  for (int j = 0; j < B_IT; ++j) {
    const int row = lrow + Cfg::PASS_ROWS * j;
    const int k = n0 + row;
    if (row < BN && k < p.K) b_ok |= 1u << j;
    b_base[j] = k * p.wk * 2;
  }

  // reduction position of this thread's unit: tap rs and channel octet c8
  const int kt0 = part * p.kt_part;        // first K step of this block's range
  int rs = (kt0 * 8 + kc) / p.C8;
  int c8 = kt0 * 8 + kc - rs * p.C8;
  const int KT_all = (p.K8 + 7) >> 3;     // K steps of 64 elements in the whole reduction
  const int KT = KT_all - kt0 < p.kt_part ? KT_all - kt0 : p.kt_part;

  const __amdgpu_buffer_rsrc_t rsrc_x = __builtin_amdgcn_make_buffer_rsrc((void*)p.x, 0, (int)p.x_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_w = __builtin_amdgcn_make_buffer_rsrc((void*)p.w, 0, (int)p.w_bytes, 0x00020000);
  constexpr unsigned OOB = 0x80000000u;
  // LDS destination of this wave's DMA ops inside a stage: 64 lanes x 16 bytes = 8 consecutive rows
  lds_char* const dma_a = (lds_char*)smem + (wave * 8) * ROW_B;
  lds_char* const dma_b = dma_a + BM * ROW_B;

  // Buffer offsets of the next K step to fetch.  Within a tap they advance by one step (128 bytes)
  // per fetch; only when a lane's unit crosses into the next tap are they rebuilt from (rs, c8).
  // An out-of-range entry stays out of range under the increments (it starts at 2^31).
  unsigned dma_off[L];
  auto locate = [&]() {
    const bool u_ok = rs < RS;
    const int r = (rs * p.inv_s) >> 16, s = rs - r * S;
    const int tx = ((r * Wd + s) * C + c8 * 8) * 2, tw = (r * p.wr + s * p.ws + c8 * 8) * 2;
#pragma unroll
    for (int i = 0; i < A_IT; ++i) {
      const bool ok = u_ok && ((a_mask[i] >> (rs & 63)) & 1ull);
      dma_off[i] = ok ? (unsigned)(a_base[i] + tx) : OOB;
    }
#pragma unroll
    for (int j = 0; j < B_IT; ++j) {
      const bool ok = u_ok && ((b_ok >> j) & 1u);
      dma_off[A_IT + j] = ok ? (unsigned)(b_base[j] + tw) : OOB;
    }
  };
  locate();
  auto issue = [&](int stage) {
#pragma unroll
    for (int i = 0; i < A_IT; ++i)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_x, dma_a + stage * Cfg::STAGE_B + Cfg::PASS_ROWS * i * ROW_B, 16,
                                               dma_off[i], 0, 0, 0);
#pragma unroll
    for (int j = 0; j < B_IT; ++j)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_w, dma_b + stage * Cfg::STAGE_B + Cfg::PASS_ROWS * j * ROW_B, 16,
                                               dma_off[A_IT + j], 0, 0, 0);
    c8 += 8;                              // advance one K step
    if (c8 >= p.C8) {
      do { c8 -= p.C8; ++rs; } while (c8 >= p.C8);
      locate();
    } else {
#pragma unroll
      for (int i = 0; i < L; ++i) dma_off[i] += BK * 2;
    }
  };

  f32x16 acc[TM][TN];                      // written by the first MFMA of the first step

  const int frag_row = lane & 31, frag_hi = lane >> 5, frag_sw = (frag_row >> 1) & 7;
  unsigned frag_off[BK / 16];              // swizzled byte offset of this lane's chunk in each 16-wide slice
#pragma unroll
  for (int ks = 0; ks < BK / 16; ++ks) frag_off[ks] = (unsigned)(((ks * 2 + frag_hi) ^ frag_sw) * 16);
  const unsigned a_lane = lds0 + (wm * WTM + frag_row) * ROW_B;
  const unsigned b_lane = lds0 + (BM + wn * WTN + frag_row) * ROW_B;

  // `fresh`: the accumulators start a new sum at this step (first MFMA of each takes C = 0)
  auto compute = [&](int stage, const bool fresh) {
    const unsigned ab = a_lane + stage * Cfg::STAGE_B, bb = b_lane + stage * Cfg::STAGE_B;
    u32x4 af[2][TM], bfr[2][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) af[0][i] = lds_read_b128(ab + frag_off[0], i * 32 * ROW_B);
#pragma unroll
    for (int j = 0; j < TN; ++j) bfr[0][j] = lds_read_b128(bb + frag_off[0], j * 32 * ROW_B);
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      const int cur = ks & 1, nxt = cur ^ 1;
      // fragments of slice ks were requested one slice ago: wait for them, then request slice ks+1
      // before the MFMAs of slice ks so that the LDS latency runs under the matrix pipe
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
      for (int i = 0; i < TM; ++i) asm volatile("" : "+v"(af[cur][i]));
#pragma unroll
      for (int j = 0; j < TN; ++j) asm volatile("" : "+v"(bfr[cur][j]));
      if (ks + 1 < BK / 16) {
#pragma unroll
        for (int i = 0; i < TM; ++i) af[nxt][i] = lds_read_b128(ab + frag_off[ks + 1], i * 32 * ROW_B);
#pragma unroll
        for (int j = 0; j < TN; ++j) bfr[nxt][j] = lds_read_b128(bb + frag_off[ks + 1], j * 32 * ROW_B);
      }
      __builtin_amdgcn_sched_barrier(0);    // keep the requests ahead of the MFMAs that hide their latency
      if (ks == 0 && fresh) {
        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, af[cur][i]),
                                                                __builtin_bit_cast(bf16x8, bfr[cur][j]), zero, 0, 0, 0);
      } else {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, af[cur][i]),
                                                                __builtin_bit_cast(bf16x8, bfr[cur][j]), acc[i][j], 0, 0, 0);
      }
    }
  };

  // ---- main loop: ring of NS stages ----------------------------------------------------------
  if (do_load) {
#pragma unroll
    for (int st = 0; st < NS - 1; ++st)
      if (st < KT) issue(st);
  }

  // SubnetNorm scale / shift of this lane's output columns, requested behind the first stages' loads so
  // that they arrive under the main loop
  const int col_l = lane & 31, row_l = (lane >> 5) * 4;
  // reduction finished inside this launch: the blocks store bare chunk sums, the last one to arrive at a
  // tile applies scale / shift / residual / activation after adding them up
  const bool in_kernel_reduce = p.parts > 1 && p.counters != nullptr;
  float sc[TN], sh[TN];
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int k = n0 + wn * WTN + j * 32 + col_l;
    sc[j] = (do_math && !in_kernel_reduce && p.scale && k < p.K) ? p.scale[k] : 1.f;
    sh[j] = (do_math && !in_kernel_reduce && p.shift && k < p.K) ? p.shift[k] : 0.f;
  }

  // CHUNKED: the reduction is summed in chunks of p.kt_chunk steps, each accumulated from zero and
  // added to a running total in fp32, so that one block reducing over all chunks gives the same
  // bits as one block per chunk plus the reduction kernel.
  f32x16 tot[CHUNKED ? TM : 1][CHUNKED ? TN : 1];
  int to_fold = p.kt_chunk;
  if (CHUNKED) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) tot[i][j][v] = 0.f;
  }
  int stage = 0, fill = NS - 1;            // stage holding step kt; stage that step kt + NS - 1 goes to
  bool fresh = true;
  for (int kt = 0; kt < KT; ++kt) {
    if constexpr (NS == 1) {
      // a single stage: the step is fetched, awaited and consumed in turn.  Nothing overlaps inside the
      // block; the small LDS footprint lets more blocks share a CU, which is what short reductions need.
      if (kt > 0) __builtin_amdgcn_s_barrier();            // every wave is done reading the stage
      if (do_load) {
        issue(0);
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
      }
      __builtin_amdgcn_s_barrier();                        // every wave's part of step kt is in LDS
    } else {
      // step kt's loads were issued NS-1 steps ago; up to NS-2 newer steps may stay in flight
      if (do_load) {
        if (kt + NS - 1 <= KT) __builtin_amdgcn_s_waitcnt(vmcnt_imm((NS - 2) * L));
        else __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
      }
      __builtin_amdgcn_s_barrier();          // every wave's part of step kt is in LDS; step kt-1 fully consumed
      if (do_load && kt + NS - 1 < KT) issue(fill);
    }
    if (do_math) compute(stage, fresh);
    fresh = false;
    stage = stage + 1 == NS ? 0 : stage + 1;
    fill = fill + 1 == NS ? 0 : fill + 1;
    if (CHUNKED && --to_fold == 0 && kt + 1 < KT) {       // chunk boundary: bank the chunk's sum
      to_fold = p.kt_chunk;
      fresh = true;
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int v = 0; v < 16; ++v) tot[i][j][v] = tot[i][j][v] + acc[i][j][v];
    }
  }
  __syncthreads();
  if (WS && fetcher) return;               // no barrier below this point

  // ---- epilogue -----------------------------------------------------------------------------
  // accumulator element v of lane l is row 8*(v/4) + 4*(l/32) + v%4, column l%32 of a 32x32 tile.
  // Per 32-row strip: SubnetNorm scale/shift on the accumulators, fp32 strip into this wave's LDS
  // region, then each lane takes (row, 8 consecutive channels): residual, activation, store.
  float* epi = (float*)smem + wave * 32 * Cfg::EPI_STRIDE;
  constexpr int OCT = WTN / 8;                 // channel octets per staged row
  constexpr int PAIRS = 32 * OCT / 64;         // (row, octet) pairs per lane
  // ACT, RES (0 none, 1 added before the activation, 2 after) and F32 are uniform over the launch's
  // problem: one dispatch below instead of per-element tests.
  auto epilogue = [&](auto act_c, auto res_c, auto f32_c) {
    constexpr int ACT = decltype(act_c)::value, RES = decltype(res_c)::value;
    constexpr bool F32 = decltype(f32_c)::value;
    // Residual rows.  With several 32-row strips per wave they are all requested up front, so that
    // one round trip runs under the staging of the first strip instead of one per strip; with a
    // single strip the request goes after the staging writes, when the accumulators' registers are free.
    constexpr bool RES_UP_FRONT = TM > 1;
    uint4 r4[TM][PAIRS];
    auto load_res = [&](int i) {
#pragma unroll
      for (int t = 0; t < PAIRS; ++t) {
        const int id = t * 64 + lane;
        const int row = id / OCT, oct = id - row * OCT;
        const int m = m0 + wm * WTM + i * 32 + row;
        const int k = n0 + wn * WTN + oct * 8;
        r4[i][t] = (m < p.M && k < p.K) ? *(const uint4*)((const bf16_t*)p.res + (long)m * p.res_stride + k)
                                        : make_uint4(0, 0, 0, 0);
      }
    };
    if (RES != 0 && RES_UP_FRONT) {
#pragma unroll
      for (int i = 0; i < TM; ++i) load_res(i);
    }
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          epi[(8 * (v >> 2) + row_l + (v & 3)) * Cfg::EPI_STRIDE + j * 32 + col_l] =
              fmaf(CHUNKED ? tot[i][j][v] + acc[i][j][v] : acc[i][j][v], sc[j], sh[j]);
      if (RES != 0 && !RES_UP_FRONT) load_res(i);
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
        const float4 v0 = *(const float4*)(epi + row * Cfg::EPI_STRIDE + oct * 8);
        const float4 v1 = *(const float4*)(epi + row * Cfg::EPI_STRIDE + oct * 8 + 4);
        float val[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
        float rv[8];
        if (RES != 0) {
          const unsigned ru[4] = {r4[i][t].x, r4[i][t].y, r4[i][t].z, r4[i][t].w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            rv[2 * e] = __uint_as_float(ru[e] << 16);
            rv[2 * e + 1] = __uint_as_float(ru[e] & 0xffff0000u);
          }
        }
        if (RES == 1) {
#pragma unroll
          for (int e = 0; e < 8; ++e) val[e] += rv[e];
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) val[e] = apply_act(val[e], ACT);
        if (RES == 2) {
#pragma unroll
          for (int e = 0; e < 8; ++e) val[e] += rv[e];
        }
        if (m < p.M && k < p.K) {
          if (F32) {
            if (in_kernel_reduce) {
              // tile-major: every tile's sums fill whole cache lines of their own, so that no block ever
              // pulls a line into its L2 that another tile's blocks have yet to write
              float* yo = (float*)((char*)p.part_buf + (size_t)part * p.part_stride) + (size_t)local * (BM * BN) +
                          (m - m0) * BN + (k - n0);
              store_f8_agent(yo, val);
            } else {
              float* yo = (float*)((char*)p.y + (size_t)part * p.part_stride) + (long)m * p.y_stride + k;
              *(float4*)yo = make_float4(val[0], val[1], val[2], val[3]);
              *(float4*)(yo + 4) = make_float4(val[4], val[5], val[6], val[7]);
            }
          } else {
            uint4 o;
            o.x = pack_bf16x2(val[0], val[1]);
            o.y = pack_bf16x2(val[2], val[3]);
            o.z = pack_bf16x2(val[4], val[5]);
            o.w = pack_bf16x2(val[6], val[7]);
            *(uint4*)((bf16_t*)p.y + (long)m * p.y_stride + k) = o;
          }
        }
      }
      __builtin_amdgcn_wave_barrier();
    }
  };
  using std::integral_constant;
  typedef integral_constant<bool, true> yes_t;
  typedef integral_constant<bool, false> no_t;
#define SNA_EPI(A, R) epilogue(integral_constant<int, A>{}, integral_constant<int, R>{}, no_t{})
  const int res_mode = p.res ? (p.res_after_act ? 2 : 1) : 0;
  if (in_kernel_reduce) {
    epilogue(integral_constant<int, SNA_ACT_NONE>{}, integral_constant<int, 0>{}, yes_t{});      // bare chunk sums to part_buf
    // Count arrivals at this tile.  The chunk sums went out as write-through agent-scope stores; once
    // every thread's stores have completed, the block's one atomic publishes them.  The block that sees
    // parts - 1 earlier arrivals is the last and owns the tile from here on (nobody waits for anybody).
    // It puts the counter back to zero for the next launch that uses it.
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    __syncthreads();
    int* const flag = (int*)smem;               // the ring is dead by now
    if (threadIdx.x == 0) {
      int* const cnt = p.counters + local;
      const int seen = atomicAdd(cnt, 1);
      const int last = seen == p.parts - 1;
      if (last) atomicExch(cnt, 0);
      *flag = last;
    }
    __syncthreads();
    if (*flag == 0) return;
    constexpr int OCT_T = BN / 8;
    const int nthr = 64 * NW;                   // fetching waves of a wave-specialised block have left
    for (int id = threadIdx.x; id < BM * OCT_T; id += nthr) {
      const int row = id / OCT_T, oct = id - row * OCT_T;
      const int m = m0 + row, k = n0 + oct * 8;
      if (m < p.M && k < p.K) reduce_octet<true>(p, p.part_buf + (size_t)local * (BM * BN) + row * BN + oct * 8, m, k);
    }
  } else if (p.out_fp32) {                                     // logits: no activation, no residual
    if (p.act == SNA_ACT_NONE && res_mode == 0) epilogue(integral_constant<int, SNA_ACT_NONE>{}, integral_constant<int, 0>{}, yes_t{});
  } else if (p.act == SNA_ACT_RELU) {
    if (res_mode == 0) SNA_EPI(SNA_ACT_RELU, 0); else if (res_mode == 1) SNA_EPI(SNA_ACT_RELU, 1); else SNA_EPI(SNA_ACT_RELU, 2);
  } else if (p.act == SNA_ACT_NONE) {
    if (res_mode == 0) SNA_EPI(SNA_ACT_NONE, 0); else SNA_EPI(SNA_ACT_NONE, 1);
  } else if (p.act == SNA_ACT_HSWISH) {
    if (res_mode == 0) SNA_EPI(SNA_ACT_HSWISH, 0); else if (res_mode == 1) SNA_EPI(SNA_ACT_HSWISH, 1); else SNA_EPI(SNA_ACT_HSWISH, 2);
  } else {
    if (res_mode == 0) SNA_EPI(SNA_ACT_GELU, 0); else if (res_mode == 1) SNA_EPI(SNA_ACT_GELU, 1); else SNA_EPI(SNA_ACT_GELU, 2);
  }
#undef SNA_EPI
#endif
}

// ---------------------------------------------------------------------------------------------
// 3x3 stride-1 pad-1 convolution with the activation operand resident in LDS ("slab").
//
// The implicit GEMM above fetches every activation row of a tile once per tap: nine trips through
// the texture path, each a 16-byte gather at a pixel stride that is rarely a multiple of the cache
// line.  For a 3x3 stride-1 layer the BM consecutive output pixels of a tile read, over all nine
// taps, only the BM + 2 W + 2 consecutive input pixels around them (NHWC, images back to back), so
// this kernel loads that slab once, linearly, and the matrix pipe takes its A fragments from it at
// tap-shifted addresses; only the weights stream through the ring.  A tap that falls outside the
// image (or a row past M) reads a 16-byte block of zeros instead.  The slab's pixel stride is the
// channel count rounded up to an odd number of 16-byte units (the spare unit is zero-filled), which
// spreads consecutive pixels over the LDS banks.  The reduction runs in the same order and in the
// same 16-element MFMA slices as the implicit GEMM (tap-major, then channels), and chunk sums
// are folded at the same steps, so the output has the same bits.
// ---------------------------------------------------------------------------------------------
constexpr int slab_units(int bm, int w, int c8, int nthreads) {
  const int c8p = c8 | 1;
  const int units = (bm + 2 * w + 2) * c8p + 1;          // + the block of zeros
  return (units + nthreads - 1) / nthreads * nthreads;
}

template <int BM, int BN, int WARPS_M, int WARPS_N, int NS, bool CHUNKED>
__global__ __launch_bounds__(64 * WARPS_M * WARPS_N, BM * BN > 128 * 128 ? 1 : 2)
void conv3_slab_kernel(const ConvGroupArgs args) {
#if defined(__HIP_DEVICE_COMPILE__)        // the host pass needs the symbol only, not the body
  using Cfg = IgemmCfg<BM, BN, WARPS_M, WARPS_N, NS>;
  constexpr int WTM = Cfg::WTM, WTN = Cfg::WTN, TM = Cfg::TM, TN = Cfg::TN, NT = Cfg::NTHREADS;
  constexpr int B_IT = Cfg::B_IT, L = B_IT;                // ring loads per thread per stage: weights only
  constexpr int RING_STAGE_B = BN * ROW_B;
  static_assert(BN % Cfg::PASS_ROWS == 0, "every wave issues the same number of loads");
  static_assert((NS - 2) * L < 64, "vmcnt range");

  extern __shared__ __attribute__((aligned(16))) char smem[];
  const unsigned lds0 = (unsigned)(size_t)(lds_char*)smem;

  const int per_xcd = gridDim.x >> 3;
  const int tile_id = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (tile_id >= args.total_tiles) return;
  ConvProblem p = args.p[0];
  if (args.n > 1) {
    const int g = find_problem(args, tile_id);
    if (g > 0) p = args.p[g];
  }
  const int local = tile_id - p.tile_start;
  const int tn = local % p.tiles_n, tm = local / p.tiles_n;
  const int m0 = tm * BM, n0 = tn * BN;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, tid = threadIdx.x;
  const int wm = wave / WARPS_N, wn = wave % WARPS_N;
  const int lrow = tid >> 3;
  const int kc = (tid & 7) ^ ((lrow >> 1) & 7);
  const int C = p.C, H = p.H, Wd = p.W, C8 = p.C8;
  const int C8p = C8 | 1;                                  // slab pixel stride in 16-byte units, odd
  const int P = BM + 2 * Wd + 2;                           // slab pixels
  const int units = P * C8p;                               // unit `units` is the block of zeros
  const int n_it = (units + 1 + NT - 1) / NT;
  const unsigned ring0 = lds0 + (unsigned)n_it * NT * 16;

  const __amdgpu_buffer_rsrc_t rsrc_x = __builtin_amdgcn_make_buffer_rsrc((void*)p.x, 0, (int)p.x_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_w = __builtin_amdgcn_make_buffer_rsrc((void*)p.w, 0, (int)p.w_bytes, 0x00020000);
  constexpr unsigned OOB = 0x80000000u;

  // ---- slab: input pixels m0 - W - 1 .. m0 + BM + W of the flattened (n, y, x) order, once ------
  {
    const int pix0 = m0 - Wd - 1, n_pix = p.N * H * Wd;
    const unsigned magic = 0xFFFFFFFFu / (unsigned)C8p + 1u;        // e / C8p = mulhi(e, magic) for e < 2^16 * C8p
    lds_char* const dst = (lds_char*)smem + wave * 64 * 16;
#pragma unroll 1
    for (int it = 0; it < n_it; ++it) {
      const unsigned e = (unsigned)(it * NT + tid);
      const int px = C8p == 1 ? (int)e : (int)__umulhi(e, magic), c = (int)e - px * C8p;      // (2^32 / 1 does not fit the magic)
      const int gp = pix0 + px;
      const bool ok = c < C8 && px < P && gp >= 0 && gp < n_pix;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_x, dst + it * NT * 16, 16, ok ? (unsigned)((gp * C + c * 8) * 2) : OOB,
                                               0, 0, 0);
    }
  }

  // ---- weights: ring of NS stages, as in the implicit GEMM ------------------------------------
  int b_base[B_IT];
  unsigned b_ok = 0;
#pragma unroll
  for (int j = 0; j < B_IT; ++j) {
    const int row = lrow + Cfg::PASS_ROWS * j;
    const int k = n0 + row;
    if (row < BN && k < p.K) b_ok |= 1u << j;
    b_base[j] = k * p.wk * 2;
  }
  int rs = kc / C8;
  int c8 = kc - rs * C8;
  const int KT = (p.K8 + 7) >> 3;
  lds_char* const dma_b = (lds_char*)smem + n_it * NT * 16 + (wave * 8) * ROW_B;
  unsigned dma_off[L];
  auto locate = [&]() {
    const bool u_ok = rs < 9;
    const int r = (rs * 11) >> 5, s = rs - r * 3;              // rs / 3 for rs < 32
    const int tw = (r * p.wr + s * p.ws + c8 * 8) * 2;
#pragma unroll
    for (int j = 0; j < B_IT; ++j) dma_off[j] = (u_ok && ((b_ok >> j) & 1u)) ? (unsigned)(b_base[j] + tw) : OOB;
  };
  locate();
  auto issue = [&](int stage) {
#pragma unroll
    for (int j = 0; j < B_IT; ++j)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_w, dma_b + stage * RING_STAGE_B + Cfg::PASS_ROWS * j * ROW_B, 16,
                                               dma_off[j], 0, 0, 0);
    c8 += 8;
    if (c8 >= C8) {
      do { c8 -= C8; ++rs; } while (c8 >= C8);
      locate();
    } else {
#pragma unroll
      for (int j = 0; j < L; ++j) dma_off[j] += BK * 2;
    }
  };

  // ---- this lane's A rows: slab address of tap (0, 0) and which taps lie inside the image ------
  const int frag_row = lane & 31, frag_hi = lane >> 5, frag_sw = (frag_row >> 1) & 7;
  unsigned a_row[TM], a_taps[TM];
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int row = wm * WTM + i * 32 + frag_row;
    const int m = m0 + row;
    a_row[i] = lds0 + (unsigned)(row * C8p) * 16;
    unsigned mk = 0;
    if (m < p.M) {
      const int t = (int)__umulhi((unsigned)m, p.magic_wo);            // W >= 2 for a padded 3x3 to make sense
      const int xq = m - t * Wd;
      const int n = H == 1 ? t : (int)__umulhi((unsigned)t, p.magic_ho);
      const int yq = t - n * H;
      unsigned colm = 0;
#pragma unroll
      for (int s = 0; s < 3; ++s)
        if (xq + s - 1 >= 0 && xq + s - 1 < Wd) colm |= 1u << s;
#pragma unroll
      for (int r = 0; r < 3; ++r)
        if (yq + r - 1 >= 0 && yq + r - 1 < H) mk |= colm << (3 * r);
    }
    a_taps[i] = mk;
  }
  const unsigned zero_addr = lds0 + (unsigned)units * 16;
  // reduction position of this lane's unit in the slice about to be read: tap (ar, as), octet ac8
  int ars = frag_hi / C8, ac8 = frag_hi - ars * C8;
  int a_r = 0, a_s = ars;                                   // ars <= 1 here
  unsigned a_addr[TM];
  auto a_next = [&]() {                                     // addresses of the current slice, then advance by two units
    const unsigned tap = (unsigned)(((a_r * Wd + a_s) * C8p + ac8) * 16);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const bool ok = ars < 9 && ((a_taps[i] >> ars) & 1u);
      a_addr[i] = ok ? a_row[i] + tap : zero_addr;
    }
    ac8 += 2;
    while (ac8 >= C8) {
      ac8 -= C8; ++ars; ++a_s;
      if (a_s == 3) { a_s = 0; ++a_r; }
    }
  };

  f32x16 acc[TM][TN];
  unsigned frag_off[BK / 16];
#pragma unroll
  for (int ks = 0; ks < BK / 16; ++ks) frag_off[ks] = (unsigned)(((ks * 2 + frag_hi) ^ frag_sw) * 16);
  const unsigned b_lane = ring0 + (wn * WTN + frag_row) * ROW_B;

  // All fragment reads of a step are requested up front (LDS returns them in order) and each
  // 16-wide slice waits only for its own: a wave then has up to 4 (TM + TN) reads in flight, which
  // the LDS needs to come near its bandwidth (measured: 105 B/clk/CU with 4 reads in flight per wave,
  // 208 with 8 on 8 waves); one slice ahead leaves the step bound by LDS latency.
  constexpr int NSL = BK / 16, RPS = TM + TN;               // slices per step, reads per slice
  auto compute = [&](int stage, const bool fresh) {
    const unsigned bb = b_lane + stage * RING_STAGE_B;
    u32x4 af[NSL][TM], bfr[NSL][TN];
#pragma unroll
    for (int ks = 0; ks < NSL; ++ks) {                      // every read of the step up front, in slice order
      a_next();
#pragma unroll
      for (int i = 0; i < TM; ++i) af[ks][i] = lds_read_b128(a_addr[i], 0);
#pragma unroll
      for (int j = 0; j < TN; ++j) bfr[ks][j] = lds_read_b128(bb + frag_off[ks], j * 32 * ROW_B);
    }
    auto slice = [&](auto ks_c) {
      constexpr int ks = decltype(ks_c)::value;
      constexpr int later = (NSL - 1 - ks) * RPS;
      __builtin_amdgcn_s_waitcnt(0xc07f | ((later > 15 ? 15 : later) << 8));      // lgkmcnt(later)
#pragma unroll
      for (int i = 0; i < TM; ++i) asm volatile("" : "+v"(af[ks][i]));
#pragma unroll
      for (int j = 0; j < TN; ++j) asm volatile("" : "+v"(bfr[ks][j]));
      __builtin_amdgcn_sched_barrier(0);
      if (ks == 0 && fresh) {
        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, af[ks][i]),
                                                                __builtin_bit_cast(bf16x8, bfr[ks][j]), zero, 0, 0, 0);
      } else {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, af[ks][i]),
                                                                __builtin_bit_cast(bf16x8, bfr[ks][j]), acc[i][j], 0, 0, 0);
      }
    };
    static_assert(NSL == 4, "four slices per step");
    slice(std::integral_constant<int, 0>{});
    slice(std::integral_constant<int, 1>{});
    slice(std::integral_constant<int, 2>{});
    slice(std::integral_constant<int, 3>{});
  };

#pragma unroll
  for (int st = 0; st < NS - 1; ++st)
    if (st < KT) issue(st);

  const int col_l = lane & 31, row_l = (lane >> 5) * 4;
  float sc[TN], sh[TN];
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int k = n0 + wn * WTN + j * 32 + col_l;
    sc[j] = (p.scale && k < p.K) ? p.scale[k] : 1.f;
    sh[j] = (p.shift && k < p.K) ? p.shift[k] : 0.f;
  }

  f32x16 tot[CHUNKED ? TM : 1][CHUNKED ? TN : 1];
  int to_fold = p.kt_chunk;
  if (CHUNKED) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) tot[i][j][v] = 0.f;
  }
  int stage = 0, fill = NS - 1;
  bool fresh = true;
  for (int kt = 0; kt < KT; ++kt) {
    // the slab's loads were issued ahead of every ring load, and loads complete in order
    if (kt + NS - 1 <= KT) __builtin_amdgcn_s_waitcnt(vmcnt_imm((NS - 2) * L));
    else __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    __builtin_amdgcn_s_barrier();
    if (kt + NS - 1 < KT) issue(fill);
    compute(stage, fresh);
    fresh = false;
    stage = stage + 1 == NS ? 0 : stage + 1;
    fill = fill + 1 == NS ? 0 : fill + 1;
    if (CHUNKED && --to_fold == 0 && kt + 1 < KT) {
      to_fold = p.kt_chunk;
      fresh = true;
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int v = 0; v < 16; ++v) tot[i][j][v] = tot[i][j][v] + acc[i][j][v];
    }
  }
  __syncthreads();

  // ---- epilogue: as in the implicit GEMM (bf16 output, no split parts) -------------------------
  float* epi = (float*)smem + wave * 32 * Cfg::EPI_STRIDE;
  constexpr int OCT = WTN / 8;
  constexpr int PAIRS = 32 * OCT / 64;
  auto epilogue = [&](auto act_c, auto res_c) {
    constexpr int ACT = decltype(act_c)::value, RES = decltype(res_c)::value;
    // Residual rows.  With several 32-row strips per wave they are all requested up front, so that
    // one round trip runs under the staging of the first strip instead of one per strip; with a
    // single strip the request goes after the staging writes, when the accumulators' registers are free.
    constexpr bool RES_UP_FRONT = TM > 1;
    uint4 r4[TM][PAIRS];
    auto load_res = [&](int i) {
#pragma unroll
      for (int t = 0; t < PAIRS; ++t) {
        const int id = t * 64 + lane;
        const int row = id / OCT, oct = id - row * OCT;
        const int m = m0 + wm * WTM + i * 32 + row;
        const int k = n0 + wn * WTN + oct * 8;
        r4[i][t] = (m < p.M && k < p.K) ? *(const uint4*)((const bf16_t*)p.res + (long)m * p.res_stride + k)
                                        : make_uint4(0, 0, 0, 0);
      }
    };
    if (RES != 0 && RES_UP_FRONT) {
#pragma unroll
      for (int i = 0; i < TM; ++i) load_res(i);
    }
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          epi[(8 * (v >> 2) + row_l + (v & 3)) * Cfg::EPI_STRIDE + j * 32 + col_l] =
              fmaf(CHUNKED ? tot[i][j][v] + acc[i][j][v] : acc[i][j][v], sc[j], sh[j]);
      if (RES != 0 && !RES_UP_FRONT) load_res(i);
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_s_waitcnt(0xc07f);        // lgkmcnt(0)
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int t = 0; t < PAIRS; ++t) {
        const int id = t * 64 + lane;
        const int row = id / OCT, oct = id - row * OCT;
        const int m = m0 + wm * WTM + i * 32 + row;
        const int k = n0 + wn * WTN + oct * 8;
        const float4 v0 = *(const float4*)(epi + row * Cfg::EPI_STRIDE + oct * 8);
        const float4 v1 = *(const float4*)(epi + row * Cfg::EPI_STRIDE + oct * 8 + 4);
        float val[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
        float rv[8];
        if (RES != 0) {
          const unsigned ru[4] = {r4[i][t].x, r4[i][t].y, r4[i][t].z, r4[i][t].w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            rv[2 * e] = __uint_as_float(ru[e] << 16);
            rv[2 * e + 1] = __uint_as_float(ru[e] & 0xffff0000u);
          }
        }
        if (RES == 1) {
#pragma unroll
          for (int e = 0; e < 8; ++e) val[e] += rv[e];
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) val[e] = apply_act(val[e], ACT);
        if (RES == 2) {
#pragma unroll
          for (int e = 0; e < 8; ++e) val[e] += rv[e];
        }
        if (m < p.M && k < p.K) {
          uint4 o;
          o.x = pack_bf16x2(val[0], val[1]);
          o.y = pack_bf16x2(val[2], val[3]);
          o.z = pack_bf16x2(val[4], val[5]);
          o.w = pack_bf16x2(val[6], val[7]);
          *(uint4*)((bf16_t*)p.y + (long)m * p.y_stride + k) = o;
        }
      }
      __builtin_amdgcn_wave_barrier();
    }
  };
  using std::integral_constant;
#define SNA_EPI(A, R) epilogue(integral_constant<int, A>{}, integral_constant<int, R>{})
  const int res_mode = p.res ? (p.res_after_act ? 2 : 1) : 0;
  if (p.act == SNA_ACT_RELU) {
    if (res_mode == 0) SNA_EPI(SNA_ACT_RELU, 0); else if (res_mode == 1) SNA_EPI(SNA_ACT_RELU, 1); else SNA_EPI(SNA_ACT_RELU, 2);
  } else if (p.act == SNA_ACT_NONE) {
    if (res_mode == 0) SNA_EPI(SNA_ACT_NONE, 0); else SNA_EPI(SNA_ACT_NONE, 1);
  } else if (p.act == SNA_ACT_HSWISH) {
    if (res_mode == 0) SNA_EPI(SNA_ACT_HSWISH, 0); else if (res_mode == 1) SNA_EPI(SNA_ACT_HSWISH, 1); else SNA_EPI(SNA_ACT_HSWISH, 2);
  } else {
    if (res_mode == 0) SNA_EPI(SNA_ACT_GELU, 0); else if (res_mode == 1) SNA_EPI(SNA_ACT_GELU, 1); else SNA_EPI(SNA_ACT_GELU, 2);
  }
#undef SNA_EPI
#endif
}

// Second half of a reduction that was split over blocks: adds the fp32 chunk sums in chunk order,
// then SubnetNorm scale/shift, residual and activation exactly as the fused epilogue does, so
// the output has the same bits as the one-block-per-tile path.  One thread = 8 channels of a row.
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const ConvGroupArgs args) {
  const int g = find_problem(args, blockIdx.x);
  const ConvProblem& p = args.p[g];
  const int k8n = p.K >> 3;
  const long idx = (long)(blockIdx.x - p.tile_start) * 256 + threadIdx.x;
  if (idx >= (long)p.M * k8n) return;
  const int m = (int)(idx / k8n);
  const int k = (int)(idx - (long)m * k8n) * 8;
  reduce_octet<false>(p, (const float*)p.x, m, k);
}

hipError_t launch_splitk_reduce(const ConvGroupArgs& a, hipStream_t s) {
  if (a.n == 0 || a.total_tiles == 0) return hipSuccess;
  hipLaunchKernelGGL(splitk_reduce_kernel, dim3(a.total_tiles), dim3(256), 0, s, a);
  return hipGetLastError();
}

struct Variant {
  int bm, bn, threads, smem, ns, stage_bytes, epi_bytes;
  void (*fn)(const ConvGroupArgs); void (*fn_chunked)(const ConvGroupArgs);
  bool slab;             // conv3_slab_kernel: 3x3 stride-1 layers only; stage_bytes is the weight ring's
};
#define SNA_VARIANT(BM, BN, WM, WN, NS) \
  { BM, BN, 64 * WM * WN, IgemmCfg<BM, BN, WM, WN, NS>::SMEM, NS, IgemmCfg<BM, BN, WM, WN, NS>::STAGE_B, \
    IgemmCfg<BM, BN, WM, WN, NS>::EPI_BYTES, igemm_kernel<BM, BN, WM, WN, NS, false, false>, igemm_kernel<BM, BN, WM, WN, NS, true, false>, false }
#define SNA_WS_VARIANT(BM, BN, WM, WN, NS) \
  { BM, BN, 128 * WM * WN, IgemmCfg<BM, BN, WM, WN, NS>::SMEM, NS, IgemmCfg<BM, BN, WM, WN, NS>::STAGE_B, \
    IgemmCfg<BM, BN, WM, WN, NS>::EPI_BYTES, igemm_kernel<BM, BN, WM, WN, NS, false, true>, igemm_kernel<BM, BN, WM, WN, NS, true, true>, false }
#define SNA_SLAB_VARIANT(BM, BN, WM, WN, NS) \
  { BM, BN, 64 * WM * WN, 0, NS, BN * ROW_B, IgemmCfg<BM, BN, WM, WN, NS>::EPI_BYTES, \
    conv3_slab_kernel<BM, BN, WM, WN, NS, false>, conv3_slab_kernel<BM, BN, WM, WN, NS, true>, true }
// 0..6 are the variants the shape heuristic chooses from; the rest are reached through tuning only.
static const Variant kVariants[] = {
    SNA_VARIANT(128, 128, 2, 2, 2), SNA_VARIANT(128, 64, 2, 2, 2), SNA_VARIANT(128, 96, 4, 1, 2),
    SNA_VARIANT(128, 32, 4, 1, 4),  SNA_VARIANT(64, 64, 2, 2, 4),  SNA_VARIANT(64, 128, 1, 4, 3),
    SNA_VARIANT(32, 128, 1, 4, 4),
    SNA_WS_VARIANT(64, 64, 2, 2, 4), SNA_WS_VARIANT(64, 128, 1, 4, 3), SNA_WS_VARIANT(128, 64, 2, 2, 3),
    SNA_WS_VARIANT(128, 96, 4, 1, 3), SNA_WS_VARIANT(128, 128, 2, 2, 3), SNA_VARIANT(128, 32, 4, 1, 2),
    SNA_WS_VARIANT(32, 128, 1, 4, 4), SNA_VARIANT(128, 192, 2, 2, 2), SNA_WS_VARIANT(128, 192, 2, 2, 3),
    // 16..: 3x3 stride-1 layers with the activation slab in LDS
    SNA_SLAB_VARIANT(128, 128, 2, 2, 2), SNA_SLAB_VARIANT(128, 64, 2, 2, 2), SNA_SLAB_VARIANT(128, 96, 4, 1, 2),
    SNA_SLAB_VARIANT(64, 64, 2, 2, 2), SNA_SLAB_VARIANT(64, 128, 1, 4, 2), SNA_SLAB_VARIANT(128, 96, 4, 1, 3),
    // 22..: one LDS stage, for short reductions: less LDS per block, more blocks per CU
    SNA_VARIANT(128, 128, 2, 2, 1), SNA_VARIANT(128, 64, 2, 2, 1), SNA_VARIANT(128, 96, 4, 1, 1), SNA_VARIANT(64, 128, 1, 4, 1),
    SNA_VARIANT(128, 32, 4, 1, 1), SNA_VARIANT(64, 64, 2, 2, 1),
};
constexpr int kNumVariants = sizeof(kVariants) / sizeof(kVariants[0]);
constexpr int kLdsMax = 160 * 1024;

int igemm_num_variants() { return kNumVariants; }
void igemm_tile_shape(int variant, int* bm, int* bn) {
  *bm = kVariants[variant].bm;
  *bn = kVariants[variant].bn;
}

// LDS a slab variant needs for one problem (all ring stages)
static int slab_smem(const Variant& v, const ConvProblem& p, int stages) {
  const int tiles = slab_units(v.bm, p.W, p.C8, v.threads) * 16 + stages * v.stage_bytes;
  return tiles > v.epi_bytes ? tiles : v.epi_bytes;
}

bool igemm_variant_ok(int variant, const ConvProblem& p) {
  if (variant < 0 || variant >= kNumVariants) return false;
  const Variant& v = kVariants[variant];
  if (!v.slab) return true;
  return p.R == 3 && p.S == 3 && p.stride == 1 && p.pad == 1 && p.parts == 1 && !p.out_fp32 && p.W >= 2 &&
         p.Ho == p.H && p.Wo == p.W && (long)(v.bm + 2 * p.W + 2) * (p.C8 | 1) < (1 << 20) &&
         slab_smem(v, p, v.ns) <= kLdsMax;
}

hipError_t launch_igemm(const ConvGroupArgs& a, int variant, bool chunked, hipStream_t s) {
  if (a.n == 0) return hipSuccess;
  if (variant < 0 || variant >= kNumVariants) return hipErrorInvalidValue;
  static std::atomic<bool> attr_done[kNumVariants][2];     // handles on several threads may get here together
  const Variant& v = kVariants[variant];
  void (*fn)(const ConvGroupArgs) = chunked ? v.fn_chunked : v.fn;
  if (!attr_done[variant][chunked].load(std::memory_order_acquire)) {
    hipError_t e = hipFuncSetAttribute((const void*)fn, hipFuncAttributeMaxDynamicSharedMemorySize, v.slab ? kLdsMax : v.smem);
    if (e != hipSuccess) return e;
    attr_done[variant][chunked].store(true, std::memory_order_release);
  }
  // a launch whose problems all have fewer K steps than the ring has stages only touches the
  // leading stages: asking for less LDS lets more blocks share a CU
  int kt_max = 1;
  for (int i = 0; i < a.n; ++i) {
    int kt = (a.p[i].K8 + 7) >> 3;
    if (kt > a.p[i].kt_part) kt = a.p[i].kt_part;
    if (kt > kt_max) kt_max = kt;
  }
  const int stages = kt_max < v.ns ? kt_max : v.ns;
  int smem = stages * v.stage_bytes > v.epi_bytes ? stages * v.stage_bytes : v.epi_bytes;
  if (v.slab) {
    smem = 0;
    for (int i = 0; i < a.n; ++i) {
      if (!igemm_variant_ok(variant, a.p[i])) return hipErrorInvalidValue;
      const int need = slab_smem(v, a.p[i], v.ns);
      if (need > smem) smem = need;
    }
  }
  const int blocks = (a.total_tiles + 7) / 8 * 8;
  hipLaunchKernelGGL(fn, dim3(blocks), dim3(v.threads), smem, s, a);
  return hipGetLastError();
}

}  // namespace sna
