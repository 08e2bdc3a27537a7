// HIP kernels of the PB tick engine (gfx950).
//
// One kernel, k_phase, executes every step of one pipeline phase: each
// workgroup looks up which step of the step table its block index falls in
// and runs that step's tile.  All stages' forward and backward work of a tick
// therefore goes out as a handful of launches (Appendix "GPU Bottlenecks for
// Fine-Grained Pipelined Training" names the launch rate as the limit for
// small networks).  Reductions use fixed trees: results are bit-reproducible.
#include "pb_device.h"

namespace pb {

// ------------------------------------------------------------------ helpers
// Pointers read out of the step table are generic to the compiler; accesses
// through generic pointers become flat loads whose completion has to be
// awaited conservatively.  Every buffer of the engine lives in global memory
// (address space 1) and every staging array in LDS (address space 3): say so.
typedef __attribute__((address_space(1))) float gfloat;
typedef __attribute__((address_space(1))) int32_t gint;
typedef __attribute__((address_space(3))) float lfloat;
typedef __attribute__((address_space(3))) int lint;

__device__ __forceinline__ gfloat* GP(float* p) { return (gfloat*)p; }
__device__ __forceinline__ const gfloat* GP(const float* p) { return (const gfloat*)p; }

// the workgroup's step descriptor lives in LDS
typedef __attribute__((address_space(3))) StepDesc LDesc;
typedef __attribute__((address_space(3))) TRef LTRef;
typedef __attribute__((address_space(3))) GemmCfg LGemmCfg;
#define UNI(x) __builtin_amdgcn_readfirstlane(x)   /* integer value that is the same in every lane: keep it scalar */
#define UNIF(x) __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(x)))   /* the same for a float */
#ifdef PB_TIMING
__shared__ long long ts_sh[4][24];
__device__ long long pb_ts_out[16384 * 100];
__device__ int pb_ts_n;
__device__ int pb_ts_tick;
__device__ int pb_ts_grid;   // 0: record every phase, else only the launch with this many workgroups
#if PB_TIMING == 2   /* light form: start and end of a workgroup only, no atomics */
#define PB_TS(i) do { if ((i) == 0 || (i) == 11) { if ((threadIdx.x & 63) == 0) ts_sh[threadIdx.x >> 6][i] = (long long)__builtin_amdgcn_s_memrealtime(); } } while (0)
#else
#define PB_TS(i) do { if ((threadIdx.x & 63) == 0) ts_sh[threadIdx.x >> 6][i] = (long long)__builtin_amdgcn_s_memrealtime(); } while (0)
#endif
#else
#define PB_TS(i)
#endif

// floor(n / d) for 0 <= n < 2^21, d >= 1, with inv = rcp(d): a few instructions
// instead of the long expansion of an integer division
__device__ __forceinline__ float frcp(int d) { return __builtin_amdgcn_rcpf((float)d); }
__device__ __forceinline__ int fdiv(int n, float inv) { return (int)(((float)n + 0.5f) * inv); }

// Round to the nearest bf16 value (ties to even), kept in a float.  bf16 activation mode rounds
// every tensor that crosses a stage boundary or is kept for the backward pass.
__device__ __forceinline__ float rbf(float x) {
  unsigned u = __float_as_uint(x);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return __uint_as_float(u & 0xFFFF0000u);
}
__device__ __forceinline__ float rbf_if(bool on, float x) { return on ? rbf(x) : x; }

__device__ __forceinline__ gfloat* at(const LTRef& r, int t) {
  const int depth = UNI(r.depth), stride = UNI(r.stride), lag = UNI(r.lag);
  int slot = (t - lag) % depth;
  if (slot < 0) slot += depth;
  return (gfloat*)r.base + (size_t)slot * (size_t)stride;
}

__device__ __forceinline__ gfloat* at(const TRef& r, int t) {
  int u = t - r.lag;
  int slot = u % r.depth;
  if (slot < 0) slot += r.depth;
  return (gfloat*)r.base + (size_t)slot * (size_t)r.stride;
}

// Cross-lane operand through the data-parallel-primitive path of the vector
// ALU (no LDS round trip): lanes without a source, or in rows masked out,
// read 0.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_src(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, ROW_MASK, 0xF, false));
}

// Sum over the wavefront, returned to every lane (fixed order).
__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_src<0xB1, 0xF>(v);    // quad_perm [1,0,3,2]
  v += dpp_src<0x4E, 0xF>(v);    // quad_perm [2,3,0,1]
  v += dpp_src<0x141, 0xF>(v);   // row_half_mirror
  v += dpp_src<0x140, 0xF>(v);   // row_mirror: every lane holds the sum of its row of 16
  v += dpp_src<0x142, 0xA>(v);   // row_bcast:15 into rows 1 and 3
  v += dpp_src<0x143, 0xC>(v);   // row_bcast:31 into rows 2 and 3: lane 63 holds the total
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

// Sum over each row of 16 lanes, returned to every lane of the row (fixed order).
__device__ __forceinline__ float row_sum(float v) {
  v += dpp_src<0xB1, 0xF>(v);    // quad_perm [1,0,3,2]
  v += dpp_src<0x4E, 0xF>(v);    // quad_perm [2,3,0,1]
  v += dpp_src<0x141, 0xF>(v);   // row_half_mirror
  v += dpp_src<0x140, 0xF>(v);   // row_mirror
  return v;
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// Sum over the workgroup, same value returned to every thread.
__device__ __forceinline__ float block_sum(float v, lfloat* red) {
  v = wave_sum(v);
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 0) red[wv] = v;
  __syncthreads();
  return (red[0] + red[1]) + (red[2] + red[3]);
}

__device__ __forceinline__ float block_max(float v, lfloat* red) {
  v = wave_max(v);
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 0) red[wv] = v;
  __syncthreads();
  return fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}

}  // namespace pb
#include "pb_gemm.h"
namespace pb {

// Sum of the `parts` partial results p[0], p[stride], ... (at most MAX_PARTS of them) in order, BATCH
// loads requested before the first of them is added: a loop of load-then-add pays a memory round
// trip per part.
constexpr int MAX_PARTS = 8;
template <class T, int BATCH, class P>
__device__ __forceinline__ T sum_parts(const P* p, size_t stride, int parts) {
  T a;
#pragma unroll
  for (int q0 = 0; q0 < MAX_PARTS; q0 += BATCH) {
    if (q0 < parts) {
      T v[BATCH];
#pragma unroll
      for (int q = 0; q < BATCH; ++q)
        if (q0 + q < parts) v[q] = p[(q0 + q) * stride];
#pragma unroll
      for (int q = 0; q < BATCH; ++q)
        if (q0 + q < parts) a = (q0 + q == 0) ? v[q] : a + v[q];
    }
  }
  return a;
}

// ------------------------------------------------------------ forward steps
// GroupNorm statistics of one group (biased variance, two passes) and the
// folded per-channel scale/shift built from the forward (predicted) affine
// parameters; kept for the backward pass of the same sample.
// GU: 16-byte registers per thread; a group of up to GU * 1024 elements stays in registers
template <int GU>
__device__ __forceinline__ bool step_gn_stats_reg(const LDesc& d, int tile, int t, lfloat* red, lfloat* smem, const bool nt) {
  const int tid = threadIdx.x;
  const int C = UNI(d.C), G = UNI(d.G), HW = UNI(d.H) * UNI(d.W);
  const int g = tile, cpg = UNI(fdiv(C, frcp(G))), n = cpg * HW;
  const gfloat* xp = at(d.x, t) + (size_t)g * n;
  gfloat* st = at(d.st, t);
  const bool rl = UNI(d.flags) & F_PRE_RELU;
  {
    // one burst of reads: the group, and its channels' affine parameters
    v4f xr[GU];
#pragma unroll
    for (int u = 0; u < GU; ++u) {
      const int i = (tid + u * BLK) * 4;
      xr[u] = (v4f){0.f, 0.f, 0.f, 0.f};
      if (i < n) xr[u] = *(const gv4*)(xp + i);
    }
    // The layer's forward GEMM was split over its reduction and left partial sums: the
    // statistics step adds them up in order (the first part stands in for the tensor read
    // above) and writes the tensor for the steps that read it after this one.
    const int gparts = nt ? 1 : UNI(d.gparts);   // (only in the instantiation for networks tiled for throughput)
    if (gparts > 1) {
      const gfloat* part = GP(d.gw) + (size_t)g * n;
      const size_t ps = (size_t)UNI(d.gpstride);
#pragma unroll
      for (int u = 0; u < GU; ++u) {
        const int i = (tid + u * BLK) * 4;
        if (i < n) {
          const v4f a = sum_parts<v4f, 2>((const gv4*)(part + i), ps >> 2, gparts);
          xr[u] = a;
          *(gv4*)((gfloat*)xp + i) = a;
        }
      }
    }
    float gam = 0.f, bet = 0.f;
    if (tid < cpg) { gam = GP(d.gamma)[g * cpg + tid]; bet = GP(d.beta)[g * cpg + tid]; }
    float s = 0.f;
#pragma unroll
    for (int u = 0; u < GU; ++u) s += (xr[u][0] + xr[u][1]) + (xr[u][2] + xr[u][3]);
    const float mean = block_sum(s, red) / (float)n;
    float q = 0.f;
#pragma unroll
    for (int u = 0; u < GU; ++u)
      if ((tid + u * BLK) * 4 < n) {
#pragma unroll
        for (int e = 0; e < 4; ++e) { const float dl = xr[u][e] - mean; q = fmaf(dl, dl, q); }
      }
    const float var = block_sum(q, red) / (float)n;
    const float rstd = 1.0f / sqrtf(var + GN_EPS);
    if (tid == 0) { st[g] = mean; st[G + g] = rstd; }
    if (tid < cpg) {
      const int ch = g * cpg + tid;
      const float sc = gam * rstd, sh = fmaf(-mean, sc, bet);
      st[2 * G + ch] = sc;
      st[2 * G + C + ch] = sh;
      smem[tid] = sc; smem[cpg + tid] = sh;
    }
    if (d.y.base) {
      // the normalised (and rectified) group, kept for the convolution of this
      // tick and for the weight gradient of the same sample D ticks later
      __syncthreads();
      gfloat* yo = at(d.y, t) + (size_t)g * n;
      const float ihw = frcp(HW);
#pragma unroll
      for (int u = 0; u < GU; ++u) {
        const int i = (tid + u * BLK) * 4;
        if (i < n) {
          v4f o;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int c = fdiv(i + e, ihw);
            float v = fmaf(smem[c], xr[u][e], smem[cpg + c]);
            if (rl) v = fmaxf(v, 0.f);
            o[e] = v;
          }
          PB_ST(nt, (gv4*)(yo + i), o);
        }
      }
    }
    return true;
  }
}

__device__ __forceinline__ void step_gn_stats(const LDesc& d, int tile, int t, lfloat* red, lfloat* smem, const bool nt) {
  const int tid = threadIdx.x;
  const int C = UNI(d.C), G = UNI(d.G), HW = UNI(d.H) * UNI(d.W);
  const int g = tile, cpg = UNI(fdiv(C, frcp(G))), n = cpg * HW;
  const gfloat* xp = at(d.x, t) + (size_t)g * n;
  gfloat* st = at(d.st, t);
  const bool rl = UNI(d.flags) & F_PRE_RELU;
  if ((n & 3) == 0 && cpg <= BLK) {
    if (n <= 8 * 4 * BLK) { step_gn_stats_reg<8>(d, tile, t, red, smem, nt); return; }
    if (n <= 32 * 4 * BLK) { step_gn_stats_reg<32>(d, tile, t, red, smem, nt); return; }
  }
  float s = 0.f;
  for (int i = tid; i < n; i += BLK) s += xp[i];
  const float mean = block_sum(s, red) / (float)n;
  float q = 0.f;
  for (int i = tid; i < n; i += BLK) { float dl = xp[i] - mean; q = fmaf(dl, dl, q); }
  const float var = block_sum(q, red) / (float)n;
  const float rstd = 1.0f / sqrtf(var + GN_EPS);
  if (tid == 0) { st[g] = mean; st[G + g] = rstd; }
  for (int c = tid; c < cpg; c += BLK) {
    const int ch = g * cpg + c;
    const float sc = GP(d.gamma)[ch] * rstd;
    st[2 * G + ch] = sc;
    st[2 * G + C + ch] = fmaf(-mean, sc, GP(d.beta)[ch]);
  }
  if (d.y.base) {
    gfloat* yo = at(d.y, t) + (size_t)g * n;
    for (int i = tid; i < n; i += BLK) {
      const int ch = g * cpg + i / HW;
      const float sc = GP(d.gamma)[ch] * rstd;
      float v = fmaf(sc, xp[i], fmaf(-mean, sc, GP(d.beta)[ch]));
      if (rl) v = fmaxf(v, 0.f);
      yo[i] = v;
    }
  }
}

// The same with one wavefront per group and all four groups of the layer in one
// workgroup (grain = 1; groups of at most 4096 elements, at most 64 channels per
// group): sums across lanes only, no barrier, and a quarter of the workgroups.
// LDS: per wavefront sc[64] | sh[64].
constexpr int GNS_WAVE_MAX_N = 4096;
__device__ __forceinline__ void step_gn_stats_wave(const LDesc& d, int t, lfloat* smem, const bool nt) {
  const int lane = threadIdx.x & 63, g = UNI(threadIdx.x >> 6);
  const int C = UNI(d.C), G = UNI(d.G), HW = UNI(d.H) * UNI(d.W);
  const int cpg = UNI(fdiv(C, frcp(G))), n = cpg * HW;
  if (g >= G) return;
  const gfloat* xp = at(d.x, t) + (size_t)g * n;
  gfloat* st = at(d.st, t);
  const bool rl = UNI(d.flags) & F_PRE_RELU;
  constexpr int WU = GNS_WAVE_MAX_N / (4 * 64);
  v4f xr[WU];
#pragma unroll
  for (int u = 0; u < WU; ++u) {
    const int i = (lane + u * 64) * 4;
    xr[u] = (v4f){0.f, 0.f, 0.f, 0.f};
    if (u * 256 < n) {
      if (i < n) xr[u] = *(const gv4*)(xp + i);
    }
  }
  float gam = 0.f, bet = 0.f;
  if (lane < cpg) { gam = GP(d.gamma)[g * cpg + lane]; bet = GP(d.beta)[g * cpg + lane]; }
  float s = 0.f;
#pragma unroll
  for (int u = 0; u < WU; ++u) s += (xr[u][0] + xr[u][1]) + (xr[u][2] + xr[u][3]);
  const float mean = wave_sum(s) / (float)n;
  float q = 0.f;
#pragma unroll
  for (int u = 0; u < WU; ++u)
    if ((lane + u * 64) * 4 < n) {
#pragma unroll
      for (int e = 0; e < 4; ++e) { const float dl = xr[u][e] - mean; q = fmaf(dl, dl, q); }
    }
  const float var = wave_sum(q) / (float)n;
  const float rstd = 1.0f / sqrtf(var + GN_EPS);
  if (lane == 0) { st[g] = mean; st[G + g] = rstd; }
  lfloat* sc_l = smem + g * 128;
  lfloat* sh_l = sc_l + 64;
  if (lane < cpg) {
    const int ch = g * cpg + lane;
    const float sc = gam * rstd, sh = fmaf(-mean, sc, bet);
    st[2 * G + ch] = sc;
    st[2 * G + C + ch] = sh;
    sc_l[lane] = sc; sh_l[lane] = sh;
  }
  if (!d.y.base) return;
  // (LDS operations of one wavefront complete in order: the values are there)
  __builtin_amdgcn_wave_barrier();
  gfloat* yo = at(d.y, t) + (size_t)g * n;
  const float ihw = frcp(HW);
#pragma unroll
  for (int u = 0; u < WU; ++u) {
    const int i = (lane + u * 64) * 4;
    if (u * 256 < n) {
      if (i < n) {
        const int c = fdiv(i, ihw);   // H*W is a multiple of 4: the four elements share a channel
        const float sc = sc_l[c], sh = sh_l[c];
        v4f o;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          float v = fmaf(sc, xr[u][e], sh);
          if (rl) v = fmaxf(v, 0.f);
          o[e] = v;
        }
        PB_ST(nt, (gv4*)(yo + i), o);
      }
    }
  }
}

// pooled[c] = mean_hw relu(sc*x+sh)
__device__ __forceinline__ void step_gap_fwd(const LDesc& d, int tile, int t, lfloat* red) {
  const int c = tile, HW = d.H * d.W;
  const gfloat* xp = at(d.x, t) + (size_t)c * HW;
  const bool aff = d.flags & F_PRE_AFFINE, rl = d.flags & F_PRE_RELU;
  const gfloat* st = aff ? at(d.st, t) : nullptr;
  const float sc = aff ? st[2 * d.G + c] : 1.f, sh = aff ? st[2 * d.G + d.C + c] : 0.f;
  float s = 0.f;
  for (int i = threadIdx.x; i < HW; i += BLK) {
    float v = fmaf(sc, xp[i], sh);
    if (rl) v = fmaxf(v, 0.f);
    s += v;
  }
  s = block_sum(s, red);
  if (threadIdx.x == 0) at(d.y, t)[c] = s / (float)HW;
}

// Direct convolution / linear forward, one thread per output element.
__device__ __forceinline__ void step_conv_fwd(const LDesc& d, int tile, int t) {
  const int P = d.OH * d.OW;
  const int o = tile * BLK + threadIdx.x;
  if (o >= d.K * P) return;
  const int co = o / P, p = o - co * P, oh = p / d.OW, ow = p - oh * d.OW;
  const gfloat* x = at(d.x, t);
  const gfloat* st = (d.flags & F_PRE_AFFINE) ? at(d.st, t) : nullptr;
  const bool aff = d.flags & F_PRE_AFFINE, rl = d.flags & F_PRE_RELU;
  const int HW = d.H * d.W, kk = d.k * d.k;
  float acc = (d.flags & F_BIAS) ? GP(d.b)[co] : 0.f;
  const gfloat* wr = GP(d.w) + (size_t)co * d.C * kk;
  for (int ci = 0; ci < d.C; ++ci) {
    const float sc = aff ? st[2 * d.G + ci] : 1.f, sh = aff ? st[2 * d.G + d.C + ci] : 0.f;
    const gfloat* xc = x + (size_t)ci * HW;
    for (int kh = 0; kh < d.k; ++kh) {
      const int ih = oh * d.stride - d.pad + kh;
      if (ih < 0 || ih >= d.H) continue;
      for (int kw = 0; kw < d.k; ++kw) {
        const int iw = ow * d.stride - d.pad + kw;
        if (iw < 0 || iw >= d.W) continue;
        float v = xc[ih * d.W + iw];
        if (aff) v = fmaf(sc, v, sh);
        if (rl) v = fmaxf(v, 0.f);
        acc = fmaf(wr[ci * kk + kh * d.k + kw], v, acc);
      }
    }
  }
  if (d.flags & F_SKIP) {
    const gfloat* sk = at(d.skip, t);
    if (d.flags & F_PROJ) {
      const int sHW = d.sH * d.sW;
      const gfloat* s0 = sk + (size_t)(oh * d.sstride) * d.sW + ow * d.sstride;
      float a2 = 0.f;
      for (int ci = 0; ci < d.sC; ++ci) a2 = fmaf(GP(d.wp)[(size_t)co * d.sC + ci], s0[(size_t)ci * sHW], a2);
      acc += a2;
    } else {
      acc += sk[o];
    }
  }
  at(d.y, t)[o] = acc;
}

// y = [maxpool] relu(sc*z+sh), one thread per output element.
__device__ __forceinline__ void step_post_fwd(const LDesc& d, int tile, int t) {
  const gfloat* z = at(d.x, t);
  const gfloat* st = at(d.st, t);
  gfloat* y = at(d.y, t);
  const int HW = d.H * d.W;
  if (d.flags & F_POOL) {
    const int PP = d.PH * d.PW;
    const int o = tile * BLK + threadIdx.x;
    if (o >= d.C * PP) return;
    const int c = o / PP, p = o - c * PP, ph = p / d.PW, pw = p - ph * d.PW;
    const float sc = st[2 * d.G + c], sh = st[2 * d.G + d.C + c];
    const gfloat* zc = z + (size_t)c * HW;
    float best = -1.f;
    for (int kh = 0; kh < d.pk; ++kh) {
      const int ih = ph * d.ps - d.pp + kh;
      if (ih < 0 || ih >= d.H) continue;
      for (int kw = 0; kw < d.pk; ++kw) {
        const int iw = pw * d.ps - d.pp + kw;
        if (iw < 0 || iw >= d.W) continue;
        best = fmaxf(best, fmaxf(fmaf(sc, zc[ih * d.W + iw], sh), 0.f));
      }
    }
    y[o] = rbf_if(d.flags & F_BF16_OUT, best);
  } else {
    const int o = tile * BLK + threadIdx.x;
    if (o >= d.C * HW) return;
    const int c = o / HW;
    y[o] = rbf_if(d.flags & F_BF16_OUT, fmaxf(fmaf(st[2 * d.G + c], z[o], st[2 * d.G + d.C + c]), 0.f));
  }
}

// Softmax cross-entropy of the sample that reaches the last stage at tick t
// (sample index t-(S-1)); writes dlogits = softmax - onehot.
__device__ __forceinline__ void step_ce(const LDesc& d, int tile, int t, lfloat* red) {
  const gfloat* z = at(d.x, t);
  gfloat* dz = at(d.dx, t);
  const int n = d.n;
  const int sample = t - (d.n_stages - 1);
  const int label = ((const gint*)d.labels)[sample % d.n_stages];
  float mx = -3.0e38f;
  for (int i = threadIdx.x; i < n; i += BLK) mx = fmaxf(mx, z[i]);
  mx = block_max(mx, red);
  float s = 0.f;
  for (int i = threadIdx.x; i < n; i += BLK) s += expf(z[i] - mx);
  s = block_sum(s, red);
  for (int i = threadIdx.x; i < n; i += BLK) {
    float p = expf(z[i] - mx) / s;
    dz[i] = p - (i == label ? 1.f : 0.f);
  }
  if (threadIdx.x == 0) GP(d.loss_log)[sample % d.loss_cap] = logf(s) + mx - z[label];
}

// ----------------------------------------------------------- backward steps
// Gradient arriving at element (h,w) of channel c of the tensor u = relu(affine(z))
// that feeds a max-pool: the sum of dY over the windows whose first maximum
// (row-major scan, strict >) sits at (h,w).
// PK > 0: window size known at compile time (the nine reads of a 3x3 window are then
// requested together instead of one by one)
template <int PK, class PZ, class PD>   // pointers to the channel's map and to its pooled gradient: global memory or LDS
__device__ __forceinline__ float pool_routed_k(const LDesc& d, PZ zc, float sc, float sh,
                                               int h, int w, PD dyc) {
  // window geometry in scalar registers; divisions by the pooling stride through a reciprocal
  const int pk = PK > 0 ? PK : UNI(d.pk);
  const int ps = UNI(d.ps), pp = UNI(d.pp), H = UNI(d.H), W = UNI(d.W), PH = UNI(d.PH), PW = UNI(d.PW);
  const float ips = frcp(ps);
  float sum = 0.f;
  int ph_lo = h + pp - pk + 1;
  ph_lo = ph_lo <= 0 ? 0 : fdiv(ph_lo + ps - 1, ips);
  int ph_hi = fdiv(h + pp, ips);
  if (ph_hi >= PH) ph_hi = PH - 1;
  int pw_lo = w + pp - pk + 1;
  pw_lo = pw_lo <= 0 ? 0 : fdiv(pw_lo + ps - 1, ips);
  int pw_hi = fdiv(w + pp, ips);
  if (pw_hi >= PW) pw_hi = PW - 1;
  for (int ph = ph_lo; ph <= ph_hi; ++ph)
    for (int pw = pw_lo; pw <= pw_hi; ++pw) {
      float best = -1.f;
      int bi = -1;
      const int ih0 = ph * ps - pp, iw0 = pw * ps - pp;
      if (PK > 0) {
        float zv[PK > 0 ? PK * PK : 1];
#pragma unroll
        for (int kh = 0; kh < PK; ++kh)
#pragma unroll
          for (int kw = 0; kw < PK; ++kw) {
            const int ih = ih0 + kh, iw = iw0 + kw;
            const bool in = ih >= 0 && ih < H && iw >= 0 && iw < W;
            zv[kh * PK + kw] = zc[in ? ih * W + iw : 0];
          }
#pragma unroll
        for (int kh = 0; kh < PK; ++kh)
#pragma unroll
          for (int kw = 0; kw < PK; ++kw) {
            const int ih = ih0 + kh, iw = iw0 + kw;
            const bool in = ih >= 0 && ih < H && iw >= 0 && iw < W;
            const float v = fmaxf(fmaf(sc, zv[kh * PK + kw], sh), 0.f);
            if (in && v > best) { best = v; bi = ih * W + iw; }
          }
      } else {
        for (int kh = 0; kh < pk; ++kh) {
          const int ih = ih0 + kh;
          if (ih < 0 || ih >= H) continue;
          for (int kw = 0; kw < pk; ++kw) {
            const int iw = iw0 + kw;
            if (iw < 0 || iw >= W) continue;
            const float v = fmaxf(fmaf(sc, zc[ih * W + iw], sh), 0.f);
            if (v > best) { best = v; bi = ih * W + iw; }
          }
        }
      }
      if (bi == h * W + w) sum += dyc[ph * PW + pw];
    }
  return sum;
}

template <class PZ, class PD>
__device__ __forceinline__ float pool_routed(const LDesc& d, PZ zc, float sc, float sh, int h, int w, PD dyc) {
  if (UNI(d.pk) == 3) return pool_routed_k<3>(d, zc, sc, sh, h, w, dyc);
  if (UNI(d.pk) == 2) return pool_routed_k<2>(d, zc, sc, sh, h, w, dyc);
  return pool_routed_k<0>(d, zc, sc, sh, h, w, dyc);
}

__device__ __forceinline__ float gn_du(const LDesc& d, const gfloat* dy, const gfloat* xc, float sc,
                                       float sh, int c, int i, int HW) {
  if (d.flags & F_DU_BUF) return dy[(size_t)c * HW + i];
  if (d.flags & F_DU_GAP) return dy[c] / (float)HW;
  const int h = i / d.W, w = i - h * d.W;
  return pool_routed(d, xc, sc, sh, h, w, dy + (size_t)c * d.PH * d.PW);
}

// Per channel: dgamma = sum dyv*xh, dbeta = sum dyv (dyv = gradient after the
// ReLU mask); also gamma_b*dbeta and gamma_b*dgamma for the group sums.
// One wavefront per channel, GNB_WAVE_CH channels per wavefront (small maps: a
// workgroup per channel would leave most of its lanes without an element, and a
// workgroup that lives for one memory round trip wastes its slot).  The loads of
// all of a wavefront's channels are requested before the first sum.  Plain
// gradient buffers, or gradients routed back through a max-pool.
__device__ __forceinline__ void step_gnb_reduce_wave(const LDesc& d, int tile, int t, lfloat* smem, const bool nt) {
  const int lane = threadIdx.x & 63;
  const int c0 = (tile * (BLK / 64) + UNI((int)(threadIdx.x >> 6))) * GNB_WAVE_CH;
  const int C = UNI(d.C), G = UNI(d.G), HW = UNI(d.H) * UNI(d.W);
  if (c0 >= C) return;
  const int cpg = UNI(fdiv(C, frcp(G)));
  const gfloat* st = at(d.st, t);
  const gfloat* x = at(d.x, t);
  const gfloat* dy = at(d.dy, t);
  const bool rl = UNI(d.flags) & F_GN_RELU, pooled = UNI(d.flags) & F_DU_POOL;
  constexpr int RU = 4;
  // The incoming gradient was left as partial sums by a backward-data GEMM split over its
  // reduction (at most 64 values per channel): add them up in order, write the gradient for
  // the elementwise pass that reads it in a later launch, and keep it in LDS for this step.
  const int gparts = nt ? 1 : UNI(d.gparts);   // (only in the instantiation for networks tiled for throughput)
  lfloat* ls = smem + UNI((int)(threadIdx.x >> 6)) * (GNB_WAVE_CH * 64);
  if (gparts > 1) {
    const int n_dy = pooled ? UNI(d.PH) * UNI(d.PW) : HW;
    const gfloat* part = GP(d.gw);
    const size_t ps = (size_t)UNI(d.gpstride);
#pragma unroll
    for (int q = 0; q < GNB_WAVE_CH; ++q) {
      const int c = c0 + q;
      if (c < C && lane < n_dy) {
        const size_t o = (size_t)c * n_dy + lane;
        const float s = sum_parts<float, 8>(part + o, ps, gparts);
        ((gfloat*)dy)[o] = s;
        ls[q * 64 + lane] = s;
      }
    }
    __builtin_amdgcn_wave_barrier();
  }
  float xv[GNB_WAVE_CH][RU], dv[GNB_WAVE_CH][RU], mean[GNB_WAVE_CH], rstd[GNB_WAVE_CH], sc[GNB_WAVE_CH], sh[GNB_WAVE_CH],
      gm[GNB_WAVE_CH];
#pragma unroll
  for (int q = 0; q < GNB_WAVE_CH; ++q) {
    const int c = c0 + q;
    mean[q] = rstd[q] = sc[q] = sh[q] = gm[q] = 0.f;
#pragma unroll
    for (int u = 0; u < RU; ++u) { xv[q][u] = 0.f; dv[q][u] = 0.f; }
    if (c < C) {
      const int g = UNI(fdiv(c, frcp(cpg)));
#pragma unroll
      for (int u = 0; u < RU; ++u) {
        const int i = lane + u * 64;
        if (i < HW) { xv[q][u] = x[(size_t)c * HW + i]; if (!pooled) dv[q][u] = dy[(size_t)c * HW + i]; }
      }
      mean[q] = st[g]; rstd[q] = st[G + g]; sc[q] = st[2 * G + c]; sh[q] = st[2 * G + C + c];
      gm[q] = GP(d.gamma)[c];
      if (pooled) {   // gradient routed back through the max-pool (needs the channel's scale and shift)
#pragma unroll
        for (int u = 0; u < RU; ++u) {
          const int i = lane + u * 64;
          if (i < HW && gparts <= 1) dv[q][u] = gn_du(d, dy, x + (size_t)c * HW, sc[q], sh[q], c, i, HW);
        }
      }
    }
  }
  if (gparts > 1) {   // (maps of at most 64 pixels: u = 0 only) the summed gradient from LDS
    const int W = UNI(d.W), h = fdiv(lane, frcp(W)), w = lane - h * W;
#pragma unroll
    for (int q = 0; q < GNB_WAVE_CH; ++q) {
      const int c = c0 + q;
      if (c < C && lane < HW)
        dv[q][0] = pooled ? pool_routed(d, x + (size_t)c * HW, sc[q], sh[q], h, w, (const lfloat*)(ls + q * 64)) : ls[q * 64 + lane];
    }
  }
#pragma unroll
  for (int q = 0; q < GNB_WAVE_CH; ++q) {
    const int c = c0 + q;
    if (c >= C) break;
    float sg = 0.f, sb = 0.f;
#pragma unroll
    for (int u = 0; u < RU; ++u) {
      if (lane + u * 64 < HW) {
        const float yv = fmaf(sc[q], xv[q][u], sh[q]);
        float du = dv[q][u];
        if (rl && !(yv > 0.f)) du = 0.f;
        sg = fmaf(du, (xv[q][u] - mean[q]) * rstd[q], sg);
        sb += du;
      }
    }
    for (int i = lane + RU * 64; i < HW; i += 64) {
      const float x1 = x[(size_t)c * HW + i];
      const float yv = fmaf(sc[q], x1, sh[q]);
      float du = pooled ? gn_du(d, dy, x + (size_t)c * HW, sc[q], sh[q], c, i, HW) : dy[(size_t)c * HW + i];
      if (rl && !(yv > 0.f)) du = 0.f;
      sg = fmaf(du, (x1 - mean[q]) * rstd[q], sg);
      sb += du;
    }
    sg = wave_sum(sg);
    sb = wave_sum(sb);
    if (lane == 0) {
      GP(d.ggamma)[c] = sg;
      GP(d.gbeta)[c] = sb;
      GP(d.part)[c] = gm[q] * sb;
      GP(d.part)[C + c] = gm[q] * sg;
      GP(d.part)[2 * C + c] = gm[q];
    }
  }
}

__device__ __forceinline__ void step_gnb_reduce(const LDesc& d, int tile, int t, lfloat* red, lfloat* smem, const bool nt) {
  if (UNI(d.grain) == 1) { step_gnb_reduce_wave(d, tile, t, smem, nt); return; }
  const int c = tile, HW = UNI(d.H) * UNI(d.W), cpg = UNI(fdiv(UNI(d.C), frcp(UNI(d.G)))), g = UNI(fdiv(c, frcp(cpg)));
  const gfloat* st = at(d.st, t);
  const float mean = st[g], rstd = st[d.G + g], sc = st[2 * d.G + c], sh = st[2 * d.G + d.C + c];
  const gfloat* xc = at(d.x, t) + (size_t)c * HW;
  const gfloat* dy = at(d.dy, t);
  const bool rl = d.flags & F_GN_RELU;
  float sg = 0.f, sb = 0.f;
  if ((d.flags & (F_DU_BUF | F_DU_GAP)) && (HW & 3) == 0) {
    // plain gradient buffer (or a pooled one): both operands with 16-byte loads, all in flight
    const float dug = (d.flags & F_DU_GAP) ? dy[c] / (float)HW : 0.f;
    constexpr int RU = 4;
    for (int base = threadIdx.x * 4; base < HW; base += RU * 4 * BLK) {
      v4f xv[RU], dv[RU];
#pragma unroll
      for (int u = 0; u < RU; ++u) {
        const int i = base + u * 4 * BLK;
        xv[u] = (v4f){0.f, 0.f, 0.f, 0.f}; dv[u] = xv[u];
        if (i < HW) {
          xv[u] = *(const gv4*)(xc + i);
          if (d.flags & F_DU_BUF) dv[u] = *(const gv4*)(dy + (size_t)c * HW + i);
          else dv[u] = (v4f){dug, dug, dug, dug};
        }
      }
#pragma unroll
      for (int u = 0; u < RU; ++u)
        if (base + u * 4 * BLK < HW) {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float yv = fmaf(sc, xv[u][e], sh);
            float du = dv[u][e];
            if (rl && !(yv > 0.f)) du = 0.f;
            sg = fmaf(du, (xv[u][e] - mean) * rstd, sg);
            sb += du;
          }
        }
    }
  } else if ((d.flags & F_DU_POOL) && HW + UNI(d.PH) * UNI(d.PW) <= LDS_FLOATS) {
    // gradient routed back through a max-pool: every element looks at up to four pooling
    // windows of nine inputs.  The channel's map and its pooled gradient are fetched once,
    // with coalesced loads, and the window searches read LDS.
    const int PHW = UNI(d.PH) * UNI(d.PW), W = UNI(d.W);
    lfloat* zs = smem;
    lfloat* ds = smem + HW;
    const gfloat* dyc = dy + (size_t)c * PHW;
    if ((HW & 3) == 0) {
      for (int i = threadIdx.x * 4; i < HW; i += 4 * BLK) *(lv4*)(zs + i) = *(const gv4*)(xc + i);
    } else {
      for (int i = threadIdx.x; i < HW; i += BLK) zs[i] = xc[i];
    }
    // (the pooled gradient may have been left as partial sums by a backward-data GEMM split over its reduction:
    // add them up in order and write the gradient for the elementwise pass of a later launch)
    const int gparts = nt ? 1 : UNI(d.gparts);
    if (gparts > 1) {
      const gfloat* part = GP(d.gw) + (size_t)c * PHW;
      for (int i = threadIdx.x; i < PHW; i += BLK) {
        const float sv = sum_parts<float, 8>(part + i, (size_t)UNI(d.gpstride), gparts);
        ds[i] = sv;
        ((gfloat*)dyc)[i] = sv;
      }
    } else {
      for (int i = threadIdx.x; i < PHW; i += BLK) ds[i] = dyc[i];
    }
    __syncthreads();
    const float iw = frcp(W);
    for (int i = threadIdx.x; i < HW; i += BLK) {
      const float xv = zs[i];
      const float yv = fmaf(sc, xv, sh);
      const int h = fdiv(i, iw), w = i - h * W;
      float du = pool_routed(d, (const lfloat*)zs, sc, sh, h, w, (const lfloat*)ds);
      if (rl && !(yv > 0.f)) du = 0.f;
      sg = fmaf(du, (xv - mean) * rstd, sg);
      sb += du;
    }
  } else {
    for (int i = threadIdx.x; i < HW; i += BLK) {
      const float xv = xc[i];
      const float yv = fmaf(sc, xv, sh);
      float du = gn_du(d, dy, xc, sc, sh, c, i, HW);
      if (rl && !(yv > 0.f)) du = 0.f;
      sg = fmaf(du, (xv - mean) * rstd, sg);
      sb += du;
    }
  }
  sg = block_sum(sg, red);
  sb = block_sum(sb, red);
  if (threadIdx.x == 0) {
    GP(d.ggamma)[c] = sg;
    GP(d.gbeta)[c] = sb;
    const float gm = GP(d.gamma)[c];
    GP(d.part)[c] = gm * sb;
    GP(d.part)[d.C + c] = gm * sg;
    GP(d.part)[2 * d.C + c] = gm;   // the elementwise pass must not read the parameter arena (it may run beside the update)
  }
}

// dx = rstd * (dxh - mean(dxh) - xh * mean(dxh*xh)), dxh = dyv * gamma_b
// Streaming form: a workgroup takes d.grain consecutive floats of ONE group
// (d.n workgroups per group), 16 bytes per access, every operand of a thread
// requested before the first is used.  Plain gradient buffers, H*W a multiple of 4.
__device__ __forceinline__ void step_gnb_apply_stream(const LDesc& d, int tile, int t) {
  const int tid = threadIdx.x, lane = tid & 63;
  const int C = UNI(d.C), G = UNI(d.G), HW = UNI(d.H) * UNI(d.W), grain = UNI(d.grain), tpg = UNI(d.n);
  const int cpg = UNI(fdiv(C, frcp(G))), gsz = cpg * HW;
  const int g = UNI(fdiv(tile, frcp(tpg))), k = tile - g * tpg;
  const int lo = k * grain, hi = (gsz < lo + grain) ? gsz : lo + grain;
  const size_t gbase = (size_t)g * gsz;
  const gfloat* st = at(d.st, t);
  const gfloat* x = at(d.x, t) + gbase;
  const gfloat* dy = at(d.dy, t) + gbase;
  gfloat* dx = at(d.dx, t) + gbase;
  const int flags = UNI(d.flags);
  const gfloat* skg = (flags & F_ADD_SKG) ? (const gfloat*)at(d.skg, t) + gbase : nullptr;
  const gfloat* part = GP(d.part);
  const float ihw = frcp(HW);
  // group sums of the per-channel partial sums (fixed order: lanes, then the wave
  // tree), taken while every lane is active
  float p1 = 0.f, p2 = 0.f;
  for (int j = lane; j < cpg; j += 64) { p1 += part[g * cpg + j]; p2 += part[C + g * cpg + j]; }
  const float mean = st[g], rstd = st[G + g];
  const float inv_n = 1.0f / (float)gsz;
  const float m1 = wave_sum(p1) * inv_n, m2 = wave_sum(p2) * inv_n;
  constexpr int U = 4;
  for (int base = lo + tid * 4; base < hi; base += U * 4 * BLK) {
    v4f xv[U], dv[U], sk[U];
    float sc[U], sh[U], gm[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int i = base + u * 4 * BLK;
      xv[u] = (v4f){0.f, 0.f, 0.f, 0.f}; dv[u] = xv[u]; sk[u] = xv[u];
      sc[u] = 0.f; sh[u] = 0.f; gm[u] = 0.f;
      if (i < hi) {
        const int c = g * cpg + fdiv(i, ihw);
        xv[u] = *(const gv4*)(x + i);
        dv[u] = *(const gv4*)(dy + i);
        if (skg) sk[u] = *(const gv4*)(skg + i);
        sc[u] = st[2 * G + c]; sh[u] = st[2 * G + C + c]; gm[u] = part[2 * C + c];
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int i = base + u * 4 * BLK;
      if (i < hi) {
        v4f r;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float yv = fmaf(sc[u], xv[u][e], sh[u]);
          float du = dv[u][e];
          if ((flags & F_GN_RELU) && !(yv > 0.f)) du = 0.f;
          const float xh = (xv[u][e] - mean) * rstd;
          r[e] = rbf_if(flags & F_BF16_OUT, rstd * (du * gm[u] - m1 - xh * m2) + sk[u][e]);
        }
        *(gv4*)(dx + i) = r;
      }
    }
  }
}

__device__ __forceinline__ void step_gnb_apply(const LDesc& d, int tile, int t) {
  if (UNI(d.grain) > 0) { step_gnb_apply_stream(d, tile, t); return; }
  const int HW = UNI(d.H) * UNI(d.W), cpg = UNI(fdiv(UNI(d.C), frcp(UNI(d.G)))), n = cpg * HW;
  const int o = tile * BLK + threadIdx.x;
  if (o >= d.C * HW) return;
  const int c = fdiv(o, frcp(HW)), i = o - c * HW, g = fdiv(c, frcp(cpg));
  const gfloat* st = at(d.st, t);
  const float mean = st[g], rstd = st[d.G + g], sc = st[2 * d.G + c], sh = st[2 * d.G + d.C + c];
  float S1 = 0.f, S2 = 0.f;
  for (int j0 = 0; j0 < cpg; j0 += 8) {           // 16 reads in flight per round trip
    float p1[8], p2[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      p1[u] = 0.f; p2[u] = 0.f;
      if (j0 + u < cpg) { p1[u] = GP(d.part)[g * cpg + j0 + u]; p2[u] = GP(d.part)[d.C + g * cpg + j0 + u]; }
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) { S1 += p1[u]; S2 += p2[u]; }
  }
  const gfloat* xc = at(d.x, t) + (size_t)c * HW;
  const float xv = xc[i];
  const float yv = fmaf(sc, xv, sh);
  float du = gn_du(d, at(d.dy, t), xc, sc, sh, c, i, HW);
  if ((d.flags & F_GN_RELU) && !(yv > 0.f)) du = 0.f;
  const float xh = (xv - mean) * rstd;
  const float inv_n = 1.0f / (float)n;
  float r = rstd * (du * GP(d.part)[2 * d.C + c] - S1 * inv_n - xh * (S2 * inv_n));
  if (d.flags & F_ADD_SKG) r += at(d.skg, t)[o];
  at(d.dx, t)[o] = rbf_if(d.flags & F_BF16_OUT, r);
}

// The same update for one parameter (GroupNorm scale or shift updated by the
// step that produced its gradient): w, v at index i in place, w_hat into the other copy.
// (the same with the parameter and its velocity already in registers)
__device__ __forceinline__ void update_loaded(const LDesc& d, int i, float g, float vv, float wv) {
  const float w_old = wv;
  vv = fmaf(UNIF(d.fm), vv, g);
  wv = fmaf(-UNIF(d.flr), fmaf(UNIF(d.fa), vv, UNIF(d.fb) * g), wv);
  GP((float*)d.b)[i] = vv;
  GP((float*)d.w)[i] = wv;
  if (d.what) GP(d.what)[i] = (UNI(d.flags) & F_LWP_W) ? fmaf(UNIF(d.flrT), wv - w_old, wv) : fmaf(-UNIF(d.flrT), vv, wv);
}

__device__ __forceinline__ void update_one(const LDesc& d, int i, float g) {
  float vv = GP(d.v)[i], wv = GP(d.w)[i];
  const float w_old = wv;
  vv = fmaf(UNIF(d.fm), vv, g);
  wv = fmaf(-UNIF(d.flr), fmaf(UNIF(d.fa), vv, UNIF(d.fb) * g), wv);
  GP((float*)d.b)[i] = vv;
  GP((float*)d.w)[i] = wv;
  if (d.what) GP(d.what)[i] = (UNI(d.flags) & F_LWP_W) ? fmaf(UNIF(d.flrT), wv - w_old, wv) : fmaf(-UNIF(d.flrT), vv, wv);
}

// Limit of the one-workgroup GroupNorm backward: elements of a group (they
// stay in registers together with their gradients).
constexpr int GNB_MAX_N = 4096;

// GroupNorm (+ReLU) backward of one group in one workgroup: the group and its
// incoming gradient are read once, in one burst, and stay in registers (thread
// holds the 4-element slots tid, tid + 256, ...; H*W is a multiple of 4, so a
// slot lies inside one channel).  Per-channel sums (dgamma, dbeta) go through
// per-slot partial sums in LDS, then the group sums, then dx.
// LDS: psum[n/4] | psum2[n/4] | cs[2*cpg] | cs2[3*cpg] | grp[2]
__device__ __forceinline__ void step_gn_bwd(const LDesc& d, int tile, int t, bool live, lfloat* smem, const bool nt) {
  const int tid = threadIdx.x;
  const int C = UNI(d.C), G = UNI(d.G), HW = UNI(d.H) * UNI(d.W), flags = UNI(d.flags);
  const int g = tile, cpg = UNI(fdiv(C, frcp(G))), n = cpg * HW, ns = n >> 2, HW4 = HW >> 2;
  if (!live) {
    // no gradient has reached this stage yet: carry scale and shift over to the other forward copy
    if ((flags & F_UPD_GN) && tid < cpg) { update_one(d, g * cpg + tid, 0.f); update_one(d, C + g * cpg + tid, 0.f); }
    return;
  }
  const bool rl = flags & F_GN_RELU, gapd = flags & F_DU_GAP, has_skg = flags & F_ADD_SKG;
  const float ihw4 = frcp(HW4);
  lfloat* psum = smem;
  lfloat* psum2 = psum + ns;
  lfloat* cs = psum2 + ns;            // sc, sh per channel of the group
  lfloat* cs2 = cs + 2 * cpg;         // gm*sb, gm*sg, gm per channel
  lfloat* grp = cs2 + 3 * cpg;
  const gfloat* st = at(d.st, t);
  const gfloat* xg = at(d.x, t) + (size_t)g * n;
  const gfloat* dy = at(d.dy, t);
  const bool has_dx = d.dx.base != nullptr;
  const gfloat* skg = (has_skg && has_dx) ? at(d.skg, t) + (size_t)g * n : nullptr;
  constexpr int GU = GNB_MAX_N / (4 * BLK);
  // ---- all reads
  v4f xr[GU], du[GU], sk[GU];
#pragma unroll
  for (int u = 0; u < GU; ++u) {
    xr[u] = (v4f){0.f, 0.f, 0.f, 0.f}; du[u] = xr[u]; sk[u] = xr[u];
    if (u * BLK < ns) {
      const int sl = tid + u * BLK;
      if (sl < ns) {
        xr[u] = *(const gv4*)(xg + 4 * sl);
        if (gapd) { const float v = dy[g * cpg + fdiv(sl, ihw4)]; du[u] = (v4f){v, v, v, v}; }
        else du[u] = *(const gv4*)(dy + (size_t)g * n + 4 * sl);
        if (skg) sk[u] = *(const gv4*)(skg + 4 * sl);
      }
    }
  }
  // Scale and shift of the group's channels are updated by lane 4c of channel c once their gradients are summed: their
  // master values and velocities are requested here, with the step's other reads, not after the sums (a memory round
  // trip in the middle of the step, with the whole workgroup waiting at the next barrier).
  const bool upd_pre = (flags & F_UPD_GN) && 4 * cpg <= BLK;
  float uv0 = 0.f, uw0 = 0.f, uv1 = 0.f, uw1 = 0.f;
  if (upd_pre && tid < 4 * cpg && (tid & 3) == 0) {
    const int i0 = g * cpg + (tid >> 2), i1 = C + i0;
    uv0 = GP(d.v)[i0]; uw0 = GP(d.w)[i0]; uv1 = GP(d.v)[i1]; uw1 = GP(d.w)[i1];
  }
  if (!nt && UNI(d.gparts) > 1 && !gapd) {
    // the gradient was left as partial sums by a backward-data GEMM split over its reduction
    // (the buffer read above holds nothing yet): add them up in order
    const int gparts = UNI(d.gparts);
    const size_t ps = (size_t)UNI(d.gpstride);
    for (int u = 0; u < GU; ++u) {
      const int sl = tid + u * BLK;
      if (sl < ns) {
        const gfloat* part = GP(d.gw) + (size_t)g * n + 4 * sl;
        du[u] = sum_parts<v4f, 2>((const gv4*)part, ps >> 2, gparts);
      }
    }
  }
  const float mean = st[g], rstd = st[G + g];
  float sc_c = 0.f, sh_c = 0.f, gm_c = 0.f;         // thread c < cpg holds its channel's constants
  if (tid < cpg) {
    sc_c = st[2 * G + g * cpg + tid]; sh_c = st[2 * G + C + g * cpg + tid]; gm_c = GP(d.gamma)[g * cpg + tid];
  }
  if (tid < cpg) { cs[tid] = sc_c; cs[cpg + tid] = sh_c; }
  __syncthreads();
  // ---- mask by the ReLU, per-slot partial sums of du*xh and du.  When a channel is a
  // whole number of rows of 16 slots (H*W a multiple of 64) the 16 lanes of a row add
  // their partial sums up across lanes first and LDS holds one pair per row.
  const bool rows16 = (HW4 & 15) == 0;
  const int per_c = rows16 ? HW4 >> 4 : HW4;          // partial sums per channel in LDS
#pragma unroll
  for (int u = 0; u < GU; ++u)
    if (u * BLK < ns) {
      const int sl = tid + u * BLK;
      float sg = 0.f, sb = 0.f;
      if (sl < ns) {
        const int c = fdiv(sl, ihw4);
        const float sc = cs[c], sh = cs[cpg + c];
        const float dpool = gapd ? du[u][0] / (float)HW : 0.f;   // gradient of every element under an average pool
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          float dv = gapd ? dpool : du[u][e];
          if (rl && !(fmaf(sc, xr[u][e], sh) > 0.f)) dv = 0.f;
          du[u][e] = dv;
          sg = fmaf(dv, (xr[u][e] - mean) * rstd, sg);
          sb += dv;
        }
      }
      if (rows16) {
        sg = row_sum(sg); sb = row_sum(sb);
        if (sl < ns && (tid & 15) == 0) { psum[sl >> 4] = sg; psum2[sl >> 4] = sb; }
      } else if (sl < ns) {
        psum[sl] = sg; psum2[sl] = sb;
      }
    }
  __syncthreads();
  for (int j = tid; j < 4 * cpg; j += BLK) {          // lanes 4c..4c+3 share channel c
    const int c = j >> 2, p = j & 3;
    float sg = 0.f, sb = 0.f;
    for (int i = p; i < per_c; i += 4) { sg += psum[c * per_c + i]; sb += psum2[c * per_c + i]; }
    sg += dpp_src<0xB1, 0xF>(sg); sb += dpp_src<0xB1, 0xF>(sb);
    sg += dpp_src<0x4E, 0xF>(sg); sb += dpp_src<0x4E, 0xF>(sb);
    if (p == 0) {
      GP(d.ggamma)[g * cpg + c] = sg; GP(d.gbeta)[g * cpg + c] = sb;
      cs2[c] = sb; cs2[cpg + c] = sg;
      if (upd_pre) { update_loaded(d, g * cpg + c, sg, uv0, uw0); update_loaded(d, C + g * cpg + c, sb, uv1, uw1); }
      else if (flags & F_UPD_GN) { update_one(d, g * cpg + c, sg); update_one(d, C + g * cpg + c, sb); }
    }
  }
  __syncthreads();
  if (tid < cpg) { cs2[tid] *= gm_c; cs2[cpg + tid] *= gm_c; cs2[2 * cpg + tid] = gm_c; }
  __syncthreads();
  if (!has_dx) return;
  if (tid < 64) {
    float s1 = 0.f, s2 = 0.f;
    for (int c = tid; c < cpg; c += 64) { s1 += cs2[c]; s2 += cs2[cpg + c]; }
    s1 = wave_sum(s1); s2 = wave_sum(s2);
    if (tid == 0) { grp[0] = s1 / (float)n; grp[1] = s2 / (float)n; }
  }
  __syncthreads();
  const float m1 = grp[0], m2 = grp[1];
  gfloat* dx = at(d.dx, t) + (size_t)g * n;
#pragma unroll
  for (int u = 0; u < GU; ++u)
    if (u * BLK < ns) {
      const int sl = tid + u * BLK;
      if (sl < ns) {
        const float gm = cs2[2 * cpg + fdiv(sl, ihw4)];
        v4f o;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float xh = (xr[u][e] - mean) * rstd;
          o[e] = rbf_if(flags & F_BF16_OUT, rstd * (du[u][e] * gm - m1 - xh * m2) + sk[u][e]);
        }
        PB_ST(nt, (gv4*)(dx + 4 * sl), o);
      }
    }
}

// Backward data: dX = W^T dZ (transposed convolution), one thread per input
// element, gathering.
__device__ __forceinline__ void step_conv_bwd_x(const LDesc& d, int tile, int t) {
  const int HW = d.H * d.W, P = d.OH * d.OW, kk = d.k * d.k;
  const int o = tile * BLK + threadIdx.x;
  if (o >= d.C * HW) return;
  const int ci = o / HW, r = o - ci * HW, ih = r / d.W, iw = r - ih * d.W;
  const gfloat* dz = at(d.dy, t);
  float acc = 0.f;
  for (int kh = 0; kh < d.k; ++kh) {
    const int th = ih + d.pad - kh;
    if (th < 0 || th % d.stride) continue;
    const int oh = th / d.stride;
    if (oh >= d.OH) continue;
    for (int kw = 0; kw < d.k; ++kw) {
      const int tw = iw + d.pad - kw;
      if (tw < 0 || tw % d.stride) continue;
      const int ow = tw / d.stride;
      if (ow >= d.OW) continue;
      const gfloat* wq = GP(d.w) + (size_t)ci * kk + kh * d.k + kw;
      const gfloat* dq = dz + oh * d.OW + ow;
      for (int co = 0; co < d.K; ++co) acc = fmaf(wq[(size_t)co * d.C * kk], dq[(size_t)co * P], acc);
    }
  }
  if (d.flags & F_MASK_X) { if (!(at(d.x, t)[o] > 0.f)) acc = 0.f; }
  if (d.flags & F_ADD_SKG) acc += at(d.skg, t)[o];
  at(d.dx, t)[o] = acc;
}

// Backward weights: dW[co,ci,kh,kw] = sum_p dZ[co,p] * a[ci, p*s-pad+k],
// a = the forward's transformed input recomputed from the saved input.
// Large maps: one wavefront per weight element; small maps: one thread.
__device__ __forceinline__ void step_conv_bwd_w(const LDesc& d, int tile, int t) {
  const int HW = d.H * d.W, P = d.OH * d.OW, kk = d.k * d.k;
  const int nW = d.K * d.C * kk;
  const bool wave_mode = P > 16;
  const int per_tile = wave_mode ? BLK / 64 : BLK;
  const int w_tiles = (nW + per_tile - 1) / per_tile;
  const gfloat* dz = at(d.dy, t);
  if (tile >= w_tiles) {                      // bias tiles
    const int lane = threadIdx.x & 63;
    if (wave_mode) {
      const int co = (tile - w_tiles) * per_tile + (threadIdx.x >> 6);
      if (co >= d.K) return;
      float s = 0.f;
      for (int p = lane; p < P; p += 64) s += dz[(size_t)co * P + p];
      s = wave_sum(s);
      if (lane == 0) GP(d.gb)[co] = s;
    } else {
      const int co = (tile - w_tiles) * per_tile + threadIdx.x;
      if (co >= d.K) return;
      float s = 0.f;
      for (int p = 0; p < P; ++p) s += dz[(size_t)co * P + p];
      GP(d.gb)[co] = s;
    }
    return;
  }
  const gfloat* x = at(d.x, t);
  const bool aff = d.flags & F_PRE_AFFINE, rl = d.flags & F_PRE_RELU;
  const gfloat* st = aff ? at(d.st, t) : nullptr;
  const int e = wave_mode ? tile * per_tile + (threadIdx.x >> 6) : tile * per_tile + threadIdx.x;
  if (e >= nW) return;
  const int co = e / (d.C * kk), r = e - co * d.C * kk, ci = r / kk, q = r - ci * kk;
  const int kh = q / d.k, kw = q - kh * d.k;
  const float sc = aff ? st[2 * d.G + ci] : 1.f, sh = aff ? st[2 * d.G + d.C + ci] : 0.f;
  const gfloat* xc = x + (size_t)ci * HW;
  const gfloat* dzc = dz + (size_t)co * P;
  float acc = 0.f;
  const int p0 = wave_mode ? (threadIdx.x & 63) : 0, dp = wave_mode ? 64 : 1;
  for (int p = p0; p < P; p += dp) {
    const int oh = p / d.OW, ow = p - oh * d.OW;
    const int ih = oh * d.stride - d.pad + kh, iw = ow * d.stride - d.pad + kw;
    if (ih < 0 || ih >= d.H || iw < 0 || iw >= d.W) continue;
    float v = xc[ih * d.W + iw];
    if (aff) v = fmaf(sc, v, sh);
    if (rl) v = fmaxf(v, 0.f);
    acc = fmaf(dzc[p], v, acc);
  }
  if (wave_mode) {
    acc = wave_sum(acc);
    if ((threadIdx.x & 63) == 0) GP(d.gw)[e] = acc;
  } else {
    GP(d.gw)[e] = acc;
  }
}

__device__ __forceinline__ void step_copy(const LDesc& d, int tile, int t, const bool nt) {
  const int grain = UNI(d.grain), n = UNI(d.n);
  if (grain > 0) {   // streaming form: grain floats per workgroup, 16 bytes per access (n a multiple of 4)
    const gfloat* src = at(d.dy, t);
    gfloat* dst = at(d.dx, t);
    const int lo = tile * grain, hi = (n < lo + grain) ? n : lo + grain;
    constexpr int U = 4;
    for (int base = lo + (int)threadIdx.x * 4; base < hi; base += U * 4 * BLK) {
      v4f v[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int i = base + u * 4 * BLK;
        v[u] = (v4f){0.f, 0.f, 0.f, 0.f};
        if (i < hi) v[u] = *(const gv4*)(src + i);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int i = base + u * 4 * BLK;
        if (i < hi) PB_ST(nt, (gv4*)(dst + i), v[u]);
      }
    }
    return;
  }
  const int o = tile * BLK + threadIdx.x;
  if (o < n) at(d.dx, t)[o] = at(d.dy, t)[o];
}


// The tick's sample into the first stage's input ring, its label into the
// label ring.  src != nullptr: handed over by the host call; otherwise pool
// item (idx_base + k) mod n_pool.
__device__ __forceinline__ void step_ingest(const LDesc& d, int tile, int t, const Globals* __restrict__ G, int k,
                            const float* src_override, int label_override) {
  const gfloat* src = (const gfloat*)src_override;
  int lab = label_override;
  if (!src_override) {
    const int item = (int)(((int64_t)G->idx_base + k) % G->n_pool);
    src = (const gfloat*)G->pool + (size_t)item * d.n;
    lab = ((const gint*)G->pool_labels)[item];
  }
  gfloat* dst = at(d.dx, t);
  constexpr int U = 4;   // elements per thread
  const int i0 = tile * U * BLK + threadIdx.x;
  float v[U];
#pragma unroll
  for (int u = 0; u < U; ++u) v[u] = (i0 + u * BLK < d.n) ? src[i0 + u * BLK] : 0.f;
#pragma unroll
  for (int u = 0; u < U; ++u)
    if (i0 + u * BLK < d.n) dst[i0 + u * BLK] = rbf_if(d.flags & F_BF16_OUT, v[u]);
  if (i0 == 0) ((gint*)d.labels)[t % d.n_stages] = lab;
}

// Fused Spike-Compensated momentum update with Linear Weight Prediction of one
// tile of a stage: v' = m v + g; w' = w - lr (a v' + b g);
// w_hat' = w' - lr T v'.  The predicted weights are double-buffered by tick
// parity: the tick's forward passes read one copy while the update writes the
// other (d.what), so the update may run beside forward work of the same tick
// as soon as the stage's gradients are complete.  Master weights and velocity
// (read d.w, d.v; written d.wp, d.b) are updated in place.
// Update size N above one (the paper's setting is one; this path is not tuned): the gradients of N
// consecutive samples are added up in d.gacc and one update with their mean is applied after the
// backward pass of the last of them.  On every other tick the parameters stand still and the
// predicted weights are carried over from the slot of this tick to the slot of the next one.
// Two vectors per thread at a time: the step shares its kernel with steps that need every register.
__device__ __forceinline__ void step_update_acc(const LDesc& d, int tile, int t) {
  const int N = UNI(d.upd_n);
  const int n4 = UNI(d.n) >> 2;
  const int j = t - UNI(d.upd_t0);                      // sample whose gradient arrived in this tick
  const int pos = j >= 0 ? j % N : -1;
  const float a = UNIF(d.fa), b = UNIF(d.fb), lrT = UNIF(d.flrT), lr = UNIF(d.flr), m = UNIF(d.fm);
  const bool wform = UNI(d.flags) & F_LWP_W;
  const int gparts = UNI(d.gparts), ps4 = UNI(d.gpstride) >> 2;
  const gv4* gp = (const gv4*)d.gw;
  gv4* ap = (gv4*)d.gacc;
  gv4* vp = (gv4*)d.v;
  gv4* wp = (gv4*)(float*)d.w;
  gv4* ho = (gv4*)d.what;
  const gv4* hs = (const gv4*)(d.what0 + (size_t)(t % UNI(d.pdepth)) * (size_t)UNI(d.pstride));
  const float inv = 1.0f / (float)N;
  const int lo = tile * (UPD_TILE / 4), hi = (n4 < lo + UPD_TILE / 4) ? n4 : lo + UPD_TILE / 4;
#pragma unroll 2
  for (int i = lo + (int)threadIdx.x; i < hi; i += BLK) {
    if (pos < 0) { if (ho) ho[i] = hs[i]; continue; }
    v4f g = gp[i];
    for (int p = 1; p < gparts; ++p) g += gp[(size_t)p * ps4 + i];
    if (pos > 0) g += ap[i];
    if (pos != N - 1) {
      ap[i] = g;
      if (ho) ho[i] = hs[i];
      continue;
    }
    const v4f v0 = vp[i], w0 = wp[i];
    v4f v2, w2, h;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float ge = g[e] * inv;
      v2[e] = fmaf(m, v0[e], ge);
      w2[e] = fmaf(-lr, fmaf(a, v2[e], b * ge), w0[e]);
      h[e] = wform ? fmaf(lrT, w2[e] - w0[e], w2[e]) : fmaf(-lrT, v2[e], w2[e]);
    }
    vp[i] = v2;
    wp[i] = w2;
    if (ho) ho[i] = h;
  }
}

// Weight gradient of a 3x3 convolution (stride 1, padding 1) on an S x S map, S = 2 or 4, for the
// parameters [p0, p0 + cnt) of the layer's weight tensor [K][C][3][3], written to LDS (gl[idx - p0]).
// g[k][c][kh][kw] = sum_{oh,ow} dz[k][oh][ow] * x[c][oh-1+kh][ow-1+kw]: with at most 16 pixels this is an
// outer product, not a contraction -- 2.4 M outputs of 4-11 multiply-adds each for a 512x512 layer --,
// so it is not worth a GEMM step of its own, and not worth 8 bytes per parameter of memory traffic
// (gradient written, then read by the update): the update step that streams the parameters anyway
// computes it on the fly.  A thread takes (k, c) pairs: the pair's two maps sit in registers (read from
// LDS with 16-byte loads) and its nine sums are fully unrolled.
// xs: the layer's input [C][S*S]; dzs: the rows k_lo.. of the output gradient [rows][S*S].
template <int S>
__device__ __forceinline__ void wgrad_small_map(const lfloat* xs, const lfloat* dzs, lfloat* gl, int C, int k_lo, int p0, int cnt) {
  constexpr int HW = S * S;
  const int pc0 = p0 / 9, pc1 = (p0 + cnt - 1) / 9;        // (k, c) pairs, flattened, that the range touches
  const float iC = frcp(C);
  for (int pc = pc0 + (int)threadIdx.x; pc <= pc1; pc += BLK) {
    const int rel = pc - k_lo * C;                          // < 8 * C: small enough for the reciprocal division
    const int kr = fdiv(rel, iC), c = rel - kr * C;
    float xv[HW], dv[HW];
#pragma unroll
    for (int q = 0; q < HW / 4; ++q) {
      const v4f a = *(const lv4*)(xs + c * HW + 4 * q), b = *(const lv4*)(dzs + kr * HW + 4 * q);
#pragma unroll
      for (int e = 0; e < 4; ++e) { xv[4 * q + e] = a[e]; dv[4 * q + e] = b[e]; }
    }
    const int base = pc * 9 - p0;
#pragma unroll
    for (int kh = 0; kh < 3; ++kh)
#pragma unroll
      for (int kw = 0; kw < 3; ++kw) {
        float acc = 0.f;
#pragma unroll
        for (int oh = 0; oh < S; ++oh)
#pragma unroll
          for (int ow = 0; ow < S; ++ow) {
            const int ih = oh - 1 + kh, iw = ow - 1 + kw;   // compile-time after unrolling
            if (ih >= 0 && ih < S && iw >= 0 && iw < S) acc = fmaf(dv[oh * S + ow], xv[ih * S + iw], acc);
          }
        const int o = base + kh * 3 + kw;
        if (o >= 0 && o < cnt) gl[o] = acc;
      }
  }
}

__device__ __forceinline__ void step_update(const LDesc& d, int tile, int t, lfloat* smem, const bool nt_kernel) {
  if (UNI(d.upd_n) > 1) { step_update_acc(d, tile, t); return; }
  // the step streams 24 bytes per parameter and nothing else: what it needs is bytes in
  // flight, so every thread requests its 8 vectors of all three arrays before using any.
  // Plain accesses: the parameter arrays of the VGG-11 and wide configurations fit the
  // Infinity Cache, and non-temporal hints (which pay on arrays beyond it) cost 2 % there
  constexpr int UU = UPD_TILE / (4 * BLK);
  const int n4 = UNI(d.n) >> 2;
  const int i0 = tile * (UPD_TILE / 4) + threadIdx.x;
  const float a = UNIF(d.fa), b = UNIF(d.fb), lrT = UNIF(d.flrT), lr = UNIF(d.flr), m = UNIF(d.fm);
  const bool wform = UNI(d.flags) & F_LWP_W, nt = nt_kernel && (UNI(d.flags) & F_NT);
  const gv4* gp = (const gv4*)d.gw;
  const gv4* vp = (const gv4*)d.v;
  const gv4* wp = (const gv4*)d.w;
  v4f gv[UU], vv[UU], wv[UU];
  // (nt kernels serve the networks tiled for latency, which have no layer this pays for)
  const bool fused = !nt_kernel && (UNI(d.flags) & F_WGRAD);
  const int nwg4 = fused ? (UNI(d.K) * UNI(d.C) * 9) >> 2 : 0;     // vectors of the weight tensor: gradient computed here
#pragma unroll
  for (int u = 0; u < UU; ++u) {
    const int i = i0 + u * BLK;
    if (i < n4) {
      if (i >= nwg4) gv[u] = gp[i];
      vv[u] = vp[i]; wv[u] = wp[i];
    }
  }
  if (fused && tile * (UPD_TILE / 4) < nwg4) {
    // the layer's input and the rows of dz this tile's parameters belong to, into LDS; then the tile's
    // gradient in two halves of 4096 parameters (LDS: xs[C*S*S] | dzs[8*S*S] | gl[4096])
    const int C = UNI(d.C), K = UNI(d.K), S = UNI(d.H), HW = S * S, CKK = C * 9;
    const int p_lo = tile * UPD_TILE, k_lo = p_lo / CKK;
    lfloat* xs = smem;
    lfloat* dzs = xs + C * HW;
    lfloat* gl = dzs + 8 * 16;
    const gfloat* xg = at(d.x, t);
    const gfloat* dzg = at(d.dy, t) + (size_t)k_lo * HW;
    for (int i = threadIdx.x * 4; i < C * HW; i += 4 * BLK) *(lv4*)(xs + i) = *(const gv4*)(xg + i);
    const int rows = (K - k_lo < 8) ? K - k_lo : 8;
    if ((int)threadIdx.x * 4 < rows * HW) *(lv4*)(dzs + threadIdx.x * 4) = *(const gv4*)(dzg + threadIdx.x * 4);
    const int n_w = nwg4 << 2;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int p0 = p_lo + h * (UPD_TILE / 2);
      int cnt = n_w - p0;
      if (cnt > UPD_TILE / 2) cnt = UPD_TILE / 2;
      __syncthreads();                 // operands staged (h = 0) / previous half consumed (h = 1)
      if (cnt > 0) {
        if (S == 4) wgrad_small_map<4>(xs, dzs, gl, C, k_lo, p0, cnt);
        else wgrad_small_map<2>(xs, dzs, gl, C, k_lo, p0, cnt);
      }
      __syncthreads();
#pragma unroll
      for (int u = 0; u < UU / 2; ++u) {
        const int uu = h * (UU / 2) + u;
        const int i = i0 + uu * BLK;
        if (i < nwg4) gv[uu] = *(const lv4*)(gl + 4 * ((int)threadIdx.x + u * BLK));
      }
    }
  }
  // a stage whose weight gradient was computed in parts (split reduction of the
  // backward-weights GEMM): add the other parts, in order
  const int gparts = UNI(d.gparts);
  if (gparts > 1) {
    const int ps4 = UNI(d.gpstride) >> 2;
    for (int p = 1; p < gparts; ++p) {
      v4f pv[UU];
#pragma unroll
      for (int u = 0; u < UU; ++u) {
        const int i = i0 + u * BLK;
        pv[u] = (v4f){0.f, 0.f, 0.f, 0.f};
        if (i < n4) pv[u] = gp[(size_t)p * ps4 + i];
      }
#pragma unroll
      for (int u = 0; u < UU; ++u)
        if (i0 + u * BLK < n4) gv[u] += pv[u];
    }
  }
  gv4* vo = (gv4*)(float*)d.b;
  gv4* wo = (gv4*)(float*)d.wp;
  gv4* ho = (gv4*)d.what;
#pragma unroll
  for (int u = 0; u < UU; ++u) {
    const int i = i0 + u * BLK;
    if (i < n4) {
      v4f v2, w2;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        v2[e] = fmaf(m, vv[u][e], gv[u][e]);
        w2[e] = fmaf(-lr, fmaf(a, v2[e], b * gv[u][e]), wv[u][e]);
      }
      PB_ST(nt, vo + i, v2);
      PB_ST(nt, wo + i, w2);
      if (ho) {
        v4f p;
#pragma unroll
        for (int e = 0; e < 4; ++e) p[e] = wform ? fmaf(lrT, w2[e] - wv[u][e], w2[e]) : fmaf(-lrT, v2[e], w2[e]);
        PB_ST(nt, ho + i, p);
      }
    }
  }
}

// ---- 3x3 layers on 2x2 and 4x4 maps (the 512-channel layers of VGG-11): matrix-vector products.
// With 4 or 16 output pixels a 16-row MFMA tile is mostly padding and what matters is that the 9.4 MB of
// weights go by once, in few workgroups.  A thread works on (output channel, input channel) pairs: the
// pair's nine weights (36 contiguous bytes; consecutive lanes take consecutive input channels, so a
// wavefront reads 2304 contiguous bytes) against the pair's two S x S maps, all index arithmetic of the
// nine taps resolved at compile time.
template <int S>
__device__ __forceinline__ void corr_fwd(float (&acc)[S * S], const float (&w)[9], const float (&x)[S * S]) {
#pragma unroll
  for (int oh = 0; oh < S; ++oh)
#pragma unroll
    for (int ow = 0; ow < S; ++ow)
#pragma unroll
      for (int kh = 0; kh < 3; ++kh)
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) {
          const int ih = oh - 1 + kh, iw = ow - 1 + kw;
          if (ih >= 0 && ih < S && iw >= 0 && iw < S) acc[oh * S + ow] = fmaf(w[kh * 3 + kw], x[ih * S + iw], acc[oh * S + ow]);
        }
}
// dx[ih][iw] += sum_taps w[kh][kw] * dz[ih+1-kh][iw+1-kw]
template <int S>
__device__ __forceinline__ void corr_bwd(float (&acc)[S * S], const float (&w)[9], const float (&dz)[S * S]) {
#pragma unroll
  for (int ih = 0; ih < S; ++ih)
#pragma unroll
    for (int iw = 0; iw < S; ++iw)
#pragma unroll
      for (int kh = 0; kh < 3; ++kh)
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) {
          const int oh = ih + 1 - kh, ow = iw + 1 - kw;
          if (oh >= 0 && oh < S && ow >= 0 && ow < S) acc[ih * S + iw] = fmaf(w[kh * 3 + kw], dz[oh * S + ow], acc[ih * S + iw]);
        }
}

// Forward: workgroup `tile` computes output channels tile*R .. tile*R+R-1 (R = d.n).  Thread tid takes input
// channels tid, tid+256, ...; per channel it holds the channel's map in registers and runs through the R rows,
// RB rows of weights in flight at a time.  The R*S*S sums are then added up across the workgroup (lanes by DPP,
// wavefronts through LDS, fixed order).
template <int S, int R>
__device__ __forceinline__ void step_dot_fwd_t(const LDesc& d, int tile, int t, lfloat* smem) {
  constexpr int HW = S * S;
  const int tid = threadIdx.x, lane = tid & 63, wv = UNI(tid >> 6);
  const int C = UNI(d.C), k0 = tile * R;
  const gfloat* x = at(d.x, t);
  const gfloat* w = GP(d.w) + (size_t)k0 * C * 9;
  float acc[R][HW];
#pragma unroll
  for (int r = 0; r < R; ++r)
#pragma unroll
    for (int i = 0; i < HW; ++i) acc[r][i] = 0.f;
  for (int c = tid; c < C; c += BLK) {
    float xv[HW];
#pragma unroll
    for (int q = 0; q < HW / 4; ++q) {
      const v4f a = *(const gv4*)(x + c * HW + 4 * q);
#pragma unroll
      for (int e = 0; e < 4; ++e) xv[4 * q + e] = a[e];
    }
    float wr[R][9];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int j = 0; j < 9; ++j) wr[r][j] = w[((size_t)r * C + c) * 9 + j];
#pragma unroll
    for (int r = 0; r < R; ++r) corr_fwd<S>(acc[r], wr[r], xv);
  }
  lfloat* red = smem;   // [4 wavefronts][R*HW]
#pragma unroll
  for (int r = 0; r < R; ++r)
#pragma unroll
    for (int i = 0; i < HW; ++i) {
      const float sv = wave_sum(acc[r][i]);
      if (lane == 0) red[wv * (R * HW) + r * HW + i] = sv;
    }
  __syncthreads();
  if (tid < R * HW) {
    const float sv = (red[tid] + red[R * HW + tid]) + (red[2 * R * HW + tid] + red[3 * R * HW + tid]);
    at(d.y, t)[(size_t)k0 * HW + tid] = sv;
  }
}

// Backward data: workgroup (cb, part) = (tile / parts, tile % parts) computes, for input channels cb*64 ..
// cb*64+63, the sum over the part's output channels; wavefront wv takes every fourth of them.  dz of the
// part sits in LDS.  The four wavefronts' sums are added through LDS in fixed order and written to the
// gradient buffer (one part) or to the part's own copy, which the consumer of the gradient adds up.
template <int S>
__device__ __forceinline__ void step_dot_bwd_t(const LDesc& d, int tile, int t, lfloat* smem) {
  constexpr int HW = S * S;
  const int tid = threadIdx.x, lane = tid & 63, wv = UNI(tid >> 6);
  const int C = UNI(d.C), K = UNI(d.K), parts = UNI(d.gparts) > 1 ? UNI(d.gparts) : 1;
  const int cb = UNI(fdiv(tile, frcp(parts))), part = tile - cb * parts;
  const int kn = UNI(d.n), kbeg = part * kn, kcnt = (K - kbeg < kn) ? K - kbeg : kn;
  const int c = cb * 64 + lane;
  lfloat* dzs = smem;                     // [kn][HW]
  lfloat* red = smem + kn * HW;           // [4][64][HW]
  const gfloat* dz = at(d.dy, t) + (size_t)kbeg * HW;
  for (int i = tid * 4; i < kcnt * HW; i += 4 * BLK) *(lv4*)(dzs + i) = *(const gv4*)(dz + i);
  __syncthreads();
  float acc[HW];
#pragma unroll
  for (int i = 0; i < HW; ++i) acc[i] = 0.f;
  const gfloat* w = GP(d.w) + ((size_t)kbeg * C + c) * 9;
  constexpr int KB = 4;                   // output channels whose weights are in flight together
  for (int kk0 = wv; kk0 < kcnt; kk0 += 4 * KB) {
    float wr[KB][9];
#pragma unroll
    for (int b = 0; b < KB; ++b) {
      const int kk = kk0 + 4 * b;
#pragma unroll
      for (int j = 0; j < 9; ++j) wr[b][j] = (kk < kcnt && c < C) ? w[(size_t)kk * C * 9 + j] : 0.f;
    }
#pragma unroll
    for (int b = 0; b < KB; ++b) {
      const int kk = kk0 + 4 * b;
      if (kk < kcnt) {
        float dv[HW];
#pragma unroll
        for (int q = 0; q < HW / 4; ++q) {
          const v4f a = *(const lv4*)(dzs + kk * HW + 4 * q);
#pragma unroll
          for (int e = 0; e < 4; ++e) dv[4 * q + e] = a[e];
        }
        corr_bwd<S>(acc, wr[b], dv);
      }
    }
  }
#pragma unroll
  for (int q = 0; q < HW / 4; ++q)
    *(lv4*)(red + (wv * 64 + lane) * HW + 4 * q) = (v4f){acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]};
  __syncthreads();
  if (wv == 0 && c < C) {
    gfloat* out = (parts > 1) ? GP(d.gw) + (size_t)part * (size_t)UNI(d.gpstride) : at(d.dx, t);
#pragma unroll
    for (int q = 0; q < HW / 4; ++q) {
      v4f a = *(const lv4*)(red + lane * HW + 4 * q);
#pragma unroll
      for (int w2 = 1; w2 < 4; ++w2) a += *(const lv4*)(red + (w2 * 64 + lane) * HW + 4 * q);
      *(gv4*)(out + (size_t)c * HW + 4 * q) = a;
    }
  }
}

__device__ __forceinline__ void step_dot_fwd(const LDesc& d, int tile, int t, lfloat* smem) {
  if (UNI(d.H) == 4) step_dot_fwd_t<4, 4>(d, tile, t, smem);
  else step_dot_fwd_t<2, 8>(d, tile, t, smem);
}
__device__ __forceinline__ void step_dot_bwd_x(const LDesc& d, int tile, int t, lfloat* smem) {
  if (UNI(d.H) == 4) step_dot_bwd_t<4>(d, tile, t, smem);
  else step_dot_bwd_t<2>(d, tile, t, smem);
}

// ---- Dense layer on one sample (a matrix-vector product): the weight matrix is streamed once, with 16-byte
// loads; C (inputs) is a multiple of 4, the operands are 16-byte aligned.
// Forward, y[k] = b[k] + sum_c w[k][c] x[c]: a wavefront per output k.
__device__ __forceinline__ void step_fc_fwd(const LDesc& d, int tile, int t) {
  const int lane = threadIdx.x & 63, k = tile * (BLK / 64) + UNI((int)(threadIdx.x >> 6));
  const int C = UNI(d.C);
  if (k >= UNI(d.K)) return;
  const gfloat* x = at(d.x, t);
  const gfloat* w = GP(d.w) + (size_t)k * C;
  float s0 = 0.f, s1 = 0.f;
  int c = 4 * lane;
  for (; c + 256 < C; c += 512) {
    const v4f a0 = *(const gv4*)(w + c), b0 = *(const gv4*)(x + c);
    const v4f a1 = *(const gv4*)(w + c + 256), b1 = *(const gv4*)(x + c + 256);
    s0 = fmaf(a0[3], b0[3], fmaf(a0[2], b0[2], fmaf(a0[1], b0[1], fmaf(a0[0], b0[0], s0))));
    s1 = fmaf(a1[3], b1[3], fmaf(a1[2], b1[2], fmaf(a1[1], b1[1], fmaf(a1[0], b1[0], s1))));
  }
  if (c < C) {
    const v4f a0 = *(const gv4*)(w + c), b0 = *(const gv4*)(x + c);
    s0 = fmaf(a0[3], b0[3], fmaf(a0[2], b0[2], fmaf(a0[1], b0[1], fmaf(a0[0], b0[0], s0))));
  }
  const float s = wave_sum(s0 + s1);
  if (lane == 0) {
    const float v = s + ((UNI(d.flags) & F_BIAS) ? GP(d.b)[k] : 0.f);
    at(d.y, t)[k] = rbf_if(UNI(d.flags) & F_BF16_OUT, v);
  }
}

// Backward data, dx[c] = sum_k w[k][c] dy[k]: a workgroup takes 64 inputs c (16 lanes x 4) and deals the outputs
// k out to its 16 groups of 16 lanes, group g taking k = g, g + 16, ...; the 16 partial sums of an input are
// added in the order of the groups.  LDS: dy[K] | part[16][64].
__device__ __forceinline__ void step_fc_bwd_x(const LDesc& d, int tile, int t, lfloat* smem) {
  const int tid = threadIdx.x, l = tid & 15, g = tid >> 4;
  const int C = UNI(d.C), K = UNI(d.K);
  const int Kp = (K + 3) & ~3;
  lfloat* dyl = smem;
  lfloat* part = smem + Kp;
  const gfloat* dy = at(d.dy, t);
  for (int i = tid; i < K; i += BLK) dyl[i] = dy[i];
  __syncthreads();
  const int c = tile * 64 + 4 * l;
  v4f acc = (v4f){0.f, 0.f, 0.f, 0.f};
  if (c < C) {
    const gfloat* w = GP(d.w) + c;
    int k = g;
    for (; k + 48 < K; k += 64) {
      const v4f a0 = *(const gv4*)(w + (size_t)k * C), a1 = *(const gv4*)(w + (size_t)(k + 16) * C);
      const v4f a2 = *(const gv4*)(w + (size_t)(k + 32) * C), a3 = *(const gv4*)(w + (size_t)(k + 48) * C);
      const float e0 = dyl[k], e1 = dyl[k + 16], e2 = dyl[k + 32], e3 = dyl[k + 48];
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[j] = fmaf(a3[j], e3, fmaf(a2[j], e2, fmaf(a1[j], e1, fmaf(a0[j], e0, acc[j]))));
    }
    for (; k < K; k += 16) {
      const v4f a0 = *(const gv4*)(w + (size_t)k * C);
      const float e0 = dyl[k];
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[j] = fmaf(a0[j], e0, acc[j]);
    }
  }
  *(lv4*)(part + g * 64 + 4 * l) = acc;
  __syncthreads();
  if (tid < 64 && tile * 64 + tid < C) {
    float s = 0.f;
#pragma unroll
    for (int q = 0; q < 16; ++q) s += part[q * 64 + tid];
    at(d.dx, t)[tile * 64 + tid] = rbf_if(UNI(d.flags) & F_BF16_OUT, s);
  }
}

// Backward weights, gW[k][c] = dy[k] x[c] (an outer product): 4096 consecutive weights per workgroup.
__device__ __forceinline__ void step_fc_bwd_w(const LDesc& d, int tile, int t) {
  const int C = UNI(d.C);
  const int64_t n = (int64_t)UNI(d.K) * C;
  const gfloat* x = at(d.x, t);
  const gfloat* dy = at(d.dy, t);
  gfloat* gw = GP(d.gw);
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int e = tile * 4096 + j * 1024 + 4 * (int)threadIdx.x;
    if (e < n) {
      const int k = e / C, c = e - k * C;
      const v4f xv = *(const gv4*)(x + c);
      const float s = dy[k];
      *(gv4*)(gw + e) = (v4f){s * xv[0], s * xv[1], s * xv[2], s * xv[3]};
    }
  }
}

// Limits of the fused last stage (checked on the host): its input, the vector
// the linear layer sees and the logits live in LDS / registers of one workgroup.
constexpr int HEAD_MAX_IN = 8192;   // C*H*W
constexpr int HEAD_MAX_CV = 512;    // inputs of the linear layer
constexpr int HEAD_MAX_K = 16;      // classes

// Last stage of the form GroupNorm -> ReLU -> global average pool -> linear ->
// cross-entropy with H*W a multiple of 4: the input stays in registers (thread
// holds the 4-element slots tid, tid + 256, ...; a slot lies inside one
// channel) and every reduction over a group or a channel goes through one
// array of per-slot partial sums in LDS.
// LDS: psum[n/4] | psum2[n/4] | vec[512] | dvec[512] | logit[16] | ebuf[16] | chan[9*C] | grp[2*G]
template <int XU>   // 16-byte vectors of the input a thread keeps: 8 (up to 8192 inputs) or 16
__device__ __forceinline__ void step_head_gap4(const LDesc& d, int t, lfloat* smem, const bool nt) {
  const int tid = threadIdx.x, lane = tid & 63, wv = UNI(tid >> 6);
  const int C = UNI(d.C), HW = UNI(d.H) * UNI(d.W), K = UNI(d.K), G = UNI(d.G), flags = UNI(d.flags);
  const bool rl = flags & F_PRE_RELU, has_b = flags & F_BIAS;
  const int n_in = C * HW, nslot = n_in >> 2, HW4 = HW >> 2;
  const int cpg = UNI(fdiv(C, frcp(G))), n = cpg * HW, ns = n >> 2;      // per group: channels, elements, slots
  const float ihw4 = frcp(HW4), ins = frcp(ns);
  lfloat* psum = smem;
  lfloat* psum2 = psum + nslot;
  lfloat* vec = psum2 + nslot;
  lfloat* dvec = vec + HEAD_MAX_CV;
  lfloat* logit = dvec + HEAD_MAX_CV;
  lfloat* ebuf = logit + HEAD_MAX_K;
  lfloat* chan = ebuf + HEAD_MAX_K;                // sc, sh, mean, rstd, gamma_f, beta_f, gamma_b, gm*sb, gm*sg
  lfloat* grp = chan + 9 * C;
  const gfloat* x = at(d.x, t);
  // ---- all global reads in one burst
  v4f xr[XU];
#pragma unroll
  for (int u = 0; u < XU; ++u) {
    xr[u] = (v4f){0.f, 0.f, 0.f, 0.f};
    if (u * BLK < nslot) {
      const int sl = tid + u * BLK;
      if (sl < nslot) xr[u] = *(const gv4*)(x + 4 * sl);
    }
  }
  constexpr int KU = HEAD_MAX_K / 4, IU = HEAD_MAX_CV / 64, JU = HEAD_MAX_CV / BLK;
  float wf[KU][IU];      // forward weights: wave wv holds rows wv, wv + 4, ...
#pragma unroll
  for (int ku = 0; ku < KU; ++ku)
#pragma unroll
    for (int iu = 0; iu < IU; ++iu) {
      const int k = wv + 4 * ku, i = lane + 64 * iu;
      wf[ku][iu] = 0.f;
      if (4 * ku < K && 64 * iu < C) {
        if (k < K && i < C) wf[ku][iu] = GP(d.w)[k * C + i];
      }
    }
  float wb[JU][HEAD_MAX_K];   // backward (current) weights: thread holds columns tid, tid + 256
#pragma unroll
  for (int ju = 0; ju < JU; ++ju)
#pragma unroll
    for (int k = 0; k < HEAD_MAX_K; ++k) {
      const int i = tid + ju * BLK;
      wb[ju][k] = 0.f;
      if (k < K && ju * BLK < C) {
        if (i < C) wb[ju][k] = GP(d.wp)[k * C + i];
      }
    }
  float pg[JU][3];
#pragma unroll
  for (int ju = 0; ju < JU; ++ju) {
    const int c = tid + ju * BLK;
    pg[ju][0] = pg[ju][1] = pg[ju][2] = 0.f;
    if (ju * BLK < C && c < C) { pg[ju][0] = GP(d.gamma)[c]; pg[ju][1] = GP(d.beta)[c]; pg[ju][2] = ((const gfloat*)d.skip.base)[c]; }
  }
  const float bz = (has_b && tid < K) ? GP(d.b)[tid] : 0.f;
  const int sample = t - (UNI(d.n_stages) - 1);
  const int label = ((const gint*)d.labels)[sample % UNI(d.n_stages)];
  // ---- GroupNorm statistics: per-slot partial sums, one wavefront per group
#pragma unroll
  for (int u = 0; u < XU; ++u)
    if (u * BLK < nslot) {
      const int sl = tid + u * BLK;
      if (sl < nslot) psum[sl] = (xr[u][0] + xr[u][1]) + (xr[u][2] + xr[u][3]);
    }
#pragma unroll
  for (int ju = 0; ju < JU; ++ju) {
    const int c = tid + ju * BLK;
    if (ju * BLK < C && c < C) { chan[4 * C + c] = pg[ju][0]; chan[5 * C + c] = pg[ju][1]; chan[6 * C + c] = pg[ju][2]; }
  }
  __syncthreads();
  for (int g = wv; g < G; g += BLK / 64) {
    float sm = 0.f;
    for (int j = lane; j < ns; j += 64) sm += psum[g * ns + j];
    sm = wave_sum(sm);
    if (lane == 0) grp[g] = sm / (float)n;
  }
  __syncthreads();
#pragma unroll
  for (int u = 0; u < XU; ++u)
    if (u * BLK < nslot) {
      const int sl = tid + u * BLK;
      if (sl < nslot) {
        const float m = grp[fdiv(sl, ins)];
        float q = 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e) { const float dl = xr[u][e] - m; q = fmaf(dl, dl, q); }
        psum2[sl] = q;
      }
    }
  __syncthreads();
  for (int g = wv; g < G; g += BLK / 64) {
    float q = 0.f;
    for (int j = lane; j < ns; j += 64) q += psum2[g * ns + j];
    q = wave_sum(q);
    const float mean = grp[g];
    const float rstd = 1.0f / sqrtf(q / (float)n + GN_EPS);
    for (int c = lane; c < cpg; c += 64) {
      const int ch = g * cpg + c;
      const float sc = chan[4 * C + ch] * rstd;
      chan[ch] = sc;
      chan[C + ch] = fmaf(-mean, sc, chan[5 * C + ch]);
      chan[2 * C + ch] = mean;
      chan[3 * C + ch] = rstd;
    }
  }
  __syncthreads();
  // ---- ReLU and average pool: per-slot partial sums, then 4 lanes per channel
#pragma unroll
  for (int u = 0; u < XU; ++u)
    if (u * BLK < nslot) {
      const int sl = tid + u * BLK;
      if (sl < nslot) {
        const int c = fdiv(sl, ihw4);
        const float sc = chan[c], sh = chan[C + c];
        float sm = 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e) { float v = fmaf(sc, xr[u][e], sh); if (rl) v = fmaxf(v, 0.f); sm += v; }
        psum[sl] = sm;
      }
    }
  __syncthreads();
  for (int j = tid; j < 4 * C; j += BLK) {           // lanes 4c..4c+3 share channel c
    const int c = j >> 2, p = j & 3;
    float sm = 0.f;
    for (int i = p; i < HW4; i += 4) sm += psum[c * HW4 + i];
    sm += dpp_src<0xB1, 0xF>(sm);
    sm += dpp_src<0x4E, 0xF>(sm);
    if (p == 0) vec[c] = sm / (float)HW;
  }
  if (tid < K) ebuf[tid] = bz;
  __syncthreads();
#pragma unroll
  for (int ku = 0; ku < KU; ++ku) {
    const int k = wv + 4 * ku;
    if (k < K) {
      float sm = 0.f;
#pragma unroll
      for (int iu = 0; iu < IU; ++iu) {
        const int i = lane + 64 * iu;
        if (64 * iu < C && i < C) sm = fmaf(wf[ku][iu], vec[i], sm);
      }
      sm = wave_sum(sm);
      if (lane == 0) logit[k] = sm + ebuf[k];
    }
  }
  __syncthreads();
  // ---- loss and dlogits
  float mx = -3.0e38f;
#pragma unroll
  for (int k = 0; k < HEAD_MAX_K; ++k)
    if (k < K) mx = fmaxf(mx, logit[k]);
  const float zl = logit[label];
  __syncthreads();
  if (tid < K) ebuf[tid] = expf(logit[tid] - mx);
  __syncthreads();
  float dl[HEAD_MAX_K];
  float sm = 0.f;
#pragma unroll
  for (int k = 0; k < HEAD_MAX_K; ++k) { dl[k] = (k < K) ? ebuf[k] : 0.f; sm += dl[k]; }
  if (tid == 0) GP(d.loss_log)[sample % UNI(d.loss_cap)] = logf(sm) + mx - zl;
#pragma unroll
  for (int k = 0; k < HEAD_MAX_K; ++k) dl[k] = dl[k] / sm - (k == label ? 1.f : 0.f);
  // ---- backward of the linear layer: dW = dl (x) vec, db = dl, dvec = W_cur^T dl
#pragma unroll
  for (int ju = 0; ju < JU; ++ju) {
    const int i = tid + ju * BLK;
    if (ju * BLK < C && i < C) {
      const float vi = vec[i];
      float a = 0.f;
#pragma unroll
      for (int k = 0; k < HEAD_MAX_K; ++k)
        if (k < K) {
          GP(d.gw)[k * C + i] = dl[k] * vi;
          a = fmaf(wb[ju][k], dl[k], a);
        }
      dvec[i] = a / (float)HW;                      // gradient of every element under the pool
    }
  }
  if (has_b) {
#pragma unroll
    for (int k = 0; k < HEAD_MAX_K; ++k)
      if (k < K && tid == k) GP(d.gb)[k] = dl[k];
  }
  __syncthreads();
  // ---- GroupNorm backward: per-slot partial sums of du*xh and du
#pragma unroll
  for (int u = 0; u < XU; ++u)
    if (u * BLK < nslot) {
      const int sl = tid + u * BLK;
      if (sl < nslot) {
        const int c = fdiv(sl, ihw4);
        const float sc = chan[c], sh = chan[C + c], mean = chan[2 * C + c], rstd = chan[3 * C + c], du0 = dvec[c];
        float sg = 0.f, sb = 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          float du = du0;
          if (rl && !(fmaf(sc, xr[u][e], sh) > 0.f)) du = 0.f;
          sg = fmaf(du, (xr[u][e] - mean) * rstd, sg);
          sb += du;
        }
        psum[sl] = sg; psum2[sl] = sb;
      }
    }
  __syncthreads();
  for (int j = tid; j < 4 * C; j += BLK) {
    const int c = j >> 2, p = j & 3;
    float sg = 0.f, sb = 0.f;
    for (int i = p; i < HW4; i += 4) { sg += psum[c * HW4 + i]; sb += psum2[c * HW4 + i]; }
    sg += dpp_src<0xB1, 0xF>(sg); sb += dpp_src<0xB1, 0xF>(sb);
    sg += dpp_src<0x4E, 0xF>(sg); sb += dpp_src<0x4E, 0xF>(sb);
    if (p == 0) {
      GP(d.ggamma)[c] = sg; GP(d.gbeta)[c] = sb;
      const float gm = chan[6 * C + c];
      chan[7 * C + c] = gm * sb; chan[8 * C + c] = gm * sg;
    }
  }
  __syncthreads();
  if (d.dx.base == nullptr) return;
  if (tid < G) {
    float S1 = 0.f, S2 = 0.f;
    for (int j = 0; j < cpg; ++j) { S1 += chan[7 * C + tid * cpg + j]; S2 += chan[8 * C + tid * cpg + j]; }
    const float inv_n = 1.0f / (float)n;
    grp[tid] = S1 * inv_n; grp[G + tid] = S2 * inv_n;
  }
  __syncthreads();
  gfloat* dx = at(d.dx, t);
#pragma unroll
  for (int u = 0; u < XU; ++u)
    if (u * BLK < nslot) {
      const int sl = tid + u * BLK;
      if (sl < nslot) {
        const int c = fdiv(sl, ihw4), g = fdiv(sl, ins);
        const float sc = chan[c], sh = chan[C + c], mean = chan[2 * C + c], rstd = chan[3 * C + c];
        const float dug = dvec[c] * chan[6 * C + c], m1 = grp[g], m2 = grp[G + g];
        v4f o;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          float du = dug;
          if (rl && !(fmaf(sc, xr[u][e], sh) > 0.f)) du = 0.f;
          const float xh = (xr[u][e] - mean) * rstd;
          o[e] = rbf_if(flags & F_BF16_OUT, rstd * (du - m1 - xh * m2));
        }
        PB_ST(nt, (gv4*)(dx + 4 * sl), o);
      }
    }
}

// Pooled last stage with FOUR GroupNorm groups on an 8x8 map (the CIFAR ResNets): one group per
// wavefront.  A group's 16 * C/4 vectors sit in the registers of one wavefront, slot lane + 64 u, so
// that a channel (16 vectors) is one row of 16 lanes at a fixed u: group statistics are wavefront
// sums, channel sums are row sums, and neither needs LDS or a barrier.  The workgroup meets three
// times: pooled activations -> linear layer (rows dealt out to the wavefronts) -> logits -> loss and
// gradient of the pooled activations -> GroupNorm backward, again inside the wavefront.  The general
// form above needs fourteen barriers for the same work.  XW = vectors per lane = C / 16.
template <int XW>
__device__ __forceinline__ void step_head_wave(const LDesc& d, int t, lfloat* smem) {
  const int tid = threadIdx.x, lane = tid & 63, wv = UNI(tid >> 6);
  const int C = UNI(d.C), K = UNI(d.K), flags = UNI(d.flags);
  constexpr int HW = 64;
  const int cpg = C >> 2, n = cpg * HW, nu = cpg >> 2;       // per group: channels, elements, vectors per lane
  const bool rl = flags & F_PRE_RELU, has_b = flags & F_BIAS;
  lfloat* vec = smem;                  // [256] pooled activations
  lfloat* dvec = vec + 256;            // [256] gradient of an element under the pool
  lfloat* logit = dvec + 256;          // [HEAD_MAX_K]
  const int c0 = wv * cpg + (lane >> 4);                     // channel of the lane's vector u: c0 + 4 u
  const gfloat* xg = at(d.x, t) + (size_t)wv * n;
  // ---- all global reads in one burst
  v4f xr[XW];
  float gf[XW], bfw[XW], gbk[XW];
#pragma unroll
  for (int u = 0; u < XW; ++u) {
    xr[u] = (v4f){0.f, 0.f, 0.f, 0.f};
    gf[u] = bfw[u] = gbk[u] = 0.f;
    if (u < nu) {
      xr[u] = *(const gv4*)(xg + 4 * (lane + 64 * u));
      const int c = c0 + 4 * u;
      gf[u] = GP(d.gamma)[c]; bfw[u] = GP(d.beta)[c]; gbk[u] = ((const gfloat*)d.skip.base)[c];
    }
  }
  constexpr int KU = HEAD_MAX_K / 4, IU = 4;
  float wf[KU][IU];        // forward weights: wavefront wv holds rows wv, wv + 4, ..., lane holds columns lane + 64 i
#pragma unroll
  for (int ku = 0; ku < KU; ++ku)
#pragma unroll
    for (int iu = 0; iu < IU; ++iu) {
      const int k = wv + 4 * ku, i = lane + 64 * iu;
      wf[ku][iu] = 0.f;
      if (4 * ku < K && 64 * iu < C) {
        if (k < K && i < C) wf[ku][iu] = GP(d.w)[k * C + i];
      }
    }
  float wb[HEAD_MAX_K];    // backward (current) weights: thread holds column tid
#pragma unroll
  for (int k = 0; k < HEAD_MAX_K; ++k) {
    wb[k] = 0.f;
    if (k < K && tid < C) wb[k] = GP(d.wp)[k * C + tid];
  }
  const float bz = (has_b && tid < K) ? GP(d.b)[tid] : 0.f;
  const int sample = t - (UNI(d.n_stages) - 1);
  const int label = ((const gint*)d.labels)[sample % UNI(d.n_stages)];
  // ---- GroupNorm statistics of the wavefront's group (two passes over registers)
  float sm = 0.f;
#pragma unroll
  for (int u = 0; u < XW; ++u) sm += (xr[u][0] + xr[u][1]) + (xr[u][2] + xr[u][3]);
  const float mean = wave_sum(sm) / (float)n;
  float q = 0.f;
#pragma unroll
  for (int u = 0; u < XW; ++u)
    if (u < nu) {
#pragma unroll
      for (int e = 0; e < 4; ++e) { const float dl = xr[u][e] - mean; q = fmaf(dl, dl, q); }
    }
  const float rstd = 1.0f / sqrtf(wave_sum(q) / (float)n + GN_EPS);
  // ---- normalise, ReLU, average pool: a channel is a row of 16 lanes
  float sc[XW], sh[XW];
#pragma unroll
  for (int u = 0; u < XW; ++u) {
    sc[u] = gf[u] * rstd;
    sh[u] = fmaf(-mean, sc[u], bfw[u]);
    float ps = 0.f;
#pragma unroll
    for (int e = 0; e < 4; ++e) { float v = fmaf(sc[u], xr[u][e], sh[u]); if (rl) v = fmaxf(v, 0.f); ps += v; }
    ps = row_sum(ps);
    if (u < nu && (lane & 15) == 0) vec[c0 + 4 * u] = ps / (float)HW;
  }
  __syncthreads();
  // ---- linear layer: wavefront wv computes rows wv, wv + 4, ...
#pragma unroll
  for (int ku = 0; ku < KU; ++ku) {
    const int k = wv + 4 * ku;
    if (k < K) {
      float a = 0.f;
#pragma unroll
      for (int iu = 0; iu < IU; ++iu) {
        const int i = lane + 64 * iu;
        if (64 * iu < C && i < C) a = fmaf(wf[ku][iu], vec[i], a);
      }
      a = wave_sum(a);
      if (lane == 0) logit[k] = a;
    }
  }
  if (tid < K) dvec[tid] = bz;           // the bias rides in dvec[0..K) until the next barrier
  __syncthreads();
  // ---- loss and dlogits (every thread, from LDS)
  float dl[HEAD_MAX_K];
  float mx = -3.0e38f;
#pragma unroll
  for (int k = 0; k < HEAD_MAX_K; ++k) {
    dl[k] = (k < K) ? logit[k] + dvec[k] : -3.0e38f;
    mx = fmaxf(mx, dl[k]);
  }
  const float zl = logit[label] + dvec[label];
  float se = 0.f;
#pragma unroll
  for (int k = 0; k < HEAD_MAX_K; ++k) { dl[k] = (k < K) ? expf(dl[k] - mx) : 0.f; se += dl[k]; }
  if (tid == 0) GP(d.loss_log)[sample % UNI(d.loss_cap)] = logf(se) + mx - zl;
#pragma unroll
  for (int k = 0; k < HEAD_MAX_K; ++k) dl[k] = dl[k] / se - (k == label ? 1.f : 0.f);
  __syncthreads();                       // every thread has read the bias out of dvec
  // ---- backward of the linear layer: dW = dl (x) vec, db = dl, dvec = W_cur^T dl / HW
  if (tid < C) {
    const float vi = vec[tid];
    float a = 0.f;
#pragma unroll
    for (int k = 0; k < HEAD_MAX_K; ++k)
      if (k < K) {
        GP(d.gw)[k * C + tid] = dl[k] * vi;
        a = fmaf(wb[k], dl[k], a);
      }
    dvec[tid] = a / (float)HW;
  }
  if (has_b) {
#pragma unroll
    for (int k = 0; k < HEAD_MAX_K; ++k)
      if (k < K && tid == k) GP(d.gb)[k] = dl[k];
  }
  __syncthreads();
  // ---- GroupNorm backward inside the wavefront
  float s1 = 0.f, s2 = 0.f;              // group sums of gamma_b * (channel sums), taken from one lane per row
  float dug[XW];
#pragma unroll
  for (int u = 0; u < XW; ++u) {
    dug[u] = 0.f;
    if (u < nu) {
      const int c = c0 + 4 * u;
      const float du0 = dvec[c];
      float sg = 0.f, sb = 0.f;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float du = du0;
        if (rl && !(fmaf(sc[u], xr[u][e], sh[u]) > 0.f)) du = 0.f;
        sg = fmaf(du, (xr[u][e] - mean) * rstd, sg);
        sb += du;
      }
      sg = row_sum(sg); sb = row_sum(sb);
      if ((lane & 15) == 0) {
        GP(d.ggamma)[c] = sg; GP(d.gbeta)[c] = sb;
        s1 = fmaf(gbk[u], sb, s1); s2 = fmaf(gbk[u], sg, s2);
      }
      dug[u] = du0 * gbk[u];
    }
  }
  if (d.dx.base == nullptr) return;
  const float inv_n = 1.0f / (float)n;
  const float m1 = wave_sum(s1) * inv_n, m2 = wave_sum(s2) * inv_n;
  gfloat* dx = at(d.dx, t) + (size_t)wv * n;
#pragma unroll
  for (int u = 0; u < XW; ++u)
    if (u < nu) {
      v4f o;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float du = dug[u];
        if (rl && !(fmaf(sc[u], xr[u][e], sh[u]) > 0.f)) du = 0.f;
        const float xh = (xr[u][e] - mean) * rstd;
        o[e] = rbf_if(flags & F_BF16_OUT, rstd * (du - m1 - xh * m2));
      }
      *(gv4*)(dx + 4 * (lane + 64 * u)) = o;
    }
}

// The whole last stage in one workgroup: [GroupNorm, ReLU, global average
// pool |  ReLU | nothing] -> linear -> softmax cross-entropy -> backward of all
// of it.  Forward parameters: d.w / d.b / d.gamma / d.beta point into the
// predicted arena; the backward ones (current weights) are d.wp (weight) and
// d.skip.base (GroupNorm scale).
//
// A single workgroup cannot hide memory latency behind other work, so every
// global read of the step is requested in one burst at the start (the input
// goes to LDS, the weights stay in registers) and everything after that runs
// out of LDS and registers.
// LDS: xs[C*H*W] | vec[512] | dvec[512] | logit[16] | bias[16] | chan[9*C] | grp[2*G]
__device__ __forceinline__ void step_head(const LDesc& d, int t, lfloat* red, lfloat* smem, const bool nt) {
  (void)red;
  if ((UNI(d.flags) & F_PRE_AFFINE) && (UNI(d.flags) & F_DU_GAP) && UNI(d.H) * UNI(d.W) == 64 && UNI(d.G) == 4 &&
      (UNI(d.C) & 15) == 0 && UNI(d.C) <= 256) {
    if (UNI(d.C) <= 64) step_head_wave<4>(d, t, smem);
    else step_head_wave<16>(d, t, smem);
    return;
  }
  if ((UNI(d.flags) & F_PRE_AFFINE) && (UNI(d.flags) & F_DU_GAP) && ((UNI(d.H) * UNI(d.W)) & 3) == 0) {
    if (UNI(d.C) * UNI(d.H) * UNI(d.W) <= HEAD_MAX_IN) step_head_gap4<HEAD_MAX_IN / (4 * BLK)>(d, t, smem, nt);
    else step_head_gap4<2 * HEAD_MAX_IN / (4 * BLK)>(d, t, smem, nt);
    return;
  }
  const int tid = threadIdx.x, lane = tid & 63, wv = UNI(tid >> 6);
  const int C = UNI(d.C), HW = UNI(d.H) * UNI(d.W), K = UNI(d.K), G = UNI(d.G), flags = UNI(d.flags);
  const bool gn = flags & F_PRE_AFFINE, rl = flags & F_PRE_RELU, gap = flags & F_DU_GAP, has_b = flags & F_BIAS;
  const int n_in = C * HW;
  const int Cv = gap ? C : n_in;                   // length of the vector the linear layer sees
  lfloat* xs = smem;
  lfloat* vec = xs + ((n_in + 3) & ~3);
  lfloat* dvec = vec + HEAD_MAX_CV;
  lfloat* logit = dvec + HEAD_MAX_CV;
  lfloat* bias = logit + HEAD_MAX_K;
  lfloat* chan = bias + HEAD_MAX_K;                // sc, sh, mean, rstd, gamma_f, beta_f, gamma_b, S1 part, S2 part
  lfloat* grp = chan + 9 * C;                      // S1[G], S2[G]
  const gfloat* x = at(d.x, t);
  // ---- all global reads
  constexpr int XU = HEAD_MAX_IN / (4 * BLK);
  v4f xr[XU];
  const bool x4 = (n_in & 3) == 0;
#pragma unroll
  for (int u = 0; u < XU; ++u) {
    xr[u] = (v4f){0.f, 0.f, 0.f, 0.f};
    if (x4) {
      const int i = (tid + u * BLK) * 4;
      if (i < n_in) xr[u] = *(const gv4*)(x + i);
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int i = tid + (4 * u + e) * BLK;
        if (i < n_in) xr[u][e] = x[i];
      }
    }
  }
  constexpr int KU = HEAD_MAX_K / 4, IU = HEAD_MAX_CV / 64, JU = HEAD_MAX_CV / BLK;
  float wf[KU][IU];      // forward weights: wave wv holds rows wv, wv + 4, ...
#pragma unroll
  for (int ku = 0; ku < KU; ++ku)
#pragma unroll
    for (int iu = 0; iu < IU; ++iu) {
      const int k = wv + 4 * ku, i = lane + 64 * iu;
      wf[ku][iu] = 0.f;
      if (4 * ku < K && 64 * iu < Cv) {            // scalar test first: whole blocks are skipped
        if (k < K && i < Cv) wf[ku][iu] = GP(d.w)[k * Cv + i];
      }
    }
  float wb[JU][HEAD_MAX_K];   // backward (current) weights: thread holds columns tid, tid + 256
#pragma unroll
  for (int ju = 0; ju < JU; ++ju)
#pragma unroll
    for (int k = 0; k < HEAD_MAX_K; ++k) {
      const int i = tid + ju * BLK;
      wb[ju][k] = 0.f;
      if (k < K && ju * BLK < Cv) {
        if (i < Cv) wb[ju][k] = GP(d.wp)[k * Cv + i];
      }
    }
  float pg[JU][3];
#pragma unroll
  for (int ju = 0; ju < JU; ++ju) {
    const int c = tid + ju * BLK;
    pg[ju][0] = pg[ju][1] = pg[ju][2] = 0.f;
    if (gn && c < C) { pg[ju][0] = GP(d.gamma)[c]; pg[ju][1] = GP(d.beta)[c]; pg[ju][2] = ((const gfloat*)d.skip.base)[c]; }
  }
  const float bz = (has_b && tid < K) ? GP(d.b)[tid] : 0.f;
  const int sample = t - (UNI(d.n_stages) - 1);
  const int label = ((const gint*)d.labels)[sample % UNI(d.n_stages)];
  PB_TS(1);
  // ---- park them
#pragma unroll
  for (int u = 0; u < XU; ++u) {
    if (x4) {
      const int i = (tid + u * BLK) * 4;
      if (i < n_in) *(lv4*)(xs + i) = xr[u];
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int i = tid + (4 * u + e) * BLK;
        if (i < n_in) xs[i] = xr[u][e];
      }
    }
  }
#pragma unroll
  for (int ju = 0; ju < JU; ++ju) {
    const int c = tid + ju * BLK;
    if (gn && c < C) { chan[4 * C + c] = pg[ju][0]; chan[5 * C + c] = pg[ju][1]; chan[6 * C + c] = pg[ju][2]; }
  }
  if (tid < K) bias[tid] = bz;
  __syncthreads();
  PB_TS(2);
  // ---- forward
  const int cpg = gn ? C / G : 1, n = cpg * HW;
  if (gn) {
    for (int g = wv; g < G; g += BLK / 64) {          // one wavefront per group
      const lfloat* xp = xs + g * n;
      float sm = 0.f;
      for (int i = lane; i < n; i += 64) sm += xp[i];
      const float mean = wave_sum(sm) / (float)n;
      float q = 0.f;
      for (int i = lane; i < n; i += 64) { const float dl = xp[i] - mean; q = fmaf(dl, dl, q); }
      const float var = wave_sum(q) / (float)n;
      const float rstd = 1.0f / sqrtf(var + GN_EPS);
      for (int c = lane; c < cpg; c += 64) {
        const int ch = g * cpg + c;
        const float sc = chan[4 * C + ch] * rstd;
        chan[ch] = sc;
        chan[C + ch] = fmaf(-mean, sc, chan[5 * C + ch]);
        chan[2 * C + ch] = mean;
        chan[3 * C + ch] = rstd;
      }
    }
    __syncthreads();
  }
  PB_TS(3);
  if (gap) {
    for (int c = wv; c < C; c += BLK / 64) {
      const float sc = gn ? chan[c] : 1.f, sh = gn ? chan[C + c] : 0.f;
      float sm = 0.f;
      for (int i = lane; i < HW; i += 64) {
        float v = fmaf(sc, xs[c * HW + i], sh);
        if (rl) v = fmaxf(v, 0.f);
        sm += v;
      }
      sm = wave_sum(sm);
      if (lane == 0) vec[c] = sm / (float)HW;
    }
  } else {
    for (int i = tid; i < Cv; i += BLK) { const float v = xs[i]; vec[i] = rl ? fmaxf(v, 0.f) : v; }
  }
  __syncthreads();
  PB_TS(4);
#pragma unroll
  for (int ku = 0; ku < KU; ++ku) {
    const int k = wv + 4 * ku;
    if (k < K) {
      float sm = 0.f;
#pragma unroll
      for (int iu = 0; iu < IU; ++iu) {
        const int i = lane + 64 * iu;
        if (i < Cv) sm = fmaf(wf[ku][iu], vec[i], sm);
      }
      sm = wave_sum(sm);
      if (lane == 0) logit[k] = sm + bias[k];
    }
  }
  __syncthreads();
  PB_TS(5);
  // ---- loss and dlogits: K is small, every thread computes them
  float dl[HEAD_MAX_K];
  {
    float mx = -3.0e38f;
#pragma unroll
    for (int k = 0; k < HEAD_MAX_K; ++k) { dl[k] = (k < K) ? logit[k] : -3.0e38f; mx = fmaxf(mx, dl[k]); }
    float sm = 0.f;
#pragma unroll
    for (int k = 0; k < HEAD_MAX_K; ++k) { dl[k] = (k < K) ? expf(dl[k] - mx) : 0.f; sm += dl[k]; }
    if (tid == 0) GP(d.loss_log)[sample % UNI(d.loss_cap)] = logf(sm) + mx - logit[label];
#pragma unroll
    for (int k = 0; k < HEAD_MAX_K; ++k) dl[k] = dl[k] / sm - (k == label ? 1.f : 0.f);
  }
  PB_TS(6);
  // ---- backward of the linear layer: dW = dl (x) vec, db = dl, dvec = W_cur^T dl
#pragma unroll
  for (int ju = 0; ju < JU; ++ju) {
    const int i = tid + ju * BLK;
    if (i < Cv) {
      const float vi = vec[i];
      float sm = 0.f;
#pragma unroll
      for (int k = 0; k < HEAD_MAX_K; ++k)
        if (k < K) {
          GP(d.gw)[(size_t)k * Cv + i] = dl[k] * vi;
          sm = fmaf(wb[ju][k], dl[k], sm);
        }
      dvec[i] = sm;
    }
  }
  if (has_b) {
#pragma unroll
    for (int k = 0; k < HEAD_MAX_K; ++k)
      if (k < K && tid == k) GP(d.gb)[k] = dl[k];
  }
  if (d.dx.base == nullptr && !gn) return;
  gfloat* dx = d.dx.base ? at(d.dx, t) : nullptr;
  if (!gn) {
    // dvec[i] was written by this thread
    for (int i = tid; i < Cv; i += BLK) { float r = dvec[i]; if (rl && !(xs[i] > 0.f)) r = 0.f; dx[i] = rbf_if(flags & F_BF16_OUT, r); }
    return;
  }
  __syncthreads();
  PB_TS(7);
  // ---- GroupNorm backward with du[c,hw] = dvec[c]/HW (after the pool) or dvec[c*HW+hw]
  for (int c = wv; c < C; c += BLK / 64) {
    const float sc = chan[c], sh = chan[C + c], mean = chan[2 * C + c], rstd = chan[3 * C + c];
    float sg = 0.f, sb = 0.f;
    for (int i = lane; i < HW; i += 64) {
      const float xv = xs[c * HW + i];
      float du = gap ? dvec[c] / (float)HW : dvec[c * HW + i];
      if (rl && !(fmaf(sc, xv, sh) > 0.f)) du = 0.f;
      sg = fmaf(du, (xv - mean) * rstd, sg);
      sb += du;
    }
    sg = wave_sum(sg); sb = wave_sum(sb);
    if (lane == 0) {
      GP(d.ggamma)[c] = sg; GP(d.gbeta)[c] = sb;
      const float gm = chan[6 * C + c];
      chan[7 * C + c] = gm * sb; chan[8 * C + c] = gm * sg;
    }
  }
  __syncthreads();
  PB_TS(8);
  if (!dx) return;
  if (tid < G) {
    float S1 = 0.f, S2 = 0.f;
    for (int j = 0; j < cpg; ++j) { S1 += chan[7 * C + tid * cpg + j]; S2 += chan[8 * C + tid * cpg + j]; }
    grp[tid] = S1; grp[G + tid] = S2;
  }
  __syncthreads();
  const float inv_n = 1.0f / (float)n;
  const float ihw = frcp(HW), icpg = frcp(cpg);
  for (int o = tid; o < n_in; o += BLK) {
    const int c = fdiv(o, ihw), g = fdiv(c, icpg);
    const float sc = chan[c], sh = chan[C + c], mean = chan[2 * C + c], rstd = chan[3 * C + c];
    const float xv = xs[o];
    float du = gap ? dvec[c] / (float)HW : dvec[o];
    if (rl && !(fmaf(sc, xv, sh) > 0.f)) du = 0.f;
    const float xh = (xv - mean) * rstd;
    dx[o] = rbf_if(flags & F_BF16_OUT, rstd * (du * chan[6 * C + c] - grp[g] * inv_n - xh * (grp[G + g] * inv_n)));
  }
}

// ------------------------------------------------------------------ kernels
// One workgroup = one tile of one step.  recs[] holds, per workgroup of the
// phase, a full copy of its step descriptor with the tile index filled in, so
// that a single burst of scalar loads (one memory round trip) delivers all a
// workgroup needs to know.
// NT: bulk outputs are stored with the non-temporal hint (networks tiled for latency, see PB_ST).
template <bool NT>
__global__ void __launch_bounds__(BLK) __attribute__((amdgpu_waves_per_eu(2, 2)))
k_phase(const StepDesc* __restrict__ recs, const Globals* __restrict__ G, int k,
        const float* __restrict__ sample_override, int label_override, int32_t* __restrict__ sync, uint32_t tick_ordinal) {
  __shared__ float red_[8];
  __shared__ __attribute__((aligned(16))) float smem_[LDS_FLOATS];
  lfloat* red = (lfloat*)red_;
  lfloat* smem = (lfloat*)smem_;
  const int t = G->t_base + k;
#ifdef PB_TIMING
  if (threadIdx.x < 96) ts_sh[threadIdx.x / 24][threadIdx.x % 24] = 0;
  __syncthreads();
  PB_TS(0);
#endif
  // The descriptor arrives through the vector memory path (one coalesced
  // request) and is parked in LDS; a burst of scalar loads of data no other
  // workgroup shares would miss the scalar cache line after line.
  constexpr int NW = (int)(sizeof(StepDesc) / 4);
  static_assert(sizeof(StepDesc) % 4 == 0 && NW <= BLK, "descriptor must fit one word per thread");
  __shared__ StepDesc sd_;
  {
    const gint* dp = (const gint*)(recs + blockIdx.x);
    if (threadIdx.x < NW) ((lint*)&sd_)[threadIdx.x] = dp[threadIdx.x];
  }
  __syncthreads();
  const LDesc& d = *(const LDesc*)&sd_;
  // Predicted weights live in a ring of versions per stage (the update of tick t writes slot t+1, the
  // forward pass of tick t reads slot t - extra delay): move the step's pointers to its slot.
  if (UNI(d.pmask) != 0) {
    const int depth = UNI(d.pdepth), u = t - UNI(d.plag);
    const int slot = u < 0 ? 0 : u % depth;
    const size_t off = (size_t)slot * (size_t)UNI(d.pstride);
    const int f = threadIdx.x;
    if (f < 7 && ((UNI(d.pmask) >> f) & 1)) {
      switch (f) {
        case 0: sd_.w += off; break;
        case 1: sd_.b += off; break;
        case 2: sd_.wp += off; break;
        case 3: sd_.gamma += off; break;
        case 4: sd_.beta += off; break;
        case 5: sd_.what += off; break;
        default: sd_.skip.base += off; break;
      }
    }
    __syncthreads();
  }
  if (UNI(d.ppstride) != 0) {
    // update of a stage with two copies of its master parameters: read the tick's copy, write the other
    if (threadIdx.x == 0) {
      if (t & 1) sd_.w += (size_t)UNI(d.ppstride);
      else sd_.wp += (size_t)UNI(d.ppstride);
    }
    __syncthreads();
  }
  const int tile = UNI(d.tile);
  const bool live = t >= UNI(d.first_tick);
  bool run = live || (UNI(d.flags) & F_ALWAYS);
  // One launch per tick: the grid holds the workgroups of every phase, in phase order.  Workgroups are handed
  // out in index order, so when a workgroup of a later phase runs, the workgroups it depends on (lower
  // indices: the same stage's steps of the earlier phases) are running or done; it waits for their completion
  // counters.  The wait is bounded: on expiry the error word is set and the step is skipped, so that the grid
  // always drains.
  if (sync != nullptr && UNI(d.nwait) > 0) {
    __shared__ int wait_ok_;
    if (threadIdx.x == 0) {
      const int limit = ((const gint*)sync)[SYNC_SPIN];
      // (once a wait has expired anywhere, nobody waits any more: the rest of the work drains at once)
      int ok = __hip_atomic_load(sync + SYNC_ERR, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0, it = 0;
      for (int q = 0; q < d.nwait && ok; ++q) {
        const uint32_t target = tick_ordinal * (uint32_t)d.wait_n[q];
        while ((int32_t)((uint32_t)__hip_atomic_load(sync + SYNC_CNT + d.wait_idx[q], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - target) < 0) {
          if (++it > limit) { ok = 0; break; }
          __builtin_amdgcn_s_sleep(2);
        }
      }
      if (!ok) __hip_atomic_fetch_or(sync + SYNC_ERR, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      // what the producers wrote before they counted themselves done is visible from here on: one wavefront's
      // acquire drops the stale lines of this compute unit's vector cache and of this XCD's L2 for all four,
      // which read nothing of it before the barrier
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
      wait_ok_ = ok;
    }
    __syncthreads();
    if (!wait_ok_) run = false;
  }
  if (run) {
  switch (UNI(d.kind)) {
    case K_GN_STATS:
      if (UNI(d.grain) == 1) step_gn_stats_wave(d, t, smem, NT); else step_gn_stats(d, tile, t, red, smem, NT);
      break;
    case K_GAP_FWD: step_gap_fwd(d, tile, t, red); break;
    case K_CONV_FWD: step_conv_fwd(d, tile, t); break;
    case K_POST_FWD: step_post_fwd(d, tile, t); break;
    case K_CE: step_ce(d, tile, t, red); break;
    case K_GNB_REDUCE: step_gnb_reduce(d, tile, t, red, smem, NT); break;
    case K_GNB_APPLY: step_gnb_apply(d, tile, t); break;
    case K_CONV_BWD_X: step_conv_bwd_x(d, tile, t); break;
    case K_CONV_BWD_W: step_conv_bwd_w(d, tile, t); break;
    case K_COPY: step_copy(d, tile, t, NT); break;
    case K_GEMM: step_gemm<NT>(d, tile, t, smem); break;
    case K_BIAS_GRAD: step_bias_grad(d, tile, t); break;
    case K_INGEST: step_ingest(d, tile, t, G, k, sample_override, label_override); break;
    case K_UPDATE: step_update(d, tile, t, smem, NT); break;
    case K_HEAD: step_head(d, t, red, smem, NT); break;
    case K_GN_BWD: step_gn_bwd(d, tile, t, live, smem, NT); break;
    // (planned only for networks tiled for throughput: the other instantiation carries no code for them)
    case K_DOT_FWD: if (!NT) step_dot_fwd(d, tile, t, smem); break;
    case K_DOT_BWD_X: if (!NT) step_dot_bwd_x(d, tile, t, smem); break;
    case K_FC_FWD: if (!NT) step_fc_fwd(d, tile, t); break;
    case K_FC_BWD_X: if (!NT) step_fc_bwd_x(d, tile, t, smem); break;
    case K_FC_BWD_W: if (!NT) step_fc_bwd_w(d, tile, t); break;
    default: break;
  }
  }
  if (sync != nullptr && UNI(d.sig_idx) >= 0) {
    // every wavefront waits until its own stores have reached the L2, then the barrier; the release by one
    // thread then writes that L2's dirty lines back, so that the other XCDs see them before the counter says so
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
    __syncthreads();
    if (threadIdx.x == 0) {
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
      __hip_atomic_fetch_add(sync + SYNC_CNT + d.sig_idx, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
#ifdef PB_TIMING
  PB_TS(11);
#if PB_TIMING == 2
  if (t == pb_ts_tick && (threadIdx.x & 63) == 0 && (int)gridDim.x == pb_ts_grid) {
    // slot = workgroup index; only the launch with pb_ts_grid workgroups is recorded
    const int slot = (int)blockIdx.x;
    const int w = threadIdx.x >> 6;
    if (slot < 16384) {
      pb_ts_out[slot * 100 + 4 + w * 24 + 0] = ts_sh[w][0];
      pb_ts_out[slot * 100 + 4 + w * 24 + 11] = ts_sh[w][11];
      if (w == 0) {
        pb_ts_out[slot * 100 + 0] = d.kind; pb_ts_out[slot * 100 + 1] = d.stage;
        pb_ts_out[slot * 100 + 2] = d.g.gm + 8 * d.g.M; pb_ts_out[slot * 100 + 3] = tile;
      }
    }
  }
  return;
#endif
  __syncthreads();
  if (t == pb_ts_tick && (pb_ts_grid == 0 || pb_ts_grid == (int)gridDim.x)) {
    __shared__ int slot_;
    if (threadIdx.x == 0) slot_ = atomicAdd(&pb_ts_n, 1);
    __syncthreads();
    const int slot = slot_;
    if (slot < 16384) {
      if (threadIdx.x < 96) pb_ts_out[slot * 100 + 4 + threadIdx.x] = ts_sh[threadIdx.x / 24][threadIdx.x % 24];
      if (threadIdx.x == 0) {
        pb_ts_out[slot * 100 + 0] = d.kind; pb_ts_out[slot * 100 + 1] = d.stage;
        pb_ts_out[slot * 100 + 2] = d.g.gm + 8 * d.g.M; pb_ts_out[slot * 100 + 3] = tile;
      }
    }
  }
#endif
}

// Copies the tick's sample into the first stage's input ring and its label
// into the label ring.  staging != nullptr: sample/label were handed over by
// the host call; otherwise they come from the resident pool.
__global__ void __launch_bounds__(BLK)
k_ingest(TRef ring0, int n_elems, const float* __restrict__ staging, int label,
         int32_t* __restrict__ label_ring, int n_stages, const Globals* __restrict__ G, int k) {
  const int t = G->t_base + k;
  const gfloat* src = (const gfloat*)staging;
  int lab = label;
  if (!staging) {
    const int item = (int)(((int64_t)G->idx_base + k) % G->n_pool);
    src = (const gfloat*)G->pool + (size_t)item * n_elems;
    lab = ((const gint*)G->pool_labels)[item];
  }
  gfloat* dst = at(ring0, t);
  const int i = blockIdx.x * BLK + threadIdx.x;
  if (i < n_elems) dst[i] = src[i];
  if (i == 0) label_ring[t % n_stages] = lab;
}


// Same arithmetic over plain arrays with one coefficient set.  A workgroup
// takes U * 1024 consecutive floats; all 3 U loads of a thread are requested
// before the first use, and every access carries the non-temporal hint: the
// arrays are streamed once per launch (on arrays far beyond the caches this is
// worth ~3 % of HBM peak over plain accesses, U = 4 over U = 1 another ~1 %).
template <int U>
__global__ void __launch_bounds__(BLK)
k_update_flat(float* __restrict__ w, float* __restrict__ v, const float* __restrict__ g,
              float* __restrict__ what, float lr, float m, float a, float b, float lrT) {
  const size_t base = (size_t)blockIdx.x * U * (UPD_CHUNK / 4) + threadIdx.x;
  v4f gv[U], vv[U], wv[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const size_t i = base + (size_t)u * (UPD_CHUNK / 4);
    gv[u] = __builtin_nontemporal_load((const v4f*)g + i);
    vv[u] = __builtin_nontemporal_load((const v4f*)v + i);
    wv[u] = __builtin_nontemporal_load((const v4f*)w + i);
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const size_t i = base + (size_t)u * (UPD_CHUNK / 4);
    v4f p;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      vv[u][e] = fmaf(m, vv[u][e], gv[u][e]);
      wv[u][e] = fmaf(-lr, fmaf(a, vv[u][e], b * gv[u][e]), wv[u][e]);
      p[e] = fmaf(-lrT, vv[u][e], wv[u][e]);
    }
    __builtin_nontemporal_store(vv[u], (v4f*)v + i);
    __builtin_nontemporal_store(wv[u], (v4f*)w + i);
    if (what) __builtin_nontemporal_store(p, (v4f*)what + i);
  }
}

__global__ void k_set_globals(Globals* G, Globals val) {
  if (threadIdx.x == 0 && blockIdx.x == 0) *G = val;
}

__global__ void k_advance(Globals* G, int dt, int didx) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    G->t_base += dt;
    G->idx_base = (int)(((int64_t)G->idx_base + didx) % G->n_pool);
  }
}

__global__ void __launch_bounds__(BLK) k_fill_zero(v4f* __restrict__ p, size_t n16) {
  for (size_t i = (size_t)blockIdx.x * BLK + threadIdx.x; i < n16; i += (size_t)gridDim.x * BLK) p[i] = (v4f){0.f, 0.f, 0.f, 0.f};
}

// Device memory of contexts that must not allocate: one array per GPU, held from the moment the
// library's code object is loaded on that GPU until the process ends.  Host code never uses the
// array's name as an address: static_arena() asks the runtime for the array's address on the current
// device, once per device, and everything else works with that pointer.
static __device__ __align__(256) unsigned char scratch[STATIC_ARENA_BYTES];

hipError_t static_arena(void** ptr, int* device) {
  constexpr int MAX_DEVS = 64;
  static void* addr[MAX_DEVS] = {};
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= MAX_DEVS) return hipErrorInvalidDevice;
  if (!addr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    addr[dev] = p;
  }
  *ptr = addr[dev];
  *device = dev;
  return hipSuccess;
}

// --------------------------------------------------------- launch wrappers
void launch_fill_zero(void* p, size_t bytes, hipStream_t s) {
  const size_t n16 = bytes / 16;
  if (!n16) return;
  const size_t want = (n16 + BLK - 1) / BLK;
  const unsigned grid = (unsigned)(want < 4096 ? want : 4096);
  hipLaunchKernelGGL(k_fill_zero, dim3(grid), dim3(BLK), 0, s, (v4f*)p, n16);
}

void launch_phase(const StepDesc* recs_dev, int total_tiles, const Globals* G, int k, const float* sample_override,
                  int label_override, bool nt, hipStream_t s, int32_t* sync, uint32_t tick_ordinal) {
  if (total_tiles <= 0) return;
  if (nt) hipLaunchKernelGGL(k_phase<true>, dim3(total_tiles), dim3(BLK), 0, s, recs_dev, G, k, sample_override, label_override, sync, tick_ordinal);
  else hipLaunchKernelGGL(k_phase<false>, dim3(total_tiles), dim3(BLK), 0, s, recs_dev, G, k, sample_override, label_override, sync, tick_ordinal);
}

void launch_ingest(TRef ring0, int n_elems, const float* staging, int label, int32_t* label_ring,
                   int n_stages, const Globals* G, int k, hipStream_t s) {
  hipLaunchKernelGGL(k_ingest, dim3((n_elems + BLK - 1) / BLK), dim3(BLK), 0, s, ring0, n_elems,
                     staging, label, label_ring, n_stages, G, k);
}


void launch_update_flat(float* w, float* v, const float* g, float* what, int64_t n, float lr, float m,
                        float a, float b, float lrT, hipStream_t s) {
  // n is a multiple of UPD_CHUNK: workgroups of 4 chunks, then single chunks for the rest
  const int64_t big = n / (4 * UPD_CHUNK), done = big * 4 * UPD_CHUNK, rest = (n - done) / UPD_CHUNK;
  if (big)
    hipLaunchKernelGGL(k_update_flat<4>, dim3((unsigned)big), dim3(BLK), 0, s, w, v, g, what, lr, m, a, b, lrT);
  if (rest)
    hipLaunchKernelGGL(k_update_flat<1>, dim3((unsigned)rest), dim3(BLK), 0, s, w + done, v + done, g + done,
                       what ? what + done : nullptr, lr, m, a, b, lrT);
}

void launch_set_globals(Globals* G, Globals val, hipStream_t s) {
  hipLaunchKernelGGL(k_set_globals, dim3(1), dim3(64), 0, s, G, val);
}

void launch_advance(Globals* G, int dt, int didx, hipStream_t s) {
  hipLaunchKernelGGL(k_advance, dim3(1), dim3(64), 0, s, G, dt, didx);
}

}  // namespace pb

#ifdef PB_TIMING
extern "C" int pb_debug_set_tick(int t) {
  int z = 0;
  hipMemcpyToSymbol(HIP_SYMBOL(pb::pb_ts_n), &z, sizeof(int));
  return (int)hipMemcpyToSymbol(HIP_SYMBOL(pb::pb_ts_tick), &t, sizeof(int));
}
extern "C" int pb_debug_set_grid(int g) { return (int)hipMemcpyToSymbol(HIP_SYMBOL(pb::pb_ts_grid), &g, sizeof(int)); }
extern "C" int pb_debug_clear(void) {
  void* p = nullptr;
  hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(pb::pb_ts_out));
  if (e != hipSuccess) return (int)e;
  hipDeviceSynchronize();
  return (int)hipMemset(p, 0, sizeof(long long) * 16384 * 100);
}
extern "C" int pb_debug_dump(long long* host, int max_recs) {
  int n = 0;
  hipDeviceSynchronize();
  hipMemcpyFromSymbol(&n, HIP_SYMBOL(pb::pb_ts_n), sizeof(int));
#if PB_TIMING == 2
  n = 16384;
#endif
  if (n > max_recs) n = max_recs;
  if (n > 16384) n = 16384;
  hipMemcpyFromSymbol(host, HIP_SYMBOL(pb::pb_ts_out), (size_t)n * 100 * sizeof(long long));
  return n;
}
#endif
