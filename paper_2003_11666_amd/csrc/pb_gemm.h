// MFMA implicit-GEMM core shared by the convolution / linear forward,
// backward-data and backward-weights steps (fp32, v_mfma_f32_16x16x4_f32).
//
// Every pass of a layer is C[M x N] += A[M x Q] * B[Q x N]:
//   forward           M = cout,  N = output pixels, q = (cin, kh, kw)
//   backward data     M = cin,   N = input pixels,  q = (cout, kh, kw)
//   backward weights  M = cout,  N = (cin, kh, kw), q = output pixels
// B is never materialised: B[q][n] = patch[offq(q) + offn(n)], where the patch
// is a zero-padded window of the (normalised, rectified) input -- or of the
// output gradient placed at stride spacing -- staged in LDS per chunk of the
// reduction, and offq / offn are separable offsets into it.
#pragma once
#include "pb_device.h"

namespace pb {

typedef float v4f __attribute__((ext_vector_type(4)));

struct Geo { int C, H, W, K, OH, OW, k, s, pad; };

// Accumulate one operand set into acc[0..ni).  Aglob: weights (forward,
// backward data) or dZ (backward weights); src: activation (forward, backward
// weights) or dZ (backward data); st != nullptr applies sc[c]*x+sh[c], relu
// then max(.,0), while staging.
__device__ __forceinline__ void gemm_accumulate(const Geo& ge, const GemmCfg& g, const float* __restrict__ Aglob,
                                                const float* __restrict__ src, const float* __restrict__ st,
                                                int stG, int stC, bool relu, int m0, int n0, float* smem,
                                                v4f acc[4]) {
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int wk_id = wv % g.wk, wn_id = (wv / g.wk) % g.wn, wm_id = wv / (g.wk * g.wn);
  float* As = smem;
  int* offq = reinterpret_cast<int*>(smem + g.o_offq);
  float* patch = smem + g.o_patch;
  const int kk = ge.k * ge.k, PRW = g.PR * g.Wp;
  const int HW = ge.H * ge.W, P = ge.OH * ge.OW;

  // first row (of the output map for forward / backward weights, of the input
  // map for backward data) this tile touches, and per-lane column offsets
  int tile_row0 = 0, c_lo = 0;
  if (g.gm == 1) tile_row0 = n0 / ge.OW;
  else if (g.gm == 2) tile_row0 = n0 / ge.W;
  else c_lo = n0 / kk;
  int offn[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int n = n0 + (wn_id * g.ni + j) * 16 + (lane & 15);
    int o = 0;
    if (j < g.ni && n < g.N) {
      if (g.gm == 1) { const int oh = n / ge.OW, ow = n - oh * ge.OW; o = (oh - tile_row0) * ge.s * g.Wp + ow * ge.s; }
      else if (g.gm == 2) { const int ih = n / ge.W, iw = n - ih * ge.W; o = (ih - tile_row0) * g.Wp + iw; }
      else { const int ci = n / kk, tap = n - ci * kk, kh = tap / ge.k, kw = tap - kh * ge.k; o = (ci - c_lo) * PRW + kh * g.Wp + kw; }
    }
    offn[j] = o;
  }
  __syncthreads();   // LDS may still be in use by a previous operand set
  for (int i = tid; i < g.QCpad; i += BLK) {
    int o = 0;
    if (i < g.QC) {
      if (g.gm == 3) { const int r = i / ge.OW, ow = i - r * ge.OW; o = r * ge.s * g.Wp + ow * ge.s; }
      else {
        const int c = i / kk, tap = i - c * kk, kh = tap / ge.k, kw = tap - kh * ge.k;
        o = (g.gm == 1) ? c * PRW + kh * g.Wp + kw : c * PRW + (ge.k - 1 - kh) * g.Wp + (ge.k - 1 - kw);
      }
    }
    offq[i] = o;
  }
  const int a_row = (wm_id * 16 + (lane & 15)) * g.LDA + (lane >> 4);
  const int nsteps = g.QCpad >> 2;
  const int patch_elems = g.CC * PRW;
  for (int ch = 0; ch < g.n_chunks; ++ch) {
    if (ch) __syncthreads();
    const int q0 = ch * g.QC;
    // ---- A chunk: As[m][qr]
    for (int idx = tid; idx < g.MT * g.QCpad; idx += BLK) {
      const int m = idx / g.QCpad, qr = idx - m * g.QCpad, q = q0 + qr;
      float v = 0.f;
      if (m0 + m < g.M && qr < g.QC && q < g.Q) {
        if (g.gm == 2) { const int co = q / kk, tap = q - co * kk; v = Aglob[(size_t)co * ge.C * kk + (size_t)(m0 + m) * kk + tap]; }
        else v = Aglob[(size_t)(m0 + m) * g.Q + q];
      }
      As[m * g.LDA + qr] = v;
    }
    // ---- patch
    int chan0, row0;
    if (g.gm == 1) { chan0 = ch * g.CC; row0 = tile_row0 * ge.s - ge.pad; }
    else if (g.gm == 2) { chan0 = ch * g.CC; row0 = tile_row0; }
    else { chan0 = c_lo; row0 = ch * g.rows_c * ge.s - ge.pad; }
    for (int idx = tid; idx < patch_elems; idx += BLK) {
      const int c = idx / PRW, rem = idx - c * PRW, y = rem / g.Wp, x = rem - y * g.Wp;
      const int chn = chan0 + c;
      float v = 0.f;
      if (g.gm == 2) {
        // output gradient placed at stride spacing with a (k-1-pad) border
        const int ty = row0 + y - (ge.k - 1 - ge.pad), tx = x - (ge.k - 1 - ge.pad);
        if (chn < ge.K && ty >= 0 && tx >= 0 && ty % ge.s == 0 && tx % ge.s == 0) {
          const int oh = ty / ge.s, ow = tx / ge.s;
          if (oh < ge.OH && ow < ge.OW) v = src[(size_t)chn * P + oh * ge.OW + ow];
        }
      } else {
        const int ih = row0 + y, iw = x - ge.pad;
        if (chn < ge.C && ih >= 0 && ih < ge.H && iw >= 0 && iw < ge.W) {
          v = src[(size_t)chn * HW + ih * ge.W + iw];
          if (st) v = fmaf(st[2 * stG + chn], v, st[2 * stG + stC + chn]);
          if (relu) v = fmaxf(v, 0.f);
        }
      }
      patch[idx] = v;
    }
    __syncthreads();
    // ---- MFMA loop: lane holds A[i = lane%16][k = lane/16] and B[k = lane/16][j = lane%16]
    for (int ks = wk_id; ks < nsteps; ks += g.wk) {
      const float a = As[a_row + ks * 4];
      const int oq = offq[ks * 4 + (lane >> 4)];
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (j < g.ni) acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, patch[oq + offn[j]], acc[j], 0, 0, 0);
    }
  }
}

// One tile of a K_GEMM step.
__device__ void step_gemm(const StepDesc& d, int tile, int t, float* smem) {
  const GemmCfg& g = d.g;
  const int tm = tile / g.tiles_n, tn = tile - tm * g.tiles_n;
  const int m0 = tm * g.MT, n0 = tn * g.NT;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int wk_id = wv % g.wk, wn_id = (wv / g.wk) % g.wn, wm_id = wv / (g.wk * g.wn);
  v4f acc[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) acc[j] = (v4f){0.f, 0.f, 0.f, 0.f};
  const Geo ge{d.C, d.H, d.W, d.K, d.OH, d.OW, d.k, d.stride, d.pad};
  const float* st = (d.flags & F_PRE_AFFINE) ? at(d.st, t) : nullptr;
  if (g.gm == 1) {
    gemm_accumulate(ge, g, d.w, at(d.x, t), st, d.G, d.C, d.flags & F_PRE_RELU, m0, n0, smem, acc);
    if (d.flags & F_PROJ) {
      const Geo gs{d.sC, d.sH, d.sW, d.K, d.OH, d.OW, 1, d.sstride, 0};
      gemm_accumulate(gs, d.gp, d.wp, at(d.skip, t), nullptr, 0, 0, false, m0, n0, smem, acc);
    }
  } else if (g.gm == 2) {
    gemm_accumulate(ge, g, d.w, at(d.dy, t), nullptr, 0, 0, false, m0, n0, smem, acc);
  } else {
    gemm_accumulate(ge, g, at(d.dy, t), at(d.x, t), st, d.G, d.C, d.flags & F_PRE_RELU, m0, n0, smem, acc);
  }
  // ---- reduce the split of the reduction across waves (fixed order)
  if (g.wk > 1) {
    __syncthreads();
    float* red = smem;   // [wave][j][lane] float4
    if (wk_id > 0) {
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (j < g.ni) *reinterpret_cast<v4f*>(red + ((wv * 4 + j) * 64 + lane) * 4) = acc[j];
    }
    __syncthreads();
    if (wk_id == 0) {
      for (int w2 = 1; w2 < g.wk; ++w2)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          if (j < g.ni) acc[j] += *reinterpret_cast<const v4f*>(red + (((wv + w2) * 4 + j) * 64 + lane) * 4);
    }
  }
  if (wk_id != 0) return;
  // ---- epilogue: lane holds C[i = 4*(lane/16) + r][j = lane%16]
  float* out = (g.gm == 1) ? at(d.y, t) : (g.gm == 2) ? at(d.dx, t) : d.gw;
  const float* skip = (g.gm == 1 && (d.flags & F_SKIP) && !(d.flags & F_PROJ)) ? at(d.skip, t) : nullptr;
  const float* xm = (g.gm == 2 && (d.flags & F_MASK_X)) ? at(d.x, t) : nullptr;
  const float* skg = (g.gm == 2 && (d.flags & F_ADD_SKG)) ? at(d.skg, t) : nullptr;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    if (j >= g.ni) continue;
    const int n = n0 + (wn_id * g.ni + j) * 16 + (lane & 15);
    if (n >= g.N) continue;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int m = m0 + wm_id * 16 + 4 * (lane >> 4) + r;
      if (m >= g.M) continue;
      const size_t o = (size_t)m * g.N + n;
      float v = acc[j][r];
      if (g.gm == 1) {
        if (d.flags & F_BIAS) v += d.b[m];
        if (skip) v += skip[o];
      } else if (g.gm == 2) {
        if (xm && !(xm[o] > 0.f)) v = 0.f;
        if (skg) v += skg[o];
      }
      out[o] = v;
    }
  }
}

// db[co] = sum_p dZ[co,p], one wavefront per channel.
__device__ void step_bias_grad(const StepDesc& d, int tile, int t) {
  const int co = tile * (BLK / 64) + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (co >= d.K) return;
  const int P = d.OH * d.OW;
  const float* dz = at(d.dy, t) + (size_t)co * P;
  float s = 0.f;
  for (int p = lane; p < P; p += 64) s += dz[p];
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) s += __shfl_down(s, o, 64);
  if (lane == 0) d.gb[co] = s;
}

}  // namespace pb
