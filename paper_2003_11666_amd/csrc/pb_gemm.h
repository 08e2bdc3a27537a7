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
// reduction, and offq / offn are separable offsets into it.  A goes from
// global memory straight into the MFMA operand registers.
//
// The code is kept small on purpose: a tile's work is a few hundred MFMAs, so
// instruction fetch of a long unrolled path costs more than it saves.
//
// Included by pb_kernels.hip after its address-space helpers.
#pragma once
#include "pb_device.h"

namespace pb {

typedef float v4f __attribute__((ext_vector_type(4)));

// One tile of a K_GEMM step, GM = 1 forward, 2 backward data, 3 backward
// weights.  A forward step may carry a second operand set (the 1x1 projection
// of the skip tensor) that accumulates into the same tile.
//
// The per-step offset tables (tq: reduction index -> patch offset, tn: column
// -> patch offset) are built on the host, so the tile does no index division.
template <int GM>
__device__ __forceinline__ void step_gemm_t(const LDesc& d, int tile, int t, lfloat* smem) {
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int wk = UNI(d.g.wk), wn = UNI(d.g.wn), ni = UNI(d.g.ni);
  const int wk_id = wv % wk, wn_id = (wv / wk) % wn, wm_id = wv / (wk * wn);
  const int tiles_n = UNI(d.g.tiles_n);
  const int tm = tile / tiles_n, tn = tile - tm * tiles_n;
  const int m0 = tm * UNI(d.g.MT), n0 = tn * UNI(d.g.NT);
  const int flags = UNI(d.flags);
  const int kq = lane >> 4;
  v4f acc[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) acc[j] = (v4f){0.f, 0.f, 0.f, 0.f};
  const int nops = (GM == 1 && (flags & F_PROJ)) ? 2 : 1;

  for (int op = 0; op < nops; ++op) {
    const bool second = GM == 1 && op == 1;
    const LGemmCfg& g = second ? d.gp : d.g;
    const int gC = UNI(second ? d.sC : d.C), gH = UNI(second ? d.sH : d.H), gW = UNI(second ? d.sW : d.W);
    const int gK = UNI(d.K), gOH = UNI(d.OH), gOW = UNI(d.OW);
    const int gk = second ? 1 : UNI(d.k), gs = UNI(second ? d.sstride : d.stride), gpad = second ? 0 : UNI(d.pad);
    // A: weights (forward, backward data) or dZ (backward weights);
    // src: activation (forward, backward weights) or dZ (backward data)
    const gfloat* Aglob = second ? GP(d.wp) : (GM == 3 ? (const gfloat*)at(d.dy, t) : GP(d.w));
    const gfloat* src = second ? (const gfloat*)at(d.skip, t)
                               : (GM == 2 ? (const gfloat*)at(d.dy, t) : (const gfloat*)at(d.x, t));
    const gfloat* st = (GM != 2 && !second && (flags & F_PRE_AFFINE)) ? (const gfloat*)at(d.st, t) : nullptr;
    const bool relu = GM != 2 && !second && (flags & F_PRE_RELU);
    const int stG = UNI(d.G), stC = UNI(d.C);
    const gint* tq = (const gint*)(second ? d.tq2 : d.tq);
    const gint* tnb = (const gint*)(second ? d.tn2 : d.tn);

    lint* offq = (lint*)(smem + UNI(g.o_offq));
    lfloat* patch = smem + UNI(g.o_patch);
    const int kk = gk * gk, Wp = UNI(g.Wp), PR = UNI(g.PR), PRW = PR * Wp;
    const int HW = gH * gW, P = gOH * gOW;
    const int QC = UNI(g.QC), QCpad = UNI(g.QCpad), CC = UNI(g.CC), M = UNI(g.M), N = UNI(g.N), Q = UNI(g.Q);
    const int n_chunks = UNI(g.n_chunks), rows_c = UNI(g.rows_c);
    const int vec = UNI(g.vec);
    const int border = gk - 1 - gpad;

    // first row (of the output map for forward / backward weights, of the input
    // map for backward data) this tile touches; per-lane column offsets
    int tile_row0 = 0, c_lo = 0, adj;
    if (GM == 1) { tile_row0 = n0 / gOW; adj = tile_row0 * gs * Wp; }
    else if (GM == 2) { tile_row0 = n0 / gW; adj = tile_row0 * Wp; }
    else { c_lo = n0 / kk; adj = c_lo * PRW; }
    adj -= UNI(g.xoff);
    int offn[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + (wn_id * ni + j) * 16 + (lane & 15);
      offn[j] = (j < ni && n < N) ? tnb[n] - adj : 0;
    }
    __syncthreads();   // LDS may still be in use by the previous operand set
    for (int i = tid; i < QCpad; i += BLK) offq[i] = tq[i];
    const int patch_elems = CC * PRW;
    constexpr int SU = 8;
    const int p_c0 = tid / PRW, p_rem = tid - p_c0 * PRW, p_y0 = p_rem / Wp, p_x0 = p_rem - p_y0 * Wp;
    const int p_dc = BLK / PRW, p_r2 = BLK - p_dc * PRW, p_dy = p_r2 / Wp, p_dx = p_r2 - p_dy * Wp;
    // ---- A operand: lane (row i = lane%16, kq = lane/16) needs A[m][4*ks + kq] for
    // the k-steps ks = wk_id, wk_id + wk, ... of its wave.  Rows beyond M are
    // clamped (their results are never stored), so only the last, partial
    // k-step of a chunk needs a predicate.
    constexpr int KB = 8;
    int am = m0 + wm_id * 16 + (lane & 15);
    if (am >= M) am = M - 1;
    const int dq = 4 * wk, dq_co = dq / kk, dq_tap = dq - dq_co * kk;
    const gfloat* arow = Aglob + (GM == 2 ? (size_t)am * kk : (size_t)am * Q);
    const size_t co_stride = (size_t)gC * kk;

    for (int ch = 0; ch < n_chunks; ++ch) {
      const int q0 = ch * QC;
      const int qc_eff = (Q - q0 < QC) ? Q - q0 : QC;       // valid reduction entries in this chunk
      const int nfull = qc_eff >> 2;                        // k-steps in which all 4 lane groups are valid
      const int nk = (nfull > wk_id) ? (nfull - wk_id + wk - 1) / wk : 0;   // ... that belong to this wave
      int qr = 4 * wk_id + kq;
      int a_co = 0, a_tap = 0;
      if (GM == 2) { a_co = (q0 + qr) / kk; a_tap = q0 + qr - a_co * kk; }
      float a0[KB], a1[KB];
      auto load1 = [&]() -> float {
        const float v = (GM == 2) ? arow[a_co * co_stride + a_tap] : arow[q0 + qr];
        qr += dq;
        if (GM == 2) { a_tap += dq_tap; a_co += dq_co; if (a_tap >= kk) { a_tap -= kk; ++a_co; } }
        return v;
      };
      int issued = 0;                                       // k-steps of this wave whose A load has been issued
      if (nk >= KB) {
#pragma unroll
        for (int u = 0; u < KB; ++u) a0[u] = load1();
        issued = KB;
      } else {
#pragma unroll
        for (int u = 0; u < KB; ++u)
          if (u < nk) a1[u] = load1();
      }
      if (ch) __syncthreads();
      // ---- patch
      int chan0, row0;
      if (GM == 1) { chan0 = ch * CC; row0 = tile_row0 * gs - gpad; }
      else if (GM == 2) { chan0 = ch * CC; row0 = tile_row0; }
      else { chan0 = c_lo; row0 = ch * rows_c * gs - gpad; }
      if (vec) {
        // rows of the source map go to LDS with 16-byte copies; the interior of a
        // patch row starts at column 4, columns 0..3 and Wsrc+4..Wsrc+7 are halo
        typedef __attribute__((address_space(1))) v4f gv4;
        typedef __attribute__((address_space(3))) v4f lv4;
        const int Wsrc = (GM == 2) ? gOW : gW, Hsrc = (GM == 2) ? gOH : gH, Cred = (GM == 2) ? gK : gC;
        const int W4 = Wsrc >> 2, nrow = CC * PR, nslot = nrow * W4;
        const int rshift = (GM == 2) ? border : 0;
        constexpr int VU = 4;
        int r = tid / W4, xs = tid - r * W4;
        int c = r / PR, y = r - c * PR;
        const int dr = BLK / W4, dxs = BLK - dr * W4, dc = dr / PR, dy = dr - dc * PR;
        for (int base = tid; base < nslot; base += BLK * VU) {
          v4f v[VU];
          int dst[VU];
#pragma unroll
          for (int u = 0; u < VU; ++u) {
            v[u] = (v4f){0.f, 0.f, 0.f, 0.f};
            dst[u] = -1;
            if (base + u * BLK < nslot) {
              const int chn = chan0 + c, srow = row0 + y - rshift;
              dst[u] = c * PRW + y * Wp + 4 + 4 * xs;
              if (chn < Cred && srow >= 0 && srow < Hsrc)
                v[u] = *(const gv4*)(src + ((size_t)chn * Hsrc + srow) * Wsrc + 4 * xs);
            }
            xs += dxs; y += dy; c += dc;
            if (xs >= W4) { xs -= W4; ++y; }
            if (y >= PR) { y -= PR; ++c; }
            if (y >= PR) { y -= PR; ++c; }
          }
#pragma unroll
          for (int u = 0; u < VU; ++u)
            if (dst[u] >= 0) *(lv4*)(patch + dst[u]) = v[u];
        }
        for (int h = tid; h < 2 * nrow; h += BLK) {
          const int rr = h >> 1;
          *(lv4*)(patch + rr * Wp + ((h & 1) ? Wsrc + 4 : 0)) = (v4f){0.f, 0.f, 0.f, 0.f};
        }
      } else
      {
        int c = p_c0, y = p_y0, x = p_x0;
        for (int base = tid; base < patch_elems; base += BLK * SU) {
          float v[SU], sc[SU], sh[SU];
#pragma unroll
          for (int u = 0; u < SU; ++u) {
            v[u] = 0.f; sc[u] = 0.f; sh[u] = 0.f;     // sc = sh = 0: the zero padding
            if (base + u * BLK < patch_elems) {
              const int chn = chan0 + c;
              if (GM == 2) {
                // output gradient placed at stride spacing with a (k-1-pad) border
                const int ty = row0 + y - border, tx = x - border;
                if (chn < gK && ty >= 0 && tx >= 0 && ty % gs == 0 && tx % gs == 0) {
                  const int oh = ty / gs, ow = tx / gs;
                  if (oh < gOH && ow < gOW) v[u] = src[(size_t)chn * P + oh * gOW + ow];
                }
              } else {
                const int ih = row0 + y, iw = x - gpad;
                if (chn < gC && ih >= 0 && ih < gH && iw >= 0 && iw < gW) {
                  v[u] = src[(size_t)chn * HW + ih * gW + iw];
                  sc[u] = 1.f;
                  if (st) { sc[u] = st[2 * stG + chn]; sh[u] = st[2 * stG + stC + chn]; }
                }
              }
            }
            x += p_dx; y += p_dy; c += p_dc;
            if (x >= Wp) { x -= Wp; ++y; }
            if (y >= PR) { y -= PR; ++c; }
          }
#pragma unroll
          for (int u = 0; u < SU; ++u) {
            if (base + u * BLK < patch_elems) {
              float r = v[u];
              if (GM != 2) {
                r = fmaf(sc[u], r, sh[u]);
                if (relu) r = fmaxf(r, 0.f);
              }
              patch[base + u * BLK] = r;
            }
          }
        }
      }
      __syncthreads();
      // ---- MFMA loop: lane holds A[i = lane%16][k = lane/16] and B[k = lane/16][j = lane%16]
      const lint* oqp = offq + 4 * wk_id + kq;
      int done = 0;
      while (done + KB <= nk) {
        // a0 holds the A values of k-steps done..done+KB-1; fetch the next batch first
        const bool more = issued + KB <= nk;
        if (more) {
#pragma unroll
          for (int u = 0; u < KB; ++u) a1[u] = load1();
          issued += KB;
        }
#pragma unroll
        for (int u = 0; u < KB; ++u) {
          const int oq = oqp[(done + u) * dq];
#pragma unroll
          for (int j = 0; j < 4; ++j)
            if (j < ni) acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a0[u], patch[oq + offn[j]], acc[j], 0, 0, 0);
        }
        done += KB;
        if (more) {
#pragma unroll
          for (int u = 0; u < KB; ++u) a0[u] = a1[u];
        }
      }
      // remaining full k-steps of this wave (fewer than KB), then the chunk's partial k-step
      {
        const int rem = nk - done;
        if (nk >= KB) {
#pragma unroll
          for (int u = 0; u < KB; ++u)
            if (u < rem) a1[u] = load1();
        }
#pragma unroll
        for (int u = 0; u < KB; ++u)
          if (u < rem) {
            const int oq = oqp[(done + u) * dq];
#pragma unroll
            for (int j = 0; j < 4; ++j)
              if (j < ni) acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a1[u], patch[oq + offn[j]], acc[j], 0, 0, 0);
          }
      }
      if ((qc_eff & 3) && (nfull % wk) == wk_id) {
        const int qt = 4 * nfull + kq;
        float av = 0.f;
        if (qt < qc_eff) {
          if (GM == 2) { const int co = (q0 + qt) / kk; av = arow[co * co_stride + (q0 + qt - co * kk)]; }
          else av = arow[q0 + qt];
        }
        const int oq = offq[qt];
#pragma unroll
        for (int j = 0; j < 4; ++j)
          if (j < ni) acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, patch[oq + offn[j]], acc[j], 0, 0, 0);
      }
    }
  }

  // ---- reduce the split of the reduction across waves (fixed order)
  if (wk > 1) {
    __syncthreads();
    lfloat* red = smem;   // [wave][j][lane] float4
    if (wk_id > 0) {
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (j < ni) {
          lfloat* r = red + ((wv * 4 + j) * 64 + lane) * 4;
          r[0] = acc[j][0]; r[1] = acc[j][1]; r[2] = acc[j][2]; r[3] = acc[j][3];
        }
    }
    __syncthreads();
    if (wk_id == 0) {
      for (int w2 = 1; w2 < wk; ++w2)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          if (j < ni) {
            const lfloat* r = red + (((wv + w2) * 4 + j) * 64 + lane) * 4;
            acc[j][0] += r[0]; acc[j][1] += r[1]; acc[j][2] += r[2]; acc[j][3] += r[3];
          }
    }
  }
  if (wk_id != 0) return;
  // ---- epilogue: lane holds C[i = 4*(lane/16) + r][j = lane%16]
  const int M = UNI(d.g.M), N = UNI(d.g.N);
  gfloat* out = (GM == 1) ? at(d.y, t) : (GM == 2) ? at(d.dx, t) : GP(d.gw);
  const int mrow = m0 + wm_id * 16 + 4 * kq;
  const bool extras = (GM == 1 && (flags & (F_BIAS | F_SKIP))) || (GM == 2 && (flags & (F_MASK_X | F_ADD_SKG)));
  if (!extras) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + (wn_id * ni + j) * 16 + (lane & 15);
      if (j < ni && n < N) {
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (mrow + r < M) out[(size_t)(mrow + r) * N + n] = acc[j][r];
      }
    }
    return;
  }
  const gfloat* skip = (GM == 1 && (flags & F_SKIP) && !(flags & F_PROJ)) ? (const gfloat*)at(d.skip, t) : nullptr;
  const gfloat* xm = (GM == 2 && (flags & F_MASK_X)) ? (const gfloat*)at(d.x, t) : nullptr;
  const gfloat* skg = (GM == 2 && (flags & F_ADD_SKG)) ? (const gfloat*)at(d.skg, t) : nullptr;
  const gfloat* bias = (GM == 1 && (flags & F_BIAS)) ? GP(d.b) : nullptr;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int n = n0 + (wn_id * ni + j) * 16 + (lane & 15);
    if (j >= ni || n >= N) continue;
    float add[4], msk[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      add[r] = 0.f; msk[r] = 1.f;
      if (mrow + r < M) {
        const size_t o = (size_t)(mrow + r) * N + n;
        if (bias) add[r] = bias[mrow + r];
        if (skip) add[r] += skip[o];
        if (skg) add[r] = skg[o];
        if (xm) msk[r] = xm[o];
      }
    }
#pragma unroll
    for (int r = 0; r < 4; ++r)
      if (mrow + r < M) {
        float v = acc[j][r];
        if (GM == 2 && !(msk[r] > 0.f)) v = 0.f;
        out[(size_t)(mrow + r) * N + n] = v + add[r];
      }
  }
}

__device__ __forceinline__ void step_gemm(const LDesc& d, int tile, int t, lfloat* smem) {
  const int gm = UNI(d.g.gm);
  if (gm == 1) step_gemm_t<1>(d, tile, t, smem);
  else if (gm == 2) step_gemm_t<2>(d, tile, t, smem);
  else step_gemm_t<3>(d, tile, t, smem);
}

// db[co] = sum_p dZ[co,p], one wavefront per channel.
__device__ void step_bias_grad(const LDesc& d, int tile, int t) {
  const int co = tile * (BLK / 64) + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (co >= d.K) return;
  const int P = d.OH * d.OW;
  const gfloat* dz = at(d.dy, t) + (size_t)co * P;
  float s = 0.f;
  for (int p = lane; p < P; p += 64) s += dz[p];
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) s += __shfl_down(s, o, 64);
  if (lane == 0) GP(d.gb)[co] = s;
}

}  // namespace pb
