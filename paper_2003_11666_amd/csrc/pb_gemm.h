// MFMA implicit-GEMM core shared by the convolution / linear forward,
// backward-data and backward-weights steps (fp32, v_mfma_f32_16x16x4_f32).
//
// Every pass of a layer is C[M x N] += A[M x Q] * B[Q x N]:
//   forward           M = cout,  N = output pixels, q = (cin, kh, kw)
//   backward data     M = cin,   N = input pixels,  q = (cout, kh, kw)
//   backward weights  M = cout,  N = (cin, kh, kw), q = output pixels
// B is never materialised: B[q][n] = patch[offq(q) + offn(n)], where the patch
// is a zero-padded window of the (normalised, rectified) input -- or of the
// output gradient placed at stride spacing -- and offq / offn are separable
// offsets into it (tables built on the host).
//
// A batch-1 tile is a few hundred MFMAs, so what bounds it is the latency of
// memory, not its bandwidth and not the matrix cores: the data a tile reads
// was written by other workgroups one launch earlier and comes from beyond the
// L2.  Everything a chunk of the reduction needs -- the A block and the patch
// -- is therefore requested with coalesced loads that are all in flight
// together, parked in LDS, and only then contracted.
//
// Included by pb_kernels.hip after its address-space helpers.
#pragma once
#include "pb_device.h"

namespace pb {

template <int V> struct IConst { static constexpr int value = V; };
typedef float v4f __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(1))) v4f gv4;
typedef int v4i __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) v4i lvi4;
typedef float v2f __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(1))) v2f gv2;
typedef __attribute__((address_space(3))) v4f lv4;

// One tile of a K_GEMM step, GM = 1 forward, 2 backward data, 3 backward
// weights; NI = 16-column subtiles per wave.  A forward step may carry a second
// operand set (the 1x1 projection of the skip tensor) that accumulates into the
// same tile.
//
// LDS per chunk: offq[QCpad] | A block | patch.
//   A block, GM 1 and 3: MT rows of the chunk's reduction range, row stride LDA
//   A block, GM 2:       one segment of MT*k*k floats per output channel of the
//                        chunk -- the layout the weights have in memory
// Store of a step's bulk output.  What a phase writes is read by the next launch, from
// any XCD, so nothing is gained by keeping it in the writer's L2; lines left dirty there
// are written back when the kernel ends, which a short tick feels (ResNet-20: 1 us of 26).
// With the non-temporal hint they leave while the other workgroups still run.  Larger
// networks, whose parameters and activations are re-read from the caches, are quicker
// without it: nt is a compile-time constant of the kernel instantiation (k_phase<NT>).
// (The hinted store goes through an opaque copy of the address: otherwise the compiler
// may merge the two stores of the branch into one plain store.)
#define PB_ST(nt, p, v) do { if (nt) { auto q_ = (p); asm volatile("" : "+v"(q_)); __builtin_nontemporal_store((v), q_); } else *(p) = (v); } while (0)
// one MFMA, then up to three LDS reads and V other vector instructions, N times
template <int N, int V>
__device__ __forceinline__ void sched_interleave() {
#pragma unroll
  for (int i = 0; i < N; ++i) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    __builtin_amdgcn_sched_group_barrier(0x100, 3, 0);
    __builtin_amdgcn_sched_group_barrier(0x002, V, 0);
  }
}

template <int GM, int NI, bool NTK, int AU>
__device__ __forceinline__ void step_gemm_t(const LDesc& d, int tile_, int t, lfloat* smem) {
  constexpr bool nt = NTK;
  PB_TS(1);
  // an opaque copy of the tile index: what is derived from it is then worked out
  // inside this instantiation, not once ahead of all of them and kept in scratch
  // memory across the dispatch on (GM, NI)
  int tile = tile_;
  asm volatile("" : "+s"(tile));
  const int tid = threadIdx.x, lane = tid & 63, wv = UNI(tid >> 6);   // wave index: scalar
  const int wk = UNI(d.g.wk), wn = UNI(d.g.wn);
  constexpr int ni = NI;
  // wk, wn are powers of two (4 waves = wm x wn x wk)
  auto lg = [](int x) { return x == 1 ? 0 : (x == 2 ? 1 : 2); };
  const int wk_id = wv & (wk - 1), wn_id = (wv >> lg(wk)) & (wn - 1), wm_id = wv >> (lg(wk) + lg(wn));
  const int tiles_n = UNI(d.g.tiles_n);
  // backward weights, and the forward or backward-data pass of a thin layer whose consumer
  // adds the parts up: part of the reduction (a range of chunks) this workgroup takes
  // (forward and backward data are split only in networks tiled for throughput, which run the
  // kernel instantiation without the non-temporal hint: the other one carries no code for it)
  int qpart = 0;
  if (GM == 3 || !nt) {
    const int tpp = UNI(d.g.tpp);
    qpart = UNI(fdiv(tile, frcp(tpp)));
    tile -= qpart * tpp;
  }
  const int tm = UNI(fdiv(tile, frcp(tiles_n))), tn = tile - tm * tiles_n;
  const int MT = UNI(d.g.MT), NT = UNI(d.g.NT);
  // a workgroup runs nsub consecutive column tiles one after the other: the
  // descriptor and the offset table are fetched once, an A block that is a single
  // chunk stays in LDS, and the requests of the next column tile are in flight
  // while this one is contracted and stored
  // (several column tiles per workgroup and flattened 1x1 layers are planned only for networks
  // tiled for throughput: the instantiation for the others carries no code for them)
  const int nsub = nt ? 1 : UNI(d.g.nsub);
  const int m0 = tm * MT, n0 = tn * nsub * NT;
  const int flags = UNI(d.flags);
  const int kq = lane >> 4;
  // with one or two subtiles per wave consecutive MFMAs would wait for each other's
  // result: odd k-steps of the unrolled loop go to a second accumulator set
  constexpr bool DUAL = NI <= 2;
  v4f acc[NI], acc2[NI];
#pragma unroll
  for (int j = 0; j < NI; ++j) { acc[j] = (v4f){0.f, 0.f, 0.f, 0.f}; acc2[j] = (v4f){0.f, 0.f, 0.f, 0.f}; }
  // Operands of the epilogue (bias, skip tensor, ReLU mask source, skip-path gradient).  With
  // one or two column subtiles per wave they are few enough to be requested before the
  // contraction and kept in registers, so that the epilogue does not pay a memory round
  // trip of its own; with four subtiles they are requested in the epilogue.
  constexpr bool EARLY = NI <= 2 && GM != 3;
  float ea[EARLY ? NI : 1][4], em[EARLY ? NI : 1][4];
#pragma unroll
  for (int j = 0; j < (EARLY ? NI : 1); ++j)
#pragma unroll
    for (int r = 0; r < 4; ++r) { ea[j][r] = 0.f; em[j][r] = 1.f; }
  auto epi_operands = [&](int n0s, int tt, float (*add)[4], float (*msk)[4]) {
    const int M = UNI(d.g.M), N = UNI(d.g.N);
    const int mrow = m0 + wm_id * 16 + 4 * kq;
    const int ncol = n0s + wn_id * ni * 16 + (lane & 15);
    const gfloat* skip = (GM == 1 && (flags & F_SKIP) && !(flags & F_PROJ)) ? (const gfloat*)at(d.skip, tt) : nullptr;
    const gfloat* xm = (GM == 2 && (flags & F_MASK_X)) ? (const gfloat*)at(d.x, tt) : nullptr;
    const gfloat* skg = (GM == 2 && (flags & F_ADD_SKG)) ? (const gfloat*)at(d.skg, tt) : nullptr;
    const gfloat* bias = (GM == 1 && (flags & F_BIAS) && qpart == 0) ? GP(d.b) : nullptr;   // (a split forward pass: once)
    // straight-line loads from clamped positions (what lies beyond the matrix is never stored): with a branch per
    // element every load would wait for the one before it
    int o[NI][4];
#pragma unroll
    for (int j = 0; j < NI; ++j) {
      const int n = ncol + j * 16, nc = n < N ? n : N - 1;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int rr = mrow + r < M ? mrow + r : M - 1;
        o[j][r] = rr * N + nc;
        add[j][r] = 0.f; msk[j][r] = 1.f;
      }
    }
    if (bias) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float bv = bias[mrow + r < M ? mrow + r : M - 1];
#pragma unroll
        for (int j = 0; j < NI; ++j) add[j][r] = bv;
      }
    }
    if (skip) {
      float sv[NI][4];
#pragma unroll
      for (int j = 0; j < NI; ++j)
#pragma unroll
        for (int r = 0; r < 4; ++r) sv[j][r] = skip[o[j][r]];
#pragma unroll
      for (int j = 0; j < NI; ++j)
#pragma unroll
        for (int r = 0; r < 4; ++r) add[j][r] += sv[j][r];
    }
    if (skg) {
#pragma unroll
      for (int j = 0; j < NI; ++j)
#pragma unroll
        for (int r = 0; r < 4; ++r) add[j][r] = skg[o[j][r]];
    }
    if (xm) {
#pragma unroll
      for (int j = 0; j < NI; ++j)
#pragma unroll
        for (int r = 0; r < 4; ++r) msk[j][r] = xm[o[j][r]];
    }
  };
  const bool extras_any = (GM == 1 && (flags & (F_BIAS | F_SKIP))) || (GM == 2 && (flags & (F_MASK_X | F_ADD_SKG)));
  // sums of a tile: split of the reduction across waves, epilogue, store
  auto finish = [&](int n0s) {
    // the addresses the epilogue needs are worked out here, not before the
    // contraction: an opaque copy of the tick index keeps the compiler from
    // hoisting them to the top of the function, where they would have to be
    // kept (in scratch memory) across the MFMA loop
    int te = t;
    asm volatile("" : "+s"(te));
    if (DUAL) {
#pragma unroll
      for (int j = 0; j < NI; ++j) acc[j] += acc2[j];
    }
    PB_TS(7);
    // ---- reduce the split of the reduction across waves (fixed order)
    if (wk > 1) {
      __syncthreads();
      lfloat* red = smem;   // [wave][j][lane] float4
      if (wk_id > 0) {
#pragma unroll
        for (int j = 0; j < NI; ++j) *(lv4*)(red + ((wv * 4 + j) * 64 + lane) * 4) = acc[j];
      }
      __syncthreads();
      if (wk_id == 0) {
        for (int w2 = 1; w2 < wk; ++w2)
#pragma unroll
          for (int j = 0; j < NI; ++j) {
            const v4f r = *(const lv4*)(red + (((wv + w2) * 4 + j) * 64 + lane) * 4);
            acc[j][0] += r[0]; acc[j][1] += r[1]; acc[j][2] += r[2]; acc[j][3] += r[3];
          }
      }
    }
    PB_TS(8);
    if (wk_id != 0) return;
    // ---- epilogue: lane holds C[i = 4*(lane/16) + r][j = lane%16]
    const int M = UNI(d.g.M), N = UNI(d.g.N);
    gfloat* out = (GM == 3 || (!nt && UNI(d.g.parts) > 1)) ? GP(d.gw) + (size_t)qpart * (size_t)UNI(d.gpstride)
                  : (GM == 2) ? at(d.dx, te) : at(d.y, te);
    const int zero = te - t;                              // 0, opaque to the compiler (see above)
    const int mrow = m0 + wm_id * 16 + 4 * kq + zero;
    const int ncol = n0s + wn_id * ni * 16 + (lane & 15) + zero;
    int ro[4];                                            // element offset of the lane's four rows, -1 beyond M
#pragma unroll
    for (int r = 0; r < 4; ++r) ro[r] = (mrow + r < M) ? (mrow + r) * N : -1;
    const bool extras = (GM == 1 && (flags & (F_BIAS | F_SKIP))) || (GM == 2 && (flags & (F_MASK_X | F_ADD_SKG))) ||
                        (GM != 3 && (flags & F_BF16_OUT));
    if (!extras) {
#pragma unroll
      for (int j = 0; j < NI; ++j) {
        const int n = ncol + j * 16;
        if (n < N) {
#pragma unroll
          for (int r = 0; r < 4; ++r)
            if (ro[r] >= 0) PB_ST(nt, out + ro[r] + n, acc[j][r]);
        }
      }
      return;
    }
    // every operand of the epilogue is requested before the first one is used
    PB_TS(18);
    float add[NI][4], msk[NI][4];
    if (EARLY) {
#pragma unroll
      for (int j = 0; j < NI; ++j)
#pragma unroll
        for (int r = 0; r < 4; ++r) { add[j][r] = ea[EARLY ? j : 0][r]; msk[j][r] = em[EARLY ? j : 0][r]; }
    } else {
      epi_operands(n0s, te, add, msk);
    }
    PB_TS(19);
#pragma unroll
    for (int j = 0; j < NI; ++j) {
      const int n = ncol + j * 16;
      if (n >= N) continue;
#pragma unroll
      for (int r = 0; r < 4; ++r)
        if (ro[r] >= 0) {
          float v = acc[j][r];
          if (GM == 2 && !(msk[j][r] > 0.f)) v = 0.f;
          PB_ST(nt, out + ro[r] + n, rbf_if(GM != 3 && (flags & F_BF16_OUT), v + add[j][r]));
        }
      if (j == 0) PB_TS(21);
      if (j == 1) PB_TS(22);
      if (j == 2) PB_TS(23);
    }
    PB_TS(20);

  };
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
    lfloat* Alds = smem + UNI(g.o_A);
    lfloat* patch = smem + UNI(g.o_patch);
    const int kk = gk * gk, Wp = UNI(g.Wp), PR = UNI(g.PR), PRW = PR * Wp;
    const int HW = gH * gW, P = gOH * gOW;
    const int QC = UNI(g.QC), QCpad = UNI(g.QCpad), CC = UNI(g.CC), M = UNI(g.M), N = UNI(g.N), Q = UNI(g.Q);
    const int n_chunks = UNI(g.n_chunks), rows_c = UNI(g.rows_c), LDA = UNI(g.LDA);
    // chunks this workgroup contracts (all of them except for a split backward-weights step)
    const int ch0 = (GM == 3 || !nt) ? qpart * UNI(g.cpp) : 0;
    const int ch_end = ((GM == 3 || !nt) && ch0 + UNI(g.cpp) < n_chunks) ? ch0 + UNI(g.cpp) : n_chunks;
    const int nch = ch_end - ch0;
    const int vec = UNI(g.vec), avec = UNI(g.avec);
    const int border = gk - 1 - gpad;

    // first row (of the output map for forward / backward weights, of the input
    // map for backward data) the current column tile touches; per-lane column offsets
    int tile_row0 = 0, c_lo = 0, adj = 0, col0 = 0;
    const int win = (GM == 3 || nt) ? 0 : UNI(g.win);   // > 0: flattened 1x1 layer, the patch holds the tile's own columns only
    auto tile_geometry = [&](int n0s) {
      if (GM == 1) { tile_row0 = UNI(fdiv(n0s, frcp(gOW))); adj = tile_row0 * gs * Wp; }
      else if (GM == 2) { tile_row0 = UNI(fdiv(n0s, frcp(gW))); adj = tile_row0 * Wp; }
      else { c_lo = UNI(fdiv(n0s, frcp(kk))); adj = c_lo * PRW; }
      col0 = win ? n0s : 0;
      adj += col0 - UNI(g.xoff);
    };
    int tnv[NI], offn[NI];   // column offsets as the table has them, and relative to the patch of the column tile
    auto tn_load = [&](int n0s) {
#pragma unroll
      for (int j = 0; j < NI; ++j) {
        const int n = n0s + (wn_id * ni + j) * 16 + (lane & 15);
        tnv[j] = (n < N) ? tnb[n] : -1;
      }
    };
    tn_load(n0);
    if (!op) PB_TS(2);
    const int patch_elems = CC * PRW;
    const int mte = (M - m0 < MT) ? M - m0 : MT;        // rows of the tile that exist
    const size_t co_stride = (size_t)gC * kk;           // GM 2: floats between the weights of consecutive output channels
    const int i_row = wm_id * 16 + (lane & 15);
    const int lstride = (GM == 2) ? MT * kk : LDA;

    // ---- A block as a 2-D copy: nseg segments of seg_pad floats, of which the first
    // seg_len of the first nvalid segments come from memory and the rest is zero.
    // Requests (a_issue) and the stores into LDS (a_commit) are separate so that the
    // requests of chunk ch+1 can be in flight while chunk ch is contracted.
    const int av = avec ? 4 : 1;                          // floats per request
    struct APar { int nvalid, seg_len, spr, slots; float ispr; };
    auto a_par = [&](int ch) {
      const int q0 = ch * QC;
      // rows of the A block are zero beyond the chunk's reduction entries up to the next multiple
      // of 16 (forward, backward weights: the MFMA loop walks the reduction in blocks of 16) or of 4
      const int qe = (Q - q0 < QC) ? Q - q0 : QC, q4 = (GM == 2) ? (qe + 3) & ~3 : (qe + 15) & ~15;
      int nseg, seg_pad;
      APar p;
      if (GM == 2) {
        const float ikk = frcp(kk);
        nseg = UNI(fdiv(q4 + kk - 1, ikk)); p.nvalid = UNI(fdiv(qe, ikk)); p.seg_len = mte * kk; seg_pad = MT * kk;
      } else {
        nseg = MT; p.nvalid = MT; p.seg_len = qe; seg_pad = q4;
      }
      p.spr = avec ? (seg_pad + 3) >> 2 : seg_pad;        // requests per segment
      p.ispr = frcp(p.spr);
      p.slots = nseg * p.spr;
      return p;
    };
    auto a_src = [&](int ch, int r, int c) -> const gfloat* {
      if (GM == 2) return Aglob + (size_t)(ch * CC + r) * co_stride + (size_t)m0 * kk + c;
      int rr = m0 + r;
      if (rr >= M) rr = M - 1;                            // rows beyond M repeat the last one; never stored
      return Aglob + (size_t)rr * Q + ch * QC + c;
    };
    v4f ra[AU];
    auto a_issue = [&](int ch, int first_slot) {
      const APar p = a_par(ch);
      const int a_dr = UNI(fdiv(BLK, p.ispr)), a_dc = BLK - a_dr * p.spr;
      int r = fdiv(first_slot, p.ispr), c = first_slot - r * p.spr;
#pragma unroll
      for (int u = 0; u < AU; ++u) {
        ra[u] = (v4f){0.f, 0.f, 0.f, 0.f};
        if (first_slot + u * BLK < p.slots && r < p.nvalid && c * av < p.seg_len) {
          if (avec) ra[u] = *(const gv4*)a_src(ch, r, 4 * c);
          else ra[u][0] = *a_src(ch, r, c);
        }
        c += a_dc; r += a_dr;
        if (c >= p.spr) { c -= p.spr; ++r; }
      }
    };
    auto a_commit = [&](int ch, int first_slot) {
      const APar p = a_par(ch);
      const int a_dr = UNI(fdiv(BLK, p.ispr)), a_dc = BLK - a_dr * p.spr;
      int r = fdiv(first_slot, p.ispr), c = first_slot - r * p.spr;
#pragma unroll
      for (int u = 0; u < AU; ++u) {
        if (first_slot + u * BLK < p.slots) {
          if (avec) *(lv4*)(Alds + r * lstride + 4 * c) = ra[u];
          else Alds[r * lstride + c] = ra[u][0];
        }
        c += a_dc; r += a_dr;
        if (c >= p.spr) { c -= p.spr; ++r; }
      }
    };
    // ---- patch origin of a chunk: first channel and first source row
    auto p_origin = [&](int ch, int clo, int trow, int& chan0, int& row0) {
      if (GM == 1) { chan0 = ch * CC; row0 = trow * gs - gpad; }
      else if (GM == 2) { chan0 = ch * CC; row0 = trow; }
      else { chan0 = clo; row0 = ch * rows_c * gs - gpad; }
    };
    // ---- patch staged with 16-byte copies (vec == 1): rows of the source map go to
    // LDS as they are; the interior of a patch row starts at column 4, columns 0..3
    // and Wsrc+4..Wsrc+7 are halo.  Requests and stores separate, as for the A block.
    constexpr int VU = 6;
    const int Wsrc = (GM == 2) ? gOW : gW, Hsrc = (GM == 2) ? gOH : gH, Cred = (GM == 2) ? gK : gC;
    const int Wwin = win ? win : Wsrc;                    // columns of a source row that go into the patch
    const int W4 = Wwin >> 2, pv_nrow = CC * PR, pv_nslot = pv_nrow * W4;
    v4f pv[VU];
    int pdst[VU];
    auto p_issue = [&](int ch, int base, int clo, int trow, int pcol) {
      int chan0, row0;
      p_origin(ch, clo, trow, chan0, row0);
      const int rshift = (GM == 2) ? border : 0;
      const float iW4 = frcp(W4), iPR = frcp(PR);
      int r = fdiv(base, iW4), xs = base - r * W4;
      int c = fdiv(r, iPR), y = r - c * PR;
      const int dr = UNI(fdiv(BLK, iW4)), dxs = BLK - dr * W4, dc = UNI(fdiv(dr, iPR)), dy = dr - dc * PR;
#pragma unroll
      for (int u = 0; u < VU; ++u) {
        pv[u] = (v4f){0.f, 0.f, 0.f, 0.f};
        pdst[u] = -1;
        if (base + u * BLK < pv_nslot) {
          const int chn = chan0 + c, srow = row0 + y - rshift;
          pdst[u] = c * PRW + y * Wp + 4 + 4 * xs;
          if (chn < Cred && srow >= 0 && srow < Hsrc && pcol + 4 * xs < Wsrc)
            pv[u] = *(const gv4*)(src + ((size_t)chn * Hsrc + srow) * Wsrc + pcol + 4 * xs);
        }
        xs += dxs; y += dy; c += dc;
        if (xs >= W4) { xs -= W4; ++y; }
        if (y >= PR) { y -= PR; ++c; }
        if (y >= PR) { y -= PR; ++c; }
      }
    };
    auto p_commit = [&]() {
#pragma unroll
      for (int u = 0; u < VU; ++u)
        if (pdst[u] >= 0) *(lv4*)(patch + pdst[u]) = pv[u];
    };

    // ---- requests of the first chunk: offset table, A block, patch
    int tv[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) tv[u] = (tid + u * BLK < QCpad) ? tq[tid + u * BLK] : 0;
    a_issue(ch0, tid);
    if (!op) PB_TS(10);
    tile_geometry(n0);
    if (vec == 1) p_issue(ch0, tid, c_lo, tile_row0, col0);

    for (int sub = 0; sub < nsub; ++sub) {
    const int n0s = n0 + sub * NT;
    if (sub && n0s >= N) break;
    const bool more = sub + 1 < nsub && n0s + NT < N;   // another column tile follows
    tile_geometry(n0s);
    if (EARLY && !op && wk_id == 0 && extras_any) epi_operands(n0s, t, ea, em);
#pragma unroll
    for (int j = 0; j < NI; ++j) offn[j] = (tnv[j] >= 0) ? tnv[j] - adj : 0;
    __syncthreads();   // LDS may still be in use by the previous operand set / column tile
    if (!op && !sub) PB_TS(9);

    for (int ch = ch0; ch < ch_end; ++ch) {
      const int q0 = ch * QC;
      const int qc_eff = (Q - q0 < QC) ? Q - q0 : QC;       // valid reduction entries in this chunk
      const int qc4 = (qc_eff + 3) & ~3;
      if (ch != ch0) __syncthreads();                       // the previous chunk has been contracted
      if (ch == ch0 + 1 && !op) PB_TS(12);
      int chan0, row0;
      p_origin(ch, c_lo, tile_row0, chan0, row0);
      if (vec == 1) {
        p_commit();
        for (int base = tid + BLK * VU; base < pv_nslot; base += BLK * VU) { p_issue(ch, base, c_lo, tile_row0, col0); p_commit(); }
        for (int h = tid; h < 2 * pv_nrow; h += BLK) {
          const int rr = h >> 1;
          *(lv4*)(patch + rr * Wp + ((h & 1) ? Wwin + 4 : 0)) = (v4f){0.f, 0.f, 0.f, 0.f};
        }
      } else if (GM == 2 && vec == 3) {
        // layer of stride 2 (border 0 or 1, even gradient width, patch width a multiple
        // of 4): a 16-byte vector of a patch row holds two neighbouring gradient values
        // with zeros between them, or zeros only: one 8-byte request and one 16-byte
        // store per vector, no clearing pass.
        const int W4p = Wp >> 2, rows4 = PR * W4p, nslot = CC * rows4;
        constexpr int DU = 6;
        const float ir4 = frcp(rows4), iw4 = frcp(W4p);
        v2f v[DU];
        for (int base = tid; base < nslot; base += DU * BLK) {
#pragma unroll
          for (int u = 0; u < DU; ++u) {
            const int sl = base + u * BLK;
            v[u] = (v2f){0.f, 0.f};
            if (sl < nslot) {
              const int c = fdiv(sl, ir4), rem = sl - c * rows4, y = fdiv(rem, iw4), j = rem - y * W4p;
              const int chn = chan0 + c, ty = row0 + y - border, oh = ty >> 1;
              if (chn < gK && ty >= 0 && !(ty & 1) && oh < gOH && 2 * j < gOW)
                v[u] = *(const gv2*)(src + (size_t)chn * P + oh * gOW + 2 * j);
            }
          }
#pragma unroll
          for (int u = 0; u < DU; ++u) {
            const int sl = base + u * BLK;
            if (sl < nslot)
              *(lv4*)(patch + 4 * sl) = border ? (v4f){0.f, v[u][0], 0.f, v[u][1]} : (v4f){v[u][0], 0.f, v[u][1], 0.f};
          }
        }
      } else if (GM == 2 && vec == 2) {
        // strided layer: the output gradient sits at stride spacing inside a patch
        // of zeros.  Request its rows, clear the patch, then scatter them.
        const float igs = frcp(gs);
        const int nrow_src = UNI(fdiv(PR + gs - 1, igs)) + 1;   // source rows that can fall into the patch
        const int oh0 = (row0 - border + gs - 1 >= 0) ? UNI(fdiv(row0 - border + gs - 1, igs)) : 0;
        const int rowlen = nrow_src * gOW, nslot = CC * rowlen;
        constexpr int DU = 8;
        const float irl = frcp(rowlen), iow = frcp(gOW);
        int c = fdiv(tid, irl), rem = tid - c * rowlen, yr = fdiv(rem, iow), x = rem - yr * gOW;
        const int dc = UNI(fdiv(BLK, irl)), drem = BLK - dc * rowlen, dyr = UNI(fdiv(drem, iow)), dx = drem - dyr * gOW;
        float v[DU];
        int dst[DU];
        auto d_issue = [&](int first_slot) {
#pragma unroll
          for (int u = 0; u < DU; ++u) {
            dst[u] = -1; v[u] = 0.f;
            if (first_slot + u * BLK < nslot) {
              const int chn = chan0 + c, oh = oh0 + yr;
              const int py = oh * gs + border - row0, px = x * gs + border;
              if (chn < gK && oh < gOH && py >= 0 && py < PR) {
                dst[u] = c * PRW + py * Wp + px;
                v[u] = src[(size_t)chn * P + oh * gOW + x];
              }
            }
            x += dx; yr += dyr; c += dc;
            if (x >= gOW) { x -= gOW; ++yr; }
            if (yr >= nrow_src) { yr -= nrow_src; ++c; }
          }
        };
        auto d_commit = [&]() {
#pragma unroll
          for (int u = 0; u < DU; ++u)
            if (dst[u] >= 0) patch[dst[u]] = v[u];
        };
        d_issue(tid);
        for (int i = tid; i < ((patch_elems + 3) >> 2); i += BLK) *(lv4*)(patch + 4 * i) = (v4f){0.f, 0.f, 0.f, 0.f};
        __syncthreads();                                    // the patch has been cleared
        d_commit();
        for (int s0 = tid + DU * BLK; s0 < nslot; s0 += DU * BLK) { d_issue(s0); d_commit(); }
      } else {
        constexpr int SU = 8;
        const float iprw = frcp(PRW), iwp = frcp(Wp);
        int c = fdiv(tid, iprw), rem = tid - c * PRW, y = fdiv(rem, iwp), x = rem - y * Wp;
        const int p_dc = UNI(fdiv(BLK, iprw)), p_r2 = BLK - p_dc * PRW, p_dy = UNI(fdiv(p_r2, iwp)), p_dx = p_r2 - p_dy * Wp;
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
      if (ch == ch0 && !op) PB_TS(3);
      if (ch == ch0 + 1 && !op) PB_TS(14);
      // ---- park the offset table and the A block
      if (ch == ch0 && sub == 0) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
          if (tid + u * BLK < QCpad) offq[tid + u * BLK] = tv[u];
        for (int i = tid + 4 * BLK; i < QCpad; i += BLK) offq[i] = tq[i];
      }
      if (sub == 0 || nch > 1) {   // a single chunk's A block serves every column tile
        a_commit(ch, tid);
        const int a_slots = a_par(ch).slots;
        for (int s0 = tid + AU * BLK; s0 < a_slots; s0 += AU * BLK) { a_issue(ch, s0); a_commit(ch, s0); }
      }
      if (ch == ch0 && !op) PB_TS(4);
      if (ch == ch0 + 1 && !op) PB_TS(15);
      __syncthreads();
      if (ch == ch0 && !op) PB_TS(5);
      if (ch == ch0 + 1 && !op) PB_TS(16);
      // ---- requests of the next chunk (or of the first chunk of the next column
      // tile): in flight while this one is contracted
      if (ch + 1 < ch_end) {
        a_issue(ch + 1, tid);
        if (vec == 1) p_issue(ch + 1, tid, c_lo, tile_row0, col0);
      } else if (more) {
        if (nch > 1) a_issue(ch0, tid);
        if (vec == 1) {
          const int nn = n0s + NT;
          p_issue(ch0, tid, GM == 3 ? UNI(fdiv(nn, frcp(kk))) : 0,
                  GM == 1 ? UNI(fdiv(nn, frcp(gOW))) : (GM == 2 ? UNI(fdiv(nn, frcp(gW))) : 0), win ? nn : 0);
        }
        tn_load(n0s + NT);
      }
      if (ch == ch0 + 1 && !op) PB_TS(13);
      // ---- MFMA loop: lane holds A[i = lane%16][k = lane/16] and B[k = lane/16][j = lane%16];
      // the waves of a reduction split take k-steps wk_id, wk_id + wk, ...
      {
        // Forward and backward weights (K16): the reduction is walked in blocks of 16 entries;
        // in a block's four MFMAs lane group kq = lane / 16 supplies entries 4 kq .. 4 kq + 3, so
        // that its four A values and its four patch offsets are one 16-byte LDS read each.  The
        // waves of a reduction split take blocks wk_id, wk_id + wk, ...  Backward data (A block
        // in the weights' own layout): k-steps of 4 entries, lane group kq supplies entry kq.
        constexpr bool K16 = GM != 2;
        const int nsteps = K16 ? 4 * ((qc_eff + 15) >> 4) : qc4 >> 2;
        const int nunit = K16 ? nsteps >> 2 : nsteps;      // blocks / k-steps dealt out to the waves
        const int nmine = (nunit > wk_id) ? (nunit - wk_id + wk - 1) >> lg(wk) : 0;
        const int nk = K16 ? 4 * nmine : nmine;            // MFMA steps of this wave
        const int dq = K16 ? 16 * wk : 4 * wk;             // K16: advance per block; else per k-step
        const lint* oqp = offq + (K16 ? 16 * wk_id + 4 * kq : 4 * wk_id + kq);
        const lfloat* ap;
        int a_tap = 0, dq_co = 0, dq_tap = 0;
        if (GM == 2) {
          const float ikk = frcp(kk);
          const int q = 4 * wk_id + kq, co = fdiv(q, ikk);
          a_tap = q - co * kk;
          ap = Alds + co * lstride + i_row * kk + a_tap;
          dq_co = UNI(fdiv(dq, ikk)); dq_tap = dq - dq_co * kk;
        } else {
          ap = Alds + i_row * LDA + (K16 ? 16 * wk_id + 4 * kq : 4 * wk_id + kq);
        }
        const int a_adv = (GM == 2) ? dq_co * lstride + dq_tap : dq;
        const int a_wrap = (GM == 2) ? lstride - kk : 0;    // extra advance when the tap index wraps into the next channel
        // Software pipeline over groups of G k-steps: while the MFMAs of group g
        // run, the A and B values of group g+1 and the offsets of group g+2 (the
        // addresses of the B reads) are on their way from LDS.  Two cursors: the A
        // values, and the offset table one group ahead of them.  A load that would
        // run past the last group (live = false) re-reads the first entries instead
        // and leaves its cursor alone: the loop body has no branch around a load, so
        // that the wait before an MFMA counts the loads behind it exactly.  The
        // scheduling barriers keep the compiler from sinking reads to their first use.
        constexpr int G = 4;
        const int ng = nk / G;
        const lfloat* const ap0 = ap;
        const lint* const oqp0 = oqp;
        const int a_tap0 = a_tap;
        float av[2][G], bv[2][G][NI];
        int oqv[G];
        auto load_oq = [&](bool live) {
          const lint* p = live ? oqp : oqp0;
          const int st = live ? dq : 0;
          if (K16) {
            const v4i o = *(const lvi4*)p;
#pragma unroll
            for (int u = 0; u < G; ++u) oqv[u] = o[u];
            oqp += st;
          } else {
#pragma unroll
            for (int u = 0; u < G; ++u) { oqv[u] = *p; p += st; }
            oqp += G * st;
          }
        };
        auto load_ab = [&](auto NB, bool live) {
          constexpr int nb = decltype(NB)::value;
          const lfloat* p = live ? ap : ap0;
          int tap = live ? a_tap : a_tap0;
          const int adv = live ? a_adv : 0, dtap = live ? dq_tap : 0;
          if (K16) {
            const v4f a4 = *(const lv4*)p;
            p += adv;
#pragma unroll
            for (int u = 0; u < G; ++u) {
              av[nb][u] = a4[u];
#pragma unroll
              for (int j = 0; j < NI; ++j) bv[nb][u][j] = patch[oqv[u] + offn[j]];
            }
          } else {
#pragma unroll
          for (int u = 0; u < G; ++u) {
            av[nb][u] = *p;
            p += adv;
            if (GM == 2) { tap += dtap; if (tap >= kk) { tap -= kk; p += a_wrap; } }
#pragma unroll
            for (int j = 0; j < NI; ++j) bv[nb][u][j] = patch[oqv[u] + offn[j]];
          }
          }
          ap = live ? p : ap;
          a_tap = live ? tap : a_tap;
        };
        auto mfmas = [&](auto CB) {
          constexpr int cb = decltype(CB)::value;
#pragma unroll
          for (int u = 0; u < G; ++u)
#pragma unroll
            for (int j = 0; j < NI; ++j) {
              if (DUAL && (u & 1)) acc2[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[cb][u], bv[cb][u][j], acc2[j], 0, 0, 0);
              else acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[cb][u], bv[cb][u][j], acc[j], 0, 0, 0);
            }
        };
        using I0 = IConst<0>;
        using I1 = IConst<1>;
        int g = 0;
        if (ng > 0) {
          load_oq(true);
          load_ab(I0(), true);
          load_oq(ng > 1);
          for (; g + 2 <= ng; g += 2) {
            // One or two subtiles per wave: the reads of the next groups first, then the MFMAs.
            // Four subtiles: each of the 16 MFMAs is followed by a share of the LDS reads and of
            // the address arithmetic (measured: wide +0.8 %, ResNet-50 +1.5 %; with fewer
            // subtiles the plain order is as fast or faster).
            load_ab(I1(), true);
            load_oq(g + 2 < ng);
            if (NI < 4) __builtin_amdgcn_sched_barrier(0);
            mfmas(I0());
            if (NI == 4) sched_interleave<G * NI, (GM == 2 ? 8 : 3)>();
            __builtin_amdgcn_sched_barrier(0);
            load_ab(I0(), g + 2 < ng);
            load_oq(g + 3 < ng);
            if (NI < 4) __builtin_amdgcn_sched_barrier(0);
            mfmas(I1());
            if (NI == 4) sched_interleave<G * NI, (GM == 2 ? 8 : 3)>();
            __builtin_amdgcn_sched_barrier(0);
          }
          if (g < ng) mfmas(I0());   // odd number of groups: the last one is in buffer 0
        }
        for (int s = ng * G; s < nk; ++s) {
          const float a = *ap;
          const int oq = *oqp;
          ap += a_adv; oqp += dq;
          if (GM == 2) { a_tap += dq_tap; if (a_tap >= kk) { a_tap -= kk; ap += a_wrap; } }
#pragma unroll
          for (int j = 0; j < NI; ++j)
            acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, patch[oq + offn[j]], acc[j], 0, 0, 0);
        }
      }
      if (ch == ch0 && !op) PB_TS(6);
      if (ch == ch0 + 1 && !op) PB_TS(17);
    }
    if (nops == 1) {
      finish(n0s);
#pragma unroll
      for (int j = 0; j < NI; ++j) { acc[j] = (v4f){0.f, 0.f, 0.f, 0.f}; acc2[j] = (v4f){0.f, 0.f, 0.f, 0.f}; }
    }
    }   // column tiles
  }
  if (nops != 1) finish(n0);   // both operand sets have been accumulated (one column tile per workgroup)
}

}  // namespace pb
#include "pb_mm.h"
namespace pb {

template <bool NTK>
__device__ __forceinline__ void step_gemm(const LDesc& d, int tile, int t, lfloat* smem) {
  // the number of column subtiles per wave (1, 2 or 4) is a compile-time
  // constant so that the accumulators stay in fixed registers
  if (!NTK && UNI(d.g.mm)) { step_mm(d, tile, t, smem); return; }   // (planned only for networks tiled for throughput)
  const int gm = UNI(d.g.gm), ni = UNI(d.g.ni);
  if (gm == 1) {
    if (ni == 1) step_gemm_t<1, 1, NTK, (NTK ? 9 : 6)>(d, tile, t, smem);
    else if (ni == 2) step_gemm_t<1, 2, NTK, 6>(d, tile, t, smem);
    else step_gemm_t<1, 4, NTK, 6>(d, tile, t, smem);
  } else if (gm == 2) {
    if (ni == 1) step_gemm_t<2, 1, NTK, (NTK ? 9 : 6)>(d, tile, t, smem);
    else if (ni == 2) step_gemm_t<2, 2, NTK, 6>(d, tile, t, smem);
    else step_gemm_t<2, 4, NTK, 6>(d, tile, t, smem);
  } else {
    if (ni == 1) step_gemm_t<3, 1, NTK, 6>(d, tile, t, smem);
    else if (ni == 2) step_gemm_t<3, 2, NTK, 6>(d, tile, t, smem);
    else step_gemm_t<3, 4, NTK, 6>(d, tile, t, smem);
  }
}

// db[co] = sum_p dZ[co,p], one wavefront per channel.
__device__ __forceinline__ void step_bias_grad(const LDesc& d, int tile, int t) {
  const int co = tile * (BLK / 64) + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (co >= d.K) return;
  const int P = d.OH * d.OW;
  const gfloat* dz = at(d.dy, t) + (size_t)co * P;
  float s = 0.f;
  for (int p = lane; p < P; p += 64) s += dz[p];
  s = wave_sum(s);
  if (lane == 0) GP(d.gb)[co] = s;
}

}  // namespace pb
