// Dense matrix-product core for the 1x1 layers of networks tiled for
// throughput (fp32, v_mfma_f32_16x16x4_f32).
//
// A 1x1 layer of stride 1 on one sample is a plain matrix product over the flattened map:
//   forward           Y[K x P]  = W[K x C] * X[C x P]
//   backward data     dX[C x P] = W^T[C x K] * dY[K x P]
//   backward weights  gW[K x C] = dY[K x P] * X^T[P x C]
// with P pixels and all three matrices row-major in memory.  There is no patch
// and no offset table: the operands of a chunk of 32 reduction entries are
// copied into LDS as they are, and a wave keeps a register tile of MI x NI
// 16x16 accumulators (a workgroup of 2 x 2 waves: 32 MI rows, 32 NI columns),
// so that one LDS read feeds MI or NI MFMAs and an operand byte fetched from
// memory is used 32 MI (32 NI) times.  LDS holds two chunks: while chunk c is
// contracted from one half, the requests of chunk c + 1 are in flight and are
// stored into the other half at the end, one barrier per chunk.
//
// The k index of an MFMA is a free choice as long as both operands agree: in a
// block of 16 reduction entries, MFMA u (0..3) lets lane group kq = lane / 16
// supply entry 4 kq + u.  An operand whose rows run along the reduction (W
// forward, dY and X backward weights) then gives a lane its values for all four
// MFMAs of a block in one 16-byte LDS read.
//
// Operands that cannot be copied 16 bytes at a time -- maps whose pixel count
// is not a multiple of 4, the input of a projection of stride 2 -- are
// gathered element by element with the same tiles; the geometry is that of a
// general k x k layer (reduction or columns over (channel, tap)), which the
// planner uses for k > 1 only on request: a tap-by-tap gather fetches nine
// times what a patch in LDS serves once.
//
// Included by pb_gemm.h.
#pragma once
#include "pb_device.h"

namespace pb {

template <int MODE, int MI, int NI>
__device__ __forceinline__ void step_mm_t(const LDesc& d, int tile_, int t, lfloat* smem) {
  int tile = tile_;
  asm volatile("" : "+s"(tile));
  constexpr int MT = 32 * MI, NT = 32 * NI;
  constexpr int LDAT = MT + 4;       // backward data: A stored [reduction][row]
  constexpr int LDB = NT + 4;        // forward, backward data: B stored [reduction][column]; the four lane groups of a
                                     // wave read rows 4 apart: 4 LDB = 16 (mod 32) keeps them on different banks
  constexpr int A_FLOATS = MODE == 2 ? MM_QC * LDAT : MT * MM_LDK;
  constexpr int CHUNK = mm_chunk_floats(MODE, MT, NT);
  const int tid = threadIdx.x, lane = tid & 63, wv = UNI(tid >> 6);
  const int wr = wv >> 1, wc = wv & 1, li = lane & 15, kq = lane >> 4;
  const int M = UNI(d.g.M), N = UNI(d.g.N), Q = UNI(d.g.Q);
  const int flags = UNI(d.flags);
  const int tiles_n = UNI(d.g.tiles_n);
  int qpart = 0;
  if (MODE == 3) {
    const int tpp = UNI(d.g.tpp);
    qpart = UNI(fdiv(tile, frcp(tpp)));
    tile -= qpart * tpp;
  }
  const int tm = UNI(fdiv(tile, frcp(tiles_n))), tn = tile - tm * tiles_n;
  const int m0 = tm * MT, n0 = tn * NT;
  const int n_chunks = UNI(d.g.n_chunks);
  const int ch0 = MODE == 3 ? qpart * UNI(d.g.cpp) : 0;
  const int ch_end = (MODE == 3 && ch0 + UNI(d.g.cpp) < n_chunks) ? ch0 + UNI(d.g.cpp) : n_chunks;

  // operands in memory: Ag has lda floats per row, Bg ldb
  const gfloat* Ag = MODE == 3 ? (const gfloat*)at(d.dy, t) : GP(d.w);
  const gfloat* Bg = MODE == 2 ? (const gfloat*)at(d.dy, t) : (const gfloat*)at(d.x, t);
  // forward: A = W[M][Q] rows m0.., B = X[Q][N] columns n0..
  // backward data: A^T = W[Q][M] columns m0.., B = dY[Q][N] columns n0..
  // backward weights: A = dY[M][Q] rows m0.., B^T = X[N][Q] rows n0..
  // Pixel-indexed operands that cannot be fetched 16 bytes at a time (rows of 49 pixels; the input of a 1x1 layer of
  // stride 2, of which every second pixel of every second row takes part) are fetched element by element: dense pixel
  // p lies at poff(p) inside its channel's map, channels shw floats apart.
  const int gather = UNI(d.g.gather), ps = UNI(d.g.ps), pw = UNI(d.g.pw), sw = UNI(d.g.sw), shw = UNI(d.g.shw);
  const float ipw = frcp(pw);
  auto poff = [&](int p) {
    if (ps == 1) return p;
    const int oy = fdiv(p, ipw);
    return (oy * sw + (p - oy * pw)) * ps;
  };
  constexpr int AV = MT * MM_QC / 4 / BLK;     // 16-byte requests per thread and chunk: A
  constexpr int BV = NT * MM_QC / 4 / BLK;     //                                        B
  v4f ra[AV], rb[BV];
  // Convolution geometry of the gathered operands.  A k x k layer is the same product with the reduction (forward,
  // backward data) or the columns (backward weights) running over (channel, tap): the element for tap (kh, kw) and
  // pixel (y, x) of the step's pixel space lies at row ps y + dy, column ps x + dx of the source map (dy = kh - pad
  // forward and backward weights, pad - kh backward data), and is zero outside the map.
  const int ck = UNI(d.g.ck), kk = ck * ck, cpad = UNI(d.g.cpad), srcH = UNI(d.g.sh);
  const float ikk = frcp(kk), ick = frcp(ck);
  auto tap_of = [&](int q, int& c, int& dy, int& dx) {
    c = fdiv(q, ikk);
    const int tap = q - c * kk, kh = fdiv(tap, ick), kw = tap - kh * ck;
    dy = MODE == 2 ? cpad - kh : kh - cpad;
    dx = MODE == 2 ? cpad - kw : kw - cpad;
  };
  auto pix_of = [&](int p, int& y, int& x) {
    y = fdiv(p, ipw);
    x = (p - y * pw) * ps;
    y *= ps;
  };
  // (a load from a clamped position and a select: no branch between two loads)
  auto src_at = [&](const gfloat* base, int c, int y, int x, bool ok) -> float {
    const bool in = ok && y >= 0 && y < srcH && x >= 0 && x < sw;
    const float v = base[(unsigned)(in ? c * shw + y * sw + x : 0)];   // (unsigned: a 32-bit offset from a scalar base)
    return in ? v : 0.f;
  };
  // Gathered operands are dealt out so that the lanes of a wavefront read neighbouring addresses (a request that
  // touches 64 scattered lines costs the memory pipeline many times one that touches two): element i of a thread is
  // entry tid + 256 i of the operand's chunk in its LDS order, [reduction][column] (forward, backward data) or
  // [row][reduction] (backward weights), so a thread keeps one column (one reduction entry) for all its elements.
  const bool a_gather = MODE == 3 && (Q & 3) != 0;       // rows of dY that cannot be fetched 16 bytes at a time
  int gy = 0, gx = 0;
  bool gok = false;
  if (gather && MODE != 3) {
    const int p = n0 + tid % NT;
    gok = p < N;
    pix_of(gok ? p : 0, gy, gx);
  }
  auto issue_gather = [&](int ch) {
    const int q0 = ch * MM_QC;
    if (a_gather) {
#pragma unroll
      for (int i = 0; i < 4 * AV; ++i) {
        const int idx = tid + i * BLK, r = idx >> 5, p = q0 + (idx & 31), pc = p < Q ? p : Q - 1;
        const float x = Ag[(unsigned)((m0 + r) * Q + pc)];
        ra[i >> 2][i & 3] = p < Q ? x : 0.f;
      }
    } else {
#pragma unroll
      for (int u = 0; u < AV; ++u) {
        const int v = tid + u * BLK;
        if (MODE == 2) {
          const int q = v / (MT / 4), c4 = v % (MT / 4);
          ra[u] = *(const gv4*)(Ag + (size_t)(q0 + q) * M + m0 + 4 * c4);
        } else {
          const int r = v >> 3, c4 = v & 7;
          ra[u] = (v4f){0.f, 0.f, 0.f, 0.f};
          if (q0 + 4 * c4 < Q) ra[u] = *(const gv4*)(Ag + (size_t)(m0 + r) * Q + q0 + 4 * c4);
        }
      }
    }
    if (MODE == 3) {
      const int p = q0 + (tid & 31);
      int y, x;
      pix_of(p < Q ? p : 0, y, x);
      // (an opaque copy of the first column: its rows' taps are worked out again for every chunk instead of being
      // kept, 48 registers of them, across the whole contraction)
      int nb = n0;
      asm volatile("" : "+v"(nb));
#pragma unroll
      for (int i = 0; i < 4 * BV; ++i) {
        const int r = (tid >> 5) + i * (BLK / 32);
        int c, dy, dx;
        tap_of(nb + r, c, dy, dx);
        rb[i >> 2][i & 3] = src_at(Bg, c, y + dy, x + dx, p < Q);
      }
    } else if (MODE == 2) {
      // (a 1x1 layer: the gradient as it lies, also for stride 2, where the product runs over the output pixels)
      const int p = n0 + tid % NT, pc = p < N ? p : N - 1;
#pragma unroll
      for (int i = 0; i < 4 * BV; ++i) {
        const int q = tid / NT + i * (BLK / NT);
        const float x = Bg[(unsigned)((q0 + q) * N + pc)];
        rb[i >> 2][i & 3] = p < N ? x : 0.f;
      }
    } else {
#pragma unroll
      for (int i = 0; i < 4 * BV; ++i) {
        const int q = tid / NT + i * (BLK / NT);
        int c, dy, dx;
        tap_of(q0 + q, c, dy, dx);
        rb[i >> 2][i & 3] = src_at(Bg, c, gy + dy, gx + dx, gok);
      }
    }
  };
  auto issue = [&](int ch) {
    if (gather) { issue_gather(ch); return; }
    const int q0 = ch * MM_QC;
#pragma unroll
    for (int u = 0; u < AV; ++u) {
      const int v = tid + u * BLK;
      ra[u] = (v4f){0.f, 0.f, 0.f, 0.f};
      if (MODE == 2) {
        const int q = v / (MT / 4), c4 = v % (MT / 4);               // row q of W, columns m0 + 4 c4
        ra[u] = *(const gv4*)(Ag + (size_t)(q0 + q) * M + m0 + 4 * c4);
      } else {
        const int r = v >> 3, c4 = v & 7;                            // row m0 + r, reduction entries q0 + 4 c4
        if (q0 + 4 * c4 < Q) ra[u] = *(const gv4*)(Ag + (size_t)(m0 + r) * Q + q0 + 4 * c4);
      }
    }
#pragma unroll
    for (int u = 0; u < BV; ++u) {
      const int v = tid + u * BLK;
      rb[u] = (v4f){0.f, 0.f, 0.f, 0.f};
      if (MODE == 3) {
        const int r = v >> 3, c4 = v & 7;
        if (q0 + 4 * c4 < Q) rb[u] = *(const gv4*)(Bg + (size_t)(n0 + r) * Q + q0 + 4 * c4);
      } else {
        const int q = v / (NT / 4), c4 = v % (NT / 4);
        if (n0 + 4 * c4 < N) rb[u] = *(const gv4*)(Bg + (size_t)(q0 + q) * N + n0 + 4 * c4);
      }
    }
  };
  auto commit = [&](lfloat* buf) {
    lfloat* Al = buf;
    lfloat* Bl = buf + A_FLOATS;
    if (a_gather) {
#pragma unroll
      for (int i = 0; i < 4 * AV; ++i) {
        const int idx = tid + i * BLK;
        Al[(idx >> 5) * MM_LDK + (idx & 31)] = ra[i >> 2][i & 3];
      }
    } else {
#pragma unroll
      for (int u = 0; u < AV; ++u) {
        const int v = tid + u * BLK;
        if (MODE == 2) *(lv4*)(Al + (v / (MT / 4)) * LDAT + 4 * (v % (MT / 4))) = ra[u];
        else *(lv4*)(Al + (v >> 3) * MM_LDK + 4 * (v & 7)) = ra[u];
      }
    }
    if (gather) {
#pragma unroll
      for (int i = 0; i < 4 * BV; ++i) {
        const int idx = tid + i * BLK;
        if (MODE == 3) Bl[(idx >> 5) * MM_LDK + (idx & 31)] = rb[i >> 2][i & 3];
        else Bl[(idx / NT) * LDB + idx % NT] = rb[i >> 2][i & 3];
      }
    } else {
#pragma unroll
      for (int u = 0; u < BV; ++u) {
        const int v = tid + u * BLK;
        if (MODE == 3) *(lv4*)(Bl + (v >> 3) * MM_LDK + 4 * (v & 7)) = rb[u];
        else *(lv4*)(Bl + (v / (NT / 4)) * LDB + 4 * (v % (NT / 4))) = rb[u];
      }
    }
  };

  v4f acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j) acc[i][j] = (v4f){0.f, 0.f, 0.f, 0.f};

  issue(ch0);
  __syncthreads();                       // (the descriptor's LDS neighbours: nothing of an earlier step is live)
  commit(smem);
  __syncthreads();
  for (int ch = ch0; ch < ch_end; ++ch) {
    lfloat* cur = smem + ((ch - ch0) & 1) * CHUNK;
    lfloat* nxt = smem + (((ch - ch0) & 1) ^ 1) * CHUNK;
    const bool more = ch + 1 < ch_end;
    if (more) issue(ch + 1);
    const lfloat* Al = cur;
    const lfloat* Bl = cur + A_FLOATS;
    // lane's operand addresses for block 0 of the chunk
    const lfloat* ap = MODE == 2 ? Al + (4 * kq) * LDAT + wr * 16 * MI + li : Al + (wr * 16 * MI + li) * MM_LDK + 4 * kq;
    const lfloat* bp = MODE == 3 ? Bl + (wc * 16 * NI + li) * MM_LDK + 4 * kq : Bl + (4 * kq) * LDB + wc * 16 * NI + li;
    v4f a[2][MI], b[2][NI];
    auto fetch = [&](auto SB, int blk) {
      constexpr int sb = decltype(SB)::value;
#pragma unroll
      for (int i = 0; i < MI; ++i) {
        if (MODE == 2) {
#pragma unroll
          for (int u = 0; u < 4; ++u) a[sb][i][u] = ap[(16 * blk + u) * LDAT + 16 * i];
        } else {
          a[sb][i] = *(const lv4*)(ap + 16 * i * MM_LDK + 16 * blk);
        }
      }
#pragma unroll
      for (int j = 0; j < NI; ++j) {
        if (MODE == 3) {
          b[sb][j] = *(const lv4*)(bp + 16 * j * MM_LDK + 16 * blk);
        } else {
#pragma unroll
          for (int u = 0; u < 4; ++u) b[sb][j][u] = bp[(16 * blk + u) * LDB + 16 * j];
        }
      }
    };
    auto mfmas = [&](auto SB) {
      constexpr int sb = decltype(SB)::value;
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
          for (int j = 0; j < NI; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[sb][i][u], b[sb][j][u], acc[i][j], 0, 0, 0);
    };
    // the second block's operands come from LDS while the first block's MFMAs run (each MFMA is followed by a share
    // of the reads)
    fetch(IConst<0>(), 0);
    __builtin_amdgcn_sched_barrier(0);
    fetch(IConst<1>(), 1);
    mfmas(IConst<0>());
    sched_interleave<4 * MI * NI, 0>();
    __builtin_amdgcn_sched_barrier(0);
    mfmas(IConst<1>());
    __builtin_amdgcn_sched_barrier(0);
    if (more) commit(nxt);
    __syncthreads();
  }

  // ---- epilogue: lane holds C[4 kq + r][li] of each 16x16 subtile
  int te = t;
  asm volatile("" : "+s"(te));
  gfloat* out = MODE == 3 ? GP(d.gw) + (size_t)qpart * (size_t)UNI(d.gpstride) : MODE == 2 ? at(d.dx, te) : at(d.y, te);
  const gfloat* skip = (MODE == 1 && (flags & F_SKIP)) ? (const gfloat*)at(d.skip, te) : nullptr;
  const gfloat* bias = (MODE == 1 && (flags & F_BIAS)) ? GP(d.b) : nullptr;
  const gfloat* xm = (MODE == 2 && (flags & F_MASK_X)) ? (const gfloat*)at(d.x, te) : nullptr;
  const gfloat* skg = (MODE == 2 && (flags & F_ADD_SKG)) ? (const gfloat*)at(d.skg, te) : nullptr;
  const bool round = MODE != 3 && (flags & F_BF16_OUT);
  // every operand of the epilogue is requested before the first one is used (the registers of the
  // contraction's operands are free by now): one memory round trip for the whole tile
  float add[MI][NI][4], msk[MI][NI][4];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int r = 0; r < 4; ++r) { add[i][j][r] = 0.f; msk[i][j][r] = 1.f; }
  // (straight-line loads from clamped addresses: a branch per element would make every load wait for the one before)
  auto epi_fetch = [&](const gfloat* src, float (&dst)[MI][NI][4]) {
#pragma unroll
    for (int i = 0; i < MI; ++i) {
      const int row = m0 + wr * 16 * MI + 16 * i + 4 * kq;
#pragma unroll
      for (int j = 0; j < NI; ++j) {
        const int col = n0 + wc * 16 * NI + 16 * j + li;
        const int cc = col < N ? col : N - 1;
#pragma unroll
        for (int r = 0; r < 4; ++r) dst[i][j][r] = src[(size_t)(row + r) * N + cc];
      }
    }
  };
  if (MODE == 1 && skip) epi_fetch(skip, add);
  if (MODE == 2 && skg) epi_fetch(skg, add);
  if (MODE == 2 && xm) epi_fetch(xm, msk);
  if (MODE == 1 && bias) {
#pragma unroll
    for (int i = 0; i < MI; ++i) {
      float bv[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) bv[r] = bias[m0 + wr * 16 * MI + 16 * i + 4 * kq + r];
#pragma unroll
      for (int j = 0; j < NI; ++j)
#pragma unroll
        for (int r = 0; r < 4; ++r) add[i][j][r] += bv[r];
    }
  }
#pragma unroll
  for (int i = 0; i < MI; ++i) {
    const int row = m0 + wr * 16 * MI + 16 * i + 4 * kq;
#pragma unroll
    for (int j = 0; j < NI; ++j) {
      const int col = n0 + wc * 16 * NI + 16 * j + li;
      if (col >= N) continue;
      if (MODE == 2 && ps == 2) {
        // backward data of a layer of stride 2: the gradient of dense pixel (oy, ox) belongs to input pixel (2 oy, 2 ox);
        // its three neighbours in the 2 x 2 block took no part in the forward pass
        const int o = poff(col);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          gfloat* q = out + (size_t)(row + r) * shw + o;
          *(gv2*)q = (v2f){rbf_if(round, acc[i][j][r]), 0.f};
          *(gv2*)(q + sw) = (v2f){0.f, 0.f};
        }
        continue;
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        float v = acc[i][j][r];
        if (MODE == 2 && !(msk[i][j][r] > 0.f)) v = 0.f;
        out[(size_t)(row + r) * N + col] = rbf_if(round, v + add[i][j][r]);
      }
    }
  }
}

__device__ __forceinline__ void step_mm(const LDesc& d, int tile, int t, lfloat* smem) {
  // forward and backward data: tiles of 128 x 128, 64 x 128 (layers of 64 channels) or 128 x 64 (maps of at most 64 pixels)
  const int gm = UNI(d.g.gm), mi = UNI(d.g.mi), ni = UNI(d.g.ni);
  if (gm == 1) {
    if (mi == 4 && ni == 4) step_mm_t<1, 4, 4>(d, tile, t, smem);
    else if (mi == 4) step_mm_t<1, 4, 2>(d, tile, t, smem);
    else step_mm_t<1, 2, 4>(d, tile, t, smem);
  } else if (gm == 2) {
    if (mi == 4 && ni == 4) step_mm_t<2, 4, 4>(d, tile, t, smem);
    else if (mi == 4) step_mm_t<2, 4, 2>(d, tile, t, smem);
    else step_mm_t<2, 2, 4>(d, tile, t, smem);
  } else {
    if (mi == 4 && ni == 4) step_mm_t<3, 4, 4>(d, tile, t, smem);
    else if (mi == 4) step_mm_t<3, 4, 2>(d, tile, t, smem);
    else if (ni == 4) step_mm_t<3, 2, 4>(d, tile, t, smem);
    else step_mm_t<3, 2, 2>(d, tile, t, smem);
  }
}

}  // namespace pb
