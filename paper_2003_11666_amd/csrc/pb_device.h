// Shared between the host runtime and the kernels of the PB tick engine:
// the step table that describes, once at pb_init, every piece of work a
// pipeline tick consists of.  Plain data only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pb {

constexpr int BLK = 256;          // threads per workgroup (4 wavefronts of 64)
constexpr int UPD_CHUNK = 1024;   // stages are padded to this many floats
constexpr int UPD_TILE = 8192;    // floats per workgroup of an update step (8 float4 per thread and array in flight)
constexpr float GN_EPS = 1e-5f;
constexpr int GNB_WAVE_CH = 4;    // channels per wavefront in the one-wavefront-per-channel form of K_GNB_REDUCE

// A tensor that lives in a ring of `depth` slots.  At tick t the slot in use
// is (t - lag) mod depth: lag 0 = the slot of the sample handled now, lag D =
// the sample whose forward pass ran D ticks ago, lag -1 = the slot the next
// tick will read.  depth 1 = plain buffer.
struct TRef {
  float* base;
  int32_t depth;
  int32_t stride;   // floats per slot
  int32_t lag;
  int32_t pad_;
};

enum StepKind : int32_t {
  K_GN_STATS = 0,    // group mean / rstd and per-channel scale, shift
  K_GAP_FWD = 1,     // mean over H*W of relu(affine(x))
  K_CONV_FWD = 2,    // convolution / linear forward with fused input transform and skip add
  K_POST_FWD = 3,    // relu(affine(z)) [+ max-pool]
  K_CE = 4,          // softmax cross-entropy + dlogits
  K_GNB_REDUCE = 5,  // GroupNorm backward: per-channel sums (dgamma, dbeta)
  K_GNB_APPLY = 6,   // GroupNorm backward: elementwise dx
  K_CONV_BWD_X = 7,  // backward data
  K_CONV_BWD_W = 8,  // backward weights (+ bias)
  K_COPY = 9,
  K_GEMM = 10,       // conv / linear forward, backward data or backward weights as an MFMA implicit GEMM
  K_BIAS_GRAD = 11,  // db[co] = sum_p dZ[co,p]
  K_INGEST = 12,     // the tick's sample and label into the first stage's ring
  K_UPDATE = 13,     // fused SC+LWP update of one stage's parameter block (reads one copy of w, v; writes the other)
  K_HEAD = 14,       // whole last stage (forward, loss, backward) in one workgroup
  K_GN_BWD = 15,     // GroupNorm backward of one group in one workgroup: channel sums and dx together
  K_DOT_FWD = 16,    // forward of a 3x3 layer (stride 1, padding 1) on a 2x2 or 4x4 map as dot products: d.n output
                     // channels per workgroup, the weights streamed once, no MFMA, no LDS tiles
  K_DOT_BWD_X = 17,  // backward data of such a layer: 64 input channels per workgroup and a d.n-th of the output
                     // channels (d.gparts parts, summed by the consumer of the gradient when there are several)
  // A dense layer on one sample is a matrix-vector product (networks tiled for throughput, input length a multiple
  // of 4): nothing for the matrix cores, a stream of the weight matrix.
  K_FC_FWD = 18,     // y = W x + b: a wavefront per output, four outputs per workgroup
  K_FC_BWD_X = 19,   // dx = W^T dy: 64 inputs per workgroup, the outputs dealt out to 16 groups of 16 lanes
  K_FC_BWD_W = 20    // gW = dy x^T: 4096 consecutive weights per workgroup
};

constexpr int LDS_FLOATS = 19456;   // 76 KB of LDS per workgroup (a compute unit has 160 KB and holds two workgroups); the
                                    // planner gives GEMM tiles all of it or 62 KB (pb_tuning.gemm_lds_kb)

// Tiling of one implicit-GEMM operand set: C[M x N] += A[M x Q] * B[Q x N] with
// B[q][n] = patch[offq(q) + offn(n)], the patch being a zero-padded window of
// the activation (or of the dilated output gradient) staged in LDS.
struct GemmCfg {
  int32_t gm;             // 0 = none, 1 = forward, 2 = backward data, 3 = backward weights
  int32_t M, N, Q;
  int32_t wm, wn, wk, ni; // 4 waves = wm x wn x wk (split of the reduction); ni 16-column subtiles per wave
  int32_t MT, NT, tiles_n, tiles;
  int32_t QC;             // reduction elements per chunk
  int32_t QCpad;          // rounded up to a multiple of 16
  int32_t CC;             // channels per patch
  int32_t rows_c;         // backward weights: output rows per chunk
  int32_t PR, Wp;         // patch rows / width
  int32_t avec;           // 1: the A block is fetched with 16-byte loads (segments 16-byte aligned, lengths multiples of 4)
  int32_t o_offq, o_patch;   // LDS offsets (floats)
  int32_t n_chunks;
  int32_t LDA, o_A;        // row stride of the A block in LDS (forward, backward weights) and its LDS offset
  int32_t vec;             // 1: patch rows are staged with 16-byte copies (source rows a multiple of 4 wide, no transform);
                           // 2: backward data of a strided layer: patch cleared, then the gradient scattered into it
  int32_t xoff;            // LDS column of logical patch column 0
  int32_t nsub;            // consecutive column tiles one workgroup runs (tiles_n counts groups of nsub)
  int32_t win;             // > 0: 1x1 layer seen as a plain matrix product (map flattened to one row of H*W pixels):
                           // the patch holds only the win = NT columns of the current column tile
  int32_t parts;           // backward weights: the reduction is split over `parts` groups of workgroups, each taking
  int32_t cpp;             // cpp consecutive chunks and writing a partial gradient of its own (summed by the update step);
  int32_t tpp;             // tiles per part (tiles = parts * tpp)
  int32_t mm;              // 1: dense matrix-product form of a 1x1 layer of stride 1 (no patch, no offset tables): a workgroup of
  int32_t mi;              // 2 x 2 waves, each with mi x ni accumulators (tile 32 mi x 32 ni), chunks of 32 reduction entries
  int32_t gather;          // dense form: pixel-indexed operands are fetched element by element (rows not a multiple of 4 pixels,
  int32_t ps, pw;          // or a layer of stride ps = 2): dense pixel p = (oy, ox) of a pw-wide map lies at ps (oy sw + ox) in its
  int32_t sw, shw;         // channel's map, whose rows are sw floats and whose channels are shw floats apart
  int32_t ck, cpad, sh;    // dense form of a k x k layer (ck = k, its padding, rows of the source map): the reduction or the
                           // columns run over (channel, tap), see pb_mm.h
  int32_t a_req;           // requests per thread that the A block of a full chunk takes (the kernel built for latency keeps
                           // nine of them in flight when there are more than six, six otherwise)
};

// Dense matrix-product form of a 1x1 layer (GemmCfg::mm)
constexpr int MM_QC = 32;            // reduction entries per chunk
constexpr int MM_LDK = MM_QC + 4;    // row stride of an operand stored [row][reduction]: 4 * odd, 16 rows on distinct banks

// LDS floats of one chunk (both operands); the step needs twice that
__host__ __device__ constexpr int mm_chunk_floats(int mode, int MT, int NT) {
  return (mode == 2 ? MM_QC * (MT + 4) : MT * MM_LDK) + (mode == 3 ? NT * MM_LDK : MM_QC * (NT + 4));
}

// Pointer fields of a step that point into slot 0 of the stage's ring of predicted-weight versions;
// k_phase moves them to the slot of the tick before the step runs.
enum ParamField : int32_t { PF_W = 1, PF_B = 2, PF_WP = 4, PF_GAMMA = 8, PF_BETA = 16, PF_WHAT = 32, PF_SKIPBASE = 64 };

enum StepFlags : int32_t {
  F_PRE_AFFINE = 1,   // input is sc[c]*x + sh[c] (GroupNorm folded into the load)
  F_PRE_RELU = 2,     // then max(.,0)
  F_BIAS = 4,
  F_SKIP = 8,         // epilogue adds the skip tensor
  F_PROJ = 16,        // ... through a 1x1 projection
  F_POOL = 32,        // max-pool after relu(affine(z))
  F_DU_BUF = 64,      // GN backward: incoming gradient is a plain buffer
  F_DU_GAP = 128,     // ... is dpooled[c] / (H*W)
  F_DU_POOL = 256,    // ... is dY routed through the max-pool
  F_ADD_SKG = 512,    // epilogue adds the skip-path gradient
  F_MASK_X = 1024,    // backward data: multiply by [x > 0] (ReLU directly on the stage input)
  F_GN_RELU = 2048,   // GN backward: a ReLU follows the normalisation
  F_UPD_GN = 4096,    // K_GN_BWD also applies the update of the GroupNorm scale / shift it has the gradients of
  F_ALWAYS = 8192,    // the step runs before its first_tick too (then it only carries parameters over)
  F_BF16_OUT = 16384, // the step's output crosses a stage boundary in bf16 mode: round it to bf16 (nearest even)
  F_LWP_W = 32768,    // update: weight-difference form of the prediction, w_hat = w' + T (w' - w); flrT then holds T
  F_NT = 65536,       // K_UPDATE, in a kernel built for non-temporal output stores: this step uses them too
  F_WGRAD = 131072    // K_UPDATE of a 3x3 layer on a 2x2 or 4x4 map: the weight gradient is not read from memory but
                      // computed inside the step from the layer's saved input (x) and output gradient (dy)
};

struct StepDesc {
  int32_t kind, stage, first_tick, ntiles;
  int32_t tile;             // per-workgroup records: which tile of the step this workgroup runs
  int32_t flags;
  int32_t C, H, W;          // input tensor of the op
  int32_t K, OH, OW;        // output tensor of the op
  int32_t k, stride, pad;
  int32_t G;                // GroupNorm groups
  int32_t pk, ps, pp, PH, PW;   // max-pool window / stride / pad / output size
  int32_t sC, sH, sW, sstride;  // skip tensor dims and projection stride
  int32_t n;                // generic element count (CE: classes, COPY: floats)
  int32_t loss_cap, n_stages;
  float fa, fb, flrT, flr, fm;   // K_UPDATE: SC coefficients a, b, lr*T, lr, momentum
  int32_t pmask;            // which pointer fields address the stage's ring of predicted weights (PF_* bits)
  int32_t pdepth, plag, pstride;   // that ring: slots, lag of the slot this step uses, floats per slot
  int32_t gparts, gpstride; // partial weight gradients of the stage: their number, floats between two of them
                            // (K_GEMM backward weights writes one of them, K_UPDATE sums them in order)
  int32_t ppstride;         // K_UPDATE, > 0: the stage keeps two copies of its master parameters, ppstride floats apart; the
                            // update of tick t reads copy t mod 2 and writes the other (its backward readers of the tick
                            // read copy t mod 2 through the ring fields above), so that it may run beside them
  int32_t upd_n, upd_t0;    // K_UPDATE: update size N (gradients of N consecutive samples per update) and the tick of the
                            // stage's first backward pass
  // One launch per tick (all phases in one grid): a workgroup of a later phase waits until the counters
  // wait_idx[i] have reached wait_n[i] x (ticks so far), i.e. until the stage's workgroups of the earlier
  // phases are done, and every workgroup adds one to counter sig_idx when it is done
  int32_t sig_idx, nwait;
  int32_t wait_idx[3], wait_n[3];
  int32_t grain;            // > 0: streaming form of an elementwise step, floats per workgroup (K_COPY, K_GNB_APPLY);
                            // K_GNB_REDUCE: 1 = one wavefront per channel
  GemmCfg g;     // main operand set of a K_GEMM step
  GemmCfg gp;    // projection of the skip tensor accumulated into the same tile (forward only)
  TRef x;        // op input (forward) / saved input (backward)
  TRef st;       // statistics slot: mean[G], rstd[G], sc[C], sh[C]
  TRef y;        // op output
  TRef dy;       // incoming gradient
  TRef dx;       // outgoing gradient
  TRef skip;     // skip tensor (forward epilogue / projection weight gradient)
  TRef skg;      // skip-path gradient
  const float* w;      // weight used by this step (predicted on forward, current on backward)
  const float* b;
  const float* wp;
  const float* gamma;
  const float* beta;
  float* v;            // K_UPDATE / fused GroupNorm update: velocity read
  float* what;         // ... predicted weights written (nullptr without LWP)
  float* gw;           // gradient outputs
  float* gb;
  float* ggamma;
  float* gbeta;
  float* gacc;         // K_UPDATE with an update size above one: gradients added up since the stage's latest update
  const float* what0;  // ... and slot 0 of the stage's ring of predicted weights (never moved to the tick's slot)
  float* part;         // per-channel partial sums of the GN backward
  float* loss_log;
  int32_t* labels;     // label ring [n_stages]
  const int32_t* tq;   // K_GEMM: reduction index (chunk-relative) -> patch offset, QCpad entries
  const int32_t* tn;   // K_GEMM: column index -> patch offset, N entries
  const int32_t* tq2;  // the same for the projection operand set
  const int32_t* tn2;
};

// State that changes from tick to tick lives in device memory so that a
// recorded launch sequence can be replayed unchanged.
struct Globals {
  int32_t t_base;      // tick index = t_base + k (k = launch argument)
  int32_t idx_base;    // pool item = (idx_base + k) mod n_pool
  int32_t n_pool;
  int32_t pad_;
  const float* pool;
  const int32_t* pool_labels;
};

// ---- launch wrappers implemented in pb_kernels.hip ----
// sync != nullptr: the grid holds every phase of the tick; sync[SYNC_ERR] collects errors, sync[SYNC_SPIN] is the
// bound of a dependency wait (iterations), sync[SYNC_CNT + i] are the completion counters; tick_ordinal counts the
// ticks launched in this form since the counters were cleared, starting at 1
constexpr int SYNC_ERR = 0, SYNC_SPIN = 1, SYNC_CNT = 16;
void launch_phase(const StepDesc* recs_dev, int total_tiles, const Globals* G, int k, const float* sample_override,
                  int label_override, bool nt, hipStream_t s, int32_t* sync = nullptr, uint32_t tick_ordinal = 0);
void launch_ingest(TRef ring0, int n_elems, const float* staging, int label, int32_t* label_ring,
                   int n_stages, const Globals* G, int k, hipStream_t s);
void launch_update_flat(float* w, float* v, const float* g, float* what, int64_t n, float lr, float m,
                        float a, float b, float lrT, hipStream_t s);
void launch_advance(Globals* G, int dt, int didx, hipStream_t s);
void launch_set_globals(Globals* G, Globals val, hipStream_t s);
void launch_fill_zero(void* p, size_t bytes, hipStream_t s);   // bytes a multiple of 16, p 16-byte aligned

// The library's own device array for contexts that must not allocate (pb_init_static): its
// address on the current device (looked up once per device) and that device's ordinal.
constexpr size_t STATIC_ARENA_BYTES = (size_t)64 << 20;
hipError_t static_arena(void** ptr, int* device);

}  // namespace pb
