// Launch wrappers of the gfx950 kernels behind the stairs C ABI (see include/stairs.h).
// Host code only sees these functions; every pointer is a device pointer unless named h_*.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

namespace stairs {

constexpr int kMaxRows = 32;        // rows (new tokens) of ONE sequence a forward of the decode kernels can take
constexpr int kMaxFwdRows = 64;     // rows of all sequences together a forward of the decode kernels can take (bf16)
constexpr int kMaxBlockRows = 256;  // rows one forward of several sequences can take on the block kernels (beyond kMaxRows)
constexpr int kAttnChunk = 128;     // keys per attention work-group of the fp32-cache kernels and the unit callers count chunks in; boundaries are absolute positions
constexpr int kAttnChunkH = 256;    // keys per attention work-group of the half-cache kernels (a wave owns 64)
constexpr int kAttnFusedMaxChunks = 24;   // more chunks per head than this: the chunk merge runs as a second kernel
constexpr size_t kAttnMergeMaxLds = 150 * 1024;   // most dynamic LDS the chunk merge may take
constexpr int kSsqGroupF32 = 1024;  // residual columns per sum-of-squares partial, fp32 models
constexpr int kSsqGroupBf16 = 16;   // ... bf16 models (= one weight tile of the residual-writing GEMMs)
constexpr int kUnitK = 256;         // k extent of one weight "unit" (8 MFMA k-steps of 32)
constexpr int kSliceUnits = 2;      // units per split-K slice (512 k)
constexpr int kSpwRows = 9;         // 9..16 rows: a split-K work-group takes two k chunks (see launch_gemm)
// most LDS the small-M GEMM (whole X block in LDS) may take per work-group: projections with many weight tiles keep
// two work-groups per CU, the residual-writing ones (one work-group per CU) take most of the CU's LDS
constexpr size_t kRowsPathMaxLds = 68 * 1024;
constexpr size_t kRowsPathMaxLdsWide = 150 * 1024;
constexpr size_t kWideMaxLds = 150 * 1024;      // chunk sums of k_gemm_bf16_wide: chunks * rows * 16 NT * 4 bytes
constexpr int kWideDepth8 = 2, kWideDepth6 = 2, kWideDepth4 = 3, kWideDepth3 = 4, kWideDepth2 = 5, kWideDepth1 = 8;   // k-steps in flight per wave at 4 / 2 / 1 tiles per wave
constexpr size_t kRowsPathSmallMatrix = 16u << 20;   // residual-writing projections with fewer tiles than CUs: up to this many bytes

// Where the rows of a forward sit.  One sequence (rps == 0): row r is at position *base + offset + r (base lives
// in device memory so that the same launch sequence can be replayed without the host knowing the sequence length).
// Several sequences ("slots", rps > 0): the forward holds rps consecutive rows per slot; slot s = r / rps keeps its
// state in base[s * kSlotState + ...] = {L, n of the last iteration, 0, active}; row r is at position
// L_s + offset + r % rps, or nowhere (negative) when the slot is not active.
constexpr int kSlotState = 4;
struct PosRef {
  const int* base;
  int offset;
  int rps;
};
#ifdef __HIPCC__
__device__ __forceinline__ int slot_of(const PosRef& p, int r) { return p.rps ? r / p.rps : 0; }
__device__ __forceinline__ int pos_of(const PosRef& p, int r) {
  if (!p.rps) return *p.base + p.offset + r;
  const int s = r / p.rps;
  const int* st = p.base + s * kSlotState;
  return st[3] ? st[0] + p.offset + (r - s * p.rps) : -(1 << 24);
}
#endif

// Row normalisation folded into a GEMM: the input is x[m][k] * gain[k] * rstd[m] with
// rstd[m] = 1/sqrt(sum_p ssq_part[m*ssq_n + p] / K + eps).  gain == nullptr: no scaling at all.
// (bf16 kernels: the gain goes into the activation fragments, rstd[m] multiplies the row's finished sums; the
// split-K kernel forms it in the work-group that finishes a column group, the small-M kernel in every work-group.)
struct RowNorm {
  const float* gain;
  const float* ssq_part;
  int ssq_n;
  float eps;
};

inline int ssq_groups(int d, int bf16) {
  const int g = bf16 ? kSsqGroupBf16 : kSsqGroupF32;
  return (d + g - 1) / g;
}
inline int gemm_slices(int K, int dtype_bf16) {
  if (!dtype_bf16) return 1;
  int units = K / kUnitK;
  return (units + kSliceUnits - 1) / kSliceUnits;
}

// ---- weights --------------------------------------------------------------------------
// bf16 [N, K] row-major -> MFMA-operand tiles: tile (nt, kt) covers rows nt*16.., k kt*32.., is 1 KiB;
// inside it lane l = r + 16*g holds W[nt*16+r][kt*32+g*8..+8].  Tiles are stored slice-major:
// [split-K slice of 16 k-steps][nt][k-step inside the slice], so that one work-group of the GEMM
// (one slice, 4*NT adjacent row tiles) reads one contiguous run.
// perm: order of the rows (= output columns of the GEMM): kPermGateUp (p0 = f) puts the gate and up rows of 8
// features into one tile, kPermQKV (p0 = d, p1 = head_dim) the two halves of 8 rotation pairs; the epilogues undo it.
enum { kPermNone = 0, kPermGateUp = 1, kPermQKV = 2 };
void launch_swizzle_bf16(const uint16_t* W, uint4* Wsw, int N, int K, int perm, int p0, int p1, hipStream_t st);

enum { kRoleQKV = 0, kRoleWo = 1, kRoleGateUp = 2, kRoleDown = 3, kRoleHead = 4 };   // which projection a GEMM launch is

// What the GEMM does with its result (by role):
//   QKV    : columns [0,d) q, [d,2d) k, [2d,3d) v: rotate q and k by the row's position, out = q as
//            float [M, d], append k and v to the layer's cache at that position
//   Wo/Down: out = x [M, N] += result; ssq_out[m][g] = sum over column group g of x^2
//   GateUp : out = h [M, N/2] = silu(gate) * up
//   Head   : out = logits [M, N]; with act == kActRelu out = max(result, 0) (the first matrix of an ungated
//            feed-forward block)
enum { kActNone = 0, kActRelu = 1 };
struct GemmEpi {
  int* counters;            // bf16 path: one int per column group, zero between launches
  float* out;
  float* ssq_out;
  const float2* rope_cs;    // [M][64] (cos, sin)
  PosRef pos;
  _Float16* Kc;             // bf16 models: half caches of this layer, tiled layout
  _Float16* Vc;
  float* Kc32;              // fp32 models: float caches of this layer, [H][cap][hd]
  float* Vc32;
  int cap, H, hd;
  size_t kv_slot_stride;    // elements between the caches of consecutive slots (several sequences), else unused
  // k_gemm_bf16_wide, residual-writing and gate/up roles: where the fragments of the result go for the next
  // projection (see frag_bytes), with frag_gain[k] folded in; nullptr: none
  uint4* frag_out;
  const float* frag_gain;
  int act;                  // Head role only: kActNone / kActRelu
  int stream_weights;       // bf16: read the weights with the streaming hint (models far larger than the memory-side cache)
};

// ---- skinny GEMM + epilogue ---------------------------------------------------------------
// bf16: W is swizzled, split-K slices of 512 k, epilogue fused; fp32: W row-major, epilogue in a
// second kernel.  partial: scratch of gemm_slices() * M * N floats.
// xfrag (bf16, M > 4): the fragments of X with nrm.gain folded in, left by X's producer or by launch_split_frag; with
// them the launch takes the hand-off-free kernel k_gemm_bf16_wide (no partial sums), without them the split-K kernel.
void launch_gemm(int role, int dtype_bf16, const void* W, int N, int K, const float* X, int ldx, int M,
                 RowNorm nrm, float* partial, const GemmEpi& epi, hipStream_t st, const uint4* xfrag = nullptr);

// Activation fragments of a [M <= 32, K] block: K / 32 k-steps x 2 column tiles x (high, low) x 1 KiB
// (+ kFragChunkPad uint4 after every 16 k-steps: the k chunks the waves of a work-group read at the same time then do
// not sit a power of two apart)
constexpr int kFragChunkPad = 272;
// rows 32..63 of a forward have a second fragment block of the same layout kFragHalfU4 uint4 after the first
constexpr size_t kFragHalfU4 = (4u << 20) / 16;
inline size_t frag_bytes(int K) { return ((size_t)(K / 32) * 256 + (size_t)(K / 512 + 1) * kFragChunkPad) * 16; }   // one block of 32 rows
inline size_t frag_alloc_bytes(int K) { return kFragHalfU4 * 16 + frag_bytes(K); }                                      // both blocks
// frag = fragments of x [M, K] (row stride ldx) times gain (nullptr: none)
// whether launch_gemm takes M > kMaxRows rows of a bf16 projection with k = K (the chunk sums of all rows fit the LDS)
bool gemm_takes_rows(int M, int K);
void launch_split_frag(const float* X, int ldx, int M, int K, const float* gain, uint4* frag, hipStream_t st);

// The next bf16 launch_gemm records `start` at the beginning and `stop` at the end of its kernel (the events of the
// launch itself, not records around it in the stream); one launch only.  Measurement aid.
void set_gemm_launch_events(hipEvent_t start, hipEvent_t stop);

// ---- small kernels ----------------------------------------------------------------------
// x[m][:] = emb[tokens[pos+m]][:] (row of zeros if pos+m lies outside [0, tok_cap) or the id found there outside
// [0, vocab)), plus sum-of-squares partials; the same launch fills the rotation table cs of the M positions (see
// launch_rope_table); theta <= 0: the identity rotation (1, 0).  tok_cap = ints one sequence's token array holds.
void launch_embed(const void* emb, int emb_bf16, const int* tokens, int tok_slot_stride, int tok_cap, int vocab, PosRef pos,
                  int M, int d, float* x, float* ssq_part, int hd, float theta, float2* cs, hipStream_t st,
                  uint4* frag = nullptr, const float* frag_gain = nullptr);   // bf16: also the fragments of x * frag_gain
// cs[m][i] = (cos, sin)((pos+m) * theta^(-2i/hd)), angle formed in double
void launch_rope_table(PosRef pos, int M, int hd, float theta, float2* cs, hipStream_t st);
// split-KV attention of M query rows at positions pos..pos+M-1 against keys 0..pos+M-1
// (kv_half: half caches in the tiled layout; else float caches [H][cap][hd]); counters: one int per (slot, head).
// Several sequences (pos.rps > 0, half caches only): M = pos.rps rows per slot, nslots slots, caches kv_slot_stride
// elements apart.
// am (half caches only): score scale, additive bias by relative position, fixed key set (see AttnMode).
struct AttnMode {
  float scale;        // multiplies q; <= 0: 1/sqrt(head_dim)
  const float* bias;  // nullptr, or [H][bias_ld]: score += bias[h][key position - query position + bias_zero]
  int bias_ld, bias_zero;
  int kv_fixed;       // > 0: no causal mask, every row sees the keys 0 .. kv_fixed-1 (nchunk_launch must cover them)
  uint4* frag_out;    // half caches: also leave the output's activation fragments here (nullptr: none)
};
void launch_attention(const float* q_rot, const void* Kc, const void* Vc, int kv_half, int cap, int d, int H, int M,
                      PosRef pos, int nslots, size_t kv_slot_stride, int nchunk_launch, int nchunk_cap, float* part_o,
                      float* part_ml, int* counters, float* out, hipStream_t st,
                      const AttnMode& am = AttnMode{0.f, nullptr, 0, 0, 0, nullptr});
// out[o(r)] = argmax_v logits[row0 + r * row_stride][v], ties -> lowest v, r < nrows.  One sequence:
// o(r) = *out_pos.base + out_pos.offset + r (base == nullptr: r).  Several: o(r) = s * out_slot_stride + position of
// out_pos for row r, nothing written for a slot that is not active.
void launch_argmax(const float* logits, int ld, int V, int nrows, int row0, int row_stride, int* out, PosRef out_pos,
                   int out_slot_stride, hipStream_t st);
// stairs validation on device, one block per slot s (one sequence: nslots = 1, strides unused): state = {L, n, 0,
// active}.  n = longest run with tokens[L+i] == tgt[i]; tokens[L+n] = tgt[n]; state[0] = L+n+1; state[1] = n.
// tokens of slot s start at s * tok_slot_stride, its tgt at s * (k+1), its state at s * kSlotState.
void launch_accept(int* tokens, const int* tgt, int k, int* state, int nslots, int tok_slot_stride, hipStream_t st);

// ---- sampling variant -------------------------------------------------------------------------------------
// Device-resident parameters of a sampled generation (so that captured launches stay valid across seeds)
struct SampleParams {
  float inv_temp;      // 1 / temperature
  uint64_t key;        // key of the counter-based generator (from the seed)
};
// Scratch of a draw spread over several blocks: one (score, index) per block and the ticket of the last arrival
// (zero at allocation, zero again after every launch)
constexpr int kSampleBlocksMax = 512;
struct SampleWs {
  int ticket;
  int pad;
  unsigned long long score[kSampleBlocksMax];
  int idx[kSampleBlocksMax];
};
// lse[r] = log sum_v exp(row_r[v] * inv_temp) for the n_a rows of a followed by the n_b rows of b (row stride ld)
void launch_row_lse(const float* a, int n_a, const float* b, int n_b, int ld, int V, const SampleParams* sp, float* lse,
                    hipStream_t st);
// tokens[o] = one draw from softmax(logits / T) by Gumbel-max with the random numbers of (o, stream), o = out_pos
void launch_sample(const float* logits, int V, const SampleParams* sp, int stream, int* tokens, PosRef out_pos,
                   SampleWs* ws, hipStream_t st);
// keep / replace walk over a sampled stair batch of one sequence (see k_accept_sampled); lse = launch_row_lse over
// the k+1 rows of tl followed by the k rows of dl
void launch_accept_sampled(int* tokens, const float* tl, const float* dl, int ld, int V, int k, const float* lse,
                           const SampleParams* sp, int* state, int* emitted, SampleWs* ws, hipStream_t st);

// ---- prompt ingestion in large row blocks (bf16 models) ------------------------------------------------
// The projections of a block of up to kPfRows prompt rows run on the MFMA-bound kernel k_gemm_bf16_block: the weights
// in the decode kernels' layout, the activations as fragments (bf16 high + low parts in operand order) written by
// the element-wise kernel in front of each projection.
constexpr int kPfRows = 2048;
constexpr int kBlkRows = 128;       // rows of one GEMM work-group; fragment buffers are laid out for whole groups
inline int pf_col_tiles(int R) { return (R + kBlkRows - 1) / kBlkRows * (kBlkRows / 16); }
// bytes of the fragments of a [R, K] activation block
inline size_t pf_frag_bytes(int R, int K) { return (size_t)(K / 32) * pf_col_tiles(R) * 2 * 1024; }
// Y[R, N] = (accumulate ? Y : 0) + X . W^T; W [N, K] in the operand-tile layout with row permutation (perm, p0, p1)
// as given to launch_swizzle_bf16 (Y's columns are in natural order), xfrag the fragments of X [R, K]
// part (optional, part_floats floats): scratch that lets a launch with few rows cut k into pieces for more work-groups
// (the pieces' results are added in a fixed order by a second kernel)
void launch_gemm_block(const void* W, int N, int K, const uint4* xfrag, int R, float* Y, int ldy, int perm, int p0, int p1,
                       int accumulate, hipStream_t st, float* part = nullptr, size_t part_floats = 0);
// x[r][:] = emb[tokens[p0 + r]][:] as float, r < R (zeros for a position outside [0, tok_cap) or an id outside [0, vocab))
void launch_pf_embed(const uint16_t* emb, const int* tokens, int p0, int tok_cap, int vocab, int R, int d, float* x,
                     hipStream_t st);
// one row per work-group: v = x (gain == nullptr) or x * rstd * gain with rstd = 1/sqrt(mean(x^2) + eps);
// frag = the block fragments of v (bf16(v) and bf16(v - bf16(v)))
void launch_pf_norm_split(const float* x, const float* gain, float eps, int R, int d, uint4* frag, hipStream_t st);
// cs[r][i] = (cos, sin)((p0 + r) * theta^(-2i/hd)), angle in double
void launch_pf_rope_table(int p0, int R, int hd, float theta, float2* cs, hipStream_t st);
// y = [R, 3d] (q | k | v, natural column order): rotate q and k, q -> q_rot [R, d] float, k and v -> the tiled half
// caches of one layer at positions p0 .. p0+R-1
void launch_pf_rope_kv(const float* y, int R, int d, int H, int p0, const float2* cs, float* q_rot, _Float16* Kc,
                       _Float16* Vc, int cap, hipStream_t st);
// the same for R rows positioned by `pos` (several sequences: slot s's caches start s * kv_slot_stride elements in);
// rows without a position write nothing to the caches
void launch_pf_rope_kv_rows(const float* y, int R, int d, int H, PosRef pos, size_t kv_slot_stride, const float2* cs,
                            float* q_rot, _Float16* Kc, _Float16* Vc, int cap, hipStream_t st);
// attention of a prefill block: R consecutive rows at positions p0.. of ONE sequence against its half caches (keys
// 0 .. own position), q and out [R, d]; running softmax in registers (no partial results, no merge), a wave per 16 rows
void launch_attention_flash(const float* q, const void* Kc, const void* Vc, int cap, int d, int H, int R, int p0, float* out,
                            hipStream_t st);
// y = [R, 2f] (gate | up): h = silu(gate) * up, written as block fragments of [R, f]
void launch_pf_swiglu_split(const float* y, int R, int f, uint4* frag, hipStream_t st);

// dst[0..bytes) = src[0..bytes), bytes a multiple of 16: reads `bytes` and writes `bytes` of HBM
void launch_copy_probe(const void* src, void* dst, size_t bytes, hipStream_t st);

// opt in to large dynamic LDS for the kernels that need it (once per process/device)
hipError_t configure_kernels();

}  // namespace stairs
