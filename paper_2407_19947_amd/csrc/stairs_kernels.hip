// gfx950 kernels of the stairs library.  Written for wave64 / MFMA / LDS of CDNA4 only.
//
// Numerics contract shared by all kernels: activations, residual stream, logits and every
// accumulation are fp32; bf16 appears only as stored weights, stored keys/values and as the
// MFMA activation operand, which is fed as a bf16 high part plus a bf16 low part (two MFMAs
// per weight tile) so that the activation keeps ~16 mantissa bits.  Every reduction runs in
// an order that does not depend on the number of rows M of the launch, so a row of a stair
// batch gets bit-identical results to the same position computed alone (the property that
// makes the stair batch return what plain greedy decoding returns, paper abstract / Sec. 3.3).
#include "stairs_kernels.h"
#include <hip/hip_ext.h>

#include <math.h>
#include <stdio.h>
#include <stdlib.h>

#include <algorithm>
#include <vector>

namespace stairs {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

// ---------------------------------------------------------------------------------------
// helpers
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t bf16_bits_rne(float x) {
  uint32_t u = __float_as_uint(x);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return u >> 16;
}
__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }
// Two floats -> a packed pair of bf16 (a in the low half), round to nearest even, by the conversion instruction of
// gfx950 (one instruction for the pair; same bits as bf16_bits_rne for every value that is not a NaN), and the split
// of the pair into that high part and the bf16 of the remainders.
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t bf16_pack2_rne(float a, float b) {
  const f32x2_t v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
__device__ __forceinline__ void bf16_split2(float a, float b, uint32_t& hi, uint32_t& lo) {
  hi = bf16_pack2_rne(a, b);
  lo = bf16_pack2_rne(a - __uint_as_float(hi << 16), b - __uint_as_float(hi & 0xFFFF0000u));
}

// Activation fragments: the MFMA B operand of a forward with more than 4 rows is formed ONCE by whoever produces the
// activation (embedding gather, attention, the previous projection's epilogue) and kept beside the fp32 values as
// [k-step of 32][column tile of 16 rows (2)][high, low][lane] x 16 bytes: lane r + 16 g of k-step kt holds
// x[16 ct + r][32 kt + 8 g .. + 8] * gain as bf16 (high part) and the bf16 of the remainders (low part), the very
// values split_bf16x8 gives.  A consumer wave loads a fragment as one coalesced 1 KiB read.
// Rows 32..63 (forwards of several sequences) have a second block of the same layout kFragHalfU4 uint4 further on.
__device__ __forceinline__ size_t frag_off(int m, int k) {        // in units of 8 bytes: 4 consecutive k of row m, high part
  return (size_t)(m >> 5) * (kFragHalfU4 * 2) +
         ((((size_t)(k >> 5) * 2 + ((m >> 4) & 1)) * 2) * 64 + (size_t)(k >> 9) * kFragChunkPad + (m & 15) + 16 * ((k & 31) >> 3)) * 2 +
         ((k & 7) >> 2);
}
// row m, columns k .. k+3 (k a multiple of 4); g = the gain of those columns or nullptr
__device__ __forceinline__ void store_frag4(uint4* frag, int m, int k, float4 v, const float* gain) {
  if (gain) {
    const float4 g = *reinterpret_cast<const float4*>(gain + k);
    v.x = v.x * g.x; v.y = v.y * g.y; v.z = v.z * g.z; v.w = v.w * g.w;
  }
  uint2 hi, lo;
  bf16_split2(v.x, v.y, hi.x, lo.x);
  bf16_split2(v.z, v.w, hi.y, lo.y);
  uint2* dst = reinterpret_cast<uint2*>(frag) + frag_off(m, k);
  dst[0] = hi;
  dst[128] = lo;                                               // the low fragment follows 64 lanes x 16 bytes later
}
__device__ __forceinline__ float load_kv(const float* p) { return *p; }
__device__ __forceinline__ float load_kv(const uint16_t* p) { return bf16_bits_to_float(*p); }
__device__ __forceinline__ void store_kv(float* p, float v) { *p = v; }
__device__ __forceinline__ void store_kv(uint16_t* p, float v) { *p = (uint16_t)bf16_bits_rne(v); }
// keys/values of bf16 models are cached as IEEE half: same bytes as bf16, 8x smaller rounding step
// (bf16 storage alone moves 1B-class logits by 1.7e-2); saturates at the half range
__device__ __forceinline__ float load_kv(const _Float16* p) { return (float)*p; }
__device__ __forceinline__ void store_kv(_Float16* p, float v) { *p = (_Float16)fminf(fmaxf(v, -65504.f), 65504.f); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
  return v;
}
// sum over a 256-thread block, fixed order; sm: 4 floats of LDS
__device__ __forceinline__ float block_sum_256(float v, float* sm) {
  v = wave_sum(v);
  if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = v;
  __syncthreads();
  return (sm[0] + sm[1]) + (sm[2] + sm[3]);
}

// Data handed from one work-group to another inside a kernel (split-K partial sums, attention chunk
// partials) is written and read with relaxed device-scope atomic accesses: they write through to / read
// from the level all XCDs share, so the hand-off needs no cache-wide write-back or invalidate; the
// writer only waits for its own stores (s_waitcnt) before it takes its ticket.
__device__ __forceinline__ void st_dev2(float* p, float a, float b) {
  const unsigned long long v = (unsigned long long)__float_as_uint(a) | ((unsigned long long)__float_as_uint(b) << 32);
  __hip_atomic_store(reinterpret_cast<unsigned long long*>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_dev(float* p, float a) {
  __hip_atomic_store(p, a, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_dev(const float* p) {
  return __hip_atomic_load(const_cast<float*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float2 ld_dev2(const float* p) {
  const unsigned long long v = __hip_atomic_load(reinterpret_cast<unsigned long long*>(const_cast<float*>(p)),
                                                 __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return make_float2(__uint_as_float((unsigned)v), __uint_as_float((unsigned)(v >> 32)));
}
// all of this work-group's stores have completed; then one thread takes the ticket.  Returns true in
// every thread of the work-group that arrived last of `expected`.
__device__ __forceinline__ bool last_arrival(int* counter, int expected, int* s_flag) {
  // The hand-off rests on two things the memory model does not promise for relaxed accesses: (1) a device-scope
  // write-through store is acknowledged only once it sits at the level all XCDs share, so "vmcnt == 0" means the
  // partial results are visible there; (2) the last arrival's loads of the others' results are issued after its
  // ticket.  (1) is the hardware's behaviour for sc1 stores; for (2) the signal fences keep the compiler from moving
  // memory accesses across the ticket in either direction (they emit no instruction).  Should either stop holding,
  // the fix is a release fence before and an acquire fence after the ticket (__atomic_thread_fence at agent scope):
  // correct by the model, at the price of an L2 write-back / invalidate per work-group.
  __atomic_signal_fence(__ATOMIC_SEQ_CST);
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();
  if (threadIdx.x == 0)
    *s_flag = (__hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == expected - 1) ? 1 : 0;
  __syncthreads();
  __atomic_signal_fence(__ATOMIC_SEQ_CST);
  return *s_flag != 0;
}

__device__ __forceinline__ float row_rstd(const RowNorm& nrm, int m, int K) {
  float ss = 0.f;
  for (int p = 0; p < nrm.ssq_n; ++p) ss += nrm.ssq_part[m * nrm.ssq_n + p];
  return 1.0f / sqrtf(ss / (float)K + nrm.eps);
}

// ---------------------------------------------------------------------------------------
// weight re-layout
// ---------------------------------------------------------------------------------------
// Row order of the re-laid-out matrix.  Output column n' of the GEMM is source row perm(n'):
//   kPermNone  : identity
//   kPermGateUp: W = [f gate rows; f up rows]; tile t holds gate rows 8t..8t+7 then up rows 8t..8t+7, so a SwiGLU
//                pair sits at columns (j, j+8) of one 16-column tile
//   kPermQKV   : W = [q; k; v] of d rows each, heads of hd rows; inside a q or k head tile t holds dims 8t..8t+7 then
//                hd/2+8t..hd/2+8t+7, so a rotation pair (e, e+hd/2) sits at columns (j, j+8) of one tile; v unchanged
__device__ __forceinline__ size_t perm_row(int nprime, int perm, int p0, int p1) {
  const int r = nprime & 15;
  if (perm == kPermGateUp) return (size_t)((r >> 3) ? p0 : 0) + (size_t)(nprime >> 4) * 8 + (r & 7);
  if (perm == kPermQKV) {
    const int d = p0, hd = p1;
    const int part = nprime / d, c = nprime - part * d;
    if (part == 2) return (size_t)nprime;
    const int h = c / hd, w = c - h * hd;
    return (size_t)part * d + (size_t)h * hd + (w >> 4) * 8 + (r & 7) + (r >> 3) * (hd >> 1);
  }
  return (size_t)nprime;
}

__global__ __launch_bounds__(256) void k_swizzle_bf16(const uint16_t* __restrict__ W, uint4* __restrict__ Wsw,
                                                      int KT, int NTILES, size_t total, int K, int perm, int p0, int p1) {
  size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  // destination order: [k-slice][row tile][k-step inside the slice][lane]
  const int lane = (int)(idx & 63);
  const size_t tile_idx = idx >> 6;
  constexpr int SK = kSliceUnits * 8;                    // k-steps of a full slice
  const size_t full = (size_t)NTILES * SK;               // tiles per full slice
  const int s = (int)(tile_idx / full);
  const size_t rem = tile_idx - (size_t)s * full;
  const int ks = min(SK, KT - s * SK);                   // k-steps of this slice (the last one may be short)
  const int nt = (int)(rem / ks), kk = (int)(rem - (size_t)nt * ks);
  const int kt = s * SK + kk;
  const int r = lane & 15, g = lane >> 4;
  const size_t row = perm_row(nt * 16 + r, perm, p0, p1);
  Wsw[idx] = *reinterpret_cast<const uint4*>(W + row * K + kt * 32 + g * 8);
}

void launch_swizzle_bf16(const uint16_t* W, uint4* Wsw, int N, int K, int perm, int p0, int p1, hipStream_t st) {
  int KT = K / 32;
  size_t total = (size_t)(N / 16) * KT * 64;
  unsigned blocks = (unsigned)((total + 255) / 256);
  hipLaunchKernelGGL(k_swizzle_bf16, dim3(blocks), dim3(256), 0, st, W, Wsw, KT, N / 16, total, K, perm, p0, p1);
}

// ---------------------------------------------------------------------------------------
// skinny GEMM, bf16 weights, MFMA 16x16x32, with the projection's epilogue fused in
//   work-group = 4 waves; all four work on the same 512-wide k-slice (the X slice is staged once
//   in LDS as MFMA B fragments, high and low halves) and on 4*NT consecutive 16-row weight tiles.
//   The weight tile is the MFMA A operand and is loaded straight from HBM in operand order
//   (1 KiB per wave-load, fully coalesced); the X rows are the B operand.
//   Split-K: every work-group writes its partial sums; the one that arrives last at the column
//   group's counter adds the slices up in slice order (so the result does not depend on which
//   one that is) and applies the epilogue of the projection (ROLE).
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ size_t k_cache_off(int pos, int e, int hd) {   // element offset inside one head
  return ((size_t)((pos >> 4) * (hd >> 5) + (e >> 5)) * 64 + (pos & 15) + 16 * ((e & 31) >> 3)) * 8 + (e & 7);
}
__device__ __forceinline__ size_t v_cache_off(int pos, int e, int hd) {
  const int p32 = pos & 31, k16 = p32 & 15;
  return ((size_t)((pos >> 5) * (hd >> 4) + (e >> 4)) * 64 + (e & 15) + 16 * (k16 >> 2)) * 8 + (k16 & 3) + 4 * (p32 >> 4);
}

// Sum of the split-K partial sums of one element (or 4 adjacent ones).  The order is fixed for every GEMM variant:
// the 512-wide k chunks are added in pairs, (c0 + c1), (c2 + c3), ..., and the pair sums one after the other.
// PAIRS = true: the S partials are single chunks (the pairs are formed here); false: they already are pair sums.
// The loads of up to 8 partials are issued together (they are full round trips to the memory side).
template <bool PAIRS>
__device__ __forceinline__ float slice_sum(const float* partial, int S, size_t stride, size_t off) {
  float a = 0.f;
  for (int s0 = 0; s0 < S; s0 += 8) {
    float v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = ld_dev(partial + (size_t)min(s0 + i, S - 1) * stride + off);
    if (PAIRS) {
#pragma unroll
      for (int i = 0; i < 8; i += 2)
        if (s0 + i < S) a += (s0 + i + 1 < S) ? (v[i] + v[i + 1]) : v[i];
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) a += (s0 + i < S) ? v[i] : 0.f;
    }
  }
  return a;
}
template <bool PAIRS>
__device__ __forceinline__ float4 slice_sum4(const float* partial, int S, size_t stride, size_t off) {
  float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int s0 = 0; s0 < S; s0 += 8) {
    float2 p[8], q[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float* src = partial + (size_t)min(s0 + i, S - 1) * stride + off;
      p[i] = ld_dev2(src);
      q[i] = ld_dev2(src + 2);
    }
    if (PAIRS) {
#pragma unroll
      for (int i = 0; i < 8; i += 2) {
        if (s0 + i < S) {
          const bool two = s0 + i + 1 < S;
          a.x += two ? (p[i].x + p[i + 1].x) : p[i].x; a.y += two ? (p[i].y + p[i + 1].y) : p[i].y;
          a.z += two ? (q[i].x + q[i + 1].x) : q[i].x; a.w += two ? (q[i].y + q[i + 1].y) : q[i].y;
        }
      }
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const bool ok = s0 + i < S;
        a.x += ok ? p[i].x : 0.f; a.y += ok ? p[i].y : 0.f; a.z += ok ? q[i].x : 0.f; a.w += ok ? q[i].y : 0.f;
      }
    }
  }
  return a;
}

// The arithmetic of the epilogues lives in these helpers so that every GEMM variant produces the same bits.
__device__ __forceinline__ float swiglu(float g, float u) {
#pragma clang fp contract(off)
  return g / (1.0f + expf(-g)) * u;
}
// sum of squares of 4 adjacent residual values; a 16-column tile's partial is ((s0 + s1) + (s2 + s3)) of these
__device__ __forceinline__ float sumsq4(float x, float y, float z, float w) {
#pragma clang fp contract(off)
  return (x * x + y * y) + (z * z + w * w);
}
__device__ __forceinline__ float2 rope_rotate(float a, float b, float2 cs) {
#pragma clang fp contract(off)
  return make_float2(a * cs.x - b * cs.y, b * cs.x + a * cs.y);
}
// Row m, columns col and col+8 of the permuted QKV output (col & 15 < 8): a rotation pair of q or k, or two
// plain values of v.  pos0 = position of row 0.
// index of the rotation entry of columns (col, col + 8) of row m (q and k parts; for the v part some valid index)
__device__ __forceinline__ int qkv_rope_index(int m, int col, int d, int hd) {
  const int c = col % d, w = c % hd;
  return m * 64 + (w >> 4) * 8 + (w & 7);
}
// p: the row's position (pos_of), cs: its rotation entry (epi.rope_cs[qkv_rope_index]); a caller may have loaded both early
__device__ __forceinline__ void qkv_pair_at(float a, float b, int m, int col, int d, const GemmEpi& epi, int p, float2 cs) {
  if (p < 0) return;
  const size_t slot_off = (size_t)slot_of(epi.pos, m) * epi.kv_slot_stride;
  const int hd = epi.hd, half = hd >> 1;
  const int part = col / d, c = col - part * d;
  const int h = c / hd, w = c - h * hd;
  if (part == 2) {
    _Float16* dst = epi.Vc + slot_off + (size_t)h * epi.cap * hd;
    store_kv(dst + v_cache_off(p, w, hd), a);
    store_kv(dst + v_cache_off(p, w + 8, hd), b);
    return;
  }
  const int e = (w >> 4) * 8 + (w & 7);
  const float2 r = rope_rotate(a, b, cs);
  if (part == 0) {
    epi.out[(size_t)m * d + h * hd + e] = r.x;
    epi.out[(size_t)m * d + h * hd + e + half] = r.y;
  } else {
    _Float16* dst = epi.Kc + slot_off + (size_t)h * epi.cap * hd;
    store_kv(dst + k_cache_off(p, e, hd), r.x);
    store_kv(dst + k_cache_off(p, e + half, hd), r.y);
  }
}
__device__ __forceinline__ void qkv_pair(float a, float b, int m, int col, int d, const GemmEpi& epi) {
  const int p = pos_of(epi.pos, m);
  if (p < 0) return;
  qkv_pair_at(a, b, m, col, d, epi, p, epi.rope_cs[qkv_rope_index(m, col, d, epi.hd)]);
}

// Epilogue of one column group [c0, c0+W) for all M rows, run by the 256 threads of one work-group.
// rs: the rows' 1/rms in LDS when the GEMM's input is normalised (the X fragments carry x * gain only), else null.
template <int ROLE, int W, bool PAIRS>
__device__ __forceinline__ void gemm_epilogue(const float* partial, int S, int M, int N, int c0, const GemmEpi& epi,
                                              const float* rs) {
  const int tid = threadIdx.x;
  const size_t stride = (size_t)M * N;
  if (ROLE == kRoleHead) {
    constexpr int PR = W / 4;
    for (int idx = tid; idx < M * PR; idx += 256) {
      const int m = idx / PR, col = c0 + (idx - m * PR) * 4;
      if (col < N) {
        float4 a = slice_sum4<PAIRS>(partial, S, stride, (size_t)m * N + col);
        if (rs) { const float r = rs[m]; a.x *= r; a.y *= r; a.z *= r; a.w *= r; }
        if (epi.act == kActRelu) a = make_float4(fmaxf(a.x, 0.f), fmaxf(a.y, 0.f), fmaxf(a.z, 0.f), fmaxf(a.w, 0.f));
        *reinterpret_cast<float4*>(epi.out + (size_t)m * N + col) = a;
        if (epi.frag_out) store_frag4(epi.frag_out, m, col, a, epi.frag_gain);
      }
    }
  } else if (ROLE == kRoleWo || ROLE == kRoleDown) {
    constexpr int PR = W / 4;                       // threads per row; 4 adjacent threads = one 16-column tile
    const int total = M * PR;
    for (int idx0 = 0; idx0 < total; idx0 += 256) {
      const int idx = idx0 + tid;
      const int m = idx / PR, col = c0 + (idx - m * PR) * 4;
      float ss = 0.f;
      if (idx < total && col < N) {
        float4 a = slice_sum4<PAIRS>(partial, S, stride, (size_t)m * N + col);
        if (rs) { const float q = rs[m]; a.x *= q; a.y *= q; a.z *= q; a.w *= q; }
        float4* xp = reinterpret_cast<float4*>(epi.out + (size_t)m * N + col);
        const float4 r = *xp;
        a.x += r.x; a.y += r.y; a.z += r.z; a.w += r.w;
        *xp = a;
        ss = sumsq4(a.x, a.y, a.z, a.w);
        if (epi.frag_out) store_frag4(epi.frag_out, m, col, a, epi.frag_gain);
      }
      ss += __shfl_xor(ss, 1);
      ss += __shfl_xor(ss, 2);
      if (idx < total && col < N && (idx & 3) == 0) epi.ssq_out[m * (N >> 4) + (col >> 4)] = ss;
    }
  } else if (ROLE == kRoleGateUp) {
    // tile t = 8 gate columns then the 8 up columns of features 8t..8t+7; a thread takes 4 features
    constexpr int PR = W / 8;
    const int f = N / 2;
    for (int idx = tid; idx < M * PR; idx += 256) {
      const int m = idx / PR, r = idx - m * PR;
      const int gcol = c0 + 16 * (r >> 1) + 4 * (r & 1);
      if (gcol < N) {
        float4 g = slice_sum4<PAIRS>(partial, S, stride, (size_t)m * N + gcol);
        float4 u = slice_sum4<PAIRS>(partial, S, stride, (size_t)m * N + gcol + 8);
        if (rs) {
          const float q = rs[m];
          g.x *= q; g.y *= q; g.z *= q; g.w *= q;
          u.x *= q; u.y *= q; u.z *= q; u.w *= q;
        }
        const float4 o = make_float4(swiglu(g.x, u.x), swiglu(g.y, u.y), swiglu(g.z, u.z), swiglu(g.w, u.w));
        *reinterpret_cast<float4*>(epi.out + (size_t)m * f + (gcol >> 4) * 8 + (gcol & 7)) = o;
        if (epi.frag_out) store_frag4(epi.frag_out, m, (gcol >> 4) * 8 + (gcol & 7), o, nullptr);
      }
    }
  } else {   // kRoleQKV: rotate q and k, append k and v to the cache
    constexpr int PR = W / 2;
    for (int idx = tid; idx < M * PR; idx += 256) {
      const int m = idx / PR, r = idx - m * PR;
      const int col = c0 + 16 * (r >> 3) + (r & 7);
      if (col < N) {
        float a = slice_sum<PAIRS>(partial, S, stride, (size_t)m * N + col);
        float b = slice_sum<PAIRS>(partial, S, stride, (size_t)m * N + col + 8);
        if (rs) { a *= rs[m]; b *= rs[m]; }
        qkv_pair(a, b, m, col, N / 3, epi);
      }
    }
  }
}

// 1/rms of the rows from the sum-of-squares partials: half a wave (32 lanes) per row; a lane adds partials
// p = lane, lane + 32, ... in that order, then the 32 lanes are combined by a butterfly.  Wave w takes the row
// pairs w, w+4, ... (PASSES of them: 8 * PASSES >= M).  The first 256 partials of every pass are requested before any
// of them is used, so a work-group pays one round trip for all its rows.
template <int PASSES>
__device__ __forceinline__ void rows_rstd(const RowNorm& nrm, int M, int K, float* s_rstd) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int half = lane >> 5, pl = lane & 31;
  float v[PASSES][8];
#pragma unroll
  for (int ps = 0; ps < PASSES; ++ps) {
    const int m = min(2 * wave + 8 * ps + half, M - 1);
    const float* sp = nrm.ssq_part + (size_t)m * nrm.ssq_n;
#pragma unroll
    for (int i = 0; i < 8; ++i) v[ps][i] = sp[min(pl + 32 * i, nrm.ssq_n - 1)];
  }
#pragma unroll
  for (int ps = 0; ps < PASSES; ++ps) {
    const int m = 2 * wave + 8 * ps + half;
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) ss += (pl + 32 * i < nrm.ssq_n) ? v[ps][i] : 0.f;
    if (m < M) {
      for (int p0 = pl + 256; p0 < nrm.ssq_n; p0 += 256) {   // rows wider than 4096: the rest, 8 loads at a time
        float u[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) u[i] = (p0 + 32 * i < nrm.ssq_n) ? nrm.ssq_part[m * nrm.ssq_n + p0 + 32 * i] : 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) ss += u[i];
      }
    }
#pragma unroll
    for (int off = 16; off >= 1; off >>= 1) ss += __shfl_xor(ss, off);
    if (pl == 0 && m < M) s_rstd[m] = 1.0f / sqrtf(ss / (float)K + nrm.eps);
  }
}

// 8 consecutive x of one row -> (x * gain) -> bf16 high part and the bf16 of the remainder
__device__ __forceinline__ void split_bf16x8(const float4& xa, const float4& xb, const float4& g0, const float4& g1,
                                             bool scale, uint4& hi, uint4& lo) {
  // the row's 1/rms is not applied here: it is a scalar per row and multiplies the finished sums in the epilogue, so
  // the conversion does not wait for the row statistics
  float v[8] = {xa.x, xa.y, xa.z, xa.w, xb.x, xb.y, xb.z, xb.w};
  if (scale) {
    v[0] = v[0] * g0.x; v[1] = v[1] * g0.y; v[2] = v[2] * g0.z; v[3] = v[3] * g0.w;
    v[4] = v[4] * g1.x; v[5] = v[5] * g1.y; v[6] = v[6] * g1.z; v[7] = v[7] * g1.w;
  }
  bf16_split2(v[0], v[1], hi.x, lo.x);
  bf16_split2(v[2], v[3], hi.y, lo.y);
  bf16_split2(v[4], v[5], hi.z, lo.z);
  bf16_split2(v[6], v[7], hi.w, lo.w);
}

typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
// streaming load: the line is not kept in the caches on its way
__device__ __forceinline__ uint4 ld_nt(const uint4* p) {
  const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}
// One 8 KiB weight unit of a wave (8 loads of 1 KiB).  STREAM (a template argument: a run-time choice between the two
// load forms cost the whole gain in the kernels' prologues): weights of a model far larger than the
// 256 MB memory-side cache are read once per forward and gain from the streaming hint (a bare 2 GB read: 6.2 -> 7.05
// TB/s); a model that about fits that cache is served from it forward after forward and must keep plain loads.
template <bool STREAM>
__device__ __forceinline__ void load_unit(const uint4* p, uint4 (&wb)[8]) {
#pragma unroll
  for (int i = 0; i < 8; ++i) wb[i] = STREAM ? ld_nt(&p[i * 64]) : p[i * 64];
}

template <int CT, int NT, int ROLE, int SPW, bool STREAM>
__global__ __launch_bounds__(256) void k_gemm_bf16(const uint4* __restrict__ Wsw, int KT, int NTILES,
                                                   const float* __restrict__ X, int ldx, int M,
                                                   RowNorm nrm, int K, float* partial, int N, GemmEpi epi) {
  // SPW = k chunks (512 wide) a work-group takes, one after the other through the same LDS buffer: 1, or 2 (then
  // it writes the sum of its two chunk sums, which halves the partial sums in memory; used for many rows)
  extern __shared__ uint4 lds[];   // [16 k-steps][CT][hi,lo][64 lanes]
  __shared__ int s_last;
  __shared__ float s_rstd[kMaxRows];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int sp = blockIdx.y, SG = gridDim.y;               // this work-group's partial slice, number of them
  const int units_total = K / kUnitK;
  // weights are stored slice-major: [k chunk][row tile][k-step][lane]; the four waves take adjacent tiles, so
  // the work-group reads contiguous runs of 64*NT KiB
  const int tile0 = blockIdx.x * 4 * NT + wave;          // this wave's tiles: tile0 + 4 t
  auto chunk_units = [&](int j) { return max(0, min(kSliceUnits, units_total - (sp * SPW + j) * kSliceUnits)); };
  // unit u of this wave's sequence: chunk j = u / (2 NT), tile t = (u / 2) % NT, unit ku = u % 2 of the chunk
  auto unit_ok = [&](int u) {
    const int j = u / (kSliceUnits * NT), t = (u / kSliceUnits) % NT, ku = u % kSliceUnits;
    return ku < chunk_units(j) && (tile0 + 4 * t) < NTILES;
  };
  auto unit_ptr = [&](int u) {
    const int j = u / (kSliceUnits * NT), t = (u / kSliceUnits) % NT, ku = u % kSliceUnits;
    return Wsw + (size_t)(sp * SPW + j) * NTILES * (kSliceUnits * 8) * 64 +
           ((size_t)(tile0 + 4 * t) * chunk_units(j) + ku) * 8 * 64 + lane;
  };

  uint4 wb[2][8];
  // first weight unit goes out before anything else: it depends on nothing
  if (unit_ok(0)) {
    const uint4* p = unit_ptr(0);
    load_unit<STREAM>(p, wb[0]);
  }

  f32x4 sum[NT][CT];
#pragma unroll
  for (int j = 0; j < SPW; ++j) {
    const int units = chunk_units(j);
    const int unit0 = (sp * SPW + j) * kSliceUnits;
    // the X chunk: this thread's items are (row m, 8 consecutive k)
    const int kgs = max(units, 1) * 32;    // groups of 8 k per row
    const int k0 = unit0 * kUnitK;
    constexpr int ITEMS = 4 * CT;          // 16*CT rows x 64 groups / 256 threads (a full chunk)
    float4 xa[ITEMS], xb[ITEMS];
    if (j > 0) __syncthreads();            // the previous chunk's fragments have been read
    if (units > 0) {
#pragma unroll
      for (int it = 0; it < ITEMS; ++it) {
        const int w = tid + 256 * it;
        const int m = w / kgs, kg = w - m * kgs;
        xa[it] = make_float4(0.f, 0.f, 0.f, 0.f);
        xb[it] = xa[it];
        if (w < 16 * CT * kgs && m < M) {
          const float4* xp = reinterpret_cast<const float4*>(X + (size_t)m * ldx + k0 + kg * 8);
          xa[it] = xp[0];
          xb[it] = xp[1];
        }
      }
    }
    // the norm gain of this thread's k group (every item of a thread has kg = lane)
    float4 g0 = make_float4(1.f, 1.f, 1.f, 1.f), g1 = g0;
    if (nrm.gain && units > 0) {
      const float4* gp = reinterpret_cast<const float4*>(nrm.gain + k0 + min(lane, kgs - 1) * 8);
      g0 = gp[0];
      g1 = gp[1];
    }

    // fp32 -> (x * gain) -> bf16 hi + lo, stored in B-fragment order
    if (units > 0) {
#pragma unroll
      for (int it = 0; it < ITEMS; ++it) {
        const int w = tid + 256 * it;                       // w < 16*CT*kgs is uniform per wave
        const int m = min(w / kgs, 16 * CT - 1), kg = w - (w / kgs) * kgs;
        if (w < 16 * CT * kgs) {
          const bool scale = nrm.gain && m < M;
          uint4 hi, lo;
          split_bf16x8(xa[it], xb[it], g0, g1, scale, hi, lo);
          const int kt = kg >> 2, g = kg & 3, ct = m >> 4, jj = m & 15;
          const int base = ((kt * CT + ct) * 2) * 64 + g * 16 + jj;
          lds[base] = hi;
          lds[base + 64] = lo;
        }
      }
    }
    __syncthreads();

#pragma unroll
    for (int t = 0; t < NT; ++t) {
      f32x4 acc[CT];
#pragma unroll
      for (int ct = 0; ct < CT; ++ct) acc[ct] = f32x4{0.f, 0.f, 0.f, 0.f};
      const bool tile_ok = (tile0 + 4 * t) < NTILES;
#pragma unroll
      for (int ku = 0; ku < kSliceUnits; ++ku) {
        const int u = (j * NT + t) * kSliceUnits + ku;
        // prefetch the next unit into the other buffer (it may belong to the next chunk)
        if (u + 1 < SPW * NT * kSliceUnits) {
          if (unit_ok(u + 1)) {
            const uint4* p = unit_ptr(u + 1);
            load_unit<STREAM>(p, wb[(u + 1) & 1]);
          }
        }
        if (ku < units && tile_ok) {
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            const bf16x8 a = __builtin_bit_cast(bf16x8, wb[u & 1][i]);
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) {
              const int base = (((ku * 8 + i) * CT + ct) * 2) * 64 + lane;
              const bf16x8 bh = __builtin_bit_cast(bf16x8, lds[base]);
              const bf16x8 bl = __builtin_bit_cast(bf16x8, lds[base + 64]);
              acc[ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, bh, acc[ct], 0, 0, 0);
              acc[ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, bl, acc[ct], 0, 0, 0);
            }
          }
        }
      }
      // chunk sums of a pair are added once, first + second
#pragma unroll
      for (int ct = 0; ct < CT; ++ct) {
        if (j == 0) {
          sum[t][ct] = acc[ct];
        } else if (units > 0) {
          sum[t][ct][0] += acc[ct][0]; sum[t][ct][1] += acc[ct][1];
          sum[t][ct][2] += acc[ct][2]; sum[t][ct][3] += acc[ct][3];
        }
      }
    }
  }

#pragma unroll
  for (int t = 0; t < NT; ++t) {
    if ((tile0 + 4 * t) < NTILES) {
      const int n = (tile0 + 4 * t) * 16 + 4 * (lane >> 4);
#pragma unroll
      for (int ct = 0; ct < CT; ++ct) {
        const int m = ct * 16 + (lane & 15);
        if (m < M) {
          float* dst = partial + ((size_t)sp * M + m) * N + n;
          st_dev2(dst, sum[t][ct][0], sum[t][ct][1]);
          st_dev2(dst + 2, sum[t][ct][2], sum[t][ct][3]);
        }
      }
    }
  }

  // split-K hand-off: the partial sums are out, take a ticket; the last arrival finishes the group
  if (!last_arrival(&epi.counters[blockIdx.x], SG, &s_last)) return;
  // the rows' 1/rms is needed here only: the work-group that finishes a column group forms it
  const bool normed = nrm.gain && nrm.ssq_part;
  if (normed) {
    rows_rstd<2 * CT>(nrm, M, K, s_rstd);
    __syncthreads();
  }
  gemm_epilogue<ROLE, 64 * NT, SPW == 1>(partial, SG, M, N, blockIdx.x * 64 * NT, epi, normed ? s_rstd : nullptr);
  if (tid == 0) epi.counters[blockIdx.x] = 0;   // ready for the next launch on this stream
}

// ---------------------------------------------------------------------------------------
// The same GEMM for R <= 4 rows when the whole X block fits in LDS (K * R * 4 bytes): one work-group owns ONE
// 16-row weight tile over the whole k range, its four waves split the 512-wide k chunks between them, the chunk
// sums meet in LDS and the epilogue follows in the same work-group.  No partial sums in memory and no hand-off
// between work-groups, so the tail of one work-group overlaps the streaming of the others.  Chunk boundaries,
// the MFMA order inside a chunk and the order in which the chunk sums are added are those of the split-K
// kernel: both give the same bits for a row.
//   LDS: X high parts [K/8][R] uint4, X low parts [K/8][R] uint4, chunk sums float [chunks][R][16]
// ---------------------------------------------------------------------------------------
// Sum of one element's chunk sums held in LDS (stride floats apart), in the order of slice_sum<true>: pairs first.
// 8 chunks are read before any is used.
__device__ __forceinline__ float lds_chunk_sum(const float* base, int stride, int nchunks) {
  float a = 0.f;
  for (int c0 = 0; c0 < nchunks; c0 += 8) {
    float v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = base[min(c0 + i, nchunks - 1) * stride];
#pragma unroll
    for (int i = 0; i < 8; i += 2)
      if (c0 + i < nchunks) a += (c0 + i + 1 < nchunks) ? (v[i] + v[i + 1]) : v[i];
  }
  return a;
}

template <int R, int ROLE, int NW, int GP, bool STREAM>
__global__ __launch_bounds__(64 * NW) void k_gemm_bf16_rows(const uint4* __restrict__ Wsw, int NTILES,
                                                            const float* __restrict__ X, int ldx, RowNorm nrm,
                                                            int K, int N, GemmEpi epi) {
  // NW waves; GP = k groups a thread takes in the first staging pass (covers K <= 8 * 64 * NW * GP)
  constexpr int NTH = 64 * NW;
  extern __shared__ uint4 lds[];
  __shared__ float s_rstd[8];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // a work-group takes the tiles blockIdx.x, blockIdx.x + gridDim.x, ...: the X block is staged once for all of them
  int cur_tile = blockIdx.x;
  const int KG = K >> 3;                                   // groups of 8 k per row
  const int units_total = K / kUnitK;
  const int nchunks = (units_total + kSliceUnits - 1) / kSliceUnits;
  const int cpw = (nchunks + NW - 1) / NW;                 // chunks per wave
  const int c_begin = min(wave * cpw, nchunks), c_end = min(nchunks, c_begin + cpw);
  const int nu = min(units_total, c_end * kSliceUnits) - c_begin * kSliceUnits;   // this wave's units (<= 0: none)

  // address of unit u of this wave: chunk c_begin + u/2 (= split-K slice), unit u%2 inside it
  auto unit_ptr = [&](int u) {
    const int c = c_begin + (u >> 1);
    const int units_c = min(kSliceUnits, units_total - c * kSliceUnits);
    return Wsw + (size_t)c * NTILES * (kSliceUnits * 8) * 64 + ((size_t)cur_tile * units_c + (u & 1)) * 8 * 64 + lane;
  };

  // first pass over the X block: a thread takes all R rows of k group kg (the gain is per k, so it is fetched
  // once).  These loads (x, gain, row statistics) go out before the weights, so they are not queued behind them.
  float4 xa[GP][R], xb[GP][R], ga[GP], gb[GP];
#pragma unroll
  for (int j = 0; j < GP; ++j) {
    const int kg = tid + NTH * j;
    ga[j] = make_float4(1.f, 1.f, 1.f, 1.f);
    gb[j] = ga[j];
#pragma unroll
    for (int m = 0; m < R; ++m) {
      xa[j][m] = make_float4(0.f, 0.f, 0.f, 0.f);
      xb[j][m] = xa[j][m];
    }
    // no condition around the loads (a k group past the end re-reads the last one and is dropped later): the
    // compiler can then count them exactly and later waits do not have to cover the weight loads as well
    const int kgc = min(kg, KG - 1);
#pragma unroll
    for (int m = 0; m < R; ++m) {
      const float4* xp = reinterpret_cast<const float4*>(X + (size_t)m * ldx + kgc * 8);
      xa[j][m] = xp[0];
      xb[j][m] = xp[1];
    }
    if (nrm.gain) {
      const float4* gp = reinterpret_cast<const float4*>(nrm.gain + kgc * 8);
      ga[j] = gp[0];
      gb[j] = gp[1];
    }
  }
  // row statistics: half a wave per row (R <= 8 rows: the first (R + 1) / 2 waves).  The first 256 partials of the row are
  // requested here, without conditions (indices clamped, values masked later), and added up after the conversion of
  // the X block, in the order rows_rstd uses: the 1/rms multiplies the finished sums in the epilogue.
  const bool has_stats = nrm.gain && nrm.ssq_part;
  const int st_row = 2 * wave + (lane >> 5), st_pl = lane & 31;
  float sv[8];
  if (has_stats) {
    const float* sp = nrm.ssq_part + (size_t)min(st_row, R - 1) * nrm.ssq_n;
#pragma unroll
    for (int i = 0; i < 8; ++i) sv[i] = sp[min(st_pl + 32 * i, nrm.ssq_n - 1)];
  }

  // the wave's first two weight units, again without conditions: a wave with fewer units (short K) loads a valid
  // unit it will not use
  uint4 wb0[8], wb1[8];
  // (a macro, not a lambda: register arrays a lambda captures by reference end up in scratch memory)
#define STAIRS_FIRST_UNITS()                                                                                              \
  do {                                                                                                                    \
    const uint4* p0 = (nu > 0) ? unit_ptr(0) : Wsw + (size_t)cur_tile * min(kSliceUnits, units_total) * 8 * 64 + lane;   \
    const uint4* p1 = (nu > 1) ? unit_ptr(1) : p0;                                                                        \
    load_unit<STREAM>(p0, wb0);                                                                                           \
    load_unit<STREAM>(p1, wb1);                                                                                           \
  } while (0)
  STAIRS_FIRST_UNITS();
  uint4* xhi = lds;
  uint4* xlo = lds + KG * R;
  float* csum = reinterpret_cast<float*>(lds + 2 * KG * R); // [chunk][R][16]
  float* sq = csum + nchunks * R * 16;                      // [R][16], residual-writing roles only
  const bool scale = nrm.gain != nullptr;
#pragma unroll
  for (int j = 0; j < GP; ++j) {
    const int kg = tid + NTH * j;
    if (kg < KG) {
#pragma unroll
      for (int m = 0; m < R; ++m) {
        uint4 hi, lo;
        split_bf16x8(xa[j][m], xb[j][m], ga[j], gb[j], scale, hi, lo);
        xhi[kg * R + m] = hi;
        xlo[kg * R + m] = lo;
      }
    }
  }
  // further passes (longer K): same thing, loads and conversion back to back
  for (int kg = NTH * GP + tid; kg < KG; kg += NTH) {
    float4 g0 = make_float4(1.f, 1.f, 1.f, 1.f), g1 = g0;
    if (scale) {
      const float4* gp = reinterpret_cast<const float4*>(nrm.gain + kg * 8);
      g0 = gp[0];
      g1 = gp[1];
    }
#pragma unroll
    for (int m = 0; m < R; ++m) {
      const float4* xp = reinterpret_cast<const float4*>(X + (size_t)m * ldx + kg * 8);
      uint4 hi, lo;
      split_bf16x8(xp[0], xp[1], g0, g1, scale, hi, lo);
      xhi[kg * R + m] = hi;
      xlo[kg * R + m] = lo;
    }
  }
  if (has_stats && wave < (R + 1) / 2) {                   // wave-uniform
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) ss += (st_pl + 32 * i < nrm.ssq_n) ? sv[i] : 0.f;
    if (st_row < R) {
      for (int p0 = st_pl + 256; p0 < nrm.ssq_n; p0 += 256) {
        float v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = (p0 + 32 * i < nrm.ssq_n) ? nrm.ssq_part[st_row * nrm.ssq_n + p0 + 32 * i] : 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) ss += v[i];
      }
    }
#pragma unroll
    for (int off = 16; off >= 1; off >>= 1) ss += __shfl_xor(ss, off);
    if (st_pl == 0 && st_row < R) s_rstd[st_row] = 1.0f / sqrtf(ss / (float)K + nrm.eps);
  }
  __syncthreads();

  // B fragment of lane l at k-step kt: row (l & 15) of X (lanes of rows >= R take row 0; their columns of the
  // result are never read), k group kt*4 + (l >> 4)
  const int bofs = (lane >> 4) * R + (((lane & 15) < R) ? (lane & 15) : 0);
  auto mfma_unit = [&](const uint4 (&wb)[8], int u, f32x4& acc) {
    const int kt0 = ((c_begin + (u >> 1)) * kSliceUnits + (u & 1)) * 8;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const bf16x8 a = __builtin_bit_cast(bf16x8, wb[i]);
      const int idx = (kt0 + i) * 4 * R + bofs;
      const bf16x8 bh = __builtin_bit_cast(bf16x8, xhi[idx]);
      const bf16x8 bl = __builtin_bit_cast(bf16x8, xlo[idx]);
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, bh, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, bl, acc, 0, 0, 0);
    }
  };
  // the roles whose epilogue loads nothing from memory request the next tile's first units before it (a load in
  // the epilogue would have to wait for them)
  constexpr bool kPrefetchNextTile = ROLE == kRoleGateUp || ROLE == kRoleHead || ROLE == kRoleQKV;
  // (QKV: what its epilogue loads -- the row's position, the rotation entry -- is requested before that)
  int q_pos = 0;
  if (ROLE == kRoleQKV && tid < R * 8) q_pos = pos_of(epi.pos, tid >> 3);
  for (;;) {
  const int tile = cur_tile;
  for (int u = 0; u < nu; u += 2) {                        // one chunk per pass
    f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
    mfma_unit(wb0, u, acc);
    if (u + 2 < nu) {
      const uint4* p = unit_ptr(u + 2);
      load_unit<STREAM>(p, wb0);
    }
    if (u + 1 < nu) {
      mfma_unit(wb1, u + 1, acc);
      if (u + 3 < nu) {
        const uint4* p = unit_ptr(u + 3);
        load_unit<STREAM>(p, wb1);
      }
    }
    const int m = lane & 15;
    if (m < R) {
      float* dst = csum + (((c_begin + (u >> 1)) * R + m) << 4) + 4 * (lane >> 4);
      dst[0] = acc[0]; dst[1] = acc[1]; dst[2] = acc[2]; dst[3] = acc[3];
    }
  }
  float2 q_cs = make_float2(1.f, 0.f);
  if (ROLE == kRoleQKV && tid < R * 8) q_cs = epi.rope_cs[qkv_rope_index(tid >> 3, tile * 16 + (tid & 7), N / 3, epi.hd)];
  __builtin_amdgcn_sched_barrier(0);                       // these requests stay in front of the next tile's
  const int next_tile = tile + (int)gridDim.x;
  if (kPrefetchNextTile && next_tile < NTILES) {
    cur_tile = next_tile;
    STAIRS_FIRST_UNITS();
  }
  __syncthreads();

  if (ROLE == kRoleWo || ROLE == kRoleDown) {
    // a thread takes one element of the tile; then one thread per row adds the 16 squares up in the order of
    // the split-K kernel's epilogue
    if (tid < R * 16) {
      const int m = tid >> 4, n = tid & 15;
      float a = lds_chunk_sum(csum + (m << 4) + n, R * 16, nchunks);
      if (has_stats) a *= s_rstd[m];
      float* xp = epi.out + (size_t)m * N + tile * 16 + n;
      a += *xp;
      *xp = a;
      sq[tid] = a;
    }
    __syncthreads();
    if (tid < R) {
      const float* q = sq + tid * 16;
      const float s0 = sumsq4(q[0], q[1], q[2], q[3]), s1 = sumsq4(q[4], q[5], q[6], q[7]);
      const float s2 = sumsq4(q[8], q[9], q[10], q[11]), s3 = sumsq4(q[12], q[13], q[14], q[15]);
      epi.ssq_out[tid * (N >> 4) + tile] = (s0 + s1) + (s2 + s3);
    }
    // more than 4 rows: the next projection may take the kernel that reads activation fragments
    if (R > 4 && epi.frag_out && tid >= 64 && tid < 64 + R * 4) {
      const int t = tid - 64, m = t >> 2, q = (t & 3) * 4;
      const float* v = sq + m * 16 + q;
      store_frag4(epi.frag_out, m, tile * 16 + q, make_float4(v[0], v[1], v[2], v[3]), epi.frag_gain);
    }
  } else if (tid < R * 8) {                                // a thread takes row m, columns j and j+8 of the tile
    const int m = tid >> 3, j = tid & 7;
    float a = lds_chunk_sum(csum + (m << 4) + j, R * 16, nchunks);
    float b = lds_chunk_sum(csum + (m << 4) + j + 8, R * 16, nchunks);
    if (has_stats) {
      a *= s_rstd[m];
      b *= s_rstd[m];
    }
    const int col = tile * 16 + j;
    // (more than 4 rows: also the result's activation fragments -- the four threads of columns 4q .. 4q+3 sit in
    // adjacent lanes of wave 0, which holds all R * 8 <= 64 threads of this branch)
    const int l4 = lane & ~3;
    if (ROLE == kRoleHead) {
      const bool relu = epi.act == kActRelu;
      if (relu) {
        a = fmaxf(a, 0.f);
        b = fmaxf(b, 0.f);
      }
      epi.out[(size_t)m * N + col] = a;
      epi.out[(size_t)m * N + col + 8] = b;
      if (R > 4 && epi.frag_out) {
        const float4 va = make_float4(__shfl(a, l4), __shfl(a, l4 + 1), __shfl(a, l4 + 2), __shfl(a, l4 + 3));
        const float4 vb = make_float4(__shfl(b, l4), __shfl(b, l4 + 1), __shfl(b, l4 + 2), __shfl(b, l4 + 3));
        if ((j & 3) == 0) {
          store_frag4(epi.frag_out, m, col, va, epi.frag_gain);
          store_frag4(epi.frag_out, m, col + 8, vb, epi.frag_gain);
        }
      }
    } else if (ROLE == kRoleGateUp) {
      const float o = swiglu(a, b);
      epi.out[(size_t)m * (N >> 1) + tile * 8 + j] = o;
      if (R > 4 && epi.frag_out) {
        const float4 vo = make_float4(__shfl(o, l4), __shfl(o, l4 + 1), __shfl(o, l4 + 2), __shfl(o, l4 + 3));
        if ((j & 3) == 0) store_frag4(epi.frag_out, m, tile * 8 + j, vo, nullptr);
      }
    } else {
      qkv_pair_at(a, b, m, col, N / 3, epi, q_pos, q_cs);
    }
  }
  if (next_tile >= NTILES) break;
  if (!kPrefetchNextTile) {
    cur_tile = next_tile;
    STAIRS_FIRST_UNITS();
  }
  __syncthreads();                                         // the chunk sums are free for the next tile
  }
#undef STAIRS_FIRST_UNITS
}

// ---------------------------------------------------------------------------------------
// The hand-off-free GEMM for more than 4 rows (M <= 32): a work-group owns NT adjacent 16-row weight tiles over the
// WHOLE k range, its waves split the 512-wide k chunks between them, and a wave feeds every k-step's weight tiles
// with the activation fragments their producer left in memory (see frag_off): per k-step NT coalesced 1 KiB reads of
// weights (HBM) and 2 CT of fragments (L2), no conversion, nothing staged in LDS, no barrier before the first MFMA.
// A fragment is shared by the wave's NT tiles.  The chunk sums meet in LDS as in k_gemm_bf16_rows and the epilogue
// runs in the same work-group: no partial sums in memory, no ticket.  Chunk boundaries, the MFMA order inside a chunk
// and the order of the chunk sums are those of the other two kernels: all three give the same bits for a row.
//   CT = 16-row column tiles (rows of x) per MFMA pass: 1 (M <= 16) or 2; DEPTH = k-steps whose loads are in flight
//   LDS: chunk sums float [chunks][M][NT * 16]
// The epilogue can leave the fragments of ITS result for the next projection (epi.frag_out, with epi.frag_gain
// folded in): residual stream and SwiGLU output.
// ---------------------------------------------------------------------------------------
// 1/rms of the rows for a work-group of any size: half a wave per row, the additions in the order of rows_rstd
__device__ __forceinline__ void rows_rstd_any(const RowNorm& nrm, int M, int K, float* s_rstd) {
  const int pl = threadIdx.x & 31, hw = threadIdx.x >> 5, nhw = blockDim.x >> 5;
  for (int m = hw; m < M; m += nhw) {
    const float* sp = nrm.ssq_part + (size_t)m * nrm.ssq_n;
    float v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = sp[min(pl + 32 * i, nrm.ssq_n - 1)];
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) ss += (pl + 32 * i < nrm.ssq_n) ? v[i] : 0.f;
    for (int p0 = pl + 256; p0 < nrm.ssq_n; p0 += 256) {
      float u[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) u[i] = (p0 + 32 * i < nrm.ssq_n) ? sp[p0 + 32 * i] : 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) ss += u[i];
    }
#pragma unroll
    for (int off = 16; off >= 1; off >>= 1) ss += __shfl_xor(ss, off);
    if (pl == 0) s_rstd[m] = 1.0f / sqrtf(ss / (float)K + nrm.eps);
  }
}

// The epilogue of gemm_epilogue with the chunk sums in LDS ([chunk][M][W] floats) instead of partial sums in memory;
// run by all threads of the work-group.  The additions are those of slice_sum<true>: chunk pairs first.
template <int ROLE, int W>
__device__ __forceinline__ void gemm_epilogue_lds(const float* csum, int nchunks, int M, int N, int c0, const GemmEpi& epi,
                                                  const float* rs) {
  const int tid = threadIdx.x, nth = blockDim.x;
  const int cstride = M * W;
  auto sum4 = [&](int m, int lc) {
    const float* src = csum + m * W + lc;
    float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int c = 0; c < nchunks; c += 2) {
      const float4 p = *reinterpret_cast<const float4*>(src + c * cstride);
      if (c + 1 < nchunks) {
        const float4 q = *reinterpret_cast<const float4*>(src + (c + 1) * cstride);
        a.x += p.x + q.x; a.y += p.y + q.y; a.z += p.z + q.z; a.w += p.w + q.w;
      } else {
        a.x += p.x; a.y += p.y; a.z += p.z; a.w += p.w;
      }
    }
    return a;
  };
  auto sum1 = [&](int m, int lc) {
    const float* src = csum + m * W + lc;
    float a = 0.f;
    for (int c = 0; c < nchunks; c += 2) a += (c + 1 < nchunks) ? (src[c * cstride] + src[(c + 1) * cstride]) : src[c * cstride];
    return a;
  };
  if (ROLE == kRoleHead) {
    constexpr int PR = W / 4;
    for (int idx = tid; idx < M * PR; idx += nth) {
      const int m = idx / PR, lc = (idx - m * PR) * 4, col = c0 + lc;
      if (col < N) {
        float4 a = sum4(m, lc);
        if (rs) { const float r = rs[m]; a.x *= r; a.y *= r; a.z *= r; a.w *= r; }
        if (epi.act == kActRelu) a = make_float4(fmaxf(a.x, 0.f), fmaxf(a.y, 0.f), fmaxf(a.z, 0.f), fmaxf(a.w, 0.f));
        *reinterpret_cast<float4*>(epi.out + (size_t)m * N + col) = a;
        if (epi.frag_out) store_frag4(epi.frag_out, m, col, a, epi.frag_gain);
      }
    }
  } else if (ROLE == kRoleWo || ROLE == kRoleDown) {
    constexpr int PR = W / 4;                       // 4 adjacent threads = one 16-column tile
    const int total = M * PR;
    for (int idx0 = 0; idx0 < total; idx0 += nth) {
      const int idx = idx0 + tid;
      const int m = idx / PR, lc = (idx - m * PR) * 4, col = c0 + lc;
      float ss = 0.f;
      if (idx < total && col < N) {
        float4 a = sum4(m, lc);
        if (rs) { const float q = rs[m]; a.x *= q; a.y *= q; a.z *= q; a.w *= q; }
        float4* xp = reinterpret_cast<float4*>(epi.out + (size_t)m * N + col);
        const float4 r = *xp;
        a.x += r.x; a.y += r.y; a.z += r.z; a.w += r.w;
        *xp = a;
        ss = sumsq4(a.x, a.y, a.z, a.w);
        if (epi.frag_out) store_frag4(epi.frag_out, m, col, a, epi.frag_gain);
      }
      ss += __shfl_xor(ss, 1);
      ss += __shfl_xor(ss, 2);
      if (idx < total && col < N && (idx & 3) == 0) epi.ssq_out[m * (N >> 4) + (col >> 4)] = ss;
    }
  } else if (ROLE == kRoleGateUp) {
    constexpr int PR = W / 8;
    const int f = N / 2;
    for (int idx = tid; idx < M * PR; idx += nth) {
      const int m = idx / PR, r = idx - m * PR;
      const int lc = 16 * (r >> 1) + 4 * (r & 1), gcol = c0 + lc;
      if (gcol < N) {
        float4 g = sum4(m, lc);
        float4 u = sum4(m, lc + 8);
        if (rs) {
          const float q = rs[m];
          g.x *= q; g.y *= q; g.z *= q; g.w *= q;
          u.x *= q; u.y *= q; u.z *= q; u.w *= q;
        }
        const float4 o = make_float4(swiglu(g.x, u.x), swiglu(g.y, u.y), swiglu(g.z, u.z), swiglu(g.w, u.w));
        *reinterpret_cast<float4*>(epi.out + (size_t)m * f + (gcol >> 4) * 8 + (gcol & 7)) = o;
        if (epi.frag_out) store_frag4(epi.frag_out, m, (gcol >> 4) * 8 + (gcol & 7), o, nullptr);
      }
    }
  } else {   // kRoleQKV
    constexpr int PR = W / 2;
    for (int idx = tid; idx < M * PR; idx += nth) {
      const int m = idx / PR, r = idx - m * PR;
      const int lc = 16 * (r >> 3) + (r & 7), col = c0 + lc;
      if (col < N) {
        float a = sum1(m, lc);
        float b = sum1(m, lc + 8);
        if (rs) { a *= rs[m]; b *= rs[m]; }
        qkv_pair(a, b, m, col, N / 3, epi);
      }
    }
  }
}

template <int CT, int NT, int DEPTH, bool STREAM>
__global__ __launch_bounds__(512) void k_gemm_bf16_wide(const uint4* __restrict__ Wsw, int NTILES,
                                                        const uint4* __restrict__ XF, int M, RowNorm nrm, int K, int N,
                                                        int role, GemmEpi epi) {
  constexpr int RING = DEPTH + 1;
  constexpr int W = NT * 16;
  extern __shared__ float csum[];                          // [chunk][M][W]
  __shared__ float s_rstd[kMaxFwdRows];
  const int tid = threadIdx.x, lane = tid & 63, NW = blockDim.x >> 6;
  // (the wave index as a scalar: everything derived from it -- chunk, k-step, addresses -- is then scalar arithmetic)
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int j = lane & 15, g = lane >> 4;
  const int tile0 = blockIdx.x * NT;
  const int units_total = K / kUnitK;
  const int nchunks = (units_total + kSliceUnits - 1) / kSliceUnits;
  const int cpw = (nchunks + NW - 1) / NW;                 // chunks per wave
  const int c_begin = min(wave * cpw, nchunks), c_end = min(nchunks, c_begin + cpw);
  const int s_begin = c_begin * 16, s_end = min(K >> 5, c_end * 16);   // this wave's k-steps (32 k each)
  const bool has_stats = nrm.gain && nrm.ssq_part;

  struct Stage {
    uint4 a[NT], bh[CT], bl[CT];
  };
  // what a k-step needs, requested without conditions (tiles past the end re-read the last one and are dropped
  // later), so that the outstanding loads can be counted exactly
  int tile_c[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) tile_c[t] = min(tile0 + t, NTILES - 1);
  auto load_stage = [&](Stage& st, int s) {
    const int c = s >> 4, kk = s & 15;
    const int ksteps_c = min(kSliceUnits, units_total - c * kSliceUnits) * 8;
    const uint4* wbase = Wsw + (size_t)c * NTILES * (kSliceUnits * 8) * 64 + (size_t)kk * 64 + lane;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const uint4* p = wbase + (size_t)tile_c[t] * ksteps_c * 64;
      st.a[t] = STREAM ? ld_nt(p) : *p;
    }
    const uint4* xb = XF + (size_t)s * 4 * 64 + (size_t)c * kFragChunkPad + lane;
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {                      // column tiles 2, 3: the second fragment block
      const uint4* xc = xb + (size_t)(ct >> 1) * kFragHalfU4 + ((ct & 1) * 2) * 64;
      st.bh[ct] = xc[0];
      st.bl[ct] = xc[64];
    }
  };

  f32x4 acc[NT][CT];
  auto compute_stage = [&](const Stage& st, int s) {
    if ((s & 15) == 0) {
#pragma unroll
      for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) acc[t][ct] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const bf16x8 a = __builtin_bit_cast(bf16x8, st.a[t]);
#pragma unroll
      for (int ct = 0; ct < CT; ++ct) {
        acc[t][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8, st.bh[ct]), acc[t][ct], 0, 0, 0);
        acc[t][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8, st.bl[ct]), acc[t][ct], 0, 0, 0);
      }
    }
    if ((s & 15) == 15 || s == s_end - 1) {                // the chunk is complete (the last one may be short)
      float* dst = csum + (size_t)(s >> 4) * M * W;
#pragma unroll
      for (int ct = 0; ct < CT; ++ct) {
        const int m = ct * 16 + j;
        if (m < M) {
#pragma unroll
          for (int t = 0; t < NT; ++t)
            *reinterpret_cast<float4*>(dst + m * W + t * 16 + 4 * g) =
                make_float4(acc[t][ct][0], acc[t][ct][1], acc[t][ct][2], acc[t][ct][3]);
        }
      }
    }
  };

  Stage st[RING];
  const bool work = s_begin < s_end;                       // (a wave without k chunks only helps in the epilogue)
  if (work) {
#pragma unroll
    for (int i = 0; i < DEPTH; ++i) load_stage(st[i], min(s_begin + i, s_end - 1));
  }
  // the rows' 1/rms, needed by the epilogue only: its loads go out behind the first weight requests and come back
  // (from L2) long before those
  if (has_stats) rows_rstd_any(nrm, M, K, s_rstd);
  if (work) {
    // whole turns of the ring without a condition around a request (a branch would make the compiler assume the
    // fewest outstanding loads at every join and wait for nearly all of them); the last DEPTH or fewer k-steps have
    // been requested by then
    int s = s_begin;
    for (; s + RING <= s_end; s += RING) {
#pragma unroll
      for (int i = 0; i < RING; ++i) {
        load_stage(st[(i + DEPTH) % RING], min(s + i + DEPTH, s_end - 1));
        __builtin_amdgcn_sched_barrier(0);         // the requests stay in front of the arithmetic they overlap with
        compute_stage(st[i], s + i);
      }
    }
#pragma unroll
    for (int i = 0; i < DEPTH; ++i)
      if (s + i < s_end) compute_stage(st[i], s + i);
  }
  __syncthreads();

  const float* rs = has_stats ? s_rstd : nullptr;
  const int c0 = tile0 * 16;
  switch (role) {
    case kRoleQKV: gemm_epilogue_lds<kRoleQKV, W>(csum, nchunks, M, N, c0, epi, rs); break;
    case kRoleWo:
    case kRoleDown: gemm_epilogue_lds<kRoleWo, W>(csum, nchunks, M, N, c0, epi, rs); break;
    case kRoleGateUp: gemm_epilogue_lds<kRoleGateUp, W>(csum, nchunks, M, N, c0, epi, rs); break;
    default: gemm_epilogue_lds<kRoleHead, W>(csum, nchunks, M, N, c0, epi, rs); break;
  }
}

// x [M, K] (row stride ldx) -> its fragments, gain folded in (nullptr: none): for activations whose producer does not
// leave them itself.  One thread per (row, 4 consecutive k).
__global__ __launch_bounds__(256) void k_split_frag(const float* __restrict__ X, int ldx, int M, int K,
                                                    const float* __restrict__ gain, uint4* __restrict__ frag) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  const int k4 = K >> 2;
  if (idx >= M * k4) return;
  const int m = idx / k4, k = (idx - m * k4) * 4;
  store_frag4(frag, m, k, *reinterpret_cast<const float4*>(X + (size_t)m * ldx + k), gain);
}
void launch_split_frag(const float* X, int ldx, int M, int K, const float* gain, uint4* frag, hipStream_t st) {
  hipLaunchKernelGGL(k_split_frag, dim3((M * (K / 4) + 255) / 256), dim3(256), 0, st, X, ldx, M, K, gain, frag);
}

// LDS bytes of k_gemm_bf16_rows, or 0 if this shape does not take that path.  The residual-writing projections
// have few weight tiles (N = d_model): they run one 8-wave work-group per CU and only when the tiles about
// cover the chip.
static size_t rows_path_lds(int role, int M, int N, int K) {
  static const int max_rows = [] { const char* e = getenv("STAIRS_ROWS_MAX"); return e ? atoi(e) : 7; }();   // tuning aid
  if (M > 7 || M > max_rows) return 0;
  const size_t bytes = (size_t)K * M * 4 + (size_t)(gemm_slices(K, 1) + 1) * M * 16 * 4;
  // 5..7 rows (at 8 the fragment-reading kernel is as fast): the block takes more than half a CU's LDS, so one work-group per CU walks through the tiles; only
  // with a k chunk for each of its waves (k >= 2048) does that beat the fragment-reading kernel
  if (M > 4)
    return (role != kRoleDown && bytes <= kRowsPathMaxLdsWide && N / 16 >= 192 && K >= 2048) ? std::max(bytes, (size_t)81 * 1024) : 0;
  if (role == kRoleWo || role == kRoleDown) {
    // few tiles: only matrices so small that the launch is latency-bound anyway (no partial sums, no hand-off)
    if (N / 16 < 192) {
      if ((size_t)N * K * 2 <= kRowsPathSmallMatrix) return bytes <= kRowsPathMaxLdsWide ? bytes : 0;
      // a larger matrix with few tiles but a long k range (down projection of a 1B-class model: 128 tiles x 16
      // chunks): 16 waves per work-group, a k chunk each -- half the CUs stream it faster than split-K work-groups
      // on all of them with their hand-off (measured: 12.4 -> 9.7 us per launch)
      return (role == kRoleDown && gemm_slices(K, 1) >= 12 && gemm_slices(K, 1) <= 16 && bytes <= kRowsPathMaxLdsWide)
                 ? std::max(bytes, (size_t)81 * 1024) : 0;
    }
    return bytes <= kRowsPathMaxLdsWide ? std::max(bytes, (size_t)81 * 1024) : 0;   // > half a CU's LDS: one per CU
  }
  return bytes <= kRowsPathMaxLds ? bytes : 0;
}

// Launch shape of k_gemm_bf16_wide: NT weight tiles per wave and NW waves that split the k chunks; nt == 0: the
// split-K kernel instead.  Measured on 7B-class projections (isolated launches, 8 / 17 rows, microseconds; split-K
// in brackets): gate/up 1376 tiles 8/4 33 / 36 (37 / 48), unembedding 2000 tiles 8/4 41 / 43 (48 / 63), QKV 768 tiles
// 4/4 21 / 25 (23 / 33), attention-out 256 tiles 1/8 10.4 / 13.4 (11.4 / 15.4), down 256 tiles and 22 chunks 1/4 23 /
// 32 (21 / 34).  More tiles per wave means fewer fragment reads and fewer, longer-lived waves per weight byte; with
// few tiles (N = d_model) that leaves too few work-groups, and for a long k at up to 16 rows split-K's extra
// parallelism still wins.
struct WideCfg { int nt, nw; };
constexpr int wide_depth2(int depth1) { return depth1 <= 2 ? 1 : depth1 <= 3 ? 2 : depth1 <= 5 ? 3 : 5; }   // ring depth at two column tiles
constexpr int wide_depth3(int depth1) { return depth1 <= 3 ? 1 : depth1 <= 5 ? 2 : 3; }                      // at three (33..48 rows)
constexpr int wide_depth4(int depth1) { return depth1 <= 3 ? 1 : 2; }                                        // at four (49..64 rows; 3 spills at one tile)
static WideCfg wide_cfg(int role, int M, int NTILES, int K) {
  // STAIRS_WIDE_CFG="nt/nw,nt/nw,nt/nw,nt/nw,nt/nw" (QKV, out, gate-up, down, head; nt = 0: split-K) overrides the
  // choice: tuning aid
  static const std::vector<WideCfg> forced = [] {
    std::vector<WideCfg> v;
    if (const char* e = getenv("STAIRS_WIDE_CFG")) {
      int nt = 0, nw = 0, n = 0;
      while (sscanf(e, "%d/%d%n", &nt, &nw, &n) == 2) {
        v.push_back({nt, nw});
        e += n;
        if (*e == ',') ++e;
      }
    }
    return v;
  }();
  const int nchunks = gemm_slices(K, 1);
  // Measured on the 125M, 1B and 7B workloads (5..32 rows): about one work-group per CU, i.e. the smallest number of
  // tiles per wave (1, 2, 3, 4, 6, 8) that covers the matrix with at most 256 work-groups, as long as about 170 remain
  // (7B: gate/up 1376 tiles -> 6, 230 work-groups: 29.6 us at 9 rows against 32.4 us for 172 work-groups of 8; QKV
  // 768 -> 3, 256 work-groups: 19.6 against 22.0 us for 192 of 4; unembedding 2000 -> 8); with one tile per wave up
  // to 8 waves share the k chunks, else 4 (8 and 2 measured slower).  Few tiles with a long k range (down projections:
  // 128 x 8192 at 1B, 256 x 11008 at 7B) stream better through the split-K kernel, whose grid also cuts k; from 17
  // rows on the 7B shape is the exception.  Small matrices are latency-bound either way and the missing hand-off is
  // what counts (125M at 16 rows: 595 -> 470 us per forward).
  WideCfg c{0, 0};
  if (nchunks > 8 && NTILES < 512) {
    if (NTILES >= 192 && M > 16) c = {1, 4};
  } else {
    static const int kNts[] = {1, 2, 3, 4, 6, 8};
    int i = 0;
    while (i < 5 && kNts[i] * 256 < NTILES) ++i;
    while (i > 0 && NTILES / kNts[i] < 170) --i;
    const int nt = kNts[i];
    c = {nt, std::min(nt == 1 ? 8 : 4, nchunks)};
  }
  if ((int)forced.size() == 5) {
    const WideCfg f = forced[role];
    if ((f.nt == 0 || f.nt == 1 || f.nt == 2 || f.nt == 3 || f.nt == 4 || f.nt == 6 || f.nt == 8) && f.nw >= 1 && f.nw <= 8) c = f;
  }
  if (M > 2 * 16) {                      // 33..64 rows: this kernel only (split-K stops at two column tiles)
    if (c.nt == 0) c = {1, 4};
    if (c.nt > 4) c.nt = 4;                 // (the three- and four-column-tile forms exist for 1, 2 and 4 tiles per wave)
    if (c.nt == 3) c.nt = 4;
  }
  return c;
}

// fp32 weights, row-major: one wave per output feature, lanes stride over k.
template <int MR>
__global__ __launch_bounds__(256) void k_gemm_f32(const float* __restrict__ W, int N, int K,
                                                  const float* __restrict__ X, int ldx, int M, RowNorm nrm,
                                                  float* __restrict__ partial) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = blockIdx.x * 4 + wave;
  if (n >= N) return;
  float rs[MR], acc[MR];
#pragma unroll
  for (int i = 0; i < MR; ++i) {
    acc[i] = 0.f;
    rs[i] = (nrm.gain && nrm.ssq_part && i < M) ? row_rstd(nrm, i, K) : 1.0f;
  }
  for (int k = lane * 4; k < K; k += 256) {
    const float4 w = *reinterpret_cast<const float4*>(W + (size_t)n * K + k);
    float4 g = make_float4(1.f, 1.f, 1.f, 1.f);
    if (nrm.gain) g = *reinterpret_cast<const float4*>(nrm.gain + k);
#pragma unroll
    for (int i = 0; i < MR; ++i) {
      if (i < M) {
        const float4 x = *reinterpret_cast<const float4*>(X + (size_t)i * ldx + k);
        float a = acc[i];
        a = fmaf(w.x, x.x * rs[i] * g.x, a);
        a = fmaf(w.y, x.y * rs[i] * g.y, a);
        a = fmaf(w.z, x.z * rs[i] * g.z, a);
        a = fmaf(w.w, x.w * rs[i] * g.w, a);
        acc[i] = a;
      }
    }
  }
#pragma unroll
  for (int i = 0; i < MR; ++i) {
    if (i < M) {
      const float v = wave_sum(acc[i]);
      if (lane == 0) partial[(size_t)i * N + n] = v;
    }
  }
}

// weight tiles per wave (1 or 2) of the split-K kernel: two when that still leaves enough work-groups to cover
// the chip a few times over (more tiles per work-group = fewer activation slices staged per weight byte)
static int pick_nt(int NTILES, int SG, int want_wgs) {
  return ((size_t)((NTILES + 7) / 8) * SG >= (size_t)want_wgs) ? 2 : 1;
}

// forward declarations of the unfused epilogues (fp32 models)
void launch_fin_plain(const float* partial, int S, int M, int N, float* out, int ldo, hipStream_t st);
void launch_fin_resid(const float* partial, int S, int M, int N, float* x, float* ssq_part, hipStream_t st);
void launch_fin_swiglu(const float* partial, int S, int M, int f, float* h, hipStream_t st);
void launch_fin_qkv_rope_f32(const float* partial, int S, int M, int d, int H, const float2* rope_cs, PosRef pos,
                             float* q_rot, float* Kc, float* Vc, int cap, hipStream_t st);

// Events the next GEMM launch records at the kernel's own start and end (set_gemm_launch_events): lets a measurement
// take one kernel's duration inside a running forward without event records around it in the stream.  (fp32 models
// run two kernels per projection: there the events are recorded around the pair.)
// (per thread: a context is used by one thread at a time)
static thread_local hipEvent_t g_gemm_ev_start = nullptr, g_gemm_ev_stop = nullptr;
void set_gemm_launch_events(hipEvent_t start, hipEvent_t stop) {
  g_gemm_ev_start = start;
  g_gemm_ev_stop = stop;
}
template <typename F, typename... Args>
static void launch_gemm_kernel(F kernel, dim3 grid, dim3 block, size_t lds, hipStream_t st, Args... args) {
  if (g_gemm_ev_start && g_gemm_ev_stop) {
    hipExtLaunchKernelGGL(kernel, grid, block, (std::uint32_t)lds, st, g_gemm_ev_start, g_gemm_ev_stop, 0, args...);
    g_gemm_ev_start = g_gemm_ev_stop = nullptr;
  } else {
    hipLaunchKernelGGL(kernel, grid, block, lds, st, args...);
  }
}

bool gemm_takes_rows(int M, int K) {
  return M <= kMaxFwdRows && (size_t)gemm_slices(K, 1) * M * 16 * sizeof(float) <= kWideMaxLds;
}

void launch_gemm(int role, int dtype_bf16, const void* W, int N, int K, const float* X, int ldx, int M, RowNorm nrm,
                 float* partial, const GemmEpi& epi, hipStream_t st, const uint4* xfrag) {
  if (!dtype_bf16) {
    dim3 grid((N + 3) / 4), block(256);
    const float* Wf = static_cast<const float*>(W);
    // two kernels here: requested launch events become records around the pair
    hipEvent_t ev_stop = nullptr;
    if (g_gemm_ev_start && g_gemm_ev_stop) {
      (void)hipEventRecord(g_gemm_ev_start, st);
      ev_stop = g_gemm_ev_stop;
      g_gemm_ev_start = g_gemm_ev_stop = nullptr;
    }
    if (M <= 4) hipLaunchKernelGGL(k_gemm_f32<4>, grid, block, 0, st, Wf, N, K, X, ldx, M, nrm, partial);
    else if (M <= 16) hipLaunchKernelGGL(k_gemm_f32<16>, grid, block, 0, st, Wf, N, K, X, ldx, M, nrm, partial);
    else hipLaunchKernelGGL(k_gemm_f32<32>, grid, block, 0, st, Wf, N, K, X, ldx, M, nrm, partial);
    switch (role) {
      case kRoleQKV:
        launch_fin_qkv_rope_f32(partial, 1, M, N / 3, epi.H, epi.rope_cs, epi.pos, epi.out, static_cast<float*>(epi.Kc32),
                                static_cast<float*>(epi.Vc32), epi.cap, st);
        break;
      case kRoleWo:
      case kRoleDown: launch_fin_resid(partial, 1, M, N, epi.out, epi.ssq_out, st); break;
      case kRoleGateUp: launch_fin_swiglu(partial, 1, M, N / 2, epi.out, st); break;
      default: launch_fin_plain(partial, 1, M, N, epi.out, N, st); break;
    }
    if (ev_stop) (void)hipEventRecord(ev_stop, st);
    return;
  }
  const int S = gemm_slices(K, 1);
  const int NTILES = N / 16, KT = K / 32;
  const uint4* Wsw = static_cast<const uint4*>(W);
  if (const size_t rl = rows_path_lds(role, M, N, K)) {
    // gate/up has several times more tiles than the chip has CUs: one work-group per CU that walks through its
    // share of the tiles (X block staged once, the next tile's first units requested before the epilogue, all
    // work-groups resident from the start and done together) streams better than a work-group per tile (7B, 1376
    // tiles, isolated: 30.1 -> 28.5 us at 3 rows with 230 work-groups of 6 tiles; 459 x 3: 29.1, 344 x 4: 32.5 -- two
    // work-groups on some CUs and one on others is the worst case; the unembedding's 2000 tiles and, with its
    // epilogue's loads requested early, QKV's 768 gain nothing)
    int tpw = 1;
    if ((role == kRoleGateUp && NTILES >= 4 * 256) || (M > 4 && NTILES > 256)) tpw = (NTILES + 255) / 256;
    {
      static const int forced = [] { const char* e = getenv("STAIRS_ROWS_TPW"); return e ? atoi(e) : 0; }();
      if (forced > 0 && (role == kRoleGateUp || role == kRoleHead)) tpw = forced;    // tuning aid
    }
    const dim3 rgrid((NTILES + tpw - 1) / tpw);
    // (walking work-groups ask for more than half a CU's LDS, so that no CU gets two of them while another has none)
    const size_t rl_launch = tpw > 1 ? std::max(rl, (size_t)81 * 1024) : rl;
#define STAIRS_ROWS(r, role, nw, gp)                                                                                  \
  do {                                                                                                                 \
  if (epi.stream_weights)                                                                                            \
    launch_gemm_kernel(k_gemm_bf16_rows<r, role, nw, gp, true>, rgrid, dim3(64 * nw), rl_launch, st, Wsw, NTILES, X,    \
                       ldx, nrm, K, N, epi);                                                                            \
  else                                                                                                                 \
    launch_gemm_kernel(k_gemm_bf16_rows<r, role, nw, gp, false>, rgrid, dim3(64 * nw), rl_launch, st, Wsw, NTILES, X,   \
                       ldx, nrm, K, N, epi);                                                                            \
  } while (0)
#define STAIRS_ROWS_ROLE4(role, nw, gp)          \
  if (M <= 1) STAIRS_ROWS(1, role, nw, gp);      \
  else if (M == 2) STAIRS_ROWS(2, role, nw, gp); \
  else if (M == 3) STAIRS_ROWS(3, role, nw, gp); \
  else STAIRS_ROWS(4, role, nw, gp)
#define STAIRS_ROWS_ROLE(role, nw, gp)                \
  if (M <= 4) { STAIRS_ROWS_ROLE4(role, nw, gp); }    \
  else if (M == 5) STAIRS_ROWS(5, role, nw, gp);      \
  else if (M == 6) STAIRS_ROWS(6, role, nw, gp);      \
  else STAIRS_ROWS(7, role, nw, gp)
    if (role == kRoleQKV) { STAIRS_ROWS_ROLE(kRoleQKV, 4, 2); }
    else if (role == kRoleGateUp) { STAIRS_ROWS_ROLE(kRoleGateUp, 4, 2); }
    else if (role == kRoleHead) { STAIRS_ROWS_ROLE(kRoleHead, 4, 2); }
    else if (role == kRoleWo) { STAIRS_ROWS_ROLE(kRoleWo, 8, 1); }
    else if (NTILES < 192 && (size_t)N * K * 2 > kRowsPathSmallMatrix) { STAIRS_ROWS_ROLE4(kRoleDown, 16, 1); }
    else { STAIRS_ROWS_ROLE4(kRoleDown, 8, 3); }           // (down never takes this path beyond 4 rows: its k is long)
#undef STAIRS_ROWS_ROLE
#undef STAIRS_ROWS_ROLE4
#undef STAIRS_ROWS
    return;
  }
  // more than 4 rows with the activation fragments at hand: the hand-off-free kernel
  WideCfg wc = wide_cfg(role, M, NTILES, K);
  const int nchunks = gemm_slices(K, 1);
  auto wide_lds = [&](int nt) { return (size_t)nchunks * M * nt * 16 * sizeof(float); };
  while (wc.nt > 1 && wide_lds(wc.nt) > kWideMaxLds) wc.nt = wc.nt == 6 ? 4 : wc.nt == 3 ? 2 : wc.nt / 2;   // very long k: fewer tiles per work-group
  if (xfrag && wc.nt > 0 && wide_lds(wc.nt) <= kWideMaxLds) {
    const int CT = (M + 15) / 16;
    dim3 grid((NTILES + wc.nt - 1) / wc.nt), block(64 * wc.nw);
    const size_t lds = wide_lds(wc.nt);
#define STAIRS_WIDE(ct, nt, dp)                                                                                          \
  do {                                                                                                                   \
    if (epi.stream_weights)                                                                                              \
      launch_gemm_kernel(k_gemm_bf16_wide<ct, nt, dp, true>, grid, block, lds, st, Wsw, NTILES, xfrag, M, nrm, K, N,     \
                         role, epi);                                                                                     \
    else                                                                                                                 \
      launch_gemm_kernel(k_gemm_bf16_wide<ct, nt, dp, false>, grid, block, lds, st, Wsw, NTILES, xfrag, M, nrm, K, N,    \
                         role, epi);                                                                                     \
  } while (0)
  // (two column tiles hold one k-step less in flight: a deeper ring would not fit the 256 registers of a wave)
  // (three and four column tiles: one more; 8 tiles per wave do not occur there, their chunk sums exceed the LDS)
#define STAIRS_WIDE_CT2(nt, dp)        \
  if (CT == 1) STAIRS_WIDE(1, nt, dp); \
  else STAIRS_WIDE(2, nt, wide_depth2(dp))
#define STAIRS_WIDE_CT(nt, dp)                          \
  if (CT <= 2) { STAIRS_WIDE_CT2(nt, dp); }             \
  else if (CT == 3) STAIRS_WIDE(3, nt, wide_depth3(dp)); \
  else STAIRS_WIDE(4, nt, wide_depth4(dp))
    if (wc.nt == 8) { STAIRS_WIDE_CT2(8, kWideDepth8); }
    else if (wc.nt == 6) { STAIRS_WIDE_CT2(6, kWideDepth6); }
    else if (wc.nt == 3) { STAIRS_WIDE_CT2(3, kWideDepth3); }
    else if (wc.nt == 4) { STAIRS_WIDE_CT(4, kWideDepth4); }
    else if (wc.nt == 2) { STAIRS_WIDE_CT(2, kWideDepth2); }
    else { STAIRS_WIDE_CT(1, kWideDepth1); }
#undef STAIRS_WIDE_CT
#undef STAIRS_WIDE_CT2
#undef STAIRS_WIDE
    return;
  }
  // 9..16 rows: a work-group takes two k chunks and writes the sum of the pair (half the partial sums in memory;
  // measured -7 % on a 7B layer at 16 rows).  With two column tiles (17..32 rows) the halved work-group count
  // or, with one weight tile per wave, the doubled activation staging cost more than the partial sums saved.
  const int CT = (M <= 16) ? 1 : 2;
  const int SPW = (M >= kSpwRows && CT == 1 && S >= 2) ? 2 : 1;
  const int SG = (S + SPW - 1) / SPW;
  int NT;
  if (SPW == 1) NT = (role == kRoleWo || role == kRoleDown) ? 2 : pick_nt(NTILES, SG, 1024);
  else NT = pick_nt(NTILES, SG, 640);
  dim3 grid((NTILES + 4 * NT - 1) / (4 * NT), SG), block(256);
  const size_t lds = (size_t)16 * CT * 2 * 64 * sizeof(uint4);
#define STAIRS_GEMM(ct, nt, role, spw) \
  do {                                                                                                                \
    if (epi.stream_weights)                                                                                           \
      launch_gemm_kernel(k_gemm_bf16<ct, nt, role, spw, true>, grid, block, lds, st, Wsw, KT, NTILES, X, ldx, M, nrm, K, \
                         partial, N, epi);                                                                            \
    else                                                                                                              \
      launch_gemm_kernel(k_gemm_bf16<ct, nt, role, spw, false>, grid, block, lds, st, Wsw, KT, NTILES, X, ldx, M, nrm,   \
                         K, partial, N, epi);                                                                         \
  } while (0)
#define STAIRS_GEMM_NT(ct, role, spw)             \
  if (NT == 1) STAIRS_GEMM(ct, 1, role, spw);     \
  else STAIRS_GEMM(ct, 2, role, spw)
#define STAIRS_GEMM_ROLE(role)                                  \
  if (CT == 1 && SPW == 1) { STAIRS_GEMM_NT(1, role, 1); }      \
  else if (CT == 1) { STAIRS_GEMM_NT(1, role, 2); }             \
  else { STAIRS_GEMM_NT(2, role, 1); }
  switch (role) {
    case kRoleQKV: STAIRS_GEMM_ROLE(kRoleQKV); break;
    case kRoleWo: STAIRS_GEMM_ROLE(kRoleWo); break;
    case kRoleGateUp: STAIRS_GEMM_ROLE(kRoleGateUp); break;
    case kRoleDown: STAIRS_GEMM_ROLE(kRoleDown); break;
    default: STAIRS_GEMM_ROLE(kRoleHead); break;
  }
#undef STAIRS_GEMM_NT
#undef STAIRS_GEMM_ROLE
#undef STAIRS_GEMM
}

// ---------------------------------------------------------------------------------------
// GEMM epilogues
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ float4 sum_slices4(const float* partial, int S, int M, int N, int m, int n) {
  float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int s = 0; s < S; ++s) {
    const float4 p = *reinterpret_cast<const float4*>(partial + ((size_t)s * M + m) * N + n);
    a.x += p.x; a.y += p.y; a.z += p.z; a.w += p.w;
  }
  return a;
}
__device__ __forceinline__ float sum_slices1(const float* partial, int S, int M, int N, int m, int n) {
  float a = 0.f;
  for (int s = 0; s < S; ++s) a += partial[((size_t)s * M + m) * N + n];
  return a;
}

__global__ __launch_bounds__(256) void k_fin_plain(const float* __restrict__ partial, int S, int M, int N,
                                                   float* __restrict__ out, int ldo) {
  const int n = (blockIdx.x * 256 + threadIdx.x) * 4, m = blockIdx.y;
  if (n >= N) return;
  *reinterpret_cast<float4*>(out + (size_t)m * ldo + n) = sum_slices4(partial, S, M, N, m, n);
}

__global__ __launch_bounds__(256) void k_fin_resid(const float* __restrict__ partial, int S, int M, int N,
                                                   float* __restrict__ x, float* __restrict__ ssq_part) {
  __shared__ float sm[4];
  const int n = (blockIdx.x * 256 + threadIdx.x) * 4, m = blockIdx.y;
  float ss = 0.f;
  if (n < N) {
    float4 a = sum_slices4(partial, S, M, N, m, n);
    float4* xp = reinterpret_cast<float4*>(x + (size_t)m * N + n);
    const float4 r = *xp;
    a.x += r.x; a.y += r.y; a.z += r.z; a.w += r.w;
    *xp = a;
    ss = (a.x * a.x + a.y * a.y) + (a.z * a.z + a.w * a.w);
  }
  ss = block_sum_256(ss, sm);
  if (threadIdx.x == 0) ssq_part[m * gridDim.x + blockIdx.x] = ss;
}

__global__ __launch_bounds__(256) void k_fin_swiglu(const float* __restrict__ partial, int S, int M, int f,
                                                    float* __restrict__ h) {
  const int j = (blockIdx.x * 256 + threadIdx.x) * 4, m = blockIdx.y;
  if (j >= f) return;
  const float4 g = sum_slices4(partial, S, M, 2 * f, m, j);
  const float4 u = sum_slices4(partial, S, M, 2 * f, m, f + j);
  float4 o;
  o.x = g.x / (1.0f + expf(-g.x)) * u.x;
  o.y = g.y / (1.0f + expf(-g.y)) * u.y;
  o.z = g.z / (1.0f + expf(-g.z)) * u.z;
  o.w = g.w / (1.0f + expf(-g.w)) * u.w;
  *reinterpret_cast<float4*>(h + (size_t)m * f + j) = o;
}

template <typename KV>
__global__ __launch_bounds__(256) void k_fin_qkv_rope(const float* __restrict__ partial, int S, int M, int d, int H,
                                                      const float2* __restrict__ rope_cs, PosRef pos,
                                                      float* __restrict__ q_rot, KV* __restrict__ Kc,
                                                      KV* __restrict__ Vc, int cap) {
  const int hd = d / H, half = hd / 2;
  const int per_row = 3 * H * half;
  const int idx = blockIdx.x * 256 + threadIdx.x;
  const int m = blockIdx.y;
  if (idx >= per_row) return;
  const int e = idx % half;
  const int h = (idx / half) % H;
  const int which = idx / (half * H);
  const int p = *pos.base + pos.offset + m;
  if (p < 0) return;
  const int N = 3 * d;
  const int col = which * d + h * hd + e;
  const float a = sum_slices1(partial, S, M, N, m, col);
  const float b = sum_slices1(partial, S, M, N, m, col + half);
  if (which == 2) {
    KV* dst = Vc + ((size_t)h * cap + p) * hd + e;
    store_kv(dst, a);
    store_kv(dst + half, b);
    return;
  }
  const float2 cs = rope_cs[m * 64 + e];
  const float ra = a * cs.x - b * cs.y;
  const float rb = b * cs.x + a * cs.y;
  if (which == 0) {
    q_rot[(size_t)m * d + h * hd + e] = ra;
    q_rot[(size_t)m * d + h * hd + e + half] = rb;
  } else {
    KV* dst = Kc + ((size_t)h * cap + p) * hd + e;
    store_kv(dst, ra);
    store_kv(dst + half, rb);
  }
}

void launch_fin_plain(const float* partial, int S, int M, int N, float* out, int ldo, hipStream_t st) {
  hipLaunchKernelGGL(k_fin_plain, dim3((N / 4 + 255) / 256, M), dim3(256), 0, st, partial, S, M, N, out, ldo);
}
void launch_fin_resid(const float* partial, int S, int M, int N, float* x, float* ssq_part, hipStream_t st) {
  hipLaunchKernelGGL(k_fin_resid, dim3(ssq_groups(N, 0), M), dim3(256), 0, st, partial, S, M, N, x, ssq_part);
}
void launch_fin_swiglu(const float* partial, int S, int M, int f, float* h, hipStream_t st) {
  hipLaunchKernelGGL(k_fin_swiglu, dim3((f / 4 + 255) / 256, M), dim3(256), 0, st, partial, S, M, f, h);
}
void launch_fin_qkv_rope_f32(const float* partial, int S, int M, int d, int H, const float2* rope_cs, PosRef pos,
                             float* q_rot, float* Kc, float* Vc, int cap, hipStream_t st) {
  const int per_row = 3 * H * (d / H / 2);
  dim3 grid((per_row + 255) / 256, M), block(256);
  hipLaunchKernelGGL(k_fin_qkv_rope<float>, grid, block, 0, st, partial, S, M, d, H, rope_cs, pos, q_rot, Kc, Vc, cap);
}

// ---------------------------------------------------------------------------------------
// embedding gather, rope table
// ---------------------------------------------------------------------------------------
// GW = residual columns per sum-of-squares partial: 1024 (one per block) or 16 (one per 4 lanes)
// The block column after the last embedding column fills the row's rotation table instead:
// cs[m][i] = (cos, sin)(position * theta^(-2i/hd)), the angle formed in double.
// A row whose position lies outside [0, tok_cap) or whose token id lies outside [0, vocab) becomes a row of zeros:
// the gather never leaves the token array or the embedding table, whatever the array holds.
template <typename E, int GW>
__global__ __launch_bounds__(256) void k_embed(const E* __restrict__ emb, const int* __restrict__ tokens,
                                               int tok_slot_stride, int tok_cap, int vocab, PosRef pos, int d,
                                               float* __restrict__ x, float* __restrict__ ssq_part, int ssq_n, int hd,
                                               double theta, float2* __restrict__ cs, uint4* frag,
                                               const float* __restrict__ frag_gain) {
  __shared__ float sm[4];
  const int m = blockIdx.y;
  const int p = pos_of(pos, m);
  tokens += (size_t)slot_of(pos, m) * tok_slot_stride;
  if (blockIdx.x == gridDim.x - 1) {
    const int i = threadIdx.x;
    if (i < hd / 2) {
      const double ang = (double)p * pow(theta, -2.0 * (double)i / (double)hd);
      cs[m * 64 + i] = theta > 0.0 ? make_float2((float)cos(ang), (float)sin(ang)) : make_float2(1.f, 0.f);
    }
    return;
  }
  const int c = (blockIdx.x * 256 + threadIdx.x) * 4;
  float ss = 0.f;
  if (c < d) {
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    const int id = (p >= 0 && p < tok_cap) ? tokens[p] : -1;
    if (id >= 0 && id < vocab) {
      const E* row = emb + (size_t)id * d + c;
      v.x = load_kv(row); v.y = load_kv(row + 1); v.z = load_kv(row + 2); v.w = load_kv(row + 3);
    }
    *reinterpret_cast<float4*>(x + (size_t)m * d + c) = v;
    ss = (v.x * v.x + v.y * v.y) + (v.z * v.z + v.w * v.w);
    if (frag) store_frag4(frag, m, c, v, frag_gain);
  }
  if (GW == 1024) {
    ss = block_sum_256(ss, sm);
    if (threadIdx.x == 0) ssq_part[m * ssq_n + blockIdx.x] = ss;
  } else {
    ss += __shfl_xor(ss, 1);
    ss += __shfl_xor(ss, 2);
    if ((threadIdx.x & 3) == 0 && c < d) ssq_part[m * ssq_n + c / 16] = ss;
  }
}

void launch_embed(const void* emb, int emb_bf16, const int* tokens, int tok_slot_stride, int tok_cap, int vocab, PosRef pos,
                  int M, int d, float* x, float* ssq_part, int hd, float theta, float2* cs, hipStream_t st, uint4* frag,
                  const float* frag_gain) {
  dim3 grid((d + 1023) / 1024 + 1, M), block(256);
  const int sn = ssq_groups(d, emb_bf16);
  if (emb_bf16)
    hipLaunchKernelGGL((k_embed<uint16_t, 16>), grid, block, 0, st, static_cast<const uint16_t*>(emb), tokens,
                       tok_slot_stride, tok_cap, vocab, pos, d, x, ssq_part, sn, hd, (double)theta, cs, frag, frag_gain);
  else
    hipLaunchKernelGGL((k_embed<float, 1024>), grid, block, 0, st, static_cast<const float*>(emb), tokens,
                       tok_slot_stride, tok_cap, vocab, pos, d, x, ssq_part, sn, hd, (double)theta, cs, nullptr, nullptr);
}

__global__ void k_rope_table(PosRef pos, int hd, double theta, float2* __restrict__ cs) {
  const int m = blockIdx.x, i = threadIdx.x;
  if (i >= hd / 2) return;
  const double p = (double)(*pos.base + pos.offset + m);
  const double inv_freq = pow(theta, -2.0 * (double)i / (double)hd);
  const double ang = p * inv_freq;
  cs[m * 64 + i] = make_float2((float)cos(ang), (float)sin(ang));
}

void launch_rope_table(PosRef pos, int M, int hd, float theta, float2* cs, hipStream_t st) {
  hipLaunchKernelGGL(k_rope_table, dim3(M), dim3(64), 0, st, pos, hd, (double)theta, cs);
}

// ---------------------------------------------------------------------------------------
// KV-cache attention: work-group = (128-key chunk, head, group of up to 16 query rows).
// The chunk's keys, then its values, are staged in LDS once and used by all the rows.
// Chunk boundaries are absolute key positions and chunks are combined in index order.
// ---------------------------------------------------------------------------------------
template <typename KV, int HD, int MR>
__global__ __launch_bounds__(128) void k_attn(const float* __restrict__ q, const KV* __restrict__ Kc,
                                              const KV* __restrict__ Vc, int cap, int d, int H, int M, PosRef pos,
                                              float scale, int nchunk_cap, float* __restrict__ part_o,
                                              float* __restrict__ part_ml) {
  constexpr int EPV = 16 / sizeof(KV);     // elements per 16-byte vector
  constexpr int ROW = HD + EPV;            // padded LDS row
  extern __shared__ uint4 smem_u4[];
  KV* s_kv = reinterpret_cast<KV*>(smem_u4);                                   // [128][ROW]
  float* s_q = reinterpret_cast<float*>(s_kv + 128 * ROW);                     // [MR][HD]
  float* s_p = s_q + MR * HD;                                                  // [MR][128]
  float* s_ml = s_p + MR * 128;                                                // [MR][2]

  const int c = blockIdx.x, h = blockIdx.y, row0 = blockIdx.z * 16;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int pos0 = *pos.base + pos.offset;
  const int kv_len = pos0 + M;
  const int key0 = c * kAttnChunk;
  if (key0 >= kv_len) return;
  const int nkeys = min(kAttnChunk, kv_len - key0);
  const int rows = min(MR, M - row0);      // valid query rows of this group

  for (int idx = tid; idx < MR * HD; idx += 128) {
    const int i = idx / HD, e = idx - i * HD;
    s_q[idx] = (i < rows) ? q[(size_t)(row0 + i) * d + h * HD + e] : 0.f;
  }
  {
    const uint4* src = reinterpret_cast<const uint4*>(Kc + ((size_t)h * cap + key0) * HD);
    constexpr int VPR = HD / EPV;
    for (int idx = tid; idx < nkeys * VPR; idx += 128) {
      const int r = idx / VPR, cc = idx - r * VPR;
      *reinterpret_cast<uint4*>(s_kv + r * ROW + cc * EPV) = src[idx];
    }
  }
  __syncthreads();

  float sacc[MR];
#pragma unroll
  for (int i = 0; i < MR; ++i) sacc[i] = 0.f;
  if (tid < nkeys) {
    const KV* krow = s_kv + tid * ROW;
    for (int e0 = 0; e0 < HD; e0 += EPV) {
      float kf[EPV];
#pragma unroll
      for (int j = 0; j < EPV; ++j) kf[j] = load_kv(krow + e0 + j);
#pragma unroll
      for (int i = 0; i < MR; ++i) {
        float a = sacc[i];
#pragma unroll
        for (int j = 0; j < EPV; ++j) a = fmaf(s_q[i * HD + e0 + j], kf[j], a);
        sacc[i] = a;
      }
    }
  }
#pragma unroll
  for (int i = 0; i < MR; ++i) {
    const bool ok = (tid < nkeys) && (i < rows) && (key0 + tid <= pos0 + row0 + i);
    s_p[i * 128 + tid] = ok ? sacc[i] * scale : -INFINITY;
  }
  __syncthreads();   // everybody is done with the keys; scores are in LDS

  {
    const uint4* src = reinterpret_cast<const uint4*>(Vc + ((size_t)h * cap + key0) * HD);
    constexpr int VPR = HD / EPV;
    for (int idx = tid; idx < nkeys * VPR; idx += 128) {
      const int r = idx / VPR, cc = idx - r * VPR;
      *reinterpret_cast<uint4*>(s_kv + r * ROW + cc * EPV) = src[idx];
    }
  }
  for (int i = wave; i < MR; i += 2) {
    const float a = s_p[i * 128 + lane], b = s_p[i * 128 + lane + 64];
    const float mx = wave_max(fmaxf(a, b));
    float pa = 0.f, pb = 0.f;
    if (mx != -INFINITY) {
      pa = expf(a - mx);
      pb = expf(b - mx);
    }
    const float l = wave_sum(pa + pb);
    s_p[i * 128 + lane] = pa;
    s_p[i * 128 + lane + 64] = pb;
    if (lane == 0) {
      s_ml[i * 2] = mx;
      s_ml[i * 2 + 1] = l;
    }
  }
  __syncthreads();

  if (tid < HD) {
    float o[MR];
#pragma unroll
    for (int i = 0; i < MR; ++i) o[i] = 0.f;
    for (int t = 0; t < nkeys; ++t) {
      const float v = load_kv(s_kv + t * ROW + tid);
#pragma unroll
      for (int i = 0; i < MR; ++i) o[i] = fmaf(s_p[i * 128 + t], v, o[i]);
    }
#pragma unroll
    for (int i = 0; i < MR; ++i)
      if (i < rows) part_o[(((size_t)(row0 + i) * H + h) * nchunk_cap + c) * HD + tid] = o[i];
  }
  if (tid < rows) {
    float* ml = part_ml + (((size_t)(row0 + tid) * H + h) * nchunk_cap + c) * 2;
    ml[0] = s_ml[tid * 2];
    ml[1] = s_ml[tid * 2 + 1];
  }
}

template <int HD>
__global__ void k_attn_combine(const float* __restrict__ part_o, const float* __restrict__ part_ml, int H, PosRef pos,
                               int nchunk_cap, float* __restrict__ out, int d) {
  const int h = blockIdx.x, m = blockIdx.y, e = threadIdx.x;
  const int p = *pos.base + pos.offset + m;
  float* dst = out + (size_t)m * d + h * HD + e;
  if (p < 0) {
    *dst = 0.f;
    return;
  }
  const int nch = p / kAttnChunk + 1;
  const size_t base = ((size_t)m * H + h) * nchunk_cap;
  float gmax = -INFINITY;
  for (int c = 0; c < nch; ++c) gmax = fmaxf(gmax, part_ml[(base + c) * 2]);
  float num = 0.f, den = 0.f;
  for (int c = 0; c < nch; ++c) {
    const float mc = part_ml[(base + c) * 2];
    if (mc == -INFINITY) continue;
    const float w = expf(mc - gmax);
    num = fmaf(w, part_o[(base + c) * HD + e], num);
    den = fmaf(w, part_ml[(base + c) * 2 + 1], den);
  }
  *dst = num / den;
}

// ---------------------------------------------------------------------------------------
// KV-cache attention for half-precision caches, MFMA 16x16x32 f16.
//   Cache layout (per layer, per head): keys in 16-position blocks stored as MFMA A tiles
//   [16 keys x 32 dims] (k_cache_off), values in 32-position blocks stored as A tiles of V^T
//   [16 dims x 32 key slots] whose slot order is the one the score tiles come out in (v_cache_off),
//   so neither K, V nor the probabilities ever pass through LDS for a transpose.
//   Work-group = (128-key chunk at an absolute position, head); wave w owns keys 32w..32w+31 of the
//   chunk: scores^T = K . q^T (q as half hi+lo), masked softmax over its 32 keys, out^T = V^T . p^T
//   (p as half hi+lo).  The four waves are merged in LDS in wave order, the chunks of a head by the
//   work-group that arrives last at the head's counter, in chunk order.
// ---------------------------------------------------------------------------------------
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;

__device__ __forceinline__ void split_half8(const float* v, f16x8& hi, f16x8& lo) {
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const _Float16 h = (_Float16)v[e];
    hi[e] = h;
    lo[e] = (_Float16)(v[e] - (float)h);
  }
}

// Merge of the chunk partials of one head (one slot): out[m] = sum_c w_c o_c / sum_c w_c l_c with w_c = exp(max_c - max).
// Step A: all (max, sum) pairs of all rows go to LDS in one round trip, then the row maxima and, in place of the chunk
// maxima, the weights w_c (one exp per row and chunk; formed per thread they made up most of the merge's time).
// Step B, up to kMergeCB chunks: one thread per (row, 4 adjacent dims) adds its chunks up in chunk order, all loads in
// flight together.
// More chunks: groups of kMergeCB chunks are summed by different threads in parallel (each as above, from zero) and the
// group sums added in group order; the grouping depends only on the row's own position.  Dynamic LDS:
// [M][nch_lds][2] pairs (weight, sum), [kMaxRows] unused, [rows_per_pass][HD/4][groups][5] group sums.
// e^x for the attention softmax of the half-cache kernels: the hardware's exp2 on x * log2(e) (two instructions, about
// 1 ulp; the library expf costs ten times that and a wave evaluates 16 per key block).  Arguments are <= 0 here.
__device__ __forceinline__ float exp_fast(float x) { return __builtin_amdgcn_exp2f(x * 1.44269504088896340736f); }

constexpr int kMergeCB = 20;
// Step A of the merge: the (weight, sum) table of all rows and chunks in LDS (see attn_merge)
__device__ __forceinline__ void attn_merge_table(const float* part_ml, int H, int h, int M, int pos0, int step, int nch_max,
                                                 int nchunk_cap, int nch_lds, float* s_ml) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  for (int idx = tid; idx < M * nch_max; idx += 256) {
    const int m = idx / nch_max, cc = idx - m * nch_max;
    const float2 ml = ld_dev2(&part_ml[(((size_t)m * H + h) * nchunk_cap + cc) * 2]);
    s_ml[((size_t)m * nch_lds + cc) * 2] = ml.x;
    s_ml[((size_t)m * nch_lds + cc) * 2 + 1] = ml.y;
  }
  __syncthreads();
  if (nch_max <= 16) {
    // few chunks: 16 lanes per row, four rows per wave at a time (max is exact in any order)
    const int cc = lane & 15;
    for (int m = wave * 4 + (lane >> 4); m < M; m += 16) {
      const int p = pos0 + m * step;
      const int nch = p >= 0 ? p / kAttnChunkH + 1 : 0;
      const float mc = cc < nch ? s_ml[((size_t)m * nch_lds + cc) * 2] : -INFINITY;
      float g = mc;
#pragma unroll
      for (int off = 8; off >= 1; off >>= 1) g = fmaxf(g, __shfl_xor(g, off));
      if (cc < nch) s_ml[((size_t)m * nch_lds + cc) * 2] = (mc == -INFINITY) ? 0.f : exp_fast(mc - g);
    }
    __syncthreads();
    return;
  }
  for (int m = wave; m < M; m += 4) {                 // row maxima (max is exact in any order)
    const int p = pos0 + m * step;
    const int nch = p >= 0 ? p / kAttnChunkH + 1 : 0;
    float g = -INFINITY;
    for (int cc = lane; cc < nch; cc += 64) g = fmaxf(g, s_ml[((size_t)m * nch_lds + cc) * 2]);
    g = wave_max(g);
    // the chunk weights, once per (row, chunk) instead of once per thread that uses them: each replaces its chunk's
    // maximum in the table (the lane that read the slot writes it)
    for (int cc = lane; cc < nch; cc += 64) {
      const float mc = s_ml[((size_t)m * nch_lds + cc) * 2];
      s_ml[((size_t)m * nch_lds + cc) * 2] = (mc == -INFINITY) ? 0.f : exp_fast(mc - g);
    }
  }
  __syncthreads();
}

// The merge for at most CB chunks: a thread takes IPT items (row, 4 adjacent dims) per pass and requests all their
// chunks' outputs before the table is built -- they do not depend on it, so the merge's two round trips to memory
// become one -- then adds them up in chunk order, from zero (the order of attn_merge's step B).
template <int HD, int CB, int IPT>
__device__ __forceinline__ void attn_merge_direct(const float* part_o, const float* part_ml, int H, int h, int M, int pos0,
                                                  int step, int nch_max, int nchunk_cap, int nch_lds, float* out, int d,
                                                  float* s_ml, uint4* frag, int frag_row0) {
  constexpr int QPR = HD / 4;                         // threads per row
  const int tid = threadIdx.x, items = M * QPR;
  float2 va[IPT][CB], vb[IPT][CB];
  // (a chunk past the row's last re-reads its last: no condition inside an item's requests)
#define STAIRS_MERGE_LOADS(base)                                                         \
  _Pragma("unroll") for (int ip = 0; ip < IPT; ++ip) {                                   \
    const int idx = (base) + ip * 256 + tid;                                             \
    if (idx < items) {                                                                   \
      const int m = idx / QPR, e = (idx - m * QPR) * 4;                                  \
      const int p = pos0 + m * step;                                                     \
      const int last = p >= 0 ? p / kAttnChunkH : 0;                                     \
      const float* src = part_o + ((size_t)m * H + h) * nchunk_cap * HD + e;             \
      _Pragma("unroll") for (int i = 0; i < CB; ++i) {                                   \
        const float* q = src + (size_t)min(i, last) * HD;                                \
        va[ip][i] = ld_dev2(q);                                                          \
        vb[ip][i] = ld_dev2(q + 2);                                                      \
      }                                                                                  \
    }                                                                                    \
  }
  STAIRS_MERGE_LOADS(0);
  attn_merge_table(part_ml, H, h, M, pos0, step, nch_max, nchunk_cap, nch_lds, s_ml);
  for (int base = 0; base < items; base += 256 * IPT) {
    if (base > 0) { STAIRS_MERGE_LOADS(base); }
#pragma unroll
    for (int ip = 0; ip < IPT; ++ip) {
      const int idx = base + ip * 256 + tid;
      if (idx < items) {
        const int m = idx / QPR, e = (idx - m * QPR) * 4;
        const int p = pos0 + m * step;
        float4 res = make_float4(0.f, 0.f, 0.f, 0.f);
        if (p >= 0) {
          const int nch = p / kAttnChunkH + 1;
          const float* mlr = s_ml + (size_t)m * nch_lds * 2;
          float4 num = make_float4(0.f, 0.f, 0.f, 0.f);
          float den = 0.f;
#pragma unroll
          for (int i = 0; i < CB; ++i) {
            if (i < nch) {
              const float w = mlr[i * 2];
              num.x = fmaf(w, va[ip][i].x, num.x); num.y = fmaf(w, va[ip][i].y, num.y);
              num.z = fmaf(w, vb[ip][i].x, num.z); num.w = fmaf(w, vb[ip][i].y, num.w);
              den = fmaf(w, mlr[i * 2 + 1], den);
            }
          }
          res = make_float4(num.x / den, num.y / den, num.z / den, num.w / den);
        }
        *reinterpret_cast<float4*>(out + (size_t)m * d + h * HD + e) = res;
        if (frag) store_frag4(frag, frag_row0 + m, h * HD + e, res, nullptr);
      }
    }
  }
#undef STAIRS_MERGE_LOADS
}

template <int HD>
__device__ __forceinline__ void attn_merge(const float* part_o, const float* part_ml, int H, int h, int M, int pos0, int step,
                                           int kv_len, int nchunk_cap, int nch_lds, int rows_per_pass, float* out, int d,
                                           float* s_ml, uint4* frag, int frag_row0) {
  const int tid = threadIdx.x;
  const int nch_max = (kv_len > 0) ? (kv_len - 1) / kAttnChunkH + 1 : 0;
  if (nch_max <= kMergeCB / 2)                        // (no chunk at all: every row gets zeros)
    return attn_merge_direct<HD, kMergeCB / 2, 2>(part_o, part_ml, H, h, M, pos0, step, nch_max, nchunk_cap, nch_lds, out, d,
                                                  s_ml, frag, frag_row0);
  if (nch_max <= kMergeCB)
    return attn_merge_direct<HD, kMergeCB, 1>(part_o, part_ml, H, h, M, pos0, step, nch_max, nchunk_cap, nch_lds, out, d,
                                              s_ml, frag, frag_row0);
  // more chunks: groups of kMergeCB chunks summed in parallel, the group sums added in group order
  float* grp = s_ml + (size_t)M * nch_lds * 2 + kMaxRows;   // (kMaxRows floats after the table stay unused)
  attn_merge_table(part_ml, H, h, M, pos0, step, nch_max, nchunk_cap, nch_lds, s_ml);
  constexpr int QPR = HD / 4;                         // threads per row
  constexpr int CB = kMergeCB;
  const int G = (nch_max + CB - 1) / CB;
  // sum of the chunks [c0, c1) of row m, dims e..e+3, weighted; all loads of the (at most CB) chunks together
  auto group_sum = [&](int m, int e, int c0, int c1, float4& num, float& den) {
    const float* mlr = s_ml + (size_t)m * nch_lds * 2;
    const float* src = part_o + ((size_t)m * H + h) * nchunk_cap * HD + e;
    float2 va[CB], vb[CB];
#pragma unroll
    for (int i = 0; i < CB; ++i) {
      const float* q = src + (size_t)min(c0 + i, c1 - 1) * HD;
      va[i] = ld_dev2(q);
      vb[i] = ld_dev2(q + 2);
    }
#pragma unroll
    for (int i = 0; i < CB; ++i) {
      if (c0 + i < c1) {
        const float w = mlr[(c0 + i) * 2];
        num.x = fmaf(w, va[i].x, num.x); num.y = fmaf(w, va[i].y, num.y);
        num.z = fmaf(w, vb[i].x, num.z); num.w = fmaf(w, vb[i].y, num.w);
        den = fmaf(w, mlr[(c0 + i) * 2 + 1], den);
      }
    }
  };
  for (int m0 = 0; m0 < M; m0 += rows_per_pass) {
    const int rows = min(rows_per_pass, M - m0);
    for (int idx = tid; idx < rows * QPR * G; idx += 256) {
      const int g = idx % G, rq = idx / G;
      const int ml = rq / QPR, e = (rq - ml * QPR) * 4, m = m0 + ml;
      const int p = pos0 + m * step;
      float4 num = make_float4(0.f, 0.f, 0.f, 0.f);
      float den = 0.f;
      if (p >= 0) {
        const int nch = p / kAttnChunkH + 1;
        if (g * CB < nch) group_sum(m, e, g * CB, min(nch, (g + 1) * CB), num, den);
      }
      float* o = grp + (size_t)idx * 5;
      o[0] = num.x; o[1] = num.y; o[2] = num.z; o[3] = num.w; o[4] = den;
    }
    __syncthreads();
    for (int idx = tid; idx < rows * QPR; idx += 256) {
      const int ml = idx / QPR, e = (idx - ml * QPR) * 4, m = m0 + ml;
      const int p = pos0 + m * step;
      float4 res = make_float4(0.f, 0.f, 0.f, 0.f);
      if (p >= 0) {
        const int ng = (p / kAttnChunkH + 1 + CB - 1) / CB;
        float4 num = make_float4(0.f, 0.f, 0.f, 0.f);
        float den = 0.f;
        for (int g = 0; g < ng; ++g) {
          const float* o = grp + ((size_t)idx * G + g) * 5;
          num.x += o[0]; num.y += o[1]; num.z += o[2]; num.w += o[3]; den += o[4];
        }
        res = make_float4(num.x / den, num.y / den, num.z / den, num.w / den);
      }
      *reinterpret_cast<float4*>(out + (size_t)m * d + h * HD + e) = res;
      if (frag) store_frag4(frag, frag_row0 + m, h * HD + e, res, nullptr);
    }
    __syncthreads();
  }
}

// (two work-groups per CU: the register budget that keeps both resident)
template <int HD, int CT, bool FUSED>
__global__ __launch_bounds__(256, 2) void k_attn_f16(const float* __restrict__ q, const _Float16* __restrict__ Kc,
                                                  const _Float16* __restrict__ Vc, int cap, int d, int H, int M,
                                                  PosRef pos, size_t kv_slot_stride, float scale, AttnMode am, int nchunk_cap,
                                                  int rows_per_pass, float* part_o, float* part_ml, int* counters,
                                                  float* __restrict__ out) {
  constexpr int KK = HD / 32;   // k-steps of the score MFMA
  constexpr int ET = HD / 16;   // output-dim tiles of the value MFMA
  __shared__ float s_o[4][16][HD + 4];               // (+4: the 16 rows a wave writes at once fall into different banks)
  __shared__ float s_m[4][16], s_l[4][16];
  __shared__ int s_last;
  const int c = blockIdx.x, h = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j = lane & 15, g = lane >> 4;
  // several sequences: blockIdx.z is the slot; its M = pos.rps rows, caches, partial results and counters follow
  // those of the slots before it, and everything below sees only this slot
  const int row0 = blockIdx.z * M;
  q += (size_t)row0 * d;
  out += (size_t)row0 * d;
  part_o += (size_t)row0 * H * nchunk_cap * HD;
  part_ml += (size_t)row0 * H * nchunk_cap * 2;
  counters += blockIdx.z * H;
  Kc += blockIdx.z * kv_slot_stride;
  Vc += blockIdx.z * kv_slot_stride;
  // causal: row i sees the keys 0 .. qpos0 + i; fixed key set (am.kv_fixed > 0): every row sees the keys 0 .. kv_fixed-1
  const int qpos0 = pos_of(pos, row0);
  const bool fixed = am.kv_fixed > 0;   // (then also for rows that sit nowhere: their result is unused)
  const int pos0 = fixed ? am.kv_fixed - 1 : qpos0;   // last key row 0 sees
  const int step = fixed ? 0 : 1;
  const int kv_len = pos0 + (fixed ? 1 : M);
  const float* brow = am.bias ? am.bias + (size_t)h * am.bias_ld + am.bias_zero : nullptr;
  // a wave owns 64 keys of the chunk as two blocks of 32 (the tiles of the cache layout)
  const int kb = c * kAttnChunkH + wave * 64;         // first key of this wave
  const bool have_keys = kb < kv_len;
  const bool have_second = kb + 32 < kv_len;
  // all keys in the first chunk: its work-group writes the result itself (what the merge would give for one chunk:
  // weight exp(0) = 1), the others have nothing to do; no partial results, no ticket
  const bool single = FUSED && kv_len <= kAttnChunkH;
  if (single && c > 0) return;

  // the first query tile's rows are requested before the keys and values: they come from L2 and are
  // converted while the cache tiles are still on their way
  float4 qa0[KK], qb0[KK];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) {
    qa0[kk] = make_float4(0.f, 0.f, 0.f, 0.f);
    qb0[kk] = qa0[kk];
    if (have_keys && j < M) {
      const float4* qp = reinterpret_cast<const float4*>(q + (size_t)j * d + h * HD + kk * 32 + g * 8);
      qa0[kk] = qp[0];
      qb0[kk] = qp[1];
    }
  }

  // the wave's whole share of the chunk is requested at once (keys and values of both blocks: 16 KiB at head_dim 128)
  uint4 kreg[2][2][KK], vreg[2][ET];
#pragma unroll
  for (int sb = 0; sb < 2; ++sb) {
    const bool ok = sb ? have_second : have_keys;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) kreg[sb][t][kk] = make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
    for (int et = 0; et < ET; ++et) vreg[sb][et] = make_uint4(0u, 0u, 0u, 0u);   // (a block without keys meets probability 0)
    if (ok) {
      const uint4* Kh = reinterpret_cast<const uint4*>(Kc + (size_t)h * cap * HD);
      const uint4* Vh = reinterpret_cast<const uint4*>(Vc + (size_t)h * cap * HD);
      const int kbs = kb + 32 * sb;
#pragma unroll
      // (the two-kernel form runs at long contexts only, where a layer's keys and values exceed what the memory-side
      // cache could keep until the next forward: streaming loads there, as for the weights of a large model)
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
          const uint4* p = &Kh[((size_t)((kbs >> 4) + t) * KK + kk) * 64 + lane];
          kreg[sb][t][kk] = FUSED ? *p : ld_nt(p);
        }
#pragma unroll
      for (int et = 0; et < ET; ++et) {
        const uint4* p = &Vh[((size_t)(kbs >> 5) * ET + et) * 64 + lane];
        vreg[sb][et] = FUSED ? *p : ld_nt(p);
      }
    }
  }

#pragma unroll
  for (int ct = 0; ct < CT; ++ct) {
    const int qi = ct * 16 + j;                      // this lane's query row
    f32x4 oacc[ET];
#pragma unroll
    for (int et = 0; et < ET; ++et) oacc[et] = f32x4{0.f, 0.f, 0.f, 0.f};
    float mw = -INFINITY, lw = 0.f;
    if (have_keys) {
      f16x8 qh[KK], ql[KK];
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) {
        const float4 a = qa0[kk], b = qb0[kk];
        const float v[8] = {a.x * scale, a.y * scale, a.z * scale, a.w * scale,
                            b.x * scale, b.y * scale, b.z * scale, b.w * scale};
        split_half8(v, qh[kk], ql[kk]);
      }
      // the next query tile's rows are requested now, into the registers just converted: they arrive while this
      // tile's scores and outputs are computed
      if (ct + 1 < CT) {
        const int qn = (ct + 1) * 16 + j;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
          qa0[kk] = make_float4(0.f, 0.f, 0.f, 0.f);
          qb0[kk] = qa0[kk];
          if (qn < M) {
            const float4* qp = reinterpret_cast<const float4*>(q + (size_t)qn * d + h * HD + kk * 32 + g * 8);
            qa0[kk] = qp[0];
            qb0[kk] = qp[1];
          }
        }
      }
      // scores of the wave's 64 keys, their joint maximum, the exponentials, then the two value products
      float sc[2][8];
#pragma unroll
      for (int sb = 0; sb < 2; ++sb) {
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          f32x4 sacc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int kk = 0; kk < KK; ++kk) {
            const f16x8 a = __builtin_bit_cast(f16x8, kreg[sb][t][kk]);
            sacc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, qh[kk], sacc, 0, 0, 0);
            sacc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, ql[kk], sacc, 0, 0, 0);
          }
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            const int key = kb + sb * 32 + t * 16 + g * 4 + v;
            const bool seen = qi < M && key <= pos0 + qi * step;
            const float bv = (brow && seen) ? brow[key - (qpos0 + qi)] : 0.f;   // bias by key position - query position
            sc[sb][t * 4 + v] = seen ? sacc[v] + bv : -INFINITY;
          }
        }
      }
      float mx = sc[0][0];
#pragma unroll
      for (int i = 1; i < 8; ++i) mx = fmaxf(mx, sc[0][i]);
#pragma unroll
      for (int i = 0; i < 8; ++i) mx = fmaxf(mx, sc[1][i]);
      mx = fmaxf(mx, __shfl_xor(mx, 16));
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      float sum = 0.f;
      f16x8 ph[2], pl[2];
#pragma unroll
      for (int sb = 0; sb < 2; ++sb) {
        float pv[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          pv[i] = (mx == -INFINITY) ? 0.f : exp_fast(sc[sb][i] - mx);
          sum += pv[i];
        }
        split_half8(pv, ph[sb], pl[sb]);
      }
      sum += __shfl_xor(sum, 16);
      sum += __shfl_xor(sum, 32);
      mw = mx;
      lw = sum;
#pragma unroll
      for (int sb = 0; sb < 2; ++sb)
#pragma unroll
        for (int et = 0; et < ET; ++et) {
          const f16x8 a = __builtin_bit_cast(f16x8, vreg[sb][et]);
          oacc[et] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, ph[sb], oacc[et], 0, 0, 0);
          oacc[et] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, pl[sb], oacc[et], 0, 0, 0);
        }
    }
    // merge the four waves (wave order): every wave leaves its maximum, its sum and its output rows as they are; the
    // threads that add the four outputs up scale them by exp(max_w - max) on the way (product rounded, then added)
    if (ct > 0) __syncthreads();                     // LDS of the previous query tile has been read
    if (g == 0) {
      s_m[wave][j] = mw;
      s_l[wave][j] = lw;
    }
    if (qi < M) {                                    // rows past the last one are never read back
#pragma unroll
      for (int et = 0; et < ET; ++et)
        *reinterpret_cast<float4*>(&s_o[wave][j][et * 16 + g * 4]) =
            make_float4(oacc[et][0], oacc[et][1], oacc[et][2], oacc[et][3]);
    }
    __syncthreads();
    const int rows_here = min(16, M - ct * 16);      // (<= 0 for a second tile no row falls into)
    // (a thread takes 4 adjacent dims of a row: 16 rows are two passes of the 256 threads)
    for (int idx = tid; idx < rows_here * (HD / 4); idx += 256) {
      const int jj = idx / (HD / 4), e = (idx - jj * (HD / 4)) * 4;
      const int m = ct * 16 + jj;
      if (m < M) {
        const float m0 = s_m[0][jj], m1 = s_m[1][jj], m2 = s_m[2][jj], m3 = s_m[3][jj];
        const float mcc = fmaxf(fmaxf(m0, m1), fmaxf(m2, m3));
        const float f0 = (m0 == -INFINITY) ? 0.f : exp_fast(m0 - mcc), f1 = (m1 == -INFINITY) ? 0.f : exp_fast(m1 - mcc);
        const float f2 = (m2 == -INFINITY) ? 0.f : exp_fast(m2 - mcc), f3 = (m3 == -INFINITY) ? 0.f : exp_fast(m3 - mcc);
        const float4 a0 = *reinterpret_cast<const float4*>(&s_o[0][jj][e]), a1 = *reinterpret_cast<const float4*>(&s_o[1][jj][e]);
        const float4 a2 = *reinterpret_cast<const float4*>(&s_o[2][jj][e]), a3 = *reinterpret_cast<const float4*>(&s_o[3][jj][e]);
        const float o0 = __fadd_rn(__fadd_rn(__fadd_rn(__fmul_rn(a0.x, f0), __fmul_rn(a1.x, f1)), __fmul_rn(a2.x, f2)), __fmul_rn(a3.x, f3));
        const float o1 = __fadd_rn(__fadd_rn(__fadd_rn(__fmul_rn(a0.y, f0), __fmul_rn(a1.y, f1)), __fmul_rn(a2.y, f2)), __fmul_rn(a3.y, f3));
        const float o2 = __fadd_rn(__fadd_rn(__fadd_rn(__fmul_rn(a0.z, f0), __fmul_rn(a1.z, f1)), __fmul_rn(a2.z, f2)), __fmul_rn(a3.z, f3));
        const float o3 = __fadd_rn(__fadd_rn(__fadd_rn(__fmul_rn(a0.w, f0), __fmul_rn(a1.w, f1)), __fmul_rn(a2.w, f2)), __fmul_rn(a3.w, f3));
        // the chunk's sum of exponentials (a wave without keys has weight 0 and sum 0: it adds nothing); no branch
        // around the LDS reads
        const float l0 = s_l[0][jj], l1 = s_l[1][jj], l2 = s_l[2][jj], l3 = s_l[3][jj];
        float lc = 0.f;
        lc += f0 * l0;
        lc += f1 * l1;
        lc += f2 * l2;
        lc += f3 * l3;
        if (single) {
          float4 res = make_float4(0.f, 0.f, 0.f, 0.f);
          if (pos0 + m * step >= 0) res = make_float4(o0 / lc, o1 / lc, o2 / lc, o3 / lc);
          *reinterpret_cast<float4*>(out + (size_t)m * d + h * HD + e) = res;
          if (am.frag_out) store_frag4(am.frag_out, row0 + m, h * HD + e, res, nullptr);
        } else {
          float* po = &part_o[(((size_t)m * H + h) * nchunk_cap + c) * HD + e];
          st_dev2(po, o0, o1);
          st_dev2(po + 2, o2, o3);
          // the thread with the row's first dims also leaves the chunk's (max, sum) pair
          if (e == 0) st_dev2(part_ml + (((size_t)m * H + h) * nchunk_cap + c) * 2, mcc, lc);
        }
      }
    }
  }

  // FUSED: the work-group that arrives last at the head's counter merges the chunks; otherwise a second kernel does
  if (!FUSED || single) return;
  if (!last_arrival(&counters[h], (int)gridDim.x, &s_last)) return;
  extern __shared__ float s_ml[];
  attn_merge<HD>(part_o, part_ml, H, h, M, pos0, step, kv_len, nchunk_cap, (int)gridDim.x, rows_per_pass, out, d, s_ml,
                 am.frag_out, row0);
  if (tid == 0) counters[h] = 0;
}

// the merge alone (long contexts: the attention work-groups then leave without waiting for their stores)
template <int HD>
__global__ __launch_bounds__(256) void k_attn_merge(const float* part_o, const float* part_ml, int d, int H, int M, PosRef pos,
                                                    int kv_fixed, int nchunk_cap, int nch_lds, int rows_per_pass,
                                                    float* __restrict__ out, uint4* frag) {
  extern __shared__ float s_ml[];
  const int h = blockIdx.x, row0 = blockIdx.y * M;
  const bool fixed = kv_fixed > 0;
  const int pos0 = fixed ? kv_fixed - 1 : pos_of(pos, row0);
  attn_merge<HD>(part_o + (size_t)row0 * H * nchunk_cap * HD, part_ml + (size_t)row0 * H * nchunk_cap * 2, H, h, M, pos0,
                 fixed ? 0 : 1, pos0 + (fixed ? 1 : M), nchunk_cap, nch_lds, rows_per_pass, out + (size_t)row0 * d, d, s_ml,
                 frag, row0);
}

// Attention of a prefill block (R consecutive rows at positions p0 .. p0+R-1 of one sequence) without partial
// results: a wave owns 16 query rows (a work-group 64) of one head and
// walks over the keys 0 .. its last row's position, 32 at a time, keeping the running maximum, the running sum and the
// running output of its rows in registers (rescaled whenever the maximum grows).  Same operands and splits as
// k_attn_f16 (scores^T = K q^T with q as half high + low, out^T = V^T p^T with p as half high + low); the order of
// the additions differs from the decode kernels, which only ever see their own results.
template <int HD>
__global__ __launch_bounds__(256, 2) void k_attn_flash(const float* __restrict__ q, const _Float16* __restrict__ Kc,
                                                    const _Float16* __restrict__ Vc, int cap, int d, int H, int R, int p0,
                                                    float scale, float* __restrict__ out) {
  constexpr int KK = HD / 32, ET = HD / 16;
  const int h = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int j = lane & 15, g = lane >> 4;
  const int r0 = blockIdx.y * 64 + wave * 16;         // first row of this wave's tile
  if (r0 >= R) return;                                // no barriers in this kernel: waves are independent
  const int row = r0 + j;
  const bool row_ok = row < R;
  const int p_row = p0 + row;
  const int tile_last = p0 + min(r0 + 15, R - 1);     // last position of the tile = last key any of its rows sees
  f16x8 qh[KK], ql[KK];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) {
    float4 a = make_float4(0.f, 0.f, 0.f, 0.f), b = a;
    if (row_ok) {
      const float4* qp = reinterpret_cast<const float4*>(q + (size_t)row * d + h * HD + kk * 32 + g * 8);
      a = qp[0];
      b = qp[1];
    }
    const float v[8] = {a.x * scale, a.y * scale, a.z * scale, a.w * scale, b.x * scale, b.y * scale, b.z * scale, b.w * scale};
    split_half8(v, qh[kk], ql[kk]);
  }
  const uint4* Kh = reinterpret_cast<const uint4*>(Kc + (size_t)h * cap * HD) + lane;
  const uint4* Vh = reinterpret_cast<const uint4*>(Vc + (size_t)h * cap * HD) + lane;
  f32x4 oacc[ET];
#pragma unroll
  for (int et = 0; et < ET; ++et) oacc[et] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY, l_run = 0.f;
  // two register sets: the keys and values of the next step are requested before this step's arithmetic
  uint4 kA[2][KK], vA[ET], kB[2][KK], vB[ET];
  auto load_kv = [&](int kb, uint4 (&kreg)[2][KK], uint4 (&vreg)[ET]) {
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) kreg[t][kk] = Kh[((size_t)((kb >> 4) + t) * KK + kk) * 64];
#pragma unroll
    for (int et = 0; et < ET; ++et) vreg[et] = Vh[((size_t)(kb >> 5) * ET + et) * 64];
  };
  auto step = [&](int kb, const uint4 (&kreg)[2][KK], const uint4 (&vreg)[ET]) {
    float sc[8];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      f32x4 sacc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) {
        const f16x8 a = __builtin_bit_cast(f16x8, kreg[t][kk]);
        sacc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, qh[kk], sacc, 0, 0, 0);
        sacc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, ql[kk], sacc, 0, 0, 0);
      }
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int key = kb + t * 16 + g * 4 + v;
        sc[t * 4 + v] = (row_ok && key <= p_row) ? sacc[v] : -INFINITY;
      }
    }
    float mx = sc[0];
#pragma unroll
    for (int i = 1; i < 8; ++i) mx = fmaxf(mx, sc[i]);
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m_run, mx);
    const float alpha = (m_run == -INFINITY) ? 0.f : exp_fast(m_run - m_new);   // m_new >= m_run > -inf there
    float pv[8], sum = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      pv[i] = (m_new == -INFINITY) ? 0.f : exp_fast(sc[i] - m_new);
      sum += pv[i];
    }
    sum += __shfl_xor(sum, 16);
    sum += __shfl_xor(sum, 32);
    l_run = l_run * alpha + sum;
    m_run = m_new;
    f16x8 ph, pl;
    split_half8(pv, ph, pl);
#pragma unroll
    for (int et = 0; et < ET; ++et) {
      oacc[et][0] *= alpha; oacc[et][1] *= alpha; oacc[et][2] *= alpha; oacc[et][3] *= alpha;
      const f16x8 a = __builtin_bit_cast(f16x8, vreg[et]);
      oacc[et] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, ph, oacc[et], 0, 0, 0);
      oacc[et] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, pl, oacc[et], 0, 0, 0);
    }
  };
  load_kv(0, kA, vA);
#pragma nounroll
  for (int kb = 0; kb <= tile_last; kb += 64) {
    if (kb + 32 <= tile_last) load_kv(kb + 32, kB, vB);
    step(kb, kA, vA);
    if (kb + 32 > tile_last) break;
    if (kb + 64 <= tile_last) load_kv(kb + 64, kA, vA);
    step(kb + 32, kB, vB);
  }
  if (row_ok) {
    const float inv = 1.0f / l_run;
#pragma unroll
    for (int et = 0; et < ET; ++et)
      *reinterpret_cast<float4*>(out + (size_t)row * d + h * HD + et * 16 + g * 4) =
          make_float4(oacc[et][0] * inv, oacc[et][1] * inv, oacc[et][2] * inv, oacc[et][3] * inv);
  }
}

void launch_attention_flash(const float* q, const void* Kc, const void* Vc, int cap, int d, int H, int R, int p0, float* out,
                            hipStream_t st) {
  const int hd = d / H;
  const float scale = 1.0f / sqrtf((float)hd);
  const _Float16* K = static_cast<const _Float16*>(Kc);
  const _Float16* V = static_cast<const _Float16*>(Vc);
  dim3 grid(H, (R + 63) / 64);
  if (hd == 128)
    hipLaunchKernelGGL((k_attn_flash<128>), grid, dim3(256), 0, st, q, K, V, cap, d, H, R, p0, scale, out);
  else
    hipLaunchKernelGGL((k_attn_flash<64>), grid, dim3(256), 0, st, q, K, V, cap, d, H, R, p0, scale, out);
}

template <typename KV, int HD>
static void attn_dispatch(const float* q, const void* Kc, const void* Vc, int cap, int d, int H, int M, PosRef pos,
                          int nchunk_launch, int nchunk_cap, float* part_o, float* part_ml, hipStream_t st) {
  const float scale = 1.0f / sqrtf((float)HD);
  const KV* K = static_cast<const KV*>(Kc);
  const KV* V = static_cast<const KV*>(Vc);
  dim3 grid(nchunk_launch, H, (M + 15) / 16), block(128);
  constexpr int EPV = 16 / sizeof(KV);
#define STAIRS_ATTN(mr)                                                                                   \
  {                                                                                                       \
    const size_t lds = (size_t)128 * (HD + EPV) * sizeof(KV) + (size_t)(mr) * (HD + 128 + 2) * sizeof(float); \
    hipLaunchKernelGGL((k_attn<KV, HD, mr>), grid, block, lds, st, q, K, V, cap, d, H, M, pos, scale,       \
                       nchunk_cap, part_o, part_ml);                                                      \
  }
  if (M <= 2) STAIRS_ATTN(2)
  else if (M <= 8) STAIRS_ATTN(8)
  else STAIRS_ATTN(16)
#undef STAIRS_ATTN
}

void launch_attention(const float* q_rot, const void* Kc, const void* Vc, int kv_half, int cap, int d, int H, int M,
                      PosRef pos, int nslots, size_t kv_slot_stride, int nchunk_launch, int nchunk_cap, float* part_o,
                      float* part_ml, int* counters, float* out, hipStream_t st, const AttnMode& am) {
  const int hd = d / H;
  if (kv_half) {
    const float scale = am.scale > 0.f ? am.scale : 1.0f / sqrtf((float)hd);
    const _Float16* K = static_cast<const _Float16*>(Kc);
    const _Float16* V = static_cast<const _Float16*>(Vc);
    // the half-cache kernels take 256-key chunks: half as many work-groups as the 128-key units the callers count in
    nchunk_launch = (nchunk_launch * kAttnChunk + kAttnChunkH - 1) / kAttnChunkH;
    dim3 grid(nchunk_launch, H, nslots), block(256);
    // merge step's LDS: (max, sum) table, row maxima, and for more than kMergeCB chunks the group sums of as many
    // rows per pass as fit in 48 KiB, less when the table is large (the whole stays under kAttnMergeMaxLds)
    const int G = (nchunk_launch + kMergeCB - 1) / kMergeCB;
    const size_t table = ((size_t)M * nchunk_launch * 2 + kMaxRows) * sizeof(float);
    const size_t per_row = (size_t)(hd / 4) * G * 5 * sizeof(float);
    const size_t budget = std::min<size_t>(48 * 1024, kAttnMergeMaxLds > table ? kAttnMergeMaxLds - table : 0);
    const int rpp = G > 1 ? std::max(1, std::min(M, (int)(budget / per_row))) : M;
    const size_t lds = table + (G > 1 ? (size_t)rpp * per_row : 0);
    // long contexts: attention work-groups only store their partials, a second kernel merges (no wait, no ticket)
    const bool fused = nchunk_launch <= kAttnFusedMaxChunks;
#define STAIRS_ATTN16(hdv, ct)                                                                                              \
  if (fused)                                                                                                                \
    hipLaunchKernelGGL((k_attn_f16<hdv, ct, true>), grid, block, lds, st, q_rot, K, V, cap, d, H, M, pos, kv_slot_stride,   \
                       scale, am, nchunk_cap, rpp, part_o, part_ml, counters, out);                                         \
  else {                                                                                                                    \
    hipLaunchKernelGGL((k_attn_f16<hdv, ct, false>), grid, block, 0, st, q_rot, K, V, cap, d, H, M, pos, kv_slot_stride,    \
                       scale, am, nchunk_cap, rpp, part_o, part_ml, counters, out);                                         \
    hipLaunchKernelGGL((k_attn_merge<hdv>), dim3(H, nslots), dim3(256), lds, st, part_o, part_ml, d, H, M, pos,             \
                       am.kv_fixed, nchunk_cap, nchunk_launch, rpp, out, am.frag_out);                                      \
  }
    if (hd == 128) {
      if (M <= 16) STAIRS_ATTN16(128, 1) else STAIRS_ATTN16(128, 2)
    } else {
      if (M <= 16) STAIRS_ATTN16(64, 1) else STAIRS_ATTN16(64, 2)
    }
#undef STAIRS_ATTN16
    return;
  }
  if (hd == 128) attn_dispatch<float, 128>(q_rot, Kc, Vc, cap, d, H, M, pos, nchunk_launch, nchunk_cap, part_o, part_ml, st);
  else attn_dispatch<float, 64>(q_rot, Kc, Vc, cap, d, H, M, pos, nchunk_launch, nchunk_cap, part_o, part_ml, st);
  if (hd == 128)
    hipLaunchKernelGGL(k_attn_combine<128>, dim3(H, M), dim3(128), 0, st, part_o, part_ml, H, pos, nchunk_cap, out, d);
  else
    hipLaunchKernelGGL(k_attn_combine<64>, dim3(H, M), dim3(64), 0, st, part_o, part_ml, H, pos, nchunk_cap, out, d);
}

// ---------------------------------------------------------------------------------------
// per-row vocabulary argmax (ties -> lowest index) and stairs validation
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void k_argmax(const float* __restrict__ logits, int ld, int V, int row0, int row_stride,
                                                 int* __restrict__ out, PosRef out_pos, int out_slot_stride) {
  __shared__ float sv[16];
  __shared__ int si[16];
  const int r = blockIdx.x, tid = threadIdx.x;
  const float* row = logits + (size_t)(row0 + r * row_stride) * ld;
  float best = -INFINITY;
  int bi = 0x7fffffff;
  // a thread walks its candidates in ascending index order, 8 loads in flight at a time
  for (int v0 = tid * 4; v0 < V; v0 += 8 * 4096) {
    float4 x[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int v = v0 + 4096 * i;
      x[i] = (v < V) ? *reinterpret_cast<const float4*>(row + v) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int v = v0 + 4096 * i;
      if (v < V) {
        if (x[i].x > best || bi == 0x7fffffff) { best = x[i].x; bi = v; }
        if (x[i].y > best) { best = x[i].y; bi = v + 1; }
        if (x[i].z > best) { best = x[i].z; bi = v + 2; }
        if (x[i].w > best) { best = x[i].w; bi = v + 3; }
      }
    }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const float ov = __shfl_xor(best, off);
    const int oi = __shfl_xor(bi, off);
    if (ov > best || (ov == best && oi < bi)) { best = ov; bi = oi; }
  }
  if ((tid & 63) == 0) { sv[tid >> 6] = best; si[tid >> 6] = bi; }
  __syncthreads();
  if (tid == 0) {
    for (int w = 1; w < 16; ++w)
      if (sv[w] > best || (sv[w] == best && si[w] < bi)) { best = sv[w]; bi = si[w]; }
    if (out_pos.rps) {                     // several sequences: the slot's own token array, only while it is active
      const int o = pos_of(out_pos, r);
      if (o >= 0) out[(size_t)slot_of(out_pos, r) * out_slot_stride + o] = bi;
    } else {
      out[(out_pos.base ? *out_pos.base : 0) + out_pos.offset + r] = bi;
    }
  }
}

void launch_argmax(const float* logits, int ld, int V, int nrows, int row0, int row_stride, int* out, PosRef out_pos,
                   int out_slot_stride, hipStream_t st) {
  hipLaunchKernelGGL(k_argmax, dim3(nrows), dim3(1024), 0, st, logits, ld, V, row0, row_stride, out, out_pos, out_slot_stride);
}

__global__ void k_accept(int* __restrict__ tokens, const int* __restrict__ tgt, int k, int* __restrict__ state,
                         int tok_slot_stride) {
  if (threadIdx.x != 0) return;
  const int s = blockIdx.x;                 // slot
  state += s * kSlotState;
  if (!state[3]) return;                    // the slot is not generating (any more)
  tokens += (size_t)s * tok_slot_stride;
  tgt += s * (k + 1);
  const int L = state[0];
  int n = 0;
  while (n < k && tokens[L + n] == tgt[n]) ++n;
  tokens[L + n] = tgt[n];
  state[0] = L + n + 1;
  state[1] = n;
}

void launch_accept(int* tokens, const int* tgt, int k, int* state, int nslots, int tok_slot_stride, hipStream_t st) {
  hipLaunchKernelGGL(k_accept, dim3(nslots), dim3(64), 0, st, tokens, tgt, k, state, tok_slot_stride);
}

// ---------------------------------------------------------------------------------------
// sampling variant: counter-based random numbers, Gumbel-max draws, keep / replace walk
// ---------------------------------------------------------------------------------------
// "squares" counter-based generator (Widynski 2020): four rounds of squaring, 32-bit output
__device__ __forceinline__ uint32_t squares32(uint64_t ctr, uint64_t key) {
  uint64_t x = ctr * key;
  const uint64_t y = x, z = y + key;
  x = x * x + y; x = (x >> 32) | (x << 32);
  x = x * x + z; x = (x >> 32) | (x << 32);
  x = x * x + y; x = (x >> 32) | (x << 32);
  return (uint32_t)((x * x + z) >> 32);
}
// the draw of (position of the token being decided, stream, vocabulary index) as a uniform in (0, 1)
__device__ __forceinline__ double sample_uniform(int pos, int stream, int v, uint64_t key) {
  const uint64_t ctr = ((uint64_t)pos << 34) | ((uint64_t)stream << 32) | (uint32_t)v;
  return ((double)squares32(ctr, key) + 0.5) * (1.0 / 4294967296.0);
}
__device__ __forceinline__ double sample_gumbel(int pos, int stream, int v, uint64_t key) {
  return -log(-log(sample_uniform(pos, stream, v, key)));
}

// (max, index) over a 256-thread block, ties -> lowest index; result valid in thread 0
__device__ __forceinline__ void block_argmax_256(double& best, int& bi, double* sv, int* si) {
  const int tid = threadIdx.x;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const double ov = __shfl_xor(best, off);
    const int oi = __shfl_xor(bi, off);
    if (ov > best || (ov == best && oi < bi)) { best = ov; bi = oi; }
  }
  if ((tid & 63) == 0) { sv[tid >> 6] = best; si[tid >> 6] = bi; }
  __syncthreads();
  if (tid == 0)
    for (int w = 1; w < 4; ++w)
      if (sv[w] > best || (sv[w] == best && si[w] < bi)) { best = sv[w]; bi = si[w]; }
  __syncthreads();
}

// A draw over the whole vocabulary spread over the blocks of a launch: every block reduces its candidates to one
// (score, index), stores it, and the block that arrives last at the ticket reduces those.  Returns true (in every
// thread of that last block) with the winner in best / bi of thread 0; the ticket is zero again afterwards.
__device__ __forceinline__ bool grid_argmax(double& best, int& bi, SampleWs* ws, double* sv, int* si, int* s_flag) {
  block_argmax_256(best, bi, sv, si);
  if (threadIdx.x == 0) {
    __hip_atomic_store(&ws->score[blockIdx.x], (unsigned long long)__double_as_longlong(best), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(&ws->idx[blockIdx.x], bi, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  if (!last_arrival(&ws->ticket, (int)gridDim.x, s_flag)) return false;
  best = -INFINITY;
  bi = 0x7fffffff;
  for (int i = threadIdx.x; i < (int)gridDim.x; i += 256) {
    const double ov = __longlong_as_double((long long)__hip_atomic_load(&ws->score[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    const int oi = __hip_atomic_load(&ws->idx[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (ov > best || (ov == best && oi < bi)) { best = ov; bi = oi; }
  }
  block_argmax_256(best, bi, sv, si);
  if (threadIdx.x == 0) __hip_atomic_store(&ws->ticket, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return true;
}

// lse[r] = log sum_v exp(rows[r][v] * inv_temp): one 1024-thread block per row; rows 0..n_a-1 from a, the rest from b
__global__ __launch_bounds__(1024) void k_row_lse(const float* __restrict__ a, int n_a, const float* __restrict__ b, int ld,
                                                  int V, const SampleParams* __restrict__ sp, float* __restrict__ lse) {
  __shared__ float red[16];
  const int r = blockIdx.x, tid = threadIdx.x;
  const float* row = r < n_a ? a + (size_t)r * ld : b + (size_t)(r - n_a) * ld;
  const float it = sp->inv_temp;
  float mx = -INFINITY;
  for (int v = tid; v < V; v += 1024) mx = fmaxf(mx, row[v] * it);
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
  if ((tid & 63) == 0) red[tid >> 6] = mx;
  __syncthreads();
  mx = red[0];
  for (int w = 1; w < 16; ++w) mx = fmaxf(mx, red[w]);
  __syncthreads();
  float sum = 0.f;
  for (int v = tid; v < V; v += 1024) sum += expf(row[v] * it - mx);
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off);
  if ((tid & 63) == 0) red[tid >> 6] = sum;
  __syncthreads();
  if (tid == 0) {
    float t = 0.f;
    for (int w = 0; w < 16; ++w) t += red[w];
    lse[r] = mx + logf(t);
  }
}

// tokens[o] = argmax_v(logits[v] / T + gumbel(o, stream, v)) with o = the position out_pos gives: one categorical
// draw, one candidate per thread (grid-stride for very large vocabularies)
__global__ __launch_bounds__(256) void k_sample(const float* __restrict__ logits, int V, const SampleParams* __restrict__ sp,
                                                int stream, int* __restrict__ tokens, PosRef out_pos, SampleWs* ws) {
  __shared__ double sv[4];
  __shared__ int si[4];
  __shared__ int s_flag;
  const int o = *out_pos.base + out_pos.offset;
  const float it = sp->inv_temp;
  const uint64_t key = sp->key;
  double best = -INFINITY;
  int bi = 0x7fffffff;
  for (int v = blockIdx.x * 256 + threadIdx.x; v < V; v += gridDim.x * 256) {
    const double sc = (double)(logits[v] * it) + sample_gumbel(o, stream, v, key);
    if (sc > best || bi == 0x7fffffff) { best = sc; bi = v; }
  }
  if (!grid_argmax(best, bi, ws, sv, si, &s_flag)) return;
  if (threadIdx.x == 0) tokens[o] = bi;
}

// Validation of a sampled stair batch (one sequence).  tokens[L .. L+k) hold the assistant's draws d_1..d_k, dl[j-1]
// the logits d_j was drawn from, tl[i] the main model's logits of stair row i, lse[0..k] / lse[k+1..2k] their
// log-sum-exps at the temperature.  d_i is kept while u_i * q_i(d_i) < p_{i-1}(d_i); at the first one that is not,
// tokens[L+n] is drawn from the positive part of p_n - q_{n+1}; with all kept, tokens[L+k] from p_k.
// state = {L + n + 1, n}; emitted[0..n] = the n + 1 tokens of this iteration.  Every block repeats the (cheap) walk
// and scores its share of the vocabulary; the block that arrives last picks the winner and writes the results.
__global__ __launch_bounds__(256) void k_accept_sampled(int* __restrict__ tokens, const float* __restrict__ tl,
                                                        const float* __restrict__ dl, int ld, int V, int k,
                                                        const float* __restrict__ lse, const SampleParams* __restrict__ sp,
                                                        int* __restrict__ state, int* __restrict__ emitted, SampleWs* ws) {
  __shared__ double sv[4];
  __shared__ int si[4];
  __shared__ int s_n, s_flag, s_empty;
  const int tid = threadIdx.x;
  const int L = state[0];
  const float it = sp->inv_temp;
  const uint64_t key = sp->key;
  if (tid == 0) {
    int n = 0;
    while (n < k) {
      const int d = tokens[L + n];
      const float logp = tl[(size_t)n * ld + d] * it - lse[n];
      const float logq = dl[(size_t)n * ld + d] * it - lse[k + 1 + n];
      const double u = sample_uniform(L + n, 1, 0, key);
      if (!(u < (double)expf(logp - logq))) break;
      ++n;
    }
    s_n = n;
  }
  __syncthreads();
  const int n = s_n;
  const int pos = L + n;
  const float* trow = tl + (size_t)n * ld;
  const float* drow = dl + (size_t)n * ld;     // only read when n < k
  const float lt = lse[n], lq = n < k ? lse[k + 1 + n] : 0.f;
  double best = -INFINITY;
  int bi = 0x7fffffff;
  for (int v = blockIdx.x * 256 + tid; v < V; v += gridDim.x * 256) {
    double sc;
    if (n < k) {                               // the positive part of p - q (a token was not kept)
      const float diff = expf(trow[v] * it - lt) - expf(drow[v] * it - lq);
      sc = diff > 0.f ? (double)logf(diff) + sample_gumbel(pos, 2, v, key) : -INFINITY;
    } else {                                   // all kept: p itself
      sc = (double)(trow[v] * it) + sample_gumbel(pos, 2, v, key);
    }
    if (sc > best || bi == 0x7fffffff) { best = sc; bi = v; }
  }
  if (!grid_argmax(best, bi, ws, sv, si, &s_flag)) return;
  if (tid == 0) s_empty = best == -INFINITY;
  __syncthreads();
  if (s_empty) {
    // possible only in rounding (p and q agree to the last bit and a token was still not kept): draw from p, by
    // this block alone
    best = -INFINITY;
    bi = 0x7fffffff;
    for (int v = tid; v < V; v += 256) {
      const double sc = (double)(trow[v] * it) + sample_gumbel(pos, 2, v, key);
      if (sc > best || bi == 0x7fffffff) { best = sc; bi = v; }
    }
    block_argmax_256(best, bi, sv, si);
  }
  if (tid == 0) {
    for (int i = 0; i < n; ++i) emitted[i] = tokens[L + i];
    emitted[n] = bi;
    tokens[pos] = bi;
    state[0] = L + n + 1;
    state[1] = n;
  }
}

void launch_row_lse(const float* a, int n_a, const float* b, int n_b, int ld, int V, const SampleParams* sp, float* lse,
                    hipStream_t st) {
  hipLaunchKernelGGL(k_row_lse, dim3(n_a + n_b), dim3(1024), 0, st, a, n_a, b, ld, V, sp, lse);
}
static int sample_blocks(int V) { return std::min(kSampleBlocksMax, (V + 255) / 256); }
void launch_sample(const float* logits, int V, const SampleParams* sp, int stream, int* tokens, PosRef out_pos,
                   SampleWs* ws, hipStream_t st) {
  hipLaunchKernelGGL(k_sample, dim3(sample_blocks(V)), dim3(256), 0, st, logits, V, sp, stream, tokens, out_pos, ws);
}
void launch_accept_sampled(int* tokens, const float* tl, const float* dl, int ld, int V, int k, const float* lse,
                           const SampleParams* sp, int* state, int* emitted, SampleWs* ws, hipStream_t st) {
  hipLaunchKernelGGL(k_accept_sampled, dim3(sample_blocks(V)), dim3(256), 0, st, tokens, tl, dl, ld, V, k, lse, sp, state,
                     emitted, ws);
}

// ---------------------------------------------------------------------------------------
// prompt ingestion in large row blocks: an MFMA-bound GEMM and the element-wise work around it
// ---------------------------------------------------------------------------------------
// Activations of a row block as MFMA B-operand fragments, written once by their producer: [k-step of 32][column tile
// of 16 rows][high, low][lane] x 16 bytes (lane r + 16 g: x[16 ct + r][32 kt + 8 g .. + 8] as bf16 high part / bf16 of
// the remainders).  RT = column tiles the buffer is laid out for (rows rounded up to a multiple of kBlkRows).
__device__ __forceinline__ void pf_store_frag4(uint4* frag, int RT, int r, int k, const float (&v)[4]) {
  uint2 hi, lo;
  bf16_split2(v[0], v[1], hi.x, lo.x);
  bf16_split2(v[2], v[3], hi.y, lo.y);
  const size_t u4 = (((size_t)(k >> 5) * RT + (r >> 4)) * 2) * 64 + (r & 15) + 16 * ((k & 31) >> 3);
  uint2* dst = reinterpret_cast<uint2*>(frag) + u4 * 2 + ((k & 7) >> 2);
  dst[0] = hi;
  dst[128] = lo;
}

// Y[R, N] (+)= X[R, K] . W[N, K]^T for row blocks of up to thousands of rows: the MFMA-bound regime.
//   W: the operand-tile layout of the decode kernels (read as the MFMA A operand straight from memory, 1 KiB per load);
//   X: block fragments (above), staged through LDS one k-step at a time, double-buffered, shared by the 8 waves.
//   Work-group = 256 output features (16 weight tiles) x 128 rows (8 column tiles) on 8 waves, each 4 weight tiles x
//   4 column tiles: a wave's k-step is 4 KiB of weights from memory, 8 KiB of fragments from LDS and 32 MFMAs (high and
//   low part of x), fp32 accumulators [4][4] tiles.  Output columns are stored in natural order (the row permutation of the weight layout is undone:
//   4 consecutive permuted rows are 4 consecutive features).  accumulate: Y += (the residual connections).
//   One order of additions per output (k ascending, high before low): results do not depend on R or on the grid.
constexpr int kBlkKs = 2;                              // k-steps per stage (the unit the k splits are counted in)
constexpr int kBlkStageU4 = (kBlkRows / 16) * 2 * 64;  // uint4 per LDS buffer (one k-step): 1024 (16 KiB)
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_gemm_bf16_block(const uint4* __restrict__ Wsw, int NTILES, int K,
                                                         const uint4* __restrict__ XF, int RT, int R,
                                                         float* __restrict__ Y, int ldy, int perm, int p0, int p1,
                                                         int accumulate, int stages_per_split, size_t split_stride) {
  // 8 waves: wave = (row half rh, feature group fw); a wave owns 4 weight tiles x 4 column tiles (64 x 64 outputs)
  // blockIdx.z = k split: with few rows and few features there are too few (feature, row) blocks to fill the chip, so
  // the k range is cut into gridDim.z pieces whose results go to Y + z * split_stride and are added up, in split
  // order, by k_block_reduce
  constexpr int NT = 4, CT = kBlkRows / 32, CTW = kBlkRows / 16;
  extern __shared__ uint4 lds[];                       // [2][kBlkStageU4]
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int fw = wave & 3, rh = wave >> 2;
  const int j = lane & 15, g = lane >> 4;
  const int tile0 = (blockIdx.x * 4 + fw) * NT;
  const int ct0 = blockIdx.y * CTW;                    // first column tile of the work-group
  const int units_total = K / kUnitK;
  const int nstages_all = (K >> 5) / kBlkKs;           // K is a multiple of 256: whole stages
  const int stage0 = blockIdx.z * stages_per_split;
  const int nstages = min(nstages_all, stage0 + stages_per_split);     // this split's stages: [stage0, nstages)
  Y += blockIdx.z * split_stride;
  int tile_c[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) tile_c[t] = min(tile0 + t, NTILES - 1);

  // this split's k-steps: [ks0, ks_end), a multiple of 4 (K is a multiple of 256 and a split an even number of stages)
  const int ks0 = stage0 * kBlkKs, ks_end = nstages * kBlkKs, ks_last = ks_end - 1;
  // weights of k-step s (past the split's end the last one is read again): 4 tiles x 1 KiB
  auto load_a = [&](uint4 (&a)[NT], int s_) {
    const int s = min(s_, ks_last), c = s >> 4, kk = s & 15;
    const int ksteps_c = min(kSliceUnits, units_total - c * kSliceUnits) * 8;
    const uint4* wbase = Wsw + (size_t)c * NTILES * (kSliceUnits * 8) * 64 + (size_t)kk * 64 + lane;
#pragma unroll
    for (int t = 0; t < NT; ++t) a[t] = wbase[(size_t)tile_c[t] * ksteps_c * 64];
  };
  f32x4 acc[NT][CT];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) acc[t][ct] = f32x4{0.f, 0.f, 0.f, 0.f};

  // one k-step: the work-group's 8 column tiles x (high, low) are 1024 consecutive uint4 of LDS buffer buf
  auto compute = [&](const uint4 (&a)[NT], int buf) {
    const uint4* src = lds + buf * kBlkStageU4 + (rh * CT * 2) * 64 + lane;
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
      const bf16x8 vh = __builtin_bit_cast(bf16x8, src[(ct * 2) * 64]);
      const bf16x8 vl = __builtin_bit_cast(bf16x8, src[(ct * 2 + 1) * 64]);
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        const bf16x8 av = __builtin_bit_cast(bf16x8, a[t]);
        acc[t][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, vh, acc[t][ct], 0, 0, 0);
      }
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        const bf16x8 av = __builtin_bit_cast(bf16x8, a[t]);
        acc[t][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, vl, acc[t][ct], 0, 0, 0);
      }
    }
  };
  // Rings of four k-steps in registers, for the weights (4 x 16) and for the fragments on their way to LDS (4 x 8):
  // before the arithmetic of k-step s, weights and fragments of k-step s + 3 are requested, so a request has three
  // k-steps' arithmetic to come back in (with one stage of two k-steps the waves spent nearly half their cycles waiting for memory, also at
  // thousands of rows); after the arithmetic the fragments of k-step s + 1 go to the other LDS buffer.  Four k-steps
  // per turn of the loop name the rings' registers statically; a split's k-steps are a multiple of four, so no turn
  // ends early.  All requests are unconditional.  Two waves per SIMD fill each other's waits for LDS and memory.
  uint4 a0[NT], a1[NT], a2[NT], a3[NT];
  uint4 b0_0, b0_1, b1_0, b1_1, b2_0, b2_1, b3_0, b3_1;    // (plain variables: small arrays ended up in scratch memory)
#define STAIRS_LOAD_B(b, s_)                                                                      \
  do {                                                                                            \
    const uint4* src_ = XF + ((size_t)min((s_), ks_last) * RT + ct0) * 2 * 64 + tid;              \
    b##_0 = src_[0];                                                                              \
    b##_1 = src_[512];                                                                            \
  } while (0)
#define STAIRS_STORE_B(buf, b)                               \
  do {                                                       \
    uint4* dst_ = lds + (buf) * kBlkStageU4 + tid;           \
    dst_[0] = b##_0;                                         \
    dst_[512] = b##_1;                                       \
  } while (0)
  // k-step s in LDS buffer buf: ac = its weights, an / bn = the ring slots for k-step s + 3, bs = the fragments of s + 1
#define STAIRS_BLOCK_STEP(ac, an, bn, bs, s, buf)            \
  do {                                                       \
    STAIRS_LOAD_B(bn, (s) + 3);                              \
    load_a(an, (s) + 3);                                     \
    __builtin_amdgcn_sched_barrier(0);                       \
    compute(ac, buf);                                        \
    STAIRS_STORE_B((buf) ^ 1, bs);                           \
    __syncthreads();                                         \
  } while (0)
  STAIRS_LOAD_B(b0, ks0);
  load_a(a0, ks0);
  STAIRS_LOAD_B(b1, ks0 + 1);
  load_a(a1, ks0 + 1);
  STAIRS_LOAD_B(b2, ks0 + 2);
  load_a(a2, ks0 + 2);
  STAIRS_STORE_B(0, b0);
  __syncthreads();
  for (int ks = ks0; ks < ks_end; ks += 4) {
    STAIRS_BLOCK_STEP(a0, a3, b3, b1, ks, 0);
    STAIRS_BLOCK_STEP(a1, a0, b0, b2, ks + 1, 1);
    STAIRS_BLOCK_STEP(a2, a1, b1, b3, ks + 2, 0);
    STAIRS_BLOCK_STEP(a3, a2, b2, b0, ks + 3, 1);
  }
#undef STAIRS_BLOCK_STEP
#undef STAIRS_LOAD_B
#undef STAIRS_STORE_B

#pragma unroll
  for (int t = 0; t < NT; ++t) {
    if (tile0 + t < NTILES) {
      const size_t col = perm_row((tile0 + t) * 16 + 4 * g, perm, p0, p1);
#pragma unroll
      for (int ct = 0; ct < CT; ++ct) {
        const int row = (ct0 + rh * CT + ct) * 16 + j;
        if (row < R) {
          float4* dst = reinterpret_cast<float4*>(Y + (size_t)row * ldy + col);
          float4 v = make_float4(acc[t][ct][0], acc[t][ct][1], acc[t][ct][2], acc[t][ct][3]);
          if (accumulate) {
            const float4 o = *dst;
            v.x = v.x + o.x; v.y = v.y + o.y; v.z = v.z + o.z; v.w = v.w + o.w;
          }
          *dst = v;
        }
      }
    }
  }
}

// Y = (accumulate ? Y : 0) + part[0] + part[1] + ... (in that order): the k splits of a block GEMM with few rows
__global__ __launch_bounds__(256) void k_block_reduce(const float* __restrict__ part, int nsplit, size_t split_stride, int R, int N,
                                                      float* __restrict__ Y, int ldy, int accumulate) {
  const int r = blockIdx.y, c = (blockIdx.x * 256 + threadIdx.x) * 4;
  if (c >= N) return;
  float4* dst = reinterpret_cast<float4*>(Y + (size_t)r * ldy + c);
  float4 a = accumulate ? *dst : make_float4(0.f, 0.f, 0.f, 0.f);
  for (int z = 0; z < nsplit; ++z) {
    const float4 v = *reinterpret_cast<const float4*>(part + z * split_stride + (size_t)r * N + c);
    a.x = a.x + v.x; a.y = a.y + v.y; a.z = a.z + v.z; a.w = a.w + v.w;
  }
  *dst = a;
}

void launch_gemm_block(const void* W, int N, int K, const uint4* xfrag, int R, float* Y, int ldy, int perm, int p0, int p1,
                       int accumulate, hipStream_t st, float* part, size_t part_floats) {
  const int NTILES = N / 16;
  const int FB = (NTILES + 15) / 16, RB = (R + kBlkRows - 1) / kBlkRows;
  const int nstages = (K / 32) / kBlkKs;
  // few (feature, row) blocks: cut k into pieces until about every CU has a work-group (each piece at least 8 stages
  // and an even number of them), as far as the scratch for the pieces' results reaches
  int nsplit = 1;
  if (part && FB * RB < 160) {
    nsplit = std::min({(256 + FB * RB - 1) / (FB * RB), nstages / 8, (int)(part_floats / ((size_t)R * N))});
    nsplit = std::max(nsplit, 1);
  }
  int per = (nstages + nsplit - 1) / nsplit;
  per += per & 1;
  nsplit = (nstages + per - 1) / per;
  dim3 grid(FB, RB, nsplit), block(512);
  const size_t lds = 2 * kBlkStageU4 * sizeof(uint4);
  if (nsplit == 1) {
    hipLaunchKernelGGL(k_gemm_bf16_block, grid, block, lds, st, static_cast<const uint4*>(W), NTILES, K, xfrag, pf_col_tiles(R), R, Y,
                       ldy, perm, p0, p1, accumulate, per, (size_t)0);
    return;
  }
  const size_t stride = (size_t)R * N;
  hipLaunchKernelGGL(k_gemm_bf16_block, grid, block, lds, st, static_cast<const uint4*>(W), NTILES, K, xfrag, pf_col_tiles(R), R, part,
                     N, perm, p0, p1, 0, per, stride);
  hipLaunchKernelGGL(k_block_reduce, dim3((N / 4 + 255) / 256, R), dim3(256), 0, st, part, nsplit, stride, R, N, Y, ldy, accumulate);
}

__global__ __launch_bounds__(256) void k_pf_embed(const uint16_t* __restrict__ emb, const int* __restrict__ tokens, int p0,
                                                  int tok_cap, int vocab, int d, float* __restrict__ x) {
  const int r = blockIdx.y, c = (blockIdx.x * 256 + threadIdx.x) * 4;
  if (c >= d) return;
  const int p = p0 + r;
  const int id = (p >= 0 && p < tok_cap) ? tokens[p] : -1;     // as k_embed: never outside the array or the table
  float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
  if (id >= 0 && id < vocab) {
    const uint16_t* row = emb + (size_t)id * d + c;
    v = make_float4(load_kv(row), load_kv(row + 1), load_kv(row + 2), load_kv(row + 3));
  }
  *reinterpret_cast<float4*>(x + (size_t)r * d + c) = v;
}
void launch_pf_embed(const uint16_t* emb, const int* tokens, int p0, int tok_cap, int vocab, int R, int d, float* x,
                     hipStream_t st) {
  hipLaunchKernelGGL(k_pf_embed, dim3((d + 1023) / 1024, R), dim3(256), 0, st, emb, tokens, p0, tok_cap, vocab, d, x);
}

__global__ __launch_bounds__(256) void k_pf_norm_split(const float* __restrict__ x, const float* __restrict__ gain, float eps,
                                                       int d, uint4* __restrict__ frag, int RT) {
  __shared__ float sm[4];
  const int r = blockIdx.x, tid = threadIdx.x;
  const float* row = x + (size_t)r * d;
  float rstd = 1.0f;
  if (gain) {
    float ss = 0.f;
    for (int c = tid * 4; c < d; c += 1024) {
      const float4 v = *reinterpret_cast<const float4*>(row + c);
      ss += sumsq4(v.x, v.y, v.z, v.w);
    }
    ss = block_sum_256(ss, sm);
    rstd = 1.0f / sqrtf(ss / (float)d + eps);
  }
  for (int c = tid * 4; c < d; c += 1024) {
    const float4 v = *reinterpret_cast<const float4*>(row + c);
    float e[4] = {v.x, v.y, v.z, v.w};
    if (gain) {
      const float4 g = *reinterpret_cast<const float4*>(gain + c);
      e[0] = e[0] * rstd * g.x; e[1] = e[1] * rstd * g.y; e[2] = e[2] * rstd * g.z; e[3] = e[3] * rstd * g.w;
    }
    pf_store_frag4(frag, RT, r, c, e);
  }
}
void launch_pf_norm_split(const float* x, const float* gain, float eps, int R, int d, uint4* frag, hipStream_t st) {
  hipLaunchKernelGGL(k_pf_norm_split, dim3(R), dim3(256), 0, st, x, gain, eps, d, frag, pf_col_tiles(R));
}

__global__ void k_pf_rope_table(int p0, int hd, double theta, float2* __restrict__ cs) {
  const int r = blockIdx.x, i = threadIdx.x;
  if (i >= hd / 2) return;
  const double ang = (double)(p0 + r) * pow(theta, -2.0 * (double)i / (double)hd);
  cs[r * 64 + i] = make_float2((float)cos(ang), (float)sin(ang));
}
void launch_pf_rope_table(int p0, int R, int hd, float theta, float2* cs, hipStream_t st) {
  hipLaunchKernelGGL(k_pf_rope_table, dim3(R), dim3(64), 0, st, p0, hd, (double)theta, cs);
}

__global__ __launch_bounds__(256) void k_pf_rope_kv(const float* __restrict__ y, int d, int H, int hd, int p0,
                                                    const float2* __restrict__ cs, float* __restrict__ q_rot,
                                                    _Float16* __restrict__ Kc, _Float16* __restrict__ Vc, int cap) {
  // thread = (row r, head h, pair e < hd/2)
  const int r = blockIdx.y, half = hd >> 1;
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx >= H * half) return;
  const int h = idx / half, e = idx - h * half;
  const int p = p0 + r;
  const float* yr = y + (size_t)r * 3 * d + h * hd;
  const float2 c = cs[r * 64 + e];
  const float2 q = rope_rotate(yr[e], yr[e + half], c);
  q_rot[(size_t)r * d + h * hd + e] = q.x;
  q_rot[(size_t)r * d + h * hd + e + half] = q.y;
  const float2 k = rope_rotate(yr[d + e], yr[d + e + half], c);
  _Float16* kd = Kc + (size_t)h * cap * hd;
  store_kv(kd + k_cache_off(p, e, hd), k.x);
  store_kv(kd + k_cache_off(p, e + half, hd), k.y);
  _Float16* vd = Vc + (size_t)h * cap * hd;
  store_kv(vd + v_cache_off(p, e, hd), yr[2 * d + e]);
  store_kv(vd + v_cache_off(p, e + half, hd), yr[2 * d + e + half]);
}
// The same for rows that sit wherever `pos` puts them (several sequences: row r belongs to slot slot_of(pos, r), whose
// caches start kv_slot_stride elements after the previous slot's); a row without a position writes nothing.
__global__ __launch_bounds__(256) void k_pf_rope_kv_rows(const float* __restrict__ y, int d, int H, int hd, PosRef pos,
                                                         size_t kv_slot_stride, const float2* __restrict__ cs,
                                                         float* __restrict__ q_rot, _Float16* __restrict__ Kc,
                                                         _Float16* __restrict__ Vc, int cap) {
  const int r = blockIdx.y, half = hd >> 1;
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx >= H * half) return;
  const int h = idx / half, e = idx - h * half;
  const int p = pos_of(pos, r);
  const float* yr = y + (size_t)r * 3 * d + h * hd;
  const float2 c = cs[r * 64 + e];
  const float2 q = rope_rotate(yr[e], yr[e + half], c);
  q_rot[(size_t)r * d + h * hd + e] = q.x;
  q_rot[(size_t)r * d + h * hd + e + half] = q.y;
  if (p < 0 || p >= cap) return;
  const size_t off = (size_t)slot_of(pos, r) * kv_slot_stride + (size_t)h * cap * hd;
  const float2 k = rope_rotate(yr[d + e], yr[d + e + half], c);
  store_kv(Kc + off + k_cache_off(p, e, hd), k.x);
  store_kv(Kc + off + k_cache_off(p, e + half, hd), k.y);
  store_kv(Vc + off + v_cache_off(p, e, hd), yr[2 * d + e]);
  store_kv(Vc + off + v_cache_off(p, e + half, hd), yr[2 * d + e + half]);
}
void launch_pf_rope_kv_rows(const float* y, int R, int d, int H, PosRef pos, size_t kv_slot_stride, const float2* cs,
                            float* q_rot, _Float16* Kc, _Float16* Vc, int cap, hipStream_t st) {
  const int hd = d / H;
  hipLaunchKernelGGL(k_pf_rope_kv_rows, dim3((H * hd / 2 + 255) / 256, R), dim3(256), 0, st, y, d, H, hd, pos, kv_slot_stride, cs,
                     q_rot, Kc, Vc, cap);
}

void launch_pf_rope_kv(const float* y, int R, int d, int H, int p0, const float2* cs, float* q_rot, _Float16* Kc,
                       _Float16* Vc, int cap, hipStream_t st) {
  const int hd = d / H;
  hipLaunchKernelGGL(k_pf_rope_kv, dim3((H * hd / 2 + 255) / 256, R), dim3(256), 0, st, y, d, H, hd, p0, cs, q_rot, Kc, Vc, cap);
}

__global__ __launch_bounds__(256) void k_pf_swiglu_split(const float* __restrict__ y, int f, uint4* __restrict__ frag, int RT) {
  const int r = blockIdx.y, c = (blockIdx.x * 256 + threadIdx.x) * 4;
  if (c >= f) return;
  const float4 g = *reinterpret_cast<const float4*>(y + (size_t)r * 2 * f + c);
  const float4 u = *reinterpret_cast<const float4*>(y + (size_t)r * 2 * f + f + c);
  const float e[4] = {swiglu(g.x, u.x), swiglu(g.y, u.y), swiglu(g.z, u.z), swiglu(g.w, u.w)};
  pf_store_frag4(frag, RT, r, c, e);
}
void launch_pf_swiglu_split(const float* y, int R, int f, uint4* frag, hipStream_t st) {
  hipLaunchKernelGGL(k_pf_swiglu_split, dim3((f + 1023) / 1024, R), dim3(256), 0, st, y, f, frag, pf_col_tiles(R));
}

// plain streaming copy, the calibration kernel for HBM traffic counters
__global__ __launch_bounds__(256) void k_copy_probe(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) dst[i] = src[i];
}

void launch_copy_probe(const void* src, void* dst, size_t bytes, hipStream_t st) {
  const size_t n = bytes / 16;
  hipLaunchKernelGGL(k_copy_probe, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st,
                     static_cast<const uint4*>(src), static_cast<uint4*>(dst), n);
}

hipError_t configure_kernels() {
  hipError_t e = hipSuccess;
  auto optin = [&](const void* fn, size_t bytes) {
    const hipError_t r = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (r != hipSuccess) e = r;
  };
#define STAIRS_OPTIN2(r, st)                                                                       \
  optin((const void*)k_gemm_bf16_rows<r, kRoleQKV, 4, 2, st>, kRowsPathMaxLds);                    \
  optin((const void*)k_gemm_bf16_rows<r, kRoleGateUp, 4, 2, st>, kRowsPathMaxLdsWide);             \
  optin((const void*)k_gemm_bf16_rows<r, kRoleHead, 4, 2, st>, kRowsPathMaxLds);                   \
  optin((const void*)k_gemm_bf16_rows<r, kRoleWo, 8, 1, st>, kRowsPathMaxLdsWide);                 \
  optin((const void*)k_gemm_bf16_rows<r, kRoleDown, 8, 3, st>, kRowsPathMaxLdsWide);               \
  optin((const void*)k_gemm_bf16_rows<r, kRoleDown, 16, 1, st>, kRowsPathMaxLdsWide)
#define STAIRS_OPTIN(r)    \
  STAIRS_OPTIN2(r, true);  \
  STAIRS_OPTIN2(r, false)
  STAIRS_OPTIN(1);
  STAIRS_OPTIN(2);
  STAIRS_OPTIN(3);
  STAIRS_OPTIN(4);
#undef STAIRS_OPTIN2
#define STAIRS_OPTIN2(r, st)                                                                       \
  optin((const void*)k_gemm_bf16_rows<r, kRoleQKV, 4, 2, st>, kRowsPathMaxLdsWide);                \
  optin((const void*)k_gemm_bf16_rows<r, kRoleGateUp, 4, 2, st>, kRowsPathMaxLdsWide);             \
  optin((const void*)k_gemm_bf16_rows<r, kRoleHead, 4, 2, st>, kRowsPathMaxLdsWide);               \
  optin((const void*)k_gemm_bf16_rows<r, kRoleWo, 8, 1, st>, kRowsPathMaxLdsWide)
  STAIRS_OPTIN(5);
  STAIRS_OPTIN(6);
  STAIRS_OPTIN(7);
#undef STAIRS_OPTIN2
#undef STAIRS_OPTIN
#define STAIRS_OPTIN_WIDE(ct, nt, dp0)                                                                   \
  constexpr int dp_##ct##_##nt = (ct) == 1 ? (dp0) : (ct) == 2 ? wide_depth2(dp0) : (ct) == 3 ? wide_depth3(dp0) : wide_depth4(dp0);   \
  STAIRS_OPTIN_WIDE_(ct, nt, dp_##ct##_##nt)
#define STAIRS_OPTIN_WIDE_(ct, nt, dp)                                           \
  optin((const void*)k_gemm_bf16_wide<ct, nt, dp, true>, kWideMaxLds);            \
  optin((const void*)k_gemm_bf16_wide<ct, nt, dp, false>, kWideMaxLds)
  STAIRS_OPTIN_WIDE(1, 8, kWideDepth8); STAIRS_OPTIN_WIDE(2, 8, kWideDepth8);
  STAIRS_OPTIN_WIDE(1, 6, kWideDepth6); STAIRS_OPTIN_WIDE(2, 6, kWideDepth6);
  STAIRS_OPTIN_WIDE(1, 3, kWideDepth3); STAIRS_OPTIN_WIDE(2, 3, kWideDepth3);
  STAIRS_OPTIN_WIDE(1, 4, kWideDepth4); STAIRS_OPTIN_WIDE(2, 4, kWideDepth4);
  STAIRS_OPTIN_WIDE(1, 2, kWideDepth2); STAIRS_OPTIN_WIDE(2, 2, kWideDepth2);
  STAIRS_OPTIN_WIDE(1, 1, kWideDepth1); STAIRS_OPTIN_WIDE(2, 1, kWideDepth1);
  STAIRS_OPTIN_WIDE(3, 4, kWideDepth4); STAIRS_OPTIN_WIDE(4, 4, kWideDepth4);
  STAIRS_OPTIN_WIDE(3, 2, kWideDepth2); STAIRS_OPTIN_WIDE(4, 2, kWideDepth2);
  STAIRS_OPTIN_WIDE(3, 1, kWideDepth1); STAIRS_OPTIN_WIDE(4, 1, kWideDepth1);
#undef STAIRS_OPTIN_WIDE
#undef STAIRS_OPTIN_WIDE_
  optin((const void*)k_gemm_bf16_block, 2 * kBlkStageU4 * sizeof(uint4));
  // the stand-alone attention merge keeps a table of all chunks in LDS: large for long contexts (the fused
  // merge runs for at most kAttnFusedMaxChunks chunks and stays small)
  optin((const void*)k_attn_merge<128>, kAttnMergeMaxLds);
  optin((const void*)k_attn_merge<64>, kAttnMergeMaxLds);
  return e;
}

}  // namespace stairs
