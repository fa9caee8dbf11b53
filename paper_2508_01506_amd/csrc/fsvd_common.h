// Device-side building blocks shared by the fsvd kernels (gfx950 only).
//
// Matrix-core convention used everywhere (v_mfma_f32_32x32x16_f16, one wavefront of 64 lanes):
//   A operand: lane l supplies 8 halves of row (l % 32), contraction slots 8*(l / 32) .. +7
//   B operand: lane l supplies 8 halves of column (l % 32), same contraction slots
//   accumulator register v (0..15) of lane l holds row 8*(v/4) + 4*(l/32) + (v%4), column l % 32
// Which logical index a contraction slot stands for is free as long as A and B agree; the kernels
// use that freedom to feed accumulators of one product straight into the next product.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fsvd {

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h4 __attribute__((ext_vector_type(4)));
typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef float f16v __attribute__((ext_vector_type(16)));
typedef float f8v __attribute__((ext_vector_type(8)));
typedef float f4v __attribute__((ext_vector_type(4)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));
typedef uint32_t u2 __attribute__((ext_vector_type(2)));

enum : int { DT_F16 = 0, DT_BF16 = 1, DT_F32 = 2 };

constexpr int kWave = 64;

__device__ __forceinline__ f16v mfma32(h8 a, h8 b, f16v c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ f16v zero16() {
  f16v z;
#pragma unroll
  for (int i = 0; i < 16; ++i) z[i] = 0.f;
  return z;
}

// two bf16 packed in one dword -> two fp16 packed in one dword (exact in fp16's normal range)
__device__ __forceinline__ uint32_t bf16x2_to_f16x2(uint32_t w) {
  float lo = __uint_as_float(w << 16);
  float hi = __uint_as_float(w & 0xffff0000u);
  auto p = __builtin_amdgcn_cvt_pkrtz(lo, hi);
  return __builtin_bit_cast(uint32_t, p);
}

// 8 stored 16-bit values (one 16-byte load) -> 8 halves
template <int DT>
__device__ __forceinline__ h8 raw_to_h8(u4 raw) {
  if constexpr (DT == DT_BF16) {
    u4 c;
#pragma unroll
    for (int i = 0; i < 4; ++i) c[i] = bf16x2_to_f16x2(raw[i]);
    return __builtin_bit_cast(h8, c);
  } else {
    return __builtin_bit_cast(h8, raw);
  }
}

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// scalar read of a stored parameter (bias, gamma, beta) as float
__device__ __forceinline__ float load_param(const void* p, size_t i, int dt) {
  if (dt == DT_F16) return (float)((const _Float16*)p)[i];
  if (dt == DT_BF16) return bf16_bits_to_float(((const uint16_t*)p)[i]);
  return ((const float*)p)[i];
}

__device__ __forceinline__ uint16_t float_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

__device__ __forceinline__ void store_out(void* p, size_t i, float v, int dt) {
  if (dt == DT_F32) ((float*)p)[i] = v;
  else if (dt == DT_F16) ((_Float16*)p)[i] = (_Float16)v;
  else ((uint16_t*)p)[i] = float_to_bf16_bits(v);
}

// 4 consecutive elements (index a multiple of 4, base 16-byte aligned) of a typed array
__device__ __forceinline__ f4v load4(const void* p, size_t i, int dt) {
  if (dt == DT_F32) return *(const f4v*)((const float*)p + i);
  const u2 raw = *(const u2*)((const uint16_t*)p + i);
  f4v o;
  if (dt == DT_F16) {
    const h4 h = __builtin_bit_cast(h4, raw);
    o[0] = (float)h[0]; o[1] = (float)h[1]; o[2] = (float)h[2]; o[3] = (float)h[3];
  } else {
    o[0] = __uint_as_float(raw[0] << 16); o[1] = __uint_as_float(raw[0] & 0xffff0000u);
    o[2] = __uint_as_float(raw[1] << 16); o[3] = __uint_as_float(raw[1] & 0xffff0000u);
  }
  return o;
}
__device__ __forceinline__ void store4(void* p, size_t i, f4v x, int dt) {
  if (dt == DT_F32) {
    *(f4v*)((float*)p + i) = x;
  } else if (dt == DT_F16) {
    h4 h;
    h[0] = (_Float16)x[0]; h[1] = (_Float16)x[1]; h[2] = (_Float16)x[2]; h[3] = (_Float16)x[3];
    *(h4*)((_Float16*)p + i) = h;
  } else {
    u2 raw;
    raw[0] = (uint32_t)float_to_bf16_bits(x[0]) | ((uint32_t)float_to_bf16_bits(x[1]) << 16);
    raw[1] = (uint32_t)float_to_bf16_bits(x[2]) | ((uint32_t)float_to_bf16_bits(x[3]) << 16);
    *(u2*)((uint16_t*)p + i) = raw;
  }
}

// 8 consecutive elements of a row-major activation (row pointer already applied) as an MFMA fragment.
// AT: storage type of the activation.  `ok` false yields zeros (ragged contraction tails).
template <int AT>
__device__ __forceinline__ h8 load_act8(const void* base, size_t elem_off, bool ok) {
  if constexpr (AT == DT_F32) {
    f4v lo = {0.f, 0.f, 0.f, 0.f}, hi = {0.f, 0.f, 0.f, 0.f};
    if (ok) {
      const f4v* p = (const f4v*)((const float*)base + elem_off);
      lo = p[0];
      hi = p[1];
    }
    h8 r;
    r[0] = (_Float16)lo[0]; r[1] = (_Float16)lo[1]; r[2] = (_Float16)lo[2]; r[3] = (_Float16)lo[3];
    r[4] = (_Float16)hi[0]; r[5] = (_Float16)hi[1]; r[6] = (_Float16)hi[2]; r[7] = (_Float16)hi[3];
    return r;
  } else {
    u4 raw = {0u, 0u, 0u, 0u};
    if (ok) raw = *(const u4*)((const uint16_t*)base + elem_off);
    return raw_to_h8<AT>(raw);
  }
}

// ---------------------------------------------------------------------------------------------
// Buffer addressing.  A tensor (or the part of it that starts at some scalar byte offset) is
// described by a 128-bit resource held in scalar registers; an access is resource + one 32-bit
// per-lane byte offset (+ immediate), and an access whose per-lane offset reaches the resource's
// size returns zero instead of touching memory.  Only the per-lane offset takes part in that
// range check, so a tile base is folded into the resource itself (rsrc_at) rather than passed as
// a scalar offset; row tails of a contraction (k >= K) then need no code, and a lane that must
// read nothing passes kOobOffset.  Tensors addressed this way must be smaller than 2 GiB.
// ---------------------------------------------------------------------------------------------
typedef __amdgpu_buffer_rsrc_t rsrc_t;
constexpr int kOobOffset = 0x7fff0000;   // plus any immediate it stays above every resource size and below 2^31

// resource covering [base + off, base + total)
__device__ __forceinline__ rsrc_t rsrc_at(const void* base, long long total, long long off) {
  long long left = total - off;
  left = left < 0 ? 0 : left;
  return __builtin_amdgcn_make_buffer_rsrc((void*)((const char*)base + (left > 0 ? off : 0)), 0, (int)left, 0x00020000);
}
__device__ __forceinline__ u4 buf_load16(rsrc_t r, int voff) { return __builtin_amdgcn_raw_buffer_load_b128(r, voff, 0, 0); }
__device__ __forceinline__ u2 buf_load8(rsrc_t r, int voff) { return __builtin_amdgcn_raw_buffer_load_b64(r, voff, 0, 0); }

// 4 consecutive stored parameters (e.g. bias) as floats
template <int WT>
__device__ __forceinline__ f4v raw_to_f4(u2 raw) {
  f4v o;
  if constexpr (WT == DT_BF16) {
    o[0] = __uint_as_float(raw[0] << 16); o[1] = __uint_as_float(raw[0] & 0xffff0000u);
    o[2] = __uint_as_float(raw[1] << 16); o[3] = __uint_as_float(raw[1] & 0xffff0000u);
  } else {
    h4 h = __builtin_bit_cast(h4, raw);
    o[0] = (float)h[0]; o[1] = (float)h[1]; o[2] = (float)h[2]; o[3] = (float)h[3];
  }
  return o;
}

// The two halves of a wavefront combined: lanes l and l ^ 32 both receive op(x[l % 32], x[l % 32 + 32]).  One
// v_permlane32_swap exchanges the upper half of one register with the lower half of another: no LDS round trip.
__device__ __forceinline__ float halves_max(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float halves_sum(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// ---------------------------------------------------------------------------------------------
// Fragment-major ("FM") layout of an fp16 activation A[T, K] that will be an MFMA operand.
// Tokens are grouped in tiles of 32 and the contraction axis in chunks of 64; one (tile, chunk)
// block is 4 KiB holding, for MFMA step kk = 0..3, the 64 lanes' 16-byte operand registers in
// lane order: lane (t % 32) + 32 g owns k = 64 c + 32 g + 8 kk + 0..7 of token t.  A wavefront
// therefore fetches an operand with ONE fully contiguous 1 KiB load, and a producer whose
// accumulators hold 4 consecutive k per lane writes contiguous 512-byte runs.
// ---------------------------------------------------------------------------------------------
__host__ __device__ __forceinline__ size_t fm_bytes(size_t T, size_t K) {
  return ((T + 31) / 32) * ((K + 63) / 64) * 4096;
}
// byte offset of the 16-byte unit of (token t, lane group g) inside block (t / 32, chunk 0), step 0
__device__ __forceinline__ int fm_voff(int t, int kchunks, int g) {
  return (((t >> 5) * kchunks) * 256 + g * 32 + (t & 31)) * 16;
}
constexpr int kFmChunkBytes = 4096;
constexpr int kFmStepBytes = 1024;

// ---------------------------------------------------------------------------------------------
// Weight tiles in LDS.  Weights are row-major [K, N] with the contraction index K as the slow axis,
// while an MFMA operand wants 8 consecutive contraction slots per lane.  A tile is copied into LDS
// as it lies in memory ([k][n], 16 bytes = 8 columns per lane, rows fully coalesced, bf16 widened to
// fp16 on the way) and the transposition is done by the LDS itself on the way out: the gfx950
// transposing read ds_read_b64_tr_b16 lets every 16 lanes fetch a 4 (k) x 16 (n) block such that
// lane i receives column i's four k-values.  Two such reads make one operand register set.
// Rows are padded by 64 bytes so that the four 64-byte row segments touched by 32 lanes of a
// transposing read fall into disjoint banks.
// ---------------------------------------------------------------------------------------------
typedef short s4v __attribute__((ext_vector_type(4)));
constexpr int kChunkK = 64;                                   // contraction chunk staged per step
__host__ __device__ constexpr int wtile_stride(int ncols) { return ncols + 32; }   // halves per LDS row

// per-lane part of a transposing read's address (in halves): lane = 16 * group + i supplies row i / 4,
// columns 4 * (i % 4) of its group's 4 x 16 block; groups 0..3 are (columns 0-15 | 16-31) x (g = 0 | 1)
__device__ __forceinline__ int tr_lane_off(int lane, int stride) {
  const int i = lane & 15;
  return (i >> 2) * stride + 16 * ((lane >> 4) & 1) + 4 * (i & 3);
}
// operand registers of lane (column l % 32): k-rows of p0 then k-rows of p1 (4 each)
__device__ __forceinline__ h8 tr_frag(const _Float16* p0, const _Float16* p1) {
  const s4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s4v*)p0);
  const s4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s4v*)p1);
  typedef short s8v __attribute__((ext_vector_type(8)));
  const s8v r = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(h8, r);
}
// 8 stored weights (one 16-byte load) -> LDS as fp16
template <int WT>
__device__ __forceinline__ void stage_store16(_Float16* dst, u4 raw) {
  *(u4*)dst = __builtin_bit_cast(u4, raw_to_h8<WT>(raw));
}

// ---------------------------------------------------------------------------------------------
// Prepacked weights ("tile images").  A weight matrix [K, N] that is packed once, when the model is loaded, is
// stored as fp16 tiles of 128 (k) x 128 (n), zero-padded to whole tiles, tile (kt, nt) at
// (kt * ceil(N / 128) + nt) * 32 KiB.  A tile is stored exactly as it will lie in LDS, so a kernel moves it with
// loads that write LDS directly (no registers, no conversion).  Inside a tile, row k holds its 256 bytes with the
// four 64-byte segments permuted: element (k, n) sits at half  k * 128 + (((n / 32) ^ (k % 4)) * 32) + n % 32.
// The permutation does for unpadded rows what the 64-byte padding does for staged tiles: the four rows touched by
// 32 lanes of a transposing read fall into disjoint banks.
// ---------------------------------------------------------------------------------------------
constexpr int kWtTiled = 3;                                   // "weight type" of kernels reading tile images
constexpr int kTileImageBytes = 128 * 128 * 2;
__host__ __device__ __forceinline__ size_t tiled_bytes(size_t K, size_t N) {
  return ((K + 127) / 128) * ((N + 127) / 128) * (size_t)kTileImageBytes;
}
// per-lane part of a transposing read's address (in halves) inside a tile image, for the 32 columns 32 * seg ..;
// row offsets added to it must be multiples of 4
__device__ __forceinline__ int tr_lane_off_swz(int lane, int seg) {
  const int i = lane & 15;
  return (i >> 2) * 128 + ((seg ^ (i >> 2)) << 5) + 16 * ((lane >> 4) & 1) + 4 * (i & 3);
}
// One wavefront-wide 16-byte-per-lane load that writes LDS directly: lane l's 16 bytes at (resource base + soff +
// voff_l) go to LDS byte address lds_addr + 16 l (lds_addr wave-uniform).  Issued as inline assembly so that the
// compiler's wait-count bookkeeping does not see it: the compiler would otherwise wait for ALL such loads before any
// LDS read and before every barrier, which defeats requesting tiles ahead.  The caller orders these loads against
// their consumers with lds_dma_wait_barrier<N>() (they complete in issue order and are counted by vmcnt).  The
// statement is volatile (it keeps its place among the other requests and the wait/barrier statements) but does not
// clobber memory: ordinary LDS reads of other buffers may be scheduled across it.
__device__ __forceinline__ u4 lds_dma_rsrc(const void* base, unsigned bytes) {
  const unsigned long long b = (unsigned long long)base;
  u4 r;      // pinned to scalar registers: the load's resource operand cannot be a vector register
  r[0] = __builtin_amdgcn_readfirstlane((unsigned)b);
  r[1] = __builtin_amdgcn_readfirstlane((unsigned)(b >> 32) & 0xffffu);
  r[2] = __builtin_amdgcn_readfirstlane(bytes);
  r[3] = 0x00020000u;
  return r;
}
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"   // m0 is reserved; naming it documents that the statement overwrites it
__device__ __forceinline__ void lds_dma16(u4 rsrc, unsigned lds_addr, int voff, int soff) {
  lds_addr = __builtin_amdgcn_readfirstlane(lds_addr);
  soff = __builtin_amdgcn_readfirstlane(soff);
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
               :: "s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff) : "m0");
}
#pragma clang diagnostic pop
// wait until at most N of this wavefront's vector-memory operations are outstanding and all its LDS operations are
// done, then the workgroup barrier
template <int N>
__device__ __forceinline__ void lds_dma_wait_barrier() {
  asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" :: "n"(N) : "memory");
}
__device__ __forceinline__ unsigned lds_addr_of(const void* p) {
  return (unsigned)(size_t)(__attribute__((address_space(3))) const void*)p;
}

// ---------------------------------------------------------------------------------------------
// Activation functions of the FFN (applied to fp32 accumulators).
// Exact (erf) GELU as  max(x, 0) - |x| * Q(|x|),  Q(t) = 0.5 erfc(t / sqrt 2)  the upper Gaussian tail, with
// log2 Q(t) replaced on [0, 6] by a degree-6 polynomial (weighted least-squares fit on Chebyshev nodes, weight t Q(t)):
// 6 FMAs and one hardware exp2 per element.  |error| <= 5e-7 over the whole real line in fp32 (beyond t = 6 the tail
// is below 1e-9 and the clamp keeps the polynomial inside its interval).
__device__ constexpr float kGeluTail[7] = {-0.999994874f, -1.15118682f, -0.458807677f, -0.0533762164f,
                                           0.00806691311f, -0.000768144673f, 3.33612952e-05f};
__device__ __forceinline__ float gelu_erf_f(float x) {
  const float t = fminf(fabsf(x), 6.0f);
  float p = kGeluTail[6];
#pragma unroll
  for (int k = 5; k >= 0; --k) p = fmaf(p, t, kGeluTail[k]);
  return fmaf(-fabsf(x), __builtin_amdgcn_exp2f(p), fmaxf(x, 0.f));
}
__device__ __forceinline__ float gelu_tanh_f(float x) {
  const float u = 0.7978845608028654f * (x + 0.044715f * x * x * x);
  return x * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-2.0f * u * 1.4426950408889634f));
}

// Contraction-slot mapping inside one 64-wide chunk: MFMA step kk (0..3), lane group g (0..1),
// slot s (0..7) stand for chunk offset 32*g + 8*kk + s.  An activation lane therefore reads 64
// contiguous bytes of its row over the four steps of a chunk.
__device__ __forceinline__ int chunk_off(int kk, int g) { return 32 * g + 8 * kk; }

// blockIdx -> tile index so that each of the 8 XCDs (round-robin workgroup dispatch) walks a
// contiguous range of tiles and its L2 sees neighbouring tiles.
__device__ __forceinline__ int xcd_tile(int linear, int total) {
  if ((total & 7) != 0) return linear;
  return (linear & 7) * (total >> 3) + (linear >> 3);
}

// A kernel-argument pointer as an opaque wave-uniform value in scalar registers.  Selecting between two such
// pointers with a run-time condition then stays a scalar select instead of a lookup in a stack table of arguments.
__device__ __forceinline__ const char* uniform_ptr(const void* p) {
  const unsigned long long u = (unsigned long long)p;
  const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)u);
  const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(u >> 32));
  return (const char*)(((unsigned long long)hi << 32) | lo);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

}  // namespace fsvd
