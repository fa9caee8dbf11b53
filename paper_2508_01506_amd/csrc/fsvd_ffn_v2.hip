// FlashSVDFFN V2 (Alg. 3): the whole factored FFN of a block of tokens in one kernel,
//   out = phi((X U_1) V_1 + b_1) U_2 V_2 + b_2,
// with the rank projection X U_1 and the up-projection Z V_2 done inside the kernel as well, so that neither the
// rank-space activations P1 = X U_1 and Z nor the hidden activation ever exist in device memory: the kernel reads X and
// the four factor matrices and writes the result, and needs no workspace.
//
// One workgroup (8 wavefronts) owns 32 MT tokens and runs a chain of four products of the same shape,
//   Out^T [N, tokens] = W^T [N, K] . In^T [K, tokens],
// "transposed" so that tokens lie along the lanes: the accumulators of one product, rounded to fp16, are the operand
// registers of the next.  The activations between two products stay in LDS as ready operand fragments
// ([16-wide contraction step][token tile][lane] x 16 bytes): X is staged in slabs of 512 / MT columns, P1^T (later Z^T)
// takes up to 64 KiB, the activated hidden chunk (512 / MT features) 32 KiB; what is left of the 160 KiB holds weight
// steps.  All weights are prepacked tile images, copied straight into LDS one step at a time (16 contraction rows x 512
// columns, 16 KiB per workgroup) as ONE request stream over the whole kernel, NB - 1 steps ahead (a cursor walks the same
// loop nest as the consumers), so that the copies never drain between the products.  Within a 512-column block
// wavefront w owns columns 64 w .. 64 w + 63, and every wavefront requests, waits for and reads ITS OWN columns of a
// step (2 KiB, in a private part of LDS): no workgroup barrier separates the steps, the wavefronts drift apart inside a
// pass and meet only where the shared activation fragments change hands.
//   step 1: P1^T = U_1^T X^T                         (sum over D in slabs; all slabs of r1 per X slab)
//   step 2: per chunk of F: H^T = V_1^T P1^T + b_1, G = phi(H) -> LDS;  Z^T += U_2^T G^T  (Z^T stays in registers)
//   step 3: out^T = V_2^T Z^T + b_2 per 512-column slab of D, written row-major.
// Limits: r1, r2 <= 1024 / MT (the register and LDS budget of Z^T and P1^T).
#include "fsvd_common.h"
#include "fsvd_kernels.h"
#include <type_traits>

namespace fsvd {

namespace {

constexpr int kV2Threads = 512;
constexpr int kV2StepBytes = 16 * 512 * 2;     // one staged step of the workgroup: 16 rows x 512 columns (or 32 x 256)
constexpr int kV2WaveStepBytes = kV2StepBytes / 8;   // a wavefront's part of it

// The request stream of the kernel below: which 16-row x 512-column step of which factor matrix is copied into LDS
// next.  A pass is a run of consecutive 16-row steps of one matrix under one block of columns; the passes follow the
// loop nest of the four products in the order in which the consumer loops use the steps.  Inside a pass the next
// request is the previous one plus constants (a few scalar instructions per step); the loop nest is only consulted
// when a pass ends.  All of it is wave-uniform (scalar registers).
template <int MT, int NB>
struct WeightStream {
  static constexpr int KS = 32 / MT, FC = 16 * KS;
  u4 rs_u1, rs_v1, rs_u2, rs_v2;               // buffer descriptors of the four tile-image arrays
  int ntn_u1, ntn_v1, ntn_u2, ntn_v2;          // tile images per row of tiles
  int D, F, r1, r2, nxs, nsl1, nk1, nch, nsl2, nk2, nds;
  int ph, i0, i1;                              // pass cursor: product, outer index (X slab, chunk of F, slab of D), rank slab
  // the pass being requested
  u4 rs;                                       // its matrix
  int soff;                                    // byte offset (in the matrix) of the tile-image rows of the next step
  int left;                                    // steps of the pass not yet requested
  int krow;                                    // 16-row position of the next step inside its 128-row tile
  int kinc, adv;                               // 16-row units and bytes per step: 1 and 4096 (wide), 2 and 8192 (narrow)
  int jump;                                    // added when the next step enters the next row of tiles
  unsigned req_buf, lds_w0;                    // LDS address of this wavefront's buffer of the next request; of its buffer 0
  int buf;                                     // buffer of the step being consumed
  int wave;
  int voff_wide, voff_narrow;                  // this lane's source offset inside a group of 8 (wide) or 16 (narrow) image rows
  int pvoff;                                   // the one in use, or out of range when the wavefront's tile image lies right of the matrix

  __device__ __forceinline__ int steps_in(int total, int part) const {   // 16-row steps of part `part` (FC wide) of an axis
    const int k = (total - FC * part + 15) / 16;
    return k < KS ? k : KS;
  }
  // A pass whose block of columns is at most 256 wide is NARROW: its steps are 32 rows x 256 columns (two tile images)
  // instead of 16 x 512 (four), so that all eight wavefronts own a 32-column tile and the pass has half as many steps.
  static __device__ __forceinline__ bool is_narrow(int width) { return width <= 256; }
  static __device__ __forceinline__ int pass_steps(int k16, bool narrow) { return narrow ? (k16 + 1) >> 1 : k16; }
  // describe the pass the cursor points at
  __device__ __forceinline__ void load_pass() {
    int ntn, k0, n0, k16, width;
    const int xs = i0, ch = i0, ds = i0;
    if (ph == 0)      { rs = rs_u1; ntn = ntn_u1; k0 = FC * xs; n0 = 512 * i1; k16 = steps_in(D, xs); width = r1 - n0; }
    else if (ph == 1) { rs = rs_v1; ntn = ntn_v1; k0 = 0; n0 = FC * ch; k16 = nk1; width = FC; }
    else if (ph == 2) { rs = rs_u2; ntn = ntn_u2; k0 = FC * ch; n0 = 512 * i1; k16 = steps_in(F, ch); width = r2 - n0; }
    else if (ph == 3) { rs = rs_v2; ntn = ntn_v2; k0 = 0; n0 = 512 * ds; k16 = nk2; width = D - n0; }
    else              { rs = rs_v2; ntn = 1; k0 = 0; n0 = 0; k16 = 1 << 30; width = 512; }   // past the end: requests nobody consumes
#pragma unroll
    for (int i = 0; i < 4; ++i) rs[i] = __builtin_amdgcn_readfirstlane(rs[i]);   // the selected descriptor stays in scalar registers
    const bool narrow = is_narrow(width);
    left = pass_steps(k16, narrow);
    kinc = narrow ? 2 : 1;
    adv = narrow ? 8192 : 4096;
    krow = 0;                                          // every pass starts on a tile boundary (k0 is a multiple of 128)
    jump = ph < 4 ? (ntn - 1) * kTileImageBytes : -8 * 4096;   // past the end: the same tile again and again
    // this wavefront's columns: tile image (n0 / 128 + w / 2) wide, (n0 / 128 + w / 4) narrow
    int nt = (n0 >> 7) + (narrow ? wave >> 2 : wave >> 1);
    pvoff = nt < ntn ? (narrow ? voff_narrow : voff_wide) : kOobOffset;   // right of the matrix: nothing is read, zeros arrive
    nt = nt < ntn ? nt : ntn - 1;
    soff = __builtin_amdgcn_readfirstlane(((k0 >> 7) * ntn + nt) * kTileImageBytes);
    left = __builtin_amdgcn_readfirstlane(left);
    jump = __builtin_amdgcn_readfirstlane(jump);
    kinc = __builtin_amdgcn_readfirstlane(kinc);
    adv = __builtin_amdgcn_readfirstlane(adv);
  }
  __device__ __forceinline__ void next_pass() {
    if (ph == 0) {
      if (++i1 == nsl1) { i1 = 0; if (++i0 == nxs) { i0 = 0; ph = 1; } }
    } else if (ph == 1) {
      i1 = 0; ph = 2;
    } else if (ph == 2) {
      if (++i1 == nsl2) { i1 = 0; if (++i0 == nch) { i0 = 0; ph = 3; } else ph = 1; }
    } else if (ph == 3) {
      if (++i0 == nds) ph = 4;
    }
    ph = __builtin_amdgcn_readfirstlane(ph); i0 = __builtin_amdgcn_readfirstlane(i0); i1 = __builtin_amdgcn_readfirstlane(i1);
    load_pass();
  }
  __device__ __forceinline__ void init(const FfnV2Args& a, int wave_, int vw, int vn, unsigned lds_w0_) {
    D = a.D; F = a.F; r1 = a.r1; r2 = a.r2;
    rs_u1 = lds_dma_rsrc(a.U1, (unsigned)tiled_bytes(a.D, a.r1));
    rs_v1 = lds_dma_rsrc(a.V1, (unsigned)tiled_bytes(a.r1, a.F));
    rs_u2 = lds_dma_rsrc(a.U2, (unsigned)tiled_bytes(a.F, a.r2));
    rs_v2 = lds_dma_rsrc(a.V2, (unsigned)tiled_bytes(a.r2, a.D));
    ntn_u1 = (a.r1 + 127) / 128; ntn_v1 = (a.F + 127) / 128; ntn_u2 = (a.r2 + 127) / 128; ntn_v2 = (a.D + 127) / 128;
    nxs = (a.D + FC - 1) / FC; nsl1 = (a.r1 + 511) / 512; nk1 = (a.r1 + 15) / 16;
    nch = (a.F + FC - 1) / FC; nsl2 = (a.r2 + 511) / 512; nk2 = (a.r2 + 15) / 16;
    nds = (a.D + 511) / 512;
    ph = i0 = i1 = 0; buf = 0;
    wave = wave_; voff_wide = vw; voff_narrow = vn; lds_w0 = lds_w0_; req_buf = lds_w0_;
    load_pass();
  }
  // request the next step of the stream (this wavefront's 2 KiB of it) into the next buffer: two loads of 1 KiB, the
  // first and the second half of the step's rows
  __device__ __forceinline__ void request() {
    lds_dma16(rs, req_buf, pvoff, soff);
    lds_dma16(rs, req_buf + 1024, pvoff, soff + (adv >> 1));
    req_buf = req_buf + kV2WaveStepBytes == lds_w0 + NB * kV2WaveStepBytes ? lds_w0 : req_buf + kV2WaveStepBytes;
    soff += adv;
    krow += kinc;
    if (krow == 8) { krow = 0; soff += jump; }
    if (--left == 0) next_pass();
  }
  __device__ __forceinline__ void start() {      // the first NB - 1 steps
#pragma unroll
    for (int b = 0; b < NB - 1; ++b) request();
  }
  // Begins step s: requests step s + NB - 1 into the buffer this wavefront read during step s - 1 (those reads were
  // issued long before the new data can arrive), then waits until all but the newest NB - 1 requests (two loads each)
  // have landed: step s is in LDS.  Nobody else reads or writes this wavefront's buffers, so there is no barrier.
  __device__ __forceinline__ void begin_step() {
    asm volatile("" ::: "memory");               // the previous step's LDS reads stay ahead of the request in program order
    request();
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(2 * (NB - 1)) : "memory");
  }
  __device__ __forceinline__ void end_step() { buf = buf == NB - 1 ? 0 : buf + 1; }
};

template <int MT, int NB>
__global__ void __launch_bounds__(kV2Threads, 1) ffn_v2_kernel(FfnV2Args a) {
  constexpr int PK = 160 - 32 - 16 * NB;       // fragments (KiB) left for P1^T / Z^T: ranks up to 16 PK / MT
  constexpr int KS = 32 / MT;                  // contraction steps per X slab and per chunk of F (gfr holds KS * MT fragments)
  constexpr int FC = 16 * KS;                  // chunk of F, and X slab width
  constexpr int NTA = 2 / MT;                  // 32-feature tiles per wavefront in the hidden product
  constexpr int NSL = 2 / MT;                  // 512-column slabs of the ranks
  __shared__ __attribute__((aligned(16))) h8 pfr[PK][64];                  // P1^T, later Z^T: [step * MT + tile][lane]
  __shared__ __attribute__((aligned(16))) h8 gfr[32][64];                  // X slab, later the activated chunk
  __shared__ __attribute__((aligned(16))) _Float16 wbuf[8][NB][kV2WaveStepBytes / 2];   // [wavefront][buffer][its part of a step]

  const int tid = threadIdx.x;
  const int lane = tid & 63, l32 = lane & 31, g = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int T = a.T, D = a.D, F = a.F, r1 = a.r1, r2 = a.r2;
  const int tok0 = blockIdx.x * 32 * MT;

  // Where a lane's 16 bytes of a request come from (the 16-byte slot l of the 1 KiB that one load writes is LDS offset
  // 16 l).  A wavefront's part of a step is kept in blocks of 4 rows; inside a block the 64-byte segments (one row of one
  // 32-column tile) are ordered tile-major, row-minor, so that the four rows a transposing read touches lie in four
  // different groups of banks.  In the tile image, row k holds its 32-column segments permuted by k % 4.
  //   wide (8 rows x 128 bytes per load):  slot -> block l / 32, tile j = (l % 32) / 16, row (l % 16) / 4, piece l % 4
  //   narrow (16 rows x 64 bytes per load): slot -> block l / 16, row (l % 16) / 4, piece l % 4
  int vw, vn;
  {
    const int blk = lane >> 5, j = (lane >> 4) & 1, row = (lane >> 2) & 3, piece = lane & 3;
    vw = (4 * blk + row) * 256 + (((2 * (wave & 1) + j) ^ row) * 64) + piece * 16;
    const int blkn = lane >> 4;
    vn = (4 * blkn + row) * 256 + (((wave & 3) ^ row) * 64) + piece * 16;
  }
  WeightStream<MT, NB> ws;
  ws.init(a, wave, vw, vn, lds_addr_of(&wbuf[wave][0][0]));
  const int nxs = ws.nxs, nsl1 = ws.nsl1, nk1 = ws.nk1, nch = ws.nch, nsl2 = ws.nsl2, nk2 = ws.nk2, nds = ws.nds;
  auto steps_in = [&](int total, int part) __attribute__((always_inline)) { return ws.steps_in(total, part); };
  auto begin_step = [&]() __attribute__((always_inline)) { ws.begin_step(); };
  auto end_step = [&]() __attribute__((always_inline)) { ws.end_step(); };
  // Transposing-read offsets of this lane (halves inside this wavefront's part of a step).  Wide steps are kept in 4-row
  // blocks of 256 halves (tile j at + 128 j), narrow steps in 4-row blocks of 128 halves.  Which rows a lane reads
  // depends on where the activation operand comes from:
  //   accumulator order (every product but the first): rows 4 g .. + 3 and 8 + 4 g .. + 3 of a 16-row contraction step, the
  //     order in which an accumulator tile, rounded to fp16, supplies the contraction slots of the next product;
  //   plain order (the first product, whose X operand is staged from row-major memory): rows 8 g .. + 3 and 8 g + 4 .. + 3.
  const int trl = ((lane & 15) >> 2) * 32 + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
  // operand registers of one column tile for one 16-row contraction step: `off` = the lane's offset of its first four
  // rows, `second` = distance to its other four
  auto wfrag = [&](int bufi, int off, int second) __attribute__((always_inline)) {
    const _Float16* wt = &wbuf[wave][0][0] + bufi * (kV2WaveStepBytes / 2) + off;
    return tr_frag(wt, wt + second);
  };
  // One pass over `k16` 16-row contraction steps of a block of columns `width` wide that starts at this wavefront's
  // first column tile `first` of a matrix `n` columns wide: acc[j][mt] += (column tile)^T . act.  Wide blocks: two tiles
  // per wavefront (j = 0, 1), one contraction step per staged step; narrow blocks (see WeightStream): tile j = 0 only,
  // two contraction steps per staged step.
  auto mm_pass = [&](auto& acc, auto plain_c, bool narrow, int n_on, int k16, const h8* act) __attribute__((always_inline)) {
    constexpr bool PLAIN = decltype(plain_c)::value;
    const int nsteps = ws.pass_steps(k16, narrow);
    if (n_on == 0) {                                   // no tile of this wavefront inside the matrix: requests and barriers only
      for (int ks = 0; ks < nsteps; ++ks) { begin_step(); end_step(); }
      return;
    }
    if (narrow) {
      const int off = trl + (PLAIN ? 256 : 128) * g, second = PLAIN ? 128 : 256;
      for (int ks = 0; ks < nsteps; ++ks) {
        begin_step();
        const bool two = 2 * ks + 1 < k16;             // an odd number of contraction steps: the last staged step holds one
        h8 b[2], af[2][MT];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const int kk = two ? 2 * ks + u : 2 * ks;
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) af[u][mt] = act[(kk * MT + mt) * 64 + lane];
          b[u] = wfrag(ws.buf, off + u * 4 * 128, second);
        }
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[0][mt] = mfma32(b[0], af[0][mt], acc[0][mt]);
        if (two) {
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) acc[0][mt] = mfma32(b[1], af[1][mt], acc[0][mt]);
        }
        end_step();
      }
      return;
    }
    const int off = trl + (PLAIN ? 512 : 256) * g, second = PLAIN ? 256 : 512;
    for (int ks = 0; ks < nsteps; ++ks) {
      begin_step();
      h8 b[2], af[MT];
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) af[mt] = act[(ks * MT + mt) * 64 + lane];
#pragma unroll
      for (int j = 0; j < 2; ++j) b[j] = wfrag(ws.buf, off + 128 * j, second);   // (a wavefront with one tile inside the matrix reads both)
#pragma unroll
      for (int j = 0; j < 2; ++j)
        if (j < n_on) {
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) acc[j][mt] = mfma32(b[j], af[mt], acc[j][mt]);
        }
      end_step();
    }
  };
  // first column (relative to the block start) and number of this wavefront's tiles of a block `width` wide
  auto first_col = [&](bool narrow) __attribute__((always_inline)) { return narrow ? 32 * wave : 64 * wave; };
  auto tiles_on = [&](int first, int width, bool narrow) __attribute__((always_inline)) {   // tiles of this wavefront that start inside the block
    const int k = (width - first + 31) / 32, nt = narrow ? 1 : 2;
    return k < 0 ? 0 : (k < nt ? k : nt);
  };

  f16v zacc[NSL][2][MT];                       // P1^T in step 1, Z^T in step 2: slab, column tile, token tile
  auto clear_z = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int sl = 0; sl < NSL; ++sl)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) zacc[sl][j][mt] = zero16();
  };
  // rank-space accumulators -> operand fragments of the next product (ranks below `n` only)
  auto publish_z = [&](int n) __attribute__((always_inline)) {
#pragma unroll
    for (int sl = 0; sl < NSL; ++sl) {
      const bool narrow = ws.is_narrow(n - 512 * sl);
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int row0 = 512 * sl + first_col(narrow) + 32 * j;
        if (row0 < n && !(narrow && j > 0)) {
#pragma unroll
          for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
              h8 o;
#pragma unroll
              for (int i = 0; i < 8; ++i) o[i] = (_Float16)zacc[sl][j][mt][8 * s2 + i];
              pfr[(row0 / 16 + s2) * MT + mt][lane] = o;
            }
        }
      }
    }
  };
  // one slab of a rank-space product: z += W^T[512 sl .., steps] . act
  auto rank_pass = [&](f16v (&z)[2][MT], auto plain_c, int sl, int k16, int n, const h8* act) __attribute__((always_inline)) {
    const bool narrow = ws.is_narrow(n - 512 * sl);
    mm_pass(z, plain_c, narrow, tiles_on(first_col(narrow), n - 512 * sl, narrow), k16, act);
  };
  typedef std::true_type plain_order;
  typedef std::false_type acc_order;

  ws.start();

  // ================= step 1: P1^T = U_1^T X^T =================
  clear_z();
  for (int xs = 0; xs < nxs; ++xs) {
    const int kc = steps_in(D, xs);
    // X slab -> operand fragments in the plain order: lane (token, g) of step s holds columns 16 s + 8 g .. + 7 of its
    // token.  The slab is 32 MT rows x FC columns; a wavefront copies blocks of 8 rows x 64 columns (128 contiguous
    // bytes per row), 16 bytes per lane, four blocks each.
    {
      constexpr int CB = FC / 64;                      // 64-column blocks per row of the slab
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int blk = wave + 8 * i;                  // 32 blocks: (row group, column block)
        const int row = 8 * (blk / CB) + (lane & 7), pc = 8 * (blk % CB) + (lane >> 3);   // pc: 16-byte piece of the slab row
        const int tok = tok0 + row, col = FC * xs + 8 * pc;
        u4 raw = {0u, 0u, 0u, 0u};
        if (tok < T && col < D) raw = *(const u4*)((const uint16_t*)a.X + (size_t)tok * D + col);
        const h8 v = a.x_dt == DT_BF16 ? raw_to_h8<DT_BF16>(raw) : raw_to_h8<DT_F16>(raw);
        gfr[(pc >> 1) * MT + (row >> 5)][(row & 31) + 32 * (pc & 1)] = v;
      }
    }
    __syncthreads();
#pragma unroll
    for (int sl = 0; sl < NSL; ++sl)
      if (sl < nsl1) rank_pass(zacc[sl], plain_order{}, sl, kc, r1, &gfr[0][0]);
    __syncthreads();                             // every wavefront is done with this X slab
  }
  publish_z(r1);
  clear_z();
  __syncthreads();

  // ================= step 2: chunks of F =================
  for (int ch = 0; ch < nch; ++ch) {
    f16v hacc[2][MT];                           // (narrow chunks use tile 0 only)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) hacc[j][mt] = zero16();
    constexpr bool narrowA = FC <= 256;
    const int fl = narrowA ? 32 * wave : 64 * wave;          // first feature of this wavefront inside the chunk
    const int f0 = FC * ch + fl;
    const int wchunk = F - FC * ch < FC ? F - FC * ch : FC;   // width of this chunk
    const int nf_on = tiles_on(fl, wchunk, narrowA);
    bool onf[NTA];
#pragma unroll
    for (int j = 0; j < NTA; ++j) onf[j] = j < nf_on;
    mm_pass(hacc, acc_order{}, narrowA, nf_on, nk1, &pfr[0][0]);
    // + b_1, activation, fp16 -> operand fragments of the second product, once no wavefront reads the previous chunk's any more
    __syncthreads();
#pragma unroll
    for (int j = 0; j < NTA; ++j)
      if (onf[j]) {
        f4v bias[4];
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
          const int f = f0 + 32 * j + 8 * jj + 4 * g;
          bias[jj] = (a.b1 && f < F) ? load4(a.b1, f, a.w_dt) : f4v{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) {
            h8 o;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
              const float x = hacc[j][mt][8 * s2 + i] + bias[2 * s2 + (i >> 2)][i & 3];
              const float y = a.act == 0 ? gelu_erf_f(x) : (a.act == 1 ? gelu_tanh_f(x) : fmaxf(x, 0.f));
              o[i] = (_Float16)y;
            }
            gfr[(fl / 16 + 2 * j + s2) * MT + mt][lane] = o;
          }
      }
    __syncthreads();
    const int kc = steps_in(F, ch);
#pragma unroll
    for (int sl = 0; sl < NSL; ++sl)
      if (sl < nsl2) rank_pass(zacc[sl], acc_order{}, sl, kc, r2, &gfr[0][0]);
  }

  // ================= step 3: out^T = V_2^T Z^T + b_2 =================
  publish_z(r2);
  __syncthreads();
  for (int ds = 0; ds < nds; ++ds) {
    f16v oacc[2][MT];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) oacc[j][mt] = zero16();
    const bool narrowD = ws.is_narrow(D - 512 * ds);
    const int n0 = 512 * ds + first_col(narrowD);
    const int nd_on = tiles_on(first_col(narrowD), D - 512 * ds, narrowD);
    mm_pass(oacc, acc_order{}, narrowD, nd_on, nk2, &pfr[0][0]);
    // + b_2, then row-major stores.  The accumulators have lane = token; each 32 x 32 block goes through a
    // wavefront-private fp32 patch in the (now idle) activation area so that a store instruction covers 128-byte row
    // segments.  Element (token t, column c) of the patch sits at 32 t + (c ^ 4 (t % 8)): both the 16-byte writes
    // (lane = token) and the 16-byte reads (lane = row part) then use every bank equally.
    float* const patch = (float*)&gfr[4 * wave][0];
#pragma unroll
    for (int j = 0; j < 2; ++j)
      if (j < nd_on) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
          for (int jj = 0; jj < 4; ++jj) {
            const int c = 8 * jj + 4 * g;
            const f4v b = a.b2 ? load4(a.b2, n0 + 32 * j + c, a.w_dt) : f4v{0.f, 0.f, 0.f, 0.f};
            f4v y;
#pragma unroll
            for (int e = 0; e < 4; ++e) y[e] = oacc[j][mt][4 * jj + e] + b[e];
            *(f4v*)&patch[32 * l32 + (c ^ (4 * (l32 & 7)))] = y;
          }
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int r = (lane >> 3) + 8 * i, c = 4 * (lane & 7);
            const f4v y = *(const f4v*)&patch[32 * r + (c ^ (4 * (r & 7)))];
            const int tok = tok0 + 32 * mt + r;
            if (tok < T) store4(a.out, (size_t)tok * D + n0 + 32 * j + c, y, a.out_dt);
          }
        }
      }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the two requests past the end have landed before the workgroup retires
}

}  // namespace

bool ffn_v2_supported(int D, int F, int r1, int r2) {
  return D % 32 == 0 && F % 16 == 0 && r1 % 16 == 0 && r2 % 16 == 0 && r1 <= 1024 && r2 <= 1024;
}

hipError_t launch_ffn_v2(const FfnV2Args& a, hipStream_t s) {
  if (!ffn_v2_supported(a.D, a.F, a.r1, a.r2) || a.T <= 0) return hipErrorInvalidValue;
  const int r = a.r1 > a.r2 ? a.r1 : a.r2;
  // 64 tokens per workgroup halve the weight traffic; they need both ranks <= 512 and enough tokens to fill the chip.
  // The LDS that the rank-space fragments do not need holds more weight steps in flight (4, 6 or 7 buffers of 16 KiB).
  const bool wide = r <= 512 && (a.T + 63) / 64 >= 200;
  const dim3 grid(wide ? (a.T + 63) / 64 : (a.T + 31) / 32), block(kV2Threads);
  const int rm = wide ? 2 * r : r;             // fragments of P1^T / Z^T in KiB = rm / 16
  if (wide) {
    if (rm <= 256) hipLaunchKernelGGL((ffn_v2_kernel<2, 7>), grid, block, 0, s, a);
    else if (rm <= 512) hipLaunchKernelGGL((ffn_v2_kernel<2, 6>), grid, block, 0, s, a);
    else if (rm <= 768) hipLaunchKernelGGL((ffn_v2_kernel<2, 5>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((ffn_v2_kernel<2, 4>), grid, block, 0, s, a);
  } else {
    if (rm <= 256) hipLaunchKernelGGL((ffn_v2_kernel<1, 7>), grid, block, 0, s, a);
    else if (rm <= 512) hipLaunchKernelGGL((ffn_v2_kernel<1, 6>), grid, block, 0, s, a);
    else if (rm <= 768) hipLaunchKernelGGL((ffn_v2_kernel<1, 5>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((ffn_v2_kernel<1, 4>), grid, block, 0, s, a);
  }
  return hipGetLastError();
}

}  // namespace fsvd
