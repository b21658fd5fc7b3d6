// Matrix-core kernel for pre-packed weights with the input block staged in LDS:
// 64 features per workgroup.
//
// In the 16-feature matrix-core kernels every workgroup pulls the whole input
// block X (Eq. 4 of arXiv 1803.11389: the T columns all rows of W are
// multiplied with) through its compute unit's vector memory path, 256 times per
// stage at d = 4096.  Here a workgroup owns 64 features; its four waves own one
// 16-feature tile each (three 16-row M tiles: candidate, forget, reset/output)
// and walk ALL k*d columns in step, so a piece of X is needed by all four at the
// same time and is fetched ONCE per workgroup, straight from memory into LDS
// (buffer loads with the LDS bit, 16 bytes per lane, no staging registers), and
// read from there as MFMA B fragments.  A wave's accumulators then hold complete sums, so
// the gates and the recurrence of Eq. 2 / Eq. 3 are applied to them in
// registers: no sum across waves, no LDS round trip and no barrier in the
// epilogue.  A stage is d/64 workgroups; the host picks this kernel when a launch
// holds enough independent stages to fill the chip.
//
// Weights: the packed layout of kernel_mfma_packed.hip.h.  A wave streams the
// fragments of its own tile, 6 KiB per k-step (128 bytes of each of its 48
// rows), non-temporal, through a register ring.
//
// 8-bit weights (E4M3 codes, widened to bf16 right before the multiply; the row
// scales multiply the finished sums).  128 bytes of a row are 128 columns, twice
// what one LDS tile of bf16 inputs holds, so the kernel's "k-step" is HALF a
// packed k-step: the three fragments (one per gate) with the packed layout's
// half index h, whose 16 bytes per lane are columns (lane/16)*32 + h*16 .. +16
// of the packed k-step, i.e. two MFMA K-slices of 8, and the eight 8-column
// chunk columns (lane/16)*4 + h*2 + {0, 1} of the input block that they multiply.
//
// Pipeline.  The unit is a "B-step": NSUB k-steps whose X columns form one LDS
// tile of at most 32 KiB; there are four LDS buffers and four ring slots of
// weight fragments.  The MFMAs of consecutive steps form one uninterrupted
// stream: every B fragment is read from LDS three fragments ahead of its use,
// across step boundaries.  In the middle of B-step s a wave waits until its own
// pieces of the X tile of step s+1 have landed and meets the other waves at a
// barrier (after it, tile s+1 is complete and every wave has long finished
// reading tile s-1), then requests its share of the X tile of step s+3 into the
// buffer that held tile s-1 and its weight fragments of step s+3 into the ring
// slot step s-1 has left.  Vector memory operations of a wave complete in issue
// order, so "all but the N youngest have completed" (s_waitcnt vmcnt(N)) names
// exactly the pieces of tile s+1: what was requested after them -- two steps of
// weight fragments and one X tile -- stays in flight across the barrier.  The
// X tiles are moved by buffer loads with the LDS bit (buffer_load_dwordx4 ... lds):
// the compiler counts those like any other load, so the waits it inserts for
// the weight fragments are exact as well.  The loop body is four B-steps (ring
// slots and LDS buffers are compile-time) and free of branches; the last four
// steps are a second instance that requests nothing past the end.
#pragma once

#include <type_traits>

#include "kernel_mfma.hip.h"

namespace ssrnn {

constexpr int XLDS_TILES = 4;                 // feature tiles (of 16) per workgroup = waves
constexpr int XLDS_F = XLDS_TILES * MFMA_F;   // features per workgroup
constexpr int XLDS_DEPTH = 3;                 // B-steps between a request and its use
constexpr int XLDS_NBUF = XLDS_DEPTH + 1;     // LDS buffers = weight ring slots (in B-steps)

// A read-only window on device memory (buffer descriptor) and the 16-bytes-per-lane load through it that
// writes LDS instead of registers: lane l's bytes land at lds + l*16, lds being the same for the whole wave.
// Requests outside the window return zeros.  The descriptor type exists in the device compilation only; the
// host compilation, which needs the kernel's signature and nothing of its body, sees an empty stand-in.
#if defined(__HIP_DEVICE_COMPILE__)
struct LdsLoadWindow { __amdgpu_buffer_rsrc_t rsrc; };
__device__ __forceinline__ LdsLoadWindow make_lds_load_window(const void* base, int bytes) {
  return LdsLoadWindow{__builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000)};
}
__device__ __forceinline__ void load_to_lds16(const LdsLoadWindow& w, char* lds, int byte_offset) {
  __builtin_amdgcn_raw_ptr_buffer_load_lds(w.rsrc, (__attribute__((address_space(3))) void*)lds, 16, byte_offset, 0, 0, 0);
}
#else
struct LdsLoadWindow {};
__device__ __forceinline__ LdsLoadWindow make_lds_load_window(const void*, int) { return LdsLoadWindow{}; }
__device__ __forceinline__ void load_to_lds16(const LdsLoadWindow&, char*, int) {}
#endif

template <int WT, int NT>
struct XldsCfg {
  static constexpr int R = NT * 16;                       // time rows of an X tile
  static_assert(R >= 16, "at least one time tile");
  static constexpr int NSUB = (R >= 256) ? 1 : 2;         // k-steps per B-step
  static constexpr int KCOLS = (WT == W_F32) ? 32 : 64;   // weight columns per k-step (fp32, bf16: 128 bytes of a row; 8-bit: 64)
  static constexpr int VEC = (WT == W_F32) ? 4 : 8;       // X elements per 16-byte chunk of the operand copy
  static constexpr int AFR = (WT == W_FP8) ? 3 : 6;       // weight fragments (1 KiB each) of a wave per k-step
  static constexpr int KSTEP_BYTES = 8 * R * 16;          // one k-step of X in LDS: 8 chunk columns x R rows x 16 B
  static constexpr int BSTEP_BYTES = NSUB * KSTEP_BYTES;
  static constexpr int NTHREADS = XLDS_TILES * 64;
  static_assert(BSTEP_BYTES % (NTHREADS * 16) == 0, "every thread moves whole 16-byte pieces");
  static constexpr int NCOPY = BSTEP_BYTES / (NTHREADS * 16);   // X pieces a thread requests per B-step
  static constexpr int PER_KSTEP = NCOPY / NSUB;                 // of which per k-step (0: one piece per thread covers both)
  static constexpr int NA = AFR * NSUB;                          // weight fragments a wave requests per B-step
  static constexpr int NFRAG = NSUB * 2 * NT;                    // B fragments (k-step, half, time tile) per B-step
  static constexpr int KSTEPS_PER_ITER = XLDS_NBUF * NSUB;       // k-steps of one loop body
};

// Columns (k*d) the kernel takes: whole loop bodies.
template <int WT, int NT>
constexpr int xlds_col_multiple() { return XldsCfg<WT, NT>::KSTEPS_PER_ITER * XldsCfg<WT, NT>::KCOLS; }

// Requirements (checked by the host): packed weights, d % 64 == 0 (8-bit: d % 128 == 0), k*d a multiple of
// xlds_col_multiple(), 1 <= nt <= NT*16, an operand copy of the input block smaller than 2 GiB, no
// split of the columns.
template <int CELL, int WT, int NT>
__global__ __launch_bounds__(XLDS_TILES * 64) void stage_mfma_xlds_kernel(const StageBatch batch, int d, int k) {
  using Cfg = XldsCfg<WT, NT>;
  constexpr int R = Cfg::R, NSUB = Cfg::NSUB, NCOPY = Cfg::NCOPY, KCOLS = Cfg::KCOLS, VEC = Cfg::VEC;
  constexpr int NFRAG = Cfg::NFRAG, NA = Cfg::NA, AFR = Cfg::AFR;
  constexpr int NBUF = XLDS_NBUF, DEPTH = XLDS_DEPTH;
  // Which (stage, feature group) this workgroup takes.  The hardware hands consecutive workgroups to the
  // eight compute dies in turn, each with an L2 of its own, and every workgroup of a stage reads that
  // stage's whole input block: with the plain order (blockIdx.y = stage) all eight L2s would fetch every
  // stage's block.  Instead die x -- the workgroups whose launch-order number is x modulo 8 -- takes the
  // x-th eighth of the (stage, group) pairs in stage-major order, so that a stage's workgroups share one or
  // two L2s and its input block leaves memory once or twice, not eight times.  Where the input block is
  // small next to the weights (bf16, up to 128 steps) the plain order measured 1 to 2 % faster and is kept
  // (d = 4096, k = 2, us per stage, plain against by die: T = 64 32.5 / 33.2, T = 128 36.6 / 37.1, T = 256
  // 55.2 / 54.2; fp32, T = 32: 33.8 / 33.5).
  constexpr bool BY_DIE = NT >= 16 || WT == W_F32;
  if (batch.in.dst && blockIdx.y == 0) { stage_input_rows(batch.in); return; }   // the launch's staging row
  int stage_no = blockIdx.y - (batch.in.dst ? 1 : 0), group_no = blockIdx.x;
  if constexpr (BY_DIE) {
    const int total = gridDim.x * batch.n;
    if (total % 8 == 0) {
      const int p = stage_no * gridDim.x + blockIdx.x;     // launch order among the stage workgroups
      const int q = (p % 8) * (total / 8) + p / 8;
      stage_no = q / gridDim.x;
      group_no = q - stage_no * gridDim.x;
    }
  }
  const Stage s = batch.s[stage_no];     // independent stages share a launch
  __shared__ __attribute__((aligned(16))) char smem[NBUF * Cfg::BSTEP_BYTES];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // a scalar: LDS addresses derived from it stay scalar
  const int li = lane & 15;
  const int kg = lane >> 4;
  const int ncol = k * d;
  const int nks = ncol / KCOLS;                      // every wave walks all k-steps
  const int nsteps = nks / NSUB;
  const int ft = group_no * XLDS_TILES + wave;       // this wave's feature tile
  const int f0 = ft * MFMA_F;

  if (CELL == CELL_QRNN && tid < XLDS_F) refresh_history(s, d, k, group_no * XLDS_F + tid);

  // ---- epilogue operands that live in memory, requested before the main loop.  In the MFMA result
  // layout lane (tl = lane % 16, fg = lane / 16) holds time step tl of a tile for features 4*fg .. 4*fg+3.
  const int fl = f0 + 4 * kg;                        // first of this lane's four features
  float4 bias0 = make_float4(0.f, 0.f, 0.f, 0.f), bias1 = bias0, bias2 = bias0;
  if (s.bias) {
    if (CELL == CELL_SRU) {
      bias1 = *reinterpret_cast<const float4*>(s.bias + fl);
      bias2 = *reinterpret_cast<const float4*>(s.bias + d + fl);
    } else {
      bias0 = *reinterpret_cast<const float4*>(s.bias + fl);
      bias1 = *reinterpret_cast<const float4*>(s.bias + d + fl);
      bias2 = *reinterpret_cast<const float4*>(s.bias + 2 * d + fl);
    }
  }
  const float4 cst = *reinterpret_cast<const float4*>(s.c + fl);      // running cell state of the four features
  float4 sc0 = make_float4(1.f, 1.f, 1.f, 1.f), sc1 = sc0, sc2 = sc0;  // 8-bit weights: the rows' scales
  if constexpr (WT == W_FP8) {
    sc0 = *reinterpret_cast<const float4*>(s.wscale + fl);
    sc1 = *reinterpret_cast<const float4*>(s.wscale + d + fl);
    sc2 = *reinterpret_cast<const float4*>(s.wscale + 2 * d + fl);
  }

  floatx4_t acc[3][NT];
#pragma unroll
  for (int g = 0; g < 3; ++g)
#pragma unroll
    for (int n = 0; n < NT; ++n) acc[g][n] = floatx4_t{0.f, 0.f, 0.f, 0.f};

  // ---- X side.  Piece e = i * 256 + tid of a B-step's tile is row e % R of chunk column e / R (chunk
  // columns 0..7 belong to the first k-step of the B-step, 8..15 to the second); the tile is stored in
  // that order, so the 64 pieces of a wave's request are 1 KiB contiguous in LDS, which is what a load
  // with the LDS bit writes (lane l at byte l*16 behind the address in M0).  Rows past the end of a
  // short block repeat its last row; the columns they produce are never read out.  The operand copy is
  // addressed through a window that starts at its first byte (row -(k-1) of chunk column 0) and ends
  // with it, so that a request outside of it could only return zeros.
  const int ldtb = s.ldt * 16;                       // bytes per chunk column of the operand copy
  const LdsLoadWindow xwin = make_lds_load_window(static_cast<const char*>(s.xop) - (k - 1) * 16, (d / VEC) * ldtb);
  int cp_off[NCOPY];                                 // byte offset of the piece behind (row 0 of) its k-step's first chunk column
#pragma unroll
  for (int i = 0; i < NCOPY; ++i) {
    const int e = i * Cfg::NTHREADS + tid;
    const int c = e / R, r = e - c * R;
    // LDS chunk column c & 7 = 2 * (K group of 16 lanes) + K-slice; with 8-bit weights a K group's 32
    // columns of the packed k-step are four chunk columns, of which a half takes two
    const int csrc = (WT == W_FP8) ? ((c & 7) >> 1) * 4 + (c & 1) : (c & 7);
    cp_off[i] = csrc * ldtb + (k - 1 + min(r, s.nt - 1)) * 16;
  }
  // cursor of the next k-step whose X columns are requested: lag block x_j, first column x_m within it
  int x_j = 0, x_m = 0;
  int xbase[NSUB];                                   // byte offset of (row 0 of) the first chunk column of each k-step of the tile on request
  auto advance_x = [&]() {                           // moves the cursor one B-step on
#pragma unroll
    for (int u = 0; u < NSUB; ++u) {
      if constexpr (WT == W_FP8) xbase[u] = ((x_m & ~127) / VEC + ((x_m >> 6) & 1) * 2) * ldtb - x_j * 16;   // packed k-step, half
      else xbase[u] = (x_m / VEC) * ldtb - x_j * 16;  // rows shifted back by the lag
      x_m += KCOLS;
      if (x_m >= d) { x_m -= d; ++x_j; }
    }
  };
  auto request_x_piece = [&](int buf, int i) {       // piece i lies in k-step (i*256 + tid) / (8*R) of the B-step
    int xb;
    if constexpr (Cfg::PER_KSTEP > 0) xb = xbase[i / Cfg::PER_KSTEP];
    else xb = (wave * 64 >= 8 * R) ? xbase[NSUB - 1] : xbase[0];      // one tile: waves 0, 1 move the first k-step, 2, 3 the second
    load_to_lds16(xwin, smem + buf * Cfg::BSTEP_BYTES + wave * 1024 + i * (Cfg::NTHREADS * 16), xb + cp_off[i]);
  };

  // ---- weight side: ring of NBUF B-steps of this wave's fragments
  const char* aptr = static_cast<const char*>(s.W) + static_cast<size_t>(ft) * nks * (AFR * 1024) + lane * 16;
  floatx4_t aring[NBUF][NSUB][AFR];
  int a_ks = 0;                                      // first k-step of the B-step whose fragments are requested
  auto request_a_piece = [&](int slot, int i) {      // fragment i % AFR of k-step i / AFR of the B-step
    const int ks = a_ks + i / AFR;
    if constexpr (WT == W_FP8)                       // gate i % 3, half ks % 2 of packed k-step ks / 2
      aring[slot][i / AFR][i % AFR] = load_stream16(aptr + static_cast<size_t>(ks >> 1) * 6144 + ((i % AFR) * 2 + (ks & 1)) * 1024);
    else
      aring[slot][i / AFR][i % AFR] = load_stream16(aptr + static_cast<size_t>(ks) * 6144 + (i % AFR) * 1024);
  };

  // ---- B fragments: fragment q of a B-step is (k-step q / 2NT, half (q / NT) % 2, time tile q % NT); lane
  // (li, kg) reads time row li of the tile from chunk column 2*kg + half.  They pass through a ring of BQ
  // register sets, BQ-1 reads ahead of the MFMAs that use them.
  constexpr int BQ = (NFRAG >= 8) ? 4 : 2;
  static_assert(NFRAG % BQ == 0 && NFRAG >= 2 * BQ, "the fragment ring repeats with the B-step");
  using bfrag_t = std::conditional_t<WT == W_F32, floatx4_t, bf16x8_t>;
  bfrag_t bq[BQ];
  const char* bt = smem + kg * 2 * (R * 16) + li * 16;
  auto read_b = [&](int buf, int q) {
    const int u = q / (2 * NT), h = (q / NT) & 1, n = q % NT;
    bq[q % BQ] = *reinterpret_cast<const bfrag_t*>(bt + buf * Cfg::BSTEP_BYTES + u * Cfg::KSTEP_BYTES + h * (R * 16) + n * 256);
  };
  bf16x8_t awide[3];                                  // 8-bit weights: the K-slice in use, widened, one per gate
  auto mfma_b = [&](int slot, int q) {
    const int u = q / (2 * NT), h = (q / NT) & 1, n = q % NT;
    if constexpr (WT == W_FP8) {
      if (n == 0) {                                   // a new K-slice: words 2h, 2h+1 of the lane's 16 codes
#pragma unroll
        for (int g = 0; g < 3; ++g) {
          const floatx4_t a4 = aring[slot][u][g];
          awide[g] = fp8x8_to_bf16(__float_as_uint(a4[h * 2]), __float_as_uint(a4[h * 2 + 1]));
        }
      }
    }
    if constexpr (WT == W_F32) {
      // four K-slices of four columns; the gates innermost, so that consecutive MFMAs write different accumulators
      const floatx4_t bv = bq[q % BQ];
#pragma unroll
      for (int e = 0; e < 4; ++e)
#pragma unroll
        for (int g = 0; g < 3; ++g)
          acc[g][n] = __builtin_amdgcn_mfma_f32_16x16x4f32(aring[slot][u][g * 2 + h][e], bv[e], acc[g][n], 0, 0, 0);
    } else {
#pragma unroll
      for (int g = 0; g < 3; ++g) {
        if constexpr (WT == W_FP8) {
          acc[g][n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(awide[g], bq[q % BQ], acc[g][n], 0, 0, 0);
        } else {
          bf16x8_t a;
          __builtin_memcpy(&a, &aring[slot][u][g * 2 + h], sizeof a);
          acc[g][n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, bq[q % BQ], acc[g][n], 0, 0, 0);
        }
      }
    }
  };

  // B-step at ring position P.  LAST: the final loop body, whose steps P >= 1 have nothing left to request
  // and whose last step has no successor.
  constexpr int QSYNC = NFRAG / 2;                   // fragment index in front of which the waves meet
  auto bstep = [&](auto last_tag, auto p_tag) {
    constexpr bool LAST = decltype(last_tag)::value;
    constexpr int P = decltype(p_tag)::value;
    constexpr bool has_next = !LAST || P < NBUF - 1;         // step s+1 exists
    constexpr bool req = !LAST || P == 0;                    // step s+DEPTH exists
    constexpr int nxt = (P + DEPTH) % NBUF;                  // buffer / slot of step s-1 = of step s+DEPTH
    // requests younger than this wave's pieces of tile s+1 at the meeting point: the weight fragments of
    // steps s+1 and s+2 and the X tile of step s+2, as far as those steps exist
    constexpr int exist2 = (!LAST || P + 2 <= NBUF - 1) ? 1 : 0;
    constexpr int younger = NA + exist2 * (NA + NCOPY);
    // the requests of step s+DEPTH (X pieces first, then weight fragments: the wait above counts on that
    // order) are spread over the fragment groups behind the meeting point, a few per group
    constexpr int NREQ = NCOPY + NA;
    constexpr int NGRP = NFRAG - QSYNC;                      // groups they are spread over
#pragma unroll
    for (int q = 0; q < NFRAG; ++q) {
      if (q == QSYNC && has_next) {
        asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(younger) : "memory");   // tile s+1 is in place, tile s-1 is free
        if constexpr (req) advance_x();
      }
      // read ahead: the last BQ-1 fragments' successors are the first fragments of the next step
      if (q + BQ - 1 < NFRAG) read_b(P, q + BQ - 1);
      else if (has_next) read_b((P + 1) % NBUF, q + BQ - 1 - NFRAG);
      if (req && q >= QSYNC) {
#pragma unroll
        for (int i = ((q - QSYNC) * NREQ) / NGRP; i < ((q - QSYNC + 1) * NREQ) / NGRP; ++i) {
          if (i < NCOPY) request_x_piece(nxt, i);
          else request_a_piece(nxt, i - NCOPY);
        }
      }
      mfma_b(P, q);
      __builtin_amdgcn_sched_barrier(0);
    }
    if constexpr (req) a_ks += NSUB;
  };
  auto body = [&](auto last_tag) {
    static_assert(NBUF == 4, "ring positions are spelled out below");
    bstep(last_tag, std::integral_constant<int, 0>{});
    bstep(last_tag, std::integral_constant<int, 1>{});
    bstep(last_tag, std::integral_constant<int, 2>{});
    bstep(last_tag, std::integral_constant<int, 3>{});
  };

  // ---- prologue: steps 0 .. DEPTH-1 requested (tile before fragments, the order of the loop), tile 0
  // landed, its first fragments on their way.  Behind the pieces of tile 0 lie the fragments of steps 0, 1, 2
  // and the tiles of steps 1, 2.
#pragma unroll
  for (int p = 0; p < DEPTH; ++p) {
    advance_x();
#pragma unroll
    for (int i = 0; i < NCOPY; ++i) request_x_piece(p, i);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < NA; ++i) request_a_piece(p, i);
    a_ks += NSUB;
    __builtin_amdgcn_sched_barrier(0);
  }
  asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(DEPTH * NA + (DEPTH - 1) * NCOPY) : "memory");
#pragma unroll
  for (int q = 0; q < BQ - 1; ++q) read_b(0, q);
  for (int s0 = 0; s0 < nsteps - NBUF; s0 += NBUF) body(std::false_type{});
  body(std::true_type{});

  // ---- epilogue in registers.  Lane (tl, fg) holds, for each time tile n, step n*16 + tl of features
  // fl .. fl+3 in all three gates, so the gate non-linearities need no exchange; the recurrence
  // c_t = f_t c_{t-1} + (1 - f_t) cand_t is a prefix scan of affine maps over the 16 lanes of a row,
  // carried from tile to tile by a broadcast of the row's last valid lane.
  const float b0[4] = {bias0.x, bias0.y, bias0.z, bias0.w};
  const float b1[4] = {bias1.x, bias1.y, bias1.z, bias1.w};
  const float b2[4] = {bias2.x, bias2.y, bias2.z, bias2.w};
  const float w0[4] = {sc0.x, sc0.y, sc0.z, sc0.w};
  const float w1[4] = {sc1.x, sc1.y, sc1.z, sc1.w};
  const float w2[4] = {sc2.x, sc2.y, sc2.z, sc2.w};
  float cin[4] = {cst.x, cst.y, cst.z, cst.w};
  const int rowbase = lane & 48;
#pragma unroll
  for (int n = 0; n < NT; ++n) {
    if (n * 16 < s.nt) {                                     // uniform over the workgroup
      const int t = n * 16 + li;
      const int tlast = min(16, s.nt - n * 16) - 1;          // last valid step of this tile
      const bool valid = li <= tlast;
      float4 xt = make_float4(0.f, 0.f, 0.f, 0.f);
      if (CELL == CELL_SRU && valid) xt = *reinterpret_cast<const float4*>(s.xcur + static_cast<long>(t) * s.ldx + fl);
      const float xv[4] = {xt.x, xt.y, xt.z, xt.w};
      float hv[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        float u0, u1, u2;
        if constexpr (WT == W_FP8) {
          u0 = fmaf(w0[r], acc[0][n][r], b0[r]); u1 = fmaf(w1[r], acc[1][n][r], b1[r]); u2 = fmaf(w2[r], acc[2][n][r], b2[r]);
        } else {
          u0 = acc[0][n][r] + b0[r]; u1 = acc[1][n][r] + b1[r]; u2 = acc[2][n][r] + b2[r];
        }
        const float f = sigmoidf_fast(u1);
        const float o = sigmoidf_fast(u2);
        const float cand = (CELL == CELL_SRU) ? u0 : tanhf_fast(u0);
        float a = f, b = (1.0f - f) * cand;
        affine_scan<16>(a, b);
        const float c = fmaf(a, cin[r], b);                  // state after step t
        hv[r] = o * tanhf_fast(c);
        if (CELL == CELL_SRU) hv[r] += (1.0f - o) * xv[r];
        cin[r] = __shfl(c, rowbase + tlast);                 // state after the tile's last valid step
      }
      if (valid) {
        *reinterpret_cast<float4*>(s.hout + static_cast<long>(t) * s.ldh + fl) = make_float4(hv[0], hv[1], hv[2], hv[3]);
        if (s.hop) {
          if (s.op_bf16) {
            uint2 pk;
            pk.x = f32_to_bf16_rne(hv[0]) | (static_cast<uint32_t>(f32_to_bf16_rne(hv[1])) << 16);
            pk.y = f32_to_bf16_rne(hv[2]) | (static_cast<uint32_t>(f32_to_bf16_rne(hv[3])) << 16);
            *reinterpret_cast<uint2*>(static_cast<char*>(s.hop) + (static_cast<long>(fl >> 3) * s.ldt + t) * 16 + (fl & 7) * 2) = pk;
          } else {
            *reinterpret_cast<float4*>(static_cast<char*>(s.hop) + (static_cast<long>(fl >> 2) * s.ldt + t) * 16) =
                make_float4(hv[0], hv[1], hv[2], hv[3]);
          }
        }
      }
    }
  }
  if (li == 0) *reinterpret_cast<float4*>(s.c + fl) = make_float4(cin[0], cin[1], cin[2], cin[3]);
}

}  // namespace ssrnn
