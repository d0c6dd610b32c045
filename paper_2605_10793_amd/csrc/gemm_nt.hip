// bf16 MFMA "NT" GEMM with fused epilogues (see gemm_nt.h).
//
// Tiling: a workgroup of WGM x WGN wavefronts owns a BM x BN tile of the output; each
// 64-lane wavefront owns (BM/WGM) x (BN/WGN) as a grid of 32x32 MFMA tiles
// (v_mfma_f32_32x32x16_bf16 / _f16, fp32 accumulators).  The large tiles run 8
// wavefronts (2 per SIMD) so that one wave's MFMAs cover the other's LDS / barrier /
// load-issue latencies.
//
// Operand path: HBM/L2 -> LDS directly (buffer_load ... lds, 16 bytes per lane, no
// register staging), 2 or 3 LDS stages of 64 K-elements (what fits in 160 KiB), fragments
// double buffered in registers, one fence-free barrier per K step placed between MFMA groups.
//
// LDS layout: a tile row is 64 bf16 = 128 bytes = 8 chunks of 16 bytes; chunk c of row r
// sits at physical chunk c ^ ((r >> 1) & 7), which spreads any 16 consecutive rows of
// one logical chunk (what a ds_read_b128 quarter-wave touches) over all 64 banks;
// measured SQ_LDS_BANK_CONFLICT = 0.
#include "gemm_nt.h"

#include <type_traits>

namespace conqur {

namespace {

constexpr int BK = 64;      // K elements per pipeline stage (one LDS tile row = 128 bytes = 8 chunks of 16 bytes)

__device__ __forceinline__ int lds_off(int row, int chunk) {
  return row * 128 + ((chunk ^ ((row >> 1) & 7)) << 4);
}

// s_waitcnt vmcnt(N) only (gfx9 encoding: vmcnt = simm16[15:14]:[3:0], expcnt and lgkmcnt left at max).
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt range");
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// Workgroup barrier without the release/acquire fence of __syncthreads(): the fence
// would drain every outstanding LDS-direct load (vmcnt(0)) and serialise the
// pipeline.  Ordering here is explicit: each wave waits (vmcnt) for its own loads of
// the tile that is consumed next, and its LDS reads of the current tile have
// returned before its last MFMA of the step could issue.  The "memory" clobber keeps
// the compiler from moving LDS accesses across the barrier.
__device__ __forceinline__ void pipeline_barrier() { asm volatile("s_barrier" ::: "memory"); }

// K-tail / invalid-row loads are pointed past the end of the buffer descriptor, where
// the hardware returns zeros (also for loads whose destination is LDS).
constexpr uint32_t kOobOffset = 0x80000000u;

template <int BM, int BN, int WGM, int WGN, int NSTAGE, int EPI, bool F16, bool SYM>
__global__ void __launch_bounds__(64 * WGM * WGN) gemm_nt_kernel(const GemmArgs g, const int tiles_m, const int tiles_n) {
  static_assert(!SYM || (BM == BN && (EPI == EPI_GRAMW || EPI == EPI_SQUARE || EPI == EPI_FRO2)),
                "mirrored tiles: square tiles, symmetric results");
  constexpr int NW = WGM * WGN;                 // wavefronts per workgroup
  constexpr int WM = BM / WGM, WN = BN / WGN, TM = WM / 32, TN = WN / 32;
  constexpr int NLA = BM / 8, NLB = BN / 8;     // wave-wide 1 KiB loads per stage (8 tile rows each)
  constexpr int QA = NLA / NW, QB = NLB / NW;   // ... per wavefront
  static_assert(NLA % NW == 0 && NLB % NW == 0 && WM % 32 == 0 && WN % 32 == 0, "tile shape");
  constexpr int STAGE = (BM + BN) * 128;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  // Optional clock probe (g.clk != null): wall-clock ticks (100 MHz) of the prologue, main loop and epilogue
  // of this workgroup and the shader-clock cycles of the main loop, from which the host derives the clock
  // frequency the chip sustained while the MFMAs ran.
  const unsigned long long pr_w0 = g.clk ? wall_clock64() : 0;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WGN, wn = wave % WGN;
  const int half = lane >> 5, col = lane & 31;

  // Workgroups are dealt round-robin to the 8 XCDs (bid % 8), each with its own L2, and
  // an XCD runs 32 of them at a time.  Map the 32 workgroups that are co-resident on an
  // XCD to a compact 4 x 8 block of output tiles, so that per K step the XCD pulls
  // (4 + 8) operand panels through its L2 instead of up to (32 + 1).
  int bid = blockIdx.x;
  const int ntiles = tiles_m * tiles_n;
  int tm, tn;
  if constexpr (SYM) {
    // Tiles on and above the diagonal only: tile rows r and T-1-r together hold T+1 of them, and such a pair of rows
    // needs few operand panels (2 of A, T-r of B).  With T a multiple of 16 every XCD (bid % 8) gets whole pairs.
    const int T = tiles_m;
    int pair, within;
    if ((T & 15) == 0) {
      const int xcd = bid & 7, local = bid >> 3;
      pair = xcd + 8 * (local / (T + 1));
      within = local % (T + 1);
    } else {
      pair = bid / (T + 1);
      within = bid % (T + 1);
    }
    if (within < T - pair) { tm = pair; tn = pair + within; }
    else { tm = T - 1 - pair; tn = tm + (within - (T - pair)); }
  } else if ((tiles_m & 3) == 0 && (tiles_n & 7) == 0 && (((tiles_m >> 2) * (tiles_n >> 3)) & 7) == 0) {
    const int xcd = bid & 7, local = bid >> 3;
    const int group = (local >> 5) * 8 + xcd, within = local & 31;
    const int gm = tiles_m >> 2;
    tm = (group % gm) * 4 + (within & 3);
    tn = (group / gm) * 8 + (within >> 2);
  } else {
    if ((ntiles & 7) == 0) bid = (bid & 7) * (ntiles >> 3) + (bid >> 3);
    tm = bid % tiles_m;
    tn = bid / tiles_m;
  }
  const int m0 = tm * BM, n0 = tn * BN;
  const int bz = blockIdx.z;
  const bf16_bits* Ab = g.A + (int64_t)bz * g.batchA;
  const bf16_bits* Bb = g.B + (int64_t)bz * g.batchB;

  // Global -> LDS without passing through registers: each buffer_load ... lds moves
  // 64 lanes x 16 bytes = 8 tile rows into 1 KiB of LDS (lane L lands at L*16).
  // Lane L therefore fetches the chunk that the swizzled layout stores at row L/8,
  // physical chunk L%8.  Rows past M (N) lie past the descriptor's range and read 0.
  const int lrow = lane >> 3, lpc = lane & 7;
  uint32_t offA[QA], offB[QB];
  int chunkA[QA], chunkB[QB];
#pragma unroll
  for (int q = 0; q < QA; ++q) {
    const int row = (q * NW + wave) * 8 + lrow;
    chunkA[q] = lpc ^ ((row >> 1) & 7);
    offA[q] = (m0 + row < g.M) ? (uint32_t)(((int64_t)(m0 + row) * g.lda + chunkA[q] * 8) * 2) : kOobOffset;
  }
#pragma unroll
  for (int q = 0; q < QB; ++q) {
    const int row = (q * NW + wave) * 8 + lrow;
    chunkB[q] = lpc ^ ((row >> 1) & 7);
    offB[q] = (n0 + row < g.N) ? (uint32_t)(((int64_t)(n0 + row) * g.ldb + chunkB[q] * 8) * 2) : kOobOffset;
  }
  const uint32_t recA = (uint32_t)((((int64_t)g.M - 1) * g.lda + BK) * 2);
  const uint32_t recB = (uint32_t)((((int64_t)g.N - 1) * g.ldb + BK) * 2);
  const int nkb = (g.K + BK - 1) / BK;
  const int nit = nkb * g.nseg;
  const bool ktail = (g.K % BK) != 0;
  // offsets for the last, partial K step of a segment: chunks past K read zeros
  uint32_t offAt[QA], offBt[QB];
  {
    const int kleft = g.K - (nkb - 1) * BK;
#pragma unroll
    for (int q = 0; q < QA; ++q) offAt[q] = (chunkA[q] * 8 < kleft) ? offA[q] : kOobOffset;
#pragma unroll
    for (int q = 0; q < QB; ++q) offBt[q] = (chunkB[q] * 8 < kleft) ? offB[q] : kOobOffset;
  }

  // Issue state: the next tile to fetch is K step is_kb of segment is_s; its operand
  // pointers advance incrementally (wave-uniform, scalar registers).
  int is_s = 0, is_kb = 0;
  const bf16_bits* pa = Ab + g.a_seg[0];
  const bf16_bits* pb = Bb + g.b_seg[0];
  __amdgpu_buffer_rsrc_t ra, rb;
  bool tail = false;
  auto issue_prep = [&]() {
    // Past the last tile the pipeline keeps issuing (so that every step has the same
    // number of loads in flight and needs no branches); those loads get an empty
    // descriptor range, fetch nothing and write zeros to a stage nobody reads again.
    const bool real = is_s < g.nseg;
    ra = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_bits*>(pa), 0, real ? recA : 0u, 0x00020000);
    rb = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_bits*>(pb), 0, real ? recB : 0u, 0x00020000);
    tail = ktail && is_kb == nkb - 1;
    if (++is_kb == nkb) {
      is_kb = 0;
      ++is_s;
      const int sc = is_s < g.nseg ? is_s : g.nseg - 1;
      pa = Ab + g.a_seg[sc];
      pb = Bb + g.b_seg[sc];
    } else {
      pa += BK; pb += BK;
    }
  };
  auto issue_one = [&](int q, int stage) {   // load q of LPT of the prepared tile
    unsigned char* sa = smem + stage * STAGE;
    if (q < QA) {
      const uint32_t off = tail ? offAt[q] : offA[q];
      __builtin_amdgcn_raw_ptr_buffer_load_lds(ra, (__attribute__((address_space(3))) void*)(sa + (q * NW + wave) * 1024), 16,
                                               off, 0, 0, 0);
    } else {
      const int qb = q - QA;
      const uint32_t off = tail ? offBt[qb] : offB[qb];
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rb, (__attribute__((address_space(3))) void*)(sa + BM * 128 + (qb * NW + wave) * 1024),
                                               16, off, 0, 0, 0);
    }
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

  // Software pipeline.  LDS holds NSTAGE tiles; tile t lives in stage t % NSTAGE.
  // Operand fragments are double buffered in registers: while the MFMAs of K-substep
  // kk run, the fragments of substep kk+1 are read from LDS (one ds_read per MFMA, so
  // the reads issue in the MFMA's shadow).  The step's only synchronisation sits in the
  // middle of its last substep: wait for this wave's loads of the next tile (vmcnt
  // counts outstanding loads, which retire in order), barrier (now every wave's part of
  // the next tile is visible and every wave has finished reading the current stage),
  // refill the current stage with tile it+NSTAGE, read the first fragments of the next
  // tile, and cover that latency with the second half of the substep's MFMAs.
  constexpr int LPT = QA + QB;   // loads per thread per tile
  constexpr int KS = BK / 16;    // MFMA K-substeps per tile
  constexpr int NMF = TM * TN;
  constexpr int LQ0 = NMF - NMF / 2;   // loads issued behind the second half of a step's last substep; the rest of the
                                       // tile's loads follow behind the first MFMAs of the next step
  static_assert(KS % 2 == 0, "fragment double buffering assumes an even number of substeps");
  bf16x8 fa[2][TM], fb[2][TN];

  auto read_frag = [&](int buf, int r, const unsigned char* sa, int kk) {
    // read number r of a substep, in the order the MFMAs need them: a0, b0..b(TN-1), a1..a(TM-1)
    const unsigned char* sb = sa + BM * 128;
    if (r == 0) fa[buf][0] = *reinterpret_cast<const bf16x8*>(sa + lds_off(wm * WM + col, kk * 2 + half));
    else if (r <= TN) fb[buf][r - 1] = *reinterpret_cast<const bf16x8*>(sb + lds_off(wn * WN + (r - 1) * 32 + col, kk * 2 + half));
    else fa[buf][r - TN] = *reinterpret_cast<const bf16x8*>(sa + lds_off(wm * WM + (r - TN) * 32 + col, kk * 2 + half));
  };
  auto mfma = [&](int buf, int m) {
    const int i = m / TN, j = m % TN;
    if constexpr (F16)
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, fa[buf][i]), __builtin_bit_cast(f16x8, fb[buf][j]),
                                                         acc[i][j], 0, 0, 0);
    else
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[buf][i], fb[buf][j], acc[i][j], 0, 0, 0);
  };

#pragma unroll
  for (int p = 0; p < NSTAGE; ++p) {
    issue_prep();
#pragma unroll
    for (int q = 0; q < LPT; ++q) issue_one(q, p);
  }
  wait_vmcnt<(NSTAGE - 1) * LPT>();   // tile 0 has landed
  pipeline_barrier();
#pragma unroll
  for (int r = 0; r < TM + TN; ++r) read_frag(0, r, smem, 0);

  const unsigned long long pr_w1 = g.clk ? wall_clock64() : 0, pr_c1 = g.clk ? clock64() : 0;
  int stage = 0;   // it % NSTAGE
  for (int it = 0; it < nit; ++it) {
    const int prev_stage = stage == 0 ? NSTAGE - 1 : stage - 1, next_stage = stage == NSTAGE - 1 ? 0 : stage + 1;
    const unsigned char* sa = smem + stage * STAGE;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
      const int cur = kk & 1, nxt = cur ^ 1;
      if (kk + 1 < KS) {
#pragma unroll
        for (int m = 0; m < NMF; ++m) {
          mfma(cur, m);
          if (m < TM + TN) read_frag(nxt, m, sa, kk + 1);
          // the loads of tile it-1+NSTAGE that did not fit behind the previous step's last MFMAs
          if (kk == 0 && it > 0 && LQ0 + m < LPT) issue_one(LQ0 + m, prev_stage);
          __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int r = NMF; r < TM + TN; ++r) read_frag(nxt, r, sa, kk + 1);
      } else {
        issue_prep();   // tile it+NSTAGE refills the stage being consumed; scalar work, hidden behind the MFMAs
#pragma unroll
        for (int m = 0; m < NMF / 2; ++m) mfma(cur, m);
        __builtin_amdgcn_sched_barrier(0);
        // tiles up to it+NSTAGE-1 have been issued; all but the newest NSTAGE-2 have landed => tile it+1 is in LDS
        wait_vmcnt<(NSTAGE - 2) * LPT>();
        pipeline_barrier();
        const unsigned char* sn = smem + next_stage * STAGE;
#pragma unroll
        for (int r = 0; r < TM + TN; ++r) read_frag(nxt, r, sn, 0);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int m = NMF / 2; m < NMF; ++m) {
          mfma(cur, m);
          if (m - NMF / 2 < LPT) issue_one(m - NMF / 2, stage);
          __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int q = LQ0 + NMF; q < LPT; ++q) issue_one(q, stage);   // (none for the tile shapes in use)
      }
    }
    stage = next_stage;
  }
  const unsigned long long pr_w2 = g.clk ? wall_clock64() : 0, pr_c2 = g.clk ? clock64() : 0;
  wait_vmcnt<0>();   // drain the padding loads before the epilogue reuses nothing of LDS (keeps exit clean)

  // Accumulator element e = 4*j + i of tile (im, in) is output row
  //   m = m0 + wm*WM + im*32 + 8*j + 4*half + i,   column n = n0 + wn*WN + in*32 + col.
  const int mw = m0 + wm * WM, nw = n0 + wn * WN;

  // Addressing of the epilogues that write matrices [row][ldc]: buffer instructions with 32-bit byte offsets, so that
  // a store is one instruction (no 64-bit address arithmetic per element) and bounds need no branches.  An offset at
  // or beyond the range of its array (rows past the last one; kOobOffset for lanes whose column, or whose rows in the
  // transposed layout, do not exist) makes a store a no-op and a load return zero.  With the per-element pointer
  // arithmetic and branches these epilogues ran 4000-5000 instructions per wavefront for 128 values per lane, and
  // instruction issue, not memory, was what they waited for.
  //   natural layout     [m][n]: byte offset nat{2,4}[j] + row_off(rows below the lane's first) * element size
  //   transposed layout  [n][m]: byte offset tr_off(j, rows below the lane's first), 4 consecutive m = 8 bytes
  [[maybe_unused]] const uint32_t ldc_u = (uint32_t)g.ldc;
  [[maybe_unused]] const uint32_t nat_rows = (uint32_t)g.M * ldc_u, tr_rows = (uint32_t)g.N * ldc_u;   // elements
  [[maybe_unused]] const int mlim = g.M - (mw + 4 * half);   // rows ml .. ml + 3 of this lane exist iff ml < mlim
  [[maybe_unused]] bool n_ok[TN];
  [[maybe_unused]] uint32_t nat2[TN], nat4[TN], tr2[TN];
  {
    const uint32_t lane_nat = (uint32_t)(mw + 4 * half) * ldc_u + (uint32_t)(nw + col);
    const uint32_t lane_tr = (uint32_t)(nw + col) * ldc_u + (uint32_t)(mw + 4 * half);
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      n_ok[j] = nw + 32 * j + col < g.N;
      nat2[j] = n_ok[j] ? (lane_nat + 32u * j) * 2u : kOobOffset;
      nat4[j] = n_ok[j] ? (lane_nat + 32u * j) * 4u : kOobOffset;
      tr2[j] = (lane_tr + 32u * j * ldc_u) * 2u;   // columns n >= N are rows past the end of the transposed array
    }
  }
  [[maybe_unused]] auto row_off = [&](int ml) { return (uint32_t)ml * ldc_u; };
  [[maybe_unused]] auto tr_off = [&](int j, int ml) { return ml < mlim ? tr2[j] + 2u * (uint32_t)ml : kOobOffset; };
  [[maybe_unused]] auto out_rsrc = [](void* p, uint32_t bytes) { return __builtin_amdgcn_make_buffer_rsrc(p, 0, (int)bytes, 0x00020000); };
  [[maybe_unused]] auto in_rsrc = [](const void* p, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
  };
  [[maybe_unused]] auto ld32 = [](__amdgpu_buffer_rsrc_t r, uint32_t off) {
    return __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r, off, 0, 0));
  };
  [[maybe_unused]] auto ld16 = [](__amdgpu_buffer_rsrc_t r, uint32_t off) {
    return (bf16_bits)__builtin_amdgcn_raw_buffer_load_b16(r, off, 0, 0);
  };
  [[maybe_unused]] auto st32 = [](__amdgpu_buffer_rsrc_t r, uint32_t off, float v) {
    __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), r, off, 0, 0);
  };
  [[maybe_unused]] auto st64 = [](__amdgpu_buffer_rsrc_t r, uint32_t off, const uint2& t) {
    typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
    const u32x2 v = {t.x, t.y};
    __builtin_amdgcn_raw_buffer_store_b64(v, r, off, 0, 0);
  };
  // the 4 packed 16-bit values of t to rows 0 .. 3 below byte offset off of a natural-layout plane
  [[maybe_unused]] auto st_rows4 = [&](__amdgpu_buffer_rsrc_t r, uint32_t off, const uint2& t) {
    const uint32_t rb = 2u * ldc_u;
    __builtin_amdgcn_raw_buffer_store_b16((unsigned short)t.x, r, off, 0, 0);
    __builtin_amdgcn_raw_buffer_store_b16((unsigned short)(t.x >> 16), r, off + rb, 0, 0);
    __builtin_amdgcn_raw_buffer_store_b16((unsigned short)t.y, r, off + 2u * rb, 0, 0);
    __builtin_amdgcn_raw_buffer_store_b16((unsigned short)(t.y >> 16), r, off + 3u * rb, 0, 0);
  };
  // The accumulators as activations Y[m][n] (bf16 or fp32 by g.c_is_f32), row pitch `pitch`: the pitch is the caller's,
  // so the offsets are taken relative to the tile's first row (at most BM rows x pitch x 4 bytes, which the launcher
  // keeps below 2^31); rows past M lie beyond the range, columns past N are masked.
  [[maybe_unused]] auto store_act = [&](void* base, int64_t pitch, int64_t batch_off) {
    const uint32_t pu = (uint32_t)pitch;
    const uint32_t rows = (uint32_t)(g.M - m0 < BM ? g.M - m0 : BM);
    const uint32_t lane_el = (uint32_t)(wm * WM + 4 * half) * pu + (uint32_t)(nw + col);
    const int64_t tile_el = (int64_t)bz * batch_off + (int64_t)m0 * pitch;
    if (g.c_is_f32) {
      const auto r = out_rsrc(reinterpret_cast<float*>(base) + tile_el, rows * pu * 4u);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          const uint32_t o = n_ok[j] ? (lane_el + 32u * j) * 4u : kOobOffset;
#pragma unroll
          for (int e = 0; e < 16; ++e) st32(r, o + (uint32_t)(32 * i + 8 * (e >> 2) + (e & 3)) * pu * 4u, acc[i][j][e]);
        }
    } else {
      const auto r = out_rsrc(reinterpret_cast<bf16_bits*>(base) + tile_el, rows * pu * 2u);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          const uint32_t o = n_ok[j] ? (lane_el + 32u * j) * 2u : kOobOffset;
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            uint2 t;
            t.x = f32x2_to_bf16x2(acc[i][j][4 * q], acc[i][j][4 * q + 1]);
            t.y = f32x2_to_bf16x2(acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
            const uint32_t oq = o + (uint32_t)(32 * i + 8 * q) * pu * 2u, rb = 2u * pu;
            __builtin_amdgcn_raw_buffer_store_b16((unsigned short)t.x, r, oq, 0, 0);
            __builtin_amdgcn_raw_buffer_store_b16((unsigned short)(t.x >> 16), r, oq + rb, 0, 0);
            __builtin_amdgcn_raw_buffer_store_b16((unsigned short)t.y, r, oq + 2u * rb, 0, 0);
            __builtin_amdgcn_raw_buffer_store_b16((unsigned short)(t.y >> 16), r, oq + 3u * rb, 0, 0);
          }
        }
    }
  };

  if constexpr (EPI == EPI_SIGN_ACT) {   // the rotated rows themselves, as EPI_ACT writes them
    store_act(g.Yact, g.ldy, g.batchY);
  }
  if constexpr (EPI == EPI_SIGN || EPI == EPI_SIGN_ACT || EPI == EPI_SIGN_XT) {
    // St is the transpose of the accumulator tile.  Storing it straight from the registers gives every lane 8 bytes of
    // a different row (64 cache lines per store instruction); instead each wavefront transposes its WM x WN block
    // through its own slice of the (now idle) stage memory and stores whole 16-byte chunks, 8 or 16 lanes per row.
    bf16_bits* St = reinterpret_cast<bf16_bits*>(g.C) + (int64_t)bz * g.batchC;
    const uint32_t one = g.sign_f16 ? 0x3C00u : 0x3F80u;
    constexpr int SROW = WM * 2;                      // bytes per staged row (one output column n, WM tokens)
    constexpr int CPR = WM / 8;                       // 16-byte chunks per staged row, XOR swizzled by the row
    static_assert(NW * WN * SROW <= NSTAGE * STAGE && (CPR & (CPR - 1)) == 0, "sign staging fits the stage memory");
    unsigned char* stg = smem + wave * (WN * SROW);
    // EPI_SIGN_XT: the block of A this wavefront transposes below, loaded now so that the sign staging covers the latency
    constexpr int XT_ITEMS = EPI == EPI_SIGN_XT ? (WM / 2) * (WN / 8) / 64 : 1;
    [[maybe_unused]] uint4 xt_a[XT_ITEMS], xt_b[XT_ITEMS];
    [[maybe_unused]] float xt_w0[XT_ITEMS], xt_w1[XT_ITEMS];
    if constexpr (EPI == EPI_SIGN_XT) {
      constexpr int CH = WN / 8;
      const bf16_bits* Xb = Ab + g.a_seg[0];
      const float* wrow = g.xt_w + (int64_t)bz * g.xt_ldw;
#pragma unroll
      for (int q = 0; q < XT_ITEMS; ++q) {
        const int item = q * 64 + lane, c = item % CH, p = item / CH;
        const int m = mw + 2 * p, k = nw + 8 * c;
        xt_a[q] = make_uint4(0u, 0u, 0u, 0u); xt_b[q] = xt_a[q];
        xt_w0[q] = 0.0f; xt_w1[q] = 0.0f;
        if (k < g.N) {
          if (m < g.M) { xt_a[q] = *reinterpret_cast<const uint4*>(Xb + (int64_t)m * g.lda + k); xt_w0[q] = wrow[m]; }
          if (m + 1 < g.M) { xt_b[q] = *reinterpret_cast<const uint4*>(Xb + (int64_t)(m + 1) * g.lda + k); xt_w1[q] = wrow[m + 1]; }
        }
      }
    }
    __syncthreads();                                  // every wavefront has finished reading operand tiles
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const f32x16& a = acc[i][j];
          uint2 v;  // +1 with the sign bit of each accumulator (sgn(+-0) = +1, so test >= 0)
          v.x = (a[4 * q + 0] >= 0.0f ? one : one | 0x8000u) | ((a[4 * q + 1] >= 0.0f ? one : one | 0x8000u) << 16);
          v.y = (a[4 * q + 2] >= 0.0f ? one : one | 0x8000u) | ((a[4 * q + 3] >= 0.0f ? one : one | 0x8000u) << 16);
          const int r = j * 32 + col, c = i * 4 + q;   // tokens 8 c + 4 half .. + 3 of row r
          *reinterpret_cast<uint2*>(stg + r * SROW + ((c ^ (r & (CPR - 1))) << 4) + 8 * half) = v;
        }
    // the slice is private to the wavefront: its own LDS writes are visible to it after the wait the compiler inserts
#pragma unroll
    for (int it2 = 0; it2 < WN * CPR / 64; ++it2) {
      const int idx = it2 * 64 + lane, r = idx / CPR, c = idx % CPR;
      const int n = nw + r, m = mw + c * 8;
      const uint4 v = *reinterpret_cast<const uint4*>(stg + r * SROW + ((c ^ (r & (CPR - 1))) << 4));
      if (n < g.N && m < g.st_rows_valid) *reinterpret_cast<uint4*>(St + (int64_t)n * g.ldc + m) = v;
    }
    if constexpr (EPI == EPI_SIGN_XT) {
      // The scaled, transposed fp16 copy of A's block under this wavefront's output block: tokens [mw, mw + WM) x
      // channels [nw, nw + WN).  A lane takes items (token pair p, 16-byte chunk c of 8 channels), chunk fastest so
      // that 8 lanes read 128 contiguous bytes of a row; the pair's two values of a channel go to the staging slice as
      // one 4-byte write (row = channel, position = token pair); 16-byte chunks of 8 tokens come back and are stored
      // like the signs.  The slice is this wavefront's own and LDS operations of one wavefront complete in order, so
      // no barrier separates this from the sign staging above.
      constexpr int PAIRS = WM / 2, CH = WN / 8;
      static_assert((PAIRS * CH) % 64 == 0, "whole wavefronts of items");
      const float* wrow = g.xt_w + (int64_t)bz * g.xt_ldw;
      bf16_bits* Xt = g.Xt + (int64_t)bz * g.batchC;
      auto phys = [](int r, int cc) { return cc ^ ((r ^ (r >> 3)) & (CPR - 1)); };
#pragma unroll
      for (int q = 0; q < PAIRS * CH / 64; ++q) {
        const int item = q * 64 + lane, c = item % CH, p = item / CH;
        const uint4 xa = xt_a[q], xb = xt_b[q];
        const float w0 = xt_w0[q], w1 = xt_w1[q];
        const uint32_t ua[4] = {xa.x, xa.y, xa.z, xa.w}, ub[4] = {xb.x, xb.y, xb.z, xb.w};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const uint32_t ba = (e & 1) ? (ua[e >> 1] & 0xffff0000u) : (ua[e >> 1] << 16);
          const uint32_t bb = (e & 1) ? (ub[e >> 1] & 0xffff0000u) : (ub[e >> 1] << 16);
          // a skipped row has w = 0 and possibly Inf / NaN values: select, do not multiply
          const float fa = w0 != 0.0f ? __uint_as_float(ba) * w0 : 0.0f;
          const float fb = w1 != 0.0f ? __uint_as_float(bb) * w1 : 0.0f;
          const int r = c * 8 + e;
          *reinterpret_cast<uint32_t*>(stg + r * SROW + (phys(r, p >> 2) << 4) + (p & 3) * 4) = f32x2_to_f16x2(fa, fb);
        }
      }
#pragma unroll
      for (int it2 = 0; it2 < WN * CPR / 64; ++it2) {
        const int idx = it2 * 64 + lane, r = idx / CPR, cc = idx % CPR;
        const int n = nw + r, m = mw + cc * 8;
        const uint4 v = *reinterpret_cast<const uint4*>(stg + r * SROW + (phys(r, cc) << 4));
        if (n < g.N && m < g.st_rows_valid) *reinterpret_cast<uint4*>(Xt + (int64_t)n * g.ldc + m) = v;
      }
      if (tn == 0 && wn == 0) {   // one wavefront per 64 tokens of the tile row counts them
#pragma unroll
        for (int t0 = 0; t0 < WM; t0 += 64) {
          const int m = mw + t0 + lane;
          const bool in_block = t0 + lane < WM && m < g.M;
          const float wv = in_block ? wrow[m] : 0.0f;
          const unsigned long long in = __ballot(in_block && wv != 0.0f), out = __ballot(in_block && wv == 0.0f);
          if (lane == 0) {
            unsigned long long* slot = g.cnt + ((int64_t)bz * g.cnt_slots + (tm % g.cnt_slots)) * 2;
            if (in) atomicAdd(slot, (unsigned long long)__popcll(in));
            if (out) atomicAdd(slot + 1, (unsigned long long)__popcll(out));
          }
        }
      }
    }
  } else if constexpr (EPI == EPI_ACT) {
    store_act(g.C, g.ldc, g.batchC);
  } else if constexpr (EPI == EPI_F32) {
    const auto rC = out_rsrc(reinterpret_cast<float*>(g.C) + (int64_t)bz * g.batchC, nat_rows * 4u);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        float v[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) v[e] = g.out_scale * acc[i][j][e];
        if (g.accumulate) {
#pragma unroll
          for (int e = 0; e < 16; ++e) v[e] += ld32(rC, nat4[j] + row_off(32 * i + 8 * (e >> 2) + (e & 3)) * 4u);
        }
#pragma unroll
        for (int e = 0; e < 16; ++e) st32(rC, nat4[j] + row_off(32 * i + 8 * (e >> 2) + (e & 3)) * 4u, v[e]);
      }
  } else if constexpr (EPI == EPI_GRAMW) {
    const int64_t boff = (int64_t)bz * g.batchC;
    [[maybe_unused]] const bool mirror = SYM && tm != tn;   // this tile is also the transpose of tile (tn, tm)
    double rsum = 0.0;
    // Only a workgroup whose tile meets the diagonal has entries of the identity to add and subtract: the others run
    // the version of the code without them (a wave-uniform choice).
    auto tiles = [&](auto on_diagonal) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          float part = 0.0f;
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int ml = 32 * i + 8 * q;            // rows ml .. ml + 3 of this lane's block (M is a multiple of 4)
            float w[4], part_q = 0.0f;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              const float a = acc[i][j][4 * q + r];
              if constexpr (decltype(on_diagonal)::value) {
                const float eye = (mw + 4 * half + ml + r == nw + 32 * j + col) ? 1.0f : 0.0f;
                const float d = a - eye;
                part_q += d * d;
                w[r] = g.coef_i * eye + g.coef_g * a;
              } else {
                part_q += a * a;
                w[r] = g.coef_g * a;
              }
            }
            part += (n_ok[j] && ml < mlim) ? part_q : 0.0f;
            if constexpr (!F16) {   // (fp16 operands: no planes to add)
              for (int p = 0; p < g.np_add; ++p) {
                const auto rA = in_rsrc(g.Padd + p * g.plane_out + boff, nat_rows * 2u);
#pragma unroll
                for (int r = 0; r < 4; ++r) w[r] += bf16_to_f32(ld16(rA, nat2[j] + row_off(ml + r) * 2u));
              }
            }
            for (int p = 0; p < (F16 ? 1 : g.np_out); ++p) {
              uint2 t;
              if constexpr (F16) {   // fp16 operands: the factor is one fp16 plane
                t.x = f32x2_to_f16x2(w[0], w[1]);
                t.y = f32x2_to_f16x2(w[2], w[3]);
              } else {
                t.x = f32x2_to_bf16x2(w[0], w[1]);
                t.y = f32x2_to_bf16x2(w[2], w[3]);
                w[0] -= __uint_as_float(t.x << 16); w[1] -= __uint_as_float(t.x & 0xffff0000u);
                w[2] -= __uint_as_float(t.y << 16); w[3] -= __uint_as_float(t.y & 0xffff0000u);
              }
              const auto rP = out_rsrc(g.Pn + p * g.plane_out + boff, nat_rows * 2u);
              st_rows4(rP, nat2[j] + row_off(ml) * 2u, t);
              if constexpr (SYM) {
                if (mirror) st64(rP, tr_off(j, ml), t);
              }
            }
          }
          rsum += (double)part;
        }
    };
    if (m0 < n0 + BN && n0 < m0 + BM) tiles(std::true_type{});
    else tiles(std::false_type{});
    if (g.resid_part) {
      rsum = wave_sum_d(rsum);
      if (lane == 0) {
        g.resid_part[((int64_t)bz * ntiles + tn * tiles_m + tm) * NW + wave] = rsum;
        if constexpr (SYM) {   // the mirrored tile's slot: the sum over all slots stays the sum over the whole matrix
          if (mirror) g.resid_part[((int64_t)bz * ntiles + tm * tiles_m + tn) * NW + wave] = rsum;
        }
      }
    }
  } else if constexpr (EPI == EPI_SQUARE) {
    const int64_t boff = (int64_t)bz * g.batchC;
    [[maybe_unused]] const bool mirror = SYM && tm != tn;
    const auto rA0 = in_rsrc(g.Padd + boff, nat_rows * 2u), rA1 = in_rsrc(g.Padd + g.plane_out + boff, nat_rows * 2u);
    const auto rSq = out_rsrc(g.Pacc + boff, nat_rows * 2u);
    const auto rW0 = out_rsrc(g.Pn + boff, nat_rows * 2u), rW1 = out_rsrc(g.Pn + g.plane_out + boff, nat_rows * 2u);
    double rsum = 0.0;   // sum of the squares of this wavefront's accumulators: ||D^2||_F^2 over the whole launch
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        float part = 0.0f;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int ml = 32 * i + 8 * q;
          const bool in = n_ok[j] && ml < mlim;
          float a[4], w[4];
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const uint32_t off = nat2[j] + row_off(ml + r) * 2u;
            a[r] = acc[i][j][4 * q + r];
            part += in ? a[r] * a[r] : 0.0f;
            w[r] = g.coef_g * a[r] + bf16_to_f32(ld16(rA0, off)) + bf16_to_f32(ld16(rA1, off));
          }
          uint2 ta, t0, t1;
          ta.x = f32x2_to_bf16x2(a[0], a[1]);
          ta.y = f32x2_to_bf16x2(a[2], a[3]);
          t0.x = f32x2_to_bf16x2(w[0], w[1]);
          t0.y = f32x2_to_bf16x2(w[2], w[3]);
          t1.x = f32x2_to_bf16x2(w[0] - __uint_as_float(t0.x << 16), w[1] - __uint_as_float(t0.x & 0xffff0000u));
          t1.y = f32x2_to_bf16x2(w[2] - __uint_as_float(t0.y << 16), w[3] - __uint_as_float(t0.y & 0xffff0000u));
          const uint32_t off = nat2[j] + row_off(ml) * 2u;
          st_rows4(rSq, off, ta);
          st_rows4(rW0, off, t0);
          st_rows4(rW1, off, t1);
          if constexpr (SYM) {
            if (mirror) {
              const uint32_t offt = tr_off(j, ml);
              st64(rSq, offt, ta);
              st64(rW0, offt, t0);
              st64(rW1, offt, t1);
            }
          }
        }
        rsum += (double)part;
      }
    if (g.resid_part) {
      rsum = wave_sum_d(rsum);
      if (lane == 0) {
        g.resid_part[((int64_t)bz * ntiles + tn * tiles_m + tm) * NW + wave] = rsum;
        if constexpr (SYM) {   // a tile above the diagonal stands for its mirror image as well
          if (mirror) g.resid_part[((int64_t)bz * ntiles + tm * tiles_m + tn) * NW + wave] = rsum;
        }
      }
    }
  } else if constexpr (EPI == EPI_FRO2) {
    double rsum = 0.0;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        float part = 0.0f;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const bool in = n_ok[j] && 32 * i + 8 * (e >> 2) + (e & 3) < mlim;
          part += in ? acc[i][j][e] * acc[i][j][e] : 0.0f;
        }
        rsum += (double)part;
      }
    rsum = wave_sum_d(rsum);
    if (lane == 0) {
      g.resid_part[((int64_t)bz * ntiles + tn * tiles_m + tm) * NW + wave] = rsum;
      if constexpr (SYM) {   // a tile above the diagonal stands for its mirror image as well
        if (tm != tn) g.resid_part[((int64_t)bz * ntiles + tm * tiles_m + tn) * NW + wave] = rsum;
      }
    }
  } else if constexpr (EPI == EPI_XLAST) {
    const int64_t boff = (int64_t)bz * g.batchC;
    const bool two = g.np_out == 2;
    const auto rC = out_rsrc(g.C32 + boff, nat_rows * 4u);
    const auto rN0 = out_rsrc(g.Pn + boff, nat_rows * 2u), rN1 = out_rsrc(g.Pn + g.plane_out + boff, two ? nat_rows * 2u : 0u);
    const auto rT0 = out_rsrc(g.Pt + boff, tr_rows * 2u), rT1 = out_rsrc(g.Pt + g.plane_out + boff, two ? tr_rows * 2u : 0u);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int ml = 32 * i + 8 * q;
          const float v0 = acc[i][j][4 * q], v1 = acc[i][j][4 * q + 1], v2 = acc[i][j][4 * q + 2], v3 = acc[i][j][4 * q + 3];
          uint2 hi;
          hi.x = f32x2_to_bf16x2(v0, v1);
          hi.y = f32x2_to_bf16x2(v2, v3);
          float h0 = __uint_as_float(hi.x << 16), h1 = __uint_as_float(hi.x & 0xffff0000u);
          float h2 = __uint_as_float(hi.y << 16), h3 = __uint_as_float(hi.y & 0xffff0000u);
          const uint32_t off = nat2[j] + row_off(ml) * 2u, offt = tr_off(j, ml);
          st_rows4(rN0, off, hi);
          st64(rT0, offt, hi);
          if (two) {
            uint2 lo;
            lo.x = f32x2_to_bf16x2(v0 - h0, v1 - h1);
            lo.y = f32x2_to_bf16x2(v2 - h2, v3 - h3);
            st_rows4(rN1, off, lo);
            st64(rT1, offt, lo);
            // hi + lo has at most 17 significant bits: the fp32 sums are exact
            h0 += __uint_as_float(lo.x << 16); h1 += __uint_as_float(lo.x & 0xffff0000u);
            h2 += __uint_as_float(lo.y << 16); h3 += __uint_as_float(lo.y & 0xffff0000u);
          }
          st32(rC, nat4[j] + row_off(ml) * 4u, h0);
          st32(rC, nat4[j] + row_off(ml + 1) * 4u, h1);
          st32(rC, nat4[j] + row_off(ml + 2) * 4u, h2);
          st32(rC, nat4[j] + row_off(ml + 3) * 4u, h3);
        }
      }
  } else {  // EPI_XOUT
    const int64_t boff = (int64_t)bz * g.batchC;
    // an absent array gets an empty range: its loads return zero and its stores are dropped
    const auto rX = in_rsrc(g.Xadd ? g.Xadd + boff : nullptr, g.Xadd ? nat_rows * 4u : 0u);
    const auto rC = out_rsrc(g.C32 ? g.C32 + boff : nullptr, g.C32 ? nat_rows * 4u : 0u);
    const int np_max = F16 ? 1 : (g.np_out > g.np_out_n ? g.np_out : g.np_out_n);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        float v[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) v[e] = acc[i][j][e];
        if (g.Xadd) {
#pragma unroll
          for (int e = 0; e < 16; ++e) v[e] += ld32(rX, nat4[j] + row_off(32 * i + 8 * (e >> 2) + (e & 3)) * 4u);
        }
        if (g.C32) {
#pragma unroll
          for (int e = 0; e < 16; ++e) st32(rC, nat4[j] + row_off(32 * i + 8 * (e >> 2) + (e & 3)) * 4u, v[e]);
        }
        for (int p = 0; p < np_max; ++p) {
          const auto rN = out_rsrc(g.Pn + p * g.plane_out + boff, p < g.np_out_n ? nat_rows * 2u : 0u);
          const auto rT = out_rsrc(g.Pt + p * g.plane_out + boff, p < g.np_out ? tr_rows * 2u : 0u);
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int ml = 32 * i + 8 * q;
            uint2 t;   // the 4 values of rows ml .. ml + 3, packed; the remainder goes on to the next plane
            if constexpr (F16) {   // fp16 operands: the iterate is one fp16 plane of each layout
              t.x = f32x2_to_f16x2(v[4 * q], v[4 * q + 1]);
              t.y = f32x2_to_f16x2(v[4 * q + 2], v[4 * q + 3]);
            } else {
              t.x = f32x2_to_bf16x2(v[4 * q], v[4 * q + 1]);
              t.y = f32x2_to_bf16x2(v[4 * q + 2], v[4 * q + 3]);
              v[4 * q] -= __uint_as_float(t.x << 16); v[4 * q + 1] -= __uint_as_float(t.x & 0xffff0000u);
              v[4 * q + 2] -= __uint_as_float(t.y << 16); v[4 * q + 3] -= __uint_as_float(t.y & 0xffff0000u);
            }
            st_rows4(rN, nat2[j] + row_off(ml) * 2u, t);
            st64(rT, tr_off(j, ml), t);
          }
        }
      }
  }
  if (g.clk) {
    wait_vmcnt<0>();   // the epilogue's stores have left the wavefront
    if (tid == 0) {
      unsigned long long* o = g.clk + 4 * ((int64_t)blockIdx.z * gridDim.x + blockIdx.x);
      o[0] = pr_c2 - pr_c1;
      o[1] = pr_w2 - pr_w1;
      o[2] = pr_w1 - pr_w0;
      o[3] = wall_clock64() - pr_w2;
    }
  }
}

struct Tile { int bm, bn, wgm, wgn; float eff; };
constexpr Tile kTiles[] = {{256, 256, 2, 4, 1.0f}, {256, 128, 4, 2, 0.85f}, {128, 128, 2, 2, 0.7f}, {64, 64, 2, 2, 0.35f},
                           {192, 192, 3, 2, 0.9f}};   // 192: fills the chip exactly at d = 3072
constexpr int kNumTiles = 5;

int pick_tile(int M, int N, int batch) {
  int best = 0;
  double best_cost = 1e300;
  for (int t = 0; t < kNumTiles; ++t) {
    const int64_t tiles = (int64_t)((M + kTiles[t].bm - 1) / kTiles[t].bm) * ((N + kTiles[t].bn - 1) / kTiles[t].bn) * batch;
    const int64_t waves = (tiles + 255) / 256;
    const double cost = (double)waves * kTiles[t].bm * kTiles[t].bn / kTiles[t].eff;
    if (cost < best_cost) { best_cost = cost; best = t; }
  }
  return best;
}

constexpr int kSymMinTiles = 8;   // tiles per side from which the mirrored form is used

// Tile for a symmetric product (only the t (t + 1) / 2 tiles on and above the diagonal run): the square tile with the
// least rounds x tile area / efficiency, or -1 if no square tile gives at least kSymMinTiles per side.  Counting the
// tiles that really run matters: at 4096 the 256 x 256 tile leaves 136 workgroups on 256 compute units, the 192 x 192
// tile 253 (measured 80 against 96 us for a Gram matrix); at 8192 it is 946 tiles in 4 rounds against 528 in 3.
int pick_tile_sym(int M, int batch) {
  int best = -1;
  double best_cost = 1e300;
  for (int t = 0; t < kNumTiles; ++t) {
    if (kTiles[t].bm != kTiles[t].bn) continue;
    const int64_t side = (M + kTiles[t].bm - 1) / kTiles[t].bm;
    if (side < kSymMinTiles) continue;
    const int64_t rounds = (side * (side + 1) / 2 * batch + 255) / 256;
    const double cost = (double)rounds * kTiles[t].bm * kTiles[t].bn / kTiles[t].eff;
    if (cost < best_cost) { best_cost = cost; best = t; }
  }
  return best;
}

template <int BM, int BN, int WGM, int WGN, int NSTAGE, int EPI, bool F16, bool SYM = false>
hipError_t launch_one(const GemmArgs& a, int batch, hipStream_t stream) {
  constexpr int smem = NSTAGE * (BM + BN) * BK * 2;
  static_assert(smem <= 160 * 1024, "LDS of one CU");
  static PerDeviceOnce configured;
  auto kern = gemm_nt_kernel<BM, BN, WGM, WGN, NSTAGE, EPI, F16, SYM>;
  hipError_t e = configured.run([&] {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, smem);
  });
  if (e != hipSuccess) return e;
  const int tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.N + BN - 1) / BN;
  dim3 grid(SYM ? tiles_m * (tiles_m + 1) / 2 : tiles_m * tiles_n, 1, batch);
  hipLaunchKernelGGL(kern, grid, dim3(64 * WGM * WGN), smem, stream, a, tiles_m, tiles_n);
  return hipGetLastError();
}

template <int EPI, bool F16 = false>
hipError_t launch_epi(const GemmArgs& a, int batch, hipStream_t stream) {
  if constexpr (EPI == EPI_GRAMW || EPI == EPI_SQUARE || EPI == EPI_FRO2) {
    if (a.symmetric) {   // tiles on and above the diagonal only, where a square tile gives enough of them per side
      switch (pick_tile_sym(a.M, batch)) {
        case 0: return launch_one<256, 256, 2, 4, 2, EPI, F16, true>(a, batch, stream);
        case 2: return launch_one<128, 128, 2, 2, 3, EPI, F16, true>(a, batch, stream);
        case 4: return launch_one<192, 192, 3, 2, 3, EPI, F16, true>(a, batch, stream);
        case 3: return launch_one<64, 64, 2, 2, 3, EPI, F16, true>(a, batch, stream);
        default: break;
      }
    }
  }
  switch (pick_tile(a.M, a.N, batch)) {
    // LDS stages: as many 64-deep tiles as fit (two of 64 KiB for 256 x 256; smaller tiles take a third, which
    // puts two K steps instead of one between a load's issue and its use)
    case 0: return launch_one<256, 256, 2, 4, 2, EPI, F16>(a, batch, stream);
    case 1: return launch_one<256, 128, 4, 2, 3, EPI, F16>(a, batch, stream);
    case 2: return launch_one<128, 128, 2, 2, 3, EPI, F16>(a, batch, stream);
    case 4: return launch_one<192, 192, 3, 2, 3, EPI, F16>(a, batch, stream);
    default: return launch_one<64, 64, 2, 2, 3, EPI, F16>(a, batch, stream);
  }
}

}  // namespace

int gemm_num_partials(int M, int N, int batch, int symmetric) {
  int t = pick_tile(M, N, batch);
  if (symmetric && M == N) {
    const int ts = pick_tile_sym(M, batch);
    if (ts >= 0) t = ts;
  }
  const Tile& u = kTiles[t];
  return ((M + u.bm - 1) / u.bm) * ((N + u.bn - 1) / u.bn) * u.wgm * u.wgn;
}

double gemm_issued_flop(const GemmArgs& a, GemmEpilogue epi, int batch) {
  int t = pick_tile(a.M, a.N, batch);
  bool sym = false;
  if (a.symmetric && (epi == EPI_GRAMW || epi == EPI_SQUARE || epi == EPI_FRO2)) {
    const int ts = pick_tile_sym(a.M, batch);
    if (ts >= 0) { t = ts; sym = true; }
  }
  const Tile& u = kTiles[t];
  const int64_t tm = (a.M + u.bm - 1) / u.bm, tn = (a.N + u.bn - 1) / u.bn;
  const int64_t tiles = sym ? tm * (tm + 1) / 2 : tm * tn;
  return 2.0 * (double)tiles * u.bm * u.bn * (double)a.K * a.nseg * batch;
}

int gemm_num_workgroups(int M, int N, int batch) {
  const Tile& t = kTiles[pick_tile(M, N, batch)];
  return ((M + t.bm - 1) / t.bm) * ((N + t.bn - 1) / t.bn) * batch;
}

hipError_t launch_gemm_nt(const GemmArgs& a, GemmEpilogue epi, int batch, hipStream_t stream) {
  if (a.M <= 0 || a.N <= 0 || a.K <= 0 || (a.K & 7) || (a.lda & 7) || (a.ldb & 7) || a.nseg < 1 || a.nseg > kMaxSegments ||
      batch < 1 || (a.ab_f16 && epi != EPI_F32 && epi != EPI_GRAMW && epi != EPI_XOUT && epi != EPI_XLAST) ||
      (a.ab_f16 && ((epi == EPI_GRAMW && (a.np_out != 1 || a.np_add != 0)) ||
                    (epi == EPI_XOUT && (a.np_out != 1 || a.np_out_n != 1 || a.Xadd || a.C32)))) || (int64_t)a.M * a.lda >= (1ll << 30) || (int64_t)a.N * a.ldb >= (1ll << 30))
    return hipErrorInvalidValue;
  if (a.symmetric && ((epi != EPI_GRAMW && epi != EPI_SQUARE && epi != EPI_FRO2) || (epi != EPI_FRO2 && a.A != a.B) ||
                      a.M != a.N || a.lda != a.ldb || (a.M & 3)))
    return hipErrorInvalidValue;
  // the matrix-writing epilogues address their arrays [M or N rows][ldc] through 32-bit byte offsets
  if ((epi == EPI_F32 || epi == EPI_GRAMW || epi == EPI_SQUARE || epi == EPI_XLAST || epi == EPI_XOUT) &&
      (a.ldc < a.N || (epi != EPI_F32 && a.ldc < a.M) || (int64_t)((a.M > a.N ? a.M : a.N) + 256) * a.ldc >= (1ll << 29)))
    return hipErrorInvalidValue;
  // EPI_ACT / EPI_SIGN_ACT address Y relative to a tile's first row: 256 rows x pitch x 4 bytes below 2^31
  if ((epi == EPI_ACT && (a.ldc < a.N || a.ldc >= (1ll << 21))) || (epi == EPI_SIGN_ACT && (a.ldy < a.N || a.ldy >= (1ll << 21))))
    return hipErrorInvalidValue;
  if (epi == EPI_XLAST && (!a.C32 || !a.Pn || !a.Pt || (a.M & 3) || a.np_out < 1 || a.np_out > 2)) return hipErrorInvalidValue;
  switch (epi) {
    case EPI_SIGN: return launch_epi<EPI_SIGN>(a, batch, stream);
    case EPI_SIGN_XT:
      if (!a.xt_w || !a.Xt || !a.cnt || a.cnt_slots < 1 || a.N != a.K || a.nseg != 1) return hipErrorInvalidValue;
      return launch_epi<EPI_SIGN_XT>(a, batch, stream);
    case EPI_SIGN_ACT: return a.Yact ? launch_epi<EPI_SIGN_ACT>(a, batch, stream) : hipErrorInvalidValue;
    case EPI_ACT: return launch_epi<EPI_ACT>(a, batch, stream);
    case EPI_F32: return a.ab_f16 ? launch_epi<EPI_F32, true>(a, batch, stream) : launch_epi<EPI_F32>(a, batch, stream);
    case EPI_GRAMW: return a.ab_f16 ? launch_epi<EPI_GRAMW, true>(a, batch, stream) : launch_epi<EPI_GRAMW>(a, batch, stream);
    case EPI_XLAST: return a.ab_f16 ? launch_epi<EPI_XLAST, true>(a, batch, stream) : launch_epi<EPI_XLAST>(a, batch, stream);
    case EPI_XOUT: return a.ab_f16 ? launch_epi<EPI_XOUT, true>(a, batch, stream) : launch_epi<EPI_XOUT>(a, batch, stream);
    case EPI_SQUARE: return launch_epi<EPI_SQUARE>(a, batch, stream);
    case EPI_FRO2: return launch_epi<EPI_FRO2>(a, batch, stream);
  }
  return hipErrorInvalidValue;
}

}  // namespace conqur
