// Half-precision-operand variant of the STFT contraction (gfx950 / CDNA4).
//
// Same contraction and same sliding LDS tile of the waveform as the fp32 kernel, but both MFMA
// operands are float16 (the bank is rounded once at plan time, the waveform as it is written to
// LDS) and the products are accumulated in float32 by v_mfma_f32_32x32x16_f16, whose rate is 16
// times that of the fp32 MFMA.  At that rate a wave cannot stream its bank fragments from the
// L2 any more, so both operands go through LDS and every fragment read is re-used four times:
// a workgroup (4 waves, one per SIMD) owns 256 bank rows x 192 frames, each wave 128 x 96
// (12 accumulator tiles of 32 x 32 = 192 registers; 16 tiles would fill the accumulator file to
// the last register and make the compiler spill).
//
// Per step (one 32-tap chunk of the hop at one hop-shift): the A tile (256 rows x 32 taps of the
// bank, 16 KB, contiguous in device memory) is copied to LDS; the B tile (the waveform rows the
// chunk needs, shared by all hop-shifts of the chunk) once per chunk.  Global loads are issued two
// steps ahead of their use and written to the LDS buffer that the previous step has finished
// with; one barrier per step.
//
// Rounding: float16 has an 11-bit significand; bank entries lie in [-1, 1] and the rounding errors
// of the 2,048 products of a frame are independent, so the error of a bin stays near 1e-5 of the
// spectrogram's peak (the parity bar is 1e-3).
#include "nna_device.h"

#include <type_traits>

namespace nna {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef f32x4 f32x4_u __attribute__((aligned(4)));

constexpr int H_RPP = 256 / (H_KC / 4);       // LDS rows written per loader pass (32)
constexpr int H_NPASS = H_LB_ROWS / H_RPP;    // 224 / 32 = 7
constexpr int H_JT = H_FRAMES / 64;           // 32-frame sub-tiles per wave (3)

// the B tile of one chunk goes to LDS as float16: 4 samples (8 bytes) per thread and pass
template <int NPASS>
__device__ __forceinline__ void store_chunk_f16(const f32x4 (&R)[NPASS], const TileFix<NPASS>& fx, _Float16* lds, int tid) {
  constexpr int V = H_KC / 4;
  const int cv = tid % V, r0 = tid / V;
  _Float16* dst = lds + r0 * H_PITCH + cv * 4;
#pragma unroll
  for (int p = 0; p < NPASS; ++p) {
    f32x4 v;
    if (fx.cls == 2) {
      const unsigned s = fx.sel[p];
      v = (f32x4){pick4(R[p], s & 3), pick4(R[p], (s >> 2) & 3), pick4(R[p], (s >> 4) & 3), pick4(R[p], (s >> 6) & 3)};
    } else {
      v = fixed_up<NPASS>(R[p], fx, p);
    }
    const f16x4 hv = {(_Float16)v.x, (_Float16)v.y, (_Float16)v.z, (_Float16)v.w};  // round to nearest even
    *reinterpret_cast<f16x4*>(dst + p * H_RPP * H_PITCH) = hv;
  }
}

// NJ = hop-shifts per chunk (n_fft / hop) when it is one the kernel is specialised for, else 0:
// with NJ known the steps of a chunk are unrolled into one loop body, which keeps the
// accumulators in place (with a run-time step loop the compiler peels the steps that load or
// store the B tile and shuffles all accumulators between the copies).
template <int NJ>
__global__ __launch_bounds__(256, 1) void stft16_kernel(const Stft16Params P) {
  __shared__ __attribute__((aligned(16))) _Float16 ldsA[2][H_ROWS * H_PITCH];
  __shared__ __attribute__((aligned(16))) _Float16 ldsB[2][H_LB_ROWS * H_PITCH];

  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int wr = wave >> 1, wc = wave & 1;  // this wave's 128 rows / 96 frames of the workgroup tile
  const int n = lane & 31, h = lane >> 5;

  // work item: the frame tile is the fast index, so that the workgroups resident at one time
  // read the same row tiles of the bank
  const int n_rg = (P.n_rt + P.rt_per_block - 1) / P.rt_per_block;
  const long long bid = blockIdx.x;
  const int rg = (int)(bid / P.n_ft);
  const long long ft = bid - (long long)rg * P.n_ft;
  if (rg >= n_rg) return;
  const int rt_begin = rg * P.rt_per_block;
  const int rt_end = rt_begin + P.rt_per_block < P.n_rt ? rt_begin + P.rt_per_block : P.n_rt;

  const FrameGeom& g = P.g;
  const long long f0 = ft * P.tile_frames;
  const int m_valid = (int)((g.n_frames - f0) < P.tile_frames ? (g.n_frames - f0) : P.tile_frames);
  TileMap tm;
  tm.T = g.T;
  tm.b0 = f0 / g.T;
  tm.t0 = (int)(f0 - tm.b0 * g.T);
  tm.n0 = (g.T - tm.t0) < m_valid ? (g.T - tm.t0) : m_valid;
  tm.extra = P.nj - 1;
  const int rows_used = tm.frame_row(m_valid - 1) + tm.extra + 1;

  RowDesc<H_NPASS> rd;
  build_rowdesc<H_KC, H_NPASS>(rd, g, tm, rows_used, tid);

  // this lane's frames (one per 32-frame sub-tile)
  bool valid[H_JT];
  int b_off[H_JT];
  long long o_off[H_JT];
#pragma unroll
  for (int jt = 0; jt < H_JT; ++jt) {
    const int fi = wc * (H_FRAMES / 2) + jt * 32 + n;
    valid[jt] = fi < m_valid;
    const long long f = f0 + fi;
    const long long b = valid[jt] ? f / g.T : 0;
    const int t = valid[jt] ? (int)(f - b * g.T) : 0;
    b_off[jt] = (valid[jt] ? tm.frame_row(fi) : 0) * H_PITCH + 8 * h;
    o_off[jt] = (b * P.out_bins) * g.T + t;
  }
  const int a_off = (wr * 128 + n) * H_PITCH + 8 * h;

  const int nj = P.nj, n_chunks = P.n_chunks;
  const int steps_per_rt = n_chunks * nj;
  if (rt_end <= rt_begin) return;

  // bank tiles of this row group are consecutive in memory: [row tile][chunk][shift][256 rows][32 taps]
  const _Float16* a_src = P.bank + ((long long)rt_begin * steps_per_rt) * (H_ROWS * H_KC) + tid * H_KC;
  _Float16* const a_dst0 = &ldsA[0][0] + tid * H_PITCH;

  // ---- prologue: A tile of step 0 and B tile of chunk 0 into LDS; A tile of step 1 requested ----
  f32x4 ga[4], pa[4];
  f32x4 gB[H_NPASS];
  TileFix<H_NPASS> fxB;
  {
    const float* ptr[H_NPASS];
    prepare_chunk<H_NPASS>(ptr, fxB, g, rd, 0);
#pragma unroll
    for (int p = 0; p < H_NPASS; ++p) gB[p] = *reinterpret_cast<const f32x4_u*>(ptr[p]);
#pragma unroll
    for (int s = 0; s < 4; ++s) pa[s] = *reinterpret_cast<const f32x4*>(a_src + s * 8);
    a_src += H_ROWS * H_KC;
#pragma unroll
    for (int s = 0; s < 4; ++s) ga[s] = *reinterpret_cast<const f32x4*>(a_src + s * 8);
    a_src += H_ROWS * H_KC;
    store_chunk_f16<H_NPASS>(gB, fxB, ldsB[0], tid);
#pragma unroll
    for (int s = 0; s < 4; ++s) *reinterpret_cast<f32x4*>(a_dst0 + s * 8) = pa[s];
  }
  __syncthreads();

  int s = 0, cc = 0;  // steps and chunks done so far (they select the LDS buffers)
  for (int rt = rt_begin; rt < rt_end; ++rt) {
    f32x16 acc[H_JT][4];  // [frame sub-tile][row sub-tile]
#pragma unroll
    for (int jt = 0; jt < H_JT; ++jt)
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[jt][i][r] = 0.f;

    // one step: hop-shift j of chunk c.  B_LOAD: request the B tile of the next chunk (first step of
    // a chunk); B_STORE: write it to the other B buffer (one step later when there is one).
    auto step = [&](auto load_tag, auto store_tag, int c, int j) {
      constexpr bool B_LOAD = decltype(load_tag)::value;
      constexpr bool B_STORE = decltype(store_tag)::value;
      // the A tile requested one step ago (for step s+1) is taken over; the one for step s+2 is requested
#pragma unroll
      for (int q = 0; q < 4; ++q) pa[q] = ga[q];
#pragma unroll
      for (int q = 0; q < 4; ++q) ga[q] = *reinterpret_cast<const f32x4*>(a_src + q * 8);
      a_src += H_ROWS * H_KC;
      if (B_LOAD) {
        // (the bank tail is padded, and the chunk after the last wraps to column 0: always in bounds)
        const float* ptr[H_NPASS];
        prepare_chunk<H_NPASS>(ptr, fxB, g, rd, ((c + 1) % n_chunks) * H_KC);
#pragma unroll
        for (int p = 0; p < H_NPASS; ++p) gB[p] = *reinterpret_cast<const f32x4_u*>(ptr[p]);
      }

      // ---- 24 MFMAs: two 16-tap halves of the chunk x 3 x 4 tiles ----
      const _Float16* A = &ldsA[s & 1][0] + a_off;
      const _Float16* Bt = &ldsB[cc & 1][0] + j * H_PITCH;
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        f16x8 af[4], bf[H_JT];
#pragma unroll
        for (int i = 0; i < 4; ++i) af[i] = *reinterpret_cast<const f16x8*>(A + i * 32 * H_PITCH + ks * 16);
#pragma unroll
        for (int jt = 0; jt < H_JT; ++jt) bf[jt] = *reinterpret_cast<const f16x8*>(Bt + b_off[jt] + ks * 16);
#pragma unroll
        for (int jt = 0; jt < H_JT; ++jt)
#pragma unroll
          for (int i = 0; i < 4; ++i)
            acc[jt][i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[i], bf[jt], acc[jt][i], 0, 0, 0);
      }

      // ---- stage the A tile of step s+1 (and the B tile) ----
      {
        _Float16* a_dst = a_dst0 + ((s + 1) & 1) * (H_ROWS * H_PITCH);
#pragma unroll
        for (int q = 0; q < 4; ++q) *reinterpret_cast<f32x4*>(a_dst + q * 8) = pa[q];
      }
      if (B_STORE) store_chunk_f16<H_NPASS>(gB, fxB, ldsB[(cc + 1) & 1], tid);
      __syncthreads();
      ++s;
    };
    using Yes = std::true_type;
    using No = std::false_type;
    for (int c = 0; c < n_chunks; ++c, ++cc) {
      if constexpr (NJ == 1) {
        step(Yes{}, Yes{}, c, 0);
      } else if constexpr (NJ >= 2) {
        step(Yes{}, No{}, c, 0);
        step(No{}, Yes{}, c, 1);
#pragma unroll
        for (int j = 2; j < NJ; ++j) step(No{}, No{}, c, j);
      } else {
        step(Yes{}, No{}, c, 0);
        step(No{}, Yes{}, c, 1);
        for (int j = 2; j < nj; ++j) step(No{}, No{}, c, j);
      }
    }

    // ---- epilogue of row tile rt ----
    const int slot_base = rt * (H_ROWS / 2) + wr * 64;
#pragma unroll
    for (int jt = 0; jt < H_JT; ++jt) {
      if (valid[jt]) {
        float* __restrict__ op = P.out + o_off[jt];
        if (P.fmt == NNA_OUT_MAGNITUDE)
          stft_store_tile<NNA_OUT_MAGNITUDE>(acc[jt], op, g.T, slot_base, h, P.n_half, P.packed);
        else if (P.fmt == NNA_OUT_POWER)
          stft_store_tile<NNA_OUT_POWER>(acc[jt], op, g.T, slot_base, h, P.n_half, P.packed);
        else
          stft_store_tile<NNA_OUT_LOG>(acc[jt], op, g.T, slot_base, h, P.n_half, P.packed);
      }
    }
  }
}

// ---------------------------------------------------------------------------------------
// Streamed-bank variant (the one that runs when n_fft / hop is 2, 4 or 8).
//
// Measured on the kernel above: with one wave per SIMD nothing hides the latency of the LDS
// reads, and every 24 MFMAs end in a barrier -- the matrix pipe was busy 35 % of the time while
// the LDS was active 19 %.  (Past about half-busy matrix pipes the chip is power-limited on this
// kernel: the shader clock falls from 2.4 to 1.65-1.8 GHz and throughput stays near 0.9 PFLOP/s.)  Here only the frames go through LDS.  Each wave streams its own bank
// fragments straight from the L2 into a ring of registers, four K-steps (16 taps each) ahead,
// with the same hand-scheduled loads as the float32 kernels: the bank is stored in the order
// [row tile][chunk][hop-shift][K-step][row half][4 fragments][64 lanes] x 16 bytes, so a wave
// fetches the four A fragments of a K-step (4 KB) with four scalar-base loads.  The barrier moves
// from every step to every chunk (all hop-shifts of a 32-tap chunk share one LDS tile), and the
// tile staging (float32 -> float16 on the way to LDS) is spread behind the MFMAs of the chunk's
// first two K-steps.
// ---------------------------------------------------------------------------------------
constexpr int HS_RING = 4;  // K-steps of bank fragments in flight per wave

template <int NJ>
__global__ __launch_bounds__(256, 1) void stft16s_kernel(const Stft16Params P) {
  static_assert(NJ == 2 || NJ == 4 || NJ == 8, "K-steps per chunk must be a multiple of the ring depth");
  __shared__ __attribute__((aligned(16))) _Float16 ldsB[2][H_LB_ROWS * H_PITCH];

  const int tid = threadIdx.x;
  // the wave index is uniform over the wave: as a scalar it keeps the bank pointer in scalar registers
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int wr = wave >> 1, wc = wave & 1;
  const int n = lane & 31, h = lane >> 5;

  const int n_rg = (P.n_rt + P.rt_per_block - 1) / P.rt_per_block;
  const long long bid = blockIdx.x;
  const int rg = (int)(bid / P.n_ft);
  const long long ft = bid - (long long)rg * P.n_ft;
  if (rg >= n_rg) return;
  const int rt_begin = rg * P.rt_per_block;
  const int rt_end = rt_begin + P.rt_per_block < P.n_rt ? rt_begin + P.rt_per_block : P.n_rt;
  if (rt_end <= rt_begin) return;

  const FrameGeom& g = P.g;
  const long long f0 = ft * P.tile_frames;
  const int m_valid = (int)((g.n_frames - f0) < P.tile_frames ? (g.n_frames - f0) : P.tile_frames);
  TileMap tm;
  tm.T = g.T;
  tm.b0 = f0 / g.T;
  tm.t0 = (int)(f0 - tm.b0 * g.T);
  tm.n0 = (g.T - tm.t0) < m_valid ? (g.T - tm.t0) : m_valid;
  tm.extra = NJ - 1;
  const int rows_used = tm.frame_row(m_valid - 1) + tm.extra + 1;

  RowDesc<H_NPASS> rd;
  build_rowdesc<H_KC, H_NPASS>(rd, g, tm, rows_used, tid);

  bool valid[H_JT];
  int b_off[H_JT];
  long long o_off[H_JT];
#pragma unroll
  for (int jt = 0; jt < H_JT; ++jt) {
    const int fi = wc * (H_FRAMES / 2) + jt * 32 + n;
    valid[jt] = fi < m_valid;
    const long long f = f0 + fi;
    const long long b = valid[jt] ? f / g.T : 0;
    const int t = valid[jt] ? (int)(f - b * g.T) : 0;
    b_off[jt] = (valid[jt] ? tm.frame_row(fi) : 0) * H_PITCH + 8 * h;
    o_off[jt] = (b * P.out_bins) * g.T + t;
  }

  const int n_chunks = P.n_chunks;
  constexpr int KSTEPS = 2 * NJ;                  // K-steps per chunk
  constexpr int KSTEP_BYTES = 2 * 4 * 64 * 16;    // both row halves of one K-step (8 KB)

  // ---- prologue: tile of chunk 0 into LDS, tile of chunk 1 requested, ring filled ----
  f32x4 R[H_NPASS];
  TileFix<H_NPASS> fx;
  issue_chunk<H_NPASS>(R, fx, g, rd, 0);
  wait_vm<0>(R);
  store_chunk_f16<H_NPASS>(R, fx, ldsB[0], tid);
  issue_chunk<H_NPASS>(R, fx, g, rd, (1 % n_chunks) * H_KC);

  const unsigned lane_off = (unsigned)lane * 16u;
  const char* bank_s = reinterpret_cast<const char*>(P.bank) +
                       ((long long)rt_begin * n_chunks * KSTEPS) * KSTEP_BYTES + wr * (KSTEP_BYTES / 2);
  f32x4 bq[HS_RING][4];
#pragma unroll
  for (int sl = 0; sl < HS_RING; ++sl) {
    gload16_s<0>(bq[sl][0], lane_off, bank_s);
    gload16_s<1024>(bq[sl][1], lane_off, bank_s);
    gload16_s<2048>(bq[sl][2], lane_off, bank_s);
    gload16_s<3072>(bq[sl][3], lane_off, bank_s);
    bank_s += KSTEP_BYTES;
  }
  __syncthreads();

  // Loads retire in order.  When a K-step starts, the requests younger than its own ring slot are
  // the other HS_RING-1 slots (and possibly the chunk tile: never counted, the safe side).  The
  // tile in R was requested in the second K-step of the previous chunk (or in the prologue) and is
  // followed by at least three whole slots.
  constexpr int W_SLOT = (HS_RING - 1) * 4;
  constexpr int W_TILE = 3 * 4;
  constexpr int TASK_NONE = 0, TASK_STORE = 1, TASK_LOAD = 2;
  _Float16* const stage_dst0 = &ldsB[0][0] + (tid / (H_KC / 4)) * H_PITCH + (tid % (H_KC / 4)) * 4;

  int it = 0;  // chunks done so far
  for (int rt = rt_begin; rt < rt_end; ++rt) {
    f32x16 acc[H_JT][4];  // [frame sub-tile][row sub-tile]
#pragma unroll
    for (int jt = 0; jt < H_JT; ++jt)
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[jt][i][r] = 0.f;

    for (int c = 0; c < n_chunks; ++c, ++it) {
      // R holds the tile of chunk it+1: its LDS writes and the requests for chunk it+2 ride behind
      // the MFMAs of the first two K-steps; only the address arithmetic (and the rare edge
      // handling) happens here.
      wait_vm<W_TILE>(R);
      const TileFix<H_NPASS> fx_store = fx;
      if (fx_store.cls == 2) store_chunk_f16<H_NPASS>(R, fx_store, ldsB[(it + 1) & 1], tid);
      const float* ptr[H_NPASS];
      prepare_chunk<H_NPASS>(ptr, fx, g, rd, ((it + 2) % n_chunks) * H_KC);
      _Float16* const stage_dst = stage_dst0 + ((it + 1) & 1) * (H_LB_ROWS * H_PITCH);
      const _Float16* Bt = &ldsB[it & 1][0];
      __builtin_amdgcn_sched_barrier(0);

      f16x8 bf[H_JT];  // frames fragments of the K-step about to run
#pragma unroll
      for (int jt = 0; jt < H_JT; ++jt) bf[jt] = *reinterpret_cast<const f16x8*>(Bt + b_off[jt]);
      // one K-step: 16 taps, 12 MFMAs (3 frame sub-tiles x 4 row sub-tiles)
      auto kstep = [&](auto task_tag, auto g_tag) {
        constexpr int TASK = decltype(task_tag)::value;
        constexpr int G = decltype(g_tag)::value;
        constexpr int sl = G % HS_RING;
        // the frames fragments of the next K-step are read from LDS while this one's MFMAs run
        constexpr int G1 = G + 1 < KSTEPS ? G + 1 : G;
        f16x8 bf_nxt[H_JT];
#pragma unroll
        for (int jt = 0; jt < H_JT; ++jt)
          bf_nxt[jt] = *reinterpret_cast<const f16x8*>(Bt + b_off[jt] + (G1 / 2) * H_PITCH + (G1 % 2) * 16);
        wait_vm<W_SLOT>(bq[sl][0], bq[sl][1], bq[sl][2], bq[sl][3]);
        __builtin_amdgcn_sched_group_barrier(0x100, H_JT, 0);  // the LDS reads go first
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int m = 0; m < 4 * H_JT; ++m) {
          const int jt = m >> 2, i = m & 3;
          acc[jt][i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, bq[sl][i]), bf[jt], acc[jt][i], 0, 0, 0);
          if (TASK != TASK_NONE && m < H_NPASS) {
            const int p = m;
            __builtin_amdgcn_sched_barrier(0);
            if (TASK == TASK_STORE) {
              if (fx_store.cls != 2) {
                const f32x4 v = fixed_up<H_NPASS>(R[p], fx_store, p);
                const f16x4 hv = {(_Float16)v.x, (_Float16)v.y, (_Float16)v.z, (_Float16)v.w};
                *reinterpret_cast<f16x4*>(stage_dst + p * H_RPP * H_PITCH) = hv;
              }
            } else {
              gload16(R[p], ptr[p]);
            }
            __builtin_amdgcn_sched_barrier(0);
          }
          if (m >= 4 * (H_JT - 1)) {
            // last reader of fragment i of this slot: request the K-step HS_RING ahead (the bank
            // allocation is padded by HS_RING K-steps, so the tail stays in bounds)
            __builtin_amdgcn_sched_barrier(0);
            if (i == 0) gload16_s<0>(bq[sl][0], lane_off, bank_s);
            if (i == 1) gload16_s<1024>(bq[sl][1], lane_off, bank_s);
            if (i == 2) gload16_s<2048>(bq[sl][2], lane_off, bank_s);
            if (i == 3) gload16_s<3072>(bq[sl][3], lane_off, bank_s);
            __builtin_amdgcn_sched_barrier(0);
          }
        }
        bank_s += KSTEP_BYTES;
#pragma unroll
        for (int jt = 0; jt < H_JT; ++jt) bf[jt] = bf_nxt[jt];
      };
      kstep(std::integral_constant<int, TASK_STORE>{}, std::integral_constant<int, 0>{});
      kstep(std::integral_constant<int, TASK_LOAD>{}, std::integral_constant<int, 1>{});
      kstep(std::integral_constant<int, TASK_NONE>{}, std::integral_constant<int, 2>{});
      kstep(std::integral_constant<int, TASK_NONE>{}, std::integral_constant<int, 3>{});
      if constexpr (NJ >= 4) {
        kstep(std::integral_constant<int, TASK_NONE>{}, std::integral_constant<int, 4>{});
        kstep(std::integral_constant<int, TASK_NONE>{}, std::integral_constant<int, 5>{});
        kstep(std::integral_constant<int, TASK_NONE>{}, std::integral_constant<int, 6>{});
        kstep(std::integral_constant<int, TASK_NONE>{}, std::integral_constant<int, 7>{});
      }
      if constexpr (NJ >= 8) {
        kstep(std::integral_constant<int, TASK_NONE>{}, std::integral_constant<int, 8>{});
        kstep(std::integral_constant<int, TASK_NONE>{}, std::integral_constant<int, 9>{});
        kstep(std::integral_constant<int, TASK_NONE>{}, std::integral_constant<int, 10>{});
        kstep(std::integral_constant<int, TASK_NONE>{}, std::integral_constant<int, 11>{});
        kstep(std::integral_constant<int, TASK_NONE>{}, std::integral_constant<int, 12>{});
        kstep(std::integral_constant<int, TASK_NONE>{}, std::integral_constant<int, 13>{});
        kstep(std::integral_constant<int, TASK_NONE>{}, std::integral_constant<int, 14>{});
        kstep(std::integral_constant<int, TASK_NONE>{}, std::integral_constant<int, 15>{});
      }
      __syncthreads();
    }

    // ---- epilogue of row tile rt ----
    const int slot_base = rt * (H_ROWS / 2) + wr * 64;
#pragma unroll
    for (int jt = 0; jt < H_JT; ++jt) {
      if (valid[jt]) {
        float* __restrict__ op = P.out + o_off[jt];
        if (P.fmt == NNA_OUT_MAGNITUDE)
          stft_store_tile<NNA_OUT_MAGNITUDE>(acc[jt], op, g.T, slot_base, h, P.n_half, P.packed);
        else if (P.fmt == NNA_OUT_POWER)
          stft_store_tile<NNA_OUT_POWER>(acc[jt], op, g.T, slot_base, h, P.n_half, P.packed);
        else
          stft_store_tile<NNA_OUT_LOG>(acc[jt], op, g.T, slot_base, h, P.n_half, P.packed);
      }
    }
  }

  // drain the requests that are never consumed: their registers must stay reserved until then
  wait_vm<0>(R);
#pragma unroll
  for (int sl = 0; sl < HS_RING; ++sl) wait_vm<0>(bq[sl][0], bq[sl][1], bq[sl][2], bq[sl][3]);
}

hipError_t launch_stft16(const Stft16Params& p, hipStream_t stream) {
  clear_stale_error();
  const long long n_rg = (p.n_rt + p.rt_per_block - 1) / p.rt_per_block;
  const long long blocks = p.n_ft * n_rg;
  if (blocks <= 0 || blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  if (p.tile_frames > H_FRAMES || p.nj < 1) return hipErrorInvalidValue;
  if (p.bank_s && (p.nj == 2 || p.nj == 4 || p.nj == 8)) {
    Stft16Params q = p;
    q.bank = p.bank_s;
    switch (p.nj) {
      case 2: hipLaunchKernelGGL(stft16s_kernel<2>, dim3((unsigned)blocks), dim3(256), 0, stream, q); break;
      case 4: hipLaunchKernelGGL(stft16s_kernel<4>, dim3((unsigned)blocks), dim3(256), 0, stream, q); break;
      default: hipLaunchKernelGGL(stft16s_kernel<8>, dim3((unsigned)blocks), dim3(256), 0, stream, q); break;
    }
    return hipGetLastError();
  }
  switch (p.nj) {
    case 1: hipLaunchKernelGGL(stft16_kernel<1>, dim3((unsigned)blocks), dim3(256), 0, stream, p); break;
    case 2: hipLaunchKernelGGL(stft16_kernel<2>, dim3((unsigned)blocks), dim3(256), 0, stream, p); break;
    case 4: hipLaunchKernelGGL(stft16_kernel<4>, dim3((unsigned)blocks), dim3(256), 0, stream, p); break;
    case 8: hipLaunchKernelGGL(stft16_kernel<8>, dim3((unsigned)blocks), dim3(256), 0, stream, p); break;
    default: hipLaunchKernelGGL(stft16_kernel<0>, dim3((unsigned)blocks), dim3(256), 0, stream, p); break;
  }
  return hipGetLastError();
}

}  // namespace nna
