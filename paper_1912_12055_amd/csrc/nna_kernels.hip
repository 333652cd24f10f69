// GPU kernels (gfx950 / CDNA4) for the strided-convolution spectrogram transforms of
// arXiv 1912.12055: STFT (Sec. III-A), Mel (Sec. III-B) and time-domain CQT (Sec. III-C).
//
// All three are the contraction  C[row, frame] = sum_k bank[row, k] * xp[frame*hop + k]
// (a strided convolution, eq. (convolutionWithStride), with the kernel flip of Sec. III-A
// folded away) followed by a per-(Re,Im)-pair epilogue.  The kernels never materialise the
// frames matrix: because frames overlap, the reflect-padded waveform is viewed as a matrix
// S[r, c] = xp[r*hop + c] and frame t, tap k = j*hop + c reads S[t + j, c].  One LDS tile of
// (frames + overlap) rows x KC columns therefore serves every hop-shift j by sliding one row.
// The bank is stored in device memory in exactly the order the MFMA fragments are consumed,
// so each wave streams it with one coalesced 16-byte load per lane per fragment.
//
// MFMA operand roles: the bank supplies the "A" operand (rows = Re/Im bank rows), the frames
// supply "B" (columns = frames), so that in the accumulator the 32 (or 16) lanes of a
// register hold consecutive frames of one bin -- the output [B, bins, T] is T-fastest and the
// stores coalesce without a transpose.
#include "nna_device.h"

#include <type_traits>
#include <utility>

namespace nna {

// ---------------------------------------------------------------------------------------
// STFT / Mel kernel.
// Workgroup = 4 waves; wave w owns frames [32w, 32w+32) of the frame tile and all 128 rows of
// the current row tile: 4 accumulators of 32x32 (v_mfma_f32_32x32x2_f32).  Accumulator
// register r of lane l = (h = l/32, n = l%32) holds row 8*(r/4) + 4h + r%4 of frame n, so the
// (Re, Im) rows 2s, 2s+1 of slot s sit in registers r, r+1 of one lane.
// Row tiles are visited one after the other; in the Mel variant the power of each finished row
// tile is contracted, straight from the accumulator registers, with the matching slice of the
// filterbank by a second MFMA into 128 mel x 32 frame accumulators.
//
// Pipeline per LDS chunk `it` (KC taps of every hop-shift): the tile of chunk it+1, requested
// one chunk earlier, is written to the other LDS buffer; the tile of chunk it+2 is requested;
// then nj * ST_NKG fragment groups of 16 MFMAs run, each group waiting only for its own bank
// fragments (requested RING groups earlier) and re-requesting its ring slot afterwards.
// ---------------------------------------------------------------------------------------
constexpr int ST_RPP = 256 / (ST_KC / 4);          // LDS rows written per loader pass (32)
constexpr int ST_RING_STFT = 4;  // bank fragment groups in flight per wave
constexpr int ST_RING_MEL = 2;   // fewer in the Mel variant: its 64 extra accumulators need the registers

// MODE (ST_MODE_*): what follows the contraction of a row tile.
// LIN_NB: 32-row blocks of the second contraction's output per pass (ST_MODE_LIN); in every mode a value above 4 selects
// the one-workgroup-per-CU build with the 192-row LDS tile.
template <int MODE, int RING, int LIN_NB = ST_MEL_BLOCKS>
__global__ __launch_bounds__(256, LIN_NB > 4 ? 1 : 2) void stft_kernel(const StftParams P) {
  static_assert(ST_NKG % RING == 0, "ring depth must divide the fragment groups per LDS row");
  constexpr bool MEL = MODE == ST_MODE_MEL || MODE == ST_MODE_LIN || MODE == ST_MODE_MELSPEC;  // a second contraction follows every row tile
  constexpr bool SPEC = MODE == ST_MODE_MELSPEC;  // ... and the spectrogram itself is an output too
  constexpr bool LIN = MODE == ST_MODE_LIN;
  constexpr bool GRAD = MODE == ST_MODE_GRAD;  // backward pass: the row tile becomes dLoss/dC
  constexpr bool CPLX = MODE == ST_MODE_CPLX;  // complex or phase output
  // The six-block variant runs one workgroup per compute unit: its tile may hold more overlap rows (a tile of
  // 128 frames across two waveforms with 32 hop-shifts needs 190).
  constexpr int LDS_ROWS = LIN_NB > 4 ? ST_LDS_ROWS_WIDE : ST_LDS_ROWS;
  constexpr int NPASS = LDS_ROWS / ST_RPP;
  __shared__ __attribute__((aligned(16))) float lds[2][LDS_ROWS * ST_PITCH];

  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int h = lane >> 5, n = lane & 31;

  // ---- which work item: (frame tile, row tile range) --------------------------------
  long long ft;
  int rt_begin, rt_end, pass = 0;
  if constexpr (MEL) {
    pass_work_item(blockIdx.x, P.n_ft, P.n_pass, ft, pass);
    rt_begin = P.mel_pass_rt[2 * pass];
    rt_end = P.mel_pass_rt[2 * pass + 1];
    if (SPEC && pass == 0) {  // the spectrogram needs every row tile, also those no filter touches
      rt_begin = 0;
      rt_end = P.n_rt;
    }
  } else {
    // XCD-aware order: workgroup ids are dealt round-robin to the 8 XCDs.  Each XCD walks its
    // own contiguous range of frame tiles in groups of 64; inside a group the row group (ST_RG
    // consecutive row tiles handled by one workgroup) is the slow index, so the ~64 workgroups
    // resident on an XCD stream the same bank tiles through its L2.
    constexpr int GROUP = 64;
    const int n_rg = (P.n_rt + ST_RG - 1) / ST_RG;
    const long long bid = blockIdx.x;
    const int xcd = (int)(bid & 7);
    const long long idx = bid >> 3;
    const long long ft_per_xcd = (P.n_ft + 7) / 8;
    const long long per_group = (long long)GROUP * n_rg;
    const long long grp = idx / per_group;
    const int rem = (int)(idx - grp * per_group);
    const long long grp_first = grp * GROUP;
    long long grp_size = ft_per_xcd - grp_first;
    if (grp_size > GROUP) grp_size = GROUP;
    if (grp_size <= 0) return;
    const int rg = rem / (int)grp_size;
    const int fi = rem - rg * (int)grp_size;
    if (rg >= n_rg) return;
    const long long ft_local = grp_first + fi;
    ft = xcd * ft_per_xcd + ft_local;
    if (ft >= P.n_ft) return;
    rt_begin = rg * ST_RG;
    rt_end = rt_begin + ST_RG < P.n_rt ? rt_begin + ST_RG : P.n_rt;
  }

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

  const int n_chunks = P.n_chunks;
  const int total = (rt_end - rt_begin) * n_chunks;
  if (total <= 0) return;

  RowDesc<NPASS> rd;
  build_rowdesc<ST_KC, NPASS>(rd, g, tm, rows_used, tid);

  // this lane's frame
  const int fi_lane = wave * 32 + n;
  const bool valid = fi_lane < m_valid;
  const long long f_lane = f0 + fi_lane;
  const long long b_lane = valid ? f_lane / g.T : 0;
  const int t_lane = valid ? (int)(f_lane - b_lane * g.T) : 0;
  const int row_lane = valid ? tm.frame_row(fi_lane) : 0;
  const int a_off = row_lane * ST_PITCH + 4 * h;

  const int groups_per_rt = n_chunks * P.nj * ST_NKG;

  f32x16 acc[ST_RB];
#pragma unroll
  for (int rb = 0; rb < ST_RB; ++rb)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[rb][r] = 0.f;

  constexpr int NB = LIN ? LIN_NB : ST_MEL_BLOCKS;  // 32-row blocks of the second contraction's output
  f32x16 macc[MEL ? NB : 1];
  float nyq = 0.f;
  if constexpr (MEL) {
#pragma unroll
    for (int mb = 0; mb < NB; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) macc[mb][r] = 0.f;
  }
  // ---- prologue: chunk 0 into LDS buffer 0, chunk 1 requested, first RING bank groups requested --
  f32x4 R[NPASS];
  TileFix<NPASS> fx;
  issue_chunk<NPASS>(R, fx, g, rd, 0);
  wait_vm<0>(R);
  store_chunk<ST_KC, ST_PITCH, NPASS>(R, fx, lds[0], LDS_ROWS, tid);
  issue_chunk<NPASS>(R, fx, g, rd, (1 % n_chunks) * ST_KC);

  // The bank is streamed with scalar-base loads: `bank_s` is uniform, each lane adds its 16 bytes.
  const unsigned lane_off = (unsigned)lane * 16u;
  const char* bank_s = reinterpret_cast<const char*>(P.bank) + ((long long)rt_begin * groups_per_rt) * (ST_RB * 64 * 16);
  f32x4 bq[RING][ST_RB];
#pragma unroll
  for (int s = 0; s < RING; ++s) {
    gload16_s<0>(bq[s][0], lane_off, bank_s);
    gload16_s<1024>(bq[s][1], lane_off, bank_s);
    gload16_s<2048>(bq[s][2], lane_off, bank_s);
    gload16_s<3072>(bq[s][3], lane_off, bank_s);
    bank_s += ST_RB * 64 * 16;
  }
  __syncthreads();

  // Loads retire in order.  When a group starts, the requests younger than its own ring slot are
  // the other RING-1 slots (and, for some groups, the chunk tile: never counted, which is the
  // safe side).  The tile in R was requested in the second group of the previous chunk (or in the
  // prologue) and is followed by at least min(3, RING) whole slots.
  constexpr int W_SLOT = (RING - 1) * ST_RB;
  constexpr int W_TILE = (RING < 3 ? RING : 3) * ST_RB;
  constexpr int TASK_NONE = 0, TASK_STORE = 1, TASK_LOAD = 2;
  float* const stage_dst0 = &lds[0][0] + (tid / (ST_KC / 4)) * ST_PITCH + (tid % (ST_KC / 4)) * 4;

  int c = 0;            // chunk inside the current row tile
  int rt = rt_begin;
  const int nj = P.nj;
  for (int it = 0; it < total; ++it) {
    // R holds the tile of chunk it+1.  In the common case (every window interior) its LDS writes
    // and the requests for chunk it+2 are spread over the first two fragment groups below, one
    // instruction behind every other MFMA, so that they cost no MFMA issue time; only the address
    // arithmetic (and the rare edge handling) happens here.
    wait_vm<W_TILE>(R);
    const TileFix<NPASS> fx_store = fx;  // how to write the tile now in R; fx moves on to chunk it+2
    if (fx_store.cls == 2) store_chunk<ST_KC, ST_PITCH, NPASS>(R, fx_store, lds[(it + 1) & 1], LDS_ROWS, tid);
    const float* ptr[NPASS];
    prepare_chunk<NPASS>(ptr, fx, g, rd, ((it + 2) % n_chunks) * ST_KC);
    float* const stage_dst = stage_dst0 + ((it + 1) & 1) * (LDS_ROWS * ST_PITCH);
    __builtin_amdgcn_sched_barrier(0);

    const float* A = lds[it & 1] + a_off;
    f32x4 a_cur = *reinterpret_cast<const f32x4*>(A);

    auto group = [&](auto task_tag, int jj, auto kg_tag) {
      constexpr int TASK = decltype(task_tag)::value;
      constexpr int kg = decltype(kg_tag)::value;
      constexpr int s = kg % RING;
      // the frames fragment of the next group is read from LDS while this group's MFMAs run
      const int nxt = kg + 1 < ST_NKG ? jj * ST_PITCH + (kg + 1) * ST_KG : (jj + 1 < nj ? (jj + 1) * ST_PITCH : 0);
      const f32x4 a_nxt = *reinterpret_cast<const f32x4*>(A + nxt);
      wait_vm<W_SLOT>(bq[s][0], bq[s][1], bq[s][2], bq[s][3]);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // the LDS read goes first
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int m = 0; m < 16; ++m) {
        const int e = m >> 2, rb = m & 3;
        acc[rb] = __builtin_amdgcn_mfma_f32_32x32x2f32(bq[s][rb][e], a_cur[e], acc[rb], 0, 0, 0);
        if (TASK != TASK_NONE && (m & 1) && (m >> 1) < NPASS) {
          const int p = m >> 1;
          __builtin_amdgcn_sched_barrier(0);
          if (TASK == TASK_STORE) {
            if (fx_store.cls != 2)
              *reinterpret_cast<f32x4*>(stage_dst + p * ST_RPP * ST_PITCH) = fixed_up<NPASS>(R[p], fx_store, p);
          } else {
            gload16(R[p], ptr[p]);
          }
          __builtin_amdgcn_sched_barrier(0);
        }
        if (m >= 12) {
          // this MFMA was the last reader of fragment quad rb: re-request it (the group RING
          // ahead; the bank allocation is padded by ST_NKG groups, so the tail stays in bounds)
          __builtin_amdgcn_sched_barrier(0);
          if (rb == 0) gload16_s<0>(bq[s][0], lane_off, bank_s);
          if (rb == 1) gload16_s<1024>(bq[s][1], lane_off, bank_s);
          if (rb == 2) gload16_s<2048>(bq[s][2], lane_off, bank_s);
          if (rb == 3) gload16_s<3072>(bq[s][3], lane_off, bank_s);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      bank_s += ST_RB * 64 * 16;
      a_cur = a_nxt;
    };
    using K0 = std::integral_constant<int, 0>;
    using K1 = std::integral_constant<int, 1>;
    using K2 = std::integral_constant<int, 2>;
    using K3 = std::integral_constant<int, 3>;
    group(std::integral_constant<int, TASK_STORE>{}, 0, K0{});
    group(std::integral_constant<int, TASK_LOAD>{}, 0, K1{});
    group(std::integral_constant<int, TASK_NONE>{}, 0, K2{});
    group(std::integral_constant<int, TASK_NONE>{}, 0, K3{});
    for (int jj = 1; jj < nj; ++jj) {
      group(std::integral_constant<int, TASK_NONE>{}, jj, K0{});
      group(std::integral_constant<int, TASK_NONE>{}, jj, K1{});
      group(std::integral_constant<int, TASK_NONE>{}, jj, K2{});
      group(std::integral_constant<int, TASK_NONE>{}, jj, K3{});
    }

    if (++c == n_chunks) {
      // ---- epilogue of row tile rt ---------------------------------------------------
      c = 0;
      const int slot_base = rt * (ST_ROWS / 2);
      if constexpr (GRAD) {
        if (valid) {
          const float* __restrict__ gp = P.gout + (b_lane * P.out_bins) * g.T + t_lane;
          // G is stored in blocks of 32 frames: [frame / 32][packed row][frame % 32]
          float* __restrict__ Gp = P.gbuf + (f_lane >> 5) * ((long long)P.n_rt * ST_ROWS * 32) + (f_lane & 31);
          float* __restrict__ pp = P.pout ? P.pout + (b_lane * P.out_bins) * g.T + t_lane : nullptr;
          if (P.fmt == NNA_OUT_MAGNITUDE)
            stft_grad_tile<NNA_OUT_MAGNITUDE>(acc, gp, g.T, Gp, P.gpitch, slot_base, h, P.n_half, P.packed, pp);
          else if (P.fmt == NNA_OUT_POWER)
            stft_grad_tile<NNA_OUT_POWER>(acc, gp, g.T, Gp, P.gpitch, slot_base, h, P.n_half, P.packed, pp);
          else if (P.fmt == NNA_OUT_LOG)
            stft_grad_tile<NNA_OUT_LOG>(acc, gp, g.T, Gp, P.gpitch, slot_base, h, P.n_half, P.packed);
          else if (P.fmt == NNA_OUT_COMPLEX)
            stft_grad_tile<NNA_OUT_COMPLEX>(acc, gp, g.T, Gp, P.gpitch, slot_base, h, P.n_half, P.packed);
          else
            stft_grad_tile<NNA_OUT_PHASE>(acc, gp, g.T, Gp, P.gpitch, slot_base, h, P.n_half, P.packed);
        }
      } else if constexpr (CPLX) {
        if (valid) {
          float* __restrict__ op = P.out + (b_lane * P.out_bins) * g.T + t_lane;
          if (P.fmt == NNA_OUT_COMPLEX)
            stft_store_tile_complex<NNA_OUT_COMPLEX>(acc, op, g.T, slot_base, h, P.n_half, P.packed);
          else
            stft_store_tile_complex<NNA_OUT_PHASE>(acc, op, g.T, slot_base, h, P.n_half, P.packed);
        }
      } else if constexpr (!MEL) {
        if (valid) {
          float* __restrict__ op = P.out + (b_lane * P.out_bins) * g.T + t_lane;
          if (P.fmt == NNA_OUT_MAGNITUDE)
            stft_store_tile<NNA_OUT_MAGNITUDE>(acc, op, g.T, slot_base, h, P.n_half, P.packed);
          else if (P.fmt == NNA_OUT_POWER)
            stft_store_tile<NNA_OUT_POWER>(acc, op, g.T, slot_base, h, P.n_half, P.packed);
          else
            stft_store_tile<NNA_OUT_LOG>(acc, op, g.T, slot_base, h, P.n_half, P.packed);
        }
      } else {
        const unsigned char* __restrict__ maskp = P.mel_mask + ((long long)pass * P.n_rt + rt) * ST_RB;
        if constexpr (LIN) {
          // Accumulator register r of lane (h, n) is packed row 32 rb + 8 (r/4) + 4 h + r%4 of the row
          // tile for frame n: as the B operand of MFMA number r it meets, in lane (h, m), the weight
          // of output row m for that packed row.  16 MFMAs contract the 32 rows of block rb.
          const float4* __restrict__ wp =
              P.melw + (((long long)pass * P.n_rt + rt) * ST_RB) * (NB * 4 * 64) + lane;
#pragma unroll
          for (int rb = 0; rb < ST_RB; ++rb) {
            const unsigned mask = maskp[rb];
#pragma unroll
            for (int mb = 0; mb < NB; ++mb) {
              if (mask & (1u << mb)) {
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                  const float4 w = wp[((rb * NB + mb) * 4 + v) * 64];
                  macc[mb] = __builtin_amdgcn_mfma_f32_32x32x2f32(w.x, acc[rb][4 * v + 0], macc[mb], 0, 0, 0);
                  macc[mb] = __builtin_amdgcn_mfma_f32_32x32x2f32(w.y, acc[rb][4 * v + 1], macc[mb], 0, 0, 0);
                  macc[mb] = __builtin_amdgcn_mfma_f32_32x32x2f32(w.z, acc[rb][4 * v + 2], macc[mb], 0, 0, 0);
                  macc[mb] = __builtin_amdgcn_mfma_f32_32x32x2f32(w.w, acc[rb][4 * v + 3], macc[mb], 0, 0, 0);
                }
              }
            }
          }
        } else {
        if constexpr (SPEC) {
          if (valid && pass == 0) {
            float* __restrict__ sp = P.pout + (b_lane * (P.n_half + 1)) * g.T + t_lane;
            if (P.fmt == 1)
              stft_store_tile<NNA_OUT_MAGNITUDE>(acc, sp, g.T, slot_base, h, P.n_half, P.packed);
            else
              stft_store_tile<NNA_OUT_POWER>(acc, sp, g.T, slot_base, h, P.n_half, P.packed);
          }
        }
        const float4* __restrict__ wp =
            P.melw + (((long long)pass * P.n_rt + rt) * ST_RB) * (ST_MEL_BLOCKS * 2 * 64) + lane;
#pragma unroll
        for (int rb = 0; rb < ST_RB; ++rb) {
          float pw[8];
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            const float re = acc[rb][2 * u], im = acc[rb][2 * u + 1];
            float v = re * re + im * im;
            if (rb == 0 && u == 0 && h == 0 && slot_base == 0) {  // DC / Nyquist slot
              v = re * re;
              nyq = im * im;
              if (P.fmt == 1) nyq = __builtin_amdgcn_sqrtf(nyq);
            }
            pw[u] = P.fmt == 1 ? __builtin_amdgcn_sqrtf(v) : v;
          }
          const unsigned mask = maskp[rb];
#pragma unroll
          for (int mb = 0; mb < ST_MEL_BLOCKS; ++mb) {
            if (mask & (1u << mb)) {
              const float4 w0 = wp[((rb * ST_MEL_BLOCKS + mb) * 2 + 0) * 64];
              const float4 w1 = wp[((rb * ST_MEL_BLOCKS + mb) * 2 + 1) * 64];
              macc[mb] = __builtin_amdgcn_mfma_f32_32x32x2f32(w0.x, pw[0], macc[mb], 0, 0, 0);
              macc[mb] = __builtin_amdgcn_mfma_f32_32x32x2f32(w0.y, pw[1], macc[mb], 0, 0, 0);
              macc[mb] = __builtin_amdgcn_mfma_f32_32x32x2f32(w0.z, pw[2], macc[mb], 0, 0, 0);
              macc[mb] = __builtin_amdgcn_mfma_f32_32x32x2f32(w0.w, pw[3], macc[mb], 0, 0, 0);
              macc[mb] = __builtin_amdgcn_mfma_f32_32x32x2f32(w1.x, pw[4], macc[mb], 0, 0, 0);
              macc[mb] = __builtin_amdgcn_mfma_f32_32x32x2f32(w1.y, pw[5], macc[mb], 0, 0, 0);
              macc[mb] = __builtin_amdgcn_mfma_f32_32x32x2f32(w1.z, pw[6], macc[mb], 0, 0, 0);
              macc[mb] = __builtin_amdgcn_mfma_f32_32x32x2f32(w1.w, pw[7], macc[mb], 0, 0, 0);
            }
          }
        }
        }
      }
#pragma unroll
      for (int rb = 0; rb < ST_RB; ++rb)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[rb][r] = 0.f;
      ++rt;
    }
    __syncthreads();
  }

  // Drain: the last tile request and the last RING bank requests are never consumed.  Their
  // destination registers must stay reserved until the data has landed -- a register the
  // compiler reuses while a load into it is in flight would be overwritten behind its back.
  wait_vm<0>(R);
#pragma unroll
  for (int s = 0; s < RING; ++s) wait_vm<0>(bq[s][0], bq[s][1], bq[s][2], bq[s][3]);

  if constexpr (LIN) {
    // output rows 2q, 2q+1 = (Re, Im) of complex bin q sit in adjacent registers of one lane
    float* __restrict__ op = P.out + b_lane * P.out_wave_stride + (long long)P.row_offset * g.T + t_lane;
    const int f = P.fmt;
#pragma unroll
    for (int mb = 0; mb < NB; ++mb) {
#pragma unroll
      for (int r = 0; r < 16; r += 2) {
        const int bin = (pass * (32 * NB) + mb * 32 + 8 * (r >> 2) + 4 * h + (r & 3)) >> 1;
        if (valid && bin < P.out_bins) {
          if (f == NNA_OUT_COMPLEX) {  // rows 2q = Re, 2q+1 = Im
            op[(2LL * bin) * g.T] = macc[mb][r];
            op[(2LL * bin + 1) * g.T] = macc[mb][r + 1];
            continue;
          }
          if (f == NNA_OUT_PHASE) {
            op[(long long)bin * g.T] = atan2f(macc[mb][r + 1], macc[mb][r]);
            continue;
          }
          const float pw = macc[mb][r] * macc[mb][r] + macc[mb][r + 1] * macc[mb][r + 1];
          op[(long long)bin * g.T] = f == NNA_OUT_MAGNITUDE ? format_power<NNA_OUT_MAGNITUDE>(pw)
                                     : f == NNA_OUT_POWER   ? pw
                                                            : format_power<NNA_OUT_LOG>(pw);
        }
      }
    }
  } else if constexpr (MEL) {
    // Nyquist-bin term (its power lives in lane n of the first lane half) and the store.
    float nyq_n = 0.f;
    if (P.mel_nyq_any) nyq_n = __shfl(nyq, n, 64);
    float* __restrict__ op = P.out + (b_lane * P.n_mels) * g.T + t_lane;
#pragma unroll
    for (int mb = 0; mb < ST_MEL_BLOCKS; ++mb) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int mel = pass * (32 * ST_MEL_BLOCKS) + mb * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
        if (valid && mel < P.n_mels) {
          float v = macc[mb][r];
          if (P.mel_nyq_any) v += P.mel_wnyq[mel] * nyq_n;
          op[(long long)mel * g.T] = v;
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------------------
// CQT kernel.
// Workgroup = 4 waves, one 16-row bank block (8 bins, Re/Im interleaved) x 256 frames; wave w
// owns frames [64w, 64w+64) as 4 blocks of 16 (v_mfma_f32_16x16x4_f32).  Accumulator register
// r of lane l = (q = l/16, n = l%16) holds row 4q + r of frame n: bin 2q in r = 0,1 and bin
// 2q+1 in r = 2,3.  Only the taps inside the block's longest kernel are visited: per LDS chunk
// the planner lists the hop-shifts [jlo, jlo+nj) that hold non-zero taps.
// ---------------------------------------------------------------------------------------
constexpr int CQ_RPP = 256 / (CQ_KC / 4);            // LDS rows written per loader pass (64)
constexpr int CQ_NPASS = CQ_LDS_ROWS_MAX / CQ_RPP;  // 512 / 64 = 8

// fn(integral_constant<int, 0>), fn(integral_constant<int, 1>), ...: a loop whose index is a compile-time constant
template <typename F, int... S>
__device__ __forceinline__ void for_each_index(F&& fn, std::integer_sequence<int, S...>) {
  (fn(std::integral_constant<int, S>{}), ...);
}

// GRAD: instead of the spectrogram the kernel writes G = dLoss/dC, the derivative of the output format
// applied to the upstream gradient, in the blocked layout the backward contractions read.
template <bool GRAD>
__global__ __launch_bounds__(256, 2) void cqt_kernel(const CqtParams P) {
  extern __shared__ __attribute__((aligned(16))) float dyn_lds[];
  // dynamic LDS: this item's chunk table (read every chunk; kept out of the vector-memory path so
  // that fetching a descriptor never waits on the streaming loads), then two tile buffers
  // A table longer than CQ_TABLE_CAP chunks (kernels of tens of thousands of taps whose frames do not
  // share LDS rows) is kept as a ring of CQ_TABLE_CAP entries, refilled half a ring at a time.
  int4* s_chunks = reinterpret_cast<int4*>(dyn_lds);
  const int tbl_n = P.n_chunks < CQ_TABLE_CAP ? P.n_chunks : CQ_TABLE_CAP;  // entries held in LDS
  const int tbl_mask = P.n_chunks <= CQ_TABLE_CAP ? 0x7fffffff : CQ_TABLE_CAP - 1;
  float* lds0 = dyn_lds + (size_t)tbl_n * (sizeof(CqtChunk) / 4);
  float* lds1 = lds0 + (size_t)P.lds_rows * CQ_PITCH;

  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int q = lane >> 4, n = lane & 15;

  // longest kernels first: the work item is the slow index
  const long long bid = blockIdx.x;
  const int item_id = (int)(bid / P.n_ft);
  const long long ft = bid - (long long)item_id * P.n_ft;
  const CqtItem item = P.items[item_id];
  const int n_rb = item.n_rb;

  const FrameGeom& g = P.g;
  const long long f0 = ft * P.tile_frames;
  const int m_valid = (int)((g.n_frames - f0) < P.tile_frames ? (g.n_frames - f0) : P.tile_frames);
  TileMap tm;
  tm.T = g.T;
  tm.b0 = f0 / g.T;
  tm.t0 = (int)(f0 - tm.b0 * g.T);
  tm.n0 = (g.T - tm.t0) < m_valid ? (g.T - tm.t0) : m_valid;
  const int row_pitch = P.row_step * CQ_PITCH;  // floats between the LDS rows of consecutive shifts
  tm.extra = (item.jspan - 1) * P.row_step;
  const int rows_used = tm.frame_row(m_valid - 1) + tm.extra + 1;
  RowDesc<CQ_NPASS> rd;
  build_rowdesc<CQ_KC, CQ_NPASS>(rd, g, tm, rows_used, tid);

  bool valid[4];
  int a_off[4];
  long long o_off[4];
#pragma unroll
  for (int fb = 0; fb < 4; ++fb) {
    const int fi = wave * 64 + fb * 16 + n;
    valid[fb] = fi < m_valid;
    const long long f = f0 + fi;
    const long long b = valid[fb] ? f / g.T : 0;
    const int t = valid[fb] ? (int)(f - b * g.T) : 0;
    a_off[fb] = (valid[fb] ? tm.frame_row(fi) : 0) * CQ_PITCH + 4 * q;
    o_off[fb] = b * P.out_wave_stride + (long long)P.row_offset * g.T + t;
  }

  const int n_chunks = item.n_chunks;  // >= 1; every listed chunk starts with >= CQ_PREFETCH fragments
  const int4* __restrict__ tbl_src = reinterpret_cast<const int4*>(P.chunks + (long long)item_id * P.n_chunks);
  for (int i = tid; i < (n_chunks < tbl_n ? n_chunks : tbl_n) * 3; i += 256) s_chunks[i] = tbl_src[i];
  // the bank fragments are streamed with scalar-base loads: uniform base + 16 bytes per lane
  const unsigned lane_off = (unsigned)lane * 16u;
  const char* bank_s = reinterpret_cast<const char*>(P.bank) + item.frag0 * (64 * 16);

  f32x4 acc[CQ_ITEM_RB][4];
#pragma unroll
  for (int r = 0; r < CQ_ITEM_RB; ++r)
#pragma unroll
    for (int fb = 0; fb < 4; ++fb) acc[r][fb] = (f32x4){0.f, 0.f, 0.f, 0.f};
  __syncthreads();  // the chunk table is complete

  auto chunk_shift = [&](int i) {  // (first hop-shift) * hop + (first column) of chunk i
    const int4 v = s_chunks[3 * (i & tbl_mask)];
    return __builtin_amdgcn_readfirstlane(v.y) * P.tap_stride + __builtin_amdgcn_readfirstlane(v.x);
  };

  f32x4 R[CQ_NPASS];
  TileFix<CQ_NPASS> fx;
  issue_chunk<CQ_NPASS>(R, fx, g, rd, chunk_shift(0));
  wait_vm<0>(R);
  store_chunk<CQ_KC, CQ_PITCH, CQ_NPASS>(R, fx, lds0, P.lds_rows, tid);
  issue_chunk<CQ_NPASS>(R, fx, g, rd, chunk_shift(n_chunks > 1 ? 1 : 0));
  // bank fragment pipeline: CQ_PREFETCH requests in flight (the allocation is padded by that many)
  f32x4 bq[CQ_PREFETCH];
#pragma unroll
  for (int i = 0; i < CQ_PREFETCH; ++i) {
    gload16_s<0>(bq[i], lane_off, bank_s);
    bank_s += 64 * 16;
  }
  __syncthreads();

  // Loads retire in order.  When a group starts, the requests younger than its own fragment are
  // the other CQ_PREFETCH-1 fragments (the chunk tile is never counted: the safe side).  The tile
  // in R was requested in the second group of the previous chunk (or in the prologue) and is
  // followed by at least CQ_PREFETCH-1 fragment requests (every chunk has >= CQ_PREFETCH groups).
  constexpr int W_SLOT = CQ_PREFETCH - 1;
  constexpr int W_TILE = CQ_PREFETCH - 1;
  constexpr int TASK_NONE = 0, TASK_STORE = 1, TASK_LOAD = 2;
  const int stage_off = (tid / (CQ_KC / 4)) * CQ_PITCH + (tid % (CQ_KC / 4)) * 4;
  const int n_pass_rows = (P.lds_rows + CQ_RPP - 1) / CQ_RPP;  // loader passes that have LDS rows

  for (int it = 0; it < n_chunks; ++it) {
    float* cur = (it & 1) ? lds1 : lds0;
    float* nxt = (it & 1) ? lds0 : lds1;
    // R holds the tile of chunk it+1.  In the common case its LDS writes and the requests for
    // chunk it+2 are spread over the first two fragment groups (one instruction behind every other
    // MFMA); only the address arithmetic and the rare edge handling happen here.
    wait_vm<W_TILE>(R);
    const TileFix<CQ_NPASS> fx_store = fx;  // how to write the tile now in R; fx moves on to chunk it+2
    if (fx_store.cls == 2) store_chunk<CQ_KC, CQ_PITCH, CQ_NPASS>(R, fx_store, nxt, P.lds_rows, tid);
    const float* ptr[CQ_NPASS];
    prepare_chunk<CQ_NPASS>(ptr, fx, g, rd, chunk_shift(it + 2 < n_chunks ? it + 2 : n_chunks - 1));
    float* const stage_dst = nxt + stage_off;
    // this chunk: per row block r of the item, nj[r] fragments starting joff[r] hop-shifts in
    const int4 d1 = s_chunks[3 * (it & tbl_mask) + 1], d2 = s_chunks[3 * (it & tbl_mask) + 2];
    const int joff[CQ_ITEM_RB] = {__builtin_amdgcn_readfirstlane(d1.x), __builtin_amdgcn_readfirstlane(d1.y),
                                  __builtin_amdgcn_readfirstlane(d1.z), __builtin_amdgcn_readfirstlane(d1.w)};
    const int njr[CQ_ITEM_RB] = {__builtin_amdgcn_readfirstlane(d2.x), __builtin_amdgcn_readfirstlane(d2.y),
                                 __builtin_amdgcn_readfirstlane(d2.z), __builtin_amdgcn_readfirstlane(d2.w)};
    __builtin_amdgcn_sched_barrier(0);

    // One fragment group: 16 taps, 16 MFMAs on the accumulators of row block R_.  `slot` is the
    // ring register that holds this group's bank fragment; it is a compile-time constant because
    // a register with a load in flight must never be copied.  The planner pads every row block's
    // share of a chunk to a multiple of CQ_PREFETCH fragments (zero fragments), so the slots stay
    // aligned: group jj always lives in slot jj % CQ_PREFETCH.  A padding group (`run` false) keeps
    // the ring's rhythm -- it waits for its slot and requests the slot's next fragment -- but
    // issues no MFMA.  The wait and the request stay outside the branch: each ring register is
    // written by one and the same instruction on every path.
    f32x4 a_cur[4];
    auto group = [&](auto rb_tag, auto task_tag, auto slot_tag, const float* base, int jj, int nj, bool run) {
      constexpr int R_ = decltype(rb_tag)::value;
      constexpr int TASK = decltype(task_tag)::value;
      constexpr int slot = decltype(slot_tag)::value;
      const int nxt_off = jj + 1 < nj ? (jj + 1) * row_pitch : 0;
      f32x4 a_nxt[4];
#pragma unroll
      for (int fb = 0; fb < 4; ++fb) a_nxt[fb] = *reinterpret_cast<const f32x4*>(base + a_off[fb] + nxt_off);
      wait_vm<W_SLOT>(bq[slot]);
      __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);  // the 4 LDS reads go first
      __builtin_amdgcn_sched_barrier(0);
      if (TASK != TASK_NONE || run) {
#pragma unroll
        for (int m = 0; m < 16; ++m) {
          const int e = m >> 2, fb = m & 3;
          acc[R_][fb] = __builtin_amdgcn_mfma_f32_16x16x4f32(bq[slot][e], a_cur[fb][e], acc[R_][fb], 0, 0, 0);
          if (TASK != TASK_NONE && (m & 1)) {
            const int p = m >> 1;  // 0..7 = CQ_NPASS passes
            __builtin_amdgcn_sched_barrier(0);
            if (TASK == TASK_STORE) {
              if (fx_store.cls != 2 && p < n_pass_rows)
                *reinterpret_cast<f32x4*>(stage_dst + p * CQ_RPP * CQ_PITCH) = fixed_up<CQ_NPASS>(R[p], fx_store, p);
            } else {
              gload16(R[p], ptr[p]);
            }
            __builtin_amdgcn_sched_barrier(0);
          }
        }
      }
      __builtin_amdgcn_sched_barrier(0);
      gload16_s<0>(bq[slot], lane_off, bank_s);
      bank_s += 64 * 16;
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int fb = 0; fb < 4; ++fb) a_cur[fb] = a_nxt[fb];
    };
    static_assert(CQ_PREFETCH >= 2 && CQ_NPASS == 8 && CQ_ITEM_RB == 4, "the group sequences below assume these");
    using TNone = std::integral_constant<int, TASK_NONE>;
    using TStore = std::integral_constant<int, TASK_STORE>;
    using TLoad = std::integral_constant<int, TASK_LOAD>;
    // all fragment groups of row block R_ in this chunk: nj of them, the first nr real, the rest
    // padding; the item's first row block (always present, >= one ring of groups) carries the staging tasks in
    // its first two groups
    auto row_block = [&](auto rb_tag) {
      constexpr int R_ = decltype(rb_tag)::value;
      const int nj = njr[R_] & 0xffff, nr = njr[R_] >> 16;
      if (R_ >= n_rb || nj == 0) return;
      const float* base = cur + joff[R_] * row_pitch;
#pragma unroll
      for (int fb = 0; fb < 4; ++fb) a_cur[fb] = *reinterpret_cast<const f32x4*>(base + a_off[fb]);
      // the ring's slots in order, each with its compile-time index
      auto ring = [&](auto&& fn) { for_each_index(fn, std::make_integer_sequence<int, CQ_PREFETCH>{}); };
      int jj = 0;
      if (R_ == 0) {
        ring([&](auto s) {
          constexpr int S = decltype(s)::value;
          if constexpr (S == 0)
            group(rb_tag, TStore{}, s, base, 0, nj, true);
          else if constexpr (S == 1)
            group(rb_tag, TLoad{}, s, base, 1, nj, true);
          else
            group(rb_tag, TNone{}, s, base, S, nj, S < nr);
        });
        jj = CQ_PREFETCH;
      }
      for (; jj + CQ_PREFETCH <= nr; jj += CQ_PREFETCH)
        ring([&](auto s) { group(rb_tag, TNone{}, s, base, jj + decltype(s)::value, nj, true); });
      if (jj < nj)  // the last ring: some real groups, then padding
        ring([&](auto s) { group(rb_tag, TNone{}, s, base, jj + decltype(s)::value, nj, jj + decltype(s)::value < nr); });
    };
    row_block(std::integral_constant<int, 0>{});
    row_block(std::integral_constant<int, 1>{});
    row_block(std::integral_constant<int, 2>{});
    row_block(std::integral_constant<int, 3>{});
    // Ring refill: every wave is inside iteration `it` (the barrier below separates iterations) and reads
    // entries it .. it+2 only, so entries [it - CAP/2, it) are dead; their slots take entries
    // [it + CAP/2, it + CAP), first read CAP/2 - 2 iterations from now.
    if (tbl_mask != 0x7fffffff && it >= CQ_TABLE_CAP / 2 && (it & (CQ_TABLE_CAP / 2 - 1)) == 0) {
      const int first = it + CQ_TABLE_CAP / 2;
      int count = n_chunks - first;
      count = count < CQ_TABLE_CAP / 2 ? count : CQ_TABLE_CAP / 2;
      for (int i = tid; i < count * 3; i += 256) s_chunks[3 * (first & tbl_mask) + i] = tbl_src[3 * first + i];
    }
    __syncthreads();
  }

  // drain the requests that are never consumed (see the STFT kernel)
  wait_vm<0>(R);
#pragma unroll
  for (int i = 0; i < CQ_PREFETCH; ++i) wait_vm<0>(bq[i]);

  const int f = P.fmt;
  if constexpr (GRAD) {
    // lane (q, n), registers 0..3 of row block rb: (Re, Im) of bins 8 rb + 2 q and + 1, frame n of the
    // wave's frame block fb.  G[frame / 32][row][frame % 32], row = 2 bin (Re), 2 bin + 1 (Im).
#pragma unroll
    for (int fb = 0; fb < 4; ++fb) {
      if (!valid[fb]) continue;
      const long long fr = f0 + wave * 64 + fb * 16 + n;
      const long long b = fr / g.T;
      const float* __restrict__ gp = P.gout + b * P.gout_wave_stride + (fr - b * g.T);
      float* __restrict__ Gp = P.gbuf + (fr >> 5) * ((long long)P.rows_pad * 32) + (fr & 31);
#pragma unroll
      for (int r = 0; r < CQ_ITEM_RB; ++r) {
        if (r >= n_rb) continue;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const int bin = (item.rb_first + r) * (CQ_ROWS / 2) + 2 * q + u;
          if (bin >= P.n_bins) continue;
          const float re = acc[r][fb][2 * u], im = acc[r][fb][2 * u + 1];
          const float pw = re * re + im * im;
          float gr, gi;
          if (f == NNA_OUT_COMPLEX) {
            gr = gp[(2LL * bin) * g.T];
            gi = gp[(2LL * bin + 1) * g.T];
          } else if (f == NNA_OUT_PHASE) {  // d atan2(Im, Re) = (Re dIm - Im dRe) / P
            const float s = pw > 0.f ? gp[(long long)bin * g.T] / pw : 0.f;
            gr = -s * im;
            gi = s * re;
          } else {
            const float go = gp[(long long)bin * g.T];
            const float s = f == NNA_OUT_MAGNITUDE ? grad_scale<NNA_OUT_MAGNITUDE>(go, pw)
                            : f == NNA_OUT_POWER   ? grad_scale<NNA_OUT_POWER>(go, pw)
                                                   : grad_scale<NNA_OUT_LOG>(go, pw);
            gr = s * re;
            gi = s * im;
          }
          Gp[(2LL * bin) * 32] = gr;
          Gp[(2LL * bin + 1) * 32] = gi;
        }
      }
    }
    return;
  }
#pragma unroll
  for (int r = 0; r < CQ_ITEM_RB; ++r) {
    if (r >= n_rb) continue;
    const int bin0 = (item.rb_first + r) * (CQ_ROWS / 2) + 2 * q;
#pragma unroll
    for (int fb = 0; fb < 4; ++fb) {
      if (!valid[fb]) continue;
      float* __restrict__ op = P.out + o_off[fb];
      if (f == NNA_OUT_COMPLEX) {  // rows 2k = Re, 2k+1 = Im of bin k
        if (bin0 < P.n_bins) {
          op[(2LL * bin0) * g.T] = acc[r][fb][0];
          op[(2LL * bin0 + 1) * g.T] = acc[r][fb][1];
        }
        if (bin0 + 1 < P.n_bins) {
          op[(2LL * bin0 + 2) * g.T] = acc[r][fb][2];
          op[(2LL * bin0 + 3) * g.T] = acc[r][fb][3];
        }
        continue;
      }
      if (f == NNA_OUT_PHASE) {
        if (bin0 < P.n_bins) op[(long long)bin0 * g.T] = atan2f(acc[r][fb][1], acc[r][fb][0]);
        if (bin0 + 1 < P.n_bins) op[(long long)(bin0 + 1) * g.T] = atan2f(acc[r][fb][3], acc[r][fb][2]);
        continue;
      }
      const float p0 = acc[r][fb][0] * acc[r][fb][0] + acc[r][fb][1] * acc[r][fb][1];
      const float p1 = acc[r][fb][2] * acc[r][fb][2] + acc[r][fb][3] * acc[r][fb][3];
      if (bin0 < P.n_bins)
        op[(long long)bin0 * g.T] = f == NNA_OUT_MAGNITUDE ? format_power<NNA_OUT_MAGNITUDE>(p0)
                                    : f == NNA_OUT_POWER   ? p0
                                                           : format_power<NNA_OUT_LOG>(p0);
      if (bin0 + 1 < P.n_bins)
        op[(long long)(bin0 + 1) * g.T] = f == NNA_OUT_MAGNITUDE ? format_power<NNA_OUT_MAGNITUDE>(p1)
                                          : f == NNA_OUT_POWER   ? p1
                                                                 : format_power<NNA_OUT_LOG>(p1);
    }
  }
}

// ---------------------------------------------------------------------------------------
// Decimation by two (Sec. III-C, "Downsampling"): y[m] = sum_i h[i] x~[2 m + i - half], x~ the waveform
// mirrored at both ends.  Bound by the waveform it streams, so it runs on the vector ALUs: the input is split
// into its even and odd samples on the way to LDS, xe[i] = x~[s0 + 2 i], xo[i] = x~[s0 + 2 i + 1], and
//     y[m] = sum_v he[v] xe[m + v] + sum_v ho[v] xo[m + v],   he[v] = h[half + 2 v], ho[v] = h[half + 2 v + 1],
// two plain filters.  A half-band design has a single non-zero he (its centre tap).  A thread produces eight
// consecutive outputs from a window of samples that slides through registers: one LDS read per eight
// multiply-adds.
// ---------------------------------------------------------------------------------------
// LDS position of sample i of a stream: one float of padding per eight, so that the threads of a wave, whose
// windows start eight samples apart, read from different banks (stride 9)
__device__ __forceinline__ int fir_pos(int i) { return i + (i >> 3); }

// acc[i] += sum_k taps[k] w[off + i + k]; `wt` points at this thread's first window position for off = 0
__device__ __forceinline__ void fir_stream(float (&acc)[FIR_T], const float* __restrict__ wt, int off, const float* __restrict__ taps, int n) {
  float win[2 * FIR_T];
#pragma unroll
  for (int i = 0; i < FIR_T; ++i) win[i] = wt[fir_pos(off + i)];
  for (int k0 = 0; k0 < n; k0 += FIR_T) {  // taps are zero padded to a multiple of eight
#pragma unroll
    for (int i = 0; i < FIR_T; ++i) win[FIR_T + i] = wt[fir_pos(off + k0 + FIR_T + i)];
#pragma unroll
    for (int kk = 0; kk < FIR_T; ++kk) {
      const float t = taps[k0 + kk];
#pragma unroll
      for (int i = 0; i < FIR_T; ++i) acc[i] += t * win[i + kk];
    }
#pragma unroll
    for (int i = 0; i < FIR_T; ++i) win[i] = win[i + FIR_T];
  }
}

__global__ __launch_bounds__(256) void fir_decimate_kernel(const FirParams P) {
  extern __shared__ __attribute__((aligned(16))) float fir_lds[];
  const int tid = threadIdx.x;
  const long long b = blockIdx.y;
  const long long m0 = (long long)blockIdx.x * FIR_TILE;
  const int vmin = P.ve0 < P.vo0 ? P.ve0 : P.vo0;
  const int vend = P.ve0 + P.ne > P.vo0 + P.no ? P.ve0 + P.ne : P.vo0 + P.no;  // taps zero padded: ne, no multiples of 8
  const int n_l = FIR_TILE + (vend - vmin) + 8;  // samples of each stream this workgroup needs
  float* xe = fir_lds;
  float* xo = fir_lds + P.lds_stream;
  const float* __restrict__ xb = P.x + b * P.L;
  const long long s0 = 2 * (m0 + vmin);
  const int L = (int)P.L;
  // sample pairs in batches of four per thread, so that four loads are out before the first is written to LDS
  for (int i0 = tid; i0 < n_l; i0 += 4 * 256) {
    float2 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int i = i0 + 256 * u;
      const long long idx = s0 + 2LL * i;
      v[u] = make_float2(0.f, 0.f);
      if (i >= n_l) continue;
      if (P.vec2 && idx >= 0 && idx + 1 < P.L) {
        v[u] = *reinterpret_cast<const float2*>(xb + idx);
      } else {
        // past either end: the mirror image (far beyond it, where only padding taps reach: any sample)
        const long long lo = -(long long)L, hi = 2LL * L;
        const int ic = (int)(idx < lo ? lo : idx > hi ? hi : idx);
        v[u] = make_float2(xb[reflect_clamped(ic, L)], xb[reflect_clamped(ic + 1, L)]);
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int i = i0 + 256 * u;
      if (i < n_l) {
        xe[fir_pos(i)] = v[u].x;
        xo[fir_pos(i)] = v[u].y;
      }
    }
  }
  __syncthreads();
  const int j8 = tid * FIR_T;
  if (m0 + j8 >= P.Ln) return;
  float acc[FIR_T];
#pragma unroll
  for (int i = 0; i < FIR_T; ++i) acc[i] = 0.f;
  // sample j8 + x sits at position 9 tid + fir_pos(x) (j8 = 8 tid)
  fir_stream(acc, xe + 9 * tid, P.ve0 - vmin, P.he, P.ne);
  fir_stream(acc, xo + 9 * tid, P.vo0 - vmin, P.ho, P.no);
  float* __restrict__ op = P.y + b * P.Ln + m0 + j8;
  if (P.vec4_out && m0 + j8 + FIR_T <= P.Ln) {
    *reinterpret_cast<f32x4*>(op) = (f32x4){acc[0], acc[1], acc[2], acc[3]};
    *reinterpret_cast<f32x4*>(op + 4) = (f32x4){acc[4], acc[5], acc[6], acc[7]};
  } else {
#pragma unroll
    for (int i = 0; i < FIR_T; ++i)
      if (m0 + j8 + i < P.Ln) op[i] = acc[i];
  }
}

// ---------------------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------------------
// LDS per workgroup is 160 KB
static constexpr size_t CQ_DYN_LDS_MAX = 160 * 1024;

size_t cqt_launch_lds_bytes(int n_chunks, int lds_rows) {
  const int tbl_n = n_chunks < CQ_TABLE_CAP ? n_chunks : CQ_TABLE_CAP;
  return (size_t)tbl_n * sizeof(CqtChunk) + 2ull * lds_rows * CQ_PITCH * sizeof(float);
}

hipError_t kernels_init() {
  const void* kernels[] = {reinterpret_cast<const void*>(cqt_kernel<false>), reinterpret_cast<const void*>(cqt_kernel<true>)};
  for (const void* k : kernels) {
    const hipError_t e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)CQ_DYN_LDS_MAX);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t launch_stft(const StftParams& p, int mode, hipStream_t stream) {
  clear_stale_error();
  long long blocks;
  const bool mel = mode == ST_MODE_MEL || mode == ST_MODE_LIN || mode == ST_MODE_MELSPEC;
  if (mode == ST_MODE_MELSPEC && !p.pout) return hipErrorInvalidValue;
  if (mel) {
    blocks = p.n_ft * p.n_pass;
  } else {
    const long long ft_per_xcd = (p.n_ft + 7) / 8;
    const long long groups = (ft_per_xcd + 63) / 64;
    blocks = 8 * groups * 64 * ((p.n_rt + ST_RG - 1) / ST_RG);
  }
  if (blocks <= 0 || blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  if (mode == ST_MODE_LIN)
    // six output blocks (a pass saved when 128 < output rows <= 192 ...): their registers come out of the ring
    if (p.lin_blocks == 6)
      hipLaunchKernelGGL((stft_kernel<ST_MODE_LIN, ST_RING_STFT, 6>), dim3((unsigned)blocks), dim3(256), 0, stream, p);
    else
      hipLaunchKernelGGL((stft_kernel<ST_MODE_LIN, ST_RING_MEL, 4>), dim3((unsigned)blocks), dim3(256), 0, stream, p);
  else if (mode == ST_MODE_MEL)
    hipLaunchKernelGGL((stft_kernel<ST_MODE_MEL, ST_RING_MEL>), dim3((unsigned)blocks), dim3(256), 0, stream, p);
  else if (mode == ST_MODE_MELSPEC)
    hipLaunchKernelGGL((stft_kernel<ST_MODE_MELSPEC, ST_RING_MEL>), dim3((unsigned)blocks), dim3(256), 0, stream, p);
  else if (mode == ST_MODE_GRAD)
    hipLaunchKernelGGL((stft_kernel<ST_MODE_GRAD, ST_RING_STFT>), dim3((unsigned)blocks), dim3(256), 0, stream, p);
  else if (mode == ST_MODE_CPLX)
    // (many hop-shifts: the 192-row tile of the one-workgroup-per-CU instantiation keeps the frame tile whole)
    if (p.wide)
      hipLaunchKernelGGL((stft_kernel<ST_MODE_CPLX, ST_RING_STFT, 6>), dim3((unsigned)blocks), dim3(256), 0, stream, p);
    else
      hipLaunchKernelGGL((stft_kernel<ST_MODE_CPLX, ST_RING_STFT>), dim3((unsigned)blocks), dim3(256), 0, stream, p);
  else
    hipLaunchKernelGGL((stft_kernel<ST_MODE_STFT, ST_RING_STFT>), dim3((unsigned)blocks), dim3(256), 0, stream, p);
  return hipGetLastError();
}

hipError_t launch_fir_decimate(const FirParams& p, hipStream_t stream) {
  clear_stale_error();
  const long long tiles = (p.Ln + FIR_TILE - 1) / FIR_TILE;
  if (tiles < 1 || tiles > 0x7fffffffLL || p.B < 1 || p.B > 65535 || p.L > 0x3fffffffLL) return hipErrorInvalidValue;
  if ((p.ne & 7) || (p.no & 7) || p.lds_stream < (FIR_TILE + 8) * 9 / 8) return hipErrorInvalidValue;
  const size_t lds = 2ull * p.lds_stream * sizeof(float);
  if (lds > 64 * 1024) return hipErrorInvalidValue;
  hipLaunchKernelGGL(fir_decimate_kernel, dim3((unsigned)tiles, (unsigned)p.B), dim3(256), lds, stream, p);
  return hipGetLastError();
}

hipError_t launch_cqt(const CqtParams& p, hipStream_t stream) {
  clear_stale_error();
  const long long blocks = p.n_ft * p.n_items;
  if (blocks <= 0 || blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  if (p.lds_rows > CQ_LDS_ROWS_MAX || p.row_step < 1) return hipErrorInvalidValue;
  const size_t lds = cqt_launch_lds_bytes(p.n_chunks, p.lds_rows);
  if (lds > CQ_DYN_LDS_MAX) return hipErrorInvalidValue;
  if (p.gbuf) {
    if (!p.gout || p.rows_pad < 2 * p.n_bins) return hipErrorInvalidValue;
    hipLaunchKernelGGL(cqt_kernel<true>, dim3((unsigned)blocks), dim3(256), lds, stream, p);
  } else {
    hipLaunchKernelGGL(cqt_kernel<false>, dim3((unsigned)blocks), dim3(256), lds, stream, p);
  }
  return hipGetLastError();
}

}  // namespace nna
