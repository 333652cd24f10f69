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

hipError_t launch_stft16(const Stft16Params& p, hipStream_t stream) {
  const long long n_rg = (p.n_rt + p.rt_per_block - 1) / p.rt_per_block;
  const long long blocks = p.n_ft * n_rg;
  if (blocks <= 0 || blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  if (p.tile_frames > H_FRAMES || p.nj < 1) return hipErrorInvalidValue;
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
