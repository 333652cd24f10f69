// Backward pass of the layers with trainable kernels -- STFT, Mel, one-rate constant-Q -- (arXiv
// 1912.12055, Sec. IV-C "Trainable Transformation Kernels") on gfx950 / CDNA4.
//
// Forward:  C[r, f] = sum_n W[r, n] xp[f hop + n]  (r = packed bank row, f = global frame), then the
// output format per (Re, Im) pair.  Given the upstream gradient, the STFT kernel's gradient mode
// first writes G = dLoss/dC[packed row][global frame].  The two contractions here finish the job:
//
//   bank gradient      gW[r, n]  = sum_f G[r, f] xp[f hop + n]              (rows x taps, over frames)
//   waveform gradient  D[f, n]   = sum_r G[r, f] W[r, n], then gx[mirror(f hop + n)] += D[f, n]
//                                                              (frames x taps, over bank rows)
//
// Both are dense GEMMs on v_mfma_f32_32x32x2_f32: a 128 x 128 output tile per workgroup (4 waves, four 32 x 32
// accumulators each), the contraction in chunks of 32 (double buffered, one barrier per chunk, in the middle of it),
// two workgroups per compute unit.  Lanes of an accumulator register run along the output's contiguous axis (taps) in
// both, so the final atomic adds go out in 128-byte runs.
//   bw_bank_kernel   4 waves of 128 rows x 32 taps.  The G tile (m-major: G rows are contiguous along the contraction
//                    index) goes through LDS, read by all four waves; the frames matrix, never built, is each wave's
//                    own operand and goes from the waveform straight into registers in MFMA layout, reflection
//                    included.
//   bw_wave_kernel   2 x 2 waves of 64 x 64; both operands k-major in LDS ([k][column], 4-byte LDS reads: at the
//                    float32 MFMA rate LDS bandwidth is nowhere near a limit).
//
// A constant-Q bank (rows zero outside a tap range each, hundreds of hop-shifts) uses the same bank-gradient
// kernel restricted to the output tiles and 32-row blocks that hold taps, and a waveform-gradient kernel of
// its own (cq_wave_kernel, below).  The Mel layer's two small contractions are at the end of the file.
//
// Sums that meet in memory -- the split contraction of the bank gradient, the overlapping frames
// and mirrored edge samples of the waveform gradient -- are combined with float atomic adds on
// buffers the caller of these launchers has zeroed, so their order (and with it the last bits of
// the result) may vary from run to run.
#include "nna_device.h"

#include <algorithm>
#include <type_traits>

namespace nna {

typedef f32x4 f32x4_u __attribute__((aligned(4)));

constexpr int BW_PA_M = BW_KC + 4;   // LDS pitch of an m-major A tile (conflict-free 16-byte reads)
constexpr int BW_PK = BW_NT + 4;     // LDS pitch of a k-major tile

__global__ void fill_zero_kernel(float* __restrict__ p, long long n) {
  const long long stride = (long long)gridDim.x * blockDim.x;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = 0.f;
}

// Transposed decimation (Sec. III-C "Downsampling", backwards): the forward step is
//     y[m] = sum_v he[v] x~[2 (m + ve0 + v)] + sum_v ho[v] x~[2 (m + vo0 + v) + 1],   x~ = x mirrored at both ends,
// so sample p of the extended signal collects  u[p] = sum_v taps[v] g[i - v0 - v]  (p = 2 i even: he, ve0;
// p = 2 i + 1 odd: ho, vo0), and stored sample j collects u at j and at its mirror images -j and 2 (L - 1) - j.
__device__ __forceinline__ float firt_u(const FirTParams& P, const float* __restrict__ g, long long p) {
  const long long i = p >> 1;  // floor, also for negative p
  const bool odd = p & 1;
  const float* __restrict__ taps = odd ? P.ho : P.he;
  const long long n = odd ? P.no : P.ne, top = i - (odd ? P.vo0 : P.ve0);  // m = top - v must lie in [0, Ln)
  const long long vlo = top - (P.Ln - 1) > 0 ? top - (P.Ln - 1) : 0, vhi = top < n - 1 ? top : n - 1;
  float acc = 0.f;
  for (long long v = vlo; v <= vhi; ++v) acc += taps[v] * g[top - v];
  return acc;
}

// The main image u[p], 0 <= p < L, is two plain filters over g -- u[2 i] with he, u[2 i + 1] with ho, each applied
// back to front -- computed like the forward step: a workgroup stages the span of g its 2,048 values of i need in
// LDS (position i + i/8: threads start eight samples apart, stride 9 keeps them on different banks), and a thread
// produces eight consecutive i of both parities from a window that slides through registers.  The mirror images
// only reach the samples within a filter length of either end: those few take the direct sums of firt_u.
constexpr int FT_T = 8;                  // values of i per thread
constexpr int FT_TILE = 256 * FT_T;      // per workgroup
constexpr int FT_SPAN_MAX = 2064;        // (largest v0 + n - 1) - (smallest v0) the LDS buffer allows
__device__ __forceinline__ int ft_pos(int i) { return i + (i >> 3); }

// acc[ii] += sum_v taps[v] w[off + ii + (n - 1 - v)]   (n a multiple of eight)
__device__ __forceinline__ void ft_stream(float (&acc)[FT_T], const float* __restrict__ wt, int off, const float* __restrict__ taps, int n) {
  float win[2 * FT_T];
#pragma unroll
  for (int i = 0; i < FT_T; ++i) win[i] = wt[ft_pos(off + i)];
  for (int k0 = 0; k0 < n; k0 += FT_T) {
#pragma unroll
    for (int i = 0; i < FT_T; ++i) win[FT_T + i] = wt[ft_pos(off + k0 + FT_T + i)];
#pragma unroll
    for (int kk = 0; kk < FT_T; ++kk) {
      const float tp = taps[n - 1 - (k0 + kk)];
#pragma unroll
      for (int i = 0; i < FT_T; ++i) acc[i] += tp * win[i + kk];
    }
#pragma unroll
    for (int i = 0; i < FT_T; ++i) win[i] = win[i + FT_T];
  }
}

__global__ __launch_bounds__(256) void fir_transpose_add_kernel(const FirTParams P) {
  __shared__ float lds[(FT_TILE + FT_SPAN_MAX + 2 * FT_T) * 9 / 8 + 16];
  const int tid = threadIdx.x;
  const long long b = blockIdx.y;
  const long long i0 = (long long)blockIdx.x * FT_TILE;
  const float* __restrict__ g = P.g + b * P.Ln;
  const int ext_e = P.ve0 + P.ne - 1, ext_o = P.vo0 + P.no - 1;
  const int emax = ext_e > ext_o ? ext_e : ext_o, vmin = P.ve0 < P.vo0 ? P.ve0 : P.vo0;
  const int n_l = FT_TILE + (emax - vmin) + FT_T;  // g[i0 - emax + k], k < n_l (zero outside the array)
  for (int k = tid; k < n_l; k += 256) {
    const long long idx = i0 - emax + k;
    lds[ft_pos(k)] = (idx >= 0 && idx < P.Ln) ? g[idx] : 0.f;
  }
  __syncthreads();
  const long long ib = i0 + (long long)FT_T * tid;
  if (ib >= P.Ln) return;
  float ue[FT_T], uo[FT_T];
#pragma unroll
  for (int i = 0; i < FT_T; ++i) ue[i] = uo[i] = 0.f;
  // u[2 i] = sum_v he[v] g[i - ve0 - v]: with k = ne - 1 - v the window starts at g[i - ext_e], LDS sample i - i0 + emax - ext_e
  ft_stream(ue, lds + 9 * tid, emax - ext_e, P.he, P.ne);
  ft_stream(uo, lds + 9 * tid, emax - ext_o, P.ho, P.no);
  // the mirror images of samples this close to an end can be non-zero
  const long long margin = 2LL * (emax > -vmin ? emax : -vmin) + 4;
  float* __restrict__ out = P.gx + b * P.L;
  // Away from both ends a thread's sixteen samples are one aligned 64-byte run: four 16-byte loads and stores (one
  // sample at a time, lanes 64 bytes apart, each access touched 64 cache lines for 4 bytes of each).
  const long long p0 = 2 * ib;
  if (p0 > margin && p0 + 2 * FT_T - 1 < P.L - 1 - margin && ((reinterpret_cast<uintptr_t>(out + p0) & 15) == 0)) {
    f32x4* o4 = reinterpret_cast<f32x4*>(out + p0);
#pragma unroll
    for (int q = 0; q < FT_T / 2; ++q) {
      f32x4 v = o4[q];
      v[0] += ue[2 * q];
      v[1] += uo[2 * q];
      v[2] += ue[2 * q + 1];
      v[3] += uo[2 * q + 1];
      o4[q] = v;
    }
    return;
  }
#pragma unroll
  for (int i = 0; i < FT_T; ++i)
#pragma unroll
    for (int par = 0; par < 2; ++par) {
      const long long p = 2 * (ib + i) + par;
      if (p >= P.L) continue;
      float v = par ? uo[i] : ue[i];
      if (p >= 1 && p <= margin) v += firt_u(P, g, -p);
      if (p <= P.L - 2 && p >= P.L - 1 - margin) v += firt_u(P, g, 2 * (P.L - 1) - p);
      out[p] += v;
    }
}

// G of a stage whose output is the transform itself (complex format): the upstream gradient as it stands, moved into
// the blocked layout [frame / 32][packed row][frame % 32].  Packed banks keep (Re_0, Re_{N/2}) in rows 0, 1 and drop
// the two identically-zero sine rows; rows past the bank's are written as zeros.  One workgroup per block of 32
// frames: 8 rows x 32 frames per step, 128-byte runs on both sides.
__global__ __launch_bounds__(256) void g_from_complex_kernel(float* __restrict__ gbuf, const float* __restrict__ gout,
                                                             long long n_frames, int T, int out_rows, int rows_pad,
                                                             int n_half, int packed) {
  const long long f = (long long)blockIdx.x * 32 + (threadIdx.x & 31);
  if (f >= n_frames) return;
  const long long b = f / T;
  const int t = (int)(f - b * T);
  const float* __restrict__ gp = gout + b * (long long)out_rows * T + t;
  float* __restrict__ Gp = gbuf + (long long)blockIdx.x * rows_pad * 32 + (threadIdx.x & 31);
  for (int pr = threadIdx.x >> 5; pr < rows_pad; pr += 8) {
    float v = 0.f;
    if ((pr >> 1) < n_half) {
      const int lrow = packed && pr < 2 ? (pr == 0 ? 0 : 2 * n_half) : pr;
      v = gp[(long long)lrow * T];
    }
    Gp[(long long)pr * 32] = v;
  }
}

// frames [f0, f1) of every row of the blocked G buffer [frame / 32][rows_pad][frame % 32]
__global__ void fill_zero_frames_kernel(float* __restrict__ p, long long rows_pad, long long f0, long long f1) {
  const long long w = f1 - f0, n = rows_pad * w;
  const long long stride = (long long)gridDim.x * blockDim.x;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
    const long long r = i / w, f = f0 + (i - r * w);
    p[(f >> 5) * (rows_pad * 32) + r * 32 + (f & 31)] = 0.f;
  }
}

// ---- logical <-> streaming order of the STFT bank ----------------------------------------------
// fragment element -> (packed row, tap); the order is that of the forward kernel's bank stream:
// [row tile][chunk][hop-shift][fragment group][row block][lane] x float4
struct FragPos {
  int pr, tap;
};
__device__ __forceinline__ FragPos frag_pos(const BankPermuteParams& P, long long i4, int e) {
  const int lane = (int)(i4 & 63), rb = (int)((i4 >> 6) & 3);
  const long long G = (long long)P.n_chunks * P.nj * ST_NKG;
  const long long gi = (i4 >> 8) % G;
  const int rt = (int)((i4 >> 8) / G);
  const int kg = (int)(gi % ST_NKG), j = (int)((gi / ST_NKG) % P.nj), c = (int)(gi / ((long long)ST_NKG * P.nj));
  FragPos fp;
  fp.pr = rt * ST_ROWS + rb * 32 + (lane & 31);
  fp.tap = j * P.hop + c * ST_KC + kg * ST_KG + 4 * (lane >> 5) + e;
  return fp;
}
// packed row -> row of the logical [2 bins][K] bank
__device__ __forceinline__ int logical_row(int pr, int n_half, int packed) {
  return packed ? (pr == 0 ? 0 : pr == 1 ? 2 * n_half : pr) : pr;
}

__global__ void bank_from_logical_kernel(const BankPermuteParams P, long long n4) {
  const long long i4 = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i4 >= n4) return;
  f32x4 v;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const FragPos fp = frag_pos(P, i4, e);
    float x = 0.f;
    if ((fp.pr >> 1) < P.n_half && fp.tap < P.K) {
      x = P.logical[(long long)logical_row(fp.pr, P.n_half, P.packed) * P.K + fp.tap];
      P.wrm[(long long)fp.pr * P.kp + fp.tap] = x;
    }
    v[e] = x;
  }
  reinterpret_cast<f32x4*>(P.bank)[i4] = v;
}

__global__ void bank_to_rowmajor_kernel(const BankPermuteParams P, long long n4) {
  const long long i4 = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i4 >= n4) return;
  const f32x4 v = reinterpret_cast<const f32x4*>(P.bank)[i4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const FragPos fp = frag_pos(P, i4, e);
    if ((fp.pr >> 1) < P.n_half && fp.tap < P.K) P.wrm[(long long)fp.pr * P.kp + fp.tap] = v[e];
  }
}

__global__ void bank_to_logical_kernel(const BankPermuteParams P, long long n) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const int lrow = (int)(i / P.K), tap = (int)(i - (long long)lrow * P.K);
  int pr = lrow;
  bool zero = false;
  if (P.packed) {
    if (lrow == 0) pr = 0;
    else if (lrow == 2 * P.n_half) pr = 1;
    else if (lrow == 1 || lrow == 2 * P.n_half + 1) zero = true;  // the two identically-zero sine rows
  }
  P.logical[i] = zero ? 0.f : P.wrm[(long long)pr * P.kp + tap];
}

// ---- the contraction kernel --------------------------------------------------------------------
// Frames t .. t+3 (of T; zero outside) of row `row` of the blocked G buffer [frame / 32][rows_pad][frame % 32];
// fb0 = global index of the waveform's frame 0, blk = rows_pad * 32.
__device__ __forceinline__ f32x4 load_g4(const float* __restrict__ gbuf, long long blk, int row, long long fb0, int t, int T) {
  f32x4 v = {0.f, 0.f, 0.f, 0.f};
  if (t >= 0 && t + 3 < T) {
    const long long f = fb0 + t;
    const int off = (int)(f & 31);
    if (off <= 28) return *reinterpret_cast<const f32x4_u*>(gbuf + (f >> 5) * blk + row * 32 + off);
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = gbuf[((f + i) >> 5) * blk + row * 32 + ((f + i) & 31)];
  } else if (t + 3 >= 0 && t < T) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (t + i >= 0 && t + i < T) v[i] = gbuf[((fb0 + t + i) >> 5) * blk + row * 32 + ((fb0 + t + i) & 31)];
  }
  return v;
}

// Waveform gradient as a plain product over the bank's rows: frames x taps tile = G^T [frames, rows] x W [rows, taps],
// added onto the waveform sample each (frame, tap) pair reads.  For short kernels (the STFT's, the deep octaves of a
// downsampling CQT); the long constant-Q kernels go through cq_wave_kernel below.
__global__ __launch_bounds__(256, 2) void bw_wave_kernel(const BwParams P) {
  __shared__ __attribute__((aligned(16))) float ldsA[2][BW_KC * BW_PK];
  __shared__ __attribute__((aligned(16))) float ldsB[2][BW_KC * BW_PK];

  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int wm = wave >> 1, wn = wave & 1;  // 2 x 2 waves of 64 x 64
  const int h = lane >> 5, r32 = lane & 31;
  const FrameGeom& g = P.g;

  // the tap tiles of one frame tile are neighbours: they share its G columns in the L2
  const int n_nt = P.kp / BW_NT;
  const long long m0 = (long long)(blockIdx.x / n_nt) * BW_MT;
  const int n0 = (int)(blockIdx.x % n_nt) * BW_NT;
  const long long c_end = (2 * P.n_half + BW_KC - 1) / BW_KC;  // row chunks that hold bank rows (the padding rows of G and W are zero)
  if (c_end < 1) return;

  f32x4 ra[4], rb[4];
  // global -> registers for contraction chunk c:
  // A: G[k0 + k][m0 + 4 c4], k = tid/32 + 8 p (frame block m0/32 + c4/8);  B: wrm[k0 + k][n0 + 4 c4]
  auto fetch = [&](long long c) {
    const long long k0 = c * BW_KC;
    const float* ap = P.gbuf + ((m0 >> 5) + ((tid & 31) >> 3)) * ((long long)P.rows_pad * 32) + (k0 + (tid >> 5)) * 32 + 4 * (tid & 7);
    const float* bp = P.wrm + (k0 + (tid >> 5)) * P.kp + n0 + 4 * (tid & 31);
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      ra[p] = *reinterpret_cast<const f32x4*>(ap + 8 * p * 32);
      rb[p] = *reinterpret_cast<const f32x4*>(bp + (long long)(8 * p) * P.kp);
    }
  };
  // registers -> LDS buffer
  auto stage = [&](int buf) {
    float* a = &ldsA[buf][(tid >> 5) * BW_PK + 4 * (tid & 31)];
    float* b = &ldsB[buf][(tid >> 5) * BW_PK + 4 * (tid & 31)];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      *reinterpret_cast<f32x4*>(a + 8 * p * BW_PK) = ra[p];
      *reinterpret_cast<f32x4*>(b + 8 * p * BW_PK) = rb[p];
    }
  };

  f32x16 acc[4];  // acc[2 mi + ni]
#pragma unroll
  for (int s = 0; s < 4; ++s)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[s][r] = 0.f;

  // lane (h, r32) holds contraction indices 8 kg + 4 h + e, e = 0..3, of row / column r32
  auto load_frags = [&](const float* A, const float* B, int kg, f32x4 (&a)[2], f32x4 (&b)[2]) {
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
      for (int e = 0; e < 4; ++e) a[mi][e] = A[(8 * kg + 4 * h + e) * BW_PK + wm * 64 + mi * 32 + r32];
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
      for (int e = 0; e < 4; ++e) b[ni][e] = B[(8 * kg + 4 * h + e) * BW_PK + wn * 64 + ni * 32 + r32];
  };
  auto mfma_group = [&](const f32x4 (&a)[2], const f32x4 (&b)[2]) {
#pragma unroll
    for (int e = 0; e < 4; ++e)
#pragma unroll
      for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
          acc[2 * mi + ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[mi][e], b[ni][e], acc[2 * mi + ni], 0, 0, 0);
  };

  // Pipeline: while chunk c is multiplied out of one LDS buffer, chunk c+1 (requested one iteration
  // earlier) is written to the other and chunk c+2 is requested.  The operand fragments of a group of 8 contraction
  // indices are read from LDS two groups ahead of their 16 MFMAs -- across the chunk boundary too: the barrier sits
  // in the middle of a chunk, after every read of its buffer and every write of the next one, so the first two
  // groups of chunk c+1 are read behind the barrier while the last two groups of chunk c run, and no wave starts a
  // chunk by waiting for LDS.
  fetch(0);
  stage(0);
  if (1 < c_end) fetch(1);
  __syncthreads();
  static_assert(BW_KC == 32, "four fragment groups per chunk");
  f32x4 a0[2], b0[2], a1[2], b1[2];
  load_frags(ldsA[0], ldsB[0], 0, a0, b0);
  load_frags(ldsA[0], ldsB[0], 1, a1, b1);

  for (long long c = 0; c < c_end; ++c) {
    const int buf = (int)(c & 1);
    const float* A = ldsA[buf];
    const float* B = ldsB[buf];
    // The scheduling barriers pin the order: each group's LDS reads go out ahead of the previous
    // group's 16 MFMAs (left alone, the compiler sinks every read to just before its first use and
    // the matrix pipe idles for the LDS latency every four MFMAs), and the LDS writes of chunk c+1
    // and the global requests for chunk c+2 sit behind reads that are already on their way, with a
    // whole MFMA group to hide them.
    __builtin_amdgcn_sched_barrier(0);
    mfma_group(a0, b0);
    __builtin_amdgcn_sched_barrier(0);
    load_frags(A, B, 2, a0, b0);
    if (c + 1 < c_end) stage(buf ^ 1);
    __builtin_amdgcn_sched_barrier(0);
    mfma_group(a1, b1);
    __builtin_amdgcn_sched_barrier(0);
    load_frags(A, B, 3, a1, b1);
    if (c + 2 < c_end) fetch(c + 2);
    __syncthreads();  // buffer `buf` has been read for the last time, buffer `buf ^ 1` is complete
    __builtin_amdgcn_sched_barrier(0);
    mfma_group(a0, b0);
    __builtin_amdgcn_sched_barrier(0);
    if (c + 1 < c_end) load_frags(ldsA[buf ^ 1], ldsB[buf ^ 1], 0, a0, b0);
    __builtin_amdgcn_sched_barrier(0);
    mfma_group(a1, b1);
    __builtin_amdgcn_sched_barrier(0);
    if (c + 1 < c_end) load_frags(ldsA[buf ^ 1], ldsB[buf ^ 1], 1, a1, b1);
  }

  // ---- epilogue: accumulator register r of lane (h, r32) is output row 8 (r/4) + 4 h + r%4, column r32
  const int L = (int)g.L;
#pragma unroll
  for (int mi = 0; mi < 2; ++mi)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      // four consecutive frames per register quad
      long long f = m0 + wm * 64 + mi * 32 + 8 * q + 4 * h;
      long long b = f / g.T;
      int t = (int)(f - b * g.T);
#pragma unroll
      for (int i = 0; i < 4; ++i, ++f) {
        if (f < g.n_frames) {
          float* __restrict__ row = P.gx + b * g.L;
#pragma unroll
          for (int ni = 0; ni < 2; ++ni) {
            const int tap = n0 + wn * 64 + ni * 32 + r32;
            if (tap < P.K) {
              int j = t * g.hop + tap - g.pad;
              j = j < 0 ? -j : (j >= L ? 2 * (L - 1) - j : j);  // mirror padding folded back
              unsafeAtomicAdd(row + j, acc[2 * mi + ni][4 * q + i]);
            }
          }
        }
        if (++t == g.T) {
          t = 0;
          ++b;
        }
      }
    }
}

// ---- bank gradient with the frames operand straight from memory --------------------------------
// gw[row, tap] = sum_f G[row, f] x_pad[f hop + tap].  A workgroup owns 128 rows x 128 taps and a range of frame chunks;
// a wave owns 32 of the taps and all four 32-row blocks, so the frames operand it multiplies is its own:
// x_pad[(f0 + 8 kg + 4 h + e) hop + n0 + 32 wave + r32] is element 4 kg + e of lane (h, r32), the MFMA's B operand as
// it stands -- sixteen coalesced one-sample loads per chunk (one sample at a time the mirrored edges are an index
// fold, no special path), requested one chunk ahead into the other of two register sets.  Only the G tile, which all
// four waves read, goes through LDS.
template <bool SPARSE>
__global__ __launch_bounds__(256, 2) void bw_bank_kernel(const BwParams P) {
  __shared__ __attribute__((aligned(16))) float ldsA[2][BW_MT * BW_PA_M];

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int h = lane >> 5, r32 = lane & 31;
  const FrameGeom& g = P.g;

  const int n_nt = P.kp / BW_NT;
  const int n_mt = P.rows_pad / BW_MT;
  const long long tiles = SPARSE ? P.n_tiles : (long long)n_mt * n_nt;
  const long long split = blockIdx.x / tiles;
  int tile = (int)(blockIdx.x - split * tiles);
  long long m0;
  int n0, alive_rt = 4;
  if constexpr (SPARSE) {
    // the list is ordered heaviest tile first; neighbours in it go to different dies, which balances them
    const int2 t = P.tiles[tile];
    m0 = (long long)(t.x & 0xffff) * BW_MT;
    n0 = t.y * BW_NT;
    alive_rt = t.x >> 16;
  } else {
    // Workgroup ids are dealt round-robin to the 8 dies, each with an L2 of its own.  Give every die a contiguous
    // run of tiles in row-major order: it then reads only its own rows of G (the large operand).
    if (tiles % 8 == 0) tile = (tile & 7) * (int)(tiles / 8) + (tile >> 3);
    m0 = (long long)(tile / n_nt) * BW_MT;
    n0 = (tile % n_nt) * BW_NT;
  }
  const long long n_chunks = P.gpitch / BW_KC;
  const long long c_begin = split * P.chunks_per_split;
  const long long c_end = c_begin + P.chunks_per_split < n_chunks ? c_begin + P.chunks_per_split : n_chunks;
  if (c_begin >= c_end) return;

  f32x16 acc[4];
#pragma unroll
  for (int s = 0; s < 4; ++s)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[s][r] = 0.f;

  // (waveform, frame in it) of the first frame of the chunk the next fetch_b asks for: stepped, not divided out
  long long nfb = c_begin * BW_KC / g.T;
  int nft = (int)(c_begin * BW_KC - nfb * g.T);
  const int tap = n0 + wave * 32 + r32;
  const int L = (int)g.L;
  auto fetch_b = [&](float (&bw)[16]) {
    // Almost every chunk lies inside one waveform and clear of its mirrored ends (one test for the whole workgroup):
    // a base every lane shares plus a lane offset that never changes.
    const long long lo = (long long)nft * g.hop + n0 - g.pad;
    if (nft + BW_KC <= g.T && nfb < g.B && lo >= 0 && lo + (long long)(BW_KC - 1) * g.hop + BW_NT <= g.L) {
      const float* base = g.x + nfb * g.L + lo;
#pragma unroll
      for (int i = 0; i < 16; ++i) bw[i] = base[(8 * (i >> 2) + 4 * h + (i & 3)) * g.hop + wave * 32 + r32];
      nft += BW_KC;
      if (nft >= g.T) {
        nft -= g.T;
        ++nfb;
      }
      return;
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      int t = nft + 8 * (i >> 2) + 4 * h + (i & 3);
      long long b = nfb;
      while (t >= g.T) {
        t -= g.T;
        ++b;
      }
      b = b < g.B ? b : g.B - 1;  // frames past the last one: their G is zero, any sample serves
      int j = t * g.hop + tap - g.pad;
      j = j < 0 ? -j : j;
      j = j >= L ? 2 * (L - 1) - j : j;  // mirror padding folded back
      j = j < 0 ? 0 : (j >= L ? L - 1 : j);  // taps of the padding columns past K: never stored
      bw[i] = g.x[b * g.L + j];
    }
    nft += BW_KC;
    while (nft >= g.T) {
      nft -= g.T;
      ++nfb;
    }
  };

  // The count of live row blocks is a compile-time constant of the chunk loop (one copy of the loop per count):
  // tested at run time it put a branch around every MFMA.
  auto sweep = [&](auto alive_c) {
    constexpr int alive = decltype(alive_c)::value;
    f32x4 ra[4];
    // G[m0 + row][32 c + 4 c4], row = tid/8 + 32 p: the tile is one contiguous run of frame block c
    auto fetch_a = [&](long long c) {
      const float* ap = P.gbuf + c * ((long long)P.rows_pad * 32) + (m0 + (tid >> 3)) * 32 + 4 * (tid & 7);
#pragma unroll
      for (int p = 0; p < alive; ++p) ra[p] = *reinterpret_cast<const f32x4*>(ap + 32 * 32 * p);
    };
    auto stage_a = [&](int buf) {
      float* a = &ldsA[buf][(tid >> 3) * BW_PA_M + 4 * (tid & 7)];
#pragma unroll
      for (int p = 0; p < alive; ++p) *reinterpret_cast<f32x4*>(a + 32 * p * BW_PA_M) = ra[p];
    };
    // lane (h, r32) holds contraction indices 8 kg + 4 h + e, e = 0..3, of row r32 of each block
    auto load_a = [&](const float* A, int kg, f32x4 (&a)[4]) {
#pragma unroll
      for (int s = 0; s < alive; ++s) a[s] = *reinterpret_cast<const f32x4*>(A + (s * 32 + r32) * BW_PA_M + 8 * kg + 4 * h);
    };
    auto mfma_group = [&](const f32x4 (&a)[4], const float (&bw)[16], int kg) {
#pragma unroll
      for (int e = 0; e < 4; ++e)
#pragma unroll
        for (int s = 0; s < alive; ++s)
          acc[s] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[s][e], bw[4 * kg + e], acc[s], 0, 0, 0);
    };

    float bw0[16], bw1[16];
    f32x4 a0[4], a1[4];
    fetch_a(c_begin);
    fetch_b(bw0);
    stage_a(0);
    if (c_begin + 1 < c_end) fetch_a(c_begin + 1);
    __syncthreads();
    static_assert(BW_KC == 32, "four fragment groups per chunk");
    load_a(ldsA[0], 0, a0);
    load_a(ldsA[0], 1, a1);
    // One chunk out of LDS buffer `buf`: the next chunk's frames operand is requested at its head (on every chunk,
    // the last one's request reads frames past the range and is dropped: one path, so that the compiler's wait ahead
    // of an MFMA counts these sixteen as younger than its operand), the next chunk's G tile goes to the other
    // buffer behind the first MFMA group, the one after that is requested behind the second.  The barrier sits in
    // the middle of the chunk, after every read of its buffer and every write of the other one, and the first
    // fragments of the next chunk are read behind it while the last two groups run.
    auto chunk = [&](long long c, int buf, const float (&bw)[16], float (&next)[16]) {
      const float* A = ldsA[buf];
      fetch_b(next);
      __builtin_amdgcn_sched_barrier(0);
      mfma_group(a0, bw, 0);
      __builtin_amdgcn_sched_barrier(0);
      load_a(A, 2, a0);
      if (c + 1 < c_end) stage_a(buf ^ 1);
      __builtin_amdgcn_sched_barrier(0);
      mfma_group(a1, bw, 1);
      __builtin_amdgcn_sched_barrier(0);
      load_a(A, 3, a1);
      if (c + 2 < c_end) fetch_a(c + 2);
      __syncthreads();
      __builtin_amdgcn_sched_barrier(0);
      mfma_group(a0, bw, 2);
      __builtin_amdgcn_sched_barrier(0);
      if (c + 1 < c_end) load_a(ldsA[buf ^ 1], 0, a0);
      __builtin_amdgcn_sched_barrier(0);
      mfma_group(a1, bw, 3);
      __builtin_amdgcn_sched_barrier(0);
      if (c + 1 < c_end) load_a(ldsA[buf ^ 1], 1, a1);
    };
    for (long long c = c_begin; c < c_end; c += 2) {
      chunk(c, 0, bw0, bw1);
      if (c + 1 < c_end) chunk(c + 1, 1, bw1, bw0);
    }
  };
  if constexpr (SPARSE) {
    switch (alive_rt) {
      case 1: sweep(std::integral_constant<int, 1>{}); break;
      case 2: sweep(std::integral_constant<int, 2>{}); break;
      case 3: sweep(std::integral_constant<int, 3>{}); break;
      default: sweep(std::integral_constant<int, 4>{}); break;
    }
  } else {
    sweep(std::integral_constant<int, 4>{});
  }

  // accumulator register r of lane (h, r32) of block s is output row m0 + 32 s + 8 (r/4) + 4 h + r%4, column `tap`
  if (tap < P.K) {
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      if (s >= alive_rt) continue;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int pr = (int)m0 + s * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
        if ((pr >> 1) < P.n_half && (!SPARSE || (tap >= P.row_lo[pr] && tap < P.row_hi[pr])))
          unsafeAtomicAdd(P.gw + (long long)logical_row(pr, P.n_half, P.packed) * P.K + tap, acc[s][r]);
      }
    }
  }
}

// ---- waveform gradient of a bank with per-row supports -----------------------------------------
// Long constant-Q kernels span hundreds of hop-shifts; a tile of frames x taps (as above) would add
// every product to memory atomically and re-read G for every shift.  Here the output is tiled by
// (hop-row q, column c) of a waveform's padded signal, sample q hop + c, and the shifts are gathered
// inside the workgroup:
//   out[q, c] = sum_r sum_j G[r, q - j] W[r, j hop + c],
// a contraction over (row r, shift j) pairs whose A operand is G read j frames back.  Rows go in chunks
// of CW_KC, the outer loop; for one chunk the frames q0 - j .. q0 - j + 127 of all its shifts form
// one window of G that stays in LDS while only W tiles stream.  Each padded sample is written once
// (the atomic add only folds the mirrored samples onto the waveform).
constexpr int CW_SEG = BW_MT;             // shifts served by one window
constexpr int CW_WIN = BW_MT + CW_SEG;    // frames in the window (128 tile rows + up to 127 shifts, rounded up)
constexpr int CW_PA = CW_WIN + 4;         // its LDS pitch

// WHOLE: every W tile of the launch lies inside the hop and inside the padded bank row (the launcher checks it).
template <bool WHOLE>
__global__ __launch_bounds__(256, 2) void cq_wave_kernel(const BwParams P) {
  __shared__ __attribute__((aligned(16))) float ldsA[CW_KC * CW_PA];

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int h = lane >> 5, r32 = lane & 31;
  const FrameGeom& g = P.g;
  const int T = g.T;

  // The column tile is the slow index: the workgroups resident at one time then stream the same W tiles (the whole bank,
  // 88 MB for 168 bins of 65,536 taps, goes past every workgroup; G is a hundred times smaller) and share them in the L2s.
  const long long n_bq = (long long)gridDim.x / P.n_ct;
  const int ct = (int)(blockIdx.x / n_bq), n0 = ct * BW_NT;
  // Within a column tile the hop-row tile is the next slower index and the waveform the fast one.  Workgroups go to
  // the chip's eight dies in turn, and the row tiles of a waveform differ in work (the first and the last hold rows
  // whose frames lie outside the waveform on most shifts: 62 % and 33 % of a middle tile's MFMAs for 345 frames and
  // 128 shifts); with the row tile as the fast index and four tiles per waveform each die saw one kind of tile only,
  // and those with the middle tiles ran three times longer than those with the last.  The full tiles go first, the
  // two partial ones last.
  const long long bq = blockIdx.x - ct * n_bq;
  const int qi = (int)(bq / g.B);
  const long long gb = bq - (long long)qi * g.B;
  const int qt = qi < P.n_qt - 2 ? qi + 1 : (qi == P.n_qt - 2 ? 0 : P.n_qt - 1);
  const int q0 = qt * BW_MT;
  // shifts j with a frame q - j inside [0, T) for some row q of the tile
  const int j_lo = q0 - (T - 1) > 0 ? q0 - (T - 1) : 0;
  const int j_hi = q0 + BW_MT - 1 < P.n_shift - 1 ? q0 + BW_MT - 1 : P.n_shift - 1;

  f32x16 acc[4];
#pragma unroll
  for (int s = 0; s < 4; ++s)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[s][r] = 0.f;

  // Rows go in chunks of CW_KC = 16 (8 bins: the kernels of 16 adjacent bins differ by 2^(16/24) in length, and a
  // chunk runs over the shifts of its longest), shifts in pairs: the 32 contraction indices of an MFMA sweep are
  // 16 rows x 2 shifts, index 16 s + 8 kg + 4 h + e = shift j + s, row k0 + 8 kg + 4 h + e.
  // A wave owns 32 columns of the tile and all four of its 32-row blocks, so the W values it multiplies are its own:
  // W[k0 + 8 kg + 4 h + e][(j + s) hop + n0 + wave 32 + r32] is element 8 s + 4 kg + e of lane (h, r32), the B operand
  // of the MFMA as it stands.  They go from memory straight into registers, one pair of shifts ahead of their use (a
  // pair is 64 MFMAs of 64 cycles, far longer than a load takes), and never through LDS: only the G window is shared,
  // and the waves of a workgroup meet once per window, not once per shift (staged through LDS with a barrier per
  // shift, 45 % of the wave cycles were waits).  Columns past the hop belong to the next shift and read as zero, and
  // so does the second shift of a pair past the last one.
  float bw0[16], bw1[16];
  const int colw = n0 + wave * 32;  // first column of the wave
  // address = a base every lane of the wave shares (scalar registers) + a 32-bit lane offset that never changes
  const unsigned lane_w = (unsigned)((4u * h * (unsigned)P.kp + r32) * sizeof(float));
  auto fetch_b = [&](float (&bw)[16], int k0, int j, int je) {
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) {
      const bool there = j + s2 <= je;
      const long long tb = (long long)(there ? j + s2 : je) * g.hop + colw;
      const char* row = reinterpret_cast<const char*>(P.wrm + (long long)k0 * P.kp + tb);
      const bool in = there && (WHOLE || (colw + r32 < g.hop && tb + r32 < P.kp));
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const char* rp = row + (long long)(8 * (i >> 2) + (i & 3)) * P.kp * (long long)sizeof(float);
        if constexpr (WHOLE) {
          const float v = *reinterpret_cast<const float*>(rp + lane_w);
          bw[8 * s2 + i] = there ? v : 0.f;
        } else {
          bw[8 * s2 + i] = in ? *reinterpret_cast<const float*>(rp + lane_w) : 0.f;
        }
      }
    }
  };
  // Fragment group g4 = 0..3 of a pair: shift g4 / 2, rows 8 (g4 % 2) + 4 h + e; `w` = window index of tile row 0 on the
  // pair's first shift (one less on the second).
  // A 32-row block of the tile whose frames q - j all fall outside the waveform has a zero A operand (the first and
  // last row tiles of a waveform are half such blocks): it is skipped.  The live blocks of a pair are a run lo .. hi - 1.
  auto load_a = [&](int w, int g4, int lo, int hi, f32x4 (&a)[4]) {
    const int ws = w - (g4 >> 1) > 0 ? w - (g4 >> 1) : 0;  // (a pair's missing second shift: its W values are zero)
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
      if (mi >= lo && mi < hi) {
#pragma unroll
        for (int e = 0; e < 4; ++e) a[mi][e] = ldsA[(8 * (g4 & 1) + 4 * h + e) * CW_PA + ws + mi * 32 + r32];
      }
  };
  auto mfma_group = [&](const f32x4 (&a)[4], const float (&bw)[16], int g4, int lo, int hi) {
#pragma unroll
    for (int e = 0; e < 4; ++e)
#pragma unroll
      for (int mi = 0; mi < 4; ++mi)
        if (mi >= lo && mi < hi)
          acc[mi] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[mi][e], bw[4 * g4 + e], acc[mi], 0, 0, 0);
  };
  // the 64 MFMAs of a pair of shifts; lo_c, hi_c are compile-time constants for the runs that reach an end of the
  // tile (a run-time test puts a branch around every MFMA), plain integers otherwise
  auto pair_mfmas = [&](int w, const float (&bw)[16], auto lo_c, auto hi_c) {
    const int lo = lo_c, hi = hi_c;
    f32x4 a0[4], a1[4];
    load_a(w, 0, lo, hi, a0);
    load_a(w, 1, lo, hi, a1);
    __builtin_amdgcn_sched_barrier(0);
    mfma_group(a0, bw, 0, lo, hi);
    __builtin_amdgcn_sched_barrier(0);
    load_a(w, 2, lo, hi, a0);
    __builtin_amdgcn_sched_barrier(0);
    mfma_group(a1, bw, 1, lo, hi);
    __builtin_amdgcn_sched_barrier(0);
    load_a(w, 3, lo, hi, a1);
    __builtin_amdgcn_sched_barrier(0);
    mfma_group(a0, bw, 2, lo, hi);
    mfma_group(a1, bw, 3, lo, hi);
  };
  using std::integral_constant;

  for (int kc = 0; kc < P.n_kc; ++kc) {
    const int2 rng = P.shift_rng[ct * P.n_kc + kc];  // shifts on which rows k0 .. k0 + 15 hold taps
    const int ja = rng.x > j_lo ? rng.x : j_lo, jb = rng.y < j_hi ? rng.y : j_hi;
    const int k0 = kc * CW_KC;
    for (int js = ja; js <= jb; js += CW_SEG) {
      const int je = js + CW_SEG - 1 < jb ? js + CW_SEG - 1 : jb;
      fetch_b(bw0, k0, js, je);
      __syncthreads();  // every wave is done with the previous window
      // window: frames q0 - je .. of rows k0 .. k0 + 15 (zero outside the waveform), as many as the tile's 128 rows
      // reach over the shifts js .. je
      {
        const int row = tid >> 4;
        const int n_it = (je - js + BW_MT + 63) / 64;  // <= CW_WIN / 64
        for (int i = 0; i < n_it; ++i) {
          const int w = 4 * (tid & 15) + 64 * i;
          *reinterpret_cast<f32x4*>(&ldsA[row * CW_PA + w]) =
              load_g4(P.gbuf, (long long)P.rows_pad * 32, k0 + row, gb * T, q0 - je + w, T);
        }
      }
      __syncthreads();
      // one pair of shifts j, j + 1: the W values of the next pair are requested before its MFMAs start
      auto pair = [&](int j, const float (&bw)[16], float (&next)[16]) {
        // Requested on every pair, the last of a window included (it asks for its own values again): the compiler's
        // wait ahead of an MFMA allows as many loads in flight as every path to it guarantees were requested after the
        // operand's own, and one path without these 16 made every MFMA of every pair wait for the next pair's values.
        fetch_b(next, k0, j + 2 <= je ? j + 2 : j, je);
        const int w = je - j;
        // block mi holds frames q0 + 32 mi - j .. + 31 on the first shift (one frame earlier on the second): live while
        // the last of them is >= 0 on the first shift and the first < T on the second
        const int back = j + 1 <= je ? 1 : 0;
        int lo = 0, hi = 0;
#pragma unroll
        for (int mi = 0; mi < 4; ++mi) {
          const int t_first = q0 + mi * 32 - j;
          lo += t_first + 31 < 0 ? 1 : 0;
          hi += t_first - back < T ? 1 : 0;
        }
        if (lo >= hi) return;
        if (lo == 0 && hi == 4) {
          pair_mfmas(w, bw, integral_constant<int, 0>{}, integral_constant<int, 4>{});
        } else if (hi == 4) {
          if (lo == 1)
            pair_mfmas(w, bw, integral_constant<int, 1>{}, integral_constant<int, 4>{});
          else if (lo == 2)
            pair_mfmas(w, bw, integral_constant<int, 2>{}, integral_constant<int, 4>{});
          else
            pair_mfmas(w, bw, integral_constant<int, 3>{}, integral_constant<int, 4>{});
        } else if (lo == 0) {
          if (hi == 3)
            pair_mfmas(w, bw, integral_constant<int, 0>{}, integral_constant<int, 3>{});
          else if (hi == 2)
            pair_mfmas(w, bw, integral_constant<int, 0>{}, integral_constant<int, 2>{});
          else
            pair_mfmas(w, bw, integral_constant<int, 0>{}, integral_constant<int, 1>{});
        } else {
          pair_mfmas(w, bw, lo, hi);
        }
      };
      for (int j = js; j <= je; j += 4) {
        pair(j, bw0, bw1);
        if (j + 2 <= je) pair(j + 2, bw1, bw0);
      }
    }
  }

  // register r of lane (h, r32) of block mi: hop-row q0 + mi 32 + 8 (r/4) + 4 h + r%4, column n0 + wave 32 + r32
  const int L = (int)g.L;
  const long long ext = (long long)(T - 1) * g.hop + P.K;  // samples of the padded signal that frames cover
  float* __restrict__ xrow = P.gx + gb * g.L;
  const int col = n0 + wave * 32 + r32;
  if (col < g.hop) {
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const long long pos = (long long)(q0 + mi * 32 + 8 * (r >> 2) + 4 * h + (r & 3)) * g.hop + col;
        if (pos < ext) {
          long long j = pos - g.pad;
          j = j < 0 ? -j : (j >= L ? 2 * (L - 1) - j : j);  // mirror padding folded back
          unsafeAtomicAdd(xrow + j, acc[mi][r]);
        }
      }
  }
}

// ---- the Mel layer's backward contractions ------------------------------------------------------
// Four consecutive elements c..c+3 of a row of `lim` elements (zero beyond it, or if the row does not
// exist); rows of the caller's arrays start at any 4-byte boundary.
__device__ __forceinline__ f32x4 load4_guarded(const float* row, int c, int lim) {
  f32x4 v = {0.f, 0.f, 0.f, 0.f};
  if (row) {
    if (c + 3 < lim) {
      v = *reinterpret_cast<const f32x4_u*>(row + c);
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (c + i < lim) v[i] = row[c + i];
    }
  }
  return v;
}

constexpr int MEL_BW_SPEC = 0, MEL_BW_WEIGHTS = 1;

// Same 128 x 128 tile, wave grid and MFMA as bw_wave_kernel; these two contractions are small
// (2 n_mels F flop per frame each, 3 % of the STFT's) and bound by reading / writing the [B, F, T]
// arrays, so the chunk loop is the plain one: load, barrier, write LDS, barrier, multiply.
//   MEL_BW_SPEC:    C[k, t] (one waveform)  A = W[m][k] (k-major: row = contraction index), B = g[b][m][t] (k-major)
//   MEL_BW_WEIGHTS: C[m, k]                 A = g[b][m][t], B = P[b][k][t] (both: row = output index, contraction contiguous)
template <int MODE>
__global__ __launch_bounds__(256, 2) void mel_bw_kernel(const MelBwParams P) {
  constexpr int TILE_FLOATS = MODE == MEL_BW_SPEC ? BW_KC * BW_PK : BW_MT * BW_PA_M;
  __shared__ __attribute__((aligned(16))) float ldsA[TILE_FLOATS];
  __shared__ __attribute__((aligned(16))) float ldsB[TILE_FLOATS];

  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int wm = wave >> 1, wn = wave & 1;
  const int h = lane >> 5, r32 = lane & 31;

  f32x16 acc[2][2];
#pragma unroll
  for (int mi = 0; mi < 2; ++mi)
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;

  auto multiply = [&]() {
#pragma unroll
    for (int kg = 0; kg < BW_KC / 8; ++kg) {
      f32x4 a[2], b[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        if constexpr (MODE == MEL_BW_SPEC) {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            a[i][e] = ldsA[(8 * kg + 4 * h + e) * BW_PK + wm * 64 + i * 32 + r32];
            b[i][e] = ldsB[(8 * kg + 4 * h + e) * BW_PK + wn * 64 + i * 32 + r32];
          }
        } else {
          a[i] = *reinterpret_cast<const f32x4*>(ldsA + (wm * 64 + i * 32 + r32) * BW_PA_M + 8 * kg + 4 * h);
          b[i] = *reinterpret_cast<const f32x4*>(ldsB + (wn * 64 + i * 32 + r32) * BW_PA_M + 8 * kg + 4 * h);
        }
      }
#pragma unroll
      for (int e = 0; e < 4; ++e)
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
          for (int ni = 0; ni < 2; ++ni)
            acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[mi][e], b[ni][e], acc[mi][ni], 0, 0, 0);
    }
  };

  if constexpr (MODE == MEL_BW_SPEC) {
    const int n_mt = P.fp / BW_MT, n_nt = (P.T + BW_NT - 1) / BW_NT;
    const long long b = blockIdx.x / (n_mt * n_nt);
    const int tile = (int)(blockIdx.x - b * (n_mt * n_nt));
    const int k0 = (tile / n_nt) * BW_MT, t0 = (tile % n_nt) * BW_NT;  // bins, frames of this tile
    const float* gb = P.g + b * (long long)P.n_mels * P.T;
    for (int m0 = 0; m0 < P.mels_pad; m0 += BW_KC) {
      f32x4 ra[4], rb[4];
#pragma unroll
      for (int p = 0; p < 4; ++p) {
        const int m = m0 + (tid >> 5) + 8 * p;  // contraction index: the mel
        ra[p] = *reinterpret_cast<const f32x4*>(P.wrm + (long long)m * P.fp + k0 + 4 * (tid & 31));
        rb[p] = load4_guarded(m < P.n_mels ? gb + (long long)m * P.T : nullptr, t0 + 4 * (tid & 31), P.T);
      }
      __syncthreads();
#pragma unroll
      for (int p = 0; p < 4; ++p) {
        *reinterpret_cast<f32x4*>(ldsA + ((tid >> 5) + 8 * p) * BW_PK + 4 * (tid & 31)) = ra[p];
        *reinterpret_cast<f32x4*>(ldsB + ((tid >> 5) + 8 * p) * BW_PK + 4 * (tid & 31)) = rb[p];
      }
      __syncthreads();
      multiply();
    }
    float* __restrict__ ob = P.gP + b * (long long)P.F * P.T;
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
      for (int ni = 0; ni < 2; ++ni) {
        const int t = t0 + wn * 64 + ni * 32 + r32;
        if (t >= P.T) continue;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int k = k0 + wm * 64 + mi * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
          if (k < P.F) ob[(long long)k * P.T + t] = acc[mi][ni][r];
        }
      }
  } else {
    const int n_nt = P.fp / BW_NT, n_mt = (P.n_mels + BW_MT - 1) / BW_MT;
    const long long split = blockIdx.x / (n_mt * n_nt);
    const int tile = (int)(blockIdx.x - split * (n_mt * n_nt));
    const int m0 = (tile / n_nt) * BW_MT, k0 = (tile % n_nt) * BW_NT;  // mels, bins of this tile
    const long long b_begin = split * P.b_per_split;
    const long long b_end = b_begin + P.b_per_split < P.B ? b_begin + P.b_per_split : P.B;
    for (long long b = b_begin; b < b_end; ++b) {
      const float* gb = P.g + b * (long long)P.n_mels * P.T;
      const float* pb = P.P + b * (long long)P.F * P.T;
      for (int t0 = 0; t0 < P.T; t0 += BW_KC) {
        f32x4 ra[4], rb[4];
#pragma unroll
        for (int p = 0; p < 4; ++p) {
          const int row = (tid >> 3) + 32 * p;  // output index: mel (A), bin (B); contraction = frames
          ra[p] = load4_guarded(m0 + row < P.n_mels ? gb + (long long)(m0 + row) * P.T : nullptr, t0 + 4 * (tid & 7), P.T);
          rb[p] = load4_guarded(k0 + row < P.F ? pb + (long long)(k0 + row) * P.T : nullptr, t0 + 4 * (tid & 7), P.T);
        }
        __syncthreads();
#pragma unroll
        for (int p = 0; p < 4; ++p) {
          *reinterpret_cast<f32x4*>(ldsA + ((tid >> 3) + 32 * p) * BW_PA_M + 4 * (tid & 7)) = ra[p];
          *reinterpret_cast<f32x4*>(ldsB + ((tid >> 3) + 32 * p) * BW_PA_M + 4 * (tid & 7)) = rb[p];
        }
        __syncthreads();
        multiply();
      }
    }
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
      for (int ni = 0; ni < 2; ++ni) {
        const int k = k0 + wn * 64 + ni * 32 + r32;
        if (k >= P.F) continue;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int m = m0 + wm * 64 + mi * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
          if (m < P.n_mels) unsafeAtomicAdd(P.gW + (long long)m * P.F + k, acc[mi][ni][r]);
        }
      }
  }
}

// The filterbank from its logical layout W[n_mels][n_half + 1] into the forward kernel's fragment
// order [pass][row tile][row block][32-mel block][2][64 lanes] x float4 (lane (h, m) of quad v, element
// e holds mel pass*128 + mb*32 + m, bin rt*64 + rb*16 + 4 ((4 v + e) / 2) + 2 h + (4 v + e) % 2), the
// Nyquist-bin weights and the zero-padded row-major copy the backward pass reads.
__global__ void mel_from_logical_kernel(const float* __restrict__ w, float* __restrict__ frag, float* __restrict__ wnyq,
                                        float* __restrict__ wrm, int n_mels, int n_half, int n_rt, int n_pass, int fp,
                                        long long n4) {
  const long long i4 = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const int F = n_half + 1;
  if (i4 < (long long)n_mels * F) {  // row-major copy and Nyquist weights ride along on the first threads
    const int m = (int)(i4 / F), k = (int)(i4 - (long long)m * F);
    const float x = w[i4];
    wrm[(long long)m * fp + k] = x;
    if (k == n_half) wnyq[m] = x;
  }
  if (i4 >= n4) return;
  const int lane = (int)(i4 & 63), v = (int)((i4 >> 6) & 1), mb = (int)((i4 >> 7) % ST_MEL_BLOCKS);
  const long long rest = (i4 >> 7) / ST_MEL_BLOCKS;  // (pass * n_rt + rt) * ST_RB + rb
  const int rb = (int)(rest % ST_RB), rt = (int)((rest / ST_RB) % n_rt), pass = (int)(rest / ST_RB / n_rt);
  const int hh = lane >> 5, mel = pass * (32 * ST_MEL_BLOCKS) + mb * 32 + (lane & 31);
  f32x4 out;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int idx8 = v * 4 + e, bin = rt * (ST_ROWS / 2) + rb * 16 + 4 * (idx8 >> 1) + 2 * hh + (idx8 & 1);
    out[e] = (mel < n_mels && bin < n_half) ? w[(long long)mel * F + bin] : 0.f;
  }
  reinterpret_cast<f32x4*>(frag)[i4] = out;
  (void)n_pass;
}

// ---- spectral kernels of a trainable plan with frequency-domain constant-Q kernels -----------------------
// Entry (output row, packed spectrum column) of the second contraction's matrix: output rows 2q / 2q+1 = Re / Im
// of constant-Q bin q; packed columns 0, 1 = Re of the purely real bins 0 and n_half, 2s / 2s+1 = Re / Im of bin s.
//   Re X_cq += Xr Yr - Xi Yi,   Im X_cq += Xr Yi + Xi Yr      (eq. (CQT1992) in real arithmetic)
__device__ __forceinline__ float lin_entry(const float* __restrict__ ysk, int F, int n_half, int row, int col) {
  const int q = row >> 1, s = col == 0 ? 0 : col == 1 ? n_half : col >> 1;
  const bool im_part = col >= 2 && (col & 1);
  const float yr = ysk[(long long)(2 * q) * F + s], yi = ysk[(long long)(2 * q + 1) * F + s];
  return (row & 1) ? (im_part ? yr : yi) : (im_part ? -yi : yr);
}

__global__ void lin_from_logical_kernel(const LinLogicalParams P) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const int F = P.n_half + 1;
  if (i < P.n_frag) {
    // ((((((pass n_rt + rt) ST_RB + rb) lin_blocks + mb) 4 + v) 64 + lane) 4 + e
    const int e = (int)(i & 3), lane = (int)((i >> 2) & 63), v = (int)((i >> 8) & 3);
    long long rest = i >> 10;
    const int mb = (int)(rest % P.lin_blocks);
    rest /= P.lin_blocks;
    const int rb = (int)(rest % ST_RB);
    rest /= ST_RB;
    const int rt = (int)(rest % P.n_rt), pass = (int)(rest / P.n_rt);
    const int row = pass * 32 * P.lin_blocks + mb * 32 + (lane & 31);
    const int col = rt * ST_ROWS + rb * 32 + 8 * v + 4 * (lane >> 5) + e;
    P.frag[i] = (row < 2 * P.n_bins && col < 2 * P.n_half) ? lin_entry(P.ysk, F, P.n_half, row, col) : 0.f;
  }
  if (i < (long long)P.n_bins * F) {
    const int q = (int)(i / F), s = (int)(i - (long long)q * F);
    const float yr = P.ysk[(long long)(2 * q) * F + s], yi = P.ysk[(long long)(2 * q + 1) * F + s];
    float* a = P.ylin + (long long)(2 * q) * P.rp + 2 * s;
    a[0] = yr;
    a[1] = -yi;
    a[P.rp] = yi;
    a[P.rp + 1] = yr;
    float* t = P.ylinT + (long long)(2 * s) * P.mp + 2 * q;
    t[0] = yr;
    t[1] = yi;
    t[P.mp] = -yi;
    t[P.mp + 1] = yr;
  }
}

__global__ void lin_grad_kernel(const LinGradParams P) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= P.n) return;
  const long long per_wave = (long long)P.n_bins * P.T;
  const long long b = i / per_wave;
  const int q = (int)((i - b * per_wave) / P.T), t = (int)(i - b * per_wave - (long long)q * P.T);
  float* vr = P.v + (b * 2 * P.n_bins + 2 * q) * P.T + t;
  float* vi = vr + P.T;
  const float re = *vr, im = *vi, pw = re * re + im * im;
  const float* gp = P.gout + b * P.gout_wave_stride + t;
  float gr, gi;
  if (P.fmt == NNA_OUT_COMPLEX) {
    gr = gp[(2LL * q) * P.T];
    gi = gp[(2LL * q + 1) * P.T];
  } else if (P.fmt == NNA_OUT_PHASE) {  // d atan2(Im, Re) = (Re dIm - Im dRe) / P
    const float s = pw > 0.f ? gp[(long long)q * P.T] / pw : 0.f;
    gr = -s * im;
    gi = s * re;
  } else {
    const float go = gp[(long long)q * P.T];
    const float s = P.fmt == NNA_OUT_MAGNITUDE ? grad_scale<NNA_OUT_MAGNITUDE>(go, pw)
                    : P.fmt == NNA_OUT_POWER   ? grad_scale<NNA_OUT_POWER>(go, pw)
                                               : grad_scale<NNA_OUT_LOG>(go, pw);
    gr = s * re;
    gi = s * im;
  }
  *vr = gr;
  *vi = gi;
}

__global__ void lin_fold_gradient_kernel(const float* __restrict__ gylin, float* __restrict__ gysk, int n_bins, int F, int accumulate) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (long long)n_bins * F) return;
  const int q = (int)(i / F), s = (int)(i - (long long)q * F);
  const long long R = 2LL * F;
  const float* a = gylin + (2LL * q) * R + 2 * s;
  const float gr = a[0] + a[R + 1], gi = a[R] - a[1];
  float* o = gysk + (2LL * q) * F + s;
  if (accumulate) {
    o[0] += gr;
    o[F] += gi;
  } else {
    o[0] = gr;
    o[F] = gi;
  }
}

// ---- launchers ---------------------------------------------------------------------------------
static unsigned grid_for(long long n, int block) {
  long long b = (n + block - 1) / block;
  return (unsigned)(b < 1 ? 1 : b > 65535LL * 16 ? 65535LL * 16 : b);
}

hipError_t launch_fill_zero(float* p, long long n, hipStream_t stream) {
  clear_stale_error();
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(fill_zero_kernel, dim3(grid_for(n, 256 * 8)), dim3(256), 0, stream, p, n);
  return hipGetLastError();
}

hipError_t launch_fir_transpose_add(const FirTParams& p, hipStream_t stream) {
  clear_stale_error();
  if (p.L < 1 || p.Ln != (p.L + 1) / 2 || p.B < 1 || p.B > 65535 || p.L > 0x3fffffffLL || p.ne < FT_T || p.no < FT_T ||
      p.ne % FT_T || p.no % FT_T)
    return hipErrorInvalidValue;
  const int ext_e = p.ve0 + p.ne - 1, ext_o = p.vo0 + p.no - 1;
  const int span = (ext_e > ext_o ? ext_e : ext_o) - (p.ve0 < p.vo0 ? p.ve0 : p.vo0);
  if (span < 0 || span > FT_SPAN_MAX) return hipErrorInvalidValue;
  const long long tiles = (p.Ln + FT_TILE - 1) / FT_TILE;
  if (tiles > 0x7fffffffLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(fir_transpose_add_kernel, dim3((unsigned)tiles, (unsigned)p.B), dim3(256), 0, stream, p);
  return hipGetLastError();
}

// constant-Q bank of a trainable plan: the streaming-order bank through the plan's index map, and the
// row-major copy with everything outside a row's support forced to zero
__global__ void cqt_bank_from_logical_kernel(const CqtBankParams P) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i < P.n_bank) {
    const int src = P.map[i];
    P.bank[i] = src >= 0 ? P.logical[src] : 0.f;
  }
  if (i < (long long)P.rows * P.K) {
    const int row = (int)(i / P.K), k = (int)(i - (long long)row * P.K);
    P.wrm[(long long)row * P.kp + k] = (k >= P.row_lo[row] && k < P.row_hi[row]) ? P.logical[i] : 0.f;
  }
}

__global__ void cqt_bank_to_logical_kernel(const CqtBankParams P) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i < (long long)P.rows * P.K) {
    const int row = (int)(i / P.K), k = (int)(i - (long long)row * P.K);
    P.logical[i] = P.wrm[(long long)row * P.kp + k];
  }
}

hipError_t launch_cqt_bank_from_logical(const CqtBankParams& p, hipStream_t stream) {
  clear_stale_error();
  const long long n = std::max(p.n_bank, (long long)p.rows * p.K);
  if (n < 1 || (n + 255) / 256 > 0x7fffffffLL || (long long)p.rows * p.K > 0x7fffffffLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(cqt_bank_from_logical_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, p);
  return hipGetLastError();
}

hipError_t launch_cqt_bank_to_logical(const CqtBankParams& p, hipStream_t stream) {
  clear_stale_error();
  const long long n = (long long)p.rows * p.K;
  if (n < 1 || (n + 255) / 256 > 0x7fffffffLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(cqt_bank_to_logical_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, p);
  return hipGetLastError();
}

hipError_t launch_g_from_complex(float* gbuf, const float* gout, long long n_frames, int T, int out_rows, int rows_pad,
                                 int n_half, int packed, hipStream_t stream) {
  clear_stale_error();
  if (n_frames < 1 || T < 1 || rows_pad < 1 || 2 * n_half > rows_pad || (packed ? 2 * n_half + 1 : 2 * n_half) > out_rows)
    return hipErrorInvalidValue;
  const long long blocks = (n_frames + 31) / 32;
  if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(g_from_complex_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, gbuf, gout, n_frames, T, out_rows,
                     rows_pad, n_half, packed);
  return hipGetLastError();
}

hipError_t launch_fill_zero_frames(float* gbuf, long long rows_pad, long long f0, long long f1, hipStream_t stream) {
  clear_stale_error();
  if (rows_pad <= 0 || f1 <= f0) return hipSuccess;
  hipLaunchKernelGGL(fill_zero_frames_kernel, dim3(grid_for(rows_pad * (f1 - f0), 256)), dim3(256), 0, stream, gbuf, rows_pad, f0, f1);
  return hipGetLastError();
}

static long long bank_float4s(const BankPermuteParams& p) {
  return (long long)p.n_rt * p.n_chunks * p.nj * ST_NKG * ST_RB * 64;
}

hipError_t launch_bank_from_logical(const BankPermuteParams& p, hipStream_t stream) {
  clear_stale_error();
  const long long n4 = bank_float4s(p);
  if (n4 > 0x7fffffffLL * 256) return hipErrorInvalidValue;
  hipLaunchKernelGGL(bank_from_logical_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, stream, p, n4);
  return hipGetLastError();
}

hipError_t launch_bank_to_rowmajor(const BankPermuteParams& p, hipStream_t stream) {
  clear_stale_error();
  const long long n4 = bank_float4s(p);
  if (n4 > 0x7fffffffLL * 256) return hipErrorInvalidValue;
  hipLaunchKernelGGL(bank_to_rowmajor_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, stream, p, n4);
  return hipGetLastError();
}

hipError_t launch_bank_to_logical(const BankPermuteParams& p, hipStream_t stream) {
  clear_stale_error();
  const long long rows = 2LL * (p.packed ? p.n_half + 1 : p.n_half);
  const long long n = rows * p.K;
  hipLaunchKernelGGL(bank_to_logical_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, p, n);
  return hipGetLastError();
}

static bool bw_shapes_ok(const BwParams& p) {
  return p.rows_pad > 0 && p.rows_pad % BW_MT == 0 && p.kp > 0 && p.kp % BW_NT == 0 && p.gpitch > 0 &&
         p.gpitch % BW_MT == 0 && p.gpitch >= p.g.n_frames && p.K <= p.kp && 2 * p.n_half <= p.rows_pad;
}

hipError_t launch_bw_bank(const BwParams& p, hipStream_t stream) {
  clear_stale_error();
  if (!bw_shapes_ok(p) || p.n_split < 1 || p.chunks_per_split < 1) return hipErrorInvalidValue;
  if (p.chunks_per_split * p.n_split < p.gpitch / BW_KC) return hipErrorInvalidValue;
  const bool sparse = p.tiles != nullptr;
  if (sparse && (p.n_tiles < 1 || !p.row_lo || !p.row_hi)) return hipErrorInvalidValue;
  const long long tiles = sparse ? p.n_tiles : (long long)(p.rows_pad / BW_MT) * (p.kp / BW_NT);
  const long long blocks = tiles * p.n_split;
  if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  if (sparse)
    hipLaunchKernelGGL(bw_bank_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, stream, p);
  else
    hipLaunchKernelGGL(bw_bank_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, stream, p);
  return hipGetLastError();
}

hipError_t launch_bw_wave(const BwParams& p, hipStream_t stream) {
  clear_stale_error();
  if (!bw_shapes_ok(p)) return hipErrorInvalidValue;
  if (p.shift_rng) {
    if (p.n_shift < 1 || p.n_kc < 1 || p.n_kc > p.rows_pad / CW_KC || p.n_ct != (p.g.hop + BW_NT - 1) / BW_NT ||
        p.n_qt != (p.g.T + p.n_shift - 1 + BW_MT - 1) / BW_MT || (long long)p.n_shift * p.g.hop < p.K)
      return hipErrorInvalidValue;
    const long long blocks = p.g.B * p.n_qt * p.n_ct;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    if (p.g.hop % BW_NT == 0 && (long long)p.n_shift * p.g.hop <= p.kp)
      hipLaunchKernelGGL(cq_wave_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, stream, p);
    else
      hipLaunchKernelGGL(cq_wave_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, stream, p);
    return hipGetLastError();
  }
  const long long blocks = (p.gpitch / BW_MT) * (p.kp / BW_NT);
  if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(bw_wave_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, p);
  return hipGetLastError();
}

hipError_t launch_lin_from_logical(const LinLogicalParams& p, hipStream_t stream) {
  clear_stale_error();
  const long long n = std::max(p.n_frag, (long long)p.n_bins * (p.n_half + 1));
  if (n < 1 || (n + 255) / 256 > 0x7fffffffLL || p.lin_blocks < 1 || p.n_rt < 1) return hipErrorInvalidValue;
  if (p.mp < 2 * p.n_bins || p.rp < 2 * (p.n_half + 1)) return hipErrorInvalidValue;
  hipLaunchKernelGGL(lin_from_logical_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, p);
  return hipGetLastError();
}

hipError_t launch_lin_grad(const LinGradParams& p, hipStream_t stream) {
  clear_stale_error();
  if (p.n < 1 || (p.n + 255) / 256 > 0x7fffffffLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(lin_grad_kernel, dim3((unsigned)((p.n + 255) / 256)), dim3(256), 0, stream, p);
  return hipGetLastError();
}

hipError_t launch_lin_fold_gradient(const float* gylin, float* gysk, int n_bins, int F, int accumulate, hipStream_t stream) {
  clear_stale_error();
  const long long n = (long long)n_bins * F;
  if (n < 1) return hipErrorInvalidValue;
  hipLaunchKernelGGL(lin_fold_gradient_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, gylin, gysk, n_bins, F, accumulate);
  return hipGetLastError();
}

hipError_t launch_mel_bw_spec(const MelBwParams& p, hipStream_t stream) {
  clear_stale_error();
  if (p.fp <= 0 || p.fp % BW_MT || p.mels_pad % BW_KC || p.mels_pad < p.n_mels || p.F > p.fp || p.T < 1) return hipErrorInvalidValue;
  const long long blocks = p.B * (p.fp / BW_MT) * ((p.T + BW_NT - 1) / BW_NT);
  if (blocks < 1 || blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL((mel_bw_kernel<MEL_BW_SPEC>), dim3((unsigned)blocks), dim3(256), 0, stream, p);
  return hipGetLastError();
}

hipError_t launch_mel_bw_weights(const MelBwParams& p, hipStream_t stream) {
  clear_stale_error();
  if (p.fp <= 0 || p.fp % BW_NT || p.F > p.fp || p.T < 1 || p.b_per_split < 1) return hipErrorInvalidValue;
  const long long splits = (p.B + p.b_per_split - 1) / p.b_per_split;
  const long long blocks = splits * ((p.n_mels + BW_MT - 1) / BW_MT) * (p.fp / BW_NT);
  if (blocks < 1 || blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL((mel_bw_kernel<MEL_BW_WEIGHTS>), dim3((unsigned)blocks), dim3(256), 0, stream, p);
  return hipGetLastError();
}

hipError_t launch_mel_from_logical(const float* w, float* frag, float* wnyq, float* wrm, int n_mels, int n_half, int n_rt,
                                   int n_pass, int fp, hipStream_t stream) {
  clear_stale_error();
  const long long n4 = (long long)n_pass * n_rt * ST_RB * ST_MEL_BLOCKS * 2 * 64;
  const long long n = std::max(n4, (long long)n_mels * (n_half + 1));
  hipLaunchKernelGGL(mel_from_logical_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, w, frag, wnyq, wrm,
                     n_mels, n_half, n_rt, n_pass, fp, n4);
  return hipGetLastError();
}

}  // namespace nna
