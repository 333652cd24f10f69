// STFT / Mel contraction with the frame folded about its centre (gfx950 / CDNA4).
//
// For the plain DFT bank of eq. (DFT2) with a window that satisfies w[n] = w[N-n] (every window
// of Sec. III-A in its periodic form does), cos(2 pi k n / N) is even and sin(2 pi k n / N) odd
// about n = N/2, so with
//     e[n] = x[n] + x[N-n],   o[n] = x[n] - x[N-n]      (0 < n < N/2),   e[0] = x[0]
// the transform of one frame is
//     Re X[k] =  sum_{n < N/2} w[n] cos(2 pi k n / N) e[n]  +  w[N/2] (-1)^k x[N/2]
//     Im X[k] = -sum_{n < N/2} w[n] sin(2 pi k n / N) o[n]
// -- N/2 taps instead of N for every kernel: half the multiply-adds of the direct contraction, the
// same result up to rounding.  It applies to the kernels eq. (DFT2) defines, not to re-spaced
// frequency axes (sigma(k) is no integer) nor to trained kernels; those keep the direct kernel.
//
// Structure (the direct kernel's, see nna_kernels.hip, with these differences):
//  * A row tile is 64 bins as four 32-row blocks: Re of bins 0-31, Re of bins 32-63 (their B operand is
//    e), Im of bins 0-31, Im of bins 32-63 (B operand o).  (Re, Im) of a bin then sit in the same
//    register of the same lane in two accumulators.
//  * Two LDS tiles per chunk: S[r][c] = xp[sigma(r) hop + c0 + c] (as before, shifts j < J/2) and the
//    mirrored tile, which holds the partners xp[(sigma(r) + J/2) hop + hop - c0 - c] of the same 32 columns
//    in memory order (LDS column 31 - c).  The partner of taps (j, c..c+3) of the frame in row f is then one
//    aligned 16-byte read of row f + J/2 - 1 - j with its four elements taken back to front, and e / o
//    cost eight additions per sixteen MFMAs.  Tap 0 has no partner (x[N] belongs to the next frame): its
//    element is replaced by zero.
//  * Waveform rows are addressed as a uniform base plus a 32-bit byte offset per lane.  A wave all of whose
//    windows of a frame tile lie inside their waveforms (most tiles, most waves) keeps those offsets fixed
//    and moves the base from chunk to chunk; a wave that serves rows next to a waveform's end recomputes
//    them per chunk with the mirror classes of the direct kernel's loader.
//  * The w[N/2] (-1)^k x[N/2] term is added to the Re accumulators in the epilogue; the sign
//    alternates with the accumulator register index.
//  * Bin N/2 (purely real, sum_n (-1)^n w[n] x[n]) is no row of any tile.  The STFT launch carries one
//    extra workgroup per frame tile that computes it on the vector ALUs from per-hop-segment partial
//    sums (each sample read once); the Mel launch needs it only when a filter has weight on that bin,
//    in which case the direct kernel runs instead.
//  * The tiles of chunk it+1 are fetched and written while chunk `it` is multiplied: S requested in
//    fragment group 0 and written in group 3, the mirrored tile requested in group 4 and written in group 7,
//    through the same five registers (a chunk has 4 J/2 >= 8 groups).  Cycle counters read inside the loop
//    put the wait for a tile at under 20 cycles per chunk; requesting two chunks ahead through a second
//    register set changed nothing.
//  * Launches split by tap parity with J = 4 visit the chunks of a row tile in mirrored pairs and stage two forward
//    windows instead of a forward and a mirrored tile (template argument PAIR, described at the kernel).
#include "nna_device.h"

#include <type_traits>
#include <utility>

namespace nna {

// Four floats from p, which lies one float past a 16-byte boundary: the aligned quad below it (its last three) and one
// float more -- a 16-byte read from a 4-byte boundary becomes two 8-byte reads whose lanes collide on the LDS banks.
__device__ __forceinline__ f32x4 mirrored4(const float* p) {
  const f32x4 lo = *reinterpret_cast<const f32x4*>(p - 1);
  return (f32x4){lo.y, lo.z, lo.w, p[3]};
}

constexpr int SF_RPP = 256 / (ST_KC / 4);                      // LDS rows written per loader pass (32)
constexpr int SF_NPASS = (SF_LDS_ROWS + SF_RPP - 1) / SF_RPP;  // 5; the last pass is partial
constexpr int SF_TILE = SF_LDS_ROWS * ST_PITCH;                // floats per tile

// Rows of the two tiles as this thread serves them, one per loader pass.
struct FoldRows {
  int roff[SF_NPASS];  // first sample of the row's waveform, in samples from the tile's first waveform
  int i0s[SF_NPASS];   // S tile: padded-signal index of this thread's first column, chunk 0
  int i0m[SF_NPASS];   // mirrored tile: the same, chunk 0 (chunk c0 lies c0 samples lower)
};

// Byte offsets (from the first waveform of the tile) of the NPASS windows of a chunk and how to fix the data
// up, for a wave that has windows outside their waveforms: the direct loader's classes (nna_device.h).
__device__ __forceinline__ void fold_offsets(unsigned (&off)[SF_NPASS], TileFix<SF_NPASS>& fx, int L, const int (&roff)[SF_NPASS],
                                             const int (&i0row)[SF_NPASS], int shift) {
  unsigned rev = 0;
  bool gen = false;
#pragma unroll
  for (int p = 0; p < SF_NPASS; ++p) {
    const int i0 = i0row[p] + shift;
    int src = i0;
    if (i0 < 0) src = -i0 - 3;
    else if (i0 > L - 4) src = 2 * (L - 1) - i0 - 3;
    rev |= (src != i0 ? 1u : 0u) << p;
    gen |= (unsigned)src > (unsigned)(L - 4);
    off[p] = (unsigned)(roff[p] + src) << 2;
  }
  fx.rev = rev;
  fx.cls = __builtin_amdgcn_ballot_w64(rev != 0) != 0 ? 1 : 0;
  if (__builtin_amdgcn_ballot_w64(gen) != 0) {
    fx.cls = 2;
#pragma unroll
    for (int p = 0; p < SF_NPASS; ++p) {
      const int i0 = i0row[p] + shift;
      const int i_0 = reflect_clamped(i0, L), i_1 = reflect_clamped(i0 + 1, L);
      const int i_2 = reflect_clamped(i0 + 2, L), i_3 = reflect_clamped(i0 + 3, L);
      int w0 = min(min(i_0, i_1), min(i_2, i_3));
      w0 = min(w0, L - 4);
      off[p] = (unsigned)(roff[p] + w0) << 2;
      fx.sel[p] = (unsigned)min(i_0 - w0, 3) | ((unsigned)min(i_1 - w0, 3) << 2) | ((unsigned)min(i_2 - w0, 3) << 4) |
                  ((unsigned)min(i_3 - w0, 3) << 6);
    }
  }
}

// whole-tile LDS write of a tile with SF_LDS_ROWS rows (prologue, and class 2 in the main loop)
__device__ __forceinline__ void sf_store_chunk(const f32x4 (&R)[SF_NPASS], const TileFix<SF_NPASS>& fx, float* lds, int tid) {
  store_chunk<ST_KC, ST_PITCH, SF_NPASS>(R, fx, lds, SF_LDS_ROWS, tid);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
  return v;
}

// Bin N/2 of one frame tile: X[N/2] = sum_n (-1)^n w[n] xp[t hop + n], from partial sums over whole hop
// segments, P[row][q] = sum_{c < hop} wn[q hop + c] xp[sigma(row) hop + c] (wn = (-1)^n w[n]), so that
// every sample is read once: X_t[N/2] = sum_q P[row(t) + q][q].
// A launch split by tap parity has bin N/2 in its contraction and leaves out bin N/4 instead (its own partner):
// X[N/4] = sum_n w[n] (cos(pi n / 2) - i sin(pi n / 2)) xp[t hop + n], two real sums of the same kind, taken one after the
// other with the weight tables wn[0] (real part) and wn[1] (imaginary part).
// Power of that bin for frame f0 + tid of frame tile ft (threads tid < the tile's frames; 0 elsewhere).  Every
// thread of the workgroup must call it; `lds` is used from its start.
__device__ float extra_bin_power(const StftParams& P, long long ft, float* lds) {
  const FrameGeom& g = P.g;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int J = 2 * P.nj;  // P.nj holds J/2 for a folded launch
  const int Jp = (J + 3) & ~3;  // the segments' weights go four at a time (the table is zero padded)
  const int hop = g.hop;
  const long long f0 = ft * P.tile_frames;
  if (f0 >= g.n_frames) return 0.f;  // (the whole workgroup)
  const int m_valid = (int)((g.n_frames - f0) < P.tile_frames ? (g.n_frames - f0) : P.tile_frames);
  TileMap tm;
  tm.T = g.T;
  tm.b0 = f0 / g.T;
  tm.t0 = (int)(f0 - tm.b0 * g.T);
  tm.n0 = (g.T - tm.t0) < m_valid ? (g.T - tm.t0) : m_valid;
  tm.extra = J - 1;
  const int rows_used = tm.frame_row(m_valid - 1) + tm.extra + 1;
  const int L = (int)g.L;
  // LDS: the weights [Jp][hop] (read by every row), then the partial sums [rows][Jp]
  float* wl = lds;
  float* ps = lds + Jp * hop;
  float part[2] = {0.f, 0.f};
  const int n_part = P.split ? 2 : 1;
  for (int pt = 0; pt < n_part; ++pt) {
  if (pt) __syncthreads();  // everyone is done with the first table and its partial sums
  for (int i = tid * 4; i < Jp * hop; i += 1024)
    *reinterpret_cast<f32x4*>(wl + i) = *reinterpret_cast<const f32x4*>(P.wn + (long long)pt * Jp * hop + i);
  __syncthreads();
  // eight lanes share a row (each four consecutive columns of every 32), a wave eight rows, the workgroup 32 rows
  // per step; the loads of eight column blocks are issued together
  const int sub = lane & 7, rw = lane >> 3;
  for (int row0 = 0; row0 < rows_used; row0 += 32) {
    const int row = row0 + wave * 8 + rw;
    long long b;
    int sigma;
    tm.decode(row, b, sigma);
    const bool ok = row < rows_used && b < g.B;
    const float* __restrict__ xb = g.x + (ok ? b : 0) * g.L;
    const int base = ok ? sigma * hop - g.pad : 0;
    const bool vec = g.vec_ok && base >= 0 && base + hop <= L;
    for (int q0 = 0; q0 < Jp; q0 += 4) {
      f32x4 sum[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) sum[u] = (f32x4){0.f, 0.f, 0.f, 0.f};
      for (int c0 = 0; c0 < hop; c0 += 256) {
        f32x4 v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const int c = c0 + 32 * i + 4 * sub;
          if (c >= hop) {
            v[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
          } else if (vec) {
            v[i] = *reinterpret_cast<const f32x4*>(xb + base + c);
          } else {
            v[i] = (f32x4){xb[reflect_clamped(base + c, L)], xb[reflect_clamped(base + c + 1, L)],
                           xb[reflect_clamped(base + c + 2, L)], xb[reflect_clamped(base + c + 3, L)]};
          }
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const int c = c0 + 32 * i + 4 * sub;
          if (c < hop) {
#pragma unroll
            for (int u = 0; u < 4; ++u) sum[u] += v[i] * *reinterpret_cast<const f32x4*>(wl + (q0 + u) * hop + c);
          }
        }
      }
      f32x4 r;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        float t = sum[u].x + sum[u].y + sum[u].z + sum[u].w;
        t += __shfl_xor(t, 1, 64);
        t += __shfl_xor(t, 2, 64);
        t += __shfl_xor(t, 4, 64);
        r[u] = t;
      }
      if (sub == 0 && row < rows_used) *reinterpret_cast<f32x4*>(ps + row * Jp + q0) = r;
    }
  }
  __syncthreads();
  if (tid < m_valid) {
    const float* src = ps + tm.frame_row(tid) * Jp;
    float re = 0.f;
    for (int q = 0; q < J; ++q) re += src[q * Jp + q];
    part[pt] = re;
  }
  }
  return part[0] * part[0] + part[1] * part[1];
}

__device__ void nyquist_tile(const StftParams& P, long long ft, float* lds) {
  const FrameGeom& g = P.g;
  const int tid = threadIdx.x;
  const long long f0 = ft * P.tile_frames;
  if (f0 >= g.n_frames) return;
  const int m_valid = (int)((g.n_frames - f0) < P.tile_frames ? (g.n_frames - f0) : P.tile_frames);
  const float pw = extra_bin_power(P, ft, lds);
  if (tid < m_valid) {
    const long long f = f0 + tid;
    const long long b = f / g.T;
    const int t = (int)(f - b * g.T);
    float* op = P.out + (b * P.out_bins + (P.split ? P.n_half / 2 : P.n_half)) * g.T + t;
    *op = P.fmt == NNA_OUT_MAGNITUDE ? format_power<NNA_OUT_MAGNITUDE>(pw)
          : P.fmt == NNA_OUT_POWER   ? pw
                                     : format_power<NNA_OUT_LOG>(pw);
  }
}

// Output of one finished row tile: 64 bins x this wave's 32 frames.  `op` points at (waveform, bin 0,
// frame) of this lane; register r of lane (h, n) in block blk is bin slot_base + 32 blk + 8 (r/4) + 4 h + r%4.
template <int FMT>
__device__ __forceinline__ void fold_store_tile(const f32x16 (&acc)[ST_RB], float* __restrict__ op, long long T,
                                                int slot_base, int h, int n_half) {
  float* __restrict__ p = op + (slot_base + 4 * h) * T;
  if (slot_base + ST_ROWS / 2 <= n_half) {
#pragma unroll
    for (int blk = 0; blk < 2; ++blk)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float re = acc[blk][r], im = acc[blk + 2][r];
        p[(32 * blk + 8 * (r >> 2) + (r & 3)) * T] = format_power<FMT>(re * re + im * im);
      }
  } else {
#pragma unroll
    for (int blk = 0; blk < 2; ++blk)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float re = acc[blk][r], im = acc[blk + 2][r];
        const int k = 32 * blk + 8 * (r >> 2) + (r & 3);
        if (slot_base + 4 * h + k < n_half) p[k * T] = format_power<FMT>(re * re + im * im);
      }
  }
}

// The split launch's row tile: bins k = slot_base + .. (from E + O) and their partners N/2 - k (from E - O).  Blocks
// 0-3 = the even taps' (Re 0-31, Re 32-63, Im 0-31, Im 32-63), blocks 4-7 = the odd taps'.
template <int FMT>
__device__ __forceinline__ void fold_store_tile_split(const f32x16 (&acc)[2 * ST_RB], float* __restrict__ op, long long T,
                                                      int slot_base, int h, int n_half) {
  float* __restrict__ p = op + (slot_base + 4 * h) * T;
  float* __restrict__ pm = op + (long long)(n_half - slot_base - 4 * h) * T;
#pragma unroll
  for (int blk = 0; blk < 2; ++blk)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float re_e = acc[blk][r], im_e = acc[blk + 2][r], re_o = acc[blk + 4][r], im_o = acc[blk + 6][r];
      const int k = 32 * blk + 8 * (r >> 2) + (r & 3);
      const float a = re_e + re_o, b = im_e + im_o, c = re_e - re_o, d = im_e - im_o;
      p[k * T] = format_power<FMT>(a * a + b * b);
      pm[-k * T] = format_power<FMT>(c * c + d * d);
    }
}

// MODE: ST_MODE_STFT (per-bin epilogue) or ST_MODE_MEL (power of the row tile x filterbank slice).
// SPLIT (ST_MODE_STFT, N a multiple of 256, even hop): one more halving.  cos(2 pi (N/2 - k) n / N) =
// (-1)^n cos(2 pi k n / N) and sin(2 pi (N/2 - k) n / N) = -(-1)^n sin(2 pi k n / N), so with the folded taps summed
// separately by parity -- E over even n, O over odd n -- bin k is E + O and bin N/2 - k is E - O (imaginary part:
// -(E - O)): only the kernels of the bins below N/4 are multiplied, into two sets of accumulators.  In a fragment of four
// consecutive taps element e has the parity of e, and both halves of a two-tap MFMA step hold taps of one parity, so
// the split is a choice of accumulator per MFMA.  The centre tap n = N/2 is even; bin N/4, its own partner, is
// left to the workgroups behind the contraction's, and bin N/2 = partner of bin 0 needs none.
// The Mel variant has no registers for eight accumulator blocks beside the filterbank's four.  Its split form works
// on row tiles of 32 bins instead: two bank fragments per group (Re, Im of bins 0-31 of the tile) into four blocks
// (even taps: Re, Im; odd taps: Re, Im); the power of the 32 bins and of their 32 partners then meets the filterbank
// slices of both.  Bin N/4 is computed by the workgroup itself after its sweep (extra_bin_power) and weighed in.
// PAIR: the chunks of a row tile are visited in pairs ca = k, cb = n_chunks - 1 - k.  The partners N - n of chunk ca's
// taps are the columns hop - 32 ca - c = 32 cb + 32 - c of rows J/2 further on: chunk cb's own columns moved up by one.
// So both tiles of a step are plain windows, A = columns 32 ca .. 32 ca + 32 and B = columns 32 cb .. 32 cb + 32 (33
// columns: the last in the pitch's padding), each the forward window of one chunk and the mirrored one of the other,
// and a step multiplies both chunks: half the tile loads and twice the MFMAs per barrier.  The mirrored reads start one
// column off a 16-byte boundary (two 8-byte LDS reads instead of one of 16).  Rows: a frame's partners lie up to
// J - 1 rows below it (J/2 - 1 when the mirrored tile was stored J/2 rows on), so the launcher sizes the tile for that.
template <int MODE, int RING, bool SPLIT = false, bool PAIR = false>
__global__ __launch_bounds__(256, 2) void stft_fold_kernel(const StftParams P) {
  static_assert(ST_NKG % RING == 0, "ring depth must divide the fragment groups per LDS row");
  static_assert(!PAIR || SPLIT, "pairs of chunks: split launches only");
  constexpr bool MEL = MODE == ST_MODE_MEL;
  constexpr int FR = MEL && SPLIT ? 2 : ST_RB;          // bank fragments per group
  constexpr int NACC = SPLIT ? (MEL ? 4 : 2 * ST_RB) : ST_RB;
  constexpr int TILE_BINS = MEL && SPLIT ? 32 : ST_ROWS / 2;
  constexpr int NPASS = SF_NPASS;
  __shared__ __attribute__((aligned(16))) float lds[2][2][SF_TILE];  // [buffer][S, M]

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
  } else {
    if ((long long)blockIdx.x >= P.main_blocks) {  // the workgroups behind the contraction's: bin N/2
      nyquist_tile(P, (long long)blockIdx.x - P.main_blocks, &lds[0][0][0]);
      return;
    }
    // XCD-aware order, as in the direct kernel: ids are dealt round-robin to the 8 XCDs, each XCD walks its
    // own range of frame tiles in groups of 64 with the row group as the slow index
    constexpr int GROUP = 64;
    constexpr int RG = 4;  // row tiles per workgroup
    const int n_rg = (P.n_rt + RG - 1) / RG;
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
    ft = xcd * ft_per_xcd + grp_first + fi;
    if (ft >= P.n_ft) return;
    rt_begin = rg * RG;
    rt_end = rt_begin + RG < P.n_rt ? rt_begin + RG : P.n_rt;
  }

  const FrameGeom& g = P.g;
  const int nj2 = P.nj;  // hop-shifts of the folded frame: J / 2
  const long long f0 = ft * P.tile_frames;
  const int m_valid = (int)((g.n_frames - f0) < P.tile_frames ? (g.n_frames - f0) : P.tile_frames);
  TileMap tm;
  tm.T = g.T;
  tm.b0 = f0 / g.T;
  tm.t0 = (int)(f0 - tm.b0 * g.T);
  tm.n0 = (g.T - tm.t0) < m_valid ? (g.T - tm.t0) : m_valid;
  tm.extra = PAIR ? 2 * nj2 - 1 : nj2 - 1;
  const int rows_used = tm.frame_row(m_valid - 1) + tm.extra + 1;

  const int n_chunks = P.n_chunks;
  const int n_steps = PAIR ? n_chunks / 2 : n_chunks;  // barriers per row tile
  const int total = (rt_end - rt_begin) * n_steps;
  if (total <= 0) return;

  // Row descriptors of the two tiles.  S: sample sigma hop + 4 cv - pad (+ c0).  Mirrored tile: LDS column d
  // holds sample (sigma + J/2) hop + hop - 31 + d - pad (- c0): the partners of columns 31 - d.
  FoldRows rows;
  const char* const xbase = reinterpret_cast<const char*>(g.x + tm.b0 * g.L);
  const int L = (int)g.L;
  bool fast;
  {
    const int cv = tid % (ST_KC / 4), r0 = tid / (ST_KC / 4);
    const int smax = (n_chunks - 1) * ST_KC;  // first column of the last chunk
    bool bad = false;
#pragma unroll
    for (int p = 0; p < NPASS; ++p) {
      const int row = p * SF_RPP + r0;
      long long b;
      int sigma;
      tm.decode(row, b, sigma);
      const bool ok = row < rows_used && b < g.B;
      // a row nobody reads: any window inside the first waveform will do
      rows.roff[p] = ok ? (int)((b - tm.b0) * g.L) : 0;
      rows.i0s[p] = ok ? sigma * g.hop + 4 * cv - g.pad : 0;
      rows.i0m[p] = ok ? (sigma + nj2 + 1) * g.hop - (ST_KC - 1) + 4 * cv - g.pad : g.hop;
      if constexpr (PAIR)
        bad |= rows.i0s[p] < 0 || rows.i0s[p] + smax > L - 4;
      else
        bad |= rows.i0s[p] < 0 || rows.i0s[p] + smax > L - 4 || rows.i0m[p] - smax < 0 || rows.i0m[p] > L - 4;
    }
    fast = __builtin_amdgcn_ballot_w64(bad) == 0;  // every window of every chunk of this wave is a stored window
  }
  // PAIR: column 32 of LDS row `tid` (threads below SF_LDS_ROWS), one sample per row and tile
  int roff33 = 0, i033 = 0;
  if constexpr (PAIR) {
    if (tid < SF_LDS_ROWS) {
      long long b;
      int sigma;
      tm.decode(tid, b, sigma);
      const bool ok = tid < rows_used && b < g.B;
      roff33 = ok ? (int)((b - tm.b0) * g.L) : 0;
      i033 = ok ? sigma * g.hop + ST_KC - g.pad : 0;
    }
  }

  // this lane's frame
  const int fi_lane = wave * 32 + n;
  const bool valid = fi_lane < m_valid;
  const long long f_lane = f0 + fi_lane;
  const long long b_lane = valid ? f_lane / g.T : 0;
  const int t_lane = valid ? (int)(f_lane - b_lane * g.T) : 0;
  const int row_lane = valid ? tm.frame_row(fi_lane) : 0;
  const int s_off = row_lane * ST_PITCH + 4 * h;
  // columns run backwards (PAIR: relative to the tile that serves as the mirrored one; taps c .. c + 3 pair with its
  // columns 32 - c .. 29 - c)
  const int m_off = PAIR ? (row_lane + 2 * nj2 - 1) * ST_PITCH + (ST_KC - 3) - 4 * h
                         : SF_TILE + (row_lane + nj2 - 1) * ST_PITCH + (ST_KC - 4) - 4 * h;
  // w[N/2] x[N/2] of this lane's frame (the unpaired centre tap)
  float xmid = 0.f;
  if (valid) xmid = g.x[b_lane * g.L + reflect_clamped(t_lane * g.hop + nj2 * g.hop - g.pad, L)] * P.wmid;
  asm volatile("s_waitcnt vmcnt(0)" : "+v"(xmid));

  const int groups_per_rt = n_chunks * nj2 * ST_NKG;

  f32x16 acc[NACC];
#pragma unroll
  for (int rb = 0; rb < NACC; ++rb)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[rb][r] = 0.f;

  f32x16 macc[MEL ? ST_MEL_BLOCKS : 1];
  if constexpr (MEL) {
#pragma unroll
    for (int mb = 0; mb < ST_MEL_BLOCKS; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) macc[mb][r] = 0.f;
  }

  // ---- prologue: both tiles of chunk 0 into LDS buffer 0, first RING bank groups requested ----------
  f32x4 R[NPASS];
  float r33 = 0.f;  // PAIR: the tile's column 32 of this thread's row
  TileFix<NPASS> fx;
  // byte offset of the column-32 sample of a tile whose first column is `shift`
  auto off33 = [&](int shift) { return (unsigned)(roff33 + reflect_clamped(i033 + shift, L)) << 2; };
  {
    unsigned off[NPASS];
    fold_offsets(off, fx, L, rows.roff, rows.i0s, 0);
#pragma unroll
    for (int p = 0; p < NPASS; ++p) gload16_s<0>(R[p], off[p], xbase);
    if constexpr (PAIR) {
      gload4_s(r33, off33(0), xbase);
      wait_vm<0>(R, r33);
      if (tid < SF_LDS_ROWS) lds[0][0][tid * ST_PITCH + ST_KC] = r33;
    } else {
      wait_vm<0>(R);
    }
    sf_store_chunk(R, fx, &lds[0][0][0], tid);
    const int shiftB = (n_chunks - 1) * ST_KC;  // PAIR: tile B is the last chunk's window
    if constexpr (PAIR)
      fold_offsets(off, fx, L, rows.roff, rows.i0s, shiftB);
    else
      fold_offsets(off, fx, L, rows.roff, rows.i0m, 0);
#pragma unroll
    for (int p = 0; p < NPASS; ++p) gload16_s<0>(R[p], off[p], xbase);
    if constexpr (PAIR) {
      gload4_s(r33, off33(shiftB), xbase);
      wait_vm<0>(R, r33);
      if (tid < SF_LDS_ROWS) lds[0][1][tid * ST_PITCH + ST_KC] = r33;
    } else {
      wait_vm<0>(R);
    }
    sf_store_chunk(R, fx, &lds[0][1][0], tid);
  }

  const unsigned lane_off = (unsigned)lane * 16u;
  const char* bank_s = reinterpret_cast<const char*>(P.bankf) + ((long long)rt_begin * groups_per_rt) * (FR * 64 * 16);
  f32x4 bq[RING][FR];
#pragma unroll
  for (int s = 0; s < RING; ++s) {
    gload16_s<0>(bq[s][0], lane_off, bank_s);
    gload16_s<1024>(bq[s][1], lane_off, bank_s);
    if constexpr (FR == 4) {
      gload16_s<2048>(bq[s][2], lane_off, bank_s);
      gload16_s<3072>(bq[s][3], lane_off, bank_s);
    }
    bank_s += FR * 64 * 16;
  }
  __syncthreads();

  // Loads retire in order.  When a group starts, the requests younger than its own ring slot are at least
  // the other RING-1 slots (tile requests in between only make the wait stricter).  A tile is requested
  // during one group and written three groups later: the three groups in between each re-request one ring
  // slot (FR loads), so at least 3 FR requests are younger than the tile's.
  constexpr int W_SLOT = (RING - 1) * FR;
  // (split launches: of the group that requests the tile only the quads re-requested behind the tile's last load count)
  constexpr int W_TILE = SPLIT ? 2 * FR + (FR == 4 ? 2 : 1) : 3 * FR;
  constexpr int TASK_NONE = 0, TASK_LOAD_S = 1, TASK_STORE_S = 2, TASK_LOAD_M = 3, TASK_STORE_M = 4;
  const int stage_off = (tid / (ST_KC / 4)) * ST_PITCH + (tid % (ST_KC / 4)) * 4;
  const bool last_pass_row = tid / (ST_KC / 4) < SF_LDS_ROWS - (NPASS - 1) * SF_RPP;  // the partial fifth pass

  int c = 0;  // chunk inside the current row tile
  int rt = rt_begin;
  for (int it = 0; it < total; ++it) {
    const float* cur = &lds[it & 1][0][0];
    float* const nxt = &lds[(it + 1) & 1][0][0];
    // first column of chunk it+1 (PAIR: of the next step's chunk in tile A; tile B's is n_chunks - 1 minus that chunk)
    const int c_next = (c + 1 == n_steps ? 0 : c + 1) * ST_KC;
    const int c_next_b = (n_chunks - 1) * ST_KC - c_next;
    const bool first_chunk = c == 0;

    f32x4 s_cur = *reinterpret_cast<const f32x4*>(cur + s_off);
    f32x4 m_cur;
    if constexpr (PAIR)
      m_cur = mirrored4(cur + SF_TILE + m_off);
    else
      m_cur = *reinterpret_cast<const f32x4*>(cur + m_off);
    if (first_chunk && h == 0) m_cur.w = 0.f;  // tap 0 (the last element: columns run backwards) has no partner

    // sweep_tag (PAIR): 0 = chunk ca (forward window in tile A, mirrored in B), 1 = chunk cb (the other way round)
    auto group = [&](auto task_tag, int jj, auto kg_tag, auto sweep_tag) {
      constexpr int TASK = decltype(task_tag)::value;
      constexpr int kg = decltype(kg_tag)::value;
      constexpr int SW = decltype(sweep_tag)::value;
      constexpr int s = kg % RING;
      // the fragments of the next group are read from LDS while this group's MFMAs run
      const bool last_of_sweep = !(kg + 1 < ST_NKG) && !(jj + 1 < nj2);
      const int nj_ = kg + 1 < ST_NKG ? jj : (jj + 1 < nj2 ? jj + 1 : 0);
      const int nk_ = kg + 1 < ST_NKG ? (kg + 1) * ST_KG : 0;
      f32x4 s_nxt, m_nxt;
      if constexpr (PAIR) {
        const int sw_n = last_of_sweep ? SW ^ 1 : SW;  // (after sweep 1 the next step reads its own first fragments)
        s_nxt = *reinterpret_cast<const f32x4*>(cur + (sw_n ? SF_TILE : 0) + s_off + nj_ * ST_PITCH + nk_);
        m_nxt = mirrored4(cur + (sw_n ? 0 : SF_TILE) + m_off - nj_ * ST_PITCH - nk_);
      } else {
        s_nxt = *reinterpret_cast<const f32x4*>(cur + s_off + nj_ * ST_PITCH + nk_);
        m_nxt = *reinterpret_cast<const f32x4*>(cur + m_off - nj_ * ST_PITCH - nk_);
      }
      const f32x4 m_rev = {m_cur.w, m_cur.z, m_cur.y, m_cur.x};
      const f32x4 ev = s_cur + m_rev, ov = s_cur - m_rev;
      constexpr bool M_ = TASK == TASK_LOAD_M || TASK == TASK_STORE_M;  // which tile a staging task is about
      unsigned off[NPASS];
      const char* sb = xbase;
      // PAIR: both tiles are forward windows, the second one of the chunk that mirrors the first
      const int shift = PAIR ? (M_ ? c_next_b : c_next) : (M_ ? -c_next : c_next);
      if constexpr (TASK == TASK_LOAD_S || TASK == TASK_LOAD_M) {
        if (fast) {  // the lanes' offsets stay, the base moves with the chunk
#pragma unroll
          for (int p = 0; p < NPASS; ++p) off[p] = (unsigned)(rows.roff[p] + (M_ && !PAIR ? rows.i0m[p] : rows.i0s[p])) << 2;
          sb = xbase + 4 * shift;
          fx.cls = 0;
          fx.rev = 0;
        } else {
          fold_offsets(off, fx, L, rows.roff, M_ && !PAIR ? rows.i0m : rows.i0s, shift);
        }
      }
      float* stage_dst = nxt + stage_off + (M_ ? SF_TILE : 0);
      if constexpr (TASK == TASK_STORE_S || TASK == TASK_STORE_M) {
        if constexpr (PAIR)
          wait_vm<W_TILE>(R, r33);
        else
          wait_vm<W_TILE>(R);
        if (fx.cls == 2) sf_store_chunk(R, fx, nxt + (M_ ? SF_TILE : 0), tid);
      }
      if constexpr (FR == 4)
        wait_vm<W_SLOT>(bq[s][0], bq[s][1], bq[s][2], bq[s][3]);
      else
        wait_vm<W_SLOT>(bq[s][0], bq[s][1]);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int m = 0; m < 4 * FR; ++m) {
        // Split launches take a fragment quad's four taps in a row (even and odd taps go to different accumulators, so
        // consecutive MFMAs do not depend on each other) and re-request the quad right behind its fourth: the request
        // is out up to three quarters of a group earlier than when every quad's last tap comes in the last quarter.
        const int e = SPLIT ? m % 4 : m / FR, rb = SPLIT ? m / 4 : m % FR;
        const int ab = SPLIT && (e & 1) ? rb + FR : rb;  // odd taps: the second set
        acc[ab] = __builtin_amdgcn_mfma_f32_32x32x2f32(bq[s][rb][e], rb < FR / 2 ? ev[e] : ov[e], acc[ab], 0, 0, 0);
        // a staging task's NPASS steps go one behind every other MFMA (behind each of the first NPASS, where a group has eight)
        if (TASK != TASK_NONE && (FR == 4 ? (m & 1) && (m >> 1) < NPASS : m < NPASS)) {
          const int p = FR == 4 ? m >> 1 : m;
          __builtin_amdgcn_sched_barrier(0);
          if constexpr (TASK == TASK_STORE_S || TASK == TASK_STORE_M) {
            if (fx.cls != 2 && (p < NPASS - 1 || last_pass_row))
              *reinterpret_cast<f32x4*>(stage_dst + p * SF_RPP * ST_PITCH) = fixed_up<NPASS>(R[p], fx, p);
          } else {
            gload16_s<0>(R[p], off[p], sb);
          }
          __builtin_amdgcn_sched_barrier(0);
        }
        // PAIR: the tile's 33rd column, one step behind its last pass
        if (PAIR && TASK != TASK_NONE && m == (FR == 4 ? 2 * NPASS + 1 : NPASS)) {
          __builtin_amdgcn_sched_barrier(0);
          if constexpr (TASK == TASK_STORE_S || TASK == TASK_STORE_M) {
            if (tid < SF_LDS_ROWS) nxt[(M_ ? SF_TILE : 0) + tid * ST_PITCH + ST_KC] = r33;
          } else {
            gload4_s(r33, off33(shift), xbase);
          }
          __builtin_amdgcn_sched_barrier(0);
        }
        if (SPLIT ? (m & 3) == 3 : m >= 3 * FR) {
          // this MFMA was the last reader of fragment quad rb: re-request it (the group RING ahead; the
          // bank allocation is padded by ST_NKG groups, so the tail stays in bounds)
          __builtin_amdgcn_sched_barrier(0);
          if (rb == 0) gload16_s<0>(bq[s][0], lane_off, bank_s);
          if (rb == 1) gload16_s<1024>(bq[s][1], lane_off, bank_s);
          if constexpr (FR == 4) {
            if (rb == 2) gload16_s<2048>(bq[s][2], lane_off, bank_s);
            if (rb == 3) gload16_s<3072>(bq[s][3], lane_off, bank_s);
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      bank_s += FR * 64 * 16;
      s_cur = s_nxt;
      m_cur = m_nxt;
    };
    using K0 = std::integral_constant<int, 0>;
    using K1 = std::integral_constant<int, 1>;
    using K2 = std::integral_constant<int, 2>;
    using K3 = std::integral_constant<int, 3>;
    using TN = std::integral_constant<int, TASK_NONE>;
    using TLS = std::integral_constant<int, TASK_LOAD_S>;
    using TSS = std::integral_constant<int, TASK_STORE_S>;
    using TLM = std::integral_constant<int, TASK_LOAD_M>;
    using TSM = std::integral_constant<int, TASK_STORE_M>;
    using W0 = std::integral_constant<int, 0>;
    using W1 = std::integral_constant<int, 1>;
    group(TLS{}, 0, K0{}, W0{});
    group(TN{}, 0, K1{}, W0{});
    group(TN{}, 0, K2{}, W0{});
    group(TSS{}, 0, K3{}, W0{});
    group(TLM{}, 1, K0{}, W0{});
    group(TN{}, 1, K1{}, W0{});
    group(TN{}, 1, K2{}, W0{});
    group(TSM{}, 1, K3{}, W0{});
    for (int jj = 2; jj < nj2; ++jj) {
      group(TN{}, jj, K0{}, W0{});
      group(TN{}, jj, K1{}, W0{});
      group(TN{}, jj, K2{}, W0{});
      group(TN{}, jj, K3{}, W0{});
    }
    if constexpr (PAIR) {  // the second chunk of the pair out of the same two tiles
      for (int jj = 0; jj < nj2; ++jj) {
        group(TN{}, jj, K0{}, W1{});
        group(TN{}, jj, K1{}, W1{});
        group(TN{}, jj, K2{}, W1{});
        group(TN{}, jj, K3{}, W1{});
      }
    }

    if (++c == n_steps) {
      // ---- epilogue of row tile rt ---------------------------------------------------
      c = 0;
      const int slot_base = rt * TILE_BINS;
      // the centre tap: Re X[k] += (-1)^k w[N/2] x[N/2]; the parity of a register's bin is that of its index
#pragma unroll
      for (int blk = 0; blk < FR / 2; ++blk)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[blk][r] += (r & 1) ? -xmid : xmid;
      if constexpr (SPLIT && !MEL) {
        if (valid) {
          float* __restrict__ op = P.out + (b_lane * P.out_bins) * g.T + t_lane;
          if (P.fmt == NNA_OUT_MAGNITUDE)
            fold_store_tile_split<NNA_OUT_MAGNITUDE>(acc, op, g.T, slot_base, h, P.n_half);
          else if (P.fmt == NNA_OUT_POWER)
            fold_store_tile_split<NNA_OUT_POWER>(acc, op, g.T, slot_base, h, P.n_half);
          else
            fold_store_tile_split<NNA_OUT_LOG>(acc, op, g.T, slot_base, h, P.n_half);
        }
      } else if constexpr (!MEL) {
        if (valid) {
          float* __restrict__ op = P.out + (b_lane * P.out_bins) * g.T + t_lane;
          if (P.fmt == NNA_OUT_MAGNITUDE)
            fold_store_tile<NNA_OUT_MAGNITUDE>(acc, op, g.T, slot_base, h, P.n_half);
          else if (P.fmt == NNA_OUT_POWER)
            fold_store_tile<NNA_OUT_POWER>(acc, op, g.T, slot_base, h, P.n_half);
          else
            fold_store_tile<NNA_OUT_LOG>(acc, op, g.T, slot_base, h, P.n_half);
        }
      } else {
        // the power (or magnitude) of block blk's 32 bins sits in 16 registers that are, as they stand, the B
        // operands of 16 MFMAs against the filterbank slice: lane (h, m) supplies W[mel m][bin of (r, h)]
        // (split form: "block" 0 = the tile's 32 bins, from E + O; block 1 = their partners N/2 - k, from E - O)
        const unsigned char* __restrict__ maskp = P.mel_mask + ((long long)pass * P.n_rt + rt) * 2;
        const float4* __restrict__ wp = P.melw + (((long long)pass * P.n_rt + rt) * 2) * (ST_MEL_BLOCKS * 4 * 64) + lane;
#pragma unroll
        for (int blk = 0; blk < 2; ++blk) {
          float pw[16];
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            float re, im;
            if constexpr (SPLIT) {
              re = blk ? acc[0][r] - acc[2][r] : acc[0][r] + acc[2][r];
              im = blk ? acc[1][r] - acc[3][r] : acc[1][r] + acc[3][r];
            } else {
              re = acc[blk][r];
              im = acc[blk + 2][r];
            }
            const float v = re * re + im * im;
            pw[r] = P.fmt == 1 ? __builtin_amdgcn_sqrtf(v) : v;
          }
          if constexpr (SPLIT) {
            // the spectrogram the filterbank sees, where the caller wants it too (first pass only: it sweeps every tile then)
            if (P.pout && pass == 0 && valid) {
              float* __restrict__ sp = P.pout + (b_lane * (P.n_half + 1)) * g.T + t_lane;
#pragma unroll
              for (int r = 0; r < 16; ++r) {
                const int k = slot_base + 8 * (r >> 2) + 4 * h + (r & 3);
                sp[(long long)(blk ? P.n_half - k : k) * g.T] = pw[r];
              }
            }
          }
          const unsigned mask = maskp[blk];
#pragma unroll
          for (int mb = 0; mb < ST_MEL_BLOCKS; ++mb) {
            if (mask & (1u << mb)) {
#pragma unroll
              for (int v = 0; v < 4; ++v) {
                const float4 w = wp[((blk * ST_MEL_BLOCKS + mb) * 4 + v) * 64];
                macc[mb] = __builtin_amdgcn_mfma_f32_32x32x2f32(w.x, pw[4 * v + 0], macc[mb], 0, 0, 0);
                macc[mb] = __builtin_amdgcn_mfma_f32_32x32x2f32(w.y, pw[4 * v + 1], macc[mb], 0, 0, 0);
                macc[mb] = __builtin_amdgcn_mfma_f32_32x32x2f32(w.z, pw[4 * v + 2], macc[mb], 0, 0, 0);
                macc[mb] = __builtin_amdgcn_mfma_f32_32x32x2f32(w.w, pw[4 * v + 3], macc[mb], 0, 0, 0);
              }
            }
          }
        }
      }
#pragma unroll
      for (int rb = 0; rb < NACC; ++rb)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[rb][r] = 0.f;
      ++rt;
    }
    __syncthreads();
  }

  // Drain: the last tile requests and the last RING bank requests are never consumed; their registers
  // stay reserved until the data has landed.
  if constexpr (PAIR)
    wait_vm<0>(R, r33);
  else
    wait_vm<0>(R);
#pragma unroll
  for (int s = 0; s < RING; ++s) {
    if constexpr (FR == 4)
      wait_vm<0>(bq[s][0], bq[s][1], bq[s][2], bq[s][3]);
    else
      wait_vm<0>(bq[s][0], bq[s][1]);
  }

  if constexpr (MEL) {
    float pq = 0.f;  // power (or magnitude) of bin N/4 of this lane's frame, where a filter of the pass weighs it
    if constexpr (SPLIT) {
      const bool spec = P.pout && pass == 0;
      if (P.mel_nyq_any || spec) {  // (uniform over the workgroup)
        __syncthreads();            // every wave is done with the tiles: LDS is free
        float* fl = &lds[0][0][0];
        const float v = extra_bin_power(P, ft, fl);
        __syncthreads();
        if (tid < P.tile_frames) fl[tid] = P.fmt == 1 ? __builtin_amdgcn_sqrtf(v) : v;
        __syncthreads();
        pq = fl[fi_lane];
        if (spec && valid && h == 0) P.pout[(b_lane * (P.n_half + 1) + P.n_half / 2) * g.T + t_lane] = pq;
      }
    }
    float* __restrict__ op = P.out + (b_lane * P.n_mels) * g.T + t_lane;
#pragma unroll
    for (int mb = 0; mb < ST_MEL_BLOCKS; ++mb) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int mel = pass * (32 * ST_MEL_BLOCKS) + mb * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
        if (valid && mel < P.n_mels) {
          float v = macc[mb][r];
          if (SPLIT && P.mel_nyq_any) v += P.mel_wnyq[mel] * pq;
          op[(long long)mel * g.T] = v;
        }
      }
    }
  }
}

hipError_t launch_stft_fold(const StftParams& p, int mode, hipStream_t stream) {
  clear_stale_error();
  if (p.nj < 2 || p.tile_frames < 1 || p.tile_frames > ST_FRAMES || !p.bankf) return hipErrorInvalidValue;
  if (p.pair && (!p.split || p.nj != 2 || p.n_chunks % 2)) return hipErrorInvalidValue;
  if (mode == ST_MODE_MEL) {
    const long long blocks = p.n_ft * p.n_pass;
    if (blocks <= 0 || blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    if (p.split) {
      if (p.n_half % 2 || (p.mel_nyq_any && (!p.wn || !p.mel_wnyq)) || (p.pout && !p.wn)) return hipErrorInvalidValue;
      if (p.pair)
        hipLaunchKernelGGL((stft_fold_kernel<ST_MODE_MEL, ST_RING_FOLD_MELSPLIT, true, true>), dim3((unsigned)blocks), dim3(256), 0, stream, p);
      else
        hipLaunchKernelGGL((stft_fold_kernel<ST_MODE_MEL, ST_RING_FOLD_MELSPLIT, true>), dim3((unsigned)blocks), dim3(256), 0, stream, p);
    } else {
      hipLaunchKernelGGL((stft_fold_kernel<ST_MODE_MEL, ST_RING_FOLD_MEL>), dim3((unsigned)blocks), dim3(256), 0, stream, p);
    }
  } else if (mode == ST_MODE_STFT) {
    if (!p.wn || p.main_blocks <= 0) return hipErrorInvalidValue;
    const long long blocks = p.main_blocks + p.n_ft;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    if (p.split) {
      if (p.n_half % 2) return hipErrorInvalidValue;
      if (p.pair)
        hipLaunchKernelGGL((stft_fold_kernel<ST_MODE_STFT, ST_RING_FOLD_SPLIT, true, true>), dim3((unsigned)blocks), dim3(256), 0, stream, p);
      else
        hipLaunchKernelGGL((stft_fold_kernel<ST_MODE_STFT, ST_RING_FOLD_SPLIT, true>), dim3((unsigned)blocks), dim3(256), 0, stream, p);
    } else {
      hipLaunchKernelGGL((stft_fold_kernel<ST_MODE_STFT, ST_RING_FOLD_STFT>), dim3((unsigned)blocks), dim3(256), 0, stream, p);
    }
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace nna
