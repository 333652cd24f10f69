// Kernel banks: built on the host in double precision, rounded to float32 and laid out in the order the GPU
// kernels stream them -- the DFT bank of eq. (DFT2) (direct, folded and float16 forms) and its re-spaced
// variant of eq. (DFT3), the Mel filterbank (Sec. III-B), the spectral kernels of eq. (CQT1992), the
// time-domain constant-Q kernels of eqs. (Q), (N_k), (CQT), and the decimation filter of "Downsampling".
#include "nna_host.h"

namespace nna {
namespace host {

double window_value(int win, long long n, long long N) {
  const double a = 2.0 * kPi * (double)n / (double)N;  // periodic forms: the argument runs over n / N
  switch (win) {
    case NNA_WIN_RECT: return 1.0;
    case NNA_WIN_HAMMING: return 0.54 - 0.46 * std::cos(a);
    case NNA_WIN_BLACKMAN: return 0.42 - 0.5 * std::cos(a) + 0.08 * std::cos(2.0 * a);
    default: return 0.5 - 0.5 * std::cos(a);  // Hann
  }
}

// ---- STFT bank ----------------------------------------------------------------------
double stft_packed_value(const DftTable& t, int n_half, int pr, int k) {
  if (k >= t.N) return 0.0;
  const int slot = pr >> 1, part = pr & 1;
  if (slot >= n_half) return 0.0;
  if (slot == 0) return part == 0 ? t.re(0, k) : t.re(n_half, k);
  return part == 0 ? t.re(slot, k) : t.im(slot, k);
}

// eq. (DFT3) with the window folded in, for a real normalised frequency sigma
double scaled_value(const nna_plan* p, int pr, int k) {
  if (k >= p->K) return 0.0;
  const int slot = pr >> 1, part = pr & 1;
  if (slot >= p->n_half) return 0.0;
  // reduce sigma*k modulo N before the multiplication by 2 pi / N: the product is exact in double
  const double turns = std::fmod(p->sigma[slot] * (double)k, (double)p->K) / (double)p->K;
  const double w = window_value(p->window, k, p->K);
  return part == 0 ? w * std::cos(2.0 * kPi * turns) : -w * std::sin(2.0 * kPi * turns);
}

void build_stft_bank(nna_plan* p) {
  const int N = p->K;
  p->n_half = p->freq_scale ? p->freq_bins : N / 2;
  p->n_rt = (2 * p->n_half + ST_ROWS - 1) / ST_ROWS;  // plain DFT: packed rows = 2 * n_half = N
  const int J = (p->hop > 0 && N % p->hop == 0) ? N / p->hop : 0;
  p->sliding = J >= 1 && J <= 32 && p->hop % ST_KC == 0;
  if (p->sliding) {
    p->nj = J;
    p->n_chunks = p->hop / ST_KC;
  } else {
    p->nj = 1;
    p->n_chunks = (N + ST_KC - 1) / ST_KC;
  }
  const long long G = (long long)p->n_chunks * p->nj * ST_NKG;  // fragment groups per row tile
  p->bank_groups = G * p->n_rt;
  p->bank_floats = (size_t)(p->bank_groups + ST_NKG) * ST_RB * 64 * 4;  // + prefetch overrun
  p->h_bank.assign(p->bank_floats, 0.0f);
  DftTable tab(N, p->window);
  for (int rt = 0; rt < p->n_rt; ++rt)
    for (int c = 0; c < p->n_chunks; ++c)
      for (int j = 0; j < p->nj; ++j)
        for (int kg = 0; kg < ST_NKG; ++kg) {
          const long long g = ((long long)c * p->nj + j) * ST_NKG + kg;
          for (int rb = 0; rb < ST_RB; ++rb)
            for (int lane = 0; lane < 64; ++lane) {
              const int h = lane >> 5, r = lane & 31;
              const int pr = rt * ST_ROWS + rb * 32 + r;
              float* dst = &p->h_bank[((((size_t)rt * G + g) * ST_RB + rb) * 64 + lane) * 4];
              for (int e = 0; e < 4; ++e)
                dst[e] = (float)(p->freq_scale ? scaled_value(p, pr, stft_tap(p, c, j, kg, h, e))
                                               : stft_packed_value(tab, p->n_half, pr, stft_tap(p, c, j, kg, h, e)));
            }
        }
  const double k_exec = (double)p->n_chunks * p->nj * ST_KC;
  p->exec_flops = 2.0 * k_exec * (double)p->n_rt * ST_ROWS;
  // plain DFT: N non-zero rows (cos 0..N/2, sin 1..N/2-1) x N taps; re-spaced: 2 rows per bin
  p->alg_flops = p->freq_scale ? 2.0 * (double)N * 2.0 * (double)p->n_half : 2.0 * (double)N * (double)N;
}

// The bank of the folded-frame kernel: Re and Im kernels of eq. (DFT2) over the taps n < N/2 only (they
// meet x[n] + x[N-n] and x[n] - x[N-n]).  Row tile = 64 bins as four 32-row blocks (Re 0-31, Re 32-63,
// Im 0-31, Im 32-63); fragment order as in the direct bank with J/2 hop-shifts.
void build_stft_bank_fold(nna_plan* p) {
  const int N = p->K, J = p->nj;
  // (last condition: the workgroups that compute bin N/2 keep its weights, (J rounded up to 4) x hop floats,
  // and up to 420 rows of partial sums in the kernel's 19,584 floats of LDS)
  p->fold = !p->freq_scale && p->sliding && p->precision == 0 && J >= 4 && J % 2 == 0 &&
            (long long)((J + 3) / 4 * 4) * (p->hop + 420) <= 4LL * nna::SF_LDS_ROWS * nna::ST_PITCH;
  if (!p->fold) return;
  const int nj2 = J / 2;
  const long long G = (long long)p->n_chunks * nj2 * ST_NKG;
  // Split launches with J = 4 visit the chunks in pairs 0, n-1, 1, n-2, ...: position ci of the bank's stream holds
  // chunk visit(ci)
  const bool will_split = (p->kind == NNA_KIND_MEL && N % 128 == 0 && p->hop % 2 == 0) ||
                          (p->kind == NNA_KIND_STFT && N % 256 == 0 && p->hop % 2 == 0);
  p->fold_pair = will_split && nj2 == 2 && p->n_chunks % 2 == 0;
  const bool pair = p->fold_pair;
  const int n_ch = p->n_chunks;
  auto visit = [pair, n_ch](int ci) { return !pair ? ci : (ci & 1) ? n_ch - 1 - ci / 2 : ci / 2; };
  if (p->kind == NNA_KIND_MEL && N % 128 == 0 && p->hop % 2 == 0) {
    // The Mel launch split by tap parity (see nna_kernels_fold.hip) replaces the plain folded one: row tiles of 32 bins
    // below N/4, two fragments per group (Re, Im kernels of the tile's bins).
    p->fold_split = true;
    p->n_rt_split = N / 128;
    p->bankf_floats = (size_t)(G * p->n_rt_split + ST_NKG) * 2 * 64 * 4;
    p->h_bankf.assign(p->bankf_floats, 0.0f);
    DftTable tab(N, p->window);
    for (int rt = 0; rt < p->n_rt_split; ++rt)
      for (int ci = 0; ci < p->n_chunks; ++ci)
        for (int j = 0; j < nj2; ++j)
          for (int kg = 0; kg < ST_NKG; ++kg) {
            const int c = visit(ci);
            const long long g = ((long long)ci * nj2 + j) * ST_NKG + kg;
            for (int rb = 0; rb < 2; ++rb)
              for (int lane = 0; lane < 64; ++lane) {
                const int h = lane >> 5, bin = rt * 32 + (lane & 31);
                float* dst = &p->h_bankf[((((size_t)rt * G + g) * 2 + rb) * 64 + lane) * 4];
                for (int e = 0; e < 4; ++e) {
                  const int n = stft_tap(p, c, j, kg, h, e);  // < N/2
                  dst[e] = (float)(rb == 0 ? tab.re(bin, n) : tab.im(bin, n));
                }
              }
          }
    const size_t tbl = (size_t)(J + 3) / 4 * 4 * p->hop;
    p->h_wq.assign(2 * tbl, 0.0f);
    for (int n = 0; n < N; ++n) {
      const double w = tab.w[n];
      p->h_wq[n] = (float)((n & 1) ? 0.0 : (n & 2) ? -w : w);
      p->h_wq[tbl + n] = (float)((n & 1) ? ((n & 2) ? w : -w) : 0.0);
    }
    p->h_wn.assign(4, 0.0f);  // (unused by a split launch)
    p->wmid = (float)tab.w[N / 2];
    return;
  }
  p->bankf_floats = (size_t)(G * p->n_rt + ST_NKG) * ST_RB * 64 * 4;
  p->h_bankf.assign(p->bankf_floats, 0.0f);
  DftTable tab(N, p->window);
  for (int rt = 0; rt < p->n_rt; ++rt)
    for (int ci = 0; ci < p->n_chunks; ++ci)
      for (int j = 0; j < nj2; ++j)
        for (int kg = 0; kg < ST_NKG; ++kg) {
          const int c = visit(ci);
          const long long g = ((long long)ci * nj2 + j) * ST_NKG + kg;
          for (int rb = 0; rb < ST_RB; ++rb)
            for (int lane = 0; lane < 64; ++lane) {
              const int h = lane >> 5, bin = rt * (ST_ROWS / 2) + (rb & 1) * 32 + (lane & 31);
              float* dst = &p->h_bankf[((((size_t)rt * G + g) * ST_RB + rb) * 64 + lane) * 4];
              if (bin >= p->n_half) continue;
              for (int e = 0; e < 4; ++e) {
                const int n = stft_tap(p, c, j, kg, h, e);  // < N/2
                dst[e] = (float)(rb < 2 ? tab.re(bin, n) : tab.im(bin, n));
              }
            }
        }
  // bin N/2: (-1)^n w[n], padded with zeros to a whole number of four-segment groups
  p->h_wn.assign((size_t)(J + 3) / 4 * 4 * p->hop, 0.0f);
  for (int n = 0; n < N; ++n) p->h_wn[n] = (float)((n & 1) ? -tab.w[n] : tab.w[n]);
  p->wmid = (float)tab.w[N / 2];
  // per frame: N/2 folded taps x all rows of the row tiles, and the N multiply-adds of bin N/2
  p->exec_flops_fold = 2.0 * ((double)p->n_chunks * nj2 * ST_KC) * (double)p->n_rt * ST_ROWS + 2.0 * N;
  // One more halving for the plain STFT (see nna_kernels_fold.hip): row tiles of the bins below N/4 only -- N/4 must be
  // a whole number of 64-bin row tiles -- and taps whose parity is that of their position in a fragment (even hop).
  p->fold_split = p->kind == NNA_KIND_STFT && N % 256 == 0 && p->hop % 2 == 0;
  if (p->fold_split) {
    p->n_rt_split = p->n_rt / 2;
    // bin N/4: cos(pi n / 2) = 1, 0, -1, 0, ...; -sin(pi n / 2) = 0, -1, 0, 1, ...
    const size_t tbl = (size_t)(J + 3) / 4 * 4 * p->hop;
    p->h_wq.assign(2 * tbl, 0.0f);
    for (int n = 0; n < N; ++n) {
      const double w = tab.w[n];
      p->h_wq[n] = (float)((n & 1) ? 0.0 : (n & 2) ? -w : w);
      p->h_wq[tbl + n] = (float)((n & 1) ? ((n & 2) ? w : -w) : 0.0);
    }
    p->exec_flops_split = 2.0 * ((double)p->n_chunks * nj2 * ST_KC) * (double)(p->n_rt / 2) * ST_ROWS + 4.0 * N;
  }
}

// float16 copy of the STFT bank for the half-precision kernel: same packed rows, cut into row
// tiles of H_ROWS; each (row tile, chunk, hop-shift) tile of H_ROWS x H_KC halves is contiguous,
// in the order the kernel walks them.  Needs the sliding layout.
bool build_stft_bank_f16(nna_plan* p) {
  using nna::H_KC;
  using nna::H_ROWS;
  const int N = p->K;
  const int J = (p->hop > 0 && N % p->hop == 0) ? N / p->hop : 0;
  if (!(J >= 1 && J <= 32 && p->hop % H_KC == 0)) return false;
  const int n_chunks = p->hop / H_KC;
  p->n_rt16 = (2 * p->n_half + H_ROWS - 1) / H_ROWS;
  const size_t tiles = (size_t)p->n_rt16 * n_chunks * J;
  p->bank16_halves = (tiles + 2) * H_ROWS * H_KC;  // + the two tiles the kernel requests past the end
  p->h_bank16.assign(p->bank16_halves, (_Float16)0.0f);
  DftTable tab(N, p->window);
  for (int rt = 0; rt < p->n_rt16; ++rt)
    for (int c = 0; c < n_chunks; ++c)
      for (int j = 0; j < J; ++j) {
        _Float16* tile = &p->h_bank16[(((size_t)rt * n_chunks + c) * J + j) * H_ROWS * H_KC];
        for (int r = 0; r < H_ROWS; ++r)
          for (int e = 0; e < H_KC; ++e) {
            const int pr = rt * H_ROWS + r, tap = j * p->hop + c * H_KC + e;
            const double v = p->freq_scale ? scaled_value(p, pr, tap) : stft_packed_value(tab, p->n_half, pr, tap);
            tile[r * H_KC + e] = (_Float16)(float)v;
          }
      }
  if (J == 2 || J == 4 || J == 8) {
    // streaming order: lane (n = lane % 32, h = lane / 32) of fragment i in row half wr holds row
    // wr*128 + i*32 + n of the tile, taps ks*16 + 8h .. + 8 of the chunk
    const size_t ksteps = tiles * 2;
    p->bank16s_halves = (ksteps + 4) * (size_t)H_ROWS * 16;  // + the ring's requests past the end
    p->h_bank16s.assign(p->bank16s_halves, (_Float16)0.0f);
    for (size_t t = 0; t < tiles; ++t) {
      const _Float16* tile = &p->h_bank16[t * H_ROWS * H_KC];
      for (int ks = 0; ks < 2; ++ks)
        for (int wr = 0; wr < 2; ++wr)
          for (int i = 0; i < 4; ++i)
            for (int lane = 0; lane < 64; ++lane) {
              const int n = lane & 31, h = lane >> 5, row = wr * 128 + i * 32 + n;
              _Float16* dst = &p->h_bank16s[((((t * 2 + ks) * 2 + wr) * 4 + i) * 64 + lane) * 8];
              for (int e = 0; e < 8; ++e) dst[e] = tile[row * H_KC + ks * 16 + 8 * h + e];
            }
    }
  }
  return true;
}

// ---- Mel filterbank (Sec. III-B) ------------------------------------------------------
struct MelAxis {
  int scale;
  // Slaney / Auditory-Toolbox constants of eq. (mel-stanley): 200/3 Hz per mel below the
  // 1 kHz break (mel 15), 27 mels per factor 6.4 above
  static constexpr double hz_per_mel = 200.0 / 3.0;
  static constexpr double brk_hz = 1000.0;
  static constexpr double brk_mel = 15.0;
  double to_mel(double f) const {
    if (scale == NNA_MEL_HTK) return 2595.0 * std::log10(1.0 + f / 700.0);
    return f < brk_hz ? f / hz_per_mel : brk_mel + std::log(f / brk_hz) * 27.0 / std::log(6.4);
  }
  double to_hz(double m) const {
    if (scale == NNA_MEL_HTK) return 700.0 * (std::pow(10.0, m / 2595.0) - 1.0);
    return m < brk_mel ? m * hz_per_mel : brk_hz * std::exp((m - brk_mel) * std::log(6.4) / 27.0);
  }
};

void build_mel_weights(nna_plan* p, double fmin, double fmax, int scale, int norm_area) {
  const int F = p->n_half + 1, M = p->n_mels;
  MelAxis ax{scale};
  std::vector<double> edge(M + 2);
  const double m0 = ax.to_mel(fmin), m1 = ax.to_mel(fmax);
  for (int i = 0; i < M + 2; ++i) edge[i] = ax.to_hz(m0 + (m1 - m0) * i / (double)(M + 1));
  edge[0] = fmin;  // end points exactly as given
  edge[M + 1] = fmax;
  p->h_melW.assign((size_t)M * F, 0.0f);
  for (int m = 0; m < M; ++m) {
    const double lo = edge[m], mid = edge[m + 1], hi = edge[m + 2];
    const double scale_m = norm_area ? 2.0 / (hi - lo) : 1.0;
    for (int j = 0; j < F; ++j) {
      const double nu = (double)j * (double)p->sr / (double)p->K;  // eq. (f-k-conversion)
      double v = 0.0;
      if (nu > lo && nu < hi) v = nu <= mid ? (nu - lo) / (mid - lo) : (hi - nu) / (hi - mid);
      p->h_melW[(size_t)m * F + j] = (float)(v * scale_m);
    }
  }
}

MelDeviceLayout layout_mel(nna_plan* p) {
  MelDeviceLayout out;
  const int F = p->n_half + 1, M = p->n_mels;
  const int per_pass = 32 * ST_MEL_BLOCKS;
  p->n_pass = (M + per_pass - 1) / per_pass;
  out.frag.assign((size_t)p->n_pass * p->n_rt * ST_RB * ST_MEL_BLOCKS * 2 * 64 * 4, 0.0f);
  out.mask.assign((size_t)p->n_pass * p->n_rt * ST_RB, 0);
  out.wnyq.assign(M, 0.0f);
  out.pass_rt.assign((size_t)p->n_pass * 2, 0);
  p->mel_nyq_any = 0;
  for (int m = 0; m < M; ++m) {
    out.wnyq[m] = p->h_melW[(size_t)m * F + p->n_half];
    if (out.wnyq[m] != 0.0f) p->mel_nyq_any = 1;
  }
  double nnz = 0, exec_blocks = 0;
  for (size_t i = 0; i < p->h_melW.size(); ++i) nnz += p->h_melW[i] != 0.0f;
  for (int pass = 0; pass < p->n_pass; ++pass) {
    int rt_lo = p->n_rt, rt_hi = 0;
    bool nyq = false;
    for (int m = pass * per_pass; m < std::min(M, (pass + 1) * per_pass); ++m) {
      for (int j = 0; j < p->n_half; ++j)
        if (p->h_melW[(size_t)m * F + j] != 0.0f) {
          rt_lo = std::min(rt_lo, j / (ST_ROWS / 2));
          rt_hi = std::max(rt_hi, j / (ST_ROWS / 2) + 1);
        }
      nyq = nyq || out.wnyq[m] != 0.0f;
    }
    if (nyq) rt_lo = 0;
    if (rt_hi <= rt_lo) {  // no non-zero weight at all: still visit one tile so the zeros get written
      rt_lo = 0;
      rt_hi = std::max(rt_hi, 1);
    }
    out.pass_rt[2 * pass] = rt_lo;
    out.pass_rt[2 * pass + 1] = rt_hi;
    for (int rt = rt_lo; rt < rt_hi; ++rt)
      for (int rb = 0; rb < ST_RB; ++rb)
        for (int mb = 0; mb < ST_MEL_BLOCKS; ++mb) {
          bool any = false;
          for (int v = 0; v < 2; ++v)
            for (int lane = 0; lane < 64; ++lane) {
              const int h = lane >> 5, mm = lane & 31;
              const int mel = pass * per_pass + mb * 32 + mm;
              for (int e = 0; e < 4; ++e) {
                const int idx8 = v * 4 + e, q = idx8 >> 1, e2 = idx8 & 1;
                const int bin = rt * (ST_ROWS / 2) + rb * 16 + 4 * q + 2 * h + e2;
                float w = 0.0f;
                if (mel < M && bin < p->n_half) w = p->h_melW[(size_t)mel * F + bin];
                out.frag[((((((size_t)pass * p->n_rt + rt) * ST_RB + rb) * ST_MEL_BLOCKS + mb) * 2 + v) * 64 + lane) * 4 + e] = w;
                any = any || w != 0.0f;
              }
            }
          if (any) {
            out.mask[((size_t)pass * p->n_rt + rt) * ST_RB + rb] |= (unsigned char)(1u << mb);
            exec_blocks += 1;
          }
        }
  }
  if (p->fold && p->fold_split) {
    // Split form: row tile rt = bins 32 rt .. 32 rt + 31 (block 0) and their partners N/2 - k (block 1); register r
    // of lane (h, n) holds bin 32 rt + 8 (r/4) + 4 h + r%4 (or its partner).  Bin N/2 is bin 0's partner; bin N/4
    // belongs to no tile and is weighed in by the kernel's own epilogue.
    const int n_rts = p->n_rt_split, Nh = p->n_half;
    out.fragf.assign((size_t)p->n_pass * n_rts * 2 * ST_MEL_BLOCKS * 4 * 64 * 4, 0.0f);
    out.maskf.assign((size_t)p->n_pass * n_rts * 2, 0);
    out.pass_rtf.assign((size_t)p->n_pass * 2, 0);
    out.wq.assign(M, 0.0f);
    p->mel_q_any = 0;
    for (int m = 0; m < M; ++m) {
      out.wq[m] = p->h_melW[(size_t)m * F + Nh / 2];
      if (out.wq[m] != 0.0f) p->mel_q_any = 1;
    }
    double rts = 0;
    for (int pass = 0; pass < p->n_pass; ++pass) {
      int lo = n_rts, hi = 0;
      for (int m = pass * per_pass; m < std::min(M, (pass + 1) * per_pass); ++m)
        for (int j = 0; j <= Nh; ++j)
          if (j != Nh / 2 && p->h_melW[(size_t)m * F + j] != 0.0f) {
            const int t32 = std::min(j, Nh - j) / 32;  // the tile that holds bin j or its partner
            lo = std::min(lo, t32);
            hi = std::max(hi, t32 + 1);
          }
      if (hi <= lo) {  // no weight outside bin N/4: still visit one tile so that the output gets written
        lo = 0;
        hi = 1;
      }
      out.pass_rtf[2 * pass] = lo;
      out.pass_rtf[2 * pass + 1] = hi;
      rts += hi - lo;
      for (int rt = lo; rt < hi; ++rt)
        for (int blk = 0; blk < 2; ++blk)
          for (int mb = 0; mb < ST_MEL_BLOCKS; ++mb) {
            bool any = false;
            for (int v = 0; v < 4; ++v)
              for (int lane = 0; lane < 64; ++lane)
                for (int e = 0; e < 4; ++e) {
                  const int r = 4 * v + e, mel = pass * per_pass + mb * 32 + (lane & 31);
                  const int k = rt * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                  const int bin = blk ? Nh - k : k;
                  const float w = mel < M ? p->h_melW[(size_t)mel * F + bin] : 0.0f;
                  out.fragf[((((((size_t)pass * n_rts + rt) * 2 + blk) * ST_MEL_BLOCKS + mb) * 4 + v) * 64 + lane) * 4 + e] = w;
                  any = any || w != 0.0f;
                }
            if (any) {
              out.maskf[((size_t)pass * n_rts + rt) * 2 + blk] |= (unsigned char)(1u << mb);
              out.exec_blocks_f += 1;
            }
          }
    }
    // per frame: N/2 folded taps x the 64 rows of every tile visited, the filterbank blocks, and bin N/4's two sums
    p->exec_flops_split = 2.0 * ((double)p->n_chunks * (p->nj / 2) * ST_KC) * 64.0 * rts + out.exec_blocks_f * 2.0 * 32 * 32 +
                          (p->mel_q_any ? 4.0 * p->K * p->n_pass : 0.0);
  } else if (p->fold) {
    // folded kernel: register r of lane (h, n) in block blk holds bin 64 rt + 32 blk + 8 (r/4) + 4 h + r%4;
    // as the B operand of MFMA number r it meets, in lane (h, m), the weight of mel m for that bin
    out.fragf.assign((size_t)p->n_pass * p->n_rt * 2 * ST_MEL_BLOCKS * 4 * 64 * 4, 0.0f);
    out.maskf.assign((size_t)p->n_pass * p->n_rt * 2, 0);
    for (int pass = 0; pass < p->n_pass; ++pass)
      for (int rt = out.pass_rt[2 * pass]; rt < out.pass_rt[2 * pass + 1]; ++rt)
        for (int blk = 0; blk < 2; ++blk)
          for (int mb = 0; mb < ST_MEL_BLOCKS; ++mb) {
            bool any = false;
            for (int v = 0; v < 4; ++v)
              for (int lane = 0; lane < 64; ++lane)
                for (int e = 0; e < 4; ++e) {
                  const int r = 4 * v + e, mel = pass * per_pass + mb * 32 + (lane & 31);
                  const int bin = rt * (ST_ROWS / 2) + 32 * blk + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                  const float w = mel < M && bin < p->n_half ? p->h_melW[(size_t)mel * F + bin] : 0.0f;
                  out.fragf[((((((size_t)pass * p->n_rt + rt) * 2 + blk) * ST_MEL_BLOCKS + mb) * 4 + v) * 64 + lane) * 4 + e] = w;
                  any = any || w != 0.0f;
                }
            if (any) {
              out.maskf[((size_t)pass * p->n_rt + rt) * 2 + blk] |= (unsigned char)(1u << mb);
              out.exec_blocks_f += 1;
            }
          }
  }
  // executed flops: every pass sweeps its row tile range with the full DFT contraction
  double dft_exec = 0;
  const double k_exec = (double)p->n_chunks * p->nj * ST_KC;
  for (int pass = 0; pass < p->n_pass; ++pass)
    dft_exec += 2.0 * k_exec * ST_ROWS * (out.pass_rt[2 * pass + 1] - out.pass_rt[2 * pass]);
  p->exec_flops = dft_exec + exec_blocks * 2.0 * 32 * 16;  // 8 MFMA 32x32x2 per block, per frame: 32 mels x 16 slots
  if (p->fold && !p->fold_split) {
    if (p->mel_nyq_any) {
      p->fold = false;  // a filter weighs bin N/2, which the folded contraction does not produce
    } else {
      double rts = 0;
      for (int pass = 0; pass < p->n_pass; ++pass) rts += out.pass_rt[2 * pass + 1] - out.pass_rt[2 * pass];
      p->exec_flops_fold = 2.0 * ((double)p->n_chunks * (p->nj / 2) * ST_KC) * ST_ROWS * rts + out.exec_blocks_f * 2.0 * 32 * 32;
    }
  }
  p->alg_flops = 2.0 * (double)p->K * (double)p->K + 2.0 * nnz;
  return out;
}

// ---- CQT with frequency-domain kernels (Sec. III-C, eq. (CQT1992)) -----------------------
// In-place radix-2 decimation-in-time FFT, forward sign, n a power of two.
void fft_pow2(std::vector<std::complex<double>>& a) {
  const size_t n = a.size();
  for (size_t i = 1, j = 0; i < n; ++i) {
    size_t bit = n >> 1;
    for (; j & bit; bit >>= 1) j ^= bit;
    j ^= bit;
    if (i < j) std::swap(a[i], a[j]);
  }
  std::vector<std::complex<double>> tw(n / 2);
  for (size_t k = 0; k < n / 2; ++k) tw[k] = std::polar(1.0, -2.0 * kPi * (double)k / (double)n);
  for (size_t len = 2; len <= n; len <<= 1) {
    const size_t half = len >> 1, step = n / len;
    for (size_t i = 0; i < n; i += len)
      for (size_t k = 0; k < half; ++k) {
        const std::complex<double> u = a[i + k], v = a[i + k + half] * tw[k * step];
        a[i + k] = u + v;
        a[i + k + half] = u - v;
      }
  }
}

// The spectral kernels and the real matrix the kernel multiplies with.  kappa_q[n] = window(N_q)[n]
// exp(-2 pi i Q n / N_q) / sum(window) is the kernel of eq. (CQT), centred in K taps.  With
// B_q = DFT(conj(kappa_q)) (a positive-frequency signal, so B_q lives in bins 0..K/2) Parseval gives
//   sum_n x[n] kappa_q[n] = (1/K) sum_k X[k] conj(B_q[k]),
// and eq. (CQT1992) keeps k = 0..K/2.  Y[q, k] = conj(B_q[k]).  In real arithmetic, per bin k:
//   Re X_cq += (Xr Yr - Xi Yi)/K,   Im X_cq += (Xr Yi + Xi Yr)/K.
// Packed STFT rows: 2s = Re X[s], 2s+1 = Im X[s]; slot 0 holds the two purely real bins 0 and K/2.
void build_cqt1992_matrix(nna_plan* p) {
  const int K = p->K, n_half = p->n_half, R = 2 * p->n_bins, C = 2 * n_half;
  p->h_linW.assign((size_t)R * C, 0.0f);
  std::vector<std::complex<double>> a(K);
  const double inv = 1.0 / (double)K;
  for (int q = 0; q < p->n_bins; ++q) {
    std::fill(a.begin(), a.end(), std::complex<double>(0.0, 0.0));
    double wsum = 0;
    for (long long n = 0; n < p->Nk[q]; ++n) wsum += window_value(p->cq_window, n, p->Nk[q]);
    for (long long n = 0; n < p->Nk[q]; ++n) {
      const double w = window_value(p->cq_window, n, p->Nk[q]) / wsum;
      a[p->sk[q] + n] = std::polar(w, 2.0 * kPi * p->Q * (double)n / (double)p->Nk[q]);  // conj(kappa)
    }
    fft_pow2(a);
    float* re_row = &p->h_linW[(size_t)(2 * q) * C];
    float* im_row = &p->h_linW[(size_t)(2 * q + 1) * C];
    for (int s = 0; s <= n_half; ++s) {
      const double yr = a[s].real() * inv, yi = -a[s].imag() * inv;  // Y = conj(B), with the 1/K folded in
      if (s == 0 || s == n_half) {  // purely real STFT bins: packed rows 0 and 1
        re_row[s == 0 ? 0 : 1] = (float)yr;
        im_row[s == 0 ? 0 : 1] = (float)yi;
      } else {
        re_row[2 * s] = (float)yr;
        re_row[2 * s + 1] = (float)(-yi);
        im_row[2 * s] = (float)yi;
        im_row[2 * s + 1] = (float)yr;
      }
    }
  }
}

MelDeviceLayout layout_cqt1992(nna_plan* p) {
  MelDeviceLayout out;
  const int R = 2 * p->n_bins, C = 2 * p->n_half;
  // every pass repeats the whole first stage: six output blocks per pass (fewer registers left for the
  // bank ring) when that saves one, e.g. the 168 rows of 84 bins in one pass instead of two
  p->lin_blocks = (R + 191) / 192 < (R + 127) / 128 ? 6 : 4;
  const int per_pass = 32 * p->lin_blocks;
  p->n_pass = (R + per_pass - 1) / per_pass;
  p->lin_frag_floats = (size_t)p->n_pass * p->n_rt * ST_RB * p->lin_blocks * 4 * 64 * 4;
  out.frag.assign(p->lin_frag_floats, 0.0f);
  out.mask.assign((size_t)p->n_pass * p->n_rt * ST_RB, 0);
  out.wnyq.assign(1, 0.0f);
  out.pass_rt.assign((size_t)p->n_pass * 2, 0);
  p->mel_nyq_any = 0;
  double exec_blocks = 0;
  for (int pass = 0; pass < p->n_pass; ++pass) {
    // the paper applies no threshold to the spectral kernels: every row tile is visited
    out.pass_rt[2 * pass] = 0;
    out.pass_rt[2 * pass + 1] = p->n_rt;
    for (int rt = 0; rt < p->n_rt; ++rt)
      for (int rb = 0; rb < ST_RB; ++rb)
        for (int mb = 0; mb < p->lin_blocks; ++mb) {
          bool any = false;
          for (int v = 0; v < 4; ++v)
            for (int lane = 0; lane < 64; ++lane)
              for (int e = 0; e < 4; ++e) {
                const int row = pass * per_pass + mb * 32 + (lane & 31);
                const int col = rt * ST_ROWS + rb * 32 + 8 * v + 4 * (lane >> 5) + e;
                const float w = row < R && col < C ? p->h_linW[(size_t)row * C + col] : 0.0f;
                out.frag[lin_frag_index(p, pass, rt, rb, mb, v, lane, e)] = w;
                any = any || w != 0.0f;
              }
          if (any) {
            out.mask[((size_t)pass * p->n_rt + rt) * ST_RB + rb] |= (unsigned char)(1u << mb);
            exec_blocks += 1;
          }
        }
  }
  const double k_exec = (double)p->n_chunks * p->nj * ST_KC;
  p->exec_flops = p->n_pass * 2.0 * k_exec * ST_ROWS * p->n_rt + exec_blocks * 2.0 * 32 * 32;
  // the DFT of a frame (K non-zero rows x K taps) + one complex multiply-add per (bin, kept DFT bin)
  p->alg_flops = 2.0 * (double)p->K * (double)p->K + 8.0 * (double)p->n_bins * (double)(p->n_half + 1);
  return out;
}

// ---- CQT bank (Sec. III-C) ------------------------------------------------------------
// Lays out, for the CQT kernel, a bank of p->conv_rows rows x p->K taps whose row r is zero
// outside [row_s[r], row_e[r]); value(row, tap) gives the logical entries.
template <typename ValueFn>
void build_conv_bank(nna_plan* p, ValueFn value) {
  const long long K = p->K;
  p->n_rb = (p->conv_rows + CQ_ROWS - 1) / CQ_ROWS;
  const long long J = (K % p->hop == 0) ? K / p->hop : 0;
  // tap support [s, e) of every row block
  std::vector<long long> s_rb(p->n_rb), e_rb(p->n_rb);
  for (int rb = 0; rb < p->n_rb; ++rb) {
    long long s = K, e = 0;
    for (int r = rb * CQ_ROWS; r < std::min(p->conv_rows, (rb + 1) * CQ_ROWS); ++r) {
      s = std::min(s, p->row_s[r]);
      e = std::max(e, p->row_e[r]);
    }
    s_rb[rb] = s;
    e_rb[rb] = e;
  }
  // Overlapping frames share LDS rows when the hop divides the taps and is a whole number of
  // chunks, and the longest kernel's hop-shifts (+ ring padding) leave room for at least 16
  // frames of a tile that spans two waveforms: 16 + 2 * (shifts - 1) <= CQ_LDS_ROWS_MAX.
  long long span_max = 0;
  for (int rb = 0; rb < p->n_rb; ++rb) span_max = std::max(span_max, e_rb[rb] - s_rb[rb]);
  const long long shifts_max = (ceil_div(span_max, p->hop) + 1 + CQ_PREFETCH - 1) / CQ_PREFETCH * CQ_PREFETCH;
  p->sliding = J >= 1 && p->hop % CQ_KC == 0 && 16 + 2 * (shifts_max - 1) <= CQ_LDS_ROWS_MAX;
  p->tap_stride = p->sliding ? p->hop : 0;
  p->row_step = 1;
  if (!p->sliding && p->hop < CQ_KC && CQ_KC % p->hop == 0 && K % CQ_KC == 0) {
    // A hop that divides the 16-tap chunk (the deep octaves of a downsampling plan): the LDS rows still step
    // by one hop, so tap 16 j + c of the frame in row t is column c of row t + j (16 / hop) -- one tile of 16
    // columns serves every tap, shift j now counting chunks of 16 taps.
    const int step = CQ_KC / p->hop;
    const long long sm = (ceil_div(span_max, CQ_KC) + 1 + CQ_PREFETCH - 1) / CQ_PREFETCH * CQ_PREFETCH;
    if (16 + 2 * (sm - 1) * step <= CQ_LDS_ROWS_MAX) {
      p->sliding = true;
      p->tap_stride = CQ_KC;
      p->row_step = step;
    }
  }
  const long long ts = p->tap_stride, Jts = p->sliding ? K / ts : 0;
  // chunk grid: 16-tap column chunks of the shift stride (shared LDS rows) or of the whole tap range
  const int n_grid = p->sliding ? (int)(ts / CQ_KC) : (int)ceil_div(K, CQ_KC);
  // shifts [jlo, jlo + nj) of row block rb that hold taps in grid chunk c
  auto shifts_of = [&](int rb, int c, int& jlo, int& nj) {
    const long long c0 = (long long)c * CQ_KC;
    if (p->sliding) {
      // taps j*ts + c0 + [0, KC) intersect [s, e)  <=>  j*ts + c0 + KC > s  and  j*ts + c0 < e
      long long lo = floor_div(s_rb[rb] - c0 - CQ_KC, ts) + 1;
      long long hi = ceil_div(e_rb[rb] - c0, ts);
      lo = std::max(lo, 0LL);
      hi = std::min(hi, Jts);
      jlo = (int)lo;
      nj = (int)std::max(0LL, hi - lo);
    } else {
      jlo = 0;
      nj = (c0 + CQ_KC > s_rb[rb] && c0 < e_rb[rb]) ? 1 : 0;
    }
    if (nj == 0) jlo = 0;
  };
  auto ring_pad = [](int nj) { return (nj + CQ_PREFETCH - 1) / CQ_PREFETCH * CQ_PREFETCH; };
  // most fragments any chunk of a row block has
  std::vector<int> rb_nj(p->n_rb, 0);
  for (int rb = 0; rb < p->n_rb; ++rb)
    for (int c = 0; c < n_grid; ++c) {
      int jlo, nj;
      shifts_of(rb, c, jlo, nj);
      rb_nj[rb] = std::max(rb_nj[rb], ring_pad(nj));
    }
  // Work items: the long kernels get a workgroup per row block; short ones are grouped (they
  // share the first block's LDS tiles) until a chunk holds about 48 fragments.
  p->h_items.clear();
  for (int rb = 0; rb < p->n_rb;) {
    nna::CqtItem item{};
    item.rb_first = rb;
    int sum = 0;
    do {
      sum += rb_nj[rb];
      ++item.n_rb;
      ++rb;
    } while (rb < p->n_rb && item.n_rb < CQ_ITEM_RB && sum < 48);
    p->h_items.push_back(item);
  }
  // per item: the chunks that hold taps, and for each the fragments of every row block
  std::vector<std::vector<nna::CqtChunk>> item_chunks(p->h_items.size());
  long long exec_groups = 0;
  long long frag = 0;
  p->max_jspan = 1;
  p->n_chunks = 1;
  for (size_t it = 0; it < p->h_items.size(); ++it) {
    nna::CqtItem& item = p->h_items[it];
    item.frag0 = frag;
    item.jspan = 1;
    for (int c = 0; c < n_grid; ++c) {
      // the chunk is listed if any row block of the item has taps in it; its LDS rows start at the
      // smallest hop-shift any of them needs
      int jl[CQ_ITEM_RB] = {0, 0, 0, 0}, nn[CQ_ITEM_RB] = {0, 0, 0, 0};
      int jmin = INT_MAX;
      for (int r = 0; r < item.n_rb; ++r) {
        shifts_of(item.rb_first + r, c, jl[r], nn[r]);
        if (nn[r] > 0) jmin = std::min(jmin, jl[r]);
      }
      if (jmin == INT_MAX) continue;
      nna::CqtChunk ck{};
      ck.c0 = c * CQ_KC;
      ck.jlo = jmin;
      for (int r = 0; r < CQ_ITEM_RB; ++r) {
        const int nj = nn[r];
        ck.joff[r] = nj > 0 ? jl[r] - jmin : 0;
        // whole rings of CQ_PREFETCH fragments (zero fragments pad); the item's first row block always
        // has one ring, because its first two groups carry the tile staging
        const int padded = r == 0 ? std::max(ring_pad(nj), CQ_PREFETCH) : ring_pad(nj);
        ck.nj[r] = padded | (nj << 16);
        item.jspan = std::max(item.jspan, ck.joff[r] + padded);
        frag += padded;
        // the kernel runs MFMAs for the real fragments only, and for those two groups
        exec_groups += r == 0 ? std::max(nj, 2) : nj;
      }
      item_chunks[it].push_back(ck);
    }
    item.n_chunks = (int)item_chunks[it].size();
    p->n_chunks = std::max(p->n_chunks, item.n_chunks);  // stride of the chunk table
    p->max_jspan = std::max(p->max_jspan, item.jspan);
  }
  p->h_chunks.assign(p->h_items.size() * (size_t)p->n_chunks, nna::CqtChunk{});
  for (size_t it = 0; it < p->h_items.size(); ++it)
    for (size_t c = 0; c < item_chunks[it].size(); ++c) {
      p->h_chunks[it * p->n_chunks + c] = item_chunks[it][c];
    }
  p->bank_groups = frag;
  p->bank_floats = (size_t)(frag + CQ_PREFETCH) * 64 * 4;
  p->h_bank.assign(p->bank_floats, 0.0f);
  for_each_cqt_fragment(p, [&](long long f, int rb, int j, int c0, bool real) {
    if (!real) return;
    for (int lane = 0; lane < 64; ++lane) {
      const int q = lane >> 4, r = lane & 15;
      const int row = rb * CQ_ROWS + r;
      const long long tap0 = (long long)j * p->tap_stride + c0 + 4 * q;
      float* dst = &p->h_bank[((size_t)f * 64 + lane) * 4];
      for (int e = 0; e < 4; ++e) dst[e] = row < p->conv_rows && tap0 + e < K ? (float)value(row, tap0 + e) : 0.0f;
    }
  });
  p->exec_flops = 2.0 * (double)exec_groups * CQ_KC * CQ_ROWS;
}

void build_cqt_bank(nna_plan* p) {
  p->conv_rows = 2 * p->n_bins;
  p->row_s.resize(p->conv_rows);
  p->row_e.resize(p->conv_rows);
  double sumN = 0;
  for (int k = 0; k < p->n_bins; ++k) {
    p->row_s[2 * k] = p->row_s[2 * k + 1] = p->sk[k];
    p->row_e[2 * k] = p->row_e[2 * k + 1] = p->sk[k] + p->Nk[k];
    sumN += (double)p->Nk[k];
  }
  CqtKernelGen gen(p);
  build_conv_bank(p, [&](int row, long long tap) { return gen.value(row, tap); });
  p->alg_flops = 4.0 * sumN;
}

// ---- CQT bank folded about the kernels' centres (nna_kernels_cqf.hip) --------------------------
// Kernel k of eq. (CQT) is window(N_k)[n] exp(-2 pi i Q n / N_k): a symmetric window times a phase that is linear
// in n, so about its centre n = N_k / 2 the kernel is exp(-i pi Q) times a sequence g with g[-m] = conj(g[m]).
// Centred in K taps (K even), kernels of even length have that centre on tap K/2, kernels of odd length half a
// tap before it.  With the frame folded about the same point, e[m] = x[K/2 + m] + x[K/2 - p - m] and
// o[m] = x[K/2 + m] - x[K/2 - p - m] (p = 0 / 1 for even / odd lengths),
//     C_k = exp(-i pi Q) ( sum_m e[m] Re g_k[m]  +  i sum_m o[m] Im g_k[m] ),
// half the multiply-adds.  Rows that share an MFMA share its frame operand, so a 16-row block holds the
// cosine kernels Re g (or the sine kernels Im g) of 16 bins of one parity; the bins of each parity are taken in
// order of length, 16 at a time.  The symmetry is checked on the values themselves: a window that does not
// vanish at n = 0 (its partner n = N_k lies outside the kernel) leaves the plan on the direct bank.
void build_cqt_bank_fold(nna_plan* p) {
  p->cq_fold = false;
  const long long K = p->K, hop = p->hop;
  if (!p->sliding || p->tap_stride != p->hop || p->row_step != 1) return;
  if (K % (2 * hop) != 0 || K / hop < 8 || hop / CQ_KC > CQF_TABLE_CAP) return;
  const long long c = K / 2;
  const double rc = std::cos(kPi * std::fmod(p->Q, 2.0)), rs = std::sin(kPi * std::fmod(p->Q, 2.0));
  CqtKernelGen gen(p);
  // g_k[m] = exp(+i pi Q) h_k[c + m]; its mirrored partner exp(+i pi Q) h_k[c - par - m] must be its conjugate
  auto g_at = [&](int k, long long tap, double& re, double& im) {
    const double hr = tap >= 0 && tap < K ? gen.value(2 * k, tap) : 0.0, hi = tap >= 0 && tap < K ? gen.value(2 * k + 1, tap) : 0.0;
    re = rc * hr - rs * hi;
    im = rs * hr + rc * hi;
  };
  std::vector<int> par(p->n_bins);
  std::vector<long long> M(p->n_bins);  // folded taps of bin k: m in [0, M[k])
  for (int k = 0; k < p->n_bins; ++k) {
    par[k] = (int)(p->Nk[k] & 1);
    const long long reach = p->Nk[k] / 2 + 2;  // no tap of the kernel lies further from the centre
    double peak = 0;
    for (long long m = 0; m < reach; ++m) {
      double a, b;
      g_at(k, c + m, a, b);
      peak = std::max(peak, std::max(std::fabs(a), std::fabs(b)));
    }
    long long last = -1;
    for (long long m = 0; m < reach; ++m) {
      double a, b, ma, mb;
      g_at(k, c + m, a, b);
      g_at(k, c - par[k] - m, ma, mb);
      if (std::fabs(a - ma) > 1e-9 * peak || std::fabs(b + mb) > 1e-9 * peak) return;  // not symmetric: stay direct
      if (a != 0.0 || b != 0.0) last = m;
    }
    M[k] = std::max(1LL, last + 1);
  }
  // groups: the bins of each parity in order of decreasing length, 16 at a time; groups ordered by their longest kernel
  struct Group { int parity; std::vector<int> bins; long long Mmax; };
  std::vector<Group> groups;
  for (int parity = 0; parity < 2; ++parity) {
    std::vector<int> ks;
    for (int k = 0; k < p->n_bins; ++k)
      if (par[k] == parity) ks.push_back(k);
    std::stable_sort(ks.begin(), ks.end(), [&](int a, int b) { return M[a] > M[b]; });
    for (size_t i = 0; i < ks.size(); i += CQ_ROWS) {
      Group gp{parity, {}, 0};
      for (size_t u = i; u < std::min(ks.size(), i + CQ_ROWS); ++u) {
        gp.bins.push_back(ks[u]);
        gp.Mmax = std::max(gp.Mmax, M[ks[u]]);
      }
      groups.push_back(gp);
    }
  }
  // items: groups of one parity, consecutive in that parity's order; a short group takes the next one along
  std::vector<std::vector<int>> items;  // indices into groups
  for (int parity = 0; parity < 2; ++parity) {
    std::vector<int> gs;
    for (size_t gi = 0; gi < groups.size(); ++gi)
      if (groups[gi].parity == parity) gs.push_back((int)gi);
    for (size_t i = 0; i < gs.size();) {
      const long long shifts = ceil_div(groups[gs[i]].Mmax, hop);
      if (i + 1 < gs.size() && shifts < 24) {
        items.push_back({gs[i], gs[i + 1]});
        i += 2;
      } else {
        items.push_back({gs[i]});
        i += 1;
      }
    }
  }
  std::stable_sort(items.begin(), items.end(), [&](const std::vector<int>& a, const std::vector<int>& b) {
    return groups[a[0]].Mmax > groups[b[0]].Mmax;
  });
  // device order of the groups = order of appearance in the items
  p->h_qbins.clear();
  p->h_qitems.clear();
  std::vector<std::vector<nna::CqfChunk>> item_chunks(items.size());
  const int n_grid = (int)(hop / CQ_KC);
  long long frag = 0, exec_pair_groups = 0;
  p->q_n_chunks = 1;
  p->q_max_jspan = 1;
  auto ring_pad = [](long long n) { return (n + 1) / 2 * 2; };  // a ring of CQ_PREFETCH = 4 fragments is two pair groups
  static_assert(CQ_PREFETCH == 4, "two pair groups per ring");
  for (size_t it = 0; it < items.size(); ++it) {
    nna::CqfItem item{};
    item.frag0 = frag;
    item.grp_first = (int)(p->h_qbins.size() / CQ_ROWS);
    item.n_pair = (int)items[it].size();
    item.parity = groups[items[it][0]].parity;
    item.jspan = 1;
    for (int gi : items[it]) {
      const Group& gp = groups[gi];
      for (int r = 0; r < CQ_ROWS; ++r) p->h_qbins.push_back(r < (int)gp.bins.size() ? gp.bins[r] : -1);
    }
    for (int cidx = 0; cidx < n_grid; ++cidx) {
      const long long c0 = (long long)cidx * CQ_KC;
      nna::CqfChunk ck{};
      ck.c0 = (int)c0;
      bool any = false;
      for (int u = 0; u < item.n_pair; ++u) {
        const long long Mm = groups[items[it][u]].Mmax;
        // shifts j with j hop + c0 < Mm
        const long long nj = Mm > c0 ? ceil_div(Mm - c0, hop) : 0;
        // the first pair always runs one ring: its waits are the ones that let the tile requests pass
        const long long padded = u == 0 ? std::max(ring_pad(nj), 2LL) : ring_pad(nj);
        ck.nj[u] = (int)(padded | (nj << 16));
        item.jspan = std::max(item.jspan, (int)std::max(nj, 1LL));
        any = any || nj > 0;
      }
      if (!any) continue;
      for (int u = 0; u < item.n_pair; ++u) {
        frag += 2 * (ck.nj[u] & 0xffff);
        exec_pair_groups += ck.nj[u] >> 16;
      }
      item_chunks[it].push_back(ck);
    }
    item.n_chunks = (int)item_chunks[it].size();
    p->q_n_chunks = std::max(p->q_n_chunks, item.n_chunks);
    p->q_max_jspan = std::max(p->q_max_jspan, item.jspan);
    p->h_qitems.push_back(item);
  }
  if (p->q_max_jspan > K / (2 * hop)) return;  // (cannot happen: the folded taps end before K/2)
  if (16 + 2 * (p->q_max_jspan - 1) > CQF_LDS_ROWS) return;  // no room for a tile that spans two waveforms
  p->h_qchunks.assign(items.size() * (size_t)p->q_n_chunks, nna::CqfChunk{});
  for (size_t it = 0; it < items.size(); ++it)
    for (size_t ci = 0; ci < item_chunks[it].size(); ++ci) p->h_qchunks[it * p->q_n_chunks + ci] = item_chunks[it][ci];
  // fragments in loop order: per chunk, per pair, per shift: cosine rows, then sine rows
  p->h_bankq.assign((size_t)(frag + CQ_PREFETCH) * 64 * 4, 0.0f);
  long long f = 0;
  for (size_t it = 0; it < items.size(); ++it)
    for (const nna::CqfChunk& ck : item_chunks[it])
      for (int u = 0; u < (int)items[it].size(); ++u) {
        const Group& gp = groups[items[it][u]];
        const int padded = ck.nj[u] & 0xffff, real = ck.nj[u] >> 16;
        for (int jj = 0; jj < padded; ++jj, f += 2) {
          if (jj >= real) continue;
          for (int lane = 0; lane < 64; ++lane) {
            const int q = lane >> 4, r = lane & 15;
            if (r >= (int)gp.bins.size()) continue;
            const int k = gp.bins[r];
            float* dc = &p->h_bankq[((size_t)f * 64 + lane) * 4];
            float* ds = &p->h_bankq[((size_t)(f + 1) * 64 + lane) * 4];
            for (int e = 0; e < 4; ++e) {
              const long long m = (long long)jj * hop + ck.c0 + 4 * q + e;
              if (m >= M[k]) continue;
              double a, b;
              g_at(k, c + m, a, b);
              if (m == 0 && gp.parity == 0) a *= 0.5;  // the centre tap meets itself in the fold
              dc[e] = (float)a;
              ds[e] = (float)b;
            }
          }
        }
      }
  p->exec_flops_cqf = 2.0 * (double)exec_pair_groups * 2.0 * CQ_KC * CQ_ROWS;
  // Blocks of one parity span twice as many adjacent bins as the direct bank's (16 bins of a parity against 8 of
  // either), so with few bins per octave the longest kernel of a block dwarfs the others and the fold's half is
  // eaten up; the folded kernel also keeps the matrix pipe less busy (it forms the folds on the vector ALUs: 0.77
  // against 0.86 measured).  Timed on 1,770 waveforms it breaks even where it multiplies 0.86 of what the direct
  // kernel does (12 bins per octave, 0.84-0.85: 1-5 % faster); beyond that the direct kernel runs.
  p->cq_fold = p->exec_flops_cqf <= 0.86 * p->exec_flops;
}

// Window-method low-pass at half the Nyquist frequency (Sec. III-C, "Downsampling"): the ideal
// response's samples under a Hamming window, scaled to unit gain at 0 Hz.
std::vector<double> half_band_taps(int n) {
  std::vector<double> h(n);
  double sum = 0;
  for (int i = 0; i < n; ++i) {
    const double u = i - 0.5 * (n - 1);
    const double ideal = u == 0.0 ? 0.5 : std::sin(0.5 * kPi * u) / (kPi * u);  // 0.5 sinc(u / 2)
    h[i] = ideal * (0.54 - 0.46 * std::cos(2.0 * kPi * i / (n - 1)));
    sum += h[i];
  }
  for (double& v : h) v /= sum;
  return h;
}

// The decimation filter: the taps, then (for inspection) the filter + keep-every-second-sample step as a bank
// in the CQT kernel's layout -- a "frame" is FIR_ROWS consecutive output samples y[FIR_ROWS t + r], it reads input
// samples 2 FIR_ROWS t - half + [0, K), and row r holds the filter shifted by 2 r taps (y[m] is centred on
// x[2 m]) -- and the taps split by parity as the decimation kernel applies them.
void build_fir_bank(nna_plan* p, int fir_taps) {
  p->h_fir = half_band_taps(fir_taps);
  p->conv_rows = FIR_ROWS;
  p->row_s.resize(FIR_ROWS);
  p->row_e.resize(FIR_ROWS);
  for (int r = 0; r < FIR_ROWS; ++r) {
    p->row_s[r] = 2 * r;
    p->row_e[r] = 2 * r + fir_taps;
  }
  build_conv_bank(p, [&](int row, long long tap) {
    const long long i = tap - 2 * row;
    return i >= 0 && i < fir_taps ? p->h_fir[i] : 0.0;
  });
  p->alg_flops = 2.0 * fir_taps * FIR_ROWS;  // per frame of FIR_ROWS output samples
  // The decimation itself runs on the vector ALUs from the taps split by the parity of their offset u = i - half
  // from the centre: y[m] = sum_v h[half + 2v] x~[2 (m + v)] + sum_v h[half + 2v + 1] x~[2 (m + v) + 1].  A half-band
  // design is zero on every even offset but 0 (sin(pi u / 2) = 0; in double the taps come out as ~1e-17):
  // those taps are dropped, which leaves the centre tap on the even samples.
  const int half = (fir_taps - 1) / 2;
  double hmax = 0, zmax = 0;
  for (int i = 0; i < fir_taps; ++i) {
    hmax = std::max(hmax, std::fabs(p->h_fir[i]));
    if (i != half && ((i - half) & 1) == 0) zmax = std::max(zmax, std::fabs(p->h_fir[i]));
  }
  const bool half_band = zmax <= 1e-12 * hmax;
  const int ve_lo = half_band ? 0 : -(half / 2), ve_hi = half_band ? 0 : half / 2;
  const int vo_lo = -((half + 1) / 2), vo_hi = (half - 1) / 2;
  auto pad4 = [](int n) { return (n + 7) / 8 * 8; };  // the kernel takes eight taps per step
  p->fir_ve0 = ve_lo;
  p->fir_vo0 = vo_lo;
  p->h_fir_he.assign(pad4(ve_hi - ve_lo + 1), 0.0f);
  p->h_fir_ho.assign(pad4(std::max(vo_hi - vo_lo + 1, 1)), 0.0f);
  for (int v = ve_lo; v <= ve_hi; ++v) p->h_fir_he[v - ve_lo] = (float)p->h_fir[half + 2 * v];
  for (int v = vo_lo; v <= vo_hi; ++v) p->h_fir_ho[v - vo_lo] = (float)p->h_fir[half + 2 * v + 1];
  p->fir_mode = half_band ? 1 : 0;
  // flops per frame of FIR_ROWS output samples: the taps kept
  p->alg_flops = 2.0 * ((ve_hi - ve_lo + 1) + (vo_hi - vo_lo + 1)) * FIR_ROWS;
  p->exec_flops = 2.0 * (double)(p->h_fir_he.size() + p->h_fir_ho.size()) * FIR_ROWS;
}

}  // namespace host
}  // namespace nna
