/*
 * nna_oracle.c -- float64 CPU oracle for the waveform -> spectrogram transforms
 * of arXiv 1912.12055 (STFT, Mel spectrogram, constant-Q transform by strided
 * convolution with fixed kernel banks).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  It is the plain definition of
 * what the GPU path must compute, written out with naive loops in double
 * precision.  Only the test-suite, the smoke check and the bench's
 * "cpu_baseline" leg may call it; the GPU library never links or loads it and
 * shares no source, table or helper with it.
 *
 * Every transform here is exact (up to rounding order): a windowed DFT of each
 * frame, a linear map, direct inner products.  Nothing is blocked, fused or
 * reordered beyond what the definitions state.  The only concession to speed is
 * an OpenMP "parallel for" over independent (waveform, frame) pairs.
 *
 * Readings taken where the paper is silent (all listed in the design notes):
 *   - 'hann' is the periodic Hann window  w[n] = 1/2 - 1/2 cos(2 pi n / N); the Hamming and
 *     Blackman windows the paper also names are taken in the same periodic form.
 *   - center=True pads by N/2 on both sides by mirror reflection that does not
 *     repeat the edge sample; frame t then starts at padded index t*hop.
 *   - number of frames T = 1 + floor((L + 2*pad - N) / hop).
 *   - the convolution with flipped kernels (Sec. III-A) is, per frame, the plain
 *     DFT of eq. (DFT2) with un-flipped n; the oracle never flips.
 *   - Mel filterbank: triangles between equally spaced points on the mel axis,
 *     optional "area" normalisation 2/(f[m+2]-f[m]); applied to |X|^power.
 *   - CQT: eqs. (Q), (N_k), (CQT); kernel k is the periodic Hann window of
 *     length N_k times exp(-2 pi i Q n / N_k), divided by the window sum (L1
 *     norm), centred in n_taps taps with the odd spare zero on the right.
 *
 * Parity status of each function (what pins it is in tests/test_oracle_*.py):
 *   orc_reflect_index, orc_num_frames      pinned (hand-worked example, shapes)
 *   orc_window                              pinned (closed forms)
 *   orc_stft_complex / orc_stft             pinned (textbook DFT, tone peak,
 *                                           Parseval, impulse support)
 *   orc_freq_sigma                          pinned (worked values of Sec. II-B)
 *   orc_stft_sigma_complex / orc_stft_scaled pinned (integer sigma = textbook DFT,
 *                                           tone peak at the bin's frequency)
 *   orc_hz_to_mel / orc_mel_to_hz           pinned (inverse pair, continuity)
 *   orc_mel_filterbank                      pinned (Table 1 of the paper)
 *   orc_mel                                 pinned (Fig. 2 scenario, linearity)
 *   orc_cqt_lengths / orc_cqt_kernels       pinned (lengths quoted in Sec. III-C)
 *   orc_cqt_complex / orc_cqt               pinned (tone magnitude A/2, argmax; phase of a tone)
 *   orc_lowpass_fir / orc_downsample2       pinned (SciPy's window-method design and
 *                                           convolution; tap count and window are this
 *                                           build's choice: the paper gives neither)
 *   orc_cqt2010v2                           pinned (octave by octave against orc_cqt on
 *                                           SciPy-downsampled signals; tones A/2)
 *   output format 2 (log)                   parity unpinned beyond log of the
 *                                           pinned power (paper gives no formula)
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_OK 0
#define ORC_EINVAL 1
#define ORC_ENOMEM 2

#define ORC_PI 3.14159265358979323846264338327950288

/* output formats */
#define ORC_MAGNITUDE 0
#define ORC_POWER 1
#define ORC_LOG 2
/* floor inside the logarithm of format 2: ln(max(power, ORC_LOG_FLOOR)) */
#define ORC_LOG_FLOOR 1e-10

/* windows */
#define ORC_WIN_HANN 0
#define ORC_WIN_RECT 1
#define ORC_WIN_HAMMING 2
#define ORC_WIN_BLACKMAN 3

/* frequency axis of the STFT (Sec. II-B) */
#define ORC_FREQ_DFT 0
#define ORC_FREQ_LINEAR 1
#define ORC_FREQ_LOG 2

/* mel scales */
#define ORC_MEL_SLANEY 0
#define ORC_MEL_HTK 1

int orc_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* Mirror reflection about the first and last sample without repeating them
 * (pad_mode='reflect', Sec. III-A API paragraph).  Valid for -(L-1) <= j <= 2L-2. */
long long orc_reflect_index(long long j, long long L) {
  if (j < 0) return -j;
  if (j >= L) return 2 * (L - 1) - j;
  return j;
}

/* Number of frames of a length-L signal: windows of N samples every hop samples
 * over the (optionally padded) signal (Sec. III-A, "T windows"). */
long long orc_num_frames(long long L, long long N, long long hop, int center) {
  long long padded = L + (center ? 2 * (N / 2) : 0);
  if (padded < N || hop < 1) return 0;
  return 1 + (padded - N) / hop;
}

/* Sample n of the length-N window (Sec. III-A, window paragraph: Hann, Hamming and Blackman are the
 * types it names), in the periodic form that suits a DFT of the same length: the textbook cosine
 * sums with 2 pi n / N (not N - 1) as their argument. */
static int window_known(int kind) { return kind >= ORC_WIN_HANN && kind <= ORC_WIN_BLACKMAN; }
static double window_at(int kind, long long n, long long N) {
  const double a = 2.0 * ORC_PI * (double)n / (double)N;
  switch (kind) {
    case ORC_WIN_HANN: return 0.5 - 0.5 * cos(a);
    case ORC_WIN_HAMMING: return 0.54 - 0.46 * cos(a);
    case ORC_WIN_BLACKMAN: return 0.42 - 0.5 * cos(a) + 0.08 * cos(2.0 * a);
    default: return 1.0;
  }
}

int orc_window(int kind, long long N, double *w) {
  if (N < 1 || !w || !window_known(kind)) return ORC_EINVAL;
  for (long long n = 0; n < N; ++n) w[n] = window_at(kind, n, N);
  return ORC_OK;
}

/* sample i of the padded waveform (padding by `pad` on both sides) */
static inline double padded_sample(const float *x, long long L, long long pad, long long i) {
  return (double)x[orc_reflect_index(i - pad, L)];
}

/* STFT, eq. (DFT2) applied to every window:
 *   Re[b,k,t] =  sum_n w[n] xp_b[t hop + n] cos(2 pi k n / N)
 *   Im[b,k,t] = -sum_n w[n] xp_b[t hop + n] sin(2 pi k n / N),   k = 0..N/2.
 * The cos/sin values come from a table of cos/sin(2 pi m / N), m = 0..N-1, read at
 * m = (k n) mod N: exact argument reduction, still N multiply-adds per (k, frame).
 * re, im: [B, N/2+1, T] row-major (T fastest). */
int orc_stft_complex(const float *x, long long B, long long L, int n_fft, int hop,
                     int window, int center, double *re, double *im) {
  if (!x || !re || !im || B < 1 || n_fft < 2 || (n_fft & 1) || hop < 1) return ORC_EINVAL;
  const long long N = n_fft, F = N / 2 + 1, pad = center ? N / 2 : 0;
  if (center && L <= pad) return ORC_EINVAL; /* reflection undefined */
  const long long T = orc_num_frames(L, N, hop, center);
  if (T < 1) return ORC_EINVAL;
  double *w = (double *)malloc(sizeof(double) * N);
  double *ct = (double *)malloc(sizeof(double) * N);
  double *st = (double *)malloc(sizeof(double) * N);
  if (!w || !ct || !st) { free(w); free(ct); free(st); return ORC_ENOMEM; }
  if (orc_window(window, N, w) != ORC_OK) { free(w); free(ct); free(st); return ORC_EINVAL; }
  for (long long m = 0; m < N; ++m) {
    ct[m] = cos(2.0 * ORC_PI * (double)m / (double)N);
    st[m] = sin(2.0 * ORC_PI * (double)m / (double)N);
  }
  int fail = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 4)
  for (long long b = 0; b < B; ++b) {
    for (long long t = 0; t < T; ++t) {
      double *frame = (double *)malloc(sizeof(double) * N);
      if (!frame) { fail = 1; continue; }
      const float *xb = x + b * L;
      for (long long n = 0; n < N; ++n) frame[n] = w[n] * padded_sample(xb, L, pad, t * hop + n);
      for (long long k = 0; k < F; ++k) {
        double sr = 0.0, si = 0.0;
        long long m = 0; /* m = (k n) mod N, stepped by k (k <= N/2 < N) */
        for (long long n = 0; n < N; ++n) {
          sr += frame[n] * ct[m];
          si += frame[n] * st[m];
          m += k;
          if (m >= N) m -= N;
        }
        re[(b * F + k) * T + t] = sr;
        im[(b * F + k) * T + t] = -si;
      }
      free(frame);
    }
  }
  free(w); free(ct); free(st);
  return fail ? ORC_ENOMEM : ORC_OK;
}

static inline double apply_format(double pw, int fmt) {
  if (fmt == ORC_MAGNITUDE) return sqrt(pw);
  if (fmt == ORC_POWER) return pw;
  return log(pw > ORC_LOG_FLOOR ? pw : ORC_LOG_FLOOR);
}

/* Spectrogram: magnitude sqrt(Re^2+Im^2), power Re^2+Im^2, or ln(max(power, floor))
 * (Fig. 1 and its caption).  out: [B, N/2+1, T]. */
int orc_stft(const float *x, long long B, long long L, int n_fft, int hop, int window,
             int center, int fmt, double *out) {
  if (!out || fmt < 0 || fmt > 2) return ORC_EINVAL;
  const long long F = n_fft / 2 + 1;
  const long long T = orc_num_frames(L, n_fft, hop, center);
  if (T < 1 || B < 1) return ORC_EINVAL;
  const long long n = B * F * T;
  double *re = (double *)malloc(sizeof(double) * n);
  double *im = (double *)malloc(sizeof(double) * n);
  if (!re || !im) { free(re); free(im); return ORC_ENOMEM; }
  int rc = orc_stft_complex(x, B, L, n_fft, hop, window, center, re, im);
  if (rc == ORC_OK)
    for (long long i = 0; i < n; ++i) out[i] = apply_format(re[i] * re[i] + im[i] * im[i], fmt);
  free(re); free(im);
  return rc;
}

/* Normalised frequency sigma(k) of bin k when the DFT's basis frequencies are re-spaced
 * between f_s and f_e over mu bins (Sec. II-B):
 *   linear, eq. (linear-frequency-DFT):  sigma(k) = (f_e - f_s) N / (mu s) * k + f_s N / s
 *   log,    eq. (log-frequency-DFT):     sigma(k) = (f_s N / s) * (f_e / f_s)^(k / mu)
 * with k = 0..mu-1, as in the worked example of that section (f_s = 50, f_e = 6000,
 * N = 2048, s = 44100, 1025 bins).  scale 0 gives the plain DFT, sigma(k) = k. */
double orc_freq_sigma(int scale, long long k, double f_s, double f_e, long long mu, long long N, double s) {
  if (scale == ORC_FREQ_LINEAR) return (f_e - f_s) * (double)N / ((double)mu * s) * (double)k + f_s * (double)N / s;
  if (scale == ORC_FREQ_LOG) return f_s * (double)N / s * pow(f_e / f_s, (double)k / (double)mu);
  return (double)k;
}

/* STFT with re-spaced basis frequencies, eq. (DFT3) applied to every window:
 *   Re[b,k,t] =  sum_n w[n] xp_b[t hop + n] cos(2 pi sigma[k] n / N)
 *   Im[b,k,t] = -sum_n w[n] xp_b[t hop + n] sin(2 pi sigma[k] n / N),   k = 0..n_bins-1,
 * for any real sigma[k] (no table trick: sigma is not an integer).  re, im: [B, n_bins, T]. */
int orc_stft_sigma_complex(const float *x, long long B, long long L, int n_fft, int hop, int window,
                           int center, long long n_bins, const double *sigma, double *re, double *im) {
  if (!x || !re || !im || !sigma || B < 1 || n_fft < 2 || (n_fft & 1) || hop < 1 || n_bins < 1) return ORC_EINVAL;
  const long long N = n_fft, pad = center ? N / 2 : 0;
  if (center && L <= pad) return ORC_EINVAL;
  const long long T = orc_num_frames(L, N, hop, center);
  if (T < 1) return ORC_EINVAL;
  double *w = (double *)malloc(sizeof(double) * N);
  double *ct = (double *)malloc(sizeof(double) * N * n_bins);
  double *st = (double *)malloc(sizeof(double) * N * n_bins);
  if (!w || !ct || !st) { free(w); free(ct); free(st); return ORC_ENOMEM; }
  if (orc_window(window, N, w) != ORC_OK) { free(w); free(ct); free(st); return ORC_EINVAL; }
  for (long long k = 0; k < n_bins; ++k)
    for (long long n = 0; n < N; ++n) {
      const double a = 2.0 * ORC_PI * sigma[k] * (double)n / (double)N;
      ct[k * N + n] = cos(a);
      st[k * N + n] = sin(a);
    }
  int fail = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 4)
  for (long long b = 0; b < B; ++b) {
    for (long long t = 0; t < T; ++t) {
      double *frame = (double *)malloc(sizeof(double) * N);
      if (!frame) { fail = 1; continue; }
      const float *xb = x + b * L;
      for (long long n = 0; n < N; ++n) frame[n] = w[n] * padded_sample(xb, L, pad, t * hop + n);
      for (long long k = 0; k < n_bins; ++k) {
        double sr = 0.0, si = 0.0;
        for (long long n = 0; n < N; ++n) {
          sr += frame[n] * ct[k * N + n];
          si += frame[n] * st[k * N + n];
        }
        re[(b * n_bins + k) * T + t] = sr;
        im[(b * n_bins + k) * T + t] = -si;
      }
      free(frame);
    }
  }
  free(w); free(ct); free(st);
  return fail ? ORC_ENOMEM : ORC_OK;
}

/* Spectrogram on a linear or log frequency axis (Sec. II-B; the STFT's freq_scale argument,
 * Sec. III-A): bins k = 0..freq_bins-1 at sigma(k) between fmin and fmax.  out: [B, freq_bins, T]. */
int orc_stft_scaled(const float *x, long long B, long long L, int sr, int n_fft, int hop, int window,
                    int center, int scale, double fmin, double fmax, long long freq_bins, int fmt, double *out) {
  if (!out || fmt < 0 || fmt > 2 || freq_bins < 1) return ORC_EINVAL;
  if (scale != ORC_FREQ_LINEAR && scale != ORC_FREQ_LOG) return ORC_EINVAL;
  if (!(fmax > fmin) || fmin < 0.0 || (scale == ORC_FREQ_LOG && !(fmin > 0.0))) return ORC_EINVAL;
  const long long T = orc_num_frames(L, n_fft, hop, center);
  if (T < 1 || B < 1) return ORC_EINVAL;
  const long long n = B * freq_bins * T;
  double *sigma = (double *)malloc(sizeof(double) * freq_bins);
  double *re = (double *)malloc(sizeof(double) * n);
  double *im = (double *)malloc(sizeof(double) * n);
  if (!sigma || !re || !im) { free(sigma); free(re); free(im); return ORC_ENOMEM; }
  for (long long k = 0; k < freq_bins; ++k) sigma[k] = orc_freq_sigma(scale, k, fmin, fmax, freq_bins, n_fft, (double)sr);
  int rc = orc_stft_sigma_complex(x, B, L, n_fft, hop, window, center, freq_bins, sigma, re, im);
  if (rc == ORC_OK)
    for (long long i = 0; i < n; ++i) out[i] = apply_format(re[i] * re[i] + im[i] * im[i], fmt);
  free(sigma); free(re); free(im);
  return rc;
}

/* Hz -> mel.  HTK form: eq. (mel-o); Slaney / Auditory-Toolbox form: eq. (mel-stanley),
 * linear 3f/200 below 1000 Hz and 15 + 27 ln(f/1000)/ln(6.4) above. */
double orc_hz_to_mel(double f, int scale) {
  if (scale == ORC_MEL_HTK) return 2595.0 * log10(1.0 + f / 700.0);
  if (f < 1000.0) return 3.0 * f / 200.0;
  return 15.0 + 27.0 * log(f / 1000.0) / log(6.4);
}

/* inverse of orc_hz_to_mel */
double orc_mel_to_hz(double m, int scale) {
  if (scale == ORC_MEL_HTK) return 700.0 * (pow(10.0, m / 2595.0) - 1.0);
  if (m < 15.0) return 200.0 * m / 3.0;
  return 1000.0 * exp((m - 15.0) * log(6.4) / 27.0);
}

/* Triangular Mel filterbank (Sec. III-B): n_mels+2 edge frequencies equally spaced on
 * the mel axis between fmin and fmax; filter m rises linearly from edge m to edge m+1
 * and falls to edge m+2, evaluated at the DFT bin frequencies j*sr/n_fft (eq.
 * f-k-conversion).  norm_area=1 scales row m by 2/(edge[m+2]-edge[m]).
 * W: [n_mels, n_fft/2+1]; edges (may be NULL): [n_mels+2] in Hz. */
int orc_mel_filterbank(int sr, int n_fft, int n_mels, double fmin, double fmax, int scale,
                       int norm_area, double *W, double *edges_out) {
  if (!W || sr < 1 || n_fft < 2 || (n_fft & 1) || n_mels < 1) return ORC_EINVAL;
  if (fmax <= 0.0) fmax = 0.5 * (double)sr;
  if (fmin < 0.0 || fmax <= fmin || fmax > 0.5 * (double)sr) return ORC_EINVAL;
  if (scale != ORC_MEL_SLANEY && scale != ORC_MEL_HTK) return ORC_EINVAL;
  const long long F = n_fft / 2 + 1;
  double *e = (double *)malloc(sizeof(double) * (n_mels + 2));
  if (!e) return ORC_ENOMEM;
  const double m_lo = orc_hz_to_mel(fmin, scale), m_hi = orc_hz_to_mel(fmax, scale);
  for (int i = 0; i < n_mels + 2; ++i)
    e[i] = orc_mel_to_hz(m_lo + (m_hi - m_lo) * (double)i / (double)(n_mels + 1), scale);
  for (int m = 0; m < n_mels; ++m) {
    for (long long j = 0; j < F; ++j) {
      const double nu = (double)j * (double)sr / (double)n_fft;
      const double up = (nu - e[m]) / (e[m + 1] - e[m]);
      const double down = (e[m + 2] - nu) / (e[m + 2] - e[m + 1]);
      double v = up < down ? up : down;
      if (v < 0.0) v = 0.0;
      if (norm_area) v *= 2.0 / (e[m + 2] - e[m]);
      W[m * F + j] = v;
    }
  }
  if (edges_out) memcpy(edges_out, e, sizeof(double) * (n_mels + 2));
  free(e);
  return ORC_OK;
}

/* Mel spectrogram (Sec. III-B, Fig. 3): Mel[b,m,t] = sum_j W[m,j] |X_t[j]|^power,
 * power = 1 (magnitude) or 2.  out: [B, n_mels, T]. */
int orc_mel(const float *x, long long B, long long L, int sr, int n_fft, int hop, int window,
            int center, int n_mels, double fmin, double fmax, int scale, int norm_area,
            double power, double *out) {
  if (!out || (power != 1.0 && power != 2.0)) return ORC_EINVAL;
  const long long F = n_fft / 2 + 1;
  const long long T = orc_num_frames(L, n_fft, hop, center);
  if (T < 1 || B < 1 || n_mels < 1) return ORC_EINVAL;
  double *W = (double *)malloc(sizeof(double) * n_mels * F);
  double *S = (double *)malloc(sizeof(double) * B * F * T);
  if (!W || !S) { free(W); free(S); return ORC_ENOMEM; }
  int rc = orc_mel_filterbank(sr, n_fft, n_mels, fmin, fmax, scale, norm_area, W, NULL);
  if (rc == ORC_OK)
    rc = orc_stft(x, B, L, n_fft, hop, window, center, power == 2.0 ? ORC_POWER : ORC_MAGNITUDE, S);
  if (rc == ORC_OK) {
#pragma omp parallel for collapse(2)
    for (long long b = 0; b < B; ++b)
      for (long long m = 0; m < n_mels; ++m)
        for (long long t = 0; t < T; ++t) {
          double acc = 0.0;
          for (long long j = 0; j < F; ++j) acc += W[m * F + j] * S[(b * F + j) * T + t];
          out[(b * n_mels + m) * T + t] = acc;
        }
  }
  free(W); free(S);
  return rc;
}

/* eq. (Q): number of cycles in every constant-Q kernel */
double orc_cqt_Q(int bins_per_octave) { return 1.0 / (pow(2.0, 1.0 / (double)bins_per_octave) - 1.0); }

/* Centre frequencies f_k = fmin 2^(k/b) and kernel lengths N_k = ceil(Q sr / f_k),
 * eq. (N_k), in double precision.  Either output may be NULL. */
int orc_cqt_lengths(int sr, double fmin, int n_bins, int bins_per_octave, long long *N_k, double *f_k) {
  if (sr < 1 || fmin <= 0.0 || n_bins < 1 || bins_per_octave < 1) return ORC_EINVAL;
  const double Q = orc_cqt_Q(bins_per_octave);
  for (int k = 0; k < n_bins; ++k) {
    const double f = fmin * pow(2.0, (double)k / (double)bins_per_octave);
    if (f_k) f_k[k] = f;
    if (N_k) N_k[k] = (long long)ceil(Q * (double)sr / f);
  }
  return ORC_OK;
}

/* smallest power of two >= the longest kernel (the default n_taps, Sec. III-C) */
long long orc_cqt_default_taps(int sr, double fmin, int bins_per_octave) {
  long long n0 = 0;
  if (orc_cqt_lengths(sr, fmin, 1, bins_per_octave, &n0, NULL) != ORC_OK) return 0;
  long long p = 1;
  while (p < n0) p <<= 1;
  return p;
}

/* one tap of kernel k: window(N_k)[n] * exp(-2 pi i Q n / N_k) / sum(window) */
static void cqt_tap(int window, double Q, long long Nk, double wsum, long long n, double *re, double *im) {
  const double w = window_at(window, n, Nk);
  const double ph = 2.0 * ORC_PI * Q * (double)n / (double)Nk;
  *re = w * cos(ph) / wsum;
  *im = -w * sin(ph) / wsum;
}

static double window_sum(int window, long long Nk) {
  double s = 0.0;
  for (long long n = 0; n < Nk; ++n)
    s += window_at(window, n, Nk);
  return s;
}

/* Time-domain CQT kernel bank (Sec. III-C "CQT with time domain kernels", Fig. 4):
 * row k holds kernel k in taps [s_k, s_k+N_k), s_k = (n_taps-N_k)/2 (integer
 * division), zeros elsewhere.  kre, kim: [n_bins, n_taps]. */
int orc_cqt_kernels(int sr, double fmin, int n_bins, int bins_per_octave, int window,
                    long long n_taps, double *kre, double *kim) {
  if (!kre || !kim || n_taps < 1) return ORC_EINVAL;
  if (!window_known(window)) return ORC_EINVAL;
  long long *Nk = (long long *)malloc(sizeof(long long) * n_bins);
  if (!Nk) return ORC_ENOMEM;
  int rc = orc_cqt_lengths(sr, fmin, n_bins, bins_per_octave, Nk, NULL);
  if (rc == ORC_OK && Nk[0] > n_taps) rc = ORC_EINVAL;
  if (rc != ORC_OK) { free(Nk); return rc; }
  const double Q = orc_cqt_Q(bins_per_octave);
  memset(kre, 0, sizeof(double) * n_bins * n_taps);
  memset(kim, 0, sizeof(double) * n_bins * n_taps);
  for (int k = 0; k < n_bins; ++k) {
    const long long s = (n_taps - Nk[k]) / 2;
    const double ws = window_sum(window, Nk[k]);
    for (long long n = 0; n < Nk[k]; ++n)
      cqt_tap(window, Q, Nk[k], ws, n, &kre[k * n_taps + s + n], &kim[k * n_taps + s + n]);
  }
  free(Nk);
  return ORC_OK;
}

/* Constant-Q transform by direct inner products (eq. (CQT) per bin and frame; the "naive" loop of
 * Sec. III-C), complex result:
 *   X[b,k,t] = sum_{n<N_k} xp_b[t hop + s_k + n] w_k[n] exp(-2 pi i Q n / N_k) / sum(w_k)
 * with xp padded by n_taps/2 when center.  re, im: [B, n_bins, T]. */
int orc_cqt_complex(const float *x, long long B, long long L, int sr, int hop, double fmin, int n_bins,
                    int bins_per_octave, int window, int center, long long n_taps, double *re, double *im) {
  if (!x || !re || !im || B < 1 || hop < 1) return ORC_EINVAL;
  if (!window_known(window)) return ORC_EINVAL;
  if (n_taps <= 0) n_taps = orc_cqt_default_taps(sr, fmin, bins_per_octave);
  if (n_taps < 2 || (n_taps & 1)) return ORC_EINVAL;
  const long long pad = center ? n_taps / 2 : 0;
  if (center && L <= pad) return ORC_EINVAL;
  const long long T = orc_num_frames(L, n_taps, hop, center);
  if (T < 1) return ORC_EINVAL;
  long long *Nk = (long long *)malloc(sizeof(long long) * n_bins);
  if (!Nk) return ORC_ENOMEM;
  int rc = orc_cqt_lengths(sr, fmin, n_bins, bins_per_octave, Nk, NULL);
  if (rc == ORC_OK && Nk[0] > n_taps) rc = ORC_EINVAL;
  if (rc != ORC_OK) { free(Nk); return rc; }
  const double Q = orc_cqt_Q(bins_per_octave);
  /* kernels stored compactly: bin k at offset off[k], N_k complex taps */
  long long total = 0;
  long long *off = (long long *)malloc(sizeof(long long) * n_bins);
  if (!off) { free(Nk); return ORC_ENOMEM; }
  for (int k = 0; k < n_bins; ++k) { off[k] = total; total += Nk[k]; }
  double *yre = (double *)malloc(sizeof(double) * total);
  double *yim = (double *)malloc(sizeof(double) * total);
  if (!yre || !yim) { free(Nk); free(off); free(yre); free(yim); return ORC_ENOMEM; }
  for (int k = 0; k < n_bins; ++k) {
    const double ws = window_sum(window, Nk[k]);
    for (long long n = 0; n < Nk[k]; ++n) cqt_tap(window, Q, Nk[k], ws, n, &yre[off[k] + n], &yim[off[k] + n]);
  }
#pragma omp parallel for collapse(2) schedule(dynamic, 4)
  for (long long b = 0; b < B; ++b) {
    for (long long t = 0; t < T; ++t) {
      const float *xb = x + b * L;
      for (int k = 0; k < n_bins; ++k) {
        const long long s = (n_taps - Nk[k]) / 2;
        double sr_ = 0.0, si_ = 0.0;
        for (long long n = 0; n < Nk[k]; ++n) {
          const double v = padded_sample(xb, L, pad, t * hop + s + n);
          sr_ += v * yre[off[k] + n];
          si_ += v * yim[off[k] + n];
        }
        re[(b * n_bins + k) * T + t] = sr_;
        im[(b * n_bins + k) * T + t] = si_;
      }
    }
  }
  free(Nk); free(off); free(yre); free(yim);
  return ORC_OK;
}

/* Constant-Q spectrogram: the transform above, formatted like orc_stft.  out: [B, n_bins, T]. */
int orc_cqt(const float *x, long long B, long long L, int sr, int hop, double fmin, int n_bins,
            int bins_per_octave, int window, int center, long long n_taps, int fmt, double *out) {
  if (!out || fmt < 0 || fmt > 2 || B < 1 || hop < 1) return ORC_EINVAL;
  if (n_taps <= 0) n_taps = orc_cqt_default_taps(sr, fmin, bins_per_octave);
  const long long T = orc_num_frames(L, n_taps, hop, center);
  if (T < 1) return ORC_EINVAL;
  const long long n = B * (long long)n_bins * T;
  double *re = (double *)malloc(sizeof(double) * n);
  double *im = (double *)malloc(sizeof(double) * n);
  if (!re || !im) { free(re); free(im); return ORC_ENOMEM; }
  int rc = orc_cqt_complex(x, B, L, sr, hop, fmin, n_bins, bins_per_octave, window, center, n_taps, re, im);
  if (rc == ORC_OK)
    for (long long i = 0; i < n; ++i) out[i] = apply_format(re[i] * re[i] + im[i] * im[i], fmt);
  free(re); free(im);
  return rc;
}

/* ---------------------------------------------------------------------------------------
 * CQT by recursive downsampling with time-domain kernels (Sec. III-C, "Downsampling",
 * "Constant-Q transform (2010 version)" and "CQT with time domain kernels"; Figs. CQT2010,
 * CQT2010v2).
 *
 * Readings taken where the paper is silent (all listed in the design notes):
 *   - the anti-alias filter is the textbook window-method design: ideal low-pass impulse
 *     response with its cutoff half-way between the stated pass-band end (0.4995) and
 *     stop-band start (0.5005), i.e. at 0.5 of the Nyquist frequency, times a Hamming window
 *     (the default of the SciPy routine the paper names), scaled to unit gain at 0 Hz; the
 *     tap count is an argument (odd, so that the filter has an integer delay);
 *   - the filter is centred on the sample it produces (zero delay) and the waveform is
 *     extended by the same mirror reflection as everywhere else (pad_mode = 'reflect');
 *     a length-L waveform downsamples to ceil(L/2) samples, y[m] centred on x[2m];
 *   - octave a (0 = top) is computed from the waveform downsampled a times, with hop / 2^a,
 *     so that every octave has the frames of the top one (T = 1 + floor(L / hop));
 *   - the kernels of octave a are those of eq. (CQT)/(N_k) for its bins' frequencies times 2^a
 *     at the original sample rate (one kernel set when n_bins is a multiple of the bins per
 *     octave), L1-normalised as in orc_cqt_kernels; no further per-octave scaling is applied
 *     (the filter has unit pass-band gain, so a tone reads A/2 in every octave);
 *   - no "early downsampling" before the top octave.
 * ------------------------------------------------------------------------------------- */

/* Window-method low-pass FIR, cutoff as a fraction of the Nyquist frequency:
 *   h[i] = cutoff sinc(cutoff (i - (n-1)/2)) (0.54 - 0.46 cos(2 pi i / (n-1))),  then h /= sum(h). */
int orc_lowpass_fir(int n_taps, double cutoff, double *h) {
  if (!h || n_taps < 3 || !(cutoff > 0.0 && cutoff < 1.0)) return ORC_EINVAL;
  double sum = 0.0;
  for (int i = 0; i < n_taps; ++i) {
    const double u = (double)i - 0.5 * (double)(n_taps - 1);
    const double a = ORC_PI * cutoff * u;
    const double sinc = (u == 0.0) ? 1.0 : sin(a) / a;
    h[i] = cutoff * sinc * (0.54 - 0.46 * cos(2.0 * ORC_PI * (double)i / (double)(n_taps - 1)));
    sum += h[i];
  }
  for (int i = 0; i < n_taps; ++i) h[i] /= sum;
  return ORC_OK;
}

/* y[m] = sum_i h[i] x~[2m + i - (n_taps-1)/2],  m = 0..ceil(L/2)-1, x~ = x mirrored at both
 * ends (eq. (FIR) followed by keeping every second sample; h is symmetric). */
int orc_downsample2(const double *x, long long L, const double *h, int n_taps, double *y) {
  if (!x || !h || !y || n_taps < 1 || !(n_taps & 1)) return ORC_EINVAL;
  const long long half = (n_taps - 1) / 2;
  if (L <= half) return ORC_EINVAL; /* reflection undefined */
  const long long Ly = (L + 1) / 2;
  for (long long m = 0; m < Ly; ++m) {
    double s = 0.0;
    for (long long i = 0; i < n_taps; ++i) s += h[i] * x[orc_reflect_index(2 * m + i - half, L)];
    y[m] = s;
  }
  return ORC_OK;
}

/* number of octaves and, for octave a (0 = top), its bins [lo, hi) */
static int cqt2010_octaves(int n_bins, int b) { return (n_bins + b - 1) / b; }
static void cqt2010_bins(int n_bins, int b, int a, int *lo, int *hi) {
  *hi = n_bins - a * b;
  *lo = *hi - b > 0 ? *hi - b : 0;
}
/* length of the kernel of global bin k, which belongs to octave a: N = ceil(Q sr / (f_k 2^a)) */
static long long cqt2010_length(int sr, double fmin, int b, int k, int a) {
  const double f = fmin * pow(2.0, (double)(k + a * b) / (double)b);
  return (long long)ceil(orc_cqt_Q(b) * (double)sr / f);
}

/* default taps: smallest power of two >= the longest top-octave kernel */
long long orc_cqt2010_default_taps(int sr, double fmin, int n_bins, int bins_per_octave) {
  if (sr < 1 || fmin <= 0.0 || n_bins < 1 || bins_per_octave < 1) return 0;
  int lo, hi;
  cqt2010_bins(n_bins, bins_per_octave, 0, &lo, &hi);
  const long long n0 = cqt2010_length(sr, fmin, bins_per_octave, lo, 0);
  long long p = 1;
  while (p < n0) p <<= 1;
  return p;
}

int orc_cqt2010v2(const float *x, long long B, long long L, int sr, int hop, double fmin, int n_bins,
                  int bins_per_octave, int window, long long n_taps, int fir_taps, int fmt, double *out) {
  if (!x || !out || B < 1 || hop < 1 || fmt < 0 || fmt > 2 || n_bins < 1 || bins_per_octave < 1) return ORC_EINVAL;
  if (!window_known(window)) return ORC_EINVAL;
  if (sr < 1 || fmin <= 0.0 || fir_taps < 3 || !(fir_taps & 1)) return ORC_EINVAL;
  const int b = bins_per_octave, n_oct = cqt2010_octaves(n_bins, b);
  if (n_oct > 30 || hop % (1 << (n_oct - 1)) != 0) return ORC_EINVAL; /* every octave needs an integer hop */
  if (n_taps <= 0) n_taps = orc_cqt2010_default_taps(sr, fmin, n_bins, b);
  if (n_taps < 2 || (n_taps & 1)) return ORC_EINVAL;
  const long long pad = n_taps / 2, T = 1 + L / hop;
  const double Q = orc_cqt_Q(b);
  double *h = (double *)malloc(sizeof(double) * fir_taps);
  if (!h) return ORC_ENOMEM;
  if (orc_lowpass_fir(fir_taps, 0.5, h) != ORC_OK) { free(h); return ORC_EINVAL; }
  int rc = ORC_OK;
#pragma omp parallel for schedule(dynamic, 1)
  for (long long bi = 0; bi < B; ++bi) {
    long long La = L;
    double *xa = (double *)malloc(sizeof(double) * L);
    double *xn = (double *)malloc(sizeof(double) * ((L + 1) / 2));
    double *kre = (double *)malloc(sizeof(double) * n_taps);
    double *kim = (double *)malloc(sizeof(double) * n_taps);
    if (!xa || !xn || !kre || !kim) { rc = ORC_ENOMEM; free(xa); free(xn); free(kre); free(kim); continue; }
    for (long long i = 0; i < L; ++i) xa[i] = (double)x[bi * L + i];
    for (int a = 0; a < n_oct; ++a) {
      const long long hop_a = hop >> a;
      int lo, hi;
      cqt2010_bins(n_bins, b, a, &lo, &hi);
      if (La <= pad) { rc = ORC_EINVAL; break; }
      for (int k = lo; k < hi; ++k) {
        const long long Nk = cqt2010_length(sr, fmin, b, k, a);
        if (Nk > n_taps) { rc = ORC_EINVAL; break; }
        const long long s = (n_taps - Nk) / 2;
        const double ws = window_sum(window, Nk);
        for (long long n = 0; n < Nk; ++n) cqt_tap(window, Q, Nk, ws, n, &kre[n], &kim[n]);
        for (long long t = 0; t < T; ++t) {
          double sr_ = 0.0, si_ = 0.0;
          for (long long n = 0; n < Nk; ++n) {
            const double v = xa[orc_reflect_index(t * hop_a + s + n - pad, La)];
            sr_ += v * kre[n];
            si_ += v * kim[n];
          }
          out[(bi * n_bins + k) * T + t] = apply_format(sr_ * sr_ + si_ * si_, fmt);
        }
      }
      if (rc != ORC_OK) break;
      if (a + 1 < n_oct) {
        if (orc_downsample2(xa, La, h, fir_taps, xn) != ORC_OK) { rc = ORC_EINVAL; break; }
        La = (La + 1) / 2;
        memcpy(xa, xn, sizeof(double) * La);
      }
    }
    free(xa); free(xn); free(kre); free(kim);
  }
  free(h);
  return rc;
}
