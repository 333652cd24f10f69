// Host side of the library: argument checking, kernel-bank construction in double precision,
// permutation of the banks into the order the GPU kernels stream them, and the C ABI itself.
#include <algorithm>
#include <climits>
#include <cmath>
#include <complex>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>

#include "nna_internal.h"

namespace {

thread_local std::string g_err;

nna_status fail(nna_status s, const std::string& msg) {
  g_err = msg;
  return s;
}

nna_status fail_hip(hipError_t e, const char* what) {
  g_err = std::string(what) + ": " + hipGetErrorString(e);
  return NNA_ERR_HIP;
}

constexpr double kPi = 3.141592653589793238462643383279502884;

}  // namespace

struct nna_plan {
  int kind = 0;
  int device = -1;
  int sr = 0, hop = 0, center = 0, window = 0, fmt = 0;
  int K = 0;    // taps: n_fft or n_taps
  int pad = 0;  // reflection padding in front
  bool sliding = false;
  // CQT kernel: taps between consecutive shifts of a chunk's LDS rows (hop when frames share LDS rows, 16 when
  // the hop divides the 16-tap chunk, 0 when every chunk is fetched per frame), and LDS rows per shift
  int tap_stride = 0, row_step = 1;
  // decimation filter: 1 = half-band (zero on the even offsets from its centre, which are then not multiplied)
  int fir_mode = 0;
  // the decimation kernel's taps: he[k] = h[half + 2 (fir_ve0 + k)] on the even samples, ho[k] = h[half + 2 (fir_vo0 + k) + 1]
  // on the odd ones, each zero padded to a multiple of eight
  std::vector<float> h_fir_he, h_fir_ho;
  int fir_ve0 = 0, fir_vo0 = 0;
  float* d_fir_he = nullptr;
  float* d_fir_ho = nullptr;

  // STFT / Mel
  int n_half = 0, n_rt = 0, n_chunks = 0, nj = 1;  // n_half: (Re, Im) slots of the packed bank
  long long bank_groups = 0;
  int freq_scale = 0;         // 0: plain DFT bins; else nna_freq_scale (STFT only)
  int freq_bins = 0;          // re-spaced axis: number of bins
  std::vector<double> sigma;  // re-spaced axis: normalised frequency of each bin

  // output bins of an STFT plan; a plain DFT packs bins 0 and N/2 (both purely real) into slot 0
  int stft_bins() const { return freq_scale ? n_half : n_half + 1; }
  // rows of the output per waveform: the complex format writes (Re, Im) row pairs
  int out_rows() const {
    const int bins = kind == NNA_KIND_STFT ? stft_bins() : kind == NNA_KIND_MEL ? n_mels : n_bins;
    return fmt == NNA_OUT_COMPLEX ? 2 * bins : bins;
  }
  // Mel
  int n_mels = 0, mel_power = 2, n_pass = 0, mel_nyq_any = 0;
  std::vector<float> h_melW;  // [n_mels, F] as rounded to float32
  // CQT with frequency-domain kernels: the real matrix that takes the packed (Re, Im) rows of one
  // STFT frame to the (Re, Im) rows of the constant-Q bins, [2 n_bins, 2 n_half], float32 as uploaded
  std::vector<float> h_linW;
  int cq_window = 0;
  size_t lin_frag_floats = 0;
  int lin_blocks = 4;  // 32-row output blocks per pass of the second contraction (4 or 6)

  // CQT
  int n_bins = 0, bpo = 0, n_rb = 0;
  int k_first = 0;  // bin k sits at fmin 2^((k_first + k) / bpo): non-zero for the octaves of a downsampling plan
  double cq_fmin = 0, Q = 0;
  std::vector<long long> Nk, sk;
  // any bank the CQT kernel runs: row r has its non-zero taps inside [row_s[r], row_e[r])
  int conv_rows = 0;
  std::vector<long long> row_s, row_e;
  // CQT by recursive downsampling: one CQT sub-plan per octave (0 = top) and the decimating filter
  std::vector<nna_plan*> octave;
  nna_plan* fir = nullptr;
  int fir_taps = 0;
  std::vector<double> h_fir;
  std::vector<nna::CqtItem> h_items;
  std::vector<nna::CqtChunk> h_chunks;   // [item][n_chunks]
  int max_jspan = 1;

  double exec_flops = 0, alg_flops = 0;

  // Folded-frame contraction (nna_kernels_fold.hip): plain DFT bank, hop dividing n_fft an even number of
  // times >= 4.  The direct bank stays (inspection, trainable plans, complex / phase output).
  bool fold = false;
  double exec_flops_fold = 0;
  std::vector<float> h_bankf, h_wn;
  size_t bankf_floats = 0;
  float wmid = 0;
  float* d_bankf = nullptr;
  float* d_wn = nullptr;
  float* d_melwf = nullptr;            // Mel weights as the folded kernel's second MFMA reads them
  unsigned char* d_mel_maskf = nullptr;
  bool runs_folded() const { return fold && !d_wrm && precision == 0; }

  // host copy of the packed bank (host-only plans keep it; device plans drop it after upload)
  std::vector<float> h_bank;
  size_t bank_floats = 0;

  // device buffers
  float* d_bank = nullptr;
  // float16-operand STFT: the bank as [row tile][chunk][hop-shift][H_ROWS][H_KC] halves
  int precision = 0;
  int n_rt16 = 0;
  std::vector<_Float16> h_bank16;
  size_t bank16_halves = 0;
  _Float16* d_bank16 = nullptr;
  // the same values in the order a wave of the streamed-bank kernel consumes them:
  // [row tile][chunk][hop-shift][K-step][row half][fragment][64 lanes][8 halves]
  std::vector<_Float16> h_bank16s;
  size_t bank16s_halves = 0;
  _Float16* d_bank16s = nullptr;
  // trainable STFT plans: the packed bank once more, row-major [rows_pad][kp] (zero padded), for the
  // backward pass's waveform gradient; kept in step with d_bank by nna_plan_set_bank
  float* d_wrm = nullptr;
  int kp = 0, rows_pad = 0;
  // trainable Mel plans: the filterbank row-major [mels_pad][fp], zero padded
  float* d_melw_rm = nullptr;
  int fp = 0, mels_pad = 0;
  float* d_melw = nullptr;
  unsigned char* d_mel_mask = nullptr;
  float* d_mel_wnyq = nullptr;
  int* d_mel_pass_rt = nullptr;
  nna::CqtItem* d_items = nullptr;
  nna::CqtChunk* d_chunks = nullptr;
  // trainable CQT plans: index map caller's tensor -> streaming order, each row's tap support, and the
  // tables that let the backward contractions skip what lies outside every support
  int* d_cq_map = nullptr;
  int* d_row_lo = nullptr;
  int* d_row_hi = nullptr;
  int2* d_bw_tiles = nullptr;
  int n_bw_tiles = 0;
  int2* d_shift_rng = nullptr;
  int n_shift = 0, n_ct = 0, n_kc = 0;
};

// Workspace of nna_cqt2010v2_static: the downsampled waveforms of two consecutive octaves live here instead
// of in caller memory.  Every device the library's code is loaded on holds its own copy of the array, at its
// own address; in host code the name is only a handle for hipGetSymbolAddress, never a device address.
static __device__ __align__(256) unsigned char scratch[NNA_STATIC_SCRATCH_BYTES];

namespace {

using nna::CQ_FRAMES;
using nna::CQ_ITEM_RB;
using nna::CQ_KC;
using nna::CQ_LDS_ROWS_MAX;
using nna::CQ_PREFETCH;
using nna::CQ_ROWS;
using nna::ST_FRAMES;
using nna::ST_KC;
using nna::ST_KG;
using nna::ST_LDS_ROWS;
using nna::ST_MEL_BLOCKS;
using nna::ST_NKG;
using nna::ST_RB;
using nna::ST_ROWS;

double window_value(int win, long long n, long long N) {
  const double a = 2.0 * kPi * (double)n / (double)N;  // periodic forms: the argument runs over n / N
  switch (win) {
    case NNA_WIN_RECT: return 1.0;
    case NNA_WIN_HAMMING: return 0.54 - 0.46 * std::cos(a);
    case NNA_WIN_BLACKMAN: return 0.42 - 0.5 * std::cos(a) + 0.08 * std::cos(2.0 * a);
    default: return 0.5 - 0.5 * std::cos(a);  // Hann
  }
}

// ---- device helpers -----------------------------------------------------------------
// Per-device set-up, done once on every device a plan is built for (that device current): the kernels'
// dynamic-LDS attribute, and the address of this device's copy of `scratch`.
std::mutex g_init_mutex;
std::vector<char> g_init_done;
std::vector<void*> g_scratch_ptr;
hipError_t ensure_kernels_init(int device) {
  std::lock_guard<std::mutex> lock(g_init_mutex);
  if ((int)g_init_done.size() <= device) {
    g_init_done.resize(device + 1, 0);
    g_scratch_ptr.resize(device + 1, nullptr);
  }
  if (!g_init_done[device]) {
    hipError_t e = nna::kernels_init();
    if (e != hipSuccess) return e;
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!ptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[device] = ptr;
    g_init_done[device] = 1;
  }
  return hipSuccess;
}

// this device's `scratch`, or NULL if no plan was ever built for it
void* scratch_of(int device) {
  std::lock_guard<std::mutex> lock(g_init_mutex);
  return device >= 0 && device < (int)g_scratch_ptr.size() ? g_scratch_ptr[device] : nullptr;
}

template <typename T>
nna_status upload(T** dst, const void* src, size_t bytes, const char* what) {
  *dst = nullptr;
  if (bytes == 0) bytes = 16;
  hipError_t e = hipMalloc(reinterpret_cast<void**>(dst), bytes);
  if (e != hipSuccess) {
    *dst = nullptr;
    if (e == hipErrorOutOfMemory) return fail(NNA_ERR_ALLOC, std::string("hipMalloc failed for ") + what);
    return fail_hip(e, what);
  }
  if (src) {
    e = hipMemcpy(*dst, src, bytes, hipMemcpyHostToDevice);
    if (e != hipSuccess) return fail_hip(e, what);
  }
  return NNA_OK;
}

struct DeviceGuard {
  int prev = -1;
  bool switched = false;
  hipError_t enter(int dev) {
    hipError_t e = hipGetDevice(&prev);
    if (e != hipSuccess) return e;
    if (prev != dev) {
      e = hipSetDevice(dev);
      if (e != hipSuccess) return e;
      switched = true;
    }
    return hipSuccess;
  }
  ~DeviceGuard() {
    if (switched) (void)hipSetDevice(prev);
  }
};

nna_status check_device(int device) {
  if (device < -1) return fail(NNA_ERR_INVALID_ARG, "device must be >= -1");
  if (device >= 0) {
    int count = 0;
    hipError_t e = hipGetDeviceCount(&count);
    if (e != hipSuccess) return fail_hip(e, "hipGetDeviceCount");
    if (device >= count) return fail(NNA_ERR_HIP, "no such HIP device");
  }
  return NNA_OK;
}

// ---- STFT bank ----------------------------------------------------------------------
// Logical bank value of packed row `pr`, tap k (double).  Packed rows interleave (Re, Im)
// per slot; slot 0 carries the two purely real bins k = 0 and k = N/2, slot s carries bin s.
struct DftTable {
  std::vector<double> c, s, w;
  int N;
  DftTable(int N_, int win) : c(N_), s(N_), w(N_), N(N_) {
    for (int m = 0; m < N; ++m) {
      c[m] = std::cos(2.0 * kPi * (double)m / (double)N);
      s[m] = std::sin(2.0 * kPi * (double)m / (double)N);
      w[m] = window_value(win, m, N);
    }
  }
  // eq. (DFT2) with the window folded in: Re kernel w cos(2 pi k n/N), Im kernel -w sin(...)
  double re(int k, int n) const { return w[n] * c[(int)(((long long)k * n) % N)]; }
  double im(int k, int n) const { return -w[n] * s[(int)(((long long)k * n) % N)]; }
};

double stft_packed_value(const DftTable& t, int n_half, int pr, int k) {
  if (k >= t.N) return 0.0;
  const int slot = pr >> 1, part = pr & 1;
  if (slot >= n_half) return 0.0;
  if (slot == 0) return part == 0 ? t.re(0, k) : t.re(n_half, k);
  return part == 0 ? t.re(slot, k) : t.im(slot, k);
}

// tap index of (chunk c, shift j, fragment kg, lane half h, element e)
inline int stft_tap(const nna_plan* p, int c, int j, int kg, int h, int e) {
  return j * p->hop + c * ST_KC + kg * ST_KG + 4 * h + e;
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
  p->bankf_floats = (size_t)(G * p->n_rt + ST_NKG) * ST_RB * 64 * 4;
  p->h_bankf.assign(p->bankf_floats, 0.0f);
  DftTable tab(N, p->window);
  for (int rt = 0; rt < p->n_rt; ++rt)
    for (int c = 0; c < p->n_chunks; ++c)
      for (int j = 0; j < nj2; ++j)
        for (int kg = 0; kg < ST_NKG; ++kg) {
          const long long g = ((long long)c * nj2 + j) * ST_NKG + kg;
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

struct MelDeviceLayout {
  std::vector<float> fragf;         // folded kernel: [pass][rt][blk 2][mb][4][64][4]
  std::vector<unsigned char> maskf; // folded kernel: [pass][rt][blk 2]
  double exec_blocks_f = 0;
  std::vector<float> frag;          // [pass][rt][rb][mb][2][64][4]
  std::vector<unsigned char> mask;  // [pass][rt][rb]
  std::vector<float> wnyq;          // [n_mels]
  std::vector<int> pass_rt;         // [pass][2]
};

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
  if (p->fold) {
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
  if (p->fold) {
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

// index of (pass, row tile, row block, out block, quad v, lane, element e) in the fragment array of
// the second contraction, and the matrix entry it holds: output row pass*128 + mb*32 + lane%32,
// packed row rt*128 + rb*32 + 8 v + 4 (lane/32) + e
inline size_t lin_frag_index(const nna_plan* p, int pass, int rt, int rb, int mb, int v, int lane, int e) {
  return ((((((size_t)pass * p->n_rt + rt) * ST_RB + rb) * p->lin_blocks + mb) * 4 + v) * 64 + lane) * 4 + e;
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
struct CqtKernelGen {
  const nna_plan* p;
  std::vector<double> wsum;
  explicit CqtKernelGen(const nna_plan* p_) : p(p_), wsum(p_->n_bins) {
    for (int k = 0; k < p->n_bins; ++k) {
      double s = 0;
      for (long long n = 0; n < p->Nk[k]; ++n) s += window_value(p->window, n, p->Nk[k]);
      wsum[k] = s;
    }
  }
  // logical bank value: row 2k = Re, 2k+1 = Im of window(N_k)[n] exp(-2 pi i Q n / N_k) / sum(window)
  double value(int row, long long tap) const {
    const int k = row >> 1;
    if (k >= p->n_bins || tap >= p->K) return 0.0;
    const long long n = tap - p->sk[k];
    if (n < 0 || n >= p->Nk[k]) return 0.0;
    const double w = window_value(p->window, n, p->Nk[k]) / wsum[k];
    const double ph = 2.0 * kPi * p->Q * (double)n / (double)p->Nk[k];
    return (row & 1) ? -w * std::sin(ph) : w * std::cos(ph);
  }
};

inline long long floor_div(long long a, long long b) { return a >= 0 ? a / b : -((-a + b - 1) / b); }
inline long long ceil_div(long long a, long long b) { return -floor_div(-a, b); }

// Visit every bank fragment of a CQT plan in the order the kernel consumes them:
// fn(fragment index, row block, hop-shift j (absolute), c0, is_real)
template <typename Fn>
void for_each_cqt_fragment(const nna_plan* p, Fn fn) {
  for (size_t it = 0; it < p->h_items.size(); ++it) {
    const nna::CqtItem& item = p->h_items[it];
    long long f = item.frag0;
    for (int c = 0; c < item.n_chunks; ++c) {
      const nna::CqtChunk& ck = p->h_chunks[it * p->n_chunks + c];
      for (int r = 0; r < item.n_rb; ++r)
        for (int jj = 0; jj < (ck.nj[r] & 0xffff); ++jj, ++f)
          fn(f, item.rb_first + r, ck.jlo + ck.joff[r] + jj, ck.c0, jj < (ck.nj[r] >> 16));
    }
  }
}

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

nna_status finish_plan(nna_plan* p, nna_plan** out, const MelDeviceLayout* mel) {
  if (p->device >= 0) {
    DeviceGuard guard;
    hipError_t e = guard.enter(p->device);
    if (e != hipSuccess) {
      delete p;
      return fail_hip(e, "hipSetDevice");
    }
    e = ensure_kernels_init(p->device);
    if (e != hipSuccess) {
      delete p;
      return fail_hip(e, "kernel attribute setup");
    }
    nna_status s = upload(&p->d_bank, p->h_bank.data(), p->bank_floats * sizeof(float), "kernel bank");
    if (s == NNA_OK && p->precision == NNA_PREC_F16)
      s = upload(&p->d_bank16, p->h_bank16.data(), p->bank16_halves * sizeof(_Float16), "float16 kernel bank");
    if (s == NNA_OK && p->precision == NNA_PREC_F16 && p->bank16s_halves)
      s = upload(&p->d_bank16s, p->h_bank16s.data(), p->bank16s_halves * sizeof(_Float16), "float16 kernel bank (streaming order)");
    if (s == NNA_OK && p->fold) {
      s = upload(&p->d_bankf, p->h_bankf.data(), p->bankf_floats * sizeof(float), "folded kernel bank");
      if (s == NNA_OK) s = upload(&p->d_wn, p->h_wn.data(), p->h_wn.size() * sizeof(float), "alternating window");
      if (s == NNA_OK && mel && p->kind == NNA_KIND_MEL) {
        s = upload(&p->d_melwf, mel->fragf.data(), mel->fragf.size() * sizeof(float), "mel weights (folded kernel)");
        if (s == NNA_OK) s = upload(&p->d_mel_maskf, mel->maskf.data(), mel->maskf.size(), "mel mask (folded kernel)");
      }
    }
    if (s == NNA_OK && mel) {
      s = upload(&p->d_melw, mel->frag.data(), mel->frag.size() * sizeof(float), "mel weights");
      if (s == NNA_OK) s = upload(&p->d_mel_mask, mel->mask.data(), mel->mask.size(), "mel mask");
      if (s == NNA_OK) s = upload(&p->d_mel_wnyq, mel->wnyq.data(), mel->wnyq.size() * sizeof(float), "mel nyquist weights");
      if (s == NNA_OK) s = upload(&p->d_mel_pass_rt, mel->pass_rt.data(), mel->pass_rt.size() * sizeof(int), "mel pass table");
    }
    if (s == NNA_OK && !p->h_fir_he.empty()) {
      s = upload(&p->d_fir_he, p->h_fir_he.data(), p->h_fir_he.size() * sizeof(float), "decimation taps");
      if (s == NNA_OK) s = upload(&p->d_fir_ho, p->h_fir_ho.data(), p->h_fir_ho.size() * sizeof(float), "decimation taps");
    }
    if (s == NNA_OK && p->kind == NNA_KIND_CQT) {
      s = upload(&p->d_items, p->h_items.data(), p->h_items.size() * sizeof(nna::CqtItem), "cqt item table");
      if (s == NNA_OK) s = upload(&p->d_chunks, p->h_chunks.data(), p->h_chunks.size() * sizeof(nna::CqtChunk), "cqt chunk table");
    }
    if (s != NNA_OK) {
      const std::string keep = g_err;
      nna_plan_destroy(p);
      g_err = keep;
      return s;
    }
    std::vector<float>().swap(p->h_bank);  // the device copy is the bank from here on
    std::vector<float>().swap(p->h_bankf);
    std::vector<_Float16>().swap(p->h_bank16);
    std::vector<_Float16>().swap(p->h_bank16s);
  }
  *out = p;
  return NNA_OK;
}

nna_status check_common(nna_plan** plan, int sr, int hop, int win, int center, int device) {
  if (!plan) return fail(NNA_ERR_INVALID_ARG, "plan output pointer is NULL");
  *plan = nullptr;
  if (sr < 1) return fail(NNA_ERR_INVALID_ARG, "sr must be >= 1");
  if (hop < 1) return fail(NNA_ERR_INVALID_ARG, "hop must be >= 1");
  if (win < NNA_WIN_HANN || win > NNA_WIN_BLACKMAN) return fail(NNA_ERR_INVALID_ARG, "unknown window");
  if (center != 0 && center != 1) return fail(NNA_ERR_INVALID_ARG, "center must be 0 or 1");
  return check_device(device);
}

// magnitude / power / log everywhere; the complex and phase outputs where `allow_complex`
nna_status check_fmt(int fmt, bool allow_complex) {
  if (fmt == NNA_OUT_MAGNITUDE || fmt == NNA_OUT_POWER || fmt == NNA_OUT_LOG) return NNA_OK;
  if (fmt == NNA_OUT_COMPLEX || fmt == NNA_OUT_PHASE) {
    if (allow_complex) return NNA_OK;
    return fail(NNA_ERR_UNSUPPORTED, "the complex and phase outputs exist for nna_stft (float32) and nna_cqt only");
  }
  return fail(NNA_ERR_INVALID_ARG, "unknown output format");
}

nna_status check_stft_args(int n_fft) {
  if (n_fft < 8 || (n_fft & 1)) return fail(NNA_ERR_INVALID_ARG, "n_fft must be even and >= 8");
  if (n_fft > (1 << 20)) return fail(NNA_ERR_UNSUPPORTED, "n_fft above 2^20 is not supported");
  return NNA_OK;
}

// frames per waveform, or 0 if the signal is too short
long long frames_of(const nna_plan* p, long long L) {
  if (p->center) {
    if (L <= p->pad) return 0;  // mirror reflection needs pad <= L-1
  } else if (L < p->K) {
    return 0;
  }
  return 1 + (L + 2LL * p->pad - p->K) / p->hop;
}

// Largest frame tile (<= cap) whose LDS rows  M + segments(M,T)*extra  fit in `rows_max`.
int pick_tile_frames(int cap, long long T, int extra, int rows_max) {
  for (int M = cap; M >= 1; --M) {
    const long long nseg = 1 + (M - 1 + T - 1) / T;
    if ((long long)M + nseg * extra <= rows_max) return M;
  }
  return 0;
}

nna_status check_call(const nna_plan* plan, int kind, const float* x, long long B, long long L, float* out,
                      long long* T_out) {
  if (!plan) return fail(NNA_ERR_INVALID_ARG, "plan is NULL");
  if (plan->kind != kind) return fail(NNA_ERR_INVALID_ARG, "plan was built for a different transform");
  if (!x || !out) return fail(NNA_ERR_INVALID_ARG, "x_dev / out_dev is NULL");
  if (plan->device < 0) return fail(NNA_ERR_UNSUPPORTED, "host-only plan (device = -1) cannot run transforms");
  if (B < 1) return fail(NNA_ERR_SHAPE, "B must be >= 1");
  // the framing loader fetches windows of four consecutive stored samples
  if (L < 4) return fail(NNA_ERR_SHAPE, "L must be at least 4 samples");
  const long long T = frames_of(plan, L);
  if (T < 1) return fail(NNA_ERR_SHAPE, plan->center ? "L must exceed the reflection padding (K/2)" : "L is shorter than one window");
  // the kernels index samples of one waveform with 32-bit integers (padded index < L + 2K)
  if (T > 0x7fffffffLL / 4 || L > 0x7fffffffLL - 4LL * plan->K - 64 || B > 0x7fffffffLL || B > (1LL << 40) / T)
    return fail(NNA_ERR_SHAPE, "batch too large");
  *T_out = T;
  return NNA_OK;
}

nna::FrameGeom make_geom(const nna_plan* p, const float* x, long long B, long long L, long long T) {
  nna::FrameGeom g;
  g.x = x;
  g.B = B;
  g.L = L;
  g.T = (int)T;
  g.n_frames = B * T;
  g.hop = p->hop;
  g.pad = p->pad;
  g.vec_ok = (L % 4 == 0) && (p->hop % 4 == 0) && (p->pad % 4 == 0) && ((reinterpret_cast<uintptr_t>(x) & 15) == 0);
  return g;
}

// One launch of the STFT kernel family: T frames of each of the B waveforms (arguments checked by the
// caller).  out_wave_stride / bin_offset place a two-stage CQT plan's bins inside a larger output
// (octave of a downsampling plan); 0 / 0 = the plan's own [B, bins, T].
nna_status run_stft_core(const nna_plan* plan, int kind, const float* x, long long B, long long L, long long T,
                         float* out, long long out_wave_stride, int bin_offset, void* stream, float* spec_out = nullptr) {
  if (plan->precision == NNA_PREC_F16) {
    const int M = pick_tile_frames(nna::H_FRAMES, T, plan->nj - 1, nna::H_LB_ROWS);
    if (M < 1) return fail(NNA_ERR_UNSUPPORTED, "frame tile does not fit in LDS");
    nna::Stft16Params P;
    std::memset(&P, 0, sizeof(P));
    P.g = make_geom(plan, x, B, L, T);
    P.bank = plan->d_bank16;
    P.bank_s = plan->d_bank16s;
    P.out = out;
    P.n_rt = plan->n_rt16;
    P.n_chunks = plan->hop / nna::H_KC;
    P.nj = plan->nj;
    P.n_half = plan->n_half;
    P.packed = plan->freq_scale ? 0 : 1;
    P.out_bins = plan->stft_bins();
    P.fmt = plan->fmt;
    P.rt_per_block = plan->n_rt16;
    P.tile_frames = M;
    P.n_ft = (P.g.n_frames + M - 1) / M;
    DeviceGuard guard;
    hipError_t e = guard.enter(plan->device);
    if (e != hipSuccess) return fail_hip(e, "hipSetDevice");
    e = nna::launch_stft16(P, reinterpret_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail_hip(e, "kernel launch");
    return NNA_OK;
  }
  // The folded kernel addresses the rows of a frame tile as 32-bit byte offsets from the tile's first waveform:
  // the waveforms a tile can span must lie within 2^31 bytes (else the direct kernel runs).
  const int fold_M = plan->runs_folded() ? pick_tile_frames(ST_FRAMES, T, plan->nj / 2 - 1, nna::SF_LDS_ROWS) : 0;
  const bool fold_fits = fold_M >= 1 && (1 + (fold_M - 1 + T - 1) / T) * L <= (1LL << 29);
  if (fold_fits && !spec_out && (kind == NNA_KIND_STFT || kind == NNA_KIND_MEL)) {
    const int nj2 = plan->nj / 2;
    const int M = fold_M;
    nna::StftParams P;
    std::memset(&P, 0, sizeof(P));
    P.g = make_geom(plan, x, B, L, T);
    P.bankf = reinterpret_cast<const float4*>(plan->d_bankf);
    P.wn = plan->d_wn;
    P.wmid = plan->wmid;
    P.out = out;
    P.n_rt = plan->n_rt;
    P.n_chunks = plan->n_chunks;
    P.nj = nj2;
    P.n_half = plan->n_half;
    P.packed = 0;
    P.tile_frames = M;
    P.n_ft = (P.g.n_frames + M - 1) / M;
    if (kind == NNA_KIND_MEL) {
      P.out_bins = plan->n_mels;
      P.fmt = plan->mel_power;
      P.melw = reinterpret_cast<const float4*>(plan->d_melwf);
      P.mel_mask = plan->d_mel_maskf;
      P.mel_pass_rt = plan->d_mel_pass_rt;
      P.n_mels = plan->n_mels;
      P.n_pass = plan->n_pass;
    } else {
      P.out_bins = plan->n_half + 1;
      P.fmt = plan->fmt;
      const long long ft_per_xcd = (P.n_ft + 7) / 8;
      P.main_blocks = 8 * ((ft_per_xcd + 63) / 64) * 64 * ((plan->n_rt + nna::ST_RG - 1) / nna::ST_RG);
    }
    DeviceGuard guard;
    hipError_t e = guard.enter(plan->device);
    if (e != hipSuccess) return fail_hip(e, "hipSetDevice");
    e = nna::launch_stft_fold(P, kind == NNA_KIND_MEL ? nna::ST_MODE_MEL : nna::ST_MODE_STFT, reinterpret_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail_hip(e, "kernel launch");
    return NNA_OK;
  }
  const int lds_rows = kind == NNA_KIND_CQT1992 && plan->lin_blocks == 6 ? nna::ST_LDS_ROWS_WIDE : ST_LDS_ROWS;
  const int M = pick_tile_frames(ST_FRAMES, T, plan->nj - 1, lds_rows);
  if (M < 1) return fail(NNA_ERR_UNSUPPORTED, "frame tile does not fit in LDS");
  nna::StftParams P;
  std::memset(&P, 0, sizeof(P));
  P.g = make_geom(plan, x, B, L, T);
  P.bank = reinterpret_cast<const float4*>(plan->d_bank);
  P.out = out;
  P.n_rt = plan->n_rt;
  P.n_chunks = plan->n_chunks;
  P.nj = plan->nj;
  P.n_half = plan->n_half;
  P.packed = plan->freq_scale ? 0 : 1;
  P.out_bins = kind == NNA_KIND_MEL ? plan->n_mels : kind == NNA_KIND_CQT1992 ? plan->n_bins : plan->out_rows();
  P.tile_frames = M;
  P.n_ft = (P.g.n_frames + M - 1) / M;
  if (kind == NNA_KIND_MEL) {
    P.fmt = plan->mel_power;
    P.melw = reinterpret_cast<const float4*>(plan->d_melw);
    P.mel_mask = plan->d_mel_mask;
    P.mel_wnyq = plan->d_mel_wnyq;
    P.mel_pass_rt = plan->d_mel_pass_rt;
    P.n_mels = plan->n_mels;
    P.n_pass = plan->n_pass;
    P.mel_nyq_any = plan->mel_nyq_any;
  } else if (kind == NNA_KIND_CQT1992) {
    P.fmt = plan->fmt;
    P.out_wave_stride = out_wave_stride > 0 ? out_wave_stride : (long long)plan->n_bins * T;
    P.bin_offset = bin_offset;
    P.melw = reinterpret_cast<const float4*>(plan->d_melw);
    P.mel_mask = plan->d_mel_mask;
    P.mel_wnyq = plan->d_mel_wnyq;
    P.mel_pass_rt = plan->d_mel_pass_rt;
    P.n_mels = 2 * plan->n_bins;
    P.n_pass = plan->n_pass;
    P.lin_blocks = plan->lin_blocks;
  } else {
    P.fmt = plan->fmt;
  }
  DeviceGuard guard;
  hipError_t e = guard.enter(plan->device);
  if (e != hipSuccess) return fail_hip(e, "hipSetDevice");
  P.pout = spec_out;
  const int mode = kind == NNA_KIND_MEL       ? (spec_out ? nna::ST_MODE_MELSPEC : nna::ST_MODE_MEL)
                   : kind == NNA_KIND_CQT1992 ? nna::ST_MODE_LIN
                   : (plan->fmt == NNA_OUT_COMPLEX || plan->fmt == NNA_OUT_PHASE) ? nna::ST_MODE_CPLX
                                                                                  : nna::ST_MODE_STFT;
  e = nna::launch_stft(P, mode, reinterpret_cast<hipStream_t>(stream));
  if (e != hipSuccess) return fail_hip(e, "kernel launch");
  return NNA_OK;
}

nna_status run_stft_like(const nna_plan* plan, int kind, const float* x, long long B, long long L, float* out,
                         void* stream) {
  long long T = 0;
  nna_status s = check_call(plan, kind, x, B, L, out, &T);
  if (s != NNA_OK) return s;
  return run_stft_core(plan, kind, x, B, L, T, out, 0, 0, stream);
}

nna_status check_cqt_args(double fmin, int n_bins, int bins_per_octave, int n_taps, int fmt, int sr,
                          bool allow_complex = false) {
  if (!(fmin > 0.0)) return fail(NNA_ERR_INVALID_ARG, "fmin must be > 0");
  if (n_bins < 1 || n_bins > 4096) return fail(NNA_ERR_INVALID_ARG, "n_bins must be in [1, 4096]");
  if (bins_per_octave < 1 || bins_per_octave > 1024) return fail(NNA_ERR_INVALID_ARG, "bins_per_octave must be in [1, 1024]");
  if (nna_status sf = check_fmt(fmt, allow_complex); sf != NNA_OK) return sf;
  if (n_taps < 0) return fail(NNA_ERR_INVALID_ARG, "n_taps must be >= 0");
  const double top = fmin * std::pow(2.0, (double)(n_bins - 1) / bins_per_octave);
  if (!(top < 0.5 * sr)) return fail(NNA_ERR_INVALID_ARG, "the top CQT bin must lie below sr/2");
  return NNA_OK;
}

// CQT plan whose bin k sits at fmin 2^((k_first + k) / bins_per_octave); arguments already checked
nna_status make_cqt_plan(nna_plan** plan, int sr, int hop, double fmin, int k_first, int n_bins, int bins_per_octave,
                         int win, int center, int n_taps, int fmt, int device) {
  nna_plan* p = new (std::nothrow) nna_plan;
  if (!p) return fail(NNA_ERR_ALLOC, "out of host memory");
  try {
    p->kind = NNA_KIND_CQT;
    p->device = device;
    p->sr = sr;
    p->hop = hop;
    p->center = center;
    p->window = win;
    p->fmt = fmt;
    p->n_bins = n_bins;
    p->bpo = bins_per_octave;
    p->k_first = k_first;
    p->cq_fmin = fmin;
    p->Q = 1.0 / (std::exp2(1.0 / bins_per_octave) - 1.0);  // eq. (Q)
    p->Nk.resize(n_bins);
    p->sk.resize(n_bins);
    for (int k = 0; k < n_bins; ++k) {
      const double fk = fmin * std::exp2((double)(k_first + k) / bins_per_octave);
      p->Nk[k] = (long long)std::ceil(p->Q * (double)sr / fk);  // eq. (N_k), in double
    }
    if (p->Nk[0] > (1LL << 24)) {
      delete p;
      return fail(NNA_ERR_UNSUPPORTED, "CQT kernels longer than 2^24 taps are not supported");
    }
    long long taps = n_taps;
    if (taps == 0) {
      taps = 1;
      while (taps < p->Nk[0]) taps <<= 1;
      if (taps < 2) taps = 2;
    }
    if (taps & 1) {
      delete p;
      return fail(NNA_ERR_INVALID_ARG, "n_taps must be even");
    }
    if (taps < p->Nk[0]) {
      char msg[160];
      std::snprintf(msg, sizeof msg, "n_taps = %lld is shorter than the longest kernel (%lld taps)", taps, p->Nk[0]);
      delete p;
      return fail(NNA_ERR_INVALID_ARG, msg);
    }
    p->K = (int)taps;
    p->pad = center ? (int)(taps / 2) : 0;
    for (int k = 0; k < n_bins; ++k) p->sk[k] = (taps - p->Nk[k]) / 2;
    build_cqt_bank(p);
  } catch (const std::bad_alloc&) {
    delete p;
    return fail(NNA_ERR_ALLOC, "out of host memory while building the CQT bank");
  }
  return finish_plan(p, plan, nullptr);
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

// The filter + keep-every-second-sample step as a bank for the CQT kernel: a "frame" is FIR_ROWS
// consecutive output samples y[FIR_ROWS t + r]; it reads input samples 2 FIR_ROWS t - half + [0, K)
// and row r holds the filter shifted by 2 r taps (y[m] is centred on x[2 m]).  Four row blocks =
// one work item, so a workgroup produces 64 samples per frame from one set of LDS tiles.
constexpr int FIR_ROWS = CQ_ITEM_RB * CQ_ROWS;
constexpr int FIR_HOP = 2 * FIR_ROWS;
nna_status make_fir_plan(nna_plan** plan, int fir_taps, int device) {
  nna_plan* p = new (std::nothrow) nna_plan;
  if (!p) return fail(NNA_ERR_ALLOC, "out of host memory");
  try {
    p->kind = NNA_KIND_CQT;
    p->device = device;
    p->sr = 1;
    p->hop = FIR_HOP;
    p->center = 1;
    p->window = NNA_WIN_RECT;
    p->fmt = NNA_OUT_MAGNITUDE;
    p->fir_taps = fir_taps;
    p->K = (fir_taps + 2 * (FIR_ROWS - 1) + FIR_HOP - 1) / FIR_HOP * FIR_HOP;
    p->pad = (fir_taps - 1) / 2;
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
  } catch (const std::bad_alloc&) {
    delete p;
    return fail(NNA_ERR_ALLOC, "out of host memory while building the filter bank");
  }
  return finish_plan(p, plan, nullptr);
}

// one launch of the CQT kernel: `sub`'s bank over T frames of each of the B waveforms in x
nna_status run_conv(const nna_plan* sub, const float* x, long long B, long long L, long long T, float* out,
                    long long out_wave_stride, int bin_offset, void* hip_stream) {
  const int extra = (sub->max_jspan - 1) * sub->row_step;
  const int M = pick_tile_frames(CQ_FRAMES, T, extra, CQ_LDS_ROWS_MAX);
  if (M < 1) return fail(NNA_ERR_UNSUPPORTED, "frame tile does not fit in LDS");
  nna::CqtParams P;
  std::memset(&P, 0, sizeof(P));
  P.g = make_geom(sub, x, B, L, T);
  P.tap_stride = sub->tap_stride;
  P.row_step = sub->row_step;
  P.bank = reinterpret_cast<const float4*>(sub->d_bank);
  P.items = sub->d_items;
  P.chunks = sub->d_chunks;
  P.out = out;
  P.out_wave_stride = out_wave_stride;
  P.bin_offset = bin_offset;
  P.n_items = (int)sub->h_items.size();
  P.n_chunks = sub->n_chunks;
  P.n_bins = sub->n_bins;
  P.fmt = sub->fmt;
  P.tile_frames = M;
  const long long nseg = 1 + (M - 1 + T - 1) / T;
  P.lds_rows = (int)((M + nseg * extra + 63) / 64 * 64);  // whole loader passes of 64 rows (<= CQ_LDS_ROWS_MAX)
  P.n_ft = (P.g.n_frames + M - 1) / M;
  hipError_t e = nna::launch_cqt(P, reinterpret_cast<hipStream_t>(hip_stream));
  if (e != hipSuccess) return fail_hip(e, "kernel launch");
  return NNA_OK;
}

// one decimation step: y[B, Ln] from x[B, L], Ln = ceil(L / 2) (arguments checked by the caller)
nna_status run_fir(const nna_plan* fir, const float* x, long long B, long long L, float* y, long long Ln, void* hip_stream) {
  nna::FirParams P;
  std::memset(&P, 0, sizeof(P));
  P.L = L;
  P.Ln = Ln;
  P.he = fir->d_fir_he;
  P.ho = fir->d_fir_ho;
  P.ne = (int)fir->h_fir_he.size();
  P.no = (int)fir->h_fir_ho.size();
  P.ve0 = fir->fir_ve0;
  P.vo0 = fir->fir_vo0;
  const int vmin = std::min(P.ve0, P.vo0), vend = std::max(P.ve0 + P.ne, P.vo0 + P.no);
  P.lds_stream = (nna::FIR_TILE + (vend - vmin) + 16) * 9 / 8 + 8;  // one float of padding per eight samples
  // the grid's second dimension holds at most 65,535 waveforms
  for (long long b0 = 0; b0 < B; b0 += 65535) {
    P.B = std::min(B - b0, 65535LL);
    P.x = x + b0 * L;
    P.y = y + b0 * Ln;
    P.vec2 = ((reinterpret_cast<uintptr_t>(P.x) & 7) == 0 && (L % 2 == 0 || P.B == 1)) ? 1 : 0;
    P.vec4_out = ((reinterpret_cast<uintptr_t>(P.y) & 15) == 0 && (Ln % 4 == 0 || P.B == 1)) ? 1 : 0;
    const hipError_t e = nna::launch_fir_decimate(P, reinterpret_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return fail_hip(e, "kernel launch");
  }
  return NNA_OK;
}

// octaves of a downsampling plan and the bins [lo, hi) of octave a (0 = top)
inline int octaves_of(int n_bins, int bpo) { return (n_bins + bpo - 1) / bpo; }
inline void octave_bins(int n_bins, int bpo, int a, int& lo, int& hi) {
  hi = n_bins - a * bpo;
  lo = std::max(0, hi - bpo);
}
inline size_t ws_round(long long floats) { return ((size_t)floats * sizeof(float) + 255) / 256 * 256; }

// lengths of the waveform at every octave; false if some octave is too short for its padding
constexpr int MAX_OCTAVES = 16;
bool cqt2010_lengths(const nna_plan* plan, long long L, long long (&La)[MAX_OCTAVES]) {
  const int n_oct = (int)plan->octave.size();
  long long l = L;
  for (int a = 0; a < n_oct; ++a) {
    La[a] = l;
    if (l < 4 || l <= plan->pad) return false;             // mirror reflection of the CQT kernels
    if (a + 1 < n_oct && l < plan->fir->K) return false;   // and of the filter's frames
    l = (l + 1) / 2;
  }
  return true;
}

}  // namespace

// =======================================================================================
// C ABI
// =======================================================================================
extern "C" {

nna_status nna_plan_stft(nna_plan** plan, int sr, int n_fft, int hop, nna_window win, int center, nna_output fmt,
                         int device) {
  nna_status s = check_common(plan, sr, hop, win, center, device);
  if (s != NNA_OK) return s;
  if ((s = check_stft_args(n_fft)) != NNA_OK) return s;
  if ((s = check_fmt(fmt, true)) != NNA_OK) return s;
  nna_plan* p = new (std::nothrow) nna_plan;
  if (!p) return fail(NNA_ERR_ALLOC, "out of host memory");
  try {
    p->kind = NNA_KIND_STFT;
    p->device = device;
    p->sr = sr;
    p->hop = hop;
    p->center = center;
    p->window = win;
    p->fmt = fmt;
    p->K = n_fft;
    p->pad = center ? n_fft / 2 : 0;
    build_stft_bank(p);
    if (fmt == NNA_OUT_MAGNITUDE || fmt == NNA_OUT_POWER || fmt == NNA_OUT_LOG) build_stft_bank_fold(p);
  } catch (const std::bad_alloc&) {
    delete p;
    return fail(NNA_ERR_ALLOC, "out of host memory while building the DFT bank");
  }
  return finish_plan(p, plan, nullptr);
}

nna_status nna_plan_stft_prec(nna_plan** plan, int sr, int n_fft, int hop, nna_window win, int center, nna_output fmt,
                              nna_precision precision, int device) {
  if (precision == NNA_PREC_F32) return nna_plan_stft(plan, sr, n_fft, hop, win, center, fmt, device);
  if (precision != NNA_PREC_F16) {
    if (plan) *plan = nullptr;
    return fail(NNA_ERR_INVALID_ARG, "unknown precision");
  }
  nna_status s = check_common(plan, sr, hop, win, center, device);
  if (s != NNA_OK) return s;
  if ((s = check_stft_args(n_fft)) != NNA_OK) return s;
  if ((s = check_fmt(fmt, false)) != NNA_OK) return s;
  nna_plan* p = new (std::nothrow) nna_plan;
  if (!p) return fail(NNA_ERR_ALLOC, "out of host memory");
  try {
    p->kind = NNA_KIND_STFT;
    p->device = device;
    p->sr = sr;
    p->hop = hop;
    p->center = center;
    p->window = win;
    p->fmt = fmt;
    p->K = n_fft;
    p->pad = center ? n_fft / 2 : 0;
    p->precision = NNA_PREC_F16;
    build_stft_bank(p);
    if (!build_stft_bank_f16(p)) {
      delete p;
      return fail(NNA_ERR_UNSUPPORTED,
                  "the float16 kernel needs hop to divide n_fft (at most 32 times) and to be a multiple of 32");
    }
    p->exec_flops = 2.0 * (double)n_fft * (double)p->n_rt16 * nna::H_ROWS;
  } catch (const std::bad_alloc&) {
    delete p;
    return fail(NNA_ERR_ALLOC, "out of host memory while building the DFT bank");
  }
  return finish_plan(p, plan, nullptr);
}

nna_status nna_plan_stft_scaled(nna_plan** plan, int sr, int n_fft, int hop, nna_window win, int center,
                                nna_output fmt, nna_freq_scale freq_scale, double fmin, double fmax, int freq_bins,
                                int device) {
  nna_status s = check_common(plan, sr, hop, win, center, device);
  if (s != NNA_OK) return s;
  if ((s = check_stft_args(n_fft)) != NNA_OK) return s;
  if ((s = check_fmt(fmt, true)) != NNA_OK) return s;
  if (freq_scale != NNA_FREQ_LINEAR && freq_scale != NNA_FREQ_LOG)
    return fail(NNA_ERR_INVALID_ARG, "freq_scale must be NNA_FREQ_LINEAR or NNA_FREQ_LOG");
  if (freq_bins == 0) freq_bins = n_fft / 2 + 1;
  if (freq_bins < 1 || freq_bins > 16384) return fail(NNA_ERR_INVALID_ARG, "freq_bins must be in [1, 16384]");
  if (!(fmin >= 0.0) || !(fmax > fmin) || fmax > 0.5 * sr)
    return fail(NNA_ERR_INVALID_ARG, "need 0 <= fmin < fmax <= sr/2");
  if (freq_scale == NNA_FREQ_LOG && !(fmin > 0.0))
    return fail(NNA_ERR_INVALID_ARG, "a log frequency axis needs fmin > 0");
  nna_plan* p = new (std::nothrow) nna_plan;
  if (!p) return fail(NNA_ERR_ALLOC, "out of host memory");
  try {
    p->kind = NNA_KIND_STFT;
    p->device = device;
    p->sr = sr;
    p->hop = hop;
    p->center = center;
    p->window = win;
    p->fmt = fmt;
    p->K = n_fft;
    p->pad = center ? n_fft / 2 : 0;
    p->freq_scale = freq_scale;
    p->freq_bins = freq_bins;
    p->sigma.resize(freq_bins);
    const double N = n_fft, mu = freq_bins;
    for (int k = 0; k < freq_bins; ++k)
      p->sigma[k] = freq_scale == NNA_FREQ_LINEAR ? (fmax - fmin) * N / (mu * sr) * k + fmin * N / sr
                                                  : fmin * N / sr * std::pow(fmax / fmin, k / mu);
    build_stft_bank(p);
  } catch (const std::bad_alloc&) {
    delete p;
    return fail(NNA_ERR_ALLOC, "out of host memory while building the DFT bank");
  }
  return finish_plan(p, plan, nullptr);
}

nna_status nna_plan_mel(nna_plan** plan, int sr, int n_fft, int hop, nna_window win, int center, int n_mels,
                        double fmin, double fmax, nna_mel_scale scale, int norm_area, double power, int device) {
  nna_status s = check_common(plan, sr, hop, win, center, device);
  if (s != NNA_OK) return s;
  if ((s = check_stft_args(n_fft)) != NNA_OK) return s;
  if (n_mels < 1 || n_mels > 4096) return fail(NNA_ERR_INVALID_ARG, "n_mels must be in [1, 4096]");
  if (scale != NNA_MEL_SLANEY && scale != NNA_MEL_HTK) return fail(NNA_ERR_INVALID_ARG, "unknown mel scale");
  if (!(power == 1.0 || power == 2.0)) return fail(NNA_ERR_INVALID_ARG, "power must be 1 or 2");
  if (!(fmax > 0.0)) fmax = 0.5 * sr;
  if (!(fmin >= 0.0) || !(fmax > fmin) || fmax > 0.5 * sr)
    return fail(NNA_ERR_INVALID_ARG, "need 0 <= fmin < fmax <= sr/2");
  nna_plan* p = new (std::nothrow) nna_plan;
  if (!p) return fail(NNA_ERR_ALLOC, "out of host memory");
  MelDeviceLayout mel;
  try {
    p->kind = NNA_KIND_MEL;
    p->device = device;
    p->sr = sr;
    p->hop = hop;
    p->center = center;
    p->window = win;
    p->K = n_fft;
    p->pad = center ? n_fft / 2 : 0;
    p->n_mels = n_mels;
    p->mel_power = power == 1.0 ? 1 : 2;
    build_stft_bank(p);
    build_stft_bank_fold(p);
    build_mel_weights(p, fmin, fmax, scale, norm_area);
    mel = layout_mel(p);
  } catch (const std::bad_alloc&) {
    delete p;
    return fail(NNA_ERR_ALLOC, "out of host memory while building the Mel plan");
  }
  return finish_plan(p, plan, &mel);
}

nna_status nna_plan_cqt(nna_plan** plan, int sr, int hop, double fmin, int n_bins, int bins_per_octave,
                        nna_window win, int center, int n_taps, nna_output fmt, int device) {
  nna_status s = check_common(plan, sr, hop, win, center, device);
  if (s != NNA_OK) return s;
  if ((s = check_cqt_args(fmin, n_bins, bins_per_octave, n_taps, fmt, sr, true)) != NNA_OK) return s;
  return make_cqt_plan(plan, sr, hop, fmin, 0, n_bins, bins_per_octave, win, center, n_taps, fmt, device);
}

// two-stage CQT plan whose bin k sits at fmin 2^((k_first + k) / bins_per_octave); arguments already checked
static nna_status make_cqt1992_plan(nna_plan** plan, int sr, int hop, double fmin, int k_first, int n_bins,
                                    int bins_per_octave, int win, int center, int n_fft, int fmt, int device) {
  nna_plan* p = new (std::nothrow) nna_plan;
  if (!p) return fail(NNA_ERR_ALLOC, "out of host memory");
  MelDeviceLayout lin;
  try {
    p->kind = NNA_KIND_CQT1992;
    p->device = device;
    p->sr = sr;
    p->hop = hop;
    p->center = center;
    p->window = NNA_WIN_RECT;  // the STFT stage is un-windowed: the window lives in the CQT kernels
    p->cq_window = win;
    p->fmt = fmt;
    p->n_bins = n_bins;
    p->bpo = bins_per_octave;
    p->cq_fmin = fmin;
    p->k_first = k_first;
    p->Q = 1.0 / (std::exp2(1.0 / bins_per_octave) - 1.0);  // eq. (Q)
    p->Nk.resize(n_bins);
    p->sk.resize(n_bins);
    for (int k = 0; k < n_bins; ++k)
      p->Nk[k] = (long long)std::ceil(p->Q * (double)sr / (fmin * std::exp2((double)(k_first + k) / bins_per_octave)));  // eq. (N_k)
    long long N = n_fft;
    if (N == 0) {
      N = 8;
      while (N < p->Nk[0] && N < (1LL << 30)) N <<= 1;
    }
    if (N < 8 || (N & (N - 1))) {
      delete p;
      return fail(NNA_ERR_INVALID_ARG, "n_fft must be a power of two >= 8 (0 picks the smallest that holds the longest kernel)");
    }
    if (N < p->Nk[0]) {
      char msg[160];
      std::snprintf(msg, sizeof msg, "n_fft = %lld is shorter than the longest kernel (%lld taps)", N, p->Nk[0]);
      delete p;
      return fail(NNA_ERR_INVALID_ARG, msg);
    }
    if (N > 65536) {
      delete p;
      return fail(NNA_ERR_UNSUPPORTED, "the DFT bank of n_fft above 65,536 (17 GB at 65,536) is not supported");
    }
    p->K = (int)N;
    p->pad = center ? (int)(N / 2) : 0;
    for (int k = 0; k < n_bins; ++k) p->sk[k] = (N - p->Nk[k]) / 2;
    build_stft_bank(p);
    build_cqt1992_matrix(p);
    lin = layout_cqt1992(p);
  } catch (const std::bad_alloc&) {
    delete p;
    return fail(NNA_ERR_ALLOC, "out of host memory while building the DFT bank and the spectral kernels");
  }
  return finish_plan(p, plan, &lin);
}

nna_status nna_plan_cqt1992(nna_plan** plan, int sr, int hop, double fmin, int n_bins, int bins_per_octave,
                            nna_window win, int center, int n_fft, nna_output fmt, int device) {
  nna_status s = check_common(plan, sr, hop, win, center, device);
  if (s != NNA_OK) return s;
  if ((s = check_cqt_args(fmin, n_bins, bins_per_octave, n_fft, fmt, sr)) != NNA_OK) return s;
  return make_cqt1992_plan(plan, sr, hop, fmin, 0, n_bins, bins_per_octave, win, center, n_fft, fmt, device);
}

// Both downsampling plans: one sub-plan per octave (time-domain kernels: a plan as from nna_plan_cqt;
// frequency-domain kernels: one as from nna_plan_cqt1992) and the decimation filter.
static nna_status make_downsampling_plan(int kind, nna_plan** plan, int sr, int hop, double fmin, int n_bins,
                                         int bins_per_octave, nna_window win, int n_taps, int fir_taps, nna_output fmt,
                                         int device) {
  nna_status s = check_common(plan, sr, hop, win, 1, device);
  if (s != NNA_OK) return s;
  if ((s = check_cqt_args(fmin, n_bins, bins_per_octave, n_taps, fmt, sr)) != NNA_OK) return s;
  if (fir_taps == 0) fir_taps = 257;
  if (fir_taps < 3 || fir_taps > 4095 || !(fir_taps & 1))
    return fail(NNA_ERR_INVALID_ARG, "fir_taps must be odd and in [3, 4095]");
  const int n_oct = octaves_of(n_bins, bins_per_octave);
  if (n_oct > MAX_OCTAVES) return fail(NNA_ERR_UNSUPPORTED, "more than 16 octaves are not supported");
  if (hop % (1 << (n_oct - 1)) != 0)
    return fail(NNA_ERR_INVALID_ARG, "hop must be a multiple of 2^(octaves - 1): every octave halves it");
  int lo, hi;
  octave_bins(n_bins, bins_per_octave, 0, lo, hi);
  if (n_taps == 0) {
    // next power of two >= the longest kernel of the top octave
    const double Q = 1.0 / (std::exp2(1.0 / bins_per_octave) - 1.0);
    const long long n0 = (long long)std::ceil(Q * (double)sr / (fmin * std::exp2((double)lo / bins_per_octave)));
    long long t = 2;
    while (t < n0) t <<= 1;
    if (t > (1LL << 24)) return fail(NNA_ERR_UNSUPPORTED, "CQT kernels longer than 2^24 taps are not supported");
    n_taps = (int)t;
    if (kind == NNA_KIND_CQT2010 && n_taps < 8) n_taps = 8;
  }
  nna_plan* p = new (std::nothrow) nna_plan;
  if (!p) return fail(NNA_ERR_ALLOC, "out of host memory");
  p->kind = kind;
  p->device = device;
  p->sr = sr;
  p->hop = hop;
  p->center = 1;
  p->window = win;
  p->fmt = fmt;
  p->n_bins = n_bins;
  p->bpo = bins_per_octave;
  p->cq_fmin = fmin;
  p->K = n_taps;
  p->pad = n_taps / 2;
  p->fir_taps = fir_taps;
  // octave a: the bins [lo, hi) one factor 2^a up the frequency axis, hop / 2^a, same taps
  for (int a = 0; a < n_oct && s == NNA_OK; ++a) {
    octave_bins(n_bins, bins_per_octave, a, lo, hi);
    nna_plan* sub = nullptr;
    if (kind == NNA_KIND_CQT2010V2)
      s = make_cqt_plan(&sub, sr, hop >> a, fmin, lo + a * bins_per_octave, hi - lo, bins_per_octave, win, 1, n_taps,
                        fmt, device);
    else
      s = make_cqt1992_plan(&sub, sr, hop >> a, fmin, lo + a * bins_per_octave, hi - lo, bins_per_octave, win, 1,
                            n_taps, fmt, device);
    if (s == NNA_OK) p->octave.push_back(sub);
  }
  if (s == NNA_OK && n_oct > 1) s = make_fir_plan(&p->fir, fir_taps, device);
  if (s != NNA_OK) {
    const std::string keep = g_err;
    nna_plan_destroy(p);
    g_err = keep;
    return s;
  }
  // per frame of the output: every octave's kernels once, and hop / 2^(a+1) filter outputs for
  // each downsampling step a -> a+1 (the filter plan counts flops per frame of FIR_ROWS outputs)
  for (int a = 0; a < n_oct; ++a) {
    p->exec_flops += p->octave[a]->exec_flops;
    p->alg_flops += p->octave[a]->alg_flops;
    if (a + 1 < n_oct) {
      const double fir_frames = (double)(hop >> (a + 1)) / FIR_ROWS;
      p->exec_flops += fir_frames * p->fir->exec_flops;
      p->alg_flops += fir_frames * p->fir->alg_flops;
    }
  }
  *plan = p;
  return NNA_OK;
}

nna_status nna_plan_cqt2010v2(nna_plan** plan, int sr, int hop, double fmin, int n_bins, int bins_per_octave,
                              nna_window win, int n_taps, int fir_taps, nna_output fmt, int device) {
  return make_downsampling_plan(NNA_KIND_CQT2010V2, plan, sr, hop, fmin, n_bins, bins_per_octave, win, n_taps, fir_taps,
                                fmt, device);
}

nna_status nna_plan_cqt2010(nna_plan** plan, int sr, int hop, double fmin, int n_bins, int bins_per_octave,
                            nna_window win, int n_fft, int fir_taps, nna_output fmt, int device) {
  if (n_fft != 0 && (n_fft < 8 || (n_fft & (n_fft - 1)))) {
    if (plan) *plan = nullptr;
    return fail(NNA_ERR_INVALID_ARG, "n_fft must be a power of two >= 8 (0 picks the smallest that holds the longest top-octave kernel)");
  }
  return make_downsampling_plan(NNA_KIND_CQT2010, plan, sr, hop, fmin, n_bins, bins_per_octave, win, n_fft, fir_taps,
                                fmt, device);
}

nna_status nna_cqt1992(const nna_plan* plan, const float* x_dev, long long B, long long L, float* out_dev, void* hip_stream) {
  return run_stft_like(plan, NNA_KIND_CQT1992, x_dev, B, L, out_dev, hip_stream);
}

nna_status nna_plan_spectral_kernels(const nna_plan* plan, double* host_out, size_t cap) {
  if (!plan || !host_out) return fail(NNA_ERR_INVALID_ARG, "plan / host_out is NULL");
  if (plan->kind != NNA_KIND_CQT1992) return fail(NNA_ERR_INVALID_ARG, "not a plan from nna_plan_cqt1992");
  const size_t F = (size_t)plan->n_half + 1, R = 2 * (size_t)plan->n_bins, C = 2 * (size_t)plan->n_half;
  if (cap < R * F) return fail(NNA_ERR_INVALID_ARG, "host_out is too small");
  std::vector<float> W;  // the matrix [R, C] as the GPU holds it
  try {
    if (plan->device < 0) {
      W = plan->h_linW;
    } else {
      std::vector<float> frag(plan->lin_frag_floats);
      {
        DeviceGuard guard;
        hipError_t e = guard.enter(plan->device);
        if (e == hipSuccess) e = hipMemcpy(frag.data(), plan->d_melw, frag.size() * sizeof(float), hipMemcpyDeviceToHost);
        if (e != hipSuccess) return fail_hip(e, "spectral kernel read-back");
      }
      W.assign(R * C, 0.0f);
      const int per_pass = 32 * plan->lin_blocks;
      for (int pass = 0; pass < plan->n_pass; ++pass)
        for (int rt = 0; rt < plan->n_rt; ++rt)
          for (int rb = 0; rb < ST_RB; ++rb)
            for (int mb = 0; mb < plan->lin_blocks; ++mb)
              for (int v = 0; v < 4; ++v)
                for (int lane = 0; lane < 64; ++lane)
                  for (int e = 0; e < 4; ++e) {
                    const size_t row = (size_t)pass * per_pass + mb * 32 + (lane & 31);
                    const size_t col = (size_t)rt * ST_ROWS + rb * 32 + 8 * v + 4 * (lane >> 5) + e;
                    if (row < R && col < C) W[row * C + col] = frag[lin_frag_index(plan, pass, rt, rb, mb, v, lane, e)];
                  }
    }
  } catch (const std::bad_alloc&) {
    return fail(NNA_ERR_ALLOC, "out of host memory");
  }
  // un-pack: bins 0 and K/2 sit in packed columns 0 and 1, bin s in columns 2s (its Re weight)
  for (size_t q = 0; q < (size_t)plan->n_bins; ++q)
    for (size_t s2 = 0; s2 < F; ++s2) {
      const size_t col = s2 == 0 ? 0 : s2 == F - 1 ? 1 : 2 * s2;
      host_out[(2 * q) * F + s2] = (double)W[(2 * q) * C + col];
      host_out[(2 * q + 1) * F + s2] = (double)W[(2 * q + 1) * C + col];
    }
  return NNA_OK;
}

nna_status nna_cqt2010v2_workspace(const nna_plan* plan, long long B, long long L, size_t* bytes) {
  if (!plan || !bytes) return fail(NNA_ERR_INVALID_ARG, "plan / bytes is NULL");
  if (plan->kind != NNA_KIND_CQT2010V2 && plan->kind != NNA_KIND_CQT2010)
    return fail(NNA_ERR_INVALID_ARG, "plan was built for a different transform");
  if (B < 1 || L < 1) return fail(NNA_ERR_SHAPE, "B and L must be >= 1");
  const int n_oct = (int)plan->octave.size();
  const long long L1 = (L + 1) / 2, L2 = (L1 + 1) / 2;
  *bytes = (n_oct > 1 ? ws_round(B * L1) : 0) + (n_oct > 2 ? ws_round(B * L2) : 0);
  return NNA_OK;
}

// the octave loop of both downsampling plans (time-domain or frequency-domain kernels per octave)
static nna_status run_octaves(const nna_plan* plan, int kind, const float* x_dev, long long B, long long L,
                              float* out_dev, void* workspace_dev, size_t workspace_bytes, void* hip_stream) {
  if (!plan) return fail(NNA_ERR_INVALID_ARG, "plan is NULL");
  if (plan->kind != kind) return fail(NNA_ERR_INVALID_ARG, "plan was built for a different transform");
  if (!x_dev || !out_dev) return fail(NNA_ERR_INVALID_ARG, "x_dev / out_dev is NULL");
  if (plan->device < 0) return fail(NNA_ERR_UNSUPPORTED, "host-only plan (device = -1) cannot run transforms");
  if (B < 1) return fail(NNA_ERR_SHAPE, "B must be >= 1");
  long long La[MAX_OCTAVES];
  if (L < 1 || !cqt2010_lengths(plan, L, La))
    return fail(NNA_ERR_SHAPE, "L is too short: every octave's waveform must exceed the reflection padding, and all but the lowest hold one frame of the decimation filter");
  const long long T = 1 + L / plan->hop;
  if (T > 0x7fffffffLL / 4 || L > 0x7fffffffLL - 4LL * plan->K - 64 || B > 0x7fffffffLL || B > (1LL << 40) / T)
    return fail(NNA_ERR_SHAPE, "batch too large");
  size_t need = 0;
  nna_status s = nna_cqt2010v2_workspace(plan, B, L, &need);
  if (s != NNA_OK) return s;
  if (need > 0 && (!workspace_dev || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace_dev) & 15)))
    return fail(NNA_ERR_INVALID_ARG, "workspace_dev is NULL, misaligned or smaller than nna_cqt2010v2_workspace asks for");
  const int n_oct = (int)plan->octave.size();
  // every launch of the call must fit before the first one is enqueued
  for (int a = 0; a < n_oct; ++a) {
    const nna_plan* sub = plan->octave[a];
    const int lds_rows = sub->kind == NNA_KIND_CQT1992 && sub->lin_blocks == 6 ? nna::ST_LDS_ROWS_WIDE : ST_LDS_ROWS;
    const int M = kind == NNA_KIND_CQT2010V2 ? pick_tile_frames(CQ_FRAMES, T, (sub->max_jspan - 1) * sub->row_step, CQ_LDS_ROWS_MAX)
                                             : pick_tile_frames(ST_FRAMES, T, sub->nj - 1, lds_rows);
    if (M < 1) return fail(NNA_ERR_UNSUPPORTED, "frame tile does not fit in LDS");
  }
  float* buf[2] = {static_cast<float*>(workspace_dev), nullptr};
  if (n_oct > 2) buf[1] = reinterpret_cast<float*>(static_cast<char*>(workspace_dev) + ws_round(B * ((L + 1) / 2)));
  DeviceGuard guard;
  hipError_t e = guard.enter(plan->device);
  if (e != hipSuccess) return fail_hip(e, "hipSetDevice");
  const float* cur = x_dev;
  for (int a = 0; a < n_oct; ++a) {
    int lo, hi;
    octave_bins(plan->n_bins, plan->bpo, a, lo, hi);
    if (kind == NNA_KIND_CQT2010V2)
      s = run_conv(plan->octave[a], cur, B, La[a], T, out_dev, (long long)plan->n_bins * T, lo, hip_stream);
    else
      s = run_stft_core(plan->octave[a], NNA_KIND_CQT1992, cur, B, La[a], T, out_dev, (long long)plan->n_bins * T, lo,
                        hip_stream);
    if (s != NNA_OK) return s;
    if (a + 1 < n_oct) {
      float* dst = buf[a & 1];
      const long long Ln = La[a + 1];
      if ((s = run_fir(plan->fir, cur, B, La[a], dst, Ln, hip_stream)) != NNA_OK) return s;
      cur = dst;
    }
  }
  return NNA_OK;
}

nna_status nna_cqt2010v2(const nna_plan* plan, const float* x_dev, long long B, long long L, float* out_dev,
                         void* workspace_dev, size_t workspace_bytes, void* hip_stream) {
  return run_octaves(plan, NNA_KIND_CQT2010V2, x_dev, B, L, out_dev, workspace_dev, workspace_bytes, hip_stream);
}

nna_status nna_cqt2010v2_static(const nna_plan* plan, const float* x_dev, long long B, long long L, float* out_dev,
                                void* hip_stream) {
  if (!plan) return fail(NNA_ERR_INVALID_ARG, "plan is NULL");
  if (plan->kind != NNA_KIND_CQT2010V2) return fail(NNA_ERR_INVALID_ARG, "plan was built for a different transform");
  if (plan->device < 0) return fail(NNA_ERR_UNSUPPORTED, "host-only plan (device = -1) cannot run transforms");
  if (B < 1 || L < 1) return fail(NNA_ERR_SHAPE, "B and L must be >= 1");
  // the workspace the batch needs, before any size is turned into bytes that could wrap around
  if (B > (long long)NNA_STATIC_SCRATCH_BYTES || L > (long long)NNA_STATIC_SCRATCH_BYTES)
    return fail(NNA_ERR_SHAPE, "batch too large for the library's static workspace (NNA_STATIC_SCRATCH_BYTES)");
  size_t need = 0;
  nna_status s = nna_cqt2010v2_workspace(plan, B, L, &need);
  if (s != NNA_OK) return s;
  if (need > (size_t)NNA_STATIC_SCRATCH_BYTES) {
    char msg[200];
    std::snprintf(msg, sizeof msg,
                  "this batch needs %zu bytes of workspace; the library's static workspace holds %zu "
                  "(NNA_STATIC_SCRATCH_BYTES): use nna_cqt2010v2 with a caller-owned workspace",
                  need, (size_t)NNA_STATIC_SCRATCH_BYTES);
    return fail(NNA_ERR_SHAPE, msg);
  }
  void* ws = scratch_of(plan->device);  // found when the plan was built, with its device current
  if (!ws) return fail(NNA_ERR_HIP, "the static workspace of the plan's device was never located");
  return run_octaves(plan, NNA_KIND_CQT2010V2, x_dev, B, L, out_dev, ws, (size_t)NNA_STATIC_SCRATCH_BYTES, hip_stream);
}

nna_status nna_cqt2010(const nna_plan* plan, const float* x_dev, long long B, long long L, float* out_dev,
                       void* workspace_dev, size_t workspace_bytes, void* hip_stream) {
  return run_octaves(plan, NNA_KIND_CQT2010, x_dev, B, L, out_dev, workspace_dev, workspace_bytes, hip_stream);
}

nna_status nna_plan_part(const nna_plan* plan, int index, const nna_plan** part) {
  if (!plan || !part) return fail(NNA_ERR_INVALID_ARG, "plan / part is NULL");
  *part = nullptr;
  if (plan->kind != NNA_KIND_CQT2010V2 && plan->kind != NNA_KIND_CQT2010)
    return fail(NNA_ERR_INVALID_ARG, "not a downsampling CQT plan");
  if (index == -1) {
    if (!plan->fir) return fail(NNA_ERR_INVALID_ARG, "a single-octave plan has no filter");
    *part = plan->fir;
    return NNA_OK;
  }
  if (index < 0 || index >= (int)plan->octave.size()) return fail(NNA_ERR_INVALID_ARG, "no such octave");
  *part = plan->octave[index];
  return NNA_OK;
}

nna_status nna_out_shape(const nna_plan* plan, long long B, long long L, long long* n_bins, long long* n_frames) {
  if (!plan) return fail(NNA_ERR_INVALID_ARG, "plan is NULL");
  if (B < 1) return fail(NNA_ERR_SHAPE, "B must be >= 1");
  if (plan->kind == NNA_KIND_CQT2010V2 || plan->kind == NNA_KIND_CQT2010) {
    long long La[MAX_OCTAVES];
    if (L < 1 || !cqt2010_lengths(plan, L, La))
      return fail(NNA_ERR_SHAPE, "L is too short: every octave's waveform must exceed the reflection padding, and all but the lowest hold one frame of the decimation filter");
    if (n_bins) *n_bins = plan->n_bins;
    if (n_frames) *n_frames = 1 + L / plan->hop;
    return NNA_OK;
  }
  if (L < 4) return fail(NNA_ERR_SHAPE, "L must be at least 4 samples");
  const long long T = frames_of(plan, L);
  if (T < 1) return fail(NNA_ERR_SHAPE, plan->center ? "L must exceed the reflection padding (K/2)" : "L is shorter than one window");
  if (n_bins) *n_bins = plan->out_rows();
  if (n_frames) *n_frames = T;
  return NNA_OK;
}

nna_status nna_stft(const nna_plan* plan, const float* x_dev, long long B, long long L, float* out_dev, void* hip_stream) {
  return run_stft_like(plan, NNA_KIND_STFT, x_dev, B, L, out_dev, hip_stream);
}

nna_status nna_mel(const nna_plan* plan, const float* x_dev, long long B, long long L, float* out_dev, void* hip_stream) {
  return run_stft_like(plan, NNA_KIND_MEL, x_dev, B, L, out_dev, hip_stream);
}

nna_status nna_mel_with_stft(const nna_plan* plan, const float* x_dev, long long B, long long L, float* mel_dev,
                             float* spec_dev, void* hip_stream) {
  if (!spec_dev) return fail(NNA_ERR_INVALID_ARG, "spec_dev is NULL");
  long long T = 0;
  nna_status s = check_call(plan, NNA_KIND_MEL, x_dev, B, L, mel_dev, &T);
  if (s != NNA_OK) return s;
  if (plan->precision != NNA_PREC_F32) return fail(NNA_ERR_UNSUPPORTED, "float32 plans only");
  return run_stft_core(plan, NNA_KIND_MEL, x_dev, B, L, T, mel_dev, 0, 0, hip_stream, spec_dev);
}

nna_status nna_cqt(const nna_plan* plan, const float* x_dev, long long B, long long L, float* out_dev, void* hip_stream) {
  long long T = 0;
  nna_status s = check_call(plan, NNA_KIND_CQT, x_dev, B, L, out_dev, &T);
  if (s != NNA_OK) return s;
  DeviceGuard guard;
  hipError_t e = guard.enter(plan->device);
  if (e != hipSuccess) return fail_hip(e, "hipSetDevice");
  return run_conv(plan, x_dev, B, L, T, out_dev, (long long)plan->out_rows() * T, 0, hip_stream);
}

// ---- trainable Fourier kernels (Sec. IV-C) ----------------------------------------------------
static nna_status check_trainable_kind(const nna_plan* plan) {
  if (!plan) return fail(NNA_ERR_INVALID_ARG, "plan is NULL");
  if (plan->kind != NNA_KIND_STFT && plan->kind != NNA_KIND_MEL && plan->kind != NNA_KIND_CQT)
    return fail(NNA_ERR_INVALID_ARG, "only plans from nna_plan_stft, nna_plan_stft_scaled, nna_plan_mel and nna_plan_cqt have trainable kernels");
  if (plan->precision != NNA_PREC_F32) return fail(NNA_ERR_UNSUPPORTED, "trainable kernels need a float32 plan");
  if (plan->device < 0) return fail(NNA_ERR_UNSUPPORTED, "host-only plan (device = -1)");
  return NNA_OK;
}

static nna::BankPermuteParams permute_params(const nna_plan* plan, float* logical) {
  nna::BankPermuteParams q;
  q.bank = plan->d_bank;
  q.wrm = plan->d_wrm;
  q.logical = logical;
  q.n_rt = plan->n_rt;
  q.n_chunks = plan->n_chunks;
  q.nj = plan->nj;
  q.hop = plan->hop;
  q.K = plan->K;
  q.kp = plan->kp;
  q.n_half = plan->n_half;
  q.packed = plan->freq_scale ? 0 : 1;
  return q;
}

static nna::CqtBankParams cqt_bank_params(const nna_plan* plan, float* logical) {
  nna::CqtBankParams q;
  q.bank = plan->d_bank;
  q.map = plan->d_cq_map;
  q.n_bank = (long long)plan->bank_floats;
  q.wrm = plan->d_wrm;
  q.row_lo = plan->d_row_lo;
  q.row_hi = plan->d_row_hi;
  q.logical = logical;
  q.rows = plan->conv_rows;
  q.K = plan->K;
  q.kp = plan->kp;
  return q;
}

// A constant-Q plan becomes trainable (device current): the parameters are the taps inside each kernel's
// support [s_k, s_k + N_k); the zeros that centre a kernel among n_taps stay zeros.
static nna_status make_cqt_trainable(nna_plan* plan) {
  const int rows = plan->conv_rows;
  const long long K = plan->K;
  if ((long long)rows * K > 0x7fffffffLL) return fail(NNA_ERR_UNSUPPORTED, "bank of more than 2^31 - 1 entries");
  const int rows_pad = (rows + nna::BW_MT - 1) / nna::BW_MT * nna::BW_MT;
  const int kp = (int)((K + nna::BW_NT - 1) / nna::BW_NT * nna::BW_NT);
  const int n_nt = kp / nna::BW_NT;
  std::vector<int> map, lo(rows_pad, 0), hi(rows_pad, 0), nt_chunks(n_nt, 0);
  std::vector<int2> shift_rng;
  std::vector<int2> tiles;
  std::vector<float> logical;
  try {
    // streaming order <- [row][tap]: the inverse of the layout build_conv_bank writes
    map.assign(plan->bank_floats, -1);
    for_each_cqt_fragment(plan, [&](long long f, int rb, int j, int c0, bool real) {
      if (!real) return;
      for (int lane = 0; lane < 64; ++lane) {
        const int q = lane >> 4, row = rb * CQ_ROWS + (lane & 15);
        const long long tap0 = (long long)j * plan->tap_stride + c0 + 4 * q;
        for (int e = 0; e < 4; ++e)
          if (row < rows && tap0 + e >= plan->row_s[row] && tap0 + e < plan->row_e[row])
            map[((size_t)f * 64 + lane) * 4 + e] = (int)(row * K + tap0 + e);
      }
    });
    for (int r = 0; r < rows; ++r) {
      lo[r] = (int)plan->row_s[r];
      hi[r] = (int)plan->row_e[r];
    }
    // bank gradient: output tiles (128 rows x 128 taps) that hold a parameter
    for (int mt = 0; mt < rows_pad / nna::BW_MT; ++mt) {
      long long s = K, e = 0;
      for (int r = mt * nna::BW_MT; r < std::min(rows, (mt + 1) * nna::BW_MT); ++r) {
        s = std::min(s, plan->row_s[r]);
        e = std::max(e, plan->row_e[r]);
      }
      for (long long nt = s / nna::BW_NT; nt * nna::BW_NT < e; ++nt) {
        // 32-row blocks of the tile with taps on this tap tile (rows are ordered longest first: a prefix)
        int alive = 0;
        for (int r = mt * nna::BW_MT; r < std::min(rows, (mt + 1) * nna::BW_MT); ++r)
          if (plan->row_s[r] < (nt + 1) * nna::BW_NT && plan->row_e[r] > nt * nna::BW_NT) alive = (r - mt * nna::BW_MT) / 32 + 1;
        tiles.push_back(make_int2(mt | (alive << 16), (int)nt));
      }
    }
    // heaviest tiles first (a tile's time goes with its live row blocks): the light ones fill the launch's tail
    std::stable_sort(tiles.begin(), tiles.end(), [](const int2& a, const int2& b) { return (a.x >> 16) > (b.x >> 16); });
    // waveform gradient: how many rows (in chunks of 32; rows are ordered longest first) hold taps on each
    // 128-tap tile, and from that, per 128-column tile of the hop, the running count over the hop-shifts
    for (int nt = 0; nt < n_nt; ++nt) {
      int r_max = 0;
      for (int r = 0; r < rows; ++r)
        if (plan->row_s[r] < (long long)(nt + 1) * nna::BW_NT && plan->row_e[r] > (long long)nt * nna::BW_NT) r_max = r + 1;
      nt_chunks[nt] = (r_max + nna::BW_KC - 1) / nna::BW_KC;
    }
    if (tiles.empty()) return fail(NNA_ERR_UNSUPPORTED, "the bank has no taps");
    const int J = (int)((K + plan->hop - 1) / plan->hop), n_ct = (plan->hop + nna::BW_NT - 1) / nna::BW_NT;
    int n_kc = 0;
    for (int nt = 0; nt < n_nt; ++nt) n_kc = std::max(n_kc, nt_chunks[nt]);
    shift_rng.assign((size_t)n_ct * n_kc, make_int2(1, 0));
    for (int ct = 0; ct < n_ct; ++ct)
      for (int j = 0; j < J; ++j) {
        const long long tb = (long long)j * plan->hop + (long long)ct * nna::BW_NT;
        int chunks = 0;
        if (tb < K) {
          const long long last = std::min({tb + nna::BW_NT - 1, (long long)(j + 1) * plan->hop - 1, K - 1});
          for (long long nt = tb / nna::BW_NT; nt <= last / nna::BW_NT; ++nt) chunks = std::max(chunks, nt_chunks[nt]);
        }
        for (int kc = 0; kc < chunks; ++kc) {
          int2& r = shift_rng[(size_t)ct * n_kc + kc];
          if (r.x > r.y) r = make_int2(j, j);
          r.y = j;
        }
      }
    plan->n_kc = n_kc;
    plan->n_shift = J;
    plan->n_ct = n_ct;
    plan->n_bw_tiles = (int)tiles.size();
    // the bank as the caller's tensor: the values the plan was built with
    logical.assign((size_t)rows * K, 0.0f);
    CqtKernelGen gen(plan);
    for (int r = 0; r < rows; ++r)
      for (long long n = plan->row_s[r]; n < plan->row_e[r]; ++n) logical[(size_t)r * K + n] = (float)gen.value(r, n);
  } catch (const std::bad_alloc&) {
    return fail(NNA_ERR_ALLOC, "out of host memory");
  }
  plan->rows_pad = rows_pad;
  plan->kp = kp;
  float* d_logical = nullptr;
  const size_t wrm_bytes = (size_t)rows_pad * kp * sizeof(float);
  nna_status s = upload(&plan->d_wrm, nullptr, wrm_bytes, "row-major kernel bank");
  if (s == NNA_OK) s = upload(&plan->d_cq_map, map.data(), map.size() * sizeof(int), "bank index map");
  if (s == NNA_OK) s = upload(&plan->d_row_lo, lo.data(), lo.size() * sizeof(int), "row supports");
  if (s == NNA_OK) s = upload(&plan->d_row_hi, hi.data(), hi.size() * sizeof(int), "row supports");
  if (s == NNA_OK) s = upload(&plan->d_bw_tiles, tiles.data(), tiles.size() * sizeof(int2), "gradient tile list");
  if (s == NNA_OK) s = upload(&plan->d_shift_rng, shift_rng.data(), shift_rng.size() * sizeof(int2), "hop-shift table");
  if (s == NNA_OK) s = upload(&d_logical, logical.data(), logical.size() * sizeof(float), "kernel bank");
  if (s == NNA_OK) {
    hipError_t e = hipMemset(plan->d_wrm, 0, wrm_bytes);
    if (e == hipSuccess) e = nna::launch_cqt_bank_from_logical(cqt_bank_params(plan, d_logical), nullptr);
    if (e == hipSuccess) e = hipStreamSynchronize(nullptr);
    if (e != hipSuccess) s = fail_hip(e, "row-major kernel bank");
  }
  (void)hipFree(d_logical);
  if (s != NNA_OK) {
    (void)hipFree(plan->d_wrm);
    (void)hipFree(plan->d_cq_map);
    (void)hipFree(plan->d_row_lo);
    (void)hipFree(plan->d_row_hi);
    (void)hipFree(plan->d_bw_tiles);
    (void)hipFree(plan->d_shift_rng);
    plan->d_wrm = nullptr;
    plan->d_cq_map = plan->d_row_lo = plan->d_row_hi = nullptr;
    plan->d_shift_rng = nullptr;
    plan->d_bw_tiles = nullptr;
  }
  return s;
}

nna_status nna_plan_trainable(nna_plan* plan) {
  nna_status s = check_trainable_kind(plan);
  if (s != NNA_OK) return s;
  if (plan->d_wrm) return NNA_OK;
  DeviceGuard guard;
  hipError_t e = guard.enter(plan->device);
  if (e != hipSuccess) return fail_hip(e, "hipSetDevice");
  if (plan->kind == NNA_KIND_CQT) return make_cqt_trainable(plan);
  plan->rows_pad = plan->n_rt * ST_ROWS;
  plan->kp = (plan->K + nna::BW_NT - 1) / nna::BW_NT * nna::BW_NT;
  const size_t bytes = (size_t)plan->rows_pad * plan->kp * sizeof(float);
  if ((s = upload(&plan->d_wrm, nullptr, bytes, "row-major kernel bank")) != NNA_OK) return s;
  e = hipMemset(plan->d_wrm, 0, bytes);
  if (e == hipSuccess) e = nna::launch_bank_to_rowmajor(permute_params(plan, nullptr), nullptr);
  if (e == hipSuccess) e = hipStreamSynchronize(nullptr);
  if (e != hipSuccess) {
    (void)hipFree(plan->d_wrm);
    plan->d_wrm = nullptr;
    return fail_hip(e, "row-major kernel bank");
  }
  if (plan->kind == NNA_KIND_MEL) {
    // Trained filters are no longer triangles: from here on every 32 x 16 weight block is multiplied
    // and every pass sweeps all row tiles.  The filterbank gets its row-major copy.
    const int F = plan->n_half + 1;
    plan->fp = (F + nna::BW_MT - 1) / nna::BW_MT * nna::BW_MT;
    plan->mels_pad = (plan->n_mels + nna::BW_KC - 1) / nna::BW_KC * nna::BW_KC;
    std::vector<unsigned char> mask((size_t)plan->n_pass * plan->n_rt * ST_RB, (unsigned char)((1u << ST_MEL_BLOCKS) - 1));
    std::vector<int> pass_rt((size_t)plan->n_pass * 2);
    for (int p = 0; p < plan->n_pass; ++p) {
      pass_rt[2 * p] = 0;
      pass_rt[2 * p + 1] = plan->n_rt;
    }
    std::vector<float> rm((size_t)plan->mels_pad * plan->fp, 0.0f);
    for (int m = 0; m < plan->n_mels; ++m)
      for (int k = 0; k < F; ++k) rm[(size_t)m * plan->fp + k] = plan->h_melW[(size_t)m * F + k];
    s = upload(&plan->d_melw_rm, rm.data(), rm.size() * sizeof(float), "row-major filterbank");
    if (s == NNA_OK) {
      e = hipMemcpy(plan->d_mel_mask, mask.data(), mask.size(), hipMemcpyHostToDevice);
      if (e == hipSuccess) e = hipMemcpy(plan->d_mel_pass_rt, pass_rt.data(), pass_rt.size() * sizeof(int), hipMemcpyHostToDevice);
      if (e != hipSuccess) s = fail_hip(e, "filterbank tables");
    }
    if (s != NNA_OK) {
      (void)hipFree(plan->d_wrm);
      (void)hipFree(plan->d_melw_rm);
      plan->d_wrm = plan->d_melw_rm = nullptr;
      return s;
    }
    plan->mel_nyq_any = 1;
    const double k_exec = (double)plan->n_chunks * plan->nj * ST_KC;
    plan->exec_flops = plan->n_pass * (2.0 * k_exec * ST_ROWS * plan->n_rt + (double)plan->n_rt * ST_RB * ST_MEL_BLOCKS * 2.0 * 32 * 16);
    plan->alg_flops = 2.0 * (double)plan->K * (double)plan->K + 2.0 * (double)plan->n_mels * F;
  }
  return NNA_OK;
}

static nna_status check_trainable(const nna_plan* plan) {
  nna_status s = check_trainable_kind(plan);
  if (s != NNA_OK) return s;
  if (!plan->d_wrm) return fail(NNA_ERR_INVALID_ARG, "call nna_plan_trainable on the plan first");
  return NNA_OK;
}

nna_status nna_plan_get_bank(const nna_plan* plan, float* w_dev, void* hip_stream) {
  nna_status s = check_trainable(plan);
  if (s != NNA_OK) return s;
  if (!w_dev) return fail(NNA_ERR_INVALID_ARG, "w_dev is NULL");
  DeviceGuard guard;
  hipError_t e = guard.enter(plan->device);
  if (e != hipSuccess) return fail_hip(e, "hipSetDevice");
  if (plan->kind == NNA_KIND_CQT)
    e = nna::launch_cqt_bank_to_logical(cqt_bank_params(plan, w_dev), reinterpret_cast<hipStream_t>(hip_stream));
  else
    e = nna::launch_bank_to_logical(permute_params(plan, w_dev), reinterpret_cast<hipStream_t>(hip_stream));
  if (e != hipSuccess) return fail_hip(e, "kernel launch");
  return NNA_OK;
}

nna_status nna_plan_set_bank(nna_plan* plan, const float* w_dev, void* hip_stream) {
  nna_status s = check_trainable(plan);
  if (s != NNA_OK) return s;
  if (!w_dev) return fail(NNA_ERR_INVALID_ARG, "w_dev is NULL");
  DeviceGuard guard;
  hipError_t e = guard.enter(plan->device);
  if (e != hipSuccess) return fail_hip(e, "hipSetDevice");
  if (plan->kind == NNA_KIND_CQT)
    e = nna::launch_cqt_bank_from_logical(cqt_bank_params(plan, const_cast<float*>(w_dev)), reinterpret_cast<hipStream_t>(hip_stream));
  else
    e = nna::launch_bank_from_logical(permute_params(plan, const_cast<float*>(w_dev)), reinterpret_cast<hipStream_t>(hip_stream));
  if (e != hipSuccess) return fail_hip(e, "kernel launch");
  return NNA_OK;
}

static long long bw_gpitch(long long n_frames) { return (n_frames + nna::BW_MT - 1) / nna::BW_MT * nna::BW_MT; }

nna_status nna_stft_backward_workspace(const nna_plan* plan, long long B, long long L, size_t* bytes) {
  nna_status s = check_trainable(plan);
  if (s != NNA_OK) return s;
  if (!bytes) return fail(NNA_ERR_INVALID_ARG, "bytes is NULL");
  if (B < 1) return fail(NNA_ERR_SHAPE, "B must be >= 1");
  const long long T = frames_of(plan, L);
  if (T < 1) return fail(NNA_ERR_SHAPE, plan->center ? "L must exceed the reflection padding (K/2)" : "L is shorter than one window");
  *bytes = (size_t)plan->rows_pad * (size_t)bw_gpitch(B * T) * sizeof(float);
  return NNA_OK;
}

// The backward pass of the STFT stage: gout[B, out_bins, T] is the gradient with respect to the stage's
// output in format `fmt`; gbuf holds G (rows_pad x padded frames floats).  Arguments already checked.
// pout (optional, magnitude / power formats): the stage's own output is written there on the way.
// With gw_dev and gx_dev both NULL only G (and pout) are produced.
static nna_status stft_backward_core(const nna_plan* plan, const float* x_dev, long long B, long long L, long long T,
                                     const float* gout_dev, int fmt, int out_bins, float* gw_dev, float* gx_dev,
                                     float* gbuf, void* hip_stream, float* pout = nullptr) {
  const int M = pick_tile_frames(ST_FRAMES, T, plan->nj - 1, ST_LDS_ROWS);
  if (M < 1) return fail(NNA_ERR_UNSUPPORTED, "frame tile does not fit in LDS");
  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
  DeviceGuard guard;
  hipError_t e = guard.enter(plan->device);
  if (e != hipSuccess) return fail_hip(e, "hipSetDevice");

  const long long n_frames = B * T, gpitch = bw_gpitch(n_frames);
  const int packed = plan->freq_scale ? 0 : 1;
  // 1. G = dLoss/dC: the forward contraction again, its epilogue turned into the output format's derivative
  e = nna::launch_fill_zero_frames(gbuf, plan->rows_pad, n_frames, gpitch, stream);
  if (e != hipSuccess) return fail_hip(e, "kernel launch");
  nna::StftParams P;
  std::memset(&P, 0, sizeof(P));
  P.g = make_geom(plan, x_dev, B, L, T);
  P.bank = reinterpret_cast<const float4*>(plan->d_bank);
  P.n_rt = plan->n_rt;
  P.n_chunks = plan->n_chunks;
  P.nj = plan->nj;
  P.n_half = plan->n_half;
  P.packed = packed;
  P.out_bins = out_bins;
  P.fmt = fmt;
  P.tile_frames = M;
  P.n_ft = (n_frames + M - 1) / M;
  P.gout = gout_dev;
  P.pout = pout;
  P.gbuf = gbuf;
  P.gpitch = 32;  // G is stored in blocks of 32 frames: [frame / 32][packed row][frame % 32]
  e = nna::launch_stft(P, nna::ST_MODE_GRAD, stream);
  if (e != hipSuccess) return fail_hip(e, "kernel launch");
  // 2. the two contractions with G
  nna::BwParams Q;
  std::memset(&Q, 0, sizeof(Q));
  Q.g = P.g;
  Q.gbuf = gbuf;
  Q.gpitch = gpitch;
  Q.wrm = plan->d_wrm;
  Q.kp = plan->kp;
  Q.rows_pad = plan->rows_pad;
  Q.n_half = plan->n_half;
  Q.packed = packed;
  Q.K = plan->K;
  Q.gw = gw_dev;
  Q.gx = gx_dev;
  if (gw_dev) {
    e = nna::launch_fill_zero(gw_dev, 2LL * plan->stft_bins() * plan->K, stream);
    if (e != hipSuccess) return fail_hip(e, "kernel launch");
    // split the contraction over the frames so that about 1,024 workgroups exist (two per compute
    // unit, twice over), each with at least 64 chunks to amortise its start-up
    const long long tiles = (long long)(plan->rows_pad / nna::BW_MT) * (plan->kp / nna::BW_NT);
    const long long chunks = gpitch / nna::BW_KC;
    long long split = std::max(1LL, std::min((1024 + tiles - 1) / tiles, chunks / 64));
    Q.chunks_per_split = (chunks + split - 1) / split;
    Q.n_split = (int)((chunks + Q.chunks_per_split - 1) / Q.chunks_per_split);
    e = nna::launch_bw_bank(Q, stream);
    if (e != hipSuccess) return fail_hip(e, "kernel launch");
  }
  if (gx_dev) {
    e = nna::launch_fill_zero(gx_dev, B * L, stream);
    if (e != hipSuccess) return fail_hip(e, "kernel launch");
    e = nna::launch_bw_wave(Q, stream);
    if (e != hipSuccess) return fail_hip(e, "kernel launch");
  }
  return NNA_OK;
}

nna_status nna_stft_backward(const nna_plan* plan, const float* x_dev, long long B, long long L, const float* gout_dev,
                             float* gw_dev, float* gx_dev, void* workspace_dev, size_t workspace_bytes, void* hip_stream) {
  nna_status s = check_trainable(plan);
  if (s != NNA_OK) return s;
  if (plan->kind != NNA_KIND_STFT) return fail(NNA_ERR_INVALID_ARG, "plan was built for a different transform");
  if (!gout_dev) return fail(NNA_ERR_INVALID_ARG, "gout_dev is NULL");
  if (!gw_dev && !gx_dev) return fail(NNA_ERR_INVALID_ARG, "gw_dev and gx_dev are both NULL: nothing to compute");
  long long T = 0;
  // (check_call wants an output pointer; the gradient buffers play that part)
  if ((s = check_call(plan, NNA_KIND_STFT, x_dev, B, L, gw_dev ? gw_dev : gx_dev, &T)) != NNA_OK) return s;
  size_t need = 0;
  if ((s = nna_stft_backward_workspace(plan, B, L, &need)) != NNA_OK) return s;
  if (!workspace_dev || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace_dev) & 255))
    return fail(NNA_ERR_INVALID_ARG, "workspace_dev is NULL, not 256-byte aligned or smaller than nna_stft_backward_workspace asks for");
  return stft_backward_core(plan, x_dev, B, L, T, gout_dev, plan->fmt, plan->out_rows(), gw_dev, gx_dev,
                            static_cast<float*>(workspace_dev), hip_stream);
}

// ---- trainable constant-Q kernels (time-domain kernels at one rate) ------------------------------
nna_status nna_cqt_backward_workspace(const nna_plan* plan, long long B, long long L, size_t* bytes) {
  nna_status s = check_trainable(plan);
  if (s != NNA_OK) return s;
  if (plan->kind != NNA_KIND_CQT) return fail(NNA_ERR_INVALID_ARG, "plan was built for a different transform");
  if (!bytes) return fail(NNA_ERR_INVALID_ARG, "bytes is NULL");
  if (B < 1) return fail(NNA_ERR_SHAPE, "B must be >= 1");
  const long long T = frames_of(plan, L);
  if (T < 1) return fail(NNA_ERR_SHAPE, plan->center ? "L must exceed the reflection padding (K/2)" : "L is shorter than one window");
  *bytes = (size_t)plan->rows_pad * (size_t)bw_gpitch(B * T) * sizeof(float);
  return NNA_OK;
}

nna_status nna_cqt_backward(const nna_plan* plan, const float* x_dev, long long B, long long L, const float* gout_dev,
                            float* gw_dev, float* gx_dev, void* workspace_dev, size_t workspace_bytes, void* hip_stream) {
  nna_status s = check_trainable(plan);
  if (s != NNA_OK) return s;
  if (plan->kind != NNA_KIND_CQT) return fail(NNA_ERR_INVALID_ARG, "plan was built for a different transform");
  if (!gout_dev) return fail(NNA_ERR_INVALID_ARG, "gout_dev is NULL");
  if (!gw_dev && !gx_dev) return fail(NNA_ERR_INVALID_ARG, "gw_dev and gx_dev are both NULL: nothing to compute");
  long long T = 0;
  if ((s = check_call(plan, NNA_KIND_CQT, x_dev, B, L, gw_dev ? gw_dev : gx_dev, &T)) != NNA_OK) return s;
  size_t need = 0;
  if ((s = nna_cqt_backward_workspace(plan, B, L, &need)) != NNA_OK) return s;
  if (!workspace_dev || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace_dev) & 255))
    return fail(NNA_ERR_INVALID_ARG, "workspace_dev is NULL, not 256-byte aligned or smaller than nna_cqt_backward_workspace asks for");
  const int extra = (plan->max_jspan - 1) * plan->row_step;
  const int M = pick_tile_frames(CQ_FRAMES, T, extra, CQ_LDS_ROWS_MAX);
  if (M < 1) return fail(NNA_ERR_UNSUPPORTED, "frame tile does not fit in LDS");
  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
  DeviceGuard guard;
  hipError_t e = guard.enter(plan->device);
  if (e != hipSuccess) return fail_hip(e, "hipSetDevice");

  float* gbuf = static_cast<float*>(workspace_dev);
  const long long n_frames = B * T, gpitch = bw_gpitch(n_frames);
  // 1. G = dLoss/dC: the forward contraction again with the derivative of the output format as its
  //    epilogue.  The kernel writes the rows of existing bins and frames; the padding stays zero.
  e = nna::launch_fill_zero(gbuf, (long long)plan->rows_pad * gpitch, stream);
  if (e != hipSuccess) return fail_hip(e, "kernel launch");
  nna::CqtParams P;
  std::memset(&P, 0, sizeof(P));
  P.g = make_geom(plan, x_dev, B, L, T);
  P.bank = reinterpret_cast<const float4*>(plan->d_bank);
  P.items = plan->d_items;
  P.chunks = plan->d_chunks;
  P.n_items = (int)plan->h_items.size();
  P.n_chunks = plan->n_chunks;
  P.n_bins = plan->n_bins;
  P.fmt = plan->fmt;
  P.tap_stride = plan->tap_stride;
  P.row_step = plan->row_step;
  P.tile_frames = M;
  const long long nseg = 1 + (M - 1 + T - 1) / T;
  P.lds_rows = (int)((M + nseg * extra + 63) / 64 * 64);
  P.n_ft = (n_frames + M - 1) / M;
  P.gout = gout_dev;
  P.gout_wave_stride = (long long)plan->out_rows() * T;
  P.gbuf = gbuf;
  P.rows_pad = plan->rows_pad;
  e = nna::launch_cqt(P, stream);
  if (e != hipSuccess) return fail_hip(e, "kernel launch");
  // 2. the two contractions with G, restricted to the tiles that hold taps
  nna::BwParams Q;
  std::memset(&Q, 0, sizeof(Q));
  Q.g = P.g;
  Q.gbuf = gbuf;
  Q.gpitch = gpitch;
  Q.wrm = plan->d_wrm;
  Q.kp = plan->kp;
  Q.rows_pad = plan->rows_pad;
  Q.n_half = plan->n_bins;
  Q.packed = 0;
  Q.K = plan->K;
  Q.gw = gw_dev;
  Q.gx = gx_dev;
  Q.tiles = plan->d_bw_tiles;
  Q.n_tiles = plan->n_bw_tiles;
  Q.row_lo = plan->d_row_lo;
  Q.row_hi = plan->d_row_hi;
  Q.shift_rng = plan->d_shift_rng;
  Q.n_kc = plan->n_kc;
  Q.n_shift = plan->n_shift;
  Q.n_ct = plan->n_ct;
  Q.n_qt = (T + plan->n_shift - 1 + nna::BW_MT - 1) / nna::BW_MT;
  if (gw_dev) {
    e = nna::launch_fill_zero(gw_dev, (long long)plan->conv_rows * plan->K, stream);
    if (e != hipSuccess) return fail_hip(e, "kernel launch");
    const long long chunks = gpitch / nna::BW_KC;
    // the tile count is whatever the supports give: aim at eight rounds of the 512 resident workgroups, so
    // that a partly filled last round costs little
    long long split = std::max(1LL, std::min((4096 + (long long)Q.n_tiles - 1) / Q.n_tiles, chunks / 64));
    Q.chunks_per_split = (chunks + split - 1) / split;
    Q.n_split = (int)((chunks + Q.chunks_per_split - 1) / Q.chunks_per_split);
    e = nna::launch_bw_bank(Q, stream);
    if (e != hipSuccess) return fail_hip(e, "kernel launch");
  }
  if (gx_dev) {
    e = nna::launch_fill_zero(gx_dev, B * L, stream);
    if (e != hipSuccess) return fail_hip(e, "kernel launch");
    e = nna::launch_bw_wave(Q, stream);
    if (e != hipSuccess) return fail_hip(e, "kernel launch");
  }
  return NNA_OK;
}

// ---- trainable Mel layer -----------------------------------------------------------------------
static nna_status check_trainable_mel(const nna_plan* plan) {
  nna_status s = check_trainable(plan);
  if (s != NNA_OK) return s;
  if (plan->kind != NNA_KIND_MEL) return fail(NNA_ERR_INVALID_ARG, "not a Mel plan");
  return NNA_OK;
}

nna_status nna_plan_get_mel_weights(const nna_plan* plan, float* w_dev, void* hip_stream) {
  nna_status s = check_trainable_mel(plan);
  if (s != NNA_OK) return s;
  if (!w_dev) return fail(NNA_ERR_INVALID_ARG, "w_dev is NULL");
  DeviceGuard guard;
  hipError_t e = guard.enter(plan->device);
  if (e != hipSuccess) return fail_hip(e, "hipSetDevice");
  const size_t F = plan->n_half + 1;
  e = hipMemcpy2DAsync(w_dev, F * sizeof(float), plan->d_melw_rm, (size_t)plan->fp * sizeof(float), F * sizeof(float),
                       plan->n_mels, hipMemcpyDeviceToDevice, reinterpret_cast<hipStream_t>(hip_stream));
  if (e != hipSuccess) return fail_hip(e, "filterbank copy");
  return NNA_OK;
}

nna_status nna_plan_set_mel_weights(nna_plan* plan, const float* w_dev, void* hip_stream) {
  nna_status s = check_trainable_mel(plan);
  if (s != NNA_OK) return s;
  if (!w_dev) return fail(NNA_ERR_INVALID_ARG, "w_dev is NULL");
  DeviceGuard guard;
  hipError_t e = guard.enter(plan->device);
  if (e != hipSuccess) return fail_hip(e, "hipSetDevice");
  e = nna::launch_mel_from_logical(w_dev, plan->d_melw, plan->d_mel_wnyq, plan->d_melw_rm, plan->n_mels, plan->n_half,
                                   plan->n_rt, plan->n_pass, plan->fp, reinterpret_cast<hipStream_t>(hip_stream));
  if (e != hipSuccess) return fail_hip(e, "kernel launch");
  return NNA_OK;
}

static size_t ws256(size_t bytes) { return (bytes + 255) / 256 * 256; }

nna_status nna_mel_backward_workspace(const nna_plan* plan, long long B, long long L, size_t* bytes) {
  nna_status s = check_trainable_mel(plan);
  if (s != NNA_OK) return s;
  if (!bytes) return fail(NNA_ERR_INVALID_ARG, "bytes is NULL");
  if (B < 1) return fail(NNA_ERR_SHAPE, "B must be >= 1");
  const long long T = frames_of(plan, L);
  if (T < 1) return fail(NNA_ERR_SHAPE, plan->center ? "L must exceed the reflection padding (K/2)" : "L is shorter than one window");
  const size_t spec = ws256((size_t)B * (plan->n_half + 1) * T * sizeof(float));
  *bytes = 2 * spec + (size_t)plan->rows_pad * (size_t)bw_gpitch(B * T) * sizeof(float);
  return NNA_OK;
}

nna_status nna_mel_backward(const nna_plan* plan, const float* x_dev, long long B, long long L, const float* gout_dev,
                            float* gmelw_dev, float* gw_dev, float* gx_dev, void* workspace_dev, size_t workspace_bytes,
                            void* hip_stream) {
  nna_status s = check_trainable_mel(plan);
  if (s != NNA_OK) return s;
  if (!gout_dev) return fail(NNA_ERR_INVALID_ARG, "gout_dev is NULL");
  if (!gmelw_dev && !gw_dev && !gx_dev) return fail(NNA_ERR_INVALID_ARG, "all three gradient pointers are NULL: nothing to compute");
  long long T = 0;
  float* any_out = gmelw_dev ? gmelw_dev : gw_dev ? gw_dev : gx_dev;
  if ((s = check_call(plan, NNA_KIND_MEL, x_dev, B, L, any_out, &T)) != NNA_OK) return s;
  size_t need = 0;
  if ((s = nna_mel_backward_workspace(plan, B, L, &need)) != NNA_OK) return s;
  if (!workspace_dev || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace_dev) & 255))
    return fail(NNA_ERR_INVALID_ARG, "workspace_dev is NULL, not 256-byte aligned or smaller than nna_mel_backward_workspace asks for");
  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
  const int F = plan->n_half + 1;
  const size_t spec = ws256((size_t)B * F * T * sizeof(float));
  float* pbuf = static_cast<float*>(workspace_dev);
  float* gpbuf = reinterpret_cast<float*>(static_cast<char*>(workspace_dev) + spec);
  float* gbuf = reinterpret_cast<float*>(static_cast<char*>(workspace_dev) + 2 * spec);
  const int fmt = plan->mel_power == 2 ? NNA_OUT_POWER : NNA_OUT_MAGNITUDE;  // what the filterbank is applied to
  DeviceGuard guard;
  hipError_t e = guard.enter(plan->device);
  if (e != hipSuccess) return fail_hip(e, "hipSetDevice");
  nna::MelBwParams Q;
  std::memset(&Q, 0, sizeof(Q));
  Q.g = gout_dev;
  Q.wrm = plan->d_melw_rm;
  Q.P = pbuf;
  Q.gP = gpbuf;
  Q.gW = gmelw_dev;
  Q.B = B;
  Q.T = (int)T;
  Q.F = F;
  Q.n_mels = plan->n_mels;
  Q.fp = plan->fp;
  Q.mels_pad = plan->mels_pad;
  // 1. gP, the gradient reaching the STFT stage's output;  2. the STFT stage's backward pass, whose
  // recomputed contraction also writes the spectrogram P the filterbank saw when its gradient is
  // wanted;  3. filterbank gradient = gout x P.
  e = nna::launch_mel_bw_spec(Q, stream);
  if (e != hipSuccess) return fail_hip(e, "kernel launch");
  if ((s = stft_backward_core(plan, x_dev, B, L, T, gpbuf, fmt, F, gw_dev, gx_dev, gbuf, hip_stream,
                              gmelw_dev ? pbuf : nullptr)) != NNA_OK)
    return s;
  if (gmelw_dev) {
    e = nna::launch_fill_zero(gmelw_dev, (long long)plan->n_mels * F, stream);
    if (e != hipSuccess) return fail_hip(e, "kernel launch");
    // about 1,024 workgroups share the output tiles
    const long long tiles = (long long)((plan->n_mels + nna::BW_MT - 1) / nna::BW_MT) * (plan->fp / nna::BW_NT);
    const long long splits = std::max(1LL, std::min(B, (1024 + tiles - 1) / tiles));
    Q.b_per_split = (int)((B + splits - 1) / splits);
    e = nna::launch_mel_bw_weights(Q, stream);
    if (e != hipSuccess) return fail_hip(e, "kernel launch");
  }
  return NNA_OK;
}

nna_status nna_plan_bank(const nna_plan* plan, double* host_out, size_t cap) {
  if (!plan || !host_out) return fail(NNA_ERR_INVALID_ARG, "plan / host_out is NULL");
  if (plan->kind == NNA_KIND_CQT2010V2 || plan->kind == NNA_KIND_CQT2010)
    return fail(NNA_ERR_INVALID_ARG, "a downsampling CQT plan holds several banks");
  const long long rows = plan->kind == NNA_KIND_CQT ? (long long)plan->conv_rows : 2LL * (plan->freq_scale ? plan->n_half : plan->n_half + 1);
  const long long K = plan->K;
  if ((unsigned long long)cap < (unsigned long long)(rows * K)) return fail(NNA_ERR_INVALID_ARG, "host_out is too small");
  if (plan->precision == NNA_PREC_F16) {
    // the float16 bank, un-permuted from [row tile][chunk][hop-shift][H_ROWS][H_KC]
    std::vector<_Float16> tmp16;
    const _Float16* src16 = nullptr;
    try {
      if (plan->device >= 0) {
        tmp16.resize(plan->bank16_halves);
        DeviceGuard guard;
        hipError_t e = guard.enter(plan->device);
        if (e == hipSuccess) e = hipMemcpy(tmp16.data(), plan->d_bank16, plan->bank16_halves * sizeof(_Float16), hipMemcpyDeviceToHost);
        if (e != hipSuccess) return fail_hip(e, "bank read-back");
        src16 = tmp16.data();
      } else {
        src16 = plan->h_bank16.data();
      }
    } catch (const std::bad_alloc&) {
      return fail(NNA_ERR_ALLOC, "out of host memory");
    }
    std::fill(host_out, host_out + rows * K, 0.0);
    const int n_chunks = plan->hop / nna::H_KC, J = plan->nj;
    for (int rt = 0; rt < plan->n_rt16; ++rt)
      for (int c = 0; c < n_chunks; ++c)
        for (int j = 0; j < J; ++j)
          for (int r = 0; r < nna::H_ROWS; ++r) {
            const int pr = rt * nna::H_ROWS + r, slot = pr >> 1, part = pr & 1;
            if (slot >= plan->n_half) continue;
            const long long row = slot == 0 && !plan->freq_scale ? (part == 0 ? 0 : 2LL * plan->n_half) : 2LL * slot + part;
            const _Float16* t = src16 + ((((size_t)rt * n_chunks + c) * J + j) * nna::H_ROWS + r) * nna::H_KC;
            for (int e = 0; e < nna::H_KC; ++e) host_out[row * K + (long long)j * plan->hop + c * nna::H_KC + e] = (double)(float)t[e];
          }
    return NNA_OK;
  }
  std::vector<float> tmp;
  const float* src = nullptr;
  try {
    if (plan->device >= 0) {
      tmp.resize(plan->bank_floats);
      DeviceGuard guard;
      hipError_t e = guard.enter(plan->device);
      if (e == hipSuccess) e = hipMemcpy(tmp.data(), plan->d_bank, plan->bank_floats * sizeof(float), hipMemcpyDeviceToHost);
      if (e != hipSuccess) return fail_hip(e, "bank read-back");
      src = tmp.data();
    } else {
      src = plan->h_bank.data();
    }
  } catch (const std::bad_alloc&) {
    return fail(NNA_ERR_ALLOC, "out of host memory");
  }
  std::fill(host_out, host_out + rows * K, 0.0);
  if (plan->kind == NNA_KIND_CQT) {
    for_each_cqt_fragment(plan, [&](long long f, int rb, int j, int c0, bool real) {
      if (!real) return;
      for (int lane = 0; lane < 64; ++lane) {
        const int q = lane >> 4, r = lane & 15;
        const long long row = (long long)rb * CQ_ROWS + r;
        const long long tap0 = (long long)j * plan->tap_stride + c0 + 4 * q;
        for (int e = 0; e < 4; ++e)
          if (row < rows && tap0 + e < K) host_out[row * K + tap0 + e] = (double)src[((size_t)f * 64 + lane) * 4 + e];
      }
    });
  } else {
    const long long G = (long long)plan->n_chunks * plan->nj * ST_NKG;
    for (int rt = 0; rt < plan->n_rt; ++rt)
      for (int c = 0; c < plan->n_chunks; ++c)
        for (int j = 0; j < plan->nj; ++j)
          for (int kg = 0; kg < ST_NKG; ++kg) {
            const long long g = ((long long)c * plan->nj + j) * ST_NKG + kg;
            for (int rb = 0; rb < ST_RB; ++rb)
              for (int lane = 0; lane < 64; ++lane) {
                const int h = lane >> 5, r = lane & 31;
                const int pr = rt * ST_ROWS + rb * 32 + r;
                const int slot = pr >> 1, part = pr & 1;
                if (slot >= plan->n_half) continue;
                // packed slot 0 = (Re bin 0, Re bin N/2); slot s = (Re, Im) of bin s
                const long long row = slot == 0 && !plan->freq_scale ? (part == 0 ? 0 : 2LL * plan->n_half) : 2LL * slot + part;
                for (int e = 0; e < 4; ++e) {
                  const int k = stft_tap(plan, c, j, kg, h, e);
                  if (k < K) host_out[row * K + k] = (double)src[((((size_t)rt * G + g) * ST_RB + rb) * 64 + lane) * 4 + e];
                }
              }
          }
  }
  return NNA_OK;
}

nna_status nna_plan_mel_weights(const nna_plan* plan, double* host_out, size_t cap) {
  if (!plan || !host_out) return fail(NNA_ERR_INVALID_ARG, "plan / host_out is NULL");
  if (plan->kind != NNA_KIND_MEL) return fail(NNA_ERR_INVALID_ARG, "not a Mel plan");
  const size_t F = plan->n_half + 1, M = plan->n_mels;
  if (cap < M * F) return fail(NNA_ERR_INVALID_ARG, "host_out is too small");
  if (plan->device < 0) {
    for (size_t i = 0; i < M * F; ++i) host_out[i] = (double)plan->h_melW[i];
    return NNA_OK;
  }
  // read the device fragments back and undo the permutation
  const int per_pass = 32 * ST_MEL_BLOCKS;
  const size_t n = (size_t)plan->n_pass * plan->n_rt * ST_RB * ST_MEL_BLOCKS * 2 * 64 * 4;
  std::vector<float> frag, wnyq;
  try {
    frag.resize(n);
    wnyq.resize(M);
  } catch (const std::bad_alloc&) {
    return fail(NNA_ERR_ALLOC, "out of host memory");
  }
  {
    DeviceGuard guard;
    hipError_t e = guard.enter(plan->device);
    if (e == hipSuccess) e = hipMemcpy(frag.data(), plan->d_melw, n * sizeof(float), hipMemcpyDeviceToHost);
    if (e == hipSuccess) e = hipMemcpy(wnyq.data(), plan->d_mel_wnyq, M * sizeof(float), hipMemcpyDeviceToHost);
    if (e != hipSuccess) return fail_hip(e, "mel weight read-back");
  }
  std::fill(host_out, host_out + M * F, 0.0);
  for (int pass = 0; pass < plan->n_pass; ++pass)
    for (int rt = 0; rt < plan->n_rt; ++rt)
      for (int rb = 0; rb < ST_RB; ++rb)
        for (int mb = 0; mb < ST_MEL_BLOCKS; ++mb)
          for (int v = 0; v < 2; ++v)
            for (int lane = 0; lane < 64; ++lane) {
              const int h = lane >> 5, mm = lane & 31;
              const size_t mel = (size_t)pass * per_pass + mb * 32 + mm;
              for (int e = 0; e < 4; ++e) {
                const int idx8 = v * 4 + e, q = idx8 >> 1, e2 = idx8 & 1;
                const size_t bin = (size_t)rt * (ST_ROWS / 2) + rb * 16 + 4 * q + 2 * h + e2;
                const float w = frag[((((((size_t)pass * plan->n_rt + rt) * ST_RB + rb) * ST_MEL_BLOCKS + mb) * 2 + v) * 64 + lane) * 4 + e];
                if (mel < M && bin < (size_t)plan->n_half && w != 0.0f) host_out[mel * F + bin] = (double)w;
              }
            }
  for (size_t m = 0; m < M; ++m) host_out[m * F + plan->n_half] = (double)wnyq[m];
  return NNA_OK;
}

nna_status nna_plan_info(const nna_plan* plan, int* kind, long long* bank_rows, long long* taps, long long* out_bins,
                         double* executed_flops_per_frame, double* algorithmic_flops_per_frame) {
  if (!plan) return fail(NNA_ERR_INVALID_ARG, "plan is NULL");
  if (kind) *kind = plan->kind;
  if (bank_rows)
    *bank_rows = plan->kind == NNA_KIND_CQT2010V2 || plan->kind == NNA_KIND_CQT2010 ? 0
                 : plan->kind == NNA_KIND_CQT     ? (long long)plan->conv_rows
                                                  : 2LL * (plan->freq_scale ? plan->n_half : plan->n_half + 1);
  if (taps) *taps = plan->K;
  if (out_bins) *out_bins = plan->out_rows();
  if (executed_flops_per_frame) *executed_flops_per_frame = plan->runs_folded() ? plan->exec_flops_fold : plan->exec_flops;
  if (algorithmic_flops_per_frame) *algorithmic_flops_per_frame = plan->alg_flops;
  return NNA_OK;
}

nna_status nna_plan_sigma(const nna_plan* plan, double* host_out, size_t cap) {
  if (!plan || !host_out) return fail(NNA_ERR_INVALID_ARG, "plan / host_out is NULL");
  if (plan->kind != NNA_KIND_STFT) return fail(NNA_ERR_INVALID_ARG, "not an STFT plan");
  const int F = plan->stft_bins();
  if (cap < (size_t)F) return fail(NNA_ERR_INVALID_ARG, "host_out is too small");
  for (int k = 0; k < F; ++k) host_out[k] = plan->freq_scale ? plan->sigma[k] : (double)k;
  return NNA_OK;
}

nna_status nna_plan_cqt_lengths(const nna_plan* plan, long long* host_out, size_t cap) {
  if (!plan || !host_out) return fail(NNA_ERR_INVALID_ARG, "plan / host_out is NULL");
  if (plan->kind != NNA_KIND_CQT && plan->kind != NNA_KIND_CQT1992) return fail(NNA_ERR_INVALID_ARG, "not a CQT plan");
  if (cap < (size_t)plan->n_bins) return fail(NNA_ERR_INVALID_ARG, "host_out is too small");
  for (int k = 0; k < plan->n_bins; ++k) host_out[k] = plan->Nk[k];
  return NNA_OK;
}

void nna_plan_destroy(nna_plan* plan) {
  if (!plan) return;
  for (nna_plan* sub : plan->octave) nna_plan_destroy(sub);
  nna_plan_destroy(plan->fir);
  if (plan->device >= 0) {
    DeviceGuard guard;
    if (guard.enter(plan->device) == hipSuccess) {
      (void)hipFree(plan->d_bank);
      (void)hipFree(plan->d_bank16);
      (void)hipFree(plan->d_bankf);
      (void)hipFree(plan->d_fir_he);
      (void)hipFree(plan->d_fir_ho);
      (void)hipFree(plan->d_wn);
      (void)hipFree(plan->d_melwf);
      (void)hipFree(plan->d_mel_maskf);
      (void)hipFree(plan->d_bank16s);
      (void)hipFree(plan->d_wrm);
      (void)hipFree(plan->d_melw_rm);
      (void)hipFree(plan->d_melw);
      (void)hipFree(plan->d_mel_mask);
      (void)hipFree(plan->d_mel_wnyq);
      (void)hipFree(plan->d_mel_pass_rt);
      (void)hipFree(plan->d_items);
      (void)hipFree(plan->d_chunks);
      (void)hipFree(plan->d_cq_map);
      (void)hipFree(plan->d_row_lo);
      (void)hipFree(plan->d_row_hi);
      (void)hipFree(plan->d_bw_tiles);
      (void)hipFree(plan->d_shift_rng);
    }
  }
  delete plan;
}

const char* nna_status_str(nna_status s) {
  switch (s) {
    case NNA_OK: return "ok";
    case NNA_ERR_INVALID_ARG: return "invalid argument";
    case NNA_ERR_UNSUPPORTED: return "unsupported";
    case NNA_ERR_SHAPE: return "unusable batch shape";
    case NNA_ERR_ALLOC: return "allocation failed";
    case NNA_ERR_HIP: return "HIP runtime error";
  }
  return "unknown status";
}

const char* nna_last_error(void) { return g_err.c_str(); }

}  // extern "C"
