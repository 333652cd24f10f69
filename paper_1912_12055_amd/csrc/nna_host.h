// Host-side declarations shared by the translation units of the library's host code: the plan object,
// error reporting, device helpers, and the functions each file offers the others.  Nothing here is part of
// the C ABI.
//   nna_banks.hip     kernel banks built in double precision and laid out in streaming order
//   nna_plan.hip      plan constructors, inspection calls, destruction (C ABI)
//   nna_run.hip       transform calls (C ABI), per-device set-up, the library's static workspace
//   nna_backward.hip  trainable plans and the backward calls (C ABI)
#pragma once

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
  // Device plans with more than one octave: two streams of their own and the events that order a call's launches
  // across them (the filter chain stays on the caller's stream, the octaves' kernels go to the two others in turn);
  // created with the plan, so that a call allocates nothing.  oct_mutex: one call enqueues at a time.
  static constexpr int OCT_EVENTS = 16;  // = MAX_OCTAVES
  hipStream_t oct_stream[2] = {nullptr, nullptr};
  hipEvent_t ev_fork = nullptr;
  hipEvent_t ev_fir[OCT_EVENTS] = {};
  hipEvent_t ev_oct[OCT_EVENTS] = {};
  mutable std::mutex oct_mutex;
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
  // STFT plans whose n_fft is a multiple of 256 and whose hop is even: the folded contraction split once more by tap
  // parity (bins below N/4 only; their partners N/2 - k from the same sums).  h_wq / d_wq: the two weight tables of
  // bin N/4, [2][J rounded up to 4][hop]
  bool fold_split = false;
  // ... with its chunks visited in pairs c, n_chunks - 1 - c: each chunk's tile then holds the other's mirrored partners
  // (J = 4 and an even number of chunks; the folded bank is stored in the visiting order)
  bool fold_pair = false;
  double exec_flops_split = 0;
  std::vector<float> h_wq;
  float* d_wq = nullptr;
  bool runs_split() const { return runs_folded() && fold_split; }
  // Mel plans that run split: the split kernel's own pass table, the filters' weights on bin N/4 (all zero: mel_q_any = 0)
  int* d_mel_pass_rtf = nullptr;
  int* d_mel_pass_rtf_spec = nullptr;  // the same with the first pass sweeping every tile (nna_mel_with_stft)
  float* d_mel_wq = nullptr;
  int mel_q_any = 0;
  int n_rt_split = 0;  // row tiles of the split launch (STFT: 64 bins each, Mel: 32)

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
  // trainable plans with frequency-domain constant-Q kernels: the spectral kernels as the caller's tensor
  // Ysk[2 n_bins][n_half + 1] (row 2q = Re, 2q+1 = Im, 1/n_fft included), and the real matrix they form on the
  // (Re, Im) rows of a spectrum, row-major both ways round, zero padded: Ylin[lin_mp][lin_rp], YlinT[lin_rp][lin_mp]
  // (lin_mp = 2 n_bins, lin_rp = 2 (n_half + 1), each rounded up to 128)
  float* d_ysk = nullptr;
  float* d_ylin = nullptr;
  float* d_ylinT = nullptr;
  int lin_mp = 0, lin_rp = 0;
  float* d_melw = nullptr;
  unsigned char* d_mel_mask = nullptr;
  float* d_mel_wnyq = nullptr;
  int* d_mel_pass_rt = nullptr;
  nna::CqtItem* d_items = nullptr;
  nna::CqtChunk* d_chunks = nullptr;
  // Constant-Q kernels folded about their centres (nna_kernels_cqf.hip): one-rate plans with time-domain kernels
  // whose kernels are mirror symmetric up to one common phase and span at least eight hops.  The direct bank stays
  // (inspection, trainable plans).
  bool cq_fold = false;
  std::vector<nna::CqfItem> h_qitems;
  std::vector<nna::CqfChunk> h_qchunks;  // [item][q_n_chunks]
  std::vector<int> h_qbins;              // [group][16]
  std::vector<float> h_bankq;
  int q_n_chunks = 1, q_max_jspan = 1;
  double exec_flops_cqf = 0;
  float* d_bankq = nullptr;
  nna::CqfItem* d_qitems = nullptr;
  nna::CqfChunk* d_qchunks = nullptr;
  int* d_qbins = nullptr;
  bool runs_cqfold() const { return cq_fold && !d_wrm; }
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

namespace nna {
namespace host {

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

constexpr double kPi = 3.141592653589793238462643383279502884;

// ---- error reporting (nna_plan.hip): the text nna_last_error() returns, per thread ------------------
extern thread_local std::string g_err;
nna_status fail(nna_status s, const std::string& msg);
nna_status fail_hip(hipError_t e, const char* what);

// ---- device helpers -------------------------------------------------------------------------------
hipError_t ensure_kernels_init(int device);  // nna_run.hip: per-device set-up, once per device (that device current)
void* scratch_of(int device);                // nna_run.hip: the device's copy of the static workspace, or NULL
nna_status check_device(int device);

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

// ---- kernel banks (nna_banks.hip) --------------------------------------------------------------------
double window_value(int win, long long n, long long N);
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

// tap index of (chunk c, shift j, fragment kg, lane half h, element e)
inline int stft_tap(const nna_plan* p, int c, int j, int kg, int h, int e) {
  return j * p->hop + c * ST_KC + kg * ST_KG + 4 * h + e;
}

struct MelDeviceLayout {
  std::vector<float> fragf;         // folded kernel: [pass][rt][blk 2][mb][4][64][4]
  std::vector<unsigned char> maskf; // folded kernel: [pass][rt][blk 2]
  double exec_blocks_f = 0;
  std::vector<float> frag;          // [pass][rt][rb][mb][2][64][4]
  std::vector<unsigned char> mask;  // [pass][rt][rb]
  std::vector<float> wnyq;          // [n_mels]
  std::vector<int> pass_rt;         // [pass][2]
  // split form of the folded kernel (32-bin row tiles, blk 0 = the tile's bins, blk 1 = their partners N/2 - k): fragf /
  // maskf in that layout, the row tile range of every pass, the filters' weights on bin N/4
  std::vector<int> pass_rtf;        // [pass][2]
  std::vector<float> wq;            // [n_mels]
};

// index of (pass, row tile, row block, out block, quad v, lane, element e) in the fragment array of
// the second contraction, and the matrix entry it holds: output row pass*128 + mb*32 + lane%32,
// packed row rt*128 + rb*32 + 8 v + 4 (lane/32) + e
inline size_t lin_frag_index(const nna_plan* p, int pass, int rt, int rb, int mb, int v, int lane, int e) {
  return ((((((size_t)pass * p->n_rt + rt) * ST_RB + rb) * p->lin_blocks + mb) * 4 + v) * 64 + lane) * 4 + e;
}

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

void build_stft_bank(nna_plan* p);
void build_stft_bank_fold(nna_plan* p);
bool build_stft_bank_f16(nna_plan* p);
void build_mel_weights(nna_plan* p, double fmin, double fmax, int scale, int norm_area);
MelDeviceLayout layout_mel(nna_plan* p);
void build_cqt1992_matrix(nna_plan* p);
MelDeviceLayout layout_cqt1992(nna_plan* p);
void build_cqt_bank(nna_plan* p);
void build_cqt_bank_fold(nna_plan* p);  // sets p->cq_fold if the plan qualifies
// the decimation filter of `fir_taps` taps: its taps, their split by parity for the decimation kernel, and the
// 64-row bank form kept for inspection
constexpr int FIR_ROWS = CQ_ITEM_RB * CQ_ROWS;
constexpr int FIR_HOP = 2 * FIR_ROWS;
void build_fir_bank(nna_plan* p, int fir_taps);

// ---- plans (nna_plan.hip) ---------------------------------------------------------------------------------
nna_status finish_plan(nna_plan* p, nna_plan** out, const MelDeviceLayout* mel);

// ---- running a plan (nna_run.hip) -------------------------------------------------------------------------
long long frames_of(const nna_plan* p, long long L);
int pick_tile_frames(int cap, long long T, int extra, int rows_max);
nna_status check_call(const nna_plan* plan, int kind, const float* x, long long B, long long L, float* out, long long* T_out);
nna::FrameGeom make_geom(const nna_plan* p, const float* x, long long B, long long L, long long T);
constexpr int MAX_OCTAVES = 16;
static_assert(MAX_OCTAVES == nna_plan::OCT_EVENTS, "one event per octave");
inline int octaves_of(int n_bins, int bpo) { return (n_bins + bpo - 1) / bpo; }
inline void octave_bins(int n_bins, int bpo, int a, int& lo, int& hi) {
  hi = n_bins - a * bpo;
  lo = std::max(0, hi - bpo);
}
bool cqt2010_lengths(const nna_plan* plan, long long L, long long (&La)[MAX_OCTAVES]);
// one decimation step: y[B, Ln] from x[B, L], Ln = ceil(L / 2) (arguments checked by the caller)
nna_status run_fir(const nna_plan* fir, const float* x, long long B, long long L, float* y, long long Ln, void* hip_stream);

}  // namespace host
}  // namespace nna
