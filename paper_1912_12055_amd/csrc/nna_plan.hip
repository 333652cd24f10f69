// Plans: argument checks, plan construction from the banks of nna_banks.hip and their upload, the inspection
// calls, destruction and error text of the C ABI.
#include "nna_host.h"

namespace nna {
namespace host {

thread_local std::string g_err;

nna_status fail(nna_status s, const std::string& msg) {
  g_err = msg;
  return s;
}

nna_status fail_hip(hipError_t e, const char* what) {
  g_err = std::string(what) + ": " + hipGetErrorString(e);
  return NNA_ERR_HIP;
}

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
      if (s == NNA_OK && p->fold_split) s = upload(&p->d_wq, p->h_wq.data(), p->h_wq.size() * sizeof(float), "weights of bin N/4");
      if (s == NNA_OK && mel && p->kind == NNA_KIND_MEL) {
        s = upload(&p->d_melwf, mel->fragf.data(), mel->fragf.size() * sizeof(float), "mel weights (folded kernel)");
        if (s == NNA_OK) s = upload(&p->d_mel_maskf, mel->maskf.data(), mel->maskf.size(), "mel mask (folded kernel)");
        if (s == NNA_OK && p->fold_split) {
          s = upload(&p->d_mel_pass_rtf, mel->pass_rtf.data(), mel->pass_rtf.size() * sizeof(int), "mel pass table (folded kernel)");
          if (s == NNA_OK) {
            std::vector<int> spec = mel->pass_rtf;
            spec[0] = 0;
            spec[1] = p->n_rt_split;
            s = upload(&p->d_mel_pass_rtf_spec, spec.data(), spec.size() * sizeof(int), "mel pass table (folded kernel)");
          }
          if (s == NNA_OK) s = upload(&p->d_mel_wq, mel->wq.data(), mel->wq.size() * sizeof(float), "mel weights of bin N/4");
        }
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
      if (s == NNA_OK && p->cq_fold) {
        s = upload(&p->d_bankq, p->h_bankq.data(), p->h_bankq.size() * sizeof(float), "folded cqt bank");
        if (s == NNA_OK) s = upload(&p->d_qitems, p->h_qitems.data(), p->h_qitems.size() * sizeof(nna::CqfItem), "folded cqt item table");
        if (s == NNA_OK) s = upload(&p->d_qchunks, p->h_qchunks.data(), p->h_qchunks.size() * sizeof(nna::CqfChunk), "folded cqt chunk table");
        if (s == NNA_OK) s = upload(&p->d_qbins, p->h_qbins.data(), p->h_qbins.size() * sizeof(int), "folded cqt bin table");
      }
    }
    if (s != NNA_OK) {
      const std::string keep = g_err;
      nna_plan_destroy(p);
      g_err = keep;
      return s;
    }
    std::vector<float>().swap(p->h_bank);  // the device copy is the bank from here on
    std::vector<float>().swap(p->h_bankf);
    std::vector<float>().swap(p->h_bankq);
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
    return fail(NNA_ERR_UNSUPPORTED, "the complex and phase outputs exist for the float32 STFT and the constant-Q transforms, not for float16 plans");
  }
  return fail(NNA_ERR_INVALID_ARG, "unknown output format");
}

nna_status check_stft_args(int n_fft) {
  if (n_fft < 8 || (n_fft & 1)) return fail(NNA_ERR_INVALID_ARG, "n_fft must be even and >= 8");
  if (n_fft > (1 << 20)) return fail(NNA_ERR_UNSUPPORTED, "n_fft above 2^20 is not supported");
  return NNA_OK;
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
    build_cqt_bank_fold(p);
  } catch (const std::bad_alloc&) {
    delete p;
    return fail(NNA_ERR_ALLOC, "out of host memory while building the CQT bank");
  }
  return finish_plan(p, plan, nullptr);
}

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
    build_fir_bank(p, fir_taps);
  } catch (const std::bad_alloc&) {
    delete p;
    return fail(NNA_ERR_ALLOC, "out of host memory while building the filter bank");
  }
  return finish_plan(p, plan, nullptr);
}

}  // namespace host
}  // namespace nna

using namespace nna::host;

// =======================================================================================
// C ABI: plan construction, inspection, destruction
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
  if ((s = check_cqt_args(fmin, n_bins, bins_per_octave, n_fft, fmt, sr, true)) != NNA_OK) return s;
  return make_cqt1992_plan(plan, sr, hop, fmin, 0, n_bins, bins_per_octave, win, center, n_fft, fmt, device);
}

// Both downsampling plans: one sub-plan per octave (time-domain kernels: a plan as from nna_plan_cqt;
// frequency-domain kernels: one as from nna_plan_cqt1992) and the decimation filter.
static nna_status make_downsampling_plan(int kind, nna_plan** plan, int sr, int hop, double fmin, int n_bins,
                                         int bins_per_octave, nna_window win, int n_taps, int fir_taps, nna_output fmt,
                                         int device) {
  nna_status s = check_common(plan, sr, hop, win, 1, device);
  if (s != NNA_OK) return s;
  if ((s = check_cqt_args(fmin, n_bins, bins_per_octave, n_taps, fmt, sr, true)) != NNA_OK) return s;
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
  if (device >= 0 && n_oct > 1) {
    // streams at the default priority; events carry no timestamps
    DeviceGuard guard;
    hipError_t e = guard.enter(device);
    for (int i = 0; i < 2 && e == hipSuccess; ++i) e = hipStreamCreateWithFlags(&p->oct_stream[i], hipStreamNonBlocking);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&p->ev_fork, hipEventDisableTiming);
    for (int a = 0; a < n_oct && e == hipSuccess; ++a) {
      e = hipEventCreateWithFlags(&p->ev_fir[a], hipEventDisableTiming);
      if (e == hipSuccess) e = hipEventCreateWithFlags(&p->ev_oct[a], hipEventDisableTiming);
    }
    if (e != hipSuccess) {
      nna_plan_destroy(p);
      return fail_hip(e, "stream / event creation");
    }
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
    *bank_rows = plan->kind == NNA_KIND_CQT2010   ? 2LL * (plan->octave[0]->n_half + 1)   // the DFT bank all octaves share
                 : plan->kind == NNA_KIND_CQT2010V2 ? (long long)plan->octave[0]->conv_rows  // the one weight all octaves share
                 : plan->kind == NNA_KIND_CQT     ? (long long)plan->conv_rows
                                                  : 2LL * (plan->freq_scale ? plan->n_half : plan->n_half + 1);
  if (taps) *taps = plan->K;
  if (out_bins) *out_bins = plan->out_rows();
  if (executed_flops_per_frame)
    *executed_flops_per_frame = plan->runs_split()    ? plan->exec_flops_split
                                : plan->runs_folded() ? plan->exec_flops_fold
                                : plan->runs_cqfold() ? plan->exec_flops_cqf
                                                      : plan->exec_flops;
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
      for (hipStream_t st : plan->oct_stream)
        if (st) {
          (void)hipStreamSynchronize(st);
          (void)hipStreamDestroy(st);
        }
      if (plan->ev_fork) (void)hipEventDestroy(plan->ev_fork);
      for (hipEvent_t ev : plan->ev_fir)
        if (ev) (void)hipEventDestroy(ev);
      for (hipEvent_t ev : plan->ev_oct)
        if (ev) (void)hipEventDestroy(ev);
      (void)hipFree(plan->d_bank);
      (void)hipFree(plan->d_bank16);
      (void)hipFree(plan->d_bankf);
      (void)hipFree(plan->d_fir_he);
      (void)hipFree(plan->d_fir_ho);
      (void)hipFree(plan->d_wn);
      (void)hipFree(plan->d_wq);
      (void)hipFree(plan->d_mel_pass_rtf);
      (void)hipFree(plan->d_mel_pass_rtf_spec);
      (void)hipFree(plan->d_mel_wq);
      (void)hipFree(plan->d_melwf);
      (void)hipFree(plan->d_mel_maskf);
      (void)hipFree(plan->d_bank16s);
      (void)hipFree(plan->d_wrm);
      (void)hipFree(plan->d_melw_rm);
      (void)hipFree(plan->d_ysk);
      (void)hipFree(plan->d_ylin);
      (void)hipFree(plan->d_ylinT);
      (void)hipFree(plan->d_melw);
      (void)hipFree(plan->d_mel_mask);
      (void)hipFree(plan->d_mel_wnyq);
      (void)hipFree(plan->d_mel_pass_rt);
      (void)hipFree(plan->d_items);
      (void)hipFree(plan->d_chunks);
      (void)hipFree(plan->d_bankq);
      (void)hipFree(plan->d_qitems);
      (void)hipFree(plan->d_qchunks);
      (void)hipFree(plan->d_qbins);
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
