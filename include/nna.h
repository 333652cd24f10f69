/*
 * nna.h -- C ABI of the MI355X (gfx950) waveform -> spectrogram library.
 *
 * The library computes the transforms of arXiv 1912.12055 ("nnAudio") as strided
 * 1-D convolutions of a batch of waveforms with fixed kernel banks:
 *   STFT   windowed cos/sin DFT kernels, eq. (DFT2) and Sec. III-A
 *   Mel    triangular Mel filterbank applied to the STFT magnitude/power, Sec. III-B
 *   CQT    full-length time-domain complex constant-Q kernels ("CQT1992v2"),
 *          eqs. (Q), (N_k), (CQT) and Sec. III-C "CQT with time domain kernels"
 *
 * A plan (nna_plan_*) builds the kernel bank once on the host in double precision,
 * rounds it to float32 and uploads it in the tile order the GPU kernels read; the
 * paper calls this step initialisation and excludes it from its timings (Sec. IV-A).
 * A transform call (nna_stft / nna_mel / nna_cqt) enqueues one fused GPU kernel on
 * the caller's HIP stream.
 *
 * Conventions for every entry point
 *   - All arrays are contiguous, row-major float32.  x_dev is [B, L] (B waveforms of
 *     L samples); outputs are [B, bins, T] with the frame axis T fastest, in the
 *     same waveform order as the input (Sec. IV-A: "maintaining the order").
 *   - x_dev / out_dev are DEVICE pointers on the plan's device, owned by the caller.
 *     host_out of nna_plan_bank is a HOST pointer.
 *   - T = 1 + floor((L + 2*pad - K) / hop), K = n_fft or n_taps, pad = K/2 when
 *     center != 0 (mirror reflection that does not repeat the edge sample) else 0.
 *   - Transform calls allocate nothing, do not synchronise and return as soon as the
 *     kernel is enqueued on `hip_stream` (a hipStream_t cast to void*; NULL = the
 *     default stream).  Plans are immutable after creation and may be shared
 *     between threads (the one exception, nna_plan_set_bank, says so).
 *   - Every function returns an nna_status; on failure an output plan pointer is set
 *     to NULL and nna_last_error() describes the problem (thread-local text).  All
 *     argument, shape, capacity and workspace checks are made before anything is
 *     enqueued, so a call that fails them leaves the stream and the outputs alone.
 *     The calls that enqueue several kernels (nna_cqt2010v2, nna_cqt2010 and the
 *     *_backward calls) can still fail with NNA_ERR_HIP when the runtime itself
 *     rejects one of the later launches; the earlier kernels of that call are then
 *     already enqueued and the outputs and workspace hold unspecified values.
 *     Nothing throws or aborts across this boundary.
 *   - There is no CPU fallback: on a machine without a usable GPU plan creation for
 *     device >= 0 fails with NNA_ERR_HIP.  device == -1 builds a host-only plan that
 *     can be inspected (nna_out_shape, nna_plan_bank, nna_plan_info) but not run.
 */
#ifndef NNA_H
#define NNA_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct nna_plan nna_plan; /* opaque; owns the device kernel banks */

typedef enum {
  NNA_OK = 0,
  NNA_ERR_INVALID_ARG = 1, /* null pointer, out-of-range parameter, wrong plan kind */
  NNA_ERR_UNSUPPORTED = 2, /* valid request this build does not implement */
  NNA_ERR_SHAPE = 3,       /* B or L unusable with this plan (too short, too large) */
  NNA_ERR_ALLOC = 4,       /* host or device allocation failed */
  NNA_ERR_HIP = 5          /* a HIP runtime call failed (no device, launch error) */
} nna_status;

typedef enum {
  NNA_OUT_MAGNITUDE = 0, /* sqrt(Re^2 + Im^2) */
  NNA_OUT_POWER = 1,     /* Re^2 + Im^2 */
  NNA_OUT_LOG = 2,       /* ln(max(Re^2 + Im^2, 1e-10)): log compression, Fig. 1 caption */
  /* The transform itself, before the magnitude is taken (the output_format argument of the paper's
   * CQT layers, Sec. III-C): nna_stft (float32 plans) and the four constant-Q transforms (nna_cqt, nna_cqt1992,
   * nna_cqt2010, nna_cqt2010v2); not float16 plans. */
  NNA_OUT_COMPLEX = 3,   /* out[B, 2 bins, T]: row 2k = Re, row 2k+1 = Im of bin k (eq. (DFT2)'s signs: Im = -sum x sin) */
  NNA_OUT_PHASE = 4      /* atan2(Im, Re) in [-pi, pi] */
} nna_output;

typedef enum {       /* Sec. III-A names Hann, Hamming and Blackman; all in their periodic form */
  NNA_WIN_HANN = 0,     /* w[n] = 1/2 - 1/2 cos(2 pi n / N) */
  NNA_WIN_RECT = 1,
  NNA_WIN_HAMMING = 2,  /* 0.54 - 0.46 cos(2 pi n / N) */
  NNA_WIN_BLACKMAN = 3  /* 0.42 - 0.5 cos(2 pi n / N) + 0.08 cos(4 pi n / N) */
} nna_window;

typedef enum {
  NNA_MEL_SLANEY = 0, /* eq. (mel-stanley): linear below 1 kHz, logarithmic above */
  NNA_MEL_HTK = 1     /* eq. (mel-o): 2595 log10(1 + f/700) */
} nna_mel_scale;

typedef enum {
  NNA_FREQ_LINEAR = 1, /* eq. (linear-frequency-DFT): bins equally spaced in Hz from fmin */
  NNA_FREQ_LOG = 2     /* eq. (log-frequency-DFT): bins in geometric progression from fmin */
} nna_freq_scale;

typedef enum {
  NNA_PREC_F32 = 0, /* float32 operands, float32 accumulation */
  NNA_PREC_F16 = 1  /* bank and waveform rounded to float16 (to nearest even), float32 accumulation */
} nna_precision;

typedef enum {
  NNA_KIND_STFT = 0,
  NNA_KIND_MEL = 1,
  NNA_KIND_CQT = 2,
  NNA_KIND_CQT2010V2 = 3,
  NNA_KIND_CQT1992 = 4,
  NNA_KIND_CQT2010 = 5
} nna_kind;

/*
 * STFT plan (Sec. III-A; defaults of the paper's STFT layer: n_fft 2048, hop 512,
 * Hann, center, reflect).  Bank: rows Re_k[n] = w[n] cos(2 pi k n / N) and
 * Im_k[n] = -w[n] sin(2 pi k n / N), k = 0..N/2 (eq. (DFT2) with the window folded
 * into the kernels).  Output bins F = n_fft/2 + 1 (2F output rows for NNA_OUT_COMPLEX).
 *   sr     sample rate in Hz (kept for reporting; the DFT bank does not depend on it)
 *   n_fft  even, >= 8;  hop >= 1;  center 0/1;  device: HIP device index or -1.
 */
nna_status nna_plan_stft(nna_plan** plan, int sr, int n_fft, int hop, nna_window win, int center,
                         nna_output fmt, int device);

/*
 * nna_plan_stft with a choice of operand precision.  NNA_PREC_F16 runs the same contraction on
 * the float16 matrix instructions (16 times the float32 rate): the bank is rounded to float16
 * when the plan is built, the waveform when it is staged on chip; products are exact and sums
 * are float32, so the result differs from the float32 plan's by about 1e-5 of the spectrogram's
 * peak (bar: 1e-3).  It needs hop to divide n_fft at most 32 times and to be a multiple of 32
 * (NNA_ERR_UNSUPPORTED otherwise).  nna_plan_bank returns the bank as rounded.
 */
nna_status nna_plan_stft_prec(nna_plan** plan, int sr, int n_fft, int hop, nna_window win, int center,
                              nna_output fmt, nna_precision precision, int device);

/*
 * STFT plan on a re-spaced frequency axis (Sec. II-B; the freq_scale / fmin / fmax /
 * freq_bins arguments of the paper's STFT layer, Sec. III-A).  Bin k = 0..freq_bins-1 has
 * the normalised frequency
 *   linear: sigma(k) = (fmax - fmin) N / (freq_bins sr) k + fmin N / sr
 *   log:    sigma(k) = (fmin N / sr) (fmax / fmin)^(k / freq_bins)
 * and the bank rows are eq. (DFT3) with the window folded in:
 * Re_k[n] = w[n] cos(2 pi sigma(k) n / N), Im_k[n] = -w[n] sin(2 pi sigma(k) n / N).
 * Only the bank differs from nna_plan_stft; the plan runs through nna_stft.
 *   freq_bins  1..16384, or 0 for n_fft/2 + 1;  0 <= fmin < fmax <= sr/2 (log: fmin > 0).
 * Output bins = freq_bins.
 */
nna_status nna_plan_stft_scaled(nna_plan** plan, int sr, int n_fft, int hop, nna_window win, int center,
                                nna_output fmt, nna_freq_scale freq_scale, double fmin, double fmax,
                                int freq_bins, int device);

/*
 * Mel-spectrogram plan (Sec. III-B, Fig. 3): the STFT above followed, inside the same
 * kernel, by Mel[m,t] = sum_j W[m,j] |X_t[j]|^power.  W is the triangular filterbank
 * between n_mels+2 points equally spaced on the chosen mel scale from fmin to fmax
 * (fmax <= 0 means sr/2), evaluated at the bin frequencies j*sr/n_fft (eq.
 * (f-k-conversion)); norm_area != 0 scales filter m by 2/(f[m+2]-f[m]).
 * power must be 1 or 2.  Output bins = n_mels.
 */
nna_status nna_plan_mel(nna_plan** plan, int sr, int n_fft, int hop, nna_window win, int center,
                        int n_mels, double fmin, double fmax, nna_mel_scale scale, int norm_area,
                        double power, int device);

/*
 * Constant-Q plan with time-domain kernels (Sec. III-C).  Bin k has centre frequency
 * f_k = fmin 2^(k/b), Q = 1/(2^(1/b) - 1) cycles and length N_k = ceil(Q sr / f_k);
 * its kernel is window(N_k)[n] exp(-2 pi i Q n / N_k) / sum(window(N_k)) (L1 norm),
 * placed in taps [s_k, s_k + N_k), s_k = (n_taps - N_k) / 2 (integer division), of a
 * bank row of n_taps taps.  n_taps == 0 picks the next power of two >= N_0; n_taps
 * must be even and >= N_0, and the top bin must lie below sr/2.  Output bins = n_bins.
 * How nna_cqt evaluates eq. (CQT) is the plan's choice and changes no result beyond rounding:
 * the kernels are symmetric about their centres up to the common phase exp(-i pi Q), and where
 * that pays (a seventh or more of the multiply-adds saved: 12 or more bins per octave, kernels of
 * eight hops or more, hop a multiple of 16 dividing n_taps / 2, a window that vanishes at n = 0) they are
 * applied to the frame folded about that centre.  nna_plan_info reports the flops of the form
 * that runs; nna_plan_bank always returns the kernels as defined above.
 */
nna_status nna_plan_cqt(nna_plan** plan, int sr, int hop, double fmin, int n_bins, int bins_per_octave,
                        nna_window win, int center, int n_taps, nna_output fmt, int device);

/*
 * Constant-Q plan by recursive downsampling with time-domain kernels (Sec. III-C:
 * "Downsampling", "Constant-Q transform (2010 version)", "CQT with time domain kernels").
 * The bins are split into octaves from the top; octave a (0 = top) holds bins
 * [max(0, n_bins - (a+1) b), n_bins - a b).  Octave a is computed from the waveform
 * downsampled a times by two, with hop / 2^a and the kernels of nna_plan_cqt for the octave's
 * frequencies times 2^a (one kernel set when n_bins is a multiple of b), so every octave has
 * the frames of the top one: T = 1 + L / hop, always centred with mirror reflection.
 * Each downsampling step is y[m] = sum_i h[i] x~[2 m + i - (fir_taps-1)/2], x~ = x mirrored at
 * both ends, a length-L waveform giving ceil(L/2) samples; h is the window-method low-pass
 * named in "Downsampling" with its cutoff at half the Nyquist frequency (between the stated
 * pass-band end 0.4995 and stop-band start 0.5005), Hamming window, unit gain at 0 Hz.
 *   hop        a multiple of 2^(octaves-1)
 *   n_taps     0 = next power of two >= the longest top-octave kernel; else even and >= it
 *   fir_taps   0 = 257; else odd, 3..4095 (the paper gives no tap count)
 * Output bins = n_bins, lowest frequency first.
 * Waveform length: with l_0 = L, l_(a+1) = ceil(l_a / 2), every octave needs l_a > n_taps/2 (its mirror
 * reflection) and every octave but the lowest l_a >= fir_taps + 126 rounded up to a multiple of 128 (one
 * whole frame of the filter stage, 64 outputs: 384 samples for 257 taps); else NNA_ERR_SHAPE.
 */
nna_status nna_plan_cqt2010v2(nna_plan** plan, int sr, int hop, double fmin, int n_bins, int bins_per_octave,
                              nna_window win, int n_taps, int fir_taps, nna_output fmt, int device);

/*
 * Constant-Q plan with frequency-domain kernels (Sec. III-C "CQT using neural networks",
 * eqs. (Parseval), (CQT1992), Fig. 5; the paper's CQT1992 layer).  Two stages, run in one kernel:
 *   1. the un-windowed STFT X_t[k], k = 0..n_fft/2, of the waveform (the DFT bank of nna_plan_stft
 *      with a rectangular window; the constant-Q window lives in the kernels);
 *   2. X_cq[q, t] = (1/n_fft) sum_{k=0}^{n_fft/2} X_t[k] Y[q, k], followed by the output format.
 * Y[q, .] is the kernel of bin q -- that of nna_plan_cqt, centred in n_fft taps -- taken to the
 * frequency domain: Y[q, k] = conj(DFT(conj(kernel_q))[k]), the reading under which eq. (CQT1992)'s
 * two sides agree when k runs over all n_fft bins.  Only the half k <= n_fft/2 is kept, as in the
 * paper, so the result approximates nna_cqt's (to about 1e-4 of the peak for 12 bins per octave well
 * below the Nyquist frequency, a few 1e-3 for 6 bins per octave reaching 0.8 of it); no
 * sparsity threshold is applied to Y.  Cost per frame is that of an STFT with n_fft taps, for every
 * 64 constant-Q bins: the paper itself calls this form inefficient and offers it for research.
 *   n_fft  0 = the smallest power of two >= the longest kernel; else a power of two >= it, <= 65536
 * Output bins = n_bins; frames as for nna_plan_cqt with n_taps = n_fft.
 */
nna_status nna_plan_cqt1992(nna_plan** plan, int sr, int hop, double fmin, int n_bins, int bins_per_octave,
                            nna_window win, int center, int n_fft, nna_output fmt, int device);

/*
 * Constant-Q plan by recursive downsampling with frequency-domain kernels (Sec. III-C,
 * "Constant-Q transform (2010 version)", Fig. CQT2010; the paper's CQT2010 layer).  Octaves, bins per
 * octave, hop per octave, kernels, filter and frames are those of nna_plan_cqt2010v2; each octave is
 * computed as in nna_plan_cqt1992 -- un-windowed STFT of the (downsampled) waveform with n_fft taps,
 * times the octave's spectral kernels -- instead of with time-domain kernels.
 *   n_fft     0 = the smallest power of two >= the longest top-octave kernel; else a power of two >= it
 *   fir_taps  0 = 257; else odd, 3..4095
 * Runs through nna_cqt2010 with the workspace nna_cqt2010v2_workspace reports.
 */
nna_status nna_plan_cqt2010(nna_plan** plan, int sr, int hop, double fmin, int n_bins, int bins_per_octave,
                            nna_window win, int n_fft, int fir_taps, nna_output fmt, int device);

/* Output shape [B, *n_bins, *n_frames] for a batch of B waveforms of L samples.
 * NNA_ERR_SHAPE if L is too short (center: L <= pad; otherwise L < K; in any case L < 4) or B < 1. */
nna_status nna_out_shape(const nna_plan* plan, long long B, long long L, long long* n_bins,
                         long long* n_frames);

/* out_dev[B, F, T] = STFT of x_dev[B, L] in the plan's output format; F = n_fft/2+1 for a
 * plan from nna_plan_stft, freq_bins for one from nna_plan_stft_scaled.
 * A plan from nna_plan_stft (magnitude, power or log output, not made trainable) whose hop divides n_fft an
 * even number of times >= 4 and is a multiple of 32 is computed from the folded frame: the windows of Sec.
 * III-A satisfy w[n] = w[N-n], so eq. (DFT2)'s real kernels meet x[n] + x[N-n] and its imaginary kernels
 * x[n] - x[N-n] over n < N/2 only -- half the multiply-adds, the same result to rounding.  Where n_fft is also a
 * multiple of 256 the folded taps are summed by parity, E over even n and O over odd n: cos(2 pi (N/2 - k) n / N) =
 * (-1)^n cos(2 pi k n / N) (and -(-1)^n for the sine), so bin k is E + O and bin N/2 - k is E - O and only the kernels of
 * the bins below N/4 are multiplied -- a quarter of the direct form's multiply-adds.  Every other plan runs eq. (DFT2)
 * as it stands. */
nna_status nna_stft(const nna_plan* plan, const float* x_dev, long long B, long long L, float* out_dev,
                    void* hip_stream);

/* out_dev[B, n_mels, T] = Mel spectrogram of x_dev[B, L]; plan from nna_plan_mel.
 * The STFT itself is never written to memory.  Folded frames, split by tap parity where n_fft is a multiple of 128, as
 * for nna_stft, unless the plan was made trainable (a plan that is folded but not split also runs the direct form when
 * a filter has weight on bin n_fft/2). */
nna_status nna_mel(const nna_plan* plan, const float* x_dev, long long B, long long L, float* out_dev,
                   void* hip_stream);

/* nna_mel that also hands out the spectrogram its filterbank is applied to (Fig. 3: the STFT layer's
 * output feeding the Mel layer), from the one contraction: mel_dev[B, n_mels, T] as nna_mel writes it and
 * spec_dev[B, n_fft/2+1, T] = |X|^power (power 2: the power spectrogram; power 1: the magnitude).  For a
 * caller that wants both, this is one kernel launch of nna_mel's cost plus the spectrogram's stores (the first pass
 * of a plan with more than 128 filters then sweeps every bin; a plan that does not run split by tap parity takes the
 * direct contraction for this call).
 * Plan from nna_plan_mel (float32); errors as nna_mel, NNA_ERR_INVALID_ARG for a NULL spec_dev. */
nna_status nna_mel_with_stft(const nna_plan* plan, const float* x_dev, long long B, long long L,
                             float* mel_dev, float* spec_dev, void* hip_stream);

/* out_dev[B, n_bins, T] = constant-Q spectrogram of x_dev[B, L]; plan from nna_plan_cqt. */
nna_status nna_cqt(const nna_plan* plan, const float* x_dev, long long B, long long L, float* out_dev,
                   void* hip_stream);

/* out_dev[B, n_bins, T] = constant-Q spectrogram of x_dev[B, L]; plan from nna_plan_cqt1992.
 * The STFT itself is never written to memory. */
nna_status nna_cqt1992(const nna_plan* plan, const float* x_dev, long long B, long long L, float* out_dev,
                       void* hip_stream);

/* Bytes of device workspace nna_cqt2010v2 / nna_cqt2010 need for a batch [B, L]: the downsampled
 * waveforms of two consecutive octaves (about 3/4 of the input's size; 0 for a single octave).
 * Plans from nna_plan_cqt2010v2 and nna_plan_cqt2010. */
nna_status nna_cqt2010v2_workspace(const nna_plan* plan, long long B, long long L, size_t* bytes);

/* out_dev[B, n_bins, T] = constant-Q spectrogram of x_dev[B, L]; plan from nna_plan_cqt2010v2.
 * workspace_dev: caller-owned device memory, 16-byte aligned, of at least the size above; its
 * contents are overwritten and mean nothing afterwards.  Launches 2*octaves - 1 kernels (one constant-Q contraction per
 * octave, one decimation between octaves); nothing is allocated.  The decimations run on hip_stream; an octave's
 * contraction needs only that octave's waveform, so the contractions go to two streams the plan owns (created with the
 * plan, default priority), which wait for hip_stream's work queued before the call and for the decimation they need, and
 * which hip_stream waits for before the call returns: to the caller the call is one piece of work on hip_stream, and
 * under stream capture those streams join the capture and leave it again.  Calls on one plan from several host threads
 * enqueue one after the other (a lock in the plan).  NNA_ERR_SHAPE if some octave's waveform is not longer
 * than the kernels' half length n_taps/2 or shorter than the filter's frame (fir_taps + 126
 * samples, rounded up to a multiple of 128). */
nna_status nna_cqt2010v2(const nna_plan* plan, const float* x_dev, long long B, long long L, float* out_dev,
                         void* workspace_dev, size_t workspace_bytes, void* hip_stream);

/* nna_cqt2010v2 for callers that cannot allocate device memory for the workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid allocation.  Same plan, kernels and result as
 * nna_cqt2010v2; the downsampled waveforms go to a workspace of NNA_STATIC_SCRATCH_BYTES that is part of the
 * library's device image (every GPU the library runs on holds it until the process ends), so the call
 * itself allocates and frees nothing, on the host or the device.  NNA_ERR_SHAPE, with the sizes in
 * nna_last_error(), if the batch needs more than that (nna_cqt2010v2_workspace tells how much: about
 * 3 B L bytes, e.g. 126 waveforms of 176,400 samples).  All calls on one GPU share the one workspace, whose
 * contents mean nothing between calls (each call overwrites what it reads): two calls that overlap in
 * time on the same GPU -- from two streams or two threads -- race, and must be ordered by the caller. */
#define NNA_STATIC_SCRATCH_BYTES (64u << 20)
nna_status nna_cqt2010v2_static(const nna_plan* plan, const float* x_dev, long long B, long long L, float* out_dev,
                                void* hip_stream);

/* out_dev[B, n_bins, T] = constant-Q spectrogram of x_dev[B, L]; plan from nna_plan_cqt2010.
 * Workspace, launches (2*octaves - 1, of the STFT kernel and of the filter) and errors as for
 * nna_cqt2010v2; an octave's waveform must also be longer than n_fft/2. */
nna_status nna_cqt2010(const nna_plan* plan, const float* x_dev, long long B, long long L, float* out_dev,
                       void* workspace_dev, size_t workspace_bytes, void* hip_stream);

/*
 * Trainable Fourier kernels (Sec. IV-C, "Trainable Transformation Kernels"): the STFT layer's kernel
 * bank as a parameter that a training loop reads, updates and differentiates through.  Plans from
 * nna_plan_stft and nna_plan_stft_scaled (float32; for nna_plan_mel see the next group).  The bank's logical layout is the layer's weight
 * W[2 F, K], float32 row-major on the device: row 2k = real-part kernel, row 2k+1 = imaginary-part
 * kernel of bin k, K = n_fft taps, F = the plan's output bins.  For a plan from nna_plan_stft rows 1
 * and 2F-1 (the sine kernels of bins 0 and n_fft/2, identically zero in eq. (DFT2)) are not
 * parameters: they read as zero, writes to them are ignored and their gradient is zero -- which is
 * also what training would give, since d|X|/dIm = Im/|X| vanishes where Im is zero.  (With
 * NNA_OUT_COMPLEX the output rows these two kernels would produce are identically zero.)
 *
 * nna_plan_trainable  makes a plan trainable: allocates a second, row-major device copy of its bank
 *                     (the only allocation of this group; synchronises).  Idempotent.
 * nna_plan_get_bank   w_dev[2F, K] = the current bank.
 * nna_plan_set_bank   the bank = w_dev[2F, K] (after an optimiser step).  The plan is modified: no
 *                     transform using it may be in flight on another stream.  Kernels written here
 *                     need not be DFT kernels; nna_stft then computes out = format(C[2k]^2 + C[2k+1]^2),
 *                     C[r, t] = sum_n W[r, n] xp[t hop + n].
 * nna_stft_backward   given gout_dev[B, F, T] = dLoss/d(output of nna_stft for x_dev), writes
 *                     gw_dev[2F, K] = dLoss/dW and/or gx_dev[B, L] = dLoss/dx (either may be NULL):
 *                       G[r, f]  = dLoss/dC: gout times the output format's derivative -- magnitude
 *                                  Re/|X| (0 where |X| = 0), power 2 Re, log 2 Re/P where the power P
 *                                  exceeds the logarithm's floor (else 0); likewise Im;
 *                       gw[r, n] = sum over all frames f of G[r, f] xp[f hop + n];
 *                       gx[j]    = sum over all (t, n) whose padded sample t hop + n mirrors onto j
 *                                  of sum_r W[r, n] G[r, t].
 *                     Both outputs are overwritten (zeroed, then accumulated with float atomic adds:
 *                     the last bits may differ between runs).  workspace_dev: caller-owned device
 *                     memory, 256-byte aligned, of nna_stft_backward_workspace bytes (G itself:
 *                     128-row-padded bank rows x frames x 4 bytes); nothing is allocated, four to
 *                     six kernels are enqueued on hip_stream.  The forward pass is recomputed inside,
 *                     so nothing needs to be kept from nna_stft.
 * Errors: NNA_ERR_INVALID_ARG for a plan of another kind or one not made trainable, NULL pointers, a
 * small or misaligned workspace; NNA_ERR_UNSUPPORTED for float16 or host-only plans; NNA_ERR_SHAPE as
 * for nna_stft.
 */
nna_status nna_plan_trainable(nna_plan* plan);
nna_status nna_plan_get_bank(const nna_plan* plan, float* w_dev, void* hip_stream);
nna_status nna_plan_set_bank(nna_plan* plan, const float* w_dev, void* hip_stream);
nna_status nna_stft_backward_workspace(const nna_plan* plan, long long B, long long L, size_t* bytes);
nna_status nna_stft_backward(const nna_plan* plan, const float* x_dev, long long B, long long L,
                             const float* gout_dev, float* gw_dev, float* gx_dev, void* workspace_dev,
                             size_t workspace_bytes, void* hip_stream);

/*
 * Trainable constant-Q kernels (Sec. IV-C; the `trainable` argument of the paper's CQT layers, Sec.
 * III-C): nna_plan_trainable also accepts plans from nna_plan_cqt.  The bank's logical layout is
 * W[2 n_bins, n_taps], float32 row-major on the device: row 2k = real part, row 2k+1 = imaginary part of
 * the kernel eq. (CQT) multiplies the signal with, w_k[n] exp(-2 pi i Q n / N_k) / sum(w_k) (row 2k+1
 * starts out as the negative sine).  The parameters are the taps inside each kernel's support [s_k, s_k + N_k); the zeros
 * that centre the kernel among n_taps are structure, not parameters (the kernel that multiplies only
 * stored taps depends on it): they read as zero, writes to them are ignored, their gradient is zero.
 *   nna_plan_get_bank / nna_plan_set_bank   as above, with w_dev[2 n_bins, n_taps].
 *   nna_cqt_backward   given gout_dev[B, n_bins, T] ([B, 2 n_bins, T] for NNA_OUT_COMPLEX) = dLoss/d(output
 *                      of nna_cqt for x_dev), writes gw_dev[2 n_bins, n_taps] and/or gx_dev[B, L] with
 *                      the definitions given for nna_stft_backward (phase: d atan2(Im, Re) =
 *                      (Re dIm - Im dRe)/P; complex: G = gout).  workspace_dev: 256-byte aligned,
 *                      nna_cqt_backward_workspace bytes (G: 128-row-padded bank rows x padded frames x 4).
 *                      Outputs are overwritten; atomics and errors as in nna_stft_backward.
 */
nna_status nna_cqt_backward_workspace(const nna_plan* plan, long long B, long long L, size_t* bytes);
nna_status nna_cqt_backward(const nna_plan* plan, const float* x_dev, long long B, long long L,
                            const float* gout_dev, float* gw_dev, float* gx_dev, void* workspace_dev,
                            size_t workspace_bytes, void* hip_stream);

/*
 * Trainable kernels of the downsampling CQT with time-domain kernels (Sec. IV-C; the `trainable` argument of the
 * paper's CQT2010v2 layer, Sec. III-C "Downsampling"): nna_plan_trainable also accepts plans from
 * nna_plan_cqt2010v2.  The layer has ONE weight, the top octave's kernels W[2 n_top, n_taps] (n_top =
 * min(bins_per_octave, n_bins); rows and supports as for nna_plan_cqt with the top octave's bins): octave a
 * convolves the waveform downsampled a times with the same rows at hop / 2^a; a partial lowest octave of m < n_top
 * bins uses the rows of the upper m bins, 2 (n_top - m) onwards.  The decimation filter is not a parameter.
 *   nna_plan_get_bank / nna_plan_set_bank   w_dev[2 n_top, n_taps]; set rewrites every octave's copy.
 *   nna_cqt2010v2_backward   given gout_dev[B, n_bins, T] ([B, 2 n_bins, T] for NNA_OUT_COMPLEX) = dLoss/d(output of
 *                      nna_cqt2010v2 for x_dev), writes gw_dev[2 n_top, n_taps] = the sum over the octaves of each
 *                      octave's kernel gradient (definitions of nna_stft_backward, on that octave's waveform and
 *                      rows of gout) and/or gx_dev[B, L]: from the lowest octave up, the octave's own waveform
 *                      gradient plus the transposed decimation step (filter taps and mirror padding of the
 *                      forward step, transposed) applied to the gradient of the octave below.  The downsampled
 *                      waveforms are recomputed inside.  workspace_dev: 256-byte aligned,
 *                      nna_cqt2010v2_backward_workspace bytes (the octaves' waveforms, one octave's G, two
 *                      waveform gradients).  Outputs are overwritten; atomics as in nna_stft_backward; errors
 *                      as there and as for nna_cqt2010v2.  The deepest octaves (hop below 128) run the one-rate
 *                      layer's waveform-gradient kernel far below its best: correct, not tuned.
 */
nna_status nna_cqt2010v2_backward_workspace(const nna_plan* plan, long long B, long long L, size_t* bytes);
nna_status nna_cqt2010v2_backward(const nna_plan* plan, const float* x_dev, long long B, long long L,
                                  const float* gout_dev, float* gw_dev, float* gx_dev, void* workspace_dev,
                                  size_t workspace_bytes, void* hip_stream);

/*
 * Trainable kernels of the CQT layers with frequency-domain kernels (Sec. IV-C applied to Sec. III-C "CQT using neural
 * networks", eq. (CQT1992), and its downsampling form): nna_plan_trainable also accepts plans from nna_plan_cqt1992
 * and nna_plan_cqt2010 and makes both stages trainable.
 *   STFT stage: nna_plan_get_bank / nna_plan_set_bank with W[2F, n_fft], F = n_fft/2 + 1 (the un-windowed kernels of
 *     eq. (DFT2); rows 1 and 2F-1 are structural zeros as for nna_plan_stft).  A downsampling plan has one such bank,
 *     shared by its octaves.
 *   Spectral kernels: Ysk[2 n_bins, F], float32 row-major on the device, row 2q = Re, row 2q+1 = Im of Y[q, .]/n_fft
 *     (the layout of nna_plan_spectral_kernels): X_cq[q, t] = sum_k X_t[k] (Ysk[2q, k] + i Ysk[2q+1, k]).  For a
 *     plan from nna_plan_cqt2010: the top octave's kernels, n_bins -> n_top = min(bins_per_octave, n_bins), shared by
 *     the octaves as in nna_cqt2010v2_backward.  A trained matrix is dense: no block of the second contraction
 *     is skipped any more.
 *     nna_plan_get_spectral_kernels   y_dev[2 n_bins, F] = the current kernels.
 *     nna_plan_set_spectral_kernels   the kernels = y_dev (enqueued on hip_stream; the plan is modified).
 *   nna_cqt1992_backward / nna_cqt2010_backward   given gout_dev = dLoss/d(output of nna_cqt1992 / nna_cqt2010 for
 *     x_dev) ([B, n_bins, T], or [B, 2 n_bins, T] for NNA_OUT_COMPLEX), write any of
 *       gy_dev[2 n_bins, F]:  gV = gout times the output format's derivative at V = X_cq (as in nna_stft_backward);
 *                             dLoss/dRe Y[q,k] = sum (gVr Xr + gVi Xi), dLoss/dIm Y[q,k] = sum (gVi Xr - gVr Xi)
 *                             over waveforms and frames (X = Xr + i Xi the STFT stage's output);
 *       gw_dev[2F, n_fft] and gx_dev[B, L]: the gradient reaching the spectrum, gX = sum_q conj-transposed product
 *                             (gXr = gVr Yr + gVi Yi, gXi = gVi Yr - gVr Yi), carried through the STFT stage as
 *                             nna_stft_backward does for the complex output format;
 *     NULL pointers are skipped (at least one must be given).  The downsampling form sums gy and gw over the octaves
 *     and carries gx up through the transposed decimation steps.  workspace_dev: 256-byte aligned,
 *     nna_cqt1992_backward_workspace / nna_cqt2010_backward_workspace bytes (the spectrum [B, 2F, T] twice, the
 *     constant-Q values, the STFT stage's G; for nna_cqt2010 the octaves' waveforms and two waveform gradients).
 *     Outputs are overwritten; atomics, launches on hip_stream and errors as in nna_stft_backward.  The second
 *     stage's contractions run as plain tiled MFMA products bound by the [B, 2F, T] arrays they stream: correct,
 *     not tuned.
 */
nna_status nna_plan_get_spectral_kernels(const nna_plan* plan, float* y_dev, void* hip_stream);
nna_status nna_plan_set_spectral_kernels(nna_plan* plan, const float* y_dev, void* hip_stream);
nna_status nna_cqt1992_backward_workspace(const nna_plan* plan, long long B, long long L, size_t* bytes);
nna_status nna_cqt1992_backward(const nna_plan* plan, const float* x_dev, long long B, long long L, const float* gout_dev,
                                float* gy_dev, float* gw_dev, float* gx_dev, void* workspace_dev, size_t workspace_bytes,
                                void* hip_stream);
nna_status nna_cqt2010_backward_workspace(const nna_plan* plan, long long B, long long L, size_t* bytes);
nna_status nna_cqt2010_backward(const nna_plan* plan, const float* x_dev, long long B, long long L, const float* gout_dev,
                                float* gy_dev, float* gw_dev, float* gx_dev, void* workspace_dev, size_t workspace_bytes,
                                void* hip_stream);

/*
 * Trainable Mel layer (Sec. IV-C; the trainable_mel / trainable_STFT arguments of the paper's
 * MelSpectrogram layer, Sec. III-B): both stages of a plan from nna_plan_mel as parameters.
 * nna_plan_trainable also accepts Mel plans; nna_plan_get_bank / nna_plan_set_bank then address the
 * STFT stage's kernels W[2F, K] as above, and
 *   nna_plan_get_mel_weights / nna_plan_set_mel_weights   the filterbank Wmel[n_mels, F], float32
 *                      row-major on the device, F = n_fft/2 + 1.  Once a Mel plan is trainable its
 *                      filters are treated as dense (a trained filter is no triangle any more), which
 *                      costs nna_mel about 3 % more multiply-adds.
 *   nna_mel_backward   given gout_dev[B, n_mels, T] = dLoss/d(output of nna_mel for x_dev), writes any of
 *                        gmelw_dev[n_mels, F] = sum_{b,t} gout[b, m, t] P[b, k, t],  P = |X|^power,
 *                        gw_dev[2F, K] and gx_dev[B, L]: the gradient gP[b, k, t] = sum_m Wmel[m, k]
 *                        gout[b, m, t] reaching the STFT stage, carried on as in nna_stft_backward
 *                        (format power or magnitude according to the plan's `power`).
 *                      NULL pointers are skipped (at least one must be given).  workspace_dev: 256-byte
 *                      aligned, nna_mel_backward_workspace bytes (the spectrogram P, gP and the STFT
 *                      stage's G).  Outputs are overwritten; atomics as in nna_stft_backward.
 */
nna_status nna_plan_get_mel_weights(const nna_plan* plan, float* w_dev, void* hip_stream);
nna_status nna_plan_set_mel_weights(nna_plan* plan, const float* w_dev, void* hip_stream);
nna_status nna_mel_backward_workspace(const nna_plan* plan, long long B, long long L, size_t* bytes);
nna_status nna_mel_backward(const nna_plan* plan, const float* x_dev, long long B, long long L, const float* gout_dev,
                            float* gmelw_dev, float* gw_dev, float* gx_dev, void* workspace_dev,
                            size_t workspace_bytes, void* hip_stream);

/* Downsampling CQT plans only: *part = the plan of octave `index` (0 = top; a plan as from
 * nna_plan_cqt -- from nna_plan_cqt1992 for a plan made by nna_plan_cqt2010 -- for nna_plan_bank /
 * nna_plan_info / nna_plan_cqt_lengths / nna_plan_spectral_kernels), or with index -1 the
 * decimation filter, for inspection, as a bank of 64 rows: row r = the taps h shifted right by 2 r
 * (64 consecutive output samples per frame of 128 input samples).  The decimation itself runs on the
 * vector ALUs from the same taps split by the parity of their offset from the centre (a half-band design
 * is zero on the even offsets but for the centre: those are not multiplied).  The parts belong to `plan`. */
nna_status nna_plan_part(const nna_plan* plan, int index, const nna_plan** part);

/*
 * Inspection: the kernel bank exactly as the GPU holds it (float32 values widened to
 * double), un-permuted to the logical layout [rows, K] with row 2k = Re part and row
 * 2k+1 = Im part of bin k (rows = 2*(n_fft/2+1) for STFT/Mel, 2*n_bins for CQT;
 * K = n_fft or n_taps).  For a device plan the data is read back from device memory
 * (synchronous).  cap = capacity of host_out in doubles; NNA_ERR_INVALID_ARG if too
 * small.  The required size is returned by nna_plan_info (rows * K).
 */
nna_status nna_plan_bank(const nna_plan* plan, double* host_out, size_t cap);

/* Mel plans only: the filterbank W[n_mels, n_fft/2+1] as the GPU holds it. */
nna_status nna_plan_mel_weights(const nna_plan* plan, double* host_out, size_t cap);

/* Plans from nna_plan_cqt1992 only: the spectral kernels as the GPU holds them (float32 widened to
 * double, the factor 1/n_fft included), host_out[2 n_bins, n_fft/2+1] with row 2q = Re Y[q, .]/n_fft
 * and row 2q+1 = Im Y[q, .]/n_fft.  nna_plan_bank returns the plan's DFT bank, nna_plan_cqt_lengths
 * its kernel lengths. */
nna_status nna_plan_spectral_kernels(const nna_plan* plan, double* host_out, size_t cap);

/*
 * Plan facts, each written if its pointer is non-NULL: kind, logical bank rows (nna_plan_cqt2010v2: of the top
 * octave's kernels, which every octave uses; nna_plan_cqt2010: of the DFT bank its octaves share), taps K,
 * output bins, flops the kernels execute per frame (multiply-add = 2, zero-padded
 * taps they do not skip included) and algorithmic flops per frame (non-zero taps only:
 * 2*K*rows_nonzero for the DFT bank, 4*sum_k N_k for the CQT, plus 2*nnz(W) for Mel;
 * nna_plan_cqt1992: the DFT plus 8 per (constant-Q bin, kept DFT bin)).  The algorithmic figure of an
 * STFT or Mel plan is that of eq. (DFT2) taken directly, 2 K^2; a plan that runs folded frames (see
 * nna_stft) executes about half of it, K^2 + 2K.
 */
nna_status nna_plan_info(const nna_plan* plan, int* kind, long long* bank_rows, long long* taps,
                         long long* out_bins, double* executed_flops_per_frame,
                         double* algorithmic_flops_per_frame);

/* CQT plans (nna_plan_cqt, nna_plan_cqt1992) only: kernel lengths N_k, k = 0..n_bins-1 (host array of n_bins entries). */
nna_status nna_plan_cqt_lengths(const nna_plan* plan, long long* host_out, size_t cap);

/* STFT plans only: normalised bin frequencies sigma(k), k = 0..out_bins-1, in units of sr/n_fft
 * (host array; k itself for a plan from nna_plan_stft). */
nna_status nna_plan_sigma(const nna_plan* plan, double* host_out, size_t cap);

void nna_plan_destroy(nna_plan* plan); /* NULL is allowed */

const char* nna_status_str(nna_status s);
const char* nna_last_error(void); /* text of this thread's last failure, "" if none */

#ifdef __cplusplus
}
#endif
#endif /* NNA_H */
