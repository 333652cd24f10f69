// Running a plan: shape checks, launch parameters and the transform calls of the C ABI, the per-device
// set-up, and the library's static workspace with the entry point that uses it.
#include "nna_host.h"

// Workspace of nna_cqt2010v2_static: the downsampled waveforms of two consecutive octaves live here instead
// of in caller memory.  Every device the library's code is loaded on holds its own copy of the array, at its
// own address; in host code the name is only a handle for hipGetSymbolAddress, never a device address.
static __device__ __align__(256) unsigned char scratch[NNA_STATIC_SCRATCH_BYTES];

namespace nna {
namespace host {

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
    if (e == hipSuccess) e = nna::cqf_kernels_init();
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
// caller).  out_wave_stride / row_offset place a two-stage CQT plan's rows inside a larger output
// (octave of a downsampling plan); 0 / 0 = the plan's own [B, bins, T].
nna_status run_stft_core(const nna_plan* plan, int kind, const float* x, long long B, long long L, long long T,
                         float* out, long long out_wave_stride, int row_offset, void* stream, float* spec_out = nullptr) {
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
  // (chunks visited in pairs: a tile also holds the mirrored partners' rows, J/2 further on)
  const bool fold_pair = plan->runs_split() && plan->fold_pair;
  const int fold_M = plan->runs_folded() ? pick_tile_frames(ST_FRAMES, T, fold_pair ? plan->nj - 1 : plan->nj / 2 - 1, nna::SF_LDS_ROWS) : 0;
  const bool fold_fits = fold_M >= 1 && (1 + (fold_M - 1 + T - 1) / T) * L <= (1LL << 29);
  // (the Mel launch split by tap parity can write the spectrogram it forms on the way; the once-folded one cannot)
  if (fold_fits && (!spec_out || (kind == NNA_KIND_MEL && plan->runs_split())) && (kind == NNA_KIND_STFT || kind == NNA_KIND_MEL)) {
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
      if (plan->runs_split()) {  // 32-bin row tiles below N/4, their own pass table; bin N/4 weighed in at the end
        P.split = 1;
        P.pair = plan->fold_pair ? 1 : 0;
        P.n_rt = plan->n_rt_split;
        P.mel_pass_rt = plan->d_mel_pass_rtf;
        P.wn = plan->d_wq;
        P.mel_wnyq = plan->d_mel_wq;
        P.mel_nyq_any = plan->mel_q_any;
        if (spec_out) {
          P.pout = spec_out;
          P.mel_pass_rt = plan->d_mel_pass_rtf_spec;
        }
      }
    } else {
      P.out_bins = plan->n_half + 1;
      P.fmt = plan->fmt;
      if (plan->runs_split()) {  // the bins below N/4 only; bin N/4 from the workgroups behind the contraction's
        P.split = 1;
        P.pair = plan->fold_pair ? 1 : 0;
        P.n_rt = plan->n_rt_split;
        P.wn = plan->d_wq;
      }
      const long long ft_per_xcd = (P.n_ft + 7) / 8;
      P.main_blocks = 8 * ((ft_per_xcd + 63) / 64) * 64 * ((P.n_rt + nna::ST_RG - 1) / nna::ST_RG);
    }
    DeviceGuard guard;
    hipError_t e = guard.enter(plan->device);
    if (e != hipSuccess) return fail_hip(e, "hipSetDevice");
    e = nna::launch_stft_fold(P, kind == NNA_KIND_MEL ? nna::ST_MODE_MEL : nna::ST_MODE_STFT, reinterpret_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail_hip(e, "kernel launch");
    return NNA_OK;
  }
  const bool cplx = kind == NNA_KIND_STFT && (plan->fmt == NNA_OUT_COMPLEX || plan->fmt == NNA_OUT_PHASE);
  int lds_rows = kind == NNA_KIND_CQT1992 && plan->lin_blocks == 6 ? nna::ST_LDS_ROWS_WIDE : ST_LDS_ROWS;
  // complex / phase output with many hop-shifts: the one-workgroup-per-CU build when its 192-row tile holds more than
  // 8/7 of the frames the 160-row tile does
  const bool wide = cplx && pick_tile_frames(ST_FRAMES, T, plan->nj - 1, nna::ST_LDS_ROWS_WIDE) * 7 >
                                pick_tile_frames(ST_FRAMES, T, plan->nj - 1, ST_LDS_ROWS) * 8;
  if (wide) lds_rows = nna::ST_LDS_ROWS_WIDE;
  const int M = pick_tile_frames(ST_FRAMES, T, plan->nj - 1, lds_rows);
  if (M < 1) return fail(NNA_ERR_UNSUPPORTED, "frame tile does not fit in LDS");
  nna::StftParams P;
  std::memset(&P, 0, sizeof(P));
  P.wide = wide ? 1 : 0;
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
    P.out_wave_stride = out_wave_stride > 0 ? out_wave_stride : (long long)plan->out_rows() * T;
    P.row_offset = row_offset;
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

// the kernels folded about their centres (nna_kernels_cqf.hip): M frames per tile
nna_status run_conv_fold(const nna_plan* sub, const float* x, long long B, long long L, long long T, float* out,
                         long long out_wave_stride, int row_offset, int M, void* hip_stream) {
  nna::CqfParams P;
  std::memset(&P, 0, sizeof(P));
  P.g = make_geom(sub, x, B, L, T);
  P.bank = reinterpret_cast<const float4*>(sub->d_bankq);
  P.items = sub->d_qitems;
  P.chunks = sub->d_qchunks;
  P.bins = sub->d_qbins;
  P.out = out;
  P.out_wave_stride = out_wave_stride;
  P.row_offset = row_offset;
  P.n_items = (int)sub->h_qitems.size();
  P.n_chunks = sub->q_n_chunks;
  P.fmt = sub->fmt;
  P.tile_frames = M;
  const int extra = sub->q_max_jspan - 1;
  const long long nseg = 1 + (M - 1 + T - 1) / T;
  P.lds_rows = (int)((M + nseg * extra + 63) / 64 * 64);
  P.centre = sub->K / 2;
  const double turn = std::fmod(sub->Q, 2.0);
  P.rot_c = (float)std::cos(kPi * turn);
  P.rot_s = (float)std::sin(kPi * turn);
  P.n_ft = (P.g.n_frames + M - 1) / M;
  hipError_t e = nna::launch_cqt_fold(P, reinterpret_cast<hipStream_t>(hip_stream));
  if (e != hipSuccess) return fail_hip(e, "kernel launch");
  return NNA_OK;
}

// one launch of the CQT kernel: `sub`'s bank over T frames of each of the B waveforms in x
nna_status run_conv(const nna_plan* sub, const float* x, long long B, long long L, long long T, float* out,
                    long long out_wave_stride, int row_offset, void* hip_stream, bool may_fold = false) {
  const int extra = (sub->max_jspan - 1) * sub->row_step;
  const int M = pick_tile_frames(CQ_FRAMES, T, extra, CQ_LDS_ROWS_MAX);
  if (may_fold && sub->runs_cqfold()) {
    // the folded kernel does half the work per frame; its tiles hold fewer rows, so batches of very short
    // waveforms (many waveform segments, each with its overlap rows, in one tile) can leave it the smaller tile
    const int Mf = pick_tile_frames(CQ_FRAMES, T, sub->q_max_jspan - 1, nna::CQF_LDS_ROWS);
    if (Mf >= 1 && 2 * Mf >= M) return run_conv_fold(sub, x, B, L, T, out, out_wave_stride, row_offset, Mf, hip_stream);
  }
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
  P.row_offset = row_offset;
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

inline size_t ws_round(long long floats) { return ((size_t)floats * sizeof(float) + 255) / 256 * 256; }

// lengths of the waveform at every octave; false if some octave is too short for its padding
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

}  // namespace host
}  // namespace nna

using namespace nna::host;

// =======================================================================================
// C ABI: transforms
// =======================================================================================
extern "C" {

nna_status nna_cqt1992(const nna_plan* plan, const float* x_dev, long long B, long long L, float* out_dev, void* hip_stream) {
  return run_stft_like(plan, NNA_KIND_CQT1992, x_dev, B, L, out_dev, hip_stream);
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
  // The filter chain x_0 -> x_1 -> ... runs on the caller's stream; octave a's kernels need x_a only and go to one of the
  // plan's two streams (even / odd octaves), so they run beside the next filter steps and beside each other: the
  // filter is bound by the vector ALUs, the octaves' kernels by the matrix pipe, and the deep octaves' launches are too
  // small to fill the chip alone.  Every stream is back on the caller's before the call returns, so the call still
  // is one piece of work on that stream (under stream capture: a fork and a join).
  hipStream_t main_stream = static_cast<hipStream_t>(hip_stream);
  const bool forked = n_oct > 1 && plan->oct_stream[0] != nullptr;
  std::unique_lock<std::mutex> lock(plan->oct_mutex, std::defer_lock);
  if (forked) {
    lock.lock();
    if ((e = hipEventRecord(plan->ev_fork, main_stream)) != hipSuccess) return fail_hip(e, "hipEventRecord");
    for (hipStream_t st : plan->oct_stream)
      if ((e = hipStreamWaitEvent(st, plan->ev_fork, 0)) != hipSuccess) return fail_hip(e, "hipStreamWaitEvent");
  }
  int launched = 0;  // octaves whose kernels were enqueued on the plan's streams
  // the caller's stream waits for the last octave enqueued on each of the plan's streams (also on an error path)
  auto join = [&]() -> hipError_t {
    hipError_t r = hipSuccess;
    for (int a = std::max(0, launched - 2); a < launched; ++a) {
      const hipError_t w = hipStreamWaitEvent(main_stream, plan->ev_oct[a], 0);
      if (r == hipSuccess) r = w;
    }
    return r;
  };
  const float* cur = x_dev;
  for (int a = 0; a < n_oct; ++a) {
    int lo, hi;
    octave_bins(plan->n_bins, plan->bpo, a, lo, hi);
    // the octave's rows inside each waveform's output (the complex format writes two rows per bin)
    const int row0 = plan->fmt == NNA_OUT_COMPLEX ? 2 * lo : lo;
    hipStream_t st = forked ? plan->oct_stream[a & 1] : main_stream;
    if (forked && a >= 1 && (e = hipStreamWaitEvent(st, plan->ev_fir[a], 0)) != hipSuccess) {  // x_a is complete
      (void)join();
      return fail_hip(e, "hipStreamWaitEvent");
    }
    if (kind == NNA_KIND_CQT2010V2)
      s = run_conv(plan->octave[a], cur, B, La[a], T, out_dev, (long long)plan->out_rows() * T, row0, st);
    else
      s = run_stft_core(plan->octave[a], NNA_KIND_CQT1992, cur, B, La[a], T, out_dev, (long long)plan->out_rows() * T, row0, st);
    if (forked) {
      e = hipEventRecord(plan->ev_oct[a], st);
      if (e == hipSuccess) launched = a + 1;
      if (s == NNA_OK && e != hipSuccess) s = fail_hip(e, "hipEventRecord");
    }
    if (s != NNA_OK) {
      if (forked) (void)join();
      return s;
    }
    if (a + 1 < n_oct) {
      float* dst = buf[a & 1];
      const long long Ln = La[a + 1];
      // dst held x_(a-1): octave a-1 must have read it
      if (forked && a >= 2 && (e = hipStreamWaitEvent(main_stream, plan->ev_oct[a - 1], 0)) != hipSuccess) {
        (void)join();
        return fail_hip(e, "hipStreamWaitEvent");
      }
      s = run_fir(plan->fir, cur, B, La[a], dst, Ln, main_stream);
      if (s == NNA_OK && forked && (e = hipEventRecord(plan->ev_fir[a + 1], main_stream)) != hipSuccess)
        s = fail_hip(e, "hipEventRecord");
      if (s != NNA_OK) {
        if (forked) (void)join();
        return s;
      }
      cur = dst;
    }
  }
  if (forked && (e = join()) != hipSuccess) return fail_hip(e, "hipStreamWaitEvent");
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

nna_status nna_out_shape(const nna_plan* plan, long long B, long long L, long long* n_bins, long long* n_frames) {
  if (!plan) return fail(NNA_ERR_INVALID_ARG, "plan is NULL");
  if (B < 1) return fail(NNA_ERR_SHAPE, "B must be >= 1");
  if (plan->kind == NNA_KIND_CQT2010V2 || plan->kind == NNA_KIND_CQT2010) {
    long long La[MAX_OCTAVES];
    if (L < 1 || !cqt2010_lengths(plan, L, La))
      return fail(NNA_ERR_SHAPE, "L is too short: every octave's waveform must exceed the reflection padding, and all but the lowest hold one frame of the decimation filter");
    if (n_bins) *n_bins = plan->out_rows();
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
  return run_conv(plan, x_dev, B, L, T, out_dev, (long long)plan->out_rows() * T, 0, hip_stream, true);
}
}  // extern "C"
