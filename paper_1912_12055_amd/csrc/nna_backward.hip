// Trainable plans (Sec. IV-C): the bank as a parameter the caller reads and writes, and the backward calls of
// the STFT, Mel and one-rate constant-Q layers (C ABI).
#include "nna_host.h"

using namespace nna::host;

extern "C" {

// ---- trainable Fourier kernels (Sec. IV-C) ----------------------------------------------------
static nna_status check_trainable_kind(const nna_plan* plan) {
  if (!plan) return fail(NNA_ERR_INVALID_ARG, "plan is NULL");
  if (plan->kind < NNA_KIND_STFT || plan->kind > NNA_KIND_CQT2010) return fail(NNA_ERR_INVALID_ARG, "unknown kind of plan");
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
    // waveform gradient: how many rows (in chunks of CW_KC; rows are ordered longest first) hold taps on each
    // 128-tap tile, and from that, per 128-column tile of the hop, the running count over the hop-shifts
    for (int nt = 0; nt < n_nt; ++nt) {
      int r_max = 0;
      for (int r = 0; r < rows; ++r)
        if (plan->row_s[r] < (long long)(nt + 1) * nna::BW_NT && plan->row_e[r] > (long long)nt * nna::BW_NT) r_max = r + 1;
      nt_chunks[nt] = (r_max + nna::CW_KC - 1) / nna::CW_KC;
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

static bool is_trainable(const nna_plan* plan) {
  if (plan->kind == NNA_KIND_CQT1992) return plan->d_wrm != nullptr && plan->d_ysk != nullptr;
  if (plan->kind != NNA_KIND_CQT2010V2 && plan->kind != NNA_KIND_CQT2010) return plan->d_wrm != nullptr;
  for (const nna_plan* sub : plan->octave)
    if (!is_trainable(sub)) return false;
  return true;
}

static nna::LinLogicalParams lin_logical_params(const nna_plan* plan, const float* ysk) {
  nna::LinLogicalParams q;
  q.ysk = ysk;
  q.frag = plan->d_melw;
  q.ylin = plan->d_ylin;
  q.ylinT = plan->d_ylinT;
  q.n_frag = (long long)plan->lin_frag_floats;
  q.n_bins = plan->n_bins;
  q.n_half = plan->n_half;
  q.n_rt = plan->n_rt;
  q.lin_blocks = plan->lin_blocks;
  q.mp = plan->lin_mp;
  q.rp = plan->lin_rp;
  return q;
}

// The second stage of a plan with frequency-domain kernels becomes trainable (device current, the STFT stage
// already is): the spectral kernels as a tensor of their own, the two row-major forms of the matrix they make,
// and -- a trained matrix is dense -- every block of the forward kernel's second contraction switched on.
static nna_status make_spectral_trainable(nna_plan* plan) {
  const int F = plan->n_half + 1, C = 2 * plan->n_half;
  plan->lin_mp = (2 * plan->n_bins + nna::BW_MT - 1) / nna::BW_MT * nna::BW_MT;
  plan->lin_rp = (2 * F + nna::BW_MT - 1) / nna::BW_MT * nna::BW_MT;
  std::vector<float> ysk;
  std::vector<unsigned char> mask;
  try {
    ysk.assign((size_t)2 * plan->n_bins * F, 0.0f);
    for (int q = 0; q < plan->n_bins; ++q)
      for (int s = 0; s < F; ++s) {
        const size_t col = s == 0 ? 0 : s == F - 1 ? 1 : 2 * (size_t)s;  // the packed column of bin s's real part
        ysk[(size_t)(2 * q) * F + s] = plan->h_linW[(size_t)(2 * q) * C + col];
        ysk[(size_t)(2 * q + 1) * F + s] = plan->h_linW[(size_t)(2 * q + 1) * C + col];
      }
    mask.assign((size_t)plan->n_pass * plan->n_rt * ST_RB, (unsigned char)((1u << plan->lin_blocks) - 1));
  } catch (const std::bad_alloc&) {
    return fail(NNA_ERR_ALLOC, "out of host memory");
  }
  const size_t lin_bytes = (size_t)plan->lin_mp * plan->lin_rp * sizeof(float);
  nna_status s = upload(&plan->d_ysk, ysk.data(), ysk.size() * sizeof(float), "spectral kernels");
  if (s == NNA_OK) s = upload(&plan->d_ylin, nullptr, lin_bytes, "spectral kernel matrix");
  if (s == NNA_OK) s = upload(&plan->d_ylinT, nullptr, lin_bytes, "spectral kernel matrix");
  if (s == NNA_OK) {
    hipError_t e = hipMemset(plan->d_ylin, 0, lin_bytes);
    if (e == hipSuccess) e = hipMemset(plan->d_ylinT, 0, lin_bytes);
    if (e == hipSuccess) e = hipMemcpy(plan->d_mel_mask, mask.data(), mask.size(), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = nna::launch_lin_from_logical(lin_logical_params(plan, plan->d_ysk), nullptr);
    if (e == hipSuccess) e = hipStreamSynchronize(nullptr);
    if (e != hipSuccess) s = fail_hip(e, "spectral kernel matrix");
  }
  if (s != NNA_OK) {
    (void)hipFree(plan->d_ysk);
    (void)hipFree(plan->d_ylin);
    (void)hipFree(plan->d_ylinT);
    plan->d_ysk = plan->d_ylin = plan->d_ylinT = nullptr;
  }
  return s;
}

nna_status nna_plan_trainable(nna_plan* plan) {
  nna_status s = check_trainable_kind(plan);
  if (s != NNA_OK) return s;
  if (is_trainable(plan)) return NNA_OK;
  DeviceGuard guard;
  hipError_t e = guard.enter(plan->device);
  if (e != hipSuccess) return fail_hip(e, "hipSetDevice");
  if (plan->kind == NNA_KIND_CQT) return make_cqt_trainable(plan);
  if (plan->kind == NNA_KIND_CQT2010V2) {
    // every octave convolves with (rows of) the one weight: each keeps its own streaming-order copy
    for (nna_plan* sub : plan->octave)
      if (!sub->d_wrm && (s = make_cqt_trainable(sub)) != NNA_OK) return s;
    return NNA_OK;
  }
  if (plan->kind == NNA_KIND_CQT2010) {
    for (nna_plan* sub : plan->octave)
      if ((s = nna_plan_trainable(sub)) != NNA_OK) return s;
    return NNA_OK;
  }
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
  if (plan->kind == NNA_KIND_CQT1992 && (s = make_spectral_trainable(plan)) != NNA_OK) {
    (void)hipFree(plan->d_wrm);
    plan->d_wrm = nullptr;
    return s;
  }
  return NNA_OK;
}

static nna_status check_trainable(const nna_plan* plan) {
  nna_status s = check_trainable_kind(plan);
  if (s != NNA_OK) return s;
  if (!is_trainable(plan)) return fail(NNA_ERR_INVALID_ARG, "call nna_plan_trainable on the plan first");
  return NNA_OK;
}

// first row, in the weight W[2 n_top, n_taps] of a downsampling plan, of the kernels octave `sub` uses: a partial
// lowest octave holds the upper bins of an octave
static long long octave_weight_row(const nna_plan* plan, const nna_plan* sub) {
  return plan->octave[0]->conv_rows - sub->conv_rows;
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
  else if (plan->kind == NNA_KIND_CQT2010V2)
    e = nna::launch_cqt_bank_to_logical(cqt_bank_params(plan->octave[0], w_dev), reinterpret_cast<hipStream_t>(hip_stream));
  else if (plan->kind == NNA_KIND_CQT2010)
    e = nna::launch_bank_to_logical(permute_params(plan->octave[0], w_dev), reinterpret_cast<hipStream_t>(hip_stream));
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
  else if (plan->kind == NNA_KIND_CQT2010V2) {
    for (const nna_plan* sub : plan->octave) {
      float* rows = const_cast<float*>(w_dev) + octave_weight_row(plan, sub) * sub->K;
      e = nna::launch_cqt_bank_from_logical(cqt_bank_params(sub, rows), reinterpret_cast<hipStream_t>(hip_stream));
      if (e != hipSuccess) break;
    }
  } else if (plan->kind == NNA_KIND_CQT2010) {
    for (const nna_plan* sub : plan->octave) {  // the octaves share the DFT kernels; each holds them in its own hop's order
      e = nna::launch_bank_from_logical(permute_params(sub, const_cast<float*>(w_dev)), reinterpret_cast<hipStream_t>(hip_stream));
      if (e != hipSuccess) break;
    }
  } else
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
                                     float* gbuf, void* hip_stream, float* pout = nullptr, bool zero_gw = true) {
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
  // (a complex-format output is C itself: its gradient is G, and nothing needs to be recomputed)
  if (fmt == NNA_OUT_COMPLEX && !pout)
    e = nna::launch_g_from_complex(gbuf, gout_dev, n_frames, (int)T, out_bins, plan->rows_pad, plan->n_half, packed, stream);
  else
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
    if (zero_gw) {
      e = nna::launch_fill_zero(gw_dev, 2LL * plan->stft_bins() * plan->K, stream);
      if (e != hipSuccess) return fail_hip(e, "kernel launch");
    }
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

// The backward pass of one constant-Q convolution: plan's bank over T frames of each of the B waveforms in x_dev.
// gout points at the plan's first output row of waveform 0 (consecutive waveforms gout_wave_stride floats apart);
// gw (may be NULL) receives atomic adds -- zeroed here if zero_gw, else accumulated onto; gx (may be NULL) is
// overwritten.  gbuf: rows_pad x padded frames floats.  Arguments already checked, device current.
static nna_status cqt_backward_core(const nna_plan* plan, const float* x_dev, long long B, long long L, long long T,
                                    const float* gout, long long gout_wave_stride, float* gw_dev, bool zero_gw,
                                    float* gx_dev, float* gbuf, hipStream_t stream) {
  const int extra = (plan->max_jspan - 1) * plan->row_step;
  const int M = pick_tile_frames(CQ_FRAMES, T, extra, CQ_LDS_ROWS_MAX);
  if (M < 1) return fail(NNA_ERR_UNSUPPORTED, "frame tile does not fit in LDS");
  const long long n_frames = B * T, gpitch = bw_gpitch(n_frames);
  // 1. G = dLoss/dC: the forward contraction again with the derivative of the output format as its
  //    epilogue.  The kernel writes the rows of existing bins and frames; the padding stays zero.
  hipError_t e = nna::launch_fill_zero(gbuf, (long long)plan->rows_pad * gpitch, stream);
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
  P.gout = gout;
  P.gout_wave_stride = gout_wave_stride;
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
    if (zero_gw) {
      e = nna::launch_fill_zero(gw_dev, (long long)plan->conv_rows * plan->K, stream);
      if (e != hipSuccess) return fail_hip(e, "kernel launch");
    }
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
    // The shift-gathering kernel tiles the hop in 128 columns: a hop far below that (the deep octaves of a
    // downsampling plan) leaves most of every tile empty, and the plain frames x taps product over the zero-padded
    // row-major bank does less work (multiply-adds per frame: shifts x column tiles x row chunks x 128 x 32
    // against taps x rows).
    const double gathered = (double)plan->n_shift * plan->n_ct * plan->n_kc * nna::BW_NT * nna::CW_KC;
    const double dense = (double)plan->kp * plan->rows_pad;
    if (plan->hop < nna::BW_NT && 2.0 * dense <= gathered) Q.shift_rng = nullptr;
    e = nna::launch_bw_wave(Q, stream);
    if (e != hipSuccess) return fail_hip(e, "kernel launch");
  }
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
  DeviceGuard guard;
  hipError_t e = guard.enter(plan->device);
  if (e != hipSuccess) return fail_hip(e, "hipSetDevice");
  return cqt_backward_core(plan, x_dev, B, L, T, gout_dev, (long long)plan->out_rows() * T, gw_dev, true, gx_dev,
                           static_cast<float*>(workspace_dev), reinterpret_cast<hipStream_t>(hip_stream));
}

// ---- trainable kernels of the downsampling CQT (time-domain kernels; the paper's CQT2010v2 layer) -----------------
static size_t ws256f(long long floats) { return ((size_t)floats * sizeof(float) + 255) / 256 * 256; }

// gx[B, L] += (transposed decimation step) g[B, Ln]: what the octave below sends back up through the filter
static nna_status fir_transpose_add(const nna_plan* fir, const float* g, float* gx, long long B, long long L, long long Ln,
                                    hipStream_t stream) {
  nna::FirTParams F;
  std::memset(&F, 0, sizeof(F));
  F.he = fir->d_fir_he;
  F.ho = fir->d_fir_ho;
  F.ne = (int)fir->h_fir_he.size();
  F.no = (int)fir->h_fir_ho.size();
  F.ve0 = fir->fir_ve0;
  F.vo0 = fir->fir_vo0;
  F.L = L;
  F.Ln = Ln;
  for (long long b0 = 0; b0 < B; b0 += 65535) {  // the grid's second dimension holds at most 65,535 waveforms
    F.B = std::min(B - b0, 65535LL);
    F.g = g + b0 * Ln;
    F.gx = gx + b0 * L;
    const hipError_t e = nna::launch_fir_transpose_add(F, stream);
    if (e != hipSuccess) return fail_hip(e, "kernel launch");
  }
  return NNA_OK;
}

// The workspace: the waveforms of octaves 1.. (kept from the forward recursion), G of one octave, and two waveform
// gradients (octaves 1 and 2: the deeper ones alternate between them).  Offsets in bytes; false if L is too short.
struct Cqt2010BwLayout {
  long long La[MAX_OCTAVES];
  size_t x_off[MAX_OCTAVES];  // [a] for a >= 1
  size_t g_off, gx_off[2], total;
};
static bool cqt2010v2_bw_layout(const nna_plan* plan, long long B, long long L, Cqt2010BwLayout& W) {
  if (!cqt2010_lengths(plan, L, W.La)) return false;
  const int n_oct = (int)plan->octave.size();
  const long long T = 1 + L / plan->hop;
  size_t off = 0;
  for (int a = 1; a < n_oct; ++a) {
    W.x_off[a] = off;
    off += ws256f(B * W.La[a]);
  }
  int rows_pad = 0;
  for (const nna_plan* sub : plan->octave) rows_pad = std::max(rows_pad, sub->rows_pad);
  W.g_off = off;
  off += ws256f((long long)rows_pad * bw_gpitch(B * T));
  for (int i = 0; i < 2; ++i) {
    W.gx_off[i] = off;
    if (n_oct > 1 + i) off += ws256f(B * W.La[1 + i]);
  }
  W.total = off;
  return true;
}

static nna_status check_cqt2010v2_bw(const nna_plan* plan, long long B, long long L) {
  nna_status s = check_trainable(plan);
  if (s != NNA_OK) return s;
  if (plan->kind != NNA_KIND_CQT2010V2) return fail(NNA_ERR_INVALID_ARG, "plan was built for a different transform");
  if (B < 1) return fail(NNA_ERR_SHAPE, "B must be >= 1");
  const long long T = 1 + L / plan->hop;
  if (L < 1 || T > 0x7fffffffLL / 4 || L > 0x7fffffffLL - 4LL * plan->K - 64 || B > 0x7fffffffLL || B > (1LL << 40) / T)
    return fail(NNA_ERR_SHAPE, "batch too large");
  return NNA_OK;
}

nna_status nna_cqt2010v2_backward_workspace(const nna_plan* plan, long long B, long long L, size_t* bytes) {
  nna_status s = check_cqt2010v2_bw(plan, B, L);
  if (s != NNA_OK) return s;
  if (!bytes) return fail(NNA_ERR_INVALID_ARG, "bytes is NULL");
  Cqt2010BwLayout W;
  if (!cqt2010v2_bw_layout(plan, B, L, W))
    return fail(NNA_ERR_SHAPE, "L is too short: every octave's waveform must exceed the reflection padding, and all but the lowest hold one frame of the decimation filter");
  *bytes = W.total;
  return NNA_OK;
}

nna_status nna_cqt2010v2_backward(const nna_plan* plan, const float* x_dev, long long B, long long L,
                                  const float* gout_dev, float* gw_dev, float* gx_dev, void* workspace_dev,
                                  size_t workspace_bytes, void* hip_stream) {
  nna_status s = check_cqt2010v2_bw(plan, B, L);
  if (s != NNA_OK) return s;
  if (!x_dev || !gout_dev) return fail(NNA_ERR_INVALID_ARG, "x_dev / gout_dev is NULL");
  if (!gw_dev && !gx_dev) return fail(NNA_ERR_INVALID_ARG, "gw_dev and gx_dev are both NULL: nothing to compute");
  Cqt2010BwLayout W;
  if (!cqt2010v2_bw_layout(plan, B, L, W))
    return fail(NNA_ERR_SHAPE, "L is too short: every octave's waveform must exceed the reflection padding, and all but the lowest hold one frame of the decimation filter");
  if (!workspace_dev || workspace_bytes < W.total || (reinterpret_cast<uintptr_t>(workspace_dev) & 255))
    return fail(NNA_ERR_INVALID_ARG, "workspace_dev is NULL, not 256-byte aligned or smaller than nna_cqt2010v2_backward_workspace asks for");
  const int n_oct = (int)plan->octave.size();
  const long long T = 1 + L / plan->hop;
  // every launch of the call must fit before the first one is enqueued
  for (const nna_plan* sub : plan->octave)
    if (pick_tile_frames(CQ_FRAMES, T, (sub->max_jspan - 1) * sub->row_step, CQ_LDS_ROWS_MAX) < 1)
      return fail(NNA_ERR_UNSUPPORTED, "frame tile does not fit in LDS");
  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
  DeviceGuard guard;
  hipError_t e = guard.enter(plan->device);
  if (e != hipSuccess) return fail_hip(e, "hipSetDevice");
  char* ws = static_cast<char*>(workspace_dev);
  const float* xa[MAX_OCTAVES];
  xa[0] = x_dev;
  // the forward recursion: every octave's waveform is kept
  for (int a = 1; a < n_oct; ++a) {
    float* dst = reinterpret_cast<float*>(ws + W.x_off[a]);
    if ((s = run_fir(plan->fir, xa[a - 1], B, W.La[a - 1], dst, W.La[a], hip_stream)) != NNA_OK) return s;
    xa[a] = dst;
  }
  float* gbuf = reinterpret_cast<float*>(ws + W.g_off);
  const nna_plan* top = plan->octave[0];
  if (gw_dev) {
    e = nna::launch_fill_zero(gw_dev, (long long)top->conv_rows * top->K, stream);
    if (e != hipSuccess) return fail_hip(e, "kernel launch");
  }
  const long long out_stride = (long long)plan->out_rows() * T;
  const int rpb = plan->fmt == NNA_OUT_COMPLEX ? 2 : 1;
  // from the lowest octave up: octave a's own convolution, then what octave a + 1 sends back through the filter
  for (int a = n_oct - 1; a >= 0; --a) {
    const nna_plan* sub = plan->octave[a];
    int lo, hi;
    octave_bins(plan->n_bins, plan->bpo, a, lo, hi);
    float* ga = !gx_dev ? nullptr : a == 0 ? gx_dev : reinterpret_cast<float*>(ws + W.gx_off[(a - 1) & 1]);
    float* gwa = gw_dev ? gw_dev + octave_weight_row(plan, sub) * sub->K : nullptr;
    if ((s = cqt_backward_core(sub, xa[a], B, W.La[a], T, gout_dev + (long long)rpb * lo * T, out_stride, gwa, false, ga, gbuf,
                               stream)) != NNA_OK)
      return s;
    if (ga && a + 1 < n_oct) {
      const float* gb = reinterpret_cast<const float*>(ws + W.gx_off[a & 1]);
      if ((s = fir_transpose_add(plan->fir, gb, ga, B, W.La[a], W.La[a + 1], stream)) != NNA_OK) return s;
    }
  }
  return NNA_OK;
}

// ---- trainable kernels of the CQT layers with frequency-domain kernels (CQT1992, CQT2010) ---------------------------
static nna_status check_spectral(const nna_plan* plan) {
  nna_status s = check_trainable(plan);
  if (s != NNA_OK) return s;
  if (plan->kind != NNA_KIND_CQT1992 && plan->kind != NNA_KIND_CQT2010)
    return fail(NNA_ERR_INVALID_ARG, "not a plan with frequency-domain constant-Q kernels");
  return NNA_OK;
}

nna_status nna_plan_get_spectral_kernels(const nna_plan* plan, float* y_dev, void* hip_stream) {
  nna_status s = check_spectral(plan);
  if (s != NNA_OK) return s;
  if (!y_dev) return fail(NNA_ERR_INVALID_ARG, "y_dev is NULL");
  const nna_plan* top = plan->kind == NNA_KIND_CQT2010 ? plan->octave[0] : plan;
  DeviceGuard guard;
  hipError_t e = guard.enter(plan->device);
  if (e != hipSuccess) return fail_hip(e, "hipSetDevice");
  e = hipMemcpyAsync(y_dev, top->d_ysk, (size_t)2 * top->n_bins * (top->n_half + 1) * sizeof(float), hipMemcpyDeviceToDevice,
                     reinterpret_cast<hipStream_t>(hip_stream));
  if (e != hipSuccess) return fail_hip(e, "spectral kernel copy");
  return NNA_OK;
}

// rows of the weight Ysk[2 n_top, F] that octave `sub` of a downsampling plan uses (a partial lowest octave: the upper bins)
static long long octave_spectral_row(const nna_plan* plan, const nna_plan* sub) {
  return 2LL * (plan->octave[0]->n_bins - sub->n_bins);
}

nna_status nna_plan_set_spectral_kernels(nna_plan* plan, const float* y_dev, void* hip_stream) {
  nna_status s = check_spectral(plan);
  if (s != NNA_OK) return s;
  if (!y_dev) return fail(NNA_ERR_INVALID_ARG, "y_dev is NULL");
  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
  DeviceGuard guard;
  hipError_t e = guard.enter(plan->device);
  if (e != hipSuccess) return fail_hip(e, "hipSetDevice");
  auto set_one = [&](nna_plan* p, const float* rows) -> hipError_t {
    hipError_t e1 = hipMemcpyAsync(p->d_ysk, rows, (size_t)2 * p->n_bins * (p->n_half + 1) * sizeof(float),
                                   hipMemcpyDeviceToDevice, stream);
    if (e1 != hipSuccess) return e1;
    return nna::launch_lin_from_logical(lin_logical_params(p, p->d_ysk), stream);
  };
  if (plan->kind == NNA_KIND_CQT1992) {
    e = set_one(plan, y_dev);
  } else {
    for (nna_plan* sub : plan->octave) {
      e = set_one(sub, y_dev + octave_spectral_row(plan, sub) * (sub->n_half + 1));
      if (e != hipSuccess) break;
    }
  }
  if (e != hipSuccess) return fail_hip(e, "spectral kernel update");
  return NNA_OK;
}

// Workspace of one two-stage backward pass over T frames of B waveforms: the spectrum X[B][R][T] (R = 2 F rows,
// (Re, Im) pairs), the constant-Q values V[B][M][T] (M = 2 n_bins; overwritten by their gradient), the gradient
// reaching the spectrum, the matrix form of the spectral kernels' gradient, and the STFT stage's G.
struct SpectralBwLayout {
  size_t x_off, v_off, gx_off, gy_off, g_off, total;
};
static SpectralBwLayout spectral_bw_layout(const nna_plan* p, long long B, long long T, size_t base) {
  SpectralBwLayout W;
  const long long R = 2LL * (p->n_half + 1), M = 2LL * p->n_bins;
  size_t off = base;
  W.x_off = off;
  off += ws256f(B * R * T);
  W.v_off = off;
  off += ws256f(B * M * T);
  W.gx_off = off;
  off += ws256f(B * R * T);
  W.gy_off = off;
  off += ws256f(M * R);
  W.g_off = off;
  off += ws256f((long long)p->rows_pad * bw_gpitch(B * T));
  W.total = off;
  return W;
}

// The backward pass of one two-stage transform (plan of kind CQT1992, trainable): gout points at the plan's first
// output row of waveform 0.  gy_dev [2 n_bins][F] is overwritten or, with accumulate_gy, added to; gw_dev is
// added to (the caller zeroes it); gx_dev is overwritten.  Any of the three may be NULL.  Device current.
static nna_status spectral_backward_core(const nna_plan* plan, const float* x_dev, long long B, long long L, long long T,
                                         const float* gout, long long gout_wave_stride, float* gy_dev, bool accumulate_gy,
                                         float* gw_dev, float* gx_dev, char* ws, const SpectralBwLayout& W, void* hip_stream) {
  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
  const int F = plan->n_half + 1, R = 2 * F, M = 2 * plan->n_bins;
  float* X = reinterpret_cast<float*>(ws + W.x_off);
  float* V = reinterpret_cast<float*>(ws + W.v_off);
  float* GX = reinterpret_cast<float*>(ws + W.gx_off);
  float* GY = reinterpret_cast<float*>(ws + W.gy_off);
  float* gbuf = reinterpret_cast<float*>(ws + W.g_off);
  // 1. the spectrum itself, rows (Re, Im) per bin: the first stage's contraction with the complex epilogue
  {
    // With many hop-shifts (n_fft 16,384 at hop 512: 32) the 160-row tile of the two-workgroups-per-CU build holds
    // 98 frames of the 128 the MFMA tile multiplies; the 192-row tile of the one-workgroup build holds them all.
    int Mf = pick_tile_frames(ST_FRAMES, T, plan->nj - 1, ST_LDS_ROWS);
    const int Mw = pick_tile_frames(ST_FRAMES, T, plan->nj - 1, nna::ST_LDS_ROWS_WIDE);
    const bool wide = Mw * 7 > Mf * 8;  // (more than 8/7 of the frames per tile)
    if (wide) Mf = Mw;
    if (Mf < 1) return fail(NNA_ERR_UNSUPPORTED, "frame tile does not fit in LDS");
    nna::StftParams P;
    std::memset(&P, 0, sizeof(P));
    P.wide = wide ? 1 : 0;
    P.g = make_geom(plan, x_dev, B, L, T);
    P.bank = reinterpret_cast<const float4*>(plan->d_bank);
    P.out = X;
    P.n_rt = plan->n_rt;
    P.n_chunks = plan->n_chunks;
    P.nj = plan->nj;
    P.n_half = plan->n_half;
    P.packed = 1;
    P.out_bins = R;
    P.fmt = NNA_OUT_COMPLEX;
    P.tile_frames = Mf;
    P.n_ft = (P.g.n_frames + Mf - 1) / Mf;
    hipError_t e = nna::launch_stft(P, nna::ST_MODE_CPLX, stream);
    if (e != hipSuccess) return fail_hip(e, "kernel launch");
  }
  nna::MelBwParams Q;
  std::memset(&Q, 0, sizeof(Q));
  Q.B = B;
  Q.T = (int)T;
  // 2. V[b, m, t] = sum_r Ylin[m, r] X[b, r, t]
  Q.g = X;
  Q.wrm = plan->d_ylinT;
  Q.n_mels = R;
  Q.mels_pad = (R + nna::BW_KC - 1) / nna::BW_KC * nna::BW_KC;
  Q.F = M;
  Q.fp = plan->lin_mp;
  Q.gP = V;
  hipError_t e = nna::launch_mel_bw_spec(Q, stream);
  if (e != hipSuccess) return fail_hip(e, "kernel launch");
  // 3. V <- dLoss/dV through the output format
  nna::LinGradParams Gd;
  std::memset(&Gd, 0, sizeof(Gd));
  Gd.v = V;
  Gd.gout = gout;
  Gd.gout_wave_stride = gout_wave_stride;
  Gd.n = B * plan->n_bins * T;
  Gd.n_bins = plan->n_bins;
  Gd.T = (int)T;
  Gd.fmt = plan->fmt;
  e = nna::launch_lin_grad(Gd, stream);
  if (e != hipSuccess) return fail_hip(e, "kernel launch");
  // 4. gradient of the spectral kernels: gYlin[m, r] = sum_{b,t} gV[b, m, t] X[b, r, t], folded onto (Re Y, Im Y)
  if (gy_dev) {
    e = nna::launch_fill_zero(GY, (long long)M * R, stream);
    if (e != hipSuccess) return fail_hip(e, "kernel launch");
    Q.g = V;
    Q.P = X;
    Q.gW = GY;
    Q.n_mels = M;
    Q.F = R;
    Q.fp = plan->lin_rp;
    const long long tiles = (long long)((M + nna::BW_MT - 1) / nna::BW_MT) * (Q.fp / nna::BW_NT);
    const long long splits = std::max(1LL, std::min(B, (1024 + tiles - 1) / tiles));
    Q.b_per_split = (int)((B + splits - 1) / splits);
    e = nna::launch_mel_bw_weights(Q, stream);
    if (e != hipSuccess) return fail_hip(e, "kernel launch");
    e = nna::launch_lin_fold_gradient(GY, gy_dev, plan->n_bins, F, accumulate_gy ? 1 : 0, stream);
    if (e != hipSuccess) return fail_hip(e, "kernel launch");
  }
  if (!gw_dev && !gx_dev) return NNA_OK;
  // 5. gradient reaching the spectrum: gX[b, r, t] = sum_m Ylin[m, r] gV[b, m, t]
  Q.g = V;
  Q.wrm = plan->d_ylin;
  Q.n_mels = M;
  Q.mels_pad = (M + nna::BW_KC - 1) / nna::BW_KC * nna::BW_KC;
  Q.F = R;
  Q.fp = plan->lin_rp;
  Q.gP = GX;
  e = nna::launch_mel_bw_spec(Q, stream);
  if (e != hipSuccess) return fail_hip(e, "kernel launch");
  // 6. the STFT stage's backward pass with gX as the gradient of its complex output
  return stft_backward_core(plan, x_dev, B, L, T, GX, NNA_OUT_COMPLEX, R, gw_dev, gx_dev, gbuf, hip_stream, nullptr, false);
}

static nna_status check_cqt1992_bw(const nna_plan* plan, long long B, long long L, long long* T) {
  nna_status s = check_trainable(plan);
  if (s != NNA_OK) return s;
  if (plan->kind != NNA_KIND_CQT1992) return fail(NNA_ERR_INVALID_ARG, "plan was built for a different transform");
  if (B < 1) return fail(NNA_ERR_SHAPE, "B must be >= 1");
  if (L < 4) return fail(NNA_ERR_SHAPE, "L must be at least 4 samples");
  *T = frames_of(plan, L);
  if (*T < 1) return fail(NNA_ERR_SHAPE, plan->center ? "L must exceed the reflection padding (K/2)" : "L is shorter than one window");
  return NNA_OK;
}

nna_status nna_cqt1992_backward_workspace(const nna_plan* plan, long long B, long long L, size_t* bytes) {
  long long T = 0;
  nna_status s = check_cqt1992_bw(plan, B, L, &T);
  if (s != NNA_OK) return s;
  if (!bytes) return fail(NNA_ERR_INVALID_ARG, "bytes is NULL");
  *bytes = spectral_bw_layout(plan, B, T, 0).total;
  return NNA_OK;
}

nna_status nna_cqt1992_backward(const nna_plan* plan, const float* x_dev, long long B, long long L, const float* gout_dev,
                                float* gy_dev, float* gw_dev, float* gx_dev, void* workspace_dev, size_t workspace_bytes,
                                void* hip_stream) {
  long long T = 0;
  nna_status s = check_cqt1992_bw(plan, B, L, &T);
  if (s != NNA_OK) return s;
  if (!gout_dev) return fail(NNA_ERR_INVALID_ARG, "gout_dev is NULL");
  if (!gy_dev && !gw_dev && !gx_dev) return fail(NNA_ERR_INVALID_ARG, "all three gradient pointers are NULL: nothing to compute");
  float* any_out = gy_dev ? gy_dev : gw_dev ? gw_dev : gx_dev;
  if ((s = check_call(plan, NNA_KIND_CQT1992, x_dev, B, L, any_out, &T)) != NNA_OK) return s;
  const SpectralBwLayout W = spectral_bw_layout(plan, B, T, 0);
  if (!workspace_dev || workspace_bytes < W.total || (reinterpret_cast<uintptr_t>(workspace_dev) & 255))
    return fail(NNA_ERR_INVALID_ARG, "workspace_dev is NULL, not 256-byte aligned or smaller than nna_cqt1992_backward_workspace asks for");
  DeviceGuard guard;
  hipError_t e = guard.enter(plan->device);
  if (e != hipSuccess) return fail_hip(e, "hipSetDevice");
  if (gw_dev) {
    e = nna::launch_fill_zero(gw_dev, 2LL * plan->stft_bins() * plan->K, reinterpret_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return fail_hip(e, "kernel launch");
  }
  return spectral_backward_core(plan, x_dev, B, L, T, gout_dev, (long long)plan->out_rows() * T, gy_dev, false, gw_dev, gx_dev,
                                static_cast<char*>(workspace_dev), W, hip_stream);
}

// The downsampling flavour: the octaves' waveforms, two waveform gradients (as for nna_cqt2010v2_backward), then one
// octave's two-stage workspace.
struct Cqt2010SpectralLayout {
  Cqt2010BwLayout oct;  // x_off / gx_off (its g_off is unused)
  SpectralBwLayout st;
};
static bool cqt2010_spectral_layout(const nna_plan* plan, long long B, long long L, Cqt2010SpectralLayout& W) {
  Cqt2010BwLayout& O = W.oct;
  if (!cqt2010_lengths(plan, L, O.La)) return false;
  const int n_oct = (int)plan->octave.size();
  const long long T = 1 + L / plan->hop;
  size_t off = 0;
  for (int a = 1; a < n_oct; ++a) {
    O.x_off[a] = off;
    off += ws256f(B * O.La[a]);
  }
  O.g_off = off;
  for (int i = 0; i < 2; ++i) {
    O.gx_off[i] = off;
    if (n_oct > 1 + i) off += ws256f(B * O.La[1 + i]);
  }
  W.st = spectral_bw_layout(plan->octave[0], B, T, off);  // the top octave has the most bins: the largest
  O.total = W.st.total;
  return true;
}

static nna_status check_cqt2010_bw(const nna_plan* plan, long long B, long long L) {
  nna_status s = check_trainable(plan);
  if (s != NNA_OK) return s;
  if (plan->kind != NNA_KIND_CQT2010) return fail(NNA_ERR_INVALID_ARG, "plan was built for a different transform");
  if (B < 1) return fail(NNA_ERR_SHAPE, "B must be >= 1");
  const long long T = 1 + L / plan->hop;
  if (L < 1 || T > 0x7fffffffLL / 4 || L > 0x7fffffffLL - 4LL * plan->K - 64 || B > 0x7fffffffLL || B > (1LL << 40) / T)
    return fail(NNA_ERR_SHAPE, "batch too large");
  return NNA_OK;
}

nna_status nna_cqt2010_backward_workspace(const nna_plan* plan, long long B, long long L, size_t* bytes) {
  nna_status s = check_cqt2010_bw(plan, B, L);
  if (s != NNA_OK) return s;
  if (!bytes) return fail(NNA_ERR_INVALID_ARG, "bytes is NULL");
  Cqt2010SpectralLayout W;
  if (!cqt2010_spectral_layout(plan, B, L, W))
    return fail(NNA_ERR_SHAPE, "L is too short: every octave's waveform must exceed the reflection padding, and all but the lowest hold one frame of the decimation filter");
  *bytes = W.oct.total;
  return NNA_OK;
}

nna_status nna_cqt2010_backward(const nna_plan* plan, const float* x_dev, long long B, long long L, const float* gout_dev,
                                float* gy_dev, float* gw_dev, float* gx_dev, void* workspace_dev, size_t workspace_bytes,
                                void* hip_stream) {
  nna_status s = check_cqt2010_bw(plan, B, L);
  if (s != NNA_OK) return s;
  if (!x_dev || !gout_dev) return fail(NNA_ERR_INVALID_ARG, "x_dev / gout_dev is NULL");
  if (!gy_dev && !gw_dev && !gx_dev) return fail(NNA_ERR_INVALID_ARG, "all three gradient pointers are NULL: nothing to compute");
  Cqt2010SpectralLayout W;
  if (!cqt2010_spectral_layout(plan, B, L, W))
    return fail(NNA_ERR_SHAPE, "L is too short: every octave's waveform must exceed the reflection padding, and all but the lowest hold one frame of the decimation filter");
  if (!workspace_dev || workspace_bytes < W.oct.total || (reinterpret_cast<uintptr_t>(workspace_dev) & 255))
    return fail(NNA_ERR_INVALID_ARG, "workspace_dev is NULL, not 256-byte aligned or smaller than nna_cqt2010_backward_workspace asks for");
  const int n_oct = (int)plan->octave.size();
  const long long T = 1 + L / plan->hop;
  for (const nna_plan* sub : plan->octave)
    if (pick_tile_frames(ST_FRAMES, T, sub->nj - 1, ST_LDS_ROWS) < 1) return fail(NNA_ERR_UNSUPPORTED, "frame tile does not fit in LDS");
  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
  DeviceGuard guard;
  hipError_t e = guard.enter(plan->device);
  if (e != hipSuccess) return fail_hip(e, "hipSetDevice");
  char* ws = static_cast<char*>(workspace_dev);
  const long long* La = W.oct.La;
  const float* xa[MAX_OCTAVES];
  xa[0] = x_dev;
  for (int a = 1; a < n_oct; ++a) {
    float* dst = reinterpret_cast<float*>(ws + W.oct.x_off[a]);
    if ((s = run_fir(plan->fir, xa[a - 1], B, La[a - 1], dst, La[a], hip_stream)) != NNA_OK) return s;
    xa[a] = dst;
  }
  const nna_plan* top = plan->octave[0];
  const int F = top->n_half + 1;
  if (gw_dev) {
    e = nna::launch_fill_zero(gw_dev, 2LL * F * top->K, stream);
    if (e != hipSuccess) return fail_hip(e, "kernel launch");
  }
  if (gy_dev) {
    e = nna::launch_fill_zero(gy_dev, 2LL * top->n_bins * F, stream);
    if (e != hipSuccess) return fail_hip(e, "kernel launch");
  }
  const long long out_stride = (long long)plan->out_rows() * T;
  const int rpb = plan->fmt == NNA_OUT_COMPLEX ? 2 : 1;
  for (int a = n_oct - 1; a >= 0; --a) {
    const nna_plan* sub = plan->octave[a];
    int lo, hi;
    octave_bins(plan->n_bins, plan->bpo, a, lo, hi);
    float* ga = !gx_dev ? nullptr : a == 0 ? gx_dev : reinterpret_cast<float*>(ws + W.oct.gx_off[(a - 1) & 1]);
    float* gya = gy_dev ? gy_dev + octave_spectral_row(plan, sub) * F : nullptr;
    if ((s = spectral_backward_core(sub, xa[a], B, La[a], T, gout_dev + (long long)rpb * lo * T, out_stride, gya, true, gw_dev, ga,
                                    ws, W.st, hip_stream)) != NNA_OK)
      return s;
    if (ga && a + 1 < n_oct) {
      const float* gb = reinterpret_cast<const float*>(ws + W.oct.gx_off[a & 1]);
      if ((s = fir_transpose_add(plan->fir, gb, ga, B, La[a], La[a + 1], stream)) != NNA_OK) return s;
    }
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
}  // extern "C"
