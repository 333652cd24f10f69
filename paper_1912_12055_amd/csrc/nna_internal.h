// Internal declarations shared by the host planner (nna_plan.hip) and the kernels
// (nna_kernels.hip).  Nothing here is part of the C ABI.
#pragma once

#include <hip/hip_runtime.h>

#include <string>
#include <vector>

#include "../../include/nna.h"

namespace nna {

// ---- tile geometry (compile-time, shared by planner and kernels) ---------------------
// STFT / Mel kernel: v_mfma_f32_32x32x2_f32, workgroup tile 128 bank rows x 128 frames.
constexpr int ST_ROWS = 128;      // bank rows per row tile (= 64 bins: Re/Im interleaved)
constexpr int ST_RB = 4;          // 32-row MFMA blocks per row tile
constexpr int ST_FRAMES = 128;    // frames per workgroup (4 waves x 32)
constexpr int ST_KC = 32;         // taps per LDS chunk
constexpr int ST_PITCH = 36;      // LDS row pitch in floats (KC + 4: conflict-free b128 reads)
constexpr int ST_KG = 8;          // taps per bank fragment (float4 per lane, two lane halves)
constexpr int ST_NKG = ST_KC / ST_KG;
constexpr int ST_LDS_ROWS = 160;  // LDS rows per buffer (frames + overlap rows)
constexpr int ST_LDS_ROWS_WIDE = 192;  // ... of the one-workgroup-per-CU variant (ST_MODE_LIN with six output blocks)
constexpr int ST_MEL_BLOCKS = 4;  // 32-mel MFMA blocks per pass (128 mels)
constexpr int ST_RG = 4;          // row tiles one STFT workgroup handles (amortises its start-up, re-uses its frames)
// folded-frame variant of the STFT / Mel kernel (nna_kernels_fold.hip): two LDS tiles per chunk
constexpr int SF_LDS_ROWS = 136;  // LDS rows per tile: 128 frames + (J/2 - 1) overlap rows for each of two waveform segments, J <= 8
                                  // (chunks in mirrored pairs, J = 4: J - 1 overlap rows per segment)
constexpr int ST_RING_FOLD_STFT = 4;  // bank fragment groups in flight per wave
constexpr int ST_RING_FOLD_MEL = 2;
constexpr int ST_RING_FOLD_MELSPLIT = 4;  // two fragments per group: four groups in flight are as many registers as the Mel ring's
constexpr int ST_RING_FOLD_SPLIT = 2;  // the launch split by tap parity: its second set of accumulators takes the registers
constexpr int ST_LIN_BLOCKS_MAX = 6;  // ST_MODE_LIN: 4 or 6 output blocks per pass (6 when that saves a pass)
// what the STFT kernel does with a finished row tile
constexpr int ST_MODE_STFT = 0;   // per-bin epilogue, output written per row tile
constexpr int ST_MODE_MEL = 1;    // power (or magnitude) of the row tile x filterbank slice -> 128 mel accumulators
constexpr int ST_MODE_GRAD = 3;   // backward pass: dLoss/d(row tile) from the upstream gradient, written to a buffer
constexpr int ST_MODE_CPLX = 4;   // the row tile itself (Re, Im rows) or its phase is the output
constexpr int ST_MODE_MELSPEC = 5;  // ST_MODE_MEL that also writes the spectrogram the filterbank is applied to (to `pout`)
constexpr int ST_MODE_LIN = 2;    // the (Re, Im) rows themselves x a real matrix slice -> 128 output rows = 64
                                  // complex bins (constant-Q transform with frequency-domain kernels)

// float16-operand STFT kernel: v_mfma_f32_32x32x16_f16, workgroup tile 256 bank rows x 192 frames.
constexpr int H_ROWS = 256;
constexpr int H_FRAMES = 192;
constexpr int H_KC = 32;          // taps per LDS chunk (two MFMA K-steps of 16)
constexpr int H_PITCH = 40;       // LDS row pitch in halves (80 bytes: conflict-free 16-byte reads)
constexpr int H_LB_ROWS = 224;    // LDS rows of the frames tile (frames + overlap rows)

// CQT kernel: v_mfma_f32_16x16x4_f32, workgroup tile 16 bank rows (8 bins) x 256 frames.
constexpr int CQ_ROWS = 16;
constexpr int CQ_FRAMES = 256;    // 4 waves x 4 blocks of 16 frames
constexpr int CQ_KC = 16;         // taps per LDS chunk = taps per bank fragment
#ifndef NNA_CQ_PITCH
#define NNA_CQ_PITCH 20
#endif
constexpr int CQ_PITCH = NNA_CQ_PITCH;
constexpr int CQ_LDS_ROWS_MAX = 512;
#ifndef NNA_CQ_PREFETCH
#define NNA_CQ_PREFETCH 4
#endif
constexpr int CQ_PREFETCH = NNA_CQ_PREFETCH;  // bank fragments in flight per wave

// How frames map onto the batch of waveforms.
struct FrameGeom {
  const float* x;       // [B, L]
  long long B, L;
  long long n_frames;   // B * T
  int T;                // frames per waveform
  int hop;
  int pad;              // samples of reflection padding in front (K/2 or 0)
  int vec_ok;           // 16-byte loads of four consecutive samples are aligned
};

struct StftParams {
  FrameGeom g;
  const float4* bank;   // [row tile][group][ST_RB][64 lanes] float4
  // folded-frame launch only: the bank over the N/2 folded taps ([row tile of 64 bins][group][Re 0-31, Re 32-63,
  // Im 0-31, Im 32-63][64 lanes] float4), the alternating-sign window (-1)^n w[n] for bin N/2, w[N/2], and the
  // number of workgroups of the contraction itself (those behind them compute bin N/2).  `nj` then holds J/2.
  const float4* bankf;
  const float* wn;
  float wmid;
  long long main_blocks;
  // folded launch split once more by tap parity (see nna_kernels_fold.hip): n_rt then covers the bins below N/4 only,
  // and wn holds two weight tables, for the real and the imaginary part of bin N/4 (the workgroups behind the
  // contraction's compute that bin; bin N/2 comes out of the contraction)
  int split;
  // split launch whose chunks go in pairs c, n_chunks - 1 - c (the bank is stored in that order; see nna_kernels_fold.hip)
  int pair;
  float* out;
  int n_rt;             // row tiles
  int n_chunks;         // LDS chunks per row tile
  int nj;               // hop-shifts per chunk (n_fft/hop when the frames overlap in LDS, else 1)
  int n_half;           // number of (Re,Im) slots that exist (n_fft / 2 for the plain DFT)
  int packed;           // 1: slot 0 packs the two real bins 0 and n_half (plain DFT); 0: slot s = bin s
  int out_bins;         // bins per waveform in `out`
  int fmt;              // nna_output (STFT) ; Mel: 1 = magnitude before the filterbank, 2 = power
  long long n_ft;       // frame tiles
  int tile_frames;      // frames per tile (<= ST_FRAMES; smaller only when many short waveforms share a tile)
  // Mel only
  const float4* melw;   // [pass][row tile][ST_RB][ST_MEL_BLOCKS][2][64 lanes] float4 (ST_MODE_LIN: [lin_blocks][4])
  int lin_blocks;       // ST_MODE_LIN: 32-row output blocks per pass, 4 or 6
  int wide;             // ST_MODE_CPLX: the one-workgroup-per-CU instantiation with ST_LDS_ROWS_WIDE rows per tile
  const unsigned char* mel_mask;  // [pass][row tile][ST_RB]: bit mb set if that 32-mel block is non-zero
  const float* mel_wnyq;          // [n_mels] weight of the Nyquist bin
  const int* mel_pass_rt;         // [pass][2]: first row tile, one past the last
  int n_mels;
  int n_pass;
  int mel_nyq_any;
  // ST_MODE_GRAD (backward pass): nothing is written to `out`; instead the gradient
  // of the loss with respect to the contraction's result, G[packed row][global frame], is written
  // from the upstream gradient gout[B, out_bins, T] (fmt selects the derivative of the output format)
  const float* gout;
  float* pout;                // optional (magnitude / power formats): the stage's output [B, out_bins, T] as well
  float* gbuf;                // [frame / 32][n_rt * ST_ROWS packed rows][frame % 32]
  long long gpitch;           // elements between consecutive rows of gbuf (32)
  // ST_MODE_LIN only: where this plan's bins go in `out`
  long long out_wave_stride;  // elements of `out` per waveform
  int row_offset;             // the plan's first output row is row row_offset of each waveform's output
};

struct Stft16Params {
  FrameGeom g;
  const _Float16* bank;  // [row tile][chunk][hop-shift][H_ROWS][H_KC] float16
  const _Float16* bank_s;  // the same bank in MFMA-fragment streaming order, or NULL (see stft16s_kernel)
  float* out;
  int n_rt;              // row tiles of H_ROWS packed rows
  int n_chunks;          // LDS chunks per hop
  int nj;                // hop-shifts (n_fft / hop)
  int n_half, packed, out_bins, fmt;  // as in StftParams
  int rt_per_block;      // row tiles one workgroup handles
  int tile_frames;       // frames per tile (<= H_FRAMES)
  long long n_ft;
};

constexpr int CQ_ITEM_RB = 4;  // row blocks one CQT workgroup can handle (short kernels are grouped)
constexpr int CQ_TABLE_CAP = 512;  // chunk descriptors of a work item held in LDS at a time (a power of two; 24 KB)

// One LDS chunk of a CQT work item (48 bytes, read as three 16-byte words).
struct CqtChunk {
  int c0;    // first tap column of the chunk (within the hop, or absolute when frames do not overlap)
  int jlo;   // first hop-shift of the chunk's LDS rows (that of the item's first, longest row block)
  int pad0, pad1;
  int joff[CQ_ITEM_RB];  // first hop-shift of row block r, relative to jlo
  int nj[CQ_ITEM_RB];    // low 16 bits: bank fragments of row block r in this chunk, a multiple of CQ_PREFETCH
                         // (0 = none); high 16 bits: how many of them, from the front, hold taps
};

// A CQT work item: up to CQ_ITEM_RB consecutive row blocks that share the LDS tiles of the first.
struct CqtItem {
  long long frag0;  // first bank fragment of the item
  int rb_first;
  int n_rb;
  int jspan;        // LDS rows per waveform segment beyond the frames, + 1
  int n_chunks;     // chunks listed for the item (each holds taps of its first row block)
  int pad0, pad1;
};

struct CqtParams {
  FrameGeom g;
  const float4* bank;      // per item: [fragment][64 lanes] float4, fragments in loop order
  const CqtItem* items;    // [n_items]
  const CqtChunk* chunks;  // [n_items][n_chunks]
  float* out;
  long long out_wave_stride;  // elements of `out` per waveform (all bins x frames)
  int row_offset;          // the bank's first output row is row row_offset of each waveform's output
  int tap_stride;          // taps between consecutive shifts of a chunk (see CqtChunk::jlo)
  int row_step;            // LDS rows between consecutive shifts: 1, or 16 / hop when the hop divides the chunk
  int n_items;
  int n_chunks;            // stride of `chunks` (largest n_chunks of any item)
  int n_bins;
  int fmt;
  int lds_rows;            // rows per LDS buffer
  int tile_frames;         // frames per tile (<= CQ_FRAMES)
  long long n_ft;
  // backward pass (gbuf != NULL): the epilogue writes G = dLoss/dC instead of the spectrogram
  const float* gout;       // upstream gradient [B][out rows][T]
  long long gout_wave_stride;
  float* gbuf;             // G in blocks of 32 frames, [frames / 32][rows_pad][32]
  int rows_pad;
};

// ---- constant-Q kernels folded about their centres (nna_kernels_cqf.hip) ----------------------
constexpr int CQF_NPASS = 6;                  // loader passes of 64 rows per tile
constexpr int CQF_LDS_ROWS = CQF_NPASS * 64;  // rows of each of the two tiles (taps in front of / behind the centre)
constexpr int CQF_TABLE_CAP = 1024;           // chunk descriptors per work item (16 bytes each)

// One 16-tap column chunk of a work item: every hop-shift from 0 on that holds folded taps of a block pair.
struct CqfChunk {
  int c0;      // first folded-tap column of the chunk within the hop
  int nj[2];   // per block pair: low 16 bits = pair groups (one cosine + one sine fragment each), a multiple of two
               // (0 = none); high 16 bits = how many of them, from the front, hold taps
  int pad0;
};

// A work item: one or two groups of 16 bins whose kernel lengths have the same parity; each group is a block pair
// (cosine rows against the even fold, sine rows against the odd fold).  The groups share the item's two tiles.
struct CqfItem {
  long long frag0;  // first bank fragment
  int grp_first;    // first 16-bin group (row of `bins`)
  int n_pair;       // 1 or 2
  int parity;       // 0: kernels symmetric about tap K/2, 1: about K/2 - 1/2
  int jspan;        // hop-shifts the longest kernel of the item spans
  int n_chunks;
  int pad0;
};

struct CqfParams {
  FrameGeom g;
  const float4* bank;      // per item: [fragment][64 lanes] float4 in loop order
  const CqfItem* items;
  const CqfChunk* chunks;  // [n_items][n_chunks]
  const int* bins;         // [group][16]: output bin of each row, -1 = none
  float* out;
  long long out_wave_stride;
  int row_offset;
  int n_items;
  int n_chunks;            // stride of `chunks`
  int fmt;
  int lds_rows;            // rows per tile (multiple of 64, <= CQF_LDS_ROWS)
  int tile_frames;
  int centre;              // K / 2: folded tap m pairs the samples centre + m and centre - parity - m of a frame
  float rot_c, rot_s;      // cos, sin of pi Q: the kernels' common phase at their centres
  long long n_ft;
};

// ---- backward pass of the STFT layer (trainable kernel banks) --------------------------------
constexpr int BW_MT = 128;   // output tile rows per workgroup
constexpr int BW_NT = 128;   // output tile columns per workgroup
constexpr int BW_KC = 32;    // contraction chunk staged in LDS
constexpr int CW_KC = 16;    // bank rows per chunk of the shift-gathering waveform gradient (cq_wave_kernel)

struct BwParams {
  FrameGeom g;           // the batch (x may be NULL when only the waveform gradient is wanted)
  const float* gbuf;     // G = dLoss/dC in blocks of 32 frames, [gpitch / 32][rows_pad][32], zero padded: a
                         // 128-row x 32-frame operand tile is one contiguous 16 KB run
  long long gpitch;      // frames, padded to a multiple of BW_MT
  const float* wrm;      // packed bank, row-major [rows_pad][kp], zero padded
  int kp;                // row pitch of wrm (multiple of BW_NT)
  int rows_pad;          // multiple of BW_MT
  int n_half, packed;    // as in StftParams: maps packed rows to the logical rows of gw
  int K;                 // taps
  float* gw;             // [logical rows][K], zeroed; partial sums are added atomically
  float* gx;             // [B][L], zeroed; overlapping frames and mirrored samples are added atomically
  int n_split;           // bank gradient: workgroups that share one output tile (split contraction)
  long long chunks_per_split;
  // Banks whose rows are zero outside a tap range (constant-Q kernels, rows ordered longest first);
  // all NULL / 0 for a dense bank.
  const int2* tiles;     // bank gradient: the output tiles that hold taps, x = row tile | (32-row blocks of it that
                         // hold taps here) << 16, y = tap tile; NULL: every tile, all four blocks
  int n_tiles;
  const int* row_lo;     // bank gradient: row r is a parameter on taps [row_lo[r], row_hi[r]) only
  const int* row_hi;
  // waveform gradient, gathered over the hop-shifts (see cq_wave_kernel): shift_rng[ct][kc], ct = 128-column
  // tile of the hop, kc = chunk of CW_KC rows: first and last shift on which those rows hold taps (x > y: none)
  const int2* shift_rng;
  int n_kc;              // row chunks listed per column tile
  int n_shift;           // hop-shifts: ceil(K / hop)
  int n_ct;              // column tiles of the hop: ceil(hop / BW_NT)
  long long n_qt;        // hop-row tiles of a waveform's padded signal: ceil((T + n_shift - 1) / BW_MT)
};

// Transposed decimation step (backward pass of the downsampling CQT): gx[B, L] += D^T g, g[B, Ln], with the taps
// as the decimation kernel holds them (FirParams)
struct FirTParams {
  const float* g;
  float* gx;
  const float* he;
  const float* ho;
  int ne, no, ve0, vo0;
  long long B, L, Ln;
};
hipError_t launch_fir_transpose_add(const FirTParams& p, hipStream_t stream);

// constant-Q bank of a trainable plan: the caller's [rows][K] tensor <-> streaming order / row-major copy
struct CqtBankParams {
  float* bank;           // streaming order, n_bank floats
  const int* map;        // per float of `bank`: index into the caller's tensor, or -1 (structural zero)
  long long n_bank;
  float* wrm;            // row-major [rows_pad][kp], zero outside each row's support
  const int* row_lo;     // [rows]
  const int* row_hi;
  float* logical;        // caller's tensor [rows][K]
  int rows, K, kp;
};

// logical <-> streaming order of an STFT bank on the device
struct BankPermuteParams {
  float* bank;           // fragment order [row tile][group][ST_RB][64][4]
  float* wrm;            // row-major packed [rows_pad][kp]
  float* logical;        // [logical rows][K] (caller's tensor)
  int n_rt, n_chunks, nj, hop, K, kp, n_half, packed;
};

// The Mel layer's two small contractions of the backward pass (per waveform b, frames t contiguous):
//   gP[b, k, t]   = sum_m W[m, k] g[b, m, t]        (gradient reaching the STFT's output)
//   gW[m, k]     += sum_{b,t} g[b, m, t] P[b, k, t]   (gradient of the filterbank)
struct MelBwParams {
  const float* g;        // upstream gradient [B][n_mels][T]
  const float* wrm;      // filterbank, row-major [mels_pad][fp], zero padded (fp a multiple of BW_MT)
  const float* P;        // |X|^power [B][F][T]                      (filterbank gradient)
  float* gP;             // [B][F][T]                                (gradient to the STFT output)
  float* gW;             // [n_mels][F], zeroed; partial sums are added atomically
  long long B;
  int T, F, n_mels, fp, mels_pad;
  int b_per_split;       // filterbank gradient: waveforms per workgroup
};

// Spectral kernels of a trainable plan with frequency-domain constant-Q kernels: the caller's tensor
// Ysk[2 n_bins][n_half + 1] -> the fragment-order matrix of the forward kernel's second contraction and the two
// row-major copies the backward pass multiplies with
struct LinLogicalParams {
  const float* ysk;
  float* frag;           // n_frag floats, indexed as the forward kernel reads them
  float* ylin;           // [.][rp]: Ylin[2q][2s] = Yr, [2q][2s+1] = -Yi, [2q+1][2s] = Yi, [2q+1][2s+1] = Yr
  float* ylinT;          // [.][mp]: its transpose
  long long n_frag;
  int n_bins, n_half, n_rt, lin_blocks, mp, rp;
};
hipError_t launch_lin_from_logical(const LinLogicalParams& p, hipStream_t stream);

// Second stage of the backward pass of those plans, elementwise: v[B][2 n_bins][T] holds the complex constant-Q
// values (rows 2q = Re, 2q+1 = Im) and is overwritten with dLoss/d(Re, Im) given gout (the output format's
// derivative; gout: row q of a waveform, or rows 2q, 2q+1 for the complex format, waveforms gout_wave_stride apart)
struct LinGradParams {
  float* v;
  const float* gout;
  long long gout_wave_stride, n;  // n = B n_bins T
  int n_bins, T, fmt;
};
hipError_t launch_lin_grad(const LinGradParams& p, hipStream_t stream);
// gysk[2q][s] (+)= gylin[2q][2s] + gylin[2q+1][2s+1],  gysk[2q+1][s] (+)= gylin[2q+1][2s] - gylin[2q][2s+1]
// (gylin[2 n_bins][2 F], gysk[2 n_bins][F])
hipError_t launch_lin_fold_gradient(const float* gylin, float* gysk, int n_bins, int F, int accumulate, hipStream_t stream);

// The launchers report hipGetLastError() right after their launch.  That call also returns (and clears) an
// error some earlier, unrelated call of this thread left behind -- PyTorch shares the runtime -- so every
// launcher first clears whatever is pending: the status it returns is then its own launch's.
inline void clear_stale_error() { (void)hipGetLastError(); }

hipError_t launch_stft(const StftParams& p, int mode, hipStream_t stream);
hipError_t launch_stft_fold(const StftParams& p, int mode, hipStream_t stream);  // ST_MODE_STFT or ST_MODE_MEL
hipError_t launch_mel_bw_spec(const MelBwParams& p, hipStream_t stream);    // gP
hipError_t launch_mel_bw_weights(const MelBwParams& p, hipStream_t stream); // gW
hipError_t launch_mel_from_logical(const float* w, float* frag, float* wnyq, float* wrm, int n_mels, int n_half, int n_rt,
                                   int n_pass, int fp, hipStream_t stream);
hipError_t launch_fill_zero(float* p, long long n, hipStream_t stream);
hipError_t launch_fill_zero_frames(float* gbuf, long long rows_pad, long long f0, long long f1, hipStream_t stream);
// G <- the upstream gradient of a complex-format output, re-laid out (see g_from_complex_kernel)
hipError_t launch_g_from_complex(float* gbuf, const float* gout, long long n_frames, int T, int out_rows, int rows_pad,
                                 int n_half, int packed, hipStream_t stream);
hipError_t launch_bank_from_logical(const BankPermuteParams& p, hipStream_t stream);  // logical -> bank, wrm
hipError_t launch_bank_to_rowmajor(const BankPermuteParams& p, hipStream_t stream);   // bank -> wrm
hipError_t launch_bank_to_logical(const BankPermuteParams& p, hipStream_t stream);    // wrm -> logical
hipError_t launch_bw_bank(const BwParams& p, hipStream_t stream);      // gw += G x frames
hipError_t launch_bw_wave(const BwParams& p, hipStream_t stream);      // gx += transposed convolution
// decimation by two on the vector ALUs (fir_decimate_kernel)
constexpr int FIR_T = 8;                // outputs per thread
constexpr int FIR_TILE = 256 * FIR_T;   // outputs per workgroup
struct FirParams {
  const float* x;        // [B, L]
  float* y;              // [B, Ln], Ln = ceil(L / 2)
  long long B, L, Ln;
  const float* he;       // taps on the even samples, he[k] = h[half + 2 (ve0 + k)], zero padded to a multiple of 8
  const float* ho;       // taps on the odd samples, ho[k] = h[half + 2 (vo0 + k) + 1], likewise
  int ne, no;            // padded tap counts
  int ve0, vo0;          // first v of each tap list (<= 0)
  int lds_stream;        // floats of LDS per stream: (FIR_TILE + (span of v) + 8) * 9 / 8, rounded up
  int vec2;              // 8-byte loads of sample pairs are aligned
  int vec4_out;          // 16-byte stores are aligned
};
hipError_t launch_fir_decimate(const FirParams& p, hipStream_t stream);
hipError_t launch_cqt(const CqtParams& p, hipStream_t stream);
hipError_t launch_cqt_fold(const CqfParams& p, hipStream_t stream);
hipError_t cqf_kernels_init();  // per-process function attributes of nna_kernels_cqf.hip
size_t cqt_launch_lds_bytes(int n_chunks, int lds_rows);  // dynamic LDS launch_cqt asks for (limit: 160 KB)
hipError_t launch_cqt_bank_from_logical(const CqtBankParams& p, hipStream_t stream);  // bank and wrm <- logical
hipError_t launch_cqt_bank_to_logical(const CqtBankParams& p, hipStream_t stream);    // logical <- wrm
hipError_t launch_stft16(const Stft16Params& p, hipStream_t stream);
hipError_t kernels_init();  // per-process function attributes

}  // namespace nna
