// GPU kernels (gfx950 / CDNA4) for the strided-convolution spectrogram transforms of
// arXiv 1912.12055: STFT (Sec. III-A), Mel (Sec. III-B) and time-domain CQT (Sec. III-C).
//
// All three are the contraction  C[row, frame] = sum_k bank[row, k] * xp[frame*hop + k]
// (a strided convolution, eq. (convolutionWithStride), with the kernel flip of Sec. III-A
// folded away) followed by a per-(Re,Im)-pair epilogue.  The kernels never materialise the
// frames matrix: because frames overlap, the reflect-padded waveform is viewed as a matrix
// S[r, c] = xp[r*hop + c] and frame t, tap k = j*hop + c reads S[t + j, c].  One LDS tile of
// (frames + overlap) rows x KC columns therefore serves every hop-shift j by sliding one row.
// The bank is stored in device memory in exactly the order the MFMA fragments are consumed,
// so each wave streams it with one coalesced 16-byte load per lane per fragment.
//
// MFMA operand roles: the bank supplies the "A" operand (rows = Re/Im bank rows), the frames
// supply "B" (columns = frames), so that in the accumulator the 32 (or 16) lanes of a
// register hold consecutive frames of one bin -- the output [B, bins, T] is T-fastest and the
// stores coalesce without a transpose.
#include "nna_internal.h"

namespace nna {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------------------------------
// Frame tile <-> LDS row mapping.  A tile of consecutive global frames f0.. may span several
// waveforms ("segments"); each segment owns (its frames + extra) consecutive LDS rows.
// ---------------------------------------------------------------------------------------
struct TileMap {
  long long b0;  // waveform of the first frame
  int t0;        // frame index of the first frame inside waveform b0
  int n0;        // frames of waveform b0 inside this tile
  int extra;     // overlap rows per segment (hop-shifts - 1)
  int T;

  __device__ __forceinline__ int frame_row(int i) const {
    return i < n0 ? i : i + (1 + (i - n0) / T) * extra;
  }
  // LDS row -> (waveform, row index sigma of the S matrix)
  __device__ __forceinline__ void decode(int row, long long& b, int& sigma) const {
    const int first = n0 + extra;
    if (row < first) {
      b = b0;
      sigma = t0 + row;
    } else {
      const int r = row - first, seg = T + extra, s = r / seg;
      b = b0 + 1 + s;
      sigma = r - s * seg;
    }
  }
};

__device__ __forceinline__ float load_reflect(const float* __restrict__ xb, long long i, long long L) {
  long long r = i < 0 ? -i : (i >= L ? 2 * (L - 1) - i : i);
  r = r < 0 ? 0 : (r >= L ? L - 1 : r);  // only reachable under zero-padded bank columns
  return xb[r];
}

// Global -> registers for one LDS chunk: rows [0, rows_used) x KC columns starting at sample
// column c0 of S-row (sigma + jlo).  256 threads, NPASS passes of 256*4/KC rows.
template <int KC, int NPASS>
__device__ __forceinline__ void load_chunk(float4 (&R)[NPASS], const FrameGeom& g, const TileMap& tm,
                                           int rows_used, int jlo, int c0, int tid) {
  constexpr int V = KC / 4;
  constexpr int RPP = 256 / V;
  const int cv = tid % V, r0 = tid / V;
#pragma unroll
  for (int p = 0; p < NPASS; ++p) {
    const int row = p * RPP + r0;
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (row < rows_used) {
      long long b;
      int sigma;
      tm.decode(row, b, sigma);
      if (b < g.B) {
        const long long i0 = (long long)(sigma + jlo) * g.hop + c0 + cv * 4 - g.pad;
        const float* __restrict__ xb = g.x + b * g.L;
        if (g.vec_ok && i0 >= 0 && i0 + 3 < g.L) {
          v = *reinterpret_cast<const float4*>(xb + i0);
        } else {
          v.x = load_reflect(xb, i0, g.L);
          v.y = load_reflect(xb, i0 + 1, g.L);
          v.z = load_reflect(xb, i0 + 2, g.L);
          v.w = load_reflect(xb, i0 + 3, g.L);
        }
      }
    }
    R[p] = v;
  }
}

template <int KC, int PITCH, int NPASS>
__device__ __forceinline__ void store_chunk(const float4 (&R)[NPASS], float* lds, int rows_alloc, int tid) {
  constexpr int V = KC / 4;
  constexpr int RPP = 256 / V;
  const int cv = tid % V, r0 = tid / V;
#pragma unroll
  for (int p = 0; p < NPASS; ++p) {
    const int row = p * RPP + r0;
    if (row < rows_alloc) *reinterpret_cast<float4*>(lds + row * PITCH + cv * 4) = R[p];
  }
}

__device__ __forceinline__ float format_power(float pw, int fmt) {
  if (fmt == NNA_OUT_MAGNITUDE) return sqrtf(pw);
  if (fmt == NNA_OUT_POWER) return pw;
  return logf(fmaxf(pw, 1e-10f));
}

// ---------------------------------------------------------------------------------------
// STFT / Mel kernel.
// Workgroup = 4 waves; wave w owns frames [32w, 32w+32) of the frame tile and all 128 rows of
// the current row tile: 4 accumulators of 32x32 (v_mfma_f32_32x32x2_f32).  Accumulator
// register r of lane l = (h = l/32, n = l%32) holds row 8*(r/4) + 4h + r%4 of frame n, so the
// (Re, Im) rows 2s, 2s+1 of slot s sit in registers r, r+1 of one lane.
// Row tiles are visited one after the other; in the Mel variant the power of each finished row
// tile is contracted, straight from the accumulator registers, with the matching slice of the
// filterbank by a second MFMA into 128 mel x 32 frame accumulators.
// ---------------------------------------------------------------------------------------
constexpr int ST_NPASS = ST_LDS_ROWS / (256 / (ST_KC / 4));  // 192 / 32 = 6

template <bool MEL>
__global__ __launch_bounds__(256, 2) void stft_kernel(const StftParams P) {
  __shared__ __attribute__((aligned(16))) float lds[2][ST_LDS_ROWS * ST_PITCH];

  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int h = lane >> 5, n = lane & 31;

  // ---- which work item: (frame tile, row tile range) --------------------------------
  long long ft;
  int rt_begin, rt_end, pass = 0;
  if constexpr (MEL) {
    ft = (long long)blockIdx.x / P.n_pass;
    pass = (int)(blockIdx.x % P.n_pass);
    rt_begin = P.mel_pass_rt[2 * pass];
    rt_end = P.mel_pass_rt[2 * pass + 1];
  } else {
    // XCD-aware order: workgroup ids are dealt round-robin to the 8 XCDs.  Each XCD walks its
    // own contiguous range of frame tiles in groups of 64; inside a group the row tile is the
    // slow index, so the ~64 workgroups resident on an XCD share one 1 MB bank tile in its L2.
    constexpr int GROUP = 64;
    const long long bid = blockIdx.x;
    const int xcd = (int)(bid & 7);
    const long long idx = bid >> 3;
    const long long ft_per_xcd = (P.n_ft + 7) / 8;
    const long long per_group = (long long)GROUP * P.n_rt;
    const long long grp = idx / per_group;
    const int rem = (int)(idx - grp * per_group);
    const long long grp_first = grp * GROUP;
    long long grp_size = ft_per_xcd - grp_first;
    if (grp_size > GROUP) grp_size = GROUP;
    if (grp_size <= 0) return;
    const int rt = rem / (int)grp_size;
    const int fi = rem - rt * (int)grp_size;
    if (rt >= P.n_rt) return;
    const long long ft_local = grp_first + fi;
    ft = xcd * ft_per_xcd + ft_local;
    if (ft >= P.n_ft) return;
    rt_begin = rt;
    rt_end = rt + 1;
  }

  const FrameGeom& g = P.g;
  const long long f0 = ft * P.tile_frames;
  const int m_valid = (int)((g.n_frames - f0) < P.tile_frames ? (g.n_frames - f0) : P.tile_frames);
  TileMap tm;
  tm.T = g.T;
  tm.b0 = f0 / g.T;
  tm.t0 = (int)(f0 - tm.b0 * g.T);
  tm.n0 = (g.T - tm.t0) < m_valid ? (g.T - tm.t0) : m_valid;
  tm.extra = P.nj - 1;
  const int rows_used = tm.frame_row(m_valid - 1) + tm.extra + 1;

  // this lane's frame
  const int fi_lane = wave * 32 + n;
  const bool valid = fi_lane < m_valid;
  const long long f_lane = f0 + fi_lane;
  const long long b_lane = valid ? f_lane / g.T : 0;
  const int t_lane = valid ? (int)(f_lane - b_lane * g.T) : 0;
  const int row_lane = valid ? tm.frame_row(fi_lane) : 0;
  const int a_off = row_lane * ST_PITCH + 4 * h;

  const int n_chunks = P.n_chunks;
  const int total = (rt_end - rt_begin) * n_chunks;
  if (total <= 0) return;
  const int groups_per_rt = n_chunks * P.nj * ST_NKG;
  const float4* __restrict__ bankp =
      P.bank + ((long long)rt_begin * groups_per_rt) * (ST_RB * 64) + lane;

  f32x16 acc[ST_RB];
#pragma unroll
  for (int rb = 0; rb < ST_RB; ++rb)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[rb][r] = 0.f;

  f32x16 macc[MEL ? ST_MEL_BLOCKS : 1];
  float nyq = 0.f;
  if constexpr (MEL) {
#pragma unroll
    for (int mb = 0; mb < ST_MEL_BLOCKS; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) macc[mb][r] = 0.f;
  }

  // ---- prologue: chunk 0 into LDS buffer 0, chunk 1 into registers, first bank fragments --
  float4 R[ST_NPASS];
  load_chunk<ST_KC, ST_NPASS>(R, g, tm, rows_used, 0, 0, tid);
  store_chunk<ST_KC, ST_PITCH, ST_NPASS>(R, lds[0], ST_LDS_ROWS, tid);
  if (total > 1) load_chunk<ST_KC, ST_NPASS>(R, g, tm, rows_used, 0, (1 % n_chunks) * ST_KC, tid);

  float4 bq[ST_NKG][ST_RB];
#pragma unroll
  for (int kg = 0; kg < ST_NKG; ++kg)
#pragma unroll
    for (int rb = 0; rb < ST_RB; ++rb) bq[kg][rb] = bankp[(kg * ST_RB + rb) * 64];
  bankp += ST_NKG * ST_RB * 64;
  __syncthreads();

  int c = 0;            // chunk inside the current row tile
  int rt = rt_begin;
  for (int it = 0; it < total; ++it) {
    if (it + 1 < total) store_chunk<ST_KC, ST_PITCH, ST_NPASS>(R, lds[(it + 1) & 1], ST_LDS_ROWS, tid);
    if (it + 2 < total) load_chunk<ST_KC, ST_NPASS>(R, g, tm, rows_used, 0, ((it + 2) % n_chunks) * ST_KC, tid);

    const float* __restrict__ A = lds[it & 1] + a_off;
    for (int jj = 0; jj < P.nj; ++jj) {
#pragma unroll
      for (int kg = 0; kg < ST_NKG; ++kg) {
        const float4 a = *reinterpret_cast<const float4*>(A + jj * ST_PITCH + kg * ST_KG);
        const float av[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
#pragma unroll
          for (int rb = 0; rb < ST_RB; ++rb) {
            const float bv = e == 0 ? bq[kg][rb].x : e == 1 ? bq[kg][rb].y : e == 2 ? bq[kg][rb].z : bq[kg][rb].w;
            acc[rb] = __builtin_amdgcn_mfma_f32_32x32x2f32(bv, av[e], acc[rb], 0, 0, 0);
          }
        }
        // refill this ring slot with the fragment ST_NKG groups ahead (the bank allocation is
        // padded by ST_NKG groups, so the tail reads stay in bounds)
#pragma unroll
        for (int rb = 0; rb < ST_RB; ++rb) bq[kg][rb] = bankp[(kg * ST_RB + rb) * 64];
      }
      bankp += ST_NKG * ST_RB * 64;
    }

    if (++c == n_chunks) {
      // ---- epilogue of row tile rt ---------------------------------------------------
      c = 0;
      const int slot_base = rt * (ST_ROWS / 2);
      if constexpr (!MEL) {
        const long long F = P.n_half + 1;
        float* __restrict__ op = P.out + (b_lane * F) * g.T + t_lane;
#pragma unroll
        for (int rb = 0; rb < ST_RB; ++rb) {
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            const float re = acc[rb][2 * u], im = acc[rb][2 * u + 1];
            const int slot = slot_base + rb * 16 + 4 * (u >> 1) + 2 * h + (u & 1);
            if (valid) {
              if (slot == 0) {  // slot 0 packs the two purely real bins: DC and Nyquist
                op[0] = format_power(re * re, P.fmt);
                op[(long long)P.n_half * g.T] = format_power(im * im, P.fmt);
              } else if (slot < P.n_half) {
                op[(long long)slot * g.T] = format_power(re * re + im * im, P.fmt);
              }
            }
          }
        }
      } else {
        const unsigned char* __restrict__ maskp = P.mel_mask + ((long long)pass * P.n_rt + rt) * ST_RB;
        const float4* __restrict__ wp =
            P.melw + (((long long)pass * P.n_rt + rt) * ST_RB) * (ST_MEL_BLOCKS * 2 * 64) + lane;
#pragma unroll
        for (int rb = 0; rb < ST_RB; ++rb) {
          float pw[8];
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            const float re = acc[rb][2 * u], im = acc[rb][2 * u + 1];
            float v = re * re + im * im;
            if (rb == 0 && u == 0 && h == 0 && slot_base == 0) {  // DC / Nyquist slot
              v = re * re;
              nyq = im * im;
              if (P.fmt == 1) nyq = sqrtf(nyq);
            }
            pw[u] = P.fmt == 1 ? sqrtf(v) : v;
          }
          const unsigned mask = maskp[rb];
#pragma unroll
          for (int mb = 0; mb < ST_MEL_BLOCKS; ++mb) {
            if (mask & (1u << mb)) {
              const float4 w0 = wp[((rb * ST_MEL_BLOCKS + mb) * 2 + 0) * 64];
              const float4 w1 = wp[((rb * ST_MEL_BLOCKS + mb) * 2 + 1) * 64];
              macc[mb] = __builtin_amdgcn_mfma_f32_32x32x2f32(w0.x, pw[0], macc[mb], 0, 0, 0);
              macc[mb] = __builtin_amdgcn_mfma_f32_32x32x2f32(w0.y, pw[1], macc[mb], 0, 0, 0);
              macc[mb] = __builtin_amdgcn_mfma_f32_32x32x2f32(w0.z, pw[2], macc[mb], 0, 0, 0);
              macc[mb] = __builtin_amdgcn_mfma_f32_32x32x2f32(w0.w, pw[3], macc[mb], 0, 0, 0);
              macc[mb] = __builtin_amdgcn_mfma_f32_32x32x2f32(w1.x, pw[4], macc[mb], 0, 0, 0);
              macc[mb] = __builtin_amdgcn_mfma_f32_32x32x2f32(w1.y, pw[5], macc[mb], 0, 0, 0);
              macc[mb] = __builtin_amdgcn_mfma_f32_32x32x2f32(w1.z, pw[6], macc[mb], 0, 0, 0);
              macc[mb] = __builtin_amdgcn_mfma_f32_32x32x2f32(w1.w, pw[7], macc[mb], 0, 0, 0);
            }
          }
        }
      }
#pragma unroll
      for (int rb = 0; rb < ST_RB; ++rb)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[rb][r] = 0.f;
      ++rt;
    }
    __syncthreads();
  }

  if constexpr (MEL) {
    // Nyquist-bin term (its power lives in lane n of the first lane half) and the store.
    float nyq_n = 0.f;
    if (P.mel_nyq_any) nyq_n = __shfl(nyq, n, 64);
    float* __restrict__ op = P.out + (b_lane * P.n_mels) * g.T + t_lane;
#pragma unroll
    for (int mb = 0; mb < ST_MEL_BLOCKS; ++mb) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int mel = pass * (32 * ST_MEL_BLOCKS) + mb * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
        if (valid && mel < P.n_mels) {
          float v = macc[mb][r];
          if (P.mel_nyq_any) v += P.mel_wnyq[mel] * nyq_n;
          op[(long long)mel * g.T] = v;
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------------------
// CQT kernel.
// Workgroup = 4 waves, one 16-row bank block (8 bins, Re/Im interleaved) x 256 frames; wave w
// owns frames [64w, 64w+64) as 4 blocks of 16 (v_mfma_f32_16x16x4_f32).  Accumulator register
// r of lane l = (q = l/16, n = l%16) holds row 4q + r of frame n: bin 2q in r = 0,1 and bin
// 2q+1 in r = 2,3.  Only the taps inside the block's longest kernel are visited: per LDS chunk
// the planner lists the hop-shifts [jlo, jlo+nj) that hold non-zero taps.
// ---------------------------------------------------------------------------------------
constexpr int CQ_NPASS = CQ_LDS_ROWS_MAX / (256 / (CQ_KC / 4));  // 512 / 64 = 8

__global__ __launch_bounds__(256, 2) void cqt_kernel(const CqtParams P) {
  extern __shared__ __attribute__((aligned(16))) float dyn_lds[];
  float* lds0 = dyn_lds;
  float* lds1 = dyn_lds + (size_t)P.lds_rows * CQ_PITCH;

  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int q = lane >> 4, n = lane & 15;

  // longest kernels first: row block is the slow index
  const long long bid = blockIdx.x;
  const int rb = (int)(bid / P.n_ft);
  const long long ft = bid - (long long)rb * P.n_ft;

  const FrameGeom& g = P.g;
  const long long f0 = ft * P.tile_frames;
  const int m_valid = (int)((g.n_frames - f0) < P.tile_frames ? (g.n_frames - f0) : P.tile_frames);
  TileMap tm;
  tm.T = g.T;
  tm.b0 = f0 / g.T;
  tm.t0 = (int)(f0 - tm.b0 * g.T);
  tm.n0 = (g.T - tm.t0) < m_valid ? (g.T - tm.t0) : m_valid;
  tm.extra = P.rb_jspan[rb] - 1;
  const int last_row = tm.frame_row(m_valid - 1);  // a chunk with nj hop-shifts reads rows [0, last_row + nj)

  bool valid[4];
  int a_off[4];
  long long o_off[4];
#pragma unroll
  for (int fb = 0; fb < 4; ++fb) {
    const int fi = wave * 64 + fb * 16 + n;
    valid[fb] = fi < m_valid;
    const long long f = f0 + fi;
    const long long b = valid[fb] ? f / g.T : 0;
    const int t = valid[fb] ? (int)(f - b * g.T) : 0;
    a_off[fb] = (valid[fb] ? tm.frame_row(fi) : 0) * CQ_PITCH + 4 * q;
    o_off[fb] = (b * P.n_bins) * g.T + t;
  }

  const CqtChunk* __restrict__ chunks = P.chunks + (long long)rb * P.n_chunks;
  const float4* __restrict__ bankp = P.bank + P.rb_frag0[rb] * 64 + lane;

  f32x4 acc[4];
#pragma unroll
  for (int fb = 0; fb < 4; ++fb) acc[fb] = (f32x4){0.f, 0.f, 0.f, 0.f};

  const int n_chunks = P.n_chunks;
  float4 R[CQ_NPASS];
  {
    const CqtChunk ck = chunks[0];
    load_chunk<CQ_KC, CQ_NPASS>(R, g, tm, ck.nj > 0 ? last_row + ck.nj : 0, ck.jlo, ck.c0, tid);
    store_chunk<CQ_KC, CQ_PITCH, CQ_NPASS>(R, lds0, P.lds_rows, tid);
  }
  if (n_chunks > 1) {
    const CqtChunk ck = chunks[1];
    load_chunk<CQ_KC, CQ_NPASS>(R, g, tm, ck.nj > 0 ? last_row + ck.nj : 0, ck.jlo, ck.c0, tid);
  }
  // bank fragment pipeline (the allocation is padded by CQ_PREFETCH fragments)
  float4 b0 = bankp[0 * 64], b1 = bankp[1 * 64], b2 = bankp[2 * 64], b3 = bankp[3 * 64];
  bankp += CQ_PREFETCH * 64;
  __syncthreads();

  for (int it = 0; it < n_chunks; ++it) {
    float* cur = (it & 1) ? lds1 : lds0;
    float* nxt = (it & 1) ? lds0 : lds1;
    if (it + 1 < n_chunks) store_chunk<CQ_KC, CQ_PITCH, CQ_NPASS>(R, nxt, P.lds_rows, tid);
    if (it + 2 < n_chunks) {
      const CqtChunk ck = chunks[it + 2];
      load_chunk<CQ_KC, CQ_NPASS>(R, g, tm, ck.nj > 0 ? last_row + ck.nj : 0, ck.jlo, ck.c0, tid);
    }
    const int nj = chunks[it].nj;
    for (int jj = 0; jj < nj; ++jj) {
      float4 a[4];
#pragma unroll
      for (int fb = 0; fb < 4; ++fb)
        a[fb] = *reinterpret_cast<const float4*>(cur + a_off[fb] + jj * CQ_PITCH);
      const float4 bk = b0;
      b0 = b1;
      b1 = b2;
      b2 = b3;
      b3 = *bankp;
      bankp += 64;
#pragma unroll
      for (int fb = 0; fb < 4; ++fb) acc[fb] = __builtin_amdgcn_mfma_f32_16x16x4f32(bk.x, a[fb].x, acc[fb], 0, 0, 0);
#pragma unroll
      for (int fb = 0; fb < 4; ++fb) acc[fb] = __builtin_amdgcn_mfma_f32_16x16x4f32(bk.y, a[fb].y, acc[fb], 0, 0, 0);
#pragma unroll
      for (int fb = 0; fb < 4; ++fb) acc[fb] = __builtin_amdgcn_mfma_f32_16x16x4f32(bk.z, a[fb].z, acc[fb], 0, 0, 0);
#pragma unroll
      for (int fb = 0; fb < 4; ++fb) acc[fb] = __builtin_amdgcn_mfma_f32_16x16x4f32(bk.w, a[fb].w, acc[fb], 0, 0, 0);
    }
    __syncthreads();
  }

  const int bin0 = rb * (CQ_ROWS / 2) + 2 * q;
#pragma unroll
  for (int fb = 0; fb < 4; ++fb) {
    if (!valid[fb]) continue;
    float* __restrict__ op = P.out + o_off[fb];
    if (bin0 < P.n_bins)
      op[(long long)bin0 * g.T] = format_power(acc[fb][0] * acc[fb][0] + acc[fb][1] * acc[fb][1], P.fmt);
    if (bin0 + 1 < P.n_bins)
      op[(long long)(bin0 + 1) * g.T] = format_power(acc[fb][2] * acc[fb][2] + acc[fb][3] * acc[fb][3], P.fmt);
  }
}

// ---------------------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------------------
static constexpr size_t CQ_LDS_BYTES_MAX = 2ull * CQ_LDS_ROWS_MAX * CQ_PITCH * sizeof(float);

hipError_t kernels_init() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(cqt_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                             (int)CQ_LDS_BYTES_MAX);
}

hipError_t launch_stft(const StftParams& p, bool mel, hipStream_t stream) {
  long long blocks;
  if (mel) {
    blocks = p.n_ft * p.n_pass;
  } else {
    const long long ft_per_xcd = (p.n_ft + 7) / 8;
    const long long groups = (ft_per_xcd + 63) / 64;
    blocks = 8 * groups * 64 * p.n_rt;
  }
  if (blocks <= 0 || blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  if (mel)
    hipLaunchKernelGGL(stft_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, stream, p);
  else
    hipLaunchKernelGGL(stft_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, stream, p);
  return hipGetLastError();
}

hipError_t launch_cqt(const CqtParams& p, hipStream_t stream) {
  const long long blocks = p.n_ft * p.n_rb;
  if (blocks <= 0 || blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  if (p.lds_rows > CQ_LDS_ROWS_MAX) return hipErrorInvalidValue;
  const size_t lds = 2ull * p.lds_rows * CQ_PITCH * sizeof(float);
  hipLaunchKernelGGL(cqt_kernel, dim3((unsigned)blocks), dim3(256), lds, stream, p);
  return hipGetLastError();
}

}  // namespace nna
