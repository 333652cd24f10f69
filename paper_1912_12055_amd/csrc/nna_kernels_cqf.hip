// Constant-Q transform with time-domain kernels (Sec. III-C, eq. (CQT)), the kernels folded about their centres.
//
// Kernel k is a symmetric window times a phase linear in n: about its centre it is exp(-i pi Q) g_k with
// g_k[-m] = conj(g_k[m]).  All kernels are centred in the K taps of a frame, so with
//     e[m] = x[K/2 + m] + x[K/2 - p - m],   o[m] = x[K/2 + m] - x[K/2 - p - m]      (p = N_k mod 2)
//     C_k = exp(-i pi Q) ( sum_m e[m] Re g_k[m] + i sum_m o[m] Im g_k[m] ),   m < N_k / 2:
// half the multiply-adds of the direct form, nothing approximated.  The bank (nna_banks.hip) holds 16-row blocks
// in pairs: the cosine kernels Re g of 16 bins of one parity, and the sine kernels Im g of the same bins.
//
// Folded tap m = j hop + c0 + i (hop-shift j, 16-tap column chunk c0, i < 16).  Per chunk two tiles go to LDS:
// columns [c0, c0 + 16) of the hop rows behind the frame centres (row t + j serves frame t at shift j, as in the
// direct kernel), and the mirrored columns of the hop rows in front of them, written backwards so that column i of
// row t + jspan - 1 - j is the partner of tap i of frame t at shift j.  A wave reads both quads of its four 16-frame
// blocks, forms e and o in registers, and runs 16 MFMAs of the cosine block against e and 16 of the sine block
// against o (v_mfma_f32_16x16x4_f32; wave w owns frames [64 w, 64 w + 64) of the 256-frame tile).
//
// The tiles are single buffered (two of them for one chunk already fill the LDS two workgroups per CU can have):
// the next chunk's tiles are requested into registers when a chunk's sweep starts and written between two barriers
// when it ends; the other workgroup of the CU computes meanwhile.  Bank fragments stream through a ring of four
// requests per wave with hand-placed waits, as in the direct kernel.
#include <type_traits>
#include <utility>

#include "nna_device.h"

namespace nna {

// LDS write of a requested tile.  MIRROR: the tile's columns run against the taps; quad v of a row goes to quad
// 3 - v, elements reversed.
template <int NPASS, bool MIRROR>
__device__ __forceinline__ void cqf_store_tile(const f32x4 (&R)[NPASS], const TileFix<NPASS>& fx, float* lds, int rows_alloc,
                                               int tid) {
  constexpr int V = CQ_KC / 4;
  constexpr int RPP = 256 / V;
  const int cv = tid % V, r0 = tid / V;
  float* dst = lds + r0 * CQ_PITCH + (MIRROR ? V - 1 - cv : cv) * 4;
#pragma unroll
  for (int p = 0; p < NPASS; ++p) {
    f32x4 v;
    if (fx.cls == 2) {
      const unsigned s = fx.sel[p];
      v = (f32x4){pick4(R[p], s & 3), pick4(R[p], (s >> 2) & 3), pick4(R[p], (s >> 4) & 3), pick4(R[p], (s >> 6) & 3)};
    } else {
      v = fixed_up<NPASS>(R[p], fx, p);
    }
    if (MIRROR) v = (f32x4){v.w, v.z, v.y, v.x};
    if (p * RPP + r0 < rows_alloc) *reinterpret_cast<f32x4*>(dst + p * RPP * CQ_PITCH) = v;
  }
}

__global__ __launch_bounds__(256, 2) void cqt_fold_kernel(const CqfParams P) {
  extern __shared__ __attribute__((aligned(16))) float dyn_lds[];
  constexpr int NP = CQF_NPASS;
  int4* s_chunks = reinterpret_cast<int4*>(dyn_lds);  // this item's chunk table
  float* lds_f = dyn_lds + (size_t)P.n_chunks * (sizeof(CqfChunk) / 4);
  float* lds_m = lds_f + (size_t)P.lds_rows * CQ_PITCH;

  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int q = lane >> 4, n = lane & 15;

  // longest kernels first: the work item is the slow index
  const long long bid = blockIdx.x;
  const int item_id = (int)(bid / P.n_ft);
  const long long ft = bid - (long long)item_id * P.n_ft;
  const CqfItem item = P.items[item_id];
  const int n_pair = item.n_pair;
  const int jspan = item.jspan;

  const FrameGeom& g = P.g;
  const long long f0 = ft * P.tile_frames;
  const int m_valid = (int)((g.n_frames - f0) < P.tile_frames ? (g.n_frames - f0) : P.tile_frames);
  TileMap tm;
  tm.T = g.T;
  tm.b0 = f0 / g.T;
  tm.t0 = (int)(f0 - tm.b0 * g.T);
  tm.n0 = (g.T - tm.t0) < m_valid ? (g.T - tm.t0) : m_valid;
  tm.extra = jspan - 1;
  const int rows_used = tm.frame_row(m_valid - 1) + tm.extra + 1;
  RowDesc<NP> rd;
  build_rowdesc<CQ_KC, NP>(rd, g, tm, rows_used, tid);

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
    o_off[fb] = b * P.out_wave_stride + (long long)P.row_offset * g.T + t;
  }

  const int n_chunks = item.n_chunks;
  const int4* __restrict__ tbl_src = reinterpret_cast<const int4*>(P.chunks + (long long)item_id * P.n_chunks);
  for (int i = tid; i < n_chunks; i += 256) s_chunks[i] = tbl_src[i];
  const unsigned lane_off = (unsigned)lane * 16u;
  const char* bank_s = reinterpret_cast<const char*>(P.bank) + item.frag0 * (64 * 16);

  f32x4 acc[4][4];  // [2 pair + (0 cosine, 1 sine)][frame block]
#pragma unroll
  for (int r = 0; r < 4; ++r)
#pragma unroll
    for (int fb = 0; fb < 4; ++fb) acc[r][fb] = (f32x4){0.f, 0.f, 0.f, 0.f};
  __syncthreads();  // the chunk table is complete

  // sample offsets of the two tiles of the chunk at column c0 (see the loader: row sigma, column u of a tile is
  // padded-signal sample sigma hop + shift + u): behind the centres K/2 + c0; in front of them the 16 samples that
  // end at K/2 - parity - c0, of the row jspan - 1 shifts down
  const int sh_f = P.centre;
  const int sh_m = P.centre - (jspan - 1) * g.hop - item.parity - (CQ_KC - 1);
  auto c0_of = [&](int i) { return __builtin_amdgcn_readfirstlane(s_chunks[i].x); };

  f32x4 Rf[NP], Rm[NP];
  TileFix<NP> fxf, fxm;
  {
    const int c0 = c0_of(0);
    issue_chunk<NP>(Rf, fxf, g, rd, sh_f + c0);
    issue_chunk<NP>(Rm, fxm, g, rd, sh_m - c0);
  }
  f32x4 bq[CQ_PREFETCH];
#pragma unroll
  for (int i = 0; i < CQ_PREFETCH; ++i) {
    gload16_s<0>(bq[i], lane_off, bank_s);
    bank_s += 64 * 16;
  }
  static_assert(CQ_PREFETCH == 4, "a ring is two pair groups: slots 0, 1 and 2, 3");

  // Loads retire in order.  When a fragment is waited for, the requests younger than it are the ring's other three;
  // in the first ring of a chunk also the 2 NP tile requests issued just before it.  At the top of the loop the
  // tile requests are followed by at least one ring's re-requests (every chunk starts with one whole ring).
  constexpr int W_RING = CQ_PREFETCH - 1;
  constexpr int W_FIRST = CQ_PREFETCH - 1 + 2 * NP;
  const float* const mir0 = lds_m + (jspan - 1) * CQ_PITCH;

  for (int it = 0; it < n_chunks; ++it) {
    wait_vm<CQ_PREFETCH>(Rf, Rm);
    __syncthreads();  // every wave has finished with the previous chunk's tiles
    cqf_store_tile<NP, false>(Rf, fxf, lds_f, P.lds_rows, tid);
    cqf_store_tile<NP, true>(Rm, fxm, lds_m, P.lds_rows, tid);
    __syncthreads();
    {
      const int c0 = c0_of(it + 1 < n_chunks ? it + 1 : it);
      issue_chunk<NP>(Rf, fxf, g, rd, sh_f + c0);
      issue_chunk<NP>(Rm, fxm, g, rd, sh_m - c0);
    }
    const int4 d = s_chunks[it];
    const int njw[2] = {__builtin_amdgcn_readfirstlane(d.y), __builtin_amdgcn_readfirstlane(d.z)};
    __builtin_amdgcn_sched_barrier(0);

    f32x4 af[4], am[4];
    // one pair group: shift jj of block pair U, fragments in ring slots S (cosine) and S + 1 (sine)
    auto pgroup = [&](auto u_tag, auto s_tag, auto first_tag, int jj, int nr) {
      constexpr int U = decltype(u_tag)::value;
      constexpr int S = decltype(s_tag)::value;
      constexpr int W = decltype(first_tag)::value ? W_FIRST : W_RING;
      const bool run = jj < nr;
      int jn = jj + 1 < nr ? jj + 1 : nr - 1;  // the next group's shift; padding groups re-read the last one
      jn = jn < 0 ? 0 : jn;
      f32x4 e[4], o[4];
#pragma unroll
      for (int fb = 0; fb < 4; ++fb) {
        e[fb] = af[fb] + am[fb];
        o[fb] = af[fb] - am[fb];
      }
      // both folds are formed here, in front of the two runs of matrix instructions (the compiler would sink each
      // add in front of the MFMA that reads it, and a wave's MFMAs would then come one VALU result apart)
      asm volatile("" : "+v"(e[0]), "+v"(e[1]), "+v"(e[2]), "+v"(e[3]), "+v"(o[0]), "+v"(o[1]), "+v"(o[2]), "+v"(o[3]));
      wait_vm<W>(bq[S]);
      __builtin_amdgcn_sched_barrier(0);
      if (run) {
#pragma unroll
        for (int m = 0; m < 16; ++m) {
          const int k = m >> 2, fb = m & 3;
          acc[2 * U][fb] = __builtin_amdgcn_mfma_f32_16x16x4f32(bq[S][k], e[fb][k], acc[2 * U][fb], 0, 0, 0);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
      gload16_s<0>(bq[S], lane_off, bank_s);
      bank_s += 64 * 16;
#pragma unroll
      for (int fb = 0; fb < 4; ++fb) {
        af[fb] = *reinterpret_cast<const f32x4*>(lds_f + a_off[fb] + jn * CQ_PITCH);
        am[fb] = *reinterpret_cast<const f32x4*>(mir0 + a_off[fb] - jn * CQ_PITCH);
      }
      wait_vm<W>(bq[S + 1]);
      __builtin_amdgcn_sched_barrier(0);
      if (run) {
#pragma unroll
        for (int m = 0; m < 16; ++m) {
          const int k = m >> 2, fb = m & 3;
          acc[2 * U + 1][fb] = __builtin_amdgcn_mfma_f32_16x16x4f32(bq[S + 1][k], o[fb][k], acc[2 * U + 1][fb], 0, 0, 0);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
      gload16_s<0>(bq[S + 1], lane_off, bank_s);
      bank_s += 64 * 16;
      __builtin_amdgcn_sched_barrier(0);
    };
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using I2 = std::integral_constant<int, 2>;
    auto pair_block = [&](auto u_tag) {
      constexpr int U = decltype(u_tag)::value;
      const int nj = njw[U] & 0xffff, nr = njw[U] >> 16;
      // (the first pair of a listed chunk always has one whole ring, so that the ring's re-requests follow the
      // tile requests on every path)
      if (U > 0 && (U >= n_pair || nj == 0)) return;
#pragma unroll
      for (int fb = 0; fb < 4; ++fb) {
        af[fb] = *reinterpret_cast<const f32x4*>(lds_f + a_off[fb]);
        am[fb] = *reinterpret_cast<const f32x4*>(mir0 + a_off[fb]);
      }
      int jj = 0;
      if (U == 0) {  // the chunk's first ring: the tile requests are younger than its fragments
        pgroup(u_tag, I0{}, I1{}, 0, nr);
        pgroup(u_tag, I2{}, I1{}, 1, nr);
        jj = 2;
      }
      for (; jj < nj; jj += 2) {
        pgroup(u_tag, I0{}, I0{}, jj, nr);
        pgroup(u_tag, I2{}, I0{}, jj + 1, nr);
      }
    };
    pair_block(I0{});
    pair_block(I1{});
  }

  // drain the requests that are never consumed
  wait_vm<0>(Rf, Rm);
#pragma unroll
  for (int i = 0; i < CQ_PREFETCH; ++i) wait_vm<0>(bq[i]);

  // lane (q, n), register r of a block: row 4 q + r of its group, frame n of the wave's frame block.  With
  // S_c, S_s the two sums: C = exp(-i pi Q) (S_c + i S_s).
  const int fmt = P.fmt;
  const float rc = P.rot_c, rs = P.rot_s;
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    if (u >= n_pair) continue;
    const int4 bins = reinterpret_cast<const int4*>(P.bins)[(item.grp_first + u) * 4 + q];
    const int bin[4] = {bins.x, bins.y, bins.z, bins.w};
#pragma unroll
    for (int fb = 0; fb < 4; ++fb) {
      if (!valid[fb]) continue;
      float* __restrict__ op = P.out + o_off[fb];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        if (bin[r] < 0) continue;
        const float sc = acc[2 * u][fb][r], ss = acc[2 * u + 1][fb][r];
        const float re = rc * sc + rs * ss, im = rc * ss - rs * sc;
        if (fmt == NNA_OUT_COMPLEX) {
          op[(2LL * bin[r]) * g.T] = re;
          op[(2LL * bin[r] + 1) * g.T] = im;
        } else if (fmt == NNA_OUT_PHASE) {
          op[(long long)bin[r] * g.T] = atan2f(im, re);
        } else {
          const float pw = re * re + im * im;
          op[(long long)bin[r] * g.T] = fmt == NNA_OUT_MAGNITUDE ? format_power<NNA_OUT_MAGNITUDE>(pw)
                                        : fmt == NNA_OUT_POWER   ? pw
                                                                 : format_power<NNA_OUT_LOG>(pw);
        }
      }
    }
  }
}

static constexpr size_t CQF_DYN_LDS_MAX = 80 * 1024;  // two workgroups per CU

hipError_t cqf_kernels_init() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(cqt_fold_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                             (int)CQF_DYN_LDS_MAX);
}

hipError_t launch_cqt_fold(const CqfParams& p, hipStream_t stream) {
  clear_stale_error();
  const long long blocks = p.n_ft * p.n_items;
  if (blocks <= 0 || blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  if (p.lds_rows < 64 || p.lds_rows > CQF_LDS_ROWS || p.lds_rows % 64 || p.n_chunks < 1 || p.n_chunks > CQF_TABLE_CAP)
    return hipErrorInvalidValue;
  if (p.tile_frames < 1 || p.tile_frames > CQ_FRAMES || p.centre % p.g.hop) return hipErrorInvalidValue;
  const size_t lds = (size_t)p.n_chunks * sizeof(CqfChunk) + 2ull * p.lds_rows * CQ_PITCH * sizeof(float);
  if (lds > CQF_DYN_LDS_MAX) return hipErrorInvalidValue;
  hipLaunchKernelGGL(cqt_fold_kernel, dim3((unsigned)blocks), dim3(256), lds, stream, p);
  return hipGetLastError();
}

}  // namespace nna
