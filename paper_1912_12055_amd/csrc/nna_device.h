// Device-side building blocks shared by the kernel files: the frame-tile <-> LDS-row mapping,
// the hand-scheduled global loads, the framing loader with mirror reflection, and the
// (Re, Im) -> magnitude / power / log epilogue of one finished STFT row tile.
#pragma once

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

// ---------------------------------------------------------------------------------------
// Work item of a launch whose workgroups are (frame tile, pass) pairs (Mel filterbank passes of 128 filters,
// constant-Q passes of 64 bins).  The passes of a Mel plan differ widely in length (the filters of the top
// pass span half the spectrum) and sweep different row tiles of the bank.  The pass is the slow index,
// longest (highest) pass first: the workgroups resident at any time then belong to one pass and walk the
// same bank tiles together, so the bank streams through the L2s once per wave of workgroups instead of once
// per workgroup, and consecutive ids (dealt round-robin to the 8 XCDs) are frame tiles of equal length.
// Grid: n_ft * n_pass workgroups.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ void pass_work_item(long long bid, long long n_ft, int n_pass, long long& ft, int& pass) {
  const long long p = bid / n_ft;
  pass = n_pass - 1 - (int)p;
  ft = bid - p * n_ft;
}

// ---------------------------------------------------------------------------------------
// Hand-scheduled global loads.  The compiler's own wait-count insertion is conservative at loop
// headers (it waited for nearly every outstanding load at the top of each K iteration, which
// exposed the full L2 latency), so the streaming loads are issued through inline asm and waited
// for with explicit s_waitcnt vmcnt(N).  Loads return in issue order, so "vmcnt(N)" guarantees
// that everything older than the N youngest requests has landed; N must therefore never exceed
// the number of requests issued after the one being waited for.  Every code path below issues
// a fixed number of load instructions so that these counts hold.  The "+v" operands tie the
// wait to the registers it protects: no use of them can be scheduled above it.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ void gload16(f32x4& dst, const void* p) {
  asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(dst) : "v"(p));
}
template <int OFF>
__device__ __forceinline__ void gload16_off(f32x4& dst, const void* p) {
  asm volatile("global_load_dwordx4 %0, %1, off offset:%2" : "=v"(dst) : "v"(p), "n"(OFF));
}
// scalar base + per-lane 32-bit offset form: no 64-bit address registers to read, so the
// request costs the issuing wave (almost) no MFMA issue time
template <int OFF>
__device__ __forceinline__ void gload16_s(f32x4& dst, unsigned lane_off, const void* sbase) {
  asm volatile("global_load_dwordx4 %0, %1, %2 offset:%3" : "=v"(dst) : "v"(lane_off), "s"(sbase), "n"(OFF));
}
// one dword per lane, scalar base + per-lane 32-bit offset
__device__ __forceinline__ void gload4_s(float& dst, unsigned lane_off, const void* sbase) {
  asm volatile("global_load_dword %0, %1, %2" : "=v"(dst) : "v"(lane_off), "s"(sbase));
}
template <int N>
__device__ __forceinline__ void wait_vm(f32x4 (&r)[5], float& x) {
  asm volatile("s_waitcnt vmcnt(%6)" : "+v"(r[0]), "+v"(r[1]), "+v"(r[2]), "+v"(r[3]), "+v"(r[4]), "+v"(x) : "n"(N));
}
template <int N>
__device__ __forceinline__ void wait_vm(f32x4& a) {
  asm volatile("s_waitcnt vmcnt(%1)" : "+v"(a) : "n"(N));
}
template <int N>
__device__ __forceinline__ void wait_vm(f32x4& a, f32x4& b) {
  asm volatile("s_waitcnt vmcnt(%2)" : "+v"(a), "+v"(b) : "n"(N));
}
template <int N>
__device__ __forceinline__ void wait_vm(f32x4& a, f32x4& b, f32x4& c, f32x4& d) {
  asm volatile("s_waitcnt vmcnt(%4)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d) : "n"(N));
}
template <int N>
__device__ __forceinline__ void wait_vm(f32x4 (&r)[5]) {
  asm volatile("s_waitcnt vmcnt(%5)" : "+v"(r[0]), "+v"(r[1]), "+v"(r[2]), "+v"(r[3]), "+v"(r[4]) : "n"(N));
}
template <int N>
__device__ __forceinline__ void wait_vm(f32x4 (&a)[5], f32x4 (&b)[5]) {
  asm volatile("s_waitcnt vmcnt(%10)"
               : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(a[4]), "+v"(b[0]), "+v"(b[1]), "+v"(b[2]), "+v"(b[3]), "+v"(b[4])
               : "n"(N));
}
template <int N>
__device__ __forceinline__ void wait_vm(f32x4 (&a)[6], f32x4 (&b)[6]) {
  asm volatile("s_waitcnt vmcnt(%12)"
               : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(a[4]), "+v"(a[5]), "+v"(b[0]), "+v"(b[1]), "+v"(b[2]),
                 "+v"(b[3]), "+v"(b[4]), "+v"(b[5])
               : "n"(N));
}
template <int N>
__device__ __forceinline__ void wait_vm(f32x4 (&r)[6]) {
  asm volatile("s_waitcnt vmcnt(%6)" : "+v"(r[0]), "+v"(r[1]), "+v"(r[2]), "+v"(r[3]), "+v"(r[4]), "+v"(r[5]) : "n"(N));
}
template <int N>
__device__ __forceinline__ void wait_vm(f32x4 (&r)[7]) {
  asm volatile("s_waitcnt vmcnt(%7)"
               : "+v"(r[0]), "+v"(r[1]), "+v"(r[2]), "+v"(r[3]), "+v"(r[4]), "+v"(r[5]), "+v"(r[6])
               : "n"(N));
}
template <int N>
__device__ __forceinline__ void wait_vm(f32x4 (&r)[8]) {
  asm volatile("s_waitcnt vmcnt(%8)"
               : "+v"(r[0]), "+v"(r[1]), "+v"(r[2]), "+v"(r[3]), "+v"(r[4]), "+v"(r[5]), "+v"(r[6]), "+v"(r[7])
               : "n"(N));
}

// ---------------------------------------------------------------------------------------
// Framing loader.  LDS row r of a tile is S-row sigma of waveform b.  A thread fetches 4
// consecutive columns of one row per pass with ONE 16-byte load.  The 4 padded samples
// i0..i0+3 map, after mirror reflection at either end of the waveform, into one window of 4
// consecutive stored samples:
//   class 0  interior window: load it as it is;
//   class 1  window entirely inside a reflected zone: it is a stored window read backwards --
//            load that window, reverse the 4 elements when the chunk is written to LDS (long CQT
//            kernels pad by tens of hops, so this is the common case at both waveform ends);
//   class 2  window straddling an end (only when L, hop or the padding are not multiples of 4):
//            load the covering window and pick each element with a 2-bit selector.
// The class is decided per wave (ballot), so each chunk takes the cheapest path that serves all
// 64 lanes.  Rows that do not exist read a dummy window: nobody reads their LDS rows.
// The (pass -> row) descriptors are computed once per tile and kept in registers.
// ---------------------------------------------------------------------------------------

__device__ __forceinline__ int reflect_clamped(int j, int L) {
  int r = j < 0 ? -j : (j >= L ? 2 * (L - 1) - j : j);
  return r < 0 ? 0 : (r >= L ? L - 1 : r);  // the clamp is only reachable under zero bank columns
}

template <int NPASS>
struct RowDesc {
  const float* xb[NPASS];  // waveform of the row this thread serves in pass p
  int i0[NPASS];           // padded-signal sample index of (row, this thread's first column) at shift 0, column 0
};

template <int KC, int NPASS>
__device__ __forceinline__ void build_rowdesc(RowDesc<NPASS>& rd, const FrameGeom& g, const TileMap& tm,
                                              int rows_used, int tid) {
  constexpr int V = KC / 4;
  constexpr int RPP = 256 / V;
  const int cv = tid % V, r0 = tid / V;
#pragma unroll
  for (int p = 0; p < NPASS; ++p) {
    const int row = p * RPP + r0;
    long long b;
    int sigma;
    tm.decode(row, b, sigma);
    const bool ok = row < rows_used && b < g.B;
    rd.xb[p] = ok ? g.x + b * g.L : g.x;                     // a row nobody reads: any valid window will do
    rd.i0[p] = ok ? sigma * g.hop + cv * 4 - g.pad : 0;
  }
}

// State of a requested chunk tile that its LDS write needs.
template <int NPASS>
struct TileFix {
  int cls;              // 0, 1 or 2 (see above), uniform over the wave
  unsigned rev;         // class 1: bit p set if this lane's window of pass p is read backwards
  unsigned sel[NPASS];  // class 2: element selectors
};

// `shift` = (first hop-shift of the chunk) * hop + (first column of the chunk).
// Computes the NPASS load addresses of a chunk (no memory access) and how to fix the data up.
template <int NPASS>
__device__ __forceinline__ void prepare_chunk(const float* (&ptr)[NPASS], TileFix<NPASS>& fx, const FrameGeom& g,
                                              const RowDesc<NPASS>& rd, int shift) {
  const int L = (int)g.L;
  unsigned rev = 0;
  bool gen = false;
#pragma unroll
  for (int p = 0; p < NPASS; ++p) {
    const int i0 = rd.i0[p] + shift;
    int src = i0;
    if (i0 < 0) src = -i0 - 3;                      // i0..i0+3 all left of sample 0  -> x[-i0-3 .. -i0] reversed
    else if (i0 > L - 4) src = 2 * (L - 1) - i0 - 3;  // all right of sample L-1    -> x[2(L-1)-i0-3 ..] reversed
    rev |= (src != i0 ? 1u : 0u) << p;
    gen |= (unsigned)src > (unsigned)(L - 4);       // not a whole stored window: straddles an end
    ptr[p] = rd.xb[p] + src;
  }
  fx.rev = rev;
  fx.cls = __builtin_amdgcn_ballot_w64(rev != 0) != 0 ? 1 : 0;
  if (__builtin_amdgcn_ballot_w64(gen) != 0) {
    fx.cls = 2;
#pragma unroll
    for (int p = 0; p < NPASS; ++p) {
      const int i0 = rd.i0[p] + shift;
      const int i_0 = reflect_clamped(i0, L), i_1 = reflect_clamped(i0 + 1, L);
      const int i_2 = reflect_clamped(i0 + 2, L), i_3 = reflect_clamped(i0 + 3, L);
      int w0 = min(min(i_0, i_1), min(i_2, i_3));
      w0 = min(w0, L - 4);
      ptr[p] = rd.xb[p] + w0;
      fx.sel[p] = (unsigned)min(i_0 - w0, 3) | ((unsigned)min(i_1 - w0, 3) << 2) | ((unsigned)min(i_2 - w0, 3) << 4) |
                  ((unsigned)min(i_3 - w0, 3) << 6);
    }
  }
}

// Exactly NPASS loads are issued on every path.
template <int NPASS>
__device__ __forceinline__ void issue_chunk(f32x4 (&R)[NPASS], TileFix<NPASS>& fx, const FrameGeom& g,
                                            const RowDesc<NPASS>& rd, int shift) {
  const float* ptr[NPASS];
  prepare_chunk<NPASS>(ptr, fx, g, rd, shift);
#pragma unroll
  for (int p = 0; p < NPASS; ++p) gload16(R[p], ptr[p]);
}

__device__ __forceinline__ float pick4(const f32x4& v, unsigned k) {
  return k == 0 ? v.x : k == 1 ? v.y : k == 2 ? v.z : v.w;
}

// the value of pass p as it goes to LDS (classes 0 and 1; in class 0 no lane has a bit of `rev` set, and the class
// is not tested here: the compiler turns that test into a second layer of selects, and vector-ALU instructions in
// the kernels' main loops cost the matrix pipe their four cycles each)
template <int NPASS>
__device__ __forceinline__ f32x4 fixed_up(const f32x4& v, const TileFix<NPASS>& fx, int p) {
  const bool r = (fx.rev >> p) & 1u;
  return (f32x4){r ? v.w : v.x, r ? v.z : v.y, r ? v.y : v.z, r ? v.x : v.w};
}

// whole-tile LDS write (prologue, and class 2 in the main loops)
template <int KC, int PITCH, int NPASS>
__device__ __forceinline__ void store_chunk(const f32x4 (&R)[NPASS], const TileFix<NPASS>& fx, float* lds,
                                            int rows_alloc, int tid) {
  constexpr int V = KC / 4;
  constexpr int RPP = 256 / V;
  const int cv = tid % V, r0 = tid / V;
  float* dst = lds + r0 * PITCH + cv * 4;
#pragma unroll
  for (int p = 0; p < NPASS; ++p) {
    f32x4 v;
    if (fx.cls == 2) {
      const unsigned s = fx.sel[p];
      v = (f32x4){pick4(R[p], s & 3), pick4(R[p], (s >> 2) & 3), pick4(R[p], (s >> 4) & 3), pick4(R[p], (s >> 6) & 3)};
    } else {
      v = fixed_up<NPASS>(R[p], fx, p);
    }
    if (p * RPP + r0 < rows_alloc) *reinterpret_cast<f32x4*>(dst + p * RPP * PITCH) = v;
  }
}

template <int FMT>
__device__ __forceinline__ float format_power(float pw) {
  if constexpr (FMT == NNA_OUT_MAGNITUDE)
    return __builtin_amdgcn_sqrtf(pw);  // v_sqrt_f32: 1 ulp, far inside the 1e-3 tolerance
  else if constexpr (FMT == NNA_OUT_POWER)
    return pw;
  else
    return logf(fmaxf(pw, 1e-10f));
}

// Output of one finished STFT row tile: 64 (Re, Im) slots x this wave's 32 frames.  `op` points
// at (waveform, bin 0, frame) of this lane; consecutive lanes hold consecutive frames, so every
// store instruction writes two 128-byte runs.
template <int FMT>
__device__ __forceinline__ void stft_store_tile(const f32x16 (&acc)[ST_RB], float* __restrict__ op, long long T,
                                                int slot_base, int h, int n_half, int packed) {
  float* __restrict__ p = op + (slot_base + 2 * h) * T;
  if (slot_base > 0 && slot_base + ST_ROWS / 2 <= n_half) {
    // interior tile: all 64 slots exist and none is the packed DC/Nyquist slot
#pragma unroll
    for (int rb = 0; rb < ST_RB; ++rb)
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const float re = acc[rb][2 * u], im = acc[rb][2 * u + 1];
        p[(rb * 16 + 4 * (u >> 1) + (u & 1)) * T] = format_power<FMT>(re * re + im * im);
      }
  } else {
#pragma unroll
    for (int rb = 0; rb < ST_RB; ++rb)
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const float re = acc[rb][2 * u], im = acc[rb][2 * u + 1];
        const int k = rb * 16 + 4 * (u >> 1) + (u & 1);
        const int slot = slot_base + 2 * h + k;
        if (slot == 0 && packed) {  // slot 0 packs the two purely real bins: DC and Nyquist
          op[0] = format_power<FMT>(re * re);
          op[n_half * T] = format_power<FMT>(im * im);
        } else if (slot < n_half) {
          p[k * T] = format_power<FMT>(re * re + im * im);
        }
      }
  }
}

// Output of one finished row tile before the magnitude is taken: NNA_OUT_COMPLEX writes rows 2k = Re,
// 2k+1 = Im of bin k (`op` points at (waveform, row 0, frame)); NNA_OUT_PHASE writes atan2(Im, Re).
template <int FMT>
__device__ __forceinline__ void stft_store_tile_complex(const f32x16 (&acc)[ST_RB], float* __restrict__ op, long long T,
                                                        int slot_base, int h, int n_half, int packed) {
#pragma unroll
  for (int rb = 0; rb < ST_RB; ++rb)
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const float re = acc[rb][2 * u], im = acc[rb][2 * u + 1];
      const int slot = slot_base + 2 * h + rb * 16 + 4 * (u >> 1) + (u & 1);
      if (slot == 0 && packed) {  // the two purely real bins 0 and n_half
        if constexpr (FMT == NNA_OUT_COMPLEX) {
          op[0] = re;
          op[T] = 0.f;
          op[(2LL * n_half) * T] = im;
          op[(2LL * n_half + 1) * T] = 0.f;
        } else {
          op[0] = atan2f(0.f, re);
          op[(long long)n_half * T] = atan2f(0.f, im);
        }
      } else if (slot < n_half) {
        if constexpr (FMT == NNA_OUT_COMPLEX) {
          op[(2LL * slot) * T] = re;
          op[(2LL * slot + 1) * T] = im;
        } else {
          op[(long long)slot * T] = atan2f(im, re);
        }
      }
    }
}

// Backward pass: the finished row tile turned into G = dLoss/dC for the same 64 (Re, Im) slots x this
// wave's 32 frames.  `gp` points at (waveform, bin 0, frame) of the upstream gradient for this lane,
// `Gp` at (packed row 0, global frame) of the G buffer.  With P = Re^2 + Im^2 and g the upstream
// gradient of the bin: magnitude  g Re / sqrt(P)  (0 where P = 0), power  2 g Re, log  2 g Re / P
// where P exceeds the floor inside the logarithm (else 0); likewise for Im.  The packed slot 0 holds
// two real bins (0 and n_half), each with P = its own square.  Slots past n_half are written as zeros.
// NNA_OUT_COMPLEX: the output is C itself; NNA_OUT_PHASE: d atan2(Im, Re) = (Re dIm - Im dRe) / P.
template <int FMT>
__device__ __forceinline__ float grad_scale(float g, float pw) {
  if constexpr (FMT == NNA_OUT_MAGNITUDE)
    return pw > 0.f ? g * __builtin_amdgcn_rsqf(pw) : 0.f;
  else if constexpr (FMT == NNA_OUT_POWER)
    return 2.f * g;
  else
    return pw > 1e-10f ? 2.f * g / pw : 0.f;
}

template <int FMT>
__device__ __forceinline__ void stft_grad_tile(const f32x16 (&acc)[ST_RB], const float* __restrict__ gp, long long T,
                                               float* __restrict__ Gp, long long gpitch, int slot_base, int h,
                                               int n_half, int packed, float* __restrict__ pp = nullptr) {
#pragma unroll
  for (int rb = 0; rb < ST_RB; ++rb)
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const float re = acc[rb][2 * u], im = acc[rb][2 * u + 1];
      const int slot = slot_base + 2 * h + rb * 16 + 4 * (u >> 1) + (u & 1);
      float gr = 0.f, gi = 0.f;
      if constexpr (FMT == NNA_OUT_COMPLEX) {
        // the output is C itself (rows 2k, 2k+1 of the upstream gradient)
        if (slot == 0 && packed) {
          gr = gp[0];
          gi = gp[(2LL * n_half) * T];
        } else if (slot < n_half) {
          gr = gp[(2LL * slot) * T];
          gi = gp[(2LL * slot + 1) * T];
        }
      } else if constexpr (FMT == NNA_OUT_PHASE) {
        // d atan2(Im, Re) = (Re dIm - Im dRe) / P; the phase of the two real bins is piecewise constant
        if (!(slot == 0 && packed) && slot < n_half) {
          const float pw = re * re + im * im;
          const float s = pw > 0.f ? gp[slot * T] / pw : 0.f;
          gr = -s * im;
          gi = s * re;
        }
      } else if (slot == 0 && packed) {
        gr = grad_scale<FMT>(gp[0], re * re) * re;
        gi = grad_scale<FMT>(gp[n_half * T], im * im) * im;
        if (pp) {  // the stage's own output, for a caller that needs it next to the gradient
          pp[0] = format_power<FMT>(re * re);
          pp[n_half * T] = format_power<FMT>(im * im);
        }
      } else if (slot < n_half) {
        const float pw = re * re + im * im;
        const float s = grad_scale<FMT>(gp[slot * T], pw);
        gr = s * re;
        gi = s * im;
        if (pp) pp[slot * T] = format_power<FMT>(pw);
      }
      Gp[(long long)(2 * slot) * gpitch] = gr;
      Gp[(long long)(2 * slot + 1) * gpitch] = gi;
    }
}

}  // namespace nna
