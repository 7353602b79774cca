// Operator kernels for gfx950 (CDNA4) and their launcher.
//
// The paper runs vendor-library kernels (Sec. 5.1); these are this library's own.
// Dense contractions (convolution as implicit GEMM, GEMM, batched GEMM) use the
// matrix cores; everything else is a coalesced 16-byte-per-lane streaming kernel
// with wavefront (64-lane) reductions where rows are reduced.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>
#include "kernel_args.h"
#include "launch.h"

namespace opara {

typedef _Float16 half_t;
typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

// Position of a workgroup in its operator's launch grid.  An ordinary launch fills it
// from blockIdx/gridDim; the persistent executor hands out grid positions itself.
struct Blk {
  int x, y, z, gx, gy;
  bool remap;                              // apply the XCD-aware tile remap (hardware launch order only)
};
__device__ __forceinline__ Blk launch_blk() {
  return Blk{(int)blockIdx.x, (int)blockIdx.y, (int)blockIdx.z, (int)gridDim.x, (int)gridDim.y, true};
}

template <typename T> struct Vec16;
template <> struct Vec16<half_t> { typedef half8 type; typedef half4 quad; static constexpr int N = 8; };
template <> struct Vec16<float> { typedef floatx4 type; typedef floatx4 quad; static constexpr int N = 4; };

// Access policy of a body.  Ordinary launches use plain loads and stores: kernel
// boundaries make results visible.  Inside the persistent executor an operator's inputs
// were written by other workgroups of the same launch, possibly on another XCD with its
// own L2; there every access to an activation is an agent-scope (device-coherent) access,
// which the hardware completes at the point all XCDs share, so that a completion counter
// published after a wait for the stores is all the synchronisation a consumer needs: no
// cache write-back or invalidate.  Weights are never written and stay plain (L2-cached).
constexpr int kCohAct = 1;     // first operand, residual inputs, row/element inputs, outputs
constexpr int kCohW = 2;       // second operand too (batched GEMM of two activations)
constexpr int kCohStore = 4;   // outputs only: loads stay plain and follow a cache invalidate

template <bool COH, typename V, typename P>
__device__ __forceinline__ V ldg(const P *p) {
  if constexpr (!COH) {
    return *(const V *)p;
  } else {
    V v;
    if constexpr (sizeof(V) == 16) {
      uint64_t q[2];
      q[0] = __hip_atomic_load((const uint64_t *)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      q[1] = __hip_atomic_load((const uint64_t *)p + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __builtin_memcpy(&v, q, 16);
    } else if constexpr (sizeof(V) == 8) {
      const uint64_t q = __hip_atomic_load((const uint64_t *)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __builtin_memcpy(&v, &q, 8);
    } else if constexpr (sizeof(V) == 4) {
      const uint32_t q = __hip_atomic_load((const uint32_t *)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __builtin_memcpy(&v, &q, 4);
    } else {
      static_assert(sizeof(V) == 2, "access width");
      const uint16_t q = __hip_atomic_load((const uint16_t *)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __builtin_memcpy(&v, &q, 2);
    }
    return v;
  }
}

template <bool COH, typename V, typename P>
__device__ __forceinline__ void stg(P *p, const V &v) {
  if constexpr (!COH) {
    *(V *)p = v;
  } else if constexpr (sizeof(V) == 16) {
    // One 16-byte write-through store (what a relaxed agent-scope atomic store compiles to for
    // 8 bytes, `global_store_dwordx2 ... sc1`, in its four-dword form): the language has no
    // 16-byte atomic, and two 8-byte ones reach memory as two partial-line writes.  The nop
    // covers the wait state a store of more than 8 bytes needs before its data registers
    // may be overwritten.
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 q = __builtin_bit_cast(u32x4, v);
    asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" : : "v"(p), "v"(q) : "memory");
  } else if constexpr (sizeof(V) == 8) {
    uint64_t q;
    __builtin_memcpy(&q, &v, 8);
    __hip_atomic_store((uint64_t *)p, q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  } else if constexpr (sizeof(V) == 4) {
    uint32_t q;
    __builtin_memcpy(&q, &v, 4);
    __hip_atomic_store((uint32_t *)p, q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  } else {
    static_assert(sizeof(V) == 2, "access width");
    uint16_t q;
    __builtin_memcpy(&q, &v, 2);
    __hip_atomic_store((uint16_t *)p, q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

// ---------------------------------------------------------------------------------
// Implicit GEMM on the matrix cores.
//
// Workgroup tile: BN output columns (channels) x BM output rows (pixels); K is walked
// in slices of 64 bytes per row (32 halves / 16 floats).  Both operands are staged in
// LDS with K fastest and an 80-byte row pitch, so that the 16-byte fragment reads of
// 16 consecutive rows fall into distinct banks.  Weights feed the MFMA "A" side and
// pixels the "B" side: each lane then owns four consecutive output channels of one
// pixel, which is a contiguous 8/16-byte store in the [row][channel] output.
// The mapping of K positions onto MFMA K slots is the same for both operands, which is
// all a dot product needs, so the same 16-byte fragment load serves fp16 and fp32.
// ---------------------------------------------------------------------------------
template <typename T> __device__ __forceinline__ floatx4 mma16(typename Vec16<T>::type a, typename Vec16<T>::type b, floatx4 c);
template <> __device__ __forceinline__ floatx4 mma16<half_t>(half8 a, half8 b, floatx4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}
template <> __device__ __forceinline__ floatx4 mma16<float>(floatx4 a, floatx4 b, floatx4 c) {
  c = __builtin_amdgcn_mfma_f32_16x16x4f32(a[0], b[0], c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_16x16x4f32(a[1], b[1], c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_16x16x4f32(a[2], b[2], c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_16x16x4f32(a[3], b[3], c, 0, 0, 0);
  return c;
}

// Thread index as a body sees it.  Inside the persistent kernel (COH != 0) the LDS-staged
// 64 x 64 contraction takes it through a statement the optimiser cannot see through: what it
// derives from it then stays inside the body instead of becoming an invariant of the
// work-item loop that is held in registers, or spilled at kernel entry (120 bytes per
// thread, 16 MB per launch), across every other operator's body.  Doing the same in every
// body costs 7 % (each tile recomputes its index arithmetic on the critical path); in this
// one it removes the spills and is 1-2 % faster on the CNN configs (measured).
template <int COH> __device__ __forceinline__ int body_thread() {
  int t = threadIdx.x;
  if constexpr (COH != 0) {
    asm volatile("" : "+v"(t));
    __builtin_assume(t >= 0 && t < 1024);
  }
  return t;
}

template <typename T, int BN, int BM, int WN, int WM, bool VEC, int COH, typename AR>
__device__ __forceinline__ void igemm_body(const AR &a, const Blk &b, unsigned char *lds) {
  typedef typename Vec16<T>::type V;
  typedef typename Vec16<T>::quad Q;
  constexpr int VE = Vec16<T>::N;
  constexpr int BKE = 4 * VE;              // K elements per slice
  constexpr int NT = WN * WM * 64;
  constexpr int ROWB = 80;                 // LDS row pitch in bytes (64 data + 16 pad)
  constexpr int CHW = BN * 4 / NT;         // 16-byte chunks of the weight tile per thread
  constexpr int CHX = BM * 4 / NT;
  constexpr int FN = BN / WN / 16, FM = BM / WM / 16;
  static_assert((BN * 4) % NT == 0 && (BM * 4) % NT == 0, "tile/threads mismatch");
  unsigned char (*smem)[(BN + BM) * ROWB] = (unsigned char (*)[(BN + BM) * ROWB])lds;   // [2][...]

  const int t = body_thread<COH>(), lane = t & 63, wave = t >> 6;
  const int wn0 = (wave % WN) * (BN / WN), wm0 = (wave / WN) * (BM / WM);
  const int m0 = b.x * BM, n0 = b.y * BN;
  constexpr bool CA = (COH & kCohAct) != 0, CW = (COH & kCohW) != 0, CS = (COH & (kCohAct | kCohStore)) != 0;
  const T *__restrict__ x = (const T *)a.x + (int64_t)b.z * a.a_bs;
  const T *__restrict__ w = (const T *)a.w + (int64_t)b.z * a.b_bs;
  T *__restrict__ y = (T *)a.y + (int64_t)b.z * a.y_bs;
  const int kc = t & 3;                    // which 16-byte chunk of a 64-byte K slice
  const int row0 = t >> 2;                 // first tile row this thread moves
  constexpr int RSTEP = NT / 4;

  int ih0[CHX], iw0[CHX];
  const T *ximg[CHX];
  if (a.gather) {
#pragma unroll
    for (int i = 0; i < CHX; ++i) {
      const int m = m0 + row0 + i * RSTEP;
      const int img = m / a.HoWo, pix = m - img * a.HoWo;
      const int oh = pix / a.Wo, ow = pix - oh * a.Wo;
      ih0[i] = oh * a.sh - a.ph;
      iw0[i] = ow * a.sw - a.pw;
      ximg[i] = x + (int64_t)img * a.img_stride;
    }
  }
  // running decomposition of this thread's K position (vector path, gather only)
  int g_ci = 0, g_s = 0, g_r = 0;
  if (VEC && a.gather) {
    const int k = kc * VE;
    g_ci = k % a.Cin;
    const int rs = k / a.Cin;
    g_s = rs % a.kw;
    g_r = rs / a.kw;
  }

  V wreg[CHW], xreg[CHX];
  const V vzero = {};

  auto load_global = [&](int kt) {
    const int kbase = kt * BKE + kc * VE;
    // ---- pixel (im2col / matrix row) chunks
#pragma unroll
    for (int i = 0; i < CHX; ++i) {
      const int m = m0 + row0 + i * RSTEP;
      V v = vzero;
      if (VEC) {
        if (m < a.M && kbase < a.K) {
          if (!a.gather) {
            v = ldg<CA, V>(x + (int64_t)m * a.lda + kbase);
          } else {
            const int ih = ih0[i] + g_r, iw = iw0[i] + g_s;
            if ((unsigned)ih < (unsigned)a.H && (unsigned)iw < (unsigned)a.W)
              v = ldg<CA, V>(ximg[i] + ((int64_t)ih * a.W + iw) * a.Cin + g_ci);
          }
        }
      } else {
        if (m < a.M) {
#pragma unroll
          for (int e = 0; e < VE; ++e) {
            const int k = kbase + e;
            if (k < a.K) {
              if (!a.gather) {
                v[e] = ldg<CA, T>(x + (int64_t)m * a.lda + k);
              } else {
                const int ci = k % a.Cin, rs = k / a.Cin;
                const int ih = ih0[i] + rs / a.kw, iw = iw0[i] + rs % a.kw;
                if ((unsigned)ih < (unsigned)a.H && (unsigned)iw < (unsigned)a.W)
                  v[e] = ldg<CA, T>(ximg[i] + ((int64_t)ih * a.W + iw) * a.Cin + ci);
              }
            }
          }
        }
      }
      xreg[i] = v;
    }
    // ---- weight chunks
#pragma unroll
    for (int i = 0; i < CHW; ++i) {
      V v = vzero;
      if (!a.b_kmajor) {
        const int n = n0 + row0 + i * RSTEP;
        if (VEC) {
          if (n < a.N && kbase < a.K) v = ldg<CW, V>(w + (int64_t)n * a.ldb + kbase);
        } else if (n < a.N) {
#pragma unroll
          for (int e = 0; e < VE; ++e)
            if (kbase + e < a.K) v[e] = ldg<CW, T>(w + (int64_t)n * a.ldb + kbase + e);
        }
      } else {
        // operand stored [K][N]: a chunk runs along N at one K position
        const int c = t + i * NT;
        const int krow = c / (BN / VE), nch = c % (BN / VE);
        const int k = kt * BKE + krow, n = n0 + nch * VE;
        if (k < a.K) {
          if (VEC) {
            if (n < a.N) v = ldg<CW, V>(w + (int64_t)k * a.ldb + n);
          } else {
#pragma unroll
            for (int e = 0; e < VE; ++e)
              if (n + e < a.N) v[e] = ldg<CW, T>(w + (int64_t)k * a.ldb + n + e);
          }
        }
      }
      wreg[i] = v;
    }
    if (VEC && a.gather) {  // advance the running K decomposition by one slice
      g_ci += BKE;
      while (g_ci >= a.Cin) {
        g_ci -= a.Cin;
        if (++g_s == a.kw) { g_s = 0; ++g_r; }
      }
    }
  };

  auto store_lds = [&](int buf) {
    unsigned char *Wb = smem[buf];
    unsigned char *Xb = Wb + BN * ROWB;
#pragma unroll
    for (int i = 0; i < CHX; ++i) *(V *)(Xb + (row0 + i * RSTEP) * ROWB + kc * 16) = xreg[i];
#pragma unroll
    for (int i = 0; i < CHW; ++i) {
      if (!a.b_kmajor) {
        *(V *)(Wb + (row0 + i * RSTEP) * ROWB + kc * 16) = wreg[i];
      } else {
        const int c = t + i * NT;
        const int krow = c / (BN / VE), nch = c % (BN / VE);
#pragma unroll
        for (int e = 0; e < VE; ++e) *(T *)(Wb + (nch * VE + e) * ROWB + krow * (int)sizeof(T)) = wreg[i][e];
      }
    }
  };

  floatx4 acc[FN][FM];
#pragma unroll
  for (int i = 0; i < FN; ++i)
#pragma unroll
    for (int j = 0; j < FM; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};

  const int nk = (a.K + BKE - 1) / BKE;
  load_global(0);
  store_lds(0);
  __syncthreads();
  int buf = 0;
  for (int kt = 0; kt < nk; ++kt) {
    const bool more = kt + 1 < nk;
    if (more) load_global(kt + 1);
    {
      const unsigned char *Wb = smem[buf];
      const unsigned char *Xb = Wb + BN * ROWB;
      V af[FN], bf[FM];
#pragma unroll
      for (int i = 0; i < FN; ++i) af[i] = *(const V *)(Wb + (wn0 + i * 16 + (lane & 15)) * ROWB + (lane >> 4) * 16);
#pragma unroll
      for (int j = 0; j < FM; ++j) bf[j] = *(const V *)(Xb + (wm0 + j * 16 + (lane & 15)) * ROWB + (lane >> 4) * 16);
#pragma unroll
      for (int i = 0; i < FN; ++i)
#pragma unroll
        for (int j = 0; j < FM; ++j) acc[i][j] = mma16<T>(af[i], bf[j], acc[i][j]);
    }
    if (more) store_lds(buf ^ 1);
    __syncthreads();
    buf ^= 1;
  }

  // ---- epilogue: alpha, bias, residual inputs, ReLU, convert, store
#pragma unroll
  for (int i = 0; i < FN; ++i) {
    const int n = n0 + wn0 + i * 16 + (lane >> 4) * 4;
#pragma unroll
    for (int j = 0; j < FM; ++j) {
      const int m = m0 + wm0 + j * 16 + (lane & 15);
      if (m >= a.M || n >= a.N) continue;
      float v[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float r = acc[i][j][e] * a.alpha;
        if (n + e < a.N) {
          if (a.bias) r += a.bias[n + e];
          for (int q = 0; q < a.n_extra; ++q) r += (float)ldg<CA, T>((const T *)a.extra[q] + (int64_t)m * a.N + n + e);
        }
        if (a.relu) r = fmaxf(r, 0.f);
        v[e] = r;
      }
      T *dst = y + (int64_t)m * a.ldy + n;
      if (n + 3 < a.N && ((uintptr_t)dst & (4 * sizeof(T) - 1)) == 0) {
        Q q4 = {(T)v[0], (T)v[1], (T)v[2], (T)v[3]};
        stg<CS, Q>(dst, q4);
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (n + e < a.N) stg<CS, T>(dst + e, (T)v[e]);
      }
    }
  }
}

// Workgroups are handed to the eight XCDs round-robin in launch order; each XCD has its
// own L2.  Remap the linear workgroup index so that every XCD works on a contiguous
// range of tiles (row tiles of one column tile first): neighbours that share operand
// rows then share an L2 instead of fetching them eight times.
__device__ __forceinline__ void xcd_tile(const Blk &b, int &tx, int &ty) {
  constexpr int kXcds = 8;
  if (!b.remap) { tx = b.x; ty = b.y; return; }
  const int nx = b.gx, total = b.gx * b.gy;
  const int lin = b.y * nx + b.x;
  const int xcd = lin % kXcds, idx = lin / kXcds;
  const int q = total / kXcds, r = total % kXcds;
  const int tile = xcd * q + (xcd < r ? xcd : r) + idx;
  tx = tile % nx;
  ty = tile / nx;
}

struct KPos { int ci, s, r; };

__device__ __forceinline__ void kpos_advance(KPos &p, int delta, int Cin, int kw) {
  p.ci += delta;
  while (p.ci >= Cin) {
    p.ci -= Cin;
    if (++p.s == kw) { p.s = 0; ++p.r; }
  }
}

// ---------------------------------------------------------------------------------
// Throughput-oriented tiled implicit GEMM: BN x BM tile, four wavefronts, K stages of
// 128 bytes per row, LDS double buffer with a 144-byte row pitch, and global loads
// running DEPTH-1 stages ahead in DEPTH rotating register sets (at one workgroup per
// compute unit the loop is bound by memory latency, so the bytes in flight set the
// speed).  Vector loads only, second operand stored [N][K].
// ---------------------------------------------------------------------------------
template <typename T, int BN, int BM, int WN, int WM, int DEPTH, int COH, typename AR>
__device__ __forceinline__ void igemm_pipe_body(const AR &a, const Blk &b, unsigned char *lds) {
  typedef typename Vec16<T>::type V;
  typedef typename Vec16<T>::quad Q;
  constexpr int VE = Vec16<T>::N;
  constexpr int KCH = 8;                   // 16-byte chunks per row and stage
  constexpr int BKE = KCH * VE;
  constexpr int NT = WN * WM * 64;
  constexpr int ROWB = KCH * 16 + 16;
  constexpr int CHW = BN * KCH / NT, CHX = BM * KCH / NT;
  constexpr int FN = BN / WN / 16, FM = BM / WM / 16;
  constexpr int RSTEP = NT / KCH;
  static_assert((BN * KCH) % NT == 0 && (BM * KCH) % NT == 0, "tile/threads mismatch");
  unsigned char (*smem)[(BN + BM) * ROWB] = (unsigned char (*)[(BN + BM) * ROWB])lds;   // [2][...]

  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wn0 = (wave % WN) * (BN / WN), wm0 = (wave / WN) * (BM / WM);
  int tile_x, tile_y;
  xcd_tile(b, tile_x, tile_y);
  const int m0 = tile_x * BM, n0 = tile_y * BN;
  constexpr bool CA = (COH & kCohAct) != 0, CW = (COH & kCohW) != 0, CS = (COH & (kCohAct | kCohStore)) != 0;
  const T *__restrict__ x = (const T *)a.x + (int64_t)b.z * a.a_bs;
  const T *__restrict__ w = (const T *)a.w + (int64_t)b.z * a.b_bs;
  T *__restrict__ y = (T *)a.y + (int64_t)b.z * a.y_bs;
  const int kc = t % KCH, row0 = t / KCH;

  // Per-thread rows, clamped into range: every global load below is unconditional and
  // reads a valid address; out-of-range rows, K tails and padding taps are zeroed when
  // the registers are written to LDS.  (A load guarded by a branch makes the compiler
  // wait for it right inside the branch, which serialises the whole prefetch.)
  int ih0[CHX], iw0[CHX];
  const T *xrow[CHX], *ximg[CHX];
  const T *wrow[CHW];
  unsigned rowmask = 0;                       // bit i: pixel row i valid, bit 8+i: weight row i valid
#pragma unroll
  for (int i = 0; i < CHX; ++i) {
    const int m = m0 + row0 + i * RSTEP;
    const bool ok = m < a.M;
    const int mm = ok ? m : 0;
    rowmask |= (unsigned)ok << i;
    xrow[i] = x + (int64_t)mm * a.lda;
    const int img = mm / a.HoWo, pix = mm - img * a.HoWo;   // used only when gathering
    const int oh = pix / a.Wo, ow = pix - oh * a.Wo;
    ih0[i] = oh * a.sh - a.ph;
    iw0[i] = ow * a.sw - a.pw;
    ximg[i] = x + (int64_t)img * a.img_stride;
  }
#pragma unroll
  for (int i = 0; i < CHW; ++i) {
    const int n = n0 + row0 + i * RSTEP;
    const bool ok = n < a.N;
    rowmask |= (unsigned)ok << (8 + i);
    wrow[i] = w + (int64_t)(ok ? n : 0) * a.ldb;
  }
  KPos pos = {0, 0, 0};
  if (a.gather) {
    const int k = kc * VE;
    pos.ci = k % a.Cin;
    const int rs = k / a.Cin;
    pos.s = rs % a.kw;
    pos.r = rs / a.kw;
  }
  const V vzero = {};

  // Stages must be requested in increasing order.  Returns the validity mask of the set.
  auto load_global = [&](int kt, V *wr, V *xr) -> unsigned {
    const int kbase = kt * BKE + kc * VE;
    const bool kok = kbase < a.K;
    const int ks = kok ? kbase : 0;
    unsigned mask = kok ? rowmask : 0u;
    if (!a.gather) {
#pragma unroll
      for (int i = 0; i < CHX; ++i) xr[i] = ldg<CA, V>(xrow[i] + ks);
    } else {
#pragma unroll
      for (int i = 0; i < CHX; ++i) {
        const int ih = ih0[i] + pos.r, iw = iw0[i] + pos.s;
        const bool inb = kok && (unsigned)ih < (unsigned)a.H && (unsigned)iw < (unsigned)a.W;
        const int64_t off = inb ? ((int64_t)ih * a.W + iw) * a.Cin + pos.ci : 0;
        if (!inb) mask &= ~(1u << i);
        xr[i] = ldg<CA, V>(ximg[i] + off);
      }
      kpos_advance(pos, BKE, a.Cin, a.kw);
    }
#pragma unroll
    for (int i = 0; i < CHW; ++i) wr[i] = ldg<CW, V>(wrow[i] + ks);
    return mask;
  };
  auto store_lds = [&](int buf, const V *wr, const V *xr, unsigned mask) {
    unsigned char *Wb = smem[buf];
    unsigned char *Xb = Wb + BN * ROWB;
#pragma unroll
    for (int i = 0; i < CHX; ++i)
      *(V *)(Xb + (row0 + i * RSTEP) * ROWB + kc * 16) = ((mask >> i) & 1u) ? xr[i] : vzero;
#pragma unroll
    for (int i = 0; i < CHW; ++i)
      *(V *)(Wb + (row0 + i * RSTEP) * ROWB + kc * 16) = ((mask >> (8 + i)) & 1u) ? wr[i] : vzero;
  };

  floatx4 acc[FN][FM];
#pragma unroll
  for (int i = 0; i < FN; ++i)
#pragma unroll
    for (int j = 0; j < FM; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};
  auto compute = [&](int buf) {
    const unsigned char *Wb = smem[buf];
    const unsigned char *Xb = Wb + BN * ROWB;
#pragma unroll
    for (int ks = 0; ks < KCH / 4; ++ks) {
      V af[FN], bf[FM];
#pragma unroll
      for (int i = 0; i < FN; ++i)
        af[i] = *(const V *)(Wb + (wn0 + i * 16 + (lane & 15)) * ROWB + ks * 64 + (lane >> 4) * 16);
#pragma unroll
      for (int j = 0; j < FM; ++j)
        bf[j] = *(const V *)(Xb + (wm0 + j * 16 + (lane & 15)) * ROWB + ks * 64 + (lane >> 4) * 16);
#pragma unroll
      for (int i = 0; i < FN; ++i)
#pragma unroll
        for (int j = 0; j < FM; ++j) acc[i][j] = mma16<T>(af[i], bf[j], acc[i][j]);
    }
  };

  // DEPTH register sets rotate through the stages: set j carries the stages congruent to
  // j; a set is refilled right after its previous stage went to LDS, so every load has
  // DEPTH-1 stage computations to land.  Stages past the end of K are masked to zero.
  const int nst = (a.K + BKE - 1) / BKE;
  V wS[DEPTH][CHW], xS[DEPTH][CHX];
  unsigned mS[DEPTH];
#pragma unroll
  for (int d = 0; d < DEPTH; ++d) mS[d] = load_global(d, wS[d], xS[d]);
  store_lds(0, wS[0], xS[0], mS[0]);
  __syncthreads();
#pragma nounroll
  for (int s = 0; s < nst; s += DEPTH) {
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) {          // LDS buffer d&1 holds stage s+d
      mS[d] = load_global(s + d + DEPTH, wS[d], xS[d]);
      compute(d & 1);
      store_lds((d + 1) & 1, wS[(d + 1) % DEPTH], xS[(d + 1) % DEPTH], mS[(d + 1) % DEPTH]);
      __syncthreads();
    }
  }

#pragma unroll
  for (int i = 0; i < FN; ++i) {
    const int n = n0 + wn0 + i * 16 + (lane >> 4) * 4;
#pragma unroll
    for (int j = 0; j < FM; ++j) {
      const int m = m0 + wm0 + j * 16 + (lane & 15);
      if (m >= a.M || n >= a.N) continue;
      float v[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float r = acc[i][j][e] * a.alpha;
        if (n + e < a.N) {
          if (a.bias) r += a.bias[n + e];
          for (int q = 0; q < a.n_extra; ++q) r += (float)ldg<CA, T>((const T *)a.extra[q] + (int64_t)m * a.N + n + e);
        }
        if (a.relu) r = fmaxf(r, 0.f);
        v[e] = r;
      }
      T *dst = y + (int64_t)m * a.ldy + n;
      if (n + 3 < a.N && ((uintptr_t)dst & (4 * sizeof(T) - 1)) == 0) {
        Q q4 = {(T)v[0], (T)v[1], (T)v[2], (T)v[3]};
        stg<CS, Q>(dst, q4);
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (n + e < a.N) stg<CS, T>(dst + e, (T)v[e]);
      }
    }
  }
}

// ---------------------------------------------------------------------------------
// Latency-oriented implicit GEMM for small problems (batch-1 convolutions, skinny
// GEMMs): a workgroup owns a 32 x 32 output tile and its WAVES wavefronts split K
// between them.  Every lane fetches its MFMA fragments straight from global memory
// (32 contiguous bytes per row and lane group, so four lane groups consume a whole
// 128-byte line), two 64-byte-deep K steps in flight at a time, no LDS and no
// barrier inside the K loop.  Partial tiles meet in LDS once, at the end, where 256
// threads apply the epilogue and write 8/16-byte pieces of output rows.
// ---------------------------------------------------------------------------------
template <typename T, int WAVES, int U, int COH, int NI, int NJ, typename AR>
__device__ __forceinline__ void igemm_direct_body(const AR &a, const Blk &b, unsigned char *lds) {
  typedef typename Vec16<T>::type V;
  typedef typename Vec16<T>::quad Q;
  constexpr int VE = Vec16<T>::N;
  constexpr int DS = 8 * VE;               // K elements per step: 4 lane groups x 2 chunks
  constexpr int PITCH = 36;                // floats per pixel row of a partial tile in LDS
  float (*part)[32][PITCH] = (float (*)[32][PITCH])lds;                                // [WAVES][32][PITCH]

  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int grp = lane >> 4, r16 = lane & 15;
  int tile_x, tile_y;
  xcd_tile(b, tile_x, tile_y);
  const int m0 = tile_x * (16 * NJ), n0 = tile_y * (16 * NI);
  constexpr bool CA = (COH & kCohAct) != 0, CW = (COH & kCohW) != 0, CS = (COH & (kCohAct | kCohStore)) != 0;
  const T *__restrict__ x = (const T *)a.x + (int64_t)b.z * a.a_bs;
  const T *__restrict__ w = (const T *)a.w + (int64_t)b.z * a.b_bs;
  T *__restrict__ y = (T *)a.y + (int64_t)b.z * a.y_bs;

  const int nds = (a.K + DS - 1) / DS;
  const int per_wave = (nds + WAVES - 1) / WAVES;
  const int ds_begin = wave * per_wave;
  const int ds_end = min(nds, ds_begin + per_wave);

  // Rows are clamped into range and every load is unconditional (a load behind a branch
  // is waited for inside the branch).  Results of clamped rows are never stored; K
  // tails are cancelled by zeroing the weight fragment, padding taps by zeroing the
  // pixel fragment.
  const T *wrow[NI], *xrow[NJ], *ximg[NJ];
  int ih0[NJ], iw0[NJ];
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const int n = min(n0 + i * 16 + r16, a.N - 1);
    wrow[i] = w + (int64_t)n * a.ldb;
  }
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int m = min(m0 + j * 16 + r16, a.M - 1);
    xrow[j] = x + (int64_t)m * a.lda;
    const int img = m / a.HoWo, pix = m - img * a.HoWo;   // only meaningful when gathering
    const int oh = pix / a.Wo, ow = pix - oh * a.Wo;
    ih0[j] = oh * a.sh - a.ph;
    iw0[j] = ow * a.sw - a.pw;
    ximg[j] = x + (int64_t)img * a.img_stride;
  }
  KPos pos = {0, 0, 0};
  if (a.gather && ds_begin < ds_end) {
    const int k = ds_begin * DS + grp * 2 * VE;
    pos.ci = k % a.Cin;
    const int rs = k / a.Cin;
    pos.s = rs % a.kw;
    pos.r = rs / a.kw;
  }

  floatx4 acc[NI][NJ];
#pragma unroll
  for (int i = 0; i < NI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};
  const V vzero = {};

  // Epilogue operands of this thread's output piece (bias, residual inputs) are requested
  // before the K walk, so that their latency is hidden behind it.
  constexpr int PG = 4 * NI;               // four-channel pieces per tile row
  const int pm = t / PG, pn = (t % PG) * 4;
  const int m = m0 + pm, n = n0 + pn;
  const bool full = n + 3 < a.N;           // whole group of four channels inside the tensor
  const bool live = t < 16 * NJ * PG && m < a.M && n < a.N;
  floatx4 badd = {0.f, 0.f, 0.f, 0.f};
  if (live && a.bias) {
    if (full && ((uintptr_t)(a.bias + n) & 15) == 0) badd = *(const floatx4 *)(a.bias + n);
    else
      for (int e = 0; e < 4; ++e) if (n + e < a.N) badd[e] = a.bias[n + e];
  }
  if (live)
    for (int q = 0; q < a.n_extra; ++q) {
      const T *ex = (const T *)a.extra[q] + (int64_t)m * a.N + n;
      if (full && ((uintptr_t)ex & (4 * sizeof(T) - 1)) == 0) {
        const Q v = ldg<CA, Q>(ex);
#pragma unroll
        for (int e = 0; e < 4; ++e) badd[e] += (float)v[e];
      } else {
        for (int e = 0; e < 4; ++e) if (n + e < a.N) badd[e] += (float)ldg<CA, T>(ex + e);
      }
    }

  // One round = UU K steps requested together, then multiplied.  Full rounds of U steps,
  // then a shorter last round: steps past the end of a wavefront's K range would only
  // move bytes that are never used, and at these sizes the bytes set the time.
  auto round = [&](auto uu_tag, int ds) {
    constexpr int UU = decltype(uu_tag)::value;
    V wa[UU][NI][2], xb[UU][NJ][2];
    bool kok[UU][2], inb[UU][NJ][2];
#pragma unroll
    for (int u = 0; u < UU; ++u) {
      KPos pc = pos;                       // position of chunk 0 of this step
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        const int k = (ds + u) * DS + grp * 2 * VE + c * VE;
        kok[u][c] = k < a.K;
        const int ks = kok[u][c] ? k : 0;
#pragma unroll
        for (int i = 0; i < NI; ++i) wa[u][i][c] = ldg<CW, V>(wrow[i] + ks);
        if (!a.gather) {
#pragma unroll
          for (int j = 0; j < NJ; ++j) xb[u][j][c] = ldg<CA, V>(xrow[j] + ks);
        } else {
#pragma unroll
          for (int j = 0; j < NJ; ++j) {
            const int ih = ih0[j] + pc.r, iw = iw0[j] + pc.s;
            inb[u][j][c] = kok[u][c] && (unsigned)ih < (unsigned)a.H && (unsigned)iw < (unsigned)a.W;
            const int64_t off = inb[u][j][c] ? ((int64_t)ih * a.W + iw) * a.Cin + pc.ci : 0;
            xb[u][j][c] = ldg<CA, V>(ximg[j] + off);
          }
          if (c == 0) kpos_advance(pc, VE, a.Cin, a.kw);
        }
      }
      if (a.gather) kpos_advance(pos, DS, a.Cin, a.kw);
    }
#pragma unroll
    for (int u = 0; u < UU; ++u)
#pragma unroll
      for (int c = 0; c < 2; ++c) {
#pragma unroll
        for (int i = 0; i < NI; ++i) wa[u][i][c] = kok[u][c] ? wa[u][i][c] : vzero;
        if (a.gather) {
#pragma unroll
          for (int j = 0; j < NJ; ++j) xb[u][j][c] = inb[u][j][c] ? xb[u][j][c] : vzero;
        }
#pragma unroll
        for (int i = 0; i < NI; ++i)
#pragma unroll
          for (int j = 0; j < NJ; ++j) acc[i][j] = mma16<T>(wa[u][i][c], xb[u][j][c], acc[i][j]);
      }
  };
  {
    int ds = ds_begin;
    for (; ds + U <= ds_end; ds += U) round(std::integral_constant<int, U>{}, ds);
    if constexpr (U > 2) {
      if (ds + 2 <= ds_end) { round(std::integral_constant<int, 2>{}, ds); ds += 2; }
    }
    if constexpr (U > 1) {
      if (ds < ds_end) round(std::integral_constant<int, 1>{}, ds);
    }
  }

  // ---- meet in LDS: lane holds channels n = i*16 + grp*4 + e of pixel m = j*16 + r16
#pragma unroll
  for (int i = 0; i < NI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j) *(floatx4 *)&part[wave][j * 16 + r16][i * 16 + grp * 4] = acc[i][j];
  __syncthreads();
  if (t < 16 * NJ * PG) {
    floatx4 sum = *(const floatx4 *)&part[0][pm][pn];
#pragma unroll
    for (int q = 1; q < WAVES; ++q) sum += *(const floatx4 *)&part[q][pm][pn];
    if (live) {
      float v[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float r = sum[e] * a.alpha + badd[e];
        v[e] = a.relu ? fmaxf(r, 0.f) : r;
      }
      T *dst = y + (int64_t)m * a.ldy + n;
      if (full && ((uintptr_t)dst & (4 * sizeof(T) - 1)) == 0) {
        Q q4 = {(T)v[0], (T)v[1], (T)v[2], (T)v[3]};
        stg<CS, Q>(dst, q4);
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (n + e < a.N) stg<CS, T>(dst + e, (T)v[e]);
      }
    }
  }
}

// ---------------------------------------------------------------------------------
// Quad transposition.  The texture path serves a 16-byte-per-lane load at full rate only
// when four adjacent lanes read 64 contiguous bytes; lanes that each touch a different
// line are served one lane at a time (measured on gfx950: 14 against 43 bytes per clock
// and compute unit).  An MFMA operand wants adjacent lanes on different rows.  So a lane
// group of four loads four rows, 64 contiguous bytes of one row per instruction, and this
// 4 x 4 exchange inside the group (two butterfly stages of cross-lane moves) hands every
// lane the four pieces of its own row: afterwards register t of lane i holds what
// register i of lane t held.  All cross-lane moves are unconditional; only the selects
// depend on the lane.
// ---------------------------------------------------------------------------------
template <int CTRL> __device__ __forceinline__ uint32_t quad_move(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, CTRL, 0xf, 0xf, true);
}
template <int T> __device__ __forceinline__ int quad_broadcast(int v) {
  return __builtin_amdgcn_mov_dpp(v, T * 0x55, 0xf, 0xf, true);
}
template <typename V> __device__ __forceinline__ void quad_transpose(V (&r)[4], bool odd, bool hi) {
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  static_assert(sizeof(V) == 16, "fragment size");
  u32x4 u[4];
#pragma unroll
  for (int t = 0; t < 4; ++t) u[t] = __builtin_bit_cast(u32x4, r[t]);
#pragma unroll
  for (int p = 0; p < 2; ++p)              // lane bit 0 <-> register bit 0
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      const uint32_t a0 = u[2 * p][d], b0 = u[2 * p + 1][d];
      const uint32_t pa = quad_move<0xB1>(a0), pb = quad_move<0xB1>(b0);   // lanes [1,0,3,2]
      u[2 * p][d] = odd ? pb : a0;
      u[2 * p + 1][d] = odd ? b0 : pa;
    }
#pragma unroll
  for (int p = 0; p < 2; ++p)              // lane bit 1 <-> register bit 1
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      const uint32_t a0 = u[p][d], b0 = u[p + 2][d];
      const uint32_t pa = quad_move<0x4E>(a0), pb = quad_move<0x4E>(b0);   // lanes [2,3,0,1]
      u[p][d] = hi ? pb : a0;
      u[p + 2][d] = hi ? b0 : pa;
    }
#pragma unroll
  for (int t = 0; t < 4; ++t) r[t] = __builtin_bit_cast(V, u[t]);
}

// ---------------------------------------------------------------------------------
// Latency-oriented implicit GEMM for small problems (batch-1 convolutions, skinny
// GEMMs): a workgroup owns a 32 x 32 output tile and its WAVES wavefronts split K
// between them in steps of 256 bytes per row.  Operands come straight from global
// memory, no LDS and no barrier inside the K loop: in one load instruction a group of
// four lanes reads 64 contiguous bytes of one row (see quad_transpose), the next step's
// loads are in flight while the current one is transposed and multiplied.  Partial tiles
// meet in LDS once, at the end, where 256 threads apply the epilogue and write 8/16-byte
// pieces of output rows.
// ---------------------------------------------------------------------------------
template <typename T, int WAVES, int COH, int NI, int NJ, typename AR>
__device__ __forceinline__ void igemm_quad_body(const AR &a, const Blk &b, unsigned char *lds) {
  typedef typename Vec16<T>::type V;
  typedef typename Vec16<T>::quad Q;
  constexpr int VE = Vec16<T>::N;
  constexpr int DS = 16 * VE;              // K elements per step: 4 lane groups x 4 pieces of 16 bytes
  constexpr int PITCH = 36;                // floats per pixel row of a partial tile in LDS
  float (*part)[32][PITCH] = (float (*)[32][PITCH])lds;                                // [WAVES][32][PITCH]

  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int grp = lane >> 4, r16 = lane & 15, qd = (lane >> 2) & 3, pc = lane & 3;
  const bool odd = (lane & 1) != 0, hi = (lane & 2) != 0;
  int tile_x, tile_y;
  xcd_tile(b, tile_x, tile_y);
  const int m0 = tile_x * (16 * NJ), n0 = tile_y * (16 * NI);
  constexpr bool CA = (COH & kCohAct) != 0, CW = (COH & kCohW) != 0, CS = (COH & (kCohAct | kCohStore)) != 0;
  const T *__restrict__ x = (const T *)a.x + (int64_t)b.z * a.a_bs;
  const T *__restrict__ w = (const T *)a.w + (int64_t)b.z * a.b_bs;
  T *__restrict__ y = (T *)a.y + (int64_t)b.z * a.y_bs;

  const int nds = (a.K + DS - 1) / DS;
  const int per_wave = (nds + WAVES - 1) / WAVES;
  const int ds_begin = wave * per_wave;
  const int ds_end = min(nds, ds_begin + per_wave);
  // Only the last step of K can be partial; it runs apart from the pipelined steps.
  const bool owns_tail = a.K % DS != 0 && ds_begin < nds && ds_end == nds;
  const int main_end = owns_tail ? ds_end - 1 : ds_end;
  const int kc = (grp * 4 + pc) * VE;      // this lane's 16-byte piece inside a step

  // Register t of block i loads row 16*i + 4*qd + t (clamped into range; results of
  // clamped rows are never stored).  Offsets are elements from the operand's base and fit
  // 32 bits (the host selects this kernel only for operands below 2^31 elements).
  int woff[NI][4], xoff[NJ][4], ihq[NJ][4], iwq[NJ][4];
#pragma unroll
  for (int i = 0; i < NI; ++i)
#pragma unroll
    for (int tt = 0; tt < 4; ++tt) woff[i][tt] = min(n0 + i * 16 + qd * 4 + tt, a.N - 1) * (int)a.ldb + kc;
#pragma unroll
  for (int j = 0; j < NJ; ++j)
#pragma unroll
    for (int tt = 0; tt < 4; ++tt) xoff[j][tt] = min(m0 + j * 16 + qd * 4 + tt, a.M - 1) * (int)a.lda + kc;
  KPos pos = {0, 0, 0};
  if (a.gather) {
    // Pixel geometry of this lane's own row, then of the group's four rows by broadcast.
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int m = min(m0 + j * 16 + r16, a.M - 1);
      const int img = m / a.HoWo, pix = m - img * a.HoWo;
      const int oh = pix / a.Wo, ow = pix - oh * a.Wo;
      const int ih0 = oh * a.sh - a.ph, iw0 = ow * a.sw - a.pw, im0 = img * (int)a.img_stride;
      ihq[j][0] = quad_broadcast<0>(ih0); ihq[j][1] = quad_broadcast<1>(ih0);
      ihq[j][2] = quad_broadcast<2>(ih0); ihq[j][3] = quad_broadcast<3>(ih0);
      iwq[j][0] = quad_broadcast<0>(iw0); iwq[j][1] = quad_broadcast<1>(iw0);
      iwq[j][2] = quad_broadcast<2>(iw0); iwq[j][3] = quad_broadcast<3>(iw0);
      xoff[j][0] = quad_broadcast<0>(im0); xoff[j][1] = quad_broadcast<1>(im0);
      xoff[j][2] = quad_broadcast<2>(im0); xoff[j][3] = quad_broadcast<3>(im0);
    }
    if (ds_begin < ds_end) {
      const int k = ds_begin * DS + kc;
      pos.ci = k % a.Cin;
      const int rs = k / a.Cin;
      pos.s = rs % a.kw;
      pos.r = rs / a.kw;
    }
  }

  floatx4 acc[NI][NJ];
#pragma unroll
  for (int i = 0; i < NI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};
  const V vzero = {};

  // Epilogue operands of this thread's output piece (bias, residual inputs) are requested
  // before the K walk, so that their latency is hidden behind it.
  constexpr int PG = 4 * NI;               // four-channel pieces per tile row
  const int pm = t / PG, pn = (t % PG) * 4;
  const int m = m0 + pm, n = n0 + pn;
  const bool full = n + 3 < a.N;           // whole group of four channels inside the tensor
  const bool live = t < 16 * NJ * PG && m < a.M && n < a.N;
  floatx4 badd = {0.f, 0.f, 0.f, 0.f};
  if (live && a.bias) {
    if (full && ((uintptr_t)(a.bias + n) & 15) == 0) badd = *(const floatx4 *)(a.bias + n);
    else
      for (int e = 0; e < 4; ++e) if (n + e < a.N) badd[e] = a.bias[n + e];
  }
  if (live)
    for (int q = 0; q < a.n_extra; ++q) {
      const T *ex = (const T *)a.extra[q] + (int64_t)m * a.N + n;
      if (full && ((uintptr_t)ex & (4 * sizeof(T) - 1)) == 0) {
        const Q v = ldg<CA, Q>(ex);
#pragma unroll
        for (int e = 0; e < 4; ++e) badd[e] += (float)v[e];
      } else {
        for (int e = 0; e < 4; ++e) if (n + e < a.N) badd[e] += (float)ldg<CA, T>(ex + e);
      }
    }

  struct Frag { V w[NI][4], x[NJ][4]; };
  // Requests one step.  In the partial step a lane whose piece lies past the end of K
  // requests nothing and contributes zeros; padding taps of a convolution read a valid
  // address and are zeroed after arrival.
  auto issue = [&](auto tail_tag, int ds, Frag &f) {
    constexpr bool TAIL = decltype(tail_tag)::value;
    const int kb = ds * DS;
    const bool kok = !TAIL || kb + kc < a.K;
    unsigned inb = 0xffu;
    int xo[NJ][4];
    if (a.gather) {
      inb = 0;
#pragma unroll
      for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) {
          const int ih = ihq[j][tt] + pos.r, iw = iwq[j][tt] + pos.s;
          const bool in = kok && (unsigned)ih < (unsigned)a.H && (unsigned)iw < (unsigned)a.W;
          inb |= in ? 1u << (j * 4 + tt) : 0u;
          xo[j][tt] = in ? xoff[j][tt] + (ih * a.W + iw) * a.Cin + pos.ci : 0;
        }
      kpos_advance(pos, DS, a.Cin, a.kw);
    } else {
#pragma unroll
      for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) xo[j][tt] = xoff[j][tt] + kb;
    }
    if (kok) {
#pragma unroll
      for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) f.w[i][tt] = ldg<CW, V>(w + woff[i][tt] + kb);
#pragma unroll
      for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) f.x[j][tt] = ldg<CA, V>(x + xo[j][tt]);
    } else {
#pragma unroll
      for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) f.w[i][tt] = vzero;
#pragma unroll
      for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) f.x[j][tt] = vzero;
    }
    return inb;
  };
  auto compute = [&](Frag &f, unsigned inb) {
    if (a.gather) {
#pragma unroll
      for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) f.x[j][tt] = ((inb >> (j * 4 + tt)) & 1u) ? f.x[j][tt] : vzero;
    }
#pragma unroll
    for (int i = 0; i < NI; ++i) quad_transpose(f.w[i], odd, hi);
#pragma unroll
    for (int j = 0; j < NJ; ++j) quad_transpose(f.x[j], odd, hi);
#pragma unroll
    for (int tt = 0; tt < 4; ++tt)
#pragma unroll
      for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j) acc[i][j] = mma16<T>(f.w[i][tt], f.x[j][tt], acc[i][j]);
  };
  if (ds_begin < main_end) {
    // Two register sets: the loads of step ds+1 are requested before step ds is
    // transposed and multiplied.  Inside the loop the request is unconditional (after a
    // conditional one the compiler waits for everything in flight), and the empty
    // statement pins the order: nothing else keeps a plain load from sinking to its use.
    Frag cur, nxt;
    unsigned inb_cur = issue(std::false_type{}, ds_begin, cur), inb_nxt;
#pragma nounroll
    for (int ds = ds_begin + 1; ds < main_end; ++ds) {
      inb_nxt = issue(std::false_type{}, ds, nxt);
      asm volatile("" ::: "memory");
      compute(cur, inb_cur);
      cur = nxt;
      inb_cur = inb_nxt;
    }
    compute(cur, inb_cur);
  }
  if (owns_tail) {
    Frag f;
    const unsigned inb = issue(std::true_type{}, main_end, f);
    compute(f, inb);
  }

  // ---- meet in LDS: lane holds channels n = i*16 + grp*4 + e of pixel m = j*16 + r16
#pragma unroll
  for (int i = 0; i < NI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j) *(floatx4 *)&part[wave][j * 16 + r16][i * 16 + grp * 4] = acc[i][j];
  __syncthreads();
  if (t < 16 * NJ * PG) {
    floatx4 sum = *(const floatx4 *)&part[0][pm][pn];
#pragma unroll
    for (int q = 1; q < WAVES; ++q) sum += *(const floatx4 *)&part[q][pm][pn];
    if (live) {
      float v[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float r = sum[e] * a.alpha + badd[e];
        v[e] = a.relu ? fmaxf(r, 0.f) : r;
      }
      T *dst = y + (int64_t)m * a.ldy + n;
      if (full && ((uintptr_t)dst & (4 * sizeof(T) - 1)) == 0) {
        Q q4 = {(T)v[0], (T)v[1], (T)v[2], (T)v[3]};
        stg<CS, Q>(dst, q4);
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (n + e < a.N) stg<CS, T>(dst + e, (T)v[e]);
      }
    }
  }
}

// ---------------------------------------------------------------------------------
// 64 x 64-tile form of the quad-coalesced contraction, for GEMM-shaped operands (no
// im2col gather) with enough rows to fill such tiles: every wavefront of the workgroup
// multiplies the whole tile over its share of K, so each 16-byte piece a lane loads feeds
// four MFMAs instead of two and the loads and exchanges per multiply-add halve.  The
// fragments of one step take 128 registers, the accumulators 64: one register set, no
// prefetch across steps (two four-wavefront workgroups per CU overlap instead; one
// eight-wavefront workgroup per CU was slower on every shape measured), row offsets
// recomputed per load.  Partial tiles meet in LDS; each thread finishes four 4-channel pieces.
// ---------------------------------------------------------------------------------
template <typename T, int WAVES, int COH, typename AR>
__device__ __forceinline__ void igemm_quad64_body(const AR &a, const Blk &b, unsigned char *lds) {
  typedef typename Vec16<T>::type V;
  typedef typename Vec16<T>::quad Q;
  constexpr int VE = Vec16<T>::N;
  constexpr int DS = 16 * VE;              // K elements per step
  constexpr int PITCH = 68;                // floats per row of a partial tile in LDS
  float (*part)[64][PITCH] = (float (*)[64][PITCH])lds;                                // [WAVES][64][PITCH]

  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int grp = lane >> 4, r16 = lane & 15, qd = (lane >> 2) & 3, pc = lane & 3;
  const bool odd = (lane & 1) != 0, hi = (lane & 2) != 0;
  int tile_x, tile_y;
  xcd_tile(b, tile_x, tile_y);
  const int m0 = tile_x * 64, n0 = tile_y * 64;
  constexpr bool CA = (COH & kCohAct) != 0, CW = (COH & kCohW) != 0, CS = (COH & (kCohAct | kCohStore)) != 0;
  const T *__restrict__ x = (const T *)a.x + (int64_t)b.z * a.a_bs;
  const T *__restrict__ w = (const T *)a.w + (int64_t)b.z * a.b_bs;
  T *__restrict__ y = (T *)a.y + (int64_t)b.z * a.y_bs;

  const int nds = (a.K + DS - 1) / DS;
  const int per_wave = (nds + WAVES - 1) / WAVES;
  const int ds_begin = wave * per_wave;
  const int ds_end = min(nds, ds_begin + per_wave);
  const bool owns_tail = a.K % DS != 0 && ds_begin < nds && ds_end == nds;
  const int main_end = owns_tail ? ds_end - 1 : ds_end;
  const int kc = (grp * 4 + pc) * VE;      // this lane's 16-byte piece inside a step
  const int lda = (int)a.lda, ldb = (int)a.ldb;
  const int nq = n0 + qd * 4, mq = m0 + qd * 4;

  floatx4 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};
  const V vzero = {};

  struct Frag { V w[4][4], x[4][4]; };
  // Register tt of block i holds row 16*i + 4*qd + tt (clamped into range; results of
  // clamped rows are never stored), offsets in elements (below 2^31 by the host's choice).
  auto step = [&](auto tail_tag, int ds) {
    constexpr bool TAIL = decltype(tail_tag)::value;
    const int kb = ds * DS + kc;
    const bool kok = !TAIL || kb < a.K;
    Frag f;
    if (kok) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) f.w[i][tt] = ldg<CW, V>(w + (min(nq + i * 16 + tt, a.N - 1) * ldb + kb));
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) f.x[j][tt] = ldg<CA, V>(x + (min(mq + j * 16 + tt, a.M - 1) * lda + kb));
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) { f.w[i][tt] = vzero; f.x[i][tt] = vzero; }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      quad_transpose(f.w[i], odd, hi);
      quad_transpose(f.x[i], odd, hi);
    }
#pragma unroll
    for (int tt = 0; tt < 4; ++tt)
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = mma16<T>(f.w[i][tt], f.x[j][tt], acc[i][j]);
  };
#pragma nounroll
  for (int ds = ds_begin; ds < main_end; ++ds) step(std::false_type{}, ds);
  if (owns_tail) step(std::true_type{}, main_end);

  // ---- meet in LDS: lane holds channels n = i*16 + grp*4 + e of row m = j*16 + r16
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) *(floatx4 *)&part[wave][j * 16 + r16][i * 16 + grp * 4] = acc[i][j];
  __syncthreads();
  if (t < 256) {
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      const int idx = t + p * 256;
      const int pm = idx >> 4, pn = (idx & 15) * 4;
      const int m = m0 + pm, n = n0 + pn;
      if (m >= a.M || n >= a.N) continue;
      const bool full = n + 3 < a.N;
      floatx4 sum = *(const floatx4 *)&part[0][pm][pn];
#pragma unroll
      for (int q = 1; q < WAVES; ++q) sum += *(const floatx4 *)&part[q][pm][pn];
      float v[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float r = sum[e] * a.alpha;
        if (n + e < a.N) {
          if (a.bias) r += a.bias[n + e];
          for (int q = 0; q < a.n_extra; ++q) r += (float)ldg<CA, T>((const T *)a.extra[q] + (int64_t)m * a.N + n + e);
        }
        v[e] = a.relu ? fmaxf(r, 0.f) : r;
      }
      T *dst = y + (int64_t)m * a.ldy + n;
      if (full && ((uintptr_t)dst & (4 * sizeof(T) - 1)) == 0) {
        Q q4 = {(T)v[0], (T)v[1], (T)v[2], (T)v[3]};
        stg<CS, Q>(dst, q4);
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (n + e < a.N) stg<CS, T>(dst + e, (T)v[e]);
      }
    }
  }
}

// Matrix-vector shaped GEMM (M <= kGemvMaxM rows): one wavefront per output column,
// 16-byte loads along K, shuffle reduction.  Weight-bandwidth bound by construction.
template <typename T, int COH, typename AR>
__device__ __forceinline__ void gemv_body(const AR &a, const Blk &b, unsigned char *lds) {
  typedef typename Vec16<T>::type V;
  constexpr int VE = Vec16<T>::N;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = b.x * 4 + wave;
  if (n >= a.N) return;
  constexpr bool CA = (COH & kCohAct) != 0, CW = (COH & kCohW) != 0, CS = (COH & (kCohAct | kCohStore)) != 0;
  const T *__restrict__ x = (const T *)a.x;
  const T *__restrict__ wr = (const T *)a.w + (int64_t)n * a.ldb;
  float acc[kGemvMaxM] = {0.f, 0.f, 0.f, 0.f};
  for (int k0 = lane * VE; k0 < a.K; k0 += 64 * VE) {
    const V wv = ldg<CW, V>(wr + k0);
#pragma unroll
    for (int m = 0; m < kGemvMaxM; ++m) {
      if (m < a.M) {
        const V xv = ldg<CA, V>(x + (int64_t)m * a.lda + k0);
#pragma unroll
        for (int e = 0; e < VE; ++e) acc[m] += (float)wv[e] * (float)xv[e];
      }
    }
  }
#pragma unroll
  for (int m = 0; m < kGemvMaxM; ++m)
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc[m] += __shfl_xor(acc[m], off, 64);
  if (lane == 0) {
    T *y = (T *)a.y;
    for (int m = 0; m < a.M; ++m) {
      float r = acc[m] * a.alpha;
      if (a.bias) r += a.bias[n];
      for (int q = 0; q < a.n_extra; ++q) r += (float)ldg<CA, T>((const T *)a.extra[q] + (int64_t)m * a.N + n);
      if (a.relu) r = fmaxf(r, 0.f);
      stg<CS, T>(y + (int64_t)m * a.ldy + n, (T)r);
    }
  }
}

// ---------------------------------------------------------------------------------
// Pooling over [H][W][C]: one thread per output pixel and channel chunk.
// ---------------------------------------------------------------------------------
template <typename T, int VE, int COH, typename AR>
__device__ __forceinline__ void pool_body(const AR &a, const Blk &b, unsigned char *lds) {
  constexpr bool CA = (COH & kCohAct) != 0, CS = (COH & (kCohAct | kCohStore)) != 0;
  const int cch = a.C / VE;
  const int64_t item = (int64_t)b.x * 256 + threadIdx.x;
  if (item >= (int64_t)a.B * a.Ho * a.Wo * cch) return;
  const int cc = (int)(item % cch);
  const int pix = (int)(item / cch);                   // output pixel over all images
  const int img = pix / (a.Ho * a.Wo), ipix = pix - img * (a.Ho * a.Wo);
  const int ow = ipix % a.Wo, oh = ipix / a.Wo;
  const T *__restrict__ x = (const T *)a.x + (int64_t)img * a.H * a.W * a.C + cc * VE;
  const float fill = a.is_avg ? 0.f : -INFINITY;
  float acc[VE];
#pragma unroll
  for (int e = 0; e < VE; ++e) acc[e] = fill;
  auto fetch = [&](int ih, int iw, T *v) {
    const bool ok = (unsigned)ih < (unsigned)a.H && (unsigned)iw < (unsigned)a.W;
    const T *src = x + ((int64_t)(ok ? ih : 0) * a.W + (ok ? iw : 0)) * a.C;
    if constexpr (VE > 1) *(typename Vec16<T>::type *)v = ldg<CA, typename Vec16<T>::type>(src);
    else v[0] = ldg<CA, T>(src);
    return ok;
  };
  auto fold = [&](bool ok, const T *v) {
#pragma unroll
    for (int e = 0; e < VE; ++e) {
      const float f = ok ? (float)v[e] : fill;
      acc[e] = a.is_avg ? acc[e] + f : fmaxf(acc[e], f);
    }
  };
  const int ih0 = oh * a.sh - a.ph, iw0 = ow * a.sw - a.pw;
  if (a.kh == 3 && a.kw == 3) {
    // all nine taps in flight before the first use
    T v[9][VE];
    bool ok[9];
#pragma unroll
    for (int i = 0; i < 3; ++i)
#pragma unroll
      for (int j = 0; j < 3; ++j) ok[i * 3 + j] = fetch(ih0 + i, iw0 + j, v[i * 3 + j]);
#pragma unroll
    for (int q = 0; q < 9; ++q) fold(ok[q], v[q]);
  } else {
    for (int i = 0; i < a.kh; ++i)
      for (int j = 0; j < a.kw; ++j) {
        T v[VE];
        const bool ok = fetch(ih0 + i, iw0 + j, v);
        fold(ok, v);
      }
  }
  const float scale = a.is_avg ? 1.0f / (float)(a.kh * a.kw) : 1.0f;
  T o[VE];
#pragma unroll
  for (int e = 0; e < VE; ++e) o[e] = (T)(a.is_avg ? acc[e] * scale : acc[e]);
  T *dst = (T *)a.y + (int64_t)pix * a.C + cc * VE;
  if constexpr (VE > 1) stg<CS, typename Vec16<T>::type>(dst, *(const typename Vec16<T>::type *)o);
  else stg<CS, T>(dst, o[0]);
}

// Global average pool over [HW][C]: 256 threads = 64 channels x 4 pixel slices; each
// thread sums its slice with independent loads, slices meet in LDS.
template <typename T, int COH, typename AR>
__device__ __forceinline__ void gap_body(const AR &a, const Blk &b, unsigned char *lds) {
  float (*part)[64] = (float (*)[64])lds;                                              // [4][64]
  const int cl = threadIdx.x & 63, slice = threadIdx.x >> 6;
  const int c = b.x * 64 + cl;
  constexpr bool CA = (COH & kCohAct) != 0, CS = (COH & (kCohAct | kCohStore)) != 0;
  const T *__restrict__ x = (const T *)a.x + (int64_t)b.y * a.HW * a.C;
  float s = 0.f;
  if (c < a.C) {
    int p = slice;
    for (; p + 12 < a.HW; p += 16) {
      const float v0 = (float)ldg<CA, T>(x + (int64_t)p * a.C + c), v1 = (float)ldg<CA, T>(x + (int64_t)(p + 4) * a.C + c);
      const float v2 = (float)ldg<CA, T>(x + (int64_t)(p + 8) * a.C + c), v3 = (float)ldg<CA, T>(x + (int64_t)(p + 12) * a.C + c);
      s += (v0 + v1) + (v2 + v3);
    }
    for (; p < a.HW; p += 4) s += (float)ldg<CA, T>(x + (int64_t)p * a.C + c);
  }
  part[slice][cl] = s;
  __syncthreads();
  if (slice == 0 && c < a.C)
    stg<CS, T>((T *)a.y + (int64_t)b.y * a.C + c, (T)((part[0][cl] + part[1][cl] + part[2][cl] + part[3][cl]) / (float)a.HW));
}

// ---------------------------------------------------------------------------------
// Row-wise LayerNorm / softmax of the summed inputs.  G lanes share a row (a
// wavefront, or the 256-thread workgroup); the row lives in registers between the
// statistics passes, so HBM sees one read per input and one write.
// ---------------------------------------------------------------------------------
template <int G, bool IS_MAX>
__device__ __forceinline__ float group_reduce(float v, float *scratch) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const float o = __shfl_xor(v, off, 64);
    v = IS_MAX ? fmaxf(v, o) : v + o;
  }
  if (G > 64) {
    const int wave = threadIdx.x >> 6;
    __syncthreads();                    // scratch may still be read from a previous reduction
    if ((threadIdx.x & 63) == 0) scratch[wave] = v;
    __syncthreads();
    v = scratch[0];
#pragma unroll
    for (int i = 1; i < G / 64; ++i) v = IS_MAX ? fmaxf(v, scratch[i]) : v + scratch[i];
  }
  return v;
}

template <typename T, bool IS_LN, int G, int MAXCH, int COH, typename AR>
__device__ __forceinline__ void row_cached_body(const AR &a, const Blk &b, unsigned char *lds) {
  typedef typename Vec16<T>::type V;
  constexpr int VE = Vec16<T>::N;
  float *scratch = (float *)lds;                                                       // [4]
  constexpr bool CA = (COH & kCohAct) != 0, CS = (COH & (kCohAct | kCohStore)) != 0;
  const int gl = threadIdx.x % G;
  const int row = b.x * (256 / G) + threadIdx.x / G;
  if (G == 64 && row >= a.rows) return;          // whole wavefront leaves together
  float v[MAXCH][VE];
  const int64_t base = (int64_t)row * a.cols;
#pragma unroll
  for (int c = 0; c < MAXCH; ++c) {
    const int col = (c * G + gl) * VE;
#pragma unroll
    for (int e = 0; e < VE; ++e) v[c][e] = 0.f;
    if (col < a.cols) {
      for (int q = 0; q < a.n_in; ++q) {
        const V t = ldg<CA, V>((const T *)a.in[q] + base + col);
#pragma unroll
        for (int e = 0; e < VE; ++e) v[c][e] += (float)t[e];
      }
    }
  }
  if (IS_LN) {
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < MAXCH; ++c)
      if ((c * G + gl) * VE < a.cols)
#pragma unroll
        for (int e = 0; e < VE; ++e) s += v[c][e];
    const float mean = group_reduce<G, false>(s, scratch) / (float)a.cols;
    float q = 0.f;
#pragma unroll
    for (int c = 0; c < MAXCH; ++c)
      if ((c * G + gl) * VE < a.cols)
#pragma unroll
        for (int e = 0; e < VE; ++e) { const float d = v[c][e] - mean; q += d * d; }
    const float var = group_reduce<G, false>(q, scratch) / (float)a.cols;
    const float rstd = 1.0f / sqrtf(var + a.eps);
#pragma unroll
    for (int c = 0; c < MAXCH; ++c)
#pragma unroll
      for (int e = 0; e < VE; ++e) v[c][e] = (v[c][e] - mean) * rstd;
  } else {
    float mx = -INFINITY;
#pragma unroll
    for (int c = 0; c < MAXCH; ++c)
      if ((c * G + gl) * VE < a.cols)
#pragma unroll
        for (int e = 0; e < VE; ++e) mx = fmaxf(mx, v[c][e]);
    mx = group_reduce<G, true>(mx, scratch);
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < MAXCH; ++c)
      if ((c * G + gl) * VE < a.cols)
#pragma unroll
        for (int e = 0; e < VE; ++e) { v[c][e] = expf(v[c][e] - mx); s += v[c][e]; }
    const float inv = 1.0f / group_reduce<G, false>(s, scratch);
#pragma unroll
    for (int c = 0; c < MAXCH; ++c)
#pragma unroll
      for (int e = 0; e < VE; ++e) v[c][e] *= inv;
  }
#pragma unroll
  for (int c = 0; c < MAXCH; ++c) {
    const int col = (c * G + gl) * VE;
    if (col < a.cols) {
      V o;
#pragma unroll
      for (int e = 0; e < VE; ++e) o[e] = (T)v[c][e];
      stg<CS, V>((T *)a.y + base + col, o);
    }
  }
}

// Any width / alignment: one workgroup per row, scalar accesses, inputs re-read per pass.
template <typename T, bool IS_LN, int COH, typename AR>
__device__ __forceinline__ void row_generic_body(const AR &a, const Blk &b, unsigned char *lds) {
  float *scratch = (float *)lds;                                                       // [4]
  constexpr bool CA = (COH & kCohAct) != 0, CS = (COH & (kCohAct | kCohStore)) != 0;
  const int64_t base = (int64_t)b.x * a.cols;
  auto value = [&](int col) {
    float s = 0.f;
    for (int q = 0; q < a.n_in; ++q) s += (float)ldg<CA, T>((const T *)a.in[q] + base + col);
    return s;
  };
  float p1 = IS_LN ? 0.f : -INFINITY;
  for (int col = threadIdx.x; col < a.cols; col += 256) p1 = IS_LN ? p1 + value(col) : fmaxf(p1, value(col));
  const float r1 = IS_LN ? group_reduce<256, false>(p1, scratch) / (float)a.cols : group_reduce<256, true>(p1, scratch);
  float p2 = 0.f;
  for (int col = threadIdx.x; col < a.cols; col += 256) {
    const float d = value(col) - r1;
    p2 += IS_LN ? d * d : expf(d);
  }
  const float r2 = group_reduce<256, false>(p2, scratch);
  const float k = IS_LN ? 1.0f / sqrtf(r2 / (float)a.cols + a.eps) : 1.0f / r2;
  for (int col = threadIdx.x; col < a.cols; col += 256) {
    const float d = value(col) - r1;
    stg<CS, T>((T *)a.y + base + col, (T)(IS_LN ? d * k : expf(d) * k));
  }
}

// ---------------------------------------------------------------------------------
// Element-wise f(sum of inputs) and channel/column concatenation.
// ---------------------------------------------------------------------------------
// erf by the rational-times-exponential formula of Abramowitz & Stegun 7.1.26 (absolute error
// below 1.5e-7): one reciprocal, one exponential and five multiply-adds, against several
// dozen instructions of the correctly rounded library routine, which made GELU ALU-bound
// (128 MB: 60 us against 38 us for ReLU).  Used where the result is stored as fp16, whose
// spacing (2^-11 relative) is three orders of magnitude coarser than that error.
__device__ __forceinline__ float erf_as(float x) {
  const float ax = fabsf(x);
  const float t = __builtin_amdgcn_rcpf(1.0f + 0.3275911f * ax);
  const float poly = t * (0.254829592f + t * (-0.284496736f + t * (1.421413741f + t * (-1.453152027f + t * 1.061405429f))));
  const float r = 1.0f - poly * __expf(-ax * ax);
  return x < 0.f ? -r : r;
}

template <typename T> __device__ __forceinline__ float elt_apply(int op, float x) {
  if (op == 1) return fmaxf(x, 0.f);
  if (op == 2) {
    const float z = x * 0.70710678118654752f;
    return 0.5f * x * (1.0f + (std::is_same<T, half_t>::value ? erf_as(z) : erff(z)));
  }
  return x;
}

template <typename T, int VE, int COH, typename AR>
__device__ __forceinline__ void elt_body(const AR &a, const Blk &b, unsigned char *lds) {
  constexpr bool CA = (COH & kCohAct) != 0, CS = (COH & (kCohAct | kCohStore)) != 0;
  const int64_t i = ((int64_t)b.x * 256 + threadIdx.x) * VE;
  if (i >= a.n) return;
  float s[VE];
#pragma unroll
  for (int e = 0; e < VE; ++e) s[e] = 0.f;
  for (int q = 0; q < a.n_in; ++q) {
    T v[VE];
    const T *src = (const T *)a.in[q] + i;
    if constexpr (VE > 1) *(typename Vec16<T>::type *)v = ldg<CA, typename Vec16<T>::type>(src);
    else v[0] = ldg<CA, T>(src);
#pragma unroll
    for (int e = 0; e < VE; ++e) s[e] += (float)v[e];
  }
  T o[VE];
#pragma unroll
  for (int e = 0; e < VE; ++e) o[e] = (T)elt_apply<T>(a.op, s[e]);
  T *dst = (T *)a.y + i;
  if constexpr (VE > 1) stg<CS, typename Vec16<T>::type>(dst, *(const typename Vec16<T>::type *)o);
  else stg<CS, T>(dst, o[0]);
}

template <typename T, int VE, int COH, typename AR>
__device__ __forceinline__ void concat_body(const AR &a, const Blk &b, unsigned char *lds) {
  constexpr bool CA = (COH & kCohAct) != 0, CS = (COH & (kCohAct | kCohStore)) != 0;
  const int q = b.y;
  const int cch = a.cols[q] / VE;
  const int64_t item = (int64_t)b.x * 256 + threadIdx.x;
  if (item >= (int64_t)a.rows * cch) return;
  const int64_t r = item / cch;
  const int c = (int)(item % cch) * VE;
  const T *src = (const T *)a.in[q] + r * a.cols[q] + c;
  T *dst = (T *)a.y + r * a.out_cols + a.col_off[q] + c;
  if constexpr (VE > 1) stg<CS, typename Vec16<T>::type>(dst, ldg<CA, typename Vec16<T>::type>(src));
  else stg<CS, T>(dst, ldg<CA, T>(src));
}

}  // namespace opara

using namespace opara;

// Workgroup-shared memory each body needs (bytes).
constexpr int lds_igemm(int bn, int bm) { return 2 * (bn + bm) * 80; }
constexpr int lds_pipe(int bn, int bm) { return 2 * (bn + bm) * 144; }
constexpr int lds_direct(int waves) { return waves * 32 * 36 * 4; }
constexpr int lds_quad64(int waves) { return waves * 64 * 68 * 4; }
constexpr int kLdsGap = 4 * 64 * 4, kLdsRow = 16, kLdsNone = 0;

// Operator timeline (tracing aid, off by default): while a buffer is set, thread 0 of every
// workgroup folds the 100 MHz device clock at its start and end into the operator's slot
// (two 64-bit words: earliest start, latest end).  It shows what a profiler cannot show
// without disturbing it: which operators of a replay really ran at the same time.
// The buffer travels as a kernel argument (null when off) and is only looked at when the
// workgroup is done: the start time is read unconditionally (one scalar clock read) and
// both stamps are folded in at the end.  Read from a device variable, or tested at the
// start, the pointer put a dependent memory round trip in front of every workgroup's
// argument loads (GoogLeNet-like sequential graph 295 -> 327 / 309 us with tracing off).
__device__ __forceinline__ unsigned long long op_trace_begin() { return (unsigned long long)wall_clock64(); }
// Only the operator's first workgroup reports a start and only its last eight (in dispatch
// order) an end: with every workgroup of a 2,000-workgroup operator updating the same two
// words the atomics serialised and doubled the time of a replay.
__device__ __forceinline__ void op_trace_end(unsigned long long *tr, int tag, unsigned long long t0, unsigned lin,
                                             unsigned total) {
  if (tr && threadIdx.x == 0) {
    if (lin == 0) atomicMin(tr + 2 * (size_t)tag, t0);
    if (lin + 8 >= total) atomicMax(tr + 2 * (size_t)tag + 1, (unsigned long long)wall_clock64());
  }
}
__device__ __forceinline__ unsigned launch_lin() { return blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z); }
__device__ __forceinline__ unsigned launch_total() { return gridDim.x * gridDim.y * gridDim.z; }

#define KDEF(name, threads, ldsb, Args, call)                                                    \
  extern "C" __global__ void __launch_bounds__(threads) opara_k_##name(Args a, int32_t tag, unsigned long long *trace) {    \
    __shared__ __attribute__((aligned(16))) unsigned char lds[(ldsb) > 0 ? (ldsb) : 16];         \
    const Blk b = launch_blk();                                                                  \
    const unsigned long long t0 = op_trace_begin();                                              \
    call;                                                                                        \
    op_trace_end(trace, tag, t0, launch_lin(), launch_total());                                  \
  }
// second launch bound: wavefronts per SIMD the register allocation must leave room for
#define KDEF2(name, threads, waves_per_simd, ldsb, Args, call)                                                \
  extern "C" __global__ void __launch_bounds__(threads, waves_per_simd) opara_k_##name(Args a, int32_t tag, unsigned long long *trace) { \
    __shared__ __attribute__((aligned(16))) unsigned char lds[(ldsb) > 0 ? (ldsb) : 16];                      \
    const Blk b = launch_blk();                                                                               \
    const unsigned long long t0 = op_trace_begin();                                                           \
    call;                                                                                                     \
    op_trace_end(trace, tag, t0, launch_lin(), launch_total());                                               \
  }

KDEF2(igemm_f16_t128x64, 256, 2, lds_pipe(128, 64), IgemmArgs, (igemm_pipe_body<half_t, 128, 64, 2, 2, 4, 0>(a, b, lds)))
KDEF(igemm_f16_t64x64, 256, lds_igemm(64, 64), IgemmArgs, (igemm_body<half_t, 64, 64, 2, 2, true, 0>(a, b, lds)))
KDEF(igemm_f16_direct4, 256, lds_direct(4), IgemmArgs, (igemm_direct_body<half_t, 4, 2, 0, 2, 2>(a, b, lds)))
KDEF(igemm_f16_direct8, 512, lds_direct(8), IgemmArgs, (igemm_direct_body<half_t, 8, 2, 0, 2, 2>(a, b, lds)))
KDEF(igemm_f16_quad4, 256, lds_direct(4), IgemmArgs, (igemm_quad_body<half_t, 4, 0, 2, 2>(a, b, lds)))
KDEF(igemm_f16_quad8, 512, lds_direct(8), IgemmArgs, (igemm_quad_body<half_t, 8, 0, 2, 2>(a, b, lds)))
KDEF2(igemm_f16_quad64x4, 256, 2, lds_quad64(4), IgemmArgs, (igemm_quad64_body<half_t, 4, 0>(a, b, lds)))
KDEF(igemm_f16_t64x64_scalar, 256, lds_igemm(64, 64), IgemmArgs, (igemm_body<half_t, 64, 64, 2, 2, false, 0>(a, b, lds)))
KDEF2(igemm_f32_t128x64, 256, 2, lds_pipe(128, 64), IgemmArgs, (igemm_pipe_body<float, 128, 64, 2, 2, 4, 0>(a, b, lds)))
KDEF(igemm_f32_t64x64, 256, lds_igemm(64, 64), IgemmArgs, (igemm_body<float, 64, 64, 2, 2, true, 0>(a, b, lds)))
KDEF(igemm_f32_direct4, 256, lds_direct(4), IgemmArgs, (igemm_direct_body<float, 4, 2, 0, 2, 2>(a, b, lds)))
KDEF(igemm_f32_direct8, 512, lds_direct(8), IgemmArgs, (igemm_direct_body<float, 8, 2, 0, 2, 2>(a, b, lds)))
KDEF(igemm_f32_quad4, 256, lds_direct(4), IgemmArgs, (igemm_quad_body<float, 4, 0, 2, 2>(a, b, lds)))
KDEF(igemm_f32_quad8, 512, lds_direct(8), IgemmArgs, (igemm_quad_body<float, 8, 0, 2, 2>(a, b, lds)))
KDEF2(igemm_f32_quad64x4, 256, 2, lds_quad64(4), IgemmArgs, (igemm_quad64_body<float, 4, 0>(a, b, lds)))
KDEF(igemm_f32_t64x64_scalar, 256, lds_igemm(64, 64), IgemmArgs, (igemm_body<float, 64, 64, 2, 2, false, 0>(a, b, lds)))
KDEF(gemv_f16, 256, kLdsNone, IgemmArgs, (gemv_body<half_t, 0>(a, b, lds)))
KDEF(gemv_f32, 256, kLdsNone, IgemmArgs, (gemv_body<float, 0>(a, b, lds)))
KDEF(pool_f16_vec, 256, kLdsNone, PoolArgs, (pool_body<half_t, 8, 0>(a, b, lds)))
KDEF(pool_f16_scalar, 256, kLdsNone, PoolArgs, (pool_body<half_t, 1, 0>(a, b, lds)))
KDEF(pool_f32_vec, 256, kLdsNone, PoolArgs, (pool_body<float, 4, 0>(a, b, lds)))
KDEF(pool_f32_scalar, 256, kLdsNone, PoolArgs, (pool_body<float, 1, 0>(a, b, lds)))
KDEF(gap_f16, 256, kLdsGap, GapArgs, (gap_body<half_t, 0>(a, b, lds)))
KDEF(gap_f32, 256, kLdsGap, GapArgs, (gap_body<float, 0>(a, b, lds)))
KDEF(layernorm_f16_wave, 256, kLdsRow, RowArgs, (row_cached_body<half_t, true, 64, 2, 0>(a, b, lds)))
KDEF(layernorm_f16_block, 256, kLdsRow, RowArgs, (row_cached_body<half_t, true, 256, kRowCacheChunks, 0>(a, b, lds)))
KDEF(layernorm_f16_generic, 256, kLdsRow, RowArgs, (row_generic_body<half_t, true, 0>(a, b, lds)))
KDEF(layernorm_f32_wave, 256, kLdsRow, RowArgs, (row_cached_body<float, true, 64, 2, 0>(a, b, lds)))
KDEF(layernorm_f32_block, 256, kLdsRow, RowArgs, (row_cached_body<float, true, 256, kRowCacheChunks, 0>(a, b, lds)))
KDEF(layernorm_f32_generic, 256, kLdsRow, RowArgs, (row_generic_body<float, true, 0>(a, b, lds)))
KDEF(softmax_f16_wave, 256, kLdsRow, RowArgs, (row_cached_body<half_t, false, 64, 2, 0>(a, b, lds)))
KDEF(softmax_f16_block, 256, kLdsRow, RowArgs, (row_cached_body<half_t, false, 256, kRowCacheChunks, 0>(a, b, lds)))
KDEF(softmax_f16_generic, 256, kLdsRow, RowArgs, (row_generic_body<half_t, false, 0>(a, b, lds)))
KDEF(softmax_f32_wave, 256, kLdsRow, RowArgs, (row_cached_body<float, false, 64, 2, 0>(a, b, lds)))
KDEF(softmax_f32_block, 256, kLdsRow, RowArgs, (row_cached_body<float, false, 256, kRowCacheChunks, 0>(a, b, lds)))
KDEF(softmax_f32_generic, 256, kLdsRow, RowArgs, (row_generic_body<float, false, 0>(a, b, lds)))
KDEF(elt_f16_vec, 256, kLdsNone, EltArgs, (elt_body<half_t, 8, 0>(a, b, lds)))
KDEF(elt_f16_scalar, 256, kLdsNone, EltArgs, (elt_body<half_t, 1, 0>(a, b, lds)))
KDEF(elt_f32_vec, 256, kLdsNone, EltArgs, (elt_body<float, 4, 0>(a, b, lds)))
KDEF(elt_f32_scalar, 256, kLdsNone, EltArgs, (elt_body<float, 1, 0>(a, b, lds)))
KDEF(concat_f16_vec, 256, kLdsNone, ConcatArgs, (concat_body<half_t, 8, 0>(a, b, lds)))
KDEF(concat_f16_scalar, 256, kLdsNone, ConcatArgs, (concat_body<half_t, 1, 0>(a, b, lds)))
KDEF(concat_f32_vec, 256, kLdsNone, ConcatArgs, (concat_body<float, 4, 0>(a, b, lds)))
KDEF(concat_f32_scalar, 256, kLdsNone, ConcatArgs, (concat_body<float, 1, 0>(a, b, lds)))
// 16 x 16 output tiles: four times the workgroups of the 32 x 32 forms, half the operand bytes per workgroup
KDEF(igemm_f16_direct4s, 256, lds_direct(4), IgemmArgs, (igemm_direct_body<half_t, 4, 2, 0, 1, 1>(a, b, lds)))
KDEF(igemm_f16_quad4s, 256, lds_direct(4), IgemmArgs, (igemm_quad_body<half_t, 4, 0, 1, 1>(a, b, lds)))
KDEF(igemm_f32_direct4s, 256, lds_direct(4), IgemmArgs, (igemm_direct_body<float, 4, 2, 0, 1, 1>(a, b, lds)))
KDEF(igemm_f32_quad4s, 256, lds_direct(4), IgemmArgs, (igemm_quad_body<float, 4, 0, 1, 1>(a, b, lds)))

// ---------------------------------------------------------------------------------
// Persistent executor.  One launch runs the whole DAG: each workgroup repeatedly takes
// the next ticket, finds the operator and tile it denotes, waits until that operator's
// predecessors have completed all their tiles, runs the tile with the operator's own
// body, and publishes the completion.  Tickets follow the launch queue, which is a
// topological order, so the owner of the lowest unfinished ticket never waits for a
// ticket nobody holds: the launch drains whatever number of workgroups is resident.
// Every wait is bounded; a wait that runs out sets the sticky error word and all
// workgroups leave.  The last workgroup to leave clears the counters for the next launch.
// ---------------------------------------------------------------------------------
template <typename A> __device__ __forceinline__ A load_uniform(const void *p) {
  // Records are written once before the first launch and never by a kernel: read them
  // through the constant address space so they arrive in scalar registers like
  // ordinary kernel arguments.
  typedef const uint32_t __attribute__((address_space(4))) *CP;
  CP w = (CP)(uintptr_t)p;
  union { A a; uint32_t w[sizeof(A) / 4]; } u;
  static_assert(sizeof(A) % 4 == 0, "record size");
#pragma unroll
  for (unsigned i = 0; i < sizeof(A) / 4; ++i) u.w[i] = w[i];
  return u.a;
}

// Inputs inside the persistent kernel: either every load is device-coherent, or loads are
// plain and each work item starts with one cache invalidate (acquire at device scope).
#ifndef OPARA_PERSIST_COHERENT_LOADS
#define OPARA_PERSIST_COHERENT_LOADS 0
#endif
constexpr int kPersistAct = OPARA_PERSIST_COHERENT_LOADS ? kCohAct : kCohStore;
constexpr int kPersistActW = OPARA_PERSIST_COHERENT_LOADS ? (kCohAct | kCohW) : kCohStore;

template <bool F16>
__device__ __forceinline__ void persist_run(int kernel, const PersistOp *r, const Blk &b, unsigned char *lds) {
#define PCASE_(label, Args, call)                             \
  case label: {                                               \
    typedef const Args __attribute__((address_space(4))) CA;  \
    CA &a = *(CA *)(uintptr_t)&r->args;                       \
    call;                                                     \
  } break;
#define PCASE(name, Args, call) PCASE_(K_##name, Args, call)
#define PCASEW(name, Args, call) PCASE_(K_##name + kPersistActivationB, Args, call)
  if (F16) {
    switch (kernel) {
      PCASE(igemm_f16_t128x64, IgemmArgs, (igemm_pipe_body<half_t, 128, 64, 2, 2, 4, kPersistAct>(a, b, lds)))
      PCASE(igemm_f16_t64x64, IgemmArgs, (igemm_body<half_t, 64, 64, 2, 2, true, kPersistAct>(a, b, lds)))
      PCASE(igemm_f16_direct4, IgemmArgs, (igemm_direct_body<half_t, 4, 2, kPersistAct, 2, 2>(a, b, lds)))
      PCASE(igemm_f16_t64x64_scalar, IgemmArgs, (igemm_body<half_t, 64, 64, 2, 2, false, kPersistAct>(a, b, lds)))
      PCASEW(igemm_f16_t128x64, IgemmArgs, (igemm_pipe_body<half_t, 128, 64, 2, 2, 4, kPersistActW>(a, b, lds)))
      PCASEW(igemm_f16_t64x64, IgemmArgs, (igemm_body<half_t, 64, 64, 2, 2, true, kPersistActW>(a, b, lds)))
      PCASEW(igemm_f16_direct4, IgemmArgs, (igemm_direct_body<half_t, 4, 2, kPersistActW, 2, 2>(a, b, lds)))
      PCASEW(igemm_f16_t64x64_scalar, IgemmArgs, (igemm_body<half_t, 64, 64, 2, 2, false, kPersistActW>(a, b, lds)))
      PCASE(gemv_f16, IgemmArgs, (gemv_body<half_t, kPersistAct>(a, b, lds)))
      PCASE(pool_f16_vec, PoolArgs, (pool_body<half_t, 8, kPersistAct>(a, b, lds)))
      PCASE(pool_f16_scalar, PoolArgs, (pool_body<half_t, 1, kPersistAct>(a, b, lds)))
      PCASE(gap_f16, GapArgs, (gap_body<half_t, kPersistAct>(a, b, lds)))
      PCASE(layernorm_f16_wave, RowArgs, (row_cached_body<half_t, true, 64, 2, kPersistAct>(a, b, lds)))
      PCASE(layernorm_f16_block, RowArgs, (row_cached_body<half_t, true, 256, kRowCacheChunks, kPersistAct>(a, b, lds)))
      PCASE(layernorm_f16_generic, RowArgs, (row_generic_body<half_t, true, kPersistAct>(a, b, lds)))
      PCASE(softmax_f16_wave, RowArgs, (row_cached_body<half_t, false, 64, 2, kPersistAct>(a, b, lds)))
      PCASE(softmax_f16_block, RowArgs, (row_cached_body<half_t, false, 256, kRowCacheChunks, kPersistAct>(a, b, lds)))
      PCASE(softmax_f16_generic, RowArgs, (row_generic_body<half_t, false, kPersistAct>(a, b, lds)))
      PCASE(elt_f16_vec, EltArgs, (elt_body<half_t, 8, kPersistAct>(a, b, lds)))
      PCASE(elt_f16_scalar, EltArgs, (elt_body<half_t, 1, kPersistAct>(a, b, lds)))
      PCASE(concat_f16_vec, ConcatArgs, (concat_body<half_t, 8, kPersistAct>(a, b, lds)))
      PCASE(concat_f16_scalar, ConcatArgs, (concat_body<half_t, 1, kPersistAct>(a, b, lds)))
      default: break;
    }
  } else {
    switch (kernel) {
      PCASE(igemm_f32_t128x64, IgemmArgs, (igemm_pipe_body<float, 128, 64, 2, 2, 4, kPersistAct>(a, b, lds)))
      PCASE(igemm_f32_t64x64, IgemmArgs, (igemm_body<float, 64, 64, 2, 2, true, kPersistAct>(a, b, lds)))
      PCASE(igemm_f32_direct4, IgemmArgs, (igemm_direct_body<float, 4, 2, kPersistAct, 2, 2>(a, b, lds)))
      PCASE(igemm_f32_t64x64_scalar, IgemmArgs, (igemm_body<float, 64, 64, 2, 2, false, kPersistAct>(a, b, lds)))
      PCASEW(igemm_f32_t128x64, IgemmArgs, (igemm_pipe_body<float, 128, 64, 2, 2, 4, kPersistActW>(a, b, lds)))
      PCASEW(igemm_f32_t64x64, IgemmArgs, (igemm_body<float, 64, 64, 2, 2, true, kPersistActW>(a, b, lds)))
      PCASEW(igemm_f32_direct4, IgemmArgs, (igemm_direct_body<float, 4, 2, kPersistActW, 2, 2>(a, b, lds)))
      PCASEW(igemm_f32_t64x64_scalar, IgemmArgs, (igemm_body<float, 64, 64, 2, 2, false, kPersistActW>(a, b, lds)))
      PCASE(gemv_f32, IgemmArgs, (gemv_body<float, kPersistAct>(a, b, lds)))
      PCASE(pool_f32_vec, PoolArgs, (pool_body<float, 4, kPersistAct>(a, b, lds)))
      PCASE(pool_f32_scalar, PoolArgs, (pool_body<float, 1, kPersistAct>(a, b, lds)))
      PCASE(gap_f32, GapArgs, (gap_body<float, kPersistAct>(a, b, lds)))
      PCASE(layernorm_f32_wave, RowArgs, (row_cached_body<float, true, 64, 2, kPersistAct>(a, b, lds)))
      PCASE(layernorm_f32_block, RowArgs, (row_cached_body<float, true, 256, kRowCacheChunks, kPersistAct>(a, b, lds)))
      PCASE(layernorm_f32_generic, RowArgs, (row_generic_body<float, true, kPersistAct>(a, b, lds)))
      PCASE(softmax_f32_wave, RowArgs, (row_cached_body<float, false, 64, 2, kPersistAct>(a, b, lds)))
      PCASE(softmax_f32_block, RowArgs, (row_cached_body<float, false, 256, kRowCacheChunks, kPersistAct>(a, b, lds)))
      PCASE(softmax_f32_generic, RowArgs, (row_generic_body<float, false, kPersistAct>(a, b, lds)))
      PCASE(elt_f32_vec, EltArgs, (elt_body<float, 4, kPersistAct>(a, b, lds)))
      PCASE(elt_f32_scalar, EltArgs, (elt_body<float, 1, kPersistAct>(a, b, lds)))
      PCASE(concat_f32_vec, ConcatArgs, (concat_body<float, 4, kPersistAct>(a, b, lds)))
      PCASE(concat_f32_scalar, ConcatArgs, (concat_body<float, 1, kPersistAct>(a, b, lds)))
      default: break;
    }
  }
#undef PCASE
#undef PCASEW
#undef PCASE_
}

// Thread 0 only: wait until every predecessor of the operator at queue position `pos`
// has raised its flag for this launch.  Each workgroup polls its own copy of a flag
// (hundreds of workgroups polling one address queue up behind each other, and the
// counter updates behind them).  False: the wait ran out, or another workgroup's did.
__device__ __forceinline__ bool persist_wait(const PersistArgs &pa, const PersistPredsLds *pl, int pos, uint32_t epoch,
                                             uint32_t limit) {
  const int np = pl->n;
  const uint32_t copy = (blockIdx.x % kPersistReplicas) * kPersistFlagStride;
  uint32_t spins = 0;
  for (int j = 0; j < np; ++j) {
    const uint32_t *f = pa.flags + (size_t)pl->pos[j] * (kPersistReplicas * kPersistFlagStride) + copy;
    while (__hip_atomic_load(f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != epoch) {
      ++spins;
      if (spins > limit) {
        __hip_atomic_store(&pa.hdr->error, (uint32_t)pos + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return false;
      }
      if ((spins & 31u) == 0 && __hip_atomic_load(&pa.hdr->error, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0)
        return false;
      __builtin_amdgcn_s_sleep(1);
    }
  }
  return true;
}

// Thread 0 only, after the workgroup's stores are complete: count the finished tiles of
// the operator at `pos`; whoever counts the last tile clears the counter for the next
// launch and raises every copy of the operator's flag.
__device__ __forceinline__ void persist_publish(const PersistArgs &pa, const PersistPredsLds *preds, int pos, uint32_t count,
                                                uint32_t epoch) {
  uint32_t *d = pa.done + (size_t)pos * kPersistCounterStride;
  const uint32_t before = __hip_atomic_fetch_add(d, count, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (before + count == (uint32_t)preds[pos].tiles) {
    __hip_atomic_store(d, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    uint32_t *f = pa.flags + (size_t)pos * (kPersistReplicas * kPersistFlagStride);
#pragma unroll
    for (int r = 0; r < kPersistReplicas; ++r)
      __hip_atomic_store(f + r * kPersistFlagStride, epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

// Queue position of work item `item` (uniform; table in workgroup memory, begin[n] = total).
__device__ __forceinline__ int persist_find(const int32_t *begin, int n, uint32_t item) {
  int lo = 0, hi = n;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if ((uint32_t)begin[mid] <= item) lo = mid; else hi = mid;
  }
  return lo;
}

// Work items are dealt round-robin: workgroup g runs items g, g + G, g + 2G, ... of the
// launch queue, each after its operator's predecessors are complete.  The queue is a
// topological order and every workgroup of the launch is resident (the host sizes G to
// the occupancy), so the owner of the lowest unfinished item is always able to run it.
//
// Every activation access inside the bodies is device-coherent (see ldg/stg), so an item
// is published by waiting for the workgroup's stores and then bumping the operator's
// counter with relaxed atomics; a consumer that has read the full count may read the data.
//
// Each iteration has exactly ONE thread-0-only region (publish the previous item, await
// the predecessors of this one), placed before the first of its two barriers.  With a
// second such region after the last barrier the compiler threads thread 0 from the end of
// one iteration straight into the next; the other lanes of its wavefront then reach the
// barrier on their own, the wavefront arrives twice and the barrier count of the
// workgroup no longer matches.
template <bool F16>
__device__ __forceinline__ void persist_body(const PersistArgs &pa) {
  extern __shared__ __attribute__((aligned(16))) unsigned char dyn_lds[];
  unsigned char *lds = dyn_lds;                                  // kPersistBodyLds bytes for the bodies
  int32_t *ctl = (int32_t *)(dyn_lds + kPersistBodyLds);         // [4] abort flag, -, last-out flag
  int32_t *begin = ctl + 4;                                      // [n + 1]
  const PersistPredsLds *preds = (const PersistPredsLds *)(begin + pa.n + 1);   // [n]
  const int tid = threadIdx.x;
  for (int i = tid; i <= pa.n; i += 256) begin[i] = pa.item_begin[i];
  {
    const uint32_t *src = (const uint32_t *)pa.preds;
    uint32_t *dst = (uint32_t *)(begin + pa.n + 1);
    const int words = pa.n * (int)(sizeof(PersistPredsLds) / 4);
    for (int i = tid; i < words; i += 256) dst[i] = src[i];
  }
  if (tid == 0) ctl[0] = 0;
  // Optional timeline: four 64-bit words per work item (constant 100 MHz clock): lookup
  // started, predecessors complete, body finished, (queue position << 32 | workgroup).
  uint64_t *trace = nullptr;
  uint32_t limit = 0, epoch = 0;
  uint64_t t_begin = 0, t_ready = 0;
  if (tid == 0) {
    trace = (uint64_t *)__hip_atomic_load(&pa.hdr->trace, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    limit = __hip_atomic_load(&pa.hdr->spin_limit, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    epoch = __hip_atomic_load(&pa.hdr->epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  __syncthreads();
  int prev = -1;
  uint32_t prev_count = 0, sink = 0;
  for (uint32_t item = blockIdx.x; item < (uint32_t)pa.total; item += gridDim.x) {
    const int pos = __builtin_amdgcn_readfirstlane(persist_find(begin, pa.n, item));
    // A work item is `chunk` consecutive tiles of one operator (operators with more tiles
    // than the launch has workgroups: one acquire, one record, one publication for the lot).
    // Operators start at multiples of kPersistItemAlign in the item space; the items that
    // pad an operator out denote no tile.
    const int chunk = preds[pos].chunk;
    const int tile0 = (int)(item - (uint32_t)begin[pos]) * chunk;
    const int op_tiles = preds[pos].tiles;
    const bool padding = tile0 >= op_tiles;
    const int ntiles = padding ? 0 : min(chunk, op_tiles - tile0);
    if (tid == 0) {
      if (prev >= 0) {
        persist_publish(pa, preds, prev, prev_count, epoch);
        if (trace) {
          uint64_t *rec = trace + 4 * (uint64_t)(item - gridDim.x);
          const uint64_t t_end = wall_clock64();
          rec[0] = t_begin; rec[1] = t_ready; rec[2] = t_end;
          rec[3] = ((uint64_t)(uint32_t)prev << 32) | blockIdx.x;
        }
      }
      if (trace) t_begin = wall_clock64();
      if (!padding && !persist_wait(pa, preds + pos, pos, epoch, limit)) ctl[0] = 1;
      if (trace) t_ready = wall_clock64();
    }
    if (!OPARA_PERSIST_COHERENT_LOADS && tid < 64)               // one wavefront invalidates the caches this
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");         // workgroup reads through (L1 of the CU, L2 of the XCD)
    __syncthreads();                                             // predecessors complete (or abort)
    if (ctl[0]) { prev = -1; break; }
    if (padding) { prev = -1; continue; }
    const PersistOp *r = pa.rec + pos;
    const int4 hd = load_uniform<int4>(r);                       // kernel, gx, gy, gz
    Blk b;
    b.gx = hd.y; b.gy = hd.z;
    // With the workgroup count and every operator's first item multiples of the XCD count,
    // tile t of an unchunked operator runs on XCD t % 8 exactly as in an ordinary launch:
    // the same remap applies.  A chunk keeps consecutive tiles (neighbours that share
    // operand rows) in one workgroup instead.
    b.remap = chunk == 1 && (gridDim.x % kPersistItemAlign) == 0;
    for (int k = 0; k < ntiles; ++k) {
      const int tile = tile0 + k;
      b.x = tile % hd.y;
      const int rest = tile / hd.y;
      b.y = rest % hd.z;
      b.z = rest / hd.z;
      if (k > 0) __syncthreads();                                // the previous tile is done with workgroup memory
      persist_run<F16>(hd.x, r, b, lds);
    }
    // While the stores drain: touch the next item's record so that its argument loads find
    // it in the scalar cache.  The values only feed a sink that is tested after the loop.
    {
      const uint32_t nitem = item + gridDim.x;
      const int npos = nitem < (uint32_t)pa.total ? persist_find(begin, pa.n, nitem) : pos;
      const unsigned char *nr = (const unsigned char *)(pa.rec + __builtin_amdgcn_readfirstlane(npos));
      const uint32_t p0 = load_uniform<uint32_t>(nr), p1 = load_uniform<uint32_t>(nr + 64);
      const uint32_t p2 = load_uniform<uint32_t>(nr + 128), p3 = load_uniform<uint32_t>(nr + 192);
      sink += (p0 ^ p1) + (p2 ^ p3);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);                          // vmcnt(0): this wavefront's stores are complete
    __syncthreads();                                             // ... for every wavefront, and ctl has been read
    prev = pos;
    prev_count = (uint32_t)ntiles;
  }
  // Leave: publish the last item; the last workgroup out clears the counters (nobody is
  // left to read them) and advances the launch number.
  if (tid == 0) {
    if (prev >= 0) {
      persist_publish(pa, preds, prev, prev_count, epoch);
      if (trace) {
        // the loop has advanced `item` past the end: the last item of this workgroup is the
        // largest g + k*G below total
        const uint32_t last = blockIdx.x + ((uint32_t)pa.total - 1u - blockIdx.x) / gridDim.x * gridDim.x;
        uint64_t *rec = trace + 4 * (uint64_t)last;
        rec[0] = t_begin; rec[1] = t_ready; rec[2] = wall_clock64();
        rec[3] = ((uint64_t)(uint32_t)prev << 32) | blockIdx.x;
      }
    }
    if (sink == 0x9e3779b9u) pa.hdr->reserved0 = sink;           // keeps the record touches alive
    const uint32_t e = __hip_atomic_fetch_add(&pa.hdr->exited, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    ctl[2] = (e == gridDim.x - 1) ? 1 : 0;
  }
  __syncthreads();
  if (ctl[2]) {
    // Counters of operators that did not complete (abandoned launch) would poison the
    // next one; after a clean launch they are all zero already.
    for (int i = tid; i < pa.n; i += 256) pa.done[(size_t)i * kPersistCounterStride] = 0u;
    if (tid == 0) {
      pa.hdr->exited = 0u;
      pa.hdr->epoch = epoch + 1u;
    }
  }
}

extern "C" __global__ void __launch_bounds__(256, 2) opara_k_persist_f16(PersistArgs pa) { persist_body<true>(pa); }
extern "C" __global__ void __launch_bounds__(256, 2) opara_k_persist_f32(PersistArgs pa) { persist_body<false>(pa); }

// ---------------------------------------------------------------------------------
// Group kernel (fused executor): one launch runs several mutually independent operators.
// A workgroup finds its operator from the block ranges in the argument record, rebuilds
// its position in that operator's own grid and runs the operator's ordinary body on the
// operator's arguments, which it reads from the kernel-argument segment like any kernel
// does.  No flags, no coherent accesses: kernel boundaries order the groups.  Three flavours
// per element type, by the registers their bodies need: "stream" (at most 64: pooling,
// row-wise, element-wise, concatenation, matrix-vector; eight wavefronts per SIMD stay
// resident, which streaming wants), "light" (at most 128: those plus the fragment-loading
// and 16 x 16-tile contractions; four per SIMD), "heavy" (all 256-thread bodies; two).
// ---------------------------------------------------------------------------------
template <bool F16, int FLAVOR, bool TRACE>
__device__ __forceinline__ void group_body() {
  // The record is the kernel's only argument and therefore starts the kernel-argument
  // segment.  It is read in place through the segment pointer: indexing the by-value
  // parameter with a run-time operator number would make the compiler copy all of it into
  // private memory first.
  typedef const GroupArgs __attribute__((address_space(4))) CGA;
  CGA &ga = *(CGA *)__builtin_amdgcn_kernarg_segment_ptr();
  extern __shared__ __attribute__((aligned(16))) unsigned char dyn_lds[];
  const int blk = (int)blockIdx.x;
  // The member this block belongs to: all sixteen range ends arrive with one 64-byte load
  // (unused entries hold INT32_MAX), the member is the number of ends at or below the block.
  int i = 0;
#pragma unroll
  for (int j = 0; j < kGroupMaxOps - 1; ++j) i += blk >= ga.block_end[j] ? 1 : 0;
  i = __builtin_amdgcn_readfirstlane(i);
  // One 32-byte load for the member's launch shape; and, in the same round, a touch of every
  // cache line of its argument record, so that the body's own argument loads (which the
  // compiler issues only behind the switch below) find it in the scalar cache instead of
  // paying a third dependent memory round trip.  The touched words only feed a sink.
  typedef const uint32_t __attribute__((address_space(4))) *CW;
  const CW rec = (CW)&ga.args[i];
  const uint32_t touch = (rec[0] ^ rec[16]) + (rec[32] ^ rec[47]);
  typedef const GroupMeta __attribute__((address_space(4))) CM;
  CM &me = ga.meta[i];
  const int tile = blk - me.block_begin;
  if (tile >= me.tiles) return;                                    // padding of the operator's range
  Blk b;
  b.gx = me.gx; b.gy = me.gy;
  b.remap = true;
  b.x = tile % b.gx;
  const int rest = tile / b.gx;
  b.y = rest % b.gy;
  b.z = rest / b.gy;
  unsigned char *lds = dyn_lds;
  // traced instances are separate kernels: even an unused clock read at the start of this
  // kernel's chain of dependent scalar loads cost every group node 0.4 us
  const int tag = TRACE ? me.tag : 0;
  const unsigned long long t0 = TRACE ? op_trace_begin() : 0ull;
#define GCASE(name, Args, call)                               \
  case K_##name: {                                            \
    typedef const Args __attribute__((address_space(4))) CA;  \
    CA &a = *(CA *)&ga.args[i];                               \
    call;                                                     \
  } break;
  if constexpr (F16) {
    switch (me.kernel) {
      GCASE(gemv_f16, IgemmArgs, (gemv_body<half_t, 0>(a, b, lds)))
      GCASE(pool_f16_vec, PoolArgs, (pool_body<half_t, 8, 0>(a, b, lds)))
      GCASE(pool_f16_scalar, PoolArgs, (pool_body<half_t, 1, 0>(a, b, lds)))
      GCASE(gap_f16, GapArgs, (gap_body<half_t, 0>(a, b, lds)))
      GCASE(layernorm_f16_wave, RowArgs, (row_cached_body<half_t, true, 64, 2, 0>(a, b, lds)))
      GCASE(layernorm_f16_block, RowArgs, (row_cached_body<half_t, true, 256, kRowCacheChunks, 0>(a, b, lds)))
      GCASE(layernorm_f16_generic, RowArgs, (row_generic_body<half_t, true, 0>(a, b, lds)))
      GCASE(softmax_f16_wave, RowArgs, (row_cached_body<half_t, false, 64, 2, 0>(a, b, lds)))
      GCASE(softmax_f16_block, RowArgs, (row_cached_body<half_t, false, 256, kRowCacheChunks, 0>(a, b, lds)))
      GCASE(softmax_f16_generic, RowArgs, (row_generic_body<half_t, false, 0>(a, b, lds)))
      GCASE(elt_f16_vec, EltArgs, (elt_body<half_t, 8, 0>(a, b, lds)))
      GCASE(elt_f16_scalar, EltArgs, (elt_body<half_t, 1, 0>(a, b, lds)))
      GCASE(concat_f16_vec, ConcatArgs, (concat_body<half_t, 8, 0>(a, b, lds)))
      GCASE(concat_f16_scalar, ConcatArgs, (concat_body<half_t, 1, 0>(a, b, lds)))
      default:
        if constexpr (FLAVOR >= 1) {
          switch (me.kernel) {
            GCASE(igemm_f16_t64x64, IgemmArgs, (igemm_body<half_t, 64, 64, 2, 2, true, 0>(a, b, lds)))
            GCASE(igemm_f16_direct4, IgemmArgs, (igemm_direct_body<half_t, 4, 2, 0, 2, 2>(a, b, lds)))
            GCASE(igemm_f16_direct4s, IgemmArgs, (igemm_direct_body<half_t, 4, 2, 0, 1, 1>(a, b, lds)))
            GCASE(igemm_f16_quad4s, IgemmArgs, (igemm_quad_body<half_t, 4, 0, 1, 1>(a, b, lds)))
            GCASE(igemm_f16_t64x64_scalar, IgemmArgs, (igemm_body<half_t, 64, 64, 2, 2, false, 0>(a, b, lds)))
            default:
              if constexpr (FLAVOR >= 2) {
                switch (me.kernel) {
                  GCASE(igemm_f16_t128x64, IgemmArgs, (igemm_pipe_body<half_t, 128, 64, 2, 2, 4, 0>(a, b, lds)))
                  GCASE(igemm_f16_quad4, IgemmArgs, (igemm_quad_body<half_t, 4, 0, 2, 2>(a, b, lds)))
                  GCASE(igemm_f16_quad64x4, IgemmArgs, (igemm_quad64_body<half_t, 4, 0>(a, b, lds)))
                  default: break;
                }
              }
              break;
          }
        }
        break;
    }
  } else {
    switch (me.kernel) {
      GCASE(gemv_f32, IgemmArgs, (gemv_body<float, 0>(a, b, lds)))
      GCASE(pool_f32_vec, PoolArgs, (pool_body<float, 4, 0>(a, b, lds)))
      GCASE(pool_f32_scalar, PoolArgs, (pool_body<float, 1, 0>(a, b, lds)))
      GCASE(gap_f32, GapArgs, (gap_body<float, 0>(a, b, lds)))
      GCASE(layernorm_f32_wave, RowArgs, (row_cached_body<float, true, 64, 2, 0>(a, b, lds)))
      GCASE(layernorm_f32_block, RowArgs, (row_cached_body<float, true, 256, kRowCacheChunks, 0>(a, b, lds)))
      GCASE(layernorm_f32_generic, RowArgs, (row_generic_body<float, true, 0>(a, b, lds)))
      GCASE(softmax_f32_wave, RowArgs, (row_cached_body<float, false, 64, 2, 0>(a, b, lds)))
      GCASE(softmax_f32_block, RowArgs, (row_cached_body<float, false, 256, kRowCacheChunks, 0>(a, b, lds)))
      GCASE(softmax_f32_generic, RowArgs, (row_generic_body<float, false, 0>(a, b, lds)))
      GCASE(elt_f32_vec, EltArgs, (elt_body<float, 4, 0>(a, b, lds)))
      GCASE(elt_f32_scalar, EltArgs, (elt_body<float, 1, 0>(a, b, lds)))
      GCASE(concat_f32_vec, ConcatArgs, (concat_body<float, 4, 0>(a, b, lds)))
      GCASE(concat_f32_scalar, ConcatArgs, (concat_body<float, 1, 0>(a, b, lds)))
      default:
        if constexpr (FLAVOR >= 1) {
          switch (me.kernel) {
            GCASE(igemm_f32_t64x64, IgemmArgs, (igemm_body<float, 64, 64, 2, 2, true, 0>(a, b, lds)))
            GCASE(igemm_f32_direct4, IgemmArgs, (igemm_direct_body<float, 4, 2, 0, 2, 2>(a, b, lds)))
            GCASE(igemm_f32_direct4s, IgemmArgs, (igemm_direct_body<float, 4, 2, 0, 1, 1>(a, b, lds)))
            GCASE(igemm_f32_quad4s, IgemmArgs, (igemm_quad_body<float, 4, 0, 1, 1>(a, b, lds)))
            GCASE(igemm_f32_t64x64_scalar, IgemmArgs, (igemm_body<float, 64, 64, 2, 2, false, 0>(a, b, lds)))
            default:
              if constexpr (FLAVOR >= 2) {
                switch (me.kernel) {
                  GCASE(igemm_f32_t128x64, IgemmArgs, (igemm_pipe_body<float, 128, 64, 2, 2, 4, 0>(a, b, lds)))
                  GCASE(igemm_f32_quad4, IgemmArgs, (igemm_quad_body<float, 4, 0, 2, 2>(a, b, lds)))
                  GCASE(igemm_f32_quad64x4, IgemmArgs, (igemm_quad64_body<float, 4, 0>(a, b, lds)))
                  default: break;
                }
              }
              break;
          }
        }
        break;
    }
  }
#undef GCASE
  if constexpr (TRACE) op_trace_end(ga.trace, tag, t0, (unsigned)tile, (unsigned)me.tiles);
  if (touch == 0x9e3779b9u && blk == 0x7fffffff) lds[0] = 1;       // keeps the touches alive; never true
}

#define GROUPK(name, waves, F16, FLAVOR)                                                                                          \
  extern "C" __global__ void __launch_bounds__(256, waves) opara_k_group_##name(GroupArgs) { group_body<F16, FLAVOR, false>(); }     \
  extern "C" __global__ void __launch_bounds__(256, waves) opara_k_group_##name##_traced(GroupArgs) { group_body<F16, FLAVOR, true>(); }
GROUPK(f16_stream, 8, true, 0)
GROUPK(f16_light, 4, true, 1)
GROUPK(f16_heavy, 2, true, 2)
GROUPK(f32_stream, 8, false, 0)
GROUPK(f32_light, 4, false, 1)
GROUPK(f32_heavy, 2, false, 2)
#undef GROUPK

// ---------------------------------------------------------------------------------
// Chained executor: every workgroup runs one tile of one operator behind a wait for the
// operator's predecessors (see ChainArgs).  Same hand-off as the persistent kernel (results
// through device-coherent stores, completion counters and replicated flags, one cache
// invalidate per workgroup), but no loop: a body is straight-line code behind the wait, so
// nothing is hoisted across bodies, the quad-coalesced contractions can be held, and the
// launch does not depend on all its workgroups being resident at once.
// ---------------------------------------------------------------------------------
template <bool F16, bool LIGHT>
__device__ __forceinline__ void chain_body(const ChainArgs &pa) {
  extern __shared__ __attribute__((aligned(16))) unsigned char dyn_lds[];
  __shared__ int32_t ctl[2];
  typedef const int32_t __attribute__((address_space(4))) *CI;
  const int blk = (int)blockIdx.x;
  const int pos = __builtin_amdgcn_readfirstlane(((CI)(uintptr_t)pa.block_op)[blk]);
  if (pos < 0) return;                                            // padding of an operator's block range
  typedef const ChainRec __attribute__((address_space(4))) CR;
  CR &r = *(CR *)(uintptr_t)(pa.rec + pos);
  const int tid = threadIdx.x;
  uint64_t *trace = nullptr;
  uint64_t t_begin = 0, t_ready = 0;
  uint32_t epoch = 0;
  if (tid == 0) {
    trace = (uint64_t *)__hip_atomic_load(&pa.hdr->trace, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (trace) t_begin = wall_clock64();
    const uint32_t limit = __hip_atomic_load(&pa.hdr->spin_limit, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    epoch = __hip_atomic_load(&pa.hdr->epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const uint32_t copy = ((uint32_t)blk % kPersistReplicas) * kPersistFlagStride;
    const int np = r.n_preds;
    uint32_t spins = 0;
    int ok = 1;
    for (int j = 0; j < np && ok; ++j) {
      const uint32_t *f = pa.flags + (size_t)r.preds[j] * (kPersistReplicas * kPersistFlagStride) + copy;
      while (__hip_atomic_load(f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != epoch) {
        if (++spins > limit) {
          __hip_atomic_store(&pa.hdr->error, (uint32_t)pos + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          ok = 0;
          break;
        }
        if ((spins & 31u) == 0 && __hip_atomic_load(&pa.hdr->error, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) {
          ok = 0;
          break;
        }
        __builtin_amdgcn_s_sleep(1);
      }
    }
    ctl[0] = ok;
    if (trace) t_ready = wall_clock64();
  }
  if (tid < 64) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");  // after the wait (thread 0 is in this wavefront)
  __syncthreads();
  if (!ctl[0]) return;                                            // a wait ran out somewhere: leave, publish nothing
  Blk b;
  b.gx = r.gx; b.gy = r.gy;
  b.remap = true;
  const int tile = blk - r.begin;
  b.x = tile % b.gx;
  const int rest = tile / b.gx;
  b.y = rest % b.gy;
  b.z = rest / b.gy;
  unsigned char *lds = dyn_lds;
#define CCASE_(label, Args, call)                             \
  case label: {                                               \
    typedef const Args __attribute__((address_space(4))) CA;  \
    CA &a = *(CA *)&r.args;                                   \
    call;                                                     \
  } break;
#define CCASE(name, Args, call) CCASE_(K_##name, Args, call)
#define CCASEW(name, Args, call) CCASE_(K_##name + kPersistActivationB, Args, call)
  constexpr int A = kCohStore, AW = kCohStore;
  if constexpr (F16) {
    switch (r.kernel) {
      CCASE(igemm_f16_t64x64, IgemmArgs, (igemm_body<half_t, 64, 64, 2, 2, true, A>(a, b, lds)))
      CCASE(igemm_f16_direct4, IgemmArgs, (igemm_direct_body<half_t, 4, 2, A, 2, 2>(a, b, lds)))
      CCASE(igemm_f16_direct4s, IgemmArgs, (igemm_direct_body<half_t, 4, 2, A, 1, 1>(a, b, lds)))
      CCASEW(igemm_f16_direct4s, IgemmArgs, (igemm_direct_body<half_t, 4, 2, AW, 1, 1>(a, b, lds)))
      CCASE(igemm_f16_quad4s, IgemmArgs, (igemm_quad_body<half_t, 4, A, 1, 1>(a, b, lds)))
      CCASEW(igemm_f16_quad4s, IgemmArgs, (igemm_quad_body<half_t, 4, AW, 1, 1>(a, b, lds)))
      CCASE(igemm_f16_t64x64_scalar, IgemmArgs, (igemm_body<half_t, 64, 64, 2, 2, false, A>(a, b, lds)))
      CCASEW(igemm_f16_t64x64, IgemmArgs, (igemm_body<half_t, 64, 64, 2, 2, true, AW>(a, b, lds)))
      CCASEW(igemm_f16_direct4, IgemmArgs, (igemm_direct_body<half_t, 4, 2, AW, 2, 2>(a, b, lds)))
      CCASEW(igemm_f16_t64x64_scalar, IgemmArgs, (igemm_body<half_t, 64, 64, 2, 2, false, AW>(a, b, lds)))
      CCASE(gemv_f16, IgemmArgs, (gemv_body<half_t, A>(a, b, lds)))
      CCASE(pool_f16_vec, PoolArgs, (pool_body<half_t, 8, A>(a, b, lds)))
      CCASE(pool_f16_scalar, PoolArgs, (pool_body<half_t, 1, A>(a, b, lds)))
      CCASE(gap_f16, GapArgs, (gap_body<half_t, A>(a, b, lds)))
      CCASE(layernorm_f16_wave, RowArgs, (row_cached_body<half_t, true, 64, 2, A>(a, b, lds)))
      CCASE(layernorm_f16_block, RowArgs, (row_cached_body<half_t, true, 256, kRowCacheChunks, A>(a, b, lds)))
      CCASE(layernorm_f16_generic, RowArgs, (row_generic_body<half_t, true, A>(a, b, lds)))
      CCASE(softmax_f16_wave, RowArgs, (row_cached_body<half_t, false, 64, 2, A>(a, b, lds)))
      CCASE(softmax_f16_block, RowArgs, (row_cached_body<half_t, false, 256, kRowCacheChunks, A>(a, b, lds)))
      CCASE(softmax_f16_generic, RowArgs, (row_generic_body<half_t, false, A>(a, b, lds)))
      CCASE(elt_f16_vec, EltArgs, (elt_body<half_t, 8, A>(a, b, lds)))
      CCASE(elt_f16_scalar, EltArgs, (elt_body<half_t, 1, A>(a, b, lds)))
      CCASE(concat_f16_vec, ConcatArgs, (concat_body<half_t, 8, A>(a, b, lds)))
      CCASE(concat_f16_scalar, ConcatArgs, (concat_body<half_t, 1, A>(a, b, lds)))
      default:
        if constexpr (!LIGHT) {
          switch (r.kernel) {
            CCASE(igemm_f16_t128x64, IgemmArgs, (igemm_pipe_body<half_t, 128, 64, 2, 2, 4, A>(a, b, lds)))
            CCASE(igemm_f16_quad4, IgemmArgs, (igemm_quad_body<half_t, 4, A, 2, 2>(a, b, lds)))
            CCASE(igemm_f16_quad64x4, IgemmArgs, (igemm_quad64_body<half_t, 4, A>(a, b, lds)))
            CCASEW(igemm_f16_t128x64, IgemmArgs, (igemm_pipe_body<half_t, 128, 64, 2, 2, 4, AW>(a, b, lds)))
            CCASEW(igemm_f16_quad4, IgemmArgs, (igemm_quad_body<half_t, 4, AW, 2, 2>(a, b, lds)))
            CCASEW(igemm_f16_quad64x4, IgemmArgs, (igemm_quad64_body<half_t, 4, AW>(a, b, lds)))
            default: break;
          }
        }
        break;
    }
  } else {
    switch (r.kernel) {
      CCASE(igemm_f32_t64x64, IgemmArgs, (igemm_body<float, 64, 64, 2, 2, true, A>(a, b, lds)))
      CCASE(igemm_f32_direct4, IgemmArgs, (igemm_direct_body<float, 4, 2, A, 2, 2>(a, b, lds)))
      CCASE(igemm_f32_direct4s, IgemmArgs, (igemm_direct_body<float, 4, 2, A, 1, 1>(a, b, lds)))
      CCASEW(igemm_f32_direct4s, IgemmArgs, (igemm_direct_body<float, 4, 2, AW, 1, 1>(a, b, lds)))
      CCASE(igemm_f32_quad4s, IgemmArgs, (igemm_quad_body<float, 4, A, 1, 1>(a, b, lds)))
      CCASEW(igemm_f32_quad4s, IgemmArgs, (igemm_quad_body<float, 4, AW, 1, 1>(a, b, lds)))
      CCASE(igemm_f32_t64x64_scalar, IgemmArgs, (igemm_body<float, 64, 64, 2, 2, false, A>(a, b, lds)))
      CCASEW(igemm_f32_t64x64, IgemmArgs, (igemm_body<float, 64, 64, 2, 2, true, AW>(a, b, lds)))
      CCASEW(igemm_f32_direct4, IgemmArgs, (igemm_direct_body<float, 4, 2, AW, 2, 2>(a, b, lds)))
      CCASEW(igemm_f32_t64x64_scalar, IgemmArgs, (igemm_body<float, 64, 64, 2, 2, false, AW>(a, b, lds)))
      CCASE(gemv_f32, IgemmArgs, (gemv_body<float, A>(a, b, lds)))
      CCASE(pool_f32_vec, PoolArgs, (pool_body<float, 4, A>(a, b, lds)))
      CCASE(pool_f32_scalar, PoolArgs, (pool_body<float, 1, A>(a, b, lds)))
      CCASE(gap_f32, GapArgs, (gap_body<float, A>(a, b, lds)))
      CCASE(layernorm_f32_wave, RowArgs, (row_cached_body<float, true, 64, 2, A>(a, b, lds)))
      CCASE(layernorm_f32_block, RowArgs, (row_cached_body<float, true, 256, kRowCacheChunks, A>(a, b, lds)))
      CCASE(layernorm_f32_generic, RowArgs, (row_generic_body<float, true, A>(a, b, lds)))
      CCASE(softmax_f32_wave, RowArgs, (row_cached_body<float, false, 64, 2, A>(a, b, lds)))
      CCASE(softmax_f32_block, RowArgs, (row_cached_body<float, false, 256, kRowCacheChunks, A>(a, b, lds)))
      CCASE(softmax_f32_generic, RowArgs, (row_generic_body<float, false, A>(a, b, lds)))
      CCASE(elt_f32_vec, EltArgs, (elt_body<float, 4, A>(a, b, lds)))
      CCASE(elt_f32_scalar, EltArgs, (elt_body<float, 1, A>(a, b, lds)))
      CCASE(concat_f32_vec, ConcatArgs, (concat_body<float, 4, A>(a, b, lds)))
      CCASE(concat_f32_scalar, ConcatArgs, (concat_body<float, 1, A>(a, b, lds)))
      default:
        if constexpr (!LIGHT) {
          switch (r.kernel) {
            CCASE(igemm_f32_t128x64, IgemmArgs, (igemm_pipe_body<float, 128, 64, 2, 2, 4, A>(a, b, lds)))
            CCASE(igemm_f32_quad4, IgemmArgs, (igemm_quad_body<float, 4, A, 2, 2>(a, b, lds)))
            CCASE(igemm_f32_quad64x4, IgemmArgs, (igemm_quad64_body<float, 4, A>(a, b, lds)))
            CCASEW(igemm_f32_t128x64, IgemmArgs, (igemm_pipe_body<float, 128, 64, 2, 2, 4, AW>(a, b, lds)))
            CCASEW(igemm_f32_quad4, IgemmArgs, (igemm_quad_body<float, 4, AW, 2, 2>(a, b, lds)))
            CCASEW(igemm_f32_quad64x4, IgemmArgs, (igemm_quad64_body<float, 4, AW>(a, b, lds)))
            default: break;
          }
        }
        break;
    }
  }
#undef CCASE
#undef CCASEW
#undef CCASE_
  __builtin_amdgcn_s_waitcnt(0x0F70);                            // vmcnt(0): this wavefront's stores are complete
  __syncthreads();                                               // ... for every wavefront of the workgroup
  if (tid == 0) {
    uint32_t *d = pa.done + (size_t)pos * kPersistCounterStride;
    const uint32_t before = __hip_atomic_fetch_add(d, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (before + 1u == (uint32_t)r.tiles) {                      // the operator's last tile: raise its flags
      __hip_atomic_store(d, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      uint32_t *f = pa.flags + (size_t)pos * (kPersistReplicas * kPersistFlagStride);
#pragma unroll
      for (int q = 0; q < kPersistReplicas; ++q)
        __hip_atomic_store(f + q * kPersistFlagStride, epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      // the last operator to complete advances the launch number for the next replay
      const uint32_t ops = __hip_atomic_fetch_add(&pa.hdr->exited, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (ops + 1u == (uint32_t)pa.n) {
        __hip_atomic_store(&pa.hdr->exited, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(&pa.hdr->epoch, epoch + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
    if (trace) {
      uint64_t *rec = trace + 4 * (uint64_t)blk;
      rec[0] = t_begin; rec[1] = t_ready; rec[2] = wall_clock64();
      rec[3] = ((uint64_t)(uint32_t)pos << 32) | (uint32_t)blk;
    }
  }
}

extern "C" __global__ void __launch_bounds__(256, 4) opara_k_chain_f16_light(ChainArgs pa) { chain_body<true, true>(pa); }
extern "C" __global__ void __launch_bounds__(256, 2) opara_k_chain_f16_heavy(ChainArgs pa) { chain_body<true, false>(pa); }
extern "C" __global__ void __launch_bounds__(256, 4) opara_k_chain_f32_light(ChainArgs pa) { chain_body<false, true>(pa); }
extern "C" __global__ void __launch_bounds__(256, 2) opara_k_chain_f32_heavy(ChainArgs pa) { chain_body<false, false>(pa); }

// Dependency self-check: done-tokens per operator and a violation counter, in static
// device memory (nothing is allocated).
static __device__ int g_verify_tok[opara::kVerifyMaxOps];
static __device__ int g_verify_viol[4];   // violations, then 1 + operator and predecessor of the last one

extern "C" __global__ void opara_k_token(opara::TokenNodeArgs node) {
  const opara::TokenArgs &a = node.tok;
  if (threadIdx.x != 0) return;
  for (int i = 0; i < a.n_preds; ++i)
    if (__hip_atomic_load(&g_verify_tok[a.preds[i]], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != a.epoch) {
      atomicAdd(&g_verify_viol[0], 1);
      g_verify_viol[1] = a.self + 1;
      g_verify_viol[2] = a.preds[i];
    }
  for (int i = 0; i < a.delay; ++i) __builtin_amdgcn_s_sleep(127);   // bounded: a few microseconds
  __hip_atomic_store(&g_verify_tok[a.self], a.epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Workspace of the persistent executor for callers that cannot allocate device memory:
// counters, completion flags and operator records of up to kStaticWorkspaceMaxOps
// operators.  Every GPU the library runs on holds its own copy at its own address until
// the process ends; host code reaches it only through the address static_workspace()
// looks up (the array's name is a host-side stand-in, not a device address).
constexpr size_t kScratchBytes = 2560u * 1024u;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

// Kernel without work: a pure dependency node (common root / common leaf of a capture).
extern "C" __global__ void opara_k_noop(int) {}

namespace opara {

// Operator-timeline buffer that launches and captures made from now on hand to their kernels.
static unsigned long long *g_host_op_trace = nullptr;

hipError_t launch_noop(hipStream_t s) {
  hipLaunchKernelGGL(opara_k_noop, dim3(1), dim3(64), 0, s, 0);
  return hipGetLastError();
}

namespace {
template <typename A> const A &arg_of(const KernelArgs &u);
template <> const IgemmArgs &arg_of<IgemmArgs>(const KernelArgs &u) { return u.igemm; }
template <> const PoolArgs &arg_of<PoolArgs>(const KernelArgs &u) { return u.pool; }
template <> const GapArgs &arg_of<GapArgs>(const KernelArgs &u) { return u.gap; }
template <> const RowArgs &arg_of<RowArgs>(const KernelArgs &u) { return u.row; }
template <> const EltArgs &arg_of<EltArgs>(const KernelArgs &u) { return u.elt; }
template <> const ConcatArgs &arg_of<ConcatArgs>(const KernelArgs &u) { return u.concat; }
}  // namespace

hipError_t launch_plan(const KernelPlan &p, hipStream_t s) {
  const dim3 grid(p.gx, p.gy, p.gz), block(p.block);
  switch (p.kernel) {
#define X(name, A)                                                                     \
  case K_##name:                                                                       \
    hipLaunchKernelGGL(opara_k_##name, grid, block, 0, s, arg_of<A>(p.args), p.tag, g_host_op_trace);   \
    break;
    OPARA_KERNEL_LIST(X)
#undef X
    default:
      return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t add_plan_node(hipGraph_t graph, const KernelPlan &p, const hipGraphNode_t *deps, size_t n_deps,
                         hipGraphNode_t *node) {
  void *func = const_cast<void *>(kernel_symbol(p.kernel));
  if (!func) return hipErrorInvalidValue;
  KernelArgs args = p.args;              // every kernel takes one by-value record at offset 0, then the operator id
  int32_t tag = p.tag;
  unsigned long long *trace = g_host_op_trace;
  void *kparams[3] = {&args, &tag, &trace};
  hipKernelNodeParams np = {};
  np.func = func;
  np.gridDim = dim3(p.gx, p.gy, p.gz);
  np.blockDim = dim3(p.block);
  np.sharedMemBytes = 0;
  np.kernelParams = kparams;
  np.extra = nullptr;
  return hipGraphAddKernelNode(node, graph, deps, n_deps, &np);
}

hipError_t set_exec_node_plan(hipGraphExec_t exec, hipGraphNode_t node, const KernelPlan &p) {
  void *func = const_cast<void *>(kernel_symbol(p.kernel));
  if (!func) return hipErrorInvalidValue;
  KernelArgs args = p.args;
  int32_t tag = p.tag;
  unsigned long long *trace = g_host_op_trace;
  void *kparams[3] = {&args, &tag, &trace};
  hipKernelNodeParams np = {};
  np.func = func;
  np.gridDim = dim3(p.gx, p.gy, p.gz);
  np.blockDim = dim3(p.block);
  np.sharedMemBytes = 0;
  np.kernelParams = kparams;
  np.extra = nullptr;
  return hipGraphExecKernelNodeSetParams(exec, node, &np);
}

hipError_t add_noop_node(hipGraph_t graph, const hipGraphNode_t *deps, size_t n_deps, hipGraphNode_t *node) {
  int zero = 0;
  void *kparams[1] = {&zero};
  hipKernelNodeParams np = {};
  np.func = (void *)opara_k_noop;
  np.gridDim = dim3(1);
  np.blockDim = dim3(64);
  np.kernelParams = kparams;
  return hipGraphAddKernelNode(node, graph, deps, n_deps, &np);
}

hipError_t add_token_node(hipGraph_t graph, const TokenNodeArgs &t, const hipGraphNode_t *deps, size_t n_deps,
                          hipGraphNode_t *node) {
  TokenNodeArgs args = t;
  void *kparams[1] = {&args};
  hipKernelNodeParams np = {};
  np.func = (void *)opara_k_token;
  np.gridDim = dim3(1);
  np.blockDim = dim3(64);
  np.kernelParams = kparams;
  return hipGraphAddKernelNode(node, graph, deps, n_deps, &np);
}

namespace {
void *group_func(bool f16, int flavor, bool traced) {
  static void *const f[2][2][3] = {
      {{(void *)opara_k_group_f32_stream, (void *)opara_k_group_f32_light, (void *)opara_k_group_f32_heavy},
       {(void *)opara_k_group_f16_stream, (void *)opara_k_group_f16_light, (void *)opara_k_group_f16_heavy}},
      {{(void *)opara_k_group_f32_stream_traced, (void *)opara_k_group_f32_light_traced, (void *)opara_k_group_f32_heavy_traced},
       {(void *)opara_k_group_f16_stream_traced, (void *)opara_k_group_f16_light_traced, (void *)opara_k_group_f16_heavy_traced}}};
  return f[traced ? 1 : 0][f16 ? 1 : 0][flavor < 0 ? 0 : flavor > 2 ? 2 : flavor];
}
}  // namespace

int group_flavor(int id) {
  switch (id) {
    case K_igemm_f16_t128x64: case K_igemm_f32_t128x64: case K_igemm_f16_quad4: case K_igemm_f32_quad4:
    case K_igemm_f16_quad64x4: case K_igemm_f32_quad64x4:
      return 2;
    case K_igemm_f16_direct8: case K_igemm_f32_direct8: case K_igemm_f16_quad8: case K_igemm_f32_quad8:
      return -1;                          // 512-thread bodies
    case K_igemm_f16_t64x64: case K_igemm_f32_t64x64: case K_igemm_f16_direct4: case K_igemm_f32_direct4:
    case K_igemm_f16_direct4s: case K_igemm_f32_direct4s: case K_igemm_f16_quad4s: case K_igemm_f32_quad4s:
    case K_igemm_f16_t64x64_scalar: case K_igemm_f32_t64x64_scalar:
      return 1;
    default:
      return id >= 0 && id < K_COUNT ? 0 : -1;
  }
}

bool group_kernel_ok(int id, bool *light) {
  const int f = group_flavor(id);
  *light = f >= 0 && f < 2;
  return f >= 0;
}

hipError_t group_prepare(uint32_t max_lds_bytes) {
  for (int f16 = 0; f16 < 2; ++f16)
    for (int flavor = 0; flavor < 3; ++flavor)
      for (int traced = 0; traced < 2; ++traced) {
        hipError_t err = hipFuncSetAttribute(group_func(f16, flavor, traced), hipFuncAttributeMaxDynamicSharedMemorySize,
                                             (int)max_lds_bytes);
        if (err != hipSuccess) return err;
      }
  return hipSuccess;
}

hipError_t add_group_node(hipGraph_t graph, bool f16, int flavor, const GroupArgs &ga, uint32_t n_blocks,
                          uint32_t lds_bytes, const hipGraphNode_t *deps, size_t n_deps, hipGraphNode_t *node) {
  GroupArgs args = ga;
  void *kparams[1] = {&args};
  hipKernelNodeParams np = {};
  np.func = group_func(f16, flavor, ga.trace != nullptr);
  np.gridDim = dim3(n_blocks);
  np.blockDim = dim3(256);
  np.sharedMemBytes = lds_bytes;
  np.kernelParams = kparams;
  return hipGraphAddKernelNode(node, graph, deps, n_deps, &np);
}

hipError_t launch_group(bool f16, int flavor, const GroupArgs &ga, uint32_t n_blocks, uint32_t lds_bytes, hipStream_t s) {
  GroupArgs args = ga;
  void *kparams[1] = {&args};
  return hipLaunchKernel(group_func(f16, flavor, ga.trace != nullptr), dim3(n_blocks), dim3(256), kparams, lds_bytes, s);
}

namespace {
void *chain_func(bool f16, bool light) {
  return f16 ? (light ? (void *)opara_k_chain_f16_light : (void *)opara_k_chain_f16_heavy)
             : (light ? (void *)opara_k_chain_f32_light : (void *)opara_k_chain_f32_heavy);
}
}  // namespace

bool chain_kernel_ok(int id, bool *light) { return group_kernel_ok(id, light); }

hipError_t chain_max_lds(uint32_t lds_bytes) {
  for (int f16 = 0; f16 < 2; ++f16)
    for (int light = 0; light < 2; ++light) {
      hipError_t err = hipFuncSetAttribute(chain_func(f16, light), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
      if (err != hipSuccess) return err;
    }
  return hipSuccess;
}

hipError_t add_chain_node(hipGraph_t graph, bool f16, bool light, const ChainArgs &a, uint32_t lds_bytes,
                          const hipGraphNode_t *deps, size_t n_deps, hipGraphNode_t *node) {
  ChainArgs args = a;
  void *kparams[1] = {&args};
  hipKernelNodeParams np = {};
  np.func = chain_func(f16, light);
  np.gridDim = dim3((uint32_t)a.total);
  np.blockDim = dim3(256);
  np.sharedMemBytes = lds_bytes;
  np.kernelParams = kparams;
  return hipGraphAddKernelNode(node, graph, deps, n_deps, &np);
}

hipError_t launch_chain(bool f16, bool light, const ChainArgs &a, uint32_t lds_bytes, hipStream_t s) {
  const dim3 grid((uint32_t)a.total), block(256);
  if (f16) {
    if (light) hipLaunchKernelGGL(opara_k_chain_f16_light, grid, block, lds_bytes, s, a);
    else hipLaunchKernelGGL(opara_k_chain_f16_heavy, grid, block, lds_bytes, s, a);
  } else {
    if (light) hipLaunchKernelGGL(opara_k_chain_f32_light, grid, block, lds_bytes, s, a);
    else hipLaunchKernelGGL(opara_k_chain_f32_heavy, grid, block, lds_bytes, s, a);
  }
  return hipGetLastError();
}

int persist_kernel_id(int id) {
  switch (id) {
    // One tile shape, one workgroup size: inside the persistent kernel every
    // latency-oriented contraction runs the four-wavefront fragment-loading body.
    case K_igemm_f16_direct8: case K_igemm_f16_quad4: case K_igemm_f16_quad8: return K_igemm_f16_direct4;
    case K_igemm_f32_direct8: case K_igemm_f32_quad4: case K_igemm_f32_quad8: return K_igemm_f32_direct4;
    case K_igemm_f16_quad64x4: case K_igemm_f32_quad64x4:
    case K_igemm_f16_direct4s: case K_igemm_f16_quad4s: case K_igemm_f32_direct4s: case K_igemm_f32_quad4s:
      return -1;                          // never in a persistent plan
    default: return (id >= 0 && id < K_COUNT) ? id : -1;
  }
}

bool kernel_is_f16(int id) {
  switch (id) {
#define X(name, A) case K_##name: return sizeof(#name) > 1 && __builtin_strstr(#name, "_f16") != nullptr;
    OPARA_KERNEL_LIST(X)
#undef X
    default: return false;
  }
}

hipError_t persist_max_workgroups(bool f16, uint32_t lds_bytes, uint32_t *n_workgroups) {
  int dev = 0, cus = 0, per_cu = 0;
  hipError_t err = hipGetDevice(&dev);
  if (err != hipSuccess) return err;
  err = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
  if (err != hipSuccess) return err;
  const void *func = f16 ? (const void *)opara_k_persist_f16 : (const void *)opara_k_persist_f32;
  err = hipFuncSetAttribute(func, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
  if (err != hipSuccess) return err;
  err = f16 ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, opara_k_persist_f16, 256, lds_bytes)
            : hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, opara_k_persist_f32, 256, lds_bytes);
  if (err != hipSuccess) return err;
  *n_workgroups = (uint32_t)(per_cu > 0 ? per_cu : 0) * (uint32_t)cus;
  return hipSuccess;
}

hipError_t add_persist_node(hipGraph_t graph, bool f16, const PersistArgs &a, uint32_t n_workgroups,
                            uint32_t lds_bytes, const hipGraphNode_t *deps, size_t n_deps, hipGraphNode_t *node) {
  PersistArgs args = a;
  void *kparams[1] = {&args};
  hipKernelNodeParams np = {};
  np.func = f16 ? (void *)opara_k_persist_f16 : (void *)opara_k_persist_f32;
  np.gridDim = dim3(n_workgroups);
  np.blockDim = dim3(256);
  np.sharedMemBytes = lds_bytes;
  np.kernelParams = kparams;
  return hipGraphAddKernelNode(node, graph, deps, n_deps, &np);
}

hipError_t launch_persist(bool f16, const PersistArgs &a, uint32_t n_workgroups, uint32_t lds_bytes, hipStream_t s) {
  if (f16) hipLaunchKernelGGL(opara_k_persist_f16, dim3(n_workgroups), dim3(256), lds_bytes, s, a);
  else hipLaunchKernelGGL(opara_k_persist_f32, dim3(n_workgroups), dim3(256), lds_bytes, s, a);
  return hipGetLastError();
}

hipError_t static_workspace(void **ptr, size_t *bytes) {
  constexpr int kMaxDevices = 64;
  static void *addr[kMaxDevices];          // per device, written once (the lookup is idempotent)
  int dev = 0;
  hipError_t err = hipGetDevice(&dev);
  if (err != hipSuccess) return err;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  void *p = __atomic_load_n(&addr[dev], __ATOMIC_ACQUIRE);
  if (!p) {
    err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (err != hipSuccess) return err;
    if (!p) return hipErrorInvalidSymbol;
    __atomic_store_n(&addr[dev], p, __ATOMIC_RELEASE);
  }
  *ptr = p;
  *bytes = kScratchBytes;
  return hipSuccess;
}

hipError_t set_op_trace(void *device_buffer) {
  g_host_op_trace = (unsigned long long *)device_buffer;
  return hipSuccess;
}

void *current_op_trace() { return g_host_op_trace; }

hipError_t verify_reset(hipStream_t s) {
  void *tok = nullptr, *viol = nullptr;
  hipError_t err = hipGetSymbolAddress(&tok, HIP_SYMBOL(g_verify_tok));
  if (err != hipSuccess) return err;
  err = hipGetSymbolAddress(&viol, HIP_SYMBOL(g_verify_viol));
  if (err != hipSuccess) return err;
  err = hipMemsetAsync(tok, 0, sizeof(int) * kVerifyMaxOps, s);
  if (err != hipSuccess) return err;
  return hipMemsetAsync(viol, 0, sizeof(int) * 4, s);
}

hipError_t verify_read(hipStream_t s, int *viol, int *op, int *pred) {
  void *p = nullptr;
  int v[4] = {0, 0, 0, 0};
  hipError_t err = hipGetSymbolAddress(&p, HIP_SYMBOL(g_verify_viol));
  if (err != hipSuccess) return err;
  err = hipMemcpyAsync(v, p, sizeof v, hipMemcpyDeviceToHost, s);
  if (err != hipSuccess) return err;
  err = hipStreamSynchronize(s);
  *viol = v[0];
  if (op) *op = v[1] - 1;
  if (pred) *pred = v[2];
  return err;
}

const void *kernel_symbol(int id) {
  switch (id) {
#define X(name, A) \
  case K_##name:   \
    return (const void *)opara_k_##name;
    OPARA_KERNEL_LIST(X)
#undef X
    default:
      return nullptr;
  }
}

}  // namespace opara
