// HIP kernels of the Flag Aggregator hot path for gfx950 (MI355X), and their launchers.
//
//   K1 fa_gram_kernel        norms + Gram matrix K = G^T G, one streaming pass over G
//                            (fp64 matrix core; the bf16 matrix-core pass is fa_gram_lp.hip)
//   K2 fa_gram_reduce_kernel fixed-order reduction of the per-workgroup partial results
//                            (optionally scaled: diag(u) K diag(u), a weighted Gram matrix)
//   K3 fa_irls_kernel        the p x p part for any p <= 64: normalisation, IRLS (weighted
//                            PCA by Jacobi), coefficients c with out = G c
//                            (p <= 16 has its own kernel, fa_irls16.hip)
//   K4 fa_combine_kernel     out = G c, second streaming pass over G
//   K5 fa_proj_kernel        projections G^T (G A) by streaming (re-streaming schedule)
//   K6 fa_restream_weights_kernel  IRLS weights from the streamed projections
//
// Paper: Sec. 2.1 (explained variance needs |g_i|^2 and Y^T g_i), Sec. 2.3 (D_ij^2),
// Eq. 5 (objective), Alg. 1 (IRLS step and d = (1/p) Y Y^T G 1).
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>
#include <type_traits>

#include "fa.h"
#include "fa_internal.h"

typedef double v4f64 __attribute__((ext_vector_type(4)));

// tuning of the p <= 16 fp32 Gram kernel: columns per load instruction and waves per CU
// (measured at p = 15, n = 11.2M: CPL 4 x 12 waves 105 us; 2 x 12 111 us; 1 x 8 119 us; wave
// counts that are not a multiple of the four SIMDs lose 10-20 us)
#ifndef FA_GRAM_CPL1
#define FA_GRAM_CPL1 4
#endif
#ifndef FA_GRAM_W1
#define FA_GRAM_W1 12
#endif
// 16 < p <= 32: sixteen waves per CU (measured at p = 32 bf16, n = 124M: 3.00 ms; 8 waves 3.06)
#ifndef FA_GRAM_W2
#define FA_GRAM_W2 16
#endif
#ifndef FA_GRAM_CPL2
#define FA_GRAM_CPL2 4
#endif
#ifndef FA_GRAM_W4
#define FA_GRAM_W4 8
#endif
// 48 < p <= 64 (measured at p = 64, n = 50M: 4 columns per load x 8 waves 4.4 ms; 8 columns per
// load, i.e. tiles of 32 rows, x 12 waves 4.7 ms, x 16 waves 8.5 ms - the accumulators of ten
// tile pairs do not fit 128 registers; the matrix pipe is 77 % busy at the default)
#ifndef FA_GRAM_CPL4
#define FA_GRAM_CPL4 4
#endif

// ------------------------------------------------------------------------------------------
// storage element types: 16 bytes per lane per load
struct ElemF32 {
  static constexpr int SIZE = 4;
  static constexpr int EPL = 4;  // elements per 16-byte lane load
};
struct ElemBF16 {
  static constexpr int SIZE = 2;
  static constexpr int EPL = 8;
};

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

// Streaming access to G and out: every byte is used once per pass, so the loads carry the
// non-temporal hint (measured on MI355X: 15 column streams read at 7.0 TB/s with it, 6.2 TB/s
// without) and the output is written through (one output stream beside the 15 input
// streams: 114 us with write-through stores, 119 us with default ones, n = 11.2M).
__device__ __forceinline__ uint4 load16_stream(const void* src) {
  const uint32_t* s = reinterpret_cast<const uint32_t*>(src);
  uint4 v;   // the four dword loads are merged into one global_load_dwordx4 nt
  v.x = __builtin_nontemporal_load(s);
  v.y = __builtin_nontemporal_load(s + 1);
  v.z = __builtin_nontemporal_load(s + 2);
  v.w = __builtin_nontemporal_load(s + 3);
  return v;
}

typedef uint32_t fa_u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void store16_through(float* dst, float4 r) {
  const fa_u32x4 v = {__float_as_uint(r.x), __float_as_uint(r.y), __float_as_uint(r.z),
                      __float_as_uint(r.w)};
  // the trailing s_nop covers the wait states a VALU write of the data registers needs
  // after a store wider than 64 bits (the compiler cannot see inside the asm)
  asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1\n\ts_nop 2" ::"v"(dst), "v"(v) : "memory");
}

// 16 bytes of column `base` starting at element row0, zero-filled past row n.
template <typename E>
__device__ __forceinline__ uint4 load16_guarded(const unsigned char* base, int64_t row0,
                                                int64_t n) {
  uint4 v = make_uint4(0u, 0u, 0u, 0u);
  if (row0 + E::EPL <= n) {
    v = load16_stream(base + row0 * E::SIZE);
  } else if (row0 < n) {
    uint32_t w[4] = {0u, 0u, 0u, 0u};
    if constexpr (E::SIZE == 4) {
      const uint32_t* src = reinterpret_cast<const uint32_t*>(base) + row0;
      for (int e = 0; e < 4; ++e)
        if (row0 + e < n) w[e] = src[e];
    } else {
      const uint16_t* src = reinterpret_cast<const uint16_t*>(base) + row0;
      for (int e = 0; e < 8; ++e)
        if (row0 + e < n) w[e >> 1] |= (uint32_t)src[e] << (16 * (e & 1));
    }
    v = make_uint4(w[0], w[1], w[2], w[3]);
  }
  return v;
}

// ------------------------------------------------------------------------------------------
// K1: Gram matrix by fp64 matrix-core accumulation.
//
// Each wavefront owns a private LDS tile and walks the row tiles w, w + W, w + 2W, ... (w its
// index among the W wavefronts of the launch: a fixed assignment, so results are
// reproducible).  Per tile: 16-byte coalesced global loads (next tile's loads are in flight while this
// tile is multiplied) -> LDS laid out [column][row] -> each lane reads the four rows of "its"
// column -> v_mfma_f64_16x16x4_f64, whose A and B operands are the same register for a
// diagonal 16x16 block of G^T G: lane (c, k) supplies G[row_k][c].
// Products of fp32 (or bf16) inputs are exact in fp64 and the accumulation is fp64, which the
// small differences 1 - v_i of the IRLS weights need.
//
// The operands of step t+1 are read from LDS and converted before the matrix instructions
// of step t are issued, so their LDS latency is hidden behind those.
// LDS columns p..16T-1 are zeroed once and never written, so no masking is needed.
//
// Launch shape: one workgroup of WAVES wavefronts (a multiple of the four SIMDs) per compute
// unit, each wavefront with its private LDS tile; the workgroup's LDS request is sized so
// that exactly one fits per CU.  The tile assignment is static (reproducible sums), so an uneven placement
// of workgroups would last for the whole kernel; this shape leaves the dispatcher no choice.
//
// T   = number of 16-column blocks (p <= 16 T)
// CPL = columns covered by one load instruction (1: a wave reads 1 KiB of one column;
//       4: 256 B of each of four columns, which keeps the LDS tile small for large p)
__device__ __forceinline__ void wave_lds_fence() {
  // orders this wavefront's LDS accesses for the compiler; the hardware executes one
  // wavefront's LDS instructions in order
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

template <typename E>
__device__ __forceinline__ void unpack4(const unsigned char* src, double* x) {
  if constexpr (E::SIZE == 4) {
    const float4 f = *reinterpret_cast<const float4*>(src);
    x[0] = (double)f.x; x[1] = (double)f.y; x[2] = (double)f.z; x[3] = (double)f.w;
  } else {
    const uint2 h = *reinterpret_cast<const uint2*>(src);
    x[0] = (double)bf16_bits_to_f32(h.x & 0xffffu); x[1] = (double)bf16_bits_to_f32(h.x >> 16);
    x[2] = (double)bf16_bits_to_f32(h.y & 0xffffu); x[3] = (double)bf16_bits_to_f32(h.y >> 16);
  }
}

// ROWS: G is stored row by row ("interleaved": element i of coordinate k at G + (k*ldg + i)
// * elem_size, ldg <= 16 T).  A tile of R rows is then one contiguous span of memory; it is
// read with the same 16-byte coalesced loads, and each lane scatters the four (eight)
// elements of its pieces to their [column][row] places in LDS.  Where the elements of a piece
// go is the same for every tile, so it is worked out once.
template <int T, int CPL, typename E, int WAVES, bool ROWS>
__global__ __launch_bounds__(64 * WAVES) void fa_gram_kernel(
                                                     const unsigned char* __restrict__ G,
                                                     int64_t ldg, int p, int64_t n,
                                                     int64_t ntiles,
                                                     double* __restrict__ partials,
                                                     const int* __restrict__ gate) {
  // as the stand-by of the bf16 matrix-core pass: nothing to do unless that one overflowed
  if (gate != nullptr && *gate == 0) return;
  constexpr int EPL = E::EPL;
  constexpr int LPC = 64 / CPL;            // lanes per column in one load instruction
  constexpr int R = LPC * EPL;             // rows per tile
  constexpr int NCG = T * 16 / CPL;        // load instructions per tile
  constexpr int CS = R * E::SIZE + 16;     // LDS bytes per column (+16: bank spread)
  constexpr int NTP = T * (T + 1) / 2;
  constexpr int NSTEP = R / 16;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_all[];
  const int wave = threadIdx.x >> 6;
  unsigned char* lds = lds_all + wave * (T * 16 * CS);
  const int64_t wid = (int64_t)blockIdx.x * WAVES + wave;   // global wave index
  const int64_t nwaves = (int64_t)gridDim.x * WAVES;

  const int lane = threadIdx.x & 63;
  const int lcol = lane / LPC;
  const int lrow = (lane % LPC) * EPL;
  const int c16 = lane & 15, kq = lane >> 4;

  v4f64 acc[NTP];
#pragma unroll
  for (int i = 0; i < NTP; ++i) acc[i] = v4f64{0.0, 0.0, 0.0, 0.0};

  // zero the whole tile once: columns >= p stay zero for the life of the kernel
  for (int off = lane * 16; off < T * 16 * CS; off += 64 * 16)
    *reinterpret_cast<uint4*>(lds + off) = make_uint4(0u, 0u, 0u, 0u);

  // this lane's source column for each load instruction (clamped: lanes of columns >= p
  // re-read column p-1 and their data is dropped before the LDS write)
  const unsigned char* colbase[NCG];
  bool colon[NCG];
#pragma unroll
  for (int cg = 0; cg < NCG; ++cg) {
    const int col = cg * CPL + lcol;
    colon[cg] = col < p;
    colbase[cg] = G + (int64_t)(colon[cg] ? col : p - 1) * ldg * E::SIZE;
  }

  // interleaved storage: (row in tile, column) of the first element of each of this lane's
  // pieces; the span of a tile is R * ldg elements (<= NCG * 64 pieces)
  int prow[NCG], pcol[NCG];
  bool pon[NCG];
  const int ldr = (int)ldg;
#pragma unroll
  for (int cg = 0; cg < NCG; ++cg) {
    const int e0 = (cg * 64 + lane) * EPL;
    pon[cg] = ROWS && e0 < R * ldr;
    prow[cg] = ROWS ? e0 / ldr : 0;
    pcol[cg] = ROWS ? e0 - prow[cg] * ldr : 0;
  }

  uint4 regs[NCG];
  auto load_tile = [&](int64_t tl) {
    if constexpr (ROWS) {
      const unsigned char* base = G + tl * R * ldr * E::SIZE;
      const int64_t rows_here = n - tl * R < R ? n - tl * R : R;
      const int lim = (int)rows_here * ldr;          // elements of this tile that exist
#pragma unroll
      for (int cg = 0; cg < NCG; ++cg) {
        regs[cg] = make_uint4(0u, 0u, 0u, 0u);
        const int e0 = (cg * 64 + lane) * EPL;
        if (pon[cg]) {
          if (e0 + EPL <= lim) regs[cg] = load16_stream(base + (int64_t)e0 * E::SIZE);
          else if (e0 < lim) regs[cg] = load16_guarded<E>(base, e0, lim);
        }
      }
      return;
    }
    const int64_t row0 = tl * R + lrow;
    if ((tl + 1) * R <= n) {               // uniform: a full tile needs no row guards
#pragma unroll
      for (int cg = 0; cg < NCG; ++cg)
        regs[cg] = load16_stream(colbase[cg] + row0 * E::SIZE);
    } else {
#pragma unroll
      for (int cg = 0; cg < NCG; ++cg) regs[cg] = load16_guarded<E>(colbase[cg], row0, n);
    }
  };
  auto store_tile_lds = [&]() {
    if constexpr (ROWS) {
#pragma unroll
      for (int cg = 0; cg < NCG; ++cg) {
        if (!pon[cg]) continue;
        int r = prow[cg], c = pcol[cg];
        const uint32_t wds[4] = {regs[cg].x, regs[cg].y, regs[cg].z, regs[cg].w};
#pragma unroll
        for (int j = 0; j < EPL; ++j) {
          if (c < p) {
            if constexpr (E::SIZE == 4)
              *reinterpret_cast<uint32_t*>(lds + c * CS + r * 4) = wds[j];
            else
              *reinterpret_cast<uint16_t*>(lds + c * CS + r * 2) =
                  (uint16_t)(wds[j >> 1] >> (16 * (j & 1)));
          }
          if (++c == ldr) { c = 0; ++r; }
        }
      }
      return;
    }
#pragma unroll
    for (int cg = 0; cg < NCG; ++cg)
      if (colon[cg])
        *reinterpret_cast<uint4*>(lds + (cg * CPL + lcol) * CS + lrow * E::SIZE) = regs[cg];
  };
  auto operand = [&](const unsigned char* src, int tt, double* x) { unpack4<E>(src, x); };

  wave_lds_fence();
  int64_t tile = wid;
  if (tile < ntiles) load_tile(tile);
  for (; tile < ntiles; tile += nwaves) {
    wave_lds_fence();  // the previous tile's LDS reads precede these writes
    store_tile_lds();
    wave_lds_fence();
    const int64_t next = tile + nwaves;
    if (next < ntiles) load_tile(next);

    const unsigned char* src = lds + c16 * CS + 4 * kq * E::SIZE;
    double xc[T][4], xn[T][4];
#pragma unroll
    for (int tt = 0; tt < T; ++tt) operand(src + tt * 16 * CS, tt, xc[tt]);
#pragma unroll 4
    for (int t = 0; t < NSTEP; ++t) {
      // operands of the next step (the last step re-reads step 0; harmless)
      const int tn = (t + 1 < NSTEP) ? t + 1 : 0;
#pragma unroll
      for (int tt = 0; tt < T; ++tt) operand(src + tt * 16 * CS + 16 * tn * E::SIZE, tt, xn[tt]);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        int tp = 0;
#pragma unroll
        for (int a = 0; a < T; ++a)
#pragma unroll
          for (int b = a; b < T; ++b) {
            acc[tp] = __builtin_amdgcn_mfma_f64_16x16x4f64(xc[a][j], xc[b][j], acc[tp], 0, 0, 0);
            ++tp;
          }
      }
#pragma unroll
      for (int tt = 0; tt < T; ++tt)
#pragma unroll
        for (int j = 0; j < 4; ++j) xc[tt][j] = xn[tt][j];
    }
  }

  // accumulator register r of lane l is entry (row 4*r + l/16, column l%16) of the block.
  // The workgroup's wavefronts add up in wave order through LDS (the tiles are dead now),
  // one partial Gram per workgroup leaves the kernel.
  __syncthreads();
  double* red = reinterpret_cast<double*>(lds_all);   // WAVES * 256 doubles <= 32 KiB
  double* dst = partials + (int64_t)blockIdx.x * NTP * 256;
#pragma unroll
  for (int tp = 0; tp < NTP; ++tp) {
#pragma unroll
    for (int r = 0; r < 4; ++r) red[wave * 256 + r * 64 + lane] = acc[tp][r];
    __syncthreads();
    for (int e = threadIdx.x; e < 256; e += 64 * WAVES) {
      double tot = 0.0;
#pragma unroll
      for (int w = 0; w < WAVES; ++w) tot += red[w * 256 + e];
      dst[tp * 256 + e] = tot;
    }
    __syncthreads();
  }
}

// ------------------------------------------------------------------------------------------
// K5: the projections of the gradients on the current basis, measured by streaming G:
//   P = G^T (G A)   (p x m; row i is Y^T g_i for Y = G A, the quantity in the explained
//   variance |Y^T g_i|^2 / |g_i|^2 of Sec. 2.1).
// Same data path as the Gram kernel (coalesced loads -> LDS [column][row] -> matrix core), two
// contractions per 16 rows: first Y_blk = G_blk A (16 rows x m) with the rows of the block as
// the M index of the product, permuted so that the accumulator registers of Y_blk are at once
// the B operand of the second product P += G_blk^T Y_blk (contraction over the 16 rows).
// Y is never written anywhere.  A sits in LDS, zero-padded to 16 T x 16 TM.
template <typename E>
__device__ __forceinline__ double lds_elem(const unsigned char* src) {
  if constexpr (E::SIZE == 4) return (double)*reinterpret_cast<const float*>(src);
  else return (double)bf16_bits_to_f32(*reinterpret_cast<const uint16_t*>(src));
}

template <int T, int TM, int CPL, typename E, int WAVES>
__global__ __launch_bounds__(64 * WAVES) void fa_proj_kernel(
                                                     const unsigned char* __restrict__ G,
                                                     int64_t ldg, int p, int m, int64_t n,
                                                     int64_t ntiles,
                                                     const double* __restrict__ Acoef,
                                                     double* __restrict__ partials) {
  constexpr int EPL = E::EPL;
  constexpr int LPC = 64 / CPL;
  constexpr int R = LPC * EPL;
  constexpr int NCG = T * 16 / CPL;
  constexpr int CS = R * E::SIZE + 16;
  constexpr int NSTEP = R / 16;
  constexpr int NTILE = T * TM;
  constexpr int ALD = TM * 16;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_all[];
  double* Alds = reinterpret_cast<double*>(lds_all);
  unsigned char* tiles = lds_all + (size_t)T * 16 * ALD * sizeof(double);
  const int wave = threadIdx.x >> 6;
  unsigned char* lds = tiles + wave * (T * 16 * CS);
  const int64_t wid = (int64_t)blockIdx.x * WAVES + wave;
  const int64_t nwaves = (int64_t)gridDim.x * WAVES;
  const int lane = threadIdx.x & 63;
  const int lcol = lane / LPC;
  const int lrow = (lane % LPC) * EPL;
  const int c16 = lane & 15, kq = lane >> 4;

  for (int idx = threadIdx.x; idx < T * 16 * ALD; idx += 64 * WAVES) {
    const int i = idx / ALD, a = idx - i * ALD;
    Alds[idx] = (i < p && a < m) ? Acoef[i * m + a] : 0.0;
  }
  for (int off = lane * 16; off < T * 16 * CS; off += 64 * 16)
    *reinterpret_cast<uint4*>(lds + off) = make_uint4(0u, 0u, 0u, 0u);
  __syncthreads();

  v4f64 acc[NTILE];
#pragma unroll
  for (int i = 0; i < NTILE; ++i) acc[i] = v4f64{0.0, 0.0, 0.0, 0.0};

  const unsigned char* colbase[NCG];
  bool colon[NCG];
#pragma unroll
  for (int cg = 0; cg < NCG; ++cg) {
    const int col = cg * CPL + lcol;
    colon[cg] = col < p;
    colbase[cg] = G + (int64_t)(colon[cg] ? col : p - 1) * ldg * E::SIZE;
  }
  uint4 regs[NCG];
  auto load_tile = [&](int64_t tl) {
    const int64_t row0 = tl * R + lrow;
    if ((tl + 1) * R <= n) {
#pragma unroll
      for (int cg = 0; cg < NCG; ++cg) regs[cg] = load16_stream(colbase[cg] + row0 * E::SIZE);
    } else {
#pragma unroll
      for (int cg = 0; cg < NCG; ++cg) regs[cg] = load16_guarded<E>(colbase[cg], row0, n);
    }
  };

  // first product: lane (i = c16, k = kq) supplies G[row(i)][4 s + k] with
  // row(i) = 4 (i mod 4) + i / 4, so that register r of lane (kq, a) of the result holds
  // Y[4 kq + r][a]: exactly what the second product wants from that lane for its step j = r
  const int rowA = 4 * (c16 & 3) + (c16 >> 2);
  int64_t tile = wid;
  if (tile < ntiles) load_tile(tile);
  for (; tile < ntiles; tile += nwaves) {
    wave_lds_fence();
#pragma unroll
    for (int cg = 0; cg < NCG; ++cg)
      if (colon[cg])
        *reinterpret_cast<uint4*>(lds + (cg * CPL + lcol) * CS + lrow * E::SIZE) = regs[cg];
    wave_lds_fence();
    const int64_t next = tile + nwaves;
    if (next < ntiles) load_tile(next);

#pragma unroll 2
    for (int t = 0; t < NSTEP; ++t) {
      v4f64 y[TM];
#pragma unroll
      for (int ta = 0; ta < TM; ++ta) y[ta] = v4f64{0.0, 0.0, 0.0, 0.0};
#pragma unroll
      for (int tt = 0; tt < T; ++tt)
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          const int col = 16 * tt + 4 * s + kq;
          const double a1 = lds_elem<E>(lds + col * CS + (16 * t + rowA) * E::SIZE);
#pragma unroll
          for (int ta = 0; ta < TM; ++ta)
            y[ta] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, Alds[col * ALD + 16 * ta + c16],
                                                         y[ta], 0, 0, 0);
        }
      double xc[T][4];
#pragma unroll
      for (int tt = 0; tt < T; ++tt)
        unpack4<E>(lds + (16 * tt + c16) * CS + (16 * t + 4 * kq) * E::SIZE, xc[tt]);
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int tt = 0; tt < T; ++tt)
#pragma unroll
          for (int ta = 0; ta < TM; ++ta)
            acc[tt * TM + ta] = __builtin_amdgcn_mfma_f64_16x16x4f64(xc[tt][j], y[ta][j],
                                                                     acc[tt * TM + ta], 0, 0, 0);
    }
  }

  // one partial result per workgroup, summed over its wavefronts in wave order
  __syncthreads();
  double* red = reinterpret_cast<double*>(tiles);
  double* dst = partials + (int64_t)blockIdx.x * NTILE * 256;
#pragma unroll
  for (int tp = 0; tp < NTILE; ++tp) {
#pragma unroll
    for (int r = 0; r < 4; ++r) red[wave * 256 + r * 64 + lane] = acc[tp][r];
    __syncthreads();
    for (int e = threadIdx.x; e < 256; e += 64 * WAVES) {
      double tot = 0.0;
#pragma unroll
      for (int w = 0; w < WAVES; ++w) tot += red[w * 256 + e];
      dst[tp * 256 + e] = tot;
    }
    __syncthreads();
  }
}

// K4 for interleaved storage (G row by row, row pitch ldr elements): a workgroup copies the
// contiguous span of its 256 rows to LDS as it is, 16 bytes per lane per load and per LDS
// write (no decoding of rows and columns on the way); then thread r adds up row r (fp64) and
// the workgroup writes 256 consecutive outputs.  Rows of 16 k elements would put a wavefront's
// reads of element i on a few banks only, so the copy leaves 16 bytes free after every 256:
// byte b of the span sits at b + 16 (b / 256).
#define FA_ROWS_MULTI 8   // columns of a materialised basis per pass over row-major G
__host__ __device__ inline size_t fa_rows_lds_bytes(int ldr, int es) {
  const size_t span = (size_t)256 * ldr * es;
  return span + (span >> 8) * 16 + 16;
}
// MB > 1: up to MB combinations from one pass over G (column a of the output, at out + a*ldo,
// uses the coefficients c[i*cstride + a]): the materialised basis Y = G A of row-major storage.
template <typename E, int MB>
__global__ __launch_bounds__(256) void fa_combine_rows_kernel(const unsigned char* __restrict__ G,
                                                              int ldr, int p, int64_t n,
                                                              const double* __restrict__ c,
                                                              int cstride, int ncols,
                                                              float* __restrict__ out, int64_t ldo) {
  constexpr int EPL = E::EPL;
  constexpr int RB = 256;                  // rows per workgroup pass
  extern __shared__ __attribute__((aligned(16))) unsigned char tile[];
  __shared__ double cs[MB][FA_P_MAX];
  for (int idx = threadIdx.x; idx < MB * FA_P_MAX; idx += 256) {
    const int a = idx / FA_P_MAX, i = idx % FA_P_MAX;
    cs[a][i] = (i < p && a < ncols) ? c[(int64_t)i * cstride + a] : 0.0;
  }
  const int64_t nblk = (n + RB - 1) / RB;
  for (int64_t blk = blockIdx.x; blk < nblk; blk += gridDim.x) {
    const int64_t row_base = blk * RB;
    const int rows_here = (int)(n - row_base < RB ? n - row_base : RB);
    const int lim = rows_here * ldr;                        // elements of this span
    const int npieces = (lim + EPL - 1) / EPL;              // 16-byte pieces, the last one ragged
    const unsigned char* base = G + row_base * ldr * E::SIZE;
    __syncthreads();                                        // the previous pass has been read
    // (fetching the next span into registers before the rows are added up was measured:
    // 126 instead of 134 us at a pitch of 16 fp32 values, 140 instead of 130 at 15)
    constexpr int PCH = 4;                                  // pieces in flight per thread
    for (int pb = (int)threadIdx.x; pb < npieces; pb += 256 * PCH) {
      uint4 v[PCH];
#pragma unroll
      for (int q = 0; q < PCH; ++q) {
        const int pc = pb + q * 256;
        v[q] = make_uint4(0u, 0u, 0u, 0u);
        if ((pc + 1) * EPL <= lim) v[q] = load16_stream(base + (int64_t)pc * 16);
        else if (pc < npieces) v[q] = load16_guarded<E>(base, (int64_t)pc * EPL, lim);
      }
#pragma unroll
      for (int q = 0; q < PCH; ++q) {
        const int pc = pb + q * 256;
        if (pc < npieces) *reinterpret_cast<uint4*>(tile + pc * 16 + (pc >> 4) * 16) = v[q];
      }
    }
    __syncthreads();
    const int r = (int)threadIdx.x;
    if (r < rows_here) {
      const int b0 = r * ldr * E::SIZE;                     // first byte of row r in the span
      auto elem = [&](int i) -> double {
        const int b = b0 + i * E::SIZE;
        const unsigned char* at = tile + b + (b >> 8) * 16;
        if constexpr (E::SIZE == 4) return (double)*reinterpret_cast<const float*>(at);
        else return (double)bf16_bits_to_f32(*reinterpret_cast<const uint16_t*>(at));
      };
      if constexpr (MB == 1) {
        double a0 = 0.0, a1 = 0.0;
        int i = 0;
        for (; i + 1 < p; i += 2) {
          a0 = fma(cs[0][i], elem(i), a0);
          a1 = fma(cs[0][i + 1], elem(i + 1), a1);
        }
        if (i < p) a0 = fma(cs[0][i], elem(i), a0);
        out[row_base + r] = (float)(a0 + a1);
      } else {
        double acc[MB];
#pragma unroll
        for (int a = 0; a < MB; ++a) acc[a] = 0.0;
        for (int i = 0; i < p; ++i) {
          const double t = elem(i);
#pragma unroll
          for (int a = 0; a < MB; ++a) acc[a] = fma(cs[a][i], t, acc[a]);
        }
#pragma unroll
        for (int a = 0; a < MB; ++a)
          if (a < ncols) out[(int64_t)a * ldo + row_base + r] = (float)acc[a];
      }
    }
  }
}

// The p x p solver text (any p): parallel-for phases over one workgroup.  Included here
// because the kernel below shares its term / weight functions.
#define FA_FN __device__
#define FA_TID ((int)threadIdx.x)
#define FA_NT ((int)blockDim.x)
#define FA_FOR(i, n) for (int i = FA_TID; i < (n); i += FA_NT)
#define FA_SYNC() __syncthreads()
#include "fa_irls_core.inc"

// K6: IRLS weights from the streamed projections (the re-streaming schedule's counterpart of
// the residual step inside the p x p kernel): explained variances v_i = |P_i|^2 / |g_i|^2,
// residuals 1 - v_i and 1 - |P_i - P_j|^2 / D_ij^2 (Eq. 5), the objective, the weights
// max(residual, delta)^(-1/2), and the column scales sqrt(w_i) / |g_i| of the next weighted
// Gram pass.  One workgroup.
__global__ __launch_bounds__(256) void fa_restream_weights_kernel(const fa_info* __restrict__ info,
                                                                  const double* __restrict__ P,
                                                                  int p, int m, double coef,
                                                                  double delta, double pair_tol,
                                                                  double expo,
                                                                  fa_resume* __restrict__ rs) {
  __shared__ double red[256];
  const int tid = threadIdx.x;
  const double* K = info->K;
  double part = 0.0;
  for (int i = tid; i < p; i += 256) {
    const double si = K[i * p + i];
    double pr = 0.0;
    for (int a = 0; a < m; ++a) pr = fma(P[i * m + a], P[i * m + a], pr);
    const double v = si > 0.0 ? pr / si : 0.0;
    const double rho = v < 1.0 ? 1.0 - v : 0.0;
    const double w = si > 0.0 ? fa_weight(rho, delta, expo) : 0.0;
    const double u = si > 0.0 ? sqrt(w / si) : 0.0;
    rs->w[i] = w;
    rs->v_streamed[i] = v;
    rs->u[i] = u;
    rs->uinv[i] = u > 0.0 ? 1.0 / u : 1.0;
    if (si > 0.0) part += fa_term(rho, expo);
  }
  for (int idx = tid; idx < p * p; idx += 256) {
    const int i = idx / p, j = idx - i * p;
    double cpv = 0.0;
    if (i != j && coef > 0.0) {
      const double si = K[i * p + i], sj = K[j * p + j];
      const double d2 = si + sj - 2.0 * K[idx];
      if (d2 > pair_tol * (si + sj)) {
        double pr = 0.0;
        for (int a = 0; a < m; ++a) {
          const double df = P[i * m + a] - P[j * m + a];
          pr = fma(df, df, pr);
        }
        const double q = pr / d2;
        const double rho = q < 1.0 ? 1.0 - q : 0.0;
        part += coef * fa_term(rho, expo);              // ordered pair (i, j)
        cpv = -2.0 * coef * fa_weight(rho, delta, expo) / d2;
      }
    }
    rs->cp[idx] = cpv;
  }
  red[tid] = part;
  __syncthreads();
  if (tid == 0) {
    double tot = 0.0;
    for (int t = 0; t < 256; ++t) tot += red[t];
    const int it = rs->it0 - 1;                         // the solve whose basis was measured
    if (it >= 0 && it < FA_ITERS_MAX) rs->obj_streamed[it] = tot;
    rs->scaled = 1;                                     // the next Gram pass uses rs->u
  }
}

// K2: K = sum over workgroups of their partial Grams, in a fixed order (sixteen interleaved
// strands, each summed in four interleaved sub-strands, then combined in a fixed tree), so the
// result does not depend on timing.  One 1024-thread block per 64 entries.
// TM = 0: the tiles are the upper-triangular tile pairs of a symmetric p x p matrix.
// TM > 0: the tiles are the T x TM blocks of a p x m matrix (row-major, leading dimension m).
// colscale (may be null; symmetric case only): entry (i, j) is multiplied by u_i u_j, which
// makes the result the Gram matrix G^T W G of the columns scaled by u = W^(1/2).
__global__ __launch_bounds__(1024) void fa_gram_reduce_kernel(const double* __restrict__ partials,
                                                              int nparts, int T, int p,
                                                              double* __restrict__ K, int TM,
                                                              int m,
                                                              const double* __restrict__ colscale,
                                                              const int* __restrict__ gate) {
  if (gate != nullptr && *gate == 0) return;   // stand-by of a pass that did not need it
  const int NTP = TM > 0 ? T * TM : T * (T + 1) / 2;
  const int ei = threadIdx.x & 63, g = threadIdx.x >> 6;   // entry, strand 0..15
  const int E = blockIdx.x * 64 + ei;                      // entry in [0, NTP*256)
  const int64_t stride = (int64_t)NTP * 256;
  double a[4] = {0.0, 0.0, 0.0, 0.0};
  for (int b0 = g; b0 < nparts; b0 += 64) {
    double v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int b = b0 + 16 * u;
      v[u] = b < nparts ? partials[(int64_t)b * stride + E] : 0.0;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) a[u] += v[u];
  }
  __shared__ double sh[1024];
  sh[threadIdx.x] = (a[0] + a[1]) + (a[2] + a[3]);
  __syncthreads();
  if (g == 0) {
    double t[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) t[k] = sh[k * 64 + ei];
#pragma unroll
    for (int w = 8; w >= 1; w >>= 1)
#pragma unroll
      for (int k = 0; k < w; ++k) t[k] += t[k + w];
    const double tot = t[0];
    const int tp = E >> 8, e = E & 255;
    const int r = e >> 6, l = e & 63;
    if (TM > 0) {
      const int gi = (tp / TM) * 16 + 4 * r + (l >> 4), ga = (tp % TM) * 16 + (l & 15);
      if (gi < p && ga < m) K[gi * m + ga] = tot;
      return;
    }
    int ta = 0, tb = 0;
    for (int aa = 0, k = 0; aa < T; ++aa)
      for (int bb = aa; bb < T; ++bb, ++k)
        if (k == tp) { ta = aa; tb = bb; }
    const int gi = ta * 16 + 4 * r + (l >> 4), gj = tb * 16 + (l & 15);
    if (gi < p && gj < p && gi <= gj) {
      const double v = colscale ? tot * (colscale[gi] * colscale[gj]) : tot;
      K[gi * p + gj] = v;
      K[gj * p + gi] = v;
    }
  }
}

// ------------------------------------------------------------------------------------------
// K4: out[k] = sum_i c[i] G[k][i]  (Alg. 1: d = (1/p) Y Y^T G 1 = G c).  Each thread owns 16
// bytes of every column (coalesced 16-byte loads: four rows of fp32, eight of bf16).
// fp32 storage: fp64 accumulation, one rounding to fp32 at the end; a thread's four outputs
// are one 16-byte store and a wavefront's store covers 1 KiB without gaps.
// bf16 storage: fp32 accumulation with c rounded to fp32 (per element at most (p + 1) 2^-24 of
// sum_i |c_i g_i|).  A thread's eight outputs are 32 bytes; stored as they are, each of its two
// stores would leave every other 16 bytes of a line to the other one, so the wavefront turns
// its 2 KiB of outputs round through LDS and stores two gap-free KiB instead.
#ifndef FA_COMBINE_NL
#define FA_COMBINE_NL 8
#endif
template <typename E>
__global__ __launch_bounds__(256) void fa_combine_kernel(const unsigned char* __restrict__ G,
                                                         int64_t ldg, int p, int64_t n,
                                                         const double* __restrict__ c,
                                                         int cstride, float* __restrict__ out) {
  constexpr int EPL = E::EPL;
  constexpr int NL = FA_COMBINE_NL;   // columns in flight per thread
  typedef typename std::conditional<E::SIZE == 4, double, float>::type acc_t;
  __shared__ acc_t cs[FA_P_MAX + NL];
  __shared__ __attribute__((aligned(16))) float turn[E::SIZE == 2 ? 256 * 8 : 4];
  if (threadIdx.x < FA_P_MAX + NL)
    cs[threadIdx.x] = (int)threadIdx.x < p ? (acc_t)c[(int64_t)threadIdx.x * cstride] : (acc_t)0;
  __syncthreads();
  const int64_t ngroups = (n + EPL - 1) / EPL;
  for (int64_t gbase = (int64_t)blockIdx.x * 256; gbase < ngroups;
       gbase += (int64_t)gridDim.x * 256) {
    const int64_t gidx = gbase + threadIdx.x;
    const int64_t row0 = gidx * EPL;
    const bool block_full = (gbase + 256) * EPL <= n;   // uniform: no row guards needed
    if (!block_full && gidx >= ngroups) continue;
    acc_t acc[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = (acc_t)0;
    const unsigned char* src = G + row0 * E::SIZE;
    for (int c0 = 0; c0 < p; c0 += NL) {
      uint4 v[NL];
      if (block_full) {
#pragma unroll
        for (int u = 0; u < NL; ++u) {
          // columns past p re-read column p-1; their coefficient is zero
          const int col = c0 + u < p ? c0 + u : p - 1;
          v[u] = load16_stream(src + (int64_t)col * ldg * E::SIZE);
        }
      } else {
#pragma unroll
        for (int u = 0; u < NL; ++u) {
          const int col = c0 + u < p ? c0 + u : p - 1;
          v[u] = load16_guarded<E>(G + (int64_t)col * ldg * E::SIZE, row0, n);
        }
      }
#pragma unroll
      for (int u = 0; u < NL; ++u) {
        const acc_t cc = cs[c0 + u];
        if constexpr (E::SIZE == 4) {
          acc[0] += cc * (double)__uint_as_float(v[u].x);
          acc[1] += cc * (double)__uint_as_float(v[u].y);
          acc[2] += cc * (double)__uint_as_float(v[u].z);
          acc[3] += cc * (double)__uint_as_float(v[u].w);
        } else {
          acc[0] = fmaf(cc, __uint_as_float(v[u].x << 16), acc[0]);
          acc[1] = fmaf(cc, __uint_as_float(v[u].x & 0xffff0000u), acc[1]);
          acc[2] = fmaf(cc, __uint_as_float(v[u].y << 16), acc[2]);
          acc[3] = fmaf(cc, __uint_as_float(v[u].y & 0xffff0000u), acc[3]);
          acc[4] = fmaf(cc, __uint_as_float(v[u].z << 16), acc[4]);
          acc[5] = fmaf(cc, __uint_as_float(v[u].z & 0xffff0000u), acc[5]);
          acc[6] = fmaf(cc, __uint_as_float(v[u].w << 16), acc[6]);
          acc[7] = fmaf(cc, __uint_as_float(v[u].w & 0xffff0000u), acc[7]);
        }
      }
    }
    float* dst = out + row0;
    if constexpr (E::SIZE == 4) {
      if (row0 + 4 <= n) {
        store16_through(dst, make_float4((float)acc[0], (float)acc[1], (float)acc[2],
                                         (float)acc[3]));
      } else {
        for (int e = 0; e < 4; ++e)
          if (row0 + e < n) dst[e] = (float)acc[e];
      }
    } else {
      if (block_full) {
        // the wavefront's 512 outputs, in row order, through its own 2 KiB of LDS
        const int lane = threadIdx.x & 63;
        float* mine = turn + (threadIdx.x & ~63) * 8;
        wave_lds_fence();        // the previous pass of this wavefront has read its part
        *reinterpret_cast<float4*>(mine + lane * 8) = make_float4(acc[0], acc[1], acc[2], acc[3]);
        *reinterpret_cast<float4*>(mine + lane * 8 + 4) =
            make_float4(acc[4], acc[5], acc[6], acc[7]);
        wave_lds_fence();
        const float4 lo = *reinterpret_cast<const float4*>(mine + lane * 4);
        const float4 hi = *reinterpret_cast<const float4*>(mine + 256 + lane * 4);
        float* wdst = out + (gbase + (threadIdx.x & ~63)) * 8;    // the wavefront's first row
        store16_through(wdst + lane * 4, lo);
        store16_through(wdst + 256 + lane * 4, hi);
      } else {
        for (int e = 0; e < 8; ++e)
          if (row0 + e < n) dst[e] = acc[e];
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// One row of the Gram matrix: k_u = g_i . g_{cols[u]} for up to FA_ROW_JB resident gradients,
// for a parameter server that extends K as the gradients arrive (Alg. 1: the server receives
// the p workers' gradients) instead of waiting for all of them.  Each thread owns 16 bytes of
// gradient i and of every listed gradient per pass; products of the stored values are exact
// in fp64 and are added in fp64.  Static chunk -> workgroup map, fixed-order sums inside the
// workgroup: one partial row per workgroup, bitwise reproducible.
struct fa_row_cols { int idx[FA_ROW_JB]; };

template <typename E>
__global__ __launch_bounds__(256) void fa_gram_row_kernel(const unsigned char* __restrict__ G,
                                                          int64_t ldg, int64_t n, int i,
                                                          fa_row_cols cols, int nj,
                                                          double* __restrict__ partials) {
  constexpr int EPL = E::EPL;
  __shared__ double red[4][FA_ROW_JB];
  double acc[FA_ROW_JB];
#pragma unroll
  for (int u = 0; u < FA_ROW_JB; ++u) acc[u] = 0.0;
  const unsigned char* gi = G + (int64_t)i * ldg * E::SIZE;
  const int64_t ngroups = (n + EPL - 1) / EPL;
  for (int64_t gbase = (int64_t)blockIdx.x * 256; gbase < ngroups;
       gbase += (int64_t)gridDim.x * 256) {
    const int64_t row0 = (gbase + threadIdx.x) * EPL;
    const bool block_full = (gbase + 256) * EPL <= n;   // uniform
    uint4 xi, xj[FA_ROW_JB];
    if (block_full) {
      xi = load16_stream(gi + row0 * E::SIZE);
#pragma unroll
      for (int u = 0; u < FA_ROW_JB; ++u)   // entries past nj repeat the last listed gradient
        xj[u] = load16_stream(G + ((int64_t)cols.idx[u] * ldg + row0) * E::SIZE);
    } else {
      xi = load16_guarded<E>(gi, row0, n);
#pragma unroll
      for (int u = 0; u < FA_ROW_JB; ++u)
        xj[u] = load16_guarded<E>(G + (int64_t)cols.idx[u] * ldg * E::SIZE, row0, n);
    }
    double a[EPL];
    {
      const uint32_t w[4] = {xi.x, xi.y, xi.z, xi.w};
#pragma unroll
      for (int e = 0; e < EPL; ++e) {
        if constexpr (E::SIZE == 4) a[e] = (double)__uint_as_float(w[e]);
        else a[e] = (double)bf16_bits_to_f32((w[e >> 1] >> (16 * (e & 1))) & 0xffffu);
      }
    }
#pragma unroll
    for (int u = 0; u < FA_ROW_JB; ++u) {
      const uint32_t w[4] = {xj[u].x, xj[u].y, xj[u].z, xj[u].w};
#pragma unroll
      for (int e = 0; e < EPL; ++e) {
        double b;
        if constexpr (E::SIZE == 4) b = (double)__uint_as_float(w[e]);
        else b = (double)bf16_bits_to_f32((w[e >> 1] >> (16 * (e & 1))) & 0xffffu);
        acc[u] = fma(a[e], b, acc[u]);
      }
    }
  }
  // fixed butterfly inside each wavefront, wavefronts in order
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int u = 0; u < FA_ROW_JB; ++u) {
    double x = acc[u];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off, 64);
    if (lane == 0) red[wave][u] = x;
  }
  __syncthreads();
  if ((int)threadIdx.x < FA_ROW_JB)
    partials[(int64_t)blockIdx.x * FA_ROW_JB + threadIdx.x] =
        (red[0][threadIdx.x] + red[1][threadIdx.x]) + (red[2][threadIdx.x] + red[3][threadIdx.x]);
}

// Fixed-order sum of the partial rows (four interleaved strands per entry, then a fixed
// tree), added to row and column i of K (row-major p x p; zero when the round opens).
__global__ __launch_bounds__(64 * FA_ROW_JB) void fa_gram_row_reduce_kernel(
    const double* __restrict__ partials, int nparts, fa_row_cols cols, int nj, int i, int p,
    double* __restrict__ K) {
  __shared__ double sh[FA_ROW_JB][64];
  const int u = threadIdx.x >> 6, s = threadIdx.x & 63;
  double a = 0.0;
  for (int b = s; b < nparts; b += 64) a += partials[(int64_t)b * FA_ROW_JB + u];
  sh[u][s] = a;
  __syncthreads();
  if (s == 0 && u < nj) {
    double t[64];
#pragma unroll
    for (int k = 0; k < 64; ++k) t[k] = sh[u][k];
#pragma unroll
    for (int w = 32; w >= 1; w >>= 1)
#pragma unroll
      for (int k = 0; k < w; ++k) t[k] += t[k + w];
    const int j = cols.idx[u];
    const double v = K[i * p + j] + t[0];     // K_ij and K_ji see the same addends in the same order
    K[i * p + j] = v;
    K[j * p + i] = v;
  }
}

__global__ __launch_bounds__(256) void fa_zero_kernel(double* __restrict__ dst, int count) {
  for (int k = blockIdx.x * 256 + threadIdx.x; k < count; k += gridDim.x * 256) dst[k] = 0.0;
}

hipError_t fa_launch_zero(double* dst, int count, hipStream_t st) {
  hipLaunchKernelGGL(fa_zero_kernel, dim3((count + 255) / 256), dim3(256), 0, st, dst, count);
  return hipGetLastError();
}

hipError_t fa_launch_gram_row(const void* G, int64_t ldg, int p, int64_t n, int dtype, int i,
                              uint64_t resident, double* partials, int max_parts, double* Kd,
                              hipStream_t st) {
  const int epl = dtype == FA_F32 ? 4 : 8;
  const int64_t ngroups = (n + epl - 1) / epl;
  int64_t blocks = (ngroups + 255) / 256;
  if (blocks > max_parts) blocks = max_parts;
  // gradient i against itself and against every resident one, FA_ROW_JB of them per pass
  int list[FA_P_MAX], nl = 0;
  for (int j = 0; j < p; ++j)
    if (j == i || ((resident >> j) & 1u)) list[nl++] = j;
  for (int a0 = 0; a0 < nl; a0 += FA_ROW_JB) {
    fa_row_cols cols;
    const int nj = nl - a0 < FA_ROW_JB ? nl - a0 : FA_ROW_JB;
    for (int u = 0; u < FA_ROW_JB; ++u) cols.idx[u] = list[a0 + (u < nj ? u : nj - 1)];
    if (dtype == FA_F32)
      hipLaunchKernelGGL((fa_gram_row_kernel<ElemF32>), dim3((unsigned)blocks), dim3(256), 0, st,
                         (const unsigned char*)G, ldg, n, i, cols, nj, partials);
    else
      hipLaunchKernelGGL((fa_gram_row_kernel<ElemBF16>), dim3((unsigned)blocks), dim3(256), 0, st,
                         (const unsigned char*)G, ldg, n, i, cols, nj, partials);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(fa_gram_row_reduce_kernel, dim3(1), dim3(64 * FA_ROW_JB), 0, st,
                       (const double*)partials, (int)blocks, cols, nj, i, p, Kd);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

// ------------------------------------------------------------------------------------------
// Y = G A for MB columns of A at once (the basis of Sec. 2.1 materialised: column a of Y is
// sum_i A[i][a] g_i): the aggregate pass with MB coefficient vectors, so G is read once per MB
// columns of Y instead of once per column.  A is row-major p x lda in device memory; column a
// of Y at Y + a*ldy.  Same thread-to-data map and loads as fa_combine_kernel.
template <typename E, int MB>
__global__ __launch_bounds__(256) void fa_combine_multi_kernel(
    const unsigned char* __restrict__ G, int64_t ldg, int p, int64_t n,
    const double* __restrict__ A, int lda, int ncols, float* __restrict__ Y, int64_t ldy) {
  constexpr int EPL = E::EPL;
  constexpr int NL = 4;                     // columns of G in flight per thread
  // fp32 storage: fp64 sums, one rounding per output; bf16 storage: fp32 sums with the
  // coefficients rounded to fp32, as in the aggregate pass of that storage
  typedef typename std::conditional<E::SIZE == 4, double, float>::type acc_t;
  __shared__ acc_t cs[(FA_P_MAX + NL) * MB];
  for (int t = threadIdx.x; t < (FA_P_MAX + NL) * MB; t += 256) {
    const int i = t / MB, a = t - i * MB;
    cs[t] = (i < p && a < ncols) ? (acc_t)A[(int64_t)i * lda + a] : (acc_t)0;
  }
  __syncthreads();
  const int64_t ngroups = (n + EPL - 1) / EPL;
  for (int64_t gbase = (int64_t)blockIdx.x * 256; gbase < ngroups;
       gbase += (int64_t)gridDim.x * 256) {
    const int64_t gidx = gbase + threadIdx.x;
    const int64_t row0 = gidx * EPL;
    const bool block_full = (gbase + 256) * EPL <= n;   // uniform: no row guards needed
    if (!block_full && gidx >= ngroups) continue;
    acc_t acc[MB][EPL];
#pragma unroll
    for (int a = 0; a < MB; ++a)
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[a][e] = (acc_t)0;
    const unsigned char* src = G + row0 * E::SIZE;
    for (int c0 = 0; c0 < p; c0 += NL) {
      uint4 v[NL];
#pragma unroll
      for (int u = 0; u < NL; ++u) {
        const int col = c0 + u < p ? c0 + u : p - 1;    // past p: coefficient zero
        if (block_full) v[u] = load16_stream(src + (int64_t)col * ldg * E::SIZE);
        else v[u] = load16_guarded<E>(G + (int64_t)col * ldg * E::SIZE, row0, n);
      }
#pragma unroll
      for (int u = 0; u < NL; ++u) {
        acc_t x[EPL];
        if constexpr (E::SIZE == 4) {
          x[0] = (double)__uint_as_float(v[u].x); x[1] = (double)__uint_as_float(v[u].y);
          x[2] = (double)__uint_as_float(v[u].z); x[3] = (double)__uint_as_float(v[u].w);
        } else {
          x[0] = __uint_as_float(v[u].x << 16); x[1] = __uint_as_float(v[u].x & 0xffff0000u);
          x[2] = __uint_as_float(v[u].y << 16); x[3] = __uint_as_float(v[u].y & 0xffff0000u);
          x[4] = __uint_as_float(v[u].z << 16); x[5] = __uint_as_float(v[u].z & 0xffff0000u);
          x[6] = __uint_as_float(v[u].w << 16); x[7] = __uint_as_float(v[u].w & 0xffff0000u);
        }
#pragma unroll
        for (int a = 0; a < MB; ++a) {
          const acc_t cc = cs[(c0 + u) * MB + a];
#pragma unroll
          for (int e = 0; e < EPL; ++e) {
            if constexpr (E::SIZE == 4) acc[a][e] = fma(cc, x[e], acc[a][e]);
            else acc[a][e] = fmaf(cc, x[e], acc[a][e]);
          }
        }
      }
    }
#pragma unroll
    for (int a = 0; a < MB; ++a) {
      if (a >= ncols) break;
      float* dst = Y + (int64_t)a * ldy + row0;
      if (row0 + EPL <= n) {
#pragma unroll
        for (int e = 0; e < EPL; e += 4)
          store16_through(dst + e, make_float4((float)acc[a][e], (float)acc[a][e + 1],
                                               (float)acc[a][e + 2], (float)acc[a][e + 3]));
      } else {
        for (int e = 0; e < EPL; ++e)
          if (row0 + e < n) dst[e] = (float)acc[a][e];
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// Multi-Krum from the Gram matrix (the distance-based aggregator the paper compares with,
// Sec. 3 "Baselines", Sec. 2.3; rule of Blanchard et al., 2017): D_ij^2 = K_ii + K_jj - 2 K_ij,
// worker i is scored by the sum of its k = p - f - 2 smallest distances to the others (added
// in ascending order), the q smallest scores are selected (ties: smaller index), and the
// coefficients of out = G c are 1/q on the selected workers.  One thread per worker; p <= 64.
__global__ __launch_bounds__(64) void fa_krum_kernel(const double* __restrict__ K, int p, int k,
                                                     int q, double* __restrict__ c,
                                                     double* __restrict__ scores,
                                                     int* __restrict__ selected) {
  __shared__ double sc[FA_P_MAX];
  __shared__ double dist[FA_P_MAX][FA_P_MAX + 1];
  const int i = threadIdx.x;
  double s = 0.0;
  if (i < p) {
    double* d = dist[i];
    const double kii = K[i * p + i];
    int cnt = 0;
    for (int j = 0; j < p; ++j) {
      if (j == i) continue;
      double x = kii + K[j * p + j] - 2.0 * K[i * p + j];
      x = x > 0.0 ? x : 0.0;
      int pos = cnt++;                       // insertion sort, ascending
      while (pos > 0 && d[pos - 1] > x) { d[pos] = d[pos - 1]; --pos; }
      d[pos] = x;
    }
    for (int t = 0; t < k; ++t) s += d[t];
    sc[i] = s;
    scores[i] = s;
  }
  __syncthreads();
  if (i < p) {
    int rank = 0;
    for (int j = 0; j < p; ++j) rank += (sc[j] < s || (sc[j] == s && j < i)) ? 1 : 0;
    const int sel = rank < q ? 1 : 0;
    selected[i] = sel;
    c[i] = sel ? 1.0 / (double)q : 0.0;
  }
}

// Y (+ a*ldy, a < m) = G A, A row-major p x m in device memory; eight columns per pass over G
// in either layout.
hipError_t fa_launch_combine_multi(const void* G, int64_t ldg, int p, int64_t n, int dtype,
                                   int layout, const double* A, int m, float* Y, int64_t ldy,
                                   int max_blocks, hipStream_t st) {
  if (layout == FA_ROW_MAJOR) {
    const int ldr = (int)ldg;
    const size_t lds = fa_rows_lds_bytes(ldr, dtype == FA_F32 ? 4 : 2);
    int64_t blocks = (n + 255) / 256;
    // one workgroup per span of 256 rows (measured at p = 15, n = 11.2M: 124 us; eight
    // persistent workgroups per compute unit 133 us, sixty-four 121-127 us)
    if (blocks > 0x7fffffff) blocks = 0x7fffffff;
    for (int a0 = 0; a0 < m; a0 += FA_ROWS_MULTI) {
      const int nc = m - a0 < FA_ROWS_MULTI ? m - a0 : FA_ROWS_MULTI;
      if (dtype == FA_F32)
        hipLaunchKernelGGL((fa_combine_rows_kernel<ElemF32, FA_ROWS_MULTI>), dim3((unsigned)blocks),
                           dim3(256), lds, st, (const unsigned char*)G, ldr, p, n, A + a0, m, nc,
                           Y + (int64_t)a0 * ldy, ldy);
      else
        hipLaunchKernelGGL((fa_combine_rows_kernel<ElemBF16, FA_ROWS_MULTI>), dim3((unsigned)blocks),
                           dim3(256), lds, st, (const unsigned char*)G, ldr, p, n, A + a0, m, nc,
                           Y + (int64_t)a0 * ldy, ldy);
      hipError_t e = hipGetLastError();
      if (e != hipSuccess) return e;
    }
    return hipSuccess;
  }
  constexpr int MB = 8;
  const int epl = dtype == FA_F32 ? 4 : 8;
  const int64_t ngroups = (n + epl - 1) / epl;
  int64_t blocks = (ngroups + 255) / 256;
  if (blocks > max_blocks) blocks = max_blocks;
  for (int a0 = 0; a0 < m; a0 += MB) {
    const int nc = m - a0 < MB ? m - a0 : MB;
    if (dtype == FA_F32)
      hipLaunchKernelGGL((fa_combine_multi_kernel<ElemF32, MB>), dim3((unsigned)blocks), dim3(256),
                         0, st, (const unsigned char*)G, ldg, p, n, A + a0, m, nc,
                         Y + (int64_t)a0 * ldy, ldy);
    else
      hipLaunchKernelGGL((fa_combine_multi_kernel<ElemBF16, MB>), dim3((unsigned)blocks), dim3(256),
                         0, st, (const unsigned char*)G, ldg, p, n, A + a0, m, nc,
                         Y + (int64_t)a0 * ldy, ldy);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t fa_launch_krum(const double* Kd, int p, int f, int q, double* cd, double* scores_d,
                          int* selected_d, hipStream_t st) {
  hipLaunchKernelGGL(fa_krum_kernel, dim3(1), dim3(64), 0, st, Kd, p, p - f - 2, q, cd, scores_d,
                     selected_d);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Streamed check of a materialised basis Y (n x m, fp32, column a at Y + a*ldy): one pass
// computes W = Y^T [Y | G] in fp64 on the matrix cores: Y^T Y (the identity for the
// orthonormal basis of Sec. 2.1) and Y^T G (row a, column i: the projection of g_i on y_a,
// whose squares add up to the explained variance of Sec. 2.1 times |g_i|^2).
// One workgroup (eight wavefronts) per (row stripe, tile row ta of the result); a wavefront
// takes 16 rows at a time: lane (c, k) holds rows 4k..4k+3 of column c of each 16-column tile
// of [Y | G] (one 16-byte load where the rows are contiguous), and feeds row 4k+s of tile ta
// of Y and of every tile to the s-th matrix instruction - the contraction does not care in
// which order the rows come, as long as both operands agree, and the registers of a tile
// serve as either operand.  [Y | G] is therefore read once per tile row of Y (once at
// m <= 16), all TC result tiles of the row accumulate in registers.
// G is addressed by strides (elements): g_rs between rows, g_cs between columns, which
// covers both storage orders.
template <typename E>
__device__ __forceinline__ double load_elem(const unsigned char* base, int64_t idx) {
  if constexpr (E::SIZE == 4) return (double)reinterpret_cast<const float*>(base)[idx];
  else return (double)bf16_bits_to_f32(reinterpret_cast<const uint16_t*>(base)[idx]);
}
// rows row0..row0+3 of one column (zero past n, zero if the column does not exist)
template <typename E>
__device__ __forceinline__ void load_rows4(const unsigned char* base, int64_t col_off,
                                           int64_t rs, int64_t row0, int64_t n, bool on,
                                           double* x) {
  x[0] = x[1] = x[2] = x[3] = 0.0;
  if (!on || row0 >= n) return;
  if (rs == 1 && row0 + 4 <= n) {
    const unsigned char* src = base + (col_off + row0) * E::SIZE;
    if constexpr (E::SIZE == 4) {
      if (((uintptr_t)src & 15u) == 0) {
        const float4 f = *reinterpret_cast<const float4*>(src);
        x[0] = (double)f.x; x[1] = (double)f.y; x[2] = (double)f.z; x[3] = (double)f.w;
        return;
      }
    } else {
      if (((uintptr_t)src & 7u) == 0) {
        const uint2 h = *reinterpret_cast<const uint2*>(src);
        x[0] = (double)bf16_bits_to_f32(h.x & 0xffffu); x[1] = (double)bf16_bits_to_f32(h.x >> 16);
        x[2] = (double)bf16_bits_to_f32(h.y & 0xffffu); x[3] = (double)bf16_bits_to_f32(h.y >> 16);
        return;
      }
    }
  }
  for (int s = 0; s < 4; ++s)
    if (row0 + s < n) x[s] = load_elem<E>(base, col_off + (row0 + s) * rs);
}

// four rows row0..row0+3 (all inside the matrix) of one column as raw bits: the loads of a
// stage are all issued before any of them is used
template <typename E, bool ROWS>
__device__ __forceinline__ uint4 cross_raw(const unsigned char* base, int64_t col_off, int64_t rs,
                                           int64_t row0) {
  uint4 r = {0u, 0u, 0u, 0u};
  if constexpr (!ROWS) {
    const unsigned char* src = base + (col_off + row0) * E::SIZE;
    if constexpr (E::SIZE == 4) {
      r = *reinterpret_cast<const uint4*>(src);
    } else {
      const uint2 h = *reinterpret_cast<const uint2*>(src);
      r.x = h.x; r.y = h.y;
    }
  } else if constexpr (E::SIZE == 4) {
    const uint32_t* g = reinterpret_cast<const uint32_t*>(base) + col_off + row0 * rs;
    r.x = g[0]; r.y = g[rs]; r.z = g[2 * rs]; r.w = g[3 * rs];
  } else {
    const uint16_t* g = reinterpret_cast<const uint16_t*>(base) + col_off + row0 * rs;
    r.x = g[0]; r.y = g[rs]; r.z = g[2 * rs]; r.w = g[3 * rs];
  }
  return r;
}
template <typename E, bool ROWS>
__device__ __forceinline__ void cross_decode(const uint4& r, double* x) {
  if constexpr (E::SIZE == 4) {
    x[0] = (double)__uint_as_float(r.x); x[1] = (double)__uint_as_float(r.y);
    x[2] = (double)__uint_as_float(r.z); x[3] = (double)__uint_as_float(r.w);
  } else if constexpr (!ROWS) {
    x[0] = (double)bf16_bits_to_f32(r.x & 0xffffu); x[1] = (double)bf16_bits_to_f32(r.x >> 16);
    x[2] = (double)bf16_bits_to_f32(r.y & 0xffffu); x[3] = (double)bf16_bits_to_f32(r.y >> 16);
  } else {
    x[0] = (double)bf16_bits_to_f32(r.x); x[1] = (double)bf16_bits_to_f32(r.y);
    x[2] = (double)bf16_bits_to_f32(r.z); x[3] = (double)bf16_bits_to_f32(r.w);
  }
}

// ROWS: G is stored row-major (g_rs = row pitch, g_cs = 1); otherwise g_rs = 1 and the four
// rows of a lane are one 16-byte (fp32) or 8-byte (bf16) load, aligned because G, Y and their
// column pitches are (the caller checks).
template <typename E, int TC, bool ROWS>
__global__ __launch_bounds__(512) void fa_cross_kernel(const float* __restrict__ Y, int64_t ldy,
                                                       int m,
                                                       const unsigned char* __restrict__ G,
                                                       int64_t g_rs, int64_t g_cs, int p,
                                                       int64_t n, int TMr,
                                                       double* __restrict__ partials) {
  // wavefronts; 16-row chunks per stage (the next stage's loads are in flight while this
  // one is multiplied: two stages of raw bits and TC accumulators share the registers)
  constexpr int NWV = 8, U = TC <= 2 ? 4 : TC <= 4 ? 2 : 1;
  __shared__ double red[NWV * 256];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c16 = lane & 15, kq = lane >> 4;
  const int ta = (int)blockIdx.y;            // tile row: columns 16 ta .. of Y on the left
  const unsigned char* Yb = reinterpret_cast<const unsigned char*>(Y);
  const int64_t wid = (int64_t)blockIdx.x * NWV + wave, nw = (int64_t)gridDim.x * NWV;
  v4f64 acc[TC];
#pragma unroll
  for (int tb = 0; tb < TC; ++tb) acc[tb] = v4f64{0.0, 0.0, 0.0, 0.0};

  // operands of tile tb for the rows of one chunk, already as doubles -> TC products
  auto multiply = [&](double (&b)[TC][4]) {
    double a[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      a[s] = b[0][s];
#pragma unroll
      for (int t = 1; t < TC && t < 4; ++t) a[s] = ta == t ? b[t][s] : a[s];
    }
#pragma unroll
    for (int tb = 0; tb < TC; ++tb)
#pragma unroll
      for (int s = 0; s < 4; ++s)
        acc[tb] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[s], b[tb][s], acc[tb], 0, 0, 0);
  };
  auto issue = [&](int64_t group, uint4 (&raw)[U][TC]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t row0 = (group * U + u) * 16 + 4 * kq;
#pragma unroll
      for (int tb = 0; tb < TC; ++tb) {
        raw[u][tb] = uint4{0u, 0u, 0u, 0u};
        if (tb < TMr) {                      // a tile of Y
          const int col = tb * 16 + c16;
          if (col < m) raw[u][tb] = cross_raw<ElemF32, false>(Yb, (int64_t)col * ldy, 1, row0);
        } else {                             // a tile of G
          const int col = (tb - TMr) * 16 + c16;
          if (col < p) raw[u][tb] = cross_raw<E, ROWS>(G, (int64_t)col * g_cs, g_rs, row0);
        }
      }
    }
  };
  auto consume = [&](uint4 (&raw)[U][TC]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      double b[TC][4];
#pragma unroll
      for (int tb = 0; tb < TC; ++tb) {
        if (tb < TMr) cross_decode<ElemF32, false>(raw[u][tb], b[tb]);
        else cross_decode<E, ROWS>(raw[u][tb], b[tb]);
      }
      multiply(b);
    }
  };

  // groups of U whole chunks, two stages in flight
  const int64_t ngroups = (n / 16) / U;
  uint4 cur[U][TC], nxt[U][TC];
  int64_t g = wid;
  if (g < ngroups) issue(g, cur);
  while (g < ngroups) {
    const int64_t gn = g + nw;
    if (gn < ngroups) issue(gn, nxt);
    consume(cur);
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int tb = 0; tb < TC; ++tb) cur[u][tb] = nxt[u][tb];
    g = gn;
  }
  // what is left: fewer than U whole chunks and the ragged one, one wavefront each, with
  // the careful loads
  const int64_t nchunks = (n + 15) / 16;
  const int64_t ch = ngroups * U + wid;
  if (ch < nchunks) {
    const int64_t row0 = ch * 16 + 4 * kq;
    double b[TC][4];
#pragma unroll
    for (int tb = 0; tb < TC; ++tb) {
      if (tb < TMr) {
        const int col = tb * 16 + c16;
        load_rows4<ElemF32>(Yb, (int64_t)col * ldy, 1, row0, n, col < m, b[tb]);
      } else {
        const int col = (tb - TMr) * 16 + c16;
        load_rows4<E>(G, (int64_t)col * g_cs, g_rs, row0, n, col < p, b[tb]);
      }
    }
    multiply(b);
  }
  // the wavefronts add up in wave order; one partial tile per workgroup and result tile
#pragma unroll
  for (int tb = 0; tb < TC; ++tb) {
#pragma unroll
    for (int r = 0; r < 4; ++r) red[wave * 256 + r * 64 + lane] = acc[tb][r];
    __syncthreads();
    double* dst = partials + (((int64_t)blockIdx.x * gridDim.y + ta) * TC + tb) * 256;
    for (int e = threadIdx.x; e < 256; e += 64 * NWV) {
      double tot = 0.0;
#pragma unroll
      for (int w = 0; w < NWV; ++w) tot += red[w * 256 + e];
      dst[e] = tot;
    }
    __syncthreads();
  }
}

// ------------------------------------------------------------------------------------------
// K3: the p x p solver, one workgroup, matrices in LDS.

__global__ __launch_bounds__(FA_IRLS_THREADS) void fa_irls_kernel(const double* __restrict__ Kg,
                                                                  fa_irls_args ar, double* cg,
                                                                  fa_info* info, double* gws,
                                                                  int big_in_global,
                                                                  fa_resume* rs, int retry_only) {
  // as the stand-by of the matrix-core solver: nothing to do unless that one gave up
  if (retry_only && info->status != FA_ST_RETRY) return;
  extern __shared__ __attribute__((aligned(16))) double dyn[];
  const int p = ar.p;
  const int ld = p | 1;
  fa_irls_mem sm;
  sm.ld = ld;
  double* q = dyn;
  const size_t msz = (size_t)p * ld;
  sm.R = q; q += msz;
  sm.Ut = q; q += msz;
  sm.CM = q; q += msz;
  sm.T = q; q += msz;
  if (big_in_global) {
    sm.D2inv = gws;
    sm.Vt = gws + msz;
  } else {
    sm.D2inv = q; q += msz;
    sm.Vt = q; q += msz;
  }
  sm.s = q; q += FA_P_MAX;
  sm.dinv = q; q += FA_P_MAX;
  sm.w = q; q += FA_P_MAX;
  sm.rho = q; q += FA_P_MAX;
  sm.v = q; q += FA_P_MAX;
  sm.lam0 = q; q += FA_P_MAX;
  sm.mu = q; q += FA_P_MAX;
  sm.beta = q; q += FA_P_MAX;
  sm.ginv = q; q += FA_P_MAX;
  sm.ctop = q; q += FA_P_MAX;
  sm.cbot = q; q += FA_P_MAX;
  sm.rot_c = q; q += FA_P_MAX / 2;
  sm.rot_s = q; q += FA_P_MAX / 2;
  sm.red = q; q += FA_IRLS_THREADS;
  int* qi = reinterpret_cast<int*>(q);
  sm.rot_p = qi; qi += FA_P_MAX / 2;
  sm.rot_q = qi; qi += FA_P_MAX / 2;
  sm.pos = qi; qi += FA_P_MAX;
  sm.order = qi; qi += FA_P_MAX;
  sm.gfirst = qi; qi += FA_P_MAX;
  sm.gcnt = qi; qi += FA_P_MAX;
  sm.flag = qi; qi += 8;
  fa_irls_solve(Kg, ar, sm, cg, info, rs);
}

size_t fa_irls_lds_bytes(int p, int* big_in_global) {
  const size_t msz = (size_t)p * (p | 1) * sizeof(double);
  const size_t small = (11 * FA_P_MAX + FA_P_MAX + FA_IRLS_THREADS) * sizeof(double) +
                       (5 * FA_P_MAX + 8) * sizeof(int);
  size_t need = 6 * msz + small;
  *big_in_global = 0;
  if (need > 60 * 1024) {   // keep the common sizes under the default dynamic-LDS limit
    need = 4 * msz + small;
    *big_in_global = 1;
  }
  return need;
}

// ------------------------------------------------------------------------------------------
// launchers (host).  Shapes are validated by the callers in fa_api.hip.
template <int T, int CPL, typename E, int WAVES, bool ROWS>
static hipError_t launch_gram_t(const void* G, int64_t ldg, int p, int64_t n, int max_blocks,
                                double* partials, int* nparts, hipStream_t st,
                                const fa_ktime* tm, const int* gate) {
  static_assert(WAVES <= FA_GRAM_WAVES_PER_CU, "partials buffer is sized for this many");
  constexpr int R = (64 / CPL) * E::EPL;
  constexpr int CS = R * E::SIZE + 16;
  constexpr size_t tile_bytes = (size_t)T * 16 * CS;
  static_assert(WAVES * tile_bytes <= 160 * 1024, "LDS tiles of one workgroup must fit a CU");
  // more than half of the CU's 160 KiB, so that no second workgroup fits beside this one
  const size_t lds_bytes = WAVES * tile_bytes > 84 * 1024 ? WAVES * tile_bytes : 84 * 1024;
  const int64_t ntiles = (n + R - 1) / R;
  int64_t wgs = (ntiles + WAVES - 1) / WAVES;
  if (wgs > max_blocks) wgs = max_blocks;
  *nparts = (int)wgs;
  FA_LAUNCH(tm, (fa_gram_kernel<T, CPL, E, WAVES, ROWS>), dim3((unsigned)wgs),
            dim3(64 * WAVES), lds_bytes, st, (const unsigned char*)G, ldg, p, n, ntiles,
            partials, gate);
  return hipGetLastError();
}

// the tiling of each width class: T -> (columns per load, wavefronts per CU)
#define FA_GRAM_TILINGS(X) \
  X(1, FA_GRAM_CPL1, FA_GRAM_W1) X(2, FA_GRAM_CPL2, FA_GRAM_W2) X(3, 4, 8) X(4, FA_GRAM_CPL4, FA_GRAM_W4)

template <typename E, bool ROWS>
static hipError_t launch_gram_e(const void* G, int64_t ldg, int p, int64_t n, int max_blocks,
                                double* partials, int* nparts, hipStream_t st,
                                const fa_ktime* tm, const int* gate) {
  switch ((p + 15) / 16) {
#define FA_X(t, cpl, w)                                                                        \
    case t: return launch_gram_t<t, cpl, E, w, ROWS>(G, ldg, p, n, max_blocks, partials, nparts, \
                                                     st, tm, gate);
    FA_GRAM_TILINGS(FA_X)
#undef FA_X
  }
  return hipErrorInvalidValue;
}

template <typename E, bool ROWS>
static hipError_t prepare_gram_e() {
  hipError_t e = hipSuccess;
#define FA_X(t, cpl, w)                                                                          \
  if (e == hipSuccess)                                                                           \
    e = hipFuncSetAttribute(                                                                     \
        reinterpret_cast<const void*>(fa_gram_kernel<t, cpl, E, w, ROWS>),                       \
        hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
  FA_GRAM_TILINGS(FA_X)
#undef FA_X
  return e;
}

bool fa_gram_takes_matrix_core(int p, int64_t n, int dtype, int layout, int gram_mode) {
  const bool want_lp = gram_mode == FA_GRAM_BF16_MATRIX ||
                       (gram_mode == FA_GRAM_AUTO && n >= FA_GRAM_AUTO_MIN_ROWS);
  return want_lp && layout == FA_WORKER_MAJOR && fa_gram_lp_applies(p, dtype);
}

hipError_t fa_launch_gram_partials(const void* G, int64_t ldg, int p, int64_t n, int dtype,
                                   int layout, int gram_mode, int max_blocks, double* partials,
                                   int* nparts, hipStream_t st, const fa_ktime* tm,
                                   const int* gate) {
  if (fa_gram_takes_matrix_core(p, n, dtype, layout, gram_mode))
    return fa_launch_gram_lp_partials(G, ldg, p, n, dtype, max_blocks, partials, nparts, st, tm);
  const bool rows = layout == FA_ROW_MAJOR;
  if (dtype == FA_F32)
    return rows ? launch_gram_e<ElemF32, true>(G, ldg, p, n, max_blocks, partials, nparts, st, tm, gate)
                : launch_gram_e<ElemF32, false>(G, ldg, p, n, max_blocks, partials, nparts, st, tm, gate);
  return rows ? launch_gram_e<ElemBF16, true>(G, ldg, p, n, max_blocks, partials, nparts, st, tm, gate)
              : launch_gram_e<ElemBF16, false>(G, ldg, p, n, max_blocks, partials, nparts, st, tm, gate);
}

hipError_t fa_launch_gram_reduce(const double* partials, int nparts, int p, double* Kd,
                                 const double* colscale, hipStream_t st, const fa_ktime* tm,
                                 const int* gate) {
  const int T = (p + 15) / 16;
  const int NTP = T * (T + 1) / 2;
  FA_LAUNCH(tm, fa_gram_reduce_kernel, dim3(NTP * 4), dim3(1024), 0, st, partials, nparts, T, p,
            Kd, 0, 0, colscale, gate);
  return hipGetLastError();
}

// *flag = 1 if any of the count doubles at K is NaN or infinite, else 0
__global__ __launch_bounds__(256) void fa_nonfinite_flag_kernel(const double* __restrict__ K,
                                                                int count, int* __restrict__ flag) {
  bool bad = false;
  for (int k = threadIdx.x; k < count; k += 256) bad = bad || !(fabs(K[k]) <= 1.79e308);
  const int any = __syncthreads_or(bad ? 1 : 0);
  if (threadIdx.x == 0) *flag = any ? 1 : 0;
}

// K1 + K2: K = G^T G into Kd.  Where the pass runs on the bf16 matrix core, whose 32-row sums
// are fp32 and overflow for values beyond ~1e18, the fp64 pass stands by behind it: it is
// always enqueued and returns at once unless K came out non-finite (flag_d: one int of device
// scratch), so that large finite values - a Byzantine worker may send anything - cost a second
// pass instead of the result.  tm_gram / tm_reduce time the first pass and its reduction.
hipError_t fa_launch_gram(const void* G, int64_t ldg, int p, int64_t n, int dtype, int layout,
                          int gram_mode, int max_blocks, double* partials, double* Kd,
                          int* flag_d, int* nparts, hipStream_t st, const fa_ktime* tm_gram,
                          const fa_ktime* tm_reduce) {
  hipError_t e = fa_launch_gram_partials(G, ldg, p, n, dtype, layout, gram_mode, max_blocks,
                                         partials, nparts, st, tm_gram, nullptr);
  if (e != hipSuccess) return e;
  e = fa_launch_gram_reduce(partials, *nparts, p, Kd, nullptr, st, tm_reduce, nullptr);
  if (e != hipSuccess || !fa_gram_takes_matrix_core(p, n, dtype, layout, gram_mode)) return e;
  hipLaunchKernelGGL(fa_nonfinite_flag_kernel, dim3(1), dim3(256), 0, st, (const double*)Kd, p * p,
                     flag_d);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  int np2 = 0;
  e = fa_launch_gram_partials(G, ldg, p, n, dtype, layout, FA_GRAM_FP64, max_blocks, partials, &np2,
                              st, nullptr, flag_d);
  if (e != hipSuccess) return e;
  return fa_launch_gram_reduce(partials, np2, p, Kd, nullptr, st, nullptr, flag_d);
}

hipError_t fa_launch_proj_reduce(const double* partials, int nparts, int p, int m, double* Td,
                                 hipStream_t st, const fa_ktime* tm) {
  const int T = (p + 15) / 16, TM = (m + 15) / 16;
  FA_LAUNCH(tm, fa_gram_reduce_kernel, dim3(T * TM * 4), dim3(1024), 0, st, partials, nparts, T,
            p, Td, TM, m, (const double*)nullptr, (const int*)nullptr);
  return hipGetLastError();
}

// W = Y^T [Y | G], m x (16 ceil(m/16) + p) row-major into Wd: the partial tiles of at most
// max_parts row stripes go to `partials` (max_parts * tiles * 256 doubles), then K2 adds them.
hipError_t fa_launch_cross(const float* Y, int64_t ldy, int m, const void* G, int64_t ldg, int p,
                           int64_t n, int dtype, int layout, int max_parts, double* partials,
                           double* Wd, hipStream_t st) {
  const int TMr = (m + 15) / 16, TC = TMr + (p + 15) / 16;
  const int64_t g_rs = layout == FA_ROW_MAJOR ? ldg : 1, g_cs = layout == FA_ROW_MAJOR ? 1 : ldg;
  // two workgroups of eight wavefronts per compute unit of a 256-unit chip, at most
  int64_t stripes = (n + 8 * 16 - 1) / (8 * 16);             // a chunk per wavefront at least
  if (stripes > 512 / TMr) stripes = 512 / TMr;
  if (stripes > max_parts) stripes = max_parts;
  if (stripes < 1) stripes = 1;
  const dim3 grid((unsigned)stripes, (unsigned)TMr);
  const bool rows = layout == FA_ROW_MAJOR;
  switch (TC) {
#define FA_Y(E, tc, R)                                                                     \
  hipLaunchKernelGGL((fa_cross_kernel<E, tc, R>), grid, dim3(512), 0, st, Y, ldy, m,       \
                     (const unsigned char*)G, g_rs, g_cs, p, n, TMr, partials)
#define FA_X(tc)                                                       \
    case tc:                                                           \
      if (dtype == FA_F32) {                                           \
        if (rows) FA_Y(ElemF32, tc, true); else FA_Y(ElemF32, tc, false);   \
      } else {                                                         \
        if (rows) FA_Y(ElemBF16, tc, true); else FA_Y(ElemBF16, tc, false); \
      }                                                                \
      break;
    FA_X(2) FA_X(3) FA_X(4) FA_X(5) FA_X(6) FA_X(7) FA_X(8)
#undef FA_X
#undef FA_Y
    default: return hipErrorInvalidValue;
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int ncols = 16 * TMr + p;
  hipLaunchKernelGGL(fa_gram_reduce_kernel, dim3(TMr * TC * 4), dim3(1024), 0, st,
                     (const double*)partials, (int)stripes, TMr, m, Wd, TC, ncols,
                     (const double*)nullptr, (const int*)nullptr);
  return hipGetLastError();
}

template <int T, int TM, int CPL, typename E, int WAVES>
static hipError_t launch_proj_t(const void* G, int64_t ldg, int p, int m, int64_t n,
                                int max_blocks, const double* Acoef, double* partials,
                                int* nparts, hipStream_t st, const fa_ktime* tm) {
  constexpr int R = (64 / CPL) * E::EPL;
  constexpr int CS = R * E::SIZE + 16;
  constexpr size_t a_bytes = (size_t)T * 16 * TM * 16 * sizeof(double);
  constexpr size_t tile_bytes = (size_t)T * 16 * CS;
  constexpr size_t need = a_bytes + (WAVES * tile_bytes > WAVES * 2048u ? WAVES * tile_bytes
                                                                        : WAVES * 2048u);
  static_assert(need <= 160 * 1024, "LDS of one workgroup must fit a CU");
  const size_t lds_bytes = need > 84 * 1024 ? need : 84 * 1024;   // one workgroup per CU
  const int64_t ntiles = (n + R - 1) / R;
  int64_t wgs = (ntiles + WAVES - 1) / WAVES;
  if (wgs > max_blocks) wgs = max_blocks;
  *nparts = (int)wgs;
  FA_LAUNCH(tm, (fa_proj_kernel<T, TM, CPL, E, WAVES>), dim3((unsigned)wgs), dim3(64 * WAVES),
            lds_bytes, st, (const unsigned char*)G, ldg, p, m, n, ntiles, Acoef, partials);
  return hipGetLastError();
}

// (T, TM) -> (columns per load, wavefronts per CU); the larger tilings run four wavefronts per
// CU: they need more than 256 registers a lane
#define FA_PROJ_TILINGS(X)                                                        \
  X(1, 1, 4, 12) X(2, 1, 4, 8) X(2, 2, 4, 8) X(3, 1, 4, 8) X(3, 2, 4, 8) X(3, 3, 4, 4) \
  X(4, 1, 8, 8) X(4, 2, 8, 4) X(4, 3, 8, 4) X(4, 4, 8, 4)

template <typename E>
static hipError_t launch_proj_e(const void* G, int64_t ldg, int p, int m, int64_t n,
                                int max_blocks, const double* Acoef, double* partials,
                                int* nparts, hipStream_t st, const fa_ktime* tm) {
  const int T = (p + 15) / 16, TM = (m + 15) / 16;
#define FA_PROJ_CASE(t, tmm, cpl, w)                                                            \
  if (T == t && TM == tmm)                                                                      \
    return launch_proj_t<t, tmm, cpl, E, w>(G, ldg, p, m, n, max_blocks, Acoef, partials, nparts, \
                                            st, tm);
  FA_PROJ_TILINGS(FA_PROJ_CASE)
#undef FA_PROJ_CASE
  return hipErrorInvalidValue;
}

template <typename E>
static hipError_t prepare_proj_e() {
  hipError_t e = hipSuccess;
#define FA_PROJ_CASE(t, tmm, cpl, w)                                                            \
  if (e == hipSuccess)                                                                          \
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(fa_proj_kernel<t, tmm, cpl, E, w>),   \
                            hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
  FA_PROJ_TILINGS(FA_PROJ_CASE)
#undef FA_PROJ_CASE
  return e;
}

hipError_t fa_launch_proj_partials(const void* G, int64_t ldg, int p, int m, int64_t n, int dtype,
                                   int max_blocks, const double* Acoef, double* partials,
                                   int* nparts, hipStream_t st, const fa_ktime* tm) {
  if (dtype == FA_F32)
    return launch_proj_e<ElemF32>(G, ldg, p, m, n, max_blocks, Acoef, partials, nparts, st, tm);
  return launch_proj_e<ElemBF16>(G, ldg, p, m, n, max_blocks, Acoef, partials, nparts, st, tm);
}

hipError_t fa_launch_restream_weights(const fa_info* info_d, const double* Pd, int p, int m,
                                      double lambda, double delta, double pair_tol,
                                      double exponent_a, fa_resume* rs, hipStream_t st) {
  const double coef = (lambda > 0.0 && p > 1) ? lambda / (double)(p - 1) : 0.0;
  hipLaunchKernelGGL(fa_restream_weights_kernel, dim3(1), dim3(256), 0, st, info_d, Pd, p, m, coef,
                     delta, pair_tol, 1.0 / exponent_a, rs);
  return hipGetLastError();
}

hipError_t fa_launch_irls(const double* Kd, int p, int m, double lambda, int iters, double tol,
                          double delta, double rank_tol, double pair_tol, double exponent_a,
                          double* cd,
                          fa_info* info_d, double* gws, int solver, int spin_budget,
                          fa_resume* rs, hipStream_t st, const fa_ktime* tm) {
  if (p <= 16 && solver != 2)
    return fa_launch_irls16(Kd, p, m, lambda, iters, tol, delta, exponent_a, rank_tol, pair_tol, cd,
                            info_d,
                            gws + FA_GWS_MLAST_OFF, solver == 0 ? 1 : 0, rs, st, tm);
  int retry_only = 0;
  fa_ktime first = {nullptr, nullptr}, second = {nullptr, nullptr};
  if (p > 16 && solver == 0) {
    // timing, if asked for, spans both launches: begin of the first, end of the second
    if (tm) { first.start = tm->start; second.stop = tm->stop; }
    hipError_t e = fa_launch_irls64(Kd, p, 0, nullptr, m, lambda, iters, tol, delta, exponent_a,
                                    rank_tol, pair_tol, cd,
                                    info_d, gws + FA_GWS_GENERIC, gws + FA_GWS_MLAST_OFF,
                                    spin_budget, rs, st, tm ? &first : nullptr);
    if (e != hipSuccess) return e;
    retry_only = 1;   // the Jacobi kernel below runs only if the one above gave up
    tm = tm ? &second : nullptr;
  }
  fa_irls_args ar;
  ar.p = p; ar.m = m; ar.iters = iters; ar.lambda = lambda; ar.tol = tol;
  ar.delta = delta; ar.rank_tol = rank_tol; ar.pair_tol = pair_tol;
  ar.expo = 1.0 / exponent_a;
  ar.nworkers = 0; ar.sizes = nullptr;
  int big = 0;
  const size_t lds = fa_irls_lds_bytes(p, &big);
  FA_LAUNCH(tm, fa_irls_kernel, dim3(1), dim3(FA_IRLS_THREADS), lds, st, Kd, ar, cd, info_d, gws,
            big, rs, retry_only);
  return hipGetLastError();
}

// The same for workers that send several gradients: q columns in nworkers blocks of
// sizes_d[i] consecutive columns (device memory).  solver 0: the matrix-core purification
// kernel, with the any-p kernel behind it as stand-by; otherwise the any-p kernel alone.
hipError_t fa_launch_irls_grouped(const double* Kd, int q, int nworkers, const int* sizes_d, int m,
                                  double lambda, int iters, double tol, double delta,
                                  double rank_tol, double pair_tol, double exponent_a, double* cd,
                                  fa_info* info_d, double* gws, int solver, int spin_budget,
                                  hipStream_t st) {
  int retry_only = 0;
  if (solver == 0) {
    hipError_t e = fa_launch_irls64(Kd, q, nworkers, sizes_d, m, lambda, iters, tol, delta,
                                    exponent_a, rank_tol, pair_tol, cd, info_d,
                                    gws + FA_GWS_GENERIC, gws + FA_GWS_MLAST_OFF, spin_budget,
                                    nullptr, st, nullptr);
    if (e != hipSuccess) return e;
    retry_only = 1;   // the Jacobi kernel below runs only if the one above gave up
  }
  fa_irls_args ar;
  ar.p = q; ar.m = m; ar.iters = iters; ar.lambda = lambda; ar.tol = tol;
  ar.delta = delta; ar.rank_tol = rank_tol; ar.pair_tol = pair_tol;
  ar.expo = 1.0 / exponent_a;
  ar.nworkers = nworkers; ar.sizes = sizes_d;
  int big = 0;
  const size_t lds = fa_irls_lds_bytes(q, &big);
  hipLaunchKernelGGL(fa_irls_kernel, dim3(1), dim3(FA_IRLS_THREADS), lds, st, Kd, ar, cd, info_d,
                     gws, big, (fa_resume*)nullptr, retry_only);
  return hipGetLastError();
}

// Eigenvalues of the last weighted-PCA matrix (N x N row-major, then rank and m, left by the
// purification paths) by the Jacobi routine above; writes the relative gap between
// eigenvalues m and m+1.
__global__ __launch_bounds__(256) void fa_gap_kernel(const double* __restrict__ mlast, int N,
                                                     fa_info* __restrict__ info) {
  extern __shared__ __attribute__((aligned(16))) double gl[];
  const int ld = N + 1;
  double* A = gl;                       // N x ld
  double* vals = A + N * ld;            // 64
  double* rc = vals + 64;               // 32
  double* rsn = rc + 32;                // 32
  double* red = rsn + 32;               // 256
  int* rp = reinterpret_cast<int*>(red + 256);
  int* rq = rp + 32;
  int* pos = rq + 32;
  int* order = pos + 64;
  int* flag = order + 64;
  fa_irls_mem sm;
  sm.ld = ld;
  sm.rot_c = rc; sm.rot_s = rsn; sm.rot_p = rp; sm.rot_q = rq; sm.red = red; sm.flag = flag;
  sm.pos = pos; sm.order = order;
  const int r = (int)mlast[N * N], m = (int)mlast[N * N + 1];
  for (int idx = threadIdx.x; idx < N * N; idx += 256) A[(idx / N) * ld + (idx % N)] = mlast[idx];
  if (threadIdx.x == 0) flag[4] = 0;
  __syncthreads();
  if (r < 1 || r > N) return;
  fa_jacobi(A, r, (double*)0, 0, (double*)0, 0, sm, 60);
  FA_FOR(a, r) vals[a] = A[a * ld + a];
  FA_SYNC();
  fa_rank_desc(vals, r, pos, order);
  if (threadIdx.x == 0) {
    double gap = __builtin_inf();
    if (m < r) gap = (vals[order[m - 1]] - vals[order[m]]) / vals[order[0]];
    info->eigengap = gap;
  }
}

hipError_t fa_launch_gap(const double* mlast, int N, fa_info* info_d, hipStream_t st) {
  const size_t lds = ((size_t)N * (N + 1) + 64 + 32 + 32 + 256) * sizeof(double) +
                     (32 + 32 + 64 + 64 + 8) * sizeof(int);
  hipLaunchKernelGGL(fa_gap_kernel, dim3(1), dim3(256), lds, st, mlast, N, info_d);
  return hipGetLastError();
}

hipError_t fa_kernels_prepare(void) {
  // the single-workgroup Jacobi solver's large dynamic LDS (p = 64 needs ~140 KiB)
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(fa_irls_kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
  // the streaming kernels that claim a whole compute unit's LDS
  if (e == hipSuccess) e = prepare_gram_e<ElemF32, false>();
  if (e == hipSuccess) e = prepare_gram_e<ElemF32, true>();
  if (e == hipSuccess) e = prepare_gram_e<ElemBF16, false>();
  if (e == hipSuccess) e = prepare_gram_e<ElemBF16, true>();
  if (e == hipSuccess) e = prepare_proj_e<ElemF32>();
  if (e == hipSuccess) e = prepare_proj_e<ElemBF16>();
  if (e == hipSuccess)
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(fa_combine_rows_kernel<ElemF32, 1>),
                            hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)fa_rows_lds_bytes(FA_P_MAX, 4));
  if (e == hipSuccess)
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(fa_combine_rows_kernel<ElemBF16, 1>),
                            hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)fa_rows_lds_bytes(FA_P_MAX, 4));
  if (e == hipSuccess)
    e = hipFuncSetAttribute(
        reinterpret_cast<const void*>(fa_combine_rows_kernel<ElemF32, FA_ROWS_MULTI>),
        hipFuncAttributeMaxDynamicSharedMemorySize, (int)fa_rows_lds_bytes(FA_P_MAX, 4));
  if (e == hipSuccess)
    e = hipFuncSetAttribute(
        reinterpret_cast<const void*>(fa_combine_rows_kernel<ElemBF16, FA_ROWS_MULTI>),
        hipFuncAttributeMaxDynamicSharedMemorySize, (int)fa_rows_lds_bytes(FA_P_MAX, 4));
  return e;
}

hipError_t fa_launch_combine(const void* G, int64_t ldg, int p, int64_t n, int dtype, int layout,
                             const double* c, int cstride, float* out, int max_blocks,
                             hipStream_t st, const fa_ktime* tm) {
  if (layout == FA_ROW_MAJOR) {
    const int ldr = (int)ldg;
    const size_t lds = fa_rows_lds_bytes(ldr, dtype == FA_F32 ? 4 : 2);
    int64_t blocks = (n + 255) / 256;
    // one workgroup per span of 256 rows (measured at p = 15, n = 11.2M: 124 us; eight
    // persistent workgroups per compute unit 133 us, sixty-four 121-127 us)
    if (blocks > 0x7fffffff) blocks = 0x7fffffff;
    if (dtype == FA_F32)
      FA_LAUNCH(tm, (fa_combine_rows_kernel<ElemF32, 1>), dim3((unsigned)blocks), dim3(256), lds,
                st, (const unsigned char*)G, ldr, p, n, c, cstride, 1, out, (int64_t)0);
    else
      FA_LAUNCH(tm, (fa_combine_rows_kernel<ElemBF16, 1>), dim3((unsigned)blocks), dim3(256), lds,
                st, (const unsigned char*)G, ldr, p, n, c, cstride, 1, out, (int64_t)0);
    return hipGetLastError();
  }
  const int epl = dtype == FA_F32 ? 4 : 8;
  const int64_t ngroups = (n + epl - 1) / epl;
  int64_t blocks = (ngroups + 255) / 256;
  if (blocks > max_blocks) blocks = max_blocks;
  if (dtype == FA_F32)
    FA_LAUNCH(tm, (fa_combine_kernel<ElemF32>), dim3((unsigned)blocks), dim3(256), 0, st,
              (const unsigned char*)G, ldg, p, n, c, cstride, out);
  else
    FA_LAUNCH(tm, (fa_combine_kernel<ElemBF16>), dim3((unsigned)blocks), dim3(256), 0, st,
              (const unsigned char*)G, ldg, p, n, c, cstride, out);
  return hipGetLastError();
}
