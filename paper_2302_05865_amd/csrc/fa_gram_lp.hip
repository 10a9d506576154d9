// K1 on the bf16 matrix core: norms + Gram matrix K = G^T G for the cases in which the fp64
// matrix core, not HBM, bounds the fp64 kernel of fa_kernels.hip (bf16 storage at any p, fp32
// storage at p > 16).  Sec. 2.1 (|g_i|^2), Sec. 2.3 (D_ij^2 = K_ii + K_jj - 2 K_ij).
//
// Arithmetic.  One v_mfma_f32_16x16x32_bf16 contracts 32 rows: products of two bf16 values
// are exact in fp32, the instruction adds the 32 of them with (nearly) one rounding -- measured
// on MI355X: 89 % of its results are the correctly rounded exact sum, rms error 0.6 ulp, and
// sums of squares come out low by 3.5e-9 relative on average -- and every such 32-row partial
// is added to an fp64 accumulator at once, so nothing else is ever rounded to fp32.  An entry
// of K is then good to a few 1e-9 of sqrt(K_ii K_jj) (diagonal: the bias above; off-diagonal:
// random, shrinking with 1/sqrt(n)); the fp64 kernel (about 1e-14) stays selectable.
// fp32 storage: every value is split exactly into three bf16 pieces x = h + m + l (round to
// nearest at each cut, so the remainders are zero-mean) and G^T G is the sum of the products of
// pieces; the terms m*l, l*m, l*l (2^-26 of a product and smaller) are left out, the other six
// go through one accumulator chain, smallest first.
// Identical columns give bitwise identical entries (the arithmetic does not depend on the
// position), so exact duplicates stay exact.  Range: products and 32-row sums must be finite
// in fp32 (|g| below about 1e18); beyond that K is non-finite and the call reports it.
//
// Data path as in the fp64 kernel: 16-byte coalesced non-temporal loads (next tile in flight
// while this one is multiplied) -> per-wavefront LDS tile [column][row] -> one 16-byte LDS
// read per operand (lane (c, q) holds rows 8q..8q+7 of column c: A and B operand of a
// diagonal block at once) -> matrix core.  One workgroup per compute unit, static
// wave -> tile map, fixed-order sums: results are bitwise reproducible.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fa.h"
#include "fa_internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint4 load16_nt(const void* src) {
  const uint32_t* s = reinterpret_cast<const uint32_t*>(src);
  uint4 v;   // merged into one global_load_dwordx4 nt
  v.x = __builtin_nontemporal_load(s);
  v.y = __builtin_nontemporal_load(s + 1);
  v.z = __builtin_nontemporal_load(s + 2);
  v.w = __builtin_nontemporal_load(s + 3);
  return v;
}

// 16 bytes of a column starting at element row0, zero-filled past row n (ES = element size)
template <int ES>
__device__ __forceinline__ uint4 load16_tail(const unsigned char* base, int64_t row0, int64_t n) {
  constexpr int EPL = 16 / ES;
  uint4 v = make_uint4(0u, 0u, 0u, 0u);
  if (row0 + EPL <= n) {
    v = load16_nt(base + row0 * ES);
  } else if (row0 < n) {
    uint32_t w[4] = {0u, 0u, 0u, 0u};
    if constexpr (ES == 4) {
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

__device__ __forceinline__ void lds_fence() {
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

// two fp32 -> two bf16 (round to nearest even) in one dword: low half = a, high half = b
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  const f32x2 v = {a, b};
  const bf16x2 h = __builtin_convertvector(v, bf16x2);
  return __builtin_bit_cast(uint32_t, h);
}

// x0, x1 -> the three bf16 pieces of each, packed pairwise: x = h + m + l exactly
__device__ __forceinline__ void split3(uint32_t u0, uint32_t u1, uint32_t* h, uint32_t* m,
                                       uint32_t* l) {
  const float x0 = __uint_as_float(u0), x1 = __uint_as_float(u1);
  const uint32_t hp = pack_bf16(x0, x1);
  const float r0 = x0 - __uint_as_float(hp << 16), r1 = x1 - __uint_as_float(hp & 0xffff0000u);
  const uint32_t mp = pack_bf16(r0, r1);
  const float s0 = r0 - __uint_as_float(mp << 16), s1 = r1 - __uint_as_float(mp & 0xffff0000u);
  *h = hp;
  *m = mp;
  *l = pack_bf16(s0, s1);     // exact: at most eight significant bits are left
}

}  // namespace

// T = 16-column blocks; CPL = columns per load instruction; ES = bytes per stored element
// (2: bf16, one LDS plane; 4: fp32, three planes of bf16 pieces); WAVES per workgroup.
template <int T, int CPL, int ES, int WAVES>
__global__ __launch_bounds__(64 * WAVES) void fa_gram_lp_kernel(
    const unsigned char* __restrict__ G, int64_t ldg, int p, int64_t n, int64_t ntiles,
    double* __restrict__ partials) {
  constexpr int EPL = 16 / ES;               // elements per 16-byte lane load
  constexpr int LPC = 64 / CPL;              // lanes per column in one load instruction
  constexpr int R = LPC * EPL;               // rows per tile
  constexpr int NCG = T * 16 / CPL;          // load instructions per tile
  constexpr int CS = R * 2 + 16;             // LDS bytes per column of bf16 (+16: bank spread)
  constexpr int NPL = ES == 4 ? 3 : 1;       // LDS planes
  constexpr int PLANE = T * 16 * CS;
  constexpr int NTP = T * (T + 1) / 2;
  constexpr int NSTEP = R / 32;
  static_assert(R % 32 == 0, "a tile is a whole number of 32-row contractions");
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_all[];
  const int wave = threadIdx.x >> 6;
  unsigned char* lds = lds_all + wave * (NPL * PLANE);
  const int64_t wid = (int64_t)blockIdx.x * WAVES + wave;
  const int64_t nwaves = (int64_t)gridDim.x * WAVES;
  const int lane = threadIdx.x & 63;
  const int lcol = lane / LPC;
  const int lrow = (lane % LPC) * EPL;
  const int c16 = lane & 15, q4 = lane >> 4;

  double acc[NTP][4];
#pragma unroll
  for (int i = 0; i < NTP; ++i)
#pragma unroll
    for (int r = 0; r < 4; ++r) acc[i][r] = 0.0;

  // zero the tile once: columns >= p are never written and stay zero
  for (int off = lane * 16; off < NPL * PLANE; off += 64 * 16)
    *reinterpret_cast<uint4*>(lds + off) = make_uint4(0u, 0u, 0u, 0u);

  const unsigned char* colbase[NCG];
  bool colon[NCG];
#pragma unroll
  for (int cg = 0; cg < NCG; ++cg) {
    const int col = cg * CPL + lcol;
    colon[cg] = col < p;     // lanes of columns >= p re-read column p-1 and drop the data
    colbase[cg] = G + (int64_t)(colon[cg] ? col : p - 1) * ldg * ES;
  }

  uint4 regs[NCG];
  auto load_tile = [&](int64_t tl) {
    const int64_t row0 = tl * R + lrow;
    if ((tl + 1) * R <= n) {                 // uniform: a full tile needs no row guards
#pragma unroll
      for (int cg = 0; cg < NCG; ++cg) regs[cg] = load16_nt(colbase[cg] + row0 * ES);
    } else {
#pragma unroll
      for (int cg = 0; cg < NCG; ++cg) regs[cg] = load16_tail<ES>(colbase[cg], row0, n);
    }
  };
  auto store_tile_lds = [&]() {
#pragma unroll
    for (int cg = 0; cg < NCG; ++cg) {
      if (!colon[cg]) continue;
      unsigned char* dst = lds + (cg * CPL + lcol) * CS + lrow * 2;
      if constexpr (ES == 2) {
        *reinterpret_cast<uint4*>(dst) = regs[cg];
      } else {
        uint32_t h0, m0, l0, h1, m1, l1;
        split3(regs[cg].x, regs[cg].y, &h0, &m0, &l0);
        split3(regs[cg].z, regs[cg].w, &h1, &m1, &l1);
        *reinterpret_cast<uint2*>(dst) = make_uint2(h0, h1);
        *reinterpret_cast<uint2*>(dst + PLANE) = make_uint2(m0, m1);
        *reinterpret_cast<uint2*>(dst + 2 * PLANE) = make_uint2(l0, l1);
      }
    }
  };

  lds_fence();
  int64_t tile = wid;
  if (tile < ntiles) load_tile(tile);
  for (; tile < ntiles; tile += nwaves) {
    lds_fence();   // the previous tile's LDS reads precede these writes
    store_tile_lds();
    lds_fence();
    const int64_t next = tile + nwaves;
    if (next < ntiles) load_tile(next);

    const unsigned char* src = lds + c16 * CS + 8 * q4 * 2;
#pragma unroll
    for (int t = 0; t < NSTEP; ++t) {
      bf16x8 op[NPL][T];
#pragma unroll
      for (int pl = 0; pl < NPL; ++pl)
#pragma unroll
        for (int tt = 0; tt < T; ++tt)
          op[pl][tt] = *reinterpret_cast<const bf16x8*>(src + pl * PLANE + tt * 16 * CS + 64 * t);
      int tp = 0;
#pragma unroll
      for (int a = 0; a < T; ++a)
#pragma unroll
        for (int b = a; b < T; ++b) {
          f32x4 d = {0.f, 0.f, 0.f, 0.f};
          if constexpr (ES == 2) {
            d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(op[0][a], op[0][b], d, 0, 0, 0);
          } else {
            // pieces 0 = h, 1 = m, 2 = l; smallest products first
            d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(op[2][a], op[0][b], d, 0, 0, 0);
            d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(op[0][a], op[2][b], d, 0, 0, 0);
            d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(op[1][a], op[1][b], d, 0, 0, 0);
            d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(op[1][a], op[0][b], d, 0, 0, 0);
            d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(op[0][a], op[1][b], d, 0, 0, 0);
            d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(op[0][a], op[0][b], d, 0, 0, 0);
          }
#pragma unroll
          for (int r = 0; r < 4; ++r) acc[tp][r] += (double)d[r];
          ++tp;
        }
    }
  }

  // Register r of lane (q4, c16) is entry (4 q4 + r, c16) of the block; the partial Gram
  // leaves the kernel in the order the reduction kernel reads (entry e of a block = row
  // 4 (e / 64) + (e % 64) / 16, column e % 16).  The workgroup's wavefronts add up in wave
  // order through LDS (the tiles are dead now).
  __syncthreads();
  double* red = reinterpret_cast<double*>(lds_all);   // WAVES * 256 doubles <= 32 KiB
  double* dst = partials + (int64_t)blockIdx.x * NTP * 256;
#pragma unroll
  for (int tp = 0; tp < NTP; ++tp) {
#pragma unroll
    for (int r = 0; r < 4; ++r) red[wave * 256 + q4 * 64 + r * 16 + c16] = acc[tp][r];
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

// (T, element size) -> (columns per load, wavefronts per compute unit)
#define FA_GRAM_LP_TILINGS(X)                                              \
  X(1, 4, 2, 16) X(2, 4, 2, 16) X(3, 4, 2, 8) X(4, 4, 2, 8)                \
  X(2, 8, 4, 8) X(3, 8, 4, 8) X(4, 8, 4, 8)

template <int T, int CPL, int ES, int WAVES>
static constexpr size_t lp_lds_bytes() {
  constexpr int R = (64 / CPL) * (16 / ES);
  constexpr size_t need = (size_t)WAVES * (ES == 4 ? 3 : 1) * T * 16 * (R * 2 + 16);
  static_assert(need <= 160 * 1024, "LDS tiles of one workgroup must fit a compute unit");
  // more than half of the 160 KiB: no second workgroup fits beside this one
  return need > 84 * 1024 ? need : 84 * 1024;
}

hipError_t fa_gram_lp_prepare(void) {
  hipError_t e = hipSuccess;
#define FA_X(t, cpl, es, w)                                                                     \
  if (e == hipSuccess)                                                                          \
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(fa_gram_lp_kernel<t, cpl, es, w>),    \
                            hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
  FA_GRAM_LP_TILINGS(FA_X)
#undef FA_X
  return e;
}

bool fa_gram_lp_applies(int p, int dtype) {
  return dtype == FA_BF16 || p > 16;
}

hipError_t fa_launch_gram_lp_partials(const void* G, int64_t ldg, int p, int64_t n, int dtype,
                                      int max_blocks, double* partials, int* nparts,
                                      hipStream_t st, const fa_ktime* tm) {
  const int Tn = (p + 15) / 16, es = dtype == FA_F32 ? 4 : 2;
#define FA_X(t, cpl, esz, w)                                                                    \
  if (Tn == t && es == esz) {                                                                   \
    static_assert(w <= FA_GRAM_WAVES_PER_CU, "partials buffer is sized for this many");         \
    constexpr int R = (64 / cpl) * (16 / esz);                                                  \
    const int64_t ntiles = (n + R - 1) / R;                                                     \
    int64_t wgs = (ntiles + w - 1) / w;                                                         \
    if (wgs > max_blocks) wgs = max_blocks;                                                     \
    *nparts = (int)wgs;                                                                         \
    FA_LAUNCH(tm, (fa_gram_lp_kernel<t, cpl, esz, w>), dim3((unsigned)wgs), dim3(64 * w),       \
              (lp_lds_bytes<t, cpl, esz, w>()), st, (const unsigned char*)G, ldg, p, n, ntiles,  \
              partials);                                                                        \
    return hipGetLastError();                                                                   \
  }
  FA_GRAM_LP_TILINGS(FA_X)
#undef FA_X
  return hipErrorInvalidValue;
}
