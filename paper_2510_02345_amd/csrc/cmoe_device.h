// Device-side building blocks shared by the matrix-core kernels.
#pragma once

#include "cmoe_internal.h"

namespace {

__device__ __forceinline__ float16v mfma16(half8 a, half8 b, float16v c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
}

// GELU(u) = u * Phi(u) in the erf form, Phi(u) = 1/2 + erf(u / sqrt 2) / 2.  On |u| <= 3.75
// Phi(u) - 1/2 = u P(u^2) with a seven-coefficient minimax polynomial (|dPhi| < 5.8e-5, GELU
// to 1.95e-4 absolute, 4e-5 RMS under a unit Gaussian: below the FP16 rounding of the
// result).  Beyond the range Phi is held at its value at the end of it, and the factor u at
// -3.75 on the negative side, so the error does not grow with |u|: relative 8.8e-5 for
// large positive u, -3.3e-4 absolute (instead of -0) for large negative u; NaN in, NaN out.
// Twelve full-rate FP32 operations per element.
__device__ __forceinline__ float gelu_erf(float u) {
  const float uc = __builtin_amdgcn_fmed3f(u, -3.75f, 3.75f);
  // max(u, -3.75) as a select, so that a NaN pre-activation stays a NaN in the result
  const float um = u < -3.75f ? -3.75f : u;
  const float t = uc * uc;
  float p = fmaf(t, 3.878059656e-08f, -2.362032659e-06f);
  p = fmaf(t, p, 6.212595828e-05f);
  p = fmaf(t, p, -9.425636946e-04f);
  p = fmaf(t, p, 9.357058592e-03f);
  p = fmaf(t, p, -6.578237312e-02f);
  p = fmaf(t, p, 3.987038812e-01f);
  return um * fmaf(uc, p, 0.5f);
}

__device__ __forceinline__ half4 to_half4(const float16v& a, int qd) {
  half4 o;
  o[0] = (half_t)a[4 * qd + 0];
  o[1] = (half_t)a[4 * qd + 1];
  o[2] = (half_t)a[4 * qd + 2];
  o[3] = (half_t)a[4 * qd + 3];
  return o;
}


// ---------------------------------------------------------------- 16 x 16 x 32 blocks
// The grouped products run on v_mfma_f32_16x16x32_f16: D (16 rows x 16 tokens, FP32) +=
// A (16 weight rows x 32 contraction elements) * B (32 x 16 tokens).  Lane l supplies row
// (or token) l % 16 and the eight contraction elements 8q .. 8q + 7, q = l / 16, and holds of
// D the token l % 16 and the rows 4q .. 4q + 3.  Measured on this part, the instruction
// sustains about 14 % more flops than the 32 x 32 x 16 form at the same board power (it moves
// half the accumulator bytes per flop), and board power is what limits the products.
//
// Weight rows are taken in "pair blocks" of 32 consecutive rows = two MFMA blocks.  Row i of
// block hh (0 or 1) of a pair block is the weight row 8 (i / 4) + 4 hh + i % 4 of the pair
// block, so that a lane's 4 + 4 accumulators of the two blocks are the EIGHT CONSECUTIVE rows
// 8q .. 8q + 7: a lane stores 16 contiguous bytes of FP16 output per token, four lanes a
// token's 64-byte line, and an accumulator pair is a ready-made B operand (contraction
// positions in natural order) for a further product.
__device__ __forceinline__ float4v mfma32(half8 a, half8 b, float4v c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}

// Weight row (offset inside its 32-row pair block kept in the upper bits) held by tile row rho
// of an LDS operand tile whose rows are stored in MFMA order: rho = 32 P + 16 hh + i.
__device__ __forceinline__ int pi_row(int rho) {
  return (rho & ~31) | ((rho & 12) << 1) | ((rho & 16) >> 2) | (rho & 3);
}

// Position (XOR mask over the four 16-byte chunks of a 64-byte operand-tile row) at which
// tile row `row` keeps its chunks.  A 16x16x32 fragment read has lane l fetch 16 bytes of row
// l % 16, chunk l / 16; the LDS serves such a read in groups of sixteen lanes
// {0-3, 12-15, 20-23, 24-27} and {4-7, 8-11, 16-19, 28-31} (and the same plus 32), so the
// four row quads of one group need four different chunk positions: quads 0,1,2,3 use
// masks 0,3,2,1.  Measured on gfx950: the plain mask (row >> 2) & 3 serves a 32-row fragment
// read without conflicts but gives two-way conflicts on every 16-row read.
__device__ __forceinline__ int swz(int row) { return ((row >> 2) & 3) ^ ((row >> 1) & 2); }

__device__ __forceinline__ half8 pack_half8(const float4v& lo, const float4v& hi) {
  half8 o;
  o[0] = (half_t)lo[0]; o[1] = (half_t)lo[1]; o[2] = (half_t)lo[2]; o[3] = (half_t)lo[3];
  o[4] = (half_t)hi[0]; o[5] = (half_t)hi[1]; o[6] = (half_t)hi[2]; o[7] = (half_t)hi[3];
  return o;
}

// The per-(token, selected expert) part of the fused up-projection (Sec. 3.2) on one pair
// block of the accumulators hb = (W1_base x)^T: 32 rows n of d_ff x 16 tokens; a lane owns
// one token (l % 16) and the eight rows 8q .. 8q + 7.
//   h_j = hb + U1cat^T t1ext_j   t1ext_j = the token's t1_j at the rank rows of expert
//                                e_j, zero elsewhere; contraction over the cluster's
//                                K*r rank rows in chunks of 32, chunks no token of the
//                                block needs are skipped
//   a_j = GELU(h_j),  o = sum_j g_j a_j
//   s_j += V2 a_j                the a_j pair block is fed back as B operand (contraction
//                                over its 32 rows n); the product runs over "passes" of
//                                16 rank rows, a lane contributes to a pass only if its
//                                expert's rows lie in it
template <int R, int KMAX>
struct FusedUp {
  static constexpr int NSP = (R == 32) ? 2 : 1;  // 16-row passes per expert

  struct Tok {
    int e[KMAX];      // selected experts, local to the cluster
    float g[KMAX];    // gates (0 for a padding column)
    half8 f[KMAX];    // this lane's slice of t1_j (see t1_frag)
    int p;            // sorted row
    bool valid;
  };

  __device__ static __forceinline__ void load_tok(Tok& t, int p, int m_end, int c, int K, int k, const int* perm,
                                                  const int* expert_idx, const float* gate, const half_t* t1,
                                                  int q) {
    t.p = p;
    t.valid = p < m_end;
    const int pc = t.valid ? p : m_end - 1;
    const int tok = perm[pc];
#pragma unroll
    for (int j = 0; j < KMAX; ++j) {
      t.e[j] = 0;
      t.g[j] = 0.f;
      t.f[j] = half8{0, 0, 0, 0, 0, 0, 0, 0};
      if (j < k) {
        t.e[j] = min(max(expert_idx[(size_t)tok * k + j] - c * K, 0), K - 1);
        t.g[j] = t.valid ? gate[(size_t)tok * k + j] : 0.f;
        const half_t* tr = t1 + ((size_t)pc * k + j) * R;
        if (R == 32) {
          t.f[j] = *(const half8*)(tr + 8 * q);
        } else if (R == 16) {
          t.f[j] = *(const half8*)(tr + 8 * (q & 1));
        } else if (R == 8) {
          t.f[j] = *(const half8*)(tr);
        } else {
          const half4 q4 = *(const half4*)(tr);
          t.f[j][0] = q4[0]; t.f[j][1] = q4[1]; t.f[j][2] = q4[2]; t.f[j][3] = q4[3];
        }
      }
    }
  }

  // chunk of 32 rank rows that holds expert e
  __device__ static __forceinline__ int chunk_of(int e) { return (e * R) >> 5; }
  // B operand of chunk c for a lane (contraction elements 32 c + 8 q ..) whose token selected
  // expert e and keeps the slice f of its t1
  __device__ static __forceinline__ half8 t1_frag(int e, int c, int q, const half8& f) {
    const half8 z = {0, 0, 0, 0, 0, 0, 0, 0};
    if (R == 32) return (e == c) ? f : z;
    if (R == 16) return (e == 2 * c + (q >> 1)) ? f : z;
    if (R == 8) return (e == 4 * c + q) ? f : z;
    half8 o = z;  // R == 4: elements 0..3 belong to expert 8c + 2q, elements 4..7 to expert 8c + 2q + 1
    if (e == 8 * c + 2 * q) {
      o[0] = f[0]; o[1] = f[1]; o[2] = f[2]; o[3] = f[3];
    } else if (e == 8 * c + 2 * q + 1) {
      o[4] = f[0]; o[5] = f[1]; o[6] = f[2]; o[7] = f[3];
    }
    return o;
  }

  // Chunks of 32 rank rows and passes of 16 rank rows that at least one valid token of the
  // 16-token block needs for its j-th expert (wavefront-uniform bit masks, taken once per
  // token block).
  struct Need {
    unsigned chunks[KMAX], passes[KMAX];
  };
  __device__ static __forceinline__ void need_of(const Tok& t, int k, int n_chunks, int n_pass, Need& nd) {
#pragma unroll
    for (int j = 0; j < KMAX; ++j) {
      nd.chunks[j] = 0u;
      nd.passes[j] = 0u;
      if (j >= k) continue;
      for (int c = 0; c < n_chunks; ++c)
        if (__ballot(t.valid && chunk_of(t.e[j]) == c) != 0ull) nd.chunks[j] |= 1u << c;
      for (int pp = 0; pp < n_pass; ++pp)
        if (__ballot(t.valid && (pp & ~(NSP - 1)) == ((t.e[j] * R) >> 4)) != 0ull) nd.passes[j] |= 1u << pp;
    }
  }

  // uf(c, hh): A operand of U1cat^T for rank chunk c and block hh of the pair block;
  // vf(pp): A operand of V2 for pass pp (rank rows 16 pp + l % 16, the pair block's rows
  // 8q .. 8q + 7 as contraction elements).
  template <class UF, class VF>
  __device__ static __forceinline__ void pair_block(const float4v& hb0, const float4v& hb1, const Tok& t,
                                                    const Need& nd, int k, int q, UF uf, VF vf, float (&o)[8],
                                                    float4v (&sacc)[KMAX][NSP]) {
#pragma unroll
    for (int j = 0; j < KMAX; ++j) {
      if (j >= k) {
        if (j == 0) {   // k >= 1 always; keeps o defined for the compiler
#pragma unroll
          for (int i = 0; i < 8; ++i) o[i] = 0.f;
        }
        continue;
      }
      const int ej = t.e[j];
      float4v h0 = hb0, h1 = hb1;
      for (unsigned m = nd.chunks[j]; m != 0u; m &= m - 1u) {
        const int c = __builtin_ctz(m);
        const half8 fb = t1_frag(ej, c, q, t.f[j]);
        h0 = mfma32(uf(c, 0), fb, h0);
        h1 = mfma32(uf(c, 1), fb, h1);
      }
      float a[8];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        a[i] = gelu_erf(h0[i]);
        a[4 + i] = gelu_erf(h1[i]);
      }
      half8 ab;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        o[i] = j == 0 ? t.g[0] * a[i] : fmaf(t.g[j], a[i], o[i]);
        ab[i] = (half_t)a[i];
      }
      const int p0 = (ej * R) >> 4;   // first pass of the expert's rank rows
      for (unsigned m = nd.passes[j]; m != 0u; m &= m - 1u) {
        const int pp = __builtin_ctz(m);
        const bool on = t.valid && (pp & ~(NSP - 1)) == p0;
        const half8 z = {0, 0, 0, 0, 0, 0, 0, 0};
        sacc[j][pp & (NSP - 1)] = mfma32(vf(pp), on ? ab : z, sacc[j][pp & (NSP - 1)]);
      }
    }
  }

  // The lane holds rank rows 4q .. 4q + 3 of each pass accumulator; those inside the expert's
  // rows are the token's s_j.  dst_tile: [T][k][R] FP32 partial of this row tile.
  __device__ static __forceinline__ void store_s(const Tok& t, const float4v (&sacc)[KMAX][NSP], float* dst_tile,
                                                 int k, int q) {
    if (!t.valid) return;
#pragma unroll
    for (int j = 0; j < KMAX; ++j) {
      if (j >= k) continue;
      const int be = (t.e[j] * R) & 15;   // first row of the expert inside its pass
      float* dst = dst_tile + ((size_t)t.p * k + j) * R;
      const int row0 = 4 * q;
      if (row0 >= be && row0 < be + (R < 16 ? R : 16)) {
#pragma unroll
        for (int s = 0; s < NSP; ++s) *(float4v*)(dst + 16 * s + row0 - be) = sacc[j][s];
      }
    }
  }
};

}  // namespace
