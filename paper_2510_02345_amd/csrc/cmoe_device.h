// Device-side building blocks shared by the matrix-core kernels.
#pragma once

#include "cmoe_internal.h"

namespace {

__device__ __forceinline__ float16v mfma16(half8 a, half8 b, float16v c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
}

// GELU(u) = u * Phi(u) in the erf form, Phi(u) = 1/2 + erf(u / sqrt 2) / 2.  On |u| <= 4
// Phi(u) - 1/2 = u P(u^2) with an eight-coefficient minimax polynomial (absolute error
// of Phi below 5.5e-5 over the reals once u is clamped to [-4, 4], far below the FP16
// rounding of the result); eleven full-rate FP32 operations per element.
__device__ __forceinline__ float gelu_erf(float u) {
  const float uc = fminf(fmaxf(u, -4.0f), 4.0f);
  const float t = uc * uc;
  float p = fmaf(t, -1.580786058e-09f, 1.217110963e-07f);
  p = fmaf(t, p, -4.100866136e-06f);
  p = fmaf(t, p, 8.066739247e-05f);
  p = fmaf(t, p, -1.048204373e-03f);
  p = fmaf(t, p, 9.664873593e-03f);
  p = fmaf(t, p, -6.617537886e-02f);
  p = fmaf(t, p, 3.988475204e-01f);
  return u * fmaf(uc, p, 0.5f);
}

__device__ __forceinline__ half4 to_half4(const float16v& a, int qd) {
  half4 o;
  o[0] = (half_t)a[4 * qd + 0];
  o[1] = (half_t)a[4 * qd + 1];
  o[2] = (half_t)a[4 * qd + 2];
  o[3] = (half_t)a[4 * qd + 3];
  return o;
}


// The per-(token, selected expert) part of the fused up-projection (Sec. 3.2), on one
// 32x32 accumulator block hb = (W1_base x)^T: rows n of d_ff, columns = tokens, so a lane
// owns one token (column lane % 32) and 16 rows.
//   h_j = hb + U1cat^T t1ext_j   t1ext_j = the token's t1_j at the rank rows of expert
//                                e_j, zero elsewhere; contraction over the cluster's
//                                K*r rank rows in chunks of 16, chunks no token of the
//                                block needs are skipped
//   a_j = GELU(h_j),  o = sum_j g_j a_j
//   s_j += V2 a_j                the a_j block is fed back as B operand (contraction over
//                                the block's 32 rows n); the product runs over "passes"
//                                of 32 rank rows (32/r experts), a lane contributes to a
//                                pass only if its expert lies in it, so afterwards row
//                                (e_j % (32/r))*r + rho of the accumulator is s_j[rho]
template <int R, int KMAX>
struct FusedUp {
  static constexpr int EPB = 32 / R;  // experts per 32 rank rows
  static constexpr int NF = (R == 32) ? 2 : 1;

  struct Tok {
    int e[KMAX];          // selected experts, local to the cluster
    float g[KMAX];        // gates (0 for a padding column)
    half8 f[KMAX][NF];    // this lane's slice of t1_j
    int p;                // sorted row
    bool valid;
  };

  __device__ static __forceinline__ void load_tok(Tok& t, int p, int m_end, int c, int K, int k, const int* perm,
                                                  const int* expert_idx, const float* gate, const half_t* t1,
                                                  int h) {
    t.p = p;
    t.valid = p < m_end;
    const int pc = t.valid ? p : m_end - 1;
    const int tok = perm[pc];
#pragma unroll
    for (int j = 0; j < KMAX; ++j) {
      t.e[j] = 0;
      t.g[j] = 0.f;
#pragma unroll
      for (int i = 0; i < NF; ++i) t.f[j][i] = half8{0, 0, 0, 0, 0, 0, 0, 0};
      if (j < k) {
        t.e[j] = min(max(expert_idx[(size_t)tok * k + j] - c * K, 0), K - 1);
        t.g[j] = t.valid ? gate[(size_t)tok * k + j] : 0.f;
        const half_t* tr = t1 + ((size_t)pc * k + j) * R;
        if (R == 32) {
          t.f[j][0] = *(const half8*)(tr + 8 * h);
          t.f[j][NF - 1] = *(const half8*)(tr + 16 + 8 * h);
        } else if (R == 16) {
          t.f[j][0] = *(const half8*)(tr + 8 * h);
        } else if (R == 8) {
          t.f[j][0] = *(const half8*)(tr);
        } else {
          half4 q4 = *(const half4*)(tr);
          t.f[j][0][0] = q4[0]; t.f[j][0][1] = q4[1]; t.f[j][0][2] = q4[2]; t.f[j][0][3] = q4[3];
        }
      }
    }
  }

  __device__ static __forceinline__ bool chunk_has(int e, int kc) {
    return R == 32 ? (e == (kc >> 1)) : R == 16 ? (e == kc) : R == 8 ? ((e >> 1) == kc) : ((e >> 2) == kc);
  }
  // B operand of chunk kc for a lane whose token selected expert e with t1 fragments f
  __device__ static __forceinline__ half8 t1_frag(int e, int kc, int h, const half8 (&f)[NF]) {
    const half8 z = {0, 0, 0, 0, 0, 0, 0, 0};
    if (R == 32) return (e == (kc >> 1)) ? ((kc & 1) ? f[NF - 1] : f[0]) : z;
    if (R == 16) return (e == kc) ? f[0] : z;
    if (R == 8) return (e == 2 * kc + h) ? f[0] : z;
    half8 o = z;  // R == 4: slots 0..3 are expert 4kc+2h, slots 4..7 expert 4kc+2h+1
    if (e == 4 * kc + 2 * h) {
      o[0] = f[0][0]; o[1] = f[0][1]; o[2] = f[0][2]; o[3] = f[0][3];
    } else if (e == 4 * kc + 2 * h + 1) {
      o[4] = f[0][0]; o[5] = f[0][1]; o[6] = f[0][2]; o[7] = f[0][3];
    }
    return o;
  }

  // uf(kc): A operand of U1cat^T for rank chunk kc (8 consecutive kk at row n = lane % 32);
  // vf(q, s): A operand of V2 for pass q, rows n 16 s .. 16 s + 15 of the block in the
  // lane order of the accumulator.
  template <class UF, class VF>
  __device__ static __forceinline__ void block(const float16v& hb, const Tok& t, int k, int n_chunks, int n_pass,
                                               int h, UF uf, VF vf, float16v& o, float16v (&sacc)[KMAX]) {
#pragma unroll
    for (int v = 0; v < 16; ++v) o[v] = 0.f;
#pragma unroll
    for (int j = 0; j < KMAX; ++j) {
      if (j >= k) continue;
      const int ej = t.e[j];
      float16v hj = hb;
      for (int kc = 0; kc < n_chunks; ++kc) {
        if (__ballot(t.valid && chunk_has(ej, kc)) == 0ull) continue;
        hj = mfma16(uf(kc), t1_frag(ej, kc, h, t.f[j]), hj);
      }
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        hj[v] = gelu_erf(hj[v]);
        o[v] = fmaf(t.g[j], hj[v], o[v]);
      }
      for (int q = 0; q < n_pass; ++q) {
        const bool on = t.valid && (ej / EPB == q);
        if (__ballot(on) == 0ull) continue;
#pragma unroll
        for (int s = 0; s < 2; ++s) {
          half8 fb;
#pragma unroll
          for (int i = 0; i < 8; ++i) fb[i] = on ? (half_t)hj[8 * s + i] : (half_t)0.f;
          sacc[j] = mfma16(vf(q, s), fb, sacc[j]);
        }
      }
    }
  }

  // The lane holds rows 8*qd + 4h + (0..3) of the pass accumulator; those inside
  // [b_e*R, b_e*R + R) are the token's s_j.  dst_tile: [T][k][R] partial of this row tile
  // (FP32, or FP16 where many partials are summed afterwards in FP32).
  template <class ST>
  __device__ static __forceinline__ void store_s(const Tok& t, const float16v (&sacc)[KMAX], ST* dst_tile, int k,
                                                 int h) {
    if (!t.valid) return;
#pragma unroll
    for (int j = 0; j < KMAX; ++j) {
      if (j >= k) continue;
      const int be = (t.e[j] % EPB) * R;
      ST* dst = dst_tile + ((size_t)t.p * k + j) * R;
#pragma unroll
      for (int qd = 0; qd < 4; ++qd) {
        int row0 = 8 * qd + 4 * h;
        if (row0 >= be && row0 < be + R) {
          if constexpr (sizeof(ST) == 2) {
            *(half4*)(dst + row0 - be) = half4{(half_t)sacc[j][4 * qd], (half_t)sacc[j][4 * qd + 1],
                                               (half_t)sacc[j][4 * qd + 2], (half_t)sacc[j][4 * qd + 3]};
          } else {
            float4v v4 = {sacc[j][4 * qd], sacc[j][4 * qd + 1], sacc[j][4 * qd + 2], sacc[j][4 * qd + 3]};
            *(float4v*)(dst + row0 - be) = v4;
          }
        }
      }
    }
  }
};

}  // namespace
