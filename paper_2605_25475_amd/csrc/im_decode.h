// Fused decode step: the whole path for one new token per sequence in two launches.
//   k_dec_prep : query-side indexer features (U_q, G GEMVs + QK-Norm), append of the new
//                (k, v), its indexer key.
//   k_dec_main : per (unit, 128-key split) workgroups score their keys, find their local
//                eviction candidate and accumulate softmax-attention partials without it;
//                one tail workgroup per unit prepares the memory readout meanwhile, then waits
//                for its splits, picks the evicted entry, folds it into the memory state,
//                merges the partials, fills the hole and writes the output.
// Same results as append -> index_score (n_q = 1) -> topb_select -> memory_update -> compact_kv
// -> decode_attn_with_readout whenever every unit enters with len <= budget.
#pragma once
#include "im_device.h"

#define DEC_KEYS 128                 // keys per split workgroup (8 MFMA tiles of 16)
#define DEC_REC (IM_D + 2)           // partial record per (unit, split, head): max, denom, 128 numerators
#define DEC_GMAX 8                   // query heads per KV head supported
#define DEC_CAND 16                  // words per candidate record
#define DEC_SPIN_LIMIT (1 << 20)

#define IM_STATUS_APPEND_OVERFLOW_BIT 1
#define IM_STATUS_LIVE_EXCEEDED_BIT 2
#define IM_STATUS_WAIT_TIMEOUT_BIT 4
#define IM_STATUS_OVER_BUDGET_BIT 8

typedef short v4s __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));

struct DecArgs {
  // state
  bf16_t *K, *V, *Kidx;
  int32_t *pos, *len, *nproj;
  float *M, *bvec;
  // slow weights
  const bf16_t *Uq, *Gw, *Uk, *nqw, *nkw, *Wt, *wg;
  float cg;
  // inputs
  const bf16_t *q, *xg, *k_new, *v_new;
  const int32_t *pos_new, *q_pos;
  // outputs
  bf16_t* out;
  float* readout;
  float* scores;      // optional
  int32_t* evicted;   // optional
  // workspace
  double *qy, *alpha;
  int32_t *cnt_head, *cnt_unit, *status, *maxpos;
  float* part;
  uint32_t* cand;
  // scalars
  int B, H, H_kv, C, H_idx, gate_in, n_sink, n_recent, budget, S, S_alloc, max_live, r_first;
  float rms_eps, mem_eps, scale, lambda, eta;
};

__device__ __forceinline__ void unpack8(const uint4& u, float* f) {
  f[0] = bf_lo(u.x); f[1] = bf_hi(u.x); f[2] = bf_lo(u.y); f[3] = bf_hi(u.y);
  f[4] = bf_lo(u.z); f[5] = bf_hi(u.z); f[6] = bf_lo(u.w); f[7] = bf_hi(u.w);
}

// --------------------------------------------------------------------------------------------
// k_dec_prep.  Blocks [0, nU): two rows of U_q each, all batch rows; the last block of an
// indexer head to finish normalises that head.  Blocks [nU, nU + nG): two rows of G.
// Blocks after: one per unit, append + indexer key of the new token.
// --------------------------------------------------------------------------------------------
__device__ void dec_gemv2(const bf16_t* __restrict__ A, const bf16_t* __restrict__ Bm, int n0, int N,
                          int M, int Kd, double (*red)[16], double* out_rows /* [M][2] in LDS */) {
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  for (int mb = 0; mb < M; mb += 8) {
    double acc[8][2];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i][0] = acc[i][1] = 0.0;
    for (int k = tid * 8; k < Kd; k += 256 * 8) {
      float bv[2][8];
#pragma unroll
      for (int r = 0; r < 2; ++r) {
        uint4 u = make_uint4(0, 0, 0, 0);
        if (n0 + r < N) u = *(const uint4*)(Bm + (size_t)(n0 + r) * Kd + k);
        unpack8(u, bv[r]);
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        if (mb + i < M) {
          const uint4 u = *(const uint4*)(A + (size_t)(mb + i) * Kd + k);
          float av[8];
          unpack8(u, av);
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            acc[i][0] = fma((double)av[e], (double)bv[0][e], acc[i][0]);
            acc[i][1] = fma((double)av[e], (double)bv[1][e], acc[i][1]);
          }
        }
      }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      acc[i][0] = wave_sum_d(acc[i][0]);
      acc[i][1] = wave_sum_d(acc[i][1]);
    }
    __syncthreads();
    if (lane == 0) {
#pragma unroll
      for (int i = 0; i < 8; ++i) { red[w][2 * i] = acc[i][0]; red[w][2 * i + 1] = acc[i][1]; }
    }
    __syncthreads();
    if (tid < 16 && mb + (tid >> 1) < M)
      out_rows[(mb + (tid >> 1)) * 2 + (tid & 1)] = red[0][tid] + red[1][tid] + red[2][tid] + red[3][tid];
  }
  __syncthreads();
}

__global__ __launch_bounds__(256) void k_dec_prep(const DecArgs a) {
  __shared__ double red[4][16];
  __shared__ double rows[64 * 2];   // up to 64 batch rows x 2 outputs
  __shared__ int s_last;
  __shared__ float s_k[IM_D];
  __shared__ double s_u[IM_DI];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int Nq = a.H_idx * IM_DI;
  const int nU = Nq / 2, nG = (a.H_idx + 1) / 2;
  const int blk = blockIdx.x;
  if (blk < nU) {
    const int n0 = blk * 2;
    dec_gemv2(a.q, a.Uq, n0, Nq, a.B, a.H * IM_D, red, rows);
    for (int i = tid; i < a.B * 2; i += 256) a.qy[(size_t)(i >> 1) * Nq + n0 + (i & 1)] = rows[i];
    __threadfence();
    __syncthreads();
    const int head = n0 / IM_DI;
    if (tid == 0) {
      const int old = __hip_atomic_fetch_add(a.cnt_head + head, 1, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
      s_last = (old == IM_DI / 2 - 1);
    }
    __syncthreads();
    if (s_last) {  // every row of this head is in memory: QK-Norm for all batch rows
      __threadfence();
      for (int b = w; b < a.B; b += 4) {
        double* y = a.qy + (size_t)b * Nq + head * IM_DI;
        const double v = __hip_atomic_load(y + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const double ss = wave_sum_d(v * v);
        const double rr = sqrt(ss / (double)IM_DI + (double)a.rms_eps);
        const double wt = a.nqw ? (double)bf2f(a.nqw[lane]) : 1.0;
        y[lane] = (double)(float)(v / rr * wt);
      }
      if (tid == 0) a.cnt_head[head] = 0;
    }
    return;
  }
  if (blk < nU + nG) {
    const int n0 = (blk - nU) * 2;
    dec_gemv2(a.xg, a.Gw, n0, a.H_idx, a.B, a.gate_in, red, rows);
    const double denom = sqrt((double)(a.H_idx * IM_DI));
    for (int i = tid; i < a.B * 2; i += 256) {
      const int r = n0 + (i & 1);
      if (r < a.H_idx) a.alpha[(size_t)(i >> 1) * a.H_idx + r] = (double)(float)(rows[i] / denom);
    }
    return;
  }
  // ---- unit block: append the new (k, v, pos) at slot len, compute its indexer key
  const int u = blk - nU - nG;
  const int b = u / a.H_kv;
  const int n_old = a.len[u];
  if (a.n_recent > 0) {  // newest position of the unit (new token included) for the recent window
    int m = INT_MIN;
    const int nn = min(n_old, a.max_live);
    for (int i = tid; i < nn; i += 256) m = max(m, a.pos[(size_t)u * a.C + i]);
    if (n_old + 1 <= a.C) m = max(m, a.pos_new[b]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) m = max(m, __shfl_xor(m, o, 64));
    __shared__ int s_mp[4];
    if (lane == 0) s_mp[w] = m;
    __syncthreads();
    if (tid == 0) a.maxpos[u] = max(max(s_mp[0], s_mp[1]), max(s_mp[2], s_mp[3]));
  }
  if (n_old + 1 > a.C) {
    if (tid == 0) atomicOr(a.status, IM_STATUS_APPEND_OVERFLOW_BIT);
    return;
  }
  if (n_old + 1 > a.max_live && tid == 0) atomicOr(a.status, IM_STATUS_LIVE_EXCEEDED_BIT);
  const size_t slot = (size_t)u * a.C + n_old;
  if (tid < 16) {
    const uint4 kk = *(const uint4*)(a.k_new + (size_t)u * IM_D + tid * 8);
    *(uint4*)(a.K + slot * IM_D + tid * 8) = kk;
    float f[8];
    unpack8(kk, f);
#pragma unroll
    for (int e = 0; e < 8; ++e) s_k[tid * 8 + e] = f[e];
  } else if (tid < 32) {
    const int t = tid - 16;
    *(uint4*)(a.V + slot * IM_D + t * 8) = *(const uint4*)(a.v_new + (size_t)u * IM_D + t * 8);
  } else if (tid == 32) {
    a.pos[slot] = a.pos_new[b];
  }
  __syncthreads();
  {  // u_c = Uk[c] . k : thread (c = tid/4, quarter = tid%4)
    const int c = tid >> 2, qd = tid & 3;
    const uint4* ur = (const uint4*)(a.Uk + c * IM_D + qd * 32);
    double acc = 0.0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float f[8];
      unpack8(ur[i], f);
#pragma unroll
      for (int e = 0; e < 8; ++e) acc = fma((double)f[e], (double)s_k[qd * 32 + i * 8 + e], acc);
    }
    acc += __shfl_xor(acc, 1, 64);
    acc += __shfl_xor(acc, 2, 64);
    if (qd == 0) s_u[c] = acc;
  }
  __syncthreads();
  if (tid < 64) {
    const double v = s_u[tid];
    const double ss = wave_sum_d(v * v);
    const double rr = sqrt(ss / (double)IM_DI + (double)a.rms_eps);
    const double wt = a.nkw ? (double)bf2f(a.nkw[tid]) : 1.0;
    a.Kidx[slot * IM_DI + tid] = d2bf_rne(v / rr * wt);
  }
}

// --------------------------------------------------------------------------------------------
// k_dec_main
// --------------------------------------------------------------------------------------------
struct DecSplitSmem {
  bf16_t ks[DEC_KEYS][72];           // indexer keys of the split, row stride 144 B
  double pa[DEC_KEYS];               // second half of the heads' gated sum
  float pl[DEC_KEYS][8];             // logits, then probabilities, [key][head]
  float oacc[4][DEC_GMAX][IM_D];     // per-wave output partials
  float wm[4][8], wl[4][8];
  float clog[8];
  unsigned long long c64[2];
  int cslot[2];
};

struct DecTailSmem {
  float qs[DEC_GMAX][IM_D];
  float php[2][DEC_GMAX][IM_DM];
  float phq[DEC_GMAX][IM_DM];
  float red[4][DEC_GMAX][IM_D];
  float rold[DEC_GMAX][IM_D];
  float ke[IM_D], ve[IM_D], phe2[2][IM_DM], phe[IM_DM], bnew[IM_DM];
  float gate[DEC_GMAX], den[DEC_GMAX], dot[DEC_GMAX];
  unsigned long long c64[4];
  int cidx[4];
  int e_slot, e_split, timeout;
};

template <int G>
__device__ __forceinline__ void dec_split(const DecArgs& a, const int u, const int s, DecSplitSmem& sm) {
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
  const int b = u / a.H_kv, h = u % a.H_kv;
  const int n_old = a.len[u];
  const int n = min(n_old + ((n_old + 1 <= a.C) ? 1 : 0), a.max_live);
  const int k0 = s * DEC_KEYS;
  const int nk = max(0, min(DEC_KEYS, n - k0));
  uint32_t* crec = a.cand + ((size_t)u * a.S_alloc + s) * DEC_CAND;
  if (nk > 0) {
    const size_t base = (size_t)u * a.C + k0;
    const int l16 = lane & 15, kq = lane >> 4;
    // ---- issue every load of this split up front
    uint4 kst[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int ch = tid + 256 * i, row = ch >> 3, c8 = ch & 7;
      kst[i] = (row < nk) ? *(const uint4*)(a.Kidx + (base + row) * IM_DI + c8 * 8) : make_uint4(0, 0, 0, 0);
    }
    uint4 kf[2][4], vf[2][4], qf[4];
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
      const int T = 2 * w + tt;
      const int kr = 16 * T + l16;
#pragma unroll
      for (int c = 0; c < 4; ++c)
        kf[tt][c] = (kr < nk) ? *(const uint4*)(a.K + (base + kr) * IM_D + 32 * c + 8 * kq) : make_uint4(0, 0, 0, 0);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int vr = 16 * T + 4 * i + kq;
        vf[tt][i] = (vr < nk) ? *(const uint4*)(a.V + (base + vr) * IM_D + 8 * l16) : make_uint4(0, 0, 0, 0);
      }
    }
#pragma unroll
    for (int c = 0; c < 4; ++c)
      qf[c] = (l16 < G) ? *(const uint4*)(a.q + ((size_t)b * a.H + h * G + l16) * IM_D + 32 * c + 8 * kq)
                        : make_uint4(0, 0, 0, 0);
    const int kk = tid & 127, half = tid >> 7;
    const int mypos = (kk < nk) ? a.pos[base + kk] : 0;
    const int qpos = a.q_pos[b];
    // ---- indexer keys to LDS, then one key per thread (two threads share a key, half the heads each)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int ch = tid + 256 * i, row = ch >> 3, c8 = ch & 7;
      *(uint4*)&sm.ks[row][c8 * 8] = kst[i];
    }
    __syncthreads();
    double part = 0.0;
    {
      double kd[IM_DI];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const uint4 v = *(const uint4*)&sm.ks[kk][i * 8];
        float f[8];
        unpack8(v, f);
#pragma unroll
        for (int e = 0; e < 8; ++e) kd[8 * i + e] = (double)f[e];
      }
      const int Hh = (a.H_idx + 1) >> 1;
      const int j0 = half ? Hh : 0, j1 = half ? a.H_idx : Hh;
      const double* __restrict__ qh = a.qy + (size_t)b * a.H_idx * IM_DI;
      const double* __restrict__ al = a.alpha + (size_t)b * a.H_idx;
      for (int j = j0; j < j1; ++j) {
        double z0 = 0.0, z1 = 0.0;
#pragma unroll
        for (int c = 0; c < IM_DI; c += 2) {
          z0 = fma(qh[j * IM_DI + c], kd[c], z0);
          z1 = fma(qh[j * IM_DI + c + 1], kd[c + 1], z1);
        }
        part = fma(al[j], fmax(z0 + z1, 0.0), part);
      }
    }
    if (half) sm.pa[kk] = part;
    __syncthreads();
    // ---- score, forced flag, split-local candidate = the entry ranked last
    if (!half) {
      unsigned long long c64 = ~0ull;
      if (kk < nk) {
        const float sc = (mypos <= qpos) ? (float)(part + sm.pa[kk]) : -INFINITY;
        if (a.scores) a.scores[base + kk] = sc;
        const bool forced = (mypos < a.n_sink) ||
                            (a.n_recent > 0 && (long long)mypos > (long long)a.maxpos[u] - a.n_recent);
        const uint32_t skey = forced ? IM_KEY_PINF : score_key(sc);
        c64 = ((unsigned long long)skey << 32) | (uint32_t)(~((uint32_t)mypos ^ 0x80000000u));
      }
      unsigned long long mn = c64;
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) {
        const unsigned long long other = __shfl_xor(mn, o, 64);
        mn = other < mn ? other : mn;
      }
      // equal (score, position): the largest slot is ranked last
      const unsigned long long bal = __ballot(c64 == mn && kk < nk);
      if (lane == 0) {
        sm.c64[w] = mn;
        sm.cslot[w] = bal ? (w * 64 + 63 - __builtin_clzll(bal)) : -1;
      }
    }
    __syncthreads();
    int cl;  // candidate's key index inside the split
    unsigned long long cbest;
    {
      const unsigned long long c0 = sm.c64[0], c1 = sm.c64[1];
      const int s0 = sm.cslot[0], s1 = sm.cslot[1];
      if (s1 >= 0 && (s0 < 0 || c1 <= c0)) { cl = s1; cbest = c1; } else { cl = s0; cbest = c0; }
    }
    // ---- logits of the 2 tiles of this wave:  S[key][head] = K_tile . Q^T  (bf16 MFMA, fp32 acc)
    float sreg[2][4];
    float lmax = -INFINITY;
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
      v4f acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const uint4 ka = kf[tt][c], qb = qf[c];
        const v4s a0 = __builtin_bit_cast(v4s, make_uint2(ka.x, ka.y));
        const v4s a1 = __builtin_bit_cast(v4s, make_uint2(ka.z, ka.w));
        const v4s b0 = __builtin_bit_cast(v4s, make_uint2(qb.x, qb.y));
        const v4s b1 = __builtin_bit_cast(v4s, make_uint2(qb.z, qb.w));
        acc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a0, b0, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a1, b1, acc, 0, 0, 0);
      }
      const int T = 2 * w + tt;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int kl = 16 * T + 4 * kq + r;  // this lane: head l16, key kl
        float sv = acc[r] * a.scale;
        if (kl == cl && l16 < G) sm.clog[l16] = sv;
        if (kl >= nk || kl == cl) sv = -INFINITY;
        sreg[tt][r] = sv;
        lmax = fmaxf(lmax, sv);
      }
    }
    lmax = fmaxf(lmax, __shfl_xor(lmax, 16, 64));
    lmax = fmaxf(lmax, __shfl_xor(lmax, 32, 64));
    if (kq == 0 && l16 < 8) sm.wm[w][l16] = lmax;
    __syncthreads();
    float mj = fmaxf(fmaxf(sm.wm[0][l16 & 7], sm.wm[1][l16 & 7]), fmaxf(sm.wm[2][l16 & 7], sm.wm[3][l16 & 7]));
    if (mj == -INFINITY) mj = -1e30f;
    float lsum = 0.f;
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
      const int T = 2 * w + tt;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float p = (sreg[tt][r] == -INFINITY) ? 0.f : __expf(sreg[tt][r] - mj);
        lsum += p;
        if (l16 < 8) sm.pl[16 * T + 4 * kq + r][l16] = p;
      }
    }
    lsum += __shfl_xor(lsum, 16, 64);
    lsum += __shfl_xor(lsum, 32, 64);
    if (kq == 0 && l16 < 8) sm.wl[w][l16] = lsum;
    __syncthreads();
    // ---- O[head][d] += P[head][key] V[key][d]; 16 lanes share a key row (8 dims each)
    float acc[G][8];
#pragma unroll
    for (int j = 0; j < G; ++j)
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[j][e] = 0.f;
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
      const int T = 2 * w + tt;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int kl = 16 * T + 4 * i + kq;
        float pv[8], v[8];
        *(float4*)&pv[0] = *(const float4*)&sm.pl[kl][0];
        if (G > 4) *(float4*)&pv[4] = *(const float4*)&sm.pl[kl][4];
        unpack8(vf[tt][i], v);
#pragma unroll
        for (int j = 0; j < G; ++j)
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[j][e] = fmaf(pv[j], v[e], acc[j][e]);
      }
    }
#pragma unroll
    for (int j = 0; j < G; ++j)
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        float x = acc[j][e];
        x += __shfl_xor(x, 16, 64);
        x += __shfl_xor(x, 32, 64);
        if (kq == 0) sm.oacc[w][j][8 * l16 + e] = x;
      }
    __syncthreads();
    float* prec = a.part + ((size_t)u * a.S_alloc + s) * DEC_GMAX * DEC_REC;
    for (int idx = tid; idx < G * IM_D; idx += 256) {
      const int j = idx >> 7, d = idx & 127;
      prec[j * DEC_REC + 2 + d] = sm.oacc[0][j][d] + sm.oacc[1][j][d] + sm.oacc[2][j][d] + sm.oacc[3][j][d];
      if (d == 0) {
        float m = fmaxf(fmaxf(sm.wm[0][j], sm.wm[1][j]), fmaxf(sm.wm[2][j], sm.wm[3][j]));
        prec[j * DEC_REC] = (m == -INFINITY) ? -1e30f : m;
        prec[j * DEC_REC + 1] = sm.wl[0][j] + sm.wl[1][j] + sm.wl[2][j] + sm.wl[3][j];
      }
    }
    if (tid == 0) {
      crec[0] = (uint32_t)(cbest >> 32);
      crec[1] = (uint32_t)cbest;
      crec[2] = (uint32_t)(k0 + cl);
    }
    if (tid < G) crec[4 + tid] = __float_as_uint(sm.clog[tid]);
  }
  __threadfence();
  __syncthreads();
  if (tid == 0) __hip_atomic_fetch_add(a.cnt_unit + u, 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
}

template <int G>
__device__ __forceinline__ void dec_tail(const DecArgs& a, const int u, DecTailSmem& sm) {
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
  const int b = u / a.H_kv, h = u % a.H_kv;
  const int n_old = a.len[u];
  const bool has_new = n_old + 1 <= a.C;
  const int n = min(n_old + (has_new ? 1 : 0), a.max_live);
  // ---------------- independent of the eviction decision ----------------
  const int d4 = tid & 31, cg = tid >> 5;
  float4 Mr[16];
  float* Mu = a.M + (size_t)u * IM_DM * IM_D;
#pragma unroll
  for (int i = 0; i < 16; ++i) Mr[i] = *(const float4*)(Mu + (cg * 16 + i) * IM_D + 4 * d4);
  const int wc = tid & 127, hh = tid >> 7;
  uint4 Wr[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) Wr[i] = *(const uint4*)(a.Wt + wc * IM_D + hh * 64 + i * 8);
  const float b_old = (tid < IM_DM) ? a.bvec[(size_t)u * IM_DM + tid] : 0.f;
  for (int idx = tid; idx < G * IM_D; idx += 256)
    sm.qs[idx >> 7][idx & 127] = bf2f(a.q[((size_t)b * a.H + h * G) * IM_D + idx]);
  if (tid == 0) sm.timeout = 0;
  __syncthreads();
  {  // phi(q_j)[c], two threads per c (64 dims each)
    float pq[G];
#pragma unroll
    for (int j = 0; j < G; ++j) pq[j] = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      float wv[8];
      unpack8(Wr[i], wv);
#pragma unroll
      for (int e = 0; e < 8; ++e)
#pragma unroll
        for (int j = 0; j < G; ++j) pq[j] = fmaf(wv[e], sm.qs[j][hh * 64 + i * 8 + e], pq[j]);
    }
#pragma unroll
    for (int j = 0; j < G; ++j) sm.php[hh][j][wc] = pq[j];
  }
  __syncthreads();
  for (int idx = tid; idx < G * IM_DM; idx += 256) {
    const int j = idx >> 7, c = idx & 127;
    sm.phq[j][c] = sm.php[0][j][c] + sm.php[1][j][c];
  }
  __syncthreads();
  // gate and the old denominator: one wave per head
  for (int j = w; j < G; j += 4) {
    float gz = bf2f(a.wg[lane]) * sm.qs[j][lane] + bf2f(a.wg[lane + 64]) * sm.qs[j][lane + 64];
    gz = wave_sum_f(gz);
    if (lane == 0) sm.gate[j] = 1.f / (1.f + __expf(-(gz + a.cg)));
  }
  {  // r_old[j][d] = sum_c phi_q[j][c] M[c][d] over this thread's 16 rows and 4 columns
    float ra[G][4];
#pragma unroll
    for (int j = 0; j < G; ++j) ra[j][0] = ra[j][1] = ra[j][2] = ra[j][3] = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
#pragma unroll
      for (int j = 0; j < G; ++j) {
        const float f = sm.phq[j][cg * 16 + i];
        ra[j][0] = fmaf(f, Mr[i].x, ra[j][0]); ra[j][1] = fmaf(f, Mr[i].y, ra[j][1]);
        ra[j][2] = fmaf(f, Mr[i].z, ra[j][2]); ra[j][3] = fmaf(f, Mr[i].w, ra[j][3]);
      }
    }
#pragma unroll
    for (int j = 0; j < G; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float x = ra[j][e];
        x += __shfl_xor(x, 32, 64);
        if (lane < 32) sm.red[w][j][4 * d4 + e] = x;
      }
  }
  __syncthreads();
  for (int idx = tid; idx < G * IM_D; idx += 256) {
    const int j = idx >> 7, d = idx & 127;
    sm.rold[j][d] = sm.red[0][j][d] + sm.red[1][j][d] + sm.red[2][j][d] + sm.red[3][j][d];
  }
  // ---------------- wait for the splits of this unit ----------------
  if (tid == 0) {
    int spins = 0;
    while (__hip_atomic_load(a.cnt_unit + u, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) < a.S) {
      if (++spins > DEC_SPIN_LIMIT) { sm.timeout = 1; break; }
      __builtin_amdgcn_s_sleep(4);
    }
  }
  __syncthreads();
  __threadfence();
  if (sm.timeout && tid == 0) atomicOr(a.status, IM_STATUS_WAIT_TIMEOUT_BIT);
  const int n_act = (n + DEC_KEYS - 1) / DEC_KEYS;
  const uint32_t* cbase = a.cand + (size_t)u * a.S_alloc * DEC_CAND;
  const float* pbase = a.part + (size_t)u * a.S_alloc * DEC_GMAX * DEC_REC;
  // ---------------- the evicted entry: ranked last over all splits ----------------
  const bool evict = n > a.budget;
  if (n > a.budget + 1 && tid == 0) atomicOr(a.status, IM_STATUS_OVER_BUDGET_BIT);
  {
    unsigned long long best = ~0ull;
    int bidx = -1;
    for (int sp = tid; sp < n_act; sp += 256) {
      const unsigned long long c = ((unsigned long long)cbase[sp * DEC_CAND] << 32) |
                                   cbase[sp * DEC_CAND + 1];
      // later splits hold larger slots: on a full tie the larger slot is ranked last
      if (c <= best) { best = c; bidx = sp; }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      const unsigned long long ob = __shfl_xor(best, o, 64);
      const int oi = __shfl_xor(bidx, o, 64);
      if (ob < best || (ob == best && oi > bidx)) { best = ob; bidx = oi; }
    }
    if (lane == 0) { sm.c64[w] = best; sm.cidx[w] = bidx; }
    __syncthreads();
    if (tid == 0) {
      unsigned long long bb = sm.c64[0];
      int bi = sm.cidx[0];
      for (int i = 1; i < 4; ++i)
        if (sm.c64[i] < bb || (sm.c64[i] == bb && sm.cidx[i] > bi)) { bb = sm.c64[i]; bi = sm.cidx[i]; }
      sm.e_split = (evict && bi >= 0) ? bi : -1;
      sm.e_slot = (evict && bi >= 0) ? (int)cbase[bi * DEC_CAND + 2] : -1;
    }
    __syncthreads();
  }
  const int e_split = sm.e_split, e_slot = sm.e_slot;
  // ---------------- memory write (rank one) and readout with the new state ----------------
  if (e_slot >= 0) {
    if (tid < IM_D) {
      sm.ke[tid] = bf2f(a.K[((size_t)u * a.C + e_slot) * IM_D + tid]);
      sm.ve[tid] = bf2f(a.V[((size_t)u * a.C + e_slot) * IM_D + tid]);
    }
    __syncthreads();
    {
      float pe = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        float wv[8];
        unpack8(Wr[i], wv);
#pragma unroll
        for (int e = 0; e < 8; ++e) pe = fmaf(wv[e], sm.ke[hh * 64 + i * 8 + e], pe);
      }
      sm.phe2[hh][wc] = pe;
    }
    __syncthreads();
    if (tid < IM_DM) {
      const float pe = sm.phe2[0][tid] + sm.phe2[1][tid];
      sm.phe[tid] = pe;
      const float bn = fmaf(a.lambda, b_old, a.eta * pe * pe);
      sm.bnew[tid] = bn;
      a.bvec[(size_t)u * IM_DM + tid] = bn;
    }
    __syncthreads();
    // M <- lambda M + eta phi_e v_e^T for this thread's 16 x 4 patch
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const float f = a.eta * sm.phe[cg * 16 + i];
      float4 m = Mr[i];
      m.x = fmaf(a.lambda, m.x, f * sm.ve[4 * d4 + 0]); m.y = fmaf(a.lambda, m.y, f * sm.ve[4 * d4 + 1]);
      m.z = fmaf(a.lambda, m.z, f * sm.ve[4 * d4 + 2]); m.w = fmaf(a.lambda, m.w, f * sm.ve[4 * d4 + 3]);
      *(float4*)(Mu + (cg * 16 + i) * IM_D + 4 * d4) = m;
    }
  } else {
    if (tid < IM_DM) sm.bnew[tid] = b_old;
    __syncthreads();
  }
  for (int j = w; j < G; j += 4) {
    float dn = sm.phq[j][lane] * sm.phq[j][lane] * sm.bnew[lane] +
               sm.phq[j][lane + 64] * sm.phq[j][lane + 64] * sm.bnew[lane + 64];
    dn = wave_sum_f(dn);
    float dt = 0.f;
    if (e_slot >= 0) dt = wave_sum_f(sm.phq[j][lane] * sm.phe[lane] + sm.phq[j][lane + 64] * sm.phe[lane + 64]);
    if (lane == 0) { sm.den[j] = dn + a.mem_eps; sm.dot[j] = dt; }
  }
  __syncthreads();
  // ---------------- merge the attention partials, add back the candidates that stay ----------------
  for (int idx = tid; idx < G * IM_D; idx += 256) {
    const int j = idx >> 7, d = idx & 127;
    float m = -1e30f;
    for (int sp = 0; sp < n_act; ++sp) {
      m = fmaxf(m, pbase[(sp * DEC_GMAX + j) * DEC_REC]);
      if (sp != e_split) m = fmaxf(m, __uint_as_float(cbase[sp * DEC_CAND + 4 + j]));
    }
    float o = 0.f, l = 0.f;
    for (int sp = 0; sp < n_act; ++sp) {
      const float* rec = pbase + (sp * DEC_GMAX + j) * DEC_REC;
      const float sc = __expf(rec[0] - m);
      o = fmaf(sc, rec[2 + d], o);
      l = fmaf(sc, rec[1], l);
      if (sp != e_split) {
        const float pc = __expf(__uint_as_float(cbase[sp * DEC_CAND + 4 + j]) - m);
        const int cs = (int)cbase[sp * DEC_CAND + 2];
        o = fmaf(pc, bf2f(a.V[((size_t)u * a.C + cs) * IM_D + d]), o);
        l += pc;
      }
    }
    const float o_attn = (n_act > 0 && l > 0.f) ? o / l : 0.f;
    float mr = sm.rold[j][d];
    if (e_slot >= 0) mr = fmaf(a.lambda, mr, a.eta * sm.dot[j] * sm.ve[d]);
    const float res = sm.gate[j] * (mr / sm.den[j]);
    const size_t oi = ((size_t)b * a.H + h * G + j) * IM_D + d;
    a.out[oi] = f2bf_rne(o_attn + res);
    if (a.readout) a.readout[oi] = res;
  }
  __syncthreads();
  // ---------------- fill the hole with the last entry, publish the new length ----------------
  const int n_keep = (e_slot >= 0) ? n - 1 : n;
  if (e_slot >= 0 && e_slot < n_keep) {
    const size_t src = (size_t)u * a.C + n_keep, dst = (size_t)u * a.C + e_slot;
    if (tid < 16) *(uint4*)(a.K + dst * IM_D + tid * 8) = *(const uint4*)(a.K + src * IM_D + tid * 8);
    else if (tid < 32) *(uint4*)(a.V + dst * IM_D + (tid - 16) * 8) = *(const uint4*)(a.V + src * IM_D + (tid - 16) * 8);
    else if (tid < 40) *(uint4*)(a.Kidx + dst * IM_DI + (tid - 32) * 8) = *(const uint4*)(a.Kidx + src * IM_DI + (tid - 32) * 8);
    else if (tid == 40) a.pos[dst] = a.pos[src];
  }
  if (tid == 0) {
    a.len[u] = n_keep;
    a.nproj[u] = n_keep;
    if (a.evicted) a.evicted[u] = e_slot;
    a.cnt_unit[u] = 0;
  }
}

union DecSmem {
  DecSplitSmem s;
  DecTailSmem t;
};

// grid: units tail blocks + units * S split blocks (tail blocks first when r_first)
template <int G>
__global__ __launch_bounds__(256, 2) void k_dec_main(const DecArgs a) {
  __shared__ __attribute__((aligned(16))) DecSmem sm;
  const int U = a.B * a.H_kv;
  int blk = blockIdx.x;
  if (a.r_first) {
    if (blk < U) { dec_tail<G>(a, blk, sm.t); return; }
    blk -= U;
  } else if (blk >= U * a.S) {
    dec_tail<G>(a, blk - U * a.S, sm.t);
    return;
  }
  // consecutive blocks take different units: the short last splits come last
  dec_split<G>(a, blk % U, blk / U, sm.s);
}
