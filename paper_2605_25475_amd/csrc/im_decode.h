// Fused decode step: the whole path for one new token per sequence in three launches.
//   k_dec_prep : query-side indexer features (U_q, G GEMVs; the consumer applies the QK-Norm),
//                append of the new (k, v), its indexer key, and the terms of the memory readout
//                that do not depend on this step's eviction (phi_q, phi_q^T M, phi_q^2 . b, gate).
//   k_dec_main : per (unit, 128-key split) workgroups of two wave roles.  Scoring waves score
//                the split's keys and find its local eviction candidate (the entry ranked last);
//                attention waves stream K / V and accumulate the softmax-attention partial
//                WITHOUT that candidate; the candidate's logits and K / V rows go to a record.
//   k_att_main : the attend-only variant (no scoring waves; nothing left out unless the slot to
//                evict is named).  k_att_merged: the same with the prep roles in its launch, for
//                steps that score nothing (two launches per step instead of three).
//   k_dec_tail : one workgroup per unit picks the evicted entry among the candidates, folds it
//                into the memory state, merges the partials plus the candidates that stay,
//                adds the gated readout, fills the hole and writes the output.
//                k_dec_tail_head: the same with one workgroup per (unit, query head).
// Head-shared layout (one indexer key per token, one decision and one memory per sequence):
//   k_hs_prep, k_hs_score, k_att_main, k_dec_tail_head; see the comments at k_hs_prep.
// Kernel boundaries separate the three on purpose: on this chip a device-scope release (L2
// write-back) per workgroup or an in-kernel wait costs several microseconds more than a launch.
// Same results as append -> index_score (n_q = 1) -> topb_select -> memory_update -> compact_kv
// -> decode_attn_with_readout whenever every unit enters with len <= budget.
#pragma once
#include "im_device.h"

#define DEC_KEYS 128                 // keys per split workgroup (8 MFMA tiles of 16)
#define DEC_REC (IM_D + 2)           // partial record per (unit, split, head): max, denom, 128 numerators
#define DEC_GMAX 8                   // query heads per KV head supported
#define DEC_CAND 176                 // words per candidate record: 16 header, 64 K row, 64 V row, 32 Kidx row
#define DEC_CAND_K 16
#define DEC_CAND_V 80
#define DEC_CAND_KI 144
// header words: 0 rank key (score part), 1 rank key (position part), 2 slot, 3 live entries n of the
// unit (at most max_live), 4..11 attention logits of the entry, 12 its token position, 13 the unit's
// true length (above word 3 only if the live-length promise is broken).  Record index S (one past the
// splits) describes the LAST live slot: the entry that moves into the hole, and, when n = 128 S + 1,
// the one key no split covers (then it also carries that key's rank key and logits).

typedef short v4s __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef double v4d __attribute__((ext_vector_type(4)));

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
  const int32_t* ext_evict;   // optional [units]: the slot to evict is given (no scoring), -1 for none
  // outputs
  bf16_t* out;
  float* readout;
  float* scores;      // optional
  int32_t* evicted;   // optional
  // workspace
  double *qy, *alpha;
  int32_t *status, *maxpos;
  float* part;
  uint32_t* cand;
  float* qm;          // per unit: the eviction-independent terms of the memory readout (DEC_QM floats per head)
  double* xk;         // head-shared layout: U_k x of the new token, [B][16]
  uint4* hs_part;     // head-shared layout: [B][HS_NSC] last-ranked entry of each scoring workgroup
                      // (rank key hi, lo, slot or -1, unused)
  int32_t* hs_evict;  // head-shared layout: [units] the slot the unit's sequence evicts (-1: none), written
                      // by the attention kernel for the tail (ext_evict points here)
  // scalars
  int B, H, H_kv, C, H_idx, gate_in, n_sink, n_recent, budget, S, S_alloc, max_live;
  // head-shared layout (hs = 1): the H_set = H_kv units of a sequence form one set; len, pos, Kidx
  // (di = 16 values per row), nproj, M, bvec are indexed by the set u / H_set.  Else H_set = 1, di = 64.
  int hs, H_set, di;
  int attend;         // head-shared layout, attend-only step: no query-side projections, no decision; the
                      // new token's indexer key is stored by the tail
  int kidx_in_cache;  // per-unit layout, merged follower launch: the last-slot record holds no indexer key
                      // (the new token's is made in the same launch), so the tail moves it from the cache
  const int32_t* hs_named;   // head-shared layout, optional [B]: with attend = 1, the slot each sequence
                             // evicts is given by the caller (-1 or >= len: none)
  float rms_eps, mem_eps, scale, lambda, eta;
};

#define HS_NSC 8   // scoring workgroups per sequence in the head-shared layout

// The entry a sequence would evict in the head-shared layout: the last-ranked one over the results of
// its HS_NSC scoring workgroups (on a full tie the largest slot: chunks ascend); -1 if there is none.
__device__ __forceinline__ int hs_pick(const uint4 (&pk)[HS_NSC]) {
  uint32_t bh = 0xffffffffu, bl = 0xffffffffu;
  int at = -1;
#pragma unroll
  for (int c = 0; c < HS_NSC; ++c)
    if ((int)pk[c].z >= 0 && (pk[c].x < bh || (pk[c].x == bh && pk[c].y <= bl))) { bh = pk[c].x; bl = pk[c].y; at = (int)pk[c].z; }
  return at;
}

// wait until at most 4 of this wave's vector memory loads are outstanding (loads return in order)
__device__ __forceinline__ void dec_pace4() { asm volatile("s_waitcnt vmcnt(4)" ::: "memory"); }

__device__ __forceinline__ void unpack8(const uint4& u, float* f) {
  f[0] = bf_lo(u.x); f[1] = bf_hi(u.x); f[2] = bf_lo(u.y); f[3] = bf_hi(u.y);
  f[4] = bf_lo(u.z); f[5] = bf_hi(u.z); f[6] = bf_lo(u.w); f[7] = bf_hi(u.w);
}

// --------------------------------------------------------------------------------------------
// k_dec_prep.  Block roles, in the order of `blk` below.  Blocks [0, nU): two rows of U_q each against PR
// batch rows (raw projections, fp64; a larger batch takes more blocks per row pair, not more rounds per block).
// Blocks [nU, nU + nG): two rows of G, likewise.
// Blocks after: one per unit, append + indexer key of the new token; then DEC_MP more per unit, the
// eviction-independent terms of the memory readout.
// --------------------------------------------------------------------------------------------
// out_rows[m][r] = sum_k A[m][k] Bm[n0 + r][k] for r = 0, 1 and every batch row m (bf16 inputs, fp64
// accumulation).  Each round issues the loads of two 2048-wide slabs before any arithmetic.
template <int MB>
__device__ __forceinline__ void dec_gemv2(const bf16_t* __restrict__ A, const bf16_t* __restrict__ Bm, int n0,
                                          int N, int M, int Kd, double (*part)[16], double* out_rows,
                                          int m_first = 0, int m_end = 1 << 30) {
  const int tid = threadIdx.x;
  const int r1 = (n0 + 1 < N) ? n0 + 1 : n0;   // an absent second row repeats the first (result unused)
  m_end = min(m_end, M);                       // batch rows [m_first, m_end) only
  for (int mb = m_first; mb < m_end; mb += MB) {
    double acc[MB][2];
#pragma unroll
    for (int i = 0; i < MB; ++i) acc[i][0] = acc[i][1] = 0.0;
    for (int k0 = tid * 8; k0 < Kd; k0 += 2 * 2048) {
      uint4 bu[2][2], au[2][MB];
#pragma unroll
      for (int it = 0; it < 2; ++it) {
        const int k = (k0 + it * 2048 < Kd) ? k0 + it * 2048 : k0;
        bu[it][0] = *(const uint4*)(Bm + (size_t)n0 * Kd + k);
        bu[it][1] = *(const uint4*)(Bm + (size_t)r1 * Kd + k);
#pragma unroll
        for (int i = 0; i < MB; ++i) {
          const int m = (mb + i < M) ? mb + i : M - 1;
          au[it][i] = *(const uint4*)(A + (size_t)m * Kd + k);
        }
      }
      // MB = 4: every load above is issued before the arithmetic starts.  The empty statement needs a word of
      // each, and nothing is scheduled across the barrier; else the second slab's loads sink into its branch
      // below and their latency is paid a second time.  (With 8 batch rows the registers this takes would
      // halve the number of resident workgroups.)
      if constexpr (MB == 4) {
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("" : "+v"(bu[0][0].x), "+v"(bu[0][1].x), "+v"(bu[1][0].x), "+v"(bu[1][1].x),
                          "+v"(au[0][0].x), "+v"(au[0][1].x), "+v"(au[0][2].x), "+v"(au[0][3].x),
                          "+v"(au[1][0].x), "+v"(au[1][1].x), "+v"(au[1][2].x), "+v"(au[1][3].x));
      }
#pragma unroll
      for (int it = 0; it < 2; ++it) {
        if (k0 + it * 2048 < Kd) {
          float b0[8], b1[8];
          unpack8(bu[it][0], b0);
          unpack8(bu[it][1], b1);
#pragma unroll
          for (int i = 0; i < MB; ++i) {
            float av[8];
            unpack8(au[it][i], av);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
              acc[i][0] = fma((double)av[e], (double)b0[e], acc[i][0]);
              acc[i][1] = fma((double)av[e], (double)b1[e], acc[i][1]);
            }
          }
        }
      }
    }
    // the 2 MB wave sums as one butterfly (value 2 i + r = batch row i, weight row r), then the 4 waves
    // meet in LDS: lane 15 of row rho of register i holds value 4 i + 2 (rho & 1) + (rho >> 1)
    double ws[MB / 2];
    wave_sums_butterfly_d<2 * MB>(&acc[0][0], ws);
    __syncthreads();
    if ((tid & 15) == 15) {
      const int rho = (tid >> 4) & 3;
#pragma unroll
      for (int i = 0; i < MB / 2; ++i) part[tid >> 6][4 * i + 2 * (rho & 1) + (rho >> 1)] = ws[i];
    }
    __syncthreads();
    if (tid < 2 * MB && mb + (tid >> 1) < m_end)
      out_rows[(mb + (tid >> 1)) * 2 + (tid & 1)] = part[0][tid] + part[1][tid] + part[2][tid] + part[3][tid];
  }
  __syncthreads();
}

#define DEC_MP 4                        // workgroups sharing the memory-readout terms of one unit
#define DEC_QM (IM_DM + DEC_MP * IM_D + 2 + DEC_MP)
// per unit, G * DEC_QM floats: phi(q) [G][128] | partial phi(q)^T M [DEC_MP][G][128] | gate [G] |
// unused [G] | partial phi(q)^2 . b [DEC_MP][G]

// The terms of the memory readout that do not depend on this step's eviction, for the G query heads
// of one unit against the memory state as it stands: phi_q = W_theta q, phi_q^T M, sum_c phi_q[c]^2
// b[c], and the gate sigmoid(w_g . q + c_g).  Workgroup mp of a unit takes rows 32 mp .. 32 mp + 31
// of the memory (its slice of phi_q, and partial sums over those rows).  The tail kernel applies
// the rank-one update of this step to these terms instead of reading the updated state back.
// LDS of the prep roles (a struct, so that a kernel that also holds split workgroups can overlay it)
struct DecPrepSmem {
  float phq[DEC_GMAX][32];
  float red[4][DEC_GMAX][IM_D];
  double part[4][16];
  double rows[64 * 2];   // up to 64 batch rows x 2 outputs
  float k[IM_D];
  double u[IM_DI];
  int mp[4];
};

// Workgroups go to the 8 XCDs round-robin by their index.  Everything a unit owns (its memory state,
// readout terms, split records, appended rows) is touched by several launches per step; with the
// unit's workgroups of every launch on XCD u % 8 those lines are found in that XCD's L2.  For a block
// range that starts at a multiple of 8 and holds `per` workgroups for each of U units (U a multiple of
// 8), index r maps to unit (r % 8) + 8 ((r / 8) / per) and item (r / 8) % per; else plain division.
__device__ __forceinline__ void xcd_unit_map(const int r, const int per, const int U, int& u, int& item) {
  if (U % 8 == 0) {
    const int x = r & 7, k = r >> 3;
    u = x + 8 * (k / per);
    item = k % per;
  } else {
    u = r / per;
    item = r % per;
  }
}

__device__ __forceinline__ void dec_prep_memory(const DecArgs& a, const int u, const int mp, DecPrepSmem& ps) {
  float (*s_phq)[32] = ps.phq;
  float (*s_red)[DEC_GMAX][IM_D] = ps.red;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int b = u / a.H_kv, h = u % a.H_kv, G = a.H / a.H_kv;
  float* qm = a.qm + (size_t)u * G * DEC_QM;
  // every load first
  const int d4 = tid & 31, rg = tid >> 5;    // patch of M: rows 32 mp + 4 rg .. + 3, columns 4 d4 .. 4 d4 + 3
  const float* Mu = a.M + ((size_t)(u / a.H_set) * IM_DM + 32 * mp) * IM_D;
  float4 Mr[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) Mr[i] = *(const float4*)(Mu + (rg * 4 + i) * IM_D + 4 * d4);
  const int cl = tid >> 3, pt = tid & 7;     // W_theta row 32 mp + cl, dims 16 pt .. 16 pt + 15
  const uint4 Wr0 = *(const uint4*)(a.Wt + (32 * mp + cl) * IM_D + 16 * pt);
  const uint4 Wr1 = *(const uint4*)(a.Wt + (32 * mp + cl) * IM_D + 16 * pt + 8);
  const float bc = a.bvec[(size_t)(u / a.H_set) * IM_DM + 32 * mp + (lane & 31)];
  const float g0 = bf2f(a.wg[lane]), g1 = bf2f(a.wg[lane + 64]);
  const bf16_t* qb = a.q + ((size_t)b * a.H + h * G) * IM_D;
  // (the query rows too: inside the loop over the heads each pair of loads would be a round trip of its
  // own; heads past the group repeat its last row and are not used)
  uint4 qr[DEC_GMAX][2];
#pragma unroll
  for (int j = 0; j < DEC_GMAX; ++j) {
    const bf16_t* qj = qb + min(j, G - 1) * IM_D + 16 * pt;
    qr[j][0] = *(const uint4*)qj;
    qr[j][1] = *(const uint4*)(qj + 8);
  }
  float wv[16];
  unpack8(Wr0, wv);
  unpack8(Wr1, wv + 8);
#pragma unroll
  for (int j = 0; j < DEC_GMAX; ++j) {
    if (j >= G) break;
    float qv[16];
    unpack8(qr[j][0], qv);
    unpack8(qr[j][1], qv + 8);
    float pq = 0.f;
#pragma unroll
    for (int e = 0; e < 16; ++e) pq = fmaf(wv[e], qv[e], pq);
    // the 8 parts of a row sit in adjacent lanes: after three shifted adds lane pt = 7 has the sum
    pq += dpp_zero_f<0x111, 0xF>(pq);
    pq += dpp_zero_f<0x112, 0xF>(pq);
    pq += dpp_zero_f<0x114, 0xF>(pq);
    if (pt == 7) {
      s_phq[j][cl] = pq;
      qm[j * IM_DM + 32 * mp + cl] = pq;
    }
  }
  if (mp == 0) {
    for (int j = w; j < G; j += 4) {   // gate: one wave per head
      const float gz = wave_sum_f(fmaf(g0, bf2f(qb[j * IM_D + lane]), g1 * bf2f(qb[j * IM_D + lane + 64])));
      if (lane == 0) qm[G * (IM_DM + DEC_MP * IM_D) + j] = 1.f / (1.f + __expf(-(gz + a.cg)));
    }
  }
  __syncthreads();
  for (int j = 0; j < G; ++j) {   // partial phi_q^T M over this thread's 4 rows, then over the wave's 8
    float r0 = 0.f, r1 = 0.f, r2 = 0.f, r3 = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float f = s_phq[j][rg * 4 + i];
      r0 = fmaf(f, Mr[i].x, r0); r1 = fmaf(f, Mr[i].y, r1);
      r2 = fmaf(f, Mr[i].z, r2); r3 = fmaf(f, Mr[i].w, r3);
    }
    r0 = halves_sum_f(r0); r1 = halves_sum_f(r1); r2 = halves_sum_f(r2); r3 = halves_sum_f(r3);
    if (lane < 32) *(float4*)&s_red[w][j][4 * d4] = make_float4(r0, r1, r2, r3);
  }
  for (int j = w; j < G; j += 4) {
    const float p = s_phq[j][lane & 31];
    const float dn = wave_sum_f((lane < 32) ? p * p * bc : 0.f);
    if (lane == 0) qm[G * (IM_DM + DEC_MP * IM_D + 2) + mp * G + j] = dn;
  }
  __syncthreads();
  for (int idx = tid; idx < G * IM_D; idx += 256) {
    const int j = idx >> 7, d = idx & 127;
    qm[G * IM_DM + (mp * G + j) * IM_D + d] = s_red[0][j][d] + s_red[1][j][d] + s_red[2][j][d] + s_red[3][j][d];
  }
}

// One unit's append in the per-unit layout: the new (k, v, pos) go to slot len, and the slot's
// indexer key bf16(Norm(U_k k)) is computed (fp64) and stored.
__device__ __forceinline__ void dec_prep_unit(const DecArgs& a, const int u, DecPrepSmem& ps) {
  float* s_k = ps.k;
  double* s_u = ps.u;
  int* s_mp = ps.mp;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int b = u / a.H_kv;
  const int n_old = a.len[u];
  // loads that do not depend on the length go out together with it
  uint4 ukr[4], newrow;
  {
    const uint4* ur = (const uint4*)(a.Uk + (tid >> 2) * IM_D + (tid & 3) * 32);
#pragma unroll
    for (int i = 0; i < 4; ++i) ukr[i] = ur[i];
    // (no branch around this load: a value defined in one arm of a branch is waited for at the arm's end;
    // threads past 31 repeat thread 31's piece)
    const int t = min(tid, 31);
    newrow = *(const uint4*)(((t < 16) ? a.k_new : a.v_new) + (size_t)u * IM_D + (t & 15) * 8);
  }
  const int newpos = a.pos_new[b];
  asm volatile("" : "+v"(ukr[0].x), "+v"(ukr[1].x), "+v"(ukr[2].x), "+v"(ukr[3].x), "+v"(newrow.x));
  if (a.n_recent > 0) {  // newest position of the unit (new token included) for the recent window
    int m = INT_MIN;
    const int nn = min(n_old, a.max_live);
    for (int i = tid; i < nn; i += 256) m = max(m, a.pos[(size_t)u * a.C + i]);
    if (n_old + 1 <= a.C) m = max(m, newpos);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) m = max(m, __shfl_xor(m, o, 64));
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
    *(uint4*)(a.K + slot * IM_D + tid * 8) = newrow;
    float f[8];
    unpack8(newrow, f);
#pragma unroll
    for (int e = 0; e < 8; ++e) s_k[tid * 8 + e] = f[e];
  } else if (tid < 32) {
    *(uint4*)(a.V + slot * IM_D + (tid - 16) * 8) = newrow;
  } else if (tid == 32) {
    a.pos[slot] = newpos;
  }
  __syncthreads();
  {  // u_c = Uk[c] . k : thread (c = tid/4, quarter = tid%4)
    const int c = tid >> 2, qd = tid & 3;
    double acc = 0.0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float f[8];
      unpack8(ukr[i], f);
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

template <int PR>   // batch rows per projection block: 4 or 8
__global__ __launch_bounds__(256) void k_dec_prep(const DecArgs a) {
  __shared__ DecPrepSmem ps;
  double (*part)[16] = ps.part;
  double* rows = ps.rows;
  const int tid = threadIdx.x;
  const int Nq = a.H_idx * IM_DI;
  // a projection block takes two weight rows and PR batch rows (one round of loads): nB blocks per row pair
  const int nB = (a.B + PR - 1) / PR;
  const int nU = Nq / 2 * nB, nG = (a.H_idx + 1) / 2 * nB;
  const int U = a.B * a.H_kv;
  // the per-unit blocks (longer chains of short phases) are dispatched first
  const int blk = ((int)blockIdx.x >= (1 + DEC_MP) * U) ? (int)blockIdx.x - (1 + DEC_MP) * U
                                                        : nU + nG + (int)blockIdx.x;
  if (blk < nU) {
    const int rp = (nB == 1) ? blk : blk / nB;   // (no division on the common path)
    const int n0 = rp * 2, m0 = (blk - rp * nB) * PR, m1 = min(m0 + PR, a.B);
    dec_gemv2<PR>(a.q, a.Uq, n0, Nq, a.B, a.H * IM_D, part, rows, m0, m1);
    // raw projections; the consumer applies the QK-Norm (it needs a whole head, this block has 2 rows)
    for (int i = 2 * m0 + tid; i < 2 * m1; i += 256) a.qy[(size_t)(i >> 1) * Nq + n0 + (i & 1)] = rows[i];
    return;
  }
  if (blk < nU + nG) {
    const int rp = (nB == 1) ? blk - nU : (blk - nU) / nB;
    const int n0 = rp * 2, m0 = (blk - nU - rp * nB) * PR, m1 = min(m0 + PR, a.B);
    dec_gemv2<PR>(a.xg, a.Gw, n0, a.H_idx, a.B, a.gate_in, part, rows, m0, m1);
    for (int i = 2 * m0 + tid; i < 2 * m1; i += 256) {
      const int r = n0 + (i & 1);
      if (r < a.H_idx) a.alpha[(size_t)(i >> 1) * a.H_idx + r] = rows[i];   // raw G x; scaled by the consumer
    }
    return;
  }
  if (blk >= nU + nG + U) {
    int mu, mp;
    xcd_unit_map(blk - nU - nG - U, DEC_MP, U, mu, mp);   // (these blocks start at grid index U: a multiple of 8 with U)
    dec_prep_memory(a, mu, mp, ps);
    return;
  }
  dec_prep_unit(a, blk - nU - nG, ps);
}

// --------------------------------------------------------------------------------------------
// Head-shared layout: k_hs_prep and k_hs_score take the place of k_dec_prep and of the scoring
// waves.  One indexer key per token (from its hidden state) and one score per token mean one
// decision per sequence, so a few workgroups per sequence rank all its keys (16 values each) before
// the attention launch, which then treats the decision as given (the path of a named slot).
// --------------------------------------------------------------------------------------------
// Block roles: [0, U) append the new (k, v) of a unit (the set's position by its first head);
// [U, (1 + DEC_MP) U) the readout terms; then two rows each of U_q (input q), G and U_k (input x).
__device__ __forceinline__ void hs_prep_unit(const DecArgs& a, const int u) {
  const int tid = threadIdx.x, b = u / a.H_kv;
  const int n_old = a.len[b];
  const int t = min(tid, 31);   // (one load without a branch around it; threads past 31 repeat thread 31's piece)
  uint4 newrow = *(const uint4*)(((t < 16) ? a.k_new : a.v_new) + (size_t)u * IM_D + (t & 15) * 8);
  const int newpos = a.pos_new[b];
  const bool lead = u % a.H_kv == 0;
  if (n_old + 1 > a.C) {
    if (tid == 0 && lead) atomicOr(a.status, IM_STATUS_APPEND_OVERFLOW_BIT);
    return;
  }
  if (n_old + 1 > a.max_live && tid == 0 && lead) atomicOr(a.status, IM_STATUS_LIVE_EXCEEDED_BIT);
  const size_t slot = (size_t)u * a.C + n_old;
  if (tid < 16) *(uint4*)(a.K + slot * IM_D + tid * 8) = newrow;
  else if (tid < 32) *(uint4*)(a.V + slot * IM_D + (tid - 16) * 8) = newrow;
  else if (tid == 32 && lead) a.pos[(size_t)b * a.C + n_old] = newpos;
}

// two rows of one of the three projections: g counts U_q (input q), then G, then U_k (input x) row pairs
__device__ __forceinline__ void hs_prep_gemv(const DecArgs& a, const int g, DecPrepSmem& ps) {
  const int tid = threadIdx.x;
  const int Nq = a.H_idx * IM_DI_SHARED;
  const int nU = Nq / 2, nG = (a.H_idx + 1) / 2;
  const bool isq = g < nU, isg = !isq && g < nU + nG;
  const int n0 = (isq ? g : isg ? g - nU : g - nU - nG) * 2;
  const int N = isq ? Nq : isg ? a.H_idx : IM_DI_SHARED;
  const bf16_t* A = isq ? a.q : a.xg;
  const bf16_t* W = isq ? a.Uq : isg ? a.Gw : a.Uk;
  const int Kd = isq ? a.H * IM_D : a.gate_in;
  double* out = isq ? a.qy : isg ? a.alpha : a.xk;
  if (a.B <= 4) dec_gemv2<4>(A, W, n0, N, a.B, Kd, ps.part, ps.rows);
  else dec_gemv2<8>(A, W, n0, N, a.B, Kd, ps.part, ps.rows);
  for (int i = tid; i < a.B * 2; i += 256) {   // raw projections; the consumer normalises and scales
    const int r = n0 + (i & 1);
    if (r < N) out[(size_t)(i >> 1) * N + r] = ps.rows[i];
  }
}

__global__ __launch_bounds__(256) void k_hs_prep(const DecArgs a) {
  __shared__ DecPrepSmem ps;
  const int U = a.B * a.H_kv;
  const int blk = blockIdx.x;
  if (blk < U) {
    hs_prep_unit(a, blk);
  } else if (blk < (1 + DEC_MP) * U) {
    int mu, mp;
    xcd_unit_map(blk - U, DEC_MP, U, mu, mp);
    dec_prep_memory(a, mu, mp, ps);
  } else {   // an attend-only step has the U_k blocks alone
    const int nUG = a.H_idx * IM_DI_SHARED / 2 + (a.H_idx + 1) / 2;
    hs_prep_gemv(a, blk - (1 + DEC_MP) * U + (a.attend ? nUG : 0), ps);
  }
}

// grid (B * HS_NSC), 512 threads.  Workgroup (b, c) scores chunk c of sequence b's live keys: QK-Norm
// of the step's query features and the head gates (every workgroup, for itself), the new token's
// indexer key (stored by c = 0), the scores of the chunk's keys, and the chunk's entry ranked last by
// (score, then position, then slot) with sinks and the recent window forced to the top.  The
// attention kernel takes the last-ranked of the HS_NSC results (hs_pick) and hands it to the tail.
// Optionally writes the scores to a.scores [B][C].
#define HS_ST 512
__global__ __launch_bounds__(HS_ST) void k_hs_score(const DecArgs a) {
  constexpr int DI = IM_DI_SHARED;
  __shared__ double s_q[16][DI];
  __shared__ double s_al[16];
  __shared__ float s_kn[DI];
  constexpr int NW = HS_ST / 64;
  __shared__ uint32_t s_hi[NW], s_lo[NW];
  __shared__ int s_at[NW], s_mp[NW];
  const int b = blockIdx.x / HS_NSC, ck = blockIdx.x % HS_NSC, tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int n_old = a.len[b];
  const bool fits = n_old + 1 <= a.C;
  const int n = min(n_old + (fits ? 1 : 0), a.max_live);
  const int newpos = a.pos_new[b], qpos = a.q_pos[b];
  const bf16_t* kx = a.Kidx + (size_t)b * a.C * DI;
  const int32_t* ps = a.pos + (size_t)b * a.C;
  if (tid < 256) {   // thread (head j, dim d)
    const int j = tid >> 4, d = tid & 15;
    const bool hv = j < a.H_idx;
    const double y = hv ? a.qy[((size_t)b * a.H_idx + j) * DI + d] : 0.0;
    const double ss = row16_sum_d(y * y);
    const double rr = sqrt(ss / (double)DI + (double)a.rms_eps);
    const double wq = a.nqw ? (double)bf2f(a.nqw[d]) : 1.0;
    s_q[j][d] = hv ? (double)(float)(y / rr * wq) : 0.0;
    if (d == 0) s_al[j] = hv ? (double)(float)(a.alpha[(size_t)b * a.H_idx + j] / sqrt((double)(a.H_idx * DI))) : 0.0;
  } else if (tid < 256 + DI) {   // one 16-lane row: the new token's key
    const int d = tid - 256;
    const double v = a.xk[(size_t)b * DI + d];
    const double ss = row16_sum_d(v * v);
    const double rr = sqrt(ss / (double)DI + (double)a.rms_eps);
    const double wk = a.nkw ? (double)bf2f(a.nkw[d]) : 1.0;
    const bf16_t kb = d2bf_rne(v / rr * wk);
    s_kn[d] = bf2f(kb);
    if (fits && ck == 0) a.Kidx[((size_t)b * a.C + n_old) * DI + d] = kb;
  }
  int mxp = 0;
  if (a.n_recent > 0) {   // newest position of the sequence, the new token included
    int m = fits ? newpos : INT_MIN;
    for (int i = tid; i < min(n_old, a.max_live); i += HS_ST) m = max(m, ps[i]);
    m = (int)(wave_max_u((uint32_t)m ^ 0x80000000u) ^ 0x80000000u);
    if (lane == 0) s_mp[w] = m;
  }
  __syncthreads();
  if (a.n_recent > 0) {
    mxp = s_mp[0];
#pragma unroll
    for (int i = 1; i < NW; ++i) mxp = max(mxp, s_mp[i]);
  }
  // Scores on the fp64 matrix cores, a tile of 16 keys per wave at a time: Z[head][key] = q . Kidx_tile^T
  // as 4 steps of the 16x16x4 product (lane (l16, kq) supplies dims 4 kq .. 4 kq + 3 of head l16 and of
  // key l16; result register r is head 4 r + kq, key l16).  A lane adds the gated terms of its 4 heads,
  // the 4 lanes of a key meet by two half-swaps, and the lanes kq = 0 rank their key.
  const int l16 = lane & 15, kq = lane >> 4;
  double qd[4], al4[4];
#pragma unroll
  for (int m = 0; m < 4; ++m) { qd[m] = s_q[l16][4 * kq + m]; al4[m] = s_al[4 * m + kq]; }
  uint32_t bhi = 0xffffffffu, blo = 0xffffffffu;
  int bat = -1;
  const int tpc = ((n + 15) / 16 + HS_NSC - 1) / HS_NSC;           // tiles per chunk
  const int n_tiles = min((n + 15) / 16, (ck + 1) * tpc);          // this chunk: tiles [ck tpc, n_tiles)
  constexpr int PF = 4;   // tiles in flight per wave
#pragma unroll 1
  for (int t0 = ck * tpc + w; t0 < n_tiles; t0 += NW * PF) {
    uint2 ka[PF];
    int pk[PF];
#pragma unroll
    for (int i = 0; i < PF; ++i) {
      const int key = 16 * (t0 + NW * i) + l16;
      ka[i] = *(const uint2*)(kx + (size_t)max(min(key, n_old - 1), 0) * DI + 4 * kq);
      pk[i] = ps[max(min(key, n_old - 1), 0)];
    }
#pragma unroll
    for (int i = 0; i < PF; ++i) {
      const int key = (t0 + NW * i < n_tiles) ? 16 * (t0 + NW * i) + l16 : n;   // past the chunk: never ranked
      float f[4] = {bf_lo(ka[i].x), bf_hi(ka[i].x), bf_lo(ka[i].y), bf_hi(ka[i].y)};
      if (key >= n_old) {   // the new token's key (columns past it are never ranked)
#pragma unroll
        for (int m = 0; m < 4; ++m) f[m] = s_kn[4 * kq + m];
      }
      v4d z = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
      for (int m = 0; m < 4; ++m) z = __builtin_amdgcn_mfma_f64_16x16x4f64(qd[m], (double)f[m], z, 0, 0, 0);
      double asum = 0.0;
#pragma unroll
      for (int r = 0; r < 4; ++r) asum = fma(al4[r], fmax(z[r], 0.0), asum);
      asum = rows_sum_d(asum);
      if (kq == 0 && key < n) {
        const int p = (key < n_old) ? pk[i] : newpos;
        const float sc = (p <= qpos) ? (float)asum : -INFINITY;
        if (a.scores) a.scores[(size_t)b * a.C + key] = sc;
        const bool forced = (p < a.n_sink) || (a.n_recent > 0 && (long long)p > (long long)mxp - a.n_recent);
        const uint32_t khi = forced ? IM_KEY_PINF : score_key(sc);
        const uint32_t klo = (uint32_t)(~((uint32_t)p ^ 0x80000000u));
        if (khi < bhi || (khi == bhi && klo <= blo)) { bhi = khi; blo = klo; bat = key; }   // ascending keys: <= keeps the largest slot
      }
    }
  }
  {
    const uint32_t mh = wave_min_u(bhi);
    const uint32_t ml = wave_min_u(bhi == mh ? blo : 0xffffffffu);
    const int win = (int)wave_max_u((bat >= 0 && bhi == mh && blo == ml) ? (uint32_t)bat + 1u : 0u) - 1;
    if (lane == 0) { s_hi[w] = mh; s_lo[w] = ml; s_at[w] = win; }
  }
  __syncthreads();
  if (tid < 64) {
    const bool on = lane < NW && s_at[lane & (NW - 1)] >= 0;
    const uint32_t khi = on ? s_hi[lane & (NW - 1)] : 0xffffffffu, klo = on ? s_lo[lane & (NW - 1)] : 0xffffffffu;
    const uint32_t mh = wave_min_u(khi);
    const uint32_t ml = wave_min_u((on && khi == mh) ? klo : 0xffffffffu);
    const int win = (int)wave_max_u((on && khi == mh && klo == ml) ? (uint32_t)s_at[lane & (NW - 1)] + 1u : 0u) - 1;
    if (lane == 0) {
      a.hs_part[(size_t)b * HS_NSC + ck] = make_uint4(mh, ml, (uint32_t)win, 0u);
      if (ck == 0 && n > a.budget + 1) atomicOr(a.status, IM_STATUS_OVER_BUDGET_BIT);
    }
  }
}

// --------------------------------------------------------------------------------------------
// k_dec_main
// --------------------------------------------------------------------------------------------
struct DecSplitSmem {
  union {
    double zs[DEC_KEYS][17];         // gated similarities alpha_j ReLU(q_j . k) [key][indexer head]
    float oacc[16][4][IM_D];         // later: output partials of the 16 (wave, key group) streams,
  };                                 //        4 heads at a time
  float pl[DEC_KEYS][8];             // probabilities [key][head]
  float wm[4][8], wl[4][8];
  float clog[8];
  float xlp[4][8];                   // the leftover key's partial logits [scoring wave][head]
  unsigned long long c64[4];         // per scoring wave: rank key and key index of its last-ranked entry
  int cslot[4];
};

#define DEC_MT 512   // threads of a split workgroup: 4 attention waves and 4 scoring waves

// One (unit, split) workgroup.  Waves 0-3 stream the split's K and V rows (64 KB) and do the
// attention partial; waves 4-7 stream the indexer keys (16 KB), score them and find the split's
// last-ranked entry while the K / V rows are still arriving.  The two roles meet at the first
// workgroup barrier, when the attention waves have issued their loads.
// SCORE = false is the attend-only step: no scoring waves (the workgroup is the 4 attention waves
// alone, so more of them fit on a CU), nothing is left out of the partial.
// MERGED: the launch also holds the prep roles, so the new token's rows come from the inputs.
template <int G, bool SCORE, bool MERGED = false>
__device__ __forceinline__ void dec_split(const DecArgs& a, const int u, const int s, DecSplitSmem& sm,
                                          const double* __restrict__ qy, const double* __restrict__ alpha) {
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);   // a scalar, so that branches on the wave's role are uniform
  const int wl = w & 3;                 // wave within its role
  const bool scoring = SCORE && w >= 4; // wave-uniform role
  const int b = u / a.H_kv, h = u % a.H_kv;
  const int su = u / a.H_set;           // the set that owns the length, positions and indexer keys
  const int n_old = a.len[su];
  const int n_true = n_old + ((n_old + 1 <= a.C) ? 1 : 0);
  const int n = min(n_true, a.max_live);
  const int k0 = s * DEC_KEYS;
  const int nk = max(0, min(DEC_KEYS, n - k0));
  uint32_t* crec = a.cand + ((size_t)u * a.S_alloc + s) * DEC_CAND;
  if (nk <= 0) {
    if (s == 0 && tid == 0) {
      crec[3] = (uint32_t)n;   // an empty unit still tells the tail its length
      crec[13] = (uint32_t)n_true;
      if (a.hs) a.hs_evict[u] = -1;
    }
    return;
  }
  const size_t base = (size_t)u * a.C + k0;
  const int l16 = lane & 15, kq = lane >> 4;
  const bool own_last = (n <= a.S * DEC_KEYS) && (k0 + nk == n);   // this split holds the last live slot
  uint32_t* lrec = a.cand + ((size_t)u * a.S_alloc + a.S) * DEC_CAND;
  const int ll = n - 1 - k0;
  const bool do_x_any = (s == 0) && (n > a.S * DEC_KEYS);   // split 0 also covers the one key beyond the splits
  // rows past the end of the split are read from its last row instead (finite values, no branches):
  // their logits are masked and their probabilities are zero further down
  uint4 kif[2][2], kf[2][4], vf[2][4], qf[4];
  float sreg[2][4];
  int mypos = 0;
  uint4 lkx = make_uint4(0, 0, 0, 0);
  int lpos = 0;
  uint4 pk[HS_NSC];
  int ev_in = -1;
  if (!SCORE) {
    // no scoring waves: nothing is left out of the partial, unless the slot to evict is named: by the
    // caller, or (head-shared layout) by the sequence's scoring workgroups.  The loads go out here and
    // are looked at once the wave's stream loads are in flight.
    if (tid < 4) {
      if (a.hs && !a.attend) {
#pragma unroll
        for (int c = 0; c < HS_NSC; ++c) pk[c] = a.hs_part[(size_t)b * HS_NSC + c];
      } else if (a.hs && a.hs_named) {
        ev_in = a.hs_named[b];
      } else if (a.ext_evict && !a.hs) {
        ev_in = a.ext_evict[u];
      }
    }
    // the last live slot's indexer key and position for the last-slot record
    // (merged launch: the new token's position comes from the input and its indexer key is not made yet)
    const bool last_is_new = MERGED && n - 1 == n_old;
    if (own_last && tid < a.di / 8 && !last_is_new)
      lkx = *(const uint4*)(a.Kidx + ((size_t)su * a.C + (n - 1)) * a.di + 8 * tid);
    if (own_last && tid == 8) lpos = last_is_new ? a.pos_new[b] : a.pos[(size_t)su * a.C + (n - 1)];
  }
  if (scoring) {
    // ================= scoring waves: tiles 2 wl, 2 wl + 1 (keys 32 wl .. 32 wl + 31) =================
    // their few loads go ahead of the attention waves' many: the scoring chain is the longer one
    __builtin_amdgcn_s_setprio(3);
    // Indexer query features as the B operand of the fp64 MFMA: lane (head l16, kq) holds dims
    // 16 kq .. 16 kq + 15 of head l16.
    const bool hv = l16 < a.H_idx;
    double qd[16];
    {
      const uint4* yrow = (const uint4*)(qy + ((size_t)b * a.H_idx + (hv ? l16 : 0)) * IM_DI + 16 * kq);
#pragma unroll
      for (int m = 0; m < 8; ++m) {
        const uint4 t = yrow[m];
        qd[2 * m] = __longlong_as_double(((long long)t.y << 32) | t.x);
        qd[2 * m + 1] = __longlong_as_double(((long long)t.w << 32) | t.z);
      }
    }
    const double araw = alpha[(size_t)b * a.H_idx + (hv ? l16 : 0)];
    uint4 nw[2] = {make_uint4(0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u),
                   make_uint4(0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u)};   // bf16 ones
    if (a.nqw) {
      nw[0] = *(const uint4*)(a.nqw + 16 * kq);
      nw[1] = *(const uint4*)(a.nqw + 16 * kq + 8);
    }
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
      const int kr = min(16 * (2 * wl + tt) + l16, nk - 1);
#pragma unroll
      for (int i = 0; i < 2; ++i)
        kif[tt][i] = load_stream16(a.Kidx + (base + kr) * IM_DI + 16 * kq + 8 * i);
    }
    const int kk = 32 * wl + (lane & 31);       // the key this lane ranks (both half-waves hold it)
    mypos = a.pos[base + min(kk, nk - 1)];
    const int qpos = a.q_pos[b];
    const int mxp = (a.n_recent > 0) ? a.maxpos[u] : 0;
    // split 0 also looks after the one key beyond the splits, when there is one
    const bool do_x = do_x_any;
    // (its attention logits: wave wl takes dims 32 wl .. 32 wl + 31, lane (head l16, kq) 8 of them)
    uint4 xk = make_uint4(0, 0, 0, 0), xq = xk, xkv = xk, xki0 = xk, xki1 = xk;
    int xpos = 0;
    if (do_x) {
      const size_t last = (size_t)u * a.C + (n - 1);
      xki0 = *(const uint4*)(a.Kidx + last * IM_DI + 16 * kq);
      xki1 = *(const uint4*)(a.Kidx + last * IM_DI + 16 * kq + 8);
      xk = *(const uint4*)(a.K + last * IM_D + 32 * wl + 8 * kq);
      xq = *(const uint4*)(a.q + ((size_t)b * a.H + h * G + min(l16, G - 1)) * IM_D + 32 * wl + 8 * kq);
      // rows for the record: lanes 0-15 the K row, lanes 16-31 the V row (8 elements each)
      xkv = *(const uint4*)(((lane & 16) ? a.V : a.K) + last * IM_D + 8 * l16);
      xpos = a.pos[last];
    }
    __asm__ volatile("" ::: "memory");   // every load above is issued before the arithmetic below
    // ---- QK-Norm of the query features (per head over its 64 dims), head gate
    double alj;
    {
      double ss = 0.0;
#pragma unroll
      for (int m = 0; m < 16; ++m) ss = fma(qd[m], qd[m], ss);
      ss = rows_sum_d(ss);
      const double rr = sqrt(ss / (double)IM_DI + (double)a.rms_eps);
      const double inv = 1.0 / rr;
      float wf[16];
      unpack8(nw[0], wf);
      unpack8(nw[1], wf + 8);
#pragma unroll
      for (int m = 0; m < 16; ++m) {
        // y / rr, correctly rounded, without 16 division sequences per lane: inv is the correctly
        // rounded reciprocal; the first residual step leaves a quotient within one ulp, and a residual
        // step on such a quotient yields the correctly rounded one (Markstein's theorem on
        // FMA-based division).  The step-by-step path and the oracle divide; all three then round the
        // same fp64 value to fp32.
        double qq = qd[m] * inv;
        qq = fma(fma(-qq, rr, qd[m]), inv, qq);
        qq = fma(fma(-qq, rr, qd[m]), inv, qq);
        // (lanes past the last indexer head hold head 0's values: finite, and never used: their columns of
        // the similarity product are not stored and their gate is zero)
        qd[m] = (double)(float)(qq * (double)wf[m]);
      }
      alj = hv ? (double)(float)(araw / sqrt((double)(a.H_idx * IM_DI))) : 0.0;
    }
    if (do_x) {   // uniform per workgroup; every scoring wave computes, the first writes
      float fx[16];
      unpack8(xki0, fx);
      unpack8(xki1, fx + 8);
      double zp = 0.0;
#pragma unroll
      for (int m = 0; m < 16; ++m) zp = fma(qd[m], (double)fx[m], zp);
      zp = rows_sum_d(zp);                                   // q_j . k over the 64 dims, in all 4 rows
      const double asum = wave_sum_d((kq == 0) ? alj * fmax(zp, 0.0) : 0.0);
      float lp = 0.f;
      {
        float qv[8], kv[8];
        unpack8(xq, qv);
        unpack8(xk, kv);
#pragma unroll
        for (int e = 0; e < 8; ++e) lp = fmaf(qv[e], kv[e], lp);
      }
      lp = rows_sum_f(lp);
      if (kq == 0 && l16 < 8) sm.xlp[wl][l16] = lp;   // summed over the 4 waves after the barrier
      if (wl == 0) {
        if (l16 == 0) {
          *(uint4*)(lrec + DEC_CAND_KI + 8 * kq) = xki0;
          *(uint4*)(lrec + DEC_CAND_KI + 8 * kq + 4) = xki1;
        }
        if (lane < 32) *(uint4*)(lrec + ((lane & 16) ? DEC_CAND_V : DEC_CAND_K) + 4 * l16) = xkv;
        if (lane == 0) {
          const float sc = (xpos <= qpos) ? (float)asum : -INFINITY;
          if (a.scores) a.scores[(size_t)u * a.C + (n - 1)] = sc;
          const bool forced = (xpos < a.n_sink) || (a.n_recent > 0 && (long long)xpos > (long long)mxp - a.n_recent);
          const uint32_t skey = forced ? IM_KEY_PINF : score_key(sc);
          lrec[0] = skey;
          lrec[1] = (uint32_t)(~((uint32_t)xpos ^ 0x80000000u));
          lrec[2] = (uint32_t)(n - 1);
          lrec[3] = (uint32_t)n;
          lrec[12] = (uint32_t)xpos;
        }
      }
    }
    // ---- gated similarities of the 2 tiles of this wave: Z[key][head] = Kidx_tile . q^T (fp64 MFMA)
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
      float f[16];
      unpack8(kif[tt][0], f);
      unpack8(kif[tt][1], f + 8);
      v4d z = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
      for (int m = 0; m < 16; ++m) z = __builtin_amdgcn_mfma_f64_16x16x4f64((double)f[m], qd[m], z, 0, 0, 0);
      const int T = 2 * wl + tt;
      if (hv) {
#pragma unroll
        // fp64 16x16x4 result layout: register r of lane (l16, kq) is row 4 r + kq, column l16
        for (int r = 0; r < 4; ++r) sm.zs[16 * T + 4 * r + kq][l16] = alj * fmax(z[r], 0.0);
      }
    }
    if (own_last) {   // the last live slot's indexer key and position go to the last-slot record
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) {
        if (16 * (2 * wl + tt) + l16 == ll) {
          *(uint4*)(lrec + DEC_CAND_KI + 8 * kq) = kif[tt][0];
          *(uint4*)(lrec + DEC_CAND_KI + 8 * kq + 4) = kif[tt][1];
        }
      }
      if (lane < 32 && kk == ll) { lrec[2] = (uint32_t)(n - 1); lrec[3] = (uint32_t)n; lrec[12] = (uint32_t)mypos; }
    }
    // the rows just written belong to this wave's own keys: it reads them back without a
    // workgroup barrier (LDS operations of one wave complete in order)
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    // ---- score, forced flag, and the wave's last-ranked entry: smallest rank key; on equal
    // (score, position) the largest slot
    const bool valid = lane < 32 && kk < nk;
    uint32_t khi = 0xffffffffu, klo = 0xffffffffu;
    if (valid) {
      double asum = 0.0;
      for (int j = 0; j < a.H_idx; ++j) asum += sm.zs[kk][j];
      const float sc = (mypos <= qpos) ? (float)asum : -INFINITY;
      if (a.scores) a.scores[base + kk] = sc;
      const bool forced = (mypos < a.n_sink) || (a.n_recent > 0 && (long long)mypos > (long long)mxp - a.n_recent);
      khi = forced ? IM_KEY_PINF : score_key(sc);
      klo = (uint32_t)(~((uint32_t)mypos ^ 0x80000000u));
    }
    const uint32_t mh = wave_min_u(khi);
    const uint32_t ml = wave_min_u(khi == mh ? klo : 0xffffffffu);
    const int win = (int)wave_max_u((valid && khi == mh && klo == ml) ? (uint32_t)(lane + 1) : 0u) - 1;
    if (lane == 0) {
      sm.c64[wl] = ((unsigned long long)mh << 32) | ml;
      sm.cslot[wl] = (win >= 0) ? 32 * wl + win : -1;
    }
  } else {
    // ================= attention waves: issue the K, Q and V loads =================
    // Five groups of 4 loads per lane (K tile 0, K tile 1, Q, V tile 0, V tile 1), paced: a group goes out
    // when all but the last 4 loads before it have arrived, so a lane has at most 8 in flight.  With every
    // workgroup of the launch resident at once, issuing all 20 at the start oversubscribes the memory queues
    // (measured at configuration 3: 0.832 ms per step unpaced, 0.821 paced; stricter pacing loses again).
    // Without scoring waves in the workgroup one wait, behind the Q group, does best (the periodic schedule:
    // 0.699 ms per step unpaced, 0.697 with all three waits, 0.688 with this one).
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
      const int kr = min(16 * (2 * wl + tt) + l16, nk - 1);
      const bf16_t* krow = (MERGED && k0 + kr == n_old) ? a.k_new + (size_t)u * IM_D : a.K + (base + kr) * IM_D;
#pragma unroll
      for (int c = 0; c < 4; ++c) kf[tt][c] = load_stream16(krow + 32 * c + 8 * kq);
    }
    if constexpr (SCORE) dec_pace4();
    {
      // lanes past the group read its last head; they are zeroed where the fragments are used (zeroing a
      // register here would wait for its load, and with it for every load issued before it)
      const int jq = min(l16, G - 1);
#pragma unroll
      for (int c = 0; c < 4; ++c)
        qf[c] = *(const uint4*)(a.q + ((size_t)b * a.H + h * G + jq) * IM_D + 32 * c + 8 * kq);
      dec_pace4();
    }
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int vr = min(16 * (2 * wl + tt) + 4 * i + kq, nk - 1);
        const bf16_t* vrow = (MERGED && k0 + vr == n_old) ? a.v_new + (size_t)u * IM_D : a.V + (base + vr) * IM_D;
        vf[tt][i] = load_stream16(vrow + 8 * l16);
      }
      if (SCORE && tt == 0) dec_pace4();
    }
    // without scoring waves, split 0's attention waves look after the one key beyond the splits
    // (wave wl: dims 32 wl .. 32 wl + 31 of its logits; wave 0: its rows for the last-slot record)
    uint4 yk = make_uint4(0, 0, 0, 0), yq = yk, ykv = yk, yki0 = yk, yki1 = yk;
    int ypos = 0;
    if (!SCORE && do_x_any) {
      const size_t last = (size_t)u * a.C + (n - 1), ilast = (size_t)su * a.C + (n - 1);
      const bool x_new = MERGED && n - 1 == n_old;   // the leftover key is the new token: rows from the inputs
      const bf16_t* lk = x_new ? a.k_new + (size_t)u * IM_D : a.K + last * IM_D;
      const bf16_t* lv = x_new ? a.v_new + (size_t)u * IM_D : a.V + last * IM_D;
      if (x_new) {
      } else if (a.hs) {   // 16 values per indexer key: lanes kq = 0, 1 carry 8 each
        if (kq < 2) yki0 = *(const uint4*)(a.Kidx + ilast * IM_DI_SHARED + 8 * kq);
      } else {
        yki0 = *(const uint4*)(a.Kidx + ilast * IM_DI + 16 * kq);
        yki1 = *(const uint4*)(a.Kidx + ilast * IM_DI + 16 * kq + 8);
      }
      yk = *(const uint4*)(lk + 32 * wl + 8 * kq);
      yq = *(const uint4*)(a.q + ((size_t)b * a.H + h * G + min(l16, G - 1)) * IM_D + 32 * wl + 8 * kq);
      ykv = *(const uint4*)(((lane & 16) ? lv : lk) + 8 * l16);
      ypos = x_new ? a.pos_new[b] : a.pos[ilast];
    }
    // keep every load above this line, in this order: loads return in order, so each phase below
    // waits only for what it uses while the rest is still streaming in
    __asm__ volatile("" ::: "memory");
    if (!SCORE && tid < 4) {
      // the named entry is this split's candidate if it lies here (wave tid's 32 keys)
      int ev = ev_in;
      if (a.hs) {   // the sequence's decision is found here and handed to the tail per unit
        const int at = a.attend ? -1 : hs_pick(pk);
        ev = a.hs_named ? ev_in : (n > a.budget) ? at : -1;
        if (s == 0 && tid == 0) a.hs_evict[u] = ev;
      }
      const int fl = ev - k0;
      const bool here = fl >= 32 * tid && fl < 32 * tid + 32 && fl < nk;
      sm.c64[tid] = here ? 0ull : ~0ull;
      sm.cslot[tid] = here ? fl : -1;
    }
    if (!SCORE && do_x_any) {
      float qv[8], kv[8], lp = 0.f;
      unpack8(yq, qv);
      unpack8(yk, kv);
#pragma unroll
      for (int e = 0; e < 8; ++e) lp = fmaf(qv[e], kv[e], lp);
      lp = rows_sum_f(lp);
      if (kq == 0 && l16 < 8) sm.xlp[wl][l16] = lp;   // summed over the 4 waves after the barrier
      if (wl == 0) {
        if (l16 == 0 && a.hs) {
          if (kq < 2) *(uint4*)(lrec + DEC_CAND_KI + 4 * kq) = yki0;
        } else if (l16 == 0) {
          *(uint4*)(lrec + DEC_CAND_KI + 8 * kq) = yki0;
          *(uint4*)(lrec + DEC_CAND_KI + 8 * kq + 4) = yki1;
        }
        if (lane < 32) *(uint4*)(lrec + ((lane & 16) ? DEC_CAND_V : DEC_CAND_K) + 4 * l16) = ykv;
        if (lane == 0) {
          lrec[0] = 0xffffffffu;   // never ranked: the caller names the evicted slot, if any
          lrec[1] = 0xffffffffu;
          lrec[2] = (uint32_t)(n - 1);
          lrec[3] = (uint32_t)n;
          lrec[12] = (uint32_t)ypos;
        }
      }
    }
    // ---- raw logits of the wave's 2 tiles:  S[key][head] = K_tile . Q^T  (bf16 MFMA, fp32 acc);
    // they need no score, so they are taken while the scoring waves are still at work
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
      v4f acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const uint4 ka = kf[tt][c], qb = (l16 < G) ? qf[c] : make_uint4(0, 0, 0, 0);
        const v4s a0 = __builtin_bit_cast(v4s, make_uint2(ka.x, ka.y));
        const v4s a1 = __builtin_bit_cast(v4s, make_uint2(ka.z, ka.w));
        const v4s b0 = __builtin_bit_cast(v4s, make_uint2(qb.x, qb.y));
        const v4s b1 = __builtin_bit_cast(v4s, make_uint2(qb.z, qb.w));
        acc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a0, b0, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a1, b1, acc, 0, 0, 0);
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) sreg[tt][r] = acc[r] * a.scale;   // this lane: head l16, key 16 T + 4 kq + r
    }
  }
  __syncthreads();
  // ---- the split's candidate: last-ranked over the 4 scoring waves (upwards with <= keeps the largest slot)
  int cl = -1;  // candidate's key index inside the split
  unsigned long long cbest = ~0ull;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const unsigned long long c = sm.c64[e];
    const int at = sm.cslot[e];
    if (at >= 0 && c <= cbest) { cbest = c; cl = at; }
  }
  // ---- attention waves: leave the candidate out, softmax statistics and probabilities PER WAVE
  // (each wave relative to the maximum of its own 32 keys; the final reduction rescales), P V
  float acc[G][8];
  if (!scoring) {
    float lmax = -INFINITY;
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
      const int T = 2 * wl + tt;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int kl = 16 * T + 4 * kq + r;  // this lane: head l16, key kl
        float sv = sreg[tt][r];
        if (kl == cl && l16 < G) sm.clog[l16] = sv;
        if (kl >= nk || kl == cl) sv = -INFINITY;
        sreg[tt][r] = sv;
        lmax = fmaxf(lmax, sv);
      }
    }
    lmax = rows_max_f(lmax);               // over the wave's 32 keys, per head (lane column)
    const float mw = (lmax == -INFINITY) ? -1e30f : lmax;
    float lsum = 0.f;
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
      const int T = 2 * wl + tt;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float p = (sreg[tt][r] == -INFINITY) ? 0.f : __expf(sreg[tt][r] - mw);
        lsum += p;
        if (l16 < 8) sm.pl[16 * T + 4 * kq + r][l16] = p;
      }
    }
    lsum = rows_sum_f(lsum);
    if (kq == 0 && l16 < 8) { sm.wm[wl][l16] = mw; sm.wl[wl][l16] = lsum; }
    // the candidate's rows travel with the record (straight from the fragments), so the tail has
    // no dependent loads; the split that holds the last live slot also fills the last-slot record
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
      const int T = 2 * wl + tt;
      if (16 * T + l16 == cl) {
#pragma unroll
        for (int c = 0; c < 4; ++c) *(uint4*)(crec + DEC_CAND_K + 16 * c + 4 * kq) = kf[tt][c];
      }
      if (own_last && 16 * T + l16 == ll) {
#pragma unroll
        for (int c = 0; c < 4; ++c) *(uint4*)(lrec + DEC_CAND_K + 16 * c + 4 * kq) = kf[tt][c];
      }
    }
    // the probabilities just written are this wave's own keys: read back without a workgroup barrier
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    // O[head][d] += P[head][key] V[key][d]; 16 lanes share a key row (8 dims each)
#pragma unroll
    for (int j = 0; j < G; ++j)
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[j][e] = 0.f;
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
      const int T = 2 * wl + tt;
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
    if (!SCORE && do_x_any && tid < G)   // the leftover key's logits: the 4 waves' partial dot products
      lrec[4 + tid] = __float_as_uint((sm.xlp[0][tid] + sm.xlp[1][tid] + sm.xlp[2][tid] + sm.xlp[3][tid]) * a.scale);
  } else if (SCORE && do_x_any && tid - 256 < G) {
    // the leftover key's logits: the 4 scoring waves' partial dot products
    const int j = tid - 256;
    lrec[4 + j] = __float_as_uint((sm.xlp[0][j] + sm.xlp[1][j] + sm.xlp[2][j] + sm.xlp[3][j]) * a.scale);
  }
  // the 16 (attention wave, key group) streams meet in LDS, 4 heads at a time; all 8 waves add them up
  float* prec = a.part + ((size_t)u * a.S_alloc + s) * G * DEC_REC;   // dense [split][head][record]
#pragma unroll
  for (int j0 = 0; j0 < G; j0 += 4) {
    if (j0 > 0) __syncthreads();
    if (!scoring) {
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        if (j0 + jj < G) {
          float* dst = &sm.oacc[wl * 4 + kq][jj][8 * l16];
          *(float4*)dst = make_float4(acc[j0 + jj][0], acc[j0 + jj][1], acc[j0 + jj][2], acc[j0 + jj][3]);
          *(float4*)(dst + 4) = make_float4(acc[j0 + jj][4], acc[j0 + jj][5], acc[j0 + jj][6], acc[j0 + jj][7]);
        }
      }
    }
    __syncthreads();
    const int nj = (G - j0 < 4) ? G - j0 : 4;
    for (int idx = tid; idx < nj * IM_D; idx += (SCORE ? DEC_MT : DEC_MT / 2)) {
      const int jj = idx >> 7, d = idx & 127, j = j0 + jj;
      // every wave's partial is relative to its own maximum: rescale to the split's
      const float m = fmaxf(fmaxf(sm.wm[0][j], sm.wm[1][j]), fmaxf(sm.wm[2][j], sm.wm[3][j]));
      float o = 0.f, l = 0.f;
#pragma unroll
      for (int wv = 0; wv < 4; ++wv) {
        const float sc = __expf(sm.wm[wv][j] - m);
        o = fmaf(sc, (sm.oacc[4 * wv][jj][d] + sm.oacc[4 * wv + 1][jj][d]) +
                     (sm.oacc[4 * wv + 2][jj][d] + sm.oacc[4 * wv + 3][jj][d]), o);
        l = fmaf(sc, sm.wl[wv][j], l);
      }
      prec[j * DEC_REC + 2 + d] = o;
      if (d == 0) {
        prec[j * DEC_REC] = m;
        prec[j * DEC_REC + 1] = l;
      }
    }
  }
  if (tid == 0) {
    crec[0] = (uint32_t)(cbest >> 32);
    crec[1] = (uint32_t)cbest;
    crec[2] = (uint32_t)(k0 + cl);
    crec[3] = (uint32_t)n;
    crec[13] = (uint32_t)n_true;
  }
  if (tid < G) crec[4 + tid] = __float_as_uint(cl >= 0 ? sm.clog[tid] : -INFINITY);   // -inf: no candidate
  if (!SCORE && own_last) {
    if (tid < a.di / 8) *(uint4*)(lrec + DEC_CAND_KI + 4 * tid) = lkx;
    if (tid == 8) { lrec[2] = (uint32_t)(n - 1); lrec[3] = (uint32_t)n; lrec[12] = (uint32_t)lpos; }
  }
  if (!scoring) {
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
      const int T = 2 * wl + tt;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int vr = 16 * T + 4 * i + kq;
        if (vr == cl) *(uint4*)(crec + DEC_CAND_V + 4 * l16) = vf[tt][i];
        if (own_last && vr == ll) *(uint4*)(lrec + DEC_CAND_V + 4 * l16) = vf[tt][i];
      }
    }
  }
}

#define DEC_TT 1024   // threads of a tail workgroup: the tail is a chain of short phases, so it is
                      // spread thin over 16 waves of one CU

// CHW: splits staged per round; a thread of a head group of up to 4 handles CHW / 2 of them per
// round, so the host picks the smallest CHW that holds the launch's splits
template <int G, int CHW>
struct DecTailSmem {
  static constexpr int CH = CHW;                 // splits staged per round
  static constexpr int NS = (G <= 4) ? 2 : 1;    // threads sharing one output in the merge
  float pst[CH][G][DEC_REC];                      // partial records of the staged splits
  uint32_t cst[CH + 1][DEC_CAND];                 // their candidate records (+ the last-slot record)
  float phq[G][IM_DM];                            // the unit's readout terms, in the order k_dec_prep
  float rpart[DEC_MP][G][IM_D];                   //   writes them: these five arrays are one block
  float gate[G];
  float unused[G];
  float denp[DEC_MP][G];
  float mrg[3][G * IM_D];                         // second half's (max, denominator, numerator) in the merge
  float phe2[8][IM_DM], phe[IM_DM];
  float den[G], dot[G];
  unsigned long long c64[16];
  int cidx[16];
  int e_slot, e_split;
};

// copy `count` floats (count even, both sides 8-byte aligned), every load in flight before the
// first store; one round handles DEC_TT * 2 * NB floats
template <int NB>
__device__ __forceinline__ void dec_stage(float* dst, const float* __restrict__ src, int count) {
  const int n2 = count >> 1;
  if (n2 <= 0) return;
  for (int base = 0; base < n2; base += DEC_TT * NB) {
    float2 r[NB];
#pragma unroll
    for (int k = 0; k < NB; ++k) {
      const int i = base + threadIdx.x + DEC_TT * k;
      r[k] = ((const float2*)src)[min(i, n2 - 1)];   // clamped: no branch around the load
    }
#pragma unroll
    for (int k = 0; k < NB; ++k) {
      const int i = base + threadIdx.x + DEC_TT * k;
      if (i < n2) ((float2*)dst)[i] = r[k];
    }
  }
}

template <int G, int CHW>
__device__ __forceinline__ void dec_tail(const DecArgs& a, const int u, DecTailSmem<G, CHW>& sm) {
  constexpr int CH = DecTailSmem<G, CHW>::CH;
  constexpr int NS = DecTailSmem<G, CHW>::NS;
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);   // a scalar, so that branches on the wave's role are uniform
  const int b = u / a.H_kv, h = u % a.H_kv;
  const uint32_t* cbase = a.cand + (size_t)u * a.S_alloc * DEC_CAND;
  const float* pbase = a.part + (size_t)u * a.S_alloc * G * DEC_REC;
  // ---------------- every load is issued now: no address depends on another load ----------------
  const int d4 = tid & 31, rg = tid >> 5;    // this thread's patch of M: rows 4 rg .. 4 rg + 3, columns 4 d4 .. 4 d4 + 3
  float* Mu = a.M + (size_t)u * IM_DM * IM_D;
  const int wc = tid & 127, hh = tid >> 7;   // W_theta row wc, dims 16 hh .. 16 hh + 15
  // first round of split records (all launched splits; which are live is known once n is read
  // from record 0), the last-slot record, and the readout terms of the queries
  const int cs0 = min(CH, a.S);
  const int LS = a.S;                          // index of the last-slot record
  const int LSI = min(LS, CH);                 // where it is staged
  {
    // one batch: every load of the regions is in flight before the first LDS store
    constexpr int NBP = (CH * G * DEC_REC / 2 + DEC_TT - 1) / DEC_TT;
    constexpr int NBC = (CH * DEC_CAND / 2 + DEC_TT - 1) / DEC_TT;
    constexpr int NBQ = (G * DEC_QM / 2 + DEC_TT - 1) / DEC_TT;
    const int np2 = cs0 * G * DEC_REC / 2, nc2 = cs0 * DEC_CAND / 2;
    constexpr int nq2 = G * DEC_QM / 2;
    const float2* qsrc = (const float2*)(a.qm + (size_t)u * G * DEC_QM);
    float2 rp[NBP], rc[NBC], rq[NBQ];
    const float2 rl = ((const float2*)(cbase + (size_t)LS * DEC_CAND))[min(tid, DEC_CAND / 2 - 1)];
#pragma unroll
    for (int k = 0; k < NBP; ++k) rp[k] = ((const float2*)pbase)[min(tid + DEC_TT * k, np2 - 1)];
#pragma unroll
    for (int k = 0; k < NBC; ++k) rc[k] = ((const float2*)cbase)[min(tid + DEC_TT * k, nc2 - 1)];
#pragma unroll
    for (int k = 0; k < NBQ; ++k) rq[k] = qsrc[min(tid + DEC_TT * k, nq2 - 1)];
    __asm__ volatile("" ::: "memory");
    if (tid < DEC_CAND / 2) ((float2*)&sm.cst[LSI][0])[tid] = rl;
#pragma unroll
    for (int k = 0; k < NBC; ++k)
      if (tid + DEC_TT * k < nc2) ((float2*)&sm.cst[0][0])[tid + DEC_TT * k] = rc[k];
#pragma unroll
    for (int k = 0; k < NBP; ++k)
      if (tid + DEC_TT * k < np2) ((float2*)&sm.pst[0][0][0])[tid + DEC_TT * k] = rp[k];
#pragma unroll
    for (int k = 0; k < NBQ; ++k)
      if (tid + DEC_TT * k < nq2) ((float2*)&sm.phq[0][0])[tid + DEC_TT * k] = rq[k];
  }
  // the memory state and W_theta are used further down (rank-one update, phi_e): their loads go out
  // behind the staging batch, whose registers are free again (issued with it, they delay it: measured)
  float4 Mr[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) Mr[i] = *(const float4*)(Mu + (rg * 4 + i) * IM_D + 4 * d4);
  const uint4 Wr0 = *(const uint4*)(a.Wt + wc * IM_D + hh * 16);
  const uint4 Wr1 = *(const uint4*)(a.Wt + wc * IM_D + hh * 16 + 8);
  const float b_old = a.bvec[(size_t)u * IM_DM + wc];
  __syncthreads();
  const int n = (int)sm.cst[0][3];
  // a unit longer than the caller's promise (flagged by the prep launch) evicts nothing and keeps its
  // true length: the entries beyond max_live were not looked at
  const int n_true = (int)sm.cst[0][13];
  const bool over = n_true > n;
  const int n_act = min((n + DEC_KEYS - 1) / DEC_KEYS, a.S);
  const bool has_x = n > a.S * DEC_KEYS;      // one key beyond the splits: described by the last-slot record
  const int n_last = n - 1;
  const uint32_t* lsrec = (const uint32_t*)&sm.cst[LSI][0];
  const int x_split = has_x ? n_act : -2;   // index the leftover key goes by in the ranking
  const int cn0 = min(CH, n_act);
  const bool evict = n > a.budget && !over;
  // ---------------- the evicted entry: ranked last over all splits and the leftover key ----------------
  if (n_act > CH) {   // rare: more splits than one staged round; their rank keys come from global memory
    unsigned long long best = ~0ull;
    int bidx = -1;
    for (int sp = CH + tid; sp < n_act; sp += DEC_TT) {
      const unsigned long long c = ((unsigned long long)cbase[(size_t)sp * DEC_CAND] << 32) | cbase[(size_t)sp * DEC_CAND + 1];
      if (c <= best) { best = c; bidx = sp; }   // later splits hold larger slots: they win full ties
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      const unsigned long long ob = __shfl_xor(best, o, 64);
      const int oi = __shfl_xor(bidx, o, 64);
      if (oi >= 0 && (bidx < 0 || ob < best || (ob == best && oi > bidx))) { best = ob; bidx = oi; }
    }
    if (lane == 0) { sm.c64[w] = best; sm.cidx[w] = bidx; }
    __syncthreads();
  }
  if (w == 0) {
    // smallest rank key over the staged candidates, lane = split; on a full tie the later split
    // (larger slot) wins
    const bool on = lane < cn0;
    const int ls = on ? lane : 0;
    const uint32_t khi = on ? sm.cst[ls][0] : 0xffffffffu;
    const uint32_t klo = on ? sm.cst[ls][1] : 0xffffffffu;
    const uint32_t mh = wave_min_u(khi);
    const uint32_t ml = wave_min_u(khi == mh ? klo : 0xffffffffu);
    const int win = (int)wave_max_u((on && khi == mh && klo == ml) ? (uint32_t)lane + 1u : 0u) - 1;
    if (lane == 0) {
      unsigned long long bb = ((unsigned long long)mh << 32) | ml;
      int bi = win;
      if (n_act > CH) {
        for (int i = 0; i < DEC_TT / 64; ++i) {
          const int oi = sm.cidx[i];
          if (oi >= 0 && (bi < 0 || sm.c64[i] < bb || (sm.c64[i] == bb && oi > bi))) { bb = sm.c64[i]; bi = oi; }
        }
      }
      if (has_x) {
        const unsigned long long xc = ((unsigned long long)lsrec[0] << 32) | lsrec[1];
        if (bi < 0 || xc <= bb) { bb = xc; bi = x_split; }
      }
      if (a.ext_evict) {   // the caller names the slot: the record of its split holds its rows
        const int e = a.ext_evict[u];
        const bool ev = e >= 0 && e < n && !over;
        sm.e_split = ev ? e / DEC_KEYS : -1;
        sm.e_slot = ev ? e : -1;
      } else {
        const bool ev = evict && bi >= 0;
        sm.e_split = ev ? bi : -1;
        sm.e_slot = !ev ? -1 : (bi == x_split) ? n_last : (int)((bi < CH) ? sm.cst[bi][2] : cbase[(size_t)bi * DEC_CAND + 2]);
        if (n > a.budget + 1) atomicOr(a.status, IM_STATUS_OVER_BUDGET_BIT);
      }
    }
  }
  // ---------------- merge, first pass: the attention partials of the staged splits ----------------
  // (does not depend on the eviction: it runs beside the ranking above)
  // NS threads share one output (head j, dim d): each takes CH / NS of the staged splits
  constexpr int NO = G * IM_D;                    // outputs
  constexpr int PER = CH / NS;                    // splits per thread and round
  const int oidx = (NS == 2) ? (tid & 511) : tid;
  const int part = (NS == 2) ? (tid >> 9) : 0;
  const bool act = oidx < NO;
  const int j = act ? (oidx >> 7) : 0, d = oidx & 127;
  constexpr int CK = (PER <= 8) ? PER : (PER % 8 == 0) ? 8 : (PER % 6 == 0) ? 6 : 4;   // splits folded at a time
  static_assert(PER % CK == 0, "the fold size divides the splits per thread");
  float rm = -1e30f, rl = 0.f, ro = 0.f;
#pragma unroll
  for (int k0 = 0; k0 < PER; k0 += CK) {
    // unconditional LDS reads (slots past cn0 hold stale words), then selects: no branches
    float pm[CK], plv[CK], po[CK];
#pragma unroll
    for (int k = 0; k < CK; ++k) {
      const int sp = part * PER + k0 + k;
      const float r0 = sm.pst[sp][j][0], r1 = sm.pst[sp][j][1], r2 = sm.pst[sp][j][2 + d];
      const bool on = sp < cn0;
      pm[k] = on ? r0 : -1e30f;
      plv[k] = on ? r1 : 0.f;
      po[k] = on ? r2 : 0.f;
    }
    float m = rm;
#pragma unroll
    for (int k = 0; k < CK; ++k) m = fmaxf(m, pm[k]);
    const float resc = __expf(rm - m);
    ro *= resc;
    rl *= resc;
#pragma unroll
    for (int k = 0; k < CK; ++k) {
      const float sc = __expf(pm[k] - m);
      ro = fmaf(sc, po[k], ro);
      rl = fmaf(sc, plv[k], rl);
    }
    rm = m;
  }
  __syncthreads();
  const int e_split = sm.e_split, e_slot = sm.e_slot;
  // the evicted entry's rows: in the staged record of its split or the last-slot record (LDS), or,
  // with more splits than one staging round holds, in its split's record in global memory
  const bool e_lds = (e_split == x_split) || (e_split < CH);
  const uint32_t* erl = (e_split == x_split) ? lsrec
                      : (const uint32_t*)&sm.cst[(e_split >= 0 && e_split < CH) ? e_split : 0][0];
  const uint32_t* erg = cbase + (size_t)max(e_split, 0) * DEC_CAND;
  // ---------------- memory write (rank one): phi_e = W_theta k_e, eight threads per row ----------------
  float ve_d = 0.f;
  float4 ve4 = make_float4(0.f, 0.f, 0.f, 0.f);
  if (e_slot >= 0) {
    uint4 k0, k1;
    uint2 t;
    if (e_lds) {
      k0 = *(const uint4*)(erl + DEC_CAND_K + 8 * hh);
      k1 = *(const uint4*)(erl + DEC_CAND_K + 8 * hh + 4);
      ve_d = bf2f(((const bf16_t*)(erl + DEC_CAND_V))[d]);
      t = *(const uint2*)(erl + DEC_CAND_V + 2 * d4);
    } else {
      k0 = *(const uint4*)(erg + DEC_CAND_K + 8 * hh);
      k1 = *(const uint4*)(erg + DEC_CAND_K + 8 * hh + 4);
      ve_d = bf2f(((const bf16_t*)(erg + DEC_CAND_V))[d]);
      t = *(const uint2*)(erg + DEC_CAND_V + 2 * d4);
    }
    ve4 = make_float4(bf_lo(t.x), bf_hi(t.x), bf_lo(t.y), bf_hi(t.y));
    float wv[16], kv[16];
    unpack8(Wr0, wv);
    unpack8(Wr1, wv + 8);
    unpack8(k0, kv);
    unpack8(k1, kv + 8);
    float pe = 0.f;
#pragma unroll
    for (int e = 0; e < 16; ++e) pe = fmaf(wv[e], kv[e], pe);
    sm.phe2[hh][wc] = pe;
  }
  // the last live slot's rows (they move into the hole): K, V and indexer-key rows are adjacent in the record
  uint4 mv = make_uint4(0, 0, 0, 0);
  if (tid < 40) mv = *(const uint4*)(lsrec + DEC_CAND_K + 4 * tid);
  if (a.kidx_in_cache && tid >= 32 && tid < 40 && n > 0)
    mv = *(const uint4*)(a.Kidx + ((size_t)u * a.C + (n - 1)) * IM_DI + (tid - 32) * 8);
  const int mvpos = (int)lsrec[12];
  // ---------------- merge, second pass: add back the candidates that stay ----------------
#pragma unroll
  for (int k0 = 0; k0 < PER; k0 += CK) {
    float cl[CK], cv[CK];
#pragma unroll
    for (int k = 0; k < CK; ++k) {
      const int sp = part * PER + k0 + k;
      const float r3 = __uint_as_float(sm.cst[sp][4 + j]);
      const float r4 = bf2f(((const bf16_t*)&sm.cst[sp][DEC_CAND_V])[d]);
      const bool stays = sp < cn0 && sp != e_split && r3 != -INFINITY;   // -inf: the split left nothing out
      cl[k] = stays ? r3 : -INFINITY;
      cv[k] = stays ? r4 : 0.f;
    }
    float m = rm;
#pragma unroll
    for (int k = 0; k < CK; ++k) m = fmaxf(m, cl[k]);
    const float resc = __expf(rm - m);
    float o = ro * resc, l = rl * resc;
#pragma unroll
    for (int k = 0; k < CK; ++k) {
      const float pc = __expf(cl[k] - m);   // exp(-inf) = 0 for the evicted / absent candidate
      o = fmaf(pc, cv[k], o);
      l += pc;
    }
    rm = m; rl = l; ro = o;
  }
  if (has_x && e_split != x_split && part == 0) {   // the leftover key stays
    const float xl = __uint_as_float(lsrec[4 + j]);
    const float xv = bf2f(((const bf16_t*)(lsrec + DEC_CAND_V))[d]);
    const float mn = fmaxf(rm, xl);
    const float resc = __expf(rm - mn), pc = __expf(xl - mn);
    ro = fmaf(pc, xv, ro * resc);
    rl = fmaf(rl, resc, pc);
    rm = mn;
  }
  // splits beyond the first staged round (none in the usual case): restage, both passes at once
  for (int c0 = CH; c0 < n_act; c0 += CH) {
    const int cn = min(CH, n_act - c0);
    __syncthreads();
    dec_stage<5>(&sm.pst[0][0][0], pbase + (size_t)c0 * G * DEC_REC, cn * G * DEC_REC);
    dec_stage<2>((float*)&sm.cst[0][0], (const float*)(cbase + (size_t)c0 * DEC_CAND), cn * DEC_CAND);
    __syncthreads();
#pragma unroll
    for (int k0 = 0; k0 < PER; k0 += CK) {
      float pm[CK], plv[CK], po[CK], cl[CK], cv[CK];
#pragma unroll
      for (int k = 0; k < CK; ++k) {
        const int sp = part * PER + k0 + k;
        const float r0 = sm.pst[sp][j][0], r1 = sm.pst[sp][j][1], r2 = sm.pst[sp][j][2 + d];
        const float r3 = __uint_as_float(sm.cst[sp][4 + j]);
        const float r4 = bf2f(((const bf16_t*)&sm.cst[sp][DEC_CAND_V])[d]);
        const bool on = sp < cn;
        const bool stays = on && (c0 + sp != e_split) && r3 != -INFINITY;
        pm[k] = on ? r0 : -1e30f;
        plv[k] = on ? r1 : 0.f;
        po[k] = on ? r2 : 0.f;
        cl[k] = stays ? r3 : -INFINITY;
        cv[k] = stays ? r4 : 0.f;
      }
      float m = rm;
#pragma unroll
      for (int k = 0; k < CK; ++k) m = fmaxf(m, fmaxf(pm[k], cl[k]));
      const float resc = __expf(rm - m);
      float o = ro * resc, l = rl * resc;
#pragma unroll
      for (int k = 0; k < CK; ++k) {
        const float sc = __expf(pm[k] - m);
        o = fmaf(sc, po[k], o);
        l = fmaf(sc, plv[k], l);
        const float pc = __expf(cl[k] - m);
        o = fmaf(pc, cv[k], o);
        l += pc;
      }
      rm = m; rl = l; ro = o;
    }
  }
  if (NS == 2) {
    if (part == 1 && act) { sm.mrg[0][oidx] = rm; sm.mrg[1][oidx] = rl; sm.mrg[2][oidx] = ro; }
  }
  __syncthreads();
  if (w >= 16 - G) {   // one wave per head: phi_q . phi_e and the readout's denominator
    const int jj = 15 - w;
    float dn = 0.f, dt = 0.f;
#pragma unroll
    for (int k = 0; k < DEC_MP; ++k) dn += sm.denp[k][jj];
    if (e_slot >= 0) {
      float p0 = 0.f, p1 = 0.f;
#pragma unroll
      for (int k = 0; k < 8; ++k) { p0 += sm.phe2[k][lane]; p1 += sm.phe2[k][lane + 64]; }
      const float q0 = sm.phq[jj][lane], q1 = sm.phq[jj][lane + 64];
      dt = wave_sum_f(fmaf(q0, p0, q1 * p1));
      const float sq = wave_sum_f(fmaf(q0 * q0, p0 * p0, q1 * q1 * p1 * p1));
      dn = fmaf(a.lambda, dn, a.eta * sq);
    }
    if (lane == 0) { sm.den[jj] = dn + a.mem_eps; sm.dot[jj] = dt; }
  } else if (w >= 6 && w < 8 && e_slot >= 0) {   // b <- lambda b + eta phi_e^2 (wc = tid - 384 here)
    float pe = 0.f;
#pragma unroll
    for (int k = 0; k < 8; ++k) pe += sm.phe2[k][wc];
    sm.phe[wc] = pe;
    a.bvec[(size_t)u * IM_DM + wc] = fmaf(a.lambda, b_old, a.eta * pe * pe);
  }
  float o_attn = 0.f;
  if (part == 0 && act) {
    float m = rm, o = ro, l = rl;
    if (NS == 2) {
      const float m2 = sm.mrg[0][oidx];
      const float mn = fmaxf(m, m2);
      const float s1 = __expf(m - mn), s2 = __expf(m2 - mn);
      o = fmaf(o, s1, s2 * sm.mrg[2][oidx]);
      l = fmaf(l, s1, s2 * sm.mrg[1][oidx]);
    }
    o_attn = (l > 0.f) ? o / l : 0.f;
  }
  __syncthreads();
  if (part == 0 && act) {
    // phi_q^T (lambda M + eta phi_e v_e^T) = lambda phi_q^T M + eta (phi_q . phi_e) v_e
    float mr = 0.f;
#pragma unroll
    for (int k = 0; k < DEC_MP; ++k) mr += sm.rpart[k][j][d];
    if (e_slot >= 0) mr = fmaf(a.lambda, mr, a.eta * sm.dot[j] * ve_d);
    const float res = sm.gate[j] * (mr / sm.den[j]);
    const size_t oi = ((size_t)b * a.H + h * G + j) * IM_D + d;
    a.out[oi] = f2bf_rne(o_attn + res);
    if (a.readout) a.readout[oi] = res;
  }
  if (e_slot >= 0) {
    // M <- lambda M + eta phi_e v_e^T for this thread's 4 x 4 patch
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float f = a.eta * sm.phe[rg * 4 + i];
      float4 m = Mr[i];
      m.x = fmaf(a.lambda, m.x, f * ve4.x); m.y = fmaf(a.lambda, m.y, f * ve4.y);
      m.z = fmaf(a.lambda, m.z, f * ve4.z); m.w = fmaf(a.lambda, m.w, f * ve4.w);
      *(float4*)(Mu + (rg * 4 + i) * IM_D + 4 * d4) = m;
    }
  }
  // ---------------- fill the hole with the last entry, publish the new length ----------------
  const int n_keep = (e_slot >= 0) ? n - 1 : n;
  if (e_slot >= 0 && e_slot < n_keep) {
    const size_t dst = (size_t)u * a.C + e_slot;
    if (tid < 16) *(uint4*)(a.K + dst * IM_D + tid * 8) = mv;
    else if (tid < 32) *(uint4*)(a.V + dst * IM_D + (tid - 16) * 8) = mv;
    else if (tid < 40) *(uint4*)(a.Kidx + dst * IM_DI + (tid - 32) * 8) = mv;
    else if (tid == 40) a.pos[dst] = mvpos;
  }
  if (tid == 0) {
    a.len[u] = over ? n_true : n_keep;
    a.nproj[u] = over ? n_true : n_keep;
    if (a.evicted) a.evicted[u] = e_slot;
  }
}

// --------------------------------------------------------------------------------------------
// k_dec_tail_head: the tail with one workgroup per (unit, query head), for launches whose units x
// heads fit the chip once (at most one such workgroup per CU).  Every workgroup ranks the
// candidates and forms phi_e for itself; it merges only its head's partials, 8 threads per output;
// the unit's workgroups share the rows of the memory update, and that of head 0 also fills the hole
// and publishes the length.  CHW (a multiple of 8, at most 64) must hold every split of the launch.
// --------------------------------------------------------------------------------------------
template <int CHW>
struct DecTailHeadSmem {
  float pst[CHW][DEC_REC];                        // this head's partial records
  uint32_t cst[CHW + 1][DEC_CAND];                // candidate records (+ the last-slot record)
  float phq[IM_DM];                               // this head's readout terms from k_dec_prep
  float rpart[DEC_MP][IM_D];
  float sc[8];                                    // gate, then DEC_MP partial phi_q^2 . b
  float mrg[3][8][IM_D];                          // (max, denominator, numerator) of the 8 thread groups
  float phe2[8][IM_DM], phe[IM_DM];
  float den, dot;
  int e_slot, e_split;
  float hk[8][IM_D], hv[8][IM_D];                 // head-shared layout: the evicted rows of the set's heads,
  float kbar[IM_D], vbar[IM_D];                   // and their sums over the heads
};

template <int G, int CHW>
__device__ __forceinline__ void dec_tail_head(const DecArgs& a, const int u, const int j, DecTailHeadSmem<CHW>& sm) {
  constexpr int CH = CHW, PER = CH / 8;
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);   // a scalar, so that branches on the wave's role are uniform
  const int b = u / a.H_kv, h = u % a.H_kv;
  const uint32_t* cbase = a.cand + (size_t)u * a.S_alloc * DEC_CAND;
  const float* pbase = a.part + (size_t)u * a.S_alloc * G * DEC_REC;
  const int su = u / a.H_set;                // the set that owns the lengths, indexer keys and the memory
  const bool lead = u % a.H_set == 0;        // ... and the unit that updates them
  const int d4 = tid & 31, rg = tid >> 5;    // this thread's part of M: row group rg, columns 4 d4 .. 4 d4 + 3
  float* Mu = a.M + (size_t)su * IM_DM * IM_D;
  const int wc = tid & 127, hh = tid >> 7;   // W_theta row wc, dims 16 hh .. 16 hh + 15
  const int cs0 = min(CH, a.S);
  const int LS = min(a.S, CH);               // index (and staged slot) of the last-slot record
  // The rank-one update of M is shared by the G head workgroups of the unit that owns the memory (rows
  // MROWS j .. MROWS j + MROWS - 1 each) when G divides 128; else head 0 takes all rows.
  constexpr int MROWS = (IM_DM % G == 0) ? IM_DM / G : IM_DM;
  constexpr int MPT = (MROWS + 31) / 32;          // rows per thread (thread = (row group tid >> 5, 4 columns tid & 31))
  const bool m_mine = lead && ((IM_DM % G == 0) || j == 0);
  const int m_row0 = (IM_DM % G == 0) ? MROWS * j : 0;
  float4 Mr[MPT] = {};
  float b_old = 0.f;
  const bool writer = j == 0 && lead;   // uniform per workgroup: it updates b, fills the hole, publishes the length
  uint4 Wr0, Wr1;
  // the loads of the later phases (this thread's patch of M, b, its piece of W_theta) go out with the
  // staging batch when that is small, else behind it: next to a long batch they delay the records the
  // first phases wait for (measured: 8 splits gain 1 %, 16 splits lose 2 %)
  constexpr bool ML_EARLY = CHW <= 8;
  auto later_loads = [&]() {
    if (m_mine) {
#pragma unroll
      for (int i = 0; i < MPT; ++i)
        if (rg + 32 * i < MROWS) Mr[i] = *(const float4*)(Mu + (m_row0 + rg + 32 * i) * IM_D + 4 * d4);
    }
    if (writer) b_old = a.bvec[(size_t)su * IM_DM + wc];
    Wr0 = *(const uint4*)(a.Wt + wc * IM_D + hh * 16);
    Wr1 = *(const uint4*)(a.Wt + wc * IM_D + hh * 16 + 8);
  };
  {
    // one batch: every load of the regions is in flight before the first LDS store
    constexpr int NBP = (CH * (DEC_REC / 2) + DEC_TT - 1) / DEC_TT;
    constexpr int NBC = (CH * DEC_CAND / 2 + DEC_TT - 1) / DEC_TT;
    const int np2 = cs0 * (DEC_REC / 2), nc2 = cs0 * DEC_CAND / 2;
    float2 rp[NBP], rc[NBC];
    const float2 rl = ((const float2*)(cbase + (size_t)LS * DEC_CAND))[min(tid, DEC_CAND / 2 - 1)];
#pragma unroll
    for (int k = 0; k < NBP; ++k) {
      const int idx = min(tid + DEC_TT * k, np2 - 1), sp = idx / (DEC_REC / 2), o = idx % (DEC_REC / 2);
      rp[k] = ((const float2*)(pbase + ((size_t)sp * G + j) * DEC_REC))[o];
    }
#pragma unroll
    for (int k = 0; k < NBC; ++k) rc[k] = ((const float2*)cbase)[min(tid + DEC_TT * k, nc2 - 1)];
    // readout terms of head j: phi_q (64 pairs), the DEC_MP partial phi_q^T M (64 pairs each), 5 scalars
    const float* qb = a.qm + (size_t)u * G * DEC_QM;
    const int t2 = min(tid, 64 * (1 + DEC_MP) - 1), pp = (t2 - 64) / 64, oo = (t2 - 64) % 64;
    const float* qsrc = (t2 < 64) ? qb + j * IM_DM + 2 * t2 : qb + G * IM_DM + ((size_t)pp * G + j) * IM_D + 2 * oo;
    const float2 rq = *(const float2*)qsrc;
    const int t3 = min(max(tid - 64 * (1 + DEC_MP), 0), DEC_MP);
    const float rs = qb[(t3 == 0) ? G * (IM_DM + DEC_MP * IM_D) + j : G * (IM_DM + DEC_MP * IM_D + 2) + (t3 - 1) * G + j];
    // head-shared layout: the memory takes the evicted rows summed over the set's heads (Algorithm 1,
    // `mem_write`).  The slot is named before the launch, so every head's copy of the rows (in the
    // candidate record of the slot's split, or the last-slot record) is fetched with the staging loads.
    float hks = 0.f, hvs = 0.f;
    if (a.hs) {
      const int e_raw = a.ext_evict[u];
      const int rec = (e_raw >= 0) ? min(e_raw / DEC_KEYS, LS) : 0;
#pragma unroll
      for (int it = 0; it < 2; ++it) {   // heads (tid >> 7) and (tid >> 7) + 8; absent ones re-read the last, unused
        const int hh = (tid >> 7) + 8 * it;
        const uint32_t* r = a.cand + ((size_t)(su * a.H_set + min(hh, a.H_set - 1)) * a.S_alloc + rec) * DEC_CAND;
        const float kx = bf2f(((const bf16_t*)(r + DEC_CAND_K))[tid & 127]);
        const float vx = bf2f(((const bf16_t*)(r + DEC_CAND_V))[tid & 127]);
        hks += (hh < a.H_set) ? kx : 0.f;
        hvs += (hh < a.H_set) ? vx : 0.f;
      }
    }
    if constexpr (ML_EARLY) later_loads();
    __asm__ volatile("" ::: "memory");
    if (a.hs) { sm.hk[tid >> 7][tid & 127] = hks; sm.hv[tid >> 7][tid & 127] = hvs; }
    if (tid < DEC_CAND / 2) ((float2*)&sm.cst[LS][0])[tid] = rl;
#pragma unroll
    for (int k = 0; k < NBC; ++k)
      if (tid + DEC_TT * k < nc2) ((float2*)&sm.cst[0][0])[tid + DEC_TT * k] = rc[k];
#pragma unroll
    for (int k = 0; k < NBP; ++k)
      if (tid + DEC_TT * k < np2) ((float2*)&sm.pst[0][0])[tid + DEC_TT * k] = rp[k];
    if (tid < 64) ((float2*)&sm.phq[0])[tid] = rq;
    else if (tid < 64 * (1 + DEC_MP)) ((float2*)&sm.rpart[0][0])[tid - 64] = rq;
    else if (tid <= 64 * (1 + DEC_MP) + DEC_MP) sm.sc[t3] = rs;
  }
  // attend-only / follower step of the head-shared layout: nothing scored the new token, so its
  // indexer key Norm(U_k x) is made here (one 16-lane row of the writer workgroup) and stored at the
  // end, where the token's final slot is known
  bf16_t new_key = 0;
  const bool new_fits = a.attend && writer && a.len[su] + 1 <= a.C;   // the append took place
  if (new_fits && tid >= 128 && tid < 128 + IM_DI_SHARED) {
    const int dd = tid - 128, bq = u / a.H_kv;
    const double v = a.xk[(size_t)bq * IM_DI_SHARED + dd];
    const double ss = row16_sum_d(v * v);
    const double rr = sqrt(ss / (double)IM_DI_SHARED + (double)a.rms_eps);
    const double wk = a.nkw ? (double)bf2f(a.nkw[dd]) : 1.0;
    new_key = d2bf_rne(v / rr * wk);
  }
  if constexpr (!ML_EARLY) later_loads();
  __syncthreads();
  const int n = (int)sm.cst[0][3];
  const int n_true = (int)sm.cst[0][13];      // above n only if the live-length promise is broken: then
  const bool over = n_true > n;               // nothing is evicted and the true length stays
  const int n_act = min((n + DEC_KEYS - 1) / DEC_KEYS, a.S);
  const bool has_x = n > a.S * DEC_KEYS;      // one key beyond the splits: described by the last-slot record
  const uint32_t* lsrec = (const uint32_t*)&sm.cst[LS][0];
  const int x_split = has_x ? n_act : -2;
  const int cn0 = min(CH, n_act);
  if (w == 0) {
    // smallest rank key over the candidates, lane = split; on a full tie the later split wins
    const bool on = lane < cn0;
    const int ls = on ? lane : 0;
    const uint32_t khi = on ? sm.cst[ls][0] : 0xffffffffu;
    const uint32_t klo = on ? sm.cst[ls][1] : 0xffffffffu;
    const uint32_t mh = wave_min_u(khi);
    const uint32_t ml = wave_min_u(khi == mh ? klo : 0xffffffffu);
    const int win = (int)wave_max_u((on && khi == mh && klo == ml) ? (uint32_t)lane + 1u : 0u) - 1;
    if (lane == 0) {
      if (a.ext_evict) {   // the caller names the slot: the record of its split holds its rows
        const int e = a.ext_evict[u];
        const bool ev = e >= 0 && e < n && !over;
        sm.e_split = ev ? e / DEC_KEYS : -1;
        sm.e_slot = ev ? e : -1;
      } else {
        unsigned long long bb = ((unsigned long long)mh << 32) | ml;
        int bi = win;
        if (has_x) {
          const unsigned long long xc = ((unsigned long long)lsrec[0] << 32) | lsrec[1];
          if (bi < 0 || xc <= bb) { bb = xc; bi = x_split; }
        }
        const bool ev = n > a.budget && bi >= 0 && !over;
        sm.e_split = ev ? bi : -1;
        sm.e_slot = !ev ? -1 : (bi == x_split) ? n - 1 : (int)sm.cst[bi][2];
        if (j == 0 && n > a.budget + 1) atomicOr(a.status, IM_STATUS_OVER_BUDGET_BIT);
      }
    }
  }
  if (a.hs && tid >= 768) {   // (waves 12-15) the rows' sums over the heads
    const int dd = tid & 127;
    float t = 0.f;
    if (tid < 896) {
#pragma unroll
      for (int p = 0; p < 8; ++p) t += sm.hk[p][dd];
      sm.kbar[dd] = t;
    } else {
#pragma unroll
      for (int p = 0; p < 8; ++p) t += sm.hv[p][dd];
      sm.vbar[dd] = t;
    }
  }
  // merge, first pass (beside the ranking): this thread's PER splits of output d
  const int d = tid & 127, part = tid >> 7;
  float rm = -1e30f, rl = 0.f, ro = 0.f;
  {
    float pm[PER], plv[PER], po[PER];
#pragma unroll
    for (int k = 0; k < PER; ++k) {
      const int sp = part * PER + k;
      const float r0 = sm.pst[sp][0], r1 = sm.pst[sp][1], r2 = sm.pst[sp][2 + d];
      const bool on = sp < cn0;
      pm[k] = on ? r0 : -1e30f;
      plv[k] = on ? r1 : 0.f;
      po[k] = on ? r2 : 0.f;
    }
#pragma unroll
    for (int k = 0; k < PER; ++k) rm = fmaxf(rm, pm[k]);
#pragma unroll
    for (int k = 0; k < PER; ++k) {
      const float s = __expf(pm[k] - rm);
      ro = fmaf(s, po[k], ro);
      rl = fmaf(s, plv[k], rl);
    }
  }
  __syncthreads();
  const int e_split = sm.e_split, e_slot = sm.e_slot;
  const uint32_t* er = (e_split == x_split) ? lsrec : (const uint32_t*)&sm.cst[max(e_split, 0)][0];
  float ve_d = 0.f;
  float4 ve4 = make_float4(0.f, 0.f, 0.f, 0.f);
  if (e_slot >= 0) {   // phi_e = W_theta k_e, eight threads per row
    float wv[16], kv[16];
    unpack8(Wr0, wv);
    unpack8(Wr1, wv + 8);
    if (a.hs) {
      ve_d = sm.vbar[d];
      ve4 = *(const float4*)&sm.vbar[4 * d4];
#pragma unroll
      for (int e = 0; e < 16; e += 4) *(float4*)&kv[e] = *(const float4*)&sm.kbar[16 * hh + e];
    } else {
      ve_d = bf2f(((const bf16_t*)(er + DEC_CAND_V))[d]);
      const uint2 t = *(const uint2*)(er + DEC_CAND_V + 2 * d4);
      ve4 = make_float4(bf_lo(t.x), bf_hi(t.x), bf_lo(t.y), bf_hi(t.y));
      unpack8(*(const uint4*)(er + DEC_CAND_K + 8 * hh), kv);
      unpack8(*(const uint4*)(er + DEC_CAND_K + 8 * hh + 4), kv + 8);
    }
    float pe = 0.f;
#pragma unroll
    for (int e = 0; e < 16; ++e) pe = fmaf(wv[e], kv[e], pe);
    sm.phe2[hh][wc] = pe;
  }
  uint4 mv = make_uint4(0, 0, 0, 0);           // the last live slot's rows (they move into the hole)
  if (tid < 40) mv = *(const uint4*)(lsrec + DEC_CAND_K + 4 * tid);
  if (a.kidx_in_cache && tid >= 32 && tid < 40 && n > 0)
    mv = *(const uint4*)(a.Kidx + ((size_t)u * a.C + (n - 1)) * IM_DI + (tid - 32) * 8);
  const int mvpos = (int)lsrec[12];
  {   // merge, second pass: add back the candidates that stay
    float cl[PER], cv[PER];
#pragma unroll
    for (int k = 0; k < PER; ++k) {
      const int sp = part * PER + k;
      const float r3 = __uint_as_float(sm.cst[sp][4 + j]);
      const float r4 = bf2f(((const bf16_t*)&sm.cst[sp][DEC_CAND_V])[d]);
      const bool stays = sp < cn0 && sp != e_split && r3 != -INFINITY;   // -inf: the split left nothing out
      cl[k] = stays ? r3 : -INFINITY;
      cv[k] = stays ? r4 : 0.f;
    }
    float m = rm;
#pragma unroll
    for (int k = 0; k < PER; ++k) m = fmaxf(m, cl[k]);
    const float resc = __expf(rm - m);
    float o = ro * resc, l = rl * resc;
#pragma unroll
    for (int k = 0; k < PER; ++k) {
      const float pc = __expf(cl[k] - m);
      o = fmaf(pc, cv[k], o);
      l += pc;
    }
    rm = m; rl = l; ro = o;
  }
  if (has_x && e_split != x_split && part == 0) {   // the leftover key stays
    const float xl = __uint_as_float(lsrec[4 + j]);
    const float xv = bf2f(((const bf16_t*)(lsrec + DEC_CAND_V))[d]);
    const float mn = fmaxf(rm, xl);
    const float resc = __expf(rm - mn), pc = __expf(xl - mn);
    ro = fmaf(pc, xv, ro * resc);
    rl = fmaf(rl, resc, pc);
    rm = mn;
  }
  sm.mrg[0][part][d] = rm; sm.mrg[1][part][d] = rl; sm.mrg[2][part][d] = ro;
  __syncthreads();
  if (w == 15) {   // phi_q . phi_e and the readout's denominator
    float dn = 0.f, dt = 0.f;
#pragma unroll
    for (int k = 0; k < DEC_MP; ++k) dn += sm.sc[1 + k];
    if (e_slot >= 0) {
      float p0 = 0.f, p1 = 0.f;
#pragma unroll
      for (int k = 0; k < 8; ++k) { p0 += sm.phe2[k][lane]; p1 += sm.phe2[k][lane + 64]; }
      const float q0 = sm.phq[lane], q1 = sm.phq[lane + 64];
      dt = wave_sum_f(fmaf(q0, p0, q1 * p1));
      const float sq = wave_sum_f(fmaf(q0 * q0, p0 * p0, q1 * q1 * p1 * p1));
      dn = fmaf(a.lambda, dn, a.eta * sq);
    }
    if (lane == 0) { sm.den = dn + a.mem_eps; sm.dot = dt; }
  } else if (m_mine && w >= 6 && w < 8 && e_slot >= 0) {   // phi_e; b <- lambda b + eta phi_e^2 (wc = tid - 384 here)
    float pe = 0.f;
#pragma unroll
    for (int k = 0; k < 8; ++k) pe += sm.phe2[k][wc];
    sm.phe[wc] = pe;
    if (writer) a.bvec[(size_t)su * IM_DM + wc] = fmaf(a.lambda, b_old, a.eta * pe * pe);
  }
  float o_attn = 0.f;
  if (tid < IM_D) {   // fold the 8 thread groups of output d
    float m = sm.mrg[0][0][d], l = sm.mrg[1][0][d], o = sm.mrg[2][0][d];
#pragma unroll
    for (int p = 1; p < 8; ++p) {
      const float m2 = sm.mrg[0][p][d], mn = fmaxf(m, m2);
      const float s1 = __expf(m - mn), s2 = __expf(m2 - mn);
      o = fmaf(o, s1, s2 * sm.mrg[2][p][d]);
      l = fmaf(l, s1, s2 * sm.mrg[1][p][d]);
      m = mn;
    }
    o_attn = (l > 0.f) ? o / l : 0.f;
  }
  __syncthreads();
  if (tid < IM_D) {
    // phi_q^T (lambda M + eta phi_e v_e^T) = lambda phi_q^T M + eta (phi_q . phi_e) v_e
    float mr = 0.f;
#pragma unroll
    for (int k = 0; k < DEC_MP; ++k) mr += sm.rpart[k][d];
    if (e_slot >= 0) mr = fmaf(a.lambda, mr, a.eta * sm.dot * ve_d);
    const float res = sm.sc[0] * (mr / sm.den);
    const size_t oi = ((size_t)b * a.H + h * G + j) * IM_D + d;
    a.out[oi] = f2bf_rne(o_attn + res);
    if (a.readout) a.readout[oi] = res;
  }
  if (e_slot >= 0 && m_mine) {
    // M <- lambda M + eta phi_e v_e^T for this thread's rows, 4 columns each
#pragma unroll
    for (int i = 0; i < MPT; ++i) {
      const int row = m_row0 + rg + 32 * i;
      if (rg + 32 * i < MROWS) {
        const float f = a.eta * sm.phe[row];
        float4 m = Mr[i];
        m.x = fmaf(a.lambda, m.x, f * ve4.x); m.y = fmaf(a.lambda, m.y, f * ve4.y);
        m.z = fmaf(a.lambda, m.z, f * ve4.z); m.w = fmaf(a.lambda, m.w, f * ve4.w);
        *(float4*)(Mu + row * IM_D + 4 * d4) = m;
      }
    }
  }
  if (j != 0) return;
  // fill the hole with the last entry, publish the new length
  const int n_keep = (e_slot >= 0) ? n - 1 : n;
  if (e_slot >= 0 && e_slot < n_keep) {
    const size_t dst = (size_t)u * a.C + e_slot, idst = (size_t)su * a.C + e_slot;
    if (tid < 16) *(uint4*)(a.K + dst * IM_D + tid * 8) = mv;
    else if (tid < 32) *(uint4*)(a.V + dst * IM_D + (tid - 16) * 8) = mv;
    else if (tid < 32 + a.di / 8) { if (lead && !new_fits) *(uint4*)(a.Kidx + idst * a.di + (tid - 32) * 8) = mv; }
    else if (tid == 40 && lead) a.pos[idst] = mvpos;
  }
  if (new_fits && tid >= 128 && tid < 128 + IM_DI_SHARED) {
    // the new token sits in the last live slot n - 1, unless that entry has just moved into the hole
    const int at = (e_slot >= 0 && e_slot < n_keep) ? e_slot : n_true - 1;
    if (!(e_slot == n - 1)) a.Kidx[((size_t)su * a.C + at) * IM_DI_SHARED + (tid - 128)] = new_key;
  }
  if (tid == 0 && lead) {
    a.len[su] = over ? n_true : n_keep;
    a.nproj[su] = over ? n_true : n_keep;
    if (a.evicted) a.evicted[su] = e_slot;
  }
}

// grid: units * S blocks; consecutive blocks take different units, the short last splits come last
template <int G>
__global__ __launch_bounds__(DEC_MT, 4) void k_dec_main(const DecArgs a, const double* __restrict__ qy,
                                                        const double* __restrict__ alpha) {
  __shared__ __attribute__((aligned(16))) DecSplitSmem sm;
  const int U = a.B * a.H_kv;
  dec_split<G, true>(a, blockIdx.x % U, blockIdx.x / U, sm, qy, alpha);
}

// the attend-only variant: same grid, 4 waves per workgroup
template <int G>
__global__ __launch_bounds__(DEC_MT / 2, G <= 4 ? 3 : 2) void k_att_main(const DecArgs a) {
  __shared__ __attribute__((aligned(16))) DecSplitSmem sm;
  const int U = a.B * a.H_kv;
  dec_split<G, false>(a, blockIdx.x % U, blockIdx.x / U, sm, nullptr, nullptr);
}

// grid: units
template <int G, int CHW>
__global__ __launch_bounds__(DEC_TT) void k_dec_tail(const DecArgs a) {
  __shared__ __attribute__((aligned(16))) DecTailSmem<G, CHW> sm;
  dec_tail<G, CHW>(a, blockIdx.x, sm);
}

// grid: units * G blocks, one per (unit, query head)
template <int G, int CHW>
__global__ __launch_bounds__(DEC_TT) void k_dec_tail_head(const DecArgs a) {
  __shared__ __attribute__((aligned(16))) DecTailHeadSmem<CHW> sm;
  int u, j;   // the unit's tail on the XCD whose L2 has just seen its records (xcd_unit_map)
  xcd_unit_map(blockIdx.x, G, a.B * a.H_kv, u, j);
  dec_tail_head<G, CHW>(a, u, j, sm);
}

// The attend-only split kernel with the prep roles in the same launch (they do not feed it: the
// split workgroups take the new token's rows from the inputs): role blocks first, then the
// (unit, split) workgroups.  Two launches per layer-step instead of three.
template <int G>
__global__ __launch_bounds__(DEC_MT / 2, G <= 4 ? 3 : 2) void k_att_merged(const DecArgs a, const int n_roles) {
  __shared__ __attribute__((aligned(16))) union SM { DecSplitSmem sm; DecPrepSmem ps; __device__ SM() {} } s;
  const int U = a.B * a.H_kv;
  if ((int)blockIdx.x >= n_roles) {
    const int blk = blockIdx.x - n_roles;
    dec_split<G, false, true>(a, blk % U, blk / U, s.sm, nullptr, nullptr);
    return;
  }
  const int r = blockIdx.x;
  if (r < U) {
    if (a.hs) hs_prep_unit(a, r); else dec_prep_unit(a, r, s.ps);
  } else if (r < (1 + DEC_MP) * U) {
    int mu, mp;
    xcd_unit_map(r - U, DEC_MP, U, mu, mp);
    dec_prep_memory(a, mu, mp, s.ps);
  } else {   // head-shared layout: the U_k rows
    hs_prep_gemv(a, r - (1 + DEC_MP) * U + a.H_idx * IM_DI_SHARED / 2 + (a.H_idx + 1) / 2, s.ps);
  }
}
