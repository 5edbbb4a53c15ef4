// Device-side bodies of the stage step and of the tree step (Sec. 3.1, 4.1 of the
// paper).
#pragma once
#include "merge.h"
#include "spec_internal.h"

namespace specdraft {

// One node (child row r) of a stage, computed by a whole workgroup of NT threads:
//   state = GELU(LayerNorm(w_s * (W s_parent) + w_e * Emb[token]))
// The token the node carries is the rank-th best of its parent's head row; that row's
// partial results are merged here (every sibling repeats the small merge, which saves
// a separate launch on the latency-critical batch-1 chain).
// NCH = 8-element chunks per thread held in registers (D <= NCH * NT * 8).
// `lds`: 32 + (NT / 256) * kMergeLds words of scratch.  Contains workgroup barriers.
// States are stored as whole 16-byte slots; the L2 gathers the eight rows that share a 128-byte line.
template <bool BF16, int NCH, int NT>
__device__ __forceinline__ void stage_row(const StageJob& j, int r, float* lds) {
  float* scratch = lds;                 // NT / 64 <= 16 words
  const int tid = opaque_tid(), lane = tid & 63;
  float* merge_lds = lds + 32 + (tid >> 8) * kMergeLds;
  int parent = r / j.k_prev, rank = r - parent * j.k_prev;
  if (j.row_parent) {  // per-sequence trees: the host laid the rows out
    parent = j.row_parent[r];
    rank = j.row_rank[r];
  }
  const int D = j.D, nchunk = D / 8;

  // everything that does not depend on the token is requested first: the
  // projected parent state and the LayerNorm affine
  const float* pz = j.pz + (int64_t)parent * D;
  float z[NCH][8], ga[NCH][8], be[NCH][8];
#pragma unroll
  for (int ci = 0; ci < NCH; ++ci) {
    const int c = tid + ci * NT;
    if (c < nchunk) {
      float4 p0 = *reinterpret_cast<const float4*>(pz + c * 8);
      float4 p1 = *reinterpret_cast<const float4*>(pz + c * 8 + 4);
      for (int q = 1; q < j.pz_parts; ++q) {  // a projection split along K: add the parts in order
        const float* pq = pz + q * j.pz_part_stride + c * 8;
        const float4 q0 = *reinterpret_cast<const float4*>(pq);
        const float4 q1 = *reinterpret_cast<const float4*>(pq + 4);
        p0.x += q0.x; p0.y += q0.y; p0.z += q0.z; p0.w += q0.w;
        p1.x += q1.x; p1.y += q1.y; p1.z += q1.z; p1.w += q1.w;
      }
      const float4 g0 = *reinterpret_cast<const float4*>(j.gamma + c * 8);
      const float4 g1 = *reinterpret_cast<const float4*>(j.gamma + c * 8 + 4);
      const float4 b0 = *reinterpret_cast<const float4*>(j.beta + c * 8);
      const float4 b1 = *reinterpret_cast<const float4*>(j.beta + c * 8 + 4);
      z[ci][0] = p0.x; z[ci][1] = p0.y; z[ci][2] = p0.z; z[ci][3] = p0.w;
      z[ci][4] = p1.x; z[ci][5] = p1.y; z[ci][6] = p1.z; z[ci][7] = p1.w;
      ga[ci][0] = g0.x; ga[ci][1] = g0.y; ga[ci][2] = g0.z; ga[ci][3] = g0.w;
      ga[ci][4] = g1.x; ga[ci][5] = g1.y; ga[ci][6] = g1.z; ga[ci][7] = g1.w;
      be[ci][0] = b0.x; be[ci][1] = b0.y; be[ci][2] = b0.z; be[ci][3] = b0.w;
      be[ci][4] = b1.x; be[ci][5] = b1.y; be[ci][6] = b1.z; be[ci][7] = b1.w;
    }
  }

  int tok;
  if (j.stage == 0) {
    tok = j.last_tok[parent];   // (uniform tree: parent == r)
  } else {
    float v[kMaxTopK];
    int32_t ix[kMaxTopK];
    float lse;
    // every 256-thread group merges the same parent row (one group would do; the
    // barriers inside need all of them anyway)
    group_merge_partials(j.part, parent, j.nparts, j.k_prev, v, ix, lse, merge_lds);
    tok = ix[0];
#pragma unroll
    for (int q = 1; q < kMaxTopK; ++q)
      if (q == rank) tok = ix[q];
    if (rank == 0 && tid < 64) {
#pragma unroll
      for (int q = 0; q < kMaxTopK; ++q)
        if (lane == q && q < j.k_prev) {
          j.prev_tok[(int64_t)parent * j.k_prev + q] = ix[q];
          j.prev_logp[(int64_t)parent * j.k_prev + q] = v[q] - lse;
        }
      if (lane == 0) j.prev_lse[parent] = lse;
    }
  }
  tok = min(max(tok, 0), j.V - 1);  // a wild token from the caller must not leave the table

  // gather + mix
  float lsum = 0.f;
#pragma unroll
  for (int ci = 0; ci < NCH; ++ci) {
    const int c = tid + ci * NT;
    if (c < nchunk) {
      float e[8];
      if (BF16) {
        const uint4 raw =
            *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(j.emb) + (int64_t)tok * D + c * 8);
        const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          e[2 * q] = bf16_bits_to_f32(w[q] & 0xffffu);
          e[2 * q + 1] = bf16_bits_to_f32(w[q] >> 16);
        }
      } else {
        const float* er = static_cast<const float*>(j.emb) + (int64_t)tok * D + c * 8;
        const float4 e0 = *reinterpret_cast<const float4*>(er);
        const float4 e1 = *reinterpret_cast<const float4*>(er + 4);
        e[0] = e0.x; e[1] = e0.y; e[2] = e0.z; e[3] = e0.w;
        e[4] = e1.x; e[5] = e1.y; e[6] = e1.z; e[7] = e1.w;
      }
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        z[ci][q] = j.w_s * z[ci][q] + j.w_e * e[q];
        lsum += z[ci][q];
      }
    }
  }
  const float mean = block_sum<NT>(lsum, scratch) / (float)D;
  float lvar = 0.f;
#pragma unroll
  for (int ci = 0; ci < NCH; ++ci) {
    if (tid + ci * NT < nchunk) {
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const float d = z[ci][q] - mean;
        lvar += d * d;
      }
    }
  }
  const float var = block_sum<NT>(lvar, scratch) / (float)D;
  const float rstd = 1.0f / sqrtf(var + j.eps);

#pragma unroll
  for (int ci = 0; ci < NCH; ++ci) {
    const int c = tid + ci * NT;
    if (c < nchunk) {
      float s[8];
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const float y = (z[ci][q] - mean) * rstd * ga[ci][q] + be[ci][q];
        s[q] = 0.5f * y * (1.0f + erf_as(y * 0.70710678118654752440f));
      }
      if (BF16) {
        uint4 o;
        o.x = f32_to_bf16_bits(s[0]) | (f32_to_bf16_bits(s[1]) << 16);
        o.y = f32_to_bf16_bits(s[2]) | (f32_to_bf16_bits(s[3]) << 16);
        o.z = f32_to_bf16_bits(s[4]) | (f32_to_bf16_bits(s[5]) << 16);
        o.w = f32_to_bf16_bits(s[6]) | (f32_to_bf16_bits(s[7]) << 16);
        // tiled layout: row tile r/16, column fragment c/4, lane slot (c%4)*16 + r%16
        const int64_t slot = ((int64_t)(r >> 4) * (D / 32) + (c >> 2)) * 64 + ((c & 3) << 4) + (r & 15);
        reinterpret_cast<uint4*>(j.state_out)[slot] = o;
        if (j.state_dbg) reinterpret_cast<uint4*>(j.state_dbg)[((int64_t)r * D) / 8 + c] = o;
      } else {
        float* so = static_cast<float*>(j.state_out) + (int64_t)r * D + c * 8;
        *reinterpret_cast<float4*>(so) = make_float4(s[0], s[1], s[2], s[3]);
        *reinterpret_cast<float4*>(so + 4) = make_float4(s[4], s[5], s[6], s[7]);
        if (j.state_dbg) {
          float* sd = static_cast<float*>(j.state_dbg) + (int64_t)r * D + c * 8;
          *reinterpret_cast<float4*>(sd) = make_float4(s[0], s[1], s[2], s[3]);
          *reinterpret_cast<float4*>(sd + 4) = make_float4(s[4], s[5], s[6], s[7]);
        }
      }
    }
  }
}

// Tree step for one sequence q, by a whole workgroup of NT threads: merge the last
// head's partial results, score every leaf by the sum of its tokens' log-probabilities
// (added in stage order), keep the B best.
struct TreeArgs {
  int n, B, B_pad, L, k_last, kw_last, nparts;
  int64_t off_last, row_off_last;   // the last stage's offsets in tok / logp and in lse
  int64_t rbase_last;               // first row of this sequence at the last stage
  Partials part;                    // last head
  int32_t* tok;                     // per-stage tables [R_i][width_i], concatenated
  float* logp;
  float* lse;
  int32_t* cand_tokens;
  float* cand_scores;
  int32_t* cand_leaf;
};

// One sequence q of the tree step, by a whole workgroup of NT threads.
// B candidates are kept out of L = prod(k_i) leaves; k_last = this sequence's branching at the last
// stage, kw_last = width of the last stage's tables and partial lists (>= k_last; equal for a uniform
// tree).  B = 0 (speculation off): only padding is written.
// s_k / s_off / s_rbase / s_kw: per stage, in LDS (indexing kernel arguments with a run-time stage
// number would make the compiler spill the argument block to scratch): this sequence's branching,
// the table's element offset, this sequence's first row, the table's width.
// sk: kMaxLeaves 64-bit words of LDS (the leaves' scores as keys, see best_key); merge_lds: (NT / 256) * kMergeLds words; c_tok / c_logp: kMaxLeaves words
// each, the last stage's tables of this sequence for the leaf scores (the tables in memory are written all
// the same: the debug outputs and the caller's next step read them).
// KWAVE: widest kw_last merged one row per wave (register-hungry for wide lists: a wave
// of a 1024-thread workgroup has 128 registers); wider ones are merged one row per
// 256-thread group.  Contains workgroup barriers.
template <int NT, int KWAVE>
__device__ __forceinline__ void tree_body(const TreeArgs& j, int q, const int* s_k, const int64_t* s_off,
                                          const int64_t* s_rbase, const int* s_kw, uint64_t* sk, float* merge_lds,
                                          int32_t* c_tok, float* c_logp) {
  const int tid = opaque_tid(), lane = tid & 63, wave = tid >> 6;
  const int n = j.n, L = j.L, kw = j.kw_last;
  const int rows_last = j.B > 0 ? L / j.k_last : 0;
  const int nleaf = j.B > 0 ? L : 0;

  // A leaf's path, walking up from the leaf: q_{n-1} = leaf, q_{i-1} = q_i / k_i; its node at stage i is
  // row q_{i-1} of the sequence with rank q_i - q_{i-1} k_i.  at[i] = element of stage i's table.
  // All of a leaf's table reads are issued together: one round trip, not one per stage.
  auto path_of = [&](int leaf, int64_t (&at)[kMaxStages]) {
    int q = leaf;
#pragma unroll
    for (int i = kMaxStages - 1; i >= 0; --i) {
      at[i] = 0;
      if (i < n) {
        const int k = s_k[i];
        // q < 4096, k <= 8: the float quotient of q + 1/2 is farther from an integer than its rounding error
        const int up = (int)(((float)q + 0.5f) * __frcp_rn((float)k));
        at[i] = s_off[i] + (s_rbase[i] + up) * s_kw[i] + (q - up * k);
        q = up;
      }
    }
  };
  // One leaf per thread and the last stage's tables small enough for LDS (the paper's trees): a leaf's
  // entries of the EARLIER stages are requested before the merge and arrive under it; the last stage's
  // come from the merge through LDS.  The leaf scores then wait for no memory at all.
  const bool one_pass = nleaf <= NT;   // every thread has at most one leaf: its tokens stay in registers
  constexpr int kEarly = 3;            // earlier stages whose entries a thread holds across the merge (registers)
  const bool early = one_pass && n - 1 <= kEarly && (int64_t)rows_last * kw <= kMaxLeaves;
  float lp_e[kEarly];
  int32_t tk_e[kEarly];
  int last_at = 0;
  if (early && tid < nleaf) {
    int64_t at[kMaxStages];
    path_of(tid, at);
#pragma unroll
    for (int i = 0; i < kMaxStages; ++i) {
      if (i < kEarly) {
        lp_e[i] = i < n - 1 ? j.logp[at[i]] : 0.f;
        tk_e[i] = i < n - 1 ? j.tok[at[i]] : 0;
      }
      if (i == n - 1) last_at = (int)(at[i] - (j.off_last + j.rbase_last * kw));
    }
  }

  if (kw <= KWAVE) {
    // (the first wave has just spent its time on the leaves' paths: it stays out of the merge when the
    // other waves cover the rows in one pass)
    const int w0 = (early && rows_last <= NT / 64 - 1) ? 1 : 0;
    for (int rl = wave - w0; rl >= 0 && rl < rows_last; rl += NT / 64 - w0) {
      const int64_t row = j.rbase_last + rl;
      float v[kMaxTopK];
      int32_t ix[kMaxTopK];
      float lse;
      if (KWAVE >= kMaxTopK) {
        wave_merge_partials(j.part, row, j.nparts, kw, v, ix, lse);
      } else {
        switch (kw) {
          case 1: wave_merge_partials_k<1>(j.part, row, j.nparts, kw, v, ix, lse); break;
          case 2: wave_merge_partials_k<2>(j.part, row, j.nparts, kw, v, ix, lse); break;
          case 3: wave_merge_partials_k<3>(j.part, row, j.nparts, kw, v, ix, lse); break;
          default: wave_merge_partials_k<4>(j.part, row, j.nparts, kw, v, ix, lse); break;
        }
      }
#pragma unroll
      for (int t = 0; t < kMaxTopK; ++t)
        if (lane == t && t < kw) {
          j.tok[j.off_last + row * kw + t] = ix[t];
          j.logp[j.off_last + row * kw + t] = v[t] - lse;
          if (early) {
            c_tok[rl * kw + t] = ix[t];
            c_logp[rl * kw + t] = v[t] - lse;
          }
        }
      if (lane == 0) j.lse[j.row_off_last + row] = lse;
    }
  } else {
    const int grp = tid >> 8, gl = tid & 255;
    for (int r0 = 0; r0 < rows_last; r0 += NT / 256) {
      const int rl = r0 + grp;
      const bool live = rl < rows_last;
      const int64_t row = j.rbase_last + (live ? rl : rows_last - 1);
      float v[kMaxTopK];
      int32_t ix[kMaxTopK];
      float lse;
      group_merge_partials(j.part, row, j.nparts, kw, v, ix, lse, merge_lds + grp * kMergeLds);
#pragma unroll
      for (int t = 0; t < kMaxTopK; ++t)
        if (live && gl == t && t < kw) {
          j.tok[j.off_last + row * kw + t] = ix[t];
          j.logp[j.off_last + row * kw + t] = v[t] - lse;
          if (early) {
            c_tok[rl * kw + t] = ix[t];
            c_logp[rl * kw + t] = v[t] - lse;
          }
        }
      if (live && gl == 0) j.lse[j.row_off_last + row] = lse;
    }
  }
  __threadfence_block();
  __syncthreads();

  int32_t tk[kMaxStages];
  if (early) {
    if (tid < nleaf) {
      float score = 0.f;   // added in stage order
#pragma unroll
      for (int i = 0; i < kMaxStages; ++i) {
        tk[i] = 0;
        if (i < kEarly && i < n - 1) {
          score += lp_e[i];
          tk[i] = tk_e[i];
        }
        if (i == n - 1) {
          score += c_logp[last_at];
          tk[i] = c_tok[last_at];
        }
      }
      sk[tid] = best_key(score, tid);
    }
  } else {
    for (int leaf = tid; leaf < nleaf; leaf += NT) {
      int64_t at[kMaxStages];
      path_of(leaf, at);
      float lp[kMaxStages];
#pragma unroll
      for (int i = 0; i < kMaxStages; ++i) {
        lp[i] = i < n ? j.logp[at[i]] : 0.f;
        tk[i] = (one_pass && i < n) ? j.tok[at[i]] : 0;
      }
      float score = 0.f;
#pragma unroll
      for (int i = 0; i < kMaxStages; ++i)
        if (i < n) score += lp[i];
      sk[leaf] = best_key(score, leaf);
    }
  }
  // (the ranking reads two keys at a time: fill the last pair)
  if (tid == 0 && (nleaf & 1) && nleaf < kMaxLeaves) sk[nleaf] = 0;
  __syncthreads();

  // rank of a leaf = number of leaves before it in (score, then smaller leaf index): one 64-bit compare each
  for (int leaf = tid; leaf < nleaf; leaf += NT) {
    const uint64_t mine = sk[leaf];
    int pos = 0;
#pragma unroll 4
    for (int o = 0; o < nleaf; o += 2) {
      const uint64_t k0 = sk[o], k1 = sk[o + 1];
      pos += k0 > mine ? 1 : 0;
      pos += k1 > mine ? 1 : 0;
    }
    float s;
    int32_t self;
    best_unkey(mine, s, self);
    if (pos < j.B) {
      const int64_t c = (int64_t)q * j.B_pad + pos;
      j.cand_leaf[c] = leaf;
      j.cand_scores[c] = s;
      if (!one_pass) {
        int64_t at[kMaxStages];
        path_of(leaf, at);
#pragma unroll
        for (int i = 0; i < kMaxStages; ++i) tk[i] = i < n ? j.tok[at[i]] : 0;
      }
#pragma unroll
      for (int i = 0; i < kMaxStages; ++i)
        if (i < n) j.cand_tokens[c * n + i] = tk[i];
    }
  }
  // slots past this sequence's candidates: padding
  for (int pos = j.B + tid; pos < j.B_pad; pos += NT) {
    const int64_t c = (int64_t)q * j.B_pad + pos;
    j.cand_leaf[c] = -1;
    j.cand_scores[c] = SPEC_NEG_INF;
    for (int i = 0; i < n; ++i) j.cand_tokens[c * n + i] = -1;
  }
}

// Fills the per-sequence arguments of tree_body for sequence q from a TreeJob: lanes 0 .. n-1 of EVERY wave
// write the LDS arrays (the same values: a wave may then read them back without a workgroup barrier, its own
// LDS accesses execute in order), every thread computes the scalars.  Call with all threads.
__device__ __forceinline__ void tree_args_for_sequence(const TreeJob& j, int q, TreeArgs& a, int* s_k, int64_t* s_off,
                                                       int64_t* s_rbase, int* s_kw) {
  const int tid = opaque_tid();
  const int n = j.n;
  a.n = n; a.B_pad = j.B_pad; a.nparts = j.nparts;
  a.part = j.part; a.tok = j.tok; a.logp = j.logp; a.lse = j.lse;
  a.cand_tokens = j.cand_tokens; a.cand_scores = j.cand_scores; a.cand_leaf = j.cand_leaf;
  a.B = j.B; a.L = j.L; a.k_last = 1; a.kw_last = 1; a.off_last = 0; a.row_off_last = 0; a.rbase_last = 0;
  const int32_t* d = j.seq_desc ? j.seq_desc + (int64_t)q * (2 * n + 1) : nullptr;
  if (d) {
    a.B = d[2 * n];
    a.L = 1;
  }
  int64_t cnt = 1;   // rows of one sequence at stage i (uniform tree)
#pragma unroll
  for (int i = 0; i < kMaxStages; ++i) {
    if (i < n) {
      const int k = d ? d[i] : j.top_k[i];
      const int64_t rbase = d ? (int64_t)d[n + i] : (int64_t)q * cnt;
      if (d) a.L *= k;
      if ((tid & 63) == i) { s_k[i] = k; s_off[i] = j.off[i]; s_rbase[i] = rbase; s_kw[i] = j.kstride[i]; }
      if (i == n - 1) {
        a.k_last = k; a.kw_last = j.kstride[i]; a.off_last = j.off[i]; a.row_off_last = j.row_off[i];
        a.rbase_last = rbase;
      }
      cnt *= k;
    }
  }
}

}  // namespace specdraft
