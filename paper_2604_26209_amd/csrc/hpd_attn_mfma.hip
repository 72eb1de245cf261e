// MFMA shared-prefix attention kernel for gfx950 (bf16, head_dim 128).
//
// Work unit = (document with live branches, kv head[, row group]).  All G * n_live query
// rows of the document share the header and document keys (Section 4.3.5: instruction and
// attribute definitions are shared among stacked documents; related-work paragraph on
// parallel inference: memory *and* computation of the shared context are shared), so the
// unit streams header ++ document K/V once and contracts it against every row with MFMA:
//
//   S^T[key, row]  = K[key, :] . Q[row, :]        v_mfma_f32_32x32x16_bf16, A = K, B = Q
//   O^T[d,  row]  += V^T[d, key] . P^T[key, row]  A = V (8-key interleaved pool), B = P
//
// Computing the transposed products keeps one query row per lane column: the softmax
// statistics of a row live in lanes n and n+32 only, and the fp32 scores of the first
// product are, after exponentiation and bf16 packing, exactly the B operand of the second
// one - no cross-lane movement.  The key order inside a 32-key block is permuted on the K
// side (free: it is only an address) so that the 8 probabilities a lane holds for one MFMA
// belong to 8 consecutive keys, which is what the interleaved V pool delivers in 16 bytes.
//
// A workgroup has W waves arranged as (row block of 32 rows) x (key group); key groups
// take the 32-key blocks round-robin and their partial (max, sum, O^T) are merged through
// LDS at the end (same lane layout on both sides, so the merge is lane-private).
// Per-branch tails (Section 4.3.3: each value still grows autoregressively) are not
// shared, have G rows per key and are handled with lane-private dot products plus one
// cross-lane add, merged into the same running statistics.
#include <cmath>

#include "hpd_internal.h"
#include "hpd_device.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int D = 128;
constexpr int MAX_WAVES = 8;
constexpr int MERGE_REGIONS = 4;
constexpr int MERGE_FLOATS = 66 * 64;  // 64 accumulators + max + sum per lane
constexpr float NEG_BIG = -1.0e30f;

struct MfmaArgs {
  hpd_dev_tables tb;
  int32_t step, Hq, Hkv, G, Tcap, P, n_docs, W, RG, psplit, out_f32;
  int64_t NP;
  float scale_log2;
};

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return hpd::float_to_bf16_bits(lo) | (hpd::float_to_bf16_bits(hi) << 16);
}

__device__ __forceinline__ bf16x8 pack8(const float* v) {
  uint4 u;
  u.x = pack_bf16x2(v[0], v[1]); u.y = pack_bf16x2(v[2], v[3]);
  u.z = pack_bf16x2(v[4], v[5]); u.w = pack_bf16x2(v[6], v[7]);
  return __builtin_bit_cast(bf16x8, u);
}

__device__ __forceinline__ void unpack8(uint4 a, float out[8]) {
  out[0] = hpd::bf16_bits_to_float(a.x & 0xffffu); out[1] = hpd::bf16_bits_to_float(a.x >> 16);
  out[2] = hpd::bf16_bits_to_float(a.y & 0xffffu); out[3] = hpd::bf16_bits_to_float(a.y >> 16);
  out[4] = hpd::bf16_bits_to_float(a.z & 0xffffu); out[5] = hpd::bf16_bits_to_float(a.z >> 16);
  out[6] = hpd::bf16_bits_to_float(a.w & 0xffffu); out[7] = hpd::bf16_bits_to_float(a.w >> 16);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Online-softmax state of one query row, spread over lanes n and n+32.
struct RowState {
  float m, l;
  floatx16 acc[4];  // O^T[d = blk*32 + (i/4)*8 + g2*4 + i%4][row n]
};

__device__ __forceinline__ void rescale(RowState& st, float alpha) {
  st.l *= alpha;
#pragma unroll
  for (int blk = 0; blk < 4; ++blk)
#pragma unroll
    for (int i = 0; i < 16; ++i) st.acc[blk][i] *= alpha;
}

// QSPLIT: the rotated query enters the score product as bf16 hi + lo parts (two MFMA passes),
// which removes its rounding from the error budget.  a.psplit does the same for the
// probabilities in the P.V product: 2 = always, 1 = only for a 16-key half-block in which
// some row holds a weight of at least 2^-6 of its running sum, 0 = never.
template <bool QSPLIT>
__global__ void __launch_bounds__(MAX_WAVES * 64)
attn_mfma_kernel(MfmaArgs a, const uint16_t* __restrict__ q, const uint16_t* __restrict__ k_prefix,
                 const uint16_t* __restrict__ v_prefix, const uint16_t* __restrict__ k_tail,
                 const uint16_t* __restrict__ v_tail, void* __restrict__ out) {
  extern __shared__ float merge_buf[];

  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int n = lane & 31, g2 = lane >> 5;

  // ---- which unit
  const int32_t rg = blockIdx.x % a.RG;
  const int32_t hk = (blockIdx.x / a.RG) % a.Hkv;
  const int32_t u = blockIdx.x / (a.RG * a.Hkv);
  const int32_t d = a.tb.unit_doc[a.tb.unit_ptr[a.step] + u];
  const int32_t p = a.tb.doc_prompt[d];
  const int32_t* dlp = a.tb.doc_live_ptr + (int64_t)a.step * (a.n_docs + 1);
  const int32_t row0_live = dlp[d];
  const int32_t nb = dlp[d + 1] - row0_live;
  const int32_t R = nb * a.G;
  const int32_t nblk = (R + 31) >> 5;
  const int32_t per_group = (nblk + a.RG - 1) / a.RG;
  const int32_t first_blk = rg * per_group;
  const int32_t nblk_here = min(per_group, nblk - first_blk);
  if (nblk_here <= 0) return;  // uniform over the workgroup
  const int32_t KGu = a.W / nblk_here;  // >= 1: the host picks RG so that per_group <= W
  const int32_t rb = wave % nblk_here;
  const int32_t kg = wave / nblk_here;
  const bool active = kg < KGu;

  RowState st;
  st.m = NEG_BIG;
  st.l = 0.f;
#pragma unroll
  for (int blk = 0; blk < 4; ++blk)
#pragma unroll
    for (int i = 0; i < 16; ++i) st.acc[blk][i] = 0.f;

  // ---- this lane's query row
  const int32_t r = (first_blk + rb) * 32 + n;
  const bool row_valid = r < R;
  const int32_t bi = min(r / a.G, nb - 1);
  const int32_t gq = r % a.G;
  const int32_t live_row = row0_live + bi;
  const int32_t b = a.tb.live_branch[a.tb.live_ptr[a.step] + live_row];
  const int64_t q_off = ((int64_t)live_row * a.Hq + hk * a.G + gq) * D;

  if (active) {
    // ---- Q: load, rotate at the branch's position, round once to bf16.  B-operand layout:
    //      Qf[kk] holds channels kk*16 + g2*8 + 0..7 of row n; the rotation partner of
    //      channel c is c + 64, i.e. Qf[kk + 4] of the same lane.
    bf16x8 Qf[8];
    bf16x8 Ql[QSPLIT ? 8 : 1];
    {
      const int32_t pos = a.tb.branch_base_pos[b] + 1 + a.step;
      const float2* cs_row = a.tb.rope + (int64_t)pos * (D / 2);
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const int c0 = kk * 16 + g2 * 8;
        float lo[8], hi[8], rl[8], rh[8];
        if (row_valid) {
          unpack8(*reinterpret_cast<const uint4*>(q + q_off + c0), lo);
          unpack8(*reinterpret_cast<const uint4*>(q + q_off + c0 + 64), hi);
        } else {
#pragma unroll
          for (int e = 0; e < 8; ++e) lo[e] = hi[e] = 0.f;
        }
        const float4* csp = reinterpret_cast<const float4*>(cs_row + c0);
#pragma unroll
        for (int e2 = 0; e2 < 4; ++e2) {
          const float4 cs = csp[e2];  // (cos, sin) of channels c0 + 2*e2, c0 + 2*e2 + 1
          rl[2 * e2] = lo[2 * e2] * cs.x - hi[2 * e2] * cs.y;
          rh[2 * e2] = hi[2 * e2] * cs.x + lo[2 * e2] * cs.y;
          rl[2 * e2 + 1] = lo[2 * e2 + 1] * cs.z - hi[2 * e2 + 1] * cs.w;
          rh[2 * e2 + 1] = hi[2 * e2 + 1] * cs.z + lo[2 * e2 + 1] * cs.w;
        }
        Qf[kk] = pack8(rl);
        Qf[kk + 4] = pack8(rh);
        if (QSPLIT) {
          float hl[8], hh[8];
          unpack8(__builtin_bit_cast(uint4, Qf[kk]), hl);
          unpack8(__builtin_bit_cast(uint4, Qf[kk + 4]), hh);
#pragma unroll
          for (int e = 0; e < 8; ++e) { rl[e] -= hl[e]; rh[e] -= hh[e]; }
          Ql[kk] = pack8(rl);
          Ql[kk + 4] = pack8(rh);
        }
      }
    }

    // ---- shared prefix: header ++ document, 32 keys per block, blocks round-robin over
    //      the key groups
    const int32_t Hlen = a.tb.seg_len[p], Llen = a.tb.seg_len[a.P + d];
    const int32_t hoff = a.tb.seg_off[p], doff = a.tb.seg_off[a.P + d];
    const int32_t NBh = (Hlen + 31) >> 5, NBd = (Llen + 31) >> 5;
    // MFMA row m of the score tile carries this key of the block (see file header)
    const int32_t krow = ((n >> 4) << 4) | (((n >> 2) & 1) << 3) | (((n >> 3) & 1) << 2) | (n & 3);
    const uint16_t* kbase = k_prefix + (int64_t)hk * a.NP * D + g2 * 8;
    const uint16_t* vbase = v_prefix + (int64_t)hk * (a.NP / 8) * D * 8;

    for (int32_t kb = kg; kb < NBh + NBd; kb += KGu) {
      int32_t slot0, valid;
      if (kb < NBh) { slot0 = hoff + kb * 32; valid = min(32, Hlen - kb * 32); }
      else { slot0 = doff + (kb - NBh) * 32; valid = min(32, Llen - (kb - NBh) * 32); }

      const uint16_t* kp = kbase + (int64_t)(slot0 + krow) * D;
      floatx16 S;
#pragma unroll
      for (int i = 0; i < 16; ++i) S[i] = 0.f;
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) {
        const bf16x8 kf = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(kp + kk * 16));
        S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, Qf[kk], S, 0, 0, 0);
        if (QSPLIT) S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, Ql[kk], S, 0, 0, 0);
      }
      // V operands can be requested before the softmax arithmetic
      uint4 vf[8];
#pragma unroll
      for (int blk = 0; blk < 4; ++blk)
#pragma unroll
        for (int hf = 0; hf < 2; ++hf)
          vf[blk * 2 + hf] = *reinterpret_cast<const uint4*>(
              vbase + ((int64_t)(slot0 / 8 + hf * 2 + g2) * D + blk * 32 + n) * 8);

      float s[16];
      float bm = -INFINITY;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int key = ((i >> 3) << 4) + g2 * 8 + (i & 7);
        s[i] = key < valid ? S[i] * a.scale_log2 : -INFINITY;
        bm = fmaxf(bm, s[i]);
      }
      bm = fmaxf(bm, __shfl_xor(bm, 32));
      const float m_new = fmaxf(st.m, bm);
      const float alpha = fast_exp2(st.m - m_new);
      float ps = 0.f;
#pragma unroll
      for (int i = 0; i < 16; ++i) { s[i] = fast_exp2(s[i] - m_new); ps += s[i]; }
      ps += __shfl_xor(ps, 32);
      rescale(st, alpha);
      st.l += ps;
      st.m = m_new;
      const bf16x8 P0 = pack8(s), P1 = pack8(s + 8);
      bool lo0 = false, lo1 = false;
      bf16x8 L0 = P0, L1 = P1;
      if (a.psplit) {
        float h0[8], h1[8], r0[8], r1[8];
        unpack8(__builtin_bit_cast(uint4, P0), h0);
        unpack8(__builtin_bit_cast(uint4, P1), h1);
        float big0 = 0.f, big1 = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          big0 = fmaxf(big0, s[e]); big1 = fmaxf(big1, s[8 + e]);
          r0[e] = s[e] - h0[e]; r1[e] = s[8 + e] - h1[e];
        }
        L0 = pack8(r0); L1 = pack8(r1);
        const float thr = st.l * 0.015625f;
        lo0 = a.psplit == 2 || __any(big0 >= thr);
        lo1 = a.psplit == 2 || __any(big1 >= thr);
      }

      if (valid < 32) {
        // padding slots may hold NaN patterns: 0 * NaN must not reach the accumulators
#pragma unroll
        for (int f = 0; f < 8; ++f) {
          const int key0 = (f & 1) * 16 + g2 * 8;
          uint32_t w[4] = {vf[f].x, vf[f].y, vf[f].z, vf[f].w};
#pragma unroll
          for (int e = 0; e < 8; ++e)
            if (key0 + e >= valid) w[e >> 1] &= (e & 1) ? 0x0000ffffu : 0xffff0000u;
          vf[f] = make_uint4(w[0], w[1], w[2], w[3]);
        }
      }
#pragma unroll
      for (int blk = 0; blk < 4; ++blk) {
        st.acc[blk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
            __builtin_bit_cast(bf16x8, vf[blk * 2]), P0, st.acc[blk], 0, 0, 0);
        st.acc[blk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
            __builtin_bit_cast(bf16x8, vf[blk * 2 + 1]), P1, st.acc[blk], 0, 0, 0);
      }
      if (lo0) {
#pragma unroll
        for (int blk = 0; blk < 4; ++blk)
          st.acc[blk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
              __builtin_bit_cast(bf16x8, vf[blk * 2]), L0, st.acc[blk], 0, 0, 0);
      }
      if (lo1) {
#pragma unroll
        for (int blk = 0; blk < 4; ++blk)
          st.acc[blk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
              __builtin_bit_cast(bf16x8, vf[blk * 2 + 1]), L1, st.acc[blk], 0, 0, 0);
      }
    }

    // ---- per-branch tail: keys 0..step of the lane's own branch, split over key groups.
    //      The lane holds half of its row's channels; the other half is in lane ^ 32.
    {
      const int64_t tbase = (((int64_t)b * a.Hkv + hk) * a.Tcap) * D;
      for (int32_t tt = kg; tt <= a.step; tt += KGu) {
        const uint16_t* kp = k_tail + tbase + (int64_t)tt * D + g2 * 8;
        float dot = 0.f;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
          float kv[8], qv[8];
          unpack8(*reinterpret_cast<const uint4*>(kp + kk * 16), kv);
          unpack8(__builtin_bit_cast(uint4, Qf[kk]), qv);
          if (QSPLIT) {
            float ql[8];
            unpack8(__builtin_bit_cast(uint4, Ql[kk]), ql);
#pragma unroll
            for (int e = 0; e < 8; ++e) qv[e] += ql[e];
          }
#pragma unroll
          for (int e = 0; e < 8; ++e) dot = fmaf(kv[e], qv[e], dot);
        }
        dot += __shfl_xor(dot, 32);
        const float sc = dot * a.scale_log2;
        const float m_new = fmaxf(st.m, sc);
        const float alpha = fast_exp2(st.m - m_new);
        const float pr = fast_exp2(sc - m_new);
        rescale(st, alpha);
        st.l += pr;
        st.m = m_new;
        const uint16_t* vp = v_tail + tbase + (int64_t)tt * D + g2 * 4;
#pragma unroll
        for (int blk = 0; blk < 4; ++blk)
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const uint2 vv = *reinterpret_cast<const uint2*>(vp + blk * 32 + c * 8);
            st.acc[blk][c * 4 + 0] = fmaf(pr, hpd::bf16_bits_to_float(vv.x & 0xffffu), st.acc[blk][c * 4 + 0]);
            st.acc[blk][c * 4 + 1] = fmaf(pr, hpd::bf16_bits_to_float(vv.x >> 16), st.acc[blk][c * 4 + 1]);
            st.acc[blk][c * 4 + 2] = fmaf(pr, hpd::bf16_bits_to_float(vv.y & 0xffffu), st.acc[blk][c * 4 + 2]);
            st.acc[blk][c * 4 + 3] = fmaf(pr, hpd::bf16_bits_to_float(vv.y >> 16), st.acc[blk][c * 4 + 3]);
          }
      }
    }
  }

  // ---- merge the key groups (tree over kg; writer and reader use the same lane layout)
  for (int32_t s = 1; s < KGu; s <<= 1) {
    const bool writer = active && (kg % (2 * s)) == s;
    const bool reader = active && (kg % (2 * s)) == 0 && kg + s < KGu;
    const int32_t pair = kg / (2 * s);
    float* buf = merge_buf + (int64_t)(rb + nblk_here * pair) * MERGE_FLOATS + lane;
    if (writer) {
#pragma unroll
      for (int blk = 0; blk < 4; ++blk)
#pragma unroll
        for (int i = 0; i < 16; ++i) buf[(blk * 16 + i) * 64] = st.acc[blk][i];
      buf[64 * 64] = st.m;
      buf[65 * 64] = st.l;
    }
    __syncthreads();
    if (reader) {
      const float m2 = buf[64 * 64], l2 = buf[65 * 64];
      const float m_new = fmaxf(st.m, m2);
      const float a1 = fast_exp2(st.m - m_new), a2 = fast_exp2(m2 - m_new);
      st.l = st.l * a1 + l2 * a2;
      st.m = m_new;
#pragma unroll
      for (int blk = 0; blk < 4; ++blk)
#pragma unroll
        for (int i = 0; i < 16; ++i)
          st.acc[blk][i] = st.acc[blk][i] * a1 + buf[(blk * 16 + i) * 64] * a2;
    }
    __syncthreads();
  }

  // ---- normalise and store
  if (active && kg == 0 && row_valid) {
    const float inv = 1.0f / st.l;
    if (a.out_f32) {
      float* op = reinterpret_cast<float*>(out) + q_off + g2 * 4;
#pragma unroll
      for (int blk = 0; blk < 4; ++blk)
#pragma unroll
        for (int c = 0; c < 4; ++c)
          *reinterpret_cast<float4*>(op + blk * 32 + c * 8) =
              make_float4(st.acc[blk][c * 4 + 0] * inv, st.acc[blk][c * 4 + 1] * inv,
                          st.acc[blk][c * 4 + 2] * inv, st.acc[blk][c * 4 + 3] * inv);
    } else {
      uint16_t* op = reinterpret_cast<uint16_t*>(out) + q_off + g2 * 4;
#pragma unroll
      for (int blk = 0; blk < 4; ++blk)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          uint2 w;
          w.x = pack_bf16x2(st.acc[blk][c * 4 + 0] * inv, st.acc[blk][c * 4 + 1] * inv);
          w.y = pack_bf16x2(st.acc[blk][c * 4 + 2] * inv, st.acc[blk][c * 4 + 3] * inv);
          *reinterpret_cast<uint2*>(op + blk * 32 + c * 8) = w;
        }
    }
  }
}

}  // namespace

bool hpd_mfma_supported(const hpd_layout* L) {
  return L->cfg.dtype == HPD_BF16 && L->cfg.head_dim == D;
}

hipError_t hpd_launch_attention_mfma(const hpd_layout* L, int32_t step, const void* q,
                                     const void* k_prefix, const void* v_prefix, const void* k_tail,
                                     const void* v_tail, void* out, hipStream_t s) {
  static bool attr_set = false;
  const size_t smem = (size_t)MERGE_REGIONS * MERGE_FLOATS * sizeof(float);
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)attn_mfma_kernel<false>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e == hipSuccess)
      e = hipFuncSetAttribute((const void*)attn_mfma_kernel<true>,
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  MfmaArgs a;
  a.tb = L->dev;
  a.step = step; a.Hq = L->cfg.n_q_heads; a.Hkv = L->cfg.n_kv_heads; a.G = a.Hq / a.Hkv;
  a.Tcap = L->T; a.P = L->P; a.n_docs = L->n_docs; a.NP = L->NP;
  a.W = (L->mfma_waves == 4) ? 4 : MAX_WAVES;
  const int32_t max_nblk = (L->max_rows[step] * a.G + 31) / 32;
  a.RG = (max_nblk + a.W - 1) / a.W;
  if (a.RG < 1) a.RG = 1;
  a.scale_log2 = (float)(1.4426950408889634 / std::sqrt((double)D));
  const int32_t n_units = L->unit_ptr[step + 1] - L->unit_ptr[step];
  const dim3 grid((unsigned)((int64_t)n_units * a.Hkv * a.RG));
  a.psplit = L->psplit;
  a.out_f32 = L->cfg.out_dtype == HPD_OUT_F32 ? 1 : 0;
  if (L->qsplit)
    attn_mfma_kernel<true><<<grid, a.W * 64, smem, s>>>(
        a, (const uint16_t*)q, (const uint16_t*)k_prefix, (const uint16_t*)v_prefix,
        (const uint16_t*)k_tail, (const uint16_t*)v_tail, out);
  else
    attn_mfma_kernel<false><<<grid, a.W * 64, smem, s>>>(
        a, (const uint16_t*)q, (const uint16_t*)k_prefix, (const uint16_t*)v_prefix,
        (const uint16_t*)k_tail, (const uint16_t*)v_tail, out);
  return hipGetLastError();
}
