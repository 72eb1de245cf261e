// Streaming MFMA attention kernel for gfx950 (bf16, head_dim 128): the production path of
// hpd_decode_attention / hpd_decode_step.
//
// Work unit = (document with live branches, kv head, row group).  All G * n_live query rows
// of the document share the header and document keys (Section 4.3.5: the instruction and the
// attribute definitions are shared among the stacked documents; related work, "Parallel LLM
// Inference": memory and computation of the shared context are shared), so the workgroup
// pulls header ++ document K/V from HBM exactly once, through LDS, and every query row
// consumes it from there.
//
//  * Loading.  Key blocks of 32 keys travel HBM -> LDS with direct-to-LDS 16-byte loads
//    (global_load_lds_dwordx4): no VGPRs are held by data in flight.  A lane fetches exactly
//    the 16 bytes that the same lane will later feed to an MFMA, so LDS is a pure delay line:
//    fragment f of a block sits at lds[f][lane], reads are lane-linear and conflict-free.
//    Two 64 KB stages of four blocks are used alternately: while stage A is consumed, the
//    64 KB of stage B are in flight.  The two stages are distinct __shared__ arrays on
//    purpose: the compiler then knows that reading one does not alias the DMA into the
//    other and does not drain the DMA queue before every LDS read.
//  * Contraction (transposed, see hpd_attn_mfma.hip for the derivation):
//        S^T[key,row] = K.Q^T   (A = K fragment from LDS, B = rotated Q in registers, bf16
//                                hi + lo parts: two MFMA passes, Q rounding drops out)
//        O^T[d,row]  += V^T.P^T (A = V fragment from the 8-key interleaved pool, B = P)
//    One query row lives in lanes n and n+32; softmax statistics never leave them.
//  * Softmax.  Online max/sum in registers.  The running maximum is exact (the accumulators
//    are rescaled whenever some row of the wave sees a larger score; the rescale is skipped,
//    wave-uniformly, when no row does).  Exactness matters for accuracy: the dominant key of a
//    row then has probability exactly 1.0, which bf16 represents without error; with a stale
//    maximum the largest weight would carry a 2^-9 rounding error into P.V (measured: 3x
//    larger max-abs error).
//  * Waves.  8 waves = (row block of 32 rows) x (key group).  KG = 8 / row blocks rounded
//    down to a power of two; the key groups split each stage's four blocks and are merged
//    through LDS at the end (identical lane layout on both sides).
//  * Tails (Section 4.3.3: every value still grows token by token) are private to a branch:
//    G rows per key, no reuse, so no MFMA.  Each wave takes branches round-robin and does
//    wavefront-reduction dot products: 16 lanes cover one 256-byte key row (DPP row
//    reductions), 4 keys per load instruction, coalesced; the next branch's loads are issued
//    before the current branch is computed.  In fused mode (hpd_decode_step) the newest key
//    is rotated, rounded, stored to the tail pool and used in the same pass.
//  * Order.  With at most 128 rows the tails are done FIRST, while the first stage's DMA is
//    in flight: their (max, sum, O) are parked row-major (XOR-swizzled) in the idle second
//    stage and become the initial online-softmax state of the MFMA waves; at the end the
//    finished rows are parked again and written with full-line stores.  With more rows the
//    second stage is too small: the prefix partials are parked at the end and the tail pass
//    merges into them.
#include <cmath>

#include "hpd_internal.h"
#include "hpd_device.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int D = 128;
constexpr int WAVES = 8;
constexpr int SLOT_U4 = 16 * 64;       // one 32-key block: 8 K + 8 V fragments of 64 x 16 bytes
constexpr int STAGE_BLOCKS = 4;
constexpr int STAGE_U4 = STAGE_BLOCKS * SLOT_U4;  // 64 KB
constexpr int MERGE_FLOATS = 66 * 64;  // 64 accumulators + max + sum per lane
constexpr int MAX_ROWS = 256;          // rows per workgroup (8 row blocks)
constexpr float NEG_BIG = -1.0e30f;

struct StreamArgs {
  hpd_dev_tables tb;
  int32_t step, Hq, Hkv, Tcap, P, n_docs, RG, out_f32, fused, live_base;
  int64_t NP;
  float scale_log2;
};

#define HPD_GLL(gptr, lptr)                                                                   \
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(gptr),   \
                                   (__attribute__((address_space(3))) void*)(lptr), 16, 0, 0)

__device__ __forceinline__ uint32_t cvt_pk_bf16(float lo, float hi) {
  floatx2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
__device__ __forceinline__ bf16x8 pack8(const float* v) {
  uint4 u;
  u.x = cvt_pk_bf16(v[0], v[1]); u.y = cvt_pk_bf16(v[2], v[3]);
  u.z = cvt_pk_bf16(v[4], v[5]); u.w = cvt_pk_bf16(v[6], v[7]);
  return __builtin_bit_cast(bf16x8, u);
}
__device__ __forceinline__ void unpack8(uint4 a, float out[8]) {
  out[0] = __uint_as_float(a.x << 16); out[1] = __uint_as_float(a.x & 0xffff0000u);
  out[2] = __uint_as_float(a.y << 16); out[3] = __uint_as_float(a.y & 0xffff0000u);
  out[4] = __uint_as_float(a.z << 16); out[5] = __uint_as_float(a.z & 0xffff0000u);
  out[6] = __uint_as_float(a.w << 16); out[7] = __uint_as_float(a.w & 0xffff0000u);
}
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// sum over the 16 lanes of a DPP row; every lane of the row gets the total
__device__ __forceinline__ float row16_sum(float v) {
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true));   // quad_perm [2,3,0,1]
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xF, 0xF, true));  // row_half_mirror
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x140, 0xF, 0xF, true));  // row_mirror
  return v;
}

// XOR-swizzled row-major park buffer: element (row, 4-float chunk c4) of a 128-float row.
__device__ __forceinline__ int park_off(int row, int c4) { return row * 128 + ((c4 ^ (row & 31)) << 2); }

template <int G>
__global__ void __launch_bounds__(WAVES * 64)
attn_stream_kernel(StreamArgs a, const uint16_t* __restrict__ q, const uint16_t* __restrict__ k_prefix,
                   const uint16_t* __restrict__ v_prefix, uint16_t* __restrict__ k_tail,
                   uint16_t* __restrict__ v_tail, const uint16_t* __restrict__ k_new,
                   const uint16_t* __restrict__ v_new, void* __restrict__ out) {
  __shared__ uint4 ringA[STAGE_U4];
  __shared__ uint4 ringB[STAGE_U4];
  __shared__ float ml_buf[MAX_ROWS * 2];

  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int n = lane & 31, g2 = lane >> 5;

  // ---- unit descriptor (one dependent load): {hoff, Hlen, doff, Llen, row0_live, nb, pos, doc}
  const int32_t rg = blockIdx.x % a.RG;
  const int32_t hk = (blockIdx.x / a.RG) % a.Hkv;
  const int32_t u = blockIdx.x / (a.RG * a.Hkv);
  const int32_t* desc = a.tb.unit_desc + (int64_t)u * 8;  // pre-offset to this step by the host
  const int32_t hoff = desc[0], Hlen = desc[1], doff = desc[2], Llen = desc[3];
  const int32_t row0_live = desc[4], nb = desc[5], upos = desc[6];

  const int32_t R = nb * G;
  const int32_t nblk = (R + 31) >> 5;
  const int32_t per_group = (nblk + a.RG - 1) / a.RG;  // <= 8 by the host's choice of RG
  const int32_t first_blk = rg * per_group;
  const int32_t nblk_here = min(per_group, nblk - first_blk);
  if (nblk_here <= 0) return;  // uniform over the workgroup
  const int32_t KG = nblk_here <= 2 ? 4 : (nblk_here <= 4 ? 2 : 1);
  const int32_t kg = wave % KG;
  const int32_t rb = wave / KG;
  const bool active = rb < nblk_here;

  const int32_t NBh = (Hlen + 31) >> 5, NBd = (Llen + 31) >> 5;
  const int32_t NB = NBh + NBd;
  const int32_t NR = (NB + STAGE_BLOCKS - 1) / STAGE_BLOCKS;

  // ---- loader role: wave w fills block slot w/2 of a stage, K fragments (even w) or V (odd w)
  const int32_t ld_slot = wave >> 1;
  const bool ld_v = wave & 1;
  const int32_t krow = ((n >> 4) << 4) | (((n >> 2) & 1) << 3) | (((n >> 3) & 1) << 2) | (n & 3);
  const uint16_t* kbase = k_prefix + (int64_t)hk * a.NP * D;
  const uint16_t* vbase = v_prefix + (int64_t)hk * (a.NP / 8) * D * 8;

  auto issue_round = [&](int32_t r, uint4* stage) {
    const int32_t gb = r * STAGE_BLOCKS + ld_slot;
    if (gb >= NB) return;  // uniform per wave
    const int32_t slot0 = gb < NBh ? hoff + gb * 32 : doff + (gb - NBh) * 32;
    uint4* dst = stage + ld_slot * SLOT_U4 + (ld_v ? 8 * 64 : 0);
    if (!ld_v) {
      const uint16_t* src = kbase + (int64_t)(slot0 + krow) * D + g2 * 8;
#pragma unroll
      for (int f = 0; f < 8; ++f) HPD_GLL(src + f * 16, dst + f * 64);
    } else {
      const uint16_t* src = vbase + ((int64_t)(slot0 / 8 + g2) * D + n) * 8;
#pragma unroll
      for (int f = 0; f < 8; ++f)  // f = d-block * 2 + key half
        HPD_GLL(src + ((int64_t)(f & 1) * 2 * D + (f >> 1) * 32) * 8, dst + f * 64);
    }
  };

  issue_round(0, ringA);

  const int32_t rows_here = min(R - first_blk * 32, nblk_here * 32);
  const bool tails_first = nblk_here <= 4;  // the idle second stage can park 128 rows
  float* const parkA = reinterpret_cast<float*>(ringA);
  float* const parkB = reinterpret_cast<float*>(ringB);

  // =====================================================================================
  // Tail pass.  lane = (ks, c): the 16 lanes c of a DPP row cover one key row (8 channels
  // each), ks = key within a group of 4.
  //   merge_prefix = false: park (max, sum, O) of every row in `park`/ml_buf
  //   merge_prefix = true : combine with the prefix partials parked there and store `out`
  // =====================================================================================
  const int32_t ks = lane >> 4, c = lane & 15;
  const int32_t br0 = first_blk * 32 / G;
  const int32_t nbr_here = min(nb - br0, nblk_here * 32 / G);
  const int32_t nkeys_pool = a.step;  // older keys; the newest one is handled separately

  // A branch with G = 8 is handled as two half-branches of GH = 4 rows (same keys).
  constexpr int GH = G < 4 ? G : 4;
  constexpr int NH = G / GH;
  struct TailLoads {  // what is prefetched one (half-)branch ahead
    uint4 kraw[4], vraw[4], qa[GH], qb[GH];
    int64_t tbase;
    int32_t live_row;
  };
  auto tail_issue = [&](int32_t vb, TailLoads& t) {
    const int32_t bl = vb / NH, g0 = (vb % NH) * GH;
    t.live_row = row0_live + br0 + bl;
    const int32_t b = a.tb.live_branch[a.live_base + t.live_row];
    t.tbase = (((int64_t)b * a.Hkv + hk) * a.Tcap) * D;
#pragma unroll
    for (int g = 0; g < GH; ++g) {
      const uint16_t* qp = q + ((int64_t)t.live_row * a.Hq + hk * G + g0 + g) * D;
      t.qa[g] = *reinterpret_cast<const uint4*>(qp + c * 8);
      t.qb[g] = *reinterpret_cast<const uint4*>(qp + (c ^ 8) * 8);
    }
#pragma unroll
    for (int uu = 0; uu < 4; ++uu) {
      const int32_t tt = uu * 4 + ks;
      t.kraw[uu] = make_uint4(0, 0, 0, 0);
      t.vraw[uu] = make_uint4(0, 0, 0, 0);
      if (tt < nkeys_pool) {
        t.kraw[uu] = *reinterpret_cast<const uint4*>(k_tail + t.tbase + (int64_t)tt * D + c * 8);
        t.vraw[uu] = *reinterpret_cast<const uint4*>(v_tail + t.tbase + (int64_t)tt * D + c * 8);
      }
    }
  };

  auto tail_compute = [&](int32_t vb, TailLoads& t, bool merge_prefix, float* park_lo, float* park_hi) {
    const int32_t bl = vb / NH, g0 = (vb % NH) * GH;
    // the newest token's inputs are requested now and used at the very end
    uint4 kna = make_uint4(0, 0, 0, 0), knb = kna, vn = kna;
    if (a.fused) {
      const uint16_t* kp = k_new + ((int64_t)t.live_row * a.Hkv + hk) * D;
      kna = *reinterpret_cast<const uint4*>(kp + c * 8);
      knb = *reinterpret_cast<const uint4*>(kp + (c ^ 8) * 8);
      vn = *reinterpret_cast<const uint4*>(v_new + ((int64_t)t.live_row * a.Hkv + hk) * D + c * 8);
    } else {  // already appended by hpd_kv_append: rotated and rounded
      kna = *reinterpret_cast<const uint4*>(k_tail + t.tbase + (int64_t)a.step * D + c * 8);
      vn = *reinterpret_cast<const uint4*>(v_tail + t.tbase + (int64_t)a.step * D + c * 8);
    }
    int32_t pos = upos;
    if (upos < 0) {
      const int32_t b = a.tb.live_branch[a.live_base + t.live_row];
      pos = a.tb.branch_base_pos[b] + 1 + a.step;
    }
    const float4* csp = reinterpret_cast<const float4*>(a.tb.rope + (int64_t)pos * (D / 2) + (c & 7) * 8);
    // rotated query rows in fp32, pre-multiplied by scale * log2(e)
    float qf[GH][8];
    {
      float cs_c[8], cs_s[8];
#pragma unroll
      for (int e2 = 0; e2 < 4; ++e2) {
        const float4 cs = csp[e2];
        cs_c[2 * e2] = cs.x; cs_s[2 * e2] = cs.y; cs_c[2 * e2 + 1] = cs.z; cs_s[2 * e2 + 1] = cs.w;
      }
#pragma unroll
      for (int g = 0; g < GH; ++g) {
        float x[8], y[8];
        unpack8(t.qa[g], x);
        unpack8(t.qb[g], y);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          float r1, r2;
          if (c < 8) hpd::rope_pair(x[e], y[e], cs_c[e], cs_s[e], r1, r2);  // x = first half
          else { hpd::rope_pair(y[e], x[e], cs_c[e], cs_s[e], r2, r1); }    // x = second half
          qf[g][e] = r1 * a.scale_log2;
        }
      }
    }
    float tm[GH], tl[GH], ta[GH][8];
#pragma unroll
    for (int g = 0; g < GH; ++g) {
      tm[g] = NEG_BIG; tl[g] = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) ta[g][e] = 0.f;
    }
    // ---- keys already in the pool, 16 per batch (the first batch was loaded by tail_issue)
    for (int32_t base = 0; base < nkeys_pool; base += 16) {
      if (base > 0) {
#pragma unroll
        for (int uu = 0; uu < 4; ++uu) {
          const int32_t tt = base + uu * 4 + ks;
          t.kraw[uu] = make_uint4(0, 0, 0, 0);
          t.vraw[uu] = make_uint4(0, 0, 0, 0);
          if (tt < nkeys_pool) {
            t.kraw[uu] = *reinterpret_cast<const uint4*>(k_tail + t.tbase + (int64_t)tt * D + c * 8);
            t.vraw[uu] = *reinterpret_cast<const uint4*>(v_tail + t.tbase + (int64_t)tt * D + c * 8);
          }
        }
      }
      float sc[GH][4];
#pragma unroll
      for (int uu = 0; uu < 4; ++uu) {
        const bool ok = base + uu * 4 + ks < nkeys_pool;
        float kv[8];
        unpack8(t.kraw[uu], kv);
#pragma unroll
        for (int g = 0; g < GH; ++g) {
          float dot = 0.f;
#pragma unroll
          for (int e = 0; e < 8; ++e) dot = fmaf(kv[e], qf[g][e], dot);
          dot = row16_sum(dot);
          sc[g][uu] = ok ? dot : -INFINITY;
        }
      }
#pragma unroll
      for (int g = 0; g < GH; ++g) {
        const float bmax = fmaxf(fmaxf(sc[g][0], sc[g][1]), fmaxf(sc[g][2], sc[g][3]));
        const float m_new = fmaxf(tm[g], bmax);
        const float alpha = fast_exp2(tm[g] - m_new);
        tm[g] = m_new;
        tl[g] *= alpha;
#pragma unroll
        for (int e = 0; e < 8; ++e) ta[g][e] *= alpha;
#pragma unroll
        for (int uu = 0; uu < 4; ++uu) sc[g][uu] = fast_exp2(sc[g][uu] - m_new);
        tl[g] += (sc[g][0] + sc[g][1]) + (sc[g][2] + sc[g][3]);
      }
#pragma unroll
      for (int uu = 0; uu < 4; ++uu) {
        float vv[8];
        unpack8(t.vraw[uu], vv);
#pragma unroll
        for (int g = 0; g < GH; ++g)
#pragma unroll
          for (int e = 0; e < 8; ++e) ta[g][e] = fmaf(sc[g][uu], vv[e], ta[g][e]);
      }
    }
    // ---- merge the 4 key lane-groups (lanes l, l^16, l^32, l^48)
#pragma unroll
    for (int g = 0; g < GH; ++g) {
      float mm = fmaxf(tm[g], __shfl_xor(tm[g], 16));
      mm = fmaxf(mm, __shfl_xor(mm, 32));
      const float f = fast_exp2(tm[g] - mm);
      tm[g] = mm;
      tl[g] *= f;
      tl[g] += __shfl_xor(tl[g], 16);
      tl[g] += __shfl_xor(tl[g], 32);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        float v = ta[g][e] * f;
        v += __shfl_xor(v, 16);
        v += __shfl_xor(v, 32);
        ta[g][e] = v;
      }
    }
    // ---- the newest token, after the older ones in both modes so that the fused and the
    //      two-call sequence add up in the same order.  Fused: rotate, round once, store, use
    //      the stored value.
    {
      float kv[8], vv[8];
      uint4 kst = kna;
      if (a.fused) {
      float x[8], y[8], rr[8];
      unpack8(kna, x);
      unpack8(knb, y);
      // the table row is read again (cache hit) rather than held in registers throughout:
      // the empty asm hides the pointer's origin so the two reads are not merged
      const float4* csp2 = csp;
      asm volatile("" : "+v"(csp2));
#pragma unroll
      for (int e2 = 0; e2 < 4; ++e2) {
        const float4 cs = csp2[e2];
        float r1, r2;
        if (c < 8) hpd::rope_pair(x[2 * e2], y[2 * e2], cs.x, cs.y, r1, r2);
        else { hpd::rope_pair(y[2 * e2], x[2 * e2], cs.x, cs.y, r2, r1); }
        rr[2 * e2] = r1;
        if (c < 8) hpd::rope_pair(x[2 * e2 + 1], y[2 * e2 + 1], cs.z, cs.w, r1, r2);
        else { hpd::rope_pair(y[2 * e2 + 1], x[2 * e2 + 1], cs.z, cs.w, r2, r1); }
        rr[2 * e2 + 1] = r1;
      }
      kst = __builtin_bit_cast(uint4, pack8(rr));
      if (ks == 0 && g0 == 0) {
        *reinterpret_cast<uint4*>(k_tail + t.tbase + (int64_t)a.step * D + c * 8) = kst;
        *reinterpret_cast<uint4*>(v_tail + t.tbase + (int64_t)a.step * D + c * 8) = vn;
      }
      }
      unpack8(kst, kv);
      unpack8(vn, vv);
#pragma unroll
      for (int g = 0; g < GH; ++g) {
        float dot = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) dot = fmaf(kv[e], qf[g][e], dot);
        dot = row16_sum(dot);
        const float m_new = fmaxf(tm[g], dot);
        const float alpha = fast_exp2(tm[g] - m_new);
        const float pr = fast_exp2(dot - m_new);
        tm[g] = m_new;
        tl[g] = tl[g] * alpha + pr;
#pragma unroll
        for (int e = 0; e < 8; ++e) ta[g][e] = fmaf(pr, vv[e], ta[g][e] * alpha);
      }
    }
    // ---- lane group ks finishes row g0 + ks
#pragma unroll
    for (int g = 0; g < GH; ++g) {
      if (g == ks) {
        const int32_t lr = bl * G + g0 + g;
        float* park = lr < 128 ? park_lo : park_hi;
        const int32_t lrr = lr & 127;
        if (!merge_prefix) {
          *reinterpret_cast<float4*>(park + park_off(lrr, 2 * c)) =
              make_float4(ta[g][0], ta[g][1], ta[g][2], ta[g][3]);
          *reinterpret_cast<float4*>(park + park_off(lrr, 2 * c + 1)) =
              make_float4(ta[g][4], ta[g][5], ta[g][6], ta[g][7]);
          if (c == 0) { ml_buf[lr * 2] = tm[g]; ml_buf[lr * 2 + 1] = tl[g]; }
        } else {
          const float mp = ml_buf[lr * 2], lp = ml_buf[lr * 2 + 1];
          const float4 p0 = *reinterpret_cast<const float4*>(park + park_off(lrr, 2 * c));
          const float4 p1 = *reinterpret_cast<const float4*>(park + park_off(lrr, 2 * c + 1));
          const float mx = fmaxf(mp, tm[g]);
          const float ap = fast_exp2(mp - mx), at = fast_exp2(tm[g] - mx);
          const float inv = 1.0f / (lp * ap + tl[g] * at);
          float o[8] = {p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w};
#pragma unroll
          for (int e = 0; e < 8; ++e) o[e] = (o[e] * ap + ta[g][e] * at) * inv;
          const int64_t o_off = ((int64_t)t.live_row * a.Hq + hk * G + g0 + g) * D + c * 8;
          if (a.out_f32) {
            float* op = reinterpret_cast<float*>(out) + o_off;
            *reinterpret_cast<float4*>(op) = make_float4(o[0], o[1], o[2], o[3]);
            *reinterpret_cast<float4*>(op + 4) = make_float4(o[4], o[5], o[6], o[7]);
          } else {
            *reinterpret_cast<uint4*>(reinterpret_cast<uint16_t*>(out) + o_off) =
                __builtin_bit_cast(uint4, pack8(o));
          }
        }
      }
    }
  };

  auto tail_pass = [&](bool merge_prefix, float* park_lo, float* park_hi) {
    const int32_t nvb = nbr_here * NH;
    TailLoads cur, nxt;
    if (wave < nvb) tail_issue(wave, cur);
    for (int32_t vb = wave; vb < nvb; vb += WAVES) {
      const bool more = vb + WAVES < nvb;
      if (more) tail_issue(vb + WAVES, nxt);
      tail_compute(vb, cur, merge_prefix, park_lo, park_hi);
      if (more) cur = nxt;
    }
  };

  if (tails_first) tail_pass(false, parkB, parkB);

  // ---- this lane's query row, rotated, as bf16 hi + lo MFMA B operands
  const int32_t r_row = (first_blk + rb) * 32 + n;
  const bool row_valid = active && r_row < R;
  bf16x8 Qh[8], Ql[8];
  {
    const int32_t bi = min(r_row / G, nb - 1);
    const int32_t gq = r_row % G;
    const int32_t live_row = row0_live + bi;
    int32_t pos = upos;
    if (upos < 0) {
      const int32_t b = a.tb.live_branch[a.live_base + live_row];
      pos = a.tb.branch_base_pos[b] + 1 + a.step;
    }
    const int64_t q_off = ((int64_t)live_row * a.Hq + hk * G + gq) * D;
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
        const float4 cs = csp[e2];
        hpd::rope_pair(lo[2 * e2], hi[2 * e2], cs.x, cs.y, rl[2 * e2], rh[2 * e2]);
        hpd::rope_pair(lo[2 * e2 + 1], hi[2 * e2 + 1], cs.z, cs.w, rl[2 * e2 + 1], rh[2 * e2 + 1]);
      }
      Qh[kk] = pack8(rl);
      Qh[kk + 4] = pack8(rh);
      float hl[8], hh[8];
      unpack8(__builtin_bit_cast(uint4, Qh[kk]), hl);
      unpack8(__builtin_bit_cast(uint4, Qh[kk + 4]), hh);
#pragma unroll
      for (int e = 0; e < 8; ++e) { rl[e] -= hl[e]; rh[e] -= hh[e]; }
      Ql[kk] = pack8(rl);
      Ql[kk + 4] = pack8(rh);
    }
  }

  // ---- online-softmax state: (max, this lane's share of the sum, O^T accumulators)
  float m_used = NEG_BIG;  // running maximum (log2 units), equal in lanes n and n+32
  float l_lane = 0.f;
  floatx16 acc[4];
#pragma unroll
  for (int blk = 0; blk < 4; ++blk)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[blk][i] = 0.f;

  if (tails_first) {
    __syncthreads();  // tail partials are parked in the second stage
    if (active && kg == 0 && r_row < R) {
      const int32_t lr = rb * 32 + n;
      m_used = ml_buf[lr * 2];
      l_lane = g2 == 0 ? ml_buf[lr * 2 + 1] : 0.f;
#pragma unroll
      for (int blk = 0; blk < 4; ++blk)
#pragma unroll
        for (int cc = 0; cc < 4; ++cc) {
          const float4 v = *reinterpret_cast<const float4*>(parkB + park_off(lr, blk * 8 + cc * 2 + g2));
          acc[blk][cc * 4 + 0] = v.x; acc[blk][cc * 4 + 1] = v.y;
          acc[blk][cc * 4 + 2] = v.z; acc[blk][cc * 4 + 3] = v.w;
        }
    }
    // the first round's barrier comes before any DMA into the second stage
  }

  auto compute_block = [&](const uint4* slot, int32_t valid) {
    const uint4* fr = slot + lane;
    floatx16 S;
#pragma unroll
    for (int i = 0; i < 16; ++i) S[i] = 0.f;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      const bf16x8 kf = __builtin_bit_cast(bf16x8, fr[kk * 64]);
      S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, Qh[kk], S, 0, 0, 0);
      S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, Ql[kk], S, 0, 0, 0);
    }
    uint4 vf[8];
#pragma unroll
    for (int f = 0; f < 8; ++f) vf[f] = fr[(8 + f) * 64];

    float s[16];
    float bm = NEG_BIG;
    if (valid < 32) {
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int key = ((i >> 3) << 4) + g2 * 8 + (i & 7);
        s[i] = key < valid ? S[i] * a.scale_log2 : -INFINITY;
        bm = fmaxf(bm, s[i]);
      }
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
    } else {
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        s[i] = S[i] * a.scale_log2;
        bm = fmaxf(bm, s[i]);
      }
    }
    if (__any(bm > m_used)) {
      bm = fmaxf(bm, __shfl_xor(bm, 32));
      const float m_new = fmaxf(m_used, bm);
      const float alpha = fast_exp2(m_used - m_new);
      m_used = m_new;
      l_lane *= alpha;
#pragma unroll
      for (int blk = 0; blk < 4; ++blk)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[blk][i] *= alpha;
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      s[i] = fast_exp2(s[i] - m_used);
      l_lane += s[i];
    }
    const bf16x8 P0 = pack8(s), P1 = pack8(s + 8);
#pragma unroll
    for (int blk = 0; blk < 4; ++blk) {
      acc[blk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vf[blk * 2]), P0,
                                                         acc[blk], 0, 0, 0);
      acc[blk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vf[blk * 2 + 1]), P1,
                                                         acc[blk], 0, 0, 0);
    }
  };

  auto round_body = [&](int32_t r, const uint4* cur, uint4* nxt) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (r + 1 < NR) issue_round(r + 1, nxt);
    if (active) {
      for (int32_t j = kg; j < STAGE_BLOCKS; j += KG) {
        const int32_t gb = r * STAGE_BLOCKS + j;
        if (gb < NB) {
          const int32_t valid = gb < NBh ? min(32, Hlen - gb * 32) : min(32, Llen - (gb - NBh) * 32);
          compute_block(cur + j * SLOT_U4, valid);
        }
      }
    }
  };

  for (int32_t r = 0; r < NR; r += 2) {
    round_body(r, ringA, ringB);
    if (r + 1 < NR) round_body(r + 1, ringB, ringA);
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();  // both stages are dead from here on and get reused

  // ---- merge the key groups: regions 0,1 in ringA, 2,3 in ringB
  for (int32_t s = 1; s < KG; s <<= 1) {
    const bool writer = active && (kg % (2 * s)) == s;
    const bool reader = active && (kg % (2 * s)) == 0 && kg + s < KG;
    const int32_t region = rb + nblk_here * (kg / (2 * s));  // < 4
    float* buf = (region < 2 ? parkA + region * MERGE_FLOATS : parkB + (region - 2) * MERGE_FLOATS) + lane;
    if (writer) {
#pragma unroll
      for (int blk = 0; blk < 4; ++blk)
#pragma unroll
        for (int i = 0; i < 16; ++i) buf[(blk * 16 + i) * 64] = acc[blk][i];
      buf[64 * 64] = m_used;
      buf[65 * 64] = l_lane;
    }
    __syncthreads();
    if (reader) {
      const float m2 = buf[64 * 64], l2 = buf[65 * 64];
      const float m_new = fmaxf(m_used, m2);
      const float a1 = fast_exp2(m_used - m_new), a2 = fast_exp2(m2 - m_new);
      l_lane = l_lane * a1 + l2 * a2;
      m_used = m_new;
#pragma unroll
      for (int blk = 0; blk < 4; ++blk)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[blk][i] = acc[blk][i] * a1 + buf[(blk * 16 + i) * 64] * a2;
    }
    __syncthreads();
  }

  // ---- park the MFMA waves' state row-major (rows 0..127 in ringA, 128..255 in ringB)
  if (active && kg == 0) {
    const int32_t lr = rb * 32 + n;
    float* park = lr < 128 ? parkA : parkB;
    const int32_t lrr = lr & 127;
#pragma unroll
    for (int blk = 0; blk < 4; ++blk)
#pragma unroll
      for (int cc = 0; cc < 4; ++cc)
        *reinterpret_cast<float4*>(park + park_off(lrr, blk * 8 + cc * 2 + g2)) =
            make_float4(acc[blk][cc * 4 + 0], acc[blk][cc * 4 + 1], acc[blk][cc * 4 + 2], acc[blk][cc * 4 + 3]);
    const float l_row = l_lane + __shfl_xor(l_lane, 32);
    if (g2 == 0) { ml_buf[lr * 2] = m_used; ml_buf[lr * 2 + 1] = l_row; }
  }
  __syncthreads();

  if (!tails_first) {
    tail_pass(true, parkA, parkB);
  } else {
    // rows are complete: normalise and store, 4 rows per wave pass, 512 contiguous bytes each
    for (int32_t lr = wave * 4 + ks; lr < rows_here; lr += WAVES * 4) {
      const float inv = 1.0f / ml_buf[lr * 2 + 1];
      const float4 p0 = *reinterpret_cast<const float4*>(parkA + park_off(lr, 2 * c));
      const float4 p1 = *reinterpret_cast<const float4*>(parkA + park_off(lr, 2 * c + 1));
      float o[8] = {p0.x * inv, p0.y * inv, p0.z * inv, p0.w * inv, p1.x * inv, p1.y * inv, p1.z * inv, p1.w * inv};
      const int32_t live_row = row0_live + br0 + lr / G;
      const int64_t o_off = ((int64_t)live_row * a.Hq + hk * G + lr % G) * D + c * 8;
      if (a.out_f32) {
        float* op = reinterpret_cast<float*>(out) + o_off;
        *reinterpret_cast<float4*>(op) = make_float4(o[0], o[1], o[2], o[3]);
        *reinterpret_cast<float4*>(op + 4) = make_float4(o[4], o[5], o[6], o[7]);
      } else {
        *reinterpret_cast<uint4*>(reinterpret_cast<uint16_t*>(out) + o_off) = __builtin_bit_cast(uint4, pack8(o));
      }
    }
  }
}

template <int G>
hipError_t launch_g(const StreamArgs& a, dim3 grid, const void* q, const void* k_prefix,
                    const void* v_prefix, void* k_tail, void* v_tail, const void* k_new,
                    const void* v_new, void* out, hipStream_t s) {
  attn_stream_kernel<G><<<grid, WAVES * 64, 0, s>>>(
      a, (const uint16_t*)q, (const uint16_t*)k_prefix, (const uint16_t*)v_prefix, (uint16_t*)k_tail,
      (uint16_t*)v_tail, (const uint16_t*)k_new, (const uint16_t*)v_new, out);
  return hipGetLastError();
}

}  // namespace

bool hpd_stream_supported(const hpd_layout* L) {
  const int G = L->cfg.n_q_heads / L->cfg.n_kv_heads;
  return L->cfg.dtype == HPD_BF16 && L->cfg.head_dim == D && (G == 1 || G == 2 || G == 4 || G == 8);
}

hipError_t hpd_launch_attention_stream(const hpd_layout* L, int32_t step, const void* q,
                                       const void* k_prefix, const void* v_prefix, void* k_tail,
                                       void* v_tail, const void* k_new, const void* v_new, void* out,
                                       hipStream_t s) {
  StreamArgs a;
  a.tb = L->dev;
  a.step = step; a.Hq = L->cfg.n_q_heads; a.Hkv = L->cfg.n_kv_heads;
  const int G = a.Hq / a.Hkv;
  a.Tcap = L->T; a.P = L->P; a.n_docs = L->n_docs; a.NP = L->NP;
  const int32_t max_nblk = (L->max_rows[step] * G + 31) / 32;
  a.RG = (max_nblk + 7) / 8;
  if (a.RG < 1) a.RG = 1;
  a.out_f32 = L->cfg.out_dtype == HPD_OUT_F32 ? 1 : 0;
  a.fused = (k_new != nullptr) ? 1 : 0;
  a.live_base = L->live_ptr[step];
  a.scale_log2 = (float)(1.4426950408889634 / std::sqrt((double)D));
  a.tb.unit_desc = L->dev.unit_desc + (int64_t)L->unit_ptr[step] * 8;
  const int32_t n_units = L->unit_ptr[step + 1] - L->unit_ptr[step];
  const dim3 grid((unsigned)((int64_t)n_units * a.Hkv * a.RG));
  switch (G) {
    case 1: return launch_g<1>(a, grid, q, k_prefix, v_prefix, k_tail, v_tail, k_new, v_new, out, s);
    case 2: return launch_g<2>(a, grid, q, k_prefix, v_prefix, k_tail, v_tail, k_new, v_new, out, s);
    case 4: return launch_g<4>(a, grid, q, k_prefix, v_prefix, k_tail, v_tail, k_new, v_new, out, s);
    case 8: return launch_g<8>(a, grid, q, k_prefix, v_prefix, k_tail, v_tail, k_new, v_new, out, s);
    default: return hipErrorInvalidValue;
  }
}
