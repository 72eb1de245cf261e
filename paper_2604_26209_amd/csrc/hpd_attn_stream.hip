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
//    Four 32 KB stages of two blocks form a ring: while one stage is consumed up to three
//    are in flight, and a round only waits (s_waitcnt vmcnt(N)) for its own stage.  The
//    stages are distinct __shared__ arrays on purpose: the compiler then knows that reading
//    one does not alias the DMA into the others and does not drain the DMA queue before
//    every LDS read.  Measured with two 64 KB stages drained every round: 3.4 TB/s in the
//    steady state, because HBM idled between the bursts.
//  * Contraction (transposed):
//        S^T[key,row] = K.Q^T   (A = K fragment, B = rotated Q in registers as bf16 hi + lo
//                                parts: two MFMA passes, Q rounding drops out of the error)
//        O^T[d,row]  += V^T.P^T (A = V fragment, B = P)
//    with v_mfma_f32_32x32x16_bf16.  One query row lives in lanes n and n+32; softmax
//    statistics never leave them, and the fp32 scores of the first product become, after
//    exponentiation and bf16 packing, the B operand of the second without any cross-lane
//    movement.  The key order inside a block is permuted on the K side (an address, free) so
//    that the 8 probabilities a lane holds for one MFMA belong to 8 consecutive keys, which
//    is what the 8-key interleaved V pool delivers in 16 bytes.
//  * Softmax.  Online max/sum in registers.  The running maximum is exact (the accumulators
//    are rescaled whenever some row of the wave sees a larger score; the rescale is skipped,
//    wave-uniformly, when no row does).  Exactness matters for accuracy: the dominant key of a
//    row then has probability exactly 1.0, which bf16 represents without error; with a stale
//    maximum the largest weight would carry a 2^-9 rounding error into P.V (measured: 3x
//    larger max-abs error).
//  * Waves.  8 waves = (row block of 32 rows) x (key group), KG = 4 / 2 / 1 for <= 2 / <= 4 /
//    <= 8 row blocks; key group kg takes the key blocks gb with gb % KG == kg and every
//    KG-th tail tile.  At the end the groups are merged through LDS in one exchange in which
//    every wave of a row block reduces its own 32-channel slice (identical lane layout on
//    both sides, so the exchange is lane-private).
//  * Tails (Section 4.3.3: every value still grows token by token) are private to a branch.
//    A first version used wavefront-reduction dot products (16 lanes per key row); measured
//    on MI355X it needed ~1000 VALU instructions per branch and 5 us per branch per wave,
//    more than the whole prefix.  The tails now go through the same MFMA code as masked
//    "virtual key blocks": a tile holds G tail positions of each of the 32/G branches of the
//    row block, the score tile is block-diagonal (a row keeps only its own branch's keys,
//    the rest get -inf), K fragments are loaded straight from the row-major tail pool, and
//    the V fragments - which need 8 keys of one channel - are transposed through a
//    wave-private 8 KB LDS buffer (coalesced 16-byte writes, 2-byte reads, XOR-swizzled so
//    that the two half-waves hit different banks).  The MFMA work wasted on the masked
//    entries is irrelevant: the matrix pipe is idle while the first stage is in flight.
//    Tail tiles are processed first and simply initialise the online-softmax state.
//  * Fused mode (hpd_decode_step): the lanes whose tail-tile entry is the newest token take
//    it from k_new / v_new instead of the pool, rotate and round it with the same arithmetic
//    as hpd_kv_append, store it, and use the rounded registers - bit-identical to the
//    two-call sequence, with no read-back and no extra synchronisation.
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
constexpr int STAGE_BLOCKS = 2;
constexpr int STAGE_U4 = STAGE_BLOCKS * SLOT_U4;  // 32 KB
constexpr int LOADS_PER_ROUND = STAGE_BLOCKS * 16 / WAVES;  // DMA instructions per wave per round
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

// XOR-swizzled row-major park buffer: element (row, 4-float chunk c4) of a 128-float row.
__device__ __forceinline__ int park_off(int row, int c4) { return row * 128 + ((c4 ^ (row & 31)) << 2); }

template <int G>
__global__ void __launch_bounds__(WAVES * 64)
attn_stream_kernel(StreamArgs a, const uint16_t* __restrict__ q, const uint16_t* __restrict__ k_prefix,
                   const uint16_t* __restrict__ v_prefix, uint16_t* __restrict__ k_tail,
                   uint16_t* __restrict__ v_tail, const uint16_t* __restrict__ k_new,
                   const uint16_t* __restrict__ v_new, void* __restrict__ out) {
  constexpr int BPB = 32 / G;  // branches per row block; a tail tile holds G positions of each

  __shared__ uint4 ring0[STAGE_U4];
  __shared__ uint4 ring1[STAGE_U4];
  __shared__ uint4 ring2[STAGE_U4];
  __shared__ uint4 ring3[STAGE_U4];
  __shared__ float l_buf[MAX_ROWS];

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keep it scalar
  const int lane = tid & 63;
  const int n = lane & 31, g2 = lane >> 5;

  // ---- unit descriptor (one dependent load):
  //      {hoff, Hlen, doff, Llen, first live row, live branches, position | -1, first branch | -1}
  const int32_t rg = blockIdx.x % a.RG;
  const int32_t hk = (blockIdx.x / a.RG) % a.Hkv;
  const int32_t u = blockIdx.x / (a.RG * a.Hkv);
  const int32_t* desc = a.tb.unit_desc + (int64_t)u * 8;  // pre-offset to this step by the host
  const int32_t hoff = desc[0], Hlen = desc[1], doff = desc[2], Llen = desc[3];
  const int32_t row0_live = desc[4], nb = desc[5], upos = desc[6], ub0 = desc[7];

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

  // ---- loader role: wave w fills a quarter of block slot w/4 of a stage (K fragments for
  //      quarters 0 and 1, V fragments for 2 and 3): LOADS_PER_ROUND instructions per round,
  //      always the same number, so that vmcnt(N) means the same thing in every wave
  const int32_t ld_slot = wave >> 2;
  const int32_t ld_part = wave & 3;
  // MFMA row m of a score tile carries this key of the block (see the file header)
  const int32_t krow = ((n >> 4) << 4) | (((n >> 2) & 1) << 3) | (((n >> 3) & 1) << 2) | (n & 3);
  const uint16_t* kbase = k_prefix + (int64_t)hk * a.NP * D;
  const uint16_t* vbase = v_prefix + (int64_t)hk * (a.NP / 8) * D * 8;

  // one 32-bit per-lane element offset; everything else in the load addresses is wave-uniform
  const int32_t ld_off = ld_part < 2 ? krow * D + g2 * 8 + ld_part * 64
                                     : (g2 * D + (ld_part - 2) * 64 + n) * 8;
  auto issue_round = [&](int32_t r, uint4* stage) {
    // a slot past the last block re-loads the last block (never read): the count stays fixed
    const int32_t gb = min(r * STAGE_BLOCKS + ld_slot, NB - 1);
    const int32_t slot0 = gb < NBh ? hoff + gb * 32 : doff + (gb - NBh) * 32;
    uint4* dst = stage + ld_slot * SLOT_U4 + ld_part * 4 * 64;
    if (ld_part < 2) {
      const uint16_t* src = kbase + (int64_t)slot0 * D;
#pragma unroll
      for (int f = 0; f < 4; ++f) HPD_GLL(src + (ld_off + f * 16), dst + f * 64);
    } else {
      // V fragment f = d-block * 2 + key half; this wave loads d-blocks 2*(part-2), +1
      const uint16_t* src = vbase + (int64_t)(slot0 / 8) * D * 8;
#pragma unroll
      for (int f = 0; f < 4; ++f)
        HPD_GLL(src + (ld_off + ((f & 1) * 2 * D + (f >> 1) * 32) * 8), dst + f * 64);
    }
  };

  // ---- branches of this row group
  const int32_t br0 = first_blk * BPB;
  const int32_t nbr_here = min(nb - br0, nblk_here * BPB);
  const int32_t rows_here = nbr_here * G;
  auto branch_id = [&](int32_t lb) -> int32_t {
    return ub0 >= 0 ? ub0 + br0 + lb : a.tb.live_branch[a.live_base + row0_live + br0 + lb];
  };
  auto tail_offset = [&](int32_t b) -> int64_t { return (((int64_t)b * a.Hkv + hk) * a.Tcap) * D; };

  // ---- first request, ahead of the DMA in the memory queue: this lane's query row
  const int32_t r_row = (first_blk + rb) * 32 + n;
  const bool row_valid = active && r_row < R;
  const int32_t q_bi = min(r_row / G, nb - 1);
  const int64_t q_off = ((int64_t)(row0_live + q_bi) * a.Hq + hk * G + r_row % G) * D;
  int32_t q_pos = upos;
  if (upos < 0) q_pos = a.tb.branch_base_pos[branch_id(q_bi - br0)] + 1 + a.step;
  uint4 qraw[8];
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) {
    qraw[kk] = make_uint4(0, 0, 0, 0);
    if (row_valid) qraw[kk] = *reinterpret_cast<const uint4*>(q + q_off + kk * 16 + g2 * 8);
  }

  // ---- tail tiles
  // Virtual key k of pool tile ti = (position ti*G + k / BPB, branch k % BPB of this row
  // block), positions 0 .. step-1; the newest token (position step) gets a tile of its own
  // with one key per branch, in both modes, so that the fused and the two-call sequence add
  // up in the same order.  A row may only see the keys of its own branch.
  const int32_t NT = (a.step + G - 1) / G;  // pool tiles: ceil(step / G)
  const int32_t lb0 = rb * BPB;
  const int32_t r4 = lane >> 4, c16 = lane & 15;

  // ---- start the DMA ring: rounds 0 and 1 now; stages 2 and 3 serve as tail staging first
  issue_round(0, ring0);
  if (NR > 1) issue_round(1, ring1);

  // ---- rotate the query: bf16 hi + lo MFMA B operands
  bf16x8 Qh[8], Ql[8];
  {
    const float2* cs_row = a.tb.rope + (int64_t)q_pos * (D / 2);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      const int c0 = kk * 16 + g2 * 8;
      float lo[8], hi[8], rl[8], rh[8];
      unpack8(qraw[kk], lo);
      unpack8(qraw[kk + 4], hi);
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

  // softmax update + P.V for one 32-key tile: S = raw scores (C layout: value i of lane
  // (n, g2) is key (i>>3)*16 + g2*8 + (i&7)), ok = which of them exist for this row,
  // vf = the 8 V fragments (d-block * 2 + key half).
  auto softmax_pv = [&](const floatx16& S, uint32_t ok, const uint4* vf) {
    float s[16];
    float bm = NEG_BIG;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      s[i] = (ok >> i) & 1 ? S[i] * a.scale_log2 : -INFINITY;
      bm = fmaxf(bm, s[i]);
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

  // =====================================================================================
  // Tail tiles
  // =====================================================================================
  if (active) {
    // 8 KB of wave-private staging in the two stages the DMA has not been pointed at yet
    uint16_t* const stage = reinterpret_cast<uint16_t*>(wave < 4 ? ring2 : ring3) + (wave & 3) * 4096;

    // scores from K fragments in registers, V^T fragments out of the staging area (row-major
    // rows, 16-byte chunk index XOR-swizzled by bit 3 of the key), softmax, P.V
    auto tile_core = [&](const uint4* kf, uint32_t ok) {
      floatx16 S;
#pragma unroll
      for (int i = 0; i < 16; ++i) S[i] = 0.f;
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) {
        const bf16x8 kfr = __builtin_bit_cast(bf16x8, kf[kk]);
        S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr, Qh[kk], S, 0, 0, 0);
        S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr, Ql[kk], S, 0, 0, 0);
      }
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the V rows have landed in LDS
      uint4 vf[8];
#pragma unroll
      for (int f = 0; f < 8; ++f) {
        const int blk = f >> 1, hf = f & 1;
        const int d = blk * 32 + n;
        const uint16_t* col = stage + (hf * 16 + g2 * 8) * 128 + ((((d >> 3) ^ (g2 << 2)) << 3) | (d & 7));
        uint32_t w[4];
#pragma unroll
        for (int e2 = 0; e2 < 4; ++e2)
          w[e2] = (uint32_t)col[(2 * e2) * 128] | ((uint32_t)col[(2 * e2 + 1) * 128] << 16);
        vf[f] = make_uint4(w[0], w[1], w[2], w[3]);
      }
      softmax_pv(S, ok, vf);
    };

    // ---- positions 0 .. step-1 from the pool
    for (int32_t ti = kg; ti < NT; ti += KG) {
      const int32_t tau0 = ti * G;
      const int32_t last = a.step - 1;  // clamp: always a written row of a live branch
      uint4 kf[8];
      {
        const int32_t lb = min(lb0 + krow % BPB, nbr_here - 1);
        const uint16_t* kp = k_tail + tail_offset(branch_id(lb)) + (int64_t)min(tau0 + krow / BPB, last) * D + g2 * 8;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) kf[kk] = *reinterpret_cast<const uint4*>(kp + kk * 16);
      }
      // V rows by DMA: lane (r4, c16) of instruction j = chunk c16 of virtual key 4j + r4
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int32_t k = j * 4 + r4;
        const int32_t lb = min(lb0 + k % BPB, nbr_here - 1);
        const uint16_t* vp = v_tail + tail_offset(branch_id(lb)) + (int64_t)min(tau0 + k / BPB, last) * D;
        HPD_GLL(vp + ((c16 ^ (((k >> 3) & 1) << 2)) << 3), stage + j * 4 * 128);
      }
      uint32_t ok = 0;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int k = ((i >> 3) << 4) + g2 * 8 + (i & 7);
        if (k % BPB == n / G && tau0 + k / BPB < a.step) ok |= 1u << i;
      }
      tile_core(kf, ok);
    }

    // ---- the newest token: virtual key k < BPB = branch k (larger k repeat valid rows and
    //      are masked).  Fused mode: take it from k_new / v_new, rotate and round with the
    //      arithmetic of hpd_kv_append, store, and use the rounded registers.
    if (kg == NT % KG) {
      const int32_t lbu = lb0 + krow % BPB;
      const int32_t lb = min(lbu, nbr_here - 1);
      const int32_t b = branch_id(lb);
      const int64_t toff = tail_offset(b) + (int64_t)a.step * D;
      const int64_t noff = ((int64_t)(row0_live + br0 + lb) * a.Hkv + hk) * D;
      uint4 kf[8];
      {
        const uint16_t* kp = (a.fused ? k_new + noff : k_tail + toff) + g2 * 8;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) kf[kk] = *reinterpret_cast<const uint4*>(kp + kk * 16);
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int32_t k = j * 4 + r4;
        const int32_t lbv = min(lb0 + k % BPB, nbr_here - 1);
        const uint16_t* vp = a.fused ? v_new + ((int64_t)(row0_live + br0 + lbv) * a.Hkv + hk) * D
                                     : v_tail + tail_offset(branch_id(lbv)) + (int64_t)a.step * D;
        HPD_GLL(vp + ((c16 ^ (((k >> 3) & 1) << 2)) << 3), stage + j * 4 * 128);
      }
      if (a.fused) {
        const int32_t pos = upos >= 0 ? upos : a.tb.branch_base_pos[b] + 1 + a.step;
        const float2* cs_row = a.tb.rope + (int64_t)pos * (D / 2);
        const bool owner = lbu < nbr_here && krow < BPB;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
          float lo[8], hi[8], rl[8], rh[8];
          unpack8(kf[kk], lo);
          unpack8(kf[kk + 4], hi);
          const float4* csp = reinterpret_cast<const float4*>(cs_row + kk * 16 + g2 * 8);
#pragma unroll
          for (int e2 = 0; e2 < 4; ++e2) {
            const float4 cs = csp[e2];
            hpd::rope_pair(lo[2 * e2], hi[2 * e2], cs.x, cs.y, rl[2 * e2], rh[2 * e2]);
            hpd::rope_pair(lo[2 * e2 + 1], hi[2 * e2 + 1], cs.z, cs.w, rl[2 * e2 + 1], rh[2 * e2 + 1]);
          }
          kf[kk] = __builtin_bit_cast(uint4, pack8(rl));
          kf[kk + 4] = __builtin_bit_cast(uint4, pack8(rh));
          if (owner) {
            *reinterpret_cast<uint4*>(k_tail + toff + g2 * 8 + kk * 16) = kf[kk];
            *reinterpret_cast<uint4*>(k_tail + toff + g2 * 8 + (kk + 4) * 16) = kf[kk + 4];
          }
        }
      }
      uint32_t ok = 0;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int k = ((i >> 3) << 4) + g2 * 8 + (i & 7);
        if (k < BPB && k == n / G) ok |= 1u << i;
      }
      if (a.fused) {
        // the value rows of the newest token: out of the staging area into the pool
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
        for (int j = 0; j < (BPB + 3) / 4; ++j) {
          const int32_t k = j * 4 + r4;
          if (k < BPB && lb0 + k < nbr_here) {
            const uint4 v = *reinterpret_cast<const uint4*>(stage + k * 128 + (c16 << 3));
            *reinterpret_cast<uint4*>(v_tail + tail_offset(branch_id(lb0 + k)) + (int64_t)a.step * D +
                                      ((c16 ^ (((k >> 3) & 1) << 2)) << 3)) = v;
          }
        }
      }
      tile_core(kf, ok);
    }
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
    uint32_t ok = 0xffffu;
    if (valid < 32) {
      ok = 0;
#pragma unroll
      for (int i = 0; i < 16; ++i)
        if (((i >> 3) << 4) + g2 * 8 + (i & 7) < valid) ok |= 1u << i;
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
    softmax_pv(S, ok, vf);
  };

  // Round r: wait until its stage has landed (newer rounds may stay in flight: the DMA
  // instructions of a wave complete in order and every wave issues LOADS_PER_ROUND per
  // round), meet, refill the stage that was consumed last round, compute.
  auto round_body = [&](int32_t r, const uint4* cur, uint4* refill, uint4* refill0) {
    const int32_t newer = r == 0 ? min(1, NR - 1) : min(2, NR - 1 - r);  // rounds issued after r
    if (newer >= 2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * LOADS_PER_ROUND) : "memory");
    else if (newer == 1) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LOADS_PER_ROUND) : "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): LDS reads of the previous round are done
    __builtin_amdgcn_s_barrier();
    if (r == 0) {
      // the tail staging is finished in every wave: point the DMA at stages 2 and 3
      if (NR > 2) issue_round(2, refill0);
      if (NR > 3) issue_round(3, refill);
    } else if (r + 3 < NR) {
      issue_round(r + 3, refill);
    }
    if (active) {
#pragma unroll
      for (int32_t j = 0; j < STAGE_BLOCKS; ++j) {
        const int32_t gb = r * STAGE_BLOCKS + j;
        if (gb < NB && gb % KG == kg) {
          const int32_t valid = gb < NBh ? min(32, Hlen - gb * 32) : min(32, Llen - (gb - NBh) * 32);
          compute_block(cur + j * SLOT_U4, valid);
        }
      }
    }
  };

  // stage of round r is ring[r % 4]; round r refills ring[(r + 3) % 4] (consumed in round r-1)
  for (int32_t r = 0; r < NR; r += 4) {
    round_body(r, ring0, ring3, ring2);
    if (r + 1 < NR) round_body(r + 1, ring1, ring0, nullptr);
    if (r + 2 < NR) round_body(r + 2, ring2, ring1, nullptr);
    if (r + 3 < NR) round_body(r + 3, ring3, ring2, nullptr);
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();  // all stages are dead from here on and get reused

  // ---- merge the key groups: every wave of a row block reduces its own d-blocks.
  //      Wave w parks what the others need in region w: stage (w & 3), half (w >> 2).
  float* const park0 = reinterpret_cast<float*>(ring0);
  float* const park1 = reinterpret_cast<float*>(ring1);
  float* const park2 = reinterpret_cast<float*>(ring2);
  float* const park3 = reinterpret_cast<float*>(ring3);
  auto region = [&](int32_t w) -> float* {
    float* base = (w & 2) ? ((w & 1) ? park3 : park2) : ((w & 1) ? park1 : park0);
    return base + (w >> 2) * (50 * 64) + lane;
  };
  const int32_t DB = 4 / KG;  // d-blocks reduced by one wave: blocks kg*DB .. kg*DB + DB - 1
  if (KG > 1) {
    if (active) {
      float* buf = region(wave);
      int32_t sidx = 0;
#pragma unroll
      for (int blk = 0; blk < 4; ++blk) {
        if (blk / DB != kg) {  // not mine: somebody else reduces it
#pragma unroll
          for (int i = 0; i < 16; ++i) buf[(sidx * 16 + i) * 64] = acc[blk][i];
          ++sidx;
        }
      }
      buf[48 * 64] = m_used;
      buf[49 * 64] = l_lane;
    }
    __syncthreads();
    if (active) {
      float m_o[3], l_o[3];
      float m_new = m_used;
      for (int32_t o = 0; o < KG - 1; ++o) {
        const int32_t okg = o < kg ? o : o + 1;  // the other key groups of this row block
        const float* buf = region(rb * KG + okg);
        m_o[o] = buf[48 * 64];
        l_o[o] = buf[49 * 64];
        m_new = fmaxf(m_new, m_o[o]);
      }
      const float a_own = fast_exp2(m_used - m_new);
      l_lane *= a_own;
#pragma unroll
      for (int blk = 0; blk < 4; ++blk)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[blk][i] *= a_own;
      for (int32_t o = 0; o < KG - 1; ++o) {
        const int32_t okg = o < kg ? o : o + 1;
        const float* buf = region(rb * KG + okg);
        const float a_o = fast_exp2(m_o[o] - m_new);
        l_lane += l_o[o] * a_o;
        // my blocks sit in the other wave's region at the index that skips ITS own blocks
#pragma unroll
        for (int blk = 0; blk < 4; ++blk) {
          if (blk / DB == kg) {
            const int32_t sidx = blk - (blk / DB > okg ? DB : 0);
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[blk][i] += buf[(sidx * 16 + i) * 64] * a_o;
          }
        }
      }
      m_used = m_new;
    }
    __syncthreads();
  }

  // ---- park the finished rows row-major (64 rows per stage): each wave its own d-blocks ...
  if (active) {
    const int32_t lr = rb * 32 + n;
    float* park = (lr & 128) ? ((lr & 64) ? park3 : park2) : ((lr & 64) ? park1 : park0);
    const int32_t lrr = lr & 63;
#pragma unroll
    for (int blk = 0; blk < 4; ++blk) {
      if (blk / DB == kg) {
#pragma unroll
        for (int cc = 0; cc < 4; ++cc)
          *reinterpret_cast<float4*>(park + park_off(lrr, blk * 8 + cc * 2 + g2)) =
              make_float4(acc[blk][cc * 4 + 0], acc[blk][cc * 4 + 1], acc[blk][cc * 4 + 2], acc[blk][cc * 4 + 3]);
      }
    }
    if (kg == 0) {
      const float l_row = l_lane + __shfl_xor(l_lane, 32);
      if (g2 == 0) l_buf[lr] = l_row;
    }
  }
  __syncthreads();

  // ---- ... and write them normalised, 4 rows per wave pass, 512 contiguous bytes per row
  {
    const int32_t ks = lane >> 4, c = lane & 15;
    for (int32_t lr = wave * 4 + ks; lr < rows_here; lr += WAVES * 4) {
      const float inv = 1.0f / l_buf[lr];
      const float* park = (lr & 128) ? ((lr & 64) ? park3 : park2) : ((lr & 64) ? park1 : park0);
      const int32_t lrr = lr & 63;
      const float4 p0 = *reinterpret_cast<const float4*>(park + park_off(lrr, 2 * c));
      const float4 p1 = *reinterpret_cast<const float4*>(park + park_off(lrr, 2 * c + 1));
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
