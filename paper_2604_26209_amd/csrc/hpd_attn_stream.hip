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
//  * One stream of key blocks.  Everything a unit attends to is cut into blocks of 32 keys
//    (16 KB: a K half and a V half): the header blocks, the document blocks, and then "tail
//    tiles" that hold 8 positions of each of 4 branches (Section 4.3.3: every value still
//    grows token by token; the tails are private to a branch, so a row keeps only the keys of
//    its own branch in a tile and the rest get probability 0).  A tail tile is gathered by the
//    same 16-byte loads as a prefix block from the row-major tail pools.  Its K half looks
//    like a prefix block's; its V half arrives as 32 rows of 256 bytes (the pool order: an
//    append then is one coalesced row, where an 8-position interleave would cost a 2-byte
//    scatter per channel) and is transposed by the consumer's LDS reads (the transposing
//    8-byte read of gfx950; rows swizzled at load time so that a read hits every bank once).
//  * Loading.  Blocks travel HBM -> LDS with direct-to-LDS 16-byte loads
//    (global_load_lds_dwordx4): no VGPRs are held by data in flight.  The V half of a prefix
//    block is fetched in fragment order (a lane fetches exactly the 16 bytes that the same
//    lane of a consumer feeds to an MFMA; the interleaved pool makes that 512-byte runs); the
//    K half is fetched as 32 whole rows, whose 16-byte chunks are XOR-permuted at fetch time so
//    that the per-lane fragment reads are conflict-free.  Loads that gather 32 bytes per row
//    instead were measured to stall the issuing wave: every distinct cache line of an
//    instruction is a separate request.  Four stages form a ring: while one is consumed up
//    to three are in flight, and a round only waits (s_waitcnt vmcnt(N)) for its own stage.
//  * Roles.  The last waves of the workgroup only load; the others only compute.  Under load
//    a DMA instruction blocks the issuing wave until the memory pipeline takes it, so
//    whatever a loading wave computes is time in which nothing is requested; and vector
//    memory operations of a wave complete in order, so a wave with a deep DMA queue cannot
//    get a latency-critical load through.  The two roles run different code paths and meet
//    at barriers only.  (The prefill attention, which is bound by the compute waves and far
//    from saturating the memory pipeline, runs a shape without loader waves: see DenseShape.)
//  * Contraction (transposed):
//        S^T[key,row] = K.Q^T   (A = K fragment, B = rotated, pre-scaled Q in registers)
//        O^T[d,row]  += V^T.P^T (A = V fragment, B = P)
//    both with v_mfma_f32_32x32x16_f16: the pools hold their bf16 values in half format,
//    exactly, and the query and the softmax weights keep 11 significant bits (with a bf16
//    query the error was 2.5e-2 x RMS, and a bf16 hi + lo pair costs a second pass).  One query
//    row lives in lanes n and n+32; softmax statistics never leave them, and the fp32 scores of
//    the first product become, after exponentiation and packing, the B operand of the second
//    without any cross-lane movement.  The key order inside a block is permuted on the K side
//    (an address, free) so that the 8 probabilities a lane holds for one MFMA belong to 8
//    consecutive keys, which is what the 8-key interleaved V pool delivers in 16 bytes.
//  * Softmax.  Online max/sum in registers.  The reference point of a row's exponentials
//    follows its running maximum within a factor of 2^8: the accumulators are rescaled, wave-
//    uniformly, only when some row of the wave sees a score that exceeds its reference point
//    by more - in the first blocks of a row, then hardly ever (with the exact maximum, most
//    blocks of 32 keys raise the maximum of one of the wave's 32 rows, and the 64 multiplies
//    of a rescale were a quarter of the vector instructions).  This rests on the weights being
//    halves: with bf16 weights the largest weight of a row has to be exactly 1.0 - an exact
//    maximum - or its 2^-9 rounding error shows in rows that one or two keys dominate
//    (measured: 2.4e-2 x RMS against 0.9e-2).
//  * Compute waves = (row block of 32 rows) x (key group), with as many key groups (at most
//    4) as fit; key group kg takes the prefix blocks gb with gb % KG == kg, and the tail tiles
//    of a row block go round its key groups.  At the end the groups are merged through LDS in
//    one exchange in which every wave of a row block reduces its own 32-channel slices
//    (identical lane layout on both sides, so the exchange is lane-private), normalises them
//    and writes them out.
//  * Cache policy.  What is touched once per launch - document blocks (when a single row
//    group streams them), tail rows, the output rows of a wave that holds whole rows - moves
//    with the streaming (non-temporal) hint; what is re-read (header blocks, query rows, the
//    appended rows) does not.
//  * Fused mode (hpd_decode_step): the compute waves rotate, round and store the new keys and
//    values of the unit's branches (the arithmetic of hpd_kv_append) right after they have
//    rotated the query - the rotated query is what the first round waits for, the stores can
//    complete behind it; a ring barrier publishes them before the first tail tile is
//    requested, and the tail tiles - which are last in the stream - read them back like any
//    other token.  Both modes therefore add up in the same order and give identical bits.
//  * HPD_MASK_PAPER (the literal mask of Section 4.3.2 over the whole stacked prompt) is a
//    second instantiation of the same kernel; see the comment at the kernel.
#include <algorithm>
#include <cmath>

#include "hpd_internal.h"
#include "hpd_device.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int D = 128;
constexpr int SLOT_U4 = 16 * 64;  // one 32-key block: 8 K + 8 V fragments of 64 x 16 bytes
constexpr float NEG_BIG = -1.0e30f;

// Two shapes of workgroup:
//   wide    6 compute waves + 2 loaders, stages of two blocks: 128.5 KB of LDS, one workgroup
//           per CU.  For launches with about one unit per CU: all of the CU's resources go
//           into streaming that one unit.
//   narrow  3 compute waves + 1 loader, stages of one block: 64.5 KB of LDS, two workgroups
//           per CU.  For launches with many units per CU: the start (query staging, rotation)
//           and the end (merge, stores) of one unit overlap with the stream of another.
template <int CW_, int LW_, int SB_>
struct Shape {
  static constexpr int CW = CW_;                 // compute waves (waves 0 .. CW-1)
  static constexpr int LW = LW_;                 // loader waves (waves CW ..)
  static constexpr int SB = SB_;                 // blocks per stage
  static constexpr int WAVES = CW + LW;
  static constexpr int STAGE_U4 = SB * SLOT_U4;
  static constexpr int STAGE_ROWS = STAGE_U4 / 16;        // 256-byte rows a stage can hold
  static constexpr int LOADS_PER_ROUND = SB * 16 / (LW ? LW : CW);  // DMA instructions per loading wave per stage
  static constexpr int MAX_BLOCKS = CW;                   // row blocks per workgroup
};
using WideShape = Shape<6, 2, 2>;
using NarrowShape = Shape<3, 1, 1>;
//   dense   4 compute waves that also load (no loader waves), stages of one block, two
//           workgroups per CU.  For the prefill attention, which is bound by the matrix and
//           vector work of the compute waves: two compute waves on every SIMD (a wave overlaps
//           its matrix and its vector instructions only with those of another wave on its
//           SIMD), and the memory pipeline, far from saturated there, takes the 4 DMA
//           instructions a wave issues per stage without holding it up.
using DenseShape = Shape<4, 0, 1>;

struct StreamArgs {
  hpd_dev_tables tb;
  int32_t step, Hq, Hkv, Tcap, RG, n_groups, out_f32, fused, live_base;
  int32_t Gr;  // query heads per kv head; the kernel's G is the next power of two (padding rows are neither loaded nor stored)
  int64_t NP;
  float scale_log2;
};

#define HPD_GLL(gptr, lptr)                                                                   \
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(gptr),   \
                                   (__attribute__((address_space(3))) void*)(lptr), 16, 0, 0)
// the same with the streaming (non-temporal) cache hint
#define HPD_GLL_NT(gptr, lptr)                                                                \
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(gptr),   \
                                   (__attribute__((address_space(3))) void*)(lptr), 16, 0, 2)

// The same two instructions (M0 = LDS byte address of lane 0's 16 bytes, then the load) written
// out, for waves that request blocks and also read them: the compiler makes every LDS read of a
// wave wait for all loads-to-LDS the wave has in flight (it cannot tell the stage that is read
// from the stages that are being filled), and the ring lives on loads that stay in flight across
// the reads.  Which stage may be read is what the barriers of the rounds establish.
__device__ __forceinline__ void dma16(const void* g, const void* l) {
  const uint32_t la = (uint32_t)__builtin_amdgcn_readfirstlane(
      (int32_t)reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) const void*)l));
  uint32_t keep;  // M0 is the compiler's: put back what it held
  asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %1, off\n\ts_mov_b32 m0, %0"
               : "=&s"(keep)
               : "v"(g), "s"(la)
               : "memory");
}
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
// 8 keys of the cache: rounded to bf16, written as halves
__device__ __forceinline__ uint4 pack8_key(const float* v) {
  float r[8];
  unpack8(__builtin_bit_cast(uint4, pack8(v)), r);
  return make_uint4(hpd::cache_bits_pair(r[0], r[1]), hpd::cache_bits_pair(r[2], r[3]),
                    hpd::cache_bits_pair(r[4], r[5]), hpd::cache_bits_pair(r[6], r[7]));
}
// 8 bf16 values as cache elements
__device__ __forceinline__ uint4 cache8(uint4 w) {
  return make_uint4(hpd::cache_bits_from_bf16_pair(w.x), hpd::cache_bits_from_bf16_pair(w.y),
                    hpd::cache_bits_from_bf16_pair(w.z), hpd::cache_bits_from_bf16_pair(w.w));
}
// 8 values (of the query, of the softmax weights) as halves, rounded to nearest
__device__ __forceinline__ f16x8 pack8_half(const float* v) {
  f16x8 h;
#pragma unroll
  for (int e = 0; e < 8; ++e) h[e] = (_Float16)v[e];
  return h;
}
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
constexpr float MAX_SLACK = 8.f;  // log2 units: how far a score may exceed the reference point of its row

// c + the two halves of w (v_dot2_f32_f16 with a pair of ones)
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float sum_half_pair(uint32_t w, float c) {
  return __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, w), __builtin_bit_cast(f16x2, 0x3c003c00u), c, false);
}

// ds_read_b64_tr_b16: within each 16 lanes, lane i receives element i % 4 of the 8 bytes that the
// lanes 4*j + i/4 (j = 0..3) address, in the order of j: a 4 x 16 transpose of 2-byte elements.
typedef short short4v __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint2 lds_read_tr16(const char* p) {
  const short4v v = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (__attribute__((address_space(3))) short4v*)(uintptr_t)p);
  return __builtin_bit_cast(uint2, v);
}

// A 32-bit word at a wave-uniform address through the scalar data cache (read only).  The
// loaders use it for table lookups: a vector load would have to wait for every DMA instruction
// in front of it, because vector memory operations of a wave complete in order.
__device__ __forceinline__ int32_t scalar_load(const int32_t* p) {
  // (the address is wave-uniform by the caller's construction; where the compiler keeps it in
  // vector registers all the same, it is moved to scalar ones here)
  const uint64_t u = reinterpret_cast<uint64_t>(p);
  // (readfirstlane returns a signed int: without the casts a low half with its top bit set
  // would be sign-extended over the high half)
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int32_t)(u >> 32));
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int32_t)(uint32_t)u);
  p = reinterpret_cast<const int32_t*>(((uint64_t)hi << 32) | (uint64_t)lo);
  int32_t v;
  asm volatile("s_load_dword %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=s"(v) : "s"(p) : "memory");
  return v;
}

// 8 channel pairs (c .. c+7, 64+c .. 64+c+7) of one row, rotated at the (cos, sin) row cs_row
__device__ __forceinline__ void rotate16(uint4 raw_lo, uint4 raw_hi, const float2* cs_row, int c,
                                         float rl[8], float rh[8]) {
  float lo[8], hi[8];
  unpack8(raw_lo, lo);
  unpack8(raw_hi, hi);
  const float4* csp = reinterpret_cast<const float4*>(cs_row + c);
#pragma unroll
  for (int e2 = 0; e2 < 4; ++e2) {
    const float4 cs = csp[e2];
    hpd::rope_pair(lo[2 * e2], hi[2 * e2], cs.x, cs.y, rl[2 * e2], rh[2 * e2]);
    hpd::rope_pair(lo[2 * e2 + 1], hi[2 * e2 + 1], cs.z, cs.w, rl[2 * e2 + 1], rh[2 * e2 + 1]);
  }
}

// PAPER = the literal mask of Section 4.3.2 (one causal order by position ID over the whole
// stacked prompt).  The work unit is then (prompt, kv head, row group): the rows are the live
// branches of the prompt, the prefix is the header and ALL documents of the prompt (block list
// from a table), and the tail tiles run over every branch of the prompt from the first to the
// row group's last - finished ones included, up to the length they reached -, a row keeping
// the keys of the branches that are not later than its own.
//
// MODE_PREFILL = the attention of the prefix tokens themselves (Section 4.3.2, first inference
// step, under the block mask): the work unit is (segment, kv head, row group), a segment being
// a header or a document; the rows are the segment's tokens (x G heads), each rotated at its
// own position ID; the keys are the header (documents only) and the segment itself up to the
// row's token: the stream stops at the row group's last token, a wave skips the blocks behind
// its last row, and the blocks on the diagonal get a per-row count.  No tails, no append.
// MODE_PAGED = MODE_BLOCK with the tail rows found through the caller's page table.
// MODE_PREFILL_LIST = MODE_PREFILL under the literal mask: what a segment sees in full (the
// header and the earlier documents of its prompt) is a list of blocks with a key count each
// instead of the header's run of slots, and the names' positions come from a table.
enum { MODE_BLOCK = 0, MODE_PAPER = 1, MODE_PREFILL = 2, MODE_PAGED = 3, MODE_PREFILL_LIST = 4 };
template <int G, typename SH, int MODE>
__global__ void __launch_bounds__(SH::WAVES * 64, 2)
attn_stream_kernel(StreamArgs a, const uint16_t* __restrict__ q, const uint16_t* __restrict__ k_prefix,
                   const uint16_t* __restrict__ v_prefix, uint16_t* __restrict__ k_tail,
                   uint16_t* __restrict__ v_tail, const uint16_t* __restrict__ k_new,
                   const uint16_t* __restrict__ v_new, void* __restrict__ out) {
  constexpr bool PAPER = MODE == MODE_PAPER, PAGED = MODE == MODE_PAGED, PLIST = MODE == MODE_PREFILL_LIST;
  constexpr bool PREFILL = MODE == MODE_PREFILL || PLIST;
  constexpr int BPB = 32 / G;              // branches (PREFILL: tokens) per row block
  constexpr int QPR = G >= 8 ? 1 : 8 / G;  // branch quads (tail tiles per 8 positions) per row block
  constexpr int CWAVES = SH::CW, LOADERS = SH::LW, STAGE_BLOCKS = SH::SB, STAGE_U4 = SH::STAGE_U4;
  constexpr bool SELF = LOADERS == 0;  // the compute waves issue the loads themselves
  static_assert(!SELF || (STAGE_BLOCKS * 4 == CWAVES), "one quarter of a block per wave and stage");
  constexpr int LOADS_PER_ROUND = SH::LOADS_PER_ROUND, STAGE_ROWS = SH::STAGE_ROWS;
  static_assert(2 * STAGE_ROWS >= CWAVES * 32, "stages 2 and 3 must hold the query rows of a row group");
  static_assert(3 * LOADS_PER_ROUND <= 63, "three rounds in flight must fit the vmcnt counter");

  __shared__ uint4 ring0[STAGE_U4];
  __shared__ uint4 ring1[STAGE_U4];
  __shared__ uint4 ring2[STAGE_U4];
  __shared__ uint4 ring3[STAGE_U4];
  __shared__ float4 rope_q[32];  // (cos, sin) row of the unit's shared position
  // first pool row of the newest chunk of tail positions, per branch of the row group
  __shared__ int64_t chunk_row[(MODE == MODE_BLOCK || MODE == MODE_PAGED) ? SH::CW * 32 : 1];
  constexpr int MAX_KEY_BRANCHES = 256;
  __shared__ int32_t klen[PAPER ? MAX_KEY_BRANCHES : 1];  // tokens in memory of every key branch
  constexpr int MAX_LIST_BLOCKS = 512;
  __shared__ int32_t bvalid[(PAPER || PLIST) ? MAX_LIST_BLOCKS : 1];  // second entry of the prompt's block list

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keep it scalar
  const int lane = tid & 63;
  const int n = lane & 31, g2 = lane >> 5;

  // ---- unit descriptor (one dependent load):
  //      {hoff, Hlen, doff, Llen, first live row, live branches, position | -1, first branch | -1}
  // Workgroup b runs on XCD b % 8, and every XCD has an L2 of its own: the row groups of one
  // (unit, kv head), which stream the same prefix, get indices 8 apart - same XCD, dispatched
  // together - so that the second one finds the blocks in that L2.
  const int32_t rg = (blockIdx.x >> 3) % a.RG;
  const int32_t grp = ((blockIdx.x >> 3) / a.RG) * 8 + (blockIdx.x & 7);  // (unit, kv head)
  if (grp >= a.n_groups) return;  // the grid is padded to a multiple of 8 groups
  const int32_t hk = grp % a.Hkv;
  const int32_t u = grp / a.Hkv;
  // PAPER: {hoff, Hlen, first entry of the prompt's block list, document blocks, first live
  //         row, live branches, first branch of the prompt, first live branch | -1, key branches}
  // PREFILL: {hoff, Hlen (0 for a header unit), first slot of the segment, its tokens, first
  //         token in the order of q / out, tokens again, position ID of the first token, 0}
  // PLIST:  {first entry of the prompt's block list, list blocks the segment sees in full, then
  //         as PREFILL; for the names the position entry is -(1 + first entry in skel_pos)}
  const int32_t* desc = (PAPER ? a.tb.punit_desc : PREFILL ? a.tb.funit_desc : a.tb.unit_desc) +
                        (int64_t)u * (PAPER ? 16 : 8);  // pre-offset to this step by the host
  const int32_t hoff = desc[0], Hlen = desc[1], doff = desc[2], Llen = desc[3];
  const int32_t row0_live = desc[4], nb = desc[5], upos = (PAPER || PREFILL) ? -1 : desc[6], ub0 = desc[7];
  const int32_t pb0 = PAPER ? desc[6] : 0;
  const int32_t seg_pos0 = PREFILL ? desc[6] : 0;

  const int32_t R = nb * G;
  const int32_t nblk = (R + 31) >> 5;
  // (decode: the row blocks of a unit are shared out evenly over its row groups; prefill, where
  // the host sizes RG for the longest segment of the batch: full row groups one after the
  // other, so that a short segment is not cut into many small ones)
  const int32_t per_group = PREFILL ? CWAVES : (nblk + a.RG - 1) / a.RG;  // <= MAX_BLOCKS by the host's choice of RG
  const int32_t first_blk = rg * per_group;
  const int32_t nblk_here = min(per_group, nblk - first_blk);
  if (nblk_here <= 0) return;  // uniform over the workgroup
  // compute waves = (row block) x (key group), with as many key groups (at most 4) as fit:
  // 6 waves: 1 row block x 4, 2 x 2, 3 x 2, 4..6 x 1; 3 waves: 1 x 3, 2..3 x 1.  (Two row blocks
  // x 3 key groups would use all six waves, but then two compute waves share each of two
  // SIMDs and the prologue - every wave rotates its query - takes twice as long there;
  // measured: 4 waves, one per SIMD, are 3 % faster on the Llama-3-8B configuration.)
  int32_t KG = 1;
  for (int32_t k = 2; k <= 4; ++k)
    if (k * nblk_here <= CWAVES) KG = k;
  if (CWAVES == 6 && nblk_here == 2) KG = 2;
  const int32_t NRB = KG == 1 ? CWAVES : nblk_here;  // row-block slots
  const bool loader = wave >= CWAVES;
  int32_t kg = 0;
  while ((kg + 1) * NRB <= wave) ++kg;
  const int32_t rb = wave - kg * NRB;
  const bool active = kg < KG && rb < nblk_here;

  // ---- branches of this row group
  const int32_t br0 = first_blk * BPB;
  const int32_t nbr_here = min(nb - br0, nblk_here * BPB);
  const int32_t rows_here = nbr_here * G;
  // global id of the unit's li-th live branch / of the row group's lb-th
  auto unit_branch = [&](int32_t li) -> int32_t {
    return ub0 >= 0 ? ub0 + li : a.tb.live_branch[a.live_base + row0_live + li];
  };
  auto branch_id = [&](int32_t lb) -> int32_t { return unit_branch(br0 + lb); };
  // PAPER: the tails the row group sees are those of the prompt's branches 0 .. kb_end-1
  // (numbered from the prompt's first), kb_end-1 being the branch of its last row
  const int32_t kb_end = PAPER ? __builtin_amdgcn_readfirstlane(branch_id(nbr_here - 1)) - pb0 + 1 : 0;

  // ---- the stream: NB prefix blocks, then NQ * NC tail tiles (quad-major inside a chunk of 8
  //      positions), two blocks per round
  // (PREFILL: the document blocks up to the row group's last token)
  const int32_t NBh = PLIST ? Hlen : (Hlen + 31) >> 5;
  const int32_t NBd = PAPER ? Llen : PREFILL ? ((br0 + nbr_here - 1) >> 5) + 1 : (Llen + 31) >> 5;
  const int32_t NB = NBh + NBd;
  const int32_t NQ = ((PAPER ? kb_end : nbr_here) + 3) >> 2;  // quads of 4 (key) branches
  const int32_t NC = (a.step >> 3) + 1;    // chunks of 8 positions that hold positions 0 .. step
  // The newest chunk holds step % 8 + 1 positions.  A tile of 8 positions x 4 branches would
  // be loaded and multiplied in full for them; instead the tile takes fewer positions of more
  // branches - 4 x 8, 2 x 16 or 1 x 32, key k = position k % NPOS of branch k / NPOS - so that
  // the number of tiles, hence of loads and of matrix blocks, follows the number of tail keys
  // that exist (which is what the tails cost in bytes).  The rows come from everywhere in the
  // tail pools; where each branch's rows start is kept in LDS (chunk_row).
  constexpr bool FMT = MODE == MODE_BLOCK || MODE == MODE_PAGED;
  const int32_t newest = (a.step & 7) + 1;  // positions in the newest chunk
  const int32_t fmt_lg = !FMT ? 3 : newest <= 1 ? 0 : newest <= 2 ? 1 : newest <= 4 ? 2 : 3;  // log2(NPOS)
  const bool use_fmt = FMT && fmt_lg < 3;
  const int32_t n_full_tiles = use_fmt ? NQ * (NC - 1) : NQ * NC;  // tiles of 8 positions x 4 branches
  const int32_t n_fmt_tiles = use_fmt ? (nbr_here + (32 >> fmt_lg) - 1) >> (5 - fmt_lg) : 0;
  const int32_t NTT = PREFILL ? 0 : n_full_tiles + n_fmt_tiles;
  const int32_t NBT = NB + NTT;
  const int32_t NR = (NBT + STAGE_BLOCKS - 1) / STAGE_BLOCKS;
  // A round is one stage while the stream is in the prefix and two stages from the first
  // tail tile on: a tail tile keeps a single wave busy (a prefix block: a whole key group),
  // so the more tiles meet in a round, the more waves work on them side by side.  Two stages
  // are what the ring allows (the other two are in flight).
  const int32_t s_tail = NB / STAGE_BLOCKS;  // first stage that holds a tail tile
  auto round_end = [&](int32_t s0) -> int32_t { return s0 < s_tail ? s0 + 1 : min(s0 + 2, NR); };
  // Tail tile tt is chunk tt / NQ (8 positions) of the quad of branches quad_of(tt % NQ): the
  // quads are taken row block by row block first (the first quad of every row block, then the
  // second, ...), so that neighbouring tiles go to different waves.
  auto quad_of = [&](int32_t o) -> int32_t {
    if (PAPER) return o;
    int32_t m = 0;
    for (;;) {
      const int32_t n_m = (NQ - m + QPR - 1) / QPR;  // quads whose index within the row block is m
      if (o < n_m) break;
      o -= n_m;
      ++m;
    }
    return o * QPR + m;
  };
  // ---- rows
  const int32_t lr = rb * 32 + n;  // row within the row group
  const int32_t r_row = first_blk * 32 + lr;
  const bool row_valid = active && lr < rows_here;
  const int32_t r4 = lane >> 4, c16 = lane & 15;

  // ---- loader role (the waves after the compute waves): loader j fills block slot j of a
  //      stage (slots j, j + LW, ... if there are fewer loaders than slots), quarter by quarter
  //      (the K half in quarters 0 and 1, the V half in 2 and 3): LOADS_PER_ROUND instructions
  //      per round, always the same number, so that vmcnt(N) means the same thing in every
  //      round.  A loader does nothing else: under load a DMA instruction blocks the issuing
  //      wave until the memory pipeline takes it, and whatever that wave would compute
  //      afterwards is time in which nothing is requested (measured: bandwidth dropped by the
  //      full compute time when the loading waves also computed).  Every instruction reads
  //      whole 256-byte rows or 512-byte runs: a load whose lanes touch 64 different cache
  //      lines costs the memory pipeline 8 times as much as one whose lanes touch 8.
  // MFMA row m of a score tile carries this key of the block (see the file header)
  const int32_t krow = ((n >> 4) << 4) | (((n >> 2) & 1) << 3) | (((n >> 3) & 1) << 2) | (n & 3);
  // K half of a slot (prefix and tail): 32 rows of 256 bytes, row = key, the 16-byte chunk c of
  // row k at position c ^ (k & 15) (conflict-free fragment reads).  Load f of quarter h brings
  // rows k = h*16 + f*4 + lane/16: lane%16 is the position, so the chunk to fetch is
  // (lane%16) ^ (f*4 + lane/16).
  // V half of a prefix block: fragment order, straight out of the 8-key interleaved pool:
  // key halves 0 / 1 (2*D*8 elements apart) of d-blocks 2*h, 2*h+1 (32 channels * 8 apart).
  // V half of a tail tile: 32 rows of 256 bytes like K, chunk position c ^ 2*(k & 3): the
  // transposing fragment read of the consumer takes 32 bytes of each of 4 consecutive rows per
  // 16 lanes, which this spreads over all banks.
  //
  // A wave issues one instruction every few cycles at best, and a loader's requests are the
  // stream: whatever it executes between two DMA instructions is time in which nothing is
  // requested (measured: with ~150 scalar and vector instructions per four loads the issue of a
  // block took longer than its transfer).  So everything that depends on the lane alone is
  // computed once (byte offsets of its 16 bytes inside a block: ck, kq, vq, cv), the address of a
  // load is a wave-uniform base plus such a 32-bit offset, and a block is 16 loads in a row.
  uint32_t ck[4], kq[4];
#pragma unroll
  for (int f = 0; f < 4; ++f) {
    ck[f] = (uint32_t)((c16 ^ r4 ^ (4 * f)) << 4);   // chunk of row f*4 + r4 this lane fetches (K rows)
    kq[f] = (uint32_t)(f * 1024 + r4 * 256) + ck[f];  // ... plus the row inside the quarter of a prefix block
  }
  const uint32_t cv = (uint32_t)((c16 ^ (2 * r4)) << 4);  // chunk of a V row of a tail tile (row % 4 = r4)
  const uint32_t vq = (uint32_t)((g2 * 128 + n) << 4);  // this lane's 16 bytes of a V fragment run
  const char* const kpool = reinterpret_cast<const char*>(k_prefix) + (int64_t)hk * a.NP * (D * 2);
  const char* const vpool = reinterpret_cast<const char*>(v_prefix) + (int64_t)hk * a.NP * (D * 2);
  const char* const ktb = reinterpret_cast<const char*>(k_tail);
  const char* const vtb = reinterpret_cast<const char*>(v_tail);
  // 16 loads of a prefix block: K quarters 0, 1 (rows 0..15, 16..31), V quarters 2, 3
#define HPD_PREFIX_BLOCK(GL)                                                                      \
  GL(sK + kq[0], dst); GL(sK + kq[1], dst + 1024); GL(sK + kq[2], dst + 2048); GL(sK + kq[3], dst + 3072); \
  GL(sK + 4096 + kq[0], dst + 4096); GL(sK + 4096 + kq[1], dst + 5120);                          \
  GL(sK + 4096 + kq[2], dst + 6144); GL(sK + 4096 + kq[3], dst + 7168);                          \
  GL(sV + vq, dst + 8192); GL(sV + 4096 + vq, dst + 9216); GL(sV + 512 + vq, dst + 10240);       \
  GL(sV + 4608 + vq, dst + 11264);                                                               \
  GL(sV + 1024 + vq, dst + 12288); GL(sV + 5120 + vq, dst + 13312); GL(sV + 1536 + vq, dst + 14336); \
  GL(sV + 5632 + vq, dst + 15360)
  // first byte of the rows of the quad's i-th branch (of the page that holds the chunk) in both
  // pools, and its last position in memory
  auto tile_branch_rows = [&](int32_t tc, int32_t tq, int32_t i, int64_t& rowb, int32_t& last) {
    const bool paged = PAGED || (PAPER && a.tb.tail_pages);
    int32_t b;
    last = a.step;
    if (PAPER) {
      // key branches are consecutive ids from the prompt's first; a finished branch stops at
      // its own length, the rows behind it were never written
      b = pb0 + min(tq * 4 + i, kb_end - 1);
      last = min(a.step, scalar_load(a.tb.branch_len + b) - 1);
    } else {
      const int32_t lb = min(tq * 4 + i, nbr_here - 1);
      b = ub0 >= 0 ? ub0 + br0 + lb : scalar_load(a.tb.live_branch + (a.live_base + row0_live + br0) + lb);
    }
    if (paged) {
      // a page holds a multiple of 8 steps, so the 8 positions of the tile (clamped to the
      // newest row of the branch, which lies in or behind them) share one page per branch
      int32_t pg = scalar_load(a.tb.tail_pages + (int64_t)b * a.tb.pages_per_branch +
                               (min(tc * 8, last) >> a.tb.page_shift));
      pg = min(max(pg, 0), a.tb.n_pages - 1);
      rowb = ((((int64_t)pg * a.Hkv + hk)) << a.tb.page_shift) * (D * 2);
    } else {
      rowb = ((int64_t)b * a.Hkv + hk) * a.Tcap * (D * 2);
    }
  };
  auto issue_block = [&](int32_t gb_raw, uint4* dst_slot) {
    // a slot past the last block re-loads the last block (never read): the count stays fixed
    const int32_t gb = min(gb_raw, NBT - 1);
    char* const dst = reinterpret_cast<char*>(dst_slot);
    if (gb < NB) {
      int32_t slot0;
      if (PAPER) slot0 = gb < NBh ? hoff + gb * 32 : scalar_load(a.tb.pblk + 2 * (doff + gb - NBh));
      else if (PLIST) slot0 = gb < NBh ? scalar_load(a.tb.fblk + 2 * (hoff + gb)) : doff + (gb - NBh) * 32;
      else slot0 = gb < NBh ? hoff + gb * 32 : doff + (gb - NBh) * 32;
      const char* const sK = kpool + (int64_t)slot0 * (D * 2);
      const char* const sV = vpool + (int64_t)slot0 * (D * 2);
      // Document blocks - unless several row groups stream the same prefix - are read once per
      // launch: ask the caches not to keep them (measured: 4-5 % on the memory-bound
      // configurations).  The header is shared by the documents of its prompt and stays cacheable.
      if (a.RG == 1 && gb >= NBh) {
        HPD_PREFIX_BLOCK(HPD_GLL_NT);
      } else {
        HPD_PREFIX_BLOCK(HPD_GLL);
      }
      return;
    }
    const int32_t tt = gb - NB;
    if (FMT && tt >= n_full_tiles) {
      // a tile of the newest chunk in the format fmt_lg: row k = h*16 + f*4 + lane/16 of the
      // slot is position k % NPOS of the tile's branch k / NPOS, a per-lane address from the
      // table in LDS (the same row of the K and of the V pool).  Branches and positions past
      // the end repeat the last valid one.
      const int32_t tb0 = (tt - n_full_tiles) << (5 - fmt_lg);
      const int32_t pmask = (1 << fmt_lg) - 1, last = newest - 1;
#pragma nounroll
      for (int32_t half = 0; half < 2; ++half) {
        char* const dk = dst + half * 4096;
#pragma unroll
        for (int f = 0; f < 4; ++f) {
          const int32_t k = half * 16 + f * 4 + r4;
          const int32_t j = min(tb0 + (k >> fmt_lg), nbr_here - 1);
          const int64_t row = (chunk_row[j] + min(k & pmask, last)) * (D * 2);
          HPD_GLL_NT(ktb + row + ck[f], dk + f * 1024);
          HPD_GLL_NT(vtb + row + cv, dk + 8192 + f * 1024);
        }
      }
      return;
    }
    // tail tile: key k = position c*8 + k%8 of branch qd*4 + k/8; row k = h*16 + f*4 + lane/16
    // is position (f&1)*4 + lane/16 of branch 2*h + f/2.  Branches and positions past the end
    // repeat the last valid one (masked by the consumer).  The branch of a load is the same in
    // all lanes: scalar lookups, once per tile.
    const int32_t tc = tt / NQ;
    const int32_t tq = quad_of(tt - tc * NQ);
    const bool paged = PAGED || (PAPER && a.tb.tail_pages);
    const int32_t pg_mask = paged ? (1 << a.tb.page_shift) - 1 : 0x7fffffff;
    auto branch_rows = [&](int32_t i, int64_t& rowb, int32_t& last) { tile_branch_rows(tc, tq, i, rowb, last); };
#pragma nounroll
    for (int32_t half = 0; half < 2; ++half) {
      int64_t rowA, rowB;
      int32_t lastA, lastB;
      branch_rows(2 * half, rowA, lastA);
      branch_rows(2 * half + 1, rowB, lastB);
      const uint32_t pA0 = (uint32_t)((min(tc * 8 + r4, lastA) & pg_mask) << 8);
      const uint32_t pA1 = (uint32_t)((min(tc * 8 + 4 + r4, lastA) & pg_mask) << 8);
      const uint32_t pB0 = (uint32_t)((min(tc * 8 + r4, lastB) & pg_mask) << 8);
      const uint32_t pB1 = (uint32_t)((min(tc * 8 + 4 + r4, lastB) & pg_mask) << 8);
      char* const dk = dst + half * 4096;
      char* const dv = dst + 8192 + half * 4096;
      HPD_GLL_NT(ktb + rowA + (pA0 + ck[0]), dk);
      HPD_GLL_NT(ktb + rowA + (pA1 + ck[1]), dk + 1024);
      HPD_GLL_NT(ktb + rowB + (pB0 + ck[2]), dk + 2048);
      HPD_GLL_NT(ktb + rowB + (pB1 + ck[3]), dk + 3072);
      HPD_GLL_NT(vtb + rowA + (pA0 + cv), dv);
      HPD_GLL_NT(vtb + rowA + (pA1 + cv), dv + 1024);
      HPD_GLL_NT(vtb + rowB + (pB0 + cv), dv + 2048);
      HPD_GLL_NT(vtb + rowB + (pB1 + cv), dv + 3072);
    }
  };
#undef HPD_PREFIX_BLOCK
  // ---- fused mode: the compute waves append the newest token of the row group's branches (the
  //      arithmetic of hpd_kv_append), 8 lanes per branch: channels c .. c+7 and 64+c .. 64+c+7.
  //      PAPER: the rows also see the newest token of every earlier live branch of the prompt,
  //      which belongs to another row group's workgroup when there are several: every
  //      workgroup appends all live branches up to its own last (the same bytes from every
  //      writer) instead of waiting for its neighbours.
  //      `li` counts the unit's live branches.
  const int32_t ap_first = PAPER ? 0 : br0, ap_end = br0 + nbr_here;
  const int32_t ap_c = (tid & 7) * 8;
  struct NewRows { uint4 klo, khi, vlo, vhi; };
  auto append_load = [&](int32_t li) -> NewRows {
    const int64_t noff = ((int64_t)(row0_live + li) * a.Hkv + hk) * D;
    NewRows r;
    r.klo = *reinterpret_cast<const uint4*>(k_new + noff + ap_c);
    r.khi = *reinterpret_cast<const uint4*>(k_new + noff + 64 + ap_c);
    r.vlo = *reinterpret_cast<const uint4*>(v_new + noff + ap_c);
    r.vhi = *reinterpret_cast<const uint4*>(v_new + noff + 64 + ap_c);
    return r;
  };
  auto append_store = [&](int32_t li, const NewRows& r, bool use_rope_q) {
    const int32_t b = unit_branch(li);
    const int32_t pos = upos >= 0 ? upos : a.tb.branch_base_pos[b] + 1 + a.step;
    float rl[8], rh[8];
    if (use_rope_q) rotate16(r.klo, r.khi, reinterpret_cast<const float2*>(rope_q), ap_c, rl, rh);
    else rotate16(r.klo, r.khi, a.tb.rope + (int64_t)pos * (D / 2), ap_c, rl, rh);
    const int64_t trow = ((PAGED || PAPER) ? hpd_tail_row(a.tb, b, hk, a.Hkv, a.Tcap, a.step)
                                : ((int64_t)b * a.Hkv + hk) * a.Tcap + a.step) * D;
    uint16_t* kd = k_tail + trow;
    *reinterpret_cast<uint4*>(kd + ap_c) = pack8_key(rl);
    *reinterpret_cast<uint4*>(kd + 64 + ap_c) = pack8_key(rh);
    uint16_t* vd = v_tail + trow;
    *reinterpret_cast<uint4*>(vd + ap_c) = cache8(r.vlo);
    *reinterpret_cast<uint4*>(vd + 64 + ap_c) = cache8(r.vhi);
  };
  auto append_from = [&](int32_t li0) {
    for (int32_t li = li0; li < ap_end; li += CWAVES * 8) append_store(li, append_load(li), false);
  };
  // Rounds 0..3 are requested before any barrier; round x >= 4 after the barrier of round
  // x - 3.  The appending waves make sure their stores are complete before they enter the
  // barrier of round 1, so a prefix of at least 8 blocks keeps every tail tile behind it;
  // with a shorter prefix the append is completed before anything is loaded.
  const bool append_first = a.fused && NB < 4 * STAGE_BLOCKS;
  const int32_t r_pub = (a.fused && !append_first) ? 1 : -1;
  // The table of the newest chunk's rows is written by the compute waves before the first of
  // the two barriers of the query staging; the loaders request rounds 0 and 1 before that
  // barrier.  If a tile of the newest chunk can be among them the table is written first.
  auto fill_chunk_rows = [&]() {
    if constexpr (FMT) {
      for (int32_t j = tid; j < nbr_here; j += CWAVES * 64)
        chunk_row[j] = hpd_tail_row(a.tb, branch_id(j), hk, a.Hkv, a.Tcap, (NC - 1) * 8);
    }
  };
  const bool table_first = use_fmt && NB + n_full_tiles < 2 * STAGE_BLOCKS;
  // ---- the dense shape (prefill: prefix blocks only): wave w issues quarter w % 4 of block
  //      w / 4 of a stage - the same loads as a loader's (quarters 0, 1: the K rows 0..15,
  //      16..31; quarters 2, 3: the V half), 4 per wave and stage
  auto issue_quarter = [&](int32_t pos, uint4* dst_slot, int32_t qt) {
    static_assert(!SELF || PREFILL, "the compute waves load prefix blocks only");
    const int32_t gb = min(pos, NBT - 1);
    char* const dst = reinterpret_cast<char*>(dst_slot);
    const int32_t half = qt & 1;
    int32_t slot0;
    if (PLIST) slot0 = gb < NBh ? scalar_load(a.tb.fblk + 2 * (hoff + gb)) : doff + (gb - NBh) * 32;
    else slot0 = gb < NBh ? hoff + gb * 32 : doff + (gb - NBh) * 32;
    if (qt < 2) {
      const char* const sK = kpool + (int64_t)slot0 * (D * 2) + half * 4096;
      char* const dk = dst + half * 4096;
      dma16(sK + kq[0], dk); dma16(sK + kq[1], dk + 1024); dma16(sK + kq[2], dk + 2048); dma16(sK + kq[3], dk + 3072);
    } else {
      const char* const sV = vpool + (int64_t)slot0 * (D * 2) + half * 1024;
      char* const dv = dst + 8192 + half * 4096;
      dma16(sV + vq, dv); dma16(sV + 4096 + vq, dv + 1024); dma16(sV + 512 + vq, dv + 2048); dma16(sV + 4608 + vq, dv + 3072);
    }
  };
  if (append_first || table_first) {
    if (!loader) {
      if (append_first) append_from(ap_first + (tid >> 3));
      if (table_first) fill_chunk_rows();
    }
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    __syncthreads();
  }

  // =====================================================================================
  // Loader waves: request round after round; meet the compute waves at every barrier
  // =====================================================================================
  if (loader) {
    auto issue_round = [&](int32_t r) {
      const int32_t x = r & 3;  // stage of round r
      uint4* stage = x == 0 ? ring0 : (x == 1 ? ring1 : (x == 2 ? ring2 : ring3));
      for (int32_t j = wave - CWAVES; j < STAGE_BLOCKS; j += LOADERS)
        issue_block(r * STAGE_BLOCKS + j, stage + j * SLOT_U4);
    };
    // half the ring; the two barriers of the query staging, which borrows stages 2 and 3 (and
    // the compute waves must not wait there for a loader that is stuck in the queue); the
    // other half
    int32_t issued = 0;
    for (; issued < min(NR, 2); ++issued) issue_round(issued);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_s_barrier();
    for (; issued < min(NR, 4); ++issued) issue_round(issued);
    for (int32_t s0 = 0; s0 < NR;) {
      // wait until the stages of the round have landed: the DMA instructions of a wave complete
      // in order, every stage is LOADS_PER_ROUND of them, and the newer ones may stay in flight
      const int32_t s1 = round_end(s0);
      const int32_t newer = issued - s1;
      if (newer >= 3) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(3 * LOADS_PER_ROUND) : "memory");
      else if (newer == 2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * LOADS_PER_ROUND) : "memory");
      else if (newer == 1) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LOADS_PER_ROUND) : "memory");
      else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __builtin_amdgcn_s_barrier();  // the round is published; the stages before s0 are free
      for (; issued < min(NR, s0 + 4); ++issued) issue_round(issued);
      s0 = s1;
    }
    __syncthreads();              // end of the stream
    if (KG > 1) __syncthreads();  // the exchange of the key groups
    return;
  }

  // =====================================================================================
  // Compute waves
  // =====================================================================================

  // ---- the loaders fill the ring.  The compute waves - whose memory queues stay short, so that
  //      their loads come back with one latency - fetch the raw query rows of the row group, 4
  //      whole rows per instruction, and exchange them through stages 2 and 3 (which the
  //      loaders leave alone until the second barrier): chunk c of row r at position
  //      c ^ (r & 15).  One wave fetches the (cos, sin) row of the shared position.  The new
  //      rows of the append are requested in the same breath.
  // (dense shape: the waves request their quarters of rounds 0 and 1 first, of rounds 2 and 3
  // when the query staging has given stages 2 and 3 back, and of round r + 3 behind the barrier
  // of round r; before that barrier a wave waits for its own loads of round r.  The shape serves
  // the prefill only: nothing is appended, so loads are the only vector memory operations a wave
  // has in flight during the rounds and their count says which have landed.)
  int32_t issued = 0;
  auto issue_upto = [&](int32_t lim) {
    if constexpr (SELF) {
      for (; issued < min(NR, lim); ++issued) {
        const int32_t x = issued & 3;
        uint4* stage = x == 0 ? ring0 : (x == 1 ? ring1 : (x == 2 ? ring2 : ring3));
        issue_quarter(issued * STAGE_BLOCKS + (wave >> 2), stage + (wave >> 2) * SLOT_U4, wave & 3);
      }
    }
  };
  auto own_loads_landed = [&](int32_t s1) {  // of the stages before s1
    if constexpr (SELF) {
      const int32_t newer = issued - s1;
      if (newer >= 3) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(3 * LOADS_PER_ROUND) : "memory");
      else if (newer == 2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * LOADS_PER_ROUND) : "memory");
      else if (newer == 1) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LOADS_PER_ROUND) : "memory");
      else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
  };
  issue_upto(2);
  const bool append_late = a.fused && !append_first;
  const bool append_mine = append_late && ap_first + (tid >> 3) < ap_end;
  NewRows new_rows = {};
  uint4 qv[8];  // instruction i = wave + CWAVES * b covers rows 4 i .. 4 i + 3 (32 * CWAVES rows at most)
#pragma unroll
  for (int b = 0; b < 8; ++b) {
    qv[b] = make_uint4(0, 0, 0, 0);
    const int32_t i = wave + b * CWAVES;
    const int32_t urow = first_blk * 32 + min(i * 4 + r4, rows_here - 1);  // row within the unit
    const int64_t off = ((int64_t)(row0_live + urow / G) * a.Hq + hk * a.Gr + urow % G) * D;
    if (i * 4 < rows_here && urow % G < a.Gr) qv[b] = *reinterpret_cast<const uint4*>(q + off + (c16 << 3));
  }
  if (append_mine) new_rows = append_load(ap_first + (tid >> 3));
  float4 rope_v = make_float4(0.f, 0.f, 0.f, 0.f);
  if (upos >= 0 && wave == 0 && lane < 32)
    rope_v = reinterpret_cast<const float4*>(a.tb.rope + (int64_t)upos * (D / 2))[lane];
#pragma unroll
  for (int b = 0; b < 8; ++b) {
    const int32_t i = wave + b * CWAVES;
    const int32_t row = i * 4 + r4;
    if (i * 4 < rows_here)
      (row < STAGE_ROWS ? ring2 : ring3)[(row % STAGE_ROWS) * 16 + (c16 ^ (row & 15))] = qv[b];
  }
  if (upos >= 0 && wave == 0 && lane < 32) rope_q[lane] = rope_v;
  if (use_fmt && !table_first) fill_chunk_rows();
  if constexpr (PAPER) {
    // tokens in memory of every key branch: min(step + 1, its length)
    for (int32_t i = tid; i < kb_end; i += CWAVES * 64) klen[i] = min(a.step + 1, a.tb.branch_len[pb0 + i]);
    // the block list's key counts: a lookup in global memory per block would stall every wave
    for (int32_t i = tid; i < NBd; i += CWAVES * 64) bvalid[i] = a.tb.pblk[2 * (doff + i) + 1];
  }
  if constexpr (PLIST) {
    for (int32_t i = tid; i < NBh; i += CWAVES * 64) bvalid[i] = a.tb.fblk[2 * (hoff + i) + 1];
  }
  __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): the rows are in LDS
  __builtin_amdgcn_s_barrier();        // bare barriers: __syncthreads() would wait for every store
  uint4 qraw[8];
  {
    const uint4* qrow = (lr < STAGE_ROWS ? ring2 : ring3) + (lr % STAGE_ROWS) * 16;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      qraw[kk] = make_uint4(0, 0, 0, 0);
      if (row_valid) qraw[kk] = qrow[(kk * 2 + g2) ^ (lr & 15)];
    }
  }
  __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): this wave has its rows
  __builtin_amdgcn_s_barrier();        // stages 2 and 3 go back to the loaders
  issue_upto(4);

  // ---- rotate the query: MFMA B operands in half precision (11 significant bits; the keys of
  //      the cache hold bf16 values in half format, so one pass of the f16 matrix instruction
  //      gives the score).  The softmax scale and the change to base 2 ride on the query:
  //      scores come out of the MFMA ready for exp2.
  f16x8 Qf[8];
  auto rotate_query = [&](auto cos_sin) {
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      float lo[8], hi[8], rl[8], rh[8];
      unpack8(qraw[kk], lo);
      unpack8(qraw[kk + 4], hi);
#pragma unroll
      for (int e2 = 0; e2 < 4; ++e2) {
        const float4 cs = cos_sin(kk * 8 + g2 * 4 + e2);  // pairs kk*16 + g2*8 + 2*e2, +1
        hpd::rope_pair(lo[2 * e2], hi[2 * e2], cs.x, cs.y, rl[2 * e2], rh[2 * e2]);
        hpd::rope_pair(lo[2 * e2 + 1], hi[2 * e2 + 1], cs.z, cs.w, rl[2 * e2 + 1], rh[2 * e2 + 1]);
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) { rl[e] *= a.scale_log2; rh[e] *= a.scale_log2; }
      Qf[kk] = pack8_half(rl);
      Qf[kk + 4] = pack8_half(rh);
    }
  };
  if (upos >= 0) {
    rotate_query([&](int i4) -> float4 { return rope_q[i4]; });
  } else {
    // per-branch positions: straight from the table
    const int32_t q_bi = min(r_row / G, nb - 1);
    const int32_t q_pos = PREFILL ? ((!PLIST || seg_pos0 >= 0) ? seg_pos0 + q_bi : a.tb.skel_pos[q_bi - seg_pos0 - 1])
                                  : a.tb.branch_base_pos[branch_id(q_bi - br0)] + 1 + a.step;
    const float4* cs_row = reinterpret_cast<const float4*>(a.tb.rope + (int64_t)q_pos * (D / 2));
    rotate_query([&](int i4) -> float4 { return cs_row[i4]; });
  }

  // ---- the append, after the rotation (the rotation is what the first round waits for): the
  //      stores complete during round 0 and are published at the barrier of round 1
  if (append_late) {
    if (append_mine) append_store(ap_first + (tid >> 3), new_rows, upos >= 0);
    append_from(ap_first + (tid >> 3) + CWAVES * 8);
  }

  // ---- online-softmax state: (max, this lane's share of the sum, O^T accumulators)
  float m_used = NEG_BIG;  // reference point of the row's exponentials (log2 units), equal in lanes n and n+32
  float l_lane = 0.f;
  floatx16 acc[4];
#pragma unroll
  for (int blk = 0; blk < 4; ++blk)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[blk][i] = 0.f;

  // One block for this wave's 32 rows.  Score value i of lane (n, g2) belongs to key
  // (i>>3)*16 + g2*8 + (i&7); bit i of `ok` says whether the row may see it (`masked` is
  // wave-uniform: false means all 32 keys count for every row).
  auto compute_block = [&](const uint4* slot, bool masked, uint32_t ok, bool tail) {
    const uint4* fr = slot + lane;
    const char* krows = reinterpret_cast<const char*>(slot) + krow * 256;
    floatx16 S;
#pragma unroll
    for (int i = 0; i < 16; ++i) S[i] = 0.f;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      const f16x8 kf = __builtin_bit_cast(
          f16x8, *reinterpret_cast<const uint4*>(krows + (((kk * 2 + g2) ^ (krow & 15)) << 4)));
      S = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf, Qf[kk], S, 0, 0, 0);
    }
    uint4 vf[8];
    if (!tail) {
#pragma unroll
      for (int f = 0; f < 8; ++f) vf[f] = fr[(8 + f) * 64];
    } else {
      // V half of a tail tile: row k at 256 * k bytes, 16-byte chunk c at position c ^ 2*(k & 3).
      // Fragment f = d-block * 2 + key half wants keys half*16 + g2*8 + 0..7 of channel
      // d-block*32 + n, a column of the tile: two transposing 8-byte reads.  In such a read each
      // 16 lanes form a 4 x 4 arrangement, lane 4*j + r of them addresses 4 channels (quad r of
      // the group's 16) of key j, and lane i receives channel i of keys 0..3.
      const char* vrows = reinterpret_cast<const char*>(slot + 8 * 64);
      const int tj = (lane >> 2) & 3, tr = lane & 3;
      const int tx = ((lane >> 4) & 1) * 2 + (tr >> 1);  // chunk inside the d-block's four
      const char* vlane = vrows + (g2 * 8 + tj) * 256 + (tr & 1) * 8;
#pragma unroll
      for (int f = 0; f < 8; ++f) {
        const int chunk = ((f >> 1) * 4 + tx) ^ (2 * tj);
        const char* p = vlane + (f & 1) * 4096 + chunk * 16;
        const uint2 k03 = lds_read_tr16(p), k47 = lds_read_tr16(p + 4 * 256);
        vf[f] = make_uint4(k03.x, k03.y, k47.x, k47.y);
      }
    }
    float s[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) s[i] = S[i];
    if (masked) {
#pragma unroll
      for (int i = 0; i < 16; ++i) s[i] = (ok >> i) & 1 ? s[i] : -INFINITY;
    }
    float bm = NEG_BIG;
#pragma unroll
    for (int i = 0; i < 16; ++i) bm = fmaxf(bm, s[i]);
    // The reference point of the exponentials follows the maximum of a row within 2^8: it
    // moves (and the 64 accumulator values are rescaled) only when a score exceeds it by more,
    // which after the first blocks of a row is rare.  The weights go into the value product as
    // halves - 11 significant bits whatever their size, up to 2^8 - so the largest weight of a
    // row need not be exactly 1 to be exact enough.
    if (__any(bm > m_used + MAX_SLACK)) {
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
    for (int i = 0; i < 16; ++i) s[i] = fast_exp2(s[i] - m_used);
    const f16x8 P0 = pack8_half(s), P1 = pack8_half(s + 8);
    // the sum of the weights as the value product sees them (rounded to half): numerator and
    // denominator of a row carry the same rounding
    {
      const uint4 w0 = __builtin_bit_cast(uint4, P0), w1 = __builtin_bit_cast(uint4, P1);
      float la = sum_half_pair(w0.x, l_lane), lb = sum_half_pair(w1.x, 0.f);
      la = sum_half_pair(w0.y, la); lb = sum_half_pair(w1.y, lb);
      la = sum_half_pair(w0.z, la); lb = sum_half_pair(w1.z, lb);
      la = sum_half_pair(w0.w, la); lb = sum_half_pair(w1.w, lb);
      l_lane = la + lb;
    }
#pragma unroll
    for (int blk = 0; blk < 4; ++blk) {
      acc[blk] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, vf[blk * 2]), P0,
                                                        acc[blk], 0, 0, 0);
      acc[blk] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, vf[blk * 2 + 1]), P1,
                                                        acc[blk], 0, 0, 0);
    }
  };

  // bits 0..7 of a mask byte: the first `cnt` (clamped to 0..8) of 8 consecutive keys
  auto first_bits = [](int32_t cnt) -> uint32_t { return (1u << min(max(cnt, 0), 8)) - 1u; };
  const int32_t lb_row = rb * BPB + n / G;  // this row's branch within the row group
  // PAPER: the branch of this row and of the last row of the row block, counted from the
  // prompt's first branch like the key branches
  // ... and the attribute-name tokens they see (names up to the own branch's)
  int32_t kb_row = 0, kb_row_max = 0, names_row = 0, names_max = 0;
  if constexpr (PAPER) {
    if (active) {
      kb_row = branch_id(min(lb_row, nbr_here - 1)) - pb0;
      kb_row_max = __builtin_amdgcn_readfirstlane(branch_id(min(rb * BPB + BPB - 1, nbr_here - 1))) - pb0;
      names_row = a.tb.skel_cum[pb0 + kb_row];
      names_max = __builtin_amdgcn_readfirstlane(a.tb.skel_cum[pb0 + kb_row_max]);
    }
  }

  // Prefix rounds (one stage each) under the block mask, with as little scalar work per block
  // as possible: every scalar instruction of a compute wave is issue time the wave does not
  // spend on its matrix and vector work (measured on the 70B-like configuration: 112 scalar
  // against 168 vector instructions per block before this loop was split off).  Blocks are
  // full except the last of the header and the last of the document; the key group of a
  // block is counted along instead of divided out.
  int32_t s_first = 0;
  if constexpr (MODE == MODE_BLOCK || MODE == MODE_PAGED) {
    int32_t ph = 0;  // (block index) % KG
    const int32_t gb_h_part = (Hlen & 31) ? NBh - 1 : -1, gb_d_part = (Llen & 31) ? NB - 1 : -1;
    for (int32_t s0 = 0; s0 < s_tail; ++s0) {
      if (s0 == r_pub) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the stores of the append are complete
      own_loads_landed(s0 + 1);
      __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): LDS reads of the previous round are done
      __builtin_amdgcn_s_barrier();
      issue_upto(s0 + 4);
      const int32_t st = s0 & 3;
      const uint4* stage = st == 0 ? ring0 : (st == 1 ? ring1 : (st == 2 ? ring2 : ring3));
#pragma nounroll
      for (int32_t j = 0; j < STAGE_BLOCKS; ++j) {
        const int32_t gb = s0 * STAGE_BLOCKS + j;
        const bool mine = active && ph == kg;
        ph = ph + 1 == KG ? 0 : ph + 1;
        const bool masked = gb == gb_h_part || gb == gb_d_part;
        uint32_t ok = 0xffffu;
        if (masked) {
          const int32_t valid = gb == gb_h_part ? (Hlen & 31) : (Llen & 31);
          ok = first_bits(valid - g2 * 8) | (first_bits(valid - 16 - g2 * 8) << 8);
        }
        if (mine) compute_block(stage + j * SLOT_U4, masked, ok, false);
      }
    }
    s_first = s_tail;
  }
  // Round r: meet the loaders (the stage has landed), compute.
  for (int32_t s0 = s_first; s0 < NR;) {
    const int32_t s1 = round_end(s0);
    if (s0 == r_pub) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the stores of the append are complete
    own_loads_landed(s1);
    __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): LDS reads of the previous round are done
    __builtin_amdgcn_s_barrier();
    issue_upto(s0 + 4);
    if (active) {
#pragma nounroll
      for (int32_t gb = s0 * STAGE_BLOCKS; gb < min(s1 * STAGE_BLOCKS, NBT); ++gb) {
        const int32_t st = (gb / STAGE_BLOCKS) & 3;  // no DMA on this path: any stage may be addressed
        const uint4* cur = (st == 0 ? ring0 : (st == 1 ? ring1 : (st == 2 ? ring2 : ring3))) +
                           (gb % STAGE_BLOCKS) * SLOT_U4;
        bool mine = false, masked = false, tail = false;
        uint32_t ok = 0xffffu;
        if (gb < NB) {
          mine = gb % KG == kg;
          int32_t valid = gb < NBh ? (PLIST ? bvalid[gb] : min(32, Hlen - gb * 32))
                          : PAPER ? bvalid[gb - NBh] : min(32, Llen - (gb - NBh) * 32);
          masked = valid < 32;
          if (PAPER && valid >= 1000) {
            // a block of attribute names: the row keeps the names up to its own branch's
            const int32_t k0 = valid - 1000;  // first name token of the block
            mine = mine && k0 < names_max;
            masked = true;
            valid = names_row - k0;
          }
          if (PREFILL && gb >= NBh) {
            // causal inside the segment: the row of token x keeps keys 0 .. x.  Blocks behind
            // the last token of the row block are not this wave's; blocks that end before its
            // first token need no mask.
            const int32_t k0 = (gb - NBh) * 32;  // first key of the block
            const int32_t tok_first = br0 + rb * BPB, tok_last = min(tok_first + BPB, br0 + nbr_here) - 1;
            mine = mine && k0 <= tok_last;
            masked = masked || k0 + 31 > tok_first;
            valid = min(valid, br0 + min(lb_row, nbr_here - 1) - k0 + 1);
          }
          ok = first_bits(valid - g2 * 8) | (first_bits(valid - 16 - g2 * 8) << 8);
        } else {
          const int32_t tt = gb - NB;
          masked = true;
          tail = true;
          if (FMT && tt >= n_full_tiles) {
            // a tile of the newest chunk: positions 0 .. newest-1 of the branches tb0 .. of the
            // row group, NPOS keys apart; every row block that holds one of them works on it
            const int32_t li = tt - n_full_tiles;
            const int32_t tb0 = li << (5 - fmt_lg);
            mine = rb * BPB < tb0 + (32 >> fmt_lg) && (rb + 1) * BPB > tb0 && li % KG == kg;
            const int32_t k0 = (lb_row - tb0) << fmt_lg;  // this row's first key in the tile
            const int32_t lo = k0 - g2 * 8, hi = lo + newest;
            ok = (k0 >= 0 && k0 < 32) ? ((first_bits(hi) & ~first_bits(lo)) |
                                         ((first_bits(hi - 16) & ~first_bits(lo - 16)) << 8)) : 0u;
          } else if constexpr (PAPER) {
            const int32_t c = tt / NQ, qd = quad_of(tt - c * NQ);
            // every row block that holds a branch not earlier than the quad's first works on
            // the tile; a row keeps the tokens in memory of the branches up to its own
            mine = qd * 4 <= kb_row_max && (c + qd) % KG == kg;
            const int32_t kA = qd * 4 + g2, kB = kA + 2;
            const int32_t cntA = kA < kb_end ? klen[kA] : 0, cntB = kB < kb_end ? klen[kB] : 0;
            ok = (kA <= kb_row ? first_bits(cntA - c * 8) : 0u) | (kB <= kb_row ? first_bits(cntB - c * 8) << 8 : 0u);
          } else {
            const int32_t c = tt / NQ, qd = quad_of(tt - c * NQ);
            mine = qd / QPR == rb && (c * QPR + qd % QPR) % KG == kg;
            const uint32_t pm = first_bits(a.step + 1 - c * 8);
            ok = (qd * 4 + g2 == lb_row ? pm : 0u) | (qd * 4 + 2 + g2 == lb_row ? pm << 8 : 0u);
          }
        }
        if (mine) compute_block(cur, masked, ok, tail);
      }
    }
    s0 = s1;
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();  // all stages are dead from here on and get reused

  // ---- merge the key groups: every wave of a row block reduces its own d-blocks.
  //      Wave w parks what the others need in region w: stage (w & 3), half (w >> 2).
  // d-block blk is reduced by key group blk % KG (KG = 3: group 0 takes blocks 0 and 3)
  auto owner = [&](int blk) -> int32_t { return blk >= KG ? blk - KG : blk; };
  if (KG > 1) {
    float* const park0 = reinterpret_cast<float*>(ring0);
    float* const park1 = reinterpret_cast<float*>(ring1);
    float* const park2 = reinterpret_cast<float*>(ring2);
    float* const park3 = reinterpret_cast<float*>(ring3);
    static_assert(STAGE_U4 * 16 >= (CWAVES > 4 ? 2 : 1) * 50 * 64 * 4, "a stage holds the regions of its waves");
    auto region = [&](int32_t w) -> float* {
      float* base = (w & 2) ? ((w & 1) ? park3 : park2) : ((w & 1) ? park1 : park0);
      return base + (w >> 2) * (50 * 64) + lane;
    };
    if (active) {
      float* buf = region(wave);
      int32_t sidx = 0;
#pragma unroll
      for (int blk = 0; blk < 4; ++blk) {
        if (owner(blk) != kg) {  // not mine: somebody else reduces it
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
        const float* buf = region(okg * NRB + rb);
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
        const float* buf = region(okg * NRB + rb);
        const float a_o = fast_exp2(m_o[o] - m_new);
        l_lane += l_o[o] * a_o;
        // my blocks sit in the other wave's region at the index that skips ITS own blocks
        int32_t skipped = 0;  // blocks below blk that the other wave owns
#pragma unroll
        for (int blk = 0; blk < 4; ++blk) {
          if (owner(blk) == kg) {
            const int32_t sidx = blk - skipped;
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[blk][i] += buf[(sidx * 16 + i) * 64] * a_o;
          }
          if (owner(blk) == okg) ++skipped;
        }
      }
    }
  }

  // ---- normalise and write.  Accumulator value i of d-block blk is channel
  //      blk*32 + (i/4)*8 + g2*4 + i%4 of row n.
  const float inv = 1.0f / (l_lane + __shfl_xor(l_lane, 32));
  if (KG == 1 && active) {
    // The wave holds whole rows.  Stored from the accumulator layout every instruction would
    // touch 32 rows in pieces of 8 or 16 bytes; instead the wave turns its rows through a private
    // 16 KB of the (now dead) ring - 16-byte chunk c of row r at position c ^ r resp.
    // c ^ (r & 15) - and stores runs of whole rows, consecutive lanes = consecutive chunks, past
    // the L2 (nobody reads them here, and write-backs of dirty lines compete with the next
    // workgroup's stream).  Measured: 4 % on the 96-row units of the multi-document
    // configuration; without the streaming hint there is no gain, and the hint on the
    // piecewise stores costs 15 %.
    constexpr int WPS = STAGE_U4 / 1024;  // waves per stage
    static_assert(WPS >= 1 && 4 * WPS >= CWAVES, "the ring holds 16 KB per compute wave");
    const int32_t st = wave / WPS;
    uint4* mine = (st == 0 ? ring0 : (st == 1 ? ring1 : (st == 2 ? ring2 : ring3))) + (wave % WPS) * 1024;
    typedef uint32_t u4v __attribute__((ext_vector_type(4)));
    if (a.out_f32) {
      float4* rowp = reinterpret_cast<float4*>(mine) + n * 32;  // 32 chunks of 4 floats per row
#pragma unroll
      for (int blk = 0; blk < 4; ++blk)
#pragma unroll
        for (int cc = 0; cc < 4; ++cc)
          rowp[(blk * 8 + cc * 2 + g2) ^ n] =
              make_float4(acc[blk][cc * 4 + 0] * inv, acc[blk][cc * 4 + 1] * inv,
                          acc[blk][cc * 4 + 2] * inv, acc[blk][cc * 4 + 3] * inv);
      __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0)
      __builtin_amdgcn_wave_barrier();
#pragma unroll 4
      for (int32_t i = 0; i < 16; ++i) {  // 2 rows per instruction
        const int32_t row = i * 2 + (lane >> 5), chunk = lane & 31;
        const int32_t lrr = rb * 32 + row;
        if (lrr < rows_here && lrr % G < a.Gr) {
          const uint4 v = mine[row * 32 + (chunk ^ row)];
          const int64_t off = ((int64_t)(row0_live + br0 + lrr / G) * a.Hq + hk * a.Gr + lrr % G) * D + chunk * 4;
          u4v vv = {v.x, v.y, v.z, v.w};
          __builtin_nontemporal_store(vv, reinterpret_cast<u4v*>(reinterpret_cast<float*>(out) + off));
        }
      }
    } else {
      uint2* rowp = reinterpret_cast<uint2*>(mine) + n * 32;  // 16 chunks of 8 bf16 per row, in halves
#pragma unroll
      for (int blk = 0; blk < 4; ++blk)
#pragma unroll
        for (int cc = 0; cc < 4; ++cc)
          rowp[(((blk * 4 + cc) ^ (n & 15)) << 1) | g2] =
              make_uint2(cvt_pk_bf16(acc[blk][cc * 4 + 0] * inv, acc[blk][cc * 4 + 1] * inv),
                         cvt_pk_bf16(acc[blk][cc * 4 + 2] * inv, acc[blk][cc * 4 + 3] * inv));
      __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0)
      __builtin_amdgcn_wave_barrier();
#pragma unroll 4
      for (int32_t i = 0; i < 8; ++i) {  // 4 rows per instruction
        const int32_t row = i * 4 + (lane >> 4), chunk = lane & 15;
        const int32_t lrr = rb * 32 + row;
        if (lrr < rows_here && lrr % G < a.Gr) {
          const uint4 v = mine[row * 16 + (chunk ^ (row & 15))];
          const int64_t off = ((int64_t)(row0_live + br0 + lrr / G) * a.Hq + hk * a.Gr + lrr % G) * D + chunk * 8;
          u4v vv = {v.x, v.y, v.z, v.w};
          __builtin_nontemporal_store(vv, reinterpret_cast<u4v*>(reinterpret_cast<uint16_t*>(out) + off));
        }
      }
    }
  } else if (row_valid && lr % G < a.Gr) {
    // key groups: a wave owns some d-blocks of its rows; a lane stores 4 consecutive channels at a time
    const int32_t live_row = row0_live + br0 + lr / G;
    const int64_t o_off = ((int64_t)live_row * a.Hq + hk * a.Gr + lr % G) * D + g2 * 4;
#pragma unroll
    for (int blk = 0; blk < 4; ++blk) {
      if (owner(blk) == kg) {
#pragma unroll
        for (int cc = 0; cc < 4; ++cc) {
          const float o0 = acc[blk][cc * 4 + 0] * inv, o1 = acc[blk][cc * 4 + 1] * inv;
          const float o2 = acc[blk][cc * 4 + 2] * inv, o3 = acc[blk][cc * 4 + 3] * inv;
          const int64_t off = o_off + blk * 32 + cc * 8;
          if (a.out_f32) {
            *reinterpret_cast<float4*>(reinterpret_cast<float*>(out) + off) = make_float4(o0, o1, o2, o3);
          } else {
            *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(out) + off) =
                make_uint2(cvt_pk_bf16(o0, o1), cvt_pk_bf16(o2, o3));
          }
        }
      }
    }
  }
}

template <int G, typename SH, int MODE>
hipError_t launch_g(const StreamArgs& a, int64_t items, const void* q, const void* k_prefix,
                    const void* v_prefix, void* k_tail, void* v_tail, const void* k_new,
                    const void* v_new, void* out, hipStream_t s) {
  attn_stream_kernel<G, SH, MODE><<<dim3((unsigned)items), SH::WAVES * 64, 0, s>>>(
      a, (const uint16_t*)q, (const uint16_t*)k_prefix, (const uint16_t*)v_prefix, (uint16_t*)k_tail,
      (uint16_t*)v_tail, (const uint16_t*)k_new, (const uint16_t*)v_new, out);
  return hipGetLastError();
}

}  // namespace

bool hpd_stream_supported(const hpd_layout* L) {
  const int G = L->cfg.n_q_heads / L->cfg.n_kv_heads;
  // the literal mask keeps one counter per branch and per 32-key block of a prompt in LDS
  if (L->cfg.mask_mode == HPD_MASK_PAPER) {
    if (L->max_prompt_branches > 256) return false;
    for (int32_t p = 0; p < L->P; ++p)
      if (L->pblk_ptr[p + 1] - L->pblk_ptr[p] > 512) return false;
  }
  return L->cfg.dtype == HPD_BF16 && L->cfg.head_dim == D && G >= 1 && G <= 8;
}

hipError_t hpd_launch_attention_stream(const hpd_layout* L, int32_t step, const void* q,
                                       const void* k_prefix, const void* v_prefix, void* k_tail,
                                       void* v_tail, const void* k_new, const void* v_new, void* out,
                                       hipStream_t s, bool dynamic) {
  StreamArgs a;
  a.tb = L->dev;
  a.step = step; a.Hq = L->cfg.n_q_heads; a.Hkv = L->cfg.n_kv_heads;
  a.Gr = a.Hq / a.Hkv;
  const int G = a.Gr <= 2 ? a.Gr : a.Gr <= 4 ? 4 : 8;  // the kernel's rows per branch
  a.Tcap = L->T; a.NP = L->NP;
  a.out_f32 = L->cfg.out_dtype == HPD_OUT_F32 ? 1 : 0;
  a.fused = (k_new != nullptr) ? 1 : 0;
  a.live_base = L->live_ptr[step];
  a.scale_log2 = (float)(1.4426950408889634 / std::sqrt((double)D));
  const bool paper = L->cfg.mask_mode == HPD_MASK_PAPER;
  a.tb.unit_desc = L->dev.unit_desc + (int64_t)L->unit_ptr[step] * 8;
  if (paper) a.tb.punit_desc = L->dev.punit_desc + (int64_t)L->punit_ptr[step] * 16;
  int64_t n_units = paper ? L->punit_ptr[step + 1] - L->punit_ptr[step] : L->unit_ptr[step + 1] - L->unit_ptr[step];
  int32_t max_nblk = std::max(1, ((paper ? L->pmax_rows[step] : L->max_rows[step]) * G + 31) / 32);
  if (dynamic) {
    // liveness lives on the device: a unit per document (one without live branches exits at
    // its descriptor), row groups for the most branches any document can have
    a.tb.unit_desc = L->dyn_desc;
    a.tb.live_branch = L->dyn_live;
    a.live_base = 0;
    n_units = L->n_docs;
    max_nblk = std::max(1, (L->max_doc_branches * G + 31) / 32);
    if (paper) {  // units are prompts; a finished branch stays visible as far as it got
      a.tb.punit_desc = L->dyn_desc;
      a.tb.branch_len = L->dyn_len;
      n_units = L->P;
      max_nblk = std::max(1, (L->max_prompt_branches * G + 31) / 32);
    }
  }
  // row groups per unit, and with them the number of workgroups, for the two shapes
  const int32_t rg_wide = (max_nblk + WideShape::MAX_BLOCKS - 1) / WideShape::MAX_BLOCKS;
  const int32_t rg_narrow = (max_nblk + NarrowShape::MAX_BLOCKS - 1) / NarrowShape::MAX_BLOCKS;
  const int64_t items_wide = n_units * a.Hkv * rg_wide;
  // kernel_mode 3 / 4 force a shape; otherwise the narrow shape from two workgroups per CU on,
  // unless the units have so many rows (more than two narrow row groups) that the launch is
  // bound by the matrix pipes and splitting the rows further only re-streams the prefix
  bool narrow = items_wide >= 2 * (int64_t)L->n_cus && max_nblk <= 2 * NarrowShape::MAX_BLOCKS;
  if (L->kernel_mode == 3) narrow = false;
  if (L->kernel_mode == 4) narrow = true;
  a.RG = narrow ? rg_narrow : rg_wide;
  a.n_groups = (int32_t)(n_units * a.Hkv);
  const int64_t items = ((int64_t)(a.n_groups + 7) / 8 * 8) * a.RG;
#define HPD_LAUNCH_M(GG, PP)                                                                            \
  (narrow ? launch_g<GG, NarrowShape, PP>(a, items, q, k_prefix, v_prefix, k_tail, v_tail, k_new, v_new, out, s) \
          : launch_g<GG, WideShape, PP>(a, items, q, k_prefix, v_prefix, k_tail, v_tail, k_new, v_new, out, s))
#define HPD_LAUNCH(GG)                                                   \
  (paper ? HPD_LAUNCH_M(GG, MODE_PAPER)                                  \
         : a.tb.tail_pages ? HPD_LAUNCH_M(GG, MODE_PAGED) : HPD_LAUNCH_M(GG, MODE_BLOCK))
  switch (G) {
    case 1: return HPD_LAUNCH(1);
    case 2: return HPD_LAUNCH(2);
    case 4: return HPD_LAUNCH(4);
    case 8: return HPD_LAUNCH(8);
    default: return hipErrorInvalidValue;
  }
#undef HPD_LAUNCH
#undef HPD_LAUNCH_M
}

// Attention of the prefix tokens (first inference step): one unit per header / document.
hipError_t hpd_launch_prefill_stream(const hpd_layout* L, const void* q, const void* k_prefix,
                                     const void* v_prefix, void* out, hipStream_t s) {
  StreamArgs a;
  a.tb = L->dev;
  a.step = 0; a.Hq = L->cfg.n_q_heads; a.Hkv = L->cfg.n_kv_heads;
  a.Gr = a.Hq / a.Hkv;
  const int G = a.Gr <= 2 ? a.Gr : a.Gr <= 4 ? 4 : 8;  // the kernel's rows per token
  a.Tcap = L->T; a.NP = L->NP;
  a.out_f32 = L->cfg.out_dtype == HPD_OUT_F32 ? 1 : 0;
  a.fused = 0;
  a.live_base = 0;
  a.scale_log2 = (float)(1.4426950408889634 / std::sqrt((double)D));
  const int64_t n_units = (int64_t)L->funit_desc.size() / 8;
  if (n_units == 0) return hipSuccess;
  const int32_t max_nblk = std::max(1, (L->fmax_rows * G + 31) / 32);
  // Every token is a query, so a segment has many row groups, and a row group streams only the
  // keys up to its last token: many short workgroups, whose starts and ends overlap better
  // with two workgroups per CU (the narrow shape measured 3 % to 23 % faster than the wide one
  // on the four bf16 configurations), and whose time goes into the compute waves' matrix and
  // vector work, not into memory: the dense shape (0 % to 5 % faster than the narrow one).
  // kernel_mode 3 / 4 force the wide / the narrow shape.
  const bool narrow = L->kernel_mode == 4, wide = L->kernel_mode == 3, dense = !narrow && !wide;
  const int32_t shape_blocks = narrow ? NarrowShape::MAX_BLOCKS : dense ? DenseShape::MAX_BLOCKS : WideShape::MAX_BLOCKS;
  a.RG = (max_nblk + shape_blocks - 1) / shape_blocks;
  a.n_groups = (int32_t)(n_units * a.Hkv);
  const int64_t items = ((int64_t)(a.n_groups + 7) / 8 * 8) * a.RG;
  if (items > 0x7fffffff) return hipErrorInvalidValue;
  const bool list = L->cfg.mask_mode == HPD_MASK_PAPER;
#define HPD_LAUNCH_M(GG, PP)                                                                   \
  (narrow ? launch_g<GG, NarrowShape, PP>(a, items, q, k_prefix, v_prefix, nullptr, nullptr,  \
                                          nullptr, nullptr, out, s)                           \
   : dense ? launch_g<GG, DenseShape, PP>(a, items, q, k_prefix, v_prefix, nullptr, nullptr,  \
                                          nullptr, nullptr, out, s)                           \
          : launch_g<GG, WideShape, PP>(a, items, q, k_prefix, v_prefix, nullptr, nullptr,    \
                                        nullptr, nullptr, out, s))
#define HPD_LAUNCH(GG) (list ? HPD_LAUNCH_M(GG, MODE_PREFILL_LIST) : HPD_LAUNCH_M(GG, MODE_PREFILL))
  switch (G) {
    case 1: return HPD_LAUNCH(1);
    case 2: return HPD_LAUNCH(2);
    case 4: return HPD_LAUNCH(4);
    case 8: return HPD_LAUNCH(8);
    default: return hipErrorInvalidValue;
  }
#undef HPD_LAUNCH
#undef HPD_LAUNCH_M
}
