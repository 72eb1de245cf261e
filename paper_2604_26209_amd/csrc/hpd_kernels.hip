// HIP kernels (gfx950) for HPD masked decode attention: helper kernels (prefix fill,
// positions, append, mask export) and the generic wave-reduction attention kernel that
// covers fp32, odd shapes and serves as the fallback.  The MFMA shared-prefix kernel is
// in hpd_attn_stream.hip.
#include <algorithm>
#include <mutex>

#include "hpd_internal.h"
#include "hpd_device.h"

namespace {

// ---------------------------------------------------------------------------------------
// Prefix fill: RoPE(K) at the token's position ID, store K row-major and V with 8 keys
// interleaved.  One thread per (raw token, kv head, rotation pair).
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ void prefix_fill_kernel(hpd_dev_tables tb, int32_t n_seg, int32_t P, int64_t n_tok, int32_t Hkv,
                                   int32_t D, int64_t NP, const T* __restrict__ k_raw,
                                   const T* __restrict__ v_raw, T* __restrict__ k_prefix,
                                   T* __restrict__ v_prefix) {
  const int32_t half = D / 2;
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t total = n_tok * Hkv * half;
  if (gid >= total) return;
  const int32_t i = (int32_t)(gid % half);
  const int32_t h = (int32_t)((gid / half) % Hkv);
  const int64_t tok = gid / ((int64_t)half * Hkv);
  // segment that holds raw token `tok`: last entry of the sorted start table <= tok
  int32_t lo = 0, hi = n_seg;  // invariant: start[lo] <= tok < start[hi]
  while (hi - lo > 1) {
    const int32_t mid = (lo + hi) >> 1;
    if (tb.seg_raw_off[mid] <= tok) lo = mid; else hi = mid;
  }
  // skip empty segments that share the same start
  while (lo + 1 < n_seg && tb.seg_raw_off[lo + 1] <= tok) ++lo;
  const int32_t sid = tb.raw_seg[lo];
  const int32_t idx = (int32_t)(tok - tb.seg_raw_off[lo]);
  // (a skeleton segment - the last P of the segments, where there are any - has gaps between
  // its attributes: positions from a table)
  const bool skeleton = tb.skel_pos != nullptr && sid >= n_seg - P;
  const int32_t pos = skeleton ? tb.skel_pos[tb.skel_off[sid - (n_seg - P)] + idx] : tb.seg_pos0[sid] + idx;
  const int64_t slot = (int64_t)tb.seg_off[sid] + idx;
  const float2 cs = tb.rope[(int64_t)pos * half + i];
  const int64_t src = (tok * Hkv + h) * D;
  const float a = hpd::to_float(k_raw[src + i]);
  const float b = hpd::to_float(k_raw[src + i + half]);
  const int64_t kdst = ((int64_t)h * NP + slot) * D;
  float r1, r2;
  hpd::rope_pair(a, b, cs.x, cs.y, r1, r2);
  k_prefix[kdst + i] = hpd::cache_from_float<T>(r1);
  k_prefix[kdst + i + half] = hpd::cache_from_float<T>(r2);
  const int64_t vblk = ((int64_t)h * (NP / 8) + slot / 8) * D;
  v_prefix[(vblk + i) * 8 + (slot & 7)] = hpd::cache_from_float<T>(hpd::to_float(v_raw[src + i]));
  v_prefix[(vblk + i + half) * 8 + (slot & 7)] = hpd::cache_from_float<T>(hpd::to_float(v_raw[src + i + half]));
}

// The same for bf16 with 128 channels, the shape the streaming attention kernel serves: one
// 256-thread workgroup per (32-slot block of the pools, kv head), a wave per 8 slots.  Rows move
// as 16-byte pieces (8 lanes per K row); the 8-key interleave of the V pool is a transpose of
// 8 rows x 128 channels through LDS, written back as one contiguous 2 KB run per wave.  Slots
// behind the segment's end get V = 0 (what prefix_pad_kernel does for the general kernel).
// fill_blk[b] = (segment that owns block b | -1, raw index of the block's first token).
__global__ void __launch_bounds__(256)
prefix_fill_bf16_128_kernel(hpd_dev_tables tb, int32_t n_seg, int32_t P, int32_t Hkv, int64_t NP,
                            const int32_t* __restrict__ fill_blk, const uint16_t* __restrict__ k_raw,
                            const uint16_t* __restrict__ v_raw, uint16_t* __restrict__ k_prefix,
                            uint16_t* __restrict__ v_prefix) {
  constexpr int D = 128;
  __shared__ uint16_t vt[4][8][D];
  const int32_t blk = blockIdx.x / Hkv, h = blockIdx.x % Hkv;
  const int32_t sid = fill_blk[2 * blk];
  if (sid < 0) return;  // uniform over the workgroup
  const int32_t raw0 = fill_blk[2 * blk + 1];
  const int32_t idx0 = blk * 32 - tb.seg_off[sid], len = tb.seg_len[sid];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, r = lane >> 3, cc = lane & 7;
  const int32_t idx = idx0 + wave * 8 + r;
  const bool valid = idx < len;
  const int64_t slot = (int64_t)blk * 32 + wave * 8 + r;
  uint4 vlo = make_uint4(0, 0, 0, 0), vhi = vlo;
  if (valid) {
    const int64_t src = ((int64_t)(raw0 + wave * 8 + r) * Hkv + h) * D;
    const uint4 klo = *reinterpret_cast<const uint4*>(k_raw + src + cc * 8);
    const uint4 khi = *reinterpret_cast<const uint4*>(k_raw + src + 64 + cc * 8);
    vlo = *reinterpret_cast<const uint4*>(v_raw + src + cc * 8);
    vhi = *reinterpret_cast<const uint4*>(v_raw + src + 64 + cc * 8);
    const bool skeleton = tb.skel_pos != nullptr && sid >= n_seg - P;
    const int32_t pos = skeleton ? tb.skel_pos[tb.skel_off[sid - (n_seg - P)] + idx] : tb.seg_pos0[sid] + idx;
    const float4* cs = reinterpret_cast<const float4*>(tb.rope + (int64_t)pos * (D / 2) + cc * 8);
    const uint32_t lo[4] = {klo.x, klo.y, klo.z, klo.w}, hi[4] = {khi.x, khi.y, khi.z, khi.w};
    uint32_t olo[4], ohi[4];
#pragma unroll
    for (int e2 = 0; e2 < 4; ++e2) {
      const float4 c4 = cs[e2];  // (cos, sin) of pairs 2*e2, 2*e2 + 1
      float a0, b0, a1, b1;
      hpd::rope_pair(hpd::bf16_bits_to_float(lo[e2] & 0xffffu), hpd::bf16_bits_to_float(hi[e2] & 0xffffu),
                     c4.x, c4.y, a0, b0);
      hpd::rope_pair(hpd::bf16_bits_to_float(lo[e2] >> 16), hpd::bf16_bits_to_float(hi[e2] >> 16),
                     c4.z, c4.w, a1, b1);
      olo[e2] = hpd::cache_bits_pair(hpd::bf16_bits_to_float(hpd::float_to_bf16_bits(a0)),
                                   hpd::bf16_bits_to_float(hpd::float_to_bf16_bits(a1)));
      ohi[e2] = hpd::cache_bits_pair(hpd::bf16_bits_to_float(hpd::float_to_bf16_bits(b0)),
                                   hpd::bf16_bits_to_float(hpd::float_to_bf16_bits(b1)));
    }
    uint16_t* kd = k_prefix + ((int64_t)h * NP + slot) * D;
    *reinterpret_cast<uint4*>(kd + cc * 8) = make_uint4(olo[0], olo[1], olo[2], olo[3]);
    *reinterpret_cast<uint4*>(kd + 64 + cc * 8) = make_uint4(ohi[0], ohi[1], ohi[2], ohi[3]);
  }
  vlo = make_uint4(hpd::cache_bits_from_bf16_pair(vlo.x), hpd::cache_bits_from_bf16_pair(vlo.y),
                   hpd::cache_bits_from_bf16_pair(vlo.z), hpd::cache_bits_from_bf16_pair(vlo.w));
  vhi = make_uint4(hpd::cache_bits_from_bf16_pair(vhi.x), hpd::cache_bits_from_bf16_pair(vhi.y),
                   hpd::cache_bits_from_bf16_pair(vhi.z), hpd::cache_bits_from_bf16_pair(vhi.w));
  *reinterpret_cast<uint4*>(&vt[wave][r][cc * 8]) = vlo;
  *reinterpret_cast<uint4*>(&vt[wave][r][64 + cc * 8]) = vhi;
  __syncthreads();
  uint16_t* vd = v_prefix + (((int64_t)h * (NP / 8) + (int64_t)blk * 4 + wave) * D) * 8;
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    const int c = half * 64 + lane;
    uint32_t w[4];
#pragma unroll
    for (int e2 = 0; e2 < 4; ++e2)
      w[e2] = (uint32_t)vt[wave][2 * e2][c] | ((uint32_t)vt[wave][2 * e2 + 1][c] << 16);
    *reinterpret_cast<uint4*>(vd + (int64_t)c * 8) = make_uint4(w[0], w[1], w[2], w[3]);
  }
}

// Zero values in the padding slots between a segment's end and the next multiple of the key
// block: the attention kernels give those keys probability 0 and rely on 0 * V being 0.
// One thread per (segment, kv head, padding slot, channel).
template <typename T>
__global__ void prefix_pad_kernel(hpd_dev_tables tb, int32_t n_seg, int32_t Hkv, int32_t D, int64_t NP,
                                  T* __restrict__ v_prefix) {
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t total = (int64_t)n_seg * Hkv * (HPD_KEY_BLOCK - 1) * D;
  if (gid >= total) return;
  const int32_t c = (int32_t)(gid % D);
  const int32_t j = (int32_t)((gid / D) % (HPD_KEY_BLOCK - 1));
  const int32_t h = (int32_t)((gid / ((int64_t)D * (HPD_KEY_BLOCK - 1))) % Hkv);
  const int32_t sid = (int32_t)(gid / ((int64_t)D * (HPD_KEY_BLOCK - 1) * Hkv));
  const int32_t len = tb.seg_len[sid];
  const int32_t pad = (HPD_KEY_BLOCK - len % HPD_KEY_BLOCK) % HPD_KEY_BLOCK;
  if (j >= pad) return;
  const int64_t slot = (int64_t)tb.seg_off[sid] + len + j;
  v_prefix[(((int64_t)h * (NP / 8) + slot / 8) * D + c) * 8 + (slot & 7)] = hpd::from_float<T>(0.f);
}

// ---------------------------------------------------------------------------------------
// Position IDs of the live branches of one step.
// ---------------------------------------------------------------------------------------
__global__ void positions_kernel(hpd_dev_tables tb, int32_t step, int32_t n_live,
                                 int32_t* __restrict__ pos_out) {
  const int32_t r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= n_live) return;
  const int32_t b = tb.live_branch[tb.live_ptr[step] + r];
  pos_out[r] = tb.branch_base_pos[b] + 1 + step;
}

// ---------------------------------------------------------------------------------------
// Append: RoPE(K) + store K, V of every live branch at tail slot b*T + step (or the slot its
// page table names).
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ void append_kernel(hpd_dev_tables tb, int32_t step, int32_t n_live, int32_t Hkv,
                              int32_t D, int32_t Tcap, const T* __restrict__ k_new,
                              const T* __restrict__ v_new, T* __restrict__ k_tail,
                              T* __restrict__ v_tail, int64_t* __restrict__ slot_out) {
  const int32_t half = D / 2;
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t total = (int64_t)n_live * Hkv * half;
  if (gid >= total) return;
  const int32_t i = (int32_t)(gid % half);
  const int32_t h = (int32_t)((gid / half) % Hkv);
  const int32_t r = (int32_t)(gid / ((int64_t)half * Hkv));
  const int32_t b = tb.live_branch[tb.live_ptr[step] + r];
  const int32_t pos = tb.branch_base_pos[b] + 1 + step;
  const float2 cs = tb.rope[(int64_t)pos * half + i];
  const int64_t src = ((int64_t)r * Hkv + h) * D;
  const float a = hpd::to_float(k_new[src + i]);
  const float bb = hpd::to_float(k_new[src + i + half]);
  const int64_t row = hpd_tail_row(tb, b, h, Hkv, Tcap, step);
  const int64_t dst = row * D;
  // the slot number leaves the kv heads out: the row of a pool with one kv head
  const int64_t slot = hpd_tail_row(tb, b, 0, 1, Tcap, step);
  float r1, r2;
  hpd::rope_pair(a, bb, cs.x, cs.y, r1, r2);
  k_tail[dst + i] = hpd::cache_from_float<T>(r1);
  k_tail[dst + i + half] = hpd::cache_from_float<T>(r2);
  v_tail[dst + i] = hpd::cache_from_float<T>(hpd::to_float(v_new[src + i]));
  v_tail[dst + i + half] = hpd::cache_from_float<T>(hpd::to_float(v_new[src + i + half]));
  if (slot_out && h == 0 && i == 0) slot_out[r] = slot;
}

// ---------------------------------------------------------------------------------------
// Dense mask export (debugging aid).  desc[S][4] = (kind, document, branch, step); for the
// paper-literal mask the last entry is the position ID and the rule is Section 4.3.2's:
// already in memory and not later in position order.
// ---------------------------------------------------------------------------------------
__global__ void expand_mask_kernel(const int32_t* __restrict__ desc, int32_t S, int32_t paper,
                                   uint8_t* __restrict__ mask) {
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= (int64_t)S * S) return;
  const int32_t qi = (int32_t)(gid / S), ki = (int32_t)(gid % S);
  const int32_t qk = desc[qi * 4], qd = desc[qi * 4 + 1], qb = desc[qi * 4 + 2], qs = desc[qi * 4 + 3];
  const int32_t kk = desc[ki * 4], kd = desc[ki * 4 + 1], kb = desc[ki * 4 + 2], ks = desc[ki * 4 + 3];
  bool ok;
  if (paper) ok = ki <= qi && ks <= qs;
  else if (kk == 0) ok = (qk != 0) || (ki <= qi);                    // header key
  else if (kk == 1) ok = (qk == 1 && qd == kd && ki <= qi) || (qk == 2 && qd == kd);  // doc key
  else ok = (qk == 2 && qb == kb && ks <= qs);                        // branch key
  mask[gid] = ok ? 1 : 0;
}

// ---------------------------------------------------------------------------------------
// Device-side pruning (Section 4.3.4): one workgroup turns the live list of the step just
// taken and its "finished" flags into the next step's live list (ascending branch id) and one
// work-unit descriptor per document, in the order of `fixed` (documents without live branches
// get a descriptor with 0 branches).  live / n_live / desc are the layout's state; `fixed` holds
// {hoff, Hlen, doff, Llen, first branch, end of branches, position of step 0 | -1, 0} per
// document.  The liveness of every branch is kept in LDS, one byte each, for the length of
// the kernel; nothing the kernel writes to global memory is read back.
// Literal mask (`len` given): the units are prompts - `fixed` holds {hoff, Hlen, first entry
// of the prompt's block list, its blocks, first branch, end of branches, 0, 0} and a descriptor
// has 16 words, as the host builds them - and since a finished branch stays visible to the
// later ones, the number of tokens it reached is kept in `len` (the step budget while it runs).
// ---------------------------------------------------------------------------------------
constexpr int PRUNE_THREADS = 1024;
constexpr int PRUNE_MAX_BRANCHES = 65536;
__global__ void __launch_bounds__(PRUNE_THREADS)
dynamic_prune_kernel(int32_t n_docs, int32_t B, int32_t next_step, const uint8_t* __restrict__ finished,
                     const int4* __restrict__ fixed, int32_t* __restrict__ live,
                     int32_t* __restrict__ n_live, int4* __restrict__ desc, int32_t* __restrict__ len,
                     int32_t Tcap) {
  __shared__ uint32_t al_words[PRUNE_MAX_BRANCHES / 4];
  __shared__ int32_t pex[PRUNE_THREADS];   // branches alive before each thread's run
  __shared__ int32_t wsum[PRUNE_THREADS / 64];
  uint8_t* al = reinterpret_cast<uint8_t*>(al_words);
  const int32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // the first document of this thread: requested now, needed at the end
  int4 fx0 = make_int4(0, 0, 0, 0), fx1 = fx0;
  if (tid < n_docs) { fx0 = fixed[2 * tid]; fx1 = fixed[2 * tid + 1]; }
  // 1. liveness after the step just taken (no flags: a fresh start, all live)
  const uint32_t fill = finished ? 0u : 0x01010101u;
  for (int32_t w = tid; w < (B + 3) / 4; w += PRUNE_THREADS) al_words[w] = fill;
  __syncthreads();
  if (finished) {
    const int32_t n_prev = n_live[0];
    // eight rows per thread and pass, all sixteen loads requested before the first is used
    for (int32_t r0 = tid; r0 < n_prev; r0 += 8 * PRUNE_THREADS) {
      uint8_t f[8];
      int32_t lb[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const int32_t r = r0 + k * PRUNE_THREADS;
        f[k] = r < n_prev ? finished[r] : (uint8_t)1;
        lb[k] = r < n_prev ? live[r] : 0;
      }
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        if (!f[k]) al[lb[k]] = 1;
        else if (len && r0 + k * PRUNE_THREADS < n_prev) len[lb[k]] = next_step;  // tokens 0 .. next_step-1 exist
      }
    }
    __syncthreads();  // the old list has been read; it is overwritten below
  }
  if (!finished && len)
    for (int32_t b = tid; b < B; b += PRUNE_THREADS) len[b] = Tcap;
  // 2. exclusive prefix sums over the branches: thread t owns a run of `chunk` branches; the
  //    run sums are scanned inside each wave, the 16 wave sums by every thread for itself
  const int32_t chunk = (B + PRUNE_THREADS - 1) / PRUNE_THREADS;
  const int32_t b0 = min(tid * chunk, B), b1 = min(b0 + chunk, B);
  int32_t cnt = 0;
  for (int32_t b = b0; b < b1; ++b) cnt += al[b];
  int32_t incl = cnt;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int32_t v = __shfl_up(incl, o);
    if (lane >= o) incl += v;
  }
  if (lane == 63) wsum[wave] = incl;
  __syncthreads();
  int32_t run = incl - cnt, total = 0;
#pragma unroll
  for (int w = 0; w < PRUNE_THREADS / 64; ++w) {
    const int32_t x = wsum[w];
    if (w < wave) run += x;
    total += x;
  }
  pex[tid] = run;
  for (int32_t b = b0; b < b1; ++b)
    if (al[b]) live[run++] = b;
  if (tid == 0) n_live[0] = total;
  __syncthreads();  // pex is read below by other threads
  // live branches with an id below x
  auto rank = [&](int32_t x) -> int32_t {
    if (x >= B) return total;
    const int32_t t = x / chunk;
    int32_t r = pex[t];
    for (int32_t b = t * chunk; b < x; ++b) r += al[b];
    return r;
  };
  // 3. one descriptor per document: {hoff, Hlen, doff, Llen, first live row, live branches,
  //    shared position | -1, first branch id if the live ones are consecutive | -1}
  for (int32_t u = tid; u < n_docs; u += PRUNE_THREADS) {
    if (u != tid) { fx0 = fixed[2 * u]; fx1 = fixed[2 * u + 1]; }
    const int32_t lo = fx1.x, hi = fx1.y;
    const int32_t first = rank(lo), nb = rank(hi) - first;
    int32_t b_first = -1;
    if (nb > 0) {
      int32_t x = lo, y = hi - 1;  // the document's first and last live branch
      while (!al[x]) ++x;
      while (!al[y]) --y;
      if (y - x == nb - 1) b_first = x;
    }
    if (!len) {
      desc[2 * u] = fx0;
      desc[2 * u + 1] = make_int4(first, nb, fx1.z >= 0 ? fx1.z + next_step : -1, b_first);
    } else {
      // {hoff, Hlen, list entry, blocks | first live row, live branches, first branch of the
      //  prompt, first live branch if consecutive | key branches: first .. last live | 0}
      int32_t y = hi - 1;
      while (nb > 0 && !al[y]) --y;
      desc[4 * u] = fx0;
      desc[4 * u + 1] = make_int4(first, nb, lo, b_first);
      desc[4 * u + 2] = make_int4(nb > 0 ? y - lo + 1 : 0, 0, 0, 0);
      desc[4 * u + 3] = make_int4(0, 0, 0, 0);
    }
  }
}

// ---------------------------------------------------------------------------------------
// Fine-tuning mask (Section 4.4).  desc[S][4] = (kind, attribute, k, position ID) in the regular
// token order; kind 0 prompt, 1 attribute, 2 value token.
// ---------------------------------------------------------------------------------------
__global__ void finetune_mask_kernel(const int32_t* __restrict__ desc, int32_t S,
                                     uint8_t* __restrict__ mask) {
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= (int64_t)S * S) return;
  const int32_t qi = (int32_t)(gid / S), ki = (int32_t)(gid % S);
  const int32_t qk = desc[qi * 4], qn = desc[qi * 4 + 1], qs = desc[qi * 4 + 2];
  const int32_t kk = desc[ki * 4], kn = desc[ki * 4 + 1], ks = desc[ki * 4 + 2];
  bool ok = ki <= qi;                                       // causal
  if (kk == 2 && qk == 1) ok = false;                       // attributes never see values
  if (kk == 2 && qk == 2 && kn < qn && ks > qs) ok = false;  // not generated yet
  mask[gid] = ok ? 1 : 0;
}

__global__ void finetune_pos_kernel(const int32_t* __restrict__ desc, int32_t S, int32_t* __restrict__ pos) {
  const int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < S) pos[i] = desc[i * 4 + 3];
}

// ---------------------------------------------------------------------------------------
// Generic attention: one 256-thread block per (live row, query head).
//   phase 1  one key per thread: full dot product with the rotated query (kept in LDS),
//            scores to LDS, block max
//   phase 2  p = exp(s - max), block sum
//   phase 3  one channel per thread, keys split over 256/D thread groups, reduce in LDS
// ---------------------------------------------------------------------------------------
constexpr int GEN_THREADS = 256;

__device__ inline float block_reduce(float v, bool is_max, float* red) {
  for (int o = 32; o > 0; o >>= 1) {
    const float w = __shfl_xor(v, o);
    v = is_max ? fmaxf(v, w) : v + w;
  }
  const int wave = threadIdx.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[wave] = v;
  __syncthreads();
  float r = red[0];
  for (int w = 1; w < GEN_THREADS / 64; ++w) r = is_max ? fmaxf(r, red[w]) : r + red[w];
  return r;
}

// PAPER = the literal mask of Section 4.3.2: the keys of a row are the header, every document
// of the prompt, and positions 0..step of every branch of the prompt up to the row's own (a
// position a finished branch never reached gets probability 0).
// GM_PREFILL = the attention of the prefix tokens themselves (first inference step, block
// mask): row r is token r of hpd_prefix_fill's order, at its own position ID; its keys are the
// header (for a document token) and its own segment up to itself.  `step` then carries the
// number of segments.
// GM_PREFILL_PAPER = the same under the literal mask: header, documents and attribute names of
// a prompt are one causal sequence (a document token also sees the earlier documents, a name
// token everything before it).
enum { GM_BLOCK = 0, GM_PAPER = 1, GM_PREFILL = 2, GM_PREFILL_PAPER = 3 };
template <typename T, int GM>
__global__ void __launch_bounds__(GEN_THREADS)
attention_generic_kernel(hpd_dev_tables tb, int32_t step, int32_t Hq, int32_t Hkv, int32_t D,
                         int32_t Tcap, int32_t P, int64_t NP, const T* __restrict__ q,
                         const T* __restrict__ k_prefix, const T* __restrict__ v_prefix,
                         const T* __restrict__ k_tail, const T* __restrict__ v_tail,
                         void* __restrict__ out, int32_t out_f32) {
  extern __shared__ float smem[];
  float* q_rot = smem;             // [D]
  float* red = smem + D;           // [8]
  float* part = red + 8;           // [256] partial outputs
  float* scores = part + GEN_THREADS;  // [n_keys]

  constexpr bool PAPER = GM == GM_PAPER, PPL = GM == GM_PREFILL_PAPER, PREFILL = GM == GM_PREFILL || PPL;
  const int32_t r = blockIdx.x / Hq;
  const int32_t h = blockIdx.x % Hq;
  const int32_t hk = h / (Hq / Hkv);
  int32_t b = 0, d = 0, p = 0, pos = 0, Hlen = 0, Llen = 0, d_lo = 0, d_hi = 0, b_lo = 0, n_tail = 0;
  int32_t n_names = 0;  // PPL: name tokens the row sees (itself included)
  if (PREFILL) {
    // segment that holds token r: last entry of the sorted start table <= r (empty ones skipped)
    const int32_t n_seg = step;
    int32_t lo = 0, hi = n_seg;
    while (hi - lo > 1) {
      const int32_t mid = (lo + hi) >> 1;
      if (tb.seg_raw_off[mid] <= r) lo = mid; else hi = mid;
    }
    while (lo + 1 < n_seg && tb.seg_raw_off[lo + 1] <= r) ++lo;
    const int32_t sid = tb.raw_seg[lo], idx = r - tb.seg_raw_off[lo];
    pos = tb.seg_pos0[sid] + idx;
    const int32_t n_docs = PPL ? n_seg - 2 * P : n_seg - P;
    if (sid < P) {  // a header token: the header up to itself
      p = sid;
      Hlen = idx + 1;
    } else if (sid < P + n_docs) {  // a document token: the header, the document up to itself
      d = sid - P;
      p = tb.doc_prompt[d];
      Hlen = tb.seg_len[p];
      Llen = idx + 1;
      d_lo = d; d_hi = d + 1;
      if (PPL) {    // ... and the earlier documents of the prompt
        d_lo = tb.prompt_doc_ptr[p];
        for (int32_t dd = d_lo; dd < d; ++dd) Llen += tb.seg_len[P + dd];
      }
    } else {        // a name token: header, every document, the names up to itself
      p = sid - P - n_docs;
      Hlen = tb.seg_len[p];
      d_lo = tb.prompt_doc_ptr[p]; d_hi = tb.prompt_doc_ptr[p + 1];
      for (int32_t dd = d_lo; dd < d_hi; ++dd) Llen += tb.seg_len[P + dd];
      n_names = idx + 1;
      pos = tb.skel_pos[tb.skel_off[p] + idx];
    }
  } else {
    b = tb.live_branch[tb.live_ptr[step] + r];
    d = tb.branch_doc[b];
    p = tb.doc_prompt[d];
    pos = tb.branch_base_pos[b] + 1 + step;
    Hlen = tb.seg_len[p];
    // documents the row sees: its own, or all of its prompt
    d_lo = PAPER ? tb.prompt_doc_ptr[p] : d;
    d_hi = PAPER ? tb.prompt_doc_ptr[p + 1] : d + 1;
    for (int32_t dd = d_lo; dd < d_hi; ++dd) Llen += tb.seg_len[P + dd];
    // branches whose tails the row sees: its own, or the prompt's first .. its own
    b_lo = PAPER ? tb.prompt_branch_ptr[p] : b;
    n_tail = (b - b_lo + 1) * (step + 1);
  }
  const int64_t hoff = tb.seg_off[p];
  // PAPER: the attribute names up to the row's own branch, counted with the documents
  const int32_t Dlen = Llen;
  if (PAPER) Llen += tb.skel_cum[b];
  if (PPL) Llen += n_names;
  const int32_t n_keys = Hlen + Llen + n_tail;
  const int32_t half = D / 2;
  const int tid = threadIdx.x;
  // pool slot of prefix key kk (>= Hlen: the documents one after the other)
  auto doc_slot = [&](int32_t kk) -> int64_t {
    if ((PAPER || PPL) && kk >= Hlen + Dlen) return (int64_t)tb.skel_seg_off[p] + (kk - Hlen - Dlen);
    int32_t i = kk - Hlen, dd = d_lo;
    while (i >= tb.seg_len[P + dd]) { i -= tb.seg_len[P + dd]; ++dd; }
    return (int64_t)tb.seg_off[P + dd] + i;
  };
  // tail key i: position i % (step+1) of branch b_lo + i / (step+1); -1 if it does not exist
  auto tail_row = [&](int32_t i) -> int64_t {
    const int32_t bb = b_lo + i / (step + 1), tt = i % (step + 1);
    if (tt >= tb.branch_len[bb]) return -1;
    return hpd_tail_row(tb, bb, hk, Hkv, Tcap, tt) * D;
  };

  if (tid < half) {
    const float2 cs = tb.rope[(int64_t)pos * half + tid];
    const int64_t src = ((int64_t)r * Hq + h) * D;
    const float a = hpd::to_float(q[src + tid]), bb = hpd::to_float(q[src + tid + half]);
    hpd::rope_pair(a, bb, cs.x, cs.y, q_rot[tid], q_rot[tid + half]);
  }
  __syncthreads();

  const float scale = 1.0f / sqrtf((float)D);
  float lmax = -INFINITY;
  for (int32_t kk = tid; kk < n_keys; kk += GEN_THREADS) {
    const T* kp;
    if (kk < Hlen) kp = k_prefix + ((int64_t)hk * NP + hoff + kk) * D;
    else if (kk < Hlen + Llen) kp = k_prefix + ((int64_t)hk * NP + doc_slot(kk)) * D;
    else {
      const int64_t row = tail_row(kk - Hlen - Llen);
      if (row < 0) { scores[kk] = -INFINITY; continue; }
      kp = k_tail + row;
    }
    float acc = 0.f;
    for (int32_t c = 0; c < D; c += 8) {
      float kv[8];
      hpd::load8_cache(kp + c, kv);
#pragma unroll
      for (int e = 0; e < 8; ++e) acc = fmaf(kv[e], q_rot[c + e], acc);
    }
    acc *= scale;
    scores[kk] = acc;
    lmax = fmaxf(lmax, acc);
  }
  const float m = block_reduce(lmax, true, red);
  float lsum = 0.f;
  for (int32_t kk = tid; kk < n_keys; kk += GEN_THREADS) {
    const float pr = expf(scores[kk] - m);
    scores[kk] = pr;
    lsum += pr;
  }
  const float l = block_reduce(lsum, false, red);  // contains the barrier that publishes scores

  const int32_t groups = GEN_THREADS / D > 0 ? GEN_THREADS / D : 1;
  const int32_t c = tid % D, g = tid / D;
  float acc = 0.f;
  if (g < groups && tid < groups * D) {
    const int64_t vhead = (int64_t)hk * (NP / 8);
    for (int32_t kk = g; kk < n_keys; kk += groups) {
      float vv;
      if (kk < Hlen + Llen) {
        const int64_t slot = (kk < Hlen) ? hoff + kk : doc_slot(kk);
        vv = hpd::cache_to_float(v_prefix[((vhead + slot / 8) * D + c) * 8 + (slot & 7)]);
      } else {
        const int64_t row = tail_row(kk - Hlen - Llen);
        if (row < 0) continue;  // probability 0
        vv = hpd::cache_to_float(v_tail[row + c]);
      }
      acc = fmaf(scores[kk], vv, acc);
    }
  }
  part[tid] = acc;
  __syncthreads();
  if (tid < D) {
    float o = 0.f;
    for (int32_t gg = 0; gg < groups; ++gg) o += part[gg * D + tid];
    const int64_t oi = ((int64_t)r * Hq + h) * D + tid;
    if (out_f32) reinterpret_cast<float*>(out)[oi] = o / l;
    else reinterpret_cast<T*>(out)[oi] = hpd::from_float<T>(o / l);
  }
}

inline dim3 grid1d(int64_t n, int block) { return dim3((unsigned)((n + block - 1) / block)); }

}  // namespace

hipError_t hpd_launch_prefix_fill(const hpd_layout* L, const void* k_raw, const void* v_raw,
                                  void* k_prefix, void* v_prefix, hipStream_t s) {
  const int64_t total = L->n_prefix_tokens * L->cfg.n_kv_heads * (L->cfg.head_dim / 2);
  if (total == 0) return hipSuccess;
  const int64_t pad_total = (int64_t)L->n_seg * L->cfg.n_kv_heads * (HPD_KEY_BLOCK - 1) * L->cfg.head_dim;
  if (L->cfg.dtype == HPD_BF16 && L->cfg.head_dim == 128 && L->kernel_mode != 1 && L->dev.fill_blk) {
    const int64_t items = (L->NP / HPD_KEY_BLOCK) * L->cfg.n_kv_heads;
    if (items > 0x7fffffff) return hipErrorInvalidValue;
    prefix_fill_bf16_128_kernel<<<dim3((unsigned)items), 256, 0, s>>>(
        L->dev, L->n_seg, L->P, L->cfg.n_kv_heads, L->NP, L->dev.fill_blk, (const uint16_t*)k_raw,
        (const uint16_t*)v_raw, (uint16_t*)k_prefix, (uint16_t*)v_prefix);
    return hipGetLastError();
  }
  if (L->cfg.dtype == HPD_F32) {
    prefix_fill_kernel<float><<<grid1d(total, 256), 256, 0, s>>>(
        L->dev, L->n_seg, L->P, L->n_prefix_tokens, L->cfg.n_kv_heads, L->cfg.head_dim, L->NP,
        (const float*)k_raw, (const float*)v_raw, (float*)k_prefix, (float*)v_prefix);
    prefix_pad_kernel<float><<<grid1d(pad_total, 256), 256, 0, s>>>(
        L->dev, L->n_seg, L->cfg.n_kv_heads, L->cfg.head_dim, L->NP, (float*)v_prefix);
  } else {
    prefix_fill_kernel<hpd::bf16_t><<<grid1d(total, 256), 256, 0, s>>>(
        L->dev, L->n_seg, L->P, L->n_prefix_tokens, L->cfg.n_kv_heads, L->cfg.head_dim, L->NP,
        (const hpd::bf16_t*)k_raw, (const hpd::bf16_t*)v_raw, (hpd::bf16_t*)k_prefix,
        (hpd::bf16_t*)v_prefix);
    prefix_pad_kernel<hpd::bf16_t><<<grid1d(pad_total, 256), 256, 0, s>>>(
        L->dev, L->n_seg, L->cfg.n_kv_heads, L->cfg.head_dim, L->NP, (hpd::bf16_t*)v_prefix);
  }
  return hipGetLastError();
}

hipError_t hpd_launch_positions(const hpd_layout* L, int32_t step, int32_t* pos_out, hipStream_t s) {
  const int32_t n_live = L->live_ptr[step + 1] - L->live_ptr[step];
  positions_kernel<<<grid1d(n_live, 256), 256, 0, s>>>(L->dev, step, n_live, pos_out);
  return hipGetLastError();
}

hipError_t hpd_launch_append(const hpd_layout* L, int32_t step, const void* k_new, const void* v_new,
                             void* k_tail, void* v_tail, int64_t* slot_out, hipStream_t s) {
  const int32_t n_live = L->live_ptr[step + 1] - L->live_ptr[step];
  const int64_t total = (int64_t)n_live * L->cfg.n_kv_heads * (L->cfg.head_dim / 2);
  if (L->cfg.dtype == HPD_F32)
    append_kernel<float><<<grid1d(total, 256), 256, 0, s>>>(
        L->dev, step, n_live, L->cfg.n_kv_heads, L->cfg.head_dim, L->T, (const float*)k_new,
        (const float*)v_new, (float*)k_tail, (float*)v_tail, slot_out);
  else
    append_kernel<hpd::bf16_t><<<grid1d(total, 256), 256, 0, s>>>(
        L->dev, step, n_live, L->cfg.n_kv_heads, L->cfg.head_dim, L->T, (const hpd::bf16_t*)k_new,
        (const hpd::bf16_t*)v_new, (hpd::bf16_t*)k_tail, (hpd::bf16_t*)v_tail, slot_out);
  return hipGetLastError();
}

int64_t hpd_generic_max_keys(const hpd_layout* L, int32_t step) {
  int64_t max_keys = 0;
  if (L->cfg.mask_mode == HPD_MASK_PAPER) {
    for (int32_t p = 0; p < L->P; ++p) {
      int64_t n = L->seg_len[p];
      for (int32_t d = L->prompt_doc_ptr[p]; d < L->prompt_doc_ptr[p + 1]; ++d) n += L->seg_len[L->P + d];
      n += (int64_t)(L->prompt_branch_ptr[p + 1] - L->prompt_branch_ptr[p]) * (step + 1);
      n += L->seg_len[L->P + L->n_docs + p];  // attribute names
      max_keys = std::max(max_keys, n);
    }
    return max_keys;
  }
  for (int32_t u = L->unit_ptr[step]; u < L->unit_ptr[step + 1]; ++u) {
    const int32_t d = L->unit_doc[u];
    max_keys = std::max<int64_t>(max_keys, (int64_t)L->seg_len[L->doc_prompt[d]] +
                                               L->seg_len[L->P + d] + step + 1);
  }
  return max_keys;
}

template <typename T, int GM>
static hipError_t launch_generic(const hpd_layout* L, int32_t step, const void* q, const void* k_prefix,
                                 const void* v_prefix, const void* k_tail, const void* v_tail, void* out,
                                 hipStream_t s) {
  int64_t n_rows = 0, max_keys = 0;
  if (GM == GM_PREFILL || GM == GM_PREFILL_PAPER) {
    n_rows = L->n_prefix_tokens;
    if (GM == GM_PREFILL_PAPER)  // a prompt's last name token sees the whole prefix of the prompt
      for (int32_t p = 0; p < L->P; ++p) {
        int64_t keys = (int64_t)L->seg_len[p] + L->seg_len[L->P + L->n_docs + p];
        for (int32_t d = L->prompt_doc_ptr[p]; d < L->prompt_doc_ptr[p + 1]; ++d) keys += L->seg_len[L->P + d];
        max_keys = std::max(max_keys, keys);
      }
    for (int32_t d = 0; d < L->n_docs; ++d)
      max_keys = std::max<int64_t>(max_keys, (int64_t)L->seg_len[L->doc_prompt[d]] + L->seg_len[L->P + d]);
    for (int32_t p = 0; p < L->P; ++p) max_keys = std::max<int64_t>(max_keys, L->seg_len[p]);
    step = L->n_seg;
  } else {
    n_rows = L->live_ptr[step + 1] - L->live_ptr[step];
    max_keys = hpd_generic_max_keys(L, step);
  }
  const size_t smem = (size_t)(L->cfg.head_dim + 8 + GEN_THREADS + max_keys) * sizeof(float);
  const dim3 grid((unsigned)(n_rows * L->cfg.n_q_heads));
  const int32_t out_f32 = (L->cfg.dtype == HPD_F32 || L->cfg.out_dtype == HPD_OUT_F32) ? 1 : 0;
  attention_generic_kernel<T, GM><<<grid, GEN_THREADS, smem, s>>>(
      L->dev, step, L->cfg.n_q_heads, L->cfg.n_kv_heads, L->cfg.head_dim, L->T, L->P, L->NP, (const T*)q,
      (const T*)k_prefix, (const T*)v_prefix, (const T*)k_tail, (const T*)v_tail, out, out_f32);
  return hipGetLastError();
}

hipError_t hpd_launch_attention_generic(const hpd_layout* L, int32_t step, const void* q,
                                        const void* k_prefix, const void* v_prefix,
                                        const void* k_tail, const void* v_tail, void* out,
                                        hipStream_t s) {
  const bool paper = L->cfg.mask_mode == HPD_MASK_PAPER;
  if (L->cfg.dtype == HPD_F32)
    return paper ? launch_generic<float, GM_PAPER>(L, step, q, k_prefix, v_prefix, k_tail, v_tail, out, s)
                 : launch_generic<float, GM_BLOCK>(L, step, q, k_prefix, v_prefix, k_tail, v_tail, out, s);
  return paper ? launch_generic<hpd::bf16_t, GM_PAPER>(L, step, q, k_prefix, v_prefix, k_tail, v_tail, out, s)
               : launch_generic<hpd::bf16_t, GM_BLOCK>(L, step, q, k_prefix, v_prefix, k_tail, v_tail, out, s);
}

hipError_t hpd_launch_prefill_generic(const hpd_layout* L, const void* q, const void* k_prefix,
                                      const void* v_prefix, void* out, hipStream_t s) {
  // no tail key exists: the tail pools are never addressed
  const bool paper = L->cfg.mask_mode == HPD_MASK_PAPER;
  if (L->cfg.dtype == HPD_F32)
    return paper ? launch_generic<float, GM_PREFILL_PAPER>(L, 0, q, k_prefix, v_prefix, k_prefix, v_prefix, out, s)
                 : launch_generic<float, GM_PREFILL>(L, 0, q, k_prefix, v_prefix, k_prefix, v_prefix, out, s);
  return paper ? launch_generic<hpd::bf16_t, GM_PREFILL_PAPER>(L, 0, q, k_prefix, v_prefix, k_prefix, v_prefix, out, s)
               : launch_generic<hpd::bf16_t, GM_PREFILL>(L, 0, q, k_prefix, v_prefix, k_prefix, v_prefix, out, s);
}

hipError_t hpd_launch_expand_mask(const int32_t* d_desc, int32_t S, int32_t paper, uint8_t* mask_out,
                                  hipStream_t s) {
  expand_mask_kernel<<<grid1d((int64_t)S * S, 256), 256, 0, s>>>(d_desc, S, paper, mask_out);
  return hipGetLastError();
}

hipError_t hpd_launch_finetune_mask(const int32_t* d_desc, int32_t S, int32_t* pos_out, uint8_t* mask_out,
                                    hipStream_t s) {
  if (pos_out) finetune_pos_kernel<<<grid1d(S, 256), 256, 0, s>>>(d_desc, S, pos_out);
  if (mask_out) finetune_mask_kernel<<<grid1d((int64_t)S * S, 256), 256, 0, s>>>(d_desc, S, mask_out);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// File-scope device memory for hpd_dynamic_begin_static (callers that cannot allocate): the
// pruning state of one layout per GPU.  In host code the array's name is only a handle for
// hipGetSymbolAddress; the address kernels may use is looked up once per device, with that
// device current, and kept.
// ---------------------------------------------------------------------------------------
static __device__ __align__(256) int32_t scratch[HPD_DYNAMIC_STATIC_MAX_BYTES / sizeof(int32_t)];

hipError_t hpd_dynamic_scratch(int device, void** ptr, size_t* bytes) {
  constexpr int MAX_DEVICES = 64;
  static std::mutex mu;
  static void* dev_ptr[MAX_DEVICES] = {};
  if (device < 0 || device >= MAX_DEVICES || !ptr || !bytes) return hipErrorInvalidValue;
  std::lock_guard<std::mutex> lock(mu);
  if (!dev_ptr[device]) {
    int cur = -1;
    hipError_t e = hipGetDevice(&cur);
    if (e != hipSuccess) return e;
    if (cur != device && (e = hipSetDevice(device)) != hipSuccess) return e;
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (cur != device) {
      const hipError_t e2 = hipSetDevice(cur);
      if (e == hipSuccess) e = e2;
    }
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    dev_ptr[device] = p;
  }
  *ptr = dev_ptr[device];
  *bytes = sizeof(scratch);
  return hipSuccess;
}

hipError_t hpd_launch_dynamic_prune(const hpd_layout* L, int32_t next_step, const uint8_t* finished,
                                    hipStream_t s) {
  const bool paper = L->cfg.mask_mode == HPD_MASK_PAPER;
  dynamic_prune_kernel<<<1, PRUNE_THREADS, 0, s>>>(paper ? L->P : L->n_docs, L->B, next_step, finished,
                                                   (const int4*)L->dyn_fixed_dev, L->dyn_live, L->dyn_n_live,
                                                   (int4*)L->dyn_desc, paper ? L->dyn_len : nullptr, L->T);
  return hipGetLastError();
}
