// Internal declarations shared by the host side (layout builder, C ABI) and the
// kernel launchers.  Not part of the public interface.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "hpd.h"

// Device-resident tables of one layout.  All int32 tables live in one allocation.
struct hpd_dev_tables {
  const int32_t* seg_off;       // [n_seg] first pool slot of header p (index p) / document d (index P+d)
  const int32_t* seg_len;       // [n_seg]
  const int32_t* seg_pos0;      // [n_seg] position ID of the first token
  const int32_t* seg_raw_off;   // [n_seg+1] first token in prefix_fill input order (sorted by raw order, see raw_seg)
  const int32_t* raw_seg;       // [n_seg] segment ids in raw (prompt-major) order
  const int32_t* doc_prompt;    // [n_docs]
  const int32_t* branch_doc;    // [B]
  const int32_t* branch_base_pos;  // [B]
  const int32_t* live_ptr;      // [T+1]
  const int32_t* live_branch;   // [total_live]
  const int32_t* doc_live_ptr;  // [T][n_docs+1] first live row (within the step's list) of each document
  const int32_t* unit_ptr;      // [T+1]
  const int32_t* unit_doc;      // [total_units] documents with live branches, heaviest first
  const int32_t* unit_desc;     // [total_units][8] {hoff, Hlen, doff, Llen, first live row, live branches, position or -1, first branch id or -1}
  const int32_t* prompt_doc_ptr;     // [P+1] first document of each prompt
  const int32_t* prompt_branch_ptr;  // [P+1] first branch of each prompt
  const int32_t* branch_len;         // [B] steps a branch is decoded for
  // paper-literal mask only: work units are prompts
  const int32_t* pblk;        // [total document blocks][2] (first pool slot, keys) of every 32-key block of a prompt's documents
  const int32_t* punit_desc;  // [total_punits][16] {hoff, Hlen, first pblk entry, document blocks, first live row, live branches, first branch of the prompt, first live branch id or -1, key branches (first .. last live), 0...}
  // paper-literal mask only: the attribute-name (skeleton) tokens of a prompt are a segment of
  // their own (id P + n_docs + p), fed after the prompt's documents
  const int32_t* skel_pos;      // [total name tokens] position IDs (Algorithm 2), prompt by prompt; null without skeleton segments
  const int32_t* skel_off;      // [P+1] first entry of each prompt in skel_pos
  const int32_t* skel_seg_off;  // [P] first pool slot of each prompt's skeleton segment
  const int32_t* skel_cum;      // [B] name tokens of the prompt's branches up to and including b
  // attention of the prefix tokens (block mask): one unit per non-empty header / document
  const int32_t* funit_desc;  // [n_funits][8] {hoff, Hlen (0 for a header), first slot, tokens, first token in q / out order, tokens, position ID of the first token, 0}
  // the same under the literal mask: one unit per non-empty header / document / names segment,
  // {first entry of the prompt in fblk, list blocks seen in full, first slot, tokens, first token in
  //  q / out order, tokens, position ID of the first token | -(1 + first entry in skel_pos), 0}
  const int32_t* fblk;        // [total header and document blocks][2] (first pool slot, keys), prompt by prompt
  const int32_t* fill_blk;    // [NP/32][2] (segment that owns the 32-slot block | -1, raw index of its first token)
  const float2* rope;           // [max_pos+1][D/2] (cos, sin)
  // paged tails (null: token t of branch b is row b*T + t of every kv head's tail rows)
  const int32_t* tail_pages;    // [B][pages_per_branch], the caller's device memory
  int32_t page_shift, pages_per_branch, n_pages;
};

// Row (of D elements) of the tail pools that holds token t of branch b for kv head hk:
// [B][Hkv][T] rows, or [n_pages][Hkv][page] rows under a page table.  A page id is clamped
// to the pool instead of trusted.
__device__ __forceinline__ int64_t hpd_tail_row(const hpd_dev_tables& tb, int32_t b, int32_t hk,
                                                int32_t Hkv, int32_t Tcap, int32_t t) {
  if (!tb.tail_pages) return ((int64_t)b * Hkv + hk) * Tcap + t;
  int32_t pg = tb.tail_pages[(int64_t)b * tb.pages_per_branch + (t >> tb.page_shift)];
  pg = min(max(pg, 0), tb.n_pages - 1);
  return ((((int64_t)pg * Hkv + hk)) << tb.page_shift) + (t & ((1 << tb.page_shift) - 1));
}

struct hpd_layout {
  hpd_config cfg;
  int32_t P = 0, n_docs = 0, B = 0, T = 0, n_seg = 0;
  int64_t n_prefix_tokens = 0, NP = 0, total_live = 0, total_units = 0;
  int32_t max_pos = 0;
  int32_t kernel_mode = 0;

  std::vector<int32_t> seg_off, seg_len, seg_pos0, seg_raw_off, raw_seg;
  std::vector<int32_t> doc_prompt, branch_doc, branch_base_pos, branch_len;
  std::vector<int32_t> prompt_doc_ptr, prompt_branch_ptr;
  // paper-literal mask: document blocks per prompt, per-step prompt units
  std::vector<int32_t> pblk_ptr, pblk, punit_ptr, punit_desc, pmax_rows;
  int32_t max_prompt_branches = 0;
  std::vector<int32_t> skel_pos, skel_off, skel_seg_off, skel_cum;
  std::vector<int32_t> funit_desc;  // prefix-token attention units, heaviest first
  std::vector<int32_t> fblk;        // literal mask: header and document blocks of every prompt
  std::vector<int32_t> fill_blk;    // owner and first raw token of every 32-slot block of the prefix pools
  int32_t fmax_rows = 0;            // most tokens of any segment
  int32_t fmax_list_blocks = 0;     // literal mask: most list blocks any segment sees in full
  std::vector<int32_t> live_ptr, live_branch, doc_live_ptr, unit_ptr, unit_doc, unit_desc;
  std::vector<int32_t> max_rows;  // [T] largest number of live branches of any document at step t
  std::vector<float> rope;        // host copy of the (cos, sin) table

  // device-side pruning: state built by dynamic_prune_kernel (one allocation, d_dyn)
  std::vector<int32_t> doc_branch_ptr;  // [n_docs+1]
  std::vector<int32_t> dyn_fixed;       // [units][8] per-unit constants of the descriptors, heaviest first (uploaded with the tables)
  int32_t max_doc_branches = 0;
  void* d_dyn = nullptr;
  int32_t *dyn_live = nullptr, *dyn_n_live = nullptr, *dyn_desc = nullptr, *dyn_fixed_dev = nullptr,
          *dyn_len = nullptr;  // literal mask: tokens every branch has reached (the step budget while it runs)
  int32_t dyn_next_step = 0;  // the step the device state describes (host-side counter)

  bool on_device = false;
  int device = -1;
  int n_cus = 256;  // compute units of that device
  void* d_ints = nullptr;
  void* d_rope = nullptr;
  hpd_dev_tables dev{};
};

struct hpd_shape {
  int32_t Hq, Hkv, D, T, P, n_docs;
  int64_t NP;
};

// Launchers (hpd_kernels.hip).  Each returns a hipError_t from the launch.
hipError_t hpd_launch_prefix_fill(const hpd_layout* L, const void* k_raw, const void* v_raw,
                                  void* k_prefix, void* v_prefix, hipStream_t s);
hipError_t hpd_launch_positions(const hpd_layout* L, int32_t step, int32_t* pos_out, hipStream_t s);
hipError_t hpd_launch_append(const hpd_layout* L, int32_t step, const void* k_new, const void* v_new,
                             void* k_tail, void* v_tail, int64_t* slot_out, hipStream_t s);
hipError_t hpd_launch_attention_generic(const hpd_layout* L, int32_t step, const void* q,
                                        const void* k_prefix, const void* v_prefix,
                                        const void* k_tail, const void* v_tail, void* out,
                                        hipStream_t s);
hipError_t hpd_launch_expand_mask(const int32_t* d_desc, int32_t S, int32_t paper, uint8_t* mask_out,
                                  hipStream_t s);

// desc[S][4] = (kind 0 prompt / 1 attribute / 2 value, attribute index, k, position ID)
hipError_t hpd_launch_finetune_mask(const int32_t* d_desc, int32_t S, int32_t* pos_out, uint8_t* mask_out,
                                    hipStream_t s);

// most keys any row of the step has in the generic kernel (it keeps one score per key in LDS)
int64_t hpd_generic_max_keys(const hpd_layout* L, int32_t step);

bool hpd_stream_supported(const hpd_layout* L);
hipError_t hpd_launch_prefill_stream(const hpd_layout* L, const void* q, const void* k_prefix,
                                     const void* v_prefix, void* out, hipStream_t s);
hipError_t hpd_launch_prefill_generic(const hpd_layout* L, const void* q, const void* k_prefix,
                                      const void* v_prefix, void* out, hipStream_t s);
// k_new / v_new may be null: then the newest token is read from the tail pool like the others
// dynamic: work lists and live list from the device-side pruning state instead of the tables
// built from branch_len
hipError_t hpd_launch_attention_stream(const hpd_layout* L, int32_t step, const void* q,
                                       const void* k_prefix, const void* v_prefix, void* k_tail,
                                       void* v_tail, const void* k_new, const void* v_new, void* out,
                                       hipStream_t s, bool dynamic = false);
hipError_t hpd_launch_dynamic_prune(const hpd_layout* L, int32_t next_step, const uint8_t* finished,
                                    hipStream_t s);
// Address (on `device`) and size of the library's file-scope scratch array, resolved on first
// use per device.  Allocates nothing.
hipError_t hpd_dynamic_scratch(int device, void** ptr, size_t* bytes);
