/*
 * hpd.h - C ABI of the MI355X (gfx950) library for Hyper-Parallel Decoding (HPD)
 * masked decode attention.
 *
 * One decode step of HPD (paper Section 4.3.3) feeds only the newest token of every
 * unfinished attribute value ("branch").  Each of those queries is RoPE-rotated at a
 * manipulated position ID (Section 4.3.1, Appendix A.1), attends to the shared
 * instruction/attribute header, to its own document and to its own earlier value
 * tokens (Section 4.3.2, with the per-document restriction that makes Eq. 3's
 * conditional independence exact), and its new K/V is appended to the cache
 * (Section 4.3.2: the cache only grows at its end).  Documents are stacked in one
 * prompt (Section 4.3.5), prompts are batched (Section 4.3.6), finished values are
 * pruned (Section 4.3.4).
 *
 * Conventions
 *   - "host" / "device" on every pointer says where the memory lives.  Device memory
 *     is caller-owned (e.g. a torch tensor's data_ptr); the library allocates only the
 *     small tables inside hpd_layout.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Per-step
 *     calls only enqueue work; they never synchronise or allocate (the two exceptions say
 *     so where they are declared: the first hpd_dynamic_begin of a layout, hpd_dynamic_read),
 *     and they enqueue kernels only (no memset or copy nodes): a decode pass may be captured
 *     in a HIP graph and replayed.  The host-side step counter of the hpd_dynamic_* calls
 *     advances at capture time, not at replay.
 *   - Every function returns HPD_OK (0) or a negative HPD_E_* code; on error no output
 *     is written.  No exception or abort crosses this boundary.
 *   - Global ids: prompts p in [0,P); documents d in CSR order (p, j); branches b in
 *     CSR order (p, j, n), which is Algorithm 1's d[jN+i] order.
 *   - Steps are 0-based decode steps t in [0, max_new); of the paper's step t = 1 (the
 *     prefill) the library has the attention over header and documents
 *     (hpd_prefill_attention) and the filling of the prefix pools (hpd_prefix_fill).
 *   - Live rows: at step t the rows of q / k_new / v_new / out / pos_out / slot_out
 *     are the branches {b : branch_len[b] > t} in ascending b (the pruned input of
 *     Section 4.3.4).
 *
 * KV pool layouts (element type = cfg.dtype; Hkv = n_kv_heads, D = head_dim,
 * T = max_new, B = number of branches):
 *   k_prefix : [Hkv][NP][D]          NP = HPD_Q_COUNTS.n_prefix_slots.  A segment
 *                                    (header of a prompt, a document, or - under
 *                                    HPD_MASK_PAPER - the attribute names of a prompt) occupies slots
 *                                    [seg_off, seg_off + seg_len); seg_off is a multiple
 *                                    of HPD_KEY_BLOCK.  K is stored already rotated.
 *                                    (HPD_BF16: see "element format" below.)
 *   v_prefix : [Hkv][NP/8][D][8]     same slots; 8 consecutive keys are interleaved so
 *                                    that the P.V contraction reads 8 keys of one
 *                                    channel with one 16-byte load.
 *   k_tail   : [B][Hkv][T][D]        slot b*T + t holds the rotated key of branch b's
 *   v_tail   : [B][Hkv][T][D]        t-th value token (Algorithm 1's values[j,i,t]).
 *   Element format of the four pools under HPD_BF16: an element holds a bf16 value - the
 *   rotated key rounded to bf16 (the precision of a bf16 cache), the value as the caller gave
 *   it - written in IEEE half format: the same 2 bytes, exact for 2^-14 <= |x| <= 65504,
 *   within 2^-25 below, saturating above.  Both products of the attention then take their other
 *   operand (query, softmax weights) with 11 significant bits in one pass of the
 *   half-precision matrix instruction.  A scaled rotated query above 65504 in magnitude is not
 *   supported (it would overflow the exponential as well).
 *   hpd_prefix_fill zeroes the V padding slots between a segment's end and the next
 *   multiple of HPD_KEY_BLOCK; K padding and unwritten tail slots may hold anything
 *   (including NaN patterns).  HPD_Q_POOL_BYTES reports the four sizes.
 *   With a page table (hpd_set_tail_pages) the tail pools are [n_pages][Hkv][page_size][D]
 *   instead and slot page(b, t / page_size) * page_size + t % page_size holds that token.
 */
#ifndef HPD_H
#define HPD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define HPD_KEY_BLOCK 32 /* alignment (in key slots) of every prefix segment */

enum hpd_status {
  HPD_OK = 0,
  HPD_E_INVALID = -1,     /* bad shapes, non-monotone CSR, lengths out of range, null pointers */
  HPD_E_OVERFLOW = -2,    /* a position or an offset does not fit its integer type */
  HPD_E_UNSUPPORTED = -3, /* dtype / head_dim / mode the kernels do not cover */
  HPD_E_HIP = -4,         /* HIP runtime error; hpd_status_string(HPD_E_HIP) gives the text */
  HPD_E_NOMEM = -5,
  HPD_E_CAPACITY = -6     /* the layout needs more than the fixed scratch memory of an
                             allocation-free call (hpd_dynamic_begin_static) */
};

enum hpd_dtype { HPD_F32 = 0, HPD_BF16 = 1 };
enum hpd_pos_mode {
  HPD_POS_CONTIG = 0,   /* every document restarts right after the header; a branch
                           continues from the end of its own document */
  HPD_POS_PAPER_GAP = 1 /* Algorithm 2: ordinary positions over header + documents,
                           then a gap of max_new after every attribute */
};
enum hpd_mask_mode {
  HPD_MASK_BLOCK = 0, /* header + own document + own branch */
  HPD_MASK_PAPER = 1  /* Section 4.3.2 taken literally: one causal order by position ID over
                         the whole stacked prompt.  A branch sees the header, every document
                         of its prompt, the tokens of every earlier branch of the prompt (in
                         the (document, attribute) order) up to the current step, finished
                         branches included, and its own tokens.  Needs HPD_POS_PAPER_GAP
                         (positions that restart per document do not order a prompt).
                         The skeleton (attribute-name) tokens a_1..a_N of Section 4.3.1's input
                         s = cat(p, a_1:N) are cache entries in this mode: per prompt a third
                         kind of prefix segment (after the documents in hpd_prefix_fill's
                         order, attribute by attribute, at Algorithm 2's positions), of which
                         a branch sees the names up to its own.  Under HPD_MASK_BLOCK they only
                         shape the position IDs. */
};
enum hpd_out_dtype {
  HPD_OUT_SAME = 0, /* `out` has the element type of the inputs */
  HPD_OUT_F32 = 1   /* `out` is fp32 whatever the inputs are: bf16 cannot resolve 2e-2 x RMS
                       on the largest outputs (half an ulp at |o| = 8 x RMS is 3e-2 x RMS) */
};
enum hpd_flags {
  HPD_FLAG_HOST_ONLY = 1 /* build host tables only (no HIP call); only hpd_layout_query
                            and hpd_layout_free may then be used on the layout */
};

typedef struct hpd_config {
  int32_t n_q_heads;  /* Hq */
  int32_t n_kv_heads; /* Hkv, divides Hq; query head h uses kv head h / (Hq/Hkv) */
  int32_t head_dim;   /* D: multiple of 8, <= 256; the MFMA path needs D = 128 */
  int32_t dtype;      /* hpd_dtype of q, k, v, out and of the pools */
  double rope_base;   /* rotate-half RoPE, theta_i = base^(-2i/D), no scaling */
  int32_t max_new;    /* T = K_max (Section 4.3.1): tail capacity and number of steps */
  int32_t pos_mode;   /* hpd_pos_mode */
  int32_t mask_mode;  /* hpd_mask_mode */
  int32_t flags;      /* hpd_flags */
  int32_t out_dtype;  /* hpd_out_dtype */
} hpd_config;

typedef struct hpd_layout hpd_layout; /* opaque; created and destroyed by the library */

/* hpd_layout_query selectors.  All outputs are host arrays. */
enum hpd_query {
  HPD_Q_COUNTS = 0,      /* int64[HPD_N_COUNTS], see hpd_count */
  HPD_Q_POOL_BYTES = 1,  /* int64[4]: bytes of k_prefix, v_prefix, k_tail, v_tail */
  HPD_Q_N_LIVE = 2,      /* int32[T]: live branches per step */
  HPD_Q_LIVE_BRANCH = 3, /* int32[total_live]: live lists of steps 0..T-1 back to back */
  HPD_Q_BRANCH_BASE_POS = 4, /* int32[B]: position of the token a branch continues from */
  HPD_Q_BRANCH_DOC = 5,  /* int32[B] */
  /* segments: P headers, then n_docs documents, then - under HPD_MASK_PAPER only - P skeleton
     segments (n_seg = P + n_docs [+ P]) */
  HPD_Q_SEG_OFF = 6,     /* int32[n_seg]: first pool slot */
  HPD_Q_SEG_LEN = 7,     /* int32[n_seg] */
  HPD_Q_SEG_POS0 = 8,    /* int32[n_seg]: position ID of the segment's first token (-1 for a
                            skeleton segment: its positions have gaps) */
  HPD_Q_SEG_RAW_OFF = 9, /* int32[n_seg]: first token in hpd_prefix_fill's input order */
  HPD_Q_N_UNITS = 10     /* int32[T]: documents (prompts, under HPD_MASK_PAPER) with at least one
                            live branch per step: the work units of the attention kernel */
};
enum hpd_count {
  HPD_C_N_PROMPTS = 0,
  HPD_C_N_DOCS = 1,
  HPD_C_N_BRANCHES = 2,
  HPD_C_N_PREFIX_TOKENS = 3, /* header + document (+ skeleton) tokens, unpadded */
  HPD_C_N_PREFIX_SLOTS = 4,  /* NP */
  HPD_C_N_TAIL_SLOTS = 5,    /* B * T */
  HPD_C_MAX_POS = 6,         /* largest position ID any token can take within the step budget
                                (base position + max_new, whatever branch_len says: the
                                hpd_dynamic_* calls may decode a branch up to step max_new - 1) */
  HPD_C_TOTAL_LIVE = 7,      /* sum over steps of live branches = sum of branch_len */
  HPD_N_COUNTS = 8
};

/*
 * hpd_build_layout - Sections 4.3.1, 4.3.4-4.3.6, Appendix A.1.
 * Validates the batch description, builds the CSR tables (segments, branches, per-step
 * live lists, per-step work lists, RoPE table) and, unless HPD_FLAG_HOST_ONLY, uploads
 * them (synchronises `stream` once).  All input arrays are host memory and are copied.
 *   header_len [P]        H_p >= 0
 *   doc_ptr    [P+1]      CSR prompts -> documents, doc_ptr[0] = 0, non-decreasing
 *   doc_len    [n_docs]   L_d >= 1
 *   branch_ptr [n_docs+1] CSR documents -> branches, non-decreasing
 *   branch_len [B] or NULL  number of steps branch b is decoded, in [1, T]; NULL = all T
 *   attr_len   [B] or NULL  A_b >= 1, skeleton attribute lengths (tokens of the attribute's
 *                           name in the output template); required for HPD_POS_PAPER_GAP,
 *                           ignored otherwise
 * On success *out owns the layout (release with hpd_layout_free).
 */
int hpd_build_layout(const hpd_config* cfg, int32_t n_prompts, const int32_t* header_len,
                     const int32_t* doc_ptr, const int32_t* doc_len, const int32_t* branch_ptr,
                     const int32_t* branch_len, const int32_t* attr_len, void* stream,
                     hpd_layout** out);

void hpd_layout_free(hpd_layout* layout);

/* Copies one table to host memory.  `bytes` must be at least the table's size. */
int hpd_layout_query(const hpd_layout* layout, int32_t what, void* host_out, size_t bytes);

/*
 * hpd_prefix_fill - batched form of the append for the tokens that exist before
 * decoding starts (header and documents; the paper's prefill writes them).
 *   k_raw, v_raw : device [n_prefix_tokens][Hkv][D], un-rotated, token order = prompts in
 *                  order, each as [header | doc_0 | doc_1 | ...]; under HPD_MASK_PAPER
 *                  followed by the prompt's attribute names a_1 .. a_N (A_b tokens each, in
 *                  branch order).  n_prefix_tokens = HPD_Q_COUNTS[HPD_C_N_PREFIX_TOKENS].
 *   k_prefix, v_prefix : device pools (layouts above).  K is rotated at the token's
 *                  position ID (HPD_Q_SEG_POS0 + index in segment; attribute names at
 *                  Algorithm 2's positions) and stored.
 */
int hpd_prefix_fill(const hpd_layout* layout, const void* k_raw, const void* v_raw,
                    void* k_prefix, void* v_prefix, void* stream);

/*
 * hpd_rope_positions - Appendix A.1 ("value token k of attribute n gets
 * pos_id[end(a_n)] + k") and Section 4.3.3 (previous position + 1):
 *   pos_out[r] = base_pos[b_r] + 1 + step   for the r-th live branch b_r.
 *   pos_out    : device int32 [n_live(step)]
 *   n_live_out : host int32*, may be NULL
 */
int hpd_rope_positions(const hpd_layout* layout, int32_t step, int32_t* pos_out,
                       int32_t* n_live_out, void* stream);

/*
 * hpd_kv_append - Section 4.3.2 (new tokens are appended at the end of the cache).
 * Rotates the new key of every live branch at its position ID and stores key and value
 * at tail slot b*T + step.
 *   k_new, v_new : device [n_live(step)][Hkv][D], K un-rotated
 *   k_tail, v_tail : device tail pools
 *   slot_out : device int64 [n_live(step)] or NULL; receives b*T + step
 */
int hpd_kv_append(const hpd_layout* layout, int32_t step, const void* k_new, const void* v_new,
                  void* k_tail, void* v_tail, int64_t* slot_out, void* stream);

/*
 * hpd_decode_attention - Sections 4.3.2-4.3.3.  For every live branch b and query head h:
 *   out = softmax( RoPE(q, pos) . K^T / sqrt(D) ) V  over the keys
 *   header(prompt of b)  ++  document(b)  ++  tail slots 0..step of b
 * (the block form of the position-ordered causal mask; under HPD_MASK_PAPER: header ++ every
 * document of the prompt ++ the attribute names up to b's ++ tail slots 0..min(step, len-1)
 * of every branch of the prompt up to b).  Call after hpd_kv_append of the same step: a query attends to its own token.
 *   q   : device [n_live(step)][Hq][D], un-rotated
 *   out : device [n_live(step)][Hq][D]
 */
int hpd_decode_attention(const hpd_layout* layout, int32_t step, const void* q,
                         const void* k_prefix, const void* v_prefix, const void* k_tail,
                         const void* v_tail, void* out, void* stream);

/*
 * hpd_decode_step - hpd_kv_append followed by hpd_decode_attention of the same step with
 * fewer launches; results equal the two-call sequence.
 */
int hpd_decode_step(const hpd_layout* layout, int32_t step, const void* q, const void* k_new,
                    const void* v_new, const void* k_prefix, const void* v_prefix, void* k_tail,
                    void* v_tail, void* out, void* stream);

/*
 * hpd_prefill_attention - Section 4.3.2, "First Inference Step": the attention of the pass
 * that feeds the whole input once.  Every prefix token is a query at its own position ID.
 * Under HPD_MASK_BLOCK a header token attends to the header up to itself, a document token to
 * the whole header and to its own document up to itself.  Under HPD_MASK_PAPER header,
 * documents and attribute names of a prompt are one causal sequence, as the section has it: a
 * document token also sees the earlier documents, a name token everything before it; the rows
 * of the names' last tokens are the ones whose outputs start the branches.  Call after
 * hpd_prefix_fill (the keys are read from the prefix pools).
 *   q   : device [n_prefix_tokens][Hq][D], un-rotated, token order of hpd_prefix_fill
 *   out : device [n_prefix_tokens][Hq][D] (element type per hpd_config.out_dtype)
 */
int hpd_prefill_attention(const hpd_layout* layout, const void* q, const void* k_prefix,
                          const void* v_prefix, void* out, void* stream);

/*
 * hpd_expand_mask - debugging export of the mask of Section 4.3.2 as the library
 * understands it.  Memory order of prompt `prompt` after step `step_hi`:
 *   [header | doc_0 | ... | step-0 live branches | step-1 live branches | ... ].
 *   mask_out : device uint8 [S][S] row-major (query row, key column), S = *s_out
 *   s_out    : host int32*, receives S; if mask_out is NULL only S is reported.
 * Allocates and frees a small descriptor table and synchronises: test use only.
 */
int hpd_expand_mask(const hpd_layout* layout, int32_t prompt, int32_t step_hi, uint8_t* mask_out,
                    int32_t* s_out, void* stream);

/*
 * Device-side pruning - Section 4.3.4 ("Early Stopping") without a host round trip.  The
 * calls above take the liveness of every step from branch_len, which a serving loop does not
 * know in advance: it learns that a value has ended from the token it has just sampled.  With
 * the calls below the live list of the next step and the work lists of the attention kernel
 * are built on the GPU from a per-row "finished" flag; the host never reads them back (its
 * launches cover every document; a document without live branches costs a workgroup that
 * exits at its descriptor; under HPD_MASK_PAPER the units are prompts, and the device also
 * keeps how many tokens every branch that has left had reached, since the later branches
 * still see them).  The streaming kernel's shapes only (bf16, head_dim 128, at most 8 query
 * heads per kv head; under HPD_MASK_PAPER at most 256 branches per prompt), at most 65536
 * branches; else HPD_E_UNSUPPORTED.
 *
 * hpd_dynamic_begin - allocates the device-side state on first use (it lives as long as the
 *   layout) and resets it: every branch live.  branch_len is ignored by the dynamic calls.
 * hpd_dynamic_prune - `finished`: device uint8 [n_live] in the row order of the step just
 *   taken; non-zero = that branch is not decoded any further.  Builds the next step's state.
 * hpd_dynamic_step  - hpd_decode_step of step `step` for the rows of the current live list
 *   (the same kernel; a document's rows are split over workgroups by its full branch count,
 *   the live count being unknown to the host, so sums may be grouped differently and results
 *   agree with hpd_decode_step to rounding, not always bit for bit):
 *   rows r of q / k_new / v_new / out are the live branches in ascending b, r < n_live (the
 *   kernels touch no row beyond; buffers need n_live rows, B rows always suffice).
 * hpd_dynamic_state - device addresses of the live list (int32 [B], first n_live valid) and of
 *   n_live (int32 [1]) so that the caller's own kernels can gather and scatter by them.
 * hpd_dynamic_read  - copies n_live and the first min(n_live, capacity) entries of the live
 *   list to host memory; synchronises the stream: for tests and debugging.
 * The first four only enqueue on `stream` (hpd_dynamic_begin allocates on its first call).
 */
int hpd_dynamic_begin(hpd_layout* layout, void* stream);

/*
 * hpd_dynamic_begin_static - hpd_dynamic_begin for callers that cannot allocate device memory
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).  Same
 * effect - every branch live, hpd_dynamic_prune / _step / _state / _read then work on this state -
 * but the state lives in a file-scope device array of HPD_DYNAMIC_STATIC_MAX_BYTES that every
 * GPU the library runs on holds until the process ends, and the call allocates and frees
 * nothing, on the device or on the host: it only enqueues the kernel that writes the state
 * (the first call on a device also looks the array's address up).
 *   - The state needs 4 * (8 * n_docs + B + 20) bytes (HPD_MASK_PAPER: 4 * (16 * P + 2 * B + 20));
 *     a layout that needs more than HPD_DYNAMIC_STATIC_MAX_BYTES gets HPD_E_CAPACITY and nothing
 *     is enqueued.
 *   - One state per GPU: the array is shared by every layout and every call on that GPU and
 *     keeps the last call's contents (the kernel rewrites every word it later reads; nothing
 *     has to be cleared).  A second hpd_dynamic_begin_static on the same GPU - for this or
 *     another layout - replaces the state of the first; calls whose work overlaps on one GPU
 *     (different streams, different threads) race.  hpd_dynamic_begin switches a layout back to
 *     a state of its own.
 */
#define HPD_DYNAMIC_STATIC_MAX_BYTES (1 << 20)
int hpd_dynamic_begin_static(hpd_layout* layout, void* stream);
int hpd_dynamic_prune(hpd_layout* layout, const uint8_t* finished, void* stream);
int hpd_dynamic_step(const hpd_layout* layout, int32_t step, const void* q, const void* k_new,
                     const void* v_new, const void* k_prefix, const void* v_prefix, void* k_tail,
                     void* v_tail, void* out, void* stream);
int hpd_dynamic_state(const hpd_layout* layout, const int32_t** live_branch, const int32_t** n_live);
int hpd_dynamic_read(const hpd_layout* layout, int32_t* live_host, int32_t capacity, int32_t* n_live_host,
                     void* stream);

/*
 * hpd_set_tail_pages - paged tail pools (the paper's Limitations paragraph names paged
 * attention as an untried combination).  B*T tail slots are reserved for values that mostly
 * end early (Section 4.3.4); with a page table the pools hold n_pages pages of page_size
 * consecutive steps of one branch, [n_pages][Hkv][page_size][D], and the pages of a pruned
 * branch can be handed to another one.
 *   page_size  : 8, 16, 32, ... (a power of two, at least 8); 0 switches paging off again
 *   n_pages    : pages the caller's tail pools hold (at least 1)
 *   page_table : device int32 [B][ceil(T / page_size)], owned and updated by the caller (on the
 *                stream of the calls that read it).  Entry (b, i) must name b's page for steps
 *                i*page_size .. (i+1)*page_size - 1 before the first call for such a step in
 *                which b is live, and must not change while b is live; entries of pages a branch
 *                has not reached, and those of branches that are no longer live, are not read.
 *                (Under HPD_MASK_PAPER the later branches of a prompt keep reading the tokens of
 *                a branch that has left: its pages stay until the prompt's last branch has left.)
 *                The kernels clamp an entry to [0, n_pages) instead of trusting it.
 * Affects hpd_kv_append (slot_out reports page * page_size + t % page_size), hpd_decode_attention,
 * hpd_decode_step and hpd_dynamic_step of this layout from the next call on, and the tail
 * sizes HPD_Q_POOL_BYTES reports.  Host-side only: nothing is enqueued.
 */
int hpd_set_tail_pages(hpd_layout* layout, int32_t page_size, int32_t n_pages, const int32_t* page_table);

/*
 * hpd_finetune_mask - Section 4.4 ("Fine-tuning and Distillation"), Appendix A.1.  Position IDs
 * and attention mask of one training sequence in the regular token order
 *   s_train = cat(p, a_1, v_1, ..., a_N, v_N):
 * the attributes keep Algorithm 2's positions (a gap of k_max after every attribute), value
 * token k (1-based) of attribute n sits at pos_id[end(a_n)] + k; the mask is the causal mask
 * minus (i) v_{n,k} -> v_{n',k'} for n' < n, k' > k and (ii) attribute token -> any value
 * token: what a token could see while being decoded in parallel.
 *   prompt_len >= 0; attr_len [n_attr] >= 1, value_len [n_attr] in [0, k_max]: host arrays
 *   pos_out  : device int32 [S] or NULL
 *   mask_out : device uint8 [S][S] row-major (query row, key column) or NULL
 *   s_out    : host int64*, receives S = prompt_len + sum(attr_len) + sum(value_len)
 * Integer work only.  Allocates and frees a token table of 16 S bytes and synchronises the
 * stream: a data-preparation call, not a per-step one.  HPD_E_INVALID for lengths out of
 * range, HPD_E_OVERFLOW if S exceeds 46000 or a position 2^30.
 */
int hpd_finetune_mask(int32_t prompt_len, int32_t n_attr, const int32_t* attr_len,
                      const int32_t* value_len, int32_t k_max, int32_t* pos_out, uint8_t* mask_out,
                      int64_t* s_out, void* stream);

/* Selects the attention kernel: 0 = automatic, 1 = generic wave-reduction kernel for
 * everything, 2 = LDS-streaming MFMA kernel, workgroup shape chosen per launch (decode: wide
 * or narrow; hpd_prefill_attention: the dense shape), 3 / 4 = the same with the wide / the
 * narrow workgroup shape forced for both calls (2..4 return HPD_E_UNSUPPORTED if
 * the shape does not allow the kernel: it needs bf16, head_dim 128 and a group size of 1,
 * 2, 4 or 8, and under HPD_MASK_PAPER at most 256 branches and 512 blocks of 32 keys per
 * prompt). */
int hpd_set_kernel_mode(hpd_layout* layout, int32_t mode);

const char* hpd_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* HPD_H */
