// Host side of the HPD library: validation, layout tables and the C ABI.
// The layout follows the paper's problem statement: a shared header per prompt,
// J stacked documents (Section 4.3.5), N attribute branches per document decoded for at
// most K_max steps (Sections 4.3.1, 4.3.4), prompts batched (Section 4.3.6).
#include <algorithm>
#include <cmath>
#include <cstring>
#include <limits>
#include <new>
#include <numeric>
#include <string>

#include "hpd_internal.h"

namespace {

thread_local std::string g_hip_text = "no HIP error recorded";

int hip_fail(hipError_t e) {
  g_hip_text = std::string("HIP error: ") + hipGetErrorString(e);
  return HPD_E_HIP;
}

#define HPD_HIP(expr)                        \
  do {                                       \
    hipError_t e_ = (expr);                  \
    if (e_ != hipSuccess) return hip_fail(e_); \
  } while (0)

inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

size_t elem_bytes(const hpd_config& c) { return c.dtype == HPD_F32 ? 4 : 2; }
bool paper_mode(const hpd_layout* L) { return L->cfg.mask_mode == HPD_MASK_PAPER; }

int validate_config(const hpd_config* c) {
  if (!c) return HPD_E_INVALID;
  if (c->n_q_heads < 1 || c->n_kv_heads < 1 || c->n_q_heads % c->n_kv_heads != 0) return HPD_E_INVALID;
  if (c->head_dim < 2 || (c->head_dim & 1)) return HPD_E_INVALID;
  if (c->max_new < 1) return HPD_E_INVALID;
  if (!(c->rope_base > 1.0) || !std::isfinite(c->rope_base)) return HPD_E_INVALID;
  if (c->dtype != HPD_F32 && c->dtype != HPD_BF16) return HPD_E_UNSUPPORTED;
  if (c->head_dim % 8 != 0 || c->head_dim > 256) return HPD_E_UNSUPPORTED;
  if (c->pos_mode != HPD_POS_CONTIG && c->pos_mode != HPD_POS_PAPER_GAP) return HPD_E_UNSUPPORTED;
  if (c->mask_mode != HPD_MASK_BLOCK && c->mask_mode != HPD_MASK_PAPER) return HPD_E_UNSUPPORTED;
  if (c->mask_mode == HPD_MASK_PAPER && c->pos_mode != HPD_POS_PAPER_GAP) return HPD_E_INVALID;
  if (c->flags & ~HPD_FLAG_HOST_ONLY) return HPD_E_INVALID;
  if (c->out_dtype != HPD_OUT_SAME && c->out_dtype != HPD_OUT_F32) return HPD_E_UNSUPPORTED;
  return HPD_OK;
}

// Copies a host vector into the device int arena and returns its device address.
struct IntArena {
  std::vector<int32_t> host;
  std::vector<size_t> offs;
  size_t add(const std::vector<int32_t>& v) {
    size_t o = host.size();
    host.insert(host.end(), v.begin(), v.end());
    // keep every table 16-byte aligned
    while (host.size() % 4) host.push_back(0);
    if (v.empty()) { host.insert(host.end(), 4, 0); }
    return o;
  }
};

}  // namespace

extern "C" {

const char* hpd_status_string(int status) {
  switch (status) {
    case HPD_OK: return "ok";
    case HPD_E_INVALID: return "invalid argument";
    case HPD_E_OVERFLOW: return "integer overflow in positions or offsets";
    case HPD_E_UNSUPPORTED: return "unsupported dtype, head_dim or mode";
    case HPD_E_HIP: return g_hip_text.c_str();
    case HPD_E_NOMEM: return "out of host memory";
    case HPD_E_CAPACITY: return "the layout exceeds the fixed scratch memory of the allocation-free call";
    default: return "unknown status";
  }
}

int hpd_build_layout(const hpd_config* cfg, int32_t n_prompts, const int32_t* header_len,
                     const int32_t* doc_ptr, const int32_t* doc_len, const int32_t* branch_ptr,
                     const int32_t* branch_len, const int32_t* attr_len, void* stream,
                     hpd_layout** out) {
  if (!out) return HPD_E_INVALID;
  int rc = validate_config(cfg);
  if (rc != HPD_OK) return rc;
  if (n_prompts < 1 || !header_len || !doc_ptr || !doc_len || !branch_ptr) return HPD_E_INVALID;
  if (cfg->pos_mode == HPD_POS_PAPER_GAP && !attr_len) return HPD_E_INVALID;
  const int32_t P = n_prompts;
  const int32_t T = cfg->max_new;
  if (doc_ptr[0] != 0) return HPD_E_INVALID;
  for (int32_t p = 0; p < P; ++p) {
    if (header_len[p] < 0) return HPD_E_INVALID;
    if (doc_ptr[p + 1] < doc_ptr[p]) return HPD_E_INVALID;
  }
  const int32_t n_docs = doc_ptr[P];
  if (branch_ptr[0] != 0) return HPD_E_INVALID;
  for (int32_t d = 0; d < n_docs; ++d) {
    if (doc_len[d] < 1) return HPD_E_INVALID;
    if (branch_ptr[d + 1] < branch_ptr[d]) return HPD_E_INVALID;
  }
  const int32_t B = branch_ptr[n_docs];
  for (int32_t b = 0; b < B; ++b) {
    if (branch_len && (branch_len[b] < 1 || branch_len[b] > T)) return HPD_E_INVALID;
    if (cfg->pos_mode == HPD_POS_PAPER_GAP && attr_len[b] < 1) return HPD_E_INVALID;
  }
  if ((int64_t)B * T > (int64_t)1 << 40) return HPD_E_OVERFLOW;

  hpd_layout* L = new (std::nothrow) hpd_layout();
  if (!L) return HPD_E_NOMEM;
  try {
    L->cfg = *cfg;
    const bool paper = cfg->mask_mode == HPD_MASK_PAPER;
    // (under the literal mask every prompt has a third kind of segment: its attribute names)
    L->P = P; L->n_docs = n_docs; L->B = B; L->T = T; L->n_seg = P + n_docs + (paper ? P : 0);
    const int32_t n_seg = L->n_seg;
    L->seg_off.assign(n_seg, 0); L->seg_len.assign(n_seg, 0); L->seg_pos0.assign(n_seg, 0);
    L->seg_raw_off.assign(n_seg + 1, 0); L->raw_seg.assign(n_seg, 0);
    L->doc_prompt.assign(n_docs, 0);
    L->branch_doc.assign(B, 0); L->branch_base_pos.assign(B, 0); L->branch_len.assign(B, T);
    if (branch_len) std::copy(branch_len, branch_len + B, L->branch_len.begin());
    if (paper) { L->skel_cum.assign(B, 0); L->skel_seg_off.assign(P, 0); }
    L->prompt_doc_ptr.assign(doc_ptr, doc_ptr + P + 1);
    L->doc_branch_ptr.assign(branch_ptr, branch_ptr + n_docs + 1);
    for (int32_t d = 0; d < n_docs; ++d)
      L->max_doc_branches = std::max(L->max_doc_branches, branch_ptr[d + 1] - branch_ptr[d]);
    L->prompt_branch_ptr.resize(P + 1);
    for (int32_t p = 0; p <= P; ++p) L->prompt_branch_ptr[p] = branch_ptr[doc_ptr[p]];

    // ---- segments: pool slots (each segment starts on a HPD_KEY_BLOCK boundary), raw
    //      token order [header | doc_0 | doc_1 ...] per prompt, position of first token
    int64_t slot = 0, raw = 0, max_pos = 0;
    int32_t ri = 0;
    for (int32_t p = 0; p < P; ++p) {
      const int64_t H = header_len[p];
      L->seg_off[p] = (int32_t)slot; L->seg_len[p] = (int32_t)H; L->seg_pos0[p] = 0;
      L->seg_raw_off[ri] = (int32_t)raw; L->raw_seg[ri] = p; ++ri;
      slot += round_up(H, HPD_KEY_BLOCK); raw += H;
      int64_t run_pos = H;  // paper-gap mode: ordinary increasing positions across documents
      for (int32_t d = doc_ptr[p]; d < doc_ptr[p + 1]; ++d) {
        const int64_t Ld = doc_len[d];
        const int32_t sid = P + d;
        L->doc_prompt[d] = p;
        L->seg_off[sid] = (int32_t)slot; L->seg_len[sid] = (int32_t)Ld;
        const int64_t pos0 = (cfg->pos_mode == HPD_POS_CONTIG) ? H : run_pos;
        L->seg_pos0[sid] = (int32_t)pos0;
        L->seg_raw_off[ri] = (int32_t)raw; L->raw_seg[ri] = sid; ++ri;
        slot += round_up(Ld, HPD_KEY_BLOCK); raw += Ld; run_pos += Ld;
        max_pos = std::max(max_pos, pos0 + Ld - 1);
        if (slot > std::numeric_limits<int32_t>::max() - 4096 || run_pos > (1 << 30)) {
          delete L; return HPD_E_OVERFLOW;
        }
      }
      // ---- branches of this prompt: base position = position of the token they continue from
      if (cfg->pos_mode == HPD_POS_CONTIG) {
        for (int32_t d = doc_ptr[p]; d < doc_ptr[p + 1]; ++d)
          for (int32_t b = branch_ptr[d]; b < branch_ptr[d + 1]; ++b) {
            L->branch_doc[b] = d;
            L->branch_base_pos[b] = (int32_t)(H + doc_len[d] - 1);
          }
      } else {
        // Algorithm 2 over s = cat(prompt, a_1..a_N): attribute n keeps its ordinary
        // position plus n*K_max; a branch continues from its attribute's last token.
        int64_t idx = run_pos;  // index in s of the next skeleton token
        int64_t offset = 0;
        int32_t cum = 0;
        if (paper) L->skel_off.push_back((int32_t)L->skel_pos.size());
        for (int32_t d = doc_ptr[p]; d < doc_ptr[p + 1]; ++d)
          for (int32_t b = branch_ptr[d]; b < branch_ptr[d + 1]; ++b) {
            L->branch_doc[b] = d;
            const int64_t end = idx + attr_len[b] - 1;
            const int64_t bp = end + offset;
            if (bp + T > (1 << 30)) { delete L; return HPD_E_OVERFLOW; }
            L->branch_base_pos[b] = (int32_t)bp;
            if (paper) {
              for (int64_t i = idx; i <= end; ++i) L->skel_pos.push_back((int32_t)(i + offset));
              cum += attr_len[b];
              L->skel_cum[b] = cum;
            }
            idx = end + 1;
            offset += T;
          }
        if (paper) {
          // the skeleton segment of the prompt: after its documents in the input order
          const int32_t sid = P + n_docs + p;
          L->seg_off[sid] = (int32_t)slot; L->seg_len[sid] = cum; L->seg_pos0[sid] = -1;
          L->skel_seg_off[p] = (int32_t)slot;
          L->seg_raw_off[ri] = (int32_t)raw; L->raw_seg[ri] = sid; ++ri;
          slot += round_up(cum, HPD_KEY_BLOCK); raw += cum;
          if (slot > std::numeric_limits<int32_t>::max() - 4096) { delete L; return HPD_E_OVERFLOW; }
        }
      }
    }
    if (paper) L->skel_off.push_back((int32_t)L->skel_pos.size());
    L->seg_raw_off[n_seg] = (int32_t)raw;
    L->n_prefix_tokens = raw;
    // slack of 128 slots so that a kernel tile that starts inside the last segment never
    // leaves the pool
    L->NP = round_up(slot, HPD_KEY_BLOCK) + 128;
    // the RoPE table covers the whole step budget of every branch, not only the steps branch_len
    // announces: the device-side pruning calls ignore branch_len and keep a branch alive until
    // its flag comes, at most up to step T - 1 (position base + T)
    for (int32_t b = 0; b < B; ++b)
      max_pos = std::max<int64_t>(max_pos, (int64_t)L->branch_base_pos[b] + T);
    if (max_pos > (1 << 30)) { delete L; return HPD_E_OVERFLOW; }
    L->max_pos = (int32_t)max_pos;

    // ---- per-step live lists (Section 4.3.4: a finished value is no longer fed)
    L->live_ptr.assign(T + 1, 0);
    for (int32_t t = 0; t < T; ++t) {
      int32_t n = 0;
      for (int32_t b = 0; b < B; ++b) n += L->branch_len[b] > t;
      L->live_ptr[t + 1] = L->live_ptr[t] + n;
    }
    L->total_live = L->live_ptr[T];
    L->live_branch.assign((size_t)L->total_live, 0);
    L->doc_live_ptr.assign((size_t)T * (n_docs + 1), 0);
    L->unit_ptr.assign(T + 1, 0);
    L->max_rows.assign(T, 0);
    for (int32_t t = 0; t < T; ++t) {
      int32_t w = L->live_ptr[t];
      int32_t* dlp = &L->doc_live_ptr[(size_t)t * (n_docs + 1)];
      std::vector<int32_t> units;
      for (int32_t d = 0; d < n_docs; ++d) {
        dlp[d] = w - L->live_ptr[t];
        for (int32_t b = branch_ptr[d]; b < branch_ptr[d + 1]; ++b)
          if (L->branch_len[b] > t) L->live_branch[w++] = b;
        const int32_t nb = w - L->live_ptr[t] - dlp[d];
        if (nb > 0) units.push_back(d);
        L->max_rows[t] = std::max(L->max_rows[t], nb);
      }
      dlp[n_docs] = w - L->live_ptr[t];
      // heaviest documents first: cost ~ keys streamed
      std::stable_sort(units.begin(), units.end(), [&](int32_t a, int32_t b) {
        const int64_t ca = (int64_t)header_len[L->doc_prompt[a]] + doc_len[a];
        const int64_t cb = (int64_t)header_len[L->doc_prompt[b]] + doc_len[b];
        return ca > cb;
      });
      L->unit_doc.insert(L->unit_doc.end(), units.begin(), units.end());
      L->unit_ptr[t + 1] = (int32_t)L->unit_doc.size();
      for (int32_t d : units) {
        const int32_t p = L->doc_prompt[d];
        // all live branches of a document share one position in the contiguous mode
        int32_t pos = -1;
        if (cfg->pos_mode == HPD_POS_CONTIG) pos = L->seg_len[p] + L->seg_len[P + d] + t;
        // first branch id if the document's live branches are consecutive ids (no finished
        // branch in between): the kernels then need no lookup in the live list
        const int32_t nbl = dlp[d + 1] - dlp[d];
        const int32_t bf = L->live_branch[L->live_ptr[t] + dlp[d]];
        const int32_t bl = L->live_branch[L->live_ptr[t] + dlp[d + 1] - 1];
        const int32_t b_first = (bl - bf == nbl - 1) ? bf : -1;
        const int32_t desc[8] = {L->seg_off[p], L->seg_len[p], L->seg_off[P + d], L->seg_len[P + d],
                                 dlp[d], nbl, pos, b_first};
        L->unit_desc.insert(L->unit_desc.end(), desc, desc + 8);
      }
    }
    L->total_units = (int64_t)L->unit_doc.size();

    // ---- paper-literal mask: the work unit is the prompt (its rows see every document and the
    //      tails of all earlier branches).  Document blocks of a prompt in stream order; per
    //      step the prompts with live branches, heaviest first.
    if (cfg->mask_mode == HPD_MASK_PAPER) {
      L->pblk_ptr.assign(P + 1, 0);
      for (int32_t p = 0; p < P; ++p) {
        for (int32_t d = doc_ptr[p]; d < doc_ptr[p + 1]; ++d)
          for (int32_t i = 0; i < doc_len[d]; i += HPD_KEY_BLOCK) {
            L->pblk.push_back(L->seg_off[P + d] + i);
            L->pblk.push_back(std::min<int32_t>(HPD_KEY_BLOCK, doc_len[d] - i));
          }
        // then the blocks of the attribute names: a row keeps the names up to its own branch's,
        // so the second entry is 1000 + the index of the block's first name token
        for (int32_t i = 0; i < L->seg_len[P + n_docs + p]; i += HPD_KEY_BLOCK) {
          L->pblk.push_back(L->skel_seg_off[p] + i);
          L->pblk.push_back(1000 + i);
        }
        L->pblk_ptr[p + 1] = (int32_t)(L->pblk.size() / 2);
        L->max_prompt_branches = std::max(L->max_prompt_branches,
                                          L->prompt_branch_ptr[p + 1] - L->prompt_branch_ptr[p]);
      }
      L->punit_ptr.assign(T + 1, 0);
      L->pmax_rows.assign(T, 0);
      for (int32_t t = 0; t < T; ++t) {
        const int32_t* dlp = &L->doc_live_ptr[(size_t)t * (n_docs + 1)];
        std::vector<int32_t> units;
        for (int32_t p = 0; p < P; ++p)
          if (dlp[doc_ptr[p + 1]] > dlp[doc_ptr[p]]) units.push_back(p);
        std::stable_sort(units.begin(), units.end(), [&](int32_t x, int32_t y) {
          return L->pblk_ptr[x + 1] - L->pblk_ptr[x] > L->pblk_ptr[y + 1] - L->pblk_ptr[y];
        });
        for (int32_t p : units) {
          const int32_t r0 = dlp[doc_ptr[p]], nbl = dlp[doc_ptr[p + 1]] - r0;
          const int32_t bf = L->live_branch[L->live_ptr[t] + r0];
          const int32_t bl = L->live_branch[L->live_ptr[t] + r0 + nbl - 1];
          const int32_t pb0 = L->prompt_branch_ptr[p];
          const int32_t desc[16] = {L->seg_off[p], L->seg_len[p], L->pblk_ptr[p],
                                    L->pblk_ptr[p + 1] - L->pblk_ptr[p], r0, nbl, pb0,
                                    (bl - bf == nbl - 1) ? bf : -1, bl - pb0 + 1, 0, 0, 0, 0, 0, 0, 0};
          L->punit_desc.insert(L->punit_desc.end(), desc, desc + 16);
          L->pmax_rows[t] = std::max(L->pmax_rows[t], nbl);
        }
        L->punit_ptr[t + 1] = L->punit_ptr[t] + (int32_t)units.size();
      }
    }

    // ---- attention of the prefix tokens (first inference step, block mask): a unit per
    //      non-empty header and per document, the most expensive (tokens x keys) first
    if (cfg->mask_mode == HPD_MASK_BLOCK) {
      std::vector<int32_t> segs;
      for (int32_t sid = 0; sid < n_seg; ++sid)
        if (L->seg_len[sid] > 0) segs.push_back(sid);
      std::vector<int32_t> raw_of(n_seg);
      for (int32_t i = 0; i < n_seg; ++i) raw_of[L->raw_seg[i]] = L->seg_raw_off[i];
      auto cost = [&](int32_t sid) -> int64_t {
        const int64_t hl = sid < P ? 0 : L->seg_len[L->doc_prompt[sid - P]];
        return (int64_t)L->seg_len[sid] * (hl + L->seg_len[sid]);
      };
      std::stable_sort(segs.begin(), segs.end(), [&](int32_t x, int32_t y) { return cost(x) > cost(y); });
      for (int32_t sid : segs) {
        const int32_t p = sid < P ? sid : L->doc_prompt[sid - P];
        const int32_t desc[8] = {L->seg_off[p], sid < P ? 0 : L->seg_len[p], L->seg_off[sid], L->seg_len[sid],
                                 raw_of[sid], L->seg_len[sid], L->seg_pos0[sid], 0};
        L->funit_desc.insert(L->funit_desc.end(), desc, desc + 8);
        L->fmax_rows = std::max(L->fmax_rows, L->seg_len[sid]);
      }
    }

    // ---- the same under the literal mask: header, documents and attribute names of a prompt
    //      are one causal sequence.  A segment sees the earlier segments of its prompt in full -
    //      a list of their 32-key blocks (first pool slot, keys), of which every segment takes
    //      a prefix - and itself up to the query.  A unit per non-empty segment:
    //      {first list entry of the prompt, list blocks the segment sees, first slot, tokens,
    //       first token in q / out order, tokens, position ID of the first token or
    //       -(1 + first entry in skel_pos) for the names, 0}
    if (cfg->mask_mode == HPD_MASK_PAPER) {
      std::vector<int32_t> raw_of(n_seg), before(n_seg, 0), list0(n_seg, 0);
      for (int32_t i = 0; i < n_seg; ++i) raw_of[L->raw_seg[i]] = L->seg_raw_off[i];
      for (int32_t p = 0; p < P; ++p) {
        const int32_t base = (int32_t)(L->fblk.size() / 2);
        auto add = [&](int32_t sid, bool keys) {
          list0[sid] = base;
          before[sid] = (int32_t)(L->fblk.size() / 2) - base;
          for (int32_t i = 0; keys && i < L->seg_len[sid]; i += HPD_KEY_BLOCK) {
            L->fblk.push_back(L->seg_off[sid] + i);
            L->fblk.push_back(std::min<int32_t>(HPD_KEY_BLOCK, L->seg_len[sid] - i));
          }
        };
        add(p, true);
        for (int32_t d = doc_ptr[p]; d < doc_ptr[p + 1]; ++d) add(P + d, true);
        add(P + n_docs + p, false);  // nothing comes after the names
      }
      std::vector<int32_t> segs;
      for (int32_t sid = 0; sid < n_seg; ++sid)
        if (L->seg_len[sid] > 0) segs.push_back(sid);
      auto cost = [&](int32_t sid) -> int64_t {
        return (int64_t)L->seg_len[sid] * ((int64_t)before[sid] * HPD_KEY_BLOCK + L->seg_len[sid]);
      };
      std::stable_sort(segs.begin(), segs.end(), [&](int32_t x, int32_t y) { return cost(x) > cost(y); });
      for (int32_t sid : segs) {
        const bool names = sid >= P + n_docs;
        const int32_t desc[8] = {list0[sid], before[sid], L->seg_off[sid], L->seg_len[sid], raw_of[sid],
                                 L->seg_len[sid], names ? -(1 + L->skel_off[sid - P - n_docs]) : L->seg_pos0[sid], 0};
        L->funit_desc.insert(L->funit_desc.end(), desc, desc + 8);
        L->fmax_rows = std::max(L->fmax_rows, L->seg_len[sid]);
        L->fmax_list_blocks = std::max(L->fmax_list_blocks, before[sid]);
      }
    }

    // ---- for hpd_prefix_fill: which segment owns a 32-slot block of the pools, and where its
    //      first token sits in the input order
    {
      std::vector<int32_t> raw_of(n_seg);
      for (int32_t i = 0; i < n_seg; ++i) raw_of[L->raw_seg[i]] = L->seg_raw_off[i];
      L->fill_blk.assign((size_t)(L->NP / HPD_KEY_BLOCK) * 2, -1);
      for (int32_t sid = 0; sid < n_seg; ++sid)
        for (int32_t i = 0; i < L->seg_len[sid]; i += HPD_KEY_BLOCK) {
          const size_t b = (size_t)(L->seg_off[sid] + i) / HPD_KEY_BLOCK;
          L->fill_blk[2 * b] = sid;
          L->fill_blk[2 * b + 1] = raw_of[sid] + i;
        }
    }

    // ---- device-side pruning: what never changes, one record of 8 words per unit (document, or
    //      prompt under the literal mask), the units with the most keys first.  Documents:
    //      {hoff, Hlen, doff, Llen, first branch, end of branches, position of step 0 | -1, 0};
    //      prompts: {hoff, Hlen, first entry of the block list, its blocks, first branch, end of
    //      branches, 0, 0}
    {
      const size_t nU = paper ? (size_t)P : (size_t)n_docs;
      std::vector<int32_t> order(nU);
      std::iota(order.begin(), order.end(), 0);
      std::stable_sort(order.begin(), order.end(), [&](int32_t x, int32_t y) {
        if (paper) return L->pblk_ptr[x + 1] - L->pblk_ptr[x] > L->pblk_ptr[y + 1] - L->pblk_ptr[y];
        return (int64_t)L->seg_len[L->doc_prompt[x]] + L->seg_len[L->P + x] >
               (int64_t)L->seg_len[L->doc_prompt[y]] + L->seg_len[L->P + y];
      });
      L->dyn_fixed.assign(nU * 8, 0);
      for (size_t u = 0; u < nU; ++u) {
        int32_t* o = L->dyn_fixed.data() + u * 8;
        if (paper) {
          const int32_t p = order[u];
          o[0] = L->seg_off[p]; o[1] = L->seg_len[p]; o[2] = L->pblk_ptr[p]; o[3] = L->pblk_ptr[p + 1] - L->pblk_ptr[p];
          o[4] = L->prompt_branch_ptr[p]; o[5] = L->prompt_branch_ptr[p + 1];
        } else {
          const int32_t d = order[u], p = L->doc_prompt[d];
          o[0] = L->seg_off[p]; o[1] = L->seg_len[p]; o[2] = L->seg_off[L->P + d]; o[3] = L->seg_len[L->P + d];
          o[4] = L->doc_branch_ptr[d]; o[5] = L->doc_branch_ptr[d + 1];
          o[6] = L->cfg.pos_mode == HPD_POS_CONTIG ? L->seg_len[p] + L->seg_len[L->P + d] : -1;
        }
      }
    }

    // ---- RoPE table: angles in double, stored as float (cos, sin)
    const int32_t half = cfg->head_dim / 2;
    L->rope.resize((size_t)(L->max_pos + 1) * half * 2);
    std::vector<double> theta(half);
    for (int32_t i = 0; i < half; ++i)
      theta[i] = std::pow(cfg->rope_base, -2.0 * (double)i / (double)cfg->head_dim);
    for (int64_t pos = 0; pos <= L->max_pos; ++pos)
      for (int32_t i = 0; i < half; ++i) {
        const double a = (double)pos * theta[i];
        L->rope[((size_t)pos * half + i) * 2 + 0] = (float)std::cos(a);
        L->rope[((size_t)pos * half + i) * 2 + 1] = (float)std::sin(a);
      }
  } catch (const std::bad_alloc&) {
    delete L;
    return HPD_E_NOMEM;
  }

  if (!(cfg->flags & HPD_FLAG_HOST_ONLY)) {
    // ---- upload
    IntArena A;
    const size_t o_seg_off = A.add(L->seg_off), o_seg_len = A.add(L->seg_len),
                 o_seg_pos0 = A.add(L->seg_pos0), o_raw_off = A.add(L->seg_raw_off),
                 o_raw_seg = A.add(L->raw_seg), o_doc_prompt = A.add(L->doc_prompt),
                 o_branch_doc = A.add(L->branch_doc), o_base = A.add(L->branch_base_pos),
                 o_live_ptr = A.add(L->live_ptr), o_live_branch = A.add(L->live_branch),
                 o_dlp = A.add(L->doc_live_ptr), o_unit_ptr = A.add(L->unit_ptr),
                 o_unit_doc = A.add(L->unit_doc), o_unit_desc = A.add(L->unit_desc),
                 o_pdp = A.add(L->prompt_doc_ptr), o_pbp = A.add(L->prompt_branch_ptr),
                 o_blen = A.add(L->branch_len), o_pblk = A.add(L->pblk), o_pdesc = A.add(L->punit_desc),
                 o_fdesc = A.add(L->funit_desc), o_spos = A.add(L->skel_pos), o_soff = A.add(L->skel_off),
                 o_sseg = A.add(L->skel_seg_off), o_scum = A.add(L->skel_cum), o_fblk = A.add(L->fblk),
                 o_fill = A.add(L->fill_blk), o_dynfix = A.add(L->dyn_fixed);
    hipStream_t s = (hipStream_t)stream;
    hipError_t e = hipGetDevice(&L->device);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&L->n_cus, hipDeviceAttributeMultiprocessorCount, L->device);
    if (e == hipSuccess) e = hipMalloc(&L->d_ints, A.host.size() * sizeof(int32_t));
    if (e == hipSuccess) e = hipMalloc(&L->d_rope, L->rope.size() * sizeof(float));
    if (e == hipSuccess)
      e = hipMemcpyAsync(L->d_ints, A.host.data(), A.host.size() * sizeof(int32_t),
                         hipMemcpyHostToDevice, s);
    if (e == hipSuccess)
      e = hipMemcpyAsync(L->d_rope, L->rope.data(), L->rope.size() * sizeof(float),
                         hipMemcpyHostToDevice, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) {
      if (L->d_ints) (void)hipFree(L->d_ints);
      if (L->d_rope) (void)hipFree(L->d_rope);
      delete L;
      return hip_fail(e);
    }
    const int32_t* base = (const int32_t*)L->d_ints;
    L->dev.seg_off = base + o_seg_off; L->dev.seg_len = base + o_seg_len;
    L->dev.seg_pos0 = base + o_seg_pos0; L->dev.seg_raw_off = base + o_raw_off;
    L->dev.raw_seg = base + o_raw_seg; L->dev.doc_prompt = base + o_doc_prompt;
    L->dev.branch_doc = base + o_branch_doc; L->dev.branch_base_pos = base + o_base;
    L->dev.live_ptr = base + o_live_ptr; L->dev.live_branch = base + o_live_branch;
    L->dev.doc_live_ptr = base + o_dlp; L->dev.unit_ptr = base + o_unit_ptr;
    L->dev.unit_doc = base + o_unit_doc; L->dev.unit_desc = base + o_unit_desc;
    L->dev.prompt_doc_ptr = base + o_pdp; L->dev.prompt_branch_ptr = base + o_pbp;
    L->dev.branch_len = base + o_blen; L->dev.pblk = base + o_pblk; L->dev.punit_desc = base + o_pdesc;
    L->dev.funit_desc = base + o_fdesc; L->dev.fblk = base + o_fblk;
    L->dev.fill_blk = base + o_fill;
    L->dyn_fixed_dev = const_cast<int32_t*>(base) + o_dynfix;
    L->dev.skel_pos = paper_mode(L) ? base + o_spos : nullptr; L->dev.skel_off = base + o_soff;
    L->dev.skel_seg_off = base + o_sseg; L->dev.skel_cum = base + o_scum;
    L->dev.rope = (const float2*)L->d_rope;
    L->on_device = true;
  }
  *out = L;
  return HPD_OK;
}

void hpd_layout_free(hpd_layout* L) {
  if (!L) return;
  if (L->d_dyn) (void)hipFree(L->d_dyn);
  if (L->d_ints) (void)hipFree(L->d_ints);
  if (L->d_rope) (void)hipFree(L->d_rope);
  delete L;
}

int hpd_layout_query(const hpd_layout* L, int32_t what, void* host_out, size_t bytes) {
  if (!L || !host_out) return HPD_E_INVALID;
  auto copy32 = [&](const std::vector<int32_t>& v, size_t n) -> int {
    if (bytes < n * sizeof(int32_t)) return HPD_E_INVALID;
    if (n) std::memcpy(host_out, v.data(), n * sizeof(int32_t));
    return HPD_OK;
  };
  const size_t eb = elem_bytes(L->cfg);
  switch (what) {
    case HPD_Q_COUNTS: {
      if (bytes < HPD_N_COUNTS * sizeof(int64_t)) return HPD_E_INVALID;
      int64_t c[HPD_N_COUNTS];
      c[HPD_C_N_PROMPTS] = L->P; c[HPD_C_N_DOCS] = L->n_docs; c[HPD_C_N_BRANCHES] = L->B;
      c[HPD_C_N_PREFIX_TOKENS] = L->n_prefix_tokens; c[HPD_C_N_PREFIX_SLOTS] = L->NP;
      c[HPD_C_N_TAIL_SLOTS] = (int64_t)L->B * L->T; c[HPD_C_MAX_POS] = L->max_pos;
      c[HPD_C_TOTAL_LIVE] = L->total_live;
      std::memcpy(host_out, c, sizeof(c));
      return HPD_OK;
    }
    case HPD_Q_POOL_BYTES: {
      if (bytes < 4 * sizeof(int64_t)) return HPD_E_INVALID;
      const int64_t per_slot = (int64_t)L->cfg.n_kv_heads * L->cfg.head_dim * (int64_t)eb;
      const int64_t tail_slots = L->dev.tail_pages ? ((int64_t)L->dev.n_pages << L->dev.page_shift)
                                                   : (int64_t)L->B * L->T;
      int64_t c[4] = {L->NP * per_slot, L->NP * per_slot, tail_slots * per_slot, tail_slots * per_slot};
      std::memcpy(host_out, c, sizeof(c));
      return HPD_OK;
    }
    case HPD_Q_N_LIVE: {
      if (bytes < (size_t)L->T * sizeof(int32_t)) return HPD_E_INVALID;
      int32_t* o = (int32_t*)host_out;
      for (int32_t t = 0; t < L->T; ++t) o[t] = L->live_ptr[t + 1] - L->live_ptr[t];
      return HPD_OK;
    }
    case HPD_Q_N_UNITS: {
      if (bytes < (size_t)L->T * sizeof(int32_t)) return HPD_E_INVALID;
      int32_t* o = (int32_t*)host_out;
      const std::vector<int32_t>& up = L->cfg.mask_mode == HPD_MASK_PAPER ? L->punit_ptr : L->unit_ptr;
      for (int32_t t = 0; t < L->T; ++t) o[t] = up[t + 1] - up[t];
      return HPD_OK;
    }
    case HPD_Q_LIVE_BRANCH: return copy32(L->live_branch, (size_t)L->total_live);
    case HPD_Q_BRANCH_BASE_POS: return copy32(L->branch_base_pos, (size_t)L->B);
    case HPD_Q_BRANCH_DOC: return copy32(L->branch_doc, (size_t)L->B);
    case HPD_Q_SEG_OFF: return copy32(L->seg_off, (size_t)L->n_seg);
    case HPD_Q_SEG_LEN: return copy32(L->seg_len, (size_t)L->n_seg);
    case HPD_Q_SEG_POS0: return copy32(L->seg_pos0, (size_t)L->n_seg);
    case HPD_Q_SEG_RAW_OFF: {
      if (bytes < (size_t)L->n_seg * sizeof(int32_t)) return HPD_E_INVALID;
      int32_t* o = (int32_t*)host_out;
      for (int32_t i = 0; i < L->n_seg; ++i) o[L->raw_seg[i]] = L->seg_raw_off[i];
      return HPD_OK;
    }
    default: return HPD_E_INVALID;
  }
}

int hpd_set_kernel_mode(hpd_layout* L, int32_t mode) {
  if (!L || mode < 0 || mode > 4) return HPD_E_INVALID;
  if (mode >= 2 && !hpd_stream_supported(L)) return HPD_E_UNSUPPORTED;
  L->kernel_mode = mode;
  return HPD_OK;
}

static int check_step(const hpd_layout* L, int32_t step) {
  if (!L) return HPD_E_INVALID;
  if (!L->on_device) return HPD_E_INVALID;
  if (step < 0 || step >= L->T) return HPD_E_INVALID;
  return HPD_OK;
}

int hpd_prefix_fill(const hpd_layout* L, const void* k_raw, const void* v_raw, void* k_prefix,
                    void* v_prefix, void* stream) {
  if (!L || !L->on_device || !k_prefix || !v_prefix) return HPD_E_INVALID;
  if (L->n_prefix_tokens == 0) return HPD_OK;
  if (!k_raw || !v_raw) return HPD_E_INVALID;
  HPD_HIP(hpd_launch_prefix_fill(L, k_raw, v_raw, k_prefix, v_prefix, (hipStream_t)stream));
  return HPD_OK;
}

int hpd_rope_positions(const hpd_layout* L, int32_t step, int32_t* pos_out, int32_t* n_live_out,
                       void* stream) {
  int rc = check_step(L, step);
  if (rc != HPD_OK) return rc;
  const int32_t n_live = L->live_ptr[step + 1] - L->live_ptr[step];
  if (n_live > 0 && !pos_out) return HPD_E_INVALID;
  if (n_live > 0) HPD_HIP(hpd_launch_positions(L, step, pos_out, (hipStream_t)stream));
  if (n_live_out) *n_live_out = n_live;
  return HPD_OK;
}

int hpd_kv_append(const hpd_layout* L, int32_t step, const void* k_new, const void* v_new,
                  void* k_tail, void* v_tail, int64_t* slot_out, void* stream) {
  int rc = check_step(L, step);
  if (rc != HPD_OK) return rc;
  const int32_t n_live = L->live_ptr[step + 1] - L->live_ptr[step];
  if (n_live == 0) return HPD_OK;
  if (!k_new || !v_new || !k_tail || !v_tail) return HPD_E_INVALID;
  HPD_HIP(hpd_launch_append(L, step, k_new, v_new, k_tail, v_tail, slot_out, (hipStream_t)stream));
  return HPD_OK;
}

int hpd_decode_attention(const hpd_layout* L, int32_t step, const void* q, const void* k_prefix,
                         const void* v_prefix, const void* k_tail, const void* v_tail, void* out,
                         void* stream) {
  int rc = check_step(L, step);
  if (rc != HPD_OK) return rc;
  const int32_t n_live = L->live_ptr[step + 1] - L->live_ptr[step];
  if (n_live == 0) return HPD_OK;
  if (!q || !k_prefix || !v_prefix || !k_tail || !v_tail || !out) return HPD_E_INVALID;
  const bool use_stream = L->kernel_mode >= 2 || (L->kernel_mode == 0 && hpd_stream_supported(L));
  if (use_stream) {
    HPD_HIP(hpd_launch_attention_stream(L, step, q, k_prefix, v_prefix, const_cast<void*>(k_tail),
                                        const_cast<void*>(v_tail), nullptr, nullptr, out,
                                        (hipStream_t)stream));
  } else {
    // the generic kernel keeps one score per key in LDS
    if (hpd_generic_max_keys(L, step) > 15000) return HPD_E_UNSUPPORTED;
    HPD_HIP(hpd_launch_attention_generic(L, step, q, k_prefix, v_prefix, k_tail, v_tail, out,
                                         (hipStream_t)stream));
  }
  return HPD_OK;
}

int hpd_prefill_attention(const hpd_layout* L, const void* q, const void* k_prefix, const void* v_prefix,
                          void* out, void* stream) {
  if (!L || !L->on_device) return HPD_E_INVALID;
  if (L->n_prefix_tokens == 0) return HPD_OK;
  if (!q || !k_prefix || !v_prefix || !out) return HPD_E_INVALID;
  const bool paper = L->cfg.mask_mode == HPD_MASK_PAPER;
  // (the streaming kernel keeps the key counts of a unit's block list in LDS: 512 entries)
  if ((L->kernel_mode >= 2 || (L->kernel_mode == 0 && hpd_stream_supported(L))) &&
      (!paper || L->fmax_list_blocks <= 512)) {
    HPD_HIP(hpd_launch_prefill_stream(L, q, k_prefix, v_prefix, out, (hipStream_t)stream));
    return HPD_OK;
  }
  // the generic kernel keeps one score per key in LDS
  int64_t max_keys = 0;
  for (int32_t d = 0; d < L->n_docs; ++d)
    max_keys = std::max<int64_t>(max_keys, (int64_t)L->seg_len[L->doc_prompt[d]] + L->seg_len[L->P + d]);
  for (int32_t p = 0; p < L->P; ++p) max_keys = std::max<int64_t>(max_keys, L->seg_len[p]);
  if (paper)  // a prompt's last name token sees the whole prefix of the prompt
    for (int32_t p = 0; p < L->P; ++p) {
      int64_t keys = (int64_t)L->seg_len[p] + L->seg_len[L->P + L->n_docs + p];
      for (int32_t d = L->prompt_doc_ptr[p]; d < L->prompt_doc_ptr[p + 1]; ++d) keys += L->seg_len[L->P + d];
      max_keys = std::max(max_keys, keys);
    }
  if (max_keys > 15000) return HPD_E_UNSUPPORTED;
  HPD_HIP(hpd_launch_prefill_generic(L, q, k_prefix, v_prefix, out, (hipStream_t)stream));
  return HPD_OK;
}

int hpd_decode_step(const hpd_layout* L, int32_t step, const void* q, const void* k_new,
                    const void* v_new, const void* k_prefix, const void* v_prefix, void* k_tail,
                    void* v_tail, void* out, void* stream) {
  int rc = check_step(L, step);
  if (rc != HPD_OK) return rc;
  const int32_t n_live = L->live_ptr[step + 1] - L->live_ptr[step];
  if (n_live == 0) return HPD_OK;
  if (!q || !k_new || !v_new || !k_prefix || !v_prefix || !k_tail || !v_tail || !out)
    return HPD_E_INVALID;
  if (L->kernel_mode >= 2 || (L->kernel_mode == 0 && hpd_stream_supported(L))) {
    // one launch: the attention kernel rotates, stores and uses the new keys itself
    HPD_HIP(hpd_launch_attention_stream(L, step, q, k_prefix, v_prefix, k_tail, v_tail, k_new, v_new,
                                        out, (hipStream_t)stream));
    return HPD_OK;
  }
  rc = hpd_kv_append(L, step, k_new, v_new, k_tail, v_tail, nullptr, stream);
  if (rc != HPD_OK) return rc;
  return hpd_decode_attention(L, step, q, k_prefix, v_prefix, k_tail, v_tail, out, stream);
}

int hpd_expand_mask(const hpd_layout* L, int32_t prompt, int32_t step_hi, uint8_t* mask_out,
                    int32_t* s_out, void* stream) {
  if (!L || !L->on_device || !s_out) return HPD_E_INVALID;
  if (prompt < 0 || prompt >= L->P || step_hi < -1 || step_hi >= L->T) return HPD_E_INVALID;
  // token descriptors in memory order: (kind, document, branch, step | position for the
  // paper-literal mask);  kind 0 header, 1 document, 2 branch token
  const bool paper = L->cfg.mask_mode == HPD_MASK_PAPER;
  std::vector<int32_t> desc;
  const int32_t H = L->seg_len[prompt];
  for (int32_t i = 0; i < H; ++i) { desc.insert(desc.end(), {0, -1, -1, paper ? i : -1}); }
  int32_t d0 = -1, d1 = -1;
  for (int32_t d = 0; d < L->n_docs; ++d)
    if (L->doc_prompt[d] == prompt) { if (d0 < 0) d0 = d; d1 = d + 1; }
  for (int32_t d = d0; d >= 0 && d < d1; ++d)
    for (int32_t i = 0; i < L->seg_len[L->P + d]; ++i)
      desc.insert(desc.end(), {1, d, -1, paper ? L->seg_pos0[L->P + d] + i : -1});
  if (paper)  // the attribute names, fed with the prompt (kind 3)
    for (int32_t i = L->skel_off[prompt]; i < L->skel_off[prompt + 1]; ++i)
      desc.insert(desc.end(), {3, -1, -1, L->skel_pos[i]});
  for (int32_t t = 0; t <= step_hi; ++t)
    for (int32_t r = L->live_ptr[t]; r < L->live_ptr[t + 1]; ++r) {
      const int32_t b = L->live_branch[r];
      const int32_t d = L->branch_doc[b];
      if (L->doc_prompt[d] == prompt)
        desc.insert(desc.end(), {2, d, b, paper ? L->branch_base_pos[b] + 1 + t : t});
    }
  const int64_t S = (int64_t)desc.size() / 4;
  if (S > 46000) return HPD_E_OVERFLOW;
  *s_out = (int32_t)S;
  if (!mask_out || S == 0) return HPD_OK;
  int32_t* d_desc = nullptr;
  hipStream_t s = (hipStream_t)stream;
  HPD_HIP(hipMalloc((void**)&d_desc, desc.size() * sizeof(int32_t)));
  hipError_t e = hipMemcpyAsync(d_desc, desc.data(), desc.size() * sizeof(int32_t),
                                hipMemcpyHostToDevice, s);
  if (e == hipSuccess) e = hpd_launch_expand_mask(d_desc, (int32_t)S, paper ? 1 : 0, mask_out, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  (void)hipFree(d_desc);
  if (e != hipSuccess) return hip_fail(e);
  return HPD_OK;
}

static int dynamic_supported(const hpd_layout* L) {
  if (!L || !L->on_device) return HPD_E_INVALID;
  if (!hpd_stream_supported(L) || L->kernel_mode == 1 || L->B > 65536) return HPD_E_UNSUPPORTED;
  return HPD_OK;
}

// words of device-side pruning state a layout needs: desc [units * 8 | 16] (read and written 16
// bytes at a time), n_live [4], live [B], and for the literal mask len [B]; units = documents, or
// prompts under the literal mask
static size_t dynamic_state_words(const hpd_layout* L) {
  const bool paper = L->cfg.mask_mode == HPD_MASK_PAPER;
  const size_t nB = (size_t)L->B, nU = paper ? (size_t)L->P : (size_t)L->n_docs, dw = paper ? 16 : 8;
  return nU * dw + 4 + nB + (paper ? nB : 0) + 16;
}

// points the layout's state at `mem` (dynamic_state_words(L) words, 16-byte aligned)
static void dynamic_state_bind(hpd_layout* L, void* mem) {
  const bool paper = L->cfg.mask_mode == HPD_MASK_PAPER;
  const size_t nB = (size_t)L->B, nU = paper ? (size_t)L->P : (size_t)L->n_docs, dw = paper ? 16 : 8;
  int32_t* w = (int32_t*)mem;
  L->dyn_desc = w; w += nU * dw;
  L->dyn_n_live = w; w += 4;
  L->dyn_live = w; w += nB;
  L->dyn_len = paper ? w : nullptr;
}

int hpd_dynamic_begin(hpd_layout* L, void* stream) {
  int rc = dynamic_supported(L);
  if (rc != HPD_OK) return rc;
  hipStream_t s = (hipStream_t)stream;
  if (!L->d_dyn) HPD_HIP(hipMalloc(&L->d_dyn, dynamic_state_words(L) * sizeof(int32_t)));
  dynamic_state_bind(L, L->d_dyn);
  L->dyn_next_step = 0;
  HPD_HIP(hpd_launch_dynamic_prune(L, 0, nullptr, s));
  return HPD_OK;
}

int hpd_dynamic_begin_static(hpd_layout* L, void* stream) {
  int rc = dynamic_supported(L);
  if (rc != HPD_OK) return rc;
  if (dynamic_state_words(L) * sizeof(int32_t) > (size_t)HPD_DYNAMIC_STATIC_MAX_BYTES) return HPD_E_CAPACITY;
  void* mem = nullptr;
  size_t bytes = 0;
  HPD_HIP(hpd_dynamic_scratch(L->device, &mem, &bytes));
  if (dynamic_state_words(L) * sizeof(int32_t) > bytes) return HPD_E_CAPACITY;
  dynamic_state_bind(L, mem);
  L->dyn_next_step = 0;
  HPD_HIP(hpd_launch_dynamic_prune(L, 0, nullptr, (hipStream_t)stream));
  return HPD_OK;
}

int hpd_dynamic_prune(hpd_layout* L, const uint8_t* finished, void* stream) {
  int rc = dynamic_supported(L);
  if (rc != HPD_OK) return rc;
  if (!L->dyn_live || !finished) return HPD_E_INVALID;
  if (L->dyn_next_step + 1 >= L->T) return HPD_E_INVALID;  // no step left to prune for
  L->dyn_next_step += 1;
  HPD_HIP(hpd_launch_dynamic_prune(L, L->dyn_next_step, finished, (hipStream_t)stream));
  return HPD_OK;
}

int hpd_dynamic_step(const hpd_layout* L, int32_t step, const void* q, const void* k_new,
                     const void* v_new, const void* k_prefix, const void* v_prefix, void* k_tail,
                     void* v_tail, void* out, void* stream) {
  int rc = dynamic_supported(L);
  if (rc != HPD_OK) return rc;
  if (!L->dyn_live || step != L->dyn_next_step) return HPD_E_INVALID;  // the state describes another step
  if (!q || !k_new || !v_new || !k_prefix || !v_prefix || !k_tail || !v_tail || !out) return HPD_E_INVALID;
  if (L->n_docs == 0) return HPD_OK;
  HPD_HIP(hpd_launch_attention_stream(L, step, q, k_prefix, v_prefix, k_tail, v_tail, k_new, v_new, out,
                                      (hipStream_t)stream, true));
  return HPD_OK;
}

int hpd_dynamic_state(const hpd_layout* L, const int32_t** live_branch, const int32_t** n_live) {
  if (!L || !L->dyn_live) return HPD_E_INVALID;
  if (live_branch) *live_branch = L->dyn_live;
  if (n_live) *n_live = L->dyn_n_live;
  return HPD_OK;
}

int hpd_dynamic_read(const hpd_layout* L, int32_t* live_host, int32_t capacity, int32_t* n_live_host,
                     void* stream) {
  if (!L || !L->dyn_live || !n_live_host || capacity < 0 || (capacity > 0 && !live_host)) return HPD_E_INVALID;
  hipStream_t s = (hipStream_t)stream;
  HPD_HIP(hipMemcpyAsync(n_live_host, L->dyn_n_live, sizeof(int32_t), hipMemcpyDeviceToHost, s));
  HPD_HIP(hipStreamSynchronize(s));
  const int32_t n = std::min(*n_live_host, capacity);
  if (n > 0) {
    HPD_HIP(hipMemcpyAsync(live_host, L->dyn_live, (size_t)n * sizeof(int32_t), hipMemcpyDeviceToHost, s));
    HPD_HIP(hipStreamSynchronize(s));
  }
  return HPD_OK;
}

int hpd_set_tail_pages(hpd_layout* L, int32_t page_size, int32_t n_pages, const int32_t* page_table) {
  if (!L || !L->on_device) return HPD_E_INVALID;
  if (page_size == 0) {
    L->dev.tail_pages = nullptr;
    L->dev.page_shift = L->dev.pages_per_branch = L->dev.n_pages = 0;
    return HPD_OK;
  }
  if (page_size < 8 || (page_size & (page_size - 1)) != 0 || n_pages < 1 || !page_table) return HPD_E_INVALID;
  if ((int64_t)n_pages * page_size > ((int64_t)1 << 40)) return HPD_E_OVERFLOW;
  int32_t shift = 0;
  while ((1 << shift) < page_size) ++shift;
  L->dev.tail_pages = page_table;
  L->dev.page_shift = shift;
  L->dev.pages_per_branch = (L->T + page_size - 1) / page_size;
  L->dev.n_pages = n_pages;
  return HPD_OK;
}

int hpd_finetune_mask(int32_t prompt_len, int32_t n_attr, const int32_t* attr_len,
                      const int32_t* value_len, int32_t k_max, int32_t* pos_out, uint8_t* mask_out,
                      int64_t* s_out, void* stream) {
  if (!s_out || prompt_len < 0 || n_attr < 0 || k_max < 1) return HPD_E_INVALID;
  if (n_attr > 0 && (!attr_len || !value_len)) return HPD_E_INVALID;
  int64_t S = prompt_len;
  for (int32_t n = 0; n < n_attr; ++n) {
    if (attr_len[n] < 1 || value_len[n] < 0 || value_len[n] > k_max) return HPD_E_INVALID;
    S += (int64_t)attr_len[n] + value_len[n];
    if (S > 46000) return HPD_E_OVERFLOW;
  }
  if (S > 46000 || S + (int64_t)n_attr * k_max > ((int64_t)1 << 30)) return HPD_E_OVERFLOW;
  *s_out = S;
  if (S == 0 || (!pos_out && !mask_out)) return HPD_OK;
  // token table in the regular order; Algorithm 2 for the skeleton, end(a_n) + k for values
  std::vector<int32_t> desc;
  desc.reserve((size_t)S * 4);
  for (int32_t i = 0; i < prompt_len; ++i) desc.insert(desc.end(), {0, -1, 0, i});
  int32_t next = prompt_len, offset = 0;
  for (int32_t n = 0; n < n_attr; ++n) {
    for (int32_t i = 0; i < attr_len[n]; ++i) desc.insert(desc.end(), {1, n, 0, next++ + offset});
    const int32_t end_pos = desc[desc.size() - 1];
    for (int32_t k = 1; k <= value_len[n]; ++k) desc.insert(desc.end(), {2, n, k, end_pos + k});
    offset += k_max;
  }
  int32_t* d_desc = nullptr;
  hipStream_t s = (hipStream_t)stream;
  HPD_HIP(hipMalloc((void**)&d_desc, desc.size() * sizeof(int32_t)));
  hipError_t e = hipMemcpyAsync(d_desc, desc.data(), desc.size() * sizeof(int32_t), hipMemcpyHostToDevice, s);
  if (e == hipSuccess) e = hpd_launch_finetune_mask(d_desc, (int32_t)S, pos_out, mask_out, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  (void)hipFree(d_desc);
  if (e != hipSuccess) return hip_fail(e);
  return HPD_OK;
}

}  // extern "C"
