// Host-side exerciser for a sanitizer build (-fsanitize=address,undefined on the host pass) of
// hpd_host.cpp: random valid and invalid batch descriptions through hpd_build_layout with
// HPD_FLAG_HOST_ONLY (no GPU call), every table read back into a buffer of exactly the
// reported size, the host-side argument checks of the other entry points.  The kernel
// launchers are stubbed out: nothing here may reach them.  Exit code 0 = no finding; a
// sanitizer report aborts the program.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

#include "hpd_internal.h"

static int g_stub_calls = 0;
#define STUB(...) { ++g_stub_calls; return hipErrorInvalidValue; }
hipError_t hpd_launch_prefix_fill(const hpd_layout*, const void*, const void*, void*, void*, hipStream_t) STUB()
hipError_t hpd_launch_positions(const hpd_layout*, int32_t, int32_t*, hipStream_t) STUB()
hipError_t hpd_launch_append(const hpd_layout*, int32_t, const void*, const void*, void*, void*, int64_t*,
                             hipStream_t) STUB()
hipError_t hpd_launch_attention_generic(const hpd_layout*, int32_t, const void*, const void*, const void*,
                                        const void*, const void*, void*, hipStream_t) STUB()
hipError_t hpd_launch_expand_mask(const int32_t*, int32_t, int32_t, uint8_t*, hipStream_t) STUB()
hipError_t hpd_launch_finetune_mask(const int32_t*, int32_t, int32_t*, uint8_t*, hipStream_t) STUB()
int64_t hpd_generic_max_keys(const hpd_layout*, int32_t) { ++g_stub_calls; return 0; }
bool hpd_stream_supported(const hpd_layout*) { return false; }
hipError_t hpd_launch_prefill_stream(const hpd_layout*, const void*, const void*, const void*, void*, hipStream_t) STUB()
hipError_t hpd_launch_prefill_generic(const hpd_layout*, const void*, const void*, const void*, void*, hipStream_t) STUB()
hipError_t hpd_launch_attention_stream(const hpd_layout*, int32_t, const void*, const void*, const void*, void*,
                                       void*, const void*, const void*, void*, hipStream_t, bool) STUB()
hipError_t hpd_launch_dynamic_prune(const hpd_layout*, int32_t, const uint8_t*, hipStream_t) STUB()
hipError_t hpd_dynamic_scratch(int, void**, size_t*) STUB()

#define CHECK(cond)                                                          \
  do {                                                                       \
    if (!(cond)) {                                                           \
      std::fprintf(stderr, "CHECK failed at line %d: %s\n", __LINE__, #cond); \
      std::exit(1);                                                          \
    }                                                                        \
  } while (0)

// reads a table into a heap buffer of exactly `n` elements: one element too many written by the
// library is a heap-buffer-overflow report
template <typename T>
static std::vector<T> query(const hpd_layout* L, int32_t what, size_t n) {
  std::vector<T> v(n);
  T dummy;
  CHECK(hpd_layout_query(L, what, n ? (void*)v.data() : (void*)&dummy, n * sizeof(T)) == HPD_OK);
  if (n > 0) CHECK(hpd_layout_query(L, what, v.data(), n * sizeof(T) - 1) == HPD_E_INVALID);
  return v;
}

int main() {
  std::mt19937 rng(26209);
  auto uni = [&](int lo, int hi) { return std::uniform_int_distribution<int>(lo, hi)(rng); };
  int built = 0, refused = 0;
  for (int iter = 0; iter < 400; ++iter) {
    hpd_config cfg{};
    const int hkv = 1 << uni(0, 3);
    cfg.n_kv_heads = hkv; cfg.n_q_heads = hkv * uni(1, 8);
    cfg.head_dim = 8 * uni(1, 32); cfg.dtype = uni(0, 1); cfg.rope_base = iter % 2 ? 10000.0 : 500000.0;
    cfg.max_new = uni(1, 12); cfg.flags = HPD_FLAG_HOST_ONLY; cfg.out_dtype = uni(0, 1);
    const bool paper = iter % 3 == 0, gap = paper || iter % 5 == 0;
    cfg.pos_mode = gap ? HPD_POS_PAPER_GAP : HPD_POS_CONTIG;
    cfg.mask_mode = paper ? HPD_MASK_PAPER : HPD_MASK_BLOCK;
    const int P = uni(1, 6);
    std::vector<int32_t> header(P), doc_ptr(P + 1, 0), doc_len, branch_ptr{0}, branch_len, attr_len;
    for (int p = 0; p < P; ++p) {
      header[p] = uni(0, 70);
      const int J = uni(0, 4);  // a prompt without documents is allowed
      doc_ptr[p + 1] = doc_ptr[p] + J;
      for (int j = 0; j < J; ++j) {
        doc_len.push_back(uni(1, 200));
        const int N = uni(0, 9);
        branch_ptr.push_back(branch_ptr.back() + N);
        for (int n = 0; n < N; ++n) { branch_len.push_back(uni(1, cfg.max_new)); attr_len.push_back(uni(1, 5)); }
      }
    }
    // every fourth batch is broken in one place and has to be refused
    const int breakage = iter % 4 == 3 ? uni(0, 6) : -1;
    if (breakage == 0 && !branch_len.empty()) branch_len[uni(0, (int)branch_len.size() - 1)] = cfg.max_new + 1;
    if (breakage == 1 && !doc_len.empty()) doc_len[uni(0, (int)doc_len.size() - 1)] = 0;
    if (breakage == 2) header[uni(0, P - 1)] = -1;
    if (breakage == 3) doc_ptr[0] = 1;
    if (breakage == 4) cfg.head_dim += 1;
    if (breakage == 5) { cfg.n_kv_heads = 3; cfg.n_q_heads = 4; }
    if (breakage == 6 && !attr_len.empty() && gap) attr_len[0] = 0;
    static int32_t none = 0;
    hpd_layout* L = nullptr;
    const int rc = hpd_build_layout(&cfg, P, header.data(), doc_ptr.data(), doc_len.empty() ? &none : doc_len.data(),
                                    branch_ptr.data(), branch_len.empty() ? &none : branch_len.data(),
                                    gap ? (attr_len.empty() ? &none : attr_len.data()) : nullptr, nullptr, &L);
    if (rc != HPD_OK) {
      CHECK(L == nullptr);
      CHECK(hpd_status_string(rc) != nullptr);
      ++refused;
      continue;
    }
    ++built;
    const auto c = query<int64_t>(L, HPD_Q_COUNTS, HPD_N_COUNTS);
    CHECK(c[HPD_C_N_PROMPTS] == P && c[HPD_C_N_DOCS] == (int64_t)doc_len.size());
    const size_t B = (size_t)c[HPD_C_N_BRANCHES], T = (size_t)cfg.max_new;
    const size_t n_seg = (size_t)P + doc_len.size() + (paper ? P : 0);
    query<int64_t>(L, HPD_Q_POOL_BYTES, 4);
    const auto n_live = query<int32_t>(L, HPD_Q_N_LIVE, T);
    int64_t total = 0;
    for (int32_t x : n_live) total += x;
    CHECK(total == c[HPD_C_TOTAL_LIVE]);
    const auto live = query<int32_t>(L, HPD_Q_LIVE_BRANCH, (size_t)total);
    for (int32_t b : live) CHECK(b >= 0 && (size_t)b < B);
    const auto base = query<int32_t>(L, HPD_Q_BRANCH_BASE_POS, B);
    for (size_t b = 0; b < B; ++b) CHECK(base[b] + (int64_t)T <= c[HPD_C_MAX_POS]);
    query<int32_t>(L, HPD_Q_BRANCH_DOC, B);
    const auto seg_off = query<int32_t>(L, HPD_Q_SEG_OFF, n_seg);
    const auto seg_len = query<int32_t>(L, HPD_Q_SEG_LEN, n_seg);
    for (size_t s = 0; s < n_seg; ++s) CHECK(seg_off[s] % HPD_KEY_BLOCK == 0 && seg_off[s] + seg_len[s] <= c[HPD_C_N_PREFIX_SLOTS]);
    query<int32_t>(L, HPD_Q_SEG_POS0, n_seg);
    query<int32_t>(L, HPD_Q_SEG_RAW_OFF, n_seg);
    query<int32_t>(L, HPD_Q_N_UNITS, T);
    CHECK(hpd_layout_query(L, 99, (void*)&none, 4) == HPD_E_INVALID);
    // a host-only layout refuses every device call before anything is launched
    CHECK(hpd_rope_positions(L, 0, &none, nullptr, nullptr) == HPD_E_INVALID);
    CHECK(hpd_kv_append(L, 0, &none, &none, &none, &none, nullptr, nullptr) == HPD_E_INVALID);
    CHECK(hpd_decode_attention(L, 0, &none, &none, &none, &none, &none, &none, nullptr) == HPD_E_INVALID);
    CHECK(hpd_decode_step(L, 0, &none, &none, &none, &none, &none, &none, &none, &none, nullptr) == HPD_E_INVALID);
    CHECK(hpd_prefix_fill(L, &none, &none, &none, &none, nullptr) == HPD_E_INVALID);
    CHECK(hpd_prefill_attention(L, &none, &none, &none, &none, nullptr) == HPD_E_INVALID);
    CHECK(hpd_dynamic_begin(L, nullptr) == HPD_E_INVALID);
    CHECK(hpd_dynamic_begin_static(L, nullptr) == HPD_E_INVALID);
    CHECK(hpd_set_tail_pages(L, 8, 4, &none) == HPD_E_INVALID);
    int32_t s_out = 0;
    CHECK(hpd_expand_mask(L, 0, -1, nullptr, &s_out, nullptr) == HPD_E_INVALID);
    CHECK(hpd_set_kernel_mode(L, 7) == HPD_E_INVALID);
    hpd_layout_free(L);
  }
  // fine-tuning mask: sizes and argument checks (outputs NULL: nothing is launched)
  for (int iter = 0; iter < 200; ++iter) {
    const int n = uni(0, 12), k_max = uni(1, 9);
    std::vector<int32_t> a(n), v(n);
    int64_t want = uni(0, 50);
    const int32_t plen = (int32_t)want;
    for (int i = 0; i < n; ++i) { a[i] = uni(1, 6); v[i] = uni(0, k_max); want += a[i] + v[i]; }
    int64_t S = -1;
    CHECK(hpd_finetune_mask(plen, n, a.data(), v.data(), k_max, nullptr, nullptr, &S, nullptr) == HPD_OK && S == want);
    if (n > 0) {
      v[uni(0, n - 1)] = k_max + 1;
      CHECK(hpd_finetune_mask(plen, n, a.data(), v.data(), k_max, nullptr, nullptr, &S, nullptr) == HPD_E_INVALID);
    }
  }
  hpd_layout_free(nullptr);
  CHECK(g_stub_calls == 0);
  std::printf("host sanitizer run: %d layouts built, %d refused, no finding\n", built, refused);
  return 0;
}
