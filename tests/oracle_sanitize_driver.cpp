// Drives every entry point of the CPU oracle over seeded random pool life cycles and attention
// matrices.  It checks nothing itself: it is built together with oracle/cp_oracle.cpp under
// AddressSanitizer and UndefinedBehaviorSanitizer (tests/test_oracle_sanitizers.py), which stop the
// run at the first out-of-bounds access, use after free, leak or undefined operation.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

#include "../oracle/cp_oracle.h"

namespace {

constexpr uint32_t L = 2, H = 2, D = 8;     // a small KV shape: row = 32 bytes
constexpr uint32_t ROW = H * D * 2, TOKB = L * 2 * ROW;

cpo_layout token_major() { return cpo_layout{L, H, D, TOKB, 2 * ROW, ROW}; }
cpo_layout layer_major(uint32_t n) { return cpo_layout{L, H, D, ROW, 2ull * n * ROW, (uint64_t)n * ROW}; }

void life_cycle(uint32_t seed, uint32_t vocab, uint32_t W, bool rope, bool dedup, uint64_t capacity) {
  std::mt19937 rng(seed);
  const uint32_t S = 180 + seed % 50;
  std::vector<uint32_t> free_list(S);
  for (uint32_t s = 0; s < S; ++s) free_list[s] = s;
  std::shuffle(free_list.begin(), free_list.end(), rng);
  cpo_index *ix = cpo_index_new();
  if (capacity) cpo_index_rebuild(ix, capacity);  // a table so small that some batches do not fit
  cpo_anchor_set *anchors = cpo_anchor_set_new();
  cpo_text *text = cpo_text_new(S);
  std::vector<uint8_t> pool((size_t)S * TOKB, 0x5A), marks(S, 0);
  std::vector<int32_t> slot_pos(S, 0);
  std::vector<uint32_t> stamps(S, 0), slot_tok(S, 0);
  std::vector<std::vector<uint32_t>> corpus(5, std::vector<uint32_t>(60));
  for (auto &c : corpus)
    for (auto &t : c) t = rng() % vocab;
  const cpo_rope rp{500000.0, seed & 1};

  for (uint32_t epoch = 1; epoch <= 14; ++epoch) {
    // a batch of one to four requests (one of them possibly empty), each some text in front of a piece of the corpus
    std::vector<uint32_t> tok, off{0};
    const uint32_t R = 1 + rng() % 4;
    for (uint32_t r = 0; r < R; ++r) {
      if (rng() % 7 != 0) {
        for (uint32_t k = rng() % 6; k > 0; --k) tok.push_back(rng() % vocab);
        const auto &c = corpus[rng() % corpus.size()];
        const uint32_t a = rng() % 20, n = 1 + rng() % 40;
        for (uint32_t k = a; k < a + n && k < c.size(); ++k) tok.push_back(c[k]);
      }
      off.push_back((uint32_t)tok.size());
    }
    const uint32_t N = (uint32_t)tok.size();
    std::vector<uint8_t> mask(N), rec(N);
    for (uint32_t i = 0; i < N; ++i) mask[i] = rng() % 12 == 0, rec[i] = rng() % 4 == 0;
    std::vector<uint64_t> h(N), hf(N), hl(N);
    std::vector<uint32_t> ro(N), fo(N), lo(N), cand(N), got(N), own_a(N), own_b(N), own_c(N), served(N);
    cpo_hash_segments(tok.data(), mask.data(), off.data(), R, 0x100000001B3ull, h.data());
    cpo_run_offsets(mask.data(), off.data(), R, ro.data());
    // lookup: run-start keys and the two candidate streams, each confirmed, merged; policies; spans; gather; zero fill
    cpo_probe(ix, h.data(), N, cand.data());
    cpo_verify(text, tok.data(), ro.data(), cand.data(), N, 0, got.data());
    own_a = got;
    cpo_hash_floating(anchors, ix, h.data(), ro.data(), N, 0x100000001B3ull, W, hf.data(), fo.data(), hl.data(), lo.data());
    cpo_probe(ix, hf.data(), N, cand.data());
    cpo_verify(text, tok.data(), fo.data(), cand.data(), N, 0, own_b.data());
    cpo_verify(text, tok.data(), fo.data(), cand.data(), N, 1, got.data());
    cpo_probe(ix, hl.data(), N, cand.data());
    cpo_verify(text, tok.data(), lo.data(), cand.data(), N, 0, own_c.data());
    cpo_verify(text, tok.data(), lo.data(), cand.data(), N, 1, got.data());
    cpo_probe2(ix, h.data(), hf.data(), N, cand.data());
    cpo_probe3(ix, h.data(), hf.data(), hl.data(), N, cand.data());
    cpo_probe3(ix, h.data(), nullptr, nullptr, N, cand.data());
    cpo_touch(own_b.data(), N, epoch, S, stamps.data());
    cpo_touch(own_c.data(), N, epoch, S, stamps.data());
    cpo_touch(got.data(), N, epoch, S, stamps.data());
    cpo_filter_matches(got.data(), off.data(), R, 1 + seed % 4, marks.data(), S, served.data());
    const uint32_t max_spans = N ? 1 + rng() % N : 1;  // sometimes too few: the overflow path
    std::vector<uint32_t> s_src(max_spans), s_dst(max_spans), s_len(max_spans);
    std::vector<int32_t> s_delta(max_spans);
    uint32_t flags = 0;
    uint32_t n_spans = cpo_build_spans(served.data(), off.data(), R, rope ? slot_pos.data() : nullptr, max_spans,
                                       s_src.data(), s_dst.data(), s_len.data(), s_delta.data(), &flags);
    if (n_spans > max_spans) n_spans = max_spans;
    std::vector<uint8_t> dst((size_t)N * TOKB + 1, 0xA5);
    cpo_gather_kv(pool.data(), token_major(), dst.data(), layer_major(N), s_src.data(), s_dst.data(), s_len.data(),
                  rope ? s_delta.data() : nullptr, n_spans, rope ? &rp : nullptr);
    cpo_fill_unmatched(served.data(), N, dst.data(), layer_major(N));
    // room for the batch, then insert it
    uint32_t need = 0;
    for (uint32_t i = 0; i < N; ++i) need += h[i] != CPO_HASH_NONE;
    if (need > free_list.size()) {
      const uint32_t T = cpo_lru_threshold(stamps.data(), S, epoch, need - (uint32_t)free_list.size(), 4096);
      std::vector<uint32_t> freed(S);
      const uint32_t n_freed = cpo_evict(ix, stamps.data(), S, T, freed.data(), text, marks.data(), anchors);
      free_list.insert(free_list.end(), freed.begin(), freed.begin() + n_freed);
    }
    std::vector<uint8_t> src((size_t)N * TOKB + 1);
    for (auto &b : src) b = (uint8_t)rng();
    std::vector<uint32_t> slot_out(N);
    uint32_t n_new;
    if (dedup) {  // every text once: the lookup above says what the pool has already
      const uint32_t *seg[3] = {ro.data(), fo.data(), lo.data()}, *found_in[3] = {own_a.data(), own_b.data(), own_c.data()};
      std::vector<uint64_t> ins_hash(N);
      std::vector<uint32_t> ins_off(N), found(N);
      cpo_insert_keys(h.data(), ro.data(), seg, found_in, 1 + 2 * (seed % 2), N, 0x100000001B3ull, ins_hash.data(),
                      ins_off.data(), found.data());
      n_new = cpo_insert_kv_dedup(ix, ins_hash.data(), found.data(), off.data(), R, free_list.data(),
                                  (uint32_t)free_list.size(), src.data(), layer_major(N), pool.data(), token_major(),
                                  slot_pos.data(), slot_out.data(), &flags, tok.data(), slot_tok.data());
      cpo_text_record_dedup(text, tok.data(), ins_off.data(), found.data(), N, slot_out.data());
      cpo_insert_anchors(anchors, ins_hash.data(), ins_off.data(), slot_out.data(), N, W);
    } else {
      n_new = cpo_insert_kv(ix, h.data(), off.data(), R, free_list.data(), (uint32_t)free_list.size(), src.data(),
                            layer_major(N), pool.data(), token_major(), slot_pos.data(), slot_out.data(), &flags,
                            tok.data(), slot_tok.data());
      cpo_text_record(text, tok.data(), ro.data(), N, slot_out.data());
      cpo_insert_anchors(anchors, h.data(), ro.data(), slot_out.data(), N, W);
    }
    free_list.erase(free_list.begin(), free_list.begin() + n_new);
    if (capacity && (flags & CPO_FLAG_TABLE_FULL)) cpo_index_rebuild(ix, capacity);  // drop the keys without a slot
    cpo_mark_recompute(slot_out.data(), rec.data(), N, S, marks.data());
    cpo_touch(slot_out.data(), N, epoch, S, stamps.data());
  }
  std::printf("life cycle %u: %llu keys in %llu entries, %llu prefix hashes\n", seed,
              (unsigned long long)cpo_index_size(ix), (unsigned long long)cpo_index_entries(ix),
              (unsigned long long)cpo_anchor_set_size(anchors));
  cpo_text_free(text);
  cpo_anchor_set_free(anchors);
  cpo_index_free(ix);
}

void annotator(uint32_t seed, uint32_t n, uint32_t pad) {
  std::mt19937 rng(seed);
  const uint64_t ld = n + pad;
  std::vector<float> a((size_t)n * ld, 7.0f);  // the padding holds junk the oracle must not read as weights
  for (uint32_t i = 0; i < n; ++i) {
    double sum = 0;
    for (uint32_t j = 0; j <= i; ++j) sum += (a[i * ld + j] = (float)((rng() % 1000) + 1));
    for (uint32_t j = 0; j <= i; ++j) a[i * ld + j] /= (float)sum;
    for (uint32_t j = i + 1; j < n; ++j) a[i * ld + j] = 0.25f;  // above the diagonal: ignored
  }
  if (n > 5) a[3 * ld + 1] = NAN, a[4 * ld + 2] = INFINITY, a[5 * ld + 0] = -1e30f;
  std::vector<int64_t> T((size_t)n * n);
  cpo_sat_build(a.data(), n, ld, T.data());
  (void)cpo_sat_rect(T.data(), n, 0, (int64_t)n - 1, 0, (int64_t)n - 1);
  (void)cpo_sat_rect(T.data(), n, 2, 1, 0, 0);
  std::vector<uint8_t> mask(n), reusable(n), recompute(n);
  for (auto &m : mask) m = rng() % 9 == 0;
  std::vector<uint32_t> bl(n), br(n);
  std::vector<int64_t> bs(n);
  cpo_annotate(T.data(), n, mask.data(), seed % 5, 25 * (seed % 5), bl.data(), br.data(), bs.data(), reusable.data(),
               recompute.data());
}

void rotation() {
  uint16_t in[64], out[64];
  double din[64], dout[64];
  for (int j = 0; j < 64; ++j) in[j] = cpo_double_to_bf16(0.01 * j - 0.3), din[j] = cpo_bf16_to_double(in[j]);
  for (int32_t delta : {0, 1, -1, 511, -100000, 2147483647})
    for (uint32_t style = 0; style < 2; ++style) {
      cpo_rope_head(in, out, 64, delta, 500000.0, style);
      cpo_rope_head_f64(din, dout, 64, (double)delta, 500000.0, style);
    }
}

}  // namespace

int main() {
  for (uint32_t seed = 0; seed < 48; ++seed)
    life_cycle(seed, seed % 3 == 0 ? 32000 : 2 + seed % 4, 1 + seed % 5, seed % 2, seed >= 24 && seed % 4 < 3,
               seed >= 36 ? 96 + 16 * (seed % 5) : 0);
  for (uint32_t seed = 0; seed < 8; ++seed) annotator(seed, 1 + 13 * seed, seed % 3);
  rotation();
  std::puts("done");
  return 0;
}
