// CPU oracle for the token-granular KV sharing path of CachePrune.
//
// TEST INFRASTRUCTURE ONLY: see cp_oracle.h.  Plain sequential code, one loop
// per definition, no blocking, no threads, no tuning.  It shares nothing with
// the GPU library.
#include "cp_oracle.h"

#include <algorithm>
#include <cfenv>
#include <cmath>
#include <cstring>
#include <unordered_map>
#include <unordered_set>
#include <vector>

struct cpo_index {
  std::unordered_map<uint64_t, uint32_t> map;
  // Bookkeeping for a table of bounded size (capacity 0 = unbounded): the keys that hold a table entry.
  // A key takes an entry when it is first seen by an insert and keeps it while its token is stored, after
  // its token was dropped for lack of a pool slot, and after its slot was evicted; only rebuilding the
  // table (cpo_index_rebuild) gives the entries of keys without a slot back.
  std::unordered_set<uint64_t> entries;
  uint64_t capacity = 0;
};

extern "C" cpo_index *cpo_index_new(void) { return new cpo_index(); }
extern "C" void cpo_index_free(cpo_index *ix) { delete ix; }
extern "C" uint64_t cpo_index_size(const cpo_index *ix) { return ix->map.size(); }
extern "C" void cpo_index_rebuild(cpo_index *ix, uint64_t capacity) {
  ix->capacity = capacity;
  ix->entries.clear();
  for (const auto &kv : ix->map) ix->entries.insert(kv.first);
}
extern "C" uint64_t cpo_index_entries(const cpo_index *ix) { return ix->entries.size(); }

// Sec. 4.2.1: sensitive tokens are separators; Sec. 4.2.2: polynomial rolling
// hash.  Horner form of  sum (t_m + 1) * base^(k-m)  with unsigned wrap-around
// (= arithmetic mod 2^64).
extern "C" void cpo_hash_segments(const uint32_t *tok, const uint8_t *mask, const uint32_t *off,
                                  uint32_t R, uint64_t base, uint64_t *hash_out) {
  for (uint32_t r = 0; r < R; ++r) {
    uint64_t c = 0;
    for (uint32_t i = off[r]; i < off[r + 1]; ++i) {
      if (mask[i]) {
        hash_out[i] = CPO_HASH_NONE;
        c = 0;
      } else {
        c = c * base + (uint64_t)tok[i] + 1u;
        hash_out[i] = (c == CPO_HASH_NONE) ? CPO_HASH_NONE - 1 : c;
      }
    }
  }
}

// Sec. 4.3.5 "Storage format and indexing": segments are found through a hash
// index.  Here: one key per pooled token, looked up in an ordinary map.
extern "C" void cpo_probe(const cpo_index *ix, const uint64_t *hash, uint32_t N,
                          uint32_t *slot_out) {
  for (uint32_t i = 0; i < N; ++i) {
    slot_out[i] = CPO_SLOT_NONE;
    if (hash[i] == CPO_HASH_NONE) continue;
    auto it = ix->map.find(hash[i]);
    if (it != ix->map.end()) slot_out[i] = it->second;
  }
}

// Sec. 4.3.1: the retriever's metadata are token spans.  Sequential run-length
// encoding of the slot array.
extern "C" uint32_t cpo_build_spans(const uint32_t *slot, const uint32_t *off, uint32_t R,
                                    const int32_t *slot_pos, uint32_t max_spans,
                                    uint32_t *span_src, uint32_t *span_dst, uint32_t *span_len,
                                    int32_t *span_delta, uint32_t *flags) {
  uint32_t n = 0; // spans opened so far
  for (uint32_t r = 0; r < R; ++r) {
    bool open = false;
    uint32_t cur_src = 0, cur_dst = 0, cur_len = 0;
    int32_t cur_delta = 0;
    auto close = [&]() {
      if (!open) return;
      if (n < max_spans) {
        span_src[n] = cur_src;
        span_dst[n] = cur_dst;
        span_len[n] = cur_len;
        if (span_delta) span_delta[n] = cur_delta;
      }
      ++n;
      open = false;
    };
    for (uint32_t i = off[r]; i < off[r + 1]; ++i) {
      if (slot[i] == CPO_SLOT_NONE) {
        close();
        continue;
      }
      int32_t p = (int32_t)(i - off[r]);
      int32_t d = slot_pos ? p - slot_pos[slot[i]] : 0;
      if (open && slot[i] == cur_src + cur_len && d == cur_delta) {
        ++cur_len; // position i follows position i-1 because the span is open
      } else {
        close();
        open = true;
        cur_src = slot[i];
        cur_dst = i;
        cur_len = 1;
        cur_delta = d;
      }
    }
    close();
  }
  if (n > max_spans && flags) *flags |= CPO_FLAG_SPANS_OVERFLOW;
  return n;
}

extern "C" double cpo_bf16_to_double(uint16_t bits) {
  uint32_t u = (uint32_t)bits << 16; // bf16 is the upper half of an IEEE float
  float f;
  std::memcpy(&f, &u, 4);
  return (double)f;
}

// One rounding, to nearest, ties to even, from double to the bf16 grid
// (8 significant bits, float's exponent range).
extern "C" uint16_t cpo_double_to_bf16(double x) {
  float f;
  if (std::isnan(x)) {
    f = std::nanf("");
  } else if (std::isinf(x) || x == 0.0) {
    f = (float)x;
  } else {
    int e;
    std::frexp(x, &e);                 // |x| = m * 2^e, m in [0.5, 1)
    int q = e - 8;                     // spacing of bf16 values around x is 2^q
    if (q < -133) q = -133;            // subnormal range: fixed spacing 2^-133
    int old = std::fegetround();
    std::fesetround(FE_TONEAREST);     // nearbyint: ties to even
    double n = std::nearbyint(std::ldexp(x, -q));
    std::fesetround(old);
    double y = std::ldexp(n, q);
    if (std::fabs(y) >= std::ldexp(1.0, 128)) y = std::copysign(INFINITY, x);
    f = (float)y;                      // exact: y is on the bf16 grid
  }
  uint32_t u;
  std::memcpy(&u, &f, 4);
  return (uint16_t)(u >> 16);
}

// Rotary embedding: the pair (a, b) at frequency index j turns by the angle
// delta * theta^(-2j/head_dim).
extern "C" void cpo_rope_head_f64(const double *in, double *out, uint32_t head_dim, double delta,
                                  double theta, uint32_t style) {
  uint32_t half = head_dim / 2;
  for (uint32_t j = 0; j < half; ++j) {
    double inv_freq = std::pow(theta, -2.0 * (double)j / (double)head_dim);
    double phi = delta * inv_freq;
    double c = std::cos(phi), s = std::sin(phi);
    uint32_t ia = style == 0 ? j : 2 * j;
    uint32_t ib = style == 0 ? j + half : 2 * j + 1;
    double a = in[ia], b = in[ib];
    out[ia] = a * c - b * s;
    out[ib] = b * c + a * s;
  }
}

extern "C" void cpo_rope_head(const uint16_t *in, uint16_t *out, uint32_t head_dim,
                              int32_t delta, double theta, uint32_t style) {
  std::vector<double> x(head_dim), y(head_dim);
  for (uint32_t e = 0; e < head_dim; ++e) x[e] = cpo_bf16_to_double(in[e]);
  cpo_rope_head_f64(x.data(), y.data(), head_dim, (double)delta, theta, style);
  for (uint32_t e = 0; e < head_dim; ++e) out[e] = cpo_double_to_bf16(y[e]);
}

static inline const uint8_t *row_ptr(const void *base, const cpo_layout &l, uint64_t t,
                                     uint32_t layer, uint32_t kv) {
  return (const uint8_t *)base + t * l.tok_stride + layer * l.layer_stride + kv * l.kv_stride;
}

// Sec. 4.1 / 4.3.1: matched segments are placed into the request; everything
// else is left alone.
extern "C" void cpo_gather_kv(const void *pool, cpo_layout pool_l, void *dst, cpo_layout dst_l,
                              const uint32_t *span_src, const uint32_t *span_dst,
                              const uint32_t *span_len, const int32_t *span_delta,
                              uint32_t n_spans, const cpo_rope *rope) {
  const uint32_t H = pool_l.n_kv_heads, D = pool_l.head_dim;
  const size_t row_bytes = (size_t)H * D * 2;
  for (uint32_t s = 0; s < n_spans; ++s) {
    int32_t delta = (span_delta && rope) ? span_delta[s] : 0;
    for (uint32_t k = 0; k < span_len[s]; ++k) {
      for (uint32_t l = 0; l < pool_l.n_layers; ++l) {
        for (uint32_t kv = 0; kv < 2; ++kv) {
          const uint8_t *from = row_ptr(pool, pool_l, (uint64_t)span_src[s] + k, l, kv);
          uint8_t *to = (uint8_t *)row_ptr(dst, dst_l, (uint64_t)span_dst[s] + k, l, kv);
          if (kv == 0 && delta != 0) {
            for (uint32_t h = 0; h < H; ++h)
              cpo_rope_head((const uint16_t *)from + (size_t)h * D, (uint16_t *)to + (size_t)h * D,
                            D, delta, rope->theta, rope->style);
          } else {
            std::memcpy(to, from, row_bytes);
          }
        }
      }
    }
  }
}

// Sec. 4.1 "Workflow" (post-inference storing) and Sec. 4.3.5 (one copy of a
// duplicate): first occurrence in packed order owns the key.
static uint32_t insert_tokens(cpo_index *ix, const uint64_t *hash, const uint32_t *found,
                              const uint32_t *off, uint32_t R, const uint32_t *free_slots,
                              uint32_t n_free, const void *src, cpo_layout src_l, void *pool,
                              cpo_layout pool_l, int32_t *slot_pos, uint32_t *slot_out, uint32_t *flags,
                              const uint32_t *tok, uint32_t *slot_tok) {
  const size_t row_bytes = (size_t)pool_l.n_kv_heads * pool_l.head_dim * 2;
  // A table of bounded size: if it cannot take every key that the batch brings and it does not hold yet,
  // the batch stores nothing (keys already stored are still reported).
  bool table_full = false;
  if (ix->capacity) {
    std::unordered_set<uint64_t> fresh;
    for (uint32_t i = 0; i < off[R]; ++i)
      if (hash[i] != CPO_HASH_NONE && !(found && found[i] != CPO_SLOT_NONE) && !ix->entries.count(hash[i]))
        fresh.insert(hash[i]);
    table_full = ix->entries.size() + fresh.size() > ix->capacity;
    if (table_full && flags) *flags |= CPO_FLAG_TABLE_FULL;
  }
  uint32_t n_new = 0;
  for (uint32_t r = 0; r < R; ++r) {
    for (uint32_t i = off[r]; i < off[r + 1]; ++i) {
      slot_out[i] = CPO_SLOT_NONE;
      if (hash[i] == CPO_HASH_NONE) continue;
      if (found && found[i] != CPO_SLOT_NONE) {  // its text is in the pool already: kept once
        slot_out[i] = found[i];
        continue;
      }
      auto it = ix->map.find(hash[i]);
      if (it != ix->map.end()) {
        slot_out[i] = it->second;
        continue;
      }
      if (table_full) continue;
      ix->entries.insert(hash[i]);  // the key has its entry from now on, with or without a slot
      if (n_new == n_free) {
        if (flags) *flags |= CPO_FLAG_POOL_FULL;
        continue;
      }
      uint32_t s = free_slots[n_new++];
      ix->map.emplace(hash[i], s);
      slot_pos[s] = (int32_t)(i - off[r]);
      slot_out[i] = s;
      if (tok && slot_tok) slot_tok[s] = tok[i];
      for (uint32_t l = 0; l < pool_l.n_layers; ++l)
        for (uint32_t kv = 0; kv < 2; ++kv)
          std::memcpy((uint8_t *)row_ptr(pool, pool_l, s, l, kv), row_ptr(src, src_l, i, l, kv),
                      row_bytes);
    }
  }
  return n_new;
}

extern "C" uint32_t cpo_insert_kv(cpo_index *ix, const uint64_t *hash, const uint32_t *off,
                                  uint32_t R, const uint32_t *free_slots, uint32_t n_free,
                                  const void *src, cpo_layout src_l, void *pool, cpo_layout pool_l,
                                  int32_t *slot_pos, uint32_t *slot_out, uint32_t *flags,
                                  const uint32_t *tok, uint32_t *slot_tok) {
  return insert_tokens(ix, hash, nullptr, off, R, free_slots, n_free, src, src_l, pool, pool_l, slot_pos,
                       slot_out, flags, tok, slot_tok);
}

// Sec. 4.3.5 "Lifecycle management": a text that the pool already holds inside a longer stored text,
// or behind other text, is kept once.
extern "C" void cpo_insert_keys(const uint64_t *hash, const uint32_t *run_off, const uint32_t *const *seg_off,
                                const uint32_t *const *slot, uint32_t n_streams, uint32_t N, uint64_t base,
                                uint64_t *ins_hash_out, uint32_t *ins_off_out, uint32_t *found_out) {
  std::vector<uint64_t> pw((size_t)N + 1);
  pw[0] = 1;
  for (uint32_t k = 1; k <= N; ++k) pw[k] = pw[k - 1] * base;
  uint32_t c = 0;  // where the stored text that the current token continues starts
  for (uint32_t i = 0; i < N; ++i) {
    ins_hash_out[i] = CPO_HASH_NONE;
    ins_off_out[i] = 0xFFFFFFFFu;
    found_out[i] = CPO_SLOT_NONE;
    if (hash[i] == CPO_HASH_NONE) continue;
    if (run_off[i] == 0) c = i;  // a new run starts a text of its own ...
    for (uint32_t k = 0; k < n_streams; ++k)
      if (slot[k][i] != CPO_SLOT_NONE) {  // ... unless a lookup stream finds the token: then that text goes on
        found_out[i] = slot[k][i];
        c = i - seg_off[k][i];
        break;
      }
    ins_off_out[i] = i - c;
    const uint64_t before = run_off[c] == 0 ? 0 : hash[c - 1];
    const uint64_t h = hash[i] - before * pw[i - c + 1];
    ins_hash_out[i] = h == CPO_HASH_NONE ? CPO_HASH_NONE - 1 : h;
  }
}

extern "C" uint32_t cpo_insert_kv_dedup(cpo_index *ix, const uint64_t *ins_hash, const uint32_t *found,
                                        const uint32_t *off, uint32_t R, const uint32_t *free_slots,
                                        uint32_t n_free, const void *src, cpo_layout src_l, void *pool,
                                        cpo_layout pool_l, int32_t *slot_pos, uint32_t *slot_out,
                                        uint32_t *flags, const uint32_t *tok, uint32_t *slot_tok) {
  return insert_tokens(ix, ins_hash, found, off, R, free_slots, n_free, src, src_l, pool, pool_l, slot_pos,
                       slot_out, flags, tok, slot_tok);
}

// ---- floating anchors (Sec. 4.2.2 Step 1 and Step 2) -------------------------------------------

struct cpo_anchor_set {
  std::unordered_map<uint64_t, uint32_t> set;  // prefix hash -> slot of the run's W-th token
};

extern "C" cpo_anchor_set *cpo_anchor_set_new(void) { return new cpo_anchor_set(); }
extern "C" void cpo_anchor_set_free(cpo_anchor_set *a) { delete a; }
extern "C" uint64_t cpo_anchor_set_size(const cpo_anchor_set *a) { return a->set.size(); }

extern "C" void cpo_run_offsets(const uint8_t *mask, const uint32_t *off, uint32_t R,
                                uint32_t *run_off_out) {
  for (uint32_t r = 0; r < R; ++r) {
    uint32_t n = 0;  // non-sensitive tokens seen since the run started
    for (uint32_t i = off[r]; i < off[r + 1]; ++i) {
      if (mask[i]) {
        run_off_out[i] = 0xFFFFFFFFu;
        n = 0;
      } else {
        run_off_out[i] = n++;
      }
    }
  }
}

extern "C" void cpo_insert_anchors(cpo_anchor_set *as, const uint64_t *hash, const uint32_t *run_off,
                                   const uint32_t *slot, uint32_t N, uint32_t W) {
  for (uint32_t i = 0; i < N; ++i)
    if (hash[i] != CPO_HASH_NONE && run_off[i] == W - 1 && slot[i] != CPO_SLOT_NONE)
      as->set.emplace(hash[i], slot[i]);
}

extern "C" void cpo_hash_floating(const cpo_anchor_set *as, const cpo_index *ix, const uint64_t *hash,
                                  const uint32_t *run_off, uint32_t N, uint64_t base, uint32_t W,
                                  uint64_t *hash_a_out, uint32_t *off_a_out, uint64_t *hash_b_out,
                                  uint32_t *off_b_out) {
  // precomputed powers of the base
  std::vector<uint64_t> pw((size_t)N + 1);
  pw[0] = 1;
  for (uint32_t k = 1; k <= N; ++k) pw[k] = pw[k - 1] * base;
  // key of tokens a..i of one run, from the run's chain hashes: h[i] - h[a-1] * base^(i-a+1)
  auto sub = [&](uint32_t a, uint32_t i) {
    uint64_t before = run_off[a] == 0 ? 0 : hash[a - 1];
    uint64_t h = hash[i] - before * pw[i - a + 1];
    return h == CPO_HASH_NONE ? CPO_HASH_NONE - 1 : h;  // stored hashes never take the reserved value
  };
  for (uint32_t i = 0; i < N; ++i) {
    hash_a_out[i] = CPO_HASH_NONE;
    if (off_a_out) off_a_out[i] = 0xFFFFFFFFu;
    if (hash_b_out) hash_b_out[i] = CPO_HASH_NONE;
    if (off_b_out) off_b_out[i] = 0xFFFFFFFFu;
  }
  // run by run
  for (uint32_t s0 = 0; s0 < N;) {
    if (hash[s0] == CPO_HASH_NONE) {
      ++s0;
      continue;
    }
    uint32_t s1 = s0 + 1;  // the run is s0 .. s1-1
    while (s1 < N && hash[s1] != CPO_HASH_NONE && run_off[s1] != 0) ++s1;
    // Step 1: the candidates.  A window that starts at a (after the run's first token: there the
    // plain chain hash already is this key) and lies inside the run is compared with the stored
    // prefix hashes.
    std::vector<uint32_t> cand;
    for (uint32_t a = s0 + 1; a + W <= s1; ++a)
      if (as->set.count(sub(a, a + W - 1))) cand.push_back(a);
    // Step 2, pre-check by substring hashes: how far does the stored text that starts at candidate a
    // go on?  end[c] = 1 + the last token e such that every key (a .. j), a+W-1 <= j <= e, is stored:
    // candidate c covers the tokens cand[c] .. end[c]-1.
    std::vector<uint32_t> end(cand.size());
    for (size_t c = 0; c < cand.size(); ++c) {
      uint32_t e = cand[c] + W - 1;
      while (e + 1 < s1 && ix->map.count(sub(cand[c], e + 1))) ++e;
      end[c] = e + 1;
    }
    // Which candidate serves which token: the candidates' texts are laid over the run like intervals in
    // the textbook greedy cover.  A piece of covered text begins at the first candidate not yet passed;
    // then, as long as some candidate that starts inside the text covered so far reaches beyond it,
    // the one that reaches furthest (the earliest of those) is taken next.  Every token that any
    // candidate covers is then covered by a chosen one, and a chosen candidate overlaps only with the
    // one chosen before it and the one chosen after it, so giving the chosen candidates of a piece
    // alternately to stream a and stream b leaves each stream a sequence of whole texts that do not
    // overlap.  Each chosen candidate keys all of its tokens in its stream.
    size_t c = 0;
    while (c < cand.size()) {
      uint32_t stream = 0;  // a piece starts in stream a
      for (;;) {
        for (uint32_t i = cand[c]; i < end[c]; ++i) {
          uint64_t *h = stream == 0 ? hash_a_out : hash_b_out;
          uint32_t *o = stream == 0 ? off_a_out : off_b_out;
          if (h) h[i] = sub(cand[c], i);
          if (o) o[i] = i - cand[c];
        }
        size_t best = cand.size();
        for (size_t d = c + 1; d < cand.size() && cand[d] < end[c]; ++d)
          if (end[d] > end[c] && (best == cand.size() || end[d] > end[best])) best = d;
        if (best == cand.size()) break;
        c = best;
        stream ^= 1u;
      }
      const uint32_t covered_to = end[c];  // nothing that starts before this reaches further
      while (c < cand.size() && cand[c] < covered_to) ++c;
    }
    s0 = s1;
  }
}

extern "C" void cpo_probe3(const cpo_index *ix, const uint64_t *hash_a, const uint64_t *hash_b,
                           const uint64_t *hash_c, uint32_t N, uint32_t *slot_out) {
  for (uint32_t i = 0; i < N; ++i) {
    slot_out[i] = CPO_SLOT_NONE;
    for (const uint64_t *keys : {hash_a, hash_b, hash_c}) {
      if (slot_out[i] != CPO_SLOT_NONE || keys == nullptr || keys[i] == CPO_HASH_NONE) continue;
      auto it = ix->map.find(keys[i]);
      if (it != ix->map.end()) slot_out[i] = it->second;
    }
  }
}

// ---- exact verification -------------------------------------------------------------------------

struct cpo_text {
  std::vector<uint32_t> archive;  // every token of every recorded batch, in arrival order
  std::vector<uint64_t> last;     // per slot: archive index of the slot's own token
  std::vector<uint32_t> len;      // per slot: length of the text (0 = none yet, 0xFFFFFFFF = never matches)
};

extern "C" cpo_text *cpo_text_new(uint32_t n_slots) {
  cpo_text *t = new cpo_text;
  t->last.assign(n_slots, 0);
  t->len.assign(n_slots, 0);
  return t;
}
extern "C" void cpo_text_free(cpo_text *t) { delete t; }

// Does slot s hold exactly the `n` tokens that end at tok[i]?  Compared one token at a time.
static bool text_equals(const cpo_text *t, uint32_t s, const uint32_t *tok, uint32_t i, uint32_t n) {
  if (s >= t->len.size() || t->len[s] != n) return false;
  for (uint32_t k = 0; k < n; ++k)
    if (t->archive[t->last[s] - k] != tok[i - k]) return false;
  return true;
}

static void text_record(cpo_text *t, const uint32_t *tok, const uint32_t *run_off, const uint32_t *found,
                        uint32_t N, uint32_t *slot_out) {
  const uint64_t base = t->archive.size();
  t->archive.insert(t->archive.end(), tok, tok + N);
  bool prev_ok = false;
  for (uint32_t i = 0; i < N; ++i) {
    if (run_off[i] == 0xFFFFFFFFu) {  // sensitive
      prev_ok = false;
      continue;
    }
    const bool start_ok = run_off[i] == 0 || prev_ok;
    const uint32_t s = slot_out[i], n = run_off[i] + 1;
    bool ok = false;
    if (found && found[i] != CPO_SLOT_NONE) {
      // a token that a confirmed lookup found: its slot holds exactly the n tokens that end here
      ok = text_equals(t, s, tok, i, n);
    } else if (s < t->len.size()) {
      if (t->len[s] == 0) {  // a slot filled by this batch, seen at its first (storing) token
        if (start_ok) {
          t->last[s] = base + i;
          t->len[s] = n;
          ok = true;
        } else {
          t->len[s] = 0xFFFFFFFFu;  // stored behind a prefix that was not verified: unusable
        }
      } else {
        ok = start_ok && text_equals(t, s, tok, i, n);
      }
    }
    if (!ok) slot_out[i] = CPO_SLOT_NONE;
    prev_ok = ok;
  }
}

extern "C" void cpo_text_record(cpo_text *t, const uint32_t *tok, const uint32_t *run_off, uint32_t N,
                                uint32_t *slot_out) {
  text_record(t, tok, run_off, nullptr, N, slot_out);
}

extern "C" void cpo_text_record_dedup(cpo_text *t, const uint32_t *tok, const uint32_t *ins_off,
                                      const uint32_t *found, uint32_t N, uint32_t *slot_out) {
  text_record(t, tok, ins_off, found, N, slot_out);
}

extern "C" void cpo_verify(const cpo_text *t, const uint32_t *tok, const uint32_t *seg_off,
                           const uint32_t *cand, uint32_t N, int merge, uint32_t *slot_out) {
  bool prev_ok = false;
  for (uint32_t i = 0; i < N; ++i) {
    bool ok = false;
    if (seg_off[i] != 0xFFFFFFFFu && (seg_off[i] == 0 || prev_ok))
      ok = text_equals(t, cand[i], tok, i, seg_off[i] + 1);
    prev_ok = ok;
    const uint32_t r = ok ? cand[i] : CPO_SLOT_NONE;
    if (!merge || slot_out[i] == CPO_SLOT_NONE) slot_out[i] = r;
  }
}

extern "C" void cpo_probe2(const cpo_index *ix, const uint64_t *hash_a, const uint64_t *hash_b,
                           uint32_t N, uint32_t *slot_out) {
  for (uint32_t i = 0; i < N; ++i) {
    slot_out[i] = CPO_SLOT_NONE;
    for (const uint64_t *h : {hash_a, hash_b}) {
      if (h[i] == CPO_HASH_NONE) continue;
      auto it = ix->map.find(h[i]);
      if (it != ix->map.end()) {
        slot_out[i] = it->second;
        break;
      }
    }
  }
}

// ---- pool policies ------------------------------------------------------------------------------

// Sec. 4.2.1 "Optimization": a reusable segment must have a minimum length.  Step 3: tokens marked
// for recomputation are not reused.  One pass per request: find each maximal stretch of matched
// tokens, drop it when it is too short, else drop only its marked tokens.
extern "C" void cpo_filter_matches(const uint32_t *slot_in, const uint32_t *off, uint32_t R,
                                   uint32_t min_len, const uint8_t *slot_recompute,
                                   uint32_t n_pool_slots, uint32_t *slot_out) {
  for (uint32_t r = 0; r < R; ++r) {
    uint32_t i = off[r];
    while (i < off[r + 1]) {
      if (slot_in[i] == CPO_SLOT_NONE) {
        slot_out[i++] = CPO_SLOT_NONE;
        continue;
      }
      uint32_t e = i;
      while (e < off[r + 1] && slot_in[e] != CPO_SLOT_NONE) ++e;  // stretch [i, e)
      for (uint32_t k = i; k < e; ++k) {
        uint32_t s = slot_in[k];
        bool keep = e - i >= min_len;
        if (keep && slot_recompute && s < n_pool_slots && slot_recompute[s]) keep = false;
        slot_out[k] = keep ? s : CPO_SLOT_NONE;
      }
      i = e;
    }
  }
}

extern "C" void cpo_mark_recompute(const uint32_t *slot, const uint8_t *recompute, uint32_t N,
                                   uint32_t n_pool_slots, uint8_t *slot_recompute) {
  for (uint32_t i = 0; i < N; ++i)
    if (slot[i] < n_pool_slots && recompute[i]) slot_recompute[slot[i]] = 1;
}

// Sec. 4.3.1 "Operational details": tokens that are not linked are zero placeholders.
extern "C" void cpo_fill_unmatched(const uint32_t *slot, uint32_t N, void *dst, cpo_layout dst_l) {
  const size_t row_bytes = (size_t)dst_l.n_kv_heads * dst_l.head_dim * 2;
  for (uint32_t i = 0; i < N; ++i) {
    if (slot[i] != CPO_SLOT_NONE) continue;
    for (uint32_t l = 0; l < dst_l.n_layers; ++l)
      for (uint32_t kv = 0; kv < 2; ++kv) std::memset((uint8_t *)row_ptr(dst, dst_l, i, l, kv), 0, row_bytes);
  }
}

// Sec. 4.3.5 "Lifecycle management": least-recently-used eviction.  Every slot remembers the
// number (epoch) of the last batch that used it; 0 = the slot is free.
extern "C" void cpo_touch(const uint32_t *slot, uint32_t N, uint32_t epoch, uint32_t n_pool_slots,
                          uint32_t *slot_stamp) {
  for (uint32_t i = 0; i < N; ++i)
    if (slot[i] < n_pool_slots && slot_stamp[slot[i]] < epoch) slot_stamp[slot[i]] = epoch;
}

extern "C" uint32_t cpo_lru_threshold(const uint32_t *slot_stamp, uint32_t n_pool_slots,
                                      uint32_t epoch_now, uint32_t n_needed, uint32_t max_age) {
  if (n_needed == 0) return 0;
  // oldest first: all slots of age >= a go together; ages of max_age - 1 and more are one class
  for (int64_t a = (int64_t)max_age - 1; a >= 0; --a) {
    int64_t T = (int64_t)epoch_now - a + 1;  // "last used before epoch T"
    if (T <= 1) continue;
    uint64_t n = 0;
    for (uint32_t s = 0; s < n_pool_slots; ++s)
      if (slot_stamp[s] != 0 && (int64_t)slot_stamp[s] < T) ++n;
    if (n >= n_needed) return (uint32_t)T;
  }
  return epoch_now + 1;  // not enough even so: everything that is in use goes
}

extern "C" uint32_t cpo_evict(cpo_index *ix, uint32_t *slot_stamp, uint32_t n_pool_slots,
                              uint32_t threshold, uint32_t *freed_slots, cpo_text *text,
                              uint8_t *slot_recompute, cpo_anchor_set *anchors) {
  std::vector<uint8_t> gone(n_pool_slots, 0);
  uint32_t n = 0;
  for (uint32_t s = 0; s < n_pool_slots; ++s) {
    if (slot_stamp[s] == 0 || slot_stamp[s] >= threshold) continue;
    gone[s] = 1;
    freed_slots[n++] = s;  // ascending slot order
    slot_stamp[s] = 0;
    if (slot_recompute) slot_recompute[s] = 0;
    if (text) text->len[s] = 0;
  }
  for (auto it = ix->map.begin(); it != ix->map.end();)
    it = (it->second < n_pool_slots && gone[it->second]) ? ix->map.erase(it) : std::next(it);
  if (anchors)
    for (auto it = anchors->set.begin(); it != anchors->set.end();)
      it = (it->second < n_pool_slots && gone[it->second]) ? anchors->set.erase(it) : std::next(it);
  return n;
}

// ---- KV annotator: summed-area table over the attention matrix (Sec. 4.2.1, Steps 1-3) ----------

// Fixed-point image of an attention weight: x * 2^32 rounded to the nearest integer (ties to even).
// Entries above the diagonal (a token does not attend to later tokens) and values that are not
// finite or not in [-2^18, 2^18] count as 0.
static int64_t quantise(float x, uint32_t i, uint32_t j) {
  if (j > i || !(std::fabs(x) <= 262144.0f)) return 0;
  return (int64_t)std::nearbyint((double)x * 4294967296.0);  // default rounding mode: to nearest even
}

// Step 1: T[i,j] = A[i,j] + T[i-1,j] + T[i,j-1] - T[i-1,j-1], indices below 0 count as zero.
extern "C" void cpo_sat_build(const float *attn, uint32_t n, uint64_t ld, int64_t *T) {
  for (uint32_t i = 0; i < n; ++i)
    for (uint32_t j = 0; j < n; ++j) {
      int64_t up = i ? T[(uint64_t)(i - 1) * n + j] : 0;
      int64_t left = j ? T[(uint64_t)i * n + j - 1] : 0;
      int64_t diag = (i && j) ? T[(uint64_t)(i - 1) * n + j - 1] : 0;
      T[(uint64_t)i * n + j] = quantise(attn[(uint64_t)i * ld + j], i, j) + up + left - diag;
    }
}

// Sum of the original matrix over rows x1..x2 and columns y1..y2 (inclusive; an empty range gives 0).
static int64_t rect(const int64_t *T, uint32_t n, int64_t x1, int64_t x2, int64_t y1, int64_t y2) {
  if (x2 < x1 || y2 < y1) return 0;
  auto at = [&](int64_t x, int64_t y) -> int64_t { return (x < 0 || y < 0) ? 0 : T[(uint64_t)x * n + y]; };
  return at(x2, y2) - at(x1 - 1, y2) - at(x2, y1 - 1) + at(x1 - 1, y1 - 1);
}

extern "C" int64_t cpo_sat_rect(const int64_t *T, uint32_t n, int64_t x1, int64_t x2, int64_t y1,
                                int64_t y2) {
  return rect(T, n, x1, x2, y1, y2);
}

// Steps 2 and 3 for every coarse segment (maximal run of tokens with mask 0).
extern "C" void cpo_annotate(const int64_t *T, uint32_t n, const uint8_t *mask, uint32_t min_len,
                             uint32_t rho_percent, uint32_t *best_l, uint32_t *best_r,
                             int64_t *best_score, uint8_t *reusable, uint8_t *recompute) {
  for (uint32_t i = 0; i < n; ++i) {
    best_l[i] = best_r[i] = 0xFFFFFFFFu;
    best_score[i] = 0;
    reusable[i] = recompute[i] = 0;
  }
  if (min_len == 0) min_len = 1;
  uint32_t a = 0;
  while (a < n) {
    if (mask[a]) {
      ++a;
      continue;
    }
    uint32_t b = a;
    while (b + 1 < n && !mask[b + 1]) ++b;  // coarse segment [a, b]
    // Step 2: the substring with the largest intra - inter attention; the first one on ties
    bool found = false;
    int64_t best = 0;
    uint32_t bl = 0, br = 0;
    for (uint32_t l = a; l <= b; ++l)
      for (uint32_t r = l; r <= b; ++r) {
        if (r - l + 1 < min_len) continue;
        int64_t intra = rect(T, n, l, r, l, r);                // rows l..r, columns l..r
        int64_t inter = rect(T, n, l, r, 0, (int64_t)l - 1);   // rows l..r, columns before l
        int64_t score = intra - inter;
        if (!found || score > best) {
          found = true;
          best = score;
          bl = l;
          br = r;
        }
      }
    if (found)
      for (uint32_t i = a; i <= b; ++i) {
        best_l[i] = bl;
        best_r[i] = br;
        best_score[i] = best;
      }
    // Reuse criterion: a substring is reusable if its intra-attention exceeds its inter-attention.
    if (found && best > 0) {
      // Step 3: rank the tokens of the chosen substring by inter - intra attention (their own row),
      // largest first, earlier token first on ties; the top rho percent are recomputed
      const uint32_t len = br - bl + 1;
      std::vector<int64_t> d(len);
      for (uint32_t i = bl; i <= br; ++i) {
        int64_t inter_i = rect(T, n, i, i, 0, (int64_t)bl - 1);
        int64_t intra_i = rect(T, n, i, i, bl, i);
        d[i - bl] = inter_i - intra_i;
        reusable[i] = 1;
      }
      std::vector<uint32_t> order(len);
      for (uint32_t k = 0; k < len; ++k) order[k] = k;
      std::stable_sort(order.begin(), order.end(), [&](uint32_t x, uint32_t y) { return d[x] > d[y]; });
      const uint32_t n_marked = (uint32_t)((uint64_t)len * rho_percent / 100);
      for (uint32_t k = 0; k < n_marked; ++k) recompute[bl + order[k]] = 1;
    }
    a = b + 1;
  }
}
