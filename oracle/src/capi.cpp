// TEST INFRASTRUCTURE ONLY: C entry points of the slow CPU oracle, loaded
// with ctypes by the tests, the smoke check and the benchmark's CPU-baseline
// leg.  The product library never links or calls this.
#include <cstring>
#include <memory>
#include <string>
#include <thread>
#include <vector>

#include "earley.hpp"
#include "grammar.hpp"
#include "pda.hpp"

namespace {

thread_local std::string g_error;

struct GrammarBox {
  orc::Grammar g;
  orc::Bnf bnf;
  orc::Nfa nfa;
};
struct EarleyBox {
  const GrammarBox* g;
  orc::Earley e;
};
struct PdaBox {
  const GrammarBox* g;
  orc::Pda pda;
  orc::ConfigSet cur;
};
struct PosBox {
  int rule;
  std::set<int> pos;
};

template <class F>
void for_tokens(int64_t V, int nthreads, F fn) {
  if (nthreads < 1) nthreads = 1;
  std::vector<std::thread> pool;
  std::vector<std::string> errs(nthreads);
  for (int t = 0; t < nthreads; ++t)
    pool.emplace_back([&, t] {
      try {
        for (int64_t i = t; i < V; i += nthreads) fn(i);
      } catch (const std::exception& ex) { errs[t] = ex.what(); }
    });
  for (auto& th : pool) th.join();
  for (auto& e : errs)
    if (!e.empty()) throw std::runtime_error(e);
}

}  // namespace

#define ORC_TRY try {
#define ORC_CATCH(ret) } catch (const std::exception& ex) { g_error = ex.what(); return ret; }

extern "C" {

const char* orc_last_error() { return g_error.c_str(); }

void* orc_grammar_new(const char* text, int64_t len, const char* root) {
  ORC_TRY
  auto box = std::make_unique<GrammarBox>();
  box->g = orc::read_grammar(std::string(text, (size_t)len), root);
  box->bnf = orc::BnfBuilder(box->g).build();
  box->nfa = orc::NfaBuilder(box->g).build();
  return box.release();
  ORC_CATCH(nullptr)
}
void orc_grammar_free(void* g) { delete (GrammarBox*)g; }

int orc_rule_index(void* g, const char* name) {
  auto& m = ((GrammarBox*)g)->g.rule_index;
  auto it = m.find(name);
  return it == m.end() ? -1 : it->second;
}
int orc_num_rules(void* g) { return (int)((GrammarBox*)g)->g.rule_names.size(); }
// 256 flags: out[c] = 1 iff byte c can come right after an instance of the rule
int orc_follow(void* g, int rule, unsigned char* out) {
  auto& f = ((GrammarBox*)g)->nfa.follow;
  if (rule < 0 || rule >= (int)f.size()) return -1;
  for (int c = 0; c < 256; ++c) out[c] = f[rule].test(c) ? 1 : 0;
  return 0;
}

// 0 = not a viable prefix, 1 = viable prefix but not a sentence, 2 = sentence
int orc_recognize(void* g, const unsigned char* bytes, int64_t n) {
  ORC_TRY
  orc::Earley e(&((GrammarBox*)g)->bnf);
  if (!e.advance(bytes, (int)n)) return 0;
  return e.complete() ? 2 : 1;
  ORC_CATCH(-1)
}
// the same question answered by the literal pushdown automaton
int orc_recognize_pda(void* g, const unsigned char* bytes, int64_t n) {
  ORC_TRY
  orc::Pda pda(&((GrammarBox*)g)->nfa);
  orc::ConfigSet cur = pda.run(pda.initial(), bytes, (int)n);
  if (cur.empty()) return 0;
  return pda.is_sentence_state(cur) ? 2 : 1;
  ORC_CATCH(-1)
}

// ---- O1: Earley matcher over the text accepted so far
void* orc_earley_new(void* g) {
  ORC_TRY
  return new EarleyBox{(GrammarBox*)g, orc::Earley(&((GrammarBox*)g)->bnf)};
  ORC_CATCH(nullptr)
}
void* orc_earley_clone(void* m) { return new EarleyBox(*(EarleyBox*)m); }
void orc_earley_free(void* m) { delete (EarleyBox*)m; }
int orc_earley_advance(void* m, const unsigned char* bytes, int64_t n) {
  ORC_TRY
  return ((EarleyBox*)m)->e.advance(bytes, (int)n) ? 1 : 0;
  ORC_CATCH(-1)
}
int orc_earley_complete(void* m) { return ((EarleyBox*)m)->e.complete() ? 1 : 0; }
int orc_earley_length(void* m) { return ((EarleyBox*)m)->e.length(); }
// out[i] = 1 iff token i (non-empty) keeps the text a viable prefix
int orc_earley_mask(void* m, const unsigned char* data, const int64_t* offsets, int64_t V,
                    unsigned char* out, int nthreads) {
  ORC_TRY
  const orc::Earley& e = ((EarleyBox*)m)->e;
  for_tokens(V, nthreads, [&](int64_t i) {
    int64_t n = offsets[i + 1] - offsets[i];
    out[i] = (n > 0 && e.probe(data + offsets[i], (int)n)) ? 1 : 0;
  });
  return 0;
  ORC_CATCH(-1)
}
int64_t orc_earley_completion(void* m, unsigned char* out, int64_t cap) {
  ORC_TRY
  std::string s = ((EarleyBox*)m)->e.completion();
  if ((int64_t)s.size() > cap) throw std::runtime_error("completion buffer too small");
  std::memcpy(out, s.data(), s.size());
  return (int64_t)s.size();
  ORC_CATCH(-1)
}

// ---- O2: literal pushdown automaton matcher
void* orc_pda_new(void* g) {
  ORC_TRY
  auto* gb = (GrammarBox*)g;
  auto box = std::make_unique<PdaBox>(PdaBox{gb, orc::Pda(&gb->nfa), {}});
  box->cur = box->pda.initial();
  return box.release();
  ORC_CATCH(nullptr)
}
void orc_pda_free(void* m) { delete (PdaBox*)m; }
int orc_pda_advance(void* m, const unsigned char* bytes, int64_t n) {
  ORC_TRY
  auto* b = (PdaBox*)m;
  orc::ConfigSet nxt = b->pda.run(b->cur, bytes, (int)n);
  if (nxt.empty()) return 0;
  b->cur = std::move(nxt);
  return 1;
  ORC_CATCH(-1)
}
int orc_pda_complete(void* m) {
  ORC_TRY
  auto* b = (PdaBox*)m;
  return b->pda.is_sentence_state(b->cur) ? 1 : 0;
  ORC_CATCH(-1)
}
int orc_pda_num_configs(void* m) { return (int)((PdaBox*)m)->cur.size(); }
int orc_pda_mask(void* m, const unsigned char* data, const int64_t* offsets, int64_t V,
                 unsigned char* out, int nthreads) {
  ORC_TRY
  auto* b = (PdaBox*)m;
  for_tokens(V, nthreads, [&](int64_t i) {
    int64_t n = offsets[i + 1] - offsets[i];
    out[i] = (n > 0 && !b->pda.run(b->cur, data + offsets[i], (int)n).empty()) ? 1 : 0;
  });
  return 0;
  ORC_CATCH(-1)
}
// mask of one configuration alone (for the union-over-stacks property)
int orc_pda_mask_single(void* m, int which, const unsigned char* data, const int64_t* offsets,
                        int64_t V, unsigned char* out, int nthreads) {
  ORC_TRY
  auto* b = (PdaBox*)m;
  auto it = b->cur.begin();
  std::advance(it, which);
  orc::ConfigSet one{*it};
  for_tokens(V, nthreads, [&](int64_t i) {
    int64_t n = offsets[i + 1] - offsets[i];
    out[i] = (n > 0 && !b->pda.run(one, data + offsets[i], (int)n).empty()) ? 1 : 0;
  });
  return 0;
  ORC_CATCH(-1)
}

// ---- positions inside a rule and their three-way token classes
void* orc_positions(void* g, int rule, const int32_t* symbols, int n) {
  ORC_TRY
  auto* gb = (GrammarBox*)g;
  orc::Pda pda(&gb->nfa);
  return new PosBox{rule, pda.positions(rule, symbols, n)};
  ORC_CATCH(nullptr)
}
void orc_positions_free(void* p) { delete (PosBox*)p; }
int orc_positions_size(void* p) { return (int)((PosBox*)p)->pos.size(); }
// out[i]: 0 rejected, 2 accepted, 1 uncertain (context-dependent) also after the
// one-byte narrowing, 4 uncertain by section 3.1 alone
int orc_classify(void* g, void* p, const unsigned char* data, const int64_t* offsets, int64_t V,
                 unsigned char* out, int nthreads) {
  ORC_TRY
  auto* gb = (GrammarBox*)g;
  orc::Pda pda(&gb->nfa);
  const std::set<int>& pos = ((PosBox*)p)->pos;
  const int rule = ((PosBox*)p)->rule;
  for_tokens(V, nthreads, [&](int64_t i) {
    out[i] = (unsigned char)pda.classify(rule, pos, data + offsets[i], (int)(offsets[i + 1] - offsets[i]));
  });
  return 0;
  ORC_CATCH(-1)
}

}  // extern "C"
