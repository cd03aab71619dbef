// The token walk shared by the classify and fill kernels.  It is plain C++
// over the flattened tables, so the same code also compiles for the host,
// where the library's tests run it against the CPU oracle without a GPU.
#pragma once
#include <hip/hip_runtime_api.h>
#include <hip/hip_vector_types.h>

#include <cstdint>

#include "kernels.hpp"

#if defined(__HIPCC__) || defined(__HIP__)
#define XGM_HD __host__ __device__ __forceinline__
#else
#define XGM_HD inline
#endif

namespace xgm {

constexpr uint32_t kAltFlagD = 0x8000;
constexpr uint32_t kMoveTagD = 0xFFFF;
constexpr uint32_t kTailTagD = 0xFFFE;
constexpr uint32_t kLiveBase = 0x8000;  // stack handles >= this refer to the request's live frames

// Table access for the walk: at node n on byte c, how many move / call
// alternatives are there (k), which (a single packed one, or k entries in the
// alternatives pool from `base`), may the rule end at n (fin), and can c come
// right after an instance of n's rule at all (after).
struct CompactTab {
  TabView v;
  XGM_HD void lookup(uint32_t n, uint32_t c, uint32_t& k, uint32_t& single, uint32_t& base, bool& pooled,
                     uint32_t& fin, uint32_t& after) const {
    const uint2 h = (n < (uint32_t)v.n_near) ? v.hdr_near[n] : v.hdr_far[n];
    k = 0; single = 0; base = 0; pooled = false;
    fin = h.y & 1u;
    after = (v.follow_rules[(h.y >> 16) * 8 + (c >> 5)] >> (c & 31)) & 1u;
    if (h.y & 2u) {
      const uint32_t si = v.shapes[(h.x & 0xFFFFu) * v.n_cls + v.cls[c]];
      if (si != 0xFFu) {
        const uint32_t a = v.targets[(h.x >> 16) + si];
        if (a < 0x8000u) { k = 1; single = (0xFFFFu << 16) | a; }
        else { base = a & 0x7FFFu; k = v.alts[base]; pooled = true; }
      }
    } else {
      const uint32_t lo = h.x & 0xFFu, hi = (h.x >> 8) & 0xFFu;
      if (c >= lo && c <= hi) { k = 1; single = (0xFFFFu << 16) | (h.x >> 16); }
    }
  }
  XGM_HD uint32_t alt(uint32_t idx) const { return v.alts[idx]; }
  XGM_HD bool is_final(uint32_t n) const { return ((n < (uint32_t)v.n_near) ? v.hdr_near[n] : v.hdr_far[n]).y & 1u; }
  XGM_HD bool is_dead_end(uint32_t n) const { return ((n < (uint32_t)v.n_near) ? v.hdr_near[n] : v.hdr_far[n]).y & 4u; }
  // the rule of node n, as the handle of its 256-bit FOLLOW set; is byte c in the set of rule r?
  XGM_HD uint32_t follow_of(uint32_t n) const { return ((n < (uint32_t)v.n_near) ? v.hdr_near[n] : v.hdr_far[n]).y >> 16; }
  XGM_HD uint32_t follows(uint32_t r, uint32_t c) const { return (v.follow_rules[r * 8 + (c >> 5)] >> (c & 31)) & 1u; }
};

// The first 15 bytes of a token as four plain words (kept in registers: the
// byte at a run-time index is picked with selects, never through memory).
struct TokenWords {
  uint32_t w0, w1, w2, w3;
  XGM_HD explicit TokenWords(const uint4& tk) : w0(tk.x), w1(tk.y), w2(tk.z), w3(tk.w) {}
};
XGM_HD uint32_t token_byte(const TokenWords& t, const uint8_t* ext, int i) {
  if (i < 15) {
    // bit masks instead of selects: a select between loaded values invites the
    // compiler to index a copy in scratch memory
    const uint32_t m4 = 0u - (((uint32_t)i >> 2) & 1u), m8 = 0u - (((uint32_t)i >> 3) & 1u);
    const uint32_t lo = (t.w1 & m4) | (t.w0 & ~m4), hi = (t.w3 & m4) | (t.w2 & ~m4);
    const uint32_t w = (hi & m8) | (lo & ~m8);
    return (w >> (((uint32_t)i & 3u) * 8u)) & 0xFFu;
  }
  return ext[i];
}
XGM_HD uint32_t token_byte(const uint4& tk, const uint8_t* ext, int i) { return token_byte(TokenWords(tk), ext, i); }

// Depth-first walk of one token through the pushdown automaton (section 2.2,
// Appendix A) from the configuration (node on top, `depth - 1` live frames
// below it).  Alternatives at a configuration, in the order they are tried:
// the byte edge, the rule references whose callee can start with the next
// byte (push the return node, enter the callee), and - if the node is
// accepting and a byte was consumed since the last push - the return to the
// frame below.  When the walk only has to decide whether the token is allowed
// (BUILD = false), a return in front of a byte that can never follow the
// node's rule is not tried at all: it cannot lead anywhere, and leaving it out
// keeps runs like the inside of a string free of pending alternatives.  Frames pushed during the walk live in a small arena with
// parent links, so that backing up to a pending alternative never copies a
// stack (the persistent stack of section 3.3, in miniature).
//
// BUILD = true:  nothing is known below the start frame (depth must be 1);
//                result kAccept / kUncertain / kReject as in section 3.1,
//                refined by one byte of context (section 3.2 in miniature):
//                leaving the start frame while bytes remain only counts if
//                the next byte is in the FOLLOW set of rule `follow` (the bytes
//                that can come right after an instance of the start node's rule
//                in any context; `T.follow_of(start_node)`); a token that left the frame only in front of other
//                bytes is kUncertainPlain: context-dependent by section 3.1
//                alone, rejected in every context by the refinement.
// BUILD = false: frames below are live[0 .. depth-2]; result kAccept (token
//                allowed) or kReject.
// kOverflow: a limit was hit; the caller records the pair.
// `steps_out` (may be null) receives the number of automaton steps taken.
// `i0`: index of the first byte to consume (the walk may start inside the token).
// `exits_out` (BUILD only, may be null): bit min(k, 31) is set for every
// position k at which the start frame is left in front of a byte of `follow`.
// `Live` is anything indexable that yields the live frames (a plain pointer,
// or a view that knows which of them sit in LDS).
// `End` decides what the end of the token means.  The default returns kAccept
// at the first path that consumes every byte.  An enumerating End is instead
// called with every configuration (node, stack handle, arena, live frames) in
// which the token can end, and the walk goes on to the next path; the result
// is then kReject (or kOverflow).
struct FirstPathEnds {
  static constexpr bool kEnumerate = false;
  template <class Live>
  XGM_HD void operator()(uint32_t, uint32_t, const uint32_t*, const Live&) const {}
};
template <bool BUILD, class Tab, class Live, class End = FirstPathEnds>
XGM_HD int walk_token(const Tab& T, const uint4 tk, const uint8_t* ext, const int len,
                      const uint32_t start_node, const Live& live, const uint32_t depth,
                      uint32_t* steps_out = nullptr, const uint32_t follow = 0u, const int i0 = 0,
                      uint32_t* exits_out = nullptr, const End& at_end = End()) {
  if (len > kMaxTokenLen) return kOverflow;
  const TokenWords tw(tk);
  uint32_t arena[kArenaFrames];  // ret | parent handle << 16
  uint2 choice[kChoicePoints];   // x = node | sp << 16 ; y = i | alt << 8 | top << 16 | f << 24
  uint32_t n = start_node, sp = kLiveBase + depth - 1, f = 1, alt = 0, top = 0, csp = 0;
  int i = i0;
  uint32_t left_frame = 0u;  // bit 0: the start frame was left with bytes remaining, bit 1: in front of a byte of `follow`
  for (int steps = 0;; ++steps) {
    if (steps_out) *steps_out = (uint32_t)steps;
    if (i == len && !End::kEnumerate) return kAccept;
    if (steps >= kMaxSteps) return kOverflow;
    bool advanced = false;
    if (i == len) {
      at_end(n, sp, arena, live);      // then on to the next path
    } else {
      const uint32_t c = token_byte(tw, ext, i);
      uint32_t k, single, base, fin, after;
      bool pooled;
      T.lookup(n, c, k, single, base, pooled, fin, after);
      uint32_t can_pop = fin & f;
      if (BUILD && can_pop && sp == kLiveBase) {
        // The start frame may end here (nothing is known below it): noted at once instead of kept as a
        // pending alternative, so that a run through a rule that may end after every byte (the inside of
        // a string, a number) leaves nothing to come back to.
        const uint32_t fo = T.follows(follow, c);
        left_frame |= 1u | (fo << 1);
        if (exits_out && fo) *exits_out |= 1u << (i < 31 ? i : 31);
        can_pop = 0u;
      }
      if (!BUILD) can_pop &= after;  // a return in front of a byte that can never follow the rule leads nowhere
      const uint32_t total = k + can_pop;
      // nothing but a move along a byte edge (most steps inside a string, a number, a name): taken at once
      if (alt == 0u && total == 1u && k == 1u && !pooled) {
        n = single & 0xFFFFu;
        ++i;
        f = 1;
        continue;
      }
      if (alt < total) {
        bool ok = true;
        if (alt + 1 < total) {
          if (csp == kChoicePoints) return kOverflow;
          choice[csp++] = make_uint2(n | (sp << 16), (uint32_t)i | ((alt + 1) << 8) | (top << 16) | (f << 24));
        }
        if (alt < k) {
          const uint32_t e = pooled ? T.alt(base + 1 + alt) : single;
          const uint32_t tag = e >> 16, dst = e & 0xFFFFu;
          if (tag == kMoveTagD) { n = dst; ++i; f = 1; }
          else if (tag == kTailTagD) { n = dst; f = 0; }  // enter the callee, it returns to our parent
          else {
            if (top == kArenaFrames) return kOverflow;
            arena[top] = tag | (sp << 16);
            sp = top++;
            n = dst;
            f = 0;
          }
        } else if (sp < kLiveBase) {   // return into a frame pushed during this walk
          const uint32_t fr = arena[sp], old = sp;
          n = fr & 0xFFFFu;
          sp = fr >> 16;
          // frames from `old` upwards are garbage unless a pending alternative still needs them
          if (csp == 0 || ((choice[csp - 1].y >> 16) & 0xFFu) <= old) top = old;
        } else {                       // return into a live frame
          const uint32_t d = sp - kLiveBase;
          if (d == 0) {                // nothing below: the end of the root rule (BUILD notes this case above)
            ok = false;
          } else {
            n = live[d - 1];
            sp = kLiveBase + d - 1;
          }
        }
        if (ok) { alt = 0; advanced = true; }
      }
    }
    if (!advanced) {                 // back up to the most recent pending alternative
      if (csp == 0) break;
      const uint2 ch = choice[--csp];
      n = ch.x & 0xFFFFu;
      sp = ch.x >> 16;
      i = (int)(ch.y & 0xFFu);
      alt = (ch.y >> 8) & 0xFFu;
      top = (ch.y >> 16) & 0xFFu;
      f = (ch.y >> 24) & 1u;
    }
  }
  if (BUILD && left_frame) return (left_frame & 2u) ? kUncertain : kUncertainPlain;
  return kReject;
}

// End policy that writes out the stack of every configuration a token can end
// in (section 3.3: the sampled token moves every parallel stack on).  A top
// node that can only return is returned from first, so that equal states get
// equal stacks.  A stack goes to the slot that `sink.claim()` hands out:
//   sink.frames  [capacity][max_depth] uint16, bottom frame first, the current node last
//   sink.depth   [capacity]
// A stack deeper than max_depth, or more stacks than capacity, set *sink.overflow.
// The same stack may be written more than once (several paths): the caller
// removes duplicates.
template <class Tab, class Sink>
struct CollectStacks {
  static constexpr bool kEnumerate = true;
  const Tab* T;
  Sink* sink;
  template <class Live>
  XGM_HD void operator()(uint32_t n, uint32_t sp, const uint32_t* arena, const Live& live) const {
    while (T->is_dead_end(n)) {
      if (sp < kLiveBase) {
        const uint32_t fr = arena[sp];
        n = fr & 0xFFFFu;
        sp = fr >> 16;
      } else {
        const uint32_t d = sp - kLiveBase;
        if (d == 0) break;
        n = live[d - 1];
        sp = kLiveBase + d - 1;
      }
    }
    uint32_t depth = 1, h = sp;
    for (; h < kLiveBase; h = arena[h] >> 16) ++depth;
    const uint32_t d = h - kLiveBase;  // live frames kept
    depth += d;
    if (depth > sink->max_depth) { *sink->overflow = 1u; return; }
    const uint32_t idx = sink->claim();
    if (idx >= sink->capacity) { *sink->overflow = 1u; return; }
    auto* out = sink->frames + (size_t)idx * sink->max_depth;
    out[depth - 1] = (uint16_t)n;
    uint32_t k = depth - 1;
    for (h = sp; h < kLiveBase; h = arena[h] >> 16) out[--k] = (uint16_t)(arena[h] & 0xFFFFu);
    for (uint32_t j = 0; j < d; ++j) out[j] = (uint16_t)live[j];
    sink->depth[idx] = depth;
  }
};

}  // namespace xgm
