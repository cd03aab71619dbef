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

constexpr uint32_t kNoRowD = 0xFFFF;
constexpr uint32_t kDeadD = 0xFFFF;
constexpr uint32_t kAltFlagD = 0x8000;
constexpr uint32_t kMoveTagD = 0xFFFF;
constexpr uint32_t kLiveBase = 0x8000;  // stack handles >= this refer to the request's live frames

XGM_HD uint32_t token_byte(const uint4& tk, const uint8_t* ext, int i) {
  if (i < 15) {
    uint32_t w = (i < 8) ? ((i < 4) ? tk.x : tk.y) : ((i < 12) ? tk.z : tk.w);
    return (w >> ((i & 3) * 8)) & 0xFFu;
  }
  return ext[i];
}

// Depth-first walk of one token through the pushdown automaton (section 2.2,
// Appendix A) from the configuration (node on top, `depth - 1` live frames
// below it).  Alternatives at a configuration, in the order they are tried:
// the byte edge, the rule references whose callee can start with the next
// byte (push the return node, enter the callee), and - if the node is
// accepting and a byte was consumed since the last push - the return to the
// frame below.  Frames pushed during the walk live in a small arena with
// parent links, so that backing up to a pending alternative never copies a
// stack (the persistent stack of section 3.3, in miniature).
//
// BUILD = true:  nothing is known below the start frame (depth must be 1);
//                result kAccept / kUncertain / kReject as in section 3.1.
// BUILD = false: frames below are live[0 .. depth-2]; result kAccept (token
//                allowed) or kReject.
// kOverflow: a limit was hit; the caller records the pair.
// `steps_out` (may be null) receives the number of automaton steps taken.
template <bool BUILD>
XGM_HD int walk_token(const DevTables& T, const uint4 tk, const uint8_t* ext, const int len,
                      const uint32_t start_node, const uint16_t* live, const uint32_t depth,
                      uint32_t* steps_out = nullptr) {
  if (len > kMaxTokenLen) return kOverflow;
  uint32_t arena[kArenaFrames];  // ret | parent handle << 16
  uint2 choice[kChoicePoints];   // x = node | sp << 16 ; y = i | alt << 8 | top << 16 | f << 24
  uint32_t n = start_node, sp = kLiveBase + depth - 1, f = 1, alt = 0, top = 0, csp = 0;
  int i = 0;
  bool left_frame = false;
  for (int steps = 0;; ++steps) {
    if (steps_out) *steps_out = (uint32_t)steps;
    if (i == len) return kAccept;
    if (steps >= kMaxSteps) return kOverflow;
    const uint32_t c = token_byte(tk, ext, i);
    const uint2 h = T.hdr[n];
    const uint32_t lo = h.x & 0xFFu, hi = (h.x >> 8) & 0xFFu, row = h.y & 0xFFFFu;
    uint32_t k = 0, single = 0, base = 0;
    bool pooled = false;
    if (c >= lo && c <= hi) {
      k = 1;
      single = (kMoveTagD << 16) | (h.x >> 16);
    } else if (row != kNoRowD) {
      const uint32_t a = T.rows[row * T.n_cls + T.cls[c]];
      if (a != kDeadD) {
        if (a < kAltFlagD) { k = 1; single = (kMoveTagD << 16) | a; }
        else { base = a & 0x7FFFu; k = T.alts[base]; pooled = true; }
      }
    }
    const uint32_t can_pop = (h.y >> 16) & f & 1u;
    const uint32_t total = k + can_pop;
    bool advanced = false;
    if (alt < total) {
      bool ok = true;
      if (alt + 1 < total) {
        if (csp == kChoicePoints) return kOverflow;
        choice[csp++] = make_uint2(n | (sp << 16), (uint32_t)i | ((alt + 1) << 8) | (top << 16) | (f << 24));
      }
      if (alt < k) {
        const uint32_t e = pooled ? T.alts[base + 1 + alt] : single;
        const uint32_t tag = e >> 16, dst = e & 0xFFFFu;
        if (tag == kMoveTagD) { n = dst; ++i; f = 1; }
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
        if (d == 0) {                // nothing below: end of the start frame (BUILD) or of the root rule
          if (BUILD) left_frame = true;
          ok = false;
        } else {
          n = live[d - 1];
          sp = kLiveBase + d - 1;
        }
      }
      if (ok) { alt = 0; advanced = true; }
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
  return (BUILD && left_frame) ? kUncertain : kReject;
}

}  // namespace xgm
