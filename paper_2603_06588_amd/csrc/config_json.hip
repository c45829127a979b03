// Host-only reader for the JSON configuration file of the hook (Section 2, config file example):
// a small recursive-descent JSON walker that keeps two things, params.important_heads (a list
// of [layer, head] pairs) and hookq.hookq_mode ("last_token" or "all_tokens"), and skips the
// rest of the document whatever it holds.
#include "../../include/hook_api.h"

#include <cstring>
#include <string>

namespace {

struct Reader {
  const char* c;
  int32_t* layers;
  int32_t* heads;
  int32_t capacity;
  int32_t n = 0;
  int32_t mode = -1;
  bool bad = false;

  void blank() { while (*c == ' ' || *c == '\t' || *c == '\n' || *c == '\r') ++c; }
  bool eat(char ch) { blank(); if (*c != ch) return false; ++c; return true; }

  bool string(std::string* out) {
    blank();
    if (*c != '"') return false;
    ++c;
    out->clear();
    while (*c && *c != '"') {
      if (*c == '\\') {
        ++c;
        if (!*c) return false;
        if (*c == 'u') {                      // keep escapes opaque: no key or mode needs them
          for (int k = 0; k < 4; ++k) { ++c; if (!*c) return false; }
          out->push_back('?');
          ++c;
          continue;
        }
        out->push_back(*c == 'n' ? '\n' : *c == 't' ? '\t' : *c);
        ++c;
        continue;
      }
      out->push_back(*c++);
    }
    if (*c != '"') return false;
    ++c;
    return true;
  }

  // a JSON number; *ival receives it when it is a non-negative integer no larger than 2^30
  bool number(bool* is_index, int32_t* ival) {
    blank();
    const char* s = c;
    bool integral = true;
    if (*c == '-') { ++c; integral = false; }
    if (*c < '0' || *c > '9') return false;
    long long v = 0;
    while (*c >= '0' && *c <= '9') { if (v <= (1ll << 31)) v = v * 10 + (*c - '0'); ++c; }
    if (*c == '.') { integral = false; ++c; if (*c < '0' || *c > '9') return false; while (*c >= '0' && *c <= '9') ++c; }
    if (*c == 'e' || *c == 'E') {
      integral = false; ++c;
      if (*c == '+' || *c == '-') ++c;
      if (*c < '0' || *c > '9') return false;
      while (*c >= '0' && *c <= '9') ++c;
    }
    (void)s;
    *is_index = integral && v <= (1ll << 30);
    *ival = (int32_t)(*is_index ? v : 0);
    return true;
  }

  bool literal(const char* w) { blank(); size_t k = std::strlen(w); if (std::strncmp(c, w, k) != 0) return false; c += k; return true; }

  // the value of params.important_heads: [[layer, head], ...]
  bool head_list() {
    if (!eat('[')) return false;
    if (eat(']')) return true;
    for (;;) {
      bool i0, i1; int32_t l, h;
      if (!eat('[') || !number(&i0, &l) || !eat(',') || !number(&i1, &h) || !eat(']') || !i0 || !i1) return false;
      if (n < capacity) { layers[n] = l; heads[n] = h; }
      ++n;
      if (eat(',')) continue;
      return eat(']');
    }
  }

  // depth-limited walk; `path` is "" at the top, "params" / "hookq" one level down
  bool value(const std::string& path, int depth) {
    if (depth > 64) return false;
    blank();
    if (*c == '{') {
      ++c;
      if (eat('}')) return true;
      for (;;) {
        std::string key;
        if (!string(&key) || !eat(':')) return false;
        if (depth == 1 && path == "params" && key == "important_heads") {
          n = 0;                              // a repeated key: the last one wins, as in JSON readers
          if (!head_list()) return false;
        } else if (depth == 1 && path == "hookq" && key == "hookq_mode") {
          std::string m;
          if (!string(&m)) return false;
          if (m == "last_token") mode = 0; else if (m == "all_tokens") mode = 1; else return false;
        } else if (!value(depth == 0 ? key : std::string("\x01"), depth + 1)) {
          return false;
        }
        if (eat(',')) continue;
        return eat('}');
      }
    }
    if (*c == '[') {
      ++c;
      if (eat(']')) return true;
      for (;;) {
        if (!value("\x01", depth + 1)) return false;
        if (eat(',')) continue;
        return eat(']');
      }
    }
    if (*c == '"') { std::string s; return string(&s); }
    if (*c == 't') return literal("true");
    if (*c == 'f') return literal("false");
    if (*c == 'n') return literal("null");
    bool ii; int32_t iv;
    return number(&ii, &iv);
  }
};

}  // namespace

extern "C" hook_status hook_parse_config_json(const char* text, int32_t* layers, int32_t* heads, int32_t capacity,
                                              int32_t* count, int32_t* hookq_mode) {
  if (!text || !count || !hookq_mode || capacity < 0 || (capacity > 0 && (!layers || !heads))) return HOOK_ERR_NULL;
  *count = 0;
  *hookq_mode = -1;
  Reader r{text, layers, heads, capacity};
  r.blank();
  if (*r.c != '{') return HOOK_ERR_SHAPE;
  if (!r.value("", 0)) return HOOK_ERR_SHAPE;
  r.blank();
  if (*r.c != '\0') return HOOK_ERR_SHAPE;
  *count = r.n;
  *hookq_mode = r.mode;
  return r.n > capacity ? HOOK_ERR_WORKSPACE : HOOK_OK;
}
