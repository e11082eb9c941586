// Structure-aware chunking of a token stream (Section 4.3, Appendix B separator table).
// Host code only: the boundaries feed lc_build_index and the close bits of lc_append.
#include "lychee.h"

#include <cstring>

namespace {

struct Tok {
    const char* p;
    int64_t len;
    bool has(const char* s) const {
        const int64_t m = (int64_t)std::strlen(s);
        for (int64_t i = 0; i + m <= len; ++i)
            if (std::memcmp(p + i, s, (size_t)m) == 0) return true;
        return false;
    }
    bool ends(const char* s, int64_t upto) const {
        const int64_t m = (int64_t)std::strlen(s);
        return m <= upto && std::memcmp(p + upto - m, s, (size_t)m) == 0;
    }
};

template <int N>
bool ends_any(const Tok& t, int64_t upto, const char* const (&set)[N]) {
    for (const char* s : set)
        if (t.ends(s, upto)) return true;
    return false;
}

const char* const kStructural[] = {"}", "]", ">"};
const char* const kSentence[] = {".", "?", "!", "\xE3\x80\x82", "\xEF\xBC\x9F", "\xEF\xBC\x81"};
const char* const kClause[] = {",", ";", ":", "\xEF\xBC\x8C", "\xEF\xBC\x9B", "\xEF\xBC\x9A", "\xE3\x80\x81"};

// 1 strongest .. 4 whitespace, 0 none.
int separator_level(const Tok& t) {
    int64_t body = t.len;                       // length without trailing blanks and tabs
    while (body > 0 && (t.p[body - 1] == ' ' || t.p[body - 1] == '\t')) --body;
    if (t.has("\n\n") || t.has("---") || t.has("***") || t.has("```") || ends_any(t, body, kStructural)) return 1;
    if (t.has("\n") || ends_any(t, body, kSentence)) return 2;
    if (ends_any(t, body, kClause)) return 3;
    if (t.len > 0 && body < t.len) return 4;    // ends in a blank (an all-blank token included)
    return 0;
}

}  // namespace

extern "C" int lc_chunk_tokens(const char* text, const int64_t* offsets, int n, int min_len, int max_len,
                               int32_t* bounds, int capacity, int* n_chunks) {
    if (!offsets || !bounds || !n_chunks || n < 0 || min_len < 1 || max_len < min_len || (!text && n > 0))
        return LC_ERR_INVALID_ARG;
    for (int i = 0; i < n; ++i)
        if (offsets[i + 1] < offsets[i]) return LC_ERR_INVALID_ARG;
    if (capacity < 1) return LC_ERR_CAPACITY;
    int m = 0;
    bounds[0] = 0;
    int pos = 0;
    while (pos < n) {
        const int64_t hi = ((int64_t)pos + max_len < n ? (int64_t)pos + max_len : n) - 1;
        int64_t cut = hi;
        int best = 5;
        for (int64_t e = (int64_t)pos + min_len - 1; e <= hi && best > 1; ++e) {
            const Tok t{text + offsets[e], offsets[e + 1] - offsets[e]};
            const int lv = separator_level(t);
            if (lv != 0 && lv < best) { best = lv; cut = e; }
        }
        pos = (int)cut + 1;
        if (m + 2 > capacity) return LC_ERR_CAPACITY;
        bounds[++m] = pos;
    }
    *n_chunks = m;
    return LC_OK;
}
