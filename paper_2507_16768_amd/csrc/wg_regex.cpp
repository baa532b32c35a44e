// Regular expression -> operator template text (host only).
//
// The translation of the section "Operator Building and State Tracking", paragraph "From
// Regular Expressions to Wait/Write Operator Composition": literal runs become Write, byte
// classes become Wait, repetition and branching become DoWhile / IfElse around condition
// Waits.  The operators decide on one byte and consume it, and a checkpoint has at most two
// ways out, so only expressions with that shape translate; the others are refused with a
// message that says which rule they break:
//   - a repeated or optional group, and each side of an alternation, starts with a single byte
//     or class; the byte sets that a decision tells apart are disjoint;
//   - what follows an optional or repeated group is a single byte or class (or the end of the
//     expression): the decision consumes it when the group is left;
//   - a class repetition X* / X+ is carried as the `allow` set of the next checkpoint, which
//     must not share a byte with it (matching is not greedy: the first terminator ends a Wait);
//   - three-way decisions do not exist: (a|b|c) works only when every side is a single byte.
// The paper's worked example, \d+(\.\d+)*, yields the operator tree of its listing.
#include <array>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <stdexcept>
#include <string>
#include <vector>

#include "wg_internal.h"

namespace wg {
namespace {

using ByteSet = std::array<bool, 256>;

struct RegexError : std::runtime_error { using std::runtime_error::runtime_error; };

// ---- syntax tree ---------------------------------------------------------------------------
struct Node {
    enum Kind { SET, CAT, ALT, REP } kind = SET;
    ByteSet set{};                 // SET
    std::vector<Node> kids;        // CAT / ALT; REP has one kid
    uint32_t min = 1, max = 1;     // REP; max == kInf for an open count
};
constexpr uint32_t kInf = 0xFFFFFFFFu;
constexpr uint32_t kMaxCount = 1000;

class Parser {
  public:
    explicit Parser(const char *s) : s_(s), n_(std::strlen(s)) {}
    Node parse() {
        if (i_ < n_ && s_[i_] == '^') i_++;                     // the match is a full match anyway
        Node r = alt();
        if (i_ < n_) die(s_[i_] == ')' ? "unbalanced ')'" : "unexpected character");
        return r;
    }

  private:
    const char *s_; size_t n_, i_ = 0;

    [[noreturn]] void die(const std::string &m) const {
        throw RegexError("regex, at offset " + std::to_string(i_) + ": " + m);
    }
    static void span(ByteSet &b, int lo, int hi) { for (int x = lo; x <= hi; x++) b[x] = true; }
    static int hex(int c) {
        if (c >= '0' && c <= '9') return c - '0';
        c |= 0x20;
        return (c >= 'a' && c <= 'f') ? c - 'a' + 10 : -1;
    }
    // After a backslash: adds a class to `out` and returns -1, or returns the escaped byte.
    int escape(ByteSet &out) {
        if (i_ >= n_) die("dangling backslash");
        const int c = static_cast<unsigned char>(s_[i_++]);
        ByteSet cls{};
        switch (c) {
        case 'd': case 'D': span(cls, '0', '9'); break;
        case 'w': case 'W': span(cls, '0', '9'); span(cls, 'a', 'z'); span(cls, 'A', 'Z'); cls['_'] = true; break;
        case 's': case 'S': for (int x : {32, 9, 10, 13, 12, 11}) cls[x] = true; break;
        case 'n': return 10;
        case 't': return 9;
        case 'r': return 13;
        case 'f': return 12;
        case 'v': return 11;
        case '0': return 0;
        case 'x': {
            if (i_ + 2 > n_) die("short \\x escape");
            const int h = hex(static_cast<unsigned char>(s_[i_])), l = hex(static_cast<unsigned char>(s_[i_ + 1]));
            if (h < 0 || l < 0) die("bad \\x escape");
            i_ += 2;
            return (h << 4) | l;
        }
        default:
            if ((c >= '1' && c <= '9') || c == 'b' || c == 'B' || c == 'A' || c == 'Z' || c == 'z')
                die("back-references and anchors inside the expression are not supported");
            if ((c >= 'a' && c <= 'z') || (c >= 'A' && c <= 'Z')) die("unknown escape");
            return c;
        }
        const bool negate = c == 'D' || c == 'W' || c == 'S';
        for (int x = 0; x < 256; x++) if (cls[x] != negate) out[x] = true;
        return -1;
    }
    Node bracket() {                                           // after '['
        Node n;
        bool negate = false;
        if (i_ < n_ && s_[i_] == '^') { negate = true; i_++; }
        bool first = true;
        ByteSet b{};
        while (true) {
            if (i_ >= n_) die("unterminated [class]");
            int lo = static_cast<unsigned char>(s_[i_++]);
            if (lo == ']' && !first) break;
            first = false;
            if (lo == '\\') { lo = escape(b); if (lo < 0) continue; }
            if (i_ + 1 < n_ && s_[i_] == '-' && s_[i_ + 1] != ']') {
                i_++;
                int hi = static_cast<unsigned char>(s_[i_++]);
                if (hi == '\\') { ByteSet tmp{}; hi = escape(tmp); if (hi < 0) die("a class cannot end a range"); }
                if (hi < lo) die("reversed range");
                span(b, lo, hi);
            } else b[lo] = true;
        }
        for (int x = 0; x < 256; x++) n.set[x] = b[x] != negate;
        return n;
    }
    Node alt() {
        Node a; a.kind = Node::ALT;
        a.kids.push_back(cat());
        while (i_ < n_ && s_[i_] == '|') { i_++; a.kids.push_back(cat()); }
        if (a.kids.size() == 1) { Node only = std::move(a.kids[0]); return only; }
        return a;
    }
    Node cat() {
        Node c; c.kind = Node::CAT;
        while (i_ < n_ && s_[i_] != '|' && s_[i_] != ')') {
            if (s_[i_] == '$' && (i_ + 1 == n_)) { i_++; break; }   // closing anchor
            c.kids.push_back(repeat());
        }
        return c;
    }
    uint32_t number() {
        uint64_t v = 0; const size_t b = i_;
        while (i_ < n_ && s_[i_] >= '0' && s_[i_] <= '9') {
            v = v * 10 + static_cast<uint64_t>(s_[i_++] - '0');
            if (v > kMaxCount) die("repeat count above 1000");
        }
        if (i_ == b) die("expected a number");
        return static_cast<uint32_t>(v);
    }
    Node repeat() {
        Node a = atom();
        while (i_ < n_) {
            uint32_t lo, hi;
            const char c = s_[i_];
            if (c == '*') { lo = 0; hi = kInf; i_++; }
            else if (c == '+') { lo = 1; hi = kInf; i_++; }
            else if (c == '?') { lo = 0; hi = 1; i_++; }
            else if (c == '{') {
                i_++;
                lo = number(); hi = lo;
                if (i_ < n_ && s_[i_] == ',') { i_++; hi = (i_ < n_ && s_[i_] == '}') ? kInf : number(); }
                if (i_ >= n_ || s_[i_] != '}') die("expected '}'");
                i_++;
                if (hi < lo) die("reversed repeat count");
            } else break;
            if (i_ < n_ && (s_[i_] == '?' || s_[i_] == '+'))
                die("lazy and possessive quantifiers are not supported");
            Node r; r.kind = Node::REP; r.min = lo; r.max = hi;
            r.kids.push_back(std::move(a));
            a = std::move(r);
        }
        return a;
    }
    Node atom() {
        const int c = static_cast<unsigned char>(s_[i_++]);
        Node n;
        switch (c) {
        case '(': {
            if (i_ + 1 < n_ && s_[i_] == '?') {
                if (s_[i_ + 1] != ':') die("only (?: ) groups are supported");
                i_ += 2;
            }
            Node g = alt();
            if (i_ >= n_ || s_[i_] != ')') die("unbalanced '('");
            i_++;
            return g;
        }
        case '[': return bracket();
        case '.': for (int x = 0; x < 256; x++) n.set[x] = x != 10; return n;
        case '\\': { const int v = escape(n.set); if (v >= 0) n.set[v] = true; return n; }
        case '*': case '+': case '?': case '{': i_--; die("nothing to repeat");
        case '^': case '$': i_--; die("anchors inside the expression are not supported");
        default: n.set[c] = true; return n;
        }
    }
};

// ---- items: the tree with counts unrolled ----------------------------------------------------
struct Item {
    enum Kind { ONE, LOOP, OPT, STAR, ALT2 } kind = ONE;
    ByteSet set{};                       // ONE / LOOP
    bool bounded = false; uint32_t bound = 0;   // LOOP: at most `bound` bytes
    std::vector<Item> a, b;              // OPT / STAR: a; ALT2: a | b
};

bool empty_set(const ByteSet &s) { for (bool x : s) if (x) return false; return true; }
bool meet(const ByteSet &x, const ByteSet &y) { for (int i = 0; i < 256; i++) if (x[i] && y[i]) return true; return false; }

void unroll(const Node &n, std::vector<Item> &out);

std::vector<Item> items_of(const Node &n) { std::vector<Item> v; unroll(n, v); return v; }

void unroll(const Node &n, std::vector<Item> &out) {
    switch (n.kind) {
    case Node::SET: {
        if (empty_set(n.set)) throw RegexError("regex: a class that matches no byte");
        Item it; it.kind = Item::ONE; it.set = n.set;
        out.push_back(std::move(it));
        return;
    }
    case Node::CAT:
        for (const Node &k : n.kids) unroll(k, out);
        return;
    case Node::ALT: {
        // sides that are single bytes or classes merge into one class; an empty side makes the
        // rest optional
        ByteSet singles{};
        bool any_single = false, has_empty = false;
        std::vector<std::vector<Item>> sides;
        for (const Node &k : n.kids) {
            std::vector<Item> s = items_of(k);
            if (s.empty()) has_empty = true;
            else if (s.size() == 1 && s[0].kind == Item::ONE) {
                for (int x = 0; x < 256; x++) singles[x] = singles[x] || s[0].set[x];
                any_single = true;
            } else sides.push_back(std::move(s));
        }
        if (any_single) { Item it; it.kind = Item::ONE; it.set = singles; sides.insert(sides.begin(), std::vector<Item>{it}); }
        if (sides.size() > 2)
            throw RegexError("regex: an alternation with more than two sides that are not single bytes needs a "
                             "three-way decision, which the operators do not have");
        std::vector<Item> body;
        if (sides.size() == 2) {
            Item it; it.kind = Item::ALT2; it.a = std::move(sides[0]); it.b = std::move(sides[1]);
            body.push_back(std::move(it));
        } else if (sides.size() == 1) body = std::move(sides[0]);
        if (has_empty && !body.empty()) {
            Item it; it.kind = Item::OPT; it.a = std::move(body);
            out.push_back(std::move(it));
        } else for (Item &it : body) out.push_back(std::move(it));
        return;
    }
    case Node::REP: {
        const std::vector<Item> body = items_of(n.kids[0]);
        if (body.empty()) return;
        const bool single = body.size() == 1 && body[0].kind == Item::ONE;
        for (uint32_t i = 0; i < n.min; i++) for (const Item &it : body) out.push_back(it);
        if (n.max == n.min) return;
        if (single) {
            Item it; it.kind = Item::LOOP; it.set = body[0].set;
            if (n.max != kInf) { it.bounded = true; it.bound = n.max - n.min; }
            out.push_back(std::move(it));
        } else if (n.max == kInf) {
            Item it; it.kind = Item::STAR; it.a = body;
            out.push_back(std::move(it));
        } else {
            // up to max - min further copies: (G(G(G)?)?)?
            if (n.max - n.min > 16) throw RegexError("regex: a group repeated over a range wider than 16");
            Item inner; bool have = false;
            for (uint32_t i = n.min; i < n.max; i++) {
                Item it; it.kind = Item::OPT; it.a = body;
                if (have) it.a.push_back(std::move(inner));
                inner = std::move(it); have = true;
            }
            out.push_back(std::move(inner));
        }
        return;
    }
    }
}

// ---- emission --------------------------------------------------------------------------------
struct Pend {                            // a class repetition waiting for its terminator
    ByteSet set{};
    bool any = false, bounded = false;
    uint32_t bound = 0;
};

std::string set_text(const ByteSet &s, bool eos = false) {
    std::string t = "{";
    char buf[32];
    for (int lo = 0; lo < 256;) {
        if (!s[lo]) { lo++; continue; }
        int hi = lo;
        while (hi + 1 < 256 && s[hi + 1]) hi++;
        if (t.size() > 1) t += ", ";
        if (hi == lo) std::snprintf(buf, sizeof buf, "\\x%02X", lo);
        else std::snprintf(buf, sizeof buf, "[\\x%02X-\\x%02X]", lo, hi);
        t += buf;
        lo = hi + 1;
    }
    if (eos) { if (t.size() > 1) t += ", "; t += "<eos>"; }
    return t + "}";
}

struct Follow {                          // the terminator a decision consumes when it moves on
    ByteSet set{};
    bool eos = false;
    std::string text() const { return set_text(set, eos); }
};

std::string wait_text(const Pend &p, const Follow &f) {
    std::string t = "Wait(allow=" + set_text(p.any ? p.set : ByteSet{}) + ", wait=" + f.text();
    if (p.any && p.bounded) t += ", max=" + std::to_string(p.bound);
    return t + ")";
}

std::string cond_text(const Pend &p, const std::string &true_waits, const std::string &false_waits) {
    return "Wait(allow=" + set_text(p.any ? p.set : ByteSet{}) + ", true_waits=" + true_waits +
           ", false_waits=" + false_waits + ")";
}

std::string seq_text(const std::vector<std::string> &ops, bool none_ok) {
    if (ops.empty()) {
        if (!none_ok) return "Sequence()";
        return "None";
    }
    if (ops.size() == 1) return ops[0];
    std::string t = "Sequence(";
    for (size_t i = 0; i < ops.size(); i++) { if (i) t += ", "; t += ops[i]; }
    return t + ")";
}

class Emitter {
  public:
    // Translates items[from..].  `after` is the terminator that whoever holds this list consumes
    // once the list has matched (the end of generation at the top; nullptr inside a repeated
    // group, whose own decision comes next): a decision at the very end of the list may consume
    // it instead and then sets `took_after`.  Returns what is still pending at the end (always
    // nothing at the top: the end of generation consumes it).
    Pend sequence(const std::vector<Item> &items, size_t from, bool top, const Follow *after,
                  std::vector<std::string> &out, bool &took_after) {
        Pend pend;
        took_after = false;
        std::string lit;
        auto flush = [&]() {
            if (lit.empty()) return;
            std::string t = "Write(\"";
            char buf[8];
            for (unsigned char c : lit) {
                if (c >= 0x20 && c < 0x7F && c != '"' && c != '\\') t.push_back(static_cast<char>(c));
                else { std::snprintf(buf, sizeof buf, "\\x%02X", c); t += buf; }
            }
            out.push_back(t + "\")");
            lit.clear();
        };
        size_t i = from;
        while (i < items.size()) {
            const Item &it = items[i];
            switch (it.kind) {
            case Item::ONE: {
                if (!pend.any) {
                    int only = -1, count = 0;
                    for (int x = 0; x < 256; x++) if (it.set[x]) { only = x; count++; }
                    if (count == 1) lit.push_back(static_cast<char>(only));
                    else { flush(); Follow f; f.set = it.set; out.push_back(wait_text(Pend{}, f)); }
                } else {
                    if (meet(pend.set, it.set))
                        fail("a repeated class is followed by a byte it also matches (the first terminator ends a Wait)");
                    Follow f; f.set = it.set;
                    out.push_back(wait_text(pend, f));
                    pend = Pend{};
                }
                i++;
                break;
            }
            case Item::LOOP: {
                flush();
                if (pend.any) {
                    if (pend.set != it.set || pend.bounded || it.bounded)
                        fail("two repeated classes in a row");
                } else { pend.any = true; pend.set = it.set; pend.bounded = it.bounded; pend.bound = it.bound; }
                i++;
                break;
            }
            case Item::OPT:
            case Item::STAR: {
                flush();
                if (pend.bounded) fail("a counted class repetition is followed by a decision");
                const ByteSet enter = first_of(it.a);
                const Follow leave = follow_of(items, i + 1, after);
                if (i + 1 >= items.size()) took_after = true;
                if (meet(enter, leave.set)) fail("an optional part and what follows it can start with the same byte");
                if (pend.any && (meet(pend.set, enter) || meet(pend.set, leave.set)))
                    fail("a repeated class is followed by a byte it also matches (the first terminator ends a Wait)");
                std::vector<std::string> body;
                bool body_took = false;
                const Pend inner = sequence(it.a, 1, false, it.kind == Item::OPT ? &leave : nullptr, body, body_took);
                if (inner.any && (meet(inner.set, leave.set) || (it.kind == Item::STAR && meet(inner.set, enter))))
                    fail("a repeated class is followed by a byte it also matches (the first terminator ends a Wait)");
                if (it.kind == Item::OPT) {
                    if (!body_took) body.push_back(wait_text(inner, leave));
                    out.push_back("IfElse(condition=" + cond_text(pend, set_text(enter), leave.text()) +
                                  ", if_body=" + seq_text(body, true) + ", else_body=None)");
                } else {
                    if (inner.bounded) fail("a counted class repetition is followed by a decision");
                    out.push_back("IfElse(condition=" + cond_text(pend, leave.text(), set_text(enter)) +
                                  ", if_body=None, else_body=DoWhile(body=" + seq_text(body, true) +
                                  ", condition=" + cond_text(inner, set_text(enter), leave.text()) + "))");
                }
                pend = Pend{};
                i += 2;                            // the decision consumed the item after the group
                break;
            }
            case Item::ALT2: {
                flush();
                if (pend.bounded) fail("a counted class repetition is followed by a decision");
                const ByteSet sa = first_of(it.a), sb = first_of(it.b);
                if (meet(sa, sb)) fail("the sides of an alternation can start with the same byte");
                if (pend.any && (meet(pend.set, sa) || meet(pend.set, sb)))
                    fail("a repeated class is followed by a byte it also matches (the first terminator ends a Wait)");
                // A side that ends inside a class repetition, or in a decision of its own, consumes
                // what follows the alternation; then the other side does so too.
                Follow leave;
                const bool can_leave = try_follow(items, i + 1, after, leave);
                std::vector<std::string> ba, bb;
                bool ta = false, tb = false;
                const Pend pa = sequence(it.a, 1, false, can_leave ? &leave : nullptr, ba, ta);
                const Pend pb = sequence(it.b, 1, false, can_leave ? &leave : nullptr, bb, tb);
                size_t used = 1;
                if (pa.any || pb.any || ta || tb) {
                    if (!can_leave) follow_of(items, i + 1, after);          // reports why
                    if ((pa.any && meet(pa.set, leave.set)) || (pb.any && meet(pb.set, leave.set)))
                        fail("a repeated class is followed by a byte it also matches (the first terminator ends a Wait)");
                    if (!ta) ba.push_back(wait_text(pa, leave));
                    if (!tb) bb.push_back(wait_text(pb, leave));
                    if (i + 1 >= items.size()) took_after = true;
                    used = 2;
                }
                out.push_back("IfElse(condition=" + cond_text(pend, set_text(sa), set_text(sb)) +
                              ", if_body=" + seq_text(ba, true) + ", else_body=" + seq_text(bb, true) + ")");
                pend = Pend{};
                i += used;
                break;
            }
            }
        }
        flush();
        if (top && pend.any) {
            Follow f; f.eos = true;
            out.push_back(wait_text(pend, f));
            pend = Pend{};
        }
        return pend;
    }

  private:
    [[noreturn]] static void fail(const std::string &m) { throw RegexError("regex: " + m); }

    static ByteSet first_of(const std::vector<Item> &g) {
        if (g.empty() || g[0].kind != Item::ONE)
            fail("a repeated or optional group, and each side of an alternation, has to start with a single byte or class");
        return g[0].set;
    }
    // The item a decision consumes when it leaves its group: a single byte or class, or, at the
    // end of the list, what the holder of the list would consume next.
    static bool try_follow(const std::vector<Item> &items, size_t at, const Follow *after, Follow &f) {
        if (at < items.size()) {
            if (items[at].kind != Item::ONE) return false;
            f = Follow{};
            f.set = items[at].set;
            return true;
        }
        if (!after) return false;
        f = *after;
        return true;
    }
    static Follow follow_of(const std::vector<Item> &items, size_t at, const Follow *after) {
        Follow f;
        if (try_follow(items, at, after, f)) return f;
        if (at < items.size()) fail("an optional or repeated part has to be followed by a single byte or class");
        fail("an optional or repeated part at the end of a repeated group needs a byte after it inside the group");
    }
};

}  // namespace

std::string regex_to_template(const char *regex) {
    Parser p(regex);
    const Node root = p.parse();
    const std::vector<Item> items = items_of(root);
    std::vector<std::string> ops;
    Emitter e;
    Follow end;
    end.eos = true;
    bool took = false;
    e.sequence(items, 0, true, &end, ops, took);
    return seq_text(ops, false);
}

}  // namespace wg
