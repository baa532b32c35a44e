// Host operator compiler: template text + runtime snippet arguments -> flat state table.
//
// Two stages, following the paper's decomposition of a constraint into a static
// structure and dynamic arguments (section "Collaborative Parsing"): each distinct
// template text is parsed once into an operator tree with $holes left open; every
// instance then binds its own arguments while the tree is flattened into leaf
// states.  Operator semantics are those of the section "Operator Building and State
// Tracking"; a Write becomes one state per byte ("a sequence of specialised Wait
// operators", section "Mask Generation and Global Caching").
#include <array>
#include <cstring>
#include <map>
#include <memory>
#include <stdexcept>
#include <string>
#include <unordered_map>
#include <vector>

#include "wg_internal.h"

namespace wg {
namespace {

using SymbolSet = std::array<bool, 257>;

struct SetExpr {                       // a set with possibly unbound $names
    SymbolSet fixed{};
    std::vector<std::string> holes;
    bool present = false;
};

struct Op {
    enum Kind { SEQ, WRITE, WAIT, COND, IFELSE, DOWHILE } kind;
    std::vector<std::unique_ptr<Op>> kids;          // SEQ
    std::string bytes; std::string hole;            // WRITE: literal or $hole
    SetExpr allow, denies, wait, twait, fwait;      // WAIT / COND
    bool bounded = false; uint32_t max = 0;         // WAIT
    std::unique_ptr<Op> body, cond, if_body, else_body;
    explicit Op(Kind k) : kind(k) {}
};

struct ParseError : std::runtime_error { using std::runtime_error::runtime_error; };

class Reader {
  public:
    explicit Reader(const char *text) : s_(text), n_(std::strlen(text)) {}

    std::unique_ptr<Op> parse_all() {
        auto op = operator_(false);
        if (look() >= 0) die("trailing text after the operator");
        return op;
    }

  private:
    const char *s_; size_t n_; size_t i_ = 0;

    [[noreturn]] void die(const std::string &m) const {
        throw ParseError("at offset " + std::to_string(i_) + ": " + m);
    }
    int look() {
        while (i_ < n_ && (s_[i_] == ' ' || s_[i_] == '\t' || s_[i_] == '\n' || s_[i_] == '\r')) i_++;
        return i_ < n_ ? static_cast<unsigned char>(s_[i_]) : -1;
    }
    void need(char c) {
        if (look() != static_cast<unsigned char>(c)) die(std::string("expected '") + c + "'");
        i_++;
    }
    std::string word() {
        look();
        size_t b = i_;
        while (i_ < n_) {
            char c = s_[i_];
            bool alpha = (c >= 'a' && c <= 'z') || (c >= 'A' && c <= 'Z') || c == '_';
            if (alpha || (i_ > b && c >= '0' && c <= '9')) i_++; else break;
        }
        if (i_ == b) die("expected an identifier");
        return std::string(s_ + b, i_ - b);
    }
    static int hex(int c) {
        if (c >= '0' && c <= '9') return c - '0';
        c |= 0x20;
        return (c >= 'a' && c <= 'f') ? c - 'a' + 10 : -1;
    }
    // After '\'.  Returns the byte, or -1 when a class (\d \w \s) was merged into *cls.
    int backslash(SymbolSet *cls) {
        if (i_ >= n_) die("dangling backslash");
        int c = static_cast<unsigned char>(s_[i_++]);
        auto span = [&](int lo, int hi) { for (int x = lo; x <= hi; x++) (*cls)[x] = true; };
        switch (c) {
        case 'n': return 10;
        case 't': return 9;
        case 'r': return 13;
        case 'x': {
            if (i_ + 2 > n_) die("short \\x escape");
            int h = hex(static_cast<unsigned char>(s_[i_])), l = hex(static_cast<unsigned char>(s_[i_ + 1]));
            if (h < 0 || l < 0) die("bad \\x escape");
            i_ += 2;
            return (h << 4) | l;
        }
        case 'd': if (!cls) return c; span('0', '9'); return -1;
        case 'w': if (!cls) return c; span('0', '9'); span('a', 'z'); span('A', 'Z'); (*cls)['_'] = true; return -1;
        case 's': if (!cls) return c; for (int x : {32, 9, 10, 13, 12, 11}) (*cls)[x] = true; return -1;
        default: return c;
        }
    }
    void bracket(SymbolSet &out) {                  // after '['
        while (true) {
            if (i_ >= n_) die("unterminated [class]");
            int lo = static_cast<unsigned char>(s_[i_++]);
            if (lo == ']') return;
            if (lo == '\\') { lo = backslash(&out); if (lo < 0) continue; }
            if (i_ + 1 < n_ && s_[i_] == '-' && s_[i_ + 1] != ']') {
                i_++;
                int hi = static_cast<unsigned char>(s_[i_++]);
                if (hi == '\\') hi = backslash(nullptr);
                if (hi < lo) die("reversed range");
                for (int x = lo; x <= hi; x++) out[x] = true;
            } else out[lo] = true;
        }
    }
    SetExpr set() {
        SetExpr e; e.present = true;
        if (look() == '$') { i_++; e.holes.push_back(word()); return e; }
        need('{');
        while (true) {
            int c = look();
            if (c < 0) die("unterminated set");
            if (c == '}') { i_++; return e; }
            if (c == ',') { i_++; continue; }
            if (c == '<' && n_ - i_ >= 5 && std::memcmp(s_ + i_, "<eos>", 5) == 0) { i_ += 5; e.fixed[kSymEos] = true; }
            else if (c == '\\') { i_++; int v = backslash(&e.fixed); if (v >= 0) e.fixed[v] = true; }
            else if (c == '[') { i_++; bracket(e.fixed); }
            else if (c == '$') { i_++; e.holes.push_back(word()); }
            else { i_++; e.fixed[c] = true; }
        }
    }
    std::string quoted() {
        need('"');
        std::string out;
        while (true) {
            if (i_ >= n_) die("unterminated string");
            int c = static_cast<unsigned char>(s_[i_++]);
            if (c == '"') return out;
            if (c == '\\') c = backslash(nullptr);
            out.push_back(static_cast<char>(c));
        }
    }
    std::unique_ptr<Op> body_or_none() { return operator_(true); }

    // Calls fn(key) for every key=value pair up to the closing parenthesis.
    template <class F> void keywords(F fn) {
        while (true) {
            int c = look();
            if (c == ')') { i_++; return; }
            if (c == ',') { i_++; continue; }
            std::string key = word();
            need('=');
            fn(key);
        }
    }

    std::unique_ptr<Op> wait_() {
        auto op = std::make_unique<Op>(Op::WAIT);
        bool has_body = false;
        keywords([&](const std::string &k) {
            if (k == "allow") op->allow = set();
            else if (k == "denies") op->denies = set();
            else if (k == "wait") op->wait = set();
            else if (k == "true_waits") op->twait = set();
            else if (k == "false_waits") op->fwait = set();
            else if (k == "body") { op->body = body_or_none(); has_body = true; }
            else if (k == "max") {
                look();
                uint64_t v = 0; size_t b = i_;
                while (i_ < n_ && s_[i_] >= '0' && s_[i_] <= '9') {
                    v = v * 10 + static_cast<uint64_t>(s_[i_++] - '0');
                    if (v > 0x7FFFFFFFull) die("max too large");
                }
                if (i_ == b) die("max needs a number");
                op->bounded = true; op->max = static_cast<uint32_t>(v);
            } else die("unknown Wait argument '" + k + "'");
        });
        if (op->allow.present && op->denies.present) die("give allow or denies, not both");
        if (op->twait.present || op->fwait.present) {
            if (!op->twait.present || !op->fwait.present || op->wait.present || has_body || op->bounded)
                die("a condition Wait takes allow, true_waits and false_waits only");
            op->kind = Op::COND;
        } else if (!op->wait.present) die("Wait needs wait=");
        return op;
    }

    std::unique_ptr<Op> operator_(bool none_ok) {
        std::string name = word();
        if (name == "None") {
            if (!none_ok) die("None is only valid as a body");
            return nullptr;
        }
        need('(');
        if (name == "Sequence") {
            auto op = std::make_unique<Op>(Op::SEQ);
            while (true) {
                int c = look();
                if (c == ')') { i_++; return op; }
                if (c == ',') { i_++; continue; }
                op->kids.push_back(operator_(false));
            }
        }
        if (name == "Write") {
            auto op = std::make_unique<Op>(Op::WRITE);
            if (look() == '$') { i_++; op->hole = word(); } else op->bytes = quoted();
            need(')');
            return op;
        }
        if (name == "Wait") return wait_();
        if (name == "IfElse" || name == "DoWhile") {
            bool is_if = name == "IfElse";
            auto op = std::make_unique<Op>(is_if ? Op::IFELSE : Op::DOWHILE);
            keywords([&](const std::string &k) {
                if (k == "condition") op->cond = operator_(false);
                else if (is_if && k == "if_body") op->if_body = body_or_none();
                else if (is_if && k == "else_body") op->else_body = body_or_none();
                else if (!is_if && k == "body") op->body = body_or_none();
                else die("unknown " + name + " argument '" + k + "'");
            });
            if (!op->cond || op->cond->kind != Op::COND)
                die(name + " needs condition=Wait(allow, true_waits, false_waits)");
            return op;
        }
        die("unknown operator '" + name + "'");
    }
};

// ---- instantiation + flattening -------------------------------------------------------------

class Flattener {
  public:
    Flattener(Table &t, const wg_args_t *args, uint32_t instance)
        : t_(t), args_(args), inst_(instance) {}

    // Appends the states of one instance (root .. END) and returns its start state.
    uint32_t run(const Op *root) {
        uint32_t base = static_cast<uint32_t>(t_.states.size());
        uint32_t n = leaves(root);
        n_leaves_ = n;
        end_ = base + n;
        t_.states.resize(end_ + 1);
        t_.tmpl.resize(end_ + 1, inst_);
        t_.lit.resize(end_ + 1, 0);
        StateDesc &e = t_.states[end_];
        e = StateDesc{};
        e.kind_byte = WG_KIND_END;
        e.next_a = e.next_b = WG_SID_ERROR;
        e.max = WG_UNBOUNDED;
        eos_exits_.clear();
        emit(root, base, end_);
        return n ? base : end_;
    }
    uint32_t end_state() const { return end_; }
    uint32_t num_leaves() const { return n_leaves_; }
    // states whose EOS exit must be patched once the start state is known
    const std::vector<uint32_t> &eos_exits() const { return eos_exits_; }

  private:
    Table &t_; const wg_args_t *args_; uint32_t inst_; uint32_t end_ = 0, n_leaves_ = 0;
    std::vector<uint32_t> eos_exits_;
    std::unordered_map<const Op *, uint32_t> size_memo_;

    const uint8_t *arg(const std::string &name, uint64_t &len) const {
        if (args_)
            for (uint32_t a = 0; a < args_->n; a++)
                if (name == args_->names[a]) { len = args_->lens[a]; return args_->data[a]; }
        throw ParseError("unbound argument $" + name);
    }
    std::string literal(const Op *w) const {
        if (w->hole.empty()) return w->bytes;
        uint64_t len; const uint8_t *d = arg(w->hole, len);
        return std::string(reinterpret_cast<const char *>(d), len);
    }
    SymbolSet resolve(const SetExpr &e) const {
        SymbolSet s = e.fixed;
        for (const auto &h : e.holes) {
            uint64_t len; const uint8_t *d = arg(h, len);
            for (uint64_t k = 0; k < len; k++) s[d[k]] = true;
        }
        return s;
    }
    // number of leaf states an operator occupies
    uint32_t leaves(const Op *op) {
        if (!op) return 0;
        auto it = size_memo_.find(op);
        if (it != size_memo_.end()) return it->second;
        uint32_t n = 0;
        switch (op->kind) {
        case Op::SEQ: for (auto &k : op->kids) n += leaves(k.get()); break;
        case Op::WRITE: n = static_cast<uint32_t>(literal(op).size()); break;
        case Op::WAIT: n = 1 + leaves(op->body.get()); break;
        case Op::COND: n = 1; break;
        case Op::IFELSE: n = 1 + leaves(op->if_body.get()) + leaves(op->else_body.get()); break;
        case Op::DOWHILE: n = leaves(op->body.get()) + 1; break;
        }
        size_memo_[op] = n;
        return n;
    }
    // Pre-order numbering puts the first executed leaf of a non-empty operator at its
    // lowest id, so control entering `op` placed at `base` lands on base, or on the
    // continuation when op occupies no state.
    uint32_t entry(const Op *op, uint32_t base, uint32_t cont) { return leaves(op) ? base : cont; }

    uint32_t class_table(const SymbolSet &allow, const SymbolSet &a, const SymbolSet &b) {
        std::array<uint8_t, 256> c{};
        for (int x = 0; x < 256; x++)
            c[x] = a[x] ? CLS_EXIT_A : b[x] ? CLS_EXIT_B : allow[x] ? CLS_STAY : CLS_REJECT;
        auto it = class_ids_.find(c);
        if (it != class_ids_.end()) return it->second;
        uint32_t id = static_cast<uint32_t>(t_.classes.size() / 256);
        t_.classes.insert(t_.classes.end(), c.begin(), c.end());
        class_ids_[c] = id;
        return id;
    }
    void checkpoint(uint32_t sid, uint32_t kind, const SetExpr &allow_e, const SetExpr &denies_e,
                    const SetExpr &a_e, const SetExpr &b_e, uint32_t ta, uint32_t tb, uint32_t max) {
        SymbolSet allow{};
        if (denies_e.present) {
            SymbolSet d = resolve(denies_e);
            if (d[kSymEos]) throw ParseError("<eos> cannot be denied");
            for (int x = 0; x < 256; x++) allow[x] = !d[x];
        } else if (allow_e.present) allow = resolve(allow_e);
        SymbolSet a = resolve(a_e), b{};
        if (b_e.present) b = resolve(b_e);
        for (int x = 0; x <= 256; x++)
            if (a[x] && b[x]) throw ParseError("true_waits and false_waits overlap");
        if (allow[kSymEos] && !a[kSymEos] && !b[kSymEos])
            throw ParseError("<eos> in allow but in no wait set");
        StateDesc &d = t_.states[sid];
        d = StateDesc{};
        d.kind_byte = kind;
        d.next_a = ta; d.next_b = tb;
        d.max = max;
        d.cls = class_table(allow, a, b);
        d.eos_next = WG_SID_ERROR;
        if (a[kSymEos] || b[kSymEos]) {
            if ((a[kSymEos] ? ta : tb) != end_)
                throw ParseError("operators follow an exit taken on <eos>");
            eos_exits_.push_back(sid);
        }
    }
    void emit(const Op *op, uint32_t base, uint32_t cont) {
        if (!op) return;
        static const SetExpr none{};
        switch (op->kind) {
        case Op::WRITE: {
            std::string b = literal(op);
            for (size_t k = 0; k < b.size(); k++) {
                StateDesc &d = t_.states[base + k];
                d = StateDesc{};
                d.kind_byte = WG_KIND_LIT | (static_cast<uint32_t>(static_cast<uint8_t>(b[k])) << 8);
                d.next_a = (k + 1 < b.size()) ? base + static_cast<uint32_t>(k) + 1 : cont;
                d.next_b = WG_SID_ERROR; d.eos_next = WG_SID_ERROR; d.max = WG_UNBOUNDED;
                d.run = static_cast<uint32_t>(b.size() - k);
                d.cls = cont;                         // LIT states reuse cls: successor of the whole run
                t_.lit[base + k] = static_cast<uint8_t>(b[k]);
            }
            break;
        }
        case Op::WAIT:
            checkpoint(base, WG_KIND_WAIT, op->allow, op->denies, op->wait, none,
                       entry(op->body.get(), base + 1, cont), WG_SID_ERROR,
                       op->bounded ? op->max : WG_UNBOUNDED);
            emit(op->body.get(), base + 1, cont);
            break;
        case Op::COND:
            throw ParseError("a condition Wait is only valid inside IfElse / DoWhile");
        case Op::SEQ: {
            // walk the children right to left so each one knows what runs after it
            uint32_t at = base + leaves(op), after = cont;
            for (size_t k = op->kids.size(); k-- > 0;) {
                const Op *kid = op->kids[k].get();
                at -= leaves(kid);
                emit(kid, at, after);
                after = entry(kid, at, after);
            }
            break;
        }
        case Op::IFELSE: {
            uint32_t ib = base + 1, eb = ib + leaves(op->if_body.get());
            checkpoint(base, WG_KIND_COND, op->cond->allow, none, op->cond->twait, op->cond->fwait,
                       entry(op->if_body.get(), ib, cont), entry(op->else_body.get(), eb, cont),
                       WG_UNBOUNDED);
            emit(op->if_body.get(), ib, cont);
            emit(op->else_body.get(), eb, cont);
            break;
        }
        case Op::DOWHILE: {
            uint32_t c = base + leaves(op->body.get());
            checkpoint(c, WG_KIND_COND, op->cond->allow, none, op->cond->twait, op->cond->fwait,
                       entry(op->body.get(), base, c), cont, WG_UNBOUNDED);
            emit(op->body.get(), base, c);
            break;
        }
        }
    }

  public:
    std::map<std::array<uint8_t, 256>, uint32_t> class_ids_;
};

}  // namespace

struct LoweringState {
    std::unordered_map<std::string, std::unique_ptr<Op>> parsed;     // static structures, by text
    std::map<std::array<uint8_t, 256>, uint32_t> class_ids;
    // Instances seen so far by the shape of their lowered states (state ids taken relative to the
    // instance's first state): the first state of the first instance of each shape.  A later
    // instance of the same shape -- the same structure instantiated with the same arguments --
    // has, state for state, the same masks, so its states share that instance's cache keys.
    std::unordered_map<std::string, uint32_t> shapes;
    // WG_SHARE_STATES: states by what they and the states ahead of them do with bytes.  `own_part`
    // numbers the tuples {kind and literal byte, class table, bound, EOS accepted} in the order
    // they are first seen, `levels` the tuples {level, the state's own part, the numbers of its
    // two successors one level lower}.  A state's number at level lmax - 1 (its own part when
    // lmax is 1) stands for everything a token can see of it; `sig_key` has the first cache key
    // of the first state seen with each such number.
    // (an open-addressing table: a tuple's number is its place in `tuples`; the lowering of a
    // workload numbers a million tuples, which a node per tuple makes ten times slower)
    struct Numbering {
        std::vector<std::array<uint32_t, 4>> tuples;
        std::vector<uint32_t> slots;                  // number + 1, 0: free; a power of two of them
        static uint64_t mix(const std::array<uint32_t, 4> &a) {
            uint64_t h = ((uint64_t)a[0] << 32 | a[1]) * 0x9E3779B97F4A7C15ull;
            h ^= h >> 29;
            h += ((uint64_t)a[2] << 32 | a[3]) * 0xC2B2AE3D27D4EB4Full;
            h ^= h >> 31;
            return h * 0x165667B19E3779F9ull;
        }
        void grow() {
            std::vector<uint32_t> wider(slots.empty() ? 1024u : slots.size() * 2u, 0u);
            for (uint32_t i = 0; i < tuples.size(); i++) {
                size_t at = (mix(tuples[i]) >> 20) & (wider.size() - 1u);
                while (wider[at]) at = (at + 1u) & (wider.size() - 1u);
                wider[at] = i + 1u;
            }
            slots.swap(wider);
        }
        uint32_t number(const std::array<uint32_t, 4> &t) {
            if ((tuples.size() + 1u) * 2u > slots.size()) grow();
            size_t at = (mix(t) >> 20) & (slots.size() - 1u);
            while (slots[at]) {
                if (tuples[slots[at] - 1u] == t) return slots[at] - 1u;
                at = (at + 1u) & (slots.size() - 1u);
            }
            tuples.push_back(t);
            slots[at] = (uint32_t)tuples.size();
            return (uint32_t)tuples.size() - 1u;
        }
    };
    Numbering own_part, levels;
    std::unordered_map<uint32_t, uint32_t> sig_key;
};

namespace {
// The states [first, end] of one instance as bytes that do not depend on where the instance lies
// in the table.
std::string shape_of(const Table &t, uint32_t first, uint32_t end) {
    std::string out;
    out.reserve((size_t)(end - first + 1) * 29);
    auto rel = [&](uint32_t sid) { return sid == WG_SID_ERROR || sid == WG_SID_FINAL ? sid : sid - first + 1u; };
    auto put = [&](uint32_t x) { out.append(reinterpret_cast<const char *>(&x), 4); };
    for (uint32_t s = first; s <= end; s++) {
        const StateDesc &d = t.states[s];
        const bool lit = (d.kind_byte & 0xFFu) == WG_KIND_LIT;
        put(d.kind_byte); put(rel(d.next_a)); put(rel(d.next_b)); put(rel(d.eos_next));
        put(lit ? rel(d.cls) : d.cls); put(d.max); put(d.run);
    }
    return out;
}
}  // namespace

Lowering::Lowering(uint32_t flags, uint32_t lmax) : st_(new LoweringState) {
    Table &t = table;
    t.flags = flags; t.lmax = lmax;
    StateDesc fin{};
    fin.kind_byte = WG_KIND_FINAL;
    fin.next_a = fin.next_b = WG_SID_ERROR;
    fin.eos_next = WG_SID_FINAL;
    fin.max = WG_UNBOUNDED;
    fin.key_base = 0;
    t.states.push_back(fin);
    t.tmpl.push_back(0);
    t.lit.push_back(0);
    t.key_count.push_back(1);
    t.n_keys = 1;
    t.classes.assign(256, CLS_REJECT);                 // table 0: rejects every byte
    st_->class_ids[std::array<uint8_t, 256>{}] = 0;
}

Lowering::~Lowering() { delete st_; }

void Lowering::add(const char *const *templates, const wg_args_t *args, uint32_t n) {
    Table &t = table;
    const size_t n_states0 = t.states.size(), n_classes0 = t.classes.size() / 256, n_start0 = t.start.size();
    const uint32_t n_keys0 = t.n_keys;
    std::vector<std::pair<uint32_t, uint32_t>> spans;                 // first and END state of each new instance
    auto roll_back = [&]() {
        t.states.resize(n_states0); t.tmpl.resize(n_states0); t.lit.resize(n_states0);
        t.key_count.resize(n_states0); t.start.resize(n_start0); t.classes.resize(n_classes0 * 256);
        t.n_keys = n_keys0;
        for (auto it = st_->class_ids.begin(); it != st_->class_ids.end();)
            it = it->second >= n_classes0 ? st_->class_ids.erase(it) : std::next(it);
    };
    for (uint32_t i = 0; i < n; i++) {
        try {
            if (!templates[i]) throw ParseError("null template text");
            std::string text(templates[i]);
            auto it = st_->parsed.find(text);
            if (it == st_->parsed.end()) {
                Reader r(templates[i]);
                it = st_->parsed.emplace(text, r.parse_all()).first;
            }
            Flattener f(t, args ? &args[i] : nullptr, static_cast<uint32_t>(t.start.size()));
            f.class_ids_.swap(st_->class_ids);
            uint32_t start;
            try { start = f.run(it->second.get()); }
            catch (...) { f.class_ids_.swap(st_->class_ids); throw; }
            f.class_ids_.swap(st_->class_ids);
            uint32_t after_eos = (t.flags & WG_EOS_RESTART) ? start : WG_SID_FINAL;
            t.states[f.end_state()].eos_next = after_eos;
            for (uint32_t s : f.eos_exits()) t.states[s].eos_next = after_eos;
            t.start.push_back(start);
            spans.emplace_back(f.end_state() - f.num_leaves(), f.end_state());
        } catch (const ParseError &e) {
            roll_back();
            throw std::runtime_error("template " + std::to_string(i) + ": " + e.what());
        } catch (...) {
            roll_back();
            throw;
        }
    }
    // cache keys: one mask per state, lmax+1 for a bounded Wait (one per remaining budget
    // 0..lmax; a larger budget cannot bind inside a single token).  An instance whose lowered
    // states equal those of an earlier instance takes that instance's keys: the global cache
    // then serves every request of that shape from one set of rows.
    t.key_count.resize(t.states.size());
    uint32_t k = n_keys0;
    std::vector<std::string> new_shapes;                              // to take back if memory runs out half way
    std::vector<uint32_t> new_sigs;
    try {
        for (const auto &span : spans) {
            const uint32_t first = span.first, end = span.second;
            for (uint32_t s = first; s <= end; s++) {
                const StateDesc &d = t.states[s];
                const bool bounded = (d.kind_byte & 0xFF) == WG_KIND_WAIT && d.max != WG_UNBOUNDED;
                t.key_count[s] = bounded ? t.lmax + 1 : 1;
            }
            std::string shape = shape_of(t, first, end);
            const auto seen = st_->shapes.find(shape);
            if (seen != st_->shapes.end()) {
                const uint32_t twin = seen->second;
                for (uint32_t s = first; s <= end; s++) t.states[s].key_base = t.states[twin + (s - first)].key_base;
                continue;
            }
            new_shapes.push_back(shape);
            st_->shapes.emplace(std::move(shape), first);
            auto inside = [&](uint32_t sid) { return sid == WG_SID_ERROR || sid == WG_SID_FINAL || (sid >= first && sid <= end); };
            bool closed = true;                      // (every successor lies in the instance itself)
            for (uint32_t s = first; s <= end; s++) closed = closed && inside(t.states[s].next_a) && inside(t.states[s].next_b);
            if (!(t.flags & WG_SHARE_STATES) || !closed) {
                for (uint32_t s = first; s <= end; s++) {
                    t.states[s].key_base = k;
                    k += t.key_count[s];
                }
                continue;
            }
            // States with equal futures share their keys.  Level 0 numbers a state by its own
            // part: kind and literal byte, class table, bound, whether EOS is accepted (where
            // EOS leads does not show in a mask).  Level l + 1 adds the level-l numbers of the
            // two successors, which lie in the same instance or are FINAL / none.  A token of n
            // bytes sees the states up to n - 1 transitions ahead, so lmax - 1 levels decide.
            const uint32_t n_inst = end - first + 1u;
            std::vector<uint32_t> own(n_inst), cur(n_inst), nxt(n_inst);
            auto at_level = [&](const std::vector<uint32_t> &ids, uint32_t sid) {
                return sid == WG_SID_ERROR ? 0xFFFFFFFFu : sid == WG_SID_FINAL ? 0xFFFFFFFEu : ids[sid - first];
            };
            for (uint32_t s = first; s <= end; s++) {
                const StateDesc &d = t.states[s];
                const uint32_t kind = d.kind_byte & 0xFFu;
                const bool ckpt = kind == WG_KIND_WAIT || kind == WG_KIND_COND;
                own[s - first] = cur[s - first] =
                    st_->own_part.number({d.kind_byte, ckpt ? d.cls : 0u, d.max, d.eos_next != WG_SID_ERROR ? 1u : 0u});
            }
            for (uint32_t level = 1; level < t.lmax; level++) {
                for (uint32_t s = first; s <= end; s++) {
                    const StateDesc &d = t.states[s];
                    nxt[s - first] = st_->levels.number({level, own[s - first], at_level(cur, d.next_a), at_level(cur, d.next_b)});
                }
                cur.swap(nxt);
            }
            for (uint32_t s = first; s <= end; s++) {
                const auto known = st_->sig_key.find(cur[s - first]);
                if (known != st_->sig_key.end()) { t.states[s].key_base = known->second; continue; }
                st_->sig_key.emplace(cur[s - first], k);
                new_sigs.push_back(cur[s - first]);
                t.states[s].key_base = k;
                k += t.key_count[s];
            }
        }
    } catch (...) {
        for (const std::string &sh : new_shapes) st_->shapes.erase(sh);
        for (uint32_t sig : new_sigs) st_->sig_key.erase(sig);
        roll_back();
        throw;
    }
    t.n_keys = k;
}

}  // namespace wg
