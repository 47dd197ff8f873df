// Grammar text front end of the library (format in pre3.h).
#include "grammar.hpp"

#include <array>
#include <cctype>
#include <map>

#include "../../include/pre3.h"

namespace pre3 {
namespace {

[[noreturn]] void fail(const std::string &msg) { throw CompileError{PRE3_E_PARSE, msg}; }

struct RuleText {
    std::string name;
    std::string body;           // everything right of ::=, continuation lines joined by " | "
    int line;
};

// One alternative before nonterminal names are resolved.
struct RawAlt {
    bool is_class = false;
    std::array<bool, 256> cls{};
    std::vector<std::pair<bool, std::string>> items;   // (is_name, name) or (false, bytes)
};

bool ident_start(char c) { return std::isalpha((unsigned char)c) || c == '_'; }
bool ident_char(char c) { return std::isalnum((unsigned char)c) || c == '_'; }

int hex_digit(char c) {
    if (c >= '0' && c <= '9') return c - '0';
    if (c >= 'a' && c <= 'f') return c - 'a' + 10;
    if (c >= 'A' && c <= 'F') return c - 'A' + 10;
    return -1;
}

// Cursor over one rule body.
class Cursor {
  public:
    Cursor(const std::string &s, int line) : s_(s), line_(line) {}
    void skip_space() { while (p_ < s_.size() && std::isspace((unsigned char)s_[p_])) ++p_; }
    bool done() const { return p_ >= s_.size(); }
    char peek() const { return p_ < s_.size() ? s_[p_] : '\0'; }
    void bump() { ++p_; }

    int escaped_byte() {
        if (done()) err("unexpected end of rule");
        char c = s_[p_++];
        if (c != '\\') return (unsigned char)c;
        if (done()) err("dangling backslash");
        char d = s_[p_++];
        switch (d) {
            case 'n': return '\n';
            case 'r': return '\r';
            case 't': return '\t';
            case '\\': case '"': case ']': case '[': case '-': case '^': return (unsigned char)d;
            case 'x': {
                if (p_ + 1 >= s_.size()) err("bad \\x escape");
                int h = hex_digit(s_[p_]), l = hex_digit(s_[p_ + 1]);
                if (h < 0 || l < 0) err("bad \\x escape");
                p_ += 2;
                return h * 16 + l;
            }
            default: err("bad escape in string or class");
        }
    }

    std::string quoted() {       // cursor sits on the opening quote
        ++p_;
        std::string out;
        for (;;) {
            if (done()) err("unterminated string");
            if (s_[p_] == '"') { ++p_; return out; }
            out.push_back((char)escaped_byte());
        }
    }

    std::array<bool, 256> char_class() {   // cursor sits on '['
        ++p_;
        std::array<bool, 256> set{};
        bool negate = false;
        if (peek() == '^') { negate = true; ++p_; }
        for (;;) {
            if (done()) err("unterminated class");
            if (s_[p_] == ']') { ++p_; break; }
            int lo = escaped_byte(), hi = lo;
            if (peek() == '-' && p_ + 1 < s_.size() && s_[p_ + 1] != ']') {
                ++p_;
                hi = escaped_byte();
                if (hi < lo) err("bad range in class");
            }
            for (int b = lo; b <= hi; ++b) set[b] = true;
        }
        if (negate) for (auto &b : set) b = !b;
        return set;
    }

    std::string identifier() {
        size_t b = p_;
        while (p_ < s_.size() && ident_char(s_[p_])) ++p_;
        return s_.substr(b, p_ - b);
    }

    [[noreturn]] void err(const std::string &m) const { fail("line " + std::to_string(line_) + ": " + m); }

  private:
    const std::string &s_;
    size_t p_ = 0;
    int line_;
};

// Cuts the text into rules; comments are removed outside strings and classes.
std::vector<RuleText> split_rules(const std::string &text) {
    std::vector<RuleText> rules;
    size_t pos = 0;
    int line_no = 0;
    while (pos <= text.size()) {
        size_t eol = text.find('\n', pos);
        if (eol == std::string::npos) eol = text.size();
        std::string line = text.substr(pos, eol - pos);
        pos = eol + 1;
        ++line_no;
        // strip a trailing comment
        bool in_str = false, in_cls = false;
        for (size_t i = 0; i < line.size(); ++i) {
            char c = line[i];
            if (c == '\\' && (in_str || in_cls)) { ++i; continue; }
            if (in_str) { if (c == '"') in_str = false; continue; }
            if (in_cls) { if (c == ']') in_cls = false; continue; }
            if (c == '"') in_str = true;
            else if (c == '[') in_cls = true;
            else if (c == '#') { line.resize(i); break; }
        }
        if (in_str) fail("line " + std::to_string(line_no) + ": unterminated string");
        if (in_cls) fail("line " + std::to_string(line_no) + ": unterminated class");
        size_t first = line.find_first_not_of(" \t\r");
        if (first == std::string::npos) continue;
        if (line[first] == '|') {
            if (rules.empty()) fail("line " + std::to_string(line_no) + ": '|' before any rule");
            rules.back().body += " " + line.substr(first);
            continue;
        }
        size_t arrow = line.find("::=");
        if (arrow == std::string::npos || !ident_start(line[first]))
            fail("line " + std::to_string(line_no) + ": expected 'Name ::= ...'");
        size_t e = first;
        while (e < line.size() && ident_char(line[e])) ++e;
        if (line.find_first_not_of(" \t", e) != arrow)
            fail("line " + std::to_string(line_no) + ": expected 'Name ::= ...'");
        rules.push_back({line.substr(first, e - first), line.substr(arrow + 3), line_no});
    }
    return rules;
}

std::vector<RawAlt> parse_body(const RuleText &r) {
    std::vector<RawAlt> alts;
    Cursor cur(r.body, r.line);
    RawAlt alt;
    bool any = false;
    auto close_alt = [&]() {
        if (!any) cur.err("rule '" + r.name + "': empty alternative must be written \"\"");
        alts.push_back(alt);
        alt = RawAlt();
        any = false;
    };
    for (;;) {
        cur.skip_space();
        if (cur.done()) { close_alt(); return alts; }
        char c = cur.peek();
        if (c == '|') { cur.bump(); close_alt(); continue; }
        if (alt.is_class) cur.err("rule '" + r.name + "': a class must be a whole alternative");
        if (c == '"') {
            alt.items.push_back({false, cur.quoted()});
        } else if (c == '[') {
            if (any) cur.err("rule '" + r.name + "': a class must be a whole alternative");
            alt.is_class = true;
            alt.cls = cur.char_class();
        } else if (ident_start(c)) {
            alt.items.push_back({true, cur.identifier()});
        } else {
            cur.err(std::string("unexpected character '") + c + "'");
        }
        any = true;
    }
}

void check_no_useless_symbols(const Grammar &g) {
    const int n = g.n_nt();
    std::vector<char> productive(n, 0), reachable(n, 0);
    for (bool changed = true; changed;) {
        changed = false;
        for (const auto &p : g.prods) {
            if (productive[p.lhs]) continue;
            bool ok = true;
            for (int x : p.rhs)
                if (x >= kNtBase && !productive[x - kNtBase]) { ok = false; break; }
            if (ok) { productive[p.lhs] = 1; changed = true; }
        }
    }
    std::vector<int> work{g.prods[0].lhs};
    reachable[g.prods[0].lhs] = 1;
    while (!work.empty()) {
        int a = work.back();
        work.pop_back();
        for (int pi : g.prods_of[a])
            for (int x : g.prods[pi].rhs)
                if (x >= kNtBase && !reachable[x - kNtBase]) {
                    reachable[x - kNtBase] = 1;
                    work.push_back(x - kNtBase);
                }
    }
    for (int a = 0; a < n; ++a) {
        if (!productive[a]) fail("nonterminal '" + g.nt_names[a] + "' derives no string");
        if (!reachable[a]) fail("nonterminal '" + g.nt_names[a] + "' is unreachable");
    }
}

}  // namespace

Grammar parse_grammar(const std::string &text) {
    std::vector<RuleText> rules = split_rules(text);
    if (rules.empty()) fail("grammar has no rules");

    Grammar g;
    std::map<std::string, int> index;
    for (const auto &r : rules)
        if (index.emplace(r.name, (int)g.nt_names.size()).second) g.nt_names.push_back(r.name);
    const int start = 0;
    const int augmented = (int)g.nt_names.size();
    g.nt_names.push_back("$accept");
    g.prods.push_back({augmented, {kNtBase + start}});

    for (const auto &r : rules) {
        const int lhs = index[r.name];
        for (const RawAlt &alt : parse_body(r)) {
            if (alt.is_class) {
                for (int b = 0; b < 256; ++b)
                    if (alt.cls[b]) g.prods.push_back({lhs, {b}});
                continue;
            }
            Production p{lhs, {}};
            for (const auto &it : alt.items) {
                if (it.first) {
                    auto f = index.find(it.second);
                    if (f == index.end()) fail("undefined nonterminal '" + it.second + "'");
                    p.rhs.push_back(kNtBase + f->second);
                } else {
                    for (unsigned char ch : it.second) p.rhs.push_back(ch);
                }
            }
            g.prods.push_back(std::move(p));
        }
    }
    g.prods_of.assign(g.n_nt(), {});
    for (int i = 0; i < (int)g.prods.size(); ++i) g.prods_of[g.prods[i].lhs].push_back(i);
    check_no_useless_symbols(g);
    return g;
}

}  // namespace pre3
