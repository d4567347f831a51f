// Applicability inspection on the host (Section III-B: Algorithm 1 and the array-access
// isomorphism; candidate order of Section IV-A), plus text descriptions of the MFMA
// instructions and of the operations the kernels of this library execute.
//
// A tensor program is parsed into a flat node arena; loop-variable sets are 32-bit masks.
// The loop assignment is a depth-first search over the instruction's loops in declaration
// order, trying the operation's loops of equal annotation innermost-first; a partial
// assignment whose mapped variables already leave an operand's index set is cut, which is
// exact because S'(u) only grows as loops are added.
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

#include "../../include/unit.h"

namespace {

enum NodeKind { LOAD, CONSTANT, ARITH };

struct Node {
    NodeKind kind;
    std::string type;      // data type of the node's value
    std::string name;      // LOAD: tensor; CONSTANT: literal; ARITH: opcode
    std::string index;     // LOAD: index list without blanks
    uint32_t vars = 0;     // LOAD: S(.) as a mask over the program's loops
    int child[2] = {-1, -1};
};

struct Loop {
    std::string name;
    int extent;
    bool reduction;
};

struct Program {
    std::vector<Loop> loops;
    std::vector<Node> nodes;
    int out = -1, acc = -1, body = -1;

    int loop_id(const std::string &n) const {
        for (size_t i = 0; i < loops.size(); ++i)
            if (loops[i].name == n) return (int)i;
        return -1;
    }
};

struct Parser {
    Program &p;
    const char *s;
    bool ok = true;

    explicit Parser(Program &prog, const char *text) : p(prog), s(text) {}

    void blanks() { while (*s == ' ' || *s == '\t' || *s == '\r') ++s; }
    bool at_end_of_statement() { blanks(); return *s == 0 || *s == ';' || *s == '\n'; }

    std::string word() {       // up to blank, parenthesis or statement end; brackets keep blanks
        blanks();
        std::string w;
        int depth = 0;
        while (*s && *s != ';' && *s != '\n') {
            if (*s == '[') ++depth;
            if (*s == ']') --depth;
            if (depth == 0 && (*s == ' ' || *s == '\t' || *s == '\r' || *s == '(' || *s == ')')) break;
            if (depth > 0 && (*s == ' ' || *s == '\t')) { ++s; continue; }
            w.push_back(*s++);
        }
        return w;
    }

    // index list -> mask of loop variables; false on an unknown name
    bool index_vars(const std::string &idx, uint32_t *mask) {
        *mask = 0;
        size_t i = 0;
        while (i < idx.size()) {
            size_t j = i;
            while (j < idx.size() && idx[j] != ',' && idx[j] != '+' && idx[j] != '-') ++j;
            std::string term = idx.substr(i, j - i);
            i = j + 1;
            if (term.empty()) continue;
            size_t star = term.rfind('*');
            std::string name = star == std::string::npos ? term : term.substr(star + 1);
            if (name.empty()) return false;
            bool number = true;
            for (char c : name) number = number && c >= '0' && c <= '9';
            if (number) continue;
            int id = p.loop_id(name);
            if (id < 0) return false;
            *mask |= 1u << id;
        }
        return true;
    }

    int access(const std::string &w) {       // NAME:TYPE[IDX]
        size_t colon = w.find(':'), lb = w.find('['), rb = w.rfind(']');
        if (colon == std::string::npos || lb == std::string::npos || rb != w.size() - 1 ||
            colon == 0 || lb < colon + 2)
            return ok = false, -1;
        Node n;
        n.kind = LOAD;
        n.name = w.substr(0, colon);
        n.type = w.substr(colon + 1, lb - colon - 1);
        n.index = w.substr(lb + 1, rb - lb - 1);
        if (!index_vars(n.index, &n.vars)) return ok = false, -1;
        p.nodes.push_back(n);
        return (int)p.nodes.size() - 1;
    }

    int expr() {
        blanks();
        if (*s == '(') {
            ++s;
            Node n;
            n.kind = ARITH;
            n.name = word();
            if (n.name.empty()) return ok = false, -1;
            if (n.name == "cast") {
                n.type = word();
                n.child[0] = expr();
                if (!ok) return -1;
            } else {
                n.child[0] = expr();
                if (!ok) return -1;
                n.child[1] = expr();
                if (!ok) return -1;
                n.type = p.nodes[n.child[0]].type;
            }
            blanks();
            if (*s != ')') return ok = false, -1;
            ++s;
            p.nodes.push_back(n);
            return (int)p.nodes.size() - 1;
        }
        std::string w = word();
        if (w.empty()) return ok = false, -1;
        if (w.compare(0, 6, "const:") == 0) {
            size_t c2 = w.find(':', 6);
            if (c2 == std::string::npos || c2 == 6 || c2 + 1 >= w.size() ||
                w.find(':', c2 + 1) != std::string::npos)
                return ok = false, -1;
            Node n;
            n.kind = CONSTANT;
            n.type = w.substr(6, c2 - 6);
            n.name = w.substr(c2 + 1);
            p.nodes.push_back(n);
            return (int)p.nodes.size() - 1;
        }
        return access(w);
    }

    bool run() {
        while (ok) {
            while (*s == ';' || *s == '\n' || *s == ' ' || *s == '\t' || *s == '\r') ++s;
            if (*s == 0) break;
            std::string head = word();
            if (head == "loop") {
                Loop l;
                l.name = word();
                std::string ext = word(), ann = word();
                char *end = nullptr;
                long e = strtol(ext.c_str(), &end, 10);
                if (l.name.empty() || ext.empty() || *end || e < 1 || e > 0x7fffffff ||
                    (ann != "dp" && ann != "red") || p.loop_id(l.name) >= 0 || p.loops.size() >= 32)
                    return false;
                l.extent = (int)e;
                l.reduction = ann == "red";
                p.loops.push_back(l);
            } else if (head == "out" || head == "acc") {
                int id = access(word());
                if (!ok) return false;
                (head == "out" ? p.out : p.acc) = id;
            } else if (head == "body") {
                p.body = expr();
                if (!ok) return false;
            } else {
                return false;
            }
            if (!at_end_of_statement()) return false;
        }
        return ok && p.out >= 0 && p.body >= 0 && !p.loops.empty();
    }
};

// One matched leaf pair: instruction node, operation node.
struct Binding { int instr, op; };

bool same_leaf(const Node &x, const Node &y) {
    return x.kind == y.kind && x.name == y.name && x.index == y.index && (x.kind == LOAD || x.type == y.type);
}

// Algorithm 1 over node indices.
bool match_trees(const Program &I, int a, const Program &O, int b, std::vector<Binding> &bind) {
    const Node &na = I.nodes[a], &nb = O.nodes[b];
    if (na.type != nb.type) return false;
    bool leaf_a = na.kind != ARITH, leaf_b = nb.kind != ARITH;
    if (leaf_a && leaf_b) {
        if (na.kind != LOAD) return false;
        for (const Binding &x : bind)
            if (same_leaf(I.nodes[x.instr], na)) return same_leaf(O.nodes[x.op], nb);
        bind.push_back({a, b});
        return true;
    }
    if (!leaf_a && !leaf_b) {
        if (na.name != nb.name) return false;
        for (int c = 0; c < 2; ++c) {
            if ((na.child[c] < 0) != (nb.child[c] < 0)) return false;
            if (na.child[c] >= 0 && !match_trees(I, na.child[c], O, nb.child[c], bind)) return false;
        }
        return true;
    }
    return false;
}

struct Pair {               // operand correspondence fed to the access check
    int instr, op;          // node ids; op < 0: constant on the operation side
};

struct Search {
    const Program &I, &O;
    const std::vector<Pair> &pairs;
    std::vector<int> assign;       // instruction loop -> operation loop
    std::vector<int> first;
    int feasible = 0;
    uint32_t used = 0;

    Search(const Program &i, const Program &o, const std::vector<Pair> &p)
        : I(i), O(o), pairs(p), assign(i.loops.size(), -1) {}

    // every pair: image of the mapped operation variables stays inside the instruction's index set
    bool consistent(int upto) const {
        for (const Pair &pr : pairs) {
            if (pr.op < 0) continue;
            uint32_t u = O.nodes[pr.op].vars, v = I.nodes[pr.instr].vars, image = 0;
            for (int il = 0; il <= upto; ++il)
                if (u >> assign[il] & 1) image |= 1u << il;
            if (image & ~v) return false;
        }
        return true;
    }

    void descend(int il) {
        if (il == (int)I.loops.size()) {
            if (feasible++ == 0) first = assign;
            return;
        }
        for (int ol = (int)O.loops.size() - 1; ol >= 0; --ol) {      // innermost first
            if (O.loops[ol].reduction != I.loops[il].reduction || (used >> ol & 1)) continue;
            assign[il] = ol;
            used |= 1u << ol;
            if (consistent(il)) descend(il + 1);
            used &= ~(1u << ol);
            assign[il] = -1;
        }
    }
};

void put(char *dst, const std::string &s) {
    snprintf(dst, UNIT_INSPECT_NAME, "%s", s.c_str());
}

int emit(char *buf, size_t cap, const char *fmt, ...) {
    char tmp[1024];
    va_list ap;
    va_start(ap, fmt);
    int n = vsnprintf(tmp, sizeof tmp, fmt, ap);
    va_end(ap);
    if (n < 0 || n >= (int)sizeof tmp) return UNIT_EINVAL;
    if (buf && cap > 0) snprintf(buf, cap, "%s", tmp);
    return n + 1;
}

const char *in_type(int dtype) { return dtype == UNIT_I8 ? "i8" : "f16"; }
const char *acc_type(int dtype) { return dtype == UNIT_I8 ? "i32" : "f32"; }

}  // namespace

extern "C" {

int unit_inspect(const char *instruction, const char *operation, unit_inspect_result *res) {
    if (!instruction || !operation || !res) return UNIT_EINVAL;
    memset(res, 0, sizeof *res);
    Program I, O;
    if (!Parser(I, instruction).run() || !Parser(O, operation).run()) return UNIT_EINVAL;
    if (I.loops.size() > UNIT_INSPECT_MAX) return UNIT_ENOTSUP;
    if (O.acc >= 0) return UNIT_EINVAL;          // only an instruction has a separate addend register

    std::vector<Binding> bind;
    bool same = I.nodes[I.out].type == O.nodes[O.out].type && match_trees(I, I.body, O, O.body, bind);
    // a register is fed from one array only
    for (size_t x = 0; same && x < bind.size(); ++x)
        for (size_t y = 0; y < x; ++y) {
            const Node &ix = I.nodes[bind[x].instr], &iy = I.nodes[bind[y].instr];
            const Node &ox = O.nodes[bind[x].op], &oy = O.nodes[bind[y].op];
            if (ix.name == iy.name && (ox.kind != oy.kind || (ox.kind == LOAD && ox.name != oy.name)))
                same = false;
        }
    if (!same) {
        res->failed_step = 1;
        return UNIT_OK;
    }

    std::vector<Pair> pairs;
    pairs.push_back({I.out, O.out});
    if (I.acc >= 0) pairs.push_back({I.acc, O.out});
    for (const Binding &b : bind) pairs.push_back({b.instr, O.nodes[b.op].kind == LOAD ? b.op : -1});

    Search search(I, O, pairs);
    search.descend(0);
    res->num_feasible = search.feasible;
    if (search.feasible == 0) {
        res->failed_step = 2;
        return UNIT_OK;
    }
    res->applicable = 1;
    res->num_loops = (int)I.loops.size();
    for (size_t il = 0; il < I.loops.size(); ++il) {
        put(res->instr_loop[il], I.loops[il].name);
        put(res->op_loop[il], O.loops[search.first[il]].name);
    }
    int count = 0;
    for (const Pair &pr : pairs) {
        const Node &v = I.nodes[pr.instr];
        bool seen = false;
        for (int x = 0; x < count; ++x) seen = seen || v.name == res->instr_operand[x];
        if (seen) continue;
        if (count == UNIT_INSPECT_MAX) return UNIT_ENOTSUP;
        put(res->instr_operand[count], v.name);
        uint32_t bc = 0;
        if (pr.op < 0) {
            put(res->op_operand[count], "const");
        } else {
            const Node &u = O.nodes[pr.op];
            put(res->op_operand[count], u.name);
            for (size_t il = 0; il < I.loops.size(); ++il)
                if ((v.vars >> il & 1) && !(u.vars >> search.first[il] & 1)) bc |= 1u << il;
        }
        res->broadcast[count++] = bc;
    }
    res->num_operands = count;
    return UNIT_OK;
}

int unit_describe_mfma(int dtype, int32_t edge, char *buf, size_t cap) {
    if ((dtype != UNIT_I8 && dtype != UNIT_F16) || (edge != 32 && edge != 16)) return UNIT_EINVAL;
    // 16 operand bytes per lane and operand; a 32-edge tile spreads k over 2 lane groups, a
    // 16-edge tile over 4
    int kk = (edge == 32 ? 32 : 64) / (dtype == UNIT_I8 ? 1 : 2);
    return emit(buf, cap,
                "loop i %d dp; loop j %d dp; loop kk %d red\n"
                "out d:%s[i,j]\n"
                "body (mul (cast %s a:%s[i,kk]) (cast %s b:%s[j,kk]))",
                edge, edge, kk, acc_type(dtype), acc_type(dtype), in_type(dtype), acc_type(dtype),
                in_type(dtype));
}

int unit_describe_conv2d(const unit_conv2d_desc *d, int dtype, char *buf, size_t cap) {
    int32_t p, q;
    if ((dtype != UNIT_I8 && dtype != UNIT_F16) || unit_conv2d_out_dims(d, &p, &q) != UNIT_OK)
        return UNIT_EINVAL;
    // the operation as the main kernel consumes it: weights [k][r][s][c], activations [n][h][w][c]
    return emit(buf, cap,
                "loop n %d dp; loop k %d dp; loop p %d dp; loop q %d dp; "
                "loop r %d red; loop s %d red; loop c %d red\n"
                "out y:%s[n,k,p,q]\n"
                "body (mul (cast %s wp:%s[k,r,s,c]) (cast %s xp:%s[n,%d*p+r-%d,%d*q+s-%d,c]))",
                d->n, d->k, p, q, d->r, d->s, d->c, acc_type(dtype), acc_type(dtype), in_type(dtype),
                acc_type(dtype), in_type(dtype), d->stride_h, d->pad_h, d->stride_w, d->pad_w);
}

int unit_describe_matmul(int32_t m, int32_t n, int32_t k, int dtype, char *buf, size_t cap) {
    if ((dtype != UNIT_I8 && dtype != UNIT_F16) || m < 1 || n < 1 || k < 1) return UNIT_EINVAL;
    // C[m,n] += A[m,k] * B[k,n] with B stored column-major, i.e. addressed as b[n,k]
    return emit(buf, cap,
                "loop m %d dp; loop n %d dp; loop k %d red\n"
                "out c:%s[m,n]\n"
                "body (mul (cast %s a:%s[m,k]) (cast %s b:%s[n,k]))",
                m, n, k, acc_type(dtype), acc_type(dtype), in_type(dtype), acc_type(dtype),
                in_type(dtype));
}

}  // extern "C"
