// Contraction planner: mode strings -> StridedBatchedGemm arguments.  Host only, no device calls.
//
// The planner works in three stages that mirror how the paper reads a BLAS call off a notated
// contraction (section III-B, Table I):
//   1. parse the (optionally annotated) mode strings and check eq. (1) of section II-B;
//   2. fix an evaluation = which modes are batched "[x]" and which are flattened "(xy)", either
//      from the annotations or from a strategy (priorities of section IV-D, Algorithm 2);
//   3. lower that evaluation to GEMM operands: operand order by rule 4, N/T from the unit-stride
//      mode of each operand, rule 1 (no batching of an operand's unit-stride mode unless an
//      extended operation of section III-E is allowed), rules 2 and 3 for flattening.
// Table II is not stored anywhere: stage 3 applied to the 36 order-2 x order-3 cases yields it.
//
// Nothing here touches the heap: a contraction has at most 3 * SB_MAX_MODES indices, so every list
// is a fixed-capacity array on the stack and the notation is rendered into a character buffer.
// Planning a launch-bound contraction then costs a fraction of a microsecond.
#include "../../include/sbgemm.h"

#include <algorithm>
#include <cstring>

namespace {

enum { TA = 0, TB = 1, TC = 2 };
constexpr int MAX_IDX = 3 * SB_MAX_MODES;       // distinct indices of one contraction
constexpr int MAX_GROUPS = 3 * SB_MAX_MODES / 2; // flattened runs (each has at least two members)

// Fixed-capacity list with the few std::vector members the planner uses.  Capacities are chosen so
// that no input that passes parse_modes can overflow them; push_back beyond capacity is dropped.
template <typename T, int N>
struct Vec {
    T v[N];
    int n = 0;
    Vec() {}
    Vec(int count, const T &x) : n(count < N ? count : N) { for (int i = 0; i < n; ++i) v[i] = x; }
    void push_back(const T &x) { if (n < N) v[n++] = x; }
    int size() const { return n; }
    bool empty() const { return n == 0; }
    void clear() { n = 0; }
    void assign(int count, const T &x) { n = count < N ? count : N; for (int i = 0; i < n; ++i) v[i] = x; }
    T &operator[](int i) { return v[i]; }
    const T &operator[](int i) const { return v[i]; }
    T &back() { return v[n - 1]; }
    const T &back() const { return v[n - 1]; }
    T *begin() { return v; }
    T *end() { return v + n; }
    const T *begin() const { return v; }
    const T *end() const { return v + n; }
    bool operator==(const Vec &o) const
    {
        if (n != o.n) return false;
        for (int i = 0; i < n; ++i)
            if (!(v[i] == o.v[i])) return false;
        return true;
    }
};

typedef Vec<int, SB_MAX_MODES> Run;             // positions or index ids of one flattened run / one tensor's modes
typedef Vec<Run, MAX_GROUPS> Runs;
typedef Vec<bool, MAX_IDX> Flags;

// stable insertion sort (std::stable_sort may allocate a merge buffer)
template <typename T, typename Less>
void stable_sort_small(T *first, T *last, Less less)
{
    for (T *i = first; i != last; ++i)
        for (T *j = i; j != first && less(*j, *(j - 1)); --j) std::swap(*j, *(j - 1));
}

// bounded character buffer for the notation
struct Text {
    char c[192];
    int n = 0;
    Text() { c[0] = 0; }
    Text &operator+=(char ch) { if (n + 1 < (int)sizeof(c)) { c[n++] = ch; c[n] = 0; } return *this; }
    Text &operator+=(const char *s) { while (*s) *this += *s++; return *this; }
    Text &operator+=(const Text &t) { return *this += t.c; }
};

struct ParsedTensor {
    Vec<char, SB_MAX_MODES + 1> label;      // one spare slot so that "too many modes" is seen
    Vec<bool, SB_MAX_MODES + 1> batched;
    Runs groups;                            // positions (within this tensor) of flattened runs
    bool annotated = false;
};

struct Index {
    char label;
    int64_t ext;
    int pos[3];       // position in A, B, C or -1
    int64_t s[3];     // element stride in A, B, C (0 if absent)
    int owner;        // TA or TB for a free index, -1 for the contracted one
};

struct Problem {
    Vec<Index, MAX_IDX> idx;
    int order[3];
    Run modes[3];                // index ids in stored order
    int k;                       // id of the contracted index
};

// A free mode of the evaluation after flattening: one index or a run of flattened indices.
struct SMode {
    Run mem;                // index ids, first (fastest) member first
    int64_t ext;
    int64_t sOwner, sC;     // stride of the first member in the owning input tensor and in C
    int owner;
    int posC;               // position of the first member in C
    bool batched;
};

bool is_letter(char c) { return (c >= 'a' && c <= 'z') || (c >= 'A' && c <= 'Z'); }

int parse_modes(const char *s, ParsedTensor &t)
{
    size_t n = std::strlen(s);
    size_t i = 0;
    while (i < n) {
        char c = s[i];
        if (is_letter(c)) {
            if (t.label.size() >= SB_MAX_MODES) return SB_ERR_MODES;
            t.label.push_back(c);
            t.batched.push_back(false);
            ++i;
        } else if (c == '[' || c == '(') {
            char close = (c == '[') ? ']' : ')';
            size_t j = i + 1;
            Run run;
            while (j < n && is_letter(s[j])) {
                if (t.label.size() >= SB_MAX_MODES) return SB_ERR_MODES;
                run.push_back((int)t.label.size());
                t.label.push_back(s[j]);
                t.batched.push_back(c == '[');
                ++j;
            }
            if (j >= n || s[j] != close) return SB_ERR_MODES;
            if (run.empty() || (c == '(' && run.size() < 2)) return SB_ERR_MODES;
            if (c == '(') t.groups.push_back(run);
            t.annotated = true;
            i = j + 1;
        } else {
            return SB_ERR_MODES;
        }
    }
    for (int a = 0; a < t.label.size(); ++a)
        for (int b = 0; b < a; ++b)
            if (t.label[a] == t.label[b]) return SB_ERR_MODES;
    return SB_OK;
}

int find_index(const Problem &P, char label)
{
    for (int i = 0; i < P.idx.size(); ++i)
        if (P.idx[i].label == label) return i;
    return -1;
}

// Stage 1: index table, eq. (1) checks, strides (packed when none are given).
int build_problem(const ParsedTensor pt[3], const int64_t *dims[3], const int64_t *strides[3], Problem &P)
{
    for (int t = 0; t < 3; ++t) {
        P.order[t] = (int)pt[t].label.size();
        int64_t packed = 1;
        for (int j = 0; j < P.order[t]; ++j) {
            int id = find_index(P, pt[t].label[j]);
            int64_t ext;
            if (dims[t]) {
                ext = dims[t][j];
            } else {                      // only C may omit its extents (checked by the caller)
                if (id < 0) return SB_ERR_CONTRACTION;
                ext = P.idx[id].ext;
            }
            if (ext < 0) return SB_ERR_EXTENT;
            if (id < 0) {
                Index ix;
                ix.label = pt[t].label[j];
                ix.ext = ext;
                ix.owner = -1;
                for (int q = 0; q < 3; ++q) { ix.pos[q] = -1; ix.s[q] = 0; }
                P.idx.push_back(ix);
                id = (int)P.idx.size() - 1;
            } else if (P.idx[id].ext != ext) {
                return SB_ERR_EXTENT;
            }
            int64_t st = strides[t] ? strides[t][j] : packed;
            if (st < 0 || (st == 0 && ext > 1)) return SB_ERR_STRIDE;
            P.idx[id].pos[t] = j;
            P.idx[id].s[t] = st;
            P.modes[t].push_back(id);
            packed *= std::max<int64_t>(ext, 1);     // an empty mode keeps later strides usable
        }
    }
    // eq. (1): C's indices are those in exactly one of A, B; the ones in both are contracted.
    P.k = -1;
    int ncontracted = 0;
    for (int i = 0; i < P.idx.size(); ++i) {
        Index &ix = P.idx[i];
        bool a = ix.pos[TA] >= 0, b = ix.pos[TB] >= 0, c = ix.pos[TC] >= 0;
        if (a && b) {
            if (c) return SB_ERR_CONTRACTION;
            ++ncontracted;
            P.k = (int)i;
        } else if (a || b) {
            if (!c) return SB_ERR_CONTRACTION;
            ix.owner = a ? TA : TB;
        } else {
            return SB_ERR_CONTRACTION;      // an index of C that neither input has
        }
    }
    if (ncontracted != 1) return SB_ERR_CONTRACTION;   // single-index contractions only
    // The output must not alias itself: sorted by stride, every mode of C has to step over the
    // whole extent of the previous one (padding allowed).
    Run byStride;
    for (int j = 0; j < P.order[TC]; ++j)
        if (P.idx[P.modes[TC][j]].ext > 1) byStride.push_back(P.modes[TC][j]);
    stable_sort_small(byStride.begin(), byStride.end(), [&](int x, int y) { return P.idx[x].s[TC] < P.idx[y].s[TC]; });
    for (int j = 1; j < byStride.size(); ++j) {
        const Index &lo = P.idx[byStride[j - 1]], &hi = P.idx[byStride[j]];
        if (hi.s[TC] < lo.s[TC] * lo.ext) return SB_ERR_STRIDE;
    }
    return SB_OK;
}

// Rules 2 and 3 for flattening index b directly after index a (a runs faster).
bool can_flatten_pair(const Problem &P, int a, int b)
{
    const Index &x = P.idx[a], &y = P.idx[b];
    if (x.owner < 0 || y.owner < 0 || x.owner != y.owner) return false;
    int o = x.owner;
    if (y.pos[TC] != x.pos[TC] + 1 || y.pos[o] != x.pos[o] + 1) return false;   // same order on both sides
    return y.s[TC] == x.s[TC] * x.ext && y.s[o] == x.s[o] * x.ext;              // ld<j> = ld<i> * dim<i>
}

// Free modes of the evaluation in C's order, given the batched flags and the flattened runs.
typedef Vec<SMode, SB_MAX_MODES> SModes;

int make_smodes(const Problem &P, const Flags &batched, const Runs &groups, SModes &out)
{
    Vec<int, MAX_IDX> group_of(P.idx.size(), -1);
    for (int g = 0; g < groups.size(); ++g) {
        const Run &run = groups[g];
        for (int j = 0; j < run.size(); ++j) {
            if (run[j] == P.k || group_of[run[j]] >= 0 || batched[run[j]]) return SB_ERR_ILLEGAL_EVAL;
            group_of[run[j]] = (int)g;
            if (j > 0 && !can_flatten_pair(P, run[j - 1], run[j])) return SB_ERR_ILLEGAL_EVAL;
        }
    }
    out.clear();
    for (int j = 0; j < P.order[TC]; ++j) {
        int id = P.modes[TC][j];
        int g = group_of[id];
        if (g >= 0 && groups[g][0] != id) continue;      // later member of a run already emitted
        SMode m;
        if (g >= 0) m.mem = groups[g]; else m.mem.push_back(id);
        m.ext = 1;
        for (int q = 0; q < m.mem.size(); ++q) m.ext *= P.idx[m.mem[q]].ext;
        const Index &first = P.idx[m.mem[0]];
        m.owner = first.owner;
        m.sOwner = first.s[first.owner];
        m.sC = first.s[TC];
        m.posC = first.pos[TC];
        m.batched = batched[id];
        out.push_back(m);
    }
    return SB_OK;
}

struct Operand {
    int op;
    int64_t ld, ex;
    bool needs_ex;
};

// A rows x cols matrix whose element (i,j) sits at i*rs + j*cs: which GEMM op reads it?
int lower_operand(int64_t rows, int64_t cols, int64_t rs, int64_t cs, Operand &o)
{
    o.ex = 0;
    o.needs_ex = false;
    if (rows == 1 || rs == 1) {                 // stored as is: columns are contiguous
        o.op = SB_OP_N;
        o.ld = (cols > 1) ? cs : std::max<int64_t>(1, rows);
        if (cols > 1 && o.ld < rows) return SB_ERR_STRIDE;
        return SB_OK;
    }
    if (cols == 1 || cs == 1) {                 // stored transposed
        o.op = SB_OP_T;
        o.ld = rs;
        if (o.ld < cols) return SB_ERR_STRIDE;
        return SB_OK;
    }
    o.needs_ex = true;                          // strided in rows and columns (rule 1 violated)
    return SB_OK;
}

Text render_tensor(const Problem &P, int t, char name, const SModes &sm)
{
    Text s;
    s += name;
    s += '_';
    const Run &modes = P.modes[t];
    for (int j = 0; j < modes.size();) {
        int id = modes[j];
        const SMode *hit = nullptr;
        for (int q = 0; q < sm.size(); ++q)
            if (sm[q].mem[0] == id) hit = &sm[q];
        if (hit && hit->mem.size() > 1) {
            s += '(';
            for (int q = 0; q < hit->mem.size(); ++q) s += P.idx[hit->mem[q]].label;
            s += ')';
            j += hit->mem.size();
        } else if (hit && hit->batched) {
            s += '[';
            s += P.idx[id].label;
            s += ']';
            ++j;
        } else {
            s += P.idx[id].label;
            ++j;
        }
    }
    return s;
}

// Stage 3: lower an evaluation (free modes with batched flags) to StridedBatchedGemm arguments.
int lower(const Problem &P, const SModes &sm, bool allow_ex, sb_plan *out)
{
    Run fr, bt;
    for (int i = 0; i < sm.size(); ++i) (sm[i].batched ? bt : fr).push_back(i);
    if (fr.size() > 2) return SB_ERR_ILLEGAL_EVAL;
    int r = -1, c = -1;
    if (fr.size() == 2) {
        int a = fr[0], b = fr[1];
        if (sm[a].owner == sm[b].owner) return SB_ERR_ILLEGAL_EVAL;   // two free modes of one tensor are no matrix product
        if (sm[a].sC == 1 || sm[a].ext == 1) { r = a; c = b; }
        else if (sm[b].sC == 1 || sm[b].ext == 1) { r = b; c = a; }
        else return SB_ERR_ILLEGAL_EVAL;                              // C strided in rows and columns
    } else if (fr.size() == 1) {
        int f = fr[0];
        if (sm[f].sC == 1 || sm[f].ext == 1) r = f; else c = f;
    }
    // rule 4: the tensor that owns C's row mode is the first GEMM operand
    int L, R;
    if (r >= 0) { L = sm[r].owner; R = 1 - L; }
    else if (c >= 0) { R = sm[c].owner; L = 1 - R; }
    else { L = TA; R = TB; }
    const Index &K = P.idx[P.k];
    int64_t M = (r >= 0) ? sm[r].ext : 1;
    int64_t N = (c >= 0) ? sm[c].ext : 1;
    Operand oL, oR;
    int rc = lower_operand(M, K.ext, (r >= 0) ? sm[r].sOwner : 0, K.s[L], oL);
    if (rc) return rc;
    rc = lower_operand(K.ext, N, K.s[R], (c >= 0) ? sm[c].sOwner : 0, oR);
    if (rc) return rc;
    if (oL.needs_ex && oR.needs_ex) return SB_ERR_ILLEGAL_EVAL;
    int ex_mode = -1;                       // batched mode that is an operand's unit-stride mode
    if (oL.needs_ex || oR.needs_ex) {
        if (!allow_ex) return SB_ERR_ILLEGAL_EVAL;
        int X = oL.needs_ex ? L : R;
        for (int q = 0; q < bt.size(); ++q)
            if (sm[bt[q]].owner == X && sm[bt[q]].sOwner == 1) ex_mode = bt[q];
        if (ex_mode < 0) return SB_ERR_ILLEGAL_EVAL;
        // stored matrix = the operand's two remaining modes in stored order (section III-E)
        Operand &o = oL.needs_ex ? oL : oR;
        int other = oL.needs_ex ? r : c;
        int pos_other = P.idx[sm[other].mem[0]].pos[X], pos_k = K.pos[X];
        int64_t s_other = sm[other].sOwner, s_k = K.s[X];
        bool other_first = pos_other < pos_k;
        o.ld = other_first ? s_other : s_k;
        o.ex = other_first ? s_k : s_other;
        // op(L) is (r x k): plain if r is stored first; op(R) is (k x c): plain if k is stored first
        bool plain = oL.needs_ex ? other_first : !other_first;
        o.op = plain ? SB_OP_EX_N : SB_OP_EX_T;
    }
    int64_t ldC = (c >= 0 && N > 1) ? sm[c].sC : std::max<int64_t>(1, M);
    if (N > 1 && ldC < M) return SB_ERR_STRIDE;
    if (bt.size() > SB_MAX_BATCH_LEVELS) return SB_ERR_ILLEGAL_EVAL;
    // Batch levels: the extended-operation mode must be level 0; otherwise the mode with the
    // largest extent goes innermost (section IV-D, priority 2), ties to the earlier mode of C.
    Run lv(bt);
    stable_sort_small(lv.begin(), lv.end(), [&](int x, int y) {
        if ((x == ex_mode) != (y == ex_mode)) return x == ex_mode;
        if (sm[x].ext != sm[y].ext) return sm[x].ext > sm[y].ext;
        return sm[x].posC < sm[y].posC;
    });
    std::memset(out, 0, sizeof(*out));
    out->nbatch = (int32_t)lv.size();
    out->left_is_B = (L == TB);
    out->opL = oL.op;  out->opR = oR.op;
    out->m = M;  out->n = N;  out->k = K.ext;
    out->ldL = oL.ld;  out->ldR = oR.ld;  out->ldC = ldC;
    out->exL = oL.ex;  out->exR = oR.ex;
    out->exceptional = (ex_mode >= 0);
    for (int q = 0; q < lv.size(); ++q) {
        const SMode &b = sm[lv[q]];
        if (b.sC == 0 && b.ext > 1) return SB_ERR_STRIDE;
        if (b.sC == 1 && b.ext > 1) out->exceptional = 1;   // C's first mode batched: a matrix-vector form
        out->batch[q] = b.ext;
        out->strideL[q] = (b.owner == L) ? b.sOwner : 0;
        out->strideR[q] = (b.owner == R) ? b.sOwner : 0;
        out->strideC[q] = b.sC;
    }
    // the evaluation in the paper's notation
    char nameL = (L == TA) ? 'A' : 'B', nameR = (R == TA) ? 'A' : 'B';
    const Text lhs = render_tensor(P, TC, 'C', sm);
    const Text tl = render_tensor(P, L, nameL, sm), tr = render_tensor(P, R, nameR, sm);
    Text text;
    if (r < 0 && c >= 0) {
        // row-vector times matrix: written as the matrix-vector product it is (Table II, kernel 2
        // of the exceptional rows): the matrix first, transposed relative to the GEMM's view of it
        bool t = (oR.op == SB_OP_N || oR.op == SB_OP_EX_N);
        text += lhs;  text += " = ";  text += tr;  text += (t ? "^T " : " ");  text += tl;
    } else {
        bool tL = (oL.op == SB_OP_T || oL.op == SB_OP_EX_T) && r >= 0;
        bool tR = (oR.op == SB_OP_T || oR.op == SB_OP_EX_T) && c >= 0;
        text += lhs;  text += " = ";  text += tl;  text += (tL ? "^T " : " ");  text += tr;  text += (tR ? "^T" : "");
    }
    static_assert(sizeof(text.c) == sizeof(out->notation), "the notation buffer");
    std::memcpy(out->notation, text.c, sizeof(out->notation));
    return SB_OK;
}

// Maximal runs of modes that rules 2 and 3 allow to be flattened.
Runs flatten_candidates(const Problem &P)
{
    Runs groups;
    Run run;
    for (int j = 0; j < P.order[TC]; ++j) {
        int id = P.modes[TC][j];
        if (!run.empty() && can_flatten_pair(P, run.back(), id)) {
            run.push_back(id);
        } else {
            if (run.size() > 1) groups.push_back(run);
            run.assign(1, id);
        }
    }
    if (run.size() > 1) groups.push_back(run);
    return groups;
}

// Pick the GEMM's column mode among the second operand's free modes (largest extent first, ties
// to the earlier mode of C: Algorithm 2 chooses the GEMM mode by maximum dimension), batch
// every other free mode, and keep the first choice that lowers.
int choose_columns(const Problem &P, const Runs &groups, bool allow_ex, sb_plan *out)
{
    Flags none(P.idx.size(), false);
    SModes sm;
    int rc = make_smodes(P, none, groups, sm);
    if (rc) return rc;
    if (sm.empty()) return lower(P, sm, allow_ex, out);
    int L = sm[0].owner;                    // sm[0] holds C's first mode: the row mode
    Run cand;
    for (int i = 1; i < sm.size(); ++i)
        if (sm[i].owner != L) cand.push_back(i);
    stable_sort_small(cand.begin(), cand.end(), [&](int x, int y) { return sm[x].ext > sm[y].ext; });
    if (cand.empty()) cand.push_back(-1);   // second operand is a vector: one-column GEMM
    int last = SB_ERR_ILLEGAL_EVAL;
    for (int q = 0; q < cand.size(); ++q) {
        for (int i = 1; i < sm.size(); ++i) sm[i].batched = (i != cand[q]);
        sm[0].batched = false;
        last = lower(P, sm, allow_ex, out);
        if (last == SB_OK) return SB_OK;
    }
    return last;
}

// Batched matrix-vector evaluation: C's row mode is batched too, one free mode stays.
int choose_level2(const Problem &P, sb_plan *out)
{
    Flags none(P.idx.size(), false);
    Runs nogroups;
    SModes sm;
    int rc = make_smodes(P, none, nogroups, sm);
    if (rc) return rc;
    if (sm.size() < 2) return lower(P, sm, false, out);
    int L = sm[0].owner;
    Run cand;
    for (int i = 1; i < sm.size(); ++i) cand.push_back(i);
    // the matrix comes from the tensor that holds C's first mode when it can (Table II), largest extent first
    stable_sort_small(cand.begin(), cand.end(), [&](int x, int y) {
        if ((sm[x].owner == L) != (sm[y].owner == L)) return sm[x].owner == L;
        return sm[x].ext > sm[y].ext;
    });
    int last = SB_ERR_ILLEGAL_EVAL;
    for (int q = 0; q < cand.size(); ++q) {
        for (int i = 0; i < sm.size(); ++i) sm[i].batched = (i != cand[q]);
        last = lower(P, sm, false, out);
        if (last == SB_OK) { out->exceptional = 1; return SB_OK; }
    }
    return last;
}

int plan_from_annotations(const Problem &P, const ParsedTensor pt[3], sb_plan *out)
{
    Flags batched(P.idx.size(), false);
    Runs groups;
    for (int t = 0; t < 3; ++t) {
        for (int j = 0; j < pt[t].label.size(); ++j)
            if (pt[t].batched[j]) batched[P.modes[t][j]] = true;
        for (int g = 0; g < pt[t].groups.size(); ++g) {
            Run run;
            for (int j = 0; j < pt[t].groups[g].size(); ++j) run.push_back(P.modes[t][pt[t].groups[g][j]]);
            bool seen = false;
            for (int h = 0; h < groups.size(); ++h) {
                if (groups[h] == run) { seen = true; break; }
                for (int j = 0; j < run.size(); ++j)      // overlapping but different: rule 3
                    if (std::find(groups[h].begin(), groups[h].end(), run[j]) != groups[h].end())
                        return SB_ERR_ILLEGAL_EVAL;
            }
            if (!seen) groups.push_back(run);
        }
    }
    if (batched[P.k]) return SB_ERR_ILLEGAL_EVAL;
    SModes sm;
    int rc = make_smodes(P, batched, groups, sm);
    if (rc) return rc;
    return lower(P, sm, true, out);
}

int plan_impl(const char *modesA, const char *modesB, const char *modesC,
              const int64_t *dimsA, const int64_t *stridesA,
              const int64_t *dimsB, const int64_t *stridesB,
              const int64_t *dimsC, const int64_t *stridesC,
              sb_strategy strat, sb_plan *out)
{
    if (!modesA) return -1;
    if (!modesB) return -2;
    if (!modesC) return -3;
    if (!out) return -11;
    if ((int)strat < SB_AUTO || (int)strat > SB_LEVEL2) return -10;
    ParsedTensor pt[3];
    int rc;
    if ((rc = parse_modes(modesA, pt[TA])) != 0) return rc;
    if ((rc = parse_modes(modesB, pt[TB])) != 0) return rc;
    if ((rc = parse_modes(modesC, pt[TC])) != 0) return rc;
    if (!dimsA && !pt[TA].label.empty()) return -4;
    if (!dimsB && !pt[TB].label.empty()) return -6;
    const int64_t *dims[3] = {dimsA, dimsB, dimsC};
    const int64_t *strides[3] = {stridesA, stridesB, stridesC};
    Problem P;
    if ((rc = build_problem(pt, dims, strides, P)) != 0) return rc;

    bool annotated = pt[TA].annotated || pt[TB].annotated || pt[TC].annotated;
    if (annotated) {
        if (strat != SB_AUTO) return -10;
        rc = plan_from_annotations(P, pt, out);
    } else {
        Runs nogroups;
        switch (strat) {
        case SB_AUTO: {
            // priority 1: flatten whenever possible; then the largest GEMM, batching the rest;
            // extended operations only when no plain evaluation exists (section III-E)
            const Runs groups = flatten_candidates(P);
            rc = choose_columns(P, groups, false, out);
            if (rc == SB_ERR_ILLEGAL_EVAL) rc = choose_columns(P, groups, true, out);
            if (rc == SB_ERR_ILLEGAL_EVAL) rc = choose_level2(P, out);
            break;
        }
        case SB_FLATTEN:
            rc = choose_columns(P, flatten_candidates(P), false, out);
            if (rc == SB_OK && out->nbatch != 0) rc = SB_ERR_ILLEGAL_EVAL;
            break;
        case SB_NESTED:
            rc = choose_columns(P, nogroups, false, out);
            if (rc == SB_ERR_ILLEGAL_EVAL) rc = choose_columns(P, nogroups, true, out);
            break;
        case SB_BATCH_LAST:
        case SB_BATCH_MID: {
            Flags batched(P.idx.size(), false);
            int nC = P.order[TC];
            int col = (strat == SB_BATCH_LAST) ? 1 : nC - 1;
            for (int j = 1; j < nC; ++j)
                if (j != col) batched[P.modes[TC][j]] = true;
            SModes sm;
            rc = make_smodes(P, batched, nogroups, sm);
            if (rc == SB_OK) rc = lower(P, sm, true, out);
            break;
        }
        case SB_LEVEL2:
            rc = choose_level2(P, out);
            break;
        }
    }
    return rc;
}

}  // namespace

extern "C" int sb_contract_plan(const char *modesA, const char *modesB, const char *modesC,
                                const int64_t *dimsA, const int64_t *stridesA,
                                const int64_t *dimsB, const int64_t *stridesB,
                                const int64_t *dimsC, const int64_t *stridesC,
                                sb_strategy strat, sb_plan *out)
{
    return plan_impl(modesA, modesB, modesC, dimsA, stridesA, dimsB, stridesB, dimsC, stridesC, strat, out);
}
