/*
 * wg_oracle.c -- CPU ORACLE.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, single-threaded, byte-at-a-time implementation of what the
 * structured-decoding hot path computes: operator trees (Sequence / Write /
 * Wait / IfElse / DoWhile) as the paper's section "Operator Building and State
 * Tracking" defines them, token verdicts and packed vocabulary masks as in
 * "Mask Generation and Global Caching", and the masking of logits described in
 * the introduction (ones = allowed, applied before sampling).  Only the test
 * suite, the smoke check and the benchmark's CPU-baseline leg use this file.
 * It shares no code with the HIP library and is never a fallback for it.
 *
 * Reading of the paper taken here (byte-level; the paper's sets are token sets,
 * the two coincide when every token is a single symbol):
 *   - Alphabet: bytes 0..255 and EOS = 256.
 *   - Write(b0 b1 ...) is a chain of one-byte checkpoints ("a sequence of
 *     specialised Wait operators", Mask Generation section).
 *   - Wait(allow|denies, wait, max, body): a symbol in `wait` ends the operator
 *     and is consumed; this test comes first (non-greedy matching, Limitations
 *     section; the worked example's Wait(allow={\d}, wait={\d}) means exactly
 *     one digit).  Otherwise a symbol in `allow` is consumed and the operator
 *     stays, as long as fewer than `max` such symbols were consumed.  Anything
 *     else is rejected.  body, if present, runs after the Wait.
 *   - Wait(allow, true_waits, false_waits): the boolean checkpoint that IfElse
 *     and DoWhile are built on; true/false select the branch.
 *   - IfElse: true -> if_body, false -> else_body, a None body is skipped.
 *   - DoWhile: body, then condition; true -> body again, false -> leave.
 *   - A token is allowed from a state iff feeding its bytes one at a time never
 *     hits a rejection; the state after the last byte is the request's next
 *     state.  Mask bit t of word t>>5 is bit (t & 31), least significant first.
 *
 * Conventions that are not facts of the paper (numbering of leaf states, what a
 * finished request does next, bit order) are "parity unpinned": the tests pin
 * them only by self-consistency with the documented convention.
 *
 * Leaf numbering: id 0 is FINAL, 0xFFFFFFFF is ERROR.  Within a template ids
 * are consecutive in pre-order (Sequence children in order; a Wait, then its
 * body; IfElse: condition, if_body, else_body; DoWhile: body, then condition),
 * one id per Write byte, followed by one END id; template k starts where k-1
 * ended.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <stdarg.h>

#define WGO_EOS 256
#define WGO_SID_FINAL 0u
#define WGO_SID_ERROR 0xFFFFFFFFu
#define WGO_FLAG_EOS_RESTART 1u

typedef struct { uint64_t w[5]; } SymSet;             /* 257 symbols */

static void set_add(SymSet *s, int x) { s->w[x >> 6] |= 1ull << (x & 63); }
static int  set_has(const SymSet *s, int x) { return (int)((s->w[x >> 6] >> (x & 63)) & 1ull); }

typedef enum { N_SEQ, N_WRITE, N_WAIT, N_COND, N_IFELSE, N_DOWHILE } NodeKind;

typedef struct Node {
    NodeKind kind;
    struct Node **kids; int nkids;                    /* N_SEQ */
    uint8_t *bytes; size_t nbytes;                    /* N_WRITE */
    SymSet allow, wait, twait, fwait;                 /* N_WAIT, N_COND */
    int64_t max;                                      /* N_WAIT, -1 = unbounded */
    struct Node *body;                                /* N_WAIT, N_DOWHILE */
    struct Node *cond, *if_body, *else_body;          /* N_IFELSE (cond also N_DOWHILE) */
    uint32_t sid;                                     /* first leaf id of this node */
} Node;

typedef enum { L_FINAL = 0, L_LIT = 1, L_WAIT = 2, L_COND = 3, L_END = 4 } LeafKind;

typedef struct {
    LeafKind kind;
    uint8_t byte;
    SymSet allow, wait, twait, fwait;
    int64_t max;
    uint32_t next, tnext, fnext;
    uint32_t tmpl;
} Leaf;

typedef struct {
    Leaf *leaf; uint32_t nleaf;
    uint32_t *start; uint32_t *end; uint32_t ntmpl;
    uint32_t flags;
} wgo_handle;

typedef struct {                                      /* runtime snippet arguments */
    uint32_t n;
    const char *const *names;
    const uint8_t *const *data;
    const uint64_t *lens;
} wgo_args;

/* ------------------------------------------------------------------ parser */

typedef struct {
    const char *s; size_t i, n;
    const wgo_args *args;
    char *err; size_t errlen; int failed;
    void **allocs; size_t nalloc, capalloc;
} Parser;

static void fail(Parser *p, const char *fmt, ...)
{
    if (p->failed) return;
    p->failed = 1;
    if (p->err && p->errlen) {
        va_list ap; va_start(ap, fmt);
        int k = snprintf(p->err, p->errlen, "at offset %zu: ", p->i);
        if (k < 0) k = 0;
        if ((size_t)k < p->errlen) vsnprintf(p->err + k, p->errlen - (size_t)k, fmt, ap);
        va_end(ap);
    }
}

static void *palloc(Parser *p, size_t bytes)
{
    void *m = calloc(1, bytes ? bytes : 1);
    if (p->nalloc == p->capalloc) {
        p->capalloc = p->capalloc ? 2 * p->capalloc : 64;
        p->allocs = (void **)realloc(p->allocs, p->capalloc * sizeof(void *));
    }
    p->allocs[p->nalloc++] = m;
    return m;
}

static void skip_ws(Parser *p)
{
    while (p->i < p->n) {
        char c = p->s[p->i];
        if (c == ' ' || c == '\t' || c == '\n' || c == '\r') p->i++; else break;
    }
}

static int peek(Parser *p) { skip_ws(p); return p->i < p->n ? (unsigned char)p->s[p->i] : -1; }

static void expect(Parser *p, char c)
{
    if (p->failed) return;
    if (peek(p) != (unsigned char)c) { fail(p, "expected '%c'", c); return; }
    p->i++;
}

static int is_ident_char(int c, int first)
{
    if ((c >= 'A' && c <= 'Z') || (c >= 'a' && c <= 'z') || c == '_') return 1;
    return !first && c >= '0' && c <= '9';
}

static size_t ident(Parser *p, char *out, size_t cap)
{
    skip_ws(p);
    size_t k = 0;
    while (p->i < p->n && is_ident_char((unsigned char)p->s[p->i], k == 0)) {
        if (k + 1 < cap) out[k] = p->s[p->i];
        k++; p->i++;
    }
    out[k < cap ? k : cap - 1] = 0;
    if (k == 0) fail(p, "expected an identifier");
    return k;
}

static int lookup_arg(Parser *p, const char *name, const uint8_t **data, uint64_t *len)
{
    if (p->args)
        for (uint32_t a = 0; a < p->args->n; a++)
            if (strcmp(p->args->names[a], name) == 0) {
                *data = p->args->data[a]; *len = p->args->lens[a];
                return 1;
            }
    fail(p, "unbound argument $%s", name);
    return 0;
}

static int hexval(int c)
{
    if (c >= '0' && c <= '9') return c - '0';
    if (c >= 'a' && c <= 'f') return c - 'a' + 10;
    if (c >= 'A' && c <= 'F') return c - 'A' + 10;
    return -1;
}

/* After a backslash.  Returns a byte value, or -2 after adding a class to *cls. */
static int escape(Parser *p, SymSet *cls)
{
    if (p->i >= p->n) { fail(p, "dangling backslash"); return 0; }
    int c = (unsigned char)p->s[p->i++];
    switch (c) {
    case 'n': return '\n';
    case 't': return '\t';
    case 'r': return '\r';
    case 'x': {
        if (p->i + 1 >= p->n) { fail(p, "short \\x escape"); return 0; }
        int h = hexval((unsigned char)p->s[p->i]), l = hexval((unsigned char)p->s[p->i + 1]);
        if (h < 0 || l < 0) { fail(p, "bad \\x escape"); return 0; }
        p->i += 2;
        return h * 16 + l;
    }
    case 'd': case 'w': case 's':
        if (!cls) return c;                           /* in a string these are plain letters */
        if (c == 'd' || c == 'w') for (int x = '0'; x <= '9'; x++) set_add(cls, x);
        if (c == 'w') {
            for (int x = 'a'; x <= 'z'; x++) set_add(cls, x);
            for (int x = 'A'; x <= 'Z'; x++) set_add(cls, x);
            set_add(cls, '_');
        }
        if (c == 's') { set_add(cls, ' '); set_add(cls, '\t'); set_add(cls, '\n');
                        set_add(cls, '\r'); set_add(cls, '\f'); set_add(cls, '\v'); }
        return -2;
    default: return c;
    }
}

static void parse_bracket(Parser *p, SymSet *out)     /* after '[' */
{
    for (;;) {
        if (p->i >= p->n) { fail(p, "unterminated [class]"); return; }
        int c = (unsigned char)p->s[p->i++];
        if (c == ']') return;
        int lo = c;
        if (c == '\\') { lo = escape(p, out); if (p->failed) return; if (lo == -2) continue; }
        if (p->i + 1 < p->n && p->s[p->i] == '-' && p->s[p->i + 1] != ']') {
            p->i++;
            int hi = (unsigned char)p->s[p->i++];
            if (hi == '\\') { hi = escape(p, NULL); if (p->failed) return; }
            if (hi < lo) { fail(p, "reversed range"); return; }
            for (int x = lo; x <= hi; x++) set_add(out, x);
        } else set_add(out, lo);
    }
}

static void parse_set(Parser *p, SymSet *out)
{
    memset(out, 0, sizeof *out);
    int c = peek(p);
    if (c == '$') {
        char name[128]; p->i++; ident(p, name, sizeof name);
        const uint8_t *d; uint64_t len;
        if (p->failed || !lookup_arg(p, name, &d, &len)) return;
        for (uint64_t k = 0; k < len; k++) set_add(out, d[k]);
        return;
    }
    expect(p, '{');
    for (;;) {
        if (p->failed) return;
        c = peek(p);
        if (c < 0) { fail(p, "unterminated set"); return; }
        if (c == '}') { p->i++; return; }
        if (c == ',') { p->i++; continue; }
        if (c == '<' && p->n - p->i >= 5 && memcmp(p->s + p->i, "<eos>", 5) == 0) {
            p->i += 5; set_add(out, WGO_EOS);
        } else if (c == '\\') {
            p->i++;
            int v = escape(p, out);
            if (!p->failed && v >= 0) set_add(out, v);
        } else if (c == '[') {
            p->i++; parse_bracket(p, out);
        } else if (c == '$') {
            char name[128]; p->i++; ident(p, name, sizeof name);
            const uint8_t *d; uint64_t len;
            if (p->failed || !lookup_arg(p, name, &d, &len)) return;
            for (uint64_t k = 0; k < len; k++) set_add(out, d[k]);
        } else {
            p->i++; set_add(out, c);
        }
    }
}

static void parse_string(Parser *p, uint8_t **out, size_t *outlen)
{
    expect(p, '"');
    if (p->failed) return;
    uint8_t *buf = (uint8_t *)palloc(p, p->n - p->i + 1);
    size_t k = 0;
    for (;;) {
        if (p->i >= p->n) { fail(p, "unterminated string"); return; }
        int c = (unsigned char)p->s[p->i++];
        if (c == '"') break;
        if (c == '\\') { c = escape(p, NULL); if (p->failed) return; }
        buf[k++] = (uint8_t)c;
    }
    *out = buf; *outlen = k;
}

static Node *parse_op(Parser *p, int *is_none);

static Node *parse_body(Parser *p)                    /* an operator or None */
{
    int none = 0;
    Node *n = parse_op(p, &none);
    if (n && n->kind == N_COND) { fail(p, "a condition Wait is only valid inside IfElse / DoWhile"); return NULL; }
    return none ? NULL : n;
}

static Node *new_node(Parser *p, NodeKind k)
{
    Node *n = (Node *)palloc(p, sizeof(Node));
    n->kind = k; n->max = -1;
    return n;
}

static Node *parse_wait(Parser *p)
{
    SymSet allow, denies, wait, tw, fw;
    int has_allow = 0, has_denies = 0, has_wait = 0, has_t = 0, has_f = 0, has_body = 0;
    int64_t max = -1; Node *body = NULL;
    memset(&allow, 0, sizeof allow);
    for (;;) {
        if (p->failed) return NULL;
        int c = peek(p);
        if (c == ')') { p->i++; break; }
        if (c == ',') { p->i++; continue; }
        char key[32]; ident(p, key, sizeof key); expect(p, '=');
        if (p->failed) return NULL;
        if (!strcmp(key, "allow")) { parse_set(p, &allow); has_allow = 1; }
        else if (!strcmp(key, "denies")) { parse_set(p, &denies); has_denies = 1; }
        else if (!strcmp(key, "wait")) { parse_set(p, &wait); has_wait = 1; }
        else if (!strcmp(key, "true_waits")) { parse_set(p, &tw); has_t = 1; }
        else if (!strcmp(key, "false_waits")) { parse_set(p, &fw); has_f = 1; }
        else if (!strcmp(key, "body")) { body = parse_body(p); has_body = 1; }
        else if (!strcmp(key, "max")) {
            skip_ws(p);
            int64_t v = 0; int digits = 0;
            while (p->i < p->n && p->s[p->i] >= '0' && p->s[p->i] <= '9') {
                v = v * 10 + (p->s[p->i++] - '0'); digits++;
                if (v > 0x7FFFFFFF) { fail(p, "max too large"); return NULL; }
            }
            if (!digits) { fail(p, "max needs a number"); return NULL; }
            max = v;
        } else { fail(p, "unknown Wait argument '%s'", key); return NULL; }
    }
    if (has_allow && has_denies) { fail(p, "give allow or denies, not both"); return NULL; }
    if (has_denies) {                                 /* denies = D  means  allow = bytes \ D */
        memset(&allow, 0, sizeof allow);
        for (int x = 0; x < 256; x++) if (!set_has(&denies, x)) set_add(&allow, x);
        if (set_has(&denies, WGO_EOS)) { fail(p, "<eos> cannot be denied"); return NULL; }
    }
    Node *n;
    if (has_t || has_f) {
        if (!has_t || !has_f || has_wait || has_body || max >= 0) {
            fail(p, "a condition Wait takes allow, true_waits and false_waits only"); return NULL;
        }
        for (int x = 0; x <= WGO_EOS; x++)
            if (set_has(&tw, x) && set_has(&fw, x)) {
                fail(p, "true_waits and false_waits overlap"); return NULL;
            }
        n = new_node(p, N_COND);
        n->twait = tw; n->fwait = fw;
        if (set_has(&allow, WGO_EOS) && !set_has(&tw, WGO_EOS) && !set_has(&fw, WGO_EOS)) {
            fail(p, "<eos> in allow but in no wait set"); return NULL;
        }
    } else {
        if (!has_wait) { fail(p, "Wait needs wait="); return NULL; }
        n = new_node(p, N_WAIT);
        n->wait = wait; n->max = max; n->body = body;
        if (set_has(&allow, WGO_EOS) && !set_has(&wait, WGO_EOS)) {
            fail(p, "<eos> in allow but not in wait"); return NULL;
        }
    }
    n->allow = allow;
    return n;
}

static Node *parse_op(Parser *p, int *is_none)
{
    char name[32];
    if (is_none) *is_none = 0;
    ident(p, name, sizeof name);
    if (p->failed) return NULL;
    if (!strcmp(name, "None")) {
        if (!is_none) { fail(p, "None is only valid as a body"); return NULL; }
        *is_none = 1; return NULL;
    }
    expect(p, '(');
    if (p->failed) return NULL;
    if (!strcmp(name, "Sequence")) {
        Node *n = new_node(p, N_SEQ);
        int cap = 0;
        for (;;) {
            int c = peek(p);
            if (c == ')') { p->i++; break; }
            if (c == ',') { p->i++; continue; }
            Node *k = parse_op(p, NULL);
            if (p->failed) return NULL;
            if (k->kind == N_COND) { fail(p, "a condition Wait is only valid inside IfElse / DoWhile"); return NULL; }
            if (n->nkids == cap) {
                cap = cap ? 2 * cap : 8;
                Node **nk = (Node **)palloc(p, (size_t)cap * sizeof(Node *));
                if (n->nkids) memcpy(nk, n->kids, (size_t)n->nkids * sizeof(Node *));
                n->kids = nk;
            }
            n->kids[n->nkids++] = k;
        }
        return n;
    }
    if (!strcmp(name, "Write")) {
        Node *n = new_node(p, N_WRITE);
        if (peek(p) == '$') {
            char an[128]; p->i++; ident(p, an, sizeof an);
            const uint8_t *d; uint64_t len;
            if (p->failed || !lookup_arg(p, an, &d, &len)) return NULL;
            n->bytes = (uint8_t *)palloc(p, len);
            memcpy(n->bytes, d, len); n->nbytes = len;
        } else parse_string(p, &n->bytes, &n->nbytes);
        expect(p, ')');
        return p->failed ? NULL : n;
    }
    if (!strcmp(name, "Wait")) return parse_wait(p);
    if (!strcmp(name, "IfElse") || !strcmp(name, "DoWhile")) {
        int is_if = name[0] == 'I';
        Node *n = new_node(p, is_if ? N_IFELSE : N_DOWHILE);
        int got_cond = 0;
        for (;;) {
            if (p->failed) return NULL;
            int c = peek(p);
            if (c == ')') { p->i++; break; }
            if (c == ',') { p->i++; continue; }
            char key[32]; ident(p, key, sizeof key); expect(p, '=');
            if (p->failed) return NULL;
            if (!strcmp(key, "condition")) { n->cond = parse_op(p, NULL); got_cond = 1; }
            else if (is_if && !strcmp(key, "if_body")) n->if_body = parse_body(p);
            else if (is_if && !strcmp(key, "else_body")) n->else_body = parse_body(p);
            else if (!is_if && !strcmp(key, "body")) n->body = parse_body(p);
            else { fail(p, "unknown %s argument '%s'", name, key); return NULL; }
        }
        if (!got_cond || !n->cond || n->cond->kind != N_COND) {
            fail(p, "%s needs condition=Wait(allow, true_waits, false_waits)", name); return NULL;
        }
        return n;
    }
    fail(p, "unknown operator '%s'", name);
    return NULL;
}

/* ------------------------------------------- numbering and continuations */

static int is_empty(const Node *n)                    /* occupies no leaf state */
{
    if (!n) return 1;
    if (n->kind == N_WRITE) return n->nbytes == 0;
    if (n->kind == N_SEQ) { for (int i = 0; i < n->nkids; i++) if (!is_empty(n->kids[i])) return 0; return 1; }
    return 0;
}

static void number(Node *n, uint32_t *next_id)
{
    if (!n) return;
    n->sid = *next_id;
    switch (n->kind) {
    case N_WRITE: *next_id += (uint32_t)n->nbytes; break;
    case N_WAIT:  *next_id += 1; number(n->body, next_id); break;
    case N_COND:  *next_id += 1; break;
    case N_SEQ:   for (int i = 0; i < n->nkids; i++) number(n->kids[i], next_id); break;
    case N_IFELSE: number(n->cond, next_id); number(n->if_body, next_id); number(n->else_body, next_id); break;
    case N_DOWHILE: number(n->body, next_id); number(n->cond, next_id); break;
    }
}

/* First leaf executed when control enters n; `cont` if n occupies no state. */
static uint32_t first_of(const Node *n, uint32_t cont)
{
    if (is_empty(n)) return cont;
    switch (n->kind) {
    case N_WRITE: case N_WAIT: case N_COND: return n->sid;
    case N_IFELSE: return n->cond->sid;
    case N_DOWHILE: return is_empty(n->body) ? n->cond->sid : first_of(n->body, n->cond->sid);
    case N_SEQ:
        for (int i = 0; i < n->nkids; i++) if (!is_empty(n->kids[i])) return first_of(n->kids[i], cont);
        return cont;
    }
    return cont;
}

/* Fill the leaf table for n, given the leaf `cont` that runs after n. */
static void link_node(wgo_handle *h, Node *n, uint32_t cont, uint32_t tmpl)
{
    if (!n) return;
    switch (n->kind) {
    case N_WRITE:
        for (size_t i = 0; i < n->nbytes; i++) {
            Leaf *l = &h->leaf[n->sid + i];
            l->kind = L_LIT; l->byte = n->bytes[i]; l->tmpl = tmpl;
            l->next = (i + 1 < n->nbytes) ? n->sid + (uint32_t)i + 1 : cont;
        }
        break;
    case N_WAIT: {
        Leaf *l = &h->leaf[n->sid];
        l->kind = L_WAIT; l->allow = n->allow; l->wait = n->wait; l->max = n->max; l->tmpl = tmpl;
        l->next = first_of(n->body, cont);
        link_node(h, n->body, cont, tmpl);
        break;
    }
    case N_COND: break;                               /* linked by its IfElse / DoWhile */
    case N_SEQ:
        for (int i = 0; i < n->nkids; i++) {
            uint32_t after = cont;                    /* first leaf of what follows child i */
            for (int j = n->nkids - 1; j > i; j--) after = first_of(n->kids[j], after);
            link_node(h, n->kids[i], after, tmpl);
        }
        break;
    case N_IFELSE: {
        Leaf *l = &h->leaf[n->cond->sid];
        l->kind = L_COND; l->allow = n->cond->allow; l->twait = n->cond->twait;
        l->fwait = n->cond->fwait; l->max = -1; l->tmpl = tmpl;
        l->tnext = first_of(n->if_body, cont);
        l->fnext = first_of(n->else_body, cont);
        link_node(h, n->if_body, cont, tmpl);
        link_node(h, n->else_body, cont, tmpl);
        break;
    }
    case N_DOWHILE: {
        Leaf *l = &h->leaf[n->cond->sid];
        l->kind = L_COND; l->allow = n->cond->allow; l->twait = n->cond->twait;
        l->fwait = n->cond->fwait; l->max = -1; l->tmpl = tmpl;
        l->tnext = first_of(n->body, n->cond->sid);   /* true: run the body again */
        l->fnext = cont;                              /* false: leave the loop */
        link_node(h, n->body, n->cond->sid, tmpl);
        break;
    }
    }
}

/* ---------------------------------------------------------------- public */

void wgo_destroy(wgo_handle *h)
{
    if (!h) return;
    free(h->leaf); free(h->start); free(h->end); free(h);
}

static void seterr(char *err, size_t errlen, const char *msg, uint32_t t)
{
    if (err && errlen) snprintf(err, errlen, "template %u: %s", t, msg);
}

/* texts[i] is compiled with args[i] (args may be NULL when no template has holes). */
wgo_handle *wgo_compile(const char *const *texts, const wgo_args *args, uint32_t n,
                        uint32_t flags, char *err, uint64_t errlen)
{
    if (err && errlen) err[0] = 0;
    Node **roots = (Node **)calloc(n ? n : 1, sizeof(Node *));
    Parser *ps = (Parser *)calloc(n ? n : 1, sizeof(Parser));
    wgo_handle *h = (wgo_handle *)calloc(1, sizeof *h);
    h->flags = flags; h->ntmpl = n;
    h->start = (uint32_t *)calloc(n ? n : 1, sizeof(uint32_t));
    h->end = (uint32_t *)calloc(n ? n : 1, sizeof(uint32_t));
    int ok = 1;
    uint32_t next_id = 1;                             /* 0 is FINAL */
    for (uint32_t t = 0; t < n && ok; t++) {
        Parser *p = &ps[t];
        p->s = texts[t]; p->n = strlen(texts[t]); p->args = args ? &args[t] : NULL;
        char msg[256]; msg[0] = 0;
        p->err = msg; p->errlen = sizeof msg;
        roots[t] = parse_op(p, NULL);
        if (!p->failed && peek(p) >= 0) fail(p, "trailing text after the operator");
        if (!p->failed && roots[t]->kind == N_COND) fail(p, "a condition Wait is only valid inside IfElse / DoWhile");
        if (p->failed) { seterr(err, errlen, msg, t); ok = 0; break; }
        number(roots[t], &next_id);
        h->end[t] = next_id++;
        h->start[t] = first_of(roots[t], h->end[t]);
    }
    if (ok) {
        h->nleaf = next_id;
        h->leaf = (Leaf *)calloc(next_id, sizeof(Leaf));
        h->leaf[0].kind = L_FINAL;
        for (uint32_t t = 0; t < n; t++) {
            h->leaf[h->end[t]].kind = L_END; h->leaf[h->end[t]].tmpl = t;
            link_node(h, roots[t], h->end[t], t);
        }
        /* an exit taken on <eos> finishes the output: nothing may follow it */
        for (uint32_t s = 1; s < h->nleaf && ok; s++) {
            Leaf *l = &h->leaf[s];
            uint32_t e = h->end[l->tmpl];
            if ((l->kind == L_WAIT && set_has(&l->wait, WGO_EOS) && l->next != e) ||
                (l->kind == L_COND && set_has(&l->twait, WGO_EOS) && l->tnext != e) ||
                (l->kind == L_COND && set_has(&l->fwait, WGO_EOS) && l->fnext != e)) {
                seterr(err, errlen, "operators follow an exit taken on <eos>", l->tmpl); ok = 0;
            }
        }
    }
    for (uint32_t t = 0; t < n; t++) {
        for (size_t k = 0; k < ps[t].nalloc; k++) free(ps[t].allocs[k]);
        free(ps[t].allocs);
    }
    free(ps); free(roots);
    if (!ok) { wgo_destroy(h); return NULL; }
    return h;
}

uint32_t wgo_num_states(const wgo_handle *h) { return h->nleaf; }
uint32_t wgo_start_state(const wgo_handle *h, uint32_t t) { return h->start[t]; }
uint32_t wgo_end_state(const wgo_handle *h, uint32_t t) { return h->end[t]; }

/* For tests of the numbering: out = {kind, byte, max (or -1), next, tnext, fnext, tmpl}. */
int wgo_describe(const wgo_handle *h, uint32_t sid, int64_t out[7])
{
    if (sid >= h->nleaf) return -1;
    const Leaf *l = &h->leaf[sid];
    out[0] = l->kind; out[1] = l->byte; out[2] = l->max;
    out[3] = l->next; out[4] = l->tnext; out[5] = l->fnext; out[6] = l->tmpl;
    return 0;
}

static uint32_t after_eos(const wgo_handle *h, uint32_t tmpl)
{
    return (h->flags & WGO_FLAG_EOS_RESTART) ? h->start[tmpl] : WGO_SID_FINAL;
}

/* One transition.  Returns 1 and writes the new state, or 0 if x is rejected.
 * aux counts the allow-symbols consumed so far inside a bounded Wait, else 0. */
int wgo_step(const wgo_handle *h, uint32_t sid, uint32_t aux, int x, uint32_t *nsid, uint32_t *naux)
{
    if (sid == WGO_SID_ERROR || sid >= h->nleaf || x < 0 || x > WGO_EOS) return 0;
    const Leaf *l = &h->leaf[sid];
    *naux = 0;
    switch (l->kind) {
    case L_FINAL:
        if (x != WGO_EOS) return 0;
        *nsid = WGO_SID_FINAL; return 1;
    case L_END:
        if (x != WGO_EOS) return 0;
        *nsid = after_eos(h, l->tmpl); return 1;
    case L_LIT:
        if (x != l->byte) return 0;
        *nsid = l->next; return 1;
    case L_WAIT:
        if (set_has(&l->wait, x)) {                   /* terminator first: non-greedy */
            *nsid = (x == WGO_EOS) ? after_eos(h, l->tmpl) : l->next; return 1;
        }
        if (set_has(&l->allow, x) && (l->max < 0 || (int64_t)aux < l->max)) {
            *nsid = sid; *naux = l->max < 0 ? 0 : aux + 1; return 1;
        }
        return 0;
    case L_COND:
        if (set_has(&l->twait, x)) { *nsid = (x == WGO_EOS) ? after_eos(h, l->tmpl) : l->tnext; return 1; }
        if (set_has(&l->fwait, x)) { *nsid = (x == WGO_EOS) ? after_eos(h, l->tmpl) : l->fnext; return 1; }
        if (set_has(&l->allow, x)) { *nsid = sid; return 1; }
        return 0;
    }
    return 0;
}

typedef struct {
    const uint8_t *bytes; const uint64_t *offsets; uint32_t V; int32_t eos_id;
} wgo_vocab;

/* Feed token t symbol by symbol.  Returns 1 and the resulting state if every
 * symbol is accepted, else 0.  The EOS token is the one-symbol string [EOS]; any
 * other token without bytes is never allowed. */
int wgo_walk_token(const wgo_handle *h, const wgo_vocab *v, uint32_t sid, uint32_t aux,
                   int64_t t, uint32_t *nsid, uint32_t *naux)
{
    if (t < 0 || t >= (int64_t)v->V) return 0;
    if (v->eos_id >= 0 && t == v->eos_id) return wgo_step(h, sid, aux, WGO_EOS, nsid, naux);
    uint64_t lo = v->offsets[t], hi = v->offsets[t + 1];
    if (hi <= lo) return 0;
    for (uint64_t i = lo; i < hi; i++) {
        if (!wgo_step(h, sid, aux, v->bytes[i], &sid, &aux)) return 0;
    }
    *nsid = sid; *naux = aux;
    return 1;
}

/* One mask row: W = ceil(V/32) little-endian words, bit (t & 31) of word t >> 5. */
void wgo_mask_row(const wgo_handle *h, const wgo_vocab *v, uint32_t sid, uint32_t aux, uint32_t *row)
{
    uint32_t W = (v->V + 31u) / 32u;
    memset(row, 0, (size_t)W * 4);
    for (uint32_t t = 0; t < v->V; t++) {
        uint32_t s2, a2;
        if (wgo_walk_token(h, v, sid, aux, t, &s2, &a2)) row[t >> 5] |= 1u << (t & 31);
    }
}

void wgo_fill_masks(const wgo_handle *h, const wgo_vocab *v, const uint32_t *states /*[B][2]*/,
                    uint32_t B, uint32_t *bitmask /*[B][W]*/)
{
    uint32_t W = (v->V + 31u) / 32u;
    for (uint32_t b = 0; b < B; b++)
        wgo_mask_row(h, v, states[2 * b], states[2 * b + 1], bitmask + (size_t)b * W);
}

/* Disallowed logits take the bit pattern of -inf; allowed ones are untouched.
 * dtype 0 = float32, 1 = bfloat16.  row_stride is in elements. */
void wgo_apply_mask(void *logits, int dtype, uint32_t B, uint32_t V, int64_t row_stride,
                    const uint32_t *bitmask)
{
    uint32_t W = (V + 31u) / 32u;
    for (uint32_t b = 0; b < B; b++)
        for (uint32_t t = 0; t < V; t++) {
            int bit = (bitmask[(size_t)b * W + (t >> 5)] >> (t & 31)) & 1u;
            if (bit) continue;
            if (dtype == 0) ((uint32_t *)logits)[(int64_t)b * row_stride + t] = 0xFF800000u;
            else            ((uint16_t *)logits)[(int64_t)b * row_stride + t] = 0xFF80u;
        }
}

/* Greedy choice over the allowed tokens, logits untouched: tokens_out[b] = the allowed token
 * with the largest logit; a NaN ranks below every number (also below -inf), equal values
 * (-0.0 equals +0.0) keep the lowest token id; -1 if the row allows nothing. */
static double elem_value(const void *logits, int dtype, int64_t idx)
{
    if (dtype == 0) { float f; memcpy(&f, (const char *)logits + 4 * idx, 4); return (double)f; }
    uint32_t u = (uint32_t)((const uint16_t *)logits)[idx] << 16;       /* bfloat16 -> float32, exact */
    float f; memcpy(&f, &u, 4);
    return (double)f;
}

void wgo_masked_argmax(const void *logits, int dtype, uint32_t B, uint32_t V, int64_t row_stride,
                       const uint32_t *bitmask, int32_t *tokens_out)
{
    uint32_t W = (V + 31u) / 32u;
    for (uint32_t b = 0; b < B; b++) {
        int64_t best = -1; double best_v = 0.0; int best_nan = 1;
        for (uint32_t t = 0; t < V; t++) {
            if (!((bitmask[(size_t)b * W + (t >> 5)] >> (t & 31)) & 1u)) continue;
            double v = elem_value(logits, dtype, (int64_t)b * row_stride + t);
            int is_nan = v != v;
            int better;
            if (best < 0) better = 1;
            else if (best_nan) better = !is_nan;                  /* any number beats a NaN */
            else better = !is_nan && v > best_v;
            if (better) { best = t; best_v = v; best_nan = is_nan; }
        }
        tokens_out[b] = (int32_t)best;
    }
}

/* The k best allowed tokens of every row, best first: the greedy choice above made k times,
 * each time among the allowed tokens not chosen yet (so the order is: larger logit first, equal
 * values by lower token id, NaNs after every number).  ids_out[b][r] = -1 and values_out[b][r]
 * = the bit pattern of -inf once the row's allowed tokens are used up.  values_out holds raw
 * elements of the logits' type. */
void wgo_masked_topk(const void *logits, int dtype, uint32_t B, uint32_t V, int64_t row_stride,
                     const uint32_t *bitmask, uint32_t k, int32_t *ids_out, void *values_out)
{
    uint32_t W = (V + 31u) / 32u;
    uint8_t *taken = (uint8_t *)malloc(V ? V : 1);
    for (uint32_t b = 0; b < B; b++) {
        memset(taken, 0, V);
        for (uint32_t r = 0; r < k; r++) {
            int64_t best = -1; double best_v = 0.0; int best_nan = 1;
            for (uint32_t t = 0; t < V; t++) {
                if (taken[t] || !((bitmask[(size_t)b * W + (t >> 5)] >> (t & 31)) & 1u)) continue;
                double v = elem_value(logits, dtype, (int64_t)b * row_stride + t);
                int is_nan = v != v;
                int better;
                if (best < 0) better = 1;
                else if (best_nan) better = !is_nan;
                else better = !is_nan && v > best_v;
                if (better) { best = t; best_v = v; best_nan = is_nan; }
            }
            ids_out[(size_t)b * k + r] = (int32_t)best;
            if (best >= 0) taken[best] = 1;
            if (dtype == 0)
                ((uint32_t *)values_out)[(size_t)b * k + r] =
                    best >= 0 ? ((const uint32_t *)logits)[(int64_t)b * row_stride + best] : 0xFF800000u;
            else
                ((uint16_t *)values_out)[(size_t)b * k + r] =
                    best >= 0 ? ((const uint16_t *)logits)[(int64_t)b * row_stride + best] : 0xFF80u;
        }
    }
    free(taken);
}

/* states[b] <- state after tokens[b]; a rejected or out-of-range token gives ERROR. */
void wgo_advance(const wgo_handle *h, const wgo_vocab *v, uint32_t *states /*[B][2]*/,
                 const int32_t *tokens, uint32_t B)
{
    for (uint32_t b = 0; b < B; b++) {
        uint32_t s2, a2;
        if (wgo_walk_token(h, v, states[2 * b], states[2 * b + 1], tokens[b], &s2, &a2)) {
            states[2 * b] = s2; states[2 * b + 1] = a2;
        } else { states[2 * b] = WGO_SID_ERROR; states[2 * b + 1] = 0; }
    }
}

/* --------------------------------------------------- trajectory generation
 * Runs B requests for `steps` steps: mask of the current state, pick the
 * (draw mod popcount)-th allowed token, advance.  Masks are memoised per
 * (sid, rem) with rem = min(max - aux, lmax) for a bounded Wait and 0 otherwise:
 * inside one token at most lmax symbols are consumed, so a larger remaining
 * budget cannot change a verdict.  The tests compare memoised rows with fresh
 * wgo_mask_row walks.  Only this generator memoises; wgo_mask_row never does.
 */
typedef struct MemoEnt { uint32_t sid, rem; uint32_t *row; uint64_t pop; struct MemoEnt *nxt; } MemoEnt;

static uint32_t key_rem(const wgo_handle *h, uint32_t sid, uint32_t aux, uint32_t lmax)
{
    if (sid == WGO_SID_ERROR || sid >= h->nleaf) return 0;
    const Leaf *l = &h->leaf[sid];
    if (l->kind != L_WAIT || l->max < 0) return 0;
    int64_t left = l->max - (int64_t)aux;
    if (left < 0) left = 0;
    return (uint32_t)(left < (int64_t)lmax ? left : (int64_t)lmax);
}

uint32_t wgo_key_rem(const wgo_handle *h, uint32_t sid, uint32_t aux, uint32_t lmax)
{
    return key_rem(h, sid, aux, lmax);
}

/* The bytes a request in state sid is forced to produce next: a Write is a chain of
 * checkpoints that each admit one symbol ("a sequence of specialised Wait operators", Mask
 * Generation and Global Caching), so from a state inside a Write the only walkable
 * continuation is the rest of that Write -- and of the Writes that follow it directly -- up to
 * the next state that is not a Write byte (a Wait, a condition, the end of the template).
 * Writes at most cap bytes to out, returns how many; *end_sid is the state after them (sid
 * itself when it is not a Write byte, when cap is 0, or when sid is no state at all). */
uint32_t wgo_forced_bytes(const wgo_handle *h, uint32_t sid, uint8_t *out, uint32_t cap, uint32_t *end_sid)
{
    uint32_t n = 0;
    while (n < cap && sid != WGO_SID_ERROR && sid < h->nleaf && h->leaf[sid].kind == L_LIT) {
        out[n++] = h->leaf[sid].byte;
        sid = h->leaf[sid].next;
    }
    *end_sid = sid;
    return n;
}

/* Index of the k-th (0-based) set bit of the row, or -1. */
int64_t wgo_select_bit(const uint32_t *row, uint32_t W, uint64_t k)
{
    for (uint32_t w = 0; w < W; w++) {
        uint32_t x = row[w];
        uint64_t c = (uint64_t)__builtin_popcount(x);
        if (k >= c) { k -= c; continue; }
        for (int b = 0; b < 32; b++)
            if ((x >> b) & 1u) { if (k == 0) return (int64_t)w * 32 + b; k--; }
    }
    return -1;
}

/* Returns the number of distinct memoised masks, or -1 on allocation failure.
 * tokens_out [steps][B], states_out [steps][B][2] (state after each step),
 * states [B][2] is updated in place to the final states. */
int64_t wgo_trajectory(const wgo_handle *h, const wgo_vocab *v, uint32_t lmax,
                       uint32_t *states, uint32_t B, uint32_t steps,
                       const uint64_t *draws /*[steps][B]*/,
                       int32_t *tokens_out, uint32_t *states_out)
{
    uint32_t W = (v->V + 31u) / 32u;
    uint32_t nb = 1u << 16;
    MemoEnt **bucket = (MemoEnt **)calloc(nb, sizeof(MemoEnt *));
    int64_t nmemo = 0;
    if (!bucket) return -1;
    for (uint32_t k = 0; k < steps; k++) {
        for (uint32_t b = 0; b < B; b++) {
            uint32_t sid = states[2 * b], aux = states[2 * b + 1];
            uint32_t rem = key_rem(h, sid, aux, lmax);
            uint32_t hsh = (sid * 2654435761u ^ rem * 40503u) & (nb - 1);
            MemoEnt *e = bucket[hsh];
            while (e && !(e->sid == sid && e->rem == rem)) e = e->nxt;
            if (!e) {
                e = (MemoEnt *)malloc(sizeof *e);
                uint32_t *row = (uint32_t *)malloc((size_t)W * 4);
                if (!e || !row) return -1;
                wgo_mask_row(h, v, sid, aux, row);
                uint64_t pop = 0;
                for (uint32_t w = 0; w < W; w++) pop += (uint64_t)__builtin_popcount(row[w]);
                e->sid = sid; e->rem = rem; e->row = row; e->pop = pop; e->nxt = bucket[hsh];
                bucket[hsh] = e; nmemo++;
            }
            int64_t tok = e->pop ? wgo_select_bit(e->row, W, draws[(size_t)k * B + b] % e->pop) : -1;
            int32_t tk = (int32_t)tok;
            wgo_advance(h, v, states + 2 * b, &tk, 1);
            tokens_out[(size_t)k * B + b] = tk;
            states_out[((size_t)k * B + b) * 2] = states[2 * b];
            states_out[((size_t)k * B + b) * 2 + 1] = states[2 * b + 1];
        }
    }
    for (uint32_t i = 0; i < nb; i++)
        for (MemoEnt *e = bucket[i]; e;) { MemoEnt *n = e->nxt; free(e->row); free(e); e = n; }
    free(bucket);
    return nmemo;
}
