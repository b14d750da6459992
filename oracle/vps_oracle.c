/* CPU oracle for the VPS state transition: see vps_oracle.h.  TEST INFRASTRUCTURE ONLY.
 *
 * Everything here works one element at a time.  A configuration is two maps:
 *   coord  : (rank, buffer, local offset)      -> (tensor, global coordinate) or padding
 *   owners : (kind, tensor, global coordinate) -> all (rank, buffer, local offset)
 * (DynaTrain Section 4.1: F_P projects the global space onto a rank; Section 4.2.2: flat
 * ZeRO offsets are positions in the flattened parameter order of the data-parallel group.)
 *
 * Conventions where the paper is silent (each is a declared reading of this repository):
 *   rank order      g = tp + TP*(ddp + DDP*pp); the expert group sees the same ranks as
 *                   g = etp + ETP*(ep + EP*(edp + EDP*pp)) with ETP*EP*EDP = TP*DDP.
 *                   ep_placement 0: EP and expert-DP form a grid beside TP (ETP = TP, EDP = DP,
 *                   DDP = EP*DP, world = TP*PP*DP*EP); ep_placement 1: EP is carved out of the
 *                   TP x DP ranks of a stage (ETP = 1, DDP = DP, EDP = TP*DP/EP, world =
 *                   TP*PP*DP), as in the MoE rows of the paper's hybrid reconfiguration table
 *   pipeline split  stage p owns layers [floor(p*L/PP), floor((p+1)*L/PP)); embedding on the
 *                   first stage, final norm and output layer on the last, untied
 *   flat buffer     per rank one dense and one expert group; local shards concatenated in
 *                   tensor-id order, no gaps, tail padded to a multiple of 8*D elements;
 *                   DP-group member r owns [r*Lpad/D, (r+1)*Lpad/D) of the fp32 kinds
 */
#include "vps_oracle.h"

#include <limits.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#include "../datagen/pattern.h"

enum { PERM_NONE = 0, PERM_GATE_UP = 1, PERM_DOWN = 2 };

typedef struct {
    int32_t shape[4];
    int32_t tp_axis;  /* -1 replicated over TP */
    int32_t group;    /* 0 dense, 1 expert */
    int32_t blk_axis; /* axis that holds the fused Q/K/V slot index, or -1 */
    int32_t perm;     /* which transposed storage applies when expert_layout == 1 */
    int32_t layer;    /* -1 before the first layer, L after the last */
    int32_t expert;   /* -1 or expert id */
    /* derived per configuration */
    int32_t cls;        /* flat-buffer class (which ranks' buffer this tensor lives in) */
    uint64_t start;     /* offset of the local shard in the (unsharded) flat buffer */
    uint64_t shard_len; /* elements of one local shard */
} tensor_t;

typedef struct {
    int32_t n;
    int32_t* tid;    /* tensors of this class in flat order */
    uint64_t* start; /* n+1 prefix offsets */
    uint64_t len;    /* unpadded flat length L */
    uint64_t padded; /* Lpad */
} class_t;

struct orc_config {
    orc_model m;
    orc_parallel p;
    int32_t nt;
    tensor_t* t;
    int32_t ddp;      /* dense data-parallel degree */
    int32_t etp, edp; /* tensor- and data-parallel degree of the expert group */
    int32_t q_per_g;  /* query heads per kv group */
    int32_t ncls[2];  /* classes per group: dense pp, expert pp*ep */
    class_t* cls[2];
};

/* ------------------------------------------------------------------ inventory */

static void add_tensor(orc_config* c, int* cap, int s0, int s1, int s2, int s3, int tp_axis,
                       int group, int blk_axis, int perm, int layer, int expert)
{
    if (c->nt == *cap) {
        *cap = *cap ? *cap * 2 : 64;
        c->t = (tensor_t*)realloc(c->t, sizeof(tensor_t) * (size_t)*cap);
    }
    tensor_t* t = &c->t[c->nt++];
    memset(t, 0, sizeof(*t));
    t->shape[0] = s0; t->shape[1] = s1; t->shape[2] = s2; t->shape[3] = s3;
    t->tp_axis = tp_axis; t->group = group; t->blk_axis = blk_axis; t->perm = perm;
    t->layer = layer; t->expert = expert;
}

/* Logical tensors in forward order.  Column-parallel weights [out, in] are cut on `out`,
 * row-parallel ones on `in`; norms, row-parallel biases, the router and the q/k norms are
 * replicated over TP.  Fused QKV is the 4-D tensor (kv group, slot, head_dim, hidden) whose
 * last two slots of every group are K and V; fused SwiGLU is (2, ffn, hidden). */
static void build_inventory(orc_config* c)
{
    const orc_model* m = &c->m;
    int cap = 0;
    const int h = m->hidden, d = m->head_dim, g = m->kv_heads, s = c->q_per_g + 2;
    const int qd = m->q_heads * d, L = m->layers;
    add_tensor(c, &cap, 1, 1, m->vocab, h, 2, 0, -1, PERM_NONE, -1, -1); /* word embedding */
    for (int l = 0; l < L; ++l) {
        if (m->family == ORC_FAMILY_GPT) {
            add_tensor(c, &cap, 1, 1, 1, h, -1, 0, -1, 0, l, -1);        /* ln1.w */
            add_tensor(c, &cap, 1, 1, 1, h, -1, 0, -1, 0, l, -1);        /* ln1.b */
            add_tensor(c, &cap, g, s, d, h, 0, 0, 1, 0, l, -1);          /* qkv.w */
            add_tensor(c, &cap, 1, g, s, d, 1, 0, 2, 0, l, -1);          /* qkv.b */
            add_tensor(c, &cap, 1, 1, h, qd, 3, 0, -1, 0, l, -1);        /* proj.w (row-parallel) */
            add_tensor(c, &cap, 1, 1, 1, h, -1, 0, -1, 0, l, -1);        /* proj.b */
            add_tensor(c, &cap, 1, 1, 1, h, -1, 0, -1, 0, l, -1);        /* ln2.w */
            add_tensor(c, &cap, 1, 1, 1, h, -1, 0, -1, 0, l, -1);        /* ln2.b */
            add_tensor(c, &cap, 1, 1, m->ffn, h, 2, 0, -1, 0, l, -1);    /* fc1.w */
            add_tensor(c, &cap, 1, 1, 1, m->ffn, 3, 0, -1, 0, l, -1);    /* fc1.b */
            add_tensor(c, &cap, 1, 1, h, m->ffn, 3, 0, -1, 0, l, -1);    /* fc2.w (row-parallel) */
            add_tensor(c, &cap, 1, 1, 1, h, -1, 0, -1, 0, l, -1);        /* fc2.b */
        } else {
            add_tensor(c, &cap, 1, 1, 1, h, -1, 0, -1, 0, l, -1);        /* input norm */
            add_tensor(c, &cap, g, s, d, h, 0, 0, 1, 0, l, -1);          /* qkv.w */
            if (m->family == ORC_FAMILY_MOE) {
                add_tensor(c, &cap, 1, 1, 1, d, -1, 0, -1, 0, l, -1);    /* q_norm */
                add_tensor(c, &cap, 1, 1, 1, d, -1, 0, -1, 0, l, -1);    /* k_norm */
            }
            add_tensor(c, &cap, 1, 1, h, qd, 3, 0, -1, 0, l, -1);        /* o.w (row-parallel) */
            add_tensor(c, &cap, 1, 1, 1, h, -1, 0, -1, 0, l, -1);        /* post-attention norm */
            if (m->family == ORC_FAMILY_GQA) {
                add_tensor(c, &cap, 1, 2, m->ffn, h, 2, 0, -1, 0, l, -1); /* gate_up.w */
                add_tensor(c, &cap, 1, 1, h, m->ffn, 3, 0, -1, 0, l, -1); /* down.w */
            } else {
                add_tensor(c, &cap, 1, 1, m->experts, h, -1, 0, -1, 0, l, -1); /* router.w */
                for (int e = 0; e < m->experts; ++e) {
                    add_tensor(c, &cap, 1, 2, m->expert_ffn, h, 2, 1, -1, PERM_GATE_UP, l, e);
                    add_tensor(c, &cap, 1, 1, h, m->expert_ffn, 3, 1, -1, PERM_DOWN, l, e);
                }
            }
        }
    }
    if (m->family == ORC_FAMILY_GPT) {
        add_tensor(c, &cap, 1, 1, 1, h, -1, 0, -1, 0, L, -1); /* final ln.w */
        add_tensor(c, &cap, 1, 1, 1, h, -1, 0, -1, 0, L, -1); /* final ln.b */
    } else {
        add_tensor(c, &cap, 1, 1, 1, h, -1, 0, -1, 0, L, -1); /* final norm */
    }
    add_tensor(c, &cap, 1, 1, m->vocab, h, 2, 0, -1, 0, L, -1); /* output layer */
}

/* ------------------------------------------------------------------ configuration */

static int stage_of_layer(const orc_config* c, int layer)
{
    const int L = c->m.layers, PP = c->p.pp;
    if (layer < 0) return 0;
    if (layer >= L) return PP - 1;
    for (int p = 0; p < PP; ++p) {
        long lo = ((long)p * L) / PP, hi = ((long)(p + 1) * L) / PP;
        if (layer >= lo && layer < hi) return p;
    }
    return -1;
}

static int ep_of_expert(const orc_config* c, int expert)
{
    return expert / (c->m.experts / c->p.ep);
}

static uint64_t numel4(const int32_t* s)
{
    return (uint64_t)s[0] * (uint64_t)s[1] * (uint64_t)s[2] * (uint64_t)s[3];
}

#define FAIL(...)                                              \
    do {                                                       \
        if (err && errlen > 0) snprintf(err, (size_t)errlen, __VA_ARGS__); \
        orc_config_destroy(c);                                 \
        return NULL;                                           \
    } while (0)

orc_config* orc_config_create(const orc_model* m, const orc_parallel* p, char* err, int errlen)
{
    orc_config* c = (orc_config*)calloc(1, sizeof(orc_config));
    c->m = *m;
    c->p = *p;
    if (m->family < 0 || m->family > 2) FAIL("unknown model family %d", m->family);
    if (m->layers < 1 || m->hidden < 1 || m->q_heads < 1 || m->kv_heads < 1 || m->head_dim < 1 ||
        m->vocab < 1)
        FAIL("model sizes must be positive");
    if (p->tp < 1 || p->pp < 1 || p->dp < 1 || p->ep < 1 || p->gpus_per_node < 1)
        FAIL("parallel degrees must be positive");
    if (m->q_heads % m->kv_heads) FAIL("q_heads %d not a multiple of kv_heads %d", m->q_heads, m->kv_heads);
    if (m->family == ORC_FAMILY_GPT && m->q_heads != m->kv_heads) FAIL("GPT family is multi-head: kv_heads must equal q_heads");
    if (m->family != ORC_FAMILY_MOE && m->ffn < 1) FAIL("ffn must be positive");
    if (m->family == ORC_FAMILY_MOE && (m->experts < 1 || m->expert_ffn < 1)) FAIL("MoE needs experts and expert_ffn");
    if (m->family != ORC_FAMILY_MOE && p->ep != 1) FAIL("ep > 1 needs the MoE family");
    if (m->kv_heads % p->tp) FAIL("tp %d does not divide kv groups %d", p->tp, m->kv_heads);
    if (m->vocab % p->tp) FAIL("tp %d does not divide vocab %d", p->tp, m->vocab);
    if (m->family != ORC_FAMILY_MOE && m->ffn % p->tp) FAIL("tp %d does not divide ffn %d", p->tp, m->ffn);
    if (m->family == ORC_FAMILY_MOE && p->ep_placement == 0 && m->expert_ffn % p->tp)
        FAIL("tp %d does not divide expert_ffn %d", p->tp, m->expert_ffn);
    if (m->family == ORC_FAMILY_MOE && m->experts % p->ep) FAIL("ep %d does not divide experts %d", p->ep, m->experts);
    if (p->pp > m->layers) FAIL("pp %d exceeds layers %d", p->pp, m->layers);
    if (p->zero != 0 && p->zero != 1) FAIL("zero stage must be 0 or 1");
    if (p->ep_placement != 0 && p->ep_placement != 1) FAIL("ep_placement must be 0 or 1");
    if (p->ep_placement == 0) {
        c->ddp = p->dp * p->ep; c->etp = p->tp; c->edp = p->dp;
    } else {
        if ((p->tp * p->dp) % p->ep) FAIL("ep %d does not divide tp*dp = %d", p->ep, p->tp * p->dp);
        c->ddp = p->dp; c->etp = 1; c->edp = p->tp * p->dp / p->ep;
    }
    c->q_per_g = m->q_heads / m->kv_heads;
    build_inventory(c);

    c->ncls[0] = p->pp;
    c->ncls[1] = p->pp * p->ep;
    for (int g = 0; g < 2; ++g) c->cls[g] = (class_t*)calloc((size_t)c->ncls[g], sizeof(class_t));
    /* count, then list tensors of each class in flat order */
    for (int t = 0; t < c->nt; ++t) {
        tensor_t* x = &c->t[t];
        int pp = stage_of_layer(c, x->layer);
        x->cls = x->group == 0 ? pp : pp * p->ep + ep_of_expert(c, x->expert);
        x->shard_len = numel4(x->shape) / (uint64_t)(x->tp_axis >= 0 ? (x->group ? c->etp : p->tp) : 1);
        c->cls[x->group][x->cls].n++;
    }
    for (int g = 0; g < 2; ++g)
        for (int k = 0; k < c->ncls[g]; ++k) {
            class_t* cl = &c->cls[g][k];
            cl->tid = (int32_t*)malloc(sizeof(int32_t) * (size_t)(cl->n + 1));
            cl->start = (uint64_t*)malloc(sizeof(uint64_t) * (size_t)(cl->n + 1));
            cl->n = 0;
        }
    for (int q = 0; q < c->nt; ++q) {
        int t = p->flat_order ? c->nt - 1 - q : q;
        tensor_t* x = &c->t[t];
        class_t* cl = &c->cls[x->group][x->cls];
        cl->tid[cl->n] = t;
        cl->start[cl->n] = cl->len;
        x->start = cl->len;
        cl->len += x->shard_len;
        cl->n++;
    }
    for (int g = 0; g < 2; ++g)
        for (int k = 0; k < c->ncls[g]; ++k) {
            class_t* cl = &c->cls[g][k];
            cl->start[cl->n] = cl->len;
            uint64_t q = 8ull * (uint64_t)(g == 0 ? c->ddp : c->edp);
            cl->padded = (cl->len + q - 1) / q * q;
        }
    return c;
}

void orc_config_destroy(orc_config* c)
{
    if (!c) return;
    for (int g = 0; g < 2; ++g) {
        if (!c->cls[g]) continue;
        for (int k = 0; k < c->ncls[g]; ++k) {
            free(c->cls[g][k].tid);
            free(c->cls[g][k].start);
        }
        free(c->cls[g]);
    }
    free(c->t);
    free(c);
}

int32_t orc_world(const orc_config* c) { return c->p.tp * c->p.pp * c->ddp; }
int32_t orc_num_tensors(const orc_config* c) { return c->nt; }

void orc_tensor_info(const orc_config* c, int32_t t, int32_t* shape, int32_t* info)
{
    const tensor_t* x = &c->t[t];
    for (int a = 0; a < 4; ++a) shape[a] = x->shape[a];
    info[0] = x->tp_axis; info[1] = x->group; info[2] = x->layer; info[3] = x->expert;
}

uint64_t orc_tensor_numel(const orc_config* c, int32_t t) { return numel4(c->t[t].shape); }

uint64_t orc_total_params(const orc_config* c)
{
    uint64_t s = 0;
    for (int t = 0; t < c->nt; ++t) s += numel4(c->t[t].shape);
    return s;
}

void orc_rank_coords(const orc_config* c, int32_t rank, int32_t* o)
{
    const int TP = c->p.tp, DDP = c->ddp, EP = c->p.ep, ETP = c->etp;
    int tp = rank % TP, ddp = (rank / TP) % DDP, pp = rank / (TP * DDP);
    int q = rank % (TP * DDP); /* position inside the pipeline stage */
    o[0] = tp; o[1] = ddp; o[2] = pp;
    o[5] = q % ETP; o[3] = (q / ETP) % EP; o[4] = q / (ETP * EP);
}

static int rank_of(const orc_config* c, int tp, int ddp, int pp)
{
    return tp + c->p.tp * (ddp + c->ddp * pp);
}

static int rank_of_expert(const orc_config* c, int etp, int ep, int edp, int pp)
{
    return etp + c->etp * (ep + c->p.ep * (edp + c->edp * pp));
}

/* The flat buffer that (rank, group) sees, its data-parallel group size and the rank's index
 * in that group. */
static const class_t* class_of_rank(const orc_config* c, int rank, int group, int* D, int* didx)
{
    int rc[6];
    orc_rank_coords(c, rank, rc);
    if (group == 0) {
        *D = c->ddp; *didx = rc[1];
        return &c->cls[0][rc[2]];
    }
    *D = c->edp; *didx = rc[4];
    return &c->cls[1][rc[2] * c->p.ep + rc[3]];
}

static int kind_sharded(const orc_config* c, int kind) { return c->p.zero == 1 && kind != 0; }

uint64_t orc_buffer_elems(const orc_config* c, int32_t rank, int32_t buf)
{
    int D, didx;
    const class_t* cl = class_of_rank(c, rank, buf / 4, &D, &didx);
    return kind_sharded(c, buf % 4) ? cl->padded / (uint64_t)D : cl->padded;
}

uint64_t orc_payload_elems(const orc_config* c, int32_t rank, int32_t buf)
{
    int D, didx;
    const class_t* cl = class_of_rank(c, rank, buf / 4, &D, &didx);
    if (!kind_sharded(c, buf % 4)) return cl->len;
    uint64_t per = cl->padded / (uint64_t)D, lo = per * (uint64_t)didx, hi = lo + per;
    if (lo >= cl->len) return 0;
    return (hi < cl->len ? hi : cl->len) - lo;
}

/* ------------------------------------------------------------------ local shard storage */

typedef struct {
    int32_t lo[4], ext[4]; /* the shard's box in global coordinates */
    int32_t nblk;
    int32_t blo[3], blen[3]; /* blocks along blk_axis, relative to the shard */
    int32_t blk_axis;
    int32_t order[4]; /* storage order of the axes, outermost first */
} shard_t;

static void shard_of(const orc_config* c, const tensor_t* x, int tp, shard_t* s)
{
    for (int a = 0; a < 4; ++a) { s->lo[a] = 0; s->ext[a] = x->shape[a]; }
    if (x->tp_axis >= 0) {
        s->ext[x->tp_axis] = x->shape[x->tp_axis] / (x->group ? c->etp : c->p.tp);
        s->lo[x->tp_axis] = tp * s->ext[x->tp_axis];
    }
    s->blk_axis = x->blk_axis;
    if (x->blk_axis >= 0 && c->p.qkv_layout == 1) {
        s->nblk = 3;
        s->blo[0] = 0;               s->blen[0] = c->q_per_g; /* all Q slots */
        s->blo[1] = c->q_per_g;      s->blen[1] = 1;          /* K */
        s->blo[2] = c->q_per_g + 1;  s->blen[2] = 1;          /* V */
    } else {
        s->nblk = 1;
        s->blk_axis = 0;
        s->blo[0] = 0; s->blen[0] = s->ext[0];
    }
    s->order[0] = 0; s->order[1] = 1; s->order[2] = 2; s->order[3] = 3;
    if (c->p.expert_layout == 1 && x->perm == PERM_GATE_UP) { /* (2, f, h) stored as (h, 2, f) */
        s->order[1] = 3; s->order[2] = 1; s->order[3] = 2;
    } else if (c->p.expert_layout == 1 && x->perm == PERM_DOWN) { /* (h, f) stored as (f, h) */
        s->order[2] = 3; s->order[3] = 2;
    }
}

/* Where global coordinate cd (inside the shard) is stored: the storage block, the block's
 * offset in the shard, the row-major index u inside the block and the block's dimensions n in
 * storage order (outermost first). */
static void shard_locate(const shard_t* s, const int32_t* cd, int* blk, uint64_t* base, uint64_t* u,
                         uint64_t* n)
{
    int32_t rel[4], e[4];
    for (int a = 0; a < 4; ++a) { rel[a] = cd[a] - s->lo[a]; e[a] = s->ext[a]; }
    *base = 0;
    int k = 0;
    for (; k < s->nblk; ++k) {
        if (rel[s->blk_axis] >= s->blo[k] && rel[s->blk_axis] < s->blo[k] + s->blen[k]) break;
        int32_t ee[4] = { e[0], e[1], e[2], e[3] };
        ee[s->blk_axis] = s->blen[k];
        *base += numel4(ee);
    }
    rel[s->blk_axis] -= s->blo[k];
    e[s->blk_axis] = s->blen[k];
    *u = 0;
    for (int q = 0; q < 4; ++q) {
        int a = s->order[q];
        *u = *u * (uint64_t)e[a] + (uint64_t)rel[a];
        n[q] = (uint64_t)e[a];
    }
    *blk = k;
}

/* shard-local storage index of global coordinate cd (must lie inside the shard) */
static uint64_t shard_index(const shard_t* s, const int32_t* cd)
{
    int blk;
    uint64_t base, u, n[4];
    shard_locate(s, cd, &blk, &base, &u, n);
    return base + u;
}

/* inverse of shard_index */
static void shard_coord(const shard_t* s, uint64_t u, int32_t* cd)
{
    int32_t e[4] = { s->ext[0], s->ext[1], s->ext[2], s->ext[3] };
    int k = 0;
    for (; k < s->nblk; ++k) {
        int32_t ee[4] = { e[0], e[1], e[2], e[3] };
        ee[s->blk_axis] = s->blen[k];
        uint64_t v = numel4(ee);
        if (u < v) break;
        u -= v;
    }
    e[s->blk_axis] = s->blen[k];
    int32_t rel[4];
    for (int q = 3; q >= 0; --q) { int a = s->order[q]; rel[a] = (int32_t)(u % (uint64_t)e[a]); u /= (uint64_t)e[a]; }
    rel[s->blk_axis] += s->blo[k];
    for (int a = 0; a < 4; ++a) cd[a] = s->lo[a] + rel[a];
}

/* ------------------------------------------------------------------ the two maps */

int orc_coord(const orc_config* c, int32_t rank, int32_t buf, uint64_t off, int32_t* tensor,
              int32_t* coord)
{
    int D, didx;
    const int group = buf / 4, kind = buf % 4;
    const class_t* cl = class_of_rank(c, rank, group, &D, &didx);
    uint64_t f = off;
    if (kind_sharded(c, kind)) {
        uint64_t per = cl->padded / (uint64_t)D;
        if (off >= per) return -1;
        f = off + per * (uint64_t)didx;
    } else if (off >= cl->padded) {
        return -1;
    }
    if (f >= cl->len) return 0; /* tail padding */
    /* the tensor whose shard covers flat offset f */
    int lo = 0, hi = cl->n - 1;
    while (lo < hi) {
        int mid = (lo + hi + 1) / 2;
        if (cl->start[mid] <= f) lo = mid; else hi = mid - 1;
    }
    const int t = cl->tid[lo];
    int rc[6];
    orc_rank_coords(c, rank, rc);
    shard_t s;
    shard_of(c, &c->t[t], group == 0 ? rc[0] : rc[5], &s);
    shard_coord(&s, f - cl->start[lo], coord);
    *tensor = t;
    return 1;
}

int orc_owners(const orc_config* c, int32_t kind, int32_t tensor, const int32_t* coord, int max,
               int32_t* ranks, int32_t* bufs, uint64_t* offs)
{
    const tensor_t* x = &c->t[tensor];
    const int TP = x->group == 0 ? c->p.tp : c->etp;
    const int pp = stage_of_layer(c, x->layer);
    const class_t* cl = &c->cls[x->group][x->cls];
    const int D = x->group == 0 ? c->ddp : c->edp;
    int tp_lo = 0, tp_hi = TP;
    if (x->tp_axis >= 0) {
        tp_lo = coord[x->tp_axis] / (x->shape[x->tp_axis] / TP);
        tp_hi = tp_lo + 1;
    }
    int n = 0;
    for (int di = 0; di < D; ++di) {
        for (int tp = tp_lo; tp < tp_hi; ++tp) {
            shard_t s;
            shard_of(c, x, tp, &s);
            uint64_t f = x->start + shard_index(&s, coord);
            uint64_t off = f;
            if (kind_sharded(c, kind)) {
                uint64_t per = cl->padded / (uint64_t)D;
                if (f / per != (uint64_t)di) continue;
                off = f - per * (uint64_t)di;
            }
            if (n < max) {
                ranks[n] = x->group == 0 ? rank_of(c, tp, di, pp)
                                         : rank_of_expert(c, tp, ep_of_expert(c, x->expert), di, pp);
                bufs[n] = x->group * 4 + kind;
                offs[n] = off;
            }
            ++n;
        }
    }
    return n;
}

uint64_t orc_linear(const orc_config* c, int32_t tensor, const int32_t* cd)
{
    const int32_t* s = c->t[tensor].shape;
    return (((uint64_t)cd[0] * (uint64_t)s[1] + (uint64_t)cd[1]) * (uint64_t)s[2] + (uint64_t)cd[2]) *
               (uint64_t)s[3] + (uint64_t)cd[3];
}

/* ------------------------------------------------------------------ source selection */

enum { MAX_OWNERS = 4096 };

int orc_select_source(const orc_config* a, const orc_config* b, int32_t j, int32_t kind,
                      int32_t tensor, const int32_t* coord, int32_t* rank, int32_t* buf,
                      uint64_t* off)
{
    int32_t r[MAX_OWNERS], bf[MAX_OWNERS];
    uint64_t of[MAX_OWNERS];
    int n = orc_owners(a, kind, tensor, coord, MAX_OWNERS, r, bf, of);
    if (n <= 0 || n > MAX_OWNERS) return 0;
    int pick = -1;
    for (int k = 0; k < n; ++k)
        if (r[k] == j) pick = k; /* the destination rank already holds it: retain */
    if (pick < 0) {
        /* owners are in ascending rank order; prefer the ones on j's node */
        int idx[MAX_OWNERS], m = 0;
        const int node = j / a->p.gpus_per_node;
        for (int k = 0; k < n; ++k)
            if (r[k] / a->p.gpus_per_node == node) idx[m++] = k;
        if (m == 0)
            for (int k = 0; k < n; ++k) idx[m++] = k;
        int rc[6];
        orc_rank_coords(b, j, rc);
        const int dpi = b->t[tensor].group == 0 ? rc[1] : rc[4];
        pick = idx[dpi % m];
    }
    *rank = r[pick]; *buf = bf[pick]; *off = of[pick];
    return 1;
}

/* ------------------------------------------------------------------ bulk helpers */

static void put_word(void* out, uint64_t k, int kind, uint32_t w)
{
    if (kind == 0) ((uint16_t*)out)[k] = (uint16_t)w; else ((uint32_t*)out)[k] = w;
}

int orc_fill(const orc_config* c, int32_t rank, int32_t buf, uint64_t seed, uint64_t rank_salt,
             uint64_t off0, uint64_t n, void* out, uint32_t pad_word)
{
    const int kind = buf % 4;
    const uint64_t sd = vps_pattern_seed_for_rank(seed, rank_salt, (uint32_t)rank);
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t k = 0; k < (int64_t)n; ++k) {
        int32_t t, cd[4];
        int r = orc_coord(c, rank, buf, off0 + (uint64_t)k, &t, cd);
        if (r < 0) { bad = 1; continue; }
        uint32_t w = r == 0 ? pad_word
                            : vps_pattern_word(sd, (uint32_t)kind, (uint32_t)t, orc_linear(c, t, cd));
        put_word(out, (uint64_t)k, kind, w);
    }
    return bad ? -1 : 0;
}

int orc_expected(const orc_config* a, const orc_config* b, int32_t j, int32_t buf, uint64_t seed,
                 uint64_t rank_salt, uint64_t off0, uint64_t n, void* out, uint32_t pad_word)
{
    const int kind = buf % 4;
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t k = 0; k < (int64_t)n; ++k) {
        int32_t t, cd[4], sr, sb;
        uint64_t so;
        int r = orc_coord(b, j, buf, off0 + (uint64_t)k, &t, cd);
        if (r < 0) { bad = 1; continue; }
        if (r == 0) { put_word(out, (uint64_t)k, kind, pad_word); continue; }
        if (!orc_select_source(a, b, j, kind, t, cd, &sr, &sb, &so)) { bad = 1; continue; }
        const uint64_t sd = vps_pattern_seed_for_rank(seed, rank_salt, (uint32_t)sr);
        put_word(out, (uint64_t)k, kind,
                 vps_pattern_word(sd, (uint32_t)kind, (uint32_t)t, orc_linear(a, t, cd)));
    }
    return bad ? -1 : 0;
}

int orc_transition(const orc_config* a, const orc_config* b, int32_t j, int32_t buf,
                   const void* const* src_bufs, uint64_t off0, uint64_t n, void* dst)
{
    const int kind = buf % 4;
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t k = 0; k < (int64_t)n; ++k) {
        int32_t t, cd[4], sr, sb;
        uint64_t so;
        int r = orc_coord(b, j, buf, off0 + (uint64_t)k, &t, cd);
        if (r < 0) { bad = 1; continue; }
        if (r == 0) continue;
        if (!orc_select_source(a, b, j, kind, t, cd, &sr, &sb, &so)) { bad = 1; continue; }
        const void* src = src_bufs[(size_t)sr * ORC_NBUF + (size_t)sb];
        if (!src) { bad = 1; continue; }
        if (kind == 0) ((uint16_t*)dst)[k] = ((const uint16_t*)src)[so];
        else ((uint32_t*)dst)[k] = ((const uint32_t*)src)[so];
    }
    return bad ? -1 : 0;
}

int orc_route_bytes(const orc_config* a, const orc_config* b, int32_t j, uint32_t buf_mask,
                    uint64_t* from_bytes)
{
    const int WA = orc_world(a);
    for (int i = 0; i < WA; ++i) from_bytes[i] = 0;
    int bad = 0;
    for (int buf = 0; buf < ORC_NBUF; ++buf) {
        if (!(buf_mask & (1u << buf))) continue;
        const int kind = buf % 4;
        const uint64_t es = kind == 0 ? 2 : 4;
        const int64_t n = (int64_t)orc_buffer_elems(b, j, buf);
#pragma omp parallel
        {
            uint64_t* loc = (uint64_t*)calloc((size_t)WA, sizeof(uint64_t));
#pragma omp for schedule(static) reduction(| : bad)
            for (int64_t k = 0; k < n; ++k) {
                int32_t t, cd[4], sr, sb;
                uint64_t so;
                int r = orc_coord(b, j, buf, (uint64_t)k, &t, cd);
                if (r <= 0) continue;
                if (!orc_select_source(a, b, j, kind, t, cd, &sr, &sb, &so)) { bad = 1; continue; }
                loc[sr] += es;
            }
#pragma omp critical
            for (int i = 0; i < WA; ++i) from_bytes[i] += loc[i];
            free(loc);
        }
    }
    return bad ? -1 : 0;
}

int orc_send_bytes(const orc_config* a, const orc_config* b, int32_t i, uint32_t buf_mask,
                   uint64_t* to_bytes)
{
    const int WB = orc_world(b);
    for (int j = 0; j < WB; ++j) to_bytes[j] = 0;
    int bad = 0;
    for (int buf = 0; buf < ORC_NBUF; ++buf) {
        if (!(buf_mask & (1u << buf))) continue;
        const int kind = buf % 4;
        const uint64_t es = kind == 0 ? 2 : 4;
        const int64_t n = (int64_t)orc_buffer_elems(a, i, buf);
#pragma omp parallel
        {
            uint64_t* loc = (uint64_t*)calloc((size_t)WB, sizeof(uint64_t));
            int32_t* dr = (int32_t*)malloc(sizeof(int32_t) * MAX_OWNERS);
            int32_t* db = (int32_t*)malloc(sizeof(int32_t) * MAX_OWNERS);
            uint64_t* dof = (uint64_t*)malloc(sizeof(uint64_t) * MAX_OWNERS);
#pragma omp for schedule(static) reduction(| : bad)
            for (int64_t k = 0; k < n; ++k) {
                int32_t t, cd[4], sr, sb;
                uint64_t so;
                int r = orc_coord(a, i, buf, (uint64_t)k, &t, cd);
                if (r <= 0) continue;
                int nd = orc_owners(b, kind, t, cd, MAX_OWNERS, dr, db, dof);
                if (nd > MAX_OWNERS) { bad = 1; continue; }
                for (int q = 0; q < nd; ++q) {
                    if (!orc_select_source(a, b, dr[q], kind, t, cd, &sr, &sb, &so)) { bad = 1; continue; }
                    if (sr == i) loc[dr[q]] += es;
                }
            }
#pragma omp critical
            for (int j = 0; j < WB; ++j) to_bytes[j] += loc[j];
            free(loc); free(dr); free(db); free(dof);
        }
    }
    return bad ? -1 : 0;
}

/* ------------------------------------------------------------------ per-peer buffers */

/* The order of data inside a per-peer buffer (Algorithm 1, PackData; Section 4.3 "Memory-Aware
 * Contiguous Buffer") is a convention of this repository, the paper leaves it open:
 *
 *   A rank stores, per tensor and storage block, one contiguous stretch [v0, v1) of the block's
 *   row-major storage (its flat range clipped to the block).  A stored element belongs to the
 *   coarsest aligned unit of that storage (an element, a row, a plane, ...) that lies completely
 *   inside [v0, v1); the units of one level under one parent unit form a *piece*, which is an
 *   axis-aligned box of the logical tensor.  The elements that travel from rank i to rank j and
 *   share a piece of i and a piece of j form a *routed box*.  Inside the segment i -> j the
 *   routed boxes are ordered by (state kind 1, 2, 3, 0; tensor id; lo corner in row-major order
 *   of the unsharded tensor); every box is serialised row-major in global axis order and starts
 *   at a multiple of 16 bytes.  A rank's receive buffer is the concatenation of the segments of
 *   its sources in ascending rank order, its send buffer that of its destinations. */

typedef struct {
    int32_t blk, level;
    uint64_t parent;
} piece_key_t;

/* The piece of `rank` that holds element (kind, tensor, cd); 0 if the rank does not store it. */
static int piece_of(const orc_config* c, int rank, int kind, int tensor, const int32_t* cd,
                    piece_key_t* k)
{
    const tensor_t* x = &c->t[tensor];
    int rc[6], D, didx;
    orc_rank_coords(c, rank, rc);
    shard_t s;
    shard_of(c, x, x->group == 0 ? rc[0] : rc[5], &s);
    for (int a = 0; a < 4; ++a)
        if (cd[a] < s.lo[a] || cd[a] >= s.lo[a] + s.ext[a]) return 0;
    int blk;
    uint64_t base, u, n[4];
    shard_locate(&s, cd, &blk, &base, &u, n);
    const class_t* cl = class_of_rank(c, rank, x->group, &D, &didx);
    if (cl != &c->cls[x->group][x->cls]) return 0; /* another pipeline stage or expert block */
    uint64_t r0 = 0, r1 = cl->padded;
    if (kind_sharded(c, kind)) {
        const uint64_t per = cl->padded / (uint64_t)D;
        r0 = per * (uint64_t)didx;
        r1 = r0 + per;
    }
    /* the rank's flat range, clipped to this block and relative to it */
    const uint64_t b0 = x->start + base, b1 = b0 + n[0] * n[1] * n[2] * n[3];
    const uint64_t lo = r0 > b0 ? r0 : b0, hi = r1 < b1 ? r1 : b1;
    if (lo >= hi) return 0;
    const uint64_t v0 = lo - b0, v1 = hi - b0;
    if (u < v0 || u >= v1) return 0;
    uint64_t st[4];
    st[3] = 1; st[2] = n[3]; st[1] = n[3] * n[2]; st[0] = n[3] * n[2] * n[1];
    int q = 0;
    for (; q < 3; ++q) {
        const uint64_t unit = u / st[q] * st[q];
        if (unit >= v0 && unit + st[q] <= v1) break;
    }
    k->blk = blk;
    k->level = q;
    k->parent = q == 0 ? 0 : u / st[q - 1];
    return 1;
}

int orc_piece_key(const orc_config* c, int32_t rank, int32_t buf, uint64_t off, int64_t* out3)
{
    int32_t t, cd[4];
    const int r = orc_coord(c, rank, buf, off, &t, cd);
    if (r <= 0) return r;
    piece_key_t k;
    if (!piece_of(c, rank, buf % 4, t, cd, &k)) return -2;
    out3[0] = k.blk; out3[1] = k.level; out3[2] = (int64_t)k.parent;
    return 1;
}

typedef struct {
    int32_t src, kind, tensor, ablk, alevel, bblk, blevel;
    uint64_t aparent, bparent;
} box_id_t;

typedef struct {
    box_id_t id;
    int32_t used;
    int32_t lo[4], hi[4]; /* componentwise smallest and largest coordinate seen */
    uint64_t count;       /* elements seen */
    uint64_t lin_lo;      /* row-major index of the lo corner in the unsharded tensor */
    uint64_t pos;         /* byte position of the box in the receive buffer */
} box_acc_t;

typedef struct {
    box_acc_t* e;
    size_t cap, n;
} box_table_t;

static int box_id_equal(const box_id_t* a, const box_id_t* b)
{
    return a->src == b->src && a->kind == b->kind && a->tensor == b->tensor && a->ablk == b->ablk &&
           a->alevel == b->alevel && a->bblk == b->bblk && a->blevel == b->blevel &&
           a->aparent == b->aparent && a->bparent == b->bparent;
}

static uint64_t box_id_hash(const box_id_t* a)
{
    uint64_t h = vps_pattern_mix64((uint64_t)a->src, (uint32_t)a->kind, (uint32_t)a->tensor, a->aparent);
    h = vps_pattern_mix64(h, (uint32_t)(a->ablk * 4 + a->alevel), (uint32_t)(a->bblk * 4 + a->blevel), a->bparent);
    return h;
}

static box_acc_t* box_find(box_table_t* t, const box_id_t* id, int insert);

static void box_grow(box_table_t* t)
{
    box_table_t old = *t;
    t->cap = old.cap ? old.cap * 2 : 256;
    t->e = (box_acc_t*)calloc(t->cap, sizeof(box_acc_t));
    t->n = 0;
    for (size_t i = 0; i < old.cap; ++i)
        if (old.e[i].used) *box_find(t, &old.e[i].id, 1) = old.e[i];
    free(old.e);
}

static box_acc_t* box_find(box_table_t* t, const box_id_t* id, int insert)
{
    if (insert && (t->n + 1) * 2 > t->cap) box_grow(t);
    if (!t->cap) return NULL;
    size_t i = (size_t)box_id_hash(id) & (t->cap - 1);
    while (t->e[i].used) {
        if (box_id_equal(&t->e[i].id, id)) return &t->e[i];
        i = (i + 1) & (t->cap - 1);
    }
    if (!insert) return NULL;
    box_acc_t* e = &t->e[i];
    e->id = *id;
    e->used = 1;
    e->count = 0;
    for (int a = 0; a < 4; ++a) { e->lo[a] = INT32_MAX; e->hi[a] = INT32_MIN; }
    t->n++;
    return e;
}

static void box_absorb(box_acc_t* e, const int32_t* lo, const int32_t* hi, uint64_t count)
{
    for (int a = 0; a < 4; ++a) {
        if (lo[a] < e->lo[a]) e->lo[a] = lo[a];
        if (hi[a] > e->hi[a]) e->hi[a] = hi[a];
    }
    e->count += count;
}

/* The routed box of destination slot (j, buf, off): 1 and id filled if the element travels
 * (or stays, when `through` routes retained data through the buffers too), 0 otherwise. */
static int routed_box_of(const orc_config* a, const orc_config* b, int j, int buf, uint64_t off,
                         int through, box_id_t* id, int32_t* cd)
{
    int32_t t, sr, sb;
    uint64_t so;
    if (orc_coord(b, j, buf, off, &t, cd) != 1) return 0;
    const int kind = buf % 4;
    if (!orc_select_source(a, b, j, kind, t, cd, &sr, &sb, &so)) return -1;
    if (sr == j && !through) return 0;
    piece_key_t ka, kb;
    if (!piece_of(a, sr, kind, t, cd, &ka) || !piece_of(b, j, kind, t, cd, &kb)) return -1;
    id->src = sr; id->kind = kind; id->tensor = t;
    id->ablk = ka.blk; id->alevel = ka.level; id->aparent = ka.parent;
    id->bblk = kb.blk; id->blevel = kb.level; id->bparent = kb.parent;
    return 1;
}

static int box_order(const void* pa, const void* pb)
{
    const box_acc_t* x = *(box_acc_t* const*)pa;
    const box_acc_t* y = *(box_acc_t* const*)pb;
    if (x->id.src != y->id.src) return x->id.src < y->id.src ? -1 : 1;
    const int kx = (x->id.kind + 3) & 3, ky = (y->id.kind + 3) & 3; /* kinds 1, 2, 3, then 0 */
    if (kx != ky) return kx < ky ? -1 : 1;
    if (x->id.tensor != y->id.tensor) return x->id.tensor < y->id.tensor ? -1 : 1;
    if (x->lin_lo != y->lin_lo) return x->lin_lo < y->lin_lo ? -1 : 1;
    return 0;
}

int64_t orc_recv_payload(const orc_config* a, const orc_config* b, int32_t j, int through,
                         uint64_t seed, uint64_t rank_salt, uint8_t pad_byte, void* out,
                         uint64_t cap, uint64_t* seg_off)
{
    const int WA = orc_world(a);
    box_table_t all = { NULL, 0, 0 };
    int bad = 0;
    /* pass 1: which routed boxes exist, their corners and element counts */
#pragma omp parallel
    {
        box_table_t mine = { NULL, 0, 0 };
        for (int buf = 0; buf < ORC_NBUF; ++buf) {
            const int64_t n = (int64_t)orc_buffer_elems(b, j, buf);
#pragma omp for schedule(static) reduction(| : bad)
            for (int64_t k = 0; k < n; ++k) {
                box_id_t id;
                int32_t cd[4];
                const int r = routed_box_of(a, b, j, buf, (uint64_t)k, through, &id, cd);
                if (r < 0) bad = 1;
                if (r <= 0) continue;
                box_absorb(box_find(&mine, &id, 1), cd, cd, 1);
            }
        }
#pragma omp critical
        for (size_t i = 0; i < mine.cap; ++i)
            if (mine.e[i].used) box_absorb(box_find(&all, &mine.e[i].id, 1), mine.e[i].lo, mine.e[i].hi, mine.e[i].count);
        free(mine.e);
    }
    if (bad) { free(all.e); return -1; }
    /* order and positions */
    box_acc_t** ord = (box_acc_t**)malloc(sizeof(box_acc_t*) * (all.n ? all.n : 1));
    size_t nb = 0;
    for (size_t i = 0; i < all.cap; ++i) {
        box_acc_t* e = &all.e[i];
        if (!e->used) continue;
        uint64_t vol = 1;
        for (int ax = 0; ax < 4; ++ax) vol *= (uint64_t)(e->hi[ax] - e->lo[ax] + 1);
        if (vol != e->count) bad = 1; /* the elements of a piece pair must fill their bounding box */
        e->lin_lo = orc_linear(a, e->id.tensor, e->lo);
        ord[nb++] = e;
    }
    qsort(ord, nb, sizeof(box_acc_t*), box_order);
    uint64_t pos = 0;
    size_t k = 0;
    for (int i = 0; i <= WA; ++i) {
        if (seg_off) seg_off[i] = pos;
        for (; k < nb && ord[k]->id.src == i; ++k) {
            ord[k]->pos = pos;
            pos += (ord[k]->count * (ord[k]->id.kind == 0 ? 2u : 4u) + 15u) & ~(uint64_t)15;
        }
    }
    free(ord);
    if (bad || pos > cap) { free(all.e); return bad ? -2 : -3; }
    memset(out, pad_byte, (size_t)pos);
    /* pass 2: every travelling element to its place in its box */
    for (int buf = 0; buf < ORC_NBUF; ++buf) {
        const int64_t n = (int64_t)orc_buffer_elems(b, j, buf);
#pragma omp parallel for schedule(static) reduction(| : bad)
        for (int64_t q = 0; q < n; ++q) {
            box_id_t id;
            int32_t cd[4];
            if (routed_box_of(a, b, j, buf, (uint64_t)q, through, &id, cd) <= 0) continue;
            const box_acc_t* e = box_find(&all, &id, 0);
            if (!e) { bad = 1; continue; }
            uint64_t idx = 0; /* row-major index inside the box, global axis order */
            for (int ax = 0; ax < 4; ++ax) idx = idx * (uint64_t)(e->hi[ax] - e->lo[ax] + 1) + (uint64_t)(cd[ax] - e->lo[ax]);
            const uint64_t sd = vps_pattern_seed_for_rank(seed, rank_salt, (uint32_t)id.src);
            const uint32_t w = vps_pattern_word(sd, (uint32_t)id.kind, (uint32_t)id.tensor, orc_linear(a, id.tensor, cd));
            if (id.kind == 0) ((uint16_t*)((char*)out + e->pos))[idx] = (uint16_t)w;
            else ((uint32_t*)((char*)out + e->pos))[idx] = w;
        }
    }
    free(all.e);
    return bad ? -1 : (int64_t)pos;
}

/* ------------------------------------------------------------------ box validation */

static int check_one(const orc_config* a, const orc_config* b, const int32_t* I, const int64_t* O,
                     const int32_t* rel)
{
    const int kind = I[0], tensor = I[1], srank = I[2], drank = I[3], sbuf = I[4], dbuf = I[5];
    int32_t cd[4];
    uint64_t so = (uint64_t)O[0], dof = (uint64_t)O[1];
    for (int ax = 0; ax < 4; ++ax) {
        cd[ax] = I[6 + ax] + rel[ax];
        so += (uint64_t)((int64_t)rel[ax] * O[2 + ax]);
        dof += (uint64_t)((int64_t)rel[ax] * O[6 + ax]);
    }
    /* destination slot must decode to this element under B */
    int32_t t2, c2[4];
    if (dbuf % 4 != kind || sbuf % 4 != kind) return 1;
    if (orc_coord(b, drank, dbuf, dof, &t2, c2) != 1) return 1;
    if (t2 != tensor || memcmp(c2, cd, sizeof(cd))) return 1;
    /* source slot must decode to this element under A */
    if (orc_coord(a, srank, sbuf, so, &t2, c2) != 1) return 1;
    if (t2 != tensor || memcmp(c2, cd, sizeof(cd))) return 1;
    /* and the source must be the selected one */
    int32_t sr, sb;
    uint64_t so2;
    if (!orc_select_source(a, b, drank, kind, tensor, cd, &sr, &sb, &so2)) return 1;
    if (sr != srank || sb != sbuf || so2 != so) return 1;
    return 0;
}

int64_t orc_check_boxes(const orc_config* a, const orc_config* b, const int32_t* ints,
                        const int64_t* offs, int64_t nboxes, int32_t samples, int64_t* first_bad)
{
    int64_t nbad = 0, first = -1;
#pragma omp parallel for schedule(dynamic, 16) reduction(+ : nbad)
    for (int64_t k = 0; k < nboxes; ++k) {
        const int32_t* I = ints + k * 16;
        const int64_t* O = offs + k * 10;
        const int32_t* e = I + 10;
        int64_t vol = (int64_t)e[0] * e[1] * e[2] * e[3];
        int64_t bad = 0;
        if (vol <= 0) bad = 1;
        else if (samples <= 0 || vol <= samples + 16) {
            for (int64_t u = 0; u < vol; ++u) {
                int64_t v = u;
                int32_t rel[4];
                for (int ax = 3; ax >= 0; --ax) { rel[ax] = (int32_t)(v % e[ax]); v /= e[ax]; }
                bad += check_one(a, b, I, O, rel);
            }
        } else {
            for (int cn = 0; cn < 16; ++cn) { /* the 16 corners */
                int32_t rel[4];
                for (int ax = 0; ax < 4; ++ax) rel[ax] = (cn >> ax) & 1 ? e[ax] - 1 : 0;
                bad += check_one(a, b, I, O, rel);
            }
            uint64_t st = 0x1234567ull + (uint64_t)k;
            for (int sidx = 0; sidx < samples; ++sidx) {
                int32_t rel[4];
                for (int ax = 0; ax < 4; ++ax) {
                    st = vps_pattern_mix64(st, 0, (uint32_t)sidx, (uint64_t)ax);
                    rel[ax] = (int32_t)(st % (uint64_t)e[ax]);
                }
                bad += check_one(a, b, I, O, rel);
            }
        }
        if (bad) {
#pragma omp critical
            if (first < 0 || k < first) first = k;
        }
        nbad += bad;
    }
    if (first_bad) *first_bad = first;
    return nbad;
}

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Number of OpenMP threads for the calls that follow (timing with one core and with all). */
void orc_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}
