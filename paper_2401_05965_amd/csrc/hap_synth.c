/*
 * Distributed program synthesis on small graphs (Sec. 4): the background theory of Hoare triples
 * (Fig. "semantics", plus the Grouped-Broadcast and replicated-MatMul rules of Sec. 4.4), the cost
 * model t(Q, B) of Sec. 3.2, and the A* search with dominance pruning of Fig. "a*".  Host, plain C.
 *
 * A property is (reference tensor e, form): form says which collective turns the distributed tensor
 * into e on every device - none (replicated), All-Gather along dimension 0 or 1 (sharded), or
 * All-Reduce (partial sums).  Properties are bits of a 64-bit set (4 per tensor, so <= 16 tensors).
 *
 * Search-space restrictions: a reference tensor is communicated at most once and the outputs of
 * Placeholder / Parameter are never communicated (Sec. 4.5, second optimisation); in addition every
 * reference tensor is computed exactly once and computations follow the graph's order, so a program
 * is fixed by the form chosen for every tensor and by where the collectives are placed.  Properties
 * of a tensor whose consumers have all been computed are dropped (Sec. 4.5, third optimisation).
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include "hap_internal.h"

#define MAX_NODES 16
#define MAX_DEV 16
#define MAX_TRIPLES 512

enum { F_ID = HAP_FORM_ID, F_AG0 = HAP_FORM_AG0, F_AG1 = HAP_FORM_AG1, F_AR = HAP_FORM_AR };

typedef struct { uint64_t pre, post; hap_instr ins; } triple;

static uint64_t bit(int e, int form) { return (uint64_t)1 << (e * 4 + form); }
static int is_comm(int kind) { return kind >= HAP_I_ALL_REDUCE; }

static int add_triple(triple* T, int* n, uint64_t pre, uint64_t post, int kind, int e, int a0, int a1) {
  if (*n >= MAX_TRIPLES) return -1;
  T[*n].pre = pre; T[*n].post = post;
  T[*n].ins.kind = kind; T[*n].ins.tensor = e; T[*n].ins.arg0 = a0; T[*n].ins.arg1 = a1;
  ++*n;
  return 0;
}

/* Builds the background theory: every rule is matched against every node of the graph (Sec. 4.2). */
static int build_theory(int n_nodes, const hap_graph_node* g, const hap_synth_rules* r, triple* T, int* nt) {
  *nt = 0;
  int bad = 0;
  for (int e = 0; e < n_nodes; ++e) {
    const int a = g[e].a, b = g[e].b;
    switch (g[e].op) {
      case HAP_OP_PLACEHOLDER:
        if (r->placeholder_replicated) bad |= add_triple(T, nt, 0, bit(e, F_ID), HAP_I_PLACEHOLDER, e, 0, 0);
        for (int d = 0; d < 2; ++d)
          if (r->placeholder_dims_mask >> d & 1) bad |= add_triple(T, nt, 0, bit(e, F_AG0 + d), HAP_I_PLACEHOLDER_SHARD, e, d, 0);
        break;
      case HAP_OP_PARAMETER:
        bad |= add_triple(T, nt, 0, bit(e, F_ID), HAP_I_PARAMETER, e, 0, 0);
        for (int d = 0; d < 2; ++d)
          if (r->parameter_dims_mask >> d & 1) bad |= add_triple(T, nt, 0, bit(e, F_AG0 + d), HAP_I_PARAMETER_SHARD, e, d, 0);
        break;
      case HAP_OP_MATMUL:      /* the three rules of Fig. "semantics" and the replicated rule of Sec. 4.4 */
        bad |= add_triple(T, nt, bit(a, F_AG0) | bit(b, F_ID), bit(e, F_AG0), HAP_I_MATMUL, e, F_AG0, F_ID);
        bad |= add_triple(T, nt, bit(a, F_ID) | bit(b, F_AG1), bit(e, F_AG1), HAP_I_MATMUL, e, F_ID, F_AG1);
        bad |= add_triple(T, nt, bit(a, F_AG1) | bit(b, F_AG0), bit(e, F_AR), HAP_I_MATMUL, e, F_AG1, F_AG0);
        if (r->replicated_matmul) bad |= add_triple(T, nt, bit(a, F_ID) | bit(b, F_ID), bit(e, F_ID), HAP_I_MATMUL, e, F_ID, F_ID);
        break;
      case HAP_OP_UNARY:       /* element-wise and non-linear: any layout except partial sums */
        for (int f = F_ID; f <= F_AG1; ++f) bad |= add_triple(T, nt, bit(a, f), bit(e, f), HAP_I_UNARY, e, f, 0);
        break;
      case HAP_OP_ADD:         /* element-wise and linear */
        for (int f = F_ID; f <= F_AR; ++f) bad |= add_triple(T, nt, bit(a, f) | bit(b, f), bit(e, f), HAP_I_ADD, e, f, 0);
        break;
      case HAP_OP_TRANSPOSE:
        bad |= add_triple(T, nt, bit(a, F_ID), bit(e, F_ID), HAP_I_TRANSPOSE, e, F_ID, 0);
        bad |= add_triple(T, nt, bit(a, F_AG0), bit(e, F_AG1), HAP_I_TRANSPOSE, e, F_AG0, 0);
        bad |= add_triple(T, nt, bit(a, F_AG1), bit(e, F_AG0), HAP_I_TRANSPOSE, e, F_AG1, 0);
        bad |= add_triple(T, nt, bit(a, F_AR), bit(e, F_AR), HAP_I_TRANSPOSE, e, F_AR, 0);
        break;
      case HAP_OP_SUM:         /* the local sums of shards or of partial sums add up to the whole sum */
        bad |= add_triple(T, nt, bit(a, F_AG0), bit(e, F_AR), HAP_I_SUM, e, F_AG0, 0);
        bad |= add_triple(T, nt, bit(a, F_AG1), bit(e, F_AR), HAP_I_SUM, e, F_AG1, 0);
        bad |= add_triple(T, nt, bit(a, F_AR), bit(e, F_AR), HAP_I_SUM, e, F_AR, 0);
        bad |= add_triple(T, nt, bit(a, F_ID), bit(e, F_ID), HAP_I_SUM, e, F_ID, 0);
        break;
      default:
        return hap_fail(HAP_EINVAL, "node %d: bad op %d", e, g[e].op);
    }
    if (g[e].op != HAP_OP_PLACEHOLDER && g[e].op != HAP_OP_PARAMETER && g[e].op != HAP_OP_SUM) {   /* the collectives of Fig. "semantics" */
      bad |= add_triple(T, nt, bit(e, F_AR), bit(e, F_ID), HAP_I_ALL_REDUCE, e, 0, 0);
      for (int d = 0; d < 2; ++d) {
        bad |= add_triple(T, nt, bit(e, F_AR), bit(e, F_AG0 + d), HAP_I_REDUCE_SCATTER, e, d, 0);
        bad |= add_triple(T, nt, bit(e, F_AG0 + d), bit(e, F_ID), HAP_I_ALL_GATHER, e, d, 0);
        if (r->grouped_broadcast) bad |= add_triple(T, nt, bit(e, F_AG0 + d), bit(e, F_ID), HAP_I_GROUPED_BROADCAST, e, d, 0);
        bad |= add_triple(T, nt, bit(e, F_AG0 + d), bit(e, F_AG0 + 1 - d), HAP_I_ALL_TO_ALL, e, d, 1 - d);
      }
    }
  }
  if (bad) return hap_fail(HAP_EUNSUPPORTED, "theory has more than %d triples", MAX_TRIPLES);
  return HAP_OK;
}

/* Flops of a computation instruction on a device with ratio Bj (Sec. 3.2). */
static double instr_flops(const hap_graph_node* g, const hap_instr* ins, double Bj) {
  const hap_graph_node* n = &g[ins->tensor];
  switch (ins->kind) {
    case HAP_I_MATMUL: {
      const double full = 2.0 * (double)g[n->a].rows * (double)g[n->a].cols * (double)n->cols;
      return (ins->arg0 == F_ID && ins->arg1 == F_ID) ? full : full * Bj;
    }
    case HAP_I_UNARY: case HAP_I_TRANSPOSE: case HAP_I_SUM: {
      const double full = (double)g[n->a].rows * (double)g[n->a].cols;
      return (ins->arg0 == F_AG0 || ins->arg0 == F_AG1) ? full * Bj : full;
    }
    case HAP_I_ADD: {
      const double full = (double)n->rows * (double)n->cols;
      return (ins->arg0 == F_AG0 || ins->arg0 == F_AG1) ? full * Bj : full;
    }
    default: return 0.0;     /* loading instructions */
  }
}

/* Linear latency + size / bandwidth model; the largest shard decides (Sec. 3.2, Sec. 5.1). */
static double comm_seconds(const hap_graph_node* g, const hap_instr* ins, int m, double bmax, const hap_net* net) {
  const double size = (double)g[ins->tensor].rows * (double)g[ins->tensor].cols * net->elem_bytes;
  if (ins->kind == HAP_I_ALL_REDUCE) return net->latency + 2.0 * size / net->bandwidth;
  if (ins->kind == HAP_I_GROUPED_BROADCAST) return m * net->latency + size / net->bandwidth;      /* no padding, one launch per shard */
  return net->latency + m * bmax * size / net->bandwidth;                                         /* m equal slots of the largest shard */
}

static int check_graph(int n_nodes, const hap_graph_node* g) {
  if (n_nodes < 1 || n_nodes > MAX_NODES) return hap_fail(HAP_EUNSUPPORTED, "n_nodes = %d outside [1, %d]", n_nodes, MAX_NODES);
  if (!g) return hap_fail(HAP_EINVAL, "graph is NULL");
  for (int e = 0; e < n_nodes; ++e) {
    const int op = g[e].op;
    const int unary = op == HAP_OP_UNARY || op == HAP_OP_TRANSPOSE || op == HAP_OP_SUM, binary = op == HAP_OP_MATMUL || op == HAP_OP_ADD;
    if (g[e].rows < 1 || g[e].cols < 1) return hap_fail(HAP_EINVAL, "node %d: bad shape", e);
    if ((unary || binary) && (g[e].a < 0 || g[e].a >= e)) return hap_fail(HAP_ESHAPE, "node %d: input a must be an earlier node", e);
    if (binary && (g[e].b < 0 || g[e].b >= e)) return hap_fail(HAP_ESHAPE, "node %d: input b must be an earlier node", e);
    if (op == HAP_OP_MATMUL && (g[g[e].a].cols != g[g[e].b].rows || g[e].rows != g[g[e].a].rows || g[e].cols != g[g[e].b].cols))
      return hap_fail(HAP_ESHAPE, "node %d: MatMul shapes do not agree", e);
  }
  if (g[n_nodes - 1].op != HAP_OP_SUM) return hap_fail(HAP_EINVAL, "the last node must be the loss (a Sum)");
  return HAP_OK;
}

static int check_cluster(int m, const double* ratios, const double* speed, const hap_net* net) {
  if (m < 1 || m > MAX_DEV) return hap_fail(HAP_EUNSUPPORTED, "m = %d outside [1, %d]", m, MAX_DEV);
  if (!ratios || !speed || !net) return hap_fail(HAP_EINVAL, "NULL argument");
  for (int j = 0; j < m; ++j)
    if (!(ratios[j] >= 0.0) || !(speed[j] > 0.0)) return hap_fail(HAP_EINVAL, "device %d: ratio must be >= 0 and speed > 0", j);
  if (!(net->latency >= 0.0) || !(net->bandwidth > 0.0) || net->elem_bytes < 1) return hap_fail(HAP_EINVAL, "bad network model");
  return HAP_OK;
}

int hap_program_time(int n_nodes, const hap_graph_node* graph, int n_instr, const hap_instr* program, int m,
                     const double* ratios, const double* speed, const hap_net* net, double* seconds) {
  hap_clear_error();
  int rc = check_graph(n_nodes, graph);
  if (rc) return rc;
  if ((rc = check_cluster(m, ratios, speed, net))) return rc;
  if (n_instr < 0 || (n_instr > 0 && !program) || !seconds) return hap_fail(HAP_EINVAL, "bad program or NULL result");
  double bmax = 0.0, busy[MAX_DEV] = {0}, total = 0.0;
  for (int j = 0; j < m; ++j) if (ratios[j] > bmax) bmax = ratios[j];
  for (int i = 0; i < n_instr; ++i) {
    if (program[i].tensor < 0 || program[i].tensor >= n_nodes) return hap_fail(HAP_EINVAL, "instruction %d names no tensor of the graph", i);
    if (is_comm(program[i].kind)) {      /* a collective synchronises the devices: the stage ends with its slowest device */
      double mx = 0.0;
      for (int j = 0; j < m; ++j) { if (busy[j] > mx) mx = busy[j]; busy[j] = 0.0; }
      total += mx + comm_seconds(graph, &program[i], m, bmax, net);
    } else {
      for (int j = 0; j < m; ++j) busy[j] += instr_flops(graph, &program[i], ratios[j]) / speed[j];
    }
  }
  double mx = 0.0;
  for (int j = 0; j < m; ++j) if (busy[j] > mx) mx = busy[j];
  *seconds = total + mx;
  return HAP_OK;
}

/* The stages of a program in the form Eq. (opt_B) takes (Sec. 3.2): a collective opens a stage; its time is
 * latency + per_ratio * max_j B_j; the stage's computation is (sharded * B_j + fixed) / speed_j. */
int hap_program_stages(int n_nodes, const hap_graph_node* graph, int n_instr, const hap_instr* program, int m,
                       const hap_net* net, hap_stage* stages, int capacity, int* n_stages) {
  hap_clear_error();
  int rc = check_graph(n_nodes, graph);
  if (rc) return rc;
  if (m < 1 || m > MAX_DEV || !net) return hap_fail(HAP_EINVAL, "bad m or NULL network model");
  if (n_instr < 0 || (n_instr > 0 && !program) || !stages || !n_stages || capacity < 1) return hap_fail(HAP_EINVAL, "bad program or no room for stages");
  int ns = 0;
  memset(&stages[0], 0, sizeof(hap_stage));
  for (int i = 0; i < n_instr; ++i) {
    if (program[i].tensor < 0 || program[i].tensor >= n_nodes) return hap_fail(HAP_EINVAL, "instruction %d names no tensor of the graph", i);
    if (is_comm(program[i].kind)) {
      if (++ns >= capacity) return hap_fail(HAP_EWORKSPACE, "more than %d stages", capacity);
      memset(&stages[ns], 0, sizeof(hap_stage));
      /* comm_seconds() is affine in the largest ratio: read off its two coefficients */
      stages[ns].comm_latency = comm_seconds(graph, &program[i], m, 0.0, net);
      stages[ns].comm_per_ratio = comm_seconds(graph, &program[i], m, 1.0, net) - stages[ns].comm_latency;
    } else {
      const double f1 = instr_flops(graph, &program[i], 1.0), f0 = instr_flops(graph, &program[i], 0.0);
      stages[ns].flops_sharded += f1 - f0;
      stages[ns].flops_fixed += f0;
    }
  }
  *n_stages = ns + 1;
  return HAP_OK;
}

/* Sec. 3.1: alternate Q(s) = argmin_Q t(Q, B(s-1)) and B(s) = argmin_B t(Q(s), B), starting from ratios proportional to the
 * speeds, until the pair repeats or max_steps is reached; the best pair seen is returned. */
int hap_optimize(int n_nodes, const hap_graph_node* graph, int m, const double* speed, const hap_net* net,
                 const hap_synth_rules* rules, int max_steps, hap_instr* program, int capacity, int* n_instr,
                 double* ratios, double* seconds, int* steps) {
  hap_clear_error();
  if (!speed || !ratios || !program || !n_instr) return hap_fail(HAP_EINVAL, "NULL argument");
  if (m < 1 || m > MAX_DEV) return hap_fail(HAP_EUNSUPPORTED, "m = %d outside [1, %d]", m, MAX_DEV);
  if (max_steps < 1) max_steps = 1;
  double B[MAX_DEV], total = 0.0, best_t = INFINITY, prev_t = INFINITY;
  for (int j = 0; j < m; ++j) { if (!(speed[j] > 0.0)) return hap_fail(HAP_EINVAL, "speed[%d] must be positive", j); total += speed[j]; }
  for (int j = 0; j < m; ++j) B[j] = speed[j] / total;
  hap_instr* cur = (hap_instr*)malloc(sizeof(hap_instr) * (size_t)capacity);
  hap_stage* st = (hap_stage*)malloc(sizeof(hap_stage) * (size_t)(capacity + 1));
  if (!cur || !st) { free(cur); free(st); return hap_fail(HAP_EINVAL, "out of host memory"); }
  int rc = HAP_OK, s = 0;
  for (s = 1; s <= max_steps; ++s) {
    int len = 0, ns = 0;
    double tq = 0.0, tb = 0.0;
    if ((rc = hap_synthesize(n_nodes, graph, m, B, speed, net, rules, cur, capacity, &len, &tq, NULL))) break;
    if (tq < best_t) { best_t = tq; memcpy(program, cur, sizeof(hap_instr) * (size_t)len); *n_instr = len; memcpy(ratios, B, sizeof(double) * (size_t)m); }
    if ((rc = hap_program_stages(n_nodes, graph, len, cur, m, net, st, capacity + 1, &ns))) break;
    double Bn[MAX_DEV];
    if ((rc = hap_shard_ratios(m, speed, ns, st, Bn, &tb))) break;
    if (tb < best_t) { best_t = tb; memcpy(program, cur, sizeof(hap_instr) * (size_t)len); *n_instr = len; memcpy(ratios, Bn, sizeof(double) * (size_t)m); }
    memcpy(B, Bn, sizeof(double) * (size_t)m);
    if (!(tb < prev_t * (1.0 - 1e-12))) break;      /* no further gain: converged (or about to oscillate) */
    prev_t = tb;
  }
  free(cur); free(st);
  if (rc) return rc;
  if (seconds) *seconds = best_t;
  if (steps) *steps = s > max_steps ? max_steps : s;
  return HAP_OK;
}

/* A partial program: its last instruction and its parent (the program is the chain back to the root). */
typedef struct {
  int parent;
  hap_instr ins;
  uint64_t props;          /* P(Q) after dropping the properties nothing can use any more */
  uint32_t communicated;   /* reference tensors that already went through a collective */
  int next;                /* next node to compute */
  int depth;
  int alive;
  double closed;           /* time up to the last synchronisation point */
  double busy[MAX_DEV];    /* computation of the open stage, per device */
  double score;            /* cost(Q) + ecost(Q) */
} state;

typedef struct { state* s; int n, cap; int* heap; int hn, hcap; } pool;

static double state_cost(const state* s, int m) {
  double mx = 0.0;
  for (int j = 0; j < m; ++j) if (s->busy[j] > mx) mx = s->busy[j];
  return s->closed + mx;
}

static int heap_push(pool* p, int idx) {
  if (p->hn == p->hcap) {
    const int nc = p->hcap ? p->hcap * 2 : 256;
    int* nh = (int*)realloc(p->heap, (size_t)nc * sizeof(int));
    if (!nh) return -1;
    p->heap = nh; p->hcap = nc;
  }
  int i = p->hn++;
  p->heap[i] = idx;
  while (i > 0) {
    const int par = (i - 1) / 2;
    if (p->s[p->heap[par]].score <= p->s[p->heap[i]].score) break;
    const int t = p->heap[par]; p->heap[par] = p->heap[i]; p->heap[i] = t; i = par;
  }
  return 0;
}

static int heap_pop(pool* p) {
  const int top = p->heap[0];
  p->heap[0] = p->heap[--p->hn];
  int i = 0;
  for (;;) {
    int l = 2 * i + 1, r = l + 1, b = i;
    if (l < p->hn && p->s[p->heap[l]].score < p->s[p->heap[b]].score) b = l;
    if (r < p->hn && p->s[p->heap[r]].score < p->s[p->heap[b]].score) b = r;
    if (b == i) break;
    const int t = p->heap[b]; p->heap[b] = p->heap[i]; p->heap[i] = t; i = b;
  }
  return top;
}

int hap_synthesize(int n_nodes, const hap_graph_node* graph, int m, const double* ratios, const double* speed,
                   const hap_net* net, const hap_synth_rules* rules, hap_instr* program, int capacity, int* n_instr,
                   double* seconds, int64_t* expanded) {
  hap_clear_error();
  int rc = check_graph(n_nodes, graph);
  if (rc) return rc;
  if ((rc = check_cluster(m, ratios, speed, net))) return rc;
  if (!program || !n_instr || capacity < 1) return hap_fail(HAP_EINVAL, "no room for the program");
  const hap_synth_rules all = {3, 3, 1, 1, 1};
  if (!rules) rules = &all;
  triple* T = (triple*)malloc(sizeof(triple) * MAX_TRIPLES);
  if (!T) return hap_fail(HAP_EINVAL, "out of host memory");
  int nt = 0;
  if ((rc = build_theory(n_nodes, graph, rules, T, &nt))) { free(T); return rc; }

  double bmax = 0.0;
  for (int j = 0; j < m; ++j) if (ratios[j] > bmax) bmax = ratios[j];
  /* users[e]: the nodes that read e; lastuse[e]: the last of them */
  int lastuse[MAX_NODES];
  for (int e = 0; e < n_nodes; ++e) lastuse[e] = -1;
  for (int e = 0; e < n_nodes; ++e) {
    if (graph[e].op >= HAP_OP_MATMUL) { if (graph[e].a >= 0) lastuse[graph[e].a] = e; }
    if (graph[e].op == HAP_OP_MATMUL || graph[e].op == HAP_OP_ADD) lastuse[graph[e].b] = e;
  }
  /* ecost: with infinite bandwidth and every remaining operation sharded, device j still needs rest[e][j] seconds for nodes >= e */
  double rest[MAX_NODES + 1][MAX_DEV];
  for (int j = 0; j < m; ++j) rest[n_nodes][j] = 0.0;
  for (int e = n_nodes - 1; e >= 0; --e)
    for (int j = 0; j < m; ++j) {
      double full = 0.0;
      const hap_graph_node* n = &graph[e];
      if (n->op == HAP_OP_MATMUL) full = 2.0 * (double)graph[n->a].rows * (double)graph[n->a].cols * (double)n->cols;
      else if (n->op == HAP_OP_UNARY || n->op == HAP_OP_TRANSPOSE || n->op == HAP_OP_SUM) full = (double)graph[n->a].rows * (double)graph[n->a].cols;
      else if (n->op == HAP_OP_ADD) full = (double)n->rows * (double)n->cols;
      rest[e][j] = rest[e + 1][j] + full * ratios[j] / speed[j];
    }
  const int loss = n_nodes - 1;
  const uint64_t goal = bit(loss, F_AR);

  pool p = {0};
  p.cap = 1024;
  p.s = (state*)malloc(sizeof(state) * (size_t)p.cap);
  if (!p.s) { free(T); return hap_fail(HAP_EINVAL, "out of host memory"); }
  memset(&p.s[0], 0, sizeof(state));
  p.s[0].parent = -1; p.s[0].alive = 1; p.n = 1;
  { double mx = 0.0; for (int j = 0; j < m; ++j) if (rest[0][j] > mx) mx = rest[0][j]; p.s[0].score = mx; }
  int status = HAP_OK;
  if (heap_push(&p, 0)) status = hap_fail(HAP_EINVAL, "out of host memory");
  int best = -1;
  double best_cost = INFINITY;
  int64_t pops = 0;

  while (status == HAP_OK && p.hn > 0) {
    const int qi = heap_pop(&p);
    if (!p.s[qi].alive) continue;
    if (p.s[qi].score >= best_cost) break;          /* no program in the queue can beat the best complete one */
    p.s[qi].alive = 0;
    ++pops;
    for (int ti = 0; ti < nt && status == HAP_OK; ++ti) {
      const state* q = &p.s[qi];
      const triple* t = &T[ti];
      if ((t->pre & ~q->props) || !(t->post & ~q->props)) continue;         /* precondition in P(Q), postcondition not yet */
      const int e = t->ins.tensor;
      if (is_comm(t->ins.kind)) { if (q->communicated >> e & 1) continue; }
      else if (e != q->next) continue;
      if (p.n == p.cap) {
        state* ns = (state*)realloc(p.s, sizeof(state) * (size_t)p.cap * 2);
        if (!ns) { status = hap_fail(HAP_EINVAL, "out of host memory"); break; }
        p.s = ns; p.cap *= 2; q = &p.s[qi];
      }
      state* c = &p.s[p.n];
      *c = *q;
      c->parent = qi; c->ins = t->ins; c->depth = q->depth + 1; c->alive = 1;
      c->props |= t->post;
      if (is_comm(t->ins.kind)) {
        double mx = 0.0;
        for (int j = 0; j < m; ++j) { if (c->busy[j] > mx) mx = c->busy[j]; c->busy[j] = 0.0; }
        c->closed += mx + comm_seconds(graph, &t->ins, m, bmax, net);
        c->communicated |= 1u << e;
      } else {
        for (int j = 0; j < m; ++j) c->busy[j] += instr_flops(graph, &t->ins, ratios[j]) / speed[j];
        c->next = q->next + 1;
        /* properties of tensors whose last consumer is now computed cannot enable anything new (Sec. 4.5) */
        for (int x = 0; x < n_nodes; ++x)
          if (x != loss && lastuse[x] >= 0 && lastuse[x] < c->next) c->props &= ~((uint64_t)0xF << (x * 4));
      }
      const double cost = state_cost(c, m);
      if (c->props & goal) {                          /* complete: loss | All-Reduce */
        if (cost < best_cost) { best_cost = cost; best = p.n; ++p.n; }
        continue;
      }
      double lb = 0.0;
      for (int j = 0; j < m; ++j) { const double v = c->busy[j] + rest[c->next][j]; if (v > lb) lb = v; }
      c->score = c->closed + lb;
      if (c->score >= best_cost) continue;
      /* dominance (lines 9-14 of Fig. "a*"): Qs is at least as good as Q' if it has every property of Q', has used no
       * collective Q' has not, and is no later on any device; then every completion of Q' completes Qs as cheaply */
      int dominated = 0;
      for (int si = 0; si < p.n && !dominated; ++si) {
        const state* s = &p.s[si];
        if (!s->alive || s->next != c->next) continue;
        if ((c->props & ~s->props) || (s->communicated & ~c->communicated) || s->closed > c->closed) continue;
        int ok = 1;
        for (int j = 0; j < m && ok; ++j) ok = s->closed + s->busy[j] <= c->closed + c->busy[j];
        dominated = ok;
      }
      if (dominated) continue;
      for (int si = 0; si < p.n; ++si) {
        state* s = &p.s[si];
        if (!s->alive || s->next != c->next) continue;
        if ((s->props & ~c->props) || (c->communicated & ~s->communicated) || c->closed > s->closed) continue;
        int ok = 1;
        for (int j = 0; j < m && ok; ++j) ok = c->closed + c->busy[j] <= s->closed + s->busy[j];
        if (ok) s->alive = 0;
      }
      const int ci = p.n++;
      if (heap_push(&p, ci)) status = hap_fail(HAP_EINVAL, "out of host memory");
    }
  }
  if (status == HAP_OK && best < 0) status = hap_fail(HAP_EINFEASIBLE, "no program establishes loss | All-Reduce under these rules");
  if (status == HAP_OK) {
    const int len = p.s[best].depth;
    if (len > capacity) status = hap_fail(HAP_EWORKSPACE, "program has %d instructions, room for %d", len, capacity);
    else {
      int i = best;
      for (int k = len - 1; k >= 0; --k) { program[k] = p.s[i].ins; i = p.s[i].parent; }
      *n_instr = len;
      if (seconds) *seconds = best_cost;
      if (expanded) *expanded = pops;
    }
  }
  free(p.s); free(p.heap); free(T);
  return status;
}
