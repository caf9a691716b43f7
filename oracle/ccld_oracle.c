/*
 * CPU oracle of the CCL-D decision analyzer's cross-rank anomaly computation.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, single-threaded
 * statement of what the analyzer computes; tests and the benchmark's CPU
 * baseline call it, the GPU library never does, and the two share no code.
 *
 * Every step below follows the paper's decision analyzer (Section 4.2):
 * metrics are grouped by communicator and by Trace ID (communicator id,
 * operation counter; Section 5.1), each round's per-rank Duration Time
 * (Section 4.1.2) gives T_max and T_min, Eq. 1-3 detect a slow communicator,
 * Eq. 4 attributes it, and the hang rules of Sections 4.2.1 / 4.2.2 raise and
 * classify hang alerts.  The cross-rank arrival/completion statistics (lower
 * median, median absolute deviation, per-rank lag) are the statistical test
 * that stands in for the paper's "theta determined statistically".
 *
 * All arithmetic is 64-bit integer; products are compared in 128 bits, so no
 * ratio is ever materialised.  Medians are found by fully sorting a copy.
 *
 * Pinned by tests/test_oracle_*.py (closed forms of Eq. 1-4, brute force,
 * invariants, injected-fault recovery).  The choices the paper leaves open
 * (segment usability, detection groups by operation type and size class,
 * watermarks under re-analysis, tie rules) are definitions made here and
 * are "parity unpinned" by the paper itself.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_INFLIGHT INT64_MAX
#define ORC_NO_RANK 0xFFFFFFFFll

enum { ORC_OK = 0, ORC_E_UNKNOWN_COMM = -1, ORC_E_RANK_NOT_MEMBER = -2, ORC_E_RANGE = -3,
       ORC_E_DUPLICATE_KEY = -4, ORC_E_SNAPSHOT_GAP = -5, ORC_E_BAD_ARG = -6 };

/* parameter vector (int64 each) */
enum { P_HANG_THRESHOLD_NS, P_TBASE_INIT_NS, P_TBASE_ROUNDS, P_TBASE_WARMUP_NS, P_THETA_NUM, P_THETA_DEN,
       P_ALPHA_NUM, P_BETA_NUM, P_AB_DEN, P_REPEAT_THRESHOLD, P_BARRIER_BYTES, P_KMAD_NUM, P_KMAD_DEN,
       P_LAG_FLOOR_NS, P_STALL_SNAPSHOTS, P_FIFO_DEPTH, P_COUNT };

enum { OP_ALLREDUCE = 0, OP_MAX = 16, CLS_MAX = 64 };

/* segment state bits */
enum { SEG_COMPLETE = 1, SEG_CONSISTENT = 2, SEG_BARRIER = 4, SEG_USABLE = 8 };
enum { FLAG_LATE_ENTER = 1, FLAG_LATE_EXIT = 2 };

/* table layouts: every table is a row-major int64 matrix */
enum { SEG_COMM, SEG_SEQ, SEG_N, SEG_INFLIGHT, SEG_STATE, SEG_OP, SEG_BYTES,
       SEG_ENTER_MIN, SEG_ENTER_MED, SEG_ENTER_MAX, SEG_ENTER_MAD,
       SEG_EXIT_MIN, SEG_EXIT_MED, SEG_EXIT_MAX, SEG_EXIT_MAD,
       SEG_DUR_MIN, SEG_DUR_MAX, SEG_ARGMIN_RANK, SEG_ARGMAX_RANK, SEG_INFLIGHT_ENTER_MIN, SEG_FIRST, SEG_NCOL };
enum { FLG_COMM, FLG_SEQ, FLG_RANK, FLG_KIND, FLG_LAG_ENTER, FLG_LAG_EXIT, FLG_NCOL };
enum { GRP_COMM, GRP_OP, GRP_CLS, GRP_N_USABLE, GRP_RSTAR_SEQ, GRP_TMAX, GRP_TMIN, GRP_TBASE, GRP_STATIC,
       GRP_FROZEN, GRP_M, GRP_SLOW, GRP_CLASS, GRP_ROOT_S1, GRP_ROOT_S2, GRP_REPEATS, GRP_LOCATE, GRP_NCOL };
enum { ALR_COMM, ALR_SEQ, ALR_AGE, ALR_CLASS, ALR_NCAND, ALR_CAND_OFF, ALR_NCOL };
enum { BLM_N_LATE_ENTER, BLM_N_LATE_EXIT, BLM_SUM_LAG_ENTER, BLM_SUM_LAG_EXIT, BLM_N_RECORDS, BLM_NCOL };
enum { REC_LAG_ENTER, REC_LAG_EXIT, REC_FLAG, REC_NCOL };

typedef struct {
  uint32_t n_ranks, n_comms;
  const uint8_t *algo;
  const uint32_t *size, *member_off, *members;
  const int32_t *tree_parent;
} orc_topology;

typedef struct {
  int32_t status;
  uint64_t n, n_seg, n_flag, n_group, n_alert, n_cand, n_ranks;
  uint64_t *perm;     /* [n]  input index of the j-th record in (comm, seq, rank) order */
  int64_t *rec;       /* [n][REC_NCOL]  per sorted record */
  int64_t *seg;       /* [n_seg][SEG_NCOL] */
  int64_t *flag;      /* [n_flag][FLG_NCOL]  ordered by (comm, seq, rank) */
  int64_t *group;     /* [n_group][GRP_NCOL] ordered by (comm, op, cls) */
  int64_t *alert;     /* [n_alert][ALR_NCOL] ordered by (comm, seq) */
  int64_t *cand;      /* [n_cand] candidate ranks of the alerts, ascending per alert */
  int64_t *blame;     /* [n_ranks][BLM_NCOL] */
  int64_t *order;     /* [n_ranks] ranks by (n_flags desc, sum_lag desc, rank asc) */
} orc_window_result;

/* per detection group (communicator, operation, size class): Eq. 1 state and the repetition counter */
typedef struct {
  uint32_t cnt, frozen, repeats, pad;
  int64_t sum, t0, tbase_dyn;
  uint64_t baselined_wm;      /* seq+1 of the last round visited for Eq. 1 (0 = none) */
  uint64_t baseline_last_seq; /* seq of the last round summed into the baseline */
  uint64_t detected_wm;       /* seq+1 of the last round counted as a slow detection */
} orc_group_state;

typedef struct {
  uint32_t n_comms;
  orc_group_state *g;         /* [n_comms][OP_MAX][CLS_MAX] */
  int64_t *rate_root;         /* [n_comms] rank of minimal SendRate / RecvRate from the latest rate pass, or none */
} orc_state;

/* ------------------------------------------------------------------ */
orc_state *orc_state_create(uint32_t n_comms) {
  orc_state *s = (orc_state *)calloc(1, sizeof(orc_state));
  if (!s) return NULL;
  s->n_comms = n_comms;
  s->g = (orc_group_state *)calloc((size_t)n_comms * OP_MAX * CLS_MAX, sizeof(orc_group_state));
  s->rate_root = (int64_t *)malloc(sizeof(int64_t) * (n_comms ? n_comms : 1));
  if (!s->g || !s->rate_root) { free(s->g); free(s->rate_root); free(s); return NULL; }
  for (uint32_t c = 0; c < n_comms; ++c) s->rate_root[c] = ORC_NO_RANK;
  return s;
}
void orc_state_destroy(orc_state *s) { if (s) { free(s->g); free(s->rate_root); free(s); } }

void orc_window_result_free(orc_window_result *r) {
  if (!r) return;
  free(r->perm); free(r->rec); free(r->seg); free(r->flag); free(r->group);
  free(r->alert); free(r->cand); free(r->blame); free(r->order);
  memset(r, 0, sizeof(*r));
}

/* ------------------------------------------------------------------ */
typedef struct {
  const uint32_t *rank, *comm; const uint64_t *seq;
} key_cols;
static key_cols g_kc;   /* comparison context for qsort (the oracle is single-threaded) */

static int cmp_record(const void *pa, const void *pb) {
  uint64_t a = *(const uint64_t *)pa, b = *(const uint64_t *)pb;
  if (g_kc.comm[a] != g_kc.comm[b]) return g_kc.comm[a] < g_kc.comm[b] ? -1 : 1;
  if (g_kc.seq[a] != g_kc.seq[b]) return g_kc.seq[a] < g_kc.seq[b] ? -1 : 1;
  if (g_kc.rank[a] != g_kc.rank[b]) return g_kc.rank[a] < g_kc.rank[b] ? -1 : 1;
  return 0;
}
static int cmp_i64(const void *pa, const void *pb) {
  int64_t a = *(const int64_t *)pa, b = *(const int64_t *)pb;
  return a < b ? -1 : (a > b ? 1 : 0);
}

/* lower median: element floor((n-1)/2) of the ascending order */
static int64_t lower_median(const int64_t *v, size_t n, int64_t *scratch) {
  memcpy(scratch, v, n * sizeof(int64_t));
  qsort(scratch, n, sizeof(int64_t), cmp_i64);
  return scratch[(n - 1) / 2];
}
static int64_t abs_diff(int64_t a, int64_t b) { return a >= b ? a - b : b - a; }

static int is_member(const orc_topology *t, uint32_t comm, uint32_t rank) {
  uint32_t o = t->member_off[comm];
  for (uint32_t i = 0; i < t->size[comm]; ++i) if (t->members[o + i] == rank) return 1;
  return 0;
}
static int floor_log2_u64(uint64_t b) { int c = 0; if (b == 0) b = 1; while (b >>= 1) ++c; return c; }

typedef struct { uint32_t comm, op, cls; uint64_t seq, seg; } grp_item;
static int cmp_grp_item(const void *pa, const void *pb) {
  const grp_item *a = (const grp_item *)pa, *b = (const grp_item *)pb;
  if (a->comm != b->comm) return a->comm < b->comm ? -1 : 1;
  if (a->op != b->op) return a->op < b->op ? -1 : 1;
  if (a->cls != b->cls) return a->cls < b->cls ? -1 : 1;
  if (a->seq != b->seq) return a->seq < b->seq ? -1 : 1;
  return 0;
}

static const int64_t *g_blame;
static int cmp_blame_order(const void *pa, const void *pb) {
  int64_t a = *(const int64_t *)pa, b = *(const int64_t *)pb;
  const int64_t *ba = g_blame + a * BLM_NCOL, *bb = g_blame + b * BLM_NCOL;
  int64_t na = ba[BLM_N_LATE_ENTER] + ba[BLM_N_LATE_EXIT], nb = bb[BLM_N_LATE_ENTER] + bb[BLM_N_LATE_EXIT];
  if (na != nb) return na > nb ? -1 : 1;
  int64_t sa = (int64_t)((uint64_t)ba[BLM_SUM_LAG_ENTER] + (uint64_t)ba[BLM_SUM_LAG_EXIT]);
  int64_t sb = (int64_t)((uint64_t)bb[BLM_SUM_LAG_ENTER] + (uint64_t)bb[BLM_SUM_LAG_EXIT]);
  if (sa != sb) return sa > sb ? -1 : 1;
  return a < b ? -1 : (a > b ? 1 : 0);
}

/* ------------------------------------------------------------------ */
int orc_analyze_window(const int64_t *P, const orc_topology *T, uint64_t n,
                       const uint32_t *rank, const uint32_t *comm, const uint64_t *seq, const uint8_t *op,
                       const uint64_t *bytes, const int64_t *t_enter, const int64_t *t_exit,
                       int64_t now_ns, orc_state *st, orc_window_result *R) {
  memset(R, 0, sizeof(*R));
  R->n = n; R->n_ranks = T->n_ranks;
  if (!st || st->n_comms != T->n_comms || P[P_TBASE_ROUNDS] < 1 || P[P_THETA_DEN] < 1 || P[P_AB_DEN] < 1 ||
      P[P_KMAD_DEN] < 1) { R->status = ORC_E_BAD_ARG; return R->status; }

  /* ---- validation: the status does not depend on the order of the records ---- */
  int bad_comm = 0, bad_member = 0, bad_range = 0;
  for (uint64_t i = 0; i < n; ++i) {
    if (comm[i] >= T->n_comms) { bad_comm = 1; continue; }
    if (rank[i] >= T->n_ranks || !is_member(T, comm[i], rank[i])) bad_member = 1;
    if (op[i] >= OP_MAX || t_enter[i] < 0 || t_enter[i] == ORC_INFLIGHT || t_exit[i] < t_enter[i]) bad_range = 1;
  }
  if (bad_comm) { R->status = ORC_E_UNKNOWN_COMM; return R->status; }
  if (bad_member) { R->status = ORC_E_RANK_NOT_MEMBER; return R->status; }
  if (bad_range) { R->status = ORC_E_RANGE; return R->status; }

  /* ---- group by Trace ID (communicator, operation counter), ranks ascending inside a round ---- */
  uint64_t *perm = (uint64_t *)malloc((n ? n : 1) * sizeof(uint64_t));
  for (uint64_t i = 0; i < n; ++i) perm[i] = i;
  g_kc.rank = rank; g_kc.comm = comm; g_kc.seq = seq;
  qsort(perm, n, sizeof(uint64_t), cmp_record);
  R->perm = perm;
  for (uint64_t j = 1; j < n; ++j)
    if (cmp_record(&perm[j - 1], &perm[j]) == 0) { R->status = ORC_E_DUPLICATE_KEY; return R->status; }

  uint64_t n_seg = 0;
  for (uint64_t j = 0; j < n; ++j)
    if (j == 0 || comm[perm[j]] != comm[perm[j - 1]] || seq[perm[j]] != seq[perm[j - 1]]) ++n_seg;
  R->n_seg = n_seg;
  R->seg = (int64_t *)calloc((n_seg ? n_seg : 1) * SEG_NCOL, sizeof(int64_t));
  R->rec = (int64_t *)calloc((n ? n : 1) * REC_NCOL, sizeof(int64_t));
  R->blame = (int64_t *)calloc((size_t)(T->n_ranks ? T->n_ranks : 1) * BLM_NCOL, sizeof(int64_t));
  R->order = (int64_t *)calloc(T->n_ranks ? T->n_ranks : 1, sizeof(int64_t));
  uint64_t *seg_first = (uint64_t *)malloc((n_seg + 1) * sizeof(uint64_t));

  uint32_t max_size = 1;
  for (uint64_t j = 0, s = 0; j < n; ++j)
    if (j == 0 || comm[perm[j]] != comm[perm[j - 1]] || seq[perm[j]] != seq[perm[j - 1]]) seg_first[s++] = j;
  seg_first[n_seg] = n;
  for (uint64_t s = 0; s < n_seg; ++s)
    if (seg_first[s + 1] - seg_first[s] > max_size) max_size = (uint32_t)(seg_first[s + 1] - seg_first[s]);
  int64_t *va = (int64_t *)malloc(max_size * sizeof(int64_t));
  int64_t *vb = (int64_t *)malloc(max_size * sizeof(int64_t));
  int64_t *vs = (int64_t *)malloc(max_size * sizeof(int64_t));

  uint64_t n_flag = 0, n_alert = 0, n_cand = 0;
  /* ---- per-round state and statistics ---- */
  for (uint64_t s = 0; s < n_seg; ++s) {
    int64_t *S = R->seg + s * SEG_NCOL;
    uint64_t a = seg_first[s], b = seg_first[s + 1];
    uint64_t i0 = perm[a];
    uint32_t c = comm[i0];
    uint64_t nn = b - a, n_infl = 0, n_done = 0;
    int consistent = 1;
    int64_t infl_enter_min = ORC_INFLIGHT;
    for (uint64_t j = a; j < b; ++j) {
      uint64_t i = perm[j];
      if (op[i] != op[i0] || bytes[i] != bytes[i0]) consistent = 0;
      if (t_exit[i] == ORC_INFLIGHT) { ++n_infl; if (t_enter[i] < infl_enter_min) infl_enter_min = t_enter[i]; }
    }
    int complete = (nn == T->size[c]) && n_infl == 0;
    int barrier = (op[i0] == OP_ALLREDUCE) && (bytes[i0] < (uint64_t)P[P_BARRIER_BYTES]);
    int usable = complete && consistent && !barrier;
    S[SEG_COMM] = c; S[SEG_SEQ] = (int64_t)seq[i0]; S[SEG_N] = (int64_t)nn; S[SEG_INFLIGHT] = (int64_t)n_infl;
    S[SEG_STATE] = (complete ? SEG_COMPLETE : 0) | (consistent ? SEG_CONSISTENT : 0) |
                   (barrier ? SEG_BARRIER : 0) | (usable ? SEG_USABLE : 0);
    S[SEG_OP] = op[i0]; S[SEG_BYTES] = (int64_t)bytes[i0];
    S[SEG_INFLIGHT_ENTER_MIN] = infl_enter_min;
    S[SEG_FIRST] = (int64_t)a;   /* position of the round's first record in the sorted order */
    S[SEG_ARGMIN_RANK] = ORC_NO_RANK; S[SEG_ARGMAX_RANK] = ORC_NO_RANK;
    /* statistics over the records of this round that have completed */
    int64_t dmin = 0, dmax = 0;
    for (uint64_t j = a; j < b; ++j) {
      uint64_t i = perm[j];
      if (t_exit[i] == ORC_INFLIGHT) continue;
      va[n_done] = t_enter[i]; vb[n_done] = t_exit[i];
      int64_t d = t_exit[i] - t_enter[i];               /* Duration Time of this rank */
      if (n_done == 0 || d < dmin) { dmin = d; S[SEG_ARGMIN_RANK] = rank[i]; }   /* tie -> smallest rank */
      if (n_done == 0 || d > dmax) { dmax = d; S[SEG_ARGMAX_RANK] = rank[i]; }
      ++n_done;
    }
    if (n_done > 0) {
      int64_t emin = va[0], emax = va[0], xmin = vb[0], xmax = vb[0];
      for (uint64_t k = 1; k < n_done; ++k) {
        if (va[k] < emin) emin = va[k];
        if (va[k] > emax) emax = va[k];
        if (vb[k] < xmin) xmin = vb[k];
        if (vb[k] > xmax) xmax = vb[k];
      }
      int64_t emed = lower_median(va, n_done, vs), xmed = lower_median(vb, n_done, vs);
      for (uint64_t k = 0; k < n_done; ++k) { va[k] = abs_diff(va[k], emed); vb[k] = abs_diff(vb[k], xmed); }
      int64_t emad = lower_median(va, n_done, vs), xmad = lower_median(vb, n_done, vs);
      S[SEG_ENTER_MIN] = emin; S[SEG_ENTER_MED] = emed; S[SEG_ENTER_MAX] = emax; S[SEG_ENTER_MAD] = emad;
      S[SEG_EXIT_MIN] = xmin; S[SEG_EXIT_MED] = xmed; S[SEG_EXIT_MAX] = xmax; S[SEG_EXIT_MAD] = xmad;
      S[SEG_DUR_MIN] = dmin; S[SEG_DUR_MAX] = dmax;
    }
    /* per-rank lag and slow-rank flags, on usable rounds only */
    if (usable) {
      for (uint64_t j = a; j < b; ++j) {
        uint64_t i = perm[j];
        int64_t le = t_enter[i] - S[SEG_ENTER_MED], lx = t_exit[i] - S[SEG_EXIT_MED];
        int f = 0;
        if (le > P[P_LAG_FLOOR_NS] &&
            (__int128)le * (__int128)P[P_KMAD_DEN] > (__int128)P[P_KMAD_NUM] * (__int128)S[SEG_ENTER_MAD])
          f |= FLAG_LATE_ENTER;
        if (lx > P[P_LAG_FLOOR_NS] &&
            (__int128)lx * (__int128)P[P_KMAD_DEN] > (__int128)P[P_KMAD_NUM] * (__int128)S[SEG_EXIT_MAD])
          f |= FLAG_LATE_EXIT;
        R->rec[j * REC_NCOL + REC_LAG_ENTER] = le;
        R->rec[j * REC_NCOL + REC_LAG_EXIT] = lx;
        R->rec[j * REC_NCOL + REC_FLAG] = f;
        if (f) ++n_flag;
      }
    }
    /* hang alert: an operation still in flight for longer than the threshold, barriers excepted */
    if (n_infl > 0 && !barrier && now_ns - infl_enter_min > P[P_HANG_THRESHOLD_NS]) {
      ++n_alert;
      if (nn < T->size[c]) n_cand += T->size[c] - nn; else n_cand += n_done;
    }
  }
  for (uint64_t i = 0; i < n; ++i) R->blame[(size_t)rank[i] * BLM_NCOL + BLM_N_RECORDS] += 1;

  /* ---- flag list (already in (comm, seq, rank) order) and per-rank blame ---- */
  R->n_flag = n_flag;
  R->flag = (int64_t *)calloc((n_flag ? n_flag : 1) * FLG_NCOL, sizeof(int64_t));
  for (uint64_t j = 0, k = 0; j < n; ++j) {
    int64_t f = R->rec[j * REC_NCOL + REC_FLAG];
    if (!f) continue;
    uint64_t i = perm[j];
    int64_t *F = R->flag + k * FLG_NCOL; ++k;
    F[FLG_COMM] = comm[i]; F[FLG_SEQ] = (int64_t)seq[i]; F[FLG_RANK] = rank[i]; F[FLG_KIND] = f;
    F[FLG_LAG_ENTER] = R->rec[j * REC_NCOL + REC_LAG_ENTER];
    F[FLG_LAG_EXIT] = R->rec[j * REC_NCOL + REC_LAG_EXIT];
    int64_t *B = R->blame + (size_t)rank[i] * BLM_NCOL;
    if (f & FLAG_LATE_ENTER) {
      B[BLM_N_LATE_ENTER] += 1;
      B[BLM_SUM_LAG_ENTER] = (int64_t)((uint64_t)B[BLM_SUM_LAG_ENTER] + (uint64_t)F[FLG_LAG_ENTER]);
    }
    if (f & FLAG_LATE_EXIT) {
      B[BLM_N_LATE_EXIT] += 1;
      B[BLM_SUM_LAG_EXIT] = (int64_t)((uint64_t)B[BLM_SUM_LAG_EXIT] + (uint64_t)F[FLG_LAG_EXIT]);
    }
  }
  for (uint32_t r = 0; r < T->n_ranks; ++r) R->order[r] = r;
  g_blame = R->blame;
  qsort(R->order, T->n_ranks, sizeof(int64_t), cmp_blame_order);

  /* ---- hang alerts with the first two branches of the hang decision tree ---- */
  R->n_alert = n_alert; R->n_cand = n_cand;
  R->alert = (int64_t *)calloc((n_alert ? n_alert : 1) * ALR_NCOL, sizeof(int64_t));
  R->cand = (int64_t *)calloc(n_cand ? n_cand : 1, sizeof(int64_t));
  {
    uint64_t ka = 0, kc = 0;
    int64_t *tmp = (int64_t *)malloc((size_t)(T->n_ranks ? T->n_ranks : 1) * sizeof(int64_t));
    for (uint64_t s = 0; s < n_seg; ++s) {
      int64_t *S = R->seg + s * SEG_NCOL;
      if (!(S[SEG_INFLIGHT] > 0 && !(S[SEG_STATE] & SEG_BARRIER) &&
            now_ns - S[SEG_INFLIGHT_ENTER_MIN] > P[P_HANG_THRESHOLD_NS])) continue;
      uint64_t a = seg_first[s], b = seg_first[s + 1];
      uint32_t c = (uint32_t)S[SEG_COMM];
      int64_t *A = R->alert + ka * ALR_NCOL; ++ka;
      A[ALR_COMM] = c; A[ALR_SEQ] = S[SEG_SEQ]; A[ALR_AGE] = now_ns - S[SEG_INFLIGHT_ENTER_MIN];
      A[ALR_CAND_OFF] = (int64_t)kc;
      uint64_t m = 0;
      if ((uint64_t)S[SEG_N] < T->size[c]) {
        /* a member with no record for this operation counter has not entered: Not-Entered-Hang */
        A[ALR_CLASS] = 1;
        for (uint32_t q = 0; q < T->size[c]; ++q) {
          uint32_t r = T->members[T->member_off[c] + q];
          int present = 0;
          for (uint64_t j = a; j < b; ++j) if (rank[perm[j]] == r) { present = 1; break; }
          if (!present) tmp[m++] = r;
        }
      } else if ((uint64_t)S[SEG_INFLIGHT] < (uint64_t)S[SEG_N]) {
        /* everyone entered and some ranks are not hung: Inconsistent-Hang, the non-hang ranks are the root */
        A[ALR_CLASS] = 2;
        for (uint64_t j = a; j < b; ++j) if (t_exit[perm[j]] != ORC_INFLIGHT) tmp[m++] = rank[perm[j]];
      } else {
        A[ALR_CLASS] = 3;   /* all ranks hung: needs the Send/Recv counters (orc_locate_hang) */
      }
      qsort(tmp, m, sizeof(int64_t), cmp_i64);
      for (uint64_t q = 0; q < m; ++q) R->cand[kc++] = tmp[q];
      A[ALR_NCAND] = (int64_t)m;
    }
    free(tmp);
  }

  /* ---- slow detection and location per detection group (Eq. 1-4) ---- */
  uint64_t n_us = 0;
  for (uint64_t s = 0; s < n_seg; ++s) if (R->seg[s * SEG_NCOL + SEG_STATE] & SEG_USABLE) ++n_us;
  grp_item *items = (grp_item *)malloc((n_us ? n_us : 1) * sizeof(grp_item));
  for (uint64_t s = 0, k = 0; s < n_seg; ++s) {
    const int64_t *S = R->seg + s * SEG_NCOL;
    if (!(S[SEG_STATE] & SEG_USABLE)) continue;
    items[k].comm = (uint32_t)S[SEG_COMM]; items[k].op = (uint32_t)S[SEG_OP];
    items[k].cls = (uint32_t)floor_log2_u64((uint64_t)S[SEG_BYTES]);
    items[k].seq = (uint64_t)S[SEG_SEQ]; items[k].seg = s; ++k;
  }
  qsort(items, n_us, sizeof(grp_item), cmp_grp_item);
  uint64_t n_group = 0;
  for (uint64_t k = 0; k < n_us; ++k)
    if (k == 0 || items[k].comm != items[k - 1].comm || items[k].op != items[k - 1].op ||
        items[k].cls != items[k - 1].cls) ++n_group;
  R->n_group = n_group;
  R->group = (int64_t *)calloc((n_group ? n_group : 1) * GRP_NCOL, sizeof(int64_t));
  for (uint64_t k0 = 0, gi = 0; k0 < n_us; ++gi) {
    uint64_t k1 = k0 + 1;
    while (k1 < n_us && items[k1].comm == items[k0].comm && items[k1].op == items[k0].op &&
           items[k1].cls == items[k0].cls) ++k1;
    orc_group_state *G = st->g + ((size_t)items[k0].comm * OP_MAX + items[k0].op) * CLS_MAX + items[k0].cls;
    /* Eq. 1: average T_max of the first m rounds; m = min(tbase_rounds, rounds inside the warm-up span) */
    for (uint64_t k = k0; k < k1; ++k) {
      const int64_t *S = R->seg + items[k].seg * SEG_NCOL;
      if (items[k].seq + 1 <= G->baselined_wm) continue;
      if (!G->frozen) {
        if (G->cnt == 0) G->t0 = S[SEG_ENTER_MIN];
        if (G->cnt < (uint64_t)P[P_TBASE_ROUNDS] && S[SEG_ENTER_MIN] - G->t0 <= P[P_TBASE_WARMUP_NS]) {
          G->sum += S[SEG_DUR_MAX]; G->cnt += 1; G->baseline_last_seq = items[k].seq;
        } else {
          G->frozen = 1; G->tbase_dyn = G->sum / (int64_t)G->cnt;
        }
      }
      G->baselined_wm = items[k].seq + 1;
    }
    /* Eq. 2: the round of this window with the largest intra-round range (tie -> smallest seq) */
    uint64_t kstar = k0;
    int64_t best = 0;
    for (uint64_t k = k0; k < k1; ++k) {
      const int64_t *S = R->seg + items[k].seg * SEG_NCOL;
      int64_t range = S[SEG_DUR_MAX] - S[SEG_DUR_MIN];
      if (k == k0 || range > best) { best = range; kstar = k; }
    }
    const int64_t *Sx = R->seg + items[kstar].seg * SEG_NCOL;
    int64_t tmax = Sx[SEG_DUR_MAX], tmin = Sx[SEG_DUR_MIN];
    /* Eq. 1 case split: the configured baseline applies while the round is among the first m */
    int dynamic = G->frozen && items[kstar].seq > G->baseline_last_seq;
    int64_t tbase = dynamic ? G->tbase_dyn : P[P_TBASE_INIT_NS];
    /* Eq. 3: R = (T_max - T_base)/T_base > theta, cross-multiplied */
    int slow = (__int128)(tmax - tbase) * (__int128)P[P_THETA_DEN] > (__int128)P[P_THETA_NUM] * (__int128)tbase;
    int cls = 0;
    int64_t root1 = ORC_NO_RANK;
    if (slow) {
      /* Eq. 4: P = (T_max - T_min)/(T_max - T_base); P > beta: computation-slow, P < alpha: communication-slow */
      __int128 num = (__int128)(tmax - tmin) * (__int128)P[P_AB_DEN];
      __int128 den = (__int128)(tmax - tbase);
      if (num > (__int128)P[P_BETA_NUM] * den) cls = 1;
      else if (num < (__int128)P[P_ALPHA_NUM] * den) cls = 2;
      else cls = 3;
      if (cls != 2) root1 = Sx[SEG_ARGMIN_RANK];   /* the rank with minimal communication time */
      if (items[kstar].seq + 1 > G->detected_wm) { G->repeats += 1; G->detected_wm = items[kstar].seq + 1; }
    }
    int64_t *O = R->group + gi * GRP_NCOL;
    O[GRP_COMM] = items[k0].comm; O[GRP_OP] = items[k0].op; O[GRP_CLS] = items[k0].cls;
    O[GRP_N_USABLE] = (int64_t)(k1 - k0); O[GRP_RSTAR_SEQ] = (int64_t)items[kstar].seq;
    O[GRP_TMAX] = tmax; O[GRP_TMIN] = tmin; O[GRP_TBASE] = tbase; O[GRP_STATIC] = !dynamic;
    O[GRP_FROZEN] = G->frozen; O[GRP_M] = G->cnt; O[GRP_SLOW] = slow; O[GRP_CLASS] = cls;
    /* communication-slow (and the communication half of a mixed slowdown): the rank of minimal
       SendRate / RecvRate in this communicator, known once a rate pass has run (Section 4.2.1, Eq. 4) */
    O[GRP_ROOT_S1] = root1;
    O[GRP_ROOT_S2] = (cls == 2 || cls == 3) ? st->rate_root[items[k0].comm] : ORC_NO_RANK;
    O[GRP_REPEATS] = G->repeats;
    O[GRP_LOCATE] = slow && G->repeats >= (uint64_t)P[P_REPEAT_THRESHOLD];
    k0 = k1;
  }
  free(items); free(seg_first); free(va); free(vb); free(vs);
  R->status = ORC_OK;
  return ORC_OK;
}

/* ==================================================================================================
 * Root cause and secondary effects among the late-entry flags (Section 4.2.2, first paragraph: an
 * anomaly may propagate across ranks, and the location step separates the rank that triggered it
 * from the ranks that merely pass it on).
 *
 * A rank enters a collective late either because it is slow itself or because the operation it ran
 * just before ended late, which happens when another member of that operation arrived late there.
 * For a late-entry flag F of rank r:
 *   previous operation of r = r's completed record with the largest t_exit <= t_enter(F) (r's own
 *     clock on both sides; ties: larger t_enter, then larger communicator, then larger counter;
 *     the record of F itself is left out);
 *   the member that ended that operation late = among its late-entry flags the one with the largest
 *     lag (ties: smallest rank);
 *   if there is such a member, F is a consequence of that member's late arrival and that flag is its
 *     parent (when the member is r itself the chain goes on through r's own earlier flag); if the
 *     previous operation has no late entry, F is a root flag: r is late of its own.
 * Following parents ends at a root flag (a parent's collective ended before the child was entered);
 * the output gives, per flag, its parent, its root, the root's rank and the depth, and per rank the
 * numbers of its late entries without and with a parent and the number of late entries, of any rank,
 * whose chain starts at one of its root flags.  Late-exit flags are a rank's own transfer and have no
 * parent.  These rules are a reading made here ("parity unpinned" by the paper); the
 * tests pin them on hand-built chains.
 * ================================================================================================== */
enum { CHN_PARENT, CHN_ROOT, CHN_ROOT_RANK, CHN_DEPTH, CHN_NCOL };
enum { CHR_ROOT_ENTRIES, CHR_SECONDARY_ENTRIES, CHR_CAUSED, CHR_NCOL };

int orc_flag_chains(uint64_t n, const uint32_t *rank, const uint32_t *comm, const uint64_t *seq,
                    const int64_t *t_enter, const int64_t *t_exit, uint64_t n_flag, const int64_t *flag,
                    uint32_t n_ranks, int64_t *chain, int64_t *per_rank) {
  for (uint64_t k = 0; k < n_flag; ++k) {
    const int64_t *F = flag + k * FLG_NCOL;
    int64_t *C = chain + k * CHN_NCOL;
    C[CHN_PARENT] = -1; C[CHN_ROOT] = (int64_t)k; C[CHN_ROOT_RANK] = F[FLG_RANK]; C[CHN_DEPTH] = 0;
    if (!(F[FLG_KIND] & FLAG_LATE_ENTER)) continue;
    /* the flag's own record */
    uint64_t self = n;
    for (uint64_t i = 0; i < n; ++i)
      if (rank[i] == (uint32_t)F[FLG_RANK] && comm[i] == (uint32_t)F[FLG_COMM] && seq[i] == (uint64_t)F[FLG_SEQ]) { self = i; break; }
    if (self == n) return ORC_E_BAD_ARG;
    /* the operation this rank ran just before */
    uint64_t prev = n;
    for (uint64_t i = 0; i < n; ++i) {
      if (i == self || rank[i] != rank[self] || t_exit[i] == ORC_INFLIGHT || t_exit[i] > t_enter[self]) continue;
      if (prev == n) { prev = i; continue; }
      if (t_exit[i] != t_exit[prev]) { if (t_exit[i] > t_exit[prev]) prev = i; continue; }
      if (t_enter[i] != t_enter[prev]) { if (t_enter[i] > t_enter[prev]) prev = i; continue; }
      if (comm[i] != comm[prev]) { if (comm[i] > comm[prev]) prev = i; continue; }
      if (seq[i] > seq[prev]) prev = i;
    }
    if (prev == n) continue;
    /* who ended it late */
    int64_t best = -1;
    for (uint64_t q = 0; q < n_flag; ++q) {
      const int64_t *Q = flag + q * FLG_NCOL;
      if (Q[FLG_COMM] != (int64_t)comm[prev] || Q[FLG_SEQ] != (int64_t)seq[prev] || !(Q[FLG_KIND] & FLAG_LATE_ENTER)) continue;
      if (best < 0 || Q[FLG_LAG_ENTER] > flag[best * FLG_NCOL + FLG_LAG_ENTER] ||
          (Q[FLG_LAG_ENTER] == flag[best * FLG_NCOL + FLG_LAG_ENTER] && Q[FLG_RANK] < flag[best * FLG_NCOL + FLG_RANK]))
        best = (int64_t)q;
    }
    if (best >= 0) C[CHN_PARENT] = best;
  }
  for (uint64_t k = 0; k < n_flag; ++k) {
    int64_t *C = chain + k * CHN_NCOL;
    int64_t cur = (int64_t)k, depth = 0;
    while (chain[cur * CHN_NCOL + CHN_PARENT] >= 0) {
      cur = chain[cur * CHN_NCOL + CHN_PARENT];
      if (++depth > (int64_t)n_flag) return ORC_E_BAD_ARG;      /* cannot happen: parents end earlier */
    }
    C[CHN_ROOT] = cur; C[CHN_ROOT_RANK] = flag[cur * FLG_NCOL + FLG_RANK]; C[CHN_DEPTH] = depth;
  }
  for (uint64_t i = 0; i < (uint64_t)n_ranks * CHR_NCOL; ++i) per_rank[i] = 0;
  for (uint64_t k = 0; k < n_flag; ++k) {
    const int64_t *F = flag + k * FLG_NCOL;
    if (!(F[FLG_KIND] & FLAG_LATE_ENTER)) continue;
    per_rank[F[FLG_RANK] * CHR_NCOL + (chain[k * CHN_NCOL + CHN_PARENT] < 0 ? CHR_ROOT_ENTRIES : CHR_SECONDARY_ENTRIES)] += 1;
    per_rank[chain[k * CHN_NCOL + CHN_ROOT_RANK] * CHR_NCOL + CHR_CAUSED] += 1;
  }
  return ORC_OK;
}

/* ==================================================================================================
 * Hang location from progress-counter snapshots (Section 4.2.2, hang decision tree; Section 4.1.2,
 * SendCount / RecvCount per channel; Section 4.2.1, ring vs tree comparison groups).
 *
 * Rows: one per (snapshot, rank, communicator, channel) with the operation counter the counters
 * describe and the chunks sent / received so far.  Every cell of the grid
 * [0, n_snap) x members x [0, n_ch) must be present exactly once.
 *
 * The three questions of the paper's tree are asked per communicator:
 *   a rank whose operation counter lags has not entered        -> Not-Entered-Hang, that rank
 *   all entered, some ranks still progressing ("non-hang")     -> Inconsistent-Hang, those ranks
 *   all entered, all hung                                      -> Hardware-Fault, the rank with the
 *                                                                 fewest SendCount/RecvCount
 * The operational definitions below (stall test over stall_snapshots snapshots, idle test, ring
 * wait-for edges with a FIFO depth, the filter for ranks that are blocked inside another hung
 * communicator) are readings made here and are "parity unpinned" by the paper; the tests pin
 * them by brute force on small rings and by the recovery of injected roots.
 * ================================================================================================== */
enum { PAIR_RANK, PAIR_COMM, PAIR_STALLED, PAIR_ENTERED, PAIR_SEQ, PAIR_SENT, PAIR_RECV, PAIR_WAITS_ON,
       PAIR_HOPS, PAIR_ONSET, PAIR_NCOL };
enum { HC_COMM, HC_HUNG, HC_CLASS, HC_SEQ_MAX, HC_ROOT_BY_COUNT, HC_NCAND, HC_NCOL };
enum { ROOT_RANK, ROOT_COMM, ROOT_CLASS, ROOT_NCOL };

typedef struct {
  int32_t status;
  uint64_t n_root, n_pair, n_comm;
  int64_t *root;   /* [n_root][ROOT_NCOL] ordered by (rank, comm) */
  int64_t *pair;   /* [n_pair][PAIR_NCOL] one row per member slot of every communicator, in table order */
  int64_t *comm;   /* [n_comm][HC_NCOL]   one row per communicator */
} orc_hang_result;

void orc_hang_result_free(orc_hang_result *r) {
  if (!r) return;
  free(r->root); free(r->pair); free(r->comm);
  memset(r, 0, sizeof(*r));
}

typedef struct { uint64_t seq; uint32_t sent, recv; } cell_t;

static int cmp_root(const void *pa, const void *pb) {
  const int64_t *a = (const int64_t *)pa, *b = (const int64_t *)pb;
  if (a[ROOT_RANK] != b[ROOT_RANK]) return a[ROOT_RANK] < b[ROOT_RANK] ? -1 : 1;
  if (a[ROOT_COMM] != b[ROOT_COMM]) return a[ROOT_COMM] < b[ROOT_COMM] ? -1 : 1;
  return 0;
}

/* Validates the snapshot rows and places every row in its cell [pair][channel][snapshot], where
 * pair = the member's position in the communicator table.  Returns ORC_OK and the cell array (the
 * caller frees it), or the status of the first failing check in the order unknown communicator,
 * non-member, range, duplicate, gap. */
static int place_cells(const orc_topology *T, uint64_t n_rows, uint32_t n_snap, uint32_t n_ch,
                       const uint32_t *snap, const uint32_t *rank, const uint32_t *comm, const uint32_t *channel,
                       const uint64_t *seq_posted, const uint32_t *chunks_sent, const uint32_t *chunks_recv,
                       uint64_t *n_pair_out, cell_t **cell_out) {
  *cell_out = NULL;
  if (n_snap == 0 || n_ch == 0) return ORC_E_BAD_ARG;
  uint64_t n_pair = 0;
  for (uint32_t c = 0; c < T->n_comms; ++c) n_pair += T->size[c];
  *n_pair_out = n_pair;
  const uint64_t n_cell = n_pair * n_ch * n_snap;
  int bad_comm = 0, bad_member = 0, bad_range = 0;
  for (uint64_t i = 0; i < n_rows; ++i) {
    if (comm[i] >= T->n_comms) { bad_comm = 1; continue; }
    if (rank[i] >= T->n_ranks || !is_member(T, comm[i], rank[i])) bad_member = 1;
    if (snap[i] >= n_snap || channel[i] >= n_ch) bad_range = 1;
  }
  if (bad_comm) return ORC_E_UNKNOWN_COMM;
  if (bad_member) return ORC_E_RANK_NOT_MEMBER;
  if (bad_range) return ORC_E_RANGE;
  cell_t *cell = (cell_t *)calloc(n_cell ? n_cell : 1, sizeof(cell_t));
  uint8_t *seen = (uint8_t *)calloc(n_cell ? n_cell : 1, 1);
  int dup = 0, gap = 0;
  for (uint64_t i = 0; i < n_rows; ++i) {
    uint32_t c = comm[i], slot = 0;
    while (T->members[T->member_off[c] + slot] != rank[i]) ++slot;
    uint64_t k = (((uint64_t)T->member_off[c] + slot) * n_ch + channel[i]) * n_snap + snap[i];
    if (seen[k]) dup = 1;
    seen[k] = 1;
    cell[k].seq = seq_posted[i]; cell[k].sent = chunks_sent[i]; cell[k].recv = chunks_recv[i];
  }
  for (uint64_t k = 0; k < n_cell; ++k) if (!seen[k]) gap = 1;
  free(seen);
  if (dup) { free(cell); return ORC_E_DUPLICATE_KEY; }
  if (gap) { free(cell); return ORC_E_SNAPSHOT_GAP; }
  *cell_out = cell;
  return ORC_OK;
}

int orc_locate_hang(const int64_t *P, const orc_topology *T, uint64_t n_rows, uint32_t n_snap, uint32_t n_ch,
                    const uint32_t *snap, const uint32_t *rank, const uint32_t *comm, const uint32_t *channel,
                    const uint64_t *seq_posted, const uint32_t *chunks_sent, const uint32_t *chunks_recv,
                    orc_hang_result *R) {
  memset(R, 0, sizeof(*R));
  uint64_t n_pair = 0;
  cell_t *cell = NULL;
  R->status = place_cells(T, n_rows, n_snap, n_ch, snap, rank, comm, channel, seq_posted, chunks_sent, chunks_recv,
                          &n_pair, &cell);
  if (R->status != ORC_OK) return R->status;

  const uint32_t L = n_snap - 1;
  const int64_t W = P[P_STALL_SNAPSHOTS];
  const int can_stall = W >= 0 && (int64_t)L >= W;     /* too few snapshots: nothing can be called stalled */

  R->n_pair = n_pair; R->n_comm = T->n_comms;
  R->pair = (int64_t *)calloc((n_pair ? n_pair : 1) * PAIR_NCOL, sizeof(int64_t));
  R->comm = (int64_t *)calloc((size_t)T->n_comms * HC_NCOL, sizeof(int64_t));

  /* ---- per (rank, communicator): stalled, operation counter, chunk totals, onset ---- */
  for (uint32_t c = 0; c < T->n_comms; ++c) {
    for (uint32_t q = 0; q < T->size[c]; ++q) {
      uint64_t p = (uint64_t)T->member_off[c] + q;
      int64_t *Q = R->pair + p * PAIR_NCOL;
      int stalled = can_stall;
      uint64_t seq = 0, S = 0, Rv = 0;
      uint32_t onset = 0;
      for (uint32_t ch = 0; ch < n_ch; ++ch) {
        const cell_t *s = cell + (p * n_ch + ch) * n_snap;
        if (can_stall) {
          const cell_t *o = s + (L - (uint32_t)W);
          if (!(o->seq == s[L].seq && o->sent == s[L].sent && o->recv == s[L].recv)) stalled = 0;
        }
        uint32_t on = L;       /* smallest snapshot from which this channel's state stays constant */
        while (on > 0 && s[on - 1].seq == s[L].seq && s[on - 1].sent == s[L].sent && s[on - 1].recv == s[L].recv) --on;
        if (on > onset) onset = on;
        if (s[L].seq > seq) seq = s[L].seq;
        S += s[L].sent; Rv += s[L].recv;
      }
      Q[PAIR_RANK] = T->members[p]; Q[PAIR_COMM] = c; Q[PAIR_STALLED] = stalled; Q[PAIR_SEQ] = (int64_t)seq;
      Q[PAIR_SENT] = (int64_t)S; Q[PAIR_RECV] = (int64_t)Rv; Q[PAIR_WAITS_ON] = ORC_NO_RANK; Q[PAIR_HOPS] = -1;
      Q[PAIR_ONSET] = onset;
    }
  }
  free(cell);

  /* ---- per communicator: entered, idle test, the decision tree, wait-for edges ---- */
  uint8_t *is_cand = (uint8_t *)calloc(n_pair ? n_pair : 1, 1);
  for (uint32_t c = 0; c < T->n_comms; ++c) {
    const uint32_t n = T->size[c], off = T->member_off[c];
    int64_t *H = R->comm + (size_t)c * HC_NCOL;
    int64_t *Q = R->pair + (uint64_t)off * PAIR_NCOL;
#define PQ(q, col) Q[(uint64_t)(q) * PAIR_NCOL + (col)]
    uint64_t seq_max = 0;
    for (uint32_t q = 0; q < n; ++q) if ((uint64_t)PQ(q, PAIR_SEQ) > seq_max) seq_max = (uint64_t)PQ(q, PAIR_SEQ);
    int all_entered = 1, any_stalled = 0, all_stalled = 1;
    for (uint32_t q = 0; q < n; ++q) {
      PQ(q, PAIR_ENTERED) = ((uint64_t)PQ(q, PAIR_SEQ) == seq_max);
      if (!PQ(q, PAIR_ENTERED)) all_entered = 0;
      if (PQ(q, PAIR_STALLED)) any_stalled = 1; else all_stalled = 0;
    }
    /* a completed collective leaves comparable ranks with identical counts: the whole ring, or each
       layer of the tree */
    int *depth = (int *)calloc(n, sizeof(int));
    if (T->algo[c] == 1 && T->tree_parent)
      for (uint32_t q = 0; q < n; ++q) { int32_t par = T->tree_parent[off + q]; depth[q] = par < 0 ? 0 : depth[par] + 1; }
    int idle_ok = all_entered;
    for (uint32_t q = 0; q < n && idle_ok; ++q)
      for (uint32_t r2 = 0; r2 < q; ++r2)
        if (depth[r2] == depth[q]) {
          if (PQ(r2, PAIR_SENT) != PQ(q, PAIR_SENT) || PQ(r2, PAIR_RECV) != PQ(q, PAIR_RECV)) idle_ok = 0;
          break;      /* comparing with the first member of the layer is enough */
        }
    const int hung = !idle_ok && any_stalled;
    /* the rank with the fewest SendCount/RecvCount: minimal S+R, then minimal R, then minimal rank */
    uint32_t best = 0;
    for (uint32_t q = 1; q < n; ++q) {
      int64_t a = PQ(q, PAIR_SENT) + PQ(q, PAIR_RECV), b = PQ(best, PAIR_SENT) + PQ(best, PAIR_RECV);
      if (a < b || (a == b && (PQ(q, PAIR_RECV) < PQ(best, PAIR_RECV) ||
                               (PQ(q, PAIR_RECV) == PQ(best, PAIR_RECV) && PQ(q, PAIR_RANK) < PQ(best, PAIR_RANK)))))
        best = q;
    }
    H[HC_COMM] = c; H[HC_HUNG] = hung; H[HC_SEQ_MAX] = (int64_t)seq_max;
    H[HC_ROOT_BY_COUNT] = hung ? PQ(best, PAIR_RANK) : ORC_NO_RANK; H[HC_CLASS] = 0;
    if (hung) {
      if (!all_entered) {
        H[HC_CLASS] = 1;
        for (uint32_t q = 0; q < n; ++q) if (!PQ(q, PAIR_ENTERED)) is_cand[off + q] = 1;
      } else if (!all_stalled) {
        H[HC_CLASS] = 2;
        for (uint32_t q = 0; q < n; ++q) if (!PQ(q, PAIR_STALLED)) is_cand[off + q] = 1;
      } else {
        H[HC_CLASS] = 3;
        uint32_t n_c = 0;
        if (T->algo[c] == 0) {
          /* ring: a rank that has consumed everything its predecessor sent waits on the predecessor;
             a rank whose successor has fifo_depth unconsumed chunks waits on the successor */
          for (uint32_t q = 0; q < n; ++q) {
            uint32_t pred = (q + n - 1) % n, succ = (q + 1) % n;
            if (n > 1 && PQ(q, PAIR_RECV) >= PQ(pred, PAIR_SENT)) PQ(q, PAIR_WAITS_ON) = PQ(pred, PAIR_RANK);
            else if (n > 1 && PQ(q, PAIR_SENT) - PQ(succ, PAIR_RECV) >= P[P_FIFO_DEPTH]) PQ(q, PAIR_WAITS_ON) = PQ(succ, PAIR_RANK);
            else { is_cand[off + q] = 1; ++n_c; }
          }
        } else {
          /* tree: inside a layer, the ranks furthest behind the layer's best */
          int64_t worst = 0;
          int64_t *def = (int64_t *)calloc(n, sizeof(int64_t));
          for (uint32_t q = 0; q < n; ++q) {
            int64_t mx = 0;
            for (uint32_t r2 = 0; r2 < n; ++r2)
              if (depth[r2] == depth[q] && PQ(r2, PAIR_SENT) + PQ(r2, PAIR_RECV) > mx) mx = PQ(r2, PAIR_SENT) + PQ(r2, PAIR_RECV);
            def[q] = mx - (PQ(q, PAIR_SENT) + PQ(q, PAIR_RECV));
            if (def[q] > worst) worst = def[q];
          }
          if (worst > 0) for (uint32_t q = 0; q < n; ++q) if (def[q] == worst) { is_cand[off + q] = 1; ++n_c; }
          free(def);
        }
        if (n_c == 0) is_cand[off + best] = 1;      /* a pure cycle: fall back to the fewest counts */
      }
    }
    free(depth);
#undef PQ
  }

  /* ---- a not-entered rank that is itself blocked inside another hung communicator is a victim ---- */
  uint8_t *drop = (uint8_t *)calloc(n_pair ? n_pair : 1, 1);
  for (uint32_t c = 0; c < T->n_comms; ++c) {
    if (R->comm[(size_t)c * HC_NCOL + HC_CLASS] != 1) continue;
    for (uint32_t q = 0; q < T->size[c]; ++q) {
      uint64_t p = (uint64_t)T->member_off[c] + q;
      if (!is_cand[p]) continue;
      uint32_t r = T->members[p];
      for (uint32_t c2 = 0; c2 < T->n_comms && !drop[p]; ++c2) {
        if (c2 == c || !R->comm[(size_t)c2 * HC_NCOL + HC_HUNG]) continue;
        for (uint32_t q2 = 0; q2 < T->size[c2]; ++q2) {
          uint64_t p2 = (uint64_t)T->member_off[c2] + q2;
          if (T->members[p2] == r && R->pair[p2 * PAIR_NCOL + PAIR_ENTERED]) { drop[p] = 1; break; }
        }
      }
    }
  }
  uint64_t n_root = 0;
  for (uint64_t p = 0; p < n_pair; ++p) { if (drop[p]) is_cand[p] = 0; if (is_cand[p]) ++n_root; }
  free(drop);

  /* ---- hops along the wait-for edges to a root; roots listed by (rank, communicator) ---- */
  R->n_root = n_root;
  R->root = (int64_t *)calloc((n_root ? n_root : 1) * ROOT_NCOL, sizeof(int64_t));
  uint64_t kr = 0;
  for (uint32_t c = 0; c < T->n_comms; ++c) {
    const uint32_t n = T->size[c], off = T->member_off[c];
    int64_t *H = R->comm + (size_t)c * HC_NCOL;
    uint32_t nc = 0;
    for (uint32_t q = 0; q < n; ++q) if (is_cand[off + q]) {
      ++nc;
      int64_t *O = R->root + kr * ROOT_NCOL; ++kr;
      O[ROOT_RANK] = T->members[off + q]; O[ROOT_COMM] = c; O[ROOT_CLASS] = H[HC_CLASS];
    }
    H[HC_NCAND] = nc;
    if (!H[HC_HUNG]) continue;
    for (uint32_t q = 0; q < n; ++q) {
      uint32_t cur = q;
      int64_t hops = 0;
      while (1) {
        if (is_cand[off + cur]) break;
        int64_t w = R->pair[((uint64_t)off + cur) * PAIR_NCOL + PAIR_WAITS_ON];
        if (w == ORC_NO_RANK || hops >= (int64_t)n) { hops = -1; break; }
        uint32_t nxt = 0;
        while (T->members[off + nxt] != (uint32_t)w) ++nxt;
        cur = nxt; ++hops;
      }
      R->pair[((uint64_t)off + q) * PAIR_NCOL + PAIR_HOPS] = hops;
    }
  }
  qsort(R->root, n_root, ROOT_NCOL * sizeof(int64_t), cmp_root);
  free(is_cand);
  R->status = ORC_OK;
  return ORC_OK;
}


/* ------------------------------------------------------------------ */
/* SendRate / RecvRate (Section 4.1.2, "Slow Diagnostic Metrics"): the rate of a rank's progress is
 * the reciprocal of the number of times its SendCount (RecvCount) changes between samples while an
 * operation runs; a slow rank needs more samples, hence more changes, for the same operation.
 *
 * Per (pair, channel) the series is cut into runs of equal operation counter.  The last run is
 * still open (its operation may not have finished) and is left out.  Inside a run the count is
 * compared with the previous sample of the run, or with zero for the run's first sample (the
 * count starts at zero when the operation is posted).  A run with at least one change is one
 * observed operation.  Per pair, ops and changes are summed over channels; its rate is
 * ops / changes (compared by cross-multiplication), undefined without a change.
 * Per communicator: the member of minimal SendRate, of minimal RecvRate, and of the minimal of
 * both kinds (ties: smallest rank); the last one is stored in the state for Eq. 4's
 * communication-slow root.
 * The paper fixes the reciprocal-of-changes definition and one worked example (pinned in
 * tests/golden/sendrate_example.txt); the run boundaries, the open last run, the sum over channels
 * and the tie rule are readings made here: "parity unpinned" by the paper. */
enum { RATE_RANK, RATE_COMM, RATE_OPS_SEND, RATE_CHG_SEND, RATE_OPS_RECV, RATE_CHG_RECV, RATE_NCOL };
enum { RC_COMM, RC_ROOT_SEND, RC_ROOT_RECV, RC_ROOT, RC_NCOL };

typedef struct {
  int32_t status;
  uint64_t n_pair, n_comm;
  int64_t *pair;   /* [n_pair][RATE_NCOL] one row per member slot of every communicator, in table order */
  int64_t *comm;   /* [n_comm][RC_NCOL] */
} orc_rate_result;

void orc_rate_result_free(orc_rate_result *r) {
  if (!r) return;
  free(r->pair); free(r->comm);
  memset(r, 0, sizeof(*r));
}

/* is rate a = ops_a/chg_a smaller than rate b, or equal with the smaller rank */
static int rate_less(int64_t ops_a, int64_t chg_a, int64_t rank_a, int64_t ops_b, int64_t chg_b, int64_t rank_b) {
  __int128 l = (__int128)ops_a * (__int128)chg_b, r = (__int128)ops_b * (__int128)chg_a;
  if (l != r) return l < r;
  return rank_a < rank_b;
}

int orc_progress_rates(const orc_topology *T, uint64_t n_rows, uint32_t n_snap, uint32_t n_ch,
                       const uint32_t *snap, const uint32_t *rank, const uint32_t *comm, const uint32_t *channel,
                       const uint64_t *seq_posted, const uint32_t *chunks_sent, const uint32_t *chunks_recv,
                       orc_state *st, orc_rate_result *R) {
  memset(R, 0, sizeof(*R));
  uint64_t n_pair = 0;
  cell_t *cell = NULL;
  R->status = place_cells(T, n_rows, n_snap, n_ch, snap, rank, comm, channel, seq_posted, chunks_sent, chunks_recv,
                          &n_pair, &cell);
  if (R->status != ORC_OK) return R->status;
  R->n_pair = n_pair; R->n_comm = T->n_comms;
  R->pair = (int64_t *)calloc((n_pair ? n_pair : 1) * RATE_NCOL, sizeof(int64_t));
  R->comm = (int64_t *)calloc((size_t)(T->n_comms ? T->n_comms : 1) * RC_NCOL, sizeof(int64_t));
  for (uint32_t c = 0; c < T->n_comms; ++c) {
    for (uint32_t q = 0; q < T->size[c]; ++q) {
      const uint64_t p = (uint64_t)T->member_off[c] + q;
      int64_t *Q = R->pair + p * RATE_NCOL;
      Q[RATE_RANK] = T->members[p]; Q[RATE_COMM] = c;
      for (uint32_t ch = 0; ch < n_ch; ++ch) {
        const cell_t *s = cell + (p * n_ch + ch) * n_snap;
        uint32_t open = n_snap - 1;          /* first sample of the open run */
        while (open > 0 && s[open - 1].seq == s[n_snap - 1].seq) --open;
        uint32_t t = 0;
        while (t < open) {
          const uint64_t run = s[t].seq;
          uint32_t ps = 0, pr = 0;
          int64_t cs = 0, cr = 0;
          for (; t < open && s[t].seq == run; ++t) {
            if (s[t].sent != ps) ++cs;
            if (s[t].recv != pr) ++cr;
            ps = s[t].sent; pr = s[t].recv;
          }
          if (cs) { Q[RATE_OPS_SEND] += 1; Q[RATE_CHG_SEND] += cs; }
          if (cr) { Q[RATE_OPS_RECV] += 1; Q[RATE_CHG_RECV] += cr; }
        }
      }
    }
  }
  free(cell);
  for (uint32_t c = 0; c < T->n_comms; ++c) {
    int64_t *H = R->comm + (size_t)c * RC_NCOL;
    H[RC_COMM] = c; H[RC_ROOT_SEND] = ORC_NO_RANK; H[RC_ROOT_RECV] = ORC_NO_RANK; H[RC_ROOT] = ORC_NO_RANK;
    int64_t bs[2] = {0, 0}, br[2] = {0, 0}, bb[2] = {0, 0};   /* (ops, changes) of the current minima */
    for (uint32_t q = 0; q < T->size[c]; ++q) {
      const int64_t *Q = R->pair + ((uint64_t)T->member_off[c] + q) * RATE_NCOL;
      const int64_t rk = Q[RATE_RANK];
      if (Q[RATE_CHG_SEND] > 0) {
        if (H[RC_ROOT_SEND] == ORC_NO_RANK || rate_less(Q[RATE_OPS_SEND], Q[RATE_CHG_SEND], rk, bs[0], bs[1], H[RC_ROOT_SEND])) {
          bs[0] = Q[RATE_OPS_SEND]; bs[1] = Q[RATE_CHG_SEND]; H[RC_ROOT_SEND] = rk;
        }
        if (H[RC_ROOT] == ORC_NO_RANK || rate_less(Q[RATE_OPS_SEND], Q[RATE_CHG_SEND], rk, bb[0], bb[1], H[RC_ROOT])) {
          bb[0] = Q[RATE_OPS_SEND]; bb[1] = Q[RATE_CHG_SEND]; H[RC_ROOT] = rk;
        }
      }
      if (Q[RATE_CHG_RECV] > 0) {
        if (H[RC_ROOT_RECV] == ORC_NO_RANK || rate_less(Q[RATE_OPS_RECV], Q[RATE_CHG_RECV], rk, br[0], br[1], H[RC_ROOT_RECV])) {
          br[0] = Q[RATE_OPS_RECV]; br[1] = Q[RATE_CHG_RECV]; H[RC_ROOT_RECV] = rk;
        }
        if (H[RC_ROOT] == ORC_NO_RANK || rate_less(Q[RATE_OPS_RECV], Q[RATE_CHG_RECV], rk, bb[0], bb[1], H[RC_ROOT])) {
          bb[0] = Q[RATE_OPS_RECV]; bb[1] = Q[RATE_CHG_RECV]; H[RC_ROOT] = rk;
        }
      }
    }
    if (st && c < st->n_comms) st->rate_root[c] = H[RC_ROOT];
  }
  R->status = ORC_OK;
  return R->status;
}


/* ------------------------------------------------------------------ */
/* Probing Frame decoder (Section 5.1, "Probing Frame"; sizes from Section 6.2: a 32-byte header and
 * a 1152-byte body of 8 blocks, each holding one 16-byte Trace ID and, per channel, two consecutive
 * slots for SendCount and RecvCount; 8 channels; the block of an operation is its kernel counter
 * modulo the number of blocks).
 *
 * Byte layout taken here (little-endian; the paper lists the fields, not their widths):
 *   header  u64 kernel counter | u32 mode (bit 0: measurement on) | u32 kernelIndex | u32 channels | 12 reserved
 *   block   u32 communicator id | u32 extension (bit 0: block written) | u64 operation counter
 *           then 8 x { u64 SendCount, u64 RecvCount }
 * One call decodes one frame per rank for snapshot `snap`: per frame and communicator the written
 * block with the largest operation counter (then the largest block index) describes the rank's
 * latest kernel there; it replaces the remembered state of (rank, communicator) unless that is
 * newer; communicators absent from the frame keep their remembered state (the frame only holds the
 * latest 8 kernels).  Then one snapshot row is written for every member slot and channel, in table
 * order.  Checks, in this order of precedence: unknown communicator, rank not a member (or no such
 * rank), range (more than 8 channels in a header, a count above 2^32 - 1), two frames of one rank.
 * On an error nothing is remembered and no row is written.  "parity unpinned" beyond the sizes. */
enum { FRAME_BYTES = 1184, FRAME_HEADER = 32, FRAME_BLOCKS = 8, FRAME_BLOCK_BYTES = 144, FRAME_CHANNELS = 8 };

typedef struct {
  uint64_t n_pair;
  uint32_t n_ch;
  cell_t *last;     /* [n_pair][n_ch] */
} orc_frame_state;

orc_frame_state *orc_frames_create(const orc_topology *T, uint32_t n_ch) {
  if (n_ch == 0 || n_ch > FRAME_CHANNELS) return NULL;
  orc_frame_state *s = (orc_frame_state *)calloc(1, sizeof(*s));
  if (!s) return NULL;
  for (uint32_t c = 0; c < T->n_comms; ++c) s->n_pair += T->size[c];
  s->n_ch = n_ch;
  s->last = (cell_t *)calloc((s->n_pair ? s->n_pair : 1) * n_ch, sizeof(cell_t));
  if (!s->last) { free(s); return NULL; }
  return s;
}
void orc_frames_destroy(orc_frame_state *s) { if (s) { free(s->last); free(s); } }

static uint32_t rd_u32(const uint8_t *p) { return (uint32_t)p[0] | (uint32_t)p[1] << 8 | (uint32_t)p[2] << 16 | (uint32_t)p[3] << 24; }
static uint64_t rd_u64(const uint8_t *p) { return (uint64_t)rd_u32(p) | (uint64_t)rd_u32(p + 4) << 32; }

int orc_decode_frames(const orc_topology *T, orc_frame_state *st, const uint8_t *frames, const uint32_t *frame_rank,
                      uint64_t n_frames, uint32_t snap, uint32_t *o_snap, uint32_t *o_rank, uint32_t *o_comm,
                      uint32_t *o_channel, uint64_t *o_seq, uint32_t *o_sent, uint32_t *o_recv) {
  int bad_comm = 0, bad_member = 0, bad_range = 0, dup = 0;
  uint8_t *seen = (uint8_t *)calloc(T->n_ranks ? T->n_ranks : 1, 1);
  for (uint64_t f = 0; f < n_frames; ++f) {
    const uint8_t *F = frames + f * FRAME_BYTES;
    const uint32_t r = frame_rank[f], nch = rd_u32(F + 16);
    if (nch > FRAME_CHANNELS) bad_range = 1;
    if (r < T->n_ranks) { if (seen[r]) dup = 1; seen[r] = 1; }
    for (int b = 0; b < FRAME_BLOCKS; ++b) {
      const uint8_t *B = F + FRAME_HEADER + b * FRAME_BLOCK_BYTES;
      if (!(rd_u32(B + 4) & 1u)) continue;
      const uint32_t c = rd_u32(B);
      if (c >= T->n_comms) { bad_comm = 1; continue; }
      if (r >= T->n_ranks || !is_member(T, c, r)) bad_member = 1;
      for (uint32_t ch = 0; ch < nch && ch < FRAME_CHANNELS; ++ch)
        if (rd_u64(B + 16 + ch * 16) > 0xFFFFFFFFull || rd_u64(B + 16 + ch * 16 + 8) > 0xFFFFFFFFull) bad_range = 1;
    }
  }
  free(seen);
  if (bad_comm) return ORC_E_UNKNOWN_COMM;
  if (bad_member) return ORC_E_RANK_NOT_MEMBER;
  if (bad_range) return ORC_E_RANGE;
  if (dup) return ORC_E_DUPLICATE_KEY;
  for (uint64_t f = 0; f < n_frames; ++f) {
    const uint8_t *F = frames + f * FRAME_BYTES;
    const uint32_t r = frame_rank[f], nch = rd_u32(F + 16);
    for (int b = 0; b < FRAME_BLOCKS; ++b) {
      const uint8_t *B = F + FRAME_HEADER + b * FRAME_BLOCK_BYTES;
      if (!(rd_u32(B + 4) & 1u)) continue;
      const uint32_t c = rd_u32(B);
      const uint64_t cnt = rd_u64(B + 8);
      /* is another written block of this frame the rank's later kernel on the same communicator? */
      int loses = 0;
      for (int b2 = 0; b2 < FRAME_BLOCKS; ++b2) {
        const uint8_t *B2 = F + FRAME_HEADER + b2 * FRAME_BLOCK_BYTES;
        if (b2 == b || !(rd_u32(B2 + 4) & 1u) || rd_u32(B2) != c) continue;
        const uint64_t cnt2 = rd_u64(B2 + 8);
        if (cnt2 > cnt || (cnt2 == cnt && b2 > b)) loses = 1;
      }
      if (loses) continue;
      uint32_t slot = 0;
      while (T->members[T->member_off[c] + slot] != r) ++slot;
      const uint64_t p = (uint64_t)T->member_off[c] + slot;
      for (uint32_t ch = 0; ch < st->n_ch; ++ch) {
        cell_t *L = st->last + p * st->n_ch + ch;
        if (cnt < L->seq) continue;                 /* what is remembered is newer */
        L->seq = cnt;
        L->sent = ch < nch ? (uint32_t)rd_u64(B + 16 + ch * 16) : 0;
        L->recv = ch < nch ? (uint32_t)rd_u64(B + 16 + ch * 16 + 8) : 0;
      }
    }
  }
  uint64_t k = 0;
  for (uint32_t c = 0; c < T->n_comms; ++c)
    for (uint32_t q = 0; q < T->size[c]; ++q)
      for (uint32_t ch = 0; ch < st->n_ch; ++ch, ++k) {
        const cell_t *L = st->last + ((uint64_t)T->member_off[c] + q) * st->n_ch + ch;
        o_snap[k] = snap; o_rank[k] = T->members[T->member_off[c] + q]; o_comm[k] = c; o_channel[k] = ch;
        o_seq[k] = L->seq; o_sent[k] = L->sent; o_recv[k] = L->recv;
      }
  return ORC_OK;
}
