/*
 * Stack-distance trace tools of Sec. 4.2 at scale: Alg. 1 (profile a trace of embedding
 * lookups of one categorical feature into the list u of unique accesses and the distribution p
 * of distances between repeated accesses) and Alg. 2 (generate a synthetic trace from u and p).
 *
 * INPUT GENERATION ONLY: nothing of the method's arithmetic lives here.  The stack of Alg. 1 and
 * the list of Alg. 2 are kept as "slots in order of last use" under a Fenwick tree of occupancy
 * counts, so that "position from the top" and "remove the d-th from the back" cost O(log n)
 * instead of a walk of the list; workloads/trace.py holds the same two algorithms as plain
 * list operations and the tests require both to agree exactly.
 *
 * Conventions (Sec. 4.2): d = 0 means "not seen before"; d >= 1 is the position from the top of
 * the stack (1 = the access just before).  p[d] is the fraction of the trace's accesses at
 * distance d.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define TR_OK 0
#define TR_ERR_MEM (-1)
#define TR_ERR_ARG (-2)

typedef struct {
  int64_t n;
  int64_t* t; /* 1-based */
} fenwick;

static int fw_init(fenwick* f, int64_t n) {
  f->n = n;
  f->t = (int64_t*)calloc((size_t)n + 1, sizeof(int64_t));
  return f->t ? TR_OK : TR_ERR_MEM;
}
static void fw_add(fenwick* f, int64_t i, int64_t v) { /* i: 0-based slot */
  for (i += 1; i <= f->n; i += i & (-i)) f->t[i] += v;
}
static int64_t fw_prefix(const fenwick* f, int64_t i) { /* occupied slots in [0, i) */
  int64_t s = 0;
  for (; i > 0; i -= i & (-i)) s += f->t[i];
  return s;
}
/* smallest 0-based slot whose prefix count (inclusive) reaches k (1 <= k <= total) */
static int64_t fw_find(const fenwick* f, int64_t k) {
  int64_t pos = 0, step = 1;
  while ((step << 1) <= f->n) step <<= 1;
  for (; step > 0; step >>= 1) {
    if (pos + step <= f->n && f->t[pos + step] < k) {
      pos += step;
      k -= f->t[pos];
    }
  }
  return pos; /* 0-based */
}

/*
 * Alg. 1.  tr[n]: ids in [0, id_bound).  Outputs: u (capacity n) receives the unique ids in order
 * of first appearance, *n_u their number; cnt (capacity n + 1, zeroed by the caller) receives the
 * NUMBER of accesses at every distance d (p[d] = cnt[d] / n), *max_d the largest distance seen.
 */
int trace_profile(const int64_t* tr, int64_t n, int64_t id_bound, int64_t* u, int64_t* n_u, int64_t* cnt,
                  int64_t* max_d) {
  if (n < 0 || id_bound < 1) return TR_ERR_ARG;
  int64_t* last = (int64_t*)malloc(sizeof(int64_t) * (size_t)id_bound); /* slot of the id's last use, or -1 */
  fenwick f;
  if (!last || fw_init(&f, n > 0 ? n : 1) != TR_OK) {
    free(last);
    return TR_ERR_MEM;
  }
  for (int64_t i = 0; i < id_bound; ++i) last[i] = -1;
  int64_t nu = 0, md = 0, live = 0;
  for (int64_t i = 0; i < n; ++i) {
    const int64_t a = tr[i];
    if (a < 0 || a >= id_bound) {
      free(last);
      free(f.t);
      return TR_ERR_ARG;
    }
    int64_t d = 0;
    if (last[a] < 0) {
      u[nu++] = a;
    } else {
      /* ids used after a's last use sit above it on the stack */
      d = live - fw_prefix(&f, last[a] + 1) + 1;
      fw_add(&f, last[a], -1);
      --live;
    }
    cnt[d] += 1;
    if (d > md) md = d;
    last[a] = i; /* the slot of access i is i: slots are in order of last use */
    fw_add(&f, i, 1);
    ++live;
  }
  *n_u = nu;
  *max_d = md;
  free(last);
  free(f.t);
  return TR_OK;
}

/*
 * Alg. 2.  u[n_u]: unique ids (drawn from the front while unseen), cum[0..n_p): cumulative sums of
 * p (cum[d] = p[0] + ... + p[d]); r[length]: uniform numbers in [0, 1) supplied by the caller.
 * The distance of step i is drawn from p restricted to the support [lo, s], s = number of unique ids
 * emitted so far and lo = 0 while unseen ids remain, else 1:
 *   target = base + r[i] * (cum[min(s, n_p - 1)] - base), base = (lo ? cum[0] : 0);
 *   d = the first index >= lo with cum[d] > target.
 * No mass in the support: d = 0 while unseen ids remain, else d = 1.
 * min_new > 0: while unseen ids remain, p[0] counts as max(p[0], min_new) (the adjustment Sec. 4.2
 * describes for long traces).
 */
int trace_generate(const int64_t* u, int64_t n_u, const double* cum, int64_t n_p, const double* r,
                   int64_t length, double min_new, int64_t* tr) {
  if (n_u < 1 || n_p < 1 || length < 0) return TR_ERR_ARG;
  const int64_t slots = n_u + length;
  int64_t* slot_id = (int64_t*)malloc(sizeof(int64_t) * (size_t)slots);
  fenwick f;
  if (!slot_id || fw_init(&f, slots) != TR_OK) {
    free(slot_id);
    return TR_ERR_MEM;
  }
  /* the list of Alg. 2: unseen ids at the front in order, used ids appended at the back */
  for (int64_t i = 0; i < n_u; ++i) slot_id[i] = u[i];
  int64_t front = 0, back = n_u, s = 0; /* front: next unseen; back: next free slot; s: ids emitted so far */
  int64_t seen_live = 0;                /* occupied slots at or after n_u, plus re-appended: tracked in the tree */
  const double boost = (min_new > cum[0]) ? (min_new - cum[0]) : 0.0;
  for (int64_t i = 0; i < length; ++i) {
    const int unseen = front < n_u;
    const int64_t top = s < n_p - 1 ? s : n_p - 1;
    int64_t d;
    if (unseen) {
      const double total = cum[top] + boost;
      const double target = r[i] * total;
      if (!(total > 0.0)) {
        d = 0;
      } else if (target < cum[0] + boost) {
        d = 0;
      } else { /* first d >= 1 with cum[d] + boost > target */
        int64_t lo = 1, hi = top;
        while (lo < hi) {
          const int64_t mid = (lo + hi) >> 1;
          if (cum[mid] + boost > target) hi = mid; else lo = mid + 1;
        }
        d = lo;
      }
    } else {
      const double mass = cum[top] - cum[0];
      if (!(mass > 0.0)) {
        d = 1;
      } else {
        const double target = cum[0] + r[i] * mass;
        int64_t lo = 1, hi = top;
        while (lo < hi) {
          const int64_t mid = (lo + hi) >> 1;
          if (cum[mid] > target) hi = mid; else lo = mid + 1;
        }
        d = lo;
      }
    }
    if (d > seen_live) d = seen_live; /* (cannot happen while d <= s; guards a caller's p with mass beyond s) */
    int64_t a;
    if (d == 0) {
      if (!unseen) { /* nothing to reuse and nothing new: only with n_u ids all seen and d forced to 0 */
        free(slot_id);
        free(f.t);
        return TR_ERR_ARG;
      }
      a = slot_id[front++];
      ++s;
    } else {
      /* the d-th from the back among the used ids = the (seen_live - d + 1)-th occupied slot */
      const int64_t pos = fw_find(&f, seen_live - d + 1);
      a = slot_id[pos];
      fw_add(&f, pos, -1);
      --seen_live;
    }
    slot_id[back] = a;
    fw_add(&f, back, 1);
    ++back;
    ++seen_live;
    tr[i] = a;
  }
  free(slot_id);
  free(f.t);
  return TR_OK;
}
