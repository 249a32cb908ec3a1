/* The paper's instance-selection model (Algorithm 1, Eq. 1-7): host-only, double precision. */
#include "../../include/infersave.h"

#include <math.h>
#include <stddef.h>

static int bad_model(const isv_model *m) {
  return !m || m->n_params < 0 || m->h1 < 1 || m->h2 < 1 || m->n_layers < 1 || m->precision_bytes < 1;
}

static int bad_workload(const isv_workload *w) { return !w || w->batch < 1 || w->l_in < 1 || w->l_out < 1; }

int isv_memory_requirements(const isv_model *m, const isv_workload *w, isv_memory *out) {
  if (bad_model(m) || bad_workload(w) || !out) return ISV_EINVAL;
  const double tokens = (double)w->l_in + (double)w->l_out;
  out->model = m->n_params * m->precision_bytes;
  out->activation = 2.0 * tokens * w->batch * m->h1;
  out->kvcache = 2.0 * w->batch * tokens * m->h1 * m->precision_bytes * m->n_layers;
  out->kvcache_per_layer = out->kvcache / m->n_layers;
  out->base = out->model + out->activation;
  out->total = out->base + out->kvcache;
  return ISV_OK;
}

int isv_assess(const isv_instance *inst, int32_t n, const isv_memory *mem, double p_max, isv_candidate *verdict,
               int32_t *order, int32_t *n_candidates) {
  if (!inst || n < 0 || !mem || !verdict || !order || !n_candidates || !(mem->kvcache > 0)) return ISV_EINVAL;
  int32_t k = 0;
  for (int32_t i = 0; i < n; ++i) {
    isv_candidate *v = &verdict[i];
    v->c_off = 0.0;
    v->mem_avail = inst[i].gpu_mem_bytes - mem->base;
    if (inst[i].price_per_hour > p_max) {
      v->status = ISV_TOO_DEAR;
    } else if (inst[i].gpu_mem_bytes >= mem->total) {
      v->status = ISV_RESIDENT;
    } else if (inst[i].gpu_mem_bytes < mem->model || mem->kvcache_per_layer > v->mem_avail) {
      v->status = ISV_UNSUITABLE;
    } else {
      v->status = ISV_OFFLOAD;
      v->c_off = 1.0 - v->mem_avail / mem->kvcache;
    }
    if (v->status >= 0) order[k++] = i;
  }
  /* insertion sort by price: stable, and n is a handful of instance types */
  for (int32_t a = 1; a < k; ++a) {
    const int32_t x = order[a];
    int32_t b = a;
    while (b > 0 && inst[order[b - 1]].price_per_hour > inst[x].price_per_hour) {
      order[b] = order[b - 1];
      --b;
    }
    order[b] = x;
  }
  *n_candidates = k;
  return ISV_OK;
}

int isv_predict(const isv_model *m, const isv_workload *w, const isv_instance *inst, double c_off,
                int32_t overlap_decode, isv_times *out) {
  if (bad_model(m) || bad_workload(w) || !inst || !out || !(c_off >= 0.0 && c_off <= 1.0)) return ISV_EINVAL;
  if (!(inst->flops > 0)) return ISV_EINVAL;
  if (c_off > 0 && (!(inst->bw_gpu_to_cpu > 0) || !(inst->bw_cpu_to_gpu > 0))) return ISV_EINVAL;
  const double BS = w->batch, Lin = w->l_in, Lout = w->l_out, h1 = m->h1, h2 = m->h2, prec = m->precision_bytes;
  out->t_compute_pre = (BS * (8.0 * Lin * h1 * h1 + 4.0 * Lin * h1 * h2) + 4.0 * BS * Lin * Lin * h1) / inst->flops;
  out->t_compute_dec = (BS * (8.0 * h1 * h1 + 4.0 * h1 * h2) + 4.0 * BS * (Lin + Lout / 2.0) * h1) / inst->flops;
  out->t_trans_pre = c_off > 0 ? c_off * 2.0 * (Lin + 1.0) * h1 * prec * BS / inst->bw_gpu_to_cpu : 0.0;
  out->t_trans_dec = c_off > 0 ? (c_off * 2.0 * (Lin + 1.0) + Lout) * h1 * prec * BS / inst->bw_cpu_to_gpu : 0.0;
  const double cp = inst->alpha_pre * out->t_compute_pre + inst->beta_pre;
  const double cd = inst->alpha_dec * out->t_compute_dec + inst->beta_dec;
  out->t_pre = cp > out->t_trans_pre ? cp : out->t_trans_pre;
  if (overlap_decode) out->t_dec = cd > out->t_trans_dec ? cd : out->t_trans_dec;
  else out->t_dec = cd + out->t_trans_dec;
  out->t_task = m->n_layers * (out->t_pre + (Lout - 1.0) * out->t_dec);
  out->tps = out->t_task > 0 ? BS * (Lin + Lout) / out->t_task : 0.0;
  return ISV_OK;
}

double isv_attention_flops_decode(int32_t batch, double context, int32_t h1) {
  if (batch < 1 || !(context >= 0) || h1 < 1) return -1.0;
  return 4.0 * batch * context * h1;
}

int isv_ctcf_fit(int32_t n, const double *x, const double *y, double *alpha, double *beta, double *mean_rel_err) {
  if (n < 2 || !x || !y || !alpha || !beta) return ISV_EINVAL;
  double mx = 0, my = 0;
  for (int32_t i = 0; i < n; ++i) {
    mx += x[i];
    my += y[i];
  }
  mx /= n;
  my /= n;
  double sxx = 0, sxy = 0;
  for (int32_t i = 0; i < n; ++i) {
    sxx += (x[i] - mx) * (x[i] - mx);
    sxy += (x[i] - mx) * (y[i] - my);
  }
  if (!(sxx > 0)) return ISV_EINVAL;
  *alpha = sxy / sxx;
  *beta = my - *alpha * mx;
  if (mean_rel_err) {
    double e = 0;
    for (int32_t i = 0; i < n; ++i) e += fabs(*alpha * x[i] + *beta - y[i]) / fabs(y[i]);
    *mean_rel_err = e / n;
  }
  return ISV_OK;
}

double isv_cost_efficiency(double tps_actual, double tps_slo, int64_t n_queries, const isv_workload *w,
                           double price_per_hour, double *task_hours, double *total_cost) {
  if (!(tps_actual > 0) || !(tps_slo > 0) || n_queries < 1 || bad_workload(w) || !(price_per_hour > 0)) return -1.0;
  const double eff = tps_actual < tps_slo ? tps_actual : tps_slo;
  const double hours = (double)n_queries * ((double)w->l_in + (double)w->l_out) / (eff * 3600.0);
  const double billed = ceil(hours);
  if (task_hours) *task_hours = hours;
  if (total_cost) *total_cost = billed * price_per_hour;
  return eff * 3600.0 / (billed * price_per_hour);
}

int isv_select(int32_t n, const double *tps, const double *price, double tps_slo, int64_t n_queries,
               const isv_workload *w, int32_t *ranked, int32_t *n_ranked) {
  if (n < 0 || !tps || !price || !ranked || !n_ranked || !(tps_slo > 0) || n_queries < 1 || bad_workload(w)) return ISV_EINVAL;
  int32_t k = 0;
  for (int32_t i = 0; i < n; ++i) {
    if (!(tps[i] > 0) || !(price[i] > 0)) return ISV_EINVAL;
    if (tps[i] >= tps_slo) ranked[k++] = i;
  }
  for (int32_t a = 1; a < k; ++a) {               /* insertion sort: CE descending, then TPS descending, stable */
    const int32_t x = ranked[a];
    const double cx = isv_cost_efficiency(tps[x], tps_slo, n_queries, w, price[x], NULL, NULL);
    int32_t b = a;
    while (b > 0) {
      const int32_t p = ranked[b - 1];
      const double cp = isv_cost_efficiency(tps[p], tps_slo, n_queries, w, price[p], NULL, NULL);
      if (cp > cx || (cp == cx && tps[p] >= tps[x])) break;
      ranked[b] = p;
      --b;
    }
    ranked[b] = x;
  }
  *n_ranked = k;
  return ISV_OK;
}
