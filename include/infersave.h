/*
 * infersave -- the paper's instance-selection model as a small host-only C library.
 *
 * Given a model, a workload, a price ceiling and a list of GPU instances, the paper
 * (§IV) filters the instances by price and memory (Algorithm 1, which also yields the
 * share C_off of the KV cache that has to be offloaded), predicts tokens per second
 * from flop counts, transfer volumes and a per-instance linear calibration of the
 * compute time (Eq. 4-7, §IV-F), and picks the most cost-efficient instance that
 * meets the throughput objective (Eq. 1-3, Step 4).  These are those formulas; the
 * measured bandwidths and kernel times of this repository's GPU path are what they
 * are fed with in the benchmark.
 *
 * Conventions: plain C ABI, HOST pointers only, no allocation, no global state.
 * Sizes in bytes, times in seconds, rates per second, prices per hour.  Every function
 * returns ISV_OK (0) or ISV_EINVAL (-1) unless stated otherwise.
 */
#ifndef INFERSAVE_H
#define INFERSAVE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ISV_OK      0
#define ISV_EINVAL (-1)

typedef struct isv_model {
  double  n_params;          /* number of weights                                   */
  int32_t h1;                /* hidden size                                         */
  int32_t h2;                /* intermediate (FFN) size                             */
  int32_t n_layers;          /* L                                                   */
  int32_t precision_bytes;   /* 2 for fp16                                          */
} isv_model;

typedef struct isv_workload {
  int32_t batch;             /* BS                                                  */
  int32_t l_in, l_out;       /* prompt and output lengths (l_out >= 1)              */
} isv_workload;

typedef struct isv_instance {
  double gpu_mem_bytes;
  double price_per_hour;
  double flops;              /* the GPU's theoretical FLOPS                         */
  double bw_gpu_to_cpu;      /* bytes / s                                           */
  double bw_cpu_to_gpu;      /* bytes / s                                           */
  double alpha_pre, beta_pre;   /* CTCF of the prefill compute time (Eq. 7); 1, 0 = uncalibrated */
  double alpha_dec, beta_dec;   /* CTCF of the decode compute time                  */
} isv_instance;

typedef struct isv_memory {
  double model, activation, kvcache, kvcache_per_layer, total, base;
} isv_memory;

/* Table II and §IV-C: Mem_model = n_params * precision; Mem_activation =
 * 2 (L_in + L_out) BS h1; Mem_KVcache = 2 BS (L_in + L_out) h1 precision L (h1 where the
 * table prints nh: the transfer formulas use h1); per layer = / L; total = the three;
 * base = model + activation. */
int isv_memory_requirements(const isv_model *m, const isv_workload *w, isv_memory *out);

#define ISV_RESIDENT     0   /* Case 1: everything fits, C_off = 0                  */
#define ISV_OFFLOAD      1   /* Case 3: C_off = 1 - Mem_avail / Mem_KVcache         */
#define ISV_UNSUITABLE (-1)  /* Case 2: weights, or one layer's KV, do not fit       */
#define ISV_TOO_DEAR   (-2)  /* price above p_max                                   */

typedef struct isv_candidate {
  int32_t status;            /* one of the four above                               */
  double  c_off;             /* 0 unless status == ISV_OFFLOAD                      */
  double  mem_avail;         /* GPU memory minus Mem_base                           */
} isv_candidate;

/* Algorithm 1 over n instances.  verdict[i] describes instance i; order receives the
 * indices of the candidates (ISV_RESIDENT / ISV_OFFLOAD) sorted by price, ascending,
 * equal prices in input order; *n_candidates their number.
 *   verdict  out [n];  order  out [n] */
int isv_assess(const isv_instance *inst, int32_t n, const isv_memory *mem, double p_max,
               isv_candidate *verdict, int32_t *order, int32_t *n_candidates);

typedef struct isv_times {
  double t_compute_pre, t_trans_pre, t_pre;    /* per layer, prefill (Eq. 5)          */
  double t_compute_dec, t_trans_dec, t_dec;    /* per layer and token, decode (Eq. 6) */
  double t_task;                               /* Eq. 4                               */
  double tps;                                  /* Eq. 1                               */
} isv_times;

/* §IV-D for one instance and one offloading share c_off in [0, 1]:
 *   T_compute^p = (BS (8 L_in h1^2 + 4 L_in h1 h2) + 4 BS L_in^2 h1) / FLOPS
 *   T_trans^p   = c_off 2 (L_in + 1) h1 precision BS / BW_gpu->cpu
 *   T_pre       = max(CTCF(T_compute^p), T_trans^p)
 *   T_compute^d = (BS (8 h1^2 + 4 h1 h2) + 4 BS (L_in + L_out / 2) h1) / FLOPS
 *   T_trans^d   = (c_off 2 (L_in + 1) + L_out) h1 precision BS / BW_cpu->gpu   (0 if c_off = 0)
 *   T_dec       = CTCF(T_compute^d) + T_trans^d      (overlap_decode = 0, the paper's Eq. 6)
 *               = max(CTCF(T_compute^d), T_trans^d)  (overlap_decode = 1: transfers hidden
 *                 behind compute, as this repository's copy pipeline does)
 *   T_task      = n_layers (T_pre + (L_out - 1) T_dec),  TPS = BS (L_in + L_out) / T_task */
int isv_predict(const isv_model *m, const isv_workload *w, const isv_instance *inst, double c_off,
                int32_t overlap_decode, isv_times *out);

/* The self-attention term of §IV-D's decode compute time for one step at a given
 * context: 4 BS context h1 floating-point operations per layer (two multiply-adds per
 * cached K and V element).  With context = L_in + L_out / 2 it is the term inside
 * T_compute^d.  Returns the count (a negative value on a bad argument). */
double isv_attention_flops_decode(int32_t batch, double context, int32_t h1);

/* §IV-F: least-squares line measured = alpha * theory + beta through n >= 2 points whose
 * abscissae are not all equal.  *mean_rel_err (may be NULL) receives the mean of
 * |alpha x + beta - y| / |y| over the points. */
int isv_ctcf_fit(int32_t n, const double *t_theory, const double *t_measured, double *alpha,
                 double *beta, double *mean_rel_err);

/* Eq. 2 and Eq. 3 for a task of n_queries queries: TPS_effective = min(actual, SLO);
 * hours = n_queries (L_in + L_out) / (TPS_effective 3600); whole hours are billed;
 * CE = TPS_effective 3600 / (ceil(hours) price).  Returns CE, or a negative value on a bad
 * argument.  *task_hours and *total_cost may be NULL. */
double isv_cost_efficiency(double tps_actual, double tps_slo, int64_t n_queries, const isv_workload *w,
                           double price_per_hour, double *task_hours, double *total_cost);

/* Step 4: among n instances with throughput tps[i] and price[i], drop those below the
 * SLO and rank the rest by cost efficiency, descending (ties: higher TPS first, then input
 * order).  ranked receives the indices, *n_ranked their number (0 if none qualifies).
 *   ranked  out [n] */
int isv_select(int32_t n, const double *tps, const double *price, double tps_slo, int64_t n_queries,
               const isv_workload *w, int32_t *ranked, int32_t *n_ranked);

#ifdef __cplusplus
}
#endif
#endif /* INFERSAVE_H */
