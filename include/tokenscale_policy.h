/* tokenscale_policy.h -- Token-Velocity policy functions of the TokenScale paper as pure host
 * functions (C ABI, no GPU state, no allocation, thread-safe).
 *
 * They turn measured velocities -- for a Convertible Decoder, what ts_token_velocity() reports for
 * the attention path -- into the autoscaler's instance counts and the router's decisions.
 *
 * Conventions: rates in tokens/s, times in seconds, memory in bytes.  Pointers are HOST arrays
 * owned by the caller and only read (outputs are stated).  Functions returning double return NaN
 * for arguments outside the stated domain; functions returning an index return a negative TS_POLICY_*
 * code.  Nothing is rounded: ts_tv_instances() turns a requirement into a count.
 */
#ifndef TOKENSCALE_POLICY_H
#define TOKENSCALE_POLICY_H

#include <stdint.h>
#include "tokenscale.h"

#ifdef __cplusplus
extern "C" {
#endif

#define TS_POLICY_NONE    (-1)   /* no eligible instance: queue the prefill task / reject the decode request */
#define TS_POLICY_INVALID (-2)   /* NULL array with a positive count, negative count, type out of range */

/* Decode velocity V_D (Sec. 3.2, first equation): sum of the tokens L_r held by the n requests
 * that completed during one decode iteration, over the measured TPOT.  Domain: tpot_s > 0,
 * L_r >= 0; n = 0 gives 0. */
double ts_tv_decode_velocity(const int64_t *request_tokens, int n, double tpot_s);

/* Prefillers required, I^P (Sec. 4.3, prefiller autoscaler): input token arrival rate lambda over
 * min(V_P, V_BW).  Domain: lambda >= 0, V_P > 0, V_BW > 0 (pass INFINITY to ignore the network). */
double ts_tv_prefillers(double lambda, double v_p, double v_bw);

/* Decoders required, I^D (Sec. 4.3, decoder autoscaler): sum over the n buckets of
 * lambda'[b] / v_d[b] (arrival rate of input plus predicted output tokens of bucket b over the
 * bucket's profiled velocity), summed in bucket order.  per_bucket: NULL or HOST array of n that
 * receives the terms I^(b).  Domain: lambda'[b] >= 0, v_d[b] > 0; n = 0 gives 0. */
double ts_tv_decoders(const double *lambda_b, const double *v_d_b, int n, double *per_bucket);

/* Regular decoders, I^D_r = max(I^D - I^D_c, 0) (Sec. 4.3).  Domain: both >= 0. */
double ts_tv_regular_decoders(double i_d, double i_d_c);

/* Average decode batch size (Sec. 4.4): available memory over the mean memory of a request.
 * Domain: available_bytes >= 0, mean_request_bytes > 0. */
double ts_tv_decode_batch(double available_bytes, double mean_request_bytes);

/* Prefill velocity of a Convertible Decoder, V_D^{P'} = (chunk_size - batch_size) / TPOT_SLO
 * (Sec. 4.4); 0 when the decode batch fills the chunk.  Domain: sizes >= 0, tpot_slo_s > 0. */
double ts_tv_convertible_prefill_velocity(double chunk_size, double batch_size, double tpot_slo_s);

/* Memory reserved for prefill on a Convertible Decoder, V_D^{P'} * Mem_T * TTFT_SLO (Sec. 4.4).
 * Domain: all >= 0. */
double ts_tv_reserved_memory(double v_d_p, double mem_t_bytes, double ttft_slo_s);

/* Chunk-size profiling of a Convertible Decoder (Sec. 4.4): iteration_time_s[i] is the iteration
 * time measured at the i-th chunk size of an ascending sweep.  Returns the index of the largest
 * chunk size met before the first one that exceeds tpot_slo_s (a time equal to the SLO meets it; NaN
 * does not), TS_POLICY_NONE when the first size already exceeds it or n = 0, TS_POLICY_INVALID for
 * n < 0 or a NULL array with n > 0. */
int ts_tv_largest_chunk(const double *iteration_time_s, int n, double tpot_slo_s);

/* Mem_T of a cache geometry: bytes of K and V one token occupies in num_layers layers
 * (2 * num_kv_heads * head_dim * element size * num_layers).  0 for an invalid descriptor or
 * num_layers < 1. */
int64_t ts_tv_token_bytes(const ts_attn_desc *desc, int num_layers);

/* The minimum number of instances that provides the required velocity (Sec. 4.3): the smallest
 * integer >= requirement.  TS_POLICY_INVALID for NaN, infinity or a negative requirement. */
int64_t ts_tv_instances(double requirement);
#define TS_ROUTE_PREFILLER   0
#define TS_ROUTE_CONVERTIBLE 1
#define TS_ROUTE_QUEUE       2

/* Prefill routing (Sec. 4.5, Alg. 1).  Round one: the first prefiller p (in index order) with
 * inflight_tokens[p] / velocity[p] <= slo_s takes the request; round two: the same over the
 * Convertible Decoders with their prefill velocity V_D^{P'}; otherwise the request is queued.
 * An instance with nothing in flight waits 0 s whatever its velocity; with velocity 0 and tokens
 * in flight it is never chosen.  *kind receives TS_ROUTE_*; the return value is the index within
 * that kind, TS_POLICY_NONE for the queue, TS_POLICY_INVALID for bad arguments. */
int ts_route_prefill(const double *prefiller_inflight, const double *prefiller_velocity, int n_prefillers,
                     const double *conv_inflight, const double *conv_velocity, int n_conv,
                     double slo_s, int *kind);

/* Decode routing (Sec. 4.5, decode load balancing): the decoder with the fewest in-flight
 * requests of the request's type; a Convertible Decoder whose memory utilisation exceeds
 * mem_threshold is left out; ties go to the lowest index.
 *   inflight : [n_decoders][n_types] row-major request counts
 *   convertible : [n_decoders] non-zero for Convertible Decoders;  mem_util : [n_decoders] in [0,1]
 * Returns the decoder index, TS_POLICY_NONE when none is eligible, TS_POLICY_INVALID. */
int ts_route_decode(const int32_t *inflight, int n_decoders, int n_types, int type,
                    const uint8_t *convertible, const double *mem_util, double mem_threshold);

#ifdef __cplusplus
}
#endif
#endif /* TOKENSCALE_POLICY_H */
