/*
 * axo_comm.h -- host-only C ABI of the collective-communication performance model of the 4D
 * hybrid algorithm (paper Section 5, "A Performance Model of Collective Communication in
 * Parallel Training") and of the rank <-> grid-coordinate mapping it assumes.
 *
 * Nothing here touches a GPU.  All functions are pure: they read their arguments, write their
 * outputs and keep no state; any output pointer may be NULL unless stated otherwise.  Every
 * function returns an int status from axo.h's axo_status_t (0 = ok) unless it returns a time.
 *
 * Model (Section 5.1, placement-agnostic): collectives use the bandwidth-optimal ring, start-up
 * latency and computation are ignored.  With G GPUs in the group, a buffer of `bytes` per GPU and
 * a peer-to-peer bandwidth beta (bytes per second):
 *     all-gather      t = (G - 1)        * bytes / beta
 *     reduce-scatter  t = (G - 1) / G    * bytes / beta
 *     all-reduce      t = 2 (G - 1) / G  * bytes / beta
 * One FC layer with I in R^{m x k}, W in R^{k x n} on a Gx x Gy x Gz x Gdata configuration costs
 * the sum of five terms (Section 5.1, the equations for t_AG,z  t_RS,z  t_AR,y  t_AR,x  t_AR,data):
 *     all-gather_z     of the weight shard            buffer k n / (Gx Gy Gz),  group Gz
 *     reduce-scatter_z of the weight gradient         buffer k n / (Gx Gy),     group Gz
 *     all-reduce_y     of the output activation       buffer m n / (Gz Gx),     group Gy
 *     all-reduce_x     of the input gradient          buffer m k / (Gz Gy),     group Gx
 *     all-reduce_data  of the weight gradient shard   buffer k n / (Gx Gy Gz),  group Gdata
 * These are the equations as printed; they describe Algorithm 1 as printed, where K is split over
 * the Y groups and N over the X groups, which is `transposed == 1` in axo.h's convention.  The
 * other kind of layer (every second one, Section 3.2; axo.h's default mapping `transposed == 0`,
 * K over X and N over Y) swaps Gx with Gy and beta_x with beta_y in these terms, as the last
 * paragraph of Section 5.1 prescribes.  m is the number of rows of I inside one tensor-parallel
 * group: the batch is divided into equal shards among the Gdata groups (Section 3.1), so
 * m = batch_rows / Gdata.  Buffer sizes are counted in elements by the paper; here they are
 * multiplied by bytes_per_element.
 *
 * Placement (Section 5.2): groups are nested X (innermost), Y, Z, data (outermost), i.e.
 *     rank = ix + Gx * (iy + Gy * (iz + Gz * idata)),
 * so with Gx = Gy = Gz = Gdata = 2 the X groups are the rank pairs (0,1), (2,3), (4,5), (6,7) and
 * the Y groups (0,2), (1,3), (4,6), (5,7).  With P_i = G_0 * ... * G_i (G_0 = Gx, ..., G_3 = Gdata):
 *     beta_i = beta_intra                                  if P_i <= G_node      (Case 1)
 *     beta_i = beta_inter / min(G_node, P_{i-1})           otherwise             (Case 2; P_{-1} = 1)
 */
#ifndef AXO_COMM_H
#define AXO_COMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* The four configurable performance parameters, in hierarchy order. */
typedef struct axo_comm_config {
    int32_t Gx, Gy, Gz, Gdata; /* each >= 1 */
} axo_comm_config_t;

/* The machine: bandwidths in bytes per second, GPUs per node. */
typedef struct axo_comm_net {
    double beta_intra;       /* peer-to-peer bandwidth between two GPUs of one node, > 0            */
    double beta_inter;       /* peer-to-peer bandwidth between two nodes, > 0                       */
    int32_t G_node;          /* GPUs per node, >= 1                                                 */
    int32_t placement_aware; /* 1: Section 5.2 bandwidths; 0: beta_inter for every group (Sec. 5.1) */
} axo_comm_net_t;

/* One FC layer of the network: I in R^{m x k} with m = batch_rows / Gdata, W in R^{k x n}. */
typedef struct axo_comm_layer {
    int64_t k, n;       /* in-features, out-features, each >= 1                                    */
    int32_t transposed; /* as in axo_problem_t: 0: K over Gx, N over Gy; 1: K over Gy, N over Gx  */
    int32_t reserved;   /* must be 0                                                               */
} axo_comm_layer_t;

/* The five terms of one layer, in seconds, and their sum (Section 5.1, last equation).
 * ar_fwd is the all-reduce of the output activation over the group that splits K (t_AR,y as
 * printed), ar_bwd the all-reduce of the input gradient over the group that splits N (t_AR,x). */
typedef struct axo_comm_terms {
    double ag_z, rs_z, ar_fwd, ar_bwd, ar_data, total;
} axo_comm_terms_t;

/* Ring collective times of Section 5.1 (first three equations).  G >= 1, bytes >= 0, beta > 0;
 * returns a negative value (-1.0) for arguments outside these ranges. */
double axo_comm_ring_all_gather(int32_t G, double bytes, double beta);
double axo_comm_ring_reduce_scatter(int32_t G, double bytes, double beta);
double axo_comm_ring_all_reduce(int32_t G, double bytes, double beta);

/* An MI355X node as this build assumes it: 8 GPUs per node, fully connected by xGMI links of
 * 153.6e9 bytes/s each, and one 400 Gb/s NIC (50e9 bytes/s) per GPU between nodes;
 * placement_aware = 1.  Errors: NULL_PTR. */
int axo_comm_net_mi355x(axo_comm_net_t *out);

/* beta[0..3] = (beta_x, beta_y, beta_z, beta_data) for a configuration on a machine (Section 5.2,
 * Cases 1 and 2; all beta_inter when net->placement_aware == 0).
 * Errors: NULL_PTR (cfg, net, beta), BAD_GRID (a G < 1), BAD_ARG (non-positive bandwidth, G_node < 1). */
int axo_comm_bandwidths(const axo_comm_config_t *cfg, const axo_comm_net_t *net, double beta[4]);

/* The five terms of one layer.  m_rows is the paper's m (rows of I inside one tensor-parallel
 * group).  The model needs no divisibility: buffer sizes are real numbers.
 * Errors: as axo_comm_bandwidths, plus BAD_SIZE (m_rows, k or n < 0; bytes_per_element <= 0),
 * BAD_ARG (layer->reserved != 0, transposed not 0/1), NULL_PTR (layer, out). */
int axo_comm_layer_time(const axo_comm_config_t *cfg, const axo_comm_net_t *net, const axo_comm_layer_t *layer,
                        int64_t m_rows, double bytes_per_element, axo_comm_terms_t *out);

/* Sum of axo_comm_layer_time over all layers with m = batch_rows / Gdata (Section 5.1, last
 * paragraph).  *total in seconds; terms (may be NULL) receives the per-term sums.
 * Errors: as above, plus INDIVISIBLE (batch_rows % Gdata != 0), BAD_ARG (n_layers < 0). */
int axo_comm_model_time(const axo_comm_config_t *cfg, const axo_comm_net_t *net, const axo_comm_layer_t *layers,
                        int32_t n_layers, int64_t batch_rows, double bytes_per_element, double *total,
                        axo_comm_terms_t *terms);

/* Enumerates every 4-tuple (Gx, Gy, Gz, Gdata) with Gx Gy Gz Gdata == n_gpus that the workload can
 * run on (Gdata divides batch_rows, Gz divides batch_rows / Gdata, and for every layer the K-axis
 * group divides k and the N-axis group divides n), models each with axo_comm_model_time and sorts
 * by modelled time, ascending; ties (times within 1e-12 relative of each other) are ordered by
 * (Gx, Gy, Gz, Gdata) ascending, lexicographic.
 * Writes the first min(*n_found, max_out) entries to configs / times (either may be NULL) and the
 * number of feasible configurations to *n_found (must not be NULL).  This is the ranking step of
 * Section 5 (the user then profiles the top few).
 * Errors: NULL_PTR, BAD_SIZE (n_gpus < 1 or > 2^20, batch_rows < 1), and those of axo_comm_model_time. */
int axo_comm_rank_configs(int32_t n_gpus, const axo_comm_net_t *net, const axo_comm_layer_t *layers,
                          int32_t n_layers, int64_t batch_rows, double bytes_per_element,
                          axo_comm_config_t *configs, double *times, int32_t max_out, int32_t *n_found);

/* Rank <-> coordinate under the hierarchy of Section 5.2: rank = ix + Gx (iy + Gy (iz + Gz idata)).
 * coord = (ix, iy, iz, idata).  Errors: NULL_PTR, BAD_GRID, BAD_COORD (rank or a coordinate out of range). */
int axo_comm_rank_to_coord(const axo_comm_config_t *cfg, int64_t rank, int32_t coord[4]);
int axo_comm_coord_to_rank(const axo_comm_config_t *cfg, const int32_t coord[4], int64_t *rank);

#ifdef __cplusplus
}
#endif
#endif /* AXO_COMM_H */
