// Host-only implementation of the communication performance model (paper Section 5) and of the
// rank <-> coordinate mapping of Section 5.2.  No GPU code; compiled into the same library so
// that one shared object carries the whole C ABI.
#include "../../include/axo_comm.h"

#include <algorithm>
#include <cstdint>
#include <new>
#include <vector>

#include "../../include/axo.h"

namespace {

int check_cfg(const axo_comm_config_t* c) {
    if (!c) return AXO_ERR_NULL_PTR;
    if (c->Gx < 1 || c->Gy < 1 || c->Gz < 1 || c->Gdata < 1) return AXO_ERR_BAD_GRID;
    return AXO_OK;
}

int check_net(const axo_comm_net_t* n) {
    if (!n) return AXO_ERR_NULL_PTR;
    if (!(n->beta_intra > 0.0) || !(n->beta_inter > 0.0) || n->G_node < 1) return AXO_ERR_BAD_ARG;
    if (n->placement_aware != 0 && n->placement_aware != 1) return AXO_ERR_BAD_ARG;
    return AXO_OK;
}

int check_layer(const axo_comm_layer_t* l) {
    if (!l) return AXO_ERR_NULL_PTR;
    if (l->reserved != 0 || (l->transposed != 0 && l->transposed != 1)) return AXO_ERR_BAD_ARG;
    if (l->k < 0 || l->n < 0) return AXO_ERR_BAD_SIZE;
    return AXO_OK;
}

// Section 5.1, ring equations; G >= 1 and beta > 0 already checked
double ring_ag(double G, double bytes, double beta) { return (G - 1.0) * bytes / beta; }
double ring_rs(double G, double bytes, double beta) { return (G - 1.0) / G * bytes / beta; }
double ring_ar(double G, double bytes, double beta) { return 2.0 * (G - 1.0) / G * bytes / beta; }

// Section 5.2: bandwidth of the groups at each level of the hierarchy X, Y, Z, data
void bandwidths(const axo_comm_config_t& c, const axo_comm_net_t& net, double beta[4]) {
    const int64_t G[4] = {c.Gx, c.Gy, c.Gz, c.Gdata};
    int64_t below = 1;  // product of the group sizes of the levels inside level i
    for (int i = 0; i < 4; ++i) {
        const int64_t upto = below * G[i];
        if (!net.placement_aware)
            beta[i] = net.beta_inter;
        else if (upto <= net.G_node)
            beta[i] = net.beta_intra;  // Case 1: the group lies within a node
        else
            beta[i] = net.beta_inter / (double)std::min<int64_t>(net.G_node, below);  // Case 2
        below = upto;
    }
}

void layer_terms(const axo_comm_config_t& c, const double beta[4], const axo_comm_layer_t& l, double m,
                 double bytes_per_element, axo_comm_terms_t* t) {
    // group that splits K (forward all-reduce) and group that splits N (backward all-reduce):
    // as printed (transposed == 1) these are Y and X
    const double Gk = l.transposed ? c.Gy : c.Gx, bk = l.transposed ? beta[1] : beta[0];
    const double Gn = l.transposed ? c.Gx : c.Gy, bn = l.transposed ? beta[0] : beta[1];
    const double Gz = c.Gz, Gd = c.Gdata, k = (double)l.k, n = (double)l.n, e = bytes_per_element;
    t->ag_z = ring_ag(Gz, e * k * n / (Gk * Gn * Gz), beta[2]);
    t->rs_z = ring_rs(Gz, e * k * n / (Gk * Gn), beta[2]);
    t->ar_fwd = ring_ar(Gk, e * m * n / (Gz * Gn), bk);
    t->ar_bwd = ring_ar(Gn, e * m * k / (Gz * Gk), bn);
    t->ar_data = ring_ar(Gd, e * k * n / (Gk * Gn * Gz), beta[3]);
    t->total = t->ag_z + t->rs_z + t->ar_fwd + t->ar_bwd + t->ar_data;
}

}  // namespace

extern "C" {

double axo_comm_ring_all_gather(int32_t G, double bytes, double beta) {
    if (G < 1 || !(bytes >= 0.0) || !(beta > 0.0)) return -1.0;
    return ring_ag(G, bytes, beta);
}

double axo_comm_ring_reduce_scatter(int32_t G, double bytes, double beta) {
    if (G < 1 || !(bytes >= 0.0) || !(beta > 0.0)) return -1.0;
    return ring_rs(G, bytes, beta);
}

double axo_comm_ring_all_reduce(int32_t G, double bytes, double beta) {
    if (G < 1 || !(bytes >= 0.0) || !(beta > 0.0)) return -1.0;
    return ring_ar(G, bytes, beta);
}

int axo_comm_net_mi355x(axo_comm_net_t* out) {
    if (!out) return AXO_ERR_NULL_PTR;
    out->beta_intra = 153.6e9;
    out->beta_inter = 50.0e9;
    out->G_node = 8;
    out->placement_aware = 1;
    return AXO_OK;
}

int axo_comm_bandwidths(const axo_comm_config_t* cfg, const axo_comm_net_t* net, double beta[4]) {
    int rc = check_cfg(cfg);
    if (rc) return rc;
    if ((rc = check_net(net))) return rc;
    if (!beta) return AXO_ERR_NULL_PTR;
    bandwidths(*cfg, *net, beta);
    return AXO_OK;
}

int axo_comm_layer_time(const axo_comm_config_t* cfg, const axo_comm_net_t* net, const axo_comm_layer_t* layer,
                        int64_t m_rows, double bytes_per_element, axo_comm_terms_t* out) {
    int rc = check_cfg(cfg);
    if (rc) return rc;
    if ((rc = check_net(net))) return rc;
    if ((rc = check_layer(layer))) return rc;
    if (!out) return AXO_ERR_NULL_PTR;
    if (m_rows < 0 || !(bytes_per_element > 0.0)) return AXO_ERR_BAD_SIZE;
    double beta[4];
    bandwidths(*cfg, *net, beta);
    layer_terms(*cfg, beta, *layer, (double)m_rows, bytes_per_element, out);
    return AXO_OK;
}

int axo_comm_model_time(const axo_comm_config_t* cfg, const axo_comm_net_t* net, const axo_comm_layer_t* layers,
                        int32_t n_layers, int64_t batch_rows, double bytes_per_element, double* total,
                        axo_comm_terms_t* terms) {
    int rc = check_cfg(cfg);
    if (rc) return rc;
    if ((rc = check_net(net))) return rc;
    if (n_layers < 0) return AXO_ERR_BAD_ARG;
    if (n_layers > 0 && !layers) return AXO_ERR_NULL_PTR;
    if (batch_rows < 0 || !(bytes_per_element > 0.0)) return AXO_ERR_BAD_SIZE;
    if (batch_rows % cfg->Gdata != 0) return AXO_ERR_INDIVISIBLE;
    for (int i = 0; i < n_layers; ++i)
        if ((rc = check_layer(&layers[i]))) return rc;
    double beta[4];
    bandwidths(*cfg, *net, beta);
    const double m = (double)(batch_rows / cfg->Gdata);
    axo_comm_terms_t sum = {0, 0, 0, 0, 0, 0};
    for (int i = 0; i < n_layers; ++i) {
        axo_comm_terms_t t;
        layer_terms(*cfg, beta, layers[i], m, bytes_per_element, &t);
        sum.ag_z += t.ag_z;
        sum.rs_z += t.rs_z;
        sum.ar_fwd += t.ar_fwd;
        sum.ar_bwd += t.ar_bwd;
        sum.ar_data += t.ar_data;
        sum.total += t.total;
    }
    if (total) *total = sum.total;
    if (terms) *terms = sum;
    return AXO_OK;
}

int axo_comm_rank_configs(int32_t n_gpus, const axo_comm_net_t* net, const axo_comm_layer_t* layers,
                          int32_t n_layers, int64_t batch_rows, double bytes_per_element,
                          axo_comm_config_t* configs, double* times, int32_t max_out, int32_t* n_found) {
    if (!n_found) return AXO_ERR_NULL_PTR;
    if (n_gpus < 1 || n_gpus > (1 << 20) || batch_rows < 1) return AXO_ERR_BAD_SIZE;
    int rc = check_net(net);
    if (rc) return rc;
    if (n_layers < 0) return AXO_ERR_BAD_ARG;
    if (n_layers > 0 && !layers) return AXO_ERR_NULL_PTR;
    if (!(bytes_per_element > 0.0)) return AXO_ERR_BAD_SIZE;
    for (int i = 0; i < n_layers; ++i)
        if ((rc = check_layer(&layers[i]))) return rc;
    // the candidate list lives in a standard container: no exception may leave the library
    try {
        struct Entry {
            axo_comm_config_t c;
            double t;
        };
        std::vector<Entry> found;
        for (int32_t gx = 1; gx <= n_gpus; ++gx) {
            if (n_gpus % gx) continue;
            for (int32_t gy = 1; gy <= n_gpus / gx; ++gy) {
                if ((n_gpus / gx) % gy) continue;
                const int32_t rest = n_gpus / gx / gy;
                for (int32_t gz = 1; gz <= rest; ++gz) {
                    if (rest % gz) continue;
                    const axo_comm_config_t c = {gx, gy, gz, rest / gz};
                    if (batch_rows % c.Gdata != 0 || (batch_rows / c.Gdata) % c.Gz != 0) continue;
                    bool ok = true;
                    for (int i = 0; i < n_layers && ok; ++i) {
                        const int32_t gk = layers[i].transposed ? gy : gx, gn = layers[i].transposed ? gx : gy;
                        ok = layers[i].k % gk == 0 && layers[i].n % gn == 0;
                    }
                    if (!ok) continue;
                    double t = 0.0;
                    rc = axo_comm_model_time(&c, net, layers, n_layers, batch_rows, bytes_per_element, &t, nullptr);
                    if (rc) return rc;
                    found.push_back({c, t});
                }
            }
        }
        std::stable_sort(found.begin(), found.end(), [](const Entry& a, const Entry& b) { return a.t < b.t; });
        // Configurations whose modelled times are equal as real numbers can differ in the last bits
        // of their floating-point sums: runs of times within 1e-12 (relative) of their neighbour are
        // ties, ordered by (Gx, Gy, Gz, Gdata) ascending.
        auto lex = [](const Entry& a, const Entry& b) {
            if (a.c.Gx != b.c.Gx) return a.c.Gx < b.c.Gx;
            if (a.c.Gy != b.c.Gy) return a.c.Gy < b.c.Gy;
            if (a.c.Gz != b.c.Gz) return a.c.Gz < b.c.Gz;
            return a.c.Gdata < b.c.Gdata;
        };
        for (size_t i = 0; i < found.size();) {
            size_t j = i + 1;
            while (j < found.size() && found[j].t - found[j - 1].t <= 1e-12 * found[j].t) ++j;
            std::sort(found.begin() + i, found.begin() + j, lex);
            i = j;
        }
        *n_found = (int32_t)found.size();
        const int32_t n_out = std::min<int32_t>(*n_found, max_out < 0 ? 0 : max_out);
        for (int32_t i = 0; i < n_out; ++i) {
            if (configs) configs[i] = found[i].c;
            if (times) times[i] = found[i].t;
        }
        return AXO_OK;
    } catch (const std::bad_alloc&) {
        return AXO_ERR_NO_MEMORY;
    } catch (...) {
        return AXO_ERR_BAD_ARG;
    }
}

int axo_comm_rank_to_coord(const axo_comm_config_t* cfg, int64_t rank, int32_t coord[4]) {
    int rc = check_cfg(cfg);
    if (rc) return rc;
    if (!coord) return AXO_ERR_NULL_PTR;
    const int64_t world = (int64_t)cfg->Gx * cfg->Gy * cfg->Gz * cfg->Gdata;
    if (rank < 0 || rank >= world) return AXO_ERR_BAD_COORD;
    coord[0] = (int32_t)(rank % cfg->Gx);
    rank /= cfg->Gx;
    coord[1] = (int32_t)(rank % cfg->Gy);
    rank /= cfg->Gy;
    coord[2] = (int32_t)(rank % cfg->Gz);
    coord[3] = (int32_t)(rank / cfg->Gz);
    return AXO_OK;
}

int axo_comm_coord_to_rank(const axo_comm_config_t* cfg, const int32_t coord[4], int64_t* rank) {
    int rc = check_cfg(cfg);
    if (rc) return rc;
    if (!coord || !rank) return AXO_ERR_NULL_PTR;
    const int32_t G[4] = {cfg->Gx, cfg->Gy, cfg->Gz, cfg->Gdata};
    for (int i = 0; i < 4; ++i)
        if (coord[i] < 0 || coord[i] >= G[i]) return AXO_ERR_BAD_COORD;
    *rank = coord[0] + (int64_t)cfg->Gx * (coord[1] + (int64_t)cfg->Gy * (coord[2] + (int64_t)cfg->Gz * coord[3]));
    return AXO_OK;
}

}  // extern "C"
