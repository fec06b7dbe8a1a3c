// Layer removal after a reconfiguration plan (Sec. 4.1, "Layer Removal by Overlapping Regularization Groups"; the
// removed-layer counts of the result tables): host-only graph logic, no device work.
//
// A channel edge with no survivors carries nothing, so every layer writing it and every layer reading it drops out of
// the network.  That can starve further edges: an edge all of whose producers are gone carries nothing either, and an
// edge all of whose consumers are gone is read by nobody - unless the edge is also fed or read from outside the listed
// layers (the network input, the classifier behind the last stage).  The plan is the fixed point of these rules.  In a
// residual network this takes out whole branches and leaves the shortcut, which is how depth is learned.
#include <vector>

#include "common.h"

extern "C" int32_t pt_plan_layer_removal(const pt_removal_edge* edges, int32_t n_edges, int32_t n_layers,
                                         uint8_t* removed_layers, uint8_t* dead_edges) {
    if (n_edges < 0 || n_layers < 0) return PT_ERR_SHAPE;
    if ((n_edges > 0 && (!edges || !dead_edges)) || (n_layers > 0 && !removed_layers)) return PT_ERR_NULL;
    for (int e = 0; e < n_edges; ++e) {
        const pt_removal_edge& ed = edges[e];
        if (ed.n_prod < 0 || ed.n_cons < 0 || ed.n_keep < 0) return PT_ERR_SHAPE;
        if ((ed.n_prod > 0 && !ed.producers) || (ed.n_cons > 0 && !ed.consumers)) return PT_ERR_NULL;
        if (ed.external & ~3) return PT_ERR_UNSUPPORTED;
        for (int i = 0; i < ed.n_prod; ++i)
            if (ed.producers[i] < 0 || ed.producers[i] >= n_layers) return PT_ERR_SHAPE;
        for (int i = 0; i < ed.n_cons; ++i)
            if (ed.consumers[i] < 0 || ed.consumers[i] >= n_layers) return PT_ERR_SHAPE;
    }
    for (int l = 0; l < n_layers; ++l) removed_layers[l] = 0;
    for (int e = 0; e < n_edges; ++e) dead_edges[e] = edges[e].n_keep == 0 ? 1 : 0;
    bool changed = true;
    while (changed) {
        changed = false;
        for (int e = 0; e < n_edges; ++e) {
            const pt_removal_edge& ed = edges[e];
            if (dead_edges[e]) {  // nothing flows here: its writers and readers go
                for (int i = 0; i < ed.n_prod; ++i)
                    if (!removed_layers[ed.producers[i]]) removed_layers[ed.producers[i]] = 1, changed = true;
                for (int i = 0; i < ed.n_cons; ++i)
                    if (!removed_layers[ed.consumers[i]]) removed_layers[ed.consumers[i]] = 1, changed = true;
                continue;
            }
            bool fed = (ed.external & PT_EDGE_FED_OUTSIDE) != 0 || ed.n_prod == 0;
            for (int i = 0; i < ed.n_prod && !fed; ++i) fed = !removed_layers[ed.producers[i]];
            bool read = (ed.external & PT_EDGE_READ_OUTSIDE) != 0 || ed.n_cons == 0;
            for (int i = 0; i < ed.n_cons && !read; ++i) read = !removed_layers[ed.consumers[i]];
            if (!fed || !read) dead_edges[e] = 1, changed = true;
        }
    }
    // the network is cut if an edge that something outside still reads has died
    for (int e = 0; e < n_edges; ++e)
        if (dead_edges[e] && (edges[e].external & PT_EDGE_READ_OUTSIDE)) return PT_ERR_EMPTY;
    return PT_OK;
}
