// The graph object behind the C ABI's opaque gcn_graph handle (shared by the translation units that implement
// entry points; not part of the ABI).
#pragma once

#include "common.hpp"

struct gcn_graph {
    int64_t n = 0, nnz_in = 0, E = 0, n_train = 0;
    // row classes of the whole pattern and of the residual one: a wave each / a lane group each / cut into chunks
    struct RowClasses {
        int64_t n_heavy = 0, n_light = 0, n_split = 0, n_chunks = 0, xcd_rows_max = 0;
        int phased_w = 0, phased_r = 0;   // 0: no phased schedule for this pattern
    } rows, res_rows, bwd_rows;
    int32_t f = 0, ldf = 0, n_classes = 0, max_deg = 0;
    int store_dtype = GCN_F32;
    gcn::PrepBuffers pb{};
    // dense tiles and the residual pattern beside them (in use only when the tiles hold enough of the entries)
    gcn::TileBuffers tiles{};
    gcn::PrepBuffers res{};
    int64_t n_tiles = 0, nnz_dense = 0;
    bool use_tiles = false;
    bool tiles_searched = false;   // nnz_dense is a count, not a default
    // The pattern that the default form of the aggregation gathers over (the residual one with tiles in use, else
    // the whole one) without the columns of vertices outside the train mask: the rows of dLoss/dlogits are zero
    // there, so the last layer's backward aggregation gathers over this one.  Built when it drops enough entries.
    gcn::PrepBuffers bwd{};
    int64_t bwd_nnz = 0;
    bool use_bwd = false;
    // the tile product of an aggregation runs on this stream, beside the gather kernel on the caller's; in the
    // backward pass also a layer's weight gradient, beside the input gradient of the layer below (ev_aux: its end)
    hipStream_t side = nullptr;
    hipEvent_t ev_fork = nullptr, ev_join = nullptr, ev_aux = nullptr;
    ~gcn_graph() {
        if (ev_aux) (void)hipEventDestroy(ev_aux);
        if (ev_fork) (void)hipEventDestroy(ev_fork);
        if (ev_join) (void)hipEventDestroy(ev_join);
        if (side) (void)hipStreamDestroy(side);
    }
    void *x = nullptr;           // (n + 1) x ldf elements of store_dtype, zero padded, last row zero
    int32_t *labels = nullptr;
    uint8_t *mask = nullptr;
};
