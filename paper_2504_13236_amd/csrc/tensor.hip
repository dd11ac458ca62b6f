// Tiled tensor descriptors (section 2: data cut into tiles; section 5: along any axis).
#include "internal.hpp"

using namespace nnt;

static bool tiling_ok(int32_t ndim, const int64_t* shape, const int64_t* base) {
    if (ndim < 1 || ndim > kMaxDim || !shape || !base) return false;
    for (int a = 0; a < ndim; a++)
        if (shape[a] < 1 || base[a] < 1 || shape[a] > INT32_MAX) return false;
    return true;
}

extern "C" {

int32_t nnt_tiling_ntiles(int32_t ndim, const int64_t* shape, const int64_t* base, int64_t* out) {
    if (!out || !tiling_ok(ndim, shape, base)) return NNT_EINVAL;
    int64_t n = 1;
    for (int a = 0; a < ndim; a++) n *= (shape[a] + base[a] - 1) / base[a];
    *out = n;
    return NNT_OK;
}

int32_t nnt_tiling_tile_shape(int32_t ndim, const int64_t* shape, const int64_t* base,
                              int64_t tile_index, int64_t* shape_out) {
    int64_t n;
    if (!shape_out || nnt_tiling_ntiles(ndim, shape, base, &n) != NNT_OK) return NNT_EINVAL;
    if (tile_index < 0 || tile_index >= n) return NNT_EINVAL;
    for (int a = 0; a < ndim; a++) {
        int64_t g = (shape[a] + base[a] - 1) / base[a];
        int64_t c = tile_index % g;
        tile_index /= g;
        int64_t lo = c * base[a], hi = lo + base[a];
        shape_out[a] = (hi > shape[a] ? shape[a] : hi) - lo;
    }
    return NNT_OK;
}

int32_t nnt_tensor_create(nnt_ctx* ctx, int32_t dtype, int32_t ndim, const int64_t* shape,
                          const int64_t* base, void* const* tile_ptrs, nnt_tensor** out) {
    NNT_CHECK_CTX(ctx);
    if (!out) return NNT_EINVAL;
    *out = nullptr;
    if (dtype != NNT_F32 && dtype != NNT_BF16) return fail(ctx, NNT_EDTYPE, "tensor dtype must be NNT_F32 or NNT_BF16");
    if (!tiling_ok(ndim, shape, base) || !tile_ptrs) return fail(ctx, NNT_EINVAL, "bad shape, base tile or tile pointer table");
    if (ctx->capturing) return fail(ctx, NNT_ESTATE, "tensor creation during capture");
    nnt_tensor* t = new (std::nothrow) nnt_tensor();
    if (!t) return fail(ctx, NNT_ENOMEM, "host allocation failed");
    t->ctx = ctx;
    t->dtype = dtype;
    t->ndim = ndim;
    t->ntiles = 1;
    for (int a = 0; a < kMaxDim; a++) {
        t->shape[a] = a < ndim ? shape[a] : 1;
        t->base[a] = a < ndim ? (base[a] > shape[a] ? shape[a] : base[a]) : 1;
        t->grid[a] = (t->shape[a] + t->base[a] - 1) / t->base[a];
        t->ntiles *= t->grid[a];
    }
    t->tiles.assign(tile_ptrs, tile_ptrs + t->ntiles);
    t->deps.resize(t->ntiles);
    t->d_tiles = nullptr;
    t->id = ctx->next_tensor_id++;
    hipError_t e = hipMalloc((void**)&t->d_tiles, t->ntiles * sizeof(void*));
    if (e == hipSuccess) e = hipMemcpy(t->d_tiles, t->tiles.data(), t->ntiles * sizeof(void*), hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        if (t->d_tiles) (void)hipFree(t->d_tiles);
        delete t;
        return fail(ctx, NNT_EHIP, std::string("tile table upload: ") + hipGetErrorString(e));
    }
    ctx->live_tensors++;
    ctx->table_bytes += t->ntiles * (int64_t)sizeof(void*);
    *out = t;
    return NNT_OK;
}

int32_t nnt_tensor_destroy(nnt_tensor* t) {
    if (!t) return NNT_EINVAL;
    nnt_ctx* ctx = t->ctx;
    // tasks in flight may still read the tile table
    for (int s = 0; s < ctx->n_streams; s++) (void)hipStreamSynchronize(ctx->streams[s]);
    drop_plans_of(ctx, t->id);
    (void)hipFree(t->d_tiles);
    ctx->table_bytes -= t->ntiles * (int64_t)sizeof(void*);
    ctx->live_tensors--;
    delete t;
    return NNT_OK;
}

int32_t nnt_tensor_ntiles(const nnt_tensor* t, int64_t* out) {
    if (!t || !out) return NNT_EINVAL;
    *out = t->ntiles;
    return NNT_OK;
}

int32_t nnt_tensor_tile_shape(const nnt_tensor* t, int64_t tile_index, int64_t* shape_out) {
    if (!t) return NNT_EINVAL;
    return nnt_tiling_tile_shape(t->ndim, t->shape, t->base, tile_index, shape_out);
}

int32_t nnt_tensor_tile_bytes(const nnt_tensor* t, int64_t tile_index, int64_t* out) {
    if (!t || !out || tile_index < 0 || tile_index >= t->ntiles) return NNT_EINVAL;
    *out = t->tile_numel(tile_index) * t->elem_size();
    return NNT_OK;
}

}  // extern "C"
