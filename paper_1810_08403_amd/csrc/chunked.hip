// Streamed (chunked) layer: placeholder until the scheduler lands.
#include "saga_internal.h"

struct ChunkGrid {};

void chunk_grid_destroy(saga_ctx*, ChunkGrid* grid) { delete grid; }

saga_status streamed_forward(saga_ctx* ctx, saga_graph*, const saga_tensor*, const saga_edge_params*, int32_t,
                             const saga_vertex_params*, saga_tensor*)
{
    return ctx->fail(SAGA_ERR_UNSUPPORTED, "streamed path not built yet");
}
