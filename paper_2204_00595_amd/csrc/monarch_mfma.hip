// MFMA kernel family: which shapes have a matrix-core kernel, and which one.
#include "monarch_internal.h"

namespace monarch {

bool mfma_fwd_supported(const Problem& pb)
{
    return fwd_wide_supported(pb) || sq64_supported(pb) || sq16_supported(pb) || tiled_fwd_supported(pb);
}
const char* mfma_fwd_name(const Problem& pb)
{
    if (fwd_wide_supported(pb)) return "mfma_fwd_wide_bf16";
    if (sq64_supported(pb)) return "mfma_fwd_sq64_bf16";
    if (sq16_supported(pb)) return "mfma_fwd_sq16_f32";
    if (tiled_fwd_supported(pb)) return "mfma_fwd_tiled_bf16";
    return "unsupported";
}
int mfma_fwd(const Problem& pb, const void* x, const void* R, const void* L, void* y, hipStream_t st)
{
    if (fwd_wide_supported(pb)) return fwd_wide(pb, x, R, L, y, st);
    if (sq64_supported(pb)) return fwd_sq64(pb, x, R, L, y, st);
    if (sq16_supported(pb)) return fwd_sq16(pb, x, R, L, y, st);
    if (tiled_fwd_supported(pb)) return tiled_fwd(pb, x, R, L, y, st);
    return -2;
}

bool mfma_fwd_ws_supported(const Problem& pb) { return fwd_frag_supported(pb) || sq64_supported(pb) || real32_mfma_supported(pb); }
size_t mfma_fwd_ws_workspace(const Problem& pb)
{
    if (fwd_frag_supported(pb)) return fwd_frag_workspace(pb);
    if (sq64_supported(pb)) return fwd_sq64_workspace(pb);
    if (real32_mfma_supported(pb)) return real32_mfma_workspace(pb, 0);
    return 0;
}
const char* mfma_fwd_ws_name(const Problem& pb)
{
    if (fwd_frag_supported(pb)) return "mfma_fwd_frag_bf16";
    if (sq64_supported(pb)) return "mfma_fwd_sq64_packed_bf16";
    if (real32_mfma_supported(pb)) return "mfma_fwd_stages_f32";
    return "unsupported";
}
int mfma_fwd_ws(const Problem& pb, const void* x, const void* R, const void* L, void* y, void* ws, hipStream_t st)
{
    if (fwd_frag_supported(pb)) return fwd_frag(pb, x, R, L, y, ws, st);
    if (sq64_supported(pb)) return fwd_sq64_ws(pb, x, R, L, y, ws, st);
    if (real32_mfma_supported(pb)) return real32_mfma_fwd(pb, x, R, L, y, ws, st);
    return -2;
}

// Transposed multiply y = x M: the dx stages of the three backward families on their own.
bool mfma_fwd_t_supported(const Problem& pb)
{
    return bwd_wide_supported(pb) || sq64_supported(pb) || sq16_supported(pb) || tiled_fwd_t_supported(pb) || real32_mfma_supported(pb);
}
size_t mfma_fwd_t_workspace(const Problem& pb)
{
    if (bwd_wide_supported(pb)) return fwd_t_wide_workspace(pb);
    if (sq64_supported(pb)) return fwd_t_sq64_workspace(pb);
    if (sq16_supported(pb)) return 0;
    if (tiled_fwd_t_supported(pb)) return tiled_fwd_t_workspace(pb);
    if (real32_mfma_supported(pb)) return real32_mfma_workspace(pb, 2);
    return 0;
}
const char* mfma_fwd_t_name(const Problem& pb)
{
    if (bwd_wide_supported(pb)) return "mfma_fwd_t_wide_bf16";
    if (sq64_supported(pb)) return "mfma_fwd_t_sq64_bf16";
    if (sq16_supported(pb)) return "mfma_fwd_t_sq16_f32";
    if (tiled_fwd_t_supported(pb)) return "mfma_fwd_t_tiled_bf16";
    if (real32_mfma_supported(pb)) return "mfma_fwd_t_stages_f32";
    return "unsupported";
}
int mfma_fwd_t(const Problem& pb, const void* x, const void* R, const void* L, void* y, void* ws, hipStream_t st)
{
    if (bwd_wide_supported(pb)) return fwd_t_wide(pb, x, R, L, y, ws, st);
    if (sq64_supported(pb)) return fwd_t_sq64(pb, x, R, L, y, ws, st);
    if (sq16_supported(pb)) return fwd_t_sq16(pb, x, R, L, y, st);
    if (tiled_fwd_t_supported(pb)) return tiled_fwd_t(pb, x, R, L, y, ws, st);
    if (real32_mfma_supported(pb)) return real32_mfma_fwd_t(pb, x, R, L, y, ws, st);
    return -2;
}

// Which of the forward kernels add pb.bias in their own epilogue (the others need launch_bias_add).
bool mfma_fwd_fuses_bias(const Problem& pb, bool with_ws)
{
    if (with_ws && fwd_frag_supported(pb)) return true;
    if (with_ws && sq64_supported(pb)) return false;
    // mfma_fwd's order of preference: wide, sq64 (no bias epilogue), then sq16 and the shape-generic kernel (both have one)
    return !fwd_wide_supported(pb) && !sq64_supported(pb) && (sq16_supported(pb) || tiled_fwd_supported(pb));
}

bool mfma_bwd_fuses_dbias(const Problem& pb) { return bwd_wide_supported(pb); }

// The nonlinearity of the feed-forward block: applied in the epilogue of the packed-weight forward for the
// four-block layer shapes, and in the dx epilogue of their (recomputing) backward.
bool mfma_fwd_fuses_act(const Problem& pb, bool with_ws) { return with_ws && fwd_frag_supported(pb); }
bool mfma_bwd_fuses_act(const Problem& pb) { return bwd_wide_supported(pb) && !pb.saved; }

bool mfma_bwd_supported(const Problem& pb)
{
    return bwd_wide_supported(pb) || bwd_sq64_supported(pb) || sq16_supported(pb) || tiled_bwd_supported(pb) || real32_mfma_supported(pb);
}
size_t mfma_bwd_workspace(const Problem& pb)
{
    if (bwd_wide_supported(pb)) return bwd_wide_workspace(pb);
    if (bwd_sq64_supported(pb)) return bwd_sq64_workspace(pb);
    if (sq16_supported(pb)) return bwd_sq16_workspace(pb);
    if (tiled_bwd_supported(pb)) return tiled_bwd_workspace(pb);
    if (real32_mfma_supported(pb)) return real32_mfma_workspace(pb, 1);
    return 0;
}
const char* mfma_bwd_name(const Problem& pb)
{
    if (bwd_wide_supported(pb)) return "mfma_bwd_wide_bf16";
    if (bwd_sq64_supported(pb)) return "mfma_bwd_sq64_bf16";
    if (sq16_supported(pb)) return "mfma_bwd_sq16_f32";
    if (tiled_bwd_supported(pb)) return "mfma_bwd_tiled_bf16";
    if (real32_mfma_supported(pb)) return "mfma_bwd_stages_f32";
    return "unsupported";
}
int mfma_bwd(const Problem& pb, const void* dy, const void* x, const void* R, const void* L, void* dx, void* dR,
             void* dL, void* ws, hipStream_t st)
{
    if (bwd_wide_supported(pb)) return bwd_wide(pb, dy, x, R, L, dx, dR, dL, ws, st);
    if (bwd_sq64_supported(pb)) return bwd_sq64(pb, dy, x, R, L, dx, dR, dL, ws, st);
    if (sq16_supported(pb)) return bwd_sq16(pb, dy, x, R, L, dx, dR, dL, ws, st);
    if (tiled_bwd_supported(pb)) return tiled_bwd(pb, dy, x, R, L, dx, dR, dL, ws, st);
    if (real32_mfma_supported(pb)) return real32_mfma_bwd(pb, dy, x, R, L, dx, dR, dL, ws, st);
    return -2;
}

}  // namespace monarch
