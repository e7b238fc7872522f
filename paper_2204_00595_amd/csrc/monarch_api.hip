// C-ABI front end: argument validation, kernel-family dispatch, workspace sizing.
// Everything here runs on the host; validation never touches the GPU.
#include "../../include/monarch.h"
#include "monarch_internal.h"

#include <mutex>
#include <vector>

using namespace monarch;

namespace monarch {

hipError_t allow_dynamic_lds(const void* kernel, size_t bytes)
{
    struct Slot {
        const void* kernel;
        int device;
        size_t bytes;
    };
    static std::mutex mu;
    static std::vector<Slot> table;  // a few dozen kernels: a linear scan is cheaper than the runtime call it saves
    int device = 0;
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> guard(mu);
    for (Slot& s : table) {
        if (s.kernel != kernel || s.device != device) continue;
        if (s.bytes >= bytes) return hipSuccess;
        e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
        if (e == hipSuccess) s.bytes = bytes;
        return e;
    }
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess) table.push_back(Slot{kernel, device, bytes});
    return e;
}

}  // namespace monarch

namespace {

constexpr unsigned kKnownFlags = MONARCH_FLAG_WGRAD_F32 | MONARCH_FLAG_PERM_B | MONARCH_FLAG_GENERIC | MONARCH_FLAG_WS_PACKED;

// Fills pb; returns MONARCH_OK or MONARCH_ERR_INVALID.
int make_problem(Problem& pb, int64_t batch, int n_in, int k, int q, int s, int dtype, unsigned flags)
{
    if (batch < 0 || n_in <= 0 || k <= 0 || q <= 0 || s <= 0) return MONARCH_ERR_INVALID;
    if (n_in % k != 0) return MONARCH_ERR_INVALID;
    if (dtype != MONARCH_F32 && dtype != MONARCH_BF16) return MONARCH_ERR_INVALID;
    if (flags & ~kKnownFlags) return MONARCH_ERR_INVALID;
    // keep every per-row extent and weight count inside 31 bits
    if ((int64_t)k * q > (1 << 24) || (int64_t)k * s > (1 << 24) || n_in > (1 << 24)) return MONARCH_ERR_UNSUPPORTED;
    if ((int64_t)k * q * (n_in / k) > 0x7fffffffLL || (int64_t)k * s * q > 0x7fffffffLL) return MONARCH_ERR_UNSUPPORTED;
    pb.B = batch;
    pb.n_in = n_in;
    pb.k = k;
    pb.p = n_in / k;
    pb.q = q;
    pb.s = s;
    pb.dtype = dtype;
    pb.flags = flags;
    return MONARCH_OK;
}

enum Family { FAM_NONE = 0, FAM_GENERIC, FAM_MFMA };

Family pick_fwd(const Problem& pb)
{
    if (!(pb.flags & MONARCH_FLAG_GENERIC) && mfma_fwd_supported(pb)) return FAM_MFMA;
    if (generic_fwd_supported(pb)) return FAM_GENERIC;
    return FAM_NONE;
}

Family pick_bwd(const Problem& pb)
{
    if (!(pb.flags & MONARCH_FLAG_GENERIC) && mfma_bwd_supported(pb)) return FAM_MFMA;
    if (generic_bwd_supported(pb)) return FAM_GENERIC;
    return FAM_NONE;
}

// Backward scratch: the kernel family's own area, then the partial rows of the bias gradient.
size_t bwd_kernel_need(const Problem& pb, Family fam)
{
    return align_up(fam == FAM_MFMA ? mfma_bwd_workspace(pb) : generic_bwd_workspace(pb), 256);
}
size_t bwd_need(const Problem& pb, Family fam)
{
    if (fam == FAM_NONE) return (size_t)-1;
    return bwd_kernel_need(pb, fam) + colsum_workspace(pb);
}

bool aligned(const void* p, size_t a) { return ((uintptr_t)p % a) == 0; }

__global__ void empty_kernel() {}

// ---- workspace of monarch_fwd_static: device memory that exists from program load, one copy per GPU ----
constexpr size_t kStaticWorkspaceBytes = MONARCH_STATIC_WORKSPACE_BYTES;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticWorkspaceBytes];

// Device address of `scratch` on the current device.  In host code the array's name is only a handle
// for the runtime; the address a kernel can use comes from hipGetSymbolAddress, asked once per device
// (every GPU holds its own copy at its own address) and kept.
int static_workspace(void** out)
{
    static std::mutex mu;
    static void* ptr[kMaxDevices] = {};
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess) return MONARCH_ERR_HIP;
    if (device < 0 || device >= kMaxDevices) return MONARCH_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> guard(mu);
    if (!ptr[device]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return MONARCH_ERR_HIP;
        ptr[device] = p;
    }
    *out = ptr[device];
    return MONARCH_OK;
}

// The affine layer, optionally followed by the nonlinearity: y = act(x M^T + bias).  Whatever the chosen
// kernel does not do in its own epilogue follows as a pass over y.
int fwd_layer(const void* x, const void* R, const void* L, const void* bias, bool act, void* y_pre, void* y,
              int64_t batch, int n_in, int k, int q, int s, monarch_dtype dtype, void* stream, void* workspace,
              size_t workspace_bytes, unsigned flags)
{
    Problem pb;
    int rc = make_problem(pb, batch, n_in, k, q, s, (int)dtype, flags);
    if (rc) return rc;
    if (flags & MONARCH_FLAG_WGRAD_F32) return MONARCH_ERR_INVALID;  // backward-only flag
    if (!R || !L || ((!x || !y) && batch > 0)) return MONARCH_ERR_INVALID;
    if (!aligned(x, 16) || !aligned(R, 16) || !aligned(L, 16) || !aligned(y, 16) || !aligned(bias, 16) ||
        !aligned(y_pre, 16))
        return MONARCH_ERR_INVALID;
    if (y_pre && y_pre == y) return MONARCH_ERR_INVALID;
    pb.bias = bias;
    hipStream_t st = (hipStream_t)stream;
    const bool generic = (flags & MONARCH_FLAG_GENERIC) != 0;
    bool bias_done = bias == nullptr, act_done = !act;
    if (!generic && mfma_fwd_ws_supported(pb)) {
        if (!workspace || workspace_bytes < mfma_fwd_ws_workspace(pb) || !aligned(workspace, 256))
            return MONARCH_ERR_WORKSPACE;
        if (batch == 0) return MONARCH_OK;
        if (act && mfma_fwd_fuses_act(pb, true)) {
            pb.act = 1;
            pb.y_pre = y_pre;
            act_done = true;
        }
        rc = mfma_fwd_ws(pb, x, R, L, y, workspace, st);
        bias_done = bias_done || mfma_fwd_fuses_bias(pb, true);
    } else {
        pb.flags &= ~MONARCH_FLAG_WS_PACKED;  // no packed-weight kernel: nothing to reuse
        const Family fam = pick_fwd(pb);
        if (fam == FAM_NONE) return MONARCH_ERR_UNSUPPORTED;
        if (batch == 0) return MONARCH_OK;
        if (fam == FAM_GENERIC) {
            rc = generic_fwd(pb, x, R, L, y, st);
            bias_done = true;
        } else {
            rc = mfma_fwd(pb, x, R, L, y, st);
            bias_done = bias_done || mfma_fwd_fuses_bias(pb, false);
        }
    }
    if (rc) return rc;
    if (!bias_done) {
        rc = launch_bias_add(pb, y, st);
        if (rc) return rc;
    }
    if (!act_done) rc = launch_gelu_fwd(pb, y, y_pre, st);
    return rc;
}

// Backward of the affine layer; `saved` (may be null): the vector between the factors kept by monarch_fwd_save;
// `x_pre` (may be null): the layer's input is gelu(x_pre) and dx is wanted with respect to x_pre.
int bwd_layer(const void* dy, const void* x, const void* x_pre, const void* saved, size_t saved_bytes, const void* R,
              const void* L, void* dx, void* dR, void* dL, void* dbias, int64_t batch, int n_in, int k, int q,
              int s, monarch_dtype dtype, void* stream, void* workspace, size_t workspace_bytes, unsigned flags)
{
    Problem pb;
    int rc = make_problem(pb, batch, n_in, k, q, s, (int)dtype, flags);
    if (rc) return rc;
    if (flags & MONARCH_FLAG_WS_PACKED) return MONARCH_ERR_INVALID;  // forward-with-workspace flag
    if (!R || !L || !dR || !dL || ((!dy || !x || !dx) && batch > 0)) return MONARCH_ERR_INVALID;
    if (!aligned(dy, 16) || !aligned(x, 16) || !aligned(R, 16) || !aligned(L, 16) || !aligned(dx, 16) ||
        !aligned(dR, 16) || !aligned(dL, 16) || !aligned(dbias, 16))
        return MONARCH_ERR_INVALID;
    const Family fam = pick_bwd(pb);
    if (fam == FAM_NONE) return MONARCH_ERR_UNSUPPORTED;
    if (saved) {  // ignored by the kernel families that recompute
        const size_t sneed = monarch_saved_bytes(batch, n_in, k, q, s, dtype, flags);
        if (sneed > 0) {
            if (saved_bytes < sneed || !aligned(saved, 16)) return MONARCH_ERR_WORKSPACE;
            pb.saved = const_cast<void*>(saved);
        }
    }
    const size_t need = bwd_need(pb, fam);
    if (!workspace || workspace_bytes < need || !aligned(workspace, 256)) return MONARCH_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    if (dbias) {
        void* cws = (char*)workspace + bwd_kernel_need(pb, fam);
        if (batch > 0 && fam == FAM_MFMA && mfma_bwd_fuses_dbias(pb)) {
            pb.dbias = dbias;  // computed at the tail of the backward's own launches
            pb.colsum_ws = cws;
        } else {
            rc = launch_colsum(pb, dy, dbias, cws, st);
            if (rc) return rc;
        }
    }
    if (fam == FAM_MFMA) {
        const bool fused = x_pre && mfma_bwd_fuses_act(pb);
        if (fused) pb.x_pre = x_pre;
        rc = mfma_bwd(pb, dy, x, R, L, dx, dR, dL, workspace, st);
        if (rc || fused || !x_pre) return rc;
    } else {
        rc = generic_bwd(pb, dy, x, R, L, dx, dR, dL, workspace, st);
        if (rc || !x_pre) return rc;
    }
    return launch_gelu_bwd(pb, dx, x_pre, st);  // the input was gelu(x_pre): chain rule, in place on dx
}

}  // namespace

extern "C" {

int monarch_fwd_ex(const void* x, const void* R, const void* L, void* y, int64_t batch, int n_in, int k,
                   int q, int s, monarch_dtype dtype, void* stream, unsigned flags)
{
    Problem pb;
    int rc = make_problem(pb, batch, n_in, k, q, s, (int)dtype, flags);
    if (rc) return rc;
    if (flags & (MONARCH_FLAG_WGRAD_F32 | MONARCH_FLAG_WS_PACKED)) return MONARCH_ERR_INVALID;  // not forward / not without workspace
    if (!R || !L || ((!x || !y) && batch > 0)) return MONARCH_ERR_INVALID;
    if (!aligned(x, 16) || !aligned(R, 16) || !aligned(L, 16) || !aligned(y, 16)) return MONARCH_ERR_INVALID;
    const Family fam = pick_fwd(pb);
    if (fam == FAM_NONE) return MONARCH_ERR_UNSUPPORTED;
    if (batch == 0) return MONARCH_OK;
    hipStream_t st = (hipStream_t)stream;
    return fam == FAM_MFMA ? mfma_fwd(pb, x, R, L, y, st) : generic_fwd(pb, x, R, L, y, st);
}

int monarch_fwd(const void* x, const void* R, const void* L, void* y, int64_t batch, int n_in, int k,
                int q, int s, monarch_dtype dtype, void* stream)
{
    return monarch_fwd_ex(x, R, L, y, batch, n_in, k, q, s, dtype, stream, 0u);
}

size_t monarch_fwd_workspace_bytes(int64_t batch, int n_in, int k, int q, int s, monarch_dtype dtype,
                                   unsigned flags)
{
    Problem pb;
    if (make_problem(pb, batch, n_in, k, q, s, (int)dtype, flags)) return 0;
    if ((flags & MONARCH_FLAG_GENERIC) || !mfma_fwd_ws_supported(pb)) return 0;
    return mfma_fwd_ws_workspace(pb);
}

int monarch_fwd_ws(const void* x, const void* R, const void* L, void* y, int64_t batch, int n_in, int k,
                   int q, int s, monarch_dtype dtype, void* stream, void* workspace, size_t workspace_bytes,
                   unsigned flags)
{
    Problem pb;
    int rc = make_problem(pb, batch, n_in, k, q, s, (int)dtype, flags);
    if (rc) return rc;
    if ((flags & MONARCH_FLAG_GENERIC) || !mfma_fwd_ws_supported(pb))
        return monarch_fwd_ex(x, R, L, y, batch, n_in, k, q, s, dtype, stream, flags & ~MONARCH_FLAG_WS_PACKED);
    if (flags & MONARCH_FLAG_WGRAD_F32) return MONARCH_ERR_INVALID;  // backward-only flag
    if (!R || !L || ((!x || !y) && batch > 0)) return MONARCH_ERR_INVALID;
    if (!aligned(x, 16) || !aligned(R, 16) || !aligned(L, 16) || !aligned(y, 16)) return MONARCH_ERR_INVALID;
    if (!workspace || workspace_bytes < mfma_fwd_ws_workspace(pb) || !aligned(workspace, 256))
        return MONARCH_ERR_WORKSPACE;
    if (batch == 0) return MONARCH_OK;
    return mfma_fwd_ws(pb, x, R, L, y, workspace, (hipStream_t)stream);
}

int monarch_fwd_static(const void* x, const void* R, const void* L, void* y, int64_t batch, int n_in, int k,
                       int q, int s, monarch_dtype dtype, void* stream, unsigned flags)
{
    if (flags & MONARCH_FLAG_WS_PACKED) return MONARCH_ERR_INVALID;  // the shared array is nobody's to keep between calls
    const size_t need = monarch_fwd_workspace_bytes(batch, n_in, k, q, s, dtype, flags);
    if (need > kStaticWorkspaceBytes) return MONARCH_ERR_WORKSPACE;
    void* ws = nullptr;
    if (need > 0) {
        const int rc = static_workspace(&ws);
        if (rc) return rc;
    }
    // need == 0: monarch_fwd_ws takes the kernels that use no workspace and ignores the pointer
    return monarch_fwd_ws(x, R, L, y, batch, n_in, k, q, s, dtype, stream, ws, need, flags);
}

int monarch_fwd_bias(const void* x, const void* R, const void* L, const void* bias, void* y, int64_t batch,
                     int n_in, int k, int q, int s, monarch_dtype dtype, void* stream, void* workspace,
                     size_t workspace_bytes, unsigned flags)
{
    if (!bias) return monarch_fwd_ws(x, R, L, y, batch, n_in, k, q, s, dtype, stream, workspace, workspace_bytes, flags);
    return fwd_layer(x, R, L, bias, false, nullptr, y, batch, n_in, k, q, s, dtype, stream, workspace, workspace_bytes, flags);
}

int monarch_fwd_bias_gelu(const void* x, const void* R, const void* L, const void* bias, void* y_pre, void* y,
                          int64_t batch, int n_in, int k, int q, int s, monarch_dtype dtype, void* stream,
                          void* workspace, size_t workspace_bytes, unsigned flags)
{
    return fwd_layer(x, R, L, bias, true, y_pre, y, batch, n_in, k, q, s, dtype, stream, workspace, workspace_bytes, flags);
}

size_t monarch_saved_bytes(int64_t batch, int n_in, int k, int q, int s, monarch_dtype dtype, unsigned flags)
{
    Problem pb;
    if (make_problem(pb, batch, n_in, k, q, s, (int)dtype, flags)) return 0;
    if ((flags & MONARCH_FLAG_GENERIC) || !saved_supported(pb)) return 0;
    return align_up((size_t)(batch > 0 ? batch : 1) * pb.kq() * pb.esize(), 256);
}

int monarch_fwd_save(const void* x, const void* R, const void* L, void* y, void* saved, size_t saved_bytes,
                     int64_t batch, int n_in, int k, int q, int s, monarch_dtype dtype, void* stream, unsigned flags)
{
    const size_t need = monarch_saved_bytes(batch, n_in, k, q, s, dtype, flags);
    if (need == 0) return monarch_fwd_ex(x, R, L, y, batch, n_in, k, q, s, dtype, stream, flags);
    Problem pb;
    int rc = make_problem(pb, batch, n_in, k, q, s, (int)dtype, flags);
    if (rc) return rc;
    if (flags & (MONARCH_FLAG_WGRAD_F32 | MONARCH_FLAG_WS_PACKED)) return MONARCH_ERR_INVALID;
    if (!R || !L || ((!x || !y) && batch > 0)) return MONARCH_ERR_INVALID;
    if (!aligned(x, 16) || !aligned(R, 16) || !aligned(L, 16) || !aligned(y, 16)) return MONARCH_ERR_INVALID;
    if (!saved || saved_bytes < need || !aligned(saved, 16)) return MONARCH_ERR_WORKSPACE;
    if (batch == 0) return MONARCH_OK;
    pb.saved = saved;
    return mfma_fwd(pb, x, R, L, y, (hipStream_t)stream);
}

size_t monarch_bwd_workspace_bytes(int64_t batch, int n_in, int k, int q, int s, monarch_dtype dtype,
                                   unsigned flags)
{
    Problem pb;
    if (make_problem(pb, batch, n_in, k, q, s, (int)dtype, flags)) return 0;
    const size_t need = bwd_need(pb, pick_bwd(pb));
    return need == (size_t)-1 ? 0 : need;
}

int monarch_bwd(const void* dy, const void* x, const void* R, const void* L, void* dx, void* dR, void* dL,
                int64_t batch, int n_in, int k, int q, int s, monarch_dtype dtype, void* stream,
                void* workspace, size_t workspace_bytes, unsigned flags)
{
    return monarch_bwd_bias(dy, x, R, L, dx, dR, dL, nullptr, batch, n_in, k, q, s, dtype, stream, workspace,
                            workspace_bytes, flags);
}

int monarch_bwd_bias(const void* dy, const void* x, const void* R, const void* L, void* dx, void* dR, void* dL,
                     void* dbias, int64_t batch, int n_in, int k, int q, int s, monarch_dtype dtype, void* stream,
                     void* workspace, size_t workspace_bytes, unsigned flags)
{
    return monarch_bwd_saved(dy, x, nullptr, 0, R, L, dx, dR, dL, dbias, batch, n_in, k, q, s, dtype, stream, workspace,
                             workspace_bytes, flags);
}

int monarch_bwd_saved(const void* dy, const void* x, const void* saved, size_t saved_bytes, const void* R,
                      const void* L, void* dx, void* dR, void* dL, void* dbias, int64_t batch, int n_in, int k, int q,
                      int s, monarch_dtype dtype, void* stream, void* workspace, size_t workspace_bytes, unsigned flags)
{
    return bwd_layer(dy, x, nullptr, saved, saved_bytes, R, L, dx, dR, dL, dbias, batch, n_in, k, q, s, dtype, stream,
                     workspace, workspace_bytes, flags);
}

int monarch_bwd_bias_gelu_in(const void* dy, const void* x, const void* x_pre, const void* R, const void* L,
                             void* dx_pre, void* dR, void* dL, void* dbias, int64_t batch, int n_in, int k, int q, int s,
                             monarch_dtype dtype, void* stream, void* workspace, size_t workspace_bytes, unsigned flags)
{
    if (!x_pre && batch > 0) return MONARCH_ERR_INVALID;
    if (!aligned(x_pre, 16) || (x_pre && x_pre == dx_pre)) return MONARCH_ERR_INVALID;
    return bwd_layer(dy, x, x_pre, nullptr, 0, R, L, dx_pre, dR, dL, dbias, batch, n_in, k, q, s, dtype, stream,
                     workspace, workspace_bytes, flags);
}

size_t monarch_fwd_t_workspace_bytes(int64_t batch, int n_in, int k, int q, int s, monarch_dtype dtype, unsigned flags)
{
    Problem pb;
    if (make_problem(pb, batch, n_in, k, q, s, (int)dtype, flags)) return 0;
    if ((flags & MONARCH_FLAG_GENERIC) || !mfma_fwd_t_supported(pb)) return 0;
    return mfma_fwd_t_workspace(pb);
}

int monarch_fwd_t(const void* x, const void* R, const void* L, void* y, int64_t batch, int n_in, int k, int q, int s,
                  monarch_dtype dtype, void* stream, void* workspace, size_t workspace_bytes, unsigned flags)
{
    Problem pb;
    int rc = make_problem(pb, batch, n_in, k, q, s, (int)dtype, flags);
    if (rc) return rc;
    if (flags & (MONARCH_FLAG_WGRAD_F32 | MONARCH_FLAG_WS_PACKED)) return MONARCH_ERR_INVALID;  // flags of other calls
    if (!R || !L || ((!x || !y) && batch > 0)) return MONARCH_ERR_INVALID;
    if (!aligned(x, 16) || !aligned(R, 16) || !aligned(L, 16) || !aligned(y, 16)) return MONARCH_ERR_INVALID;
    hipStream_t st = (hipStream_t)stream;
    if (!(flags & MONARCH_FLAG_GENERIC) && mfma_fwd_t_supported(pb)) {
        const size_t need = mfma_fwd_t_workspace(pb);
        if (need > 0 && (!workspace || workspace_bytes < need || !aligned(workspace, 256))) return MONARCH_ERR_WORKSPACE;
        if (batch == 0) return MONARCH_OK;
        return mfma_fwd_t(pb, x, R, L, y, workspace, st);
    }
    if (!generic_fwd_t_supported(pb)) return MONARCH_ERR_UNSUPPORTED;
    if (batch == 0) return MONARCH_OK;
    return generic_fwd_t(pb, x, R, L, y, st);
}

int monarch_to_dense(const void* R, const void* L, void* M, int n_in, int k, int q, int s, monarch_dtype dtype,
                     void* stream, unsigned flags)
{
    Problem pb;
    int rc = make_problem(pb, 1, n_in, k, q, s, (int)dtype, flags);
    if (rc) return rc;
    if (flags & ~MONARCH_FLAG_PERM_B) return MONARCH_ERR_INVALID;  // the other flags select kernels of other calls
    if (!R || !L || !M) return MONARCH_ERR_INVALID;
    if (!aligned(R, 16) || !aligned(L, 16) || !aligned(M, 16)) return MONARCH_ERR_INVALID;
    return launch_to_dense(pb, R, L, M, (hipStream_t)stream);
}

// pass: 0 forward, 1 backward, 2 conjugate-transpose forward.  The matrix-core kernels take the square block sizes
// they are built for whenever a workspace is given; everything else runs the shape-generic kernels.
static size_t c64_workspace(const Problem& pb, int pass)
{
    if (complex_mfma_supported(pb)) return complex_mfma_workspace(pb, pass);
    return pass == 1 ? complex_bwd_workspace(pb) : 0;
}

static int c64_check_workspace(const Problem& pb, int pass, const void* workspace, size_t workspace_bytes)
{
    if (workspace && (workspace_bytes < c64_workspace(pb, pass) || !aligned(workspace, 256))) return MONARCH_ERR_WORKSPACE;
    return MONARCH_OK;
}

size_t monarch_c64_workspace_bytes(int pass, int64_t batch, int n_in, int k, int q, int s, unsigned flags)
{
    Problem pb;
    if (pass < 0 || pass > 2 || make_problem(pb, batch, n_in, k, q, s, MONARCH_F32, flags)) return 0;
    if (flags & ~MONARCH_FLAG_PERM_B) return 0;
    if (!(pass == 0 ? complex_fwd_supported(pb) : pass == 1 ? complex_bwd_supported(pb) : complex_fwd_h_supported(pb))) return 0;
    return c64_workspace(pb, pass);
}

int monarch_fwd_c64_ws(const void* x, const void* R, const void* L, void* y, int64_t batch, int n_in, int k, int q, int s,
                       void* stream, void* workspace, size_t workspace_bytes, unsigned flags)
{
    Problem pb;
    int rc = make_problem(pb, batch, n_in, k, q, s, MONARCH_F32, flags);
    if (rc) return rc;
    if (flags & ~MONARCH_FLAG_PERM_B) return MONARCH_ERR_INVALID;
    if (!R || !L || ((!x || !y) && batch > 0)) return MONARCH_ERR_INVALID;
    if (!aligned(x, 16) || !aligned(R, 16) || !aligned(L, 16) || !aligned(y, 16)) return MONARCH_ERR_INVALID;
    if (!complex_fwd_supported(pb)) return MONARCH_ERR_UNSUPPORTED;
    if ((rc = c64_check_workspace(pb, 0, workspace, workspace_bytes))) return rc;
    if (batch == 0) return MONARCH_OK;
    if (workspace && complex_mfma_supported(pb)) return complex_mfma_fwd(pb, x, R, L, y, workspace, (hipStream_t)stream);
    return complex_fwd(pb, x, R, L, y, (hipStream_t)stream);
}

int monarch_fwd_c64(const void* x, const void* R, const void* L, void* y, int64_t batch, int n_in, int k, int q, int s,
                    void* stream, unsigned flags)
{
    return monarch_fwd_c64_ws(x, R, L, y, batch, n_in, k, q, s, stream, nullptr, 0, flags);
}

int monarch_fwd_h_c64_ws(const void* x, const void* R, const void* L, void* y, int64_t batch, int n_in, int k, int q,
                         int s, void* stream, void* workspace, size_t workspace_bytes, unsigned flags)
{
    Problem pb;
    int rc = make_problem(pb, batch, n_in, k, q, s, MONARCH_F32, flags);
    if (rc) return rc;
    if (flags & ~MONARCH_FLAG_PERM_B) return MONARCH_ERR_INVALID;
    if (!R || !L || ((!x || !y) && batch > 0)) return MONARCH_ERR_INVALID;
    if (!aligned(x, 16) || !aligned(R, 16) || !aligned(L, 16) || !aligned(y, 16)) return MONARCH_ERR_INVALID;
    if (!complex_fwd_h_supported(pb)) return MONARCH_ERR_UNSUPPORTED;
    if ((rc = c64_check_workspace(pb, 2, workspace, workspace_bytes))) return rc;
    if (batch == 0) return MONARCH_OK;
    if (workspace && complex_mfma_supported(pb)) return complex_mfma_fwd_h(pb, x, R, L, y, workspace, (hipStream_t)stream);
    return complex_fwd_h(pb, x, R, L, y, (hipStream_t)stream);
}

int monarch_fwd_h_c64(const void* x, const void* R, const void* L, void* y, int64_t batch, int n_in, int k, int q, int s,
                      void* stream, unsigned flags)
{
    return monarch_fwd_h_c64_ws(x, R, L, y, batch, n_in, k, q, s, stream, nullptr, 0, flags);
}

int monarch_bwd_c64_ws(const void* dy, const void* x, const void* R, const void* L, void* dx, void* dR, void* dL,
                       int64_t batch, int n_in, int k, int q, int s, void* stream, void* workspace,
                       size_t workspace_bytes, unsigned flags)
{
    Problem pb;
    int rc = make_problem(pb, batch, n_in, k, q, s, MONARCH_F32, flags);
    if (rc) return rc;
    if (flags & ~MONARCH_FLAG_PERM_B) return MONARCH_ERR_INVALID;
    if (!R || !L || !dR || !dL || ((!dy || !x || !dx) && batch > 0)) return MONARCH_ERR_INVALID;
    if (!aligned(dy, 16) || !aligned(x, 16) || !aligned(R, 16) || !aligned(L, 16) || !aligned(dx, 16) ||
        !aligned(dR, 16) || !aligned(dL, 16))
        return MONARCH_ERR_INVALID;
    if (!complex_bwd_supported(pb)) return MONARCH_ERR_UNSUPPORTED;
    if ((rc = c64_check_workspace(pb, 1, workspace, workspace_bytes))) return rc;
    if (workspace && batch > 0 && complex_mfma_supported(pb))
        return complex_mfma_bwd(pb, dy, x, R, L, dx, dR, dL, workspace, (hipStream_t)stream);
    return complex_bwd(pb, dy, x, R, L, dx, dR, dL, workspace, (hipStream_t)stream);
}

int monarch_bwd_c64(const void* dy, const void* x, const void* R, const void* L, void* dx, void* dR, void* dL,
                    int64_t batch, int n_in, int k, int q, int s, void* stream, unsigned flags)
{
    return monarch_bwd_c64_ws(dy, x, R, L, dx, dR, dL, batch, n_in, k, q, s, stream, nullptr, 0, flags);
}

int monarch_dft_factors(void* R, void* L, int m, int inverse, void* stream)
{
    if (m <= 0 || !R || !L || !aligned(R, 16) || !aligned(L, 16)) return MONARCH_ERR_INVALID;
    if (m > 1024) return MONARCH_ERR_UNSUPPORTED;  // m^3 factor entries, n = m^2 up to 2^20
    return launch_dft_factors(R, L, m, inverse ? 1 : 0, (hipStream_t)stream);
}

int monarch_project(const void* A, void* R, void* L, int n, int m, monarch_dtype dtype, void* stream, unsigned flags)
{
    if (n <= 0 || m <= 0 || (int64_t)m * m != (int64_t)n) return MONARCH_ERR_INVALID;
    if (dtype != MONARCH_F32 && dtype != MONARCH_BF16) return MONARCH_ERR_INVALID;
    if (flags != 0) return MONARCH_ERR_INVALID;
    if (!A || !R || !L) return MONARCH_ERR_INVALID;
    if (!aligned(A, 16) || !aligned(R, 16) || !aligned(L, 16)) return MONARCH_ERR_INVALID;
    if (!project_supported(m)) return MONARCH_ERR_UNSUPPORTED;
    return launch_project(A, R, L, m, (int)dtype, (hipStream_t)stream);
}

const char* monarch_kernel_name(int pass, int n_in, int k, int q, int s, monarch_dtype dtype, unsigned flags)
{
    Problem pb;
    int rc = make_problem(pb, 1, n_in, k, q, s, (int)dtype, flags);
    if (rc == MONARCH_ERR_UNSUPPORTED) return "unsupported";
    if (rc || pass < 0 || pass > 3) return "invalid";
    if (pass == 3) {
        if (!(flags & MONARCH_FLAG_GENERIC) && mfma_fwd_t_supported(pb)) return mfma_fwd_t_name(pb);
        return generic_fwd_t_supported(pb) ? "generic_fwd_t" : "unsupported";
    }
    const Family fam = pass != 1 ? pick_fwd(pb) : pick_bwd(pb);
    if (pass == 2) return (!(flags & MONARCH_FLAG_GENERIC) && mfma_fwd_ws_supported(pb)) ? mfma_fwd_ws_name(pb) : monarch_kernel_name(0, n_in, k, q, s, dtype, flags);
    if (fam == FAM_GENERIC) return pass == 0 ? "generic_fwd" : "generic_bwd";
    if (fam == FAM_MFMA) return pass == 0 ? mfma_fwd_name(pb) : mfma_bwd_name(pb);
    return "unsupported";
}

int monarch_stream_copy(void* dst, const void* src, size_t nbytes, void* stream)
{
    if (nbytes == 0) return MONARCH_OK;
    if (!dst || !src || nbytes % 16 != 0 || !aligned(dst, 16) || !aligned(src, 16)) return MONARCH_ERR_INVALID;
    const char* d = (const char*)dst;
    const char* s = (const char*)src;
    if (d < s + nbytes && s < d + nbytes) return MONARCH_ERR_INVALID;  // overlap
    return launch_stream_copy(dst, src, nbytes, (hipStream_t)stream);
}

int monarch_launch_probe(void* stream)
{
    hipLaunchKernelGGL(empty_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream);
    return hip_status(hipGetLastError());
}

const char* monarch_status_string(int status)
{
    switch (status) {
        case MONARCH_OK: return "ok";
        case MONARCH_ERR_INVALID: return "invalid argument";
        case MONARCH_ERR_UNSUPPORTED: return "unsupported shape";
        case MONARCH_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case MONARCH_ERR_HIP: return "HIP runtime error";
        default: return "unknown status";
    }
}

int monarch_version(void) { return 100; }

}  // extern "C"
