// Internal interface between the C-ABI front end and the kernel families.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

namespace monarch {

struct Problem {
    int64_t B;       // batch rows
    int n_in, k, p, q, s;
    int dtype;       // 0 = f32, 1 = bf16
    unsigned flags;  // MONARCH_FLAG_*
    const void* bias = nullptr;  // forward only: n_out values of `dtype` added to every output row (may be null)
    void* saved = nullptr;       // forward: also write the vector between the factors here; backward: read it from here
    void* dbias = nullptr;       // backward only: bias gradient wanted (fp32 when wgrad_f32(), else `dtype`)
    void* colsum_ws = nullptr;   // backward only: colsum_workspace() bytes for the bias gradient's partial rows
    int act = 0;                 // forward only: 1 = the output is gelu(product + bias)
    void* y_pre = nullptr;       // forward with act: the value before the nonlinearity also goes here (may be null)
    const void* x_pre = nullptr; // backward only: the layer's input is gelu(x_pre); dx is returned with respect to x_pre
    int n_out() const { return k * s; }
    int kq() const { return k * q; }
    size_t esize() const { return dtype == 0 ? 4 : 2; }
    bool perm_b() const { return (flags & 2u) != 0; }
    bool wgrad_f32() const { return dtype == 0 || (flags & 1u) != 0; }
    bool ws_packed() const { return (flags & 8u) != 0; }  // monarch_fwd_ws: skip the pack pass
    size_t n_R() const { return (size_t)k * q * p; }
    size_t n_L() const { return (size_t)k * s * q; }
};

// LDS a workgroup may ask for on gfx950 (160 KiB per CU, one workgroup resident).
constexpr size_t kMaxLdsBytes = 160 * 1024;

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Forward kernels of the k = 4 layer shapes: workgroups that share one 64-row tile when a short batch leaves CUs
// without a tile of their own -- as many as keep the launch within one workgroup per CU (256 CUs), at most one
// per stage-2 pass.
static inline int pass_split(int64_t row_tiles, int passes)
{
    const int64_t room = row_tiles > 0 ? 256 / row_tiles : 1;
    return (int)(room < 1 ? 1 : (room > passes ? passes : room));
}

// ---- shape-generic SIMT kernels (any k, p, q, s; both permutation readings) ----
bool generic_fwd_supported(const Problem& pb);
bool generic_bwd_supported(const Problem& pb);
size_t generic_bwd_workspace(const Problem& pb);
int generic_fwd(const Problem& pb, const void* x, const void* R, const void* L, void* y, hipStream_t st);
int generic_bwd(const Problem& pb, const void* dy, const void* x, const void* R, const void* L,
                void* dx, void* dR, void* dL, void* ws, hipStream_t st);

// dense form of the Monarch matrix, (k*s) x n_in row-major (any shape, both readings)
int launch_to_dense(const Problem& pb, const void* R, const void* L, void* M, hipStream_t st);

// bias: y += bias in place (shapes whose forward kernel has no bias epilogue; pb.bias must be set),
// and dbias = column sums of dy (two deterministic passes through `ws` of colsum_workspace bytes)
int launch_bias_add(const Problem& pb, void* y, hipStream_t st);
size_t colsum_workspace(const Problem& pb);
int launch_colsum(const Problem& pb, const void* dy, void* dbias, void* ws, hipStream_t st);
// the feed-forward block's nonlinearity as passes of their own (monarch_act.hip), for the kernel families that do
// not apply it in their epilogues: y (holding the pre-activation) -> y_pre (if not null) and y = gelu(y);
// dx *= gelu'(x_pre)
int launch_gelu_fwd(const Problem& pb, void* y, void* y_pre, hipStream_t st);
int launch_gelu_bwd(const Problem& pb, void* dx, const void* x_pre, hipStream_t st);
struct ColsumJob;
ColsumJob make_colsum_job(const Problem& pb, const void* dy, void* dbias, void* ws);

// projection of a dense n x n matrix (n = m * m) onto the square Monarch matrices (monarch_project.hip)
bool project_supported(int m);
int launch_project(const void* A, void* R, void* L, int m, int dtype, hipStream_t st);

// transposed multiply y = x M, shape-generic (x (B, k*s) -> y (B, k*p))
bool generic_fwd_t_supported(const Problem& pb);
int generic_fwd_t(const Problem& pb, const void* x, const void* R, const void* L, void* y, hipStream_t st);

// complex64 (interleaved fp32 pairs), shape-generic (monarch_complex.hip); Problem.dtype is ignored there
bool complex_fwd_supported(const Problem& pb);
bool complex_bwd_supported(const Problem& pb);
int complex_fwd(const Problem& pb, const void* x, const void* R, const void* L, void* y, hipStream_t st);
// ws == nullptr: dR / dL by fp32 atomics from every row tile; else (complex_bwd_workspace bytes): the batch-major
// operands go through the workspace and one tiled GEMM launch contracts them over the batch
size_t complex_bwd_workspace(const Problem& pb);
int complex_bwd(const Problem& pb, const void* dy, const void* x, const void* R, const void* L, void* dx, void* dR,
                void* dL, void* ws, hipStream_t st);
// y = x conj(M) (the conjugate transpose applied to every row): x (B, k*s) -> y (B, k*p)
bool complex_fwd_h_supported(const Problem& pb);
// matrix-core complex kernels (monarch_stage_mfma.hip): square blocks p = q = s in {16, 32, 64}; every call needs
// complex_mfma_workspace(pb, pass) bytes (pass: 0 forward, 1 backward, 2 conjugate-transpose forward); B > 0
// the same kernels on real fp32 layers with square blocks p = q = s in {32, 64} (any k, both readings); every call
// takes real32_mfma_workspace(pb, pass) bytes (pass: 0 forward, 1 backward, 2 transposed multiply)
bool real32_mfma_supported(const Problem& pb);
size_t real32_mfma_workspace(const Problem& pb, int pass);
int real32_mfma_fwd(const Problem& pb, const void* x, const void* R, const void* L, void* y, void* ws, hipStream_t st);
int real32_mfma_fwd_t(const Problem& pb, const void* x, const void* R, const void* L, void* y, void* ws, hipStream_t st);
int real32_mfma_bwd(const Problem& pb, const void* dy, const void* x, const void* R, const void* L, void* dx, void* dR,
                    void* dL, void* ws, hipStream_t st);
bool complex_mfma_supported(const Problem& pb);
size_t complex_mfma_workspace(const Problem& pb, int pass);
int complex_mfma_fwd(const Problem& pb, const void* x, const void* R, const void* L, void* y, void* ws, hipStream_t st);
int complex_mfma_fwd_h(const Problem& pb, const void* x, const void* R, const void* L, void* y, void* ws, hipStream_t st);
int complex_mfma_bwd(const Problem& pb, const void* dy, const void* x, const void* R, const void* L, void* dx, void* dR,
                     void* dL, void* ws, hipStream_t st);
int complex_fwd_h(const Problem& pb, const void* x, const void* R, const void* L, void* y, hipStream_t st);
int launch_dft_factors(void* R, void* L, int m, int inverse, hipStream_t st);

// ---- MFMA kernels for the shapes they are instantiated for (bf16 / fp32 matrix cores) ----
bool mfma_fwd_supported(const Problem& pb);
bool mfma_bwd_supported(const Problem& pb);
size_t mfma_bwd_workspace(const Problem& pb);
const char* mfma_fwd_name(const Problem& pb);
const char* mfma_bwd_name(const Problem& pb);
int mfma_fwd(const Problem& pb, const void* x, const void* R, const void* L, void* y, hipStream_t st);
// forward with a caller workspace (packed weights): shapes that have such a kernel
bool mfma_fwd_ws_supported(const Problem& pb);
size_t mfma_fwd_ws_workspace(const Problem& pb);
const char* mfma_fwd_ws_name(const Problem& pb);
int mfma_fwd_ws(const Problem& pb, const void* x, const void* R, const void* L, void* y, void* ws, hipStream_t st);
// transposed multiply y = x M (x (B, k*s), y (B, n_in)) on the matrix cores
bool mfma_fwd_t_supported(const Problem& pb);
size_t mfma_fwd_t_workspace(const Problem& pb);
const char* mfma_fwd_t_name(const Problem& pb);
int mfma_fwd_t(const Problem& pb, const void* x, const void* R, const void* L, void* y, void* ws, hipStream_t st);
bool mfma_fwd_fuses_bias(const Problem& pb, bool with_ws);
// the forward applies pb.act (and writes pb.y_pre) in its epilogue / the backward multiplies dx by gelu'(pb.x_pre)
// in its epilogue; else the caller runs launch_gelu_fwd / launch_gelu_bwd afterwards
bool mfma_fwd_fuses_act(const Problem& pb, bool with_ws);
bool mfma_bwd_fuses_act(const Problem& pb);
bool mfma_bwd_fuses_dbias(const Problem& pb);  // the backward computes pb.dbias inside its own launches  // else the caller adds the bias in a second pass
int mfma_bwd(const Problem& pb, const void* dy, const void* x, const void* R, const void* L,
             void* dx, void* dR, void* dL, void* ws, hipStream_t st);

// bf16, k = 4, wide blocks: fused forward on 32x32x16 MFMA (monarch_mfma_fwd_wide.hip)
bool fwd_wide_supported(const Problem& pb);
int fwd_wide(const Problem& pb, const void* x, const void* R, const void* L, void* y, hipStream_t st);

// bf16, k = 4, wide blocks: fused forward with the weights packed in MFMA fragment order into a
// caller-provided workspace (monarch_mfma_fwd_frag.hip)
bool fwd_frag_supported(const Problem& pb);
size_t fwd_frag_workspace(const Problem& pb);
int fwd_frag(const Problem& pb, const void* x, const void* R, const void* L, void* y, void* ws, hipStream_t st);

// bf16, k = 4, wide blocks: the forward can save the vector between the two factors (B x k*q bf16, stage-2
// order) and the backward can take it from there instead of recomputing it (pb.saved on both sides)
bool saved_supported(const Problem& pb);
// bf16, k = 4, wide blocks: backward (monarch_mfma_bwd_wide.hip)
bool bwd_wide_supported(const Problem& pb);
size_t bwd_wide_workspace(const Problem& pb);
int bwd_wide(const Problem& pb, const void* dy, const void* x, const void* R, const void* L, void* dx,
             void* dR, void* dL, void* ws, hipStream_t st);

// bf16, k = 4, wide blocks with long blocks (p >= 768): step 1 as a GEMM of its own, Y1[b][kk*q + j] (B x k*q bf16) from x and the
// packed R of the backward's prep pass (monarch_mfma_y1.hip)
bool y1_gemm_supported(const Problem& pb);
int y1_gemm(const Problem& pb, const void* x, const uint16_t* XF, uint16_t* Y1, hipStream_t st);

// bf16, k = 4, wide blocks: transposed multiply y = x M on the backward's data kernel
size_t fwd_t_wide_workspace(const Problem& pb);
int fwd_t_wide(const Problem& pb, const void* x, const void* R, const void* L, void* y, void* ws, hipStream_t st);

// bf16, square m = 64 (k = q = s = p = 64): fused forward and backward (monarch_mfma_sq64.hip)
bool sq64_supported(const Problem& pb);
int fwd_sq64(const Problem& pb, const void* x, const void* R, const void* L, void* y, hipStream_t st);
size_t fwd_sq64_workspace(const Problem& pb);  // forward on factors packed in fragment order
int fwd_sq64_ws(const Problem& pb, const void* x, const void* R, const void* L, void* y, void* ws, hipStream_t st);
size_t fwd_t_sq64_workspace(const Problem& pb);  // transposed multiply y = x M
int fwd_t_sq64(const Problem& pb, const void* x, const void* R, const void* L, void* y, void* ws, hipStream_t st);
bool bwd_sq64_supported(const Problem& pb);
size_t bwd_sq64_workspace(const Problem& pb);
int bwd_sq64(const Problem& pb, const void* dy, const void* x, const void* R, const void* L, void* dx,
             void* dR, void* dL, void* ws, hipStream_t st);

// fp32, square m = 16 (k = q = s = p = 16): persistent MFMA kernels (monarch_mfma_sq16.hip)
bool sq16_supported(const Problem& pb);
int fwd_sq16(const Problem& pb, const void* x, const void* R, const void* L, void* y, hipStream_t st);
int fwd_t_sq16(const Problem& pb, const void* x, const void* R, const void* L, void* y, hipStream_t st);  // y = x M
size_t bwd_sq16_workspace(const Problem& pb);
int bwd_sq16(const Problem& pb, const void* dy, const void* x, const void* R, const void* L, void* dx,
             void* dR, void* dL, void* ws, hipStream_t st);

// shape-generic bf16 matrix-core kernels (any k; block sizes multiples of 16, the backward 32;
// both permutation readings; the forward adds pb.bias)
bool tiled_fwd_supported(const Problem& pb);
int tiled_fwd(const Problem& pb, const void* x, const void* R, const void* L, void* y, hipStream_t st);
bool tiled_bwd_supported(const Problem& pb);
size_t tiled_bwd_workspace(const Problem& pb);
int tiled_bwd(const Problem& pb, const void* dy, const void* x, const void* R, const void* L, void* dx, void* dR,
              void* dL, void* ws, hipStream_t st);
bool tiled_fwd_t_supported(const Problem& pb);
size_t tiled_fwd_t_workspace(const Problem& pb);
int tiled_fwd_t(const Problem& pb, const void* x, const void* R, const void* L, void* y, void* ws, hipStream_t st);

// Batch-contracted GEMM for the weight gradients (monarch_mfma_wgrad.hip):
//   P[z][g][m][n] = sum over the rows of batch chunk z of  A[row][g, m] * Bm[row][g, n]
// A column (g, m):  a_g * g + m            (or 4*m + g when the four groups are interleaved)
// Bm column (g, n): b_g * g + (n / seg_w) * b_seg + n % seg_w
struct WgradDesc {
    const uint16_t* A;
    int64_t lda;
    int a_g;
    const uint16_t* Bm;
    int64_t ldb;
    int b_g, b_seg, seg_w;
    int M, N, G;
    float* P;        // partial tiles, nz * G * M * N floats (or as many bf16 values in the same space: p_bf16)
    int p_bf16;      // partial tiles are stored rounded to bf16: half the bytes written by the GEMM and read by the
                     // reduction; used when the gradients themselves are returned in bf16
    int64_t rows;
    int rows_per_chunk;
    int deint;       // A holds the four groups interleaved
    void* out;       // reduced result [g][m][col(n)], col(n) = (n % seg_w) * (N / seg_w) + n / seg_w
};
bool wgrad_tile_ok(int M, int N, int seg_w, int* tm, int* tn);
int wgrad_tiles(const WgradDesc& d);  // workgroups per batch chunk (0: shape not supported)
// both GEMMs over the same nz batch chunks (one launch when their tile shapes agree), then
// one launch that sums the chunks of both and writes `out` (fp32 or bf16)
int wgrad_gemm_pair(const WgradDesc& d0, const WgradDesc& d1, int nz, hipStream_t st);
// `cj` (may be null): the second pass of the bias gradient runs as extra workgroups of the same launch
int wgrad_reduce_pair(const WgradDesc& d0, const WgradDesc& d1, bool out_f32, int nz, hipStream_t st,
                      const ColsumJob* cj = nullptr);

// ---- small utility launches shared by the families ----
int launch_fill_zero_f32(float* p, size_t n, hipStream_t st);
int launch_fill_zero_u16(uint16_t* p, size_t n, hipStream_t st);
int launch_f32_to_bf16(const float* src, uint16_t* dst, size_t n, hipStream_t st);
int launch_stream_copy(void* dst, const void* src, size_t nbytes, hipStream_t st);

static inline int hip_status(hipError_t e) { return e == hipSuccess ? 0 : -4; }

// Permission for `kernel` to be launched with up to `bytes` of dynamic LDS on the current device
// (hipFuncAttributeMaxDynamicSharedMemorySize).  The attribute belongs to the (kernel, device) pair and
// never has to shrink, so the runtime is asked only the first time a pair needs it (or needs more);
// later launches cost one table lookup.  Returns hipSuccess or the runtime's error.
hipError_t allow_dynamic_lds(const void* kernel, size_t bytes);

}  // namespace monarch
