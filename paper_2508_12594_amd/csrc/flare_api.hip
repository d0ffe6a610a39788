// C ABI of libflare.so: argument checks, path selection, workspace sizing, timing hooks.
// The operator itself lives in the kernel files; see include/flare.h for the contract.
#include <stdio.h>

#include <atomic>

#include "flare_internal.h"

namespace flare {

// ---- token-axis split -----------------------------------------------------------------------
// Enough chunks that chunks*BH reaches target_blocks, but no chunk shorter than min_len tokens;
// depends only on the shape, so the reduction order (and the result bits) do too.
Split plan_split(int N, int BH, int min_len, int target_blocks)
{
    long long want = (target_blocks + BH - 1) / BH;
    long long max_chunks = ((long long)N + min_len - 1) / min_len;
    if (want > max_chunks) want = max_chunks;
    if (want < 1) want = 1;
    long long len = ((long long)N + want - 1) / want;
    len = (len + 7) / 8 * 8;
    Split s;
    s.chunk_len = (int)len;
    s.chunks = (int)(((long long)N + len - 1) / len);
    return s;
}

// ---- timing hooks ---------------------------------------------------------------------------
namespace {
constexpr int kMaxTimed = 8192;
struct ProfileState {
    bool on = false;
    bool have_events = false;
    int used = 0;
    hipEvent_t start[kMaxTimed];
    hipEvent_t stop[kMaxTimed];
    int kid[kMaxTimed];
};
ProfileState g_prof;
const char *const kKernelNames[KID_COUNT] = {
    "encode_partial", "encode_merge", "decode", "bwd_token_stats", "bwd_prep", "bwd_dz_partial",
    "bwd_dz_merge", "bwd_dq_partial", "bwd_dq_reduce", "bwd_dkdv",
    "bwd_dkdv_2exp", "decode_merge", "spectral_gram", "spectral_reduce", "spectral_eigen",
    "spectral_post", "decode_project"};
}  // namespace

LaunchTimer::LaunchTimer(int kid, hipStream_t s) : slot(-1), stream(s)
{
    if (!g_prof.on || g_prof.used >= kMaxTimed) return;
    slot = g_prof.used++;
    g_prof.kid[slot] = kid;
    (void)hipEventRecord(g_prof.start[slot], stream);
}
LaunchTimer::~LaunchTimer()
{
    if (slot >= 0) (void)hipEventRecord(g_prof.stop[slot], stream);
}

namespace {

// Scratch of flare_forward_static: one copy per GPU, inside the code object.  In host code the name below
// is only a handle for hipGetSymbolAddress; the device address is looked up once per device and kept.
static __device__ __align__(256) unsigned char scratch[FLARE_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];

// Device address of `scratch` on the current device (NULL on a HIP error or a device index beyond the table).
void *static_scratch()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (p) return p;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
    g_scratch_ptr[dev].store(p, std::memory_order_release);   // two threads may both get here: same address
    return p;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_shape(const flare_shape *s)
{
    if (!s) return FLARE_EINVAL;
    if (s->B < 1 || s->H < 1 || s->N < 1 || s->M < 1 || s->d < 1) return FLARE_EINVAL;
    if (s->dtype != FLARE_F32 && s->dtype != FLARE_BF16 && s->dtype != FLARE_F16) return FLARE_EUNSUPPORTED;
    if (s->layout != FLARE_BHND && s->layout != FLARE_BNHD) return FLARE_EUNSUPPORTED;
    if (s->shared_latents != 0 && s->shared_latents != 1) return FLARE_EINVAL;
    if (s->y_f32 != 0 && s->y_f32 != 1) return FLARE_EINVAL;
    if ((s->variant & ~(FLARE_VARIANT_TWO_EXP | FLARE_VARIANT_SEPARATE_DQ)) != 0) return FLARE_EINVAL;
    if (s->y_f32 && (s->dtype == FLARE_F32 || s->M > 2048)) return FLARE_EUNSUPPORTED;   // matrix-core shapes only
    if (s->d != 4 && s->d != 8 && s->d != 16 && s->d != 32) return FLARE_EUNSUPPORTED;
    if ((long long)s->B * s->H > 65535) return FLARE_EUNSUPPORTED;
    // token rows are addressed with a 24-bit multiply (tok_off)
    const long long sn = (s->layout == FLARE_BNHD) ? (long long)s->H * s->d : s->d;
    if (s->N >= (1 << 24) || sn >= (1 << 24) || (long long)s->N * sn >= (1LL << 32)) return FLARE_EUNSUPPORTED;
    return FLARE_OK;
}

}  // namespace
}  // namespace flare

using namespace flare;

extern "C" {

int flare_version(void) { return 400; }   // 0.4.0: flare_shape grew by variant; flare_forward_static

const char *flare_strerror(int status)
{
    switch (status) {
        case FLARE_OK: return "success";
        case FLARE_EINVAL: return "invalid argument (null pointer or non-positive dimension)";
        case FLARE_EUNSUPPORTED: return "unsupported shape, dtype or layout";
        case FLARE_EALIGN: return "pointer is not 16-byte aligned";
        case FLARE_EWORKSPACE: return "workspace missing or too small";
        case FLARE_ELAUNCH: return "HIP runtime rejected a launch";
        case FLARE_ESTATIC: return "shape needs more scratch than the static buffer of flare_forward_static holds";
        default: return "unknown flare status";
    }
}

int flare_workspace_bytes(const flare_shape *shape, size_t *fwd_bytes, size_t *bwd_bytes)
{
    const int rc = check_shape(shape);
    if (rc != FLARE_OK) return rc;
    const ValuPlan p = valu_plan(*shape);
    if (fwd_bytes) {
        *fwd_bytes = p.fwd_bytes;
        if (mfma_supported(*shape)) {   // the encode's partials are dead when the decode starts: one region
            *fwd_bytes = mfma_fwd_bytes(*shape);
            if (mfma_tok_part_bytes(*shape) > *fwd_bytes) *fwd_bytes = mfma_tok_part_bytes(*shape);
        }
    }
    if (bwd_bytes) *bwd_bytes = p.bwd_bytes;
    return FLARE_OK;
}

int flare_encode(const flare_shape *shape, const void *q_lat, const void *k, const void *v, float *z,
                 float *lse_enc, float scale, void *workspace, size_t workspace_bytes, void *stream)
{
    int rc = check_shape(shape);
    if (rc != FLARE_OK) return rc;
    if (!q_lat || !k || !v || !z || !lse_enc) return FLARE_EINVAL;
    if (!aligned16(q_lat) || !aligned16(k) || !aligned16(v) || !aligned16(z) || !aligned16(lse_enc) ||
        !aligned16(workspace))
        return FLARE_EALIGN;
    size_t need = 0;
    flare_workspace_bytes(shape, &need, nullptr);
    if (!workspace || workspace_bytes < need) return FLARE_EWORKSPACE;
    if (mfma_supported(*shape))
        return mfma_encode(*shape, q_lat, k, v, z, lse_enc, scale, workspace, static_cast<hipStream_t>(stream));
    return valu_encode(*shape, q_lat, k, v, z, lse_enc, scale, workspace, static_cast<hipStream_t>(stream));
}

int flare_decode(const flare_shape *shape, const void *q_lat, const void *k, const float *z, void *y,
                 float *lse_dec, float scale, void *workspace, size_t workspace_bytes, void *stream)
{
    int rc = check_shape(shape);
    if (rc != FLARE_OK) return rc;
    if (!q_lat || !k || !z || !y) return FLARE_EINVAL;
    if (!aligned16(q_lat) || !aligned16(k) || !aligned16(z) || !aligned16(y) || !aligned16(lse_dec) ||
        !aligned16(workspace))
        return FLARE_EALIGN;
    if (mfma_supported(*shape)) {
        const size_t need = mfma_tok_part_bytes(*shape);
        if (need != 0 && (!workspace || workspace_bytes < need)) return FLARE_EWORKSPACE;
        return mfma_decode(*shape, q_lat, k, z, y, lse_dec, scale, workspace, static_cast<hipStream_t>(stream));
    }
    return valu_decode(*shape, q_lat, k, z, y, lse_dec, scale, static_cast<hipStream_t>(stream));
}

int flare_forward(const flare_shape *shape, const void *q_lat, const void *k, const void *v, void *y,
                  float *z, float *lse_enc, float *lse_dec, float scale, void *workspace,
                  size_t workspace_bytes, void *stream)
{
    if (!y) return FLARE_EINVAL;
    if (!aligned16(y) || !aligned16(lse_dec)) return FLARE_EALIGN;
    int rc = flare_encode(shape, q_lat, k, v, z, lse_enc, scale, workspace, workspace_bytes, stream);
    if (rc != FLARE_OK) return rc;
    return flare_decode(shape, q_lat, k, z, y, lse_dec, scale, workspace, workspace_bytes, stream);
}

int flare_forward_static(const flare_shape *shape, const void *q_lat, const void *k, const void *v, void *y,
                         float *z, float *lse_enc, float *lse_dec, float scale, void *stream)
{
    const int rc = check_shape(shape);
    if (rc != FLARE_OK) return rc;
    size_t need = 0;
    flare_workspace_bytes(shape, &need, nullptr);
    if (need > FLARE_STATIC_SCRATCH_BYTES) return FLARE_ESTATIC;
    void *ws = static_scratch();
    if (!ws) return FLARE_ELAUNCH;
    return flare_forward(shape, q_lat, k, v, y, z, lse_enc, lse_dec, scale, ws, FLARE_STATIC_SCRATCH_BYTES, stream);
}

int flare_decode_project(const flare_shape *shape, const void *q_lat, const void *k, const float *z,
                         const void *w_out, const float *bias, void *out, void *y, float *lse_dec, float scale,
                         void *stream)
{
    const int rc = check_shape(shape);
    if (rc != FLARE_OK) return rc;
    if (!q_lat || !k || !z || !w_out || !out) return FLARE_EINVAL;
    if (!aligned16(q_lat) || !aligned16(k) || !aligned16(z) || !aligned16(w_out) || !aligned16(bias) ||
        !aligned16(out) || !aligned16(y) || !aligned16(lse_dec))
        return FLARE_EALIGN;
    if (!mfma_project_supported(*shape)) return FLARE_EUNSUPPORTED;
    return mfma_decode_project(*shape, q_lat, k, z, w_out, bias, out, y, lse_dec, scale,
                               static_cast<hipStream_t>(stream));
}

int flare_forward_project(const flare_shape *shape, const void *q_lat, const void *k, const void *v,
                          const void *w_out, const float *bias, void *out, void *y, float *z, float *lse_enc,
                          float *lse_dec, float scale, void *workspace, size_t workspace_bytes, void *stream)
{
    const int rc0 = check_shape(shape);
    if (rc0 != FLARE_OK) return rc0;
    if (!w_out || !out) return FLARE_EINVAL;
    if (!mfma_project_supported(*shape)) return FLARE_EUNSUPPORTED;     // before anything is launched
    if (!aligned16(w_out) || !aligned16(bias) || !aligned16(out) || !aligned16(y) || !aligned16(lse_dec))
        return FLARE_EALIGN;
    const int rc = flare_encode(shape, q_lat, k, v, z, lse_enc, scale, workspace, workspace_bytes, stream);
    if (rc != FLARE_OK) return rc;
    return flare_decode_project(shape, q_lat, k, z, w_out, bias, out, y, lse_dec, scale, stream);
}

int flare_backward(const flare_shape *shape, const void *q_lat, const void *k, const void *v,
                   const void *y, const float *lse_dec, const void *dy, const float *z,
                   const float *lse_enc, float *dq_lat, void *dk, void *dv, float scale, void *workspace,
                   size_t workspace_bytes, void *stream)
{
    int rc = check_shape(shape);
    if (rc != FLARE_OK) return rc;
    if (!q_lat || !k || !v || !dy || !z || !lse_enc || !dq_lat || !dk || !dv) return FLARE_EINVAL;
    if (!aligned16(q_lat) || !aligned16(k) || !aligned16(v) || !aligned16(dy) || !aligned16(z) ||
        !aligned16(lse_enc) || !aligned16(dq_lat) || !aligned16(dk) || !aligned16(dv) || !aligned16(workspace) ||
        !aligned16(y) || !aligned16(lse_dec))
        return FLARE_EALIGN;
    size_t need = 0;
    flare_workspace_bytes(shape, nullptr, &need);
    if (!workspace || workspace_bytes < need) return FLARE_EWORKSPACE;
    return valu_backward(*shape, q_lat, k, v, y, lse_dec, dy, z, lse_enc, dq_lat, dk, dv, scale, workspace,
                         static_cast<hipStream_t>(stream));
}

int flare_spectral_workspace_bytes(const flare_shape *shape, size_t *bytes)
{
    const int rc = check_shape(shape);
    if (rc != FLARE_OK) return rc;
    if (shape->M > 512) return FLARE_EUNSUPPORTED;
    if (bytes) *bytes = spectral_bytes(*shape);
    return FLARE_OK;
}

int flare_spectral(const flare_shape *shape, const void *q_lat, const void *k, const float *lse_enc,
                   const float *lse_dec, float scale, int first, float *eigenvalues, float *z_vec, float *gram,
                   void *workspace, size_t workspace_bytes, void *stream)
{
    const int rc = check_shape(shape);
    if (rc != FLARE_OK) return rc;
    if (shape->M > 512) return FLARE_EUNSUPPORTED;
    if (!q_lat || !k || !lse_enc || !lse_dec || !eigenvalues || !z_vec || first < 0) return FLARE_EINVAL;
    if (!aligned16(q_lat) || !aligned16(k) || !aligned16(lse_enc) || !aligned16(lse_dec) || !aligned16(eigenvalues) ||
        !aligned16(z_vec) || !aligned16(gram) || !aligned16(workspace))
        return FLARE_EALIGN;
    if (!workspace || workspace_bytes < spectral_bytes(*shape)) return FLARE_EWORKSPACE;
    return spectral_run(*shape, q_lat, k, lse_enc, lse_dec, scale, first, eigenvalues, z_vec, gram, workspace,
                        static_cast<hipStream_t>(stream));
}

int flare_profile_enable(int on)
{
    if (on) {
        if (!g_prof.have_events) {
            for (int i = 0; i < kMaxTimed; ++i) {
                if (hipEventCreate(&g_prof.start[i]) != hipSuccess) return FLARE_ELAUNCH;
                if (hipEventCreate(&g_prof.stop[i]) != hipSuccess) return FLARE_ELAUNCH;
            }
            g_prof.have_events = true;
        }
        g_prof.used = 0;
        g_prof.on = true;
    } else {
        g_prof.on = false;
    }
    return FLARE_OK;
}

int flare_profile_kernels(void) { return KID_COUNT; }

const char *flare_profile_name(int kernel_id)
{
    return (kernel_id >= 0 && kernel_id < KID_COUNT) ? kKernelNames[kernel_id] : "";
}

int flare_profile_read(int kernel_id, double *total_ms, int *launches)
{
    if (kernel_id < 0 || kernel_id >= KID_COUNT || !total_ms || !launches) return FLARE_EINVAL;
    double total = 0.0;
    int count = 0;
    for (int i = 0; i < g_prof.used; ++i) {
        if (g_prof.kid[i] != kernel_id) continue;
        if (hipEventSynchronize(g_prof.stop[i]) != hipSuccess) return FLARE_ELAUNCH;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, g_prof.start[i], g_prof.stop[i]) != hipSuccess) return FLARE_ELAUNCH;
        total += ms;
        ++count;
    }
    *total_ms = total;
    *launches = count;
    return FLARE_OK;
}

}  // extern "C"
