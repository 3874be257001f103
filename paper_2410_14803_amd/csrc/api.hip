// C ABI of the A-RIDE scoring library: host-side argument validation and kernel launches.
// Nothing here allocates, frees or waits (aride_status_read excepted, as documented).
#include "aride.h"
#include "aride_device.h"
#include <mutex>

namespace aride {
hipError_t score_logits_launch(const uint16_t*, long long, int, long long, const int*, int, float*,
                               float*, float*, float*, uint32_t*, hipStream_t, hipEvent_t, hipEvent_t);
hipError_t retrace_launch(const float*, const float*, const float*, const float*, const float*,
                          const float*, const int*, int, int, float, float, int, float, float, float*, float*,
                          float*, const PrioArgs*, hipStream_t);
hipError_t mc_returns_launch(const float*, const int*, int, int, float, float*, float*, hipStream_t);
hipError_t priorities_launch(const float*, const float*, const float*, const int*, int, int, float,
                             float, float, float, float, float, int, float*, float*, hipStream_t);
hipError_t update_launch(float*, long long, const long long*, const float*, int, float, const ReplayWs&,
                         hipStream_t);
hipError_t insert_launch(float*, long long, long long, const float*, long long, float, long long*,
                         const ReplayWs&, hipStream_t);
hipError_t sample_launch(const float*, long long, const ReplayWs&, const double*, int, long long*, float*,
                         hipStream_t);

hipError_t actor_launch(const uint16_t*, long long, int, long long, const int*, int, const float*, const float*,
                        const float*, const float*, const float*, const float*, const float*, const float*,
                        float, float, float, int, void*, float*, hipStream_t);

static_assert(sizeof(aride_status) == 24, "status block layout");
static_assert(sizeof(WsHeader) == sizeof(aride_status), "device header mirrors the status block");

__global__ void k_fill_u64(unsigned long long* p, size_t n) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        p[i] = 0ull;
}

static inline size_t index_bytes(int64_t M) { return replay_index_bytes(M); }
static inline bool misaligned(const void* p, size_t a) { return ((uintptr_t)p & (a - 1)) != 0; }

// The first 24 bytes of a workspace header, copied to a caller's device buffer.
__global__ void k_copy_status(const WsHeader* __restrict__ hdr, WsHeader* __restrict__ out) {
    if (threadIdx.x == 0 && blockIdx.x == 0) *out = *hdr;
}

// ---- The workspace of aride_sample_prioritized_static -----------------------------------------
// Device memory that belongs to the library's code object, one copy per GPU, there from the moment
// the code object is loaded until the process ends: header plus replay index for the largest
// capacity that entry point accepts.  In host code the array's name is only a handle for
// hipGetSymbolAddress; every use of the memory goes through the address that call returns.
static_assert(ARIDE_STATIC_MAX_REPLAY <= ARIDE_MAX_REPLAY, "the static workspace serves a legal capacity");
constexpr size_t kScratchBytes = kHeaderBytes + replay_index_bytes(ARIDE_STATIC_MAX_REPLAY);
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[kMaxDevices];   // address of `scratch` on each device, looked up once

// Address of the current device's copy of `scratch`; nullptr when the look-up fails.
static void* scratch_of_current_device() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
        g_scratch_ptr[dev] = p;
    }
    return g_scratch_ptr[dev];
}
}  // namespace aride

using namespace aride;

extern "C" {

int aride_workspace_bytes(int64_t M, size_t* out_bytes) {
    if (!out_bytes) return ARIDE_E_NULL;
    if (M < 0) return ARIDE_E_SHAPE;
    if (M > ARIDE_MAX_REPLAY) return ARIDE_E_RANGE;
    *out_bytes = kHeaderBytes + index_bytes(M);
    return ARIDE_OK;
}

int aride_workspace_init(void* ws, size_t ws_bytes, void* stream) {
    if (!ws || misaligned(ws, 256) || ws_bytes < kHeaderBytes) return ARIDE_E_WORKSPACE;
    const size_t n = ws_bytes / 8;
    size_t want = (n + 255) / 256;
    const unsigned g = (unsigned)(want > 1024 ? 1024 : (want < 1 ? 1 : want));
    hipLaunchKernelGGL(k_fill_u64, dim3(g), dim3(256), 0, (hipStream_t)stream,
                       (unsigned long long*)ws, n);
    return hipGetLastError() == hipSuccess ? ARIDE_OK : ARIDE_E_HIP;
}

int aride_status_read(const void* ws, aride_status* out, void* stream) {
    if (!ws || !out) return ARIDE_E_NULL;
    if (hipMemcpyAsync(out, ws, sizeof(aride_status), hipMemcpyDeviceToHost, (hipStream_t)stream) != hipSuccess)
        return ARIDE_E_HIP;
    if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return ARIDE_E_HIP;
    // the flag is sticky; the error reports the state of the index as it stands now
    return ((out->flags & ARIDE_ST_ZERO_MASS) && out->total == 0) ? ARIDE_E_ZERO_MASS : ARIDE_OK;
}

static int score_logits_checked(const void* logits_bf16, int64_t R, int64_t V, int64_t row_stride,
                                const int32_t* tokens, int32_t A, float* tok_logp, float* tok_ent,
                                float* step_logp, float* step_ent, void* ws, size_t ws_bytes, void* stream,
                                void* sweep_start, void* sweep_stop) {
    if (R < 0 || V <= 0 || A <= 0 || row_stride < V || R % A != 0) return ARIDE_E_SHAPE;
    if (V > 0x7fffffffLL || R > ARIDE_MAX_ROWS) return ARIDE_E_RANGE;
    if (!ws || misaligned(ws, 256)) return ARIDE_E_WORKSPACE;
    if (R == 0) return ARIDE_OK;
    if (!logits_bf16 || !tokens) return ARIDE_E_NULL;
    if (misaligned(logits_bf16, 16) || misaligned(tokens, 4)) return ARIDE_E_ALIGN;
    if ((step_logp && !tok_logp) || (step_ent && !tok_ent)) return ARIDE_E_NULL;
    if (R / A > 0x7fffffffLL / 64) return ARIDE_E_RANGE;
    if (ws_bytes < kHeaderBytes) return ARIDE_E_WORKSPACE;
    hipError_t err = score_logits_launch((const uint16_t*)logits_bf16, R, (int)V, row_stride, tokens, A,
                                         tok_logp, tok_ent, step_logp, step_ent, (uint32_t*)ws,
                                         (hipStream_t)stream, (hipEvent_t)sweep_start, (hipEvent_t)sweep_stop);
    return err == hipSuccess ? ARIDE_OK : ARIDE_E_HIP;
}

int aride_score_logits(const void* logits_bf16, int64_t R, int64_t V, int64_t row_stride,
                       const int32_t* tokens, int32_t A, float* tok_logp, float* tok_ent,
                       float* step_logp, float* step_ent, void* ws, size_t ws_bytes, void* stream) {
    return score_logits_checked(logits_bf16, R, V, row_stride, tokens, A, tok_logp, tok_ent, step_logp, step_ent,
                                ws, ws_bytes, stream, nullptr, nullptr);
}

int aride_score_logits_timed(const void* logits_bf16, int64_t R, int64_t V, int64_t row_stride,
                             const int32_t* tokens, int32_t A, float* tok_logp, float* tok_ent,
                             float* step_logp, float* step_ent, void* ws, size_t ws_bytes, void* stream,
                             void* sweep_start, void* sweep_stop) {
    if (!sweep_start || !sweep_stop) return ARIDE_E_NULL;
    return score_logits_checked(logits_bf16, R, V, row_stride, tokens, A, tok_logp, tok_ent, step_logp, step_ent,
                                ws, ws_bytes, stream, sweep_start, sweep_stop);
}

// Shared by aride_retrace_targets (pcfg == NULL) and aride_retrace_priorities.
static int retrace_checked(const float* logp_pi, const float* logp_mu, const float* reward, const float* value,
                           const float* q, const float* boot, const float* ent, const int32_t* traj_offsets,
                           int64_t B, int64_t N, aride_retrace_cfg cfg, const aride_prio_cfg* pcfg, float* target,
                           float* td, float* rho, float* step_prio, float* traj_prio, void* stream) {
    if (B < 0 || N < 0) return ARIDE_E_SHAPE;
    if (N > ARIDE_MAX_STEPS || B > ARIDE_MAX_TRAJECTORIES) return ARIDE_E_RANGE;
    if (pcfg && (!(pcfg->td_scale != 0.f) || !(pcfg->ent_scale != 0.f))) return ARIDE_E_RANGE;
    if (B == 0) return ARIDE_OK;
    if (!traj_offsets) return ARIDE_E_NULL;
    if (N > 0 && (!logp_pi || !logp_mu || !reward || !value || (pcfg && !ent))) return ARIDE_E_NULL;
    if (cfg.mode != ARIDE_TRACE_RETRACE && cfg.mode != ARIDE_TRACE_VTRACE) return ARIDE_E_RANGE;
    PrioArgs pa;
    if (pcfg)
        pa = PrioArgs{ent, pcfg->w_td, pcfg->w_rho, pcfg->w_ent, 1.f / pcfg->td_scale, 1.f / pcfg->ent_scale,
                      pcfg->eps, pcfg->truncate_rho != 0, step_prio, traj_prio};
    hipError_t err = retrace_launch(logp_pi, logp_mu, reward, value, q, boot, traj_offsets, (int)B,
                                    (int)N, cfg.gamma, cfg.lambda, cfg.mode == ARIDE_TRACE_VTRACE, cfg.rho_bar,
                                    cfg.c_bar, target, td, rho, pcfg ? &pa : nullptr, (hipStream_t)stream);
    return err == hipSuccess ? ARIDE_OK : ARIDE_E_HIP;
}

int aride_retrace_targets(const float* logp_pi, const float* logp_mu, const float* reward,
                          const float* value, const float* q, const float* boot,
                          const int32_t* traj_offsets, int64_t B, int64_t N, aride_retrace_cfg cfg,
                          float* target, float* td, float* rho, void* stream) {
    return retrace_checked(logp_pi, logp_mu, reward, value, q, boot, nullptr, traj_offsets, B, N, cfg, nullptr,
                           target, td, rho, nullptr, nullptr, stream);
}

int aride_retrace_priorities(const float* logp_pi, const float* logp_mu, const float* reward,
                             const float* value, const float* q, const float* boot, const float* ent,
                             const int32_t* traj_offsets, int64_t B, int64_t N, aride_retrace_cfg cfg,
                             aride_prio_cfg pcfg, float* target, float* td, float* rho, float* step_prio,
                             float* traj_prio, void* stream) {
    return retrace_checked(logp_pi, logp_mu, reward, value, q, boot, ent, traj_offsets, B, N, cfg, &pcfg, target,
                           td, rho, step_prio, traj_prio, stream);
}

int aride_mc_returns(const float* reward, const int32_t* traj_offsets, int64_t B, int64_t N, float gamma,
                     float* ret, float* label, void* stream) {
    if (B < 0 || N < 0) return ARIDE_E_SHAPE;
    if (N > ARIDE_MAX_STEPS || B > ARIDE_MAX_TRAJECTORIES) return ARIDE_E_RANGE;
    if (B == 0) return ARIDE_OK;
    if (!traj_offsets || (N > 0 && !reward)) return ARIDE_E_NULL;
    hipError_t err = mc_returns_launch(reward, traj_offsets, (int)B, (int)N, gamma, ret, label,
                                       (hipStream_t)stream);
    return err == hipSuccess ? ARIDE_OK : ARIDE_E_HIP;
}

int aride_compute_priorities(const float* td, const float* rho, const float* ent,
                             const int32_t* traj_offsets, int64_t B, int64_t N, aride_prio_cfg cfg,
                             float* step_prio, float* traj_prio, void* stream) {
    if (B < 0 || N < 0) return ARIDE_E_SHAPE;
    if (N > ARIDE_MAX_STEPS || B > ARIDE_MAX_TRAJECTORIES) return ARIDE_E_RANGE;
    if (!(cfg.td_scale != 0.f) || !(cfg.ent_scale != 0.f)) return ARIDE_E_RANGE;
    if (B == 0) return ARIDE_OK;
    if (!traj_offsets) return ARIDE_E_NULL;
    if (N > 0 && (!td || !rho || !ent)) return ARIDE_E_NULL;
    hipError_t err = priorities_launch(td, rho, ent, traj_offsets, (int)B, (int)N, cfg.w_td, cfg.w_rho,
                                       cfg.w_ent, cfg.td_scale, cfg.ent_scale, cfg.eps,
                                       cfg.truncate_rho != 0, step_prio, traj_prio, (hipStream_t)stream);
    return err == hipSuccess ? ARIDE_OK : ARIDE_E_HIP;
}

static int check_replay(const float* weights, int64_t M, const void* ws, size_t ws_bytes) {
    if (M <= 0) return ARIDE_E_SHAPE;
    if (M > ARIDE_MAX_REPLAY) return ARIDE_E_RANGE;
    if (!weights) return ARIDE_E_NULL;
    if (misaligned(weights, 16)) return ARIDE_E_ALIGN;
    if (!ws || misaligned(ws, 256) || ws_bytes < kHeaderBytes + index_bytes(M)) return ARIDE_E_WORKSPACE;
    return ARIDE_OK;
}

int aride_update_priorities(float* weights, int64_t M, const int64_t* idx, const float* prio,
                            int64_t K, float alpha, void* ws, size_t ws_bytes, void* stream) {
    if (K < 0) return ARIDE_E_SHAPE;
    int rc = check_replay(weights, M, ws, ws_bytes);
    if (rc != ARIDE_OK) return rc;
    if (K >= (1 << 23) || !(alpha >= 0.f)) return ARIDE_E_RANGE;
    if (K > 0 && (!idx || !prio)) return ARIDE_E_NULL;
    if (K > 0 && misaligned(idx, 8)) return ARIDE_E_ALIGN;
    hipError_t err = update_launch(weights, M, (const long long*)idx, prio, (int)K, alpha, replay_ws(ws, M),
                                   (hipStream_t)stream);
    return err == hipSuccess ? ARIDE_OK : ARIDE_E_HIP;
}

int aride_replay_insert(float* weights, int64_t M, int64_t cursor, const float* prio, int64_t K, float alpha,
                        int64_t* slots_out, void* ws, size_t ws_bytes, int64_t* cursor_out, void* stream) {
    if (K < 0) return ARIDE_E_SHAPE;
    int rc = check_replay(weights, M, ws, ws_bytes);
    if (rc != ARIDE_OK) return rc;
    if (cursor < 0 || cursor >= M || !(alpha >= 0.f) || K > kMaxLaunchThreads - 256) return ARIDE_E_RANGE;   // k_insert: a thread per entry, one launch
    if (K > 0 && !prio) return ARIDE_E_NULL;
    if (slots_out && misaligned(slots_out, 8)) return ARIDE_E_ALIGN;
    hipError_t err = insert_launch(weights, M, cursor, prio, K, alpha, (long long*)slots_out, replay_ws(ws, M),
                                   (hipStream_t)stream);
    if (err != hipSuccess) return ARIDE_E_HIP;
    if (cursor_out) *cursor_out = (cursor + K % M) % M;
    return ARIDE_OK;
}

int aride_sample_prioritized(const float* weights, int64_t M, void* ws, size_t ws_bytes,
                             const double* uniforms, int64_t K, int64_t* idx_out, float* prob_out,
                             void* stream) {
    if (K < 0) return ARIDE_E_SHAPE;
    int rc = check_replay(weights, M, ws, ws_bytes);
    if (rc != ARIDE_OK) return rc;
    if (K > 0x7fffffffLL / 64) return ARIDE_E_RANGE;
    if (K == 0) return ARIDE_OK;
    if (!uniforms || !idx_out) return ARIDE_E_NULL;
    if (misaligned(uniforms, 8) || misaligned(idx_out, 8)) return ARIDE_E_ALIGN;
    hipError_t err = sample_launch(weights, M, replay_ws(ws, M), uniforms, (int)K, (long long*)idx_out, prob_out,
                                   (hipStream_t)stream);
    return err == hipSuccess ? ARIDE_OK : ARIDE_E_HIP;
}

int aride_sample_prioritized_static(const float* weights, int64_t M, const double* uniforms, int64_t K,
                                    int64_t* idx_out, float* prob_out, aride_status* status_out,
                                    void* stream) {
    if (K < 0 || M <= 0) return ARIDE_E_SHAPE;
    if (M > ARIDE_STATIC_MAX_REPLAY || K > 0x7fffffffLL / 64) return ARIDE_E_RANGE;
    if (!weights) return ARIDE_E_NULL;
    if (misaligned(weights, 16)) return ARIDE_E_ALIGN;
    if (K == 0) return ARIDE_OK;
    if (!uniforms || !idx_out) return ARIDE_E_NULL;
    if (misaligned(uniforms, 8) || misaligned(idx_out, 8) || (status_out && misaligned(status_out, 8)))
        return ARIDE_E_ALIGN;
    void* ws = scratch_of_current_device();
    if (!ws) return ARIDE_E_HIP;
    hipStream_t st = (hipStream_t)stream;
    // The array keeps what the last call left: the status block starts from zero on every call (a
    // fill kernel, not a memset node, so that the call may be recorded into a graph); the index
    // arrays are all written by the rebuild before anything reads them.
    hipLaunchKernelGGL(k_fill_u64, dim3(1), dim3(64), 0, st, (unsigned long long*)ws, kHeaderBytes / 8);
    if (hipGetLastError() != hipSuccess) return ARIDE_E_HIP;
    const ReplayWs w = replay_ws(ws, M);
    if (update_launch(const_cast<float*>(weights), M, nullptr, nullptr, 0, 0.f, w, st) != hipSuccess)
        return ARIDE_E_HIP;   // K = 0: no weight is written
    if (sample_launch(weights, M, w, uniforms, (int)K, (long long*)idx_out, prob_out, st) != hipSuccess)
        return ARIDE_E_HIP;
    if (status_out) {
        hipLaunchKernelGGL(k_copy_status, dim3(1), dim3(64), 0, st, w.hdr, reinterpret_cast<WsHeader*>(status_out));
        if (hipGetLastError() != hipSuccess) return ARIDE_E_HIP;
    }
    return ARIDE_OK;
}

int aride_actor_loss_grad(const void* logits_bf16, int64_t R, int64_t V, int64_t row_stride,
                          const int32_t* tokens, int32_t A, const float* tok_logp, const float* tok_ent,
                          const float* step_logp, const float* step_ent, const float* rho,
                          const float* target, const float* baseline, const float* penalty,
                          aride_actor_cfg cfg, void* grad, float* loss, void* stream) {
    if (R < 0 || V <= 0 || A <= 0 || row_stride < V || R % A != 0) return ARIDE_E_SHAPE;
    if (V > 0x7fffffffLL || R > ARIDE_MAX_ROWS || R / A > 0x7fffffffLL) return ARIDE_E_RANGE;
    if (!grad && !loss) return ARIDE_OK;
    if (R > 0) {
        if (!rho || !target || !baseline) return ARIDE_E_NULL;
        if (grad && (!logits_bf16 || !tokens || !tok_logp || !tok_ent)) return ARIDE_E_NULL;
        if (loss && (!step_logp || !step_ent)) return ARIDE_E_NULL;
        if (grad && (misaligned(logits_bf16, 16) || misaligned(grad, 16) || misaligned(tokens, 4)))
            return ARIDE_E_ALIGN;
    }
    hipError_t err = actor_launch((const uint16_t*)logits_bf16, R, (int)V, row_stride, tokens, A, tok_logp,
                                  tok_ent, step_logp, step_ent, rho, target, baseline, penalty, cfg.beta,
                                  cfg.lambda_pen, cfg.scale, cfg.grad_f32, grad, loss, (hipStream_t)stream);
    return err == hipSuccess ? ARIDE_OK : ARIDE_E_HIP;
}

}  // extern "C"
