// vmoba_workspace_bytes: sizes of the caller-provided workspaces.
#include "common.h"

size_t vmoba_select_workspace_bytes(int B, int Hh, int64_t S, int nb);
size_t vmoba_attn_fwd_workspace_bytes(int B, int Hh, int64_t S, int D, int64_t cap, int dtype);
size_t vmoba_attn_bwd_workspace_bytes(int B, int Hh, int64_t S, int D, int64_t cap, int dtype);

extern "C" size_t vmoba_workspace_bytes(int op, int B, int Hh, int64_t S, int D, int32_t n_blocks,
                                        int64_t nnz_capacity, int dtype) {
    if (B <= 0 || Hh <= 0 || S <= 0 || n_blocks <= 0 || D <= 0 || nnz_capacity < 0) return 0;
    switch (op) {
        case VMOBA_OP_SELECT: return vmoba_select_workspace_bytes(B, Hh, S, n_blocks);
        case VMOBA_OP_ATTN_FWD: return vmoba_attn_fwd_workspace_bytes(B, Hh, S, D, nnz_capacity, dtype);
        case VMOBA_OP_ATTN_BWD: return vmoba_attn_bwd_workspace_bytes(B, Hh, S, D, nnz_capacity, dtype);
        default: return 0;
    }
}

ProfileSlot g_profile[4] = {};

extern "C" int vmoba_profile_events(int slot, void* start_event, void* stop_event) {
    if (slot < 0 || slot >= 4) return VMOBA_ERR_INVALID_ARG;
    g_profile[slot].start = (hipEvent_t)start_event;
    g_profile[slot].stop = (hipEvent_t)stop_event;
    return VMOBA_OK;
}

// vmoba_probe_mfma: measurement aid.  Every wavefront issues `iters` rounds of four independent
// v_mfma_f32_32x32x16_bf16 (nothing else in the loop), so the launch's duration gives the matrix rate this GPU
// sustains at its clock under matrix load: what a kernel made of matrix instructions alone could reach.
__global__ __launch_bounds__(256) void mfma_probe_kernel(long long iters, float* __restrict__ sink) {
    const float seed = (float)(threadIdx.x & 7) * 0.125f;
    f32x4_t lo = {seed, 0.5f, 0.25f, 1.f};
    const bf16x4_t b4 = __builtin_convertvector(lo, bf16x4_t);
    const bf16x8_t a = __builtin_shufflevector(b4, b4, 0, 1, 2, 3, 4, 5, 6, 7), b = a;
    f32x16_t c0, c1, c2, c3;
#pragma unroll
    for (int i = 0; i < 16; ++i) { c0[i] = 0.f; c1[i] = 0.f; c2[i] = 0.f; c3[i] = 0.f; }
    for (long long it = 0; it < iters; ++it) {
        c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c3, 0, 0, 0);
    }
    float r = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) r += c0[i] + c1[i] + c2[i] + c3[i];
    if (r == -1.f) sink[0] = r;          // never true (the sums are >= 0): keeps the loop alive
}

extern "C" int vmoba_probe_mfma(int64_t iters, int workgroups, float* sink, double* flop_out, void* stream) {
    if (iters <= 0 || iters > ((int64_t)1 << 24) || workgroups <= 0 || workgroups > (1 << 16) || !sink || !flop_out)
        return VMOBA_ERR_INVALID_ARG;
    mfma_probe_kernel<<<dim3((unsigned)workgroups), dim3(256), 0, (hipStream_t)stream>>>((long long)iters, sink);
    VMOBA_CHECK_LAUNCH();
    *flop_out = (double)workgroups * 4.0 * (double)iters * 4.0 * 32.0 * 32.0 * 16.0 * 2.0;
    return VMOBA_OK;
}

// vmoba_probe_atomic_rows: measurement aid.  The atomic traffic -- and nothing else -- of a backward pass that would form
// dQ inside the dK/dV kernel: workgroup (run, head) walks a query list of `cnt` rows in 64-row steps and adds one
// 128-float row per listed query into dq[head][row][:] with hardware float atomics (no return value).  `lists` holds
// n_lists lists of cnt ascending rows; run r uses list r % n_lists.
__global__ __launch_bounds__(256) void atomic_rows_probe_kernel(float* __restrict__ dq, const int* __restrict__ lists, int n_lists,
                                                                int cnt, int S) {
    const int head = blockIdx.y;
    const int* lst = lists + (size_t)(blockIdx.x % n_lists) * cnt;
    float* base = dq + (size_t)head * S * 128;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    for (int c0 = 0; c0 < cnt; c0 += 64) {
        for (int r = 0; r < 16; ++r) {
            const int e = c0 + wave * 16 + r;
            if (e >= cnt) break;
            float* row = base + (size_t)lst[e] * 128;
            unsafeAtomicAdd(row + lane, 1.0f);
            unsafeAtomicAdd(row + 64 + lane, 1.0f);
        }
    }
}

extern "C" int vmoba_probe_atomic_rows(float* dq, const int32_t* lists, int n_lists, int cnt, int64_t S, int runs, int heads,
                                       void* stream) {
    if (!dq || !lists || n_lists <= 0 || cnt <= 0 || S <= 0 || S > (1 << 30) || runs <= 0 || runs > (1 << 20) || heads <= 0 ||
        heads > 65535)
        return VMOBA_ERR_INVALID_ARG;
    atomic_rows_probe_kernel<<<dim3((unsigned)runs, (unsigned)heads), dim3(256), 0, (hipStream_t)stream>>>(dq, lists, n_lists, cnt, (int)S);
    VMOBA_CHECK_LAUNCH();
    return VMOBA_OK;
}
