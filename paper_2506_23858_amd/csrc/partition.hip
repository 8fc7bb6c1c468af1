// vmoba_partition: token -> key-block rearrangement of Sec. 3.2, Eq. 1 (and its inverse).
// Two kernels: an index kernel that writes perm / inv_perm / blk_off from the grid
// description in closed form, and a row-copy kernel that moves 16-byte pieces of the
// (token, head) rows between the caller's order and block order.
#include "common.h"
#include <algorithm>

namespace {

struct GridDesc {
    int T, H, W, bt, bh, bw;
    long long chunk;
    int nT, nH, nW;
    int S, n_blocks;
};

__global__ __launch_bounds__(256) void partition_index_kernel(GridDesc g, int* __restrict__ perm,
                                                              int* __restrict__ inv_perm,
                                                              int* __restrict__ blk_off) {
    int n = blockIdx.x * 256 + threadIdx.x;
    if (n == 0) blk_off[g.n_blocks] = g.S;
    if (n >= g.S) return;
    int pos, j, rank;
    if (g.chunk > 0) {
        pos = n;
        j = (int)(n / g.chunk);
        rank = (int)(n - (long long)j * g.chunk);
    } else {
        int w = n % g.W;
        int h = (n / g.W) % g.H;
        int t = n / (g.W * g.H);
        int it = t / g.bt, ih = h / g.bh, iw = w / g.bw;
        int t0 = it * g.bt, h0 = ih * g.bh, w0 = iw * g.bw;
        int et = min(g.bt, g.T - t0), eh = min(g.bh, g.H - h0), ew = min(g.bw, g.W - w0);
        // tokens in all blocks that precede (it, ih, iw) in row-major block order
        int off = t0 * g.H * g.W + et * (h0 * g.W) + et * eh * w0;
        rank = ((t - t0) * eh + (h - h0)) * ew + (w - w0);
        j = (it * g.nH + ih) * g.nW + iw;
        pos = off + rank;
    }
    perm[pos] = n;
    inv_perm[n] = pos;
    if (rank == 0) blk_off[j] = pos;
}

struct CopyDesc {
    TensorView in[8], out[8];
    int in_bf16[8], out_bf16[8];
    int n_tensors;
};

// One work item = one 16-byte piece of the INPUT row of (b, position/token, head).
// Items are ordered (position, head, piece) with the piece fastest, so a wavefront reads
// whole rows and, in the caller's layout, the heads of one token that lie next to each other.
template <bool INVERSE>
__global__ __launch_bounds__(256) void permute_rows_kernel(CopyDesc d, const int* __restrict__ perm,
                                                           int S, int Hh, int D) {
    const int t = blockIdx.z;
    const int b = blockIdx.y;
    const int in_es = d.in_bf16[t] ? 2 : 4;
    const int pieces = D * in_es / 16;                 // 16-byte pieces per input row
    const long long total = (long long)S * Hh * pieces;
    const TensorView in = d.in[t], out = d.out[t];
    const bool cvt = (!d.in_bf16[t]) && d.out_bf16[t];
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < total;
         i += (long long)gridDim.x * 256) {
        int piece = (int)(i % pieces);
        long long r = i / pieces;
        int h = (int)(r % Hh);
        int p = (int)(r / Hh);
        int tok = perm[p];
        int s_in = INVERSE ? p : tok;
        int s_out = INVERSE ? tok : p;
        const char* src = in.ptr + ((long long)b * in.stride_b + (long long)s_in * in.stride_s +
                                    (long long)h * in.stride_h) * in_es + piece * 16;
        u32x4_t v = *reinterpret_cast<const u32x4_t*>(src);
        if (!cvt) {
            char* dst = out.ptr + ((long long)b * out.stride_b + (long long)s_out * out.stride_s +
                                   (long long)h * out.stride_h) * in_es + piece * 16;
            *reinterpret_cast<u32x4_t*>(dst) = v;
        } else {
            char* dst = out.ptr + ((long long)b * out.stride_b + (long long)s_out * out.stride_s +
                                   (long long)h * out.stride_h) * 2 + piece * 8;
            u32x2_t w;
            w.x = pack_bf16x2(__uint_as_float(v.x), __uint_as_float(v.y));
            w.y = pack_bf16x2(__uint_as_float(v.z), __uint_as_float(v.w));
            *reinterpret_cast<u32x2_t*>(dst) = w;
        }
    }
}

bool grid_ok(const vmoba_grid* g) {
    if (!g) return false;
    if (g->T <= 0 || g->H <= 0 || g->W <= 0) return false;
    if ((int64_t)g->T * g->H * g->W > (int64_t)1 << 30) return false;
    if (g->chunk > 0) return true;
    if (g->chunk < 0) return false;
    return g->bt > 0 && g->bh > 0 && g->bw > 0;
}

}  // namespace

extern "C" int vmoba_layer_kind(int layer) { return ((layer % 3) + 3) % 3; }

extern "C" int vmoba_partition_dims(const vmoba_grid* g, int64_t* S, int32_t* n_blocks) {
    if (!grid_ok(g) || !S || !n_blocks) return VMOBA_ERR_INVALID_ARG;
    int64_t s = (int64_t)g->T * g->H * g->W;
    int64_t nb;
    if (g->chunk > 0) {
        nb = ceil_div64(s, g->chunk);
    } else {
        nb = ceil_div64(g->T, g->bt) * ceil_div64(g->H, g->bh) * ceil_div64(g->W, g->bw);
    }
    if (nb > INT32_MAX) return VMOBA_ERR_UNSUPPORTED;
    *S = s;
    *n_blocks = (int32_t)nb;
    return VMOBA_OK;
}

extern "C" int vmoba_partition(const vmoba_grid* g, int inverse, int B, int Hh, int D, int n_tensors,
                               const vmoba_tensor* in, const vmoba_tensor* out, int32_t* perm,
                               int32_t* inv_perm, int32_t* blk_off, void* stream) {
    int64_t S;
    int32_t nb;
    int rc = vmoba_partition_dims(g, &S, &nb);
    if (rc != VMOBA_OK) return rc;
    if (B <= 0 || Hh <= 0 || n_tensors < 0 || n_tensors > 8) return VMOBA_ERR_INVALID_ARG;
    if (D != 64 && D != 128) return VMOBA_ERR_UNSUPPORTED;
    if (!perm) return VMOBA_ERR_INVALID_ARG;
    const bool build_index = !inverse && (inv_perm || blk_off);   // both null: perm is reused as given
    if (build_index && (!inv_perm || !blk_off)) return VMOBA_ERR_INVALID_ARG;
    if (n_tensors > 0 && (!in || !out)) return VMOBA_ERR_INVALID_ARG;
    CopyDesc cd;
    cd.n_tensors = n_tensors;
    for (int i = 0; i < n_tensors; ++i) {
        if (!tensor_ok(&in[i]) || !tensor_ok(&out[i])) return VMOBA_ERR_INVALID_ARG;
        bool same = in[i].dtype == out[i].dtype;
        bool down = in[i].dtype == VMOBA_F32 && out[i].dtype == VMOBA_BF16;
        if (!same && !down) return VMOBA_ERR_UNSUPPORTED;
        cd.in[i] = make_view(&in[i]);
        cd.out[i] = make_view(&out[i]);
        cd.in_bf16[i] = in[i].dtype == VMOBA_BF16;
        cd.out_bf16[i] = out[i].dtype == VMOBA_BF16;
    }
    hipStream_t st = (hipStream_t)stream;
    if (build_index) {
        GridDesc gd;
        gd.T = g->T; gd.H = g->H; gd.W = g->W;
        gd.bt = g->bt; gd.bh = g->bh; gd.bw = g->bw;
        gd.chunk = g->chunk;
        if (g->chunk > 0) {
            gd.nT = gd.nH = gd.nW = 1;
            gd.bt = gd.bh = gd.bw = 1;
        } else {
            gd.nT = (int)ceil_div64(g->T, g->bt);
            gd.nH = (int)ceil_div64(g->H, g->bh);
            gd.nW = (int)ceil_div64(g->W, g->bw);
        }
        gd.S = (int)S;
        gd.n_blocks = nb;
        partition_index_kernel<<<dim3((unsigned)ceil_div64(S, 256)), dim3(256), 0, st>>>(gd, perm, inv_perm, blk_off);
        VMOBA_CHECK_LAUNCH();
    }
    if (n_tensors > 0) {
        int64_t items = S * Hh * (D * 4 / 16);
        unsigned gx = (unsigned)std::min<int64_t>(ceil_div64(items, 256 * 4), 1 << 20);
        dim3 grid(gx, (unsigned)B, (unsigned)n_tensors);
        VMOBA_PROFILE_BEGIN(3, st);
        if (inverse)
            permute_rows_kernel<true><<<grid, dim3(256), 0, st>>>(cd, perm, (int)S, Hh, D);
        else
            permute_rows_kernel<false><<<grid, dim3(256), 0, st>>>(cd, perm, (int)S, Hh, D);
        VMOBA_PROFILE_END(3, st);
        VMOBA_CHECK_LAUNCH();
    }
    return VMOBA_OK;
}

extern "C" const char* vmoba_status_string(int status) {
    switch (status) {
        case VMOBA_OK: return "ok";
        case VMOBA_ERR_INVALID_ARG: return "invalid argument";
        case VMOBA_ERR_UNSUPPORTED: return "unsupported configuration";
        case VMOBA_ERR_WORKSPACE: return "workspace too small";
        case VMOBA_ERR_CAPACITY: return "nnz capacity exceeded";
        case VMOBA_ERR_HIP: return "HIP error";
        default: return "unknown status";
    }
}
