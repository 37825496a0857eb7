// C ABI of the BitLinear library: argument checks on the host, then launches.
// Declarations and argument semantics: include/bitlinear.h.
#include <stdlib.h>
#include <string.h>

#include <mutex>

#include "../../include/bitlinear.h"
#include "common.h"
#include "kernels.h"

using namespace bl;

namespace {

// ---- launch-time switches (bitlinear_set_tuning) ----------------------------------------
struct TuningField {
    const char* name;
    int Tuning::*field;
};
const TuningField kTuningFields[] = {
    {"decode_nofuse", &Tuning::decode_nofuse},   {"decode_nosplit", &Tuning::decode_nosplit},
    {"decode_tiles", &Tuning::decode_tiles},     {"mid_nosplit", &Tuning::mid_nosplit},
    {"mid_split_tiles", &Tuning::mid_split_tiles}, {"mid_only", &Tuning::mid_only},
    {"prefill_tile", &Tuning::prefill_tile},     {"prefill_grid", &Tuning::prefill_grid},
    {"prefill_xbm", &Tuning::prefill_xbm},
    {"group_slices", &Tuning::group_slices},
    {"quant_wpr", &Tuning::quant_wpr},           {"bwd_ring", &Tuning::bwd_ring},
    {"bwd_grid", &Tuning::bwd_grid},             {"bwd_rowmajor", &Tuning::bwd_rowmajor},
    {"mid_kernel", &Tuning::mid_kernel},
};
Tuning g_tuning{};
bool g_tuning_init = false;

// "name=value,name=value": all fields not named become 0.  false: unknown name or bad syntax
// (then nothing changes).
bool parse_tuning(const char* spec, Tuning& out) {
    Tuning t{};
    const char* p = spec ? spec : "";
    while (*p) {
        const char* eq = strchr(p, '=');
        if (!eq) return false;
        const TuningField* f = nullptr;
        for (const TuningField& c : kTuningFields)
            if (strlen(c.name) == (size_t)(eq - p) && strncmp(c.name, p, eq - p) == 0) f = &c;
        if (!f) return false;
        char* end = nullptr;
        const long v = strtol(eq + 1, &end, 10);
        if (end == eq + 1 || (*end && *end != ',')) return false;
        t.*(f->field) = (int)v;
        p = *end ? end + 1 : end;
    }
    out = t;
    return true;
}

constexpr int64_t kMaxDim = (int64_t)1 << 30;
// The GEMM kernels keep partial sums scaled by up to 2^14 per element of K in int32 and byte
// offsets into a block of rows in 32 bits: both hold up to this K.
constexpr int64_t kMaxGemmK = 65536;
constexpr int kMaxGroups = 64;
constexpr unsigned kKnownFlags = BL_FLAG_SKIP_LN | BL_FLAG_OUT_ACC_I32 | BL_FLAG_BETA_CENTERED;

inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

bool shape_ok(int64_t N, int64_t K) {
    return N > 0 && K > 0 && N <= kMaxDim && K <= kMaxDim && K % 32 == 0 &&
           N * K <= ((int64_t)1 << 40);
}
bool gran_ok(int g) { return g == BL_GAMMA_PER_TOKEN || g == BL_GAMMA_PER_TENSOR; }

size_t tiles_bytes(int64_t rows, int64_t cols) { return (size_t)(tiles_n(rows) * tiles_k(cols)) * 1024; }

// workspace layouts ------------------------------------------------------------
struct QuantWs {
    size_t rowstats, gmax, total;
};
QuantWs quant_ws(int64_t M, int granularity) {
    QuantWs w{};
    size_t off = 0;
    w.rowstats = off;
    off += granularity == BL_GAMMA_PER_TENSOR ? align256((size_t)M * 16) : 0;
    w.gmax = off;  // running maxima [kMaxGroups], then (Eq. 6 per tensor) running minima [kMaxGroups]
    off += 512;
    w.total = off;
    return w;
}
struct ForwardWs {
    size_t codes, gamma, rowsum, quant, split, split_bytes, xhat, total;
};
ForwardWs forward_ws(int64_t M, int64_t N, int64_t K, int granularity) {
    ForwardWs w{};
    size_t off = 0;
    w.codes = off;
    off += align256((size_t)M * (size_t)K);
    w.gamma = off;
    off += align256((size_t)M * 4);
    w.rowsum = off;
    off += align256((size_t)M * 4);
    w.quant = off;
    off += quant_ws(M, granularity).total;
    w.split = off;  // partial sums of a K split (small M, long K), else empty
    w.split_bytes = gemm_split_ws_bytes(M, N, K);
    off += align256(w.split_bytes);
    w.xhat = off;  // one token: the normalised row, fp32 [K] (what the codes were rounded from)
    off += M == 1 ? align256((size_t)K * 4) : 0;
    w.total = off;
    return w;
}

int check_hip(hipError_t e) { return e == hipSuccess ? BL_OK : BL_ERR_HIP; }

// ---- group quantisation (Eq. 13-15) ----------------------------------------------
// 0 = fine, else the status to return
int groups_status(int64_t N, int64_t K, int groups_n, int groups_k) {
    if (groups_n < 1 || groups_k < 1 || groups_n > kMaxGroups || groups_k > kMaxGroups)
        return BL_ERR_SHAPE;
    if (N % groups_n || K % groups_k || (K / groups_k) % 32) return BL_ERR_SHAPE;
    // a 16-row weight tile carries one alpha: row groups must be whole tiles
    if (groups_n > 1 && (N / groups_n) % kTileN) return BL_ERR_UNSUPPORTED;
    return BL_OK;
}
QuantWs quant_ws_grouped(int64_t M, int groups_k, int granularity) {
    return quant_ws(M * groups_k, granularity);
}
// Up to 64 tokens all K-groups run in one launch, each group's int32 sums in a slice of its own
// that a second kernel dequantises and adds (Eq. 13-14).
size_t group_slices_bytes(int64_t M, int64_t N, int groups_k) {
    return groups_k > 1 && M <= 64 ? (size_t)groups_k * (size_t)M * (size_t)N * 4 : 0;
}
ForwardWs forward_ws_grouped(int64_t M, int64_t N, int64_t K, int groups_k, int granularity) {
    ForwardWs w{};
    size_t off = 0;
    w.codes = off;
    off += align256((size_t)M * (size_t)K);
    w.gamma = off;
    off += align256((size_t)M * groups_k * 4);
    w.rowsum = off;
    off += align256((size_t)M * groups_k * 4);
    w.quant = off;
    off += quant_ws_grouped(M, groups_k, granularity).total;
    w.split = off;
    w.split_bytes = group_slices_bytes(M, N, groups_k);
    off += align256(w.split_bytes);
    w.total = off;
    return w;
}
struct LnBackwardWs {
    size_t rowstats, partials, total;
};
LnBackwardWs ln_backward_ws(int64_t M, int64_t K, int groups_k) {
    LnBackwardWs w{};
    size_t off = 0;
    w.rowstats = off;
    off += align256((size_t)M * groups_k * 16);
    w.partials = off;
    off += align256((size_t)ln_backward_chunks(M) * 2 * (size_t)K * 8);
    w.total = off;
    return w;
}
// Eq. 6: codes, then gamma and (xhat field) eta, row sums, the quantiser's own scratch
ForwardWs forward_ws_nonneg(int64_t M, int64_t N, int64_t K, int groups_k, int granularity) {
    ForwardWs w{};
    size_t off = 0;
    w.codes = off;
    off += align256((size_t)M * (size_t)K);
    w.gamma = off;
    off += align256((size_t)M * groups_k * 4);
    w.xhat = off;  // eta, laid out like gamma
    off += align256((size_t)M * groups_k * 4);
    w.rowsum = off;
    off += align256((size_t)M * groups_k * 4);
    w.quant = off;
    off += quant_ws_grouped(M, groups_k, granularity).total;
    w.split = off;
    w.split_bytes = group_slices_bytes(M, N, groups_k);
    off += align256(w.split_bytes);
    w.total = off;
    return w;
}
void plain_fields(GemmArgs& a) {
    a.ldq = a.K;
    a.gstride = 1;
    a.beta_rows = a.N;
    a.beta_stride = 0;
    a.accumulate = false;
}

// ---- scratch memory the library owns (bitlinear_forward_static) ------------------------
// Every GPU the library runs on holds its own copy of this array, at its own address, until
// the process ends.  Its name is only a host-side stand-in: host code uses the device address
// that hipGetSymbolAddress returns, looked up once per device with that device current.
constexpr size_t kScratchBytes = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];
std::mutex g_scratch_mutex;

// device address of `scratch` on the current device; nullptr on failure
void* scratch_address() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = p;
    }
    return g_scratch_ptr[dev];
}

}  // namespace

namespace bl {
// The environment variable is looked at once, at the first launch decision of the process.
const Tuning& tuning() {
    if (!g_tuning_init) {
        g_tuning_init = true;
        parse_tuning(getenv("BITLINEAR_TUNING"), g_tuning);
    }
    return g_tuning;
}
}  // namespace bl

extern "C" {

int bitlinear_set_tuning(const char* spec) {
    g_tuning_init = true;
    return parse_tuning(spec, g_tuning) ? BL_OK : BL_ERR_UNSUPPORTED;
}

size_t bitlinear_packed_bytes(int64_t N, int64_t K, unsigned flags) {
    if (!shape_ok(N, K) || (flags & ~kKnownFlags)) return 0;
    return tiles_bytes(N, K);
}

size_t bitlinear_workspace_bytes(int op, int64_t M, int64_t N, int64_t K, int granularity,
                                 unsigned flags) {
    (void)flags;
    if (!gran_ok(granularity)) return 0;
    switch (op) {
        case BL_OP_PACK:
            if (!shape_ok(N, K)) return 0;
            return align256((size_t)reduce_grid(N * K / 4) * 16);
        case BL_OP_QUANT:
            if (M < 0 || M > kMaxDim || K <= 0 || K % 32) return 0;
            return quant_ws(M, granularity).total;
        case BL_OP_FORWARD:
            if (M < 0 || M > kMaxDim || !shape_ok(N, K)) return 0;
            return forward_ws(M, N, K, granularity).total;
        case BL_OP_BACKWARD:
            if (M < 0 || M > kMaxDim || !shape_ok(N, K)) return 0;
            return backward_workspace_bytes(M, N, K) + 256;
        case BL_OP_LN_BACKWARD:
            if (M < 0 || M > kMaxDim || K <= 0 || K > kMaxDim || K % 32) return 0;
            return ln_backward_ws(M, K, 1).total;
        case BL_OP_FORWARD_NONNEG:
            if (M < 0 || M > kMaxDim || !shape_ok(N, K)) return 0;
            return forward_ws_nonneg(M, N, K, 1, granularity).total;
        case BL_OP_MATMUL:
            if (M < 0 || M > kMaxDim || !shape_ok(N, K)) return 0;
            return gemm_split_ws_bytes(M, N, K);  // 0 for most shapes: nothing is needed
        default:
            return 0;
    }
}

int bitlinear_pack_weights(const float* W, int64_t N, int64_t K, unsigned flags, void* packed,
                           float* alpha, float* beta, void* workspace, size_t workspace_bytes,
                           void* stream) {
    if (!shape_ok(N, K)) return BL_ERR_SHAPE;
    if (flags & ~BL_FLAG_BETA_CENTERED) return BL_ERR_UNSUPPORTED;
    if (!W || !packed || !alpha || !beta) return BL_ERR_NULL;
    const size_t need = bitlinear_workspace_bytes(BL_OP_PACK, 0, N, K, 0, flags);
    if (!workspace || workspace_bytes < need) return BL_ERR_WORKSPACE;
    return check_hip(launch_pack(W, N, K, K, (flags & BL_FLAG_BETA_CENTERED) != 0,
                                 (uint32_t*)packed, alpha, beta, (double*)workspace,
                                 (hipStream_t)stream));
}

int bitlinear_packed_to_canonical(const void* packed, int64_t N, int64_t K, uint32_t* canonical,
                                  void* stream) {
    if (!shape_ok(N, K)) return BL_ERR_SHAPE;
    if (!packed || !canonical) return BL_ERR_NULL;
    return check_hip(launch_to_canonical((const uint32_t*)packed, N, K, canonical, K / 32,
                                         (hipStream_t)stream));
}

int bitlinear_quant_act(const float* X, int64_t M, int64_t K, const float* ln_gain,
                        const float* ln_bias, float ln_eps, int granularity, unsigned flags,
                        int8_t* codes, float* gamma, int32_t* rowsum, float* xhat_dump,
                        void* workspace, size_t workspace_bytes, void* stream) {
    if (M < 0 || M > kMaxDim || K <= 0 || K > kMaxDim || K % 32) return BL_ERR_SHAPE;
    if (!gran_ok(granularity) || (flags & ~BL_FLAG_SKIP_LN)) return BL_ERR_UNSUPPORTED;
    if (!quant_supported(K)) return BL_ERR_UNSUPPORTED;
    if (M == 0) return BL_OK;  // nothing to read or write: pointers may be NULL
    if (!X || !codes || !gamma) return BL_ERR_NULL;
    const QuantWs ws = quant_ws(M, granularity);
    if (!workspace || workspace_bytes < ws.total) return BL_ERR_WORKSPACE;
    QuantArgs a{};
    a.X = X; a.M = M; a.K = K; a.gain = ln_gain; a.bias = ln_bias; a.eps = ln_eps;
    a.skip_ln = (flags & BL_FLAG_SKIP_LN) != 0;
    a.per_tensor = granularity == BL_GAMMA_PER_TENSOR;
    a.codes = codes; a.gamma = gamma; a.rowsum = rowsum; a.xhat_dump = xhat_dump;
    a.rowstats = (double*)((char*)workspace + ws.rowstats);
    a.gmax_bits = (uint32_t*)((char*)workspace + ws.gmax);
    a.gmin_bits = a.gmax_bits + kMaxGroups;
    a.groups = 1;
    return check_hip(launch_quant(a, (hipStream_t)stream));
}

int bitlinear_matmul(const int8_t* codes, const float* gamma, const int32_t* rowsum, int64_t M,
                     int64_t K, const void* packed, int64_t N, const float* beta, int granularity,
                     unsigned flags, float* Y, void* workspace, size_t workspace_bytes,
                     void* stream) {
    if (M < 0 || M > kMaxDim || !shape_ok(N, K)) return BL_ERR_SHAPE;
    if (!gran_ok(granularity) || (flags & ~BL_FLAG_OUT_ACC_I32)) return BL_ERR_UNSUPPORTED;
    if (K > kMaxGemmK) return BL_ERR_UNSUPPORTED;
    if (M == 0) return BL_OK;
    if (!codes || !gamma || !rowsum || !packed || !beta || !Y) return BL_ERR_NULL;
    GemmArgs a{};
    a.codes = codes; a.gamma = gamma; a.rowsum = rowsum; a.M = M; a.K = K; a.N = N;
    a.packed = (const uint32_t*)packed; a.beta = beta;
    a.per_tensor = granularity == BL_GAMMA_PER_TENSOR;
    a.out_acc = (flags & BL_FLAG_OUT_ACC_I32) != 0;
    a.Y = Y;
    plain_fields(a);
    a.split_ws = (int32_t*)workspace;  // optional: without it K is never split
    a.split_ws_bytes = workspace ? workspace_bytes : 0;
    if (M <= 16) return check_hip(launch_gemm_decode(a, (hipStream_t)stream));
    return check_hip(launch_gemm_prefill(a, (hipStream_t)stream));
}

int bitlinear_forward(const float* X, int64_t M, int64_t K, const void* packed, int64_t N,
                      const float* beta, const float* ln_gain, const float* ln_bias, float ln_eps,
                      int granularity, unsigned flags, float* Y, void* workspace,
                      size_t workspace_bytes, void* stream) {
    if (M < 0 || M > kMaxDim || !shape_ok(N, K)) return BL_ERR_SHAPE;
    if (!gran_ok(granularity) || (flags & ~(BL_FLAG_SKIP_LN | BL_FLAG_OUT_ACC_I32)))
        return BL_ERR_UNSUPPORTED;
    if (K > kMaxGemmK) return BL_ERR_UNSUPPORTED;
    if (M == 0) return BL_OK;
    if (!X || !packed || !beta || !Y) return BL_ERR_NULL;
    const ForwardWs ws = forward_ws(M, N, K, granularity);
    if (!workspace || workspace_bytes < ws.total) return BL_ERR_WORKSPACE;
    char* base = (char*)workspace;
    int8_t* codes = (int8_t*)(base + ws.codes);
    float* gamma = (float*)(base + ws.gamma);
    int32_t* rowsum = (int32_t*)(base + ws.rowsum);
    // one token: the GEMM kernel quantises the row itself and the layer is one launch (codes,
    // gamma and rowsum still land in the workspace)
    const bool fuse = gemm_decode_fuses_quant(M, K, N);
    if (!fuse) {
        int rc = bitlinear_quant_act(X, M, K, ln_gain, ln_bias, ln_eps, granularity,
                                     flags & BL_FLAG_SKIP_LN, codes, gamma, rowsum,
                                     M == 1 ? (float*)(base + ws.xhat) : nullptr,
                                     base + ws.quant, ws.split - ws.quant, stream);
        if (rc != BL_OK) return rc;
    }
    GemmArgs a{};
    if (fuse) {
        a.x_row = X; a.ln_gain = ln_gain; a.ln_bias = ln_bias; a.ln_eps = ln_eps;
        a.skip_ln = (flags & BL_FLAG_SKIP_LN) != 0;
        a.codes_out = codes; a.gamma_out = gamma; a.rowsum_out = rowsum;
        a.xhat_out = (float*)(base + ws.xhat);
    }
    a.codes = codes; a.gamma = gamma; a.rowsum = rowsum; a.M = M; a.K = K; a.N = N;
    a.packed = (const uint32_t*)packed; a.beta = beta;
    a.per_tensor = granularity == BL_GAMMA_PER_TENSOR;
    a.out_acc = (flags & BL_FLAG_OUT_ACC_I32) != 0;
    a.Y = Y;
    plain_fields(a);
    a.split_ws = ws.split_bytes ? (int32_t*)(base + ws.split) : nullptr;
    a.split_ws_bytes = ws.split_bytes;
    if (M <= 16) return check_hip(launch_gemm_decode(a, (hipStream_t)stream));
    return check_hip(launch_gemm_prefill(a, (hipStream_t)stream));
}

int bitlinear_forward_static(const float* X, int64_t M, int64_t K, const void* packed, int64_t N,
                             const float* beta, const float* ln_gain, const float* ln_bias,
                             float ln_eps, int granularity, unsigned flags, float* Y,
                             void* stream) {
    if (M < 0 || M > kMaxDim || !shape_ok(N, K)) return BL_ERR_SHAPE;
    if (!gran_ok(granularity) || (flags & ~(BL_FLAG_SKIP_LN | BL_FLAG_OUT_ACC_I32)))
        return BL_ERR_UNSUPPORTED;
    if (K > kMaxGemmK) return BL_ERR_UNSUPPORTED;
    // the same workspace as bitlinear_forward's, inside the library's own array or not at all
    if (forward_ws(M, N, K, granularity).total > kScratchBytes) return BL_ERR_UNSUPPORTED;
    if (M == 0) return BL_OK;
    if (!X || !packed || !beta || !Y) return BL_ERR_NULL;
    void* ws = scratch_address();
    if (!ws) return BL_ERR_HIP;
    // nothing in the workspace has to start at zero: the kernels write every byte they later
    // read (the running maximum of a per-tensor gamma is cleared by a fill kernel of its own)
    return bitlinear_forward(X, M, K, packed, N, beta, ln_gain, ln_bias, ln_eps, granularity, flags,
                             Y, ws, kScratchBytes, stream);
}

int bitlinear_forward_workspace_layout(int64_t M, int64_t N, int64_t K, int granularity,
                                       size_t offsets[4]) {
    if (M < 0 || M > kMaxDim || !shape_ok(N, K)) return BL_ERR_SHAPE;
    if (!gran_ok(granularity) || K > kMaxGemmK) return BL_ERR_UNSUPPORTED;
    if (!offsets) return BL_ERR_NULL;
    const ForwardWs ws = forward_ws(M, N, K, granularity);
    offsets[0] = ws.codes;
    offsets[1] = ws.gamma;
    offsets[2] = ws.rowsum;
    offsets[3] = M == 1 ? ws.xhat : (size_t)-1;
    return BL_OK;
}

// ---- Group Quantization and Normalization (Eq. 13-15) ----------------------------------

size_t bitlinear_packed_bytes_grouped(int64_t N, int64_t K, int groups_n, int groups_k) {
    if (!shape_ok(N, K) || groups_status(N, K, groups_n, groups_k) != BL_OK) return 0;
    return (size_t)groups_k * tiles_bytes(N, K / groups_k);
}

size_t bitlinear_workspace_bytes_grouped(int op, int64_t M, int64_t N, int64_t K, int groups_n,
                                         int groups_k, int granularity) {
    if (!gran_ok(granularity) || !shape_ok(N, K) || M < 0 || M > kMaxDim) return 0;
    if (groups_status(N, K, groups_n, groups_k) != BL_OK) return 0;
    switch (op) {
        case BL_OP_PACK:
            return align256((size_t)reduce_grid(N * K / 4) * 16);
        case BL_OP_QUANT:
            return quant_ws_grouped(M, groups_k, granularity).total;
        case BL_OP_FORWARD:
            return forward_ws_grouped(M, N, K, groups_k, granularity).total;
        case BL_OP_LN_BACKWARD:
            return ln_backward_ws(M, K, groups_k).total;
        case BL_OP_FORWARD_NONNEG:
            return forward_ws_nonneg(M, N, K, groups_k, granularity).total;
        default:
            return 0;
    }
}

int bitlinear_pack_weights_grouped(const float* W, int64_t N, int64_t K, int groups_n,
                                   int groups_k, unsigned flags, void* packed, float* alpha,
                                   float* beta, void* workspace, size_t workspace_bytes,
                                   void* stream) {
    if (!shape_ok(N, K)) return BL_ERR_SHAPE;
    if (int st = groups_status(N, K, groups_n, groups_k)) return st;
    if (flags & ~BL_FLAG_BETA_CENTERED) return BL_ERR_UNSUPPORTED;
    if (!W || !packed || !alpha || !beta) return BL_ERR_NULL;
    const size_t need = bitlinear_workspace_bytes_grouped(BL_OP_PACK, 0, N, K, groups_n, groups_k, 0);
    if (!workspace || workspace_bytes < need) return BL_ERR_WORKSPACE;
    const int64_t Ng = N / groups_n, Kg = K / groups_k;
    const size_t blob_dwords = tiles_bytes(N, Kg) / 4;
    for (int gk = 0; gk < groups_k; ++gk)
        for (int gn = 0; gn < groups_n; ++gn) {
            // block (gn, gk): rows gn*Ng .., columns gk*Kg ..; its tiles are rows gn*Ng/16 .. of
            // K-group gk's blob
            uint32_t* dst = (uint32_t*)packed + gk * blob_dwords +
                            tile_dword_offset(gn * Ng / kTileN, 0, tiles_k(Kg));
            const int idx = gn * groups_k + gk;
            hipError_t e = launch_pack(W + gn * Ng * K + gk * Kg, Ng, Kg, K,
                                       (flags & BL_FLAG_BETA_CENTERED) != 0, dst, alpha + idx,
                                       beta + idx, (double*)workspace, (hipStream_t)stream);
            if (e != hipSuccess) return BL_ERR_HIP;
        }
    return BL_OK;
}

int bitlinear_packed_to_canonical_grouped(const void* packed, int64_t N, int64_t K, int groups_k,
                                          uint32_t* canonical, void* stream) {
    if (!shape_ok(N, K)) return BL_ERR_SHAPE;
    if (int st = groups_status(N, K, 1, groups_k)) return st;
    if (!packed || !canonical) return BL_ERR_NULL;
    const int64_t Kg = K / groups_k;
    const size_t blob_dwords = tiles_bytes(N, Kg) / 4;
    for (int gk = 0; gk < groups_k; ++gk) {
        hipError_t e = launch_to_canonical((const uint32_t*)packed + gk * blob_dwords, N, Kg,
                                           canonical + gk * (Kg / 32), K / 32, (hipStream_t)stream);
        if (e != hipSuccess) return BL_ERR_HIP;
    }
    return BL_OK;
}

// Eq. 14-15 for either quantiser: eta == nullptr: Eq. 4; else Eq. 6 with eta laid out like gamma
static int quant_act_grouped_impl(const float* X, int64_t M, int64_t K, int groups_k,
                                  const float* ln_gain, const float* ln_bias, float ln_eps,
                                  int granularity, unsigned flags, bool nonneg, int8_t* codes,
                                  float* gamma, float* eta, int32_t* rowsum, float* xhat_dump,
                                  void* workspace, size_t workspace_bytes, void* stream) {
    if (M < 0 || M > kMaxDim || K <= 0 || K > kMaxDim || K % 32) return BL_ERR_SHAPE;
    if (groups_k < 1 || groups_k > kMaxGroups || K % groups_k || (K / groups_k) % 32)
        return BL_ERR_SHAPE;
    if (!gran_ok(granularity) || (flags & ~BL_FLAG_SKIP_LN)) return BL_ERR_UNSUPPORTED;
    const int64_t Kg = K / groups_k;
    if (!quant_supported(Kg) || M * groups_k > kMaxDim) return BL_ERR_UNSUPPORTED;
    if (M == 0) return BL_OK;
    if (!X || !codes || !gamma || (nonneg && !eta)) return BL_ERR_NULL;
    const QuantWs ws = quant_ws_grouped(M, groups_k, granularity);
    const bool need_ws = granularity == BL_GAMMA_PER_TENSOR;
    if (need_ws && (!workspace || workspace_bytes < ws.total)) return BL_ERR_WORKSPACE;
    // a token's K-groups are consecutive rows of a [M * groups_k, Kg] matrix
    QuantArgs a{};
    a.X = X; a.M = M * groups_k; a.K = Kg; a.gain = ln_gain; a.bias = ln_bias; a.eps = ln_eps;
    a.skip_ln = (flags & BL_FLAG_SKIP_LN) != 0;
    a.per_tensor = granularity == BL_GAMMA_PER_TENSOR;
    a.codes = codes; a.gamma = gamma; a.rowsum = rowsum; a.xhat_dump = xhat_dump;
    if (need_ws) {
        a.rowstats = (double*)((char*)workspace + ws.rowstats);
        a.gmax_bits = (uint32_t*)((char*)workspace + ws.gmax);
        a.gmin_bits = a.gmax_bits + kMaxGroups;
    }
    a.groups = groups_k;
    a.nonneg = nonneg;
    a.eta = eta;
    return check_hip(launch_quant(a, (hipStream_t)stream));
}

int bitlinear_quant_act_grouped(const float* X, int64_t M, int64_t K, int groups_k,
                                const float* ln_gain, const float* ln_bias, float ln_eps,
                                int granularity, unsigned flags, int8_t* codes, float* gamma,
                                int32_t* rowsum, float* xhat_dump, void* workspace,
                                size_t workspace_bytes, void* stream) {
    return quant_act_grouped_impl(X, M, K, groups_k, ln_gain, ln_bias, ln_eps, granularity, flags,
                                  false, codes, gamma, nullptr, rowsum, xhat_dump, workspace,
                                  workspace_bytes, stream);
}

int bitlinear_quant_act_grouped_nonneg(const float* X, int64_t M, int64_t K, int groups_k,
                                       const float* ln_gain, const float* ln_bias, float ln_eps,
                                       int granularity, unsigned flags, int8_t* codes, float* gamma,
                                       float* eta, int32_t* rowsum, float* xhat_dump,
                                       void* workspace, size_t workspace_bytes, void* stream) {
    return quant_act_grouped_impl(X, M, K, groups_k, ln_gain, ln_bias, ln_eps, granularity, flags,
                                  true, codes, gamma, eta, rowsum, xhat_dump, workspace,
                                  workspace_bytes, stream);
}

// Eq. 13-15 for either quantiser: wsum == nullptr: Eq. 4; else Eq. 6 with wsum [groups_k][N]
static int forward_grouped_impl(const float* X, int64_t M, int64_t K, const void* packed, int64_t N,
                                int groups_n, int groups_k, const float* beta, const int32_t* wsum,
                                bool nonneg, const float* ln_gain, const float* ln_bias,
                                float ln_eps, int granularity, unsigned flags, float* Y,
                                void* workspace, size_t workspace_bytes, void* stream) {
    if (M < 0 || M > kMaxDim || !shape_ok(N, K)) return BL_ERR_SHAPE;
    if (int st = groups_status(N, K, groups_n, groups_k)) return st;
    if (!gran_ok(granularity) || (flags & ~BL_FLAG_SKIP_LN)) return BL_ERR_UNSUPPORTED;
    if (K / groups_k > kMaxGemmK) return BL_ERR_UNSUPPORTED;
    if (M == 0) return BL_OK;
    if (!X || !packed || !beta || !Y || (nonneg && !wsum)) return BL_ERR_NULL;
    const ForwardWs ws = nonneg ? forward_ws_nonneg(M, N, K, groups_k, granularity)
                                : forward_ws_grouped(M, N, K, groups_k, granularity);
    if (!workspace || workspace_bytes < ws.total) return BL_ERR_WORKSPACE;
    char* base = (char*)workspace;
    int8_t* codes = (int8_t*)(base + ws.codes);
    float* gamma = (float*)(base + ws.gamma);
    float* eta = nonneg ? (float*)(base + ws.xhat) : nullptr;
    int32_t* rowsum = (int32_t*)(base + ws.rowsum);
    int rc = quant_act_grouped_impl(X, M, K, groups_k, ln_gain, ln_bias, ln_eps, granularity,
                                    flags & BL_FLAG_SKIP_LN, nonneg, codes, gamma, eta, rowsum,
                                    nullptr, base + ws.quant, workspace_bytes - ws.quant, stream);
    if (rc != BL_OK) return rc;
    // one GEMM per K-group, each dequantised with its own beta_g * gamma_g (and shifted by its own
    // eta_g, Eq. 14) and added (Eq. 13-14)
    const int64_t Kg = K / groups_k;
    const size_t blob_dwords = tiles_bytes(N, Kg) / 4;
    const bool per_tensor = granularity == BL_GAMMA_PER_TENSOR;
    if (groups_k > 1) {
        // One launch for all K-groups.  Up to 64 tokens every K-group is a slice of the launch,
        // and the fold that follows dequantises each group's sums with its own scales and adds
        // them in the order 0, 1, ...; above that the large-tile kernel walks a tile's groups
        // itself and keeps the fp32 sum in registers.  Y is written once.
        GemmArgs a{};
        a.codes = codes; a.gamma = gamma; a.rowsum = rowsum;
        a.M = M; a.K = Kg; a.N = N;
        a.packed = (const uint32_t*)packed; a.beta = beta;
        a.per_tensor = per_tensor;
        a.Y = Y;
        a.ldq = K; a.gstride = groups_k; a.beta_rows = N / groups_n; a.beta_stride = groups_k;
        if (nonneg) {
            a.eta = eta;
            a.wsum = wsum;
        }
        a.kgroups = groups_k; a.group_packed = (int64_t)blob_dwords;
        a.split_ws = (int32_t*)(base + ws.split); a.split_ws_bytes = ws.split_bytes;
        return check_hip(M <= 16 ? launch_gemm_decode(a, (hipStream_t)stream)
                                 : launch_gemm_prefill(a, (hipStream_t)stream));
    }
    for (int gk = 0; gk < groups_k; ++gk) {
        GemmArgs a{};
        a.codes = codes + gk * Kg; a.gamma = gamma + gk; a.rowsum = rowsum + gk;
        a.M = M; a.K = Kg; a.N = N;
        a.packed = (const uint32_t*)packed + gk * blob_dwords; a.beta = beta + gk;
        a.per_tensor = per_tensor;
        a.out_acc = false;
        a.Y = Y;
        a.ldq = K; a.gstride = groups_k; a.beta_rows = N / groups_n; a.beta_stride = groups_k;
        a.accumulate = gk > 0;
        if (nonneg) {
            a.eta = eta + gk;
            a.wsum = wsum + (int64_t)gk * N;
        }
        const hipError_t e = M <= 16 ? launch_gemm_decode(a, (hipStream_t)stream)
                                     : launch_gemm_prefill(a, (hipStream_t)stream);
        if (e != hipSuccess) return BL_ERR_HIP;
    }
    return BL_OK;
}

int bitlinear_forward_grouped(const float* X, int64_t M, int64_t K, const void* packed, int64_t N,
                              int groups_n, int groups_k, const float* beta, const float* ln_gain,
                              const float* ln_bias, float ln_eps, int granularity, unsigned flags,
                              float* Y, void* workspace, size_t workspace_bytes, void* stream) {
    return forward_grouped_impl(X, M, K, packed, N, groups_n, groups_k, beta, nullptr, false, ln_gain,
                                ln_bias, ln_eps, granularity, flags, Y, workspace, workspace_bytes,
                                stream);
}

int bitlinear_forward_grouped_nonneg(const float* X, int64_t M, int64_t K, const void* packed,
                                     int64_t N, int groups_n, int groups_k, const float* beta,
                                     const int32_t* wsum, const float* ln_gain, const float* ln_bias,
                                     float ln_eps, int granularity, unsigned flags, float* Y,
                                     void* workspace, size_t workspace_bytes, void* stream) {
    return forward_grouped_impl(X, M, K, packed, N, groups_n, groups_k, beta, wsum, true, ln_gain,
                                ln_bias, ln_eps, granularity, flags, Y, workspace, workspace_bytes,
                                stream);
}

int bitlinear_weight_rowsums_grouped(const void* packed, int64_t N, int64_t K, int groups_k,
                                     int32_t* wsum, void* stream) {
    if (!shape_ok(N, K)) return BL_ERR_SHAPE;
    if (int st = groups_status(N, K, 1, groups_k)) return st;
    if (!packed || !wsum) return BL_ERR_NULL;
    const int64_t Kg = K / groups_k;
    const size_t blob_dwords = tiles_bytes(N, Kg) / 4;
    for (int gk = 0; gk < groups_k; ++gk) {
        const hipError_t e = launch_weight_rowsums((const uint32_t*)packed + gk * blob_dwords, N, Kg,
                                                   wsum + (int64_t)gk * N, (hipStream_t)stream);
        if (e != hipSuccess) return BL_ERR_HIP;
    }
    return BL_OK;
}

int bitlinear_backward_ste(const float* dY, int64_t M, int64_t N, int64_t K, const int8_t* codes,
                           const float* gamma, int granularity, const void* packed,
                           const float* beta, float* dX, float* dW, void* workspace,
                           size_t workspace_bytes, void* stream) {
    if (M < 0 || M > kMaxDim || !shape_ok(N, K)) return BL_ERR_SHAPE;
    if (!gran_ok(granularity)) return BL_ERR_UNSUPPORTED;
    if (M == 0 || (!dX && !dW)) return BL_OK;
    if (!dY || !gamma) return BL_ERR_NULL;
    if (dX && (!packed || !beta)) return BL_ERR_NULL;
    if (dW && !codes) return BL_ERR_NULL;
    const size_t need = bitlinear_workspace_bytes(BL_OP_BACKWARD, M, N, K, granularity, 0);
    if (!workspace || workspace_bytes < need) return BL_ERR_WORKSPACE;
    BackwardArgs a{};
    a.dY = dY; a.M = M; a.N = N; a.K = K; a.codes = codes; a.gamma = gamma;
    a.per_tensor = granularity == BL_GAMMA_PER_TENSOR;
    a.packed = (const uint32_t*)packed; a.beta = beta; a.dX = dX; a.dW = dW;
    a.workspace = (void*)(((uintptr_t)workspace + 255) & ~(uintptr_t)255);
    return check_hip(launch_backward(a, (hipStream_t)stream));
}

// ---- the non-negative quantiser (Eq. 6) ------------------------------------------------

int bitlinear_weight_rowsums(const void* packed, int64_t N, int64_t K, int32_t* wsum,
                             void* stream) {
    if (!shape_ok(N, K)) return BL_ERR_SHAPE;
    if (!packed || !wsum) return BL_ERR_NULL;
    return check_hip(launch_weight_rowsums((const uint32_t*)packed, N, K, wsum,
                                           (hipStream_t)stream));
}

int bitlinear_quant_act_nonneg(const float* X, int64_t M, int64_t K, const float* ln_gain,
                               const float* ln_bias, float ln_eps, int granularity,
                               unsigned flags, int8_t* codes, float* gamma, float* eta,
                               int32_t* rowsum, float* xhat_dump, void* workspace,
                               size_t workspace_bytes, void* stream) {
    return quant_act_grouped_impl(X, M, K, 1, ln_gain, ln_bias, ln_eps, granularity, flags, true,
                                  codes, gamma, eta, rowsum, xhat_dump, workspace, workspace_bytes,
                                  stream);
}

int bitlinear_matmul_nonneg(const int8_t* codes, const float* gamma, const float* eta,
                            const int32_t* rowsum, int64_t M, int64_t K, const void* packed,
                            int64_t N, const float* beta, const int32_t* wsum, int granularity,
                            unsigned flags, float* Y, void* stream) {
    if (M < 0 || M > kMaxDim || !shape_ok(N, K)) return BL_ERR_SHAPE;
    if (!gran_ok(granularity) || flags || K > kMaxGemmK) return BL_ERR_UNSUPPORTED;
    if (M == 0) return BL_OK;
    if (!codes || !gamma || !eta || !rowsum || !packed || !beta || !wsum || !Y) return BL_ERR_NULL;
    GemmArgs a{};
    a.codes = codes; a.gamma = gamma; a.rowsum = rowsum; a.M = M; a.K = K; a.N = N;
    a.packed = (const uint32_t*)packed; a.beta = beta;
    a.per_tensor = granularity == BL_GAMMA_PER_TENSOR;
    a.out_acc = false;
    a.Y = Y;
    plain_fields(a);
    a.eta = eta;
    a.wsum = wsum;
    if (M <= 16) return check_hip(launch_gemm_decode(a, (hipStream_t)stream));
    return check_hip(launch_gemm_prefill(a, (hipStream_t)stream));
}

int bitlinear_forward_nonneg(const float* X, int64_t M, int64_t K, const void* packed, int64_t N,
                             const float* beta, const int32_t* wsum, const float* ln_gain,
                             const float* ln_bias, float ln_eps, int granularity, unsigned flags,
                             float* Y, void* workspace, size_t workspace_bytes, void* stream) {
    return forward_grouped_impl(X, M, K, packed, N, 1, 1, beta, wsum, true, ln_gain, ln_bias, ln_eps,
                                granularity, flags, Y, workspace, workspace_bytes, stream);
}

int bitlinear_layernorm_backward(const float* dXhat, const float* X, int64_t M, int64_t K,
                                 int groups_k, const float* ln_gain, float ln_eps, float* dX,
                                 float* dgain, float* dbias, void* workspace,
                                 size_t workspace_bytes, void* stream) {
    if (M < 0 || M > kMaxDim || K <= 0 || K > kMaxDim || K % 32) return BL_ERR_SHAPE;
    if (groups_k < 1 || groups_k > kMaxGroups || K % groups_k || (K / groups_k) % 32)
        return BL_ERR_SHAPE;
    const int64_t Kg = K / groups_k;
    if (!ln_backward_supported(Kg) || M * groups_k > kMaxDim) return BL_ERR_UNSUPPORTED;
    if (M == 0 || (!dX && !dgain && !dbias)) return BL_OK;
    if (!dXhat || !X) return BL_ERR_NULL;
    const LnBackwardWs ws = ln_backward_ws(M, K, groups_k);
    const bool affine = dgain || dbias;
    if (affine && (!workspace || workspace_bytes < ws.total)) return BL_ERR_WORKSPACE;
    LnBackwardArgs a{};
    a.g = dXhat; a.X = X; a.M = M * groups_k; a.K = Kg; a.gain = ln_gain; a.eps = ln_eps;
    a.groups = groups_k; a.dX = dX;
    a.rowstats = affine ? (double*)((char*)workspace + ws.rowstats) : nullptr;
    double* partials = affine ? (double*)((char*)workspace + ws.partials) : nullptr;
    return check_hip(launch_ln_backward(a, dgain, dbias, partials, (hipStream_t)stream));
}

int bitlinear_probe_read(const void* src, size_t bytes, int workgroups, int threads, uint32_t* sink,
                         void* stream) {
    if (bytes < 16 || bytes % 16 || workgroups < 1 || workgroups > 65536 || threads < 64 ||
        threads > 1024 || threads % 64)
        return BL_ERR_SHAPE;
    if (!src) return BL_ERR_NULL;
    return check_hip(launch_read_probe(src, bytes, workgroups, threads, sink, (hipStream_t)stream));
}

const char* bitlinear_status_string(int status) {
    switch (status) {
        case BL_OK: return "ok";
        case BL_ERR_NULL: return "a required pointer is NULL";
        case BL_ERR_SHAPE:
            return "bad shape (M, N, K out of range, K not a multiple of 32, or groups that do not divide)";
        case BL_ERR_UNSUPPORTED: return "unsupported granularity, flag or size";
        case BL_ERR_WORKSPACE: return "workspace missing or too small";
        case BL_ERR_HIP: return "HIP launch failed";
        default: return "unknown status";
    }
}

}  // extern "C"
