// C ABI of libfrspec: argument validation on the host, workspace carving, dispatch.
#include <atomic>
#include <mutex>

#include "internal.hpp"

namespace frspec {

namespace {
constexpr size_t round256(size_t x) { return (x + 255) & ~static_cast<size_t>(255); }

struct WorkspaceLayout {
    size_t mail_rec_off, mail_st_off, step_rec_off, ms_off, val_off, id_off, total;
    // mail_rows: rows of H the result mailbox has records for (the caller's workspace: kMailRows)
    constexpr WorkspaceLayout(int64_t M, int32_t k, int mail_rows = kMailRows)
        : mail_rec_off(0), mail_st_off(0), step_rec_off(0), ms_off(0), val_off(0), id_off(0), total(0) {
        const size_t rows = static_cast<size_t>(M < kMatrixPathMaxM ? M : kMatrixPathMaxM);
        const size_t slots = static_cast<size_t>(kWorkspaceGridMax) * rows;
        size_t o = kWorkspaceHeaderBytes;
        mail_rec_off = o; o += kMailRecBytes / kMailRows * static_cast<size_t>(mail_rows);
        mail_st_off = o;  o += kMailStBytes / kMailRows * static_cast<size_t>(mail_rows);
        step_rec_off = o; o += kStepRecBytes;
        ms_off = o;  o += round256(slots * 2 * sizeof(float));
        val_off = o; o += round256(slots * static_cast<size_t>(k) * sizeof(float));
        id_off = o;  o += round256(slots * static_cast<size_t>(k) * sizeof(int));
        total = o;
    }
};

// Scratch of fr_draft_topk_static, the entry point for callers that cannot allocate: one
// workspace for up to kStaticRows rows of H and k <= kStaticK (header, a 16-row result mailbox,
// the plain partial arrays; about 2.2 MiB), held by every device the library runs on until the
// process ends.  The array's name is a host-side stand-in, not a device address: host code
// uses the address that hipGetSymbolAddress returns for the current device (each device has
// its own copy), kept in DeviceState::scratch.
constexpr int kStaticRows = 16, kStaticK = 16;
constexpr size_t kStaticScratchBytes = WorkspaceLayout(kStaticRows, kStaticK, kStaticRows).total;
}  // namespace
}  // namespace frspec

static __device__ __align__(256) unsigned char scratch[frspec::kStaticScratchBytes];

namespace frspec {
namespace {

// Header zero, every mailbox record empty (all ones): what fr_workspace_init does for a caller's
// workspace.  Synchronous, on the null stream.
fr_status prepare_scratch(void *ptr) {
    constexpr size_t mail = WorkspaceLayout(kStaticRows, kStaticK, kStaticRows).ms_off - kWorkspaceHeaderBytes;
    fr_status st = launch_fill_u32(static_cast<unsigned *>(ptr), kWorkspaceHeaderBytes / 4, 0u, nullptr);
    if (st != FR_OK) return st;
    st = launch_fill_u32(reinterpret_cast<unsigned *>(static_cast<char *>(ptr) + kWorkspaceHeaderBytes), mail / 4,
                         0xFFFFFFFFu, nullptr);
    if (st != FR_OK) return st;
    if (hipStreamSynchronize(nullptr) != hipSuccess) {
        (void)hipGetLastError();
        return FR_ERR_HIP;
    }
    return FR_OK;
}

constexpr int kMaxDevices = 64;
struct DeviceSlot {
    std::atomic<int> ready{0};
    DeviceState state{};
};
DeviceSlot g_device[kMaxDevices];
std::mutex g_setup_mutex;
}  // namespace

const DeviceState *device_state() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        return nullptr;
    }
    DeviceSlot &slot = g_device[dev];
    if (slot.ready.load(std::memory_order_acquire)) return &slot.state;
    std::lock_guard<std::mutex> lock(g_setup_mutex);
    if (slot.ready.load(std::memory_order_relaxed)) return &slot.state;
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) {
        (void)hipGetLastError();
        return nullptr;
    }
    slot.state.cus = n;
    if (prepare_skinny_kernels() != FR_OK || prepare_wide_kernels() != FR_OK || prepare_block_kernels() != FR_OK || prepare_glue_kernels() != FR_OK ||
        prepare_freq_kernels() != FR_OK)
        return nullptr;
    // this device's copy of the static scratch: its address, then its initial contents
    void *ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
        (void)hipGetLastError();
        return nullptr;
    }
    if (prepare_scratch(ptr) != FR_OK) return nullptr;
    slot.state.scratch = ptr;
    slot.ready.store(1, std::memory_order_release);
    return &slot.state;
}

int device_cu_count() {
    const DeviceState *st = device_state();
    return st ? st->cus : -1;
}

namespace {

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
fr_status check_head_args(const void *H, int64_t M, int64_t d, const void *W, int64_t V_rows,
                          int32_t k) {
    if (!H || !W) return FR_ERR_INVALID_ARG;
    if (M < 1 || d < 8 || (d % 8) != 0 || V_rows < 1 || V_rows > INT32_MAX) return FR_ERR_INVALID_ARG;
    if (M > INT32_MAX || d > (1 << 24)) return FR_ERR_INVALID_ARG;
    if (k < 1 || k > FR_K_MAX || k > V_rows) return FR_ERR_INVALID_ARG;
    if (V_rows * (d / 8) > INT32_MAX) return FR_ERR_INVALID_ARG;   // 16-byte chunk index fits int32
    // the kernels address W as a base plus a 32-bit byte offset (tiles of 16 rows, padded)
    if ((V_rows + 15) / 16 * 16 * d * 2 > (int64_t(1) << 32)) return FR_ERR_UNSUPPORTED;
    if (!aligned16(H) || !aligned16(W)) return FR_ERR_ALIGNMENT;
    return FR_OK;
}

fr_status head_topk(const void *H, int64_t M, int64_t d, const void *W, const int32_t *idx_map,
                    int64_t V_rows, int32_t k, int32_t *token_ids, float *logp, void *workspace,
                    size_t workspace_bytes, fr_stream stream, const fr_tuning *tuning, bool tiled = false,
                    const long long *row_delta = nullptr, const StepArgs *step = nullptr,
                    int mail_rows = kMailRows) {
    fr_status st = check_head_args(H, M, d, W, V_rows, k);
    if (st != FR_OK) return st;
    if (!token_ids || !logp || !workspace) return FR_ERR_INVALID_ARG;
    if (!aligned16(workspace)) return FR_ERR_ALIGNMENT;
    if (M > mail_rows && mail_rows < kMailRows) return FR_ERR_UNSUPPORTED;   // (a short mailbox serves few rows)
    const WorkspaceLayout wl(M, k, mail_rows);
    if (workspace_bytes < wl.total) return FR_ERR_WORKSPACE;
    if (tuning && (tuning->path < 0 || tuning->path > 3 || tuning->grid < 0 ||
                   tuning->grid > kWorkspaceGridMax || tuning->variant < 0 || tuning->ksplit < 0 ||
                   tuning->spin_limit < 0))
        return FR_ERR_INVALID_ARG;

    char *ws = static_cast<char *>(workspace);
    HeadProblem p{};
    p.W = W;
    p.tiled = tiled;
    p.scattered_rows = row_delta != nullptr;
    if (row_delta)
        for (int m = 0; m < 16; ++m) p.row_delta[m] = row_delta[m];
    p.idx_map = idx_map;
    p.d = static_cast<int>(d);
    p.V_rows = static_cast<int>(V_rows);
    p.k = k;
    p.ws.ticket = reinterpret_cast<unsigned *>(ws);
    p.ws.mail_rec = reinterpret_cast<unsigned long long *>(ws + wl.mail_rec_off);
    p.ws.mail_st = reinterpret_cast<unsigned long long *>(ws + wl.mail_st_off);
    p.ws.step_rec = reinterpret_cast<unsigned long long *>(ws + wl.step_rec_off);
    p.step = step;
    p.ws.part_ms = reinterpret_cast<float *>(ws + wl.ms_off);
    p.ws.part_val = reinterpret_cast<float *>(ws + wl.val_off);
    p.ws.part_id = reinterpret_cast<int *>(ws + wl.id_off);
    hipStream_t s = static_cast<hipStream_t>(stream);

    // paths: 3 = skinny kernel on the matrix cores, 1 = skinny kernel on the vector ALUs,
    // 2 = chunked matrix-core kernel (any M)
    int path = tuning ? tuning->path : 0;
    if (tiled) {   // only the skinny kernel's matrix-core build reads the tiled layout
        if (path == 1 || path == 2 || M > kSkinnyMaxM || (d % 128) != 0) return FR_ERR_UNSUPPORTED;
        path = 3;
    }
    if (path == 0) {
        // the skinny kernel while its eight-wavefront build holds H; beyond that the chunked
        // kernel is faster than the four-wavefront build, which remains for the calls that
        // only the skinny kernel serves (H rows in several blocks, the fused beam-search step)
        const bool skinny_only = row_delta || step;
        path = (M <= kSkinnyMaxM && (skinny_only ? skinny_fits((int)M, (int)d, k)
                                                 : skinny_fits_eight_waves((int)M, (int)d, k))) ? 3 : 2;
        // Rows of H longer than 8 KiB: the skinny kernel's 512 threads request one 16-byte column of H
        // each ahead of W and fetch the columns beyond that later, behind the first batch of W; the
        // chunked kernel stages H in pieces anyway and is 1 to 4 us faster there from two rows of H
        // on (measured at d = 4608, 5120, 6144; at 8192 the two are level), as long as there is a 128-row
        // pass for every compute unit (with fewer rows of W only the skinny kernel splits d between its
        // wavefronts).
        if (path == 3 && !skinny_only && d > 4096 && d < 8192 && M >= 2 && k <= kMailK) {
            const int cus = device_cu_count();
            if (cus > 0 && V_rows >= static_cast<int64_t>(128) * cus) path = 2;
        }
        // The other way round on small subsets: the chunked kernel works in passes of 128 rows, so
        // with few rows of W per compute unit most of the device idles; the skinny kernel's
        // four-wavefront build, which splits d, then wins where it holds H (22.5 against 30.2 us at
        // 8192 rows, 13 rows of H; at 16384 rows, 64 per compute unit, it loses: 38 against 32 us).
        if (path == 2 && M <= kSkinnyMaxM && skinny_fits((int)M, (int)d, k)) {
            const int cus = device_cu_count();
            if (cus > 0 && V_rows <= static_cast<int64_t>(48) * cus) path = 3;
        }
    }
    if ((row_delta || step) && path == 2) return FR_ERR_UNSUPPORTED;
    const bool two_launch = tuning && tuning->two_launch;
    const bool stream_only = tuning && tuning->stream_only;

    if (path == 1 || path == 3) {
        if (M > kSkinnyMaxM) return FR_ERR_UNSUPPORTED;
        p.H = H;
        p.M = static_cast<int>(M);
        p.token_ids = token_ids;
        p.logp = logp;
        return launch_skinny(p, stream_only ? Sink::kStreamOnly : two_launch ? Sink::kPartialsOnly : Sink::kFusedTopk, tuning, s);
    }

    // matrix-core path: slabs of H rows, each a full pass over W.  More than 64 rows go to the
    // block kernel, up to 256 at a time, where it serves the shape; otherwise, and for what is
    // left, the chunked kernel takes slabs of up to 128 (a build costs the same for any number
    // of rows up to its size, so full slabs first beat equal shares).
    const int slab = mfma_max_rows(k);
    if (slab <= 0) return FR_ERR_UNSUPPORTED;
    const bool chunked_only = tuning && tuning->chunked_only;
    for (int64_t m0 = 0; m0 < M;) {
        const int64_t left = M - m0;
        const int block_rows = static_cast<int>(left < kBlockMaxM ? left : kBlockMaxM);
        const bool block = !chunked_only && block_kernel_serves(block_rows, (int)d, k);
        const int rows = block ? block_rows : static_cast<int>(left < slab ? left : slab);
        p.H = static_cast<const char *>(H) + static_cast<size_t>(m0) * d * 2;
        p.M = rows;
        p.token_ids = token_ids + m0 * k;
        p.logp = logp + m0 * k;
        // Single launch while the result mailbox covers the rows (k <= 16, up to 128 rows), or,
        // through the arrival counter, while the rows are few; else a merge launch follows.
        const bool mail_ok = k <= kMailK && rows <= kMailRows && !(tuning && tuning->no_mailbox);
        const Sink sink = stream_only ? Sink::kStreamOnly
                          : (two_launch || (rows > 32 && !mail_ok)) ? Sink::kPartialsOnly : Sink::kFusedTopk;
        st = block ? launch_block(p, sink, tuning, s) : launch_mfma(p, sink, tuning, s, nullptr);
        if (st != FR_OK) return st;
        m0 += rows;
    }
    return FR_OK;
}

}  // namespace
}  // namespace frspec

using namespace frspec;

extern "C" {

const char *fr_strerror(fr_status status) {
    switch (status) {
        case FR_OK: return "ok";
        case FR_ERR_INVALID_ARG: return "invalid argument";
        case FR_ERR_ALIGNMENT: return "pointer not 16-byte aligned";
        case FR_ERR_WORKSPACE: return "workspace too small";
        case FR_ERR_HIP: return "HIP runtime error";
        case FR_ERR_UNSUPPORTED: return "shape not supported by the kernels";
        case FR_ERR_SCRATCH: return "problem larger than the library's static scratch (fr_draft_topk_static: M <= 16, k <= 16)";
    }
    return "unknown status";
}

int fr_version(void) { return 101; }

fr_status fr_init(void) {
    int dev = 0;
    const bool fresh = hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < kMaxDevices &&
                       !g_device[dev].ready.load(std::memory_order_acquire);
    const DeviceState *st = device_state();
    if (!st) return FR_ERR_HIP;
    // a repeated call prepares the device's static scratch afresh (the set-up has just done so)
    return fresh ? FR_OK : prepare_scratch(st->scratch);
}

fr_status fr_build_subset(const void *W_full, int64_t V, int64_t d, const int32_t *freq_ranked_ids,
                          int64_t V_sub, void *W_sub, int32_t *idx_map, int32_t *dev_error_flag,
                          fr_stream stream) {
    if (!W_full || !freq_ranked_ids || !W_sub || !idx_map) return FR_ERR_INVALID_ARG;
    if (V < 1 || V > INT32_MAX || d < 8 || (d % 8) != 0 || d > (1 << 24)) return FR_ERR_INVALID_ARG;
    if (V_sub < 1 || V_sub > V) return FR_ERR_INVALID_ARG;
    if (!aligned16(W_full) || !aligned16(W_sub)) return FR_ERR_ALIGNMENT;
    return launch_gather(W_full, V, d, freq_ranked_ids, V_sub, W_sub, idx_map, dev_error_flag,
                         static_cast<hipStream_t>(stream));
}

size_t fr_tiled_bytes(int64_t V_sub, int64_t d) {
    if (V_sub < 1 || d < 128 || (d % 128) != 0) return 0;
    return static_cast<size_t>((V_sub + 15) / 16) * 16u * static_cast<size_t>(d) * 2u;
}

fr_status fr_build_subset_tiled(const void *W_full, int64_t V, int64_t d, const int32_t *freq_ranked_ids,
                                int64_t V_sub, void *W_tiled, int32_t *idx_map, int32_t *dev_error_flag,
                                fr_stream stream) {
    if (!W_full || !freq_ranked_ids || !W_tiled || !idx_map) return FR_ERR_INVALID_ARG;
    if (V < 1 || V > INT32_MAX || d < 128 || (d % 128) != 0 || d > (1 << 24)) return FR_ERR_INVALID_ARG;
    if (V_sub < 1 || V_sub > V) return FR_ERR_INVALID_ARG;
    if (!aligned16(W_full) || !aligned16(W_tiled)) return FR_ERR_ALIGNMENT;
    return launch_gather_tiled(W_full, V, d, freq_ranked_ids, V_sub, W_tiled, idx_map, dev_error_flag,
                               static_cast<hipStream_t>(stream));
}

fr_status fr_draft_topk_tiled(const void *H, int64_t M, int64_t d, const void *W_tiled,
                              const int32_t *idx_map, int64_t V_sub, int32_t k, int32_t *token_ids,
                              float *logp, void *workspace, size_t workspace_bytes, fr_stream stream) {
    return head_topk(H, M, d, W_tiled, idx_map, V_sub, k, token_ids, logp, workspace, workspace_bytes, stream,
                     nullptr, true);
}

fr_status fr_draft_topk_tiled_tuned(const void *H, int64_t M, int64_t d, const void *W_tiled,
                                    const int32_t *idx_map, int64_t V_sub, int32_t k, int32_t *token_ids,
                                    float *logp, void *workspace, size_t workspace_bytes, fr_stream stream,
                                    const fr_tuning *tuning) {
    return head_topk(H, M, d, W_tiled, idx_map, V_sub, k, token_ids, logp, workspace, workspace_bytes, stream,
                     tuning, true);
}

size_t fr_workspace_bytes(int64_t M, int64_t d, int64_t V_rows, int32_t k) {
    if (M < 1 || d < 8 || (d % 8) != 0 || V_rows < 1 || k < 1 || k > FR_K_MAX || k > V_rows) return 0;
    return WorkspaceLayout(M, k).total;
}

fr_status fr_workspace_init(void *workspace, size_t workspace_bytes, fr_stream stream) {
    if (!workspace) return FR_ERR_INVALID_ARG;
    if (!aligned16(workspace)) return FR_ERR_ALIGNMENT;
    const size_t mail = kMailRecBytes + kMailStBytes + kStepRecBytes;
    if (workspace_bytes < kWorkspaceHeaderBytes + mail) return FR_ERR_WORKSPACE;
    // arrival words: zero; mailbox: all ones (= every record empty)
    fr_status st = launch_fill_u32(static_cast<unsigned *>(workspace), kWorkspaceHeaderBytes / 4, 0u,
                                   static_cast<hipStream_t>(stream));
    if (st != FR_OK) return st;
    return launch_fill_u32(reinterpret_cast<unsigned *>(static_cast<char *>(workspace) + kWorkspaceHeaderBytes),
                           mail / 4, 0xFFFFFFFFu, static_cast<hipStream_t>(stream));
}

fr_status fr_draft_topk_multi(const void *const *H_blocks, int32_t n_blocks, int64_t rows_per_block, int64_t d,
                              const void *W_sub, const int32_t *idx_map, int64_t V_sub, int32_t k,
                              int32_t *token_ids, float *logp, void *workspace, size_t workspace_bytes,
                              fr_stream stream) {
    if (!H_blocks || n_blocks < 1 || n_blocks > 16 || rows_per_block < 1) return FR_ERR_INVALID_ARG;
    for (int32_t b = 0; b < n_blocks; ++b)
        if (!H_blocks[b]) return FR_ERR_INVALID_ARG;
        else if (!aligned16(H_blocks[b])) return FR_ERR_ALIGNMENT;
    const int64_t M = static_cast<int64_t>(n_blocks) * rows_per_block;
    fr_status st = check_head_args(H_blocks[0], M, d, W_sub, V_sub, k);
    if (st != FR_OK) return st;
    if (!token_ids || !logp || !workspace) return FR_ERR_INVALID_ARG;
    if (M <= kSkinnyMaxM && skinny_fits((int)M, (int)d, k)) {
        // one launch: the skinny kernel takes the rows where they are
        long long delta[16] = {0};
        for (int64_t m = 0; m < M; ++m)
            delta[m] = (static_cast<const char *>(H_blocks[m / rows_per_block]) - static_cast<const char *>(H_blocks[0])) +
                       (m % rows_per_block) * d * 2;
        return head_topk(H_blocks[0], M, d, W_sub, idx_map, V_sub, k, token_ids, logp, workspace, workspace_bytes,
                         stream, nullptr, false, delta);
    }
    // too many rows for the skinny kernel: one call per block
    for (int32_t b = 0; b < n_blocks; ++b) {
        st = head_topk(H_blocks[b], rows_per_block, d, W_sub, idx_map, V_sub, k, token_ids + b * rows_per_block * k,
                       logp + b * rows_per_block * k, workspace, workspace_bytes, stream, nullptr);
        if (st != FR_OK) return st;
    }
    return FR_OK;
}

fr_status fr_workspace_check(const void *workspace, size_t workspace_bytes, int32_t *timed_out,
                             fr_stream stream) {
    if (!workspace || !timed_out) return FR_ERR_INVALID_ARG;
    if (!aligned16(workspace)) return FR_ERR_ALIGNMENT;
    if (workspace_bytes < kWorkspaceHeaderBytes) return FR_ERR_WORKSPACE;
    unsigned word = 0;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (hipMemcpyAsync(&word, static_cast<const unsigned *>(workspace) + 1, sizeof word, hipMemcpyDeviceToHost, s) !=
            hipSuccess ||
        hipStreamSynchronize(s) != hipSuccess) {
        (void)hipGetLastError();
        return FR_ERR_HIP;
    }
    *timed_out = word != 0;
    return FR_OK;
}

fr_status fr_draft_topk(const void *H, int64_t M, int64_t d, const void *W_sub,
                        const int32_t *idx_map, int64_t V_sub, int32_t k, int32_t *token_ids,
                        float *logp, void *workspace, size_t workspace_bytes, fr_stream stream) {
    return head_topk(H, M, d, W_sub, idx_map, V_sub, k, token_ids, logp, workspace, workspace_bytes,
                     stream, nullptr);
}

fr_status fr_draft_topk_static(const void *H, int64_t M, int64_t d, const void *W_sub,
                               const int32_t *idx_map, int64_t V_sub, int32_t k, int32_t *token_ids,
                               float *logp, fr_stream stream) {
    const fr_status chk = check_head_args(H, M, d, W_sub, V_sub, k);
    if (chk != FR_OK) return chk;
    if (M > kStaticRows || k > kStaticK) return FR_ERR_SCRATCH;
    const DeviceState *st = device_state();
    if (!st || !st->scratch) return FR_ERR_HIP;
    return head_topk(H, M, d, W_sub, idx_map, V_sub, k, token_ids, logp, st->scratch, kStaticScratchBytes, stream,
                     nullptr, false, nullptr, nullptr, kStaticRows);
}

fr_status fr_draft_topk_tuned(const void *H, int64_t M, int64_t d, const void *W_sub,
                              const int32_t *idx_map, int64_t V_sub, int32_t k, int32_t *token_ids,
                              float *logp, void *workspace, size_t workspace_bytes,
                              fr_stream stream, const fr_tuning *tuning) {
    return head_topk(H, M, d, W_sub, idx_map, V_sub, k, token_ids, logp, workspace, workspace_bytes,
                     stream, tuning);
}

fr_status fr_full_topk(const void *H, int64_t M, int64_t d, const void *W_full, int64_t V, int32_t k,
                       int32_t *token_ids, float *logp, void *workspace, size_t workspace_bytes,
                       fr_stream stream) {
    return head_topk(H, M, d, W_full, nullptr, V, k, token_ids, logp, workspace, workspace_bytes,
                     stream, nullptr);
}

fr_status fr_draft_logits(const void *H, int64_t M, int64_t d, const void *W, int64_t V_rows,
                          float *z_out, fr_stream stream) {
    fr_status st = check_head_args(H, M, d, W, V_rows, 1);
    if (st != FR_OK) return st;
    if (!z_out) return FR_ERR_INVALID_ARG;
    HeadProblem p{};
    p.W = W;
    p.d = static_cast<int>(d);
    p.V_rows = static_cast<int>(V_rows);
    p.k = 1;
    p.z_ld = static_cast<int>(V_rows);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (M <= kSkinnyMaxM && skinny_fits((int)M, (int)d, 1)) {
        p.H = H;
        p.M = static_cast<int>(M);
        p.z_out = z_out;
        return launch_skinny(p, Sink::kLogits, nullptr, s);
    }
    const int slab = mfma_max_rows(1);
    for (int64_t m0 = 0; m0 < M;) {
        const int64_t left = M - m0;
        const int block_rows = static_cast<int>(left < kBlockMaxM ? left : kBlockMaxM);
        const bool block = block_kernel_serves(block_rows, (int)d, 1);
        const int rows = block ? block_rows : static_cast<int>(left < slab ? left : slab);
        p.H = static_cast<const char *>(H) + static_cast<size_t>(m0) * d * 2;
        p.M = rows;
        p.z_out = z_out + static_cast<size_t>(m0) * V_rows;
        st = block ? launch_block(p, Sink::kLogits, nullptr, s) : launch_mfma(p, Sink::kLogits, nullptr, s, nullptr);
        if (st != FR_OK) return st;
        m0 += rows;
    }
    return FR_OK;
}

fr_status fr_draft_step(const void *H, int64_t M, int64_t d, const void *W_sub, const int32_t *idx_map,
                        int64_t V_sub, int32_t k, const float *node_score, const int32_t *node_hist,
                        int32_t width, float *hist_score, int32_t *hist_token, int32_t *hist_parent,
                        int64_t hist_offset, int32_t *token_ids, float *logp, float *next_score,
                        int32_t *next_token, int32_t *next_hist, void *workspace, size_t workspace_bytes,
                        fr_stream stream) {
    if (!node_score || !node_hist || !hist_score || !hist_token || !hist_parent || !next_score || !next_token ||
        !next_hist)
        return FR_ERR_INVALID_ARG;
    if (width < 1 || hist_offset < 0 || hist_offset > INT32_MAX) return FR_ERR_INVALID_ARG;
    if (M >= 1 && k >= 1 && (width > M * k || hist_offset + M * k > INT32_MAX)) return FR_ERR_INVALID_ARG;
    StepArgs st{};
    st.node_score = node_score;
    st.node_hist = node_hist;
    st.width = width;
    st.hist_offset = hist_offset;
    st.hist_score = hist_score;
    st.hist_token = hist_token;
    st.hist_parent = hist_parent;
    st.next_score = next_score;
    st.next_token = next_token;
    st.next_hist = next_hist;
    // one launch when the skinny kernel's mailbox merge applies; else the two calls one after the other
    fr_status s = FR_ERR_UNSUPPORTED;
    if (M <= kSkinnyMaxM && M * k <= 256)
        s = head_topk(H, M, d, W_sub, idx_map, V_sub, k, token_ids, logp, workspace, workspace_bytes, stream, nullptr,
                      false, nullptr, &st);
    if (s != FR_ERR_UNSUPPORTED) return s;
    s = head_topk(H, M, d, W_sub, idx_map, V_sub, k, token_ids, logp, workspace, workspace_bytes, stream, nullptr);
    if (s != FR_OK) return s;
    return fr_beam_expand(logp, token_ids, M, k, node_score, node_hist, width, hist_score, hist_token, hist_parent,
                          hist_offset, next_score, next_token, next_hist, stream);
}

fr_status fr_beam_expand(const float *logp, const int32_t *token_ids, int64_t M, int32_t k,
                         const float *node_score, const int32_t *node_hist, int32_t width,
                         float *hist_score, int32_t *hist_token, int32_t *hist_parent,
                         int64_t hist_offset, float *next_score, int32_t *next_token,
                         int32_t *next_hist, fr_stream stream) {
    if (!logp || !token_ids || !node_score || !node_hist || !hist_score || !hist_token || !hist_parent ||
        !next_score || !next_token || !next_hist)
        return FR_ERR_INVALID_ARG;
    if (M < 1 || k < 1 || width < 1 || hist_offset < 0 || hist_offset > INT32_MAX) return FR_ERR_INVALID_ARG;
    if (M > kGlueMaxCandidates || M * k > kGlueMaxCandidates) return FR_ERR_UNSUPPORTED;
    if (width > M * k || hist_offset + M * k > INT32_MAX) return FR_ERR_INVALID_ARG;
    return launch_beam_expand(logp, token_ids, static_cast<int>(M * k), k, node_score, node_hist, width,
                              hist_score, hist_token, hist_parent, hist_offset, next_score, next_token,
                              next_hist, static_cast<hipStream_t>(stream));
}

fr_status fr_tree_select(const float *hist_score, const int32_t *hist_token,
                         const int32_t *hist_parent, int64_t N, int32_t K, int32_t *sel_index,
                         int32_t *sel_token, int32_t *sel_parent, int32_t *sel_depth,
                         uint8_t *tree_mask, fr_stream stream) {
    if (!hist_score || !hist_token || !hist_parent || !sel_index || !sel_token || !sel_parent || !sel_depth ||
        !tree_mask)
        return FR_ERR_INVALID_ARG;
    if (N < 1 || K < 1 || K > N) return FR_ERR_INVALID_ARG;
    if (N > kGlueMaxCandidates || K > kGlueMaxTree) return FR_ERR_UNSUPPORTED;
    return launch_tree_select(hist_score, hist_token, hist_parent, static_cast<int>(N), K, sel_index, sel_token,
                              sel_parent, sel_depth, tree_mask, static_cast<hipStream_t>(stream));
}

fr_status fr_count_tokens(const int32_t *tokens, int64_t n_tokens, int64_t V, int64_t *counts,
                          int32_t *dev_error_flag, fr_stream stream) {
    if (!counts || (!tokens && n_tokens > 0) || n_tokens < 0 || V < 1 || V > INT32_MAX) return FR_ERR_INVALID_ARG;
    if (tokens && !aligned16(tokens)) return FR_ERR_ALIGNMENT;
    if ((reinterpret_cast<uintptr_t>(counts) & 7u) != 0) return FR_ERR_ALIGNMENT;
    if (V > (1 << 22)) return FR_ERR_UNSUPPORTED;   // as the ranking: vocabularies, not hash spaces
    if (n_tokens == 0) return FR_OK;
    return launch_count_tokens(tokens, n_tokens, static_cast<int>(V), reinterpret_cast<unsigned long long *>(counts),
                               dev_error_flag, static_cast<hipStream_t>(stream));
}

fr_status fr_rank_tokens(const int64_t *counts, int64_t V, int32_t *freq_ranked_ids, fr_stream stream) {
    if (!counts || !freq_ranked_ids || V < 1 || V > INT32_MAX) return FR_ERR_INVALID_ARG;
    if (V > (1 << 22)) return FR_ERR_UNSUPPORTED;   // the all-pairs ranking is meant for vocabularies
    return launch_rank_tokens(reinterpret_cast<const long long *>(counts), static_cast<int>(V), freq_ranked_ids,
                              static_cast<hipStream_t>(stream));
}

fr_status fr_calib_copy(void *dst, const void *src, size_t bytes, fr_stream stream) {
    if (!dst || !src || (bytes % 16) != 0) return FR_ERR_INVALID_ARG;
    if (!aligned16(dst) || !aligned16(src)) return FR_ERR_ALIGNMENT;
    return launch_copy(dst, src, bytes, static_cast<hipStream_t>(stream));
}

fr_status fr_calib_read(const void *src, size_t bytes, void *sink, fr_stream stream) {
    if (!src || !sink || (bytes % 16) != 0) return FR_ERR_INVALID_ARG;
    if (!aligned16(src) || !aligned16(sink)) return FR_ERR_ALIGNMENT;
    return launch_read(src, bytes, sink, static_cast<hipStream_t>(stream));
}

}  // extern "C"
