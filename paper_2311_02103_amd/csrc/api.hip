// C ABI of librelax_mi355.so: argument checks (all on the host, before anything is enqueued),
// the workspace plan, and the launch sequence of each exported call.  See include/relax_mi355.h
// for the contract and for the passages of the paper each rule comes from.
#include <atomic>
#include <cstring>
#include <mutex>

#include "relax_common.h"

using namespace relax;

namespace {

inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

// ---- Dynamic shape-aware memory planning (Sec. 4.3, Alg. 3) over the intermediates of one layer call ----------------------
// The layer is a fixed sequence of destination-passing operations; every intermediate has a symbolic size in the rows n
// of the call (a monomial c * n bytes) or an opaque expression of (n, L, B) (the workspaces lifted out of the attention
// and few-row matmul kernels, Sec. 4.4).  Tensors are walked in program order: an allocation first asks the pool for a free
// storage that PROVABLY fits whatever the symbols are (c1 * n into c2 * n when c1 <= c2; an opaque expression only into
// the same expression), smallest such first, else opens a new storage; after the last use of a tensor its storage goes
// back to the pool.  Reuse therefore never depends on the values of n, L, B: the storage structure is the same for every
// call, every storage size grows with the symbols, and a workspace sized at the upper bounds (n_max, L_max, B_max) covers
// every smaller call -- the static plan of Sec. 4.3.
enum PlanTensorId { T_XN, T_QKV, T_MMWS1, T_PART, T_ATTN, T_X1, T_MMWS3, T_ACT, T_MMWS5, T_MMWS6, T_COUNT };
const char *const kPlanNames[T_COUNT] = {"xn", "qkv", "matmul_ws.qkv", "attn_partials", "attn_out", "x1", "matmul_ws.o", "act", "matmul_ws.gate_up",
                                         "matmul_ws.down"};
struct SymBytes {
    uint64_t per_row;                // > 0: the tensor is per_row * n bytes
    int opaque;                      // per_row == 0: number of the opaque expression
    size_t value;                    // bytes at this call's (n, L, B)
};
struct PlanTensor {
    SymBytes size;
    int first_op, last_op;           // operations of the layer: 1 QKV (+ rotary, append), 2 attention, 3 output projection, 4 second norm, 5 gate/up, 6 down
    int storage;
};
struct MemPlan {
    PlanTensor t[T_COUNT];
    SymBytes storage_size[T_COUNT];
    size_t storage_off[T_COUNT];
    int n_storages;
    size_t planned, unplanned;       // bytes with and without reuse (every storage / tensor rounded up to 256 bytes)
};

inline bool provably_fits(const SymBytes &want, const SymBytes &have)
{
    if (want.per_row > 0 && have.per_row > 0) return want.per_row <= have.per_row;
    if (want.per_row == 0 && have.per_row == 0) return want.opaque == have.opaque;
    return false;
}

// The reuse rule as Sec. 4.3 states it: a storage is reused only by a tensor whose symbolic size is the SAME expression.
inline bool provably_equal(const SymBytes &want, const SymBytes &have)
{
    if (want.per_row > 0 && have.per_row > 0) return want.per_row == have.per_row;
    if (want.per_row == 0 && have.per_row == 0) return want.opaque == have.opaque;
    return false;
}

// equal_only: the paper's rule (equal expressions); otherwise the extension the workspace layout uses (provably fits)
void plan_memory(MemPlan &mp, int n_ops, bool equal_only = false)
{
    bool is_free[T_COUNT] = {};
    mp.n_storages = 0;
    mp.unplanned = 0;
    for (int op = 0; op <= n_ops; ++op) {
        for (int id = 0; id < T_COUNT; ++id) {                     // allocations in front of the operation, in declaration order
            PlanTensor &t = mp.t[id];
            if (t.first_op != op) continue;
            mp.unplanned += align256(t.size.value);
            int best = -1;
            for (int s = 0; s < mp.n_storages; ++s) {
                if (!is_free[s] || !(equal_only ? provably_equal(t.size, mp.storage_size[s]) : provably_fits(t.size, mp.storage_size[s]))) continue;
                if (best < 0 || mp.storage_size[s].value < mp.storage_size[best].value) best = s;
            }
            if (best < 0) {
                best = mp.n_storages++;
                mp.storage_size[best] = t.size;
            }
            is_free[best] = false;
            t.storage = best;
        }
        for (int id = 0; id < T_COUNT; ++id)                       // tensors dead after the operation
            if (mp.t[id].last_op == op) is_free[mp.t[id].storage] = true;
    }
    mp.planned = 0;
    for (int s = 0; s < mp.n_storages; ++s) {
        mp.storage_off[s] = mp.planned;
        mp.planned += align256(mp.storage_size[s].value);
    }
}

// Static plan of the lifted workspace (Sec. 4.3 upper bounds, Sec. 4.4 lifting).  Offsets are a
// pure function of (dims, n, L, B); a call sized by upper bounds covers every smaller call.
struct WsPlan {
    size_t flags, table, partials, partials_end, qbuf, attn, x1, act, xn, qkv, skinny, total;
    size_t mm_floats;                // fp32 elements of the matmul workspace (at `skinny`)
    MemPlan mem;
};

WsPlan plan_ws(const relax_layer_dims &dm, int32_t n, int32_t L, int32_t B, bool equal_only = false)
{
    WsPlan p;
    size_t off = 0;
    const size_t hd = (size_t)dm.n_heads * dm.head_dim;
    const size_t qkvw = (size_t)(dm.n_heads + 2 * dm.n_kv_heads) * dm.head_dim;
    // one line of flags at offset 0 (relax_workspace_init / relax_workspace_error), then the descriptor table of large batches
    p.flags = off;    off += kWsFlagBytes;
    p.table = off;    off += align256(sizeof(int32_t) * 4 * (size_t)(B > 1 ? B : 1));

    // The intermediates of the layer, their sizes and live ranges.  xn is pinned for the whole call (allocated in front of
    // operation 0, never recycled): relax_model_step hands the next layer's normalised input over in it.  q of the one-row
    // path lives in the front of the qkv tensor.  The split-K partial tiles of the few-row matmul are one lifted workspace
    // (the largest of the four matrices, at most kSkinnyMaxN rows), allocated and released around each matmul.
    const int ns = n < kSkinnyMaxN ? n : kSkinnyMaxN;
    size_t fl = gemm_skinny_partial_floats((int)qkvw, dm.hidden, ns);
    const size_t f2 = gemm_skinny_partial_floats(dm.hidden, (int)hd, ns), f3 = gemm_skinny_partial_floats(2 * dm.ffn, dm.hidden, ns),
                 f4 = gemm_skinny_partial_floats(dm.hidden, dm.ffn, ns);
    fl = fl > f2 ? fl : f2, fl = fl > f3 ? fl : f3, fl = fl > f4 ? fl : f4;
    // ... or the partial tiles of the k-split form of the tiled GEMM (a few hundred rows on a matrix with few tiles)
    fl = std::max(std::max(fl, gemm_splitk_partial_floats((int)qkvw, dm.hidden, n, EPI_F16)),
                  std::max(gemm_splitk_partial_floats(dm.hidden, (int)hd, n, EPI_RESID_F32),
                           std::max(gemm_splitk_partial_floats(2 * dm.ffn, dm.hidden, n, EPI_SWIGLU),
                                    gemm_splitk_partial_floats(dm.hidden, dm.ffn, n, EPI_RESID_F16))));
    const SymBytes mmws = {0, 1, sizeof(float) * fl};
    p.mm_floats = fl;
    auto rows = [&](size_t per_row) { return SymBytes{per_row, 0, per_row * (size_t)n}; };
    MemPlan &mp = p.mem;
    const int kNever = 1 << 20;
    mp.t[T_XN] = {rows(2 * (size_t)dm.hidden), 0, kNever, -1};
    mp.t[T_QKV] = {rows(2 * qkvw), 1, 2, -1};
    mp.t[T_MMWS1] = {mmws, 1, 1, -1};
    mp.t[T_PART] = {SymBytes{0, 2, sizeof(float) * attn_partial_floats(dm, n, L)}, 2, 3, -1};
    mp.t[T_ATTN] = {rows(2 * hd), 2, 3, -1};
    mp.t[T_X1] = {rows(4 * (size_t)dm.hidden), 3, 6, -1};
    mp.t[T_MMWS3] = {mmws, 3, 3, -1};
    mp.t[T_ACT] = {rows(2 * (size_t)dm.ffn), 5, 6, -1};
    mp.t[T_MMWS5] = {mmws, 5, 5, -1};
    mp.t[T_MMWS6] = {mmws, 6, 6, -1};
    plan_memory(mp, 6, equal_only);
    auto at = [&](int id) { return off + mp.storage_off[mp.t[id].storage]; };
    p.xn = at(T_XN), p.qkv = at(T_QKV), p.qbuf = p.qkv, p.partials = at(T_PART), p.attn = at(T_ATTN), p.x1 = at(T_X1), p.act = at(T_ACT);
    p.skinny = at(T_MMWS1);                                        // the four requests are the same expression: same storage every time
    p.partials_end = p.partials + align256(mp.t[T_PART].size.value);
    p.total = off + mp.planned;
    return p;
}

relax_status check_dims(const relax_layer_dims *dm)
{
    if (!dm) return RELAX_ERR_NULL;
    if (dm->hidden < 8 || dm->n_heads < 1 || dm->n_kv_heads < 1 || dm->ffn < 8 || dm->kv_capacity < 1 || dm->kv_slots < 1)
        return RELAX_ERR_SHAPE;
    if (dm->n_heads % dm->n_kv_heads != 0 || dm->head_dim % 2 != 0) return RELAX_ERR_SHAPE;
    if (dm->head_dim != 64 && dm->head_dim != 128) return RELAX_ERR_UNSUPPORTED;
    if (dm->group != 32 && dm->group != 64 && dm->group != 128) return RELAX_ERR_UNSUPPORTED;
    return RELAX_OK;
}

relax_status check_qmat(const relax_qmat *w)
{
    if (!w || !w->q || !w->s) return RELAX_ERR_NULL;
    if (w->m < 1 || w->k < 8 || w->k % 8 != 0) return RELAX_ERR_SHAPE;
    if (w->k > kMaxK || gshift_of(w->group) < 0) return RELAX_ERR_UNSUPPORTED;
    return RELAX_OK;
}

// Validates the ragged descriptor against n and the cache, and builds the kernel-side table.
// need_table: the batch does not fit the inline arrays and the caller keeps no device table: upload_table has to write one.
relax_status build_seqs(const relax_seqs *sq, const relax_layer_dims &dm, int32_t n, SeqTable &st, int32_t &L_max, bool &need_table)
{
    need_table = false;
    if (!sq || !sq->q_lens || !sq->kv_lens) return RELAX_ERR_NULL;
    if (n < 1 || sq->B < 1) return RELAX_ERR_SHAPE;
    long long total = 0;
    L_max = 0;
    for (int b = 0; b < sq->B; ++b) {
        if (sq->q_lens[b] < 1 || sq->kv_lens[b] < sq->q_lens[b]) return RELAX_ERR_SHAPE;
        total += sq->q_lens[b];
    }
    if (total != n) return RELAX_ERR_SHAPE;
    for (int b = 0; b < sq->B; ++b) {
        const int32_t slot = sq->slots ? sq->slots[b] : b;
        if (sq->kv_lens[b] > dm.kv_capacity || slot < 0 || slot >= dm.kv_slots) return RELAX_ERR_CAPACITY;
        if (sq->kv_lens[b] > L_max) L_max = sq->kv_lens[b];
    }
    st.B = sq->B;
    st.n = n;
    st.dev = nullptr;
    st.q_max = 0;
    for (int b = 0; b < sq->B; ++b) st.q_max = sq->q_lens[b] > st.q_max ? sq->q_lens[b] : st.q_max;
    if (sq->device_table) {
        // The caller keeps the descriptor on the device (Sec. 4.7 shape heap): kernels read positions and slots there at run
        // time; the host values above served the checks and serve the launch shapes and plans (kv_lens as upper bounds).
        if ((reinterpret_cast<uintptr_t>(sq->device_table) & 3) != 0) return RELAX_ERR_SHAPE;
        st.dev = sq->device_table;
        for (int b = 0; b < kInlineSeqs; ++b) st.q_start[b] = st.q_len[b] = st.kv_len[b] = st.slot[b] = 0;
        return RELAX_OK;
    }
    for (int b = 0; b < kInlineSeqs; ++b) st.q_start[b] = st.q_len[b] = st.kv_len[b] = st.slot[b] = 0;
    if (sq->B > kInlineSeqs) {
        need_table = true;
        return RELAX_OK;
    }
    int32_t start = 0;
    for (int b = 0; b < sq->B; ++b) {
        st.q_start[b] = start, st.q_len[b] = sq->q_lens[b], st.kv_len[b] = sq->kv_lens[b], st.slot[b] = sq->slots ? sq->slots[b] : b;
        start += sq->q_lens[b];
    }
    return RELAX_OK;
}

// Large batches: the descriptor goes to the device table at the front of the workspace, 32 sequences per launch of a small
// kernel that carries them in its arguments (the extra symbolic arguments of Sec. 3.3): no host buffer has to outlive the
// call, nothing is copied from pageable memory, the host never waits, and the launches can be captured in a graph.
relax_status upload_table(SeqTable &st, const relax_seqs *sq, bool need_table, void *ws, const WsPlan &pl, hipStream_t stream)
{
    if (!need_table) return RELAX_OK;
    int32_t *dev = reinterpret_cast<int32_t *>(static_cast<char *>(ws) + pl.table);
    TableChunk c = {};
    c.B = sq->B;
    int32_t start = 0;
    for (int first = 0; first < sq->B; first += kTableChunk) {
        c.first = first;
        c.count = sq->B - first < kTableChunk ? sq->B - first : kTableChunk;
        for (int j = 0; j < c.count; ++j) {
            const int b = first + j;
            c.q_start[j] = start, c.q_len[j] = sq->q_lens[b], c.kv_len[j] = sq->kv_lens[b], c.slot[j] = sq->slots ? sq->slots[b] : b;
            start += sq->q_lens[b];
        }
        if (launch_table_write(dev, c, stream) != hipSuccess) return RELAX_ERR_HIP;
    }
    st.dev = dev;
    return RELAX_OK;
}

// RELAX_LOG_ERRORS in the environment: the HIP error behind a RELAX_ERR_HIP goes to stderr
inline relax_status hip_status(hipError_t e)
{
    if (e == hipSuccess) return RELAX_OK;
    static const bool log = getenv("RELAX_LOG_ERRORS") != nullptr;
    if (log) fprintf(stderr, "relax_mi355: HIP error %d (%s)\n", (int)e, hipGetErrorString(e));
    return RELAX_ERR_HIP;
}

// One-shot measurement hook (relax_profile_step_events): events around one step of the next layer call.
thread_local hipEvent_t g_prof_start = nullptr, g_prof_stop = nullptr;
thread_local int g_prof_step = -1;

struct StepTimer {
    hipEvent_t start, stop;
    int step;
    hipStream_t stream;
    explicit StepTimer(hipStream_t s) : start(g_prof_start), stop(g_prof_stop), step(g_prof_step), stream(s)
    {
        g_prof_start = g_prof_stop = nullptr;
        g_prof_step = -1;
    }
    void before(int s) const { if (s == step && start) (void)hipEventRecord(start, stream); }
    void after(int s) const { if (s == step && stop) (void)hipEventRecord(stop, stream); }
};

// Test / measurement switches (relax_set_option, relax_profile_alt_gate_up; declared in relax_mi355_bench.h).  Process-wide by
// design -- they exist for A/B tests of one process -- and atomic, so setting one while another thread is inside a call is
// defined: that call sees the old or the new value.  Neither changes a result.
std::atomic<int> g_opt_fuse_finish{1};       // few-row path: light steps folded into the finishing pass of the split-K matmuls
std::atomic<int> g_opt_matvec_mb{96};        // ... and the size of the largest matrix (MB of packed codes) up to which that holds for more than two rows
std::atomic<int> g_opt_matvec_rows{4};       // relax_decoder_layer on a model whose matrices fit the last-level cache: rows up to which the matvec kernels take the call
std::atomic<int> g_opt_half_gemm_rows{0};    // relax_half_matmul: rows from which the tiled GEMM replaces the matvec passes; 0: by estimate
std::atomic<const uint32_t *> g_prof_alt_q{nullptr};      // relax_profile_alt_gate_up: another matrix of the gate/up shape
std::atomic<const uint16_t *> g_prof_alt_s{nullptr};

// CU count of the current device (the fused kernel launches exactly one workgroup per CU).
int device_cus()
{
    static int cus[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
    if (cus[dev] == 0) {
        int v = 0;
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
        cus[dev] = v;
    }
    return cus[dev];
}

// out[n,m] = x[n,k] . w[m,k]^T on plain fp16 weights (relax_half_matmul, and the LM head of relax_model_step).
// The same runtime dispatch on the symbolic n as the int4 path (Sec. 5.1): matvec passes for a few rows, tiled MFMA GEMM from
// there on.  Where "there" is depends on the matrix: a pass streams the whole matrix (5.5 TB/s; passes of 8 rows are
// bound by their dot products and take twice as long), a GEMM launch with few rows costs its k loop whatever n is
// (0.5 us per 64 columns, more when its tiles fill the device); wider passes also cost more when only one block's x rows fit
// a CU.  Measured on 4096 x 4096: matvec up to 16 rows (33 against 36 us), GEMM from 24 (36 against 47); on 22016 x 4096:
// matvec up to 4 rows (35 against 46 us), GEMM from 6 (44 against 62); on 4096 x 11008: GEMM from 16 (94 against 120).
hipError_t half_matmul_enqueue(const uint16_t *x, const uint16_t *w, uint16_t *out, int n, int m, int k, hipStream_t st_)
{
    bool use_gemm;
    const int gemm_rows = g_opt_half_gemm_rows.load();
    if (gemm_rows > 0) {
        use_gemm = n >= gemm_rows;
    } else {
        const double pass_us = (double)m * k * 2.0 / 5.5e6;
        const int per = lm_head_rows_per_pass(k);                 // rows of x the matvec kernel holds in LDS
        double mv_us = 0.0;
        for (int left = n; left > 0;) {
            const int nb = left >= 8 && per >= 8 ? 8 : left >= 4 && per >= 4 ? 4 : left >= 2 && per >= 2 ? 2 : 1;
            const bool one_block_per_cu = (size_t)2 * nb * k * 2 > 150 * 1024;      // the x rows of two blocks no longer fit a CU
            mv_us += pass_us * (nb == 8 ? 2.0 : nb == 4 ? 1.15 : 1.0) * (one_block_per_cu ? 1.35 : 1.0) + 3.0;
            left -= nb;
        }
        const double tiles = (double)((m + 127) / 128) * ((n + 63) / 64);
        // ... and never less than its own pass over the matrix (the GEMM streams a tall matrix at about 4.3 TB/s: 262 MB in 61.6 us
        // at one row, where the estimate of the k loop alone said 45 and the matvec pass takes 45.4)
        const double gemm_us = std::max((k / 64.0) * (0.5 + 0.15 * std::min(tiles / 256.0, 1.0)) * std::max(1.0, tiles / 256.0),
                                        (double)m * k * 2.0 / 4.3e6) + 4.0;
        use_gemm = n > 64 || gemm_us < mv_us;
    }
    if (use_gemm && gemm_f16_eligible(x, w, out, m, k)) return launch_gemm_f16(x, w, n, m, k, out, st_);
    return launch_lm_head(x, w, out, n, k, m, device_cus(), st_);
}

// Scratch of relax_attention_static: the split-L partials of one call live in this file-scope device array instead of a
// caller workspace.  Every GPU holds its own copy at its own address; the name is a host-side stand-in, so the address is
// asked for once per device (with that device current) and only that pointer is ever handed to kernels.
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
__device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

relax_status static_scratch(void **out)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return RELAX_ERR_HIP;
    if (dev < 0 || dev >= kMaxDevices) return RELAX_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        const relax_status rc = hip_status(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (rc != RELAX_OK) return rc;
        if (!p) return RELAX_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return RELAX_OK;
}

}  // namespace

extern "C" {

void relax_profile_alt_gate_up(const void *q_alt, const void *s_alt)
{
    g_prof_alt_q.store(static_cast<const uint32_t *>(q_alt));
    g_prof_alt_s.store(static_cast<const uint16_t *>(s_alt));
}

relax_status relax_set_option(const char *name, int32_t value)
{
    if (!name) return RELAX_ERR_NULL;
    if (std::strcmp(name, "fuse_finish") == 0) {
        g_opt_fuse_finish.store(value);
        return RELAX_OK;
    }
    if (std::strcmp(name, "gemm_waves_per_simd") == 0) {
        if (value != 1 && value != 2) return RELAX_ERR_SHAPE;
        gemm_set_waves_per_simd(value);
        return RELAX_OK;
    }
    if (std::strcmp(name, "layer_matvec_rows") == 0) {
        if (value < 1 || value > 64) return RELAX_ERR_SHAPE;
        g_opt_matvec_rows.store(value);
        return RELAX_OK;
    }
    if (std::strcmp(name, "layer_matvec_mb") == 0) {
        if (value < 0 || value > 4096) return RELAX_ERR_SHAPE;
        g_opt_matvec_mb.store(value);
        return RELAX_OK;
    }
    if (std::strcmp(name, "half_matmul_gemm_rows") == 0) {
        if (value < 0) return RELAX_ERR_SHAPE;
        g_opt_half_gemm_rows.store(value);
        return RELAX_OK;
    }
    return RELAX_ERR_UNSUPPORTED;
}

relax_status relax_workspace_init(const relax_layer_dims *dims, void *ws, size_t ws_bytes, relax_stream stream)
{
    relax_status rc = check_dims(dims);
    if (rc != RELAX_OK) return rc;
    if (!ws) return RELAX_ERR_NULL;
    if (ws_bytes < kWsFlagBytes) return RELAX_ERR_WORKSPACE;
    if ((reinterpret_cast<uintptr_t>(ws) & 255) != 0) return RELAX_ERR_WORKSPACE;
    return hip_status(launch_ws_clear(ws, kWsFlagBytes, static_cast<hipStream_t>(stream)));
}

relax_status relax_workspace_error(const relax_layer_dims *dims, const void *ws, int32_t *flag_host)
{
    relax_status rc = check_dims(dims);
    if (rc != RELAX_OK) return rc;
    if (!ws || !flag_host) return RELAX_ERR_NULL;
    uint32_t v = 0;
    if (hipMemcpy(&v, ws, sizeof(v), hipMemcpyDeviceToHost) != hipSuccess)
        return RELAX_ERR_HIP;
    *flag_host = (int32_t)v;
    return RELAX_OK;
}

void relax_profile_step_events(void *start, void *stop, int32_t step)
{
    const bool on = start && stop && step >= 0;
    g_prof_start = on ? static_cast<hipEvent_t>(start) : nullptr;
    g_prof_stop = on ? static_cast<hipEvent_t>(stop) : nullptr;
    g_prof_step = on ? step : -1;
}

relax_status relax_probe_stream_read(const void *buf, size_t bytes, uint32_t *sink, relax_stream stream)
{
    if (!buf || !sink) return RELAX_ERR_NULL;
    if (bytes < 16 || (reinterpret_cast<uintptr_t>(buf) & 15) != 0) return RELAX_ERR_SHAPE;
    return hip_status(launch_probe_stream_read(buf, bytes, sink, device_cus(), static_cast<hipStream_t>(stream)));
}

relax_status relax_probe_mfma(float *sink, int32_t iters, int32_t random_data, int64_t *flops, relax_stream stream)
{
    if (!sink || !flops) return RELAX_ERR_NULL;
    if (iters < 1) return RELAX_ERR_SHAPE;
    const int cus = device_cus();
    *flops = (int64_t)cus * 4 * iters * 16 * (2LL * 32 * 32 * 16);
    return hip_status(launch_probe_mfma(sink, iters, random_data, cus, static_cast<hipStream_t>(stream)));
}

const char *relax_build_id(void) { return "relax_mi355 gfx950 " __DATE__ " " __TIME__; }

size_t relax_workspace_bytes(const relax_layer_dims *dims, int32_t n_max, int32_t L_max, int32_t B_max)
{
    if (check_dims(dims) != RELAX_OK || n_max < 1 || L_max < 1 || B_max < 1) return 0;
    return plan_ws(*dims, n_max, L_max, B_max).total;
}

relax_status relax_workspace_plan(const relax_layer_dims *dims, int32_t n, int32_t L, int32_t B, relax_plan_entry *entries, int32_t capacity,
                                  int32_t *count, size_t *planned_bytes, size_t *unplanned_bytes)
{
    return relax_workspace_plan_rule(dims, n, L, B, 0, entries, capacity, count, planned_bytes, unplanned_bytes);
}

relax_status relax_workspace_plan_rule(const relax_layer_dims *dims, int32_t n, int32_t L, int32_t B, int32_t rule, relax_plan_entry *entries,
                                       int32_t capacity, int32_t *count, size_t *planned_bytes, size_t *unplanned_bytes)
{
    const relax_status rc = check_dims(dims);
    if (rc != RELAX_OK) return rc;
    if (n < 1 || L < 1 || B < 1) return RELAX_ERR_SHAPE;
    if (rule != 0 && rule != 1) return RELAX_ERR_UNSUPPORTED;
    const WsPlan pl = plan_ws(*dims, n, L, B, rule == 1);
    const size_t base = pl.total - pl.mem.planned;               // the planned region follows the fixed front part
    if (count) *count = T_COUNT;
    if (planned_bytes) *planned_bytes = pl.mem.planned;
    if (unplanned_bytes) *unplanned_bytes = pl.mem.unplanned;
    if (entries) {
        if (capacity < T_COUNT) return RELAX_ERR_WORKSPACE;
        for (int id = 0; id < T_COUNT; ++id) {
            relax_plan_entry &e = entries[id];
            std::memset(&e, 0, sizeof(e));
            std::strncpy(e.name, kPlanNames[id], sizeof(e.name) - 1);
            e.first_op = pl.mem.t[id].first_op;
            e.last_op = pl.mem.t[id].last_op > 6 ? 6 : pl.mem.t[id].last_op;
            e.storage = pl.mem.t[id].storage;
            e.pinned = pl.mem.t[id].last_op > 6;
            e.offset = base + pl.mem.storage_off[pl.mem.t[id].storage];
            e.bytes = pl.mem.t[id].size.value;
            e.storage_bytes = pl.mem.storage_size[pl.mem.t[id].storage].value;
        }
    }
    return RELAX_OK;
}

size_t relax_rope_table_bytes(const relax_layer_dims *dims)
{
    if (check_dims(dims) != RELAX_OK) return 0;
    return sizeof(float) * 2 * (size_t)dims->kv_capacity * (size_t)(dims->head_dim / 2);
}

relax_status relax_rope_table_init(const relax_layer_dims *dims, float *table, relax_stream stream)
{
    relax_status rc = check_dims(dims);
    if (rc != RELAX_OK) return rc;
    if (!table) return RELAX_ERR_NULL;
    return hip_status(launch_rope_table(*dims, table, static_cast<hipStream_t>(stream)));
}

size_t relax_matmul_workspace_bytes(const relax_qmat *w, int32_t n_max)
{
    if (check_qmat(w) != RELAX_OK || n_max < 1) return 0;
    const int ns = n_max < kSkinnyMaxN ? n_max : kSkinnyMaxN;
    return align256(sizeof(float) * std::max(gemm_skinny_partial_floats(w->m, w->k, ns), gemm_splitk_partial_floats(w->m, w->k, n_max, EPI_F16)));
}

relax_status relax_dequant_matmul(const uint16_t *x, const relax_qmat *w, uint16_t *out, int32_t n, void *ws, size_t ws_bytes,
                                  relax_stream stream)
{
    if (!x || !out) return RELAX_ERR_NULL;
    relax_status rc = check_qmat(w);
    if (rc != RELAX_OK) return rc;
    if (n < 1) return RELAX_ERR_SHAPE;
    // runtime dispatch on the symbolic n (Sec. 5.1): matrix-vector kernel for one row, split-K MFMA kernel for a few
    // (when the caller brought the workspace for its partial tiles), tiled MFMA GEMM otherwise
    const bool tiled_first = gemm_prefers_tiled(w->m, n) && gemm_mfma_eligible(*w, x, EPI_F16);
    if (!tiled_first && n >= kSkinnyMinN && n <= kSkinnyMaxN && ws && gemm_skinny_eligible(*w, x, n, EPI_F16) &&
        (reinterpret_cast<uintptr_t>(ws) & 15) == 0 && ws_bytes >= sizeof(float) * gemm_skinny_partial_floats(w->m, w->k, n))
        return hip_status(launch_gemm_skinny(x, *w, n, EPI_F16, out, nullptr, nullptr, static_cast<float *>(ws),
                                             static_cast<hipStream_t>(stream)));
    if (n >= kGemmMinN && gemm_mfma_eligible(*w, x, EPI_F16))
        return hip_status(launch_gemm_mfma(x, *w, n, EPI_F16, out, nullptr, nullptr, static_cast<hipStream_t>(stream), static_cast<float *>(ws),
                                           ws ? ws_bytes / sizeof(float) : 0));
    GemvArgs a = {};
    a.x = x, a.q = w->q, a.s = w->s, a.m = w->m, a.k = w->k, a.n = n, a.out_f16 = out, a.gshift = gshift_of(w->group);
    return hip_status(launch_gemv(a, X_F16, EPI_F16, static_cast<hipStream_t>(stream)));
}

relax_status relax_rmsnorm_rope(const uint16_t *x, const uint16_t *w, uint16_t *y, int32_t n, int32_t H, float eps, uint16_t *qkv,
                                const relax_layer_dims *dims, const relax_kv_cache *cache, const relax_seqs *seqs,
                                relax_stream stream)
{
    hipStream_t st_ = static_cast<hipStream_t>(stream);
    if (!x && !qkv) return RELAX_ERR_NULL;
    if (n < 1) return RELAX_ERR_SHAPE;
    SeqTable st = {};
    bool need_table = false;
    if (x) {
        if (!w || !y) return RELAX_ERR_NULL;
        if (H < 1) return RELAX_ERR_SHAPE;
    }
    if (qkv) {
        relax_status rc = check_dims(dims);
        if (rc != RELAX_OK) return rc;
        if (!cache || !cache->k || !cache->v || !cache->rope) return RELAX_ERR_NULL;
        int32_t L_max = 0;
        rc = build_seqs(seqs, *dims, n, st, L_max, need_table);
        if (rc != RELAX_OK) return rc;
        if (need_table) return RELAX_ERR_UNSUPPORTED;            // this call takes no workspace: B <= 16, or a device table
    }
    if (x) {
        relax_status rc = hip_status(launch_rmsnorm(x, w, y, n, H, eps, st_));
        if (rc != RELAX_OK) return rc;
    }
    if (qkv) return hip_status(launch_rope_append(qkv, *dims, *cache, st, st_));
    return RELAX_OK;
}

relax_status relax_attention(const uint16_t *q, const relax_kv_cache *cache, const relax_seqs *seqs, const relax_layer_dims *dims,
                             uint16_t *out, int32_t n, void *ws, size_t ws_bytes, relax_stream stream)
{
    hipStream_t st_ = static_cast<hipStream_t>(stream);
    relax_status rc = check_dims(dims);
    if (rc != RELAX_OK) return rc;
    if (!q || !out || !cache || !cache->k || !cache->v || !ws) return RELAX_ERR_NULL;
    SeqTable st = {};
    bool need_table = false;
    int32_t L_max = 0;
    rc = build_seqs(seqs, *dims, n, st, L_max, need_table);
    if (rc != RELAX_OK) return rc;
    const WsPlan pl = plan_ws(*dims, n, L_max, seqs->B);
    if (ws_bytes < pl.partials_end || (reinterpret_cast<uintptr_t>(ws) & 255) != 0) return RELAX_ERR_WORKSPACE;   // table + partials
    rc = upload_table(st, seqs, need_table, ws, pl, st_);
    if (rc != RELAX_OK) return rc;
    float *partials = reinterpret_cast<float *>(static_cast<char *>(ws) + pl.partials);
    return hip_status(launch_attention(q, dims->n_heads * dims->head_dim, *cache, *dims, st, L_max, out, partials, st_));
}

size_t relax_attention_static_max_bytes(void) { return kStaticScratchBytes; }

relax_status relax_attention_static(const uint16_t *q, const relax_kv_cache *cache, const relax_seqs *seqs, const relax_layer_dims *dims,
                                    uint16_t *out, int32_t n, relax_stream stream)
{
    hipStream_t st_ = static_cast<hipStream_t>(stream);
    relax_status rc = check_dims(dims);
    if (rc != RELAX_OK) return rc;
    if (!q || !out || !cache || !cache->k || !cache->v) return RELAX_ERR_NULL;
    SeqTable st = {};
    bool need_table = false;
    int32_t L_max = 0;
    if (seqs && !seqs->device_table && seqs->B > kInlineSeqs) return RELAX_ERR_UNSUPPORTED;   // the copy of a long descriptor needs a workspace
    rc = build_seqs(seqs, *dims, n, st, L_max, need_table);
    if (rc != RELAX_OK) return rc;
    const size_t need = sizeof(float) * attn_partial_floats(*dims, n, L_max);
    if (need > kStaticScratchBytes) return RELAX_ERR_WORKSPACE;
    void *base = nullptr;
    rc = static_scratch(&base);
    if (rc != RELAX_OK) return rc;
    return hip_status(launch_attention(q, dims->n_heads * dims->head_dim, *cache, *dims, st, L_max, out, static_cast<float *>(base), st_));
}

}  // extern "C"

namespace {

// Shape checks of one layer's weights against the static dims.
relax_status check_layer(const relax_layer_dims &dm, const relax_layer_weights *wt)
{
    if (!wt || !wt->norm_attn || !wt->norm_ffn) return RELAX_ERR_NULL;
    const relax_qmat *mats[4] = {&wt->wqkv, &wt->wo, &wt->wgu, &wt->wdown};
    for (const relax_qmat *mq : mats) {
        const relax_status rc = check_qmat(mq);
        if (rc != RELAX_OK) return rc;
    }
    const int32_t hd = dm.n_heads * dm.head_dim, qkvw = (dm.n_heads + 2 * dm.n_kv_heads) * dm.head_dim;
    if (wt->wqkv.m != qkvw || wt->wqkv.k != dm.hidden || wt->wo.m != dm.hidden || wt->wo.k != hd ||
        wt->wgu.m != 2 * dm.ffn || wt->wgu.k != dm.hidden || wt->wdown.m != dm.hidden || wt->wdown.k != dm.ffn)
        return RELAX_ERR_SHAPE;
    for (const relax_qmat *mq : mats)
        if ((kGroup << gshift_of(mq->group)) != dm.group) return RELAX_ERR_SHAPE;   // one quantisation group per layer
    return RELAX_OK;
}

// Enqueues one decoder layer.  Everything has been validated; st is the kernel-side ragged descriptor (its device
// table, if any, already uploaded); base/pl are the layer workspace and its plan.
// next_norm (optional): the RMSNorm weights of the layer that follows; when the few-row path can, it leaves RMSNorm(out) * next_norm in the
// workspace and sets *xn_done, and the next call passes xn_ready to skip its own first RMSNorm.
relax_status layer_enqueue(const relax_layer_dims &dm, const relax_layer_weights *wt, const uint16_t *x, const relax_kv_cache *cache,
                           const SeqTable &st, int32_t L_max, uint16_t *out, int32_t n, char *base, const WsPlan &pl, hipStream_t st_,
                           const uint16_t *next_norm = nullptr, bool xn_ready = false, bool *xn_done = nullptr)
{
    if (xn_done) *xn_done = false;
    const int32_t hd = dm.n_heads * dm.head_dim, qkvw = (dm.n_heads + 2 * dm.n_kv_heads) * dm.head_dim;
    const StepTimer timer(st_);

    float *partials = reinterpret_cast<float *>(base + pl.partials);

    // More than one row: matrix path (same entry point, same binary) -- the matmuls run on MFMA, as the split-K
    // few-row kernel up to kSkinnyMaxN rows and as the tiled GEMM above, with the light steps as separate kernels.
    float *skinny_ws = reinterpret_cast<float *>(base + pl.skinny);
    auto mat_ok = [&](const relax_qmat &wq, const void *xin, int epi) {
        return (n <= kSkinnyMaxN && gemm_skinny_eligible(wq, xin, n, epi)) || (n >= kGemmMinN && gemm_mfma_eligible(wq, xin, epi));
    };
    auto few_row = [&](const relax_qmat &wq, const void *xin, int epi) {      // the few-row kernel takes this matmul
        if (gemm_prefers_tiled(wq.m, n) && n >= kGemmMinN && gemm_mfma_eligible(wq, xin, epi)) return false;
        return n <= kSkinnyMaxN && gemm_skinny_eligible(wq, xin, n, epi);
    };
    auto matmul = [&](const uint16_t *xin, const relax_qmat &wq, int epi, uint16_t *o16, float *o32, const void *resid) {
        if (few_row(wq, xin, epi)) return launch_gemm_skinny(xin, wq, n, epi, o16, o32, resid, skinny_ws, st_);
        return launch_gemm_mfma(xin, wq, n, epi, o16, o32, resid, st_, skinny_ws, pl.mm_floats);
    };
    // Up to four rows of a small model stay on the matvec kernels: two or four rows of x share one pass over the weights
    // (k <= 4096: four, k <= 8192: two; taller rows go one by one and find most of a matrix of this size in the last-level
    // cache), and the matvec path needs no separate norm / finishing launches.  Measured on the 7B layer shape, 256 cached
    // tokens: 46 against 75 us at two rows, 64 against 77 at three, 62 against 75 at four, 92 against 76 at five.
    const size_t largest = std::max(std::max((size_t)wt->wqkv.m * wt->wqkv.k, (size_t)wt->wo.m * wt->wo.k),
                                    std::max((size_t)wt->wgu.m * wt->wgu.k, (size_t)wt->wdown.m * wt->wdown.k)) / 2;
    // Two rows share one pass over the weights on every model size (measured per layer at L = 512: 13B shape 65 against 90 us on
    // the matrix path, 70B shape 112 against 167 us); three and four rows need a second pass where a lane cannot hold four rows
    // of x, which pays only while the matrices mostly stay in the last-level cache (13B: 94 against 92 us, 70B: 178 against 155).
    const bool rows_as_matvecs = n >= 2 && n <= g_opt_matvec_rows.load() && (n == 2 || largest <= ((size_t)g_opt_matvec_mb.load() << 20));
    if (n >= kSkinnyMinN && !rows_as_matvecs && mat_ok(wt->wqkv, x, EPI_F16) && mat_ok(wt->wo, x, EPI_RESID_F32) && mat_ok(wt->wgu, x, EPI_SWIGLU) &&
        mat_ok(wt->wdown, x, EPI_RESID_F16)) {
        uint16_t *xn = reinterpret_cast<uint16_t *>(base + pl.xn), *qkv = reinterpret_cast<uint16_t *>(base + pl.qkv);
        uint16_t *attn_o = reinterpret_cast<uint16_t *>(base + pl.attn), *act_o = reinterpret_cast<uint16_t *>(base + pl.act);
        float *x1f = reinterpret_cast<float *>(base + pl.x1);
        // few rows: the finishing pass of a split-K matmul also does the light step that follows it (rotary + append, RMSNorm)
        hipError_t fuse_err = hipSuccess;
        const bool fuse_finish = g_opt_fuse_finish.load() != 0;
        auto fused = [&](const uint16_t *xin, const relax_qmat &wq, int epi, uint16_t *o16, float *o32, const void *resid, const SkinnyFuse &f) {
            if (!fuse_finish || !gemm_skinny_fuse_ok(wq, epi, f)) return false;
            if (few_row(wq, xin, epi)) {
                fuse_err = launch_gemm_skinny(xin, wq, n, epi, o16, o32, resid, skinny_ws, st_, &f);
                return true;
            }
            if (n >= kGemmMinN && gemm_mfma_eligible(wq, xin, epi) && gemm_mfma_splits(wq, n, epi, skinny_ws, pl.mm_floats) > 1) {
                fuse_err = launch_gemm_mfma(xin, wq, n, epi, o16, o32, resid, st_, skinny_ws, pl.mm_floats, &f);    // k-split tiled GEMM
                return true;
            }
            return false;
        };
        timer.before(0);
        if (!xn_ready && launch_rmsnorm(x, wt->norm_attn, xn, n, dm.hidden, dm.rms_eps, st_) != hipSuccess) return RELAX_ERR_HIP;
        SkinnyFuse fq = {};
        fq.dm = &dm, fq.cache = cache, fq.st = &st;
        if (!fused(xn, wt->wqkv, EPI_F16, qkv, nullptr, nullptr, fq)) {
            if (matmul(xn, wt->wqkv, EPI_F16, qkv, nullptr, nullptr) != hipSuccess) return RELAX_ERR_HIP;
            if (launch_rope_append(qkv, dm, *cache, st, st_) != hipSuccess) return RELAX_ERR_HIP;
        }
        if (fuse_err != hipSuccess) return RELAX_ERR_HIP;
        timer.after(0);
        timer.before(1);
        if (launch_attention(qkv, qkvw, *cache, dm, st, L_max, attn_o, partials, st_) != hipSuccess) return RELAX_ERR_HIP;
        timer.after(1);
        timer.before(2);
        SkinnyFuse fo = {};
        fo.norm_w = wt->norm_ffn, fo.xn = xn, fo.eps = dm.rms_eps;
        const bool o_fused = fused(attn_o, wt->wo, EPI_RESID_F32, nullptr, x1f, x, fo);
        if (!o_fused && matmul(attn_o, wt->wo, EPI_RESID_F32, nullptr, x1f, x) != hipSuccess) return RELAX_ERR_HIP;
        if (fuse_err != hipSuccess) return RELAX_ERR_HIP;
        timer.after(2);
        if (!o_fused && launch_rmsnorm_f32(x1f, wt->norm_ffn, xn, n, dm.hidden, dm.rms_eps, st_) != hipSuccess) return RELAX_ERR_HIP;
        timer.before(3);                                  // step 3 brackets the gate/up matmul alone (the dominant kernel)
        if (matmul(xn, wt->wgu, EPI_SWIGLU, act_o, nullptr, nullptr) != hipSuccess) return RELAX_ERR_HIP;
        timer.after(3);
        timer.before(4);
        SkinnyFuse fd = {};
        fd.norm_w = next_norm, fd.xn = xn, fd.eps = dm.rms_eps;
        const bool d_fused = next_norm && xn_done && fused(act_o, wt->wdown, EPI_RESID_F16, out, nullptr, x1f, fd);
        if (!d_fused && matmul(act_o, wt->wdown, EPI_RESID_F16, out, nullptr, x1f) != hipSuccess) return RELAX_ERR_HIP;
        if (fuse_err != hipSuccess) return RELAX_ERR_HIP;
        if (d_fused) *xn_done = true;
        timer.after(4);
        return RELAX_OK;
    }

    uint16_t *qbuf = reinterpret_cast<uint16_t *>(base + pl.qbuf);
    uint16_t *attn = reinterpret_cast<uint16_t *>(base + pl.attn);
    float *x1 = reinterpret_cast<float *>(base + pl.x1);
    uint16_t *act = reinterpret_cast<uint16_t *>(base + pl.act);

    // 1. RMSNorm -> QKV matvec -> rotary embedding -> q to workspace, k/v appended to the cache
    GemvArgs a = {};
    a.x = x, a.norm_w = wt->norm_attn, a.eps = dm.rms_eps;
    a.q = wt->wqkv.q, a.s = wt->wqkv.s, a.m = wt->wqkv.m, a.k = wt->wqkv.k, a.n = n, a.gshift = gshift_of(wt->wqkv.group);
    a.out_f16 = qbuf, a.kcache = cache->k, a.vcache = cache->v, a.rope = cache->rope;
    a.h = dm.n_heads, a.g = dm.n_kv_heads, a.d = dm.head_dim, a.kv_capacity = dm.kv_capacity, a.seqs = st;
    if (n == 1 && st.dev == nullptr) a.pos0 = st.kv_len[0] - st.q_len[0] - st.q_start[0], a.slot0 = st.slot[0];
    else a.pos0 = -1;                                          // rows find their position in the descriptor
    timer.before(0);
    if (launch_gemv(a, X_F16_NORM, EPI_ROPE_KV, st_) != hipSuccess) return RELAX_ERR_HIP;
    timer.after(0);

    // 2. attention over the cache.  One row, one query head per KV head: the split kernel alone, with few enough
    //    splits for the output projection to fold the merge into its own prologue (one launch less per layer).
    GemvArgs o = {};
    o.q = wt->wo.q, o.s = wt->wo.s, o.m = wt->wo.m, o.k = wt->wo.k, o.n = n, o.gshift = gshift_of(wt->wo.group);
    o.out_f32 = x1, o.resid = x;
    bool folded = false;
    if (n == 1 && attn_mha_split_supported(dm)) {
        int splits = kAttnMergeSplits, chunk = 0, pos = -1;              // device-resident descriptor: every slice launched, plan on the device
        if (st.dev == nullptr) {
            pos = st.kv_len[0] - st.q_len[0] - st.q_start[0];
            chunk = attn_fold_chunk(pos + 1, kAttnMergeSplits);          // whole wavefront steps (16 or 32 tokens), all splits used
            splits = (pos + chunk) / chunk;
        }
        o.h = dm.n_heads, o.d = dm.head_dim, o.pos0 = pos, o.seqs = st;
        o.part = partials, o.part_splits = splits, o.part_stride = dm.head_dim / 2 + 4, o.part_chunk = chunk;
        folded = (size_t)dm.n_heads * splits * o.part_stride <= attn_partial_floats(dm, 1, 1) && gemv_merge_eligible(o);
        if (folded) {
            timer.before(1);
            if (launch_attention_mha_split(qbuf, hd, *cache, dm, st, chunk, splits, o.part_stride, partials, st_) != hipSuccess) return RELAX_ERR_HIP;
            timer.after(1);
        }
    }
    if (!folded) {
        timer.before(1);
        if (launch_attention(qbuf, hd, *cache, dm, st, L_max, attn, partials, st_) != hipSuccess) return RELAX_ERR_HIP;
        timer.after(1);
        o.x = attn;
    }

    // 3. output projection + residual: x1 = x + attn Wo^T (fp32 residual stream in the workspace)
    timer.before(2);
    if (launch_gemv(o, folded ? X_ATTN_MERGE : X_F16, EPI_RESID_F32, st_) != hipSuccess) return RELAX_ERR_HIP;
    timer.after(2);

    // 4. RMSNorm -> gate/up matvec -> SwiGLU
    GemvArgs f = {};
    f.x = x1, f.norm_w = wt->norm_ffn, f.eps = dm.rms_eps;
    f.q = wt->wgu.q, f.s = wt->wgu.s, f.m = wt->wgu.m, f.k = wt->wgu.k, f.n = n, f.gshift = gshift_of(wt->wgu.group);
    f.out_f16 = act;
    timer.before(3);
    const uint32_t *alt_q = g_prof_alt_q.load();
    const uint16_t *alt_s = g_prof_alt_s.load();
    if (alt_q && alt_s) {                        // measurement aid: one more launch of the same shape on other weights first
        GemvArgs f2 = f;
        f2.q = alt_q, f2.s = alt_s;
        if (launch_gemv(f2, X_F32_NORM, EPI_SWIGLU, st_) != hipSuccess) return RELAX_ERR_HIP;
    }
    if (launch_gemv(f, X_F32_NORM, EPI_SWIGLU, st_) != hipSuccess) return RELAX_ERR_HIP;
    timer.after(3);

    // 5. down projection + residual
    GemvArgs dn = {};
    dn.x = act, dn.q = wt->wdown.q, dn.s = wt->wdown.s, dn.m = wt->wdown.m, dn.k = wt->wdown.k, dn.n = n, dn.gshift = gshift_of(wt->wdown.group);
    dn.out_f16 = out, dn.resid = x1;
    timer.before(4);
    if (launch_gemv(dn, X_F16, EPI_RESID_F16, st_) != hipSuccess) return RELAX_ERR_HIP;
    timer.after(4);
    return RELAX_OK;
}

}  // namespace

extern "C" {

relax_status relax_decoder_layer(const relax_layer_dims *dims, const relax_layer_weights *wt, const uint16_t *x,
                                 const relax_kv_cache *cache, const relax_seqs *seqs, uint16_t *out, int32_t n, void *ws,
                                 size_t ws_bytes, relax_stream stream)
{
    hipStream_t st_ = static_cast<hipStream_t>(stream);
    relax_status rc = check_dims(dims);
    if (rc != RELAX_OK) return rc;
    if (!wt || !x || !out || !ws || !cache || !cache->k || !cache->v || !cache->rope) return RELAX_ERR_NULL;
    const relax_layer_dims &dm = *dims;
    rc = check_layer(dm, wt);
    if (rc != RELAX_OK) return rc;
    SeqTable st = {};
    bool need_table = false;
    int32_t L_max = 0;
    rc = build_seqs(seqs, dm, n, st, L_max, need_table);
    if (rc != RELAX_OK) return rc;
    const WsPlan pl = plan_ws(dm, n, L_max, seqs->B);
    if (ws_bytes < pl.total || (reinterpret_cast<uintptr_t>(ws) & 255) != 0) return RELAX_ERR_WORKSPACE;
    rc = upload_table(st, seqs, need_table, ws, pl, st_);
    if (rc != RELAX_OK) return rc;
    return layer_enqueue(dm, wt, x, cache, st, L_max, out, n, static_cast<char *>(ws), pl, st_);
}

}  // extern "C"

// ---- one decoder layer on 3-bit weights (native layout) ---------------------------------------------------------------
// The same layer, composed of launches of their own: the 3-bit matmuls have the plain fp16 epilogue only, so the light
// steps run between them (RMSNorm, rotary + append, attention, residual adds, SwiGLU).  Its workspace is laid out one
// intermediate after the other (nothing is shared: the schedule differs from the one the planner of the 4-bit layer walks).
// The layer on plain fp16 weights further down is the same sequence around relax_half_matmul's dispatch and shares the layout.
namespace {
struct Q3Plan {
    WsPlan ws;                       // flags, table and partials at their usual places (upload_table and the attention launch read them)
    size_t gu, tmp, total;
};
Q3Plan plan_q3(const relax_layer_dims &dm, int32_t n, int32_t L, int32_t B)
{
    Q3Plan p = {};
    const size_t hd = (size_t)dm.n_heads * dm.head_dim, qkvw = (size_t)(dm.n_heads + 2 * dm.n_kv_heads) * dm.head_dim;
    size_t off = 0;
    p.ws.flags = off;    off += kWsFlagBytes;
    p.ws.table = off;    off += align256(sizeof(int32_t) * 4 * (size_t)(B > 1 ? B : 1));
    p.ws.partials = off; off += align256(sizeof(float) * attn_partial_floats(dm, n, L));
    p.ws.partials_end = off;
    p.ws.xn = off;       off += align256(2 * (size_t)n * std::max((size_t)dm.hidden, hd));
    p.ws.qkv = off;      off += align256(2 * (size_t)n * qkvw);
    p.ws.attn = off;     off += align256(2 * (size_t)n * hd);
    p.ws.x1 = off;       off += align256(4 * (size_t)n * dm.hidden);
    p.ws.act = off;      off += align256(2 * (size_t)n * dm.ffn);
    p.gu = off;          off += align256(2 * (size_t)n * 2 * dm.ffn);
    p.tmp = off;         off += align256(2 * (size_t)n * dm.hidden);
    p.total = p.ws.total = off;
    return p;
}
// a relax_qmat of the native 3-bit layout that the matmul dispatch below can take for any n
relax_status check_q3mat(const relax_qmat &w, int32_t m, int32_t k)
{
    if (!w.q || !w.s) return RELAX_ERR_NULL;
    if (w.m != m || w.k != k || k % 32 != 0) return RELAX_ERR_SHAPE;
    if (w.group != 0 && w.group != 32) return RELAX_ERR_UNSUPPORTED;
    if ((reinterpret_cast<uintptr_t>(w.q) & 3) != 0 || (reinterpret_cast<uintptr_t>(w.s) & 1) != 0) return RELAX_ERR_SHAPE;
    if (!gemv_q3_supported(m, k)) return RELAX_ERR_UNSUPPORTED;   // rows longer than the matvec kernel keeps in registers
    return RELAX_OK;
}
hipError_t q3_matmul(const uint16_t *x, const relax_qmat &w, int32_t n, uint16_t *out, hipStream_t st_)
{
    if (n >= kQ3GemmRows && gemm_q3_eligible(x, w, out)) return launch_gemm_q3(x, w, n, out, st_);
    return launch_gemv_q3_native(x, w, n, out, st_);
}
}  // namespace

extern "C" {

size_t relax_layer_q3_workspace_bytes(const relax_layer_dims *dims, int32_t n_max, int32_t L_max, int32_t B_max)
{
    if (check_dims(dims) != RELAX_OK || n_max < 1 || L_max < 1 || B_max < 1) return 0;
    return plan_q3(*dims, n_max, L_max, B_max).total;
}

relax_status relax_decoder_layer_q3(const relax_layer_dims *dims, const relax_layer_weights *wt, const uint16_t *x,
                                    const relax_kv_cache *cache, const relax_seqs *seqs, uint16_t *out, int32_t n, void *ws,
                                    size_t ws_bytes, relax_stream stream)
{
    hipStream_t st_ = static_cast<hipStream_t>(stream);
    relax_status rc = check_dims(dims);
    if (rc != RELAX_OK) return rc;
    if (!wt || !x || !out || !ws || !cache || !cache->k || !cache->v || !cache->rope || !wt->norm_attn || !wt->norm_ffn) return RELAX_ERR_NULL;
    const relax_layer_dims &dm = *dims;
    const int32_t hd = dm.n_heads * dm.head_dim, qkvw = (dm.n_heads + 2 * dm.n_kv_heads) * dm.head_dim;
    if (dm.hidden % 8 != 0 || dm.ffn % 8 != 0) return RELAX_ERR_SHAPE;
    if ((rc = check_q3mat(wt->wqkv, qkvw, dm.hidden)) != RELAX_OK || (rc = check_q3mat(wt->wo, dm.hidden, hd)) != RELAX_OK ||
        (rc = check_q3mat(wt->wgu, 2 * dm.ffn, dm.hidden)) != RELAX_OK || (rc = check_q3mat(wt->wdown, dm.hidden, dm.ffn)) != RELAX_OK)
        return rc;
    if (((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(out)) & 15) != 0) return RELAX_ERR_SHAPE;
    SeqTable st = {};
    bool need_table = false;
    int32_t L_max = 0;
    rc = build_seqs(seqs, dm, n, st, L_max, need_table);
    if (rc != RELAX_OK) return rc;
    const Q3Plan pl = plan_q3(dm, n, L_max, seqs->B);
    if (ws_bytes < pl.total || (reinterpret_cast<uintptr_t>(ws) & 255) != 0) return RELAX_ERR_WORKSPACE;
    rc = upload_table(st, seqs, need_table, ws, pl.ws, st_);
    if (rc != RELAX_OK) return rc;

    char *base = static_cast<char *>(ws);
    uint16_t *xn = reinterpret_cast<uint16_t *>(base + pl.ws.xn), *qkv = reinterpret_cast<uint16_t *>(base + pl.ws.qkv);
    uint16_t *attn = reinterpret_cast<uint16_t *>(base + pl.ws.attn), *act = reinterpret_cast<uint16_t *>(base + pl.ws.act);
    uint16_t *gu = reinterpret_cast<uint16_t *>(base + pl.gu), *tmp = reinterpret_cast<uint16_t *>(base + pl.tmp);
    float *x1 = reinterpret_cast<float *>(base + pl.ws.x1), *partials = reinterpret_cast<float *>(base + pl.ws.partials);
    const size_t nh = (size_t)n * dm.hidden;

    // One row: the five launches of the 4-bit decode layer on the 3-bit stream of the same kernel (the norms, rotary + append,
    // the attention merge, the residuals and SwiGLU inside the four matrix-vector launches).
    if (n == 1) {
        GemvArgs a = {};
        a.x = x, a.norm_w = wt->norm_attn, a.eps = dm.rms_eps, a.q = wt->wqkv.q, a.s = wt->wqkv.s, a.m = qkvw, a.k = dm.hidden, a.n = 1;
        a.out_f16 = qkv, a.kcache = cache->k, a.vcache = cache->v, a.rope = cache->rope;
        a.h = dm.n_heads, a.g = dm.n_kv_heads, a.d = dm.head_dim, a.kv_capacity = dm.kv_capacity, a.seqs = st;
        if (st.dev == nullptr) a.pos0 = st.kv_len[0] - st.q_len[0] - st.q_start[0], a.slot0 = st.slot[0];
        else a.pos0 = -1;
        GemvArgs o = {};
        o.x = attn, o.q = wt->wo.q, o.s = wt->wo.s, o.m = dm.hidden, o.k = hd, o.n = 1, o.out_f32 = x1, o.resid = x;
        GemvArgs f = {};
        f.x = x1, f.norm_w = wt->norm_ffn, f.eps = dm.rms_eps, f.q = wt->wgu.q, f.s = wt->wgu.s, f.m = 2 * dm.ffn, f.k = dm.hidden, f.n = 1;
        f.out_f16 = act;
        GemvArgs dn = {};
        dn.x = act, dn.q = wt->wdown.q, dn.s = wt->wdown.s, dn.m = dm.hidden, dn.k = dm.ffn, dn.n = 1, dn.out_f16 = out, dn.resid = x1;
        if (gemv_q3w_eligible(a) && gemv_q3w_eligible(o) && gemv_q3w_eligible(f) && gemv_q3w_eligible(dn) && dm.head_dim % 2 == 0) {
            if (launch_gemv_q3w(a, X_F16_NORM, EPI_ROPE_KV, st_) != hipSuccess) return RELAX_ERR_HIP;
            bool folded = false;
            if (attn_mha_split_supported(dm)) {
                int splits = kAttnMergeSplits, chunk = 0, pos = -1;
                if (st.dev == nullptr) {
                    pos = a.pos0;
                    chunk = attn_fold_chunk(pos + 1, kAttnMergeSplits);
                    splits = (pos + chunk) / chunk;
                }
                o.h = dm.n_heads, o.d = dm.head_dim, o.pos0 = pos, o.seqs = st;
                o.part = partials, o.part_splits = splits, o.part_stride = dm.head_dim / 2 + 4, o.part_chunk = chunk;
                folded = (size_t)dm.n_heads * splits * o.part_stride <= attn_partial_floats(dm, 1, 1) && gemv_merge_eligible(o);
                if (folded && launch_attention_mha_split(qkv, hd, *cache, dm, st, chunk, splits, o.part_stride, partials, st_) != hipSuccess)
                    return RELAX_ERR_HIP;
            }
            if (!folded && launch_attention(qkv, hd, *cache, dm, st, L_max, attn, partials, st_) != hipSuccess) return RELAX_ERR_HIP;
            if (launch_gemv_q3w(o, folded ? X_ATTN_MERGE : X_F16, EPI_RESID_F32, st_) != hipSuccess) return RELAX_ERR_HIP;
            if (launch_gemv_q3w(f, X_F32_NORM, EPI_SWIGLU, st_) != hipSuccess) return RELAX_ERR_HIP;
            if (launch_gemv_q3w(dn, X_F16, EPI_RESID_F16, st_) != hipSuccess) return RELAX_ERR_HIP;
            return RELAX_OK;
        }
    }
    if (launch_rmsnorm(x, wt->norm_attn, xn, n, dm.hidden, dm.rms_eps, st_) != hipSuccess) return RELAX_ERR_HIP;
    if (q3_matmul(xn, wt->wqkv, n, qkv, st_) != hipSuccess) return RELAX_ERR_HIP;
    if (launch_rope_append(qkv, dm, *cache, st, st_) != hipSuccess) return RELAX_ERR_HIP;
    if (launch_attention(qkv, qkvw, *cache, dm, st, L_max, attn, partials, st_) != hipSuccess) return RELAX_ERR_HIP;
    if (q3_matmul(attn, wt->wo, n, tmp, st_) != hipSuccess) return RELAX_ERR_HIP;
    if (launch_add_rows(x, tmp, x1, nh, st_) != hipSuccess) return RELAX_ERR_HIP;
    if (launch_rmsnorm_f32(x1, wt->norm_ffn, xn, n, dm.hidden, dm.rms_eps, st_) != hipSuccess) return RELAX_ERR_HIP;
    if (q3_matmul(xn, wt->wgu, n, gu, st_) != hipSuccess) return RELAX_ERR_HIP;
    if (launch_swiglu_rows(gu, act, n, dm.ffn, st_) != hipSuccess) return RELAX_ERR_HIP;
    if (q3_matmul(act, wt->wdown, n, tmp, st_) != hipSuccess) return RELAX_ERR_HIP;
    if (launch_add_out(x1, tmp, out, nh, st_) != hipSuccess) return RELAX_ERR_HIP;
    return RELAX_OK;
}

// ---- the same sequence on plain fp16 weights (the fp16 models of the paper's LLM evaluation, Sec. 5.1) -----------------
size_t relax_layer_f16_workspace_bytes(const relax_layer_dims *dims, int32_t n_max, int32_t L_max, int32_t B_max)
{
    if (check_dims(dims) != RELAX_OK || n_max < 1 || L_max < 1 || B_max < 1) return 0;
    return plan_q3(*dims, n_max, L_max, B_max).total;
}

relax_status relax_decoder_layer_f16(const relax_layer_dims *dims, const relax_layer_f16_weights *wt, const uint16_t *x,
                                     const relax_kv_cache *cache, const relax_seqs *seqs, uint16_t *out, int32_t n, void *ws,
                                     size_t ws_bytes, relax_stream stream)
{
    hipStream_t st_ = static_cast<hipStream_t>(stream);
    relax_status rc = check_dims(dims);
    if (rc != RELAX_OK) return rc;
    if (!wt || !x || !out || !ws || !cache || !cache->k || !cache->v || !cache->rope) return RELAX_ERR_NULL;
    if (!wt->wqkv || !wt->wo || !wt->wgu || !wt->wdown || !wt->norm_attn || !wt->norm_ffn) return RELAX_ERR_NULL;
    const relax_layer_dims &dm = *dims;
    const int32_t hd = dm.n_heads * dm.head_dim, qkvw = (dm.n_heads + 2 * dm.n_kv_heads) * dm.head_dim;
    if (dm.hidden % 8 != 0 || dm.ffn % 8 != 0) return RELAX_ERR_SHAPE;
    const uintptr_t ptrs = reinterpret_cast<uintptr_t>(wt->wqkv) | reinterpret_cast<uintptr_t>(wt->wo) | reinterpret_cast<uintptr_t>(wt->wgu) |
                           reinterpret_cast<uintptr_t>(wt->wdown) | reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(out);
    if ((ptrs & 15) != 0) return RELAX_ERR_SHAPE;
    if (2 * (size_t)std::max(std::max(dm.hidden, hd), dm.ffn) > 144 * 1024) return RELAX_ERR_UNSUPPORTED;     // one x row has to fit the matvec kernel's LDS
    SeqTable st = {};
    bool need_table = false;
    int32_t L_max = 0;
    rc = build_seqs(seqs, dm, n, st, L_max, need_table);
    if (rc != RELAX_OK) return rc;
    const Q3Plan pl = plan_q3(dm, n, L_max, seqs->B);
    if (ws_bytes < pl.total || (reinterpret_cast<uintptr_t>(ws) & 255) != 0) return RELAX_ERR_WORKSPACE;
    rc = upload_table(st, seqs, need_table, ws, pl.ws, st_);
    if (rc != RELAX_OK) return rc;

    char *base = static_cast<char *>(ws);
    uint16_t *xn = reinterpret_cast<uint16_t *>(base + pl.ws.xn), *qkv = reinterpret_cast<uint16_t *>(base + pl.ws.qkv);
    uint16_t *attn = reinterpret_cast<uint16_t *>(base + pl.ws.attn), *act = reinterpret_cast<uint16_t *>(base + pl.ws.act);
    uint16_t *gu = reinterpret_cast<uint16_t *>(base + pl.gu), *tmp = reinterpret_cast<uint16_t *>(base + pl.tmp);
    float *x1 = reinterpret_cast<float *>(base + pl.ws.x1), *partials = reinterpret_cast<float *>(base + pl.ws.partials);
    const size_t nh = (size_t)n * dm.hidden;

    // One row: the launch sequence of the 4-bit decode layer -- five launches, the light steps folded into the matvecs'
    // prologues and epilogues -- on the fp16 stream of the same kernel.  Needs rows that fit the kernel's x registers.
    if (n == 1) {
        GemvArgs a = {};
        a.x = x, a.norm_w = wt->norm_attn, a.eps = dm.rms_eps, a.wh = wt->wqkv, a.m = qkvw, a.k = dm.hidden, a.n = 1;
        a.out_f16 = qkv, a.kcache = cache->k, a.vcache = cache->v, a.rope = cache->rope;
        a.h = dm.n_heads, a.g = dm.n_kv_heads, a.d = dm.head_dim, a.kv_capacity = dm.kv_capacity, a.seqs = st;
        if (st.dev == nullptr) a.pos0 = st.kv_len[0] - st.q_len[0] - st.q_start[0], a.slot0 = st.slot[0];
        else a.pos0 = -1;
        GemvArgs o = {};
        o.x = attn, o.wh = wt->wo, o.m = dm.hidden, o.k = hd, o.n = 1, o.out_f32 = x1, o.resid = x;
        GemvArgs f = {};
        f.x = x1, f.norm_w = wt->norm_ffn, f.eps = dm.rms_eps, f.wh = wt->wgu, f.m = 2 * dm.ffn, f.k = dm.hidden, f.n = 1, f.out_f16 = act;
        GemvArgs dn = {};
        dn.x = act, dn.wh = wt->wdown, dn.m = dm.hidden, dn.k = dm.ffn, dn.n = 1, dn.out_f16 = out, dn.resid = x1;
        if (gemv_f16w_eligible(a) && gemv_f16w_eligible(o) && gemv_f16w_eligible(f) && gemv_f16w_eligible(dn) && dm.head_dim % 2 == 0) {
            if (launch_gemv_f16w(a, X_F16_NORM, EPI_ROPE_KV, st_) != hipSuccess) return RELAX_ERR_HIP;
            bool folded = false;
            if (attn_mha_split_supported(dm)) {
                int splits = kAttnMergeSplits, chunk = 0, pos = -1;
                if (st.dev == nullptr) {
                    pos = a.pos0;
                    chunk = attn_fold_chunk(pos + 1, kAttnMergeSplits);
                    splits = (pos + chunk) / chunk;
                }
                o.h = dm.n_heads, o.d = dm.head_dim, o.pos0 = pos, o.seqs = st;
                o.part = partials, o.part_splits = splits, o.part_stride = dm.head_dim / 2 + 4, o.part_chunk = chunk;
                folded = (size_t)dm.n_heads * splits * o.part_stride <= attn_partial_floats(dm, 1, 1) && gemv_f16w_merge_eligible(o);
                if (folded && launch_attention_mha_split(qkv, hd, *cache, dm, st, chunk, splits, o.part_stride, partials, st_) != hipSuccess)
                    return RELAX_ERR_HIP;
            }
            if (!folded && launch_attention(qkv, hd, *cache, dm, st, L_max, attn, partials, st_) != hipSuccess) return RELAX_ERR_HIP;
            if (launch_gemv_f16w(o, folded ? X_ATTN_MERGE : X_F16, EPI_RESID_F32, st_) != hipSuccess) return RELAX_ERR_HIP;
            if (launch_gemv_f16w(f, X_F32_NORM, EPI_SWIGLU, st_) != hipSuccess) return RELAX_ERR_HIP;
            if (launch_gemv_f16w(dn, X_F16, EPI_RESID_F16, st_) != hipSuccess) return RELAX_ERR_HIP;
            return RELAX_OK;
        }
    }
    if (launch_rmsnorm(x, wt->norm_attn, xn, n, dm.hidden, dm.rms_eps, st_) != hipSuccess) return RELAX_ERR_HIP;
    if (half_matmul_enqueue(xn, wt->wqkv, qkv, n, qkvw, dm.hidden, st_) != hipSuccess) return RELAX_ERR_HIP;
    if (launch_rope_append(qkv, dm, *cache, st, st_) != hipSuccess) return RELAX_ERR_HIP;
    if (launch_attention(qkv, qkvw, *cache, dm, st, L_max, attn, partials, st_) != hipSuccess) return RELAX_ERR_HIP;
    if (half_matmul_enqueue(attn, wt->wo, tmp, n, dm.hidden, hd, st_) != hipSuccess) return RELAX_ERR_HIP;
    if (launch_add_rows(x, tmp, x1, nh, st_) != hipSuccess) return RELAX_ERR_HIP;
    if (launch_rmsnorm_f32(x1, wt->norm_ffn, xn, n, dm.hidden, dm.rms_eps, st_) != hipSuccess) return RELAX_ERR_HIP;
    if (half_matmul_enqueue(xn, wt->wgu, gu, n, 2 * dm.ffn, dm.hidden, st_) != hipSuccess) return RELAX_ERR_HIP;
    if (launch_swiglu_rows(gu, act, n, dm.ffn, st_) != hipSuccess) return RELAX_ERR_HIP;
    if (half_matmul_enqueue(act, wt->wdown, tmp, n, dm.hidden, dm.ffn, st_) != hipSuccess) return RELAX_ERR_HIP;
    if (launch_add_out(x1, tmp, out, nh, st_) != hipSuccess) return RELAX_ERR_HIP;
    return RELAX_OK;
}

}  // extern "C"

extern "C" {

// Workspace of a model step: [layer workspace][xa][xb][normalised last rows][logits]
struct ModelPlan {
    WsPlan layer;
    size_t xa, xb, xn, logits, total;
};

static ModelPlan plan_model(const relax_model &m, int32_t n, int32_t L, int32_t B)
{
    ModelPlan p;
    p.layer = plan_ws(m.dims, n, L, B);
    size_t off = p.layer.total;
    p.xa = off;     off += align256(2 * (size_t)n * m.dims.hidden);
    p.xb = off;     off += align256(2 * (size_t)n * m.dims.hidden);
    p.xn = off;     off += align256(2 * (size_t)B * m.dims.hidden);
    p.logits = off; off += align256(2 * (size_t)B * m.vocab);
    p.total = off;
    return p;
}

static relax_status check_model(const relax_model *m)
{
    if (!m) return RELAX_ERR_NULL;
    const relax_status rc = check_dims(&m->dims);
    if (rc != RELAX_OK) return rc;
    if (m->n_layers < 0 || m->vocab < 1 || m->dims.hidden % 8 != 0) return RELAX_ERR_SHAPE;
    if (!m->embedding || !m->norm_final || !m->lm_head || (m->n_layers > 0 && !m->layers)) return RELAX_ERR_NULL;
    return RELAX_OK;
}

size_t relax_model_workspace_bytes(const relax_model *model, int32_t n_max, int32_t L_max, int32_t B_max)
{
    if (check_model(model) != RELAX_OK || n_max < 1 || L_max < 1 || B_max < 1) return 0;
    return plan_model(*model, n_max, L_max, B_max).total;
}

relax_status relax_model_step(const relax_model *model, const int32_t *ids, const relax_kv_cache *caches, const relax_seqs *seqs,
                              uint16_t *logits, int32_t *next_ids, int32_t n, void *ws, size_t ws_bytes, relax_stream stream)
{
    hipStream_t st_ = static_cast<hipStream_t>(stream);
    relax_status rc = check_model(model);
    if (rc != RELAX_OK) return rc;
    if (!ids || !ws || (model->n_layers > 0 && !caches)) return RELAX_ERR_NULL;
    const relax_layer_dims &dm = model->dims;
    for (int l = 0; l < model->n_layers; ++l) {
        rc = check_layer(dm, &model->layers[l]);
        if (rc != RELAX_OK) return rc;
        if (!caches[l].k || !caches[l].v || !caches[l].rope) return RELAX_ERR_NULL;
    }
    SeqTable st = {};
    bool need_table = false;
    int32_t L_max = 0;
    rc = build_seqs(seqs, dm, n, st, L_max, need_table);
    if (rc != RELAX_OK) return rc;
    const ModelPlan mp = plan_model(*model, n, L_max, seqs->B);
    if (ws_bytes < mp.total || (reinterpret_cast<uintptr_t>(ws) & 255) != 0) return RELAX_ERR_WORKSPACE;
    rc = upload_table(st, seqs, need_table, ws, mp.layer, st_);
    if (rc != RELAX_OK) return rc;

    char *base = static_cast<char *>(ws);
    uint16_t *cur = reinterpret_cast<uint16_t *>(base + mp.xa), *nxt = reinterpret_cast<uint16_t *>(base + mp.xb);
    uint32_t *err = reinterpret_cast<uint32_t *>(base);        // the flag line at the front of the workspace
    if (launch_embed(ids, model->embedding, cur, n, dm.hidden, model->vocab, err, st_) != hipSuccess) return RELAX_ERR_HIP;
    bool xn_ready = false;
    for (int l = 0; l < model->n_layers; ++l) {
        const uint16_t *next_norm = l + 1 < model->n_layers ? model->layers[l + 1].norm_attn : nullptr;
        bool xn_done = false;
        rc = layer_enqueue(dm, &model->layers[l], cur, &caches[l], st, L_max, nxt, n, base, mp.layer, st_, next_norm, xn_ready, &xn_done);
        if (rc != RELAX_OK) return rc;
        xn_ready = xn_done;
        uint16_t *t = cur;
        cur = nxt, nxt = t;
    }
    uint16_t *xn = reinterpret_cast<uint16_t *>(base + mp.xn);
    uint16_t *lg = logits ? logits : reinterpret_cast<uint16_t *>(base + mp.logits);
    if (launch_final_norm(cur, model->norm_final, xn, st, dm.hidden, dm.rms_eps, st_) != hipSuccess) return RELAX_ERR_HIP;
    if (half_matmul_enqueue(xn, model->lm_head, lg, seqs->B, model->vocab, dm.hidden, st_) != hipSuccess) return RELAX_ERR_HIP;
    if (next_ids && launch_argmax(lg, next_ids, seqs->B, model->vocab, st_) != hipSuccess) return RELAX_ERR_HIP;
    return RELAX_OK;
}

relax_status relax_half_matmul(const uint16_t *x, const uint16_t *w, uint16_t *out, int32_t n, int32_t m, int32_t k, relax_stream stream)
{
    if (!x || !w || !out) return RELAX_ERR_NULL;
    if (n < 1 || m < 1 || k < 8 || k % 8 != 0) return RELAX_ERR_SHAPE;
    if (((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(w)) & 15) != 0) return RELAX_ERR_SHAPE;
    if (2 * (size_t)k > 144 * 1024) return RELAX_ERR_UNSUPPORTED;       // one x row has to fit the matvec kernel's LDS
    return hip_status(half_matmul_enqueue(x, w, out, n, m, k, static_cast<hipStream_t>(stream)));
}

relax_status relax_unpack_int4(const relax_qmat *w, int8_t *out, relax_stream stream)
{
    if (!w || !w->q || !out) return RELAX_ERR_NULL;
    if (w->m < 1 || w->k < 8 || w->k % 8 != 0) return RELAX_ERR_SHAPE;
    return hip_status(launch_unpack(*w, out, static_cast<hipStream_t>(stream)));
}

relax_status relax_dequantize(const relax_qmat *w, float *out, relax_stream stream)
{
    if (!w || !w->q || !w->s || !out) return RELAX_ERR_NULL;
    if (w->m < 1 || w->k < 8 || w->k % 8 != 0) return RELAX_ERR_SHAPE;
    if (gshift_of(w->group) < 0) return RELAX_ERR_UNSUPPORTED;
    return hip_status(launch_dequantize(*w, out, static_cast<hipStream_t>(stream)));
}

relax_status relax_unpack_q3(const relax_qmat *w, int8_t *out, relax_stream stream)
{
    if (!w || !w->q || !out) return RELAX_ERR_NULL;
    if (w->m < 1 || w->k < 32 || w->k % 32 != 0) return RELAX_ERR_SHAPE;
    return hip_status(launch_unpack_q3(*w, out, static_cast<hipStream_t>(stream)));
}

relax_status relax_dequant_matmul_q3(const uint16_t *x, const relax_qmat *w, uint16_t *out, int32_t n, relax_stream stream)
{
    if (!x || !out || !w || !w->q || !w->s) return RELAX_ERR_NULL;
    if (n < 1 || n > 65535 || w->m < 1 || w->k < 32 || w->k % 32 != 0) return RELAX_ERR_SHAPE;
    if (!gemv_q3_supported(w->m, w->k)) return RELAX_ERR_UNSUPPORTED;
    if ((reinterpret_cast<uintptr_t>(x) & 15) != 0 || (reinterpret_cast<uintptr_t>(w->q) & 3) != 0 || (reinterpret_cast<uintptr_t>(w->s) & 1) != 0)
        return RELAX_ERR_SHAPE;
    return hip_status(launch_gemv_q3(x, *w, n, out, static_cast<hipStream_t>(stream)));
}

relax_status relax_repack_q3(const relax_qmat *canonical, uint32_t *native_q, relax_stream stream)
{
    if (!canonical || !canonical->q || !native_q) return RELAX_ERR_NULL;
    if (canonical->m < 1 || canonical->k < 32 || canonical->k % 32 != 0) return RELAX_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(canonical->q) & 3) != 0 || (reinterpret_cast<uintptr_t>(native_q) & 3) != 0) return RELAX_ERR_SHAPE;
    if (static_cast<const void *>(canonical->q) == static_cast<const void *>(native_q)) return RELAX_ERR_SHAPE;   // not in place
    return hip_status(launch_repack_q3(*canonical, native_q, static_cast<hipStream_t>(stream)));
}

relax_status relax_unpack_q3_native(const relax_qmat *w, int8_t *out, relax_stream stream)
{
    if (!w || !w->q || !out) return RELAX_ERR_NULL;
    if (w->m < 1 || w->k < 32 || w->k % 32 != 0) return RELAX_ERR_SHAPE;
    return hip_status(launch_unpack_q3_native(*w, out, static_cast<hipStream_t>(stream)));
}

relax_status relax_dequant_matmul_q3_native(const uint16_t *x, const relax_qmat *w, uint16_t *out, int32_t n, relax_stream stream)
{
    if (!x || !out || !w || !w->q || !w->s) return RELAX_ERR_NULL;
    if (n < 1 || n > 4 * 65535 || w->m < 1 || w->k < 32 || w->k % 32 != 0) return RELAX_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(x) & 15) != 0 || (reinterpret_cast<uintptr_t>(w->q) & 3) != 0 || (reinterpret_cast<uintptr_t>(w->s) & 1) != 0)
        return RELAX_ERR_SHAPE;
    // From kQ3GemmRows rows on the matrix is read once by the tiled MFMA GEMM (decode on the way into LDS); below that, or
    // for a shape the GEMM does not take, it is streamed once per pass of up to four rows of x.
    if (n >= kQ3GemmRows && gemm_q3_eligible(x, *w, out))
        return hip_status(launch_gemm_q3(x, *w, n, out, static_cast<hipStream_t>(stream)));
    if (!gemv_q3_supported(w->m, w->k)) return RELAX_ERR_UNSUPPORTED;
    return hip_status(launch_gemv_q3_native(x, *w, n, out, static_cast<hipStream_t>(stream)));
}

}  // extern "C"
