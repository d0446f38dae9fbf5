// C ABI of libdbf: argument checks, the layer / stack objects and kernel dispatch.
// Every operation of the layer product itself runs in the HIP kernels; this file only
// validates, allocates at pack time, and launches.
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "dbf_kernels.h"

namespace {

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

inline bool shape_ok(int n_in, int n_out, int k) {
    return n_in >= 1 && n_out >= 1 && k >= 1 && n_in <= DBF_MAX_DIM && n_out <= DBF_MAX_DIM &&
           k <= DBF_MAX_DIM;
}

#define DBF_HIP_TRY(expr)                  \
    do {                                   \
        if ((expr) != hipSuccess) {        \
            (void)hipGetLastError();       \
            return DBF_EHIP;               \
        }                                  \
    } while (0)

// Row tiles of one stage cut into work items of at most `span` tiles.
void append_items(std::vector<DbfWorkItem>& out, int layer, int n_rt, int span) {
    for (int rt = 0; rt < n_rt; rt += span) {
        const int n = (n_rt - rt < span) ? (n_rt - rt) : span;
        out.push_back(DbfWorkItem{layer, rt, n, 0});
    }
}

// Builds the device image of a layer from canonical words and uploads it.
int build_layer(int n_in, int n_out, int k, const uint32_t* A_bits, const uint32_t* B_bits,
                const uint16_t* a, const uint16_t* m, const uint16_t* b, dbf_layer** out) {
    const size_t bytesA = dbf_tiled_bytes(n_out, k), bytesB = dbf_tiled_bytes(k, n_in);
    const int rtA = dbf_row_tiles(n_out), rtB = dbf_row_tiles(k);
    const int a_len = rtA * DBF_TILE_ROWS;
    const int m_len = rtB * DBF_TILE_ROWS;
    const int b_len = dbf_col_tiles(n_in) * DBF_TILE_COLS;
    const int t_stride = m_len;  // >= col_tiles(k)*64, so the A stage may read its padded columns

    // offsets inside the single device block (256-byte aligned sections)
    size_t off = 0;
    const size_t offA = off;  off = align_up(off + bytesA, 256);
    const size_t offB = off;  off = align_up(off + bytesB, 256);
    const size_t offa = off;  off = align_up(off + 2 * (size_t)a_len, 256);
    const size_t offm = off;  off = align_up(off + 2 * (size_t)m_len, 256);
    const size_t offb = off;  off = align_up(off + 2 * (size_t)b_len, 256);
    const size_t offs = off;  off = align_up(off + 2 * sizeof(DbfStage), 256);
    const size_t offwB = off; off = align_up(off + sizeof(DbfWorkItem) * rtB, 256);
    const size_t offwA = off; off = align_up(off + sizeof(DbfWorkItem) * rtA, 256);
    const size_t image_bytes = off;  // everything up to here is uploaded
    const size_t offt = off;  off = align_up(off + 4 * (size_t)DBF_MAX_BATCH * t_stride, 256);
    const size_t total = off;

    uint8_t* image = static_cast<uint8_t*>(std::calloc(image_bytes, 1));
    dbf_layer* L = new (std::nothrow) dbf_layer();
    if (!image || !L) {
        std::free(image);
        delete L;
        return DBF_ENOMEM;
    }
    int rc = dbf_tile_host(n_out, k, A_bits, image + offA);
    if (rc == DBF_OK) rc = dbf_tile_host(k, n_in, B_bits, image + offB);
    if (rc != DBF_OK) {
        std::free(image);
        delete L;
        return rc;
    }
    std::memcpy(image + offa, a, 2 * (size_t)n_out);
    std::memcpy(image + offm, m, 2 * (size_t)k);
    std::memcpy(image + offb, b, 2 * (size_t)n_in);

    void* dev = nullptr;
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess || hipMalloc(&dev, total) != hipSuccess) {
        (void)hipGetLastError();
        std::free(image);
        delete L;
        return DBF_EHIP;
    }
    uint8_t* d = static_cast<uint8_t*>(dev);
    L->n_in = n_in;  L->n_out = n_out;  L->k = k;  L->device = device;
    L->dev_block = dev;  L->device_bytes = total;
    L->dA = d + offA;  L->dB = d + offB;
    L->da = reinterpret_cast<uint16_t*>(d + offa);
    L->dm = reinterpret_cast<uint16_t*>(d + offm);
    L->db = reinterpret_cast<uint16_t*>(d + offb);
    L->dt = reinterpret_cast<float*>(d + offt);
    L->t_stride = t_stride;
    L->d_stages = reinterpret_cast<DbfStage*>(d + offs);
    L->d_workB = reinterpret_cast<DbfWorkItem*>(d + offwB);
    L->d_workA = reinterpret_cast<DbfWorkItem*>(d + offwA);

    DbfStage& sb = L->h_stages[0];
    sb.bits = L->dB;  sb.in_scale = L->db;  sb.row_scale = L->dm;  sb.t = L->dt;
    sb.x_off = 0;  sb.y_off = 0;
    sb.n_rt = rtB;  sb.n_ct = dbf_col_tiles(n_in);
    sb.rows = k;  sb.cols = n_in;  sb.t_stride = t_stride;  sb.pad_ = 0;
    DbfStage& sa = L->h_stages[1];
    sa.bits = L->dA;  sa.in_scale = nullptr;  sa.row_scale = L->da;  sa.t = L->dt;
    sa.x_off = 0;  sa.y_off = 0;
    sa.n_rt = rtA;  sa.n_ct = dbf_col_tiles(k);
    sa.rows = n_out;  sa.cols = k;  sa.t_stride = t_stride;  sa.pad_ = 0;
    std::memcpy(image + offs, L->h_stages, 2 * sizeof(DbfStage));
    std::vector<DbfWorkItem> wB, wA;
    append_items(wB, 0, rtB, 1);
    append_items(wA, 0, rtA, 1);
    std::memcpy(image + offwB, wB.data(), sizeof(DbfWorkItem) * wB.size());
    std::memcpy(image + offwA, wA.data(), sizeof(DbfWorkItem) * wA.size());

    hipError_t e = hipMemcpy(dev, image, image_bytes, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemset(d + offt, 0, total - offt);
    if (e == hipSuccess) e = hipDeviceSynchronize();
    std::free(image);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        (void)hipFree(dev);
        delete L;
        return DBF_EHIP;
    }
    *out = L;
    return DBF_OK;
}

// Everything a launch of the two stages needs.
struct LaunchPlan {
    const DbfStage* stagesB;
    const DbfStage* stagesA;
    const DbfWorkItem* workB1;  // one row tile per workgroup
    const DbfWorkItem* workA1;
    const DbfWorkItem* workBn;  // several row tiles per workgroup (may equal work*1)
    const DbfWorkItem* workAn;
    int blocksB1, blocksA1, blocksBn, blocksAn;
    int max_cols_B, max_cols_A;
};

// Launches the B stage and then the A stage on `stream`.  If `mid` is not NULL it is
// recorded between the two launches (used only by the timed entry point).
int launch_pair(int kind, const LaunchPlan& p, const void* x, void* y, int batch,
                hipStream_t stream, hipEvent_t mid = nullptr) {
    if (kind == DBF_GEMV_AUTO) kind = DBF_GEMV_MFMA;
#ifdef DBF_DEBUG_KINDS
    if (kind == 3 || kind == 4) {  // 3: MFMA B stage + VALU A stage, 4: VALU B + MFMA A
        if (kind == 3) DBF_HIP_TRY(dbf_launch_stage_mfma(false, p.stagesB, p.workB1, p.blocksB1, x, y, batch, p.max_cols_B, stream));
        else DBF_HIP_TRY(dbf_launch_stage_valu(false, p.stagesB, p.workB1, p.blocksB1, x, y, batch, p.max_cols_B, stream));
        if (kind == 3) DBF_HIP_TRY(dbf_launch_stage_valu(true, p.stagesA, p.workA1, p.blocksA1, x, y, batch, p.max_cols_A, stream));
        else DBF_HIP_TRY(dbf_launch_stage_mfma(true, p.stagesA, p.workA1, p.blocksA1, x, y, batch, p.max_cols_A, stream));
        return DBF_OK;
    }
#endif
    if (kind == DBF_GEMV_VALU) {
        DBF_HIP_TRY(dbf_launch_stage_valu(false, p.stagesB, p.workB1, p.blocksB1, x, y, batch,
                                          p.max_cols_B, stream));
        if (mid) DBF_HIP_TRY(hipEventRecord(mid, stream));
        DBF_HIP_TRY(dbf_launch_stage_valu(true, p.stagesA, p.workA1, p.blocksA1, x, y, batch,
                                          p.max_cols_A, stream));
        return DBF_OK;
    }
    // several row tiles per workgroup only if all columns of the stage fit one LDS chunk
    const bool spanB = dbf_mfma_chunk_tiles(batch, p.max_cols_B) >= dbf_col_tiles(p.max_cols_B);
    const bool spanA = dbf_mfma_chunk_tiles(batch, p.max_cols_A) >= dbf_col_tiles(p.max_cols_A);
    DBF_HIP_TRY(dbf_launch_stage_mfma(false, p.stagesB, spanB ? p.workBn : p.workB1,
                                      spanB ? p.blocksBn : p.blocksB1, x, y, batch, p.max_cols_B, stream));
    if (mid) DBF_HIP_TRY(hipEventRecord(mid, stream));
    DBF_HIP_TRY(dbf_launch_stage_mfma(true, p.stagesA, spanA ? p.workAn : p.workA1,
                                      spanA ? p.blocksAn : p.blocksA1, x, y, batch, p.max_cols_A, stream));
    return DBF_OK;
}

inline bool kind_ok(int kind) {
#ifdef DBF_DEBUG_KINDS
    if (kind == 3 || kind == 4) return true;
#endif
    return kind == DBF_GEMV_AUTO || kind == DBF_GEMV_VALU || kind == DBF_GEMV_MFMA;
}

LaunchPlan plan_of(const dbf_layer* L) {
    LaunchPlan p;
    p.stagesB = L->d_stages;
    p.stagesA = L->d_stages + 1;
    p.workB1 = p.workBn = L->d_workB;
    p.workA1 = p.workAn = L->d_workA;
    p.blocksB1 = p.blocksBn = L->h_stages[0].n_rt;
    p.blocksA1 = p.blocksAn = L->h_stages[1].n_rt;
    p.max_cols_B = L->n_in;
    p.max_cols_A = L->k;
    return p;
}

LaunchPlan plan_of(const dbf_stack* S) {
    LaunchPlan p;
    p.stagesB = S->d_stagesB;
    p.stagesA = S->d_stagesA;
    p.workB1 = S->d_workB1;  p.workA1 = S->d_workA1;
    p.workBn = S->d_workBn;  p.workAn = S->d_workAn;
    p.blocksB1 = S->blocksB1;  p.blocksA1 = S->blocksA1;
    p.blocksBn = S->blocksBn;  p.blocksAn = S->blocksAn;
    p.max_cols_B = S->max_cols_B;
    p.max_cols_A = S->max_cols_A;
    return p;
}

int stack_span() {
    // Row tiles per workgroup in stack launches: the input vector is quantised once per
    // workgroup, so a larger span amortises that prologue; DBF_STACK_SPAN overrides (1..16).
    const char* e = std::getenv("DBF_STACK_SPAN");
    int v = e ? std::atoi(e) : 4;
    if (v < 1) v = 1;
    if (v > 16) v = 16;
    return v;
}

}  // namespace

extern "C" {

int dbf_pack_bits(int n_in, int n_out, int k, const uint32_t* A_bits, const uint32_t* B_bits,
                  const uint16_t* a, const uint16_t* m, const uint16_t* b, dbf_layer** out) {
    if (out) *out = nullptr;
    if (!A_bits || !B_bits || !a || !m || !b || !out) return DBF_EINVAL;
    if (!shape_ok(n_in, n_out, k)) return DBF_ESHAPE;
    return build_layer(n_in, n_out, k, A_bits, B_bits, a, m, b, out);
}

int dbf_pack(int n_in, int n_out, int k, const int8_t* A_pm1, const int8_t* B_pm1,
             const uint16_t* a, const uint16_t* m, const uint16_t* b, dbf_layer** out) {
    if (out) *out = nullptr;
    if (!A_pm1 || !B_pm1 || !a || !m || !b || !out) return DBF_EINVAL;
    if (!shape_ok(n_in, n_out, k)) return DBF_ESHAPE;
    const size_t wa = (size_t)n_out * ((k + 31) / 32), wb = (size_t)k * ((n_in + 31) / 32);
    uint32_t* Ab = static_cast<uint32_t*>(std::malloc(wa * 4));
    uint32_t* Bb = static_cast<uint32_t*>(std::malloc(wb * 4));
    int rc = (Ab && Bb) ? DBF_OK : DBF_ENOMEM;
    if (rc == DBF_OK) rc = dbf_signs_to_bits_host(n_out, k, A_pm1, Ab);
    if (rc == DBF_OK) rc = dbf_signs_to_bits_host(k, n_in, B_pm1, Bb);
    if (rc == DBF_OK) rc = build_layer(n_in, n_out, k, Ab, Bb, a, m, b, out);
    std::free(Ab);
    std::free(Bb);
    return rc;
}

int dbf_unpack_bits(const dbf_layer* L, uint32_t* A_bits, uint32_t* B_bits, uint16_t* a,
                    uint16_t* m, uint16_t* b) {
    if (!L) return DBF_EINVAL;
    DBF_HIP_TRY(hipDeviceSynchronize());
    if (A_bits) {
        std::vector<uint8_t> img(dbf_tiled_bytes(L->n_out, L->k));
        DBF_HIP_TRY(hipMemcpy(img.data(), L->dA, img.size(), hipMemcpyDeviceToHost));
        const int rc = dbf_untile_host(L->n_out, L->k, img.data(), A_bits);
        if (rc != DBF_OK) return rc;
    }
    if (B_bits) {
        std::vector<uint8_t> img(dbf_tiled_bytes(L->k, L->n_in));
        DBF_HIP_TRY(hipMemcpy(img.data(), L->dB, img.size(), hipMemcpyDeviceToHost));
        const int rc = dbf_untile_host(L->k, L->n_in, img.data(), B_bits);
        if (rc != DBF_OK) return rc;
    }
    if (a) DBF_HIP_TRY(hipMemcpy(a, L->da, 2 * (size_t)L->n_out, hipMemcpyDeviceToHost));
    if (m) DBF_HIP_TRY(hipMemcpy(m, L->dm, 2 * (size_t)L->k, hipMemcpyDeviceToHost));
    if (b) DBF_HIP_TRY(hipMemcpy(b, L->db, 2 * (size_t)L->n_in, hipMemcpyDeviceToHost));
    return DBF_OK;
}

int dbf_dims(const dbf_layer* L, int* n_in, int* n_out, int* k, size_t* device_bytes) {
    if (!L) return DBF_EINVAL;
    if (n_in) *n_in = L->n_in;
    if (n_out) *n_out = L->n_out;
    if (k) *k = L->k;
    if (device_bytes) *device_bytes = L->device_bytes;
    return DBF_OK;
}

void dbf_free(dbf_layer* L) {
    if (!L) return;
    if (L->dev_block) (void)hipFree(L->dev_block);
    delete L;
}

int dbf_gemv_kind(const dbf_layer* L, const void* x_dev, void* y_dev, int batch, int kind,
                  void* hip_stream) {
    if (!L || !x_dev || !y_dev) return DBF_EINVAL;
    if (batch < 1 || batch > DBF_MAX_BATCH || !kind_ok(kind)) return DBF_EINVAL;
    return launch_pair(kind, plan_of(L), x_dev, y_dev, batch, static_cast<hipStream_t>(hip_stream));
}

int dbf_gemv(const dbf_layer* L, const void* x_dev, void* y_dev, int batch, void* hip_stream) {
    return dbf_gemv_kind(L, x_dev, y_dev, batch, DBF_GEMV_AUTO, hip_stream);
}

// ---- stacks ---------------------------------------------------------------------------------

int dbf_stack_create(const dbf_layer* const* layers, int n_layers, dbf_stack** out) {
    if (out) *out = nullptr;
    if (!layers || !out || n_layers < 1) return DBF_EINVAL;
    for (int i = 0; i < n_layers; ++i)
        if (!layers[i]) return DBF_EINVAL;
    for (int i = 1; i < n_layers; ++i)
        if (layers[i]->device != layers[0]->device) return DBF_EINVAL;

    dbf_stack* S = new (std::nothrow) dbf_stack();
    if (!S) return DBF_ENOMEM;
    std::vector<DbfStage> sB(n_layers), sA(n_layers);
    std::vector<DbfWorkItem> wB1, wA1, wBn, wAn;
    S->h_x_prefix = static_cast<long long*>(std::malloc(sizeof(long long) * (n_layers + 1)));
    S->h_y_prefix = static_cast<long long*>(std::malloc(sizeof(long long) * (n_layers + 1)));
    if (!S->h_x_prefix || !S->h_y_prefix) {
        dbf_stack_free(S);
        return DBF_ENOMEM;
    }
    const int span = stack_span();
    S->n_layers = n_layers;
    S->device = layers[0]->device;
    S->h_x_prefix[0] = S->h_y_prefix[0] = 0;
    for (int i = 0; i < n_layers; ++i) {
        const dbf_layer* L = layers[i];
        sB[i] = L->h_stages[0];
        sA[i] = L->h_stages[1];
        sB[i].x_off = sA[i].x_off = S->h_x_prefix[i];
        sB[i].y_off = sA[i].y_off = S->h_y_prefix[i];
        S->h_x_prefix[i + 1] = S->h_x_prefix[i] + L->n_in;
        S->h_y_prefix[i + 1] = S->h_y_prefix[i] + L->n_out;
        append_items(wB1, i, sB[i].n_rt, 1);
        append_items(wA1, i, sA[i].n_rt, 1);
        append_items(wBn, i, sB[i].n_rt, span);
        append_items(wAn, i, sA[i].n_rt, span);
        if (L->n_in > S->max_cols_B) S->max_cols_B = L->n_in;
        if (L->k > S->max_cols_A) S->max_cols_A = L->k;
    }
    S->blocksB1 = (int)wB1.size();  S->blocksA1 = (int)wA1.size();
    S->blocksBn = (int)wBn.size();  S->blocksAn = (int)wAn.size();

    size_t off = 0;
    const size_t o_sB = off;  off = align_up(off + sizeof(DbfStage) * n_layers, 256);
    const size_t o_sA = off;  off = align_up(off + sizeof(DbfStage) * n_layers, 256);
    const size_t o_B1 = off;  off = align_up(off + sizeof(DbfWorkItem) * wB1.size(), 256);
    const size_t o_A1 = off;  off = align_up(off + sizeof(DbfWorkItem) * wA1.size(), 256);
    const size_t o_Bn = off;  off = align_up(off + sizeof(DbfWorkItem) * wBn.size(), 256);
    const size_t o_An = off;  off = align_up(off + sizeof(DbfWorkItem) * wAn.size(), 256);
    std::vector<uint8_t> image(off, 0);
    std::memcpy(image.data() + o_sB, sB.data(), sizeof(DbfStage) * n_layers);
    std::memcpy(image.data() + o_sA, sA.data(), sizeof(DbfStage) * n_layers);
    std::memcpy(image.data() + o_B1, wB1.data(), sizeof(DbfWorkItem) * wB1.size());
    std::memcpy(image.data() + o_A1, wA1.data(), sizeof(DbfWorkItem) * wA1.size());
    std::memcpy(image.data() + o_Bn, wBn.data(), sizeof(DbfWorkItem) * wBn.size());
    std::memcpy(image.data() + o_An, wAn.data(), sizeof(DbfWorkItem) * wAn.size());
    void* dev = nullptr;
    hipError_t e = hipMalloc(&dev, off);
    if (e == hipSuccess) e = hipMemcpy(dev, image.data(), off, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
        (void)hipGetLastError();
        if (dev) (void)hipFree(dev);
        dbf_stack_free(S);
        return DBF_EHIP;
    }
    uint8_t* d = static_cast<uint8_t*>(dev);
    S->dev_block = dev;
    S->d_stagesB = reinterpret_cast<DbfStage*>(d + o_sB);
    S->d_stagesA = reinterpret_cast<DbfStage*>(d + o_sA);
    S->d_workB1 = reinterpret_cast<DbfWorkItem*>(d + o_B1);
    S->d_workA1 = reinterpret_cast<DbfWorkItem*>(d + o_A1);
    S->d_workBn = reinterpret_cast<DbfWorkItem*>(d + o_Bn);
    S->d_workAn = reinterpret_cast<DbfWorkItem*>(d + o_An);
    *out = S;
    return DBF_OK;
}

int dbf_stack_offsets(const dbf_stack* S, int layer_index, int batch, size_t* x_off, size_t* y_off) {
    if (!S || layer_index < 0 || layer_index > S->n_layers) return DBF_EINVAL;
    if (batch < 1 || batch > DBF_MAX_BATCH) return DBF_EINVAL;
    if (x_off) *x_off = (size_t)S->h_x_prefix[layer_index] * batch;
    if (y_off) *y_off = (size_t)S->h_y_prefix[layer_index] * batch;
    return DBF_OK;
}

int dbf_stack_gemv(const dbf_stack* S, const void* x_dev, void* y_dev, int batch, int kind,
                   void* hip_stream) {
    if (!S || !x_dev || !y_dev) return DBF_EINVAL;
    if (batch < 1 || batch > DBF_MAX_BATCH || !kind_ok(kind)) return DBF_EINVAL;
    return launch_pair(kind, plan_of(S), x_dev, y_dev, batch, static_cast<hipStream_t>(hip_stream));
}

int dbf_stack_gemv_timed(const dbf_stack* S, const void* x_dev, void* y_dev, int batch, int kind,
                         void* hip_stream, float* ms_stage_b, float* ms_stage_a) {
    if (!S || !x_dev || !y_dev) return DBF_EINVAL;
    if (batch < 1 || batch > DBF_MAX_BATCH || !kind_ok(kind)) return DBF_EINVAL;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    hipEvent_t ev[3] = {nullptr, nullptr, nullptr};
    int rc = DBF_OK;
    for (int i = 0; i < 3 && rc == DBF_OK; ++i)
        if (hipEventCreate(&ev[i]) != hipSuccess) rc = DBF_EHIP;
    if (rc == DBF_OK && hipEventRecord(ev[0], stream) != hipSuccess) rc = DBF_EHIP;
    if (rc == DBF_OK) rc = launch_pair(kind, plan_of(S), x_dev, y_dev, batch, stream, ev[1]);
    if (rc == DBF_OK && hipEventRecord(ev[2], stream) != hipSuccess) rc = DBF_EHIP;
    if (rc == DBF_OK && hipEventSynchronize(ev[2]) != hipSuccess) rc = DBF_EHIP;
    float mb = 0.f, ma = 0.f;
    if (rc == DBF_OK && hipEventElapsedTime(&mb, ev[0], ev[1]) != hipSuccess) rc = DBF_EHIP;
    if (rc == DBF_OK && hipEventElapsedTime(&ma, ev[1], ev[2]) != hipSuccess) rc = DBF_EHIP;
    for (int i = 0; i < 3; ++i)
        if (ev[i]) (void)hipEventDestroy(ev[i]);
    if (rc != DBF_OK) (void)hipGetLastError();
    if (ms_stage_b) *ms_stage_b = mb;
    if (ms_stage_a) *ms_stage_a = ma;
    return rc;
}

void dbf_stack_free(dbf_stack* S) {
    if (!S) return;
    if (S->dev_block) (void)hipFree(S->dev_block);
    std::free(S->h_x_prefix);
    std::free(S->h_y_prefix);
    delete S;
}

const char* dbf_strerror(int code) {
    switch (code) {
        case DBF_OK: return "ok";
        case DBF_EINVAL: return "invalid argument (null pointer, bad enum, batch or T out of range)";
        case DBF_ESHAPE: return "bad shape (n_in, n_out, k must be in [1, 2^20])";
        case DBF_ENOTSIGN: return "sign entry other than -1/+1, or non-zero tail bits";
        case DBF_ENOMEM: return "out of memory";
        case DBF_EHIP: return "HIP runtime error (no usable GPU, failed copy or launch)";
        case DBF_EWORKSPACE: return "workspace missing, misaligned or too small";
        default: return "unknown error code";
    }
}

}  // extern "C"
