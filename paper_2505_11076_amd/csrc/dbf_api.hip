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

// Builds the device image of a layer from canonical words and uploads it.
int build_layer(int n_in, int n_out, int k, const uint32_t* A_bits, const uint32_t* B_bits,
                const uint16_t* a, const uint16_t* m, const uint16_t* b, dbf_layer** out) {
    const size_t bytesA = dbf_tiled_bytes(n_out, k), bytesB = dbf_tiled_bytes(k, n_in);
    const int a_len = dbf_row_tiles(n_out) * DBF_TILE_ROWS;
    const int m_len = dbf_row_tiles(k) * DBF_TILE_ROWS;
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

    DbfStage& sb = L->h_stages[0];
    sb.bits = L->dB;  sb.in_scale = L->db;  sb.row_scale = L->dm;  sb.t = L->dt;
    sb.x_off = 0;  sb.y_off = 0;
    sb.n_rt = dbf_row_tiles(k);  sb.n_ct = dbf_col_tiles(n_in);
    sb.rows = k;  sb.cols = n_in;  sb.t_stride = t_stride;  sb.pad_ = 0;
    DbfStage& sa = L->h_stages[1];
    sa.bits = L->dA;  sa.in_scale = nullptr;  sa.row_scale = L->da;  sa.t = L->dt;
    sa.x_off = 0;  sa.y_off = 0;
    sa.n_rt = dbf_row_tiles(n_out);  sa.n_ct = dbf_col_tiles(k);
    sa.rows = n_out;  sa.cols = k;  sa.t_stride = t_stride;  sa.pad_ = 0;
    std::memcpy(image + offs, L->h_stages, 2 * sizeof(DbfStage));

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

int launch_pair(int kind, const DbfStage* dB, const DbfStage* dA, const DbfBlockRef* mapB,
                const DbfBlockRef* mapA, int blocksB, int blocksA, int max_cols_B, int max_cols_A,
                const void* x, void* y, int batch, hipStream_t stream) {
    if (kind == DBF_GEMV_AUTO) kind = DBF_GEMV_MFMA;
    if (kind == DBF_GEMV_VALU) {
        DBF_HIP_TRY(dbf_launch_stage_valu(false, dB, mapB, blocksB, x, y, batch, max_cols_B, stream));
        DBF_HIP_TRY(dbf_launch_stage_valu(true, dA, mapA, blocksA, x, y, batch, max_cols_A, stream));
    } else {
        DBF_HIP_TRY(dbf_launch_stage_mfma(false, dB, mapB, blocksB, x, y, batch, max_cols_B, stream));
        DBF_HIP_TRY(dbf_launch_stage_mfma(true, dA, mapA, blocksA, x, y, batch, max_cols_A, stream));
    }
    return DBF_OK;
}

inline bool kind_ok(int kind) {
    return kind == DBF_GEMV_AUTO || kind == DBF_GEMV_VALU || kind == DBF_GEMV_MFMA;
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
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    return launch_pair(kind, L->d_stages, L->d_stages + 1, nullptr, nullptr, L->h_stages[0].n_rt,
                       L->h_stages[1].n_rt, L->n_in, L->k, x_dev, y_dev, batch, stream);
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
    std::vector<DbfBlockRef> mB, mA;
    S->h_x_prefix = static_cast<long long*>(std::malloc(sizeof(long long) * (n_layers + 1)));
    S->h_y_prefix = static_cast<long long*>(std::malloc(sizeof(long long) * (n_layers + 1)));
    if (!S->h_x_prefix || !S->h_y_prefix) {
        dbf_stack_free(S);
        return DBF_ENOMEM;
    }
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
        for (int rt = 0; rt < sB[i].n_rt; ++rt) mB.push_back(DbfBlockRef{i, rt});
        for (int rt = 0; rt < sA[i].n_rt; ++rt) mA.push_back(DbfBlockRef{i, rt});
        if (L->n_in > S->max_cols_B) S->max_cols_B = L->n_in;
        if (L->k > S->max_cols_A) S->max_cols_A = L->k;
    }
    S->blocksB = (int)mB.size();
    S->blocksA = (int)mA.size();

    size_t off = 0;
    const size_t o_sB = off;  off = align_up(off + sizeof(DbfStage) * n_layers, 256);
    const size_t o_sA = off;  off = align_up(off + sizeof(DbfStage) * n_layers, 256);
    const size_t o_mB = off;  off = align_up(off + sizeof(DbfBlockRef) * mB.size(), 256);
    const size_t o_mA = off;  off = align_up(off + sizeof(DbfBlockRef) * mA.size(), 256);
    std::vector<uint8_t> image(off, 0);
    std::memcpy(image.data() + o_sB, sB.data(), sizeof(DbfStage) * n_layers);
    std::memcpy(image.data() + o_sA, sA.data(), sizeof(DbfStage) * n_layers);
    std::memcpy(image.data() + o_mB, mB.data(), sizeof(DbfBlockRef) * mB.size());
    std::memcpy(image.data() + o_mA, mA.data(), sizeof(DbfBlockRef) * mA.size());
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
    S->d_mapB = reinterpret_cast<DbfBlockRef*>(d + o_mB);
    S->d_mapA = reinterpret_cast<DbfBlockRef*>(d + o_mA);
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
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    return launch_pair(kind, S->d_stagesB, S->d_stagesA, S->d_mapB, S->d_mapA, S->blocksB,
                       S->blocksA, S->max_cols_B, S->max_cols_A, x_dev, y_dev, batch, stream);
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
